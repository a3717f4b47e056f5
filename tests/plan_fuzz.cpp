// Host-only replay of tests/golden/plan_fuzz_cases.txt against the library's plan and replica-array arithmetic,
// meant to be built with -fsanitize=address,undefined (no GPU, no HIP calls): plan.cpp and topology.cpp are
// compiled in directly.  The expected values in the file come from the CPU oracle.  Besides those, every accepted
// plan is checked for the invariants no oracle is needed for: chunk table covers every piece exactly once, the
// workspace layout is ordered, aligned and within the size the plan reports.
// Exit status 0 = every line agreed; otherwise the first disagreement is printed.
#include <cinttypes>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <sstream>
#include <string>
#include <vector>

#include "internal.hpp"

namespace {

const uint64_t kMod = (1ull << 61) - 1;

uint64_t mulmod(uint64_t a, uint64_t b) { return (uint64_t)((unsigned __int128)a * b % kMod); }

std::vector<std::string> split(const std::string& s, char sep) {
  std::vector<std::string> out;
  std::stringstream ss(s);
  std::string item;
  while (std::getline(ss, item, sep)) out.push_back(item);
  return out;
}

int fail(int line, const char* what, long long got, long long want) {
  std::printf("line %d: %s: library %lld, oracle %lld\n", line, what, got, want);
  return 1;
}

int check_plan(int line, const std::vector<std::string>& f, bool rows) {
  const bool must = f[1] == "must";
  const int N = std::atoi(f[2].c_str()), align = std::atoi(f[3].c_str()), chunk = std::atoi(f[4].c_str());
  const int V = std::atoi(f[5].c_str());
  std::vector<int64_t> a, c;
  if (f[6] != "-")
    for (const std::string& item : split(f[6], ',')) {
      if (rows) {
        const size_t x = item.find('x');
        a.push_back((int64_t)std::strtoull(item.substr(0, x).c_str(), nullptr, 10));
        c.push_back((int64_t)std::strtoull(item.substr(x + 1).c_str(), nullptr, 10));
      } else {
        a.push_back((int64_t)std::strtoull(item.c_str(), nullptr, 10));
      }
    }
  if ((int)a.size() != V) return fail(line, "variable count of the case itself", (long long)a.size(), V);
  static const int64_t none = 0;
  shard_plan_s p;
  const int rc = su::plan_build(&p, V, V > 0 ? a.data() : &none, rows ? (V > 0 ? c.data() : &none) : nullptr, N, align,
                                nullptr, chunk);
  if (rc != SHARD_OK) {
    if (must) return fail(line, "plan refused, status", rc, 0);
    if (rc != SHARD_EINVAL && rc != SHARD_ENOMEM) return fail(line, "unexpected status", rc, SHARD_EINVAL);
    return 0;
  }
  const uint64_t S = std::strtoull(f[7].c_str(), nullptr, 10), total = std::strtoull(f[8].c_str(), nullptr, 10);
  if ((uint64_t)p.S != S) return fail(line, "S", p.S, (long long)S);
  if ((uint64_t)p.total != total) return fail(line, "total", p.total, (long long)total);
  uint64_t fold = 0, real0 = 0, real1 = 0;
  for (int i = 0; i < V; ++i) {
    fold = (fold + mulmod((uint64_t)(i + 1), (mulmod(31, (uint64_t)p.L[i] % kMod) + (uint64_t)p.off[i]) % kMod)) % kMod;
    for (int which = 0; which < 2; ++which) {
      const int64_t r = which ? N - 1 : 0;
      const int64_t rem = p.n[i] - r * p.stride[i];
      const int64_t real = rem <= 0 ? 0 : (rem < p.stride[i] ? rem : p.stride[i]);
      uint64_t& acc = which ? real1 : real0;
      acc = (acc + mulmod((uint64_t)(i + 1), (uint64_t)real % kMod)) % kMod;
    }
  }
  if (fold != std::strtoull(f[9].c_str(), nullptr, 10)) return fail(line, "fold of L and off", (long long)fold, std::atoll(f[9].c_str()));
  if (real0 != std::strtoull(f[10].c_str(), nullptr, 10)) return fail(line, "real counts of replica 0", (long long)real0, std::atoll(f[10].c_str()));
  if (real1 != std::strtoull(f[11].c_str(), nullptr, 10)) return fail(line, "real counts of the last replica", (long long)real1, std::atoll(f[11].c_str()));
  // invariants of the tables
  int64_t covered = 0;
  size_t next = 0;
  for (int i = 0; i < V; ++i) {
    const su::VarDesc& vd = p.vars[i];
    if (vd.first_chunk != (int32_t)next) return fail(line, "first_chunk", vd.first_chunk, (long long)next);
    int64_t k = 0;
    for (int32_t j = 0; j < vd.n_chunks; ++j, ++next) {
      const su::ChunkDesc& cd = p.chunks[next];
      if (cd.var != i || cd.k0 != k || cd.len <= 0 || cd.len > p.chunk) return fail(line, "chunk entry", cd.k0, k);
      k += cd.len;
    }
    if (k != p.L[i]) return fail(line, "chunks do not cover the piece", k, p.L[i]);
    covered += k;
  }
  if (covered != p.S || next != p.chunks.size()) return fail(line, "chunk table size", covered, p.S);
  if (!rows) {
    int64_t padded = 0;
    for (const su::FullChunk& fc : p.full_chunks) padded += fc.len;
    if (padded != (int64_t)N * p.S) return fail(line, "variable-by-variable items", padded, (int64_t)N * p.S);
  }
  su::Workspace ws;
  const size_t need = su::workspace_layout(&p, &ws);
  if (need != p.ws_need) return fail(line, "workspace size", (long long)need, (long long)p.ws_need);
  const size_t offs[] = {ws.vars, ws.chunks, ws.ptrs, ws.chunk_sums, ws.var_sums};
  for (size_t o : offs)
    if (o % 16 != 0 || o > need) return fail(line, "workspace offset", (long long)o, (long long)need);
  // the memory model on this plan (Section 4.2) against the formula, in exact integers
  int64_t rep = 0, sh = 0;
  if (shard_plan_peak_bytes(&p, 4, 8, 1000, &rep, &sh) == SHARD_OK) {
    const __int128 W = (__int128)p.total * 4, Vb = (__int128)p.total * 8, Ssh = (__int128)p.S * 8;
    const __int128 a1 = W + Ssh + 1000, a2 = W + Vb;
    if ((__int128)rep != W + Vb + 1000 || (__int128)sh != (a1 > a2 ? a1 : a2)) return fail(line, "peak bytes", sh, (long long)(a1 > a2 ? a1 : a2));
  }
  return 0;
}

int check_part(int line, const std::vector<std::string>& f) {
  const int rows = std::atoi(f[1].c_str()), cols = std::atoi(f[2].c_str()), replica = std::atoi(f[3].c_str());
  int group = -1, sid = -1, two = -1;
  std::vector<int> sg(cols), rg(rows);
  if (shard_partial_sharding(rows, cols, replica, &group, &sid, sg.data(), rg.data()) != SHARD_OK) return fail(line, "partial_sharding status", -1, 0);
  if (shard_two_phase_shard_id(rows, cols, replica, &two) != SHARD_OK) return fail(line, "two_phase status", -1, 0);
  const int want[] = {std::atoi(f[4].c_str()), std::atoi(f[5].c_str()), std::atoi(f[6].c_str()), std::atoi(f[7].c_str()),
                      std::atoi(f[8].c_str()), std::atoi(f[9].c_str()), std::atoi(f[10].c_str())};
  const int got[] = {group, sid, two, sg.front(), sg.back(), rg.front(), rg.back()};
  for (int i = 0; i < 7; ++i)
    if (got[i] != want[i]) return fail(line, "replica-array field", got[i], want[i]);
  // out-of-range arguments are refused, not computed with
  if (shard_partial_sharding(rows, cols, rows * cols, &group, &sid, nullptr, nullptr) != SHARD_EINVAL) return fail(line, "replica out of range accepted", 0, SHARD_EINVAL);
  if (shard_partial_sharding(1 << 16, 1 << 16, 0, &group, &sid, nullptr, nullptr) != SHARD_EINVAL) return fail(line, "2^32 replicas accepted", 0, SHARD_EINVAL);
  return 0;
}

int check_cut(int line, const std::vector<std::string>& f) {
  const int64_t total = std::atoll(f[1].c_str());
  const int parts = std::atoi(f[2].c_str()), part = std::atoi(f[3].c_str());
  int64_t start = -1, length = -1;
  if (shard_concat_partition(total, parts, part, &start, &length) != SHARD_OK) return fail(line, "concat_partition status", -1, 0);
  if (start != std::atoll(f[4].c_str())) return fail(line, "start", start, std::atoll(f[4].c_str()));
  if (length != std::atoll(f[5].c_str())) return fail(line, "length", length, std::atoll(f[5].c_str()));
  return 0;
}

}  // namespace

int main(int argc, char** argv) {
  if (argc != 2) {
    std::printf("usage: plan_fuzz <cases file>\n");
    return 2;
  }
  FILE* in = std::fopen(argv[1], "r");
  if (!in) return 2;
  char* buf = nullptr;
  size_t cap = 0;
  int line = 0, bad = 0, plans = 0, refused = 0;
  while (getline(&buf, &cap, in) > 0) {
    ++line;
    std::string s(buf);
    while (!s.empty() && (s.back() == '\n' || s.back() == '\r')) s.pop_back();
    if (s.empty() || s[0] == '#') continue;
    const std::vector<std::string> f = split(s, ' ');
    if (f[0] == "plan" || f[0] == "rows") {
      if (f.size() != 12) { bad += fail(line, "fields", (long long)f.size(), 12); continue; }
      ++plans;
      bad += check_plan(line, f, f[0] == "rows");
    } else if (f[0] == "part" && f.size() == 11) {
      bad += check_part(line, f);
    } else if (f[0] == "cut" && f.size() == 6) {
      bad += check_cut(line, f);
    } else {
      bad += fail(line, "unknown line", 0, 0);
    }
    if (bad) break;
  }
  std::free(buf);
  std::fclose(in);
  // degenerate and invalid arguments: refused with a status, never computed with
  shard_plan_s p;
  const int64_t one = 1, neg = -1;
  if (su::plan_build(&p, -1, &one, nullptr, 1, 8, nullptr, 0) != SHARD_EINVAL) bad += fail(0, "V < 0", 0, SHARD_EINVAL);
  if (su::plan_build(&p, 1, &one, nullptr, 0, 8, nullptr, 0) != SHARD_EINVAL) bad += fail(0, "N < 1", 0, SHARD_EINVAL);
  if (su::plan_build(&p, 1, &one, nullptr, 1, 3, nullptr, 0) != SHARD_EINVAL) bad += fail(0, "align not a power of two", 0, SHARD_EINVAL);
  if (su::plan_build(&p, 1, &neg, nullptr, 1, 8, nullptr, 0) != SHARD_EINVAL) bad += fail(0, "n < 0", 0, SHARD_EINVAL);
  if (su::plan_build(&p, 1, &one, nullptr, 1, 8, nullptr, 1000) != SHARD_EINVAL) bad += fail(0, "chunk not a multiple of 1024", 0, SHARD_EINVAL);
  if (su::plan_build(&p, 1, nullptr, nullptr, 1, 8, nullptr, 0) != SHARD_EINVAL) bad += fail(0, "numel NULL", 0, SHARD_EINVAL);
  (void)refused;
  std::printf("%d lines, %d plans, %s\n", line, plans, bad ? "FAILED" : "all agree");
  return bad ? 1 : 0;
}
