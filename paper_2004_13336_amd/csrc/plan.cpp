// Host-side sharding plan: integer layout arithmetic and the chunk table.
//
// Section 4.1 ("Data formatting"): a variable is reshaped (here: fully flattened, which moves no
// data in linear memory), padded until the shard count divides it, and sliced at an offset
// computed from the replica id.  Section 5.2 ("Batched communication operators"): a replica's
// combined shard holds one piece of every variable.
#include <limits>
#include <new>

#include "internal.hpp"

namespace su {

namespace {
constexpr int kDefaultChunk = 2048;   // measured best on MI355X for the formatting kernels
constexpr int kSplitLog2 = 26;        // models from 2^26 elements on split shard_format_all by piece size
constexpr int kFlatWalkPercent = 107; // measured cross-over on MI355X (BERT-shaped: between 32 and 64 replicas)

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
}  // namespace

int plan_build(shard_plan_t* p, int V, const int64_t* numel, const int64_t* cols, int N, int align,
               const uint32_t* flags, int chunk) {
  if (V < 0 || N < 1 || align < 1 || (align & (align - 1)) != 0) return SHARD_EINVAL;
  if (V > 0 && numel == nullptr) return SHARD_EINVAL;
  if (chunk == 0) chunk = kDefaultChunk;
  if (chunk < 1024 || chunk > 16384 || chunk % 1024 != 0) return SHARD_EINVAL;

  p->V = V;
  p->N = N;
  p->align = align;
  p->chunk = chunk;
  try {
    p->n.assign(V, 0);
    p->L.resize(V);
    p->stride.resize(V);
    p->off.resize(V);
    p->flags.assign(V, 0u);
    p->vars.resize(V);
    const int64_t kMax = std::numeric_limits<int64_t>::max() / 16;   // head-room for byte offsets
    int64_t pos = 0, total = 0;
    for (int i = 0; i < V; ++i) {
      int64_t n = numel[i], per;
      if (n < 0 || n > kMax) return SHARD_EINVAL;
      if (cols) {
        // row plan: the leading (combined) dimension is padded to a multiple of N and sliced,
        // whole rows per replica; numel[i] is the row count
        const int64_t c = cols[i];
        if (c < 0 || c > kMax || (c > 0 && n > kMax / c)) return SHARD_EINVAL;
        const int64_t rows_per = c > 0 ? (n + N - 1) / N : 0;
        if (c > 0 && rows_per > kMax / c) return SHARD_EINVAL;
        per = rows_per * c;
        n = n * c;
      } else {
        per = (n + N - 1) / N;                             // ceil(n / N)
      }
      const int64_t len = (per + align - 1) / align * align;
      if (len > kMax / N || pos > kMax - len) return SHARD_EINVAL;
      if (n > kMax - total) return SHARD_EINVAL;           // the model itself must be countable
      p->n[i] = n;
      p->L[i] = len;
      p->stride[i] = cols ? per : len;
      p->off[i] = pos;
      pos += len;
      total += n;
      if (flags) {
        if (flags[i] & ~(uint32_t)(SHARD_VAR_NO_DECAY | SHARD_VAR_NO_ADAPT)) return SHARD_EINVAL;
        p->flags[i] = flags[i];
      }
    }
    if (pos > kMax / N) return SHARD_EINVAL;               // N*S must be addressable
    p->S = pos;
    p->total = total;

    // the formatting kernels launch one workgroup per (replica, chunk, 1024-slot tile): the whole table must fit a
    // launch, which is checked before anything of it is built
    int64_t n_chunks = 0;
    for (int i = 0; i < V; ++i) {
      n_chunks += (p->L[i] + chunk - 1) / chunk;
      if (n_chunks * (chunk / 1024) > (int64_t)std::numeric_limits<int32_t>::max() / N) return SHARD_EINVAL;
    }
    p->chunks.clear();
    p->chunks.reserve((size_t)n_chunks);
    for (int i = 0; i < V; ++i) {
      VarDesc& vd = p->vars[i];
      vd.n = p->n[i];
      vd.L = p->L[i];
      vd.off = p->off[i];
      vd.stride = p->stride[i];
      vd.flags = p->flags[i];
      vd.reserved = 0;
      vd.first_chunk = (int32_t)p->chunks.size();
      vd.n_chunks = (int32_t)((p->L[i] + chunk - 1) / chunk);
      for (int64_t k0 = 0; k0 < p->L[i]; k0 += chunk) {
        ChunkDesc cd;
        cd.k0 = k0;
        cd.var = i;
        cd.len = (int32_t)((p->L[i] - k0 < chunk) ? (p->L[i] - k0) : chunk);
        p->chunks.push_back(cd);
      }
    }
    for (int s = 0; s < kPtrSlots; ++s) p->slot_ptrs[s].assign(V, nullptr);

    p->full_chunks.clear();
    if (!cols) {
      // items of the whole-model copies: the padded variables cut into chunks, variable by variable;
      // their number is at most N * (number of chunks), which the check above keeps below 2^31
      for (int i = 0; i < V; ++i) {
        const int64_t padded = (int64_t)N * p->L[i];
        for (int64_t p0 = 0; p0 < padded; p0 += chunk) {
          FullChunk fc;
          fc.p0 = p0;
          fc.var = i;
          fc.len = (int32_t)((padded - p0 < chunk) ? (padded - p0) : chunk);
          p->full_chunks.push_back(fc);
        }
      }
      // The replica-by-replica walk launches N * (chunks per shard) items, the variable-by-variable
      // one a number that does not grow with N; where pieces are large the former is the faster (7 %
      // at 8 replicas), so the latter is taken once fragments make the former's item count 7 % larger.
      p->flat_copies = (int64_t)N * (int64_t)p->chunks.size() * 100 > (int64_t)p->full_chunks.size() * kFlatWalkPercent;
      // Writes that stay contiguous matter more than reads that do: unshard_format writes the full tensors, so
      // its variable-by-variable walk is the contiguous one; shard_format_all writes the gathered rows, so for
      // variables whose pieces hold whole chunks the replica-by-replica walk is (measured: 6 to 9 % faster from
      // 64 to 256 replicas); only the small pieces, which would leave that walk's workgroups mostly empty, go
      // variable by variable.
      p->major_chunks.clear();
      p->small_full_chunks.clear();
      if (p->flat_copies) {
        // a model that fits the memory-side cache copies in tens of microseconds: a second launch costs more
        // than the split gains (ResNet-50-shaped, 32 replicas: 39 against 37 us)
        const bool split = p->total >= ((int64_t)1 << kSplitLog2);
        size_t fc = 0;
        for (int i = 0; i < V; ++i) {
          const bool big = split && p->L[i] >= chunk;
          const VarDesc& vd = p->vars[i];
          if (big)
            p->major_chunks.insert(p->major_chunks.end(), p->chunks.begin() + vd.first_chunk,
                                   p->chunks.begin() + vd.first_chunk + vd.n_chunks);
          for (; fc < p->full_chunks.size() && p->full_chunks[fc].var == i; ++fc)
            if (!big) p->small_full_chunks.push_back(p->full_chunks[fc]);
        }
      }
    }

    p->row_plan = cols != nullptr;
    p->rc_vars.clear();
    p->rc_items.clear();
    p->rc_col_items.clear();
    p->rc_row_items.clear();
    if (cols) {
      const int64_t kMaxItems = (int64_t)std::numeric_limits<int32_t>::max() / 4;
      int64_t row_off = 0, col_off = 0, cp = 0, rp = 0;
      for (int i = 0; i < V; ++i) {
        RowColVar rv;
        rv.off = p->off[i];
        rv.rows = numel[i];
        rv.cols = cols[i];
        rv.Lr = cols[i] > 0 ? (numel[i] + N - 1) / N : 0;
        rv.L = p->L[i];
        const bool vec = cols[i] % 4 == 0 && p->off[i] % 4 == 0;
        const bool flat = rv.Lr <= kRowBlock / 4;
        rv.shape = (vec ? kRcVec : 0) | (flat ? kRcFlat : 0);
        const int64_t span = (kBlock / 4) * (vec ? 4 : 1);              // columns one wavefront covers
        const int64_t tile_cols = flat ? 4 * span : span;
        const int64_t tile_rows = flat ? kRowBlock / 4 : kRowBlock;
        const int64_t n_rb = (rv.Lr + tile_rows - 1) / tile_rows;
        const int64_t n_ct = rv.Lr > 0 ? (rv.cols + tile_cols - 1) / tile_cols : 0;
        const int64_t span_c = col_span((int)(n_rb > kMaxItems ? kMaxItems : n_rb));
        const int64_t n_col = (rv.cols + span_c - 1) / span_c;   // also for a variable without rows: its column sums are 0
        if (n_rb > kMaxItems || n_ct > kMaxItems || n_col > kMaxItems) return SHARD_EINVAL;
        if (n_rb * n_ct + (int64_t)p->rc_items.size() > kMaxItems) return SHARD_EINVAL;
        if (n_col + (int64_t)p->rc_col_items.size() > kMaxItems) return SHARD_EINVAL;
        rv.n_rb = (int32_t)n_rb;
        rv.n_ct = (int32_t)n_ct;
        rv.row_off = row_off;
        rv.col_off = col_off;
        rv.cp_off = cp;
        rv.rp_off = rp;
        rv.first_item = (int32_t)p->rc_items.size();
        rv.first_col_item = (int32_t)p->rc_col_items.size();
        rv.n_col_items = (int32_t)n_col;
        row_off += rv.Lr;
        col_off += rv.cols;
        cp += (n_rb * rv.cols + 3) / 4 * 4;                // keeps every variable's partials 16-byte aligned
        rp += n_ct * rv.Lr;
        p->rc_vars.push_back(rv);
        for (int64_t rb = 0; rb < n_rb; ++rb)
          for (int64_t ct = 0; ct < n_ct; ++ct) p->rc_items.push_back(RowColItem{i, (int32_t)rb, (int32_t)ct, 0});
        for (int64_t t = 0; t < n_col; ++t) p->rc_col_items.push_back(ColItem{i, (int32_t)t});
        const bool wide = n_ct > kWideTiles;
        const int64_t row_step = wide ? 1 : kBlock;
        if ((rv.Lr + row_step - 1) / row_step + (int64_t)p->rc_row_items.size() > kMaxItems) return SHARD_EINVAL;
        for (int64_t k = 0; k < rv.Lr; k += row_step) p->rc_row_items.push_back(RowItem{i, wide ? 1 : 0, k});
      }
      p->rc_total_rows = row_off;
      p->rc_total_cols = col_off;
      p->rc_colpart_elems = cp;
      p->rc_rowpart_elems = rp;
    }
  } catch (const std::bad_alloc&) {
    return SHARD_ENOMEM;
  }
  Workspace ws;
  p->ws_need = workspace_layout(p, &ws);
  return SHARD_OK;
}

size_t workspace_layout(const shard_plan_t* p, Workspace* ws) {
  size_t pos = 0;
  const size_t V = (size_t)p->V, C = p->chunks.size();
  ws->vars = pos;        pos = align_up(pos + V * sizeof(VarDesc), 256);
  ws->chunks = pos;      pos = align_up(pos + C * sizeof(ChunkDesc), 256);
  ws->ptrs = pos;        pos = align_up(pos + (size_t)kPtrSlots * V * sizeof(void*), 256);
  ws->chunk_sums = pos;  pos = align_up(pos + C * 2 * sizeof(float), 256);
  ws->var_sums = pos;    pos = align_up(pos + V * 2 * sizeof(float), 256);
  ws->full_chunks = pos; pos = align_up(pos + p->full_chunks.size() * sizeof(FullChunk), 256);
  ws->major_chunks = pos;      pos = align_up(pos + p->major_chunks.size() * sizeof(ChunkDesc), 256);
  ws->small_full_chunks = pos; pos = align_up(pos + p->small_full_chunks.size() * sizeof(FullChunk), 256);
  if (p->row_plan) {
    ws->rc_vars = pos;     pos = align_up(pos + p->rc_vars.size() * sizeof(RowColVar), 256);
    ws->rc_items = pos;    pos = align_up(pos + p->rc_items.size() * sizeof(RowColItem), 256);
    ws->rc_colpart = pos;  pos = align_up(pos + (size_t)p->rc_colpart_elems * sizeof(float), 256);
    ws->rc_rowpart = pos;  pos = align_up(pos + (size_t)p->rc_rowpart_elems * sizeof(float), 256);
    ws->rc_col_items = pos;    pos = align_up(pos + p->rc_col_items.size() * sizeof(ColItem), 256);
    ws->rc_row_items = pos;    pos = align_up(pos + p->rc_row_items.size() * sizeof(RowItem), 256);
    ws->rc_colitem_part = pos; pos = align_up(pos + p->rc_col_items.size() * sizeof(float), 256);
    const size_t items = p->rc_items.size(), rows = (size_t)p->rc_total_rows, cols = (size_t)p->rc_total_cols;
    ws->af_wpart = pos;    pos = align_up(pos + items * sizeof(float), 256);
    ws->af_upart = pos;    pos = align_up(pos + items * sizeof(float), 256);
    ws->af_inv_r = pos;    pos = align_up(pos + rows * sizeof(float), 256);
    ws->af_inv_c = pos;    pos = align_up(pos + cols * sizeof(float), 256);
    ws->af_rowsq = pos;    pos = align_up(pos + rows * sizeof(float), 256);
    ws->af_colsq = pos;    pos = align_up(pos + cols * sizeof(float), 256);
    ws->af_table = pos;    pos = align_up(pos + V * 2 * sizeof(float), 256);
    ws->af_usq = pos;      pos = align_up(pos + V * sizeof(float), 256);
  }
  return pos < 256 ? 256 : pos;
}

}  // namespace su
