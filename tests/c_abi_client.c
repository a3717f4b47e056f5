/* A plain C client of libshardupdate.so: no PyTorch, no C++.  It shows that the boundary is usable
 * from C with nothing but the HIP runtime for device memory, and checks one pass of the path
 * (plan -> bind -> format -> momentum update with mu = 0 -> unshard) against the closed form
 * w' = w - lr (g + wd w), evaluated here in double, then repeats the update with the gradient read in place
 * from the full tensors and compares the shards bit for bit, runs the copy-order set-up call, and compares LAMB with its sums
 * in the library's static array against LAMB with its sums in the workspace.  Exit status 0 = pass.
 *
 * Built by __graft_entry__.build() with gcc; run by tests/test_gpu_f_c_client.py on a GPU machine. */
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "shardupdate.h"

#define CHECK_HIP(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { \
  fprintf(stderr, "HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); return 2; } } while (0)
#define CHECK_SU(x) do { int s_ = (x); if (s_ != SHARD_OK) { \
  fprintf(stderr, "shardupdate error '%s' at line %d\n", shard_strerror(s_), __LINE__); return 3; } } while (0)

enum { V = 3, N = 3, R = 1 };

static float pattern(int var, long k, int kind) {          /* deterministic, sign-alternating values */
  unsigned long x = (unsigned long)(var + 1) * 2654435761ul + (unsigned long)k * 40503ul + (unsigned long)kind * 977ul;
  x ^= x >> 13; x *= 0x9E3779B1ul; x ^= x >> 16;
  return ((float)(x % 20001ul) - 10000.0f) * (kind == 0 ? 2e-6f : 1e-7f);
}

int main(void) {
  const int64_t numel[V] = {1000, 37, 4099};
  const float lr = 0.1f, wd = 5e-5f;
  shard_plan_t* plan = NULL;
  int64_t S = 0, total = 0, seg_off[V], seg_len[V], real[V];
  size_t ws_bytes = 0;
  void *ws = NULL, *w = NULL, *g = NULL, *m = NULL, *gathered = NULL;
  void* full_w[V]; void* full_g[V]; void* full_out[V];
  float* host[V]; float* hostg[V];
  int i, failures = 0;
  int devices = 0;
  CHECK_HIP(hipGetDeviceCount(&devices));
  if (devices < 1) { fprintf(stderr, "no GPU\n"); return 2; }

  CHECK_SU(shard_plan(V, numel, N, 8, NULL, 0, &plan));
  CHECK_SU(shard_plan_info(plan, &S, &total, NULL, NULL, &ws_bytes));
  CHECK_SU(shard_plan_segments(plan, seg_off, seg_len));
  CHECK_SU(shard_plan_real_count(plan, R, real));
  CHECK_HIP(hipMalloc(&ws, ws_bytes));
  CHECK_SU(shard_plan_bind(plan, ws, ws_bytes, NULL));

  for (i = 0; i < V; ++i) {
    long k;
    host[i] = (float*)malloc(sizeof(float) * (size_t)numel[i]);
    hostg[i] = (float*)malloc(sizeof(float) * (size_t)numel[i]);
    for (k = 0; k < numel[i]; ++k) { host[i][k] = pattern(i, k, 0); hostg[i][k] = pattern(i, k, 1); }
    CHECK_HIP(hipMalloc(&full_w[i], sizeof(float) * (size_t)numel[i]));
    CHECK_HIP(hipMalloc(&full_g[i], sizeof(float) * (size_t)numel[i]));
    CHECK_HIP(hipMalloc(&full_out[i], sizeof(float) * (size_t)numel[i]));
    CHECK_HIP(hipMemcpy(full_w[i], host[i], sizeof(float) * (size_t)numel[i], hipMemcpyHostToDevice));
    CHECK_HIP(hipMemcpy(full_g[i], hostg[i], sizeof(float) * (size_t)numel[i], hipMemcpyHostToDevice));
    CHECK_HIP(hipMemset(full_out[i], 0xFF, sizeof(float) * (size_t)numel[i]));
  }
  CHECK_HIP(hipMalloc(&gathered, sizeof(float) * (size_t)(N * S)));
  CHECK_HIP(hipMemset(gathered, 0, sizeof(float) * (size_t)(N * S)));
  w = (char*)gathered + sizeof(float) * (size_t)(R * S);      /* replica R's row of the gathered buffer */
  CHECK_HIP(hipMalloc(&g, sizeof(float) * (size_t)S));
  CHECK_HIP(hipMalloc(&m, sizeof(float) * (size_t)S));
  CHECK_HIP(hipMemset(m, 0, sizeof(float) * (size_t)S));

  CHECK_SU(shard_format(plan, R, (const void* const*)full_w, SHARD_F32, w, SHARD_F32, NULL));
  CHECK_SU(shard_format(plan, R, (const void* const*)full_g, SHARD_F32, g, SHARD_F32, NULL));
  {
    shard_momentum_hp hp;
    hp.lr = lr; hp.mu = 0.0f; hp.weight_decay = wd;
    CHECK_SU(shard_update_momentum(plan, R, (float*)w, (const float*)g, (float*)m, NULL, &hp, NULL));
  }
  CHECK_SU(unshard_format(plan, gathered, 0, SHARD_F32, full_out, SHARD_F32, NULL));
  CHECK_HIP(hipDeviceSynchronize());

  for (i = 0; i < V; ++i) {
    long k;
    float* got = (float*)malloc(sizeof(float) * (size_t)numel[i]);
    CHECK_HIP(hipMemcpy(got, full_out[i], sizeof(float) * (size_t)numel[i], hipMemcpyDeviceToHost));
    for (k = 0; k < numel[i]; ++k) {
      const long first = (long)R * (long)seg_len[i];
      const int mine = k >= first && k < first + (long)real[i];
      /* rows of the other replicas were zero, so their elements come back as +0.0 */
      const double want = mine ? (double)host[i][k] - (double)lr * ((double)hostg[i][k] + (double)wd * (double)host[i][k]) : 0.0;
      if (fabs((double)got[k] - want) > 1e-6 * (1.0 + fabs(want))) {
        if (failures < 5) fprintf(stderr, "var %d elem %ld: got %.9g want %.9g\n", i, k, (double)got[k], want);
        ++failures;
      }
    }
    free(got);
  }
  /* the same update with the gradient read in place from the full tensors: the same bits in the shard */
  {
    void *w2 = NULL, *m2 = NULL;
    float *a = (float*)malloc(sizeof(float) * (size_t)S), *b = (float*)malloc(sizeof(float) * (size_t)S);
    shard_momentum_hp hp;
    hp.lr = lr; hp.mu = 0.0f; hp.weight_decay = wd;
    CHECK_HIP(hipMalloc(&w2, sizeof(float) * (size_t)S));
    CHECK_HIP(hipMalloc(&m2, sizeof(float) * (size_t)S));
    CHECK_HIP(hipMemset(m2, 0, sizeof(float) * (size_t)S));
    CHECK_SU(shard_format(plan, R, (const void* const*)full_w, SHARD_F32, w2, SHARD_F32, NULL));
    CHECK_SU(shard_update_momentum_full_grads(plan, R, (float*)w2, (const void* const*)full_g, SHARD_F32, (float*)m2, NULL,
                                              &hp, NULL));
    CHECK_HIP(hipDeviceSynchronize());
    CHECK_HIP(hipMemcpy(a, w, sizeof(float) * (size_t)S, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(b, w2, sizeof(float) * (size_t)S, hipMemcpyDeviceToHost));
    if (memcmp(a, b, sizeof(float) * (size_t)S) != 0) {
      fprintf(stderr, "shard_update_momentum_full_grads differs from shard_format + shard_update_momentum\n");
      ++failures;
    }
    free(a); free(b); hipFree(w2); hipFree(m2);
  }
  /* the whole-model copy once more in each order: the same bytes in the full tensors */
  {
    int order, walk = -1;
    for (order = SHARD_WALK_BY_REPLICA; order <= SHARD_WALK_BY_VARIABLE; ++order) {
      CHECK_SU(shard_plan_set_copy_walk(plan, order));
      CHECK_SU(shard_plan_copy_walk(plan, SHARD_COPY_UNSHARD, (const void* const*)full_out, &walk, NULL));
      if (walk != order) { fprintf(stderr, "copy order %d reported as %d\n", order, walk); ++failures; }
      for (i = 0; i < V; ++i) {
        float* before = (float*)malloc(sizeof(float) * (size_t)numel[i]);
        float* after = (float*)malloc(sizeof(float) * (size_t)numel[i]);
        CHECK_HIP(hipMemcpy(before, full_out[i], sizeof(float) * (size_t)numel[i], hipMemcpyDeviceToHost));
        CHECK_HIP(hipMemset(full_out[i], 0xFF, sizeof(float) * (size_t)numel[i]));
        CHECK_SU(unshard_format(plan, gathered, 0, SHARD_F32, full_out, SHARD_F32, NULL));
        CHECK_HIP(hipDeviceSynchronize());
        CHECK_HIP(hipMemcpy(after, full_out[i], sizeof(float) * (size_t)numel[i], hipMemcpyDeviceToHost));
        if (memcmp(before, after, sizeof(float) * (size_t)numel[i]) != 0) {
          fprintf(stderr, "unshard_format in order %d differs in variable %d\n", order, i);
          ++failures;
        }
        free(before); free(after);
      }
    }
    CHECK_SU(shard_plan_set_copy_walk(plan, SHARD_WALK_AUTO));
    if (shard_plan_set_copy_walk(plan, 7) != SHARD_EINVAL) ++failures;
  }
  /* the set-up call that measures both orders (or reports the fixed one) leaves the full tensors as the copy does */
  {
    int walk = -1;
    float ms[2] = {-1.0f, -1.0f};
    CHECK_SU(shard_plan_tune_copy_walk(plan, SHARD_COPY_UNSHARD, gathered, 0, SHARD_F32, full_out, SHARD_F32, NULL, &walk, ms));
    if (walk != SHARD_WALK_BY_REPLICA && walk != SHARD_WALK_BY_VARIABLE) { fprintf(stderr, "tuned order %d\n", walk); ++failures; }
    if (shard_plan_tune_copy_walk(plan, 5, gathered, 0, SHARD_F32, full_out, SHARD_F32, NULL, &walk, ms) != SHARD_EINVAL) ++failures;
  }
  /* LAMB with its intermediate sums in the library's static device array: the bits of shard_update_lamb */
  {
    void *wa = NULL, *wb = NULL, *ma = NULL, *mb = NULL, *va = NULL, *vb = NULL;
    float *a = (float*)malloc(sizeof(float) * (size_t)S), *b = (float*)malloc(sizeof(float) * (size_t)S);
    shard_lamb_hp hp;
    hp.lr = 1e-3f; hp.beta1 = 0.9f; hp.beta2 = 0.999f; hp.eps = 1e-6f; hp.weight_decay = 0.01f;
    CHECK_HIP(hipMalloc(&wa, sizeof(float) * (size_t)S)); CHECK_HIP(hipMalloc(&wb, sizeof(float) * (size_t)S));
    CHECK_HIP(hipMalloc(&ma, sizeof(float) * (size_t)S)); CHECK_HIP(hipMalloc(&mb, sizeof(float) * (size_t)S));
    CHECK_HIP(hipMalloc(&va, sizeof(float) * (size_t)S)); CHECK_HIP(hipMalloc(&vb, sizeof(float) * (size_t)S));
    CHECK_HIP(hipMemset(ma, 0, sizeof(float) * (size_t)S)); CHECK_HIP(hipMemset(mb, 0, sizeof(float) * (size_t)S));
    CHECK_HIP(hipMemset(va, 0, sizeof(float) * (size_t)S)); CHECK_HIP(hipMemset(vb, 0, sizeof(float) * (size_t)S));
    CHECK_SU(shard_format(plan, R, (const void* const*)full_w, SHARD_F32, wa, SHARD_F32, NULL));
    CHECK_SU(shard_format(plan, R, (const void* const*)full_w, SHARD_F32, wb, SHARD_F32, NULL));
    CHECK_SU(shard_update_lamb(plan, R, (float*)wa, (const float*)g, (float*)ma, (float*)va, NULL, &hp, 1, NULL, NULL, NULL));
    CHECK_SU(shard_update_lamb_noalloc(plan, R, (float*)wb, (const float*)g, (float*)mb, (float*)vb, NULL, &hp, 1, NULL, NULL, NULL));
    CHECK_HIP(hipDeviceSynchronize());
    CHECK_HIP(hipMemcpy(a, wa, sizeof(float) * (size_t)S, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(b, wb, sizeof(float) * (size_t)S, hipMemcpyDeviceToHost));
    if (memcmp(a, b, sizeof(float) * (size_t)S) != 0) { fprintf(stderr, "shard_update_lamb_noalloc differs from shard_update_lamb\n"); ++failures; }
    free(a); free(b); hipFree(wa); hipFree(wb); hipFree(ma); hipFree(mb); hipFree(va); hipFree(vb);
  }
  /* an error path: replica id out of range */
  if (shard_format(plan, N, (const void* const*)full_w, SHARD_F32, w, SHARD_F32, NULL) != SHARD_EINVAL) ++failures;

  shard_plan_free(plan);
  for (i = 0; i < V; ++i) { hipFree(full_w[i]); hipFree(full_g[i]); hipFree(full_out[i]); free(host[i]); free(hostg[i]); }
  hipFree(gathered); hipFree(g); hipFree(m); hipFree(ws);
  if (failures) { fprintf(stderr, "c_abi_client: %d mismatches\n", failures); return 1; }
  printf("c_abi_client ok: S=%ld total=%ld workspace=%zu bytes\n", (long)S, (long)total, ws_bytes);
  return 0;
}
