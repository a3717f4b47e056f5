// HIP kernels for row plans (gfx950): reductions that keep a dimension, and Adafactor on a
// row-sharded shard.
//
// Section 4.1, "Non-elementwise operators": a reduce collapses some dimensions and passes others
// through, and the sharding format may not merge the two kinds.  With whole rows per replica, a
// reduce over columns is complete on the replica that owns the row, a reduce over rows gives
// per-replica partial results for an all-reduce, and padded rows contribute the identity.  Adafactor
// (named in Section 3 as an optimizer with such reduces) needs exactly these two reductions of the
// squared gradient, plus two scalars per variable.
//
// Work items are (variable, row block, column tile) triples from the plan: kRowBlock rows x one
// column tile.  Every thread owns 4 adjacent columns (1 where rows do not start on 16-byte
// boundaries) and walks down the rows in batches of kRowBatch independent 128-bit loads, so the
// reductions along rows stay in registers and those along columns go through LDS once per item.
// All sums are taken in an order fixed by the plan: results are run-to-run identical.
#include "device_common.hpp"

#ifndef SU_NT_ROWCOL
#define SU_NT_ROWCOL 1     // 1: non-temporal loads of the tensor that is only reduced
#endif
#ifndef SU_NT_ADAFACTOR
#define SU_NT_ADAFACTOR 0  // cache policy mask of the Adafactor kernels (4: g, 2: w loads, 1: stores)
#endif

namespace su {
namespace {

constexpr int kRowBatch = 8;
typedef Policy<SU_NT_ADAFACTOR> PolAf;

// The part of a work item every kernel here needs.
struct Tile {
  RowColVar v;
  int64_t col0;      // first column this thread owns
  int64_t row0;      // first row of the item inside the replica's piece
  int64_t first;     // offset, in the packed shard, of (row0, col0)
  int in_block;      // rows of the piece in this item
  int live;          // leading rows of the item that exist in the full matrix (position = replica
                     // offset + index, compared with the full row count)
  int var;
  bool vec, col_ok;
};

__device__ __forceinline__ Tile tile_of(const RowColVar* __restrict__ vars, const RowColItem* __restrict__ items, int r) {
  Tile t;
  const RowColItem it = items[blockIdx.x];
  t.var = it.var;
  t.v = vars[it.var];
  t.vec = t.v.vec != 0;
  const int w = t.vec ? 4 : 1;
  t.col0 = (int64_t)it.ct * (kBlock * w) + (int64_t)threadIdx.x * w;
  t.row0 = (int64_t)it.rb * kRowBlock;
  int64_t real_rows = t.v.rows - (int64_t)r * t.v.Lr;
  real_rows = real_rows < 0 ? 0 : (real_rows > t.v.Lr ? t.v.Lr : real_rows);
  t.in_block = (int)((t.v.Lr - t.row0 < kRowBlock) ? (t.v.Lr - t.row0) : kRowBlock);
  const int64_t left = real_rows - t.row0;
  t.live = (int)(left < 0 ? 0 : (left < t.in_block ? left : t.in_block));
  t.col_ok = t.col0 < t.v.cols;
  t.first = t.v.off + t.row0 * t.v.cols + t.col0;
  return t;
}

// Sum over the workgroup, fixed order, valid in thread 0.
__device__ __forceinline__ float block_sum1(float a) {
  __shared__ float part[kBlock / 64];
#pragma unroll
  for (int s = 32; s >= 1; s >>= 1) a += __shfl_xor(a, s, 64);
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = a;
  __syncthreads();
  if (threadIdx.x == 0) {
    a = part[0];
#pragma unroll
    for (int w = 1; w < kBlock / 64; ++w) a += part[w];
  }
  return a;
}

// Sum over the workgroup of float64 values, fixed order, valid in thread 0.
__device__ __forceinline__ double block_sum_f64(double a) {
  __shared__ double part[kBlock / 64];
#pragma unroll
  for (int s = 32; s >= 1; s >>= 1) a += __shfl_xor(a, s, 64);
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = a;
  __syncthreads();
  if (threadIdx.x == 0) {
    a = part[0];
#pragma unroll
    for (int w = 1; w < kBlock / 64; ++w) a += part[w];
  }
  return a;
}

// ---- row / column sums of squares -------------------------------------------------------------------
// One pass over x.  Per item: the item's row sums (over its column tile) and column sums (over its
// live rows) go to the workspace as partial results; rowcol_p2_kernel adds them.  WITH_W: the same
// pass also reads a second tensor y at the same positions and leaves the item's sum of y^2 over real
// elements in ypart (Adafactor's RMS of the weights).
template <bool WITH_W>
__global__ __launch_bounds__(kBlock) void rowcol_p1_kernel(const RowColVar* __restrict__ vars,
                                                           const RowColItem* __restrict__ items,
                                                           const float* __restrict__ x, const float* __restrict__ y,
                                                           float* __restrict__ colpart, float* __restrict__ rowpart,
                                                           float* __restrict__ ypart, int r) {
  __shared__ float row_lds[kRowBlock][kBlock];
  const Tile t = tile_of(vars, items, r);
  const RowColItem it = items[blockIdx.x];
  const float* base = x + t.first;
  const float* ybase = y + t.first;
  float c0 = 0.0f, c1 = 0.0f, c2 = 0.0f, c3 = 0.0f, sy = 0.0f;
  for (int rr0 = 0; rr0 < t.in_block; rr0 += kRowBatch) {
    F4 val[kRowBatch], wv[kRowBatch];
#pragma unroll
    for (int j = 0; j < kRowBatch; ++j) {
      val[j] = F4{0.0f, 0.0f, 0.0f, 0.0f};
      if constexpr (WITH_W) wv[j] = F4{0.0f, 0.0f, 0.0f, 0.0f};
      if (rr0 + j < t.live && t.col_ok) {
        const int64_t o = (int64_t)(rr0 + j) * t.v.cols;
        if (t.vec) {
          val[j] = ld4<SU_NT_ROWCOL != 0>(base + o);
          if constexpr (WITH_W) wv[j] = ld4<false>(ybase + o);
        } else {
          val[j].x = ld<SU_NT_ROWCOL != 0>(base + o);
          if constexpr (WITH_W) wv[j].x = ybase[o];
        }
      }
    }
#pragma unroll
    for (int j = 0; j < kRowBatch; ++j) {
      if (rr0 + j < t.in_block) {
        const float a = val[j].x * val[j].x, b = val[j].y * val[j].y, c = val[j].z * val[j].z, d = val[j].w * val[j].w;
        c0 += a; c1 += b; c2 += c; c3 += d;
        row_lds[rr0 + j][threadIdx.x] = (a + b) + (c + d);
        if constexpr (WITH_W)
          sy += (wv[j].x * wv[j].x + wv[j].y * wv[j].y) + (wv[j].z * wv[j].z + wv[j].w * wv[j].w);
      }
    }
  }
  if (t.col_ok) {
    float* cp = colpart + t.v.cp_off + (int64_t)it.rb * t.v.cols + t.col0;
    if (t.vec) st4<false>(cp, F4{c0, c1, c2, c3});
    else cp[0] = c0;
  }
  __syncthreads();
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  for (int row = wave; row < t.in_block; row += kBlock / 64) {
    float s = (row_lds[row][lane] + row_lds[row][lane + 64]) + (row_lds[row][lane + 128] + row_lds[row][lane + 192]);
#pragma unroll
    for (int sh = 32; sh >= 1; sh >>= 1) s += __shfl_xor(s, sh, 64);
    if (lane == 0) rowpart[t.v.rp_off + (int64_t)it.ct * t.v.Lr + t.row0 + row] = s;
  }
  if constexpr (WITH_W) {
    sy = block_sum1(sy);
    if (threadIdx.x == 0) ypart[blockIdx.x] = sy;
  }
}

// blockIdx.x = variable, blockIdx.y strides over its columns and rows.  Adds the partial results of
// phase 1 in a fixed order; other_col (nullable, laid out like col_out) is added to the column
// sums.  With table_out, the y = 0 workgroup of every variable also writes
//   table_out[2i]   = sum of ypart over the variable's items      (+ other_table)
//   table_out[2i+1] = sum of row_state over the replica's real rows (+ other_table)
__global__ __launch_bounds__(kBlock) void rowcol_p2_kernel(const RowColVar* __restrict__ vars,
                                                           const float* __restrict__ colpart,
                                                           const float* __restrict__ rowpart,
                                                           float* __restrict__ row_out, float* __restrict__ col_out,
                                                           const float* __restrict__ other_col,
                                                           const float* __restrict__ ypart,
                                                           const float* __restrict__ row_state,
                                                           const float* __restrict__ other_table,
                                                           float* __restrict__ table_out, int r) {
  const int i = blockIdx.x;
  const RowColVar v = vars[i];
  const int64_t step = (int64_t)gridDim.y * kBlock;
  for (int64_t c = (int64_t)blockIdx.y * kBlock + threadIdx.x; c < v.cols; c += step) {
    float s = 0.0f;
    for (int rb = 0; rb < v.n_rb; ++rb) s += colpart[v.cp_off + (int64_t)rb * v.cols + c];
    if (other_col) s += other_col[v.col_off + c];
    col_out[v.col_off + c] = s;
  }
  for (int64_t k = (int64_t)blockIdx.y * kBlock + threadIdx.x; k < v.Lr; k += step) {
    float s = 0.0f;
    for (int ct = 0; ct < v.n_ct; ++ct) s += rowpart[v.rp_off + (int64_t)ct * v.Lr + k];
    row_out[v.row_off + k] = s;
  }
  if (table_out != nullptr && blockIdx.y == 0) {
    const int64_t n_items = (int64_t)v.n_rb * v.n_ct;
    double a = 0.0, b = 0.0;
    for (int64_t k = threadIdx.x; k < n_items; k += kBlock) a += (double)ypart[v.first_item + k];
    int64_t real_rows = v.rows - (int64_t)r * v.Lr;
    real_rows = real_rows < 0 ? 0 : (real_rows > v.Lr ? v.Lr : real_rows);
    for (int64_t k = threadIdx.x; k < real_rows; k += kBlock) b += (double)row_state[v.row_off + k];
    a = block_sum_f64(a);
    __syncthreads();
    b = block_sum_f64(b);
    if (threadIdx.x == 0) {
      const float fa = (float)a, fb = (float)b;
      table_out[2 * i] = other_table ? fa + other_table[2 * i] : fa;
      table_out[2 * i + 1] = other_table ? fb + other_table[2 * i + 1] : fb;
    }
  }
}

// ---- Adafactor ----------------------------------------------------------------------------------------
// Factored second moments on a row-sharded matrix (rows x cols, this replica owns Lr rows):
//   R_k  = beta2 R_k + (1-beta2) (sum_j g_kj^2 + cols eps1)        local rows; padded rows keep 0
//   C_j  = beta2 C_j + (1-beta2) (sum_k g_kj^2 + rows eps1)        sums over ALL replicas' rows
//   Vhat_kj = R_k C_j / sum(R),  U = G / sqrt(Vhat) = G * rsqrt(R_k) * rsqrt(C_j / sum(R))
// A variable with cols == 1 is a vector: R holds the unfactored second moment and Vhat = R.
// sum(R) over all replicas' rows follows from all-reduced quantities:
//   sum(R) = beta2 * (all-reduced sum of the old R) + (1-beta2) * (sum_j all-reduced column sums + rows cols eps1).

// One workgroup per variable: sum(R) of the new row state.
__global__ __launch_bounds__(kBlock) void adafactor_sumr_kernel(const RowColVar* __restrict__ vars,
                                                                const float* __restrict__ col_sq_global,
                                                                const float* __restrict__ table_global,
                                                                float* __restrict__ sum_r, AdafactorK k) {
  const int i = blockIdx.x;
  const RowColVar v = vars[i];
  double s = 0.0;
  for (int64_t c = threadIdx.x; c < v.cols; c += kBlock) s += (double)col_sq_global[v.col_off + c];
  s = block_sum_f64(s);
  if (threadIdx.x == 0) {
    const double n = (double)v.rows * (double)v.cols;
    sum_r[i] = (float)((double)k.beta2 * (double)table_global[2 * i + 1] + (double)k.omb2 * (s + n * (double)k.eps1));
  }
}

// blockIdx.x = variable, blockIdx.y strides over its rows and columns: new state, and the two factors
// of 1/sqrt(Vhat): inv_r[k] = rsqrt(R_k) (0 for padded rows), inv_c[j] = rsqrt(C_j / sum(R)).
__global__ __launch_bounds__(kBlock) void adafactor_state_kernel(const RowColVar* __restrict__ vars,
                                                                 const float* __restrict__ row_sq,
                                                                 const float* __restrict__ col_sq_global,
                                                                 const float* __restrict__ sum_r, float* R, float* C,
                                                                 float* __restrict__ inv_r, float* __restrict__ inv_c,
                                                                 int r, AdafactorK k) {
  const int i = blockIdx.x;
  const RowColVar v = vars[i];
  const int64_t step = (int64_t)gridDim.y * kBlock;
  int64_t real_rows = v.rows - (int64_t)r * v.Lr;
  real_rows = real_rows < 0 ? 0 : (real_rows > v.Lr ? v.Lr : real_rows);
  const float row_eps = (float)v.cols * k.eps1, col_eps = (float)v.rows * k.eps1;
  for (int64_t q = (int64_t)blockIdx.y * kBlock + threadIdx.x; q < v.Lr; q += step) {
    float rn = 0.0f, inv = 0.0f;
    if (q < real_rows) {
      rn = fmaf(k.beta2, R[v.row_off + q], k.omb2 * (row_sq[v.row_off + q] + row_eps));
      inv = 1.0f / sqrtf(rn);
    }
    R[v.row_off + q] = rn;
    inv_r[v.row_off + q] = inv;
  }
  if (v.cols == 1) {
    if (blockIdx.y == 0 && threadIdx.x == 0) inv_c[v.col_off] = 1.0f;      // vector: Vhat = R, no column state
    return;
  }
  const float total = sum_r[i];
  for (int64_t c = (int64_t)blockIdx.y * kBlock + threadIdx.x; c < v.cols; c += step) {
    const float cn = fmaf(k.beta2, C[v.col_off + c], k.omb2 * (col_sq_global[v.col_off + c] + col_eps));
    C[v.col_off + c] = cn;
    inv_c[v.col_off + c] = 1.0f / sqrtf(cn / total);
  }
}

// The 4 (or 1) column factors of this thread.  Column offsets of different variables are not
// multiples of 4, so these are scalar loads; they are cached and read once per item.
__device__ __forceinline__ F4 column_factors(const Tile& t, const float* __restrict__ inv_c) {
  F4 f{0.0f, 0.0f, 0.0f, 0.0f};
  if (!t.col_ok) return f;
  const float* p = inv_c + t.v.col_off + t.col0;
  f.x = p[0];
  if (t.vec) {
    f.y = p[1];
    f.z = p[2];
    f.w = p[3];
  }
  return f;
}

// Per item: sum of U^2 over real elements, U = g * inv_r[row] * inv_c[col].
__global__ __launch_bounds__(kBlock) void adafactor_usq_kernel(const RowColVar* __restrict__ vars,
                                                               const RowColItem* __restrict__ items,
                                                               const float* __restrict__ g,
                                                               const float* __restrict__ inv_r,
                                                               const float* __restrict__ inv_c,
                                                               float* __restrict__ upart, int r) {
  const Tile t = tile_of(vars, items, r);
  const F4 fc = column_factors(t, inv_c);
  const float* base = g + t.first;
  const float* rows = inv_r + t.v.row_off + t.row0;
  float s = 0.0f;
  for (int rr0 = 0; rr0 < t.live; rr0 += kRowBatch) {
    F4 val[kRowBatch];
#pragma unroll
    for (int j = 0; j < kRowBatch; ++j) {
      val[j] = F4{0.0f, 0.0f, 0.0f, 0.0f};
      if (rr0 + j < t.live && t.col_ok) {
        const int64_t o = (int64_t)(rr0 + j) * t.v.cols;
        if (t.vec) val[j] = ld4<PolAf::RO>(base + o);
        else val[j].x = ld<PolAf::RO>(base + o);
      }
    }
#pragma unroll
    for (int j = 0; j < kRowBatch; ++j) {
      if (rr0 + j < t.live) {
        const float fr = rows[rr0 + j];
        const float a = (val[j].x * fr) * fc.x, b = (val[j].y * fr) * fc.y, c = (val[j].z * fr) * fc.z,
                    d = (val[j].w * fr) * fc.w;
        s += (a * a + b * b) + (c * c + d * d);
      }
    }
  }
  s = block_sum1(s);
  if (threadIdx.x == 0) upart[blockIdx.x] = s;
}

// One workgroup per variable: adds the variable's item partials in a fixed order.
__global__ __launch_bounds__(kBlock) void item_total_kernel(const RowColVar* __restrict__ vars,
                                                            const float* __restrict__ part,
                                                            const float* __restrict__ other, float* __restrict__ local_out,
                                                            float* __restrict__ total_out) {
  const int i = blockIdx.x;
  const RowColVar v = vars[i];
  const int64_t n_items = (int64_t)v.n_rb * v.n_ct;
  double a = 0.0;
  for (int64_t q = threadIdx.x; q < n_items; q += kBlock) a += (double)part[v.first_item + q];
  a = block_sum_f64(a);
  if (threadIdx.x == 0) {
    const float fa = (float)a;
    if (local_out) local_out[i] = fa;
    if (total_out) total_out[i] = other ? fa + other[i] : fa;
  }
}

// Per item: X -= alpha * U / max(1, RMS(U) / d) on real elements; padded rows and the alignment tail
// of the piece are left as they are (and copied to the bfloat16 output, if any).
template <bool BF16>
__global__ __launch_bounds__(kBlock) void adafactor_apply_kernel(const RowColVar* __restrict__ vars,
                                                                 const RowColItem* __restrict__ items, float* w,
                                                                 const float* __restrict__ g,
                                                                 const float* __restrict__ inv_r,
                                                                 const float* __restrict__ inv_c,
                                                                 const float* __restrict__ table_global,
                                                                 const float* __restrict__ usq_global,
                                                                 uint16_t* __restrict__ w16, int r, AdafactorK k) {
  const Tile t = tile_of(vars, items, r);
  const RowColItem it = items[blockIdx.x];
  const float n = (float)t.v.rows * (float)t.v.cols;
  const float rms_x = sqrtf(table_global[2 * t.var] / n), rms_u = sqrtf(usq_global[t.var] / n);
  const float alpha = fmaxf(k.eps2, rms_x) * k.rho;
  const float step = alpha / fmaxf(1.0f, rms_u * k.inv_clip);
  const F4 fc = column_factors(t, inv_c);
  const float* gbase = g + t.first;
  float* wbase = w + t.first;
  const float* rows = inv_r + t.v.row_off + t.row0;
  const int upto = BF16 ? t.in_block : t.live;      // padded rows only matter for the bfloat16 copy
  for (int rr0 = 0; rr0 < upto; rr0 += kRowBatch) {
    F4 gv[kRowBatch], wv[kRowBatch];
#pragma unroll
    for (int j = 0; j < kRowBatch; ++j) {
      if (rr0 + j < upto && t.col_ok) {
        const int64_t o = (int64_t)(rr0 + j) * t.v.cols;
        gv[j] = F4{0.0f, 0.0f, 0.0f, 0.0f};
        wv[j] = F4{0.0f, 0.0f, 0.0f, 0.0f};
        if (t.vec) {
          wv[j] = ld4<PolAf::RW>(wbase + o);
          if (rr0 + j < t.live) gv[j] = ld4<PolAf::RO>(gbase + o);
        } else {
          wv[j].x = ld<PolAf::RW>(wbase + o);
          if (rr0 + j < t.live) gv[j].x = ld<PolAf::RO>(gbase + o);
        }
      }
    }
#pragma unroll
    for (int j = 0; j < kRowBatch; ++j) {
      if (rr0 + j < upto && t.col_ok) {
        const int64_t o = (int64_t)(rr0 + j) * t.v.cols;
        if (rr0 + j < t.live) {
          const float s = step * rows[rr0 + j];
          wv[j].x = fmaf(-(s * fc.x), gv[j].x, wv[j].x);
          wv[j].y = fmaf(-(s * fc.y), gv[j].y, wv[j].y);
          wv[j].z = fmaf(-(s * fc.z), gv[j].z, wv[j].z);
          wv[j].w = fmaf(-(s * fc.w), gv[j].w, wv[j].w);
          if (t.vec) st4<PolAf::ST>(wbase + o, wv[j]);
          else st<PolAf::ST>(wbase + o, wv[j].x);
        }
        if constexpr (BF16) {
          if (t.vec) store_bf16x4<PolAf::ST>(w16 + t.first + o, wv[j]);
          else w16[t.first + o] = (uint16_t)bf16_of(wv[j].x);
        }
      }
    }
  }
  if constexpr (BF16) {
    // the alignment tail of the piece, once per variable
    if (it.rb == t.v.n_rb - 1 && it.ct == t.v.n_ct - 1) {
      const int64_t used = t.v.Lr * t.v.cols;
      for (int64_t q = used + threadIdx.x; q < t.v.L; q += kBlock) w16[t.v.off + q] = (uint16_t)bf16_of(w[t.v.off + q]);
    }
  }
}

}  // namespace

// ---- launchers ----------------------------------------------------------------------------------------

hipError_t launch_rowcol_sumsq(shard_plan_t* p, int r, const float* x, float* row_out, float* col_out,
                               hipStream_t stream) {
  if (p->V == 0) return hipSuccess;
  const RowColVar* vars = ws_at<RowColVar>(p, p->ws.rc_vars);
  float* colpart = ws_at<float>(p, p->ws.rc_colpart);
  float* rowpart = ws_at<float>(p, p->ws.rc_rowpart);
  if (!p->rc_items.empty()) {
    ProfScope ps(p, SHARD_K_ROWCOL_P1, stream);
    hipLaunchKernelGGL((rowcol_p1_kernel<false>), dim3((unsigned)p->rc_items.size()), dim3(kBlock), 0, stream, vars,
                       ws_at<RowColItem>(p, p->ws.rc_items), x, x, colpart, rowpart, (float*)nullptr, r);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  ProfScope ps(p, SHARD_K_ROWCOL_P2, stream);
  hipLaunchKernelGGL(rowcol_p2_kernel, dim3((unsigned)p->V, 16), dim3(kBlock), 0, stream, vars, colpart, rowpart,
                     row_out, col_out, (const float*)nullptr, (const float*)nullptr, (const float*)nullptr,
                     (const float*)nullptr, (float*)nullptr, r);
  return hipGetLastError();
}

hipError_t launch_adafactor_partials(shard_plan_t* p, int r, const float* w, const float* g, const float* R,
                                     const float* other_col, const float* other_table, float* row_sq, float* col_sq,
                                     float* table, hipStream_t stream) {
  if (p->V == 0) return hipSuccess;
  const RowColVar* vars = ws_at<RowColVar>(p, p->ws.rc_vars);
  float* colpart = ws_at<float>(p, p->ws.rc_colpart);
  float* rowpart = ws_at<float>(p, p->ws.rc_rowpart);
  float* wpart = ws_at<float>(p, p->ws.af_wpart);
  if (!p->rc_items.empty()) {
    ProfScope ps(p, SHARD_K_ROWCOL_P1, stream);
    hipLaunchKernelGGL((rowcol_p1_kernel<true>), dim3((unsigned)p->rc_items.size()), dim3(kBlock), 0, stream, vars,
                       ws_at<RowColItem>(p, p->ws.rc_items), g, w, colpart, rowpart, wpart, r);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  ProfScope ps(p, SHARD_K_ROWCOL_P2, stream);
  hipLaunchKernelGGL(rowcol_p2_kernel, dim3((unsigned)p->V, 16), dim3(kBlock), 0, stream, vars, colpart, rowpart, row_sq,
                     col_sq, other_col, (const float*)wpart, R, other_table, table, r);
  return hipGetLastError();
}

hipError_t launch_adafactor_moments(shard_plan_t* p, int r, const float* g, float* R, float* C, const float* row_sq,
                                    const float* col_sq_global, const float* table_global, const AdafactorK& k,
                                    const float* other_usq, float* usq_local, float* usq_total, hipStream_t stream) {
  if (p->V == 0) return hipSuccess;
  const RowColVar* vars = ws_at<RowColVar>(p, p->ws.rc_vars);
  float* sum_r = ws_at<float>(p, p->ws.af_sumr);
  float* inv_r = ws_at<float>(p, p->ws.af_inv_r);
  float* inv_c = ws_at<float>(p, p->ws.af_inv_c);
  float* upart = ws_at<float>(p, p->ws.af_upart);
  {
    ProfScope ps(p, SHARD_K_ADAFACTOR_STATE, stream);
    hipLaunchKernelGGL(adafactor_sumr_kernel, dim3((unsigned)p->V), dim3(kBlock), 0, stream, vars, col_sq_global,
                       table_global, sum_r, k);
    hipLaunchKernelGGL(adafactor_state_kernel, dim3((unsigned)p->V, 16), dim3(kBlock), 0, stream, vars, row_sq,
                       col_sq_global, (const float*)sum_r, R, C, inv_r, inv_c, r, k);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (!p->rc_items.empty()) {
    ProfScope ps(p, SHARD_K_ADAFACTOR_USQ, stream);
    hipLaunchKernelGGL(adafactor_usq_kernel, dim3((unsigned)p->rc_items.size()), dim3(kBlock), 0, stream, vars,
                       ws_at<RowColItem>(p, p->ws.rc_items), g, (const float*)inv_r, (const float*)inv_c, upart, r);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  ProfScope ps(p, SHARD_K_ADAFACTOR_STATE, stream);
  hipLaunchKernelGGL(item_total_kernel, dim3((unsigned)p->V), dim3(kBlock), 0, stream, vars, (const float*)upart, other_usq,
                     usq_local, usq_total);
  return hipGetLastError();
}

hipError_t launch_adafactor_apply(shard_plan_t* p, int r, float* w, const float* g, const float* table_global,
                                  const float* usq_global, void* w16, const AdafactorK& k, hipStream_t stream) {
  if (p->rc_items.empty()) return hipSuccess;
  ProfScope ps(p, SHARD_K_ADAFACTOR_APPLY, stream);
  const RowColVar* vars = ws_at<RowColVar>(p, p->ws.rc_vars);
  const RowColItem* items = ws_at<RowColItem>(p, p->ws.rc_items);
  const float* inv_r = ws_at<float>(p, p->ws.af_inv_r);
  const float* inv_c = ws_at<float>(p, p->ws.af_inv_c);
  const dim3 grid((unsigned)p->rc_items.size());
  if (w16)
    hipLaunchKernelGGL((adafactor_apply_kernel<true>), grid, dim3(kBlock), 0, stream, vars, items, w, g, inv_r, inv_c,
                       table_global, usq_global, (uint16_t*)w16, r, k);
  else
    hipLaunchKernelGGL((adafactor_apply_kernel<false>), grid, dim3(kBlock), 0, stream, vars, items, w, g, inv_r, inv_c,
                       table_global, usq_global, (uint16_t*)nullptr, r, k);
  return hipGetLastError();
}

}  // namespace su
