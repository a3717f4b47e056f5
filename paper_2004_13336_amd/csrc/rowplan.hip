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
// Work items of the streaming kernels are (variable, row block, column tile) triples from the plan.
// Every thread owns 4 adjacent columns (1 where rows do not start on 16-byte boundaries) of 8 rows and
// issues its 8 independent 128-bit loads at once; a workgroup's four wavefronts are stacked along the
// rows (32 rows x 256 columns) or, for pieces of at most 8 rows, laid side by side (8 rows x 1024
// columns).  The small per-column and per-row kernels run over item tables of their own, so that a
// matrix with millions of columns and two rows spreads over the chip like one with the opposite shape.
// All sums are taken in an order fixed by the plan: results are run-to-run identical.
#include "device_common.hpp"

// Cache policies, measured on MI355X.  A tensor that is reduced once and not needed again is loaded
// non-temporally; Adafactor's gradient is read by three kernels in a row and stays cacheable (one
// replica's piece fits the 256 MB memory-side cache), its weights are loaded non-temporally and stored
// non-temporally by the last kernel.

namespace su {
namespace {

constexpr int kWaves = kBlock / 64;
constexpr int kRowsPerWave = kRowBlock / kWaves;     // 8 rows per wavefront: one batch of independent loads
constexpr bool kRowColNt = true;   // non-temporal loads in shard_reduce_sq_rows_cols
typedef Policy<3> PolAf;           // mask of the Adafactor kernels (4: g loads, 2: w loads, 1: stores)

// This thread's part of a tile item.  Tall tile: wavefront w takes rows 8w .. 8w+7, lane l the columns
// 4l .. 4l+3 (or the single column l).  Flat tile: all wavefronts take the same 8 rows, wavefront w the
// w-th span of columns.
struct Tile {
  RowColVar v;
  int64_t col0;      // first column this thread owns
  int64_t wrow0;     // first row of this wavefront inside the replica's piece
  int64_t first;     // offset, in the packed shard, of (wrow0, col0)
  int rows_here;     // rows of the piece among this wavefront's 8
  int live_here;     // leading ones of those that exist in the full matrix (position = replica offset
                     // + index, compared with the full row count)
  int var, rb, ct;
  bool vec, flat, col_ok;
};

__device__ __forceinline__ int64_t real_rows_of(const RowColVar& v, int r) {
  const int64_t left = v.rows - (int64_t)r * v.Lr;
  return left < 0 ? 0 : (left > v.Lr ? v.Lr : left);
}

__device__ __forceinline__ int clamp8(int64_t x) { return (int)(x < 0 ? 0 : (x > kRowsPerWave ? kRowsPerWave : x)); }

__device__ __forceinline__ Tile tile_of(const RowColVar* __restrict__ vars, const RowColItem* __restrict__ items, int r) {
  Tile t;
  const RowColItem it = items[blockIdx.x];
  t.var = it.var;
  t.rb = it.rb;
  t.ct = it.ct;
  t.v = vars[it.var];
  t.vec = (t.v.shape & kRcVec) != 0;
  t.flat = (t.v.shape & kRcFlat) != 0;
  const int w = t.vec ? 4 : 1;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  if (t.flat) {
    t.col0 = ((int64_t)it.ct * kWaves + wave) * (64 * w) + (int64_t)lane * w;
    t.wrow0 = (int64_t)it.rb * kRowsPerWave;
  } else {
    t.col0 = (int64_t)it.ct * (64 * w) + (int64_t)lane * w;
    t.wrow0 = (int64_t)it.rb * kRowBlock + (int64_t)wave * kRowsPerWave;
  }
  t.rows_here = clamp8(t.v.Lr - t.wrow0);
  const int live = clamp8(real_rows_of(t.v, r) - t.wrow0);
  t.live_here = live < t.rows_here ? live : t.rows_here;
  t.col_ok = t.col0 < t.v.cols;
  t.first = t.v.off + t.wrow0 * t.v.cols + t.col0;
  return t;
}

__device__ __forceinline__ float wave_sum(float a) {
#pragma unroll
  for (int s = 32; s >= 1; s >>= 1) a += __shfl_xor(a, s, 64);
  return a;
}

// Sum over the workgroup, fixed order, valid in thread 0.
__device__ __forceinline__ float block_sum1(float a) {
  __shared__ float part[kWaves];
  a = wave_sum(a);
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = a;
  __syncthreads();
  if (threadIdx.x == 0) {
    a = part[0];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) a += part[w];
  }
  return a;
}

// Sum over the workgroup of float64 values, fixed order, valid in thread 0.
__device__ __forceinline__ double block_sum_f64(double a) {
  __shared__ double part[kWaves];
#pragma unroll
  for (int s = 32; s >= 1; s >>= 1) a += __shfl_xor(a, s, 64);
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = a;
  __syncthreads();
  if (threadIdx.x == 0) {
    a = part[0];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) a += part[w];
  }
  return a;
}

// ---- row / column sums of squares -------------------------------------------------------------------
// One pass over x.  Per tile: every thread loads its 8 rows x 4 columns at once; the tile's column
// sums (over its live rows) and row sums (over the tile's columns) are formed with shuffles across the
// 64 lanes and combined across the four wavefronts in LDS along whichever direction the wavefronts
// share; both go to the workspace as partial results that rowcol_p2_kernel adds.  WITH_W: the same pass also reads a second tensor y at the same positions and
// leaves the tile's sum of y^2 over real elements in ypart (Adafactor's RMS of the weights).
template <bool WITH_W>
__global__ __launch_bounds__(kBlock) void rowcol_p1_kernel(const RowColVar* __restrict__ vars,
                                                           const RowColItem* __restrict__ items,
                                                           const float* __restrict__ x, const float* __restrict__ y,
                                                           float* __restrict__ colpart, float* __restrict__ rowpart,
                                                           float* __restrict__ ypart, int r) {
  __shared__ float col_lds[kWaves][64][4];
  const Tile t = tile_of(vars, items, r);
  const float* base = x + t.first;
  const float* ybase = y + t.first;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  F4 val[kRowsPerWave], wv[kRowsPerWave];
#pragma unroll
  for (int j = 0; j < kRowsPerWave; ++j) {
    val[j] = F4{0.0f, 0.0f, 0.0f, 0.0f};
    if constexpr (WITH_W) wv[j] = F4{0.0f, 0.0f, 0.0f, 0.0f};
    if (j < t.live_here && t.col_ok) {
      const int64_t o = (int64_t)j * t.v.cols;
      if (t.vec) {
        val[j] = ld4<kRowColNt && !WITH_W>(base + o);
        if constexpr (WITH_W) wv[j] = ld4<false>(ybase + o);
      } else {
        val[j].x = ld<kRowColNt && !WITH_W>(base + o);
        if constexpr (WITH_W) wv[j].x = ybase[o];
      }
    }
  }
  float c0 = 0.0f, c1 = 0.0f, c2 = 0.0f, c3 = 0.0f, sy = 0.0f;
  float rs[kRowsPerWave];
#pragma unroll
  for (int j = 0; j < kRowsPerWave; ++j) {
    const float a = val[j].x * val[j].x, b = val[j].y * val[j].y, c = val[j].z * val[j].z, d = val[j].w * val[j].w;
    c0 += a; c1 += b; c2 += c; c3 += d;
    rs[j] = (a + b) + (c + d);
    if constexpr (WITH_W) sy += (wv[j].x * wv[j].x + wv[j].y * wv[j].y) + (wv[j].z * wv[j].z + wv[j].w * wv[j].w);
  }
  __shared__ float row_lds[kWaves][kRowsPerWave];
  float* cp = colpart + t.v.cp_off + (int64_t)t.rb * t.v.cols + t.col0;
  float* rp = rowpart + t.v.rp_off + (int64_t)t.ct * t.v.Lr + t.wrow0;
  if (t.flat) {
    // the wavefronts hold different columns of the same rows: column sums are final, row sums are
    // combined across the wavefronts
    if (t.col_ok) {
      if (t.vec) st4<false>(cp, F4{c0, c1, c2, c3});
      else cp[0] = c0;
    }
#pragma unroll
    for (int j = 0; j < kRowsPerWave; ++j) {
      const float s = wave_sum(rs[j]);
      if (lane == 0) row_lds[wave][j] = s;
    }
    __syncthreads();
    if ((int)threadIdx.x < t.rows_here)                 // rows_here is clamped to [0, 8]
      rp[threadIdx.x] = (row_lds[0][threadIdx.x] + row_lds[1][threadIdx.x]) + (row_lds[2][threadIdx.x] + row_lds[3][threadIdx.x]);
  } else {
    // the wavefronts hold different rows of the same columns: row sums are final, column sums are
    // combined across the wavefronts
    col_lds[wave][lane][0] = c0; col_lds[wave][lane][1] = c1; col_lds[wave][lane][2] = c2; col_lds[wave][lane][3] = c3;
#pragma unroll
    for (int j = 0; j < kRowsPerWave; ++j) {
      const float s = wave_sum(rs[j]);
      if (lane == 0 && j < t.rows_here) rp[j] = s;
    }
    __syncthreads();
    if (wave == 0 && t.col_ok) {
      F4 tot;
      tot.x = (col_lds[0][lane][0] + col_lds[1][lane][0]) + (col_lds[2][lane][0] + col_lds[3][lane][0]);
      tot.y = (col_lds[0][lane][1] + col_lds[1][lane][1]) + (col_lds[2][lane][1] + col_lds[3][lane][1]);
      tot.z = (col_lds[0][lane][2] + col_lds[1][lane][2]) + (col_lds[2][lane][2] + col_lds[3][lane][2]);
      tot.w = (col_lds[0][lane][3] + col_lds[1][lane][3]) + (col_lds[2][lane][3] + col_lds[3][lane][3]);
      if (t.vec) st4<false>(cp, tot);
      else cp[0] = tot.x;
    }
  }
  if constexpr (WITH_W) {
    sy = block_sum1(sy);
    if (threadIdx.x == 0) ypart[blockIdx.x] = sy;
  }
}

// The small kernels below are all latency: a loop that loads, waits and adds once per iteration pays a trip to
// memory for every element.  Both helpers issue kInFlight independent, unconditional loads per batch (in a last,
// partial batch the indices past the end are redirected to the batch's first element and only the additions are
// predicated: a conditional load makes the compiler wait for each one) and then add them in index order, so the
// order of the additions, and with it every result, is that of the plain loop.
constexpr int kInFlight = 8;

// p[first * stride] + p[(first + step) * stride] + ... over the indices below n, added in exactly that order.
__device__ __forceinline__ float ordered_sum(const float* __restrict__ p, int64_t stride, int first, int step, int n) {
  float s = 0.0f;
  for (int i = first; i < n; i += kInFlight * step) {
    float a[kInFlight];
#pragma unroll
    for (int j = 0; j < kInFlight; ++j) {
      const int ij = i + j * step;
      a[j] = p[(int64_t)(ij < n ? ij : i) * stride];
    }
#pragma unroll
    for (int j = 0; j < kInFlight; ++j)
      if (i + j * step < n) s += a[j];
  }
  return s;
}

// This thread's share of p[0 .. n): p[t] + p[t + kBlock] + ..., t = threadIdx.x, accumulated in float64 in that order.
__device__ __forceinline__ double thread_share_f64(const float* __restrict__ p, int64_t n) {
  double s = 0.0;
  for (int64_t k = threadIdx.x; k < n; k += (int64_t)kInFlight * kBlock) {
    float a[kInFlight];
#pragma unroll
    for (int j = 0; j < kInFlight; ++j) {
      const int64_t kj = k + (int64_t)j * kBlock;
      a[j] = p[kj < n ? kj : k];
    }
#pragma unroll
    for (int j = 0; j < kInFlight; ++j)
      if (k + (int64_t)j * kBlock < n) s += (double)a[j];
  }
  return s;
}

// Adds the partial results of phase 1 in a fixed order.  The grid holds, in this order,
//   one workgroup per column item: 64 columns whose row blocks the four wavefronts share (results
//     combined in LDS), or 256 columns with a thread each where row blocks are few; other_col
//     (nullable, laid out like col_out) is added; with colitem_part the item's sum over its columns
//     is kept too (for sum(R) of Adafactor);
//   one workgroup per row item: 256 rows with a thread each, or one row of a variable with very many
//     column tiles, added by the whole workgroup;
//   with table_out, one workgroup per variable:
//     table_out[2i]   = sum of ypart over the variable's tiles        (+ other_table)
//     table_out[2i+1] = sum of row_state over the replica's real rows (+ other_table)
__global__ __launch_bounds__(kBlock) void rowcol_p2_kernel(const RowColVar* __restrict__ vars,
                                                           const ColItem* __restrict__ col_items,
                                                           const RowItem* __restrict__ row_items, int n_col_items,
                                                           int n_row_items, const float* __restrict__ colpart,
                                                           const float* __restrict__ rowpart,
                                                           float* __restrict__ row_out, float* __restrict__ col_out,
                                                           const float* __restrict__ other_col,
                                                           float* __restrict__ colitem_part,
                                                           const float* __restrict__ ypart,
                                                           const float* __restrict__ row_state,
                                                           const float* __restrict__ other_table,
                                                           float* __restrict__ table_out, int r) {
  __shared__ float lds[kWaves][64];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  int b = blockIdx.x;
  if (b < n_col_items) {
    const ColItem it = col_items[b];
    const RowColVar v = vars[it.var];
    if (col_span(v.n_rb) == 64) {
      // many row blocks: 64 columns, wavefront w adds the row blocks w, w+4, ...
      const int64_t c = (int64_t)it.tile * 64 + lane;
      const bool ok = c < v.cols;
      float s = 0.0f;
      if (ok)
        s = ordered_sum(colpart + v.cp_off + c, v.cols, wave, kWaves, v.n_rb);
      lds[wave][lane] = s;
      __syncthreads();
      if (wave == 0) {
        float tot = (lds[0][lane] + lds[1][lane]) + (lds[2][lane] + lds[3][lane]);
        if (ok) {
          if (other_col) tot += other_col[v.col_off + c];
          col_out[v.col_off + c] = tot;
        } else {
          tot = 0.0f;
        }
        if (colitem_part) {
          tot = wave_sum(tot);
          if (lane == 0) colitem_part[b] = tot;
        }
      }
    } else {
      // few row blocks: 256 columns, a thread per column
      const int64_t c = (int64_t)it.tile * 256 + threadIdx.x;
      float tot = 0.0f;
      if (c < v.cols) {
        tot = ordered_sum(colpart + v.cp_off + c, v.cols, 0, 1, v.n_rb);
        if (other_col) tot += other_col[v.col_off + c];
        col_out[v.col_off + c] = tot;
      }
      if (colitem_part) {
        tot = block_sum1(tot);
        if (threadIdx.x == 0) colitem_part[b] = tot;
      }
    }
    return;
  }
  b -= n_col_items;
  if (b < n_row_items) {
    const RowItem it = row_items[b];
    const RowColVar v = vars[it.var];
    if (it.wide) {
      float s = 0.0f;
      s = ordered_sum(rowpart + v.rp_off + it.first_row, v.Lr, threadIdx.x, kBlock, v.n_ct);
      s = block_sum1(s);
      if (threadIdx.x == 0) row_out[v.row_off + it.first_row] = s;
    } else {
      const int64_t k = it.first_row + threadIdx.x;
      if (k < v.Lr) {
        float s = 0.0f;
        s = ordered_sum(rowpart + v.rp_off + k, v.Lr, 0, 1, v.n_ct);
        row_out[v.row_off + k] = s;
      }
    }
    return;
  }
  const int i = b - n_row_items;
  const RowColVar v = vars[i];
  const int64_t n_items = (int64_t)v.n_rb * v.n_ct;
  double ya = thread_share_f64(ypart + v.first_item, n_items);
  double ra = thread_share_f64(row_state + v.row_off, real_rows_of(v, r));
  ya = block_sum_f64(ya);
  __syncthreads();
  ra = block_sum_f64(ra);
  if (threadIdx.x == 0) {
    const float fa = (float)ya, fb = (float)ra;
    table_out[2 * i] = other_table ? fa + other_table[2 * i] : fa;
    table_out[2 * i + 1] = other_table ? fb + other_table[2 * i + 1] : fb;
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

// One workgroup per column item: the item's sum of the all-reduced column sums (when phase 1 ran
// elsewhere and rowcol_p2_kernel could not leave it).
__global__ __launch_bounds__(kBlock) void adafactor_colsum_kernel(const RowColVar* __restrict__ vars,
                                                                  const ColItem* __restrict__ col_items,
                                                                  const float* __restrict__ col_sq_global,
                                                                  float* __restrict__ colitem_part) {
  const ColItem it = col_items[blockIdx.x];
  const RowColVar v = vars[it.var];
  const int span = col_span(v.n_rb);
  const int64_t c = (int64_t)it.tile * span + threadIdx.x;
  float s = ((int)threadIdx.x < span && c < v.cols) ? col_sq_global[v.col_off + c] : 0.0f;
  s = block_sum1(s);
  if (threadIdx.x == 0) colitem_part[blockIdx.x] = s;
}

// Column items, then row items: new state, and the two factors of 1/sqrt(Vhat):
// inv_r[k] = rsqrt(R_k) (0 for padded rows), inv_c[j] = rsqrt(C_j / sum(R)).
// sum(R) over all replicas' rows = beta2 * (all-reduced sum of the old R) + (1-beta2) * (sum of the all-reduced
// column sums + rows cols eps1); every column item adds its variable's few hundred item sums anew, in one fixed
// order with float64 accumulators (cheaper than a launch of its own for one number per variable).
__global__ __launch_bounds__(kBlock) void adafactor_state_kernel(const RowColVar* __restrict__ vars,
                                                                 const ColItem* __restrict__ col_items,
                                                                 const RowItem* __restrict__ row_items, int n_col_items,
                                                                 const float* __restrict__ row_sq,
                                                                 const float* __restrict__ col_sq_global,
                                                                 const float* __restrict__ colitem_part,
                                                                 const float* __restrict__ table_global, float* R, float* C,
                                                                 float* __restrict__ inv_r, float* __restrict__ inv_c,
                                                                 int r, AdafactorK k) {
  int b = blockIdx.x;
  if (b < n_col_items) {
    const ColItem it = col_items[b];
    const RowColVar v = vars[it.var];
    __shared__ float sum_r;
    double s = block_sum_f64(thread_share_f64(colitem_part + v.first_col_item, v.n_col_items));
    if (threadIdx.x == 0) {
      const double n = (double)v.rows * (double)v.cols;
      sum_r = (float)((double)k.beta2 * (double)table_global[2 * it.var + 1] + (double)k.omb2 * (s + n * (double)k.eps1));
    }
    __syncthreads();
    const int span = col_span(v.n_rb);
    const int64_t c = (int64_t)it.tile * span + threadIdx.x;
    if ((int)threadIdx.x >= span || c >= v.cols || v.rows == 0) return;    // no rows: the state stays as it is
    if (v.cols == 1) {
      inv_c[v.col_off] = 1.0f;                     // vector: Vhat = R, no column state
      return;
    }
    const float col_eps = (float)v.rows * k.eps1;
    const float cn = fmaf(k.beta2, C[v.col_off + c], k.omb2 * (col_sq_global[v.col_off + c] + col_eps));
    C[v.col_off + c] = cn;
    inv_c[v.col_off + c] = 1.0f / sqrtf(cn / sum_r);
    return;
  }
  const RowItem it = row_items[b - n_col_items];
  const RowColVar v = vars[it.var];
  const int64_t q = it.first_row + (it.wide ? 0 : (int64_t)threadIdx.x);
  if ((it.wide && threadIdx.x != 0) || q >= v.Lr) return;
  float rn = 0.0f, inv = 0.0f;
  if (q < real_rows_of(v, r)) {
    const float row_eps = (float)v.cols * k.eps1;
    rn = fmaf(k.beta2, R[v.row_off + q], k.omb2 * (row_sq[v.row_off + q] + row_eps));
    inv = 1.0f / sqrtf(rn);
  }
  R[v.row_off + q] = rn;
  inv_r[v.row_off + q] = inv;
}

// The 4 (or 1) column factors of this thread.  Column offsets of different variables are not
// multiples of 4, so these are scalar loads; they are cached and read once per tile.
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

// Per tile: sum of U^2 over real elements, U = g * inv_r[row] * inv_c[col].
__global__ __launch_bounds__(kBlock) void adafactor_usq_kernel(const RowColVar* __restrict__ vars,
                                                               const RowColItem* __restrict__ items,
                                                               const float* __restrict__ g,
                                                               const float* __restrict__ inv_r,
                                                               const float* __restrict__ inv_c,
                                                               float* __restrict__ upart, int r) {
  const Tile t = tile_of(vars, items, r);
  const F4 fc = column_factors(t, inv_c);
  const float* base = g + t.first;
  const float* rows = inv_r + t.v.row_off + t.wrow0;
  F4 val[kRowsPerWave];
  float fr[kRowsPerWave];
#pragma unroll
  for (int j = 0; j < kRowsPerWave; ++j) {
    val[j] = F4{0.0f, 0.0f, 0.0f, 0.0f};
    fr[j] = 0.0f;
    if (j < t.live_here && t.col_ok) {
      const int64_t o = (int64_t)j * t.v.cols;
      if (t.vec) val[j] = ld4<PolAf::RO>(base + o);
      else val[j].x = ld<PolAf::RO>(base + o);
      fr[j] = rows[j];
    }
  }
  float s = 0.0f;
#pragma unroll
  for (int j = 0; j < kRowsPerWave; ++j) {
    const float a = (val[j].x * fr[j]) * fc.x, b = (val[j].y * fr[j]) * fc.y, c = (val[j].z * fr[j]) * fc.z,
                d = (val[j].w * fr[j]) * fc.w;
    s += (a * a + b * b) + (c * c + d * d);
  }
  s = block_sum1(s);
  if (threadIdx.x == 0) upart[blockIdx.x] = s;
}

// One workgroup per variable: adds the variable's tile partials in a fixed order.
__global__ __launch_bounds__(kBlock) void item_total_kernel(const RowColVar* __restrict__ vars,
                                                            const float* __restrict__ part,
                                                            const float* __restrict__ other, float* __restrict__ local_out,
                                                            float* __restrict__ total_out) {
  const int i = blockIdx.x;
  const RowColVar v = vars[i];
  const int64_t n_items = (int64_t)v.n_rb * v.n_ct;
  double a = block_sum_f64(thread_share_f64(part + v.first_item, n_items));
  if (threadIdx.x == 0) {
    const float fa = (float)a;
    if (local_out) local_out[i] = fa;
    if (total_out) total_out[i] = other ? fa + other[i] : fa;
  }
}

// Per tile: X -= alpha * U / max(1, RMS(U) / d) on real elements; padded rows and the alignment tail
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
  const float n = (float)t.v.rows * (float)t.v.cols;
  const float rms_x = sqrtf(table_global[2 * t.var] / n), rms_u = sqrtf(usq_global[t.var] / n);
  const float alpha = fmaxf(k.eps2, rms_x) * k.rho;
  const float step = alpha / fmaxf(1.0f, rms_u * k.inv_clip);
  const F4 fc = column_factors(t, inv_c);
  const float* gbase = g + t.first;
  float* wbase = w + t.first;
  const float* rows = inv_r + t.v.row_off + t.wrow0;
  const int upto = BF16 ? t.rows_here : t.live_here;      // padded rows only matter for the bfloat16 copy
  F4 gv[kRowsPerWave], wv[kRowsPerWave];
  float fr[kRowsPerWave];
#pragma unroll
  for (int j = 0; j < kRowsPerWave; ++j) {
    gv[j] = F4{0.0f, 0.0f, 0.0f, 0.0f};
    wv[j] = F4{0.0f, 0.0f, 0.0f, 0.0f};
    fr[j] = 0.0f;
    if (j < upto && t.col_ok) {
      const int64_t o = (int64_t)j * t.v.cols;
      if (t.vec) wv[j] = ld4<PolAf::RW>(wbase + o);
      else wv[j].x = ld<PolAf::RW>(wbase + o);
      if (j < t.live_here) {
        if (t.vec) gv[j] = ld4<PolAf::RO>(gbase + o);
        else gv[j].x = ld<PolAf::RO>(gbase + o);
        fr[j] = rows[j];
      }
    }
  }
#pragma unroll
  for (int j = 0; j < kRowsPerWave; ++j) {
    if (j < upto && t.col_ok) {
      const int64_t o = (int64_t)j * t.v.cols;
      if (j < t.live_here) {
        const float s = step * fr[j];
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
  if constexpr (BF16) {
    // the alignment tail of the piece, once per variable
    if (t.rb == t.v.n_rb - 1 && t.ct == t.v.n_ct - 1) {
      const int64_t used = t.v.Lr * t.v.cols;
      for (int64_t q = used + threadIdx.x; q < t.v.L; q += kBlock) w16[t.v.off + q] = (uint16_t)bf16_of(w[t.v.off + q]);
    }
  }
}

}  // namespace

// ---- launchers ----------------------------------------------------------------------------------------

namespace {
// Phase-1 pair: tiles, then the additions.  table may be null (plain row/column sums).
hipError_t launch_reduce_pair(shard_plan_t* p, int r, const float* x, const float* y, const float* row_state,
                              const float* other_col, const float* other_table, float* row_out, float* col_out,
                              float* colitem_part, float* table, hipStream_t stream) {
  const RowColVar* vars = ws_at<RowColVar>(p, p->ws.rc_vars);
  float* colpart = ws_at<float>(p, p->ws.rc_colpart);
  float* rowpart = ws_at<float>(p, p->ws.rc_rowpart);
  float* ypart = ws_at<float>(p, p->ws.af_wpart);
  if (!p->rc_items.empty()) {
    ProfScope ps(p, SHARD_K_ROWCOL_P1, stream);
    const dim3 grid((unsigned)p->rc_items.size());
    if (y)
      hipLaunchKernelGGL((rowcol_p1_kernel<true>), grid, dim3(kBlock), 0, stream, vars,
                         ws_at<RowColItem>(p, p->ws.rc_items), x, y, colpart, rowpart, ypart, r);
    else
      hipLaunchKernelGGL((rowcol_p1_kernel<false>), grid, dim3(kBlock), 0, stream, vars,
                         ws_at<RowColItem>(p, p->ws.rc_items), x, x, colpart, rowpart, (float*)nullptr, r);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  const int n_col = (int)p->rc_col_items.size(), n_row = (int)p->rc_row_items.size();
  const int64_t blocks = (int64_t)n_col + n_row + (table ? p->V : 0);
  if (blocks == 0) return hipSuccess;
  ProfScope ps(p, SHARD_K_ROWCOL_P2, stream);
  hipLaunchKernelGGL(rowcol_p2_kernel, dim3((unsigned)blocks), dim3(kBlock), 0, stream, vars,
                     ws_at<ColItem>(p, p->ws.rc_col_items), ws_at<RowItem>(p, p->ws.rc_row_items), n_col, n_row,
                     (const float*)colpart, (const float*)rowpart, row_out, col_out, other_col, colitem_part,
                     (const float*)ypart, row_state, other_table, table, r);
  return hipGetLastError();
}
}  // namespace

hipError_t launch_rowcol_sumsq(shard_plan_t* p, int r, const float* x, float* row_out, float* col_out,
                               hipStream_t stream) {
  if (p->V == 0) return hipSuccess;
  return launch_reduce_pair(p, r, x, nullptr, nullptr, nullptr, nullptr, row_out, col_out, nullptr, nullptr, stream);
}

hipError_t launch_adafactor_partials(shard_plan_t* p, int r, const float* w, const float* g, const float* R,
                                     const float* other_col, const float* other_table, float* row_sq, float* col_sq,
                                     float* table, bool keep_column_item_sums, hipStream_t stream) {
  if (p->V == 0) return hipSuccess;
  float* colitem_part = keep_column_item_sums ? ws_at<float>(p, p->ws.rc_colitem_part) : nullptr;
  return launch_reduce_pair(p, r, g, w, R, other_col, other_table, row_sq, col_sq, colitem_part, table, stream);
}

hipError_t launch_adafactor_moments(shard_plan_t* p, int r, const float* g, float* R, float* C, const float* row_sq,
                                    const float* col_sq_global, const float* table_global, const AdafactorK& k,
                                    bool have_column_item_sums, const float* other_usq, float* usq_local,
                                    float* usq_total, hipStream_t stream) {
  if (p->V == 0) return hipSuccess;
  const RowColVar* vars = ws_at<RowColVar>(p, p->ws.rc_vars);
  const ColItem* col_items = ws_at<ColItem>(p, p->ws.rc_col_items);
  const RowItem* row_items = ws_at<RowItem>(p, p->ws.rc_row_items);
  const int n_col = (int)p->rc_col_items.size(), n_row = (int)p->rc_row_items.size();
  float* colitem_part = ws_at<float>(p, p->ws.rc_colitem_part);
  float* inv_r = ws_at<float>(p, p->ws.af_inv_r);
  float* inv_c = ws_at<float>(p, p->ws.af_inv_c);
  float* upart = ws_at<float>(p, p->ws.af_upart);
  {
    ProfScope ps(p, SHARD_K_ADAFACTOR_STATE, stream);
    if (!have_column_item_sums && n_col > 0)
      hipLaunchKernelGGL(adafactor_colsum_kernel, dim3((unsigned)n_col), dim3(kBlock), 0, stream, vars, col_items,
                         col_sq_global, colitem_part);
    if (n_col + n_row > 0)
      hipLaunchKernelGGL(adafactor_state_kernel, dim3((unsigned)(n_col + n_row)), dim3(kBlock), 0, stream, vars,
                         col_items, row_items, n_col, row_sq, col_sq_global, (const float*)colitem_part, table_global, R, C, inv_r,
                         inv_c, r,
                         k);
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
  ProfScope ps(p, SHARD_K_ITEM_TOTAL, stream);
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
