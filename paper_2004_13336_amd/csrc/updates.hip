// Optimizer kernels for gfx950 (MI355X) and their launchers: Adam, momentum, LAMB, LARS on a packed shard.
//
// Everything here is bound by HBM bandwidth (Section 2.2: the weight update reads the gradient,
// the weight and the auxiliary variables and writes the weight and the auxiliaries back; the
// arithmetic in between is a handful of element-wise operations).  The kernels therefore do
// nothing clever with the arithmetic and everything they can for the memory system:
//   * every lane moves 128 bits per access, a 64-lane wavefront covers 1 KiB of one stream;
//   * each thread issues all the loads of its tile before the first dependent instruction, so a
//     workgroup keeps tens of KiB in flight;
//   * one launch covers a whole shard: the element-wise updates run flat over [S], the ones with
//     per-variable reductions walk the chunk table;
//   * the per-variable sums of squares are reduced with wavefront shuffles and LDS, in a fixed
//     order, without atomics.
// The file is compiled with -ffp-contract=off: fused multiply-adds appear only where fmaf() is
// written, so every kernel (vector path, scalar path, sharded or not) performs bit-identical
// arithmetic per element.
#include <mutex>

#include "chunk_view.hpp"

namespace su {
namespace {

// Launch shapes and cache policies below are the measured best on MI355X; each note says what the alternative cost.
constexpr int kUpdBlock = 256;            // threads per workgroup of the table-driven update kernels (128 with one
                                          // or two accesses per thread and stream measured within 2 % at every size)
constexpr int kUnroll = 2;         // table-driven kernels: 128-bit accesses per thread per stream in flight; 2 makes a tile
                                   // the default 2048-slot chunk, so that whole chunks run the branch-free path (4: phase 1 +5 %)
constexpr int kAdamUnroll = 1;     // flat Adam kernel: the same (1: -2 to -5 % against 4 on shards of 12 M to 1.5 G slots)
constexpr int kMomentumUnroll = 2; // flat momentum kernel

// Cache policy per kernel family, as a 3-bit mask: 4 = non-temporal loads of streams that are only
// read, 2 = non-temporal loads of streams the same thread writes back in place, 1 = non-temporal stores.
typedef Policy<3> PolAdam;
typedef Policy<3> PolMomentum;
typedef Policy<6> PolLamb;
typedef Policy<7> PolLambLarge;    // phase 1 on large shards: every access non-temporal
typedef Policy<5> PolLambP2;       // phase 2 of LAMB: w is loaded through the caches and stored past them (measured on the
                                   // whole step: the unshard that follows gains as much as phase 2 itself)
typedef Policy<6> PolLars;
typedef Policy<5> PolLarsP2;       // phase 2 of LARS: as LAMB's (w and m loaded through the caches): 122 -> 116 us on 25.6 M slots


// Sum over the workgroup of two per-thread values, in a fixed order; the result is valid in
// thread 0.  Wavefront step: xor shuffles; cross-wavefront step: LDS.
__device__ __forceinline__ void block_sum2(float& a, float& b) {
  __shared__ float part[2 * (kUpdBlock / 64)];
#pragma unroll
  for (int s = 32; s >= 1; s >>= 1) {
    a += __shfl_xor(a, s, 64);
    b += __shfl_xor(b, s, 64);
  }
  const int wave = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) {
    part[2 * wave] = a;
    part[2 * wave + 1] = b;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    float x = part[0], y = part[1];
#pragma unroll
    for (int w = 1; w < kUpdBlock / 64; ++w) {
      x += part[2 * w];
      y += part[2 * w + 1];
    }
    a = x;
    b = y;
  }
}

// ---- where the gradient comes from -----------------------------------------------------------------
// GS 0: the packed shard gradient.  GS 1 / 2: straight from the full float32 / bfloat16 tensors (the
// *_full_grads entry points): the formatting of the gradient is fused into its consumer (Section 5.1)
// and no shard gradient is ever written.  Slots at or beyond the chunk's `valid` then read as +0.0,
// exactly what shard_format would have stored, so both routes give the same bits.
template <int GS>
struct GradChunk {
  static constexpr int SIZE = GS == 2 ? 2 : 4;     // bytes per gradient element
  const char* base;                                // the element that belongs to the chunk's first slot
  bool aligned;                                    // four elements from `base` can be one vector load
  __device__ __forceinline__ const void* tile(int first_slot) const { return base + (int64_t)first_slot * SIZE; }
  // every slot of a tile that exists (`lim`) is real and the source can be read with vector loads
  __device__ __forceinline__ bool fast(int lim, int valid) const { return GS == 0 || (aligned && valid >= lim); }
};

template <int GS>
__device__ __forceinline__ GradChunk<GS> grad_chunk(const float* g_shard, const void* const* __restrict__ g_full,
                                                    const ChunkView& cv) {
  GradChunk<GS> gc;
  if constexpr (GS == 0) {
    gc.base = (const char*)(g_shard + cv.shard0);
    gc.aligned = true;
  } else {
    // only dereferenced for slots below cv.valid, i.e. inside the tensor
    gc.base = (const char*)g_full[cv.var] + cv.flat0 * GradChunk<GS>::SIZE;
    gc.aligned = (reinterpret_cast<uintptr_t>(gc.base) & (4 * GradChunk<GS>::SIZE - 1)) == 0;
  }
  return gc;
}

__device__ __forceinline__ float bf16_up(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

// One gradient element of a chunk (the element-by-element paths).
template <int GS>
__device__ __forceinline__ float load_g1(const GradChunk<GS>& gc, int e, int valid) {
  if constexpr (GS == 0) return ((const float*)gc.base)[e];
  else if constexpr (GS == 1) return (e < valid) ? ((const float*)gc.base)[e] : 0.0f;
  else return (e < valid) ? bf16_up(((const uint16_t*)gc.base)[e]) : 0.0f;
}

// Four gradient values at offset o of a tile that starts at g.  NT0: cache policy of the shard gradient;
// full tensors are read once and always non-temporally.  GFAST: see GradChunk::fast.
template <int GS, bool GFAST, bool NT0>
__device__ __forceinline__ F4 load_g4(const void* g, int o, int valid) {
  if constexpr (GS == 0) {
    return ld4<NT0>((const float*)g + o);
  } else if constexpr (GS == 1) {
    const float* p = (const float*)g + o;
    if constexpr (GFAST) return ld4<true>(p);
    F4 x;
    x.x = (o + 0 < valid) ? ld<true>(p + 0) : 0.0f;
    x.y = (o + 1 < valid) ? ld<true>(p + 1) : 0.0f;
    x.z = (o + 2 < valid) ? ld<true>(p + 2) : 0.0f;
    x.w = (o + 3 < valid) ? ld<true>(p + 3) : 0.0f;
    return x;
  } else {
    const uint16_t* p = (const uint16_t*)g + o;
    if constexpr (GFAST) {
      const u2 t = ld<true>((const u2*)p);
      return F4{__uint_as_float(t.x << 16), __uint_as_float(t.x & 0xFFFF0000u), __uint_as_float(t.y << 16),
                __uint_as_float(t.y & 0xFFFF0000u)};
    }
    F4 x;
    x.x = (o + 0 < valid) ? bf16_up(ld<true>(p + 0)) : 0.0f;
    x.y = (o + 1 < valid) ? bf16_up(ld<true>(p + 1)) : 0.0f;
    x.z = (o + 2 < valid) ? bf16_up(ld<true>(p + 2)) : 0.0f;
    x.w = (o + 3 < valid) ? bf16_up(ld<true>(p + 3)) : 0.0f;
    return x;
  }
}

// ---- element-wise optimizer arithmetic ------------------------------------------------------------
// Reciprocal and square root use the hardware's 1-ulp approximations: the step they scale is at
// most lr in magnitude, so their error is orders of magnitude below the parity tolerance.

__device__ __forceinline__ void adam_elem(float& w, float g, float& m, float& v, const AdamK& k) {
  g = fmaf(k.wd, w, g);                                   // L2 decay folded into the gradient (wd may be 0)
  m = fmaf(k.b1, m, k.omb1 * g);
  v = fmaf(k.b2, v, (k.omb2 * g) * g);
  const float denom = __builtin_amdgcn_sqrtf(v * k.rbc2) + k.eps;
  const float upd = (m * k.rbc1) * __builtin_amdgcn_rcpf(denom);
  w = fmaf(-k.lr, upd, w);
}

__device__ __forceinline__ void momentum_elem(float& w, float g, float& m, const MomentumK& k) {
  g = fmaf(k.wd, w, g);
  m = fmaf(k.mu, m, g);
  w = fmaf(-k.lr, m, w);
}

__device__ __forceinline__ void lamb_moments(float g, float& m, float& v, const AdamK& k) {
  m = fmaf(k.b1, m, k.omb1 * g);
  v = fmaf(k.b2, v, (k.omb2 * g) * g);
}
// Update direction from the NEW moments and the OLD weight; both LAMB phases call this with the
// same inputs, so phase 2 re-creates phase 1's direction bit for bit instead of storing it.
__device__ __forceinline__ float lamb_dir(float w, float m, float v, float wd, const AdamK& k) {
  const float denom = __builtin_amdgcn_sqrtf(v * k.rbc2) + k.eps;
  return fmaf(wd, w, (m * k.rbc1) * __builtin_amdgcn_rcpf(denom));
}

// ---- flat kernels: Adam and momentum ---------------------------------------------------------------
// Padded slots are a fixed point of both updates (0 in, +0.0 out), so the packed shard is
// processed as one flat array: no table, no masks.

// One tile = kBlock * unroll 128-bit accesses per stream.  FULL tiles (all but possibly the last)
// run without a single branch: every load of the tile is issued before the first use.
// The two flat kernels come in two launch shapes (BLOCK threads per workgroup; see flat_shape below).
constexpr int kTileElems = kUpdBlock * kUnroll * 4;        // slots per tile of the table-driven kernels

template <int BLOCK, bool FULL, bool BF16>
__device__ __forceinline__ void adam_tile(float* w, const float* __restrict__ g, float* m, float* v,
                                          uint16_t* __restrict__ w16, int lim4, const AdamK& k) {
  // w, g, m, v, w16 point at the tile; lim4 = 128-bit units of the tile that exist (FULL: all)
  const int t4 = threadIdx.x * 4;
  F4 rw[kAdamUnroll], rg[kAdamUnroll], rm[kAdamUnroll], rv[kAdamUnroll];
#pragma unroll
  for (int i = 0; i < kAdamUnroll; ++i) {
    if (FULL || (int)threadIdx.x + i * BLOCK < lim4) {
      const int o = i * BLOCK * 4 + t4;
      rg[i] = ld4<PolAdam::RO>(g + o);
      rw[i] = ld4<PolAdam::RW>(w + o);
      rm[i] = ld4<PolAdam::RW>(m + o);
      rv[i] = ld4<PolAdam::RW>(v + o);
    }
  }
#pragma unroll
  for (int i = 0; i < kAdamUnroll; ++i) {
    if (FULL || (int)threadIdx.x + i * BLOCK < lim4) {
      const int o = i * BLOCK * 4 + t4;
      adam_elem(rw[i].x, rg[i].x, rm[i].x, rv[i].x, k);
      adam_elem(rw[i].y, rg[i].y, rm[i].y, rv[i].y, k);
      adam_elem(rw[i].z, rg[i].z, rm[i].z, rv[i].z, k);
      adam_elem(rw[i].w, rg[i].w, rm[i].w, rv[i].w, k);
      st4<PolAdam::ST>(w + o, rw[i]);
      st4<PolAdam::ST>(m + o, rm[i]);
      st4<PolAdam::ST>(v + o, rv[i]);
      if constexpr (BF16) store_bf16x4<PolAdam::ST>(w16 + o, rw[i]);
    }
  }
}

template <int BLOCK, bool BF16>
__global__ __launch_bounds__(BLOCK) void adam_kernel(float* w, const float* __restrict__ g, float* m, float* v,
                                                      uint16_t* __restrict__ w16, int64_t n4, int tail, AdamK k) {
  const int64_t tile4 = (int64_t)BLOCK * kAdamUnroll;
  const int64_t tiles = (n4 + tile4 - 1) / tile4;
  for (int64_t t = blockIdx.x; t < tiles; t += gridDim.x) {
    const int64_t e0 = t * (tile4 * 4);
    const int64_t left4 = n4 - t * tile4;
    if (left4 >= tile4)
      adam_tile<BLOCK, true, BF16>(w + e0, g + e0, m + e0, v + e0, w16 + e0, (int)tile4, k);
    else
      adam_tile<BLOCK, false, BF16>(w + e0, g + e0, m + e0, v + e0, w16 + e0, (int)left4, k);
  }
  if (blockIdx.x == 0 && (int)threadIdx.x < tail) {        // S % 4 leftover elements (align < 4 only)
    const int64_t e = 4 * n4 + threadIdx.x;
    float ww = w[e], mm = m[e], vv = v[e];
    adam_elem(ww, g[e], mm, vv, k);
    w[e] = ww; m[e] = mm; v[e] = vv;
    if constexpr (BF16) w16[e] = (uint16_t)bf16_of(ww);
  }
}

template <int BLOCK, bool FULL, bool BF16>
__device__ __forceinline__ void momentum_tile(float* w, const float* __restrict__ g, float* m,
                                              uint16_t* __restrict__ w16, int lim4, const MomentumK& k) {
  const int t4 = threadIdx.x * 4;
  F4 rw[kMomentumUnroll], rg[kMomentumUnroll], rm[kMomentumUnroll];
#pragma unroll
  for (int i = 0; i < kMomentumUnroll; ++i) {
    if (FULL || (int)threadIdx.x + i * BLOCK < lim4) {
      const int o = i * BLOCK * 4 + t4;
      rg[i] = ld4<PolMomentum::RO>(g + o);
      rw[i] = ld4<PolMomentum::RW>(w + o);
      rm[i] = ld4<PolMomentum::RW>(m + o);
    }
  }
#pragma unroll
  for (int i = 0; i < kMomentumUnroll; ++i) {
    if (FULL || (int)threadIdx.x + i * BLOCK < lim4) {
      const int o = i * BLOCK * 4 + t4;
      momentum_elem(rw[i].x, rg[i].x, rm[i].x, k);
      momentum_elem(rw[i].y, rg[i].y, rm[i].y, k);
      momentum_elem(rw[i].z, rg[i].z, rm[i].z, k);
      momentum_elem(rw[i].w, rg[i].w, rm[i].w, k);
      st4<PolMomentum::ST>(w + o, rw[i]);
      st4<PolMomentum::ST>(m + o, rm[i]);
      if constexpr (BF16) store_bf16x4<PolMomentum::ST>(w16 + o, rw[i]);
    }
  }
}

template <int BLOCK, bool BF16>
__global__ __launch_bounds__(BLOCK) void momentum_kernel(float* w, const float* __restrict__ g, float* m,
                                                          uint16_t* __restrict__ w16, int64_t n4, int tail,
                                                          MomentumK k) {
  const int64_t tile4 = (int64_t)BLOCK * kMomentumUnroll;
  const int64_t tiles = (n4 + tile4 - 1) / tile4;
  for (int64_t t = blockIdx.x; t < tiles; t += gridDim.x) {
    const int64_t e0 = t * (tile4 * 4);
    const int64_t left4 = n4 - t * tile4;
    if (left4 >= tile4)
      momentum_tile<BLOCK, true, BF16>(w + e0, g + e0, m + e0, w16 + e0, (int)tile4, k);
    else
      momentum_tile<BLOCK, false, BF16>(w + e0, g + e0, m + e0, w16 + e0, (int)left4, k);
  }
  if (blockIdx.x == 0 && (int)threadIdx.x < tail) {
    const int64_t e = 4 * n4 + threadIdx.x;
    float ww = w[e], mm = m[e];
    momentum_elem(ww, g[e], mm, k);
    w[e] = ww; m[e] = mm;
    if constexpr (BF16) w16[e] = (uint16_t)bf16_of(ww);
  }
}

// ---- LAMB ------------------------------------------------------------------------------------------
// Phase 1, one workgroup per chunk: moments, update direction, and the chunk's masked sums of
// w^2 and u^2 (Section 4.1: padded slots contribute the identity of the reduce; they are found
// by position, not by value).

// One tile of phase 1: `lim` = slots of the tile that exist, `valid` = leading slots that hold real
// elements (may be negative or exceed the tile).  FULL tiles run without branches; the mask on the
// sums is a select.
template <typename Pol, bool FULL, int GS, bool GFAST>
__device__ __forceinline__ void lamb_p1_tile(const float* __restrict__ w, const void* __restrict__ g, float* m,
                                             float* v, int lim, int valid, float wd, const AdamK& k, float& sw,
                                             float& su) {
  const int t4 = threadIdx.x * 4;
  F4 rw[kUnroll], rg[kUnroll], rm[kUnroll], rv[kUnroll];
#pragma unroll
  for (int i = 0; i < kUnroll; ++i) {
    const int o = i * kUpdBlock * 4 + t4;
    if (FULL || o < lim) {
      rg[i] = load_g4<GS, GFAST, Pol::RO>(g, o, valid);
      rw[i] = ld4<Pol::RO>(w + o);
      rm[i] = ld4<Pol::RW>(m + o);
      rv[i] = ld4<Pol::RW>(v + o);
    }
  }
#pragma unroll
  for (int i = 0; i < kUnroll; ++i) {
    const int o = i * kUpdBlock * 4 + t4;
    if (FULL || o < lim) {
      float d, wm;
#define SU_LAMB_P1_LANE(c, j)                       \
  lamb_moments(rg[i].c, rm[i].c, rv[i].c, k);       \
  d = lamb_dir(rw[i].c, rm[i].c, rv[i].c, wd, k);   \
  d = (o + j < valid) ? d : 0.0f;                   \
  wm = (o + j < valid) ? rw[i].c : 0.0f;            \
  sw = fmaf(wm, wm, sw);                            \
  su = fmaf(d, d, su);
      SU_LAMB_P1_LANE(x, 0)
      SU_LAMB_P1_LANE(y, 1)
      SU_LAMB_P1_LANE(z, 2)
      SU_LAMB_P1_LANE(w, 3)
#undef SU_LAMB_P1_LANE
      st4<Pol::ST>(m + o, rm[i]);
      st4<Pol::ST>(v + o, rv[i]);
    }
  }
}

template <typename Pol, bool VEC, int GS>
__global__ __launch_bounds__(kUpdBlock) void lamb_p1_kernel(const VarDesc* __restrict__ vars,
                                                         const ChunkDesc* __restrict__ chunks,
                                                         const float* __restrict__ w, const float* __restrict__ g,
                                                         const void* const* __restrict__ g_full, float* m, float* v,
                                                         float* __restrict__ chunk_sums, int r, AdamK k) {
  const int c = (int)blockIdx.x;
  const ChunkView cv = chunk_view(vars, chunks, c, r);
  const float wd = (cv.flags & SHARD_VAR_NO_DECAY) ? 0.0f : k.wd;
  const GradChunk<GS> gc = grad_chunk<GS>(g, g_full, cv);
  float sw = 0.0f, su = 0.0f;
  if constexpr (VEC) {
    for (int base = 0; base < cv.len; base += kTileElems) {
      const int64_t s0 = cv.shard0 + base;
      const int lim = cv.len - base, valid = cv.valid - base;
      if (lim >= kTileElems) {
        if (gc.fast(kTileElems, valid))
          lamb_p1_tile<Pol, true, GS, true>(w + s0, gc.tile(base), m + s0, v + s0, kTileElems, valid, wd, k, sw, su);
        else
          lamb_p1_tile<Pol, true, GS, false>(w + s0, gc.tile(base), m + s0, v + s0, kTileElems, valid, wd, k, sw, su);
      } else {
        if (gc.fast(lim, valid))
          lamb_p1_tile<Pol, false, GS, true>(w + s0, gc.tile(base), m + s0, v + s0, lim, valid, wd, k, sw, su);
        else
          lamb_p1_tile<Pol, false, GS, false>(w + s0, gc.tile(base), m + s0, v + s0, lim, valid, wd, k, sw, su);
      }
    }
  } else {
    for (int e = threadIdx.x; e < cv.len; e += kUpdBlock) {
      const int64_t s = cv.shard0 + e;
      float mm = m[s], vv = v[s];
      const float ww = w[s];
      lamb_moments(load_g1<GS>(gc, e, cv.valid), mm, vv, k);
      float d = lamb_dir(ww, mm, vv, wd, k);
      d = (e < cv.valid) ? d : 0.0f;
      const float wm = (e < cv.valid) ? ww : 0.0f;
      sw = fmaf(wm, wm, sw);
      su = fmaf(d, d, su);
      m[s] = mm;
      v[s] = vv;
    }
  }
  block_sum2(sw, su);
  if (threadIdx.x == 0) {
    chunk_sums[2 * c] = sw;
    chunk_sums[2 * c + 1] = su;
  }
}

// One workgroup per variable: adds the variable's chunk sums in an order that depends only on the
// chunk table (thread t takes chunks t, t + kUpdBlock, ...; float64 accumulators; wavefront shuffles,
// then the four wavefronts in order), optionally adds the other replicas' table (the all-reduce
// stand-in).
// (Folding this into phase 1, with the workgroup that finishes a variable's last chunk doing the
// addition, was measured and rejected: publishing a chunk's sums to workgroups on other XCDs needs a
// device-scope release, which on this multi-XCD part writes back the XCD's whole L2; with every
// workgroup doing that, phase 1 ran 9x slower.)
__global__ __launch_bounds__(kBlock) void norm_reduce_kernel(const VarDesc* __restrict__ vars,
                                                             const float* __restrict__ chunk_sums, int V,
                                                             const float* __restrict__ other, float* sums_out,
                                                             float* local_out) {
  __shared__ double part[2 * (kBlock / 64)];
  const int i = blockIdx.x;
  const VarDesc vd = vars[i];
  double a = 0.0, b = 0.0;
  // the pair of a chunk in one 8-byte load, eight unconditional loads in flight (in a last, partial batch the
  // indices past the end are redirected, and only the additions are predicated: a conditional load would make the
  // compiler wait for each one, and this kernel is all latency); each thread still adds its chunks in rising order
  const float2* pairs = reinterpret_cast<const float2*>(chunk_sums) + vd.first_chunk;
  for (int c = threadIdx.x; c < vd.n_chunks; c += 8 * kBlock) {
    float2 x[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int cj = c + j * kBlock;
      x[j] = pairs[cj < vd.n_chunks ? cj : c];       // past the end: a pair that is loaded anyway, not added
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      if (c + j * kBlock < vd.n_chunks) {
        a += (double)x[j].x;
        b += (double)x[j].y;
      }
    }
  }
#pragma unroll
  for (int s = 32; s >= 1; s >>= 1) {
    a += __shfl_xor(a, s, 64);
    b += __shfl_xor(b, s, 64);
  }
  const int wave = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) {
    part[2 * wave] = a;
    part[2 * wave + 1] = b;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    a = part[0];
    b = part[1];
#pragma unroll
    for (int w = 1; w < kBlock / 64; ++w) {
      a += part[2 * w];
      b += part[2 * w + 1];
    }
    const float la = (float)a, lb = (float)b;
    if (local_out) {
      local_out[2 * i] = la;
      local_out[2 * i + 1] = lb;
    }
    if (sums_out) {
      sums_out[2 * i] = other ? la + other[2 * i] : la;
      sums_out[2 * i + 1] = other ? lb + other[2 * i + 1] : lb;
    }
  }
}

// Phase 2, one workgroup per chunk: trust ratio of the chunk's variable from the all-reduced
// sums, then w -= lr * ratio * u with u re-created from (old w, new m, new v).
template <bool FULL, bool BF16>
__device__ __forceinline__ void lamb_p2_tile(float* w, const float* __restrict__ m, const float* __restrict__ v,
                                             uint16_t* __restrict__ w16, int lim, float wd, float step,
                                             const AdamK& k) {
  const int t4 = threadIdx.x * 4;
  F4 rw[kUnroll], rm[kUnroll], rv[kUnroll];
#pragma unroll
  for (int i = 0; i < kUnroll; ++i) {
    const int o = i * kUpdBlock * 4 + t4;
    if (FULL || o < lim) {
      rw[i] = ld4<PolLambP2::RW>(w + o);
      rm[i] = ld4<PolLambP2::RO>(m + o);
      rv[i] = ld4<PolLambP2::RO>(v + o);
    }
  }
#pragma unroll
  for (int i = 0; i < kUnroll; ++i) {
    const int o = i * kUpdBlock * 4 + t4;
    if (FULL || o < lim) {
      rw[i].x = fmaf(-step, lamb_dir(rw[i].x, rm[i].x, rv[i].x, wd, k), rw[i].x);
      rw[i].y = fmaf(-step, lamb_dir(rw[i].y, rm[i].y, rv[i].y, wd, k), rw[i].y);
      rw[i].z = fmaf(-step, lamb_dir(rw[i].z, rm[i].z, rv[i].z, wd, k), rw[i].z);
      rw[i].w = fmaf(-step, lamb_dir(rw[i].w, rm[i].w, rv[i].w, wd, k), rw[i].w);
      st4<PolLambP2::ST>(w + o, rw[i]);
      if constexpr (BF16) store_bf16x4<PolLambP2::ST>(w16 + o, rw[i]);
    }
  }
}

template <bool VEC, bool BF16>
__global__ __launch_bounds__(kUpdBlock) void lamb_p2_kernel(const VarDesc* __restrict__ vars,
                                                         const ChunkDesc* __restrict__ chunks, float* w,
                                                         const float* __restrict__ m, const float* __restrict__ v,
                                                         uint16_t* __restrict__ w16, const float* __restrict__ sums,
                                                         AdamK k) {
  const int c = (int)(gridDim.x - 1 - blockIdx.x);          // opposite direction to phase 1: starts on what it touched last
  const ChunkView cv = chunk_view(vars, chunks, c, 0);
  const float wd = (cv.flags & SHARD_VAR_NO_DECAY) ? 0.0f : k.wd;
  float ratio = 1.0f;
  if (!(cv.flags & SHARD_VAR_NO_ADAPT)) {
    const float wn = sqrtf(sums[2 * cv.var]), un = sqrtf(sums[2 * cv.var + 1]);
    if (wn > 0.0f && un > 0.0f) ratio = wn / un;
  }
  const float step = k.lr * ratio;
  if constexpr (VEC) {
    for (int base = 0; base < cv.len; base += kTileElems) {
      const int64_t s0 = cv.shard0 + base;
      if (base + kTileElems <= cv.len)
        lamb_p2_tile<true, BF16>(w + s0, m + s0, v + s0, w16 + s0, kTileElems, wd, step, k);
      else
        lamb_p2_tile<false, BF16>(w + s0, m + s0, v + s0, w16 + s0, cv.len - base, wd, step, k);
    }
  } else {
    for (int e = threadIdx.x; e < cv.len; e += kUpdBlock) {
      const int64_t s = cv.shard0 + e;
      const float ww = w[s];
      const float nw = fmaf(-step, lamb_dir(ww, m[s], v[s], wd, k), ww);
      w[s] = nw;
      if constexpr (BF16) w16[s] = (uint16_t)bf16_of(nw);
    }
  }
}

// ---- LARS ------------------------------------------------------------------------------------------
// Phase 1 only reads: masked sums of w^2 and g^2 per chunk.  Phase 2 is the momentum update with a
// per-variable learning-rate scale.

template <bool FULL, int GS, bool GFAST>
__device__ __forceinline__ void lars_p1_tile(const float* __restrict__ w, const void* __restrict__ g, int lim,
                                             int valid, float& sw, float& sg) {
  const int t4 = threadIdx.x * 4;
  F4 rw[kUnroll], rg[kUnroll];
#pragma unroll
  for (int i = 0; i < kUnroll; ++i) {
    const int o = i * kUpdBlock * 4 + t4;
    if (FULL || o < lim) {
      rg[i] = load_g4<GS, GFAST, PolLars::RO>(g, o, valid);
      rw[i] = ld4<PolLars::RO>(w + o);
    }
  }
#pragma unroll
  for (int i = 0; i < kUnroll; ++i) {
    const int o = i * kUpdBlock * 4 + t4;
    if (FULL || o < lim) {
      float a, b;
#define SU_LARS_P1_LANE(c, j)                 \
  a = (o + j < valid) ? rw[i].c : 0.0f;       \
  b = (o + j < valid) ? rg[i].c : 0.0f;       \
  sw = fmaf(a, a, sw);                        \
  sg = fmaf(b, b, sg);
      SU_LARS_P1_LANE(x, 0)
      SU_LARS_P1_LANE(y, 1)
      SU_LARS_P1_LANE(z, 2)
      SU_LARS_P1_LANE(w, 3)
#undef SU_LARS_P1_LANE
    }
  }
}

template <bool VEC, int GS>
__global__ __launch_bounds__(kUpdBlock) void lars_p1_kernel(const VarDesc* __restrict__ vars,
                                                         const ChunkDesc* __restrict__ chunks,
                                                         const float* __restrict__ w, const float* __restrict__ g,
                                                         const void* const* __restrict__ g_full,
                                                         float* __restrict__ chunk_sums, int r) {
  const int c = blockIdx.x;
  const ChunkView cv = chunk_view(vars, chunks, c, r);
  const GradChunk<GS> gc = grad_chunk<GS>(g, g_full, cv);
  float sw = 0.0f, sg = 0.0f;
  if constexpr (VEC) {
    for (int base = 0; base < cv.len; base += kTileElems) {
      const int64_t s0 = cv.shard0 + base;
      const int lim = cv.len - base, valid = cv.valid - base;
      if (lim >= kTileElems) {
        if (gc.fast(kTileElems, valid)) lars_p1_tile<true, GS, true>(w + s0, gc.tile(base), kTileElems, valid, sw, sg);
        else lars_p1_tile<true, GS, false>(w + s0, gc.tile(base), kTileElems, valid, sw, sg);
      } else {
        if (gc.fast(lim, valid)) lars_p1_tile<false, GS, true>(w + s0, gc.tile(base), lim, valid, sw, sg);
        else lars_p1_tile<false, GS, false>(w + s0, gc.tile(base), lim, valid, sw, sg);
      }
    }
  } else {
    for (int e = threadIdx.x; e < cv.len; e += kUpdBlock) {
      const float a = (e < cv.valid) ? w[cv.shard0 + e] : 0.0f;
      const float b = (e < cv.valid) ? load_g1<GS>(gc, e, cv.valid) : 0.0f;
      sw = fmaf(a, a, sw);
      sg = fmaf(b, b, sg);
    }
  }
  block_sum2(sw, sg);
  if (threadIdx.x == 0) {
    chunk_sums[2 * c] = sw;
    chunk_sums[2 * c + 1] = sg;
  }
}

__device__ __forceinline__ void lars_elem(float& w, float g, float& m, float wd, float scale, float mu) {
  g = fmaf(wd, w, g);
  m = fmaf(mu, m, scale * g);
  w = w - m;
}

template <bool FULL, bool BF16, int GS, bool GFAST>
__device__ __forceinline__ void lars_p2_tile(float* w, const void* __restrict__ g, float* m,
                                             uint16_t* __restrict__ w16, int lim, int valid, float wd, float scale,
                                             float mu) {
  const int t4 = threadIdx.x * 4;
  F4 rw[kUnroll], rg[kUnroll], rm[kUnroll];
#pragma unroll
  for (int i = 0; i < kUnroll; ++i) {
    const int o = i * kUpdBlock * 4 + t4;
    if (FULL || o < lim) {
      rg[i] = load_g4<GS, GFAST, PolLarsP2::RO>(g, o, valid);
      rw[i] = ld4<PolLarsP2::RW>(w + o);
      rm[i] = ld4<PolLarsP2::RW>(m + o);
    }
  }
#pragma unroll
  for (int i = 0; i < kUnroll; ++i) {
    const int o = i * kUpdBlock * 4 + t4;
    if (FULL || o < lim) {
      lars_elem(rw[i].x, rg[i].x, rm[i].x, wd, scale, mu);
      lars_elem(rw[i].y, rg[i].y, rm[i].y, wd, scale, mu);
      lars_elem(rw[i].z, rg[i].z, rm[i].z, wd, scale, mu);
      lars_elem(rw[i].w, rg[i].w, rm[i].w, wd, scale, mu);
      st4<PolLarsP2::ST>(w + o, rw[i]);
      st4<PolLarsP2::ST>(m + o, rm[i]);
      if constexpr (BF16) store_bf16x4<PolLarsP2::ST>(w16 + o, rw[i]);
    }
  }
}

template <bool VEC, bool BF16, int GS>
__global__ __launch_bounds__(kUpdBlock) void lars_p2_kernel(const VarDesc* __restrict__ vars,
                                                         const ChunkDesc* __restrict__ chunks, float* w,
                                                         const float* __restrict__ g,
                                                         const void* const* __restrict__ g_full, float* m,
                                                         uint16_t* __restrict__ w16, const float* __restrict__ sums,
                                                         int r, LarsK k) {
  const int c = (int)(gridDim.x - 1 - blockIdx.x);          // opposite direction to phase 1
  const ChunkView cv = chunk_view(vars, chunks, c, r);
  const GradChunk<GS> gc = grad_chunk<GS>(g, g_full, cv);
  const float wd = (cv.flags & SHARD_VAR_NO_DECAY) ? 0.0f : k.wd;
  float local_lr = 1.0f;
  if (!(cv.flags & SHARD_VAR_NO_ADAPT)) {
    const float wn = sqrtf(sums[2 * cv.var]), gn = sqrtf(sums[2 * cv.var + 1]);
    if (wn > 0.0f && gn > 0.0f) local_lr = k.trust * wn / (gn + wd * wn + k.eps);
  }
  const float scale = k.lr * local_lr;
  if constexpr (VEC) {
    for (int base = 0; base < cv.len; base += kTileElems) {
      const int64_t s0 = cv.shard0 + base;
      const int lim = cv.len - base, valid = cv.valid - base;
      if (lim >= kTileElems) {
        if (gc.fast(kTileElems, valid))
          lars_p2_tile<true, BF16, GS, true>(w + s0, gc.tile(base), m + s0, w16 + s0, kTileElems, valid, wd, scale, k.mu);
        else
          lars_p2_tile<true, BF16, GS, false>(w + s0, gc.tile(base), m + s0, w16 + s0, kTileElems, valid, wd, scale, k.mu);
      } else {
        if (gc.fast(lim, valid))
          lars_p2_tile<false, BF16, GS, true>(w + s0, gc.tile(base), m + s0, w16 + s0, lim, valid, wd, scale, k.mu);
        else
          lars_p2_tile<false, BF16, GS, false>(w + s0, gc.tile(base), m + s0, w16 + s0, lim, valid, wd, scale, k.mu);
      }
    }
  } else {
    for (int e = threadIdx.x; e < cv.len; e += kUpdBlock) {
      const int64_t s = cv.shard0 + e;
      float ww = w[s], mm = m[s];
      lars_elem(ww, load_g1<GS>(gc, e, cv.valid), mm, wd, scale, k.mu);
      w[s] = ww;
      m[s] = mm;
      if constexpr (BF16) w16[s] = (uint16_t)bf16_of(ww);
    }
  }
}

// ---- Adam and momentum with the gradient read from the full tensors ---------------------------------
// The flat kernels above need no table; reading the gradient in place does (which tensor, which
// offset, how many real slots), so these walk the chunk table like the LAMB kernels.  Per element the
// arithmetic is the flat kernels', and a padded slot sees g = +0.0: the same bits as shard_format
// followed by the flat kernel.
template <bool FULL, bool BF16, int GS, bool GFAST>
__device__ __forceinline__ void adam_chunk_tile(float* w, const void* __restrict__ g, float* m, float* v,
                                                uint16_t* __restrict__ w16, int lim, int valid, const AdamK& k) {
  const int t4 = threadIdx.x * 4;
  F4 rw[kUnroll], rg[kUnroll], rm[kUnroll], rv[kUnroll];
#pragma unroll
  for (int i = 0; i < kUnroll; ++i) {
    const int o = i * kUpdBlock * 4 + t4;
    if (FULL || o < lim) {
      rg[i] = load_g4<GS, GFAST, true>(g, o, valid);
      rw[i] = ld4<PolAdam::RW>(w + o);
      rm[i] = ld4<PolAdam::RW>(m + o);
      rv[i] = ld4<PolAdam::RW>(v + o);
    }
  }
#pragma unroll
  for (int i = 0; i < kUnroll; ++i) {
    const int o = i * kUpdBlock * 4 + t4;
    if (FULL || o < lim) {
      adam_elem(rw[i].x, rg[i].x, rm[i].x, rv[i].x, k);
      adam_elem(rw[i].y, rg[i].y, rm[i].y, rv[i].y, k);
      adam_elem(rw[i].z, rg[i].z, rm[i].z, rv[i].z, k);
      adam_elem(rw[i].w, rg[i].w, rm[i].w, rv[i].w, k);
      st4<PolAdam::ST>(w + o, rw[i]);
      st4<PolAdam::ST>(m + o, rm[i]);
      st4<PolAdam::ST>(v + o, rv[i]);
      if constexpr (BF16) store_bf16x4<PolAdam::ST>(w16 + o, rw[i]);
    }
  }
}

template <bool VEC, bool BF16, int GS>
__global__ __launch_bounds__(kUpdBlock) void adam_chunk_kernel(const VarDesc* __restrict__ vars,
                                                            const ChunkDesc* __restrict__ chunks, float* w,
                                                            const void* const* __restrict__ g_full, float* m, float* v,
                                                            uint16_t* __restrict__ w16, int r, AdamK k) {
  const ChunkView cv = chunk_view(vars, chunks, blockIdx.x, r);
  const GradChunk<GS> gc = grad_chunk<GS>(nullptr, g_full, cv);
  if constexpr (VEC) {
    for (int base = 0; base < cv.len; base += kTileElems) {
      const int64_t s0 = cv.shard0 + base;
      const int lim = cv.len - base, valid = cv.valid - base;
      if (lim >= kTileElems) {
        if (gc.fast(kTileElems, valid))
          adam_chunk_tile<true, BF16, GS, true>(w + s0, gc.tile(base), m + s0, v + s0, w16 + s0, kTileElems, valid, k);
        else
          adam_chunk_tile<true, BF16, GS, false>(w + s0, gc.tile(base), m + s0, v + s0, w16 + s0, kTileElems, valid, k);
      } else {
        if (gc.fast(lim, valid))
          adam_chunk_tile<false, BF16, GS, true>(w + s0, gc.tile(base), m + s0, v + s0, w16 + s0, lim, valid, k);
        else
          adam_chunk_tile<false, BF16, GS, false>(w + s0, gc.tile(base), m + s0, v + s0, w16 + s0, lim, valid, k);
      }
    }
  } else {
    for (int e = threadIdx.x; e < cv.len; e += kUpdBlock) {
      const int64_t s = cv.shard0 + e;
      float ww = w[s], mm = m[s], vv = v[s];
      adam_elem(ww, load_g1<GS>(gc, e, cv.valid), mm, vv, k);
      w[s] = ww; m[s] = mm; v[s] = vv;
      if constexpr (BF16) w16[s] = (uint16_t)bf16_of(ww);
    }
  }
}

template <bool FULL, bool BF16, int GS, bool GFAST>
__device__ __forceinline__ void momentum_chunk_tile(float* w, const void* __restrict__ g, float* m,
                                                    uint16_t* __restrict__ w16, int lim, int valid,
                                                    const MomentumK& k) {
  const int t4 = threadIdx.x * 4;
  F4 rw[kUnroll], rg[kUnroll], rm[kUnroll];
#pragma unroll
  for (int i = 0; i < kUnroll; ++i) {
    const int o = i * kUpdBlock * 4 + t4;
    if (FULL || o < lim) {
      rg[i] = load_g4<GS, GFAST, true>(g, o, valid);
      rw[i] = ld4<PolMomentum::RW>(w + o);
      rm[i] = ld4<PolMomentum::RW>(m + o);
    }
  }
#pragma unroll
  for (int i = 0; i < kUnroll; ++i) {
    const int o = i * kUpdBlock * 4 + t4;
    if (FULL || o < lim) {
      momentum_elem(rw[i].x, rg[i].x, rm[i].x, k);
      momentum_elem(rw[i].y, rg[i].y, rm[i].y, k);
      momentum_elem(rw[i].z, rg[i].z, rm[i].z, k);
      momentum_elem(rw[i].w, rg[i].w, rm[i].w, k);
      st4<PolMomentum::ST>(w + o, rw[i]);
      st4<PolMomentum::ST>(m + o, rm[i]);
      if constexpr (BF16) store_bf16x4<PolMomentum::ST>(w16 + o, rw[i]);
    }
  }
}

template <bool VEC, bool BF16, int GS>
__global__ __launch_bounds__(kUpdBlock) void momentum_chunk_kernel(const VarDesc* __restrict__ vars,
                                                                const ChunkDesc* __restrict__ chunks, float* w,
                                                                const void* const* __restrict__ g_full, float* m,
                                                                uint16_t* __restrict__ w16, int r, MomentumK k) {
  const ChunkView cv = chunk_view(vars, chunks, blockIdx.x, r);
  const GradChunk<GS> gc = grad_chunk<GS>(nullptr, g_full, cv);
  if constexpr (VEC) {
    for (int base = 0; base < cv.len; base += kTileElems) {
      const int64_t s0 = cv.shard0 + base;
      const int lim = cv.len - base, valid = cv.valid - base;
      if (lim >= kTileElems) {
        if (gc.fast(kTileElems, valid))
          momentum_chunk_tile<true, BF16, GS, true>(w + s0, gc.tile(base), m + s0, w16 + s0, kTileElems, valid, k);
        else
          momentum_chunk_tile<true, BF16, GS, false>(w + s0, gc.tile(base), m + s0, w16 + s0, kTileElems, valid, k);
      } else {
        if (gc.fast(lim, valid))
          momentum_chunk_tile<false, BF16, GS, true>(w + s0, gc.tile(base), m + s0, w16 + s0, lim, valid, k);
        else
          momentum_chunk_tile<false, BF16, GS, false>(w + s0, gc.tile(base), m + s0, w16 + s0, lim, valid, k);
      }
    }
  } else {
    for (int e = threadIdx.x; e < cv.len; e += kUpdBlock) {
      const int64_t s = cv.shard0 + e;
      float ww = w[s], mm = m[s];
      momentum_elem(ww, load_g1<GS>(gc, e, cv.valid), mm, k);
      w[s] = ww; m[s] = mm;
      if constexpr (BF16) w16[s] = (uint16_t)bf16_of(ww);
    }
  }
}

// ---- launch shapes: how much a CU keeps in flight --------------------------------------------------
// A streaming kernel is fastest when the loads in flight cover bandwidth x latency and little more.  Measured on
// MI355X with an Adam-shaped update (4 streams read, 3 written) on shards too large for the 256 MB memory-side
// cache to help: 40 to 48 KB of loads in flight per CU (10 to 12 wavefronts with one 128-bit load per stream)
// sustain 6.2 to 6.4 TB/s, while the 128 KB that full occupancy keeps in flight (8 workgroups of 256 threads)
// sustain 5.4 to 5.6: in-flight lines beyond what the memory system needs only crowd the L2 (4 MB per XCD for 32
// CUs).  Fewer, smaller workgroups do better still (128 threads, 5 per CU: +2.5 % over 256 threads, 2 per CU).
// Shards whose state fits the memory-side cache or nearly so behave the other way (full occupancy is up to 4 %
// faster), so the launchers choose by shard size.
// The cap on resident workgroups is LDS that the launch reserves and the kernel never touches: a CU has 160 KB,
// so workgroups that each ask for 160/k KB, less a margin for the kernel's own few bytes, fit k to a CU.
constexpr unsigned lds_for(int workgroups_per_cu) { return (unsigned)(160 * 1024 / workgroups_per_cu - 1024); }
constexpr unsigned kNoCap = 0;
// Shards from this many slots on are "large" for the table-driven kernels: a single float32 stream of the shard
// (256 MB) no longer fits the memory-side cache.  Measured on the 340 M-parameter list: 84 M slots gain 4 % from
// the large shape, 42 M slots lose 4 % on the whole step.
constexpr int64_t kLargeShard = (int64_t)1 << 26;
// The flat kernels (Adam, momentum) switch earlier: from 2^25 slots their three or four streams of state are
// several times the cache (42 M slots: +10 %; 13 M and 25 M slots, which fit: -2 to -4 %).
constexpr int64_t kLargeFlatShard = (int64_t)1 << 25;
constexpr int kFlatBlockSmall = 256, kFlatBlockLarge = 128;
constexpr unsigned kLdsFlatLarge = lds_for(5);
// Table-driven kernels (256 threads, two accesses per thread and stream: 32 KB of loads per workgroup in LAMB's
// phase 1).  Their workgroups start with two dependent table look-ups, so they need more of them resident than
// the flat kernels to hide that; three per CU is the measured optimum on large shards (LAMB on 336 M slots
// 2350 -> 2180 us, LARS 1650 -> 1580), no cap on shards that the memory-side cache helps (42 M slots: within 1 %).
// Phase 1 of LARS only reads and is fastest uncapped.  The updates that read full gradient tensors gain 2 to 5 %
// from the cap at every size measured (13 M to 336 M slots).
constexpr unsigned kLdsLambP1Large = lds_for(3);
constexpr unsigned kLdsLambP2Large = lds_for(3);
constexpr unsigned kLdsLarsP2Large = lds_for(3);
constexpr unsigned kLdsLambP1 = kNoCap;
constexpr unsigned kLdsLambP2 = kNoCap;
constexpr unsigned kLdsLarsP1 = kNoCap;
constexpr unsigned kLdsLarsP2 = kNoCap;
constexpr unsigned kLdsAdamChunk = lds_for(3);
constexpr unsigned kLdsMomentumChunk = lds_for(3);

inline unsigned flat_grid(int64_t n4, int block, int unroll) {
  const int64_t tile = (int64_t)block * unroll;
  int64_t tiles = (n4 + tile - 1) / tile;
  if (tiles < 1) tiles = 1;
  if (tiles > 0x7FFFFFFF) tiles = 0x7FFFFFFF;      // the kernels loop over tiles
  return (unsigned)tiles;
}

}  // namespace

// ---- launchers -------------------------------------------------------------------------------------

hipError_t launch_adam(shard_plan_t* p, float* w, const float* g, float* m, float* v, void* w16, const AdamK& k,
                       hipStream_t stream) {
  if (p->S == 0) return hipSuccess;
  ProfScope ps(p, SHARD_K_ADAM, stream);
  const int64_t n4 = p->S >> 2;
  const int tail = (int)(p->S & 3);
  uint16_t* o = (uint16_t*)w16;
#define SU_LAUNCH_ADAM(BLOCK, BF16, LDS)                                                                      \
  hipLaunchKernelGGL((adam_kernel<BLOCK, BF16>), dim3(flat_grid(n4, BLOCK, kAdamUnroll)), dim3(BLOCK), LDS, stream, \
                     w, g, m, v, o, n4, tail, k)
  if (p->S >= kLargeFlatShard) {
    if (o) SU_LAUNCH_ADAM(kFlatBlockLarge, true, kLdsFlatLarge); else SU_LAUNCH_ADAM(kFlatBlockLarge, false, kLdsFlatLarge);
  } else {
    if (o) SU_LAUNCH_ADAM(kFlatBlockSmall, true, kNoCap); else SU_LAUNCH_ADAM(kFlatBlockSmall, false, kNoCap);
  }
#undef SU_LAUNCH_ADAM
  return hipGetLastError();
}

// The flat Adam update in a launch shape the caller names (shard_profile_adam_shape, a measurement aid): the same
// kernels as launch_adam, so the results are the same bits; only the time differs.
hipError_t launch_adam_shape(shard_plan_t* p, float* w, const float* g, float* m, float* v, const AdamK& k,
                             int block, int workgroups_per_cu, hipStream_t stream) {
  if (p->S == 0) return hipSuccess;
  ProfScope ps(p, SHARD_K_ADAM_SHAPE, stream);
  const int64_t n4 = p->S >> 2;
  const int tail = (int)(p->S & 3);
  const unsigned lds = workgroups_per_cu > 0 ? (unsigned)(160 * 1024 / workgroups_per_cu - 1024) : 0u;
  uint16_t* none = nullptr;
  if (block == 128)
    hipLaunchKernelGGL((adam_kernel<128, false>), dim3(flat_grid(n4, 128, kAdamUnroll)), dim3(128), lds, stream, w, g, m,
                       v, none, n4, tail, k);
  else
    hipLaunchKernelGGL((adam_kernel<256, false>), dim3(flat_grid(n4, 256, kAdamUnroll)), dim3(256), lds, stream, w, g, m,
                       v, none, n4, tail, k);
  return hipGetLastError();
}

hipError_t launch_momentum(shard_plan_t* p, float* w, const float* g, float* m, void* w16, const MomentumK& k,
                           hipStream_t stream) {
  if (p->S == 0) return hipSuccess;
  ProfScope ps(p, SHARD_K_MOMENTUM, stream);
  const int64_t n4 = p->S >> 2;
  const int tail = (int)(p->S & 3);
  uint16_t* o = (uint16_t*)w16;
#define SU_LAUNCH_MOM(BLOCK, BF16, LDS)                                                                              \
  hipLaunchKernelGGL((momentum_kernel<BLOCK, BF16>), dim3(flat_grid(n4, BLOCK, kMomentumUnroll)), dim3(BLOCK), LDS, \
                     stream, w, g, m, o, n4, tail, k)
  if (p->S >= kLargeFlatShard) {
    if (o) SU_LAUNCH_MOM(kFlatBlockLarge, true, kLdsFlatLarge); else SU_LAUNCH_MOM(kFlatBlockLarge, false, kLdsFlatLarge);
  } else {
    if (o) SU_LAUNCH_MOM(kFlatBlockSmall, true, kNoCap); else SU_LAUNCH_MOM(kFlatBlockSmall, false, kNoCap);
  }
#undef SU_LAUNCH_MOM
  return hipGetLastError();
}

hipError_t launch_lamb_p1(shard_plan_t* p, int r, const float* w, const float* g, int g_source,
                          const void* const* g_full, float* m, float* v, const AdamK& k, hipStream_t stream,
                          float* chunk_sums) {
  if (p->chunks.empty()) return hipSuccess;
  ProfScope ps(p, SHARD_K_LAMB_P1, stream);
  const dim3 grid((unsigned)p->chunks.size());
  const VarDesc* vars = ws_at<VarDesc>(p, p->ws.vars);
  const ChunkDesc* chunks = ws_at<ChunkDesc>(p, p->ws.chunks);
  float* cs = chunk_sums ? chunk_sums : ws_at<float>(p, p->ws.chunk_sums);
  const bool vec = p->align % 4 == 0;
  // Large shards: m and v are stored past the caches as well (nothing the next kernel reads of them would still
  // be cached by then) and three workgroups stay resident per CU.
  const bool large = p->S >= kLargeShard;
#define SU_LAUNCH_P1(VEC, GS)                                                                                       \
  do {                                                                                                              \
    if (large)                                                                                                      \
      hipLaunchKernelGGL((lamb_p1_kernel<PolLambLarge, VEC, GS>), grid, dim3(kUpdBlock), kLdsLambP1Large, stream, vars, \
                         chunks, w, g, g_full, m, v, cs, r, k);                                                     \
    else                                                                                                            \
      hipLaunchKernelGGL((lamb_p1_kernel<PolLamb, VEC, GS>), grid, dim3(kUpdBlock), kLdsLambP1, stream, vars, chunks, w, \
                         g, g_full, m, v, cs, r, k);                                                                \
  } while (0)
  if (g_source == 0) {
    if (vec) SU_LAUNCH_P1(true, 0); else SU_LAUNCH_P1(false, 0);
  } else if (g_source == 1) {
    if (vec) SU_LAUNCH_P1(true, 1); else SU_LAUNCH_P1(false, 1);
  } else {
    if (vec) SU_LAUNCH_P1(true, 2); else SU_LAUNCH_P1(false, 2);
  }
#undef SU_LAUNCH_P1
  return hipGetLastError();
}

hipError_t launch_norm_reduce(shard_plan_t* p, const float* other, float* sums_out, float* local_out,
                              hipStream_t stream, const float* chunk_sums) {
  if (p->V == 0) return hipSuccess;
  ProfScope ps(p, SHARD_K_NORM_REDUCE, stream);
  const dim3 grid((unsigned)p->V);
  hipLaunchKernelGGL(norm_reduce_kernel, grid, dim3(kBlock), 0, stream, ws_at<VarDesc>(p, p->ws.vars),
                     chunk_sums ? chunk_sums : ws_at<float>(p, p->ws.chunk_sums), p->V, other, sums_out, local_out);
  return hipGetLastError();
}

hipError_t launch_lamb_p2(shard_plan_t* p, int r, float* w, const float* m, const float* v, void* w16, const AdamK& k,
                          const float* sums, hipStream_t stream) {
  (void)r;
  if (p->chunks.empty()) return hipSuccess;
  ProfScope ps(p, SHARD_K_LAMB_P2, stream);
  const dim3 grid((unsigned)p->chunks.size());
  const VarDesc* vars = ws_at<VarDesc>(p, p->ws.vars);
  const ChunkDesc* chunks = ws_at<ChunkDesc>(p, p->ws.chunks);
  const bool vec = p->align % 4 == 0;
  uint16_t* o = (uint16_t*)w16;
  const unsigned lds = p->S >= kLargeShard ? kLdsLambP2Large : kLdsLambP2;
  if (vec && o) hipLaunchKernelGGL((lamb_p2_kernel<true, true>), grid, dim3(kUpdBlock), lds, stream, vars, chunks, w, m, v, o, sums, k);
  else if (vec) hipLaunchKernelGGL((lamb_p2_kernel<true, false>), grid, dim3(kUpdBlock), lds, stream, vars, chunks, w, m, v, o, sums, k);
  else if (o) hipLaunchKernelGGL((lamb_p2_kernel<false, true>), grid, dim3(kUpdBlock), lds, stream, vars, chunks, w, m, v, o, sums, k);
  else hipLaunchKernelGGL((lamb_p2_kernel<false, false>), grid, dim3(kUpdBlock), lds, stream, vars, chunks, w, m, v, o, sums, k);
  return hipGetLastError();
}

hipError_t launch_lars_p1(shard_plan_t* p, int r, const float* w, const float* g, int g_source,
                          const void* const* g_full, hipStream_t stream) {
  if (p->chunks.empty()) return hipSuccess;
  ProfScope ps(p, SHARD_K_LARS_P1, stream);
  const dim3 grid((unsigned)p->chunks.size());
  const VarDesc* vars = ws_at<VarDesc>(p, p->ws.vars);
  const ChunkDesc* chunks = ws_at<ChunkDesc>(p, p->ws.chunks);
  float* cs = ws_at<float>(p, p->ws.chunk_sums);
  const bool vec = p->align % 4 == 0;
#define SU_LAUNCH(VEC, GS) \
  hipLaunchKernelGGL((lars_p1_kernel<VEC, GS>), grid, dim3(kUpdBlock), kLdsLarsP1, stream, vars, chunks, w, g, g_full, cs, r)
  if (g_source == 0) { if (vec) SU_LAUNCH(true, 0); else SU_LAUNCH(false, 0); }
  else if (g_source == 1) { if (vec) SU_LAUNCH(true, 1); else SU_LAUNCH(false, 1); }
  else { if (vec) SU_LAUNCH(true, 2); else SU_LAUNCH(false, 2); }
#undef SU_LAUNCH
  return hipGetLastError();
}

hipError_t launch_lars_p2(shard_plan_t* p, int r, float* w, const float* g, int g_source, const void* const* g_full,
                          float* m, void* w16, const LarsK& k, const float* sums, hipStream_t stream) {
  if (p->chunks.empty()) return hipSuccess;
  ProfScope ps(p, SHARD_K_LARS_P2, stream);
  const dim3 grid((unsigned)p->chunks.size());
  const VarDesc* vars = ws_at<VarDesc>(p, p->ws.vars);
  const ChunkDesc* chunks = ws_at<ChunkDesc>(p, p->ws.chunks);
  const bool vec = p->align % 4 == 0;
  uint16_t* o = (uint16_t*)w16;
  const unsigned lds = p->S >= kLargeShard ? kLdsLarsP2Large : kLdsLarsP2;
#define SU_LAUNCH(VEC, BF16, GS)                                                                                     \
  hipLaunchKernelGGL((lars_p2_kernel<VEC, BF16, GS>), grid, dim3(kUpdBlock), lds, stream, vars, chunks, w, g, g_full, m, o, \
                     sums, r, k)
#define SU_LAUNCH_GS(GS)                     \
  do {                                       \
    if (vec && o) SU_LAUNCH(true, true, GS);   \
    else if (vec) SU_LAUNCH(true, false, GS);  \
    else if (o) SU_LAUNCH(false, true, GS);    \
    else SU_LAUNCH(false, false, GS);          \
  } while (0)
  if (g_source == 0) SU_LAUNCH_GS(0);
  else if (g_source == 1) SU_LAUNCH_GS(1);
  else SU_LAUNCH_GS(2);
#undef SU_LAUNCH
  return hipGetLastError();
}

hipError_t launch_adam_full_grads(shard_plan_t* p, int r, float* w, int g_source, const void* const* g_full, float* m,
                                  float* v, void* w16, const AdamK& k, hipStream_t stream) {
  if (p->chunks.empty()) return hipSuccess;
  ProfScope ps(p, SHARD_K_ADAM, stream);
  const dim3 grid((unsigned)p->chunks.size());
  const VarDesc* vars = ws_at<VarDesc>(p, p->ws.vars);
  const ChunkDesc* chunks = ws_at<ChunkDesc>(p, p->ws.chunks);
  const bool vec = p->align % 4 == 0;
  uint16_t* o = (uint16_t*)w16;
#define SU_LAUNCH(VEC, BF16, GS)                                                                                       \
  hipLaunchKernelGGL((adam_chunk_kernel<VEC, BF16, GS>), grid, dim3(kUpdBlock), kLdsAdamChunk, stream, vars, chunks, w, g_full, m, v, \
                     o, r, k)
  if (g_source == 1) SU_LAUNCH_GS(1);
  else SU_LAUNCH_GS(2);
#undef SU_LAUNCH
  return hipGetLastError();
}

hipError_t launch_momentum_full_grads(shard_plan_t* p, int r, float* w, int g_source, const void* const* g_full,
                                      float* m, void* w16, const MomentumK& k, hipStream_t stream) {
  if (p->chunks.empty()) return hipSuccess;
  ProfScope ps(p, SHARD_K_MOMENTUM, stream);
  const dim3 grid((unsigned)p->chunks.size());
  const VarDesc* vars = ws_at<VarDesc>(p, p->ws.vars);
  const ChunkDesc* chunks = ws_at<ChunkDesc>(p, p->ws.chunks);
  const bool vec = p->align % 4 == 0;
  uint16_t* o = (uint16_t*)w16;
#define SU_LAUNCH(VEC, BF16, GS)                                                                                        \
  hipLaunchKernelGGL((momentum_chunk_kernel<VEC, BF16, GS>), grid, dim3(kUpdBlock), kLdsMomentumChunk, stream, vars, chunks, w, g_full, m, \
                     o, r, k)
  if (g_source == 1) SU_LAUNCH_GS(1);
  else SU_LAUNCH_GS(2);
#undef SU_LAUNCH
#undef SU_LAUNCH_GS
  return hipGetLastError();
}

// ---- the sums of a LAMB step in memory the library owns (shard_update_lamb_noalloc) ------------------
// One array per GPU, part of the loaded code object, for callers that cannot bring a buffer for the chunk sums
// and the per-variable sums.  In host code the array's name is only a handle for hipGetSymbolAddress; the
// address the kernels get is resolved once per device and kept.
namespace {
static __device__ __align__(256) float scratch[2 * (SHARD_NOALLOC_MAX_CHUNKS + SHARD_NOALLOC_MAX_VARS)];
constexpr int kMaxDevices = 64;
std::mutex scratch_mutex;
float* scratch_ptr[kMaxDevices] = {};
}  // namespace

hipError_t static_lamb_scratch(float** chunk_sums, float** var_sums) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(scratch_mutex);
  if (scratch_ptr[dev] == nullptr) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));       // this device's copy of the array
    if (e != hipSuccess) return e;
    if (ptr == nullptr) return hipErrorInvalidSymbol;
    scratch_ptr[dev] = static_cast<float*>(ptr);
  }
  *chunk_sums = scratch_ptr[dev];
  *var_sums = scratch_ptr[dev] + 2 * (size_t)SHARD_NOALLOC_MAX_CHUNKS;
  return hipSuccess;
}

}  // namespace su
