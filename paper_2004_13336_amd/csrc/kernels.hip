// HIP kernels for gfx950 (MI355X) and their launchers.
//
// Everything here is bound by HBM bandwidth (Section 2.2: the weight update reads the gradient,
// the weight and the auxiliary variables and writes the weight and the auxiliaries back; the
// arithmetic in between is a handful of element-wise operations).  The kernels therefore do
// nothing clever with the arithmetic and everything they can for the memory system:
//   * every lane moves 128 bits per access, a 64-lane wavefront covers 1 KiB of one stream;
//   * each thread issues all the loads of its tile (kUnroll accesses per stream) before the
//     first dependent instruction, so a workgroup keeps tens of KiB in flight;
//   * one launch covers a whole shard: variables are addressed through a chunk table, so
//     hundreds of small variables cost no launches of their own (the single-GPU analogue of
//     the paper's batching of small tensors, Section 5.2);
//   * the per-variable sums of squares are reduced with wavefront shuffles and LDS, in a fixed
//     order, without atomics.
// The file is compiled with -ffp-contract=off: fused multiply-adds appear only where fmaf() is
// written, so every kernel (vector path, scalar path, sharded or not) performs bit-identical
// arithmetic per element.
#include "internal.hpp"

#ifndef SU_UNROLL
#define SU_UNROLL 4        // 128-bit accesses per thread per stream in flight
#endif
#ifndef SU_NT_LOAD
#define SU_NT_LOAD 0       // 1: mark streaming loads non-temporal
#endif
#ifndef SU_NT_STORE
#define SU_NT_STORE 0      // 1: mark streaming stores non-temporal
#endif
#ifndef SU_GRID_CAP
#define SU_GRID_CAP 0      // >0: flat kernels launch at most this many workgroups and loop
#endif

namespace su {
namespace {

typedef float f4 __attribute__((ext_vector_type(4)));
typedef uint32_t u4 __attribute__((ext_vector_type(4)));
typedef uint32_t u2 __attribute__((ext_vector_type(2)));

constexpr int kUnroll = SU_UNROLL;

// Four consecutive floats held in registers; moved with one 128-bit access.
struct F4 {
  float x, y, z, w;
};

template <typename T>
__device__ __forceinline__ T ld(const T* p) {
#if SU_NT_LOAD
  return __builtin_nontemporal_load(p);
#else
  return *p;
#endif
}
template <typename T>
__device__ __forceinline__ void st(T* p, T x) {
#if SU_NT_STORE
  __builtin_nontemporal_store(x, p);
#else
  *p = x;
#endif
}

__device__ __forceinline__ F4 ld4(const float* p) {
  const f4 t = ld((const f4*)p);
  return F4{t.x, t.y, t.z, t.w};
}
__device__ __forceinline__ void st4(float* p, const F4& a) {
  f4 t;
  t.x = a.x; t.y = a.y; t.z = a.z; t.w = a.w;
  st((f4*)p, t);
}

// ---- bfloat16 ---------------------------------------------------------------------------------
// Round to nearest, ties to even, on the bit pattern; NaN keeps sign and upper payload and gets
// the quiet bit.
__device__ __forceinline__ uint32_t bf16_from_f32_bits(uint32_t b) {
  const uint32_t rounded = (b + 0x7FFFu + ((b >> 16) & 1u)) >> 16;
  const uint32_t quiet = (b >> 16) | 0x0040u;
  return ((b & 0x7FFFFFFFu) > 0x7F800000u) ? quiet : rounded;
}
__device__ __forceinline__ uint32_t bf16_of(float x) { return bf16_from_f32_bits(__float_as_uint(x)); }

// ---- pieces shared by the table-driven kernels ----------------------------------------------------

struct ChunkView {
  int var;
  int len;          // slots in this chunk
  int valid;        // leading slots that hold real elements on replica r (Section 4.1: position
                    // in the full variable = replica offset + index, compared with its length)
  int64_t shard0;   // offset of the chunk inside a packed shard
  int64_t flat0;    // offset of the chunk inside the flat variable
  uint32_t flags;
};

__device__ __forceinline__ ChunkView chunk_view(const VarDesc* __restrict__ vars, const ChunkDesc* __restrict__ chunks,
                                                int c, int r) {
  const ChunkDesc cd = chunks[c];
  const VarDesc vd = vars[cd.var];
  ChunkView cv;
  cv.var = cd.var;
  cv.len = cd.len;
  cv.flat0 = (int64_t)r * vd.L + cd.k0;
  const int64_t rem = vd.n - cv.flat0;
  cv.valid = rem <= 0 ? 0 : (rem < (int64_t)cd.len ? (int)rem : cd.len);
  cv.shard0 = vd.off + cd.k0;
  cv.flags = vd.flags;
  return cv;
}

// Sum over the workgroup of two per-thread values, in a fixed order; the result is valid in
// thread 0.  Wavefront step: xor shuffles; cross-wavefront step: LDS.
__device__ __forceinline__ void block_sum2(float& a, float& b) {
  __shared__ float part[2 * (kBlock / 64)];
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
    for (int w = 1; w < kBlock / 64; ++w) {
      x += part[2 * w];
      y += part[2 * w + 1];
    }
    a = x;
    b = y;
  }
}

// ---- pointer table --------------------------------------------------------------------------------
// Device pointer tables are written by a kernel that carries the pointers as launch arguments:
// stream-ordered, no host staging buffer whose lifetime would have to be tracked.
__global__ __launch_bounds__(kPtrBatch) void ptr_table_kernel(PtrBatch b, const void** dst, int count) {
  const int i = threadIdx.x;
  if (i < count) dst[i] = b.p[i];
}

// ---- shard_format / unshard_format ----------------------------------------------------------------
// A unit is 8 elements: two 128-bit accesses of float32 or one of bfloat16.

template <int DT> struct ElemOf;
template <> struct ElemOf<SHARD_F32> { typedef uint32_t type; };
template <> struct ElemOf<SHARD_BF16> { typedef uint16_t type; };

template <int DT>
__device__ __forceinline__ void load8(const typename ElemOf<DT>::type* p, uint32_t (&x)[8]) {
  if constexpr (DT == SHARD_F32) {
    const u4 a = ld((const u4*)p), b = ld((const u4*)p + 1);
    x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w; x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
  } else {
    const u4 a = ld((const u4*)p);
    x[0] = a.x & 0xFFFFu; x[1] = a.x >> 16; x[2] = a.y & 0xFFFFu; x[3] = a.y >> 16;
    x[4] = a.z & 0xFFFFu; x[5] = a.z >> 16; x[6] = a.w & 0xFFFFu; x[7] = a.w >> 16;
  }
}
template <int DT>
__device__ __forceinline__ void store8(typename ElemOf<DT>::type* p, const uint32_t (&x)[8]) {
  if constexpr (DT == SHARD_F32) {
    u4 a, b;
    a.x = x[0]; a.y = x[1]; a.z = x[2]; a.w = x[3]; b.x = x[4]; b.y = x[5]; b.z = x[6]; b.w = x[7];
    st((u4*)p, a);
    st((u4*)p + 1, b);
  } else {
    u4 a;
    a.x = x[0] | (x[1] << 16); a.y = x[2] | (x[3] << 16); a.z = x[4] | (x[5] << 16); a.w = x[6] | (x[7] << 16);
    st((u4*)p, a);
  }
}
template <int SRC, int DST>
__device__ __forceinline__ uint32_t convert(uint32_t b) {
  if constexpr (SRC == DST) return b;
  else if constexpr (SRC == SHARD_F32) return bf16_from_f32_bits(b);
  else return b << 16;
}

// One workgroup per chunk.  VEC: pieces and tensors are 16-byte aligned and len % 8 == 0.
template <int SRC, int DST, bool VEC>
__global__ __launch_bounds__(kBlock) void format_kernel(const VarDesc* __restrict__ vars,
                                                        const ChunkDesc* __restrict__ chunks,
                                                        const void* const* __restrict__ ptrs, void* out, int r0,
                                                        int64_t S, int n_chunks) {
  typedef typename ElemOf<SRC>::type SrcT;
  typedef typename ElemOf<DST>::type DstT;
  // blockIdx.y walks replicas for the all-replica form; r0 is the single replica otherwise
  const int r = r0 + blockIdx.y;
  const ChunkView cv = chunk_view(vars, chunks, blockIdx.x, r);
  const SrcT* src = (const SrcT*)ptrs[cv.var] + cv.flat0;      // never dereferenced when valid == 0
  DstT* dst = (DstT*)out + (int64_t)blockIdx.y * S + cv.shard0;
  (void)n_chunks;
  if constexpr (VEC) {
    const int units = cv.len >> 3;
    for (int u0 = threadIdx.x; u0 < units; u0 += kBlock * kUnroll) {
      uint32_t x[kUnroll][8];
#pragma unroll
      for (int k = 0; k < kUnroll; ++k) {
        const int e = (u0 + k * kBlock) << 3;
        if (e + 8 <= cv.valid) {
          load8<SRC>(src + e, x[k]);
        } else if (e < cv.len) {
#pragma unroll
          for (int j = 0; j < 8; ++j) x[k][j] = (e + j < cv.valid) ? (uint32_t)src[e + j] : 0u;
        }
      }
#pragma unroll
      for (int k = 0; k < kUnroll; ++k) {
        const int e = (u0 + k * kBlock) << 3;
        if (e < cv.len) {
#pragma unroll
          for (int j = 0; j < 8; ++j) x[k][j] = convert<SRC, DST>(x[k][j]);
          store8<DST>(dst + e, x[k]);
        }
      }
    }
  } else {
    for (int e = threadIdx.x; e < cv.len; e += kBlock)
      dst[e] = (DstT)((e < cv.valid) ? convert<SRC, DST>((uint32_t)src[e]) : 0u);
  }
}

// One workgroup per (chunk, replica): copies the real elements of gathered[r][chunk] back into
// the flat variable and drops the padding.
template <int SRC, int DST, bool VEC>
__global__ __launch_bounds__(kBlock) void unshard_kernel(const VarDesc* __restrict__ vars,
                                                         const ChunkDesc* __restrict__ chunks,
                                                         void* const* __restrict__ ptrs, const void* gathered,
                                                         int64_t S) {
  typedef typename ElemOf<SRC>::type SrcT;
  typedef typename ElemOf<DST>::type DstT;
  const int r = blockIdx.y;
  const ChunkView cv = chunk_view(vars, chunks, blockIdx.x, r);
  if (cv.valid == 0) return;
  const SrcT* src = (const SrcT*)gathered + (int64_t)r * S + cv.shard0;
  DstT* dst = (DstT*)ptrs[cv.var] + cv.flat0;
  if constexpr (VEC) {
    const int units = (cv.valid + 7) >> 3;
    for (int u0 = threadIdx.x; u0 < units; u0 += kBlock * kUnroll) {
      uint32_t x[kUnroll][8];
#pragma unroll
      for (int k = 0; k < kUnroll; ++k) {
        const int e = (u0 + k * kBlock) << 3;
        if (e < cv.valid) load8<SRC>(src + e, x[k]);          // the piece itself is always whole in the shard
      }
#pragma unroll
      for (int k = 0; k < kUnroll; ++k) {
        const int e = (u0 + k * kBlock) << 3;
        if (e + 8 <= cv.valid) {
#pragma unroll
          for (int j = 0; j < 8; ++j) x[k][j] = convert<SRC, DST>(x[k][j]);
          store8<DST>(dst + e, x[k]);
        } else if (e < cv.valid) {
#pragma unroll
          for (int j = 0; j < 8; ++j)
            if (e + j < cv.valid) dst[e + j] = (DstT)convert<SRC, DST>(x[k][j]);
        }
      }
    }
  } else {
    for (int e = threadIdx.x; e < cv.valid; e += kBlock) dst[e] = (DstT)convert<SRC, DST>((uint32_t)src[e]);
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

__device__ __forceinline__ void store_bf16x4(uint16_t* p, const F4& w) {
  u2 o;
  o.x = bf16_of(w.x) | (bf16_of(w.y) << 16);
  o.y = bf16_of(w.z) | (bf16_of(w.w) << 16);
  st((u2*)p, o);
}

// ---- flat kernels: Adam and momentum ---------------------------------------------------------------
// Padded slots are a fixed point of both updates (0 in, +0.0 out), so the packed shard is
// processed as one flat array: no table, no masks.

template <bool BF16>
__global__ __launch_bounds__(kBlock) void adam_kernel(float* w, const float* __restrict__ g, float* m, float* v,
                                                      uint16_t* __restrict__ w16, int64_t n4, int tail, AdamK k) {
  const int64_t tile = (int64_t)kBlock * kUnroll;
  const int64_t tiles = (n4 + tile - 1) / tile;
  for (int64_t t = blockIdx.x; t < tiles; t += gridDim.x) {
    const int64_t u0 = t * tile + threadIdx.x;
    F4 rw[kUnroll], rg[kUnroll], rm[kUnroll], rv[kUnroll];
#pragma unroll
    for (int i = 0; i < kUnroll; ++i) {
      const int64_t u = u0 + (int64_t)i * kBlock;
      if (u < n4) {
        rg[i] = ld4(g + 4 * u);
        rw[i] = ld4(w + 4 * u);
        rm[i] = ld4(m + 4 * u);
        rv[i] = ld4(v + 4 * u);
      }
    }
#pragma unroll
    for (int i = 0; i < kUnroll; ++i) {
      const int64_t u = u0 + (int64_t)i * kBlock;
      if (u < n4) {
        adam_elem(rw[i].x, rg[i].x, rm[i].x, rv[i].x, k);
        adam_elem(rw[i].y, rg[i].y, rm[i].y, rv[i].y, k);
        adam_elem(rw[i].z, rg[i].z, rm[i].z, rv[i].z, k);
        adam_elem(rw[i].w, rg[i].w, rm[i].w, rv[i].w, k);
        st4(w + 4 * u, rw[i]);
        st4(m + 4 * u, rm[i]);
        st4(v + 4 * u, rv[i]);
        if constexpr (BF16) store_bf16x4(w16 + 4 * u, rw[i]);
      }
    }
  }
  if (blockIdx.x == 0 && (int)threadIdx.x < tail) {        // S % 4 leftover elements (align < 4 only)
    const int64_t e = 4 * n4 + threadIdx.x;
    float ww = w[e], mm = m[e], vv = v[e];
    adam_elem(ww, g[e], mm, vv, k);
    w[e] = ww; m[e] = mm; v[e] = vv;
    if constexpr (BF16) w16[e] = (uint16_t)bf16_of(ww);
  }
}

template <bool BF16>
__global__ __launch_bounds__(kBlock) void momentum_kernel(float* w, const float* __restrict__ g, float* m,
                                                          uint16_t* __restrict__ w16, int64_t n4, int tail,
                                                          MomentumK k) {
  const int64_t tile = (int64_t)kBlock * kUnroll;
  const int64_t tiles = (n4 + tile - 1) / tile;
  for (int64_t t = blockIdx.x; t < tiles; t += gridDim.x) {
    const int64_t u0 = t * tile + threadIdx.x;
    F4 rw[kUnroll], rg[kUnroll], rm[kUnroll];
#pragma unroll
    for (int i = 0; i < kUnroll; ++i) {
      const int64_t u = u0 + (int64_t)i * kBlock;
      if (u < n4) {
        rg[i] = ld4(g + 4 * u);
        rw[i] = ld4(w + 4 * u);
        rm[i] = ld4(m + 4 * u);
      }
    }
#pragma unroll
    for (int i = 0; i < kUnroll; ++i) {
      const int64_t u = u0 + (int64_t)i * kBlock;
      if (u < n4) {
        momentum_elem(rw[i].x, rg[i].x, rm[i].x, k);
        momentum_elem(rw[i].y, rg[i].y, rm[i].y, k);
        momentum_elem(rw[i].z, rg[i].z, rm[i].z, k);
        momentum_elem(rw[i].w, rg[i].w, rm[i].w, k);
        st4(w + 4 * u, rw[i]);
        st4(m + 4 * u, rm[i]);
        if constexpr (BF16) store_bf16x4(w16 + 4 * u, rw[i]);
      }
    }
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

template <bool VEC>
__global__ __launch_bounds__(kBlock) void lamb_p1_kernel(const VarDesc* __restrict__ vars,
                                                         const ChunkDesc* __restrict__ chunks,
                                                         const float* __restrict__ w, const float* __restrict__ g,
                                                         float* m, float* v, float* __restrict__ chunk_sums, int r,
                                                         AdamK k) {
  const ChunkView cv = chunk_view(vars, chunks, blockIdx.x, r);
  const float wd = (cv.flags & SHARD_VAR_NO_DECAY) ? 0.0f : k.wd;
  float sw = 0.0f, su = 0.0f;
  if constexpr (VEC) {
    const float* w4 = w + cv.shard0;
    const float* g4 = g + cv.shard0;
    float* m4 = m + cv.shard0;
    float* v4 = v + cv.shard0;
    const int units = cv.len >> 2;
    for (int u0 = threadIdx.x; u0 < units; u0 += kBlock * kUnroll) {
      F4 rw[kUnroll], rg[kUnroll], rm[kUnroll], rv[kUnroll];
#pragma unroll
      for (int i = 0; i < kUnroll; ++i) {
        const int u = u0 + i * kBlock;
        if (u < units) {
          rg[i] = ld4(g4 + 4 * u);
          rw[i] = ld4(w4 + 4 * u);
          rm[i] = ld4(m4 + 4 * u);
          rv[i] = ld4(v4 + 4 * u);
        }
      }
#pragma unroll
      for (int i = 0; i < kUnroll; ++i) {
        const int u = u0 + i * kBlock;
        if (u < units) {
          const int e = u << 2;
          float d;
#define SU_LAMB_P1_LANE(c, j)                                  \
  lamb_moments(rg[i].c, rm[i].c, rv[i].c, k);                  \
  d = lamb_dir(rw[i].c, rm[i].c, rv[i].c, wd, k);              \
  if (e + j < cv.valid) {                                      \
    sw = fmaf(rw[i].c, rw[i].c, sw);                           \
    su = fmaf(d, d, su);                                       \
  }
          SU_LAMB_P1_LANE(x, 0)
          SU_LAMB_P1_LANE(y, 1)
          SU_LAMB_P1_LANE(z, 2)
          SU_LAMB_P1_LANE(w, 3)
#undef SU_LAMB_P1_LANE
          st4(m4 + 4 * u, rm[i]);
          st4(v4 + 4 * u, rv[i]);
        }
      }
    }
  } else {
    for (int e = threadIdx.x; e < cv.len; e += kBlock) {
      const int64_t s = cv.shard0 + e;
      float mm = m[s], vv = v[s];
      const float ww = w[s];
      lamb_moments(g[s], mm, vv, k);
      const float d = lamb_dir(ww, mm, vv, wd, k);
      if (e < cv.valid) {
        sw = fmaf(ww, ww, sw);
        su = fmaf(d, d, su);
      }
      m[s] = mm;
      v[s] = vv;
    }
  }
  block_sum2(sw, su);
  if (threadIdx.x == 0) {
    chunk_sums[2 * blockIdx.x] = sw;
    chunk_sums[2 * blockIdx.x + 1] = su;
  }
}

// One wavefront per variable: adds the variable's chunk sums in a fixed order (float64
// accumulators), optionally adds the other replicas' table (the all-reduce stand-in).
__global__ __launch_bounds__(kBlock) void norm_reduce_kernel(const VarDesc* __restrict__ vars,
                                                             const float* __restrict__ chunk_sums, int V,
                                                             const float* __restrict__ other, float* sums_out,
                                                             float* local_out) {
  const int i = (blockIdx.x * kBlock + threadIdx.x) >> 6;    // uniform per wavefront
  if (i >= V) return;
  const int lane = threadIdx.x & 63;
  const VarDesc vd = vars[i];
  double a = 0.0, b = 0.0;
  for (int c = lane; c < vd.n_chunks; c += 64) {
    a += (double)chunk_sums[2 * (int64_t)(vd.first_chunk + c)];
    b += (double)chunk_sums[2 * (int64_t)(vd.first_chunk + c) + 1];
  }
#pragma unroll
  for (int s = 32; s >= 1; s >>= 1) {
    a += __shfl_xor(a, s, 64);
    b += __shfl_xor(b, s, 64);
  }
  if (lane == 0) {
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
template <bool VEC, bool BF16>
__global__ __launch_bounds__(kBlock) void lamb_p2_kernel(const VarDesc* __restrict__ vars,
                                                         const ChunkDesc* __restrict__ chunks, float* w,
                                                         const float* __restrict__ m, const float* __restrict__ v,
                                                         uint16_t* __restrict__ w16, const float* __restrict__ sums,
                                                         AdamK k) {
  const ChunkView cv = chunk_view(vars, chunks, blockIdx.x, 0);
  const float wd = (cv.flags & SHARD_VAR_NO_DECAY) ? 0.0f : k.wd;
  float ratio = 1.0f;
  if (!(cv.flags & SHARD_VAR_NO_ADAPT)) {
    const float wn = sqrtf(sums[2 * cv.var]), un = sqrtf(sums[2 * cv.var + 1]);
    if (wn > 0.0f && un > 0.0f) ratio = wn / un;
  }
  const float step = k.lr * ratio;
  if constexpr (VEC) {
    float* w4 = w + cv.shard0;
    const float* m4 = m + cv.shard0;
    const float* v4 = v + cv.shard0;
    const int units = cv.len >> 2;
    for (int u0 = threadIdx.x; u0 < units; u0 += kBlock * kUnroll) {
      F4 rw[kUnroll], rm[kUnroll], rv[kUnroll];
#pragma unroll
      for (int i = 0; i < kUnroll; ++i) {
        const int u = u0 + i * kBlock;
        if (u < units) {
          rw[i] = ld4(w4 + 4 * u);
          rm[i] = ld4(m4 + 4 * u);
          rv[i] = ld4(v4 + 4 * u);
        }
      }
#pragma unroll
      for (int i = 0; i < kUnroll; ++i) {
        const int u = u0 + i * kBlock;
        if (u < units) {
          rw[i].x = fmaf(-step, lamb_dir(rw[i].x, rm[i].x, rv[i].x, wd, k), rw[i].x);
          rw[i].y = fmaf(-step, lamb_dir(rw[i].y, rm[i].y, rv[i].y, wd, k), rw[i].y);
          rw[i].z = fmaf(-step, lamb_dir(rw[i].z, rm[i].z, rv[i].z, wd, k), rw[i].z);
          rw[i].w = fmaf(-step, lamb_dir(rw[i].w, rm[i].w, rv[i].w, wd, k), rw[i].w);
          st4(w4 + 4 * u, rw[i]);
          if constexpr (BF16) store_bf16x4(w16 + cv.shard0 + 4 * u, rw[i]);
        }
      }
    }
  } else {
    for (int e = threadIdx.x; e < cv.len; e += kBlock) {
      const int64_t s = cv.shard0 + e;
      const float ww = w[s];
      const float nw = fmaf(-step, lamb_dir(ww, m[s], v[s], wd, k), ww);
      w[s] = nw;
      if constexpr (BF16) w16[s] = (uint16_t)bf16_of(nw);
    }
  }
}

inline unsigned flat_grid(int64_t n4) {
  const int64_t tile = (int64_t)kBlock * kUnroll;
  int64_t tiles = (n4 + tile - 1) / tile;
  if (tiles < 1) tiles = 1;
#if SU_GRID_CAP > 0
  if (tiles > SU_GRID_CAP) tiles = SU_GRID_CAP;
#endif
  if (tiles > 0x7FFFFFFF) tiles = 0x7FFFFFFF;
  return (unsigned)tiles;
}

template <typename T>
inline T* ws_at(const shard_plan_t* p, size_t off) {
  return reinterpret_cast<T*>(p->ws.base + off);
}

}  // namespace

// ---- profiling scope -------------------------------------------------------------------------------

ProfScope::ProfScope(shard_plan_t* plan, int kernel, hipStream_t s) : p(plan), stream(s), on(plan->prof) {
  if (!on) return;
  if (!p->prof_free.empty()) {
    rec = p->prof_free.back();
    p->prof_free.pop_back();
  } else if (hipEventCreate(&rec.start) != hipSuccess || hipEventCreate(&rec.stop) != hipSuccess) {
    on = false;
    return;
  }
  rec.kernel = kernel;
  (void)hipEventRecord(rec.start, stream);
}

ProfScope::~ProfScope() {
  if (!on) return;
  (void)hipEventRecord(rec.stop, stream);
  p->prof_live.push_back(rec);
}

// ---- launchers -------------------------------------------------------------------------------------

hipError_t launch_ptr_table(shard_plan_t* p, const void* const* host_ptrs, const void** dev_table, hipStream_t stream) {
  ProfScope ps(p, SHARD_K_PTR_TABLE, stream);
  for (int base = 0; base < p->V; base += kPtrBatch) {
    PtrBatch b;
    const int count = (p->V - base < kPtrBatch) ? (p->V - base) : kPtrBatch;
    for (int i = 0; i < kPtrBatch; ++i) b.p[i] = (i < count) ? host_ptrs[base + i] : nullptr;
    hipLaunchKernelGGL(ptr_table_kernel, dim3(1), dim3(kPtrBatch), 0, stream, b, dev_table + base, count);
  }
  return hipGetLastError();
}

namespace {
template <int SRC, int DST>
void format_dispatch(shard_plan_t* p, int r, int replicas, const void* const* tab, void* out, bool vec,
                     hipStream_t stream) {
  const dim3 grid((unsigned)p->chunks.size(), (unsigned)replicas);
  const VarDesc* vars = ws_at<VarDesc>(p, p->ws.vars);
  const ChunkDesc* chunks = ws_at<ChunkDesc>(p, p->ws.chunks);
  if (vec)
    hipLaunchKernelGGL((format_kernel<SRC, DST, true>), grid, dim3(kBlock), 0, stream, vars, chunks, tab, out, r, p->S,
                       (int)p->chunks.size());
  else
    hipLaunchKernelGGL((format_kernel<SRC, DST, false>), grid, dim3(kBlock), 0, stream, vars, chunks, tab, out, r,
                       p->S, (int)p->chunks.size());
}
template <int SRC, int DST>
void unshard_dispatch(shard_plan_t* p, const void* gathered, void* const* tab, bool vec, hipStream_t stream) {
  const dim3 grid((unsigned)p->chunks.size(), (unsigned)p->N);
  const VarDesc* vars = ws_at<VarDesc>(p, p->ws.vars);
  const ChunkDesc* chunks = ws_at<ChunkDesc>(p, p->ws.chunks);
  if (vec)
    hipLaunchKernelGGL((unshard_kernel<SRC, DST, true>), grid, dim3(kBlock), 0, stream, vars, chunks, tab, gathered,
                       p->S);
  else
    hipLaunchKernelGGL((unshard_kernel<SRC, DST, false>), grid, dim3(kBlock), 0, stream, vars, chunks, tab, gathered,
                       p->S);
}
}  // namespace

hipError_t launch_format(shard_plan_t* p, int r, const void* const* tab, int src_dtype, void* out, int dst_dtype,
                         bool vec, hipStream_t stream) {
  if (p->chunks.empty()) return hipSuccess;
  ProfScope ps(p, SHARD_K_FORMAT, stream);
  if (src_dtype == SHARD_F32 && dst_dtype == SHARD_F32) format_dispatch<SHARD_F32, SHARD_F32>(p, r, 1, tab, out, vec, stream);
  else if (src_dtype == SHARD_F32) format_dispatch<SHARD_F32, SHARD_BF16>(p, r, 1, tab, out, vec, stream);
  else if (dst_dtype == SHARD_F32) format_dispatch<SHARD_BF16, SHARD_F32>(p, r, 1, tab, out, vec, stream);
  else format_dispatch<SHARD_BF16, SHARD_BF16>(p, r, 1, tab, out, vec, stream);
  return hipGetLastError();
}

hipError_t launch_unshard(shard_plan_t* p, const void* gathered, int src_dtype, void* const* tab, int dst_dtype,
                          bool vec, hipStream_t stream) {
  if (p->chunks.empty()) return hipSuccess;
  ProfScope ps(p, SHARD_K_UNSHARD, stream);
  if (src_dtype == SHARD_F32 && dst_dtype == SHARD_F32) unshard_dispatch<SHARD_F32, SHARD_F32>(p, gathered, tab, vec, stream);
  else if (src_dtype == SHARD_F32) unshard_dispatch<SHARD_F32, SHARD_BF16>(p, gathered, tab, vec, stream);
  else if (dst_dtype == SHARD_F32) unshard_dispatch<SHARD_BF16, SHARD_F32>(p, gathered, tab, vec, stream);
  else unshard_dispatch<SHARD_BF16, SHARD_BF16>(p, gathered, tab, vec, stream);
  return hipGetLastError();
}

hipError_t launch_adam(shard_plan_t* p, float* w, const float* g, float* m, float* v, void* w16, const AdamK& k,
                       hipStream_t stream) {
  if (p->S == 0) return hipSuccess;
  ProfScope ps(p, SHARD_K_ADAM, stream);
  const int64_t n4 = p->S >> 2;
  const int tail = (int)(p->S & 3);
  if (w16)
    hipLaunchKernelGGL((adam_kernel<true>), dim3(flat_grid(n4)), dim3(kBlock), 0, stream, w, g, m, v, (uint16_t*)w16,
                       n4, tail, k);
  else
    hipLaunchKernelGGL((adam_kernel<false>), dim3(flat_grid(n4)), dim3(kBlock), 0, stream, w, g, m, v,
                       (uint16_t*)nullptr, n4, tail, k);
  return hipGetLastError();
}

hipError_t launch_momentum(shard_plan_t* p, float* w, const float* g, float* m, void* w16, const MomentumK& k,
                           hipStream_t stream) {
  if (p->S == 0) return hipSuccess;
  ProfScope ps(p, SHARD_K_MOMENTUM, stream);
  const int64_t n4 = p->S >> 2;
  const int tail = (int)(p->S & 3);
  if (w16)
    hipLaunchKernelGGL((momentum_kernel<true>), dim3(flat_grid(n4)), dim3(kBlock), 0, stream, w, g, m, (uint16_t*)w16,
                       n4, tail, k);
  else
    hipLaunchKernelGGL((momentum_kernel<false>), dim3(flat_grid(n4)), dim3(kBlock), 0, stream, w, g, m,
                       (uint16_t*)nullptr, n4, tail, k);
  return hipGetLastError();
}

hipError_t launch_lamb_p1(shard_plan_t* p, int r, const float* w, const float* g, float* m, float* v, const AdamK& k,
                          hipStream_t stream) {
  if (p->chunks.empty()) return hipSuccess;
  ProfScope ps(p, SHARD_K_LAMB_P1, stream);
  const dim3 grid((unsigned)p->chunks.size());
  const VarDesc* vars = ws_at<VarDesc>(p, p->ws.vars);
  const ChunkDesc* chunks = ws_at<ChunkDesc>(p, p->ws.chunks);
  float* cs = ws_at<float>(p, p->ws.chunk_sums);
  if (p->align % 4 == 0)
    hipLaunchKernelGGL((lamb_p1_kernel<true>), grid, dim3(kBlock), 0, stream, vars, chunks, w, g, m, v, cs, r, k);
  else
    hipLaunchKernelGGL((lamb_p1_kernel<false>), grid, dim3(kBlock), 0, stream, vars, chunks, w, g, m, v, cs, r, k);
  return hipGetLastError();
}

hipError_t launch_norm_reduce(shard_plan_t* p, const float* other, float* sums_out, float* local_out,
                              hipStream_t stream) {
  if (p->V == 0) return hipSuccess;
  ProfScope ps(p, SHARD_K_NORM_REDUCE, stream);
  const int waves_per_block = kBlock / 64;
  const dim3 grid((unsigned)((p->V + waves_per_block - 1) / waves_per_block));
  hipLaunchKernelGGL(norm_reduce_kernel, grid, dim3(kBlock), 0, stream, ws_at<VarDesc>(p, p->ws.vars),
                     ws_at<float>(p, p->ws.chunk_sums), p->V, other, sums_out, local_out);
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
  if (vec && o) hipLaunchKernelGGL((lamb_p2_kernel<true, true>), grid, dim3(kBlock), 0, stream, vars, chunks, w, m, v, o, sums, k);
  else if (vec) hipLaunchKernelGGL((lamb_p2_kernel<true, false>), grid, dim3(kBlock), 0, stream, vars, chunks, w, m, v, o, sums, k);
  else if (o) hipLaunchKernelGGL((lamb_p2_kernel<false, true>), grid, dim3(kBlock), 0, stream, vars, chunks, w, m, v, o, sums, k);
  else hipLaunchKernelGGL((lamb_p2_kernel<false, false>), grid, dim3(kBlock), 0, stream, vars, chunks, w, m, v, o, sums, k);
  return hipGetLastError();
}

}  // namespace su
