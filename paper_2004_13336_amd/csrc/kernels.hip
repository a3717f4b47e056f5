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
#include <type_traits>

#include "device_common.hpp"

#ifndef SU_UNROLL
#define SU_UNROLL 2        // chunk-table kernels: 128-bit accesses per thread per stream in flight; 2 makes a tile the
                           // default 2048-slot chunk, so that whole chunks run the branch-free path (4: phase 1 +5 %)
#endif
#ifndef SU_ADAM_UNROLL
#define SU_ADAM_UNROLL 1       // flat Adam kernel: the same (1: -2 to -5 % against 4 on shards of 12 M to 1.5 G slots)
#endif
#ifndef SU_MOMENTUM_UNROLL
#define SU_MOMENTUM_UNROLL 2   // flat momentum kernel
#endif
// Cache policy per kernel family, as a 3-bit mask: 4 = non-temporal loads of streams that are only
// read, 2 = non-temporal loads of streams the same thread writes back in place, 1 = non-temporal
// stores.  The defaults are the measured best on MI355X for each access pattern.
#ifndef SU_NT_ADAM
#define SU_NT_ADAM 3
#endif
#ifndef SU_NT_MOMENTUM
#define SU_NT_MOMENTUM 3
#endif
#ifndef SU_NT_LAMB
#define SU_NT_LAMB 6
#endif
#ifndef SU_NT_LAMB_P2
#define SU_NT_LAMB_P2 5    // phase 2 of LAMB: w is loaded through the caches and stored past them (measured on the
                           // whole step: the unshard that follows gains as much as phase 2 itself)
#endif
#ifndef SU_NT_LARS
#define SU_NT_LARS 6
#endif
#ifndef SU_NT_LARS_P2
#define SU_NT_LARS_P2 5    // phase 2 of LARS: as LAMB's (w and m loaded through the caches): 122 -> 116 us on 25.6 M slots
#endif
#ifndef SU_NT_FORMAT
#define SU_NT_FORMAT 4
#endif
#ifndef SU_NT_FORMAT_ALL
#define SU_NT_FORMAT_ALL 5    // all-replica formatting: the output goes to a collective, not to the next kernel
#endif
#ifndef SU_NT_UNSHARD
#define SU_NT_UNSHARD 5
#endif
#ifndef SU_COPY_BLOCK
#define SU_COPY_BLOCK 256     // threads per workgroup of the formatting kernels
#endif
// Units per thread of the formatting kernels, all loaded before the first store.  One replica's
// formatting (a few hundred MB, partly served by the memory-side cache) measures fastest with 2;
// the whole-model copies (unshard, all-replica formatting) with 1.
#ifndef SU_FORMAT_UNROLL
#define SU_FORMAT_UNROLL 2
#endif
#ifndef SU_UNSHARD_UNROLL
#define SU_UNSHARD_UNROLL 1
#endif
#ifndef SU_FORMAT_ALL_UNROLL
#define SU_FORMAT_ALL_UNROLL 1
#endif
#ifndef SU_P1_REVERSE
#define SU_P1_REVERSE 0        // 1: LAMB phase 1 walks the chunk table from the end
#endif
#ifndef SU_P2_REVERSE
#define SU_P2_REVERSE 1        // 1: LAMB phase 2 walks it in the opposite direction to phase 1's default
#endif
#ifndef SU_GRID_CAP
#define SU_GRID_CAP 0      // >0: flat kernels launch at most this many workgroups and loop
#endif

namespace su {
namespace {

constexpr int kUnroll = SU_UNROLL;
constexpr int kAdamUnroll = SU_ADAM_UNROLL;
constexpr int kMomentumUnroll = SU_MOMENTUM_UNROLL;
constexpr int kCopyBlock = SU_COPY_BLOCK;

typedef Policy<SU_NT_ADAM> PolAdam;
typedef Policy<SU_NT_MOMENTUM> PolMomentum;
typedef Policy<SU_NT_LAMB> PolLamb;
typedef Policy<SU_NT_LAMB_P2> PolLambP2;
typedef Policy<SU_NT_LARS> PolLars;
typedef Policy<SU_NT_LARS_P2> PolLarsP2;
typedef Policy<SU_NT_FORMAT> PolFormat;
typedef Policy<SU_NT_UNSHARD> PolUnshard;
typedef Policy<SU_NT_FORMAT_ALL> PolFormatAll;

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
  cv.flat0 = (int64_t)r * vd.stride + cd.k0;
  int64_t rem = vd.n - cv.flat0;                            // up to the end of the variable ...
  if (vd.stride - cd.k0 < rem) rem = vd.stride - cd.k0;     // ... and of the piece's real slots
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

// ---- pointer table --------------------------------------------------------------------------------
// Device pointer tables are written by a kernel that carries the pointers as launch arguments:
// stream-ordered, no host staging buffer whose lifetime would have to be tracked.
__global__ __launch_bounds__(kPtrBatch) void ptr_table_kernel(PtrBatch b, const void** dst, int count) {
  const int i = threadIdx.x;
  if (i < count) dst[i] = b.p[i];
}

// ---- shard_format / unshard_format ----------------------------------------------------------------
// A unit is what one lane moves per access: 4 elements whenever float32 is involved (one 128-bit
// access on the float32 side, 64 bits on the bfloat16 side), 8 elements for bfloat16 -> bfloat16
// (128 bits on both sides).  Consecutive lanes take consecutive units, so every wavefront access
// covers one contiguous span of memory.

template <int DT> struct ElemOf;
template <> struct ElemOf<SHARD_F32> { typedef uint32_t type; };
template <> struct ElemOf<SHARD_BF16> { typedef uint16_t type; };

template <int SRC, int DST>
struct UnitOf {
  static constexpr int n = (SRC == SHARD_BF16 && DST == SHARD_BF16) ? 8 : 4;
};

template <typename Pol, int DT, int UNIT>
__device__ __forceinline__ void load_unit(const typename ElemOf<DT>::type* p, uint32_t (&x)[UNIT]) {
  if constexpr (DT == SHARD_F32) {
    static_assert(UNIT == 4, "float32 units are 4 elements");
    const u4 a = ld<Pol::RO>((const u4*)p);
    x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w;
  } else if constexpr (UNIT == 8) {
    const u4 a = ld<Pol::RO>((const u4*)p);
    x[0] = a.x & 0xFFFFu; x[1] = a.x >> 16; x[2] = a.y & 0xFFFFu; x[3] = a.y >> 16;
    x[4] = a.z & 0xFFFFu; x[5] = a.z >> 16; x[6] = a.w & 0xFFFFu; x[7] = a.w >> 16;
  } else {
    const u2 a = ld<Pol::RO>((const u2*)p);
    x[0] = a.x & 0xFFFFu; x[1] = a.x >> 16; x[2] = a.y & 0xFFFFu; x[3] = a.y >> 16;
  }
}
template <typename Pol, int DT, int UNIT>
__device__ __forceinline__ void store_unit(typename ElemOf<DT>::type* p, const uint32_t (&x)[UNIT]) {
  if constexpr (DT == SHARD_F32) {
    static_assert(UNIT == 4, "float32 units are 4 elements");
    u4 a;
    a.x = x[0]; a.y = x[1]; a.z = x[2]; a.w = x[3];
    st<Pol::ST>((u4*)p, a);
  } else if constexpr (UNIT == 8) {
    u4 a;
    a.x = x[0] | (x[1] << 16); a.y = x[2] | (x[3] << 16); a.z = x[4] | (x[5] << 16); a.w = x[6] | (x[7] << 16);
    st<Pol::ST>((u4*)p, a);
  } else {
    u2 a;
    a.x = x[0] | (x[1] << 16); a.y = x[2] | (x[3] << 16);
    st<Pol::ST>((u2*)p, a);
  }
}
template <int SRC, int DST>
__device__ __forceinline__ uint32_t convert(uint32_t b) {
  if constexpr (SRC == DST) return b;
  else if constexpr (SRC == SHARD_F32) return bf16_from_f32_bits(b);
  else return b << 16;
}

// Work items of the formatting kernels are (replica, chunk, tile) triples: a chunk is cut into
// tiles of kCopyBlock * U units (U per thread) and every tile is one short-lived workgroup.  Many small workgroups,
// dispatched in address order, keep the set of DRAM pages in flight compact, which measures
// faster on MI355X than fewer workgroups that each loop over more data.  The table look-ups
// (chunk -> variable -> pointer) of the tiles of one chunk hit the same cache lines.
// VEC: pieces (and gathered rows) are 16-byte aligned and every chunk length is a multiple of 8;
// whether a variable's full tensor is aligned too is tested per item.

// One tile of a copy: consecutive lanes on consecutive units.
// ALL: every unit of the tile holds real elements only; the tile moves without a branch.
// Otherwise units that end at or before `whole` are moved whole, and (shard_format only) units
// that start at or after `zero_from` and before `len` are written as zeros.  The one unit that
// straddles the end of the variable, if any, is left to copy_tile's caller.
template <typename Pol, int SRC, int DST, int U, bool ALL, bool UNSHARD>
__device__ __forceinline__ void copy_units(const typename ElemOf<SRC>::type* src, typename ElemOf<DST>::type* dst,
                                           int whole, int zero_from, int len) {
  constexpr int UNIT = UnitOf<SRC, DST>::n;
  uint32_t x[U][UNIT];
#pragma unroll
  for (int i = 0; i < U; ++i) {
    const int e = (i * kCopyBlock + (int)threadIdx.x) * UNIT;
    if (ALL || e + UNIT <= whole) load_unit<Pol, SRC, UNIT>(src + e, x[i]);
  }
#pragma unroll
  for (int i = 0; i < U; ++i) {
    const int e = (i * kCopyBlock + (int)threadIdx.x) * UNIT;
    if (ALL || e + UNIT <= whole) {
#pragma unroll
      for (int j = 0; j < UNIT; ++j) x[i][j] = convert<SRC, DST>(x[i][j]);
      store_unit<Pol, DST, UNIT>(dst + e, x[i]);
    } else if (!UNSHARD && e >= zero_from && e < len) {
#pragma unroll
      for (int j = 0; j < UNIT; ++j) x[i][j] = 0u;
      store_unit<Pol, DST, UNIT>(dst + e, x[i]);
    }
  }
}

// Moves tile `t` of a chunk.  shard_format: zero-padded piece of the flat variable -> packed shard
// (all `len` slots written).  unshard_format: the `valid` real elements of a gathered piece -> flat
// variable (padding dropped).  src and dst point at the chunk's first slot.
template <typename Pol, int SRC, int DST, int U, bool VEC, bool UNSHARD>
__device__ __forceinline__ void copy_tile(const ChunkView& cv, int t, const typename ElemOf<SRC>::type* src,
                                          typename ElemOf<DST>::type* dst) {
  typedef typename ElemOf<DST>::type DstT;
  constexpr int UNIT = UnitOf<SRC, DST>::n;
  constexpr int TILE = kCopyBlock * U * UNIT;
  const int base = t * TILE;
  if (base >= (UNSHARD ? cv.valid : cv.len)) return;
  if constexpr (VEC) {
    if (base + TILE <= cv.valid) {
      copy_units<Pol, SRC, DST, U, true, UNSHARD>(src + base, dst + base, TILE, TILE, TILE);
      return;
    }
    const int whole = cv.valid / UNIT * UNIT;                  // slots covered by fully real units
    const int zero_from = (cv.valid + UNIT - 1) / UNIT * UNIT; // first unit that is all padding
    copy_units<Pol, SRC, DST, U, false, UNSHARD>(src + base, dst + base, whole - base, zero_from - base, cv.len - base);
    // the unit that straddles the end of the variable: real elements, then (shard_format) zeros
    if (whole != cv.valid && whole >= base && whole < base + TILE && (int)threadIdx.x < UNIT) {
      const int e = whole + threadIdx.x;
      if (e < cv.valid) dst[e] = (DstT)convert<SRC, DST>((uint32_t)src[e]);
      else if (!UNSHARD) dst[e] = (DstT)0;
    }
  } else {
    const int end = (UNSHARD ? cv.valid : cv.len) < base + TILE ? (UNSHARD ? cv.valid : cv.len) : base + TILE;
    for (int e = base + threadIdx.x; e < end; e += kCopyBlock)
      dst[e] = (DstT)((e < cv.valid) ? convert<SRC, DST>((uint32_t)src[e]) : 0u);
  }
}

// UNSHARD = false: shard_format; `packed` is the output, shard r0 + replica goes to row `replica`.
// UNSHARD = true : unshard_format; `packed` is the gathered buffer, r0 = 0.
// blockIdx.x = (replica * n_chunks + chunk) * tiles_per_chunk + tile.
template <typename Pol, int SRC, int DST, int U, bool VEC, bool UNSHARD>
__device__ __forceinline__ void reformat_body(const VarDesc* __restrict__ vars, const ChunkDesc* __restrict__ chunks,
                                              const void* const* __restrict__ ptrs, void* packed, int r0,
                                              int64_t row_stride, int n_chunks, int tiles_per_chunk) {
  typedef typename ElemOf<SRC>::type SrcT;
  typedef typename ElemOf<DST>::type DstT;
  const int item = blockIdx.x / tiles_per_chunk;
  const int tile = blockIdx.x - item * tiles_per_chunk;
  const int replica = item / n_chunks;
  const ChunkView cv = chunk_view(vars, chunks, item - replica * n_chunks, r0 + replica);
  // skip the pointer look-up for tiles with nothing to do (beyond a short chunk, or all padding)
  constexpr int TILE = kCopyBlock * U * UnitOf<SRC, DST>::n;
  if (tile * TILE >= (UNSHARD ? cv.valid : cv.len)) return;
  const void* ptr = ptrs[cv.var];
  // 128-bit accesses need this chunk's place in the full tensor on a 16-byte boundary (VEC already
  // says its place in the shard is); a tensor or a row-plan piece that is not takes the
  // element-wise path, the others are unaffected
  const uintptr_t full_addr = reinterpret_cast<uintptr_t>(ptr) + (uintptr_t)cv.flat0 * sizeof(typename ElemOf<UNSHARD ? DST : SRC>::type);
  const bool vec = VEC && (full_addr & 15u) == 0;
  if constexpr (UNSHARD) {
    const SrcT* src = (const SrcT*)packed + (int64_t)replica * row_stride + cv.shard0;
    DstT* dst = (DstT*)const_cast<void*>(ptr) + cv.flat0;
    if (vec) copy_tile<Pol, SRC, DST, U, true, true>(cv, tile, src, dst);
    else copy_tile<Pol, SRC, DST, U, false, true>(cv, tile, src, dst);
  } else {
    const SrcT* src = (const SrcT*)ptr + cv.flat0;      // not dereferenced where there is no real element
    DstT* dst = (DstT*)packed + (int64_t)replica * row_stride + cv.shard0;
    if (vec) copy_tile<Pol, SRC, DST, U, true, false>(cv, tile, src, dst);
    else copy_tile<Pol, SRC, DST, U, false, false>(cv, tile, src, dst);
  }
}

// ---- whole-model copies on a flat plan, variable by variable ---------------------------------------
// unshard_format and shard_format_all move every variable between its full tensor and the N rows of
// the gathered buffer.  On a flat plan the gathered buffer holds, for variable i, an [N][L_i] view of
// the variable padded to N*L_i slots: padded slot p lives in row p / L_i at off_i + p % L_i, and
// the full tensor is the first n_i padded slots.  Work items are chunks of padded slots (FullChunk),
// cut into tiles like the items above: the full-tensor side of a tile is one contiguous span, the
// gathered side consists of runs of L_i slots.  The number of workgroups follows the model size, so
// thousands of replicas with pieces of a few slots cost no more launches' worth of work than eight.
// Units (4 or 8 slots) never straddle two pieces because L_i is a multiple of 8 on the VEC path.

// Slot `d` counted from the start of piece r0 (d < L + 16384): which piece and where in it.
__device__ __forceinline__ void locate(int64_t d, int64_t L, int64_t r0, int64_t& r, int64_t& k) {
  if (L >= (int64_t)1 << 30) {               // a tile can reach into the next piece at most
    const bool next = d >= L;
    r = r0 + (next ? 1 : 0);
    k = next ? d - L : d;
  } else {                                    // d < 2^30 + 2^14: 32-bit division
    const uint32_t q = (uint32_t)d / (uint32_t)L;
    r = r0 + q;
    k = (int64_t)((uint32_t)d - q * (uint32_t)L);
  }
}

// TO_FULL: gathered -> full tensors (unshard_format), padding dropped.
// otherwise: full tensors -> gathered rows (shard_format_all), padding written as zeros.
template <typename Pol, int SRC, int DST, int U, bool VEC, bool TO_FULL>
__device__ __forceinline__ void reformat_flat_body(const VarDesc* __restrict__ vars,
                                                   const FullChunk* __restrict__ fchunks,
                                                   const void* const* __restrict__ ptrs, void* packed,
                                                   int64_t row_stride, int tiles_per_chunk) {
  typedef typename ElemOf<SRC>::type SrcT;
  typedef typename ElemOf<DST>::type DstT;
  typedef typename ElemOf<TO_FULL ? DST : SRC>::type FullT;
  typedef typename ElemOf<TO_FULL ? SRC : DST>::type PackT;
  constexpr int UNIT = UnitOf<SRC, DST>::n;
  constexpr int TILE = kCopyBlock * U * UNIT;
  const int item = blockIdx.x / tiles_per_chunk;
  const int tile = blockIdx.x - item * tiles_per_chunk;
  const FullChunk fc = fchunks[item];
  const int base = tile * TILE;
  if (base >= fc.len) return;
  const VarDesc vd = vars[fc.var];
  const int64_t p_tile = fc.p0 + base;                       // first padded slot of the tile = flat index
  if (TO_FULL && p_tile >= vd.n) return;                     // a tile of padding: nothing to restore
  const int here = fc.len - base < TILE ? fc.len - base : TILE;
  const int64_t r0 = p_tile / vd.L;
  const int64_t k0 = p_tile - r0 * vd.L;
  const void* ptr = ptrs[fc.var];
  FullT* full = (FullT*)const_cast<void*>(ptr) + p_tile;     // not dereferenced past the variable's end
  PackT* rows = (PackT*)packed + vd.off;
  const bool vec = VEC && (reinterpret_cast<uintptr_t>(full) & 15u) == 0;
  const int64_t real = vd.n - p_tile;                        // slots of the tile that exist in the full tensor (may exceed it)
  if (vec) {
    uint32_t x[U][UNIT];
    int64_t po[U];                                           // offset of the unit in the gathered buffer, -1: none
    const bool single = k0 + here <= vd.L;                   // the whole tile lies in piece r0
#pragma unroll
    for (int i = 0; i < U; ++i) {
      const int e = (i * kCopyBlock + (int)threadIdx.x) * UNIT;
      po[i] = -1;
      if (e < here) {
        int64_t r = r0, k = k0 + e;
        if (!single) locate(k0 + e, vd.L, r0, r, k);
        po[i] = r * row_stride + k;
        if (TO_FULL) {
          if (e + UNIT <= real) load_unit<Pol, SRC, UNIT>((const SrcT*)rows + po[i], x[i]);
        } else {
          if (e + UNIT <= real) load_unit<Pol, SRC, UNIT>((const SrcT*)full + e, x[i]);
        }
      }
    }
#pragma unroll
    for (int i = 0; i < U; ++i) {
      const int e = (i * kCopyBlock + (int)threadIdx.x) * UNIT;
      if (po[i] < 0) continue;
      if (e + UNIT <= real) {
#pragma unroll
        for (int j = 0; j < UNIT; ++j) x[i][j] = convert<SRC, DST>(x[i][j]);
        if (TO_FULL) store_unit<Pol, DST, UNIT>((DstT*)full + e, x[i]);
        else store_unit<Pol, DST, UNIT>((DstT*)rows + po[i], x[i]);
      } else if (TO_FULL) {
        // the unit that straddles the end of the variable: its real slots one by one
        for (int j = 0; j < UNIT; ++j)
          if (e + j < real) ((DstT*)full)[e + j] = (DstT)convert<SRC, DST>((uint32_t)((const SrcT*)rows)[po[i] + j]);
      } else {
        // past (or across) the end of the variable: real slots, then zeros
#pragma unroll
        for (int j = 0; j < UNIT; ++j)
          x[i][j] = (e + j < real) ? convert<SRC, DST>((uint32_t)((const SrcT*)full)[e + j]) : 0u;
        store_unit<Pol, DST, UNIT>((DstT*)rows + po[i], x[i]);
      }
    }
  } else {
    for (int e = threadIdx.x; e < here; e += kCopyBlock) {
      const int64_t p = p_tile + e;
      const int64_t r = p / vd.L, k = p - r * vd.L;
      const int64_t o = r * row_stride + k;
      if (TO_FULL) {
        if (e < real) ((DstT*)full)[e] = (DstT)convert<SRC, DST>((uint32_t)((const SrcT*)rows)[o]);
      } else {
        ((DstT*)rows)[o] = (DstT)((e < real) ? convert<SRC, DST>((uint32_t)((const SrcT*)full)[e]) : 0u);
      }
    }
  }
}

template <int SRC, int DST, bool VEC>
__global__ __launch_bounds__(kCopyBlock) void unshard_flat_kernel(const VarDesc* __restrict__ vars,
                                                              const FullChunk* __restrict__ fchunks,
                                                              const void* const* __restrict__ ptrs, void* gathered,
                                                              int64_t row_stride, int tiles_per_chunk) {
  reformat_flat_body<PolUnshard, SRC, DST, SU_UNSHARD_UNROLL, VEC, true>(vars, fchunks, ptrs, gathered, row_stride, tiles_per_chunk);
}

template <int SRC, int DST, bool VEC>
__global__ __launch_bounds__(kCopyBlock) void format_all_flat_kernel(const VarDesc* __restrict__ vars,
                                                                 const FullChunk* __restrict__ fchunks,
                                                                 const void* const* __restrict__ ptrs, void* out,
                                                                 int64_t row_stride, int tiles_per_chunk) {
  reformat_flat_body<PolFormatAll, SRC, DST, SU_FORMAT_ALL_UNROLL, VEC, false>(vars, fchunks, ptrs, out, row_stride, tiles_per_chunk);
}

template <int SRC, int DST, bool VEC>
__global__ __launch_bounds__(kCopyBlock) void format_kernel(const VarDesc* __restrict__ vars,
                                                        const ChunkDesc* __restrict__ chunks,
                                                        const void* const* __restrict__ ptrs, void* out, int r0,
                                                        int64_t row_stride, int n_chunks, int tiles_per_chunk) {
  reformat_body<PolFormat, SRC, DST, SU_FORMAT_UNROLL, VEC, false>(vars, chunks, ptrs, out, r0, row_stride, n_chunks, tiles_per_chunk);
}

template <int SRC, int DST, bool VEC>
__global__ __launch_bounds__(kCopyBlock) void format_all_kernel(const VarDesc* __restrict__ vars,
                                                            const ChunkDesc* __restrict__ chunks,
                                                            const void* const* __restrict__ ptrs, void* out,
                                                            int64_t row_stride, int n_chunks, int tiles_per_chunk) {
  reformat_body<PolFormatAll, SRC, DST, SU_FORMAT_ALL_UNROLL, VEC, false>(vars, chunks, ptrs, out, 0, row_stride, n_chunks, tiles_per_chunk);
}

template <int SRC, int DST, bool VEC>
__global__ __launch_bounds__(kCopyBlock) void unshard_kernel(const VarDesc* __restrict__ vars,
                                                         const ChunkDesc* __restrict__ chunks,
                                                         const void* const* __restrict__ ptrs, void* gathered,
                                                         int64_t row_stride, int n_chunks, int tiles_per_chunk) {
  reformat_body<PolUnshard, SRC, DST, SU_UNSHARD_UNROLL, VEC, true>(vars, chunks, ptrs, gathered, 0, row_stride, n_chunks, tiles_per_chunk);
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
constexpr int kAdamTileElems = kBlock * kAdamUnroll * 4;   // float32 elements per tile and stream
constexpr int kMomentumTileElems = kBlock * kMomentumUnroll * 4;
constexpr int kTileElems = kBlock * kUnroll * 4;           // the same for the LAMB kernels

template <bool FULL, bool BF16>
__device__ __forceinline__ void adam_tile(float* w, const float* __restrict__ g, float* m, float* v,
                                          uint16_t* __restrict__ w16, int lim4, const AdamK& k) {
  // w, g, m, v, w16 point at the tile; lim4 = 128-bit units of the tile that exist (FULL: all)
  const int t4 = threadIdx.x * 4;
  F4 rw[kAdamUnroll], rg[kAdamUnroll], rm[kAdamUnroll], rv[kAdamUnroll];
#pragma unroll
  for (int i = 0; i < kAdamUnroll; ++i) {
    if (FULL || (int)threadIdx.x + i * kBlock < lim4) {
      const int o = i * kBlock * 4 + t4;
      rg[i] = ld4<PolAdam::RO>(g + o);
      rw[i] = ld4<PolAdam::RW>(w + o);
      rm[i] = ld4<PolAdam::RW>(m + o);
      rv[i] = ld4<PolAdam::RW>(v + o);
    }
  }
#pragma unroll
  for (int i = 0; i < kAdamUnroll; ++i) {
    if (FULL || (int)threadIdx.x + i * kBlock < lim4) {
      const int o = i * kBlock * 4 + t4;
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

template <bool BF16>
__global__ __launch_bounds__(kBlock) void adam_kernel(float* w, const float* __restrict__ g, float* m, float* v,
                                                      uint16_t* __restrict__ w16, int64_t n4, int tail, AdamK k) {
  const int64_t tile4 = (int64_t)kBlock * kAdamUnroll;
  const int64_t tiles = (n4 + tile4 - 1) / tile4;
  for (int64_t t = blockIdx.x; t < tiles; t += gridDim.x) {
    const int64_t e0 = t * kAdamTileElems;
    const int64_t left4 = n4 - t * tile4;
    if (left4 >= tile4)
      adam_tile<true, BF16>(w + e0, g + e0, m + e0, v + e0, w16 + e0, (int)tile4, k);
    else
      adam_tile<false, BF16>(w + e0, g + e0, m + e0, v + e0, w16 + e0, (int)left4, k);
  }
  if (blockIdx.x == 0 && (int)threadIdx.x < tail) {        // S % 4 leftover elements (align < 4 only)
    const int64_t e = 4 * n4 + threadIdx.x;
    float ww = w[e], mm = m[e], vv = v[e];
    adam_elem(ww, g[e], mm, vv, k);
    w[e] = ww; m[e] = mm; v[e] = vv;
    if constexpr (BF16) w16[e] = (uint16_t)bf16_of(ww);
  }
}

template <bool FULL, bool BF16>
__device__ __forceinline__ void momentum_tile(float* w, const float* __restrict__ g, float* m,
                                              uint16_t* __restrict__ w16, int lim4, const MomentumK& k) {
  const int t4 = threadIdx.x * 4;
  F4 rw[kMomentumUnroll], rg[kMomentumUnroll], rm[kMomentumUnroll];
#pragma unroll
  for (int i = 0; i < kMomentumUnroll; ++i) {
    if (FULL || (int)threadIdx.x + i * kBlock < lim4) {
      const int o = i * kBlock * 4 + t4;
      rg[i] = ld4<PolMomentum::RO>(g + o);
      rw[i] = ld4<PolMomentum::RW>(w + o);
      rm[i] = ld4<PolMomentum::RW>(m + o);
    }
  }
#pragma unroll
  for (int i = 0; i < kMomentumUnroll; ++i) {
    if (FULL || (int)threadIdx.x + i * kBlock < lim4) {
      const int o = i * kBlock * 4 + t4;
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

template <bool BF16>
__global__ __launch_bounds__(kBlock) void momentum_kernel(float* w, const float* __restrict__ g, float* m,
                                                          uint16_t* __restrict__ w16, int64_t n4, int tail,
                                                          MomentumK k) {
  const int64_t tile4 = (int64_t)kBlock * kMomentumUnroll;
  const int64_t tiles = (n4 + tile4 - 1) / tile4;
  for (int64_t t = blockIdx.x; t < tiles; t += gridDim.x) {
    const int64_t e0 = t * kMomentumTileElems;
    const int64_t left4 = n4 - t * tile4;
    if (left4 >= tile4)
      momentum_tile<true, BF16>(w + e0, g + e0, m + e0, w16 + e0, (int)tile4, k);
    else
      momentum_tile<false, BF16>(w + e0, g + e0, m + e0, w16 + e0, (int)left4, k);
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
template <bool FULL, int GS, bool GFAST>
__device__ __forceinline__ void lamb_p1_tile(const float* __restrict__ w, const void* __restrict__ g, float* m,
                                             float* v, int lim, int valid, float wd, const AdamK& k, float& sw,
                                             float& su) {
  const int t4 = threadIdx.x * 4;
  F4 rw[kUnroll], rg[kUnroll], rm[kUnroll], rv[kUnroll];
#pragma unroll
  for (int i = 0; i < kUnroll; ++i) {
    const int o = i * kBlock * 4 + t4;
    if (FULL || o < lim) {
      rg[i] = load_g4<GS, GFAST, PolLamb::RO>(g, o, valid);
      rw[i] = ld4<PolLamb::RO>(w + o);
      rm[i] = ld4<PolLamb::RW>(m + o);
      rv[i] = ld4<PolLamb::RW>(v + o);
    }
  }
#pragma unroll
  for (int i = 0; i < kUnroll; ++i) {
    const int o = i * kBlock * 4 + t4;
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
      st4<PolLamb::ST>(m + o, rm[i]);
      st4<PolLamb::ST>(v + o, rv[i]);
    }
  }
}

template <bool VEC, int GS>
__global__ __launch_bounds__(kBlock) void lamb_p1_kernel(const VarDesc* __restrict__ vars,
                                                         const ChunkDesc* __restrict__ chunks,
                                                         const float* __restrict__ w, const float* __restrict__ g,
                                                         const void* const* __restrict__ g_full, float* m, float* v,
                                                         float* __restrict__ chunk_sums, int r, AdamK k) {
  const int c = SU_P1_REVERSE ? (int)(gridDim.x - 1 - blockIdx.x) : (int)blockIdx.x;
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
          lamb_p1_tile<true, GS, true>(w + s0, gc.tile(base), m + s0, v + s0, kTileElems, valid, wd, k, sw, su);
        else
          lamb_p1_tile<true, GS, false>(w + s0, gc.tile(base), m + s0, v + s0, kTileElems, valid, wd, k, sw, su);
      } else {
        if (gc.fast(lim, valid))
          lamb_p1_tile<false, GS, true>(w + s0, gc.tile(base), m + s0, v + s0, lim, valid, wd, k, sw, su);
        else
          lamb_p1_tile<false, GS, false>(w + s0, gc.tile(base), m + s0, v + s0, lim, valid, wd, k, sw, su);
      }
    }
  } else {
    for (int e = threadIdx.x; e < cv.len; e += kBlock) {
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
// chunk table (thread t takes chunks t, t + kBlock, ...; float64 accumulators; wavefront shuffles,
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
  for (int c = threadIdx.x; c < vd.n_chunks; c += kBlock) {
    a += (double)chunk_sums[2 * (int64_t)(vd.first_chunk + c)];
    b += (double)chunk_sums[2 * (int64_t)(vd.first_chunk + c) + 1];
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
    const int o = i * kBlock * 4 + t4;
    if (FULL || o < lim) {
      rw[i] = ld4<PolLambP2::RW>(w + o);
      rm[i] = ld4<PolLambP2::RO>(m + o);
      rv[i] = ld4<PolLambP2::RO>(v + o);
    }
  }
#pragma unroll
  for (int i = 0; i < kUnroll; ++i) {
    const int o = i * kBlock * 4 + t4;
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
__global__ __launch_bounds__(kBlock) void lamb_p2_kernel(const VarDesc* __restrict__ vars,
                                                         const ChunkDesc* __restrict__ chunks, float* w,
                                                         const float* __restrict__ m, const float* __restrict__ v,
                                                         uint16_t* __restrict__ w16, const float* __restrict__ sums,
                                                         AdamK k) {
  const int c = SU_P2_REVERSE ? (int)(gridDim.x - 1 - blockIdx.x) : (int)blockIdx.x;
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
    for (int e = threadIdx.x; e < cv.len; e += kBlock) {
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
    const int o = i * kBlock * 4 + t4;
    if (FULL || o < lim) {
      rg[i] = load_g4<GS, GFAST, PolLars::RO>(g, o, valid);
      rw[i] = ld4<PolLars::RO>(w + o);
    }
  }
#pragma unroll
  for (int i = 0; i < kUnroll; ++i) {
    const int o = i * kBlock * 4 + t4;
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
__global__ __launch_bounds__(kBlock) void lars_p1_kernel(const VarDesc* __restrict__ vars,
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
    for (int e = threadIdx.x; e < cv.len; e += kBlock) {
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
    const int o = i * kBlock * 4 + t4;
    if (FULL || o < lim) {
      rg[i] = load_g4<GS, GFAST, PolLarsP2::RO>(g, o, valid);
      rw[i] = ld4<PolLarsP2::RW>(w + o);
      rm[i] = ld4<PolLarsP2::RW>(m + o);
    }
  }
#pragma unroll
  for (int i = 0; i < kUnroll; ++i) {
    const int o = i * kBlock * 4 + t4;
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
__global__ __launch_bounds__(kBlock) void lars_p2_kernel(const VarDesc* __restrict__ vars,
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
    for (int e = threadIdx.x; e < cv.len; e += kBlock) {
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
    const int o = i * kBlock * 4 + t4;
    if (FULL || o < lim) {
      rg[i] = load_g4<GS, GFAST, true>(g, o, valid);
      rw[i] = ld4<PolAdam::RW>(w + o);
      rm[i] = ld4<PolAdam::RW>(m + o);
      rv[i] = ld4<PolAdam::RW>(v + o);
    }
  }
#pragma unroll
  for (int i = 0; i < kUnroll; ++i) {
    const int o = i * kBlock * 4 + t4;
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
__global__ __launch_bounds__(kBlock) void adam_chunk_kernel(const VarDesc* __restrict__ vars,
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
    for (int e = threadIdx.x; e < cv.len; e += kBlock) {
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
    const int o = i * kBlock * 4 + t4;
    if (FULL || o < lim) {
      rg[i] = load_g4<GS, GFAST, true>(g, o, valid);
      rw[i] = ld4<PolMomentum::RW>(w + o);
      rm[i] = ld4<PolMomentum::RW>(m + o);
    }
  }
#pragma unroll
  for (int i = 0; i < kUnroll; ++i) {
    const int o = i * kBlock * 4 + t4;
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
__global__ __launch_bounds__(kBlock) void momentum_chunk_kernel(const VarDesc* __restrict__ vars,
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
    for (int e = threadIdx.x; e < cv.len; e += kBlock) {
      const int64_t s = cv.shard0 + e;
      float ww = w[s], mm = m[s];
      momentum_elem(ww, load_g1<GS>(gc, e, cv.valid), mm, k);
      w[s] = ww; m[s] = mm;
      if constexpr (BF16) w16[s] = (uint16_t)bf16_of(ww);
    }
  }
}

inline unsigned flat_grid(int64_t n4, int unroll) {
  const int64_t tile = (int64_t)kBlock * unroll;
  int64_t tiles = (n4 + tile - 1) / tile;
  if (tiles < 1) tiles = 1;
#if SU_GRID_CAP > 0
  if (tiles > SU_GRID_CAP) tiles = SU_GRID_CAP;
#endif
  if (tiles > 0x7FFFFFFF) tiles = 0x7FFFFFFF;
  return (unsigned)tiles;
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

// MODE: 0 = shard_format (one replica), 1 = unshard_format, 2 = shard_format_all
template <int SRC, int DST, int MODE>
void reformat_dispatch(shard_plan_t* p, int r0, int replicas, const void* const* tab, void* packed, int64_t stride,
                       bool vec, hipStream_t stream) {
  const int n_chunks = (int)p->chunks.size();
  constexpr int U = MODE == 0 ? SU_FORMAT_UNROLL : (MODE == 1 ? SU_UNSHARD_UNROLL : SU_FORMAT_ALL_UNROLL);
  constexpr int TILE = kCopyBlock * U * UnitOf<SRC, DST>::n;
  const int tiles_per_chunk = (p->chunk + TILE - 1) / TILE;
  // plan_build keeps n_chunks * N * (chunk / 1024) below 2^31, and a tile is at least 1024 slots
  const dim3 g((unsigned)((int64_t)n_chunks * replicas * tiles_per_chunk)), b(kCopyBlock);
  const VarDesc* vars = ws_at<VarDesc>(p, p->ws.vars);
  const ChunkDesc* chunks = ws_at<ChunkDesc>(p, p->ws.chunks);
  if (MODE != 0 && p->flat_copies) {
    // flat plan: variable by variable over the padded variables (same tiles, another item table)
    const FullChunk* fchunks = ws_at<FullChunk>(p, p->ws.full_chunks);
    const dim3 gf((unsigned)((int64_t)p->full_chunks.size() * tiles_per_chunk));
    if constexpr (MODE == 2) {
      if (vec) hipLaunchKernelGGL((format_all_flat_kernel<SRC, DST, true>), gf, b, 0, stream, vars, fchunks, tab, packed, stride, tiles_per_chunk);
      else hipLaunchKernelGGL((format_all_flat_kernel<SRC, DST, false>), gf, b, 0, stream, vars, fchunks, tab, packed, stride, tiles_per_chunk);
    } else if constexpr (MODE == 1) {
      if (vec) hipLaunchKernelGGL((unshard_flat_kernel<SRC, DST, true>), gf, b, 0, stream, vars, fchunks, tab, packed, stride, tiles_per_chunk);
      else hipLaunchKernelGGL((unshard_flat_kernel<SRC, DST, false>), gf, b, 0, stream, vars, fchunks, tab, packed, stride, tiles_per_chunk);
    }
    return;
  }
  if constexpr (MODE == 2) {
    if (vec)
      hipLaunchKernelGGL((format_all_kernel<SRC, DST, true>), g, b, 0, stream, vars, chunks, tab, packed, stride,
                         n_chunks, tiles_per_chunk);
    else
      hipLaunchKernelGGL((format_all_kernel<SRC, DST, false>), g, b, 0, stream, vars, chunks, tab, packed, stride,
                         n_chunks, tiles_per_chunk);
  } else if constexpr (MODE == 1) {
    if (vec)
      hipLaunchKernelGGL((unshard_kernel<SRC, DST, true>), g, b, 0, stream, vars, chunks, tab, packed, stride, n_chunks,
                         tiles_per_chunk);
    else
      hipLaunchKernelGGL((unshard_kernel<SRC, DST, false>), g, b, 0, stream, vars, chunks, tab, packed, stride,
                         n_chunks, tiles_per_chunk);
  } else {
    if (vec)
      hipLaunchKernelGGL((format_kernel<SRC, DST, true>), g, b, 0, stream, vars, chunks, tab, packed, r0, stride,
                         n_chunks, tiles_per_chunk);
    else
      hipLaunchKernelGGL((format_kernel<SRC, DST, false>), g, b, 0, stream, vars, chunks, tab, packed, r0, stride,
                         n_chunks, tiles_per_chunk);
  }
}

template <int MODE>
void reformat_any(shard_plan_t* p, int r0, int replicas, const void* const* tab, int src_dtype, void* packed,
                  int64_t stride, int dst_dtype, bool vec, hipStream_t stream) {
  if (src_dtype == SHARD_F32 && dst_dtype == SHARD_F32)
    reformat_dispatch<SHARD_F32, SHARD_F32, MODE>(p, r0, replicas, tab, packed, stride, vec, stream);
  else if (src_dtype == SHARD_F32)
    reformat_dispatch<SHARD_F32, SHARD_BF16, MODE>(p, r0, replicas, tab, packed, stride, vec, stream);
  else if (dst_dtype == SHARD_F32)
    reformat_dispatch<SHARD_BF16, SHARD_F32, MODE>(p, r0, replicas, tab, packed, stride, vec, stream);
  else
    reformat_dispatch<SHARD_BF16, SHARD_BF16, MODE>(p, r0, replicas, tab, packed, stride, vec, stream);
}
}  // namespace

hipError_t launch_format(shard_plan_t* p, int r, const void* const* tab, int src_dtype, void* out, int dst_dtype,
                         bool vec, hipStream_t stream) {
  if (p->chunks.empty()) return hipSuccess;
  ProfScope ps(p, SHARD_K_FORMAT, stream);
  reformat_any<0>(p, r, 1, tab, src_dtype, out, p->S, dst_dtype, vec, stream);
  return hipGetLastError();
}

hipError_t launch_format_all(shard_plan_t* p, const void* const* tab, int src_dtype, void* out, int64_t row_stride,
                             int dst_dtype, bool vec, hipStream_t stream) {
  if (p->chunks.empty()) return hipSuccess;
  ProfScope ps(p, SHARD_K_FORMAT, stream);
  reformat_any<2>(p, 0, p->N, tab, src_dtype, out, row_stride, dst_dtype, vec, stream);
  return hipGetLastError();
}

hipError_t launch_unshard(shard_plan_t* p, const void* gathered, int64_t row_stride, int src_dtype, void* const* tab,
                          int dst_dtype, bool vec, hipStream_t stream) {
  if (p->chunks.empty()) return hipSuccess;
  ProfScope ps(p, SHARD_K_UNSHARD, stream);
  reformat_any<1>(p, 0, p->N, reinterpret_cast<const void* const*>(tab), src_dtype, const_cast<void*>(gathered),
                     row_stride, dst_dtype, vec, stream);
  return hipGetLastError();
}

hipError_t launch_adam(shard_plan_t* p, float* w, const float* g, float* m, float* v, void* w16, const AdamK& k,
                       hipStream_t stream) {
  if (p->S == 0) return hipSuccess;
  ProfScope ps(p, SHARD_K_ADAM, stream);
  const int64_t n4 = p->S >> 2;
  const int tail = (int)(p->S & 3);
  if (w16)
    hipLaunchKernelGGL((adam_kernel<true>), dim3(flat_grid(n4, kAdamUnroll)), dim3(kBlock), 0, stream, w, g, m, v, (uint16_t*)w16,
                       n4, tail, k);
  else
    hipLaunchKernelGGL((adam_kernel<false>), dim3(flat_grid(n4, kAdamUnroll)), dim3(kBlock), 0, stream, w, g, m, v,
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
    hipLaunchKernelGGL((momentum_kernel<true>), dim3(flat_grid(n4, kMomentumUnroll)), dim3(kBlock), 0, stream, w, g, m, (uint16_t*)w16,
                       n4, tail, k);
  else
    hipLaunchKernelGGL((momentum_kernel<false>), dim3(flat_grid(n4, kMomentumUnroll)), dim3(kBlock), 0, stream, w, g, m,
                       (uint16_t*)nullptr, n4, tail, k);
  return hipGetLastError();
}

hipError_t launch_lamb_p1(shard_plan_t* p, int r, const float* w, const float* g, int g_source,
                          const void* const* g_full, float* m, float* v, const AdamK& k, hipStream_t stream) {
  if (p->chunks.empty()) return hipSuccess;
  ProfScope ps(p, SHARD_K_LAMB_P1, stream);
  const dim3 grid((unsigned)p->chunks.size());
  const VarDesc* vars = ws_at<VarDesc>(p, p->ws.vars);
  const ChunkDesc* chunks = ws_at<ChunkDesc>(p, p->ws.chunks);
  float* cs = ws_at<float>(p, p->ws.chunk_sums);
  const bool vec = p->align % 4 == 0;
#define SU_LAUNCH_P1(VEC, GS) \
  hipLaunchKernelGGL((lamb_p1_kernel<VEC, GS>), grid, dim3(kBlock), 0, stream, vars, chunks, w, g, g_full, m, v, cs, r, k)
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
                              hipStream_t stream) {
  if (p->V == 0) return hipSuccess;
  ProfScope ps(p, SHARD_K_NORM_REDUCE, stream);
  const dim3 grid((unsigned)p->V);
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
  hipLaunchKernelGGL((lars_p1_kernel<VEC, GS>), grid, dim3(kBlock), 0, stream, vars, chunks, w, g, g_full, cs, r)
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
#define SU_LAUNCH(VEC, BF16, GS)                                                                                     \
  hipLaunchKernelGGL((lars_p2_kernel<VEC, BF16, GS>), grid, dim3(kBlock), 0, stream, vars, chunks, w, g, g_full, m, o, \
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
  hipLaunchKernelGGL((adam_chunk_kernel<VEC, BF16, GS>), grid, dim3(kBlock), 0, stream, vars, chunks, w, g_full, m, v, \
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
  hipLaunchKernelGGL((momentum_chunk_kernel<VEC, BF16, GS>), grid, dim3(kBlock), 0, stream, vars, chunks, w, g_full, m, \
                     o, r, k)
  if (g_source == 1) SU_LAUNCH_GS(1);
  else SU_LAUNCH_GS(2);
#undef SU_LAUNCH
#undef SU_LAUNCH_GS
  return hipGetLastError();
}

}  // namespace su
