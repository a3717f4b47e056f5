// Formatting kernels for gfx950 (MI355X) and their launchers: shard_format, shard_format_all,
// unshard_format and the device pointer tables they read.
//
// Pure data movement, bound by HBM bandwidth.  Every lane moves 128 bits per access (a 64-lane
// wavefront covers 1 KiB of one stream), every thread issues all the loads of its tile before the
// first store, and one launch covers the whole model: variables are addressed through a chunk table,
// so hundreds of small variables cost no launches of their own (the single-GPU analogue of the
// paper's batching of small tensors, Section 5.2).
#include <type_traits>

#include "chunk_view.hpp"

namespace su {
namespace {

constexpr int kCopyBlock = 256;    // threads per workgroup of the formatting kernels (128 or 64: -1 to -7 %; 512 and 1024: -3 to -30 %)

// Cache policy per kernel, as a 3-bit mask: 4 = non-temporal loads, 1 = non-temporal stores (2 is unused
// here: nothing is updated in place).  Measured best on MI355X, scored on the whole step (format, update,
// unshard), since a kernel's policy decides what the next kernel finds in the caches.
typedef Policy<4> PolFormat;
typedef Policy<5> PolUnshard;
typedef Policy<5> PolFormatAll;    // all-replica formatting: the output goes to a collective, not to the next kernel

// Units per thread of the formatting kernels, all loaded before the first store.  One replica's
// formatting (a few hundred MB, partly served by the memory-side cache) measures fastest with 2;
// the whole-model copies (unshard, all-replica formatting) with 1.
constexpr int kFormatUnroll = 2, kUnshardUnroll = 1, kFormatAllUnroll = 1;

// ---- pointer table --------------------------------------------------------------------------------
// Device pointer tables are written by a kernel that carries the pointers as launch arguments:
// stream-ordered, no host staging buffer whose lifetime would have to be tracked.
__global__ __launch_bounds__(kPtrBatch) void ptr_table_kernel(PtrBatch b, const void** dst, int count) {
  const int i = threadIdx.x;
  if (i < count) dst[i] = b.p[i];
}

// ---- the plain copy the formatting kernels are measured against -----------------------------------
__global__ __launch_bounds__(kCopyBlock) void plain_copy_kernel(const u4* __restrict__ src, u4* __restrict__ dst,
                                                             size_t units16) {
  const size_t u = (size_t)blockIdx.x * kCopyBlock + threadIdx.x;
  if (u < units16) st<true>(dst + u, ld<true>(src + u));
}

// ---- shard_format / unshard_format ----------------------------------------------------------------
// A unit is what one lane moves at a time: 8 elements when the destination is bfloat16, so that every store is
// a 128-bit access (from float32 that is two 128-bit loads; with 4-element units and 64-bit stores the
// float32 -> bfloat16 unshard of the 340 M-parameter model ran at 5.2 instead of 5.8 TB/s; full tiles of that pair
// take the lane-pair exchange in copy_units, which keeps the loads coalesced as well: 6.0 TB/s), 4 elements when it is
// float32 (bfloat16 -> float32 then loads 64 bits per lane, which measured 4 % faster than 8-element units).
// Consecutive lanes take consecutive units, so the accesses of a wavefront cover one contiguous span of memory.

template <int DT> struct ElemOf;
template <> struct ElemOf<SHARD_F32> { typedef uint32_t type; };
template <> struct ElemOf<SHARD_BF16> { typedef uint16_t type; };

template <int SRC, int DST>
struct UnitOf {
  static constexpr int n = DST == SHARD_BF16 ? 8 : 4;
};

template <typename Pol, int DT, int UNIT>
__device__ __forceinline__ void load_unit(const typename ElemOf<DT>::type* p, uint32_t (&x)[UNIT]) {
  if constexpr (DT == SHARD_F32 && UNIT == 4) {
    const u4 a = ld<Pol::RO>((const u4*)p);
    x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w;
  } else if constexpr (DT == SHARD_F32) {
    static_assert(UNIT == 8, "float32 units are 4 or 8 elements");
    const u4 a = ld<Pol::RO>((const u4*)p);
    const u4 b = ld<Pol::RO>((const u4*)p + 1);
    x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w;
    x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
  } else {
    if constexpr (UNIT == 8) {
      const u4 a = ld<Pol::RO>((const u4*)p);
      x[0] = a.x & 0xFFFFu; x[1] = a.x >> 16; x[2] = a.y & 0xFFFFu; x[3] = a.y >> 16;
      x[4] = a.z & 0xFFFFu; x[5] = a.z >> 16; x[6] = a.w & 0xFFFFu; x[7] = a.w >> 16;
    } else {
      const u2 a = ld<Pol::RO>((const u2*)p);
      x[0] = a.x & 0xFFFFu; x[1] = a.x >> 16; x[2] = a.y & 0xFFFFu; x[3] = a.y >> 16;
    }
  }
}
template <typename Pol, int DT, int UNIT>
__device__ __forceinline__ void store_unit(typename ElemOf<DT>::type* p, const uint32_t (&x)[UNIT]) {
  if constexpr (DT == SHARD_F32 && UNIT == 4) {
    u4 a;
    a.x = x[0]; a.y = x[1]; a.z = x[2]; a.w = x[3];
    st<Pol::ST>((u4*)p, a);
  } else if constexpr (DT == SHARD_F32) {
    static_assert(UNIT == 8, "float32 units are 4 or 8 elements");
    u4 a, b;
    a.x = x[0]; a.y = x[1]; a.z = x[2]; a.w = x[3];
    b.x = x[4]; b.y = x[5]; b.z = x[6]; b.w = x[7];
    st<Pol::ST>((u4*)p, a);
    st<Pol::ST>((u4*)p + 1, b);
  } else {
    static_assert(UNIT == 8, "bfloat16 units are 8 elements");
    u4 a;
    a.x = x[0] | (x[1] << 16); a.y = x[2] | (x[3] << 16); a.z = x[4] | (x[5] << 16); a.w = x[6] | (x[7] << 16);
    st<Pol::ST>((u4*)p, a);
  }
}
// One replica's formatting takes two units per thread only where the tile then still is the default chunk
// (2048 slots): with 8-element units a second one would send every chunk down the predicated path.
template <int SRC, int DST>
constexpr int format_unroll() { return UnitOf<SRC, DST>::n == 8 ? 1 : kFormatUnroll; }

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
  if constexpr (ALL && U == 1 && SRC == SHARD_F32 && DST == SHARD_BF16) {
    // A full tile of float32 -> bfloat16 (2048 elements).  Loading a thread's 8 consecutive floats takes two
    // 128-bit loads 32 bytes apart, which leaves every load instruction of a wavefront half-used.  Instead thread
    // t loads the 4 floats at 4t and the 4 floats at 1024 + 4t (both instructions fully coalesced), converts them,
    // and neighbouring lanes swap halves so that the even lane holds 8 consecutive bfloat16 of the tile's first
    // half and the odd lane 8 of its second half: every store is 128 bits.  Same bytes as the generic path.
    constexpr int HALF = kCopyBlock * 4;
    const int t = (int)threadIdx.x;
    const u4 a = ld<Pol::RO>((const u4*)(src + 4 * t));
    const u4 b = ld<Pol::RO>((const u4*)(src + HALF + 4 * t));
    const uint32_t a0 = bf16_from_f32_bits(a.x) | (bf16_from_f32_bits(a.y) << 16);
    const uint32_t a1 = bf16_from_f32_bits(a.z) | (bf16_from_f32_bits(a.w) << 16);
    const uint32_t b0 = bf16_from_f32_bits(b.x) | (bf16_from_f32_bits(b.y) << 16);
    const uint32_t b1 = bf16_from_f32_bits(b.z) | (bf16_from_f32_bits(b.w) << 16);
    const bool odd = (t & 1) != 0;
    // what the neighbour needs: the even lane's second-half pair goes to the odd lane, the odd lane's first-half pair
    // to the even one (quad_perm [1,0,3,2] = lane ^ 1)
    const uint32_t s0 = odd ? a0 : b0, s1 = odd ? a1 : b1;
    const uint32_t r0 = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)s0, 0xB1, 0xF, 0xF, false);
    const uint32_t r1 = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)s1, 0xB1, 0xF, 0xF, false);
    u4 o;
    if (odd) { o.x = r0; o.y = r1; o.z = b0; o.w = b1; }      // elements 1024 + 4(t-1) .. 1024 + 4t + 3
    else     { o.x = a0; o.y = a1; o.z = r0; o.w = r1; }      // elements 4t .. 4t + 7
    uint16_t* out = (uint16_t*)dst + (odd ? HALF + 4 * (t - 1) : 4 * t);
    st<Pol::ST>((u4*)out, o);
    return;
  }
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
                                              int64_t row_stride, int n_chunks, int tiles_per_chunk,
                                              int wg_per_replica) {
  typedef typename ElemOf<SRC>::type SrcT;
  typedef typename ElemOf<DST>::type DstT;
  // wg_per_replica = n_chunks * tiles_per_chunk, plus one idle workgroup where that is even (see odd_count)
  const int replica = blockIdx.x / wg_per_replica;
  const int j = blockIdx.x - replica * wg_per_replica;
  const int item = j / tiles_per_chunk;
  if (item >= n_chunks) return;
  const int tile = j - item * tiles_per_chunk;
  const ChunkView cv = chunk_view(vars, chunks, item, r0 + replica);
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
  if (vec && here == TILE && k0 + TILE <= vd.L && real >= TILE) {
    // a full tile of real elements inside one piece: two contiguous spans, moved without a branch
    if (TO_FULL) copy_units<Pol, SRC, DST, U, true, true>((const SrcT*)rows + r0 * row_stride + k0, (DstT*)full, TILE, TILE, TILE);
    else copy_units<Pol, SRC, DST, U, true, false>((const SrcT*)full, (DstT*)rows + r0 * row_stride + k0, TILE, TILE, TILE);
    return;
  }
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
  reformat_flat_body<PolUnshard, SRC, DST, kUnshardUnroll, VEC, true>(vars, fchunks, ptrs, gathered, row_stride, tiles_per_chunk);
}

template <int SRC, int DST, bool VEC>
__global__ __launch_bounds__(kCopyBlock) void format_all_flat_kernel(const VarDesc* __restrict__ vars,
                                                                 const FullChunk* __restrict__ fchunks,
                                                                 const void* const* __restrict__ ptrs, void* out,
                                                                 int64_t row_stride, int tiles_per_chunk) {
  reformat_flat_body<PolFormatAll, SRC, DST, kFormatAllUnroll, VEC, false>(vars, fchunks, ptrs, out, row_stride, tiles_per_chunk);
}

template <int SRC, int DST, bool VEC>
__global__ __launch_bounds__(kCopyBlock) void format_kernel(const VarDesc* __restrict__ vars,
                                                        const ChunkDesc* __restrict__ chunks,
                                                        const void* const* __restrict__ ptrs, void* out, int r0,
                                                        int64_t row_stride, int n_chunks, int tiles_per_chunk,
                                                        int wg_per_replica) {
  reformat_body<PolFormat, SRC, DST, format_unroll<SRC, DST>(), VEC, false>(vars, chunks, ptrs, out, r0, row_stride, n_chunks, tiles_per_chunk, wg_per_replica);
}

template <int SRC, int DST, bool VEC>
__global__ __launch_bounds__(kCopyBlock) void format_all_kernel(const VarDesc* __restrict__ vars,
                                                            const ChunkDesc* __restrict__ chunks,
                                                            const void* const* __restrict__ ptrs, void* out,
                                                            int64_t row_stride, int n_chunks, int tiles_per_chunk,
                                                            int wg_per_replica) {
  reformat_body<PolFormatAll, SRC, DST, kFormatAllUnroll, VEC, false>(vars, chunks, ptrs, out, 0, row_stride, n_chunks, tiles_per_chunk, wg_per_replica);
}

template <int SRC, int DST, bool VEC>
__global__ __launch_bounds__(kCopyBlock) void unshard_kernel(const VarDesc* __restrict__ vars,
                                                         const ChunkDesc* __restrict__ chunks,
                                                         const void* const* __restrict__ ptrs, void* gathered,
                                                         int64_t row_stride, int n_chunks, int tiles_per_chunk,
                                                         int wg_per_replica) {
  reformat_body<PolUnshard, SRC, DST, kUnshardUnroll, VEC, true>(vars, chunks, ptrs, gathered, 0, row_stride, n_chunks, tiles_per_chunk, wg_per_replica);
}

}  // namespace

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

// Workgroups are dealt out to the 8 XCDs in turn, and the light ones (the last, partly filled tiles of a
// variable, the empty second tile of a short chunk) sit at the same places of every replica's sequence.  With an
// even number of workgroups per replica the same XCDs would get them replica after replica and run out of work
// while the others are still busy (measured: 5 % on the 1.5 G-parameter list at 128 replicas); an odd count moves
// the sequence on by one XCD per replica.
inline int odd_count(int64_t wgs, int replicas) {
  if (replicas > 1 && (wgs & 1) == 0 && (wgs + 1) * replicas <= 0x7FFFFFFF) return (int)wgs + 1;
  return (int)wgs;
}

// LDS reserved per workgroup (never touched) to cap the workgroups resident per CU: 0 = no cap.
constexpr unsigned kLdsFormat = 0, kLdsUnshard = 0, kLdsFormatAll = 0, kLdsUnshardFlat = 0, kLdsFormatAllFlat = 0;

// MODE: 0 = shard_format (one replica), 1 = unshard_format, 2 = shard_format_all
template <int SRC, int DST, int MODE>
void reformat_dispatch(shard_plan_t* p, int r0, int replicas, const void* const* tab, void* packed, int64_t stride,
                       bool vec, bool by_variable, hipStream_t stream) {
  const int n_chunks = (int)p->chunks.size();
  constexpr int U = MODE == 0 ? format_unroll<SRC, DST>() : (MODE == 1 ? kUnshardUnroll : kFormatAllUnroll);
  constexpr int TILE = kCopyBlock * U * UnitOf<SRC, DST>::n;
  const int tiles_per_chunk = (p->chunk + TILE - 1) / TILE;
  // plan_build keeps n_chunks * N * (chunk / 1024) below 2^31, and a tile is at least 1024 slots
  const int per = odd_count((int64_t)n_chunks * tiles_per_chunk, replicas);
  const dim3 g((unsigned)((int64_t)per * replicas)), b(kCopyBlock);
  const VarDesc* vars = ws_at<VarDesc>(p, p->ws.vars);
  const ChunkDesc* chunks = ws_at<ChunkDesc>(p, p->ws.chunks);
  if (MODE != 0 && by_variable && !p->full_chunks.empty()) {
    // flat plan: variable by variable over the padded variables (same tiles, another item table)
    const FullChunk* fchunks = ws_at<FullChunk>(p, p->ws.full_chunks);
    const dim3 gf((unsigned)((int64_t)p->full_chunks.size() * tiles_per_chunk));
    if constexpr (MODE == 2) {
      // Formatting writes the gathered rows: variables with whole-chunk pieces go replica by replica (contiguous
      // writes), the small ones variable by variable (full tiles); two launches over two sub-tables.
      const int n_major = (int)p->major_chunks.size();
      const ChunkDesc* major = ws_at<ChunkDesc>(p, p->ws.major_chunks);
      const int per_major = odd_count((int64_t)n_major * tiles_per_chunk, replicas);
      const dim3 gm((unsigned)((int64_t)per_major * replicas));
      if (n_major > 0) {
        if (vec) hipLaunchKernelGGL((format_all_kernel<SRC, DST, true>), gm, b, kLdsFormatAll, stream, vars, major, tab, packed, stride, n_major, tiles_per_chunk, per_major);
        else hipLaunchKernelGGL((format_all_kernel<SRC, DST, false>), gm, b, kLdsFormatAll, stream, vars, major, tab, packed, stride, n_major, tiles_per_chunk, per_major);
      }
      // no split (large pieces throughout, this order picked by measurement): every item variable by variable
      const bool split = p->flat_copies;
      const FullChunk* small = split ? ws_at<FullChunk>(p, p->ws.small_full_chunks) : fchunks;
      const size_t n_small = split ? p->small_full_chunks.size() : p->full_chunks.size();
      const dim3 gs((unsigned)((int64_t)n_small * tiles_per_chunk));
      if (n_small > 0) {
        if (vec) hipLaunchKernelGGL((format_all_flat_kernel<SRC, DST, true>), gs, b, kLdsFormatAllFlat, stream, vars, small, tab, packed, stride, tiles_per_chunk);
        else hipLaunchKernelGGL((format_all_flat_kernel<SRC, DST, false>), gs, b, kLdsFormatAllFlat, stream, vars, small, tab, packed, stride, tiles_per_chunk);
      }
    } else if constexpr (MODE == 1) {
      if (vec) hipLaunchKernelGGL((unshard_flat_kernel<SRC, DST, true>), gf, b, kLdsUnshardFlat, stream, vars, fchunks, tab, packed, stride, tiles_per_chunk);
      else hipLaunchKernelGGL((unshard_flat_kernel<SRC, DST, false>), gf, b, kLdsUnshardFlat, stream, vars, fchunks, tab, packed, stride, tiles_per_chunk);
    }
    return;
  }
  if constexpr (MODE == 2) {
    if (vec)
      hipLaunchKernelGGL((format_all_kernel<SRC, DST, true>), g, b, kLdsFormatAll, stream, vars, chunks, tab, packed, stride,
                         n_chunks, tiles_per_chunk, per);
    else
      hipLaunchKernelGGL((format_all_kernel<SRC, DST, false>), g, b, kLdsFormatAll, stream, vars, chunks, tab, packed, stride,
                         n_chunks, tiles_per_chunk, per);
  } else if constexpr (MODE == 1) {
    if (vec)
      hipLaunchKernelGGL((unshard_kernel<SRC, DST, true>), g, b, kLdsUnshard, stream, vars, chunks, tab, packed, stride, n_chunks,
                         tiles_per_chunk, per);
    else
      hipLaunchKernelGGL((unshard_kernel<SRC, DST, false>), g, b, kLdsUnshard, stream, vars, chunks, tab, packed, stride,
                         n_chunks, tiles_per_chunk, per);
  } else {
    if (vec)
      hipLaunchKernelGGL((format_kernel<SRC, DST, true>), g, b, kLdsFormat, stream, vars, chunks, tab, packed, r0, stride,
                         n_chunks, tiles_per_chunk, per);
    else
      hipLaunchKernelGGL((format_kernel<SRC, DST, false>), g, b, kLdsFormat, stream, vars, chunks, tab, packed, r0, stride,
                         n_chunks, tiles_per_chunk, per);
  }
}

template <int MODE>
void reformat_any(shard_plan_t* p, int r0, int replicas, const void* const* tab, int src_dtype, void* packed,
                  int64_t stride, int dst_dtype, bool vec, bool by_variable, hipStream_t stream) {
  if (src_dtype == SHARD_F32 && dst_dtype == SHARD_F32)
    reformat_dispatch<SHARD_F32, SHARD_F32, MODE>(p, r0, replicas, tab, packed, stride, vec, by_variable, stream);
  else if (src_dtype == SHARD_F32)
    reformat_dispatch<SHARD_F32, SHARD_BF16, MODE>(p, r0, replicas, tab, packed, stride, vec, by_variable, stream);
  else if (dst_dtype == SHARD_F32)
    reformat_dispatch<SHARD_BF16, SHARD_F32, MODE>(p, r0, replicas, tab, packed, stride, vec, by_variable, stream);
  else
    reformat_dispatch<SHARD_BF16, SHARD_BF16, MODE>(p, r0, replicas, tab, packed, stride, vec, by_variable, stream);
}
}  // namespace

hipError_t launch_plain_copy(shard_plan_t* p, void* dst, const void* src, size_t units16, hipStream_t stream) {
  ProfScope ps(p, SHARD_K_PLAIN_COPY, stream);
  const size_t blocks = (units16 + kCopyBlock - 1) / kCopyBlock;
  hipLaunchKernelGGL(plain_copy_kernel, dim3((unsigned)blocks), dim3(kCopyBlock), 0, stream, (const u4*)src, (u4*)dst,
                     units16);
  return hipGetLastError();
}

hipError_t launch_format(shard_plan_t* p, int r, const void* const* tab, int src_dtype, void* out, int dst_dtype,
                         bool vec, hipStream_t stream) {
  if (p->chunks.empty()) return hipSuccess;
  ProfScope ps(p, SHARD_K_FORMAT, stream);
  reformat_any<0>(p, r, 1, tab, src_dtype, out, p->S, dst_dtype, vec, false, stream);
  return hipGetLastError();
}

hipError_t launch_format_all(shard_plan_t* p, const void* const* tab, int src_dtype, void* out, int64_t row_stride,
                             int dst_dtype, bool vec, bool by_variable, hipStream_t stream) {
  if (p->chunks.empty()) return hipSuccess;
  ProfScope ps(p, SHARD_K_FORMAT, stream);
  reformat_any<2>(p, 0, p->N, tab, src_dtype, out, row_stride, dst_dtype, vec, by_variable, stream);
  return hipGetLastError();
}

hipError_t launch_unshard(shard_plan_t* p, const void* gathered, int64_t row_stride, int src_dtype, void* const* tab,
                          int dst_dtype, bool vec, bool by_variable, hipStream_t stream) {
  if (p->chunks.empty()) return hipSuccess;
  ProfScope ps(p, SHARD_K_UNSHARD, stream);
  reformat_any<1>(p, 0, p->N, reinterpret_cast<const void* const*>(tab), src_dtype, const_cast<void*>(gathered),
                     row_stride, dst_dtype, vec, by_variable, stream);
  return hipGetLastError();
}

}  // namespace su
