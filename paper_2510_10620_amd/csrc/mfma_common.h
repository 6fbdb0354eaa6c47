// Shared device code of the bf16 MFMA kernels (gfx950): fragment types, the LDS tile layout,
// tile staging, per-row mask ranges and tile classification.
//
// MFMA used: v_mfma_f32_32x32x16_bf16.  Operand layouts (lane l, i = l % 32, h = l / 32):
//   A (32 x 16): lane holds row i, k = 8h .. 8h+7          (8 bf16)
//   B (16 x 32): lane holds column i, k = 8h .. 8h+7       (8 bf16)
//   C (32 x 32): lane holds column i, register r holds row 8*(r/4) + 4h + (r%4)   (16 fp32)
// Because the contraction index k may be permuted as long as A and B agree, registers
// 8c .. 8c+7 of a C tile (rows 16c + 8a + 4h + b, a in {0,1}, b in 0..3) serve directly as the
// B operand of a following MFMA whose A operand supplies k-slot 8h + 4a + b from row 16c+8a+4h+b.
//
// LDS tiles are [rows][128] bf16, 256 bytes per row, no padding; the 16-byte chunk c of a row is
// stored at chunk c ^ swz(row).  With swz(row) = ((row & 3) << 2) | ((row >> 2) & 3) both access
// patterns are bank-conflict free: 16 consecutive rows at one chunk (row-major ds_read_b128) land
// in 16 different chunks, and 4 consecutive rows x 64 bytes (ds_read_b64_tr_b16 of a half-wave)
// land in 4 different 64-byte groups.
#pragma once
#include <hip/hip_runtime.h>
#include <cstdint>

#include "device_utils.h"
#include "dcp_internal.h"
#include "kernels.h"

namespace dcp {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

static constexpr int kD = 128;        // head dim of the MFMA family
static constexpr int kRowBytes = 256; // one tile row
static constexpr int kTN = 64;        // rows of a streamed tile (keys in fwd/dQ, queries in dK/dV)
static constexpr int kTileBytes = kTN * kRowBytes;

__device__ __forceinline__ int swz(int row) { return ((row & 3) << 2) | ((row >> 2) & 3); }
__device__ __forceinline__ int tile_off(int row, int c16) { return row * kRowBytes + ((c16 ^ swz(row)) << 4); }

__device__ __forceinline__ f32x16 mfma(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ bf16x8 as_frag(uint4 u) { return __builtin_bit_cast(bf16x8, u); }

// Row-major A/B fragment: 16 bytes of `row` at chunk c16.
__device__ __forceinline__ bf16x8 lds_frag(const char* tile, int row, int c16) {
  return as_frag(*(const uint4*)(tile + tile_off(row, c16)));
}

// Transposed fragment via two ds_read_b64_tr_b16: the lane receives, for tile column `col0 + l%32`
// (l%32 = 16*(blk%2) + j), the 8 values of rows  row0 + 8a + 4h + b  (a = 0,1; b = 0..3) in k-slot
// order 4a + b.  Inside a 16-lane block, lane j supplies the address of row (j / 4), columns
// 4*(j % 4) .. +3 and receives column j of the 4 rows.
__device__ __forceinline__ bf16x8 lds_frag_tr(const char* tile, int row0, int col0, int lane) {
  const int j = lane & 15, blk = lane >> 4, h = blk >> 1;
  const int col = col0 + 16 * (blk & 1) + 4 * (j & 3);
  const int r0 = row0 + 4 * h + (j >> 2);
  typedef __attribute__((address_space(3))) s16x4* lds_p;
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_p)(tile + tile_off(r0, col >> 3) + (col & 7) * 2));
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_p)(tile + tile_off(r0 + 8, col >> 3) + (col & 7) * 2));
  s16x8 v;
  v[0] = lo[0]; v[1] = lo[1]; v[2] = lo[2]; v[3] = lo[3]; v[4] = hi[0]; v[5] = hi[1]; v[6] = hi[2]; v[7] = hi[3];
  return __builtin_bit_cast(bf16x8, v);
}

// Lane-dependent parts of the fragment addresses, computed once.  Rows enter the swizzle only
// through row % 16, so a fragment whose first row is a multiple of 16 (resp. 32) is reached from
// these by adding a compile-time multiple of the row pitch, which folds into the LDS
// instruction's immediate offset.
struct FragAddr {
  int rm[8];     // row-major fragment of row (l % 32), chunk 2 ks + (l / 32), ks = 0..7
  int tr[4][2];  // transposed fragment for columns 32 dt .. 32 dt + 31: rows 4h + j/4 (+8)
  __device__ __forceinline__ void init(int lane) {
    const int li = lane & 31, lh = lane >> 5;
#pragma unroll
    for (int ks = 0; ks < 8; ks++) rm[ks] = tile_off(li, 2 * ks + lh);
    const int j = lane & 15, blk = lane >> 4, h = blk >> 1;
#pragma unroll
    for (int dt = 0; dt < 4; dt++) {
      const int col = 32 * dt + 16 * (blk & 1) + 4 * (j & 3);
      const int r0 = 4 * h + (j >> 2);
      tr[dt][0] = tile_off(r0, col >> 3) + (col & 7) * 2;
      tr[dt][1] = tile_off(r0 + 8, col >> 3) + (col & 7) * 2;
    }
  }
};

// Row-major fragment of rows row0 .. row0+31 (row0 a multiple of 32), k-step ks.
__device__ __forceinline__ bf16x8 frag_rm(const char* tile, const FragAddr& fa, int row0, int ks) {
  return as_frag(*(const uint4*)(tile + row0 * kRowBytes + fa.rm[ks]));
}
// Transposed fragment: rows row0 + 8a + 4h + b (row0 a multiple of 16), columns 32 dt + l % 32.
__device__ __forceinline__ bf16x8 frag_tr(const char* tile, const FragAddr& fa, int row0, int dt) {
  typedef __attribute__((address_space(3))) s16x4* lds_p;
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_p)(tile + row0 * kRowBytes + fa.tr[dt][0]));
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_p)(tile + row0 * kRowBytes + fa.tr[dt][1]));
  s16x8 v;
  v[0] = lo[0]; v[1] = lo[1]; v[2] = lo[2]; v[3] = lo[3]; v[4] = hi[0]; v[5] = hi[1]; v[6] = hi[2]; v[7] = hi[3];
  return __builtin_bit_cast(bf16x8, v);
}

// Packs registers 8c .. 8c+7 of a C tile to bf16 (B operand of the next MFMA).
__device__ __forceinline__ bf16x8 pack_frag(const f32x16& s, int c) {
  bf16x8 p;
#pragma unroll
  for (int e = 0; e < 8; e++) p[e] = (__bf16)s[8 * c + e];
  return p;
}

// Asynchronous global -> LDS copy of a 64-row tile (rows [row_start, row_start + 64) of a
// [T, H, 128] bf16 tensor, head already applied to `base`).  global_load_lds_dwordx4 writes lane
// L's 16 bytes at (wave-uniform LDS address in M0) + 16 L, so one wave instruction fills 4
// consecutive tile rows; the swizzle is applied on the global side: the lane that fills physical
// chunk p of a row fetches logical chunk p ^ swz(row).  Each of the workgroup's waves issues
// PW = 16 / (waves per workgroup) of the 16 instructions of a tile.
//
// The copy is issued from inline assembly in the (scalar base + 32-bit lane offset) form: the
// lane offset is computed once per kernel, the base moves on the scalar unit, so a tile costs
// no vector-ALU work.  The compiler does not see these copies: the caller must execute
// DCP_WAIT_VMCNT(0) before the barrier that publishes the tile.  A tile that runs past row_last
// (ragged end) clamps its rows so that every load reads real data.
// M0 is written inside the statement, so it is on the clobber list: the backend then sees the write (its pass that
// merges M0 initialisations must not carry a value across these statements).  The compiler's note that it will not
// save and restore a reserved register around the statement is expected here: nothing else in these kernels keeps M0.
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void dma16(unsigned voffset, const void* sbase, unsigned lds) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(voffset), "s"(sbase), "s"(lds) : "memory", "m0");
}
__device__ __forceinline__ void dma4(unsigned voffset, const void* sbase, unsigned lds) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1" ::"v"(voffset), "s"(sbase), "s"(lds) : "memory", "m0");
}
#pragma clang diagnostic pop
// a pointer that is wave-uniform by construction, made provably so (it must live in SGPRs)
__device__ __forceinline__ const void* uni_ptr(const void* p) {
  const uint64_t v = (uint64_t)p;
  return (const void*)(((uint64_t)(unsigned)__builtin_amdgcn_readfirstlane((int)(v >> 32)) << 32) |
                       (unsigned)__builtin_amdgcn_readfirstlane((int)v));
}
// s_waitcnt vmcnt(N) only (expcnt and lgkmcnt left at their maxima)
#define DCP_WAIT_VMCNT(N) __builtin_amdgcn_s_waitcnt(((N)&15) | (7 << 4) | (15 << 8) | (((N) >> 4) << 14))

__device__ __forceinline__ unsigned lds_addr(const void* p) { return (unsigned)(size_t)(__attribute__((address_space(3))) const char*)p; }

// Instruction u of wave w fills tile rows 4 (w + NW u) .. + 3 (NW waves): lane >> 4 picks the row, lane & 15 the
// physical 16-byte chunk, which receives the logical chunk (lane & 15) ^ swz(row).  The rows of a wave's instructions
// are 4 NW >= 16 apart, so they share row & 15 and with it the swizzle: one lane offset serves all of them, and
// instruction u only moves the scalar base by 4 NW u rows.
template <int PW>
struct TileDmaT {
  static_assert(PW <= 4, "needs 4 or more waves: the rows of a wave's instructions must be a multiple of 16 apart");
  static constexpr int NW = 16 / PW;
  unsigned off0;      // row * stride + chunk of the 16 bytes this lane fetches in instruction 0
  int sb;             // row stride, bytes
  static __device__ __forceinline__ int row0_of(int wave, int lane) { return 4 * wave + (lane >> 4); }
  static __device__ __forceinline__ int chunk_of(int lane, int row) { return ((lane & 15) ^ swz(row)) * 16; }
  static __device__ __forceinline__ unsigned lds_of(const void* tile, int wave) { return lds_addr(tile) + wave * 1024; }
  __device__ __forceinline__ void init(int wave, int lane, int64_t stride_t) {
    sb = (int)stride_t * 2;
    const int row = row0_of(wave, lane);
    off0 = (unsigned)(row * sb + chunk_of(lane, row));
  }
  // instruction u of a whole tile whose first row is at b (wave-uniform), into the wave's part l0 of the LDS tile
  __device__ __forceinline__ void issue(int u, const void* b, unsigned l0) const {
    dma16(off0, (const char*)b + (int64_t)(4 * NW * u) * sb, l0 + u * NW * 1024);
  }
  __device__ __forceinline__ void load(char* tile, const bf16_t* base, int row_start, int row_last, int wave) const {
    // wave-uniform by construction; readfirstlane makes it provably so (it must live in SGPRs)
    const void* b = uni_ptr((const char*)base + (int64_t)row_start * sb);
    const unsigned l0 = lds_of(tile, wave);
    if (row_start + kTN - 1 <= row_last) {
#pragma unroll
      for (int u = 0; u < PW; u++) issue(u, b, l0);
    } else {
      // ragged end: rows past row_last repeat it (recomputed here: this path is rare and the lane's
      // row / chunk numbers are not worth registers)
      const int lim = row_last - row_start, lane = threadIdx.x & 63;
      const int row = row0_of(wave, lane), ch = chunk_of(lane, row);
#pragma unroll
      for (int u = 0; u < PW; u++) dma16((unsigned)(min(row + 4 * NW * u, lim) * sb + ch), b, l0 + u * NW * 1024);
    }
  }
};

// The same copy with nothing kept in registers between calls (for kernels that have none to spare): the lane
// offset is recomputed from an opaque copy of the lane number at every call.
template <int PW>
__device__ __forceinline__ void tile_dma_lean(char* tile, const bf16_t* base, int sb, int row_start, int row_last, int wave) {
  int lane = threadIdx.x & 63;
  asm volatile("" : "+v"(lane));
  const void* b = uni_ptr((const char*)base + (int64_t)row_start * sb);
  const unsigned l0 = TileDmaT<PW>::lds_of(tile, wave);
  constexpr int NW = 16 / PW;
  const int row = TileDmaT<PW>::row0_of(wave, lane), ch = TileDmaT<PW>::chunk_of(lane, row);
  if (row_start + kTN - 1 <= row_last) {
    const unsigned off0 = (unsigned)(row * sb + ch);
#pragma unroll
    for (int u = 0; u < PW; u++) dma16(off0, (const char*)b + (int64_t)(4 * NW * u) * sb, l0 + u * NW * 1024);
  } else {
    const int lim = row_last - row_start;
#pragma unroll
    for (int u = 0; u < PW; u++) dma16((unsigned)(min(row + 4 * NW * u, lim) * sb + ch), b, l0 + u * NW * 1024);
  }
}

typedef TileDmaT<4> TileDma;   // 4 waves per workgroup

// Two half-open key ranges of one query row, clipped to a KV block.
struct RowRanges {
  int lo1, n1, lo2, n2;  // start and length (0 when empty)
  __device__ __forceinline__ bool sees(int key) const {
    return (unsigned)(key - lo1) < (unsigned)n1 || (unsigned)(key - lo2) < (unsigned)n2;
  }
};

// Effective ranges of query `i` (packed index) for one table row of kind `kind` over the block
// [c0, c1); `r` holds the query's range array entry (RANGES only).
__device__ __forceinline__ RowRanges row_ranges(int kind, int i, int c0, int c1, int4 r) {
  RowRanges g;
  int lo1 = c0, hi1 = c1, lo2 = 0, hi2 = 0;
  if (kind == 1) hi1 = min(i + 1, c1);
  if (kind == 2) { lo1 = max(r.x, c0); hi1 = min(r.y, c1); lo2 = max(r.z, c0); hi2 = min(r.w, c1); }
  g.lo1 = lo1; g.n1 = max(hi1 - lo1, 0); g.lo2 = lo2; g.n2 = max(hi2 - lo2, 0);
  return g;
}

// Bounds of a set of rows' range arrays: for each of the two ranges the smallest start, largest
// start, smallest end, largest end over rows whose range is not empty (`any` = some row has one).
struct RangeBounds {
  int lo_min[2], lo_max[2], hi_min[2], hi_max[2];
  __device__ __forceinline__ void init() {
#pragma unroll
    for (int k = 0; k < 2; k++) { lo_min[k] = INT32_MAX; lo_max[k] = INT32_MIN; hi_min[k] = INT32_MAX; hi_max[k] = INT32_MIN; }
  }
  // rows with an empty range make "all rows cover the tile" impossible: lo_max = +inf
  __device__ __forceinline__ void add(int4 r) {
    const int lo[2] = {r.x, r.z}, hi[2] = {r.y, r.w};
#pragma unroll
    for (int k = 0; k < 2; k++) {
      if (hi[k] > lo[k]) {
        lo_min[k] = min(lo_min[k], lo[k]); lo_max[k] = max(lo_max[k], lo[k]);
        hi_min[k] = min(hi_min[k], hi[k]); hi_max[k] = max(hi_max[k], hi[k]);
      } else {
        lo_max[k] = INT32_MAX; hi_min[k] = INT32_MIN;
      }
    }
  }
  __device__ __forceinline__ void wave_reduce() {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
#pragma unroll
      for (int k = 0; k < 2; k++) {
        lo_min[k] = min(lo_min[k], __shfl_xor(lo_min[k], off)); lo_max[k] = max(lo_max[k], __shfl_xor(lo_max[k], off));
        hi_min[k] = min(hi_min[k], __shfl_xor(hi_min[k], off)); hi_max[k] = max(hi_max[k], __shfl_xor(hi_max[k], off));
      }
    }
  }
  // some row may see a key of [ks, ke)
  __device__ __forceinline__ bool may_see(int ks, int ke) const {
    return (ks < hi_max[0] && ke > lo_min[0]) || (ks < hi_max[1] && ke > lo_min[1]);
  }
  // every row sees every key of [ks, ke)
  __device__ __forceinline__ bool all_see(int ks, int ke) const {
    return (ks >= lo_max[0] && ke <= hi_min[0]) || (ks >= lo_max[1] && ke <= hi_min[1]);
  }
};

enum TileClass { kSkip = 0, kFull = 1, kPartial = 2 };

// Class of the key tile [ks, ks + 64) of the block ending at c1 for query rows [q_lo, q_hi]
// (packed, inclusive, all valid) with range bounds rb.
__device__ __forceinline__ int classify(int kind, int ks, int c1, int q_lo, int q_hi, const RangeBounds& rb) {
  const int ke = min(ks + kTN, c1);
  const bool whole = ks + kTN <= c1;
  if (kind == 0) return whole ? kFull : kPartial;
  if (kind == 1) {
    if (ks > q_hi) return kSkip;
    return (whole && ke - 1 <= q_lo) ? kFull : kPartial;
  }
  if (!rb.may_see(ks, ke)) return kSkip;
  return (whole && rb.all_see(ks, ke)) ? kFull : kPartial;
}

__device__ __forceinline__ int uni(int x) { return __builtin_amdgcn_readfirstlane(x); }

// Combine a value with the one held by lane (l ^ 32), in every lane, without an LDS round trip:
// v_permlane32_swap exchanges lanes 32..63 of its first operand with lanes 0..31 of its second, so
// with the same value in both, each lane ends up holding the lower half's value in one result and
// the upper half's in the other.
__device__ __forceinline__ float xhalf_max(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
// Writes a wave's 32 x 128 result tile to memory as bf16, turned round through LDS.
// acc is the accumulator of a transposed product: lane (li, lh) holds row li of the tile in 8-byte pieces scattered
// over the row (columns 32 dt + 8 a + 4 lh .. + 3 in acc[dt][4 a .. 4 a + 3]), so stored straight from the registers
// every store instruction touches 32 rows with 16 bytes each.  Here the wave writes the pieces into a region of LDS
// of its own (32 rows of kORow bytes at `ot`; no other wave may use it meanwhile, and no barrier between waves is
// needed), reads them back as whole rows, and each store instruction writes four full 256-byte rows.
// mul: factor of the lane's row.  Rows r < n_valid go to row0_ptr + r * stride (elements).
static constexpr int kORow = kRowBytes + 16;   // staged row pitch: 16 bytes of padding spread the rows over the banks
__device__ __forceinline__ void store_tile32(char* ot, const f32x16 (&acc)[4], float mul, int lane, int n_valid, bf16_t* row0_ptr,
                                             int64_t stride) {
  const int li = lane & 31, lh = lane >> 5, lr = lane >> 4, lc = lane & 15;
#pragma unroll
  for (int dt = 0; dt < 4; dt++)
#pragma unroll
    for (int a = 0; a < 4; a++) {
      uint2 pk;
      pk.x = pack_bf16x2(acc[dt][4 * a] * mul, acc[dt][4 * a + 1] * mul);
      pk.y = pack_bf16x2(acc[dt][4 * a + 2] * mul, acc[dt][4 * a + 3] * mul);
      *(uint2*)(ot + li * kORow + 2 * (32 * dt + 8 * a + 4 * lh)) = pk;
    }
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
  for (int i = 0; i < 8; i++) {
    const int r = 4 * i + lr;
    const uint4 piece = *(const uint4*)(ot + r * kORow + 16 * lc);
    if (r < n_valid) *(uint4*)(row0_ptr + (int64_t)r * stride + 8 * lc) = piece;
  }
  // the next use of the region by this wave comes after these reads
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
}

__device__ __forceinline__ float xhalf_sum(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// Walks the (table row, key tile) pairs of a unit that the workgroup cannot skip.  All state is
// wave-uniform.
struct KvIter {
  const int4* rec;   // per table row: {first key, length, mask kind, memory offset of the KV block}, {..}
  int e, e_end, jt, n_t;
  int c0, c1, kind;
  int moff;  // the KV block's rows sit at (packed index + moff) in the KV-type buffers
  int ks;    // first key of the current tile
  // [e0, e1): the unit's table rows (from the work item)
  __device__ KvIter(const DevGroup& g, int e0, int e1) : rec((const int4*)g.ent_rec) {
    e = e0 - 1; e_end = e1; jt = 0; n_t = 0; c0 = c1 = kind = 0; moff = 0; ks = 0;
  }
  // Advances to the next tile some row of [.., q_hi] may see; false when the unit is done.
  // RANGES = false: the table has no RANGES row (nothing of the range machinery is compiled in).
  template <bool RANGES>
  __device__ bool next(int q_hi, const RangeBounds& rb) {
    for (;;) {
      jt++;
      if (jt >= n_t) {
        e++;
        if (e >= e_end) return false;
        const int4 r = rec[2 * e];
        c0 = uni(r.x); c1 = c0 + uni(r.y); kind = uni(r.z); moff = uni(r.w);
        n_t = (c1 - c0 + kTN - 1) / kTN;
        if (kind == 1) n_t = min(n_t, max(0, (q_hi - c0) / kTN + 1));  // tiles starting after q_hi are empty
        jt = -1;
        continue;
      }
      ks = c0 + jt * kTN;
      if (!RANGES || kind != 2 || rb.may_see(ks, min(ks + kTN, c1))) return true;
    }
  }
};

// Class of the 32-key sub-tile [ks, ks + 32) for the rows [q_lo, q_hi] with bounds rb.
__device__ __forceinline__ int classify32(int kind, int ks, int c1, int q_lo, int q_hi, const RangeBounds& rb) {
  if (ks >= c1) return kSkip;
  const int ke = min(ks + 32, c1);
  const bool whole = ks + 32 <= c1;
  if (kind == 0) return whole ? kFull : kPartial;
  if (kind == 1) {
    if (ks > q_hi) return kSkip;
    return (whole && ke - 1 <= q_lo) ? kFull : kPartial;
  }
  if (!rb.may_see(ks, ke)) return kSkip;
  return (whole && rb.all_see(ks, ke)) ? kFull : kPartial;
}

// XCD-aware decode of the flat workgroup id.  Consecutive workgroup ids are dealt round-robin to the 8 XCDs, so
// workgroup id b is the (b / 8)-th of XCD b % 8.  The work is cut into (KV head, segment of the work list) units,
// heads_outer * n_seg of them, a multiple of 8; XCD x takes units x * U / 8 .. in (head, segment) order and walks
// each in (item, head of the group) order: workgroups that run at the same time on an XCD work on neighbouring
// items of one KV head, whose K / V (or Q / dO) rows that XCD's L2 then holds once.  With a multiple of 8 KV heads
// an XCD takes whole heads and the list is one segment.
__device__ __forceinline__ bool decode_wg(const DevGroup& g, int heads_outer, int heads_inner, int* item, int* head) {
  const int upx = (heads_outer * g.n_seg) >> 3;
  int p = blockIdx.x >> 3;
  for (int u = (blockIdx.x & 7) * upx, ue = u + upx; u < ue; u++) {
    const int s = u % g.n_seg;
    const int s0 = g.seg[s], len = (g.seg[s + 1] - s0) * heads_inner;
    if (p < len) {
      *item = s0 + p / heads_inner;
      *head = (u / g.n_seg) * heads_inner + p % heads_inner;
      return true;
    }
    p -= len;
  }
  return false;
}

}  // namespace dcp
