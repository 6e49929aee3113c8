// Brute-force Euclidean-distance epsilon self-join for gfx950 (MI355X): kernels and C ABI.
//
// Method (arXiv 2508.21230, Section 3.1): Step 1 norms s_i, Step 2 Gram products a_ij on the
// matrix cores with FP16 inputs / FP32 accumulation, Step 3 dist^2 = s_i + s_j - 2 a_ij, then
// the "<= epsilon" filter of Section 2.2.1.  The tiling below is designed for CDNA4 (64-wide
// wavefronts, v_mfma_f32_16x16x32_f16, 160 KB LDS with 64 banks, 8 XCDs with private L2s); the
// paper's A100 tiling (Section 3.2-3.3) is prior art, not the blueprint.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <string.h>
#include <math.h>
#include <new>
#include <type_traits>

#include "ejoin.h"
#include "ejoin_bench.h"
#include "panel_layout.h"
#include "tile_cursor.h"

namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float float16v __attribute__((ext_vector_type(16)));
typedef float float4v __attribute__((ext_vector_type(4)));

#define EJ_LDS(p) ((__attribute__((address_space(3))) void*)(p))
#define EJ_GLB(p) ((const __attribute__((address_space(1))) void*)(p))

// ------------------------------------------------------------------------------------------
// Tiling constants
// ------------------------------------------------------------------------------------------
constexpr int TILE = 256;     // a workgroup computes a TILE x TILE block of the distance matrix
constexpr int KPAD = 64;      // d is processed rounded up to a multiple of KPAD (zero padded by the caller)
constexpr int KSLICE = 32;    // coordinates per LDS stage (64 B per row)
// Ablation builds (bench_ablation.py) take one design element out at a time; every variant computes the
// same results.  EJOIN_ABL_NSTAGE=3 (one LDS stage less), EJOIN_ABL_NOSWIZZLE (plain LDS rows),
// EJOIN_ABL_ROWMAJOR_TILES (tiles dealt round-robin in row-major order), EJOIN_ABL_NOALIGN (workgroups of
// an XCD never re-aligned), EJOIN_ABL_NOPREFILTER (every block goes through the exact path).
#ifndef EJOIN_ABL_NSTAGE
#define EJOIN_ABL_NSTAGE 4
#endif
// Three measurement builds whose RESULTS ARE MEANINGLESS (timing only, never loaded by the product path or the tests):
// EJOIN_EXP_HOT_PANELS: every global->LDS copy reads one of four panels, so that every copy hits in the L2 while
//   tiles, MFMAs, LDS traffic and operand values stay what they are -- what the memory-side fetch costs in clock.
// EJOIN_EXP_NO_COPIES: after the first NSTAGE slices and the first tile's augmentation operands no global->LDS copy is
//   issued at all, and the rare path is switched off: every later slice computes on what those copies left in the LDS --
//   the same MFMAs, LDS reads and barriers on real operand bits with the copy path, the L2 and the fabric idle: what
//   feeding the LDS costs in cycles and clock (compared with the full kernel at epsilon = 0).
// EJOIN_EXP_CYCLE_MARKS: s_memtime marks between the sections of a tile; the per-section sums of all wavefronts
//   are added into the last 16 u64 of the pair buffer (waves 0-3, then waves 4-7) -- where a tile's cycles go.
#ifdef EJOIN_EXP_HOT_PANELS
#define EJ_PANEL_A(I) ((I) & 1u)
#define EJ_PANEL_B(J) (2u + ((J) & 1u))
#else
#define EJ_PANEL_A(I) (I)
#define EJ_PANEL_B(J) (J)
#endif
constexpr int NSTAGE = EJOIN_ABL_NSTAGE;  // ring of LDS stages; NSTAGE-1 slices are in flight from L2/HBM
constexpr int DIST = NSTAGE - 1;
constexpr int THREADS = 512;  // 8 wavefronts: 2 (rows) x 4 (columns), wave tile 128 x 64
constexpr int SB = (int)EJ_SB;
constexpr int PANEL_BYTES = TILE * KSLICE * 2;  // 16 KB : one operand panel of one stage
constexpr int STAGE_BYTES = 2 * PANEL_BYTES;    // A panel + B panel
constexpr int DUMP_OFF = NSTAGE * STAGE_BYTES;  // 1 KB that absorbs the copies issued past the end of the work
// Operands of the augmentation step of the tile being computed: 16 bytes per row of the A panel (4 KB), 16 bytes per
// column of the B panel (4 KB), and the two constant chunks of that step (layout: panel_layout.h, "a tile's
// augmentation buffer")
constexpr int AUG_OFF = DUMP_OFF + 1024;
constexpr int AUG_PART_BYTES = EJ_AUG_PART;
constexpr int AUGC_OFF = AUG_OFF + EJ_AUG_CONST;
constexpr int AUG_REGION_STEP = EJ_AUG_REGION_STEP;
constexpr int STG_OFF = AUG_OFF + EJ_AUG_BYTES;  // per-wave result staging: STG_CAP entries of (i, j, d2)
constexpr int STG_CAP = 128;
constexpr int STG_WAVE_BYTES = STG_CAP * 12;
constexpr int LDS_BYTES = STG_OFF + 8 * STG_WAVE_BYTES;
constexpr int NUM_XCD = (int)EJ_NUM_XCD;
static_assert(LDS_BYTES <= 160 * 1024, "LDS budget of one CU");
static_assert(NSTAGE == 3 || NSTAGE == 4, "the slice pipeline reads one slice ahead: at least two slices in flight");

// Device status word written by k_aux, read by the other kernels.
constexpr uint32_t ST_OK = 0, ST_NORM_RANGE = 1, ST_NONFINITE = 2;

struct JoinArgs {
  // "points" (rows of the distance matrix) and "query points" (columns); the self-join passes the same set twice
  const uint4* XpA;        // packed copy of the points plus their augmentation block, see k_norms / k_aux
  const uint4* XpB;        // ... of the query points
  int64_t nA, nB;
  int self;                // 1: self-join (upper triangle, self pairs), 0: two different sets (full rectangle)
  uint32_t* status;        // status block of the workspace (see k_reset)
  int nslices;  // roundup(d, 64) / 32 : k-blocks of data per panel = slices per tile (the augmentation block follows them)
  float thr;    // pass <=> acc' >= thr, thr = -eps^2 / 2
  uint32_t ntilesA, ntilesB;  // ceil(n / TILE)
  uint32_t sb_row_begin, sb_row_end;  // rows of super-blocks this launch covers (a join returned in batches is cut by them)
  // pair mode
  uint32_t* pairs;
  float* dist2;
  unsigned long long capacity;
  unsigned long long* n_pairs;
  // count mode
  uint32_t* counts;    // per point (self-join: per point of the one set)
  uint32_t* counts_b;  // per query point (two-set join only; may be null)
  unsigned long long* total;
  // XCD-wide alignment of the workgroups (performance hint, see xcd_align)
  uint32_t* xcd_bar;  // NUM_XCD counters, zeroed before the launch
  int sync_mode;      // 0: never; k > 0: at the start and then before every k-th tile
};

// ------------------------------------------------------------------------------------------
// Small kernels
// ------------------------------------------------------------------------------------------
// Status block of a workspace (64 words): [0] status word, [1] largest norm seen so far in the call (FP32 bits),
// [2..3] the constant C = { c, c, c, 0 } of the call's augmentation step (FP16 bits, written by k_aux),
// [8..15] alignment counters of the XCDs.  Between calls [1] and [8..15] are zero: k_aux clears the counters
// (and the result counter of the call), k_join clears the maximum.  k_reset restores that state after a call
// that did not get as far as its join kernel, and before every call on the shared static workspace.
__global__ void k_reset(uint32_t* status_and_max) {
  if (threadIdx.x < 8) status_and_max[8 + threadIdx.x] = 0;
  if (threadIdx.x == 0) {
    status_and_max[0] = ST_OK;
    status_and_max[1] = 0;
  }
}

// Folds the largest norm of a prepared set (stored as FP32 bits) into the running maximum of a call.
__global__ void k_merge_max(uint32_t* max_bits, const uint32_t* set_max) {
  if (threadIdx.x == 0) atomicMax(max_bits, *set_max);
}

__global__ void k_fill_u32(uint32_t* p, int64_t n, uint32_t v) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

// Step 1 (Section 3.1): s_i = sum_k x_ik^2.  One wavefront per 16 consecutive points; the 16 x 16
// Gram block of those points is accumulated with the same MFMA steps, in the same k order, as
// the join kernel uses, and its diagonal is stored.  That makes s_i bit-identical to a_ii, and
// to a_ij for a duplicate j of i, so duplicates come out at distance exactly 0.  (The paper
// matches its norm rounding to its tensor cores' for the same reason.)  Also tracks max_i s_i
// (as FP32 bits; s >= 0 so unsigned order is numeric order, and NaN/Inf sort above every finite value).
//
// PACK: the same pass also writes the packed copy of X for the join kernel.  A panel (256 points) is cut into
// k-blocks of 32 coordinates; a k-block holds, for each of the panel's rows, the 64 bytes of a row of the LDS
// panel, already arranged the way the LDS wants them (see place_of); points n .. npad-1 are zero.  A k-block is
// 16 KB of contiguous memory, so the global->LDS copies of the join are straight 1 KB block copies made of full
// 128-byte lines (in the row-major X a 32-coordinate slice of a row is half a line, and the L2 would be asked for
// every line twice), and the `blocks` k-blocks of a panel follow each other (packed_index).  The 16 bytes a lane
// loads as its part of the MFMA operand (point l%16, chunk l/16 of the k-block) are exactly one chunk of that layout.
template <bool PACK>
__global__ __launch_bounds__(256) void k_norms(const uint16_t* __restrict__ X, int64_t n, int64_t npad, int64_t ld, int k32steps,
                                               float* __restrict__ s, uint32_t* __restrict__ max_bits, uint4* __restrict__ Xp,
                                               int blocks /* k-blocks per panel of Xp: k32steps + 1 */) {
  const int lane = threadIdx.x & 63;
  const int64_t blk = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  const int64_t row0 = blk * 16;
  if (row0 >= (PACK ? npad : n)) return;
  const int64_t row_own = row0 + (lane & 15);
  int64_t at = 0;
  if (PACK) at = place_of(row_own, lane >> 4);
  if (PACK && row0 >= n) {  // padding rows only
    for (int k = 0; k < k32steps; ++k) Xp[packed_index(at, k, blocks)] = make_uint4(0, 0, 0, 0);
    return;
  }
  const bool valid = row_own < n;
  const int64_t row = valid ? row_own : n - 1;
  const half8* p = reinterpret_cast<const half8*>(X + row * ld) + (lane >> 4);
  float4v acc = {0.f, 0.f, 0.f, 0.f};
  for (int k = 0; k < k32steps; ++k) {
    half8 a = p[4 * k];
    acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, a, acc, 0, 0, 0);
    if (PACK) Xp[packed_index(at, k, blocks)] = valid ? __builtin_bit_cast(uint4, a) : make_uint4(0, 0, 0, 0);
  }
  // element (row, col) of the 16 x 16 block sits in lane col + 16 * (row / 4), register row % 4
  const int c = lane & 15, g = lane >> 4;
  uint32_t bits = 0;
  if ((c >> 2) == g && row0 + c < n) {
    const int want = c & 3;
    float v = 0.f;
#pragma unroll
    for (int r = 0; r < 4; ++r)
      if (r == want) v = acc[r];
    s[row0 + c] = v;
    bits = __float_as_uint(v);
  }
  if (max_bits) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
      const uint32_t o = (uint32_t)__shfl_xor((int)bits, off);
      bits = bits > o ? bits : o;
    }
    if (lane == 0) atomicMax(max_bits, bits);
  }
}

// Rows past the end of the data set carry -60000 c in place of -s/2 (at least the largest norm of the
// data), so that none of their pairs passes the filter for any ordinary epsilon (the rare path masks
// them exactly) and nothing non-finite enters the matrix cores.
constexpr uint32_t P1_OUT_OF_RANGE = 0xFB53u;  // -60000 in FP16

// Augmentation rows.  Step 3 of Section 3.1 (dist^2 = s_i + s_j - 2 a_ij) is folded into the
// matrix-core accumulation: after the Gram steps one more MFMA step (16 wide) adds
// -s_i/2 - s_j/2 to a_ij, so the accumulator ends as acc' = -dist^2 / 2 and the filter becomes a
// sign-like test against -eps^2/2.  -s/2 is FP32; scaled by 2^-m it is split into three FP16 pieces
// p1 + p2 + p3, where m puts the largest norm of the data just below 2^16 (s_max / 2 < 2^15 2^m),
// within -14 <= m <= 15 so that c = 2^m is a normal FP16 value (the matrix cores align the products
// of a step by their exponent fields; a subnormal c would cost them low bits).  The split is exact
// for every point with s >= max(2^-16 s_max, 2^-14): the 24 mantissa bits of s / 2^(m+1) then lie
// above FP16's smallest subnormal.  A smaller norm is carried to 2^-25 2^m absolute.  Point i's
// 16-byte row is  H_i = { P_i, C } = { p1, p2, p3, 0, c, c, c, 0 }; the extra step multiplies
// pieces by constants, c (p1 + p2 + p3)_i + c (q1 + q2 + q3)_j = -s_i/2 - s_j/2, every product exact in FP32.
// H (npad rows) serves the dense-tile kernel.  For the join the operands of the extra step are also
// written, ready made, into one more k-block behind the data k-blocks of each panel of the packed set (`Xp`,
// may be null; k-block `aug_kb` of `blocks`): 16 bytes per row for the panel as the A operand (chunk 0 of
// panel_layout.h, "the augmentation step": 256 x 16 B), then 16 bytes per row for the panel as the B operand
// (chunk 1); the rest of the 16 KB is not used.  The join kernel copies the 4 KB + 4 KB of a tile's two panels
// to the LDS once per tile; the constant chunks 2 and 3 it builds itself from C, which is left in the status block.
// The kernel also clears what the join kernel expects to find zero (the join kernel of the call before has
// finished by now): the XCD alignment counters, the call's result counter `counter` and, in count mode,
// the per-point counts `counts` (n entries; may be null).
__global__ void k_aux(const float* __restrict__ s, int64_t n, int64_t npad, uint32_t* __restrict__ status_and_max,
                      uint4* __restrict__ H, uint4* __restrict__ Xp, int aug_kb, int blocks,
                      unsigned long long* __restrict__ counter, uint32_t* __restrict__ counts) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const uint32_t mb = status_and_max[1];
  if (blockIdx.x == 0) {
    if (threadIdx.x < 8) status_and_max[8 + threadIdx.x] = 0;
    if (threadIdx.x == 8 && counter) *counter = 0;
  }
  if (counts && i < n) counts[i] = 0;
  int m = 0;
  uint32_t st = ST_OK;
  if (mb >= 0x7f800000u) st = ST_NONFINITE;  // Inf or NaN among the norms
  else {
    const int e = (int)(mb >> 23) - 127;  // max s < 2^(e+1)
    m = e - 15 < -14 ? -14 : e - 15;
    if (m > 15) st = ST_NORM_RANGE;  // 2^m must be an FP16 value: needs max s < 2^31
  }
  const _Float16 c = (_Float16)ldexpf(1.f, m > 15 ? 15 : m);
  auto bits = [](_Float16 x) { return (uint32_t)__builtin_bit_cast(uint16_t, x); };
  if (i == 0) {
    status_and_max[0] = st;
    status_and_max[2] = bits(c) | (bits(c) << 16);
    status_and_max[3] = bits(c);
  }
  if (i >= npad) return;
  // the pieces of point x as two 32-bit words { p1 | p2 << 16, p3 }
  auto pieces = [&](int64_t x) -> uint2 {
    if (x >= n) return make_uint2(P1_OUT_OF_RANGE, 0u);
    if (st != ST_OK) return make_uint2(0u, 0u);
    const float v = ldexpf(-0.5f * s[x], -m);
    const _Float16 p1 = (_Float16)v;
    const float r1 = v - (float)p1;
    const _Float16 p2 = (_Float16)r1;
    const _Float16 p3 = (_Float16)(r1 - (float)p2);
    return make_uint2(bits(p1) | (bits(p2) << 16), bits(p3));
  };
  const uint2 cc = (i >= n || st == ST_OK) ? make_uint2(bits(c) | (bits(c) << 16), bits(c)) : make_uint2(0u, 0u);
  const uint2 own = pieces(i);
  H[i] = make_uint4(own.x, own.y, cc.x, cc.y);
  if (Xp) {
    const int r = (int)(i & 31);
    const int64_t b = i - r;
    const int64_t xa = b + aug_row_point(r), xb = b + aug_col_point(r);
    const uint2 a0 = pieces(xa), a1 = pieces(xa + 4), b0 = pieces(xb), b1 = pieces(xb + 16);
    uint4* blk = Xp + packed_index((i >> 8) << 10, aug_kb, blocks);  // the panel's augmentation block
    blk[aug_block_unit((int)(i & 255), 0)] = make_uint4(a0.x, a0.y, a1.x, a1.y);
    blk[aug_block_unit((int)(i & 255), 1)] = make_uint4(b0.x, b0.y, b1.x, b1.y);
  }
}

__device__ __forceinline__ half8 as_half8(uint4 v) { return __builtin_bit_cast(half8, v); }
__device__ __forceinline__ float16v cat4(float4v a, float4v b, float4v c, float4v d) {
  return __builtin_shufflevector(__builtin_shufflevector(a, b, 0, 1, 2, 3, 4, 5, 6, 7), __builtin_shufflevector(c, d, 0, 1, 2, 3, 4, 5, 6, 7),
                                 0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15);
}

// Ingestion: FP32 rows -> FP16 rows in the layout the join expects (row stride ld16, a multiple of 64,
// columns d .. ld16-1 zero).  y = fp16_rne(fl32(scale * fl32(x - center_k))).  One thread per 8 output columns.
__global__ void k_convert_f32(const float* __restrict__ X32, int64_t n, int32_t d, int64_t ld32, const float* __restrict__ center,
                              float scale, uint16_t* __restrict__ X16, int64_t ld16) {
  const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t per_row = ld16 / 8;
  if (t >= n * per_row) return;
  const int64_t i = t / per_row;
  const int k0 = (int)(t - i * per_row) * 8;
  half8 h;
#pragma unroll
  for (int k = 0; k < 8; ++k) {
    float p = 0.f;
    if (k0 + k < d) {
      float t = X32[i * ld32 + k0 + k] - (center ? center[k0 + k] : 0.f);
      asm volatile("" : "+v"(t));  // keep the FP32 rounding of every step: no fused subtract-multiply-convert
      p = scale * t;
    }
    asm volatile("" : "+v"(p));
    h[k] = (_Float16)p;
  }
  *reinterpret_cast<half8*>(X16 + i * ld16 + k0) = h;
}

// Split-FP16 variant (higher accuracy for FP32 inputs).  Each FP32 coordinate is cut into two FP16
// numbers, x ~ hi + lo with hi = fp16(x), lo = fp16(x - hi) (22 significant bits together), and the
// inner product is taken as hi.hi + lo.hi + hi.lo (the lo.lo term is below the 22 bits kept).  That is
// an ordinary inner product of the 3d-dimensional rows A' = [hi | lo | hi] and B' = [hi | hi | lo], so
// the join kernel runs unchanged on two packed arrays: row operands come from A', column operands from
// B'.  This kernel writes both arrays straight from the FP32 rows, in the packed k-block layout of
// k_norms<true> (nkb blocks per part, 3 nkb blocks per array; rows n .. npad-1 and columns d .. are zero).
// Thread t handles the 8 coordinates of one 16-byte chunk.
__global__ void k_split_pack(const float* __restrict__ X32, int64_t n, int64_t npad, int32_t d, int64_t ld32, int nkb,
                             uint4* __restrict__ XpA, uint4* __restrict__ XpB) {
  const int blocks = 3 * nkb + 1;  // k-blocks per panel of either array
  const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t total = (int64_t)nkb * npad * 4;
  if (t >= total) return;
  const int p = (int)(t & 3);
  const int64_t rk = t >> 2;
  const int64_t kb = rk / npad, r = rk - kb * npad;
  int64_t point;
  int chunk;
  stored_at(r, p, point, chunk);
  const int k0 = (int)kb * KSLICE + (chunk << 3);  // first coordinate of the chunk stored here
  half8 hi, lo;
#pragma unroll
  for (int k = 0; k < 8; ++k) {
    const float x = (point < n && k0 + k < d) ? X32[point * ld32 + k0 + k] : 0.f;
    const _Float16 h = (_Float16)x;
    float rest = x - (float)h;
    asm volatile("" : "+v"(rest));  // the residual is an FP32 number: no fused subtract-convert
    hi[k] = h;
    lo[k] = (_Float16)rest;
  }
  const uint4 vh = __builtin_bit_cast(uint4, hi), vl = __builtin_bit_cast(uint4, lo);
  const int64_t place = r * 4 + p;
  const int64_t i0 = packed_index(place, (int)kb, blocks), i1 = packed_index(place, nkb + (int)kb, blocks),
                i2 = packed_index(place, 2 * nkb + (int)kb, blocks);
  XpA[i0] = vh;
  XpA[i1] = vl;
  XpA[i2] = vh;
  XpB[i0] = vh;
  XpB[i1] = vh;
  XpB[i2] = vl;
}

// Norms for the split variant: s_i = A'_i . B'_i, accumulated by the same MFMA steps in the same
// order as the join kernel accumulates a_ii (k-blocks in order, one 32-wide step per block), read
// from the packed arrays.  One wavefront per 16 consecutive points, like k_norms.
__global__ __launch_bounds__(256) void k_norms_packed(const uint4* __restrict__ XpA, const uint4* __restrict__ XpB, int64_t n,
                                                      int64_t npad, int nkb_total, float* __restrict__ s,
                                                      uint32_t* __restrict__ max_bits) {
  const int lane = threadIdx.x & 63;
  const int64_t blk = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  const int64_t row0 = blk * 16;
  if (row0 >= n) return;
  const int g = lane >> 4;
  const int64_t at = place_of(row0 + (lane & 15), g);  // (< npad: points past n are zero)
  float4v acc = {0.f, 0.f, 0.f, 0.f};
  for (int kb = 0; kb < nkb_total; ++kb) {
    const int64_t off = packed_index(at, kb, nkb_total + 1);
    acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_half8(XpA[off]), as_half8(XpB[off]), acc, 0, 0, 0);
  }
  const int c = lane & 15;
  uint32_t bits = 0;
  if ((c >> 2) == g && row0 + c < n) {
    const int want = c & 3;
    float v = 0.f;
#pragma unroll
    for (int r = 0; r < 4; ++r)
      if (r == want) v = acc[r];
    s[row0 + c] = v;
    bits = v < 0.f ? 0u : __float_as_uint(v);  // (a sum that rounds below zero counts as zero; NaN stays NaN)
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) bits = max(bits, (uint32_t)__shfl_xor((int)bits, off));
  if (lane == 0) atomicMax(max_bits, bits);
}

// Dense block of squared distances with the join's arithmetic: one wavefront per 32 x 32 region, computed
// the way the join kernel computes a region of its wave tile: four 16 x 16 blocks accumulated with
// v_mfma_f32_16x16x32_f16, then one v_mfma_f32_32x32x16_f16 on the four blocks' registers side by side that
// adds -s_i/2 - s_j/2 (operand layout: see the augmentation step of k_join).
__global__ __launch_bounds__(64) void k_dist2_tile(const uint16_t* __restrict__ X, const uint4* __restrict__ H,
                                                  const uint32_t* __restrict__ status, int64_t n, int64_t ld, int k32steps,
                                                  int64_t i0, int64_t j0, int rows, int cols, float* __restrict__ out) {
  if (*status != ST_OK) return;
  const int lane = threadIdx.x & 63;
  const int bi = blockIdx.y * 32, bj = blockIdx.x * 32;
  const int r16 = lane & 15, g = lane >> 4;
  auto row_a = [&](int local) { const int64_t r = i0 + bi + local; return r >= n ? n - 1 : r; };
  auto row_b = [&](int local) { const int64_t r = j0 + bj + local; return r >= n ? n - 1 : r; };
  const half8* pa0 = reinterpret_cast<const half8*>(X + row_a(r16) * ld) + g;
  const half8* pa1 = reinterpret_cast<const half8*>(X + row_a(16 + r16) * ld) + g;
  const half8* pb0 = reinterpret_cast<const half8*>(X + row_b(r16) * ld) + g;
  const half8* pb1 = reinterpret_cast<const half8*>(X + row_b(16 + r16) * ld) + g;
  float4v acc[2][2];
  for (int a = 0; a < 2; ++a)
    for (int c = 0; c < 2; ++c) acc[a][c] = float4v{0.f, 0.f, 0.f, 0.f};
  for (int k = 0; k < k32steps; ++k) {
    const half8 a0 = pa0[4 * k], a1 = pa1[4 * k], b0 = pb0[4 * k], b1 = pb1[4 * k];
    acc[0][0] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a0, b0, acc[0][0], 0, 0, 0);
    acc[0][1] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a0, b1, acc[0][1], 0, 0, 0);
    acc[1][0] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a1, b0, acc[1][0], 0, 0, 0);
    acc[1][1] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a1, b1, acc[1][1], 0, 0, 0);
  }
  // augmentation operands: H_x = { p1, p2, p3, 0, c, c, c, 0 } (16 bytes): pieces in .x .y, constant in .z .w
  const int m = lane & 31;
  uint4 ha, hb;
  {
    const int ra = aug_row_point(m), rb = aug_col_point(m);
    const uint4 h0 = H[row_a(ra)], h1 = H[row_a(ra + 4)];
    const uint4 q0 = H[row_b(rb)], q1 = H[row_b(rb + 16)];
    // the four chunks of the operand rows (panel_layout.h, "the augmentation step"), built here from the H rows
    const uint4 chunks_a[4] = {make_uint4(h0.x, h0.y, h1.x, h1.y), make_uint4(0, 0, 0, 0), make_uint4(h0.z, h0.w, 0, 0), make_uint4(0, 0, h0.z, h0.w)};
    const uint4 chunks_b[4] = {make_uint4(0, 0, 0, 0), make_uint4(q0.x, q0.y, q1.x, q1.y), make_uint4(q0.z, q0.w, 0, 0), make_uint4(0, 0, q0.z, q0.w)};
    const int ca = aug_chunk_a(lane), cb = aug_chunk_b(lane);
    ha = chunks_a[0];
    hb = chunks_b[1];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      if (c == ca) ha = chunks_a[c];
      if (c == cb) hb = chunks_b[c];
    }
  }
  const float16v res = __builtin_amdgcn_mfma_f32_32x32x16_f16(as_half8(ha), as_half8(hb), cat4(acc[0][0], acc[0][1], acc[1][0], acc[1][1]), 0, 0, 0);
#pragma unroll
  for (int q = 0; q < 16; ++q) {
    int pi, pj;
    region_pair(lane, q, pi, pj);
    const int rr = bi + pi, cc = bj + pj;
    if (rr < rows && cc < cols) out[(int64_t)rr * cols + cc] = (i0 + rr == j0 + cc) ? 0.f : fmaxf(-2.f * res[q], 0.f);
  }
}

// ------------------------------------------------------------------------------------------
// The join kernel
// ------------------------------------------------------------------------------------------
// Workgroup barrier without the fences of __syncthreads(): those make the compiler wait for every
// outstanding global->LDS copy (vmcnt(0)) at each barrier, which would serialise the copy pipeline.
// The kernel orders its LDS traffic itself: copies are certified with counted vmcnt waits before the
// barrier, and fragment reads are complete once the MFMAs consuming them have issued.
__device__ __forceinline__ void wg_barrier() { asm volatile("s_barrier" ::: "memory"); }

// One global->LDS copy instruction: every lane moves 16 bytes from sbase + voff (sbase uniform) to
// LDS address lds_addr + LDS_IMM + 16 * lane (lds_addr uniform, goes through M0).  Written as inline
// assembly on purpose: for the builtin form the compiler assumes the instruction may also count on
// lgkmcnt, and from then on turns every LDS wait into lgkmcnt(0), which breaks the overlap of
// fragment reads with MFMAs.  The copies are tracked by hand with counted vmcnt waits.
template <int LDS_IMM>
__device__ __forceinline__ void copy16_to_lds(uint32_t lds_addr, const void* sbase, uint32_t voff) {
  asm volatile(
      "s_add_u32 m0, %0, %3\n\t"
      "s_nop 0\n\t"
      "global_load_lds_dwordx4 %1, %2"
      :
      : "s"(lds_addr), "v"(voff), "s"(sbase), "n"(LDS_IMM)
      : "memory", "m0", "scc");
}

// Brings the workgroups of one XCD back in step: each adds one to its XCD's counter and waits until
// the counter reaches `expect` (workgroups per XCD x number of alignments so far).  Workgroups that
// share operand panels only hit each other's lines in the XCD's L2 while they are within a few slices
// of each other.  Purely a performance hint: the wait is bounded, so a grid that is not fully
// resident cannot hang, and nothing depends on the counter's value.  A workgroup that has run out of
// tiles adds 2^24, which satisfies every later expectation of the others.
__device__ __forceinline__ void xcd_align(uint32_t* bar, uint32_t expect) {
  if (threadIdx.x == 0) {
    __hip_atomic_fetch_add(bar, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    for (int spin = 0; spin < 20000; ++spin) {
      if (__hip_atomic_load(bar, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= expect) break;
      __builtin_amdgcn_s_sleep(8);
    }
  }
  __syncthreads();
}

// KEEP_A: the instance for tiles of exactly NSTAGE slices (96 < d <= 128), which leaves a row panel in the LDS across
// the consecutive tiles that share it (see keep_a_cur); the other instance carries none of that logic.
template <bool COUNT, bool KEEP_A>
__global__ __launch_bounds__(THREADS) void k_join(const JoinArgs a) {
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  // the largest norm of the call has been consumed by k_aux: cleared here for the next call
  if (blockIdx.x == 0 && threadIdx.x == 0) a.status[1] = 0;
  if (*a.status != ST_OK) return;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 2, wn = wave & 3;
  const int r16 = lane & 15, g = lane >> 4;
  const int nsl = a.nslices;       // slices per tile (nsl >= 2: d is padded to 64)
  const uint32_t lds0 = (uint32_t)(uintptr_t)lds;
  // the constant chunks of the augmentation step (made visible by the barrier of the prologue)
  if (tid < 8) {
    const uint32_t c0 = a.status[2], c1 = a.status[3];
    *reinterpret_cast<uint4*>(lds + AUGC_OFF + (tid >> 1) * AUG_REGION_STEP + (tid & 1) * 16) =
        (tid & 1) ? make_uint4(0u, 0u, c0, c1) : make_uint4(c0, c1, 0u, 0u);
  }

  // --- global->LDS copies.  One global_load_lds_dwordx4 moves 1 KB (64 lanes x 16 B) = 16 rows of a
  // panel; in the packed layout that is 1 KB of contiguous global memory.  Only waves 4..7 copy: wave
  // 4 + c moves blocks c, c + 4, c + 8, c + 12 of both 16 KB panels of a slice, 8 copy instructions per
  // slice, always (past the end of the work they are pointed at a dump area), so the number of their
  // outstanding copies is a constant.  The copy unit of the CU accepts the instructions one after the
  // other and a wave waits at the issue of its own until they are taken; waves 0..3, which share the
  // SIMDs with 4..7 one to one, issue none and keep the MFMA pipes busy meanwhile.
  const char* XbA = reinterpret_cast<const char*>(a.XpA);
  const char* XbB = reinterpret_cast<const char*>(a.XpB);
  // a panel's k-blocks (16 KB each) follow each other in memory: the data blocks, then the augmentation block
  const int64_t panel_stride = (int64_t)(nsl + 1) * PANEL_BYTES;
  const int cw = wave & 3;
  const bool copier = wave >= 4;
  const uint32_t voff0 = lane * 16 + cw * 1024;
  // (a copy takes its base address in scalar registers; the addresses are uniform, which is said explicitly because the
  // compiler, when it keeps such a pointer in vector registers, does not always move it back by itself)
  auto uniform_ptr = [](const char* p) -> const char* {
    const uint64_t b = reinterpret_cast<uint64_t>(p);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)b), hi = __builtin_amdgcn_readfirstlane((uint32_t)(b >> 32));
    return reinterpret_cast<const char*>(((uint64_t)hi << 32) | lo);
  };
  auto issue_slice = [&](const char* pa_, const char* pb_, uint32_t lds_stage /* LDS address of the stage + cw*1024 */, bool keep_a) {
    const char* pa = uniform_ptr(pa_);
    const char* pb = uniform_ptr(pb_);
    if (!(KEEP_A && keep_a)) {
      copy16_to_lds<0>(lds_stage, pa, voff0);
      copy16_to_lds<4096>(lds_stage, pa, voff0 + 4096);
      copy16_to_lds<8192>(lds_stage, pa, voff0 + 8192);
      copy16_to_lds<12288>(lds_stage, pa, voff0 + 12288);
    }
    copy16_to_lds<PANEL_BYTES>(lds_stage, pb, voff0);
    copy16_to_lds<PANEL_BYTES + 4096>(lds_stage, pb, voff0 + 4096);
    copy16_to_lds<PANEL_BYTES + 8192>(lds_stage, pb, voff0 + 8192);
    copy16_to_lds<PANEL_BYTES + 12288>(lds_stage, pb, voff0 + 12288);
  };
  constexpr int NCOPY = 8;  // copy instructions per slice and copying wave
  // The operands of a tile's augmentation step: 4 KB of panel I's augmentation block and 4 KB of panel J's, into a
  // buffer of their own: eight copy instructions per tile, issued in the tile's first slice (every wave has then left the
  // tile before and its reads of the buffer behind) and read in its last.  In the general instance they are the job of
  // the four waves that do not copy slices, two each, behind their MFMAs of the first slice: they have nothing to do from
  // there to the next barrier, and their copies do not enter the counted waits of the copying waves; they wait for them
  // (nothing else of theirs is outstanding) before the barrier of the tile's last slice.  In the KEEP_A instance, where
  // the copying waves have half the copies and the others no time to spare, the copying waves issue them ahead of the
  // slice's copies (NAUG each) and allow for them in the one counted wait where they are younger than what must have
  // landed (a tile's second slice; from the third on they are older than everything that may be outstanding).
  constexpr bool AUG_BY_IDLE_WAVES = !KEEP_A;
  constexpr int NAUG = 2;
#ifdef EJOIN_EXP_NO_COPIES
  bool aug_copied = false;
#endif
  auto issue_aug = [&](uint32_t I, uint32_t J) {
#ifdef EJOIN_EXP_NO_COPIES
    if (aug_copied) return;
    aug_copied = true;
#endif
    const char* ga = uniform_ptr(XbA + (int64_t)EJ_PANEL_A(I) * panel_stride + (int64_t)nsl * PANEL_BYTES);
    const char* gb = uniform_ptr(XbB + (int64_t)EJ_PANEL_B(J) * panel_stride + (int64_t)nsl * PANEL_BYTES);
    copy16_to_lds<AUG_OFF>(lds0 + cw * 1024, ga, voff0);
    copy16_to_lds<AUG_OFF + AUG_PART_BYTES>(lds0 + cw * 1024, gb, voff0 + AUG_PART_BYTES);
  };

  // --- fragment read addressing (byte offsets inside a stage).  Operands of v_mfma_f32_16x16x32_f16:
  // lane l supplies point l%16 of the fragment, coordinates 8*(l/16) .. +7 of the 32-wide step; in the
  // panel layout (see stored_at) that is row l%32 of the fragment's group of 32 rows, chunk 2 h + l/32
  // for fragment t = 2 T + h.  Group T adds 32 rows = 2048 B (swz unchanged: 32 rows = 8 groups of 4).
  // (= fragment_offset(lane, h) of panel_layout.h on top of the wave's first row)
  uint32_t offA[2], offB[2];
  {
    const int rowA = wm * 128 + (lane & 31), rowB = wn * 64 + (lane & 31);
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      offA[h] = lds0 + rowA * 64 + (((2 * h + (lane >> 5)) ^ swz(rowA)) << 4);
      offB[h] = lds0 + PANEL_BYTES + rowB * 64 + (((2 * h + (lane >> 5)) ^ swz(rowB)) << 4);
    }
  }
  // Operands of the augmentation step (one v_mfma_f32_32x32x16_f16 per 32 x 32 region, see there): lane l
  // supplies row (or column) m = l%32 of the region, k = 8*(l/32) .. +7, and finds its 16 bytes ready made in
  // the LDS (panel_layout.h, "the augmentation step"): the A operand in the A part of the tile's augmentation
  // buffer, row m (chunk 0, k = 0..7) or, for k = 8..15, the constant chunk chosen by bit 3 of m (chunk 2 or 3);
  // the B operand the constant chunk chosen by bit 4 of m (k = 0..7) or column m of the B part (chunk 1,
  // k = 8..15).  Region t adds 32 rows = AUG_REGION_STEP in either place.
  const uint32_t offA_aug = lds0 + AUG_OFF + aug_lds_offset_a(lane, wm * 128);
  const uint32_t offB_aug = lds0 + AUG_OFF + aug_lds_offset_b(lane, wn * 64);
  typedef const __attribute__((address_space(3))) char* lds_cptr;
  typedef const __attribute__((address_space(3))) half8* lds_h8ptr;
  // fragment t (points 16 t .. 16 t + 15 of the wave tile's rows or columns); off: offA or offB (+ stage offset)
  auto frag = [&](uint32_t stage_off, const uint32_t (&off)[2], int t) -> half8 {
    return *reinterpret_cast<lds_h8ptr>((lds_cptr)(uintptr_t)(off[t & 1] + stage_off) + (t >> 1) * 2048);
  };
  // augmentation operand of region t (points 32 t .. 32 t + 31); addr: offA_aug or offB_aug + stage offset
  auto aug_operand = [&](uint32_t addr, int t) -> half8 { return *reinterpret_cast<lds_h8ptr>((lds_cptr)(uintptr_t)addr + t * AUG_REGION_STEP); };

  // acc[mt][nt]: the 16 x 16 block at rows 16 mt, columns 16 nt of the wave tile
  float4v acc[8][4];
  // Four MFMAs: column block nt of half H of the wave tile (rows 64 H .. 64 H + 63); they share their B
  // operand.  (The 16x16x32 shape accumulates 32 products per accumulator access, against 16 for 32x32x16:
  // on operands that toggle, the chip's power limit allows it a 14 % higher rate.)
  auto mma4 = [&](auto first_c, auto h_c, auto nt_c, const half8 (&fa)[4], const half8& b) {
    constexpr bool FIRST = decltype(first_c)::value;
    constexpr int H = decltype(h_c)::value, NT = decltype(nt_c)::value;
    const float4v z = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int t = (NT & 1) ? 3 - u : u;  // up, down, up, down: only one operand changes from one MFMA to the next
      acc[4 * H + t][NT] = __builtin_amdgcn_mfma_f32_16x16x32_f16(fa[t], b, FIRST ? z : acc[4 * H + t][NT], 0, 0, 0);
    }
  };
  // scheduling hints: one LDS read, then `M` MFMAs.  The reads of a half step are spread one by one between
  // its MFMAs (two reads in a row already cost 2-3 %: the MFMA pipe runs dry while the wave issues them).
  auto read_then_mfma = [&](auto m_c) {
    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
    __builtin_amdgcn_sched_group_barrier(0x008, decltype(m_c)::value, 0);
  };

  // --- per-wave result staging (pair mode): entries are appended in LDS and written out in bulk
  // with one atomic per flush (wavefront ballot + prefix ranks + one atomic per wavefront flush).
  uint32_t* stg = reinterpret_cast<uint32_t*>(lds + STG_OFF + wave * STG_WAVE_BYTES);
  uint32_t fill = 0;               // wave-uniform
  unsigned long long hits = 0;     // count mode: pairs found by this wave
  bool dirty = false;              // stores/atomics issued by the rare path of the current tile (see there)
  auto flush = [&]() {
    if (fill == 0) return;
    unsigned long long base = 0;
    if (lane == 0) base = atomicAdd(a.n_pairs, (unsigned long long)fill);
    const uint32_t blo = __builtin_amdgcn_readfirstlane((uint32_t)base);
    const uint32_t bhi = __builtin_amdgcn_readfirstlane((uint32_t)(base >> 32));
    base = ((unsigned long long)bhi << 32) | blo;
    for (uint32_t e = lane; e < fill; e += 64) {
      const unsigned long long idx = base + e;
      if (idx < a.capacity) {
        reinterpret_cast<uint2*>(a.pairs)[idx] = make_uint2(stg[3 * e], stg[3 * e + 1]);
        if (a.dist2) a.dist2[idx] = __uint_as_float(stg[3 * e + 2]);
      }
    }
    fill = 0;
    dirty = true;
  };

  // 32 x 32 regions of this wave's tile that the diagonal of a diagonal tile crosses (bit mt2*2 + nt2)
  uint32_t diag_blocks = 0;
#pragma unroll
  for (int nt = 0; nt < 2; ++nt) {
    const int mt = 2 * wn + nt - 4 * wm;
    if (mt >= 0 && mt < 4) diag_blocks |= 1u << (mt * 2 + nt);
  }

  // ---------------- prologue
  TileCursor tc;
  tc.init(blockIdx.x, gridDim.x, (uint32_t)a.self, a.ntilesA, a.ntilesB, a.sb_row_begin, a.sb_row_end);
  // the tile being computed and the two after it (the copies run up to two tiles ahead, see issue_one)
  uint32_t I = 0, J = 0, In = 0, Jn = 0, In2 = 0, Jn2 = 0;
  bool have = tc.next(I, J);
  // a workgroup that leaves (now, or after its last tile) releases every later alignment of its XCD
  auto xcd_leave = [&]() {
    if (a.sync_mode >= 1 && tid == 0) __hip_atomic_fetch_add(a.xcd_bar + tc.xcd, 1u << 24, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  };
  if (!have) {
    xcd_leave();
    return;
  }
  bool have_next = tc.next(In, Jn);
  bool have_next2 = have_next && tc.next(In2, Jn2);
  uint32_t epoch = 0;
  // tiles until the next re-alignment of the XCD's workgroups (never: a count no workgroup reaches)
  uint32_t sync_left = a.sync_mode >= 1 ? (uint32_t)a.sync_mode : 0xFFFFFFFFu;
  if (a.sync_mode >= 1) xcd_align(a.xcd_bar + tc.xcd, tc.wpx * ++epoch);
  uint32_t G = 0;  // slices computed so far (stage = G % NSTAGE); slices issued so far = G + DIST
  // The issue cursor runs DIST slices ahead of the compute cursor: slice `iks` (0 .. nsl-1) of the tile
  // `ahead` tiles after the one being computed.  With nsl >= 2 and DIST <= 3 that is at most two tiles ahead
  // (two when a tile has no more slices than are in flight: d <= 96).  After the last tile it keeps issuing
  // copies of valid memory into the dump area.
  int iks = 0;
  int ahead = 0;
  bool issue_live = true;       // the issue cursor points at real work
  // KEEP_A (a tile has exactly as many slices as the ring has stages, 96 < d <= 128): slice ks of every tile lands in
  // stage ks.  Three of four consecutive tiles of a workgroup have the same row panel (tile_cursor.h): the A half of
  // each stage then already holds what the next tile needs, and the copies of its A panel are left out (NCOPY / 2 per
  // slice instead of NCOPY; the counted waits are told through the flags of the tile being issued, the tile being
  // computed and the one after it).
  uint32_t issue_I = I;
  bool keep_a_issue = false, keep_a_cur = false, keep_a_next = false;
  const char* pa = XbA + (int64_t)EJ_PANEL_A(I) * panel_stride;
  const char* pb = XbB + (int64_t)EJ_PANEL_B(J) * panel_stride;
  const uint32_t lds_w = lds0 + cw * 1024;
  auto issue_one = [&](uint32_t Gissue) {
    if (!copier) return;
#ifdef EJOIN_EXP_NO_COPIES
    if (Gissue >= (uint32_t)NSTAGE) return;
#endif
    if (issue_live) {
      issue_slice(pa, pb, lds_w + (Gissue % NSTAGE) * STAGE_BYTES, keep_a_issue);
    } else {
#pragma unroll
      for (int q = 0; q < NCOPY; ++q) copy16_to_lds<0>(lds0 + DUMP_OFF, XbA, lane * 16);
    }
    pa += PANEL_BYTES;
    pb += PANEL_BYTES;
    if (++iks == nsl) {
      iks = 0;
      ++ahead;
      const bool first_after = ahead == 1;
      issue_live = first_after ? have_next : have_next2;
      const uint32_t ti = first_after ? In : In2, tj = first_after ? Jn : Jn2;
      pa = XbA + (int64_t)(issue_live ? EJ_PANEL_A(ti) : 0) * panel_stride;
      pb = XbB + (int64_t)(issue_live ? EJ_PANEL_B(tj) : 0) * panel_stride;
      if constexpr (KEEP_A) {
        keep_a_issue = issue_live && ti == issue_I;
        keep_a_next = keep_a_issue;  // (with nsl == NSTAGE the cursor is one tile ahead at every wrap)
        issue_I = ti;
      }
    }
  };
  for (int q = 0; q < DIST; ++q) issue_one(q);
  // slice 0 has landed when only the copies of the DIST-1 younger slices (NCOPY per slice and copying wave) are
  // outstanding (the waves that do not copy have nothing outstanding: their waits pass at once)
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(NCOPY * (DIST - 1)) : "memory");
  __syncthreads();
  using T_ = std::true_type;
  using F_ = std::false_type;
  using I0_ = std::integral_constant<int, 0>;
  using I1_ = std::integral_constant<int, 1>;
  using I2_ = std::integral_constant<int, 2>;
  using I3_ = std::integral_constant<int, 3>;
  using I4_ = std::integral_constant<int, 4>;
  using I6_ = std::integral_constant<int, 6>;
  // Fragment registers: the A fragments of the two halves of the wave tile and the four B fragments.  A slice
  // starts with faL and fb[0..2] in registers (read under the slice before); fb[3] and faH follow under its first half.
  half8 faL[4], faH[4], fb[4];
  auto load_first = [&](uint32_t stage_off) {
#pragma unroll
    for (int t = 0; t < 4; ++t) faL[t] = frag(stage_off, offA, t);
#pragma unroll
    for (int t = 0; t < 3; ++t) fb[t] = frag(stage_off, offB, t);
  };
  load_first(0);

  // One slice (G-th of the stream) = one 32-wide step: 32 MFMAs, upper half of the wave tile then lower half, each
  // column block by column block.  A B fragment is dead after its four MFMAs of the lower half, and the fragment of
  // the next slice is read into its place right away; the A fragments of the upper half are re-read under the lower
  // half.  FIRST: first slice of a tile (accumulators start from zero).  oa, ob: lane addresses of this slice's
  // fragments, oa_n, ob_n: of the next slice's, which the barrier of this slice has certified.
  auto mma_slice = [&](auto first_c, auto last_c, uint32_t st_cur, uint32_t st_nxt) {
    constexpr bool LAST = decltype(last_c)::value;
    fb[3] = frag(st_cur, offB, 3);
#pragma unroll
    for (int t = 0; t < 4; ++t) faH[t] = frag(st_cur, offA, 4 + t);
    mma4(first_c, I0_{}, I0_{}, faL, fb[0]);
    mma4(first_c, I0_{}, I1_{}, faL, fb[1]);
    mma4(first_c, I0_{}, I2_{}, faL, fb[2]);
    mma4(first_c, I0_{}, I3_{}, faL, fb[3]);
    read_then_mfma(I3_{});
    read_then_mfma(I3_{});
    read_then_mfma(I3_{});
    read_then_mfma(I3_{});
    read_then_mfma(I4_{});
    __builtin_amdgcn_sched_barrier(0);  // keep the two halves apart: each has its own interleave pattern
    if constexpr (!LAST) {
      faL[0] = frag(st_nxt, offA, 0);
      faL[1] = frag(st_nxt, offA, 1);
      mma4(first_c, I1_{}, I0_{}, faH, fb[0]);
      fb[0] = frag(st_nxt, offB, 0);
      faL[2] = frag(st_nxt, offA, 2);
      mma4(first_c, I1_{}, I1_{}, faH, fb[1]);
      fb[1] = frag(st_nxt, offB, 1);
      faL[3] = frag(st_nxt, offA, 3);
      mma4(first_c, I1_{}, I2_{}, faH, fb[2]);
      fb[2] = frag(st_nxt, offB, 2);
      mma4(first_c, I1_{}, I3_{}, faH, fb[3]);
      read_then_mfma(I2_{});
      read_then_mfma(I2_{});
      read_then_mfma(I2_{});
      read_then_mfma(I2_{});
      read_then_mfma(I2_{});
      read_then_mfma(I2_{});
      read_then_mfma(I4_{});
    } else {
      // the augmentation step follows: its six operands go where the fragments would
      // (faL[t]: A operand of region t, fb[0], fb[1]: B operands)
      const uint32_t oa_n = offA_aug, ob_n = offB_aug;
      faL[0] = aug_operand(oa_n, 0);
      faL[1] = aug_operand(oa_n, 1);
      mma4(first_c, I1_{}, I0_{}, faH, fb[0]);
      fb[0] = aug_operand(ob_n, 0);
      faL[2] = aug_operand(oa_n, 2);
      mma4(first_c, I1_{}, I1_{}, faH, fb[1]);
      fb[1] = aug_operand(ob_n, 1);
      faL[3] = aug_operand(oa_n, 3);
      mma4(first_c, I1_{}, I2_{}, faH, fb[2]);
      mma4(first_c, I1_{}, I3_{}, faH, fb[3]);
      read_then_mfma(I2_{});
      read_then_mfma(I2_{});
      read_then_mfma(I2_{});
      read_then_mfma(I2_{});
      read_then_mfma(I2_{});
      read_then_mfma(I6_{});
    }
  };
  // One slice.  LAST: last slice of a tile (what is read ahead are the operands of the augmentation step).
  // COPIER: the instance the copying waves run; the other waves run one without any copy code in it
  // (the copy instructions are opaque to the scheduler and would break up the MFMA / LDS-read interleave for nothing).
  // second: the slice after a tile's first.
  auto data_slice = [&](auto first_c, auto last_c, auto copier_c, bool second) {
    constexpr bool FIRST = decltype(first_c)::value;
    constexpr bool COPIER = decltype(copier_c)::value;
    const uint32_t st_cur = (G % NSTAGE) * STAGE_BYTES, st_nxt = ((G + 1) % NSTAGE) * STAGE_BYTES;
    // (a) this wave's copies of slice G+1 have landed once only those of slice G+2 are outstanding.
    //     A tile whose A panel was kept has NCOPY / 2 copies per slice; the slice two ahead belongs to the tile being
    //     computed in its first two slices and to the next one after that (KEEP_A: nsl == NSTAGE).
    //     The waves that do not copy slices have at most the tile's augmentation copies outstanding, which must have
    //     landed before the barrier of the last slice.
    constexpr bool LAST_ = decltype(last_c)::value;
    if constexpr (!COPIER) {
      if constexpr (AUG_BY_IDLE_WAVES && LAST_) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    } else if constexpr (AUG_BY_IDLE_WAVES) {
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"(NCOPY * (DIST - 2)) : "memory");
    } else if (KEEP_A && ((FIRST || second) ? keep_a_cur : keep_a_next)) {
      if (DIST >= 3 && second) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(NCOPY / 2 * (DIST - 2) + NAUG) : "memory");
      else asm volatile("s_waitcnt vmcnt(%0)" ::"n"(NCOPY / 2 * (DIST - 2)) : "memory");
    } else if (DIST >= 3 && second) {
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"(NCOPY * (DIST - 2) + NAUG) : "memory");
    } else {
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"(NCOPY * (DIST - 2)) : "memory");
    }
    // (b) after the barrier slice G+1 is complete in LDS for everybody, and everybody is done with slice G-1
    wg_barrier();
    // (c) the copying waves refill the stage slice G-1 occupied with slice G+DIST, while the other wave of
    //     their SIMD starts on the MFMAs of the slice
    if constexpr (COPIER && FIRST && !AUG_BY_IDLE_WAVES) issue_aug(I, J);
    if constexpr (COPIER) issue_one(G + DIST);
    // (d) the MFMAs of slice G, overlapped with the LDS reads of what follows
    mma_slice(first_c, last_c, st_cur, st_nxt);
    if constexpr (!COPIER && FIRST && AUG_BY_IDLE_WAVES) issue_aug(I, J);
    ++G;
  };

#ifdef EJOIN_EXP_CYCLE_MARKS
  // sections: 0 tile cursor, 1 first slice, 2 middle slices, 3 last slice, 4 augmentation MFMAs + filter + exact path,
  // 5 reads of the next tile's first fragments (a mark waits for them to arrive: the section is their latency),
  // 6 the periodic re-alignment of the XCD's workgroups, 7 the wait for all copies in flight before it
  unsigned long long mark_sum[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  unsigned long long mark_prev = __builtin_amdgcn_s_memtime();
#define EJ_MARK(k)                                                  \
  {                                                                 \
    const unsigned long long now_ = __builtin_amdgcn_s_memtime();   \
    mark_sum[k] += now_ - mark_prev;                                \
    mark_prev = now_;                                               \
  }
#else
#define EJ_MARK(k)
#endif
  while (have) {
    // ---------------- the nsl >= 2 slices of the tile
    EJ_MARK(0)
    if (copier) {
      data_slice(T_{}, F_{}, T_{}, false);
      EJ_MARK(1)
      for (int ks = 1; ks < nsl - 1; ++ks) data_slice(F_{}, F_{}, T_{}, ks == 1);
      EJ_MARK(2)
      data_slice(F_{}, T_{}, T_{}, false);
    } else {
      data_slice(T_{}, F_{}, F_{}, false);
      EJ_MARK(1)
      for (int ks = 1; ks < nsl - 1; ++ks) data_slice(F_{}, F_{}, F_{}, false);
      EJ_MARK(2)
      data_slice(F_{}, T_{}, F_{}, false);
    }
    EJ_MARK(3)
    // ---------------- the augmentation step, then the filter.
    // The step adds -s_i/2 - s_j/2 to every accumulator with eight v_mfma_f32_32x32x16_f16, one per 32 x 32
    // region of the wave tile, half the matrix-core time that 32 more 16x16x32 (with 26 of 32 products zero)
    // would take.  A region's accumulator is its four 16 x 16 blocks' registers side by side, R = (mt2, nt2):
    // register q = 8 a + 4 c + r of lane l holds the pair  i = 16 a + 4 (l/16) + r,  j = 16 c + l%16  of the
    // region, where the 32 x 32 MFMA puts its element  m = 8 (q/4) + 4 (l/32) + q%4,  n = l%32.  So the step
    // needs  D[m][n] = -s_i/2 - s_j/2  with  i = i(m; bit 4 of n),  j = j(n%16; bit 3 of m),  which is bilinear
    // in indicator columns:  row m of the A operand = { P(i(m;0)), P(i(m;1)), c [bit3(m)=0], c [bit3(m)=1] },
    // row n of the B operand = { c [bit4(n)=0], c [bit4(n)=1], P(j(n;0)), P(j(n;1)) }, where P(x) = {p1, p2, p3, 0}
    // are the pieces of -s_x/2 and c stands for {c, c, c, 0}.  Of the 16 products of an element 6 are non-zero
    // and each is exact, as in a plain { P, c } . { c, P } step.
    float16v R[4][2];
    {
#pragma unroll
      for (int mt2 = 0; mt2 < 4; ++mt2)
#pragma unroll
        for (int nt2 = 0; nt2 < 2; ++nt2)
          R[mt2][nt2] = __builtin_amdgcn_mfma_f32_32x32x16_f16(
              faL[mt2], fb[nt2], cat4(acc[2 * mt2][2 * nt2], acc[2 * mt2][2 * nt2 + 1], acc[2 * mt2 + 1][2 * nt2], acc[2 * mt2 + 1][2 * nt2 + 1]),
              0, 0, 0);
    }
    {
      // acc' = a_ij - s_i/2 - s_j/2 = -dist^2/2 ; register r of block (mt, nt) in lane l is the pair
      //   i = I*256 + wm*128 + mt*16 + 4*(l/16) + r ,  j = J*256 + wn*64 + nt*16 + l%16.
      const bool diag = a.self && (I == J);
      // a wave tile of a diagonal block that lies entirely below the diagonal holds no pair i <= j
      const bool skip = diag && (wm * 128 >= wn * 64 + 64);
      // cheap filter: which of the eight 32 x 32 regions of this wave tile (2 x 2 blocks each, bit mt2*2 + nt2)
      // hold a passing pair at all
      uint32_t blocks_hit = 0;
      {
        // x >= thr for a threshold thr <= 0 reads, on the bit patterns taken as unsigned integers, bits(x) <=
        // bits(thr) with thr's sign bit set: a positive x has a smaller pattern than any negative number, and a
        // negative one passes iff its magnitude is at most |thr|.  (A NaN with a clear sign bit would be flagged;
        // the exact path below compares as floats and drops it.)  Integer minima need no NaN quieting, which
        // costs the float version two more instructions per region.
        const uint32_t thr_bits = __float_as_uint(a.thr) | 0x80000000u;
#pragma unroll
        for (int mt2 = 0; mt2 < 4; ++mt2) {
#pragma unroll
          for (int nt2 = 0; nt2 < 2; ++nt2) {
            const float16v& v = R[mt2][nt2];
            auto u = [&](int r) { return __float_as_uint(v[r]); };
            uint32_t m = min(min(u(0), u(1)), u(2));
#pragma unroll
            for (int r = 3; r < 15; r += 2) m = min(min(m, u(r)), u(r + 1));
            m = min(m, u(15));
            if (__ballot(m <= thr_bits)) blocks_hit |= 1u << (mt2 * 2 + nt2);
          }
        }
        // the filter of a region only needs that region's MFMA: let the VALU work of a region run
        // under the augmentation MFMAs of the regions after it
        __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
#pragma unroll
        for (int b = 0; b < 6; ++b) {
          __builtin_amdgcn_sched_group_barrier(0x002, 9, 0);
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        }
      }
#ifdef EJOIN_ABL_NOPREFILTER
      blocks_hit = 0xFF;
#endif
#ifdef EJOIN_EXP_NO_COPIES
      blocks_hit = 0;  // (every tile holds the first tile's distances: keep the rare path out of the comparison)
#endif
      if (skip) blocks_hit = 0;
      else if (diag && !COUNT) blocks_hit |= diag_blocks;  // self pairs are emitted whatever the arithmetic says
      // rare path, one block at a time.  Two instances: the common one for tiles off the diagonal, and
      // the one for diagonal tiles of the self-join, which keeps i < j only and emits the self pairs.
      auto exact_path = [&](auto diag_c) {
        constexpr bool DIAG = decltype(diag_c)::value;
        while (blocks_hit) {
          const int b = __builtin_ctz(blocks_hit);
          blocks_hit &= blocks_hit - 1;
          float16v v;  // element q = 8 a + 4 c + r : register r of block (2 mt2 + a, 2 nt2 + c)
          switch (b) {
            case 0: v = R[0][0]; break;
            case 1: v = R[0][1]; break;
            case 2: v = R[1][0]; break;
            case 3: v = R[1][1]; break;
            case 4: v = R[2][0]; break;
            case 5: v = R[2][1]; break;
            case 6: v = R[3][0]; break;
            default: v = R[3][1]; break;
          }
          asm volatile("" : "+v"(v));  // one copy of the region's registers, in one place (the compiler otherwise makes two)
          const int mt2 = b >> 1, nt2 = b & 1;
          const uint32_t nnA = (uint32_t)a.nA, nnB = (uint32_t)a.nB;
          // region_pair(lane, r) with the lane's part taken out of the loop
          const uint32_t jb = J * TILE + wn * 64 + nt2 * 32 + r16;
          const uint32_t ib = I * TILE + wm * 128 + mt2 * 32 + 4 * g;
          // Which of the region's four 16 x 16 blocks (registers 4 q .. 4 q + 3) hold a candidate at all: the filter's
          // test again, on a quarter of the registers each.  Usually one does, and the other twelve registers are
          // not looked at one by one.  (Diagonal tiles scan everything: their self pairs are not found by value.)
          uint32_t quarters = 0xF;
          if (!DIAG) {
            const uint32_t thr_bits = __float_as_uint(a.thr) | 0x80000000u;
            quarters = 0;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
              const uint32_t m = min(min(min(__float_as_uint(v[4 * q]), __float_as_uint(v[4 * q + 1])), __float_as_uint(v[4 * q + 2])),
                                     __float_as_uint(v[4 * q + 3]));
              if (__ballot(m <= thr_bits)) quarters |= 1u << q;
            }
          }
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            if (!((quarters >> (r >> 2)) & 1)) continue;
            const uint32_t i = ib + 16 * (r >> 3) + (r & 3);
            const uint32_t j = jb + 16 * ((r >> 2) & 1);
            // (i, i) belongs to the result by definition, whatever the arithmetic says
            const bool selfp = DIAG && !COUNT && i == j && i < nnA;
            if (__ballot(v[r] >= a.thr || selfp) == 0) continue;  // most registers of a flagged block hold no hit
            // rows/columns past n carry a large negative marker, which a huge epsilon can still reach: mask them here
            bool pass = v[r] >= a.thr && i < nnA && j < nnB;
            if (DIAG) pass = (pass && i < j) || selfp;
            const unsigned long long mask = __ballot(pass);
            if (mask) {
              const uint32_t cnt = __popcll(mask);
              if (COUNT) {
                if (pass) {
                  atomicAdd(&a.counts[i], 1u);
                  if (a.self) atomicAdd(&a.counts[j], 1u);
                  else if (a.counts_b) atomicAdd(&a.counts_b[j], 1u);
                }
                hits += cnt;
                dirty = true;
              } else {
                if (fill + cnt > STG_CAP) flush();
                const uint32_t rank = __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
                if (pass) {
                  const uint32_t e = fill + rank;
                  stg[3 * e] = i;
                  stg[3 * e + 1] = j;
                  stg[3 * e + 2] = selfp ? 0u : __float_as_uint(fmaxf(-2.f * v[r], 0.f));
                }
                fill += cnt;
              }
            }
          }
        }
      };
      if (blocks_hit) {
        if (diag) exact_path(T_{});
        else exact_path(F_{});
        // The stores and atomics of the path count on vmcnt like the copies, but complete in any order: the counted
        // waits of the slices hold only once they are all done.
        if (dirty) {
          asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
          dirty = false;
        }
      }
    }
    EJ_MARK(4)
    // first fragments of the next tile (slice G was certified by the barrier of the tile's last slice);
    // read after the filter to keep its registers free
    load_first((G % NSTAGE) * STAGE_BYTES);
    EJ_MARK(5)
    I = In;
    J = Jn;
    have = have_next;
    In = In2;
    Jn = Jn2;
    have_next = have_next2;
    --ahead;  // (at least 1 before: the issue cursor has left the tile that was just finished)
    if constexpr (KEEP_A) keep_a_cur = keep_a_next;
    if (have) {
      if (--sync_left == 0) {
        sync_left = (uint32_t)a.sync_mode;
        EJ_MARK(0)
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        EJ_MARK(7)
        xcd_align(a.xcd_bar + tc.xcd, tc.wpx * ++epoch);
        EJ_MARK(6)
      }
      have_next2 = have_next && tc.next(In2, Jn2);
    }
  }
#ifdef EJOIN_EXP_CYCLE_MARKS
  if (lane == 0 && !COUNT && a.capacity >= 16) {
    unsigned long long* out = reinterpret_cast<unsigned long long*>(a.pairs) + (a.capacity - 16) + 8 * (wave >> 2);
    for (int k = 0; k < 8; ++k) atomicAdd(out + k, mark_sum[k]);
  }
#endif
  xcd_leave();
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the dump copies must land before the wave ends
  if (!COUNT) flush();
  if (COUNT && hits && lane == 0) atomicAdd(a.total, hits);
}


}  // namespace

// ------------------------------------------------------------------------------------------
// Host side
// ------------------------------------------------------------------------------------------

// Workspace of the allocation-free entry point (ejoin_selfjoin_pairs_noalloc): device memory that exists from
// the moment the library is loaded, one copy per GPU.  Host code never uses this name as an address; it asks
// the runtime for the device address once per context (ejoin_create) and passes that to the kernels.
static __device__ __align__(256) unsigned char scratch[EJOIN_STATIC_SCRATCH_BYTES];

namespace {

// Device memory one call works in: either the context's own (grown on demand) or a carving of the static scratch.
struct Workspace {
  uint32_t* status;  // status block, 64 words (see k_reset)
  float* s;          // norms (4 B per point)
  uint4* H;          // augmentation rows (16 B per point, padded to a multiple of TILE)
  uint4* Xp;         // packed copy of X plus the augmentation k-block
};

}  // namespace

struct ejoin_ctx {
  int device;
  int num_cu;
  Workspace ws;      // owned by the context
  int64_t s_cap;     // points ws.s and ws.H hold
  int64_t xp_bytes;  // bytes of ws.Xp
  bool ws_dirty;     // a call on ws did not reach its join kernel: the status block may hold leftovers
  unsigned char* static_scratch;  // device address of `scratch` on this context's device
  uint32_t* last_status;          // status block of the last join or dense-tile call, and the stream it ran on
  hipStream_t last_stream;
  int profiling;
  hipEvent_t ev[4];
  int ev_valid;
  // batched result return (ejoin_selfjoin_pairs_to_host): a stream for the device-to-host copies, one event per
  // batch and the pair counter's value after each batch (pinned host memory)
  hipStream_t copy_stream;
  hipEvent_t batch_ev[EJOIN_MAX_BATCHES];
  unsigned long long* batch_count;
  char hip_error[256];
};

// A point set prepared once for many joins: its packed copy (data k-blocks + room for the augmentation
// block, which depends on the other set of each join and is rewritten per call), norms and largest norm.
struct ejoin_set {
  ejoin_ctx* ctx;
  int64_t n, pad;
  int32_t d;
  uint4* Xp;
  float* s;
  uint4* H;
  uint32_t* max_bits;  // device: FP32 bits of the largest norm
};

namespace {

int fail_hip(ejoin_ctx* ctx, hipError_t e, const char* what) {
  if (ctx) snprintf(ctx->hip_error, sizeof(ctx->hip_error), "%s: %s", what, hipGetErrorString(e));
  (void)hipGetLastError();
  return EJOIN_EHIP;
}

#define EJ_TRY(call)                                     \
  do {                                                   \
    hipError_t e_ = (call);                              \
    if (e_ != hipSuccess) return fail_hip(ctx, e_, #call); \
  } while (0)
#define EJ_RC(call)                 \
  do {                              \
    const int rc_ = (call);         \
    if (rc_ != EJOIN_OK) return rc_; \
  } while (0)

int64_t pad_rows(int64_t n) { return (n + TILE - 1) / TILE * TILE; }
int64_t pad_dims(int32_t d) { return ((int64_t)d + KPAD - 1) / KPAD * KPAD; }
int k_blocks(int32_t d) { return (int)(pad_dims(d) / KSLICE); }  // 32-coordinate k-blocks = MFMA steps per inner product

int check_common(const ejoin_ctx* ctx, const void* X, int64_t n, int32_t d, int64_t ld) {
  if (!ctx || !X) return EJOIN_EINVAL;
  if (n < 1 || n >= (int64_t)0xFFFFFFFFll - TILE) return EJOIN_EINVAL;
  if (d < 1 || d > 65536) return EJOIN_EINVAL;
  if (ld < pad_dims(d) || (ld % KPAD) != 0) return EJOIN_EINVAL;
  if ((reinterpret_cast<uintptr_t>(X) & 127) != 0) return EJOIN_EINVAL;
  return EJOIN_OK;
}

bool bad_eps(float eps) { return !(eps >= 0.f) || !isfinite(eps); }

// Bytes of packed copy for `rows` (padded) points of dpad coordinates: the data k-blocks plus the augmentation block.
int64_t packed_bytes(int64_t rows, int64_t dpad) { return rows * (dpad + KSLICE) * 2; }

// The context's own workspace for `rows` points in total (each set padded to a multiple of TILE).
// dpad = 0: only the per-point arrays (norms, augmentation rows); dpad > 0: also the packed copies.
// Growing frees the old arrays, which first waits for the device to be idle.
int ensure_workspace(ejoin_ctx* ctx, int64_t rows, int64_t dpad) {
  Workspace& w = ctx->ws;
  if (rows > ctx->s_cap) {
    if (w.s || w.H) {
      EJ_TRY(hipDeviceSynchronize());
      if (w.s) EJ_TRY(hipFree(w.s));
      w.s = nullptr;
      if (w.H) EJ_TRY(hipFree(w.H));
      w.H = nullptr;
      ctx->s_cap = 0;
    }
    hipError_t e = hipMalloc(reinterpret_cast<void**>(&w.s), (size_t)rows * sizeof(float));
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&w.H), (size_t)rows * sizeof(uint4));
    if (e != hipSuccess) {
      (void)hipGetLastError();
      if (w.s) (void)hipFree(w.s);
      w.s = nullptr;
      if (e == hipErrorOutOfMemory) return EJOIN_ENOMEM;
      return fail_hip(ctx, e, "hipMalloc(workspace)");
    }
    ctx->s_cap = rows;
  }
  const int64_t need = dpad > 0 ? packed_bytes(rows, dpad) : 0;
  if (need > ctx->xp_bytes) {
    if (w.Xp) {
      EJ_TRY(hipDeviceSynchronize());
      EJ_TRY(hipFree(w.Xp));
      w.Xp = nullptr;
      ctx->xp_bytes = 0;
    }
    hipError_t e = hipMalloc(reinterpret_cast<void**>(&w.Xp), (size_t)need);
    if (e != hipSuccess) {
      (void)hipGetLastError();
      if (e == hipErrorOutOfMemory) return EJOIN_ENOMEM;
      return fail_hip(ctx, e, "hipMalloc(packed X)");
    }
    ctx->xp_bytes = need;
  }
  return EJOIN_OK;
}

// The static scratch cut up for a self-join of `pad` (padded) points of dpad coordinates; false if it does not fit.
// Every piece starts on a 256-byte boundary.
bool carve_static(unsigned char* base, int64_t pad, int64_t dpad, Workspace& w) {
  auto up = [](int64_t x) { return (x + 255) / 256 * 256; };
  const int64_t off_s = 256, off_H = off_s + up(pad * 4), off_Xp = off_H + up(pad * 16);
  const int64_t end = off_Xp + packed_bytes(pad, dpad);
  if (end > (int64_t)EJOIN_STATIC_SCRATCH_BYTES) return false;
  w.status = reinterpret_cast<uint32_t*>(base);
  w.s = reinterpret_cast<float*>(base + off_s);
  w.H = reinterpret_cast<uint4*>(base + off_H);
  w.Xp = reinterpret_cast<uint4*>(base + off_Xp);
  return true;
}

// Norms of X into s (and, with Xp given, the packed copy of X); max_bits may be null.
int launch_norms(ejoin_ctx* ctx, const uint16_t* X, int64_t n, int32_t d, int64_t ld, float* s, uint32_t* max_bits, uint4* Xp,
                 hipStream_t st) {
  const int64_t npad = pad_rows(n);
  const int64_t waves = ((Xp ? npad : n) + 15) / 16;
  const dim3 grid((unsigned)((waves + 3) / 4));
  if (Xp) hipLaunchKernelGGL(k_norms<true>, grid, dim3(256), 0, st, X, n, npad, ld, k_blocks(d), s, max_bits, Xp, k_blocks(d) + 1);
  else hipLaunchKernelGGL(k_norms<false>, grid, dim3(256), 0, st, X, n, npad, ld, k_blocks(d), s, max_bits, Xp, 0);
  EJ_TRY(hipGetLastError());
  return EJOIN_OK;
}

// Augmentation rows of one set from its norms and the running maximum of all norms.
// Xp: the set's packed copy, whose panels get their augmentation k-block (k-block number `data_blocks`, behind the
// data blocks; null for the dense-tile call); counter / counts: what the kernel clears on the way (may be null).
int launch_aux(ejoin_ctx* ctx, uint32_t* status, const float* s, int64_t n, uint4* H, uint4* Xp, int data_blocks,
               unsigned long long* counter, uint32_t* counts, hipStream_t st) {
  const int64_t npad = pad_rows(n);
  hipLaunchKernelGGL(k_aux, dim3((unsigned)(npad / 256)), dim3(256), 0, st, s, n, npad, status, H, Xp, data_blocks, data_blocks + 1, counter,
                     counts);
  EJ_TRY(hipGetLastError());
  return EJOIN_OK;
}

struct DeviceGuard {
  int prev;
  bool ok;
  explicit DeviceGuard(int dev) : prev(-1), ok(false) {
    if (hipGetDevice(&prev) != hipSuccess) return;
    ok = (prev == dev) || (hipSetDevice(dev) == hipSuccess);
  }
  ~DeviceGuard() {
    int cur = -1;
    if (prev >= 0 && hipGetDevice(&cur) == hipSuccess && cur != prev) (void)hipSetDevice(prev);
  }
};

// Where a call's results go.
struct Results {
  uint32_t* pairs = nullptr;
  float* dist2 = nullptr;
  uint64_t capacity = 0;
  uint64_t* n_pairs = nullptr;
  uint32_t* counts = nullptr;
  uint32_t* counts_b = nullptr;
  uint64_t* total = nullptr;
  unsigned long long* counter(bool count) const { return reinterpret_cast<unsigned long long*>(count ? total : n_pairs); }
};

// One packed operand set of a join.
struct Operand {
  const uint4* Xp;
  int64_t n, pad;
};

// Opens a call on workspace w: first profiling event, and the status block brought to its between-calls state
// if it may not be in it (always for the static scratch, which every context of the device shares).
int begin_call(ejoin_ctx* ctx, const Workspace& w, bool own, hipStream_t st) {
  if (ctx->profiling) EJ_TRY(hipEventRecord(ctx->ev[0], st));
  if (!own || ctx->ws_dirty) {
    hipLaunchKernelGGL(k_reset, dim3(1), dim3(64), 0, st, w.status);
    EJ_TRY(hipGetLastError());
  }
  if (own) ctx->ws_dirty = true;  // until the join kernel, which leaves the block clean, has been launched
  ctx->last_status = w.status;
  ctx->last_stream = st;
  return EJOIN_OK;
}

// The join kernel on two packed operand sets whose augmentation blocks are in place.
template <bool COUNT>
int launch_join(ejoin_ctx* ctx, const Workspace& w, bool own, const Operand& A, const Operand& B, bool self, int nslices, float eps,
                const Results& r, hipStream_t st, uint32_t sb_row_begin = 0, uint32_t sb_row_end = 0xFFFFFFFFu) {
  JoinArgs a;
  memset(&a, 0, sizeof(a));
  a.XpA = A.Xp;
  a.XpB = B.Xp;
  a.nA = A.n;
  a.nB = B.n;
  a.self = self ? 1 : 0;
  a.status = w.status;
  a.nslices = nslices;
  a.thr = -0.5f * (eps * eps);
  a.ntilesA = (uint32_t)(A.pad / TILE);
  a.ntilesB = (uint32_t)(B.pad / TILE);
  a.sb_row_begin = sb_row_begin;
  a.sb_row_end = sb_row_end;
  a.pairs = r.pairs;
  a.dist2 = r.dist2;
  a.capacity = r.capacity;
  a.n_pairs = reinterpret_cast<unsigned long long*>(r.n_pairs);
  a.counts = r.counts;
  a.counts_b = r.counts_b;
  a.total = reinterpret_cast<unsigned long long*>(r.total);
  a.xcd_bar = w.status + 8;
  {
    // re-align the workgroups of each XCD every few hundred microseconds: about 512 slices
    // (measured on MI355X: +12..16 % over never aligning; every tile costs more than it gains)
    const int per = 512 / (a.nslices + 1);
    a.sync_mode = per < 8 ? 8 : (per > 128 ? 128 : per);
#ifdef EJOIN_ABL_NOALIGN
    a.sync_mode = 0;
#endif
  }
  if (ctx->profiling) {
    EJ_TRY(hipEventRecord(ctx->ev[1], st));
    EJ_TRY(hipEventRecord(ctx->ev[2], st));
  }
  if (a.nslices == NSTAGE) hipLaunchKernelGGL((k_join<COUNT, true>), dim3(ctx->num_cu), dim3(THREADS), LDS_BYTES, st, a);
  else hipLaunchKernelGGL((k_join<COUNT, false>), dim3(ctx->num_cu), dim3(THREADS), LDS_BYTES, st, a);
  EJ_TRY(hipGetLastError());
  if (own) ctx->ws_dirty = false;
  if (ctx->profiling) {
    EJ_TRY(hipEventRecord(ctx->ev[3], st));
    ctx->ev_valid = 1;
  }
  return EJOIN_OK;
}

// Join of FP16 rows in workspace w (the context's own, or a carving of the static scratch).  XB == nullptr: self-join of XA.
// batch_rows (self-join, pair mode only): null, or nbatches + 1 ascending bounds in rows of super-blocks; the join kernel is
// then launched once per range, and after each launch the pair counter is copied to ctx->batch_count[b] and
// ctx->batch_ev[b] recorded (the counter runs on from launch to launch: the pairs of batch b are those between the
// counts of batch b - 1 and b).
template <bool COUNT>
int run_join(ejoin_ctx* ctx, const Workspace& w, bool own, const uint16_t* XA, int64_t nA, int64_t ldA, const uint16_t* XB, int64_t nB,
             int64_t ldB, int32_t d, float eps, const Results& r, hipStream_t st, const uint32_t* batch_rows = nullptr, int nbatches = 0) {
  const bool self = (XB == nullptr);
  const int64_t padA = pad_rows(nA), padB = self ? 0 : pad_rows(nB);
  const int nkb = k_blocks(d);
  float* sA = w.s;
  float* sB = w.s + padA;
  uint4* HA = w.H;
  uint4* HB = w.H + padA;
  uint4* XpA = w.Xp;
  uint4* XpB = w.Xp + padA * (int64_t)(nkb + 1) * 4;
  EJ_RC(begin_call(ctx, w, own, st));
  EJ_RC(launch_norms(ctx, XA, nA, d, ldA, sA, w.status + 1, XpA, st));
  if (!self) EJ_RC(launch_norms(ctx, XB, nB, d, ldB, sB, w.status + 1, XpB, st));
  // the augmentation rows need the maximum over both sets, so they follow both norm kernels
  EJ_RC(launch_aux(ctx, w.status, sA, nA, HA, XpA, nkb, r.counter(COUNT), COUNT ? r.counts : nullptr, st));
  if (!self) EJ_RC(launch_aux(ctx, w.status, sB, nB, HB, XpB, nkb, nullptr, COUNT ? r.counts_b : nullptr, st));
  const Operand A{XpA, nA, padA}, B{self ? XpA : XpB, self ? nA : nB, self ? padA : padB};
  if (!batch_rows) return launch_join<COUNT>(ctx, w, own, A, B, self, nkb, eps, r, st);
  for (int b = 0; b < nbatches; ++b) {
    if (b > 0) {  // the XCD alignment counters start every launch from zero
      hipLaunchKernelGGL(k_fill_u32, dim3(1), dim3(64), 0, st, w.status + 8, (int64_t)NUM_XCD, 0u);
      EJ_TRY(hipGetLastError());
    }
    EJ_RC(launch_join<COUNT>(ctx, w, own, A, B, self, nkb, eps, r, st, batch_rows[b], batch_rows[b + 1]));
    EJ_TRY(hipMemcpyAsync(ctx->batch_count + b, r.n_pairs, sizeof(unsigned long long), hipMemcpyDeviceToHost, st));
    EJ_TRY(hipEventRecord(ctx->batch_ev[b], st));
  }
  return EJOIN_OK;
}

// Split-FP16 self-join of FP32 rows (see k_split_pack): the same join kernel on 3 * nkb k-blocks.
template <bool COUNT>
int run_join_split(ejoin_ctx* ctx, const float* X32, int64_t n, int32_t d, int64_t ld32, float eps, const Results& r, hipStream_t st) {
  const int64_t pad = pad_rows(n);
  EJ_RC(ensure_workspace(ctx, 2 * pad, 3 * pad_dims(d)));  // two packed arrays of 3 * nkb data blocks + 1 augmentation block each
  const Workspace& w = ctx->ws;
  const int nkb = k_blocks(d);
  uint4* XpA = w.Xp;
  uint4* XpB = w.Xp + pad * (int64_t)(3 * nkb + 1) * 4;
  EJ_RC(begin_call(ctx, w, true, st));
  {
    const int64_t chunks = (int64_t)nkb * pad * 4;
    hipLaunchKernelGGL(k_split_pack, dim3((unsigned)((chunks + 255) / 256)), dim3(256), 0, st, X32, n, pad, d, ld32, nkb, XpA, XpB);
    EJ_TRY(hipGetLastError());
    const int64_t waves = (n + 15) / 16;
    hipLaunchKernelGGL(k_norms_packed, dim3((unsigned)((waves + 3) / 4)), dim3(256), 0, st, XpA, XpB, n, pad, 3 * nkb, w.s, w.status + 1);
    EJ_TRY(hipGetLastError());
  }
  EJ_RC(launch_aux(ctx, w.status, w.s, n, w.H, XpA, 3 * nkb, r.counter(COUNT), COUNT ? r.counts : nullptr, st));
  EJ_RC(launch_aux(ctx, w.status, w.s, n, w.H, XpB, 3 * nkb, nullptr, nullptr, st));
  const Operand A{XpA, n, pad}, B{XpB, n, pad};
  return launch_join<COUNT>(ctx, w, true, A, B, true, 3 * nkb, eps, r, st);
}

// Two-set join of a prepared point set with query points given as FP16 rows.
template <bool COUNT>
int run_join_prepared(ejoin_ctx* ctx, const ejoin_set* P, const uint16_t* XQ, int64_t nQ, int64_t ldQ, float eps, const Results& r,
                      hipStream_t st) {
  const int32_t d = P->d;
  const int64_t padQ = pad_rows(nQ);
  EJ_RC(ensure_workspace(ctx, padQ, pad_dims(d)));
  const Workspace& w = ctx->ws;
  const int nkb = k_blocks(d);
  EJ_RC(begin_call(ctx, w, true, st));
  EJ_RC(launch_norms(ctx, XQ, nQ, d, ldQ, w.s, w.status + 1, w.Xp, st));
  hipLaunchKernelGGL(k_merge_max, dim3(1), dim3(64), 0, st, w.status + 1, P->max_bits);
  EJ_TRY(hipGetLastError());
  // the augmentation rows of both sets are scaled to the largest norm of the two: those of the prepared set are rewritten
  EJ_RC(launch_aux(ctx, w.status, P->s, P->n, P->H, P->Xp, nkb, r.counter(COUNT), COUNT ? r.counts : nullptr, st));
  EJ_RC(launch_aux(ctx, w.status, w.s, nQ, w.H, w.Xp, nkb, nullptr, COUNT ? r.counts_b : nullptr, st));
  const Operand A{P->Xp, P->n, P->pad}, B{w.Xp, nQ, padQ};
  return launch_join<COUNT>(ctx, w, true, A, B, false, nkb, eps, r, st);
}

int check_f32(const ejoin_ctx* ctx, const float* X32, int64_t n, int32_t d, int64_t ld32) {
  if (!ctx || !X32) return EJOIN_EINVAL;
  if (n < 1 || n >= (int64_t)0xFFFFFFFFll - TILE || d < 1 || d > 65536 / 4 || ld32 < d) return EJOIN_EINVAL;
  if ((int64_t)pad_rows(n) * k_blocks(d) * 4 / 256 > 0x7FFFFFFFll) return EJOIN_EUNSUPPORTED;  // grid of k_split_pack
  return EJOIN_OK;
}

// Arguments of a pair-list call / a count call that every entry point checks the same way.
int check_pairs_out(const uint32_t* pairs, uint64_t capacity, const uint64_t* n_pairs, float eps) {
  return (!n_pairs || (!pairs && capacity > 0) || bad_eps(eps)) ? EJOIN_EINVAL : EJOIN_OK;
}
int check_count_out(const uint32_t* counts, const uint64_t* total, float eps) {
  return (!counts || !total || bad_eps(eps)) ? EJOIN_EINVAL : EJOIN_OK;
}

Results pair_results(uint32_t* pairs, float* dist2, uint64_t capacity, uint64_t* n_pairs) {
  Results r;
  r.pairs = pairs;
  r.dist2 = dist2;
  r.capacity = capacity;
  r.n_pairs = n_pairs;
  return r;
}
Results count_results(uint32_t* counts, uint32_t* counts_b, uint64_t* total) {
  Results r;
  r.counts = counts;
  r.counts_b = counts_b;
  r.total = total;
  return r;
}

// FP16 join on the context's own workspace.
template <bool COUNT>
int join_on_ctx(ejoin_ctx* ctx, const uint16_t* XA, int64_t nA, int64_t ldA, const uint16_t* XB, int64_t nB, int64_t ldB, int32_t d,
                float eps, const Results& r, void* stream) {
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return EJOIN_EHIP;
  EJ_RC(ensure_workspace(ctx, pad_rows(nA) + (XB ? pad_rows(nB) : 0), pad_dims(d)));
  return run_join<COUNT>(ctx, ctx->ws, true, XA, nA, ldA, XB, nB, ldB, d, eps, r, static_cast<hipStream_t>(stream));
}

}  // namespace

extern "C" {

int ejoin_create(ejoin_ctx** out, int device) {
  if (!out) return EJOIN_EINVAL;
  *out = nullptr;
  int ndev = 0;
  if (hipGetDeviceCount(&ndev) != hipSuccess || device < 0 || device >= ndev) {
    (void)hipGetLastError();
    return EJOIN_EINVAL;
  }
  hipDeviceProp_t prop;
  if (hipGetDeviceProperties(&prop, device) != hipSuccess) {
    (void)hipGetLastError();
    return EJOIN_EHIP;
  }
  if (strncmp(prop.gcnArchName, "gfx950", 6) != 0) return EJOIN_EUNSUPPORTED;
  ejoin_ctx* ctx = new (std::nothrow) ejoin_ctx();
  if (!ctx) return EJOIN_ENOMEM;
  memset(ctx, 0, sizeof(*ctx));
  ctx->device = device;
  ctx->num_cu = prop.multiProcessorCount;
  DeviceGuard guard(device);
  if (!guard.ok) {
    delete ctx;
    return EJOIN_EHIP;
  }
  hipError_t e = hipMalloc(reinterpret_cast<void**>(&ctx->ws.status), 256);
  if (e == hipSuccess) e = hipMemset(ctx->ws.status, 0, 256);
  // this device's copy of the static scratch (the device is current here)
  if (e == hipSuccess) e = hipGetSymbolAddress(reinterpret_cast<void**>(&ctx->static_scratch), HIP_SYMBOL(scratch));
  for (int i = 0; i < 4 && e == hipSuccess; ++i) e = hipEventCreate(&ctx->ev[i]);
  if (e == hipSuccess) e = hipStreamCreateWithFlags(&ctx->copy_stream, hipStreamNonBlocking);
  for (int i = 0; i < EJOIN_MAX_BATCHES && e == hipSuccess; ++i) e = hipEventCreateWithFlags(&ctx->batch_ev[i], hipEventDisableTiming);
  if (e == hipSuccess) e = hipHostMalloc(reinterpret_cast<void**>(&ctx->batch_count), EJOIN_MAX_BATCHES * sizeof(unsigned long long), hipHostMallocDefault);
  if (e == hipSuccess) e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_join<false, false>), hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
  if (e == hipSuccess) e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_join<true, false>), hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
  if (e == hipSuccess) e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_join<false, true>), hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
  if (e == hipSuccess) e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_join<true, true>), hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
  if (e != hipSuccess) {
    (void)hipGetLastError();
    ejoin_destroy(ctx);
    return EJOIN_EHIP;
  }
  ctx->last_status = ctx->ws.status;
  *out = ctx;
  return EJOIN_OK;
}

int ejoin_destroy(ejoin_ctx* ctx) {
  if (!ctx) return EJOIN_EINVAL;
  DeviceGuard guard(ctx->device);
  if (ctx->ws.status) (void)hipFree(ctx->ws.status);
  if (ctx->ws.s) (void)hipFree(ctx->ws.s);
  if (ctx->ws.H) (void)hipFree(ctx->ws.H);
  if (ctx->ws.Xp) (void)hipFree(ctx->ws.Xp);
  for (int i = 0; i < 4; ++i)
    if (ctx->ev[i]) (void)hipEventDestroy(ctx->ev[i]);
  for (int i = 0; i < EJOIN_MAX_BATCHES; ++i)
    if (ctx->batch_ev[i]) (void)hipEventDestroy(ctx->batch_ev[i]);
  if (ctx->copy_stream) (void)hipStreamDestroy(ctx->copy_stream);
  if (ctx->batch_count) (void)hipHostFree(ctx->batch_count);
  delete ctx;
  return EJOIN_OK;
}

int ejoin_reserve(ejoin_ctx* ctx, int64_t n, int32_t d) {
  if (!ctx || n < 1 || d < 1 || d > 65536) return EJOIN_EINVAL;
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return EJOIN_EHIP;
  return ensure_workspace(ctx, pad_rows(n) + TILE, pad_dims(d));  // + TILE: a total split over two sets pads each of them
}

const char* ejoin_strerror(int code) {
  switch (code) {
    case EJOIN_OK: return "ok";
    case EJOIN_EINVAL: return "invalid argument (null pointer, size out of range, ld not a multiple of 64 or < roundup(d,64), X not 128-byte aligned)";
    case EJOIN_EUNSUPPORTED: return "unsupported device (gfx950 required) or problem size";
    case EJOIN_EHIP: return "HIP runtime error (see ejoin_last_hip_error)";
    case EJOIN_ENOMEM: return "out of device memory for the workspace (20 bytes per point plus a packed copy of X)";
    case EJOIN_ESCRATCH: return "problem too large for the static scratch of the allocation-free entry point (EJOIN_STATIC_SCRATCH_BYTES)";
    default: return "unknown error code";
  }
}

const char* ejoin_last_hip_error(const ejoin_ctx* ctx) { return ctx ? ctx->hip_error : ""; }

int ejoin_norms(ejoin_ctx* ctx, const uint16_t* X, int64_t n, int32_t d, int64_t ld, float* s, void* stream) {
  EJ_RC(check_common(ctx, X, n, d, ld));
  if (!s) return EJOIN_EINVAL;
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return EJOIN_EHIP;
  return launch_norms(ctx, X, n, d, ld, s, nullptr, nullptr, static_cast<hipStream_t>(stream));
}

int ejoin_selfjoin_count(ejoin_ctx* ctx, const uint16_t* X, int64_t n, int32_t d, int64_t ld, float eps, uint32_t* counts,
                         uint64_t* total_pairs, void* stream) {
  EJ_RC(check_common(ctx, X, n, d, ld));
  EJ_RC(check_count_out(counts, total_pairs, eps));
  return join_on_ctx<true>(ctx, X, n, ld, nullptr, 0, 0, d, eps, count_results(counts, nullptr, total_pairs), stream);
}

int ejoin_selfjoin_pairs(ejoin_ctx* ctx, const uint16_t* X, int64_t n, int32_t d, int64_t ld, float eps, uint32_t* pairs,
                         float* dist2, uint64_t capacity, uint64_t* n_pairs, void* stream) {
  EJ_RC(check_common(ctx, X, n, d, ld));
  EJ_RC(check_pairs_out(pairs, capacity, n_pairs, eps));
  return join_on_ctx<false>(ctx, X, n, ld, nullptr, 0, 0, d, eps, pair_results(pairs, dist2, capacity, n_pairs), stream);
}

int ejoin_selfjoin_pairs_to_host(ejoin_ctx* ctx, const uint16_t* X, int64_t n, int32_t d, int64_t ld, float eps, uint32_t* pairs,
                                 float* dist2, uint64_t capacity, int32_t batches, uint32_t* host_pairs, float* host_dist2,
                                 uint64_t* host_n_pairs, void* stream) {
  EJ_RC(check_common(ctx, X, n, d, ld));
  if (!pairs || !host_pairs || !host_n_pairs || capacity == 0 || bad_eps(eps) || batches < 1 || (dist2 == nullptr) != (host_dist2 == nullptr))
    return EJOIN_EINVAL;
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return EJOIN_EHIP;
  hipStream_t st = static_cast<hipStream_t>(stream);
  // Ranges of super-block rows with about the same number of tiles each (row P of the triangle holds nsb - P super-blocks).
  const uint32_t nsb = (uint32_t)((pad_rows(n) / TILE + SB - 1) / SB);
  int nb = batches > EJOIN_MAX_BATCHES ? EJOIN_MAX_BATCHES : batches;
  if ((uint32_t)nb > nsb) nb = (int)nsb;
#ifdef EJOIN_ABL_ROWMAJOR_TILES
  nb = 1;  // (this ablation build deals the whole grid out in one launch)
#endif
  uint32_t bounds[EJOIN_MAX_BATCHES + 1];
  {
    const double total = 0.5 * nsb * (nsb + 1.0);
    double done = 0;
    uint32_t P = 0;
    bounds[0] = 0;
    for (int b = 1; b < nb; ++b) {
      while (P < nsb && done < total * b / nb) done += nsb - P++;
      if (P <= bounds[b - 1]) P = bounds[b - 1] + 1;  // every batch gets at least one row
      bounds[b] = P;
    }
    bounds[nb] = 0xFFFFFFFFu;
  }
  // the counter lives in the context's status block (the caller gets the final count in host memory)
  uint64_t* counter = reinterpret_cast<uint64_t*>(ctx->ws.status + 32);
  EJ_RC(ensure_workspace(ctx, pad_rows(n), pad_dims(d)));
  EJ_RC(run_join<false>(ctx, ctx->ws, true, X, n, ld, nullptr, 0, 0, d, eps, pair_results(pairs, dist2, capacity, counter), st, bounds, nb));
  // As each batch completes, its pairs go to the host on the copy stream while the next batch computes.
  unsigned long long lo = 0;
  for (int b = 0; b < nb; ++b) {
    EJ_TRY(hipEventSynchronize(ctx->batch_ev[b]));
    unsigned long long hi = ctx->batch_count[b];
    if (hi > capacity) hi = capacity;
    if (hi > lo) {
      EJ_TRY(hipMemcpyAsync(host_pairs + 2 * lo, pairs + 2 * lo, (hi - lo) * 2 * sizeof(uint32_t), hipMemcpyDeviceToHost, ctx->copy_stream));
      if (dist2) EJ_TRY(hipMemcpyAsync(host_dist2 + lo, dist2 + lo, (hi - lo) * sizeof(float), hipMemcpyDeviceToHost, ctx->copy_stream));
      lo = hi;
    }
  }
  EJ_TRY(hipStreamSynchronize(ctx->copy_stream));
  *host_n_pairs = ctx->batch_count[nb - 1];
  return EJOIN_OK;
}

int ejoin_selfjoin_pairs_noalloc(ejoin_ctx* ctx, const uint16_t* X, int64_t n, int32_t d, int64_t ld, float eps, uint32_t* pairs,
                                 float* dist2, uint64_t capacity, uint64_t* n_pairs, void* stream) {
  EJ_RC(check_common(ctx, X, n, d, ld));
  EJ_RC(check_pairs_out(pairs, capacity, n_pairs, eps));
  Workspace w;
  if (!carve_static(ctx->static_scratch, pad_rows(n), pad_dims(d), w)) return EJOIN_ESCRATCH;
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return EJOIN_EHIP;
  return run_join<false>(ctx, w, false, X, n, ld, nullptr, 0, 0, d, eps, pair_results(pairs, dist2, capacity, n_pairs),
                         static_cast<hipStream_t>(stream));
}

int ejoin_selfjoin_count_f32(ejoin_ctx* ctx, const float* X32, int64_t n, int32_t d, int64_t ld32, float eps, uint32_t* counts,
                             uint64_t* total_pairs, void* stream) {
  EJ_RC(check_f32(ctx, X32, n, d, ld32));
  EJ_RC(check_count_out(counts, total_pairs, eps));
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return EJOIN_EHIP;
  return run_join_split<true>(ctx, X32, n, d, ld32, eps, count_results(counts, nullptr, total_pairs), static_cast<hipStream_t>(stream));
}

int ejoin_selfjoin_pairs_f32(ejoin_ctx* ctx, const float* X32, int64_t n, int32_t d, int64_t ld32, float eps, uint32_t* pairs,
                             float* dist2, uint64_t capacity, uint64_t* n_pairs, void* stream) {
  EJ_RC(check_f32(ctx, X32, n, d, ld32));
  EJ_RC(check_pairs_out(pairs, capacity, n_pairs, eps));
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return EJOIN_EHIP;
  return run_join_split<false>(ctx, X32, n, d, ld32, eps, pair_results(pairs, dist2, capacity, n_pairs), static_cast<hipStream_t>(stream));
}

int ejoin_join_pairs(ejoin_ctx* ctx, const uint16_t* P, int64_t np, int64_t ldp, const uint16_t* Q, int64_t nq, int64_t ldq, int32_t d,
                     float eps, uint32_t* pairs, float* dist2, uint64_t capacity, uint64_t* n_pairs, void* stream) {
  EJ_RC(check_common(ctx, P, np, d, ldp));
  EJ_RC(check_common(ctx, Q, nq, d, ldq));
  EJ_RC(check_pairs_out(pairs, capacity, n_pairs, eps));
  return join_on_ctx<false>(ctx, P, np, ldp, Q, nq, ldq, d, eps, pair_results(pairs, dist2, capacity, n_pairs), stream);
}

int ejoin_join_count(ejoin_ctx* ctx, const uint16_t* P, int64_t np, int64_t ldp, const uint16_t* Q, int64_t nq, int64_t ldq, int32_t d,
                     float eps, uint32_t* counts_p, uint32_t* counts_q, uint64_t* total, void* stream) {
  EJ_RC(check_common(ctx, P, np, d, ldp));
  EJ_RC(check_common(ctx, Q, nq, d, ldq));
  EJ_RC(check_count_out(counts_p, total, eps));
  return join_on_ctx<true>(ctx, P, np, ldp, Q, nq, ldq, d, eps, count_results(counts_p, counts_q, total), stream);
}

int ejoin_set_create(ejoin_ctx* ctx, const uint16_t* X, int64_t n, int32_t d, int64_t ld, void* stream, ejoin_set** out) {
  if (!out) return EJOIN_EINVAL;
  *out = nullptr;
  EJ_RC(check_common(ctx, X, n, d, ld));
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return EJOIN_EHIP;
  hipStream_t st = static_cast<hipStream_t>(stream);
  ejoin_set* set = new (std::nothrow) ejoin_set();
  if (!set) return EJOIN_ENOMEM;
  set->ctx = ctx;
  set->n = n;
  set->pad = pad_rows(n);
  set->d = d;
  hipError_t e = hipMalloc(reinterpret_cast<void**>(&set->Xp), (size_t)packed_bytes(set->pad, pad_dims(d)));
  if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&set->s), (size_t)set->pad * sizeof(float));
  if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&set->H), (size_t)set->pad * sizeof(uint4));
  if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&set->max_bits), 256);
  if (e != hipSuccess) {
    (void)hipGetLastError();
    (void)ejoin_set_destroy(set);
    return e == hipErrorOutOfMemory ? EJOIN_ENOMEM : fail_hip(ctx, e, "hipMalloc(prepared set)");
  }
  hipLaunchKernelGGL(k_fill_u32, dim3(1), dim3(64), 0, st, set->max_bits, (int64_t)1, 0u);
  int rc = (hipGetLastError() == hipSuccess) ? EJOIN_OK : EJOIN_EHIP;
  if (rc == EJOIN_OK) rc = launch_norms(ctx, X, n, d, ld, set->s, set->max_bits, set->Xp, st);
  if (rc != EJOIN_OK) {
    (void)hipDeviceSynchronize();
    (void)ejoin_set_destroy(set);
    return rc;
  }
  *out = set;
  return EJOIN_OK;
}

int ejoin_set_destroy(ejoin_set* set) {
  if (!set) return EJOIN_EINVAL;
  DeviceGuard guard(set->ctx->device);
  if (set->Xp) (void)hipFree(set->Xp);
  if (set->s) (void)hipFree(set->s);
  if (set->H) (void)hipFree(set->H);
  if (set->max_bits) (void)hipFree(set->max_bits);
  delete set;
  return EJOIN_OK;
}

int ejoin_set_join_pairs(ejoin_ctx* ctx, ejoin_set* P, const uint16_t* Q, int64_t nq, int64_t ldq, float eps, uint32_t* pairs,
                         float* dist2, uint64_t capacity, uint64_t* n_pairs, void* stream) {
  if (!ctx || !P || P->ctx != ctx) return EJOIN_EINVAL;
  EJ_RC(check_common(ctx, Q, nq, P->d, ldq));
  EJ_RC(check_pairs_out(pairs, capacity, n_pairs, eps));
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return EJOIN_EHIP;
  return run_join_prepared<false>(ctx, P, Q, nq, ldq, eps, pair_results(pairs, dist2, capacity, n_pairs), static_cast<hipStream_t>(stream));
}

int ejoin_set_join_count(ejoin_ctx* ctx, ejoin_set* P, const uint16_t* Q, int64_t nq, int64_t ldq, float eps, uint32_t* counts_p,
                         uint32_t* counts_q, uint64_t* total, void* stream) {
  if (!ctx || !P || P->ctx != ctx) return EJOIN_EINVAL;
  EJ_RC(check_common(ctx, Q, nq, P->d, ldq));
  EJ_RC(check_count_out(counts_p, total, eps));
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return EJOIN_EHIP;
  return run_join_prepared<true>(ctx, P, Q, nq, ldq, eps, count_results(counts_p, counts_q, total), static_cast<hipStream_t>(stream));
}

int ejoin_convert_f32(ejoin_ctx* ctx, const float* X32, int64_t n, int32_t d, int64_t ld32, const float* center, float scale,
                      uint16_t* X16, int64_t ld16, void* stream) {
  if (!ctx || !X32 || !X16) return EJOIN_EINVAL;
  if (n < 1 || n >= (int64_t)0xFFFFFFFFll - TILE || d < 1 || d > 65536) return EJOIN_EINVAL;
  if (ld32 < d || ld16 < pad_dims(d) || (ld16 % KPAD) != 0 || !isfinite(scale)) return EJOIN_EINVAL;
  if ((reinterpret_cast<uintptr_t>(X16) & 127) != 0) return EJOIN_EINVAL;
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return EJOIN_EHIP;
  const int64_t threads = n * (ld16 / 8);
  if ((threads + 255) / 256 > 0x7FFFFFFFll) return EJOIN_EUNSUPPORTED;
  hipLaunchKernelGGL(k_convert_f32, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, static_cast<hipStream_t>(stream), X32, n, d,
                     ld32, center, scale, X16, ld16);
  EJ_TRY(hipGetLastError());
  return EJOIN_OK;
}

int ejoin_dist2_tile(ejoin_ctx* ctx, const uint16_t* X, int64_t n, int32_t d, int64_t ld, int64_t i0, int64_t j0, int32_t rows,
                     int32_t cols, float* out, void* stream) {
  EJ_RC(check_common(ctx, X, n, d, ld));
  if (!out || rows < 1 || cols < 1 || i0 < 0 || j0 < 0 || i0 + rows > n || j0 + cols > n) return EJOIN_EINVAL;
  if (rows > 32 * 65535 || cols > 32 * 65535) return EJOIN_EINVAL;
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return EJOIN_EHIP;
  EJ_RC(ensure_workspace(ctx, pad_rows(n), 0));
  const Workspace& w = ctx->ws;
  hipStream_t st = static_cast<hipStream_t>(stream);
  EJ_RC(begin_call(ctx, w, true, st));  // (no join kernel follows: the status block stays marked for a reset)
  EJ_RC(launch_norms(ctx, X, n, d, ld, w.s, w.status + 1, nullptr, st));
  EJ_RC(launch_aux(ctx, w.status, w.s, n, w.H, nullptr, 0, nullptr, nullptr, st));
  hipLaunchKernelGGL(k_dist2_tile, dim3((cols + 31) / 32, (rows + 31) / 32), dim3(64), 0, st, X, w.H, w.status, n, ld, k_blocks(d), i0, j0, rows, cols, out);
  EJ_TRY(hipGetLastError());
  return EJOIN_OK;
}

int ejoin_status(ejoin_ctx* ctx, int* status) {
  if (!ctx || !status) return EJOIN_EINVAL;
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return EJOIN_EHIP;
  // the stream of the last call first: a blocking copy on the null stream does not order against non-blocking streams
  EJ_TRY(hipStreamSynchronize(ctx->last_stream));
  uint32_t st = 0;
  EJ_TRY(hipMemcpy(&st, ctx->last_status, sizeof(st), hipMemcpyDeviceToHost));
  *status = (int)st;
  return EJOIN_OK;
}

int ejoin_set_profiling(ejoin_ctx* ctx, int on) {
  if (!ctx) return EJOIN_EINVAL;
  ctx->profiling = on ? 1 : 0;
  ctx->ev_valid = 0;
  return EJOIN_OK;
}

int ejoin_last_kernel_ms(ejoin_ctx* ctx, float* prep_ms, float* join_ms) {
  if (!ctx || !ctx->ev_valid) return EJOIN_EINVAL;
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return EJOIN_EHIP;
  EJ_TRY(hipEventSynchronize(ctx->ev[3]));
  float a = 0.f, b = 0.f;
  EJ_TRY(hipEventElapsedTime(&a, ctx->ev[0], ctx->ev[1]));
  EJ_TRY(hipEventElapsedTime(&b, ctx->ev[2], ctx->ev[3]));
  if (prep_ms) *prep_ms = a;
  if (join_ms) *join_ms = b;
  return EJOIN_OK;
}

int64_t ejoin_tiles_evaluated(int64_t n) {
  if (n < 1) return 0;
  const int64_t t = (n + TILE - 1) / TILE;
  return t * (t + 1) / 2;
}

int64_t ejoin_tiles_evaluated2(int64_t np, int64_t nq) {
  if (np < 1 || nq < 1) return 0;
  return ((np + TILE - 1) / TILE) * ((nq + TILE - 1) / TILE);
}

}  // extern "C"
