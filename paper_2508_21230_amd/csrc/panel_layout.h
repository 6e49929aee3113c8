// Arrangement of an operand panel (256 points x 32 coordinates = 256 rows of 64 bytes) in the LDS, and hence in
// the packed copy of the data, which the kernel copies to the LDS as it is.  Host- and device-compilable: the CPU
// tests check it against the operand layout of the MFMA instruction.
#ifndef EJOIN_PANEL_LAYOUT_H
#define EJOIN_PANEL_LAYOUT_H

#include <stdint.h>

#if defined(__HIPCC__)
#define EJ_LAYOUT_HD __host__ __device__ __forceinline__
#else
#define EJ_LAYOUT_HD inline
#endif

// A row holds four 16-byte chunks (8 coordinates each).  Two things decide where the chunk of point r
// (0..255), coordinates 8 k .. 8 k + 7 (k = 0..3) of the slice, is stored:
//   * A v_mfma_f32_16x16x32_f16 operand wants, in lane l, point l%16 of a group of 16 and chunk k = l/16.
//     The LDS serves a ds_read_b128 16 lanes at a time, and which lanes go together is not simply
//     "16 consecutive": reading rows l%16 at chunk l/16 costs two cycles per group (measured).  A read
//     in which lane l takes row l%32 of a group of 32 and chunk l/32 is served without conflicts (measured),
//     so the layout is made such that the MFMA operand IS such a read: points come in groups of 32,
//     (point 16 h + x, chunk 2 u + v) of a group is stored in row 16 v + x, chunk 2 h + u.  Fragment
//     t = 2 T + h (points 16 t .. 16 t + 15 of the panel) is then: lane l reads row 32 T + l%32,
//     chunk 2 h + l/32.
//   * Chunk c of row r is stored at position c ^ swz(r): 16 consecutive rows at the same chunk
//     then fall into 16 distinct 16-byte bank groups (the LDS has 64 banks of 4 B; 4 rows per
//     256 B bank line x 4 positions).  This is the role the XOR swizzle of Section 3.3.5 (Eq. 2)
//     plays on the A100's 32 banks.
#ifdef EJOIN_ABL_NOSWIZZLE
EJ_LAYOUT_HD int swz(int) { return 0; }
#else
EJ_LAYOUT_HD int swz(int row) { return (row >> 2) & 3; }
#endif

// Which point (same group of 32) and which chunk of its slice the 16 bytes at (row, position p) hold.
EJ_LAYOUT_HD void stored_at(int64_t row, int p, int64_t& point, int& chunk) {
  const int c = p ^ swz((int)(row & 255));
  point = (row & ~(int64_t)31) | ((int64_t)(c >> 1) << 4) | (row & 15);
  chunk = 2 * (c & 1) + (int)((row >> 4) & 1);
}

// The inverse: index of the 16-byte chunk (row * 4 + position) that holds (point, chunk).
EJ_LAYOUT_HD int64_t place_of(int64_t point, int chunk) {
  const int64_t row = (point & ~(int64_t)31) | ((int64_t)(chunk & 1) << 4) | (point & 15);
  const int c = 2 * (int)((point >> 4) & 1) + (chunk >> 1);
  return row * 4 + (c ^ swz((int)(row & 255)));
}

// Where a panel's 16 KB k-blocks sit in the packed copy of a point set (the re-laid-out X the join kernel reads):
// panel-major -- the `blocks` k-blocks of a panel (its data blocks in order of k, then the augmentation block) follow
// each other, then the next panel.  A tile then streams through two contiguous pieces of memory (one per operand
// panel) with a constant step from slice to slice, and the walk along a row of tiles goes through the column panels
// in address order.  (With the k-blocks of ALL panels stored together instead, every slice of a tile comes from another
// 64 MB region of the copy; measured on the 2 GB copy of 10^6 x 960 points the two orders run equally fast.)
// `place` = row * 4 + position over the whole set (place_of), result in 16-byte units.
EJ_LAYOUT_HD int64_t packed_index(int64_t place, int kb, int blocks) {
  return ((place >> 10) * blocks + kb) * 1024 + (place & 1023);
}

// Byte offset inside a panel of the 16 bytes that lane `lane` reads as its part of fragment t (points
// 16 t .. 16 t + 15 of the panel, as the A or B operand of v_mfma_f32_16x16x32_f16).
// fragment_offset(lane, t) = fragment_offset(lane, t % 2) + (t / 2) * 2048.
EJ_LAYOUT_HD uint32_t fragment_offset(int lane, int t) {
  const int row = 32 * (t >> 1) + (lane & 31), chunk = 2 * (t & 1) + (lane >> 5);
  return (uint32_t)(row * 64 + ((chunk ^ swz(row)) << 4));
}

// ---- The augmentation step: one v_mfma_f32_32x32x16_f16 per 32 x 32 region adds -s_i/2 - s_j/2 to the region's
// accumulators, which are those of four v_mfma_f32_16x16x32_f16 blocks side by side (16 registers).
// Register q = 8 a + 4 c + r of lane l holds the pair (i, j) of the region (block (a, c), its register r) ...
EJ_LAYOUT_HD void region_pair(int lane, int q, int& i, int& j) {
  i = 16 * (q >> 3) + 4 * (lane >> 4) + (q & 3);
  j = 16 * ((q >> 2) & 1) + (lane & 15);
}
// ... and is where the 32 x 32 MFMA puts its element (m, n):
EJ_LAYOUT_HD void mfma32_element(int lane, int q, int& m, int& n) {
  m = 8 * (q >> 2) + 4 * (lane >> 5) + (q & 3);
  n = lane & 31;
}
// So the step needs D[m][n] = -s_i/2 - s_j/2 with i = i(m; bit 4 of n), j = j(n % 16; bit 3 of m), which is
// bilinear in indicator columns.  With P(x) = { p1, p2, p3, 0 } the pieces of -s_x/2 and C = { c, c, c, 0 }:
//   row m of the A operand = { P(x), P(x + 4), C [bit 3 of m = 0], C [bit 3 of m = 1] },  x = aug_row_point(m)
//   row n of the B operand = { C [bit 4 of n = 0], C [bit 4 of n = 1], P(y), P(y + 16) },  y = aug_col_point(n)
// (k = 0..15 left to right).  Of the 16 products of an element 6 are non-zero and each is exact, as in a plain
// { P, C } . { C, P } step.  Written as four 16-byte chunks per row: row m of a group of 32 has
//   chunk 0 = { P(x), P(x + 4) }   chunk 1 = { P(y), P(y + 16) }   chunk 2 = { C, 0 }   chunk 3 = { 0, C }
// and lane l of the MFMA (row or column l % 32, k = 8 (l / 32) .. + 7) reads chunk aug_chunk_a(l) / aug_chunk_b(l).
EJ_LAYOUT_HD int aug_row_point(int m) { return 16 * (m >> 4) + 8 * ((m >> 2) & 1) + (m & 3); }
EJ_LAYOUT_HD int aug_col_point(int n) { return n & 15; }
EJ_LAYOUT_HD int aug_chunk_a(int lane) { return (lane >> 5) ? 2 + ((lane >> 3) & 1) : 0; }
EJ_LAYOUT_HD int aug_chunk_b(int lane) { return (lane >> 5) ? 1 : 2 + ((lane >> 4) & 1); }

// Where the join kernel finds these chunks.  Chunks 2 and 3 are the same for every row, so only chunks 0 and 1 are
// stored per row: a panel's augmentation block in the packed copy (its last k-block, 1024 units of 16 bytes) holds
// chunk c (0 or 1) of row r (0..255) at unit aug_block_unit(r, c); its other 512 units are not used.
EJ_LAYOUT_HD int aug_block_unit(int row, int chunk) { return chunk * 256 + row; }
// A tile's augmentation buffer in the LDS: units 0..255 of the row panel's block (chunk 0 of its rows), units 256..511
// of the column panel's block (chunk 1 of its rows), then the constant chunks: chunk 2 at EJ_AUG_CONST + 512 t,
// chunk 3 sixteen bytes further, for t = 0..3 -- so that, for every lane of an operand read, region t of a wave tile
// (32 rows further on) is 512 bytes further on.
constexpr int EJ_AUG_PART = 256 * 16;
constexpr int EJ_AUG_CONST = 2 * EJ_AUG_PART;
constexpr int EJ_AUG_REGION_STEP = 32 * 16;
constexpr int EJ_AUG_BYTES = EJ_AUG_CONST + 4 * EJ_AUG_REGION_STEP;
// Byte offset in that buffer of the 16 bytes lane `lane` reads as its part of the A (B) operand of region t of the wave
// tile whose first row (column) is row0 of the panel: aug_lds_offset_x(lane, row0) + t * EJ_AUG_REGION_STEP.
EJ_LAYOUT_HD uint32_t aug_lds_offset_a(int lane, int row0) {
  const int c = aug_chunk_a(lane);
  return (uint32_t)(c == 0 ? 16 * (row0 + (lane & 31)) : EJ_AUG_CONST + 16 * (c - 2));
}
EJ_LAYOUT_HD uint32_t aug_lds_offset_b(int lane, int col0) {
  const int c = aug_chunk_b(lane);
  return (uint32_t)(c == 1 ? EJ_AUG_PART + 16 * (col0 + (lane & 31)) : EJ_AUG_CONST + 16 * (c - 2));
}

#endif  // EJOIN_PANEL_LAYOUT_H
