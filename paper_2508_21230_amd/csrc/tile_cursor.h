// Static tile schedule of the join kernel (host- and device-compilable: the CPU tests enumerate it).
#ifndef EJOIN_TILE_CURSOR_H
#define EJOIN_TILE_CURSOR_H

#include <stdint.h>

#if defined(__HIPCC__)
#define EJ_HD __host__ __device__
#else
#define EJ_HD
#endif
#if defined(__HIP_DEVICE_COMPILE__)
// every lane computes the same value; say so to the compiler (the values feed scalar operands)
#define EJ_UNIFORM(x) __builtin_amdgcn_readfirstlane(x)
#else
#define EJ_UNIFORM(x) (x)
#endif

constexpr uint32_t EJ_NUM_XCD = 8;  // accelerator complex dies of the MI355X, each with its own L2
constexpr uint32_t EJ_SB = 16;      // tiles per super-block edge (one super-block = 256 tiles = one pass of the chip)

// Work distribution (the counterpart of the paper's work queue that orders block tiles in small
// squares for L2 reuse, Section 3.3.1, re-derived for 8 XCDs with private 4 MB L2s):
//   * the upper triangle of the tile grid is cut into super-blocks of 16 x 16 tiles, enumerated
//     row-major; one super-block is one pass of the 256 CUs, so at any time the chip works on
//     (16+16) x 256 rows of X, which the memory-side cache holds;
//   * inside a super-block each XCD owns an 8 x 4 rectangle of tiles (12 row panels shared by its
//     32 CUs through its own L2); the rectangle's position rotates with the super-block index so
//     that partially empty (diagonal, ragged) super-blocks do not starve the same XCD every time;
//   * workgroup w runs on XCD w % 8 (hardware round-robin, verified on device).  The non-empty tiles
//     of an XCD's rectangles, in super-block order, form a list; workgroup number k of the XCD takes
//     entries k, k + 32, k + 64, ... of it.  So every workgroup of an XCD computes the same number of
//     tiles (+-1), and at any time the 32 of them sit on 32 consecutive entries -- one rectangle,
//     or the end of one and the start of the next.  That keeps them in step without any
//     synchronisation or queue, which is what makes the panels they share hit in L2: a schedule
//     that lets workgroups skip empty tiles individually drifts apart by many tiles and the L2
//     hit rate collapses (measured: 16 % instead of ~75 %).
struct TileCursor {
  uint32_t xcd, wpx;     // this workgroup's XCD; workgroups per XCD
  uint32_t self, nsbA, nsbB, ntA, ntB;
  uint32_t rem;          // position of this workgroup's next tile, counted from the first tile of the current rectangle
  uint32_t P, Q, sbi;    // current super-block: coordinates and linear index
  uint32_t fast_left;    // steps of the common kind that may follow (see next) ...
  uint32_t fast_row, fast_col;  // ... and what they need: the tile's place in its rectangle, row already in tiles of the grid
#ifdef EJOIN_ABL_ROWMAJOR_TILES
  uint32_t start, stride;  // first tile and stride of this workgroup
#endif
  // self_join: upper triangle of an nt x nt grid (nt_a == nt_b); otherwise the whole nt_a x nt_b grid.
  // sb_row_begin .. sb_row_end - 1: the rows of super-blocks this launch covers (a join may be cut into several
  // launches by rows of super-blocks; 0 .. UINT32_MAX = everything)
  EJ_HD void init(uint32_t block, uint32_t nblocks, uint32_t self_join, uint32_t nt_a, uint32_t nt_b, uint32_t sb_row_begin = 0,
                  uint32_t sb_row_end = 0xFFFFFFFFu) {
    xcd = block % EJ_NUM_XCD;
    wpx = (nblocks - xcd + EJ_NUM_XCD - 1) / EJ_NUM_XCD;  // workgroups with this XCD id
    self = self_join;
    ntA = nt_a;
    ntB = nt_b;
    nsbA = (nt_a + EJ_SB - 1) / EJ_SB;
    nsbB = (nt_b + EJ_SB - 1) / EJ_SB;
    if (sb_row_end < nsbA) nsbA = sb_row_end;  // (the rows past the range are simply not enumerated)
    rem = block / EJ_NUM_XCD;
    P = sb_row_begin;
    Q = self_join ? sb_row_begin : 0;
    sbi = 0;
    fast_left = 0;
    fast_row = fast_col = 0;
#ifdef EJOIN_ABL_ROWMAJOR_TILES
    start = block;
    stride = nblocks;
#endif
  }
  // Tiles of row r (0..7) of a rectangle on the diagonal of the self-join: columns lo .. cj-1, with
  // lo = max(0, a + r - b), where a and b are the rectangle's row and column offsets in its super-block.
  static EJ_HD uint32_t diag_row_first(uint32_t a, uint32_t b, uint32_t r) { return a + r > b ? a + r - b : 0u; }
  // next tile of this workgroup; false when the work is exhausted
  EJ_HD bool next(uint32_t& I, uint32_t& J) {
#ifdef EJOIN_ABL_ROWMAJOR_TILES
    // tiles of the triangle (or grid) in row-major order, tile t to workgroup t % nblocks; P, Q hold the
    // row and column of this workgroup's next tile
    if (rem != 0xFFFFFFFFu) {  // first call
      rem = 0xFFFFFFFFu;
      P = 0;
      Q = start;
    } else {
      Q += stride;
    }
    while (P < ntA && Q >= ntB) {
      Q -= ntB;
      ++P;
      if (self) Q += P;  // row P of the triangle starts at column P
    }
    if (P >= ntA) return false;
    I = EJ_UNIFORM(P);
    J = EJ_UNIFORM(Q);
    return true;
#endif
    // Everything here is uniform over the workgroup and meant to stay on the scalar unit: 32-bit counters,
    // closed forms for the number of tiles of a rectangle, and real branches around the rare cases.
    //
    // The common step first.  All eight wavefronts of a workgroup run this code at the same time, between two
    // tiles, with nothing else to overlap it: every instruction here is paid eight times on the one scalar unit.
    // Along a row of super-blocks nearly every rectangle is a complete 8 x 4 one; the last tile came from such
    // a rectangle and the next one sits in the next rectangle, at place (fast_row, fast_col) of it, whose offsets
    // inside its super-block rotate with the super-block index.  With 32 workgroups per XCD (the whole chip) that
    // place is the same from rectangle to rectangle and the steps of this kind go on to the end of the row; with
    // another number the general code below is asked again after each one.  (fast_left: how many may follow.)
#ifndef EJOIN_CURSOR_NO_FAST_PATH
    if (fast_left != 0) {
      --fast_left;
      ++Q;
      ++sbi;
      const uint32_t t = xcd + sbi;  // rectangle number (t % 8): row offset 8 (t / 4 % 2), column offset 4 (t % 4)
      I = EJ_UNIFORM(fast_row + ((t << 1) & 8u));
      J = EJ_UNIFORM(Q * EJ_SB + fast_col + ((t << 2) & 12u));
      rem = rem - 32u + wpx;
      return true;
    }
#endif
    while (P < nsbA) {
      const uint32_t xp = (xcd + sbi) & 7;
      const uint32_t a = (xp >> 2) * 8, b = (xp & 3) * 4;  // the rectangle's offsets inside its super-block
      const uint32_t I0 = P * EJ_SB + a, J0 = Q * EJ_SB + b;
      // columns of the rectangle inside the grid, and rows (in the self-join's off-diagonal super-blocks all 8)
      const uint32_t cj = J0 >= ntB ? 0u : (ntB - J0 < 4u ? ntB - J0 : 4u);
      const uint32_t ri = self ? 8u : (I0 >= ntA ? 0u : (ntA - I0 < 8u ? ntA - I0 : 8u));
      const bool on_diag = self && P == Q;
      uint32_t v = ri * cj;
      if (on_diag) {  // one super-block in every row of the self-join
        v = 0;
        for (uint32_t r = 0; r < 8; ++r) {
          const uint32_t lo = diag_row_first(a, b, r);
          v += lo < cj ? cj - lo : 0u;
        }
      }
      if (rem < v) {
        uint32_t r = 0, c = rem;
        if (on_diag) {
          for (; r < 8; ++r) {
            const uint32_t lo = diag_row_first(a, b, r);
            const uint32_t cnt = lo < cj ? cj - lo : 0u;
            if (c < cnt) {
              c += lo;
              break;
            }
            c -= cnt;
          }
        } else if (cj == 4) {
          r = rem >> 2;
          c = rem & 3;
        } else {  // ragged last column of rectangles
          while (c >= cj) {
            c -= cj;
            ++r;
          }
        }
        I = EJ_UNIFORM(I0 + r);
        J = EJ_UNIFORM(J0 + c);
        rem += wpx;
#ifndef EJOIN_CURSOR_NO_FAST_PATH
        // Super-blocks (P, Q + 1 ..) that are complete: every column inside the grid (Q' < ntB / 16), every
        // row too (always so right of the diagonal of the self-join, whose rows end before its columns do),
        // and off the diagonal (Q' > P; the self-join starts each row on the diagonal, so Q >= P here).
        // A rectangle of 32 tiles maps position p to (p / 4, p % 4) whatever kind it is, so the fast step
        // may follow any rectangle; it only requires the ones it enters to be complete.
        // The next tile is entry rem - 32 of the next rectangle, if that is one of its 32.
        {
          const uint32_t qf = ntB / EJ_SB;
          const bool rows_ok = self ? true : (P < ntA / EJ_SB);
          const uint32_t pos = rem - 32u;
          uint32_t steps = (v == 32u && rows_ok && Q + 1 < qf && pos < 32u) ? qf - 1 - Q : 0u;
          if (wpx != 32u && steps > 1u) steps = 1u;
          fast_left = steps;
          fast_row = P * EJ_SB + (pos >> 2);
          fast_col = pos & 3u;
        }
#endif
        return true;
      }
      rem -= v;
      ++sbi;
      if (++Q == nsbB) {  // super-blocks row-major; the self-join starts each row on the diagonal
        ++P;
        Q = self ? P : 0;
      }
    }
    return false;
  }
};

#endif  // EJOIN_TILE_CURSOR_H
