// Host build of the join kernel's tile schedule for the CPU tests: enumerates, for every workgroup, the
// tiles it would compute, in order.  Compiled by tests/test_schedule.py with g++ (no GPU code involved).
#include <stdint.h>
#include "tile_cursor.h"

extern "C" {

// Writes up to `cap` (block, step, I, J) quadruples; returns the number of tiles of the whole schedule.
// sb_row_begin .. sb_row_end - 1: rows of super-blocks covered (0 .. UINT32_MAX = all).
int64_t ejoin_test_schedule_rows(uint32_t nblocks, uint32_t self_join, uint32_t nt_a, uint32_t nt_b, uint32_t sb_row_begin,
                                 uint32_t sb_row_end, uint32_t* out, int64_t cap) {
  int64_t m = 0;
  for (uint32_t b = 0; b < nblocks; ++b) {
    TileCursor tc;
    tc.init(b, nblocks, self_join, nt_a, nt_b, sb_row_begin, sb_row_end);
    uint32_t I = 0, J = 0, step = 0;
    while (tc.next(I, J)) {
      if (m < cap) {
        out[4 * m] = b;
        out[4 * m + 1] = step;
        out[4 * m + 2] = I;
        out[4 * m + 3] = J;
      }
      ++m;
      ++step;
    }
  }
  return m;
}

int64_t ejoin_test_schedule(uint32_t nblocks, uint32_t self_join, uint32_t nt_a, uint32_t nt_b, uint32_t* out, int64_t cap) {
  return ejoin_test_schedule_rows(nblocks, self_join, nt_a, nt_b, 0, 0xFFFFFFFFu, out, cap);
}
}
