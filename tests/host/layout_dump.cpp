// Host build of the panel layout for the CPU tests (csrc/panel_layout.h compiled with g++, no GPU code involved).
#include <stdint.h>
#include "panel_layout.h"

extern "C" {

void ejoin_test_stored_at(int64_t row, int32_t p, int64_t* point, int32_t* chunk) {
  int c;
  stored_at(row, p, *point, c);
  *chunk = c;
}

int64_t ejoin_test_place_of(int64_t point, int32_t chunk) { return place_of(point, chunk); }

uint32_t ejoin_test_fragment_offset(int32_t lane, int32_t t) { return fragment_offset(lane, t); }
}
