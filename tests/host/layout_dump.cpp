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

void ejoin_test_region_pair(int32_t lane, int32_t q, int32_t* i, int32_t* j) {
  int a, b;
  region_pair(lane, q, a, b);
  *i = a;
  *j = b;
}
void ejoin_test_mfma32_element(int32_t lane, int32_t q, int32_t* m, int32_t* n) {
  int a, b;
  mfma32_element(lane, q, a, b);
  *m = a;
  *n = b;
}
int32_t ejoin_test_aug_row_point(int32_t m) { return aug_row_point(m); }
int32_t ejoin_test_aug_col_point(int32_t n) { return aug_col_point(n); }
int32_t ejoin_test_aug_chunk_a(int32_t lane) { return aug_chunk_a(lane); }
int32_t ejoin_test_aug_chunk_b(int32_t lane) { return aug_chunk_b(lane); }
int32_t ejoin_test_aug_block_unit(int32_t row, int32_t chunk) { return aug_block_unit(row, chunk); }
uint32_t ejoin_test_aug_lds_offset_a(int32_t lane, int32_t row0) { return aug_lds_offset_a(lane, row0); }
uint32_t ejoin_test_aug_lds_offset_b(int32_t lane, int32_t col0) { return aug_lds_offset_b(lane, col0); }
int32_t ejoin_test_aug_const(int32_t which) {
  return which == 0 ? EJ_AUG_PART : which == 1 ? EJ_AUG_CONST : which == 2 ? EJ_AUG_REGION_STEP : EJ_AUG_BYTES;
}
}
