// Host-side schedule object behind tasp_schedule_t (integers only).
#pragma once
#include <cstdint>
#include <vector>

#include "tasp.h"

struct tasp_schedule {
  int32_t n = 0;             // ranks
  int32_t n_rings = 0;       // rings = sub-chunks per chunk: n-1 (K_n scheme) or m ((m-K_m-m)^u scheme)
  int32_t rank = 0;
  int32_t max_arc_load = 1;
  std::vector<int32_t> rings;        // [n_rings * n]
  std::vector<int32_t> out_mapping;  // [n * n]
  std::vector<int32_t> in_mapping;   // [n * n]
  std::vector<int32_t> arrival;      // [n * n_rings]
};

namespace tasp {

struct Segment {
  int64_t start, end;   // global token range [start, end)
  int32_t diag;         // 1: straddles the causal diagonal of the query block
};

// Global position of the first row of a query block and the number of rows in it.
// FULL has one block (all L rows); ZIGZAG_CAUSAL has two (the two half-chunks of eq. (4)).
struct QueryBlock {
  int64_t local_row0;   // first local row
  int64_t rows;
  int64_t pos0;         // global position of that row; rows are contiguous in the sequence
};

int n_query_blocks(int32_t mask_mode);
int query_block(const tasp_schedule& s, int64_t S, int32_t mask_mode, int32_t q_block, QueryBlock* out);

// Visible KV segments of (step, q_block) in concatenation order; see tasp_step_segments.
int step_segments(const tasp_schedule& s, int64_t S, int32_t mask_mode, int32_t order, int32_t step,
                  int32_t q_block, std::vector<Segment>* out);

// Every key range the rank holds at `step` (visible or not), in concatenation order, diag = 0.
int step_key_ranges(const tasp_schedule& s, int64_t S, int32_t mask_mode, int32_t order, int32_t step,
                    std::vector<Segment>* out);

int check_sequence(const tasp_schedule& s, int64_t S, int32_t mask_mode);

}  // namespace tasp
