// Planning of the fill kernel's workgroups.  The arithmetic is plain C++ that
// compiles for the host (xgm_fill_next_token_bitmask plans there, per call)
// and for the device (a batch of device-resident states is planned by a small
// kernel after every change of state).
#pragma once
#include <cstdint>

#include "kernels.hpp"

#if defined(__HIPCC__) || defined(__HIP__)
#define XGM_PLAN_HD __host__ __device__ inline
#else
#define XGM_PLAN_HD inline
#endif

namespace xgm {

// Cuts every request (row) of a batch into workgroups of (row, chunk range).
// The work that depends on a request's state is the number of entries in the
// context-dependent lists of its stack tops.  All workgroups of a launch
// should be resident together, so a budget of workgroups is shared out in
// proportion to that number: every row gets at least as many as its mask
// words need (a workgroup owns at most kFillMaxChunks chunks), and its chunks
// are cut where the running entry count passes equal shares.

// workgroups every row needs at least
XGM_PLAN_HD int32_t plan_min_blocks(int32_t n_chunk) { return (n_chunk + kFillMaxChunks - 1) / kFillMaxChunks; }

// The budget for a batch: what the device holds at once (`resident`), or, for batches so large that the
// workgroups every row needs for its mask words come near that, those plus three eighths of it, so that
// rows with long lists can still be cut (the launch then runs in more than one round of workgroups;
// measured at 192, 256 and 512 rows of a 152 K vocabulary: fill 24.5 -> 22, 38 -> 29 and 53 -> 41 us).
XGM_PLAN_HD int32_t plan_budget(int32_t resident, int32_t B, int32_t n_chunk) {
  const int32_t floor_blocks = B * plan_min_blocks(n_chunk) + resident * 3 / 8;
  return resident > floor_blocks ? resident : floor_blocks;
}

// the share of a row with `row_entries` of the batch's `total` entries
XGM_PLAN_HD int32_t plan_row_share(int32_t B, int32_t n_chunk, int32_t budget, uint64_t row_entries, uint64_t total) {
  const int32_t min_blocks = plan_min_blocks(n_chunk);
  if (budget < B * min_blocks) budget = B * min_blocks;
  const int32_t spare = budget - B * min_blocks;
  int32_t k = min_blocks;
  if (total) k += (int32_t)((uint64_t)spare * row_entries / total);
  return k < n_chunk ? k : n_chunk;
}

// Where workgroup p of a plan of n goes in the launch.  Workgroups are handed
// to the eight XCDs in turn by their index, and every XCD has an L2 of its
// own: consecutive workgroups of the plan - those of one request, which stage
// the same table image - get indices that are equal modulo 8, so that they
// share an XCD and the image is fetched into one L2 instead of eight.  The
// launch has (n rounded up to a multiple of 8) or more workgroups; indices
// that no p maps to hold kNoRow.
XGM_PLAN_HD uint32_t plan_slot(uint32_t p, uint32_t n) {
  const uint32_t per_xcd = (n + 7u) / 8u;
  return (p % per_xcd) * 8u + p / per_xcd;
}

// Cuts row b into (at most k + plan_min_blocks) workgroups; upto(c) = entries
// of the row in chunks [0, c), all its stacks together (non-decreasing,
// upto(0) == 0).  emit(i, workgroup) receives the i-th of them; returns their number.
template <class Wide, class Upto, class Emit>
XGM_PLAN_HD int32_t plan_row_as(int32_t b, int32_t n_chunk, int32_t k, uint64_t row_entries, Upto upto, Emit emit) {
  int32_t c0 = 0, made = 0;
  uint64_t at_c0 = 0;  // upto(c0)
  for (int32_t c = 0; c < n_chunk; ++c) {
    const uint64_t next = upto(c + 1);  // asked for in ascending order, once each
    bool cut = c + 1 == n_chunk || c + 1 - c0 == kFillMaxChunks;
    // cut after chunk c when the entries up to and including c reach the next share
    if (!cut && made + 1 < k && row_entries) cut = (Wide)next * (Wide)k >= (Wide)row_entries * (Wide)(made + 1);
    if (cut) {
      const uint32_t idle = next == at_c0 ? kFillBlockNoEntries : 0u;  // nothing listed in these chunks
      emit(made, FillBlock{(uint32_t)b, (uint32_t)c0 | idle | ((uint32_t)(c + 1) << 16)});
      c0 = c + 1;
      at_c0 = next;
      ++made;
    }
  }
  return made;
}
template <class Upto, class Emit>
XGM_PLAN_HD int32_t plan_row(int32_t b, int32_t n_chunk, int32_t k, Upto upto, Emit emit) {
  const uint64_t row_entries = upto(n_chunk);
  // the products below fit 32 bits for every list length that occurs in practice; the comparison is exact either way
  if (row_entries * (uint64_t)(k > 0 ? k : 1) <= 0xFFFFFFFFull) return plan_row_as<uint32_t>(b, n_chunk, k, row_entries, upto, emit);
  return plan_row_as<uint64_t>(b, n_chunk, k, row_entries, upto, emit);
}

//   upto(b, c): as above for row b;
//   out:        room for B * n_chunk workgroups.
// Returns the number of workgroups written.  Every (row, chunk) is covered by
// exactly one of them; rows appear in order, chunk ranges ascending (the
// caller places them in the launch with plan_slot).
template <class Upto>
inline int32_t plan_workgroups(int32_t B, int32_t n_chunk, int32_t budget, Upto upto, FillBlock* out) {
  uint64_t total = 0;
  for (int32_t b = 0; b < B; ++b) total += upto(b, n_chunk);
  int32_t n_blocks = 0;
  for (int32_t b = 0; b < B; ++b) {
    const int32_t k = plan_row_share(B, n_chunk, budget, upto(b, n_chunk), total);
    FillBlock* dst = out + n_blocks;
    n_blocks += plan_row(b, n_chunk, k, [&](int32_t c) { return upto(b, c); },
                         [&](int32_t i, const FillBlock& f) { dst[i] = f; });
  }
  return n_blocks;
}

}  // namespace xgm
