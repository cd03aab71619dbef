// Host-side planning of the fill kernel's workgroups (no device code).
#pragma once
#include <algorithm>
#include <cstdint>

#include "kernels.hpp"

namespace xgm {

// Cuts every request (row) of a batch into workgroups of (row, chunk range).
// The work that depends on a request's state is the number of entries in the
// context-dependent lists of its stack tops.  All workgroups of a launch
// should be resident together, so a budget of workgroups is shared out in
// proportion to that number: every row gets at least as many as its mask
// words need (a workgroup owns at most kFillMaxChunks chunks), and its chunks
// are cut where the running entry count passes equal shares.
//   upto(b, c): entries of row b in chunks [0, c), all its stacks together
//               (non-decreasing in c, upto(b, 0) == 0);
//   out:        room for B * n_chunk workgroups.
// Returns the number of workgroups written.  Every (row, chunk) is covered by
// exactly one of them; rows appear in order, chunk ranges ascending.
template <class Upto>
inline int32_t plan_workgroups(int32_t B, int32_t n_chunk, int32_t budget, Upto upto, FillBlock* out) {
  const int32_t min_blocks = (n_chunk + kFillMaxChunks - 1) / kFillMaxChunks;
  budget = std::max(budget, B * min_blocks);
  uint64_t total = 0;
  for (int32_t b = 0; b < B; ++b) total += upto(b, n_chunk);
  const int32_t spare = budget - B * min_blocks;
  int32_t n_blocks = 0;
  for (int32_t b = 0; b < B; ++b) {
    const uint64_t row_entries = upto(b, n_chunk);
    int32_t k = min_blocks;
    if (total) k += (int32_t)((uint64_t)spare * row_entries / total);
    k = std::min(k, n_chunk);
    int32_t c0 = 0, made = 0;
    for (int32_t c = 0; c < n_chunk; ++c) {
      bool cut = c + 1 == n_chunk || c + 1 - c0 == kFillMaxChunks;
      // cut after chunk c when the entries up to and including c reach the next share
      if (!cut && made + 1 < k && row_entries)
        cut = upto(b, c + 1) * (uint64_t)k >= row_entries * (uint64_t)(made + 1);
      if (cut) {
        out[n_blocks++] = FillBlock{(uint32_t)b, (uint32_t)c0 | ((uint32_t)(c + 1) << 16)};
        c0 = c + 1;
        ++made;
      }
    }
  }
  return n_blocks;
}

}  // namespace xgm
