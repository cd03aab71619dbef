// Exact host-side execution of the flattened automaton on *sets* of stacks.
// Used for accept_token (arxiv 2411.15100, section 3: the sampled token
// updates the stack state; section 2.2: parallel stacks for nondeterminism)
// and for deciding the rare (position, token) pairs whose GPU walk exceeded
// its on-chip bounds.
#pragma once
#include <cstdint>
#include <vector>

#include "automaton.hpp"

namespace xgm {

using Stack = std::vector<int32_t>;  // return nodes bottom-up, current node last

constexpr int32_t kBottom = -1;      // marker: unknown context below this frame

class Engine {
 public:
  explicit Engine(const Automaton* a) : A_(a) {}

  // Advance every stack over the bytes; `out` = all surviving stacks (sorted,
  // unique).  Returns XGM_OK, XGM_ERR_TOKEN_REJECTED (nothing survives),
  // XGM_ERR_TOO_MANY_STACKS or XGM_ERR_TOO_LARGE.  If `left_frame` is given,
  // bit 0 is set when some path popped a kBottom marker with bytes remaining,
  // bit 1 when it did so in front of a byte that can follow the popped rule.
  // `follow_rule`: the rule whose instance sits right above the marker.
  int advance(const std::vector<Stack>& in, const uint8_t* bytes, int n, std::vector<Stack>* out,
              int* left_frame = nullptr, size_t max_out = 64, int32_t follow_rule = -1) const;

  // every frame of some stack is accepting: the text so far is a sentence
  bool can_terminate(const std::vector<Stack>& stacks) const;

  // 0 rejected, 1 context-dependent, 2 accepted (section 3.1 refined by one
  // byte of context), 4 context-dependent by section 3.1 alone, for `node`
  // alone on the stack with unknown context below; -1 if limits were hit
  int classify(int32_t node, const uint8_t* bytes, int n) const;

 private:
  const Automaton* A_;
};

}  // namespace xgm
