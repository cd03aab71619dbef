#include "engine.hpp"

#include <set>
#include <utility>

#include "../../include/xgm.h"

namespace xgm {

namespace {
constexpr size_t kMaxConfigs = 1 << 16;  // configurations explored per byte
}

int Engine::advance(const std::vector<Stack>& in, const uint8_t* bytes, int n, std::vector<Stack>* out,
                    int* left_frame, size_t max_out, int32_t follow_rule) const {
  const Automaton& A = *A_;
  std::set<Stack> cur(in.begin(), in.end());
  for (int i = 0; i < n; ++i) {
    const int c = bytes[i];
    std::set<Stack> next;
    // configurations before byte i: (stack, consumed-a-byte-since-last-push)
    std::set<std::pair<Stack, bool>> seen;
    std::vector<std::pair<Stack, bool>> work;
    for (auto& s : cur) { seen.insert({s, true}); work.push_back({s, true}); }
    while (!work.empty()) {
      auto cfg = std::move(work.back());
      work.pop_back();
      const Stack& st = cfg.first;
      const int32_t node = st.back();
      for (auto& e : A.bedges[node])
        if (e.lo <= c && c <= e.hi) {
          Stack s2 = st;
          s2.back() = e.to;
          next.insert(std::move(s2));
          break;
        }
      for (auto& e : A.redges[node])
        if (A.first[e.rule].test(c)) {
          if ((int)st.size() + 1 > XGM_MAX_STACK_DEPTH) return XGM_ERR_TOO_LARGE;
          Stack s2 = st;
          if (A.node_dead_end[e.to]) {
            s2.back() = A.rule_start[e.rule];     // returning to a dead end = returning to our parent
          } else {
            s2.back() = e.to;                     // return node
            s2.push_back(A.rule_start[e.rule]);   // enter the callee
          }
          std::pair<Stack, bool> c2{std::move(s2), false};
          if (seen.insert(c2).second) work.push_back(std::move(c2));
        }
      // the rule may end here; an instance must have consumed a byte
      if (A.node_final[node] && cfg.second && st.size() >= 2) {
        if (st[st.size() - 2] == kBottom) {
          if (left_frame) *left_frame |= (follow_rule >= 0 && A.follow[follow_rule].test(c)) ? 3 : 1;
        } else {
          Stack s2(st.begin(), st.end() - 1);
          std::pair<Stack, bool> c2{std::move(s2), true};
          if (seen.insert(c2).second) work.push_back(std::move(c2));
        }
      }
      if (seen.size() > kMaxConfigs) return XGM_ERR_TOO_LARGE;
    }
    if (next.empty()) return XGM_ERR_TOKEN_REJECTED;
    cur.swap(next);
  }
  // A top node that can only return is returned from right away, so that the
  // stack top is always a node with something of its own to say about the
  // next token (and equal states get equal representations).
  std::set<Stack> norm;
  for (auto& s : cur) {
    Stack t = s;
    while (t.size() >= 2 && t[t.size() - 2] != kBottom && A.node_dead_end[t.back()]) t.pop_back();
    norm.insert(std::move(t));
  }
  cur.swap(norm);
  if (cur.size() > max_out) return XGM_ERR_TOO_MANY_STACKS;
  out->assign(cur.begin(), cur.end());
  return XGM_OK;
}

bool Engine::can_terminate(const std::vector<Stack>& stacks) const {
  for (auto& s : stacks) {
    bool all = true;
    for (int32_t n : s)
      if (!A_->node_final[n]) { all = false; break; }
    if (all) return true;
  }
  return false;
}

int Engine::classify(int32_t node, const uint8_t* bytes, int n) const {
  if (n == 0) return 0;
  std::vector<Stack> in{Stack{kBottom, node}}, out;
  int left = 0;
  int rc = advance(in, bytes, n, &out, &left, (size_t)-1, A_->node_rule[node]);
  if (rc == XGM_OK) return 2;
  if (rc == XGM_ERR_TOKEN_REJECTED) return (left & 2) ? 1 : (left & 1) ? 4 : 0;
  return -1;
}

}  // namespace xgm
