// TEST INFRASTRUCTURE ONLY: part of the slow CPU oracle.
//
// O2: the pushdown automaton of Appendix A, simulated literally.
// One finite automaton per grammar rule (here a Thompson NFA built straight
// from the rule's syntax tree), with character edges and rule-reference
// edges.  A configuration is (state, stack of return states).  A character
// edge keeps the stack; a rule-reference edge pushes its target as return
// state and jumps to the callee's start; reaching a rule's accepting state
// pops the return state.  The parsing state is the *set* of configurations
// (nondeterminism = several parallel stacks); every step works on the whole
// set with a visited set, so nullable loops terminate.
//
// It also gives the three-way token classes of section 3.1 for a position
// inside a rule: start with an unknown context below the position's frame
// (a bottom marker); a token is
//   accepted   if some path consumes all its bytes without popping the marker,
//   uncertain  (context-dependent) if not accepted and some path pops the
//              marker while at least one byte is still unconsumed,
//   rejected   otherwise.
// A one-byte form of the context expansion of section 3.2 narrows the
// uncertain class: the byte that comes right after leaving the rule must be
// able to follow that rule in at least one context (its FOLLOW set: whatever
// can be consumed at the return state of some reference to the rule, plus, if
// the referencing rule can end there without consuming anything, whatever
// follows that rule).  classify() reports both: 1 = uncertain also after the
// narrowing, 4 = uncertain by section 3.1 alone (no exit in front of a byte
// that could ever follow the rule, so the token is refused in every context).
// Dead parts (unproductive rules, states that cannot reach their rule's end)
// are removed first, so "a configuration survives" means "can be completed".
#pragma once
#include <cstdint>
#include <set>
#include <stdexcept>
#include <string>
#include <utility>
#include <vector>

#include "grammar.hpp"
#include "utf8dag.hpp"

namespace orc {

struct Nfa {
  enum { EPS = 0, BYTE = 1, CALL = 2 };
  struct Edge { int kind, arg, to; };
  std::vector<std::vector<Edge>> out;
  std::vector<int> rule_of;
  std::vector<int> start, accept;  // per rule
  std::vector<ByteSet> sets;
  std::vector<bool> live;          // state can reach its rule's accepting state
  std::vector<bool> rule_ok;       // rule derives at least one string
  std::vector<bool> nullable;      // rule derives ""
  std::vector<ByteSet> first;      // per rule: bytes its sentences can start with
  std::vector<ByteSet> follow;     // per rule: bytes that can come right after an instance
  int root = -1;
};

class NfaBuilder {
 public:
  explicit NfaBuilder(const Grammar& g) : g_(g) {}
  Nfa build() {
    int R = (int)g_.rule_names.size();
    n_.root = g_.root;
    n_.start.resize(R);
    n_.accept.resize(R);
    for (int r = 0; r < R; ++r) {
      cur_rule_ = r;
      n_.start[r] = state();
      n_.accept[r] = state();
      frag(g_.rule_body[r], n_.start[r], n_.accept[r]);
    }
    analyse();
    return std::move(n_);
  }

 private:
  const Grammar& g_;
  Nfa n_;
  int cur_rule_ = 0;
  std::vector<std::vector<std::pair<int, int>>> rev_;  // state -> (source, edge index)

  int state() {
    n_.out.push_back({});
    n_.rule_of.push_back(cur_rule_);
    return (int)n_.out.size() - 1;
  }
  void edge(int from, int kind, int arg, int to) { n_.out[from].push_back({kind, arg, to}); }
  int byteset(const ByteSet& s) {
    for (size_t i = 0; i < n_.sets.size(); ++i)
      if (n_.sets[i] == s) return (int)i;
    n_.sets.push_back(s);
    return (int)n_.sets.size() - 1;
  }
  // build the fragment for expression e between states a and b
  void frag(int e, int a, int b) {
    const Expr& x = g_.pool[e];
    switch (x.kind) {
      case Expr::BYTES: {
        if (x.bytes.empty()) { edge(a, Nfa::EPS, 0, b); return; }
        int cur = a;
        for (size_t i = 0; i < x.bytes.size(); ++i) {
          int nxt = (i + 1 == x.bytes.size()) ? b : state();
          ByteSet s; s.set((unsigned char)x.bytes[i]);
          edge(cur, Nfa::BYTE, byteset(s), nxt);
          cur = nxt;
        }
        return;
      }
      case Expr::CLASS: {
        ByteDag dag = class_to_dag(x.ranges, x.negated);
        if (dag.empty) return;  // matches nothing
        std::vector<int> st(dag.nodes.size(), -1);
        st[0] = b;
        st[dag.root] = a;
        for (size_t d = 1; d < dag.nodes.size(); ++d)
          if (st[d] < 0) st[d] = state();
        for (size_t d = 1; d < dag.nodes.size(); ++d)
          for (auto& ed : dag.nodes[d]) edge(st[d], Nfa::BYTE, byteset(ed.bytes), st[ed.child]);
        return;
      }
      case Expr::REF: edge(a, Nfa::CALL, x.rule, b); return;
      case Expr::SEQ: {
        if (x.kids.empty()) { edge(a, Nfa::EPS, 0, b); return; }
        int cur = a;
        for (size_t i = 0; i < x.kids.size(); ++i) {
          int nxt = (i + 1 == x.kids.size()) ? b : state();
          frag(x.kids[i], cur, nxt);
          cur = nxt;
        }
        return;
      }
      case Expr::ALT:
        for (int k : x.kids) {
          int s = state(), t = state();
          edge(a, Nfa::EPS, 0, s);
          frag(k, s, t);
          edge(t, Nfa::EPS, 0, b);
        }
        return;
      case Expr::STAR: {
        int hub = state(), s = state(), t = state();
        edge(a, Nfa::EPS, 0, hub);
        edge(hub, Nfa::EPS, 0, b);
        edge(hub, Nfa::EPS, 0, s);
        frag(x.kids[0], s, t);
        edge(t, Nfa::EPS, 0, hub);
        return;
      }
      case Expr::PLUS: {
        int s = state(), t = state();
        edge(a, Nfa::EPS, 0, s);
        frag(x.kids[0], s, t);
        edge(t, Nfa::EPS, 0, s);
        edge(t, Nfa::EPS, 0, b);
        return;
      }
      case Expr::OPT: {
        int s = state(), t = state();
        edge(a, Nfa::EPS, 0, b);
        edge(a, Nfa::EPS, 0, s);
        frag(x.kids[0], s, t);
        edge(t, Nfa::EPS, 0, b);
        return;
      }
    }
  }
  // states of `rule` from which its accepting state is reachable using only
  // edges allowed by `ok` (backward search over reversed edges)
  template <class F>
  std::vector<bool> can_reach(int rule, F ok) {
    int N = (int)n_.out.size();
    if (rev_.empty()) {
      rev_.assign(N, {});
      for (int q = 0; q < N; ++q)
        for (size_t k = 0; k < n_.out[q].size(); ++k) rev_[n_.out[q][k].to].push_back({q, (int)k});
    }
    std::vector<bool> mark(N, false);
    std::vector<int> work{n_.accept[rule]};
    mark[n_.accept[rule]] = true;
    while (!work.empty()) {
      int t = work.back();
      work.pop_back();
      for (auto& pk : rev_[t]) {
        int q = pk.first;
        if (mark[q] || !ok(n_.out[q][pk.second])) continue;
        mark[q] = true;
        work.push_back(q);
      }
    }
    return mark;
  }
  void analyse() {
    int R = (int)n_.start.size();
    n_.rule_ok.assign(R, false);
    bool changed = true;
    auto usable = [&](const Nfa::Edge& e) {
      if (e.kind == Nfa::EPS) return true;
      if (e.kind == Nfa::BYTE) return n_.sets[e.arg].any();
      return (bool)n_.rule_ok[e.arg];
    };
    while (changed) {
      changed = false;
      for (int r = 0; r < R; ++r) {
        if (n_.rule_ok[r]) continue;
        if (can_reach(r, usable)[n_.start[r]]) { n_.rule_ok[r] = true; changed = true; }
      }
    }
    n_.live.assign(n_.out.size(), false);
    for (int r = 0; r < R; ++r) {
      auto m = can_reach(r, usable);
      for (size_t q = 0; q < m.size(); ++q)
        if (m[q] && n_.rule_of[q] == r) n_.live[q] = true;
    }
    n_.nullable.assign(R, false);
    changed = true;
    auto silent = [&](const Nfa::Edge& e) {
      if (e.kind == Nfa::EPS) return true;
      if (e.kind == Nfa::CALL) return (bool)n_.nullable[e.arg];
      return false;
    };
    while (changed) {
      changed = false;
      for (int r = 0; r < R; ++r) {
        if (n_.nullable[r]) continue;
        if (can_reach(r, silent)[n_.start[r]]) { n_.nullable[r] = true; changed = true; }
      }
    }
    if (!n_.rule_ok[n_.root]) throw std::runtime_error("the root rule derives no string");
    first_and_follow();
  }
  // states reachable from q without consuming a byte, staying inside q's rule
  // (epsilon edges, and references to rules that can match "")
  std::vector<int> silent_reach(int q) const {
    std::vector<int> seen{q}, work{q};
    std::vector<bool> mark(n_.out.size(), false);
    mark[q] = true;
    while (!work.empty()) {
      int s = work.back();
      work.pop_back();
      for (auto& e : n_.out[s]) {
        bool silent = e.kind == Nfa::EPS || (e.kind == Nfa::CALL && n_.rule_ok[e.arg] && n_.nullable[e.arg]);
        if (silent && n_.live[e.to] && !mark[e.to]) { mark[e.to] = true; seen.push_back(e.to); work.push_back(e.to); }
      }
    }
    return seen;
  }
  // bytes that can be consumed next from state q (inside its rule or in a rule it calls)
  ByteSet next_bytes(int q) const {
    ByteSet b;
    for (int s : silent_reach(q))
      for (auto& e : n_.out[s]) {
        if (!n_.live[e.to]) continue;
        if (e.kind == Nfa::BYTE) b |= n_.sets[e.arg];
        else if (e.kind == Nfa::CALL && n_.rule_ok[e.arg]) b |= n_.first[e.arg];
      }
    return b;
  }
  void first_and_follow() {
    int R = (int)n_.start.size();
    n_.first.assign(R, ByteSet());
    for (bool changed = true; changed;) {
      changed = false;
      for (int r = 0; r < R; ++r) {
        if (!n_.rule_ok[r]) continue;
        ByteSet b = next_bytes(n_.start[r]);
        if (b != n_.first[r]) { n_.first[r] = b; changed = true; }
      }
    }
    n_.follow.assign(R, ByteSet());
    for (bool changed = true; changed;) {
      changed = false;
      for (size_t q = 0; q < n_.out.size(); ++q) {
        if (!n_.live[q]) continue;
        for (auto& e : n_.out[q]) {
          if (e.kind != Nfa::CALL || !n_.rule_ok[e.arg] || !n_.live[e.to]) continue;
          ByteSet f = n_.follow[e.arg] | next_bytes(e.to);
          int caller = n_.rule_of[q];
          for (int s : silent_reach(e.to))
            if (s == n_.accept[caller]) f |= n_.follow[caller];  // the caller may end right after the call
          if (f != n_.follow[e.arg]) { n_.follow[e.arg] = f; changed = true; }
        }
      }
    }
  }
};

constexpr int BOTTOM = -1;  // marker for "unknown context below this frame"

using Config = std::pair<std::vector<int>, int>;  // (stack of return states, state)
using ConfigSet = std::set<Config>;

class Pda {
 public:
  explicit Pda(const Nfa* n) : n_(n) {}

  // All configurations reachable without consuming a byte.  Sets *popped if a
  // path pops the BOTTOM marker (that path ends there).
  ConfigSet closure(const ConfigSet& in, bool* popped) const {
    ConfigSet all = in;
    std::vector<Config> work(in.begin(), in.end());
    size_t deepest = 0;
    for (auto& c : in) deepest = std::max(deepest, c.first.size());
    size_t limit = deepest + n_->start.size() + 1;
    auto add = [&](Config c) {
      if (all.insert(c).second) work.push_back(std::move(c));
    };
    while (!work.empty()) {
      Config c = std::move(work.back());
      work.pop_back();
      int q = c.second;
      for (auto& e : n_->out[q]) {
        if (!n_->live[e.to]) continue;
        if (e.kind == Nfa::EPS) add({c.first, e.to});
        else if (e.kind == Nfa::CALL && n_->rule_ok[e.arg]) {
          std::vector<int> st = c.first;
          st.push_back(e.to);
          // more pushes in a row than there are rules: some rule re-enters
          // itself without consuming anything
          if (st.size() > limit) throw std::runtime_error("left recursion: the automaton cannot be simulated");
          add({std::move(st), n_->start[e.arg]});
        }
      }
      if (q == n_->accept[n_->rule_of[q]] && !c.first.empty()) {
        int ret = c.first.back();
        if (ret == BOTTOM) { if (popped) *popped = true; }
        else {
          std::vector<int> st(c.first.begin(), c.first.end() - 1);
          add({std::move(st), ret});
        }
      }
    }
    return all;
  }
  ConfigSet step(const ConfigSet& in, unsigned char byte) const {
    ConfigSet out;
    for (auto& c : in)
      for (auto& e : n_->out[c.second])
        if (e.kind == Nfa::BYTE && n_->live[e.to] && n_->sets[e.arg].test(byte)) out.insert({c.first, e.to});
    return out;
  }
  ConfigSet initial() const { return ConfigSet{{std::vector<int>{}, n_->start[n_->root]}}; }

  // consume bytes; empty result = not a viable prefix
  ConfigSet run(ConfigSet cur, const unsigned char* bytes, int n) const {
    for (int i = 0; i < n && !cur.empty(); ++i) cur = step(closure(cur, nullptr), bytes[i]);
    return cur;
  }
  bool is_sentence_state(const ConfigSet& cur) const {
    ConfigSet c = closure(cur, nullptr);
    return c.count({std::vector<int>{}, n_->accept[n_->root]}) != 0;
  }

  // ---- positions inside one rule, named by a path of symbols from its start
  // symbols: 0..255 a byte, 256+r a reference to rule r.  References to
  // nullable rules may be left out of the path.
  std::set<int> rule_closure(std::set<int> s) const {
    std::vector<int> work(s.begin(), s.end());
    while (!work.empty()) {
      int q = work.back();
      work.pop_back();
      for (auto& e : n_->out[q]) {
        bool silent = e.kind == Nfa::EPS || (e.kind == Nfa::CALL && n_->nullable[e.arg]);
        if (silent && n_->live[e.to] && s.insert(e.to).second) work.push_back(e.to);
      }
    }
    return s;
  }
  std::set<int> positions(int rule, const int32_t* symbols, int n) const {
    std::set<int> cur;
    if (n_->rule_ok[rule]) cur = rule_closure({n_->start[rule]});
    for (int i = 0; i < n; ++i) {
      std::set<int> nxt;
      for (int q : cur)
        for (auto& e : n_->out[q]) {
          if (!n_->live[e.to]) continue;
          if (symbols[i] < 256) {
            if (e.kind == Nfa::BYTE && n_->sets[e.arg].test(symbols[i])) nxt.insert(e.to);
          } else if (e.kind == Nfa::CALL && e.arg == symbols[i] - 256 && n_->rule_ok[e.arg]) nxt.insert(e.to);
        }
      cur = rule_closure(nxt);
    }
    return cur;
  }
  // 0 = rejected, 2 = accepted, 1 = uncertain (context-dependent) also after
  // the one-byte narrowing, 4 = uncertain by section 3.1 alone.  All
  // positions belong to `rule`.
  int classify(int rule, const std::set<int>& pos, const unsigned char* bytes, int n) const {
    if (n == 0) return 0;  // a token without bytes is never allowed
    ConfigSet cur;
    for (int q : pos) cur.insert({std::vector<int>{BOTTOM}, q});
    bool left = false, left_with_follower = false;
    for (int i = 0; i < n && !cur.empty(); ++i) {
      bool popped = false;
      ConfigSet closed = closure(cur, &popped);
      if (popped) {  // the rule ended here with bytes[i..] still to come
        left = true;
        if (n_->follow[rule].test(bytes[i])) left_with_follower = true;
      }
      cur = step(closed, bytes[i]);
    }
    if (!cur.empty()) return 2;
    return left_with_follower ? 1 : (left ? 4 : 0);
  }

 private:
  const Nfa* n_;
};

}  // namespace orc
