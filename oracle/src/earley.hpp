// TEST INFRASTRUCTURE ONLY: part of the slow CPU oracle.
//
// O1: the plain definition of the next-token mask (sections 1-2: a token is
// allowed at a decoding step iff the text generated so far followed by the
// token's bytes can still be completed to a sentence of the grammar).  The
// paper's cache, context expansion and automaton rewrites all preserve that
// result, so the oracle computes it directly, with no automaton: the grammar
// is turned into plain productions over byte sets and an Earley recogniser
// answers "is w a viable prefix?".  Unproductive productions are removed
// first, so that a non-empty Earley set is equivalent to "some completion
// exists".
#pragma once
#include <algorithm>
#include <cstdint>
#include <map>
#include <queue>
#include <stdexcept>
#include <string>
#include <tuple>
#include <unordered_set>
#include <vector>

#include "grammar.hpp"
#include "utf8dag.hpp"

namespace orc {

// Symbols: s >= 0 is nonterminal s; s < 0 is terminal set number -(s+1).
struct Bnf {
  struct Prod { int lhs; std::vector<int> rhs; };
  std::vector<Prod> prods;
  std::vector<std::vector<int>> prods_of;  // nonterminal -> production ids
  std::vector<ByteSet> terms;
  std::vector<bool> nullable;
  std::vector<std::string> minstr;  // a shortest byte string each nonterminal derives
  int n_nt = 0;
  int start = -1;                   // augmented start symbol  S' -> root
  int start_prod = -1;
};

class BnfBuilder {
 public:
  explicit BnfBuilder(const Grammar& g) : g_(g) {}

  Bnf build() {
    int R = (int)g_.rule_names.size();
    b_.n_nt = R;  // rule i is nonterminal i
    for (int r = 0; r < R; ++r) {
      // a rule body is a list of alternatives, each a symbol sequence
      for (auto& alt : alternatives(g_.rule_body[r])) add_prod(r, alt);
    }
    b_.start = fresh();
    add_prod(b_.start, {g_.root});
    prune_unproductive();
    index();
    b_.start_prod = -1;
    for (size_t p = 0; p < b_.prods.size(); ++p)
      if (b_.prods[p].lhs == b_.start) b_.start_prod = (int)p;
    if (b_.start_prod < 0) throw std::runtime_error("the root rule derives no string");
    compute_nullable();
    compute_minstr();
    return std::move(b_);
  }

 private:
  const Grammar& g_;
  Bnf b_;
  std::map<std::pair<std::vector<std::pair<uint32_t, uint32_t>>, bool>, int> class_nt_;

  int fresh() { return b_.n_nt++; }
  void add_prod(int lhs, std::vector<int> rhs) { b_.prods.push_back({lhs, std::move(rhs)}); }
  int term(const ByteSet& s) {
    for (size_t i = 0; i < b_.terms.size(); ++i)
      if (b_.terms[i] == s) return -((int)i + 1);
    b_.terms.push_back(s);
    return -(int)b_.terms.size();
  }

  std::vector<std::vector<int>> alternatives(int e) {
    const Expr& x = g_.pool[e];
    std::vector<std::vector<int>> out;
    if (x.kind == Expr::ALT) {
      for (int k : x.kids) out.push_back(sequence(k));
    } else {
      out.push_back(sequence(e));
    }
    return out;
  }
  std::vector<int> sequence(int e) {
    const Expr& x = g_.pool[e];
    std::vector<int> out;
    if (x.kind == Expr::SEQ) {
      for (int k : x.kids) { auto s = symbols(k); out.insert(out.end(), s.begin(), s.end()); }
    } else {
      out = symbols(e);
    }
    return out;
  }
  // the symbol string standing for one item
  std::vector<int> symbols(int e) {
    const Expr& x = g_.pool[e];
    switch (x.kind) {
      case Expr::BYTES: {
        std::vector<int> out;
        for (unsigned char c : x.bytes) { ByteSet s; s.set(c); out.push_back(term(s)); }
        return out;
      }
      case Expr::REF: return {x.rule};
      case Expr::CLASS: return {class_symbol(x)};
      case Expr::SEQ: return sequence(e);
      case Expr::ALT: {
        int n = fresh();
        for (auto& alt : alternatives(e)) add_prod(n, alt);
        return {n};
      }
      case Expr::STAR: {  // N -> "" | N body
        int n = fresh();
        auto body = sequence(x.kids[0]);
        add_prod(n, {});
        std::vector<int> rec{n};
        rec.insert(rec.end(), body.begin(), body.end());
        add_prod(n, rec);
        return {n};
      }
      case Expr::PLUS: {  // N -> body | N body
        int n = fresh();
        auto body = sequence(x.kids[0]);
        add_prod(n, body);
        std::vector<int> rec{n};
        rec.insert(rec.end(), body.begin(), body.end());
        add_prod(n, rec);
        return {n};
      }
      case Expr::OPT: {  // N -> "" | body
        int n = fresh();
        add_prod(n, {});
        add_prod(n, sequence(x.kids[0]));
        return {n};
      }
    }
    return {};
  }
  int class_symbol(const Expr& x) {
    auto key = std::make_pair(x.ranges, x.negated);
    auto it = class_nt_.find(key);
    if (it != class_nt_.end()) return it->second;
    ByteDag dag = class_to_dag(x.ranges, x.negated);
    int result;
    if (dag.empty) {
      result = fresh();  // no production: derives nothing
    } else {
      std::vector<int> nt(dag.nodes.size(), -1);
      for (size_t d = 1; d < dag.nodes.size(); ++d) nt[d] = fresh();
      for (size_t d = 1; d < dag.nodes.size(); ++d)
        for (auto& e : dag.nodes[d]) {
          if (e.child == 0) add_prod(nt[d], {term(e.bytes)});
          else add_prod(nt[d], {term(e.bytes), nt[e.child]});
        }
      result = nt[dag.root];
    }
    class_nt_[key] = result;
    return result;
  }

  void prune_unproductive() {
    std::vector<bool> prod_ok(b_.n_nt, false);
    bool changed = true;
    while (changed) {
      changed = false;
      for (auto& p : b_.prods) {
        if (prod_ok[p.lhs]) continue;
        bool ok = true;
        for (int s : p.rhs) {
          if (s >= 0 ? !prod_ok[s] : b_.terms[-(s + 1)].none()) { ok = false; break; }
        }
        if (ok) { prod_ok[p.lhs] = true; changed = true; }
      }
    }
    std::vector<Bnf::Prod> kept;
    for (auto& p : b_.prods) {
      bool ok = prod_ok[p.lhs];
      for (int s : p.rhs)
        if (s >= 0 ? !prod_ok[s] : b_.terms[-(s + 1)].none()) ok = false;
      if (ok) kept.push_back(p);
    }
    b_.prods.swap(kept);
  }
  void index() {
    b_.prods_of.assign(b_.n_nt, {});
    for (size_t p = 0; p < b_.prods.size(); ++p) b_.prods_of[b_.prods[p].lhs].push_back((int)p);
  }
  void compute_nullable() {
    b_.nullable.assign(b_.n_nt, false);
    bool changed = true;
    while (changed) {
      changed = false;
      for (auto& p : b_.prods) {
        if (b_.nullable[p.lhs]) continue;
        bool all = true;
        for (int s : p.rhs)
          if (s < 0 || !b_.nullable[s]) { all = false; break; }
        if (all) { b_.nullable[p.lhs] = true; changed = true; }
      }
    }
  }
  void compute_minstr() {
    std::vector<bool> have(b_.n_nt, false);
    b_.minstr.assign(b_.n_nt, "");
    bool changed = true;
    while (changed) {
      changed = false;
      for (auto& p : b_.prods) {
        std::string s;
        bool ok = true;
        for (int x : p.rhs) {
          if (x < 0) {
            const ByteSet& t = b_.terms[-(x + 1)];
            int c = 0;
            while (!t.test(c)) ++c;
            s.push_back((char)c);
          } else if (have[x]) s += b_.minstr[x];
          else { ok = false; break; }
        }
        if (!ok) continue;
        if (!have[p.lhs] || s.size() < b_.minstr[p.lhs].size()) {
          have[p.lhs] = true;
          b_.minstr[p.lhs] = s;
          changed = true;
        }
      }
    }
  }
};

struct Item {
  int prod, dot, origin;
  bool operator==(const Item& o) const { return prod == o.prod && dot == o.dot && origin == o.origin; }
};

struct ItemSet {
  std::vector<Item> items;
  std::unordered_set<uint64_t> seen;
  std::map<int, std::vector<int>> waiting;  // nonterminal -> items with the dot in front of it

  static uint64_t key(const Item& it) {
    return ((uint64_t)it.prod << 40) | ((uint64_t)it.dot << 24) | (uint64_t)it.origin;
  }
  bool add(const Item& it) {
    if (it.origin >= (1 << 24) || it.dot >= (1 << 16)) throw std::runtime_error("Earley item out of range");
    if (!seen.insert(key(it)).second) return false;
    items.push_back(it);
    return true;
  }
};

// The chart for the text accepted so far, plus probes for candidate tokens.
class Earley {
 public:
  explicit Earley(const Bnf* b) : b_(b) {
    ItemSet s0;
    s0.add({b_->start_prod, 0, 0});
    close(s0, 0, nullptr);
    chart_.push_back(std::move(s0));
  }

  int length() const { return (int)chart_.size() - 1; }

  // Append bytes to the accepted text.  Returns false (and leaves the chart
  // unchanged) if the extended text is not a viable prefix.
  bool advance(const unsigned char* bytes, int n) {
    std::vector<ItemSet> extra;
    if (!extend(bytes, n, extra)) return false;
    for (auto& s : extra) chart_.push_back(std::move(s));
    return true;
  }
  // Would the accepted text followed by these bytes still be a viable prefix?
  bool probe(const unsigned char* bytes, int n) const {
    std::vector<ItemSet> extra;
    return extend(bytes, n, extra);
  }
  // Is the accepted text itself a sentence of the grammar?
  bool complete() const {
    const ItemSet& last = chart_.back();
    Item goal{b_->start_prod, (int)b_->prods[b_->start_prod].rhs.size(), 0};
    return last.seen.count(ItemSet::key(goal)) != 0;
  }
  void truncate(int n_bytes) { chart_.resize(n_bytes + 1); }

  // Some byte string u such that accepted-text + u is a sentence: cheapest
  // way to finish an item of the last set and then, one after another, the
  // items that were waiting for it (Dijkstra on added length).  What is left
  // to do for an item depends only on (production, dot, origin): its own
  // tail, then the items of chart[origin] that wait for its left-hand side.
  std::string completion() const {
    struct Entry { size_t cost; Item it; std::string text; };
    auto cmp = [](const Entry& a, const Entry& b) { return a.cost > b.cost; };
    std::priority_queue<Entry, std::vector<Entry>, decltype(cmp)> pq(cmp);
    std::unordered_set<uint64_t> done;
    auto tail = [&](const Item& it) {
      std::string s;
      const auto& rhs = b_->prods[it.prod].rhs;
      for (size_t k = it.dot; k < rhs.size(); ++k) {
        int x = rhs[k];
        if (x < 0) { const ByteSet& t = b_->terms[-(x + 1)]; int c = 0; while (!t.test(c)) ++c; s.push_back((char)c); }
        else s += b_->minstr[x];
      }
      return s;
    };
    for (const Item& it : chart_.back().items) {
      std::string t = tail(it);
      pq.push({t.size(), it, t});
    }
    while (!pq.empty()) {
      Entry e = pq.top();
      pq.pop();
      if (!done.insert(ItemSet::key(e.it)).second) continue;
      int lhs = b_->prods[e.it.prod].lhs;
      if (lhs == b_->start) return e.text;
      const ItemSet& home = chart_[e.it.origin];
      auto w = home.waiting.find(lhs);
      if (w == home.waiting.end()) continue;
      for (int pi : w->second) {
        Item parent = home.items[pi];
        parent.dot += 1;
        if (done.count(ItemSet::key(parent))) continue;
        std::string t = e.text + tail(parent);
        pq.push({t.size(), parent, t});
      }
    }
    throw std::runtime_error("no completion found (text is not a viable prefix)");
  }

 private:
  const Bnf* b_;
  std::vector<ItemSet> chart_;

  const ItemSet& set_at(int pos, const std::vector<ItemSet>* extra) const {
    int base = (int)chart_.size();
    return pos < base ? chart_[pos] : (*extra)[pos - base];
  }
  // predictor + completer to a fixed point; `extra` holds sets beyond the chart
  void close(ItemSet& s, int pos, const std::vector<ItemSet>* extra) const {
    for (size_t i = 0; i < s.items.size(); ++i) {
      Item it = s.items[i];
      const auto& rhs = b_->prods[it.prod].rhs;
      if (it.dot < (int)rhs.size()) {
        int x = rhs[it.dot];
        if (x >= 0) {
          for (int p : b_->prods_of[x]) s.add({p, 0, pos});
          if (b_->nullable[x]) s.add({it.prod, it.dot + 1, it.origin});
        }
      } else if (it.origin != pos) {
        // (an item completed where it started derives "", which the nullable
        // step above already accounts for)
        const ItemSet& home = set_at(it.origin, extra);
        auto w = home.waiting.find(b_->prods[it.prod].lhs);
        if (w != home.waiting.end())
          for (int pi : w->second) {
            const Item& parent = home.items[pi];
            s.add({parent.prod, parent.dot + 1, parent.origin});
          }
      }
    }
    s.waiting.clear();
    for (size_t i = 0; i < s.items.size(); ++i) {
      const Item& it = s.items[i];
      const auto& rhs = b_->prods[it.prod].rhs;
      if (it.dot < (int)rhs.size() && rhs[it.dot] >= 0) s.waiting[rhs[it.dot]].push_back((int)i);
    }
  }
  bool extend(const unsigned char* bytes, int n, std::vector<ItemSet>& extra) const {
    int base = (int)chart_.size();
    for (int k = 0; k < n; ++k) {
      const ItemSet& prev = (k == 0) ? chart_.back() : extra[k - 1];
      ItemSet next;
      for (const Item& it : prev.items) {
        const auto& rhs = b_->prods[it.prod].rhs;
        if (it.dot < (int)rhs.size() && rhs[it.dot] < 0 && b_->terms[-(rhs[it.dot] + 1)].test(bytes[k]))
          next.add({it.prod, it.dot + 1, it.origin});
      }
      if (next.items.empty()) return false;
      extra.push_back(std::move(next));
      close(extra.back(), base + k, &extra);
    }
    return true;
  }
};

}  // namespace orc
