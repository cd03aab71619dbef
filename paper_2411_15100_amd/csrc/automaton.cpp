// Grammar text -> per-rule NFA -> per-rule minimal DFA over (bytes + rule
// references) -> flattened tables.  See automaton.hpp and include/xgm.h.
#include "automaton.hpp"

#include <algorithm>
#include <map>
#include <queue>
#include <set>

#include "../../include/xgm.h"

namespace xgm {
namespace {

// ------------------------------------------------------------------ lexer
enum TokKind { T_IDENT, T_DEFINE, T_PIPE, T_LP, T_RP, T_STAR, T_PLUS, T_QUEST, T_LIT, T_CLASS, T_END };
struct CpRange { uint32_t lo, hi; };
struct Token {
  TokKind kind;
  std::string text;             // identifier or literal bytes
  std::vector<CpRange> ranges;  // class, normalised and already complemented
  size_t pos;
};

[[noreturn]] void parse_fail(size_t pos, const std::string& why) {
  throw Failure(XGM_ERR_PARSE, "grammar: " + why + " (at byte " + std::to_string(pos) + ")");
}

int hex_digit(char c, size_t pos) {
  if (c >= '0' && c <= '9') return c - '0';
  if (c >= 'a' && c <= 'f') return 10 + c - 'a';
  if (c >= 'A' && c <= 'F') return 10 + c - 'A';
  parse_fail(pos, "bad hex digit");
}

void append_utf8(uint32_t cp, std::string& out) {
  if (cp <= 0x7F) out += (char)cp;
  else if (cp <= 0x7FF) { out += (char)(0xC0 | (cp >> 6)); out += (char)(0x80 | (cp & 0x3F)); }
  else if (cp <= 0xFFFF) { out += (char)(0xE0 | (cp >> 12)); out += (char)(0x80 | ((cp >> 6) & 0x3F)); out += (char)(0x80 | (cp & 0x3F)); }
  else { out += (char)(0xF0 | (cp >> 18)); out += (char)(0x80 | ((cp >> 12) & 0x3F)); out += (char)(0x80 | ((cp >> 6) & 0x3F)); out += (char)(0x80 | (cp & 0x3F)); }
}

std::vector<CpRange> normalise_class(std::vector<CpRange> r, bool negate) {
  std::sort(r.begin(), r.end(), [](const CpRange& a, const CpRange& b) { return a.lo < b.lo; });
  std::vector<CpRange> merged;
  for (auto& x : r) {
    if (!merged.empty() && x.lo <= merged.back().hi + 1) merged.back().hi = std::max(merged.back().hi, x.hi);
    else merged.push_back(x);
  }
  if (negate) {
    std::vector<CpRange> inv;
    uint32_t next = 0;
    for (auto& x : merged) {
      if (x.lo > next) inv.push_back({next, x.lo - 1});
      next = x.hi + 1;
    }
    if (next <= 0x10FFFF) inv.push_back({next, 0x10FFFF});
    merged.swap(inv);
  }
  // drop the surrogate block and anything above the last scalar value
  std::vector<CpRange> out;
  for (auto x : merged) {
    if (x.lo > 0x10FFFF) continue;
    x.hi = std::min<uint32_t>(x.hi, 0x10FFFF);
    if (x.hi < 0xD800 || x.lo > 0xDFFF) { out.push_back(x); continue; }
    if (x.lo < 0xD800) out.push_back({x.lo, 0xD7FF});
    if (x.hi > 0xDFFF) out.push_back({0xE000, x.hi});
  }
  return out;
}

std::vector<Token> lex(const std::string& s) {
  std::vector<Token> out;
  size_t i = 0, n = s.size();
  auto ident_start = [](char c) { return (c >= 'a' && c <= 'z') || (c >= 'A' && c <= 'Z') || c == '_'; };
  auto ident_part = [&](char c) { return ident_start(c) || (c >= '0' && c <= '9'); };
  // an escape after a backslash; returns a code point (or raw byte for \x in literals)
  auto escape = [&](bool in_class, bool* raw_byte) -> uint32_t {
    if (i >= n) parse_fail(i, "unterminated escape");
    char k = s[i++];
    *raw_byte = false;
    switch (k) {
      case 'n': return '\n';
      case 't': return '\t';
      case 'r': return '\r';
      case 'b': return '\b';
      case 'f': return '\f';
      case '"': case '\\': case '\'': case '/': return (unsigned char)k;
      case ']': case '[': case '-': case '^':
        if (in_class) return (unsigned char)k;
        break;
      case 'x': {
        if (i + 2 > n) parse_fail(i, "truncated \\x escape");
        uint32_t v = hex_digit(s[i], i) * 16 + hex_digit(s[i + 1], i + 1);
        i += 2;
        *raw_byte = !in_class;
        return v;
      }
      case 'u': {
        if (i + 4 > n) parse_fail(i, "truncated \\u escape");
        uint32_t v = 0;
        for (int k2 = 0; k2 < 4; ++k2) v = v * 16 + hex_digit(s[i + k2], i + k2);
        i += 4;
        return v;
      }
      default: break;
    }
    parse_fail(i - 1, std::string("unknown escape \\") + k);
  };
  while (i < n) {
    char c = s[i];
    if (c == ' ' || c == '\t' || c == '\n' || c == '\r') { ++i; continue; }
    if (c == '#') { while (i < n && s[i] != '\n') ++i; continue; }
    size_t start = i;
    if (ident_start(c)) {
      while (i < n && ident_part(s[i])) ++i;
      out.push_back({T_IDENT, s.substr(start, i - start), {}, start});
      continue;
    }
    if (c == ':' && s.compare(i, 3, "::=") == 0) { i += 3; out.push_back({T_DEFINE, "", {}, start}); continue; }
    if (c == '|') { ++i; out.push_back({T_PIPE, "", {}, start}); continue; }
    if (c == '(') { ++i; out.push_back({T_LP, "", {}, start}); continue; }
    if (c == ')') { ++i; out.push_back({T_RP, "", {}, start}); continue; }
    if (c == '*') { ++i; out.push_back({T_STAR, "", {}, start}); continue; }
    if (c == '+') { ++i; out.push_back({T_PLUS, "", {}, start}); continue; }
    if (c == '?') { ++i; out.push_back({T_QUEST, "", {}, start}); continue; }
    if (c == '"') {
      ++i;
      std::string bytes;
      for (;;) {
        if (i >= n) parse_fail(start, "unterminated literal");
        char d = s[i++];
        if (d == '"') break;
        if (d != '\\') { bytes += d; continue; }
        bool raw;
        uint32_t v = escape(false, &raw);
        if (raw) bytes += (char)v;
        else {
          if (v >= 0xD800 && v <= 0xDFFF) parse_fail(i, "surrogate code point in literal");
          append_utf8(v, bytes);
        }
      }
      out.push_back({T_LIT, bytes, {}, start});
      continue;
    }
    if (c == '[') {
      ++i;
      bool negate = false;
      if (i < n && s[i] == '^') { negate = true; ++i; }
      std::vector<CpRange> ranges;
      auto one = [&]() -> uint32_t {
        if (i >= n) parse_fail(start, "unterminated class");
        unsigned char d = (unsigned char)s[i++];
        if (d == '\\') { bool raw; return escape(true, &raw); }
        if (d < 0x80) return d;
        int extra = d >= 0xF0 ? 3 : d >= 0xE0 ? 2 : d >= 0xC0 ? 1 : -1;
        if (extra < 0) parse_fail(i - 1, "invalid UTF-8 in class");
        uint32_t cp = d & (0x3F >> extra);
        for (int k = 0; k < extra; ++k) {
          if (i >= n || ((unsigned char)s[i] & 0xC0) != 0x80) parse_fail(i, "invalid UTF-8 in class");
          cp = (cp << 6) | ((unsigned char)s[i++] & 0x3F);
        }
        return cp;
      };
      for (;;) {
        if (i >= n) parse_fail(start, "unterminated class");
        if (s[i] == ']') { ++i; break; }
        uint32_t lo = one(), hi = lo;
        if (i + 1 < n && s[i] == '-' && s[i + 1] != ']') { ++i; hi = one(); }
        if (hi < lo) parse_fail(i, "reversed range in class");
        ranges.push_back({lo, hi});
      }
      out.push_back({T_CLASS, "", normalise_class(ranges, negate), start});
      continue;
    }
    parse_fail(i, std::string("unexpected character '") + c + "'");
  }
  out.push_back({T_END, "", {}, n});
  return out;
}

// -------------------------------------------------------------------- NFA
struct NEdge { int kind; int lo, hi; int rule; int to; };  // kind 0 eps, 1 bytes [lo,hi], 2 reference
struct Nfa {
  std::vector<std::vector<NEdge>> out;
  int add() { out.emplace_back(); return (int)out.size() - 1; }
  void eps(int a, int b) { out[a].push_back({0, 0, 0, 0, b}); }
  void bytes(int a, int lo, int hi, int b) { out[a].push_back({1, lo, hi, 0, b}); }
  void ref(int a, int rule, int b) { out[a].push_back({2, 0, 0, rule, b}); }
};

struct Frag { int in, out; };

class Parser {
 public:
  Parser(const std::vector<Token>& toks, Nfa& nfa) : t_(toks), nfa_(nfa) {
    for (size_t k = 0; k + 1 < t_.size(); ++k)
      if (t_[k].kind == T_IDENT && t_[k + 1].kind == T_DEFINE) {
        if (rule_index_.count(t_[k].text)) throw Failure(XGM_ERR_PARSE, "grammar: rule '" + t_[k].text + "' defined twice");
        rule_index_[t_[k].text] = (int)names_.size();
        names_.push_back(t_[k].text);
      }
    if (names_.empty()) throw Failure(XGM_ERR_PARSE, "grammar: no rules");
  }
  void run() {
    start_.assign(names_.size(), -1);
    accept_.assign(names_.size(), -1);
    while (t_[p_].kind != T_END) {
      if (!(t_[p_].kind == T_IDENT && t_[p_ + 1].kind == T_DEFINE)) parse_fail(t_[p_].pos, "expected 'name ::='");
      int r = rule_index_[t_[p_].text];
      p_ += 2;
      Frag f = alternatives();
      if (t_[p_].kind == T_RP) parse_fail(t_[p_].pos, "unbalanced ')'");
      start_[r] = f.in;
      accept_[r] = f.out;
    }
  }
  std::vector<std::string> names_;
  std::map<std::string, int> rule_index_;
  std::vector<int> start_, accept_;

 private:
  const std::vector<Token>& t_;
  Nfa& nfa_;
  size_t p_ = 0;

  bool at_rule_head() const { return t_[p_].kind == T_IDENT && t_[p_ + 1].kind == T_DEFINE; }
  Frag alternatives() {
    Frag first = sequence();
    if (t_[p_].kind != T_PIPE) return first;
    int in = nfa_.add(), out = nfa_.add();
    nfa_.eps(in, first.in);
    nfa_.eps(first.out, out);
    while (t_[p_].kind == T_PIPE) {
      ++p_;
      Frag f = sequence();
      nfa_.eps(in, f.in);
      nfa_.eps(f.out, out);
    }
    return {in, out};
  }
  Frag sequence() {
    int in = nfa_.add();
    int cur = in;
    for (;;) {
      TokKind k = t_[p_].kind;
      if (k == T_END || k == T_PIPE || k == T_RP || at_rule_head()) break;
      Frag f = item();
      nfa_.eps(cur, f.in);
      cur = f.out;
    }
    return {in, cur};
  }
  Frag item() {
    Frag f = atom();
    for (;;) {
      TokKind k = t_[p_].kind;
      if (k == T_STAR) {
        int hub = nfa_.add();
        nfa_.eps(hub, f.in);
        nfa_.eps(f.out, hub);
        f = {hub, hub};
      } else if (k == T_PLUS) {
        int out = nfa_.add();
        nfa_.eps(f.out, out);
        nfa_.eps(out, f.in);
        f = {f.in, out};
      } else if (k == T_QUEST) {
        int in = nfa_.add(), out = nfa_.add();
        nfa_.eps(in, f.in);
        nfa_.eps(f.out, out);
        nfa_.eps(in, out);
        f = {in, out};
      } else break;
      ++p_;
    }
    return f;
  }
  Frag atom() {
    const Token& tk = t_[p_];
    switch (tk.kind) {
      case T_LIT: {
        ++p_;
        int in = nfa_.add(), cur = in;
        for (unsigned char c : tk.text) { int nx = nfa_.add(); nfa_.bytes(cur, c, c, nx); cur = nx; }
        return {in, cur};
      }
      case T_CLASS: {
        ++p_;
        int in = nfa_.add(), out = nfa_.add();
        for (auto& r : tk.ranges) add_codepoints(r.lo, r.hi, in, out);
        return {in, out};
      }
      case T_IDENT: {
        ++p_;
        auto it = rule_index_.find(tk.text);
        if (it == rule_index_.end()) throw Failure(XGM_ERR_UNDEFINED_RULE, "grammar: rule '" + tk.text + "' is not defined");
        int in = nfa_.add(), out = nfa_.add();
        nfa_.ref(in, it->second, out);
        return {in, out};
      }
      case T_LP: {
        ++p_;
        Frag f = alternatives();
        if (t_[p_].kind != T_RP) parse_fail(t_[p_].pos, "expected ')'");
        ++p_;
        return f;
      }
      default: parse_fail(tk.pos, "expected a literal, class, rule name or '('");
    }
  }
  // UTF-8 byte sequences for the scalar values lo..hi: cut the range where
  // the encoded length changes, then where a continuation byte would not
  // span its full 0x80..0xBF range, and emit one chain of byte ranges per piece.
  void add_codepoints(uint32_t lo, uint32_t hi, int in, int out) {
    static const uint32_t last_of_len[4] = {0x7F, 0x7FF, 0xFFFF, 0x10FFFF};
    for (int len = 1; len <= 4 && lo <= hi; ++len) {
      if (lo > last_of_len[len - 1]) continue;
      uint32_t top = std::min(hi, last_of_len[len - 1]);
      same_length(lo, top, len, in, out);
      lo = top + 1;
      if (top == 0x10FFFF) break;
    }
  }
  void same_length(uint32_t lo, uint32_t hi, int len, int in, int out) {
    for (int k = 1; k < len; ++k) {
      uint32_t low_bits = (1u << (6 * k)) - 1;
      if ((lo & ~low_bits) != (hi & ~low_bits)) {
        if ((lo & low_bits) != 0) {
          same_length(lo, lo | low_bits, len, in, out);
          same_length((lo | low_bits) + 1, hi, len, in, out);
          return;
        }
        if ((hi & low_bits) != low_bits) {
          same_length(lo, (hi & ~low_bits) - 1, len, in, out);
          same_length(hi & ~low_bits, hi, len, in, out);
          return;
        }
      }
    }
    std::string a, b;
    append_utf8(lo, a);
    append_utf8(hi, b);
    int cur = in;
    for (int k = 0; k < len; ++k) {
      int nx = (k + 1 == len) ? out : nfa_.add();
      nfa_.bytes(cur, (unsigned char)a[k], (unsigned char)b[k], nx);
      cur = nx;
    }
  }
};

// ------------------------------------------------------- per-rule DFA
struct DState {
  bool final_ = false;
  std::vector<ByteEdge> b;  // sorted, disjoint, maximal
  std::vector<RefEdge> r;   // sorted by rule
};
using Dfa = std::vector<DState>;  // state 0 is the start

void merge_byte_edges(std::vector<ByteEdge>& e) {
  std::sort(e.begin(), e.end(), [](const ByteEdge& x, const ByteEdge& y) { return x.lo < y.lo; });
  std::vector<ByteEdge> out;
  for (auto& x : e) {
    if (!out.empty() && out.back().to == x.to && (int)out.back().hi + 1 == (int)x.lo) out.back().hi = x.hi;
    else out.push_back(x);
  }
  e.swap(out);
}

}  // namespace

Automaton compile_grammar(const std::string& text, const std::string& root) {
  std::vector<Token> toks = lex(text);
  Nfa nfa;
  Parser parser(toks, nfa);
  parser.run();
  const int R = (int)parser.names_.size();
  auto root_it = parser.rule_index_.find(root);
  if (root_it == parser.rule_index_.end())
    throw Failure(XGM_ERR_UNDEFINED_RULE, "grammar: root rule '" + root + "' is not defined");
  const int root_rule = root_it->second;
  const int S = (int)nfa.out.size();

  // reverse edges, for backward searches
  std::vector<std::vector<std::pair<int, int>>> rev(S);
  for (int q = 0; q < S; ++q)
    for (size_t k = 0; k < nfa.out[q].size(); ++k) rev[nfa.out[q][k].to].push_back({q, (int)k});
  auto backward = [&](int target, auto usable) {
    std::vector<char> mark(S, 0);
    std::vector<int> work{target};
    mark[target] = 1;
    while (!work.empty()) {
      int t = work.back();
      work.pop_back();
      for (auto& pk : rev[t])
        if (!mark[pk.first] && usable(nfa.out[pk.first][pk.second])) { mark[pk.first] = 1; work.push_back(pk.first); }
    }
    return mark;
  };

  // productive rules (derive at least one string) and nullable rules (derive "")
  std::vector<char> productive(R, 0), nullable(R, 0);
  for (bool changed = true; changed;) {
    changed = false;
    for (int r = 0; r < R; ++r) {
      if (productive[r]) continue;
      auto m = backward(parser.accept_[r], [&](const NEdge& e) { return e.kind != 2 || productive[e.rule]; });
      if (m[parser.start_[r]]) { productive[r] = 1; changed = true; }
    }
  }
  if (!productive[root_rule]) throw Failure(XGM_ERR_UNPRODUCTIVE, "grammar: the root rule derives no string");
  for (bool changed = true; changed;) {
    changed = false;
    for (int r = 0; r < R; ++r) {
      if (nullable[r] || !productive[r]) continue;
      auto m = backward(parser.accept_[r], [&](const NEdge& e) { return e.kind == 0 || (e.kind == 2 && nullable[e.rule]); });
      if (m[parser.start_[r]]) { nullable[r] = 1; changed = true; }
    }
  }

  // silent closure: epsilon edges, and references to nullable rules skipped
  auto closure = [&](std::vector<int> seed) {
    std::set<int> seen(seed.begin(), seed.end());
    while (!seed.empty()) {
      int q = seed.back();
      seed.pop_back();
      for (auto& e : nfa.out[q]) {
        bool silent = e.kind == 0 || (e.kind == 2 && productive[e.rule] && nullable[e.rule]);
        if (silent && seen.insert(e.to).second) seed.push_back(e.to);
      }
    }
    return std::vector<int>(seen.begin(), seen.end());
  };

  // subset construction + trimming + minimisation, rule by rule
  std::vector<Dfa> dfa(R);
  for (int r = 0; r < R; ++r) {
    if (!productive[r]) continue;
    std::map<std::vector<int>, int> ids;
    std::vector<std::vector<int>> sets;
    Dfa d;
    auto intern = [&](std::vector<int> set) {
      auto it = ids.find(set);
      if (it != ids.end()) return it->second;
      int id = (int)sets.size();
      ids[set] = id;
      sets.push_back(set);
      d.emplace_back();
      return id;
    };
    intern(closure({parser.start_[r]}));
    for (size_t cur = 0; cur < sets.size(); ++cur) {
      std::vector<int> set = sets[cur];
      bool fin = false;
      std::set<int> cuts;  // interval starts
      std::map<int, std::vector<int>> by_rule;
      for (int q : set) {
        if (q == parser.accept_[r]) fin = true;
        for (auto& e : nfa.out[q]) {
          if (e.kind == 1) { cuts.insert(e.lo); cuts.insert(e.hi + 1); }
          else if (e.kind == 2 && productive[e.rule]) by_rule[e.rule].push_back(e.to);
        }
      }
      std::vector<ByteEdge> be;
      std::vector<int> cut(cuts.begin(), cuts.end());
      for (size_t k = 0; k + 1 < cut.size(); ++k) {
        int lo = cut[k], hi = cut[k + 1] - 1;
        std::vector<int> tgt;
        for (int q : set)
          for (auto& e : nfa.out[q])
            if (e.kind == 1 && e.lo <= lo && hi <= e.hi) tgt.push_back(e.to);
        if (tgt.empty()) continue;
        int to = intern(closure(tgt));
        be.push_back({(uint8_t)lo, (uint8_t)hi, to});
      }
      std::vector<RefEdge> re;
      for (auto& kv : by_rule) re.push_back({kv.first, intern(closure(kv.second))});
      merge_byte_edges(be);
      d[cur].final_ = fin;
      d[cur].b = be;
      d[cur].r = re;
    }
    // trim: keep states that can reach an accepting state
    int n = (int)d.size();
    std::vector<char> alive(n, 0);
    for (bool changed = true; changed;) {
      changed = false;
      for (int q = 0; q < n; ++q) {
        if (alive[q]) continue;
        bool ok = d[q].final_;
        for (auto& e : d[q].b) ok = ok || alive[e.to];
        for (auto& e : d[q].r) ok = ok || alive[e.to];
        if (ok) { alive[q] = 1; changed = true; }
      }
    }
    if (!alive[0]) throw Failure(XGM_ERR_INTERNAL, "grammar: productive rule lost its start state");
    for (int q = 0; q < n; ++q) {
      auto& s = d[q];
      s.b.erase(std::remove_if(s.b.begin(), s.b.end(), [&](const ByteEdge& e) { return !alive[e.to]; }), s.b.end());
      s.r.erase(std::remove_if(s.r.begin(), s.r.end(), [&](const RefEdge& e) { return !alive[e.to]; }), s.r.end());
    }
    // minimise by partition refinement on (accepting, outgoing edges by block)
    std::vector<int> block(n, 0);
    for (int q = 0; q < n; ++q) block[q] = alive[q] ? (d[q].final_ ? 1 : 0) : -1;
    for (;;) {
      std::map<std::vector<int>, int> sig_id;
      std::vector<int> next(n, -1);
      for (int q = 0; q < n; ++q) {
        if (!alive[q]) continue;
        std::vector<int> sig{block[q]};
        std::vector<ByteEdge> eb;
        for (auto& e : d[q].b) eb.push_back({e.lo, e.hi, block[e.to]});
        merge_byte_edges(eb);
        for (auto& e : eb) { sig.push_back(e.lo); sig.push_back(e.hi); sig.push_back(e.to); }
        sig.push_back(-2);
        for (auto& e : d[q].r) { sig.push_back(e.rule); sig.push_back(block[e.to]); }
        auto it = sig_id.find(sig);
        if (it == sig_id.end()) it = sig_id.emplace(sig, (int)sig_id.size()).first;
        next[q] = it->second;
      }
      std::set<int> before, after;
      for (int q = 0; q < n; ++q) if (alive[q]) { before.insert(block[q]); after.insert(next[q]); }
      block = next;
      if (before.size() == after.size()) break;
    }
    // rebuild with the start state's block first
    std::map<int, int> renum;
    renum[block[0]] = 0;
    std::vector<int> rep{0};
    for (int q = 0; q < n; ++q)
      if (alive[q] && !renum.count(block[q])) { renum[block[q]] = (int)rep.size(); rep.push_back(q); }
    Dfa m(rep.size());
    for (size_t k = 0; k < rep.size(); ++k) {
      const DState& s = d[rep[k]];
      m[k].final_ = s.final_;
      for (auto& e : s.b) m[k].b.push_back({e.lo, e.hi, renum[block[e.to]]});
      merge_byte_edges(m[k].b);
      for (auto& e : s.r) m[k].r.push_back({e.rule, renum[block[e.to]]});
    }
    dfa[r] = std::move(m);
  }

  // rules reachable from the root
  std::vector<int> new_index(R, -1), order;
  {
    std::vector<int> work{root_rule};
    new_index[root_rule] = 0;
    order.push_back(root_rule);
    while (!work.empty()) {
      int r = work.back();
      work.pop_back();
      for (auto& s : dfa[r])
        for (auto& e : s.r)
          if (new_index[e.rule] < 0) { new_index[e.rule] = (int)order.size(); order.push_back(e.rule); work.push_back(e.rule); }
    }
  }

  // Small rules first: the rules shared by many call sites (strings, numbers,
  // white space) are small, and the kernels keep the headers of the lowest
  // node ids on chip.
  std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return dfa[a].size() < dfa[b].size(); });
  for (size_t k = 0; k < order.size(); ++k) new_index[order[k]] = (int)k;

  Automaton A;
  A.root_rule = new_index[root_rule];
  int total = 0;
  for (int r : order) { A.rule_start.push_back(total); total += (int)dfa[r].size(); A.rule_names.push_back(parser.names_[r]); }
  if (total > XGM_MAX_NODES) throw Failure(XGM_ERR_TOO_LARGE, "grammar: automaton has " + std::to_string(total) + " nodes (limit 32767)");
  A.n_nodes = total;
  A.node_rule.resize(total);
  A.node_final.resize(total);
  A.bedges.resize(total);
  A.redges.resize(total);
  for (size_t k = 0; k < order.size(); ++k) {
    int base = A.rule_start[k];
    const Dfa& d = dfa[order[k]];
    for (size_t q = 0; q < d.size(); ++q) {
      int n = base + (int)q;
      A.node_rule[n] = (int)k;
      A.node_final[n] = d[q].final_;
      for (auto& e : d[q].b) A.bedges[n].push_back({e.lo, e.hi, base + e.to});
      for (auto& e : d[q].r) A.redges[n].push_back({new_index[e.rule], base + e.to});
    }
  }
  const int NR = (int)order.size();

  // left recursion: a chain of references taken at rule starts that returns to its origin
  {
    std::vector<int> color(NR, 0);
    std::vector<std::pair<int, size_t>> stack;
    for (int s = 0; s < NR; ++s) {
      if (color[s]) continue;
      stack.push_back({s, 0});
      color[s] = 1;
      while (!stack.empty()) {
        auto& top = stack.back();
        const auto& refs = A.redges[A.rule_start[top.first]];
        if (top.second < refs.size()) {
          int t = refs[top.second++].rule;
          if (color[t] == 1)
            throw Failure(XGM_ERR_LEFT_RECURSION, "grammar: rule '" + A.rule_names[t] + "' is left-recursive");
          if (color[t] == 0) { color[t] = 1; stack.push_back({t, 0}); }
        } else {
          color[top.first] = 2;
          stack.pop_back();
        }
      }
    }
  }

  // FIRST sets: bytes with which an instance of the rule can begin
  A.first.assign(NR, {});
  for (bool changed = true; changed;) {
    changed = false;
    for (int r = 0; r < NR; ++r) {
      std::bitset<256> f = A.first[r];
      int s = A.rule_start[r];
      for (auto& e : A.bedges[s]) for (int c = e.lo; c <= e.hi; ++c) f.set(c);
      for (auto& e : A.redges[s]) f |= A.first[e.rule];
      if (f != A.first[r]) { A.first[r] = f; changed = true; }
    }
  }

  A.node_first.assign(total, {});
  for (int n = 0; n < total; ++n) {
    for (auto& e : A.bedges[n]) for (int c = e.lo; c <= e.hi; ++c) A.node_first[n].set(c);
    for (auto& e : A.redges[n]) A.node_first[n] |= A.first[e.rule];
  }
  A.node_first_words.assign((size_t)total * 8, 0u);
  for (int n = 0; n < total; ++n)
    for (int c = 0; c < 256; ++c)
      if (A.node_first[n].test(c)) A.node_first_words[(size_t)n * 8 + (c >> 5)] |= 1u << (c & 31);

  // FOLLOW sets: what can be consumed at the return node of some reference to
  // the rule, and, if the referencing rule may end there, what can follow it.
  // Nothing follows the root rule itself (end of the text).
  A.follow.assign(NR, {});
  for (bool changed = true; changed;) {
    changed = false;
    for (int n = 0; n < total; ++n)
      for (auto& e : A.redges[n]) {
        std::bitset<256> f = A.follow[e.rule] | A.node_first[e.to];
        if (A.node_final[e.to]) f |= A.follow[A.node_rule[n]];
        if (f != A.follow[e.rule]) { A.follow[e.rule] = f; changed = true; }
      }
  }

  // witness paths (breadth-first from each rule start)
  A.node_path.assign(total, {});
  for (int r = 0; r < NR; ++r) {
    int s = A.rule_start[r];
    std::vector<char> seen(total, 0);
    std::queue<int> q;
    q.push(s);
    seen[s] = 1;
    while (!q.empty()) {
      int n = q.front();
      q.pop();
      for (auto& e : A.bedges[n])
        if (!seen[e.to]) { seen[e.to] = 1; A.node_path[e.to] = A.node_path[n]; A.node_path[e.to].push_back(e.lo); q.push(e.to); }
      for (auto& e : A.redges[n])
        if (!seen[e.to]) { seen[e.to] = 1; A.node_path[e.to] = A.node_path[n]; A.node_path[e.to].push_back(256 + e.rule); q.push(e.to); }
    }
  }

  // ---- flatten for the device
  // byte classes: bytes that no node's edges and no FIRST set tell apart
  std::vector<int> row_nodes;
  for (int n = 0; n < total; ++n)
    if (!(A.redges[n].empty() && A.bedges[n].size() <= 1)) row_nodes.push_back(n);
  auto byte_target = [&](int n, int c) {
    for (auto& e : A.bedges[n]) if (e.lo <= c && c <= e.hi) return e.to;
    return -1;
  };
  A.cls.assign(256, 0);
  {
    std::map<std::string, int> key_id;
    for (int c = 0; c < 256; ++c) {
      std::string key;
      for (int n = 0; n < total; ++n) { int t = byte_target(n, c); key += (char)(t & 0xFF); key += (char)((t >> 8) & 0xFF); key += (char)((t >> 16) & 0xFF); }
      for (int r = 0; r < NR; ++r) key += A.first[r].test(c) ? '1' : '0';
      auto it = key_id.find(key);
      if (it == key_id.end()) it = key_id.emplace(key, (int)key_id.size()).first;
      A.cls[c] = (uint8_t)it->second;
    }
    A.n_cls = (int)key_id.size();
  }
  std::vector<int> cls_rep(A.n_cls, -1);
  for (int c = 255; c >= 0; --c) cls_rep[A.cls[c]] = c;

  A.node_dead_end.assign(total, 0);
  for (int n = 0; n < total; ++n)
    A.node_dead_end[n] = A.node_final[n] && A.bedges[n].empty() && A.redges[n].empty();

  // contexts of every rule (see automaton.hpp)
  {
    std::vector<std::set<int32_t>> ctx(NR);
    for (bool changed = true; changed;) {
      changed = false;
      for (int n = 0; n < total; ++n)
        for (auto& e : A.redges[n]) {
          auto& c = ctx[e.rule];
          const size_t before = c.size();
          if (!A.node_dead_end[e.to]) c.insert(e.to);
          else if (e.rule != A.node_rule[n]) { const auto& p = ctx[A.node_rule[n]]; c.insert(p.begin(), p.end()); }
          if (c.size() != before) changed = true;
        }
    }
    A.contexts.assign(NR, {});
    for (int r = 0; r < NR; ++r) A.contexts[r].assign(ctx[r].begin(), ctx[r].end());
  }

  // Alternatives of node n on byte c, in the order the walk tries them:
  //  * the byte edge;
  //  * for every reference whose callee can start with c: enter the callee.
  //    - If the return node is a dead end (accepting, no outgoing edges) no
  //      frame is needed: returning there could only be followed by another
  //      return, so the callee returns straight to the caller's parent.
  //    - Otherwise, if the callee does nothing with c but consume it and end (a single
  //      byte edge from its start into a dead end, no reference of its own
  //      that could start with c), the whole call is the move "consume c, go
  //      to the return node"; the frame would be pushed and popped unseen.
  //    Both are exact for the token classes too: neither changes which bytes
  //    are consumed inside the frame the walk started in.
  auto alternatives = [&](int n, int c) {
    std::vector<uint32_t> list;
    int t = byte_target(n, c);
    if (t >= 0) list.push_back((kMoveTag << 16) | (uint32_t)t);
    for (auto& e : A.redges[n]) {
      if (!A.first[e.rule].test(c)) continue;
      const int s = A.rule_start[e.rule];
      const int m = byte_target(s, c);
      bool callee_refs = false;
      for (auto& e2 : A.redges[s]) callee_refs = callee_refs || A.first[e2.rule].test(c);
      uint32_t alt;
      if (A.node_dead_end[e.to]) alt = (kTailTag << 16) | (uint32_t)s;
      else if (m >= 0 && A.node_dead_end[m] && !callee_refs) alt = (kMoveTag << 16) | (uint32_t)e.to;
      else alt = ((uint32_t)e.to << 16) | (uint32_t)s;
      if (std::find(list.begin(), list.end(), alt) == list.end()) list.push_back(alt);
    }
    return list;
  };

  // Branching nodes: for every byte class one of the node's few outcomes.
  // Which class leads to which outcome index is the node's "shape" (shared by
  // many nodes, e.g. every  ws "," ws  position); the outcomes themselves are
  // the node's own slice of `targets`.
  A.hdr.assign(total, NodeHdr{1, 0, 0, 0});
  std::map<std::vector<uint32_t>, uint32_t> alt_ids;
  std::map<std::vector<uint8_t>, uint32_t> shape_ids;
  for (int n = 0; n < total; ++n) {
    NodeHdr& h = A.hdr[n];
    h.flags = (A.node_final[n] ? kFlagFinal : 0) | (A.node_dead_end[n] ? kFlagDeadEnd : 0);
    if (A.redges[n].empty() && A.bedges[n].size() <= 1) {
      if (A.bedges[n].size() == 1) { h.lo = A.bedges[n][0].lo; h.hi = A.bedges[n][0].hi; h.target = (uint16_t)A.bedges[n][0].to; }
      continue;
    }
    std::vector<uint8_t> shape(A.n_cls, kDeadShape);
    std::vector<uint16_t> outcomes;
    for (int k = 0; k < A.n_cls; ++k) {
      std::vector<uint32_t> list = alternatives(n, cls_rep[k]);
      if (list.empty()) continue;
      uint16_t entry;
      if (list.size() == 1 && (list[0] >> 16) == kMoveTag) entry = (uint16_t)(list[0] & 0xFFFF);
      else {
        if (list.size() > 250) throw Failure(XGM_ERR_TOO_LARGE, "grammar: too many alternatives at one node");
        auto it = alt_ids.find(list);
        if (it == alt_ids.end()) {
          uint32_t at = (uint32_t)A.alts.size();
          if (at >= 0x7FFF) throw Failure(XGM_ERR_TOO_LARGE, "grammar: alternatives pool is full");
          A.alts.push_back((uint32_t)list.size());
          A.alts.insert(A.alts.end(), list.begin(), list.end());
          it = alt_ids.emplace(list, at).first;
        }
        entry = (uint16_t)(kAltFlag | it->second);
        A.max_alts = std::max<int>(A.max_alts, (int)list.size());
      }
      size_t idx = std::find(outcomes.begin(), outcomes.end(), entry) - outcomes.begin();
      if (idx == outcomes.size()) outcomes.push_back(entry);
      if (idx >= kDeadShape) throw Failure(XGM_ERR_TOO_LARGE, "grammar: too many distinct outcomes at one node");
      shape[k] = (uint8_t)idx;
    }
    auto it = shape_ids.find(shape);
    if (it == shape_ids.end()) {
      uint32_t id = (uint32_t)shape_ids.size();
      if (id >= 0xFFFF) throw Failure(XGM_ERR_TOO_LARGE, "grammar: too many node shapes");
      A.shapes.insert(A.shapes.end(), shape.begin(), shape.end());
      it = shape_ids.emplace(shape, id).first;
    }
    if (A.targets.size() + outcomes.size() > 0xFFFF) throw Failure(XGM_ERR_TOO_LARGE, "grammar: outcome table is full");
    h.flags |= kFlagBranching;
    h.lo = (uint8_t)(it->second & 0xFF);          // shape id, low and high byte
    h.hi = (uint8_t)(it->second >> 8);
    h.target = (uint16_t)A.targets.size();        // start of this node's outcomes
    A.targets.insert(A.targets.end(), outcomes.begin(), outcomes.end());
  }
  A.n_shapes = (int32_t)shape_ids.size();
  for (int n = 0; n < total; ++n) A.hdr[n].flags |= (uint32_t)A.node_rule[n] << 16;
  A.follow_words.assign((size_t)NR * 8, 0u);
  for (int r = 0; r < NR; ++r)
    for (int c = 0; c < 256; ++c) A.follow_words[(size_t)r * 8 + (c >> 5)] |= (uint32_t)A.follow[r].test(c) << (c & 31);
  if (A.alts.empty()) A.alts.push_back(0);
  if (A.shapes.empty()) A.shapes.assign(A.n_cls, kDeadShape);
  if (A.targets.empty()) A.targets.push_back(0);
  return A;
}

}  // namespace xgm
