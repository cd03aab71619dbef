// TEST INFRASTRUCTURE ONLY: part of the slow CPU oracle.  Nothing in the
// product library includes, links or calls this file.
//
// Grammar text -> syntax tree.  The paper shows its grammar notation only in
// a figure (Figure 3: an EBNF with rules, quoted literals and character
// classes such as [^"\\]); the dialect read here is the small EBNF that the
// synthetic workloads are written in:
//
//   rule   : name "::=" alt            (a rule ends where the next one begins)
//   alt    : seq ("|" seq)*
//   seq    : item*                     (an empty sequence matches "")
//   item   : atom ("*" | "+" | "?")?
//   atom   : "literal" | [class] | name | "(" alt ")"
//   # ... comment to end of line
//
// Literals are byte strings (escapes \" \\ \' \/ \n \t \r \b \f \xHH \uHHHH;
// \xHH is one raw byte, \uHHHH the UTF-8 encoding of that code point).
// Classes are sets of Unicode scalar values (escapes as above plus \] \[ \-
// \^; \xHH there means code point HH); "^" right after "[" negates with
// respect to all scalar values 0..0x10FFFF except surrogates.
#pragma once
#include <cstdint>
#include <map>
#include <stdexcept>
#include <string>
#include <utility>
#include <vector>

namespace orc {

struct Expr {
  enum Kind { ALT, SEQ, STAR, PLUS, OPT, BYTES, CLASS, REF } kind;
  std::vector<int> kids;                               // ALT, SEQ, STAR, PLUS, OPT
  std::string bytes;                                   // BYTES
  std::vector<std::pair<uint32_t, uint32_t>> ranges;   // CLASS (inclusive)
  bool negated = false;                                // CLASS
  int rule = -1;                                       // REF (resolved index)
  std::string name;                                    // REF (as written)
};

struct Grammar {
  std::vector<Expr> pool;
  std::vector<std::string> rule_names;
  std::vector<int> rule_body;  // index into pool
  std::map<std::string, int> rule_index;
  int root = -1;
};

class TextReader {
 public:
  explicit TextReader(const std::string& s) : s_(s) {}

  Grammar read(const std::string& root_name) {
    skip();
    while (pos_ < s_.size()) {
      std::string name = ident();
      if (name.empty()) fail("expected a rule name");
      skip();
      if (!lit("::=")) fail("expected '::=' after rule name '" + name + "'");
      if (g_.rule_index.count(name)) fail("rule '" + name + "' defined twice");
      int body = alt();
      g_.rule_index[name] = (int)g_.rule_names.size();
      g_.rule_names.push_back(name);
      g_.rule_body.push_back(body);
      skip();
    }
    if (g_.rule_names.empty()) fail("no rules");
    for (auto& e : g_.pool)
      if (e.kind == Expr::REF) {
        auto it = g_.rule_index.find(e.name);
        if (it == g_.rule_index.end()) throw std::runtime_error("undefined rule '" + e.name + "'");
        e.rule = it->second;
      }
    auto it = g_.rule_index.find(root_name);
    if (it == g_.rule_index.end()) throw std::runtime_error("root rule '" + root_name + "' not found");
    g_.root = it->second;
    return std::move(g_);
  }

 private:
  const std::string& s_;
  size_t pos_ = 0;
  Grammar g_;

  [[noreturn]] void fail(const std::string& why) {
    throw std::runtime_error("grammar parse error at offset " + std::to_string(pos_) + ": " + why);
  }
  void skip() {
    for (;;) {
      while (pos_ < s_.size() && (s_[pos_] == ' ' || s_[pos_] == '\t' || s_[pos_] == '\n' || s_[pos_] == '\r')) ++pos_;
      if (pos_ < s_.size() && s_[pos_] == '#') {
        while (pos_ < s_.size() && s_[pos_] != '\n') ++pos_;
        continue;
      }
      return;
    }
  }
  bool lit(const char* t) {
    size_t n = std::char_traits<char>::length(t);
    if (s_.compare(pos_, n, t) == 0) { pos_ += n; return true; }
    return false;
  }
  static bool id_start(char c) { return (c >= 'a' && c <= 'z') || (c >= 'A' && c <= 'Z') || c == '_'; }
  static bool id_char(char c) { return id_start(c) || (c >= '0' && c <= '9'); }
  std::string ident() {
    size_t b = pos_;
    if (pos_ < s_.size() && id_start(s_[pos_])) {
      ++pos_;
      while (pos_ < s_.size() && id_char(s_[pos_])) ++pos_;
    }
    return s_.substr(b, pos_ - b);
  }
  // true if an identifier followed by "::=" starts here (the next rule)
  bool at_rule_head() {
    size_t save = pos_;
    std::string n = ident();
    bool yes = false;
    if (!n.empty()) { skip(); yes = s_.compare(pos_, 3, "::=") == 0; }
    pos_ = save;
    return yes;
  }
  int add(Expr e) { g_.pool.push_back(std::move(e)); return (int)g_.pool.size() - 1; }

  int alt() {
    std::vector<int> alts{seq()};
    skip();
    while (pos_ < s_.size() && s_[pos_] == '|') { ++pos_; alts.push_back(seq()); skip(); }
    if (alts.size() == 1) return alts[0];
    Expr e; e.kind = Expr::ALT; e.kids = alts; return add(e);
  }
  int seq() {
    std::vector<int> items;
    for (;;) {
      skip();
      if (pos_ >= s_.size()) break;
      char c = s_[pos_];
      if (c == '|' || c == ')') break;
      if (id_start(c) && at_rule_head()) break;
      items.push_back(item());
    }
    if (items.size() == 1) return items[0];
    Expr e; e.kind = Expr::SEQ; e.kids = items; return add(e);
  }
  int item() {
    int a = atom();
    for (;;) {
      skip();
      if (pos_ >= s_.size()) break;
      char c = s_[pos_];
      Expr e;
      if (c == '*') e.kind = Expr::STAR; else if (c == '+') e.kind = Expr::PLUS; else if (c == '?') e.kind = Expr::OPT; else break;
      ++pos_;
      e.kids = {a};
      a = add(e);
    }
    return a;
  }
  int atom() {
    skip();
    if (pos_ >= s_.size()) fail("unexpected end of grammar");
    char c = s_[pos_];
    if (c == '"') return literal();
    if (c == '[') return klass();
    if (c == '(') {
      ++pos_;
      int a = alt();
      skip();
      if (pos_ >= s_.size() || s_[pos_] != ')') fail("expected ')'");
      ++pos_;
      return a;
    }
    if (id_start(c)) { Expr e; e.kind = Expr::REF; e.name = ident(); return add(e); }
    fail(std::string("unexpected character '") + c + "'");
  }
  int hexval(char c) {
    if (c >= '0' && c <= '9') return c - '0';
    if (c >= 'a' && c <= 'f') return c - 'a' + 10;
    if (c >= 'A' && c <= 'F') return c - 'A' + 10;
    fail("bad hex digit");
  }
  uint32_t hexn(int n) {
    if (pos_ + n > s_.size()) fail("truncated hex escape");
    uint32_t v = 0;
    for (int i = 0; i < n; ++i) v = v * 16 + hexval(s_[pos_++]);
    return v;
  }
  static void put_utf8(uint32_t cp, std::string& out) {
    if (cp < 0x80) out.push_back((char)cp);
    else if (cp < 0x800) { out.push_back((char)(0xC0 | (cp >> 6))); out.push_back((char)(0x80 | (cp & 0x3F))); }
    else if (cp < 0x10000) { out.push_back((char)(0xE0 | (cp >> 12))); out.push_back((char)(0x80 | ((cp >> 6) & 0x3F))); out.push_back((char)(0x80 | (cp & 0x3F))); }
    else { out.push_back((char)(0xF0 | (cp >> 18))); out.push_back((char)(0x80 | ((cp >> 12) & 0x3F))); out.push_back((char)(0x80 | ((cp >> 6) & 0x3F))); out.push_back((char)(0x80 | (cp & 0x3F))); }
  }
  int literal() {
    ++pos_;  // opening quote
    Expr e; e.kind = Expr::BYTES;
    for (;;) {
      if (pos_ >= s_.size()) fail("unterminated literal");
      char c = s_[pos_++];
      if (c == '"') break;
      if (c != '\\') { e.bytes.push_back(c); continue; }
      if (pos_ >= s_.size()) fail("unterminated escape");
      char k = s_[pos_++];
      switch (k) {
        case 'n': e.bytes.push_back('\n'); break;
        case 't': e.bytes.push_back('\t'); break;
        case 'r': e.bytes.push_back('\r'); break;
        case 'b': e.bytes.push_back('\b'); break;
        case 'f': e.bytes.push_back('\f'); break;
        case '"': case '\\': case '\'': case '/': e.bytes.push_back(k); break;
        case 'x': e.bytes.push_back((char)hexn(2)); break;
        case 'u': { uint32_t cp = hexn(4); if (cp >= 0xD800 && cp <= 0xDFFF) fail("surrogate in \\u escape"); put_utf8(cp, e.bytes); break; }
        default: fail(std::string("unknown escape \\") + k);
      }
    }
    return add(e);
  }
  // one code point of a class, decoding UTF-8 text or an escape
  uint32_t class_char() {
    if (pos_ >= s_.size()) fail("unterminated class");
    unsigned char c = (unsigned char)s_[pos_++];
    if (c == '\\') {
      if (pos_ >= s_.size()) fail("unterminated escape");
      char k = s_[pos_++];
      switch (k) {
        case 'n': return '\n'; case 't': return '\t'; case 'r': return '\r';
        case 'b': return '\b'; case 'f': return '\f';
        case '"': case '\\': case '\'': case '/': case ']': case '[': case '-': case '^': return (unsigned char)k;
        case 'x': return hexn(2);
        case 'u': return hexn(4);
        default: fail(std::string("unknown escape \\") + k);
      }
    }
    if (c < 0x80) return c;
    int extra = (c >= 0xF0) ? 3 : (c >= 0xE0) ? 2 : (c >= 0xC0) ? 1 : -1;
    if (extra < 0) fail("bad UTF-8 in class");
    uint32_t cp = c & (0x3F >> extra);
    for (int i = 0; i < extra; ++i) {
      if (pos_ >= s_.size() || ((unsigned char)s_[pos_] & 0xC0) != 0x80) fail("bad UTF-8 in class");
      cp = (cp << 6) | ((unsigned char)s_[pos_++] & 0x3F);
    }
    return cp;
  }
  int klass() {
    ++pos_;  // '['
    Expr e; e.kind = Expr::CLASS;
    if (pos_ < s_.size() && s_[pos_] == '^') { e.negated = true; ++pos_; }
    for (;;) {
      if (pos_ >= s_.size()) fail("unterminated class");
      if (s_[pos_] == ']') { ++pos_; break; }
      uint32_t lo = class_char(), hi = lo;
      if (pos_ + 1 < s_.size() && s_[pos_] == '-' && s_[pos_ + 1] != ']') { ++pos_; hi = class_char(); }
      if (hi < lo) fail("reversed range in class");
      e.ranges.push_back({lo, hi});
    }
    return add(e);
  }
};

inline Grammar read_grammar(const std::string& text, const std::string& root) {
  TextReader r(text);
  return r.read(root);
}

}  // namespace orc
