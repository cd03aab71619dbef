// JSON-schema front end: turns a schema (a documented subset) into grammar
// text in this library's dialect, so that the schema-constrained workloads of
// arxiv 2411.15100 (section 4.1: JSON schema tasks) can be set up from the
// schema itself.  Host code only; the result goes through xgm_grammar_compile
// like any other grammar.
#include "schema.hpp"

#include <cstdint>
#include <set>
#include <utility>
#include <vector>

#include "../../include/xgm.h"

namespace xgm {

namespace {

// ---- a small JSON reader (objects keep the order of their members)
struct Json {
  enum Kind { kNull, kBool, kNumber, kString, kArray, kObject } kind = kNull;
  bool b = false;
  std::string text;  // string value (UTF-8), or the number as it was written
  std::vector<Json> items;
  std::vector<std::pair<std::string, Json>> members;
  const Json* find(const std::string& key) const {
    for (auto& m : members)
      if (m.first == key) return &m.second;
    return nullptr;
  }
};

[[noreturn]] void bad(const std::string& what) { throw Failure(XGM_ERR_PARSE, "schema: " + what); }

class JsonReader {
 public:
  JsonReader(const std::string& s) : s_(s) {}
  Json read() {
    Json v = value(0);
    ws();
    if (i_ != s_.size()) bad("text after the end of the JSON value at byte " + std::to_string(i_));
    return v;
  }

 private:
  const std::string& s_;
  size_t i_ = 0;
  void ws() {
    while (i_ < s_.size() && (s_[i_] == ' ' || s_[i_] == '\t' || s_[i_] == '\n' || s_[i_] == '\r')) ++i_;
  }
  bool eat(const char* lit) {
    size_t k = 0;
    while (lit[k] && i_ + k < s_.size() && s_[i_ + k] == lit[k]) ++k;
    if (lit[k]) return false;
    i_ += k;
    return true;
  }
  static void put_utf8(std::string& out, uint32_t cp) {
    if (cp < 0x80) out += (char)cp;
    else if (cp < 0x800) { out += (char)(0xC0 | (cp >> 6)); out += (char)(0x80 | (cp & 63)); }
    else if (cp < 0x10000) { out += (char)(0xE0 | (cp >> 12)); out += (char)(0x80 | ((cp >> 6) & 63)); out += (char)(0x80 | (cp & 63)); }
    else { out += (char)(0xF0 | (cp >> 18)); out += (char)(0x80 | ((cp >> 12) & 63)); out += (char)(0x80 | ((cp >> 6) & 63)); out += (char)(0x80 | (cp & 63)); }
  }
  uint32_t hex4() {
    if (i_ + 4 > s_.size()) bad("truncated \\u escape");
    uint32_t v = 0;
    for (int k = 0; k < 4; ++k) {
      const char c = s_[i_++];
      v <<= 4;
      if (c >= '0' && c <= '9') v |= (uint32_t)(c - '0');
      else if (c >= 'a' && c <= 'f') v |= (uint32_t)(c - 'a' + 10);
      else if (c >= 'A' && c <= 'F') v |= (uint32_t)(c - 'A' + 10);
      else bad("bad \\u escape");
    }
    return v;
  }
  std::string string() {
    std::string out;
    ++i_;  // opening quote
    for (;;) {
      if (i_ >= s_.size()) bad("unterminated string");
      const unsigned char c = (unsigned char)s_[i_++];
      if (c == '"') return out;
      if (c < 0x20) bad("control character inside a string");
      if (c != '\\') { out += (char)c; continue; }
      if (i_ >= s_.size()) bad("unterminated escape");
      const char e = s_[i_++];
      switch (e) {
        case '"': out += '"'; break;
        case '\\': out += '\\'; break;
        case '/': out += '/'; break;
        case 'b': out += '\b'; break;
        case 'f': out += '\f'; break;
        case 'n': out += '\n'; break;
        case 'r': out += '\r'; break;
        case 't': out += '\t'; break;
        case 'u': {
          uint32_t cp = hex4();
          if (cp >= 0xD800 && cp < 0xDC00) {
            if (!eat("\\u")) bad("lone surrogate in a string");
            const uint32_t lo = hex4();
            if (lo < 0xDC00 || lo >= 0xE000) bad("lone surrogate in a string");
            cp = 0x10000 + ((cp - 0xD800) << 10) + (lo - 0xDC00);
          } else if (cp >= 0xDC00 && cp < 0xE000) {
            bad("lone surrogate in a string");
          }
          put_utf8(out, cp);
          break;
        }
        default: bad("unknown escape in a string");
      }
    }
  }
  Json value(int depth) {
    if (depth > 64) bad("nesting deeper than 64");
    ws();
    if (i_ >= s_.size()) bad("unexpected end of text");
    Json v;
    const char c = s_[i_];
    if (c == '{') {
      v.kind = Json::kObject;
      ++i_;
      ws();
      if (i_ < s_.size() && s_[i_] == '}') { ++i_; return v; }
      for (;;) {
        ws();
        if (i_ >= s_.size() || s_[i_] != '"') bad("member name expected at byte " + std::to_string(i_));
        std::string key = string();
        ws();
        if (i_ >= s_.size() || s_[i_] != ':') bad("':' expected at byte " + std::to_string(i_));
        ++i_;
        Json member = value(depth + 1);
        if (v.find(key)) bad("member \"" + key + "\" given twice");
        v.members.emplace_back(std::move(key), std::move(member));
        ws();
        if (i_ < s_.size() && s_[i_] == ',') { ++i_; continue; }
        if (i_ < s_.size() && s_[i_] == '}') { ++i_; return v; }
        bad("',' or '}' expected at byte " + std::to_string(i_));
      }
    }
    if (c == '[') {
      v.kind = Json::kArray;
      ++i_;
      ws();
      if (i_ < s_.size() && s_[i_] == ']') { ++i_; return v; }
      for (;;) {
        v.items.push_back(value(depth + 1));
        ws();
        if (i_ < s_.size() && s_[i_] == ',') { ++i_; continue; }
        if (i_ < s_.size() && s_[i_] == ']') { ++i_; return v; }
        bad("',' or ']' expected at byte " + std::to_string(i_));
      }
    }
    if (c == '"') { v.kind = Json::kString; v.text = string(); return v; }
    if (eat("true")) { v.kind = Json::kBool; v.b = true; return v; }
    if (eat("false")) { v.kind = Json::kBool; v.b = false; return v; }
    if (eat("null")) { v.kind = Json::kNull; return v; }
    // number: -? int frac? exp?
    const size_t start = i_;
    if (i_ < s_.size() && s_[i_] == '-') ++i_;
    if (i_ >= s_.size()) bad("number expected");
    if (s_[i_] == '0') ++i_;
    else if (s_[i_] >= '1' && s_[i_] <= '9') { while (i_ < s_.size() && s_[i_] >= '0' && s_[i_] <= '9') ++i_; }
    else bad("unexpected character at byte " + std::to_string(i_));
    if (i_ < s_.size() && s_[i_] == '.') {
      ++i_;
      const size_t d = i_;
      while (i_ < s_.size() && s_[i_] >= '0' && s_[i_] <= '9') ++i_;
      if (i_ == d) bad("digits expected after '.'");
    }
    if (i_ < s_.size() && (s_[i_] == 'e' || s_[i_] == 'E')) {
      ++i_;
      if (i_ < s_.size() && (s_[i_] == '+' || s_[i_] == '-')) ++i_;
      const size_t d = i_;
      while (i_ < s_.size() && s_[i_] >= '0' && s_[i_] <= '9') ++i_;
      if (i_ == d) bad("digits expected in the exponent");
    }
    v.kind = Json::kNumber;
    v.text = s_.substr(start, i_ - start);
    return v;
  }
};

// ---- schema -> grammar text
// the text a string takes in a JSON document in its shortest form: only '"', '\\' and control
// characters are escaped (the form Python's json.dumps(..., ensure_ascii=False) writes)
std::string json_spelling(const std::string& s) {
  static const char* kHex = "0123456789abcdef";
  std::string out = "\"";
  for (unsigned char c : s) {
    switch (c) {
      case '"': out += "\\\""; break;
      case '\\': out += "\\\\"; break;
      case '\b': out += "\\b"; break;
      case '\f': out += "\\f"; break;
      case '\n': out += "\\n"; break;
      case '\r': out += "\\r"; break;
      case '\t': out += "\\t"; break;
      default:
        if (c < 0x20) { out += "\\u00"; out += kHex[c >> 4]; out += kHex[c & 15]; }
        else out += (char)c;
    }
  }
  return out + "\"";
}
// a grammar literal for document text (printable ASCII and UTF-8; see json_spelling)
std::string literal(const std::string& document_text) {
  std::string out = "\"";
  for (char c : document_text) {
    if (c == '"' || c == '\\') out += '\\';
    out += c;
  }
  return out + "\"";
}

const char* kSharedRules =
    "string  ::= \"\\\"\" chars \"\\\"\"\n"
    "chars   ::= char*\n"
    "char    ::= [^\"\\\\\\x00-\\x1f] | \"\\\\\" escape\n"
    "escape  ::= [\"\\\\/bfnrt] | \"u\" hex hex hex hex\n"
    "hex     ::= [0-9a-fA-F]\n"
    "integer ::= \"-\"? int\n"
    "number  ::= \"-\"? int frac? exp?\n"
    "int     ::= \"0\" | [1-9] [0-9]*\n"
    "frac    ::= \".\" [0-9]+\n"
    "exp     ::= [eE] [+\\-]? [0-9]+\n"
    "boolean ::= \"true\" | \"false\"\n"
    "null    ::= \"null\"\n"
    "anyvalue  ::= anyobject | anyarray | string | number | boolean | null\n"
    "anyobject ::= \"{\" ws ( string ws \":\" ws anyvalue ( ws \",\" ws string ws \":\" ws anyvalue )* ws )? \"}\"\n"
    "anyarray  ::= \"[\" ws ( anyvalue ( ws \",\" ws anyvalue )* ws )? \"]\"\n"
    "ws      ::= [ \\t\\n\\r]*\n";

class Converter {
 public:
  std::string run(const Json& schema) {
    const std::string top = emit(schema, 0);
    return "root ::= ws " + top + " ws\n" + rules_ + kSharedRules;
  }

 private:
  std::string rules_;
  int counter_ = 0;
  std::string fresh(const char* prefix) { return std::string(prefix) + "_" + std::to_string(++counter_); }
  void rule(const std::string& name, const std::string& body) { rules_ += name + " ::= " + body + "\n"; }

  static std::string value_literal(const Json& v) {
    switch (v.kind) {
      case Json::kNull: return literal("null");
      case Json::kBool: return literal(v.b ? "true" : "false");
      case Json::kNumber: return literal(v.text);
      case Json::kString: return literal(json_spelling(v.text));
      default: bad("enum and const values must be strings, numbers, booleans or null");
    }
  }

  std::string emit_typed(const std::string& type, const Json& s, int depth) {
    if (type == "string") return "string";
    if (type == "integer") return "integer";
    if (type == "number") return "number";
    if (type == "boolean") return "boolean";
    if (type == "null") return "null";
    if (type == "array") return emit_array(s, depth);
    if (type == "object") return emit_object(s, depth);
    bad("unknown type \"" + type + "\"");
  }

  std::string emit_array(const Json& s, int depth) {
    const Json* items = s.find("items");
    if (items && items->kind == Json::kArray) bad("tuple-style \"items\" is not supported");
    const std::string item = items ? emit(*items, depth + 1) : "anyvalue";
    long lo = 0, hi = -1;
    if (const Json* m = s.find("minItems")) lo = count_of(*m, "minItems");
    if (const Json* m = s.find("maxItems")) hi = count_of(*m, "maxItems");
    if (hi >= 0 && hi < lo) bad("maxItems is smaller than minItems");
    const std::string name = fresh("arr");
    const std::string more = "ws \",\" ws " + item;
    std::string tail;  // what may follow the first max(lo, 1) items
    const long fixed = lo > 1 ? lo : 1;
    if (hi < 0) tail = " ( " + more + " )*";
    else
      for (long k = fixed; k < hi; ++k) tail = " ( " + more + tail + " )?";
    std::string first = item;
    for (long k = 1; k < fixed; ++k) first += " " + more;
    if (hi == 0) rule(name, "\"[\" ws \"]\"");
    else if (lo == 0) rule(name, "\"[\" ws ( " + first + tail + " ws )? \"]\"");
    else rule(name, "\"[\" ws " + first + tail + " ws \"]\"");
    return name;
  }

  static long count_of(const Json& v, const char* what) {
    if (v.kind != Json::kNumber) bad(std::string(what) + " must be a number");
    long n = 0;
    for (char c : v.text) {
      if (c < '0' || c > '9') bad(std::string(what) + " must be a non-negative integer");
      n = n * 10 + (c - '0');
      if (n > 64) bad(std::string(what) + " above 64 is not supported");
    }
    return n;
  }

  std::string emit_object(const Json& s, int depth) {
    if (const Json* ap = s.find("additionalProperties"))
      if (!(ap->kind == Json::kBool && !ap->b)) bad("\"additionalProperties\" other than false is not supported");
    const Json* props = s.find("properties");
    if (!props) return "anyobject";
    if (props->kind != Json::kObject) bad("\"properties\" must be an object");
    std::set<std::string> required;
    bool all_required = true;
    if (const Json* req = s.find("required")) {
      if (req->kind != Json::kArray) bad("\"required\" must be an array");
      all_required = false;
      for (auto& r : req->items) {
        if (r.kind != Json::kString) bad("\"required\" must list member names");
        if (!props->find(r.text)) bad("required member \"" + r.text + "\" has no entry in \"properties\"");
        required.insert(r.text);
      }
    }
    const size_t n = props->members.size();
    const std::string name = fresh("obj");
    if (n == 0) { rule(name, "\"{\" ws \"}\""); return name; }
    std::vector<std::string> member(n);
    std::vector<bool> optional(n);
    for (size_t i = 0; i < n; ++i) {
      const std::string ref = emit(props->members[i].second, depth + 1);
      member[i] = literal(json_spelling(props->members[i].first)) + " ws \":\" ws " + ref;
      optional[i] = !all_required && !required.count(props->members[i].first);
    }
    // Members come in the order of "properties".  first_i: the members from i on when none has been
    // written yet; rest_i: when one has (every further one brings its comma).  An optional member may
    // be left out in either.
    std::vector<std::string> first(n + 1), rest(n + 1);
    bool any_optional = false;
    for (size_t i = 0; i < n; ++i) any_optional = any_optional || optional[i];
    if (!any_optional) {
      std::string body = "\"{\" ws ";
      for (size_t i = 0; i < n; ++i) body += (i ? "ws \",\" ws " : "") + member[i] + " ";
      rule(name, body + "ws \"}\"");
      return name;
    }
    for (size_t i = 0; i < n; ++i) { first[i] = name + "_f" + std::to_string(i); rest[i] = name + "_r" + std::to_string(i); }
    auto then = [&](const std::vector<std::string>& v, size_t i) { return i < n ? " " + v[i] : std::string(); };
    auto instead = [&](const std::vector<std::string>& v, size_t i) { return i < n ? " | " + v[i] : std::string(" | \"\""); };
    for (size_t i = n; i-- > 0;) {
      rule(rest[i], "ws \",\" ws " + member[i] + then(rest, i + 1) + (optional[i] ? instead(rest, i + 1) : ""));
      rule(first[i], member[i] + then(rest, i + 1) + (optional[i] ? instead(first, i + 1) : ""));
    }
    rule(name, "\"{\" ws " + first[0] + " ws \"}\"");
    return name;
  }

  std::string emit(const Json& s, int depth) {
    if (depth > 32) bad("schema nested deeper than 32");
    if (s.kind == Json::kBool) {
      if (s.b) return "anyvalue";
      bad("the schema `false` allows nothing");
    }
    if (s.kind != Json::kObject) bad("a schema must be an object (or true)");
    static const char* kUnsupported[] = {"$ref", "allOf", "not", "if", "then", "else", "pattern", "format", "minLength",
                                         "maxLength", "minimum", "maximum", "exclusiveMinimum", "exclusiveMaximum",
                                         "multipleOf", "patternProperties", "propertyNames", "minProperties",
                                         "maxProperties", "dependencies", "dependentRequired", "dependentSchemas",
                                         "prefixItems", "contains", "uniqueItems", "additionalItems",
                                         "unevaluatedProperties", "unevaluatedItems"};
    for (const char* k : kUnsupported)
      if (s.find(k)) bad(std::string("keyword \"") + k + "\" is not supported");
    if (const Json* c = s.find("const")) return named_alternatives("const", {value_literal(*c)});
    if (const Json* e = s.find("enum")) {
      if (e->kind != Json::kArray || e->items.empty()) bad("\"enum\" must be a non-empty array");
      std::vector<std::string> alts;
      for (auto& v : e->items) alts.push_back(value_literal(v));
      return named_alternatives("enum", alts);
    }
    for (const char* key : {"anyOf", "oneOf"})
      if (const Json* u = s.find(key)) {
        if (u->kind != Json::kArray || u->items.empty()) bad(std::string("\"") + key + "\" must be a non-empty array");
        std::vector<std::string> alts;
        for (auto& sub : u->items) alts.push_back(emit(sub, depth + 1));
        return named_alternatives("any", alts);
      }
    const Json* type = s.find("type");
    if (!type) {
      if (s.find("properties")) return emit_object(s, depth);
      if (s.find("items")) return emit_array(s, depth);
      return "anyvalue";
    }
    if (type->kind == Json::kString) return emit_typed(type->text, s, depth);
    if (type->kind == Json::kArray && !type->items.empty()) {
      std::vector<std::string> alts;
      for (auto& t : type->items) {
        if (t.kind != Json::kString) bad("\"type\" must be a name or a list of names");
        alts.push_back(emit_typed(t.text, s, depth));
      }
      return named_alternatives("any", alts);
    }
    bad("\"type\" must be a name or a non-empty list of names");
  }

  std::string named_alternatives(const char* prefix, const std::vector<std::string>& alts) {
    if (alts.size() == 1 && alts[0][0] != '"') return alts[0];
    const std::string name = fresh(prefix);
    std::string body;
    for (size_t i = 0; i < alts.size(); ++i) body += (i ? " | " : "") + alts[i];
    rule(name, body);
    return name;
  }
};

}  // namespace

std::string schema_to_grammar(const std::string& schema_json) {
  JsonReader reader(schema_json);
  const Json schema = reader.read();
  return Converter().run(schema);
}

}  // namespace xgm
