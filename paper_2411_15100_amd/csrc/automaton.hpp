// Host-side grammar compilation: EBNF text -> flattened byte-level pushdown
// automaton (arxiv 2411.15100, section 2.2 and Appendix A: one finite
// automaton per rule, character edges and rule-reference edges).
#pragma once
#include <bitset>
#include <cstdint>
#include <stdexcept>
#include <string>
#include <vector>

namespace xgm {

struct Failure : std::runtime_error {
  int status;
  Failure(int s, const std::string& m) : std::runtime_error(m), status(s) {}
};

struct ByteEdge { uint8_t lo, hi; int32_t to; };
struct RefEdge { int32_t rule; int32_t to; };

// Device header of one node (8 bytes).  If lo <= hi the node has a "primary"
// byte edge [lo, hi] -> target that is tested first; `row` (if not kNoRow)
// selects a dense row indexed by byte class for everything else.
struct NodeHdr {
  uint8_t lo, hi;
  uint16_t target;
  uint16_t row;
  uint16_t flags;  // bit 0: the rule may end at this node
};
static_assert(sizeof(NodeHdr) == 8, "NodeHdr must be 8 bytes");

constexpr uint16_t kNoRow = 0xFFFF;
constexpr uint16_t kDead = 0xFFFF;      // row entry: nothing to do for this byte
constexpr uint16_t kAltFlag = 0x8000;   // row entry: index into the alternatives pool
constexpr uint32_t kMoveTag = 0xFFFF;   // alternative (tag << 16 | node): byte move

struct Automaton {
  // structured form (host engine)
  int32_t n_nodes = 0;
  std::vector<int32_t> node_rule;
  std::vector<uint8_t> node_final;
  std::vector<std::vector<ByteEdge>> bedges;  // sorted, disjoint
  std::vector<std::vector<RefEdge>> redges;
  std::vector<int32_t> rule_start;            // per rule: global node id
  std::vector<std::string> rule_names;
  std::vector<std::bitset<256>> first;        // per rule: bytes an instance can start with
  int32_t root_rule = 0;
  std::vector<std::vector<int32_t>> node_path;  // witness path from the rule start

  // flattened form (device tables)
  std::vector<NodeHdr> hdr;        // [n_nodes]
  std::vector<uint8_t> cls;        // [256] byte -> class
  int32_t n_cls = 0;
  std::vector<uint16_t> rows;      // [n_rows * n_cls]
  std::vector<uint32_t> alts;      // pool: count, then count entries (tag << 16 | node)
  int32_t max_alts = 0;
};

// Throws Failure.
Automaton compile_grammar(const std::string& text, const std::string& root);

}  // namespace xgm
