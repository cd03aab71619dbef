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

// Device header of one node (8 bytes).
//  * plain node (at most one byte edge, no references): [lo, hi] -> target,
//    lo > hi if it has no edge at all;
//  * branching node (kFlagBranching): lo | hi << 8 is its shape id and
//    `target` the start of its outcomes in `targets`; for byte c the outcome
//    is targets[target + shapes[shape * n_cls + cls[c]]] unless that shape
//    entry is kDeadShape.
struct NodeHdr {
  uint8_t lo, hi;
  uint16_t target;
  uint32_t flags;  // kFlagFinal | kFlagBranching | kFlagDeadEnd | rule index << 16
};
static_assert(sizeof(NodeHdr) == 8, "NodeHdr must be 8 bytes");

constexpr uint32_t kFlagFinal = 1;      // the rule may end at this node
constexpr uint32_t kFlagBranching = 2;
constexpr uint32_t kFlagDeadEnd = 4;    // accepting and without outgoing edges: all it can do is return
constexpr uint8_t kDeadShape = 0xFF;    // shape entry: nothing to do for this byte class
constexpr uint16_t kAltFlag = 0x8000;   // outcome: index into the alternatives pool (else: move to that node)
constexpr uint32_t kMoveTag = 0xFFFF;   // alternative (tag << 16 | node): consume the byte, go to node
constexpr uint32_t kTailTag = 0xFFFE;   // alternative: enter the callee at `node` without pushing a frame
                                        // (any other tag is the return node to push)

struct Automaton {
  // structured form (host engine)
  int32_t n_nodes = 0;
  std::vector<int32_t> node_rule;
  std::vector<uint8_t> node_final;
  std::vector<uint8_t> node_dead_end;         // accepting and without outgoing edges: all it can do is return
  std::vector<std::vector<ByteEdge>> bedges;  // sorted, disjoint
  std::vector<std::vector<RefEdge>> redges;
  std::vector<int32_t> rule_start;            // per rule: global node id
  std::vector<std::string> rule_names;
  std::vector<std::bitset<256>> first;        // per rule: bytes an instance can start with
  std::vector<std::bitset<256>> node_first;   // per node: bytes that can be consumed at the node inside its frame
  std::vector<uint32_t> node_first_words;     // [n_nodes][8] the same sets as machine words
  std::vector<std::bitset<256>> follow;       // per rule: bytes that can come right after an instance, in any context
  // per rule: the nodes that can sit right below a frame of that rule (return nodes of the references to it;
  // a reference in tail position hands on the contexts of the referring rule), sorted
  std::vector<std::vector<int32_t>> contexts;
  int32_t root_rule = 0;
  std::vector<std::vector<int32_t>> node_path;  // witness path from the rule start

  // flattened form (device tables)
  std::vector<NodeHdr> hdr;        // [n_nodes]
  std::vector<uint8_t> cls;        // [256] byte -> class
  int32_t n_cls = 0;
  std::vector<uint8_t> shapes;     // [n_shapes * n_cls]
  int32_t n_shapes = 0;
  std::vector<uint16_t> targets;   // outcomes of the branching nodes, node after node
  std::vector<uint32_t> follow_words;  // [n_rules][8]: `follow` as 256-bit sets
  std::vector<uint32_t> alts;      // pool: count, then count entries (tag << 16 | node)
  int32_t max_alts = 0;
};

// Throws Failure.
Automaton compile_grammar(const std::string& text, const std::string& root);

}  // namespace xgm
