// TEST INFRASTRUCTURE ONLY: part of the slow CPU oracle.
//
// A character class is a set of Unicode scalar values; at byte level it is
// the set of their shortest-form UTF-8 encodings (section 3: the automaton
// is byte-level so that tokens may stop inside a character).  The oracle gets
// that byte language the plain way: enumerate every scalar value in the
// class, encode it with the textbook encoder, insert the bytes into a trie,
// then share identical subtrees so the result stays small.
#pragma once
#include <array>
#include <bitset>
#include <cstdint>
#include <map>
#include <mutex>
#include <utility>
#include <vector>

namespace orc {

using ByteSet = std::bitset<256>;

// A DAG over bytes: node 0 is the unique leaf ("character complete").
struct ByteDag {
  struct Edge { ByteSet bytes; int child; };
  std::vector<std::vector<Edge>> nodes;  // nodes[0] is the leaf (no edges)
  int root = 0;                          // 0 means the class is empty... see empty
  bool empty = true;                     // no scalar value in the class
};

inline int encode_utf8(uint32_t cp, unsigned char out[4]) {
  if (cp < 0x80) { out[0] = (unsigned char)cp; return 1; }
  if (cp < 0x800) { out[0] = 0xC0 | (cp >> 6); out[1] = 0x80 | (cp & 0x3F); return 2; }
  if (cp < 0x10000) { out[0] = 0xE0 | (cp >> 12); out[1] = 0x80 | ((cp >> 6) & 0x3F); out[2] = 0x80 | (cp & 0x3F); return 3; }
  out[0] = 0xF0 | (cp >> 18); out[1] = 0x80 | ((cp >> 12) & 0x3F); out[2] = 0x80 | ((cp >> 6) & 0x3F); out[3] = 0x80 | (cp & 0x3F);
  return 4;
}

inline ByteDag class_to_dag_uncached(const std::vector<std::pair<uint32_t, uint32_t>>& ranges, bool negated);

// The result depends only on the class, so it is computed once per process.
inline ByteDag class_to_dag(const std::vector<std::pair<uint32_t, uint32_t>>& ranges, bool negated) {
  static std::mutex mu;
  static std::map<std::pair<std::vector<std::pair<uint32_t, uint32_t>>, bool>, ByteDag> memo;
  std::lock_guard<std::mutex> lock(mu);
  auto key = std::make_pair(ranges, negated);
  auto it = memo.find(key);
  if (it == memo.end()) it = memo.emplace(key, class_to_dag_uncached(ranges, negated)).first;
  return it->second;
}

inline ByteDag class_to_dag_uncached(const std::vector<std::pair<uint32_t, uint32_t>>& ranges, bool negated) {
  // membership table over all code points
  std::vector<bool> in(0x110000, false);
  for (auto& r : ranges)
    for (uint32_t c = r.first; c <= r.second && c < 0x110000; ++c) in[c] = true;
  // trie
  struct TNode { std::map<int, int> kids; bool end = false; };
  std::vector<TNode> trie(1);
  bool any = false;
  for (uint32_t c = 0; c < 0x110000; ++c) {
    if (c >= 0xD800 && c <= 0xDFFF) continue;  // surrogates are not scalar values
    if (in[c] == negated) continue;
    any = true;
    unsigned char b[4];
    int n = encode_utf8(c, b);
    int cur = 0;
    for (int i = 0; i < n; ++i) {
      auto it = trie[cur].kids.find(b[i]);
      if (it == trie[cur].kids.end()) {
        trie.push_back(TNode());
        int id = (int)trie.size() - 1;
        trie[cur].kids[b[i]] = id;
        cur = id;
      } else cur = it->second;
    }
    trie[cur].end = true;
  }
  ByteDag dag;
  dag.nodes.push_back({});  // leaf
  dag.empty = !any;
  if (!any) return dag;
  // share identical subtrees, children first (UTF-8 is prefix-free, so an
  // "end" node never has children)
  std::map<std::vector<std::pair<int, int>>, int> canon;  // (byte, child id)* -> dag id
  std::vector<int> dag_id(trie.size(), -1);
  // post-order without recursion: trie nodes were created parents-first, so
  // walking indices downwards visits children before parents
  for (int t = (int)trie.size() - 1; t >= 0; --t) {
    if (trie[t].end) { dag_id[t] = 0; continue; }
    std::vector<std::pair<int, int>> sig;
    for (auto& kv : trie[t].kids) sig.push_back({kv.first, dag_id[kv.second]});
    auto it = canon.find(sig);
    if (it != canon.end()) { dag_id[t] = it->second; continue; }
    std::map<int, ByteSet> by_child;
    for (auto& s : sig) by_child[s.second].set(s.first);
    std::vector<ByteDag::Edge> edges;
    for (auto& kv : by_child) edges.push_back({kv.second, kv.first});
    dag.nodes.push_back(edges);
    int id = (int)dag.nodes.size() - 1;
    canon[sig] = id;
    dag_id[t] = id;
  }
  dag.root = dag_id[0];
  return dag;
}

}  // namespace orc
