// Device-side data layouts and the host-callable launchers of the three
// kernels (token walk / classify, batched mask fill, -inf apply).
#pragma once
#include <hip/hip_runtime_api.h>
#include <hip/hip_vector_types.h>

#include <cstdint>

namespace xgm {

// ---- limits of one GPU walk (exceeding any of them is reported, never guessed)
constexpr int kArenaFrames = 64;    // frames pushed inside one token and still needed
constexpr int kChoicePoints = 24;   // pending alternatives
constexpr int kMaxSteps = 4096;     // automaton steps per (position, token)
constexpr int kMaxTokenLen = 255;   // bytes

// ---- id space is cut into chunks of 4096 tokens = 128 mask words; one
// workgroup of the fill kernel owns one (row, chunk)
constexpr int kChunkWords = 128;
constexpr int kChunkTokens = kChunkWords * 32;

// walk results
enum : int { kReject = 0, kUncertain = 1, kAccept = 2, kOverflow = 3, kUncertainPlain = 4 };

// automaton tables of one grammar in device memory (see NodeHdr in automaton.hpp)
struct DevTables {
  const uint2* hdr;              // [n_nodes] x = lo | hi<<8 | target<<16, y = flags | rule<<16
  const uint8_t* cls;            // [256] byte -> class
  const uint8_t* shapes;         // [n_shapes * n_cls]
  const uint16_t* targets;       // [n_targets]
  const uint32_t* alts;          // [n_alts] pool: count, then count entries (tag << 16 | node)
  const uint32_t* follow_rules;  // [n_rules][8] bytes that can come right after an instance of the rule
  int32_t n_cls, n_nodes, n_shapes, n_targets, n_alts, n_rules;
  int32_t aux_bytes;             // LDS bytes for everything but the headers; 0 = too big, tables stay in global memory
};

// what the walk reads: the first n_near node headers and the small tables may
// sit in LDS, the remaining headers in global memory
struct TabView {
  const uint2* hdr_near;
  int32_t n_near;
  const uint2* hdr_far;
  const uint8_t* cls;
  const uint8_t* shapes;
  const uint16_t* targets;
  const uint32_t* alts;
  const uint32_t* follow_rules;
  int32_t n_cls;
};

// LDS budgets (bytes of dynamic shared memory) for the staged tables
constexpr int32_t kClassifyLdsBudget = 56 * 1024;
constexpr int32_t kFillLdsBudget = 40 * 1024;
// how many leading node headers fit beside the small tables (0: stage nothing)
inline int32_t near_headers(const DevTables& t, int32_t budget) {
  if (t.aux_bytes <= 0 || t.aux_bytes + 8 > budget) return 0;
  const int32_t k = (budget - t.aux_bytes) / 8;
  return k < t.n_nodes ? k : t.n_nodes;
}

// vocabulary on the device.  A token row is 16 bytes: bytes 0..14 are the
// token's first bytes, byte 15 its length (255 = read the length from the
// offsets).  Bytes past the 15th are read from the CSR arrays.
struct DevVocab {
  const uint4* tok_by_id;     // [V]
  const uint4* tok_by_rank;   // [V] same rows in byte-sorted order
  const uint32_t* off_by_id;  // [V+1] CSR offsets into bytes
  const uint8_t* bytes;       // token bytes, id order
  const uint8_t* first_by_id; // [V] first byte of each token (0 for empty tokens)
  const int32_t* rank_of_id;  // [V]
  const int32_t* id_of_rank;  // [V]
  const int32_t* stop_ids;    // [n_stop]
  int32_t n_stop;
  int32_t V;
  int32_t W;        // ceil(V/32)
  int32_t WR;       // words per row of a rank-space bitset (even)
  int32_t n_chunk;  // ceil(W / kChunkWords)
};

// one mask cache on the device
struct DevCache {
  DevTables tab;
  const uint32_t* acc;       // [n_nodes][W] accepted tokens, id space
  const uint32_t* unc_off;   // [n_nodes][n_chunk+1] offsets into unc_list
  const uint32_t* unc_list;  // context-dependent tokens, grouped by (node, chunk); see kEntry*
  int32_t n_near_fill;       // node headers the fill kernel keeps in LDS
  int32_t n_nodes;
};

// A list entry describes one context-dependent token of a node:
//   bits  0..11  token id - chunk * 4096
//   bits 12..15  the only position k (0..14) at which a walk from the node can leave the node's
//                frame (section 3.2: what remains of the token is then the parent's business), or
//                kEntryFullWalk if there are several such positions or the position is beyond 14
//   bits 16..23  the byte at that position (for kEntryFullWalk: the token's first byte)
//   bits 24..27  min(15, bytes left after that position): entries of a list are sorted by it
constexpr uint32_t kEntryFullWalk = 15;

// per-step upload of the live stacks: [RowDesc x B][stack headers][frames]
struct RowDesc {
  const DevCache* cache;  // null: terminated row (only stop bits)
  uint32_t stack_begin;   // first stack header of this request
  uint32_t n_stacks;
  uint32_t flags;         // bit 0: the text so far is a complete sentence
  uint32_t pad;
};
// A stack header is kStackHdrWords + n_chunk + 1 uint32 words:
//   [kStackHdrTop] top node, [kStackHdrDepth] number of frames,
//   [kStackHdrFrames] offset of its frames (bottom first) in the uint16 frame array,
//   [kStackHdrFirst .. +8) 256-bit set of the bytes that can be consumed from this stack,
//   [kStackHdrBelow .. +8) the same for the stack without its top frame,
//   [kStackHdrWords + c] offset of chunk c's context-dependent list of the top node
//   (c = 0 .. n_chunk; entry n_chunk is the end of the last list).
constexpr uint32_t kStackHdrTop = 0, kStackHdrDepth = 1, kStackHdrFrames = 2, kStackHdrFirst = 4, kStackHdrBelow = 12,
                   kStackHdrWords = 20;

// pairs whose walk exceeded the limits
struct OverflowLog {
  static constexpr uint32_t kCap = 1 << 16;
  uint32_t count;          // total ever recorded (entries wrap around)
  uint32_t pad;
  uint32_t entry[kCap][3]; // (sequence number, row or node, token id or rank)
};

// ---- launchers (all asynchronous on `stream`)
// (a) classify tokens [all ranks] x nodes [node0, node0+n) into rank-space bitsets
// plain_rank (may be null): tokens that are context-dependent by section 3.1 alone
// but rejected by the one-byte context refinement; plain_count[node0 + k] += their number
void launch_classify(const DevTables& tab, const DevVocab& voc, int32_t node0, int32_t n,
                     uint32_t* acc_rank, uint32_t* unc_rank, uint32_t* plain_rank, uint32_t* plain_count,
                     OverflowLog* log, uint32_t seq, hipStream_t stream);
// rank space -> id space for n node rows (two bitsets per node)
void launch_permute(const DevVocab& voc, int32_t n, const uint32_t* a_rank, const uint32_t* b_rank,
                    uint32_t* a_id, uint32_t* b_id, hipStream_t stream);
// per (node, chunk) number of context-dependent tokens
void launch_count_uncertain(const DevVocab& voc, int32_t n, const uint32_t* unc_id, uint32_t* counts,
                            hipStream_t stream);
// write the context-dependent lists; off = [n][n_chunk+1] offsets relative to list
void launch_list_uncertain(const DevVocab& voc, int32_t n, const uint32_t* unc_id, const uint32_t* off,
                           uint32_t* list, hipStream_t stream);
// find each entry's exit position (a walk per entry) and sort every (node, chunk) list by remaining length
void launch_annotate_lists(const DevTables& tab, const DevVocab& voc, int32_t n, const uint32_t* off,
                           uint32_t* list, hipStream_t stream);
// set / clear single bits of rank-space rows: items = (node - node0, rank, class)
void launch_patch_classes(const DevVocab& voc, const uint32_t* items, int32_t n_items,
                          uint32_t* acc_rank, uint32_t* unc_rank, uint32_t* plain_rank, hipStream_t stream);
// (b) batched mask fill
// step_counter: null on the hot path; otherwise the counting instantiation is launched
void launch_fill(const RowDesc* rows, const uint32_t* stack_hdrs, const uint16_t* frames, int32_t B,
                 const DevVocab& voc, uint32_t* out, OverflowLog* log, uint32_t seq,
                 unsigned long long* step_counter, hipStream_t stream);
// (c) apply; returns false if the buffer layout needs the element-wise kernel
void launch_apply(void* logits, int elem_size, uint32_t neg_inf, int32_t V_logits, int64_t row_stride,
                  const uint32_t* bitmask, int32_t V_mask, const int32_t* row_index, int32_t n_rows,
                  hipStream_t stream);

}  // namespace xgm
