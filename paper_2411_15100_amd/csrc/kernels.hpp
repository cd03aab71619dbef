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

// ---- id space is cut into segments of 8192 tokens = 256 mask words; one
// workgroup of the fill kernel owns one (row, segment)
constexpr int kSegWords = 256;
constexpr int kSegTokens = kSegWords * 32;

// walk results
enum : int { kReject = 0, kUncertain = 1, kAccept = 2, kOverflow = 3, kUncertainPlain = 4 };

// Automaton tables of one grammar in device memory (see NodeHdr in
// automaton.hpp): one contiguous image whose leading part a workgroup keeps in
// LDS (a single copy of 16-byte words).  Sections, in the order of how much a
// walk step depends on them:
//   [0, 256)                cls      byte -> class
//   [off_shapes, ..)        shapes   [n_shapes][n_cls] uint8
//   [off_targets, ..)       targets  uint16
//   [off_follow, ..)        follow   [n_rules][8] uint32: bytes that can come right after an instance of the rule
//   [off_alts, ..)          alts     uint32 pool: count, then count entries (tag << 16 | node)
//   [off_hdr, ..)           headers  [n_nodes] uint2: x = lo | hi<<8 | target<<16, y = flags | rule<<16
//   [off_first, ..)         first    [n_nodes][8] uint32: bytes a node can consume inside its frame (never staged)
// Every offset is a multiple of 4, off_hdr of 16; the image is padded to a multiple of 16 bytes.
struct DevTables {
  const uint4* image;
  uint32_t off_shapes, off_targets, off_follow, off_alts, off_hdr, off_first;
  int32_t n_cls, n_nodes, n_rules;
  // set per kernel by staged_for(): bytes [0, lds_end) of the image are in LDS
  // (whole sections, then the first n_near headers); stage_bytes = lds_end
  // rounded up to 16 is what gets copied; 0 = nothing is staged
  uint32_t lds_end, stage_bytes, n_near;
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
constexpr int32_t kClassifyLdsBudget = 76 * 1024;
constexpr int32_t kContextLdsBudget = 68 * 1024;  // the list kernels keep 8 KB of counters beside the tables
constexpr int32_t kFillLdsBudget = 12 * 1024;
// The staging split for a kernel that has `budget` bytes of LDS for the tables:
// as many whole sections as fit, then as many headers as fit.
inline DevTables staged_for(DevTables t, int32_t budget) {
  const uint32_t ends[5] = {256u, t.off_targets, t.off_follow, t.off_alts, t.off_hdr};  // section ends in image order
  t.lds_end = t.stage_bytes = t.n_near = 0;
  for (uint32_t e : ends)
    if (e <= (uint32_t)budget) t.lds_end = e;
  if (t.lds_end == t.off_hdr) {
    const uint32_t k = ((uint32_t)budget - t.off_hdr) / 8;
    t.n_near = k < (uint32_t)t.n_nodes ? k : (uint32_t)t.n_nodes;
    t.lds_end = t.off_hdr + t.n_near * 8;
  }
  t.stage_bytes = (t.lds_end + 15u) & ~15u;
  return t;
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
  int32_t n_seg;    // ceil(W / kSegWords)
};

// One mask cache on the device (section 3.1, with the context expansion of
// section 3.2 taken per call site).  What a stack contributes to a mask is kept
// in token lists, each addressed by a key and cut by segment:
//   level 0, key = node n:         the tokens accepted at n whatever lies below (only for nodes with few of
//                                  them; the others keep a bitset row in `acc`);
//   level 1, key = (n, i):         the context-dependent tokens of n that are accepted when the frame below
//                                  is the i-th context node of n's rule (the nodes that can sit right below
//                                  a frame of that rule: Automaton::contexts);
//   level 2, key = (n, i, j):      those that leave that frame as well and are accepted when the next frame
//                                  down is the j-th context node of the rule of context i;
//   ... and so on, kCtxLevels frames deep.
// Tokens that leave one more frame than that, or whose walk at build time hit a limit, are listed as "walk"
// entries: the fill kernel decides them against the live stack.
// A key of level l >= 1 has a number among its level's keys; the keys of all levels share one numbering:
// node n | n_nodes + (level-1 number) | n_nodes + n_k[0] + (level-2 number) | ...  The children of a key are
// numbered side by side: level-1 number of (n, i) = k_base[0][n] + i, level-(l+1) number of (key q of level
// l, context j) = k_base[l][q] + j.  The entries of (key, segment s) are
// entries[key_off[key * n_seg + s] .. key_off[key * n_seg + s + 1]), accepted ones first, walk entries last.
constexpr int kCtxLevels = 3;
struct DevCache {
  DevTables tab;             // staging split for the fill kernel
  const uint32_t* acc;       // [n_acc_rows][W] accepted tokens, id space: the distinct bitset rows
  const uint16_t* acc_row;   // [n_nodes] which row of `acc` is the node's, or kNoAccRow (listed under its level-0 key)
  const uint32_t* key_off;   // [n_keys * n_seg + 1]
  const uint32_t* entries;   // see kEntry*
  const uint32_t* k_base[kCtxLevels];  // [n_nodes], [n_k[0]], [n_k[1]], ...; null from the first level that is not kept
  uint32_t n_k[kCtxLevels];  // keys of level 1, 2, ...
  const uint32_t* ctx_off;   // [n_rules+1] ranges of ctx_node: the contexts of every rule
  const uint16_t* ctx_node;  // context nodes, sorted within a rule
  // the same relation by node: node_ctx[node_ctx_off[v] .. node_ctx_off[v + 1]) = (rule << 16 | index of v among the
  // contexts of that rule) for every rule that v is a context of
  const uint32_t* node_ctx_off;  // [n_nodes + 1]
  const uint32_t* node_ctx;
  int32_t n_nodes;
};
constexpr uint32_t kNoAccRow = 0xFFFFu;
// A list entry: bits 0..19 token id, bits 20..27 position, bits 28..31 kind:
//   kEntryAccepted       the token is allowed;
//   kEntryWalkTop        walk the whole token from the top of the stack;
//   kEntryWalkTop + d    walk it from byte `position` on, starting at the node d frames below the top (the
//                        only position at which it leaves the frames above), d = 1 .. kCtxLevels.
constexpr uint32_t kEntryIdBits = 20, kEntryIdMask = (1u << kEntryIdBits) - 1u, kEntryPosShift = 20, kEntryKindShift = 28;
constexpr uint32_t kEntryAccepted = 0, kEntryWalkTop = 1;
constexpr uint32_t kNoKey = 0xFFFFFFFFu;

// per-step description of the live stacks: [RowDesc x B][stack headers][frames]
struct RowDesc {
  DevTables tab;             // the request's grammar (copied in, so that a workgroup needs no further lookup)
  const uint32_t* acc;       // DevCache::acc
  const uint32_t* entries;   // DevCache::entries
  uint32_t stack_begin;      // first stack header of this request
  uint32_t n_stacks;         // 0: terminated row (only stop bits)
  uint32_t flags;            // bit 0: the text so far is a complete sentence
  uint32_t frame_begin;      // the request's frames: [frame_begin, frame_begin + n_frames) of the frame array,
  uint32_t n_frames;         // stack after stack
  uint32_t epoch;            // device-resident states: how often the row's state has changed (names the state in a record)
};
// A stack header is kStackHdrWords + (n_seg + 1) * kStackLists uint32 words (a multiple of 16 bytes):
//   [kStackHdrTop] top node | its row of DevCache::acc (or kNoAccRow) << 16, [kStackHdrDepth] number of frames,
//   [kStackHdrFrames] offset of its frames (bottom first) in the uint16 frame array, [3] unused,
//   [stack_hdr_off(s, l)] where the entries of segment s of the stack's level-l list start (s = n_seg: where
//   the last segment's end); a stack without that list (too shallow, or a level that is not kept) has all of
//   them equal.  The lists' offsets of one segment lie side by side, so that the workgroup of (row, segment)
//   finds the begin and the end of all its lists of a stack in 32 consecutive bytes.
constexpr uint32_t kStackHdrTop = 0, kStackHdrDepth = 1, kStackHdrFrames = 2, kStackHdrWords = 4;
constexpr uint32_t kStackLists = 1 + kCtxLevels;
constexpr uint32_t stack_hdr_stride(int32_t n_seg) { return kStackHdrWords + kStackLists * ((uint32_t)n_seg + 1u); }
constexpr uint32_t stack_hdr_off(uint32_t seg, uint32_t l) { return kStackHdrWords + seg * kStackLists + l; }

// ---- matcher states that live on the device (section 3.3 on the GPU: the
// sampled tokens move the stacks on without a round trip to the host).
// A batch holds, for each of its B rows, a ring of H states.  A state is what
// the fill kernel reads: up to kBatchMaxStacks stack headers and their frames,
// stack after stack.  The row's current state is named by its RowDesc;
// accepting a token writes the next slot of the ring and points the RowDesc
// there, so that going back k tokens is a matter of pointing it k slots back.
constexpr uint32_t kBatchMaxStacks = 16;      // parallel stacks per row
constexpr uint32_t kBatchMaxDepth = 128;      // frames per stack
constexpr uint32_t kBatchMaxCandidates = 32;  // stacks a token may end in before duplicates are removed
constexpr uint32_t kBatchRowFrames = kBatchMaxStacks * kBatchMaxDepth;
constexpr uint32_t kBatchMaxRows = 1024;
struct SlotMeta {
  uint32_t n_stacks, n_frames;
  uint32_t flags;  // bit 0: the text so far is a complete sentence; bit 1: the stop token has been accepted
  uint32_t pad;
};
struct OverflowLog;
struct DevBatch {
  int32_t B, H, n_seg, pad;
  const DevCache* cache;  // [B] each row's mask cache (tables staged as for the fill kernel)
  RowDesc* rows;          // [B] current states
  SlotMeta* meta;         // [B][H]
  uint32_t* hdrs;         // [B][H][kBatchMaxStacks] stack headers
  uint16_t* frames;       // [B][H][kBatchRowFrames]
  int32_t* head;          // [B] slot of the current state
  int32_t* older;         // [B] how many older states are still in the ring
  int32_t* status;        // [B] result of the last accept / rollback per row (XGM_OK or an error code)
  OverflowLog* log;       // the batch's own record of walks over the limits
};

// pairs whose walk exceeded the limits
struct OverflowLog {
  static constexpr uint32_t kCap = 1 << 14;
  uint32_t count;          // total ever recorded (entries wrap around)
  uint32_t pad;
  uint32_t entry[kCap][4]; // (sequence number of the call, row or node, token id or rank, epoch of the row's state)
};

// ---- staging memory that needs no allocation: a fixed array in every device's memory
constexpr size_t kStaticScratchBytes = (size_t)1 << 20;
// its address on the current device (looked up on the first call per device; callers serialise)
hipError_t static_scratch(void** out);

// ---- launchers (all asynchronous on `stream`)
// (a) classify tokens [all ranks] x nodes [node0, node0+n) into rank-space bitsets
// plain_rank (may be null): tokens that are context-dependent by section 3.1 alone
// but rejected by the one-byte context refinement; plain_count[node0 + k] += their number
// first_byte: what launch_first_byte() wrote for this grammar; node0 must be a multiple of 32
void launch_classify(const DevTables& tab, const DevVocab& voc, int32_t node0, int32_t n, const uint4* first_byte,
                     uint32_t* acc_rank, uint32_t* unc_rank, uint32_t* plain_rank, uint32_t* plain_count,
                     OverflowLog* log, uint32_t seq, hipStream_t stream);
// What a token's first byte settles at every node: first_byte[c * first_byte_words(N) + w] holds, for byte c and
// nodes 32 w .. 32 w + 31, the bitsets {walk needed, leaves the frame at once in front of a byte that may follow
// the rule, leaves it in front of one that may not, 0}.
inline uint32_t first_byte_words(int32_t n_nodes) { return (uint32_t)((n_nodes + 31) / 32); }
void launch_first_byte(const DevTables& tab, uint4* first_byte, hipStream_t stream);
// Rank space -> id space for n node rows (two bitsets per node), and - unless the pointers are null - per node the
// set bits of the first row per segment (seg_counts[n][n_seg]), a 64-bit digest of the first row (equal rows have
// equal digests; it only proposes which rows might be equal) and the set bits of the second row (b_counts[n]).
void launch_permute(const DevVocab& voc, int32_t n, const uint32_t* a_rank, const uint32_t* b_rank, uint32_t* a_id,
                    uint32_t* b_id, uint32_t* seg_counts, unsigned long long* digest, uint32_t* b_counts, hipStream_t stream);
// whether row k equals row rep[k], word for word (k = 0 .. n-1); rows[unique[u]] -> out[u]
void launch_rows_equal(const uint32_t* rows, int32_t n, int32_t W, const int32_t* rep, uint32_t* equal, hipStream_t stream);
void launch_gather_rows(const uint32_t* rows, int32_t W, const int32_t* unique, int32_t n_unique, uint32_t* out,
                        hipStream_t stream);
// The set bits of n bitset rows of row_words words as lists, appended through cursors: bit v of row r, in
// segment s = v / kSegTokens, goes to out[cursor[cursor_of[r] * per_row + (per_row > 1 ? s : 0)]++] as
// map[v] (map not null: rank-space rows with map = id_of_rank list token ids, neighbours in the list being
// neighbours in byte-sorted order) or as v; rows with cursor_of[r] == kNoKey are skipped.  per_row = the
// segments of a row: one list per (row, segment); 1: one per row.  out_row (may be null) receives the row
// number beside every entry.
void launch_rows_to_lists(const uint32_t* rows, int32_t row_words, const int32_t* map, int32_t n, const uint32_t* cursor_of,
                          int32_t per_row, uint32_t* cursor, uint32_t* out, uint16_t* out_row, hipStream_t stream);
// The level-1 and level-2 lists of a cache (see DevCache) from the base lists: the context-dependent
// (node, token) pairs, base_node[e] / base_ids[e] for e < total, the pairs of one node side by side.
// launch_exit_positions: exits[e] = the positions at which the token leaves the node's frame, as a bit set
// (bit 31: some position beyond 30, or the walk hit a limit).
// launch_context_lists, write = false: counts[key * n_seg + seg] += the entries each list will hold;
// write = true: the entries are written, accepted ones upwards from front[slot], walk entries downwards from
// back[slot] (both arrays are advanced).  Levels whose k_base is null are not kept: tokens that would need
// them become walk entries of the level above.
// tiles: the work of the level-1 kernel, one workgroup each: x = first pair, y = pairs (at most
// context_tile_pairs(), all of one node) | contexts << 16 (at most context_tile_contexts()), z = first
// context, w = the node.  res[l] / res_cap / res_count[l]: records of the (pair, key of level l + 1) that
// leave one more frame, made by the kernel of level l + 1 for the kernel of level l + 2 - one record for
// every chunk of context_tile_contexts() contexts of the rule whose frame comes next: x = pair, y = number of
// the key among its level's keys, z = the positions at which the frame is left, w = that rule | the way so
// far is unique << 16 | chunk << 17; a record that does not fit is dropped and counted all the same (the
// caller then runs the pass again with more room).
struct ContextListArgs {
  const uint16_t* base_node;
  const uint32_t* base_ids;
  uint32_t total;
  uint32_t* exits;             // [total]
  const uint4* tiles;
  uint32_t n_tiles;
  uint4* res[kCtxLevels];      // (the last one is not used)
  uint32_t res_cap;
  uint32_t* res_count;         // [kCtxLevels]
  const uint32_t* k_base[kCtxLevels];
  uint32_t key0[kCtxLevels];   // the first key of level 1, 2, ... in the shared numbering
  const uint32_t* ctx_off;
  const uint16_t* ctx_node;
  uint32_t* counts;            // [n_keys * n_seg]   write = false
  uint32_t* front;             // [n_keys * n_seg]   write = true
  uint32_t* back;              // [n_keys * n_seg]   write = true
  uint32_t* entries;
  // What the level-1 kernel found for every (pair, context) when it counted, kept so that the writing pass
  // need not walk again (null: it walks again).  node_info[n] = {first outcome of node n, its pairs L, its
  // first pair, 0}; the outcome of pair e and context i of node n is outcomes[info.x + i * L + (e - info.z)]:
  // 0 = no entry, else (kind + 1) | pos << 8.
  const uint4* node_info;
  uint16_t* outcomes;
  // The same for the deeper levels: deep_outcomes[l][r] holds the outcomes (8 x 16 bits, coded as above) of
  // record r of res[l - 1], that is of level l + 1, for the contexts of the record's chunk; null: the writing
  // pass of that level walks again.  Used together with `outcomes` only.
  uint4* deep_outcomes[kCtxLevels];
};
void launch_exit_positions(const DevTables& tab, const DevVocab& voc, const ContextListArgs& args, hipStream_t stream);
void launch_context_lists(const DevTables& tab, const DevVocab& voc, const ContextListArgs& args, bool write, hipStream_t stream);
uint32_t context_tile_pairs();
uint32_t context_tile_contexts();
// set / clear single bits of rank-space rows: items = (node - node0, rank, class)
void launch_patch_classes(const DevVocab& voc, const uint32_t* items, int32_t n_items,
                          uint32_t* acc_rank, uint32_t* unc_rank, uint32_t* plain_rank, hipStream_t stream);
// A stack as the host hands it over (kStackKeysWords words): the header's four scalar words, then the keys of
// the stack's kStackLists lists (kNoKey: none), then the device address of the cache's key_off (two words).
// launch_upload_stacks copies `plain_bytes` bytes (a multiple of 16: the row descriptors) and `frames_bytes`
// bytes of frames as they are and writes every stack's full header (stack_hdr_stride(n_seg) words: the
// offsets of the lists' segments looked up in key_off on the device) at dst_hdrs; src may be pinned host
// memory or device memory.
constexpr uint32_t kStackKeysWords = 12;
void launch_upload_stacks(const void* src, void* dst, size_t plain_bytes, const void* src_stacks, uint32_t n_stacks,
                          int32_t n_seg, void* dst_hdrs, const void* src_frames, void* dst_frames, size_t frames_bytes,
                          hipStream_t stream);
// (b) batched mask fill: one workgroup per (segment, row)
// step_counter: null on the hot path; otherwise the counting instantiation is launched.
// logits != null: the fused instantiation also applies each row's mask to its logits row
// (elem_size 2 or 4, rows 16-byte aligned; a walk over the limits leaves its token allowed).
void launch_fill(const RowDesc* rows, const uint32_t* stack_hdrs, const uint16_t* frames, int32_t B,
                 const DevVocab& voc, uint32_t* out, OverflowLog* log, uint32_t seq,
                 unsigned long long* step_counter, hipStream_t stream, void* logits = nullptr,
                 int elem_size = 0, uint32_t neg_inf = 0, int32_t V_logits = 0, int64_t row_stride = 0);
// device-resident states: move every row on by its token (ids < 0 leave a row alone)
void launch_batch_accept(const DevBatch& bt, const DevVocab& voc, const int32_t* d_tokens, hipStream_t stream);
// go back d_steps[b] tokens in every row (<= 0 leaves a row alone)
void launch_batch_rollback(const DevBatch& bt, const int32_t* d_steps, hipStream_t stream);
// row b continues from the current state of row d_src_rows[b] (< 0 or b itself: stays)
void launch_batch_fork(const DevBatch& bt, const int32_t* d_src_rows, hipStream_t stream);
// measurement aid: n_blocks workgroups of 1024 lanes, each lane a chain of `hops` dependent reads in a 32 KB LDS table
void launch_lds_lookups(int32_t n_blocks, uint32_t hops, uint32_t* sink, hipStream_t stream);
// (c) apply
void launch_apply(void* logits, int elem_size, uint32_t neg_inf, int32_t V_logits, int64_t row_stride,
                  const uint32_t* bitmask, int32_t V_mask, const int32_t* row_index, int32_t n_rows,
                  hipStream_t stream);

}  // namespace xgm
