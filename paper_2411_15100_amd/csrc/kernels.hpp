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
constexpr int32_t kFillLdsBudget = 40 * 1024;
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
  int32_t n_chunk;  // ceil(W / kChunkWords)
};

// one mask cache on the device
struct DevCache {
  DevTables tab;             // staging split for the fill kernel
  const uint32_t* acc;       // [n_acc_rows][W] accepted tokens, id space: the distinct rows of the nodes' bitsets
  const uint16_t* acc_row;   // [n_nodes] which row of `acc` is the node's
  const uint32_t* unc_off;   // [n_nodes][n_chunk+1] offsets into unc_list
  const uint32_t* unc_list;  // context-dependent tokens, grouped by (node, chunk); see kEntry*
  const uint32_t* unc_ctx;   // parallel to unc_list: the entry's class in each context of its node's rule; see kCtx*
  const uint32_t* ctx_off;   // [n_rules+1] ranges of ctx_node: the contexts of every rule that has at most kCtxMax
  const uint16_t* ctx_node;  // context nodes, sorted within a rule
  int32_t n_nodes;
};

// A list entry describes one context-dependent token of a node.  If there is
// exactly one position k at which a walk from the node can leave the node's
// frame, what remains of the token from k on (its suffix) is the business of
// the frames below (section 3.2), and the entry says so:
//   bits  0..11  token id - chunk * 4096
//   bits 12..15  kind: 0..12 = k, the suffix has three or more bytes;
//                kEntrySuffix2 / kEntrySuffix1 = the suffix has two bytes / one byte (k = length - that);
//                kEntryFullWalk = several such positions (walk from the node), or k > 12 with a longer suffix
//   bits 16..23  first byte of the suffix (kEntryFullWalk: of the token)
//   bits 24..31  second byte of the suffix (0 if there is none); kEntryFullWalk: k if there is a single
//                exit position after all (13..30), else 0
// Entries of a (node, chunk) list are sorted by the length of what remains to be walked.
constexpr uint32_t kEntrySuffix2 = 13, kEntrySuffix1 = 14, kEntryFullWalk = 15;
// Beside every entry sits a word of per-context classes (section 3.2 taken per
// call site): a frame of rule R can only sit on one of the few nodes that
// follow a reference to R (Automaton::contexts).  For a rule with at most
// kCtxMax of them, bits 2i..2i+1 of the word say what the entry's suffix does
// when it is walked from context node i with nothing known below it:
// kCtxReject, kCtxWalk (it leaves that frame too, or the walk hit a limit:
// decide at run time) or kCtxAccept.  Rules with more contexts, and entries
// of kind kEntryFullWalk, have kCtxWalk everywhere.
constexpr uint32_t kCtxMax = 16, kCtxReject = 0, kCtxWalk = 1, kCtxAccept = 2;
constexpr uint32_t kCtxNone = 0xFFFFFFFFu;  // stack header: the frame below is not a listed context

// per-step upload of the live stacks: [RowDesc x B][stack headers][frames][FillBlock x n_blocks]
struct RowDesc {
  DevTables tab;             // the request's grammar (copied in, so that a workgroup needs no further lookup)
  const uint32_t* acc;       // DevCache::acc
  const uint32_t* unc_list;  // DevCache::unc_list
  const uint32_t* unc_ctx;   // DevCache::unc_ctx
  uint32_t stack_begin;      // first stack header of this request
  uint32_t n_stacks;         // 0: terminated row (only stop bits)
  uint32_t flags;            // bit 0: the text so far is a complete sentence
  uint32_t frame_begin;      // the request's frames: [frame_begin, frame_begin + n_frames) of the frame array,
  uint32_t n_frames;         // stack after stack
  uint32_t pair_mask;        // device-resident states only: bit s = the two-byte table of stack s has been computed
                             // ahead of the fill (DevBatch::pair); bit 31 = the row has been examined for that
};
// A stack header is kStackHdrWords + n_chunk + 1 uint32 words:
//   [kStackHdrTop] top node | its row of DevCache::acc << 16, [kStackHdrDepth] number of frames,
//   [kStackHdrFrames] offset of its frames (bottom first) in the uint16 frame array,
//   [kStackHdrCtx] index of the node below the top frame among the contexts of the top node's rule, or kCtxNone,
//   [kStackHdrFirst .. +8) 256-bit set of the bytes that can be consumed from this stack,
//   [kStackHdrBelow .. +8) the same for the stack without its top frame,
//   [kStackHdrWords + c] offset of chunk c's context-dependent list of the top node
//   (c = 0 .. n_chunk; entry n_chunk is the end of the last list).
constexpr uint32_t kStackHdrTop = 0, kStackHdrDepth = 1, kStackHdrFrames = 2, kStackHdrCtx = 3, kStackHdrFirst = 4, kStackHdrBelow = 12,
                   kStackHdrWords = 20;

// One workgroup of the fill kernel: request `row`, chunks [c0, c1) of its
// token ids.  The host cuts every request into such ranges of about equal
// numbers of context-dependent list entries and orders them heaviest first,
// so that a request in a state with many such tokens is spread over many
// compute units instead of serialising on a few.
struct FillBlock {
  uint32_t row;
  uint32_t c0c1;  // c0 | kFillBlockNoEntries | c1 << 16
};
// set by the planner when none of the request's stacks lists a token in chunks [c0, c1): the workgroup then
// only ORs the accepted words and never touches the automaton tables
constexpr uint32_t kFillBlockNoEntries = 0x8000u;
constexpr int32_t kFillMaxChunks = 24;  // chunks one workgroup may own (its mask words live in LDS)
// A workgroup builds the two-byte table of a stack only if its lists for that stack have at least this many
// entries: building it costs about as much as one queue round of walks.
constexpr uint32_t kFillPairMinEntries = 2048;

constexpr uint32_t kNoRow = 0xFFFFFFFFu;  // FillBlock::row of a workgroup that has nothing to do
constexpr int32_t kFillGridMultiple = 8;  // a plan is padded with kNoRow entries to a multiple of the number of XCDs

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
constexpr uint32_t kPairWords = 256 * 8;    // 256 x 256 bits: which byte can follow which
struct SlotMeta {
  uint32_t n_stacks, n_frames;
  uint32_t flags;  // bit 0: the text so far is a complete sentence; bit 1: the stop token has been accepted
  uint32_t pad;
};
struct DevBatch {
  int32_t B, H, n_chunk, budget;
  const DevCache* cache;  // [B] each row's mask cache (tables staged as for the fill kernel)
  RowDesc* rows;          // [B] current states
  SlotMeta* meta;         // [B][H]
  uint32_t* hdrs;         // [B][H][kBatchMaxStacks] stack headers
  uint16_t* frames;       // [B][H][kBatchRowFrames]
  int32_t* head;          // [B] slot of the current state
  int32_t* older;         // [B] how many older states are still in the ring
  int32_t* status;        // [B] result of the last accept / rollback per row (XGM_OK or an error code)
  FillBlock* plan;        // [plan_cap] workgroups of the next fill, padded with kNoRow
  uint32_t plan_cap;
  uint32_t* pair;         // [B][kBatchMaxStacks][kPairWords] two-byte tables of the current states' stacks
};
// workgroups a plan can have at most (see plan.hpp)
inline uint32_t batch_plan_cap(int32_t B, int32_t n_chunk, int32_t budget) {
  const int32_t min_blocks = (n_chunk + kFillMaxChunks - 1) / kFillMaxChunks;
  const int32_t n = (budget > B * min_blocks ? budget : B * min_blocks) + B * min_blocks;
  return (uint32_t)((n + kFillGridMultiple - 1) / kFillGridMultiple * kFillGridMultiple);
}

// pairs whose walk exceeded the limits
struct OverflowLog {
  static constexpr uint32_t kCap = 1 << 16;
  uint32_t count;          // total ever recorded (entries wrap around)
  uint32_t pad;
  uint32_t entry[kCap][3]; // (sequence number, row or node, token id or rank)
};

// ---- staging memory that needs no allocation: a fixed array in every device's memory
constexpr size_t kStaticScratchBytes = (size_t)1 << 20;
// its address on the current device (looked up on the first call per device; callers serialise)
hipError_t static_scratch(void** out);

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
// Identical rows of a [n][W] array of bitsets: a 64-bit digest of every row; whether row k equals row
// rep[k], word for word; rows[unique[u]] -> out[u].
void launch_hash_rows(const uint32_t* rows, int32_t n, int32_t W, unsigned long long* digest, hipStream_t stream);
void launch_rows_equal(const uint32_t* rows, int32_t n, int32_t W, const int32_t* rep, uint32_t* equal, hipStream_t stream);
void launch_gather_rows(const uint32_t* rows, int32_t W, const int32_t* unique, int32_t n_unique, uint32_t* out,
                        hipStream_t stream);
void launch_count_uncertain(const DevVocab& voc, int32_t n, const uint32_t* unc_id, uint32_t* counts,
                            hipStream_t stream);
// write the context-dependent lists; off = [n][n_chunk+1] offsets relative to list
void launch_list_uncertain(const DevVocab& voc, int32_t n, const uint32_t* unc_id, const uint32_t* off,
                           uint32_t* list, hipStream_t stream);
// find each entry's exit position (a walk per entry), sort every (node, chunk) list by remaining length, then
// classify every entry's suffix in the contexts of its rule (total = number of entries of all lists)
// ctx_off [n_rules+1], ctx_node: the contexts of every rule that has at most kCtxMax (others: empty range)
void launch_annotate_lists(const DevTables& tab, const DevVocab& voc, int32_t n, const uint32_t* off, uint32_t total,
                           uint32_t* list, uint32_t* list_ctx, const uint32_t* ctx_off, const uint16_t* ctx_node,
                           hipStream_t stream);
// set / clear single bits of rank-space rows: items = (node - node0, rank, class)
void launch_patch_classes(const DevVocab& voc, const uint32_t* items, int32_t n_items,
                          uint32_t* acc_rank, uint32_t* unc_rank, uint32_t* plain_rank, hipStream_t stream);
// copy `bytes` (rounded up to 16; both buffers must hold that) from device-visible pinned host memory
void launch_upload(const void* pinned_src, void* dst, size_t bytes, hipStream_t stream);
// (b) batched mask fill
// n_blocks: entries of `plan`, a multiple of kFillGridMultiple (padded with kNoRow entries).
// step_counter: null on the hot path; otherwise the counting instantiation is launched.
// logits != null: the fused instantiation also applies each row's mask to its logits row
// (elem_size 2 or 4, rows 16-byte aligned; a walk over the limits leaves its token allowed).
void launch_fill(const RowDesc* rows, const uint32_t* stack_hdrs, const uint16_t* frames,
                 const FillBlock* plan, int32_t n_blocks, const DevVocab& voc, uint32_t* out, OverflowLog* log,
                 uint32_t seq, unsigned long long* step_counter, hipStream_t stream, void* logits = nullptr,
                 int elem_size = 0, uint32_t neg_inf = 0, int32_t V_logits = 0, int64_t row_stride = 0,
                 uint32_t pair_min_entries = kFillPairMinEntries, const uint32_t* pair_tables = nullptr);
// device-resident states: move every row on by its token (ids < 0 leave a row alone), then plan the next fill
// (the plan step also computes, ahead of the fill, the two-byte tables of stacks whose lists have at least
// pair_min_entries entries)
void launch_batch_accept(const DevBatch& bt, const DevVocab& voc, const int32_t* d_tokens, uint32_t pair_min_entries,
                         hipStream_t stream);
// go back d_steps[b] tokens in every row (<= 0 leaves a row alone), then plan
void launch_batch_rollback(const DevBatch& bt, const DevVocab& voc, const int32_t* d_steps, uint32_t pair_min_entries,
                           hipStream_t stream);
// row b continues from the current state of row d_src_rows[b] (< 0 or b itself: stays), then plan
void launch_batch_fork(const DevBatch& bt, const DevVocab& voc, const int32_t* d_src_rows, uint32_t pair_min_entries,
                       hipStream_t stream);
// plan only (after the host has written states)
void launch_batch_plan(const DevBatch& bt, const DevVocab& voc, uint32_t pair_min_entries, hipStream_t stream);
// measurement aid: n_blocks workgroups of 1024 lanes, each lane a chain of `hops` dependent reads in a 32 KB LDS table
void launch_lds_lookups(int32_t n_blocks, uint32_t hops, uint32_t* sink, hipStream_t stream);
// (c) apply; returns false if the buffer layout needs the element-wise kernel
void launch_apply(void* logits, int elem_size, uint32_t neg_inf, int32_t V_logits, int64_t row_stride,
                  const uint32_t* bitmask, int32_t V_mask, const int32_t* row_index, int32_t n_rows,
                  hipStream_t stream);

}  // namespace xgm
