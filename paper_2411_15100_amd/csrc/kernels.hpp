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
enum : int { kReject = 0, kUncertain = 1, kAccept = 2, kOverflow = 3 };

// automaton tables (device pointers, or LDS copies inside a kernel)
struct DevTables {
  const uint2* hdr;       // [n_nodes] NodeHdr: x = lo | hi<<8 | target<<16, y = row | flags<<16
  const uint8_t* cls;     // [256]
  const uint16_t* rows;   // [n_rows * n_cls]
  const uint32_t* alts;   // pool
  int32_t n_cls;
};

// vocabulary on the device.  A token row is 16 bytes: bytes 0..14 are the
// token's first bytes, byte 15 its length (255 = read the length from the
// offsets).  Bytes past the 15th are read from the CSR arrays.
struct DevVocab {
  const uint4* tok_by_id;     // [V]
  const uint4* tok_by_rank;   // [V] same rows in byte-sorted order
  const uint32_t* off_by_id;  // [V+1] CSR offsets into bytes
  const uint8_t* bytes;       // token bytes, id order
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
  const uint16_t* unc_list;  // context-dependent tokens: id - chunk*4096, grouped by (node, chunk)
  int32_t n_nodes;
};

// per-step upload of the live stacks
struct RowDesc {
  const DevCache* cache;  // null: terminated row (only stop bits)
  uint32_t stack_begin;
  uint32_t n_stacks;
  uint32_t flags;         // bit 0: the text so far is a complete sentence
  uint32_t pad;
};
struct StackDesc {
  uint32_t frame_off;     // into the uint16 frame array
  uint32_t depth;
};

// pairs whose walk exceeded the limits
struct OverflowLog {
  static constexpr uint32_t kCap = 1 << 16;
  uint32_t count;          // total ever recorded (entries wrap around)
  uint32_t pad;
  uint32_t entry[kCap][3]; // (sequence number, row or node, token id or rank)
};

// ---- launchers (all asynchronous on `stream`)
// (a) classify tokens [all ranks] x nodes [node0, node0+n) into rank-space bitsets
void launch_classify(const DevTables& tab, size_t table_bytes, int32_t n_rows_tab, int32_t n_alts,
                     int32_t n_nodes_total, const DevVocab& voc, int32_t node0, int32_t n,
                     uint32_t* acc_rank, uint32_t* unc_rank, OverflowLog* log, uint32_t seq,
                     hipStream_t stream);
// rank space -> id space for n node rows
void launch_permute(const DevVocab& voc, int32_t n, const uint32_t* acc_rank, const uint32_t* unc_rank,
                    uint32_t* acc_id, uint32_t* unc_id, hipStream_t stream);
// per (node, chunk) number of context-dependent tokens
void launch_count_uncertain(const DevVocab& voc, int32_t n, const uint32_t* unc_id, uint32_t* counts,
                            hipStream_t stream);
// write the context-dependent lists; off = [n][n_chunk+1] offsets relative to list
void launch_list_uncertain(const DevVocab& voc, int32_t n, const uint32_t* unc_id, const uint32_t* off,
                           uint16_t* list, hipStream_t stream);
// set / clear single bits of rank-space rows: items = (node - node0, rank, class)
void launch_patch_classes(const DevVocab& voc, const uint32_t* items, int32_t n_items,
                          uint32_t* acc_rank, uint32_t* unc_rank, hipStream_t stream);
// (b) batched mask fill
// step_counter: null on the hot path; otherwise the counting instantiation is launched
void launch_fill(const RowDesc* rows, const StackDesc* stacks, const uint16_t* frames, int32_t B,
                 const DevVocab& voc, uint32_t* out, OverflowLog* log, uint32_t seq,
                 unsigned long long* step_counter, hipStream_t stream);
// (c) apply; returns false if the buffer layout needs the element-wise kernel
void launch_apply(void* logits, int elem_size, uint32_t neg_inf, int32_t V_logits, int64_t row_stride,
                  const uint32_t* bitmask, int32_t V_mask, const int32_t* row_index, int32_t n_rows,
                  hipStream_t stream);

}  // namespace xgm
