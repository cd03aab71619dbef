// HIP kernels for gfx950 (wave64): token walk / classify, rank->id permute,
// context-dependent lists, batched mask fill, -inf apply.
#include <hip/hip_runtime.h>

#include <algorithm>

#include "kernels.hpp"
#include "plan.hpp"
#include "walk.hpp"

namespace xgm {

namespace {


__device__ __forceinline__ void record_overflow(OverflowLog* log, uint32_t seq, uint32_t a, uint32_t b) {
  uint32_t slot = atomicAdd(&log->count, 1u) % OverflowLog::kCap;
  log->entry[slot][0] = seq;
  log->entry[slot][1] = a;
  log->entry[slot][2] = b;
}

// Copy the staged part of a grammar's table image into LDS, 16 bytes per load
// (all threads of the workgroup call this; a barrier must follow).
__device__ __forceinline__ void stage_tables(const DevTables& tab, unsigned char* smem, int nthreads) {
  uint4* dst = reinterpret_cast<uint4*>(smem);
  for (uint32_t k = threadIdx.x; k < tab.stage_bytes / 16; k += nthreads) dst[k] = tab.image[k];
}

// The table access of the walk (same answers as CompactTab in walk.hpp) on a
// table image of which bytes [0, lds_end) have been staged by stage_tables().
// Every pointer carries its address space, so that a lookup in a staged
// section is an LDS read and one in an unstaged section a global load (a
// pointer that may point to either would make every access a much slower flat
// one).  Sections are staged whole, so "is it in LDS" is uniform per section.
// kSmallInLds = true: every section in front of the headers is known to be
// staged, so their reads carry no test at all (a lone wave pays for every
// branch of a walk step with its latency).
#define XGM_LDS __attribute__((address_space(3)))
#define XGM_GLOBAL __attribute__((address_space(1)))
template <bool kSmallInLds>
struct LdsTabT {
  const XGM_LDS unsigned char* lds;     // the staged part of the image
  const XGM_GLOBAL unsigned char* img;  // the whole image
  uint32_t n_near, n_cls, off_shapes, off_targets, off_follow, off_alts, off_hdr, off_first;
  bool cls_lds, shapes_lds, targets_lds, follow_lds, alts_lds;
  __device__ __forceinline__ LdsTabT(const DevTables& t, unsigned char* smem)
      : lds((const XGM_LDS unsigned char*)smem),
        img((const XGM_GLOBAL unsigned char*)reinterpret_cast<const unsigned char*>(t.image)),
        n_near(t.n_near), n_cls((uint32_t)t.n_cls), off_shapes(t.off_shapes), off_targets(t.off_targets),
        off_follow(t.off_follow), off_alts(t.off_alts), off_hdr(t.off_hdr), off_first(t.off_first),
        cls_lds(t.lds_end >= 256u), shapes_lds(t.lds_end >= t.off_targets), targets_lds(t.lds_end >= t.off_follow),
        follow_lds(t.lds_end >= t.off_alts), alts_lds(t.lds_end >= t.off_hdr) {}
  __device__ __forceinline__ uint32_t rd8(uint32_t off, bool in_lds) const {
    return (kSmallInLds || in_lds) ? (uint32_t)lds[off] : (uint32_t)img[off];
  }
  __device__ __forceinline__ uint32_t rd16(uint32_t off, bool in_lds) const {
    return (kSmallInLds || in_lds) ? (uint32_t)*(const XGM_LDS uint16_t*)(lds + off)
                                   : (uint32_t)*(const XGM_GLOBAL uint16_t*)(img + off);
  }
  __device__ __forceinline__ uint32_t rd32(uint32_t off, bool in_lds) const {
    return (kSmallInLds || in_lds) ? *(const XGM_LDS uint32_t*)(lds + off) : *(const XGM_GLOBAL uint32_t*)(img + off);
  }
  __device__ __forceinline__ uint2 header(uint32_t n) const {
    unsigned long long h;  // one 8-byte read
    if (n < n_near) h = *(const XGM_LDS unsigned long long*)(lds + off_hdr + n * 8u);
    else h = *(const XGM_GLOBAL unsigned long long*)(img + off_hdr + (size_t)n * 8u);
    return make_uint2((uint32_t)h, (uint32_t)(h >> 32));
  }
  __device__ __forceinline__ void lookup(uint32_t n, uint32_t c, uint32_t& k, uint32_t& single, uint32_t& base_out,
                                         bool& pooled, uint32_t& fin, uint32_t& after) const {
    const uint2 h = header(n);
    k = 0; single = 0; base_out = 0; pooled = false;
    fin = h.y & 1u;
    after = (rd32(off_follow + ((h.y >> 16) * 8u + (c >> 5)) * 4u, follow_lds) >> (c & 31)) & 1u;
    if (h.y & 2u) {
      const uint32_t cl = rd8(c, cls_lds);
      const uint32_t si = rd8(off_shapes + (h.x & 0xFFFFu) * n_cls + cl, shapes_lds);
      if (si != 0xFFu) {
        const uint32_t a = rd16(off_targets + ((h.x >> 16) + si) * 2u, targets_lds);
        if (a < 0x8000u) { k = 1; single = (0xFFFFu << 16) | a; }
        else { base_out = a & 0x7FFFu; k = alt(base_out); pooled = true; }
      }
    } else {
      const uint32_t lo = h.x & 0xFFu, hi = (h.x >> 8) & 0xFFu;
      if (c >= lo && c <= hi) { k = 1; single = (0xFFFFu << 16) | (h.x >> 16); }
    }
  }
  __device__ __forceinline__ uint32_t alt(uint32_t idx) const { return rd32(off_alts + idx * 4u, alts_lds); }
  __device__ __forceinline__ bool is_final(uint32_t n) const { return header(n).y & 1u; }
  __device__ __forceinline__ bool is_dead_end(uint32_t n) const { return header(n).y & 4u; }
  // can byte c be consumed at node n inside its frame (byte edge, or first byte of a rule it refers to)?
  __device__ __forceinline__ bool can_start(uint32_t n, uint32_t c) const {
    return (*(const XGM_GLOBAL uint32_t*)(img + off_first + ((size_t)n * 8u + (c >> 5)) * 4u) >> (c & 31)) & 1u;
  }
  // can byte c come right after an instance of node n's rule (h = header(n))?
  __device__ __forceinline__ bool can_follow(const uint2& h, uint32_t c) const {
    return (rd32(off_follow + ((h.y >> 16) * 8u + (c >> 5)) * 4u, follow_lds) >> (c & 31)) & 1u;
  }
  // generic pointer to the 256-bit FOLLOW set of node n's rule (read on the rare exit from the start frame)
  __device__ __forceinline__ const uint32_t* follow_of(uint32_t n) const {
    const uint32_t off = off_follow + (header(n).y >> 16) * 32u;
    return (kSmallInLds || follow_lds) ? (const uint32_t*)(const XGM_LDS uint32_t*)(lds + off)
                                       : (const uint32_t*)(const XGM_GLOBAL uint32_t*)(img + off);
  }
};
using LdsTab = LdsTabT<false>;
// are all sections in front of the headers staged?
__device__ __forceinline__ bool small_sections_staged(const DevTables& t) { return t.lds_end >= t.off_hdr; }

// The live frames of a request for the fill kernel: the topmost ones in LDS,
// deeper ones (stacks deeper than the LDS window) in global memory.
struct LiveView {
  const XGM_LDS uint16_t* lds;       // frames [lo, ..) of this stack
  const XGM_GLOBAL uint16_t* glob;   // all frames of this stack
  uint32_t lo;
  __device__ __forceinline__ uint32_t operator[](uint32_t k) const { return k >= lo ? lds[k - lo] : glob[k]; }
};

// ---------------------------------------------------------------- kernel (a)
// Workgroup size of the classify kernel.  A grammar whose staged tables are
// small runs with 256 threads (many workgroups per compute unit, short tails);
// one that needs most of the LDS budget runs with 768, so that two workgroups
// per compute unit still give 6 waves per SIMD.
constexpr int kClassifyThreadsSmall = 256, kClassifyThreadsLarge = 768;
constexpr uint32_t kClassifySmallStage = 24 * 1024;
// nodes a thread classifies its token at, one after the other: few for small tables (more, shorter-lived
// workgroups: the slowest walks weigh less), more where every workgroup has a large table image to stage
constexpr int kNodesPerBlockSmall = 4, kNodesPerBlockLarge = 16;

// One thread owns one token (byte-sorted order, so a wave's 64 tokens are
// neighbours in the sorted vocabulary and mostly share prefixes and control
// flow) and classifies it at several nodes, the token staying in
// registers.  Each wave packs its 64 results per node with a ballot into two
// mask words of the rank-space bitsets.  The automaton tables (as many node
// headers as `n_near`) are first copied into shared memory.
template <int kClassifyThreads, class Tab>
__device__ __forceinline__ void classify_body(const Tab& T, const DevVocab& voc, int32_t node0, int32_t n_nodes,
                                              uint32_t* __restrict__ acc_rank, uint32_t* __restrict__ unc_rank,
                                              uint32_t* __restrict__ plain_rank, uint32_t* __restrict__ plain_count,
                                              OverflowLog* log, uint32_t seq, int32_t nodes_per_block) {
  const int32_t r = blockIdx.x * kClassifyThreads + threadIdx.x;
  const bool live_lane = r < voc.V;
  uint4 tk = make_uint4(0, 0, 0, 0);
  const uint8_t* ext = voc.bytes;
  int len = 0;
  if (live_lane) {
    tk = voc.tok_by_rank[r];
    len = (int)(tk.w >> 24);
    if (len >= 15) {
      const int32_t id = voc.id_of_rank[r];
      ext = voc.bytes + voc.off_by_id[id];
      if (len == 255) len = (int)(voc.off_by_id[id + 1] - voc.off_by_id[id]);
    }
  }
  const int32_t word = (blockIdx.x * kClassifyThreads + (threadIdx.x & ~63)) >> 5;  // even
  const int32_t n_begin = blockIdx.y * nodes_per_block;
  const int32_t n_end = min(n_begin + nodes_per_block, n_nodes);
  // Most pairs are settled by the token's first byte: if the node cannot
  // consume it inside its frame, the token is rejected - or, at a node where
  // the rule may end, leaves the frame at position 0.  One bit per node of the
  // block says whether a walk is needed at all (the loads are issued together).
  const uint32_t c0 = tk.x & 0xFFu;
  uint32_t needs_walk = 0u;
  if (live_lane && len > 0)
    for (int32_t k = n_begin; k < n_end; ++k)
      needs_walk |= (uint32_t)T.can_start((uint32_t)(node0 + k), c0) << (k - n_begin);
  for (int32_t k = n_begin; k < n_end; ++k) {
    int res = kReject;
    if (live_lane && len > 0) {
      if ((needs_walk >> (k - n_begin)) & 1u) {
        res = walk_token<true>(T, tk, ext, len, (uint32_t)(node0 + k), (const uint16_t*)nullptr, 1u, nullptr, T.follow_of(node0 + k));
        if (res == kOverflow) { record_overflow(log, seq, (uint32_t)k, (uint32_t)r); res = kReject; }
      } else {
        const uint2 h = T.header((uint32_t)(node0 + k));
        if (h.y & 1u) res = T.can_follow(h, c0) ? kUncertain : kUncertainPlain;
      }
    }
    const unsigned long long a = __ballot(res == kAccept);
    const unsigned long long u = __ballot(res == kUncertain);
    const unsigned long long p = __ballot(res == kUncertainPlain);
    if ((threadIdx.x & 63) == 0 && word < voc.WR) {
      uint32_t* pa = acc_rank + (size_t)k * voc.WR + word;
      uint32_t* pu = unc_rank + (size_t)k * voc.WR + word;
      pa[0] = (uint32_t)a;
      pa[1] = (uint32_t)(a >> 32);
      pu[0] = (uint32_t)u;
      pu[1] = (uint32_t)(u >> 32);
      if (plain_rank) {
        uint32_t* pp = plain_rank + (size_t)k * voc.WR + word;
        pp[0] = (uint32_t)p;
        pp[1] = (uint32_t)(p >> 32);
      }
      if (p) atomicAdd(&plain_count[node0 + k], (uint32_t)__popcll(p));
    }
  }
}


template <int kClassifyThreads>
__global__ __launch_bounds__(kClassifyThreads) void classify_kernel(
    DevTables tab, DevVocab voc, int32_t node0, int32_t n_nodes, uint32_t* __restrict__ acc_rank,
    uint32_t* __restrict__ unc_rank, uint32_t* __restrict__ plain_rank, uint32_t* __restrict__ plain_count,
    OverflowLog* log, uint32_t seq, int32_t nodes_per_block) {
  extern __shared__ __align__(16) unsigned char smem[];
  stage_tables(tab, smem, kClassifyThreads);
  __syncthreads();
  if (small_sections_staged(tab))
    classify_body<kClassifyThreads>(LdsTabT<true>(tab, smem), voc, node0, n_nodes, acc_rank, unc_rank, plain_rank,
                                    plain_count, log, seq, nodes_per_block);
  else
    classify_body<kClassifyThreads>(LdsTab(tab, smem), voc, node0, n_nodes, acc_rank, unc_rank, plain_rank, plain_count,
                                    log, seq, nodes_per_block);
}

// Rank space -> id space: bit id of the output = bit rank_of_id[id] of the
// input.  One workgroup serves up to kPermuteNodes node rows: their rank-space
// rows sit in LDS so that the random bit lookups never leave the CU, and the
// id -> rank table is read once for all of them.
constexpr int kPermuteThreads = 1024;
constexpr int kPermuteNodes = 4;
__global__ __launch_bounds__(kPermuteThreads) void permute_kernel(DevVocab voc, int32_t n_nodes, int32_t per_block,
                                                                  const uint32_t* __restrict__ acc_rank,
                                                                  const uint32_t* __restrict__ unc_rank,
                                                                  uint32_t* __restrict__ acc_id,
                                                                  uint32_t* __restrict__ unc_id) {
  extern __shared__ __align__(16) unsigned char smem[];
  uint32_t* rows = reinterpret_cast<uint32_t*>(smem);  // [per_block][2][WR]
  const int32_t first = blockIdx.x * per_block;
  const int32_t nb = min(per_block, n_nodes - first);
  for (int32_t q = 0; q < nb; ++q)
    for (int k = threadIdx.x; k < voc.WR; k += kPermuteThreads) {
      rows[(size_t)(2 * q) * voc.WR + k] = acc_rank[(size_t)(first + q) * voc.WR + k];
      rows[(size_t)(2 * q + 1) * voc.WR + k] = unc_rank[(size_t)(first + q) * voc.WR + k];
    }
  __syncthreads();
  const int32_t v64 = (voc.V + 63) & ~63;
  for (int32_t id = threadIdx.x; id < v64; id += kPermuteThreads) {
    const bool in = id < voc.V;
    const uint32_t r = in ? (uint32_t)voc.rank_of_id[id] : 0u;
    const int32_t w = id >> 5;
#pragma unroll
    for (int32_t q = 0; q < kPermuteNodes; ++q) {
      if (q >= nb) break;
      const bool a = in && ((rows[(size_t)(2 * q) * voc.WR + (r >> 5)] >> (r & 31)) & 1u);
      const bool u = in && ((rows[(size_t)(2 * q + 1) * voc.WR + (r >> 5)] >> (r & 31)) & 1u);
      const unsigned long long ba = __ballot(a), bu = __ballot(u);
      if ((threadIdx.x & 63) == 0) {
        const size_t node = (size_t)(first + q);
        acc_id[node * voc.W + w] = (uint32_t)ba;
        unc_id[node * voc.W + w] = (uint32_t)bu;
        if (w + 1 < voc.W) {
          acc_id[node * voc.W + w + 1] = (uint32_t)(ba >> 32);
          unc_id[node * voc.W + w + 1] = (uint32_t)(bu >> 32);
        }
      }
    }
  }
}

__global__ void count_uncertain_kernel(DevVocab voc, const uint32_t* __restrict__ unc_id, uint32_t* __restrict__ counts) {
  // one workgroup of kChunkWords threads per (chunk, node)
  __shared__ uint32_t s[kChunkWords];
  const size_t node = blockIdx.y;
  const int32_t w = blockIdx.x * kChunkWords + threadIdx.x;
  s[threadIdx.x] = (w < voc.W) ? __popc(unc_id[node * voc.W + w]) : 0u;
  __syncthreads();
  for (int d = kChunkWords / 2; d > 0; d >>= 1) {
    if ((int)threadIdx.x < d) s[threadIdx.x] += s[threadIdx.x + d];
    __syncthreads();
  }
  if (threadIdx.x == 0) counts[node * voc.n_chunk + blockIdx.x] = s[0];
}

__global__ void list_uncertain_kernel(DevVocab voc, const uint32_t* __restrict__ unc_id, const uint32_t* __restrict__ off,
                                      uint32_t* __restrict__ list) {
  __shared__ uint32_t s[kChunkWords];
  const size_t node = blockIdx.y;
  const int32_t w = blockIdx.x * kChunkWords + threadIdx.x;
  uint32_t bits = (w < voc.W) ? unc_id[node * voc.W + w] : 0u;
  s[threadIdx.x] = __popc(bits);
  __syncthreads();
  // inclusive scan (Hillis-Steele) over the 128 per-word counts
  for (int d = 1; d < kChunkWords; d <<= 1) {
    uint32_t v = ((int)threadIdx.x >= d) ? s[threadIdx.x - d] : 0u;
    __syncthreads();
    s[threadIdx.x] += v;
    __syncthreads();
  }
  uint32_t pos = off[node * (voc.n_chunk + 1) + blockIdx.x] + s[threadIdx.x] - __popc(bits);
  while (bits) {
    const uint32_t b = __ffs(bits) - 1;
    bits &= bits - 1;
    list[pos++] = threadIdx.x * 32 + b;
  }
}

// One workgroup per (chunk, node) list: every entry's token is walked once
// more from the node to find where it leaves the node's frame (the walk reads
// the tables from global memory: most lists are empty or short, staging would
// cost more), then the list is sorted by the number of bytes left after that
// position, so that neighbouring lanes of the fill kernel get walks of
// similar length.
constexpr int kAnnotateThreads = 256;
__global__ __launch_bounds__(kAnnotateThreads) void annotate_lists_kernel(DevTables tab, DevVocab voc, int32_t node0,
                                                                          const uint32_t* __restrict__ off,
                                                                          uint32_t* __restrict__ list) {
  __shared__ uint32_t seg[kChunkTokens];
  __shared__ uint8_t rem_of[kChunkTokens];
  __shared__ uint32_t bucket[16];
  const int32_t node = node0 + blockIdx.y, chunk = blockIdx.x;
  const uint32_t j0 = off[(size_t)node * (voc.n_chunk + 1) + chunk], j1 = off[(size_t)node * (voc.n_chunk + 1) + chunk + 1];
  const uint32_t n = j1 - j0;
  if (n == 0) return;
  if (threadIdx.x < 16) bucket[threadIdx.x] = 0u;
  __syncthreads();
  const LdsTab T(tab, nullptr);  // launched with nothing staged
  for (uint32_t e = threadIdx.x; e < n; e += kAnnotateThreads) {
    const uint32_t lid = list[j0 + e] & 0xFFFu;
    const int32_t id = chunk * kChunkTokens + (int32_t)lid;
    const uint4 tk = voc.tok_by_id[id];
    int len = (int)(tk.w >> 24);
    const uint8_t* ext = voc.bytes;
    if (len >= 15) {
      ext = voc.bytes + voc.off_by_id[id];
      if (len == 255) len = (int)(voc.off_by_id[id + 1] - voc.off_by_id[id]);
    }
    uint32_t exits = 0;
    const int res = walk_token<true>(T, tk, ext, len, (uint32_t)node, (const uint16_t*)nullptr, 1u, nullptr, T.follow_of(node), 0, &exits);
    uint32_t meta = kEntryFullWalk, pos = 0, late = 0;
    if (res != kOverflow && exits != 0u && (exits & (exits - 1u)) == 0u && !(exits & 0x80000000u)) {
      const uint32_t k = __ffs(exits) - 1;  // the single exit position, 0..30
      const uint32_t suffix = (uint32_t)len - k;
      if (suffix == 1u) { meta = kEntrySuffix1; pos = k; }
      else if (suffix == 2u) { meta = kEntrySuffix2; pos = k; }
      else if (k <= 12u) { meta = k; pos = k; }
      else late = k;                        // kind stays kEntryFullWalk, the position goes into the second byte field
    }
    const uint32_t b1 = token_byte(tk, ext, (int)pos);
    const uint32_t b2 = meta == kEntryFullWalk ? late : ((int)pos + 1 < len ? token_byte(tk, ext, (int)pos + 1) : 0u);
    const uint32_t rem = min(15, len - (int)(late ? late : pos));
    seg[e] = lid | (meta << 12) | (b1 << 16) | (b2 << 24);
    rem_of[e] = (uint8_t)rem;
    atomicAdd(&bucket[rem], 1u);
  }
  __syncthreads();
  if (threadIdx.x == 0) {  // exclusive scan of the 16 bucket sizes
    uint32_t run = 0;
    for (int k = 0; k < 16; ++k) { const uint32_t c = bucket[k]; bucket[k] = run; run += c; }
  }
  __syncthreads();
  for (uint32_t e = threadIdx.x; e < n; e += kAnnotateThreads) {
    list[j0 + atomicAdd(&bucket[rem_of[e]], 1u)] = seg[e];
  }
}

// The per-context classes of every list entry (see kCtx*): one thread per
// entry over all lists of the grammar, tables staged as in the classify
// kernel.  For each context node of the entry's rule the entry's suffix is
// walked from that node with nothing known below it.
constexpr int kContextThreads = 768;
__global__ __launch_bounds__(kContextThreads) void context_classes_kernel(DevTables tab, DevVocab voc, int32_t n_nodes,
                                                                          uint32_t total,
                                                                          const uint32_t* __restrict__ off,
                                                                          const uint32_t* __restrict__ list,
                                                                          uint32_t* __restrict__ list_ctx,
                                                                          const uint32_t* __restrict__ ctx_off,
                                                                          const uint16_t* __restrict__ ctx_node) {
  extern __shared__ __align__(16) unsigned char smem[];
  stage_tables(tab, smem, kContextThreads);
  __syncthreads();
  auto body = [&](const auto& T) {
    const uint32_t j = blockIdx.x * kContextThreads + threadIdx.x;
    if (j >= total) return;
    // the entry's (node, chunk): the last slot of `off` that starts at or before j
    const uint32_t stride = (uint32_t)voc.n_chunk + 1u;
    uint32_t lo = 0u, hi = (uint32_t)n_nodes * stride;  // off[lo] <= j < off[hi - 1 + 1 ...]; the last slot equals total
    while (hi - lo > 1u) {
      const uint32_t mid = (lo + hi) >> 1;
      if (off[mid] <= j) lo = mid; else hi = mid;
    }
    const uint32_t node = lo / stride, chunk = lo % stride;
    const uint32_t e = list[j];
    const uint32_t lid = e & 0xFFFu, meta = (e >> 12) & 15u, b2 = e >> 24;
    const int32_t id = (int32_t)(chunk * kChunkTokens + lid);
    const uint4 tk = voc.tok_by_id[id];
    int len = (int)(tk.w >> 24);
    const uint8_t* ext = voc.bytes;
    if (len >= 15) {
      ext = voc.bytes + voc.off_by_id[id];
      if (len == 255) len = (int)(voc.off_by_id[id + 1] - voc.off_by_id[id]);
    }
    // where the suffix starts (-1: the entry has several exits)
    const int from = meta <= 12u ? (int)meta : meta == kEntrySuffix2 ? len - 2 : meta == kEntrySuffix1 ? len - 1
                                                                                  : (b2 != 0u ? (int)b2 : -1);
    const uint32_t rule = T.header(node).y >> 16;
    const uint32_t ctx0 = ctx_off[rule], n_ctx = ctx_off[rule + 1] - ctx0;  // 0 .. kCtxMax
    uint32_t classes = 0u;
    for (uint32_t i = 0; i < kCtxMax; ++i) {
      uint32_t code = kCtxWalk;
      if (from >= 0 && i < n_ctx) {
        const uint32_t r = ctx_node[ctx0 + i];
        const int c = walk_token<true>(T, tk, ext, len, r, (const uint16_t*)nullptr, 1u, nullptr, T.follow_of(r), from);
        code = c == kAccept ? kCtxAccept : (c == kUncertain || c == kOverflow) ? kCtxWalk : kCtxReject;
      }
      classes |= code << (2u * i);
    }
    list_ctx[j] = classes;
  };
  if (small_sections_staged(tab)) body(LdsTabT<true>(tab, smem));
  else body(LdsTab(tab, smem));
}

// Many nodes of a grammar have the same accepted bitset (the inside of a string is
// the inside of a string wherever it occurs), so the cache keeps every distinct
// row once.  The digest only proposes which rows might be equal: the position-
// dependent mix of every word (the finalizer of splitmix64) is summed over the
// row; equality is then checked word for word.
constexpr int kRowThreads = 256;
__device__ __forceinline__ unsigned long long mix64(unsigned long long x) {
  x ^= x >> 30; x *= 0xBF58476D1CE4E5B9ull;
  x ^= x >> 27; x *= 0x94D049BB133111EBull;
  return x ^ (x >> 31);
}
__global__ __launch_bounds__(kRowThreads) void hash_rows_kernel(const uint32_t* __restrict__ rows, int32_t W,
                                                                unsigned long long* __restrict__ digest) {
  __shared__ unsigned long long part[kRowThreads / 64];
  const uint32_t* row = rows + (size_t)blockIdx.x * W;
  unsigned long long h = 0ull;
  for (int32_t w = threadIdx.x; w < W; w += kRowThreads)
    h += mix64(((unsigned long long)(uint32_t)w << 32 | row[w]) + 0x9E3779B97F4A7C15ull);
#pragma unroll
  for (uint32_t d = 32; d > 0; d >>= 1) h += __shfl_down(h, d, 64);
  if ((threadIdx.x & 63u) == 0) part[threadIdx.x >> 6] = h;
  __syncthreads();
  if (threadIdx.x == 0) {
    unsigned long long t = 0ull;
    for (int k = 0; k < kRowThreads / 64; ++k) t += part[k];
    digest[blockIdx.x] = t;
  }
}
__global__ __launch_bounds__(kRowThreads) void rows_equal_kernel(const uint32_t* __restrict__ rows, int32_t W,
                                                                 const int32_t* __restrict__ rep,
                                                                 uint32_t* __restrict__ equal) {
  __shared__ uint32_t differs;
  if (threadIdx.x == 0) differs = 0u;
  __syncthreads();
  const uint32_t* a = rows + (size_t)blockIdx.x * W;
  const uint32_t* b = rows + (size_t)rep[blockIdx.x] * W;
  bool d = false;
  for (int32_t w = threadIdx.x; w < W; w += kRowThreads) d |= a[w] != b[w];
  if (d) differs = 1u;
  __syncthreads();
  if (threadIdx.x == 0) equal[blockIdx.x] = differs ? 0u : 1u;
}
__global__ __launch_bounds__(kRowThreads) void gather_rows_kernel(const uint32_t* __restrict__ rows, int32_t W,
                                                                  const int32_t* __restrict__ unique,
                                                                  uint32_t* __restrict__ out) {
  const uint32_t* src = rows + (size_t)unique[blockIdx.x] * W;
  uint32_t* dst = out + (size_t)blockIdx.x * W;
  for (int32_t w = threadIdx.x; w < W; w += kRowThreads) dst[w] = src[w];
}

__global__ void patch_classes_kernel(DevVocab voc, const uint32_t* __restrict__ items, int32_t n_items,
                                     uint32_t* acc_rank, uint32_t* unc_rank, uint32_t* plain_rank) {
  const int32_t k = blockIdx.x * blockDim.x + threadIdx.x;
  if (k >= n_items) return;
  const size_t node = items[3 * k];
  const uint32_t r = items[3 * k + 1], cls = items[3 * k + 2];
  const uint32_t bit = 1u << (r & 31);
  uint32_t* pa = acc_rank + node * voc.WR + (r >> 5);
  uint32_t* pu = unc_rank + node * voc.WR + (r >> 5);
  if (cls == (uint32_t)kAccept) atomicOr(pa, bit); else atomicAnd(pa, ~bit);
  if (cls == (uint32_t)kUncertain) atomicOr(pu, bit); else atomicAnd(pu, ~bit);
  if (plain_rank) {
    uint32_t* pp = plain_rank + node * voc.WR + (r >> 5);
    if (cls == (uint32_t)kUncertainPlain) atomicOr(pp, bit); else atomicAnd(pp, ~bit);
  }
}

// One 16-byte group of a logits row (section 2.1): `mk` holds the mask bits of
// its EPT = 16 / ESIZE elements, e0 is the index of its first element.  All
// allowed: nothing is touched.  None allowed: one 16-byte store of the -inf
// pattern.  One or two disallowed: those elements are stored by themselves,
// nothing is read.  More: the group is read, blended and stored whole (many
// small stores cost more than the read).
template <int ESIZE>
__device__ __forceinline__ void apply_group(unsigned char* p, uint32_t mk, int32_t e0, int32_t V_logits, uint32_t neg_inf) {
  constexpr int EPT = 16 / ESIZE;
  constexpr uint32_t kAll = (1u << EPT) - 1u;
  if (mk == kAll) return;
  const uint32_t two = neg_inf | (neg_inf << 16);
  const bool whole = e0 + EPT <= V_logits;
  if (mk == 0u && whole) {
    // a streaming store: the line is written whole and not read again here, so it need not stay in the
    // caches (measured on the serving masks: 10.7 -> 8.6 us for the stand-alone kernel; the same hint on
    // the single-element stores below costs time, their lines are better merged in the cache)
    typedef uint32_t v4u __attribute__((ext_vector_type(4)));
    const uint32_t w = ESIZE == 2 ? two : neg_inf;
    const v4u val = {w, w, w, w};
    __builtin_nontemporal_store(val, reinterpret_cast<v4u*>(p));
  } else if (whole && EPT - __popc(mk) > 2) {
    uint4 v = *reinterpret_cast<const uint4*>(p);
    if (ESIZE == 2) {
      uint32_t* q = reinterpret_cast<uint32_t*>(&v);
#pragma unroll
      for (int h = 0; h < 4; ++h) {
        const uint32_t keep = ((mk >> (2 * h)) & 1u ? 0x0000FFFFu : 0u) | ((mk >> (2 * h + 1)) & 1u ? 0xFFFF0000u : 0u);
        q[h] = (q[h] & keep) | (two & ~keep);
      }
    } else {
      if (!(mk & 1u)) v.x = neg_inf;
      if (!(mk & 2u)) v.y = neg_inf;
      if (!(mk & 4u)) v.z = neg_inf;
      if (!(mk & 8u)) v.w = neg_inf;
    }
    *reinterpret_cast<uint4*>(p) = v;
  } else {
#pragma unroll
    for (int h = 0; h < EPT; ++h)
      if (e0 + h < V_logits && !((mk >> h) & 1u)) {
        if (ESIZE == 2) reinterpret_cast<uint16_t*>(p)[h] = (uint16_t)neg_inf;
        else reinterpret_cast<uint32_t*>(p)[h] = neg_inf;
      }
  }
}

// The logits of one workgroup of the fused kernel: its request's row, the
// elements [e_begin, e_end) that its mask words in LDS cover (section 2.1).
// APPLY = bytes per logit; 0 = the kernel leaves the logits alone.
template <int APPLY>
struct LogitsRange {
  unsigned char* row;
  const uint32_t* words;  // the workgroup's mask words; bit 0 of words[0] is element e_begin
  int32_t e_begin, e_end, V, V_logits;
  uint32_t neg_inf;
  // thread t of nt: the range's groups t, t + nt, ...  (One group after the other: fetching the groups
  // that must be read several at a time made the launch longer, not shorter.)
  __device__ __forceinline__ void groups(uint32_t t, uint32_t nt) const {
    if constexpr (APPLY != 0) {
      constexpr int EPT = 16 / APPLY;
      constexpr uint32_t kAll = (1u << EPT) - 1u;
      for (int32_t e0 = e_begin + (int32_t)t * EPT; e0 < e_end; e0 += (int32_t)nt * EPT) {
        uint32_t mk = 0u;
        if (e0 < V) {
          mk = (words[(e0 - e_begin) >> 5] >> (e0 & 31)) & kAll;
          if (e0 + EPT > V) mk &= (1u << (V - e0)) - 1u;
        }
        apply_group<APPLY>(row + (size_t)e0 * APPLY, mk, e0, V_logits, neg_inf);
      }
    }
  }
  // one element by itself
  __device__ __forceinline__ void reject(int32_t id) const {
    if constexpr (APPLY != 0) {
      if (id < V_logits) {
        if (APPLY == 2) reinterpret_cast<uint16_t*>(row)[id] = (uint16_t)neg_inf;
        else reinterpret_cast<uint32_t*>(row)[id] = neg_inf;
      }
    }
  }
};

// ---------------------------------------------------------------- kernel (b)
// The per-step stack upload: a plain copy from pinned host memory (which the
// device reads over the bus) into device memory, as a kernel on the caller's
// stream.  For the few tens of kilobytes of a step this takes a fraction of
// the time a copy-engine transfer with its cross-queue synchronisation does.
constexpr int kUploadThreads = 256;
__global__ __launch_bounds__(kUploadThreads) void upload_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst,
                                                                uint32_t n16) {
  const uint32_t i = blockIdx.x * kUploadThreads + threadIdx.x;
  if (i < n16) dst[i] = src[i];
}

constexpr int kFillThreads = 1024;
constexpr int kFillQueue = 4096;                // survivors walked per round
constexpr int kFillFramesLds = 1024;            // live frames kept in LDS (deeper stacks: global memory)
constexpr uint32_t kQueueRejected = 1u << 23;   // in a queue entry: walked and found disallowed (see fill_lists)

// accumulates a 256-bit set into 8 LDS words
struct LdsSetAcc {
  uint32_t* words;
  __device__ __forceinline__ void add(uint32_t w, uint32_t bits) { if (bits) atomicOr(words + w, bits); }
};

// One workgroup of 16 waves serves one request and a contiguous range of its
// chunks of 4096 token ids, as planned on the host or by the plan kernel
// (FillBlock).  Once per
// workgroup the request's automaton tables and live stacks are copied into
// LDS; from then on a step of a token walk costs LDS lookups only.  The
// workgroup owns its mask words in LDS:
//   1. every word = OR of the accepted bitsets of the tops of all stacks
//      (Algorithm 1: the result is the union over the parallel stacks);
//   2. per stack, the context-dependent lists of its chunks are read once,
//      coalesced.  Most entries name the suffix of their token that is left
//      when the token leaves the top frame, and carry its first two bytes.
//      Whether the rest of the stack can consume those two bytes is looked up
//      in a 256 x 256-bit table that the workgroup first computes for the
//      stack (one lane per first byte: an enumerating walk of that byte
//      collects the bytes that can follow it) or copies, if it was computed
//      when the state was entered; the per-context word of the entry settles
//      it without any of this if the node below the top frame is one of the
//      top rule's few contexts; a suffix of one or two bytes
//      is thereby decided outright, a longer one is dropped or queued.
//      Entries that need a walk from the top are tested on their first byte
//      against a 256-bit set the host packed with the stack.  All these tests
//      are exact and need only the list entry; survivors are compacted into
//      an LDS queue (one LDS atomic per wave);
//   3. the queue is walked (one lane per survivor); allowed tokens are ORed
//      into the words with LDS atomics.  Long lists take several rounds of 2;
//      the walk waits until the queue might not hold another round's
//      survivors, which as a rule means: one walk, after the last round;
//   4. the words are stored once, coalesced (the stop tokens were added in 1).
// No global atomics, no second pass over the mask.
// When the kernel also masks the logits, the last walks of a workgroup - a
// few tokens in one wave, as a rule, and what the whole launch ends up waiting
// for - run beside that work instead of in front of it: queued tokens count as
// allowed for the moment, the waves without a walk write -inf for everything
// else in the workgroup's range, and the tokens whose walk says no get theirs
// after the walks (one element each).
// COUNT = true additionally sums the automaton steps of all walks into
// *step_counter (instrumentation for the benchmark; never used on the hot path).
struct FillShared {
  uint32_t words[kFillMaxChunks * kChunkWords];
  uint32_t queue[kFillQueue];     // late exit position << 24 | kQueueRejected | (chunk - c0) << 16 | kind << 12 | local id
  uint16_t live[kFillFramesLds];
  uint32_t hdr[kStackHdrWords];   // the current stack's header: top, depth, frame offset, and 2 x 256 bits: the
                                  // bytes consumable from the stack / from the stack without its top frame
  uint32_t off[kFillMaxChunks + 1];  // list offsets of the current stack's top for chunks c0 .. c1
  uint32_t pair[256 * 8];         // per first byte: the bytes that can follow it, from the stack without its top frame
  uint32_t queue_n;
};

// The two-byte table of a stack without its top frame, into LDS (all threads of
// the workgroup call this; it ends with a barrier): one lane per first byte
// that the stack can consume at all (`first_ok`, 256 bits) runs an enumerating
// walk of that byte from `below` (the node under the top frame; `depth` counts
// the top frame) and collects the bytes that can follow it.  A walk over the
// limits leaves its row all ones: the decision then falls to the token walks.
template <int kThreads, class Tab, class Live>
__device__ __forceinline__ void build_pair_table(const Tab& T, uint32_t* pair, const uint32_t* first_ok, uint32_t below,
                                                 const Live& live, uint32_t depth, const uint32_t* node_first,
                                                 const DevVocab& voc) {
  const uint32_t tid = threadIdx.x;
  for (uint32_t k = tid; k < kPairWords; k += kThreads) pair[k] = 0u;
  __syncthreads();
  if (tid < 256u && ((first_ok[tid >> 5] >> (tid & 31u)) & 1u)) {
    LdsSetAcc acc{pair + tid * 8u};
    const CollectNextBytes<Tab, LdsSetAcc> collect{&T, node_first, &acc};
    const int res = walk_token<false>(T, make_uint4(tid, 0u, 0u, 1u << 24), voc.bytes, 1, below, live, depth - 1,
                                      (uint32_t*)nullptr, (const uint32_t*)nullptr, 0, (uint32_t*)nullptr, collect);
    if (res == kOverflow)
      for (uint32_t w = 0; w < 8u; ++w) pair[tid * 8u + w] = 0xFFFFFFFFu;
  }
  __syncthreads();
}

// the header of one stack and its list offsets for chunks c0 .. c1 -> LDS (a barrier must follow)
__device__ __forceinline__ void stage_stack_header(FillShared& sm, const XGM_GLOBAL uint32_t* sh, int32_t c0, int32_t c1) {
  const uint32_t tid = threadIdx.x;
  if (tid < kStackHdrWords) sm.hdr[tid] = sh[tid];
  else if (tid - kStackHdrWords <= (uint32_t)(c1 - c0)) sm.off[tid - kStackHdrWords] = sh[kStackHdrWords + c0 + tid - kStackHdrWords];
}

// Returns true if it has also written the logits of the workgroup's range (`logits`; only with APPLY != 0).
template <bool COUNT, int APPLY, class Tab>
__device__ __forceinline__ bool fill_lists(const Tab& T, FillShared& sm, const RowDesc& rd, const int32_t b,
                                           const int32_t c0, const int32_t c1, const uint32_t frame0,
                                           const bool frames_in_lds,
                                           const XGM_GLOBAL uint32_t* __restrict__ stack_hdrs,
                                           const XGM_GLOBAL uint16_t* __restrict__ frames, const DevVocab& voc,
                                           OverflowLog* log, uint32_t seq, unsigned long long& my_steps,
                                           const uint32_t pair_min_entries,
                                           const XGM_GLOBAL uint32_t* __restrict__ pair_tables,
                                           const LogitsRange<APPLY>& logits) {
  constexpr bool KEEP_UNDECIDED = APPLY != 0;
  bool logits_done = false;
  const uint32_t tid = threadIdx.x, lane = threadIdx.x & 63u;
  const uint32_t hdr_stride = kStackHdrWords + voc.n_chunk + 1;
  const XGM_GLOBAL uint32_t* unc_list = (const XGM_GLOBAL uint32_t*)rd.unc_list;
  const XGM_GLOBAL uint32_t* unc_ctx = (const XGM_GLOBAL uint32_t*)rd.unc_ctx;
  const uint32_t* node_first = reinterpret_cast<const uint32_t*>(reinterpret_cast<const unsigned char*>(rd.tab.image) + rd.tab.off_first);
  const uint32_t* first_ok = sm.hdr + kStackHdrFirst;
  for (uint32_t s = 0; s < rd.n_stacks; ++s) {
    // the stack's header and its list offsets go to LDS with one coalesced read (the first stack's are there already)
    if (s > 0) {
      __syncthreads();  // the previous stack's header is no longer in use
      stage_stack_header(sm, stack_hdrs + (size_t)(rd.stack_begin + s) * hdr_stride, c0, c1);
      __syncthreads();
    }
    if (sm.off[c1 - c0] == sm.off[0]) continue;  // nothing listed here (uniform)
    const uint32_t top = sm.hdr[kStackHdrTop] & 0xFFFFu, depth = sm.hdr[kStackHdrDepth];
    const uint32_t ctx = sm.hdr[kStackHdrCtx];  // which context of the top's rule the frame below is, or kCtxNone
    LiveView live;
    live.lds = (const XGM_LDS uint16_t*)sm.live + (sm.hdr[kStackHdrFrames] - frame0);
    live.glob = frames + sm.hdr[kStackHdrFrames];
    live.lo = frames_in_lds ? 0u : 0xFFFFFFFFu;
    const uint32_t below = depth >= 2 ? live[depth - 2] : 0u;
    // the two-byte table of the stack below the top frame
    const bool have_table = pair_tables != nullptr && ((rd.pair_mask >> s) & 1u);  // computed ahead of this launch
    const bool use_pair = depth >= 2 && (have_table || sm.off[c1 - c0] - sm.off[0] >= pair_min_entries);
    if (use_pair) {
      if (have_table) {
        if (s > 0) {  // the first stack's table came in with the workgroup's first fetches
          const XGM_GLOBAL uint32_t* table = pair_tables + ((size_t)b * kBatchMaxStacks + s) * kPairWords;
          for (uint32_t k = tid; k < kPairWords; k += kFillThreads) sm.pair[k] = table[k];
          __syncthreads();
        }
      } else {
        build_pair_table<kFillThreads>(T, sm.pair, sm.hdr + kStackHdrBelow, below, live, depth, node_first, voc);
      }
    }
    // The last stack's queued tokens count as allowed until they have been walked (see above).
    const bool last_stack = APPLY != 0 && s + 1 == rd.n_stacks;
    // Rounds of chunks whose lists together fit the queue even if every entry survived (one chunk always
    // fits).  Few do survive, so the survivors of a round are only walked when the queue might not hold
    // the next round's as well: as a rule a workgroup walks once, after its last round.
    for (int32_t ca = c0; ca < c1;) {
      int32_t cb = ca + 1;
      while (cb < c1 && sm.off[cb + 1 - c0] - sm.off[ca - c0] <= (uint32_t)kFillQueue) ++cb;
      // the last walks of the workgroup: the logits are written beside them
      const bool beside = last_stack && cb == c1;
      // 2. filter + compact: the lists of consecutive chunks are contiguous, so one flat pass reads them all
      const uint32_t j_begin = sm.off[ca - c0], j_end = sm.off[cb - c0];
      for (uint32_t j = j_begin + (tid & ~63u); j < j_end; j += kFillThreads) {
        const uint32_t jj = j + lane;
        bool keep = false;
        uint32_t lid = 0, meta = 0, cl = 0, late_exit = 0;
        if (jj < j_end) {
          const uint32_t e = unc_list[jj];
          const uint32_t in_ctx = ctx != kCtxNone ? (unc_ctx[jj] >> (2u * ctx)) & 3u : kCtxWalk;
          // the entry's chunk: the last one whose list starts at or before jj
          uint32_t lo = (uint32_t)(ca - c0), hi = (uint32_t)(cb - c0);
          while (hi - lo > 1u) {
            const uint32_t mid = (lo + hi) >> 1;
            if (sm.off[mid] <= jj) lo = mid; else hi = mid;
          }
          cl = lo;
          uint32_t* wchunk = sm.words + cl * kChunkWords;
          lid = e & 0xFFFu;
          meta = (e >> 12) & 15u;
          const uint32_t b1 = (e >> 16) & 0xFFu, b2 = e >> 24;
          const bool seen = (wchunk[lid >> 5] >> (lid & 31)) & 1u;  // already allowed through another stack
          if (meta == kEntryFullWalk) {
            // b2 != 0: a single exit at position b2 after all; the context class may settle it
            const bool ok0 = (first_ok[b1 >> 5] >> (b1 & 31)) & 1u;
            const bool has_exit = b2 != 0u && depth >= 2u;
            if (has_exit && in_ctx != kCtxWalk) {
              if (!seen && ok0 && in_ctx == kCtxAccept) atomicOr(&wchunk[lid >> 5], 1u << (lid & 31));
            } else {
              keep = !seen && ok0;
              late_exit = has_exit ? b2 : 0u;
            }
          } else {
            const bool ok1 = (first_ok[8 + (b1 >> 5)] >> (b1 & 31)) & 1u;
            const bool ok2 = use_pair ? ((sm.pair[b1 * 8u + (b2 >> 5)] >> (b2 & 31)) & 1u) : ok1;
            const bool decided = in_ctx != kCtxWalk || meta == kEntrySuffix1 || (use_pair && meta == kEntrySuffix2);
            if (decided) {
              const bool allowed = in_ctx != kCtxWalk ? in_ctx == kCtxAccept : (meta == kEntrySuffix1 ? ok1 : ok2);
              if (!seen && allowed) atomicOr(&wchunk[lid >> 5], 1u << (lid & 31));
            } else {
              keep = !seen && ok2;
            }
          }
        }
        const unsigned long long m = __ballot(keep);
        if (m) {
          uint32_t base = 0;
          if (lane == 0) base = atomicAdd(&sm.queue_n, (uint32_t)__popcll(m));
          base = __shfl(base, 0, 64);
          if (keep) {
            sm.queue[base + __popcll(m & ((1ull << lane) - 1ull))] = (late_exit << 24) | (cl << 16) | (meta << 12) | lid;
            if (last_stack) atomicOr(&sm.words[cl * kChunkWords + (lid >> 5)], 1u << (lid & 31));  // allowed for the moment
          }
        }
      }
      __syncthreads();
      // 3. walk the survivors, unless the queue has room for all that the next round can add
      const uint32_t nq = sm.queue_n;
      if (cb < c1) {
        int32_t cn = cb + 1;
        while (cn < c1 && sm.off[cn + 1 - c0] - sm.off[cb - c0] <= (uint32_t)kFillQueue) ++cn;
        if (nq + (sm.off[cn - c0] - sm.off[cb - c0]) <= (uint32_t)kFillQueue) {
          ca = cb;
          continue;
        }
      }
      const uint32_t first_free = (min(nq, (uint32_t)kFillThreads) + 63u) & ~63u;  // the waves from here on have no walk
      if (beside && tid >= first_free) logits.groups(tid - first_free, kFillThreads - first_free);
      for (uint32_t q = tid; q < nq; q += kFillThreads) {
        const uint32_t e = sm.queue[q];
        const uint32_t lid = e & 0xFFFu, meta = (e >> 12) & 15u, cl = (e >> 16) & 0x7Fu, late_exit = e >> 24;
        const int32_t id = (c0 + (int32_t)cl) * kChunkTokens + (int32_t)lid;
        const uint4 tk = voc.tok_by_id[id];
        int len = (int)(tk.w >> 24);
        const uint8_t* ext = voc.bytes;
        if (len >= 15) {
          ext = voc.bytes + voc.off_by_id[id];
          if (len == 255) len = (int)(voc.off_by_id[id + 1] - voc.off_by_id[id]);
        }
        uint32_t n_steps = 0;
        // a token with a single exit continues right there, in the frame below the top
        const bool full = meta == kEntryFullWalk && late_exit == 0u;
        const int i0 = full ? 0 : late_exit ? (int)late_exit : (meta == kEntrySuffix2 ? len - 2 : (int)meta);
        const int res = walk_token<false>(T, tk, ext, len, full ? top : below, live, full ? depth : depth - 1,
                                          COUNT ? &n_steps : nullptr, (const uint32_t*)nullptr, i0);
        if (COUNT) my_steps += n_steps;
        if (last_stack) {
          if (res == kReject) {
            atomicAnd(&sm.words[cl * kChunkWords + (lid >> 5)], ~(1u << (lid & 31)));
            if (beside) sm.queue[q] = e | kQueueRejected;
          } else if (res == kOverflow) {
            record_overflow(log, seq, (uint32_t)b, (uint32_t)id);  // stays allowed until the host has decided it
          }
        } else if (res == kAccept) {
          atomicOr(&sm.words[cl * kChunkWords + (lid >> 5)], 1u << (lid & 31));
        } else if (res == kOverflow) {
          record_overflow(log, seq, (uint32_t)b, (uint32_t)id);
          if (KEEP_UNDECIDED) atomicOr(&sm.words[cl * kChunkWords + (lid >> 5)], 1u << (lid & 31));
        }
      }
      if (beside) {
        if (first_free >= (uint32_t)kFillThreads) logits.groups(tid, kFillThreads);  // every wave had walks
        __syncthreads();  // the group stores above come first
        for (uint32_t q = tid; q < nq; q += kFillThreads) {
          const uint32_t e = sm.queue[q];
          if (e & kQueueRejected) logits.reject((c0 + (int32_t)((e >> 16) & 0x7Fu)) * kChunkTokens + (int32_t)(e & 0xFFFu));
        }
        logits_done = true;
      }
      __syncthreads();
      if (tid == 0) sm.queue_n = 0u;
      __syncthreads();
      ca = cb;
    }
  }
  return logits_done;
}

// Two workgroups of 16 waves per compute unit need 8 waves per SIMD: the second
// launch bound keeps the kernel within the 96 scalar and 64 vector registers
// per wave that this takes.
// APPLY = 0: the mask only.  APPLY = 2 / 4 (bytes per logit): the workgroup
// also writes -inf into the logits of its (row, chunk range) straight from its
// LDS words (section 2.1), which saves a launch and the re-read of the mask.
// A token whose walk exceeded the limits is then left allowed (bit set, logit
// untouched) until the host has decided it.
struct FusedApply {
  unsigned char* logits;  // [B][row_stride] elements of APPLY bytes; 16-byte aligned rows
  int64_t row_stride;     // elements
  int32_t V_logits;
  uint32_t neg_inf;
  uint32_t pair_min_entries;  // (rides along) lists shorter than this are filtered on one byte only
  const uint32_t* pair_tables;  // (rides along) DevBatch::pair, or null
};

template <bool COUNT, int APPLY>
__global__ __launch_bounds__(kFillThreads, 8) void fill_kernel(const RowDesc* __restrict__ rows,
                                                            const uint32_t* __restrict__ stack_hdrs_,
                                                            const uint16_t* __restrict__ frames_,
                                                            const FillBlock* __restrict__ plan, DevVocab voc,
                                                            uint32_t* __restrict__ out, OverflowLog* log, uint32_t seq,
                                                            unsigned long long* step_counter, FusedApply fa) {
  extern __shared__ __align__(16) unsigned char smem[];
  __shared__ FillShared sm;
  const XGM_GLOBAL uint32_t* stack_hdrs = (const XGM_GLOBAL uint32_t*)stack_hdrs_;
  const XGM_GLOBAL uint16_t* frames = (const XGM_GLOBAL uint16_t*)frames_;
  unsigned long long my_steps = 0;
  const uint32_t tid = threadIdx.x;
  const FillBlock blk = plan[blockIdx.x];  // placed by the planner (plan_slot)
  if (blk.row == kNoRow) return;  // padding of the plan
  const int32_t b = (int32_t)blk.row;
  const int32_t c0 = (int32_t)(blk.c0c1 & 0x7FFFu), c1 = (int32_t)(blk.c0c1 >> 16);  // this workgroup's chunks
  const int32_t w_begin = c0 * kChunkWords;
  const int32_t n_words = min(c1 * kChunkWords, voc.W) - w_begin;
  const RowDesc rd = rows[b];
  const bool has_cache = rd.n_stacks > 0 && !(blk.c0c1 & kFillBlockNoEntries);  // are there lists to resolve?
  const uint32_t hdr_stride = kStackHdrWords + voc.n_chunk + 1;
  // everything the row descriptor points to is fetched in one go: tables, live frames, the first stack's
  // header with its list offsets, and (below) the accepted words
  const uint32_t frame0 = rd.frame_begin, n_frames = rd.n_frames;
  const bool frames_in_lds = n_frames <= kFillFramesLds;
  // may the request end here?  then its stop tokens are allowed (the first kFillThreads of them are fetched now)
  const bool may_end = rd.flags & 1u;
  const int32_t my_stop = may_end && (int32_t)tid < voc.n_stop ? voc.stop_ids[tid] : -1;
  if (has_cache) {
    stage_tables(rd.tab, smem, kFillThreads);
    if (frames_in_lds)
      for (uint32_t k = tid; k < n_frames; k += kFillThreads) sm.live[k] = frames[frame0 + k];
    stage_stack_header(sm, stack_hdrs + (size_t)rd.stack_begin * hdr_stride, c0, c1);
    if (fa.pair_tables != nullptr && (rd.pair_mask & 1u)) {  // the first stack's two-byte table, computed ahead
      const XGM_GLOBAL uint32_t* table = (const XGM_GLOBAL uint32_t*)fa.pair_tables + (size_t)b * kBatchMaxStacks * kPairWords;
      for (uint32_t k = tid; k < kPairWords; k += kFillThreads) sm.pair[k] = table[k];
    }
  }
  // 1. accepted words
  const XGM_GLOBAL uint32_t* acc = (const XGM_GLOBAL uint32_t*)rd.acc;
  for (int32_t w = tid; w < n_words; w += kFillThreads) {
    uint32_t x = 0u;
    for (uint32_t s = 0; s < rd.n_stacks; ++s) {
      const uint32_t acc_row = stack_hdrs[(size_t)(rd.stack_begin + s) * hdr_stride + kStackHdrTop] >> 16;
      x |= acc[(size_t)acc_row * voc.W + w_begin + w];
    }
    sm.words[w] = x;
  }
  if (tid == 0) sm.queue_n = 0u;
  __syncthreads();
  if (may_end) {
    for (int32_t k = tid; k < voc.n_stop; k += kFillThreads) {
      const int32_t rel = (k == (int32_t)tid ? my_stop : voc.stop_ids[k]) - w_begin * 32;
      if (rel >= 0 && rel < n_words * 32) atomicOr(&sm.words[rel >> 5], 1u << (rel & 31));
    }
    __syncthreads();  // a stop token with bytes may also be listed: the lists must find its bit set
  }
  // this workgroup's logits: its chunks; the last workgroup of a row also takes the columns beyond the vocabulary
  LogitsRange<APPLY> logits;
  if (APPLY != 0) {
    logits.row = fa.logits + (size_t)b * fa.row_stride * APPLY;
    logits.words = sm.words;
    logits.e_begin = w_begin * 32;
    logits.e_end = c1 == voc.n_chunk ? fa.V_logits : min(c1 * kChunkTokens, fa.V_logits);
    logits.V = voc.V;
    logits.V_logits = fa.V_logits;
    logits.neg_inf = fa.neg_inf;
  }
  bool logits_done = false;
  if (has_cache) {
    if (small_sections_staged(rd.tab))
      logits_done = fill_lists<COUNT, APPLY>(LdsTabT<true>(rd.tab, smem), sm, rd, b, c0, c1, frame0, frames_in_lds,
                                             stack_hdrs, frames, voc, log, seq, my_steps, fa.pair_min_entries,
                                             (const XGM_GLOBAL uint32_t*)fa.pair_tables, logits);
    else
      logits_done = fill_lists<COUNT, APPLY>(LdsTab(rd.tab, smem), sm, rd, b, c0, c1, frame0, frames_in_lds, stack_hdrs,
                                             frames, voc, log, seq, my_steps, fa.pair_min_entries,
                                             (const XGM_GLOBAL uint32_t*)fa.pair_tables, logits);
  }
  __syncthreads();
  for (int32_t w = tid; w < n_words; w += kFillThreads) out[(size_t)b * voc.W + w_begin + w] = sm.words[w];
  if (!logits_done) logits.groups(tid, kFillThreads);
  if (COUNT && my_steps) atomicAdd(step_counter, my_steps);
}


// ------------------------------------------------- device-resident states
// Candidate stacks of one row in LDS (see CollectStacks).
struct LdsStackSink {
  uint16_t* frames;
  uint32_t* depth;
  uint32_t* count;
  uint32_t* overflow;
  uint32_t capacity, max_depth;
  __device__ __forceinline__ uint32_t claim() { return atomicAdd(count, 1u); }
};

constexpr int kAcceptThreads = 256;
constexpr int kErrTokenRejected = -6, kErrTerminated = -7, kErrTooManyStacks = -8, kErrTooLarge = -9, kErrBadArg = -1;

// is stack a (depth da) ordered before stack b?  element by element, the shorter first (the host's order of stacks)
__device__ __forceinline__ int compare_stacks(const uint16_t* a, uint32_t da, const uint16_t* b, uint32_t db) {
  const uint32_t m = da < db ? da : db;
  for (uint32_t k = 0; k < m; ++k)
    if (a[k] != b[k]) return a[k] < b[k] ? -1 : 1;
  return da == db ? 0 : (da < db ? -1 : 1);
}

// Section 3.3 on the device: one workgroup per row moves the row's stacks on
// by the row's token.  Lane s of the first wave walks the token from stack s
// and writes out every stack it can end in; duplicates are removed, the rest
// is put in the host's order and packed as the next state of the row's ring,
// in the layout the fill kernel reads (stack headers with their first-byte
// sets, context index and list offsets; frames).  A row whose token is not
// allowed, or whose new state does not fit the device limits, keeps its state
// and gets an error code in `status`.
__global__ __launch_bounds__(kAcceptThreads) void batch_accept_kernel(DevBatch bt, DevVocab voc,
                                                                      const int32_t* __restrict__ tokens) {
  __shared__ uint16_t cand[kBatchMaxCandidates * kBatchMaxDepth];
  __shared__ uint32_t cdepth[kBatchMaxCandidates];
  __shared__ uint32_t order[kBatchMaxCandidates];  // rank among the distinct stacks, or kNoRow for a duplicate
  __shared__ uint32_t foff[kBatchMaxStacks + 1];
  __shared__ uint32_t slot_of[kBatchMaxStacks];    // candidate index per rank
  __shared__ uint32_t ccount, coverflow, n_new, can_end;
  const uint32_t tid = threadIdx.x;
  const int32_t b = blockIdx.x;
  const int32_t tok = tokens[b];
  if (tok < 0) return;  // this row is left alone (its status too)
  const int32_t head = bt.head[b];
  const SlotMeta cur = bt.meta[(size_t)b * bt.H + head];
  const DevCache dc = bt.cache[b];
  const uint32_t hdr_stride = kStackHdrWords + (uint32_t)bt.n_chunk + 1u;
  const int32_t next = (head + 1) % bt.H;
  const uint32_t sb = ((uint32_t)b * bt.H + next) * kBatchMaxStacks;
  const uint32_t fb = ((uint32_t)b * bt.H + next) * kBatchRowFrames;
  int32_t status = 0;
  bool stop = false;
  if (tok >= voc.V) status = kErrBadArg;
  else if (cur.flags & 2u) status = kErrTerminated;
  else {
    for (int32_t k = 0; k < voc.n_stop; ++k) stop = stop || voc.stop_ids[k] == tok;
    if (stop && !(cur.flags & 1u)) status = kErrTokenRejected;
  }
  if (status != 0) {
    if (tid == 0) bt.status[b] = status;
    return;
  }
  if (tid == 0) { ccount = 0u; coverflow = 0u; n_new = 0u; can_end = 0u; }
  __syncthreads();
  DevTables tab = dc.tab;
  tab.lds_end = tab.stage_bytes = tab.n_near = 0u;  // the walks read the tables where they are
  const LdsTab T(tab, nullptr);
  if (!stop) {
    const uint4 tk = voc.tok_by_id[tok];
    int len = (int)(tk.w >> 24);
    const uint8_t* ext = voc.bytes;
    if (len >= 15) {
      ext = voc.bytes + voc.off_by_id[tok];
      if (len == 255) len = (int)(voc.off_by_id[tok + 1] - voc.off_by_id[tok]);
    }
    if (len == 0) {
      if (tid == 0) bt.status[b] = kErrTokenRejected;
      return;
    }
    if (tid < cur.n_stacks) {
      const uint32_t* h = bt.hdrs + (size_t)(((uint32_t)b * bt.H + head) * kBatchMaxStacks + tid) * hdr_stride;
      const uint16_t* fr = bt.frames + h[kStackHdrFrames];
      LdsStackSink sink{cand, cdepth, &ccount, &coverflow, kBatchMaxCandidates, kBatchMaxDepth};
      const CollectStacks<LdsTab, LdsStackSink> collect{&T, &sink};
      const int res = walk_token<false>(T, tk, ext, len, h[kStackHdrTop] & 0xFFFFu, fr, h[kStackHdrDepth], (uint32_t*)nullptr,
                                        (const uint32_t*)nullptr, 0, (uint32_t*)nullptr, collect);
      if (res == kOverflow) coverflow = 1u;
    }
    __syncthreads();
    if (coverflow || ccount > kBatchMaxCandidates) status = kErrTooLarge;
    else if (ccount == 0u) status = kErrTokenRejected;
    if (status != 0) {
      if (tid == 0) bt.status[b] = status;
      return;
    }
    const uint32_t nc = ccount;
    // duplicates out, the rest in order
    if (tid < nc) {
      bool dup = false;
      for (uint32_t j = 0; j < tid; ++j)
        dup = dup || compare_stacks(cand + j * kBatchMaxDepth, cdepth[j], cand + tid * kBatchMaxDepth, cdepth[tid]) == 0;
      order[tid] = dup ? kNoRow : 0u;
      if (!dup) atomicAdd(&n_new, 1u);
    }
    __syncthreads();
    uint32_t before = 0u;
    if (tid < nc && order[tid] != kNoRow)
      for (uint32_t j = 0; j < nc; ++j)
        if (j != tid && order[j] != kNoRow &&
            compare_stacks(cand + j * kBatchMaxDepth, cdepth[j], cand + tid * kBatchMaxDepth, cdepth[tid]) < 0)
          ++before;
    __syncthreads();
    if (tid < nc && order[tid] != kNoRow) order[tid] = before;
    __syncthreads();
    if (n_new > kBatchMaxStacks) {
      if (tid == 0) bt.status[b] = kErrTooManyStacks;
      return;
    }
    if (tid < nc && order[tid] != kNoRow) slot_of[order[tid]] = tid;
    __syncthreads();
    if (tid == 0) {
      uint32_t run = 0;
      for (uint32_t r = 0; r < n_new; ++r) { foff[r] = run; run += cdepth[slot_of[r]]; }
      foff[n_new] = run;
    }
    __syncthreads();
    const uint32_t ns = n_new;
    // frames
    for (uint32_t r = 0; r < ns; ++r) {
      const uint32_t ci = slot_of[r], d = cdepth[ci];
      for (uint32_t k = tid; k < d; k += kAcceptThreads) bt.frames[fb + foff[r] + k] = cand[ci * kBatchMaxDepth + k];
    }
    // headers: scalars, context index, whether the stack can end the text
    if (tid < ns) {
      const uint32_t ci = slot_of[tid], d = cdepth[ci];
      const uint16_t* st = cand + ci * kBatchMaxDepth;
      uint32_t* h = bt.hdrs + (size_t)(sb + tid) * hdr_stride;
      const uint32_t top = st[d - 1];
      h[kStackHdrTop] = top | ((uint32_t)dc.acc_row[top] << 16);
      h[kStackHdrDepth] = d;
      h[kStackHdrFrames] = fb + foff[tid];
      uint32_t ctx = kCtxNone;
      if (d >= 2u) {
        const uint32_t rule = T.header(top).y >> 16, below = st[d - 2];
        for (uint32_t i = dc.ctx_off[rule]; i < dc.ctx_off[rule + 1]; ++i)
          if (dc.ctx_node[i] == below) ctx = i - dc.ctx_off[rule];
      }
      h[kStackHdrCtx] = ctx;
      bool all_final = true;
      for (uint32_t k = 0; k < d; ++k) all_final = all_final && T.is_final(st[k]);
      if (all_final) can_end = 1u;
    }
    // headers: the two first-byte sets, one thread per (stack, set, word)
    for (uint32_t item = tid; item < ns * 16u; item += kAcceptThreads) {
      const uint32_t r = item >> 4, below = (item >> 3) & 1u, w = item & 7u;
      const uint32_t ci = slot_of[r], d = cdepth[ci];
      const uint16_t* st = cand + ci * kBatchMaxDepth;
      uint32_t acc = 0u;
      for (uint32_t k = d - below; k-- > 0u;) {
        acc |= *(const XGM_GLOBAL uint32_t*)(T.img + T.off_first + ((size_t)st[k] * 8u + w) * 4u);
        if (!T.is_final(st[k])) break;
      }
      bt.hdrs[(size_t)(sb + r) * hdr_stride + (below ? kStackHdrBelow : kStackHdrFirst) + w] = acc;
    }
    // headers: list offsets of the top node
    for (uint32_t item = tid; item < ns * ((uint32_t)bt.n_chunk + 1u); item += kAcceptThreads) {
      const uint32_t r = item / ((uint32_t)bt.n_chunk + 1u), c = item % ((uint32_t)bt.n_chunk + 1u);
      const uint32_t ci = slot_of[r], top = cand[ci * kBatchMaxDepth + cdepth[ci] - 1u];
      bt.hdrs[(size_t)(sb + r) * hdr_stride + kStackHdrWords + c] = dc.unc_off[(size_t)top * ((uint32_t)bt.n_chunk + 1u) + c];
    }
    __syncthreads();
  }
  if (tid == 0) {
    SlotMeta m;
    m.n_stacks = stop ? 0u : n_new;
    m.n_frames = stop ? 0u : foff[n_new];
    m.flags = stop ? 3u : can_end;
    m.pad = 0u;
    bt.meta[(size_t)b * bt.H + next] = m;
    RowDesc r;
    r.tab = dc.tab;
    r.acc = dc.acc;
    r.unc_list = dc.unc_list;
    r.unc_ctx = dc.unc_ctx;
    r.stack_begin = sb;
    r.n_stacks = m.n_stacks;
    r.flags = m.flags & 1u;
    r.frame_begin = fb;
    r.n_frames = m.n_frames;
    r.pair_mask = 0u;
    bt.rows[b] = r;
    bt.head[b] = next;
    const int32_t o = bt.older[b] + 1;
    bt.older[b] = o < bt.H - 1 ? o : bt.H - 1;
    bt.status[b] = 0;
  }
}

// going back: one thread per row
__global__ void batch_rollback_kernel(DevBatch bt, const int32_t* __restrict__ steps) {
  const int32_t b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= bt.B) return;
  const int32_t k = steps[b];
  if (k <= 0) return;
  if (k > bt.older[b]) { bt.status[b] = kErrBadArg; return; }
  const int32_t head = ((bt.head[b] - k) % bt.H + bt.H) % bt.H;
  const SlotMeta m = bt.meta[(size_t)b * bt.H + head];
  RowDesc r = bt.rows[b];
  r.stack_begin = ((uint32_t)b * bt.H + head) * kBatchMaxStacks;
  r.frame_begin = ((uint32_t)b * bt.H + head) * kBatchRowFrames;
  r.n_stacks = m.n_stacks;
  r.n_frames = m.n_frames;
  r.flags = m.flags & 1u;
  r.pair_mask = 0u;
  bt.rows[b] = r;
  bt.head[b] = head;
  bt.older[b] -= k;
  bt.status[b] = 0;
}

// Forking (section 3.3: one state may be continued in several ways, as in tree
// decoding): row b takes over the current state of row src[b] as its next
// state.  All rows read the states as they were before the call: the first
// kernel only writes next slots, the second moves the rows over.
__global__ __launch_bounds__(256) void batch_fork_copy_kernel(DevBatch bt, const int32_t* __restrict__ src_rows) {
  const int32_t b = blockIdx.x;
  const int32_t src = src_rows[b];
  if (src < 0 || src == b) return;
  if (src >= bt.B || bt.cache[b].acc != bt.cache[src].acc) return;  // reported by the second kernel
  const uint32_t tid = threadIdx.x;
  const uint32_t hdr_stride = kStackHdrWords + (uint32_t)bt.n_chunk + 1u;
  const uint32_t from = (uint32_t)src * bt.H + bt.head[src], to = (uint32_t)b * bt.H + (bt.head[b] + 1) % bt.H;
  const SlotMeta m = bt.meta[from];
  const uint32_t* sh = bt.hdrs + (size_t)from * kBatchMaxStacks * hdr_stride;
  uint32_t* dh = bt.hdrs + (size_t)to * kBatchMaxStacks * hdr_stride;
  for (uint32_t k = tid; k < m.n_stacks * hdr_stride; k += 256u) {
    uint32_t v = sh[k];
    if (k % hdr_stride == kStackHdrFrames) v = v - from * kBatchRowFrames + to * kBatchRowFrames;
    dh[k] = v;
  }
  for (uint32_t k = tid; k < m.n_frames; k += 256u) bt.frames[(size_t)to * kBatchRowFrames + k] = bt.frames[(size_t)from * kBatchRowFrames + k];
  if (tid == 0) bt.meta[to] = m;
}
__global__ void batch_fork_commit_kernel(DevBatch bt, const int32_t* __restrict__ src_rows) {
  const int32_t b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= bt.B) return;
  const int32_t src = src_rows[b];
  if (src < 0 || src == b) return;
  if (src >= bt.B || bt.cache[b].acc != bt.cache[src].acc) { bt.status[b] = kErrBadArg; return; }
  const int32_t next = (bt.head[b] + 1) % bt.H;
  const SlotMeta m = bt.meta[(size_t)b * bt.H + next];
  RowDesc r = bt.rows[b];
  r.stack_begin = ((uint32_t)b * bt.H + next) * kBatchMaxStacks;
  r.frame_begin = ((uint32_t)b * bt.H + next) * kBatchRowFrames;
  r.n_stacks = m.n_stacks;
  r.n_frames = m.n_frames;
  r.flags = m.flags & 1u;
  r.pair_mask = 0u;
  bt.rows[b] = r;
  bt.head[b] = next;
  const int32_t o = bt.older[b] + 1;
  bt.older[b] = o < bt.H - 1 ? o : bt.H - 1;
  bt.status[b] = 0;
}

// The plan of the next fill for the batch's current states (plan.hpp), by one
// workgroup: the per-(row, chunk) running entry counts go to LDS, then one
// thread per row cuts its row.
constexpr int kPlanThreads = 1024;
// `keep_cuts`: there is room behind the counts for every row's workgroups ([B][n_chunk] words), so
// that the rows are cut once; otherwise they are cut a second time when the plan is written.
__device__ __forceinline__ void batch_plan_body(const DevBatch& bt, unsigned char* smem, bool keep_cuts) {
  uint32_t* upto = reinterpret_cast<uint32_t*>(smem);  // [B][n_chunk + 1]
  __shared__ unsigned long long total;
  __shared__ uint32_t count[kPlanThreads / 64];  // per-wave sums of the rows' workgroup counts
  const uint32_t tid = threadIdx.x, n_off = (uint32_t)bt.n_chunk + 1u;
  const uint32_t stride = (n_off + 3u) & ~3u;  // rows of `upto` start on 16 bytes
  const uint32_t hdr_stride = kStackHdrWords + n_off;
  uint32_t* cuts = upto + (size_t)bt.B * stride;  // [B][n_chunk] the rows' workgroups (FillBlock::c0c1), if kept
  if (tid == 0) total = 0ull;
  {  // a few threads per row: the row's descriptor is read once, the reads of its offsets are under way together
    const uint32_t per_row = max(1u, (uint32_t)kPlanThreads / (uint32_t)bt.B), rows_at_once = (uint32_t)kPlanThreads / per_row;
    for (uint32_t b = tid / per_row; b < (uint32_t)bt.B; b += rows_at_once) {
      const uint32_t s0 = bt.rows[b].stack_begin, ns = bt.rows[b].n_stacks;
#pragma unroll 4
      for (uint32_t c = tid % per_row; c < stride; c += per_row) {
        uint32_t run = 0u;
        if (c < n_off)
          for (uint32_t s = 0; s < ns; ++s) {
            const uint32_t* off = bt.hdrs + (size_t)(s0 + s) * hdr_stride + kStackHdrWords;
            run += off[c] - off[0];
          }
        upto[b * stride + c] = run;
      }
    }
  }
  __syncthreads();
  {  // the batch's total: per-wave sums with lane shuffles, one 64-bit atomic per wave
    unsigned long long mine_total = tid < (uint32_t)bt.B ? (unsigned long long)upto[tid * stride + bt.n_chunk] : 0ull;
#pragma unroll
    for (uint32_t d = 32; d > 0; d >>= 1) mine_total += __shfl_down(mine_total, d, 64);
    if ((tid & 63u) == 0 && mine_total) atomicAdd(&total, mine_total);
  }
  __syncthreads();
  int32_t k = 0;
  // the row's running counts, read four at a time (the cuts are made by one thread per row, one chunk after
  // the other: what it waits for is these reads)
  const uint4* mine4 = reinterpret_cast<const uint4*>(upto + tid * stride);
  uint4 held = make_uint4(0u, 0u, 0u, 0u);
  int32_t held_at = -1;
  auto upto_of = [&](int32_t c) {
    if ((c >> 2) != held_at) {
      held_at = c >> 2;
      held = mine4[held_at];
    }
    const uint32_t lo = (c & 1) ? held.y : held.x, hi = (c & 1) ? held.w : held.z;
    return (uint64_t)((c & 2) ? hi : lo);
  };
  uint32_t my_count = 0u;
  if (tid < (uint32_t)bt.B) {
    k = plan_row_share(bt.B, bt.n_chunk, bt.budget, upto[tid * stride + bt.n_chunk], total);
    my_count = (uint32_t)plan_row((int32_t)tid, bt.n_chunk, k, upto_of, [&](int32_t made, const FillBlock& f) {
      if (keep_cuts) cuts[tid * (uint32_t)bt.n_chunk + (uint32_t)made] = f.c0c1;
    });
  }
  // inclusive scan of the rows' workgroup counts: inside each wave with lane shuffles, then over the 16 wave sums
  uint32_t incl = my_count;
  const uint32_t lane = tid & 63u, wave = tid >> 6;
#pragma unroll
  for (uint32_t d = 1; d < 64u; d <<= 1) {
    const uint32_t v = __shfl_up(incl, d, 64);
    if (lane >= d) incl += v;
  }
  if (lane == 63u) count[wave] = incl;
  __syncthreads();
  uint32_t before = 0u, n_blocks = 0u;
  for (uint32_t w = 0; w < (uint32_t)kPlanThreads / 64u; ++w) {
    const uint32_t c = count[w];
    if (w < wave) before += c;
    n_blocks += c;
  }
  const uint32_t first = before + incl - my_count;
  for (uint32_t j = tid; j < bt.plan_cap; j += kPlanThreads) bt.plan[j] = FillBlock{kNoRow, 0u};
  __syncthreads();
  if (tid < (uint32_t)bt.B && n_blocks <= bt.plan_cap) {
    if (keep_cuts)
      for (uint32_t i = 0; i < my_count; ++i)
        bt.plan[plan_slot(first + i, n_blocks)] = FillBlock{tid, cuts[tid * (uint32_t)bt.n_chunk + i]};
    else
      plan_row((int32_t)tid, bt.n_chunk, k, upto_of,
               [&](int32_t made, const FillBlock& f) { bt.plan[plan_slot(first + (uint32_t)made, n_blocks)] = f; });
  }
}

// Ahead of the next fill: the two-byte tables (see build_pair_table) of the
// stacks of rows whose state has changed, for stacks whose lists are long
// enough to make the fill kernel want one.  One workgroup per row; a row that
// has been examined since its last change is skipped.
constexpr int kPairThreads = kPlanThreads;  // the two share a launch
__device__ __forceinline__ void batch_pair_body(const DevBatch& bt, const DevVocab& voc, uint32_t pair_min_entries,
                                                int32_t b, unsigned char* smem) {
  __shared__ uint32_t pair[kPairWords];
  __shared__ uint16_t live_lds[kBatchMaxDepth];
  const uint32_t tid = threadIdx.x;
  const RowDesc rd = bt.rows[b];
  if (rd.pair_mask & 0x80000000u) return;
  const uint32_t hdr_stride = kStackHdrWords + (uint32_t)bt.n_chunk + 1u;
  uint32_t need = 0u;
  for (uint32_t s = 0; s < rd.n_stacks; ++s) {
    const uint32_t* h = bt.hdrs + (size_t)(rd.stack_begin + s) * hdr_stride;
    if (h[kStackHdrDepth] >= 2u && h[kStackHdrWords + bt.n_chunk] - h[kStackHdrWords] >= pair_min_entries) need |= 1u << s;
  }
  if (need) {
    stage_tables(rd.tab, smem, kPairThreads);
    __syncthreads();
    const uint32_t* node_first = reinterpret_cast<const uint32_t*>(reinterpret_cast<const unsigned char*>(rd.tab.image) + rd.tab.off_first);
    auto body = [&](const auto& T) {
      for (uint32_t s = 0; s < rd.n_stacks; ++s) {
        if (!((need >> s) & 1u)) continue;
        const uint32_t* h = bt.hdrs + (size_t)(rd.stack_begin + s) * hdr_stride;
        const uint32_t depth = h[kStackHdrDepth];
        const uint16_t* fr = bt.frames + h[kStackHdrFrames];
        for (uint32_t k = tid; k < depth; k += kPairThreads) live_lds[k] = fr[k];
        __syncthreads();
        LiveView live;
        live.lds = (const XGM_LDS uint16_t*)live_lds;
        live.glob = (const XGM_GLOBAL uint16_t*)fr;
        live.lo = 0u;
        build_pair_table<kPairThreads>(T, pair, h + kStackHdrBelow, (uint32_t)live_lds[depth - 2], live, depth, node_first, voc);
        uint32_t* out = bt.pair + ((size_t)b * kBatchMaxStacks + s) * kPairWords;
        for (uint32_t k = tid; k < kPairWords; k += kPairThreads) out[k] = pair[k];
        __syncthreads();
      }
    };
    if (small_sections_staged(rd.tab)) body(LdsTabT<true>(rd.tab, smem));
    else body(LdsTab(rd.tab, smem));
  }
  if (tid == 0) bt.rows[b].pair_mask = 0x80000000u | need;
}

// After a change of state: the plan of the next fill (one workgroup) and, beside it, the two-byte tables
// of the rows that want one (one workgroup per row).  Neither reads what the other writes.
__global__ __launch_bounds__(kPlanThreads) void batch_plan_pair_kernel(DevBatch bt, DevVocab voc, uint32_t pair_min_entries,
                                                                       bool keep_cuts) {
  extern __shared__ __align__(16) unsigned char smem[];
  if ((int32_t)blockIdx.x == bt.B) batch_plan_body(bt, smem, keep_cuts);
  else batch_pair_body(bt, voc, pair_min_entries, (int32_t)blockIdx.x, smem);
}

// ---------------------------------------------------------------- kernel (c)
constexpr int kApplyThreads = 256;

// Section 2.1: logits of disallowed tokens become -inf.  A thread owns one
// group: 16 bytes of a logits row (8 bf16/fp16 or 4 fp32 elements) with its
// mask bits; the 64 groups of a wave are contiguous (1 KiB); see apply_group.
// ESIZE = bytes per element.
template <int ESIZE>
__global__ __launch_bounds__(kApplyThreads) void apply_kernel(unsigned char* __restrict__ logits, int64_t row_stride,
                                                              const uint32_t* __restrict__ bitmask, int32_t W_mask,
                                                              int32_t V_logits, int32_t V_mask,
                                                              const int32_t* __restrict__ row_index, uint32_t neg_inf) {
  constexpr int EPT = 16 / ESIZE;            // elements per group
  constexpr uint32_t kAll = (1u << EPT) - 1u;
  const int32_t j = blockIdx.y;
  const int64_t lrow = row_index ? row_index[j] : j;
  const int32_t e0 = (blockIdx.x * kApplyThreads + threadIdx.x) * EPT;
  if (e0 >= V_logits) return;
  uint32_t mk = 0u;
  if (e0 < V_mask) {
    mk = (bitmask[(size_t)j * W_mask + (e0 >> 5)] >> (e0 & 31)) & kAll;
    if (e0 + EPT > V_mask) mk &= (1u << (V_mask - e0)) - 1u;
  }
  apply_group<ESIZE>(logits + ((size_t)lrow * row_stride + e0) * ESIZE, mk, e0, V_logits, neg_inf);
}

// any alignment, any stride: one element per thread
template <int ESIZE>
__global__ void apply_elementwise_kernel(unsigned char* __restrict__ logits, int64_t row_stride,
                                         const uint32_t* __restrict__ bitmask, int32_t W_mask, int32_t V_logits,
                                         int32_t V_mask, const int32_t* __restrict__ row_index, uint32_t neg_inf) {
  const int32_t j = blockIdx.y;
  const int64_t lrow = row_index ? row_index[j] : j;
  const int32_t e = blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= V_logits) return;
  bool allowed = false;
  if (e < V_mask) allowed = (bitmask[(size_t)j * W_mask + (e >> 5)] >> (e & 31)) & 1u;
  if (allowed) return;
  unsigned char* p = logits + ((size_t)lrow * row_stride + e) * ESIZE;
  if (ESIZE == 2) *reinterpret_cast<uint16_t*>(p) = (uint16_t)neg_inf;
  else *reinterpret_cast<uint32_t*>(p) = neg_inf;
}

// ------------------------------------------------------------ measurement aid
// Chains of dependent LDS reads with every wave slot of the device busy: the
// ceiling for the table lookups of the token walks (each step of a walk is a
// few such reads, each depending on the one before).
constexpr int kLookupThreads = 1024;
__global__ __launch_bounds__(kLookupThreads) void lds_lookup_kernel(uint32_t n_words, uint32_t hops, uint32_t* __restrict__ sink) {
  extern __shared__ __align__(16) unsigned char smem[];
  uint32_t* table = reinterpret_cast<uint32_t*>(smem);
  // a permutation with one long cycle: i -> (i * 5 + 1) mod n_words (n_words is a power of two)
  for (uint32_t k = threadIdx.x; k < n_words; k += kLookupThreads) table[k] = (k * 5u + 1u) & (n_words - 1u);
  __syncthreads();
  uint32_t at = (threadIdx.x * 97u + blockIdx.x) & (n_words - 1u);
  for (uint32_t h = 0; h < hops; ++h) at = table[at];
  if (at == 0xFFFFFFFFu) sink[0] = at;  // never true: keeps the chain alive
}

// ------------------------------------------------------------ static scratch
// Staging memory for the fill entry point that may not allocate: the per-step
// blob (row descriptors, stack headers, frames, plan) goes here instead of into
// a buffer from hipMalloc.  Each device holds its own copy of the array at its
// own address until the process ends.
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

}  // namespace

// In host code the array's name is only a stand-in for the symbol: its device
// address is looked up once per device, with that device current, and kept.
hipError_t static_scratch(void** out) {
  constexpr int kMaxDevices = 64;
  static void* ptr_of[kMaxDevices] = {};
  *out = nullptr;
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  if (!ptr_of[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    ptr_of[dev] = p;
  }
  *out = ptr_of[dev];
  return hipSuccess;
}

// ------------------------------------------------------------------ launchers
void launch_classify(const DevTables& tab, const DevVocab& voc, int32_t node0, int32_t n, uint32_t* acc_rank,
                     uint32_t* unc_rank, uint32_t* plain_rank, uint32_t* plain_count, OverflowLog* log, uint32_t seq,
                     hipStream_t stream) {
  if (n <= 0 || voc.V <= 0) return;
  const DevTables st = staged_for(tab, kClassifyLdsBudget);
  if (st.stage_bytes <= kClassifySmallStage) {
    const int32_t ny = (n + kNodesPerBlockSmall - 1) / kNodesPerBlockSmall;
    hipLaunchKernelGGL(classify_kernel<kClassifyThreadsSmall>,
                       dim3((voc.V + kClassifyThreadsSmall - 1) / kClassifyThreadsSmall, ny), dim3(kClassifyThreadsSmall),
                       st.stage_bytes, stream, st, voc, node0, n, acc_rank, unc_rank, plain_rank, plain_count, log, seq,
                       kNodesPerBlockSmall);
  } else {
    const int32_t ny = (n + kNodesPerBlockLarge - 1) / kNodesPerBlockLarge;
    hipLaunchKernelGGL(classify_kernel<kClassifyThreadsLarge>,
                       dim3((voc.V + kClassifyThreadsLarge - 1) / kClassifyThreadsLarge, ny), dim3(kClassifyThreadsLarge),
                       st.stage_bytes, stream, st, voc, node0, n, acc_rank, unc_rank, plain_rank, plain_count, log, seq,
                       kNodesPerBlockLarge);
  }
}

void launch_permute(const DevVocab& voc, int32_t n, const uint32_t* acc_rank, const uint32_t* unc_rank,
                    uint32_t* acc_id, uint32_t* unc_id, hipStream_t stream) {
  if (n <= 0) return;
  const size_t row_pair = (size_t)voc.WR * 8;  // LDS bytes per node
  int32_t per_block = (int32_t)std::min<size_t>(kPermuteNodes, std::max<size_t>(1, (size_t)(144 * 1024) / row_pair));
  // enough workgroups to fill the device before rows are grouped
  while (per_block > 1 && (n + per_block - 1) / per_block < 512) --per_block;
  hipLaunchKernelGGL(permute_kernel, dim3((n + per_block - 1) / per_block), dim3(kPermuteThreads),
                     row_pair * per_block, stream, voc, n, per_block, acc_rank, unc_rank, acc_id, unc_id);
}

void launch_hash_rows(const uint32_t* rows, int32_t n, int32_t W, unsigned long long* digest, hipStream_t stream) {
  if (n > 0) hipLaunchKernelGGL(hash_rows_kernel, dim3(n), dim3(kRowThreads), 0, stream, rows, W, digest);
}
void launch_rows_equal(const uint32_t* rows, int32_t n, int32_t W, const int32_t* rep, uint32_t* equal, hipStream_t stream) {
  if (n > 0) hipLaunchKernelGGL(rows_equal_kernel, dim3(n), dim3(kRowThreads), 0, stream, rows, W, rep, equal);
}
void launch_gather_rows(const uint32_t* rows, int32_t W, const int32_t* unique, int32_t n_unique, uint32_t* out,
                        hipStream_t stream) {
  if (n_unique > 0) hipLaunchKernelGGL(gather_rows_kernel, dim3(n_unique), dim3(kRowThreads), 0, stream, rows, W, unique, out);
}

void launch_count_uncertain(const DevVocab& voc, int32_t n, const uint32_t* unc_id, uint32_t* counts,
                            hipStream_t stream) {
  if (n <= 0) return;
  hipLaunchKernelGGL(count_uncertain_kernel, dim3(voc.n_chunk, n), dim3(kChunkWords), 0, stream, voc, unc_id, counts);
}

void launch_list_uncertain(const DevVocab& voc, int32_t n, const uint32_t* unc_id, const uint32_t* off,
                           uint32_t* list, hipStream_t stream) {
  if (n <= 0) return;
  hipLaunchKernelGGL(list_uncertain_kernel, dim3(voc.n_chunk, n), dim3(kChunkWords), 0, stream, voc, unc_id, off, list);
}

void launch_annotate_lists(const DevTables& tab, const DevVocab& voc, int32_t n, const uint32_t* off, uint32_t total,
                           uint32_t* list, uint32_t* list_ctx, const uint32_t* ctx_off, const uint16_t* ctx_node,
                           hipStream_t stream) {
  for (int32_t node0 = 0; node0 < n; node0 += 32768) {  // grid.y limit
    const int32_t nb = std::min(32768, n - node0);
    hipLaunchKernelGGL(annotate_lists_kernel, dim3(voc.n_chunk, nb), dim3(kAnnotateThreads), 0, stream,
                       staged_for(tab, 0), voc, node0, off, list);
  }
  if (total == 0) return;
  const DevTables st = staged_for(tab, kClassifyLdsBudget);
  hipLaunchKernelGGL(context_classes_kernel, dim3((total + kContextThreads - 1) / kContextThreads), dim3(kContextThreads),
                     st.stage_bytes, stream, st, voc, n, total, off, list, list_ctx, ctx_off, ctx_node);
}

void launch_patch_classes(const DevVocab& voc, const uint32_t* items, int32_t n_items, uint32_t* acc_rank,
                          uint32_t* unc_rank, uint32_t* plain_rank, hipStream_t stream) {
  if (n_items <= 0) return;
  hipLaunchKernelGGL(patch_classes_kernel, dim3((n_items + 255) / 256), dim3(256), 0, stream, voc, items, n_items,
                     acc_rank, unc_rank, plain_rank);
}

void launch_upload(const void* pinned_src, void* dst, size_t bytes, hipStream_t stream) {
  const uint32_t n16 = (uint32_t)((bytes + 15) / 16);
  if (n16 == 0) return;
  hipLaunchKernelGGL(upload_kernel, dim3((n16 + kUploadThreads - 1) / kUploadThreads), dim3(kUploadThreads), 0, stream,
                     reinterpret_cast<const uint4*>(pinned_src), reinterpret_cast<uint4*>(dst), n16);
}

void launch_fill(const RowDesc* rows, const uint32_t* stack_hdrs, const uint16_t* frames,
                 const FillBlock* plan, int32_t n_blocks, const DevVocab& voc, uint32_t* out, OverflowLog* log,
                 uint32_t seq, unsigned long long* step_counter, hipStream_t stream, void* logits, int elem_size,
                 uint32_t neg_inf, int32_t V_logits, int64_t row_stride, uint32_t pair_min_entries,
                 const uint32_t* pair_tables) {
  if (n_blocks <= 0 || n_blocks % kFillGridMultiple != 0) return;  // callers pad the plan with kNoRow entries
  const dim3 grid(n_blocks);
  const FusedApply fa{static_cast<unsigned char*>(logits), row_stride, V_logits, neg_inf, pair_min_entries, pair_tables};
  if (logits && elem_size == 2)
    hipLaunchKernelGGL((fill_kernel<false, 2>), grid, dim3(kFillThreads), kFillLdsBudget, stream, rows, stack_hdrs, frames,
                       plan, voc, out, log, seq, step_counter, fa);
  else if (logits)
    hipLaunchKernelGGL((fill_kernel<false, 4>), grid, dim3(kFillThreads), kFillLdsBudget, stream, rows, stack_hdrs, frames,
                       plan, voc, out, log, seq, step_counter, fa);
  else if (step_counter)
    hipLaunchKernelGGL((fill_kernel<true, 0>), grid, dim3(kFillThreads), kFillLdsBudget, stream, rows, stack_hdrs, frames,
                       plan, voc, out, log, seq, step_counter, fa);
  else
    hipLaunchKernelGGL((fill_kernel<false, 0>), grid, dim3(kFillThreads), kFillLdsBudget, stream, rows, stack_hdrs, frames,
                       plan, voc, out, log, seq, step_counter, fa);
}

void launch_lds_lookups(int32_t n_blocks, uint32_t hops, uint32_t* sink, hipStream_t stream) {
  hipLaunchKernelGGL(lds_lookup_kernel, dim3(n_blocks), dim3(kLookupThreads), 8192 * 4, stream, 8192u, hops, sink);
}

void launch_batch_plan(const DevBatch& bt, const DevVocab& voc, uint32_t pair_min_entries, hipStream_t stream) {
  size_t plan_bytes = (size_t)bt.B * ((bt.n_chunk + 1 + 3) & ~3) * 4;
  const size_t cuts_bytes = (size_t)bt.B * bt.n_chunk * 4;
  const bool keep_cuts = plan_bytes + cuts_bytes <= (size_t)64 * 1024;
  if (keep_cuts) plan_bytes += cuts_bytes;
  hipLaunchKernelGGL(batch_plan_pair_kernel, dim3(bt.B + 1), dim3(kPlanThreads), std::max<size_t>(plan_bytes, kFillLdsBudget),
                     stream, bt, voc, pair_min_entries, keep_cuts);
}

void launch_batch_accept(const DevBatch& bt, const DevVocab& voc, const int32_t* d_tokens, uint32_t pair_min_entries,
                         hipStream_t stream) {
  hipLaunchKernelGGL(batch_accept_kernel, dim3(bt.B), dim3(kAcceptThreads), 0, stream, bt, voc, d_tokens);
  launch_batch_plan(bt, voc, pair_min_entries, stream);
}

void launch_batch_fork(const DevBatch& bt, const DevVocab& voc, const int32_t* d_src_rows, uint32_t pair_min_entries,
                       hipStream_t stream) {
  hipLaunchKernelGGL(batch_fork_copy_kernel, dim3(bt.B), dim3(256), 0, stream, bt, d_src_rows);
  hipLaunchKernelGGL(batch_fork_commit_kernel, dim3((bt.B + 255) / 256), dim3(256), 0, stream, bt, d_src_rows);
  launch_batch_plan(bt, voc, pair_min_entries, stream);
}

void launch_batch_rollback(const DevBatch& bt, const DevVocab& voc, const int32_t* d_steps, uint32_t pair_min_entries,
                           hipStream_t stream) {
  hipLaunchKernelGGL(batch_rollback_kernel, dim3((bt.B + 255) / 256), dim3(256), 0, stream, bt, d_steps);
  launch_batch_plan(bt, voc, pair_min_entries, stream);
}

void launch_apply(void* logits, int elem_size, uint32_t neg_inf, int32_t V_logits, int64_t row_stride,
                  const uint32_t* bitmask, int32_t V_mask, const int32_t* row_index, int32_t n_rows,
                  hipStream_t stream) {
  if (n_rows <= 0 || V_logits <= 0) return;
  const int32_t W_mask = (V_mask + 31) / 32;
  const bool aligned = (reinterpret_cast<uintptr_t>(logits) % 16 == 0) && ((row_stride * elem_size) % 16 == 0);
  unsigned char* p = static_cast<unsigned char*>(logits);
  if (aligned) {
    const int ept = 16 / elem_size;
    const int32_t groups = (V_logits + ept - 1) / ept;
    const int32_t per_block = kApplyThreads;
    dim3 grid((groups + per_block - 1) / per_block, n_rows);
    if (elem_size == 2)
      hipLaunchKernelGGL(apply_kernel<2>, grid, dim3(kApplyThreads), 0, stream, p, row_stride, bitmask, W_mask,
                         V_logits, V_mask, row_index, neg_inf);
    else
      hipLaunchKernelGGL(apply_kernel<4>, grid, dim3(kApplyThreads), 0, stream, p, row_stride, bitmask, W_mask,
                         V_logits, V_mask, row_index, neg_inf);
  } else {
    dim3 grid((V_logits + 255) / 256, n_rows);
    if (elem_size == 2)
      hipLaunchKernelGGL(apply_elementwise_kernel<2>, grid, dim3(256), 0, stream, p, row_stride, bitmask, W_mask,
                         V_logits, V_mask, row_index, neg_inf);
    else
      hipLaunchKernelGGL(apply_elementwise_kernel<4>, grid, dim3(256), 0, stream, p, row_stride, bitmask, W_mask,
                         V_logits, V_mask, row_index, neg_inf);
  }
}

}  // namespace xgm
