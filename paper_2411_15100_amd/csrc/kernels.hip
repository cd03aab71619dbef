// HIP kernels for gfx950 (wave64): token walk / classify, rank->id permute,
// context-dependent lists, batched mask fill, -inf apply.
#include <hip/hip_runtime.h>

#include <algorithm>

#include "kernels.hpp"
#include "walk.hpp"

namespace xgm {

namespace {


__device__ __forceinline__ void record_overflow(OverflowLog* log, uint32_t seq, uint32_t a, uint32_t b, uint32_t epoch = 0u) {
  uint32_t slot = atomicAdd(&log->count, 1u) % OverflowLog::kCap;
  log->entry[slot][0] = seq;
  log->entry[slot][1] = a;
  log->entry[slot][2] = b;
  log->entry[slot][3] = epoch;
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
  // the rule of node n, as the handle of its 256-bit FOLLOW set; is byte c in the set of rule r?
  __device__ __forceinline__ uint32_t follow_of(uint32_t n) const { return header(n).y >> 16; }
  __device__ __forceinline__ uint32_t follows(uint32_t r, uint32_t c) const {
    return (rd32(off_follow + (r * 8u + (c >> 5)) * 4u, follow_lds) >> (c & 31)) & 1u;
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
constexpr int kNodesPerBlockSmall = 4, kNodesPerBlockMany = 16, kNodesPerBlockLarge = 64;
constexpr int kManyNodes = 1024;  // small tables but this many nodes: plenty of workgroups anyway

// One thread owns one token (byte-sorted order, so a wave's 64 tokens are
// neighbours in the sorted vocabulary and mostly share prefixes and control
// flow) and classifies it at several nodes, the token staying in
// registers.  Each wave packs its 64 results per node with a ballot into two
// mask words of the rank-space bitsets.  The automaton tables (as many node
// headers as `n_near`) are first copied into shared memory.
// What the first byte of a token settles at every node, as bitsets over the nodes: for byte c and the 32 nodes
// of word w, `x` = the node can consume c inside its frame (a walk decides), `y` = it cannot, may end its rule
// here and c can follow that rule in some context (the token leaves the frame at position 0:
// context-dependent), `z` = the same but c follows the rule in no context (context-dependent by section 3.1
// alone, rejected everywhere).  One 16-byte load then tells a thread of the classify kernel what its token's
// first byte means at 32 nodes.
constexpr int kFirstByteThreads = 256;
__global__ __launch_bounds__(kFirstByteThreads) void first_byte_kernel(DevTables tab, uint32_t n_words, uint4* __restrict__ out) {
  const uint32_t t = blockIdx.x * kFirstByteThreads + threadIdx.x;
  if (t >= 256u * n_words) return;
  const uint32_t c = t / n_words, w = t % n_words;
  const unsigned char* img = reinterpret_cast<const unsigned char*>(tab.image);
  const uint2* hdr = reinterpret_cast<const uint2*>(img + tab.off_hdr);
  const uint32_t* first = reinterpret_cast<const uint32_t*>(img + tab.off_first);
  const uint32_t* follow = reinterpret_cast<const uint32_t*>(img + tab.off_follow);
  uint4 q = make_uint4(0u, 0u, 0u, 0u);
  for (uint32_t j = 0; j < 32u; ++j) {
    const uint32_t n = w * 32u + j;
    if (n >= (uint32_t)tab.n_nodes) break;
    if ((first[(size_t)n * 8u + (c >> 5)] >> (c & 31)) & 1u) { q.x |= 1u << j; continue; }
    const uint2 h = hdr[n];
    if (!(h.y & 1u)) continue;
    if ((follow[(h.y >> 16) * 8u + (c >> 5)] >> (c & 31)) & 1u) q.y |= 1u << j;
    else q.z |= 1u << j;
  }
  out[t] = q;
}

template <int kClassifyThreads, class Tab>
__device__ __forceinline__ void classify_body(const Tab& T, const DevVocab& voc, int32_t node0, int32_t n_nodes,
                                              const uint4* __restrict__ first_byte, uint32_t n_words,
                                              uint32_t* __restrict__ acc_rank, uint32_t* __restrict__ unc_rank,
                                              uint32_t* __restrict__ plain_rank, uint32_t* __restrict__ plain_count,
                                              OverflowLog* log, uint32_t seq, int32_t nodes_per_block,
                                              int32_t items_per_wave, uint32_t* next_item) {
  // A workgroup owns a run of kClassifyThreads * items_per_wave tokens, cut into items of 64; its waves draw
  // items from a counter in LDS, so that none of them waits for the slowest walks of another (a workgroup keeps
  // its LDS, and so its place on the compute unit, until its last wave is done).
  const int32_t chunk0 = blockIdx.x * kClassifyThreads * items_per_wave;
  const int32_t n_items = min((kClassifyThreads / 64) * items_per_wave, (voc.V - chunk0 + 63) / 64);
  for (;;) {
  int32_t item = 0;
  if ((threadIdx.x & 63u) == 0u) item = (int32_t)atomicAdd(next_item, 1u);
  item = __builtin_amdgcn_readfirstlane(item);
  if (item >= n_items) break;
  const int32_t r = chunk0 + item * 64 + (int32_t)(threadIdx.x & 63u);
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
  const int32_t word = (chunk0 + item * 64) >> 5;  // even
  // Do all tokens of the wave begin with the same byte?  (In byte-sorted order most waves' do.)  Then what the
  // first byte settles at a node is the same for every lane, and the nodes that need no walk need no loop.
  const bool has = live_lane && len > 0;
  const unsigned long long has_mask = __ballot(has);
  const uint32_t c0 = tk.x & 0xFFu;
  const uint32_t c_wave = has_mask ? (uint32_t)__shfl((int)c0, __ffsll((long long)has_mask) - 1, 64) : 0u;
  const bool one_first_byte = has_mask != 0ull && __ballot(has && c0 == c_wave) == has_mask;
  const int32_t n_begin = blockIdx.y * nodes_per_block;
  const int32_t n_end = min(n_begin + nodes_per_block, n_nodes);
  // Most pairs are settled by the token's first byte: if the node cannot
  // consume it inside its frame, the token is rejected - or, at a node where
  // the rule may end, leaves the frame at position 0.  The nodes of a block lie in whole 32-node words of
  // the first-byte bitsets, or inside one (node0 and nodes_per_block are aligned for that).
  for (int32_t k0 = n_begin; k0 < n_end; k0 += 32) {
    uint4 fb = make_uint4(0u, 0u, 0u, 0u);
    if (live_lane && len > 0) fb = first_byte[(size_t)(tk.x & 0xFFu) * n_words + ((uint32_t)(node0 + k0) >> 5)];
    const uint32_t shift = (uint32_t)(node0 + k0) & 31u;
    const uint32_t needs_walk = fb.x >> shift, exits_follow = fb.y >> shift, exits_plain = fb.z >> shift;
    const int32_t k1 = min(k0 + 32 - (int32_t)shift, n_end);
    // Lane j of the wave keeps the wave's result words for the j-th of these nodes; the lanes then write
    // them out together (a handful of store instructions per 32 nodes instead of several per node).
    const uint32_t lane = threadIdx.x & 63u;
    unsigned long long keep_a = 0ull, keep_u = 0ull, keep_p = 0ull;
    if (one_first_byte) {
      // the lane's own node, settled by the first byte unless it is walked below
      const uint4 fbw = first_byte[(size_t)c_wave * n_words + ((uint32_t)(node0 + k0) >> 5)];  // (the same for the wave)
      const uint32_t span = k1 - k0 >= 32 ? 0xFFFFFFFFu : (1u << (k1 - k0)) - 1u;
      if (lane < 32u && (((fbw.y >> shift) >> lane) & 1u)) keep_u = has_mask;
      if (lane < 32u && (((fbw.z >> shift) >> lane) & 1u)) keep_p = has_mask;
      for (uint32_t todo = (fbw.x >> shift) & span; todo; todo &= todo - 1u) {
        const int32_t k = k0 + __ffs(todo) - 1;
        int res = kReject;
        if (has) {
          res = walk_token<true>(T, tk, ext, len, (uint32_t)(node0 + k), (const uint16_t*)nullptr, 1u, nullptr, T.follow_of(node0 + k));
          if (res == kOverflow) { record_overflow(log, seq, (uint32_t)k, (uint32_t)r); res = kReject; }
        }
        const unsigned long long a = __ballot(res == kAccept);
        const unsigned long long u = __ballot(res == kUncertain);
        const unsigned long long p = __ballot(res == kUncertainPlain);
        if (lane == (uint32_t)(k - k0)) { keep_a = a; keep_u = u; keep_p = p; }
      }
    } else
    for (int32_t k = k0; k < k1; ++k) {
      const uint32_t bit = 1u << (k - k0);
      int res = (exits_follow & bit) ? kUncertain : (exits_plain & bit) ? kUncertainPlain : kReject;
      if (needs_walk & bit) {
        res = walk_token<true>(T, tk, ext, len, (uint32_t)(node0 + k), (const uint16_t*)nullptr, 1u, nullptr, T.follow_of(node0 + k));
        if (res == kOverflow) { record_overflow(log, seq, (uint32_t)k, (uint32_t)r); res = kReject; }
      }
      const unsigned long long a = __ballot(res == kAccept);
      const unsigned long long u = __ballot(res == kUncertain);
      const unsigned long long p = __ballot(res == kUncertainPlain);
      if (lane == (uint32_t)(k - k0)) { keep_a = a; keep_u = u; keep_p = p; }
    }
    if ((int32_t)lane < k1 - k0 && word < voc.WR) {
      const size_t at = (size_t)(k0 + (int32_t)lane) * voc.WR + word;  // word is even: 8-byte aligned
      *reinterpret_cast<uint2*>(acc_rank + at) = make_uint2((uint32_t)keep_a, (uint32_t)(keep_a >> 32));
      *reinterpret_cast<uint2*>(unc_rank + at) = make_uint2((uint32_t)keep_u, (uint32_t)(keep_u >> 32));
      if (plain_rank) *reinterpret_cast<uint2*>(plain_rank + at) = make_uint2((uint32_t)keep_p, (uint32_t)(keep_p >> 32));
      if (keep_p) atomicAdd(&plain_count[node0 + k0 + (int32_t)lane], (uint32_t)__popcll(keep_p));
    }
  }
  }
}


template <int kClassifyThreads>
__global__ __launch_bounds__(kClassifyThreads) void classify_kernel(
    DevTables tab, DevVocab voc, int32_t node0, int32_t n_nodes, const uint4* __restrict__ first_byte, uint32_t n_words,
    uint32_t* __restrict__ acc_rank, uint32_t* __restrict__ unc_rank, uint32_t* __restrict__ plain_rank,
    uint32_t* __restrict__ plain_count, OverflowLog* log, uint32_t seq, int32_t nodes_per_block, int32_t items_per_wave) {
  extern __shared__ __align__(16) unsigned char smem[];
  __shared__ uint32_t next_item;
  if (threadIdx.x == 0) next_item = 0u;
  stage_tables(tab, smem, kClassifyThreads);
  __syncthreads();
  if (small_sections_staged(tab))
    classify_body<kClassifyThreads>(LdsTabT<true>(tab, smem), voc, node0, n_nodes, first_byte, n_words, acc_rank, unc_rank,
                                    plain_rank, plain_count, log, seq, nodes_per_block, items_per_wave, &next_item);
  else
    classify_body<kClassifyThreads>(LdsTab(tab, smem), voc, node0, n_nodes, first_byte, n_words, acc_rank, unc_rank,
                                    plain_rank, plain_count, log, seq, nodes_per_block, items_per_wave, &next_item);
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
constexpr int kMaxSegs = 128;  // segments of the largest vocabulary (XGM_MAX_VOCAB / kSegTokens), rounded up

// Rank space -> id space: bit id_of_rank[r] of the output = bit r of the input.  One workgroup per node builds
// the node's two id-space rows in LDS.  Rows are nearly empty (most nodes reject nearly every token) or nearly
// full (the inside of a string), so only the rarer kind of bit is moved: a row with few set bits starts as zeros
// and gets its set bits, one with many starts as ones and gets its zeros.  With the rows still in LDS the
// workgroup also takes their statistics (all three outputs may be null): set bits of the first row per segment,
// its digest, and the number of set bits of the second.
__global__ __launch_bounds__(kRowThreads) void permute_kernel(DevVocab voc, const uint32_t* __restrict__ a_rank,
                                                              const uint32_t* __restrict__ b_rank,
                                                              uint32_t* a_id, uint32_t* b_id,  // (may be the same row)
                                                              uint32_t* __restrict__ seg_counts,
                                                              unsigned long long* __restrict__ digest,
                                                              uint32_t* __restrict__ b_counts) {
  extern __shared__ __align__(16) unsigned char smem[];
  uint32_t* rows = reinterpret_cast<uint32_t*>(smem);  // [2][W]
  __shared__ uint32_t set_bits[2];
  __shared__ unsigned long long part[kRowThreads / 64];
  __shared__ uint32_t seg[kMaxSegs];
  const size_t node = blockIdx.x;
  const uint32_t* in[2] = {a_rank + node * voc.WR, b_rank + node * voc.WR};
  if (threadIdx.x < 2) set_bits[threadIdx.x] = 0u;
  if (threadIdx.x < kMaxSegs) seg[threadIdx.x] = 0u;
  __syncthreads();
  uint32_t c0 = 0u, c1 = 0u;
  for (int32_t k = threadIdx.x; k < voc.WR; k += kRowThreads) {
    c0 += __popc(in[0][k]);
    c1 += __popc(in[1][k]);
  }
  if (c0) atomicAdd(&set_bits[0], c0);
  if (c1) atomicAdd(&set_bits[1], c1);
  __syncthreads();
  const bool full[2] = {set_bits[0] * 2u > (uint32_t)voc.V, set_bits[1] * 2u > (uint32_t)voc.V};
  const uint32_t tail = (voc.V & 31) ? ((1u << (voc.V & 31)) - 1u) : 0xFFFFFFFFu;  // valid bits of the last word
  for (int32_t w = threadIdx.x; w < voc.W; w += kRowThreads) {
    const uint32_t ones = (w == voc.W - 1) ? tail : 0xFFFFFFFFu;
    rows[w] = full[0] ? ones : 0u;
    rows[voc.W + w] = full[1] ? ones : 0u;
  }
  __syncthreads();
#pragma unroll
  for (int which = 0; which < 2; ++which) {
    uint32_t* row = rows + (size_t)which * voc.W;
    for (int32_t k = threadIdx.x; k < voc.WR; k += kRowThreads) {
      uint32_t x = in[which][k];
      if (full[which]) {
        x = ~x;
        const int32_t left = voc.V - k * 32;  // ranks from V on do not exist
        if (left < 32) x &= left > 0 ? ((1u << left) - 1u) : 0u;
      }
      while (x) {
        const uint32_t b = (uint32_t)__ffs((int)x) - 1u;
        x &= x - 1u;
        const uint32_t id = (uint32_t)voc.id_of_rank[k * 32 + (int32_t)b];
        if (full[which]) atomicAnd(&row[id >> 5], ~(1u << (id & 31)));
        else atomicOr(&row[id >> 5], 1u << (id & 31));
      }
    }
  }
  __syncthreads();
  unsigned long long h = 0ull;
  for (int32_t w = threadIdx.x; w < voc.W; w += kRowThreads) {
    const uint32_t x = rows[w];
    a_id[node * voc.W + w] = x;
    b_id[node * voc.W + w] = rows[voc.W + w];
    if (seg_counts && x) atomicAdd(&seg[w / kSegWords], (uint32_t)__popc(x));
    h += mix64(((unsigned long long)(uint32_t)w << 32 | x) + 0x9E3779B97F4A7C15ull);
  }
  if (!seg_counts) return;
#pragma unroll
  for (uint32_t d = 32; d > 0; d >>= 1) h += __shfl_down(h, d, 64);
  if ((threadIdx.x & 63u) == 0) part[threadIdx.x >> 6] = h;
  __syncthreads();
  if ((int32_t)threadIdx.x < voc.n_seg) seg_counts[node * voc.n_seg + threadIdx.x] = seg[threadIdx.x];
  if (threadIdx.x == 0) {
    unsigned long long t = 0ull;
    for (int k = 0; k < kRowThreads / 64; ++k) t += part[k];
    digest[node] = t;
    b_counts[node] = set_bits[1];
  }
}

// Bitset rows (row_words words each) -> lists through cursors.  One workgroup per (segment, row); a thread
// takes four words; a wave reserves room for all its tokens with one atomic.  What is listed for bit v is
// map[v] if a map is given (rank-space rows: the token ids, in byte-sorted order within a segment), else v.
constexpr int kListThreads = kSegWords / 4;
__global__ __launch_bounds__(kListThreads) void rows_to_lists_kernel(const uint32_t* __restrict__ rows, int32_t row_words,
                                                                     const int32_t* __restrict__ map,
                                                                     const uint32_t* __restrict__ cursor_of, int32_t per_row,
                                                                     uint32_t* __restrict__ cursor, uint32_t* __restrict__ out,
                                                                     uint16_t* __restrict__ out_row, int32_t row0) {
  const size_t r = blockIdx.y;
  const uint32_t key = cursor_of[r];
  if (key == kNoKey) return;
  const int32_t s = blockIdx.x;
  const int32_t w0 = s * kSegWords + (int32_t)threadIdx.x * 4;
  uint32_t bits[4];
  uint32_t n = 0u;
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    bits[k] = w0 + k < row_words ? rows[r * (size_t)row_words + w0 + k] : 0u;
    n += __popc(bits[k]);
  }
  // exclusive prefix of n over the wave, and the wave's total
  const uint32_t lane = threadIdx.x & 63u;
  uint32_t incl = n;
#pragma unroll
  for (uint32_t d = 1; d < 64u; d <<= 1) {
    const uint32_t v = __shfl_up(incl, d, 64);
    if (lane >= d) incl += v;
  }
  const uint32_t total = __shfl(incl, 63, 64);
  if (total == 0u) return;
  uint32_t base = 0u;
  if (lane == 0) base = atomicAdd(&cursor[(size_t)key * per_row + (per_row > 1 ? s : 0)], total);
  base = __shfl(base, 0, 64);
  uint32_t pos = base + incl - n;
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    uint32_t x = bits[k];
    while (x) {
      const uint32_t b = __ffs(x) - 1;
      x &= x - 1;
      if (out_row) out_row[pos] = (uint16_t)(row0 + (int32_t)r);
      const uint32_t v = (uint32_t)(w0 + k) * 32u + b;
      out[pos++] = map ? (uint32_t)map[v] : v;
    }
  }
}

// the first 15 bytes, the length and the remaining bytes of token `id`
struct TokenRef {
  uint4 tk;
  const uint8_t* ext;
  int len;
};
__device__ __forceinline__ TokenRef load_token(const DevVocab& voc, int32_t id) {
  TokenRef t;
  t.tk = voc.tok_by_id[id];
  t.len = (int)(t.tk.w >> 24);
  t.ext = voc.bytes;
  if (t.len >= 15) {
    t.ext = voc.bytes + voc.off_by_id[id];
    if (t.len == 255) t.len = (int)(voc.off_by_id[id + 1] - voc.off_by_id[id]);
  }
  return t;
}

// ---- The per-context lists (section 3.2 per call site; see DevCache), from the base lists: the
// context-dependent (node, token) pairs.  Kernels, tables staged as in the classify kernel:
//   exit_positions_kernel  one thread per pair: the token is walked once more from the node to find the
//                          positions at which it leaves the node's frame;
//   context_level1_kernel  one thread per (pair, a few contexts of the node's rule): the rest of the token is
//                          walked from the context node with nothing known below.  Accepted there: an entry
//                          of the (node, context) list.  Leaves that frame too: a record for the next level;
//   context_deeper_kernel  for level 2, 3, ...: one thread per (record of the level above, a few contexts of
//                          the rule of that record's context node): the same one frame further down; what
//                          leaves a frame beyond the last level becomes a walk entry.
// Most (pair, context) combinations end at the first byte of the rest, which the context node cannot
// take.  All but the first kernel run twice: first they count the entries of every (key, segment), then,
// with the offsets made from the counts, they write them.
constexpr int kContextThreads = 768;
constexpr uint32_t kContextsPerThread = 8;

__global__ __launch_bounds__(kContextThreads) void exit_positions_kernel(DevTables tab, DevVocab voc, ContextListArgs a) {
  extern __shared__ __align__(16) unsigned char smem[];
  stage_tables(tab, smem, kContextThreads);
  __syncthreads();
  auto body = [&](const auto& T) {
    const uint32_t e = blockIdx.x * kContextThreads + threadIdx.x;
    if (e >= a.total) return;
    const uint32_t node = a.base_node[e];
    const TokenRef t = load_token(voc, (int32_t)a.base_ids[e]);
    uint32_t x = 0u;
    const int res = walk_token<true>(T, t.tk, t.ext, t.len, node, (const uint16_t*)nullptr, 1u, nullptr, T.follow_of(node), 0, &x);
    a.exits[e] = res == kOverflow ? 0x80000000u : x;
  };
  if (small_sections_staged(tab)) body(LdsTabT<true>(tab, smem));
  else body(LdsTab(tab, smem));
}

// How an entry reaches its list, counting or writing.
template <bool WRITE>
struct ListSink {
  const DevVocab& voc;
  const ContextListArgs& a;
  // One entry for list `key`.  The lanes of a wave that get here together mostly add to the same list (they hold
  // neighbouring tokens of one node and look at the same context): they are served by one atomic per
  // distinct (list, segment, accepted or not) among them instead of one each - atomics on one address queue up.
  __device__ __forceinline__ void emit(uint32_t id, uint32_t key, uint32_t kind, uint32_t pos) const {
    const uint32_t slot = key * (uint32_t)voc.n_seg + id / (uint32_t)kSegTokens;
    const uint32_t tag = (slot << 1) | (kind == kEntryAccepted ? 0u : 1u);
    const uint32_t lane = threadIdx.x & 63u;
    for (bool pending = true; pending;) {
      const uint32_t lead = __builtin_amdgcn_readfirstlane(tag);
      const bool mine = tag == lead;
      const unsigned long long peers = __ballot(mine);
      if (mine) {
        const uint32_t n = (uint32_t)__popcll(peers), rank = (uint32_t)__popcll(peers & ((1ull << lane) - 1ull));
        const int first = __ffsll((long long)peers) - 1;
        if (!WRITE) {
          if (rank == 0u) atomicAdd(&a.counts[slot], n);
        } else {
          uint32_t base = 0u;
          if (rank == 0u) base = kind == kEntryAccepted ? atomicAdd(&a.front[slot], n) : atomicSub(&a.back[slot], n) - n;
          base = __shfl(base, first, 64);
          a.entries[base + rank] = id | (pos << kEntryPosShift) | (kind << kEntryKindShift);
        }
        pending = false;
      }
    }
  }
};
__device__ __forceinline__ uint32_t outcome_code(uint32_t kind, uint32_t pos) { return (kind + 1u) | (pos << 8); }

// What the list kernels share: the token of one pair, how its entries reach the lists, and one (pair,
// context) step: the rest of the token after it has left the frame above at the positions `ex`, walked
// from context node r.
template <bool WRITE, class Tab>
struct ContextWork {
  const Tab& T;
  const DevVocab& voc;
  const ContextListArgs& a;
  uint32_t e, id;
  TokenRef t;
  // (`outcome`, if not null, also receives what was emitted, as a code; `lds_counts`, if not null, are the
  // workgroup's own counters per segment for this list: the entry is then only counted there)
  __device__ __forceinline__ void emit(uint32_t key, uint32_t kind, uint32_t pos, uint32_t* outcome,
                                       uint32_t* lds_counts) const {
    if (!WRITE && lds_counts) atomicAdd(&lds_counts[id / (uint32_t)kSegTokens], 1u);
    else ListSink<WRITE>{voc, a}.emit(id, key, kind, pos);
    if (outcome) *outcome = outcome_code(kind, pos);
  }
  // can the rest of the token from position k on do anything at all at node r?  (its first byte is
  // consumed there, or r may end its rule in front of a byte that can follow the rule)
  __device__ __forceinline__ bool plausible(uint32_t r, uint32_t k) const {
    const uint32_t c = token_byte(t.tk, t.ext, (int)k);
    if (T.can_start(r, c)) return true;
    const uint2 h = T.header(r);
    return (h.y & 1u) && T.can_follow(h, c);
  }
  // Level `level` (1-based), context node r, whose key is `key_local` among its level's keys.  `single`:
  // every frame so far was left at exactly one position.
  __device__ __forceinline__ void step(uint32_t level, uint32_t r, uint32_t key_local, uint32_t ex, bool single,
                                       uint32_t* outcome = nullptr, uint32_t* lds_counts = nullptr) const {
    const uint32_t key = a.key0[level - 1u] + key_local;
    // how a token that needs the live stack after all is listed here: from the frame of r on, if the way there is unique
    const uint32_t walk_kind = single ? kEntryWalkTop + level : kEntryWalkTop;
    const uint32_t walk_pos = single ? (uint32_t)__ffs(ex) - 1u : 0u;
    if (ex & 0x80000000u) { emit(key, kEntryWalkTop, 0u, outcome, lds_counts); return; }
    bool accepted = false, over = false;
    uint32_t ex_next = 0u, n_res = 0u;
    for (uint32_t m = ex; m != 0u && !accepted; m &= m - 1u) {
      const uint32_t k = __ffs(m) - 1u;
      if (!plausible(r, k)) continue;
      uint32_t x = 0u;
      const int res = walk_token<true>(T, t.tk, t.ext, t.len, r, (const uint16_t*)nullptr, 1u, nullptr, T.follow_of(r), (int)k, &x);
      if (res == kAccept) accepted = true;
      else if (res == kOverflow) over = true;
      else if (res == kUncertain) { ex_next |= x; ++n_res; }
    }
    if (accepted) { emit(key, kEntryAccepted, 0u, outcome, lds_counts); return; }
    if (over) { emit(key, kEntryWalkTop, 0u, outcome, lds_counts); return; }
    if (ex_next == 0u) return;  // rejected in this context
    if (level == (uint32_t)kCtxLevels || a.k_base[level] == nullptr || (ex_next & 0x80000000u)) {
      emit(key, walk_kind, walk_pos, outcome, lds_counts);
      return;
    }
    // It leaves this frame as well: records for the next level, one per chunk of kContextsPerThread contexts
    // of this context node's rule (a rule without contexts has nothing below it: the token ends there).
    // The lanes that get here together are taken rule by rule, each group with one atomic.
    const uint32_t rule = T.header(r).y >> 16;
    const uint32_t n_ch = (a.ctx_off[rule + 1] - a.ctx_off[rule] + kContextsPerThread - 1u) / kContextsPerThread;
    const bool single_next = single && n_res == 1u && (ex_next & (ex_next - 1u)) == 0u;
    const uint32_t lane = threadIdx.x & 63u;
    for (bool pending = true; pending;) {
      const uint32_t lead = __builtin_amdgcn_readfirstlane(rule);
      const bool mine = rule == lead;
      const unsigned long long peers = __ballot(mine);
      if (mine) {
        if (n_ch != 0u) {
          const uint32_t n = (uint32_t)__popcll(peers), rank = (uint32_t)__popcll(peers & ((1ull << lane) - 1ull));
          const int first = __ffsll((long long)peers) - 1;
          uint32_t base = 0u;
          if (rank == 0u) base = atomicAdd(&a.res_count[level - 1u], n * n_ch);
          base = __shfl(base, first, 64) + rank * n_ch;
          for (uint32_t ch = 0; ch < n_ch; ++ch)
            if (base + ch < a.res_cap)
              a.res[level - 1u][base + ch] = make_uint4(e, key_local, ex_next, rule | (single_next ? 0x10000u : 0u) | (ch << 17));
        }
        pending = false;
      }
    }
  }
};

// One workgroup per tile (see ContextListArgs::tiles): up to kContextThreads pairs of one node, up to
// kContextsPerThread contexts of its rule.  All entries of a tile go to the lists of those few contexts, so the
// counting pass counts them per (context, segment) in LDS and adds each counter to the global one once; the
// writing pass does the same to reserve room in every list and then hands out the places from LDS - the
// global counters of a list are touched once per workgroup instead of once per wave and segment.
constexpr uint32_t kTileCounters = kContextsPerThread * kMaxSegs;
template <bool WRITE, class Tab>
__device__ __forceinline__ void context_level1_body(const Tab& T, const DevVocab& voc, const ContextListArgs& a, const uint4 tile,
                                                    uint32_t* tile_counts) {
  const uint32_t node = tile.w, i0 = tile.z, i1 = tile.z + (tile.y >> 16);
  const uint32_t k1b = a.k_base[0][node];
  if (threadIdx.x < (tile.y & 0xFFFFu)) {
    const uint32_t e = tile.x + threadIdx.x;
    const uint32_t id = a.base_ids[e], ex0 = a.exits[e];
    const ContextWork<WRITE, Tab> w{T, voc, a, e, id, load_token(voc, (int32_t)id)};
    const uint32_t cb = a.ctx_off[T.header(node).y >> 16];
    const bool single0 = (ex0 & (ex0 - 1u)) == 0u;
    const bool keep = !WRITE && a.outcomes != nullptr;
    const uint4 info = keep ? a.node_info[node] : make_uint4(0u, 0u, 0u, 0u);
    for (uint32_t i = i0; i < i1; ++i) {
      uint32_t outcome = 0u;
      w.step(1u, a.ctx_node[cb + i], k1b + i, ex0, single0, keep ? &outcome : nullptr,
             WRITE ? nullptr : tile_counts + (i - i0) * (uint32_t)voc.n_seg);
      if (keep) a.outcomes[(size_t)info.x + (size_t)i * info.y + (e - info.z)] = (uint16_t)outcome;
    }
  }
  if (WRITE) return;
  __syncthreads();
  for (uint32_t t = threadIdx.x; t < (i1 - i0) * (uint32_t)voc.n_seg; t += kContextThreads) {
    const uint32_t n = tile_counts[t];
    if (n) atomicAdd(&a.counts[(a.key0[0] + k1b + i0 + t / (uint32_t)voc.n_seg) * (uint32_t)voc.n_seg + t % (uint32_t)voc.n_seg], n);
  }
}
template <bool WRITE>
__global__ __launch_bounds__(kContextThreads) void context_level1_kernel(DevTables tab, DevVocab voc, ContextListArgs a) {
  extern __shared__ __align__(16) unsigned char smem[];
  __shared__ uint32_t tile_counts[WRITE ? 1 : kTileCounters];
  const uint4 tile = a.tiles[blockIdx.x];
  if (!WRITE)
    for (uint32_t t = threadIdx.x; t < kTileCounters; t += kContextThreads) tile_counts[t] = 0u;
  stage_tables(tab, smem, kContextThreads);
  __syncthreads();
  if (small_sections_staged(tab)) context_level1_body<WRITE>(LdsTabT<true>(tab, smem), voc, a, tile, tile_counts);
  else context_level1_body<WRITE>(LdsTab(tab, smem), voc, a, tile, tile_counts);
}
// The writing pass of level 1 when the counting pass kept its outcomes: the same tiles, no walks, no tables.
__global__ __launch_bounds__(kContextThreads) void context_level1_write_kernel(DevVocab voc, ContextListArgs a) {
  __shared__ uint32_t next[2 * kTileCounters];   // per (context, segment, accepted or walk entry): entries, then places handed out
  __shared__ uint32_t base[2 * kTileCounters];   // where the workgroup's entries of that kind begin in the list
  const uint4 tile = a.tiles[blockIdx.x];
  const uint32_t node = tile.w, i0 = tile.z, n_ctx = tile.y >> 16, n_seg = (uint32_t)voc.n_seg;
  const uint32_t k1b = a.key0[0] + a.k_base[0][node] + i0;
  const bool active = threadIdx.x < (tile.y & 0xFFFFu);
  for (uint32_t t = threadIdx.x; t < 2u * n_ctx * n_seg; t += kContextThreads) next[t] = 0u;
  __syncthreads();
  uint32_t code[kContextsPerThread], id = 0u, seg = 0u;
  if (active) {
    const uint32_t e = tile.x + threadIdx.x;
    const uint4 info = a.node_info[node];
    id = a.base_ids[e];
    seg = id / (uint32_t)kSegTokens;
#pragma unroll
    for (uint32_t q = 0; q < kContextsPerThread; ++q) {
      code[q] = q < n_ctx ? a.outcomes[(size_t)info.x + (size_t)(i0 + q) * info.y + (e - info.z)] : 0u;
      if (code[q]) atomicAdd(&next[2u * (q * n_seg + seg) + ((code[q] & 0xFFu) - 1u == kEntryAccepted ? 0u : 1u)], 1u);
    }
  }
  __syncthreads();
  for (uint32_t t = threadIdx.x; t < 2u * n_ctx * n_seg; t += kContextThreads) {
    const uint32_t n = next[t];
    if (n) {
      const uint32_t slot = (k1b + (t >> 1) / n_seg) * n_seg + (t >> 1) % n_seg;
      base[t] = (t & 1u) ? atomicSub(&a.back[slot], n) - n : atomicAdd(&a.front[slot], n);
      next[t] = 0u;
    }
  }
  __syncthreads();
  if (active) {
#pragma unroll
    for (uint32_t q = 0; q < kContextsPerThread; ++q) {
      if (!code[q]) continue;
      const uint32_t kind = (code[q] & 0xFFu) - 1u, pos = code[q] >> 8;
      const uint32_t t = 2u * (q * n_seg + seg) + (kind == kEntryAccepted ? 0u : 1u);
      a.entries[base[t] + atomicAdd(&next[t], 1u)] = id | (pos << kEntryPosShift) | (kind << kEntryKindShift);
    }
  }
}

// Level `level` >= 2: a fixed grid walks over the records of level - 1, each of which names a chunk of
// kContextsPerThread contexts; consecutive threads hold consecutive records (neighbouring tokens of one
// node and context, as a rule).
template <bool WRITE, class Tab>
__device__ __forceinline__ void context_deeper_body(const Tab& T, const DevVocab& voc, const ContextListArgs& a, uint32_t level) {
  const uint32_t n_res = min(a.res_count[level - 2u], a.res_cap);
  for (uint32_t item = blockIdx.x * kContextThreads + threadIdx.x; item < n_res; item += gridDim.x * kContextThreads) {
    const uint4 rec = a.res[level - 2u][item];
    const uint32_t rule = rec.w & 0xFFFFu;
    const uint32_t cb = a.ctx_off[rule], m = a.ctx_off[rule + 1] - cb;
    const uint32_t j0 = (rec.w >> 17) * kContextsPerThread;
    const uint32_t id = a.base_ids[rec.x];
    const ContextWork<WRITE, Tab> w{T, voc, a, rec.x, id, load_token(voc, (int32_t)id)};
    const uint32_t kb = a.k_base[level - 1u][rec.y];
    uint4* keep = WRITE ? nullptr : a.deep_outcomes[level - 1u];
    static_assert(kContextsPerThread == 8, "a record's outcomes are eight 16-bit codes in one uint4");
    unsigned long long lo = 0ull, hi = 0ull;  // (the loop is not unrolled: one copy of the walk, not eight)
#pragma unroll 1
    for (uint32_t q = 0; q < kContextsPerThread; ++q) {
      const uint32_t j = j0 + q;
      if (j >= m) break;
      uint32_t outcome = 0u;
      w.step(level, a.ctx_node[cb + j], kb + j, rec.z, (rec.w & 0x10000u) != 0u, keep ? &outcome : nullptr);
      if (q < 4u) lo |= (unsigned long long)outcome << (q * 16u);
      else hi |= (unsigned long long)outcome << ((q - 4u) * 16u);
    }
    if (keep) keep[item] = make_uint4((uint32_t)lo, (uint32_t)(lo >> 32), (uint32_t)hi, (uint32_t)(hi >> 32));
  }
}
template <bool WRITE>
__global__ __launch_bounds__(kContextThreads) void context_deeper_kernel(DevTables tab, DevVocab voc, ContextListArgs a, uint32_t level) {
  extern __shared__ __align__(16) unsigned char smem[];
  if (a.res_count[level - 2u] == 0u) return;
  stage_tables(tab, smem, kContextThreads);
  __syncthreads();
  if (small_sections_staged(tab)) context_deeper_body<WRITE>(LdsTabT<true>(tab, smem), voc, a, level);
  else context_deeper_body<WRITE>(LdsTab(tab, smem), voc, a, level);
}

// The writing pass of a deeper level when the counting pass kept its outcomes: the same records, no walks, no tables.
__global__ __launch_bounds__(256) void context_deeper_write_kernel(DevVocab voc, ContextListArgs a, uint32_t level) {
  const uint32_t n_res = min(a.res_count[level - 2u], a.res_cap);
  const ListSink<true> sink{voc, a};
  for (uint32_t item = blockIdx.x * 256u + threadIdx.x; item < n_res; item += gridDim.x * 256u) {
    const uint4 c = a.deep_outcomes[level - 1u][item];
    if ((c.x | c.y | c.z | c.w) == 0u) continue;
    const uint4 rec = a.res[level - 2u][item];
    const uint32_t id = a.base_ids[rec.x];
    const uint32_t key = a.key0[level - 1u] + a.k_base[level - 1u][rec.y] + (rec.w >> 17) * kContextsPerThread;
    const uint32_t codes[4] = {c.x, c.y, c.z, c.w};
#pragma unroll
    for (uint32_t q = 0; q < kContextsPerThread; ++q) {
      const uint32_t code = (codes[q >> 1] >> ((q & 1u) * 16u)) & 0xFFFFu;
      if (code) sink.emit(id, key + q, (code & 0xFFu) - 1u, code >> 8);
    }
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
// allowed: nothing is touched.  None allowed: one 16-byte streaming store of the
// -inf pattern.  Both kinds: every disallowed element is stored by itself.  The
// logits are never read: a group that is fetched, blended and stored whole makes
// its wave wait for the fetch, while stores are issued and forgotten (measured
// on the serving masks, where four rows in ten allow nearly every token and the
// others nearly none: 15.6 -> 13.5 us for the one-launch step and 7.9 -> 7.5 us
// for the stand-alone kernel against blending; merging neighbouring elements
// into 4-byte stores, or streaming stores for single elements, were slower).
template <int ESIZE>
__device__ __forceinline__ void apply_group(unsigned char* p, uint32_t mk, int32_t e0, int32_t V_logits, uint32_t neg_inf) {
  constexpr int EPT = 16 / ESIZE;
  constexpr uint32_t kAll = (1u << EPT) - 1u;
  if (mk == kAll) return;
  if (mk == 0u && e0 + EPT <= V_logits) {
    // a streaming store: the line is written whole and not read again here, so it need not stay in the caches
    typedef uint32_t v4u __attribute__((ext_vector_type(4)));
    const uint32_t w = ESIZE == 2 ? (neg_inf | (neg_inf << 16)) : neg_inf;
    const v4u val = {w, w, w, w};
    __builtin_nontemporal_store(val, reinterpret_cast<v4u*>(p));
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
  // thread t of nt: the range's groups t, t + nt, ...
  __device__ __forceinline__ void groups(uint32_t t, uint32_t nt) const {
    if constexpr (APPLY != 0) {
      constexpr int EPT = 16 / APPLY;
      constexpr uint32_t kAll = (1u << EPT) - 1u;
      for (int32_t e0 = e_begin + (int32_t)t * EPT; e0 < e_end; e0 += (int32_t)nt * EPT) {
        uint32_t mk = 0u;  // (columns beyond the vocabulary are masked)
        if (e0 < V) {
          mk = (words[(e0 - e_begin) >> 5] >> (e0 & 31)) & kAll;
          if (e0 + EPT > V) mk &= (1u << (V - e0)) - 1u;
        }
        apply_group<APPLY>(row + (size_t)e0 * APPLY, mk, e0, V_logits, neg_inf);
      }
    }
  }
  // The same for a range of kSegTokens elements that lies inside both the vocabulary and the row (every
  // segment but a row's last), written for the fewest instructions: with 2432 workgroups of four waves on
  // 1024 SIMDs the launch is bound by instruction issue, and each 60 instructions per thread cost a
  // microsecond.  Thread t of NT takes the groups t, t + NT, ...: their mask bits are fetched from LDS
  // first (one byte each for 2-byte logits), then a group with nothing allowed is one streaming store and a
  // group with both kinds one 2- or 4-byte store per disallowed element, in a loop that runs as often as
  // the lane of the wave with the most of them needs.
  template <int NT>
  __device__ __forceinline__ void whole_segment(uint32_t t) const {
    if constexpr (APPLY != 0) {
      constexpr int EPT = 16 / APPLY;
      constexpr uint32_t kAll = (1u << EPT) - 1u;
      constexpr int kGroups = kSegTokens / EPT / NT;  // per thread
      static_assert(kSegTokens % (EPT * NT) == 0, "every thread takes the same number of groups");
      typedef uint32_t v4u __attribute__((ext_vector_type(4)));
      const uint32_t fill = APPLY == 2 ? (neg_inf | (neg_inf << 16)) : neg_inf;
      const v4u val = {fill, fill, fill, fill};
      unsigned char* p = row + ((size_t)e_begin * APPLY + (size_t)t * 16u);
      uint32_t mk[kGroups];
#pragma unroll
      for (int k = 0; k < kGroups; ++k) {
        const uint32_t g = (uint32_t)k * NT + t;
        if (APPLY == 2) mk[k] = reinterpret_cast<const unsigned char*>(words)[g];
        else mk[k] = (words[g >> 3] >> ((g & 7u) * 4u)) & kAll;
      }
#pragma unroll
      for (int k = 0; k < kGroups; ++k) {
        unsigned char* q = p + (size_t)k * NT * 16u;
        if (mk[k] == 0u) {
          __builtin_nontemporal_store(val, reinterpret_cast<v4u*>(q));
        } else {
          for (uint32_t x = ~mk[k] & kAll; x; x &= x - 1u) {
            const uint32_t h = (uint32_t)__ffs(x) - 1u;
            if (APPLY == 2) reinterpret_cast<uint16_t*>(q)[h] = (uint16_t)neg_inf;
            else reinterpret_cast<uint32_t*>(q)[h] = neg_inf;
          }
        }
      }
    }
  }
};

// ---------------------------------------------------------------- kernel (b)
// The per-step stack upload, as a kernel on the caller's stream that reads pinned host memory over the bus
// (for the few tens of kilobytes of a step this takes a fraction of the time a copy-engine transfer with
// its cross-queue synchronisation does).  The stack headers are written out in full on the way: the host
// sends, per stack, the keys of its lists; the offsets of the lists' segments are read from the cache's
// key_off here.  Blocks [0, copy_blocks) copy the row descriptors and the frames, the others expand
// kStacksPerBlock stacks each, whose key words go through LDS (one read over the bus per 16 bytes).
constexpr int kUploadThreads = 256;
constexpr uint32_t kStacksPerBlock = 2;
__global__ __launch_bounds__(kUploadThreads) void upload_stacks_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst,
                                                                       uint32_t plain16, const uint4* __restrict__ src_frames,
                                                                       uint4* __restrict__ dst_frames, uint32_t frames16,
                                                                       uint32_t copy_blocks, const uint4* __restrict__ src_stacks,
                                                                       uint32_t n_stacks, uint32_t n_seg,
                                                                       uint32_t* __restrict__ dst_hdrs) {
  __shared__ uint32_t keys[kStacksPerBlock][kStackKeysWords];
  if (blockIdx.x < copy_blocks) {
    const uint32_t i = blockIdx.x * kUploadThreads + threadIdx.x;
    if (i < plain16) dst[i] = src[i];
    else if (i < plain16 + frames16) dst_frames[i - plain16] = src_frames[i - plain16];
    return;
  }
  const uint32_t s0 = (blockIdx.x - copy_blocks) * kStacksPerBlock;
  constexpr uint32_t kQuads = kStackKeysWords / 4;
  if (threadIdx.x < kStacksPerBlock * kQuads && s0 + threadIdx.x / kQuads < n_stacks) {
    const uint4 q = src_stacks[(size_t)s0 * kQuads + threadIdx.x];
    uint32_t* k = &keys[threadIdx.x / kQuads][(threadIdx.x % kQuads) * 4];
    k[0] = q.x; k[1] = q.y; k[2] = q.z; k[3] = q.w;
  }
  __syncthreads();
  const uint32_t stride = stack_hdr_stride((int32_t)n_seg);
  for (uint32_t t = threadIdx.x; t < kStacksPerBlock * stride; t += kUploadThreads) {
    const uint32_t st = t / stride, w = t % stride;
    if (s0 + st >= n_stacks) break;
    const uint32_t* k = keys[st];
    uint32_t out;
    if (w < kStackHdrWords) out = k[w];
    else {
      const uint32_t sgm = (w - kStackHdrWords) / kStackLists, l = (w - kStackHdrWords) % kStackLists, key = k[kStackHdrWords + l];
      const uint32_t* key_off = reinterpret_cast<const uint32_t*>((uintptr_t)k[kStackHdrWords + kStackLists] |
                                                                  ((uintptr_t)k[kStackHdrWords + kStackLists + 1] << 32));
      out = key == kNoKey ? 0u : key_off[(size_t)key * n_seg + sgm];
    }
    dst_hdrs[(size_t)(s0 + st) * stride + w] = out;
  }
}

constexpr int kFillThreads = 256;
constexpr int kFillFramesLds = 1024;            // live frames kept in LDS (deeper stacks: global memory)

// One workgroup of 4 waves serves one request and one segment of 8192 token
// ids = 256 mask words, which it owns in LDS:
//   1. every word = OR of the accepted bitsets of the tops of all stacks that
//      keep one (Algorithm 1: the result is the union over the parallel
//      stacks); the stop tokens if the text may end;
//   2. the stacks' token lists for this segment (up to four per stack: the
//      top node's own accepted tokens if it keeps a list instead of a bitset,
//      the tokens accepted given the node below the top frame, those accepted
//      given the two and the three nodes below) are streamed once, coalesced;
//      an accepted entry sets its bit with an LDS atomic, a walk entry is only
//      noted (one flag for the workgroup);
//   3. if there was a walk entry, the lists are gone through again and theirs
//      are decided against the live stack: only then are the request's automaton
//      tables and frames copied into LDS.  Most launches walk nothing;
//   4. the words are stored once, coalesced, and - in the fused instantiation -
//      the logits of the segment are masked straight from them.
// No global atomics, no second pass over the mask.  The launch is bound by
// instruction issue as much as by memory (2432 workgroups of four waves on 1024
// SIMDs): what every thread would do for nothing is kept behind tests that are
// the same for the whole workgroup (an empty list costs a scalar compare).
// COUNT = true additionally sums the automaton steps of all walks into
// *step_counter (instrumentation for the benchmark; never used on the hot path).
struct FillShared {
  uint32_t words[kSegWords];
  uint16_t live[kFillFramesLds];
  uint32_t any_walk;
};


// Decides the walk entries of the workgroup's lists (all threads call this).
template <bool COUNT, bool KEEP_UNDECIDED, class Tab>
__device__ __forceinline__ void fill_walks(const Tab& T, FillShared& sm, const RowDesc& rd, const int32_t b, const int32_t seg,
                                           const uint32_t n_stacks, const uint32_t frame0, const bool frames_in_lds,
                                           const XGM_GLOBAL uint32_t* __restrict__ stack_hdrs, const uint32_t hdr_stride,
                                           const XGM_GLOBAL uint16_t* __restrict__ frames, const DevVocab& voc,
                                           OverflowLog* log, uint32_t seq, unsigned long long& my_steps) {
  const XGM_GLOBAL uint32_t* entries = (const XGM_GLOBAL uint32_t*)rd.entries;
  const int32_t id0 = seg * kSegTokens;
  for (uint32_t st = 0; st < n_stacks; ++st) {
    // one round of loads per stack: its scalars and where its four lists begin in this segment and in the next
    const XGM_GLOBAL uint32_t* sh = stack_hdrs + (size_t)(rd.stack_begin + st) * hdr_stride;
    typedef uint32_t v4u __attribute__((ext_vector_type(4)));
    const XGM_GLOBAL v4u* off = (const XGM_GLOBAL v4u*)(sh + stack_hdr_off((uint32_t)seg, 0u));
    const v4u scalars = *(const XGM_GLOBAL v4u*)sh, o0 = off[0], o1 = off[1];
    const uint32_t top = scalars.x & 0xFFFFu, depth = scalars.y, f_off = scalars.z;
    static_assert(kStackHdrTop == 0 && kStackHdrDepth == 1 && kStackHdrFrames == 2 && kStackHdrWords == 4 && kStackLists == 4,
                  "a stack's scalars are one 16-byte load, a segment's list offsets another");
    LiveView live;
    live.lds = (const XGM_LDS uint16_t*)sm.live + (f_off - frame0);
    live.glob = frames + f_off;
    live.lo = frames_in_lds ? 0u : 0xFFFFFFFFu;
    for (uint32_t l = 0; l < kStackLists; ++l) {  // (not unrolled: one copy of the walk)
      // the list's entries of this segment; the accepted ones are done
      const uint32_t begin = l == 0u ? o0.x : l == 1u ? o0.y : l == 2u ? o0.z : o0.w;
      const uint32_t end = l == 0u ? o1.x : l == 1u ? o1.y : l == 2u ? o1.z : o1.w;
      for (uint32_t j = begin + threadIdx.x; j < end; j += kFillThreads) {
        const uint32_t e = entries[j];
        const uint32_t id = e & kEntryIdMask, kind = e >> kEntryKindShift, pos = (e >> kEntryPosShift) & 0xFFu;
        if (kind == kEntryAccepted) continue;
        const uint32_t rel = id - (uint32_t)id0;
        if ((sm.words[rel >> 5] >> (rel & 31u)) & 1u) continue;  // already allowed
        const uint32_t drop = kind == kEntryWalkTop ? 0u : kind - 1u;  // frames above the one the walk starts in
        int res = kReject;
        uint32_t n_steps = 0;
        if (depth > drop) {
          const TokenRef t = load_token(voc, (int32_t)id);
          const uint32_t start = drop == 0u ? top : live[depth - 1u - drop];
          res = walk_token<false>(T, t.tk, t.ext, t.len, start, live, depth - drop, COUNT ? &n_steps : nullptr,
                                  0u, drop == 0u ? 0 : (int)pos);
        }
        if (COUNT) my_steps += n_steps;
        if (res == kOverflow) record_overflow(log, seq, (uint32_t)b, id, rd.epoch);  // decided on the host
        if (res == kAccept || (KEEP_UNDECIDED && res == kOverflow)) atomicOr(&sm.words[rel >> 5], 1u << (rel & 31u));
      }
    }
  }
}

// The whole of step 3, kept out of line: the request's tables and live frames into LDS, then the walks.  Nearly
// no workgroup comes here, and inlined the walk's registers and code would weigh on every workgroup's path
// (the kernel ran out of scalar registers and kept them in lanes of a vector register).  What it needs it
// reads again: the row descriptor, and of the vocabulary the three arrays a token is fetched from.  The call
// itself costs a workgroup that walks about a microsecond (registers saved and restored through memory).
struct FillWalkArgs {
  const RowDesc* row;
  const uint32_t* stack_hdrs;
  const uint16_t* frames;
  const uint4* tok_by_id;
  const uint32_t* off_by_id;
  const uint8_t* bytes;
  OverflowLog* log;
  unsigned long long* step_counter;
  int32_t b, seg, n_seg;
  uint32_t seq;
};
template <bool COUNT, bool KEEP_UNDECIDED>
__device__ __noinline__ void fill_walk_path(const FillWalkArgs a, FillShared XGM_LDS* shared, unsigned char XGM_LDS* staged) {
  FillShared& sm = *(FillShared*)shared;
  unsigned char* smem = (unsigned char*)staged;
  const RowDesc rd = *a.row;
  const XGM_GLOBAL uint32_t* stack_hdrs = (const XGM_GLOBAL uint32_t*)a.stack_hdrs;
  const XGM_GLOBAL uint16_t* frames = (const XGM_GLOBAL uint16_t*)a.frames;
  DevVocab voc{};
  voc.tok_by_id = a.tok_by_id;
  voc.off_by_id = a.off_by_id;
  voc.bytes = a.bytes;
  unsigned long long my_steps = 0;
  const uint32_t frame0 = rd.frame_begin, n_frames = rd.n_frames;
  const uint32_t hdr_stride = stack_hdr_stride(a.n_seg);
  const bool frames_in_lds = n_frames <= kFillFramesLds;
  stage_tables(rd.tab, smem, kFillThreads);
  if (frames_in_lds)
    for (uint32_t k = threadIdx.x; k < n_frames; k += kFillThreads) sm.live[k] = frames[frame0 + k];
  __syncthreads();
  if (small_sections_staged(rd.tab))
    fill_walks<COUNT, KEEP_UNDECIDED>(LdsTabT<true>(rd.tab, smem), sm, rd, a.b, a.seg, rd.n_stacks, frame0, frames_in_lds, stack_hdrs,
                                      hdr_stride, frames, voc, a.log, a.seq, my_steps);
  else
    fill_walks<COUNT, KEEP_UNDECIDED>(LdsTab(rd.tab, smem), sm, rd, a.b, a.seg, rd.n_stacks, frame0, frames_in_lds, stack_hdrs,
                                      hdr_stride, frames, voc, a.log, a.seq, my_steps);
  __syncthreads();
  if (COUNT && my_steps) atomicAdd(a.step_counter, my_steps);
}

// Eight workgroups of 4 waves per compute unit need 8 waves per SIMD: the second
// launch bound keeps the kernel within the registers that this takes.
// APPLY = 0: the mask only.  APPLY = 2 / 4 (bytes per logit): the workgroup
// also writes -inf into the logits of its (row, segment) straight from its
// LDS words (section 2.1), which saves a launch and the re-read of the mask.
// A token whose walk exceeded the limits is then left allowed (bit set, logit
// untouched) until the host has decided it.
struct FusedApply {
  unsigned char* logits;  // [B][row_stride] elements of APPLY bytes; 16-byte aligned rows
  int64_t row_stride;     // elements
  int32_t V_logits;
  uint32_t neg_inf;
};

template <bool COUNT, int APPLY>
__global__ __launch_bounds__(kFillThreads, 8) void fill_kernel(const RowDesc* __restrict__ rows,
                                                            const uint32_t* __restrict__ stack_hdrs_,
                                                            const uint16_t* __restrict__ frames_, DevVocab voc,
                                                            uint32_t* __restrict__ out, OverflowLog* log, uint32_t seq,
                                                            unsigned long long* step_counter, FusedApply fa) {
  extern __shared__ __align__(16) unsigned char smem[];
  __shared__ FillShared sm;
  const XGM_GLOBAL uint32_t* stack_hdrs = (const XGM_GLOBAL uint32_t*)stack_hdrs_;
  const uint32_t tid = threadIdx.x;
  const int32_t b = (int32_t)blockIdx.y, seg = (int32_t)blockIdx.x;
  const int32_t w_begin = seg * kSegWords;
  const int32_t n_words = min(kSegWords, voc.W - w_begin);
  const int32_t id0 = w_begin * 32;
  // LDS is cleared before anything is fetched (a barrier waits for what its threads have in flight)
  for (int32_t w = tid; w < kSegWords; w += kFillThreads) sm.words[w] = 0u;
  if (tid == 0) sm.any_walk = 0u;
  __syncthreads();
  const RowDesc rd = rows[b];
  const uint32_t hdr_stride = stack_hdr_stride(voc.n_seg);
  // may the request end here?  then its stop tokens are allowed (the first kFillThreads of them are fetched now)
  const bool may_end = rd.flags & 1u;
  const int32_t my_stop = may_end && (int32_t)tid < voc.n_stop ? voc.stop_ids[tid] : -1;
  const XGM_GLOBAL uint32_t* acc = (const XGM_GLOBAL uint32_t*)rd.acc;
  const XGM_GLOBAL uint32_t* entries = (const XGM_GLOBAL uint32_t*)rd.entries;
  auto take = [&](uint32_t e) {
    if ((e >> kEntryKindShift) == kEntryAccepted) {
      const uint32_t rel = (e & kEntryIdMask) - (uint32_t)id0;
      atomicOr(&sm.words[rel >> 5], 1u << (rel & 31u));
    } else {
      sm.any_walk = 1u;
    }
  };
  // 1 + 2. Two stacks at a time: their headers (the same words for every thread), then, in one go, this
  // thread's words of their bitset rows (Algorithm 1: the union over the parallel stacks) and the first
  // kFillThreads entries of their lists (most lists are shorter than that); then what is left of the lists.
  constexpr int kWordsPerThread = kSegWords / kFillThreads;
  for (uint32_t s0 = 0; s0 < rd.n_stacks; s0 += 2u) {
    uint32_t acc_row[2];
    uint2 lst[2][kStackLists];
#pragma unroll
    for (uint32_t q = 0; q < 2u; ++q) {
      acc_row[q] = kNoAccRow;
#pragma unroll
      for (uint32_t l = 0; l < kStackLists; ++l) lst[q][l] = make_uint2(0u, 0u);
      if (s0 + q < rd.n_stacks) {
        const XGM_GLOBAL uint32_t* sh = stack_hdrs + (size_t)(rd.stack_begin + s0 + q) * hdr_stride;
        acc_row[q] = sh[kStackHdrTop] >> 16;
        static_assert(kStackLists == 4, "the offsets of a segment's four lists are one 16-byte load");
        const uint4* off = reinterpret_cast<const uint4*>(stack_hdrs_ + (size_t)(rd.stack_begin + s0 + q) * hdr_stride +
                                                          stack_hdr_off((uint32_t)seg, 0u));
        const uint4 o0 = off[0], o1 = off[1];  // where the lists begin in this segment, and in the next
        lst[q][0] = make_uint2(o0.x, o1.x);
        lst[q][1] = make_uint2(o0.y, o1.y);
        lst[q][2] = make_uint2(o0.z, o1.z);
        lst[q][3] = make_uint2(o0.w, o1.w);
      }
    }
    uint32_t aw[2][kWordsPerThread], first[2][kStackLists];
    bool have[2][kStackLists];
#pragma unroll
    for (uint32_t q = 0; q < 2u; ++q) {
#pragma unroll
      for (int k = 0; k < kWordsPerThread; ++k) {
        const int32_t w = (int32_t)tid + k * kFillThreads;
        aw[q][k] = acc_row[q] != kNoAccRow && w < n_words ? acc[(size_t)acc_row[q] * voc.W + w_begin + w] : 0u;
      }
#pragma unroll
      for (uint32_t l = 0; l < kStackLists; ++l) {
        have[q][l] = false;
        first[q][l] = 0u;
        if (lst[q][l].x < lst[q][l].y) {  // (the same for every thread: an empty list costs a scalar compare)
          have[q][l] = lst[q][l].x + tid < lst[q][l].y;
          if (have[q][l]) first[q][l] = entries[lst[q][l].x + tid];
        }
      }
    }
#pragma unroll
    for (uint32_t q = 0; q < 2u; ++q) {
#pragma unroll
      for (int k = 0; k < kWordsPerThread; ++k)
        if (aw[q][k]) atomicOr(&sm.words[tid + k * kFillThreads], aw[q][k]);
#pragma unroll
      for (uint32_t l = 0; l < kStackLists; ++l) {
        if (lst[q][l].x < lst[q][l].y) {
          if (have[q][l]) take(first[q][l]);
          if (lst[q][l].y - lst[q][l].x > (uint32_t)kFillThreads)
            for (uint32_t j = lst[q][l].x + kFillThreads + tid; j < lst[q][l].y; j += kFillThreads) take(entries[j]);
        }
      }
    }
  }
  if (may_end)
    for (int32_t k = tid; k < voc.n_stop; k += kFillThreads) {
      const int32_t rel = (k == (int32_t)tid ? my_stop : voc.stop_ids[k]) - id0;
      if (rel >= 0 && rel < n_words * 32) atomicOr(&sm.words[rel >> 5], 1u << (rel & 31));
    }
  __syncthreads();
  // 3. walk entries, if any
  if (sm.any_walk) {
    FillWalkArgs wa;
    wa.row = rows + b;
    wa.stack_hdrs = stack_hdrs_;
    wa.frames = frames_;
    wa.tok_by_id = voc.tok_by_id;
    wa.off_by_id = voc.off_by_id;
    wa.bytes = voc.bytes;
    wa.log = log;
    wa.step_counter = step_counter;
    wa.b = b;
    wa.seg = seg;
    wa.n_seg = voc.n_seg;
    wa.seq = seq;
    fill_walk_path<COUNT, APPLY != 0>(wa, (FillShared XGM_LDS*)&sm, (unsigned char XGM_LDS*)smem);
  }
  // 4. the words, and the logits of the segment; the last segment also takes the columns beyond the vocabulary
  for (int32_t w = tid; w < n_words; w += kFillThreads) out[(size_t)b * voc.W + w_begin + w] = sm.words[w];
  if (APPLY != 0) {
    LogitsRange<APPLY> logits;
    logits.row = fa.logits + (size_t)b * fa.row_stride * APPLY;
    logits.words = sm.words;
    logits.e_begin = id0;
    logits.e_end = seg + 1 == voc.n_seg ? fa.V_logits : min(id0 + kSegTokens, fa.V_logits);
    logits.V = voc.V;
    logits.V_logits = fa.V_logits;
    logits.neg_inf = fa.neg_inf;
    if (logits.e_end == id0 + kSegTokens && logits.e_end <= voc.V) logits.template whole_segment<kFillThreads>(tid);
    else logits.groups(tid, kFillThreads);
  }
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
constexpr int kErrTokenRejected = -6, kErrTerminated = -7, kErrTooManyStacks = -8, kErrTooLarge = -9, kErrBadArg = -1, kErrInternal = -11;

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
// list offsets; frames).  A row whose token is not
// allowed, or whose new state does not fit the device limits, keeps its state
// and gets an error code in `status`.
__global__ __launch_bounds__(kAcceptThreads) void batch_accept_kernel(DevBatch bt, DevVocab voc,
                                                                      const int32_t* __restrict__ tokens) {
  __shared__ uint16_t cand[kBatchMaxCandidates * kBatchMaxDepth];
  __shared__ uint32_t cdepth[kBatchMaxCandidates];
  __shared__ uint32_t order[kBatchMaxCandidates];  // rank among the distinct stacks, or kNoKey for a duplicate
  __shared__ uint32_t foff[kBatchMaxStacks + 1];
  __shared__ uint32_t slot_of[kBatchMaxStacks];    // candidate index per rank
  __shared__ uint32_t keys[kBatchMaxStacks][kStackLists];  // the three lists of every new stack
  __shared__ uint32_t cidx[kBatchMaxStacks][kCtxLevels];   // which context of its rule each of the top frames sits on
  __shared__ uint32_t ccount, coverflow, n_new, can_end, bad_context, not_final;
  const uint32_t tid = threadIdx.x;
  const int32_t b = blockIdx.x;
  // what the row needs is fetched before anything is decided: one round trip for the token id and the slot,
  // one for the token's bytes and the state's size (a branch in between would make each of them wait)
  const int32_t tok = tokens[b];
  const int32_t head = bt.head[b];
  const DevCache& dc = bt.cache[b];
  const int32_t first_stop = voc.n_stop > 0 ? voc.stop_ids[0] : -1;
  const uint4 tk = voc.tok_by_id[tok >= 0 && tok < voc.V ? tok : 0];
  const SlotMeta cur = bt.meta[(size_t)b * bt.H + head];
  if (tok < 0) return;  // this row is left alone (its status too)
  const uint32_t n_off = (uint32_t)bt.n_seg + 1u;
  const uint32_t hdr_stride = stack_hdr_stride(bt.n_seg);
  const int32_t next = (head + 1) % bt.H;
  const uint32_t sb = ((uint32_t)b * bt.H + next) * kBatchMaxStacks;
  const uint32_t fb = ((uint32_t)b * bt.H + next) * kBatchRowFrames;
  int32_t status = 0;
  bool stop = false;
  if (tok >= voc.V) status = kErrBadArg;
  else if (cur.flags & 2u) status = kErrTerminated;
  else {
    stop = tok == first_stop;
    for (int32_t k = 1; k < voc.n_stop; ++k) stop = stop || voc.stop_ids[k] == tok;
    if (stop && !(cur.flags & 1u)) status = kErrTokenRejected;
  }
  if (status != 0) {
    if (tid == 0) bt.status[b] = status;
    return;
  }
  if (tid == 0) { ccount = 0u; coverflow = 0u; n_new = 0u; can_end = 0u; bad_context = 0u; not_final = 0u; }
  __syncthreads();
  DevTables tab = dc.tab;
  tab.lds_end = tab.stage_bytes = tab.n_near = 0u;  // the walks read the tables where they are
  const LdsTab T(tab, nullptr);
  if (!stop) {
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
                                        0u, 0, (uint32_t*)nullptr, collect);
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
      order[tid] = dup ? kNoKey : 0u;
      if (!dup) atomicAdd(&n_new, 1u);
    }
    __syncthreads();
    uint32_t before = 0u;
    if (tid < nc && order[tid] != kNoKey)
      for (uint32_t j = 0; j < nc; ++j)
        if (j != tid && order[j] != kNoKey &&
            compare_stacks(cand + j * kBatchMaxDepth, cdepth[j], cand + tid * kBatchMaxDepth, cdepth[tid]) < 0)
          ++before;
    __syncthreads();
    if (tid < nc && order[tid] != kNoKey) order[tid] = before;
    __syncthreads();
    if (n_new > kBatchMaxStacks) {
      if (tid == 0) bt.status[b] = kErrTooManyStacks;
      return;
    }
    if (tid < nc && order[tid] != kNoKey) slot_of[order[tid]] = tid;
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
    // which context of its rule each of the top frames sits on (one thread per stack and level)
    if (tid < ns * (uint32_t)kCtxLevels) {
      const uint32_t r = tid / (uint32_t)kCtxLevels, l = tid % (uint32_t)kCtxLevels + 1u;
      const uint32_t ci = slot_of[r], d = cdepth[ci];
      const uint16_t* st = cand + ci * kBatchMaxDepth;
      uint32_t idx = kNoKey;
      if (d >= l + 1u) {
        const uint32_t rule = T.header(st[d - l]).y >> 16, below = st[d - l - 1u];
        for (uint32_t k = dc.node_ctx_off[below]; k < dc.node_ctx_off[below + 1u]; ++k) {
          const uint32_t x = dc.node_ctx[k];
          if ((x >> 16) == rule) idx = x & 0xFFFFu;
        }
        if (idx == kNoKey) bad_context = 1u;
      }
      cidx[r][l - 1u] = idx;
    }
    // whether some stack can end the text: every frame of it may end its rule
    for (uint32_t item = tid; item < ns * kBatchMaxDepth; item += kAcceptThreads) {
      const uint32_t r = item / kBatchMaxDepth, k = item % kBatchMaxDepth;
      const uint32_t ci = slot_of[r];
      if (k < cdepth[ci] && !T.is_final(cand[ci * kBatchMaxDepth + k])) atomicOr(&not_final, 1u << r);
    }
    __syncthreads();
    if (tid == 0 && (not_final & ((1u << ns) - 1u)) != ((1u << ns) - 1u)) can_end = 1u;
    // headers: scalars, the keys of the stack's lists
    if (tid < ns) {
      const uint32_t ci = slot_of[tid], d = cdepth[ci];
      const uint16_t* st = cand + ci * kBatchMaxDepth;
      uint32_t* h = bt.hdrs + (size_t)(sb + tid) * hdr_stride;
      const uint32_t top = st[d - 1];
      h[kStackHdrTop] = top | ((uint32_t)dc.acc_row[top] << 16);
      h[kStackHdrDepth] = d;
      h[kStackHdrFrames] = fb + foff[tid];
      h[3] = 0u;
      // the keys: the top node's own list, then one per frame below that a kept level reaches
      keys[tid][0] = top;
      uint32_t local = top, key0 = (uint32_t)dc.n_nodes;
      bool more = true;
#pragma unroll
      for (uint32_t l = 1; l <= (uint32_t)kCtxLevels; ++l) {
        uint32_t key = kNoKey;
        if (more && cidx[tid][l - 1u] != kNoKey && dc.k_base[l - 1u] != nullptr) {
          const uint32_t kb = dc.k_base[l - 1u][local];
          if (kb != kNoKey) {
            local = kb + cidx[tid][l - 1u];
            key = key0 + local;
          }
        }
        more = key != kNoKey;
        keys[tid][l] = key;
        key0 += dc.n_k[l - 1u];
      }
    }
    __syncthreads();
    if (bad_context) {  // a frame sits on a node that is no context of its rule: never the case for stacks the walk makes
      if (tid == 0) bt.status[b] = kErrInternal;
      return;
    }
    // headers: where the lists' segments start
    for (uint32_t item = tid; item < ns * kStackLists * n_off; item += kAcceptThreads) {
      const uint32_t r = item / (kStackLists * n_off), sgm = item / kStackLists % n_off, l = item % kStackLists;
      const uint32_t key = keys[r][l];
      bt.hdrs[(size_t)(sb + r) * hdr_stride + stack_hdr_off(sgm, l)] =
          key == kNoKey ? 0u : dc.key_off[(size_t)key * (uint32_t)bt.n_seg + sgm];
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
    r.entries = dc.entries;
    r.stack_begin = sb;
    r.n_stacks = m.n_stacks;
    r.flags = m.flags & 1u;
    r.frame_begin = fb;
    r.n_frames = m.n_frames;
    r.epoch = bt.rows[b].epoch + 1u;
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
  r.epoch += 1u;
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
  const uint32_t hdr_stride = stack_hdr_stride(bt.n_seg);
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
  r.epoch += 1u;
  bt.rows[b] = r;
  bt.head[b] = next;
  const int32_t o = bt.older[b] + 1;
  bt.older[b] = o < bt.H - 1 ? o : bt.H - 1;
  bt.status[b] = 0;
}

// ---------------------------------------------------------------- kernel (c)
constexpr int kApplyThreads = 256;

// Section 2.1: logits of disallowed tokens become -inf.  One workgroup per
// (segment of kSegTokens elements, row), as in the one-launch kernel, and with
// its code (LogitsRange): a thread takes 16-byte groups (8 bf16/fp16 or 4 fp32
// elements), the 64 groups of a wave are contiguous (1 KiB); the mask bits come
// straight from the bitmask in global memory.  ESIZE = bytes per element.
template <int ESIZE>
__global__ __launch_bounds__(kApplyThreads) void apply_kernel(unsigned char* __restrict__ logits, int64_t row_stride,
                                                              const uint32_t* __restrict__ bitmask, int32_t W_mask,
                                                              int32_t V_logits, int32_t V_mask,
                                                              const int32_t* __restrict__ row_index, uint32_t neg_inf) {
  const int32_t j = blockIdx.y, seg = blockIdx.x;
  const int64_t lrow = row_index ? row_index[j] : j;
  LogitsRange<ESIZE> r;
  r.row = logits + (size_t)lrow * row_stride * ESIZE;
  r.words = bitmask + (size_t)j * W_mask + (size_t)seg * kSegWords;
  r.e_begin = seg * kSegTokens;
  r.e_end = min(r.e_begin + kSegTokens, V_logits);
  r.V = V_mask;
  r.V_logits = V_logits;
  r.neg_inf = neg_inf;
  if (r.e_begin + kSegTokens <= min(V_mask, V_logits)) r.template whole_segment<kApplyThreads>(threadIdx.x);
  else r.groups(threadIdx.x, kApplyThreads);
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
// blob (row descriptors, stack headers, frames) goes here instead of into
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
void launch_first_byte(const DevTables& tab, uint4* first_byte, hipStream_t stream) {
  const uint32_t n_words = first_byte_words(tab.n_nodes);
  if (n_words == 0) return;
  hipLaunchKernelGGL(first_byte_kernel, dim3((256u * n_words + kFirstByteThreads - 1) / kFirstByteThreads),
                     dim3(kFirstByteThreads), 0, stream, tab, n_words, first_byte);
}

// Items of 64 tokens that a wave of the classify kernel takes on average.  Measured at 128256 tokens: the large
// workgroups (whose LDS holds a compute unit's place until their slowest wave is done) gain from four
// (11867-node schema grammar 1.68 -> 1.42 ms; eight: the same); the small ones from two when the grid has few
// node groups (JSON, 19 groups: 0.18 -> 0.14 ms) and from none when it has many (C/SQL, 187 groups: 1.62 ms
// with one, 1.66 with two, 2.0 with four).
static int32_t classify_items_per_wave(int threads, int32_t ny) {
  if (threads == kClassifyThreadsLarge) return 4;
  return ny < 64 ? 2 : 1;
}

void launch_classify(const DevTables& tab, const DevVocab& voc, int32_t node0, int32_t n, const uint4* first_byte,
                     uint32_t* acc_rank, uint32_t* unc_rank, uint32_t* plain_rank, uint32_t* plain_count, OverflowLog* log,
                     uint32_t seq, hipStream_t stream) {
  if (n <= 0 || voc.V <= 0) return;
  static_assert(32 % kNodesPerBlockSmall == 0 && 32 % kNodesPerBlockMany == 0 && kNodesPerBlockLarge % 32 == 0,
                "a block's nodes lie in whole words, or in one");
  const uint32_t n_words = first_byte_words(tab.n_nodes);
  const DevTables st = staged_for(tab, kClassifyLdsBudget);
  if (st.stage_bytes <= kClassifySmallStage) {
    const int32_t per_block = n >= kManyNodes ? kNodesPerBlockMany : kNodesPerBlockSmall;
    const int32_t ny = (n + per_block - 1) / per_block;
    const int32_t items = classify_items_per_wave(kClassifyThreadsSmall, ny);
    const int32_t chunk = kClassifyThreadsSmall * items;
    hipLaunchKernelGGL(classify_kernel<kClassifyThreadsSmall>, dim3((voc.V + chunk - 1) / chunk, ny), dim3(kClassifyThreadsSmall),
                       st.stage_bytes, stream, st, voc, node0, n, first_byte, n_words, acc_rank, unc_rank, plain_rank,
                       plain_count, log, seq, per_block, items);
  } else {
    const int32_t ny = (n + kNodesPerBlockLarge - 1) / kNodesPerBlockLarge;
    const int32_t items = classify_items_per_wave(kClassifyThreadsLarge, ny);
    const int32_t chunk = kClassifyThreadsLarge * items;
    hipLaunchKernelGGL(classify_kernel<kClassifyThreadsLarge>, dim3((voc.V + chunk - 1) / chunk, ny), dim3(kClassifyThreadsLarge),
                       st.stage_bytes, stream, st, voc, node0, n, first_byte, n_words, acc_rank, unc_rank, plain_rank,
                       plain_count, log, seq, kNodesPerBlockLarge, items);
  }
}

void launch_permute(const DevVocab& voc, int32_t n, const uint32_t* a_rank, const uint32_t* b_rank, uint32_t* a_id,
                    uint32_t* b_id, uint32_t* seg_counts, unsigned long long* digest, uint32_t* b_counts, hipStream_t stream) {
  if (n <= 0) return;
  hipLaunchKernelGGL(permute_kernel, dim3(n), dim3(kRowThreads), (size_t)voc.W * 8, stream, voc, a_rank, b_rank, a_id, b_id,
                     seg_counts, digest, b_counts);
}

void launch_rows_equal(const uint32_t* rows, int32_t n, int32_t W, const int32_t* rep, uint32_t* equal, hipStream_t stream) {
  if (n > 0) hipLaunchKernelGGL(rows_equal_kernel, dim3(n), dim3(kRowThreads), 0, stream, rows, W, rep, equal);
}
void launch_gather_rows(const uint32_t* rows, int32_t W, const int32_t* unique, int32_t n_unique, uint32_t* out,
                        hipStream_t stream) {
  if (n_unique > 0) hipLaunchKernelGGL(gather_rows_kernel, dim3(n_unique), dim3(kRowThreads), 0, stream, rows, W, unique, out);
}

void launch_rows_to_lists(const uint32_t* rows, int32_t row_words, const int32_t* map, int32_t n, const uint32_t* cursor_of,
                          int32_t per_row, uint32_t* cursor, uint32_t* out, uint16_t* out_row, hipStream_t stream) {
  const int32_t n_seg = (row_words + kSegWords - 1) / kSegWords;
  for (int32_t r0 = 0; r0 < n; r0 += 32768) {  // grid.y limit
    const int32_t nb = std::min(32768, n - r0);
    hipLaunchKernelGGL(rows_to_lists_kernel, dim3(n_seg, nb), dim3(kListThreads), 0, stream, rows + (size_t)r0 * row_words,
                       row_words, map, cursor_of + r0, per_row, cursor, out, out_row, r0);
  }
}

void launch_exit_positions(const DevTables& tab, const DevVocab& voc, const ContextListArgs& args, hipStream_t stream) {
  if (args.total == 0) return;
  const DevTables st = staged_for(tab, kContextLdsBudget);
  hipLaunchKernelGGL(exit_positions_kernel, dim3((args.total + kContextThreads - 1) / kContextThreads), dim3(kContextThreads),
                     st.stage_bytes, stream, st, voc, args);
}

void launch_context_lists(const DevTables& tab, const DevVocab& voc, const ContextListArgs& args, bool write, hipStream_t stream) {
  if (args.total == 0 || args.n_tiles == 0) return;
  const DevTables st = staged_for(tab, kContextLdsBudget);
  const dim3 g1(args.n_tiles), g2(1024);
  if (write && args.outcomes) {
    // Level 1 from the kept outcomes; its records for level 2 are still there from the counting pass, and so
    // are the deeper levels' records if their outcomes were kept too (levels that walk again make the records
    // of the next level again: those counts start at zero).
    hipLaunchKernelGGL(context_level1_write_kernel, g1, dim3(kContextThreads), 0, stream, voc, args);
    bool deep = true;  // all deeper levels from kept outcomes, or all of them by walking again
    for (uint32_t level = 2; level <= (uint32_t)kCtxLevels && args.k_base[level - 1] != nullptr; ++level)
      deep = deep && args.deep_outcomes[level - 1] != nullptr;
    if (!deep) (void)hipMemsetAsync(args.res_count + 1, 0, 4 * (kCtxLevels - 1), stream);
    for (uint32_t level = 2; level <= (uint32_t)kCtxLevels && args.k_base[level - 1] != nullptr; ++level) {
      if (deep) hipLaunchKernelGGL(context_deeper_write_kernel, g2, dim3(256), 0, stream, voc, args, level);
      else hipLaunchKernelGGL(context_deeper_kernel<true>, g2, dim3(kContextThreads), st.stage_bytes, stream, st, voc, args, level);
    }
    return;
  }
  (void)hipMemsetAsync(args.res_count, 0, 4 * kCtxLevels, stream);
  if (write) hipLaunchKernelGGL(context_level1_kernel<true>, g1, dim3(kContextThreads), st.stage_bytes, stream, st, voc, args);
  else hipLaunchKernelGGL(context_level1_kernel<false>, g1, dim3(kContextThreads), st.stage_bytes, stream, st, voc, args);
  for (uint32_t level = 2; level <= (uint32_t)kCtxLevels && args.k_base[level - 1] != nullptr; ++level) {
    if (write) hipLaunchKernelGGL(context_deeper_kernel<true>, g2, dim3(kContextThreads), st.stage_bytes, stream, st, voc, args, level);
    else hipLaunchKernelGGL(context_deeper_kernel<false>, g2, dim3(kContextThreads), st.stage_bytes, stream, st, voc, args, level);
  }
}
uint32_t context_tile_pairs() { return (uint32_t)kContextThreads; }
uint32_t context_tile_contexts() { return kContextsPerThread; }

void launch_patch_classes(const DevVocab& voc, const uint32_t* items, int32_t n_items, uint32_t* acc_rank,
                          uint32_t* unc_rank, uint32_t* plain_rank, hipStream_t stream) {
  if (n_items <= 0) return;
  hipLaunchKernelGGL(patch_classes_kernel, dim3((n_items + 255) / 256), dim3(256), 0, stream, voc, items, n_items,
                     acc_rank, unc_rank, plain_rank);
}

void launch_upload_stacks(const void* src, void* dst, size_t plain_bytes, const void* src_stacks, uint32_t n_stacks,
                          int32_t n_seg, void* dst_hdrs, const void* src_frames, void* dst_frames, size_t frames_bytes,
                          hipStream_t stream) {
  static_assert(kStackKeysWords % 4 == 0 && kStackKeysWords >= kStackHdrWords + kStackLists + 2, "the key words of a stack");
  const uint32_t plain16 = (uint32_t)(plain_bytes / 16), frames16 = (uint32_t)((frames_bytes + 15) / 16);
  const uint32_t copy_blocks = (plain16 + frames16 + kUploadThreads - 1) / kUploadThreads;
  const uint32_t stack_blocks = (n_stacks + kStacksPerBlock - 1) / kStacksPerBlock;
  if (copy_blocks + stack_blocks == 0) return;
  hipLaunchKernelGGL(upload_stacks_kernel, dim3(copy_blocks + stack_blocks), dim3(kUploadThreads), 0, stream,
                     reinterpret_cast<const uint4*>(src), reinterpret_cast<uint4*>(dst), plain16,
                     reinterpret_cast<const uint4*>(src_frames), reinterpret_cast<uint4*>(dst_frames), frames16, copy_blocks,
                     reinterpret_cast<const uint4*>(src_stacks), n_stacks, (uint32_t)n_seg, reinterpret_cast<uint32_t*>(dst_hdrs));
}

void launch_fill(const RowDesc* rows, const uint32_t* stack_hdrs, const uint16_t* frames, int32_t B, const DevVocab& voc,
                 uint32_t* out, OverflowLog* log, uint32_t seq, unsigned long long* step_counter, hipStream_t stream,
                 void* logits, int elem_size, uint32_t neg_inf, int32_t V_logits, int64_t row_stride) {
  if (B <= 0) return;
  const dim3 grid(voc.n_seg, B);
  const FusedApply fa{static_cast<unsigned char*>(logits), row_stride, V_logits, neg_inf};
  if (logits && elem_size == 2)
    hipLaunchKernelGGL((fill_kernel<false, 2>), grid, dim3(kFillThreads), kFillLdsBudget, stream, rows, stack_hdrs, frames,
                       voc, out, log, seq, step_counter, fa);
  else if (logits)
    hipLaunchKernelGGL((fill_kernel<false, 4>), grid, dim3(kFillThreads), kFillLdsBudget, stream, rows, stack_hdrs, frames,
                       voc, out, log, seq, step_counter, fa);
  else if (step_counter)
    hipLaunchKernelGGL((fill_kernel<true, 0>), grid, dim3(kFillThreads), kFillLdsBudget, stream, rows, stack_hdrs, frames,
                       voc, out, log, seq, step_counter, fa);
  else
    hipLaunchKernelGGL((fill_kernel<false, 0>), grid, dim3(kFillThreads), kFillLdsBudget, stream, rows, stack_hdrs, frames,
                       voc, out, log, seq, step_counter, fa);
}

void launch_lds_lookups(int32_t n_blocks, uint32_t hops, uint32_t* sink, hipStream_t stream) {
  hipLaunchKernelGGL(lds_lookup_kernel, dim3(n_blocks), dim3(kLookupThreads), 8192 * 4, stream, 8192u, hops, sink);
}

void launch_batch_accept(const DevBatch& bt, const DevVocab& voc, const int32_t* d_tokens, hipStream_t stream) {
  hipLaunchKernelGGL(batch_accept_kernel, dim3(bt.B), dim3(kAcceptThreads), 0, stream, bt, voc, d_tokens);
}

void launch_batch_fork(const DevBatch& bt, const int32_t* d_src_rows, hipStream_t stream) {
  hipLaunchKernelGGL(batch_fork_copy_kernel, dim3(bt.B), dim3(256), 0, stream, bt, d_src_rows);
  hipLaunchKernelGGL(batch_fork_commit_kernel, dim3((bt.B + 255) / 256), dim3(256), 0, stream, bt, d_src_rows);
}

void launch_batch_rollback(const DevBatch& bt, const int32_t* d_steps, hipStream_t stream) {
  hipLaunchKernelGGL(batch_rollback_kernel, dim3((bt.B + 255) / 256), dim3(256), 0, stream, bt, d_steps);
}

void launch_apply(void* logits, int elem_size, uint32_t neg_inf, int32_t V_logits, int64_t row_stride,
                  const uint32_t* bitmask, int32_t V_mask, const int32_t* row_index, int32_t n_rows,
                  hipStream_t stream) {
  if (n_rows <= 0 || V_logits <= 0) return;
  const int32_t W_mask = (V_mask + 31) / 32;
  const bool aligned = (reinterpret_cast<uintptr_t>(logits) % 16 == 0) && ((row_stride * elem_size) % 16 == 0);
  unsigned char* p = static_cast<unsigned char*>(logits);
  if (aligned) {
    dim3 grid((V_logits + kSegTokens - 1) / kSegTokens, n_rows);
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
