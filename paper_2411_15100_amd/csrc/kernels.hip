// HIP kernels for gfx950 (wave64): token walk / classify, rank->id permute,
// context-dependent lists, batched mask fill, -inf apply.
#include <hip/hip_runtime.h>

#include "kernels.hpp"
#include "walk.hpp"

namespace xgm {

namespace {


__device__ __forceinline__ void record_overflow(OverflowLog* log, uint32_t seq, uint32_t a, uint32_t b) {
  uint32_t slot = atomicAdd(&log->count, 1u) % OverflowLog::kCap;
  log->entry[slot][0] = seq;
  log->entry[slot][1] = a;
  log->entry[slot][2] = b;
}

// ---------------------------------------------------------------- kernel (a)
constexpr int kClassifyThreads = 256;
constexpr int kNodesPerBlock = 16;

// One thread owns one token (byte-sorted order, so a wave's 64 tokens are
// neighbours in the sorted vocabulary and mostly share prefixes and control
// flow) and classifies it at kNodesPerBlock nodes, the token staying in
// registers.  Each wave packs its 64 results per node with a ballot into two
// mask words of the rank-space bitsets.  With LDS = true the automaton tables
// are first copied into shared memory.
template <bool LDS>
__global__ __launch_bounds__(kClassifyThreads) void classify_kernel(
    DevTables tab, int32_t n_nodes_total, int32_t n_rows_tab, int32_t n_alts, DevVocab voc, int32_t node0,
    int32_t n_nodes, uint32_t* __restrict__ acc_rank, uint32_t* __restrict__ unc_rank, OverflowLog* log,
    uint32_t seq) {
  extern __shared__ __align__(16) unsigned char smem[];
  DevTables T = tab;
  if (LDS) {
    uint2* s_hdr = reinterpret_cast<uint2*>(smem);
    uint32_t* s_alts = reinterpret_cast<uint32_t*>(s_hdr + n_nodes_total);
    uint16_t* s_rows = reinterpret_cast<uint16_t*>(s_alts + n_alts);
    uint8_t* s_cls = reinterpret_cast<uint8_t*>(s_rows + (size_t)n_rows_tab * tab.n_cls);
    for (int k = threadIdx.x; k < n_nodes_total; k += kClassifyThreads) s_hdr[k] = tab.hdr[k];
    for (int k = threadIdx.x; k < n_alts; k += kClassifyThreads) s_alts[k] = tab.alts[k];
    for (int k = threadIdx.x; k < n_rows_tab * tab.n_cls; k += kClassifyThreads) s_rows[k] = tab.rows[k];
    for (int k = threadIdx.x; k < 256; k += kClassifyThreads) s_cls[k] = tab.cls[k];
    __syncthreads();
    T.hdr = s_hdr;
    T.alts = s_alts;
    T.rows = s_rows;
    T.cls = s_cls;
  }
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
  const int32_t n_begin = blockIdx.y * kNodesPerBlock;
  const int32_t n_end = min(n_begin + kNodesPerBlock, n_nodes);
  for (int32_t k = n_begin; k < n_end; ++k) {
    int res = kReject;
    if (live_lane && len > 0) {
      res = walk_token<true>(T, tk, ext, len, (uint32_t)(node0 + k), nullptr, 1u);
      if (res == kOverflow) { record_overflow(log, seq, (uint32_t)k, (uint32_t)r); res = kReject; }
    }
    const unsigned long long a = __ballot(res == kAccept);
    const unsigned long long u = __ballot(res == kUncertain);
    if ((threadIdx.x & 63) == 0 && word < voc.WR) {
      uint32_t* pa = acc_rank + (size_t)k * voc.WR + word;
      uint32_t* pu = unc_rank + (size_t)k * voc.WR + word;
      pa[0] = (uint32_t)a;
      pa[1] = (uint32_t)(a >> 32);
      pu[0] = (uint32_t)u;
      pu[1] = (uint32_t)(u >> 32);
    }
  }
}

// Rank space -> id space: bit id of the output = bit rank_of_id[id] of the
// input.  One workgroup per node row; the two rank-space rows sit in LDS so
// that the random bit lookups never leave the CU.
constexpr int kPermuteThreads = 256;
__global__ __launch_bounds__(kPermuteThreads) void permute_kernel(DevVocab voc, const uint32_t* __restrict__ acc_rank,
                                                                  const uint32_t* __restrict__ unc_rank,
                                                                  uint32_t* __restrict__ acc_id,
                                                                  uint32_t* __restrict__ unc_id) {
  extern __shared__ __align__(16) unsigned char smem[];
  uint32_t* s_acc = reinterpret_cast<uint32_t*>(smem);
  uint32_t* s_unc = s_acc + voc.WR;
  const size_t node = blockIdx.x;
  for (int k = threadIdx.x; k < voc.WR; k += kPermuteThreads) {
    s_acc[k] = acc_rank[node * voc.WR + k];
    s_unc[k] = unc_rank[node * voc.WR + k];
  }
  __syncthreads();
  const int32_t v64 = (voc.V + 63) & ~63;
  for (int32_t id = threadIdx.x; id < v64; id += kPermuteThreads) {
    bool a = false, u = false;
    if (id < voc.V) {
      const uint32_t r = (uint32_t)voc.rank_of_id[id];
      a = (s_acc[r >> 5] >> (r & 31)) & 1u;
      u = (s_unc[r >> 5] >> (r & 31)) & 1u;
    }
    const unsigned long long ba = __ballot(a), bu = __ballot(u);
    if ((threadIdx.x & 63) == 0) {
      const int32_t w = id >> 5;
      acc_id[node * voc.W + w] = (uint32_t)ba;
      unc_id[node * voc.W + w] = (uint32_t)bu;
      if (w + 1 < voc.W) {
        acc_id[node * voc.W + w + 1] = (uint32_t)(ba >> 32);
        unc_id[node * voc.W + w + 1] = (uint32_t)(bu >> 32);
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
                                      uint16_t* __restrict__ list) {
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
    list[pos++] = (uint16_t)(threadIdx.x * 32 + b);
  }
}

__global__ void patch_classes_kernel(DevVocab voc, const uint32_t* __restrict__ items, int32_t n_items,
                                     uint32_t* acc_rank, uint32_t* unc_rank) {
  const int32_t k = blockIdx.x * blockDim.x + threadIdx.x;
  if (k >= n_items) return;
  const size_t node = items[3 * k];
  const uint32_t r = items[3 * k + 1], cls = items[3 * k + 2];
  const uint32_t bit = 1u << (r & 31);
  uint32_t* pa = acc_rank + node * voc.WR + (r >> 5);
  uint32_t* pu = unc_rank + node * voc.WR + (r >> 5);
  if (cls == (uint32_t)kAccept) atomicOr(pa, bit); else atomicAnd(pa, ~bit);
  if (cls == (uint32_t)kUncertain) atomicOr(pu, bit); else atomicAnd(pu, ~bit);
}

// ---------------------------------------------------------------- kernel (b)
constexpr int kFillThreads = 256;

// One workgroup owns the 128 mask words of one (request, chunk of 4096 token
// ids): it ORs the accepted bitsets of the tops of the request's stacks
// (Algorithm 1: union over parallel stacks), then walks that chunk's
// context-dependent tokens against each full stack and ORs in the survivors
// with LDS atomics, adds the stop tokens, and stores the words once,
// coalesced.  No global atomics, no second pass.
// COUNT = true additionally sums the automaton steps of all walks into
// *step_counter (instrumentation for the benchmark; never used on the hot path).
template <bool COUNT>
__global__ __launch_bounds__(kFillThreads) void fill_kernel(const RowDesc* __restrict__ rows,
                                                            const StackDesc* __restrict__ stacks,
                                                            const uint16_t* __restrict__ frames, DevVocab voc,
                                                            uint32_t* __restrict__ out, OverflowLog* log, uint32_t seq,
                                                            unsigned long long* step_counter) {
  unsigned long long my_steps = 0;
  __shared__ uint32_t words[kChunkWords];
  const int32_t b = blockIdx.y, chunk = blockIdx.x;
  const int32_t w0 = chunk * kChunkWords;
  const int32_t nw = min(kChunkWords, voc.W - w0);
  const RowDesc rd = rows[b];
  if (threadIdx.x < kChunkWords) words[threadIdx.x] = 0u;
  __syncthreads();
  if (rd.cache != nullptr) {
    const DevCache C = *rd.cache;
    for (uint32_t s = 0; s < rd.n_stacks; ++s) {
      const StackDesc sd = stacks[rd.stack_begin + s];
      const uint16_t* live = frames + sd.frame_off;
      const uint32_t top = live[sd.depth - 1];
      if ((int)threadIdx.x < nw) words[threadIdx.x] |= C.acc[(size_t)top * voc.W + w0 + threadIdx.x];
      __syncthreads();
      const uint32_t* po = C.unc_off + (size_t)top * (voc.n_chunk + 1) + chunk;
      const uint32_t j0 = po[0], j1 = po[1];
      for (uint32_t j = j0 + threadIdx.x; j < j1; j += kFillThreads) {
        const uint32_t lid = C.unc_list[j];
        if ((words[lid >> 5] >> (lid & 31)) & 1u) continue;  // already allowed by another stack
        const int32_t id = chunk * kChunkTokens + (int32_t)lid;
        const uint4 tk = voc.tok_by_id[id];
        int len = (int)(tk.w >> 24);
        const uint8_t* ext = voc.bytes;
        if (len >= 15) {
          ext = voc.bytes + voc.off_by_id[id];
          if (len == 255) len = (int)(voc.off_by_id[id + 1] - voc.off_by_id[id]);
        }
        uint32_t n_steps = 0;
        const int res = walk_token<false>(C.tab, tk, ext, len, top, live, sd.depth, COUNT ? &n_steps : nullptr);
        if (COUNT) my_steps += n_steps;
        if (res == kAccept) atomicOr(&words[lid >> 5], 1u << (lid & 31));
        else if (res == kOverflow) record_overflow(log, seq, (uint32_t)b, (uint32_t)id);
      }
      __syncthreads();
    }
  }
  if (rd.flags & 1u) {
    for (int32_t k = threadIdx.x; k < voc.n_stop; k += kFillThreads) {
      const int32_t rel = voc.stop_ids[k] - chunk * kChunkTokens;
      if (rel >= 0 && rel < nw * 32) atomicOr(&words[rel >> 5], 1u << (rel & 31));
    }
    __syncthreads();
  }
  if ((int)threadIdx.x < nw) out[(size_t)b * voc.W + w0 + threadIdx.x] = words[threadIdx.x];
  if (COUNT && my_steps) atomicAdd(step_counter, my_steps);
}

// ---------------------------------------------------------------- kernel (c)
constexpr int kApplyThreads = 256;

// Section 2.1: logits of disallowed tokens become -inf.  One thread owns 16
// bytes of a logits row (8 bf16/fp16 or 4 fp32 elements) and the matching mask
// bits.  All allowed: nothing is touched.  None allowed: one 16-byte store of
// the -inf pattern, no read.  Mixed: read, blend, write.  ESIZE = bytes per
// element.
template <int ESIZE>
__global__ __launch_bounds__(kApplyThreads) void apply_kernel(unsigned char* __restrict__ logits, int64_t row_stride,
                                                              const uint32_t* __restrict__ bitmask, int32_t W_mask,
                                                              int32_t V_logits, int32_t V_mask,
                                                              const int32_t* __restrict__ row_index, uint32_t neg_inf) {
  constexpr int EPT = 16 / ESIZE;  // elements per thread
  const int32_t j = blockIdx.y;
  const int64_t lrow = row_index ? row_index[j] : j;
  const int32_t g = blockIdx.x * kApplyThreads + threadIdx.x;
  const int32_t e0 = g * EPT;
  if (e0 >= V_logits) return;
  uint32_t m = 0;
  if (e0 < V_mask) {
    m = (bitmask[(size_t)j * W_mask + (e0 >> 5)] >> (e0 & 31)) & ((1u << EPT) - 1u);
    if (e0 + EPT > V_mask) m &= (1u << (V_mask - e0)) - 1u;
  }
  unsigned char* p = logits + ((size_t)lrow * row_stride + e0) * ESIZE;
  if (e0 + EPT <= V_logits) {
    if (m == (1u << EPT) - 1u) return;
    uint4 v;
    if (ESIZE == 2) {
      const uint32_t two = neg_inf | (neg_inf << 16);
      if (m == 0) v = make_uint4(two, two, two, two);
      else {
        v = *reinterpret_cast<const uint4*>(p);
        uint32_t* q = reinterpret_cast<uint32_t*>(&v);
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const uint32_t keep = ((m >> (2 * k)) & 1u ? 0x0000FFFFu : 0u) | ((m >> (2 * k + 1)) & 1u ? 0xFFFF0000u : 0u);
          q[k] = (q[k] & keep) | (two & ~keep);
        }
      }
    } else {
      if (m == 0) v = make_uint4(neg_inf, neg_inf, neg_inf, neg_inf);
      else {
        v = *reinterpret_cast<const uint4*>(p);
        if (!(m & 1u)) v.x = neg_inf;
        if (!(m & 2u)) v.y = neg_inf;
        if (!(m & 4u)) v.z = neg_inf;
        if (!(m & 8u)) v.w = neg_inf;
      }
    }
    *reinterpret_cast<uint4*>(p) = v;
  } else {
    for (int k = 0; e0 + k < V_logits; ++k)
      if (!((m >> k) & 1u)) {
        if (ESIZE == 2) reinterpret_cast<uint16_t*>(p)[k] = (uint16_t)neg_inf;
        else reinterpret_cast<uint32_t*>(p)[k] = neg_inf;
      }
  }
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

}  // namespace

// ------------------------------------------------------------------ launchers
void launch_classify(const DevTables& tab, size_t table_bytes, int32_t n_rows_tab, int32_t n_alts,
                     int32_t n_nodes_total, const DevVocab& voc, int32_t node0, int32_t n, uint32_t* acc_rank,
                     uint32_t* unc_rank, OverflowLog* log, uint32_t seq, hipStream_t stream) {
  if (n <= 0 || voc.V <= 0) return;
  dim3 grid((voc.V + kClassifyThreads - 1) / kClassifyThreads, (n + kNodesPerBlock - 1) / kNodesPerBlock);
  if (table_bytes <= 64 * 1024) {
    hipLaunchKernelGGL(classify_kernel<true>, grid, dim3(kClassifyThreads), table_bytes, stream, tab, n_nodes_total,
                       n_rows_tab, n_alts, voc, node0, n, acc_rank, unc_rank, log, seq);
  } else {
    hipLaunchKernelGGL(classify_kernel<false>, grid, dim3(kClassifyThreads), 0, stream, tab, n_nodes_total,
                       n_rows_tab, n_alts, voc, node0, n, acc_rank, unc_rank, log, seq);
  }
}

void launch_permute(const DevVocab& voc, int32_t n, const uint32_t* acc_rank, const uint32_t* unc_rank,
                    uint32_t* acc_id, uint32_t* unc_id, hipStream_t stream) {
  if (n <= 0) return;
  size_t lds = (size_t)voc.WR * 8;
  hipLaunchKernelGGL(permute_kernel, dim3(n), dim3(kPermuteThreads), lds, stream, voc, acc_rank, unc_rank, acc_id,
                     unc_id);
}

void launch_count_uncertain(const DevVocab& voc, int32_t n, const uint32_t* unc_id, uint32_t* counts,
                            hipStream_t stream) {
  if (n <= 0) return;
  hipLaunchKernelGGL(count_uncertain_kernel, dim3(voc.n_chunk, n), dim3(kChunkWords), 0, stream, voc, unc_id, counts);
}

void launch_list_uncertain(const DevVocab& voc, int32_t n, const uint32_t* unc_id, const uint32_t* off,
                           uint16_t* list, hipStream_t stream) {
  if (n <= 0) return;
  hipLaunchKernelGGL(list_uncertain_kernel, dim3(voc.n_chunk, n), dim3(kChunkWords), 0, stream, voc, unc_id, off, list);
}

void launch_patch_classes(const DevVocab& voc, const uint32_t* items, int32_t n_items, uint32_t* acc_rank,
                          uint32_t* unc_rank, hipStream_t stream) {
  if (n_items <= 0) return;
  hipLaunchKernelGGL(patch_classes_kernel, dim3((n_items + 255) / 256), dim3(256), 0, stream, voc, items, n_items,
                     acc_rank, unc_rank);
}

void launch_fill(const RowDesc* rows, const StackDesc* stacks, const uint16_t* frames, int32_t B, const DevVocab& voc,
                 uint32_t* out, OverflowLog* log, uint32_t seq, unsigned long long* step_counter, hipStream_t stream) {
  if (B <= 0 || voc.n_chunk <= 0) return;
  if (step_counter)
    hipLaunchKernelGGL(fill_kernel<true>, dim3(voc.n_chunk, B), dim3(kFillThreads), 0, stream, rows, stacks, frames,
                       voc, out, log, seq, step_counter);
  else
    hipLaunchKernelGGL(fill_kernel<false>, dim3(voc.n_chunk, B), dim3(kFillThreads), 0, stream, rows, stacks, frames,
                       voc, out, log, seq, step_counter);
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
    dim3 grid((groups + kApplyThreads - 1) / kApplyThreads, n_rows);
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
