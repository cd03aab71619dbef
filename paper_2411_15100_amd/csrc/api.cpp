// C ABI (include/xgm.h): handles, device memory, staging, error translation.
#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <array>
#include <atomic>
#include <chrono>
#include <cstring>
#include <deque>
#include <mutex>
#include <numeric>
#include <string>
#include <set>
#include <unordered_map>
#include <vector>

#include "../../include/xgm.h"
#include "automaton.hpp"
#include "engine.hpp"
#include "schema.hpp"
#include "kernels.hpp"
#include "walk.hpp"

using namespace xgm;

namespace {

thread_local std::string g_error;

void hip_check(hipError_t e, const char* what) {
  if (e != hipSuccess) throw Failure(XGM_ERR_HIP, std::string(what) + ": " + hipGetErrorString(e));
}
#define HIP_OK(call) hip_check((call), #call)

template <class T>
T* dev_alloc(size_t n) {
  void* p = nullptr;
  HIP_OK(hipMalloc(&p, std::max<size_t>(n, 1) * sizeof(T)));
  return static_cast<T*>(p);
}
template <class T>
T* dev_upload(const std::vector<T>& v) {
  T* p = dev_alloc<T>(v.size());
  if (!v.empty()) HIP_OK(hipMemcpy(p, v.data(), v.size() * sizeof(T), hipMemcpyHostToDevice));
  return p;
}

// Long-lived device data (vocabulary arrays, automaton tables, cache bitsets
// and lists) is carved out of 256 MiB slabs instead of one hipMalloc per
// array: the small tables of many grammars then sit side by side in memory
// that the driver maps with large pages, so the token walks' scattered table
// reads do not thrash the GPU's address translation caches.  A slab is freed
// when the last array in it has been released.
class SlabAllocator {
 public:
  static constexpr size_t kSlab = (size_t)256 << 20;
  void* alloc(size_t bytes) {
    bytes = std::max<size_t>((bytes + 255) & ~(size_t)255, 256);
    std::lock_guard<std::mutex> lock(mu_);
    if (bytes > kSlab / 2) {  // big arrays get their own allocation (large pages anyway)
      void* p = nullptr;
      hip_check(hipMalloc(&p, bytes), "hipMalloc");
      slabs_.push_back({(char*)p, bytes, bytes, 1});
      return p;
    }
    if (cur_ < 0 || slabs_[cur_].used + bytes > slabs_[cur_].size) {
      void* p = nullptr;
      hip_check(hipMalloc(&p, kSlab), "hipMalloc");
      slabs_.push_back({(char*)p, kSlab, 0, 0});
      cur_ = (int)slabs_.size() - 1;
    }
    Slab& s = slabs_[cur_];
    void* out = s.base + s.used;
    s.used += bytes;
    ++s.live;
    return out;
  }
  void release(void* ptr) {
    std::lock_guard<std::mutex> lock(mu_);
    for (size_t k = 0; k < slabs_.size(); ++k) {
      Slab& s = slabs_[k];
      if ((char*)ptr < s.base || (char*)ptr >= s.base + s.size) continue;
      if (--s.live > 0) return;
      if ((int)k == cur_) { s.used = 0; return; }  // keep the current slab for reuse
      (void)hipFree(s.base);
      slabs_.erase(slabs_.begin() + k);
      if (cur_ > (int)k) --cur_;
      return;
    }
  }

 private:
  struct Slab { char* base; size_t size, used; int live; };
  std::mutex mu_;
  std::vector<Slab> slabs_;
  int cur_ = -1;
};
SlabAllocator& slab() {
  static SlabAllocator a;
  return a;
}
template <class T>
T* slab_alloc(size_t n) { return static_cast<T*>(slab().alloc(std::max<size_t>(n, 1) * sizeof(T))); }
template <class T>
T* slab_upload(const std::vector<T>& v) {
  T* p = slab_alloc<T>(v.size());
  if (!v.empty()) HIP_OK(hipMemcpy(p, v.data(), v.size() * sizeof(T), hipMemcpyHostToDevice));
  return p;
}

// Temporary device memory of the cache builds: one block that is reused by every build and grows to what
// the largest build so far needed (allocating and freeing two dozen arrays per build costs more than the
// kernels of a small grammar take).  Builds are serialised by `mu`.
class TempArena {
 public:
  std::mutex mu;
  void* alloc(size_t bytes) {
    bytes = std::max<size_t>((bytes + 255) & ~(size_t)255, 256);
    wanted_ += bytes;
    if (used_ + bytes <= cap_) {
      void* p = base_ + used_;
      used_ += bytes;
      return p;
    }
    void* p = nullptr;
    hip_check(hipMalloc(&p, bytes), "hipMalloc");
    extra_.push_back(p);
    return p;
  }
  // after a build (the stream is idle): blocks of their own are freed and the main block grows
  void reset() {
    for (void* p : extra_) (void)hipFree(p);
    extra_.clear();
    host_keep_.clear();
    if (wanted_ > cap_) {
      if (base_) (void)hipFree(base_);
      base_ = nullptr;
      cap_ = 0;
      void* p = nullptr;
      const size_t want = wanted_ + wanted_ / 4;
      if (hipMalloc(&p, want) == hipSuccess) { base_ = (char*)p; cap_ = want; }
    }
    used_ = wanted_ = 0;
  }
  template <class T>
  T* array(size_t n) { return static_cast<T*>(alloc(std::max<size_t>(n, 1) * sizeof(T))); }
  // (the host bytes are kept until reset(), so that the copy may run whenever the stream gets to it)
  template <class T>
  T* upload(const std::vector<T>& v, hipStream_t stream) {
    T* p = array<T>(v.size());
    if (!v.empty()) {
      host_keep_.emplace_back((const char*)v.data(), (const char*)v.data() + v.size() * sizeof(T));
      hip_check(hipMemcpyAsync(p, host_keep_.back().data(), v.size() * sizeof(T), hipMemcpyHostToDevice, stream), "hipMemcpyAsync");
    }
    return p;
  }

 private:
  char* base_ = nullptr;
  size_t cap_ = 0, used_ = 0, wanted_ = 0;
  std::vector<void*> extra_;
  std::deque<std::vector<char>> host_keep_;
};
TempArena& temp_arena() {
  static TempArena a;
  return a;
}

void require_device() {
  static std::atomic<bool> found{false};  // (asked once: the per-step calls come through here too)
  if (found.load(std::memory_order_relaxed)) return;
  int n = 0;
  hipError_t e = hipGetDeviceCount(&n);
  if (e != hipSuccess || n <= 0)
    throw Failure(XGM_ERR_HIP, "no HIP device: the mask kernels have no CPU path");
  found.store(true, std::memory_order_relaxed);
}

}  // namespace

// ------------------------------------------------------------------ handles
struct xgm_vocab {
  std::atomic<int> refs{1};
  int32_t V = 0;
  std::vector<uint8_t> bytes;
  std::vector<uint32_t> off;  // [V+1]
  std::vector<int32_t> stop;
  std::vector<char> is_stop;
  std::vector<int32_t> rank_of_id, id_of_rank;
  std::mutex mu;
  bool on_device = false;
  DevVocab dv{};
  std::vector<void*> dev_ptrs;
  ~xgm_vocab();
};
struct xgm_grammar {
  std::atomic<int> refs{1};
  Automaton A;
};
struct xgm_cache {
  std::atomic<int> refs{1};
  xgm_grammar* g = nullptr;
  xgm_vocab* v = nullptr;
  DevCache host{};           // device pointers and table layout
  std::vector<void*> dev_ptrs;
  // host copies of what packing a stack header needs (see DevCache)
  std::vector<uint16_t> acc_row_host;  // [n_nodes]
  std::vector<uint32_t> key_off_host;  // [n_keys * n_seg + 1]
  std::vector<uint32_t> k_base_host[kCtxLevels];  // [n_nodes] (kNoKey for a node without context-dependent tokens), [n_k[0]], ...
  int levels = 0;                      // levels of per-context lists kept (<= kCtxLevels)
  std::vector<uint32_t> unc_count;     // [n_nodes] context-dependent tokens
  int32_t n_acc_rows = 0;
  int64_t device_bytes = 0;            // device memory the cache holds
  int64_t stats[8] = {0, 0, 0, 0, 0, 0, 0, 0};  // see xgm_cache_stats
  std::vector<uint32_t> plain_count;   // [n_nodes] tokens that only section 3.1 calls context-dependent
  uint32_t* d_plain_id = nullptr;      // [n_nodes][W] their bitsets, if kept
  uint32_t* d_unc_id = nullptr;        // [n_nodes][W] the context-dependent tokens, if kept
  int64_t host_classified = 0;
  double kernel_seconds = 0.0;
  double build_seconds = 0.0;
  double classify_seconds = 0.0;
};
struct xgm_matcher {
  xgm_cache* c = nullptr;
  xgm_grammar* g = nullptr;
  xgm_vocab* v = nullptr;
  std::vector<Stack> stacks;
  bool terminated = false;
};

// device-resident states of a fixed batch of requests
struct xgm_batch {
  int32_t B = 0, H = 0;
  xgm_vocab* v = nullptr;
  std::vector<xgm_cache*> caches;  // one per row (referenced)
  DevBatch dev{};
  std::vector<void*> dev_ptrs;
  // walks over the on-chip limits: the batch's own log, how much of it has been examined, and where the last
  // fills wrote their masks (by sequence number)
  uint32_t seen_count = 0;
  static constexpr int kFills = 8;
  uint32_t fill_seq[kFills] = {};
  int32_t* fill_bitmask[kFills] = {};
  int next_fill = 0;
};

xgm_vocab::~xgm_vocab() { for (void* p : dev_ptrs) slab().release(p); }

namespace {

void release(xgm_vocab* v) { if (v && --v->refs == 0) delete v; }
void release(xgm_grammar* g) { if (g && --g->refs == 0) delete g; }
void release(xgm_cache* c) {
  if (c && --c->refs == 0) {
    for (void* p : c->dev_ptrs) slab().release(p);
    release(c->g);
    release(c->v);
    delete c;
  }
}

void vocab_to_device(xgm_vocab* v) {
  std::lock_guard<std::mutex> lock(v->mu);
  if (v->on_device) return;
  require_device();
  const int32_t V = v->V;
  auto row_of = [&](int32_t id) {
    uint4 r = make_uint4(0, 0, 0, 0);
    unsigned char b[16] = {0};
    uint32_t len = v->off[id + 1] - v->off[id];
    for (uint32_t k = 0; k < std::min<uint32_t>(len, 15); ++k) b[k] = v->bytes[v->off[id] + k];
    b[15] = (unsigned char)std::min<uint32_t>(len, 255);
    std::memcpy(&r, b, 16);
    return r;
  };
  std::vector<uint4> by_id(V), by_rank(V);
  for (int32_t i = 0; i < V; ++i) by_id[i] = row_of(i);
  for (int32_t r = 0; r < V; ++r) by_rank[r] = by_id[v->id_of_rank[r]];
  DevVocab& d = v->dv;
  auto keep = [&](auto* p) { v->dev_ptrs.push_back((void*)p); return p; };
  d.tok_by_id = keep(slab_upload(by_id));
  d.tok_by_rank = keep(slab_upload(by_rank));
  d.off_by_id = keep(slab_upload(v->off));
  d.bytes = keep(slab_upload(v->bytes));
  std::vector<uint8_t> first(V, 0);
  for (int32_t i = 0; i < V; ++i)
    if (v->off[i + 1] > v->off[i]) first[i] = v->bytes[v->off[i]];
  d.first_by_id = keep(slab_upload(first));
  d.rank_of_id = keep(slab_upload(v->rank_of_id));
  d.id_of_rank = keep(slab_upload(v->id_of_rank));
  d.stop_ids = keep(slab_upload(v->stop));
  d.n_stop = (int32_t)v->stop.size();
  d.V = V;
  d.W = (V + 31) / 32;
  d.WR = ((V + 63) / 64) * 2;
  d.n_seg = (d.W + kSegWords - 1) / kSegWords;
  v->on_device = true;
}

// --- process-wide device context: the fill staging ring and the record of walks over the limits
// What xgm_fill_overflow_fixup needs to decide the records of one fill from host-side states: the packed
// stacks (in the staging memory the fill used), where the mask went, and the caches (kept alive until the
// staging memory is used again).
struct PendingFill {
  uint32_t seq = 0;          // 0: none
  int32_t B = 0;
  int32_t* d_bitmask = nullptr;
  const void* blob = nullptr;
  std::vector<xgm_cache*> caches;  // referenced
};
struct FillSlot {
  void* h_buf = nullptr;  // pinned
  void* h_dev = nullptr;  // the same memory as the device addresses it
  void* d_buf = nullptr;
  size_t cap = 0;
  hipEvent_t done = nullptr;
  bool used = false;
  PendingFill fill;
};
struct Context {
  std::mutex mu;
  OverflowLog* d_log = nullptr;  // records of the fills from host-side states
  uint32_t seq = 0;
  uint32_t seen_count = 0;  // entries of d_log already examined by a fixup
  static constexpr int kSlots = 8;
  FillSlot slot[kSlots];
  int next_slot = 0;
  PendingFill static_fill;  // the last fill staged in the static arrays
  // records of logs that no longer exist (cache builds, destroyed batches), and the batches that do
  int64_t retired_records = 0;
  std::set<xgm_batch*> batches;
};
Context& ctx() {
  static Context c;
  return c;
}
OverflowLog* new_log() {
  require_device();
  OverflowLog* log = dev_alloc<OverflowLog>(1);
  HIP_OK(hipMemset(log, 0, sizeof(OverflowLog)));
  return log;
}
OverflowLog* overflow_log() {
  Context& c = ctx();
  if (!c.d_log) c.d_log = new_log();
  return c.d_log;
}
uint32_t read_overflow_count(const OverflowLog* log) {
  uint32_t n = 0;
  HIP_OK(hipMemcpy(&n, &log->count, sizeof(n), hipMemcpyDeviceToHost));
  return n;
}
void set_pending(PendingFill& f, uint32_t seq, int32_t B, int32_t* d_bitmask, const void* blob, xgm_matcher* const* ms) {
  for (xgm_cache* c : f.caches) release(c);
  f.caches.clear();
  f.seq = seq;
  f.B = B;
  f.d_bitmask = d_bitmask;
  f.blob = blob;
  for (int32_t b = 0; b < B; ++b) { ++ms[b]->c->refs; f.caches.push_back(ms[b]->c); }
}

int fail(const Failure& f) {
  g_error = f.what();
  return f.status;
}
int fail(int status, const std::string& msg) {
  g_error = msg;
  return status;
}

}  // namespace

#define API_BEGIN try {
#define API_END                                                                        \
  }                                                                                    \
  catch (const Failure& f) { return fail(f); }                                         \
  catch (const std::bad_alloc&) { return fail(XGM_ERR_INTERNAL, "out of host memory"); } \
  catch (const std::exception& e) { return fail(XGM_ERR_INTERNAL, e.what()); }

extern "C" {

const char* xgm_last_error(void) { return g_error.c_str(); }
int32_t xgm_bitmask_words(int32_t V) { return V <= 0 ? 0 : (V + 31) / 32; }

// ---------------------------------------------------------------- vocabulary
int xgm_vocab_create(const uint8_t* h_bytes, const int64_t* h_offsets, int32_t V, const int32_t* h_stop_ids,
                     int32_t n_stop, xgm_vocab** out) {
  API_BEGIN
  if (!out) return fail(XGM_ERR_BAD_ARG, "vocab_create: out is null");
  *out = nullptr;
  if (V <= 0 || !h_offsets) return fail(XGM_ERR_BAD_ARG, "vocab_create: V must be positive and offsets non-null");
  if (V > XGM_MAX_VOCAB) return fail(XGM_ERR_TOO_LARGE, "vocab_create: more than XGM_MAX_VOCAB tokens");
  if (n_stop < 0 || (n_stop > 0 && !h_stop_ids)) return fail(XGM_ERR_BAD_ARG, "vocab_create: bad stop ids");
  if (h_offsets[0] != 0) return fail(XGM_ERR_BAD_ARG, "vocab_create: offsets[0] must be 0");
  for (int32_t i = 0; i < V; ++i)
    if (h_offsets[i + 1] < h_offsets[i]) return fail(XGM_ERR_BAD_ARG, "vocab_create: offsets must not decrease");
  if (h_offsets[V] > 0 && !h_bytes) return fail(XGM_ERR_BAD_ARG, "vocab_create: bytes is null");
  if (h_offsets[V] >= (int64_t)1 << 31) return fail(XGM_ERR_TOO_LARGE, "vocab_create: more than 2 GiB of token bytes");
  auto v = new xgm_vocab();
  v->V = V;
  v->bytes.assign(h_bytes, h_bytes + h_offsets[V]);
  v->off.resize(V + 1);
  for (int32_t i = 0; i <= V; ++i) v->off[i] = (uint32_t)h_offsets[i];
  v->is_stop.assign(V, 0);
  for (int32_t k = 0; k < n_stop; ++k) {
    if (h_stop_ids[k] < 0 || h_stop_ids[k] >= V) { delete v; return fail(XGM_ERR_BAD_ARG, "vocab_create: stop id out of range"); }
    if (!v->is_stop[h_stop_ids[k]]) { v->is_stop[h_stop_ids[k]] = 1; v->stop.push_back(h_stop_ids[k]); }
  }
  v->id_of_rank.resize(V);
  std::iota(v->id_of_rank.begin(), v->id_of_rank.end(), 0);
  const uint8_t* base = v->bytes.data();
  const std::vector<uint32_t>& off = v->off;
  std::stable_sort(v->id_of_rank.begin(), v->id_of_rank.end(), [&](int32_t a, int32_t b) {
    size_t la = off[a + 1] - off[a], lb = off[b + 1] - off[b];
    int c = std::memcmp(base + off[a], base + off[b], std::min(la, lb));
    return c != 0 ? c < 0 : la < lb;
  });
  v->rank_of_id.resize(V);
  for (int32_t r = 0; r < V; ++r) v->rank_of_id[v->id_of_rank[r]] = r;
  *out = v;
  return XGM_OK;
  API_END
}
void xgm_vocab_destroy(xgm_vocab* v) { release(v); }
int32_t xgm_vocab_size(const xgm_vocab* v) { return v ? v->V : XGM_ERR_BAD_ARG; }

// ------------------------------------------------------------------- grammar
int xgm_grammar_compile(const char* text, size_t len, const char* root_rule, xgm_grammar** out) {
  API_BEGIN
  if (!out) return fail(XGM_ERR_BAD_ARG, "grammar_compile: out is null");
  *out = nullptr;
  if (!text || !root_rule) return fail(XGM_ERR_BAD_ARG, "grammar_compile: null text or root rule");
  auto g = new xgm_grammar();
  try {
    g->A = compile_grammar(std::string(text, len), root_rule);
  } catch (...) {
    delete g;
    throw;
  }
  *out = g;
  return XGM_OK;
  API_END
}
void xgm_grammar_destroy(xgm_grammar* g) { release(g); }
int32_t xgm_grammar_num_nodes(const xgm_grammar* g) { return g ? g->A.n_nodes : XGM_ERR_BAD_ARG; }
int32_t xgm_grammar_num_rules(const xgm_grammar* g) { return g ? (int32_t)g->A.rule_names.size() : XGM_ERR_BAD_ARG; }
const char* xgm_grammar_rule_name(const xgm_grammar* g, int32_t r) {
  if (!g || r < 0 || r >= (int32_t)g->A.rule_names.size()) return nullptr;
  return g->A.rule_names[r].c_str();
}
int32_t xgm_grammar_node_rule(const xgm_grammar* g, int32_t node) {
  if (!g || node < 0 || node >= g->A.n_nodes) return fail(XGM_ERR_BAD_ARG, "node out of range");
  return g->A.node_rule[node];
}
int32_t xgm_grammar_node_path(const xgm_grammar* g, int32_t node, int32_t* h_out, int32_t cap) {
  if (!g || node < 0 || node >= g->A.n_nodes || cap < 0 || (cap > 0 && !h_out)) return fail(XGM_ERR_BAD_ARG, "node_path: bad argument");
  const auto& p = g->A.node_path[node];
  for (int32_t k = 0; k < std::min<int32_t>(cap, (int32_t)p.size()); ++k) h_out[k] = p[k];
  return (int32_t)p.size();
}
int32_t xgm_grammar_node_is_final(const xgm_grammar* g, int32_t node) {
  if (!g || node < 0 || node >= g->A.n_nodes) return fail(XGM_ERR_BAD_ARG, "node out of range");
  return g->A.node_final[node];
}

int xgm_debug_classify_host(const xgm_grammar* g, int32_t node, const uint8_t* h_bytes, int32_t n) {
  API_BEGIN
  if (!g || node < 0 || node >= g->A.n_nodes || n < 0 || (n > 0 && !h_bytes)) return fail(XGM_ERR_BAD_ARG, "classify_host: bad argument");
  int cls = Engine(&g->A).classify(node, h_bytes, n);
  if (cls < 0) return fail(XGM_ERR_TOO_LARGE, "classify_host: configuration limit exceeded");
  return cls;
  API_END
}

int xgm_schema_to_grammar(const char* schema_json, size_t len, char* h_text, size_t cap, size_t* h_len) {
  API_BEGIN
  if (!schema_json || !h_len || (cap > 0 && !h_text)) return fail(XGM_ERR_BAD_ARG, "schema_to_grammar: null argument");
  const std::string text = schema_to_grammar(std::string(schema_json, len));
  *h_len = text.size();
  if (cap < text.size() + 1) return cap == 0 ? XGM_OK : fail(XGM_ERR_BAD_ARG, "schema_to_grammar: the output buffer is too small");
  std::memcpy(h_text, text.data(), text.size());
  h_text[text.size()] = 0;
  return XGM_OK;
  API_END
}

int32_t xgm_debug_context_index(const xgm_grammar* g, int32_t top, int32_t below) {
  if (!g || top < 0 || top >= g->A.n_nodes || below < 0 || below >= g->A.n_nodes)
    return fail(XGM_ERR_BAD_ARG, "context_index: bad argument");
  const auto& ctx = g->A.contexts[g->A.node_rule[top]];
  auto it = std::lower_bound(ctx.begin(), ctx.end(), below);
  if (it == ctx.end() || *it != below) return -1000;
  return (int32_t)(it - ctx.begin());
}

int xgm_debug_walk_host(const xgm_grammar* g, const int32_t* h_stack, int32_t depth, const uint8_t* h_bytes,
                        int32_t n, int32_t build, int32_t* h_steps) {
  API_BEGIN
  if (!g || !h_stack || depth < 1 || depth > XGM_MAX_STACK_DEPTH || n < 0 || (n > 0 && !h_bytes))
    return fail(XGM_ERR_BAD_ARG, "walk_host: bad argument");
  if (build && depth != 1) return fail(XGM_ERR_BAD_ARG, "walk_host: the classifying walk starts from a single node");
  const Automaton& A = g->A;
  std::vector<uint16_t> live(depth);
  for (int32_t k = 0; k < depth; ++k) {
    if (h_stack[k] < 0 || h_stack[k] >= A.n_nodes) return fail(XGM_ERR_BAD_ARG, "walk_host: node out of range");
    live[k] = (uint16_t)h_stack[k];
  }
  if (n == 0) return kReject;
  const CompactTab T{TabView{reinterpret_cast<const uint2*>(A.hdr.data()), A.n_nodes,
                             reinterpret_cast<const uint2*>(A.hdr.data()), A.cls.data(), A.shapes.data(),
                             A.targets.data(), A.alts.data(), A.follow_words.data(), A.n_cls}};
  unsigned char row[16] = {0};
  std::memcpy(row, h_bytes, std::min<int32_t>(n, 15));
  row[15] = (unsigned char)std::min<int32_t>(n, 255);
  uint4 tk;
  std::memcpy(&tk, row, 16);
  uint32_t steps = 0;
  const int rc = build ? walk_token<true>(T, tk, h_bytes, n, live[depth - 1], (const uint16_t*)nullptr, 1u, &steps, T.follow_of(live[depth - 1]))
                       : walk_token<false>(T, tk, h_bytes, n, live[depth - 1], live.data(), (uint32_t)depth, &steps);
  if (h_steps) *h_steps = (int32_t)steps;
  return rc;
  API_END
}

namespace {
struct HostStackSink {
  uint16_t* frames;
  uint32_t* depth;
  uint32_t* count;
  uint32_t* overflow;
  uint32_t capacity, max_depth;
  uint32_t claim() { return (*count)++; }
};
}  // namespace

int xgm_debug_matcher_accept_token_walk(xgm_matcher* m, int32_t token_id) {
  API_BEGIN
  if (!m || !m->v) return fail(XGM_ERR_BAD_ARG, "accept_token_walk: matcher has no vocabulary");
  if (token_id < 0 || token_id >= m->v->V) return fail(XGM_ERR_BAD_ARG, "accept_token_walk: token id out of range");
  if (m->terminated) return fail(XGM_ERR_TERMINATED, "accept: the matcher has terminated");
  const xgm_vocab& v = *m->v;
  const Automaton& A = m->g->A;
  if (v.is_stop[token_id]) {
    if (!Engine(&A).can_terminate(m->stacks)) return fail(XGM_ERR_TOKEN_REJECTED, "accept: stop token before the text is complete");
    m->terminated = true;
    return XGM_OK;
  }
  const int32_t n = (int32_t)(v.off[token_id + 1] - v.off[token_id]);
  if (n == 0) return fail(XGM_ERR_TOKEN_REJECTED, "accept: a token without bytes is never allowed");
  const uint8_t* bytes = v.bytes.data() + v.off[token_id];
  const CompactTab T{TabView{reinterpret_cast<const uint2*>(A.hdr.data()), A.n_nodes,
                             reinterpret_cast<const uint2*>(A.hdr.data()), A.cls.data(), A.shapes.data(),
                             A.targets.data(), A.alts.data(), A.follow_words.data(), A.n_cls}};
  unsigned char row[16] = {0};
  std::memcpy(row, bytes, std::min<int32_t>(n, 15));
  row[15] = (unsigned char)std::min<int32_t>(n, 255);
  uint4 tk;
  std::memcpy(&tk, row, 16);
  std::vector<uint16_t> cand((size_t)kBatchMaxCandidates * kBatchMaxDepth);
  std::vector<uint32_t> depth(kBatchMaxCandidates);
  uint32_t count = 0, overflow = 0;
  HostStackSink sink{cand.data(), depth.data(), &count, &overflow, kBatchMaxCandidates, kBatchMaxDepth};
  const CollectStacks<CompactTab, HostStackSink> collect{&T, &sink};
  std::set<Stack> next;
  for (const Stack& s : m->stacks) {
    std::vector<uint16_t> live(s.begin(), s.end());
    count = 0;
    const int rc = walk_token<false>(T, tk, bytes, n, live.back(), live.data(), (uint32_t)live.size(), (uint32_t*)nullptr,
                                     0u, 0, (uint32_t*)nullptr, collect);
    if (rc == kOverflow || overflow) return fail(XGM_ERR_TOO_LARGE, "accept_token_walk: the walk exceeded its limits");
    for (uint32_t k = 0; k < count; ++k)
      next.insert(Stack(cand.begin() + (size_t)k * kBatchMaxDepth, cand.begin() + (size_t)k * kBatchMaxDepth + depth[k]));
  }
  if (next.empty()) return fail(XGM_ERR_TOKEN_REJECTED, "accept: the bytes are not allowed here");
  m->stacks.assign(next.begin(), next.end());
  return XGM_OK;
  API_END
}

// --------------------------------------------------------------------- cache
namespace {
std::atomic<int32_t> g_build_batch_nodes{0};  // test knob: nodes classified per batch (0: as many as 1 GiB of rows holds)
}
void xgm_debug_set_build_batch_nodes(int32_t nodes) { g_build_batch_nodes = nodes > 0 ? nodes : 0; }

int xgm_cache_build(xgm_grammar* g, xgm_vocab* v, void* hip_stream, xgm_cache** out) {
  return xgm_cache_build_ex(g, v, hip_stream, 0, out);
}

int xgm_cache_build_ex(xgm_grammar* g, xgm_vocab* v, void* hip_stream, uint32_t flags, xgm_cache** out) {
  API_BEGIN
  if (!out) return fail(XGM_ERR_BAD_ARG, "cache_build: out is null");
  *out = nullptr;
  if (!g || !v) return fail(XGM_ERR_BAD_ARG, "cache_build: null grammar or vocabulary");
  require_device();
  const auto t_build0 = std::chrono::steady_clock::now();
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  vocab_to_device(v);
  const DevVocab& dv = v->dv;
  const Automaton& A = g->A;
  const int32_t N = A.n_nodes;

  auto c = new xgm_cache();
  c->g = g; ++g->refs;
  c->v = v; ++v->refs;
  TempArena& arena = temp_arena();
  std::lock_guard<std::mutex> build_lock(arena.mu);
  auto cleanup_temps = [&] { (void)hipStreamSynchronize(stream); arena.reset(); };
  try {
    auto keep = [&](auto* p) { c->dev_ptrs.push_back((void*)p); return p; };
    // automaton tables
    static_assert(sizeof(NodeHdr) == sizeof(uint2), "header layout");
    DevTables tab{};
    size_t image_bytes = 0;
    {
      std::vector<unsigned char> img;
      auto put = [&](const void* src, size_t bytes, size_t align) {
        img.resize((img.size() + align - 1) / align * align, 0);
        const size_t at = img.size();
        img.insert(img.end(), (const unsigned char*)src, (const unsigned char*)src + bytes);
        return (uint32_t)at;
      };
      if (A.cls.size() != 256 || A.follow_words.size() != A.rule_names.size() * 8)
        throw Failure(XGM_ERR_INTERNAL, "cache_build: inconsistent automaton tables");
      put(A.cls.data(), 256, 4);
      tab.off_shapes = put(A.shapes.data(), A.shapes.size(), 4);
      tab.off_targets = put(A.targets.data(), A.targets.size() * 2, 4);
      tab.off_follow = put(A.follow_words.data(), A.follow_words.size() * 4, 4);
      tab.off_alts = put(A.alts.data(), A.alts.size() * 4, 4);
      tab.off_hdr = put(A.hdr.data(), (size_t)N * sizeof(uint2), 16);
      tab.off_first = put(A.node_first_words.data(), A.node_first_words.size() * 4, 16);
      img.resize((img.size() + 15) / 16 * 16, 0);
      image_bytes = img.size();
      std::vector<uint4> image(img.size() / 16);
      std::memcpy(image.data(), img.data(), img.size());
      tab.image = keep(slab_upload(image));
      tab.n_rules = (int32_t)A.rule_names.size();
      tab.n_cls = A.n_cls;
      tab.n_nodes = N;
    }

    const int32_t n_seg = dv.n_seg;
    uint32_t* acc_id = arena.array<uint32_t>((size_t)N * dv.W);  // one row per node
    const bool keep_plain = (flags & XGM_CACHE_KEEP_PLAIN) != 0;
    uint32_t* unc_id = keep_plain ? (c->d_unc_id = keep(slab_alloc<uint32_t>((size_t)N * dv.W))) : arena.array<uint32_t>((size_t)N * dv.W);
    // rank-space scratch for a batch of nodes (at most 1 GiB for both bitsets)
    const size_t row_bytes = (size_t)dv.WR * 4;
    int32_t batch = (int32_t)std::max<size_t>(32, std::min<size_t>((size_t)N, ((size_t)512 << 20) / row_bytes));
    if (g_build_batch_nodes > 0) batch = std::max(32, std::min(N, g_build_batch_nodes.load()));
    if (batch < N) batch &= ~31;  // (the classify kernel wants batches of nodes to begin at multiples of 32)
    uint32_t* acc_rank = arena.array<uint32_t>((size_t)batch * dv.WR);
    uint32_t* unc_rank = arena.array<uint32_t>((size_t)batch * dv.WR);
    uint32_t* plain_rank = keep_plain ? arena.array<uint32_t>((size_t)batch * dv.WR) : nullptr;
    if (keep_plain) c->d_plain_id = keep(slab_alloc<uint32_t>((size_t)N * dv.W));
    uint32_t* d_plain_count = arena.array<uint32_t>((size_t)N);
    HIP_OK(hipMemsetAsync(d_plain_count, 0, (size_t)N * 4, stream));
    // walks over the on-chip limits are recorded in a log of this build's own (the one that the fills from
    // host-side states share is made here too, so that no fill has to allocate it)
    OverflowLog* log = arena.array<OverflowLog>(1);
    HIP_OK(hipMemsetAsync(log, 0, 8, stream));
    {
      std::lock_guard<std::mutex> lock(ctx().mu);
      (void)overflow_log();
    }
    const uint32_t seq = 1;
    uint32_t count_before = 0;
    hipEvent_t ev0, ev1;
    HIP_OK(hipEventCreateWithFlags(&ev0, hipEventDefault));
    HIP_OK(hipEventCreateWithFlags(&ev1, hipEventDefault));
    Engine engine(&A);
    std::vector<int32_t> host_plain;  // nodes of host-decided pairs that are context-dependent by section 3.1 alone
    uint32_t* d_seg_counts = arena.array<uint32_t>((size_t)N * n_seg);
    unsigned long long* d_digest = arena.array<unsigned long long>((size_t)N);
    uint32_t* d_unc_counts = arena.array<uint32_t>((size_t)N);
    // rank -> id space, with the rows' statistics (accepted tokens per segment, digest, context-dependent tokens)
    auto permute = [&](int32_t node0, int32_t nb) {
      launch_permute(dv, nb, acc_rank, unc_rank, acc_id + (size_t)node0 * dv.W, unc_id + (size_t)node0 * dv.W,
                     d_seg_counts + (size_t)node0 * n_seg, d_digest + node0, d_unc_counts + node0, stream);
      if (keep_plain)
        launch_permute(dv, nb, plain_rank, plain_rank, c->d_plain_id + (size_t)node0 * dv.W,
                       c->d_plain_id + (size_t)node0 * dv.W, nullptr, nullptr, nullptr, stream);
    };
    // Pairs whose walk hit a limit are decided on the host and patched into the rank-space rows of the
    // current batch of nodes.  Returns whether there were any.
    auto decide_recorded_pairs = [&](int32_t node0) {
      const uint32_t count_after = read_overflow_count(log);
      const uint32_t fresh = count_after - count_before;
      if (fresh == 0) return false;
      if (fresh > OverflowLog::kCap) throw Failure(XGM_ERR_TOO_LARGE, "cache_build: too many walks exceeded the on-chip limits");
      std::vector<uint32_t> ent((size_t)OverflowLog::kCap * 4);
      HIP_OK(hipMemcpy(ent.data(), log->entry, ent.size() * 4, hipMemcpyDeviceToHost));
      std::vector<uint32_t> items;
      for (uint32_t k = 0; k < fresh; ++k) {
        const uint32_t* e = &ent[(size_t)((count_before + k) % OverflowLog::kCap) * 4];
        const int32_t id = v->id_of_rank[e[2]];
        int cls = engine.classify(node0 + (int32_t)e[1], v->bytes.data() + v->off[id], (int)(v->off[id + 1] - v->off[id]));
        if (cls < 0) throw Failure(XGM_ERR_TOO_LARGE, "cache_build: a token walk exceeds the host limits too");
        items.push_back(e[1]); items.push_back(e[2]); items.push_back((uint32_t)cls);
        if (cls == kUncertainPlain) host_plain.push_back(node0 + (int32_t)e[1]);
        ++c->host_classified;
      }
      uint32_t* d_items = arena.upload(items, stream);
      launch_patch_classes(dv, d_items, (int32_t)(items.size() / 3), acc_rank, unc_rank, plain_rank, stream);
      count_before = count_after;
      return true;
    };
    // Classify, batch after batch of nodes.  A grammar that fits one batch (the rule) runs classify,
    // the rank -> id permutation and the row statistics back to back and looks at the record of walks
    // over the limits only afterwards; if there are any, the patched rows are permuted again.
    const bool one_batch = batch >= N;
    uint4* d_first_byte = arena.array<uint4>((size_t)256 * first_byte_words(N));
    launch_first_byte(tab, d_first_byte, stream);
    for (int32_t node0 = 0; node0 < N; node0 += batch) {
      const int32_t nb = std::min(batch, N - node0);
      HIP_OK(hipEventRecord(ev0, stream));
      launch_classify(tab, dv, node0, nb, d_first_byte, acc_rank, unc_rank, plain_rank, d_plain_count, log, seq, stream);
      HIP_OK(hipEventRecord(ev1, stream));
      HIP_OK(hipGetLastError());
      if (!one_batch) {
        HIP_OK(hipStreamSynchronize(stream));
        float ms = 0.f;
        HIP_OK(hipEventElapsedTime(&ms, ev0, ev1));
        c->kernel_seconds += ms * 1e-3;
        decide_recorded_pairs(node0);
      }
      permute(node0, nb);
    }
    HIP_OK(hipGetLastError());
    HIP_OK(hipStreamSynchronize(stream));
    if (one_batch) {
      float ms = 0.f;
      HIP_OK(hipEventElapsedTime(&ms, ev0, ev1));
      c->kernel_seconds += ms * 1e-3;
      if (decide_recorded_pairs(0)) {
        permute(0, N);
        HIP_OK(hipGetLastError());
        HIP_OK(hipStreamSynchronize(stream));
      }
    }
    (void)hipEventDestroy(ev0);
    (void)hipEventDestroy(ev1);
    {
      std::lock_guard<std::mutex> lock(ctx().mu);
      ctx().retired_records += count_before;
    }

    // ---- per node: accepted tokens per segment, digest of the accepted row, context-dependent tokens
    std::vector<uint32_t> seg_counts((size_t)N * n_seg);
    std::vector<unsigned long long> digest((size_t)N);
    c->unc_count.resize(N);
    c->plain_count.resize(N);
    HIP_OK(hipMemcpy(seg_counts.data(), d_seg_counts, seg_counts.size() * 4, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(digest.data(), d_digest, digest.size() * 8, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(c->unc_count.data(), d_unc_counts, (size_t)N * 4, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(c->plain_count.data(), d_plain_count, (size_t)N * 4, hipMemcpyDeviceToHost));
    for (int32_t n : host_plain) ++c->plain_count[n];
    c->classify_seconds = std::chrono::duration<double>(std::chrono::steady_clock::now() - t_build0).count();

    // ---- accepted tokens: a node with few of them keeps a list (its level-0 key), the others a bitset row;
    // every distinct row is kept once (rows with equal digests are compared with the first of them)
    std::vector<char> as_list((size_t)N, 0);
    for (int32_t n = 0; n < N; ++n) {
      uint64_t total = 0;
      for (int32_t sgm = 0; sgm < n_seg; ++sgm) total += seg_counts[(size_t)n * n_seg + sgm];
      as_list[n] = total * 2 <= (uint64_t)dv.W;
    }
    std::vector<int32_t> rep((size_t)N);
    {
      std::unordered_map<unsigned long long, int32_t> first_with;
      for (int32_t n = 0; n < N; ++n) rep[n] = as_list[n] ? n : first_with.emplace(digest[n], n).first->second;
    }
    int32_t* d_rep = arena.upload(rep, stream);
    uint32_t* d_equal = arena.array<uint32_t>((size_t)N);
    launch_rows_equal(acc_id, N, dv.W, d_rep, d_equal, stream);

    // ---- keys: level 1 = (node with context-dependent tokens, context of its rule), level 2 = (level-1
    // key, context of that context node's rule)
    std::vector<uint32_t> ctx_off(A.rule_names.size() + 1, 0);
    std::vector<uint16_t> ctx_node;
    for (size_t r = 0; r < A.rule_names.size(); ++r) {
      for (int32_t n : A.contexts[r]) ctx_node.push_back((uint16_t)n);
      ctx_off[r + 1] = (uint32_t)ctx_node.size();
    }
    if (ctx_node.empty()) ctx_node.push_back(0);
    auto n_ctx = [&](int32_t rule) { return (uint64_t)(ctx_off[rule + 1] - ctx_off[rule]); };
    // Level l + 1 has a key for every (key of level l, context of the rule of that key's context node).  A level is
    // kept unless its keys alone would take hundreds of megabytes (grammars whose rules are each used in
    // hundreds of places); tokens that would need it are then walked at run time.
    std::vector<uint32_t> node_off((size_t)N + 1, 0);
    uint64_t n_base = 0, n_items = 0;
    std::vector<uint16_t> key_node;  // the context node of every key of the current level
    c->k_base_host[0].assign((size_t)N, kNoKey);
    for (int32_t n = 0; n < N; ++n) {
      node_off[n] = (uint32_t)n_base;
      const uint64_t m = n_ctx(A.node_rule[n]);
      if (c->unc_count[n] > 0 && m > 0) {
        c->k_base_host[0][n] = (uint32_t)key_node.size();
        for (int32_t r1 : A.contexts[A.node_rule[n]]) key_node.push_back((uint16_t)r1);
        n_items += (uint64_t)c->unc_count[n] * m;
      }
      n_base += c->unc_count[n];
      if (n_base >= ((uint64_t)1 << 32) || key_node.size() >= ((size_t)1 << 28))
        throw Failure(XGM_ERR_TOO_LARGE, "cache_build: context-dependent lists beyond the supported size");
    }
    node_off[N] = (uint32_t)n_base;
    uint64_t n_k[kCtxLevels] = {};
    n_k[0] = key_node.size();
    c->levels = 1;
    int max_levels = (int)((flags & XGM_CACHE_DEPTH_MASK) >> XGM_CACHE_DEPTH_SHIFT);
    if (max_levels == 0 || max_levels > kCtxLevels) max_levels = kCtxLevels;
    for (int l = 1; l < max_levels; ++l) {
      uint64_t next = 0;
      for (uint16_t r : key_node) next += n_ctx(A.node_rule[r]);
      if (next * (uint64_t)n_seg > ((uint64_t)1 << 26)) break;
      std::vector<uint16_t> next_node;
      next_node.reserve((size_t)next);
      c->k_base_host[l].resize(key_node.size());
      for (size_t q = 0; q < key_node.size(); ++q) {
        c->k_base_host[l][q] = (uint32_t)next_node.size();
        for (int32_t r2 : A.contexts[A.node_rule[key_node[q]]]) next_node.push_back((uint16_t)r2);
      }
      key_node.swap(next_node);
      n_k[l] = key_node.size();
      c->levels = l + 1;
    }
    uint64_t n_keys = (uint64_t)N;
    for (int l = 0; l < c->levels; ++l) n_keys += n_k[l];
    const size_t n_slots = (size_t)(n_keys * (uint64_t)n_seg);

    // ---- base lists (every node's context-dependent tokens), then the entries of every (key, segment): counted
    const uint32_t* d_k_base[kCtxLevels] = {};
    for (int l = 0; l < c->levels; ++l) d_k_base[l] = keep(slab_upload(c->k_base_host[l]));
    uint32_t* d_ctx_off = keep(slab_upload(ctx_off));
    uint16_t* d_ctx_node = keep(slab_upload(ctx_node));
    // the same relation by node (what the accept kernel looks up: which context of a rule a frame sits on)
    std::vector<uint32_t> node_ctx_off((size_t)N + 1, 0), node_ctx;
    {
      std::vector<std::vector<uint32_t>> by_node((size_t)N);
      for (size_t r = 0; r < A.rule_names.size(); ++r)
        for (size_t i = 0; i < A.contexts[r].size(); ++i) by_node[A.contexts[r][i]].push_back((uint32_t)(r << 16 | i));
      for (int32_t n = 0; n < N; ++n) {
        node_ctx_off[n] = (uint32_t)node_ctx.size();
        node_ctx.insert(node_ctx.end(), by_node[n].begin(), by_node[n].end());
      }
      node_ctx_off[N] = (uint32_t)node_ctx.size();
      if (node_ctx.empty()) node_ctx.push_back(0u);
    }
    c->host.node_ctx_off = keep(slab_upload(node_ctx_off));
    c->host.node_ctx = keep(slab_upload(node_ctx));
    uint32_t* d_base_ids = arena.array<uint32_t>((size_t)n_base);
    uint16_t* d_base_node = arena.array<uint16_t>((size_t)n_base);
    uint32_t* d_exits = arena.array<uint32_t>((size_t)n_base);
    {
      std::vector<uint32_t> identity((size_t)N);
      std::iota(identity.begin(), identity.end(), 0u);
      uint32_t* d_identity = arena.upload(identity, stream);
      uint32_t* d_cursor = arena.upload(node_off, stream);
      // In byte-sorted order where the rank-space rows of all nodes are still there (one batch): the walks of
      // neighbouring lanes then share prefixes, as in the classify kernel.
      if (one_batch) launch_rows_to_lists(unc_rank, dv.WR, dv.id_of_rank, N, d_identity, 1, d_cursor, d_base_ids, d_base_node, stream);
      else launch_rows_to_lists(unc_id, dv.W, nullptr, N, d_identity, 1, d_cursor, d_base_ids, d_base_node, stream);
    }
    uint32_t* d_counts = arena.array<uint32_t>(n_slots);
    HIP_OK(hipMemsetAsync(d_counts, 0, n_slots * 4, stream));
    // the level-1 kernel's tiles: the pairs of a node in blocks, its rule's contexts in blocks
    std::vector<uint4> tiles;
    {
      const uint32_t tp = context_tile_pairs(), tc = context_tile_contexts();
      for (int32_t n = 0; n < N; ++n) {
        if (c->k_base_host[0][n] == kNoKey) continue;
        const uint32_t L = c->unc_count[n], m = (uint32_t)n_ctx(A.node_rule[n]);
        for (uint32_t eb = 0; eb < L; eb += tp)
          for (uint32_t ib = 0; ib < m; ib += tc)
            tiles.push_back(make_uint4(node_off[n] + eb, std::min(tp, L - eb) | (std::min(tc, m - ib) << 16), ib, (uint32_t)n));
      }
    }
    ContextListArgs args{};
    args.base_node = d_base_node;
    args.base_ids = d_base_ids;
    args.total = (uint32_t)n_base;
    args.exits = d_exits;
    args.tiles = arena.upload(tiles, stream);
    args.n_tiles = (uint32_t)tiles.size();
    // (a pair leaves at most about one record per level on the grammars measured: 0.08 per pair for schema
    // grammars, 0.8 for a C-like one; the pass is run again with more room if this is not enough)
    args.res_cap = (uint32_t)std::min<uint64_t>(std::max<uint64_t>(n_base, 1u << 16), 1u << 25);
    for (int l = 0; l + 1 < c->levels; ++l) args.res[l] = arena.array<uint4>(args.res_cap);
    args.res_count = arena.array<uint32_t>(kCtxLevels);
    {
      uint32_t key0 = (uint32_t)N;
      for (int l = 0; l < kCtxLevels; ++l) {
        args.k_base[l] = l < c->levels ? d_k_base[l] : nullptr;
        args.key0[l] = key0;
        key0 += (uint32_t)n_k[l];
      }
    }
    args.ctx_off = d_ctx_off;
    args.ctx_node = d_ctx_node;
    args.counts = d_counts;
    // the counting pass of level 1 keeps what it found for every (pair, context), 2 bytes each, unless that
    // would take more than 1 GiB (then the writing pass walks again)
    if (n_items > 0 && n_items <= ((uint64_t)1 << 29)) {
      std::vector<uint4> node_info((size_t)N, make_uint4(0u, 0u, 0u, 0u));
      uint64_t at = 0;
      for (int32_t n = 0; n < N; ++n) {
        if (c->k_base_host[0][n] == kNoKey) continue;
        node_info[n] = make_uint4((uint32_t)at, c->unc_count[n], node_off[n], 0u);
        at += (uint64_t)c->unc_count[n] * n_ctx(A.node_rule[n]);
      }
      args.node_info = arena.upload(node_info, stream);
      args.outcomes = arena.array<uint16_t>((size_t)n_items);
      // (the deeper levels keep theirs per record: 16 bytes each)
      for (int l = 1; l < c->levels; ++l) args.deep_outcomes[l] = arena.array<uint4>(args.res_cap);
    }
    launch_exit_positions(tab, dv, args, stream);
    launch_context_lists(tab, dv, args, false, stream);
    HIP_OK(hipGetLastError());
    HIP_OK(hipStreamSynchronize(stream));
    for (;;) {  // records that did not fit were dropped: count again with room for all of them (rare)
      uint32_t made[kCtxLevels] = {};
      HIP_OK(hipMemcpy(made, args.res_count, sizeof(made), hipMemcpyDeviceToHost));
      const uint32_t most = *std::max_element(made, made + kCtxLevels);
      if (most <= args.res_cap) break;
      args.res_cap = most;
      for (int l = 0; l + 1 < c->levels; ++l) args.res[l] = arena.array<uint4>(args.res_cap);
      if (args.outcomes)
        for (int l = 1; l < c->levels; ++l) args.deep_outcomes[l] = arena.array<uint4>(args.res_cap);
      HIP_OK(hipMemsetAsync(d_counts, 0, n_slots * 4, stream));
      launch_context_lists(tab, dv, args, false, stream);
      HIP_OK(hipGetLastError());
      HIP_OK(hipStreamSynchronize(stream));
    }

    // ---- the distinct bitset rows
    uint32_t* acc_rows = nullptr;
    uint16_t* d_acc_row = nullptr;
    {
      std::vector<uint32_t> equal((size_t)N);
      HIP_OK(hipMemcpy(equal.data(), d_equal, equal.size() * 4, hipMemcpyDeviceToHost));
      std::vector<int32_t> unique;
      c->acc_row_host.assign((size_t)N, (uint16_t)kNoAccRow);
      std::vector<int32_t> row_of_rep((size_t)N, -1);
      for (int32_t n = 0; n < N; ++n) {
        if (as_list[n]) continue;
        if (!equal[n]) rep[n] = n;  // same digest, different row: kept by itself
        if (rep[n] == n) {
          row_of_rep[n] = (int32_t)unique.size();
          unique.push_back(n);
        }
        c->acc_row_host[n] = (uint16_t)row_of_rep[rep[n]];  // rep[n] <= n: its row is known
      }
      if (unique.size() >= kNoAccRow) throw Failure(XGM_ERR_TOO_LARGE, "cache_build: more than 65534 distinct accepted bitsets");
      c->n_acc_rows = (int32_t)unique.size();
      acc_rows = keep(slab_alloc<uint32_t>(unique.size() * (size_t)dv.W));
      int32_t* d_unique = arena.upload(unique, stream);
      launch_gather_rows(acc_id, dv.W, d_unique, c->n_acc_rows, acc_rows, stream);
      d_acc_row = keep(slab_upload(c->acc_row_host));
      c->device_bytes += (int64_t)unique.size() * dv.W * 4 + (int64_t)N * 2;
    }
    // ---- offsets from the counts, then the entries
    std::vector<uint32_t> counts(n_slots);
    HIP_OK(hipMemcpy(counts.data(), d_counts, n_slots * 4, hipMemcpyDeviceToHost));
    uint64_t n_level0 = 0;
    for (int32_t n = 0; n < N; ++n)
      if (as_list[n])
        for (int32_t sgm = 0; sgm < n_seg; ++sgm) n_level0 += counts[(size_t)n * n_seg + sgm] = seg_counts[(size_t)n * n_seg + sgm];
    c->key_off_host.assign(n_slots + 1, 0u);
    uint64_t total = 0;
    for (size_t k = 0; k < n_slots; ++k) {
      c->key_off_host[k] = (uint32_t)total;
      total += counts[k];
      if (total >= ((uint64_t)1 << 32)) throw Failure(XGM_ERR_TOO_LARGE, "cache_build: token lists exceed 2^32 entries");
    }
    c->key_off_host[n_slots] = (uint32_t)total;
    uint32_t* d_key_off = keep(slab_upload(c->key_off_host));
    uint32_t* d_entries = keep(slab_alloc<uint32_t>((size_t)total));
    {
      uint32_t* d_front = arena.array<uint32_t>(n_slots);
      uint32_t* d_back = arena.array<uint32_t>(n_slots);
      HIP_OK(hipMemcpyAsync(d_front, d_key_off, n_slots * 4, hipMemcpyDeviceToDevice, stream));
      HIP_OK(hipMemcpyAsync(d_back, d_key_off + 1, n_slots * 4, hipMemcpyDeviceToDevice, stream));
      std::vector<uint32_t> list_key((size_t)N);
      for (int32_t n = 0; n < N; ++n) list_key[n] = as_list[n] ? (uint32_t)n : kNoKey;
      uint32_t* d_list_key = arena.upload(list_key, stream);
      launch_rows_to_lists(acc_id, dv.W, nullptr, N, d_list_key, n_seg, d_front, d_entries, nullptr, stream);
      args.front = d_front;
      args.back = d_back;
      args.entries = d_entries;
      launch_context_lists(tab, dv, args, true, stream);
    }
    HIP_OK(hipGetLastError());
    cleanup_temps();  // (synchronises the stream)

    c->host.tab = staged_for(tab, kFillLdsBudget);
    c->host.acc = acc_rows;
    c->host.acc_row = d_acc_row;
    c->host.key_off = d_key_off;
    c->host.entries = d_entries;
    for (int l = 0; l < kCtxLevels; ++l) {
      c->host.k_base[l] = d_k_base[l];
      c->host.n_k[l] = (uint32_t)n_k[l];
    }
    c->host.ctx_off = d_ctx_off;
    c->host.ctx_node = d_ctx_node;
    c->host.n_nodes = N;
    c->device_bytes += (int64_t)(n_slots + 1) * 4 + (int64_t)total * 4 + (int64_t)image_bytes + (int64_t)(n_keys - n_k[c->levels - 1]) * 4 +
                       (int64_t)ctx_off.size() * 4 + (int64_t)ctx_node.size() * 2;
    if (keep_plain) c->device_bytes += (int64_t)N * dv.W * 8;
    c->stats[0] = (int64_t)n_keys;
    c->stats[1] = (int64_t)n_k[0];
    c->stats[2] = (int64_t)(n_keys - (uint64_t)N - n_k[0]);
    c->stats[3] = (int64_t)total;
    c->stats[4] = (int64_t)n_level0;
    c->stats[5] = (int64_t)n_base;
    c->stats[6] = (int64_t)n_items;
    c->stats[7] = (int64_t)c->n_acc_rows;
    c->build_seconds = std::chrono::duration<double>(std::chrono::steady_clock::now() - t_build0).count();
  } catch (...) {
    cleanup_temps();
    release(c);
    throw;
  }
  *out = c;
  return XGM_OK;
  API_END
}
void xgm_cache_destroy(xgm_cache* c) { release(c); }
int32_t xgm_cache_num_nodes(const xgm_cache* c) { return c ? c->host.n_nodes : XGM_ERR_BAD_ARG; }
int32_t xgm_cache_num_uncertain(const xgm_cache* c, int32_t node) {
  if (!c || node < 0 || node >= c->host.n_nodes) return fail(XGM_ERR_BAD_ARG, "num_uncertain: bad cache or node");
  return (int32_t)c->unc_count[node];
}
int32_t xgm_cache_num_uncertain_plain(const xgm_cache* c, int32_t node) {
  if (!c || node < 0 || node >= c->host.n_nodes) return fail(XGM_ERR_BAD_ARG, "num_uncertain_plain: bad cache or node");
  return (int32_t)c->plain_count[node];
}
int xgm_cache_copy_node_plain(const xgm_cache* c, int32_t node, int32_t* h_plain) {
  API_BEGIN
  if (!c || !h_plain || node < 0 || node >= c->host.n_nodes) return fail(XGM_ERR_BAD_ARG, "copy_node_plain: bad argument");
  if (!c->d_plain_id) return fail(XGM_ERR_BAD_ARG, "copy_node_plain: the cache was built without XGM_CACHE_KEEP_PLAIN");
  const int32_t W = c->v->dv.W;
  HIP_OK(hipMemcpy(h_plain, c->d_plain_id + (size_t)node * W, (size_t)W * 4, hipMemcpyDeviceToHost));
  return XGM_OK;
  API_END
}
int64_t xgm_cache_host_classified(const xgm_cache* c) { return c ? c->host_classified : XGM_ERR_BAD_ARG; }
double xgm_cache_build_kernel_seconds(const xgm_cache* c) { return c ? c->kernel_seconds : -1.0; }
double xgm_cache_build_seconds(const xgm_cache* c) { return c ? c->build_seconds : -1.0; }
double xgm_cache_build_classify_seconds(const xgm_cache* c) { return c ? c->classify_seconds : -1.0; }
int32_t xgm_cache_num_accept_rows(const xgm_cache* c) { return c ? c->n_acc_rows : XGM_ERR_BAD_ARG; }
int64_t xgm_cache_device_bytes(const xgm_cache* c) { return c ? c->device_bytes : XGM_ERR_BAD_ARG; }

int xgm_cache_stats(const xgm_cache* c, int64_t* h_out8) {
  if (!c || !h_out8) return fail(XGM_ERR_BAD_ARG, "cache_stats: null argument");
  for (int k = 0; k < 8; ++k) h_out8[k] = c->stats[k];
  return XGM_OK;
}

int xgm_cache_copy_node_bits(const xgm_cache* c, int32_t node, int32_t* h_acc, int32_t* h_unc) {
  API_BEGIN
  if (!c || node < 0 || node >= c->host.n_nodes) return fail(XGM_ERR_BAD_ARG, "copy_node_bits: bad cache or node");
  const DevVocab& dv = c->v->dv;
  if (h_acc) {
    if (c->acc_row_host[node] != kNoAccRow) {
      HIP_OK(hipMemcpy(h_acc, c->host.acc + (size_t)c->acc_row_host[node] * dv.W, (size_t)dv.W * 4, hipMemcpyDeviceToHost));
    } else {  // the node keeps its accepted tokens as a list (its level-0 key)
      std::memset(h_acc, 0, (size_t)dv.W * 4);
      const uint32_t j0 = c->key_off_host[(size_t)node * dv.n_seg], j1 = c->key_off_host[(size_t)(node + 1) * dv.n_seg];
      std::vector<uint32_t> list(j1 - j0);
      if (j1 > j0) HIP_OK(hipMemcpy(list.data(), c->host.entries + j0, (size_t)(j1 - j0) * 4, hipMemcpyDeviceToHost));
      for (uint32_t e : list) {
        const uint32_t id = e & kEntryIdMask;
        reinterpret_cast<uint32_t*>(h_acc)[id >> 5] |= 1u << (id & 31);
      }
    }
  }
  if (h_unc) {
    if (!c->d_unc_id) return fail(XGM_ERR_BAD_ARG, "copy_node_bits: the context-dependent bitsets are kept only with XGM_CACHE_KEEP_PLAIN");
    HIP_OK(hipMemcpy(h_unc, c->d_unc_id + (size_t)node * dv.W, (size_t)dv.W * 4, hipMemcpyDeviceToHost));
  }
  return XGM_OK;
  API_END
}

// ------------------------------------------------------------------- matcher
static int matcher_new(xgm_cache* c, xgm_grammar* g, xgm_vocab* v, xgm_matcher** out) {
  auto m = new xgm_matcher();
  m->c = c; if (c) ++c->refs;
  m->g = g; ++g->refs;
  m->v = v; if (v) ++v->refs;
  m->stacks = {Stack{g->A.rule_start[g->A.root_rule]}};
  *out = m;
  return XGM_OK;
}
int xgm_matcher_create(xgm_cache* c, xgm_matcher** out) {
  API_BEGIN
  if (!c || !out) return fail(XGM_ERR_BAD_ARG, "matcher_create: null argument");
  return matcher_new(c, c->g, c->v, out);
  API_END
}
int xgm_matcher_create_host(xgm_grammar* g, xgm_vocab* v, xgm_matcher** out) {
  API_BEGIN
  if (!g || !out) return fail(XGM_ERR_BAD_ARG, "matcher_create_host: null argument");
  return matcher_new(nullptr, g, v, out);
  API_END
}
void xgm_matcher_destroy(xgm_matcher* m) {
  if (!m) return;
  release(m->c);
  release(m->g);
  release(m->v);
  delete m;
}
int xgm_matcher_reset(xgm_matcher* m) {
  if (!m) return fail(XGM_ERR_BAD_ARG, "matcher_reset: null matcher");
  m->stacks = {Stack{m->g->A.rule_start[m->g->A.root_rule]}};
  m->terminated = false;
  return XGM_OK;
}
int xgm_matcher_accept_bytes(xgm_matcher* m, const uint8_t* h_bytes, int32_t n) {
  API_BEGIN
  if (!m || n < 0 || (n > 0 && !h_bytes)) return fail(XGM_ERR_BAD_ARG, "accept_bytes: bad argument");
  if (m->terminated) return fail(XGM_ERR_TERMINATED, "accept: the matcher has terminated");
  if (n == 0) return XGM_OK;
  Engine e(&m->g->A);
  std::vector<Stack> next;
  int rc = e.advance(m->stacks, h_bytes, n, &next, nullptr, XGM_MAX_STACKS);
  if (rc == XGM_ERR_TOKEN_REJECTED) return fail(rc, "accept: the bytes are not allowed here");
  if (rc == XGM_ERR_TOO_MANY_STACKS) return fail(rc, "accept: more than 64 parallel stacks");
  if (rc != XGM_OK) return fail(rc, "accept: stack depth or configuration limit exceeded");
  m->stacks.swap(next);
  return XGM_OK;
  API_END
}
int xgm_matcher_accept_token(xgm_matcher* m, int32_t token_id) {
  API_BEGIN
  if (!m || !m->v) return fail(XGM_ERR_BAD_ARG, "accept_token: matcher has no vocabulary");
  if (token_id < 0 || token_id >= m->v->V) return fail(XGM_ERR_BAD_ARG, "accept_token: token id out of range");
  if (m->terminated) return fail(XGM_ERR_TERMINATED, "accept: the matcher has terminated");
  const xgm_vocab& v = *m->v;
  if (v.is_stop[token_id]) {
    if (!Engine(&m->g->A).can_terminate(m->stacks)) return fail(XGM_ERR_TOKEN_REJECTED, "accept: stop token before the text is complete");
    m->terminated = true;
    return XGM_OK;
  }
  const int32_t n = (int32_t)(v.off[token_id + 1] - v.off[token_id]);
  if (n == 0) return fail(XGM_ERR_TOKEN_REJECTED, "accept: a token without bytes is never allowed");
  return xgm_matcher_accept_bytes(m, v.bytes.data() + v.off[token_id], n);
  API_END
}
int32_t xgm_matcher_is_terminated(const xgm_matcher* m) { return m ? (m->terminated ? 1 : 0) : XGM_ERR_BAD_ARG; }
int32_t xgm_matcher_can_terminate(const xgm_matcher* m) {
  if (!m) return XGM_ERR_BAD_ARG;
  return (!m->terminated && Engine(&m->g->A).can_terminate(m->stacks)) ? 1 : 0;
}
int32_t xgm_matcher_num_stacks(const xgm_matcher* m) { return m ? (m->terminated ? 0 : (int32_t)m->stacks.size()) : XGM_ERR_BAD_ARG; }
int32_t xgm_matcher_stack(const xgm_matcher* m, int32_t s, int32_t* h_nodes, int32_t cap) {
  if (!m || s < 0 || s >= (int32_t)m->stacks.size() || cap < 0 || (cap > 0 && !h_nodes)) return fail(XGM_ERR_BAD_ARG, "matcher_stack: bad argument");
  const Stack& st = m->stacks[s];
  for (int32_t k = 0; k < std::min<int32_t>(cap, (int32_t)st.size()); ++k) h_nodes[k] = st[k];
  return (int32_t)st.size();
}

// ---------------------------------------------------------------------- fill
// `timing` (may be null): three events recorded on the stream before the upload
// kernel, between the two kernels and after the fill kernel.
// `fused` (may be null): logits to mask in the same launch.
struct FusedLogits {
  void* d_logits;
  int esize;
  uint32_t neg_inf;
  int32_t V_logits;
  int64_t row_stride;
};
// The scalar words of a stack's header and the keys of its lists (see kStackHdr* and kStackKeysWords in
// kernels.hpp): h[0 .. kStackHdrWords) and key[0 .. kStackLists).  `frame_offset`: where the stack's frames
// start in the frame array.
static void stack_keys(const Automaton& A, const xgm_cache& c, const Stack& s, uint32_t frame_offset, uint32_t* h, uint32_t* key) {
  const int32_t top = s.back();
  h[kStackHdrTop] = (uint32_t)top | ((uint32_t)c.acc_row_host[top] << 16);
  h[kStackHdrDepth] = (uint32_t)s.size();
  h[kStackHdrFrames] = frame_offset;
  h[3] = 0u;
  // the keys of the stack's lists: the top node's own; then one per frame below the top that a kept level reaches
  auto context_index = [&](int32_t frame_node, int32_t below) {
    const auto& ctx = A.contexts[A.node_rule[frame_node]];
    auto it = std::lower_bound(ctx.begin(), ctx.end(), below);
    if (it == ctx.end() || *it != below) throw Failure(XGM_ERR_INTERNAL, "fill: a frame sits on a node that is no context of its rule");
    return (uint32_t)(it - ctx.begin());
  };
  key[0] = (uint32_t)top;
  uint32_t local = (uint32_t)top, key0 = (uint32_t)c.host.n_nodes;
  bool more = true;
  for (int l = 1; l <= kCtxLevels; ++l) {
    key[l] = kNoKey;
    if (more && l <= c.levels && (int)s.size() >= l + 1 && c.k_base_host[l - 1][local] != kNoKey) {
      local = c.k_base_host[l - 1][local] + context_index(s[s.size() - l], s[s.size() - l - 1]);
      key[l] = key0 + local;
    }
    more = key[l] != kNoKey;
    key0 += c.host.n_k[l - 1];
  }
}
// One stack header as the fill kernel reads it, written out on the host (device-resident batches are set up
// this way; the fills from host-side states send the keys and let the device look the offsets up).
static void pack_stack_header(const Automaton& A, const xgm_cache& c, const Stack& s, uint32_t frame_offset, uint32_t* h) {
  const int32_t n_seg = c.v->dv.n_seg;
  uint32_t key[kStackLists];
  stack_keys(A, c, s, frame_offset, h, key);
  for (uint32_t l = 0; l < kStackLists; ++l) {
    const uint32_t* ko = key[l] == kNoKey ? nullptr : &c.key_off_host[(size_t)key[l] * n_seg];
    for (int32_t sgm = 0; sgm <= n_seg; ++sgm) h[stack_hdr_off((uint32_t)sgm, l)] = ko ? ko[sgm] : 0u;
  }
}

// Host staging of the entry point that allocates nothing: the blob is packed here and copied to the device's
// static scratch array with a stream-ordered copy (which has taken the bytes when it returns, the memory
// being pageable).  Guarded by the context's mutex.
alignas(64) static unsigned char g_static_host[kStaticScratchBytes];

// `use_static`: stage in g_static_host and the device's static scratch array instead of the ring of
// allocated slots; nothing is allocated on this path.
static int fill_impl(xgm_matcher* const* ms, int32_t B, int32_t* d_bitmask, void* hip_stream,
                     unsigned long long* d_step_counter, hipEvent_t* timing = nullptr,
                     const FusedLogits* fused = nullptr, bool use_static = false) {
  API_BEGIN
  if (!ms || B <= 0 || !d_bitmask) return fail(XGM_ERR_BAD_ARG, "fill: null argument or empty batch");
  if (B > 65535) return fail(XGM_ERR_TOO_LARGE, "fill: more than 65535 rows in one call");
  xgm_vocab* v = nullptr;
  size_t n_stacks = 0, n_frames = 0;
  for (int32_t b = 0; b < B; ++b) {
    const xgm_matcher* m = ms[b];
    if (!m || !m->c) return fail(XGM_ERR_BAD_ARG, "fill: matcher is null or has no cache");
    if (v && m->v != v) return fail(XGM_ERR_BAD_ARG, "fill: all matchers must share one vocabulary");
    v = m->v;
    if (m->terminated) continue;
    n_stacks += m->stacks.size();
    for (auto& s : m->stacks) {
      if (s.size() > XGM_MAX_STACK_DEPTH) return fail(XGM_ERR_TOO_LARGE, "fill: stack deeper than 4096 frames");
      n_frames += s.size();
    }
  }
  require_device();
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  // On the host: row descriptors | per stack its scalar words and list keys | frames.  On the device: row
  // descriptors | full stack headers | frames (the static staging keeps the host's bytes behind that).
  static_assert(sizeof(RowDesc) % 16 == 0, "the sections of the staging memory are 16-byte aligned");
  const size_t hdr_words = stack_hdr_stride(v->dv.n_seg);
  const size_t off_stacks = (size_t)B * sizeof(RowDesc);
  const size_t h_off_frames = off_stacks + n_stacks * kStackKeysWords * 4;
  const size_t h_bytes = ((h_off_frames + n_frames * 2 + 63) / 64) * 64;
  const size_t off_frames = off_stacks + n_stacks * hdr_words * 4;
  const size_t d_bytes = ((off_frames + n_frames * 2 + 63) / 64) * 64;
  const size_t bytes = use_static ? d_bytes + h_bytes : std::max(d_bytes, h_bytes);

  Context& C = ctx();
  std::lock_guard<std::mutex> lock(C.mu);
  // (the fills' record of walks over the limits is allocated when a mask cache is built: this path allocates nothing)
  if (use_static && !C.d_log) return fail(XGM_ERR_INTERNAL, "fill (static staging): the library's device context does not exist yet");
  OverflowLog* log = overflow_log();
  void* h_buf = nullptr;
  void* d_buf = nullptr;
  FillSlot* ring = nullptr;
  if (use_static) {
    if (bytes > kStaticScratchBytes)
      return fail(XGM_ERR_TOO_LARGE, "fill (static staging): the batch's stacks need " + std::to_string(bytes) +
                                         " bytes of staging, the static array holds " + std::to_string(kStaticScratchBytes));
    HIP_OK(static_scratch(&d_buf));
    h_buf = g_static_host;
  } else {
    FillSlot& slot = C.slot[C.next_slot];
    ring = &slot;
    if (slot.used) HIP_OK(hipEventSynchronize(slot.done));
    if (slot.cap < bytes) {
      if (slot.h_buf) (void)hipHostFree(slot.h_buf);
      if (slot.d_buf) (void)hipFree(slot.d_buf);
      slot.h_buf = slot.d_buf = nullptr;
      slot.cap = std::max<size_t>(bytes * 2, 1 << 16);
      HIP_OK(hipHostMalloc(&slot.h_buf, slot.cap, hipHostMallocMapped));
      HIP_OK(hipHostGetDevicePointer(&slot.h_dev, slot.h_buf, 0));
      HIP_OK(hipMalloc(&slot.d_buf, slot.cap));
    }
    if (!slot.done) HIP_OK(hipEventCreateWithFlags(&slot.done, hipEventDisableTiming));
    h_buf = slot.h_buf;
    d_buf = slot.d_buf;
  }
  auto* rows = reinterpret_cast<RowDesc*>(h_buf);
  auto* hdrs = reinterpret_cast<uint32_t*>((char*)h_buf + off_stacks);
  auto* frames = reinterpret_cast<uint16_t*>((char*)h_buf + h_off_frames);
  uint32_t si = 0, fi = 0;
  for (int32_t b = 0; b < B; ++b) {
    const xgm_matcher* m = ms[b];
    RowDesc& r = rows[b];
    r.epoch = 0;
    r.stack_begin = si;
    r.frame_begin = fi;
    r.n_frames = 0;
    if (m->terminated) {
      r.tab = DevTables{};
      r.acc = r.entries = nullptr;
      r.n_stacks = 0;
      r.flags = 1;
      continue;
    }
    const Automaton& A = m->g->A;
    r.tab = m->c->host.tab;
    r.acc = m->c->host.acc;
    r.entries = m->c->host.entries;
    r.n_stacks = (uint32_t)m->stacks.size();
    r.flags = Engine(&A).can_terminate(m->stacks) ? 1u : 0u;
    for (auto& s : m->stacks) {
      uint32_t* h = hdrs + (size_t)si * kStackKeysWords;
      stack_keys(A, *m->c, s, fi, h, h + kStackHdrWords);
      const uintptr_t key_off = reinterpret_cast<uintptr_t>(m->c->host.key_off);
      h[kStackHdrWords + kStackLists] = (uint32_t)key_off;
      h[kStackHdrWords + kStackLists + 1] = (uint32_t)((uint64_t)key_off >> 32);
      for (uint32_t w = kStackHdrWords + kStackLists + 2; w < kStackKeysWords; ++w) h[w] = 0u;
      ++si;
      for (int32_t n : s) frames[fi++] = (uint16_t)n;
      r.n_frames += (uint32_t)s.size();
    }
  }
  if (timing) HIP_OK(hipEventRecord(timing[0], stream));
  const void* src = ring ? ring->h_dev : (const void*)((char*)d_buf + d_bytes);
  if (use_static) HIP_OK(hipMemcpyAsync((char*)d_buf + d_bytes, h_buf, h_bytes, hipMemcpyHostToDevice, stream));
  launch_upload_stacks(src, d_buf, off_stacks, (const char*)src + off_stacks, (uint32_t)n_stacks, v->dv.n_seg,
                       (char*)d_buf + off_stacks, (const char*)src + h_off_frames, (char*)d_buf + off_frames, n_frames * 2, stream);
  if (timing) HIP_OK(hipEventRecord(timing[1], stream));
  const uint32_t seq = ++C.seq;
  launch_fill(reinterpret_cast<const RowDesc*>(d_buf), reinterpret_cast<const uint32_t*>((char*)d_buf + off_stacks),
              reinterpret_cast<const uint16_t*>((char*)d_buf + off_frames), B, v->dv, reinterpret_cast<uint32_t*>(d_bitmask),
              log, seq, d_step_counter, stream, fused ? fused->d_logits : nullptr, fused ? fused->esize : 0,
              fused ? fused->neg_inf : 0u, fused ? fused->V_logits : 0, fused ? fused->row_stride : 0);
  HIP_OK(hipGetLastError());
  if (timing) HIP_OK(hipEventRecord(timing[2], stream));
  if (ring) {
    HIP_OK(hipEventRecord(ring->done, stream));
    ring->used = true;
    C.next_slot = (C.next_slot + 1) % Context::kSlots;
  }
  set_pending(ring ? ring->fill : C.static_fill, seq, B, d_bitmask, h_buf, ms);
  return XGM_OK;
  API_END
}

int xgm_debug_matcher_fill_work(const xgm_matcher* m, int64_t* h_out4) {
  API_BEGIN
  if (!m || !m->c || !h_out4) return fail(XGM_ERR_BAD_ARG, "matcher_fill_work: null argument or a matcher without a cache");
  for (int k = 0; k < 4; ++k) h_out4[k] = 0;
  if (m->terminated) return XGM_OK;
  const int32_t n_seg = m->v->dv.n_seg;
  std::vector<uint32_t> h(stack_hdr_stride(n_seg));
  for (const Stack& s : m->stacks) {
    pack_stack_header(m->g->A, *m->c, s, 0u, h.data());
    if ((h[kStackHdrTop] >> 16) != kNoAccRow) ++h_out4[0];
    for (uint32_t l = 0; l < kStackLists; ++l) {
      h_out4[1 + std::min<uint32_t>(l, 2u)] += h[stack_hdr_off((uint32_t)n_seg, l)] - h[stack_hdr_off(0u, l)];
    }
  }
  return XGM_OK;
  API_END
}

int xgm_fill_next_token_bitmask(xgm_matcher* const* ms, int32_t B, int32_t* d_bitmask, void* hip_stream) {
  return fill_impl(ms, B, d_bitmask, hip_stream, nullptr);
}

int xgm_fill_next_token_bitmask_static(xgm_matcher* const* ms, int32_t B, int32_t* d_bitmask, void* hip_stream) {
  return fill_impl(ms, B, d_bitmask, hip_stream, nullptr, nullptr, nullptr, true);
}
static_assert(kStaticScratchBytes == XGM_STATIC_STAGING_BYTES, "the header states the size of the static staging array");

// checks the logits arguments of a fused call and fills in `f`
static int fused_logits(void* d_logits, xgm_dtype dt, int32_t V_logits, int64_t row_stride_elems, int32_t V, FusedLogits* f) {
  if (V_logits < V) return fail(XGM_ERR_BAD_ARG, "fill_and_apply: logits rows are narrower than the vocabulary");
  if (row_stride_elems < V_logits) return fail(XGM_ERR_BAD_ARG, "fill_and_apply: row stride smaller than the row");
  *f = FusedLogits{d_logits, 0, 0u, V_logits, row_stride_elems};
  switch (dt) {
    case XGM_F32: f->esize = 4; f->neg_inf = 0xFF800000u; break;
    case XGM_BF16: f->esize = 2; f->neg_inf = 0xFF80u; break;
    case XGM_F16: f->esize = 2; f->neg_inf = 0xFC00u; break;
    default: return fail(XGM_ERR_BAD_ARG, "fill_and_apply: unknown dtype");
  }
  if (reinterpret_cast<uintptr_t>(d_logits) % 16 != 0 || (row_stride_elems * f->esize) % 16 != 0)
    return fail(XGM_ERR_BAD_ARG, "fill_and_apply: logits rows must be 16-byte aligned (use the two separate calls)");
  return XGM_OK;
}

int xgm_fill_and_apply(xgm_matcher* const* ms, int32_t B, int32_t* d_bitmask, void* d_logits, xgm_dtype dt,
                       int32_t V_logits, int64_t row_stride_elems, void* hip_stream) {
  API_BEGIN
  if (!d_logits) return fail(XGM_ERR_BAD_ARG, "fill_and_apply: null logits");
  if (!ms || B <= 0 || !ms[0] || !ms[0]->v) return fail(XGM_ERR_BAD_ARG, "fill_and_apply: null argument or empty batch");
  FusedLogits f{};
  const int rc = fused_logits(d_logits, dt, V_logits, row_stride_elems, ms[0]->v->V, &f);
  if (rc != XGM_OK) return rc;
  return fill_impl(ms, B, d_bitmask, hip_stream, nullptr, nullptr, &f);
  API_END
}

int xgm_debug_fill_count_steps(xgm_matcher* const* ms, int32_t B, int32_t* d_bitmask, void* hip_stream,
                               int64_t* h_steps) {
  API_BEGIN
  if (!h_steps) return fail(XGM_ERR_BAD_ARG, "count_steps: null output");
  require_device();
  unsigned long long* d_counter = dev_alloc<unsigned long long>(1);
  int rc = XGM_OK;
  try {
    HIP_OK(hipMemset(d_counter, 0, sizeof(unsigned long long)));
    rc = fill_impl(ms, B, d_bitmask, hip_stream, d_counter);
    if (rc == XGM_OK) {
      HIP_OK(hipStreamSynchronize(static_cast<hipStream_t>(hip_stream)));
      unsigned long long n = 0;
      HIP_OK(hipMemcpy(&n, d_counter, sizeof(n), hipMemcpyDeviceToHost));
      *h_steps = (int64_t)n;
    }
  } catch (...) {
    (void)hipFree(d_counter);
    throw;
  }
  (void)hipFree(d_counter);
  return rc;
  API_END
}

int xgm_debug_fill_timed(xgm_matcher* const* ms, int32_t B, int32_t* d_bitmask, void* hip_stream, float* h_us2) {
  API_BEGIN
  if (!h_us2) return fail(XGM_ERR_BAD_ARG, "fill_timed: null output");
  require_device();
  hipEvent_t ev[3] = {nullptr, nullptr, nullptr};
  int rc = XGM_OK;
  try {
    for (auto& e : ev) HIP_OK(hipEventCreate(&e));
    rc = fill_impl(ms, B, d_bitmask, hip_stream, nullptr, ev);
    if (rc == XGM_OK) {
      HIP_OK(hipEventSynchronize(ev[2]));
      float ms01 = 0.f, ms12 = 0.f;
      HIP_OK(hipEventElapsedTime(&ms01, ev[0], ev[1]));
      HIP_OK(hipEventElapsedTime(&ms12, ev[1], ev[2]));
      h_us2[0] = ms01 * 1e3f;
      h_us2[1] = ms12 * 1e3f;
    }
  } catch (...) {
    for (auto& e : ev) if (e) (void)hipEventDestroy(e);
    throw;
  }
  for (auto& e : ev) if (e) (void)hipEventDestroy(e);
  return rc;
  API_END
}

// the state of one row of a batch, read back from the device (the stream must be idle)
static void read_row_state(const xgm_batch& bt, int32_t row, bool* terminated, std::vector<Stack>* stacks) {
  int32_t head = 0;
  HIP_OK(hipMemcpy(&head, bt.dev.head + row, 4, hipMemcpyDeviceToHost));
  SlotMeta m{};
  HIP_OK(hipMemcpy(&m, bt.dev.meta + (size_t)row * bt.H + head, sizeof(m), hipMemcpyDeviceToHost));
  *terminated = (m.flags & 2u) != 0;
  stacks->clear();
  if (m.n_stacks == 0) return;
  const size_t hdr_words = stack_hdr_stride(bt.dev.n_seg);
  const size_t slot = (size_t)row * bt.H + head;
  std::vector<uint32_t> hdrs((size_t)m.n_stacks * hdr_words);
  HIP_OK(hipMemcpy(hdrs.data(), bt.dev.hdrs + slot * kBatchMaxStacks * hdr_words, hdrs.size() * 4, hipMemcpyDeviceToHost));
  std::vector<uint16_t> frames(kBatchRowFrames);
  HIP_OK(hipMemcpy(frames.data(), bt.dev.frames + slot * kBatchRowFrames, frames.size() * 2, hipMemcpyDeviceToHost));
  for (uint32_t k = 0; k < m.n_stacks; ++k) {
    const uint32_t* h = &hdrs[k * hdr_words];
    const size_t f0 = h[kStackHdrFrames] - slot * kBatchRowFrames;
    if (h[kStackHdrDepth] == 0 || f0 + h[kStackHdrDepth] > kBatchRowFrames)
      throw Failure(XGM_ERR_INTERNAL, "batch: a device-resident stack header is out of range");
    stacks->emplace_back(frames.begin() + f0, frames.begin() + f0 + h[kStackHdrDepth]);
  }
}

extern "C++" {  // (helpers that return C++ types)
namespace {
// is the token allowed from some of these stacks?  (exact, on the host; throws if the host limits are exceeded too)
bool host_decides(const Automaton& A, const xgm_vocab& v, const std::vector<Stack>& stacks, int32_t id) {
  Engine engine(&A);
  for (const Stack& st : stacks) {
    std::vector<Stack> out;
    const int rc = engine.advance({st}, v.bytes.data() + v.off[id], (int)(v.off[id + 1] - v.off[id]), &out, nullptr, (size_t)-1);
    if (rc == XGM_OK) return true;
    if (rc != XGM_ERR_TOKEN_REJECTED) throw Failure(rc, "fixup: a token walk exceeds the host limits too");
  }
  return false;
}
// writes the exact bit either way (a fused fill leaves such a token allowed until now)
void patch_bit(int32_t* d_bitmask, int32_t W, int32_t row, int32_t id, bool allowed) {
  uint32_t word = 0;
  int32_t* p = d_bitmask + (size_t)row * W + (id >> 5);
  HIP_OK(hipMemcpy(&word, p, 4, hipMemcpyDeviceToHost));
  if (allowed) word |= 1u << (id & 31); else word &= ~(1u << (id & 31));
  HIP_OK(hipMemcpy(p, &word, 4, hipMemcpyHostToDevice));
}
// the records [seen, count) of a log (at most kCap of them are still there)
std::vector<std::array<uint32_t, 4>> fresh_records(const OverflowLog* log, uint32_t seen, uint32_t count) {
  std::vector<std::array<uint32_t, 4>> out;
  const uint32_t fresh = count - seen;
  if (fresh == 0) return out;
  if (fresh > OverflowLog::kCap) throw Failure(XGM_ERR_TOO_LARGE, "fixup: more recorded walks than the log holds");
  std::vector<uint32_t> ent((size_t)OverflowLog::kCap * 4);
  HIP_OK(hipMemcpy(ent.data(), log->entry, ent.size() * 4, hipMemcpyDeviceToHost));
  for (uint32_t k = 0; k < fresh; ++k) {
    const uint32_t* e = &ent[(size_t)((seen + k) % OverflowLog::kCap) * 4];
    out.push_back({e[0], e[1], e[2], e[3]});
  }
  return out;
}
}  // namespace
}  // extern "C++"

int xgm_fill_overflow_fixup(void* hip_stream) {
  API_BEGIN
  Context& C = ctx();
  std::lock_guard<std::mutex> lock(C.mu);
  if (!C.d_log) return 0;
  HIP_OK(hipStreamSynchronize(static_cast<hipStream_t>(hip_stream)));
  const uint32_t count = read_overflow_count(C.d_log);
  const auto records = fresh_records(C.d_log, C.seen_count, count);
  int handled = 0, lost = 0;
  for (const auto& e : records) {
    // the fill that recorded it: one of the last fills from the ring of staging slots, or the last one staged statically
    const PendingFill* f = C.static_fill.seq == e[0] && e[0] != 0 ? &C.static_fill : nullptr;
    for (const FillSlot& slot : C.slot)
      if (slot.fill.seq == e[0] && e[0] != 0) f = &slot.fill;
    const int32_t b = (int32_t)e[1], id = (int32_t)e[2];
    if (!f || b >= f->B) { ++lost; continue; }
    const xgm_cache& c = *f->caches[b];
    const xgm_vocab& v = *c.v;
    // the row's stacks as that fill packed them
    const auto* rows = reinterpret_cast<const RowDesc*>(f->blob);
    const size_t hdr_words = kStackKeysWords;  // (the staging memory holds the stacks as the host packed them)
    const auto* hdrs = reinterpret_cast<const uint32_t*>((const char*)f->blob + (size_t)f->B * sizeof(RowDesc));
    size_t n_stacks = 0;
    for (int32_t r = 0; r < f->B; ++r) n_stacks += rows[r].n_stacks;
    const auto* frames = reinterpret_cast<const uint16_t*>(hdrs + n_stacks * hdr_words);
    std::vector<Stack> stacks;
    for (uint32_t s = 0; s < rows[b].n_stacks; ++s) {
      const uint32_t* h = hdrs + (size_t)(rows[b].stack_begin + s) * hdr_words;
      stacks.emplace_back(frames + h[kStackHdrFrames], frames + h[kStackHdrFrames] + h[kStackHdrDepth]);
    }
    patch_bit(f->d_bitmask, v.dv.W, b, id, host_decides(c.g->A, v, stacks, id));
    ++handled;
  }
  C.seen_count = count;
  if (lost)
    return fail(XGM_ERR_TOO_LARGE, "fixup: " + std::to_string(lost) + " recorded walks belong to fills whose staging memory has been "
                                   "used again (more than 8 fills ago); " + std::to_string(handled) + " were decided");
  return handled;
  API_END
}

const uint32_t* xgm_fill_overflow_count_device(void) {
  try {
    std::lock_guard<std::mutex> lock(ctx().mu);
    return &overflow_log()->count;
  } catch (const Failure& f) { fail(f); return nullptr; }
}

// ------------------------------------------------- device-resident states
extern "C++" {  // (helpers that return C++ types)
namespace {
// what the matcher's current state looks like in slot `slot` of row `row`
struct PackedState {
  SlotMeta meta{};
  std::vector<uint32_t> hdrs;
  std::vector<uint16_t> frames;
  RowDesc row{};
};
PackedState pack_state(const xgm_batch& bt, int32_t row, int32_t slot, const xgm_matcher& m) {
  const xgm_cache& c = *bt.caches[row];
  const Automaton& A = c.g->A;
  const size_t hdr_words = stack_hdr_stride(bt.dev.n_seg);
  const size_t at = (size_t)row * bt.H + slot;
  PackedState p;
  p.row.tab = c.host.tab;
  p.row.acc = c.host.acc;
  p.row.entries = c.host.entries;
  p.row.stack_begin = (uint32_t)(at * kBatchMaxStacks);
  p.row.frame_begin = (uint32_t)(at * kBatchRowFrames);
  if (m.terminated) {
    p.meta.flags = 3u;
  } else {
    if (m.stacks.size() > kBatchMaxStacks) throw Failure(XGM_ERR_TOO_MANY_STACKS, "batch: more than 16 parallel stacks in a row");
    p.hdrs.assign(m.stacks.size() * hdr_words, 0u);
    uint32_t fi = 0;
    for (size_t k = 0; k < m.stacks.size(); ++k) {
      const Stack& s = m.stacks[k];
      if (s.size() > kBatchMaxDepth) throw Failure(XGM_ERR_TOO_LARGE, "batch: a stack deeper than 128 frames");
      pack_stack_header(A, c, s, p.row.frame_begin + fi, &p.hdrs[k * hdr_words]);
      for (int32_t n : s) p.frames.push_back((uint16_t)n);
      fi += (uint32_t)s.size();
    }
    p.meta.n_stacks = (uint32_t)m.stacks.size();
    p.meta.n_frames = fi;
    p.meta.flags = Engine(&A).can_terminate(m.stacks) ? 1u : 0u;
  }
  p.row.n_stacks = p.meta.n_stacks;
  p.row.n_frames = p.meta.n_frames;
  p.row.flags = p.meta.flags & 1u;
  return p;
}
// `epoch`: the row's count of state changes after this write
void write_state(const xgm_batch& bt, int32_t row, int32_t slot, PackedState p, uint32_t epoch) {
  const size_t hdr_words = stack_hdr_stride(bt.dev.n_seg);
  const size_t at = (size_t)row * bt.H + slot;
  p.row.epoch = epoch;
  HIP_OK(hipMemcpy(bt.dev.meta + at, &p.meta, sizeof(SlotMeta), hipMemcpyHostToDevice));
  if (!p.hdrs.empty()) HIP_OK(hipMemcpy(bt.dev.hdrs + at * kBatchMaxStacks * hdr_words, p.hdrs.data(), p.hdrs.size() * 4, hipMemcpyHostToDevice));
  if (!p.frames.empty()) HIP_OK(hipMemcpy(bt.dev.frames + at * kBatchRowFrames, p.frames.data(), p.frames.size() * 2, hipMemcpyHostToDevice));
  HIP_OK(hipMemcpy(bt.dev.rows + row, &p.row, sizeof(RowDesc), hipMemcpyHostToDevice));
}
}  // namespace
}  // extern "C++"

int xgm_batch_create(xgm_matcher* const* ms, int32_t B, int32_t history, void* hip_stream, xgm_batch** out) {
  API_BEGIN
  if (!ms || !out || B <= 0) return fail(XGM_ERR_BAD_ARG, "batch_create: null argument or empty batch");
  if (history < 0 || history > XGM_BATCH_MAX_HISTORY) return fail(XGM_ERR_BAD_ARG, "batch_create: history out of range");
  if (B > (int32_t)kBatchMaxRows) return fail(XGM_ERR_TOO_LARGE, "batch_create: more than 1024 rows");
  xgm_vocab* v = nullptr;
  for (int32_t b = 0; b < B; ++b) {
    if (!ms[b] || !ms[b]->c) return fail(XGM_ERR_BAD_ARG, "batch_create: matcher is null or has no cache");
    if (v && ms[b]->v != v) return fail(XGM_ERR_BAD_ARG, "batch_create: all matchers must share one vocabulary");
    v = ms[b]->v;
  }
  require_device();
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  auto* bt = new xgm_batch();
  try {
    bt->B = B;
    bt->H = history + 1;
    bt->v = v;
    ++v->refs;
    for (int32_t b = 0; b < B; ++b) { bt->caches.push_back(ms[b]->c); ++ms[b]->c->refs; }
    auto keep = [&](auto* p) { bt->dev_ptrs.push_back((void*)p); return p; };
    const size_t hdr_words = stack_hdr_stride(v->dv.n_seg);
    const size_t slots = (size_t)B * bt->H;
    DevBatch& d = bt->dev;
    d.B = B;
    d.H = bt->H;
    d.n_seg = v->dv.n_seg;
    std::vector<DevCache> caches(B);
    for (int32_t b = 0; b < B; ++b) caches[b] = ms[b]->c->host;
    d.cache = keep(dev_upload(caches));
    d.rows = keep(dev_alloc<RowDesc>(B));
    d.meta = keep(dev_alloc<SlotMeta>(slots));
    d.hdrs = keep(dev_alloc<uint32_t>(slots * kBatchMaxStacks * hdr_words));
    d.frames = keep(dev_alloc<uint16_t>(slots * kBatchRowFrames));
    d.head = keep(dev_alloc<int32_t>(B));
    d.older = keep(dev_alloc<int32_t>(B));
    d.status = keep(dev_alloc<int32_t>(B));
    d.log = keep(new_log());
    HIP_OK(hipMemset(d.meta, 0, slots * sizeof(SlotMeta)));
    HIP_OK(hipMemset(d.head, 0, (size_t)B * 4));
    HIP_OK(hipMemset(d.older, 0, (size_t)B * 4));
    HIP_OK(hipMemset(d.status, 0, (size_t)B * 4));
    for (int32_t b = 0; b < B; ++b) write_state(*bt, b, 0, pack_state(*bt, b, 0, *ms[b]), 0u);
    HIP_OK(hipStreamSynchronize(stream));
    std::lock_guard<std::mutex> lock(ctx().mu);
    ctx().batches.insert(bt);
  } catch (...) {
    xgm_batch_destroy(bt);
    throw;
  }
  *out = bt;
  return XGM_OK;
  API_END
}

void xgm_batch_destroy(xgm_batch* bt) {
  if (!bt) return;
  {
    Context& C = ctx();
    std::lock_guard<std::mutex> lock(C.mu);
    if (C.batches.erase(bt) && bt->dev.log) {
      uint32_t n = 0;  // its records stay in the process-wide total
      if (hipDeviceSynchronize() == hipSuccess && hipMemcpy(&n, &bt->dev.log->count, 4, hipMemcpyDeviceToHost) == hipSuccess)
        C.retired_records += n;
    }
  }
  for (void* p : bt->dev_ptrs) (void)hipFree(p);
  for (xgm_cache* c : bt->caches) release(c);
  release(bt->v);
  delete bt;
}

int32_t xgm_batch_size(const xgm_batch* bt) { return bt ? bt->B : XGM_ERR_BAD_ARG; }

int xgm_batch_accept_tokens(xgm_batch* bt, const int32_t* d_token_ids, void* hip_stream) {
  API_BEGIN
  if (!bt || !d_token_ids) return fail(XGM_ERR_BAD_ARG, "batch_accept_tokens: null argument");
  launch_batch_accept(bt->dev, bt->v->dv, d_token_ids, static_cast<hipStream_t>(hip_stream));
  HIP_OK(hipGetLastError());
  return XGM_OK;
  API_END
}

int xgm_batch_rollback(xgm_batch* bt, const int32_t* d_steps, void* hip_stream) {
  API_BEGIN
  if (!bt || !d_steps) return fail(XGM_ERR_BAD_ARG, "batch_rollback: null argument");
  launch_batch_rollback(bt->dev, d_steps, static_cast<hipStream_t>(hip_stream));
  HIP_OK(hipGetLastError());
  return XGM_OK;
  API_END
}

int xgm_batch_fork(xgm_batch* bt, const int32_t* d_src_rows, void* hip_stream) {
  API_BEGIN
  if (!bt || !d_src_rows) return fail(XGM_ERR_BAD_ARG, "batch_fork: null argument");
  if (bt->H < 2) return fail(XGM_ERR_BAD_ARG, "batch_fork: the batch was created without history (a forked state is written beside the current one)");
  launch_batch_fork(bt->dev, d_src_rows, static_cast<hipStream_t>(hip_stream));
  HIP_OK(hipGetLastError());
  return XGM_OK;
  API_END
}

int xgm_batch_status(xgm_batch* bt, int32_t* h_status, void* hip_stream) {
  API_BEGIN
  if (!bt || !h_status) return fail(XGM_ERR_BAD_ARG, "batch_status: null argument");
  HIP_OK(hipStreamSynchronize(static_cast<hipStream_t>(hip_stream)));
  HIP_OK(hipMemcpy(h_status, bt->dev.status, (size_t)bt->B * 4, hipMemcpyDeviceToHost));
  int bad = 0;
  for (int32_t b = 0; b < bt->B; ++b) bad += h_status[b] != XGM_OK;
  return bad;
  API_END
}

int xgm_batch_get_row(xgm_batch* bt, int32_t row, xgm_matcher* m, void* hip_stream) {
  API_BEGIN
  if (!bt || !m || row < 0 || row >= bt->B) return fail(XGM_ERR_BAD_ARG, "batch_get_row: bad argument");
  if (m->c != bt->caches[row]) return fail(XGM_ERR_BAD_ARG, "batch_get_row: the matcher belongs to another mask cache");
  HIP_OK(hipStreamSynchronize(static_cast<hipStream_t>(hip_stream)));
  bool terminated = false;
  std::vector<Stack> stacks;
  read_row_state(*bt, row, &terminated, &stacks);
  m->terminated = terminated;
  if (!terminated) m->stacks.swap(stacks);
  return XGM_OK;
  API_END
}

int xgm_batch_set_row(xgm_batch* bt, int32_t row, const xgm_matcher* m, void* hip_stream) {
  API_BEGIN
  if (!bt || !m || row < 0 || row >= bt->B) return fail(XGM_ERR_BAD_ARG, "batch_set_row: bad argument");
  if (m->c != bt->caches[row]) return fail(XGM_ERR_BAD_ARG, "batch_set_row: the matcher belongs to another mask cache");
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  HIP_OK(hipStreamSynchronize(stream));
  int32_t head = 0, older = 0;
  RowDesc cur{};
  HIP_OK(hipMemcpy(&head, bt->dev.head + row, 4, hipMemcpyDeviceToHost));
  HIP_OK(hipMemcpy(&older, bt->dev.older + row, 4, hipMemcpyDeviceToHost));
  HIP_OK(hipMemcpy(&cur, bt->dev.rows + row, sizeof(RowDesc), hipMemcpyDeviceToHost));
  const int32_t next = (head + 1) % bt->H;
  write_state(*bt, row, next, pack_state(*bt, row, next, *m), cur.epoch + 1u);
  older = std::min(older + 1, bt->H - 1);
  const int32_t ok = XGM_OK;
  HIP_OK(hipMemcpy(bt->dev.head + row, &next, 4, hipMemcpyHostToDevice));
  HIP_OK(hipMemcpy(bt->dev.older + row, &older, 4, hipMemcpyHostToDevice));
  HIP_OK(hipMemcpy(bt->dev.status + row, &ok, 4, hipMemcpyHostToDevice));
  return XGM_OK;
  API_END
}

int xgm_debug_lds_lookup_rate(void* hip_stream, double* h_lookups_per_second) {
  API_BEGIN
  if (!h_lookups_per_second) return fail(XGM_ERR_BAD_ARG, "lds_lookup_rate: null output");
  require_device();
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  int dev = 0, cus = 0;
  HIP_OK(hipGetDevice(&dev));
  HIP_OK(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
  const int32_t n_blocks = 2 * std::max(1, cus);
  const uint32_t hops = 4096;
  uint32_t* sink = dev_alloc<uint32_t>(1);
  hipEvent_t e0 = nullptr, e1 = nullptr;
  try {
    HIP_OK(hipEventCreate(&e0));
    HIP_OK(hipEventCreate(&e1));
    launch_lds_lookups(n_blocks, hops, sink, stream);  // warm-up
    HIP_OK(hipEventRecord(e0, stream));
    launch_lds_lookups(n_blocks, hops, sink, stream);
    HIP_OK(hipEventRecord(e1, stream));
    HIP_OK(hipGetLastError());
    HIP_OK(hipEventSynchronize(e1));
    float ms = 0.f;
    HIP_OK(hipEventElapsedTime(&ms, e0, e1));
    *h_lookups_per_second = (double)n_blocks * 1024.0 * hops / (ms * 1e-3);
  } catch (...) {
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    (void)hipFree(sink);
    throw;
  }
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  (void)hipFree(sink);
  return XGM_OK;
  API_END
}

static int batch_fill_impl(xgm_batch* bt, int32_t* d_bitmask, void* hip_stream, const FusedLogits* fused) {
  if (!bt || !d_bitmask) return fail(XGM_ERR_BAD_ARG, "batch_fill: null argument");
  uint32_t seq;
  {
    Context& C = ctx();
    std::lock_guard<std::mutex> lock(C.mu);
    seq = ++C.seq;
  }
  const DevBatch& d = bt->dev;
  launch_fill(d.rows, d.hdrs, d.frames, d.B, bt->v->dv, reinterpret_cast<uint32_t*>(d_bitmask), d.log, seq, nullptr,
              static_cast<hipStream_t>(hip_stream), fused ? fused->d_logits : nullptr, fused ? fused->esize : 0,
              fused ? fused->neg_inf : 0u, fused ? fused->V_logits : 0, fused ? fused->row_stride : 0);
  HIP_OK(hipGetLastError());
  bt->fill_seq[bt->next_fill] = seq;
  bt->fill_bitmask[bt->next_fill] = d_bitmask;
  bt->next_fill = (bt->next_fill + 1) % xgm_batch::kFills;
  return XGM_OK;
}

int xgm_batch_fill_next_token_bitmask(xgm_batch* bt, int32_t* d_bitmask, void* hip_stream) {
  API_BEGIN
  return batch_fill_impl(bt, d_bitmask, hip_stream, nullptr);
  API_END
}

int xgm_batch_fill_and_apply(xgm_batch* bt, int32_t* d_bitmask, void* d_logits, xgm_dtype dt, int32_t V_logits,
                             int64_t row_stride_elems, void* hip_stream) {
  API_BEGIN
  if (!bt || !d_logits) return fail(XGM_ERR_BAD_ARG, "batch_fill_and_apply: null argument");
  FusedLogits f{};
  const int rc = fused_logits(d_logits, dt, V_logits, row_stride_elems, bt->v->V, &f);
  if (rc != XGM_OK) return rc;
  return batch_fill_impl(bt, d_bitmask, hip_stream, &f);
  API_END
}

int xgm_batch_fill_overflow_fixup(xgm_batch* bt, void* hip_stream) {
  API_BEGIN
  if (!bt) return fail(XGM_ERR_BAD_ARG, "batch_fill_overflow_fixup: null batch");
  HIP_OK(hipStreamSynchronize(static_cast<hipStream_t>(hip_stream)));
  const uint32_t count = read_overflow_count(bt->dev.log);
  const auto records = fresh_records(bt->dev.log, bt->seen_count, count);
  const xgm_vocab& v = *bt->v;
  int handled = 0, lost = 0, stale = 0;
  for (const auto& e : records) {
    int32_t* d_bitmask = nullptr;
    for (int k = 0; k < xgm_batch::kFills; ++k)
      if (bt->fill_seq[k] == e[0] && e[0] != 0) d_bitmask = bt->fill_bitmask[k];
    const int32_t b = (int32_t)e[1], id = (int32_t)e[2];
    if (!d_bitmask || b >= bt->B) { ++lost; continue; }
    RowDesc cur{};
    HIP_OK(hipMemcpy(&cur, bt->dev.rows + b, sizeof(RowDesc), hipMemcpyDeviceToHost));
    if (cur.epoch != e[3]) { ++stale; continue; }  // the row has moved on since that fill: its stacks are gone
    bool terminated = false;
    std::vector<Stack> stacks;
    read_row_state(*bt, b, &terminated, &stacks);
    patch_bit(d_bitmask, v.dv.W, b, id, host_decides(bt->caches[b]->g->A, v, stacks, id));
    ++handled;
  }
  bt->seen_count = count;
  if (lost || stale)
    return fail(XGM_ERR_TOO_LARGE, "batch fixup: " + std::to_string(stale) + " recorded walks belong to states that the rows have left, " +
                                   std::to_string(lost) + " to fills more than 8 fills ago; " + std::to_string(handled) + " were decided");
  return handled;
  API_END
}

const uint32_t* xgm_batch_overflow_count_device(const xgm_batch* bt) { return bt ? &bt->dev.log->count : nullptr; }

int64_t xgm_overflow_total(void) {
  try {
    Context& C = ctx();
    std::lock_guard<std::mutex> lock(C.mu);
    HIP_OK(hipDeviceSynchronize());
    int64_t total = C.retired_records;
    if (C.d_log) total += read_overflow_count(C.d_log);
    for (const xgm_batch* bt : C.batches) total += read_overflow_count(bt->dev.log);
    return total;
  } catch (const Failure& f) { return fail(f); }
}

// --------------------------------------------------------------------- apply
int xgm_apply_token_bitmask_inplace(void* d_logits, xgm_dtype dt, int32_t B, int32_t V_logits, int64_t row_stride_elems,
                                    const int32_t* d_bitmask, int32_t V_mask, const int32_t* d_row_index,
                                    int32_t n_rows, void* hip_stream) {
  API_BEGIN
  if (!d_logits || !d_bitmask) return fail(XGM_ERR_BAD_ARG, "apply: null logits or bitmask");
  if (B <= 0 || V_logits <= 0 || V_mask <= 0 || n_rows < 0) return fail(XGM_ERR_BAD_ARG, "apply: sizes must be positive");
  if (row_stride_elems < V_logits) return fail(XGM_ERR_BAD_ARG, "apply: row stride smaller than the row");
  if (!d_row_index && n_rows != B) return fail(XGM_ERR_BAD_ARG, "apply: without a row index n_rows must equal B");
  if (d_row_index && n_rows > B) return fail(XGM_ERR_BAD_ARG, "apply: more mask rows than logits rows");
  int esize;
  uint32_t ninf;
  switch (dt) {
    case XGM_F32: esize = 4; ninf = 0xFF800000u; break;
    case XGM_BF16: esize = 2; ninf = 0xFF80u; break;
    case XGM_F16: esize = 2; ninf = 0xFC00u; break;
    default: return fail(XGM_ERR_BAD_ARG, "apply: unknown dtype");
  }
  if (reinterpret_cast<uintptr_t>(d_logits) % esize != 0) return fail(XGM_ERR_BAD_ARG, "apply: logits pointer is not aligned to its element size");
  require_device();
  launch_apply(d_logits, esize, ninf, V_logits, row_stride_elems, reinterpret_cast<const uint32_t*>(d_bitmask), V_mask,
               d_row_index, n_rows, static_cast<hipStream_t>(hip_stream));
  HIP_OK(hipGetLastError());
  return XGM_OK;
  API_END
}

}  // extern "C"
