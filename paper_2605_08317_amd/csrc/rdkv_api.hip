// Host side of librdkv: argument validation, planning (segment table, split
// schedule) and kernel launches behind the C ABI of include/rdkv.h.
#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <initializer_list>
#include <mutex>
#include <new>
#include <utility>

#include "decode_merge.h"
#include "rdkv_internal.h"

namespace rdkv {
hipError_t launch_tier_count(const uint8_t* bits, const int64_t* item_tok_off, const int32_t* item_T,
                             const int32_t* item_blk_off, int32_t* blk_counts, int32_t* item_counts,
                             int32_t* invalid, int n_items, int max_T, hipStream_t st);
hipError_t launch_tier_scatter(const uint8_t* bits, const int64_t* item_tok_off, const int32_t* item_T,
                               const int32_t* item_blk_off, const int32_t* blk_offsets, const int64_t* idx_base,
                               int32_t* tier_idx, int n_items, int max_T, hipStream_t st);
hipError_t launch_quant_pack(const uint16_t* K, const uint16_t* V, const int32_t* tier_idx,
                             const int64_t* idx_base, const int32_t* counts, const int64_t* seg_off,
                             const int64_t* item_row_off, uint8_t* arena, int n_items,
                             const int32_t max_count[4], const ItemK* items_k, const uint8_t* bits_ch,
                             uint32_t* k_range, int row_wide, hipStream_t st);
int partition_block();
int weights_block();
size_t weights_scratch_floats(int64_t n_blocks, int64_t n_items, int64_t total_tokens, int R_pad, bool want_ch);
hipError_t launch_weights(const rdkv_config& cfg, const int64_t* d_item_row_off, const int32_t* d_item_T,
                          const int32_t* d_item_blk_off, int64_t n_blocks, int64_t n_items, int64_t total_tokens,
                          int max_T, const uint16_t* K, const uint16_t* Q_obs, float* w_tok, float* w_ch,
                          float* scratch, hipStream_t st);
hipError_t launch_allocate(const float* w, const int64_t* d_item_off, const int32_t* d_item_U,
                           const double* d_item_budget, int n_items, int n_hull, const int* hull_tiers,
                           const double* hull_r, double rel_tol, int max_iters, uint8_t* bits, double* lam_out,
                           int32_t* iters_out, void* multi_scratch, hipStream_t st);
size_t allocate_multi_scratch_bytes(int n_items);
hipError_t launch_calibrate(const uint16_t* K, const uint16_t* V, const int64_t* item_row_off, const int32_t* item_T,
                            int n_items, int max_T, bool k_channelwise, bool k_whole_channel, bool row_wide,
                            double* acc_k, double* acc_v, uint32_t* range, hipStream_t st);
hipError_t launch_stage3_budget(const uint8_t* bits, const int64_t* d_item_off, const int32_t* d_item_U,
                                const double* d_item_avg, double rk, int n_items, int32_t* kept, double* k_budget,
                                hipStream_t st);
}  // namespace rdkv

using namespace rdkv;


namespace {

thread_local std::string g_err;

rdkv_status fail(rdkv_status s, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof(buf), fmt, ap);
  va_end(ap);
  g_err = buf;
  return s;
}

#define RDKV_HIP(expr)                                                                      \
  do {                                                                                      \
    hipError_t e_ = (expr);                                                                 \
    if (e_ != hipSuccess) return fail(RDKV_ERR_HIP, "%s: %s", #expr, hipGetErrorString(e_)); \
  } while (0)

int64_t round_up(int64_t x, int64_t a) { return (x + a - 1) / a * a; }

// ---- optional event bracketing of the main kernels ----------------------------------
struct KernelTiming {
  std::mutex mu;
  bool enabled = false;
  std::vector<std::pair<hipEvent_t, hipEvent_t>> ev[RDKV_TIME_KINDS];
  std::vector<hipEvent_t> pool;
  hipEvent_t get() {
    if (!pool.empty()) { hipEvent_t e = pool.back(); pool.pop_back(); return e; }
    hipEvent_t e = nullptr;
    return hipEventCreate(&e) == hipSuccess ? e : nullptr;
  }
};
KernelTiming g_timing;

// Device memory of the library.  What a cache owns lives until rdkv_cache_free and comes from alloc() / hipMalloc.
// Scratch of a single call is released when the call returns, while its kernels may still be queued: the release is
// stream-ordered (the caller's hooks must behave like a stream-ordered caching allocator on the call's stream; without
// hooks hipMallocAsync / hipFreeAsync on that stream).
struct Allocator {
  rdkv_alloc_fn alloc = nullptr;
  rdkv_free_fn free_ = nullptr;
  void* user = nullptr;
  void* get(size_t bytes) const {
    if (bytes == 0) bytes = 16;
    if (alloc) return alloc(bytes, user);
    void* p = nullptr;
    return hipMalloc(&p, bytes) == hipSuccess ? p : nullptr;
  }
  void put(void* p) const {
    if (!p) return;
    if (free_) free_(p, user); else (void)hipFree(p);
  }
  void* get_scratch(size_t bytes, hipStream_t st) const {
    if (bytes == 0) bytes = 16;
    if (alloc) return alloc(bytes, user);
    void* p = nullptr;
    return hipMallocAsync(&p, bytes, st) == hipSuccess ? p : nullptr;
  }
  void put_scratch(void* p, hipStream_t st) const {
    if (!p) return;
    if (free_) free_(p, user); else (void)hipFreeAsync(p, st);
  }
};

// Device scratch that is released (stream-ordered) when the call returns.  reserve() takes one allocation up front
// that the following get() calls are carved from; requests that do not fit fall back to allocations of their own.
struct Temp {
  const Allocator& al;
  hipStream_t st;
  std::vector<void*> ptrs;
  uint8_t* slab = nullptr;
  size_t slab_bytes = 0, used = 0;
  Temp(const Allocator& a, hipStream_t s) : al(a), st(s) {}
  ~Temp() { for (void* p : ptrs) al.put_scratch(p, st); }
  static size_t padded(size_t bytes) { return (std::max<size_t>(bytes, 16) + 255) / 256 * 256; }
  void reserve(std::initializer_list<size_t> sizes) {
    size_t total = 0;
    for (size_t b : sizes) total += padded(b);
    slab = static_cast<uint8_t*>(al.get_scratch(total, st));
    if (slab) {
      ptrs.push_back(slab);
      slab_bytes = total;
    }
  }
  template <typename T>
  T* get(size_t n) {
    const size_t b = padded(n * sizeof(T));
    if (slab && used + b <= slab_bytes) {
      T* p = reinterpret_cast<T*>(slab + used);
      used += b;
      return p;
    }
    void* p = al.get_scratch(n * sizeof(T), st);
    if (p) ptrs.push_back(p);
    return static_cast<T*>(p);
  }
};

// Host-to-device copies of small tables without waiting for them: the source is copied into a ring of pinned host
// memory (one per device), the copy is enqueued from there, and an event marks when the ring bytes may be reused.
// A table larger than the ring is copied from the caller's memory and the stream is synchronised.
constexpr int kMaxDevices = 64;
class Staging {
  struct Region { size_t begin, end; hipEvent_t ev; };
  std::mutex mu_;
  uint8_t* base_ = nullptr;
  size_t cap_ = 0, head_ = 0;
  std::vector<Region> live_;       // ring bytes whose copy may not have run yet
  std::vector<hipEvent_t> pool_;
  static constexpr size_t kBytes = static_cast<size_t>(2) << 20;

 public:
  hipError_t upload(void* dst, const void* src, size_t bytes, hipStream_t st) {
    if (bytes == 0) return hipSuccess;
    std::lock_guard<std::mutex> lk(mu_);
    if (!base_) {
      void* p = nullptr;
      if (hipHostMalloc(&p, kBytes, hipHostMallocDefault) == hipSuccess) { base_ = static_cast<uint8_t*>(p); cap_ = kBytes; }
    }
    const size_t need = (bytes + 255) / 256 * 256;
    if (!base_ || need > cap_ / 2) {
      hipError_t e = hipMemcpyAsync(dst, src, bytes, hipMemcpyHostToDevice, st);
      return e != hipSuccess ? e : hipStreamSynchronize(st);
    }
    if (head_ + need > cap_) head_ = 0;      // wrap: the bytes up to the end of the ring are skipped
    for (size_t k = 0; k < live_.size();) {   // copies still reading the bytes about to be overwritten
      if (live_[k].begin < head_ + need && live_[k].end > head_) {
        (void)hipEventSynchronize(live_[k].ev);
        pool_.push_back(live_[k].ev);
        live_.erase(live_.begin() + static_cast<std::ptrdiff_t>(k));
      } else {
        ++k;
      }
    }
    uint8_t* p = base_ + head_;
    std::memcpy(p, src, bytes);
    hipError_t e = hipMemcpyAsync(dst, p, bytes, hipMemcpyHostToDevice, st);
    if (e != hipSuccess) return e;
    hipEvent_t ev = nullptr;
    if (!pool_.empty()) { ev = pool_.back(); pool_.pop_back(); }
    else if ((e = hipEventCreateWithFlags(&ev, hipEventDisableTiming)) != hipSuccess) return hipStreamSynchronize(st);
    if ((e = hipEventRecord(ev, st)) != hipSuccess) { pool_.push_back(ev); return hipStreamSynchronize(st); }
    live_.push_back(Region{head_, head_ + need, ev});
    head_ += need;
    return hipSuccess;
  }
};
Staging g_staging[kMaxDevices];

hipError_t upload(void* dst, const void* src, size_t bytes, hipStream_t st) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) {
    e = hipMemcpyAsync(dst, src, bytes, hipMemcpyHostToDevice, st);
    return e != hipSuccess ? e : hipStreamSynchronize(st);
  }
  return g_staging[dev].upload(dst, src, bytes, st);
}

// Geometry of a ragged batch: one entry per item (sequence-major, head-minor).
struct Items {
  int64_t n_items = 0, total_tokens = 0;
  int32_t max_T = 0;
  std::vector<int32_t> T;          // [items]
  std::vector<int64_t> tok_off;    // [items]: first token of the item in ragged [hkv][T_s] arrays
  std::vector<int32_t> blk_off;    // [items]: first partition block
  int64_t n_blocks = 0;
};

Items make_items(const int32_t* seq_lens, int batch, int hkv) {
  Items it;
  const int pb = partition_block();
  int64_t off = 0;
  int64_t blk = 0;
  for (int s = 0; s < batch; ++s) {
    const int32_t T = seq_lens[s];
    it.max_T = std::max(it.max_T, T);
    for (int h = 0; h < hkv; ++h) {
      it.T.push_back(T);
      it.tok_off.push_back(off);
      it.blk_off.push_back(static_cast<int32_t>(blk));
      off += T;
      blk += (T + pb - 1) / pb;
    }
  }
  it.n_items = static_cast<int64_t>(batch) * hkv;
  it.total_tokens = off;
  it.n_blocks = blk;
  return it;
}

bool valid_tier(int b) { return b == 0 || b == 2 || b == 4 || b == 8 || b == 16; }

rdkv_status check_shape(int batch, int hq, int hkv, int d, const int32_t* seq_lens) {
  if (batch < 0 || hq <= 0 || hkv <= 0) return fail(RDKV_ERR_INVALID_ARG, "batch/hq/hkv must be positive");
  if (d != kHeadDim) return fail(RDKV_ERR_SHAPE, "head_dim %d unsupported (must be 128)", d);
  if (hq % hkv != 0) return fail(RDKV_ERR_SHAPE, "hq %d is not a multiple of hkv %d", hq, hkv);
  const int g = hq / hkv;
  if (!(g == 1 || g == 2 || g == 4 || g == 8)) return fail(RDKV_ERR_SHAPE, "hq/hkv = %d unsupported (1,2,4,8)", g);
  if (batch > 0 && seq_lens == nullptr) return fail(RDKV_ERR_INVALID_ARG, "seq_lens is null");
  int64_t total = 0;
  for (int s = 0; s < batch; ++s) {
    if (seq_lens[s] < 0) return fail(RDKV_ERR_SHAPE, "seq_lens[%d] = %d is negative", s, seq_lens[s]);
    total += static_cast<int64_t>(seq_lens[s]) * hkv;
  }
  if (total >= (1ll << 31)) return fail(RDKV_ERR_SHAPE, "sum of hkv*T_s exceeds 2^31 rows");
  return RDKV_OK;
}

rdkv_status check_config(const rdkv_config* cfg, bool need_budget, bool need_probe) {
  if (cfg == nullptr) return fail(RDKV_ERR_INVALID_ARG, "config is null");
  rdkv_status s = check_shape(cfg->batch, cfg->hq, cfg->hkv, cfg->head_dim, cfg->seq_lens);
  if (s != RDKV_OK) return s;
  if (cfg->group_size != kGroup && cfg->group_size != kHeadDim)
    return fail(RDKV_ERR_SHAPE, "group_size %d unsupported (32, or 128 = one scale per token row)", cfg->group_size);
  if (cfg->k_mode != RDKV_K_TOKENWISE && cfg->k_mode != RDKV_K_CHANNELWISE)
    return fail(RDKV_ERR_INVALID_ARG, "k_mode %d unknown", cfg->k_mode);
  if (need_probe) {
    if (cfg->s_obs <= 0 || cfg->s_obs > 64) return fail(RDKV_ERR_SHAPE, "s_obs %d out of range (1..64)", cfg->s_obs);
    if (cfg->pool_kernel < 1 || cfg->pool_kernel % 2 == 0 || cfg->pool_kernel > 15)
      return fail(RDKV_ERR_INVALID_ARG, "pool_kernel %d must be odd, 1..15", cfg->pool_kernel);
    for (int i = 0; i < cfg->batch; ++i)
      if (cfg->seq_lens[i] < cfg->s_obs)
        return fail(RDKV_ERR_SHAPE, "seq_lens[%d] = %d is shorter than s_obs = %d", i, cfg->seq_lens[i], cfg->s_obs);
  }
  if (need_budget) {
    if (cfg->batch > 0 && cfg->budget_bits == nullptr) return fail(RDKV_ERR_INVALID_ARG, "budget_bits is null");
    for (int i = 0; i < cfg->batch; ++i)
      if (!(cfg->budget_bits[i] >= 0.0f) || !std::isfinite(cfg->budget_bits[i]))
        return fail(RDKV_ERR_INVALID_ARG, "budget_bits[%d] must be finite and >= 0", i);
    if (cfg->n_tiers < 1 || cfg->n_tiers > RDKV_MAX_TIERS) return fail(RDKV_ERR_INVALID_ARG, "n_tiers out of range");
    for (int i = 0; i < cfg->n_tiers; ++i) {
      if (!valid_tier(cfg->tiers[i])) return fail(RDKV_ERR_INVALID_ARG, "tiers[%d] = %d not in {0,2,4,8,16}", i, cfg->tiers[i]);
      if (i > 0 && cfg->tiers[i] <= cfg->tiers[i - 1]) return fail(RDKV_ERR_INVALID_ARG, "tiers must be ascending");
      if (!std::isfinite(cfg->eps_v[i]) || !std::isfinite(cfg->eps_k[i]))
        return fail(RDKV_ERR_INVALID_ARG, "distortion table entry %d is not finite", i);
    }
    if (!(cfg->rel_tol >= 0.0f) || cfg->rel_tol >= 1.0f) return fail(RDKV_ERR_INVALID_ARG, "rel_tol must be in [0,1)");
    if (cfg->max_iters < 1 || cfg->max_iters > 200) return fail(RDKV_ERR_INVALID_ARG, "max_iters must be in 1..200");
    if (!(cfg->kv_split_rk > 0.0f) || !(cfg->kv_split_rk < 1.0f))
      return fail(RDKV_ERR_INVALID_ARG, "kv_split_rk must be in (0,1)");
  }
  return RDKV_OK;
}

// chunk size policy of the dense path; used by the workspace query and the launch alike.  The split kernel stages
// its tiles through 70 KB of LDS per workgroup, so a compute unit keeps two workgroups resident whatever the number
// of query heads: a launch is fastest when its workgroups fill the chip exactly once (512 chunks), and chunks have
// at least 256 rows.
void dense_plan(const int32_t* seq_lens, int batch, int hkv, int g, int* chunk_rows, int* max_splits) {
  int64_t total = 0;
  int max_T = 0;
  for (int s = 0; s < batch; ++s) {
    total += static_cast<int64_t>(seq_lens[s]) * hkv;
    max_T = std::max(max_T, seq_lens[s]);
  }
  (void)g;
  const int64_t resident = 512;
  int64_t cr = round_up(std::max<int64_t>(256, (total + resident - 1) / resident), 64);
  *chunk_rows = static_cast<int>(cr);
  *max_splits = std::max(1, static_cast<int>((max_T + cr - 1) / cr));
}

// What a cache owns on the device.  rdkv_pack takes one block for the arena and every table (one trip through the
// caller's allocator); what later calls add or replace (tail, rebuilt chunk tables, workspaces of other streams) are
// allocations of their own.
void free_cache_buffers(rdkv_cache* c) {
  Allocator al{c->alloc, c->free_, c->alloc_user};
  const uint8_t* b0 = c->d_block;
  const uint8_t* b1 = c->d_block ? c->d_block + c->block_bytes : nullptr;
  auto put = [&](void* p) {
    const uint8_t* q = static_cast<const uint8_t*>(p);
    if (p && !(b0 && q >= b0 && q < b1)) al.put(p);
  };
  put(c->d_arena);
  put(c->d_tier_idx);
  put(c->d_chunks);
  for (const rdkv_cache::Workspace& w : c->workspaces) put(w.block);
  c->workspaces.clear();
  put(c->d_tail_state);
  put(c->d_bits_tok);
  put(c->d_bits_ch);
  put(c->d_items_k);
  put(c->d_items_sched);
  put(c->d_tail);
  put(c->d_lambda);
  put(c->d_iters);
  al.put(c->d_block);
  c->d_block = nullptr;
  for (rdkv_cache* child : c->absorbed) {
    free_cache_buffers(child);
    delete child;
  }
  c->absorbed.clear();
}

// The split workspace of a cache for one stream (created on first use).  Calls on one stream are serialised by
// the stream and share a workspace; calls on different streams get different ones, so they may overlap.
rdkv_status workspace_for(const rdkv_cache* c, hipStream_t st, rdkv_cache::Workspace* out) {
  std::lock_guard<std::mutex> lk(c->ws_mu);
  for (const rdkv_cache::Workspace& w : c->workspaces)
    if (w.stream == st) { *out = w; return RDKV_OK; }
  // A stream under graph capture cannot allocate, and frameworks capture on streams of their own: a captured step
  // uses the cache's first workspace (the one of the stream that built the schedule).
  if (st != nullptr && !c->workspaces.empty()) {
    hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(st, &cs) == hipSuccess && cs == hipStreamCaptureStatusActive) {
      *out = c->workspaces.front();
      return RDKV_OK;
    }
  }
  Allocator al{c->alloc, c->free_, c->alloc_user};
  const int g = c->hq / c->hkv;
  const size_t slots = static_cast<size_t>(std::max<int64_t>(c->n_slots, 1));
  const size_t acc_b = slots * g * kHeadDim * sizeof(float), ml_b = (slots * g * 2 * sizeof(float) + 255) / 256 * 256;
  const size_t arr_b = static_cast<size_t>(std::max<int64_t>(c->n_items, 1)) * sizeof(int32_t);
  uint8_t* block = static_cast<uint8_t*>(al.get(acc_b + ml_b + arr_b));
  if (!block) return fail(RDKV_ERR_ALLOC, "device allocation of a split workspace failed");
  rdkv_cache::Workspace w{st, reinterpret_cast<float*>(block), reinterpret_cast<float*>(block + acc_b),
                          reinterpret_cast<int32_t*>(block + acc_b + ml_b), block};
  const hipError_t e = hipMemsetAsync(w.arrive, 0, arr_b, st);     // counters start at zero; the kernels keep them so
  if (e != hipSuccess) {
    al.put(block);
    return fail(RDKV_ERR_HIP, "clearing a split workspace: %s", hipGetErrorString(e));
  }
  c->workspaces.push_back(w);
  *out = w;
  return RDKV_OK;
}

void drop_workspaces(rdkv_cache* c) {
  std::lock_guard<std::mutex> lk(c->ws_mu);
  Allocator al{c->alloc, c->free_, c->alloc_user};
  for (const rdkv_cache::Workspace& w : c->workspaces) al.put(w.block);
  c->workspaces.clear();
}

// Launch order of a decode kernel's chunks.  Large launches: tier by tier, lowest bit-width first and largest first
// inside a tier, so that the chunks that cost most time per byte start first and the last to finish are 8-bit ones
// (measured 4-5 % faster on a mixed-tier batch than plain size order).  Launches that fit the chip in one round:
// round-robin over the items, so that with the usual round-robin placement of workgroups on the eight XCDs the
// chunks of an item share an L2 (which then also holds the partials their merge reads); only speed depends on it.
void order_chunks(std::vector<Chunk>::iterator first, std::vector<Chunk>::iterator last, int64_t n_items) {
  const int64_t count = last - first;
  std::stable_sort(first, last, [](const Chunk& x, const Chunk& y) {
    if (x.tier != y.tier) return x.tier < y.tier;
    return static_cast<int64_t>(x.rows) * x.tier > static_cast<int64_t>(y.rows) * y.tier;
  });
  if (count > 1024 || n_items <= 1) return;
  std::vector<std::vector<Chunk>> by_item(static_cast<size_t>(n_items));
  for (auto it = first; it != last; ++it) by_item[it->item].push_back(*it);
  auto out = first;
  for (size_t k = 0; out != last; ++k)
    for (int64_t i = 0; i < n_items; ++i)
      if (k < by_item[i].size()) *out++ = by_item[i][k];
}

// every chunk learns its item's first partial slot and slot count (the merge inside the decode kernels needs them)
void stamp_slots(std::vector<Chunk>& table, const std::vector<int32_t>& slot_begin, const std::vector<int32_t>& slot_count) {
  for (Chunk& ch : table) {
    ch.slot0 = slot_begin[ch.item];
    ch.nslots = slot_count[ch.item];
  }
}

// Sorted-channel layout of one item's K tiles from its channel bit map.
ItemK make_item_k(const uint8_t* bits_ch) {
  ItemK k;
  std::memset(&k, 0, sizeof(k));
  int slot = 0, words = 0, qsteps = 0;
  for (int ti = 0; ti < 4; ++ti) {
    const int b = pack_tier_bits(ti);
    const int pad = ti == 0 ? 4 : 32 / b;            // whole word pairs (16-bit) / whole words
    k.slot_base[ti] = static_cast<int16_t>(slot);
    int cnt = 0;
    for (int c = 0; c < kHeadDim; ++c)
      if (bits_ch[c] == b) k.slot_ch[slot + cnt++] = static_cast<int16_t>(c);
    const int npad = (cnt + pad - 1) / pad * pad;
    for (int j = cnt; j < npad; ++j) k.slot_ch[slot + j] = -1;
    slot += npad;
    words += npad * b / 32;
    k.word_end[ti] = static_cast<int16_t>(words);
    if (ti == 0) k.n_steps16 = static_cast<int16_t>(npad / 4); else qsteps += npad / 4;
  }
  k.n_slots = static_cast<int16_t>(slot);
  k.n_qsteps = static_cast<int16_t>(qsteps);
  k.n_words = static_cast<int16_t>(words);
  k.n_words_padded = static_cast<int16_t>((words + 1) / 2 * 2);
  k.kt_bytes = 256 * k.n_words_padded;
  k.km_bytes = 32 * k.n_qsteps;
  for (int j = slot; j < kMaxSlots; ++j) k.slot_ch[j] = -1;
  return k;
}

// Lower convex hull of (b_k, eps_k) and the threshold ratios r_k = db / (-d eps) of its edges.
void hull_thresholds(const rdkv_config* cfg, const float* eps, std::vector<int>* tiers, std::vector<double>* r) {
  struct P { double b, e; };
  std::vector<P> h;
  for (int i = 0; i < cfg->n_tiers; ++i) {
    const P p{static_cast<double>(cfg->tiers[i]), static_cast<double>(eps[i])};
    while (h.size() >= 2) {
      const P& a = h[h.size() - 2];
      const P& b = h[h.size() - 1];
      const double cross = (b.b - a.b) * (p.e - a.e) - (b.e - a.e) * (p.b - a.b);
      if (cross <= 0.0) h.pop_back(); else break;
    }
    h.push_back(p);
  }
  tiers->clear();
  r->clear();
  tiers->push_back(static_cast<int>(h[0].b));
  for (size_t k = 1; k < h.size(); ++k) {
    const double de = h[k - 1].e - h[k].e;
    if (!(de > 0.0)) break;
    tiers->push_back(static_cast<int>(h[k].b));
    r->push_back((h[k].b - h[k - 1].b) / de);
  }
}


// Device tables of one pass over a ragged batch (one entry per item), sent in a single copy.
struct Tables {
  int64_t* tok_off = nullptr;    // first token of the item in ragged [hkv][T_s] arrays
  double* budget = nullptr;      // average bits of the token map (channel-wise mode: the V share)
  double* avg = nullptr;         // average bits per cache element of the item's sequence
  int64_t* ch_off = nullptr;     // item * 128
  int32_t* T = nullptr;
  int32_t* wblk_off = nullptr;   // first workgroup of the item in the weights kernels
  int32_t* blk_off = nullptr;    // first partition block of the item
  int32_t* ch_U = nullptr;       // 128
  int64_t n_wblk = 0;
};

rdkv_status make_tables(const rdkv_config* cfg, const Items& it, bool with_budget, Temp& tmp, hipStream_t st,
                        Tables* out) {
  const size_t n = static_cast<size_t>(std::max<int64_t>(it.n_items, 1));
  const bool mixed = cfg->k_mode == RDKV_K_CHANNELWISE;
  std::vector<uint8_t> blob(48 * n, 0);
  int64_t* tok_off = reinterpret_cast<int64_t*>(blob.data());
  double* budget = reinterpret_cast<double*>(blob.data() + 8 * n);
  double* avg = reinterpret_cast<double*>(blob.data() + 16 * n);
  int64_t* ch_off = reinterpret_cast<int64_t*>(blob.data() + 24 * n);
  int32_t* T = reinterpret_cast<int32_t*>(blob.data() + 32 * n);
  int32_t* wblk = T + n;
  int32_t* blk = T + 2 * n;
  int32_t* ch_U = T + 3 * n;
  const int wb = weights_block();
  int64_t n_wblk = 0;
  for (int64_t i = 0; i < it.n_items; ++i) {
    tok_off[i] = it.tok_off[i];
    T[i] = it.T[i];
    blk[i] = it.blk_off[i];
    wblk[i] = static_cast<int32_t>(n_wblk);
    n_wblk += (it.T[i] + wb - 1) / wb;
    ch_off[i] = i * kHeadDim;
    ch_U[i] = kHeadDim;
    if (with_budget) {
      // Stage 2.  Token-wise mode: the sequence's average serves K and V alike.  Channel-wise mode: V gets the share
      // 1 - r_K of the head budget, i.e. 2 (1 - r_K) avg_bits per token unit (rounded to fp32 like every budget).
      const double a = static_cast<double>(cfg->budget_bits[i / cfg->hkv]);
      avg[i] = a;
      budget[i] = mixed ? static_cast<double>(static_cast<float>(2.0 * (1.0 - static_cast<double>(cfg->kv_split_rk)) * a)) : a;
    }
  }
  uint8_t* d = tmp.get<uint8_t>(blob.size());
  if (!d) return fail(RDKV_ERR_ALLOC, "device allocation failed");
  RDKV_HIP(upload(d, blob.data(), blob.size(), st));
  out->tok_off = reinterpret_cast<int64_t*>(d);
  out->budget = reinterpret_cast<double*>(d + 8 * n);
  out->avg = reinterpret_cast<double*>(d + 16 * n);
  out->ch_off = reinterpret_cast<int64_t*>(d + 24 * n);
  out->T = reinterpret_cast<int32_t*>(d + 32 * n);
  out->wblk_off = out->T + n;
  out->blk_off = out->T + 2 * n;
  out->ch_U = out->T + 3 * n;
  out->n_wblk = n_wblk;
  return RDKV_OK;
}

// Stage 1 of Alg. 1; everything is enqueued on st, nothing waits.
rdkv_status weights_impl(const rdkv_config* cfg, const Items& it, const Tables& tb, const void* K, const void* Q_obs,
                         float* w_tok, float* w_ch, Temp& tmp, hipStream_t st) {
  const int R_pad = (cfg->hq / cfg->hkv * cfg->s_obs + 15) / 16 * 16;
  const size_t nscr = weights_scratch_floats(tb.n_wblk, it.n_items, it.total_tokens, R_pad, w_ch != nullptr);
  float* scratch = tmp.get<float>(nscr);
  if (!scratch) return fail(RDKV_ERR_ALLOC, "device allocation failed");
  TimedScope ts(RDKV_TIME_WEIGHTS, st);
  RDKV_HIP(launch_weights(*cfg, tb.tok_off, tb.T, tb.wblk_off, tb.n_wblk, it.n_items, it.total_tokens, it.max_T,
                          static_cast<const uint16_t*>(K), static_cast<const uint16_t*>(Q_obs), w_tok, w_ch, scratch,
                          st));
  return RDKV_OK;
}

// Stages 2-3 of Alg. 1; everything is enqueued on st, nothing waits.  lam / iters: device [items] (token map), in
// channel-wise mode followed by [items] for the channel map; or null.
rdkv_status allocate_impl(const rdkv_config* cfg, const Items& it, const Tables& tb, const float* w_tok,
                          const float* w_ch, uint8_t* bits_tok, uint8_t* bits_ch, double* lam, int32_t* iters,
                          Temp& tmp, hipStream_t st) {
  const bool mixed = cfg->k_mode == RDKV_K_CHANNELWISE;
  const int n = static_cast<int>(it.n_items);
  std::vector<int> ht;
  std::vector<double> hr;
  hull_thresholds(cfg, cfg->eps_v, &ht, &hr);
  // items of 16K tokens and more: the passes over the weights run on many workgroups per item
  void* multi = nullptr;
  if (it.max_T >= 16384 && n <= 512) {
    multi = tmp.get<uint8_t>(allocate_multi_scratch_bytes(n));
    if (!multi) return fail(RDKV_ERR_ALLOC, "device allocation failed");
  }
  TimedScope ts(RDKV_TIME_ALLOCATE, st);      // every kernel of the stage
  RDKV_HIP(launch_allocate(w_tok, tb.tok_off, tb.T, tb.budget, n, static_cast<int>(ht.size()), ht.data(), hr.data(),
                           1.0 - static_cast<double>(cfg->rel_tol), cfg->max_iters, bits_tok, lam, iters, multi, st));
  if (!mixed) return RDKV_OK;
  // Stage 3, on the device: retained tokens per item, then k_avg = min(16, 2 r_K avg_bits T / n_kept)
  int32_t* d_kept = tmp.get<int32_t>(it.n_items);
  double* d_kbudget = tmp.get<double>(it.n_items);
  if (!d_kept || !d_kbudget) return fail(RDKV_ERR_ALLOC, "device allocation failed");
  RDKV_HIP(launch_stage3_budget(bits_tok, tb.tok_off, tb.T, tb.avg, static_cast<double>(cfg->kv_split_rk), n, d_kept,
                                d_kbudget, st));
  hull_thresholds(cfg, cfg->eps_k, &ht, &hr);
  RDKV_HIP(launch_allocate(w_ch, tb.ch_off, tb.ch_U, d_kbudget, n, static_cast<int>(ht.size()), ht.data(), hr.data(),
                           1.0 - static_cast<double>(cfg->rel_tol), cfg->max_iters, bits_ch, lam ? lam + n : nullptr,
                           iters ? iters + n : nullptr, nullptr, st));
  return RDKV_OK;
}

rdkv_status pack_impl(const rdkv_config* cfg, const Items& it, const Tables& tb, const void* K, const void* V,
                      const uint8_t* bits_tok, const uint8_t* bits_ch, double* lam, int32_t* iters, Temp& tmp,
                      hipStream_t st, rdkv_cache** out) {
  const bool mixed = cfg->k_mode == RDKV_K_CHANNELWISE;
  Allocator al{cfg->alloc, cfg->free_, cfg->alloc_user};
  const int g = cfg->hq / cfg->hkv;

  rdkv_cache* c = new (std::nothrow) rdkv_cache();
  if (!c) return fail(RDKV_ERR_ALLOC, "host allocation failed");
  c->batch = cfg->batch; c->hq = cfg->hq; c->hkv = cfg->hkv; c->d = cfg->head_dim; c->k_mode = cfg->k_mode;
  c->k_per_unit = (cfg->k_mode == RDKV_K_CHANNELWISE && cfg->k_scale_per_channel) ? 1 : 0;
  c->group_size = cfg->group_size;
  c->seq_lens.assign(cfg->seq_lens, cfg->seq_lens + cfg->batch);
  c->n_items = it.n_items; c->total_tokens = it.total_tokens;
  c->alloc = cfg->alloc; c->free_ = cfg->free_; c->alloc_user = cfg->alloc_user;
  auto bail = [&](rdkv_status code) { free_cache_buffers(c); delete c; return code; };
#define PACK_HIP(expr)                                                                             \
  do {                                                                                             \
    hipError_t e_ = (expr);                                                                        \
    if (e_ != hipSuccess) return bail(fail(RDKV_ERR_HIP, "%s: %s", #expr, hipGetErrorString(e_))); \
  } while (0)

  const int64_t n = it.n_items;
  c->counts.assign(n * 4, 0);
  c->seg_off.assign(n * 16, 0);
  const size_t n1 = static_cast<size_t>(std::max<int64_t>(n, 1));
  int32_t* d_blk_counts = tmp.get<int32_t>(std::max<int64_t>(it.n_blocks * 4, 1));
  int32_t* d_counts = tmp.get<int32_t>(n1 * 4 + 1);          // [items][4], then the invalid-value flag
  int64_t* d_idx_base = tmp.get<int64_t>(n1 * 20);     // [items][4] kept-position bases, then [items][16] segment offsets
  int64_t* d_seg_off = d_idx_base ? d_idx_base + n1 * 4 : nullptr;
  if (!d_blk_counts || !d_counts || !d_idx_base)
    return bail(fail(RDKV_ERR_ALLOC, "device allocation failed"));
  const int64_t* d_tok_off = tb.tok_off;
  const int32_t* d_T = tb.T;
  const int32_t* d_blk_off = tb.blk_off;

  if (n > 0) {
    // the one wait of the pass: the tier counts size the arena and the split schedule
    std::vector<int32_t> h_counts(n * 4 + 1, 0);
    PACK_HIP(hipMemsetAsync(d_counts + n * 4, 0, sizeof(int32_t), st));
    {
      TimedScope ts(RDKV_TIME_PACK, st);      // first half of the stage: the tier counts
      PACK_HIP(launch_tier_count(bits_tok, d_tok_off, d_T, d_blk_off, d_blk_counts, d_counts, d_counts + n * 4,
                                 static_cast<int>(n), it.max_T, st));
    }
    if (it.max_T > 0)
      PACK_HIP(hipMemcpyAsync(h_counts.data(), d_counts, (n * 4 + 1) * sizeof(int32_t), hipMemcpyDeviceToHost, st));
    std::vector<uint8_t> h_bits_ch;
    if (mixed) {
      h_bits_ch.resize(n * kHeadDim);
      PACK_HIP(hipMemcpyAsync(h_bits_ch.data(), bits_ch, n * kHeadDim, hipMemcpyDeviceToHost, st));
    }
    PACK_HIP(hipStreamSynchronize(st));
    if (h_counts[n * 4] != 0)
      return bail(fail(RDKV_ERR_INVALID_ARG, "bits_tok holds a value outside {0, 2, 4, 8, 16}"));
    std::copy(h_counts.begin(), h_counts.begin() + n * 4, c->counts.begin());
    if (mixed) {
      c->items_k.resize(n);
      for (int64_t i = 0; i < n; ++i) {
        for (int ch = 0; ch < kHeadDim; ++ch)
          if (!valid_tier(h_bits_ch[i * kHeadDim + ch]))
            return bail(fail(RDKV_ERR_INVALID_ARG, "bits_ch[%lld][%d] = %d is not a tier", static_cast<long long>(i),
                             ch, h_bits_ch[i * kHeadDim + ch]));
        c->items_k[i] = make_item_k(&h_bits_ch[i * kHeadDim]);
        const ItemK& ik = c->items_k[i];
        if (ik.n_words_padded > kMaxKRowWords)
          return bail(fail(RDKV_ERR_INTERNAL, "K row of item %lld has %d words, more than the decode kernel holds (%d)",
                           static_cast<long long>(i), ik.n_words_padded, kMaxKRowWords));
        c->max_k_words = std::max<int32_t>(c->max_k_words, ik.n_words_padded);
        c->max_k_steps = std::max<int32_t>(c->max_k_steps, ik.n_steps16 + ik.n_qsteps);
        c->max_k_qsteps = std::max<int32_t>(c->max_k_qsteps, ik.n_qsteps);
      }
    }
  }

  // ---- plan: kept-position lists, arena segments, split schedule -------------------------
  std::vector<int64_t> idx_base(n * 4, 0);
  int64_t kept = 0, cur = 0, stored = 0;
  int32_t max_count[4] = {0, 0, 0, 0};
  for (int64_t i = 0; i < n; ++i) {
    for (int ti = 0; ti < 4; ++ti) {
      const int bits = pack_tier_bits(ti);
      const int64_t cnt = c->counts[i * 4 + ti];
      idx_base[i * 4 + ti] = kept;
      kept += cnt;
      max_count[ti] = std::max<int32_t>(max_count[ti], static_cast<int32_t>(cnt));
      const int64_t npad = round_up(cnt, kTile64);
      int64_t sizes[4] = {npad * tier_row_bytes(bits), npad * tier_meta_bytes(bits),
                          npad * tier_row_bytes(bits), npad * tier_meta_bytes(bits)};
      if (mixed) {   // the K segments hold the channel-wise tiles of this tier's tokens
        sizes[0] = npad / kTile64 * c->items_k[i].kt_bytes;
        sizes[1] = c->k_per_unit ? (cnt > 0 ? c->items_k[i].km_bytes / 2 : 0)      // one record per segment
                                 : npad / kTile64 * c->items_k[i].km_bytes;
      }
      for (int si = 0; si < 4; ++si) {
        cur = round_up(cur, kSegAlign);
        c->seg_off[(i * 4 + ti) * 4 + si] = cur;
        cur += sizes[si];
      }
      if (mixed) {
        int64_t kbits = 0, nquant = 0;
        const ItemK& ik = c->items_k[i];
        for (int s2 = 0; s2 < ik.n_slots; ++s2)
          if (ik.slot_ch[s2] >= 0) {
            int t2 = 3;
            while (t2 > 0 && s2 < ik.slot_base[t2]) --t2;
            kbits += pack_tier_bits(t2);
            nquant += t2 > 0;
          }
        const int64_t groups = c->k_per_unit ? (cnt > 0 ? 1 : 0) : (cnt + kKTokenGroup - 1) / kKTokenGroup;
        stored += cnt * kbits / 8 + groups * 4 * nquant;
        stored += cnt * (tier_row_bytes(bits) + tier_meta_bytes(bits));
      } else {
        stored += cnt * 2 * (tier_row_bytes(bits) + tier_meta_bytes(bits));
      }
    }
  }
  c->arena_bytes = round_up(cur, kSegAlign);
  c->kept_total = kept;
  c->stored_bytes = stored;

  // byte-balanced chunks: every workgroup streams about the same number of stored bytes.  Every chunk costs its
  // workgroup a hand-over at the end (partial stores that go through to memory, an arrival atomic whose answer the
  // workgroup waits for) and its item one more partial to merge, so a launch wants exactly one round of workgroups:
  // as many chunks as the chip keeps resident (256 compute units x 2 workgroups of eight wavefronts = 512), never a
  // few more (measured on 4 x 128K tokens of 2-bit rows: 512 chunks 4.9 TB/s, 608 chunks 4.4, 2048 chunks 4.2).
  // Small launches are bound by latencies instead and want fewer, larger chunks still: at least 96 KB (measured on a
  // 16 MB layer: 96 KB chunks 12.6 us, 64 KB 13.4 us, 24 KB 20 us).  Kernels with four-wavefront workgroups (8 query
  // heads per KV head, channel-wise K) keep three workgroups per compute unit resident: 768 chunks of at least 48 KB.
  // channel-wise mode: eight-wavefront workgroups when the launch is small (one workgroup per compute unit holds
  // it) and the kernel has such an instantiation (up to 4 query heads per KV head, K rows of up to 32 words)
  const bool mixed_wide = mixed && g <= 4 && c->max_k_words <= 32 && stored < (static_cast<int64_t>(48) << 20);
  c->mixed_waves = mixed_wide ? 8 : 4;
  const bool wide = (!mixed && g <= 4) || mixed_wide;      // eight-wavefront workgroups
  const int64_t round_chunks = mixed_wide ? 256 : wide ? 512 : 768;
  // Cost of a row of a tier segment: its stored bytes, weighted in token-wise mode by what a byte of that tier costs
  // the decode kernel relative to an 8-bit byte (single-tier launches reach 4.92 / 5.41 / 5.68 / 5.38 TB/s on 2- /
  // 4- / 8- / 16-bit rows): in a launch of one round the slowest chunk sets the time, so chunks are balanced by
  // time, not bytes.
  auto row_cost = [&](int64_t i, int bits) -> int64_t {
    if (!mixed) {
      const int64_t pct = bits == 2 ? 115 : bits == 4 ? 105 : bits == 8 ? 100 : 106;
      return 2 * (tier_row_bytes(bits) + tier_meta_bytes(bits)) * pct / 100;
    }
    return tier_row_bytes(bits) + tier_meta_bytes(bits) + (c->items_k[i].kt_bytes + c->items_k[i].km_bytes + kTile64 - 1) / kTile64;
  };
  // (the 16-bit rows of a token-wise cache run in a kernel of their own and are cut separately below)
  const int ti0 = mixed ? 0 : 1;
  int64_t total_cost = 0, cost16 = 0;
  for (int64_t i = 0; i < n; ++i) {
    for (int ti = ti0; ti < 4; ++ti) total_cost += c->counts[i * 4 + ti] * row_cost(i, pack_tier_bits(ti));
    if (!mixed) cost16 += c->counts[i * 4] * row_cost(i, 16);
  }
  // Number of chunks a chunk cost of cb gives, and the largest chunk's cost.  Chunks of less than an eighth of cb (a
  // tier with a handful of rows) do not count: they finish at once and leave their workgroup slot to the next chunk
  // (16 channel-wise sequences of 64K tokens: six even chunks per item and one tiny one, 899 in all on 768 slots,
  // take 108 us; five or seven per item 127-134 us).
  auto count_chunks = [&](int64_t cb, int64_t* max_cost) {
    int64_t total = 0;
    *max_cost = 0;
    for (int64_t i = 0; i < n; ++i)
      for (int ti = ti0; ti < 4; ++ti) {
        const int64_t cnt = c->counts[i * 4 + ti];
        if (cnt == 0) continue;
        const int64_t rc = row_cost(i, pack_tier_bits(ti));
        if (cnt * rc < cb / 8) continue;
        const int64_t want = std::max<int64_t>(64, cb / rc);
        const int64_t nch = (cnt + want - 1) / want;
        const int64_t rows_per = round_up((cnt + nch - 1) / nch, 64);
        total += (cnt + rows_per - 1) / rows_per;
        *max_cost = std::max(*max_cost, std::min(rows_per, cnt) * rc);
      }
    return total;
  };
  // token-wise mode cuts an item's quantized tiers as one run of work into round(cost / chunk cost) even shares
  auto count_shares = [&](int64_t cb, int64_t* max_cost) {
    int64_t total = 0;
    *max_cost = 0;
    for (int64_t i = 0; i < n; ++i) {
      int64_t item_cost = 0;
      for (int ti = 1; ti < 4; ++ti) item_cost += c->counts[i * 4 + ti] * row_cost(i, pack_tier_bits(ti));
      if (item_cost == 0) continue;
      const int64_t n_wg = std::max<int64_t>(1, (item_cost + cb / 2) / cb);
      total += n_wg;
      *max_cost = std::max(*max_cost, item_cost / n_wg);
    }
    return total;
  };
  // Shares that span tiers pay a start-up per tier (operands rebuilt, the first tiles' latency waited for again):
  // worth it when a chunk streams for tens of microseconds (32 sequences x 128K tokens at 0.4 bit/elt: 101.6 -> 97.6
  // us), not in latency-bound launches (a 16 MB layer: 12.2 -> 13.7 us), which keep one tier per chunk.
  int64_t chunk_bytes = std::max<int64_t>((wide ? 96 : 48) << 10, total_cost / round_chunks);
  const bool shares = !mixed && chunk_bytes >= (192 << 10);
  auto count_any = [&](int64_t cb, int64_t* max_cost) { return shares ? count_shares(cb, max_cost) : count_chunks(cb, max_cost); };
  int64_t max_cost = 0, n_one_round = count_any(chunk_bytes, &max_cost);
  for (int tries = 0; tries < 64 && n_one_round > round_chunks + round_chunks / 50; ++tries) {   // (2 % over is fine)
    chunk_bytes += chunk_bytes / 16 + 1;
    n_one_round = count_any(chunk_bytes, &max_cost);
  }
  // When one round cannot be had (more tier segments than resident workgroups) or would be lopsided (its largest
  // chunk more than a fifth above the mean), about two rounds of smaller chunks even things out instead.
  // (Shares are even up to the rounding of an item's share count and stay in one round: 16 ragged sequences at 8
  // query heads per KV head, 728 chunks 52.9 us against 57.6 us for 1529.)
  if (!shares && (n_one_round > round_chunks + round_chunks / 50 || max_cost * n_one_round > total_cost + total_cost / 5))
    chunk_bytes = std::max<int64_t>((wide ? 96 : 48) << 10, total_cost / (2 * round_chunks));
  // The row-major 16-bit kernel keeps two workgroups per compute unit resident (70 KB of LDS each): one round of
  // its own.
  const int64_t round16 = 512;
  const int64_t chunk_bytes16 = std::max<int64_t>(96 << 10, (cost16 + round16 - 1) / round16);
  std::vector<int32_t> slot_begin(std::max<int64_t>(n, 1), 0), slot_count(std::max<int64_t>(n, 1), 0);
  std::vector<Chunk> conts;     // continuation pieces (token-wise mode): reached through Chunk::next, never launched
  auto make_chunk = [&](int64_t i, int ti, int64_t r0, int64_t rows) {
    const int bits = pack_tier_bits(ti);
    const int64_t* so = &c->seg_off[(i * 4 + ti) * 4];
    Chunk ch{};
    ch.k_data = so[0] + (mixed ? r0 / kTile64 * c->items_k[i].kt_bytes : r0 * tier_row_bytes(bits));
    ch.k_meta = so[1] + (mixed ? (c->k_per_unit ? 0 : r0 / kTile64 * c->items_k[i].km_bytes)
                               : r0 * tier_meta_bytes(bits));
    ch.v_data = so[2] + r0 * tier_row_bytes(bits);
    ch.v_meta = so[3] + r0 * tier_meta_bytes(bits);
    ch.rows = static_cast<int32_t>(rows);
    ch.tier = bits;
    ch.item = static_cast<int32_t>(i);
    for (int t2 = 0; t2 < 4; ++t2) ch.k_word_end[t2] = mixed ? c->items_k[i].word_end[t2] : int16_t(0);
    ch.reserved = static_cast<int32_t>(i);
    ch.next = -1;
    return ch;
  };
  for (int64_t i = 0; i < n; ++i) {
    slot_begin[i] = static_cast<int32_t>(c->chunks.size());
    // segments cut tier by tier: every tier, or only the 16-bit tier (its own kernel) when the quantized tiers of a
    // token-wise item are cut into shares below
    for (int ti = 0; ti < (shares ? 1 : 4); ++ti) {
      const int bits = pack_tier_bits(ti);
      const int64_t cnt = c->counts[i * 4 + ti];
      if (cnt == 0) continue;
      const int64_t per_row = row_cost(i, bits);
      const int64_t want = std::max<int64_t>(64, (!mixed && bits == 16 ? chunk_bytes16 : chunk_bytes) / per_row);
      const int64_t nch = (cnt + want - 1) / want;
      const int64_t rows_per = round_up((cnt + nch - 1) / nch, 64);
      for (int64_t r0 = 0; r0 < cnt; r0 += rows_per) {
        Chunk ch = make_chunk(i, ti, r0, std::min<int64_t>(rows_per, cnt - r0));
        ch.slot = static_cast<int32_t>(c->chunks.size());
        c->chunks.push_back(ch);
      }
    }
    if (shares) {
      // The quantized tiers of a token-wise item are one run of work -- 2-bit rows, then 4-bit, then 8-bit -- cut
      // into equal shares of cost whatever the tiers' sizes: a workgroup's share may span two or three tiers (its
      // pieces are chained through Chunk::next and feed one softmax state), so every launch, single-tier or not,
      // gets chunks of even cost.
      int64_t item_cost = 0;
      for (int ti = 1; ti < 4; ++ti) item_cost += c->counts[i * 4 + ti] * row_cost(i, pack_tier_bits(ti));
      const int64_t n_wg = item_cost == 0 ? 0 : std::max<int64_t>(1, (item_cost + chunk_bytes / 2) / chunk_bytes);
      int ti = 3;            // walk the segments from the 2-bit tier up
      int64_t r0 = 0;        // first row of the current segment not handed out yet
      for (int64_t k = 0; k < n_wg; ++k) {
        int64_t share = item_cost / n_wg;     // what this workgroup should take
        int32_t prev = -1;                    // index of the workgroup's previous piece: >= 0 in conts, -2 - x: chunk x
        while (ti >= 1) {
          const int64_t left = c->counts[i * 4 + ti] - r0;
          if (left <= 0) { --ti; r0 = 0; continue; }
          const int64_t rc = row_cost(i, pack_tier_bits(ti));
          int64_t take = k + 1 == n_wg ? left : std::min<int64_t>(left, round_up(std::max<int64_t>(share, rc) / rc, 64));
          if (k + 1 < n_wg && left - take < 64) take = left;     // no slivers
          Chunk ch = make_chunk(i, ti, r0, take);
          if (prev == -1) {
            ch.slot = static_cast<int32_t>(c->chunks.size());
            c->chunks.push_back(ch);
            prev = -2 - ch.slot;
          } else {
            const int32_t me = static_cast<int32_t>(conts.size());
            conts.push_back(ch);
            if (prev <= -2) c->chunks[-2 - prev].next = me; else conts[prev].next = me;   // local index for now
            prev = me;
          }
          r0 += take;
          share -= take * rc;
          if (k + 1 < n_wg && share < 64 * rc) break;            // the share is used up
        }
      }
    }
    if (static_cast<int32_t>(c->chunks.size()) == slot_begin[i]) {
      // nothing retained: an empty chunk, so that a workgroup still writes the item's output rows (0, lse = -inf)
      Chunk ch{};
      ch.tier = 2;
      ch.item = static_cast<int32_t>(i);
      ch.slot = static_cast<int32_t>(c->chunks.size());
      ch.reserved = static_cast<int32_t>(i);
      ch.next = -1;
      c->chunks.push_back(ch);
    }
    slot_count[i] = static_cast<int32_t>(c->chunks.size()) - slot_begin[i];
  }
  c->n_slots = static_cast<int64_t>(c->chunks.size());
  stamp_slots(c->chunks, slot_begin, slot_count);
  // 16-bit chunks first (their own kernel), then the launched quantized ones, then the continuation pieces
  std::stable_partition(c->chunks.begin(), c->chunks.end(), [](const Chunk& x) { return x.tier == 16; });
  {
    int64_t n16 = 0;
    for (const Chunk& ch : c->chunks) n16 += ch.tier == 16;
    order_chunks(c->chunks.begin(), c->chunks.begin() + n16, n);
    order_chunks(c->chunks.begin() + n16, c->chunks.end(), n);
  }
  c->n_chunks16 = 0;
  for (const Chunk& ch : c->chunks) c->n_chunks16 += ch.tier == 16;
  c->sched16 = c->n_chunks16;
  c->schedq = static_cast<int64_t>(c->chunks.size()) - c->n_chunks16;
  c->n_cont = static_cast<int64_t>(conts.size());
  {   // Chunk::next becomes an index into the whole table
    const int32_t base = static_cast<int32_t>(c->chunks.size());
    for (Chunk& ch : c->chunks) if (ch.next >= 0) ch.next += base;
    for (Chunk& ch : conts) if (ch.next >= 0) ch.next += base;
    c->chunks.insert(c->chunks.end(), conts.begin(), conts.end());
  }
  const int64_t n_chunks = static_cast<int64_t>(c->chunks.size());
  c->own_slot_count.assign(slot_count.begin(), slot_count.begin() + n);

  // ---- allocate what the cache owns: one block --------------------------------------------
  // [arena | tail state | arrival counters of this stream's workspace]  (cleared together)
  // [kept positions | token bit map | channel bit map | K row layouts, chunk table (one copy) | partials | lambda, steps]
  {
    auto up = [](int64_t b) { return round_up(std::max<int64_t>(b, 16), 256); };
    const int64_t o_state = c->arena_bytes, o_arrive = o_state + 256, o_idx = o_arrive + up(n * 4);
    const int64_t o_bt = o_idx + up(kept * 4), o_bc = o_bt + up(it.total_tokens);
    const int64_t o_ik = o_bc + (mixed ? up(n * kHeadDim) : 0);
    const int64_t ik_b = mixed ? round_up(n * static_cast<int64_t>(sizeof(ItemK)), 8) : 0;
    const int64_t o_acc = o_ik + up(ik_b + n_chunks * static_cast<int64_t>(sizeof(Chunk)));
    const int64_t o_ml = o_acc + up(std::max<int64_t>(n_chunks, 1) * g * kHeadDim * 4);
    const int64_t o_lam = o_ml + up(std::max<int64_t>(n_chunks, 1) * g * 2 * 4);
    const int maps = mixed ? 2 : 1;
    const int64_t o_it = o_lam + (lam ? up(maps * n * 8) : 0);
    const int64_t total = o_it + (iters ? up(maps * n * 4) : 0);
    c->d_block = static_cast<uint8_t*>(al.get(total));
    if (!c->d_block)
      return bail(fail(RDKV_ERR_ALLOC, "device allocation of the packed cache failed (%lld bytes)", static_cast<long long>(total)));
    c->block_bytes = total;
    c->d_arena = c->d_block;
    c->d_tail_state = reinterpret_cast<int32_t*>(c->d_block + o_state);
    c->d_tier_idx = reinterpret_cast<int32_t*>(c->d_block + o_idx);
    c->d_bits_tok = c->d_block + o_bt;
    if (mixed) {
      c->d_bits_ch = c->d_block + o_bc;
      c->d_items_k = reinterpret_cast<ItemK*>(c->d_block + o_ik);
    }
    c->d_chunks = reinterpret_cast<Chunk*>(c->d_block + o_ik + ik_b);
    c->index_bytes = total - c->arena_bytes;     // everything else in the block
    if (n > 0) {
      // nothing below waits: tables are copied out of pinned staging memory, and the host vectors may go
      PACK_HIP(hipMemsetAsync(c->d_block, 0, o_idx, st));     // arena (padding rows read as zeros), tail state, counters
      std::vector<int64_t> plan(idx_base);
      plan.resize(n1 * 4, 0);
      plan.insert(plan.end(), c->seg_off.begin(), c->seg_off.end());
      PACK_HIP(upload(d_idx_base, plan.data(), plan.size() * sizeof(int64_t), st));
      std::vector<uint8_t> tables(static_cast<size_t>(ik_b + n_chunks * static_cast<int64_t>(sizeof(Chunk))));
      if (mixed) std::memcpy(tables.data(), c->items_k.data(), n * sizeof(ItemK));
      if (n_chunks > 0) std::memcpy(tables.data() + ik_b, c->chunks.data(), n_chunks * sizeof(Chunk));
      if (!tables.empty()) PACK_HIP(upload(c->d_block + o_ik, tables.data(), tables.size(), st));
      c->slot_begin = slot_begin;
      c->slot_count = slot_count;
      {   // the split workspace of this stream lives in the block: a first decode under graph capture allocates nothing
        std::lock_guard<std::mutex> lk(c->ws_mu);
        c->workspaces.push_back(rdkv_cache::Workspace{st, reinterpret_cast<float*>(c->d_block + o_acc),
                                                      reinterpret_cast<float*>(c->d_block + o_ml),
                                                      reinterpret_cast<int32_t*>(c->d_block + o_arrive), nullptr});
      }
      if (lam) PACK_HIP(hipMemcpyAsync(c->d_block + o_lam, lam, maps * n * 8, hipMemcpyDeviceToDevice, st));
      if (iters) PACK_HIP(hipMemcpyAsync(c->d_block + o_it, iters, maps * n * 4, hipMemcpyDeviceToDevice, st));
    }
    if (lam) c->d_lambda = reinterpret_cast<double*>(c->d_block + o_lam);
    if (iters) c->d_iters = reinterpret_cast<int32_t*>(c->d_block + o_it);
  }

  if (n > 0) {
    if (it.total_tokens > 0)
      PACK_HIP(hipMemcpyAsync(c->d_bits_tok, bits_tok, it.total_tokens, hipMemcpyDeviceToDevice, st));
    if (mixed) PACK_HIP(hipMemcpyAsync(c->d_bits_ch, bits_ch, n * kHeadDim, hipMemcpyDeviceToDevice, st));
    if (kept > 0) {
      uint32_t* d_krange = nullptr;
      if (c->k_per_unit) {   // per-channel (minimum, maximum) over all retained tokens, as ordered integers
        d_krange = tmp.get<uint32_t>(n * kHeadDim * 2);
        if (!d_krange) return bail(fail(RDKV_ERR_ALLOC, "device allocation failed"));
        std::vector<uint32_t> h_krange(static_cast<size_t>(n) * kHeadDim * 2);
        for (size_t k = 0; k < h_krange.size(); k += 2) { h_krange[k] = 0xFFFFFFFFu; h_krange[k + 1] = 0u; }
        PACK_HIP(upload(d_krange, h_krange.data(), h_krange.size() * sizeof(uint32_t), st));
      }
      TimedScope ts(RDKV_TIME_PACK, st);      // second half: kept-position lists, quantize and pack
      PACK_HIP(launch_tier_scatter(bits_tok, d_tok_off, d_T, d_blk_off, d_blk_counts, d_idx_base, c->d_tier_idx,
                                   static_cast<int>(n), it.max_T, st));
      PACK_HIP(launch_quant_pack(static_cast<const uint16_t*>(K), static_cast<const uint16_t*>(V), c->d_tier_idx,
                                 d_idx_base, d_counts, d_seg_off, d_tok_off, c->d_arena, static_cast<int>(n),
                                 max_count, mixed ? c->d_items_k : nullptr, mixed ? c->d_bits_ch : nullptr, d_krange,
                                 c->group_size == kHeadDim ? 1 : 0, st));
    }
  }
#undef PACK_HIP
  *out = c;
  return RDKV_OK;
}


}  // namespace

namespace rdkv {
void timing_begin(int kind, hipStream_t st) {
  std::lock_guard<std::mutex> lk(g_timing.mu);
  if (!g_timing.enabled) return;
  hipEvent_t a = g_timing.get(), b = g_timing.get();
  if (!a || !b) return;
  (void)hipEventRecord(a, st);
  g_timing.ev[kind].emplace_back(a, b);
}
void timing_end(int kind, hipStream_t st) {
  std::lock_guard<std::mutex> lk(g_timing.mu);
  if (!g_timing.enabled || g_timing.ev[kind].empty()) return;
  (void)hipEventRecord(g_timing.ev[kind].back().second, st);
}
}  // namespace rdkv

extern "C" {

rdkv_status rdkv_kernel_timing_enable(int32_t enable) {
  std::lock_guard<std::mutex> lk(g_timing.mu);
  g_timing.enabled = enable != 0;
  return RDKV_OK;
}

rdkv_status rdkv_kernel_timing_read(int32_t kind, int64_t* launches, double* total_ms) {
  if (kind < 0 || kind >= RDKV_TIME_KINDS || !launches || !total_ms)
    return fail(RDKV_ERR_INVALID_ARG, "bad timing kind or null output");
  std::lock_guard<std::mutex> lk(g_timing.mu);
  double sum = 0.0;
  int64_t n = 0;
  for (auto& pr : g_timing.ev[kind]) {
    float ms = 0.f;
    if (hipEventSynchronize(pr.second) == hipSuccess && hipEventElapsedTime(&ms, pr.first, pr.second) == hipSuccess) {
      sum += ms;
      ++n;
    }
    g_timing.pool.push_back(pr.first);
    g_timing.pool.push_back(pr.second);
  }
  g_timing.ev[kind].clear();
  *launches = n;
  *total_ms = sum;
  return RDKV_OK;
}

const char* rdkv_version(void) { return "rdkv-mi355x 0.1 (gfx950)"; }
const char* rdkv_last_error(void) { return g_err.c_str(); }

rdkv_status rdkv_config_default(rdkv_config* cfg) {
  if (!cfg) return fail(RDKV_ERR_INVALID_ARG, "config is null");
  std::memset(cfg, 0, sizeof(*cfg));
  cfg->head_dim = kHeadDim;
  cfg->s_obs = 32;
  cfg->pool_kernel = 5;
  cfg->causal = 1;
  cfg->k_mode = RDKV_K_TOKENWISE;
  cfg->group_size = kGroup;
  cfg->kv_split_rk = 0.5f;
  cfg->k_scale_per_channel = 0;
  cfg->n_tiers = 5;
  const int t[5] = {0, 2, 4, 8, 16};
  const float ev[5] = {1.0f, 0.313f, 0.0140f, 4.9e-5f, 0.0f};
  const float ek[5] = {1.0f, 0.149f, 0.0062f, 2.2e-5f, 0.0f};
  for (int i = 0; i < 5; ++i) {
    cfg->tiers[i] = t[i];
    cfg->eps_v[i] = ev[i];
    cfg->eps_k[i] = ek[i];
  }
  cfg->rel_tol = 1e-2f;
  cfg->max_iters = 64;
  return RDKV_OK;
}

rdkv_status rdkv_weights(const rdkv_config* cfg, const void* K, const void* Q_obs, float* w_tok,
                         float* w_ch, void* stream) {
  rdkv_status s = check_config(cfg, false, true);
  if (s != RDKV_OK) return s;
  if (cfg->batch == 0) return RDKV_OK;       // (the buffers of an empty batch may be null)
  if (!K || !Q_obs || !w_tok) return fail(RDKV_ERR_INVALID_ARG, "K, Q_obs and w_tok must not be null");
  hipStream_t st = static_cast<hipStream_t>(stream);
  Allocator al{cfg->alloc, cfg->free_, cfg->alloc_user};
  Temp tmp(al, st);
  Items it = make_items(cfg->seq_lens, cfg->batch, cfg->hkv);
  Tables tb;
  s = make_tables(cfg, it, false, tmp, st, &tb);
  if (s != RDKV_OK) return s;
  return weights_impl(cfg, it, tb, K, Q_obs, w_tok, w_ch, tmp, st);
}

rdkv_status rdkv_calibrate_eps(const rdkv_config* cfg, const void* K, const void* V, double* eps_k, double* eps_v,
                               void* stream) {
  if (!cfg) return fail(RDKV_ERR_INVALID_ARG, "cfg must not be null");
  rdkv_status s = check_shape(cfg->batch, cfg->hq, cfg->hkv, cfg->head_dim, cfg->seq_lens);
  if (s != RDKV_OK) return s;
  if (cfg->k_mode != RDKV_K_TOKENWISE && cfg->k_mode != RDKV_K_CHANNELWISE)
    return fail(RDKV_ERR_INVALID_ARG, "k_mode must be RDKV_K_TOKENWISE or RDKV_K_CHANNELWISE");
  if (cfg->group_size != kGroup && cfg->group_size != kHeadDim)
    return fail(RDKV_ERR_SHAPE, "group_size %d unsupported (32, or 128 = one scale per token row)", cfg->group_size);
  if (!K || !V || !eps_k || !eps_v) return fail(RDKV_ERR_INVALID_ARG, "K, V, eps_k and eps_v must not be null");
  if (cfg->batch == 0) return RDKV_OK;
  for (int b = 0; b < cfg->batch; ++b)
    if (cfg->seq_lens[b] < 1) return fail(RDKV_ERR_SHAPE, "seq_lens[%d] = %d: calibration needs at least one token", b, cfg->seq_lens[b]);
  hipStream_t st = static_cast<hipStream_t>(stream);
  Allocator al{cfg->alloc, cfg->free_, cfg->alloc_user};
  Temp tmp(al, st);
  Items it = make_items(cfg->seq_lens, cfg->batch, cfg->hkv);
  const size_t n = static_cast<size_t>(it.n_items);
  const bool channelwise = cfg->k_mode == RDKV_K_CHANNELWISE;
  const bool whole = channelwise && cfg->k_scale_per_channel != 0;
  tmp.reserve({n * sizeof(int64_t), n * sizeof(int32_t), n * 8 * sizeof(double),
               whole ? n * kHeadDim * 2 * sizeof(uint32_t) : 0});
  int64_t* d_off = tmp.get<int64_t>(n);
  int32_t* d_T = tmp.get<int32_t>(n);
  double* d_acc = tmp.get<double>(n * 8);                       // [K | V][items][4]
  uint32_t* d_range = whole ? tmp.get<uint32_t>(n * kHeadDim * 2) : nullptr;
  if (!d_off || !d_T || !d_acc || (whole && !d_range)) return fail(RDKV_ERR_ALLOC, "device allocation failed");
  std::vector<double> h_acc(n * 8, 0.0);
  std::vector<uint32_t> h_range;
  RDKV_HIP(upload(d_off, it.tok_off.data(), n * sizeof(int64_t), st));
  RDKV_HIP(upload(d_T, it.T.data(), n * sizeof(int32_t), st));
  RDKV_HIP(upload(d_acc, h_acc.data(), h_acc.size() * sizeof(double), st));
  if (whole) {
    h_range.resize(n * kHeadDim * 2);
    for (size_t k = 0; k < h_range.size(); k += 2) { h_range[k] = 0xFFFFFFFFu; h_range[k + 1] = 0u; }
    RDKV_HIP(upload(d_range, h_range.data(), h_range.size() * sizeof(uint32_t), st));
  }
  {
    TimedScope ts(RDKV_TIME_CALIBRATE, st);
    RDKV_HIP(launch_calibrate(static_cast<const uint16_t*>(K), static_cast<const uint16_t*>(V), d_off, d_T,
                              static_cast<int>(n), it.max_T, channelwise, whole, cfg->group_size == kHeadDim, d_acc,
                              d_acc + n * 4, d_range, st));
  }
  RDKV_HIP(hipMemcpyAsync(h_acc.data(), d_acc, h_acc.size() * sizeof(double), hipMemcpyDeviceToHost, st));
  RDKV_HIP(hipStreamSynchronize(st));
  for (size_t i = 0; i < n; ++i)
    for (int side = 0; side < 2; ++side) {
      const double* a = h_acc.data() + (side * n + i) * 4;
      double* dst = (side == 0 ? eps_k : eps_v) + i * 3;
      for (int k = 0; k < 3; ++k) dst[k] = a[3] > 0.0 ? a[k] / a[3] : 0.0;
    }
  return RDKV_OK;
}

rdkv_status rdkv_allocate_info(const rdkv_config* cfg, const float* w_tok, const float* w_ch, uint8_t* bits_tok,
                               uint8_t* bits_ch, double* lambda_out, int32_t* iterations_out, void* stream) {
  rdkv_status s = check_config(cfg, true, false);
  if (s != RDKV_OK) return s;
  if (cfg->batch == 0) return RDKV_OK;       // (the buffers of an empty batch may be null)
  if (!w_tok || !bits_tok) return fail(RDKV_ERR_INVALID_ARG, "w_tok and bits_tok must not be null");
  const bool mixed = cfg->k_mode == RDKV_K_CHANNELWISE;
  if (mixed && (!w_ch || !bits_ch))
    return fail(RDKV_ERR_INVALID_ARG, "w_ch and bits_ch must not be null in channel-wise mode");
  hipStream_t st = static_cast<hipStream_t>(stream);
  Allocator al{cfg->alloc, cfg->free_, cfg->alloc_user};
  Temp tmp(al, st);
  Items it = make_items(cfg->seq_lens, cfg->batch, cfg->hkv);
  Tables tb;
  s = make_tables(cfg, it, true, tmp, st, &tb);
  if (s != RDKV_OK) return s;
  return allocate_impl(cfg, it, tb, w_tok, w_ch, bits_tok, bits_ch, lambda_out, iterations_out, tmp, st);
}

rdkv_status rdkv_allocate(const rdkv_config* cfg, const float* w_tok, const float* w_ch, uint8_t* bits_tok,
                          uint8_t* bits_ch, void* stream) {
  return rdkv_allocate_info(cfg, w_tok, w_ch, bits_tok, bits_ch, nullptr, nullptr, stream);
}

rdkv_status rdkv_pack(const rdkv_config* cfg, const void* K, const void* V, const uint8_t* bits_tok,
                      const uint8_t* bits_ch, void* stream, rdkv_cache** out) {
  if (out) *out = nullptr;
  rdkv_status s = check_config(cfg, false, false);
  if (s != RDKV_OK) return s;
  if (!out) return fail(RDKV_ERR_INVALID_ARG, "out is null");
  const bool mixed = cfg->k_mode == RDKV_K_CHANNELWISE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  Allocator al{cfg->alloc, cfg->free_, cfg->alloc_user};
  Items it = make_items(cfg->seq_lens, cfg->batch, cfg->hkv);
  if (it.total_tokens > 0 && (!K || !V || !bits_tok))
    return fail(RDKV_ERR_INVALID_ARG, "K, V and bits_tok must not be null");
  if (mixed && it.n_items > 0 && !bits_ch)
    return fail(RDKV_ERR_INVALID_ARG, "bits_ch must not be null in channel-wise mode");
  Temp tmp(al, st);
  Tables tb;
  s = make_tables(cfg, it, false, tmp, st, &tb);
  if (s != RDKV_OK) return s;
  return pack_impl(cfg, it, tb, K, V, bits_tok, bits_ch, nullptr, nullptr, tmp, st, out);
}

rdkv_status rdkv_compress(const rdkv_config* cfg, const void* K, const void* V, const void* Q_obs, void* stream,
                          rdkv_cache** out) {
  if (out) *out = nullptr;
  rdkv_status s = check_config(cfg, true, true);
  if (s != RDKV_OK) return s;
  if (!out) return fail(RDKV_ERR_INVALID_ARG, "out is null");
  const bool mixed = cfg->k_mode == RDKV_K_CHANNELWISE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  Allocator al{cfg->alloc, cfg->free_, cfg->alloc_user};
  Items it = make_items(cfg->seq_lens, cfg->batch, cfg->hkv);
  if (it.total_tokens > 0 && (!K || !V || !Q_obs)) return fail(RDKV_ERR_INVALID_ARG, "K, V and Q_obs must not be null");
  Temp tmp(al, st);
  const size_t nt = static_cast<size_t>(std::max<int64_t>(it.total_tokens, 1));
  const size_t ni = static_cast<size_t>(std::max<int64_t>(it.n_items, 1));
  const size_t nc = ni * kHeadDim;
  {
    const int R_pad = (cfg->hq / cfg->hkv * cfg->s_obs + 15) / 16 * 16;
    int64_t n_wblk = 0;
    for (int64_t i = 0; i < it.n_items; ++i) n_wblk += (it.T[i] + weights_block() - 1) / weights_block();
    tmp.reserve({48 * ni, nt * sizeof(float), nt, mixed ? nc * sizeof(float) : 0, mixed ? nc : 0,
                 weights_scratch_floats(n_wblk, it.n_items, it.total_tokens, R_pad, mixed) * sizeof(float),
                 mixed ? ni * sizeof(int32_t) : 0, mixed ? ni * sizeof(double) : 0,
                 static_cast<size_t>(std::max<int64_t>(it.n_blocks * 4, 1)) * sizeof(int32_t),
                 (ni * 4 + 1) * sizeof(int32_t), ni * 20 * sizeof(int64_t), ni * 2 * sizeof(double), ni * 2 * sizeof(int32_t),
                 it.max_T >= 16384 && it.n_items <= 512 ? allocate_multi_scratch_bytes(static_cast<int>(it.n_items)) : 0,
                 mixed && cfg->k_scale_per_channel ? nc * 2 * sizeof(uint32_t) : 0});
  }
  Tables tb;
  s = make_tables(cfg, it, true, tmp, st, &tb);
  if (s != RDKV_OK) return s;
  float* w = tmp.get<float>(nt);
  uint8_t* bits = tmp.get<uint8_t>(nt);
  float* w_ch = mixed ? tmp.get<float>(nc) : nullptr;
  uint8_t* bits_ch = mixed ? tmp.get<uint8_t>(nc) : nullptr;
  if (!w || !bits || (mixed && (!w_ch || !bits_ch))) return fail(RDKV_ERR_ALLOC, "device allocation failed");
  if (it.n_items == 0) return pack_impl(cfg, it, tb, K, V, bits, bits_ch, nullptr, nullptr, tmp, st, out);
  // the multiplier and the step count of every item's search stay with the cache (rdkv_cache_stats / export): the
  // pack stage copies them into the cache's block
  const int maps = mixed ? 2 : 1;
  double* lam = tmp.get<double>(maps * ni);
  int32_t* iters = tmp.get<int32_t>(maps * ni);
  if (!lam || !iters) return fail(RDKV_ERR_ALLOC, "device allocation failed");
  s = weights_impl(cfg, it, tb, K, Q_obs, w, w_ch, tmp, st);
  if (s != RDKV_OK) return s;
  s = allocate_impl(cfg, it, tb, w, w_ch, bits, bits_ch, lam, iters, tmp, st);
  if (s != RDKV_OK) return s;
  return pack_impl(cfg, it, tb, K, V, bits, bits_ch, lam, iters, tmp, st, out);
}

// A-priori bound on the packed arena from the budget alone (Sec. 3.2: sum of bit-widths <= floor(avg * units)).
// Token-wise: an item keeps at most B / b_min tokens (b_min = lowest stored bit-width of the tier set), and its rows
// cost 2 (16 b + 16) bytes each (no metadata at 16 bits), so at most 32 B + 32 B / b_min bytes, capped by all T rows
// at 16 bits; plus up to 63 padding rows per tier and the 256-byte alignment of its 16 segments.
// Channel-wise: V rows as above with the V share of the budget and one side only; a retained token's K row takes
// at most sum_c b_c / 8 <= 16 k_avg bytes of codes plus up to 24 bytes of segment padding, and a K tile of 64 tokens
// at most 32 bytes of metadata per quantized step (<= 35 steps).
static size_t cache_max_bytes(const rdkv_config* cfg) {
  const bool mixed = cfg->k_mode == RDKV_K_CHANNELWISE;
  int b_min = 16;
  for (int i = 0; i < cfg->n_tiers; ++i)
    if (cfg->tiers[i] > 0) b_min = std::min(b_min, cfg->tiers[i]);
  double total = 0.0;
  for (int s = 0; s < cfg->batch; ++s) {
    const double T = static_cast<double>(cfg->seq_lens[s]);
    const double a = static_cast<double>(cfg->budget_bits[s]);
    double item;
    if (!mixed) {
      const double B = std::min(std::floor(a * T), 16.0 * T);
      const double kept = std::min(B / b_min, T);
      item = std::min(32.0 * B + 32.0 * kept, 512.0 * T) + 63.0 * 2.0 * (256 + 144 + 80 + 48);
    } else {
      const double rk = static_cast<double>(cfg->kv_split_rk);
      const double Bv = std::min(std::floor(static_cast<double>(static_cast<float>(2.0 * (1.0 - rk) * a)) * T), 16.0 * T);
      const double kept = std::min(Bv / b_min, T);
      const double v = std::min(16.0 * Bv + 16.0 * kept, 256.0 * T) + 63.0 * (256 + 144 + 80 + 48);
      // K: codes <= 16 * (2 r_K a T) bytes over all kept tokens (k_avg n_kept = 2 r_K a T), at most 256 per token
      const double k_codes = std::min(16.0 * 2.0 * rk * a * T, 256.0 * kept) + 24.0 * kept;
      const double tiles = std::ceil(kept / 64.0) + 4.0;
      item = v + k_codes + tiles * 32.0 * 35.0 + 4.0 * 63.0 * 4.0 * kMaxKRowWords;
    }
    total += cfg->hkv * (item + 16.0 * kSegAlign);
  }
  return static_cast<size_t>(total) + kSegAlign;
}

// The same for everything else in the cache's block: kept positions (4 bytes each), the bit maps, the K row layouts,
// the chunk table and the first split workspace (at most two rounds of chunks and four per item, 80 bytes and
// g x 130 floats each), lambda and step counts, and the alignment of the parts.
static size_t cache_max_table_bytes(const rdkv_config* cfg) {
  const bool mixed = cfg->k_mode == RDKV_K_CHANNELWISE;
  const int g = cfg->hq / cfg->hkv;
  int b_min = 16;
  for (int i = 0; i < cfg->n_tiers; ++i)
    if (cfg->tiers[i] > 0) b_min = std::min(b_min, cfg->tiers[i]);
  double kept = 0.0, tokens = 0.0;
  for (int s = 0; s < cfg->batch; ++s) {
    const double T = static_cast<double>(cfg->seq_lens[s]);
    const double a = static_cast<double>(cfg->budget_bits[s]) * (mixed ? 2.0 * (1.0 - static_cast<double>(cfg->kv_split_rk)) : 1.0);
    kept += cfg->hkv * std::min(std::floor(a * T) / b_min, T);
    tokens += cfg->hkv * T;
  }
  const double items = static_cast<double>(cfg->batch) * cfg->hkv;
  const double chunks = 2.0 * 768.0 + 8.0 * items;
  return static_cast<size_t>(4.0 * kept + tokens + items * (kHeadDim + sizeof(ItemK) + 4 + 2 * 12) +
                             chunks * (sizeof(Chunk) + g * (kHeadDim + 2) * 4.0) + 16.0 * 256);
}

size_t rdkv_cache_max_bytes(const rdkv_config* cfg) {
  if (check_config(cfg, true, false) != RDKV_OK) return 0;
  return cache_max_bytes(cfg);
}

size_t rdkv_cache_max_table_bytes(const rdkv_config* cfg) {
  if (check_config(cfg, true, false) != RDKV_OK) return 0;
  return cache_max_table_bytes(cfg);
}

rdkv_status rdkv_decode_attn(const rdkv_cache* c, const void* q, float* out, float* lse, void* stream) {
  if (!c) return fail(RDKV_ERR_INVALID_ARG, "cache must not be null");
  if (c->n_items == 0) return RDKV_OK;       // nothing to compute (and q / out of an empty batch may be null)
  if (!q || !out) return fail(RDKV_ERR_INVALID_ARG, "q and out must not be null");
  hipStream_t st = static_cast<hipStream_t>(stream);
  rdkv_cache::Workspace w;
  const rdkv_status ws = workspace_for(c, st, &w);
  if (ws != RDKV_OK) return ws;
  const MergeArgs ma{w.part_acc, w.part_ml, w.arrive, out, lse, c->hq, c->hkv};
  // every chunk of the schedule is launched, the tail's included: chunks of tail rows that do not exist yet find
  // the current length in the cache's device word and contribute an empty partial
  const int n16 = static_cast<int>(c->sched16), nrest = static_cast<int>(c->schedq + c->n_tail_chunks);
  TimedScope ts(RDKV_TIME_DECODE_TIERED, st);
  if (c->k_mode == RDKV_K_CHANNELWISE) {
    RDKV_HIP(launch_decode_mixed(c->d_chunks, n16 + nrest, c->d_arena, c->d_items_sched ? c->d_items_sched : c->d_items_k,
                                 std::max(c->max_k_words, c->sched_k_words), std::max(c->max_k_steps, c->sched_k_steps),
                                 std::max(c->max_k_qsteps, c->sched_k_qsteps), static_cast<const uint16_t*>(q), ma,
                                 c->d_tail_state, c->k_per_unit,
                                 std::max(c->max_k_words, c->sched_k_words) <= 32 && c->hq / c->hkv <= 4 ? c->mixed_waves : 4,
                                 st));
    return RDKV_OK;
  }
  // the workgroups of both kernels announce themselves on the same counters: whichever finishes an item merges it
  RDKV_HIP(launch_decode_tiered_split(c->d_chunks, n16, c->d_arena, static_cast<const uint16_t*>(q), ma, st));
  bool multi = c->n_cont > 0;      // some workgroup goes through more than one tier of its item
  for (const rdkv_cache* child : c->absorbed) multi = multi || child->n_cont > 0;
  RDKV_HIP(launch_decode_tiles(c->d_chunks, n16, nrest, multi, c->d_arena, static_cast<const uint16_t*>(q), ma,
                               c->d_tail_state, st));
  return RDKV_OK;
}

// Rebuilds the decode schedule of a cache: the chunks of the cache itself and of every absorbed generation (all
// 16-bit chunks first, then the quantized ones), then the tail's chunks in (chunk index, item) order so that the
// live ones are a prefix.  Every item keeps its partial slots contiguous: own chunks, generation by generation,
// then the tail.  The decode kernels address everything relative to d_arena, so the offsets of the other
// allocations are pointer differences.  Synchronises the stream; on failure the cache is unchanged.
static rdkv_status rebuild_schedule(rdkv_cache* c, hipStream_t st) {
  Allocator al{c->alloc, c->free_, c->alloc_user};
  const int64_t n = c->n_items;
  const int npi = (c->tail_cap + kTailChunkRows - 1) / kTailChunkRows;     // tail chunks per item
  std::vector<const rdkv_cache*> gens{c};
  gens.insert(gens.end(), c->absorbed.begin(), c->absorbed.end());
  std::vector<int32_t> nb(n), nc(n);
  std::vector<std::vector<int32_t>> gen_off(gens.size(), std::vector<int32_t>(n));
  int64_t n_slots = 0, n_gen_chunks = 0;
  for (int64_t i = 0; i < n; ++i) {
    nb[i] = static_cast<int32_t>(n_slots);
    int32_t off = 0;
    for (size_t k = 0; k < gens.size(); ++k) {
      gen_off[k][i] = off;
      off += gens[k]->own_slot_count[i];
    }
    nc[i] = off + npi;
    n_slots += nc[i];
  }
  // table = [16-bit chunks of every generation | launched quantized chunks of every generation | tail chunks |
  //          continuation pieces of every generation]; a generation's own vector is [16-bit | launched | continuations]
  int64_t n_cont_total = 0;
  std::vector<int64_t> cont_off(gens.size());
  for (size_t k = 0; k < gens.size(); ++k) {
    n_gen_chunks += static_cast<int64_t>(gens[k]->chunks.size()) - gens[k]->n_cont;
    cont_off[k] = n_cont_total;
    n_cont_total += gens[k]->n_cont;
  }
  const int64_t cont_base = n_gen_chunks + n * npi;      // where the continuation pieces start in the new table
  std::vector<Chunk> table;
  table.reserve(static_cast<size_t>(cont_base + n_cont_total));
  std::vector<Chunk> own = c->chunks;   // this cache's chunks with their new slot numbers
  int64_t n16 = 0;
  auto moved = [&](size_t k, Chunk ch) {
    const rdkv_cache* gc = gens[k];
    const int64_t base = reinterpret_cast<intptr_t>(gc->d_arena) - reinterpret_cast<intptr_t>(c->d_arena);
    ch.reserved = static_cast<int32_t>(k * n + ch.item);
    ch.k_data += base;
    ch.k_meta += base;
    ch.v_data += base;
    ch.v_meta += base;
    if (ch.next >= 0) {   // an index into the generation's own vector -> into the new table
      const int64_t first_cont = static_cast<int64_t>(gc->chunks.size()) - gc->n_cont;
      ch.next = static_cast<int32_t>(cont_base + cont_off[k] + (ch.next - first_cont));
    }
    return ch;
  };
  for (int pass = 0; pass < 2; ++pass)
    for (size_t k = 0; k < gens.size(); ++k) {
      const rdkv_cache* gc = gens[k];
      const size_t launched = gc->chunks.size() - static_cast<size_t>(gc->n_cont);
      for (size_t j = 0; j < launched; ++j) {
        Chunk ch = gc->chunks[j];
        if ((ch.tier == 16) != (pass == 0)) continue;
        ch.slot = nb[ch.item] + gen_off[k][ch.item] + (ch.slot - gc->slot_begin[ch.item]);
        if (k == 0) own[j].slot = ch.slot;
        table.push_back(moved(k, ch));
        n16 += pass == 0;
      }
    }
  const int64_t tail_tiles = (c->tail_cap + kTile64 - 1) / kTile64, tile_bytes = kTile64 * kHeadDim * 2;
  const int64_t side = n * tail_tiles * tile_bytes;     // K tiles of all items, then V tiles
  const int64_t tail_base = reinterpret_cast<intptr_t>(c->d_tail) - reinterpret_cast<intptr_t>(c->d_arena);
  for (int j = 0; j < npi; ++j)
    for (int64_t i = 0; i < n; ++i) {
      Chunk ch;
      std::memset(&ch, 0, sizeof(ch));
      ch.k_data = tail_base + (i * tail_tiles + static_cast<int64_t>(j) * (kTailChunkRows / kTile64)) * tile_bytes;
      ch.v_data = ch.k_data + side;
      ch.rows = std::min<int32_t>(kTailChunkRows, c->tail_cap - j * kTailChunkRows);
      ch.tier = kTierTail;
      ch.item = static_cast<int32_t>(i);
      ch.slot = nb[i] + nc[i] - npi + j;
      ch.row0 = j * kTailChunkRows;
      ch.next = -1;
      table.push_back(ch);
    }
  for (size_t k = 0; k < gens.size(); ++k) {
    const rdkv_cache* gc = gens[k];
    for (size_t j = gc->chunks.size() - static_cast<size_t>(gc->n_cont); j < gc->chunks.size(); ++j)
      table.push_back(moved(k, gc->chunks[j]));
  }
  // launch order inside each kernel's range; the tail's chunks and the continuation pieces stay where they are
  order_chunks(table.begin(), table.begin() + n16, n);
  order_chunks(table.begin() + n16, table.begin() + n_gen_chunks, n);
  stamp_slots(table, nb, nc);
  stamp_slots(own, nb, nc);
  const int64_t n_table = static_cast<int64_t>(table.size());
  // channel-wise K: every (generation, item) has its own sorted-channel row layout
  const bool mixed = c->k_mode == RDKV_K_CHANNELWISE;
  std::vector<ItemK> items_sched;
  ItemK* d_items_sched = nullptr;
  int32_t kw = 0, ks = 0, kq = 0;
  if (mixed && gens.size() > 1) {
    for (const rdkv_cache* gc : gens) {
      items_sched.insert(items_sched.end(), gc->items_k.begin(), gc->items_k.end());
      kw = std::max(kw, gc->max_k_words);
      ks = std::max(ks, gc->max_k_steps);
      kq = std::max(kq, gc->max_k_qsteps);
    }
    d_items_sched = static_cast<ItemK*>(al.get(items_sched.size() * sizeof(ItemK)));
    if (!d_items_sched) return fail(RDKV_ERR_ALLOC, "device allocation failed");
  }
  Chunk* d_chunks = static_cast<Chunk*>(al.get(std::max<int64_t>(n_table, 1) * sizeof(Chunk)));
  if (!d_chunks) {
    al.put(d_items_sched);
    return fail(RDKV_ERR_ALLOC, "device allocation failed");
  }
  hipError_t e = hipSuccess;
  if (n_table > 0) e = upload(d_chunks, table.data(), table.size() * sizeof(Chunk), st);
  if (e == hipSuccess && d_items_sched)
    e = upload(d_items_sched, items_sched.data(), items_sched.size() * sizeof(ItemK), st);
  // the stream must be idle before the old tables and workspaces go: a decode step may still be reading them
  if (e == hipSuccess) e = hipStreamSynchronize(st);
  if (e != hipSuccess) {
    al.put(d_chunks); al.put(d_items_sched);
    return fail(RDKV_ERR_HIP, "rebuilding the decode schedule: %s", hipGetErrorString(e));
  }
  drop_workspaces(c);      // the slot count changed: workspaces are created again on first use
  c->n_slots = n_slots;
  {   // the first chunk table lives in the cache's block; rebuilt ones are allocations of their own
    const uint8_t* q = reinterpret_cast<const uint8_t*>(c->d_chunks);
    if (!(c->d_block && q >= c->d_block && q < c->d_block + c->block_bytes)) al.put(c->d_chunks);
  }
  al.put(c->d_items_sched);
  c->d_items_sched = d_items_sched;
  c->sched_k_words = kw;
  c->sched_k_steps = ks;
  c->sched_k_qsteps = kq;
  c->d_chunks = d_chunks;
  c->sched16 = n16;
  c->schedq = n_gen_chunks - n16;
  c->n_tail_chunks = n * npi;
  c->chunks.swap(own);
  c->slot_begin.swap(nb);
  c->slot_count.swap(nc);
  rdkv_cache::Workspace w;   // this stream's workspace right away: a decode under graph capture then allocates nothing
  (void)workspace_for(c, st, &w);   // (a failure here is reported by the decode call that needs the workspace)
  return RDKV_OK;
}

rdkv_status rdkv_cache_reserve_tail(rdkv_cache* c, int32_t max_new_tokens, void* stream) {
  if (!c) return fail(RDKV_ERR_INVALID_ARG, "cache is null");
  if (max_new_tokens <= 0) return fail(RDKV_ERR_INVALID_ARG, "max_new_tokens = %d must be positive", max_new_tokens);
  if (c->tail_cap != 0) return fail(RDKV_ERR_INVALID_ARG, "the tail of this cache is already reserved (%d tokens)", c->tail_cap);
  if (c->n_items == 0) { c->tail_cap = max_new_tokens; return RDKV_OK; }
  hipStream_t st = static_cast<hipStream_t>(stream);
  Allocator al{c->alloc, c->free_, c->alloc_user};
  const int64_t tail_tiles = (max_new_tokens + kTile64 - 1) / kTile64, tile_bytes = kTile64 * kHeadDim * 2;
  const int64_t side = c->n_items * tail_tiles * tile_bytes;     // K tiles of all items, then V tiles
  uint8_t* d_tail = static_cast<uint8_t*>(al.get(2 * side));
  if (!d_tail) return fail(RDKV_ERR_ALLOC, "device allocation failed");
  hipError_t e = hipMemsetAsync(d_tail, 0, 2 * side, st);   // rows not yet appended must read as zeros
  if (e != hipSuccess) {
    al.put(d_tail);
    return fail(RDKV_ERR_HIP, "rdkv_cache_reserve_tail: %s", hipGetErrorString(e));
  }
  c->d_tail = d_tail;
  c->tail_cap = max_new_tokens;
  c->tail_len = 0;
  const rdkv_status s = rebuild_schedule(c, st);
  if (s != RDKV_OK) {
    c->d_tail = nullptr;
    c->tail_cap = 0;
    al.put(d_tail);
  }
  return s;
}

rdkv_status rdkv_cache_append(rdkv_cache* c, const void* k_new, const void* v_new, void* stream) {
  if (!c || !k_new || !v_new) return fail(RDKV_ERR_INVALID_ARG, "cache, k_new and v_new must not be null");
  if (c->tail_cap == 0) return fail(RDKV_ERR_INVALID_ARG, "call rdkv_cache_reserve_tail before the first append");
  if (c->tail_len >= c->tail_cap)
    return fail(RDKV_ERR_INVALID_ARG, "the tail is full (%d tokens reserved)", c->tail_cap);
  if (c->n_items == 0) { c->tail_len += 1; return RDKV_OK; }
  RDKV_HIP(launch_append_rows(static_cast<const uint16_t*>(k_new), static_cast<const uint16_t*>(v_new), c->d_tail,
                              c->n_items, (c->tail_cap + kTile64 - 1) / kTile64, c->tail_cap, c->d_tail_state,
                              static_cast<hipStream_t>(stream)));
  c->tail_len += 1;
  return RDKV_OK;
}

int32_t rdkv_cache_tail_len(const rdkv_cache* c) { return c ? c->tail_len : 0; }

rdkv_status rdkv_cache_tail_len_sync(rdkv_cache* c, void* stream, int32_t* out) {
  if (!c) return fail(RDKV_ERR_INVALID_ARG, "cache is null");
  if (c->n_items > 0 && c->d_tail_state) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    int32_t n = 0;
    RDKV_HIP(hipMemcpyAsync(&n, c->d_tail_state, sizeof(int32_t), hipMemcpyDeviceToHost, st));
    RDKV_HIP(hipStreamSynchronize(st));
    c->tail_len = n;
  }
  if (out) *out = c->tail_len;
  return RDKV_OK;
}

rdkv_status rdkv_cache_rebudget_tail(rdkv_cache* c, const rdkv_config* cfg, const void* Q_obs, void* stream) {
  if (!c || !cfg || !Q_obs) return fail(RDKV_ERR_INVALID_ARG, "cache, cfg and Q_obs must not be null");
  if (cfg->k_mode != c->k_mode || (c->k_mode == RDKV_K_CHANNELWISE && (cfg->k_scale_per_channel != 0) != (c->k_per_unit != 0)) ||
      cfg->group_size != c->group_size)
    return fail(RDKV_ERR_INVALID_ARG, "cfg must name the cache's own format (k_mode %d, k_scale_per_channel %d, group_size %d)",
                c->k_mode, c->k_per_unit, c->group_size);
  {   // appends replayed from a captured graph advance only the device's count: take that one
    const rdkv_status s0 = rdkv_cache_tail_len_sync(c, stream, nullptr);
    if (s0 != RDKV_OK) return s0;
  }
  if (c->tail_len <= 0) return fail(RDKV_ERR_INVALID_ARG, "no appended tokens to compress");
  if (cfg->batch != c->batch || cfg->hq != c->hq || cfg->hkv != c->hkv || cfg->head_dim != c->d)
    return fail(RDKV_ERR_SHAPE, "cfg (batch %d, hq %d, hkv %d, d %d) does not match the cache (%d, %d, %d, %d)",
                cfg->batch, cfg->hq, cfg->hkv, cfg->head_dim, c->batch, c->hq, c->hkv, c->d);
  if (!cfg->seq_lens) return fail(RDKV_ERR_INVALID_ARG, "seq_lens is null");
  for (int s = 0; s < cfg->batch; ++s)
    if (cfg->seq_lens[s] != c->tail_len)
      return fail(RDKV_ERR_SHAPE, "seq_lens[%d] = %d: every sequence has %d appended tokens", s, cfg->seq_lens[s], c->tail_len);
  {   // every host-side check of the pass comes before the first launch
    const rdkv_status s0 = check_config(cfg, true, true);
    if (s0 != RDKV_OK) return s0;
  }
  hipStream_t st = static_cast<hipStream_t>(stream);
  Allocator al{cfg->alloc, cfg->free_, cfg->alloc_user};
  Temp tmp(al, st);
  const int32_t n_tail = c->tail_len;
  const size_t elems = static_cast<size_t>(c->n_items) * n_tail * kHeadDim;
  tmp.reserve({elems * sizeof(uint16_t), elems * sizeof(uint16_t)});
  uint16_t* k_rows = tmp.get<uint16_t>(elems);
  uint16_t* v_rows = tmp.get<uint16_t>(elems);
  if (!k_rows || !v_rows) return fail(RDKV_ERR_ALLOC, "device allocation failed");
  RDKV_HIP(launch_gather_tail_rows(c->d_tail, c->n_items, (c->tail_cap + kTile64 - 1) / kTile64, n_tail, k_rows, v_rows, st));
  rdkv_cache* child = nullptr;
  rdkv_status s = rdkv_compress(cfg, k_rows, v_rows, Q_obs, stream, &child);   // synchronises the stream
  if (s != RDKV_OK) return s;
  // The tail's tiles keep the rows just compressed: rows at or past tail_len are masked out of the softmax (their
  // values are finite, so a zero probability times a stale V row adds nothing), and later appends overwrite them.
  c->absorbed.push_back(child);
  s = rebuild_schedule(c, st);
  if (s != RDKV_OK) {
    c->absorbed.pop_back();
    rdkv_cache_free(child);
    return s;
  }
  c->tail_len = 0;
  const int32_t zeros[2] = {0, 0};
  RDKV_HIP(upload(c->d_tail_state, zeros, sizeof(zeros), st));
  return RDKV_OK;
}

int32_t rdkv_cache_generations(const rdkv_cache* c) { return c ? static_cast<int32_t>(c->absorbed.size()) : 0; }

const rdkv_cache* rdkv_cache_generation(const rdkv_cache* c, int32_t index) {
  if (!c || index < 0 || index >= static_cast<int32_t>(c->absorbed.size())) return nullptr;
  return c->absorbed[index];
}

size_t rdkv_decode_bf16_workspace_bytes(const int32_t* seq_lens, int32_t batch, int32_t hq, int32_t hkv,
                                        int32_t head_dim) {
  if (check_shape(batch, hq, hkv, head_dim, seq_lens) != RDKV_OK || batch == 0) return 0;
  int chunk_rows, max_splits;
  dense_plan(seq_lens, batch, hkv, hq / hkv, &chunk_rows, &max_splits);
  const int64_t slots = static_cast<int64_t>(std::min(batch, kDenseMaxSeqs)) * hkv * max_splits;
  return static_cast<size_t>(slots) * (hq / hkv) * (kHeadDim + 2) * sizeof(float);
}

rdkv_status rdkv_decode_attn_bf16(const void* K, const void* V, const int32_t* seq_lens, int32_t batch, int32_t hq,
                                  int32_t hkv, int32_t head_dim, const void* q, float* out, float* lse,
                                  void* workspace, size_t workspace_bytes, void* stream) {
  rdkv_status s = check_shape(batch, hq, hkv, head_dim, seq_lens);
  if (s != RDKV_OK) return s;
  if (batch == 0) return RDKV_OK;
  if (!K || !V || !q || !out || !workspace) return fail(RDKV_ERR_INVALID_ARG, "K, V, q, out, workspace must not be null");
  const size_t need = rdkv_decode_bf16_workspace_bytes(seq_lens, batch, hq, hkv, head_dim);
  if (workspace_bytes < need)
    return fail(RDKV_ERR_INVALID_ARG, "workspace of %zu bytes is smaller than the %zu required", workspace_bytes, need);
  const int g = hq / hkv;
  int chunk_rows, max_splits;
  dense_plan(seq_lens, batch, hkv, hq / hkv, &chunk_rows, &max_splits);
  const int64_t slots = static_cast<int64_t>(std::min(batch, kDenseMaxSeqs)) * hkv * max_splits;
  int64_t row_off = 0;
  for (int s0 = 0; s0 < batch; s0 += kDenseMaxSeqs) {
    const int ns = std::min(kDenseMaxSeqs, batch - s0);
    DenseArgs a;
    a.K = static_cast<const uint16_t*>(K);
    a.V = static_cast<const uint16_t*>(V);
    a.q = static_cast<const uint16_t*>(q);
    a.part_acc = static_cast<float*>(workspace);
    a.part_ml = a.part_acc + slots * g * kHeadDim;
    a.out = out;
    a.lse = lse;
    a.hq = hq; a.hkv = hkv; a.batch = batch; a.chunk_rows = chunk_rows; a.max_splits = max_splits; a.seq_base = s0;
    for (int i = 0; i < ns; ++i) {
      a.T[i] = seq_lens[s0 + i];
      a.row_off[i] = row_off;
      row_off += static_cast<int64_t>(seq_lens[s0 + i]) * hkv;
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    {
      TimedScope ts(RDKV_TIME_DECODE_BF16, st);
      RDKV_HIP(launch_decode_dense_split(a, g, ns, st));
    }
    RDKV_HIP(launch_decode_dense_merge(a, g, ns, st));
  }
  return RDKV_OK;
}

}  // extern "C"

// ---- the bf16 decode step for callers that cannot allocate ---------------------------------------------------------
// Its split partials live in a file-scope device array instead of a caller workspace.  In host code the array's name
// is only a stand-in for the symbol: the device address is looked up once per device and used from then on.
constexpr size_t kStaticScratchBytes = static_cast<size_t>(8) << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device (looked up on the first call on that device).
rdkv_status static_scratch(void** out) {
  int dev = -1;
  RDKV_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return fail(RDKV_ERR_UNSUPPORTED, "device index %d out of range", dev);
  std::lock_guard<std::mutex> lk(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    RDKV_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return fail(RDKV_ERR_HIP, "hipGetSymbolAddress returned a null address");
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return RDKV_OK;
}
}  // namespace

extern "C" {

size_t rdkv_decode_bf16_noalloc_max_bytes(void) { return kStaticScratchBytes; }

rdkv_status rdkv_decode_attn_bf16_noalloc(const void* K, const void* V, const int32_t* seq_lens, int32_t batch,
                                          int32_t hq, int32_t hkv, int32_t head_dim, const void* q, float* out,
                                          float* lse, void* stream) {
  rdkv_status s = check_shape(batch, hq, hkv, head_dim, seq_lens);
  if (s != RDKV_OK) return s;
  if (batch == 0) return RDKV_OK;
  const size_t need = rdkv_decode_bf16_workspace_bytes(seq_lens, batch, hq, hkv, head_dim);
  if (need > kStaticScratchBytes)
    return fail(RDKV_ERR_UNSUPPORTED,
                "this batch needs %zu bytes of split partials, more than the %zu bytes of the built-in scratch area; "
                "use rdkv_decode_attn_bf16 with a workspace",
                need, kStaticScratchBytes);
  void* ws = nullptr;
  s = static_scratch(&ws);
  if (s != RDKV_OK) return s;
  // every partial slot the merge reads is written by the split kernel of the same call: nothing to clear
  return rdkv_decode_attn_bf16(K, V, seq_lens, batch, hq, hkv, head_dim, q, out, lse, ws, kStaticScratchBytes, stream);
}

rdkv_status rdkv_cache_stats(const rdkv_cache* c, rdkv_stats* out) {
  if (!c || !out) return fail(RDKV_ERR_INVALID_ARG, "cache and out must not be null");
  std::memset(out, 0, sizeof(*out));
  out->n_items = c->n_items;
  int64_t kept = 0;
  for (int64_t i = 0; i < c->n_items; ++i)
    for (int ti = 0; ti < 4; ++ti) {
      const int bits = pack_tier_bits(ti);
      const int64_t cnt = c->counts[i * 4 + ti];
      out->rows[ti] += cnt;
      kept += cnt;
      (void)bits;
    }
  out->stored_bytes = c->stored_bytes;
  out->evicted = c->total_tokens - kept;
  out->arena_bytes = c->arena_bytes;
  out->index_bytes = c->index_bytes;
  out->n_chunks = static_cast<int64_t>(c->chunks.size()) - c->n_cont;   // launched work items (not their continuations)
  out->dense_bytes = c->total_tokens * kHeadDim * 2 * 2;
  out->lambda_min = out->lambda_max = std::nan("");
  if (c->d_lambda && c->d_iters && c->n_items > 0) {   // the token map's searches (Alg. 2); synchronous copies
    std::vector<double> lam(c->n_items);
    std::vector<int32_t> iters(c->n_items);
    RDKV_HIP(hipMemcpy(lam.data(), c->d_lambda, lam.size() * sizeof(double), hipMemcpyDeviceToHost));
    RDKV_HIP(hipMemcpy(iters.data(), c->d_iters, iters.size() * sizeof(int32_t), hipMemcpyDeviceToHost));
    out->alloc_info = 1;
    for (int64_t i = 0; i < c->n_items; ++i) {
      out->iterations_max = std::max<int64_t>(out->iterations_max, iters[i]);
      if (std::isnan(lam[i])) continue;
      out->lambda_min = std::isnan(out->lambda_min) ? lam[i] : std::min(out->lambda_min, lam[i]);
      out->lambda_max = std::isnan(out->lambda_max) ? lam[i] : std::max(out->lambda_max, lam[i]);
    }
  }
  for (const rdkv_cache* child : c->absorbed) {   // appended tokens compressed later count like the prompt's
    rdkv_stats cs;
    rdkv_cache_stats(child, &cs);
    for (int ti = 0; ti < 4; ++ti) out->rows[ti] += cs.rows[ti];
    out->evicted += cs.evicted;
    out->stored_bytes += cs.stored_bytes;
    out->arena_bytes += cs.arena_bytes;
    out->index_bytes += cs.index_bytes;
    out->n_chunks += cs.n_chunks;
    out->dense_bytes += cs.dense_bytes;
  }
  return RDKV_OK;
}

int32_t rdkv_k_row_words(const uint8_t* bits_ch) {
  if (!bits_ch) return -1;
  for (int ch = 0; ch < kHeadDim; ++ch)
    if (!valid_tier(bits_ch[ch])) return -1;
  return make_item_k(bits_ch).n_words_padded;
}

int32_t rdkv_k_row_words_max(void) { return kMaxKRowWords; }

size_t rdkv_cache_export_bytes(const rdkv_cache* c, int what) {
  if (!c) return 0;
  switch (what) {
    case RDKV_EXPORT_COUNTS: return c->counts.size() * sizeof(int32_t);
    case RDKV_EXPORT_TIER_IDX: return static_cast<size_t>(c->kept_total) * sizeof(int32_t);
    case RDKV_EXPORT_SEG_OFF: return c->seg_off.size() * sizeof(int64_t);
    case RDKV_EXPORT_ARENA: return static_cast<size_t>(c->arena_bytes);
    case RDKV_EXPORT_BITS_TOK: return static_cast<size_t>(c->total_tokens);
    case RDKV_EXPORT_BITS_CH: return c->d_bits_ch ? static_cast<size_t>(c->n_items) * kHeadDim : 0;
    case RDKV_EXPORT_LAMBDA:
      return c->d_lambda ? static_cast<size_t>(c->n_items) * (c->k_mode == RDKV_K_CHANNELWISE ? 2 : 1) * sizeof(double) : 0;
    case RDKV_EXPORT_ITERATIONS:
      return c->d_iters ? static_cast<size_t>(c->n_items) * (c->k_mode == RDKV_K_CHANNELWISE ? 2 : 1) * sizeof(int32_t) : 0;
    default: return 0;
  }
}

rdkv_status rdkv_cache_export(const rdkv_cache* c, int what, void* dst, size_t bytes) {
  if (!c || (!dst && bytes > 0)) return fail(RDKV_ERR_INVALID_ARG, "cache and dst must not be null");
  const size_t need = rdkv_cache_export_bytes(c, what);
  if (what < RDKV_EXPORT_COUNTS || what > RDKV_EXPORT_ITERATIONS) return fail(RDKV_ERR_INVALID_ARG, "unknown export %d", what);
  if (bytes < need) return fail(RDKV_ERR_INVALID_ARG, "destination of %zu bytes is smaller than the %zu required", bytes, need);
  if (need == 0) return RDKV_OK;
  switch (what) {
    case RDKV_EXPORT_COUNTS: std::memcpy(dst, c->counts.data(), need); break;
    case RDKV_EXPORT_SEG_OFF: std::memcpy(dst, c->seg_off.data(), need); break;
    case RDKV_EXPORT_TIER_IDX: RDKV_HIP(hipMemcpy(dst, c->d_tier_idx, need, hipMemcpyDeviceToHost)); break;
    case RDKV_EXPORT_ARENA: RDKV_HIP(hipMemcpy(dst, c->d_arena, need, hipMemcpyDeviceToHost)); break;
    case RDKV_EXPORT_BITS_TOK: RDKV_HIP(hipMemcpy(dst, c->d_bits_tok, need, hipMemcpyDeviceToHost)); break;
    case RDKV_EXPORT_BITS_CH: RDKV_HIP(hipMemcpy(dst, c->d_bits_ch, need, hipMemcpyDeviceToHost)); break;
    case RDKV_EXPORT_LAMBDA: RDKV_HIP(hipMemcpy(dst, c->d_lambda, need, hipMemcpyDeviceToHost)); break;
    case RDKV_EXPORT_ITERATIONS: RDKV_HIP(hipMemcpy(dst, c->d_iters, need, hipMemcpyDeviceToHost)); break;
  }
  return RDKV_OK;
}

void rdkv_cache_free(rdkv_cache* c) {
  if (!c) return;
  free_cache_buffers(c);
  delete c;
}

}  // extern "C"
