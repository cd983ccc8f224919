// Host side of the C ABI declared in include/ckv.h: argument checks,
// workspace carving, kernel launches.  No device memory is allocated here.
#include "../../include/ckv.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <climits>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "ckv_kernels.h"
#include "ckv_unit_kernel.h"

using namespace ckv;

constexpr int kSide = 2;   // streams of the context's own for deferred bookkeeping
constexpr int kBookGroup = 8;   // layers whose deferred bookkeeping goes out as one launch
constexpr size_t kLayerScanPad = 48 << 10;      // dynamic LDS of layer_scan_kernel: with its 32 KB of static LDS, two workgroups per 160 KB

// Scratch of ckv_probe_noalloc: device memory the library owns from the moment it is loaded, so that the
// call never needs a caller's workspace or an allocation.  In host code `scratch` is only a handle: the
// array's address on a device comes from hipGetSymbolAddress, once per device (scratch_setup), and that
// pointer is what kernels and fills get.  One array per GPU, shared by every context on it.
constexpr size_t kScratchBytes = (size_t)128 << 20;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];
constexpr int kMaxDevices = 64;

struct ckv_ctx {
  ckv_layout lay;
  ckv_lrfu_params par;
  ckv_buffers buf;
  Dev dev;
  int units = 0;
  int units_per_layer = 0;
  int next_layer = 0;
  int n_cu = 256;
  float* seedmi = nullptr;      // workspace of the prompt replay
  float* seedml = nullptr;
  float* seedrw = nullptr;
  int device = 0;               // the HIP device the context was created on
  size_t finish_lds = 0;
  // fused path (unit_kernel)
  int path_mode = 0;            // 0 auto, 1 separate kernels, 2 fused kernel, 3 / 4 fused with 4 / 2 wavefronts per unit,
                                // 5 fused with four book-keeping wavefronts beside four streaming ones
  struct Fused {                // one variant of the fused kernel
    bool ok = false;
    int waves = 0;              // wavefronts per workgroup (= per unit)
    int grid = 0;
    int lds_main = 0;           // bytes of the logits / values tile
    size_t lds = 0;             // dynamic LDS per workgroup
  } fused[2];                   // [0]: 4 wavefronts, 2 workgroups per CU; [1]: 2 wavefronts, 4 workgroups per CU
  std::vector<uint8_t> prompt_loaded;
  std::vector<int32_t> prompt_len;   // per layer: length of a prompt loaded whole and untouched since, else -1
  // Deferred bookkeeping of single-layer steps (CKV_DEFER_BOOKKEEPING): finish_kernel (late = 1) runs on
  // one of the `side` streams (layer l on side[l % kSide], so that the bookkeeping of consecutive layers, which
  // share nothing, can overlap), ordered by events against the caller's stream.  pending[l]: layer l's
  // bookkeeping has been queued there and nothing on the caller's side has waited for it yet.
  // The bookkeeping of up to kBookGroup consecutive layers goes out as one launch (a fork from the caller's
  // stream costs about as much as a small kernel, and more units per launch fill the chip better): after a
  // deferred step, layers [group_first, group_first + group_count) have been scanned on group_stream and wait
  // for theirs; the group goes out when it is full, with the last layer, and before anything else looks.
  hipStream_t side[kSide] = {};
  hipEvent_t ev_out = nullptr;
  std::vector<hipEvent_t> ev_book;
  std::vector<uint8_t> pending;
  bool any_pending = false;
  // Shared pools: budgets (or a prompt) have changed what units should own (dirty); once an eviction over all
  // layers has been issued since, the segments are dealt out again when the next step begins (due).
  bool dirty = false, due = false;
  int group_first = 0, group_count = 0, group_launches = 0;
  uint32_t group_flags = 0;
  hipStream_t group_stream = nullptr;
  std::string err;
  // scan timing
  bool profile = false;
  std::vector<hipEvent_t> ev;      // pairs
  size_t ev_used = 0;
  double scan_ms = 0.0;
  int scan_launches = 0;
};

namespace {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

int fail(ckv_ctx* c, int code, const std::string& msg) {
  if (c) c->err = msg;
  return code;
}

int hip_fail(ckv_ctx* c, hipError_t e, const char* what) {
  std::string m = std::string(what) + ": " + hipGetErrorString(e);
  return fail(c, CKV_EHIP, m);
}

#define CKV_HIP(ctx, call)                                   \
  do {                                                       \
    hipError_t e_ = (call);                                  \
    if (e_ != hipSuccess) return hip_fail((ctx), e_, #call); \
  } while (0)

bool layout_ok(const ckv_layout* l, std::string* why) {
  if (!l) { *why = "layout is NULL"; return false; }
  if (l->head_dim != kDim) { *why = "head_dim must be 128"; return false; }
  if (l->n_layers < 1 || l->n_layers > kMaxLayers) { *why = "n_layers must be in [1, 256]"; return false; }
  if (l->batch < 1) { *why = "batch must be >= 1"; return false; }
  if (l->n_kv_heads < 1 || l->n_kv_heads > kMaxKvHeads) { *why = "n_kv_heads must be in [1, 32]"; return false; }
  if (l->n_q_heads < l->n_kv_heads || l->n_q_heads % l->n_kv_heads != 0) { *why = "n_q_heads must be a multiple of n_kv_heads"; return false; }
  if (l->n_q_heads / l->n_kv_heads > kMaxGroup) { *why = "at most 8 query heads per KV head"; return false; }
  if (l->cap < kBlk || l->cap % kBlk != 0 || l->cap > kMaxChunks * kChunk) { *why = "cap must be a multiple of 32 in [32, 32768]"; return false; }
  if (l->out_dtype != CKV_F32 && l->out_dtype != CKV_BF16) { *why = "out_dtype must be CKV_F32 or CKV_BF16"; return false; }
  long long units = (long long)l->n_layers * l->batch * l->n_kv_heads;
  if (units * l->cap > (1ll << 40) || units > (1ll << 24)) { *why = "geometry too large"; return false; }
  const long long segs = (l->cap + kSeg - 1) / kSeg;
  if (l->headroom < 0 || l->headroom >= l->cap) { *why = "headroom must be in [0, cap)"; return false; }
  if (l->pool_slots <= 0 || l->pool_slots % kSeg != 0 || l->pool_slots > (1ll << 40)) { *why = "pool_slots must be a positive multiple of 256"; return false; }
  if (l->headroom == 0 && l->pool_slots < units * segs * kSeg) { *why = "pool_slots too small: with headroom 0 every unit owns ceil(cap / 256) segments"; return false; }
  return true;
}

bool params_ok(const ckv_layout* l, const ckv_lrfu_params* p, std::string* why) {
  if (!p) { *why = "params is NULL"; return false; }
  if (!(p->lambda >= 0.0f && p->lambda <= 1.0f)) { *why = "lambda must be in [0, 1]"; return false; }
  if (!(p->top_p > 0.0f)) { *why = "top_p must be > 0"; return false; }
  if (!(p->softmax_scale > 0.0f) || !std::isfinite(p->softmax_scale)) { *why = "softmax_scale must be positive"; return false; }
  if (p->reward_mode != CKV_REWARD_TOPP_HIT && p->reward_mode != CKV_REWARD_ATTN_WEIGHTED) { *why = "unknown reward_mode"; return false; }
  if (p->t0 < 0) { *why = "t0 must be >= 0"; return false; }
  if (p->budget_min < 1 || p->budget_min > p->budget_max || p->budget_max >= l->cap) { *why = "need 1 <= budget_min <= budget_max < cap"; return false; }
  return true;
}

// lambda^delta as float, flushed to zero below FLT_MIN; the table ends at its
// first zero entry (one entry for lambda = 1, capped at 2^20 + 1 entries).
std::vector<float> make_decay_table(float lambda) {
  std::vector<float> tab;
  tab.push_back(1.0f);
  const double lam = (double)lambda;
  if (lam == 1.0) return tab;
  for (int delta = 1; delta <= (1 << 20); ++delta) {
    float v = (float)std::pow(lam, (double)delta);
    if (v < FLT_MIN) v = 0.0f;
    tab.push_back(v);
    if (v == 0.0f) break;
  }
  return tab;
}

struct Carve {
  size_t n, budget, t_unit, nev, window, sc, stamp, tab, items, partial, ml, logits, btotal, order, layer_ts, arrive, msum, tbl, owned, spare, seedml, seedmi, seedrw, total;
};

Carve carve(const ckv_layout* l, size_t tab_len) {
  Carve c{};
  const size_t U = (size_t)l->n_layers * l->batch * l->n_kv_heads;
  const size_t G = (size_t)(l->n_q_heads / l->n_kv_heads);
  const size_t mc = (size_t)(l->cap + kChunk - 1) / kChunk;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
  c.n = take(U * 4);
  c.budget = take(U * 4);
  c.t_unit = take(U * 4);
  c.nev = take(U * 4);
  c.arrive = take(U * 4);
  c.window = take(U * 8);
  c.sc = take(SC_COUNT * 4);
  c.stamp = take(U * (mc + 1) * 4);
  c.tab = take(tab_len * 4);
  c.items = take(U * mc * 16);
  c.partial = take(U * (mc + 1) * G * kDim * 4);
  c.ml = take(U * (mc + 1) * G * 2 * 4);
  c.logits = take(U * G * (size_t)l->cap * 4);
  c.btotal = take((size_t)l->batch * 8);
  c.order = take(U * 4);
  c.layer_ts = take((size_t)l->n_layers * 8);
  c.msum = take(U * kMaxGroup * 2 * 4);
  c.tbl = take(U * mc * 4);
  c.owned = take(U * 4);
  c.spare = take((size_t)(l->pool_slots / kSeg) * 4);
  // prompt replay (ckv_seed_prompt), one layer at a time: softmax maximum and 1 / sum per query column of a
  // batch; and, for contexts whose decode workspace is too small to lend the replay room for several tiles of
  // queries, one tile's softmax partials per chunk and the weights (then rewards) of its up to 16 queries
  const size_t UL = (size_t)l->batch * l->n_kv_heads;
  c.seedmi = take((size_t)kSeedTiles * UL * kSeedCols * 2 * 4);
  c.seedml = take(UL * mc * kSeedCols * 2 * 4);
  c.seedrw = take(UL * (size_t)l->cap * kSeedCols * 4);
  c.total = off;
  return c;
}

int check_budgets(ckv_ctx* c, const ckv_layout* l, const ckv_lrfu_params* p, const int32_t* budgets) {
  if (!budgets) return fail(c, CKV_EINVAL, "budgets is NULL");
  const size_t U = (size_t)l->n_layers * l->batch * l->n_kv_heads;
  for (size_t u = 0; u < U; ++u)
    if (budgets[u] < p->budget_min || budgets[u] > p->budget_max)
      return fail(c, CKV_EINVAL, "a budget lies outside [budget_min, budget_max]");
  return CKV_OK;
}

// The variant of the fused kernel the current path mode selects (nullptr: none fits or separate kernels).
const ckv_ctx::Fused* fused_variant(const ckv_ctx* c) {
  if (c->path_mode == 1) return nullptr;
  const ckv_ctx::Fused* f = c->path_mode == 3 ? &c->fused[0] : c->path_mode == 4 ? &c->fused[1]
                            : c->fused[0].ok ? &c->fused[0] : &c->fused[1];
  return f->ok ? f : nullptr;
}

// A pair of timing events from the context's pool (ckv_profile_enable).
int profile_events(ckv_ctx* c, hipEvent_t* e0, hipEvent_t* e1) {
  if (c->ev_used + 2 > c->ev.size()) {
    for (int i = 0; i < 2; ++i) {
      hipEvent_t e;
      CKV_HIP(c, hipEventCreate(&e));
      c->ev.push_back(e);
    }
  }
  *e0 = c->ev[c->ev_used];
  *e1 = c->ev[c->ev_used + 1];
  c->ev_used += 2;
  return CKV_OK;
}

// Queue the bookkeeping of the layers scanned since the last group went out.
int flush_group(ckv_ctx* c) {
  if (c->group_count == 0) return CKV_OK;
  const int first = c->group_first, count = c->group_count;
  c->group_count = 0;
  const int upl = c->lay.batch * c->lay.n_kv_heads;
  CKV_HIP(c, hipEventRecord(c->ev_out, c->group_stream));
  hipStream_t side = c->side[c->group_launches++ % kSide];
  CKV_HIP(c, hipStreamWaitEvent(side, c->ev_out, 0));
  hipLaunchKernelGGL(finish_kernel, dim3((unsigned)(count * upl)), dim3(kThreads), c->finish_lds, side, c->dev, first * upl,
                     (void*)nullptr, c->group_flags, 0, INT_MAX, -1, 2, -2);
  CKV_HIP(c, hipGetLastError());
  CKV_HIP(c, hipEventRecord(c->ev_book[first], side));
  for (int l = first; l < first + count; ++l) c->pending[l] = 1 + first;     // whose event to wait for
  c->any_pending = true;
  return CKV_OK;
}

// Order `s` after the deferred bookkeeping still in flight on the side streams (all layers, or one).
int join_side(ckv_ctx* c, hipStream_t s, int layer = -1) {
  if (c->group_count && (layer < 0 || (layer >= c->group_first && layer < c->group_first + c->group_count)))
    if (int rc = flush_group(c)) return rc;
  if (!c->any_pending) return CKV_OK;
  bool left = false;
  for (int l = 0; l < c->lay.n_layers; ++l) {
    if (!c->pending[l]) continue;
    if (layer >= 0 && l != layer) {
      left = true;
      continue;
    }
    CKV_HIP(c, hipStreamWaitEvent(s, c->ev_book[c->pending[l] - 1], 0));
    c->pending[l] = 0;
  }
  c->any_pending = left;
  return CKV_OK;
}

// Deal the pool segments out again (shared pools only); units [x_begin, x_begin + x_count) get room for
// x_entries entries whatever their budgets say.
int launch_rebalance(ckv_ctx* c, hipStream_t s, int x_begin = 0, int x_count = 0, int x_entries = 0, const int32_t* x_len = nullptr) {
  if (c->lay.headroom == 0) return CKV_OK;
  hipLaunchKernelGGL(rebalance_kernel, dim3(1), dim3(kBalanceThreads), 0, s, c->dev, (int)c->lay.headroom, x_begin, x_count, x_entries, x_len);
  CKV_HIP(c, hipGetLastError());
  return CKV_OK;
}

// After an eviction that covered the last layer: the segments the shrunken units gave up can go to the others.
// Not yet, though: the slots behind a unit's entries hold the record of what it has just evicted, which a
// caller may still want to read, and with deferred bookkeeping the evictions have not even run.  The segments
// move when the next step begins.
int rebalance_after_eviction(ckv_ctx* c) {
  if (c->lay.headroom > 0 && c->dirty) c->due = true;
  return CKV_OK;
}

// Before a step begins: what a deferred eviction left to do.
int rebalance_if_due(ckv_ctx* c, hipStream_t s) {
  if (!c->due) return CKV_OK;
  if (int rc = join_side(c, s)) return rc;
  c->dirty = c->due = false;
  return launch_rebalance(c, s);
}

// (Re)build the fused kernel's schedule (units by descending budget) from the budgets in device memory.
int launch_schedule(ckv_ctx* c, hipStream_t s) {
  hipLaunchKernelGGL(schedule_kernel, dim3(1), dim3(1024), 0, s, c->dev);
  CKV_HIP(c, hipGetLastError());
  return CKV_OK;
}

int upload_budgets(ckv_ctx* c, const int32_t* budgets, hipStream_t s) {
  const ckv_layout& l = c->lay;
  std::vector<long long> tot(l.batch, 0);
  for (int i = 0; i < l.n_layers; ++i)
    for (int b = 0; b < l.batch; ++b)
      for (int h = 0; h < l.n_kv_heads; ++h) tot[b] += budgets[((size_t)i * l.batch + b) * l.n_kv_heads + h];
  CKV_HIP(c, hipMemcpyAsync(c->dev.budget, budgets, (size_t)c->units * 4, hipMemcpyHostToDevice, s));
  CKV_HIP(c, hipMemcpyAsync(c->dev.btotal, tot.data(), (size_t)l.batch * 8, hipMemcpyHostToDevice, s));
  if (int rc = launch_schedule(c, s)) return rc;
  CKV_HIP(c, hipStreamSynchronize(s));
  return CKV_OK;
}

int fill32(ckv_ctx* c, void* p, uint32_t v, size_t count, hipStream_t s) {
  if (count == 0) return CKV_OK;
  size_t blocks = (count + 255) / 256;
  if (blocks > 65536) blocks = 65536;
  hipLaunchKernelGGL(fill_u32_kernel, dim3((unsigned)blocks), dim3(256), 0, s, (uint32_t*)p, v, count);
  CKV_HIP(c, hipGetLastError());
  return CKV_OK;
}

// Address of the library's static scratch on each device, and whether its launch sequence number has been
// started (at 1: the array is zero when the library is loaded, and a stamp of 0 must never look current).
// The number is never restarted: partials that earlier calls left in the array carry earlier numbers.
std::mutex g_scratch_mutex;
unsigned char* g_scratch_ptr[kMaxDevices] = {};

int scratch_setup(int devid, hipStream_t s) {
  if (devid < 0 || devid >= kMaxDevices) return CKV_EINVAL;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[devid]) return CKV_OK;
  unsigned char* p = nullptr;
  if (hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return CKV_EHIP;
  hipLaunchKernelGGL(fill_u32_kernel, dim3(1), dim3(64), 0, s, reinterpret_cast<uint32_t*>(p) + SC_SEQ, 1u, (size_t)1);
  if (hipGetLastError() != hipSuccess || hipStreamSynchronize(s) != hipSuccess) return CKV_EHIP;
  g_scratch_ptr[devid] = p;
  return CKV_OK;
}

int layer_range(ckv_ctx* c, int32_t layer, int* begin, int* count) {
  if (layer == -1) {
    *begin = 0;
    *count = c->units;
  } else if (layer >= 0 && layer < c->lay.n_layers) {
    *begin = layer * c->units_per_layer;
    *count = c->units_per_layer;
  } else {
    return fail(c, CKV_EINVAL, "layer out of range");
  }
  return CKV_OK;
}

}  // namespace

extern "C" {

size_t ckv_workspace_bytes(const ckv_layout* layout, const ckv_lrfu_params* params) {
  std::string why;
  if (!layout_ok(layout, &why) || !params_ok(layout, params, &why)) return 0;
  return carve(layout, make_decay_table(params->lambda).size()).total;
}

int ckv_init(ckv_ctx** out, const ckv_layout* layout, const int32_t* budgets, const ckv_lrfu_params* params,
             const ckv_buffers* b, void* stream) {
  if (!out) return CKV_EINVAL;
  *out = nullptr;
  std::string why;
  if (!layout_ok(layout, &why) || !params_ok(layout, params, &why)) return CKV_EINVAL;
  if (!b || !b->k_pool || !b->v_pool || !b->crf || !b->tau || !b->pos || !b->flags || !b->workspace) return CKV_EINVAL;
  if (int rc = check_budgets(nullptr, layout, params, budgets)) return rc;
  std::vector<float> tab = make_decay_table(params->lambda);
  const Carve cv = carve(layout, tab.size());
  if (b->workspace_bytes < cv.total || ((uintptr_t)b->workspace % kAlign) != 0) return CKV_EWORKSPACE;
  if (((uintptr_t)b->k_pool | (uintptr_t)b->v_pool | (uintptr_t)b->crf | (uintptr_t)b->tau | (uintptr_t)b->pos) % 16 != 0)
    return CKV_EINVAL;

  ckv_ctx* c = new (std::nothrow) ckv_ctx();
  if (!c) return CKV_EINVAL;
  c->lay = *layout;
  c->par = *params;
  c->buf = *b;
  c->units_per_layer = layout->batch * layout->n_kv_heads;
  c->units = layout->n_layers * c->units_per_layer;
  c->prompt_loaded.assign(layout->n_layers, 0);
  c->prompt_len.assign(layout->n_layers, -1);
  hipStream_t s = (hipStream_t)stream;

  int devid = 0;
  hipError_t e = hipGetDevice(&devid);
  int max_lds = 65536;
  if (e == hipSuccess) {
    if (hipDeviceGetAttribute(&c->n_cu, hipDeviceAttributeMultiprocessorCount, devid) != hipSuccess) c->n_cu = 0;
    if (hipDeviceGetAttribute(&max_lds, hipDeviceAttributeMaxSharedMemoryPerBlock, devid) != hipSuccess) max_lds = 65536;
  }
  if (e != hipSuccess || c->n_cu <= 0) {
    delete c;
    return CKV_EHIP;
  }
  c->device = devid;
  if (int rc = scratch_setup(devid, s)) {        // the static scratch of ckv_probe_noalloc: its address on this device
    delete c;
    return rc;
  }
  c->finish_lds = (size_t)layout->cap * 4 + (size_t)((layout->cap + 31) / 32) * 4;
  if (c->finish_lds + 12288 > (size_t)max_lds) {   // static LDS of the kernels stays below 12 KB
    delete c;
    return CKV_EINVAL;
  }
  const void* lds_kernels[4] = {reinterpret_cast<const void*>(finish_kernel), reinterpret_cast<const void*>(evict_kernel),
                                reinterpret_cast<const void*>(probe_kernel), reinterpret_cast<const void*>(seed_hits_kernel)};
  if (hipFuncSetAttribute(reinterpret_cast<const void*>(seed_scan_kernel<false>), hipFuncAttributeMaxDynamicSharedMemorySize, kSeedTiles * 4096) != hipSuccess ||
      hipFuncSetAttribute(reinterpret_cast<const void*>(seed_scan_kernel<true>), hipFuncAttributeMaxDynamicSharedMemorySize, kSeedTiles * 4096) != hipSuccess) {
    delete c;
    return CKV_EHIP;
  }
  for (const void* fn : lds_kernels) {
    if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)c->finish_lds) != hipSuccess) {
      delete c;
      return CKV_EHIP;
    }
  }

  // fused kernel: 8 / W workgroups of W wavefronts per CU, each with its share of the CU's 160 KB of LDS
  for (int v = 0; v < 2; ++v) {
    ckv_ctx::Fused& f = c->fused[v];
    f.waves = v == 0 ? 4 : 2;
    const int wgs = 8 / f.waves;
    const int static_lds = v == 0 ? 11 * 1024 : 6 * 1024;      // upper bounds of unit_kernel<W>'s static LDS
    const int evm_bytes = ((layout->cap + 31) / 32) * 4;
    const int tbl_bytes = 2 * ((layout->cap + kSeg - 1) / kSeg) * 4;   // two rows of the segment table
    const int share = (160 * 1024 / wgs) & ~1023;
    const int per_wg = max_lds < share ? max_lds : share;
    const int main_bytes = (per_wg - static_lds - evm_bytes - tbl_bytes) & ~127;
    f.grid = wgs * c->n_cu;
    f.ok = main_bytes >= 4 * layout->cap;                       // every entry's value must fit
    f.lds_main = main_bytes;
    f.lds = (size_t)main_bytes + evm_bytes + tbl_bytes;
    const void* fn = v == 0 ? reinterpret_cast<const void*>(unit_kernel<4>) : reinterpret_cast<const void*>(unit_kernel<2>);
    if (f.ok && hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)f.lds) != hipSuccess) f.ok = false;
  }
  Dev& d = c->dev;
  d.L = layout->n_layers;
  d.Bz = layout->batch;
  d.Hq = layout->n_q_heads;
  d.Hkv = layout->n_kv_heads;
  d.G = layout->n_q_heads / layout->n_kv_heads;
  d.cap = layout->cap;
  d.units = c->units;
  d.unit0 = 0;
  d.by_order = 1;
  d.max_chunks = (layout->cap + kChunk - 1) / kChunk;
  d.slots = d.max_chunks + 1;
  d.out_bf16 = layout->out_dtype == CKV_BF16;
  d.scale_log2e = params->softmax_scale * 1.44269504088896340736f;
  d.top_p = params->top_p;
  d.reward_mode = params->reward_mode;
  d.bmin = params->budget_min;
  d.bmax = params->budget_max;
  d.tab_last = (int32_t)tab.size() - 1;
  d.K = (uint16_t*)b->k_pool;
  d.V = (uint16_t*)b->v_pool;
  d.crf = b->crf;
  d.tau = b->tau;
  d.pos = b->pos;
  d.flags = b->flags;
  uint8_t* ws = (uint8_t*)b->workspace;
  d.n = (int32_t*)(ws + cv.n);
  d.budget = (int32_t*)(ws + cv.budget);
  d.t_unit = (int32_t*)(ws + cv.t_unit);
  d.nev = (int32_t*)(ws + cv.nev);
  d.window = (u64*)(ws + cv.window);
  d.sc = (int32_t*)(ws + cv.sc);
  d.tab = (const float*)(ws + cv.tab);
  d.items = (int4*)(ws + cv.items);
  d.partial = (float*)(ws + cv.partial);
  d.ml = (float*)(ws + cv.ml);
  d.stamp = (int32_t*)(ws + cv.stamp);
  d.logits = (float*)(ws + cv.logits);
  d.btotal = (long long*)(ws + cv.btotal);
  d.order = (int32_t*)(ws + cv.order);
  d.layer_ts = (int32_t*)(ws + cv.layer_ts);
  d.arrive = (int32_t*)(ws + cv.arrive);
  d.msum = (float*)(ws + cv.msum);
  d.tbl = (int32_t*)(ws + cv.tbl);
  d.owned = (int32_t*)(ws + cv.owned);
  d.spare = (int32_t*)(ws + cv.spare);
  d.max_seg = (int32_t)((layout->cap + kSeg - 1) / kSeg);
  c->seedmi = (float*)(ws + cv.seedmi);
  c->seedml = (float*)(ws + cv.seedml);
  c->seedrw = (float*)(ws + cv.seedrw);

  auto bail = [&](int rc) {
    ckv_destroy(c);
    return rc;
  };
  c->pending.assign(layout->n_layers, 0);
  for (int i = 0; i < kSide; ++i)
    if (hipStreamCreateWithFlags(&c->side[i], hipStreamNonBlocking) != hipSuccess) return bail(CKV_EHIP);
  if (hipEventCreateWithFlags(&c->ev_out, hipEventDisableTiming) != hipSuccess) return bail(CKV_EHIP);
  for (int l = 0; l < layout->n_layers; ++l) {
    hipEvent_t e;
    if (hipEventCreateWithFlags(&e, hipEventDisableTiming) != hipSuccess) return bail(CKV_EHIP);
    c->ev_book.push_back(e);
  }
  const size_t S = (size_t)layout->pool_slots;
  int rc;
  if ((rc = fill32(c, d.K, 0u, S * kDim / 2, s))) return bail(rc);
  if ((rc = fill32(c, d.V, 0u, S * kDim / 2, s))) return bail(rc);
  if ((rc = fill32(c, d.crf, 0u, S, s))) return bail(rc);
  if ((rc = fill32(c, d.tau, 0u, S, s))) return bail(rc);
  if ((rc = fill32(c, d.pos, 0u, S, s))) return bail(rc);
  if ((rc = fill32(c, d.flags, 0u, S / 4, s))) return bail(rc);
  // per-unit state and scalars (everything up to the decay table)
  if ((rc = fill32(c, ws, 0u, cv.tab / 4, s))) return bail(rc);
  if ((rc = fill32(c, d.t_unit, (uint32_t)(params->t0 - 1), (size_t)c->units, s))) return bail(rc);
  if ((rc = fill32(c, d.sc + SC_T, (uint32_t)params->t0, 1, s))) return bail(rc);
  if ((rc = fill32(c, d.sc + SC_SEQ, 1u, 1, s))) return bail(rc);
  if ((rc = fill32(c, d.sc + SC_QUEUE, 0u, 1, s))) return bail(rc);
  if (hipMemcpyAsync((void*)d.tab, tab.data(), tab.size() * 4, hipMemcpyHostToDevice, s) != hipSuccess) return bail(CKV_EHIP);
  if ((rc = upload_budgets(c, budgets, s))) return bail(rc);
  {
    // Segment table.  headroom 0: every unit owns room for cap entries for good.  Otherwise a unit starts with
    // the segments that budget + headroom entries need, handed out in unit order (so a unit's segments are
    // contiguous to begin with); the rest of the pool is spare.
    const int mseg = d.max_seg;
    const long long pool_segs = layout->pool_slots / kSeg;
    std::vector<int32_t> tbl((size_t)c->units * mseg, 0), owned((size_t)c->units, 0), spare;
    long long next = 0;
    for (long long u = 0; u < c->units; ++u) {
      const int need = layout->headroom == 0 ? mseg : std::min<long long>(mseg, ((long long)budgets[u] + layout->headroom + kSeg - 1) / kSeg);
      if (next + need > pool_segs) return bail(fail(c, CKV_EINVAL, "pool_slots too small for these budgets: see ckv_pool_slots"));
      for (int j = 0; j < need; ++j) tbl[(size_t)u * mseg + j] = (int32_t)(next + j);
      owned[u] = need;
      next += need;
    }
    for (long long sg = pool_segs - 1; sg >= next; --sg) spare.push_back((int32_t)sg);     // popped from the end: lowest first
    const int32_t nspare = (int32_t)spare.size();
    if (hipMemcpyAsync(d.tbl, tbl.data(), tbl.size() * 4, hipMemcpyHostToDevice, s) != hipSuccess ||
        hipMemcpyAsync(d.owned, owned.data(), owned.size() * 4, hipMemcpyHostToDevice, s) != hipSuccess ||
        (nspare && hipMemcpyAsync(d.spare, spare.data(), spare.size() * 4, hipMemcpyHostToDevice, s) != hipSuccess) ||
        hipMemcpyAsync(d.sc + SC_SPARE, &nspare, 4, hipMemcpyHostToDevice, s) != hipSuccess ||
        hipStreamSynchronize(s) != hipSuccess)
      return bail(CKV_EHIP);
  }
  if (hipStreamSynchronize(s) != hipSuccess) return bail(CKV_EHIP);
  *out = c;
  return CKV_OK;
}

void ckv_destroy(ckv_ctx* c) {
  if (!c) return;
  for (int i = 0; i < kSide; ++i)
    if (c->side[i]) {
      (void)hipStreamSynchronize(c->side[i]);
      (void)hipStreamDestroy(c->side[i]);
    }
  if (c->ev_out) (void)hipEventDestroy(c->ev_out);
  for (hipEvent_t e : c->ev_book) (void)hipEventDestroy(e);
  for (hipEvent_t e : c->ev) (void)hipEventDestroy(e);
  delete c;
}

int ckv_load_cache(ckv_ctx* c, int32_t layer, const void* k, const void* v, int32_t P, const int32_t* lengths,
                   const float* crf0, const int32_t* tau0, const int32_t* pos0, void* stream) {
  if (!c) return CKV_EINVAL;
  if (layer < 0 || layer >= c->lay.n_layers) return fail(c, CKV_EINVAL, "layer out of range");
  if (!k || !v) return fail(c, CKV_EINVAL, "k or v is NULL");
  if (P <= 0 || P >= c->lay.cap) return fail(c, CKV_EINVAL, "need 0 < P < cap");
  if (c->next_layer != 0) return fail(c, CKV_ESTATE, "a per-layer step is in progress");
  if (c->prompt_loaded[layer]) return fail(c, CKV_ESTATE, "layer already holds entries");
  c->prompt_loaded[layer] = 1;
  c->prompt_len[layer] = (!lengths && !pos0) ? P : -1;
  if (int rc = join_side(c, (hipStream_t)stream)) return rc;
  if (c->lay.headroom > 0) {
    // shared pools: the layer's units get room for what is loaded (and an append behind it) from the spare list,
    // and whatever earlier layers no longer need goes back to it first; an eviction gives the surplus back
    c->due = false;
    c->dirty = true;
    if (int rc = launch_rebalance(c, (hipStream_t)stream, layer * c->units_per_layer, c->units_per_layer, (int)P + c->lay.headroom, lengths)) return rc;
  }
  dim3 grid((unsigned)((P + kBlk - 1) / kBlk), (unsigned)c->units_per_layer);
  hipLaunchKernelGGL(load_cache_kernel, grid, dim3(kThreads), 0, (hipStream_t)stream, c->dev,
                     layer * c->units_per_layer, (const uint16_t*)k, (const uint16_t*)v, (int)P, lengths, crf0, tau0,
                     pos0);
  CKV_HIP(c, hipGetLastError());
  return CKV_OK;
}

int ckv_load_prompt(ckv_ctx* c, int32_t layer, const void* k, const void* v, int32_t P, const float* crf0,
                    const int32_t* tau0, void* stream) {
  if (!c) return CKV_EINVAL;
  if (P > c->par.t0) return fail(c, CKV_EINVAL, "need P <= t0");
  return ckv_load_cache(c, layer, k, v, P, nullptr, crf0, tau0, nullptr, stream);
}

int ckv_decode_step(ckv_ctx* c, int32_t layer, const void* q, const void* k_new, const void* v_new, void* out,
                    uint32_t flags, void* stream) {
  if (!c) return CKV_EINVAL;
  if (!q || !k_new || !v_new || !out) return fail(c, CKV_EINVAL, "q, k_new, v_new or out is NULL");
  if (flags & ~(CKV_FUSE_EVICT | CKV_ATTENTION_ONLY | CKV_DEFER_BOOKKEEPING)) return fail(c, CKV_EINVAL, "unknown flag bits");
  if ((flags & CKV_DEFER_BOOKKEEPING) && (layer == -1 || (flags & CKV_ATTENTION_ONLY)))
    return fail(c, CKV_EINVAL, "CKV_DEFER_BOOKKEEPING is for single-layer steps with bookkeeping");
  if ((flags & CKV_ATTENTION_ONLY) && (flags & CKV_FUSE_EVICT))
    return fail(c, CKV_EINVAL, "CKV_ATTENTION_ONLY excludes CKV_FUSE_EVICT");
  int begin, count;
  if (int rc = layer_range(c, layer, &begin, &count)) return rc;
  if (layer == -1) {
    if (c->next_layer != 0) return fail(c, CKV_ESTATE, "a per-layer step is in progress");
  } else {
    if (layer != c->next_layer) return fail(c, CKV_ESTATE, "layers must be stepped in order");
  }
  const int advance = (layer == -1 || layer == c->lay.n_layers - 1) ? 1 : 0;
  c->next_layer = advance ? 0 : layer + 1;
  for (int l = (layer == -1 ? 0 : layer); l < (layer == -1 ? c->lay.n_layers : layer + 1); ++l) {
    c->prompt_loaded[l] = 1;
    c->prompt_len[l] = -1;
  }
  hipStream_t s = (hipStream_t)stream;

  // The fused kernel takes whole units: all layers at once, or one layer that has at least a unit per
  // workgroup.  Such a layer it also finishes sooner than a scan with deferred bookkeeping would (Llama-8B
  // shape, 512 units per layer: 74 against 78 us), so there the flag is not followed.
  const ckv_ctx::Fused* fv = fused_variant(c);
  if (fv && (c->path_mode == 0 || layer >= 0) && count < fv->grid) fv = nullptr;   // fewer units than workgroups: split the units instead
  const bool fused = fv != nullptr;
  if (fused) flags &= ~CKV_DEFER_BOOKKEEPING;
  if (layer <= 0)
    if (int rc = rebalance_if_due(c, s)) return rc;
  if (int rc = join_side(c, s, layer)) return rc;
  if (flags & CKV_DEFER_BOOKKEEPING) {
    // One kernel on the caller's stream: it appends, attends and writes the output; the bookkeeping (which also
    // records the append) follows on a side stream, a group of layers at a time.
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (c->profile) {
      if (int rc = profile_events(c, &e0, &e1)) return rc;
      CKV_HIP(c, hipEventRecord(e0, s));
    }
    // At most two of its workgroups fit on a compute unit (the unused dynamic LDS sees to that): the kernel's
    // registers would allow three, and the dispatcher then crowds some compute units while others idle
    // (2.43 against 2.11 ms per step of 48 layers of 128 units; one per compute unit: 2.22).
    hipLaunchKernelGGL((layer_scan_kernel<4, 1>), dim3((unsigned)count, (unsigned)((c->dev.max_chunks + 3) / 4)), dim3(256), kLayerScanPad, s,
                       c->dev, begin, (const uint16_t*)q, (const uint16_t*)k_new, (const uint16_t*)v_new, out, (int)layer);
    CKV_HIP(c, hipGetLastError());
    if (c->profile) CKV_HIP(c, hipEventRecord(e1, s));
    if (advance) {
      hipLaunchKernelGGL(advance_kernel, dim3(1), dim3(64), 0, s, c->dev);
      CKV_HIP(c, hipGetLastError());
    }
    const uint32_t kflags = flags & CKV_FUSE_EVICT;
    if (c->group_count && (c->group_flags != kflags || c->group_stream != s || c->group_first + c->group_count != layer))
      if (int rc = flush_group(c)) return rc;
    if (c->group_count == 0) {
      c->group_first = layer;
      c->group_flags = kflags;
      c->group_stream = s;
    }
    c->group_count += 1;
    if (advance && (flags & CKV_FUSE_EVICT))
      if (int rc = rebalance_after_eviction(c)) return rc;
    if (c->group_count == kBookGroup || advance) return flush_group(c);
    return CKV_OK;
  }
  // unit_kernel<W> appends by itself; the separate kernels get the new entries and their work list from prep_kernel
  if (!fused) {
    hipLaunchKernelGGL(prep_kernel, dim3((unsigned)((count + kPrepUnits - 1) / kPrepUnits)), dim3(kPrepThreads), 0, s, c->dev, begin, count,
                       (const uint16_t*)k_new, (const uint16_t*)v_new, 1, INT_MAX, (const uint16_t*)q);
    CKV_HIP(c, hipGetLastError());
  }

  hipEvent_t e0 = nullptr, e1 = nullptr;
  if (c->profile) {
    if (int rc = profile_events(c, &e0, &e1)) return rc;
    CKV_HIP(c, hipEventRecord(e0, s));
  }
  if (fused) {
    // The kernel takes its units from the schedule (all layers: by descending budget) or, for a single layer, in
    // the layer's own order starting at its first unit, whose rows come first in q, k_new, v_new and out.
    Dev dv = c->dev;
    dv.units = count;
    dv.unit0 = layer >= 0 ? begin : 0;
    dv.by_order = layer >= 0 ? 0 : 1;
    const uint16_t* qb = (const uint16_t*)q;
    const uint16_t* vb = (const uint16_t*)v_new;
    const uint16_t* kb = (const uint16_t*)k_new;
    void* ob = out;
    if (fv->waves == 4)
      hipLaunchKernelGGL(unit_kernel<4>, dim3((unsigned)fv->grid), dim3(256), fv->lds, s, dv, qb, ob, flags, advance, fv->lds_main, vb, kb);
    else
      hipLaunchKernelGGL(unit_kernel<2>, dim3((unsigned)fv->grid), dim3(128), fv->lds, s, dv, qb, ob, flags, advance, fv->lds_main, vb, kb);
    CKV_HIP(c, hipGetLastError());
    if (c->profile) CKV_HIP(c, hipEventRecord(e1, s));
    if (advance && (flags & CKV_FUSE_EVICT)) return rebalance_after_eviction(c);
    return CKV_OK;
  }
  const long long max_items = (long long)count * c->dev.max_chunks;
  long long blocks = 2ll * c->n_cu;
  if (blocks > (max_items + 3) / 4) blocks = (max_items + 3) / 4;
  const uint32_t kflags = flags & CKV_FUSE_EVICT;
  // when nothing but the output is due on the caller's stream, the scan merges its own partials and ends the step
  const bool scan_merges = (flags & CKV_ATTENTION_ONLY) != 0;
  if (scan_merges)
    hipLaunchKernelGGL(scan_kernel<true>, dim3((unsigned)blocks), dim3(kThreads), 0, s, c->dev, begin, (const uint16_t*)q, out,
                       advance, -1);
  else
    hipLaunchKernelGGL(scan_kernel<false>, dim3((unsigned)blocks), dim3(kThreads), 0, s, c->dev, begin, (const uint16_t*)q,
                       (void*)nullptr, 0, -1);
  CKV_HIP(c, hipGetLastError());
  if (c->profile) CKV_HIP(c, hipEventRecord(e1, s));
  if (flags & CKV_ATTENTION_ONLY) return CKV_OK;

  hipLaunchKernelGGL(finish_kernel, dim3((unsigned)count), dim3(kThreads), c->finish_lds, s, c->dev, begin, out,
                     kflags, advance, INT_MAX, -1, 0, 0);
  CKV_HIP(c, hipGetLastError());
  if (advance && kflags) return rebalance_after_eviction(c);
  return CKV_OK;
}

int ckv_seed_prompt(ckv_ctx* c, int32_t layer, const void* q_obs, int32_t W, void* stream) {
  if (!c) return CKV_EINVAL;
  if (layer < 0 || layer >= c->lay.n_layers) return fail(c, CKV_EINVAL, "layer out of range");
  if (!q_obs) return fail(c, CKV_EINVAL, "q_obs is NULL");
  if (c->next_layer != 0) return fail(c, CKV_ESTATE, "a per-layer step is in progress");
  const int P = c->prompt_len[layer];
  if (P < 0) return fail(c, CKV_ESTATE, "needs a prompt loaded whole (ckv_load_prompt) and not touched since");
  if (W < 1 || W > P) return fail(c, CKV_EINVAL, "need 1 <= W <= P");
  hipStream_t s = (hipStream_t)stream;
  if (int rc = join_side(c, s)) return rc;
  const int begin = layer * c->units_per_layer, count = c->units_per_layer;
  const dim3 sgrid((unsigned)std::min((P + kThreads - 1) / kThreads, 64), (unsigned)count);
  hipLaunchKernelGGL(seed_state_kernel, sgrid, dim3(kThreads), 0, s, c->dev, begin, P, (int)W, 0, 0);
  CKV_HIP(c, hipGetLastError());
  // A tile of 16 query columns holds the G heads of Q queries.  Per batch of tiles: a pass over the keys for the
  // softmax partials of all its queries, their maxima and sums, a second pass for the mean weights, the
  // rewards (top-p rule), the score recurrence.  The batch's weights and softmax partials live in the decode
  // paths' logits and partials (idle here, rewritten by the next scan before anything reads them) when those
  // hold at least two tiles, else in the replay's own one-tile buffers.
  const int G = c->dev.G, Q = kSeedCols / G;
  const size_t UL = (size_t)count, cap = (size_t)c->lay.cap, mc = (size_t)c->dev.max_chunks;
  const size_t tile_rw = (size_t)Q * UL * cap * 4, tile_ml = UL * mc * kSeedCols * 2 * 4;
  const size_t big_lg = (size_t)c->units * cap * (size_t)G * 4, big_ml = (size_t)c->units * (size_t)c->dev.slots * (size_t)G * kDim * 4;
  const int fit = (int)std::min<size_t>({big_lg / tile_rw, big_ml / tile_ml, (size_t)kSeedTiles});
  float *ml = c->seedml, *rw = c->seedrw, *mi = c->seedmi;
  int tiles = 1;
  if (fit >= 2) {
    tiles = fit;
    rw = c->dev.logits;
    ml = c->dev.partial;
  }
  const bool topp = c->par.reward_mode == CKV_REWARD_TOPP_HIT;
  for (int j0 = 0; j0 < W; j0 += tiles * Q) {
    const int nq = std::min(tiles * Q, (int)W - j0), nt = (nq + Q - 1) / Q;
    const int n_last = P - W + j0 + nq;                    // entries the batch's last query sees
    const int chunks = (n_last + kChunk - 1) / kChunk;
    const dim3 sgrid2((unsigned)((chunks + kThreads / 64 - 1) / (kThreads / 64)), (unsigned)count);
    hipLaunchKernelGGL(seed_scan_kernel<false>, sgrid2, dim3(kThreads), (size_t)nt * 4096, s, c->dev, begin, (const uint16_t*)q_obs, j0,
                       nq, Q, P, (int)W, ml, (const float*)mi, rw);
    CKV_HIP(c, hipGetLastError());
    hipLaunchKernelGGL(seed_stats_kernel, dim3((unsigned)count), dim3(kSeedTiles * kSeedCols), 0, s, c->dev, j0, nq, Q, P, (int)W,
                       (const float*)ml, mi);
    CKV_HIP(c, hipGetLastError());
    hipLaunchKernelGGL(seed_scan_kernel<true>, sgrid2, dim3(kThreads), (size_t)nt * 4096, s, c->dev, begin, (const uint16_t*)q_obs, j0,
                       nq, Q, P, (int)W, ml, (const float*)mi, rw);
    CKV_HIP(c, hipGetLastError());
    if (topp) {
      hipLaunchKernelGGL(seed_hits_kernel, dim3((unsigned)nq, (unsigned)count), dim3(kSeedThreads), c->finish_lds, s, c->dev, begin, j0, P,
                         (int)W, rw);
      CKV_HIP(c, hipGetLastError());
    }
    hipLaunchKernelGGL(seed_crf_kernel, dim3((unsigned)((P + 4 * kThreads - 1) / (4 * kThreads)), (unsigned)count), dim3(kThreads), 0, s,
                       c->dev, begin, j0, nq, P, (int)W, (const float*)rw);
    CKV_HIP(c, hipGetLastError());
  }
  hipLaunchKernelGGL(seed_state_kernel, dim3(1, (unsigned)count), dim3(kThreads), 0, s, c->dev, begin, P, (int)W, 1, c->par.t0 - 1);
  CKV_HIP(c, hipGetLastError());
  return CKV_OK;
}

int ckv_evict(ckv_ctx* c, int32_t layer, void* stream) {
  if (!c) return CKV_EINVAL;
  int begin, count;
  if (int rc = layer_range(c, layer, &begin, &count)) return rc;
  for (int l = (layer == -1 ? 0 : layer); l < (layer == -1 ? c->lay.n_layers : layer + 1); ++l) c->prompt_len[l] = -1;
  if (int rc = join_side(c, (hipStream_t)stream)) return rc;
  hipLaunchKernelGGL(evict_kernel, dim3((unsigned)count), dim3(kThreads), c->finish_lds, (hipStream_t)stream, c->dev, begin, -1);
  CKV_HIP(c, hipGetLastError());
  if (layer == -1 || layer == c->lay.n_layers - 1) return rebalance_after_eviction(c);
  return CKV_OK;
}

int ckv_evict_window(ckv_ctx* c, int32_t layer, int32_t n_sink, void* stream) {
  if (!c) return CKV_EINVAL;
  if (n_sink < 0) return fail(c, CKV_EINVAL, "n_sink is negative");
  int begin, count;
  if (int rc = layer_range(c, layer, &begin, &count)) return rc;
  for (int l = (layer == -1 ? 0 : layer); l < (layer == -1 ? c->lay.n_layers : layer + 1); ++l) c->prompt_len[l] = -1;
  if (int rc = join_side(c, (hipStream_t)stream)) return rc;
  hipLaunchKernelGGL(evict_kernel, dim3((unsigned)count), dim3(kThreads), c->finish_lds, (hipStream_t)stream, c->dev, begin,
                     (int)n_sink);
  CKV_HIP(c, hipGetLastError());
  if (layer == -1 || layer == c->lay.n_layers - 1) return rebalance_after_eviction(c);
  return CKV_OK;
}

int ckv_rebudget(ckv_ctx* c, void* stream) {
  if (!c) return CKV_EINVAL;
  if (c->next_layer != 0) return fail(c, CKV_ESTATE, "a per-layer step is in progress");
  if (int rc = join_side(c, (hipStream_t)stream)) return rc;
  hipLaunchKernelGGL(rebudget_kernel, dim3((unsigned)c->lay.batch), dim3(kThreads), 0, (hipStream_t)stream, c->dev);
  CKV_HIP(c, hipGetLastError());
  c->dirty = true;             // shared pools: the segments follow once the shrunken units have evicted
  return launch_schedule(c, (hipStream_t)stream);
}

int ckv_rebalance(ckv_ctx* c, void* stream) {
  if (!c) return CKV_EINVAL;
  if (c->next_layer != 0) return fail(c, CKV_ESTATE, "a per-layer step is in progress");
  if (int rc = join_side(c, (hipStream_t)stream)) return rc;
  c->due = false;
  return launch_rebalance(c, (hipStream_t)stream);
}

int64_t ckv_pool_slots(const ckv_layout* l, const int32_t* budgets, int32_t prompt_len) {
  if (!l || !budgets || l->n_layers < 1 || l->batch < 1 || l->n_kv_heads < 1 || l->cap < kBlk || prompt_len < 0) return 0;
  const long long units = (long long)l->n_layers * l->batch * l->n_kv_heads, mseg = (l->cap + kSeg - 1) / kSeg;
  if (l->headroom <= 0) return units * mseg * kSeg;
  long long total = 0;
  for (long long u = 0; u < units; ++u) total += (long long)budgets[u] + l->headroom;
  // whatever Alg. 2 makes of the budgets, rounding to segments wastes less than one segment per unit
  long long segs = (total + kSeg - 1) / kSeg + units;
  if (prompt_len > 0) segs += (long long)l->batch * l->n_kv_heads * std::min<long long>(mseg, ((long long)prompt_len + l->headroom + kSeg - 1) / kSeg);
  return std::min(segs, units * mseg) * kSeg;
}

int ckv_probe(ckv_ctx* c, int32_t layer, const void* q_probe, uint8_t* classes, void* stream) {
  if (!c) return CKV_EINVAL;
  if (!q_probe || !classes) return fail(c, CKV_EINVAL, "q_probe or classes is NULL");
  if (layer < 0 || layer >= c->lay.n_layers) return fail(c, CKV_EINVAL, "layer out of range");
  if (c->next_layer != 0) return fail(c, CKV_ESTATE, "a per-layer step is in progress");
  const int begin = layer * c->units_per_layer, count = c->units_per_layer;
  hipStream_t s = (hipStream_t)stream;
  if (int rc = join_side(c, s)) return rc;
  hipLaunchKernelGGL(prep_kernel, dim3((unsigned)((count + kPrepUnits - 1) / kPrepUnits)), dim3(kPrepThreads), 0, s, c->dev, begin, count,
                     (const uint16_t*)nullptr, (const uint16_t*)nullptr, 0, INT_MAX, (const uint16_t*)nullptr);
  CKV_HIP(c, hipGetLastError());
  const long long max_items = (long long)count * c->dev.max_chunks;
  long long blocks = 2ll * c->n_cu;
  if (blocks > (max_items + 3) / 4) blocks = (max_items + 3) / 4;
  hipLaunchKernelGGL(scan_kernel<false>, dim3((unsigned)blocks), dim3(kThreads), 0, s, c->dev, begin, (const uint16_t*)q_probe,
                     (void*)nullptr, 0, -1);
  CKV_HIP(c, hipGetLastError());
  hipLaunchKernelGGL(probe_kernel, dim3((unsigned)count), dim3(kThreads), c->finish_lds, s, c->dev, begin, classes);
  CKV_HIP(c, hipGetLastError());
  return CKV_OK;
}

int ckv_probe_noalloc(ckv_ctx* c, int32_t layer, const void* q_probe, uint8_t* classes, void* stream) {
  if (!c) return CKV_EINVAL;
  if (!q_probe || !classes) return fail(c, CKV_EINVAL, "q_probe or classes is NULL");
  if (layer < 0 || layer >= c->lay.n_layers) return fail(c, CKV_EINVAL, "layer out of range");
  if (c->next_layer != 0) return fail(c, CKV_ESTATE, "a per-layer step is in progress");
  int devid = -1;
  if (hipGetDevice(&devid) != hipSuccess) return fail(c, CKV_EHIP, "hipGetDevice failed");
  if (devid != c->device) return fail(c, CKV_ESTATE, "the context's device is not the current one");
  unsigned char* base = g_scratch_ptr[devid];     // set by ckv_init on this device
  if (!base) return fail(c, CKV_ESTATE, "the library's scratch was not set up on this device");
  const int begin = layer * c->units_per_layer, count = c->units_per_layer;
  // the layer's scan scratch, carved from the static array instead of the context's workspace
  const size_t U = (size_t)count, G = (size_t)c->dev.G, mc = (size_t)c->dev.max_chunks, slots = mc + 1;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
  const size_t o_sc = take(SC_COUNT * 4), o_items = take(U * mc * 16), o_stamp = take(U * slots * 4),
               o_ml = take(U * slots * G * 2 * 4), o_partial = take(U * slots * G * kDim * 4),
               o_logits = take(U * G * (size_t)c->dev.cap * 4);
  if (off > kScratchBytes)
    return fail(c, CKV_EWORKSPACE, "one layer's scan scratch (" + std::to_string(off >> 20) + " MiB) exceeds the library's static scratch of " +
                                       std::to_string(kScratchBytes >> 20) + " MiB: use ckv_probe");
  // the layer's units as units 0 .. count-1 of a context of their own: caches and lengths from the real context,
  // work list, partials, logits and step counters from the scratch
  Dev ds = c->dev;
  ds.units = count;
  ds.tbl += (size_t)begin * c->dev.max_seg;      // the rows name pool segments: the pools stay where they are
  ds.owned += begin;
  ds.n += begin;
  ds.budget += begin;
  ds.t_unit += begin;
  ds.nev += begin;
  ds.window += begin;
  ds.sc = reinterpret_cast<int32_t*>(base + o_sc);
  ds.items = reinterpret_cast<int4*>(base + o_items);
  ds.stamp = reinterpret_cast<int32_t*>(base + o_stamp);
  ds.ml = reinterpret_cast<float*>(base + o_ml);
  ds.partial = reinterpret_cast<float*>(base + o_partial);
  ds.logits = reinterpret_cast<float*>(base + o_logits);
  hipStream_t s = (hipStream_t)stream;
  if (int rc = join_side(c, s)) return rc;
  // counters that must start at zero (a fill kernel, not a memset: the call may be captured in a graph); the
  // launch sequence number before them keeps counting
  hipLaunchKernelGGL(fill_u32_kernel, dim3(1), dim3(64), 0, s, reinterpret_cast<uint32_t*>(ds.sc) + SC_DONE, 0u, (size_t)(SC_CLAIM + 2 - SC_DONE));
  CKV_HIP(c, hipGetLastError());
  hipLaunchKernelGGL(prep_kernel, dim3((unsigned)((count + kPrepUnits - 1) / kPrepUnits)), dim3(kPrepThreads), 0, s, ds, 0, count,
                     (const uint16_t*)nullptr, (const uint16_t*)nullptr, 0, INT_MAX, (const uint16_t*)nullptr);
  CKV_HIP(c, hipGetLastError());
  const long long max_items = (long long)count * ds.max_chunks;
  long long blocks = 2ll * c->n_cu;
  if (blocks > (max_items + 3) / 4) blocks = (max_items + 3) / 4;
  hipLaunchKernelGGL(scan_kernel<false>, dim3((unsigned)blocks), dim3(kThreads), 0, s, ds, 0, (const uint16_t*)q_probe,
                     (void*)nullptr, 0, -1);
  CKV_HIP(c, hipGetLastError());
  hipLaunchKernelGGL(probe_kernel, dim3((unsigned)count), dim3(kThreads), c->finish_lds, s, ds, 0, classes);
  CKV_HIP(c, hipGetLastError());
  return CKV_OK;
}

int ckv_get_budgets(ckv_ctx* c, int32_t* budgets) {
  if (!c || !budgets) return CKV_EINVAL;
  if (int rc = flush_group(c)) return rc;
  CKV_HIP(c, hipDeviceSynchronize());
  CKV_HIP(c, hipMemcpy(budgets, c->dev.budget, (size_t)c->units * 4, hipMemcpyDeviceToHost));
  return CKV_OK;
}

int ckv_get_lengths(ckv_ctx* c, int32_t* lengths) {
  if (!c || !lengths) return CKV_EINVAL;
  if (int rc = flush_group(c)) return rc;
  CKV_HIP(c, hipDeviceSynchronize());
  CKV_HIP(c, hipMemcpy(lengths, c->dev.n, (size_t)c->units * 4, hipMemcpyDeviceToHost));
  return CKV_OK;
}

int ckv_get_segments(ckv_ctx* c, int32_t* owned, int32_t* rows, int32_t* spare, int32_t* n_spare) {
  if (!c || !n_spare) return CKV_EINVAL;
  if (int rc = flush_group(c)) return rc;
  CKV_HIP(c, hipDeviceSynchronize());
  CKV_HIP(c, hipMemcpy(n_spare, c->dev.sc + SC_SPARE, 4, hipMemcpyDeviceToHost));
  if (*n_spare < 0 || *n_spare > c->lay.pool_slots / kSeg) return fail(c, CKV_ESTATE, "corrupt spare list");
  if (owned) CKV_HIP(c, hipMemcpy(owned, c->dev.owned, (size_t)c->units * 4, hipMemcpyDeviceToHost));
  if (rows) CKV_HIP(c, hipMemcpy(rows, c->dev.tbl, (size_t)c->units * c->dev.max_seg * 4, hipMemcpyDeviceToHost));
  if (spare && *n_spare > 0) CKV_HIP(c, hipMemcpy(spare, c->dev.spare, (size_t)*n_spare * 4, hipMemcpyDeviceToHost));
  return CKV_OK;
}

int ckv_set_budgets(ckv_ctx* c, const int32_t* budgets) {
  if (!c) return CKV_EINVAL;
  if (int rc = check_budgets(c, &c->lay, &c->par, budgets)) return rc;
  if (int rc = flush_group(c)) return rc;
  CKV_HIP(c, hipDeviceSynchronize());
  c->dirty = true;
  return upload_budgets(c, budgets, nullptr);
}

int ckv_get_time(ckv_ctx* c, int32_t* t) {
  if (!c || !t) return CKV_EINVAL;
  if (int rc = flush_group(c)) return rc;
  CKV_HIP(c, hipDeviceSynchronize());
  CKV_HIP(c, hipMemcpy(t, c->dev.sc + SC_T, 4, hipMemcpyDeviceToHost));
  return CKV_OK;
}

int ckv_set_time(ckv_ctx* c, int32_t t) {
  if (!c || t < 0) return CKV_EINVAL;
  if (c->next_layer != 0) return fail(c, CKV_ESTATE, "a per-layer step is in progress");
  CKV_HIP(c, hipDeviceSynchronize());
  int32_t zero = 0;
  CKV_HIP(c, hipMemcpy(c->dev.sc + SC_T, &t, 4, hipMemcpyHostToDevice));
  CKV_HIP(c, hipMemcpy(c->dev.sc + SC_WINDOW_STEPS, &zero, 4, hipMemcpyHostToDevice));
  if (int rc = fill32(c, c->dev.window, 0u, (size_t)c->units * 2, nullptr)) return rc;
  CKV_HIP(c, hipDeviceSynchronize());
  return CKV_OK;
}

int ckv_status(ckv_ctx* c) {
  if (!c) return CKV_EINVAL;
  CKV_HIP(c, hipDeviceSynchronize());
  int32_t st = 0, zero = 0;
  CKV_HIP(c, hipMemcpy(&st, c->dev.sc + SC_STATUS, 4, hipMemcpyDeviceToHost));
  if (st) {
    CKV_HIP(c, hipMemcpy(c->dev.sc + SC_STATUS, &zero, 4, hipMemcpyHostToDevice));
    if (st & 2) return fail(c, CKV_EHIP, "a wait between wavefronts of the fused kernel did not end: the last steps' results are invalid");
    if (st & 4) return fail(c, CKV_ECAPACITY, "the spare list ran short when the pool segments were dealt out: some units own less than budget + headroom needs");
    return fail(c, CKV_ECAPACITY, "an append found its unit full");
  }
  return CKV_OK;
}

// The unit's row of the segment table and the number of segments it owns (the device is idle).
static int read_row(ckv_ctx* c, size_t u, std::vector<int32_t>* row, int32_t* own) {
  row->resize((size_t)c->dev.max_seg);
  CKV_HIP(c, hipMemcpy(row->data(), c->dev.tbl + u * c->dev.max_seg, row->size() * 4, hipMemcpyDeviceToHost));
  CKV_HIP(c, hipMemcpy(own, c->dev.owned + u, 4, hipMemcpyDeviceToHost));
  if (*own < 0 || *own > c->dev.max_seg) return fail(c, CKV_ESTATE, "corrupt segment table");
  return CKV_OK;
}

int ckv_export_unit(ckv_ctx* c, int32_t layer, int32_t seq, int32_t head, int32_t* n_out, int32_t* nev_out,
                    int32_t* budget_out, uint16_t* K, uint16_t* V, float* crf, int32_t* tau, int32_t* pos,
                    uint8_t* flags) {
  if (!c) return CKV_EINVAL;
  if (layer < 0 || layer >= c->lay.n_layers || seq < 0 || seq >= c->lay.batch || head < 0 || head >= c->lay.n_kv_heads)
    return fail(c, CKV_EINVAL, "unit index out of range");
  const size_t u = ((size_t)layer * c->lay.batch + seq) * c->lay.n_kv_heads + head;
  const size_t cap = (size_t)c->lay.cap;
  if (int rc = flush_group(c)) return rc;
  CKV_HIP(c, hipDeviceSynchronize());
  // the unit's slots, segment by segment (what it does not own stays zero on the host side)
  std::vector<int32_t> row;
  int32_t own = 0;
  if (int rc = read_row(c, u, &row, &own)) return rc;
  auto fetch = [&](void* host, const void* pool, size_t elem_bytes) -> int {      // per-slot array
    std::memset(host, 0, cap * elem_bytes);
    for (int j = 0; j < own; ++j) {
      const size_t cnt = std::min<size_t>(kSeg, cap - (size_t)j * kSeg);
      CKV_HIP(c, hipMemcpy((char*)host + (size_t)j * kSeg * elem_bytes, (const char*)pool + (size_t)row[j] * kSeg * elem_bytes,
                           cnt * elem_bytes, hipMemcpyDeviceToHost));
    }
    return CKV_OK;
  };
  int32_t n = 0, nev = 0, bud = 0;
  CKV_HIP(c, hipMemcpy(&n, c->dev.n + u, 4, hipMemcpyDeviceToHost));
  CKV_HIP(c, hipMemcpy(&nev, c->dev.nev + u, 4, hipMemcpyDeviceToHost));
  CKV_HIP(c, hipMemcpy(&bud, c->dev.budget + u, 4, hipMemcpyDeviceToHost));
  if (n_out) *n_out = n;
  if (nev_out) *nev_out = nev;
  if (budget_out) *budget_out = bud;
  std::vector<uint16_t> tmp;
  for (int which = 0; which < 2; ++which) {
    uint16_t* dst = which == 0 ? K : V;
    if (!dst) continue;
    tmp.resize(kSegElems);
    std::memset(dst, 0, cap * kDim * 2);
    for (int j = 0; j < own; ++j) {
      CKV_HIP(c, hipMemcpy(tmp.data(), (which == 0 ? c->dev.K : c->dev.V) + (size_t)row[j] * kSegElems, (size_t)kSegElems * 2, hipMemcpyDeviceToHost));
      for (int rr = 0; rr < kSeg && (size_t)j * kSeg + rr < cap; ++rr)
        for (int col = 0; col < kDim; ++col)
          dst[((size_t)j * kSeg + rr) * kDim + col] = tmp[which == 0 ? k_offset(rr, col) : v_offset(rr, col)];
    }
  }
  if (crf) if (int rc = fetch(crf, c->dev.crf, 4)) return rc;
  if (tau) if (int rc = fetch(tau, c->dev.tau, 4)) return rc;
  if (pos) if (int rc = fetch(pos, c->dev.pos, 4)) return rc;
  if (flags) {
    if (int rc = fetch(flags, c->dev.flags, 1)) return rc;
    // the hit mark is not stored: in the top-p mode an entry was hit in the unit's last step iff its tau is that step
    int32_t tu = 0;
    CKV_HIP(c, hipMemcpy(&tu, c->dev.t_unit + u, 4, hipMemcpyDeviceToHost));
    if (c->dev.reward_mode == 0 && tu >= c->par.t0 && n > 0) {
      std::vector<int32_t> th(cap);
      if (int rc = fetch(th.data(), c->dev.tau, 4)) return rc;
      for (int i = 0; i < n; ++i)
        if (th[i] == tu) flags[i] |= CKV_FLAG_HIT;
    }
  }
  return CKV_OK;
}

int ckv_import_unit(ckv_ctx* c, int32_t layer, int32_t seq, int32_t head, int32_t n, const uint16_t* K,
                    const uint16_t* V, const float* crf, const int32_t* tau, const int32_t* pos, int32_t t_unit) {
  if (!c) return CKV_EINVAL;
  if (layer < 0 || layer >= c->lay.n_layers || seq < 0 || seq >= c->lay.batch || head < 0 || head >= c->lay.n_kv_heads)
    return fail(c, CKV_EINVAL, "unit index out of range");
  if (n < 0 || n >= c->lay.cap) return fail(c, CKV_EINVAL, "need 0 <= n < cap");
  if (n > 0 && (!K || !V || !crf || !tau || !pos)) return fail(c, CKV_EINVAL, "NULL state array");
  const size_t u = ((size_t)layer * c->lay.batch + seq) * c->lay.n_kv_heads + head;
  if (int rc = flush_group(c)) return rc;
  CKV_HIP(c, hipDeviceSynchronize());
  std::vector<int32_t> row;
  int32_t own = 0;
  if (int rc = read_row(c, u, &row, &own)) return rc;
  if (n >= std::min<long long>(c->lay.cap, (long long)own * kSeg)) return fail(c, CKV_ECAPACITY, "the unit's segments do not hold n + 1 entries");
  const int nseg = (n + kSeg - 1) / kSeg;
  std::vector<uint16_t> tmp((size_t)kSegElems);
  for (int which = 0; which < 2 && n > 0; ++which) {
    const uint16_t* src = which == 0 ? K : V;
    for (int j = 0; j < nseg; ++j) {
      std::fill(tmp.begin(), tmp.end(), (uint16_t)0);
      for (int rr = 0; rr < kSeg && j * kSeg + rr < n; ++rr)
        for (int col = 0; col < kDim; ++col)
          tmp[which == 0 ? k_offset(rr, col) : v_offset(rr, col)] = src[((size_t)j * kSeg + rr) * kDim + col];
      const size_t used = (size_t)((std::min(n - j * kSeg, kSeg) + kBlk - 1) / kBlk) * kBlkElems;      // whole blocks
      CKV_HIP(c, hipMemcpy((which == 0 ? c->dev.K : c->dev.V) + (size_t)row[j] * kSegElems, tmp.data(), used * 2, hipMemcpyHostToDevice));
    }
  }
  if (n > 0) {
    std::vector<uint8_t> zf(kSeg, 0);
    for (int j = 0; j < nseg; ++j) {
      const size_t cnt = (size_t)std::min(n - j * kSeg, kSeg), s0 = (size_t)row[j] * kSeg, h0 = (size_t)j * kSeg;
      CKV_HIP(c, hipMemcpy(c->dev.crf + s0, crf + h0, cnt * 4, hipMemcpyHostToDevice));
      CKV_HIP(c, hipMemcpy(c->dev.tau + s0, tau + h0, cnt * 4, hipMemcpyHostToDevice));
      CKV_HIP(c, hipMemcpy(c->dev.pos + s0, pos + h0, cnt * 4, hipMemcpyHostToDevice));
      CKV_HIP(c, hipMemcpy(c->dev.flags + s0, zf.data(), cnt, hipMemcpyHostToDevice));
    }
  }
  int32_t zero = 0;
  CKV_HIP(c, hipMemcpy(c->dev.n + u, &n, 4, hipMemcpyHostToDevice));
  CKV_HIP(c, hipMemcpy(c->dev.nev + u, &zero, 4, hipMemcpyHostToDevice));
  CKV_HIP(c, hipMemcpy(c->dev.t_unit + u, &t_unit, 4, hipMemcpyHostToDevice));
  c->prompt_loaded[layer] = 1;
  c->prompt_len[layer] = -1;
  return CKV_OK;
}

int ckv_profile_enable(ckv_ctx* c, int32_t on) {
  if (!c) return CKV_EINVAL;
  if (int rc = flush_group(c)) return rc;
  CKV_HIP(c, hipDeviceSynchronize());
  c->profile = on != 0;
  c->ev_used = 0;
  c->scan_ms = 0.0;
  c->scan_launches = 0;
  return CKV_OK;
}

int ckv_profile_read(ckv_ctx* c, double* scan_ms, int32_t* launches) {
  if (!c) return CKV_EINVAL;
  CKV_HIP(c, hipDeviceSynchronize());
  for (size_t i = 0; i + 1 < c->ev_used; i += 2) {
    float ms = 0.f;
    CKV_HIP(c, hipEventElapsedTime(&ms, c->ev[i], c->ev[i + 1]));
    c->scan_ms += ms;
    c->scan_launches += 1;
  }
  c->ev_used = 0;
  if (scan_ms) *scan_ms = c->scan_ms;
  if (launches) *launches = c->scan_launches;
  return CKV_OK;
}

int ckv_bandwidth_probe(const void* src, void* dst, size_t bytes, void* sink, void* stream) {
  if (!src || !sink || bytes < (1u << 20) || ((uintptr_t)src % 16) != 0 || ((uintptr_t)dst % 16) != 0) return CKV_EINVAL;
  int devid = 0, n_cu = 0;
  if (hipGetDevice(&devid) != hipSuccess ||
      hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, devid) != hipSuccess || n_cu <= 0)
    return CKV_EHIP;
  const size_t n_vec = bytes / 16;
  if (dst)
    hipLaunchKernelGGL(probe_copy_kernel, dim3((unsigned)(n_cu * 32)), dim3(kThreads), 0, (hipStream_t)stream,
                       (const u32x4*)src, (u32x4*)dst, n_vec);
  else
    hipLaunchKernelGGL(probe_read_kernel, dim3((unsigned)n_cu), dim3(kThreads), 0, (hipStream_t)stream,
                       (const u32x4*)src, n_vec, (uint32_t*)sink);
  return hipGetLastError() == hipSuccess ? CKV_OK : CKV_EHIP;
}

int ckv_set_path(ckv_ctx* c, int32_t mode) {
  if (!c || mode < 0 || mode > 4) return CKV_EINVAL;
  const bool any = c->fused[0].ok || c->fused[1].ok;
  if ((mode == 2 && !any) || (mode == 3 && !c->fused[0].ok) || (mode == 4 && !c->fused[1].ok))
    return fail(c, CKV_EINVAL, "cap too large for the fused kernel's LDS");
  c->path_mode = mode;
  return CKV_OK;
}

int ckv_path_info(ckv_ctx* c, int32_t* fused_waves, int32_t* lds_main_bytes) {
  if (!c) return CKV_EINVAL;
  const ckv_ctx::Fused* f = fused_variant(c);
  if (f && c->path_mode == 0 && c->units < f->grid) f = nullptr;
  if (fused_waves) *fused_waves = f ? f->waves : 0;
  if (lds_main_bytes) *lds_main_bytes = f ? f->lds_main : 0;
  return CKV_OK;
}

int ckv_join(ckv_ctx* c, void* stream) {
  if (!c) return CKV_EINVAL;
  return join_side(c, (hipStream_t)stream);
}

const char* ckv_strerror(int code) {
  switch (code) {
    case CKV_OK: return "ok";
    case CKV_EINVAL: return "invalid argument";
    case CKV_ECAPACITY: return "unit full at append";
    case CKV_ESTATE: return "call not valid in this state";
    case CKV_EHIP: return "HIP runtime error";
    case CKV_EWORKSPACE: return "workspace too small or misaligned";
    default: return "unknown error";
  }
}

const char* ckv_last_error(const ckv_ctx* c) { return c ? c->err.c_str() : ""; }


}  // extern "C"
