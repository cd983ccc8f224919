// Device code of the Crystal-KV decode path for gfx950 (64-lane wavefronts,
// v_mfma_f32_16x16x32_bf16).  One decode step runs as one of
//
//   unit_kernel<W> (ckv_unit_kernel.h)  everything in one persistent kernel, a workgroup per unit at a time
//   layer_scan_kernel + finish_kernel   one layer: append, attention and output in one kernel on the caller's
//                  stream, the bookkeeping (finish_kernel, late = 2) afterwards on a stream of the context's
//   prep_kernel, scan_kernel, finish_kernel   the separate path:
//     prep_kernel    append (k_new, v_new) into the tiled cache, build the list
//                    of scan work items (unit, chunk of 256 entries)
//     scan_kernel    the HBM-bound pass: stream K and V once, QK^T and PV on the
//                    matrix cores, online softmax per work item; leaves the
//                    scaled logits and one partial (max, sum, acc) per item;
//                    on request also merges the partials -> out and ends the step
//     finish_kernel  one workgroup per unit: merge partials -> out, mean
//                    attention weight per entry, top-p hit mask, CRF update,
//                    aggregated CRF, and (optionally) eviction + compaction
//
// and beside the step:
//
//   load_cache_kernel, seed_state_kernel   fill a layer's caches
//   seed_scan_kernel, seed_stats_kernel, seed_hits_kernel, seed_crf_kernel   scores of a loaded prompt from its last queries
//   evict_kernel     eviction + compaction on its own (Alg. 1 Step 4, or the sink + recent window policy)
//   probe_kernel     answer-probe classes
//   rebudget_kernel  Alg. 2 with integer apportionment, one workgroup/sequence
//   rebalance_kernel pool segments between units after budgets have changed
//   schedule_kernel  (ckv_unit_kernel.h) the fused kernel's order of units
//
// All floating-point code is compiled with -ffp-contract=off: the CRF update
// and Alg. 2 must round exactly as their definitions say.
#pragma once
#include <hip/hip_runtime.h>
#include <float.h>
#include <math.h>
#include <stdint.h>

#include "ckv_layout.h"

namespace ckv {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned long long u64;

// SC_CLAIM is a 64-bit counter (8-byte aligned): low word = work items published, high word = their blocks
enum { SC_T = 0, SC_WINDOW_STEPS = 1, SC_SEQ = 2, SC_DONE = 3, SC_STATUS = 4, SC_DONE_RB = 5, SC_QUEUE = 6, SC_SPARE = 7, SC_CLAIM = 8, SC_COUNT = 64 };
enum { FLAG_HIT = 1, FLAG_SLIP = 2 };
constexpr int kThreads = 256;
constexpr int kMaxChunks = 128;           // cap <= 32768
constexpr float kFixedOne = 1048576.0f;   // 2^20: resolution of the aggregated-CRF accumulator
constexpr int kTabLds = 256;              // decay-table entries kept in LDS by the LRFU kernels

struct Dev {
  int32_t L, Bz, Hq, Hkv, G, cap, units, max_chunks, slots, out_bf16;   // slots = partial slots per unit
  int32_t unit0;         // fused kernel: unit whose rows come first in the call's q, k_new, v_new and out (a single layer's first unit)
  int32_t by_order;      // fused kernel: schedule slot i holds unit order[i] (all layers), else unit unit0 + i (one layer)
  float scale_log2e;     // softmax_scale * log2(e): logits are kept in the base-2 domain
  float top_p;
  int32_t reward_mode, bmin, bmax, tab_last;
  uint16_t* K;
  uint16_t* V;
  float* crf;
  int32_t* tau;
  int32_t* pos;
  uint8_t* flags;
  int32_t* tbl;          // [units][max_seg] segment table: the pool segments (256 slots each) a unit's entries live in, in order
  int32_t max_seg;       // cap / 256, rounded up: columns of tbl
  int32_t* owned;        // [units] segments the unit owns: the first owned[u] entries of its row (the others hold 0)
  int32_t* spare;        // pool segments no unit owns, a stack of sc[SC_SPARE] entries
  int32_t* n;            // [units] entries held
  int32_t* budget;       // [units]
  int32_t* t_unit;       // [units] time of the unit's last decode step
  int32_t* nev;          // [units] entries evicted by the last eviction
  u64* window;           // [units] fixed-point sum of aggregated CRF since the last re-allocation
  int32_t* sc;           // scalars, SC_*
  const float* tab;      // lambda^delta, delta = 0..tab_last
  int4* items;           // scan work list: {unit, chunk, entries from the chunk's start, blocks before this item}
  float* partial;        // [units*slots][G][128]
  float* ml;             // [units*slots][G][2] (running max, sum)
  int32_t* stamp;        // [units*slots] launch sequence number that last wrote the slot
  float* logits;         // [units][cap/32][G][32] scaled logits (base-2 domain)
  long long* btotal;     // [Bz] budget total per sequence
  int32_t* order;        // [units] unit indices by descending budget (schedule of the fused kernel)
  int32_t* layer_ts;     // [layers][2] time and launch sequence number of a layer's last deferred step (scan_kernel<true> -> finish_kernel with late = 1)
  int32_t* arrive;       // [units] runs of the unit published so far by a scan that also merges (zero between launches)
  float* msum;           // [units][8][2] softmax maximum (base-2 domain) and 1 / sum per query head, left by layer_scan_kernel for its bookkeeping
};



// Where a unit's entries live.  Pool memory (K, V and the per-slot arrays) is handed out in segments of 256
// slots; row u of the segment table names unit u's segments in order, so entry i sits in pool slot
// row[i / 256] * 256 + i % 256 and whole 256-entry chunks (what one scan work item, one wavefront of the
// single-layer scan, eight blocks of the fused kernel's stream cover) are contiguous.  `row` may point to a
// copy of the row in LDS.
struct Slots {
  const int32_t* row;
  // pool slot of entry i (index into crf / tau / pos / flags)
  __device__ __forceinline__ size_t operator+(int i) const { return (size_t)row[i >> 8] * kSeg + (size_t)(i & (kSeg - 1)); }
  // element offset in the K / V pool of block b (32 entries) of the unit
  __device__ __forceinline__ size_t blk(int b) const { return (size_t)row[b >> 3] * kSegElems + (size_t)(b & (kSegBlocks - 1)) * kBlkElems; }
  // element offset in the K / V pool of K[entry r][dim c] / V[entry r][dim c]
  __device__ __forceinline__ size_t k(int r, int c) const { return (size_t)row[r >> 8] * kSegElems + (size_t)k_offset(r & (kSeg - 1), c); }
  __device__ __forceinline__ size_t v(int r, int c) const { return (size_t)row[r >> 8] * kSegElems + (size_t)v_offset(r & (kSeg - 1), c); }
};
__device__ __forceinline__ Slots slots_of(const Dev& d, int u) { return Slots{d.tbl + (size_t)u * d.max_seg}; }
// entries unit u has room for: what its segments hold, `cap` at most
__device__ __forceinline__ int unit_cap(const Dev& d, int u) { return min(d.cap, d.owned[u] * kSeg); }

// ------------------------------------------------------------------ helpers
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

template <class T>
__device__ __forceinline__ T wave_sum(T v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

// Cross-lane moves inside a row of 16 lanes without going through LDS.
template <int kCtrl>
__device__ __forceinline__ int dpp_i32(int v) {
  return __builtin_amdgcn_update_dpp(0, v, kCtrl, 0xF, 0xF, true);
}
// value of the lane `by` places further up in this lane's row of 16 (0 beyond the row's end); by = 1 .. 7
__device__ __forceinline__ float row_shl_f32(float v, int by) {
  const int x = __float_as_int(v);
  int r = 0;
  switch (by) {
    case 1: r = __builtin_amdgcn_update_dpp(0, x, 0x101, 0xF, 0xF, true); break;
    case 2: r = __builtin_amdgcn_update_dpp(0, x, 0x102, 0xF, 0xF, true); break;
    case 3: r = __builtin_amdgcn_update_dpp(0, x, 0x103, 0xF, 0xF, true); break;
    case 4: r = __builtin_amdgcn_update_dpp(0, x, 0x104, 0xF, 0xF, true); break;
    case 5: r = __builtin_amdgcn_update_dpp(0, x, 0x105, 0xF, 0xF, true); break;
    case 6: r = __builtin_amdgcn_update_dpp(0, x, 0x106, 0xF, 0xF, true); break;
    default: r = __builtin_amdgcn_update_dpp(0, x, 0x107, 0xF, 0xF, true); break;
  }
  return __int_as_float(r);
}
constexpr int kDppQuadSwap1 = 0xB1;      // quad_perm [1,0,3,2]
constexpr int kDppQuadSwap2 = 0x4E;      // quad_perm [2,3,0,1]
constexpr int kDppRowHalfMirror = 0x141;
constexpr int kDppRowMirror = 0x140;

// Sum over the 64 lanes, same fixed order in every lane: butterfly inside each
// row of 16 lanes, then the four row sums are read out and added.
__device__ __forceinline__ float wave_sum_f32(float v) {
  v += __int_as_float(dpp_i32<kDppQuadSwap1>(__float_as_int(v)));
  v += __int_as_float(dpp_i32<kDppQuadSwap2>(__float_as_int(v)));
  v += __int_as_float(dpp_i32<kDppRowHalfMirror>(__float_as_int(v)));
  v += __int_as_float(dpp_i32<kDppRowMirror>(__float_as_int(v)));
  const float r0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 0));
  const float r1 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 16));
  const float r2 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 32));
  const float r3 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 48));
  return (r0 + r1) + (r2 + r3);
}

__device__ __forceinline__ int wave_sum_i32(int v) {
  v += dpp_i32<kDppQuadSwap1>(v);
  v += dpp_i32<kDppQuadSwap2>(v);
  v += dpp_i32<kDppRowHalfMirror>(v);
  v += dpp_i32<kDppRowMirror>(v);
  return __builtin_amdgcn_readlane(v, 0) + __builtin_amdgcn_readlane(v, 16) + __builtin_amdgcn_readlane(v, 32) +
         __builtin_amdgcn_readlane(v, 48);
}

template <int kCtrl>
__device__ __forceinline__ u64 dpp_u64(u64 v) {
  const uint32_t lo = (uint32_t)dpp_i32<kCtrl>((int)(uint32_t)v);
  const uint32_t hi = (uint32_t)dpp_i32<kCtrl>((int)(uint32_t)(v >> 32));
  return ((u64)hi << 32) | lo;
}

__device__ __forceinline__ u64 readlane_u64(u64 v, int lane) {
  const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)v, lane);
  const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(v >> 32), lane);
  return ((u64)hi << 32) | lo;
}

__device__ __forceinline__ u64 wave_sum_u64(u64 v) {
  v += dpp_u64<kDppQuadSwap1>(v);
  v += dpp_u64<kDppQuadSwap2>(v);
  v += dpp_u64<kDppRowHalfMirror>(v);
  v += dpp_u64<kDppRowMirror>(v);
  return (readlane_u64(v, 0) + readlane_u64(v, 16)) + (readlane_u64(v, 32) + readlane_u64(v, 48));
}

__device__ __forceinline__ u64 min_u64(u64 a, u64 b) { return a < b ? a : b; }

__device__ __forceinline__ u64 wave_min_u64(u64 v) {
  v = min_u64(v, dpp_u64<kDppQuadSwap1>(v));
  v = min_u64(v, dpp_u64<kDppQuadSwap2>(v));
  v = min_u64(v, dpp_u64<kDppRowHalfMirror>(v));
  v = min_u64(v, dpp_u64<kDppRowMirror>(v));
  return min_u64(min_u64(readlane_u64(v, 0), readlane_u64(v, 16)), min_u64(readlane_u64(v, 32), readlane_u64(v, 48)));
}

// Barrier among the NT threads that work on one unit.  NT = 64: a single wavefront, which may be one of
// several in its workgroup and must not touch the workgroup barrier: its LDS and memory operations
// already execute in program order, only the compiler has to keep them so.
struct alignas(16) RedBuf {
  u64 v[2][8];          // one slot per wavefront: up to 512 threads
  float t[2][8][4];
};

template <int NT>
__device__ __forceinline__ void block_sync(RedBuf& rb) {
  if constexpr (NT == 64) {
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
  } else {
    __syncthreads();
  }
}

// Block-wide reductions over NT threads with a fixed combination order
// (deterministic).  `rb` is a [2][NT/64] LDS array used alternately, so one
// barrier per call suffices.  NT = 64: the wavefront's own reduction, nothing else.
template <int NT = kThreads>
__device__ __forceinline__ u64 block_sum_u64(u64 v, RedBuf& rb, int& phase, int tid) {
  v = wave_sum_u64(v);
  if constexpr (NT == 64) return v;
  if ((tid & 63) == 0) rb.v[phase][tid >> 6] = v;
  block_sync<NT>(rb);
  u64 r = rb.v[phase][0];
#pragma unroll
  for (int w = 1; w < NT / 64; ++w) r += rb.v[phase][w];
  phase ^= 1;
  return r;
}

template <int NT = kThreads>
__device__ __forceinline__ int block_sum_int(int v, RedBuf& rb, int& phase, int tid) {
  v = wave_sum_i32(v);
  if constexpr (NT == 64) return v;
  if ((tid & 63) == 0) rb.v[phase][tid >> 6] = (u64)(uint32_t)v;
  block_sync<NT>(rb);
  int r = (int)(uint32_t)rb.v[phase][0];
#pragma unroll
  for (int w = 1; w < NT / 64; ++w) r += (int)(uint32_t)rb.v[phase][w];
  phase ^= 1;
  return r;
}

template <int NT = kThreads>
__device__ __forceinline__ float block_sum_f32(float v, RedBuf& rb, int& phase, int tid) {
  v = wave_sum_f32(v);
  if constexpr (NT == 64) return v;
  if ((tid & 63) == 0) rb.v[phase][tid >> 6] = (u64)__float_as_uint(v);
  block_sync<NT>(rb);
  float r = __uint_as_float((uint32_t)rb.v[phase][0]);
#pragma unroll
  for (int w = 1; w < NT / 64; ++w) r += __uint_as_float((uint32_t)rb.v[phase][w]);
  phase ^= 1;
  return r;
}

// Three sums at once (one barrier).
template <int NT = kThreads>
__device__ __forceinline__ void block_sum3_f32(float& x, float& y, float& z, RedBuf& rb, int& phase, int tid) {
  x = wave_sum_f32(x);
  y = wave_sum_f32(y);
  z = wave_sum_f32(z);
  if constexpr (NT == 64) return;
  if ((tid & 63) == 0) *reinterpret_cast<f32x4*>(rb.t[phase][tid >> 6]) = f32x4{x, y, z, 0.f};
  block_sync<NT>(rb);
  f32x4 r = *reinterpret_cast<const f32x4*>(rb.t[phase][0]);
#pragma unroll
  for (int w = 1; w < NT / 64; ++w) {
    const f32x4 q = *reinterpret_cast<const f32x4*>(rb.t[phase][w]);
    r[0] += q[0];
    r[1] += q[1];
    r[2] += q[2];
  }
  x = r[0];
  y = r[1];
  z = r[2];
  phase ^= 1;
}

template <int NT = kThreads>
__device__ __forceinline__ u64 block_min_u64(u64 v, RedBuf& rb, int& phase, int tid) {
  v = wave_min_u64(v);
  if constexpr (NT == 64) return v;
  if ((tid & 63) == 0) rb.v[phase][tid >> 6] = v;
  block_sync<NT>(rb);
  u64 r = rb.v[phase][0];
#pragma unroll
  for (int w = 1; w < NT / 64; ++w) r = rb.v[phase][w] < r ? rb.v[phase][w] : r;
  phase ^= 1;
  return r;
}

// ------------------------------------------------------------------ fill
__global__ void fill_u32_kernel(uint32_t* p, uint32_t v, size_t count) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < count; i += stride) p[i] = v;
}

// ------------------------------------------------------------------ bandwidth probes
// Plain streaming kernels of known size: the on-box ceiling the scan kernel is
// compared with, and the calibration of the profiler's fetch/write counters.
__global__ __launch_bounds__(kThreads) void probe_read_kernel(const u32x4* __restrict__ src, size_t n_vec, uint32_t* sink) {
  const int lane = threadIdx.x & 63;
  const size_t nw = (size_t)gridDim.x * (kThreads / 64), gw = (size_t)blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
  u32x4 acc = {0u, 0u, 0u, 0u};
  for (size_t base = gw * 1024; base + 1024 <= n_vec; base += nw * 1024) {     // 16 KB per wavefront and round
    u32x4 v[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) v[i] = __builtin_nontemporal_load(src + base + i * 64 + lane);
#pragma unroll
    for (int i = 0; i < 16; ++i) acc ^= v[i];
  }
  if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9E3779B9u) sink[0] = 1u;          // keeps the loads alive
}

__global__ __launch_bounds__(kThreads) void probe_copy_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst, size_t n_vec) {
  size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * kThreads;
  for (; i < n_vec; i += stride) dst[i] = src[i];
}

// ------------------------------------------------------------------ pool segments between units
// Shared pools (headroom >= 1): a unit should own the segments that budget + headroom entries need, never
// fewer than its entries occupy, and for the units [x_begin, x_begin + x_count) at least what x_entries
// entries need (a prompt on its way in; x_len, if given, holds the units' own lengths, headroom not included).  One workgroup walks all units twice: units that own more than
// they should push the surplus (their last segments) onto the spare stack, then units that own less pop what
// they lack.  Who gets which segment follows from prefix sums over the units in index order, so the result
// does not depend on timing.  If the spare list is short nobody is given anything and bit 2 of the status
// word is set; a unit that still holds more entries than its budget (its eviction has not run yet) keeps
// its segments until a later call.  Unowned columns of a table row hold 0.
constexpr int kBalanceThreads = 1024;
__global__ __launch_bounds__(kBalanceThreads) void rebalance_kernel(Dev d, int headroom, int x_begin, int x_count, int x_entries,
                                                                    const int32_t* x_len) {
  __shared__ int s_part[kBalanceThreads / 64];
  __shared__ int s_total;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int per = (d.units + kBalanceThreads - 1) / kBalanceThreads;
  const int u0 = min(d.units, tid * per), u1 = min(d.units, u0 + per);
  // what this kernel writes and reads back (ownership, table cells, the spare stack) goes through accesses that
  // are coherent one by one, whichever thread wrote them
  auto ld = [](const int32_t* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); };
  auto st = [](int32_t* p, int32_t v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); };
  auto need_of = [&](int u) {
    int e = max(d.budget[u] + headroom, d.n[u]);
    if (u >= x_begin && u < x_begin + x_count) e = max(e, x_len ? min(max(x_len[u - x_begin], 0) + headroom, x_entries) : x_entries);
    return min(d.max_seg, (e + kSeg - 1) / kSeg);
  };
  // exclusive prefix over the threads' ranges of a per-thread count; the total lands in s_total
  auto scan = [&](int local) -> int {
    int incl = local;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int v = __shfl_up(incl, o);
      if (lane >= o) incl += v;
    }
    __syncthreads();                       // the previous scan's readers are done
    if (lane == 63) s_part[wave] = incl;
    __syncthreads();
    int before = incl - local;
    for (int w = 0; w < wave; ++w) before += s_part[w];
    if (tid == kBalanceThreads - 1) s_total = before + local;
    __syncthreads();
    return before;
  };
  int spare_n = d.sc[SC_SPARE];
  // ---- release
  int local = 0;
  for (int u = u0; u < u1; ++u) local += max(0, ld(d.owned + u) - need_of(u));
  int at = spare_n + scan(local);
  for (int u = u0; u < u1; ++u) {
    const int need = need_of(u), own = ld(d.owned + u);
    for (int j = need; j < own; ++j) {
      int32_t* cell = d.tbl + (size_t)u * d.max_seg + j;
      st(d.spare + at++, ld(cell));
      st(cell, 0);
    }
    if (own > need) st(d.owned + u, need);
  }
  spare_n += s_total;
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");      // the stack's new entries before anyone pops them
  // ---- grant
  local = 0;
  for (int u = u0; u < u1; ++u) local += max(0, need_of(u) - ld(d.owned + u));
  int from = scan(local);
  const int wanted = s_total;
  if (wanted > spare_n) {
    if (tid == 0) {
      atomicOr(&d.sc[SC_STATUS], 4);
      d.sc[SC_SPARE] = spare_n;
    }
    return;
  }
  for (int u = u0; u < u1; ++u) {
    const int need = need_of(u), own = ld(d.owned + u);
    for (int j = own; j < need; ++j) st(d.tbl + (size_t)u * d.max_seg + j, ld(d.spare + (spare_n - 1 - from++)));
    if (need > own) st(d.owned + u, need);
  }
  if (tid == 0) d.sc[SC_SPARE] = spare_n - wanted;
}

// ------------------------------------------------------------------ cache load
// grid: (ceil(P/32), units of the layer); converts 32 row-major rows to one
// tiled block.  k, v: [units][P][128]; unit `urel` holds len[urel] (or P)
// entries; rows beyond that become zero.
__global__ __launch_bounds__(kThreads) void load_cache_kernel(Dev d, int unit_begin, const uint16_t* k,
                                                              const uint16_t* v, int P, const int32_t* len,
                                                              const float* crf0, const int32_t* tau0,
                                                              const int32_t* pos0) {
  __shared__ uint16_t vt[kBlk][kDim + 8];
  const int tid = threadIdx.x;
  const int urel = blockIdx.y, u = unit_begin + urel;
  const int blk = blockIdx.x, r0 = blk * kBlk;
  int n = len ? min(max(len[urel], 0), P) : P;
  if (n >= unit_cap(d, u)) {                     // the unit's segments do not hold it (shared pools that ran short)
    n = max(unit_cap(d, u) - 1, 0);
    if (blk == 0 && tid == 0) atomicOr(&d.sc[SC_STATUS], 1);
  }
  if (blk == 0 && tid == 0) {
    d.n[u] = n;
    d.nev[u] = 0;
  }
  if (r0 >= n) return;
  const uint16_t* ksrc = k + (size_t)urel * P * kDim;
  const uint16_t* vsrc = v + (size_t)urel * P * kDim;
  const Slots sl = slots_of(d, u);
  uint16_t* kdst = d.K + sl.blk(blk);          // this block's 32 entries
  uint16_t* vdst = d.V + sl.blk(blk);
  // K: 32 rows x 16 pieces of 16 bytes
  for (int p = tid; p < kBlk * 16; p += kThreads) {
    int rr = p >> 4, piece = p & 15, r = r0 + rr;
    u32x4 x = {0u, 0u, 0u, 0u};
    if (r < n) x = *reinterpret_cast<const u32x4*>(ksrc + (size_t)r * kDim + piece * 8);
    *reinterpret_cast<u32x4*>(kdst + k_offset(rr, piece * 8)) = x;
  }
  // V: stage the rows, then write 16-byte pieces of the entry-interleaved order
  for (int p = tid; p < kBlk * 16; p += kThreads) {
    int rr = p >> 4, piece = p & 15, r = r0 + rr;
    u32x4 x = {0u, 0u, 0u, 0u};
    if (r < n) x = *reinterpret_cast<const u32x4*>(vsrc + (size_t)r * kDim + piece * 8);
    *reinterpret_cast<u32x4*>(&vt[rr][piece * 8]) = x;
  }
  __syncthreads();
  for (int p = tid; p < 8 * 64; p += kThreads) {
    int dt = p >> 6, kg = (p >> 4) & 3, j = p & 15;
    uint16_t e8[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      int rr = (e < 4) ? (4 * kg + e) : (16 + 4 * kg + (e - 4));
      e8[e] = vt[rr][16 * dt + j];
    }
    u32x4 x;
    x.x = e8[0] | ((uint32_t)e8[1] << 16);
    x.y = e8[2] | ((uint32_t)e8[3] << 16);
    x.z = e8[4] | ((uint32_t)e8[5] << 16);
    x.w = e8[6] | ((uint32_t)e8[7] << 16);
    *reinterpret_cast<u32x4*>(vdst + (size_t)p * 8) = x;
  }
  // per-slot state
  const Slots base = sl;
  for (int rr = tid; rr < kBlk; rr += kThreads) {
    int r = r0 + rr;
    if (r < n) {
      d.pos[base + r] = pos0 ? pos0[(size_t)urel * P + r] : r;
      d.crf[base + r] = crf0 ? crf0[(size_t)urel * P + r] : 1.0f;
      d.tau[base + r] = tau0 ? tau0[(size_t)urel * P + r] : (P - 1);
      d.flags[base + r] = 0;
    }
  }
}

// Before the replay of a prompt's last W queries (done = 0): every entry of the layer's units starts as
// referenced once, on arrival (CRF 1, tau = position), the W entries of the window as not yet arrived
// (CRF 0; their own query's step is their arrival).  After it (done = 1): the replay leaves no trace in
// the units' aggregated-CRF window, and their last-step time is the one a fresh context has.
__global__ __launch_bounds__(kThreads) void seed_state_kernel(Dev d, int unit_begin, int P, int W, int done, int t_unit) {
  const int u = unit_begin + blockIdx.y;
  if (done) {
    if (blockIdx.x == 0 && threadIdx.x == 0) {
      d.window[u] = 0;
      d.t_unit[u] = t_unit;
    }
    return;
  }
  const Slots base = slots_of(d, u);
  for (int i = blockIdx.x * kThreads + threadIdx.x; i < P; i += gridDim.x * kThreads) {
    d.crf[base + i] = i < P - W ? 1.0f : 0.0f;
    d.tau[base + i] = i;
  }
}

// ------------------------------------------------------------------ prep
// 32 threads per unit, 32 units per workgroup: append the new entry (unless
// bit 0 of `append` is clear) and publish the unit's scan work items {unit, chunk, entries
// from the chunk's start to the unit's end, blocks in the list before this
// item}.  One 64-bit atomic per workgroup claims the list range and the block
// range together, so the list is sorted by block offset and unit-major (its
// order only affects scheduling, never results).
constexpr int kPrepThreads = 1024;
constexpr int kPrepUnits = 32;

__global__ __launch_bounds__(kPrepThreads) void prep_kernel(Dev d, int unit_begin, int unit_count, const uint16_t* k_new,
                                                            const uint16_t* v_new, int append, int n_limit,
                                                            const uint16_t* __restrict__ q) {
  __shared__ int s_nch[kPrepUnits], s_nblk[kPrepUnits];
  __shared__ u64 s_base;
  const int tid = threadIdx.x, sub = tid & 31, slot = tid >> 5;
  const int w = blockIdx.x * kPrepUnits + slot;
  const bool active = w < unit_count;
  const int u = unit_begin + w;
  int n = 0, n_before = 0;
  if (active) {
    n = min(d.n[u], n_limit);            // n_limit < n: only the unit's first n_limit entries take part (prompt replay)
    n_before = n;
    if (append & 1) {
      const int t = d.sc[SC_T];
      if (n >= unit_cap(d, u)) {
        if (sub == 0) atomicOr(&d.sc[SC_STATUS], 1);
      } else {
        const Slots sl = slots_of(d, u);
        if (sub < 16)
          *reinterpret_cast<u32x4*>(d.K + sl.k(n, sub * 8)) =
              *reinterpret_cast<const u32x4*>(k_new + (size_t)w * kDim + sub * 8);
#pragma unroll
        for (int e = 0; e < 4; ++e) d.V[sl.v(n, sub * 4 + e)] = v_new[(size_t)w * kDim + sub * 4 + e];
        if (sub == 0) {
          const size_t s = sl + n;
          d.crf[s] = 0.0f;
          d.tau[s] = t;
          d.pos[s] = t;
          d.flags[s] = 0;
          d.n[u] = n + 1;
        }
        n += 1;
      }
    }
  }
  const int nch = active ? (n + kChunk - 1) / kChunk : 0;
  const int nblk = active ? (n + kBlk - 1) / kBlk : 0;
  if (sub == 0) {
    s_nch[slot] = nch;
    s_nblk[slot] = nblk;
  }
  __syncthreads();
  if (tid == 0) {
    int tot = 0, totb = 0;
    for (int i = 0; i < kPrepUnits; ++i) {
      const int c = s_nch[i], b = s_nblk[i];
      s_nch[i] = tot;
      s_nblk[i] = totb;
      tot += c;
      totb += b;
    }
    s_base = atomicAdd(reinterpret_cast<u64*>(&d.sc[SC_CLAIM]), (u64)(uint32_t)tot | ((u64)(uint32_t)totb << 32));
  }
  __syncthreads();
  if (active) {
    const int base = (int)(uint32_t)s_base + s_nch[slot];
    const int bbase = (int)(uint32_t)(s_base >> 32) + s_nblk[slot];
    for (int c = sub; c < nch; c += 32) d.items[base + c] = make_int4(u, c, n - c * kChunk, bbase + c * kChunkBlocks);
  }
}

// ------------------------------------------------------------------ scan
struct KFrag {
  u32x4 k[8];
};
struct VFrag {
  u32x4 v[8];
};

// K and V are read once per step and never reused: non-temporal loads keep
// them from displacing the partials and logits that the finish kernel re-reads.
__device__ __forceinline__ u32x4 stream_load(const uint16_t* p) {
  return __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
}

// `kb` / `vb` already include the lane's offset (8 bf16 per lane).
__device__ __forceinline__ void load_k(KFrag& f, const uint16_t* kb) {
#pragma unroll
  for (int i = 0; i < 8; ++i) f.k[i] = stream_load(kb + i * 512);
}

__device__ __forceinline__ void load_v(VFrag& f, const uint16_t* vb) {
#pragma unroll
  for (int i = 0; i < 8; ++i) f.v[i] = stream_load(vb + i * 512);
}

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 x) { return __builtin_bit_cast(bf16x8, x); }

// One block of 32 entries is processed in two halves so that each fragment's
// registers can be refilled as soon as it has been consumed.  The scaled logits
// leave through a wave-private LDS tile so that each block's values go to memory
// as one contiguous store.
constexpr int kLgRow = 36;     // floats per head row in the LDS tile (32 + pad against bank conflicts)

// First half of a block of 32 entries: logits on the matrix cores, masked and
// scaled into sv[8] (this lane's 4 + 4 entries), and sent on their way to the
// finish phase.  The K fragment is dead afterwards.
__device__ __forceinline__ void scan_qk(const KFrag& f, const bf16x8 (&qv)[4], float (&sv)[8], float c_scale, int e_base,
                                        int n_valid, float* lds_lg, int lds_row, float* lg_dst, int G, int lane) {
  const int j = lane & 15, kg = lane >> 4;
  f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int s = 0; s < 4; ++s) s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(f.k[s]), qv[s], s0, 0, 0, 0);
#pragma unroll
  for (int s = 0; s < 4; ++s) s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(f.k[4 + s]), qv[s], s1, 0, 0, 0);
#pragma unroll
  for (int v = 0; v < 4; ++v) {
    sv[v] = (e_base + 4 * kg + v < n_valid) ? s0[v] * c_scale : -INFINITY;
    sv[4 + v] = (e_base + 4 * kg + 16 + v < n_valid) ? s1[v] * c_scale : -INFINITY;
  }
  // logits: row j of the LDS buffer (a wave-private staging tile, or the block's
  // place in a resident logits tile); with lg_dst the tile is forwarded to memory
  // as one contiguous 128 G-byte store
  if (lds_lg == nullptr) return;            // attention only: nobody looks at the logits afterwards
  if (j < G) {
    *reinterpret_cast<f32x4*>(lds_lg + j * lds_row + 4 * kg) = f32x4{sv[0], sv[1], sv[2], sv[3]};
    *reinterpret_cast<f32x4*>(lds_lg + j * lds_row + 16 + 4 * kg) = f32x4{sv[4], sv[5], sv[6], sv[7]};
  }
  if (lg_dst) {
    __builtin_amdgcn_wave_barrier();
    if (lane < 8 * G) {
      const f32x4 row = *reinterpret_cast<const f32x4*>(lds_lg + (lane >> 3) * lds_row + 4 * (lane & 7));
      *reinterpret_cast<f32x4*>(lg_dst + e_base * G) = row;
    }
    __builtin_amdgcn_wave_barrier();
  }
}

// Second half: online softmax update and probabilities (split into two bf16
// terms) times V on the matrix cores.  The V fragment is dead afterwards.
//
// PACK: the caller has duplicated the query heads 0..7 into the MFMA's columns 8..15 (at most 8 heads are
// real), so lane (j + 8, kg) holds the same logits and probabilities as lane (j, kg).  The product's
// operand then carries the high terms in rows 0..7 and the low terms in rows 8..15: one MFMA per 16
// dims instead of two, the result rows g (high) and g + 8 (low) of head g are added by the caller at the
// end of the unit (acc of lane + 32).
template <bool PACK = false>
__device__ __forceinline__ void scan_pv(const float (&sv)[8], const VFrag& fv, f32x4 (&acc)[8], float& m_run, float& l_run,
                                        int lane) {
  float bm = fmaxf(fmaxf(fmaxf(sv[0], sv[1]), fmaxf(sv[2], sv[3])), fmaxf(fmaxf(sv[4], sv[5]), fmaxf(sv[6], sv[7])));
  bm = fmaxf(bm, __shfl_xor(bm, 16));
  bm = fmaxf(bm, __shfl_xor(bm, 32));
  if (__any(bm > m_run)) {
    const float m_new = fmaxf(m_run, bm);
    const float sc = fast_exp2(m_run - m_new);
    l_run *= sc;
    m_run = m_new;
    const int h4 = (lane >> 4) << 2;
    const float c0 = __shfl(sc, h4), c1 = __shfl(sc, h4 + 1), c2 = __shfl(sc, h4 + 2), c3 = __shfl(sc, h4 + 3);
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) {
      acc[dt][0] *= c0;
      acc[dt][1] *= c1;
      acc[dt][2] *= c2;
      acc[dt][3] *= c3;
    }
  }
  bf16x8 ph, pl;
  float ps = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const float p = fast_exp2(sv[i] - m_run);
    ps += p;
    const __bf16 h = (__bf16)p;
    ph[i] = h;
    pl[i] = (__bf16)(p - (float)h);
  }
  l_run += ps;
  if constexpr (PACK) {
    const bool low = (lane & 8) != 0;
    const u32x4 h4 = __builtin_bit_cast(u32x4, ph), l4 = __builtin_bit_cast(u32x4, pl);
    const u32x4 a4 = {low ? l4[0] : h4[0], low ? l4[1] : h4[1], low ? l4[2] : h4[2], low ? l4[3] : h4[3]};
    const bf16x8 pa = as_bf16x8(a4);
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) acc[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pa, as_bf16x8(fv.v[dt]), acc[dt], 0, 0, 0);
  } else {
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) {
      acc[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ph, as_bf16x8(fv.v[dt]), acc[dt], 0, 0, 0);
      acc[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pl, as_bf16x8(fv.v[dt]), acc[dt], 0, 0, 0);
    }
  }
}

struct Item {
  int u, c, n_valid, blk_off;
};

__device__ __forceinline__ Item fetch_item(const Dev& d, int it) {
  const int4 r = d.items[it];
  Item m;
  m.u = __builtin_amdgcn_readfirstlane(r.x);
  m.c = __builtin_amdgcn_readfirstlane(r.y);
  m.n_valid = __builtin_amdgcn_readfirstlane(r.z);
  m.blk_off = __builtin_amdgcn_readfirstlane(r.w);
  return m;
}

// Index of the work item that holds global block `b` (largest i with
// items[i].blk_off <= b): 64-way search, one probe per lane and round.
__device__ __forceinline__ int find_item(const Dev& d, int n_items, int b, int lane) {
  int lo = 0, hi = n_items;
  while (hi - lo > 1) {
    const int step = (hi - lo + 63) >> 6;
    const int idx = lo + lane * step;
    const int off = idx < hi ? d.items[idx].w : 0x7FFFFFFF;
    const u64 mask = __ballot(off <= b);
    const int k = __popcll(mask) - 1;            // lane 0 always qualifies
    lo += k * step;
    hi = min(hi, lo + step);
  }
  return __builtin_amdgcn_readfirstlane(lo);
}

// What step_epilogue leaves behind, written by the one thread that knows the launch is complete (the end of
// the kernel makes it visible).
__device__ __forceinline__ void scan_epilogue(const Dev& d, int seq, int advance, int layer) {
  const int t = d.sc[SC_T];
  if (layer >= 0) {
    d.layer_ts[2 * layer] = t;
    d.layer_ts[2 * layer + 1] = seq;
  }
  d.sc[SC_DONE] = 0;
  d.sc[SC_CLAIM] = 0;
  d.sc[SC_CLAIM + 1] = 0;
  d.sc[SC_SEQ] = seq + 1;
  if (advance) {
    d.sc[SC_T] = t + 1;
    d.sc[SC_WINDOW_STEPS] = d.sc[SC_WINDOW_STEPS] + 1;
  }
}

// Stores and loads that are coherent across the chip's L2 caches one by one (no cache-wide write-back or
// invalidation, which a fence at that scope would cost every wavefront): how a scan that merges hands its
// partials from the wavefronts that wrote them to the one that combines them.
template <bool COHERENT, class T>
__device__ __forceinline__ void put(T* p, T v) {
  if constexpr (COHERENT)
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  else
    *p = v;
}
template <class T>
__device__ __forceinline__ T get_coherent(const T* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// LDS floats one wavefront needs for merge_unit_wave: maximum/weight and sum of every run and head
constexpr int kMergeLds = 2 * (kMaxChunks + 1) * kMaxGroup;

// merge_partials for one wavefront of a scan that merges: the same values combined in the same order (slot
// after slot), so the output has the same bits; only the distribution over lanes differs.  The reads are
// coherent ones, since the partials come from other wavefronts of the same launch, and no stamp is read:
// the unit's blocks start at global block u0 and shares are `per` blocks long, so run r > 0 begins at the
// r-th share boundary inside the unit, which names its slot.  `sw` holds kMergeLds floats.
__device__ __forceinline__ void merge_unit_wave(const Dev& d, int u, int urel, int u0, int per, int runs, float* sw, void* out,
                                                int lane) {
  const int G = d.G;
  const size_t slot0 = (size_t)u * d.slots;
  float* sl = sw + (kMaxChunks + 1) * kMaxGroup;
  const int first = u0 / per;
  auto slot_of = [&](int r) { return r == 0 ? 0 : 1 + ((first + r) * per - u0) / kChunkBlocks; };
  const int g_lane = lane & 7;                         // i & 7 for every i this lane visits
  // four runs' partials (all heads, two dims per lane) are requested at once, the first four before anything else
  float2 x[4][kMaxGroup];
  auto request = [&](int r0) {
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const size_t slot = slot0 + slot_of(min(r0 + k, runs - 1));
#pragma unroll
      for (int g = 0; g < kMaxGroup; ++g) {
        const float* pp = d.partial + (slot * G + min(g, G - 1)) * kDim + 2 * lane;
        x[k][g] = make_float2(get_coherent(pp), get_coherent(pp + 1));
      }
    }
  };
  if (out) request(0);
  for (int i = lane; i < runs * kMaxGroup; i += 64) {
    const float* mlp = d.ml + ((slot0 + slot_of(i >> 3)) * G + min(g_lane, G - 1)) * 2;
    const float m = get_coherent(mlp), l = get_coherent(mlp + 1);
    sw[i] = g_lane < G ? m : -INFINITY;
    sl[i] = g_lane < G ? l : 0.f;
  }
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
  float M = -INFINITY;
  if (lane < G)
    for (int r = 0; r < runs; ++r) M = fmaxf(M, sw[r * kMaxGroup + lane]);
  const float Mg = __shfl(M, g_lane);
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
  for (int i = lane; i < runs * kMaxGroup; i += 64) {
    const float m = sw[i];
    sw[i] = (g_lane < G && m > -INFINITY) ? fast_exp2(m - Mg) : 0.f;
  }
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
  float inv = 0.f;
  if (lane < G) {
    float Lsum = 0.f;
    for (int r = 0; r < runs; ++r) {
      const float w = sw[r * kMaxGroup + lane];
      if (w != 0.f) Lsum += sl[r * kMaxGroup + lane] * w;
    }
    inv = 1.0f / Lsum;
  }
  if (!out) return;
  float2 o[kMaxGroup];
#pragma unroll
  for (int g = 0; g < kMaxGroup; ++g) o[g] = make_float2(0.f, 0.f);
  for (int r0 = 0; r0 < runs; r0 += 4) {
    if (r0 > 0) request(r0);
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      if (r0 + k < runs) {
#pragma unroll
        for (int g = 0; g < kMaxGroup; ++g) {
          const float w = sw[(r0 + k) * kMaxGroup + g];
          if (w != 0.f) {
            o[g].x += x[k][g].x * w;
            o[g].y += x[k][g].y * w;
          }
        }
      }
    }
  }
#pragma unroll
  for (int g = 0; g < kMaxGroup; ++g) {
    const float inv_g = __shfl(inv, g);
    if (g < G) {
      const size_t oi = ((size_t)urel * G + g) * kDim + 2 * lane;
      const float ox = o[g].x * inv_g, oy = o[g].y * inv_g;
      if (d.out_bf16) {
        __bf16* dst = reinterpret_cast<__bf16*>(out) + oi;
        dst[0] = (__bf16)ox;
        dst[1] = (__bf16)oy;
      } else {
        *reinterpret_cast<float2*>(reinterpret_cast<float*>(out) + oi) = make_float2(ox, oy);
      }
    }
  }
}

// Persistent grid.  The blocks (32 entries) of all work items form one
// sequence, sorted unit-major; every wavefront takes an equal contiguous share
// of it.  Its share is a few long RUNS: consecutive blocks of one unit,
// contiguous in memory, over which the online softmax simply continues.  A run
// is streamed block by block: while block b is computed the K tile of block
// b+1 (the next run's first block at the end of a run) is in flight, and V
// follows as soon as the previous V has been consumed.  All loads in the loop
// are unconditional, so the waits the compiler inserts are exact.  A run
// leaves one partial (max, sum, acc), stamped with the launch sequence number,
// in slot 0 of its unit if it starts the unit, else in slot 1 + chunk of its
// first block (shares are at least one chunk long, so no two runs collide).
// `q` holds the query rows of the units [unit_begin, ...) of this call:
// row (u - unit_begin) * G + g.
//
// MERGE: the kernel also finishes the attention.  Every run is counted on its
// unit; the wavefront that publishes a unit's last run merges the unit's
// partials and writes its output rows, so no second kernel stands between the
// scan and the caller.  The wavefront that accounts for the launch's last block
// leaves the step scalars as step_epilogue would and, for a single-layer step
// whose bookkeeping follows later, notes the step's time and sequence number
// under `layer`.
template <bool MERGE>
__global__ __launch_bounds__(kThreads, 2) void scan_kernel(Dev d, int unit_begin, const uint16_t* __restrict__ q, void* out,
                                                           int advance, int layer) {
  __shared__ float s_lg[kThreads / 64][kMaxGroup * kLgRow];
  __shared__ float s_mw[MERGE ? kThreads / 64 : 1][MERGE ? kMergeLds : 1];
  const int lane = threadIdx.x & 63;
  const int nw = gridDim.x * (kThreads / 64);
  const int gw = __builtin_amdgcn_readfirstlane(blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6));
  const int n_items = d.sc[SC_CLAIM];
  const int n_blocks = d.sc[SC_CLAIM + 1];
  const int seq = d.sc[SC_SEQ];
  const int per = max(kChunkBlocks, (n_blocks + nw - 1) / nw);
  int b_cur = gw * per;                                  // global block index
  const int b_end = min(n_blocks, b_cur + per);
  // MERGE: the launch is complete when every block is accounted for; a workgroup reports its blocks once, through
  // its last wavefront to finish (one atomic per workgroup on the shared counter instead of one per wavefront)
  __shared__ int s_waves_done;
  if (MERGE) {
    if (threadIdx.x == 0) s_waves_done = 0;
    __syncthreads();
  }
  auto wave_done = [&]() {
    if (lane != 0 || atomicAdd(&s_waves_done, 1) != kThreads / 64 - 1) return;
    const int w0 = blockIdx.x * (kThreads / 64);
    const int wg_blocks = min(n_blocks, (w0 + kThreads / 64) * per) - min(n_blocks, w0 * per);
    if (wg_blocks > 0 && atomicAdd(&d.sc[SC_DONE], wg_blocks) + wg_blocks == n_blocks) scan_epilogue(d, seq, advance, layer);
  };
  if (b_cur >= b_end) {
    if (MERGE) {
      if (n_blocks == 0 && gw == 0 && lane == 0) scan_epilogue(d, seq, advance, layer);   // nothing to scan at all
      wave_done();
    }
    return;
  }
  float* lds_lg = s_lg[threadIdx.x >> 6];
  const int j = lane & 15, kg = lane >> 4;
  const int G = d.G;
  const bool head_lane = j < G;
  const int jq = head_lane ? j : 0;

  int it = find_item(d, n_items, b_cur, lane);
  Item cur = fetch_item(d, it);
  KFrag ka;
  VFrag va;
  {
    const size_t off = slots_of(d, cur.u).blk(cur.c * kChunkBlocks + (b_cur - cur.blk_off)) + lane * 8;
    load_k(ka, d.K + off);
    load_v(va, d.V + off);
  }
  while (true) {
    // ---- one run: blocks [fb, fb + nblk) of unit cur.u, fb counted from the unit's start
    const int fb_item = b_cur - cur.blk_off;                                   // first block, inside item `it`
    const int fb = cur.c * kChunkBlocks + fb_item;
    const int run_valid = cur.n_valid - fb_item * kBlk;                        // entries from the run's start to the unit's end
    const int nblk = min((run_valid + kBlk - 1) / kBlk, b_end - b_cur);
    const int b_next = b_cur + nblk;
    const bool have_next = b_next < b_end;
    const int it_next = it + (fb_item + nblk + kChunkBlocks - 1) / kChunkBlocks;   // next unit's first item
    const Item nxt = have_next ? fetch_item(d, it_next) : cur;
    bf16x8 qv[4];
    {
      const uint16_t* qrow = q + ((size_t)(cur.u - unit_begin) * G + jq) * kDim + 8 * kg;
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        u32x4 x = *reinterpret_cast<const u32x4*>(qrow + 32 * s);
        if (!head_lane) x = u32x4{0u, 0u, 0u, 0u};
        qv[s] = as_bf16x8(x);
      }
    }
    // The run's blocks are consecutive in the unit but contiguous in memory only inside a segment (8 blocks):
    // lane i holds the pool segment of the unit's segment fb / 8 + i (reloaded every 64 segments), and a
    // block's address comes from there without another trip to memory.
    const int32_t* seg_row = d.tbl + (size_t)cur.u * d.max_seg;
    int seg_first = fb >> 3;
    int seg_reg = seg_row[min(seg_first + lane, d.max_seg - 1)];
    auto block_off = [&](int b) -> size_t {            // element offset of the unit's block b (b >= fb)
      if ((b >> 3) - seg_first >= 64) {
        seg_first = b >> 3;
        seg_reg = seg_row[min(seg_first + lane, d.max_seg - 1)];
      }
      return (size_t)__builtin_amdgcn_readlane(seg_reg, (b >> 3) - seg_first) * kSegElems + (size_t)(b & (kSegBlocks - 1)) * kBlkElems +
             lane * 8;
    };
    // after the run's last block the stream continues with the next run (whose first segment is asked for now
    // and looked at then), or re-reads this block at the very end
    const int nxt_seg = d.tbl[(size_t)nxt.u * d.max_seg + nxt.c];
    // logits of a block are stored as [head][32 entries]: 128 G contiguous bytes, 16 per lane
    float* lg_dst = d.logits + ((size_t)cur.u * d.cap + (size_t)fb * kBlk) * G + 4 * min(lane, 8 * G - 1);
    f32x4 acc[8];
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) acc[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    float m_run = -INFINITY, l_run = 0.f;
    int blk = 0;

    // stream: the K tile of block b+1 is requested right after block b's logits are done, the V tile
    // right after block b's PV; at the end of the run both continue with the next run's first block
    while (true) {
      const bool last = blk + 1 == nblk;
      const size_t n_off = !last ? block_off(fb + blk + 1) : have_next ? (size_t)nxt_seg * kSegElems + lane * 8 : block_off(fb + blk);
      float sv[8];
      scan_qk(ka, qv, sv, d.scale_log2e, blk * kBlk, run_valid, lds_lg, kLgRow, lg_dst, G, lane);
      load_k(ka, d.K + n_off);
      scan_pv(sv, va, acc, m_run, l_run, lane);
      load_v(va, d.V + n_off);
      ++blk;
      if (last) break;
    }
    // ---- publish the run's partial
    l_run += __shfl_xor(l_run, 16);
    l_run += __shfl_xor(l_run, 32);
    const size_t slot = (size_t)cur.u * d.slots + (fb == 0 ? 0 : 1 + fb / kChunkBlocks);
    if (head_lane && kg == 0) {
      put<MERGE>(&d.ml[(slot * G + j) * 2], m_run);
      put<MERGE>(&d.ml[(slot * G + j) * 2 + 1], l_run);
    }
    if (lane == 0) put<MERGE>(&d.stamp[slot], seq);
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int head = 4 * kg + v;
      if (head < G) {
        float* dst = d.partial + (slot * G + head) * kDim + j;
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) put<MERGE>(&dst[16 * dt], acc[dt][v]);
      }
    }
    if (MERGE) {
      // the partial before the count: its stores are coherent across the chip, so it is enough that they have completed
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      // runs of this unit = shares that its blocks [u0, u0 + unb) touch
      const int u0 = cur.blk_off - cur.c * kChunkBlocks;
      const int unb = (cur.n_valid + cur.c * kChunk + kBlk - 1) / kBlk;
      const int runs = (u0 + unb - 1) / per - u0 / per + 1;
      int last = 0;
      if (lane == 0) {
        last = atomicAdd(&d.arrive[cur.u], 1) == runs - 1;
        if (last) __hip_atomic_store(&d.arrive[cur.u], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // the word other wavefronts update atomically
      }
      if (__builtin_amdgcn_readfirstlane(last))          // the other runs' partials are read with coherent loads
        merge_unit_wave(d, cur.u, cur.u - unit_begin, u0, per, runs, s_mw[threadIdx.x >> 6], out, lane);
    }
    if (!have_next) break;
    b_cur = b_next;
    it = it_next;
    cur = nxt;
  }
  if (MERGE) wave_done();
}

// ------------------------------------------------------------------ single-layer scan that appends by itself
// The shape a model imposes is one call per layer, a few hundred units at most: too few for the fused kernel
// (one workgroup per unit) and too little work for the persistent scan above to amortise its work list.  Here
// the grid itself is the work list: workgroup (x, y) takes chunks 4 y .. 4 y + 3 (256 entries each, one per
// wavefront) of the layer's unit x and leaves at once if the unit is shorter.  (Units along x: consecutive
// workgroups go to different XCDs, so the workgroups that have work - every unit's first, most units' second -
// spread over all of them; with the chunk groups along x, and eight or a multiple of them, each XCD would get
// one group index, the first few all the work, and a step takes 1.6 times as long.)  Nothing has to run before it:
// every workgroup derives the unit's length after the append from the stored one (which stays as it is until
// the bookkeeping that follows, finish_kernel with late = 2, has recorded the append), and the wavefront whose
// chunk receives the new entry puts its key and value rows into the block it has just loaded (and into the
// cache), so that the entry takes part like any cached one.  The four wavefronts combine their softmax states
// in LDS; a unit of one workgroup (up to 1024 entries) is finished there and then, a longer one goes through
// one partial per workgroup, merged by the workgroup that publishes the last (coherent stores and loads as in
// scan_kernel<true>).  The unit's softmax maximum and 1 / sum per head stay in `msum` for the bookkeeping.
// kW wavefronts per workgroup, each over 1 / kSplit of a chunk; the text above describes <4, 1>, the shape in
// use.  Measured beside it on 128 units of 257 .. 8193 entries: fewer wavefronts per workgroup (<2, 1>, <1, 1>)
// 2 % and 15 % slower per step, more (<8, 1>) 8 %, shorter spans (<4, 2>, <8, 2>, <8, 4>) 8 %, 23 % and 49 %
// (also with three wavefronts per SIMD); rotating the units against the chunk groups, or the long units' last
// chunks first: no difference.  What does matter is how many workgroups a compute unit may hold: see the launch.
// grid: (units of the layer, ceil(max_chunks * kSplit / kW)), 64 kW threads.
// Entry rr of the block in (ka, va) is replaced by the rows in `rows` (LDS: 128 bf16 of the key, then 128 of the
// value), piece by piece, so that few registers are live at a time.
__device__ __forceinline__ void inject_entry(KFrag& ka, VFrag& va, int rr, const uint16_t* rows, int lane) {
  const int j = lane & 15, kg = lane >> 4;
  const int tt = rr >> 4;
  const bool krow = j == (rr & 15);
#pragma unroll
  for (int s = 0; s < 4; ++s) {
    const u32x4 kn = *reinterpret_cast<const u32x4*>(rows + 32 * s + 8 * kg);
#pragma unroll
    for (int h = 0; h < 2; ++h)
      if (krow && h == tt) ka.k[h * 4 + s] = kn;
  }
  const bool vrow = kg == ((rr & 15) >> 2);
  const int e = tt * 4 + (rr & 3);
#pragma unroll
  for (int dt = 0; dt < 8; ++dt) {
    const uint32_t vn = rows[kDim + 16 * dt + j];
#pragma unroll
    for (int wi = 0; wi < 4; ++wi) {
      const uint32_t old = va.v[dt][wi];
      const uint32_t nw = (e & 1) ? ((old & 0x0000FFFFu) | (vn << 16)) : ((old & 0xFFFF0000u) | vn);
      va.v[dt][wi] = (vrow && wi == (e >> 1)) ? nw : old;
    }
  }
}

template <int kW, int kSplit>
__global__ __launch_bounds__(64 * kW, 3) void layer_scan_kernel(Dev d, int unit_begin, const uint16_t* __restrict__ q,
                                                                const uint16_t* __restrict__ k_new,
                                                                const uint16_t* __restrict__ v_new, void* out, int layer) {
  constexpr int kT = 64 * kW;
  constexpr int kSpanBlk = kChunkBlocks / kSplit, kSpan = kSpanBlk * kBlk;      // blocks and entries one wavefront takes
  __shared__ float s_lg[kW][kMaxGroup * kLgRow];
  __shared__ float s_m[kW][kMaxGroup], s_l[kW][kMaxGroup];
  __shared__ float s_acc[kW][kMaxGroup * kDim];
  __shared__ float s_w[2 * kMaxChunks * kMaxGroup], s_M[kMaxGroup], s_L[kMaxGroup];
  __shared__ __align__(16) uint16_t s_new[kW][2 * kDim];
  __shared__ int s_last;
  const int tid = threadIdx.x, lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int urel = blockIdx.x, u = unit_begin + urel, cg = blockIdx.y;
  const int G = d.G;
  const int n_old = d.n[u];
  // this wavefront's span lies in one pool segment (asked for beside the length: neither waits for the other)
  const int c = cg * kW + w;
  const int my_seg = d.tbl[(size_t)u * d.max_seg + min(c / kSplit, d.max_seg - 1)];
  const bool full = n_old >= unit_cap(d, u);
  const int n = n_old + (full ? 0 : 1);
  const int nch = (n + kSpan - 1) / kSpan;          // spans of the unit
  if (cg == 0 && tid == 0) {
    if (urel == 0) d.layer_ts[2 * layer] = d.sc[SC_T];      // the bookkeeping runs later, perhaps after the time has moved on
    if (full) atomicOr(&d.sc[SC_STATUS], 1);
  }
  if (cg * kW >= nch) return;
  const int nwg = (nch + kW - 1) / kW;
  const int j = lane & 15, kg = lane >> 4;
  const bool head_lane = j < G;
  f32x4 acc[8];
#pragma unroll
  for (int dt = 0; dt < 8; ++dt) acc[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
  float m_run = -INFINITY, l_run = 0.f;
  if (c < nch) {
    const int e0 = c * kSpan;
    const int s0 = (c % kSplit) * kSpan;                                  // the span's first slot within its segment
    const int nv = min(n - e0, kSpan);
    const int nb = (nv + kBlk - 1) / kBlk;
    const bool inject = !full && n_old >= e0 && n_old < e0 + kSpan;      // the new entry is then the span's last: entry nv - 1
    const size_t off = (size_t)my_seg * kSegElems + (size_t)(c % kSplit) * kSpanBlk * kBlkElems + lane * 8;
    const uint16_t* kcur = d.K + off;
    const uint16_t* vcur = d.V + off;
    KFrag ka;
    VFrag va;
    load_k(ka, kcur);
    load_v(va, vcur);
    bf16x8 qv[4];
    {
      const uint16_t* qrow = q + ((size_t)urel * G + (head_lane ? j : 0)) * kDim + 8 * kg;
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        u32x4 x = *reinterpret_cast<const u32x4*>(qrow + 32 * s);
        if (!head_lane) x = u32x4{0u, 0u, 0u, 0u};
        qv[s] = as_bf16x8(x);
      }
    }
    // The new entry's rows wait in LDS for their block's turn (the span's last): held in registers through the
    // loop they would cost the kernel a third wavefront per SIMD.  They also go into the cache, where the next
    // step finds them.
    if (inject) {
      const int row = s0 + n_old - e0;                          // n_old lies in this span
      if (lane < 32) {
        const int piece = lane & 15;
        const uint16_t* src = (lane < 16 ? k_new : v_new) + (size_t)urel * kDim + piece * 8;
        const u32x4 x = *reinterpret_cast<const u32x4*>(src);
        *reinterpret_cast<u32x4*>(&s_new[w][(lane < 16 ? 0 : kDim) + piece * 8]) = x;
        if (lane < 16) *reinterpret_cast<u32x4*>(d.K + (size_t)my_seg * kSegElems + k_offset(row, piece * 8)) = x;
      }
      uint16_t* vdst = d.V + (size_t)my_seg * kSegElems;
      vdst[v_offset(row, lane)] = v_new[(size_t)urel * kDim + lane];
      vdst[v_offset(row, lane + 64)] = v_new[(size_t)urel * kDim + lane + 64];
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    }
    float* lds_lg = s_lg[w];
    float* lg_dst = d.logits + ((size_t)u * d.cap + (size_t)e0) * G + 4 * min(lane, 8 * G - 1);
    // one block ahead, as in scan_kernel (two ahead is slower here as well); the loads stay unconditional (the
    // last block is read twice), so that the waits the compiler inserts are exact
    for (int blk = 0; blk < nb; ++blk) {
      const bool last = blk + 1 == nb;
      const size_t nxt = (size_t)(last ? blk : blk + 1) * kBlkElems;
      if (last && inject) {
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        inject_entry(ka, va, (n_old - e0) & 31, s_new[w], lane);
      }
      float sv[8];
      scan_qk(ka, qv, sv, d.scale_log2e, blk * kBlk, nv, lds_lg, kLgRow, lg_dst, G, lane);
      load_k(ka, kcur + nxt);
      scan_pv(sv, va, acc, m_run, l_run, lane);
      load_v(va, vcur + nxt);
    }
    l_run += __shfl_xor(l_run, 16);
    l_run += __shfl_xor(l_run, 32);
  }
  // ---- the workgroup's four states into one
  if (head_lane && kg == 0) {
    s_m[w][j] = m_run;
    s_l[w][j] = l_run;
  }
  if (c < nch) {
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int head = 4 * kg + v;
      if (head < G) {
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) s_acc[w][head * kDim + 16 * dt + j] = acc[dt][v];
      }
    }
  }
  __syncthreads();
  const size_t slot0 = (size_t)u * d.slots;
  constexpr int kPer = (kMaxGroup * kDim) / kT;      // (head, dim) pairs per thread
  float o[kPer], Mg[kPer], Lg[kPer];
#pragma unroll
  for (int k = 0; k < kPer; ++k) {
    const int e = tid + k * kT, g = e >> 7;
    o[k] = 0.f;
    Mg[k] = -INFINITY;
    Lg[k] = 0.f;
    if (g < G) {
      float M = -INFINITY;
#pragma unroll
      for (int ww = 0; ww < kW; ++ww) M = fmaxf(M, s_m[ww][g]);
#pragma unroll
      for (int ww = 0; ww < kW; ++ww) {
        const float m = s_m[ww][g];
        if (m > -INFINITY) {
          const float wt = fast_exp2(m - M);
          o[k] += s_acc[ww][e] * wt;
          Lg[k] += s_l[ww][g] * wt;
        }
      }
      Mg[k] = M;
    }
  }
  auto write_out = [&](int k, float val, float M, float L) {
    const int e = tid + k * kT, g = e >> 7, dim = e & 127;
    const float inv = 1.0f / L;
    const float ov = val * inv;
    const size_t oi = ((size_t)urel * G + g) * kDim + dim;
    if (d.out_bf16)
      reinterpret_cast<__bf16*>(out)[oi] = (__bf16)ov;
    else
      reinterpret_cast<float*>(out)[oi] = ov;
    if (dim == 0) {
      d.msum[((size_t)u * kMaxGroup + g) * 2] = M;
      d.msum[((size_t)u * kMaxGroup + g) * 2 + 1] = inv;
    }
  };
  if (nwg == 1) {
#pragma unroll
    for (int k = 0; k < kPer; ++k)
      if (((tid + k * kT) >> 7) < G) write_out(k, o[k], Mg[k], Lg[k]);
    return;
  }
  // ---- one partial per workgroup; the workgroup that publishes the unit's last one merges them
#pragma unroll
  for (int k = 0; k < kPer; ++k) {
    const int e = tid + k * kT, g = e >> 7, dim = e & 127;
    if (g < G) {
      put<true>(&d.partial[((slot0 + cg) * G + g) * kDim + dim], o[k]);
      if (dim == 0) {
        put<true>(&d.ml[((slot0 + cg) * G + g) * 2], Mg[k]);
        put<true>(&d.ml[((slot0 + cg) * G + g) * 2 + 1], Lg[k]);
      }
    }
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");       // the partial before the count (coherent stores: completed is enough)
  __syncthreads();
  if (tid == 0) {
    const int lastone = atomicAdd(&d.arrive[u], 1) == nwg - 1;
    if (lastone) __hip_atomic_store(&d.arrive[u], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    s_last = lastone;
  }
  __syncthreads();
  if (!s_last) return;
  // the partials' values are asked for first, kRound partials at a time; their maxima and sums go through LDS,
  // where every head's overall maximum, the partials' weights and the sum's reciprocal are formed once
  constexpr int kRound = 32 / kPer < 8 ? 32 / kPer : 8;
  static_assert(kW >= kSplit, "a unit has one partial slot per chunk");
  float x[kRound][kPer];
  auto request = [&](int r0) {
#pragma unroll
    for (int i = 0; i < kRound; ++i) {
      const size_t sl = slot0 + min(r0 + i, nwg - 1);
#pragma unroll
      for (int k = 0; k < kPer; ++k) {
        const int e = tid + k * kT, g = e >> 7, dim = e & 127;
        x[i][k] = get_coherent(&d.partial[(sl * G + min(g, G - 1)) * kDim + dim]);
      }
    }
  };
  request(0);
  float* sW = s_w;
  float* sL = s_w + kMaxChunks * kMaxGroup;
  for (int i = tid; i < nwg * kMaxGroup; i += kT) {
    const int sidx = i >> 3, g = i & 7;
    const float* mlp = d.ml + ((slot0 + sidx) * G + min(g, G - 1)) * 2;
    const float m = get_coherent(mlp), l = get_coherent(mlp + 1);
    sW[i] = g < G ? m : -INFINITY;
    sL[i] = g < G ? l : 0.f;
  }
  __syncthreads();
  if (tid < kMaxGroup) {
    float M = -INFINITY;
    for (int r = 0; r < nwg; ++r) M = fmaxf(M, sW[r * kMaxGroup + tid]);
    s_M[tid] = M;
  }
  __syncthreads();
  for (int i = tid; i < nwg * kMaxGroup; i += kT) {
    const float m = sW[i];
    sW[i] = m > -INFINITY ? fast_exp2(m - s_M[i & 7]) : 0.f;
  }
  __syncthreads();
  if (tid < kMaxGroup) {
    float L = 0.f;
    for (int r = 0; r < nwg; ++r) L += sL[r * kMaxGroup + tid] * sW[r * kMaxGroup + tid];
    s_L[tid] = L;
  }
  __syncthreads();
  float val[kPer];
#pragma unroll
  for (int k = 0; k < kPer; ++k) val[k] = 0.f;
  for (int r0 = 0; r0 < nwg; r0 += kRound) {
#pragma unroll
    for (int i = 0; i < kRound; ++i) {
      if (r0 + i < nwg) {
#pragma unroll
        for (int k = 0; k < kPer; ++k) {
          const float wt = sW[(r0 + i) * kMaxGroup + ((tid + k * kT) >> 7)];
          if (wt != 0.f) val[k] += x[i][k] * wt;
        }
      }
    }
    if (r0 + kRound < nwg) request(r0 + kRound);
  }
#pragma unroll
  for (int k = 0; k < kPer; ++k) {
    const int g = (tid + k * kT) >> 7;
    if (g < G) write_out(k, val[k], s_M[g], s_L[g]);
  }
}

// The step's time moves on after the last layer (the single-layer scan above leaves the step scalars alone).
__global__ void advance_kernel(Dev d) {
  if (threadIdx.x == 0 && blockIdx.x == 0) {
    d.sc[SC_T] = d.sc[SC_T] + 1;
    d.sc[SC_WINDOW_STEPS] = d.sc[SC_WINDOW_STEPS] + 1;
  }
}

// ------------------------------------------------------------------ eviction
__device__ __forceinline__ u64 evict_key(float tmp, int pos) {
  // ascending key order = eviction order: lower score first, then higher position
  return ((u64)__float_as_uint(tmp) << 32) | (u64)(uint32_t)(~pos);
}

// One wavefront moves the entry in slot `src` to slot `dst` (both of unit
// base slot `base`); dst's position goes to src, flagged as evicted.
__device__ __forceinline__ void move_entry(const Dev& d, Slots base, int src, int dst, int lane) {
  uint16_t* K = d.K;
  uint16_t* V = d.V;
  if (lane < 16)
    *reinterpret_cast<u32x4*>(K + base.k(dst, lane * 8)) = *reinterpret_cast<const u32x4*>(K + base.k(src, lane * 8));
  V[base.v(dst, lane)] = V[base.v(src, lane)];
  V[base.v(dst, lane + 64)] = V[base.v(src, lane + 64)];
  if (lane == 0) {
    d.crf[base + dst] = d.crf[base + src];
    d.tau[base + dst] = d.tau[base + src];
    const int ps = d.pos[base + src], pd = d.pos[base + dst];
    d.pos[base + dst] = ps;
    d.pos[base + src] = pd;
    d.flags[base + dst] = d.flags[base + src];
    d.flags[base + src] = FLAG_SLIP;
  }
}

// Up to four moves at once by one wavefront: move r0 + m takes the entry in slot lst[lst_cap - 1 - (r0 + m)]
// to slot lst[r0 + m] (m < count), as move_entry does, but every load is issued before the first store, so
// the moves' memory round trips overlap.  Lane l does the key piece l & 15 of move l >> 4; all lanes do two
// value elements of every move; lanes 0..3 do the per-slot state of moves 0..3.
__device__ __forceinline__ void move_entries4(const Dev& d, Slots base, const int* lst, int lst_cap, int r0, int count, int lane) {
  uint16_t* K = d.K;
  uint16_t* V = d.V;
  const int mk = lane >> 4;
  int src[4], dst[4];
#pragma unroll
  for (int m = 0; m < 4; ++m) {
    const int mm = min(m, count - 1);
    src[m] = lst[lst_cap - 1 - (r0 + mm)];
    dst[m] = lst[r0 + mm];
  }
  const int ks = mk == 0 ? src[0] : mk == 1 ? src[1] : mk == 2 ? src[2] : src[3];
  const int kd = mk == 0 ? dst[0] : mk == 1 ? dst[1] : mk == 2 ? dst[2] : dst[3];
  const u32x4 kx = *reinterpret_cast<const u32x4*>(K + base.k(ks, (lane & 15) * 8));
  uint16_t v0[4], v1[4];
#pragma unroll
  for (int m = 0; m < 4; ++m) {
    v0[m] = V[base.v(src[m], lane)];
    v1[m] = V[base.v(src[m], lane + 64)];
  }
  float crf = 0.f;
  int tau = 0, ps = 0, pd = 0;
  uint8_t fl = 0;
  const int ms = lane == 0 ? src[0] : lane == 1 ? src[1] : lane == 2 ? src[2] : src[3];
  const int md = lane == 0 ? dst[0] : lane == 1 ? dst[1] : lane == 2 ? dst[2] : dst[3];
  if (lane < count) {
    crf = d.crf[base + ms];
    tau = d.tau[base + ms];
    ps = d.pos[base + ms];
    pd = d.pos[base + md];
    fl = d.flags[base + ms];
  }
  if (mk < count) *reinterpret_cast<u32x4*>(K + base.k(kd, (lane & 15) * 8)) = kx;
#pragma unroll
  for (int m = 0; m < 4; ++m) {
    if (m < count) {
      V[base.v(dst[m], lane)] = v0[m];
      V[base.v(dst[m], lane + 64)] = v1[m];
    }
  }
  if (lane < count) {
    d.crf[base + md] = crf;
    d.tau[base + md] = tau;
    d.pos[base + md] = ps;
    d.pos[base + ms] = pd;
    d.flags[base + md] = fl;
    d.flags[base + ms] = FLAG_SLIP;
  }
}

// Eviction of exactly one entry: the last slot's entry moves into the victim's
// slot `dst`, whose position goes to the last slot, flagged as evicted.  The K
// row, the V row and the per-slot state are handled by different wavefronts;
// the state comes from sh[1..4] = {CRF bits, tau, position} of the last slot's
// entry and the victim's position, so no per-slot array is read.
// The K and V rows of the slot that will move are read ahead of time (load_row, by the wavefronts that
// will store them), so that the eviction itself only stores.
struct EntryRow {
  u32x4 k;             // lanes 0..15 of wavefront 0: 8 dims of the K row each
  uint16_t v0, v1;     // wavefront 1 (0 if there is only one): dims lane and lane + 64 of the V row
};

template <int NT = kThreads>
__device__ __forceinline__ EntryRow load_row(const Dev& d, Slots base, int src, int tid) {
  const int wave = tid >> 6, lane = tid & 63;
  constexpr int W = NT / 64;
  const uint16_t* K = d.K;
  const uint16_t* V = d.V;
  EntryRow r{{0u, 0u, 0u, 0u}, 0, 0};
  if (wave == 0 && lane < 16) r.k = *reinterpret_cast<const u32x4*>(K + base.k(src, lane * 8));
  if (wave == (W > 1 ? 1 : 0)) {
    r.v0 = V[base.v(src, lane)];
    r.v1 = V[base.v(src, lane + 64)];
  }
  return r;
}

template <int NT = kThreads>
__device__ __forceinline__ void evict_one(const Dev& d, Slots base, int src, int dst, const int* sh, int tid, const EntryRow& row) {
  const int wave = tid >> 6, lane = tid & 63;
  constexpr int W = NT / 64;
  uint16_t* K = d.K;
  uint16_t* V = d.V;
  if (dst != src) {
    if (wave == 0 && lane < 16) *reinterpret_cast<u32x4*>(K + base.k(dst, lane * 8)) = row.k;
    if (wave == (W > 1 ? 1 : 0)) {
      V[base.v(dst, lane)] = row.v0;
      V[base.v(dst, lane + 64)] = row.v1;
    }
  }
  if (wave == (W > 2 ? 2 : 0) && lane == 32) {
    if (dst != src) {
      d.crf[base + dst] = __int_as_float(sh[1]);
      d.tau[base + dst] = sh[2];
      d.pos[base + dst] = sh[3];
    }
    d.pos[base + src] = sh[4];                 // the victim's position (the last slot's own if that is the victim)
    d.flags[base + src] = FLAG_SLIP;
  }
}

// Per-entry LDS values (mean weight, then CRF_temp) are reached through an
// accessor: a plain array in the finish kernel, a view into the logits tile in
// the fused unit kernel.
struct ValLinear {
  float* p;
  __device__ __forceinline__ float& operator()(int i) const { return p[i]; }
};

// Alg. 1 Step 4 for one unit with n > B.  val(i) = CRF_temp of slot i (LDS),
// evm = LDS bit mask of n bits, lst = LDS scratch of lst_cap >= n ints that may
// overlap the storage behind `val` (the scores are dead by the time it is used).
template <class Val, int NT = kThreads>
__device__ __forceinline__ void evict_phase(const Dev& d, int u, Slots base, int n, int B, Val val, uint32_t* evm, int* lst, int lst_cap, RedBuf& rb,
                            int& phase, int* sh, int tid) {
  const int lane = tid & 63, wave = tid >> 6;
  const int k = n - B;
  if (k == 1) {
    u64 best = ~0ull;
    int best_i = -1;
    for (int i0 = tid; i0 < n; i0 += 4 * NT) {
      int ps[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int i = i0 + r * NT;
        ps[r] = i < n ? d.pos[base + i] : 0;
      }
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int i = i0 + r * NT;
        if (i < n) {
          const u64 key = evict_key(val(i), ps[r]);
          if (key < best) {
            best = key;
            best_i = i;
          }
        }
      }
    }
    const u64 gbest = block_min_u64<NT>(best, rb, phase, tid);
    if (best == gbest && best_i >= 0) sh[0] = best_i;     // keys are unique: one writer
    block_sync<NT>(rb);
    const int e = sh[0];
    if (wave == 0) {
      if (e != n - 1) {
        move_entry(d, base, n - 1, e, lane);
      } else if (lane == 0) {
        d.flags[base + e] = FLAG_SLIP;
      }
    }
  } else {
    // The k smallest keys (score, then higher position first) in two stages, two bits per round (the three
    // candidates' counts are nested, and they are small integers, exact as floats).  Stage 1: S = the k-th
    // smallest score pattern, from the scores in LDS alone.  Stage 2, only if the entries equal to S are
    // not all evicted: which of them, by position; only those entries' positions are read.
    uint32_t S = 0;
    for (int bit = 31; bit >= 1; bit -= 2) {
      const uint32_t c1 = S | (1u << (bit - 1)), c2 = S | (1u << bit), c3 = c1 | c2;
      float n1 = 0.f, n2 = 0.f, n3 = 0.f;
      for (int i = tid; i < n; i += NT) {
        const uint32_t b = __float_as_uint(val(i));
        n1 += b < c1 ? 1.f : 0.f;
        n2 += b < c2 ? 1.f : 0.f;
        n3 += b < c3 ? 1.f : 0.f;
      }
      block_sum3_f32<NT>(n1, n2, n3, rb, phase, tid);
      const float kf = (float)k;
      S = n3 < kf ? c3 : n2 < kf ? c2 : n1 < kf ? c1 : S;          // the largest pattern with fewer than k scores below it
    }
    float below = 0.f, equal = 0.f, unused = 0.f;
    for (int i = tid; i < n; i += NT) {
      const uint32_t b = __float_as_uint(val(i));
      below += b < S ? 1.f : 0.f;
      equal += b == S ? 1.f : 0.f;
    }
    block_sum3_f32<NT>(below, equal, unused, rb, phase, tid);
    const int r = k - (int)below;                                  // of the entries equal to S, the r highest positions go
    uint32_t P = 0xFFFFFFFFu;                                      // ... those with ~position <= P
    if (r < (int)equal) {
      P = 0;
      for (int bit = 31; bit >= 1; bit -= 2) {
        const uint32_t c1 = P | (1u << (bit - 1)), c2 = P | (1u << bit), c3 = c1 | c2;
        float n1 = 0.f, n2 = 0.f, n3 = 0.f;
        for (int i = tid; i < n; i += NT) {
          if (__float_as_uint(val(i)) == S) {
            const uint32_t np = ~(uint32_t)d.pos[base + i];
            n1 += np < c1 ? 1.f : 0.f;
            n2 += np < c2 ? 1.f : 0.f;
            n3 += np < c3 ? 1.f : 0.f;
          }
        }
        block_sum3_f32<NT>(n1, n2, n3, rb, phase, tid);
        const float rf = (float)r;
        P = n3 < rf ? c3 : n2 < rf ? c2 : n1 < rf ? c1 : P;
      }
    }
    const int words = (n + 31) >> 5;
    for (int w = tid; w < words; w += NT) evm[w] = 0u;
    block_sync<NT>(rb);
    for (int i = tid; i < n; i += NT) {
      const uint32_t b = __float_as_uint(val(i));
      if (b < S || (b == S && (P == 0xFFFFFFFFu || ~(uint32_t)d.pos[base + i] <= P))) atomicOr(&evm[i >> 5], 1u << (i & 31));
    }
    block_sync<NT>(rb);
    // holes = evicted slots below B, movers = surviving slots at or above B (equal counts)
    const int wpt = (words + NT - 1) / NT;
    const int w0 = min(words, tid * wpt), w1 = min(words, w0 + wpt);
    uint32_t holes = 0, movers = 0;
    for (int w = w0; w < w1; ++w) {
      const uint32_t e = evm[w];
      const int s0 = w << 5;
      const uint32_t below = (B >= s0 + 32) ? 0xFFFFFFFFu : (B <= s0 ? 0u : ((1u << (B - s0)) - 1u));
      const uint32_t valid = (n >= s0 + 32) ? 0xFFFFFFFFu : ((1u << (n - s0)) - 1u);
      holes += __popc(e & below);
      movers += __popc(~e & ~below & valid);
    }
    const uint32_t packed = holes | (movers << 16);
    uint32_t incl = packed;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const uint32_t y = __shfl_up(incl, o);
      if (lane >= o) incl += y;
    }
    if (lane == 63) sh[4 + wave] = (int)incl;
    block_sync<NT>(rb);
    uint32_t prefix = 0, total = 0;
#pragma unroll
    for (int w = 0; w < NT / 64; ++w) {
      if (w < wave) prefix += (uint32_t)sh[4 + w];
      total += (uint32_t)sh[4 + w];
    }
    const uint32_t excl = incl - packed + prefix;
    int hrank = (int)(excl & 0xFFFFu), mrank = (int)(excl >> 16);
    const int h = (int)(total & 0xFFFFu);
    for (int w = w0; w < w1; ++w) {
      const uint32_t e = evm[w];
      const int s0 = w << 5;
      const uint32_t below = (B >= s0 + 32) ? 0xFFFFFFFFu : (B <= s0 ? 0u : ((1u << (B - s0)) - 1u));
      const uint32_t valid = (n >= s0 + 32) ? 0xFFFFFFFFu : ((1u << (n - s0)) - 1u);
      uint32_t hm = e & below, mm = ~e & ~below & valid;
      while (hm) {
        lst[hrank++] = s0 + __builtin_ctz(hm);
        hm &= hm - 1;
      }
      while (mm) {
        lst[lst_cap - 1 - (mrank++)] = s0 + __builtin_ctz(mm);
        mm &= mm - 1;
      }
    }
    block_sync<NT>(rb);
    // evicted entries that already sit at or above B just get their flag
    for (int i = B + tid; i < n; i += NT)
      if ((evm[i >> 5] >> (i & 31)) & 1u) d.flags[base + i] = FLAG_SLIP;
    // moves, four per wavefront at a time: all loads of a batch are issued before its stores
    for (int r0 = 4 * wave; r0 < h; r0 += 4 * (NT / 64)) move_entries4(d, base, lst, lst_cap, r0, min(4, h - r0), lane);
  }
  if (tid == 0) {
    d.n[u] = B;
    d.nev[u] = k;
  }
}

// ------------------------------------------------------------------ finish
// Ends a kernel that must leave the step scalars consistent: the last block
// to arrive resets the work list and, if asked, advances time.  No fence: the
// last block reads nothing the others wrote (the scalars it updates are read-only
// during the launch, and every claim on the queue has returned before its
// workgroup gets here); the end of the kernel publishes what it writes.  A
// device-scope fence here would write back a whole L2 once per workgroup.
__device__ __forceinline__ void step_epilogue(const Dev& d, int t, int advance, int tid, int queue_reset = -1) {
  __syncthreads();
  if (tid == 0) {
    const int prev = atomicAdd(&d.sc[SC_DONE], 1);
    if (prev == (int)gridDim.x - 1) {
      d.sc[SC_DONE] = 0;
      d.sc[SC_CLAIM] = 0;
      d.sc[SC_CLAIM + 1] = 0;
      d.sc[SC_SEQ] = d.sc[SC_SEQ] + 1;
      if (queue_reset >= 0) d.sc[SC_QUEUE] = queue_reset;
      if (advance) {
        d.sc[SC_T] = t + 1;
        d.sc[SC_WINDOW_STEPS] = d.sc[SC_WINDOW_STEPS] + 1;
      }
    }
  }
}

// Merge the scan partials of unit u (the slots stamped by this launch).  Leaves
// sM[g] (global max) and sInv[g] (1 / softmax denominator) in LDS and, if `out`
// is given, writes the attention output.
__device__ __forceinline__ void merge_partials(const Dev& d, int u, int urel, int nch, int seq, float* sM, float* sInv,
                                               float* sW, void* out, int tid) {
  const int G = d.G;
  const size_t slot0 = (size_t)u * d.slots;
  const int ns = nch + 1;
  float* sL = sW + (kMaxChunks + 1) * kMaxGroup;      // second half of the caller's array: the slots' sums
  // running maxima and sums of the live slots (m = -inf, l = 0 for the others), one 8-byte read each
  for (int i = tid; i < ns * kMaxGroup; i += kThreads) {
    const int sidx = i >> 3, g = i & 7;
    // both reads are issued at once (the slot's record exists whether or not this launch wrote it)
    const int stamp = d.stamp[slot0 + sidx];
    const float2 ml = *reinterpret_cast<const float2*>(d.ml + ((slot0 + sidx) * G + min(g, G - 1)) * 2);
    const bool live = g < G && stamp == seq;
    sW[i] = live ? ml.x : -INFINITY;
    sL[i] = live ? ml.y : 0.f;
  }
  __syncthreads();
  if (tid < G) {
    const int g = tid;
    float M = -INFINITY;
    for (int sidx = 0; sidx < ns; ++sidx) M = fmaxf(M, sW[sidx * kMaxGroup + g]);
    sM[g] = M;
  }
  __syncthreads();
  // weights: sW[s * 8 + g] = exp2(m_s - M) for live slots, 0 for the others
  for (int i = tid; i < ns * kMaxGroup; i += kThreads) {
    const int g = i & 7;
    const float m = sW[i];
    sW[i] = (g < G && m > -INFINITY) ? fast_exp2(m - sM[g]) : 0.f;
  }
  __syncthreads();
  if (tid < G) {
    const int g = tid;
    float Lsum = 0.f;
    for (int sidx = 0; sidx < ns; ++sidx) {
      const float w = sW[sidx * kMaxGroup + g];
      if (w != 0.f) Lsum += sL[sidx * kMaxGroup + g] * w;
    }
    sInv[g] = 1.0f / Lsum;
  }
  __syncthreads();
  if (out) {
    for (int idx = tid; idx < G * kDim; idx += kThreads) {
      const int g = idx >> 7, dim = idx & 127;
      float o = 0.f;
      // eight slots' partials are requested at once (dead slots hold stale data: read, never used)
      for (int s0 = 0; s0 < ns; s0 += 8) {
        float x[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) x[k] = d.partial[((slot0 + min(s0 + k, ns - 1)) * G + g) * kDim + dim];
#pragma unroll
        for (int k = 0; k < 8; ++k) {
          const float w = s0 + k < ns ? sW[(s0 + k) * kMaxGroup + g] : 0.f;
          if (w != 0.f) o += x[k] * w;
        }
      }
      o *= sInv[g];
      const size_t oi = ((size_t)urel * G + g) * kDim + dim;
      if (d.out_bf16)
        reinterpret_cast<__bf16*>(out)[oi] = (__bf16)o;
      else
        reinterpret_cast<float*>(out)[oi] = o;
    }
  }
}


// lambda^delta from the decay table: its first s_tab_n entries sit in LDS, the rest (long tables: lambda
// close to 1) in global memory.  Written as two loads in two address spaces on purpose: a conditional
// expression over the two pointers becomes one flat load, which waits for every vector-memory
// operation in flight.
__device__ __forceinline__ float decay_far(const Dev& d, int delta) {
  float far = d.tab[delta];
  asm volatile("" : "+v"(far));          // the wait for this load stays inside the caller's branch: placed after
  return far;                            // the branch it would be a wait for every vector-memory operation
}                                        // in flight, executed for every entry
__device__ __forceinline__ float decay_of(const Dev& d, int delta, const float* s_tab, int s_tab_n) {
  float dec = s_tab[min(delta, s_tab_n - 1)];
  asm volatile("" : "+v"(dec));          // pins the LDS load: otherwise the two loads are merged again
  if (delta >= s_tab_n) dec = decay_far(d, delta);
  return dec;
}
// Four lookups at once: the LDS reads are issued together and waited for once.
__device__ __forceinline__ void decay4_of(const Dev& d, const int (&delta)[4], const float* s_tab, int s_tab_n, float (&dec)[4]) {
#pragma unroll
  for (int e = 0; e < 4; ++e) dec[e] = s_tab[min(delta[e], s_tab_n - 1)];
#pragma unroll
  for (int e = 0; e < 4; ++e) asm volatile("" : "+v"(dec[e]));
#pragma unroll
  for (int e = 0; e < 4; ++e)
    if (delta[e] >= s_tab_n) dec[e] = decay_far(d, delta[e]);
}

// Where a unit's scaled logits lie in memory: per block of 32 entries a group of rows [row][32], of which
// the G rows from `p` on are the unit's heads (the scan kernel leaves exactly G rows per block; the prompt
// replay leaves 16, G of them per query).
struct LgView {
  const float* p;      // head 0, entry 0
  int blk_stride;      // floats from one block to the next
};
__device__ __forceinline__ LgView unit_logits(const Dev& d, int u) {
  return LgView{d.logits + (size_t)u * d.G * d.cap, d.G * kBlk};
}

// Mean attention weight of every entry of a unit into val[0..n).
template <int NT = kThreads>
__device__ __forceinline__ void mean_weights(const Dev& d, LgView lv, int n, const float* sM, const float* sInv, float* val,
                                             int tid) {
  const int G = d.G;
  const float invG = 1.0f / (float)G;
  const float* lg = lv.p;
  for (int i0 = tid; i0 < n; i0 += 4 * NT) {
    float x[4][kMaxGroup];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int i = i0 + r * NT;
      const float* row = lg + (size_t)(i >> 5) * lv.blk_stride + (i & 31);
#pragma unroll
      for (int g = 0; g < kMaxGroup; ++g) x[r][g] = (i < n && g < G) ? row[g * kBlk] : -INFINITY;
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int i = i0 + r * NT;
      float a = 0.f;
#pragma unroll
      for (int g = 0; g < kMaxGroup; ++g)
        if (g < G) a += fast_exp2(x[r][g] - sM[g]) * sInv[g];
      if (i < n) val[i] = a * invG;
    }
  }
  __syncthreads();
}

// Alg. 1 Steps 1-3 for one unit: top-p hit set from the mean weights val(i),
// score update, flags.  Leaves CRF_temp in val(i) and returns the unit's
// aggregated CRF (2^-20 fixed point), summed over the block.  s_tab: the first
// s_tab_n entries of the decay table in LDS.
// Alg. 1 Step 1 as a rule: an entry of weight pattern b and position pe is hit if b > theta, or b == theta and
// (ties_all or pe <= pos_cut).  (The entry appended in the step is hit whatever its weight: the callers add that.)
struct HitRule {
  uint32_t theta;
  bool ties_all;
  int pos_cut;
  __device__ __forceinline__ bool operator()(uint32_t b, int pe) const { return (b > theta) | ((b == theta) & (ties_all | (pe <= pos_cut))); }
};

// Step 1 over weights in val(0 .. n - 1) (LDS), any n
template <class Val, int NT = kThreads>
__device__ __forceinline__ HitRule top_p_lds(const Dev& d, Slots base, int n, Val val, RedBuf& rb, int& phase, int tid) {
  uint32_t theta = 0;
  bool ties_all = true;
  int pos_cut = 0x7FFFFFFF;
  if (d.reward_mode == 0) {
    for (int bit = 30; bit >= 0; --bit) {
      const uint32_t cand = theta | (1u << bit);
      float part = 0.f;
      for (int i = tid; i < n; i += NT) {
        const float a = val(i);
        part += (__float_as_uint(a) >= cand) ? a : 0.f;
      }
      const float tot = block_sum_f32<NT>(part, rb, phase, tid);
      if (tot > d.top_p) theta = cand;
    }
    if (theta != 0) {
      // entries equal to the threshold: only as many as needed, lower positions first
      float above = 0.f;
      int ties = 0;
      for (int i = tid; i < n; i += NT) {
        const float a = val(i);
        const uint32_t b = __float_as_uint(a);
        above += (b > theta) ? a : 0.f;
        ties += (b == theta) ? 1 : 0;
      }
      above = block_sum_f32<NT>(above, rb, phase, tid);
      ties = block_sum_int<NT>(ties, rb, phase, tid);
      if (ties > 1) {
        const float th = __uint_as_float(theta);
        float c = above;
        int r = 0;
        do {
          c += th;
          ++r;
        } while (c <= d.top_p && r < ties);
        if (r < ties) {
          ties_all = false;
          int X = 0;   // r-th smallest position among the ties
          for (int bit = 30; bit >= 0; --bit) {
            const int trial = X | (1 << bit);
            int cnt = 0;
            for (int i = tid; i < n; i += NT)
              cnt += (__float_as_uint(val(i)) == theta && d.pos[base + i] < trial) ? 1 : 0;
            cnt = block_sum_int<NT>(cnt, rb, phase, tid);
            if (cnt < r) X = trial;
          }
          pos_cut = X;
        }
      }
    }
  }
  return HitRule{theta, ties_all, pos_cut};
}

template <class Val, int NT = kThreads>
__device__ __forceinline__ u64 lrfu_update(const Dev& d, int u, Slots base, int n, int t, Val val, const float* s_tab, int s_tab_n, RedBuf& rb,
                           int& phase, int tid) {
  // ---- Alg. 1 Step 1: top-p hit set as a threshold on the weight's bit pattern
  const HitRule rule = top_p_lds<Val, NT>(d, base, n, val, rb, phase, tid);
  const bool ties_all = rule.ties_all;

  // ---- Alg. 1 Steps 2-3: scores (4 entries per thread and round: loads, table lookups, then stores)
  const bool has_new = d.pos[base + (n - 1)] == t;
  const bool need_pos = d.reward_mode == 0 && !ties_all;
  u64 sfix = 0;
  for (int i0 = tid; i0 < n; i0 += 4 * NT) {
    float crf[4], dec[4];
    int tau[4], ps[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int i = i0 + r * NT;
      const bool ok = i < n;
      crf[r] = ok ? d.crf[base + i] : 0.f;
      tau[r] = ok ? d.tau[base + i] : t;
      ps[r] = (ok && need_pos) ? d.pos[base + i] : 0;
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      int delta = t - tau[r];
      delta = delta < 0 ? 0 : (delta > d.tab_last ? d.tab_last : delta);
      dec[r] = decay_of(d, delta, s_tab, s_tab_n);
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int i = i0 + r * NT;
      if (i < n) {
        const float a = val(i);
        bool hit, store;
        float reward;
        if (d.reward_mode == 0) {
          const uint32_t b = __float_as_uint(a);
          hit = rule(b, ps[r]);
          if (i == n - 1 && has_new) hit = true;
          store = hit;
          reward = hit ? 1.0f : 0.0f;
        } else {
          store = true;
          reward = a;
        }
        float tmp = __fadd_rn(__fmul_rn(dec[r], crf[r]), reward);
        if (tmp < FLT_MIN) tmp = 0.0f;
        if (store) {
          d.crf[base + i] = tmp;
          d.tau[base + i] = t;
        }
        val(i) = tmp;
        sfix += (u64)floorf(tmp * kFixedOne);
      }
    }
  }
  return block_sum_u64<NT>(sfix, rb, phase, tid);   // its barrier also completes val() for what follows
}

typedef int i32x4 __attribute__((ext_vector_type(4)));

// Register-resident bookkeeping: thread tid of NT owns R = 4 C entries, in C
// groups of four consecutive entries 4 (tid + c NT) .. + 3 (group c), so that
// every access to the per-entry arrays is a 16-byte one: the memory pipeline of
// a CU is shared with the streaming loads of the other workgroup and every
// instruction queues behind them, so the number of memory instructions, not
// their size, is what the latency of this phase depends on.

// Mean attention weights of this thread's groups from logits in global memory
// (per block of 32 entries: [head][32]); 0 beyond n.
template <int R, int NT = kThreads>
__device__ __forceinline__ void mean_weights_regs(const Dev& d, LgView lv, int n, const float* sM, const float* sInv,
                                                  float (&a)[R], int tid) {
  const int G = d.G;
  const float invG = 1.0f / (float)G;
  const float* lg = lv.p;
#pragma unroll
  for (int c = 0; c < R / 4; ++c) {
    const int e0 = 4 * (tid + c * NT);
    f32x4 x[kMaxGroup];
    const float* row = lg + (size_t)(e0 >> 5) * lv.blk_stride + (e0 & 31);
#pragma unroll
    for (int g = 0; g < kMaxGroup; ++g)
      x[g] = (e0 < n && g < G) ? *reinterpret_cast<const f32x4*>(row + g * kBlk) : f32x4{-INFINITY, -INFINITY, -INFINITY, -INFINITY};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      float acc = 0.f;
#pragma unroll
      for (int g = 0; g < kMaxGroup; ++g)
        if (g < G) acc += fast_exp2(x[g][e] - sM[g]) * sInv[g];
      a[4 * c + e] = (e0 + e < n) ? acc * invG : 0.f;
    }
  }
}

// CRF, tau and position of group c of thread tid.  The loads are unconditional
// (a select on their result would wait for them on the spot): a group beyond
// the unit reads the unit's last group instead, and nothing looks at the values
// of entries >= n.
template <int NT = kThreads>
__device__ __forceinline__ void load_meta(const Dev& d, Slots base, int n, int t, int c, int tid, f32x4& crf, i32x4& tau, i32x4& ps) {
  const int e0 = min(4 * (tid + c * NT), (max(n, 1) - 1) & ~3);
  const size_t s0 = base + e0;                 // four consecutive entries share a segment
  crf = *reinterpret_cast<const f32x4*>(d.crf + s0);
  tau = *reinterpret_cast<const i32x4*>(d.tau + s0);
  ps = *reinterpret_cast<const i32x4*>(d.pos + s0);
}

// Alg. 1 Steps 1-4 for a unit of n <= R NT entries with the weights in
// registers (a[4 c + e] = mean weight of entry 4 (tid + c NT) + e, 0 beyond n).
// Same decisions and arithmetic as lrfu_update + evict_phase.  The groups'
// CRF, tau and position pass through register arrays of CH groups: the caller
// has loaded the first CP of them (early enough that they have arrived), the
// rest of the first CH groups are loaded here, before the bisection, whose 31
// rounds hide their latency; further chunks of CH groups (large units only, to
// bound the registers) are loaded when their turn comes.  The hit mark of an entry is not stored: in the
// top-p mode it equals tau == t.  Evicting exactly one entry is done in place
// (the owners of the two entries involved pass their registers through `sh`);
// evicting more falls back to evict_phase (scores then go to val()).
struct NoHook {
  __device__ __forceinline__ void operator()() const {}
};

// The entry appended in this step when the caller has NOT written it to the cache (the fused kernel when
// exactly one entry will be evicted): logically it is the unit's last entry, index n - 1, with CRF 0,
// tau = t and position t; its key and value rows are the step's inputs.  Its per-slot state is supplied
// here instead of being read, and if it survives the eviction its rows go straight from the inputs into
// the victim's slot (one write instead of a write, a read and a write).  k_row == nullptr: the entry is in
// the cache like any other (or nothing was appended).
struct NewEntry {
  const uint16_t* k_row;    // 128 bf16, or nullptr
  const uint16_t* v_row;
};

template <int NT = kThreads>
__device__ __forceinline__ EntryRow load_row_input(const NewEntry& ne, int tid) {
  const int wave = tid >> 6, lane = tid & 63;
  constexpr int W = NT / 64;
  EntryRow r{{0u, 0u, 0u, 0u}, 0, 0};
  if (wave == 0 && lane < 16) r.k = *reinterpret_cast<const u32x4*>(ne.k_row + lane * 8);
  if (wave == (W > 1 ? 1 : 0)) {
    r.v0 = ne.v_row[lane];
    r.v1 = ne.v_row[lane + 64];
  }
  return r;
}

// Step 1 over weights in registers (a[4 c + e] = mean weight of entry 4 (tid + c NT) + e, 0 beyond n).  lst: 64 ints of
// LDS (lst_cap >= 64, or the short list is not used); sh: the callers' exchange words (5 .. 7 are used here).
// new_last_t >= 0: the unit's last entry is not in the cache and has this position.
// kList: candidates the short list may hold (64: one per lane of the wavefront that finishes the bisection;
// 128, 256: two or four per lane, for long units with flat weights, whose bucket holds more).
template <int R, int NT = kThreads, int kList = 64>
__device__ __forceinline__ HitRule top_p_regs(const Dev& d, Slots base, int n, const float (&a)[R], int* lst, int lst_cap, int new_last_t,
                                              RedBuf& rb, int& phase, int* sh, int tid) {
  uint32_t theta = 0;
  bool ties_all = true;
  int pos_cut = 0x7FFFFFFF;
  if (d.reward_mode == 0) {
    // largest pattern theta with sum{a >= theta} > p, two bits per round (one barrier each): the three
    // candidates' sums are nested, so the largest candidate that passes is what bit-by-bit bisection
    // would reach.  Bit 30 is never set: the weights are <= 1.
    auto round = [&](int bit) {
      const uint32_t c1 = theta | (1u << (bit - 1)), c2 = theta | (1u << bit), c3 = c1 | c2;
      float p1 = 0.f, p2 = 0.f, p3 = 0.f;
#pragma unroll
      for (int k = 0; k < R; ++k) {
        const uint32_t b = __float_as_uint(a[k]);
        p1 += (b >= c1) ? a[k] : 0.f;
        p2 += (b >= c2) ? a[k] : 0.f;
        p3 += (b >= c3) ? a[k] : 0.f;
      }
      block_sum3_f32<NT>(p1, p2, p3, rb, phase, tid);
      theta = p3 > d.top_p ? c3 : p2 > d.top_p ? c2 : p1 > d.top_p ? c1 : theta;
    };
    constexpr int kListBit = 17;        // the rounds for the bits above this one run over all entries
    int bit = 29;
    bool from_list = false;             // the tail ran on the short list, which also gave:
    int list_ties = 0;                  //   entries equal to theta
    float list_above = 0.f;             //   total weight of the entries above theta
    for (; bit > kListBit; bit -= 2) round(bit);
    // With the top 12 bits fixed, the weights that can still decide a candidate, those in
    // [theta, theta + 2^18), are usually a handful.  If at most kList, they are collected in LDS (in a fixed
    // order: by wavefront, register index, lane) and one wavefront finishes the bisection on them alone:
    // nine rounds without barriers over one register instead of R.
    {
      const uint32_t lo = theta > 1u ? theta : 1u, hi = theta + (2u << kListBit);
      const int lane = tid & 63, wave = tid >> 6;
      float ab = 0.f;
      int mine = 0;
#pragma unroll
      for (int k = 0; k < R; ++k) {
        const uint32_t b = __float_as_uint(a[k]);
        ab += (b >= hi) ? a[k] : 0.f;
        mine += (b >= lo && b < hi) ? 1 : 0;
      }
      ab = wave_sum_f32(ab);
      mine = wave_sum_i32(mine);
      if (lane == 0) *reinterpret_cast<f32x4*>(rb.t[phase][wave]) = f32x4{ab, __int_as_float(mine), 0.f, 0.f};
      block_sync<NT>(rb);
      float above_bucket = 0.f;
      int m = 0, off = 0;
#pragma unroll
      for (int w = 0; w < NT / 64; ++w) {
        const f32x4 q = *reinterpret_cast<const f32x4*>(rb.t[phase][w]);
        above_bucket += q[0];
        const int cw = __float_as_int(q[1]);
        off += w < wave ? cw : 0;
        m += cw;
      }
      phase ^= 1;
      if (m <= kList && lst_cap >= kList) {
#pragma unroll
        for (int k = 0; k < R; ++k) {
          const uint32_t b = __float_as_uint(a[k]);
          const bool in = b >= lo && b < hi;
          const unsigned long long mask = __ballot(in);
          const int r = off + (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
          if (in) lst[r] = (int)b;
          off += __popcll(mask);
        }
        block_sync<NT>(rb);
        if (wave == 0) {
          // One candidate per lane.  The largest pattern theta with sum{a >= theta} > p is a candidate's own
          // pattern: the largest one whose sum of candidates at least as large, on top of what lies above the
          // bucket, exceeds p (what the remaining rounds of the bisection would arrive at).  Every entry
          // equal to theta is in the list too, so the number of such ties and the weight above theta are
          // known here as well, without two more reductions over all entries.
          if constexpr (kList == 64) {
            const uint32_t bj = lane < m ? (uint32_t)lst[lane] : 0u;
            const float aj = __uint_as_float(bj);
            float sj = 0.f;
            for (int k = 0; k < m; ++k) {                       // m is uniform; candidates in list order
              const uint32_t bk = (uint32_t)__builtin_amdgcn_readlane((int)bj, k);
              sj += (bk >= bj) ? __uint_as_float(bk) : 0.f;
            }
            const uint32_t mine_ok = (lane < m && above_bucket + sj > d.top_p) ? bj : 0u;
            uint32_t th = mine_ok;
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) th = max(th, (uint32_t)__shfl_xor((int)th, o));
            if (th != 0u) theta = th;
            const int n_ties = __popcll(__ballot(lane < m && bj == theta));
            const float above_l = above_bucket + wave_sum_f32((lane < m && bj > theta) ? aj : 0.f);
            if (lane == 0) {
              sh[7] = (int)theta;
              sh[5] = n_ties;
              sh[6] = __float_as_int(above_l);
            }
          } else {
            // the same with kList / 64 candidates per lane (candidate lane + 64 c), the others read from LDS
            constexpr int kC = kList / 64;
            uint32_t bj[kC];
            float sj[kC];
#pragma unroll
            for (int c = 0; c < kC; ++c) {
              bj[c] = lane + 64 * c < m ? (uint32_t)lst[lane + 64 * c] : 0u;
              sj[c] = 0.f;
            }
            for (int k = 0; k < m; ++k) {                     // candidates in list order
              const uint32_t bk = (uint32_t)lst[k];
              const float ak = __uint_as_float(bk);
#pragma unroll
              for (int c = 0; c < kC; ++c) sj[c] += (bk >= bj[c]) ? ak : 0.f;
            }
            uint32_t th = 0u;
#pragma unroll
            for (int c = 0; c < kC; ++c) th = max(th, (lane + 64 * c < m && above_bucket + sj[c] > d.top_p) ? bj[c] : 0u);
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) th = max(th, (uint32_t)__shfl_xor((int)th, o));
            if (th != 0u) theta = th;
            int n_ties = 0;
            float mine_above = 0.f;
#pragma unroll
            for (int c = 0; c < kC; ++c) {
              const bool in = lane + 64 * c < m;
              n_ties += __popcll(__ballot(in && bj[c] == theta));
              mine_above += (in && bj[c] > theta) ? __uint_as_float(bj[c]) : 0.f;
            }
            const float above_l = above_bucket + wave_sum_f32(mine_above);
            if (lane == 0) {
              sh[7] = (int)theta;
              sh[5] = n_ties;
              sh[6] = __float_as_int(above_l);
            }
          }
        }
        block_sync<NT>(rb);
        theta = (uint32_t)sh[7];
        list_ties = sh[5];
        list_above = __int_as_float(sh[6]);
        from_list = true;
      } else {
        for (; bit >= 1; bit -= 2) round(bit);
      }
    }
    if (theta != 0) {
      float above = list_above;
      int ties = list_ties;
      if (!from_list) {
        above = 0.f;
        ties = 0;
#pragma unroll
        for (int k = 0; k < R; ++k) {
          const uint32_t b = __float_as_uint(a[k]);
          above += (b > theta) ? a[k] : 0.f;
          ties += (b == theta) ? 1 : 0;
        }
        above = block_sum_f32<NT>(above, rb, phase, tid);
        ties = block_sum_int<NT>(ties, rb, phase, tid);
      }
      if (ties > 1) {
        const float th = __uint_as_float(theta);
        float c = above;
        int r = 0;
        do {
          c += th;
          ++r;
        } while (c <= d.top_p && r < ties);
        if (r < ties) {
          ties_all = false;
          int X = 0;   // r-th smallest position among the ties (rare: positions are re-read from memory)
          for (int bit = 30; bit >= 0; --bit) {
            const int trial = X | (1 << bit);
            int cnt = 0;
            for (int k = 0; k < R; ++k) {
              const int i = 4 * (tid + (k >> 2) * NT) + (k & 3);
              if (__float_as_uint(a[k]) == theta && i < n && ((new_last_t >= 0 && i == n - 1) ? new_last_t : d.pos[base + i]) < trial) ++cnt;
            }
            cnt = block_sum_int<NT>(cnt, rb, phase, tid);
            if (cnt < r) X = trial;
          }
          pos_cut = X;
        }
      }
    }
  }
  return HitRule{theta, ties_all, pos_cut};
}

// `after_step1` runs once between Step 1 and the score update (the fused kernel
// picks up its queue claim there).
template <int R, int CH, int CP, class Val, int NT = kThreads, class Hook = NoHook>
__device__ __forceinline__ void lrfu_regs(const Dev& d, int u, Slots base, int n, int B, int t, float (&a)[R], f32x4 (&crf)[CH],
                                          i32x4 (&tau)[CH], i32x4 (&ps)[CH], Val val, bool evict, uint32_t* evm, int* lst,
                                          int lst_cap, const float* s_tab, int s_tab_n, RedBuf& rb, int& phase, int* sh,
                                          int tid, Hook after_step1 = Hook{}, NewEntry ne = NewEntry{nullptr, nullptr}) {
  constexpr int C = R / 4;
  static_assert(C % CH == 0 && CP <= CH, "groups come in chunks of CH");
  const bool new_in_regs = ne.k_row != nullptr;          // uniform; implies that exactly one entry is evicted below
#pragma unroll
  for (int c = CP; c < CH; ++c) load_meta<NT>(d, base, n, t, c, tid, crf[c], tau[c], ps[c]);
  // what the end of the step would otherwise wait for: the unit's running sum, and the last slot's rows
  // (the entry that moves if exactly one entry is evicted)
  const u64 window0 = d.window[u];
  const bool evict_single = evict && n - B == 1;
  EntryRow last_row{{0u, 0u, 0u, 0u}, 0, 0};
  if (evict_single) last_row = new_in_regs ? load_row_input<NT>(ne, tid) : load_row<NT>(d, base, n - 1, tid);
  // ---- Step 1: top-p hit set as a threshold on the weight's bit pattern
  const HitRule rule = top_p_regs<R, NT>(d, base, n, a, lst, lst_cap, new_in_regs ? t : -1, rb, phase, sh, tid);
  after_step1();
  // ---- Steps 2-3: scores; a[k] becomes CRF_temp.  The candidate for Step 4 (lowest score, then
  // highest position) is tracked on the way.
  u64 sfix = 0;
  u64 best = ~0ull;
  int best_i = -1;
#pragma unroll
  for (int cc = 0; cc < C; ++cc) {
    const int c = cc % CH;                  // register slot of group cc
    if (cc >= CH && c == 0) {               // next chunk of groups: its state is requested only now
      __builtin_amdgcn_sched_barrier(0);    // (and not earlier: hoisted, the chunks' registers would all be live at once)
#pragma unroll
      for (int k = 0; k < CH; ++k) load_meta<NT>(d, base, n, t, cc + k, tid, crf[k], tau[k], ps[k]);
    }
    // Straight-line, predicated code (selects instead of branches; entries beyond n compute on
    // whatever was loaded and are masked out of every result): branchy per-entry code ran at a small
    // fraction of the issue rate.
    const int e0 = 4 * (tid + cc * NT);
    f32x4 ncrf = crf[c];
    i32x4 ntau = tau[c];
    uint32_t stored = 0;                    // bit e: entry e0 + e gets a new (CRF, tau)
    const bool topp = d.reward_mode == 0;
    int delta4[4];
    float dec4[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) delta4[e] = min(max(t - tau[c][e], 0), d.tab_last);
    decay4_of(d, delta4, s_tab, s_tab_n, dec4);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int i = e0 + e;
      const bool ok = i < n;
      const bool fresh = new_in_regs & (i == n - 1);                 // the new entry, not in the cache: CRF 0, tau = position = t
      const int pe = fresh ? t : ps[c][e];
      const float w = a[4 * cc + e];
      const float dec = fresh ? 1.0f : dec4[e];
      const float crf_old = fresh ? 0.0f : crf[c][e];
      const uint32_t b = __float_as_uint(w);
      const bool hit = topp & (rule(b, pe) | ((i == n - 1) & (pe == t)));          // the entry appended this step is always hit
      const bool store = ok & (hit | !topp);
      const float reward = topp ? (hit ? 1.0f : 0.0f) : w;
      float tmp = __fadd_rn(__fmul_rn(dec, crf_old), reward);
      tmp = tmp < FLT_MIN ? 0.0f : tmp;
      ncrf[e] = store ? tmp : ncrf[e];
      ntau[e] = store ? t : ntau[e];
      stored |= (store ? 1u : 0u) << e;
      a[4 * cc + e] = ok ? tmp : 0.0f;
      // 2^-20 fixed point of the score: the scaling is exact, the split into two 32-bit halves too
      const float fx = floorf(tmp * kFixedOne);
      const uint32_t fhi = (uint32_t)(fx * 2.3283064365386963e-10f);
      const uint32_t flo = (uint32_t)(fx - (float)fhi * 4294967296.0f);
      sfix += ok ? (((u64)fhi << 32) | flo) : 0ull;
      const u64 key = ok ? evict_key(tmp, pe) : ~0ull;
      best_i = key < best ? i : best_i;
      best = key < best ? key : best;
      if (i == n - 1) {                     // the last slot's final state, for the in-place eviction
        sh[1] = __float_as_int(ncrf[e]);
        sh[2] = ntau[e];
        sh[3] = pe;
      }
    }
    if (e0 + 3 < n) {
      if (stored) {
        const size_t s0 = base + e0;
        *reinterpret_cast<f32x4*>(d.crf + s0) = ncrf;
        *reinterpret_cast<i32x4*>(d.tau + s0) = ntau;
      }
    } else if (e0 < n) {                     // the unit's last, partial group: entry by entry
      for (int e = 0; e < 4 && e0 + e < n; ++e) {
        if ((stored >> e) & 1u) {
          d.crf[base + (e0 + e)] = ncrf[e];
          d.tau[base + (e0 + e)] = t;
        }
      }
    }
  }
  sfix = block_sum_u64<NT>(sfix, rb, phase, tid);
  if (tid == 0) {
    d.window[u] = window0 + sfix;
    d.t_unit[u] = t;
  }
  // ---- Step 4
  if (!(evict && n > B)) {
    if (tid == 0) d.nev[u] = 0;
    return;
  }
  if (evict_single) {
    const u64 gbest = block_min_u64<NT>(best, rb, phase, tid);
    if (best == gbest && best_i >= 0) {     // keys are unique: one writer
      sh[0] = best_i;
      sh[4] = ~(int)(uint32_t)best;         // the victim's position
    }
    block_sync<NT>(rb);
    evict_one<NT>(d, base, n - 1, sh[0], sh, tid, last_row);
    if (tid == 0) {
      d.n[u] = B;
      d.nev[u] = 1;
    }
  } else {
#pragma unroll
    for (int k = 0; k < R; ++k) {
      const int i = 4 * (tid + (k >> 2) * NT) + (k & 3);
      if (i < n) val(i) = a[k];
    }
    block_sync<NT>(rb);
    evict_phase<Val, NT>(d, u, base, n, B, val, evm, lst, lst_cap, rb, phase, sh, tid);
  }
}

// Mean weights of the unit's first n entries from its logits (softmax maxima sM and reciprocal denominators
// sInv per head in LDS), then Alg. 1 Steps 1-3 at time t and, if asked, Step 4.  One workgroup of kThreads.
// val: n floats of LDS, evm: the eviction bit mask behind them.
// sh: 4 + NT / 64 ints.
template <int NT = kThreads>
__device__ __forceinline__ void unit_bookkeeping(const Dev& d, int u, int n, int B, int t, LgView lv, const float* sM,
                                                 const float* sInv, bool evict, float* val, uint32_t* evm, const float* s_tab,
                                                 int s_tab_n, RedBuf& rb, int& phase, int* sh, int tid) {
  const Slots base = slots_of(d, u);
  if (n <= 8 * NT) {
    float a[8];
    mean_weights_regs<8, NT>(d, lv, n, sM, sInv, a, tid);
    f32x4 crf[2];
    i32x4 tau[2], ps[2];
    lrfu_regs<8, 2, 0, ValLinear, NT>(d, u, base, n, B, t, a, crf, tau, ps, ValLinear{val}, evict, evm, reinterpret_cast<int*>(val), d.cap,
                                      s_tab, s_tab_n, rb, phase, sh, tid);
  } else if (n <= 16 * NT) {
    float a[16];
    mean_weights_regs<16, NT>(d, lv, n, sM, sInv, a, tid);
    f32x4 crf[4];
    i32x4 tau[4], ps[4];
    lrfu_regs<16, 4, 0, ValLinear, NT>(d, u, base, n, B, t, a, crf, tau, ps, ValLinear{val}, evict, evm, reinterpret_cast<int*>(val), d.cap,
                                       s_tab, s_tab_n, rb, phase, sh, tid);
  } else if (n <= 32 * NT) {
    float a[32];
    mean_weights_regs<32, NT>(d, lv, n, sM, sInv, a, tid);
    f32x4 crf[8];
    i32x4 tau[8], ps[8];
    lrfu_regs<32, 8, 0, ValLinear, NT>(d, u, base, n, B, t, a, crf, tau, ps, ValLinear{val}, evict, evm, reinterpret_cast<int*>(val), d.cap,
                                       s_tab, s_tab_n, rb, phase, sh, tid);
  } else {
    mean_weights<NT>(d, lv, n, sM, sInv, val, tid);
    const u64 sfix = lrfu_update<ValLinear, NT>(d, u, base, n, t, ValLinear{val}, s_tab, s_tab_n, rb, phase, tid);
    if (tid == 0) {
      d.window[u] += sfix;
      d.t_unit[u] = t;
    }
    if (evict && n > B)
      evict_phase<ValLinear, NT>(d, u, base, n, B, ValLinear{val}, evm, reinterpret_cast<int*>(val), d.cap, rb, phase, sh, tid);
    else if (tid == 0)
      d.nev[u] = 0;
  }
}

// n_limit / t_fixed: the replay of a prompt's last queries runs the step over the unit's first n_limit
// entries at time t_fixed (otherwise INT_MAX and -1: all entries, the context's time).
// late: 0 = the whole step.  1 = the bookkeeping alone (mean weights, Alg. 1 Steps 1-4) of a single-layer
// step whose scan has already merged the partials, written the output and ended the step: it runs later,
// on another stream, from the partials and logits of that launch, whose time and sequence number the scan
// left in d.layer_ts[layer], and touches no step scalar.
__global__ __launch_bounds__(kThreads) void finish_kernel(Dev d, int unit_begin, void* out, uint32_t call_flags,
                                                          int advance, int n_limit, int t_fixed, int late, int layer) {
  extern __shared__ unsigned char smem[];
  float* val = reinterpret_cast<float*>(smem);
  uint32_t* evm = reinterpret_cast<uint32_t*>(smem + (size_t)d.cap * 4);
  __shared__ float sM[kMaxGroup], sInv[kMaxGroup], sW[2 * (kMaxChunks + 1) * kMaxGroup];
  __shared__ RedBuf rb;
  __shared__ int sh[8];
  __shared__ float s_tab[kTabLds];
  const int tid = threadIdx.x;
  const int urel = blockIdx.x, u = unit_begin + urel;
  int n = min(d.n[u], n_limit);
  if (layer == -2) layer = u / (d.Bz * d.Hkv);          // a launch over several layers: each unit looks up its own
  const int t = late ? d.layer_ts[2 * layer] : t_fixed >= 0 ? t_fixed : d.sc[SC_T];
  const int seq = late == 1 ? d.layer_ts[2 * layer + 1] : d.sc[SC_SEQ];
  const int B = d.budget[u];
  const int s_tab_n = min(kTabLds, d.tab_last + 1);
  if (tid < s_tab_n) s_tab[tid] = d.tab[tid];
  int phase = 0;
  if (late == 2) {
    // after layer_scan_kernel: the new entry's rows are in the cache and its logits with the others, the
    // unit's records still describe the step before.  Record the append, then go on as after any scan.
    // (Every wavefront has read the stored length before the first thread replaces it: a wavefront that
    // started late would otherwise count the new entry twice and part ways with the others.)
    __syncthreads();
    if (n < unit_cap(d, u)) {
      if (tid == 0) {
        const size_t s = slots_of(d, u) + n;
        d.crf[s] = 0.0f;
        d.tau[s] = t;
        d.pos[s] = t;
        d.flags[s] = 0;
        d.n[u] = n + 1;
      }
      n += 1;
    }
    if (tid < d.G) {
      sM[tid] = d.msum[((size_t)u * kMaxGroup + tid) * 2];
      sInv[tid] = d.msum[((size_t)u * kMaxGroup + tid) * 2 + 1];
    }
    __threadfence_block();
    __syncthreads();
  }
  if (n > 0) {
    const int nch = (n + kChunk - 1) / kChunk;
    if (late != 2) merge_partials(d, u, urel, nch, seq, sM, sInv, sW, late ? nullptr : out, tid);
    unit_bookkeeping(d, u, n, B, t, unit_logits(d, u), sM, sInv, (call_flags & 1u) != 0, val, evm, s_tab, s_tab_n, rb, phase, sh, tid);
  }
  if (!late) step_epilogue(d, t, advance, tid);
}

// ------------------------------------------------------------------ prompt replay (scores of a loaded prompt)
// The prompt's last W queries in a few kernels per batch of queries.  What a query does to the scores splits
// into a part that does not depend on the scores - its mean attention weights over the entries it sees and,
// from them, the reward of every entry (Alg. 1 Steps 1-2: hit or not; or the weight itself) - and the score
// recurrence (Step 3), which is sequential over the queries but independent per entry.  So:
//   seed_scan_kernel<false>  a pass over the keys for all queries of the batch: softmax partials per chunk
//   seed_stats_kernel        per query head: softmax maximum and 1 / sum over the entries the query sees
//   seed_scan_kernel<true>   a second pass: the logits again, normalised, the mean over the heads -> weights
//   seed_hits_kernel         per (unit, query): hit rule, rewards in place of the weights (top-p rule only)
//   seed_crf_kernel          per entry: the queries' rewards applied in order
// (Two passes over the keys, 256 B per entry each, instead of the logits of every query head going through
// memory, 4 G B per entry and query written and read back.)  Only the weights are wanted (no output), so V is
// never read.
//
// Columns: the matrix-core tile has 16 query columns, of which a decode step fills G; here a tile holds the G
// heads of Q = 16 / G queries (column c = head c % G of the tile's query c / G), and a batch is up to
// kSeedTiles tiles.  Buffers of a batch of nt tiles, nq queries, for the UL units of a layer:
//   sml [tile][unit][chunk][column][2]    running maximum and sum of the softmax per 256-entry chunk
//   smi [tile][unit][column][2]           maximum and 1 / sum over all the entries the column's query sees
//   srw [query][unit][cap]                mean weights, then rewards
constexpr int kSeedCols = 16;
constexpr int kSeedTiles = 16;

// seed_scan_kernel: one wavefront per 256-entry chunk of a unit; the tiles' queries sit in LDS (per tile and
// 32-dim slice one 16-byte operand piece per lane), each block of keys is loaded once and multiplied with every
// tile.  Query j of the window sees the entries of positions <= its own, i.e. indices < P - W + j + 1 (the
// prompt's entries sit in position order).  WEIGHTS = false: per chunk and column the running maximum and sum
// of the softmax go to `sml`.  WEIGHTS = true: every logit is normalised with its column's maximum and 1 / sum
// from `smi`, and the mean over a query's G heads (summed in head order, as the decode path's mean weights
// are) goes to `srw`; entries a query does not see get 0.
// grid: (ceil(chunks / 4), units of the layer), kThreads threads, nt * 4096 bytes of dynamic LDS.
template <bool WEIGHTS>
__global__ __launch_bounds__(kThreads) void seed_scan_kernel(Dev d, int unit_begin, const uint16_t* __restrict__ q_obs, int j0,
                                                             int nq, int Q, int P, int W, float* __restrict__ sml,
                                                             const float* __restrict__ smi, float* __restrict__ srw) {
  extern __shared__ unsigned char smem[];
  u32x4* s_q = reinterpret_cast<u32x4*>(smem);            // [tile][slice][lane]
  __shared__ float2 s_mi[WEIGHTS ? kSeedTiles * kSeedCols : 1];      // WEIGHTS: every column's maximum and 1 / sum
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int urel = blockIdx.y, u = unit_begin + urel;
  const int UL = gridDim.y;
  const int chunk = blockIdx.x * (kThreads / 64) + wave;
  const int G = d.G;
  const int j = lane & 15, kg = lane >> 4;
  const int nt = (nq + Q - 1) / Q;
  const int mc = d.max_chunks;
  const int n_first = P - W + j0 + 1;                     // entries the batch's first query sees
  const int n_last = n_first + nq - 1;                    // ... and its last
  if constexpr (WEIGHTS) {
    if ((int)threadIdx.x < nt * kSeedCols)
      s_mi[threadIdx.x] = *reinterpret_cast<const float2*>(smi + (((size_t)(threadIdx.x / kSeedCols) * UL + urel) * kSeedCols + threadIdx.x % kSeedCols) * 2);
  }
  {
    // this thread's piece (slice = wave, lane) of every tile's operand
    const int b = urel / d.Hkv, h = urel % d.Hkv;
    for (int tl = 0; tl < nt; ++tl) {
      const int qn = min(Q, nq - tl * Q);                 // queries in this tile
      const int qi = min(j / G, qn - 1);
      const uint16_t* qrow = q_obs + ((((size_t)(j0 + tl * Q + qi) * d.Bz + b) * d.Hq) + (size_t)h * G + (j % G)) * kDim + 8 * kg;
      u32x4 x = *reinterpret_cast<const u32x4*>(qrow + 32 * wave);
      if (j >= qn * G) x = u32x4{0u, 0u, 0u, 0u};
      s_q[(tl * 4 + wave) * 64 + lane] = x;
    }
  }
  __syncthreads();
  const int e_chunk = chunk * kChunk;
  if (e_chunk >= n_last) return;
  const int nblk = min(kChunkBlocks, (n_last - e_chunk + kBlk - 1) / kBlk);
  const uint16_t* kb = d.K + (size_t)d.tbl[(size_t)u * d.max_seg + chunk] * kSegElems + lane * 8;     // a chunk is one pool segment
  // WEIGHTS = false: this lane's running maximum and sum per tile (its entries only; the four lanes of a column
  // meet at the end)
  constexpr int kStat = WEIGHTS ? 1 : kSeedTiles;
  float m_run[kStat], l_run[kStat];
#pragma unroll
  for (int tl = 0; tl < kStat; ++tl) {
    m_run[tl] = -INFINITY;
    l_run[tl] = 0.f;
  }
  const float invG = 1.0f / (float)G;
  KFrag ka, kn;
  load_k(ka, kb);
  for (int blk = 0; blk < nblk; ++blk) {
    if (blk + 1 < nblk) load_k(kn, kb + (size_t)(blk + 1) * kBlkElems);
    const int e0 = e_chunk + blk * kBlk + 4 * kg;
    auto tile = [&](int tl, float& m_t, float& l_t) {
      const int qn = min(Q, nq - tl * Q);
      const bool col_ok = j < qn * G;
      // entries this column's query sees (columns beyond the tile's queries: none)
      const int lim = col_ok ? n_first + tl * Q + j / G : 0;
      if (e_chunk + blk * kBlk >= n_first + tl * Q + qn - 1) return;     // the tile's last query does not see the block (uniform)
      bf16x8 qv[4];
#pragma unroll
      for (int s4 = 0; s4 < 4; ++s4) qv[s4] = as_bf16x8(s_q[(tl * 4 + s4) * 64 + lane]);
      f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int s4 = 0; s4 < 4; ++s4) s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(ka.k[s4]), qv[s4], s0, 0, 0, 0);
#pragma unroll
      for (int s4 = 0; s4 < 4; ++s4) s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(ka.k[4 + s4]), qv[s4], s1, 0, 0, 0);
      float sv[8];
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        sv[v] = (e0 + v < lim) ? s0[v] * d.scale_log2e : -INFINITY;
        sv[4 + v] = (e0 + 16 + v < lim) ? s1[v] * d.scale_log2e : -INFINITY;
      }
      if constexpr (!WEIGHTS) {
        const float bm = fmaxf(fmaxf(fmaxf(sv[0], sv[1]), fmaxf(sv[2], sv[3])), fmaxf(fmaxf(sv[4], sv[5]), fmaxf(sv[6], sv[7])));
        if (bm > m_t) {
          l_t *= fast_exp2(m_t - bm);                       // exp2(-inf) = 0 the first time
          m_t = bm;
        }
        if (m_t > -INFINITY) {
#pragma unroll
          for (int i = 0; i < 8; ++i) l_t += fast_exp2(sv[i] - m_t);
        }
      } else {
        // this head's share of the weight of its 4 + 4 entries, then the query's heads in order
        const float2 mi = s_mi[tl * kSeedCols + j];
        float term[8], mean[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          term[i] = sv[i] > -INFINITY ? fast_exp2(sv[i] - mi.x) * mi.y : 0.f;
        }
        // lane c + g of the row holds head g of the query whose first head sits in lane c: the sum of a
        // query's heads, in head order, forms in its first head's lane (row_shl:g brings lane + g's value)
#pragma unroll
        for (int i = 0; i < 8; ++i) mean[i] = term[i];
#pragma unroll
        for (int g = 1; g < kMaxGroup; ++g) {
          if (g < G) {
#pragma unroll
            for (int i = 0; i < 8; ++i) mean[i] += row_shl_f32(term[i], g);
          }
        }
        if (col_ok && j % G == 0) {
          float* dst = srw + ((size_t)(tl * Q + j / G) * UL + urel) * d.cap + e0;
          *reinterpret_cast<f32x4*>(dst) = f32x4{mean[0] * invG, mean[1] * invG, mean[2] * invG, mean[3] * invG};
          *reinterpret_cast<f32x4*>(dst + 16) = f32x4{mean[4] * invG, mean[5] * invG, mean[6] * invG, mean[7] * invG};
        }
      }
    };
    if constexpr (WEIGHTS) {
#pragma unroll 1
      for (int tl = 0; tl < nt; ++tl) tile(tl, m_run[0], l_run[0]);
    } else {
#pragma unroll
      for (int tl = 0; tl < kSeedTiles; ++tl)
        if (tl < nt) tile(tl, m_run[tl], l_run[tl]);
    }
    if (blk + 1 < nblk) ka = kn;
  }
  if constexpr (!WEIGHTS) {
    // per tile, the column's four lanes (kg = 0..3): maximum, then the sums rescaled to it, in a fixed order
#pragma unroll
    for (int tl = 0; tl < kSeedTiles; ++tl) {
      if (tl < nt) {
        float M = fmaxf(m_run[tl], __shfl_xor(m_run[tl], 16));
        M = fmaxf(M, __shfl_xor(M, 32));
        const float mine = m_run[tl] > -INFINITY ? l_run[tl] * fast_exp2(m_run[tl] - M) : 0.f;
        const float l0 = __shfl(mine, j), l1 = __shfl(mine, j + 16), l2 = __shfl(mine, j + 32), l3 = __shfl(mine, j + 48);
        if (kg == 0) {
          float* dst = sml + ((((size_t)tl * UL + urel) * mc + chunk) * kSeedCols + j) * 2;
          dst[0] = M;
          dst[1] = (l0 + l1) + (l2 + l3);
        }
      }
    }
  }
}

// seed_stats_kernel: thread (tile, column) of a unit: maximum and 1 / sum of the column's softmax over the chunks
// its query sees, in chunk order.  grid: units of the layer, kSeedTiles * kSeedCols threads.
__global__ __launch_bounds__(kSeedTiles * kSeedCols) void seed_stats_kernel(Dev d, int j0, int nq, int Q, int P, int W,
                                                                         const float* __restrict__ sml, float* __restrict__ smi) {
  const int urel = blockIdx.x, UL = gridDim.x;
  const int tl = threadIdx.x / kSeedCols, col = threadIdx.x % kSeedCols;
  const int G = d.G, mc = d.max_chunks;
  const int nt = (nq + Q - 1) / Q;
  if (tl >= nt) return;
  const int qn = min(Q, nq - tl * Q);
  float M = -INFINITY, inv = 0.f;
  if (col < qn * G) {
    const int n = P - W + j0 + tl * Q + col / G + 1;      // entries the column's query sees
    const int nch = (n + kChunk - 1) / kChunk;
    const float* ml = sml + ((((size_t)tl * UL + urel) * mc) * kSeedCols + col) * 2;
    // eight chunks' partials are asked for at a time; maxima, then sums, in chunk order
    for (int c0 = 0; c0 < nch; c0 += 8) {
      float2 p[8];
#pragma unroll
      for (int k = 0; k < 8; ++k) p[k] = *reinterpret_cast<const float2*>(ml + (size_t)min(c0 + k, nch - 1) * kSeedCols * 2);
#pragma unroll
      for (int k = 0; k < 8; ++k)
        if (c0 + k < nch) M = fmaxf(M, p[k].x);
    }
    float L = 0.f;
    for (int c0 = 0; c0 < nch; c0 += 8) {
      float2 p[8];
#pragma unroll
      for (int k = 0; k < 8; ++k) p[k] = *reinterpret_cast<const float2*>(ml + (size_t)min(c0 + k, nch - 1) * kSeedCols * 2);
#pragma unroll
      for (int k = 0; k < 8; ++k)
        if (c0 + k < nch && p[k].x > -INFINITY) L += p[k].y * fast_exp2(p[k].x - M);
    }
    inv = 1.0f / L;
  }
  float* dst = smi + (((size_t)tl * UL + urel) * kSeedCols + col) * 2;
  dst[0] = M;
  dst[1] = inv;
}

// seed_hits_kernel (top-p rule only): one workgroup per (query of the batch, unit).  The query's mean weights
// from `srw`, the hit rule, and in their place the rewards: 1 or 0 (the query's own entry, the last it sees, is
// always hit).
// grid: (queries of the batch, units of the layer), kSeedThreads threads, dynamic LDS as finish_kernel.
constexpr int kSeedThreads = 512;      // twice a decode step's workgroup: prompts are long

template <int R>
__device__ __forceinline__ void seed_rewards_regs(const Dev& d, Slots base, int n, bool last_new, float* rw, int* lst, int lst_cap,
                                                  RedBuf& rb, int& phase, int* sh, int tid) {
  float a[R];
#pragma unroll
  for (int c = 0; c < R / 4; ++c) {
    const int e0 = 4 * (tid + c * kSeedThreads);
    const f32x4 x = e0 < n ? *reinterpret_cast<const f32x4*>(rw + e0) : f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int e = 0; e < 4; ++e) a[4 * c + e] = (e0 + e < n) ? x[e] : 0.f;
  }
  const HitRule rule = top_p_regs<R, kSeedThreads, 256>(d, base, n, a, lst, lst_cap, -1, rb, phase, sh, tid);
#pragma unroll
  for (int c = 0; c < R / 4; ++c) {
    const int e0 = 4 * (tid + c * kSeedThreads);
    if (e0 < n) {
      i32x4 ps = {0, 0, 0, 0};
      if (!rule.ties_all) ps = *reinterpret_cast<const i32x4*>(d.pos + (base + e0));      // rare
      f32x4 r;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const bool hit = rule(__float_as_uint(a[4 * c + e]), ps[e]) | ((e0 + e == n - 1) & last_new);
        r[e] = hit ? 1.0f : 0.0f;
      }
      *reinterpret_cast<f32x4*>(rw + e0) = r;              // entries >= n of the group: written, never read
    }
  }
}

__global__ __launch_bounds__(kSeedThreads, 4) void seed_hits_kernel(Dev d, int unit_begin, int j0, int P, int W, float* __restrict__ srw) {
  extern __shared__ unsigned char smem[];
  float* val = reinterpret_cast<float*>(smem);
  __shared__ RedBuf rb;
  __shared__ int sh[4 + kSeedThreads / 64];
  const int tid = threadIdx.x;
  const int ql = blockIdx.x, urel = blockIdx.y, u = unit_begin + urel;
  const int UL = gridDim.y;
  const int t = P - W + j0 + ql;                          // the query's position = its time
  const int n = t + 1;
  const Slots base = slots_of(d, u);
  const bool last_new = d.pos[base + (n - 1)] == t;       // the query's own entry (asked for early: nothing waits for it until the end)
  int phase = 0;
  float* rw = srw + ((size_t)ql * UL + urel) * d.cap;
  int* lst = reinterpret_cast<int*>(val);
  if (n <= 8 * kSeedThreads) {
    seed_rewards_regs<8>(d, base, n, last_new, rw, lst, d.cap, rb, phase, sh, tid);
  } else if (n <= 16 * kSeedThreads) {
    seed_rewards_regs<16>(d, base, n, last_new, rw, lst, d.cap, rb, phase, sh, tid);
  } else if (n <= 32 * kSeedThreads) {
    seed_rewards_regs<32>(d, base, n, last_new, rw, lst, d.cap, rb, phase, sh, tid);
  } else {
    for (int i = tid; i < n; i += kSeedThreads) val[i] = rw[i];
    __syncthreads();
    const HitRule rule = top_p_lds<ValLinear, kSeedThreads>(d, base, n, ValLinear{val}, rb, phase, tid);
    for (int i = tid; i < n; i += kSeedThreads) {
      const int pe = !rule.ties_all ? d.pos[base + i] : 0;
      const bool hit = rule(__float_as_uint(val[i]), pe) | ((i == n - 1) & last_new);
      rw[i] = hit ? 1.0f : 0.0f;
    }
  }
}

// seed_crf_kernel: Alg. 1 Step 3 for the batch's queries in order, four consecutive entries per thread: an entry
// takes part from the query of its own position on; under the top-p rule only a hit replaces (CRF, tau).
// grid: (ceil(P / (4 kThreads)), units of the layer), kThreads threads.
__global__ __launch_bounds__(kThreads) void seed_crf_kernel(Dev d, int unit_begin, int j0, int nq, int P, int W,
                                                            const float* __restrict__ srw) {
  __shared__ float s_tab[kTabLds];
  const int tid = threadIdx.x;
  const int urel = blockIdx.y, u = unit_begin + urel;
  const int UL = gridDim.y;
  const int s_tab_n = min(kTabLds, d.tab_last + 1);
  if (tid < s_tab_n) s_tab[tid] = d.tab[tid];
  __syncthreads();
  const int e0 = 4 * (blockIdx.x * kThreads + tid);
  if (e0 >= P) return;
  const Slots base = slots_of(d, u);
  const size_t s0 = base + e0;                            // four consecutive entries share a segment
  f32x4 crf = *reinterpret_cast<const f32x4*>(d.crf + s0);
  i32x4 tau = *reinterpret_cast<const i32x4*>(d.tau + s0);
  const bool topp = d.reward_mode == 0;
  const float* rw = srw + (size_t)urel * d.cap + e0;
  const size_t q_stride = (size_t)UL * d.cap;
  const int t_first = P - W + j0;
  bool changed = false;
  for (int q0 = 0; q0 < nq; q0 += 8) {
    f32x4 r[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) r[k] = *reinterpret_cast<const f32x4*>(rw + (size_t)min(q0 + k, nq - 1) * q_stride);
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      const int t = t_first + q0 + k;
      if (q0 + k < nq) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          if (e0 + e <= t) {                              // the query sees positions 0 .. t
            int delta = t - tau[e];
            delta = delta < 0 ? 0 : (delta > d.tab_last ? d.tab_last : delta);
            const float dec = decay_of(d, delta, s_tab, s_tab_n);
            const float reward = r[k][e];
            float tmp = __fadd_rn(__fmul_rn(dec, crf[e]), reward);
            if (tmp < FLT_MIN) tmp = 0.0f;
            if (!topp || reward != 0.0f) {
              crf[e] = tmp;
              tau[e] = t;
              changed = true;
            }
          }
        }
      }
    }
  }
  if (!changed) return;
  if (e0 + 3 < P) {
    *reinterpret_cast<f32x4*>(d.crf + s0) = crf;
    *reinterpret_cast<i32x4*>(d.tau + s0) = tau;
  } else {
    for (int e = 0; e < 4 && e0 + e < P; ++e) {
      d.crf[s0 + e] = crf[e];
      d.tau[s0 + e] = tau[e];
    }
  }
}

// Alg. 1 Step 4 on its own: scores decayed to the unit's last step, no update.
// n_sink < 0: Alg. 1 Step 4 (retain the highest CRF_temp).  n_sink >= 0: the comparison policy of Sec. 2.3
// that keeps the initial and the most recent tokens; the retention key is then the position itself, carried
// as a bit pattern (the eviction only ever compares the bits), and the largest pattern for positions below n_sink.
__global__ __launch_bounds__(kThreads) void evict_kernel(Dev d, int unit_begin, int n_sink) {
  extern __shared__ unsigned char smem[];
  float* val = reinterpret_cast<float*>(smem);
  uint32_t* evm = reinterpret_cast<uint32_t*>(smem + (size_t)d.cap * 4);
  __shared__ RedBuf rb;
  __shared__ int sh[8];
  const int tid = threadIdx.x;
  const int u = unit_begin + blockIdx.x;
  const int n = d.n[u], B = d.budget[u];
  const Slots base = slots_of(d, u);
  int phase = 0;
  if (n <= B) {
    if (tid == 0) d.nev[u] = 0;
    return;
  }
  const int t = d.t_unit[u];
  if (n_sink >= 0) {
    for (int i = tid; i < n; i += kThreads) {
      const int p = d.pos[base + i];
      val[i] = __uint_as_float(p < n_sink ? 0x7FFFFFFFu : (uint32_t)p);
    }
  } else {
    for (int i = tid; i < n; i += kThreads) {
      int delta = t - d.tau[base + i];
      delta = delta < 0 ? 0 : (delta > d.tab_last ? d.tab_last : delta);
      float tmp = __fmul_rn(d.tab[delta], d.crf[base + i]);
      if (tmp < FLT_MIN) tmp = 0.0f;
      val[i] = tmp;
    }
  }
  __syncthreads();
  evict_phase(d, u, base, n, B, ValLinear{val}, evm, reinterpret_cast<int*>(val), d.cap, rb, phase, sh, tid);
}

// ------------------------------------------------------------------ probe
// Sec. 3: classes of the entries of unit u under the probe query's weights.
__global__ __launch_bounds__(kThreads) void probe_kernel(Dev d, int unit_begin, uint8_t* classes) {
  extern __shared__ unsigned char smem[];
  float* val = reinterpret_cast<float*>(smem);
  __shared__ float sM[kMaxGroup], sInv[kMaxGroup], sW[2 * (kMaxChunks + 1) * kMaxGroup];
  __shared__ RedBuf rb;
  const int tid = threadIdx.x;
  const int urel = blockIdx.x, u = unit_begin + urel;
  const int n = d.n[u];
  const Slots base = slots_of(d, u);
  int phase = 0;
  if (n > 0) {
    merge_partials(d, u, urel, (n + kChunk - 1) / kChunk, d.sc[SC_SEQ], sM, sInv, sW, nullptr, tid);
    mean_weights(d, unit_logits(d, u), n, sM, sInv, val, tid);
    const int kq = (3 * n) / 10;
    // order key: ascending = (weight asc, position desc); Crystal = kq largest, Slip = kq smallest
    u64 lo_cut = 0, hi_cut = ~0ull;
    if (kq > 0) {
      for (int pass = 0; pass < 2; ++pass) {
        const int k = pass == 0 ? kq : (n - kq + 1);      // k-th smallest key
        u64 X = 0;
        for (int bit = 62; bit >= 0; --bit) {
          const u64 trial = X | (1ull << bit);
          int cnt = 0;
          for (int i = tid; i < n; i += kThreads) cnt += evict_key(val[i], d.pos[base + i]) < trial ? 1 : 0;
          cnt = block_sum_int(cnt, rb, phase, tid);
          if (cnt < k) X = trial;
        }
        if (pass == 0) lo_cut = X; else hi_cut = X;
      }
    }
    for (int i = tid; i < n; i += kThreads) {
      const u64 key = evict_key(val[i], d.pos[base + i]);
      uint8_t c = 1;
      if (kq > 0) {
        if (key >= hi_cut) c = 2;
        else if (key <= lo_cut) c = 0;
      }
      classes[(size_t)urel * d.cap + i] = c;
    }
  }
  step_epilogue(d, 0, 0, tid);
}

// ------------------------------------------------------------------ Alg. 2
// Integers val[k] in [lo, hi] summing to `total`, proportional to x[k] >= 0 as
// far as the bounds allow: water-filling on the reals, floor, remainder by
// largest fractional part (lower index first on ties), final spill in index order.
__device__ __forceinline__ void apportion(const double* x, int m, long long total, long long lo, long long hi, long long* val, double* y,
                          unsigned char* fixed) {
  for (int k = 0; k < m; ++k) {
    fixed[k] = 0;
    val[k] = 0;
    y[k] = 0.0;
  }
  for (int iter = 0; iter < m + 1; ++iter) {
    long long R = total;
    int n_free = 0;
    double X = 0.0;
    for (int k = 0; k < m; ++k) {
      if (fixed[k]) R -= val[k];
      else {
        ++n_free;
        X += x[k];
      }
    }
    if (n_free == 0) break;
    double over = 0.0, under = 0.0;
    for (int k = 0; k < m; ++k) {
      if (fixed[k]) continue;
      y[k] = (X > 0.0) ? (double)R * (x[k] / X) : (double)R / (double)n_free;
      if (y[k] > (double)hi) over += y[k] - (double)hi;
      if (y[k] < (double)lo) under += (double)lo - y[k];
    }
    if (over == 0.0 && under == 0.0) break;
    if (over >= under) {
      for (int k = 0; k < m; ++k)
        if (!fixed[k] && y[k] > (double)hi) {
          fixed[k] = 1;
          val[k] = hi;
        }
    } else {
      for (int k = 0; k < m; ++k)
        if (!fixed[k] && y[k] < (double)lo) {
          fixed[k] = 1;
          val[k] = lo;
        }
    }
  }
  long long sum = 0;
  for (int k = 0; k < m; ++k) {
    if (!fixed[k]) {
      const double f = floor(y[k]);
      long long fi = (long long)f;
      fi = fi < lo ? lo : (fi > hi ? hi : fi);
      val[k] = fi;
      y[k] = y[k] - f;         // fractional part
    }
    sum += val[k];
  }
  long long rem = total - sum;
  // fixed[k]: 0 = free and not yet visited, 1 = fixed at a bound, 2 = free and visited
  while (rem > 0) {
    int best = -1;
    for (int k = 0; k < m; ++k)
      if (fixed[k] == 0 && (best < 0 || y[k] > y[best])) best = k;
    if (best < 0) break;
    fixed[best] = 2;
    if (val[best] < hi) {
      val[best] += 1;
      rem -= 1;
    }
  }
  while (rem < 0) {
    int best = -1;
    for (int k = 0; k < m; ++k)
      if (fixed[k] == 0 && (best < 0 || y[k] <= y[best])) best = k;
    if (best < 0) break;
    fixed[best] = 2;
    if (val[best] > lo) {
      val[best] -= 1;
      rem += 1;
    }
  }
  while (rem != 0) {
    bool moved = false;
    for (int k = 0; k < m; ++k) {
      if (rem > 0 && val[k] < hi) {
        val[k] += 1;
        rem -= 1;
        moved = true;
      } else if (rem < 0 && val[k] > lo) {
        val[k] -= 1;
        rem += 1;
        moved = true;
      }
      if (rem == 0) break;
    }
    if (!moved) break;
  }
}

constexpr int kMaxLayers = 256;
constexpr int kMaxKvHeads = 32;

// One workgroup per sequence.
__global__ __launch_bounds__(kThreads) void rebudget_kernel(Dev d) {
  __shared__ double eta_l[kMaxLayers], y_l[kMaxLayers];
  __shared__ long long tot_l[kMaxLayers];
  __shared__ unsigned char fx_l[kMaxLayers];
  __shared__ int ok;
  const int tid = threadIdx.x, b = blockIdx.x;
  const int L = d.L, H = d.Hkv;
  const int steps = d.sc[SC_WINDOW_STEPS];
  if (steps > 0) {
    const double denom = 1048576.0 * (double)steps;
    if (tid < L) {
      double sc = 0.0, sb = 0.0;
      for (int j = 0; j < H; ++j) {
        const int u = (tid * d.Bz + b) * H + j;
        sc += (double)d.window[u] / denom;
        sb += (double)d.budget[u];
      }
      eta_l[tid] = sc / sb;
    }
    __syncthreads();
    if (tid == 0) {
      double sum_eta = 0.0;
      for (int i = 0; i < L; ++i) sum_eta += eta_l[i];
      if (!(sum_eta > 0.0) || !isfinite(sum_eta)) {
        ok = 0;
      } else {
        apportion(eta_l, L, d.btotal[b], (long long)H * d.bmin, (long long)H * d.bmax, tot_l, y_l, fx_l);
        ok = 1;
      }
    }
    __syncthreads();
    if (ok && tid < L) {
      double eta_h[kMaxKvHeads], y_h[kMaxKvHeads];
      long long val_h[kMaxKvHeads];
      unsigned char fx_h[kMaxKvHeads];
      for (int j = 0; j < H; ++j) {
        const int u = (tid * d.Bz + b) * H + j;
        eta_h[j] = ((double)d.window[u] / denom) / (double)d.budget[u];
      }
      apportion(eta_h, H, tot_l[tid], d.bmin, d.bmax, val_h, y_h, fx_h);
      for (int j = 0; j < H; ++j) d.budget[(tid * d.Bz + b) * H + j] = (int32_t)val_h[j];
    }
    __syncthreads();
    for (int i = tid; i < L * H; i += kThreads) d.window[((i / H) * d.Bz + b) * H + (i % H)] = 0ull;
  }
  __syncthreads();
  if (tid == 0) {
    __threadfence();
    const int prev = atomicAdd(&d.sc[SC_DONE_RB], 1);
    if (prev == (int)gridDim.x - 1) {
      d.sc[SC_DONE_RB] = 0;
      d.sc[SC_WINDOW_STEPS] = 0;
    }
  }
}

}  // namespace ckv
