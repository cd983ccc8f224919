// Fused decode step: one persistent kernel that, unit by unit, streams K and V,
// keeps the scaled logits in LDS, and runs the LRFU bookkeeping (merge, top-p hit
// mask, CRF update, eviction) on them without a round trip through HBM.
//
// Why: with separate scan and finish kernels the logits (4 G bytes per entry)
// have to be written and read back; that write stream alone costs the scan
// ~15 % of its bandwidth, and the finish kernel is latency-bound on its own.
// Here two workgroups share a CU, so while one does a unit's bookkeeping the
// other keeps the memory pipeline busy.
//
// Work: schedule slots (units in order of descending budget, `d.order`) are
// taken three rounds statically, then from a shared queue.  The W wavefronts of
// a workgroup split a unit's 32-entry blocks round robin (wave w takes blocks
// w, w+W, ...), each with its own online softmax state; the states are merged
// through LDS at the end of the unit.  As in the scan kernel every load in the
// streaming loop is unconditional: after a wave's last block of a unit the
// stream continues with its first block of the next unit, which therefore is
// in flight during the bookkeeping.
//
// LDS (dynamic, `lds_main` bytes + mask): the logits tile [block][head][32] f32
// of the first n_res entries; the per-entry value (mean weight, then CRF_temp)
// of a resident entry lives in its head-0 slot, values of the other entries
// follow the tile.  Units whose logits do not fit spill the logits of their
// last blocks to the global logits buffer (same layout as the scan kernel's).
#pragma once
#include <type_traits>

#include "ckv_kernels.h"

namespace ckv {

struct ValFused {
  float* lg;       // logits tile
  float* spill;    // values of entries >= n_res
  int n_res;       // resident entries (multiple of 32)
  int gstride;     // G * 32
  __device__ __forceinline__ float& operator()(int i) const {
    return i < n_res ? lg[(i >> 5) * gstride + (i & 31)] : spill[i - n_res];
  }
};

// Entries of a unit of n entries whose logits stay in LDS (multiple of 32).
__device__ __forceinline__ int resident_entries(int n, int G, int lds_main_bytes) {
  const int n_pad = (n + kBlk - 1) & ~(kBlk - 1);
  if (G == 1) return n_pad;
  int r = (lds_main_bytes - 4 * n_pad) / (4 * (G - 1));
  r = r < 0 ? 0 : r;
  r &= ~(kBlk - 1);
  return r < n_pad ? r : n_pad;
}

// Schedule of the fused kernel: the units sorted by descending budget (counting
// sort over budget / 32, one workgroup; the order inside a class is arbitrary,
// it only affects scheduling) in `order`.  Workgroups take the slots in order,
// largest units first.
__global__ __launch_bounds__(1024) void schedule_kernel(Dev d) {
  __shared__ int hist[1025];
  const int tid = threadIdx.x;
  for (int i = tid; i < 1025; i += 1024) hist[i] = 0;
  __syncthreads();
  for (int u = tid; u < d.units; u += 1024) atomicAdd(&hist[1023 - min(1023, d.budget[u] >> 5)], 1);
  __syncthreads();
  if (tid == 0) {
    int run = 0;
    for (int c = 0; c < 1024; ++c) {
      const int h = hist[c];
      hist[c] = run;
      run += h;
    }
  }
  __syncthreads();
  for (int u = tid; u < d.units; u += 1024) {
    const int slot = atomicAdd(&hist[1023 - min(1023, d.budget[u] >> 5)], 1);
    d.order[slot] = u;
  }
}

// W wavefronts per workgroup (and per unit), 8 / W workgroups per CU.
//
// The kernel also appends: there is no separate pass over the units before it.  The entry that arrives in this
// step is never streamed from the cache.  Its logits are the dot products of the step's inputs (computed here),
// it joins the merge as one more online-softmax state (max = its logit, sum = 1, accumulator = its value row),
// and its logit is put where the bookkeeping looks for it.  In the steady state (exactly one entry evicted
// per step) it is not even written to the slot behind the unit's entries first: if it survives the eviction its
// rows go straight from the inputs into the victim's slot, otherwise only its position is logged.  In the
// other cases (no eviction, several evictions, units too long for the register paths) it is written to
// slot n at the start of the unit, before anything reads that slot.
template <int W>
__global__ __launch_bounds__(64 * W, 2) void unit_kernel(Dev d, const uint16_t* __restrict__ q, void* out,
                                                             uint32_t call_flags, int advance, int lds_main,
                                                             const uint16_t* __restrict__ v_new,
                                                             const uint16_t* __restrict__ k_new) {
  constexpr int NT = 64 * W;
  constexpr int kSlices = W / 2;             // LDS slices the accumulators are merged through, two waves each
  extern __shared__ unsigned char smem[];
  float* lg = reinterpret_cast<float*>(smem);
  uint32_t* evm = reinterpret_cast<uint32_t*>(smem + lds_main);
  // the segment-table rows of this unit and the next (max_seg entries each), behind the eviction mask
  int32_t* s_tbl = reinterpret_cast<int32_t*>(smem + lds_main + ((d.cap + 31) / 32) * 4);
  // staging tiles for spilled logits while streaming, accumulator slices afterwards
  constexpr int kStageFloats = W * kMaxGroup * kLgRow, kOutFloats = kSlices * kMaxGroup * kDim;
  __shared__ float s_buf[kStageFloats > kOutFloats ? kStageFloats : kOutFloats];
  float* s_out = s_buf;
  __shared__ float s_ml[W + 1][kMaxGroup][2];   // row W: the step's new entry when it is merged as a state of its own
  __shared__ __align__(16) float sM[kMaxGroup];
  __shared__ __align__(16) float sInv[kMaxGroup];
  __shared__ float s_tab[kTabLds];
  __shared__ RedBuf rb;
  __shared__ int sh[8];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int G = d.G;
  const int max_seg = d.max_seg;
  const int n_units = d.units;
  const int t = d.sc[SC_T];
  const int s_tab_n = min(kTabLds, d.tab_last + 1);
  for (int i = tid; i < s_tab_n; i += NT) s_tab[i] = d.tab[i];
  __syncthreads();

  // Work distribution: schedule slots (units by descending budget) are taken from a shared queue, except
  // for the first three rounds, which are static (slot = round * grid + workgroup).  A slot is claimed
  // three units ahead and its entry fetched two units ahead, so that neither the atomic's return
  // value nor the entry is ever waited for: the claim made while unit r streams is picked up during
  // unit r's bookkeeping, when everything requested before it has long arrived (a wait for one
  // result of the vector memory pipeline is a wait for all results requested before it).
  __shared__ int s_claim;
  const int grid = (int)gridDim.x, wg = (int)blockIdx.x;
  // Which unit a schedule slot holds (all layers: the units by descending budget; one layer: its units in
  // order) and what the unit holds: scalar loads, the unit two iterations and its state one iteration
  // before they are needed.  `lone` = 1: an entry is appended in this step (0: the unit is full, which
  // the status word reports); n counts it.
  auto unit_of = [&](int slot) -> int {
    const int sl = min(slot, n_units - 1);
    const int uu = d.by_order ? d.order[sl] : d.unit0 + sl;
    return slot < n_units ? uu : -1;
  };
  // sg0: the unit's first segment, where every wavefront's first block lies
  auto state_of = [&](int uu, int& nn, int& bb, int& ll, int& sg0) {
    const int us = max(uu, 0);
    const int n_old = d.n[us];
    bb = d.budget[us];
    sg0 = d.tbl[(size_t)us * max_seg];
    ll = n_old < unit_cap(d, us) ? 1 : 0;
    nn = n_old + ll;
  };
  int u, n, B, lone, seg0, u1, n1 = 0, B1 = 0, lone1 = 0, seg01 = 0;
  u = unit_of(wg);
  state_of(u, n, B, lone, seg0);
  u1 = unit_of(grid + wg);
  // The table row of the unit in hand sits in LDS (s_tbl + cur * max_seg); the next unit's row is asked for at
  // the top of the unit before it, into a register, and put into the other half when that unit is done.
  int cur = 0;
  if (tid < max_seg) s_tbl[tid] = d.tbl[(size_t)max(u, 0) * max_seg + tid];
  int slot2 = 2 * grid + wg;                                   // slot of the unit after next
  // Per-lane values are re-derived, from a copy of the lane index the compiler cannot see through, at
  // the start of every phase that needs them: otherwise they are computed once, kept alive across the
  // whole unit loop, and spilled, and every reload of a spilled register waits for all loads in flight.
  int slane = lane;
  asm volatile("" : "+v"(slane));
  KFrag ka;
  VFrag va;
  bf16x8 qv[4];
  // first block of wave `wave` in a unit of nb blocks (any valid block if the wave has none there)
  auto first_off = [&](int sg, int nn) -> size_t {
    const int nb = (nn + kBlk - 1) / kBlk;
    return (size_t)sg * kSegElems + (size_t)min(wave, max(nb - 1, 0)) * kBlkElems + slane * 8;
  };
  auto load_q = [&](int uu) {
    const int jh = slane & 7;       // columns 8..15 repeat the heads 0..7 (scan_pv<true>)
    const uint16_t* qrow = q + ((size_t)(uu - d.unit0) * G + (jh < G ? jh : 0)) * kDim + 8 * (slane >> 4);
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      // lanes beyond the group read head 0's row: the columns they produce are never looked at, and
      // selecting zeros here would wait for the load on the spot
      qv[s] = as_bf16x8(*reinterpret_cast<const u32x4*>(qrow + 32 * s));
    }
  };
  if (u >= 0) {
    const size_t o = first_off(seg0, n - lone);
    load_k(ka, d.K + o);
    load_v(va, d.V + o);
    load_q(u);
  }
  const bool evict = (call_flags & 1u) != 0;

  __syncthreads();                                 // the first unit's table row is in place
  while (u >= 0) {
    const int32_t* s_row = s_tbl + cur * max_seg;
    const Slots base{s_row};
    // the next unit's table row (this thread's entry of it): asked for first, looked at last
    const int row_next = d.tbl[(size_t)max(u1, 0) * max_seg + min(tid, max_seg - 1)];
    const int ns = n - lone;                       // entries that are streamed: all but the one that arrives now
    // the new entry stays out of the cache until the eviction has chosen its slot (see above); otherwise it is
    // written to slot n - 1 now, by three wavefronts (key row, value row, per-slot state)
    const bool new_in_regs = lone && evict && n - B == 1 && n <= 32 * NT;
    if (lone && !new_in_regs) {
      const uint16_t* krow = k_new + (size_t)(u - d.unit0) * kDim;
      const uint16_t* vrow = v_new + (size_t)(u - d.unit0) * kDim;
      asm volatile("" : "+v"(slane));
      if (wave == 0 && slane < 16)
        *reinterpret_cast<u32x4*>(d.K + base.k(n - 1, slane * 8)) = *reinterpret_cast<const u32x4*>(krow + slane * 8);
      if (wave == (W > 1 ? 1 : 0)) {
        d.V[base.v(n - 1, slane)] = vrow[slane];
        d.V[base.v(n - 1, slane + 64)] = vrow[slane + 64];
      }
      if (wave == (W > 2 ? 2 : 0) && slane == 32) {
        const size_t sn = base + (n - 1);
        d.crf[sn] = 0.0f;
        d.tau[sn] = t;
        d.pos[sn] = t;
        d.flags[sn] = 0;
        d.n[u] = n;
      }
    }
    if (!lone && tid == 0) atomicOr(&d.sc[SC_STATUS], 1);        // the unit is full: nothing was appended
    const int nblk = (ns + kBlk - 1) / kBlk;
    const int n_res = resident_entries(n, G, lds_main);
    const int res_blk = n_res / kBlk;
    const int my_cnt = wave < nblk ? (nblk - wave + W - 1) / W : 0;

    asm volatile("" : "+v"(slane));
    // ---- the unit after next, and the state of the next one: scalar loads, waited for with the first LDS
    // access below, long before they are needed
    const int u2 = unit_of(slot2);
    state_of(u1, n1, B1, lone1, seg01);

    // ---- stream this wave's blocks (wave + W i, i < my_cnt): while block i is computed, block i + 1 is
    // in flight; the last block's successor is the wave's first block of the next unit, so the loads
    // never stop and every load in the loop is unconditional.  (Two blocks ahead was measured too:
    // it lowers the achieved bandwidth.)
    f32x4 acc[8];
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) acc[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    float m_run = -INFINITY, l_run = 0.f;
    // block b of the unit: segment b / 8 (from the row in LDS), block b % 8 inside it
    auto blk_off = [&](int b) -> size_t {
      return (size_t)s_row[b >> 3] * kSegElems + (size_t)(b & (kSegBlocks - 1)) * kBlkElems + slane * 8;
    };
    float* lg_glob = d.logits + (size_t)u * d.cap * G + 4 * min(slane, 8 * G - 1);
    auto qk = [&](int blk, float (&sv)[8]) {
      const bool resident = blk < res_blk;
      float* lds_dst = (call_flags & 2u) ? nullptr : resident ? lg + (size_t)blk * (G * kBlk) : s_buf + wave * (kMaxGroup * kLgRow);
      scan_qk(ka, qv, sv, d.scale_log2e, 0, ns - blk * kBlk, lds_dst, resident ? kBlk : kLgRow,
              resident ? nullptr : lg_glob + (size_t)blk * (G * kBlk), G, slane);
    };
    for (int i = 0; i + 1 < my_cnt; ++i) {
      const int blk = wave + W * i;
      const size_t o_blk = blk_off(blk + W);
      float sv[8];
      qk(blk, sv);
      load_k(ka, d.K + o_blk);
      scan_pv<true>(sv, va, acc, m_run, l_run, slane);
      load_v(va, d.V + o_blk);
    }
    // without a next unit the prefetch reads this unit's first block again and is ignored
    const bool have_next = u1 >= 0;
    const int u_next = have_next ? u1 : u;
    const int n_next = have_next ? n1 - lone1 : ns;
    const size_t o_next = first_off(have_next ? seg01 : seg0, n_next);
    // the new entry's key as one more row for the matrix cores (what a lane holds of row 0 of a key tile: dims
    // 32 s + 8 kg .. + 7) and its value element, requested a block before they are used
    const uint16_t vnew = v_new[(size_t)(u - d.unit0) * kDim + (slane & 63) + 64 * (wave & 1)];
    u32x4 knew[4];
#pragma unroll
    for (int s4 = 0; s4 < 4; ++s4)
      knew[s4] = *reinterpret_cast<const u32x4*>(k_new + (size_t)(u - d.unit0) * kDim + 32 * s4 + 8 * (slane >> 4));
    if (my_cnt > 0) {
      float sv[8];
      qk(wave + W * (my_cnt - 1), sv);
      scan_pv<true>(sv, va, acc, m_run, l_run, slane);
    }
    // the next unit's table row into the free half (every load of the stream has been consumed by now, so the
    // wait for this one, the oldest, costs nothing); the barrier that ends the unit publishes it
    if (tid < max_seg) s_tbl[(cur ^ 1) * max_seg + tid] = row_next;
    // The next unit's first block, its queries and the claim of the slot three units ahead are requested
    // once this unit's weights sit in registers (the block's 64 registers are free until then, which is
    // what lets units of up to 32 entries per thread stay in registers); they arrive during the
    // bisection.  The claim's result is picked up after the bisection.
    int claimed = 0;
    auto request_next = [&]() {
      load_k(ka, d.K + o_next);
      load_v(va, d.V + o_next);
      load_q(u_next);
      if (tid == 0) claimed = atomicAdd(&d.sc[SC_QUEUE], 1);
    };
    int ftid = tid;
    asm volatile("" : "+v"(ftid));

    // rows g + 8 of the accumulators hold the products of the probabilities' low terms (scan_pv<true>): they
    // sit 32 lanes up and join the rows g of the high terms here, once per unit
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) {
#pragma unroll
      for (int v = 0; v < 4; ++v) acc[dt][v] += __shfl_down(acc[dt][v], 32);
    }
    l_run += __shfl_xor(l_run, 16);
    l_run += __shfl_xor(l_run, 32);
    // Scaled logits of the new entry, head g in lane g: the same matrix-core products as for a cached key (the
    // key sits in row 0 of an otherwise empty tile), so that a key equal to a cached one gets the same bits
    // and ties between them are broken by position, as the definition says.
    float snew;
    {
      asm volatile("" : "+v"(slane));
      const bool row0 = (slane & 15) == 0;
      f32x4 s0 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int s4 = 0; s4 < 4; ++s4) {
        const u32x4 x = row0 ? knew[s4] : u32x4{0u, 0u, 0u, 0u};
        s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(x), qv[s4], s0, 0, 0, 0);
      }
      snew = s0[0] * d.scale_log2e;                   // lane (j, kg = 0) = lane j: row 0, head j
    }
    asm volatile("" : "+v"(slane));
    const int j = slane & 15, kg = slane >> 4;
    if (j < G && kg == 0) {
      s_ml[wave][j][0] = m_run;
      s_ml[wave][j][1] = l_run;
    }
    if (ftid < G) {
      s_ml[W][ftid][0] = lone ? snew : -INFINITY;
      s_ml[W][ftid][1] = lone ? 1.f : 0.f;
    }
    __syncthreads();
    // the new entry's logit where the bookkeeping looks for it: its column of its block.  After the barrier: the
    // wavefront that streamed that block has written the block's rows (with the column masked) by now
    if (ftid < G && lone && !(call_flags & 2u)) {
      const int bn = (n - 1) / kBlk, col = (n - 1) & (kBlk - 1);
      if (bn < res_blk)
        lg[(size_t)bn * (G * kBlk) + ftid * kBlk + col] = snew;
      else
        d.logits[(size_t)u * d.cap * G + (size_t)bn * (G * kBlk) + ftid * kBlk + col] = snew;
    }

    // ---- merge the four online-softmax states -> out.  Every thread derives the global max and
    // denominator of the heads it needs from s_ml (same fixed order everywhere); waves 0 and 1 deposit
    // their rescaled accumulators in two LDS slices, waves 2 and 3 add theirs on top.
    asm volatile("" : "+v"(ftid));
    if (ftid < G) {
      float M = -INFINITY;
      for (int w = 0; w < W + 1; ++w) M = fmaxf(M, s_ml[w][ftid][0]);
      float L = 0.f;
      for (int w = 0; w < W + 1; ++w) {
        const float m = s_ml[w][ftid][0];
        L += m > -INFINITY ? s_ml[w][ftid][1] * fast_exp2(m - M) : 0.f;
      }
      sM[ftid] = M;
      sInv[ftid] = 1.0f / L;
    }
    {
      float sc[4];
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int head = min(4 * kg + v, kMaxGroup - 1);
        float M = -INFINITY;
#pragma unroll
        for (int w = 0; w < W + 1; ++w) M = fmaxf(M, s_ml[w][head][0]);
        const float m = s_ml[wave][head][0];
        sc[v] = m > -INFINITY ? fast_exp2(m - M) : 0.f;
      }
      float* slice = s_out + (wave % kSlices) * (kMaxGroup * kDim);
      for (int half = 0; half < 2; ++half) {
        if ((wave / kSlices) == half) {
#pragma unroll
          for (int v = 0; v < 4; ++v) {
            const int head = 4 * kg + v;
            if (head < G) {
#pragma unroll
              for (int dt = 0; dt < 8; ++dt) {
                float* dst = &slice[head * kDim + 16 * dt + j];
                const float x = acc[dt][v] * sc[v];
                *dst = half == 0 ? x : *dst + x;
              }
            }
          }
        }
        __syncthreads();
      }
    }
    for (int o = ftid; o < G * kDim; o += NT) {
      const int g = o >> 7;
      float y = s_out[o];
      if (kSlices == 2) y += s_out[kMaxGroup * kDim + o];
      if (lone) y += fast_exp2(s_ml[W][g][0] - sM[g]) * __uint_as_float((uint32_t)vnew << 16);
      y *= sInv[g];
      const size_t oi = (size_t)(u - d.unit0) * G * kDim + o;
      if (d.out_bf16)
        reinterpret_cast<__bf16*>(out)[oi] = (__bf16)y;
      else
        reinterpret_cast<float*>(out)[oi] = y;
    }

    // ---- mean attention weights, then Alg. 1 Steps 1-4.  The thread index is laundered so that the
    // compiler derives this phase's per-lane addresses here instead of keeping them alive, in
    // registers the streaming loop needs, across the whole unit loop.
    asm volatile("" : "+v"(ftid));
    int phase = 0;      // block reductions of different units are separated by barriers
    const ValFused val{lg, lg + (size_t)n_res * G, n_res, G * kBlk};
    const float invG = 1.0f / (float)G;
    const NewEntry ne{new_in_regs ? k_new + (size_t)(u - d.unit0) * kDim : nullptr, v_new + (size_t)(u - d.unit0) * kDim};
    const float* lgg = d.logits + (size_t)u * d.cap * G;
    // mean weights of the four consecutive entries e0 .. e0 + 3 (one 16-byte read per head; the heads'
    // maxima and reciprocal denominators are read as four 16-byte vectors per group, not once per use)
    auto weights4 = [&](int e0, float* a4) {
      f32x4 x[kMaxGroup];
      const int off = (e0 >> 5) * (G * kBlk) + (e0 & 31);
      const f32x4 ninf = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
      if (e0 < n_res) {
#pragma unroll
        for (int g = 0; g < kMaxGroup; ++g) x[g] = g < G ? *reinterpret_cast<const f32x4*>(lg + off + g * kBlk) : ninf;
      } else {
#pragma unroll
        for (int g = 0; g < kMaxGroup; ++g)
          x[g] = (g < G && e0 < n) ? *reinterpret_cast<const f32x4*>(lgg + off + g * kBlk) : ninf;
      }
      const f32x4 hM[2] = {*reinterpret_cast<const f32x4*>(sM), *reinterpret_cast<const f32x4*>(sM + 4)};
      const f32x4 hInv[2] = {*reinterpret_cast<const f32x4*>(sInv), *reinterpret_cast<const f32x4*>(sInv + 4)};
      f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int g = 0; g < kMaxGroup; ++g) {
        if (g < G) {                      // uniform; heads in ascending order, as everywhere
#pragma unroll
          for (int e = 0; e < 4; ++e) acc[e] += fast_exp2(x[g][e] - hM[g >> 2][g & 3]) * hInv[g >> 2][g & 3];
        }
      }
#pragma unroll
      for (int e = 0; e < 4; ++e) a4[e] = (e0 + e < n) ? acc[e] * invG : 0.f;
    };
    // R entries per thread.  The groups' state that was not requested at the unit's start is requested
    // after the weights have been computed (fewer live registers) and arrives during the bisection.
    auto regs_path = [&](auto rc) {
      constexpr int R = decltype(rc)::value, C = R / 4;
      float a[R];
#pragma unroll
      for (int c = 0; c < C; ++c) {
        weights4(4 * (ftid + c * NT), a + 4 * c);
        __builtin_amdgcn_sched_barrier(0);      // one group's logits at a time: keeps the register need flat
      }
      request_next();
      // CRF, tau and position of the thread's groups (in chunks of four groups for the largest units):
      // requested behind the next unit's block, first used after the bisection
      constexpr int CH = C < 4 ? C : 4;
      f32x4 crf[CH];
      i32x4 tau[CH], ps[CH];
#pragma unroll
      for (int c = 0; c < CH; ++c) load_meta<NT>(d, base, n, t, c, ftid, crf[c], tau[c], ps[c]);
      // the queue claim is picked up after the bisection: by then everything requested before it has arrived
      auto publish = [&]() {
        if (ftid == 0) s_claim = 3 * grid + claimed;
      };
      lrfu_regs<R, CH, CH, ValFused, NT>(d, u, base, n, B, t, a, crf, tau, ps, val, evict, evm, reinterpret_cast<int*>(smem), lds_main / 4,
                                         s_tab, s_tab_n, rb, phase, sh, ftid, publish, ne);
    };
    if (call_flags & 2u) {               // attention only: no bookkeeping, just keep the stream and the queue going
      request_next();
      if (ftid == 0) s_claim = 3 * grid + claimed;
    } else if (n <= 8 * NT) {
      regs_path(std::integral_constant<int, 8>{});
    } else if (n <= 16 * NT) {
      regs_path(std::integral_constant<int, 16>{});
    } else if (n <= 32 * NT) {
      regs_path(std::integral_constant<int, 32>{});
    } else {
      for (int e0 = 4 * ftid; e0 < n; e0 += 4 * NT) {
        float a4[4];
        weights4(e0, a4);
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (e0 + e < n) val(e0 + e) = a4[e];
      }
      request_next();
      if (ftid == 0) s_claim = 3 * grid + claimed;
      __syncthreads();
      const u64 sfix = lrfu_update<ValFused, NT>(d, u, base, n, t, val, s_tab, s_tab_n, rb, phase, ftid);
      if (ftid == 0) {
        d.window[u] += sfix;
        d.t_unit[u] = t;
      }
      if (evict && n > B)
        evict_phase<ValFused, NT>(d, u, base, n, B, val, evm, reinterpret_cast<int*>(smem), lds_main / 4, rb, phase, sh, ftid);
      else if (ftid == 0)
        d.nev[u] = 0;
    }

    // ---- next unit
    __syncthreads();          // LDS of this unit is dead before the next unit's logits overwrite it; s_claim is set
    cur ^= 1;
    u = u1;
    n = n1;
    B = B1;
    lone = lone1;
    seg0 = seg01;
    u1 = u2;
    slot2 = __builtin_amdgcn_readfirstlane(s_claim);
  }
  step_epilogue(d, t, advance, tid, 0);
}

}  // namespace ckv
