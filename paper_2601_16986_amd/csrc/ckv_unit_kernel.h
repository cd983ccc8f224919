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
// Work: units are taken from a queue in order of descending budget (`d.order`),
// first round statically (unit index = blockIdx.x), then by one atomic per unit.
// The four wavefronts of a workgroup split a unit's 32-entry blocks round robin
// (wave w takes blocks w, w+4, ...), each with its own online softmax state;
// the states are merged through LDS at the end of the unit.  As in the scan
// kernel every load in the streaming loop is unconditional: after a wave's last
// block of a unit the stream continues with its first block of the next unit,
// which therefore is in flight during the bookkeeping.
//
// LDS (dynamic, `lds_main` bytes + mask): the logits tile [block][head][32] f32
// of the first n_res entries; the per-entry value (mean weight, then CRF_temp)
// of a resident entry lives in its head-0 slot, values of the other entries
// follow the tile.  Units whose logits do not fit spill the logits of their
// last blocks to the global logits buffer (same layout as the scan kernel's).
#pragma once
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

// Unit indices by descending budget: counting sort over budget / 32, one
// workgroup.  The order inside a class is arbitrary; it only affects scheduling.
__global__ __launch_bounds__(1024) void order_kernel(Dev d) {
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

__global__ __launch_bounds__(kThreads, 2) void unit_kernel(Dev d, const uint16_t* __restrict__ q, void* out,
                                                           uint32_t call_flags, int advance, int lds_main) {
  extern __shared__ unsigned char smem[];
  float* lg = reinterpret_cast<float*>(smem);
  uint32_t* evm = reinterpret_cast<uint32_t*>(smem + lds_main);
  __shared__ float s_stage[kThreads / 64][kMaxGroup * kLgRow];   // staging tiles for spilled logits
  __shared__ float s_out[kMaxGroup * kDim];
  __shared__ float s_ml[kThreads / 64][kMaxGroup][2];
  __shared__ float sM[kMaxGroup], sInv[kMaxGroup];
  __shared__ float s_tab[kTabLds];
  __shared__ RedBuf rb;
  __shared__ int sh[8];
  __shared__ int s_idx[2];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int j = lane & 15, kg = lane >> 4;
  const int G = d.G;
  const bool head_lane = j < G;
  const int jq = head_lane ? j : 0;
  const size_t unit_elems = (size_t)d.cap * kDim;
  const int n_units = d.units;
  const int t = d.sc[SC_T];
  const int s_tab_n = min(kTabLds, d.tab_last + 1);
  if (tid < s_tab_n) s_tab[tid] = d.tab[tid];
  if (tid == 0) {
    s_idx[0] = blockIdx.x;
    s_idx[1] = atomicAdd(&d.sc[SC_QUEUE], 1);
  }
  __syncthreads();
  int idx = s_idx[0], idx_next = s_idx[1];
  int phase = 0;

  KFrag ka, kb;
  VFrag va;
  int u = idx < n_units ? d.order[idx] : 0;
  int n = idx < n_units ? d.n[u] : 0;
  if (idx < n_units) {
    const int nblk0 = (n + kBlk - 1) / kBlk;
    const size_t off = (size_t)u * unit_elems + (size_t)min(wave, max(nblk0 - 1, 0)) * kBlkElems + lane * 8;
    load_k(ka, d.K + off);
    load_v(va, d.V + off);
  }

  while (idx < n_units) {
    // ---- claim the unit after next; look at the next one (its first blocks get prefetched)
    int claimed = 0;
    if (tid == 0) claimed = atomicAdd(&d.sc[SC_QUEUE], 1);
    const bool have_next = idx_next < n_units;
    const int u_next = have_next ? d.order[idx_next] : u;
    const int n_next = have_next ? d.n[u_next] : n;
    const int nblk_next = max((n_next + kBlk - 1) / kBlk, 1);
    const size_t next_off = (size_t)u_next * unit_elems + (size_t)min(wave, nblk_next - 1) * kBlkElems + lane * 8;

    const int B = d.budget[u];
    const int nblk = (n + kBlk - 1) / kBlk;
    const int n_res = resident_entries(n, G, lds_main);
    const int res_blk = n_res / kBlk;
    const int my_cnt = wave < nblk ? (nblk - wave + 3) / 4 : 0;

    // ---- stream this wave's blocks
    f32x4 acc[8];
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) acc[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    float m_run = -INFINITY, l_run = 0.f;
    if (my_cnt > 0) {
      bf16x8 qv[4];
      {
        const uint16_t* qrow = q + ((size_t)u * G + jq) * kDim + 8 * kg;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
          u32x4 x = *reinterpret_cast<const u32x4*>(qrow + 32 * s);
          if (!head_lane) x = u32x4{0u, 0u, 0u, 0u};
          qv[s] = as_bf16x8(x);
        }
      }
      const uint16_t* kcur = d.K + (size_t)u * unit_elems + lane * 8;
      const uint16_t* vcur = d.V + (size_t)u * unit_elems + lane * 8;
      float* lg_glob = d.logits + (size_t)u * d.cap * G + 4 * min(lane, 8 * G - 1);
      int i = 0;
      auto step = [&](const KFrag& kc, KFrag& kn) -> bool {
        const int blk = wave + 4 * i;
        const bool last = i + 1 == my_cnt;
        const uint16_t* kn_ptr = last ? d.K + next_off : kcur + (size_t)(blk + 4) * kBlkElems;
        const uint16_t* vn_ptr = last ? d.V + next_off : vcur + (size_t)(blk + 4) * kBlkElems;
        load_k(kn, kn_ptr);
        const bool resident = blk < res_blk;
        float* lds_dst = resident ? lg + (size_t)blk * (G * kBlk) : s_stage[wave];
        scan_block(kc, va, qv, acc, m_run, l_run, d.scale_log2e, 0, n - blk * kBlk, lds_dst, resident ? kBlk : kLgRow,
                   resident ? nullptr : lg_glob + (size_t)blk * (G * kBlk), G, lane);
        load_v(va, vn_ptr);
        ++i;
        return last;
      };
      bool in_a = true;
      while (true) {
        if (step(ka, kb)) { in_a = false; break; }
        if (step(kb, ka)) { in_a = true; break; }
      }
      if (!in_a) {
#pragma unroll
        for (int r = 0; r < 8; ++r) ka.k[r] = kb.k[r];
      }
    } else {
      load_k(ka, d.K + next_off);       // idle for this unit: just move the prefetch on
      load_v(va, d.V + next_off);
    }
    l_run += __shfl_xor(l_run, 16);
    l_run += __shfl_xor(l_run, 32);
    if (head_lane && kg == 0) {
      s_ml[wave][j][0] = m_run;
      s_ml[wave][j][1] = l_run;
    }
    __syncthreads();

    // ---- merge the four online-softmax states -> out
    if (tid < G) {
      float M = -INFINITY;
      for (int w = 0; w < 4; ++w) M = fmaxf(M, s_ml[w][tid][0]);
      float L = 0.f;
      for (int w = 0; w < 4; ++w) {
        const float m = s_ml[w][tid][0];
        L += m > -INFINITY ? s_ml[w][tid][1] * fast_exp2(m - M) : 0.f;
      }
      sM[tid] = M;
      sInv[tid] = 1.0f / L;
    }
    __syncthreads();
    for (int w = 0; w < 4; ++w) {
      if (wave == w) {
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          const int head = 4 * kg + v;
          if (head < G) {
            const float m = s_ml[w][head][0];
            const float sc = m > -INFINITY ? fast_exp2(m - sM[head]) : 0.f;
#pragma unroll
            for (int dt = 0; dt < 8; ++dt) {
              const float x = acc[dt][v] * sc;
              float* dst = &s_out[head * kDim + 16 * dt + j];
              *dst = (w == 0) ? x : *dst + x;
            }
          }
        }
      }
      __syncthreads();
    }
    for (int o = tid; o < G * kDim; o += kThreads) {
      const int g = o >> 7;
      const float y = s_out[o] * sInv[g];
      const size_t oi = (size_t)u * G * kDim + o;
      if (d.out_bf16)
        reinterpret_cast<__bf16*>(out)[oi] = (__bf16)y;
      else
        reinterpret_cast<float*>(out)[oi] = y;
    }

    // ---- mean attention weight of every entry
    const ValFused val{lg, lg + (size_t)n_res * G, n_res, G * kBlk};
    {
      const float invG = 1.0f / (float)G;
      const float* lgg = d.logits + (size_t)u * d.cap * G;
      for (int i = tid; i < n; i += kThreads) {
        const int off = (i >> 5) * (G * kBlk) + (i & 31);
        const float* row = i < n_res ? lg + off : lgg + off;
        float a = 0.f;
        for (int g = 0; g < G; ++g) a += fast_exp2(row[g * kBlk] - sM[g]) * sInv[g];
        val(i) = a * invG;
      }
    }
    __syncthreads();

    // ---- Alg. 1 Steps 1-3, then Step 4
    const u64 sfix = lrfu_update(d, u, n, t, val, s_tab, s_tab_n, rb, phase, tid);
    if (tid == 0) {
      d.window[u] += sfix;
      d.t_unit[u] = t;
    }
    if ((call_flags & 1u) && n > B)
      evict_phase(d, u, n, B, val, evm, reinterpret_cast<int*>(smem), lds_main / 4, rb, phase, sh, tid);
    else if (tid == 0)
      d.nev[u] = 0;

    // ---- next unit
    if (tid == 0) {
      s_idx[0] = idx_next;
      s_idx[1] = claimed;
    }
    __syncthreads();
    idx = s_idx[0];
    idx_next = s_idx[1];
    u = u_next;
    n = n_next;
    __syncthreads();          // everyone has read s_idx before the next round overwrites it
  }
  step_epilogue(d, t, advance, tid, (int)gridDim.x);
}

}  // namespace ckv
