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
  __shared__ float s_out[2][kMaxGroup * kDim];
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

  int u = idx < n_units ? d.order[idx] : 0;
  int n = idx < n_units ? d.n[u] : 0;

  while (idx < n_units) {
    // ---- claim the unit after next; look at the next one (its first blocks get prefetched)
    int claimed = 0;
    if (tid == 0) claimed = atomicAdd(&d.sc[SC_QUEUE], 1);
    const bool have_next = idx_next < n_units;
    const int u_next = have_next ? d.order[idx_next] : u;
    const int n_next = have_next ? d.n[u_next] : n;

    const int B = d.budget[u];
    const int nblk = (n + kBlk - 1) / kBlk;
    const int n_res = resident_entries(n, G, lds_main);
    const int res_blk = n_res / kBlk;
    const int my_cnt = wave < nblk ? (nblk - wave + 3) / 4 : 0;

    // ---- stream this wave's blocks
    int slane = lane;
    asm volatile("" : "+v"(slane));
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
      const uint16_t* kcur = d.K + (size_t)u * unit_elems + slane * 8;
      const uint16_t* vcur = d.V + (size_t)u * unit_elems + slane * 8;
      float* lg_glob = d.logits + (size_t)u * d.cap * G + 4 * min(slane, 8 * G - 1);
      KFrag ka;
      VFrag va;
      load_k(ka, kcur + (size_t)wave * kBlkElems);
      load_v(va, vcur + (size_t)wave * kBlkElems);
      for (int i = 0; i < my_cnt; ++i) {
        const int blk = wave + 4 * i;
        const int nb = (i + 1 == my_cnt) ? blk : blk + 4;     // after the last block: read it once more (keeps the loads unconditional)
        const bool resident = blk < res_blk;
        float* lds_dst = resident ? lg + (size_t)blk * (G * kBlk) : s_stage[wave];
        float sv[8];
        scan_qk(ka, qv, sv, d.scale_log2e, 0, n - blk * kBlk, lds_dst, resident ? kBlk : kLgRow,
                resident ? nullptr : lg_glob + (size_t)blk * (G * kBlk), G, slane);
        load_k(ka, kcur + (size_t)nb * kBlkElems);
        scan_pv(sv, va, acc, m_run, l_run, slane);
        load_v(va, vcur + (size_t)nb * kBlkElems);
      }
    }
    // the bookkeeping below is short and latency-bound: let it win the issue slots over the other
    // workgroup's streaming wavefronts, which mostly wait on memory anyway
    __builtin_amdgcn_s_setprio(3);
    l_run += __shfl_xor(l_run, 16);
    l_run += __shfl_xor(l_run, 32);
    if (head_lane && kg == 0) {
      s_ml[wave][j][0] = m_run;
      s_ml[wave][j][1] = l_run;
    }
    __syncthreads();

    // ---- merge the four online-softmax states -> out.  Every thread derives the global max and
    // denominator of the heads it needs from s_ml (same fixed order everywhere); waves 0 and 1 deposit
    // their rescaled accumulators in two LDS slices, waves 2 and 3 add theirs on top.
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
    {
      float sc[4];
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int head = min(4 * kg + v, kMaxGroup - 1);
        float M = -INFINITY;
#pragma unroll
        for (int w = 0; w < 4; ++w) M = fmaxf(M, s_ml[w][head][0]);
        const float m = s_ml[wave][head][0];
        sc[v] = m > -INFINITY ? fast_exp2(m - M) : 0.f;
      }
      float* slice = s_out[wave & 1];
      for (int half = 0; half < 2; ++half) {
        if ((wave >> 1) == half) {
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
    for (int o = tid; o < G * kDim; o += kThreads) {
      const int g = o >> 7;
      const float y = (s_out[0][o] + s_out[1][o]) * sInv[g];
      const size_t oi = (size_t)u * G * kDim + o;
      if (d.out_bf16)
        reinterpret_cast<__bf16*>(out)[oi] = (__bf16)y;
      else
        reinterpret_cast<float*>(out)[oi] = y;
    }

    // ---- mean attention weights, then Alg. 1 Steps 1-4.  The thread index is laundered so that the
    // compiler derives this phase's per-lane addresses here instead of keeping them alive, in
    // registers the streaming loop needs, across the whole unit loop.
    int ftid = tid;
    asm volatile("" : "+v"(ftid));
    int phase = 0;      // block reductions of different units are separated by barriers
    const ValFused val{lg, lg + (size_t)n_res * G, n_res, G * kBlk};
    const bool evict = (call_flags & 1u) != 0;
    const float invG = 1.0f / (float)G;
    const float* lgg = d.logits + (size_t)u * d.cap * G;
    auto weight_of = [&](int i) -> float {
      const int off = (i >> 5) * (G * kBlk) + (i & 31);
      float a = 0.f;
      if (i < n_res) {
        for (int g = 0; g < G; ++g) a += fast_exp2(lg[off + g * kBlk] - sM[g]) * sInv[g];
      } else {
        for (int g = 0; g < G; ++g) a += fast_exp2(lgg[off + g * kBlk] - sM[g]) * sInv[g];
      }
      return a * invG;
    };
    // four entries at a time with all their logits in flight together
    auto weights4 = [&](int i0, float* a4) {
      float x[4][kMaxGroup];
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int i = i0 + r * kThreads;
        const int off = (i >> 5) * (G * kBlk) + (i & 31);
        if (i < n_res) {
#pragma unroll
          for (int g = 0; g < kMaxGroup; ++g) x[r][g] = g < G ? lg[off + g * kBlk] : -INFINITY;
        } else {
#pragma unroll
          for (int g = 0; g < kMaxGroup; ++g) x[r][g] = (g < G && i < n) ? lgg[off + g * kBlk] : -INFINITY;
        }
      }
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        float a = 0.f;
#pragma unroll
        for (int g = 0; g < kMaxGroup; ++g)
          if (g < G) a += fast_exp2(x[r][g] - sM[g]) * sInv[g];
        a4[r] = (i0 + r * kThreads < n) ? a * invG : 0.f;
      }
    };
    if (n <= 8 * kThreads) {
      float a[8];
      weights4(ftid, a);
      weights4(ftid + 4 * kThreads, a + 4);
      lrfu_regs<8>(d, u, n, B, t, a, val, evict, evm, reinterpret_cast<int*>(smem), lds_main / 4, s_tab, s_tab_n, rb, phase,
                   sh, ftid);
    } else {
      for (int i = ftid; i < n; i += kThreads) val(i) = weight_of(i);
      __syncthreads();
      const u64 sfix = lrfu_update(d, u, n, t, val, s_tab, s_tab_n, rb, phase, ftid);
      if (ftid == 0) {
        d.window[u] += sfix;
        d.t_unit[u] = t;
      }
      if (evict && n > B)
        evict_phase(d, u, n, B, val, evm, reinterpret_cast<int*>(smem), lds_main / 4, rb, phase, sh, ftid);
      else if (ftid == 0)
        d.nev[u] = 0;
    }

    // ---- next unit
    __builtin_amdgcn_s_setprio(0);
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
