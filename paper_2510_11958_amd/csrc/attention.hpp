// GQA decode attention for gfx950, split over the KV sequence ("split-K") with a
// deterministic in-kernel merge.
//
// One block = (split, KV head g, sequence b) and all query vectors that share that KV
// head: r rows x GQ query heads, QV = r*GQ <= QVT.  K and V rows are read straight from
// HBM into registers with 16-byte per-lane loads: HD/8 lanes cover one key, so a wave
// load instruction fetches 64/(HD/8) adjacent keys (1 KiB contiguous).  A block iteration
// covers 4 keys per lane group; each group scores its keys against every query vector
// (partial dot per lane, summed inside the lane group by shuffles), keeps a running
// softmax (max shared across the wave by shuffles, sum and output per lane group) and
// accumulates p*V for the 8 output dims its lanes own.  At the end the lane groups of a
// wave are summed by shuffles, the 4 waves merge through LDS, and the split's
// (max, sum, unnormalised output) go to a partials buffer; the last block to finish for a
// (b, g) merges the splits in split order and writes the normalised output.
//
// The number of splits is the launch's grid.x; the keys per split follow from the current
// context length, which is read from the device state, so a captured launch stays valid
// as the sequence grows.
#pragma once
#include "kernels.hpp"

namespace dmtd {

constexpr int QV_MAX = 16;         // query vectors per KV head a launch can carry
constexpr int ATT_MAX_SPLITS = 64;

template <typename CT, int HD, int QVT>
__global__ void __launch_bounds__(256) attn_decode_kernel(
    const float* __restrict__ qkv, int ldq, const CT* __restrict__ kc, const CT* __restrict__ vc,
    float* __restrict__ part_o, float* __restrict__ part_ml, unsigned int* __restrict__ counters,
    float* __restrict__ out, int ldo, int nh, int nkv, int s_max,
    const DevState* st, int sel, int offset, int r) {
  typedef typename Elem<CT>::Raw Raw;
  constexpr int LPK = HD / 8;          // lanes per key (16 or 8)
  constexpr int GPW = 64 / LPK;        // lane groups per wave (4 or 8)
  constexpr int NG = 4 * GPW;          // lane groups per block
  constexpr int U = 4;                 // keys per lane group per iteration
  constexpr int KPI = NG * U;          // keys per block iteration
  constexpr int USH = LPK == 16 ? 2 : 1;   // after the score reduction, lane slice sl holds key u = sl >> USH

  const int split = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int GQ = nh / nkv, QV = r * GQ;
  const int pos0 = row_base(st, sel, offset);
  const int ctx = pos0 + r;                                    // keys 0 .. ctx-1 are visible to the last row
  const int kps = ((ctx + (int)gridDim.x - 1) / (int)gridDim.x + KPI - 1) / KPI * KPI;   // keys per split
  const int n_act = (ctx + kps - 1) / kps;
  const int key_begin = split * kps, key_end = min(ctx, key_begin + kps);
  const float scale = rsqrtf((float)HD);

  __shared__ float wacc[4][QVT][HD];
  __shared__ float wm[4][QVT], wl[4][QVT];
  __shared__ bool is_last;

  const size_t slot = ((size_t)b * nkv + g) * ATT_MAX_SPLITS;
  float* my_o = part_o + (slot + split) * QVT * HD;
  float* my_ml = part_ml + (slot + split) * QVT * 2;

  if (key_begin < ctx) {
    const int sl = lane % LPK, grp = wave * GPW + lane / LPK;
    const int my_u = sl >> USH;
    float q[QVT][8];
#pragma unroll
    for (int qv = 0; qv < QVT; ++qv) {
      if (qv < QV) {
        const float* qp = qkv + (size_t)(b * r + qv / GQ) * ldq + (size_t)(g * GQ + qv % GQ) * HD + sl * 8;
        const float4 qa = *(const float4*)qp, qb = *(const float4*)(qp + 4);
        q[qv][0] = qa.x * scale; q[qv][1] = qa.y * scale; q[qv][2] = qa.z * scale; q[qv][3] = qa.w * scale;
        q[qv][4] = qb.x * scale; q[qv][5] = qb.y * scale; q[qv][6] = qb.z * scale; q[qv][7] = qb.w * scale;
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) q[qv][e] = 0.f;
      }
    }
    float m[QVT], l[QVT], acc[QVT][8];
#pragma unroll
    for (int qv = 0; qv < QVT; ++qv) {
      m[qv] = -INFINITY; l[qv] = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[qv][e] = 0.f;
    }
    const CT* kbase = kc + (((size_t)b * nkv + g) * s_max) * HD + sl * 8;
    const CT* vbase = vc + (((size_t)b * nkv + g) * s_max) * HD + sl * 8;

    for (int it0 = key_begin; it0 < key_end; it0 += KPI) {
      float kf[U][8], vf[U][8];
      {
        Raw kr[U], vr[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const int key = it0 + u * NG + grp;
          const bool ok = key < key_end;
          kr[u] = ok ? Elem<CT>::load_raw(kbase + (size_t)key * HD) : Elem<CT>::zero_raw();
          vr[u] = ok ? Elem<CT>::load_raw(vbase + (size_t)key * HD) : Elem<CT>::zero_raw();
        }
#pragma unroll
        for (int u = 0; u < U; ++u) { Elem<CT>::unpack(kr[u], kf[u]); Elem<CT>::unpack(vr[u], vf[u]); }
      }
      const int my_key = it0 + my_u * NG + grp;       // the key whose score this lane will hold
#pragma unroll
      for (int qv = 0; qv < QVT; ++qv) {
        if (qv < QV) {
          float s4[U];
#pragma unroll
          for (int u = 0; u < U; ++u) {
            float d = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) d += q[qv][e] * kf[u][e];
            s4[u] = d;
          }
          // sum over the lane group; the 4 keys' sums end up in 4 different lane slices
          {
            const bool up1 = (sl & (LPK / 2)) != 0;
            const float a0 = (up1 ? s4[2] : s4[0]) + __shfl_xor(up1 ? s4[0] : s4[2], LPK / 2, 64);
            const float a1 = (up1 ? s4[3] : s4[1]) + __shfl_xor(up1 ? s4[1] : s4[3], LPK / 2, 64);
            const bool up2 = (sl & (LPK / 4)) != 0;
            float s = (up2 ? a1 : a0) + __shfl_xor(up2 ? a0 : a1, LPK / 4, 64);
#pragma unroll
            for (int o = LPK / 8; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
            s4[0] = s;
          }
          // causal and range mask: row i = qv / GQ sees keys <= pos0 + i
          float s = s4[0];
          if (my_key >= key_end || my_key > pos0 + qv / GQ) s = -INFINITY;
          float mx = s;
#pragma unroll
          for (int o = LPK / 4; o < 64; o <<= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));   // over keys and lane groups
          const float m_new = fmaxf(m[qv], mx);
          if (m_new != -INFINITY) {
            const float sc = __expf(m[qv] - m_new);           // exp(-inf) = 0 on the first visible key
            const float p = (s == -INFINITY) ? 0.f : __expf(s - m_new);
            l[qv] = l[qv] * sc + p;
            float pu[U];
#pragma unroll
            for (int u = 0; u < U; ++u) pu[u] = __shfl(p, (lane & ~(LPK - 1)) | (u << USH), 64);
#pragma unroll
            for (int e = 0; e < 8; ++e)
              acc[qv][e] = acc[qv][e] * sc + ((pu[0] * vf[0][e] + pu[1] * vf[1][e]) + (pu[2] * vf[2][e] + pu[3] * vf[3][e]));
            m[qv] = m_new;
          }
        }
      }
    }

    // wave totals: l over the distinct (lane group, key) holders, acc over the lane groups
#pragma unroll
    for (int qv = 0; qv < QVT; ++qv) {
      float v = l[qv];
#pragma unroll
      for (int o = LPK / 4; o < 64; o <<= 1) v += __shfl_xor(v, o, 64);
      l[qv] = v;
    }
#pragma unroll
    for (int qv = 0; qv < QVT; ++qv)
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        float v = acc[qv][e];
#pragma unroll
        for (int o = LPK; o < 64; o <<= 1) v += __shfl_xor(v, o, 64);
        acc[qv][e] = v;
      }
    if (lane < LPK) {
#pragma unroll
      for (int qv = 0; qv < QVT; ++qv)
        if (qv < QV) {
#pragma unroll
          for (int e = 0; e < 8; ++e) wacc[wave][qv][sl * 8 + e] = acc[qv][e];
          if (lane == 0) { wm[wave][qv] = m[qv]; wl[wave][qv] = l[qv]; }
        }
    }
    __syncthreads();
    for (int e = tid; e < QV * HD; e += 256) {
      const int qv = e / HD, d = e % HD;
      const float mm = fmaxf(fmaxf(wm[0][qv], wm[1][qv]), fmaxf(wm[2][qv], wm[3][qv]));
      float o = 0.f, ll = 0.f;
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const float f = (wm[w][qv] == -INFINITY) ? 0.f : __expf(wm[w][qv] - mm);
        o += f * wacc[w][qv][d];
        ll += f * wl[w][qv];
      }
      my_o[qv * HD + d] = o;
      if (d == 0) { my_ml[qv * 2] = mm; my_ml[qv * 2 + 1] = ll; }
    }
  }

  // the last block of this (b, g) to arrive merges the splits, in split order
  __threadfence();
  __syncthreads();
  unsigned int* ctr = counters + (size_t)b * nkv + g;
  if (tid == 0) is_last = (atomicAdd(ctr, 1u) == gridDim.x - 1);
  __syncthreads();
  if (!is_last) return;
  __threadfence();
  const float* po = part_o + slot * QVT * HD;
  const float* pml = part_ml + slot * QVT * 2;
  for (int e = tid; e < QV * HD; e += 256) {
    const int qv = e / HD, d = e % HD, i = qv / GQ, j = qv % GQ;
    float mm = -INFINITY;
    for (int s2 = 0; s2 < n_act; ++s2) mm = fmaxf(mm, pml[((size_t)s2 * QVT + qv) * 2]);
    float ll = 0.f, o = 0.f;
    for (int s2 = 0; s2 < n_act; ++s2) {
      const float ms = pml[((size_t)s2 * QVT + qv) * 2];
      if (ms == -INFINITY) continue;
      const float f = __expf(ms - mm);
      ll += f * pml[((size_t)s2 * QVT + qv) * 2 + 1];
      o += f * po[((size_t)s2 * QVT + qv) * HD + d];
    }
    out[(size_t)(b * r + i) * ldo + (size_t)(g * GQ + j) * HD + d] = o / ll;
  }
  if (tid == 0) *ctr = 0u;
}

}  // namespace dmtd
