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
// (max, sum, unnormalised output) go to a partials buffer.  A second, small kernel merges
// the splits in split order (deterministic) and writes the normalised output; the kernel
// boundary makes the partials visible across the chip without fences or atomics.
//
// Rows can be spread over blocks: a block carries QVT/GQ rows, and grid.x enumerates
// (split, row group).  With a short context the K/V re-reads this causes are cheap (they
// hit in L2) and the smaller per-block register footprint wins; with a long context the
// caller picks a larger QVT so that all rows share one pass over K and V.
//
// The number of splits is fixed at launch; the keys per split follow from the current
// context length, which is read from the device state, so a captured launch stays valid
// as the sequence grows.
#pragma once
#include "kernels.hpp"

namespace dmtd {

constexpr int QV_MAX = 16;         // query vectors per KV head one block can carry (and query heads per KV head)
constexpr int ATT_MAX_SPLITS = 64;

// Keys a block covers per iteration: 16 lane groups x 4 keys (head_dim 128) or 32 x 4 (head_dim 64).
template <int HD> struct AttKeysPerIter { static constexpr int value = 4 * (64 / (HD / 8)) * 4; };

// Keys per split for a launch whose last row sees ctx keys (a multiple of the block
// iteration); the split kernel and the merge kernel must agree on it.
__device__ __forceinline__ int att_keys_per_split(int ctx, int n_splits, int kpi) {
  return ((ctx + n_splits - 1) / n_splits + kpi - 1) / kpi * kpi;
}

// One block iteration of the running softmax: 4 keys per lane group (kf, vf: this lane's 8 dims of
// each), scored against every query vector.  After the in-group reduction lane slice sl holds the
// score of key u = sl >> USH, whose position is my_key; keys at or beyond key_end, or beyond the
// row's own position (row i = qv / GQ sees keys <= pos0 + i), are masked.
template <int HD, int QVT>
__device__ __forceinline__ void attn_accumulate(const float (&q)[QVT][8], const float (&kf)[4][8], const float (&vf)[4][8],
                                                int my_key, int key_end, int pos0, int GQ, int QV, int lane, int sl,
                                                float (&m)[QVT], float (&l)[QVT], float (&acc)[QVT][8]) {
  constexpr int LPK = HD / 8, U = 4;
  constexpr int USH = LPK == 16 ? 2 : 1;
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

// End of a wave's key loop: l summed over the distinct (lane group, key) holders, acc over the lane groups.
template <int HD, int QVT>
__device__ __forceinline__ void attn_wave_totals(float (&l)[QVT], float (&acc)[QVT][8]) {
  constexpr int LPK = HD / 8;
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
}

template <typename CT, int HD, int QVT>
__global__ void __launch_bounds__(256) attn_decode_kernel(
    const float* __restrict__ qkv, int ldq, const CT* __restrict__ kc, const CT* __restrict__ vc,
    float* __restrict__ part_o, float* __restrict__ part_ml, int nh, int nkv, int s_max, int n_splits, int qv_stride,
    const DevState* st, int sel, int offset, int r_total) {
  typedef typename Elem<CT>::Raw Raw;
  constexpr int LPK = HD / 8;          // lanes per key (16 or 8)
  constexpr int GPW = 64 / LPK;        // lane groups per wave (4 or 8)
  constexpr int NG = 4 * GPW;          // lane groups per block
  constexpr int U = 4;                 // keys per lane group per iteration
  constexpr int KPI = NG * U;          // keys per block iteration
  static_assert(KPI == AttKeysPerIter<HD>::value, "block iteration size");
  constexpr int USH = LPK == 16 ? 2 : 1;   // after the score reduction, lane slice sl holds key u = sl >> USH

  const int g = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int GQ = nh / nkv;
  const int rpb = QVT / GQ;                                    // rows per block
  const int n_rg = (r_total + rpb - 1) / rpb;
  const int split = blockIdx.x / n_rg, rg = blockIdx.x % n_rg;
  const int r = min(rpb, r_total - rg * rpb), QV = r * GQ;
  const int pos_first = row_base(st, sel, offset);
  const int pos0 = pos_first + rg * rpb;                        // position of this block's first row
  const int ctx = pos0 + r;                                     // keys 0 .. ctx-1 are visible to its last row
  const int kps = att_keys_per_split(pos_first + r_total, n_splits, KPI);
  const int key_begin = split * kps, key_end = min(ctx, key_begin + kps);
  const float scale = rsqrtf((float)HD);

  __shared__ float wacc[4][QVT][HD];
  __shared__ float wm[4][QVT], wl[4][QVT];

  // partials are indexed by the launch-wide query-vector number row * GQ + head
  const size_t slot = (((size_t)b * nkv + g) * ATT_MAX_SPLITS + split) * qv_stride + (size_t)rg * rpb * GQ;
  float* my_o = part_o + slot * HD;
  float* my_ml = part_ml + slot * 2;

  if (key_begin < ctx) {
    const int sl = lane % LPK, grp = wave * GPW + lane / LPK;
    const int my_u = sl >> USH;
    float q[QVT][8];
#pragma unroll
    for (int qv = 0; qv < QVT; ++qv) {
      if (qv < QV) {
        const float* qp = qkv + (size_t)(b * r_total + rg * rpb + qv / GQ) * ldq + (size_t)(g * GQ + qv % GQ) * HD + sl * 8;
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
      attn_accumulate<HD, QVT>(q, kf, vf, my_key, key_end, pos0, GQ, QV, lane, sl, m, l, acc);
    }

    attn_wave_totals<HD, QVT>(l, acc);
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

}

// Merge the splits' partial results: out[row, head, :] = sum_s f_s o_s / sum_s f_s l_s with
// f_s = exp(m_s - max_s m_s), splits taken in order.  One block per (row, KV head, sequence).
template <int HD, typename OT>   // OT: float, or bf16_t (the packed input of the O projection)
__global__ void __launch_bounds__(256) attn_merge_kernel(
    const float* __restrict__ part_o, const float* __restrict__ part_ml, OT* __restrict__ out, int ldo,
    int nh, int nkv, int n_splits, int qv_stride, const DevState* st, int sel, int offset, int r_total) {
  const int i = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x;
  const int GQ = nh / nkv;
  const int pos_first = row_base(st, sel, offset);
  const int kps = att_keys_per_split(pos_first + r_total, n_splits, AttKeysPerIter<HD>::value);
  const int n_act = (pos_first + i + 1 + kps - 1) / kps;          // splits that hold keys visible to row i
  __shared__ float f_s[ATT_MAX_SPLITS][QV_MAX];
  __shared__ float inv_l[QV_MAX];
  const size_t slot0 = ((size_t)b * nkv + g) * ATT_MAX_SPLITS;
  for (int e = tid; e < n_act * GQ; e += 256) {
    const int s2 = e / GQ, j = e % GQ;
    f_s[s2][j] = part_ml[((slot0 + s2) * qv_stride + i * GQ + j) * 2];
  }
  __syncthreads();
  if (tid < GQ) {
    float mm = -INFINITY;
    for (int s2 = 0; s2 < n_act; ++s2) mm = fmaxf(mm, f_s[s2][tid]);
    float ll = 0.f;
    for (int s2 = 0; s2 < n_act; ++s2) {
      const float f = (f_s[s2][tid] == -INFINITY) ? 0.f : __expf(f_s[s2][tid] - mm);
      ll += f * part_ml[((slot0 + s2) * qv_stride + i * GQ + tid) * 2 + 1];
      f_s[s2][tid] = f;
    }
    inv_l[tid] = 1.0f / ll;
  }
  __syncthreads();
  for (int e = tid; e < GQ * HD; e += 256) {
    const int j = e / HD, d = e % HD;
    const float* po = part_o + ((slot0 * qv_stride) + i * GQ + j) * HD + d;
    float o = 0.f;
#pragma unroll 8
    for (int s2 = 0; s2 < n_act; ++s2) {
      const float f = f_s[s2][j];
      const float v = po[(size_t)s2 * qv_stride * HD];
      o += (f == 0.f) ? 0.f : f * v;      // splits without visible keys hold stale partials: weight 0, value ignored
    }
    out[(size_t)(b * r_total + i) * ldo + (size_t)(g * GQ + j) * HD + d] = Elem<OT>::from_f32(o * inv_l[j]);
  }
}

// Short-context variant: ONE kernel per layer does QK-RMSNorm + RoPE of the new rows, the KV-cache
// append, the whole attention over the sequence and the normalisation.  A block is (row group,
// KV head, sequence) and walks all keys itself with NW waves, so there is no split to merge and
// nothing another block must see: the new keys and values are formed in LDS from the raw
// projections (rounded to the cache's type, exactly what later steps will read back) and the
// last row group's block also writes them to the cache.  Used while the K/V of a sequence is
// small enough that a handful of blocks can pull it without starving the chip.
template <typename CT, typename OT, int HD, int QVT, int NW>
__global__ void __launch_bounds__(64 * NW) attn_fused_kernel(
    const float* __restrict__ qkv, int ldq, const void* __restrict__ q_gain, const void* __restrict__ k_gain,
    const double* __restrict__ inv_freq, CT* __restrict__ kc, CT* __restrict__ vc, OT* __restrict__ out, int ldo,
    int nh, int nkv, int s_max, float eps, const DevState* st, int sel, int offset, int r_total) {
  typedef typename Elem<CT>::Raw Raw;
  constexpr int LPK = HD / 8, GPW = 64 / LPK, NG = NW * GPW, U = 4, KPI = NG * U;
  constexpr int USH = LPK == 16 ? 2 : 1;
  constexpr int NEW_MAX = 16;                                   // rows a launch can carry
  const int rg = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int GQ = nh / nkv, rpb = QVT / GQ;
  const int r = min(rpb, r_total - rg * rpb), QV = r * GQ;
  const int pos_first = row_base(st, sel, offset);
  const int pos0 = pos_first + rg * rpb, ctx = pos0 + r;
  const int n_new = rg * rpb + r;                               // new rows whose keys this block's rows can see
  const bool writer = (rg + 1) * rpb >= r_total;                // the last row group's block appends to the cache
  const float scale = rsqrtf((float)HD);

  __shared__ float q_s[QVT][HD];
  __shared__ float knew_s[NEW_MAX][HD], vnew_s[NEW_MAX][HD];
  __shared__ float wacc[NW][QVT][HD];
  __shared__ float wm[NW][QVT], wl[NW][QVT];

  // ---- prologue: per-head RMSNorm + RoPE (pair (i, i + HD/2)) of this block's queries and of the new keys
  {
    constexpr int half = HD / 2;
    const bool act = lane < half;
    const int n_vec = QV + 2 * n_new;                           // queries, new keys, new values
    for (int v = wave; v < n_vec; v += NW) {
      if (v < QV + n_new) {
        const bool is_q = v < QV;
        const int row = is_q ? rg * rpb + v / GQ : v - QV;      // row of the launch
        const int head = is_q ? g * GQ + v % GQ : nh + g;
        const float* src = qkv + (size_t)(b * r_total + row) * ldq + (size_t)head * HD;
        float x0 = act ? src[lane] : 0.f, x1 = act ? src[lane + half] : 0.f;
        const float rs = rsqrtf(wave_sum(x0 * x0 + x1 * x1) / (float)HD + eps);
        if (act) {
          const CT* gn = (const CT*)(is_q ? q_gain : k_gain);
          x0 *= rs * Elem<CT>::to_f32(gn[lane]);
          x1 *= rs * Elem<CT>::to_f32(gn[lane + half]);
          double sn, cs;
          sincos((double)(pos_first + row) * inv_freq[lane], &sn, &cs);
          const float c = (float)cs, sf = (float)sn;
          const float y0 = x0 * c - x1 * sf, y1 = x1 * c + x0 * sf;
          if (is_q) {
            q_s[v][lane] = y0 * scale; q_s[v][lane + half] = y1 * scale;
          } else {
            const CT c0 = Elem<CT>::from_f32(y0), c1 = Elem<CT>::from_f32(y1);
            knew_s[row][lane] = Elem<CT>::to_f32(c0); knew_s[row][lane + half] = Elem<CT>::to_f32(c1);
            if (writer) {
              CT* dst = kc + (((size_t)b * nkv + g) * s_max + pos_first + row) * HD;
              dst[lane] = c0; dst[lane + half] = c1;
            }
          }
        }
      } else {
        const int row = v - QV - n_new;
        const float* src = qkv + (size_t)(b * r_total + row) * ldq + (size_t)(nh + nkv + g) * HD;
        CT* dst = vc + (((size_t)b * nkv + g) * s_max + pos_first + row) * HD;
        for (int k = lane; k < HD; k += 64) {
          const CT cv = Elem<CT>::from_f32(src[k]);
          vnew_s[row][k] = Elem<CT>::to_f32(cv);
          if (writer) dst[k] = cv;
        }
      }
    }
  }
  __syncthreads();

  const int sl = lane % LPK, grp = wave * GPW + lane / LPK;
  const int my_u = sl >> USH;
  float q[QVT][8];
#pragma unroll
  for (int qv = 0; qv < QVT; ++qv)
#pragma unroll
    for (int e = 0; e < 8; ++e) q[qv][e] = qv < QV ? q_s[qv][sl * 8 + e] : 0.f;
  float m[QVT], l[QVT], acc[QVT][8];
#pragma unroll
  for (int qv = 0; qv < QVT; ++qv) {
    m[qv] = -INFINITY; l[qv] = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[qv][e] = 0.f;
  }
  const CT* kbase = kc + (((size_t)b * nkv + g) * s_max) * HD + sl * 8;
  const CT* vbase = vc + (((size_t)b * nkv + g) * s_max) * HD + sl * 8;

  // ---- cached keys 0 .. pos_first-1 (all visible to every row of the block)
  for (int it0 = 0; it0 < pos_first; it0 += KPI) {
    float kf[U][8], vf[U][8];
    {
      Raw kr[U], vr[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int key = it0 + u * NG + grp;
        const bool ok = key < pos_first;
        kr[u] = ok ? Elem<CT>::load_raw(kbase + (size_t)key * HD) : Elem<CT>::zero_raw();
        vr[u] = ok ? Elem<CT>::load_raw(vbase + (size_t)key * HD) : Elem<CT>::zero_raw();
      }
#pragma unroll
      for (int u = 0; u < U; ++u) { Elem<CT>::unpack(kr[u], kf[u]); Elem<CT>::unpack(vr[u], vf[u]); }
    }
    attn_accumulate<HD, QVT>(q, kf, vf, it0 + my_u * NG + grp, pos_first, pos0, GQ, QV, lane, sl, m, l, acc);
  }
  // ---- the new keys pos_first .. ctx-1, from LDS (one iteration: n_new <= 16 <= KPI)
  {
    float kf[U][8], vf[U][8];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int i = u * NG + grp;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        kf[u][e] = i < n_new ? knew_s[i][sl * 8 + e] : 0.f;
        vf[u][e] = i < n_new ? vnew_s[i][sl * 8 + e] : 0.f;
      }
    }
    attn_accumulate<HD, QVT>(q, kf, vf, pos_first + my_u * NG + grp, ctx, pos0, GQ, QV, lane, sl, m, l, acc);
  }

  attn_wave_totals<HD, QVT>(l, acc);
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
  for (int e = tid; e < QV * HD; e += 64 * NW) {
    const int qv = e / HD, d = e % HD;
    float mm = -INFINITY;
#pragma unroll
    for (int w = 0; w < NW; ++w) mm = fmaxf(mm, wm[w][qv]);
    float o = 0.f, ll = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      const float f = (wm[w][qv] == -INFINITY) ? 0.f : __expf(wm[w][qv] - mm);
      o += f * wacc[w][qv][d];
      ll += f * wl[w][qv];
    }
    out[(size_t)(b * r_total + rg * rpb + qv / GQ) * ldo + (size_t)(g * GQ + qv % GQ) * HD + d] = Elem<OT>::from_f32(o / ll);
  }
}

}  // namespace dmtd
