// GQA decode attention for gfx950, split over the KV sequence ("split-K"), with the
// QK-RMSNorm, the rotary embedding and the KV-cache append of the new rows folded in.
//
// Two launches per layer.  (1) attn_split_kernel: a block = (key range, row group, KV head,
// sequence) and the query vectors of that row group that share the KV head (rows x GQ query
// heads, at most QVT).  Its key range is fixed by the launch (range index x keys per range), so
// the K/V loads of its first iteration are issued at once, together with the load of the
// device-resident position and of the raw q/k/v rows; nothing waits on anything else.  K and V
// rows go straight from HBM into registers with 16-byte per-lane loads: HD/8 lanes cover one key,
// so a wave load instruction fetches 64/(HD/8) adjacent keys (1 KiB contiguous).  While they fly
// the block normalises and rotates its query vectors and the launch's new keys (per-head RMSNorm,
// then RoPE with half-split pairing at the row's absolute position, cos/sin from a table) into LDS; the block whose
// range holds a new position takes that key and value from LDS (rounded to the cache's type,
// exactly what later steps read back) and the last row group's block also writes them to the
// cache.  Scoring: partial dot per lane, summed inside the lane group by shuffles; running softmax
// with the maximum shared across the wave; p*V accumulated for the 8 output dims a lane owns;
// lane groups summed by shuffles, the 4 waves through LDS; the range's (max, sum, unnormalised
// output) go to a partials buffer.  (2) attn_merge_kernel: per (row, query head, sequence), merges the
// ranges in a fixed order (deterministic) and writes the normalised output; all its loads are issued
// before the first one is needed.  The kernel boundary makes the partials visible across the chip
// (fences and same-kernel grid barriers were measured to cost far more on this chip).
//
// Keys beyond the current context inside a block's range are loaded (they lie inside the cache
// allocation) and masked; ranges wholly beyond the context exit early and are skipped by the merge.
#pragma once
#include "kernels.hpp"

namespace dmtd {

constexpr int QV_MAX = 16;         // query vectors per KV head one block can carry (and query heads per KV head)
constexpr int ATT_MAX_SPLITS = 64;

// Keys a block covers per iteration: 16 lane groups x 4 keys (head_dim 128) or 32 x 4 (head_dim 64).
template <int HD> struct AttKeysPerIter { static constexpr int value = 4 * (64 / (HD / 8)) * 4; };


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

// Rotary table, built once: (cos, sin) of position * theta^(-2i/hd), angle and functions in double
// precision, stored rounded to float (what the attention kernel would otherwise compute per launch).
__global__ void rope_table_kernel(const double* __restrict__ inv_freq, float2* __restrict__ tab, int s_max, int half) {
  const size_t n = (size_t)s_max * half;
  for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) {
    double sn, cs;
    sincos((double)(i / half) * inv_freq[i % half], &sn, &cs);
    tab[i] = make_float2((float)cs, (float)sn);
  }
}

// Per-head RMSNorm + RoPE (pair (i, i + HD/2), cos/sin from the table) of a block's QV query vectors
// (rows row0 .. of the launch, GQ heads each, scaled by 1/sqrt(HD)) into q_s and, if the block's key
// range holds new positions, of the launch's first n_new keys and values into knew_s / vnew_s, rounded
// to the cache's type; the writer block also stores them to the cache.  Called by all 4 waves of a block.
template <typename CT, int HD>
__device__ __forceinline__ void attn_prepare_rows(
    const float* __restrict__ qkv, int ldq, const void* __restrict__ q_gain, const void* __restrict__ k_gain,
    const float2* __restrict__ rope_tab, CT* __restrict__ kc, CT* __restrict__ vc, int b, int g, int nh, int nkv, int s_max,
    float eps, int r_total, int row0, int QV, int n_new, bool holds_new, bool writer, int pos_first, int key_begin, int key_end,
    float (*q_s)[HD], float (*knew_s)[HD], float (*vnew_s)[HD], int lane, int wave) {
  constexpr int half = HD / 2;
  const int GQ = nh / nkv;
  const float scale = rsqrtf((float)HD);
  const bool act = lane < half;
  const int n_vec = QV + (holds_new ? 2 * n_new : 0);         // queries, new keys, new values
  for (int v = wave; v < n_vec; v += 4) {
    if (v < QV + n_new) {
      const bool is_q = v < QV;
      const int row = is_q ? row0 + v / GQ : v - QV;          // row of the launch
      const int hcol = is_q ? g * GQ + v % GQ : nh + g;
      const float* src = qkv + (size_t)(b * r_total + row) * ldq + (size_t)hcol * HD;
      float x0 = act ? src[lane] : 0.f, x1 = act ? src[lane + half] : 0.f;
      const float rs = rsqrtf(wave_sum(x0 * x0 + x1 * x1) / (float)HD + eps);
      if (act) {
        const CT* gn = (const CT*)(is_q ? q_gain : k_gain);
        x0 *= rs * Elem<CT>::to_f32(gn[lane]);
        x1 *= rs * Elem<CT>::to_f32(gn[lane + half]);
        const float2 cs = rope_tab[(size_t)(pos_first + row) * half + lane];
        const float c = cs.x, sf = cs.y;
        const float y0 = x0 * c - x1 * sf, y1 = x1 * c + x0 * sf;
        if (is_q) {
          q_s[v][lane] = y0 * scale; q_s[v][lane + half] = y1 * scale;
        } else {
          const CT c0 = Elem<CT>::from_f32(y0), c1 = Elem<CT>::from_f32(y1);
          knew_s[row][lane] = Elem<CT>::to_f32(c0); knew_s[row][lane + half] = Elem<CT>::to_f32(c1);
          const int key = pos_first + row;
          if (writer && key >= key_begin && key < key_end) {
            CT* dst = kc + (((size_t)b * nkv + g) * s_max + key) * HD;
            dst[lane] = c0; dst[lane + half] = c1;
          }
        }
      }
    } else {
      const int row = v - QV - n_new, key = pos_first + row;
      const float* src = qkv + (size_t)(b * r_total + row) * ldq + (size_t)(nh + nkv + g) * HD;
      CT* dst = vc + (((size_t)b * nkv + g) * s_max + key) * HD;
      const bool wr = writer && key >= key_begin && key < key_end;
      for (int k = lane; k < HD; k += 64) {
        const CT cv = Elem<CT>::from_f32(src[k]);
        vnew_s[row][k] = Elem<CT>::to_f32(cv);
        if (wr) dst[k] = cv;
      }
    }
  }
}

// QK-RMSNorm + RoPE + KV append as a launch of its own, for passes that carry more rows per sequence than an attention
// block keeps in LDS (prefill, the whole-sequence forward): per-head RMSNorm and rotation of the rows' keys, and their
// values, rounded to the cache's type and stored; the attention launch that follows then finds every key in the cache
// (do_append = 2).  One wave per (row, KV head).
template <typename CT, int HD>
__global__ void __launch_bounds__(64) kv_append_kernel(
    const float* __restrict__ qkv, int ldq, const void* __restrict__ k_gain, const float2* __restrict__ rope_tab,
    CT* __restrict__ kc, CT* __restrict__ vc, int nh, int nkv, int s_max, float eps, const DevState* st, int sel, int offset, int r_total) {
  constexpr int half = HD / 2;
  const int row_g = blockIdx.x, g = blockIdx.y, lane = threadIdx.x;
  const int b = row_g / r_total, i = row_g % r_total;
  const int key = row_base(st, sel, offset, b) + i;
  const float* ksrc = qkv + (size_t)row_g * ldq + (size_t)(nh + g) * HD;
  const float* vsrc = qkv + (size_t)row_g * ldq + (size_t)(nh + nkv + g) * HD;
  const bool act = lane < half;
  float x0 = act ? ksrc[lane] : 0.f, x1 = act ? ksrc[lane + half] : 0.f;
  const float rs = rsqrtf(wave_sum(x0 * x0 + x1 * x1) / (float)HD + eps);
  CT* kd = kc + (((size_t)b * nkv + g) * s_max + key) * HD;
  CT* vd = vc + (((size_t)b * nkv + g) * s_max + key) * HD;
  if (act) {
    const CT* gn = (const CT*)k_gain;
    x0 *= rs * Elem<CT>::to_f32(gn[lane]);
    x1 *= rs * Elem<CT>::to_f32(gn[lane + half]);
    const float2 cs = rope_tab[(size_t)key * half + lane];
    kd[lane] = Elem<CT>::from_f32(x0 * cs.x - x1 * cs.y);
    kd[lane + half] = Elem<CT>::from_f32(x1 * cs.x + x0 * cs.y);
  }
  for (int k = lane; k < HD; k += 64) vd[k] = Elem<CT>::from_f32(vsrc[k]);
}

template <typename CT, int HD, int QVT>
__global__ void __launch_bounds__(256) attn_split_kernel(
    const float* __restrict__ qkv, int ldq, const void* __restrict__ q_gain, const void* __restrict__ k_gain,
    const float2* __restrict__ rope_tab /* [s_max][HD / 2] (cos, sin) of position * theta^(-2i/HD) */, CT* __restrict__ kc, CT* __restrict__ vc,
    float* __restrict__ part_o, float* __restrict__ part_ml, int nh, int nkv, int s_max, float eps,
    int kps /* keys per range, a multiple of the block iteration */, int n_splits, int qv_stride,
    const DevState* st, int sel, int offset, int r_total,
    int do_append /* 1: the launch appends its rows' keys and values; 0: it scores them from its inputs and leaves the cache untouched (measurement); 2: they are in the cache already */,
    const int* __restrict__ fmap /* nullable: launch sequence -> sequence slot (cache rows, positions) */) {
  typedef typename Elem<CT>::Raw Raw;
  constexpr int LPK = HD / 8;          // lanes per key (16 or 8)
  constexpr int GPW = 64 / LPK;        // lane groups per wave (4 or 8)
  constexpr int NG = 4 * GPW;          // lane groups per block
  constexpr int U = 4;                 // keys per lane group per iteration
  constexpr int KPI = NG * U;          // keys per block iteration
  static_assert(KPI == AttKeysPerIter<HD>::value, "block iteration size");
  constexpr int USH = LPK == 16 ? 2 : 1;   // after the score reduction, lane slice sl holds key u = sl >> USH
  constexpr int NEW_MAX = 16;          // rows a launch can carry

  const int g = blockIdx.y, b = blockIdx.z;
  // rows and partials are indexed by the launch's sequence number b, the cache and the positions by the sequence's slot:
  // the cache pointers are moved so that index b lands on the slot
  const int bs = fmap ? fmap[b] : b;
  kc += (ptrdiff_t)(bs - b) * nkv * s_max * HD;
  vc += (ptrdiff_t)(bs - b) * nkv * s_max * HD;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int GQ = nh / nkv;
  const int rpb = QVT / GQ;                                    // rows per block
  const int n_rg = (r_total + rpb - 1) / rpb;
  const int split = blockIdx.x / n_rg, rg = blockIdx.x % n_rg;
  const int r = min(rpb, r_total - rg * rpb), QV = r * GQ;
  const int key_begin = split * kps;
  const int sl = lane % LPK, grp = wave * GPW + lane / LPK;
  const int my_u = sl >> USH;

  __shared__ float q_s[QVT][HD];
  __shared__ float knew_s[NEW_MAX][HD], vnew_s[NEW_MAX][HD];
  __shared__ float wacc[4][QVT][HD];
  __shared__ float wm[4][QVT], wl[4][QVT];

  // K/V of the first iteration: addresses depend on the launch only
  const CT* kbase = kc + (((size_t)b * nkv + g) * s_max) * HD + sl * 8;
  const CT* vbase = vc + (((size_t)b * nkv + g) * s_max) * HD + sl * 8;
  Raw kr[U], vr[U];
  auto load_kv = [&](int it0, int limit) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int key = it0 + u * NG + grp;
      const bool ok = key < limit;
      kr[u] = ok ? Elem<CT>::load_raw(kbase + (size_t)key * HD) : Elem<CT>::zero_raw();
      vr[u] = ok ? Elem<CT>::load_raw(vbase + (size_t)key * HD) : Elem<CT>::zero_raw();
    }
  };
  load_kv(key_begin, min(s_max, key_begin + kps));

  const int pos_first = row_base(st, sel, offset, bs);
  const int pos0 = pos_first + rg * rpb;                        // position of this block's first row
  const int ctx = pos0 + r;                                     // keys 0 .. ctx-1 are visible to its last row
  if (key_begin >= ctx) return;                                 // whole range beyond the context (block-uniform)
  const int key_end = min(ctx, key_begin + kps);
  const int n_new = rg * rpb + r;                               // new rows whose keys this block's rows can see
  const bool holds_new = do_append != 2 && key_end > pos_first; // a new position, not yet in the cache, falls into this range
  const bool writer = do_append == 1 && (rg + 1) * rpb >= r_total;   // the last row group's blocks append to the cache
  const float scale = rsqrtf((float)HD);

  attn_prepare_rows<CT, HD>(qkv, ldq, q_gain, k_gain, rope_tab, kc, vc, b, g, nh, nkv, s_max, eps, r_total, rg * rpb, QV, n_new, holds_new,
                            writer, pos_first, key_begin, key_end, q_s, knew_s, vnew_s, lane, wave);
  __syncthreads();

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

  for (int it0 = key_begin; it0 < key_end; it0 += KPI) {
    float kf[U][8], vf[U][8];
#pragma unroll
    for (int u = 0; u < U; ++u) { Elem<CT>::unpack(kr[u], kf[u]); Elem<CT>::unpack(vr[u], vf[u]); }
    if (it0 + KPI < key_end) load_kv(it0 + KPI, key_end);       // next iteration's keys fly during the scoring
    if (holds_new) {
      // new positions: key and value come from LDS, not from the cache slot (written by another block, or not yet)
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int i = it0 + u * NG + grp - pos_first;
        if (i >= 0 && i < n_new) {
#pragma unroll
          for (int e = 0; e < 8; ++e) { kf[u][e] = knew_s[i][sl * 8 + e]; vf[u][e] = vnew_s[i][sl * 8 + e]; }
        }
      }
    }
    attn_accumulate<HD, QVT>(q, kf, vf, it0 + my_u * NG + grp, key_end, pos0, GQ, QV, lane, sl, m, l, acc);
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
  // partials are indexed by the launch-wide query-vector number row * GQ + head
  const size_t slot = (((size_t)b * nkv + g) * ATT_MAX_SPLITS + split) * qv_stride + (size_t)rg * rpb * GQ;
  float* my_o = part_o + slot * HD;
  float* my_ml = part_ml + slot * 2;
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

// Merge the ranges' partial results: out[row, head, :] = sum_s f_s o_s / sum_s f_s l_s with
// f_s = exp(m_s - max_s m_s).  One block (256 threads) per (row, query head, sequence): thread (group, d4) takes
// 4 consecutive d of the ranges group, group + NG, ...; every load is issued before the first one is needed; the
// maximum and the denominator are wave reductions over one lane per range; the groups' sums are added in group
// order through LDS (deterministic).
template <int HD, typename OT>   // OT: float, or bf16_t (the packed input of the O projection: high parts to out, low parts to out_lo)
__global__ void __launch_bounds__(256) attn_merge_kernel(
    const float* __restrict__ part_o, const float* __restrict__ part_ml, OT* __restrict__ out, OT* __restrict__ out_lo, int ldo,
    int nh, int nkv, int kps, int n_splits, int qv_stride, const DevState* st, int sel, int offset, int r_total,
    const int* __restrict__ fmap /* nullable: launch sequence -> sequence slot (positions) */) {
  constexpr int T4 = HD / 4;              // threads per group: one per 4 consecutive d
  constexpr int NG = 256 / T4;            // groups (8 or 16); group sg takes ranges sg, sg + NG, ...
  constexpr int PRE = 4;                  // ranges per thread fetched before anything is waited for (4 * NG >= 32 ranges)
  static_assert(ATT_MAX_SPLITS <= 64, "one wave holds a lane per range");
  const int i = blockIdx.x, head = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x;
  const int GQ = nh / nkv, g = head / GQ, j = head % GQ;
  const int sg = tid / T4, d = (tid % T4) * 4;
  __shared__ float f_s[ATT_MAX_SPLITS];
  __shared__ float inv_l_s;
  __shared__ __attribute__((aligned(16))) float red[NG][HD];
  const size_t slot0 = ((size_t)b * nkv + g) * ATT_MAX_SPLITS;
  const size_t qv = (size_t)i * GQ + j;
  float mv = -INFINITY, lv = 0.f;
  {
    const float2 ml = *(const float2*)(part_ml + ((slot0 + (tid < n_splits ? tid : 0)) * qv_stride + qv) * 2);
    if (tid < n_splits) { mv = ml.x; lv = ml.y; }
  }
  const float* po = part_o + ((slot0 + sg) * qv_stride + qv) * HD + d;
  const size_t po_step = (size_t)NG * qv_stride * HD;
  f32x4 ov[PRE];
#pragma unroll
  for (int u = 0; u < PRE; ++u) {
    // unconditional, from a clamped range index (a range beyond n_splits gets factor 0 below): a load under a
    // per-lane condition would be waited for on the spot, one memory round trip after the other
    const int uc = sg + u * NG < n_splits ? u : 0;
    ov[u] = *(const f32x4*)(po + uc * po_step);
  }
  const int pos_row = row_base(st, sel, offset, fmap ? fmap[b] : b) + i;    // row i sees keys 0 .. pos_row
  const int n_act = min(n_splits, pos_row / kps + 1);   // ranges that hold keys visible to row i; later ones hold stale partials
  if (tid < 64) {
    // the first wave holds one range per lane: maximum and weighted sum by shuffles (a fixed tree: deterministic)
    const float m_l = tid < n_act ? mv : -INFINITY;
    const float mm = wave_max(m_l);
    const float f = (m_l != -INFINITY) ? __expf(m_l - mm) : 0.f;
    f_s[tid] = f;
    const float ll = wave_sum(f == 0.f ? 0.f : f * lv);     // a skipped range may hold anything
    if (tid == 0) inv_l_s = 1.0f / ll;
  }
  __syncthreads();
  f32x4 o = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int u = 0; u < PRE; ++u) {
    const int s2 = sg + u * NG;
    const float f = s2 < n_act ? f_s[s2] : 0.f;
    if (f != 0.f) o += f * ov[u];
  }
  for (int s2 = sg + PRE * NG; s2 < n_act; s2 += NG) {
    const float f = f_s[s2];
    if (f != 0.f) o += f * *(const f32x4*)(po + (size_t)(s2 / NG) * po_step);
  }
  *(f32x4*)&red[sg][d] = o;
  __syncthreads();
  if (tid < T4) {
    f32x4 t = *(const f32x4*)&red[0][d];
#pragma unroll
    for (int q = 1; q < NG; ++q) t += *(const f32x4*)&red[q][d];
    const size_t at = (size_t)(b * r_total + i) * ldo + (size_t)head * HD + d;
    const float inv_l = inv_l_s;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float res = t[e] * inv_l;
      const OT hi = Elem<OT>::from_f32(res);
      out[at + e] = hi;
      if (out_lo) out_lo[at + e] = Elem<OT>::from_f32(res - Elem<OT>::to_f32(hi));
    }
  }
}

}  // namespace dmtd
