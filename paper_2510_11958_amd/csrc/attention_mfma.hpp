// Split-K decode attention on the matrix cores, for a bf16 KV cache and up to 16 query vectors per
// KV head (rows of a sequence x query heads that share the KV head), all served by ONE pass over
// K and V.  With several rows per sequence (the refill rows of a full step) the vector kernel runs
// out of registers and of vector ALU throughput; here the 16 query vectors are the 16 columns of
// an MFMA tile, so a block reads each key and value once whatever the number of rows.
//
// Same launch shape, prologue (QK-norm, RoPE, append of the new rows) and partial-result format
// as attn_split_kernel; the same merge kernel follows.  A block = (key range, row group, KV head,
// sequence) with 16 / (query heads per KV head) rows per group (launches with more rows, e.g. prefill
// chunks, read K and V once per group); its 4 waves take interleaved groups of 16 keys.  Per group of 16 keys, in one wave:
//   scores   S^T[key, q] = sum_d K[key, d] Q[q, d]      v_mfma_f32_16x16x32_bf16, K rows as the A
//            operand (a lane loads 8 consecutive d of one key: 16 bytes straight from the cache), the
//            queries as B, each split into a bf16 high and low part (two MFMAs) so that they keep
//            16 mantissa bits; the result leaves lane (q = lane % 16, kq = lane / 16) with the
//            scores of keys 4 kq .. 4 kq + 3 for query q;
//   softmax  running maximum and sum per query in those lanes (maximum across the 4 kq lanes by
//            two shuffles);
//   output   O[q, d] += sum_key P[q, key] V[key, d]     v_mfma_f32_16x16x4_f32 (contraction over 4 keys,
//            one fp32 value per lane and operand, so no operand has to be transposed): for m = 0..3 the A
//            operand is the lane's own p of key 4 kq + m, the B operand the lane's own V[4 kq + m][8 sl + e]
//            (sl = lane % 16; the lane loaded those 8 consecutive d with one 16-byte load), one MFMA
//            per e; accumulator e of lane (sl, kq) holds O[4 kq + j][8 sl + e], j = 0..3.
// Nothing moves between lanes except the maxima and the per-query rescale factors.
#pragma once
#include "attention.hpp"
#include "gemv_mfma.hpp"

namespace dmtd {

// Sum over the 16 lanes of a DPP row by rotations (every lane ends up with the total).
template <int N>
__device__ __forceinline__ float row_ror_f32(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x120 + N, 0xF, 0xF, false));
}
__device__ __forceinline__ float row16_sum(float v) {
  v += row_ror_f32<8>(v);
  v += row_ror_f32<4>(v);
  v += row_ror_f32<2>(v);
  v += row_ror_f32<1>(v);
  return v;
}

constexpr int ATT_QPAD = 8;     // bf16 elements of padding per LDS query row

// A vector of the prologue is handled by the 16 lanes of a DPP row; lane l holds the rotary pairs
// (HL*l + e, HD/2 + HL*l + e), e < HL = HD/32, as two short vectors.
template <int HD> struct AttRowLane {
  static constexpr int HL = HD / 32;
  typedef float fvec_t __attribute__((ext_vector_type(HD / 32)));
  typedef unsigned short hvec_t __attribute__((ext_vector_type(HD / 32)));
};
// Where the launch's q/k/v rows come from: the finished fp32 rows [rows][ldq], or - when the QKV projection ran with K
// split over blocks and left its finishing step to this kernel - the splits' raw partial sums part[split][M][ldp] together
// with what their norm scale is made of (the producer's partial sums of squares ssp[part][ssp_ld] of the projection's
// input rows; scale = rsqrt(sum / K + eps)).  The sum over the splits is taken in split order, as the finishing kernel does.
struct QkvSrc {
  const float* qkv; int ldq;
  const float* part; int ksplit, M, ldp;
  const float* ssp; int n_parts, ssp_ld;
  float inv_k, eps;
};
constexpr int ATT_KSMAX = 8;      // splits fetched at once (the projection splits K at most 8 ways)

// The 2 * HL elements lane l of a 16-lane row holds of the vector at (row_g, element offset col): every load is issued
// before the first use; called by whole 16-lane rows (the scale's sum of squares is a row reduction).
template <int HD>
__device__ __forceinline__ void attn_load_vec(const QkvSrc& q, int row_g, int col, int l,
                                              typename AttRowLane<HD>::fvec_t& xa, typename AttRowLane<HD>::fvec_t& xb) {
  typedef typename AttRowLane<HD>::fvec_t fvec_t;
  constexpr int HL = AttRowLane<HD>::HL, half = HD / 2;
  if (!q.part) {
    const float* src = q.qkv + (size_t)row_g * q.ldq + col + HL * l;
    xa = *(const fvec_t*)src; xb = *(const fvec_t*)(src + half);
    return;
  }
  fvec_t pa[ATT_KSMAX], pb[ATT_KSMAX];
#pragma unroll
  for (int ks = 0; ks < ATT_KSMAX; ++ks) {
    const float* p = q.part + ((size_t)(ks < q.ksplit ? ks : q.ksplit - 1) * q.M + row_g) * q.ldp + col + HL * l;
    pa[ks] = *(const fvec_t*)p; pb[ks] = *(const fvec_t*)(p + half);
  }
  float ss = 0.f;
  for (int p0 = 0; p0 < q.n_parts; p0 += 64) {
    float sp[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int pi = p0 + l + 16 * j;
      sp[j] = q.ssp[(size_t)(pi < q.n_parts ? pi : q.n_parts - 1) * q.ssp_ld + row_g];
    }
#pragma unroll
    for (int j = 0; j < 4; ++j)
      if (p0 + l + 16 * j < q.n_parts) ss += sp[j];
  }
  const float rs = rsqrtf(row16_sum(ss) * q.inv_k + q.eps);
  fvec_t sa = pa[0], sb = pb[0];
#pragma unroll
  for (int ks = 1; ks < ATT_KSMAX; ++ks)
    if (ks < q.ksplit) { sa += pa[ks]; sb += pb[ks]; }
  xa = sa * rs; xb = sb * rs;
}

// The block's query vector of row group lane group grp (if any): loaded before the positions are known.
template <int HD> struct AttQueryPre {
  typename AttRowLane<HD>::fvec_t xa, xb;
  typename AttRowLane<HD>::hvec_t g0, g1;
};
template <int HD>
__device__ __forceinline__ AttQueryPre<HD> attn_preload_query(const QkvSrc& qs, const bf16_t* __restrict__ q_gain,
                                                              int b, int g, int GQ, int r_total, int row0, int QV, int tid) {
  typedef typename AttRowLane<HD>::fvec_t fvec_t;
  typedef typename AttRowLane<HD>::hvec_t hvec_t;
  constexpr int HL = AttRowLane<HD>::HL, half = HD / 2;
  const int l = tid & 15, v = tid >> 4;
  AttQueryPre<HD> p;
#pragma unroll
  for (int e = 0; e < HL; ++e) { p.xa[e] = 0.f; p.xb[e] = 0.f; p.g0[e] = 0; p.g1[e] = 0; }
  if (v < QV) {     // whole 16-lane rows: v is uniform within one
    attn_load_vec<HD>(qs, b * r_total + row0 + v / GQ, (g * GQ + v % GQ) * HD, l, p.xa, p.xb);
    p.g0 = *(const hvec_t*)(q_gain + HL * l); p.g1 = *(const hvec_t*)(q_gain + half + HL * l);
  }
  return p;
}

// Prologue of the matrix-core kernel: per-head RMSNorm + RoPE (pair (i, i + HD/2), cos/sin from the table) of the
// block's QV query vectors, scaled by 1/sqrt(HD) and written to LDS as the B operands of the score MFMAs (bf16 high
// and low parts, a lane's 8 consecutive d are one 16-byte read); and, if the block's key range holds new positions,
// of the launch's first n_new keys and values into knew_s / vnew_s, rounded to the cache's type (the writer block
// also stores them to the cache).  A vector is handled by the 16 lanes of a DPP row, each with HD/32 rotary pairs
// loaded as vectors, so the block's 16 rows take 16 vectors at a time and the sum of squares needs no LDS traffic.
template <int HD>
__device__ __forceinline__ void attn_prepare_rows_mfma(
    const QkvSrc& qs, const bf16_t* __restrict__ q_gain, const bf16_t* __restrict__ k_gain,
    const float2* __restrict__ rope_tab, bf16_t* __restrict__ kc, bf16_t* __restrict__ vc, int b, int g, int nh, int nkv, int s_max,
    float eps, int r_total, int row0, int QV, int n_new, bool holds_new, bool writer, int pos_first, int key_begin, int key_end,
    bf16_t (*qhi_s)[HD + ATT_QPAD], bf16_t (*qlo_s)[HD + ATT_QPAD], float (*knew_s)[HD], float (*vnew_s)[HD], int tid,
    int n_groups /* 16-lane rows in the block */, const AttQueryPre<HD>& pre) {
  constexpr int half = HD / 2;
  constexpr int HL = AttRowLane<HD>::HL;     // rotary pairs per lane (4 or 2): elements HL*l .. and half + HL*l ..
  typedef typename AttRowLane<HD>::fvec_t fvec_t;
  typedef typename AttRowLane<HD>::hvec_t hvec_t;
  const int GQ = nh / nkv;
  const float scale = rsqrtf((float)HD);
  const int l = tid & 15, grp = tid >> 4;    // lane of the row; row of the block (0 .. 15)
  const int n_vec = QV + (holds_new ? 2 * n_new : 0);         // queries, new keys, new values
  for (int v = grp; v < n_vec; v += n_groups) {
    const bool is_q = v < QV, is_k = !is_q && v < QV + n_new;
    const int row = is_q ? row0 + v / GQ : (is_k ? v - QV : v - QV - n_new);       // row of the launch
    const int hcol = is_q ? g * GQ + v % GQ : (is_k ? nh + g : nh + nkv + g);
    fvec_t xa = pre.xa, xb = pre.xb;          // queries (all in the first round: QV <= 16 <= n_groups) were fetched at kernel entry
    if (!is_q) attn_load_vec<HD>(qs, b * r_total + row, hcol * HD, l, xa, xb);
    float x0[HL], x1[HL];
#pragma unroll
    for (int e = 0; e < HL; ++e) { x0[e] = xa[e]; x1[e] = xb[e]; }
    if (!is_q && !is_k) {
      // a value vector: rounded to the cache type, kept for this launch's scores, stored by the writer
      const int key = pos_first + row;
      const bool wr = writer && key >= key_begin && key < key_end;
      bf16_t* dst = vc + (((size_t)b * nkv + g) * s_max + key) * HD + HL * l;
      hvec_t c0, c1;
#pragma unroll
      for (int e = 0; e < HL; ++e) {
        c0[e] = f32_to_bf16(x0[e]); c1[e] = f32_to_bf16(x1[e]);
        vnew_s[row][HL * l + e] = bf16_to_f32(c0[e]); vnew_s[row][half + HL * l + e] = bf16_to_f32(c1[e]);
      }
      if (wr) { *(hvec_t*)dst = c0; *(hvec_t*)(dst + half) = c1; }
      continue;
    }
    hvec_t g0 = pre.g0, g1 = pre.g1;
    if (!is_q) { g0 = *(const hvec_t*)(k_gain + HL * l); g1 = *(const hvec_t*)(k_gain + half + HL * l); }
    const float2* rp = rope_tab + (size_t)(pos_first + row) * half + HL * l;
    float2 cs[HL];
#pragma unroll
    for (int e = 0; e < HL; ++e) cs[e] = rp[e];
    float ss = 0.f;
#pragma unroll
    for (int e = 0; e < HL; ++e) ss += x0[e] * x0[e] + x1[e] * x1[e];
    const float rs = rsqrtf(row16_sum(ss) / (float)HD + eps);
    float y0[HL], y1[HL];
#pragma unroll
    for (int e = 0; e < HL; ++e) {
      const float a0 = x0[e] * (rs * bf16_to_f32(g0[e])), a1 = x1[e] * (rs * bf16_to_f32(g1[e]));
      y0[e] = a0 * cs[e].x - a1 * cs[e].y;
      y1[e] = a1 * cs[e].x + a0 * cs[e].y;
    }
    if (is_q) {
      hvec_t h0, h1, l0, l1;
#pragma unroll
      for (int e = 0; e < HL; ++e) {
        const float q0 = y0[e] * scale, q1 = y1[e] * scale;
        bf16_t hh, ll;
        split_bf16(q0, hh, ll); h0[e] = hh; l0[e] = ll;
        split_bf16(q1, hh, ll); h1[e] = hh; l1[e] = ll;
      }
      *(hvec_t*)&qhi_s[v][HL * l] = h0; *(hvec_t*)&qhi_s[v][half + HL * l] = h1;
      *(hvec_t*)&qlo_s[v][HL * l] = l0; *(hvec_t*)&qlo_s[v][half + HL * l] = l1;
    } else {
      const int key = pos_first + row;
      hvec_t c0, c1;
#pragma unroll
      for (int e = 0; e < HL; ++e) {
        c0[e] = f32_to_bf16(y0[e]); c1[e] = f32_to_bf16(y1[e]);
        knew_s[row][HL * l + e] = bf16_to_f32(c0[e]); knew_s[row][half + HL * l + e] = bf16_to_f32(c1[e]);
      }
      if (writer && key >= key_begin && key < key_end) {
        bf16_t* dst = kc + (((size_t)b * nkv + g) * s_max + key) * HD + HL * l;
        *(hvec_t*)dst = c0; *(hvec_t*)(dst + half) = c1;
      }
    }
  }
}

// NW waves per block take interleaved groups of 16 keys.  FINAL: the launch has ONE key range per (row group, KV head,
// sequence), so the block's result is the attention output itself: it is normalised and written as the packed input
// of the O projection (high parts to out, low parts to out_lo) and no merge kernel follows.  The waves' partial
// results meet in dynamic shared memory: NW * QV * HD floats (QV = the block's query vectors).
template <int HD, int NW, bool FINAL>
__global__ void __launch_bounds__(64 * NW) attn_split_mfma_kernel(
    // in order of first use: the leading 16 dwords of scalars arrive in registers with the wave (kernel-argument preload;
    // an argument struct ends it, so QkvSrc comes last), the rest after a load from the argument buffer
    bf16_t* __restrict__ kc, bf16_t* __restrict__ vc, int nh, int nkv, int s_max,
    int kps /* keys per range, a multiple of 16 * NW */, int r_total,
    const int* __restrict__ fmap /* nullable: launch sequence -> sequence slot (cache rows, positions) */,
    const DevState* st, int sel, int offset, int n_splits, const void* __restrict__ q_gain,
    const void* __restrict__ k_gain, const float2* __restrict__ rope_tab,
    float* __restrict__ part_o, float* __restrict__ part_ml, float eps, int qv_stride, int do_append,
    bf16_t* __restrict__ out, bf16_t* __restrict__ out_lo, int ldo /* FINAL only */, QkvSrc qs) {
  constexpr int QVT = 16;
  constexpr int NT = 64 * NW;
  constexpr int KSTEPS = HD / 32;      // MFMA steps over d for the scores
  constexpr int DPL = HD / 16;         // output dims per lane (8 or 4)
  constexpr int NEW_MAX = 16;
  typedef unsigned int vraw_t __attribute__((ext_vector_type(DPL / 2)));   // DPL bf16 values

  const int g = blockIdx.y, b = blockIdx.z;
  // rows and partials are indexed by the launch's sequence number b, the cache and the positions by the sequence's slot:
  // the cache pointers are moved so that index b lands on the slot (no load, no wait, when there is no map)
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
  const int sl = lane & 15, kq = lane >> 4;

  __shared__ __attribute__((aligned(16))) bf16_t qhi_s[QVT][HD + ATT_QPAD], qlo_s[QVT][HD + ATT_QPAD];
  __shared__ __attribute__((aligned(16))) float knew_s[NEW_MAX][HD], vnew_s[NEW_MAX][HD];
  extern __shared__ float4 att_dyn_smem[];
  float* wacc = (float*)att_dyn_smem;                          // [NW][QV][HD]
  __shared__ float wm[NW][QVT], wl[NW][QVT];

  const bf16_t* kbase = kc + (((size_t)b * nkv + g) * s_max) * HD;
  const bf16_t* vbase = vc + (((size_t)b * nkv + g) * s_max) * HD;
  // K: lane (key = sl, d group kq) per step t: K[key][32 t + 8 kq ..]; V: lane (dims DPL sl .., keys 4 kq + m)
  u32x4 kr[KSTEPS];
  vraw_t vr[4];
  auto load_kv = [&](int base, int limit) {
    const int kkey = base + sl;
#pragma unroll
    for (int t = 0; t < KSTEPS; ++t)
      kr[t] = kkey < limit ? __builtin_nontemporal_load((const u32x4*)(kbase + (size_t)kkey * HD + 32 * t + 8 * kq)) : u32x4{0, 0, 0, 0};
#pragma unroll
    for (int m = 0; m < 4; ++m) {
      const int vkey = base + 4 * kq + m;
      vraw_t z;
#pragma unroll
      for (int e = 0; e < DPL / 2; ++e) z[e] = 0u;
      vr[m] = vkey < limit ? __builtin_nontemporal_load((const vraw_t*)(vbase + (size_t)vkey * HD + DPL * sl)) : z;
    }
  };
  const int range_limit = min(s_max, key_begin + kps);
  load_kv(key_begin + 16 * wave, range_limit);

  // the block's query vectors do not depend on the positions: fetched now, next to K and V
  const AttQueryPre<HD> qpre = attn_preload_query<HD>(qs, (const bf16_t*)q_gain, b, g, GQ, r_total, rg * rpb, QV, tid);

  const int pos_first = row_base(st, sel, offset, bs);
  const int pos0 = pos_first + rg * rpb;                        // position of this block's first row
  const int ctx = pos0 + r;                                     // keys 0 .. ctx-1 are visible to its last row
  if (key_begin >= ctx) return;                                 // whole range beyond the context (block-uniform)
  const int key_end = min(ctx, key_begin + kps);
  const int n_new = rg * rpb + r;                               // new rows whose keys this block's rows can see
  const bool holds_new = do_append != 2 && key_end > pos_first;      // do_append = 2: the rows' keys are in the cache already
  const bool writer = do_append == 1 && (rg + 1) * rpb >= r_total;   // the last row group's blocks append to the cache

  attn_prepare_rows_mfma<HD>(qs, (const bf16_t*)q_gain, (const bf16_t*)k_gain, rope_tab, kc, vc, b, g, nh, nkv, s_max, eps, r_total,
                             rg * rpb, QV, n_new, holds_new, writer, pos_first, key_begin, key_end, qhi_s, qlo_s, knew_s, vnew_s, tid, NT / 16, qpre);
  __syncthreads();

  // queries as B operands: lane (q = sl, d group kq), high and low bf16 parts
  bf16x8_t qhi[KSTEPS], qlo[KSTEPS];
#pragma unroll
  for (int t = 0; t < KSTEPS; ++t) {
    u32x4 h = {0, 0, 0, 0}, lo = h;
    if (sl < QV) {
      h = *(const u32x4*)&qhi_s[sl][32 * t + 8 * kq];
      lo = *(const u32x4*)&qlo_s[sl][32 * t + 8 * kq];
    }
    qhi[t] = __builtin_bit_cast(bf16x8_t, h);
    qlo[t] = __builtin_bit_cast(bf16x8_t, lo);
  }
  const int my_row_pos = pos0 + sl / GQ;                   // query sl belongs to row sl / GQ: it sees keys <= this position
  float m_run = -INFINITY, l_run = 0.f;
  f32x4 acc[DPL];
#pragma unroll
  for (int e = 0; e < DPL; ++e) acc[e] = f32x4{0.f, 0.f, 0.f, 0.f};
  for (int it0 = key_begin; it0 < key_end; it0 += 16 * NW) {
    const int base = it0 + 16 * wave;                           // this wave's 16 keys
    u32x4 ka[KSTEPS];
    float vf[4][DPL];
#pragma unroll
    for (int t = 0; t < KSTEPS; ++t) ka[t] = kr[t];
#pragma unroll
    for (int m = 0; m < 4; ++m)
#pragma unroll
      for (int e = 0; e < DPL / 2; ++e) {
        vf[m][2 * e] = __uint_as_float(vr[m][e] << 16);
        vf[m][2 * e + 1] = __uint_as_float(vr[m][e] & 0xFFFF0000u);
      }
    if (it0 + 16 * NW < key_end) load_kv(base + 16 * NW, key_end);   // the next iteration's keys fly during this one
    if (holds_new) {
      // new positions: key and value come from LDS (the cache slot is written by this launch, maybe not yet)
      const int ik = base + sl - pos_first;
      if (ik >= 0 && ik < n_new) {
#pragma unroll
        for (int t = 0; t < KSTEPS; ++t) {
          const float* src = &knew_s[ik][32 * t + 8 * kq];
          ka[t] = u32x4{pack_bf16x2(src[0], src[1]), pack_bf16x2(src[2], src[3]), pack_bf16x2(src[4], src[5]), pack_bf16x2(src[6], src[7])};
        }
      }
#pragma unroll
      for (int m = 0; m < 4; ++m) {
        const int iv = base + 4 * kq + m - pos_first;
        if (iv >= 0 && iv < n_new) {
#pragma unroll
          for (int e = 0; e < DPL; ++e) vf[m][e] = vnew_s[iv][DPL * sl + e];
        }
      }
    }
    // scores of keys base + 4 kq + j for query sl
    f32x4 s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int t = 0; t < KSTEPS; ++t) {
      s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, ka[t]), qhi[t], s, 0, 0, 0);
      s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, ka[t]), qlo[t], s, 0, 0, 0);
    }
    float sc[4] = {s.x, s.y, s.z, s.w};
    float mx = -INFINITY;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int key = base + 4 * kq + j;
      if (key >= key_end || key > my_row_pos || sl >= QV) sc[j] = -INFINITY;
      mx = fmaxf(mx, sc[j]);
    }
    mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float m_new = fmaxf(m_run, mx);
    float p[4] = {0.f, 0.f, 0.f, 0.f};
    float resc = 1.f;
    if (m_new != -INFINITY) {
      resc = __expf(m_run - m_new);                             // exp(-inf) = 0 on the first visible key
      float psum = 0.f;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        p[j] = sc[j] == -INFINITY ? 0.f : __expf(sc[j] - m_new);
        psum += p[j];
      }
      l_run = l_run * resc + psum;
      m_run = m_new;
    }
    // rescale the output rows this lane holds (queries 4 kq + j) by their queries' factors
    float rj[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) rj[j] = __shfl(resc, 4 * kq + j, 64);
#pragma unroll
    for (int e = 0; e < DPL; ++e) { acc[e].x *= rj[0]; acc[e].y *= rj[1]; acc[e].z *= rj[2]; acc[e].w *= rj[3]; }
#pragma unroll
    for (int m = 0; m < 4; ++m)
#pragma unroll
      for (int e = 0; e < DPL; ++e) acc[e] = __builtin_amdgcn_mfma_f32_16x16x4f32(p[m], vf[m][e], acc[e], 0, 0, 0);
  }
  // per-wave totals: l summed over the 4 kq lanes of a query
  l_run += __shfl_xor(l_run, 16, 64);
  l_run += __shfl_xor(l_run, 32, 64);
  if (kq == 0 && sl < QV) { wm[wave][sl] = m_run; wl[wave][sl] = l_run; }
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int qv = 4 * kq + j;
    if (qv < QV) {
      float* dst = wacc + ((size_t)wave * QV + qv) * HD + DPL * sl;
#pragma unroll
      for (int e = 0; e < DPL; ++e) dst[e] = acc[e][j];
    }
  }
  __syncthreads();
  const size_t slot = (((size_t)b * nkv + g) * ATT_MAX_SPLITS + split) * qv_stride + (size_t)rg * rpb * GQ;
  float* my_o = part_o + slot * HD;
  float* my_ml = part_ml + slot * 2;
  // the waves' partials of a query vector, 4 consecutive d per thread
  for (int e = tid; e < QV * (HD / 4); e += NT) {
    const int qv = e / (HD / 4), d = (e % (HD / 4)) * 4;
    float mm = wm[0][qv];
#pragma unroll
    for (int w = 1; w < NW; ++w) mm = fmaxf(mm, wm[w][qv]);
    f32x4 o = {0.f, 0.f, 0.f, 0.f};
    float ll = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      const float f = (wm[w][qv] == -INFINITY) ? 0.f : __expf(wm[w][qv] - mm);
      o += f * *(const f32x4*)(wacc + ((size_t)w * QV + qv) * HD + d);
      ll += f * wl[w][qv];
    }
    if (FINAL) {
      // row and head of query vector qv; every row sees at least its own key, so ll > 0
      const size_t at = (size_t)(b * r_total + rg * rpb + qv / GQ) * ldo + (size_t)(g * GQ + qv % GQ) * HD + d;
      const float inv_l = 1.0f / ll;
      bf16_t hi[4], lo[4];
#pragma unroll
      for (int c = 0; c < 4; ++c) split_bf16(o[c] * inv_l, hi[c], lo[c]);
      *(uint2*)(out + at) = make_uint2(hi[0] | ((uint32_t)hi[1] << 16), hi[2] | ((uint32_t)hi[3] << 16));
      *(uint2*)(out_lo + at) = make_uint2(lo[0] | ((uint32_t)lo[1] << 16), lo[2] | ((uint32_t)lo[3] << 16));
    } else {
      *(f32x4*)(my_o + qv * HD + d) = o;
      if (d == 0) { my_ml[qv * 2] = mm; my_ml[qv * 2 + 1] = ll; }
    }
  }
}

}  // namespace dmtd
