// Device kernels of the DMTD decode path for gfx950 (wave64).
//
// Data in HBM: weights and KV cache in the model's storage type (bf16, or fp32 for
// the tiny parity model); the residual stream and all inter-kernel activations are
// fp32, as are norms, softmax and every accumulation.
//
// Every kernel reads the token positions it works on from a small device-resident
// state block, never from launch arguments, so a captured graph of one decode step
// can be replayed unchanged as the sequence grows.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dmtd {

typedef uint16_t bf16_t;
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// Device-resident scheduler mirror; written only by single-thread kernels.
struct DevState {
  int n_tok;         // position of the next token-emitting row
  int n_front;       // first position not yet in the front layers' caches
  int forced_until;  // positions < forced_until hold caller-forced input tokens
  int step_idx;      // step number inside the current decode call
};

// Where a launch's rows sit: row i of sequence b is at position base + offset + i, with
// base read from the device state (or 0 for POS_EXPLICIT) and offset a launch argument.
enum PosSel : int { POS_NTOK = 0, POS_NFRONT = 1, POS_EXPLICIT = 2 };

__device__ __forceinline__ int row_base(const DevState* st, int sel, int offset) {
  return (sel == POS_NTOK ? st->n_tok : (sel == POS_NFRONT ? st->n_front : 0)) + offset;
}

__device__ __forceinline__ float bf16_to_f32(bf16_t v) { return __uint_as_float(((uint32_t)v) << 16); }

__device__ __forceinline__ bf16_t f32_to_bf16(float f) {   // round to nearest even
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}

template <typename T> struct Elem;
template <> struct Elem<float> {
  static __device__ __forceinline__ float to_f32(float v) { return v; }
  static __device__ __forceinline__ float from_f32(float v) { return v; }
  // 8 consecutive elements starting at p (32-byte aligned)
  static __device__ __forceinline__ void load8(const float* p, float (&w)[8]) {
    const f32x4 a = __builtin_nontemporal_load((const f32x4*)p);
    const f32x4 b = __builtin_nontemporal_load((const f32x4*)p + 1);
    w[0] = a.x; w[1] = a.y; w[2] = a.z; w[3] = a.w; w[4] = b.x; w[5] = b.y; w[6] = b.z; w[7] = b.w;
  }
};
template <> struct Elem<bf16_t> {
  static __device__ __forceinline__ float to_f32(bf16_t v) { return bf16_to_f32(v); }
  static __device__ __forceinline__ bf16_t from_f32(float v) { return f32_to_bf16(v); }
  static __device__ __forceinline__ void load8(const bf16_t* p, float (&w)[8]) {   // 16-byte aligned
    const u32x4 v = __builtin_nontemporal_load((const u32x4*)p);
    w[0] = __uint_as_float(v.x << 16); w[1] = __uint_as_float(v.x & 0xFFFF0000u);
    w[2] = __uint_as_float(v.y << 16); w[3] = __uint_as_float(v.y & 0xFFFF0000u);
    w[4] = __uint_as_float(v.z << 16); w[5] = __uint_as_float(v.z & 0xFFFF0000u);
    w[6] = __uint_as_float(v.w << 16); w[7] = __uint_as_float(v.w & 0xFFFF0000u);
  }
};

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// ---------------------------------------------------------------- small kernels

// Start of a decode call: set the forced-input horizon and the step counter, and copy
// caller-forced input tokens into the token history at the positions they will occupy.
__global__ void begin_call_kernel(DevState* st, int* tokens, int s_max, const int* forced, int n_forced, int batch) {
  const int base = st->n_tok;
  for (int i = threadIdx.x; i < batch * n_forced; i += blockDim.x) {
    const int b = i / n_forced, j = i % n_forced;
    if (base + j < s_max) tokens[(size_t)b * s_max + base + j] = forced[i];
  }
  __syncthreads();
  if (threadIdx.x == 0) { st->forced_until = base + n_forced; st->step_idx = 0; }
}

__global__ void set_state_kernel(DevState* st, int n_tok, int n_front) {
  st->n_tok = n_tok; st->n_front = n_front; st->forced_until = 0; st->step_idx = 0;
}

// End of a step: one more token is in the late caches; a full step also closes the refill gap.
__global__ void advance_kernel(DevState* st, int full) {
  const int t = st->n_tok + 1;
  st->n_tok = t;
  if (full) st->n_front = t;
  st->step_idx += 1;
}

// h[row] = table[token at the row's position]  (Eq. 4: the raw embedding is also what the
// late layers read for in-cycle tokens).  Row b*r+i of the launch is sequence b, position base+i.
template <typename WT>
__global__ void embed_kernel(const WT* __restrict__ table, const int* __restrict__ tokens, int s_max,
                             const DevState* st, int sel, int explicit_pos, int r, int d, float* __restrict__ h) {
  const int row = blockIdx.x, b = row / r, i = row % r;
  const int pos = row_base(st, sel, explicit_pos) + i;
  const int tok = tokens[(size_t)b * s_max + pos];
  const WT* src = table + (size_t)tok * d;
  float* dst = h + (size_t)row * d;
  for (int k = threadIdx.x; k < d; k += blockDim.x) dst[k] = Elem<WT>::to_f32(src[k]);
}

// dst[b] = src[b*r + r-1] (+ table[token of that row] under the literal Eq. 4 reading):
// only each sequence's newest row continues into the late layers (Sec. 2.2).
template <typename WT>
__global__ void take_last_rows_kernel(const float* __restrict__ src, float* __restrict__ dst, int r, int d,
                                      int add_embed, const WT* __restrict__ table, const int* __restrict__ tokens,
                                      int s_max, const DevState* st, int sel, int explicit_pos) {
  const int b = blockIdx.x;
  const float* s = src + ((size_t)b * r + (r - 1)) * d;
  float* o = dst + (size_t)b * d;
  const WT* e = nullptr;
  if (add_embed) {
    const int pos = row_base(st, sel, explicit_pos) + r - 1;
    e = table + (size_t)tokens[(size_t)b * s_max + pos] * d;
  }
  for (int k = threadIdx.x; k < d; k += blockDim.x) o[k] = s[k] + (add_embed ? Elem<WT>::to_f32(e[k]) : 0.0f);
}

// rows[row] += table[token at the row's position]   (literal Eq. 4 during prefill)
template <typename WT>
__global__ void add_embed_rows_kernel(float* __restrict__ h, const WT* __restrict__ table, const int* __restrict__ tokens,
                                      int s_max, const DevState* st, int sel, int explicit_pos, int r, int d) {
  const int row = blockIdx.x, b = row / r, i = row % r;
  const int pos = row_base(st, sel, explicit_pos) + i;
  const WT* e = table + (size_t)tokens[(size_t)b * s_max + pos] * d;
  float* o = h + (size_t)row * d;
  for (int k = threadIdx.x; k < d; k += blockDim.x) o[k] += Elem<WT>::to_f32(e[k]);
}

// ------------------------------------------------- weight-streaming GEMV (rows <= 4)
//
// y[m, n] = sum_k W[n, k] * xhat[m, k] for M <= 4 activation rows, with W streamed from
// HBM exactly once in 16-byte per-lane loads.  A wave owns a group of output rows and
// its lanes stride K in 8-element vectors; the activation rows live in LDS (fp32) and
// are shared by the weight rows in flight.  Optional prologue: RMSNorm of the
// activation rows (xhat = x * rsqrt(mean x^2 + eps) * gain).  Epilogues: store, add to
// the residual stream, SwiGLU of a (gate, up) row pair, or logits with a running argmax.

enum GemvEpi : int { EPI_STORE = 0, EPI_RESID = 1, EPI_SWIGLU = 2, EPI_LOGITS = 3 };

struct ArgmaxPartial { float val; int idx; };

struct GemvArgs {
  const void* W;        // [N, K]; for SWIGLU the gate matrix
  const void* W2;       // SWIGLU: the up matrix [N, K]
  const void* gain;     // norm gain [K] (NORM only)
  const float* x;       // [M, ldx]
  float* y;             // [M, ldy]
  int ldx, ldy, N, K;
  float eps;
  // LOGITS only:
  ArgmaxPartial* partial;   // [gridDim.x, M]
  unsigned int* counter;    // zero on entry; reset by the last block
  int* tokens;              // token history [batch, s_max]
  int* emitted;             // [max_steps, batch]
  const DevState* st;
  int s_max, batch, m0;     // this launch covers sequences m0 .. m0+M-1
};

template <typename WT, int M, int EPI, bool NORM>
__global__ void __launch_bounds__(1024) gemv_kernel(GemvArgs a) {
  extern __shared__ float4 smem4[];
  float* xs = (float*)smem4;                       // [M][K]
  __shared__ float red[16][M];
  __shared__ float rs_s[M];
  const int tid = threadIdx.x, nt = blockDim.x, lane = tid & 63, wave = tid >> 6, nw = nt >> 6;
  const int K = a.K, N = a.N;
  const WT* __restrict__ W = (const WT*)a.W;

  // stage activation rows in LDS (K is a multiple of 4)
  float ss[M];
#pragma unroll
  for (int m = 0; m < M; ++m) ss[m] = 0.f;
  for (int k = tid * 4; k < K; k += nt * 4) {
#pragma unroll
    for (int m = 0; m < M; ++m) {
      const float4 v = *(const float4*)(a.x + (size_t)m * a.ldx + k);
      ss[m] += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
      *(float4*)(xs + m * K + k) = v;
    }
  }
  if (NORM) {
#pragma unroll
    for (int m = 0; m < M; ++m) {
      const float s = wave_sum(ss[m]);
      if (lane == 0) red[wave][m] = s;
    }
    __syncthreads();
    if (tid < M) {
      float s = 0.f;
      for (int w = 0; w < nw; ++w) s += red[w][tid];
      rs_s[tid] = rsqrtf(s / (float)K + a.eps);
    }
    __syncthreads();
    const WT* __restrict__ g = (const WT*)a.gain;
    for (int k = tid; k < K; k += nt) {
      const float gk = Elem<WT>::to_f32(g[k]);
#pragma unroll
      for (int m = 0; m < M; ++m) xs[m * K + k] *= rs_s[m] * gk;
    }
  }
  __syncthreads();

  constexpr int NR = 4;                               // weight rows in flight per wave
  constexpr int RPW = (EPI == EPI_SWIGLU) ? 2 : 4;    // outputs per wave task
  const int n_tasks = (N + RPW - 1) / RPW;
  float best_v[M];
  int best_i[M];
#pragma unroll
  for (int m = 0; m < M; ++m) { best_v[m] = -INFINITY; best_i[m] = 0x7FFFFFFF; }

  for (int task = blockIdx.x * nw + wave; task < n_tasks; task += gridDim.x * nw) {
    const int n0 = task * RPW;
    const WT* wp[NR];
#pragma unroll
    for (int r = 0; r < NR; ++r) {
      if (EPI == EPI_SWIGLU) {
        const int n = min(n0 + (r & 1), N - 1);
        wp[r] = ((r < 2) ? W : (const WT*)a.W2) + (size_t)n * K;
      } else {
        wp[r] = W + (size_t)min(n0 + r, N - 1) * K;
      }
    }
    float acc[NR][M];
#pragma unroll
    for (int r = 0; r < NR; ++r)
#pragma unroll
      for (int m = 0; m < M; ++m) acc[r][m] = 0.f;

#pragma unroll 2
    for (int k0 = lane * 8; k0 < K; k0 += 512) {
      float w[NR][8];
#pragma unroll
      for (int r = 0; r < NR; ++r) Elem<WT>::load8(wp[r] + k0, w[r]);
#pragma unroll
      for (int m = 0; m < M; ++m) {
        const float4 xa = *(const float4*)(xs + m * K + k0);
        const float4 xb = *(const float4*)(xs + m * K + k0 + 4);
#pragma unroll
        for (int r = 0; r < NR; ++r) {
          acc[r][m] += w[r][0] * xa.x + w[r][1] * xa.y + w[r][2] * xa.z + w[r][3] * xa.w +
                       w[r][4] * xb.x + w[r][5] * xb.y + w[r][6] * xb.z + w[r][7] * xb.w;
        }
      }
    }
#pragma unroll
    for (int r = 0; r < NR; ++r)
#pragma unroll
      for (int m = 0; m < M; ++m) acc[r][m] = wave_sum(acc[r][m]);

    if (EPI == EPI_SWIGLU) {
      // rows 0,1 = gate of outputs n0, n0+1; rows 2,3 = up of the same outputs
#pragma unroll
      for (int p = 0; p < 2; ++p)
#pragma unroll
        for (int m = 0; m < M; ++m)
          if (lane == p * M + m && n0 + p < N) {
            const float gt = acc[p][m], up = acc[2 + p][m];
            a.y[(size_t)m * a.ldy + n0 + p] = gt / (1.0f + __expf(-gt)) * up;
          }
    } else {
#pragma unroll
      for (int r = 0; r < NR; ++r)
#pragma unroll
        for (int m = 0; m < M; ++m) {
          if (lane == r * M + m && n0 + r < N) {
            float* dst = a.y + (size_t)m * a.ldy + n0 + r;
            if (EPI == EPI_RESID) *dst += acc[r][m]; else *dst = acc[r][m];
          }
          if (EPI == EPI_LOGITS && n0 + r < N) {
            // strict '>' keeps the lowest index among equal maxima inside a wave (indices ascend)
            if (acc[r][m] > best_v[m]) { best_v[m] = acc[r][m]; best_i[m] = n0 + r; }
          }
        }
    }
  }

  if (EPI == EPI_LOGITS) {
    __shared__ float bv[16][M];
    __shared__ int bi[16][M];
    __shared__ bool is_last;
    if (lane == 0)
#pragma unroll
      for (int m = 0; m < M; ++m) { bv[wave][m] = best_v[m]; bi[wave][m] = best_i[m]; }
    __syncthreads();
    if (tid < M) {
      float v = bv[0][tid]; int i = bi[0][tid];
      for (int w = 1; w < nw; ++w)
        if (bv[w][tid] > v || (bv[w][tid] == v && bi[w][tid] < i)) { v = bv[w][tid]; i = bi[w][tid]; }
      a.partial[blockIdx.x * M + tid].val = v;
      a.partial[blockIdx.x * M + tid].idx = i;
    }
    __threadfence();
    __syncthreads();
    if (tid == 0) is_last = (atomicAdd(a.counter, 1u) == gridDim.x - 1);
    __syncthreads();
    if (is_last) {
      __threadfence();
      if (wave == 0) {
        const int pos = a.st->n_tok, step = a.st->step_idx, forced_until = a.st->forced_until;
        for (int m = 0; m < M; ++m) {
          float v = -INFINITY; int i = 0x7FFFFFFF;
          for (int blk = lane; blk < (int)gridDim.x; blk += 64) {
            const ArgmaxPartial p = a.partial[blk * M + m];
            if (p.val > v || (p.val == v && p.idx < i)) { v = p.val; i = p.idx; }
          }
#pragma unroll
          for (int o = 32; o > 0; o >>= 1) {
            const float ov = __shfl_xor(v, o, 64);
            const int oi = __shfl_xor(i, o, 64);
            if (ov > v || (ov == v && oi < i)) { v = ov; i = oi; }
          }
          if (lane == 0 && a.tokens) {      // a null history = measurement launch: no token side effects
            const int b = a.m0 + m;
            a.emitted[step * a.batch + b] = i;
            if (pos + 1 < a.s_max && pos + 1 >= forced_until) a.tokens[(size_t)b * a.s_max + pos + 1] = i;
          }
        }
        if (lane == 0) *a.counter = 0u;
      }
    }
  }
}

// ------------------------------------------- QK-RMSNorm + RoPE + KV-cache append
//
// One wave per (row, head).  Query heads: per-head RMSNorm (gain [hd]), rotary embedding
// with half-split pairing (i, i+hd/2) at the row's absolute position, written back in
// place.  Key heads: the same, written to the cache slot of that position.  Value
// heads: copied to the cache.  Angles are formed in double from a host-computed
// double table of theta^(-2i/hd), so long contexts lose no accuracy.
template <typename CT>
__global__ void __launch_bounds__(64) qk_norm_rope_append_kernel(
    float* __restrict__ qkv, int ldq, const void* __restrict__ q_gain, const void* __restrict__ k_gain,
    const double* __restrict__ inv_freq, CT* __restrict__ kc, CT* __restrict__ vc, int nh, int nkv, int hd,
    int s_max, float eps, const DevState* st, int sel, int explicit_pos, int r) {
  const int head = blockIdx.x, row = blockIdx.y, b = row / r, i = row % r;
  const int pos = row_base(st, sel, explicit_pos) + i;
  const int lane = threadIdx.x, half = hd >> 1;
  float* src = qkv + (size_t)row * ldq + (size_t)head * hd;
  if (head >= nh + nkv) {   // value head: plain copy into the cache
    const int g = head - nh - nkv;
    CT* dst = vc + (((size_t)b * nkv + g) * s_max + pos) * hd;
    for (int k = lane; k < hd; k += 64) dst[k] = Elem<CT>::from_f32(src[k]);
    return;
  }
  const bool act = lane < half;
  float x0 = act ? src[lane] : 0.f, x1 = act ? src[lane + half] : 0.f;
  const float rs = rsqrtf(wave_sum(x0 * x0 + x1 * x1) / (float)hd + eps);
  if (!act) return;
  const CT* g = (const CT*)(head < nh ? q_gain : k_gain);
  x0 *= rs * Elem<CT>::to_f32(g[lane]);
  x1 *= rs * Elem<CT>::to_f32(g[lane + half]);
  double sn, cs;
  sincos((double)pos * inv_freq[lane], &sn, &cs);
  const float c = (float)cs, s = (float)sn;
  const float y0 = x0 * c - x1 * s, y1 = x1 * c + x0 * s;
  if (head < nh) {
    src[lane] = y0; src[lane + half] = y1;
  } else {
    const int gk = head - nh;
    CT* dst = kc + (((size_t)b * nkv + gk) * s_max + pos) * hd;
    dst[lane] = Elem<CT>::from_f32(y0); dst[lane + half] = Elem<CT>::from_f32(y1);
  }
}

// --------------------------------------------- GQA decode attention, split over keys
//
// Block (split s, kv head g, sequence b) handles keys [s*256, s*256+256) of one KV head
// for all query vectors that share it: r rows x GQ query heads (QV = r*GQ <= QV_MAX).
// Phase 1: thread t scores key s*256+t against every query vector (q staged in LDS).
// Phase 2: softmax statistics of the split (max and sum by wavefront shuffles, then
// across the 4 waves through LDS).  Phase 3: threads own output dims and accumulate
// p * V with coalesced V reads.  The split's (max, sum, unnormalised output) go to a
// partials buffer; the last block to finish for a (b, g) merges the splits in split
// order (deterministic) and writes the attention output.
constexpr int ATT_KEYS = 256;
constexpr int QV_MAX = 16;

template <typename CT, int HD>
__global__ void __launch_bounds__(256) attn_split_kernel(
    const float* __restrict__ qkv, int ldq, const CT* __restrict__ kc, const CT* __restrict__ vc,
    float* __restrict__ part_o, float* __restrict__ part_ml, unsigned int* __restrict__ counters,
    float* __restrict__ out, int ldo, int nh, int nkv, int s_max, int n_splits_cap,
    const DevState* st, int sel, int explicit_pos, int r) {
  const int split = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int GQ = nh / nkv, QV = r * GQ;
  const int pos0 = row_base(st, sel, explicit_pos);
  const int pos_last = pos0 + r - 1;
  const int key0 = split * ATT_KEYS;
  const float scale = rsqrtf((float)HD);

  __shared__ float q_s[QV_MAX][HD];
  __shared__ float p_s[QV_MAX][ATT_KEYS];
  __shared__ float wred[4][QV_MAX];
  __shared__ float m_s[QV_MAX], l_s[QV_MAX];
  __shared__ float o_s[(256 / HD) > 1 ? (256 / HD) : 1][QV_MAX][HD];
  __shared__ bool is_last;

  float* my_o = part_o + ((((size_t)b * nkv + g) * n_splits_cap + split) * QV_MAX) * HD;
  float* my_ml = part_ml + ((((size_t)b * nkv + g) * n_splits_cap + split) * QV_MAX) * 2;

  if (key0 <= pos_last) {
    for (int e = tid; e < QV * HD; e += 256) {
      const int qv = e / HD, d = e % HD, i = qv / GQ, j = qv % GQ;
      q_s[qv][d] = qkv[(size_t)(b * r + i) * ldq + (size_t)(g * GQ + j) * HD + d] * scale;
    }
    __syncthreads();
    // phase 1: scores
    const int key = key0 + tid;
    float sc[QV_MAX];
#pragma unroll
    for (int qv = 0; qv < QV_MAX; ++qv) sc[qv] = 0.f;
    if (key <= pos_last) {
      const CT* kp = kc + (((size_t)b * nkv + g) * s_max + key) * HD;
      for (int d0 = 0; d0 < HD; d0 += 8) {
        float kv[8];
        Elem<CT>::load8(kp + d0, kv);
#pragma unroll
        for (int qv = 0; qv < QV_MAX; ++qv)
          if (qv < QV) {
#pragma unroll
            for (int e = 0; e < 8; ++e) sc[qv] += kv[e] * q_s[qv][d0 + e];
          }
      }
    }
#pragma unroll
    for (int qv = 0; qv < QV_MAX; ++qv)
      if (qv < QV && !(key <= pos0 + qv / GQ)) sc[qv] = -INFINITY;   // causal: row i sees keys <= pos0 + i
    // phase 2: split-local softmax statistics
#pragma unroll
    for (int qv = 0; qv < QV_MAX; ++qv)
      if (qv < QV) {
        const float m = wave_max(sc[qv]);
        if (lane == 0) wred[wave][qv] = m;
      }
    __syncthreads();
    if (tid < QV) m_s[tid] = fmaxf(fmaxf(wred[0][tid], wred[1][tid]), fmaxf(wred[2][tid], wred[3][tid]));
    __syncthreads();
#pragma unroll
    for (int qv = 0; qv < QV_MAX; ++qv)
      if (qv < QV) {
        const float m = m_s[qv];
        const float p = (sc[qv] == -INFINITY) ? 0.f : __expf(sc[qv] - m);
        p_s[qv][tid] = p;
        const float s = wave_sum(p);
        if (lane == 0) wred[wave][qv] = s;
      }
    __syncthreads();
    if (tid < QV) l_s[tid] = wred[0][tid] + wred[1][tid] + wred[2][tid] + wred[3][tid];
    // phase 3: p * V; thread owns dim d for key slice ks
    constexpr int SL = 256 / HD;            // key slices (2 for hd 128, 4 for hd 64)
    const int d = tid % HD, ks = tid / HD;
    float acc[QV_MAX];
#pragma unroll
    for (int qv = 0; qv < QV_MAX; ++qv) acc[qv] = 0.f;
    const int nkeys = min(ATT_KEYS, pos_last + 1 - key0);
    const CT* vp = vc + (((size_t)b * nkv + g) * s_max + key0) * HD + d;
    for (int t = ks; t < nkeys; t += SL) {
      const float v = Elem<CT>::to_f32(vp[(size_t)t * HD]);
#pragma unroll
      for (int qv = 0; qv < QV_MAX; ++qv)
        if (qv < QV) acc[qv] += p_s[qv][t] * v;
    }
#pragma unroll
    for (int qv = 0; qv < QV_MAX; ++qv)
      if (qv < QV) o_s[ks][qv][d] = acc[qv];
    __syncthreads();
    for (int e = tid; e < QV * HD; e += 256) {
      const int qv = e / HD, dd = e % HD;
      float s = 0.f;
      for (int k2 = 0; k2 < SL; ++k2) s += o_s[k2][qv][dd];
      my_o[qv * HD + dd] = s;
    }
    if (tid < QV) { my_ml[tid * 2] = m_s[tid]; my_ml[tid * 2 + 1] = l_s[tid]; }
  }

  // last block of this (b, g) merges the splits
  __threadfence();
  __syncthreads();
  unsigned int* ctr = counters + (size_t)b * nkv + g;
  if (tid == 0) is_last = (atomicAdd(ctr, 1u) == gridDim.x - 1);
  __syncthreads();
  if (!is_last) return;
  __threadfence();
  const int n_act = pos_last / ATT_KEYS + 1;
  const float* po = part_o + (((size_t)b * nkv + g) * n_splits_cap) * QV_MAX * HD;
  const float* pml = part_ml + (((size_t)b * nkv + g) * n_splits_cap) * QV_MAX * 2;
  for (int e = tid; e < QV * HD; e += 256) {
    const int qv = e / HD, dd = e % HD, i = qv / GQ, j = qv % GQ;
    float m = -INFINITY;
    for (int s2 = 0; s2 < n_act; ++s2) m = fmaxf(m, pml[((size_t)s2 * QV_MAX + qv) * 2]);
    float l = 0.f, o = 0.f;
    for (int s2 = 0; s2 < n_act; ++s2) {
      const float ms = pml[((size_t)s2 * QV_MAX + qv) * 2];
      if (ms == -INFINITY) continue;
      const float w = __expf(ms - m);
      l += w * pml[((size_t)s2 * QV_MAX + qv) * 2 + 1];
      o += w * po[((size_t)s2 * QV_MAX + qv) * HD + dd];
    }
    out[(size_t)(b * r + i) * ldo + (size_t)(g * GQ + j) * HD + dd] = o / l;
  }
  if (tid == 0) *ctr = 0u;
}

}  // namespace dmtd
