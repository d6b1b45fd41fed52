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

// Device-resident scheduler mirror; written only by single-thread kernels.  The counters are those of
// the longest sequence of the batch; sequence b, whose prompt was shorter by -delta[b] tokens, sits at
// the same counters plus delta[b] (all zero for prompts of one length).  The block is followed in
// memory by the sampling parameters (byte 64), delta[max_batch] (byte 128) and last_prompt_pos[max_batch].
struct DevState {
  int n_tok;         // position of the next token-emitting row
  int n_front;       // first position not yet in the front layers' caches
  int forced_until;  // positions < forced_until hold caller-forced input tokens
  int step_idx;      // step number inside the current decode call
};
constexpr int kStateSampleOff = 64, kStateDeltaOff = 128;
// Per sequence, from byte 128 on: its position offset against the counters, and the first of its positions that is not yet in
// the front layers' caches (its own coordinates: n_front + delta while the sequences share one phase; its own value once their
// cycle boundaries differ).  One 8-byte load gives both.  last_prompt_pos[max_batch] follows the max_batch pairs.
struct SeqInfo { int delta; int front; };
__device__ __forceinline__ SeqInfo* seq_info(DevState* st) { return (SeqInfo*)((char*)st + kStateDeltaOff); }
__device__ __forceinline__ const SeqInfo* seq_info(const DevState* st) { return (const SeqInfo*)((const char*)st + kStateDeltaOff); }

// Where a launch's rows sit: row i of sequence b is at position base + offset + i, with
// base read from the device state plus the sequence's delta (or 0 for POS_EXPLICIT: explicit
// positions are the same for every sequence) and offset a launch argument.
enum PosSel : int { POS_NTOK = 0, POS_NFRONT = 1, POS_EXPLICIT = 2 };

__device__ __forceinline__ int row_base(const DevState* st, int sel, int offset, int b) {
  if (sel == POS_EXPLICIT) return offset;
  const SeqInfo si = seq_info(st)[b];
  return (sel == POS_NTOK ? st->n_tok + si.delta : si.front) + offset;
}

__device__ __forceinline__ float bf16_to_f32(bf16_t v) { return __uint_as_float(((uint32_t)v) << 16); }

__device__ __forceinline__ bf16_t f32_to_bf16(float f) {   // round to nearest even
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}

struct RawF32x8 { f32x4 a, b; };

template <typename T> struct Elem;
template <> struct Elem<float> {
  typedef RawF32x8 Raw;   // register image of 8 consecutive elements
  static __device__ __forceinline__ Raw load_raw(const float* p) {
    Raw r; r.a = __builtin_nontemporal_load((const f32x4*)p); r.b = __builtin_nontemporal_load((const f32x4*)p + 1); return r;
  }
  static __device__ __forceinline__ Raw zero_raw() { Raw r; r.a = f32x4{0, 0, 0, 0}; r.b = r.a; return r; }
  static __device__ __forceinline__ void unpack(const Raw& r, float (&w)[8]) {
    w[0] = r.a.x; w[1] = r.a.y; w[2] = r.a.z; w[3] = r.a.w; w[4] = r.b.x; w[5] = r.b.y; w[6] = r.b.z; w[7] = r.b.w;
  }
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
  typedef u32x4 Raw;
  static __device__ __forceinline__ Raw load_raw(const bf16_t* p) { return __builtin_nontemporal_load((const u32x4*)p); }
  static __device__ __forceinline__ Raw zero_raw() { return u32x4{0, 0, 0, 0}; }
  static __device__ __forceinline__ void unpack(const Raw& v, float (&w)[8]) {
    w[0] = __uint_as_float(v.x << 16); w[1] = __uint_as_float(v.x & 0xFFFF0000u);
    w[2] = __uint_as_float(v.y << 16); w[3] = __uint_as_float(v.y & 0xFFFF0000u);
    w[4] = __uint_as_float(v.z << 16); w[5] = __uint_as_float(v.z & 0xFFFF0000u);
    w[6] = __uint_as_float(v.w << 16); w[7] = __uint_as_float(v.w & 0xFFFF0000u);
  }
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
// forced: [batch, f_stride], the first n_forced entries of a row are used; ids are clamped into the vocabulary (the host
// has checked them where it can see them; a caller's DEVICE buffer it cannot).
__global__ void begin_call_kernel(DevState* st, int* tokens, int s_max, const int* forced, int n_forced, int f_stride, int vocab, int batch) {
  const int base = st->n_tok;
  for (int i = threadIdx.x; i < batch * n_forced; i += blockDim.x) {
    const int b = i / n_forced, j = i % n_forced;
    const int pos = base + seq_info(st)[b].delta + j;
    const int t = forced[(size_t)b * f_stride + j];
    if (pos < s_max) tokens[(size_t)b * s_max + pos] = t < 0 ? 0 : (t >= vocab ? vocab - 1 : t);
  }
  __syncthreads();
  if (threadIdx.x == 0) { st->forced_until = base + n_forced; st->step_idx = 0; }
}

// out[b * out_stride + i] = emitted[i * batch + b]: the steps' tokens of a call, per sequence (DEVICE to DEVICE)
__global__ void emitted_to_rows_kernel(const int* __restrict__ emitted, int* __restrict__ out, int n_steps, int batch, int out_stride) {
  for (int i = threadIdx.x; i < n_steps * batch; i += blockDim.x) out[(size_t)(i % batch) * out_stride + i / batch] = emitted[i];
}

// Reads two byte ranges (16-byte units) and does nothing else: what a launch that only streams the same bytes costs
// on this chip, to set beside the projection kernels.  Grid-stride, four independent 16-byte loads per thread in flight,
// streaming (non-temporal) loads.  The store never happens for data that is not all one magic pattern; it only keeps the loads alive.
__global__ void __launch_bounds__(256) read_only_kernel(const u32x4* __restrict__ p0, size_t n0, const u32x4* __restrict__ p1, size_t n1,
                                                        u32x4* sink) {
  const size_t stride = (size_t)gridDim.x * 256;
  u32x4 acc = {0u, 0u, 0u, 0u};
  for (int range = 0; range < 2; ++range) {
    const u32x4* __restrict__ p = range ? p1 : p0;
    const size_t n = range ? n1 : n0;
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    for (; i + 3 * stride < n; i += 4 * stride) {
      const u32x4 a = __builtin_nontemporal_load(p + i), b = __builtin_nontemporal_load(p + i + stride);
      const u32x4 c = __builtin_nontemporal_load(p + i + 2 * stride), d = __builtin_nontemporal_load(p + i + 3 * stride);
      acc ^= a ^ b ^ c ^ d;
    }
    for (; i < n; i += stride) acc ^= __builtin_nontemporal_load(p + i);
  }
  if (acc.x == 0x9e3779b9u && acc.y == 0x7f4a7c15u && acc.z == 0xf39cc060u && acc.w == 0x5cedc834u) sink[0] = acc;
}

__global__ void zero_u64_kernel(unsigned long long* p, int n) {
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) p[i] = 0ull;
}

// Counters to (n_tok, n_front), every sequence's own front position to n_front + its delta (one phase for all).
__global__ void set_state_kernel(DevState* st, int n_tok, int n_front, int max_batch) {
  for (int b = threadIdx.x; b < max_batch; b += blockDim.x) seq_info(st)[b].front = n_front + seq_info(st)[b].delta;
  if (threadIdx.x == 0) { st->n_tok = n_tok; st->n_front = n_front; st->forced_until = 0; st->step_idx = 0; }
}
// Every sequence's own front position from a list in the counters' coordinates (sequences at different points of their cycles).
__global__ void set_fronts_kernel(DevState* st, const int* __restrict__ fronts, int batch) {
  for (int b = threadIdx.x; b < batch; b += blockDim.x) seq_info(st)[b].front = fronts[b] + seq_info(st)[b].delta;
}

// Greedy selection keys: a logit and its vocabulary index packed into one 64-bit integer whose
// unsigned order is (larger logit first, then lower index), so an integer max over any
// partition of the vocabulary, in any order, gives the argmax with ties to the lowest index.
__device__ __forceinline__ unsigned long long argmax_key(float v, int idx) {
  const uint32_t u = __float_as_uint(v);
  const uint32_t ordered = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
  return ((unsigned long long)ordered << 32) | (uint32_t)(0x7FFFFFFF - idx);
}
__device__ __forceinline__ int argmax_key_index(unsigned long long key) { return 0x7FFFFFFF - (int)(uint32_t)(key & 0xFFFFFFFFu); }

// End of a step: turn each sequence's selection keys into its token (written to the step's
// output slot and, unless the caller forces the next input, to the token history), clear the
// keys, and advance the state: one more token is in the late caches; a full step also closes
// the refill gap.  With write_tokens == 0 only the keys are cleared (measurement launches).
__global__ void __launch_bounds__(1024) finish_step_kernel(DevState* st, unsigned long long* amax, int n_cells /* <= 64 */, int amax_ld,
                                                           int* tokens, int* emitted, int s_max, int batch, int full, int write_tokens,
                                                           const unsigned char* __restrict__ full_mask /* nullable: the sequences for which this was a full step */) {
  const int pos = st->n_tok, step = st->step_idx, forced_until = st->forced_until;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, n_waves = blockDim.x >> 6;
  for (int b = wave; b < batch; b += n_waves) {      // one wave per sequence; lane = cell (keys are spread over n_cells cells)
    unsigned long long best = 0ull;
    if (lane < n_cells) {
      best = amax[(size_t)lane * amax_ld + b];
      amax[(size_t)lane * amax_ld + b] = 0ull;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      const unsigned long long other = __shfl_xor(best, o, 64);
      if (other > best) best = other;
    }
    if (lane == 0 && write_tokens) {
      const int tok = argmax_key_index(best);
      emitted[step * batch + b] = tok;
      const int mine = pos + seq_info(st)[b].delta;  // this sequence's own position
      if (mine + 1 < s_max && pos + 1 >= forced_until) tokens[(size_t)b * s_max + mine + 1] = tok;
      if (full || (full_mask && full_mask[b])) seq_info(st)[b].front = mine + 1;     // its refill gap is closed
    }
  }
  __syncthreads();
  if (threadIdx.x == 0 && write_tokens) {
    st->n_tok = pos + 1;
    if (full || (full_mask && full_mask[0])) st->n_front = pos + 1;     // the shared counter follows sequence 0
    st->step_idx = step + 1;
  }
}

// h[row] = table[token at the row's position]  (Eq. 4: the raw embedding is also what the
// late layers read for in-cycle tokens).  Row b*r+i of the launch is sequence b, position base+i.
template <typename WT>
__global__ void embed_kernel(const WT* __restrict__ table, const int* __restrict__ tokens, int s_max,
                             const DevState* st, int sel, int explicit_pos, int r, int d, float* __restrict__ h,
                             const int* __restrict__ fmap /* nullable: launch sequence -> sequence slot */) {
  const int row = blockIdx.x, i = row % r;
  const int b = fmap ? fmap[row / r] : row / r;
  const int pos = row_base(st, sel, explicit_pos, b) + i;
  const int tok = tokens[(size_t)b * s_max + pos];
  const WT* src = table + (size_t)tok * d;
  float* dst = h + (size_t)row * d;
  for (int k = threadIdx.x; k < d; k += blockDim.x) dst[k] = Elem<WT>::to_f32(src[k]);
}

// dst[b] = src[b*r + r-1] (+ table[token of that row] under the literal Eq. 4 reading; ExDy variant of that
// reading: + add_rows[b], the row's encoding output, which may be dst itself): only each sequence's newest
// row continues into the late layers (Sec. 2.2).
// With last_pos (prompts of different lengths, explicit positions): sequence b's row is the one at position
// last_pos[b]; a sequence whose row is not among this launch's r positions is left alone.
template <typename WT>
__global__ void take_last_rows_kernel(const float* __restrict__ src, float* dst, int r, int d,
                                      int add_embed, const WT* __restrict__ table, const int* __restrict__ tokens,
                                      int s_max, const DevState* st, int sel, int explicit_pos, const float* add_rows,
                                      const int* __restrict__ last_pos, const int* __restrict__ fmap /* nullable: launch sequence -> sequence slot */) {
  const int bl = blockIdx.x, b = fmap ? fmap[bl] : bl;         // source rows by launch sequence, everything else by slot
  const int i = last_pos ? last_pos[b] - explicit_pos : r - 1;
  if (i < 0 || i >= r) return;
  const float* s = src + ((size_t)bl * r + i) * d;
  float* o = dst + (size_t)b * d;
  const WT* e = nullptr;
  if (add_embed) {
    const int pos = row_base(st, sel, explicit_pos, b) + i;
    e = table + (size_t)tokens[(size_t)b * s_max + pos] * d;
  }
  const float* ar = add_rows ? add_rows + (size_t)b * d : nullptr;
  for (int k = threadIdx.x; k < d; k += blockDim.x) o[k] = s[k] + (add_embed ? Elem<WT>::to_f32(e[k]) : 0.0f) + (ar ? ar[k] : 0.0f);
}

// rows[row] += table[token at the row's position]   (literal Eq. 4 during prefill)
template <typename WT>
__global__ void add_embed_rows_kernel(float* __restrict__ h, const WT* __restrict__ table, const int* __restrict__ tokens,
                                      int s_max, const DevState* st, int sel, int explicit_pos, int r, int d) {
  const int row = blockIdx.x, b = row / r, i = row % r;
  const int pos = row_base(st, sel, explicit_pos, b) + i;
  const WT* e = table + (size_t)tokens[(size_t)b * s_max + pos] * d;
  float* o = h + (size_t)row * d;
  for (int k = threadIdx.x; k < d; k += blockDim.x) o[k] += Elem<WT>::to_f32(e[k]);
}

// ---- token selection by sampling: temperature and top-k through the Gumbel-max identity.  The uniforms come
// ---- from a counter-based SplitMix64 generator keyed by (seed, sequence, position, vocabulary entry), so a draw
// ---- depends on nothing but those four numbers (graph replays and batch order do not matter).

struct SampleCfg {        // device-resident, written by the host when the setting changes
  float inv_temp;         // 1 / temperature
  int top_k;              // <= 0: no restriction
  unsigned int seed_lo, seed_hi;
};

__device__ __forceinline__ unsigned long long splitmix_mix(unsigned long long z) {
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

// floats in an unsigned order (larger float, larger integer); -0 counts as +0
__device__ __forceinline__ uint32_t ordered_u32(float v) {
  const uint32_t u = __float_as_uint(v + 0.0f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// One block of 1024 threads per sequence, after the LM head: the row at position st->n_tok draws its token from
// softmax(z / temperature) over the top_k largest logits (logits equal to the k-th largest all stay in).  The
// k-th largest logit comes from a 4-pass radix select over the ordered bit patterns (integer counts: exact and
// order independent); the draw is the argmax of z_v / temperature - log(-log(u_v)), u_v the midpoint of one of
// 2^23 cells of (0, 1) picked by the generator's top 23 bits.  The result replaces the greedy selection keys.
__global__ void __launch_bounds__(1024) sample_kernel(const float* __restrict__ logits, int V, const SampleCfg* __restrict__ cfg,
                                                      const DevState* st, unsigned long long* amax, int n_cells, int amax_ld) {
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const float* z = logits + (size_t)b * V;
  __shared__ unsigned int hist[256];
  __shared__ unsigned int sel_prefix, sel_remaining;
  __shared__ unsigned long long key_w[16];
  const int top_k = cfg->top_k;
  const float inv_temp = cfg->inv_temp;
  uint32_t thr = 0u;                    // entries whose ordered pattern is >= thr stay in
  if (top_k > 0 && top_k < V) {
    uint32_t prefix = 0u;
    unsigned int remaining = (unsigned int)top_k;
    for (int pass = 0; pass < 4; ++pass) {
      const int shift = 24 - 8 * pass;
      const uint32_t himask = pass == 0 ? 0u : (0xFFFFFFFFu << (shift + 8));
      if (tid < 256) hist[tid] = 0u;
      __syncthreads();
      for (int v = tid; v < V; v += 1024) {
        const uint32_t o = ordered_u32(z[v]);
        if ((o & himask) == prefix) atomicAdd(&hist[(o >> shift) & 255u], 1u);
      }
      __syncthreads();
      if (tid == 0) {
        unsigned int above = 0u;
        int bin = 255;
        for (; bin > 0; --bin) {
          if (above + hist[bin] >= remaining) break;
          above += hist[bin];
        }
        sel_prefix = prefix | ((uint32_t)bin << shift);
        sel_remaining = remaining - above;
      }
      __syncthreads();
      prefix = sel_prefix;
      remaining = sel_remaining;
    }
    thr = prefix;
  }
  const unsigned long long seed = ((unsigned long long)cfg->seed_hi << 32) | cfg->seed_lo;
  const unsigned long long stream = ((unsigned long long)(unsigned int)b << 32) | (unsigned int)(st->n_tok + seq_info(st)[b].delta);
  const unsigned long long base = splitmix_mix(splitmix_mix(seed + 0x9E3779B97F4A7C15ull) ^ (stream * 0xD6E8FEB86659FD93ull));
  unsigned long long key = 0ull;
  for (int v = tid; v < V; v += 1024) {
    const float zv = z[v];
    if (ordered_u32(zv) >= thr) {
      const unsigned long long r = splitmix_mix(base + (unsigned long long)(v + 1) * 0x9E3779B97F4A7C15ull);
      const float u = ((float)(r >> 41) + 0.5f) * (1.0f / 8388608.0f);
      const unsigned long long k = argmax_key(zv * inv_temp - logf(-logf(u)), v);
      if (k > key) key = k;
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const unsigned long long other = __shfl_xor(key, o, 64);
    if (other > key) key = other;
  }
  if (lane == 0) key_w[wave] = key;
  __syncthreads();
  if (tid < n_cells) {
    unsigned long long k = 0ull;
    if (tid == 0) {
      k = key_w[0];
      for (int w = 1; w < 16; ++w) if (key_w[w] > k) k = key_w[w];
    }
    amax[(size_t)tid * amax_ld + b] = k;     // cell 0: the draw; the other cells (greedy partial keys): cleared
  }
}

// Summands of the next-token loss (Eq. 6) and the greedy choice for the rows of one chunk of a whole-sequence
// forward: row b*r+i of the launch is position p0+i of sequence b; its target is the sequence's next token
// (none for the last position n-1: the summand is stored as 0).  nll = log(sum_v exp(z_v - max)) + max - z_target,
// sums taken per thread, per wave and over the waves in a fixed order.  One block of 1024 threads per row.
__global__ void __launch_bounds__(1024) nll_rows_kernel(const float* __restrict__ logits, int V, const int* __restrict__ tokens, int s_max,
                                                        int p0, int r, int n, float* __restrict__ nll, int* __restrict__ best) {
  const int row = blockIdx.x, b = row / r, pos = p0 + row % r;
  const float* z = logits + (size_t)row * V;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  __shared__ unsigned long long key_w[16];
  __shared__ float sum_w[16];
  __shared__ float top_s;
  unsigned long long key = 0ull;
  for (int v = tid; v < V; v += 1024) {
    const unsigned long long k = argmax_key(z[v], v);
    if (k > key) key = k;
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const unsigned long long other = __shfl_xor(key, o, 64);
    if (other > key) key = other;
  }
  if (lane == 0) key_w[wave] = key;
  __syncthreads();
  if (tid == 0) {
    unsigned long long k = key_w[0];
    for (int w = 1; w < 16; ++w) if (key_w[w] > k) k = key_w[w];
    const int idx = argmax_key_index(k);
    best[(size_t)b * s_max + pos] = idx;
    top_s = z[idx];
  }
  __syncthreads();
  const float top = top_s;
  float s = 0.f;
  for (int v = tid; v < V; v += 1024) s += __expf(z[v] - top);
  s = wave_sum(s);
  if (lane == 0) sum_w[wave] = s;
  __syncthreads();
  if (tid == 0) {
    float tot = 0.f;
    for (int w = 0; w < 16; ++w) tot += sum_w[w];
    float out = 0.f;
    if (pos + 1 < n) out = __logf(tot) + top - z[tokens[(size_t)b * s_max + pos + 1]];
    nll[(size_t)b * s_max + pos] = out;
  }
}

// Eq. 6 per sequence: the mean of the summands of the n-1 positions that have a successor (fixed summation order).
__global__ void __launch_bounds__(256) mean_nll_kernel(const float* __restrict__ nll, int s_max, int n, float* __restrict__ loss) {
  const int b = blockIdx.x, tid = threadIdx.x;
  __shared__ float part[256];
  float s = 0.f;
  for (int i = tid; i + 1 < n; i += 256) s += nll[(size_t)b * s_max + i];
  part[tid] = s;
  __syncthreads();
  if (tid == 0) {
    float tot = 0.f;
    for (int t = 0; t < 256; ++t) tot += part[t];
    loss[b] = n > 1 ? tot / (float)(n - 1) : 0.f;
  }
}

}  // namespace dmtd

#include "gemv.hpp"
#include "gemv_mfma.hpp"
#include "gemm_mfma.hpp"
#include "attention.hpp"
#include "attention_mfma.hpp"
