// MFMA weight-streaming "skinny GEMM" for 1..16 activation rows of a bf16 model on gfx950.
//
// y[m, n] = sum_k W[n, k] * xhat[m, k].  The weights are the A operand of
// v_mfma_f32_16x16x32_bf16.  They are stored in HBM in operand order ("swizzled", done once
// at context creation): for each tile of 16 output rows and each k-step of 64 elements,
// two 1 KiB pieces, piece h holding for lane l = (kg = l / 16, r = l % 16) the 8 elements
// W[16 t + r][64 s + 32 h + 8 kg + 0..7].  One load instruction of a wave therefore reads
// 1 KiB of contiguous memory straight into the operand registers, every weight byte is
// read exactly once, and no data passes through LDS or is converted on the way.
//
// The activation rows are the B operand (column = lane % 16, zero beyond M); they arrive
// already packed, written by the kernel that produced them, as TWO bf16 planes: hi = bf16(x)
// and lo = bf16(x - hi).  Each k-step takes two matrix-core passes (W * hi + W * lo), which the
// weight stream hides, so the activations keep 16 mantissa bits and the only bf16 roundings left
// on the path are those of the stored model (weights, KV cache).  RMSNorm is folded in
// exactly: the producer stores bf16(x * gain) and per-tile partial sums of x^2, and the
// epilogue here multiplies column m by rsqrt(mean(x_m^2) + eps).  No cross-lane reduction
// is needed: the matrix core sums over k, and a lane ends up holding 4 rows of one column.
//
// A block owns one tile of 16 output rows (SwiGLU: the gate tile and the up tile of the
// same 16 outputs); its waves split K into runs of k-steps, a wave issues all loads of a
// run (up to PF k-steps = 2*PF KiB) at once, and the waves' partial tiles are summed
// through LDS in wave order (deterministic).  Epilogues: fp32 store (QKV), SwiGLU to packed
// bf16, residual add that also emits the next norm's packed input and partial sums of
// squares, and logits with greedy-selection keys.
#pragma once
#include "gemv.hpp"

namespace dmtd {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));

// two floats to one packed bf16 pair, round to nearest even (one v_cvt_pk_bf16_f32)
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  const f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}
__device__ __forceinline__ bf16_t to_bf16_hw(float v) { return (bf16_t)(pack_bf16x2(v, 0.f) & 0xFFFFu); }
// v as the sum of two bf16 values: hi = bf16(v), lo = bf16(v - hi)
__device__ __forceinline__ void split_bf16(float v, bf16_t& hi, bf16_t& lo) {
  hi = to_bf16_hw(v);
  lo = to_bf16_hw(v - bf16_to_f32(hi));
}

constexpr int MFMA_MAX_WAVES = 16;   // waves that split K for one tile
constexpr int AMAX_CELLS = 64;       // selection keys are spread over this many cells per sequence

// Elements of the swizzled image of an [N, K] matrix (rows padded to a multiple of 16).
__host__ __device__ inline size_t swizzled_elems(size_t N, size_t K) { return (N + 15) / 16 * 16 * K; }

// One-time repack of a row-major [N, K] bf16 matrix (K a multiple of 64) into operand order.
__global__ void swizzle_weights_kernel(const bf16_t* __restrict__ W, bf16_t* __restrict__ out, int N, int K) {
  const int KS = K >> 6;
  const size_t n_chunks = (size_t)((N + 15) / 16) * KS * 2 * 64;     // 16-byte chunks
  for (size_t ch = blockIdx.x * (size_t)blockDim.x + threadIdx.x; ch < n_chunks; ch += (size_t)gridDim.x * blockDim.x) {
    const int l = ch & 63, h = (ch >> 6) & 1;
    const size_t ts = ch >> 7;
    const int s = ts % KS;
    const size_t t = ts / KS;
    const size_t n = t * 16 + (l & 15);
    u32x4 v = {0, 0, 0, 0};
    if (n < (size_t)N) v = *(const u32x4*)(W + n * K + (size_t)s * 64 + h * 32 + (l >> 4) * 8);
    *(u32x4*)(out + ch * 8) = v;
  }
}

struct MfmaArgs {
  const bf16_t* W;       // swizzled [N, K]; SwiGLU: the gate matrix
  const bf16_t* W2;      // SwiGLU: the up matrix
  const bf16_t* xb;      // packed activations, high parts [M, ldxb] (already multiplied by the norm gain if NORM)
  const bf16_t* xb_lo;   // their low parts, same layout
  int ldxb, M, N, K;
  const float* ssp;      // NORM: partial sums of squares [n_parts, ssp_ld]
  int n_parts, ssp_ld;
  float eps;
  float* y;              // STORE / LOGITS: fp32 out [M, ldy]; RESID: the residual stream, updated in place
  int ldy;
  bf16_t* yb;            // SwiGLU: packed out [M, ldyb]; RESID: packed input of the next norm (h * g_next); high parts
  bf16_t* yb_lo;         // low parts, same layout
  int ldyb;
  const bf16_t* g_next;  // RESID: gain of the next norm [N]
  float* ssp_next;       // RESID: partial sums of squares of the updated residual rows [tiles, ssp_ld]
  unsigned long long* amax;   // LOGITS: selection keys [AMAX_CELLS, amax_ld], already offset to this launch's rows
  int amax_ld;
  float* part;           // tiled kernel with K split over blocks: partial sums [ksplit][M][ldp]
  int ksplit, ldp;
};

// The block first copies the M packed activation rows (both planes) into LDS (dynamic shared
// memory, 2 * M * K * 2 bytes, plus M * n_parts * 4 for the partial sums of squares if NORM) and the
// waves take their B operands from there; the host sends rows
// that do not fit there to the LDS-tiled kernel (gemm_mfma.hpp).
// The arguments every wave needs before it can issue its first loads are passed as scalars ahead of the struct: the
// leading scalar arguments of a kernel arrive in registers at wave launch, the struct through a load.
template <int EPI, bool NORM, int PF, int NWT, bool ROLL = false>   // NWT: waves per block (all matrices)
__global__ void __launch_bounds__(64 * NWT) gemv_mfma_kernel(const bf16_t* W_, const bf16_t* W2_,
                                                             const bf16_t* xb_, const bf16_t* xb_lo_, const float* ssp_,
                                                             int M_, int N_, int K_, int n_parts_, int ssp_ld_, MfmaArgs a) {
  extern __shared__ float4 dyn_smem[];
  bf16_t* xs = (bf16_t*)dyn_smem;                        // [2 planes][M][K], then (NORM) M * n_parts floats
  constexpr int MATS = (EPI == EPI_SWIGLU) ? 2 : 1;
  constexpr int nw = NWT / MATS;                         // waves that split K for one matrix
  static_assert(nw >= 1 && nw <= MFMA_MAX_WAVES, "waves per tile");
  __shared__ float red[MATS][nw][16][17];               // [matrix][wave][column][row], padded
  __shared__ float ss_s[16][17];
  float* ss_items = (float*)(xs + (size_t)2 * M_ * K_);   // NORM: the producer's partial sums [n_parts][M], behind the rows
  __shared__ float rs_s[16];
  __shared__ unsigned long long key_s[16];
  const int tid = threadIdx.x, lane = tid & 63;
  // the wave's index as a scalar: everything derived from it (matrix, k-range, the loads' bounds) then branches
  // uniformly; left in a vector register, every bounded load became a divergent region the compiler waits on
  const int wall = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int mat = wall / nw, w = wall % nw;
  const int r = lane & 15, kg = lane >> 4;     // B and D: column r
  const int K = K_, N = N_, M = M_;
  const int tile = blockIdx.x;
  const int KS = K >> 6;                       // k-steps of 64 elements
  const int s0 = (int)((long)w * KS / nw), s1 = (int)((long)(w + 1) * KS / nw);

  const bf16_t* __restrict__ abase = (mat == 0 ? W_ : W2_) + ((size_t)tile * KS) * 1024 + lane * 8;
  const bool colact = r < M;
  const int ldxs = K;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f}, acc2 = acc;
  constexpr bool TWO_ACC = EPI == EPI_RESID && !ROLL;      // where registers allow (one block per CU)

  // small loads first (they return first): the B rows for LDS and the partial sums of squares.  Every one of them is
  // issued unconditionally, from a clamped index: a load under a per-lane condition makes the compiler wait for it
  // right there, and each such wait is a full memory round trip in front of the weight stream.
  constexpr int NT = 64 * NWT;
  // registers for the early activation loads: residual projections run one block per CU (few, wide tiles) and can
  // afford to cover long rows; the others stay within 128 registers (two 8-wave blocks per CU)
  constexpr int NBST = EPI == EPI_RESID ? (ROLL ? 8 : 16) : 5;
  u32x4 bst[NBST];
  // the rows follow each other in memory (ldxb == K); LDS holds them the same way, the low
  // plane behind the high one, so a 16-byte chunk's source and destination are linear in its index
  const int n_chunks = M * (K >> 3);                // 16-byte chunks per plane
  auto chunk_src = [&](int c) {
    return (const u32x4*)(c >= n_chunks ? xb_lo_ + (size_t)(c - n_chunks) * 8 : xb_ + (size_t)c * 8);
  };
  auto chunk_dst = [&](int c) { return (u32x4*)(xs + (size_t)c * 8); };
#pragma unroll
  for (int j = 0; j < NBST; ++j) {
    const int c = tid + j * NT;
    bst[j] = *chunk_src(c < 2 * n_chunks ? c : 2 * n_chunks - 1);
  }
  // NORM: the producer's partial sums of squares, M * n_parts floats: thread (part p = tid / 16 + j * NT / 16, row m = tid % 16)
  constexpr int NSS = 8;
  float ssr[NSS];
  const int ss_m = tid & 15, ss_p0 = tid >> 4;
  if (NORM) {
    const float* sp = ssp_ + (ss_m < M ? ss_m : M - 1);
#pragma unroll
    for (int j = 0; j < NSS; ++j) {
      const int p = ss_p0 + j * (NT / 16);
      ssr[j] = sp[(size_t)(p < n_parts_ ? p : n_parts_ - 1) * ssp_ld_];
    }
  }
  u32x4 A[PF][2];
  auto load_a = [&](int base) {
#pragma unroll
    for (int i = 0; i < PF; ++i) {
      // a step beyond the wave's range re-reads the tile's last step (finite values; its B operands are zero below):
      // unconditional loads straight into the operand registers, nothing for the compiler to merge or wait on
      const int s = base + i < s1 ? base + i : KS - 1;
      A[i][0] = __builtin_nontemporal_load((const u32x4*)(abase + (size_t)s * 1024));
      A[i][1] = __builtin_nontemporal_load((const u32x4*)(abase + (size_t)s * 1024 + 512));
    }
  };
  __builtin_amdgcn_sched_barrier(0);                      // the small loads stay ahead of the weight stream in issue order
  load_a(s0);                                             // the weight stream starts before anything waits
  __builtin_amdgcn_sched_barrier(0);
  // residual epilogue: this thread's residual value and next-norm gain, fetched now so the epilogue does not wait
  constexpr int EPN = (256 + NT - 1) / NT;
  float hpre[EPN], gpre[EPN];
  if (EPI == EPI_RESID) {
#pragma unroll
    for (int q = 0; q < EPN; ++q) {
      const int t = tid + q * NT, c = t >> 4, n = tile * 16 + (t & 15);
      const bool ok = t < 256 && c < M && n < N;
      hpre[q] = ok ? a.y[(size_t)c * a.ldy + n] : 0.f;
      gpre[q] = ok ? bf16_to_f32(a.g_next[n]) : 0.f;
    }
  }
  if (NORM) {
    if (ss_m < M) {
#pragma unroll
      for (int j = 0; j < NSS; ++j) {
        const int p = ss_p0 + j * (NT / 16);
        if (p < n_parts_) ss_items[p * M + ss_m] = ssr[j];
      }
      for (int p = ss_p0 + NSS * (NT / 16); p < n_parts_; p += NT / 16) ss_items[p * M + ss_m] = ssp_[(size_t)p * ssp_ld_ + ss_m];
    }
  }
#pragma unroll
  for (int j = 0; j < NBST; ++j) {
    const int c = tid + j * NT;
    if (c < 2 * n_chunks) *chunk_dst(c) = bst[j];
  }
  for (int c = tid + NBST * NT; c < 2 * n_chunks; c += NT) *chunk_dst(c) = *chunk_src(c);   // beyond what the early loads covered
  __syncthreads();
  if (NORM) {
    // the rows' 1/rms while the weights are still on their way: per column, 16 threads sum interleaved parts, then
    // one thread sums the 16 (fixed order: deterministic); the epilogue's barrier makes rs_s visible
    for (int t = tid; t < 256; t += NT) {
      const int c = t >> 4, j = t & 15;
      float s = 0.f;
      if (c < M) {
        for (int p = j; p < n_parts_; p += 16) s += ss_items[p * M + c];
      }
      ss_s[c][j] = s;
    }
    __syncthreads();
    if (tid < 16) {
      float s = 0.f;
#pragma unroll
      for (int j = 0; j < 16; ++j) s += ss_s[tid][j];
      rs_s[tid] = rsqrtf(s / (float)K + a.eps);
    }
  }

  for (int base = s0; base < s1; base += PF) {           // one round unless the wave's k-range exceeds PF steps
    if (!ROLL && base != s0) load_a(base);
    if (ROLL) {
      // rolling window: a k-step's weights are used for both planes at once and its registers are refilled
      // at once with the step PF ahead, so the wave keeps PF k-steps in flight through its whole k-range
      const bf16_t* xrow = xs + (size_t)(colact ? r : 0) * ldxs + kg * 8;
      const bf16_t* xrow_lo = xrow + (size_t)M * ldxs;
#pragma unroll
      for (int i = 0; i < PF; ++i) {
        const int s = base + i;
        u32x4 b0 = {0, 0, 0, 0}, b1 = b0, c0 = b0, c1 = b0;
        if (s < s1 && colact) {
          c0 = *(const u32x4*)(xrow_lo + (size_t)s * 64);
          c1 = *(const u32x4*)(xrow_lo + (size_t)s * 64 + 32);
          b0 = *(const u32x4*)(xrow + (size_t)s * 64);
          b1 = *(const u32x4*)(xrow + (size_t)s * 64 + 32);
        }
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, A[i][0]), __builtin_bit_cast(bf16x8_t, c0), acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, A[i][1]), __builtin_bit_cast(bf16x8_t, c1), acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, A[i][0]), __builtin_bit_cast(bf16x8_t, b0), acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, A[i][1]), __builtin_bit_cast(bf16x8_t, b1), acc, 0, 0, 0);
        const int sn = s + PF;
        if (sn < s1) {      // else the slot keeps its (finite) contents: a step beyond the range meets zero B operands
          A[i][0] = __builtin_nontemporal_load((const u32x4*)(abase + (size_t)sn * 1024));
          A[i][1] = __builtin_nontemporal_load((const u32x4*)(abase + (size_t)sn * 1024 + 512));
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    } else if (TWO_ACC) {
      // registers to spare: both planes of a k-step together, each into its own accumulator, so the
      // matrix-core work keeps pace with the arriving weights
      const bf16_t* xrow = xs + (size_t)(colact ? r : 0) * ldxs + kg * 8;
      const bf16_t* xrow_lo = xrow + (size_t)M * ldxs;
#pragma unroll
      for (int i = 0; i < PF; ++i) {
        const int s = base + i;
        u32x4 b0 = {0, 0, 0, 0}, b1 = b0, c0 = b0, c1 = b0;
        if (s < s1 && colact) {
          b0 = *(const u32x4*)(xrow + (size_t)s * 64);
          b1 = *(const u32x4*)(xrow + (size_t)s * 64 + 32);
          c0 = *(const u32x4*)(xrow_lo + (size_t)s * 64);
          c1 = *(const u32x4*)(xrow_lo + (size_t)s * 64 + 32);
        }
        acc2 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, A[i][0]), __builtin_bit_cast(bf16x8_t, c0), acc2, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, A[i][0]), __builtin_bit_cast(bf16x8_t, b0), acc, 0, 0, 0);
        acc2 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, A[i][1]), __builtin_bit_cast(bf16x8_t, c1), acc2, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, A[i][1]), __builtin_bit_cast(bf16x8_t, b1), acc, 0, 0, 0);
      }
    } else {
#pragma unroll
      for (int plane = 1; plane >= 0; --plane) {          // low parts first, then the high parts, with the same weights
        const bf16_t* xrow = xs + ((size_t)plane * M + (colact ? r : 0)) * ldxs + kg * 8;
#pragma unroll
        for (int i = 0; i < PF; ++i) {
          const int s = base + i;
          u32x4 b0 = {0, 0, 0, 0}, b1 = b0;
          if (s < s1 && colact) {
            b0 = *(const u32x4*)(xrow + (size_t)s * 64);
            b1 = *(const u32x4*)(xrow + (size_t)s * 64 + 32);
          }
          acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, A[i][0]), __builtin_bit_cast(bf16x8_t, b0), acc, 0, 0, 0);
          acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, A[i][1]), __builtin_bit_cast(bf16x8_t, b1), acc, 0, 0, 0);
          if (i & 1) __builtin_amdgcn_sched_barrier(0);   // keeps the LDS reads of later steps from piling up in registers
        }
      }
    }
  }
  if (TWO_ACC) acc += acc2;
  // lane (column r, kg) holds rows kg*4 .. kg*4+3 of column r
  if (colact) {
    red[mat][w][r][kg * 4 + 0] = acc.x; red[mat][w][r][kg * 4 + 1] = acc.y;
    red[mat][w][r][kg * 4 + 2] = acc.z; red[mat][w][r][kg * 4 + 3] = acc.w;
  }
  if (EPI == EPI_LOGITS && tid < 16) key_s[tid] = 0ull;
  __syncthreads();
#pragma unroll
  for (int q = 0; q < EPN; ++q) {
    const int t = tid + q * NT;
    if (t >= 256) break;
    const int c = t >> 4, row = t & 15, n = tile * 16 + row;
    float hsq = 0.f;
    if (c < M && n < N) {
      const float rs = NORM ? rs_s[c] : 1.f;
      float v0 = 0.f;
#pragma unroll
      for (int ww = 0; ww < nw; ++ww) v0 += red[0][ww][c][row];
      v0 *= rs;
      if (EPI == EPI_SWIGLU) {
        float v1 = 0.f;
#pragma unroll
        for (int ww = 0; ww < nw; ++ww) v1 += red[MATS - 1][ww][c][row];
        v1 *= rs;
        split_bf16(v0 / (1.0f + __expf(-v0)) * v1, a.yb[(size_t)c * a.ldyb + n], a.yb_lo[(size_t)c * a.ldyb + n]);
      } else if (EPI == EPI_RESID) {
        const float hn = hpre[q] + v0;
        a.y[(size_t)c * a.ldy + n] = hn;
        hsq = hn * hn;
        split_bf16(hn * gpre[q], a.yb[(size_t)c * a.ldyb + n], a.yb_lo[(size_t)c * a.ldyb + n]);
      } else {
        a.y[(size_t)c * a.ldy + n] = v0;
        if (EPI == EPI_LOGITS) atomicMax(&key_s[c], argmax_key(v0, n));
      }
    }
    if (EPI == EPI_RESID) {
      // sum of squares of the tile's 16 outputs of column c: its 16 neighbouring lanes (inactive ones hold 0)
      hsq += __shfl_xor(hsq, 1, 64);
      hsq += __shfl_xor(hsq, 2, 64);
      hsq += __shfl_xor(hsq, 4, 64);
      hsq += __shfl_xor(hsq, 8, 64);
      if (row == 0 && c < M) a.ssp_next[(size_t)tile * a.ssp_ld + c] = hsq;
    }
  }
  if (EPI == EPI_LOGITS) {
    __syncthreads();
    if (tid < M && key_s[tid] != 0ull) atomicMax(a.amax + (size_t)(tile % AMAX_CELLS) * a.amax_ld + tid, key_s[tid]);
  }
}

// Row-wise helper for the packed path: from an fp32 row h write the packed input of a norm,
// h * gain as high and low bf16 parts, and the row's sum of squares as a single partial (n_parts = 1).
// Call with all threads of the block; contains a barrier.
__device__ __forceinline__ void pack_row_for_norm(const float* __restrict__ h, const bf16_t* __restrict__ gain, int d,
                                                  bf16_t* __restrict__ xb, bf16_t* __restrict__ xb_lo, float* __restrict__ ssp_slot) {
  __shared__ float wsum[16];
  float ss = 0.f;
  for (int k = threadIdx.x; k < d; k += blockDim.x) {
    const float v = h[k];
    ss += v * v;
    split_bf16(v * bf16_to_f32(gain[k]), xb[k], xb_lo[k]);
  }
  ss = wave_sum(ss);
  if ((threadIdx.x & 63) == 0) wsum[threadIdx.x >> 6] = ss;
  __syncthreads();
  if (threadIdx.x == 0) {
    float s = 0.f;
    for (int w = 0; w < (int)(blockDim.x >> 6); ++w) s += wsum[w];
    *ssp_slot = s;
  }
}

// ---- row kernels of the packed (bf16) path: like their fp32 counterparts, and they also
// ---- emit the packed input and the sum of squares for the norm that reads the rows next

__global__ void __launch_bounds__(256) embed_pack_kernel(
    const bf16_t* __restrict__ table, const int* __restrict__ tokens, int s_max, const DevState* st, int sel, int offset,
    int r, int d, float* __restrict__ h, const bf16_t* __restrict__ gain, bf16_t* __restrict__ xb, bf16_t* __restrict__ xb_lo,
    float* __restrict__ ssp, const int* __restrict__ fmap /* nullable: launch sequence -> sequence slot */) {
  // One pass, 8 elements (16 bytes of the table row) per thread and turn, up to NCH turns' loads in flight at once;
  // the row's values stay in registers between the fp32 store, the packed store and the sum of squares.
  constexpr int NCH = 4;
  __shared__ float wsum[4];
  const int row = blockIdx.x, i = row % r;
  const int b = fmap ? fmap[row / r] : row / r;
  const int pos = row_base(st, sel, offset, b) + i;
  const bf16_t* src = table + (size_t)tokens[(size_t)b * s_max + pos] * d;
  float* dst = h + (size_t)row * d;
  bf16_t* ob = xb + (size_t)row * d;
  bf16_t* ob_lo = xb_lo + (size_t)row * d;
  const int n_ch = d >> 3;                       // d is a multiple of 64 on this path
  float ss = 0.f;
  for (int c0 = threadIdx.x; c0 < n_ch; c0 += NCH * 256) {
    u32x4 tv[NCH], gv[NCH];
#pragma unroll
    for (int u = 0; u < NCH; ++u) {
      const int c = c0 + u * 256 < n_ch ? c0 + u * 256 : c0;     // unconditional loads from a clamped chunk
      tv[u] = *(const u32x4*)(src + (size_t)c * 8);
      gv[u] = *(const u32x4*)(gain + (size_t)c * 8);
    }
#pragma unroll
    for (int u = 0; u < NCH; ++u) {
      const int c = c0 + u * 256;
      if (c < n_ch) {
        float v[8], g[8];
        Elem<bf16_t>::unpack(tv[u], v);
        Elem<bf16_t>::unpack(gv[u], g);
        uint32_t hi[4], lo[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          bf16_t h0, l0, h1, l1;
          split_bf16(v[2 * e] * g[2 * e], h0, l0);
          split_bf16(v[2 * e + 1] * g[2 * e + 1], h1, l1);
          hi[e] = h0 | ((uint32_t)h1 << 16);
          lo[e] = l0 | ((uint32_t)l1 << 16);
          ss += v[2 * e] * v[2 * e] + v[2 * e + 1] * v[2 * e + 1];
        }
        *(f32x4*)(dst + (size_t)c * 8) = f32x4{v[0], v[1], v[2], v[3]};
        *(f32x4*)(dst + (size_t)c * 8 + 4) = f32x4{v[4], v[5], v[6], v[7]};
        *(u32x4*)(ob + (size_t)c * 8) = u32x4{hi[0], hi[1], hi[2], hi[3]};
        *(u32x4*)(ob_lo + (size_t)c * 8) = u32x4{lo[0], lo[1], lo[2], lo[3]};
      }
    }
  }
  ss = wave_sum(ss);
  if ((threadIdx.x & 63) == 0) wsum[threadIdx.x >> 6] = ss;
  __syncthreads();
  if (threadIdx.x == 0) ssp[row] = wsum[0] + wsum[1] + wsum[2] + wsum[3];
}

__global__ void __launch_bounds__(256) take_last_pack_kernel(
    const float* __restrict__ src, float* dst, int r, int d, int add_embed, const bf16_t* __restrict__ table,
    const int* __restrict__ tokens, int s_max, const DevState* st, int sel, int offset, const bf16_t* __restrict__ gain,
    bf16_t* __restrict__ xb, bf16_t* __restrict__ xb_lo, float* __restrict__ ssp, const float* add_rows /* nullable; may be dst */,
    const int* __restrict__ last_pos /* nullable: sequence b's row is the one at explicit position last_pos[b], if in this launch */,
    const int* __restrict__ fmap /* nullable: launch sequence -> sequence slot */) {
  const int bl = blockIdx.x, b = fmap ? fmap[bl] : bl;         // source rows by launch sequence, everything else by slot
  const int i = last_pos ? last_pos[b] - offset : r - 1;
  if (i < 0 || i >= r) return;
  const float* s = src + ((size_t)bl * r + i) * d;
  float* o = dst + (size_t)b * d;
  const bf16_t* e = nullptr;
  if (add_embed) e = table + (size_t)tokens[(size_t)b * s_max + row_base(st, sel, offset, b) + i] * d;
  const float* ar = add_rows ? add_rows + (size_t)b * d : nullptr;
  for (int k = threadIdx.x; k < d; k += blockDim.x) o[k] = s[k] + (add_embed ? bf16_to_f32(e[k]) : 0.0f) + (ar ? ar[k] : 0.0f);
  pack_row_for_norm(o, gain, d, xb + (size_t)b * d, xb_lo + (size_t)b * d, ssp + b);
}

__global__ void __launch_bounds__(256) add_embed_pack_kernel(
    float* __restrict__ h, const bf16_t* __restrict__ table, const int* __restrict__ tokens, int s_max, const DevState* st,
    int sel, int offset, int r, int d, const bf16_t* __restrict__ gain, bf16_t* __restrict__ xb, bf16_t* __restrict__ xb_lo,
    float* __restrict__ ssp) {
  const int row = blockIdx.x, b = row / r, i = row % r;
  const bf16_t* e = table + (size_t)tokens[(size_t)b * s_max + row_base(st, sel, offset, b) + i] * d;
  float* o = h + (size_t)row * d;
  for (int k = threadIdx.x; k < d; k += blockDim.x) o[k] += bf16_to_f32(e[k]);
  pack_row_for_norm(o, gain, d, xb + (size_t)row * d, xb_lo + (size_t)row * d, ssp + row);
}

// ---- ExDy variant (Sec. 2.1, last paragraph before Eq. 5): tokens inside a cycle pass the first
// ---- (encoding) layers in their own step; their encoding outputs wait in a per-sequence store
// ---- until the next full step refills the thinking layers from them.

// dst[row] = src_a[row_a] (+ src_b[row_b]); optionally the packed input of the next norm.
// One block per destination row.  Row selection, per mode:
//   ROWS_STASH   dst = store[b][n_tok - n_front] (the slot of the newest pending token), src_a = rows[b];
//                the pack (if any) is of the SOURCE row, into xb[b] (the row goes on to the decoding layers)
//   ROWS_GATHER  launch rows c0 .. c0 + rc - 1 of the r rows of a full step: row i < r - 1 comes from
//                store[b][i], row r - 1 (the newest token) from src_b[b]; dst = rows[b * rc + (i - c0)]
//   ROWS_ADD     dst[row] = src_a[row] + src_b[row], in place allowed
enum RowsMode : int { ROWS_STASH = 0, ROWS_GATHER = 1, ROWS_ADD = 2 };

template <bool PACK>
__global__ void __launch_bounds__(256) rows_op_kernel(int mode, float* __restrict__ dst, const float* src_a, const float* src_b,
                                                      int d, int store_rows /* slots per sequence */, int r, int c0, int rc,
                                                      const DevState* st, const bf16_t* __restrict__ gain,
                                                      bf16_t* __restrict__ xb, bf16_t* __restrict__ xb_lo, float* __restrict__ ssp) {
  const int row = blockIdx.x;
  const float* a = nullptr;
  const float* bsrc = nullptr;
  float* o = nullptr;
  int pack_row = row;
  if (mode == ROWS_STASH) {
    const int slot = st->n_tok - st->n_front;
    a = src_a + (size_t)row * d;
    o = dst + ((size_t)row * store_rows + slot) * d;
  } else if (mode == ROWS_GATHER) {
    const int b = row / rc, i = c0 + row % rc;
    a = i < r - 1 ? src_a + ((size_t)b * store_rows + i) * d : src_b + (size_t)b * d;
    o = dst + (size_t)row * d;
  } else {
    a = src_a + (size_t)row * d;
    bsrc = src_b + (size_t)row * d;
    o = dst + (size_t)row * d;
  }
  for (int k = threadIdx.x; k < d; k += blockDim.x) o[k] = a[k] + (bsrc ? bsrc[k] : 0.f);
  if (PACK) {
    __syncthreads();
    pack_row_for_norm(mode == ROWS_STASH ? a : o, gain, d, xb + (size_t)pack_row * d, xb_lo + (size_t)pack_row * d, ssp + pack_row);
  }
}

// Eq. 4 over the rows of one chunk of a whole-sequence forward (row b*r+i = position p0+i of sequence b), in place
// on the thinking layers' output h: a full position (mask 1) keeps h_think, any other position takes h_emb, the raw
// embedding of its token (ExDy variant: enc, the stored output of the encoding layers); under the literal reading
// the result is h_emb (or h_enc) + mask * h_think.  PACK: also the packed input of the decoding layers' first norm.
template <typename WT, bool PACK>
__global__ void __launch_bounds__(256) mask_combine_kernel(float* __restrict__ h, const float* __restrict__ enc, const WT* __restrict__ table,
                                                           const int* __restrict__ tokens, int s_max, const int* __restrict__ mask,
                                                           int p0, int r, int d, int literal, const bf16_t* __restrict__ gain,
                                                           bf16_t* __restrict__ xb, bf16_t* __restrict__ xb_lo, float* __restrict__ ssp) {
  const int row = blockIdx.x, b = row / r, pos = p0 + row % r;
  const bool full = mask[pos] != 0;
  float* o = h + (size_t)row * d;
  const float* e = enc ? enc + (size_t)row * d : nullptr;
  const WT* t = table + (size_t)tokens[(size_t)b * s_max + pos] * d;
  if (literal || !full) {
    for (int k = threadIdx.x; k < d; k += blockDim.x) {
      const float base = e ? e[k] : Elem<WT>::to_f32(t[k]);
      o[k] = literal ? base + (full ? o[k] : 0.f) : base;
    }
  }
  if (PACK) {
    __syncthreads();
    pack_row_for_norm(o, gain, d, xb + (size_t)row * d, xb_lo + (size_t)row * d, ssp + row);
  }
}

}  // namespace dmtd
