// Weight-streaming GEMV kernels for small row counts (M <= 4 activation rows) on gfx950.
//
// y[m, n] = sum_k W[n, k] * xhat[m, k], W row-major [N, K] in HBM (bf16 or fp32), read
// exactly once per launch in 16-byte per-lane nontemporal loads; accumulation in fp32.
// The weight loads of a wave's next unit of work are issued before the current unit is
// reduced and stored, and the first unit's loads are issued before the activation rows
// are staged, so the HBM stream does not wait for the prologue or the epilogues.
//
//  gemv_rows_kernel   : a wave owns whole output rows (4 at a time), lanes stride K.  For
//                       wide outputs and short rows (QKV, gate/up, LM head).  Activation rows
//                       are staged in LDS as fp32, optionally RMS-normalised on the way.
//  gemv_ksplit_kernel : a block owns 8 output rows and its 4 waves split K.  For narrow
//                       outputs with long rows (O projection, down projection), where
//                       whole-row waves would leave most of the chip idle.  Each lane keeps
//                       its own slices of the activation rows in registers.
#pragma once
#include "kernels.hpp"

namespace dmtd {

enum GemvEpi : int { EPI_STORE = 0, EPI_RESID = 1, EPI_SWIGLU = 2, EPI_LOGITS = 3 };

struct GemvArgs {
  const void* W;        // [N, K]; for SWIGLU the gate matrix
  const void* W2;       // SWIGLU: the up matrix [N, K]
  const void* gain;     // norm gain [K] (NORM only)
  const float* x;       // [M, ldx]
  float* y;             // [M, ldy]
  int ldx, ldy, N, K;
  float eps;
  unsigned long long* amax;   // LOGITS: one selection key per sequence of this launch (already offset)
};

// Sum V (a power of two <= 64) per-lane values over the 64 lanes with V - 1 + (6 - log2 V)
// shuffles: at each of the first log2 V steps a lane hands half of its values to its
// partner and keeps the other half.  Afterwards lane L holds, in v[0], the wave total of
// the value with index L >> (6 - log2 V).
template <int V>
__device__ __forceinline__ float wave_reduce_multi(float (&v)[V], int lane) {
  static_assert(V >= 1 && V <= 64 && (V & (V - 1)) == 0, "V must be a power of two");
  constexpr int LOG = V == 1 ? 0 : V == 2 ? 1 : V == 4 ? 2 : V == 8 ? 3 : V == 16 ? 4 : V == 32 ? 5 : 6;
#pragma unroll
  for (int s = 0; s < LOG; ++s) {
    const int o = 32 >> s, n = V >> s;
    const bool up = (lane & o) != 0;
#pragma unroll
    for (int i = 0; i < n / 2; ++i) {
      const float send = up ? v[i] : v[i + n / 2];
      const float keep = up ? v[i + n / 2] : v[i];
      v[i] = keep + __shfl_xor(send, o, 64);
    }
  }
#pragma unroll
  for (int s = LOG; s < 6; ++s) v[0] += __shfl_xor(v[0], 32 >> s, 64);
  return v[0];
}

template <int M> struct PadRows { static constexpr int MP = M == 3 ? 4 : M; static constexpr int SH = MP == 1 ? 0 : MP == 2 ? 1 : 2; };

template <typename WT, int M, int EPI, bool NORM, int GEMV_ITS>   // GEMV_ITS: k-iterations (of 512) a wave prefetches per row
__global__ void __launch_bounds__(256) gemv_rows_kernel(GemvArgs a) {
  extern __shared__ float4 smem4[];
  float* xs = (float*)smem4;                       // [M][K]
  __shared__ float red[4][M];
  __shared__ float rs_s[M];
  __shared__ unsigned long long best_s[M];
  typedef typename Elem<WT>::Raw Raw;
  constexpr int MP = PadRows<M>::MP, V = 4 * MP, NR = 4;
  constexpr int LOGV = V == 4 ? 2 : V == 8 ? 3 : 4;
  constexpr int RPW = (EPI == EPI_SWIGLU) ? 2 : 4;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int K = a.K, N = a.N;
  const WT* __restrict__ W = (const WT*)a.W;
  const WT* __restrict__ W2 = (const WT*)a.W2;

  const int n_tasks = (N + RPW - 1) / RPW;
  const int n_chunks = (K + 512 * GEMV_ITS - 1) / (512 * GEMV_ITS);
  const int first = blockIdx.x * 4 + wave, stride = gridDim.x * 4;
  const int n_units = first < n_tasks ? ((n_tasks - first - 1) / stride + 1) * n_chunks : 0;

  Raw wr[NR][GEMV_ITS];
  auto load_unit = [&](int u) {
    const int n0 = (first + (u / n_chunks) * stride) * RPW;
    const int kbase = (u % n_chunks) * (512 * GEMV_ITS) + lane * 8;
#pragma unroll
    for (int r = 0; r < NR; ++r) {
      const WT* row;
      if (EPI == EPI_SWIGLU) row = ((r < 2) ? W : W2) + (size_t)min(n0 + (r & 1), N - 1) * K;
      else row = W + (size_t)min(n0 + r, N - 1) * K;
#pragma unroll
      for (int it = 0; it < GEMV_ITS; ++it) {
        const int k0 = kbase + it * 512;
        wr[r][it] = k0 < K ? Elem<WT>::load_raw(row + k0) : Elem<WT>::zero_raw();
      }
    }
  };
  if (n_units > 0) load_unit(0);

  // stage the activation rows in LDS (K is a multiple of 8), with the RMSNorm folded in
  float ss[M];
#pragma unroll
  for (int m = 0; m < M; ++m) ss[m] = 0.f;
  for (int k = tid * 4; k < K; k += 256 * 4) {
#pragma unroll
    for (int m = 0; m < M; ++m) {
      const float4 v = *(const float4*)(a.x + (size_t)m * a.ldx + k);
      ss[m] += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
      *(float4*)(xs + m * K + k) = v;
    }
  }
  if (EPI == EPI_LOGITS && tid < M) best_s[tid] = 0ull;
  if (NORM) {
#pragma unroll
    for (int m = 0; m < M; ++m) {
      const float s = wave_sum(ss[m]);
      if (lane == 0) red[wave][m] = s;
    }
    __syncthreads();
    if (tid < M) rs_s[tid] = rsqrtf((red[0][tid] + red[1][tid] + red[2][tid] + red[3][tid]) / (float)K + a.eps);
    __syncthreads();
    const WT* __restrict__ g = (const WT*)a.gain;
    for (int k = tid; k < K; k += 256) {
      const float gk = Elem<WT>::to_f32(g[k]);
#pragma unroll
      for (int m = 0; m < M; ++m) xs[m * K + k] *= rs_s[m] * gk;
    }
  }
  __syncthreads();

  float acc[V];
  unsigned long long best = 0ull;
  const int my_idx = lane >> (6 - LOGV);            // value this lane owns after the reduction
  const int my_r = my_idx >> PadRows<M>::SH, my_m = my_idx & (MP - 1);
  const bool owner = (lane & ((64 >> LOGV) - 1)) == 0 && my_m < M;

  for (int u = 0; u < n_units; ++u) {
    const int chunk = u % n_chunks;
    if (chunk == 0) {
#pragma unroll
      for (int i = 0; i < V; ++i) acc[i] = 0.f;
    }
    const int kbase = chunk * (512 * GEMV_ITS) + lane * 8;
#pragma unroll
    for (int it = 0; it < GEMV_ITS; ++it) {
      const int k0 = kbase + it * 512;
      if (k0 < K) {
        float xv[M][8];
#pragma unroll
        for (int m = 0; m < M; ++m) {
          const float4 xa = *(const float4*)(xs + m * K + k0);
          const float4 xb = *(const float4*)(xs + m * K + k0 + 4);
          xv[m][0] = xa.x; xv[m][1] = xa.y; xv[m][2] = xa.z; xv[m][3] = xa.w;
          xv[m][4] = xb.x; xv[m][5] = xb.y; xv[m][6] = xb.z; xv[m][7] = xb.w;
        }
#pragma unroll
        for (int r = 0; r < NR; ++r) {
          float w[8];
          Elem<WT>::unpack(wr[r][it], w);
#pragma unroll
          for (int m = 0; m < M; ++m) {
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[r * MP + m] += w[e] * xv[m][e];
          }
        }
      }
    }
    const int n0 = (first + (u / n_chunks) * stride) * RPW;
    if (u + 1 < n_units) load_unit(u + 1);          // next unit's weights fly while this one is reduced
    if (chunk != n_chunks - 1) continue;

    const float tot = wave_reduce_multi<V>(acc, lane);
    if (EPI == EPI_SWIGLU) {
      // values 0,1 (x MP) are the gate sums of outputs n0, n0+1; values 2,3 the up sums
      const float up = __shfl(tot, (my_idx + 2 * MP) << (6 - LOGV), 64);
      if (owner && my_r < 2 && n0 + my_r < N)
        a.y[(size_t)my_m * a.ldy + n0 + my_r] = tot / (1.0f + __expf(-tot)) * up;
    } else if (owner && n0 + my_r < N) {
      float* dst = a.y + (size_t)my_m * a.ldy + n0 + my_r;
      if (EPI == EPI_RESID) *dst += tot; else *dst = tot;
      if (EPI == EPI_LOGITS) {
        const unsigned long long key = argmax_key(tot, n0 + my_r);
        if (key > best) best = key;
      }
    }
  }

  if (EPI == EPI_LOGITS) {
    if (owner && best != 0ull) atomicMax(&best_s[my_m], best);
    __syncthreads();
    if (tid < M && best_s[tid] != 0ull) atomicMax(a.amax + tid, best_s[tid]);
  }
}

// Block = NW waves = 4*RG output rows (RG groups of 4); wave w takes the k-iterations
// w, w+NW, w+2NW, ... (ITS of them at most, so K <= NW * ITS * 512).
template <typename WT, int M, int EPI, int ITS, int NW, int RG>
__global__ void __launch_bounds__(64 * NW) gemv_ksplit_kernel(GemvArgs a) {
  typedef typename Elem<WT>::Raw Raw;
  constexpr int MP = PadRows<M>::MP, V = 4 * MP;
  constexpr int LOGV = V == 4 ? 2 : V == 8 ? 3 : 4;
  __shared__ float red[RG][NW][V];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int K = a.K, N = a.N;
  const WT* __restrict__ W = (const WT*)a.W;
  const int nb0 = blockIdx.x * (4 * RG);

  Raw wr[4][ITS];
  auto load_group = [&](int rg) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const WT* row = W + (size_t)min(nb0 + rg * 4 + r, N - 1) * K;
#pragma unroll
      for (int j = 0; j < ITS; ++j) {
        const int k0 = (wave + NW * j) * 512 + lane * 8;
        wr[r][j] = k0 < K ? Elem<WT>::load_raw(row + k0) : Elem<WT>::zero_raw();
      }
    }
  };
  load_group(0);

  float xr[M][ITS][8];
#pragma unroll
  for (int j = 0; j < ITS; ++j) {
    const int k0 = (wave + NW * j) * 512 + lane * 8;
#pragma unroll
    for (int m = 0; m < M; ++m) {
      float4 xa = make_float4(0, 0, 0, 0), xb = xa;
      if (k0 < K) {
        xa = *(const float4*)(a.x + (size_t)m * a.ldx + k0);
        xb = *(const float4*)(a.x + (size_t)m * a.ldx + k0 + 4);
      }
      xr[m][j][0] = xa.x; xr[m][j][1] = xa.y; xr[m][j][2] = xa.z; xr[m][j][3] = xa.w;
      xr[m][j][4] = xb.x; xr[m][j][5] = xb.y; xr[m][j][6] = xb.z; xr[m][j][7] = xb.w;
    }
  }

#pragma unroll
  for (int rg = 0; rg < RG; ++rg) {
    float acc[V];
#pragma unroll
    for (int i = 0; i < V; ++i) acc[i] = 0.f;
#pragma unroll
    for (int j = 0; j < ITS; ++j) {
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        float w[8];
        Elem<WT>::unpack(wr[r][j], w);
#pragma unroll
        for (int m = 0; m < M; ++m) {
#pragma unroll
          for (int e = 0; e < 8; ++e) acc[r * MP + m] += w[e] * xr[m][j][e];
        }
      }
    }
    if (rg + 1 < RG) load_group(rg + 1);
    const float tot = wave_reduce_multi<V>(acc, lane);
    if ((lane & ((64 >> LOGV) - 1)) == 0) red[rg][wave][lane >> (6 - LOGV)] = tot;
  }
  __syncthreads();
  if (tid < RG * V) {
    const int rg = tid / V, idx = tid % V, r = idx >> PadRows<M>::SH, m = idx & (MP - 1);
    const int n = nb0 + rg * 4 + r;
    if (m < M && n < N) {
      float s = 0.f;
#pragma unroll
      for (int w = 0; w < NW; ++w) s += red[rg][w][idx];
      float* dst = a.y + (size_t)m * a.ldy + n;
      if (EPI == EPI_RESID) *dst += s; else *dst = s;
    }
  }
}

}  // namespace dmtd
