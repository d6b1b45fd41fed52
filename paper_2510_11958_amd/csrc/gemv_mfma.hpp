// MFMA weight-streaming "skinny GEMM" for 2..16 activation rows of a bf16 model on gfx950.
//
// y[m, n] = sum_k W[n, k] * xhat[m, k].  The weights are the A operand of
// v_mfma_f32_16x16x32_bf16 and are loaded from HBM straight into the operand registers:
// lane (row = lane % 16, kg = lane / 16) owns 32 contiguous bytes of its row per k-step of
// 64 elements, so the four lanes of a row fetch one whole 128-byte line and every weight
// byte is read exactly once.  The activation rows are the B operand (column = lane % 16),
// converted to bf16 on the way in; columns beyond M are zero.  The order of k inside a
// k-step is permuted identically for A and B (first MFMA: elements kg*16 + 0..7, second:
// kg*16 + 8..15), which a dot product does not notice.  No cross-lane reduction is needed:
// the matrix core sums over k, and a lane ends up holding 4 rows of one output column.
//
// A block owns one tile of 16 output rows (SwiGLU: the gate tile and the up tile of the
// same 16 outputs); its waves split K into runs of at most PF k-steps, all loads of a wave
// are issued at once, and the waves' partial tiles are summed through LDS in wave order.
// RMSNorm is folded in exactly: the B operand carries x*gain and the epilogue multiplies
// column m by rsqrt(mean(x_m^2) + eps), whose sum of squares the waves gather on the way.
#pragma once
#include "gemv.hpp"

namespace dmtd {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  return (uint32_t)f32_to_bf16(lo) | ((uint32_t)f32_to_bf16(hi) << 16);
}

constexpr int MFMA_MAX_WAVES = 16;   // waves that split K for one tile

template <int EPI, bool NORM, int PF>
__global__ void __launch_bounds__(1024) gemv_mfma_kernel(GemvArgs a, int M, int nw) {
  constexpr int MATS = (EPI == EPI_SWIGLU) ? 2 : 1;
  __shared__ float red[MATS][MFMA_MAX_WAVES][16][16];   // [matrix][wave][row][column]
  __shared__ float ssred[MFMA_MAX_WAVES][16];
  const int tid = threadIdx.x, lane = tid & 63, wall = tid >> 6;
  const int mat = wall / nw, w = wall % nw;
  const int r = lane & 15, kg = lane >> 4;     // A: row r of the tile; B and D: column r
  const int K = a.K, N = a.N;
  const int tile = blockIdx.x;
  const int KS = K >> 6;                       // k-steps of 64 elements
  const int s0 = (int)((long)w * KS / nw), s1 = (int)((long)(w + 1) * KS / nw);

  const bf16_t* __restrict__ Wm = (const bf16_t*)(mat == 0 ? a.W : a.W2);
  const bf16_t* arow = Wm + (size_t)min(tile * 16 + r, N - 1) * K + kg * 16;
  u32x4 A[PF][2];
#pragma unroll
  for (int i = 0; i < PF; ++i) {
    const int s = s0 + i;
    if (s < s1) {
      A[i][0] = __builtin_nontemporal_load((const u32x4*)(arow + (size_t)s * 64));
      A[i][1] = __builtin_nontemporal_load((const u32x4*)(arow + (size_t)s * 64 + 8));
    } else {
      A[i][0] = u32x4{0, 0, 0, 0}; A[i][1] = A[i][0];
    }
  }

  // B operand: column r (activation row r) of this wave's k-range, times the norm gain
  const bool colact = r < M;
  const float* xrow = a.x + (size_t)(colact ? r : 0) * a.ldx + kg * 16;
  const bf16_t* grow = (const bf16_t*)a.gain + kg * 16;
  u32x4 B[PF][2];
  float ss = 0.f;
#pragma unroll
  for (int i = 0; i < PF; ++i) {
    const int s = s0 + i;
    B[i][0] = u32x4{0, 0, 0, 0}; B[i][1] = B[i][0];
    if (s < s1 && colact) {
      float xv[16];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const float4 v = *(const float4*)(xrow + (size_t)s * 64 + q * 4);
        xv[q * 4 + 0] = v.x; xv[q * 4 + 1] = v.y; xv[q * 4 + 2] = v.z; xv[q * 4 + 3] = v.w;
      }
      if (NORM) {
        float gv[16];
        float g8[8];
        Elem<bf16_t>::unpack(*(const u32x4*)(grow + (size_t)s * 64), g8);
#pragma unroll
        for (int e = 0; e < 8; ++e) gv[e] = g8[e];
        Elem<bf16_t>::unpack(*(const u32x4*)(grow + (size_t)s * 64 + 8), g8);
#pragma unroll
        for (int e = 0; e < 8; ++e) gv[8 + e] = g8[e];
#pragma unroll
        for (int e = 0; e < 16; ++e) { ss += xv[e] * xv[e]; xv[e] *= gv[e]; }
      }
      B[i][0] = u32x4{pack_bf16x2(xv[0], xv[1]), pack_bf16x2(xv[2], xv[3]), pack_bf16x2(xv[4], xv[5]), pack_bf16x2(xv[6], xv[7])};
      B[i][1] = u32x4{pack_bf16x2(xv[8], xv[9]), pack_bf16x2(xv[10], xv[11]), pack_bf16x2(xv[12], xv[13]), pack_bf16x2(xv[14], xv[15])};
    }
  }

  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int i = 0; i < PF; ++i) {
    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, A[i][0]), __builtin_bit_cast(bf16x8_t, B[i][0]), acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, A[i][1]), __builtin_bit_cast(bf16x8_t, B[i][1]), acc, 0, 0, 0);
  }
  // lane (column r, kg) holds rows kg*4 .. kg*4+3 of column r
  if (colact) {
    red[mat][w][kg * 4 + 0][r] = acc.x; red[mat][w][kg * 4 + 1][r] = acc.y;
    red[mat][w][kg * 4 + 2][r] = acc.z; red[mat][w][kg * 4 + 3][r] = acc.w;
  }
  if (NORM && mat == 0) {
    ss += __shfl_xor(ss, 16, 64);
    ss += __shfl_xor(ss, 32, 64);
    if (kg == 0) ssred[w][r] = ss;
  }
  __syncthreads();
  for (int t = tid; t < 256; t += blockDim.x) {
    const int row = t >> 4, c = t & 15, n = tile * 16 + row;
    if (c >= M || n >= N) continue;
    float rs = 1.f;
    if (NORM) {
      float s = 0.f;
      for (int ww = 0; ww < nw; ++ww) s += ssred[ww][c];
      rs = rsqrtf(s / (float)K + a.eps);
    }
    float v0 = 0.f;
    for (int ww = 0; ww < nw; ++ww) v0 += red[0][ww][row][c];
    v0 *= rs;
    float* dst = a.y + (size_t)c * a.ldy + n;
    if (EPI == EPI_SWIGLU) {
      float v1 = 0.f;
      for (int ww = 0; ww < nw; ++ww) v1 += red[MATS - 1][ww][row][c];
      v1 *= rs;
      *dst = v0 / (1.0f + __expf(-v0)) * v1;
    } else if (EPI == EPI_RESID) {
      *dst += v0;
    } else {
      *dst = v0;
    }
  }
}

}  // namespace dmtd
