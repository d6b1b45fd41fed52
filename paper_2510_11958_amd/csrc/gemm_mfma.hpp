// Weight-streaming projection for 6..128 activation rows of a bf16 model on gfx950 (batched
// decode steps, refill rows of several sequences, prefill of a batch): the rows form CG = 1, 2, 4 or 8
// groups of 16 MFMA columns and ONE pass over the weights serves them all.
//
// With this many rows the activations no longer fit in LDS whole, and a block that owned one
// 16-row weight tile (as the 1..16-row kernel does) would pull every activation through L2 again
// for every tile.  Here a wave owns 2 weight tiles (SwiGLU: the gate and the up tile of the same 16
// outputs), a block has 4 or 8 waves (gemm_waves) and walks K in steps of 64:
//   * weights: operand-order tiles straight from HBM into registers, PF = 3 k-steps ahead per wave
//     (2 with 64 and more rows);
//   * activations: the k-step's slice of all rows, both bf16 planes (see gemv_mfma.hpp), fetched
//     by all threads as far ahead into registers, written to one of two LDS buffers and shared
//     by the block's tiles, every B fragment feeding the matrix cores twice (one per tile of a wave);
//     with 128 rows the slices go from memory straight into a ring of LDS buffers instead (see below).
// One block barrier per k-step.  A wave owns its tiles over the block's whole k-range, so nothing is
// reduced across waves.  The loop is laid out so that every wait counts exactly the loads that may stay
// in flight: the first PF steps are issued without a bounds check, the main loop covers only steps whose
// successor PF ahead exists, and the tail is one straight-line copy per number of remaining steps.
//
// Memory-level parallelism: a tile has 3 k-steps (6 KiB) in flight, so a projection with few tiles
// (QKV 384, O and down 160 at 4B shapes) would keep only 1-2 MB in flight, far below what HBM needs
// (about 12 MB), on a fraction of the chip.  Such launches split K over gridDim.y blocks, as many as
// give the launch about one block per CU (the launcher decides); each stores its raw partial tile
// sums, and gemm_finish_kernel adds them in order and runs the epilogue.  The LM head (thousands of
// tiles) runs unsplit with the epilogue in this kernel.
#pragma once
#include <type_traits>
#include "gemv_mfma.hpp"

namespace dmtd {

#ifndef DMTD_GEMM_PF
#define DMTD_GEMM_PF 3
#endif
#ifndef DMTD_GEMM_KSMAX
#define DMTD_GEMM_KSMAX 12
#endif
#ifndef DMTD_GEMM_KSMAX_GU
#define DMTD_GEMM_KSMAX_GU 3
#endif
// compile-time loop: f(integral_constant<int, I>) for I in [I0, N)
template <int I, int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>());
    static_for<I + 1, N>(f);
  }
}

// Waves per block (a wave owns 2 weight tiles; SwiGLU: the gate and up tile of the same outputs).  With 32 and more rows a
// k-step's slice of activations is as big as the weights a 4-wave block streams against it, so projections with many
// tiles put 8 waves on a slice (measured at 4B shapes, 64 rows: gate/up 32.8 against 37.4 us, QKV 18.7 against 19.9);
// the residual projections have few tiles (160) and would leave most of the chip idle (down: 26.5 against 20.6 us).
// With 128 rows the accumulators leave registers for 8 waves only in the SwiGLU kernel (the others would spill).
constexpr int gemm_waves(int cg, int epi) { return (cg >= 2 && epi != EPI_RESID && (cg <= 4 || epi == EPI_SWIGLU)) ? 8 : 4; }

// With 64 and more rows (DMA) the activation slices do not pass through registers: every wave sends its share of a
// k-step's slice from memory straight into LDS (global_load ... lds: lane l of an instruction lands 16 bytes at the
// instruction's LDS base + 16 l), into a ring of PF + 1 slices, so the accumulators and PF k-steps of weights are all the
// registers hold and a slice is requested PF steps (several microseconds) before it is used.  LDS rows are the plain 64
// values of a k-step (128 bytes) with their eight 16-byte chunks permuted by the row number (chunk c of row i at place
// c ^ (i & 7)): an instruction's 64 lanes fill 8 whole rows, each lane fetching the chunk that belongs at its place, and
// the B-fragment reads (16 rows, one chunk each) spread over all banks.  Loads return in order, and a step's slice
// requests are issued ahead of its weight requests, so "all but the newer steps' loads have returned" (one counter
// wait before the block barrier) covers the slice.
// Measured at 4B shapes (us per launch incl. the finishing launch, slices through registers / straight to LDS): 128 rows:
// gate/up 42.5 / 40.7, down 26.7 / 26.0, QKV 23.9 / 23.6, O 20.4 / 19.8; 64 rows: gate/up 30.2 / 31.3, down 18.5 / 18.8,
// QKV 18.3 / 19.8, O 13.4 / 14.0 - so only the 128-row kernels take the direct path (3 k-steps in flight instead of 2).
constexpr bool gemm_uses_dma(int cg) { return cg >= 8; }
constexpr int gemm_pf(int cg) { return cg >= 8 ? 3 : (cg >= 4 ? (DMTD_GEMM_PF < 2 ? DMTD_GEMM_PF : 2) : DMTD_GEMM_PF); }
// dynamic LDS of a launch (bytes): the ring of activation slices
constexpr size_t gemm_dyn_lds(int cg) { return gemm_uses_dma(cg) ? (size_t)(gemm_pf(cg) + 1) * 2 * cg * 16 * 64 * 2 : 0; }

template <int EPI, bool NORM, int CG, bool SPLITK>
__global__ void __launch_bounds__(64 * gemm_waves(CG, EPI)) gemm_mfma_kernel(
    // what the prologue needs first, as leading scalars: they arrive in registers with the wave (kernel-argument preload), the
    // struct's fields only after a load from the argument buffer (~1 us before the first weight could be requested)
    const bf16_t* W_, const bf16_t* W2_, const bf16_t* xb_, const bf16_t* xb_lo_, int M_, int N_, int K_, int ldxb_, int ksplit_,
    MfmaArgs a) {
  constexpr int GEMM_WAVES = gemm_waves(CG, EPI);
  constexpr int BM = CG * 16;            // activation rows (MFMA columns) per pass
  // k-steps in flight: 3; 2 with 64 and more rows, where the accumulators leave fewer registers (measured at 4B shapes, 64 rows:
  // gate/up 37.4 against 38.8 us, QKV 19.9 against 21.9)
  constexpr bool DMA = gemm_uses_dma(CG);
  constexpr int PF = gemm_pf(CG);
  constexpr int LDB = 72;                // LDS row (register-staged slices): 64 values + 8 of padding
  constexpr int NT = 64 * GEMM_WAVES;
  constexpr int PIECES = 2 * BM * 8;     // 16-byte pieces of one k-step's activation slice (2 planes)
  constexpr int PPT = PIECES / NT;       // per thread
  static_assert(PIECES % NT == 0, "pieces per thread");
  constexpr int NBUF = PF + 1;           // DMA: slices in the ring
  constexpr int SLICE = 2 * BM * 64;     // DMA: bf16 elements of a slice (both planes, rows of 64)
  constexpr int LPS = PPT + 4;           // loads a thread issues per k-step (slice pieces, then 2 tiles x 2 halves of weights)
  static_assert(!DMA || (PF - 1) * LPS <= 63, "the counter wait has 6 bits");
  __shared__ __attribute__((aligned(16))) bf16_t bs[2][2][DMA ? 1 : BM][LDB];    // [buffer][plane][row][k] (register-staged slices)
  extern __shared__ float4 gemm_dyn_smem[];
  bf16_t* ring = (bf16_t*)gemm_dyn_smem;                                         // DMA: [NBUF][plane][row][64], chunks permuted
  __shared__ float rs_s[BM];
  __shared__ unsigned long long key_s[BM];
  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int r = lane & 15, kg = lane >> 4;
  const int M = M_, N = N_, K = K_, KS = K >> 6;
  const int n_tiles = (N + 15) >> 4;
  // this block's k-steps
  const int s_lo = SPLITK ? (int)((long)blockIdx.y * KS / ksplit_) : 0;
  const int s_hi = SPLITK ? (int)((long)(blockIdx.y + 1) * KS / ksplit_) : KS;

  int tile[2];
  const bf16_t* wp[2];
  if (EPI == EPI_SWIGLU) {
    tile[0] = tile[1] = blockIdx.x * GEMM_WAVES + w;
    wp[0] = W_; wp[1] = W2_;
  } else {
    tile[0] = (blockIdx.x * GEMM_WAVES + w) * 2; tile[1] = tile[0] + 1;
    wp[0] = wp[1] = W_;
  }
  const bool tv[2] = {tile[0] < n_tiles, tile[1] < n_tiles};
  const bf16_t* abase[2];
#pragma unroll
  for (int j = 0; j < 2; ++j) abase[j] = wp[j] + ((size_t)(tv[j] ? tile[j] : 0) * KS) * 1024 + lane * 8;

  // this thread's pieces of an activation slice: piece q = (plane, row, 16-byte column c8); rows beyond M repeat row M-1
  // (their MFMA columns are never stored)
  const bf16_t* bsrc[PPT];
  int bdst[PPT];
#pragma unroll
  for (int i = 0; i < PPT; ++i) {
    if (DMA) {
      // instruction J = w * PPT + i of a slice fills the 8 rows 8 J .. 8 J + 7 of the plane-major row space; this lane lands at
      // (row 8 J + lane / 8, place lane % 8) and therefore fetches chunk place ^ (row & 7) of that row
      const int J = w * PPT + i, plane = J / (BM / 8), row = (J % (BM / 8)) * 8 + (lane >> 3), c8 = (lane & 7) ^ (lane >> 3);
      bsrc[i] = (plane ? xb_lo_ : xb_) + (size_t)min(row, M - 1) * ldxb_ + c8 * 8;
      bdst[i] = J * 512;                   // the instruction's LDS base inside a slice (elements): wave-uniform
    } else {
      const int q = tid + i * NT, plane = q / (BM * 8), row = (q >> 3) % BM, c8 = q & 7;
      bsrc[i] = (plane ? xb_lo_ : xb_) + (size_t)min(row, M - 1) * ldxb_ + c8 * 8;
      bdst[i] = (plane * BM + row) * LDB + c8 * 8;
    }
  }

  u32x4 A[PF][2][2];     // [slot][tile][half of the k-step]
  u32x4 Bq[DMA ? 1 : PF][PPT];
  int buf_issue = 0;     // DMA: ring slice the next issue fills (advances with every issue)
  auto issue_always = [&](int s, int slot) {      // slot is a compile-time constant at every call
    if constexpr (DMA) {
      bf16_t* dst = ring + buf_issue * SLICE;
#pragma unroll
      for (int i = 0; i < PPT; ++i)
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(bsrc[i] + (size_t)s * 64),
                                         (__attribute__((address_space(3))) void*)(dst + bdst[i]), 16, 0, 0);
      buf_issue = buf_issue + 1 == NBUF ? 0 : buf_issue + 1;
    } else {
#pragma unroll
      for (int i = 0; i < PPT; ++i) Bq[slot][i] = *(const u32x4*)(bsrc[i] + (size_t)s * 64);
    }
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      A[slot][j][0] = __builtin_nontemporal_load((const u32x4*)(abase[j] + (size_t)s * 1024));
      A[slot][j][1] = __builtin_nontemporal_load((const u32x4*)(abase[j] + (size_t)s * 1024 + 512));
    }
  };
  // the first PF steps, unconditionally (a range shorter than PF re-reads its last step into slots no step consumes):
  // a bounds check here would leave the compiler unsure which loads are in flight at the head of the main loop
#pragma unroll
  for (int s = 0; s < PF; ++s) issue_always(s_lo + s < s_hi ? s_lo + s : s_hi - 1, s);

  if (NORM && !SPLITK) {
    // the rows' 1/rms while the first weights are on their way: wave w takes rows w, w + waves, ..., its lanes the producer's
    // partial sums of squares, four loads per lane in flight (one thread per row walking all parts in turn cost every block
    // of the LM head ~160 dependent loads in its epilogue: 210 us per launch in the step against 147 with a single part)
    for (int m = w; m < M; m += GEMM_WAVES) {
      float sacc = 0.f;
      for (int p0 = 0; p0 < a.n_parts; p0 += 256) {
        float v4[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int p = p0 + lane + 64 * j;
          v4[j] = a.ssp[(size_t)(p < a.n_parts ? p : a.n_parts - 1) * a.ssp_ld + m];
        }
#pragma unroll
        for (int j = 0; j < 4; ++j)
          if (p0 + lane + 64 * j < a.n_parts) sacc += v4[j];
      }
      sacc = wave_sum(sacc);
      if (lane == 0) rs_s[m] = rsqrtf(sacc / (float)K + a.eps);
    }
  }

  f32x4 acc[2][CG];
#pragma unroll
  for (int j = 0; j < 2; ++j)
#pragma unroll
    for (int g = 0; g < CG; ++g) acc[j][g] = f32x4{0.f, 0.f, 0.f, 0.f};

  int buf_use = 0;       // DMA: ring slice of the step at hand
  // DMA: this lane's two chunks of a B fragment row (k halves 0 and 1), permuted as the slices are stored
  const int rd0 = r * 64 + ((kg ^ (r & 7)) << 3), rd1 = r * 64 + (((4 + kg) ^ (r & 7)) << 3);
  auto step = [&](int s, int slot, auto mode_c) {
    constexpr int MODE = decltype(mode_c)::value;
    bf16_t* buf;
    if constexpr (DMA) {
      buf = ring + buf_use * SLICE;
      buf_use = buf_use + 1 == NBUF ? 0 : buf_use + 1;
      // this step's slice pieces (requested ahead of its weights, PF steps ago) have landed once all loads but those of
      // the PF - 1 newer steps have returned; with nothing newer on its way for certain (the tail), all loads
      // the barrier is the bare instruction: the block-wide fence of __syncthreads would wait for every load in flight, the
      // newer steps' included (the slice requests count as writes to LDS)
      constexpr int VM = MODE == 1 ? (PF - 1) * LPS : 0;
      __builtin_amdgcn_s_waitcnt((VM & 0xF) | ((VM >> 4) << 14) | (7 << 4));       // vmcnt(VM) lgkmcnt(0), expcnt untouched
      __builtin_amdgcn_s_barrier();
      asm volatile("" ::: "memory");      // no LDS read of the slice moves above the barrier
    } else {
      buf = &bs[s & 1][0][0][0];
#pragma unroll
      for (int i = 0; i < PPT; ++i) *(u32x4*)(buf + bdst[i]) = Bq[slot][i];
      __syncthreads();
    }
#pragma unroll
    for (int g = 0; g < CG; ++g) {
#pragma unroll
      for (int plane = 1; plane >= 0; --plane) {
        const bf16_t* row = DMA ? buf + (plane * BM + g * 16) * 64 + rd0 : buf + (plane * BM + g * 16 + r) * LDB + kg * 8;
        const bf16x8_t b0 = __builtin_bit_cast(bf16x8_t, *(const u32x4*)row);
        const bf16x8_t b1 = __builtin_bit_cast(bf16x8_t, *(const u32x4*)(DMA ? row - rd0 + rd1 : row + 32));
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          acc[j][g] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, A[slot][j][0]), b0, acc[j][g], 0, 0, 0);
          acc[j][g] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, A[slot][j][1]), b1, acc[j][g], 0, 0, 0);
        }
      }
    }
    // MODE 1: the step PF ahead exists for certain: an unconditional issue, so the compiler knows how many loads are
    // in flight at every wait and a step waits for its own loads only (behind a bounds check it has to assume the
    // worst at the loop head and drains every load each round).  MODE 0: nothing left to fetch.
    if (MODE == 1) issue_always(s + PF, slot);
  };
  int s0 = s_lo;
  for (; s0 + 2 * PF <= s_hi; s0 += PF) {
#pragma unroll
    for (int u = 0; u < PF; ++u) step(s0 + u, u, std::integral_constant<int, 1>());
  }
  // R < 2 PF steps left.  R >= PF: steps u < R - PF still have a step PF ahead (issued without a check, so the waits stay
  // exact), the others have none; one straight-line copy per R.  R < PF (a k-range shorter than the pipeline): plain steps.
  auto tail = [&](auto r_c) {
    constexpr int R = decltype(r_c)::value;
    static_for<0, PF>([&](auto u) {
      constexpr int U = decltype(u)::value;
      step(s0 + U, U, std::integral_constant<int, (U + PF < R) ? 1 : 0>());
    });
    static_for<0, R - PF>([&](auto u) {
      constexpr int U = decltype(u)::value;
      step(s0 + PF + U, U, std::integral_constant<int, 0>());
    });
  };
  const int rem = s_hi - s0;
  if (rem >= PF) {
    static_for<PF, 2 * PF>([&](auto r) {
      if (rem == decltype(r)::value) tail(r);
    });
  } else {
#pragma unroll
    for (int u = 0; u < PF; ++u)
      if (s0 + u < s_hi) step(s0 + u, u, std::integral_constant<int, 0>());
  }

  if (SPLITK) {
    // raw partial sums: part[split][m][n] (SwiGLU: the up tile's outputs at N + n)
    float* part = a.part + (size_t)blockIdx.y * M * a.ldp;
#pragma unroll
    for (int g = 0; g < CG; ++g) {
      const int m = g * 16 + r;
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        if (m < M && tv[j]) {
          const int n0 = tile[j] * 16 + kg * 4 + ((EPI == EPI_SWIGLU && j == 1) ? N : 0);
          *(float4*)(part + (size_t)m * a.ldp + n0) = make_float4(acc[j][g][0], acc[j][g][1], acc[j][g][2], acc[j][g][3]);
        }
      }
    }
    return;
  }

  // ---- epilogue: lane (column r of group g = activation row g*16 + r, kg) holds outputs tile*16 + kg*4 + 0..3
  if (tid < BM) key_s[tid] = 0ull;
  __syncthreads();                       // rs_s (written before the main loop) and key_s are visible
#pragma unroll
  for (int g = 0; g < CG; ++g) {
    const int m = g * 16 + r;
    const bool mact = m < M;
    const float rs = (NORM && mact) ? rs_s[m] : 1.f;
    if (EPI == EPI_SWIGLU) {
      const int n0 = tile[0] * 16 + kg * 4;
      if (mact && tv[0]) {
        float u[4];
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
          const float gt = acc[0][g][jj] * rs, up = acc[1][g][jj] * rs;
          u[jj] = gt / (1.0f + __expf(-gt)) * up;
        }
        bf16_t hi[4], lo[4];
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) split_bf16(u[jj], hi[jj], lo[jj]);
        *(uint2*)(a.yb + (size_t)m * a.ldyb + n0) = make_uint2(hi[0] | ((uint32_t)hi[1] << 16), hi[2] | ((uint32_t)hi[3] << 16));
        *(uint2*)(a.yb_lo + (size_t)m * a.ldyb + n0) = make_uint2(lo[0] | ((uint32_t)lo[1] << 16), lo[2] | ((uint32_t)lo[3] << 16));
      }
    } else {
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int n0 = tile[j] * 16 + kg * 4;
        float hsq = 0.f;
        unsigned long long best = 0ull;
        if (mact && tv[j]) {
          float v[4];
#pragma unroll
          for (int jj = 0; jj < 4; ++jj) v[jj] = acc[j][g][jj] * rs;
          if (EPI == EPI_RESID) {
            float4 h4 = *(const float4*)(a.y + (size_t)m * a.ldy + n0);
            h4.x += v[0]; h4.y += v[1]; h4.z += v[2]; h4.w += v[3];
            *(float4*)(a.y + (size_t)m * a.ldy + n0) = h4;
            const float hn[4] = {h4.x, h4.y, h4.z, h4.w};
            bf16_t hi[4], lo[4];
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) {
              hsq += hn[jj] * hn[jj];
              split_bf16(hn[jj] * bf16_to_f32(a.g_next[n0 + jj]), hi[jj], lo[jj]);
            }
            *(uint2*)(a.yb + (size_t)m * a.ldyb + n0) = make_uint2(hi[0] | ((uint32_t)hi[1] << 16), hi[2] | ((uint32_t)hi[3] << 16));
            *(uint2*)(a.yb_lo + (size_t)m * a.ldyb + n0) = make_uint2(lo[0] | ((uint32_t)lo[1] << 16), lo[2] | ((uint32_t)lo[3] << 16));
          } else {
            if (n0 + 3 < N) {
              *(float4*)(a.y + (size_t)m * a.ldy + n0) = make_float4(v[0], v[1], v[2], v[3]);
            } else {
#pragma unroll
              for (int jj = 0; jj < 4; ++jj)
                if (n0 + jj < N) a.y[(size_t)m * a.ldy + n0 + jj] = v[jj];
            }
            if (EPI == EPI_LOGITS) {
#pragma unroll
              for (int jj = 0; jj < 4; ++jj)
                if (n0 + jj < N) { const unsigned long long k = argmax_key(v[jj], n0 + jj); if (k > best) best = k; }
            }
          }
        }
        if (EPI == EPI_RESID) {
          // sum of squares of the 16 outputs of this tile for activation row m: over the 4 kg lanes
          hsq += __shfl_xor(hsq, 16, 64);
          hsq += __shfl_xor(hsq, 32, 64);
          if (mact && tv[j] && kg == 0) a.ssp_next[(size_t)tile[j] * a.ssp_ld + m] = hsq;
        }
        if (EPI == EPI_LOGITS && best != 0ull) atomicMax(&key_s[m], best);
      }
    }
  }
  if (EPI == EPI_LOGITS) {
    __syncthreads();
    if (tid < M && key_s[tid] != 0ull) atomicMax(a.amax + (size_t)(blockIdx.x % AMAX_CELLS) * a.amax_ld + tid, key_s[tid]);
  }
}

// Second stage of a K-split launch: out = epilogue(sum over the splits, in order).  One thread per
// (activation row m, 4 consecutive outputs); a block covers 1024 outputs of one row.
template <int EPI, bool NORM>
__global__ void __launch_bounds__(256) gemm_finish_kernel(const float* part_, const float* res_, const bf16_t* g_next_, int ksplit_, int M_, int N_, int ldp_, int ldy_,
                                                         MfmaArgs a) {     // leading scalars: see gemm_mfma_kernel
  __shared__ float red_s[4];
  __shared__ float rs_sh;
  const int m = blockIdx.y, tid = threadIdx.x;
  const int n0 = (blockIdx.x * 256 + tid) * 4;
  const int N = N_, M = M_;
  const bool act = n0 < N;      // N is a multiple of 16 on this path
  const int nc = act ? n0 : 0;  // inactive threads load (and drop) the row's first outputs: no load sits under a per-lane condition
  // Every load of the kernel is issued here, before the first wait: the splits' partial sums (a split beyond ksplit
  // re-reads the last one and is left out of the sum), the residual row and the next norm's gain.
  constexpr int KSMAX = EPI == EPI_SWIGLU ? DMTD_GEMM_KSMAX_GU : DMTD_GEMM_KSMAX;     // splits fetched up front (gate/up has blocks enough with 3 splits at most at the usual shapes)
  float4 x[KSMAX], y[KSMAX];
#pragma unroll
  for (int ks = 0; ks < KSMAX; ++ks) {
    const float* p = part_ + ((size_t)(ks < ksplit_ ? ks : ksplit_ - 1) * M + m) * ldp_ + nc;
    x[ks] = *(const float4*)p;
    if (EPI == EPI_SWIGLU) y[ks] = *(const float4*)(p + N);
  }
  float4 h4 = make_float4(0.f, 0.f, 0.f, 0.f);
  uint2 graw = make_uint2(0u, 0u);
  if (EPI == EPI_RESID) {
    h4 = *(const float4*)(res_ + (size_t)m * ldy_ + nc);
    graw = *(const uint2*)(g_next_ + nc);
  }
  float rs = 1.f;
  if (NORM) {
    float s = 0.f;
    for (int p = tid; p < a.n_parts; p += 256) s += a.ssp[(size_t)p * a.ssp_ld + m];
    s = wave_sum(s);
    if ((tid & 63) == 0) red_s[tid >> 6] = s;
    __syncthreads();
    if (tid == 0) rs_sh = rsqrtf((red_s[0] + red_s[1] + red_s[2] + red_s[3]) / (float)a.K + a.eps);
    __syncthreads();
    rs = rs_sh;
  }
  float v[4] = {0.f, 0.f, 0.f, 0.f}, v2[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int ks = 0; ks < KSMAX; ++ks) {
    if (ks < ksplit_) {
      v[0] += x[ks].x; v[1] += x[ks].y; v[2] += x[ks].z; v[3] += x[ks].w;
      if (EPI == EPI_SWIGLU) { v2[0] += y[ks].x; v2[1] += y[ks].y; v2[2] += y[ks].z; v2[3] += y[ks].w; }
    }
  }
  for (int ks = KSMAX; ks < ksplit_; ++ks) {      // more splits than fetched up front (unusual shapes): one at a time
    const float* p = part_ + ((size_t)ks * M + m) * ldp_ + nc;
    const float4 xv = *(const float4*)p;
    v[0] += xv.x; v[1] += xv.y; v[2] += xv.z; v[3] += xv.w;
    if (EPI == EPI_SWIGLU) {
      const float4 yv = *(const float4*)(p + N);
      v2[0] += yv.x; v2[1] += yv.y; v2[2] += yv.z; v2[3] += yv.w;
    }
  }
  float hsq = 0.f;
  if (act) {
    float o[4];
    if (EPI == EPI_STORE) {
      *(float4*)(a.y + (size_t)m * a.ldy + n0) = make_float4(v[0] * rs, v[1] * rs, v[2] * rs, v[3] * rs);
    } else {
      if (EPI == EPI_SWIGLU) {
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) { const float gt = v[jj] * rs; o[jj] = gt / (1.0f + __expf(-gt)) * (v2[jj] * rs); }
      } else {
        h4.x += v[0]; h4.y += v[1]; h4.z += v[2]; h4.w += v[3];
        *(float4*)(a.y + (size_t)m * a.ldy + n0) = h4;
        const float hn[4] = {h4.x, h4.y, h4.z, h4.w};
        const float gn[4] = {__uint_as_float(graw.x << 16), __uint_as_float(graw.x & 0xFFFF0000u),
                             __uint_as_float(graw.y << 16), __uint_as_float(graw.y & 0xFFFF0000u)};
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) { hsq += hn[jj] * hn[jj]; o[jj] = hn[jj] * gn[jj]; }
      }
      bf16_t hi[4], lo[4];
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) split_bf16(o[jj], hi[jj], lo[jj]);
      *(uint2*)(a.yb + (size_t)m * a.ldyb + n0) = make_uint2(hi[0] | ((uint32_t)hi[1] << 16), hi[2] | ((uint32_t)hi[3] << 16));
      *(uint2*)(a.yb_lo + (size_t)m * a.ldyb + n0) = make_uint2(lo[0] | ((uint32_t)lo[1] << 16), lo[2] | ((uint32_t)lo[3] << 16));
    }
  }
  if (EPI == EPI_RESID) {
    // sum of squares per tile of 16 outputs: the 4 neighbouring threads of a tile
    hsq += __shfl_xor(hsq, 1, 64);
    hsq += __shfl_xor(hsq, 2, 64);
    if (act && (tid & 3) == 0) a.ssp_next[(size_t)(n0 >> 4) * a.ssp_ld + m] = hsq;
  }
}

}  // namespace dmtd
