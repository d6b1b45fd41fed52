// C ABI of the DMTD decode path (see include/dmtd.h): context, workspace layout, step
// assembly, hipGraph capture/replay and the host-visible calls.
//
// Two kernel paths share the step assembly:
//  - bf16 models ("packed" path): weights repacked once into MFMA operand order, all
//    projections through the MFMA weight-streaming kernel, activations handed from kernel
//    to kernel as packed bf16 rows plus partial sums of squares for the next RMSNorm;
//  - the fp32 parity model: FMA weight-streaming kernels with the norm computed in-kernel.
#include "../../include/dmtd.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <cstdio>
#include <cstring>
#include <map>
#include <string>
#include <tuple>
#include <type_traits>
#include <vector>

#include "kernels.hpp"
#include "sched.hpp"

using namespace dmtd;

namespace {

constexpr int kMaxTau = 64;          // steps per decode call (size of the emitted-token buffer)
constexpr int kGemvRows = 4;         // activation rows per FMA weight-streaming pass
constexpr int kMaxRows = 16;         // rows per sequence one pass through the layers may carry
constexpr int kPassRows = 128;       // activation rows (all sequences together) a prefill or whole-sequence pass carries: one weight pass of the tiled kernel
// Row capacity of the activation buffers, and positions per sequence of a prefill pass: passes of kPassRows rows in all,
// at least kMaxRows per sequence (large batches: more passes of the tiled kernel per weight stream are not needed, B * 16 >= 128)
inline int row_capacity(int max_batch) { return max_batch * kMaxRows > kPassRows ? max_batch * kMaxRows : kPassRows; }
inline int pass_positions(int batch) { const int r = kPassRows / batch; return r > kMaxRows ? r : kMaxRows; }
constexpr int kMaxPatterns = 64;     // distinct step patterns (which sequences start a cycle, with how many rows) a context keeps on the device
constexpr size_t kPatternStride(size_t max_batch) { return (max_batch * 5 + 255) / 256 * 256; }   // int list [max_batch] + byte mask [max_batch]
constexpr int kMfmaRows = 16;        // activation rows per pass of the one-tile-per-block MFMA kernel
#ifndef DMTD_GEMM_MAXSPLIT
#define DMTD_GEMM_MAXSPLIT 12
#endif
constexpr int kGemmMaxSplit = DMTD_GEMM_MAXSPLIT;   // K splits of the tiled kernel at most (sizes the partial-sum buffer)
#ifndef DMTD_FIT_SMALL_KB
#define DMTD_FIT_SMALL_KB 60
#endif
#ifndef DMTD_GEMM_ROWS
#define DMTD_GEMM_ROWS 128
#endif
constexpr int kGemmRows = DMTD_GEMM_ROWS;   // activation rows per pass of the LDS-tiled MFMA kernel (launches with more than 16 rows)
constexpr int kMfmaPF = 10;          // k-steps (64 elements) a wave of the MFMA kernel holds in registers
// Waves that split K for one matrix (NW) and k-steps a wave keeps in flight as a rolling window (PF), per projection;
// NW = 0: the one-round rule of launch_mfma with kMfmaPF.  Defaults from sweeps at 4B shapes on MI355X, us per launch
// with 3 rows / 1 row: gate/up 4 x 2: 18.9 / 18.1 (4 x 4: 19.5 / 19.1), down 16 x 3: 11.3 / 10.7 (16 x 5: 11.3 / 10.9),
// O 8 x 4: 6.3 / 6.2 (16 x 5: 8.0 / 7.3), QKV 8 x 2: 7.6 / 7.5 (one round of 5: 8.0 / 7.7); the LM head measures
// 131 us whatever the shape (it runs at the memory system's rate).  Short windows win since every load of the
// prologue is issued without a wait in between: the first k-step's matrix-core work starts as soon as it lands.
// The macros exist so a sweep can override them at build time.
#ifndef DMTD_GU_NW
#define DMTD_GU_NW 4
#define DMTD_GU_PF 2
#endif
#ifndef DMTD_DN_NW
#define DMTD_DN_NW 16
#define DMTD_DN_PF 3
#endif
#ifndef DMTD_O_NW
#define DMTD_O_NW 8
#define DMTD_O_PF 4
#endif
#ifndef DMTD_LM_NW
#define DMTD_LM_NW 5
#define DMTD_LM_PF 4
#endif
#ifndef DMTD_Q_NW
#define DMTD_Q_NW 8
#define DMTD_Q_PF 2
#endif
constexpr int kMfmaPFQkv = 5;        // the same for the QKV projection: shorter runs put 8 waves on a tile (measured 8.3 us instead of 9.3 us at 4B shapes)

thread_local std::string g_create_error;

// The library's own scratch for dmtd_decode_cycle_noalloc (callers that cannot allocate and hand over no workspace for
// partial results).  One copy per GPU the library runs on, held until the process ends; every context on a GPU shares
// it, so two such calls that overlap on one GPU race.  The name below is a host-side stand-in: the device address is
// taken once per device with hipGetSymbolAddress (dmtd_create) and only that address is ever handed to kernels.
constexpr size_t kStaticScratchBytes = (size_t)16 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
char* g_scratch_ptr[kMaxDevices] = {};

hipError_t static_scratch_for_current_device(char** out) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    g_scratch_ptr[dev] = (char*)p;
  }
  *out = g_scratch_ptr[dev];
  return hipSuccess;
}

struct LayerW {   // tensors of one layer inside the caller's blob
  const void *attn_norm, *q, *k, *v, *q_norm, *k_norm, *o, *mlp_norm, *gate, *up, *down;
};
struct LayerSw {  // the layer's matrices in MFMA operand order (workspace; bf16 models only)
  const bf16_t *qkv, *o, *gate, *up, *down;
};

struct Ws {   // device workspace carve-up (byte offsets)
  size_t kv, kv_layer_stride, kv_v_off;
  size_t h, h_late, qkv, attn, mlp, logits, part_o, part_ml, amax;
  size_t tokens, emitted, forced, state, inv_freq, rope_tab;
  size_t xb, xb_late, ssp, ssp_late, wsw;      // packed path only
  size_t gemm_part;                            // K-split partial sums of the tiled kernel
  size_t patterns;
  size_t pend_enc, enc_tmp;                    // ExDy: stored encoding outputs of pending tokens; of a prefill chunk
  size_t mask, logits_rows, amax_rows, nll, best, loss;   // whole-sequence masked forward: mask, a chunk's logits and keys, per-position results
  size_t total;
};

// Activation rows in flight between kernels.  On the packed path xb holds bf16(h * gain of
// the norm that reads the rows next) and ssp the partial sums of h^2 (n_parts of them per row).
struct Rows {
  float* h;
  bf16_t* xb;      // high parts
  bf16_t* xb_lo;   // low parts
  float* ssp;
  int n_parts;
};

}  // namespace

struct dmtd_ctx {
  dmtd_config cfg;
  Sched sched;
  std::string err;
  hipStream_t stream = nullptr;
  int elem = 2;
  bool packed = false;        // bf16 model: MFMA path
  int num_cus = 256;
  int batch = 0;              // batch of the current sequence set (after prefill)
  int ssp_ld = 0;             // row capacity of the sum-of-squares buffers
  const char* wbase = nullptr;
  char* ws = nullptr;
  Ws o{};
  const void* embed = nullptr;
  const void* final_norm = nullptr;
  const void* lm_head = nullptr;
  const bf16_t* lm_head_sw = nullptr;
  std::vector<LayerW> layers;
  std::vector<LayerSw> sw;
  std::map<std::tuple<int, int, int, int, int>, hipGraphExec_t> graphs;   // (full, rows, n_late / n_early / sampling, bucket / share_kv, batch)
  std::map<std::vector<int>, hipGraphExec_t> group_graphs;            // several steps in one graph (dmtd_decode)
  bool sampling = false;      // tokens are drawn (dmtd_set_sampling) instead of taken greedily
  bool share_kv = false;      // attention launches: one pass over K/V for all rows of a sequence (long contexts)
  int att_bucket = 512;       // attention launches: context bucket (multiple of 512) the key ranges are laid out for
  const int* fmap = nullptr;  // launches of a front pass over SOME sequences: launch sequence -> sequence slot (device); null = all, in order
  const unsigned char* full_mask = nullptr;   // the step's bookkeeping: which sequences close their refill gap (device); null = all or none
  // sequences at different points of their cycles (dmtd_decode_per_seq): per-sequence phase and front position (in the
  // counters' coordinates); while `diverged` the single-phase calls are refused
  std::vector<int> seq_phase, seq_front;
  bool diverged = false;
  std::map<std::vector<int>, int> pattern_ids;      // rows per sequence of a step (0 = late-only) -> slot in the device pattern table
  std::map<std::vector<int>, hipGraphExec_t> mixed_graphs;
  bool fold_qkv = false;      // run_layer: a K-split QKV launch may leave its finishing step to the attention launch that follows
  QkvSrc qkv_pending{};       // ... and says so here (part != nullptr) until that launch picks it up
  // Scratch of the step kernels (partial results that live for one launch pair): the attention ranges' partial outputs
  // and softmax statistics, the LM head's selection-key cells, the K-split partial sums of the tiled kernel.  They sit
  // in the caller's workspace, except inside dmtd_decode_cycle_noalloc, which points them at the library's own array.
  float* part_o = nullptr;
  float* part_ml = nullptr;
  unsigned long long* amax = nullptr;
  float* gemm_part = nullptr;
  int part_rows = 0;          // rows per sequence the partials are laid out for (stride between ranges: part_rows * query heads per KV head)
  int test_fail_step = -1;    // tests of the failure path: the next decode call reports a launch failure before this step (once)
  char* static_scratch = nullptr;   // this device's copy of the library's own scratch array (address taken at create)
  std::vector<Step> plan_buf;       // dmtd_decode_cycle_noalloc: the call's steps (capacity reserved at create)
};

namespace {

size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

bool valid_config(const dmtd_config* c, std::string& why) {
  if (!c) { why = "null config"; return false; }
  if (c->n_layers < 1 || c->hidden < 8 || c->n_q_heads < 1 || c->n_kv_heads < 1 || c->intermediate < 8 || c->vocab < 2) {
    why = "non-positive model dimension"; return false;
  }
  if (c->hidden % 8 || c->intermediate % 8) { why = "hidden and intermediate must be multiples of 8"; return false; }
  if (c->head_dim != 64 && c->head_dim != 128) { why = "head_dim must be 64 or 128"; return false; }
  if (c->n_q_heads % c->n_kv_heads) { why = "n_q_heads must be a multiple of n_kv_heads"; return false; }
  if (c->n_q_heads / c->n_kv_heads > QV_MAX) { why = "too many query heads per KV head"; return false; }
  if (c->dtype != DMTD_DTYPE_F32 && c->dtype != DMTD_DTYPE_BF16) { why = "unknown dtype"; return false; }
  if (c->dtype == DMTD_DTYPE_BF16 && (c->hidden % 64 || c->intermediate % 64)) {
    why = "bf16 models need hidden and intermediate to be multiples of 64"; return false;
  }
  if (c->max_batch < 1 || c->max_seq_len < 2) { why = "max_batch >= 1 and max_seq_len >= 2 required"; return false; }
  if (!(c->rms_eps > 0.f) || !(c->rope_theta > 0.f)) { why = "rms_eps and rope_theta must be positive"; return false; }
  return true;
}

size_t weight_elems(const dmtd_config& c) {
  const size_t d = c.hidden, qd = (size_t)c.n_q_heads * c.head_dim, kd = (size_t)c.n_kv_heads * c.head_dim, ff = c.intermediate;
  const size_t per_layer = d + qd * d + 2 * kd * d + 2 * (size_t)c.head_dim + d * qd + d + 3 * ff * d;
  return (size_t)c.vocab * d + c.n_layers * per_layer + d + (c.tied_embeddings ? 0 : (size_t)c.vocab * d);
}

size_t swizzled_layer_elems(const dmtd_config& c) {
  const size_t d = c.hidden, qd = (size_t)c.n_q_heads * c.head_dim, ff = c.intermediate;
  const size_t nqkv = (size_t)(c.n_q_heads + 2 * c.n_kv_heads) * c.head_dim;
  return swizzled_elems(nqkv, d) + swizzled_elems(d, qd) + 2 * swizzled_elems(ff, d) + swizzled_elems(d, ff);
}

Ws layout(const dmtd_config& c) {
  Ws w{};
  const size_t e = c.dtype == DMTD_DTYPE_F32 ? 4 : 2;
  const size_t B = c.max_batch, S = c.max_seq_len, d = c.hidden, hd = c.head_dim;
  const size_t nqkv = (size_t)(c.n_q_heads + 2 * c.n_kv_heads) * hd, qd = (size_t)c.n_q_heads * hd;
  const size_t rows = row_capacity(c.max_batch);
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
  const size_t kv_one = B * c.n_kv_heads * S * hd * e;       // K (or V) of one layer
  w.kv_v_off = align_up(kv_one, 256);
  w.kv_layer_stride = 2 * w.kv_v_off;
  w.kv = take(w.kv_layer_stride * c.n_layers);
  w.h = take(rows * d * 4);
  w.h_late = take(B * d * 4);
  w.qkv = take(rows * nqkv * 4);
  w.attn = take(rows * qd * 4);                       // fp32 path: fp32 rows; packed path: bf16 rows
  w.mlp = take(rows * (size_t)c.intermediate * 4);    // likewise
  w.logits = take(B * (size_t)c.vocab * 4);
  // partial results of the attention key ranges: laid out per sequence for kMaxRows rows in decode steps and for a pass's
  // positions in prefill; sequences x rows per sequence never exceeds the row capacity
  const size_t qv_rows = rows * (c.n_q_heads / c.n_kv_heads);
  w.part_o = take(c.n_kv_heads * ATT_MAX_SPLITS * qv_rows * hd * 4);
  w.part_ml = take(c.n_kv_heads * ATT_MAX_SPLITS * qv_rows * 2 * 4);
  w.amax = take((size_t)AMAX_CELLS * B * 8);
  w.tokens = take(B * S * 4);
  w.emitted = take((size_t)kMaxTau * B * 4);
  w.forced = take((size_t)kMaxTau * B * 4);
  w.state = take(kStateDeltaOff + 12 * B);            // counters, sampling parameters, per-sequence (delta, front position) pairs, last prompt positions
  w.patterns = take((size_t)kMaxPatterns * kPatternStride(B));   // sequence lists and masks of steps whose sequences are at different points of their cycles
  w.inv_freq = take((hd / 2) * 8);
  w.pend_enc = take(B * kMaxTau * d * 4);
  w.enc_tmp = take(rows * d * 4);
  w.rope_tab = take(S * (hd / 2) * 8);                 // (cos, sin) per position and frequency
  w.mask = take(S * 4);
  w.logits_rows = take(rows * (size_t)c.vocab * 4);
  w.amax_rows = take((size_t)AMAX_CELLS * rows * 8);
  w.nll = take(B * S * 4);
  w.best = take(B * S * 4);
  w.loss = take(B * 4);
  if (c.dtype == DMTD_DTYPE_BF16) {
    const size_t parts = (d + 15) / 16;
    w.xb = take(rows * d * 2 * 2);                     // high and low planes
    w.xb_late = take(B * d * 2 * 2);
    w.ssp = take(parts * rows * 4);
    w.ssp_late = take(parts * rows * 4);
    {
      size_t widest = 2 * (size_t)c.intermediate > nqkv ? 2 * (size_t)c.intermediate : nqkv;
      if (d > widest) widest = d;
      w.gemm_part = take((size_t)kGemmMaxSplit * kGemmRows * widest * 4);
    }
    w.wsw = take((swizzled_layer_elems(c) * c.n_layers + swizzled_elems(c.vocab, d)) * 2);
  }
  w.total = off;
  return w;
}

#define HIP_TRY(ctx, expr)                                                              \
  do {                                                                                  \
    hipError_t e_ = (expr);                                                             \
    if (e_ != hipSuccess) {                                                             \
      (ctx)->err = std::string(#expr) + ": " + hipGetErrorString(e_);                   \
      return DMTD_EHIP;                                                                 \
    }                                                                                   \
  } while (0)

DevState* dev_state(dmtd_ctx* c) { return (DevState*)(c->ws + c->o.state); }
int* dev_tokens(dmtd_ctx* c) { return (int*)(c->ws + c->o.tokens); }
const void* norm_gain_for_layer(const dmtd_ctx* c, int l) {   // gain of the norm that opens layer l (the final norm after the last)
  return l < c->cfg.n_layers ? c->layers[l].attn_norm : c->final_norm;
}

// ------------------------------------------------------- fp32 path: FMA weight streaming

template <typename WT, int M, int EPI, bool NORM>
hipError_t launch_gemv(dmtd_ctx* c, GemvArgs a) {
  // narrow outputs with long rows: the waves of a block split K
  if constexpr ((EPI == EPI_RESID || EPI == EPI_STORE) && !NORM) {
    if (a.K >= 1024 && a.N <= 8192) {
      if (a.K <= 4 * 2 * 512) {
        hipLaunchKernelGGL((gemv_ksplit_kernel<WT, M, EPI, 2, 4, 1>), dim3((a.N + 3) / 4), dim3(256), 0, c->stream, a);
        return hipGetLastError();
      }
      if (a.K <= 4 * 5 * 512) {
        hipLaunchKernelGGL((gemv_ksplit_kernel<WT, M, EPI, 5, 4, 1>), dim3((a.N + 3) / 4), dim3(256), 0, c->stream, a);
        return hipGetLastError();
      }
    }
  }
  const size_t lds = (size_t)M * a.K * 4;
  auto kern = gemv_rows_kernel<WT, M, EPI, NORM, 5>;
  static int occ_cache = -1;
  static size_t occ_lds = 0;
  if (lds > 160 * 1024 - 4096) return hipErrorInvalidValue;
  if (occ_cache < 0 || occ_lds != lds) {
    if (lds > 48 * 1024) {
      hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024 - 4096);
      if (e != hipSuccess) return e;
    }
    int occ = 0;
    hipError_t e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ, kern, 256, lds);
    if (e != hipSuccess) return e;
    occ_cache = occ < 1 ? 1 : occ;
    occ_lds = lds;
  }
  constexpr int RPW = (EPI == EPI_SWIGLU) ? 2 : 4;
  const int tasks = (a.N + RPW - 1) / RPW;
  int blocks = (tasks + 3) / 4;                      // one task per wave ...
  const int cap = c->num_cus * occ_cache;            // ... unless that exceeds what is resident at once
  if (blocks > cap) blocks = cap;
  hipLaunchKernelGGL(kern, dim3(blocks), dim3(256), lds, c->stream, a);
  return hipGetLastError();
}

template <typename WT, int EPI, bool NORM>
hipError_t gemv_rows(dmtd_ctx* c, GemvArgs a, int rows) {
  // rows are processed in groups of up to kGemvRows; each group streams the matrix once
  for (int m0 = 0; m0 < rows; m0 += kGemvRows) {
    const int m = rows - m0 < kGemvRows ? rows - m0 : kGemvRows;
    GemvArgs g = a;
    g.x = a.x + (size_t)m0 * a.ldx;
    g.y = a.y + (size_t)m0 * a.ldy;
    if (a.amax) g.amax = a.amax + m0;
    hipError_t e;
    switch (m) {
      case 1: e = launch_gemv<WT, 1, EPI, NORM>(c, g); break;
      case 2: e = launch_gemv<WT, 2, EPI, NORM>(c, g); break;
      case 3: e = launch_gemv<WT, 3, EPI, NORM>(c, g); break;
      default: e = launch_gemv<WT, 4, EPI, NORM>(c, g); break;
    }
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

// ---------------------------------------------------- packed path: MFMA weight streaming

// nw waves split K for each matrix: the smallest of {2, 4, 8} (SwiGLU: {2, 4, 5}) that lets a wave
// hold its k-range in one round of PF k-steps, else the largest with several rounds.
// More than 16 rows go through the LDS-tiled kernel, up to kGemmRows per pass (each pass streams the matrix once).
// Attention launch shape for r rows per sequence: true = one key range per (row group, KV head, sequence), whose triples
// then fill the chip by themselves (see launch_attention_mfma_t).
bool attention_single_range(const dmtd_ctx* c, int r) {
  const dmtd_config& cf = c->cfg;
  const int gq = cf.n_q_heads / cf.n_kv_heads, rpb = 16 / gq, n_rg = (r + rpb - 1) / rpb;
  return (long)cf.n_kv_heads * c->batch * n_rg >= c->num_cus;
}

// Whether `rows` packed activation rows of width K (both planes, plus n_parts partial sums of squares per row) stay in
// LDS for the one-tile-per-block kernel of an [N, K] projection (otherwise the LDS-tiled kernel takes them).
bool mfma_rows_fit(const dmtd_ctx* c, int rows, int N, int K, int n_parts) {
  if (rows > kMfmaRows) return false;
  const size_t lds_rows = (size_t)rows * ((size_t)4 * K + (size_t)n_parts * 4);
  return lds_rows <= ((N + 15) / 16 <= c->num_cus ? (size_t)120 * 1024 : (size_t)DMTD_FIT_SMALL_KB * 1024);
}

template <int EPI, bool NORM, int PF = kMfmaPF, int ROLL_NW = 0>
hipError_t launch_mfma(dmtd_ctx* c, MfmaArgs a, int rows) {
  const int KS = a.K / 64;
  constexpr int MATS = EPI == EPI_SWIGLU ? 2 : 1;
  const int nw_max = EPI == EPI_SWIGLU ? 5 : 8;
  int nw = 2;
  while (nw < nw_max && (KS + nw - 1) / nw > PF) nw = (EPI == EPI_SWIGLU && nw == 4) ? 5 : nw * 2;
  // ROLL_NW: a fixed number of waves per matrix, each keeping a rolling window of PF k-steps in flight
  if (ROLL_NW > 0) nw = ROLL_NW;
  const dim3 grid((a.N + 15) / 16);
  // The one-tile-per-block kernel keeps all rows (both planes) in LDS: comfortably (two blocks per CU) in general,
  // up to most of a CU's LDS when the launch has no more blocks than the chip has CUs anyway.  Rows that do not
  // fit, and more than 16 rows (batched steps), go through the LDS-tiled kernel in passes of up to kGemmRows rows.
  const bool fits = a.ldxb == a.K && mfma_rows_fit(c, rows, a.N, a.K, NORM ? a.n_parts : 0);
  // one launch of the tiled kernel; with 64 and more rows its ring of activation slices is dynamic LDS beyond the default limit
#define DMTD_LAUNCH_GEMM(CG_, SPLIT_, GRID_)                                                                                   \
  do {                                                                                                                         \
    auto kern = gemm_mfma_kernel<EPI, NORM, CG_, SPLIT_>;                                                                      \
    constexpr size_t dyn = gemm_dyn_lds(CG_);                                                                                  \
    static bool big_lds = false;                                                                                               \
    if (dyn > 0 && !big_lds) {                                                                                                 \
      hipError_t ae = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)dyn);            \
      if (ae != hipSuccess) return ae;                                                                                         \
      big_lds = true;                                                                                                          \
    }                                                                                                                          \
    hipLaunchKernelGGL(kern, GRID_, dim3(64 * gemm_waves(CG_, EPI)), dyn, c->stream, g.W, g.W2, g.xb, g.xb_lo, g.M, g.N, g.K, \
                       g.ldxb, g.ksplit, g);                                                                                   \
  } while (0)
  if (!fits) {
    const int n_tiles = (a.N + 15) / 16;
    for (int m0 = 0; m0 < rows; m0 += kGemmRows) {
      MfmaArgs g = a;
      g.M = rows - m0 < kGemmRows ? rows - m0 : kGemmRows;
      g.xb = a.xb + (size_t)m0 * a.ldxb;
      g.xb_lo = a.xb_lo + (size_t)m0 * a.ldxb;
      if (a.ssp) g.ssp = a.ssp + m0;
      if (a.y) g.y = a.y + (size_t)m0 * a.ldy;
      if (a.yb) { g.yb = a.yb + (size_t)m0 * a.ldyb; g.yb_lo = a.yb_lo + (size_t)m0 * a.ldyb; }
      if (a.ssp_next) g.ssp_next = a.ssp_next + m0;
      if (a.amax) g.amax = a.amax + m0;
      const int cg = g.M <= 16 ? 1 : (g.M <= 32 ? 2 : (g.M <= 64 ? 4 : 8));
      const int gw = gemm_waves(cg, EPI);                  // a wave owns 2 tiles (SwiGLU: the gate and up tile of one)
      const dim3 ggrid(EPI == EPI_SWIGLU ? (n_tiles + gw - 1) / gw : (n_tiles + 2 * gw - 1) / (2 * gw));
      // K is split so that the launch has about one block per CU and no more (a partly filled second wave of blocks costs more than
      // it brings; measured at 4B shapes, 128 rows: QKV 288 blocks 32.4 us, 240 blocks 24.4 us; gate/up 152 blocks 50.0 us,
      // 228 blocks 42.4 us, 304 blocks 57.3 us; down 160 / 240 / 320 blocks 31.6 / 27.0 / 38.1 us); the LM head has
      // blocks enough without splitting
      const int KS = a.K / 64;
      int ksplit = 1;
      if constexpr (EPI != EPI_LOGITS) {
        ksplit = c->num_cus / (int)ggrid.x;
        if (ksplit < 1) ksplit = 1;
        if (EPI == EPI_STORE && ksplit > ATT_KSMAX) ksplit = ATT_KSMAX;      // what the attention launch can sum in its prologue
        if (EPI == EPI_RESID && ksplit > KS / 8) ksplit = KS / 8 > 0 ? KS / 8 : 1;
        if (ksplit > kGemmMaxSplit) ksplit = kGemmMaxSplit;
        if (ksplit > KS / 3) ksplit = KS / 3 > 0 ? KS / 3 : 1;
        // gate/up with up to 16 rows: its 1216 tile streams do without a split, and without the finishing launch (4B shapes,
        // 8 rows: 20.3 against 24.2 us); with 32 and more rows the 8-wave blocks are too few unsplit (36 against 24 us)
        if (EPI == EPI_SWIGLU && cg == 1) ksplit = 1;
      }
      if (ksplit > 1) {
        if constexpr (EPI != EPI_LOGITS) {
          g.ksplit = ksplit;
          g.ldp = (EPI == EPI_SWIGLU ? 2 : 1) * a.N;
          g.part = c->gemm_part;
          const dim3 sgrid(ggrid.x, ksplit);
          if (cg == 1) DMTD_LAUNCH_GEMM(1, true, sgrid);
          else if (cg == 2) DMTD_LAUNCH_GEMM(2, true, sgrid);
          else if (cg == 4) DMTD_LAUNCH_GEMM(4, true, sgrid);
          else DMTD_LAUNCH_GEMM(8, true, sgrid);
          if (EPI == EPI_STORE && NORM && c->fold_qkv && rows <= kGemmRows && ksplit <= ATT_KSMAX && c->batch > 0 &&
              attention_single_range(c, rows / c->batch)) {
            // the attention launch that follows sums the splits and applies the norm scale while it prepares its rows; only in
            // its one-range shape, where a vector is prepared once (with key ranges every range's block would repeat the sums:
            // C5 measured 2 % slower, C4 2 % faster)
            c->qkv_pending = QkvSrc{nullptr, 0, g.part, ksplit, g.M, g.ldp, g.ssp, g.n_parts, g.ssp_ld, 1.0f / (float)g.K, g.eps};
          } else {
            hipLaunchKernelGGL((gemm_finish_kernel<EPI, NORM>), dim3((a.N / 4 + 255) / 256, g.M), dim3(256), 0, c->stream,
                               (const float*)g.part, (const float*)g.y, (const bf16_t*)g.g_next, g.ksplit, g.M, g.N, g.ldp, g.ldy, g);
          }
        }
      } else {
        if (cg == 1) DMTD_LAUNCH_GEMM(1, false, ggrid);
        else if (cg == 2) DMTD_LAUNCH_GEMM(2, false, ggrid);
        else if (cg == 4) DMTD_LAUNCH_GEMM(4, false, ggrid);
        else DMTD_LAUNCH_GEMM(8, false, ggrid);
      }
    }
    return hipGetLastError();
  }
  for (int m0 = 0; m0 < rows; m0 += kMfmaRows) {
    MfmaArgs g = a;
    g.M = rows - m0 < kMfmaRows ? rows - m0 : kMfmaRows;
    g.xb = a.xb + (size_t)m0 * a.ldxb;
    g.xb_lo = a.xb_lo + (size_t)m0 * a.ldxb;
    if (a.ssp) g.ssp = a.ssp + m0;
    if (a.y) g.y = a.y + (size_t)m0 * a.ldy;
    if (a.yb) { g.yb = a.yb + (size_t)m0 * a.ldyb; g.yb_lo = a.yb_lo + (size_t)m0 * a.ldyb; }
    if (a.ssp_next) g.ssp_next = a.ssp_next + m0;
    if (a.amax) g.amax = a.amax + m0;
    const size_t lds = (size_t)2 * g.M * a.K * 2 + (NORM ? (size_t)g.M * a.n_parts * 4 : 0);   // the rows, both planes; partial sums of squares
#define DMTD_LAUNCH_MFMA(NWT_)                                                                                            \
    do {                                                                                                                  \
      auto kern = gemv_mfma_kernel<EPI, NORM, PF, NWT_, (ROLL_NW > 0)>;                                             \
      static bool big_lds = false;                                                                                        \
      if (lds > 48 * 1024 && !big_lds) {                                                                                  \
        hipError_t ae = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 120 * 1024);   \
        if (ae != hipSuccess) return ae;                                                                                  \
        big_lds = true;                                                                                                   \
      }                                                                                                                   \
      hipLaunchKernelGGL(kern, grid, dim3(64 * NWT_), lds, c->stream, g.W, g.W2, g.xb, g.xb_lo, (const float*)g.ssp, g.M, g.N, g.K, g.n_parts, g.ssp_ld, g); \
    } while (0)
    if constexpr (ROLL_NW > 0) DMTD_LAUNCH_MFMA(ROLL_NW * MATS);
    else if (nw == 2) DMTD_LAUNCH_MFMA(2 * MATS);
    else if (nw == 4) DMTD_LAUNCH_MFMA(4 * MATS);
    else if (nw == 5) {
      if constexpr (EPI == EPI_SWIGLU) DMTD_LAUNCH_MFMA(10);
    } else {
      if constexpr (EPI != EPI_SWIGLU) DMTD_LAUNCH_MFMA(8);
    }
#undef DMTD_LAUNCH_MFMA
  }
  return hipGetLastError();
}

hipError_t launch_lmhead(dmtd_ctx* c, MfmaArgs a, int rows) {
  if constexpr (DMTD_LM_NW > 0) return launch_mfma<EPI_LOGITS, true, DMTD_LM_PF, DMTD_LM_NW>(c, a, rows);
  else return launch_mfma<EPI_LOGITS, true>(c, a, rows);
}
hipError_t launch_qkv(dmtd_ctx* c, MfmaArgs a, int rows) {
  if constexpr (DMTD_Q_NW > 0) return launch_mfma<EPI_STORE, true, DMTD_Q_PF, DMTD_Q_NW>(c, a, rows);
  else return launch_mfma<EPI_STORE, true, kMfmaPFQkv>(c, a, rows);
}
hipError_t launch_down(dmtd_ctx* c, MfmaArgs a, int rows) {
  if constexpr (DMTD_DN_NW > 0) return launch_mfma<EPI_RESID, false, DMTD_DN_PF, DMTD_DN_NW>(c, a, rows);
  else return launch_mfma<EPI_RESID, false>(c, a, rows);
}
hipError_t launch_oproj(dmtd_ctx* c, MfmaArgs a, int rows) {
  if constexpr (DMTD_O_NW > 0) return launch_mfma<EPI_RESID, false, DMTD_O_PF, DMTD_O_NW>(c, a, rows);
  else return launch_mfma<EPI_RESID, false>(c, a, rows);
}
hipError_t launch_gateup(dmtd_ctx* c, MfmaArgs a, int rows) {
  if constexpr (DMTD_GU_NW > 0) return launch_mfma<EPI_SWIGLU, true, DMTD_GU_PF, DMTD_GU_NW>(c, a, rows);
  else return launch_mfma<EPI_SWIGLU, true>(c, a, rows);
}

// ------------------------------------------------------------------------- attention

// a3 + a4: QK-RMSNorm, RoPE, KV append and split-K attention in one launch over static key ranges, then the merge.
// The ranges follow from the context bucket (c->att_bucket, a multiple of 512 that covers the context), so a
// captured step stays valid until the sequence grows into the next bucket.
template <typename CT, typename OT, int HD, int QVT>
void launch_attention_t(dmtd_ctx* c, int l, const float* qkv, OT* attn, OT* attn_lo, int sel, int offset, int r, int append) {
  const dmtd_config& cf = c->cfg;
  const int B = c->batch, nqkv = (cf.n_q_heads + 2 * cf.n_kv_heads) * HD, qd = cf.n_q_heads * HD;
  const int gq = cf.n_q_heads / cf.n_kv_heads, rpb = QVT / gq, n_rg = (r + rpb - 1) / rpb;
  constexpr int KPI = AttKeysPerIter<HD>::value;
  CT* kc = (CT*)(c->ws + c->o.kv + (size_t)l * c->o.kv_layer_stride);
  CT* vc = (CT*)(c->ws + c->o.kv + (size_t)l * c->o.kv_layer_stride + c->o.kv_v_off);
  const LayerW& w = c->layers[l];
  // keys per range: one block iteration while that keeps the ranges within the partials buffer and puts no
  // more than about four blocks on every CU; longer ranges (several iterations) for long contexts or big batches
  const int bucket = c->att_bucket;
  long per_split_blocks = (long)cf.n_kv_heads * B * n_rg;
  int want_splits = (int)((4L * c->num_cus + per_split_blocks - 1) / per_split_blocks);
  if (want_splits > ATT_MAX_SPLITS) want_splits = ATT_MAX_SPLITS;
  if (want_splits < 1) want_splits = 1;
  int kps = ((bucket + want_splits - 1) / want_splits + KPI - 1) / KPI * KPI;
  const int ns = (bucket + kps - 1) / kps;
  float* po = c->part_o;
  float* pml = c->part_ml;
  const DevState* st = dev_state(c);
  hipLaunchKernelGGL((attn_split_kernel<CT, HD, QVT>), dim3(ns * n_rg, cf.n_kv_heads, B), dim3(256), 0, c->stream, qkv, nqkv,
                     w.q_norm, w.k_norm, (const float2*)(c->ws + c->o.rope_tab), kc, vc, po, pml, cf.n_q_heads, cf.n_kv_heads,
                     cf.max_seq_len, cf.rms_eps, kps, ns, c->part_rows * gq, st, sel, offset, r, append, c->fmap);
  hipLaunchKernelGGL((attn_merge_kernel<HD, OT>), dim3(r, cf.n_q_heads, B), dim3(256), 0, c->stream, po, pml, attn, attn_lo, qd,
                     cf.n_q_heads, cf.n_kv_heads, kps, ns, c->part_rows * gq, st, sel, offset, r, c->fmap);
}

// The matrix-core kernel (bf16 caches): one pass over K and V serves up to 16 query vectors per KV head.
// Two launch shapes.  (1) ONE key range per (row group, KV head, sequence), 8 waves per block, the output written
// by the kernel itself (no partials, no merge launch): for batches whose (KV head, sequence) pairs fill the chip
// without splitting.  (2) Key ranges over 4-wave blocks plus the merge: everything else (a single block per KV head
// would be bound by its matrix-core work: about 1300 cycles per 16 keys and wave).
template <typename OT, int HD>
hipError_t launch_attention_mfma_t(dmtd_ctx* c, int l, const float* qkv, OT* attn, OT* attn_lo, int sel, int offset, int r, int append) {
  const dmtd_config& cf = c->cfg;
  const int B = c->batch, nqkv = (cf.n_q_heads + 2 * cf.n_kv_heads) * HD, qd = cf.n_q_heads * HD;
  const int gq = cf.n_q_heads / cf.n_kv_heads, rpb = 16 / gq, n_rg = (r + rpb - 1) / rpb;
  const int qv_max = (r < rpb ? r : rpb) * gq;             // query vectors of the fullest block
  bf16_t* kc = (bf16_t*)(c->ws + c->o.kv + (size_t)l * c->o.kv_layer_stride);
  bf16_t* vc = (bf16_t*)(c->ws + c->o.kv + (size_t)l * c->o.kv_layer_stride + c->o.kv_v_off);
  const LayerW& w = c->layers[l];
  const int bucket = c->att_bucket;
  long per_split_blocks = (long)cf.n_kv_heads * B * n_rg;
  float* po = c->part_o;
  float* pml = c->part_ml;
  const DevState* st = dev_state(c);
  QkvSrc qs = c->qkv_pending;           // the QKV projection's unfinished partial sums, if it left them to this launch
  c->qkv_pending = QkvSrc{};
  qs.qkv = qkv; qs.ldq = nqkv;
  if (attention_single_range(c, r)) {
    constexpr int NW = 8;
    const int kps = (bucket + 16 * NW - 1) / (16 * NW) * (16 * NW);
    const size_t lds = (size_t)NW * qv_max * HD * 4;
    auto kern = attn_split_mfma_kernel<HD, NW, true>;
    static bool big_lds = false;
    if (lds > 32 * 1024 && !big_lds) {
      hipError_t ae = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, NW * 16 * HD * 4);
      if (ae != hipSuccess) return ae;
      big_lds = true;
    }
    hipLaunchKernelGGL(kern, dim3(n_rg, cf.n_kv_heads, B), dim3(64 * NW), lds, c->stream,
                       kc, vc, cf.n_q_heads, cf.n_kv_heads, cf.max_seq_len, kps, r, c->fmap, st, sel, offset, 1, w.q_norm,
                       w.k_norm, (const float2*)(c->ws + c->o.rope_tab), po, pml, cf.rms_eps, c->part_rows * gq, append,
                       (bf16_t*)attn, (bf16_t*)attn_lo, qd, qs);
    return hipGetLastError();
  }
  constexpr int KPI = 64;
  int want_splits = (int)((4L * c->num_cus + per_split_blocks - 1) / per_split_blocks);
  if (want_splits > ATT_MAX_SPLITS) want_splits = ATT_MAX_SPLITS;
  if (want_splits < 1) want_splits = 1;
  int kps = ((bucket + want_splits - 1) / want_splits + KPI - 1) / KPI * KPI;
  const int ns = (bucket + kps - 1) / kps;
  hipLaunchKernelGGL((attn_split_mfma_kernel<HD, 4, false>), dim3(ns * n_rg, cf.n_kv_heads, B), dim3(256), (size_t)4 * qv_max * HD * 4, c->stream,
                     kc, vc, cf.n_q_heads, cf.n_kv_heads, cf.max_seq_len, kps, r, c->fmap, st, sel, offset, ns, w.q_norm,
                     w.k_norm, (const float2*)(c->ws + c->o.rope_tab), po, pml, cf.rms_eps, c->part_rows * gq, append,
                     (bf16_t*)nullptr, (bf16_t*)nullptr, 0, qs);
  hipLaunchKernelGGL((attn_merge_kernel<HD, OT>), dim3(r, cf.n_q_heads, B), dim3(256), 0, c->stream, po, pml, attn, attn_lo, qd,
                     cf.n_q_heads, cf.n_kv_heads, kps, ns, c->part_rows * gq, st, sel, offset, r, c->fmap);
  return hipGetLastError();
}

// Kernel choice.  bf16 caches: the matrix-core kernel (measured faster than the vector kernel even for
// one row and 4 query heads per KV head: 11.7 vs 13.2 us at 1k context, 99 vs 119 us at 8 x 16k).
// fp32 caches: the vector kernel; share_kv: all rows of a sequence go through one block so that K and V
// are read once (long contexts), else rows are spread over blocks (K/V re-reads hit in L2).
template <typename CT, typename OT>
hipError_t launch_attention(dmtd_ctx* c, int l, const float* qkv, OT* attn, OT* attn_lo, int sel, int offset, int r, int append = 1) {
  const dmtd_config& cf = c->cfg;
  const int gq = cf.n_q_heads / cf.n_kv_heads;
  if (r > kMaxRows && append != 2) return hipErrorInvalidValue;    // more rows than an attention block keeps in LDS: their keys must be in the cache
  if constexpr (std::is_same<CT, bf16_t>::value) {
    if (cf.head_dim == 128) return launch_attention_mfma_t<OT, 128>(c, l, qkv, attn, attn_lo, sel, offset, r, append);
    return launch_attention_mfma_t<OT, 64>(c, l, qkv, attn, attn_lo, sel, offset, r, append);
  }
  const int want = c->share_kv ? r * gq : gq;
  const int qvt = want <= 4 ? 4 : (want <= 8 ? 8 : 16);
  if (cf.head_dim == 128) {
    if (qvt == 4) launch_attention_t<CT, OT, 128, 4>(c, l, qkv, attn, attn_lo, sel, offset, r, append);
    else if (qvt == 8) launch_attention_t<CT, OT, 128, 8>(c, l, qkv, attn, attn_lo, sel, offset, r, append);
    else launch_attention_t<CT, OT, 128, 16>(c, l, qkv, attn, attn_lo, sel, offset, r, append);
  } else {
    if (qvt == 4) launch_attention_t<CT, OT, 64, 4>(c, l, qkv, attn, attn_lo, sel, offset, r, append);
    else if (qvt == 8) launch_attention_t<CT, OT, 64, 8>(c, l, qkv, attn, attn_lo, sel, offset, r, append);
    else launch_attention_t<CT, OT, 64, 16>(c, l, qkv, attn, attn_lo, sel, offset, r, append);
  }
  return hipGetLastError();
}

// ---------------------------------------------------------------- the steps of a pass

// a1: rows <- embeddings of the tokens at the rows' positions (next reader: the norm of layer next_layer)
hipError_t embed_rows(dmtd_ctx* c, Rows& R, int sel, int offset, int r, int next_layer) {
  const dmtd_config& cf = c->cfg;
  const int rows = c->batch * r;
  if (c->packed) {
    hipLaunchKernelGGL(embed_pack_kernel, dim3(rows), dim3(256), 0, c->stream, (const bf16_t*)c->embed, dev_tokens(c),
                       cf.max_seq_len, dev_state(c), sel, offset, r, cf.hidden, R.h, (const bf16_t*)norm_gain_for_layer(c, next_layer),
                       R.xb, R.xb_lo, R.ssp, c->fmap);
    R.n_parts = 1;
  } else {
    hipLaunchKernelGGL(embed_kernel<float>, dim3(rows), dim3(256), 0, c->stream, (const float*)c->embed, dev_tokens(c),
                       cf.max_seq_len, dev_state(c), sel, offset, r, cf.hidden, R.h, c->fmap);
  }
  return hipGetLastError();
}

// literal Eq. 4 during prefill: rows += their embeddings, before layer next_layer
hipError_t add_embed_rows(dmtd_ctx* c, Rows& R, int sel, int offset, int r, int next_layer) {
  const dmtd_config& cf = c->cfg;
  const int rows = c->batch * r;
  if (c->packed) {
    hipLaunchKernelGGL(add_embed_pack_kernel, dim3(rows), dim3(256), 0, c->stream, R.h, (const bf16_t*)c->embed, dev_tokens(c),
                       cf.max_seq_len, dev_state(c), sel, offset, r, cf.hidden, (const bf16_t*)norm_gain_for_layer(c, next_layer),
                       R.xb, R.xb_lo, R.ssp);
    R.n_parts = 1;
  } else {
    hipLaunchKernelGGL(add_embed_rows_kernel<float>, dim3(rows), dim3(256), 0, c->stream, R.h, (const float*)c->embed,
                       dev_tokens(c), cf.max_seq_len, dev_state(c), sel, offset, r, cf.hidden);
  }
  return hipGetLastError();
}

// a8: only each sequence's newest row continues (Sec. 2.2); under the literal Eq. 4 reading its embedding is added
// last_pos (prefill of prompts of different lengths): sequence b's row is the one at explicit position last_pos[b]
hipError_t take_last_rows(dmtd_ctx* c, const Rows& src, Rows& dst, int r, int add_embed, int sel, int offset, int next_layer,
                          const int* last_pos = nullptr) {
  const dmtd_config& cf = c->cfg;
  if (c->packed) {
    hipLaunchKernelGGL(take_last_pack_kernel, dim3(c->batch), dim3(256), 0, c->stream, src.h, dst.h, r, cf.hidden, add_embed,
                       (const bf16_t*)c->embed, dev_tokens(c), cf.max_seq_len, dev_state(c), sel, offset,
                       (const bf16_t*)norm_gain_for_layer(c, next_layer), dst.xb, dst.xb_lo, dst.ssp, (const float*)nullptr, last_pos, c->fmap);
    dst.n_parts = 1;
  } else {
    hipLaunchKernelGGL(take_last_rows_kernel<float>, dim3(c->batch), dim3(256), 0, c->stream, src.h, dst.h, r, cf.hidden,
                       add_embed, (const float*)c->embed, dev_tokens(c), cf.max_seq_len, dev_state(c), sel, offset, (const float*)nullptr, last_pos, c->fmap);
  }
  return hipGetLastError();
}

// a3 as a launch of its own, for passes with more rows per sequence than an attention block keeps in LDS (prefill, the
// whole-sequence forward): the rows' keys (QK-RMSNorm + RoPE) and values go to the cache before the attention launch
template <typename CT>
hipError_t launch_kv_append(dmtd_ctx* c, int l, const float* qkv, int sel, int offset, int r) {
  const dmtd_config& cf = c->cfg;
  const int nqkv = (cf.n_q_heads + 2 * cf.n_kv_heads) * cf.head_dim;
  CT* kc = (CT*)(c->ws + c->o.kv + (size_t)l * c->o.kv_layer_stride);
  CT* vc = (CT*)(c->ws + c->o.kv + (size_t)l * c->o.kv_layer_stride + c->o.kv_v_off);
  const dim3 grid(c->batch * r, cf.n_kv_heads);
  if (cf.head_dim == 128)
    hipLaunchKernelGGL((kv_append_kernel<CT, 128>), grid, dim3(64), 0, c->stream, qkv, nqkv, c->layers[l].k_norm, (const float2*)(c->ws + c->o.rope_tab),
                       kc, vc, cf.n_q_heads, cf.n_kv_heads, cf.max_seq_len, cf.rms_eps, (const DevState*)dev_state(c), sel, offset, r);
  else
    hipLaunchKernelGGL((kv_append_kernel<CT, 64>), grid, dim3(64), 0, c->stream, qkv, nqkv, c->layers[l].k_norm, (const float2*)(c->ws + c->o.rope_tab),
                       kc, vc, cf.n_q_heads, cf.n_kv_heads, cf.max_seq_len, cf.rms_eps, (const DevState*)dev_state(c), sel, offset, r);
  return hipGetLastError();
}

// a2..a7: one transformer block over r rows per sequence at positions base + offset + i
hipError_t run_layer(dmtd_ctx* c, int l, Rows& R, int r, int sel, int offset) {
  const dmtd_config& cf = c->cfg;
  const int rows = c->batch * r, d = cf.hidden, hd = cf.head_dim, ff = cf.intermediate;
  const int nqkv = (cf.n_q_heads + 2 * cf.n_kv_heads) * hd, qd = cf.n_q_heads * hd;
  float* qkv = (float*)(c->ws + c->o.qkv);
  const LayerW& w = c->layers[l];
  hipError_t e;
  if (c->packed) {
    const LayerSw& s = c->sw[l];
    const size_t rows_cap = row_capacity(cf.max_batch);
    bf16_t* ab = (bf16_t*)(c->ws + c->o.attn);      // attention output, high parts; low parts behind them
    bf16_t* ab_lo = ab + rows_cap * qd;
    bf16_t* ub = (bf16_t*)(c->ws + c->o.mlp);       // SwiGLU output, likewise
    bf16_t* ub_lo = ub + rows_cap * ff;
    const int tiles_d = (d + 15) / 16;
    MfmaArgs a{};
    // a2: RMSNorm + fused QKV projection
    a.W = s.qkv; a.xb = R.xb; a.xb_lo = R.xb_lo; a.ldxb = d; a.N = nqkv; a.K = d; a.ssp = R.ssp; a.n_parts = R.n_parts; a.ssp_ld = c->ssp_ld;
    a.eps = cf.rms_eps; a.y = qkv; a.ldy = nqkv;
    const bool wide = r > kMaxRows;      // more rows per sequence than an attention block keeps in LDS: the append is a launch of its own
    c->fold_qkv = !wide;
    e = launch_qkv(c, a, rows);
    c->fold_qkv = false;
    if (e != hipSuccess) { c->qkv_pending = QkvSrc{}; return e; }
    // a3 + a4: QK-RMSNorm + RoPE + KV append + split-K attention, then the merge (output packed for the O projection)
    if (wide && (e = launch_kv_append<bf16_t>(c, l, qkv, sel, offset, r)) != hipSuccess) return e;
    if ((e = launch_attention<bf16_t, bf16_t>(c, l, qkv, ab, ab_lo, sel, offset, r, wide ? 2 : 1)) != hipSuccess) return e;
    // a5: O projection + residual; emits the MLP norm's input
    a = MfmaArgs{};
    a.W = s.o; a.xb = ab; a.xb_lo = ab_lo; a.ldxb = qd; a.N = d; a.K = qd; a.y = R.h; a.ldy = d; a.yb = R.xb; a.yb_lo = R.xb_lo; a.ldyb = d;
    a.g_next = (const bf16_t*)w.mlp_norm; a.ssp_next = R.ssp; a.ssp_ld = c->ssp_ld;
    if ((e = launch_oproj(c, a, rows)) != hipSuccess) return e;
    R.n_parts = tiles_d;
    // a6: RMSNorm + gate/up + SwiGLU
    a = MfmaArgs{};
    a.W = s.gate; a.W2 = s.up; a.xb = R.xb; a.xb_lo = R.xb_lo; a.ldxb = d; a.N = ff; a.K = d; a.ssp = R.ssp; a.n_parts = R.n_parts;
    a.ssp_ld = c->ssp_ld; a.eps = cf.rms_eps; a.yb = ub; a.yb_lo = ub_lo; a.ldyb = ff;
    if ((e = launch_gateup(c, a, rows)) != hipSuccess) return e;
    // a7: down projection + residual; emits the next layer's (or the final) norm input
    a = MfmaArgs{};
    a.W = s.down; a.xb = ub; a.xb_lo = ub_lo; a.ldxb = ff; a.N = d; a.K = ff; a.y = R.h; a.ldy = d; a.yb = R.xb; a.yb_lo = R.xb_lo; a.ldyb = d;
    a.g_next = (const bf16_t*)norm_gain_for_layer(c, l + 1); a.ssp_next = R.ssp; a.ssp_ld = c->ssp_ld;
    if ((e = launch_down(c, a, rows)) != hipSuccess) return e;
    R.n_parts = tiles_d;
    return hipSuccess;
  }
  float* attn = (float*)(c->ws + c->o.attn);
  float* mlp = (float*)(c->ws + c->o.mlp);
  GemvArgs a{};
  a.eps = cf.rms_eps;
  // a2: RMSNorm + fused QKV projection (q, k, v are contiguous in the blob)
  a.W = w.q; a.gain = w.attn_norm; a.x = R.h; a.ldx = d; a.y = qkv; a.ldy = nqkv; a.N = nqkv; a.K = d;
  if ((e = gemv_rows<float, EPI_STORE, true>(c, a, rows)) != hipSuccess) return e;
  // a3 + a4: QK-RMSNorm + RoPE + KV append + split-K attention, then the merge
  if (r > kMaxRows && (e = launch_kv_append<float>(c, l, qkv, sel, offset, r)) != hipSuccess) return e;
  if ((e = launch_attention<float, float>(c, l, qkv, attn, (float*)nullptr, sel, offset, r, r > kMaxRows ? 2 : 1)) != hipSuccess) return e;
  // a5: O projection + residual
  a = GemvArgs{};
  a.W = w.o; a.x = attn; a.ldx = qd; a.y = R.h; a.ldy = d; a.N = d; a.K = qd;
  if ((e = gemv_rows<float, EPI_RESID, false>(c, a, rows)) != hipSuccess) return e;
  // a6: RMSNorm + gate/up + SwiGLU
  a = GemvArgs{};
  a.eps = cf.rms_eps;
  a.W = w.gate; a.W2 = w.up; a.gain = w.mlp_norm; a.x = R.h; a.ldx = d; a.y = mlp; a.ldy = ff; a.N = ff; a.K = d;
  if ((e = gemv_rows<float, EPI_SWIGLU, true>(c, a, rows)) != hipSuccess) return e;
  // a7: down projection + residual
  a = GemvArgs{};
  a.W = w.down; a.x = mlp; a.ldx = ff; a.y = R.h; a.ldy = d; a.N = d; a.K = ff;
  return gemv_rows<float, EPI_RESID, false>(c, a, rows);
}

// a9, first part: final RMSNorm + LM head (Eq. 5) of n_rows rows into logits [n_rows, vocab], selection keys into amax
hipError_t head_logits(dmtd_ctx* c, const Rows& R, int n_rows, float* logits, unsigned long long* amax, int amax_ld) {
  const dmtd_config& cf = c->cfg;
  if (c->packed) {
    MfmaArgs a{};
    a.W = c->lm_head_sw; a.xb = R.xb; a.xb_lo = R.xb_lo; a.ldxb = cf.hidden; a.N = cf.vocab; a.K = cf.hidden; a.ssp = R.ssp; a.n_parts = R.n_parts;
    a.ssp_ld = c->ssp_ld; a.eps = cf.rms_eps; a.y = logits; a.ldy = cf.vocab;
    a.amax = amax; a.amax_ld = amax_ld;
    return launch_lmhead(c, a, n_rows);
  }
  GemvArgs a{};
  a.eps = cf.rms_eps;
  a.W = c->lm_head; a.gain = c->final_norm; a.x = R.h; a.ldx = cf.hidden;
  a.y = logits; a.ldy = cf.vocab; a.N = cf.vocab; a.K = cf.hidden;
  a.amax = amax;
  return gemv_rows<float, EPI_LOGITS, true>(c, a, n_rows);
}

// a9: final RMSNorm + LM head + greedy selection for one row per sequence; then the step's bookkeeping
hipError_t run_head(dmtd_ctx* c, const Rows& R, int full, int write_tokens, int n_rows) {
  const dmtd_config& cf = c->cfg;
  unsigned long long* amax = c->amax;
  hipError_t e = head_logits(c, R, n_rows, (float*)(c->ws + c->o.logits), amax, cf.max_batch);
  if (e != hipSuccess) return e;
  if (c->sampling && write_tokens) {
    hipLaunchKernelGGL(sample_kernel, dim3(n_rows), dim3(1024), 0, c->stream, (const float*)(c->ws + c->o.logits), cf.vocab,
                       (const SampleCfg*)(c->ws + c->o.state + kStateSampleOff), (const DevState*)dev_state(c), amax, AMAX_CELLS, cf.max_batch);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  hipLaunchKernelGGL(finish_step_kernel, dim3(1), dim3(n_rows >= 16 ? 1024 : 64 * n_rows), 0, c->stream, dev_state(c), amax, AMAX_CELLS, cf.max_batch,
                     dev_tokens(c), (int*)(c->ws + c->o.emitted), cf.max_seq_len, n_rows, full, write_tokens, c->full_mask);
  return hipGetLastError();
}

Rows front_rows(dmtd_ctx* c) {
  bf16_t* xb = (bf16_t*)(c->ws + c->o.xb);
  return Rows{(float*)(c->ws + c->o.h), xb, xb + (size_t)row_capacity(c->cfg.max_batch) * c->cfg.hidden, (float*)(c->ws + c->o.ssp), 1};
}
Rows late_rows(dmtd_ctx* c) {
  bf16_t* xb = (bf16_t*)(c->ws + c->o.xb_late);
  return Rows{(float*)(c->ws + c->o.h_late), xb, xb + (size_t)c->cfg.max_batch * c->cfg.hidden, (float*)(c->ws + c->o.ssp_late), 1};
}

// One decode step (Sec. 2.2).  Full: embed the pending rows and the newest row, run the front
// layers on all of them, keep the newest row, run the late layers on it.  Late: embed the
// newest token and run the late layers only (Eq. 4, m = 0).
// ExDy row moves (rows_op_kernel): with or without the packed input of the norm of layer next_layer
hipError_t rows_op(dmtd_ctx* c, int mode, int n_rows, float* dst, const float* src_a, const float* src_b, int r, int c0, int rc,
                   int next_layer, bf16_t* xb, bf16_t* xb_lo, float* ssp) {
  const dmtd_config& cf = c->cfg;
  if (c->packed)
    hipLaunchKernelGGL(rows_op_kernel<true>, dim3(n_rows), dim3(256), 0, c->stream, mode, dst, src_a, src_b, cf.hidden, kMaxTau, r, c0, rc,
                       dev_state(c), (const bf16_t*)norm_gain_for_layer(c, next_layer), xb, xb_lo, ssp);
  else
    hipLaunchKernelGGL(rows_op_kernel<false>, dim3(n_rows), dim3(256), 0, c->stream, mode, dst, src_a, src_b, cf.hidden, kMaxTau, r, c0, rc,
                       dev_state(c), (const bf16_t*)nullptr, (bf16_t*)nullptr, (bf16_t*)nullptr, (float*)nullptr);
  return hipGetLastError();
}

// One decode step (Sec. 2.2).  Full: embed the pending rows and the newest row, run the front
// layers on all of them, keep the newest row, run the late layers on it.  Late: embed the
// newest token and run the late layers only (Eq. 4, m = 0).
// ExDy variant (n_early = E > 0): every step first runs its own token through the E encoding layers; a late
// step stores that output for the refill and jumps to the late layers; a full step gathers the stored outputs
// of the pending tokens and the newest token's, runs the thinking layers E .. F-1 on them, and goes on as before.
hipError_t enqueue_step(dmtd_ctx* c, bool full, int r, int n_late) {
  const dmtd_config& cf = c->cfg;
  const int F = cf.n_layers - n_late, E = c->sched.n_early;
  Rows front = front_rows(c), late = late_rows(c);
  float* pend = (float*)(c->ws + c->o.pend_enc);
  hipError_t e;
  if (E > 0) {
    if ((e = embed_rows(c, late, POS_NTOK, 0, 1, 0)) != hipSuccess) return e;
    for (int l = 0; l < E; ++l)
      if ((e = run_layer(c, l, late, 1, POS_NTOK, 0)) != hipSuccess) return e;
  }
  if (full) {
    // the pending rows are causal among themselves, so groups of rows may pass the front
    // layers one after another (each group streams those layers' weights once)
    int c0 = 0, rc = 0;
    if (F > E) {
      for (; c0 < r; c0 += rc) {
        rc = r - c0 < kMaxRows ? r - c0 : kMaxRows;
        if (E > 0) {
          if ((e = rows_op(c, ROWS_GATHER, c->batch * rc, front.h, pend, late.h, r, c0, rc, E, front.xb, front.xb_lo, front.ssp)) != hipSuccess) return e;
          front.n_parts = 1;
        } else {
          if ((e = embed_rows(c, front, POS_NFRONT, c0, rc, 0)) != hipSuccess) return e;
        }
        for (int l = E; l < F; ++l)
          if ((e = run_layer(c, l, front, rc, POS_NFRONT, c0)) != hipSuccess) return e;
      }
      if (E > 0) {
        // the newest row continues; the literal Eq. 4 reading adds its encoding output (still in the late row buffer)
        if (c->packed)
          hipLaunchKernelGGL(take_last_pack_kernel, dim3(c->batch), dim3(256), 0, c->stream, front.h, late.h, rc, cf.hidden, 0,
                             (const bf16_t*)c->embed, dev_tokens(c), cf.max_seq_len, dev_state(c), (int)POS_NFRONT, c0 - rc,
                             (const bf16_t*)norm_gain_for_layer(c, F), late.xb, late.xb_lo, late.ssp,
                             cf.full_pos_add_embed ? (const float*)late.h : (const float*)nullptr, (const int*)nullptr, (const int*)nullptr);
        else
          hipLaunchKernelGGL(take_last_rows_kernel<float>, dim3(c->batch), dim3(256), 0, c->stream, front.h, late.h, rc, cf.hidden,
                             0, (const float*)c->embed, dev_tokens(c), cf.max_seq_len, dev_state(c), (int)POS_NFRONT, c0 - rc,
                             cf.full_pos_add_embed ? (const float*)late.h : (const float*)nullptr, (const int*)nullptr, (const int*)nullptr);
        if ((e = hipGetLastError()) != hipSuccess) return e;
        late.n_parts = 1;
      } else {
        if ((e = take_last_rows(c, front, late, rc, cf.full_pos_add_embed ? 1 : 0, POS_NFRONT, c0 - rc, F)) != hipSuccess) return e;
      }
    } else if (E > 0 && cf.full_pos_add_embed) {
      // no thinking layers: h_think = h_enc, and the literal reading feeds their sum
      if ((e = rows_op(c, ROWS_ADD, c->batch, late.h, late.h, late.h, 1, 0, 1, F, late.xb, late.xb_lo, late.ssp)) != hipSuccess) return e;
      late.n_parts = 1;
    } else if (E == 0) {
      // n_late = all layers: the newest token's embedding enters the late layers directly
      if ((e = embed_rows(c, late, POS_NTOK, 0, 1, F)) != hipSuccess) return e;
      if (cf.full_pos_add_embed && (e = add_embed_rows(c, late, POS_NTOK, 0, 1, F)) != hipSuccess) return e;
    }
  } else {
    if (E > 0) {
      // keep the encoding output for the refill; the row itself jumps to the late layers
      if (F > E) {
        if ((e = rows_op(c, ROWS_STASH, c->batch, pend, late.h, nullptr, 1, 0, 1, F, late.xb, late.xb_lo, late.ssp)) != hipSuccess) return e;
        late.n_parts = 1;
      }
    } else {
      if ((e = embed_rows(c, late, POS_NTOK, 0, 1, F)) != hipSuccess) return e;
    }
  }
  for (int l = F; l < cf.n_layers; ++l)
    if ((e = run_layer(c, l, late, 1, POS_NTOK, 0)) != hipSuccess) return e;
  return run_head(c, late, full ? 1 : 0, 1, c->batch);
}

// One decode step of a batch whose sequences are at different points of their cycles (Sec. 2.2, per sequence).  The
// sequences that start a new cycle pass the front layers with their pending rows - one front pass per distinct row count,
// over those sequences only (full_list: their slots, sorted by row count; n_rows / n_seqs: the groups) - and every
// sequence's newest token then shares ONE pass through the late layers and the LM head: the late layers read the front
// output for the former and the raw embedding for the others (Eq. 4).
hipError_t enqueue_step_mixed(dmtd_ctx* c, const std::vector<std::pair<int, int>>& groups /* (rows, sequences) */, int n_late,
                              const int* full_list, const unsigned char* full_mask) {
  const dmtd_config& cf = c->cfg;
  const int F = cf.n_layers - n_late, B = c->batch;
  Rows front = front_rows(c), late = late_rows(c);
  hipError_t e;
  if ((e = embed_rows(c, late, POS_NTOK, 0, 1, F)) != hipSuccess) return e;
  int first = 0;
  for (const auto& grp : groups) {
    const int r = grp.first, n = grp.second;
    c->batch = n;
    c->fmap = full_list + first;
    e = embed_rows(c, front, POS_NFRONT, 0, r, 0);
    for (int l = 0; l < F && e == hipSuccess; ++l) e = run_layer(c, l, front, r, POS_NFRONT, 0);
    if (e == hipSuccess) e = take_last_rows(c, front, late, r, cf.full_pos_add_embed ? 1 : 0, POS_NFRONT, 0, F);
    c->batch = B;
    c->fmap = nullptr;
    if (e != hipSuccess) return e;
    first += n;
  }
  for (int l = F; l < cf.n_layers; ++l)
    if ((e = run_layer(c, l, late, 1, POS_NTOK, 0)) != hipSuccess) return e;
  c->full_mask = full_mask;
  e = run_head(c, late, 0, 1, B);
  c->full_mask = nullptr;
  return e;
}

// K/V bytes one layer's attention reads for the whole batch at context length ctx
bool kv_is_large(const dmtd_ctx* c, int ctx) {
  const size_t bytes = (size_t)c->batch * ctx * c->cfg.n_kv_heads * c->cfg.head_dim * 2 * c->elem;
  return bytes > ((size_t)48 << 20);
}

void choose_attention(dmtd_ctx* c, int ctx) {
  c->att_bucket = (ctx + 511) / 512 * 512;
  c->share_kv = kv_is_large(c, ctx);
}

int run_step(dmtd_ctx* c, const Step& s, int n_late) {
  choose_attention(c, s.pos + 1);
  if (!c->cfg.use_graphs) {
    HIP_TRY(c, enqueue_step(c, s.full, s.rows, n_late));
    return DMTD_OK;
  }
  // everything a captured step bakes in: grids and row counts follow from the batch, the attention launch shape from the context bucket
  const auto key = std::make_tuple(s.full ? 1 : 0, s.rows, n_late * 4096 + c->sched.n_early + (c->sampling ? (1 << 30) : 0), c->att_bucket * 2 + (c->share_kv ? 1 : 0), c->batch);
  auto it = c->graphs.find(key);
  if (it == c->graphs.end()) {
    hipGraph_t graph = nullptr;
    HIP_TRY(c, hipStreamBeginCapture(c->stream, hipStreamCaptureModeThreadLocal));
    hipError_t e = enqueue_step(c, s.full, s.rows, n_late);
    hipError_t e2 = hipStreamEndCapture(c->stream, &graph);
    if (e != hipSuccess || e2 != hipSuccess) {
      if (graph) (void)hipGraphDestroy(graph);
      c->err = std::string("graph capture failed: ") + hipGetErrorString(e != hipSuccess ? e : e2);
      return DMTD_EHIP;
    }
    hipGraphExec_t exec = nullptr;
    hipError_t e3 = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
    (void)hipGraphDestroy(graph);
    if (e3 != hipSuccess) { c->err = std::string("hipGraphInstantiate: ") + hipGetErrorString(e3); return DMTD_EHIP; }
    it = c->graphs.emplace(key, exec).first;
  }
  HIP_TRY(c, hipGraphLaunch(it->second, c->stream));
  return DMTD_OK;
}

// Several consecutive steps of one call as ONE graph (dmtd_decode): the steps of a cycle - a full step and the late-only
// steps behind it - or, at tau = 1, up to kStepsPerGraph full steps.  Between two graph launches the GPU idles for ~8 us
// (end of one graph to the first kernel of the next), three times per C3 cycle with a graph per step.  The steps of a
// group share their attention launch shape (512-token context bucket, KV sharing), otherwise the group ends early.
constexpr int kStepsPerGraph = 4;
int run_steps_grouped(dmtd_ctx* c, const std::vector<Step>& steps, int tau, int n_late) {
  const int n = (int)steps.size();
  int i = 0;
  while (i < n) {
    choose_attention(c, steps[i].pos + 1);
    const int bucket = c->att_bucket;
    const bool share = c->share_kv;
    int j = i + 1;
    const int limit = tau > 1 ? tau : kStepsPerGraph;
    while (j < n && j - i < limit && !(tau > 1 && steps[j].full)) {
      choose_attention(c, steps[j].pos + 1);
      if (c->att_bucket != bucket || c->share_kv != share) break;
      ++j;
    }
    if (!c->cfg.use_graphs || j - i == 1) {
      const int rc = run_step(c, steps[i], n_late);
      if (rc != DMTD_OK) return rc;
      i += 1;
      continue;
    }
    std::vector<int> key = {c->batch, n_late, c->sched.n_early, c->sampling ? 1 : 0, bucket, share ? 1 : 0};
    for (int k = i; k < j; ++k) { key.push_back(steps[k].full ? 1 : 0); key.push_back(steps[k].rows); }
    auto it = c->group_graphs.find(key);
    if (it == c->group_graphs.end()) {
      hipGraph_t graph = nullptr;
      HIP_TRY(c, hipStreamBeginCapture(c->stream, hipStreamCaptureModeThreadLocal));
      hipError_t e = hipSuccess;
      for (int k = i; k < j && e == hipSuccess; ++k) {
        choose_attention(c, steps[k].pos + 1);
        e = enqueue_step(c, steps[k].full, steps[k].rows, n_late);
      }
      hipError_t e2 = hipStreamEndCapture(c->stream, &graph);
      if (e != hipSuccess || e2 != hipSuccess) {
        if (graph) (void)hipGraphDestroy(graph);
        c->err = std::string("graph capture failed: ") + hipGetErrorString(e != hipSuccess ? e : e2);
        return DMTD_EHIP;
      }
      hipGraphExec_t exec = nullptr;
      hipError_t e3 = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
      (void)hipGraphDestroy(graph);
      if (e3 != hipSuccess) { c->err = std::string("hipGraphInstantiate: ") + hipGetErrorString(e3); return DMTD_EHIP; }
      it = c->group_graphs.emplace(key, exec).first;
    }
    HIP_TRY(c, hipGraphLaunch(it->second, c->stream));
    i = j;
  }
  return DMTD_OK;
}

struct PartRowsGuard {     // restores the partials' row layout on every way out of a prefill-type pass
  dmtd_ctx* c; int saved;
  ~PartRowsGuard() { c->part_rows = saved; }
};

// Prefill (Sec. 2.2): all prompt positions through all layers, in chunks of rows
hipError_t enqueue_prefill(dmtd_ctx* c, int P, int n_late, bool ragged) {
  const dmtd_config& cf = c->cfg;
  Rows front = front_rows(c), late = late_rows(c);
  const int add_at = cf.full_pos_add_embed ? cf.n_layers - n_late : -1;
  hipError_t e;
  hipLaunchKernelGGL(set_state_kernel, dim3(1), dim3(64), 0, c->stream, dev_state(c), P - 1, P - 1, cf.max_batch);
  int r_last = 0, p_last = 0;
  const int chunk = pass_positions(c->batch);
  PartRowsGuard guard{c, c->part_rows};
  c->part_rows = chunk;                 // the attention partials are laid out for a pass's rows per sequence
  for (int p0 = 0; p0 < P; p0 += chunk) {
    const int r = P - p0 < chunk ? P - p0 : chunk;
    choose_attention(c, p0 + r);
    if ((e = embed_rows(c, front, POS_EXPLICIT, p0, r, 0)) != hipSuccess) return e;
    const int E = c->sched.n_early;
    for (int l = 0; l < cf.n_layers; ++l) {
      if (add_at >= 0 && E > 0 && l == E) {
        // literal Eq. 4, ExDy variant: the encoding output is what full positions get added at the late boundary
        if ((e = hipMemcpyAsync(c->ws + c->o.enc_tmp, front.h, (size_t)c->batch * r * cf.hidden * 4, hipMemcpyDeviceToDevice, c->stream)) != hipSuccess) return e;
      }
      if (l == add_at) {
        if (E > 0) {
          if ((e = rows_op(c, ROWS_ADD, c->batch * r, front.h, front.h, (const float*)(c->ws + c->o.enc_tmp), 1, 0, 1, l, front.xb, front.xb_lo, front.ssp)) != hipSuccess) return e;
          front.n_parts = 1;
        } else if ((e = add_embed_rows(c, front, POS_EXPLICIT, p0, r, l)) != hipSuccess) return e;
      }
      if ((e = run_layer(c, l, front, r, POS_EXPLICIT, p0)) != hipSuccess) return e;
    }
    r_last = r; p_last = p0;
    // prompts of different lengths: a sequence whose last prompt position lies in this chunk hands that row to the LM head
    if (ragged && (e = take_last_rows(c, front, late, r, 0, POS_EXPLICIT, p0, cf.n_layers,
                                      (const int*)(c->ws + c->o.state + kStateDeltaOff) + 2 * cf.max_batch)) != hipSuccess) return e;
  }
  if (!ragged && (e = take_last_rows(c, front, late, r_last, 0, POS_EXPLICIT, p_last, cf.n_layers)) != hipSuccess) return e;
  return run_head(c, late, 1, 1, c->batch);   // state goes from P-1 to n_tok = n_front = P
}

// One chunk of the whole-sequence masked forward (Sec. 2.1, Eqs. 1-5): positions p0 .. p0+r-1 of every sequence pass the
// encoding and thinking layers, Eq. 4 picks each position's input to the decoding layers by its mask bit, the
// decoding layers and the LM head follow for every row, and a row kernel takes the Eq. 6 summands and the argmax.
// Earlier chunks are seen through the KV caches, exactly as later decode steps would see them.
hipError_t enqueue_masked_chunk(dmtd_ctx* c, int p0, int r, int n, int n_late) {
  const dmtd_config& cf = c->cfg;
  const int F = cf.n_layers - n_late, E = c->sched.n_early, rows = c->batch * r;
  Rows R = front_rows(c);
  float* enc = (float*)(c->ws + c->o.enc_tmp);
  hipError_t e;
  choose_attention(c, p0 + r);
  if ((e = embed_rows(c, R, POS_EXPLICIT, p0, r, 0)) != hipSuccess) return e;
  for (int l = 0; l <= F; ++l) {
    if (E > 0 && l == E &&
        (e = hipMemcpyAsync(enc, R.h, (size_t)rows * cf.hidden * 4, hipMemcpyDeviceToDevice, c->stream)) != hipSuccess) return e;
    if (l < F && (e = run_layer(c, l, R, r, POS_EXPLICIT, p0)) != hipSuccess) return e;
  }
  const int* mask = (const int*)(c->ws + c->o.mask);
  if (c->packed) {
    hipLaunchKernelGGL((mask_combine_kernel<bf16_t, true>), dim3(rows), dim3(256), 0, c->stream, R.h, E > 0 ? (const float*)enc : (const float*)nullptr,
                       (const bf16_t*)c->embed, dev_tokens(c), cf.max_seq_len, mask, p0, r, cf.hidden, cf.full_pos_add_embed,
                       (const bf16_t*)norm_gain_for_layer(c, F), R.xb, R.xb_lo, R.ssp);
    R.n_parts = 1;
  } else {
    hipLaunchKernelGGL((mask_combine_kernel<float, false>), dim3(rows), dim3(256), 0, c->stream, R.h, E > 0 ? (const float*)enc : (const float*)nullptr,
                       (const float*)c->embed, dev_tokens(c), cf.max_seq_len, mask, p0, r, cf.hidden, cf.full_pos_add_embed,
                       (const bf16_t*)nullptr, (bf16_t*)nullptr, (bf16_t*)nullptr, (float*)nullptr);
  }
  if ((e = hipGetLastError()) != hipSuccess) return e;
  for (int l = F; l < cf.n_layers; ++l)
    if ((e = run_layer(c, l, R, r, POS_EXPLICIT, p0)) != hipSuccess) return e;
  float* logits = (float*)(c->ws + c->o.logits_rows);
  if ((e = head_logits(c, R, rows, logits, (unsigned long long*)(c->ws + c->o.amax_rows), row_capacity(cf.max_batch))) != hipSuccess) return e;
  hipLaunchKernelGGL(nll_rows_kernel, dim3(rows), dim3(1024), 0, c->stream, (const float*)logits, cf.vocab, (const int*)dev_tokens(c), cf.max_seq_len,
                     p0, r, n, (float*)(c->ws + c->o.nll), (int*)(c->ws + c->o.best));
  return hipGetLastError();
}

// One launch of one kernel kind on layer l, for dmtd_time_kernel.  Outputs go to scratch
// buffers only (never the late rows, the caches, the token history or the scheduler state).
hipError_t time_one(dmtd_ctx* c, int kind, int l, int rows) {
  const dmtd_config& cf = c->cfg;
  const int d = cf.hidden, hd = cf.head_dim, ff = cf.intermediate;
  const int nqkv = (cf.n_q_heads + 2 * cf.n_kv_heads) * hd, qd = cf.n_q_heads * hd;
  Rows R = front_rows(c);
  float* qkv = (float*)(c->ws + c->o.qkv);
  const LayerW& w = c->layers[l];
  if (kind >= DMTD_K_READ_QKV && kind <= DMTD_K_READ_DOWN) {
    // nothing but a read of the bytes the projection of that kind streams for layer l (the stored weight image)
    const LayerSw& s = c->sw[l];
    const bf16_t *p0 = nullptr, *p1 = nullptr;
    size_t n0 = 0, n1 = 0;                       // 16-byte units
    switch (kind) {
      case DMTD_K_READ_QKV:    p0 = s.qkv;  n0 = swizzled_elems(nqkv, d) / 8; break;
      case DMTD_K_READ_OPROJ:  p0 = s.o;    n0 = swizzled_elems(d, qd) / 8; break;
      case DMTD_K_READ_GATEUP: p0 = s.gate; n0 = swizzled_elems(ff, d) / 8; p1 = s.up; n1 = n0; break;
      default:                 p0 = s.down; n0 = swizzled_elems(d, ff) / 8; break;
    }
    hipLaunchKernelGGL(read_only_kernel, dim3(2048), dim3(256), 0, c->stream, (const u32x4*)p0, n0, (const u32x4*)(p1 ? p1 : p0), n1,
                       (u32x4*)qkv);
    return hipGetLastError();
  }
  if (kind == DMTD_K_ATTN) {
    // attention for `rows` query rows per sequence ending at the newest cached position
    const int last = c->sched.n_tok - 1;
    const int r = rows <= last + 1 ? rows : 1;
    // the cache append is switched off: the launch scores the rows' new keys from the scratch q/k/v, writes nothing
    choose_attention(c, last + 1);
    if (c->packed) return launch_attention<bf16_t, bf16_t>(c, l, qkv, (bf16_t*)(c->ws + c->o.attn), (bf16_t*)(c->ws + c->o.attn) + (size_t)row_capacity(cf.max_batch) * cf.n_q_heads * cf.head_dim, (int)POS_EXPLICIT, last - r + 1, r, 0);
    return launch_attention<float, float>(c, l, qkv, (float*)(c->ws + c->o.attn), (float*)nullptr, (int)POS_EXPLICIT, last - r + 1, r, 0);
  }
  if (kind == DMTD_K_LMHEAD) {
    R.n_parts = 1;
    return run_head(c, R, 0, 0, rows);     // the real LM-head kernel; keys cleared, no token or state side effects
  }
  if (c->packed) {
    const LayerSw& s = c->sw[l];
    const size_t rows_cap = row_capacity(cf.max_batch);
    bf16_t* ab = (bf16_t*)(c->ws + c->o.attn);
    bf16_t* ab_lo = ab + rows_cap * qd;
    bf16_t* ub = (bf16_t*)(c->ws + c->o.mlp);
    bf16_t* ub_lo = ub + rows_cap * ff;
    MfmaArgs a{};
    a.ssp_ld = c->ssp_ld; a.eps = cf.rms_eps;
    switch (kind) {
      case DMTD_K_QKV:
        a.W = s.qkv; a.xb = R.xb; a.xb_lo = R.xb_lo; a.ldxb = d; a.N = nqkv; a.K = d; a.ssp = R.ssp; a.n_parts = 1; a.y = qkv; a.ldy = nqkv;
        return launch_qkv(c, a, rows);
      case DMTD_K_OPROJ:
        a.W = s.o; a.xb = ab; a.xb_lo = ab_lo; a.ldxb = qd; a.N = d; a.K = qd; a.y = R.h; a.ldy = d; a.yb = R.xb; a.yb_lo = R.xb_lo; a.ldyb = d;
        a.g_next = (const bf16_t*)w.mlp_norm; a.ssp_next = R.ssp;
        return launch_oproj(c, a, rows);
      case DMTD_K_GATEUP:
        a.W = s.gate; a.W2 = s.up; a.xb = R.xb; a.xb_lo = R.xb_lo; a.ldxb = d; a.N = ff; a.K = d; a.ssp = R.ssp; a.n_parts = (d + 15) / 16;
        a.yb = ub; a.yb_lo = ub_lo; a.ldyb = ff;
        return launch_gateup(c, a, rows);
      default:
        a.W = s.down; a.xb = ub; a.xb_lo = ub_lo; a.ldxb = ff; a.N = d; a.K = ff; a.y = R.h; a.ldy = d; a.yb = R.xb; a.yb_lo = R.xb_lo; a.ldyb = d;
        a.g_next = (const bf16_t*)norm_gain_for_layer(c, l + 1); a.ssp_next = R.ssp;
        return launch_down(c, a, rows);
    }
  }
  float* attn = (float*)(c->ws + c->o.attn);
  float* mlp = (float*)(c->ws + c->o.mlp);
  GemvArgs a{};
  a.eps = cf.rms_eps;
  switch (kind) {
    case DMTD_K_QKV:
      a.W = w.q; a.gain = w.attn_norm; a.x = R.h; a.ldx = d; a.y = qkv; a.ldy = nqkv; a.N = nqkv; a.K = d;
      return gemv_rows<float, EPI_STORE, true>(c, a, rows);
    case DMTD_K_OPROJ:
      a.W = w.o; a.x = attn; a.ldx = qd; a.y = R.h; a.ldy = d; a.N = d; a.K = qd;
      return gemv_rows<float, EPI_RESID, false>(c, a, rows);
    case DMTD_K_GATEUP:
      a.W = w.gate; a.W2 = w.up; a.gain = w.mlp_norm; a.x = R.h; a.ldx = d; a.y = mlp; a.ldy = ff; a.N = ff; a.K = d;
      return gemv_rows<float, EPI_SWIGLU, true>(c, a, rows);
    default:
      a.W = w.down; a.x = mlp; a.ldx = ff; a.y = R.h; a.ldy = d; a.N = d; a.K = ff;
      return gemv_rows<float, EPI_RESID, false>(c, a, rows);
  }
}

void destroy_graphs(dmtd_ctx* c) {
  for (auto& kv : c->graphs) (void)hipGraphExecDestroy(kv.second);
  c->graphs.clear();
  for (auto& kv : c->group_graphs) (void)hipGraphExecDestroy(kv.second);
  c->group_graphs.clear();
  for (auto& kv : c->mixed_graphs) (void)hipGraphExecDestroy(kv.second);
  c->mixed_graphs.clear();
}

}  // namespace

// ============================================================================ C ABI

extern "C" {

size_t dmtd_workspace_bytes(const dmtd_config* cfg) {
  std::string why;
  if (!valid_config(cfg, why)) return 0;
  return layout(*cfg).total;
}

int dmtd_create(const dmtd_config* cfg, const void* weights_dev, size_t weights_bytes, void* workspace_dev,
                size_t workspace_bytes, dmtd_ctx** out) {
  std::string why;
  if (!out) { g_create_error = "null out pointer"; return DMTD_EINVAL; }
  *out = nullptr;
  if (!valid_config(cfg, why)) { g_create_error = why; return DMTD_EINVAL; }
  const size_t elem = cfg->dtype == DMTD_DTYPE_F32 ? 4 : 2;
  const Ws lay = layout(*cfg);
  if (!cfg->dry_run) {
    if (!weights_dev || !workspace_dev) { g_create_error = "null device pointer"; return DMTD_EINVAL; }
    if (((uintptr_t)weights_dev & 15) || ((uintptr_t)workspace_dev & 255)) {
      g_create_error = "weights must be 16-byte aligned and the workspace 256-byte aligned"; return DMTD_EINVAL;
    }
    if (weights_bytes != weight_elems(*cfg) * elem) {
      g_create_error = "weight blob size does not match the configuration"; return DMTD_EINVAL;
    }
    if (workspace_bytes < lay.total) { g_create_error = "workspace too small"; return DMTD_ECAPACITY; }
  }
  dmtd_ctx* c = new dmtd_ctx();
  c->cfg = *cfg;
  c->elem = (int)elem;
  c->o = lay;
  c->stream = (hipStream_t)cfg->stream;
  c->sched.n_layers = cfg->n_layers;
  c->sched.max_seq_len = cfg->max_seq_len;
  c->packed = cfg->dtype == DMTD_DTYPE_BF16;
  c->ssp_ld = row_capacity(cfg->max_batch);
  if (const char* ev = std::getenv("DMTD_TEST_FAIL_STEP")) c->test_fail_step = std::atoi(ev);
  c->plan_buf.reserve(kMaxTau + 1);
  c->sched.trace.reserve((size_t)12 * cfg->max_seq_len + 64);        // at most 3 records of 4 per step: later steps never reallocate
  if (!cfg->dry_run) {
    c->wbase = (const char*)weights_dev;
    c->ws = (char*)workspace_dev;
    c->part_o = (float*)(c->ws + lay.part_o);
    c->part_ml = (float*)(c->ws + lay.part_ml);
    c->amax = (unsigned long long*)(c->ws + lay.amax);
    c->gemm_part = c->packed ? (float*)(c->ws + lay.gemm_part) : nullptr;
    c->part_rows = kMaxRows;
    {
      hipError_t se = static_scratch_for_current_device(&c->static_scratch);
      if (se != hipSuccess) { g_create_error = std::string("hipGetSymbolAddress(scratch): ") + hipGetErrorString(se); delete c; return DMTD_EHIP; }
    }
    // carve the blob
    const size_t d = cfg->hidden, qd = (size_t)cfg->n_q_heads * cfg->head_dim, kd = (size_t)cfg->n_kv_heads * cfg->head_dim;
    const size_t ff = cfg->intermediate, hd = cfg->head_dim;
    size_t off = 0;
    auto take = [&](size_t n) { const void* p = c->wbase + off * elem; off += n; return p; };
    c->embed = take((size_t)cfg->vocab * d);
    c->layers.resize(cfg->n_layers);
    for (LayerW& w : c->layers) {
      w.attn_norm = take(d); w.q = take(qd * d); w.k = take(kd * d); w.v = take(kd * d);
      w.q_norm = take(hd); w.k_norm = take(hd); w.o = take(d * qd); w.mlp_norm = take(d);
      w.gate = take(ff * d); w.up = take(ff * d); w.down = take(d * ff);
    }
    c->final_norm = take(d);
    c->lm_head = cfg->tied_embeddings ? c->embed : take((size_t)cfg->vocab * d);

    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) {
      g_create_error = "no HIP device"; delete c; return DMTD_EHIP;
    }
    c->num_cus = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    // rotary frequency table theta^(-2i/hd) in double; counters and state cleared
    std::vector<double> inv(hd / 2);
    for (size_t i = 0; i < hd / 2; ++i) inv[i] = std::pow((double)cfg->rope_theta, -2.0 * (double)i / (double)hd);
    hipError_t e = hipMemcpyAsync(c->ws + lay.inv_freq, inv.data(), inv.size() * 8, hipMemcpyHostToDevice, c->stream);
    if (e == hipSuccess) {
      hipLaunchKernelGGL(rope_table_kernel, dim3(1024), dim3(256), 0, c->stream, (const double*)(c->ws + lay.inv_freq),
                         (float2*)(c->ws + lay.rope_tab), cfg->max_seq_len, (int)(hd / 2));
      e = hipGetLastError();
    }
    if (e == hipSuccess) e = hipMemsetAsync(c->ws + lay.amax, 0, (size_t)AMAX_CELLS * cfg->max_batch * 8, c->stream);
    if (e == hipSuccess) e = hipMemsetAsync(c->ws + lay.state, 0, kStateDeltaOff + 12 * (size_t)cfg->max_batch, c->stream);
    if (e == hipSuccess) e = hipMemsetAsync(c->ws + lay.kv, 0, lay.kv_layer_stride * cfg->n_layers, c->stream);
    if (e == hipSuccess && c->packed) {
      // one-time repack of every matrix into MFMA operand order (q, k, v are contiguous: one fused matrix)
      bf16_t* dst = (bf16_t*)(c->ws + lay.wsw);
      auto swz = [&](const void* src, size_t N, size_t K) {
        const bf16_t* out = dst;
        hipLaunchKernelGGL(swizzle_weights_kernel, dim3(2048), dim3(256), 0, c->stream, (const bf16_t*)src, dst, (int)N, (int)K);
        dst += swizzled_elems(N, K);
        return out;
      };
      const size_t nqkv = qd + 2 * kd;
      c->sw.resize(cfg->n_layers);
      for (int l = 0; l < cfg->n_layers; ++l) {
        const LayerW& w = c->layers[l];
        LayerSw& s = c->sw[l];
        s.qkv = swz(w.q, nqkv, d); s.o = swz(w.o, d, qd); s.gate = swz(w.gate, ff, d); s.up = swz(w.up, ff, d);
        s.down = swz(w.down, d, ff);
      }
      c->lm_head_sw = swz(c->lm_head, cfg->vocab, d);
      e = hipGetLastError();
    }
    if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
    if (e != hipSuccess) { g_create_error = std::string("workspace setup: ") + hipGetErrorString(e); delete c; return DMTD_EHIP; }
  }
  *out = c;
  return DMTD_OK;
}

static int prefill_impl(dmtd_ctx* c, const int32_t* tokens, int32_t batch, int32_t prompt_len, const int32_t* lengths, int32_t n_late,
                        int32_t* first_tokens) {
  if (!c) return DMTD_EINVAL;
  const dmtd_config& cf = c->cfg;
  if (!tokens) { c->err = "null tokens"; return DMTD_EINVAL; }
  if (batch < 1 || batch > cf.max_batch) { c->err = "batch outside [1, max_batch]"; return DMTD_EINVAL; }
  if (prompt_len < 1) { c->err = "prompt_len must be >= 1"; return DMTD_EINVAL; }
  if (cf.full_pos_add_embed && (n_late < 1 || n_late > cf.n_layers)) { c->err = "the literal Eq. 4 reading needs n_late at prefill"; return DMTD_EINVAL; }
  if (cf.full_pos_add_embed && c->sched.n_early + n_late > cf.n_layers) { c->err = "n_early + n_late exceeds the number of layers"; return DMTD_EINVAL; }
  if (c->sched.n_tok != 0) { c->err = "already prefilled; call dmtd_reset first"; return DMTD_ESTATE; }
  if (prompt_len >= cf.max_seq_len) { c->err = "prompt does not leave room for a generated token"; return DMTD_ECAPACITY; }
  bool ragged = false;
  if (lengths) {
    int longest = 0;
    for (int b = 0; b < batch; ++b) {
      if (lengths[b] < 1 || lengths[b] > prompt_len) { c->err = "prompt length outside [1, prompt_len]"; return DMTD_EINVAL; }
      if (lengths[b] > longest) longest = lengths[b];
      ragged = ragged || lengths[b] != prompt_len;
    }
    if (longest != prompt_len) { c->err = "prompt_len must be the longest prompt's length"; return DMTD_EINVAL; }
  }
  for (int b = 0; b < batch; ++b) {
    const int len = lengths ? lengths[b] : prompt_len;
    for (int i = 0; i < len; ++i) {
      const int32_t t = tokens[(size_t)b * prompt_len + i];
      if (t < 0 || t >= cf.vocab) { c->err = "token id outside the vocabulary"; return DMTD_EINVAL; }
    }
  }
  c->batch = batch;
  if (!cf.dry_run) {
    int* dtok = (int*)(c->ws + c->o.tokens);
    // padding behind a shorter prompt is replaced by token 0: those rows run (their results are never read) and must index the table safely
    std::vector<int32_t> tk(tokens, tokens + (size_t)batch * prompt_len);
    std::vector<int32_t> meta(3 * (size_t)cf.max_batch, 0);       // (delta, front)[max_batch], last_prompt_pos[max_batch]
    for (int b = 0; b < batch; ++b) {
      const int len = lengths ? lengths[b] : prompt_len;
      for (int i = len; i < prompt_len; ++i) tk[(size_t)b * prompt_len + i] = 0;
      meta[2 * b] = len - prompt_len;                            // the front positions are set by the prefill itself
      meta[2 * cf.max_batch + b] = len - 1;
    }
    HIP_TRY(c, hipMemcpyAsync(c->ws + c->o.state + kStateDeltaOff, meta.data(), meta.size() * 4, hipMemcpyHostToDevice, c->stream));
    HIP_TRY(c, hipMemcpy2DAsync(dtok, (size_t)cf.max_seq_len * 4, tk.data(), (size_t)prompt_len * 4, (size_t)prompt_len * 4, batch,
                                hipMemcpyHostToDevice, c->stream));
    HIP_TRY(c, enqueue_prefill(c, prompt_len, n_late, ragged));
    std::vector<int32_t> first(batch);
    HIP_TRY(c, hipMemcpyAsync(first.data(), c->ws + c->o.emitted, (size_t)batch * 4, hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    if (first_tokens) std::memcpy(first_tokens, first.data(), (size_t)batch * 4);
  } else if (first_tokens) {
    for (int b = 0; b < batch; ++b) first_tokens[b] = -1;
  }
  c->sched.note_prefill(prompt_len, cf.full_pos_add_embed ? n_late : 0);
  return DMTD_OK;
}

int dmtd_prefill(dmtd_ctx* c, const int32_t* tokens, int32_t batch, int32_t prompt_len, int32_t n_late, int32_t* first_tokens) {
  return prefill_impl(c, tokens, batch, prompt_len, nullptr, n_late, first_tokens);
}

int dmtd_prefill_ragged(dmtd_ctx* c, const int32_t* tokens, int32_t batch, int32_t prompt_len, const int32_t* lengths, int32_t n_late,
                        int32_t* first_tokens) {
  if (c && !lengths) { c->err = "null lengths"; return DMTD_EINVAL; }
  return prefill_impl(c, tokens, batch, prompt_len, lengths, n_late, first_tokens);
}

// Decode steps of one call: plan (host only), enqueue everything on the stream, one copy of the emitted tokens and one
// synchronisation at the end.  cycles: false = stop when the current cycle is complete (dmtd_decode_cycle); true = go on
// with further cycles until n_steps steps have run (dmtd_decode).
static int decode_steps(dmtd_ctx* c, int32_t tau, int32_t n_late, int32_t n_steps, bool cycles, const int32_t* forced_inputs,
                        int32_t n_forced, int32_t* out_tokens, int32_t out_stride, int32_t* n_emitted) {
  if (!c) return DMTD_EINVAL;
  const dmtd_config& cf = c->cfg;
  if (n_emitted) *n_emitted = 0;
  if (!out_tokens || !n_emitted) { c->err = "null output pointer"; return DMTD_EINVAL; }
  if (tau > kMaxTau) { c->err = "tau above the supported maximum (64)"; return DMTD_EINVAL; }
  if (forced_inputs && n_forced < 1) { c->err = "forced_inputs given with n_forced < 1"; return DMTD_EINVAL; }
  if (cycles && (n_steps < 1 || n_steps > kMaxTau)) { c->err = "n_steps must be in [1, 64]"; return DMTD_EINVAL; }
  if (c->diverged) { c->err = "the sequences are at different points of their cycles: use dmtd_decode_per_seq"; return DMTD_ESTATE; }
  const int f_stride = forced_inputs ? n_forced : 0;
  std::vector<Step> steps;
  int err = 0;
  std::string why;
  if (!cycles) {
    if (!c->sched.plan(tau, n_late, n_steps, kMaxTau, steps, err, why)) {
      c->err = why;
      return err == 1 ? DMTD_EINVAL : (err == 2 ? DMTD_ESTATE : DMTD_ECAPACITY);
    }
  } else {
    // cycle after cycle on a copy of the host state (the plan of a cycle depends on where the one before it ended);
    // nothing runs unless every cycle can be planned
    Sched ahead = c->sched;
    ahead.trace.clear();
    std::vector<Step> one;
    while ((int)steps.size() < n_steps) {
      if (!ahead.plan(tau, n_late, n_steps - (int)steps.size(), kMaxTau, one, err, why)) {
        c->err = why;
        return err == 1 ? DMTD_EINVAL : (err == 2 ? DMTD_ESTATE : DMTD_ECAPACITY);
      }
      ahead.commit(one, n_late);
      ahead.trace.clear();
      steps.insert(steps.end(), one.begin(), one.end());
    }
  }
  const int n = (int)steps.size();
  if (out_stride < n) { c->err = "out_stride smaller than the number of steps"; return DMTD_ECAPACITY; }
  const int B = c->batch;
  const int nf = f_stride < n ? f_stride : n;   // forced inputs beyond the steps run are ignored
  for (int b = 0; b < B && forced_inputs; ++b)
    for (int i = 0; i < nf; ++i) {
      const int32_t t = forced_inputs[(size_t)b * f_stride + i];
      if (t < 0 || t >= cf.vocab) { c->err = "forced token id outside the vocabulary"; return DMTD_EINVAL; }
    }
  if (!cf.dry_run) {
    int* fdev = (int*)(c->ws + c->o.forced);
    std::vector<int32_t> fhost((size_t)B * (nf > 0 ? nf : 1));
    if (nf > 0) {
      for (int b = 0; b < B; ++b)
        for (int i = 0; i < nf; ++i) fhost[(size_t)b * nf + i] = forced_inputs[(size_t)b * f_stride + i];
      HIP_TRY(c, hipMemcpyAsync(fdev, fhost.data(), (size_t)B * nf * 4, hipMemcpyHostToDevice, c->stream));
    }
    hipLaunchKernelGGL(begin_call_kernel, dim3(1), dim3(256), 0, c->stream, (DevState*)(c->ws + c->o.state),
                       (int*)(c->ws + c->o.tokens), cf.max_seq_len, fdev, nf, nf, cf.vocab, B);
    HIP_TRY(c, hipGetLastError());
    int rc = DMTD_OK;
    if (c->test_fail_step >= 0) {
      // failure injected from the host (DMTD_TEST_FAIL_STEP at create): the steps before it run, then the call fails the
      // way a refused launch would; every kernel that was enqueued completes normally
      for (int i = 0; i < n && i < c->test_fail_step && rc == DMTD_OK; ++i) rc = run_step(c, steps[i], n_late);
      if (rc == DMTD_OK) { c->err = "injected launch failure (DMTD_TEST_FAIL_STEP)"; rc = DMTD_EHIP; }
      c->test_fail_step = -1;
    } else if (cycles) rc = run_steps_grouped(c, steps, tau, n_late);
    else
      for (const Step& s : steps)
        if ((rc = run_step(c, s, n_late)) != DMTD_OK) break;
    {
      if (rc != DMTD_OK) {
        // device state may be ahead of the host's; resynchronise it to the host's unchanged view
        (void)hipStreamSynchronize(c->stream);
        hipLaunchKernelGGL(set_state_kernel, dim3(1), dim3(64), 0, c->stream, (DevState*)(c->ws + c->o.state),
                           c->sched.n_tok, c->sched.n_front, cf.max_batch);
        (void)hipStreamSynchronize(c->stream);
        return rc;
      }
    }
    std::vector<int32_t> em((size_t)n * B);
    HIP_TRY(c, hipMemcpyAsync(em.data(), c->ws + c->o.emitted, em.size() * 4, hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    for (int b = 0; b < B; ++b)
      for (int i = 0; i < n; ++i) out_tokens[(size_t)b * out_stride + i] = em[(size_t)i * B + b];
  } else {
    for (int b = 0; b < B; ++b)
      for (int i = 0; i < n; ++i) out_tokens[(size_t)b * out_stride + i] = -1;
  }
  c->sched.commit(steps, n_late);
  *n_emitted = n;
  return DMTD_OK;
}

int dmtd_decode_cycle(dmtd_ctx* c, int32_t tau, int32_t n_late, int32_t max_new, const int32_t* forced_inputs,
                      int32_t n_forced, int32_t* out_tokens, int32_t out_stride, int32_t* n_emitted) {
  return decode_steps(c, tau, n_late, max_new, false, forced_inputs, n_forced, out_tokens, out_stride, n_emitted);
}

int dmtd_decode(dmtd_ctx* c, int32_t tau, int32_t n_late, int32_t n_steps, const int32_t* forced_inputs,
                int32_t n_forced, int32_t* out_tokens, int32_t out_stride, int32_t* n_emitted) {
  return decode_steps(c, tau, n_late, n_steps, true, forced_inputs, n_forced, out_tokens, out_stride, n_emitted);
}

int dmtd_decode_cycle_noalloc(dmtd_ctx* c, int32_t tau, int32_t n_late, int32_t max_new, const int32_t* forced_dev,
                              int32_t n_forced, int32_t* out_tokens_dev, int32_t out_stride, int32_t* n_emitted) {
  if (!c) return DMTD_EINVAL;
  const dmtd_config& cf = c->cfg;
  if (n_emitted) *n_emitted = 0;
  if (!n_emitted || (!out_tokens_dev && !cf.dry_run)) { c->err = "null output pointer"; return DMTD_EINVAL; }
  if (tau > kMaxTau) { c->err = "tau above the supported maximum (64)"; return DMTD_EINVAL; }
  if (forced_dev && n_forced < 1) { c->err = "forced inputs given with n_forced < 1"; return DMTD_EINVAL; }
  if (c->diverged) { c->err = "the sequences are at different points of their cycles: use dmtd_decode_per_seq"; return DMTD_ESTATE; }
  std::vector<Step>& steps = c->plan_buf;       // capacity reserved at create: planning allocates nothing
  int err = 0;
  std::string why;
  if (!c->sched.plan(tau, n_late, max_new, kMaxTau, steps, err, why)) {
    c->err = why;
    return err == 1 ? DMTD_EINVAL : (err == 2 ? DMTD_ESTATE : DMTD_ECAPACITY);
  }
  const int n = (int)steps.size();
  if (out_stride < n) { c->err = "out_stride smaller than the number of steps"; return DMTD_ECAPACITY; }
  if (!cf.dry_run) {
    const int B = c->batch, gq = cf.n_q_heads / cf.n_kv_heads;
    const int nf = forced_dev ? (n_forced < n ? n_forced : n) : 0;
    // what the steps' kernels need beyond the workspace's state: sized for this call, carved from the library's array
    int max_rows = 1;
    bool tiled = false;
    const int d = cf.hidden, qd = cf.n_q_heads * cf.head_dim, ff = cf.intermediate, nqkv = qd + 2 * cf.n_kv_heads * cf.head_dim;
    const int tiles_d = (d + 15) / 16;
    for (const Step& s : steps) {
      if (s.rows > max_rows) max_rows = s.rows;
      const int rows = B * (s.rows < kMaxRows ? s.rows : kMaxRows);
      if (c->packed)
        for (int rr : {rows, B})
          tiled = tiled || !mfma_rows_fit(c, rr, nqkv, d, tiles_d) || !mfma_rows_fit(c, rr, d, qd, 0) || !mfma_rows_fit(c, rr, ff, d, tiles_d) ||
                  !mfma_rows_fit(c, rr, d, ff, 0) || !mfma_rows_fit(c, rr, cf.vocab, d, tiles_d);
    }
    if (max_rows > kMaxRows) max_rows = kMaxRows;
    const size_t qv_stride = (size_t)max_rows * gq;
    const size_t amax_b = align_up((size_t)AMAX_CELLS * cf.max_batch * 8, 256);
    const size_t pml_b = align_up((size_t)B * cf.n_kv_heads * ATT_MAX_SPLITS * qv_stride * 2 * 4, 256);
    const size_t po_b = align_up((size_t)B * cf.n_kv_heads * ATT_MAX_SPLITS * qv_stride * cf.head_dim * 4, 256);
    size_t gp_b = 0;
    if (tiled) {
      size_t widest = 2 * (size_t)ff > (size_t)nqkv ? 2 * (size_t)ff : (size_t)nqkv;
      if ((size_t)d > widest) widest = d;
      const size_t rows_max = (size_t)B * max_rows < (size_t)kGemmRows ? (size_t)B * max_rows : (size_t)kGemmRows;
      gp_b = align_up((size_t)kGemmMaxSplit * rows_max * widest * 4, 256);
    }
    if (amax_b + pml_b + po_b + gp_b > kStaticScratchBytes) {
      c->err = "dmtd_decode_cycle_noalloc: this call's partial results (" + std::to_string((amax_b + pml_b + po_b + gp_b) >> 10) +
               " KiB for batch " + std::to_string(B) + " with " + std::to_string(max_rows) + " rows per sequence) exceed the library's " +
               std::to_string(kStaticScratchBytes >> 20) + " MiB scratch; use dmtd_decode_cycle";
      return DMTD_ECAPACITY;
    }
    // the steps run eagerly on the context's stream with their scratch in the library's array
    struct Saved { float *po, *pml, *gp; unsigned long long* amax; int rows; } saved{c->part_o, c->part_ml, c->gemm_part, c->amax, c->part_rows};
    char* base = c->static_scratch;
    c->amax = (unsigned long long*)base;
    c->part_ml = (float*)(base + amax_b);
    c->part_o = (float*)(base + amax_b + pml_b);
    c->gemm_part = (float*)(base + amax_b + pml_b + po_b);
    c->part_rows = max_rows;
    // the array keeps the last call's contents: the selection-key cells must start at zero (a fill kernel, so that a
    // caller may capture this call into a graph)
    hipLaunchKernelGGL(zero_u64_kernel, dim3(4), dim3(256), 0, c->stream, c->amax, AMAX_CELLS * cf.max_batch);
    hipLaunchKernelGGL(begin_call_kernel, dim3(1), dim3(256), 0, c->stream, (DevState*)(c->ws + c->o.state),
                       (int*)(c->ws + c->o.tokens), cf.max_seq_len, forced_dev, nf, n_forced, cf.vocab, B);
    hipError_t e = hipGetLastError();
    for (int i = 0; i < n && e == hipSuccess; ++i) {
      choose_attention(c, steps[i].pos + 1);
      e = enqueue_step(c, steps[i].full, steps[i].rows, n_late);
    }
    if (e == hipSuccess) {
      hipLaunchKernelGGL(emitted_to_rows_kernel, dim3(1), dim3(256), 0, c->stream, (const int*)(c->ws + c->o.emitted), out_tokens_dev, n, B, out_stride);
      e = hipGetLastError();
    }
    c->part_o = saved.po; c->part_ml = saved.pml; c->gemm_part = saved.gp; c->amax = saved.amax; c->part_rows = saved.rows;
    if (e != hipSuccess) {
      c->err = std::string("dmtd_decode_cycle_noalloc: ") + hipGetErrorString(e);
      return DMTD_EHIP;
    }
  }
  c->sched.commit(steps, n_late);
  *n_emitted = n;
  return DMTD_OK;
}

int dmtd_decode_per_seq(dmtd_ctx* c, const int32_t* tau, int32_t n_late, int32_t n_steps, const int32_t* forced_inputs,
                        int32_t n_forced, int32_t* out_tokens, int32_t out_stride, int32_t* n_emitted) {
  if (!c) return DMTD_EINVAL;
  const dmtd_config& cf = c->cfg;
  if (n_emitted) *n_emitted = 0;
  if (!out_tokens || !n_emitted || !tau) { c->err = "null pointer"; return DMTD_EINVAL; }
  if (c->sched.n_tok == 0) { c->err = "decode before prefill"; return DMTD_ESTATE; }
  if (n_steps < 1 || n_steps > kMaxTau) { c->err = "n_steps must be in [1, 64]"; return DMTD_EINVAL; }
  if (n_late < 1 || n_late > cf.n_layers) { c->err = "n_late must be in [1, n_layers]"; return DMTD_EINVAL; }
  if (c->sched.n_early != 0) { c->err = "per-sequence cycle lengths are not available in the ExDy variant"; return DMTD_ESTATE; }
  if (forced_inputs && n_forced < 1) { c->err = "forced_inputs given with n_forced < 1"; return DMTD_EINVAL; }
  if (out_stride < n_steps) { c->err = "out_stride smaller than the number of steps"; return DMTD_ECAPACITY; }
  const int B = c->batch, n = n_steps;
  for (int b = 0; b < B; ++b)
    if (tau[b] < 1 || tau[b] > kMaxTau) { c->err = "every sequence's tau must be in [1, 64]"; return DMTD_EINVAL; }
  if (c->sched.n_tok + n > cf.max_seq_len) { c->err = "sequence would exceed max_seq_len"; return DMTD_ECAPACITY; }
  // plan on copies of the per-sequence state: rows[i][b] = 0 for a late-only step of sequence b, else its row count
  std::vector<int> phase = c->diverged ? c->seq_phase : std::vector<int>(B, c->sched.phase);
  std::vector<int> front = c->diverged ? c->seq_front : std::vector<int>(B, c->sched.n_front);
  if (c->sched.n_late_in_use != 0 && c->sched.n_late_in_use != n_late)
    for (int b = 0; b < B; ++b)
      if (front[b] != c->sched.n_tok) { c->err = "n_late changed while tokens await refill"; return DMTD_ESTATE; }
  std::vector<std::vector<int>> rows(n, std::vector<int>(B, 0));
  int t = c->sched.n_tok;
  for (int i = 0; i < n; ++i, ++t)
    for (int b = 0; b < B; ++b) {
      if (phase[b] >= tau[b]) {
        rows[i][b] = t - front[b] + 1;
        if (rows[i][b] > kMaxRows) { c->err = "more pending refill rows than the workspace holds"; return DMTD_ECAPACITY; }
        front[b] = t + 1; phase[b] = 1;
      } else {
        phase[b] += 1;
      }
    }
  const int f_stride = forced_inputs ? n_forced : 0;
  const int nf = f_stride < n ? f_stride : n;
  for (int b = 0; b < B && forced_inputs; ++b)
    for (int i = 0; i < nf; ++i) {
      const int32_t tk = forced_inputs[(size_t)b * f_stride + i];
      if (tk < 0 || tk >= cf.vocab) { c->err = "forced token id outside the vocabulary"; return DMTD_EINVAL; }
    }
  if (!cf.dry_run) {
    int* fdev = (int*)(c->ws + c->o.forced);
    std::vector<int32_t> fhost((size_t)B * (nf > 0 ? nf : 1));
    if (nf > 0) {
      for (int b = 0; b < B; ++b)
        for (int i = 0; i < nf; ++i) fhost[(size_t)b * nf + i] = forced_inputs[(size_t)b * f_stride + i];
      HIP_TRY(c, hipMemcpyAsync(fdev, fhost.data(), (size_t)B * nf * 4, hipMemcpyHostToDevice, c->stream));
    }
    hipLaunchKernelGGL(begin_call_kernel, dim3(1), dim3(256), 0, c->stream, (DevState*)(c->ws + c->o.state),
                       (int*)(c->ws + c->o.tokens), cf.max_seq_len, fdev, nf, nf, cf.vocab, B);
    HIP_TRY(c, hipGetLastError());
    std::vector<std::vector<char>> uploads;           // host images of new patterns: alive until the call's synchronisation
    int rc = DMTD_OK;
    for (int i = 0; i < n && rc == DMTD_OK; ++i) {
      const int pos = c->sched.n_tok + i;
      bool same = true;
      for (int b = 1; b < B; ++b) same = same && rows[i][b] == rows[i][0];
      if (same) {       // all sequences at the same point of their cycles: the ordinary step (and its graph)
        rc = run_step(c, Step{rows[i][0] > 0, rows[i][0] > 0 ? rows[i][0] : 1, pos}, n_late);
        continue;
      }
      choose_attention(c, pos + 1);
      // the sequences that start a cycle, sorted by row count (one front pass per count)
      std::vector<int> order;
      for (int b = 0; b < B; ++b) if (rows[i][b] > 0) order.push_back(b);
      std::stable_sort(order.begin(), order.end(), [&](int x, int y) { return rows[i][x] < rows[i][y]; });
      std::vector<std::pair<int, int>> groups;
      for (int b : order) {
        if (!groups.empty() && groups.back().first == rows[i][b]) groups.back().second += 1;
        else groups.emplace_back(rows[i][b], 1);
      }
      // the pattern's device image: the list (ints) and the mask (bytes); cached patterns keep their slot for good (graphs
      // refer to it), the last slot serves patterns beyond the table, without a graph
      auto it = c->pattern_ids.find(rows[i]);
      int slot;
      const bool cached = it != c->pattern_ids.end() || (int)c->pattern_ids.size() < kMaxPatterns - 1;
      if (it != c->pattern_ids.end()) slot = it->second;
      else {
        slot = cached ? (int)c->pattern_ids.size() : kMaxPatterns - 1;
        uploads.emplace_back(kPatternStride(cf.max_batch), 0);
        std::vector<char>& img = uploads.back();
        for (size_t k = 0; k < order.size(); ++k) std::memcpy(img.data() + 4 * k, &order[k], 4);
        for (int b = 0; b < B; ++b) img[(size_t)4 * cf.max_batch + b] = rows[i][b] > 0 ? 1 : 0;
        hipError_t ce = hipMemcpyAsync(c->ws + c->o.patterns + (size_t)slot * kPatternStride(cf.max_batch), img.data(), img.size(),
                                       hipMemcpyHostToDevice, c->stream);
        if (ce != hipSuccess) { c->err = std::string("pattern upload: ") + hipGetErrorString(ce); rc = DMTD_EHIP; break; }
        if (cached) c->pattern_ids.emplace(rows[i], slot);
      }
      const char* img_dev = c->ws + c->o.patterns + (size_t)slot * kPatternStride(cf.max_batch);
      const int* list_dev = (const int*)img_dev;
      const unsigned char* mask_dev = (const unsigned char*)img_dev + (size_t)4 * cf.max_batch;
      if (!cf.use_graphs || !cached) {
        hipError_t e = enqueue_step_mixed(c, groups, n_late, list_dev, mask_dev);
        if (e != hipSuccess) { c->err = std::string("mixed step: ") + hipGetErrorString(e); rc = DMTD_EHIP; }
        continue;
      }
      const std::vector<int> key = {slot, n_late, c->sampling ? 1 : 0, c->att_bucket, c->share_kv ? 1 : 0, B};
      auto git = c->mixed_graphs.find(key);
      if (git == c->mixed_graphs.end()) {
        hipGraph_t graph = nullptr;
        hipError_t e0 = hipStreamBeginCapture(c->stream, hipStreamCaptureModeThreadLocal);
        if (e0 != hipSuccess) { c->err = std::string("hipStreamBeginCapture: ") + hipGetErrorString(e0); rc = DMTD_EHIP; break; }
        hipError_t e = enqueue_step_mixed(c, groups, n_late, list_dev, mask_dev);
        hipError_t e2 = hipStreamEndCapture(c->stream, &graph);
        if (e != hipSuccess || e2 != hipSuccess) {
          if (graph) (void)hipGraphDestroy(graph);
          c->err = std::string("graph capture failed: ") + hipGetErrorString(e != hipSuccess ? e : e2);
          rc = DMTD_EHIP; break;
        }
        hipGraphExec_t exec = nullptr;
        hipError_t e3 = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
        (void)hipGraphDestroy(graph);
        if (e3 != hipSuccess) { c->err = std::string("hipGraphInstantiate: ") + hipGetErrorString(e3); rc = DMTD_EHIP; break; }
        git = c->mixed_graphs.emplace(key, exec).first;
      }
      hipError_t le = hipGraphLaunch(git->second, c->stream);
      if (le != hipSuccess) { c->err = std::string("hipGraphLaunch: ") + hipGetErrorString(le); rc = DMTD_EHIP; }
    }
    if (rc != DMTD_OK) {
      // back to the host's unchanged view: counters, and every sequence's front position
      (void)hipStreamSynchronize(c->stream);
      hipLaunchKernelGGL(set_state_kernel, dim3(1), dim3(64), 0, c->stream, (DevState*)(c->ws + c->o.state), c->sched.n_tok, c->sched.n_front, cf.max_batch);
      if (c->diverged) {
        int* tmp = (int*)(c->ws + c->o.forced);
        (void)hipMemcpyAsync(tmp, c->seq_front.data(), (size_t)B * 4, hipMemcpyHostToDevice, c->stream);
        hipLaunchKernelGGL(set_fronts_kernel, dim3(1), dim3(64), 0, c->stream, (DevState*)(c->ws + c->o.state), (const int*)tmp, B);
      }
      (void)hipStreamSynchronize(c->stream);
      return rc;
    }
    std::vector<int32_t> em((size_t)n * B);
    HIP_TRY(c, hipMemcpyAsync(em.data(), c->ws + c->o.emitted, em.size() * 4, hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    for (int b = 0; b < B; ++b)
      for (int i = 0; i < n; ++i) out_tokens[(size_t)b * out_stride + i] = em[(size_t)i * B + b];
  } else {
    for (int b = 0; b < B; ++b)
      for (int i = 0; i < n; ++i) out_tokens[(size_t)b * out_stride + i] = -1;
  }
  // commit: the counters and the trace follow sequence 0; the per-sequence state is kept while the sequences differ
  const int F = cf.n_layers - n_late;
  for (int i = 0; i < n; ++i) {
    Sched& sc = c->sched;
    sc.pass_no += 1;
    if (rows[i][0] > 0) {
      if (F > 0) sc.record(0, sc.n_tok - (rows[i][0] - 1), rows[i][0]);
      sc.record(1, sc.n_tok, 1);
      sc.gen_layer_visits += cf.n_layers;
      sc.refill_layer_visits += (int64_t)(rows[i][0] - 1) * F;
      sc.n_full_steps += 1;
    } else {
      sc.record(1, sc.n_tok, 1);
      sc.gen_layer_visits += n_late;
    }
    sc.n_tok += 1;
    sc.n_emitted += 1;
  }
  c->sched.n_late_in_use = n_late;
  c->sched.n_front = front[0];
  c->sched.phase = phase[0];
  c->seq_phase = phase;
  c->seq_front = front;
  c->diverged = false;
  for (int b = 1; b < B; ++b) c->diverged = c->diverged || phase[b] != phase[0] || front[b] != front[0];
  *n_emitted = n;
  return DMTD_OK;
}

int dmtd_get_seq_state(const dmtd_ctx* c, int32_t b, int32_t* n_front, int32_t* phase) {
  if (!c) return DMTD_EINVAL;
  if (b < 0 || b >= c->batch) return DMTD_EINVAL;
  if (n_front) *n_front = c->diverged ? c->seq_front[b] : c->sched.n_front;
  if (phase) *phase = c->diverged ? c->seq_phase[b] : c->sched.phase;
  return DMTD_OK;
}

int dmtd_logits(dmtd_ctx* c, float* out, size_t out_elems) {
  if (!c) return DMTD_EINVAL;
  if (!out) { c->err = "null output pointer"; return DMTD_EINVAL; }
  if (c->sched.n_tok == 0 || c->cfg.dry_run) { c->err = "no logits before prefill"; return DMTD_ESTATE; }
  const size_t need = (size_t)c->batch * c->cfg.vocab;
  if (out_elems < need) { c->err = "logits buffer too small"; return DMTD_ECAPACITY; }
  HIP_TRY(c, hipMemcpyAsync(out, c->ws + c->o.logits, need * 4, hipMemcpyDeviceToHost, c->stream));
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  return DMTD_OK;
}

int dmtd_get_state(const dmtd_ctx* c, int32_t* n_tok, int32_t* n_front, int32_t* phase, int64_t* counters) {
  if (!c) return DMTD_EINVAL;
  if (n_tok) *n_tok = c->sched.n_tok;
  if (n_front) *n_front = c->sched.n_front;
  if (phase) *phase = c->sched.phase;
  if (counters) {
    counters[0] = c->sched.gen_layer_visits;
    counters[1] = c->sched.refill_layer_visits;
    counters[2] = c->sched.n_emitted;
    counters[3] = c->sched.n_full_steps;
  }
  return DMTD_OK;
}

int dmtd_get_trace(const dmtd_ctx* c, int32_t* buf, int32_t cap_records, int32_t* n_records) {
  if (!c || !n_records) return DMTD_EINVAL;
  const int total = (int)(c->sched.trace.size() / 4);
  *n_records = total;
  if (buf && cap_records > 0) {
    const int n = total < cap_records ? total : cap_records;
    std::memcpy(buf, c->sched.trace.data(), (size_t)n * 16);
  }
  return DMTD_OK;
}

int dmtd_read_kv(dmtd_ctx* c, int32_t layer, int32_t b, int32_t n_pos, float* out, size_t out_elems) {
  if (!c) return DMTD_EINVAL;
  const dmtd_config& cf = c->cfg;
  if (!out || layer < 0 || layer >= cf.n_layers || b < 0 || b >= cf.max_batch || n_pos < 1 || n_pos > cf.max_seq_len) {
    c->err = "bad argument to dmtd_read_kv"; return DMTD_EINVAL;
  }
  if (cf.dry_run) { c->err = "no device state in a dry run"; return DMTD_ESTATE; }
  const size_t half = (size_t)cf.n_kv_heads * n_pos * cf.head_dim;
  if (out_elems < 2 * half) { c->err = "KV buffer too small"; return DMTD_ECAPACITY; }
  // each (b, g) owns a contiguous run of positions in the cache: copy the raw rows and widen on the host
  const size_t elem = c->elem, run = (size_t)n_pos * cf.head_dim;
  std::vector<char> raw(2 * half * elem);
  const char* kc = c->ws + c->o.kv + (size_t)layer * c->o.kv_layer_stride;
  const char* vc = kc + c->o.kv_v_off;
  for (int which = 0; which < 2; ++which)
    for (int g = 0; g < cf.n_kv_heads; ++g) {
      const char* src = (which ? vc : kc) + (((size_t)b * cf.n_kv_heads + g) * cf.max_seq_len) * cf.head_dim * elem;
      HIP_TRY(c, hipMemcpyAsync(raw.data() + ((size_t)which * cf.n_kv_heads + g) * run * elem, src, run * elem,
                                hipMemcpyDeviceToHost, c->stream));
    }
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  if (elem == 4) {
    std::memcpy(out, raw.data(), 2 * half * 4);
  } else {
    const uint16_t* r16 = (const uint16_t*)raw.data();
    for (size_t i = 0; i < 2 * half; ++i) {
      const uint32_t u = (uint32_t)r16[i] << 16;
      std::memcpy(out + i, &u, 4);
    }
  }
  return DMTD_OK;
}

int dmtd_time_kernel(dmtd_ctx* c, int32_t kind, int32_t rows, int32_t reps, float* avg_us) {
  if (!c) return DMTD_EINVAL;
  // attention: rows per sequence (at most 16); projections: total activation rows (at most max_batch * 16, the row buffers' capacity)
  const int rows_max = kind == DMTD_K_ATTN ? kMaxRows : row_capacity(c->cfg.max_batch);
  if (!avg_us || kind < 0 || kind > DMTD_K_READ_DOWN || rows < 1 || rows > rows_max || reps < 1) {
    c->err = "bad argument to dmtd_time_kernel"; return DMTD_EINVAL;
  }
  if (kind >= DMTD_K_READ_QKV && !c->packed) { c->err = "the read-only kinds need a bf16 model (they read its stored weight image)"; return DMTD_EINVAL; }
  if (c->cfg.dry_run || c->sched.n_tok == 0) { c->err = "dmtd_time_kernel needs a prefilled context"; return DMTD_ESTATE; }
  if (kind == DMTD_K_LMHEAD && rows > c->batch) { c->err = "the LM head carries one row per sequence"; return DMTD_EINVAL; }
  hipEvent_t e0, e1;
  HIP_TRY(c, hipEventCreate(&e0));
  HIP_TRY(c, hipEventCreate(&e1));
  // rows is per sequence for attention, total activation rows for the projections
  const int saved_batch = c->batch;
  long launches = 0;
  hipError_t e = hipSuccess;
  for (int pass = 0; pass < 2 && e == hipSuccess; ++pass) {   // pass 0 warms up (one repetition)
    const int n = pass == 0 ? 1 : reps;
    if (pass == 1) e = hipEventRecord(e0, c->stream);
    for (int i = 0; i < n && e == hipSuccess; ++i) {
      if (kind == DMTD_K_LMHEAD) {
        e = time_one(c, kind, 0, rows);
        if (pass == 1) launches += 1;
      } else {
        for (int l = 0; l < c->cfg.n_layers && e == hipSuccess; ++l) {
          e = time_one(c, kind, l, rows);
          if (pass == 1) launches += 1;
        }
      }
    }
    if (pass == 1 && e == hipSuccess) e = hipEventRecord(e1, c->stream);
  }
  c->batch = saved_batch;
  if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
  float ms = 0.f;
  if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (e != hipSuccess) { c->err = std::string("dmtd_time_kernel: ") + hipGetErrorString(e); return DMTD_EHIP; }
  *avg_us = ms * 1000.0f / (float)launches;
  return DMTD_OK;
}

int dmtd_masked_forward(dmtd_ctx* c, const int32_t* tokens, int32_t batch, int32_t n, const uint8_t* mask, int32_t n_late,
                        float* nll, int32_t* best, float* logits, size_t logits_elems, float* loss) {
  if (!c) return DMTD_EINVAL;
  const dmtd_config& cf = c->cfg;
  if (!tokens || !mask) { c->err = "null tokens or mask"; return DMTD_EINVAL; }
  if (batch < 1 || batch > cf.max_batch) { c->err = "batch outside [1, max_batch]"; return DMTD_EINVAL; }
  if (n < 1) { c->err = "sequence length must be >= 1"; return DMTD_EINVAL; }
  if (n_late < 1 || n_late > cf.n_layers) { c->err = "n_late must be in [1, n_layers]"; return DMTD_EINVAL; }
  if (c->sched.n_early + n_late > cf.n_layers) { c->err = "n_early + n_late exceeds the number of layers"; return DMTD_EINVAL; }
  if (c->sched.n_tok != 0) { c->err = "the masked forward needs an empty context; call dmtd_reset first"; return DMTD_ESTATE; }
  if (n > cf.max_seq_len) { c->err = "sequence longer than max_seq_len"; return DMTD_ECAPACITY; }
  if (logits && logits_elems < (size_t)batch * n * cf.vocab) { c->err = "logits buffer too small"; return DMTD_ECAPACITY; }
  for (size_t i = 0; i < (size_t)batch * n; ++i)
    if (tokens[i] < 0 || tokens[i] >= cf.vocab) { c->err = "token id outside the vocabulary"; return DMTD_EINVAL; }
  if (cf.dry_run) { c->err = "no device work in a dry run"; return DMTD_ESTATE; }
  const int saved_batch = c->batch;
  c->batch = batch;
  std::vector<int32_t> m32(n);
  for (int i = 0; i < n; ++i) m32[i] = mask[i] ? 1 : 0;
  int rc = DMTD_OK;
  hipError_t e = hipMemcpy2DAsync(c->ws + c->o.tokens, (size_t)cf.max_seq_len * 4, tokens, (size_t)n * 4, (size_t)n * 4, batch,
                                  hipMemcpyHostToDevice, c->stream);
  if (e == hipSuccess) e = hipMemcpyAsync(c->ws + c->o.mask, m32.data(), (size_t)n * 4, hipMemcpyHostToDevice, c->stream);
  const int chunk = pass_positions(batch);
  PartRowsGuard guard{c, c->part_rows};
  c->part_rows = chunk;
  for (int p0 = 0; p0 < n && e == hipSuccess; p0 += chunk) {
    const int r = n - p0 < chunk ? n - p0 : chunk;
    e = enqueue_masked_chunk(c, p0, r, n, n_late);
    if (logits && e == hipSuccess) {
      // the chunk's rows of sequence b follow each other: one copy per sequence, before the next chunk reuses the buffer
      for (int b = 0; b < batch && e == hipSuccess; ++b)
        e = hipMemcpyAsync(logits + ((size_t)b * n + p0) * cf.vocab, c->ws + c->o.logits_rows + (size_t)b * r * cf.vocab * 4,
                           (size_t)r * cf.vocab * 4, hipMemcpyDeviceToHost, c->stream);
      if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
    }
  }
  std::vector<float> nll_h((size_t)batch * n), loss_h(batch);
  if (e == hipSuccess) {
    hipLaunchKernelGGL(mean_nll_kernel, dim3(batch), dim3(256), 0, c->stream, (const float*)(c->ws + c->o.nll), cf.max_seq_len, n,
                       (float*)(c->ws + c->o.loss));
    e = hipGetLastError();
  }
  if (e == hipSuccess) e = hipMemcpyAsync(loss_h.data(), c->ws + c->o.loss, (size_t)batch * 4, hipMemcpyDeviceToHost, c->stream);
  if (e == hipSuccess) e = hipMemcpy2DAsync(nll_h.data(), (size_t)n * 4, c->ws + c->o.nll, (size_t)cf.max_seq_len * 4, (size_t)n * 4, batch,
                                            hipMemcpyDeviceToHost, c->stream);
  if (e == hipSuccess && best) e = hipMemcpy2DAsync(best, (size_t)n * 4, c->ws + c->o.best, (size_t)cf.max_seq_len * 4, (size_t)n * 4, batch,
                                                    hipMemcpyDeviceToHost, c->stream);
  // the caches served as scratch: back to the empty state on the device as on the host
  if (e == hipSuccess) {
    hipLaunchKernelGGL(set_state_kernel, dim3(1), dim3(64), 0, c->stream, dev_state(c), 0, 0, cf.max_batch);
    e = hipGetLastError();
  }
  if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
  c->batch = saved_batch;
  if (e != hipSuccess) { c->err = std::string("dmtd_masked_forward: ") + hipGetErrorString(e); (void)hipStreamSynchronize(c->stream); return DMTD_EHIP; }
  if (nll) std::memcpy(nll, nll_h.data(), nll_h.size() * 4);
  if (loss) std::memcpy(loss, loss_h.data(), (size_t)batch * 4);
  return rc;
}

int dmtd_set_sampling(dmtd_ctx* c, float temperature, int32_t top_k, uint64_t seed) {
  if (!c) return DMTD_EINVAL;
  if (!(temperature == temperature) || temperature > 1e30f) { c->err = "temperature must be a finite number"; return DMTD_EINVAL; }
  if (top_k < 0) { c->err = "top_k must be >= 0"; return DMTD_EINVAL; }
  const bool on = temperature > 0.f && top_k != 1;      // top_k = 1 is the greedy choice whatever the temperature
  if (on && !c->cfg.dry_run) {
    SampleCfg sc{1.0f / temperature, top_k, (unsigned int)(seed & 0xFFFFFFFFull), (unsigned int)(seed >> 32)};
    HIP_TRY(c, hipMemcpyAsync(c->ws + c->o.state + kStateSampleOff, &sc, sizeof sc, hipMemcpyHostToDevice, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));        // sc is a stack object
  }
  c->sampling = on;
  return DMTD_OK;
}

int dmtd_set_n_early(dmtd_ctx* c, int32_t n_early) {
  if (!c) return DMTD_EINVAL;
  if (n_early < 0 || n_early >= c->cfg.n_layers) { c->err = "n_early must be in [0, n_layers - 1]"; return DMTD_EINVAL; }
  if (c->sched.n_tok != c->sched.n_front || c->diverged) { c->err = "n_early changed while tokens await refill"; return DMTD_ESTATE; }
  if (c->sched.n_tok != 0 && c->cfg.full_pos_add_embed && n_early != c->sched.n_early) {
    c->err = "under the literal Eq. 4 reading n_early is fixed at prefill"; return DMTD_ESTATE;
  }
  c->sched.n_early = n_early;
  return DMTD_OK;
}

int dmtd_reset(dmtd_ctx* c) {
  if (!c) return DMTD_EINVAL;
  if (!c->cfg.dry_run) {
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    hipLaunchKernelGGL(set_state_kernel, dim3(1), dim3(64), 0, c->stream, (DevState*)(c->ws + c->o.state), 0, 0, c->cfg.max_batch);
    HIP_TRY(c, hipGetLastError());
    HIP_TRY(c, hipMemsetAsync(c->ws + c->o.state + kStateDeltaOff, 0, 12 * (size_t)c->cfg.max_batch, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
  }
  c->sched.reset();
  c->batch = 0;
  c->diverged = false;
  c->seq_phase.clear();
  c->seq_front.clear();
  return DMTD_OK;
}

void dmtd_destroy(dmtd_ctx* c) {
  if (!c) return;
  if (!c->cfg.dry_run) {
    (void)hipStreamSynchronize(c->stream);
    destroy_graphs(c);
  }
  delete c;
}

const char* dmtd_last_error(const dmtd_ctx* c) { return c ? c->err.c_str() : g_create_error.c_str(); }

}  // extern "C"
