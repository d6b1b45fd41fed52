// C ABI of the DMTD decode path (see include/dmtd.h): context, workspace layout, step
// assembly, hipGraph capture/replay and the host-visible calls.
#include "../../include/dmtd.h"

#include <hip/hip_runtime.h>

#include <cmath>
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
constexpr int kGemvRows = 4;         // activation rows per weight-streaming pass
constexpr int kPrefillChunk = 16;    // prompt positions per prefill pass (per sequence)
constexpr int kMaxRows = 16;         // rows per sequence one pass through the layers may carry
constexpr int kMfmaRows = 16;        // activation rows per MFMA weight-streaming pass
constexpr int kMfmaPF = 10;          // k-steps (64 elements) a wave of the MFMA kernel holds in registers

thread_local std::string g_create_error;

struct LayerW {
  const void *attn_norm, *q, *k, *v, *q_norm, *k_norm, *o, *mlp_norm, *gate, *up, *down;
};

struct Ws {   // device workspace carve-up (byte offsets)
  size_t kv, kv_layer_stride, kv_v_off;
  size_t h, h_late, qkv, attn, mlp, logits, part_o, part_ml, amax;
  size_t tokens, emitted, forced, state, inv_freq, scratch_f32;
  size_t total;
};

}  // namespace

struct dmtd_ctx {
  dmtd_config cfg;
  Sched sched;
  std::string err;
  hipStream_t stream = nullptr;
  int elem = 2;
  int num_cus = 256;
  int batch = 0;              // batch of the current sequence set (after prefill)
  int max_rows = 0;           // rows per sequence a pass may carry
  const char* wbase = nullptr;
  char* ws = nullptr;
  Ws o{};
  const void* embed = nullptr;
  const void* final_norm = nullptr;
  const void* lm_head = nullptr;
  std::vector<LayerW> layers;
  std::map<std::tuple<int, int, int, int>, hipGraphExec_t> graphs;   // (full, rows, n_late, share_kv)
  bool have_logits = false;
  bool share_kv = false;      // attention launches: one pass over K/V for all rows of a sequence (long contexts)
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
  if (c->max_batch < 1 || c->max_seq_len < 2) { why = "max_batch >= 1 and max_seq_len >= 2 required"; return false; }
  if (!(c->rms_eps > 0.f) || !(c->rope_theta > 0.f)) { why = "rms_eps and rope_theta must be positive"; return false; }
  return true;
}

int rows_cap(const dmtd_config&) { return kMaxRows; }   // rows per sequence per pass

size_t weight_elems(const dmtd_config& c) {
  const size_t d = c.hidden, qd = (size_t)c.n_q_heads * c.head_dim, kd = (size_t)c.n_kv_heads * c.head_dim, ff = c.intermediate;
  const size_t per_layer = d + qd * d + 2 * kd * d + 2 * (size_t)c.head_dim + d * qd + d + 3 * ff * d;
  return (size_t)c.vocab * d + c.n_layers * per_layer + d + (c.tied_embeddings ? 0 : (size_t)c.vocab * d);
}

Ws layout(const dmtd_config& c) {
  Ws w{};
  const size_t e = c.dtype == DMTD_DTYPE_F32 ? 4 : 2;
  const size_t B = c.max_batch, S = c.max_seq_len, d = c.hidden, hd = c.head_dim;
  const size_t nqkv = (size_t)(c.n_q_heads + 2 * c.n_kv_heads) * hd, qd = (size_t)c.n_q_heads * hd;
  const size_t rows = B * rows_cap(c);
  const size_t splits = ATT_MAX_SPLITS;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
  const size_t kv_one = B * c.n_kv_heads * S * hd * e;       // K (or V) of one layer
  w.kv_v_off = align_up(kv_one, 256);
  w.kv_layer_stride = 2 * w.kv_v_off;
  w.kv = take(w.kv_layer_stride * c.n_layers);
  w.h = take(rows * d * 4);
  w.h_late = take(B * d * 4);
  w.qkv = take(rows * nqkv * 4);
  w.attn = take(rows * qd * 4);
  w.mlp = take(rows * (size_t)c.intermediate * 4);
  w.logits = take(B * (size_t)c.vocab * 4);
  const size_t qv_stride = (size_t)kMaxRows * (c.n_q_heads / c.n_kv_heads);
  w.part_o = take(B * c.n_kv_heads * splits * qv_stride * hd * 4);
  w.part_ml = take(B * c.n_kv_heads * splits * qv_stride * 2 * 4);
  w.amax = take(B * 8);
  w.tokens = take(B * S * 4);
  w.emitted = take((size_t)kMaxTau * B * 4);
  w.forced = take((size_t)kMaxTau * B * 4);
  w.state = take(256);
  w.inv_freq = take((hd / 2) * 8);
  w.scratch_f32 = take(256);
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

// ------------------------------------------------------------------ launch helpers

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

// bf16 models, 2..16 rows: the MFMA kernel (weights are read once for up to 16 rows)
template <int EPI, bool NORM>
hipError_t launch_gemv_mfma(dmtd_ctx* c, const GemvArgs& a, int m) {
  const int KS = a.K / 64;
  const int nw = (KS + kMfmaPF - 1) / kMfmaPF;
  const int mats = EPI == EPI_SWIGLU ? 2 : 1;
  hipLaunchKernelGGL((gemv_mfma_kernel<EPI, NORM, kMfmaPF>), dim3((a.N + 15) / 16), dim3(64 * nw * mats), 0, c->stream, a, m, nw);
  return hipGetLastError();
}

template <typename WT, int EPI, bool NORM>
hipError_t gemv_rows(dmtd_ctx* c, GemvArgs a, int rows) {
  if constexpr (std::is_same<WT, bf16_t>::value && EPI != EPI_LOGITS) {
    const int nw = (a.K / 64 + kMfmaPF - 1) / kMfmaPF;
    if (rows >= 2 && a.K % 64 == 0 && nw * (EPI == EPI_SWIGLU ? 2 : 1) <= MFMA_MAX_WAVES) {
      for (int m0 = 0; m0 < rows; m0 += kMfmaRows) {
        GemvArgs g = a;
        g.x = a.x + (size_t)m0 * a.ldx;
        g.y = a.y + (size_t)m0 * a.ldy;
        hipError_t e = launch_gemv_mfma<EPI, NORM>(c, g, rows - m0 < kMfmaRows ? rows - m0 : kMfmaRows);
        if (e != hipSuccess) return e;
      }
      return hipSuccess;
    }
  }
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

template <typename WT, int HD, int QVT>
void launch_attention_t(dmtd_ctx* c, int l, const float* qkv, float* attn, int sel, int offset, int r) {
  const dmtd_config& cf = c->cfg;
  const int B = c->batch, nqkv = (cf.n_q_heads + 2 * cf.n_kv_heads) * HD, qd = cf.n_q_heads * HD;
  const int gq = cf.n_q_heads / cf.n_kv_heads, rpb = QVT / gq, n_rg = (r + rpb - 1) / rpb;
  const WT* kc = (const WT*)(c->ws + c->o.kv + (size_t)l * c->o.kv_layer_stride);
  const WT* vc = (const WT*)(c->ws + c->o.kv + (size_t)l * c->o.kv_layer_stride + c->o.kv_v_off);
  // enough splits to put about two blocks on every CU, whatever the batch
  int ns = 2 * c->num_cus / (cf.n_kv_heads * B * n_rg);
  if (ns > ATT_MAX_SPLITS) ns = ATT_MAX_SPLITS;
  if (ns < 1) ns = 1;
  float* po = (float*)(c->ws + c->o.part_o);
  float* pml = (float*)(c->ws + c->o.part_ml);
  const DevState* st = (const DevState*)(c->ws + c->o.state);
  hipLaunchKernelGGL((attn_decode_kernel<WT, HD, QVT>), dim3(ns * n_rg, cf.n_kv_heads, B), dim3(256), 0, c->stream, qkv, nqkv,
                     kc, vc, po, pml, cf.n_q_heads, cf.n_kv_heads, cf.max_seq_len, ns, kMaxRows * gq, st, sel, offset, r);
  hipLaunchKernelGGL((attn_merge_kernel<HD>), dim3(r, cf.n_kv_heads, B), dim3(256), 0, c->stream, po, pml, attn, qd,
                     cf.n_q_heads, cf.n_kv_heads, ns, kMaxRows * gq, st, sel, offset, r);
}

// share_kv: all rows of a sequence go through one block so that K and V are read once
// (long contexts); otherwise rows are spread over blocks (short contexts, K/V re-reads hit in L2).
template <typename WT>
hipError_t launch_attention(dmtd_ctx* c, int l, const float* qkv, float* attn, int sel, int offset, int r, bool share_kv) {
  const dmtd_config& cf = c->cfg;
  const int gq = cf.n_q_heads / cf.n_kv_heads;
  if (r > kMaxRows) return hipErrorInvalidValue;
  const int want = share_kv ? r * gq : gq;
  const int qvt = want <= 4 ? 4 : (want <= 8 ? 8 : 16);
  if (cf.head_dim == 128) {
    if (qvt == 4) launch_attention_t<WT, 128, 4>(c, l, qkv, attn, sel, offset, r);
    else if (qvt == 8) launch_attention_t<WT, 128, 8>(c, l, qkv, attn, sel, offset, r);
    else launch_attention_t<WT, 128, 16>(c, l, qkv, attn, sel, offset, r);
  } else {
    if (qvt == 4) launch_attention_t<WT, 64, 4>(c, l, qkv, attn, sel, offset, r);
    else if (qvt == 8) launch_attention_t<WT, 64, 8>(c, l, qkv, attn, sel, offset, r);
    else launch_attention_t<WT, 64, 16>(c, l, qkv, attn, sel, offset, r);
  }
  return hipGetLastError();
}

template <typename WT>
hipError_t run_layers(dmtd_ctx* c, int l0, int l1, float* h, int r, int sel, int explicit_pos,
                      int add_embed_at /* layer before which the embedding is re-added, or -1 */) {
  const dmtd_config& cf = c->cfg;
  const int B = c->batch, rows = B * r, d = cf.hidden, hd = cf.head_dim;
  const int nqkv = (cf.n_q_heads + 2 * cf.n_kv_heads) * hd, qd = cf.n_q_heads * hd;
  float* qkv = (float*)(c->ws + c->o.qkv);
  float* attn = (float*)(c->ws + c->o.attn);
  float* mlp = (float*)(c->ws + c->o.mlp);
  const DevState* st = (const DevState*)(c->ws + c->o.state);
  const int* tokens = (const int*)(c->ws + c->o.tokens);
  hipError_t e;
  for (int l = l0; l < l1; ++l) {
    const LayerW& w = c->layers[l];
    if (l == add_embed_at)
      hipLaunchKernelGGL(add_embed_rows_kernel<WT>, dim3(rows), dim3(256), 0, c->stream, h, (const WT*)c->embed, tokens,
                         cf.max_seq_len, st, sel, explicit_pos, r, d);
    WT* kc = (WT*)(c->ws + c->o.kv + (size_t)l * c->o.kv_layer_stride);
    WT* vc = (WT*)(c->ws + c->o.kv + (size_t)l * c->o.kv_layer_stride + c->o.kv_v_off);
    GemvArgs a{};
    a.eps = cf.rms_eps;
    // a2: RMSNorm + fused QKV projection (q, k, v are contiguous in the blob)
    a.W = w.q; a.gain = w.attn_norm; a.x = h; a.ldx = d; a.y = qkv; a.ldy = nqkv; a.N = nqkv; a.K = d;
    if ((e = gemv_rows<WT, EPI_STORE, true>(c, a, rows)) != hipSuccess) return e;
    // a3: QK-RMSNorm + RoPE + KV append
    hipLaunchKernelGGL(qk_norm_rope_append_kernel<WT>, dim3(cf.n_q_heads + 2 * cf.n_kv_heads, rows), dim3(64), 0, c->stream,
                       qkv, nqkv, w.q_norm, w.k_norm, (const double*)(c->ws + c->o.inv_freq), kc, vc, cf.n_q_heads,
                       cf.n_kv_heads, hd, cf.max_seq_len, cf.rms_eps, st, sel, explicit_pos, r);
    // a4: split-K GQA attention + merge
    if ((e = launch_attention<WT>(c, l, qkv, attn, sel, explicit_pos, r, c->share_kv)) != hipSuccess) return e;
    // a5: O projection + residual
    a = GemvArgs{};
    a.W = w.o; a.x = attn; a.ldx = qd; a.y = h; a.ldy = d; a.N = d; a.K = qd;
    if ((e = gemv_rows<WT, EPI_RESID, false>(c, a, rows)) != hipSuccess) return e;
    // a6: RMSNorm + gate/up + SwiGLU
    a = GemvArgs{};
    a.eps = cf.rms_eps;
    a.W = w.gate; a.W2 = w.up; a.gain = w.mlp_norm; a.x = h; a.ldx = d; a.y = mlp; a.ldy = cf.intermediate;
    a.N = cf.intermediate; a.K = d;
    if ((e = gemv_rows<WT, EPI_SWIGLU, true>(c, a, rows)) != hipSuccess) return e;
    // a7: down projection + residual
    a = GemvArgs{};
    a.W = w.down; a.x = mlp; a.ldx = cf.intermediate; a.y = h; a.ldy = d; a.N = d; a.K = cf.intermediate;
    if ((e = gemv_rows<WT, EPI_RESID, false>(c, a, rows)) != hipSuccess) return e;
  }
  return hipGetLastError();
}

// a9: final RMSNorm + LM head + greedy argmax for the batch rows in h_late; then advance the device state
template <typename WT>
hipError_t run_head(dmtd_ctx* c, const float* h_rows, int full) {
  const dmtd_config& cf = c->cfg;
  GemvArgs a{};
  a.eps = cf.rms_eps;
  a.W = c->lm_head; a.gain = c->final_norm; a.x = h_rows; a.ldx = cf.hidden;
  a.y = (float*)(c->ws + c->o.logits); a.ldy = cf.vocab; a.N = cf.vocab; a.K = cf.hidden;
  a.amax = (unsigned long long*)(c->ws + c->o.amax);
  hipError_t e = gemv_rows<WT, EPI_LOGITS, true>(c, a, c->batch);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(finish_step_kernel, dim3(1), dim3(64), 0, c->stream, (DevState*)(c->ws + c->o.state),
                     (unsigned long long*)(c->ws + c->o.amax), (int*)(c->ws + c->o.tokens), (int*)(c->ws + c->o.emitted),
                     cf.max_seq_len, c->batch, full, 1);
  return hipGetLastError();
}

// One decode step (Sec. 2.2).  Full: embed the pending rows and the newest row, run the front
// layers on all of them, keep the newest row, run the late layers on it.  Late: embed the
// newest token and run the late layers only (Eq. 4, m = 0).
template <typename WT>
hipError_t enqueue_step(dmtd_ctx* c, bool full, int r, int n_late) {
  const dmtd_config& cf = c->cfg;
  const int B = c->batch, d = cf.hidden, F = cf.n_layers - n_late;
  float* h = (float*)(c->ws + c->o.h);
  float* h_late = (float*)(c->ws + c->o.h_late);
  const DevState* st = (const DevState*)(c->ws + c->o.state);
  const int* tokens = (const int*)(c->ws + c->o.tokens);
  hipError_t e;
  if (full) {
    // the pending rows are causal among themselves, so groups of rows may pass the front
    // layers one after another (each group streams those layers' weights once)
    int c0 = 0, rc = 0;
    for (; c0 < r; c0 += rc) {
      rc = r - c0 < c->max_rows ? r - c0 : c->max_rows;
      hipLaunchKernelGGL(embed_kernel<WT>, dim3(B * rc), dim3(256), 0, c->stream, (const WT*)c->embed, tokens,
                         cf.max_seq_len, st, (int)POS_NFRONT, c0, rc, d, h);
      if ((e = run_layers<WT>(c, 0, F, h, rc, POS_NFRONT, c0, -1)) != hipSuccess) return e;
    }
    hipLaunchKernelGGL(take_last_rows_kernel<WT>, dim3(B), dim3(256), 0, c->stream, h, h_late, rc, d,
                       cf.full_pos_add_embed ? 1 : 0, (const WT*)c->embed, tokens, cf.max_seq_len, st, (int)POS_NFRONT,
                       c0 - rc);
  } else {
    hipLaunchKernelGGL(embed_kernel<WT>, dim3(B), dim3(256), 0, c->stream, (const WT*)c->embed, tokens, cf.max_seq_len, st,
                       (int)POS_NTOK, 0, 1, d, h_late);
  }
  if ((e = run_layers<WT>(c, F, cf.n_layers, h_late, 1, POS_NTOK, 0, -1)) != hipSuccess) return e;
  return run_head<WT>(c, h_late, full ? 1 : 0);
}

hipError_t enqueue_step_any(dmtd_ctx* c, bool full, int r, int n_late) {
  return c->cfg.dtype == DMTD_DTYPE_F32 ? enqueue_step<float>(c, full, r, n_late)
                                        : enqueue_step<bf16_t>(c, full, r, n_late);
}

// K/V bytes one layer's attention reads for the whole batch at context length ctx
bool kv_is_large(const dmtd_ctx* c, int ctx) {
  const size_t bytes = (size_t)c->batch * ctx * c->cfg.n_kv_heads * c->cfg.head_dim * 2 * c->elem;
  return bytes > ((size_t)48 << 20);
}

int run_step(dmtd_ctx* c, const Step& s, int n_late) {
  c->share_kv = kv_is_large(c, s.pos + 1);
  if (!c->cfg.use_graphs) {
    HIP_TRY(c, enqueue_step_any(c, s.full, s.rows, n_late));
    return DMTD_OK;
  }
  const auto key = std::make_tuple(s.full ? 1 : 0, s.rows, n_late, c->share_kv ? 1 : 0);
  auto it = c->graphs.find(key);
  if (it == c->graphs.end()) {
    hipGraph_t graph = nullptr;
    HIP_TRY(c, hipStreamBeginCapture(c->stream, hipStreamCaptureModeThreadLocal));
    hipError_t e = enqueue_step_any(c, s.full, s.rows, n_late);
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

template <typename WT>
hipError_t enqueue_prefill(dmtd_ctx* c, int P, int n_late) {
  const dmtd_config& cf = c->cfg;
  const int B = c->batch, d = cf.hidden;
  float* h = (float*)(c->ws + c->o.h);
  float* h_late = (float*)(c->ws + c->o.h_late);
  DevState* st = (DevState*)(c->ws + c->o.state);
  const int* tokens = (const int*)(c->ws + c->o.tokens);
  const int chunk = c->max_rows < kPrefillChunk ? c->max_rows : kPrefillChunk;
  const int add_at = cf.full_pos_add_embed ? cf.n_layers - n_late : -1;
  hipError_t e;
  hipLaunchKernelGGL(set_state_kernel, dim3(1), dim3(1), 0, c->stream, st, P - 1, P - 1);
  int r_last = 0;
  for (int p0 = 0; p0 < P; p0 += chunk) {
    const int r = P - p0 < chunk ? P - p0 : chunk;
    c->share_kv = kv_is_large(c, p0 + r);
    hipLaunchKernelGGL(embed_kernel<WT>, dim3(B * r), dim3(256), 0, c->stream, (const WT*)c->embed, tokens, cf.max_seq_len,
                       st, (int)POS_EXPLICIT, p0, r, d, h);
    if ((e = run_layers<WT>(c, 0, cf.n_layers, h, r, POS_EXPLICIT, p0, add_at)) != hipSuccess) return e;
    r_last = r;
  }
  hipLaunchKernelGGL(take_last_rows_kernel<WT>, dim3(B), dim3(256), 0, c->stream, h, h_late, r_last, d, 0,
                     (const WT*)c->embed, tokens, cf.max_seq_len, st, (int)POS_EXPLICIT, 0);
  return run_head<WT>(c, h_late, 1);   // state goes from P-1 to n_tok = n_front = P
}

// One launch of one kernel kind on layer l, for dmtd_time_kernel.  Outputs go to scratch
// buffers only: the QKV/attention/MLP activations, the residual scratch h (never h_late,
// never the caches, the token history or the scheduler state).
template <typename WT>
hipError_t time_one(dmtd_ctx* c, int kind, int l, int rows) {
  const dmtd_config& cf = c->cfg;
  const int d = cf.hidden, hd = cf.head_dim;
  const int nqkv = (cf.n_q_heads + 2 * cf.n_kv_heads) * hd, qd = cf.n_q_heads * hd;
  float* h = (float*)(c->ws + c->o.h);
  float* qkv = (float*)(c->ws + c->o.qkv);
  float* attn = (float*)(c->ws + c->o.attn);
  float* mlp = (float*)(c->ws + c->o.mlp);
  const LayerW& w = c->layers[l];
  GemvArgs a{};
  a.eps = cf.rms_eps;
  switch (kind) {
    case DMTD_K_QKV:
      a.W = w.q; a.gain = w.attn_norm; a.x = h; a.ldx = d; a.y = qkv; a.ldy = nqkv; a.N = nqkv; a.K = d;
      return gemv_rows<WT, EPI_STORE, true>(c, a, rows);
    case DMTD_K_OPROJ:
      a.W = w.o; a.x = attn; a.ldx = qd; a.y = h; a.ldy = d; a.N = d; a.K = qd;
      return gemv_rows<WT, EPI_RESID, false>(c, a, rows);
    case DMTD_K_GATEUP:
      a.W = w.gate; a.W2 = w.up; a.gain = w.mlp_norm; a.x = h; a.ldx = d; a.y = mlp; a.ldy = cf.intermediate;
      a.N = cf.intermediate; a.K = d;
      return gemv_rows<WT, EPI_SWIGLU, true>(c, a, rows);
    case DMTD_K_DOWN:
      a.W = w.down; a.x = mlp; a.ldx = cf.intermediate; a.y = h; a.ldy = d; a.N = d; a.K = cf.intermediate;
      return gemv_rows<WT, EPI_RESID, false>(c, a, rows);
    case DMTD_K_LMHEAD: {
      // the real LM-head kernel (logits + argmax); a null token history suppresses its token side effects
      a.W = c->lm_head; a.gain = c->final_norm; a.x = h; a.ldx = d; a.y = (float*)(c->ws + c->o.logits); a.ldy = cf.vocab;
      a.N = cf.vocab; a.K = d;
      a.amax = (unsigned long long*)(c->ws + c->o.amax);
      {
        hipError_t e = gemv_rows<WT, EPI_LOGITS, true>(c, a, rows);
        if (e != hipSuccess) return e;
        // clear the selection keys again without touching tokens or state
        hipLaunchKernelGGL(finish_step_kernel, dim3(1), dim3(64), 0, c->stream, (DevState*)(c->ws + c->o.state),
                           (unsigned long long*)(c->ws + c->o.amax), (int*)nullptr, (int*)nullptr, cf.max_seq_len, rows, 0, 0);
        return hipGetLastError();
      }

    }
    default: {
      // attention for `rows` query rows per sequence ending at the newest cached position
      const int last = c->sched.n_tok - 1;
      const int r = rows <= last + 1 ? rows : 1;
      return launch_attention<WT>(c, l, qkv, attn, (int)POS_EXPLICIT, last - r + 1, r, c->share_kv);
    }
  }
}

void destroy_graphs(dmtd_ctx* c) {
  for (auto& kv : c->graphs) (void)hipGraphExecDestroy(kv.second);
  c->graphs.clear();
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
  c->max_rows = rows_cap(*cfg);
  if (!cfg->dry_run) {
    c->wbase = (const char*)weights_dev;
    c->ws = (char*)workspace_dev;
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
    if (e == hipSuccess) e = hipMemsetAsync(c->ws + lay.amax, 0, (size_t)cfg->max_batch * 8, c->stream);
    if (e == hipSuccess) e = hipMemsetAsync(c->ws + lay.state, 0, 256, c->stream);
    if (e == hipSuccess) e = hipMemsetAsync(c->ws + lay.kv, 0, lay.kv_layer_stride * cfg->n_layers, c->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
    if (e != hipSuccess) { g_create_error = std::string("workspace setup: ") + hipGetErrorString(e); delete c; return DMTD_EHIP; }
  }
  *out = c;
  return DMTD_OK;
}

int dmtd_prefill(dmtd_ctx* c, const int32_t* tokens, int32_t batch, int32_t prompt_len, int32_t n_late, int32_t* first_tokens) {
  if (!c) return DMTD_EINVAL;
  const dmtd_config& cf = c->cfg;
  if (!tokens) { c->err = "null tokens"; return DMTD_EINVAL; }
  if (batch < 1 || batch > cf.max_batch) { c->err = "batch outside [1, max_batch]"; return DMTD_EINVAL; }
  if (prompt_len < 1) { c->err = "prompt_len must be >= 1"; return DMTD_EINVAL; }
  if (cf.full_pos_add_embed && (n_late < 1 || n_late > cf.n_layers)) { c->err = "the literal Eq. 4 reading needs n_late at prefill"; return DMTD_EINVAL; }
  if (c->sched.n_tok != 0) { c->err = "already prefilled; call dmtd_reset first"; return DMTD_ESTATE; }
  if (prompt_len >= cf.max_seq_len) { c->err = "prompt does not leave room for a generated token"; return DMTD_ECAPACITY; }
  for (size_t i = 0; i < (size_t)batch * prompt_len; ++i)
    if (tokens[i] < 0 || tokens[i] >= cf.vocab) { c->err = "token id outside the vocabulary"; return DMTD_EINVAL; }
  c->batch = batch;
  if (!cf.dry_run) {
    int* dtok = (int*)(c->ws + c->o.tokens);
    HIP_TRY(c, hipMemcpy2DAsync(dtok, (size_t)cf.max_seq_len * 4, tokens, (size_t)prompt_len * 4, (size_t)prompt_len * 4, batch,
                                hipMemcpyHostToDevice, c->stream));
    HIP_TRY(c, cf.dtype == DMTD_DTYPE_F32 ? enqueue_prefill<float>(c, prompt_len, n_late) : enqueue_prefill<bf16_t>(c, prompt_len, n_late));
    std::vector<int32_t> first(batch);
    HIP_TRY(c, hipMemcpyAsync(first.data(), c->ws + c->o.emitted, (size_t)batch * 4, hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    if (first_tokens) std::memcpy(first_tokens, first.data(), (size_t)batch * 4);
    c->have_logits = true;
  } else if (first_tokens) {
    for (int b = 0; b < batch; ++b) first_tokens[b] = -1;
  }
  c->sched.note_prefill(prompt_len, cf.full_pos_add_embed ? n_late : 0);
  return DMTD_OK;
}

int dmtd_decode_cycle(dmtd_ctx* c, int32_t tau, int32_t n_late, int32_t max_new, const int32_t* forced_inputs,
                      int32_t n_forced, int32_t* out_tokens, int32_t out_stride, int32_t* n_emitted) {
  if (!c) return DMTD_EINVAL;
  const dmtd_config& cf = c->cfg;
  if (n_emitted) *n_emitted = 0;
  if (!out_tokens || !n_emitted) { c->err = "null output pointer"; return DMTD_EINVAL; }
  if (tau > kMaxTau) { c->err = "tau above the supported maximum (64)"; return DMTD_EINVAL; }
  if (forced_inputs && n_forced < 1) { c->err = "forced_inputs given with n_forced < 1"; return DMTD_EINVAL; }
  const int f_stride = forced_inputs ? n_forced : 0;
  std::vector<Step> steps;
  int err = 0;
  std::string why;
  if (!c->sched.plan(tau, n_late, max_new, kMaxTau, steps, err, why)) {
    c->err = why;
    return err == 1 ? DMTD_EINVAL : (err == 2 ? DMTD_ESTATE : DMTD_ECAPACITY);
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
                       (int*)(c->ws + c->o.tokens), cf.max_seq_len, fdev, nf, B);
    HIP_TRY(c, hipGetLastError());
    for (const Step& s : steps) {
      const int rc = run_step(c, s, n_late);
      if (rc != DMTD_OK) {
        // device state may be ahead of the host's; resynchronise it to the host's unchanged view
        (void)hipStreamSynchronize(c->stream);
        hipLaunchKernelGGL(set_state_kernel, dim3(1), dim3(1), 0, c->stream, (DevState*)(c->ws + c->o.state),
                           c->sched.n_tok, c->sched.n_front);
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
  if (!avg_us || kind < 0 || kind > DMTD_K_ATTN || rows < 1 || rows > kMaxRows || reps < 1) {
    c->err = "bad argument to dmtd_time_kernel"; return DMTD_EINVAL;
  }
  if (c->cfg.dry_run || c->sched.n_tok == 0) { c->err = "dmtd_time_kernel needs a prefilled context"; return DMTD_ESTATE; }
  if (kind == DMTD_K_ATTN && rows > c->max_rows) { c->err = "too many rows for the attention kernel"; return DMTD_EINVAL; }
  if (kind == DMTD_K_LMHEAD && rows > c->batch) { c->err = "the LM head carries one row per sequence"; return DMTD_EINVAL; }
  hipEvent_t e0, e1;
  HIP_TRY(c, hipEventCreate(&e0));
  HIP_TRY(c, hipEventCreate(&e1));
  const bool f32 = c->cfg.dtype == DMTD_DTYPE_F32;
  // rows is per sequence for attention, total activation rows for the projections
  const int saved_batch = c->batch;
  long launches = 0;
  hipError_t e = hipSuccess;
  for (int pass = 0; pass < 2 && e == hipSuccess; ++pass) {   // pass 0 warms up (one repetition)
    const int n = pass == 0 ? 1 : reps;
    if (pass == 1) e = hipEventRecord(e0, c->stream);
    for (int i = 0; i < n && e == hipSuccess; ++i) {
      if (kind == DMTD_K_LMHEAD) {
        e = f32 ? time_one<float>(c, kind, 0, rows) : time_one<bf16_t>(c, kind, 0, rows);
        if (pass == 1) launches += 1;
      } else {
        for (int l = 0; l < c->cfg.n_layers && e == hipSuccess; ++l) {
          e = f32 ? time_one<float>(c, kind, l, rows) : time_one<bf16_t>(c, kind, l, rows);
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

int dmtd_reset(dmtd_ctx* c) {
  if (!c) return DMTD_EINVAL;
  if (!c->cfg.dry_run) {
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    hipLaunchKernelGGL(set_state_kernel, dim3(1), dim3(1), 0, c->stream, (DevState*)(c->ws + c->o.state), 0, 0);
    HIP_TRY(c, hipGetLastError());
    HIP_TRY(c, hipStreamSynchronize(c->stream));
  }
  c->sched.reset();
  c->batch = 0;
  c->have_logits = false;
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
