"""Thin ctypes binding of the C ABI in ``include/dmtd.h``.

Argument marshalling only: every step of the decode path runs in the HIP library.
PyTorch is used for device memory (the weight blob and the workspace) and for the
stream handle.  There is no CPU fallback: if ``libdmtd.so`` has not been built the
import of the library fails with an error.
"""
from __future__ import annotations

import ctypes as C
import dataclasses
import os

import numpy as np

DMTD_OK, DMTD_EINVAL, DMTD_ESTATE, DMTD_ECAPACITY, DMTD_EHIP = 0, -1, -2, -3, -4
_CODES = {DMTD_EINVAL: "DMTD_EINVAL", DMTD_ESTATE: "DMTD_ESTATE", DMTD_ECAPACITY: "DMTD_ECAPACITY", DMTD_EHIP: "DMTD_EHIP"}

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libdmtd.so")


class _Config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "hidden", "n_q_heads", "n_kv_heads", "head_dim", "intermediate", "vocab")] + [
        ("rms_eps", C.c_float), ("rope_theta", C.c_float),
        ("tied_embeddings", C.c_int32), ("dtype", C.c_int32), ("max_batch", C.c_int32), ("max_seq_len", C.c_int32),
        ("full_pos_add_embed", C.c_int32), ("use_graphs", C.c_int32), ("dry_run", C.c_int32), ("stream", C.c_void_p)]


class DmtdError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"{_CODES.get(code, code)}: {msg}")
        self.code = code


_lib = None


def load_library():
    """Load ``libdmtd.so`` and declare the prototypes of every exported call."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is missing: build it first (python -m paper_2510_11958_amd.build); "
                          "there is no fallback path")
    # PyTorch ships its own HIP runtime: load it first, so that the library binds to the runtime that owns the
    # device memory it is handed (loading the system runtime first leaves the process with two of them)
    import torch  # noqa: F401
    lib = C.CDLL(_LIB_PATH)
    P = C.POINTER
    lib.dmtd_workspace_bytes.restype = C.c_size_t
    lib.dmtd_workspace_bytes.argtypes = [P(_Config)]
    lib.dmtd_create.restype = C.c_int
    lib.dmtd_create.argtypes = [P(_Config), C.c_void_p, C.c_size_t, C.c_void_p, C.c_size_t, P(C.c_void_p)]
    lib.dmtd_prefill.restype = C.c_int
    lib.dmtd_prefill.argtypes = [C.c_void_p, P(C.c_int32), C.c_int32, C.c_int32, C.c_int32, P(C.c_int32)]
    lib.dmtd_prefill_ragged.restype = C.c_int
    lib.dmtd_prefill_ragged.argtypes = [C.c_void_p, P(C.c_int32), C.c_int32, C.c_int32, P(C.c_int32), C.c_int32, P(C.c_int32)]
    lib.dmtd_decode_cycle.restype = C.c_int
    lib.dmtd_decode_cycle.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, P(C.c_int32), C.c_int32,
                                      P(C.c_int32), C.c_int32, P(C.c_int32)]
    lib.dmtd_decode.restype = C.c_int
    lib.dmtd_decode.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, P(C.c_int32), C.c_int32,
                                P(C.c_int32), C.c_int32, P(C.c_int32)]
    lib.dmtd_decode_per_seq.restype = C.c_int
    lib.dmtd_decode_per_seq.argtypes = [C.c_void_p, P(C.c_int32), C.c_int32, C.c_int32, P(C.c_int32), C.c_int32,
                                        P(C.c_int32), C.c_int32, P(C.c_int32)]
    lib.dmtd_get_seq_state.restype = C.c_int
    lib.dmtd_get_seq_state.argtypes = [C.c_void_p, C.c_int32, P(C.c_int32), P(C.c_int32)]
    lib.dmtd_decode_cycle_noalloc.restype = C.c_int
    lib.dmtd_decode_cycle_noalloc.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_int32,
                                              C.c_void_p, C.c_int32, P(C.c_int32)]
    lib.dmtd_logits.restype = C.c_int
    lib.dmtd_logits.argtypes = [C.c_void_p, P(C.c_float), C.c_size_t]
    lib.dmtd_get_state.restype = C.c_int
    lib.dmtd_get_state.argtypes = [C.c_void_p, P(C.c_int32), P(C.c_int32), P(C.c_int32), P(C.c_int64)]
    lib.dmtd_get_trace.restype = C.c_int
    lib.dmtd_get_trace.argtypes = [C.c_void_p, P(C.c_int32), C.c_int32, P(C.c_int32)]
    lib.dmtd_read_kv.restype = C.c_int
    lib.dmtd_read_kv.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, P(C.c_float), C.c_size_t]
    lib.dmtd_time_kernel.restype = C.c_int
    lib.dmtd_time_kernel.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, P(C.c_float)]
    lib.dmtd_set_n_early.restype = C.c_int
    lib.dmtd_set_n_early.argtypes = [C.c_void_p, C.c_int32]
    lib.dmtd_set_sampling.restype = C.c_int
    lib.dmtd_set_sampling.argtypes = [C.c_void_p, C.c_float, C.c_int32, C.c_uint64]
    lib.dmtd_masked_forward.restype = C.c_int
    lib.dmtd_masked_forward.argtypes = [C.c_void_p, P(C.c_int32), C.c_int32, C.c_int32, P(C.c_uint8), C.c_int32, P(C.c_float),
                                        P(C.c_int32), P(C.c_float), C.c_size_t, P(C.c_float)]
    lib.dmtd_reset.restype = C.c_int
    lib.dmtd_reset.argtypes = [C.c_void_p]
    lib.dmtd_destroy.restype = None
    lib.dmtd_destroy.argtypes = [C.c_void_p]
    lib.dmtd_last_error.restype = C.c_char_p
    lib.dmtd_last_error.argtypes = [C.c_void_p]
    _lib = lib
    return lib


@dataclasses.dataclass
class ModelConfig:
    n_layers: int
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    intermediate: int
    vocab: int
    dtype: str = "bf16"
    rms_eps: float = 1e-6
    rope_theta: float = 1e6
    tied_embeddings: bool = True
    max_batch: int = 1
    max_seq_len: int = 2048
    full_pos_add_embed: bool = False
    use_graphs: bool = True
    dry_run: bool = False

    def to_c(self, stream: int = 0) -> _Config:
        return _Config(self.n_layers, self.hidden, self.n_q_heads, self.n_kv_heads, self.head_dim, self.intermediate,
                       self.vocab, self.rms_eps, self.rope_theta, int(self.tied_embeddings),
                       0 if self.dtype == "fp32" else 1, self.max_batch, self.max_seq_len,
                       int(self.full_pos_add_embed), int(self.use_graphs), int(self.dry_run), stream or None)


def _i32p(a: np.ndarray):
    return a.ctypes.data_as(C.POINTER(C.c_int32))


class Engine:
    """One decoding context.  ``weights`` is the flat weight blob (NumPy float32, or uint16 holding
    bfloat16 bits, or a torch uint8/any-dtype CUDA tensor already on the device)."""

    def __init__(self, cfg: ModelConfig, weights=None, stream: int | None = None):
        self.lib = load_library()
        self.cfg = cfg
        self._h = C.c_void_p()
        self._weights = self._workspace = None
        if cfg.dry_run:
            cc = cfg.to_c(0)
            rc = self.lib.dmtd_create(C.byref(cc), None, 0, None, 0, C.byref(self._h))
            self._check_create(rc)
            return
        import torch
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU: the DMTD decode path has no CPU fallback")
        if isinstance(weights, np.ndarray):
            weights = torch.from_numpy(weights.view(np.int16) if weights.dtype == np.uint16 else weights).cuda()
        self._weights = weights.contiguous()
        if stream is None:
            # a stream of its own (default priority): the legacy default stream cannot be captured into a graph
            self._stream = torch.cuda.Stream()
            stream = self._stream.cuda_stream
        torch.cuda.synchronize()   # the weight upload above ran on torch's current stream
        cc = cfg.to_c(stream)
        nbytes = self.lib.dmtd_workspace_bytes(C.byref(cc))
        if nbytes == 0:
            raise DmtdError(DMTD_EINVAL, "invalid configuration")
        self._workspace = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        wbytes = self._weights.numel() * self._weights.element_size()
        rc = self.lib.dmtd_create(C.byref(cc), self._weights.data_ptr(), wbytes, self._workspace.data_ptr(), nbytes,
                                  C.byref(self._h))
        self._check_create(rc)

    def _check_create(self, rc):
        if rc != DMTD_OK:
            raise DmtdError(rc, self.lib.dmtd_last_error(None).decode())

    def _check(self, rc):
        if rc != DMTD_OK:
            raise DmtdError(rc, self.lib.dmtd_last_error(self._h).decode())

    def close(self):
        if self._h:
            self.lib.dmtd_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def prefill(self, tokens, n_late: int = 0, lengths=None) -> np.ndarray:
        """``lengths`` (one per sequence): prompts of different lengths, each in the first entries of its row of ``tokens``."""
        t = np.ascontiguousarray(np.atleast_2d(np.asarray(tokens)), dtype=np.int32)
        first = np.empty(t.shape[0], np.int32)
        if lengths is None:
            self._check(self.lib.dmtd_prefill(self._h, _i32p(t), t.shape[0], t.shape[1], n_late, _i32p(first)))
        else:
            ln = np.ascontiguousarray(np.asarray(lengths), dtype=np.int32)
            if ln.shape != (t.shape[0],):
                raise ValueError("one length per sequence")
            self._check(self.lib.dmtd_prefill_ragged(self._h, _i32p(t), t.shape[0], t.shape[1], _i32p(ln), n_late, _i32p(first)))
        self._batch = t.shape[0]
        return first

    def decode_cycle(self, tau: int, n_late: int, max_new: int = 0, forced=None) -> np.ndarray:
        """Returns the argmax tokens of the steps run, ``[batch, n_steps]``."""
        B = getattr(self, "_batch", 1)
        stride = max(1, min(tau, 64))
        out = np.empty((B, stride), np.int32)
        n = C.c_int32(0)
        if forced is not None:
            f = np.ascontiguousarray(np.atleast_2d(np.asarray(forced)), dtype=np.int32)
            fp, nf = _i32p(f), f.shape[1]
        else:
            fp, nf = None, 0
        self._check(self.lib.dmtd_decode_cycle(self._h, tau, n_late, max_new, fp, nf, _i32p(out), stride, C.byref(n)))
        return out[:, :n.value].copy()

    def decode(self, tau: int, n_late: int, n_steps: int, forced=None) -> np.ndarray:
        """``n_steps`` decode steps, cycles back to back, one host synchronisation; ``[batch, n_steps]`` argmax tokens."""
        B = getattr(self, "_batch", 1)
        stride = max(1, min(n_steps, 64))
        out = np.empty((B, stride), np.int32)
        n = C.c_int32(0)
        if forced is not None:
            f = np.ascontiguousarray(np.atleast_2d(np.asarray(forced)), dtype=np.int32)
            fp, nf = _i32p(f), f.shape[1]
        else:
            fp, nf = None, 0
        self._check(self.lib.dmtd_decode(self._h, tau, n_late, n_steps, fp, nf, _i32p(out), stride, C.byref(n)))
        return out[:, :n.value].copy()

    def decode_per_seq(self, taus, n_late: int, n_steps: int, forced=None) -> np.ndarray:
        """``n_steps`` decode steps with one cycle length per sequence (``taus``); ``[batch, n_steps]`` argmax tokens."""
        B = getattr(self, "_batch", 1)
        t = np.ascontiguousarray(np.asarray(taus), dtype=np.int32)
        if t.shape != (B,):
            raise ValueError("one cycle length per sequence")
        stride = max(1, min(n_steps, 64))
        out = np.empty((B, stride), np.int32)
        n = C.c_int32(0)
        if forced is not None:
            f = np.ascontiguousarray(np.atleast_2d(np.asarray(forced)), dtype=np.int32)
            fp, nf = _i32p(f), f.shape[1]
        else:
            fp, nf = None, 0
        self._check(self.lib.dmtd_decode_per_seq(self._h, _i32p(t), n_late, n_steps, fp, nf, _i32p(out), stride, C.byref(n)))
        return out[:, :n.value].copy()

    def seq_state(self, b: int):
        f, ph = C.c_int32(), C.c_int32()
        self._check(self.lib.dmtd_get_seq_state(self._h, b, C.byref(f), C.byref(ph)))
        return {"n_front": f.value, "phase": ph.value}

    def decode_cycle_noalloc(self, tau: int, n_late: int, out_dev, max_new: int = 0, forced_dev=None) -> int:
        """dmtd_decode_cycle without allocation or synchronisation: ``out_dev`` (torch int32 CUDA tensor ``[batch, stride]``)
        receives the steps' tokens once the engine's stream has run the enqueued work, ``forced_dev`` (torch int32 CUDA
        tensor ``[batch, n_forced]`` or None) holds the forced inputs.  Returns the number of steps enqueued."""
        n = C.c_int32(0)
        if forced_dev is not None:
            assert forced_dev.is_cuda and forced_dev.dtype.itemsize == 4 and forced_dev.is_contiguous()
            fp, nf = forced_dev.data_ptr(), forced_dev.shape[1]
        else:
            fp, nf = None, 0
        assert out_dev.is_cuda and out_dev.dtype.itemsize == 4 and out_dev.is_contiguous()
        self._check(self.lib.dmtd_decode_cycle_noalloc(self._h, tau, n_late, max_new, fp, nf, out_dev.data_ptr(),
                                                       out_dev.shape[1], C.byref(n)))
        return n.value

    def synchronize(self):
        """Wait for the engine's stream (after calls that do not synchronise themselves)."""
        if getattr(self, "_stream", None) is not None:
            self._stream.synchronize()
        else:
            import torch
            torch.cuda.synchronize()

    def logits(self) -> np.ndarray:
        B = getattr(self, "_batch", 1)
        out = np.empty((B, self.cfg.vocab), np.float32)
        self._check(self.lib.dmtd_logits(self._h, out.ctypes.data_as(C.POINTER(C.c_float)), out.size))
        return out

    def state(self):
        a, b, c = C.c_int32(), C.c_int32(), C.c_int32()
        cnt = (C.c_int64 * 4)()
        self._check(self.lib.dmtd_get_state(self._h, C.byref(a), C.byref(b), C.byref(c), cnt))
        return {"n_tok": a.value, "n_front": b.value, "phase": c.value, "gen_layer_visits": cnt[0],
                "refill_layer_visits": cnt[1], "n_emitted": cnt[2], "n_full_steps": cnt[3]}

    def trace(self):
        n = C.c_int32()
        self._check(self.lib.dmtd_get_trace(self._h, None, 0, C.byref(n)))
        buf = np.empty((max(n.value, 1), 4), np.int32)
        self._check(self.lib.dmtd_get_trace(self._h, _i32p(buf), n.value, C.byref(n)))
        names = {0: "front", 1: "late", 2: "enc"}
        return [(int(p), names[int(g)], list(range(int(f), int(f) + int(c)))) for p, g, f, c in buf[:n.value]]

    def read_kv(self, layer: int, b: int, n_pos: int) -> np.ndarray:
        out = np.empty((2, self.cfg.n_kv_heads, n_pos, self.cfg.head_dim), np.float32)
        self._check(self.lib.dmtd_read_kv(self._h, layer, b, n_pos, out.ctypes.data_as(C.POINTER(C.c_float)), out.size))
        return out

    KERNEL_KINDS = {"qkv": 0, "oproj": 1, "gateup": 2, "down": 3, "lmhead": 4, "attn": 5,
                    "read_qkv": 6, "read_oproj": 7, "read_gateup": 8, "read_down": 9}

    def time_kernel(self, kind: str, rows: int = 1, reps: int = 5) -> float:
        """Average duration (microseconds) of one launch of a kernel kind, HIP-event timed on the engine's stream."""
        us = C.c_float()
        self._check(self.lib.dmtd_time_kernel(self._h, self.KERNEL_KINDS[kind], rows, reps, C.byref(us)))
        return us.value

    def set_n_early(self, n_early: int):
        """ExDy variant: in-cycle tokens also pass the first ``n_early`` layers (0 = plain method)."""
        self._check(self.lib.dmtd_set_n_early(self._h, int(n_early)))

    def set_sampling(self, temperature: float, top_k: int = 0, seed: int = 0):
        """Draw tokens from the tempered softmax over the top_k logits (temperature <= 0: greedy, the default)."""
        self._check(self.lib.dmtd_set_sampling(self._h, float(temperature), int(top_k), int(seed)))

    def masked_forward(self, tokens, mask, n_late: int, want_logits: bool = False) -> dict:
        """Whole-sequence masked forward (Eqs. 1-5) with the Eq. 6 loss; returns ``nll`` [batch, n], ``best`` [batch, n],
        ``loss`` [batch] and, if asked for, ``logits`` [batch, n, vocab]."""
        t = np.ascontiguousarray(np.atleast_2d(np.asarray(tokens)), dtype=np.int32)
        m = np.ascontiguousarray(np.asarray(mask), dtype=np.uint8)
        B, n = t.shape
        if m.shape != (n,):
            raise ValueError("mask must have one entry per position")
        nll = np.empty((B, n), np.float32)
        best = np.empty((B, n), np.int32)
        loss = np.empty(B, np.float32)
        logits = np.empty((B, n, self.cfg.vocab), np.float32) if want_logits else None
        fp = C.POINTER(C.c_float)
        self._check(self.lib.dmtd_masked_forward(
            self._h, _i32p(t), B, n, m.ctypes.data_as(C.POINTER(C.c_uint8)), n_late, nll.ctypes.data_as(fp), _i32p(best),
            logits.ctypes.data_as(fp) if want_logits else None, logits.size if want_logits else 0, loss.ctypes.data_as(fp)))
        out = {"nll": nll, "best": best, "loss": loss}
        if want_logits:
            out["logits"] = logits
        return out

    def reset(self):
        self._check(self.lib.dmtd_reset(self._h))
