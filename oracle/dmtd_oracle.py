"""CPU oracle for Direct Multi-Token Decoding (DMTD).  TEST INFRASTRUCTURE ONLY.

A plain, slow NumPy implementation of what the decode path computes: a Qwen3-style
decoder-only transformer driven by the paper's cycle schedule with cyclical KV
refilling (Sec. 2.2, Fig. 3).  Only tests, the smoke check and the benchmark's CPU
baseline may import this file; the product path never does, and this file imports
nothing from the product.  It shares no code with the HIP path.

Precision: float64 by default (weights are up-converted exactly from their stored
float32/bfloat16 values; no activation is rounded).  ``dtype=np.float32`` is offered
for the 4B-shaped models where 32 GB of float64 weights is impractical; tests bound
the difference between the two on small models.

DMTD is not an exact speed-up of ordinary decoding (tokens inside a cycle never pass
the front layers before they emit), so this oracle is the algorithm itself, step by
step, not a closed form.  Two independent formulations live here and are compared by
the tests: the incremental cache machine (:class:`DmtdOracle`) and the one-shot
masked forward of Eqs. 1-5 (:func:`masked_forward`).

Readings taken where the paper is silent or ambiguous (each also listed in the
design notes):
  * Transformer block: the paper only cites Qwen3; pre-norm residual block, RMSNorm,
    grouped-query attention with per-head RMSNorm on q and k applied before rotary
    embedding (half-split pairing), SwiGLU MLP, no biases, tied LM head.
  * Eq. 4 at full positions: default feeds the front layers' output unchanged
    (so tau=1 is ordinary decoding); ``full_pos_add_embed`` gives the literal
    ``h_emb + h_think`` form.
  * All prompt positions are full positions; cycles are anchored at the end of the
    prompt and the token emitted by prefill is the first token of cycle 1 (Sec. 2.2).
  * Refill rows are causal among themselves and carry their true absolute positions.
  * Greedy selection, lowest index among equal maxima.
  * ExDy variant (Sec. 2.1, last paragraph before Eq. 5; Sec. 3.3): with ``n_early = x`` the
    in-cycle positions feed the decoding layers the output of the first ``x`` (encoding)
    layers instead of the raw embedding; tokens inside a cycle run those ``x`` layers and
    then jump to the last ``y``; only the thinking layers in between are refilled, from the
    stored encoding outputs.  ``n_early = 0`` is the plain method.

Pins: the vanilla path is checked against the Hugging Face Qwen3 implementation and
against an independent brute-force recompute; the cycle machine against the one-shot
masked forward, the Fig. 3 walk-through and Eq. 7 (its ExDy form against cycles counted by hand);
the ExDy variant and the literal reading of Eq. 4 against the Hugging Face model where the
layers above them are made the identity.  Exact logit values for the seeded
benchmark models are printed nowhere in the paper: those values are **parity
unpinned** by the paper and rest on the pins above.
"""
from __future__ import annotations

import dataclasses
import math

import numpy as np


@dataclasses.dataclass
class OracleConfig:
    n_layers: int
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    intermediate: int
    vocab: int
    rms_eps: float = 1e-6
    rope_theta: float = 1e6
    tied_embeddings: bool = True
    full_pos_add_embed: bool = False  # literal Eq. 4 at full positions


# ----------------------------------------------------------------------------- weights

def _bf16_to_f32(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def unpack_weights(blob: np.ndarray, cfg: OracleConfig, dtype=np.float64) -> dict:
    """Split the flat weight blob into named arrays of ``dtype``.

    Blob order: token table ``[V, d]``; for each layer ``attn_norm[d]``, ``q[nh*hd, d]``,
    ``k[nkv*hd, d]``, ``v[nkv*hd, d]``, ``q_norm[hd]``, ``k_norm[hd]``, ``o[d, nh*hd]``,
    ``mlp_norm[d]``, ``gate[ff, d]``, ``up[ff, d]``, ``down[d, ff]``; ``final_norm[d]``;
    ``lm_head[V, d]`` if untied.  ``blob`` is float32, or uint16 holding bfloat16 bits.
    """
    c = cfg
    pos = 0

    def take(*dims):
        nonlocal pos
        n = int(np.prod(dims))
        raw = blob[pos:pos + n]
        pos += n
        val = _bf16_to_f32(raw) if blob.dtype == np.uint16 else raw
        return val.astype(dtype).reshape(dims)

    w = {"embed": take(c.vocab, c.hidden), "layers": []}
    for _ in range(c.n_layers):
        lw = {}
        lw["attn_norm"] = take(c.hidden)
        lw["q"] = take(c.n_q_heads * c.head_dim, c.hidden)
        lw["k"] = take(c.n_kv_heads * c.head_dim, c.hidden)
        lw["v"] = take(c.n_kv_heads * c.head_dim, c.hidden)
        lw["q_norm"] = take(c.head_dim)
        lw["k_norm"] = take(c.head_dim)
        lw["o"] = take(c.hidden, c.n_q_heads * c.head_dim)
        lw["mlp_norm"] = take(c.hidden)
        lw["gate"] = take(c.intermediate, c.hidden)
        lw["up"] = take(c.intermediate, c.hidden)
        lw["down"] = take(c.hidden, c.intermediate)
        w["layers"].append(lw)
    w["final_norm"] = take(c.hidden)
    w["lm_head"] = w["embed"] if c.tied_embeddings else take(c.vocab, c.hidden)
    if pos != blob.size:
        raise ValueError(f"weight blob has {blob.size} elements, the configuration needs {pos}")
    return w


# -------------------------------------------------------------------------- primitives

def rmsnorm(x: np.ndarray, gain: np.ndarray, eps: float) -> np.ndarray:
    """x * (mean(x^2) + eps)^(-1/2) * gain over the last axis."""
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * gain


def rope(x: np.ndarray, positions: np.ndarray, theta: float) -> np.ndarray:
    """Rotary embedding, half-split pairing.  ``x`` is ``[rows, heads, hd]``.

    Pair ``(i, i + hd/2)`` is rotated by the angle ``p * theta^(-2i/hd)``.
    """
    hd = x.shape[-1]
    half = hd // 2
    inv_freq = np.asarray(theta, dtype=np.float64) ** (-2.0 * np.arange(half, dtype=np.float64) / hd)
    ang = np.asarray(positions, dtype=np.float64)[:, None] * inv_freq[None, :]
    cos = np.cos(ang).astype(x.dtype)[:, None, :]
    sin = np.sin(ang).astype(x.dtype)[:, None, :]
    lo, hi = x[..., :half], x[..., half:]
    return np.concatenate([lo * cos - hi * sin, hi * cos + lo * sin], axis=-1)


def softmax_rows(s: np.ndarray) -> np.ndarray:
    """Softmax over the last axis with max subtraction; ``-inf`` entries get weight 0."""
    m = np.max(s, axis=-1, keepdims=True)
    e = np.exp(s - m)
    return e / np.sum(e, axis=-1, keepdims=True)


def silu(t: np.ndarray) -> np.ndarray:
    return t / (1.0 + np.exp(-t))


def causal_attention(q: np.ndarray, q_pos: np.ndarray, K: np.ndarray, V: np.ndarray) -> np.ndarray:
    """Grouped-query causal attention.

    ``q`` is ``[rows, nh, hd]`` with absolute positions ``q_pos``; ``K`` and ``V`` are
    ``[ctx, nkv, hd]`` holding positions ``0..ctx-1``.  Row ``i`` attends keys at
    positions ``<= q_pos[i]``.  Query head ``j`` reads KV head ``j // (nh // nkv)``.
    """
    rows, nh, hd = q.shape
    ctx, nkv, _ = K.shape
    group = nh // nkv
    out = np.empty_like(q)
    key_pos = np.arange(ctx)
    scale = 1.0 / math.sqrt(hd)
    step = 256  # rows evaluated together; rows are independent, this only bounds memory
    for r0 in range(0, rows, step):
        r1 = min(rows, r0 + step)
        hidden = key_pos[None, :] > np.asarray(q_pos[r0:r1])[:, None]
        for j in range(nh):
            g = j // group
            s = (q[r0:r1, j, :] @ K[:, g, :].T) * scale
            s = np.where(hidden, -np.inf, s)
            out[r0:r1, j, :] = softmax_rows(s) @ V[:, g, :]
    return out


def lm_logits(h: np.ndarray, w: dict, cfg: OracleConfig) -> np.ndarray:
    """Eq. 5's LM head: logits of the final-normed hidden state against the (tied) table."""
    return rmsnorm(h, w["final_norm"], cfg.rms_eps) @ w["lm_head"].T


def _project_qkv(lw: dict, X: np.ndarray, positions, cfg: OracleConfig):
    c = cfg
    rows = X.shape[0]
    xh = rmsnorm(X, lw["attn_norm"], c.rms_eps)
    q = (xh @ lw["q"].T).reshape(rows, c.n_q_heads, c.head_dim)
    k = (xh @ lw["k"].T).reshape(rows, c.n_kv_heads, c.head_dim)
    v = (xh @ lw["v"].T).reshape(rows, c.n_kv_heads, c.head_dim)
    q = rope(rmsnorm(q, lw["q_norm"], c.rms_eps), positions, c.rope_theta)
    k = rope(rmsnorm(k, lw["k_norm"], c.rms_eps), positions, c.rope_theta)
    return q, k, v


def _finish_block(lw: dict, X: np.ndarray, attn: np.ndarray, cfg: OracleConfig) -> np.ndarray:
    rows = X.shape[0]
    a = X + attn.reshape(rows, -1) @ lw["o"].T
    ah = rmsnorm(a, lw["mlp_norm"], cfg.rms_eps)
    return a + (silu(ah @ lw["gate"].T) * (ah @ lw["up"].T)) @ lw["down"].T


def block_full_sequence(lw: dict, X: np.ndarray, cfg: OracleConfig) -> np.ndarray:
    """One transformer block over a whole sequence at positions ``0..n-1``, no cache."""
    n = X.shape[0]
    pos = np.arange(n)
    q, k, v = _project_qkv(lw, X, pos, cfg)
    return _finish_block(lw, X, causal_attention(q, pos, k, v), cfg)


# ------------------------------------------------- one-shot masked forward (Eqs. 1-5)

def inference_mask(n: int, prompt_len: int, tau: int) -> np.ndarray:
    """Full-position mask that cycle decoding realises for a prompt of ``prompt_len`` tokens.

    Every prompt position is full; afterwards the full positions are
    ``prompt_len - 1 + k * tau`` (Sec. 2.2: the prefill pass is the first pass of
    cycle 1, and each later cycle starts with one full pass).
    """
    p = np.arange(n)
    return (p < prompt_len) | ((p - (prompt_len - 1)) % tau == 0)


def masked_forward(tokens, mask, n_late: int, w: dict, cfg: OracleConfig, n_early: int = 0) -> np.ndarray:
    """Eqs. 1-5 as one causal pass over ``tokens``; returns logits ``[n, V]``.

    Encoding layers (the first ``n_early``, Eq. 1) and thinking layers (up to layer
    ``L - n_late``, Eq. 2) run on every position; the late (decoding) layers read, at
    position ``i``, the thinking output where ``mask[i]`` and, elsewhere, the raw embedding
    (Eq. 4) or, in the ExDy variant, the encoding output.  With ``cfg.full_pos_add_embed``
    full positions read ``h_emb + h_think`` (ExDy: ``h_enc + h_think``) instead.
    """
    tokens = np.asarray(tokens)
    mask = np.asarray(mask, dtype=bool)
    h_emb = w["embed"][tokens]
    front = cfg.n_layers - n_late
    if not (0 <= n_early <= front):
        raise ValueError("n_early must lie in [0, L - n_late]")
    h = h_emb
    for l in range(n_early):
        h = block_full_sequence(w["layers"][l], h, cfg)
    h_enc = h                                    # Eq. 1 (the embedding itself when n_early = 0)
    for l in range(n_early, front):
        h = block_full_sequence(w["layers"][l], h, cfg)
    h_think = h                                  # Eq. 2
    if cfg.full_pos_add_embed:
        h_masked = h_enc + h_think * mask[:, None]
    else:
        h_masked = np.where(mask[:, None], h_think, h_enc)
    h = h_masked
    for l in range(front, cfg.n_layers):
        h = block_full_sequence(w["layers"][l], h, cfg)
    return lm_logits(h, w, cfg)


def training_mask(n: int, tau: int) -> np.ndarray:
    """Eq. 3: position ``i`` is a full position (m_i = 1) exactly when ``i mod tau == 0``."""
    return np.arange(n) % tau == 0


def next_token_nll(logits: np.ndarray, tokens) -> np.ndarray:
    """Summands of Eq. 6: ``nll[i] = CrossEntropy(z_i, x_{i+1}) = log(sum_v exp z_i[v]) - z_i[x_{i+1}]``
    for every position ``i`` that has a successor in ``tokens`` (``len(tokens) - 1`` values)."""
    z = np.asarray(logits)
    t = np.asarray(tokens)
    n = len(t) - 1
    out = np.empty(n, dtype=z.dtype)
    for i in range(n):
        row = z[i]
        top = row.max()
        out[i] = top + np.log(np.exp(row - top).sum()) - row[t[i + 1]]
    return out


def next_token_loss(logits: np.ndarray, tokens) -> float:
    """Eq. 6: the mean of the cross entropies of ``z_i`` against ``x_{i+1}`` over the positions that have a successor."""
    return float(next_token_nll(logits, tokens).mean())


def vanilla_forward(tokens, w: dict, cfg: OracleConfig) -> np.ndarray:
    """Ordinary causal forward over the whole sequence (every position full)."""
    cfg0 = dataclasses.replace(cfg, full_pos_add_embed=False)
    return masked_forward(tokens, np.ones(len(tokens), bool), cfg.n_layers, w, cfg0)


def plt_closed_form(n_layers: int, n_late: int, tau: int, n_early: int = 0) -> float:
    """Eq. 7: (L + (tau - 1) L_d) / (tau L); in the ExDy variant the in-cycle tokens also pass
    the ``n_early`` encoding layers, so L_d becomes ``n_early + n_late`` layers per in-cycle token."""
    return (n_layers + (tau - 1) * (n_early + n_late)) / (tau * n_layers)


# ------------------------------------------------------------ token selection by sampling

def sampling_uniforms(seed: int, seq: int, pos: int, vocab: int) -> np.ndarray:
    """The ``vocab`` uniform deviates of one draw, one per vocabulary entry, from the counter-based generator of
    the input module: stream ``(seed, seq * 2^32 + pos)``, entry ``v`` from counter ``v``, the top 23 bits of the
    64-bit value mapped to the midpoints ``(m + 0.5) / 2^23`` of a 23-bit grid (strictly inside (0, 1), and exactly
    representable in float32, 2 m + 1 < 2^24, so a float32 implementation draws the same numbers)."""
    import dmtd_inputs
    raw = dmtd_inputs.raw_u64(seed, (int(seq) << 32) | int(pos), 0, vocab)
    return ((raw >> np.uint64(41)).astype(np.float64) + 0.5) / float(1 << 23)


def sampling_scores(z: np.ndarray, temperature: float, top_k: int, seed: int, seq: int, pos: int) -> np.ndarray:
    """Scores whose argmax is a draw from ``softmax(z / temperature)`` restricted to the ``top_k`` largest logits
    (``top_k <= 0``: no restriction; logits equal to the k-th largest all stay in): ``z_v / temperature + g_v``
    with independent standard Gumbel deviates ``g_v = -log(-log(u_v))`` (the Gumbel-max identity); entries outside
    the restriction get ``-inf``."""
    z = np.asarray(z, dtype=np.float64)
    u = sampling_uniforms(seed, seq, pos, len(z))
    s = z / float(temperature) - np.log(-np.log(u))
    if 0 < top_k < len(z):
        kth = np.sort(z)[len(z) - top_k]
        s = np.where(z >= kth, s, -np.inf)
    return s


def sample_token(z: np.ndarray, temperature: float, top_k: int, seed: int, seq: int, pos: int) -> int:
    """One token drawn for the row at position ``pos`` of sequence ``seq`` (lowest index among equal scores)."""
    return int(np.argmax(sampling_scores(z, temperature, top_k, seed, seq, pos)))


# -------------------------------------------------------- incremental cycle machine

class DmtdOracle:
    """Cycle decoding with cyclical KV refilling for one sequence (Sec. 2.2, Fig. 3).

    State: ``n_tok`` tokens have entered the late layers' caches, ``n_front`` the front
    layers' caches (``n_tok - n_front`` tokens await refill), ``phase`` tokens of the
    current cycle have been emitted, ``last`` is the token the next step consumes.
    """

    def __init__(self, cfg: OracleConfig, weights: dict, max_seq_len: int, dtype=np.float64):
        self.cfg, self.w, self.dtype = cfg, weights, dtype
        self.max_seq_len = max_seq_len
        c = cfg
        self.K = [np.zeros((max_seq_len, c.n_kv_heads, c.head_dim), dtype) for _ in range(c.n_layers)]
        self.V = [np.zeros((max_seq_len, c.n_kv_heads, c.head_dim), dtype) for _ in range(c.n_layers)]
        self.reset()

    def reset(self):
        self.tokens: list[int] = []       # every token consumed so far, by position
        self.n_tok = 0
        self.n_front = 0
        self.phase = 0
        self.last = None
        self.last_logits = None
        self.step_logits: list[np.ndarray] = []
        self.trace: list[list[tuple[str, list[int]]]] = []   # per pass: [(group, positions)]
        self.gen_layer_visits = 0         # layers traversed by rows that emit a token
        self.refill_layer_visits = 0      # layers traversed by refill rows
        self.n_emitted = 0                # tokens emitted by decode steps (prefill's excluded)
        self.n_late_in_use = None
        self.n_early_in_use = 0
        self.pend_enc: list[np.ndarray] = []   # ExDy: encoding outputs of the tokens that await refill
        self.last_scores = None           # sampling: the scores whose argmax was the last token

    # one block over `rows` new positions with the layer's cache
    def _block(self, l: int, X: np.ndarray, positions: np.ndarray) -> np.ndarray:
        lw = self.w["layers"][l]
        q, k, v = _project_qkv(lw, X, positions, self.cfg)
        self.K[l][positions] = k
        self.V[l][positions] = v
        ctx = int(positions[-1]) + 1
        attn = causal_attention(q, positions, self.K[l][:ctx], self.V[l][:ctx])
        return _finish_block(lw, X, attn, self.cfg)

    def set_sampling(self, temperature: float, top_k: int = 0, seed: int = 0, seq: int = 0):
        """Select tokens by sampling (``temperature > 0``) instead of greedily (``temperature <= 0``, the default).
        ``seq`` is the sequence's index in its batch: it enters the random counter, so that sequences draw
        independently.  The setting survives ``reset``."""
        self.sampling = (float(temperature), int(top_k), int(seed), int(seq)) if temperature > 0 else None

    def _emit(self, h_row: np.ndarray) -> int:
        z = lm_logits(h_row, self.w, self.cfg)
        self.last_logits = z
        self.step_logits.append(z)
        sampling = getattr(self, "sampling", None)
        if sampling is None:
            return int(np.argmax(z))
        t, k, seed, seq = sampling
        # the row that emits sits at position n_tok - 1 (the callers have already counted it)
        self.last_scores = sampling_scores(z, t, k, seed, seq, self.n_tok - 1)
        return int(np.argmax(self.last_scores))

    def prefill(self, tokens, n_late: int | None = None, n_early: int = 0) -> int:
        """All prompt tokens through all layers; returns the first generated token.

        ``n_late`` (and ``n_early``) matter only under the literal Eq. 4 reading, where the
        embedding (ExDy: the encoding output) is added again at the front/late boundary of
        every (full) prompt position.
        """
        tokens = [int(t) for t in tokens]
        P = len(tokens)
        c = self.cfg
        if self.n_tok != 0:
            raise RuntimeError("prefill on a used oracle; call reset()")
        if P < 1 or P >= self.max_seq_len:
            raise ValueError("bad prompt length")
        if c.full_pos_add_embed and n_late is None:
            raise ValueError("the literal Eq. 4 reading needs n_late at prefill")
        pos = np.arange(P)
        E = self.w["embed"][np.asarray(tokens)]
        H = E
        F = c.n_layers - (n_late if n_late is not None else 0)
        base = E
        for l in range(c.n_layers):
            if l == n_early:
                base = H                                 # Eq. 1 output (the embedding when n_early = 0)
            if l == F and c.full_pos_add_embed:
                H = H + base
            H = self._block(l, H, pos)
        self.tokens = tokens
        self.trace.append([("front", list(range(P))), ("late", list(range(P)))])
        self.n_tok = self.n_front = P
        self.phase = 1
        self.n_late_in_use = n_late
        self.n_early_in_use = n_early
        self.last = self._emit(H[-1])
        return self.last

    def _late_step(self, n_late: int, n_early: int = 0) -> int:
        c = self.cfg
        F = c.n_layers - n_late
        p = self.n_tok
        self.tokens.append(self.last)
        h = self.w["embed"][self.last][None, :]          # Eq. 4, m = 0: raw embedding
        pos = np.array([p])
        for l in range(n_early):
            h = self._block(l, h, pos)                   # ExDy: the encoding layers see every token
        if n_early > 0:
            self.pend_enc.append(h[0].copy())            # kept for the refill of the thinking layers
        for l in range(F, c.n_layers):
            h = self._block(l, h, pos)
        self.trace.append(([("enc", [p])] if n_early > 0 else []) + [("late", [p])])
        self.gen_layer_visits += n_early + n_late
        self.n_tok += 1
        return self._emit(h[0])

    def _full_step(self, n_late: int, n_early: int = 0) -> int:
        c = self.cfg
        F = c.n_layers - n_late
        p = self.n_tok
        self.tokens.append(self.last)
        pos = np.arange(self.n_front, p + 1)             # pending in-cycle tokens, then the newest
        if n_early > 0:
            h_new = self.w["embed"][self.last][None, :]
            for l in range(n_early):
                h_new = self._block(l, h_new, np.array([p]))   # the pending tokens passed these layers in their own steps
            H = np.concatenate([np.asarray(self.pend_enc, dtype=h_new.dtype).reshape(len(pos) - 1, h_new.shape[1]), h_new], 0)
            base_new = h_new
        else:
            H = self.w["embed"][np.asarray(self.tokens[self.n_front:p + 1])]
            base_new = H[-1:]
        for l in range(n_early, F):
            H = self._block(l, H, pos)                   # refills the thinking (and, without ExDy, all front) caches
        h = H[-1:]
        if c.full_pos_add_embed:
            h = h + base_new
        for l in range(F, c.n_layers):
            h = self._block(l, h, np.array([p]))         # only the newest row enters the late layers
        passes = []
        if n_early > 0:
            passes.append(("enc", [p]))
        if F - n_early > 0:
            passes.append(("front", [int(x) for x in pos]))
        passes.append(("late", [p]))
        self.trace.append(passes)
        self.gen_layer_visits += c.n_layers
        self.refill_layer_visits += (len(pos) - 1) * (F - n_early)
        self.pend_enc = []
        self.n_tok += 1
        self.n_front = self.n_tok
        return self._emit(h[0])

    def decode_cycle(self, tau: int, n_late: int, max_new: int = 0, forced=None, n_early: int = 0) -> list[int]:
        """Finish the open cycle, or run one whole cycle at a cycle boundary.

        Returns the argmax tokens of the steps run.  With ``forced`` (a sequence of
        token ids), step ``i`` of this call consumes ``forced[i]`` as its input token
        instead of the previous step's argmax (teacher forcing).
        """
        c = self.cfg
        if self.n_tok == 0:
            raise RuntimeError("decode before prefill")
        if tau < 1 or not (1 <= n_late <= c.n_layers):
            raise ValueError("bad tau or n_late")
        if not (0 <= n_early <= c.n_layers - n_late):
            raise ValueError("n_early must lie in [0, L - n_late]")
        if self.n_late_in_use not in (None, n_late) and self.n_front != self.n_tok:
            raise RuntimeError("n_late changed while tokens await refill")
        if self.n_early_in_use != n_early and self.n_front != self.n_tok:
            raise RuntimeError("n_early changed while tokens await refill")
        self.n_late_in_use = n_late
        self.n_early_in_use = n_early
        cap = max_new if max_new > 0 else 1 << 30
        out = []

        def step(fn):
            if self.n_tok + 1 > self.max_seq_len:
                raise OverflowError("sequence capacity")
            if forced is not None:
                self.last = int(forced[len(out)])
            tok = fn(n_late, n_early)
            out.append(tok)
            self.n_emitted += 1
            self.last = tok

        if self.phase >= tau or self.phase == 0:
            step(self._full_step)
            self.phase = 1
        while self.phase < tau and len(out) < cap:
            step(self._late_step)
            self.phase += 1
        return out
