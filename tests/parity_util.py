"""Helpers shared by the GPU parity tests: build the HIP engine and the CPU oracle from the same
seeded inputs and compare them step by step."""
import numpy as np

import dmtd_inputs as di
import paper_2510_11958_amd as pkg
from oracle import dmtd_oracle as O

MARGIN = 0.05   # token ids must agree wherever the oracle's top-2 logit margin exceeds this


def engine_config(sh, max_seq_len, max_batch=1, **kw):
    return pkg.ModelConfig(sh.n_layers, sh.hidden, sh.n_q_heads, sh.n_kv_heads, sh.head_dim, sh.intermediate, sh.vocab,
                           dtype=sh.dtype, rms_eps=sh.rms_eps, rope_theta=sh.rope_theta,
                           tied_embeddings=sh.tied_embeddings, max_seq_len=max_seq_len, max_batch=max_batch, **kw)


def oracle_config(sh, **kw):
    return O.OracleConfig(sh.n_layers, sh.hidden, sh.n_q_heads, sh.n_kv_heads, sh.head_dim, sh.intermediate, sh.vocab,
                          sh.rms_eps, sh.rope_theta, sh.tied_embeddings, **kw)


def norm_err(z_gpu, z_ref):
    """max_i |z_gpu[i] - z_ref[i]| / max_j |z_ref[j]|"""
    return float(np.abs(z_gpu.astype(np.float64) - z_ref).max() / np.abs(z_ref).max())


def top2_margin(z):
    part = np.partition(z, -2)
    return float(part[-1] - part[-2])


class Pair:
    """The engine and one oracle per sequence, advanced in lockstep with teacher forcing."""

    def __init__(self, sh, blob, max_seq_len, batch=1, literal=False, use_graphs=True, oracle_dtype=np.float64,
                 weights_dev=None, n_early=0):
        self.sh, self.batch, self.n_early = sh, batch, n_early
        self.eng = pkg.Engine(engine_config(sh, max_seq_len, batch, full_pos_add_embed=literal, use_graphs=use_graphs),
                              blob if weights_dev is None else weights_dev)
        ocfg = oracle_config(sh, full_pos_add_embed=literal)
        w = O.unpack_weights(blob, ocfg, oracle_dtype)
        self.orcs = [O.DmtdOracle(ocfg, w, max_seq_len, oracle_dtype) for _ in range(batch)]
        if n_early:
            self.eng.set_n_early(n_early)
        self.worst = 0.0
        self.token_checks = 0
        self.token_skips = 0

    def _compare(self, gpu_tokens):
        z = self.eng.logits()
        for b, o in enumerate(self.orcs):
            ref = o.last_logits.astype(np.float64)
            self.worst = max(self.worst, norm_err(z[b], ref))
            if top2_margin(ref) > MARGIN:
                assert int(gpu_tokens[b]) == int(np.argmax(ref)), (b, o.n_tok)
                self.token_checks += 1
            else:
                self.token_skips += 1
            assert int(gpu_tokens[b]) == int(np.argmax(z[b]))   # the reported token is the argmax of the reported logits

    def prefill(self, prompts, n_late=0):
        first = self.eng.prefill(prompts, n_late)
        for b, o in enumerate(self.orcs):
            o.prefill(prompts[b], n_late if n_late else None, self.n_early)
        self._compare(first)
        return first

    def step_forced(self, tau, n_late, tokens_by_pos):
        """Run single steps (max_new=1) so that every step's logits can be compared."""
        nt = self.eng.state()["n_tok"]
        f = np.stack([tokens_by_pos[b][nt:nt + 1] for b in range(self.batch)])
        out = self.eng.decode_cycle(tau, n_late, max_new=1, forced=f)
        for b, o in enumerate(self.orcs):
            o.decode_cycle(tau, n_late, max_new=1, forced=f[b].tolist(), n_early=self.n_early)
        assert out.shape == (self.batch, 1)
        self._compare(out[:, 0])
        s = self.eng.state()
        o = self.orcs[0]
        assert (s["n_tok"], s["n_front"], s["phase"]) == (o.n_tok, o.n_front, o.phase)

    def compare_kv(self, atol_rel):
        n = self.orcs[0].n_tok
        for l in range(self.sh.n_layers):
            # front (ExDy: thinking) layers hold positions < n_front, late layers and ExDy's encoding layers < n_tok
            for b, o in enumerate(self.orcs):
                kv = self.eng.read_kv(l, b, n)
                late = l >= self.sh.n_layers - (o.n_late_in_use or self.sh.n_layers)
                upto = o.n_tok if (late or l < self.n_early) else o.n_front
                for which, ref in ((0, o.K[l]), (1, o.V[l])):
                    r = np.transpose(ref[:upto], (1, 0, 2))
                    err = np.abs(kv[which][:, :upto] - r).max() / max(np.abs(r).max(), 1e-30)
                    assert err < atol_rel, (l, b, which, err)
