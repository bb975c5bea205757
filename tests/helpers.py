"""Shared harness of the GPU parity tests: builds the CPU oracle and the GPU
context from the same seeded data and compares them.  The oracle and the
library never see each other; only data (weights, prefix K/V, tokens) is
shared."""
from __future__ import annotations

import numpy as np

import oracle.fdc_oracle as O
from synth_inputs import bf16_round, bits_to_f32

HIDDEN_TOL = 2e-3      # max |gpu - ref| / max |ref| per compared tensor (bf16 path vs fp64)
GAP_MIN = 1e-2         # greedy ids must agree wherever the oracle's top-2 gap exceeds this


def rel_err(got, ref):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    return float(np.max(np.abs(got - ref)) / max(np.max(np.abs(ref)), 1e-300))


def as_f32(a):
    a = np.asarray(a)
    return bits_to_f32(a) if a.dtype == np.uint16 else a.astype(np.float32)


class Pair:
    """Oracle decoder + GPU context over the same model, template and prefix."""

    def __init__(self, dims, tpl, weights, n_scenes=1, max_branches=None, max_tokens=1, kv_bf16=True,
                 f16_weights=None):
        from paper_2602_02864_amd import Context
        self.dims, self.tpl, self.w, self.B = dims, tpl, weights, n_scenes
        self.n_sure = self.n_rows = 0          # rows whose greedy id had to agree / rows compared
        F = tpl.n_fields
        self.Rmax = max_branches or F
        # the library's cache is bf16: the oracle stores its K/V in that format too
        self.dec = O.OracleDecoder(dims, weights, tpl.prefix_len, tpl.slot_len, tpl.edges, n_scenes,
                                   kv_bf16=kv_bf16)
        self.ctx = Context(dims, tpl.slot_len, tpl.edges, tpl.prefix_len, n_scenes, self.Rmax, max_tokens,
                           f16_weights=f16_weights)
        if f16_weights == "all":
            self.ctx.set_f16_projections(31)       # every projection single-pass on the fp16 copies
        layers = weights["layers"]
        for l in range(dims.n_layers):
            self.ctx.set_layer_weights(l, layers(l) if callable(layers) else layers[l])
        self.ctx.set_head_weights(weights["emb"], weights["gf"], weights["lm"])

    def close(self, need_sure=True):
        """need_sure: the greedy-id comparison must have had something to compare
        (rows whose top-2 gap exceeds GAP_MIN) over the life of the pair."""
        self.ctx.close()
        if need_sure and self.n_rows > 0:
            assert self.n_sure > 0, f"no row of {self.n_rows} had a top-2 gap above {GAP_MIN}: ids never compared"

    # prefix K/V are data: rounded to bf16 once, handed to both sides
    def install_prefix_kv(self, scene, K, V):
        """K, V: [L][Hkv][P][D] float arrays of bf16-representable values."""
        P = self.tpl.prefix_len
        self.dec.set_prefix_kv(scene, K, V)
        for l in range(self.dims.n_layers):
            self.ctx.kv_append(l, np.ascontiguousarray(np.transpose(K[l], (1, 0, 2)), dtype=np.float32),
                               np.ascontiguousarray(np.transpose(V[l], (1, 0, 2)), dtype=np.float32),
                               np.full(P, scene, dtype=np.int32), np.arange(P, dtype=np.int32))

    def install_slot_kv(self, scene, field, K, V):
        """History of a field as data on both sides: K, V [L][Hkv][n][D] of
        bf16-representable values become the first n tokens of the field's slot."""
        n = K.shape[2]
        s0 = self.dec.slot_start[field]
        assert n <= self.tpl.slot_len[field]
        self.dec.K[:, scene, :, s0:s0 + n] = K
        self.dec.V[:, scene, :, s0:s0 + n] = V
        self.dec.valid_len[scene, field] = n
        for l in range(self.dims.n_layers):
            self.ctx.kv_append(l, np.ascontiguousarray(np.transpose(K[l], (1, 0, 2)), dtype=np.float32),
                               np.ascontiguousarray(np.transpose(V[l], (1, 0, 2)), dtype=np.float32),
                               np.full(n, scene, dtype=np.int32), np.arange(s0, s0 + n, dtype=np.int32))
        self.ctx.set_valid_len(self.dec.valid_len)

    def prefill_with_oracle(self, scene, prefix_emb):
        P = self.tpl.prefix_len
        self.dec.prefill_prefix(scene, prefix_emb)
        K = bf16_round(self.dec.K[:, scene, :, :P].astype(np.float32))
        V = bf16_round(self.dec.V[:, scene, :, :P].astype(np.float32))
        self.install_prefix_kv(scene, K, V)

    def step_both(self, branch_field, branch_off, tok_in, T=1, check=True, tag=""):
        """Runs one step on both sides with the same (teacher-forced) inputs and
        compares; returns (oracle output, gpu output as numpy)."""
        import torch
        bf = np.asarray(branch_field, dtype=np.int32).reshape(self.B, -1)
        bo = np.asarray(branch_off, dtype=np.int32).reshape(self.B, -1)
        R = bf.shape[1]
        tok = np.asarray(tok_in, dtype=np.int32).reshape(self.B, R, T)
        ref = self.dec.step(bf, bo, tok_in=tok, T=T)
        g = self.ctx.parallel_decode_step(bf, bo, tok_in=tok, T=T, want_logits=True, want_hidden=True)
        torch.cuda.synchronize()
        got = {k: v.cpu().numpy() for k, v in g.items() if not k.startswith("_")}
        self.compare_tables(bf, bo, T, tag)
        if check:
            self.compare(ref, got, tag)
        return ref, got

    def compare_tables(self, bf, bo, T, tag=""):
        """The mask and the position ids the device used in the step it just ran
        (its visibility words and position table, expanded) against the oracle's
        dense mask under the state after the step: bit for bit (Sec. 3.3, Eq. 1)."""
        R = bf.shape[1]
        mask, pos = self.ctx.step_tables_dense(R, T)
        tpl = self.tpl
        for b in range(self.B):
            for r in range(R):
                m0 = (b * R + r) * T
                if bf[b, r] < 0:
                    assert not mask[m0:m0 + T].any() and (pos[m0:m0 + T] == -1).all(), f"{tag}: inactive rows"
                    continue
                want, wpos = O.dense_mask(tpl.prefix_len, tpl.slot_len, tpl.edges, self.dec.valid_len[b],
                                          [int(bf[b, r])] * T, [int(bo[b, r]) + t for t in range(T)])
                assert np.array_equal(mask[m0:m0 + T].astype(bool), want), f"{tag}: device mask, scene {b} branch {r}"
                assert np.array_equal(pos[m0:m0 + T], wpos), f"{tag}: device positions, scene {b} branch {r}"

    def compare(self, ref, got, tag=""):
        L = self.dims.n_layers
        rows = ref["rows"]
        assert rows.size > 0
        assert np.array_equal(self.ctx.get_valid_len(), self.dec.valid_len), f"{tag}: valid_len differs"
        errs = []
        for l in range(L + 1):
            errs.append(rel_err(got["hidden"][l][rows], ref["hidden"][l][rows]))
        errs.append(rel_err(got["hidden"][L + 1][rows], ref["normed"][rows]))
        e_log = rel_err(got["logits"][rows], ref["logits"][rows])
        assert np.isfinite(got["logits"][rows]).all(), f"{tag}: non-finite logits"
        assert max(errs) <= HIDDEN_TOL, f"{tag}: hidden-state error per layer {errs}"
        assert e_log <= HIDDEN_TOL, f"{tag}: logits error {e_log}"
        sure = rows[ref["gap"][rows] > GAP_MIN]
        self.n_sure += int(sure.size)
        self.n_rows += int(rows.size)
        assert np.array_equal(got["tok"][sure], ref["tok"][sure]), f"{tag}: greedy ids differ"
        inactive = np.setdiff1d(np.arange(ref["tok"].size), rows)
        assert (got["tok"][inactive] == -1).all(), f"{tag}: inactive rows must return -1"
        # the library's own argmax must agree with its own logits exactly
        assert np.array_equal(got["tok"][rows], np.argmax(got["logits"][rows], axis=1)), f"{tag}: argmax"
        return max(max(errs), e_log)


def run_schedule(pair, content_len, start_token, max_steps=None, tag=""):
    """Teacher-forced template decoding of scene 0 (B == 1): at every step both
    sides get the oracle's previous tokens."""
    tpl = pair.tpl
    steps = O.schedule(tpl.n_fields, tpl.edges, content_len)
    if max_steps:
        steps = steps[:max_steps]
    R = max(len(s) for s in steps)
    last = list(start_token)
    worst = 0.0
    for si, st in enumerate(steps):
        bf = [f for f, _ in st] + [-1] * (R - len(st))
        bo = [o for _, o in st] + [0] * (R - len(st))
        ti = [last[f] for f, _ in st] + [0] * (R - len(st))
        ref, got = pair.step_both([bf], [bo], ti, check=False)
        worst = max(worst, pair.compare(ref, got, f"{tag} step {si}"))
        for i, (f, _) in enumerate(st):
            last[f] = int(ref["tok"][i])
    return worst, len(steps)
