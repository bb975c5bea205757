"""Pins for the CPU oracle: every part is checked against something other
than itself - brute force, closed forms, library routines, or the invariants
the paper states (Sec. 3.2 optimality; Sec. 3.3 mask rule, Eq. 1, padding,
KV reuse; Fig. 3 caption).  All CPU, no GPU library involved."""
import itertools

import numpy as np
import pytest
import torch
import torch.nn.functional as tF

import oracle.fdc_oracle as O
from synth_inputs import (ModelDims, draw_weights, draw_prefix_embeddings, draw_tokens,
                          chain_template, edgeless_template, random_dag_template, template)

TINY = ModelDims(n_layers=2, d_model=32, n_q_heads=4, n_kv_heads=2, head_dim=8, d_mlp=48,
                 vocab=50, rope_base=1.0e6)


# ---------------------------------------------------------------- ancestors
def _warshall(F, edges):
    reach = np.zeros((F, F), dtype=bool)
    for (u, v) in edges:
        reach[u, v] = True
    for k in range(F):
        for i in range(F):
            for j in range(F):
                if reach[i, k] and reach[k, j]:
                    reach[i, j] = True
    return reach


@pytest.mark.parametrize("F", [1, 2, 3, 4, 5])
def test_ancestors_all_small_dags_bruteforce(F):
    pairs = [(i, j) for j in range(F) for i in range(j)]
    for bits in range(1 << len(pairs)):
        edges = [p for k, p in enumerate(pairs) if bits >> k & 1]
        reach = _warshall(F, edges)
        anc = O.ancestors(F, edges)
        words = O.ancestor_words(F, edges)
        for f in range(F):
            want = {g for g in range(F) if reach[g, f]}
            assert anc[f] == want
            assert int(words[f, 0]) == sum(1 << g for g in want)


@pytest.mark.parametrize("seed,F,p", [(0, 17, 0.1), (1, 64, 0.05), (2, 64, 0.3), (3, 100, 0.04),
                                      (4, 130, 0.02)])
def test_ancestors_random_vs_matrix_closure(seed, F, p):
    rng = np.random.default_rng(seed)
    edges = [(i, j) for j in range(F) for i in range(j) if rng.random() < p]
    A = np.zeros((F, F), dtype=np.int64)
    for (u, v) in edges:
        A[u, v] = 1
    reach = np.zeros_like(A)
    Pw = A.copy()
    for _ in range(F):                      # sum of powers of the adjacency matrix
        reach |= (Pw > 0)
        Pw = (Pw @ A > 0).astype(np.int64)
    words = O.ancestor_words(F, edges)
    assert words.shape == (F, (F + 63) // 64)
    for f in range(F):
        for g in range(F):
            bit = int(words[f, g // 64]) >> (g % 64) & 1
            assert bit == int(reach[g, f] > 0)


def test_levels_is_longest_path():
    # diamond with a long arm: 0->1->2->4, 0->3->4 ; 5 isolated
    edges = [(0, 1), (1, 2), (2, 4), (0, 3), (3, 4)]
    assert O.levels(6, edges) == [0, 1, 2, 1, 3, 0]


def test_check_template_rejects_cycles_and_backward_edges():
    O.check_template(3, [(0, 1), (1, 2)])
    with pytest.raises(ValueError, match="cycle"):
        O.check_template(3, [(0, 1), (1, 2), (2, 0)])
    with pytest.raises(ValueError, match="earlier"):
        O.check_template(3, [(2, 1)])
    with pytest.raises(ValueError, match="self-loop"):
        O.check_template(3, [(1, 1)])
    with pytest.raises(ValueError, match="outside"):
        O.check_template(3, [(0, 3)])


# --------------------------------------------------------------------- mask
def test_chain_dag_full_slots_is_causal_mask():
    P, F, S = 5, 4, 3
    edges = [(i, i + 1) for i in range(F - 1)]
    rf = [f for f in range(F) for _ in range(S)]
    ro = [t for _ in range(F) for t in range(S)]
    mask, pos = O.dense_mask(P, [S] * F, edges, [S] * F, rf, ro)
    N = P + F * S
    assert list(pos) == list(range(P, N))
    causal = np.tril(np.ones((N, N), dtype=bool))[P:]
    assert np.array_equal(mask, causal)


def test_edgeless_dag_is_block_diagonal_plus_prefix():
    P, F, S = 4, 3, 5
    rf = [f for f in range(F) for _ in range(S)]
    ro = [t for _ in range(F) for t in range(S)]
    mask, _ = O.dense_mask(P, [S] * F, [], [S] * F, rf, ro)
    want = np.zeros((F * S, P + F * S), dtype=bool)
    want[:, :P] = True
    for f in range(F):
        want[f * S:(f + 1) * S, P + f * S:P + (f + 1) * S] = np.tril(np.ones((S, S), dtype=bool))
    assert np.array_equal(mask, want)


def test_mask_invariants_of_the_figure_caption():
    """Independent fields never see each other, dependent ones see the whole
    written part of the ancestor, padding is seen by nobody, and the rule is
    transitive (Eq. 1 speaks of a path, not an edge)."""
    P = 3
    slot = [4, 2, 5, 3, 4]
    edges = [(0, 2), (2, 4), (1, 3)]          # 0 -> 2 -> 4 ; 1 -> 3
    valid = [3, 2, 4, 1, 2]                   # what is in the cache (rest is padding)
    start, N = O.slot_layout(P, slot)
    assert start == [3, 7, 9, 14, 17] and N == 21
    rf, ro = [4, 3, 2, 1, 0], [1, 0, 3, 1, 2]
    mask, pos = O.dense_mask(P, slot, edges, valid, rf, ro)
    assert list(pos) == [18, 14, 12, 8, 5]
    def seen(r, f):
        return mask[r, start[f]:start[f] + slot[f]]
    # row 0: field 4 offset 1: sees prefix, field 0 (3 valid), field 2 (4 valid), own 0..1
    assert mask[0, :P].all()
    assert list(seen(0, 0)) == [True, True, True, False]
    assert not seen(0, 1).any() and not seen(0, 3).any()
    assert list(seen(0, 2)) == [True, True, True, True, False]
    assert list(seen(0, 4)) == [True, True, False, False]
    # row 1: field 3 sees field 1 only (besides itself)
    assert seen(1, 1).all() and not seen(1, 0).any() and not seen(1, 2).any()
    # row 4: field 0 (a root) sees only prefix + own offsets <= 2
    assert mask[4].sum() == P + 3
    # padding columns are invisible to every row
    for f in range(5):
        assert not mask[:, start[f] + valid[f]:start[f] + slot[f]][
            [r for r in range(5) if rf[r] != f]].any()
    # never sees a later position than its own
    for r in range(5):
        assert not mask[r, pos[r] + 1:].any() and mask[r, pos[r]]


# ------------------------------------------------------------ small formulas
def test_rmsnorm_against_closed_form_and_torch():
    x = np.array([[3.0, -4.0, 0.0, 0.0]])
    g = np.array([1.0, 2.0, 3.0, 4.0])
    # mean square = 25/4, so x/rms = x / 2.5
    assert np.allclose(O.rmsnorm(x, g, 0.0), [[1.2, -3.2, 0.0, 0.0]], atol=1e-15)
    rng = np.random.default_rng(0)
    x = rng.standard_normal((5, 16))
    g = rng.standard_normal(16)
    want = tF.rms_norm(torch.from_numpy(x), (16,), torch.from_numpy(g), eps=1e-6).numpy()
    assert np.allclose(O.rmsnorm(x, g, 1e-6), want, rtol=1e-13, atol=1e-13)


def test_rope_closed_forms_and_invariants():
    # D = 2: a plain rotation of the plane by `pos` radians
    x = np.array([1.0, 0.0])
    for p in (0.0, 1.0, 2.5):
        assert np.allclose(O.rope(x, p, 1e6), [np.cos(p), np.sin(p)], atol=1e-15)
    y = np.array([0.0, 1.0])
    assert np.allclose(O.rope(y, 0.5, 1e6), [-np.sin(0.5), np.cos(0.5)], atol=1e-15)
    # D = 4, base 10000: pairs (0,2) at frequency 1 and (1,3) at frequency 1/100
    x = np.array([1.0, 1.0, 0.0, 0.0])
    got = O.rope(x, 3.0, 1.0e4)
    assert np.allclose(got, [np.cos(3.0), np.cos(0.03), np.sin(3.0), np.sin(0.03)], atol=1e-15)
    rng = np.random.default_rng(1)
    q, k = rng.standard_normal(64), rng.standard_normal(64)
    assert np.array_equal(O.rope(q, 0, 1e6), q)
    assert np.isclose(np.linalg.norm(O.rope(q, 1234, 1e6)), np.linalg.norm(q), rtol=1e-13)
    a = O.rope(q, 700, 1e6) @ O.rope(k, 650, 1e6)
    b = O.rope(q, 50, 1e6) @ O.rope(k, 0, 1e6)
    assert np.isclose(a, b, rtol=1e-9, atol=1e-9)
    # same thing written as complex multiplication of (x_i + i x_{i+D/2})
    D = 64
    z = (q[:D // 2] + 1j * q[D // 2:]) * np.exp(1j * 77 * 1e6 ** (-np.arange(D // 2) * 2.0 / D))
    assert np.allclose(O.rope(q, 77, 1e6), np.concatenate([z.real, z.imag]), atol=1e-13)


def test_silu_softmax_greedy():
    import scipy.special
    x = np.linspace(-6, 6, 25)
    assert np.allclose(O.silu(x), tF.silu(torch.from_numpy(x)).numpy(), atol=1e-15)
    assert np.allclose(O.silu(np.array([0.0, 1.0])), [0.0, 1 / (1 + np.exp(-1.0))])
    s = np.random.default_rng(2).standard_normal(33) * 5
    assert np.allclose(O.softmax(s), scipy.special.softmax(s), atol=1e-15)
    assert O.greedy(np.array([1.0, 3.0, 3.0, 2.0])) == (1, 0.0)
    tok, gap = O.greedy(np.array([0.5, -1.0, 2.0, 1.25]))
    assert tok == 2 and gap == 0.75


def test_attention_single_key_and_against_sdpa():
    rng = np.random.default_rng(3)
    q = rng.standard_normal(8)
    K = rng.standard_normal((6, 8))
    V = rng.standard_normal((6, 8))
    vis = np.zeros(6, dtype=bool)
    vis[4] = True
    assert np.allclose(O.attend(q, K, V, vis), V[4], atol=1e-15)     # one key: o = v
    # against torch's scaled_dot_product_attention with a boolean mask, fp64
    tpl = random_dag_template(5, n_fields=6, prefix_len=7, max_slot=5, edge_prob=0.4, vocab=10)
    start, N = O.slot_layout(tpl.prefix_len, tpl.slot_len)
    Hq, Hkv, D = 6, 2, 16
    rf = list(range(6))
    ro = [c - 1 for c in tpl.content_len]
    valid = tpl.content_len
    q = rng.standard_normal((6, Hq, D))
    K = rng.standard_normal((Hkv, N, D))
    V = rng.standard_normal((Hkv, N, D))
    got = O.attention_only(q, K, V, tpl.prefix_len, tpl.slot_len, tpl.edges, valid, rf, ro, Hq // Hkv)
    mask, _ = O.dense_mask(tpl.prefix_len, tpl.slot_len, tpl.edges, valid, rf, ro)
    tq = torch.from_numpy(q).permute(1, 0, 2)[None]                       # [1][Hq][rows][D]
    tk = torch.from_numpy(K).repeat_interleave(Hq // Hkv, 0)[None]
    tv = torch.from_numpy(V).repeat_interleave(Hq // Hkv, 0)[None]
    want = tF.scaled_dot_product_attention(tq, tk, tv, attn_mask=torch.from_numpy(mask)[None, None])
    assert np.allclose(got, want[0].permute(1, 0, 2).numpy(), rtol=1e-12, atol=1e-12)


def test_bf16_storage_rounding_matches_torch_and_is_off_by_default():
    rng = np.random.default_rng(9)
    x = np.concatenate([rng.standard_normal(4000) * 10.0 ** rng.integers(-6, 6, 4000),
                        [0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.0e38, -1e-40]])   # incl. exact ties
    want = torch.from_numpy(x.astype(np.float32)).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(O.to_bf16(x), want)
    # ties go to even: 1 + 2^-8 is halfway between 1 and 1 + 2^-7
    assert O.to_bf16(np.array([1.00390625]))[0] == 1.0 and O.to_bf16(np.array([1.01171875]))[0] == 1.015625
    tpl = edgeless_template(2, 2, 3, TINY.vocab)
    w, prefix = _tiny_setup(tpl, seed_cfg=7)
    outs = {}
    for flag in (False, True):
        dec = O.OracleDecoder(TINY, w, 3, tpl.slot_len, tpl.edges, kv_bf16=flag)
        assert dec.kv_bf16 is flag
        dec.prefill_prefix(0, prefix)
        dec.step([[0]], [[0]], tok_in=[[[1]]])
        outs[flag] = dec.step([[0]], [[1]], tok_in=[[[2]]])["logits"][0]
        k = dec.K[0, 0, 0, 3]
        assert np.array_equal(k, O.to_bf16(k)) is flag      # stored K is bf16 only when asked for
    assert O.OracleDecoder(TINY, w, 3, tpl.slot_len, tpl.edges).kv_bf16 is False
    assert 0 < np.max(np.abs(outs[True] - outs[False])) < 2e-2 * np.max(np.abs(outs[False]))


# ----------------------------------------------- an independent plain decoder
def _torch_reference_logits(dims, w, x_rows, pos_ids):
    """Ordinary causal decoder over one sequence, written with torch's library
    ops in fp64 and rotary embedding as complex multiplication.  x_rows [n][d],
    pos_ids [n] (need not be contiguous).  Returns logits [n][V] and the
    residual stream after every layer."""
    t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
    x = t(x_rows)
    n = x.shape[0]
    D, Hq, Hkv = dims.head_dim, dims.n_q_heads, dims.n_kv_heads
    freq = torch.tensor(dims.rope_base, dtype=torch.float64) ** (
        -torch.arange(D // 2, dtype=torch.float64) * 2.0 / D)
    rot = torch.polar(torch.ones(n, D // 2, dtype=torch.float64),
                      t(pos_ids)[:, None] * freq)[:, None, :]

    def rope(z):                                   # [n][H][D]
        zc = torch.complex(z[..., :D // 2], z[..., D // 2:]) * rot
        return torch.cat([zc.real, zc.imag], dim=-1)
    hidden = []
    for lw in w["layers"]:
        a = tF.rms_norm(x, (dims.d_model,), t(lw["g1"]), eps=dims.norm_eps)
        qkv = tF.linear(a, t(lw["wqkv"]))
        q, k, v = torch.split(qkv, [Hq * D, Hkv * D, Hkv * D], dim=-1)
        q = rope(q.reshape(n, Hq, D)).permute(1, 0, 2)[None]
        k = rope(k.reshape(n, Hkv, D)).permute(1, 0, 2)[None]
        v = v.reshape(n, Hkv, D).permute(1, 0, 2)[None]
        o = tF.scaled_dot_product_attention(q, k, v, is_causal=True, enable_gqa=True)
        x = x + tF.linear(o[0].permute(1, 0, 2).reshape(n, Hq * D), t(lw["wo"]))
        a = tF.rms_norm(x, (dims.d_model,), t(lw["g2"]), eps=dims.norm_eps)
        g, u = torch.split(tF.linear(a, t(lw["wgu"])), [dims.d_mlp, dims.d_mlp], dim=-1)
        x = x + tF.linear(tF.silu(g) * u, t(lw["wd"]))
        hidden.append(x.numpy().copy())
    xn = tF.rms_norm(x, (dims.d_model,), t(w["gf"]), eps=dims.norm_eps)
    return tF.linear(xn, t(w["lm"])).numpy(), hidden


def _tiny_setup(tpl, seed_cfg=0, scale=0.3):
    w = draw_weights(seed_cfg, TINY, random_gains=True, std=scale)
    prefix = draw_prefix_embeddings(seed_cfg, tpl.prefix_len, TINY.d_model).astype(np.float64)
    return w, prefix


def test_chain_dag_equals_ordinary_causal_decoding():
    """Sec. 4.1 baseline: with a chain-shaped graph the method is standard
    autoregressive decoding of the concatenated sequence."""
    F, S, P = 3, 3, 5
    tpl = chain_template(F, S, P, TINY.vocab)
    w, prefix = _tiny_setup(tpl)
    toks = draw_tokens(0, F * S, TINY.vocab)                  # teacher-forced inputs
    dec = O.OracleDecoder(TINY, w, P, tpl.slot_len, tpl.edges)
    dec.prefill_prefix(0, prefix)
    got_logits, got_hidden = [], []
    for i in range(F * S):
        out = dec.step([[i // S]], [[i % S]], tok_in=[[[int(toks[i])]]])
        got_logits.append(out["logits"][0])
        got_hidden.append(out["hidden"][1:, 0])
        assert out["pos"][0] == P + i
    x_all = np.concatenate([prefix, np.asarray(w["emb"], dtype=np.float64)[toks]])
    want_logits, want_hidden = _torch_reference_logits(TINY, w, x_all, np.arange(P + F * S))
    assert np.allclose(np.array(got_logits), want_logits[P:], rtol=1e-10, atol=1e-10)
    for l in range(TINY.n_layers):
        assert np.allclose(np.array(got_hidden)[:, l], want_hidden[l][P:], rtol=1e-10, atol=1e-10)
    assert np.isfinite(np.array(got_logits)).all()


def test_edgeless_dag_equals_each_field_alone_with_the_prefix():
    """Independent fields decoded together give what each gives when decoded
    alone after the prefix, at the same absolute position ids."""
    F, S, P = 4, 3, 6
    tpl = edgeless_template(F, S, P, TINY.vocab)
    w, prefix = _tiny_setup(tpl, seed_cfg=1)
    toks = draw_tokens(1, F * S, TINY.vocab).reshape(F, S)
    dec = O.OracleDecoder(TINY, w, P, tpl.slot_len, tpl.edges)
    dec.prefill_prefix(0, prefix)
    got = np.zeros((F, S, TINY.vocab))
    for t in range(S):                                         # all four fields per pass
        out = dec.step([list(range(F))], [[t] * F], tok_in=toks[:, t].reshape(1, F, 1))
        got[:, t] = out["logits"]
    emb = np.asarray(w["emb"], dtype=np.float64)
    for f in range(F):
        x = np.concatenate([prefix, emb[toks[f]]])
        pos = np.concatenate([np.arange(P), dec.slot_start[f] + np.arange(S)])
        want, _ = _torch_reference_logits(TINY, w, x, pos)
        assert np.allclose(got[f], want[P:], rtol=1e-10, atol=1e-10)


def _decode_some(dec, tpl, n_steps, toks):
    sched = O.schedule(tpl.n_fields, tpl.edges, tpl.content_len)
    R = max(len(s) for s in sched)
    outs = []
    for si, st in enumerate(sched[:n_steps]):
        bf = [f for f, _ in st] + [-1] * (R - len(st))
        bo = [o for _, o in st] + [0] * (R - len(st))
        ti = [int(toks[f, o]) for f, o in st] + [0] * (R - len(st))
        outs.append(dec.step([bf], [bo], tok_in=np.array(ti).reshape(1, R, 1)))
    return sched, outs


def test_masked_out_kv_has_no_effect_and_visible_kv_has():
    tpl = random_dag_template(11, n_fields=6, prefix_len=4, max_slot=4, edge_prob=0.35,
                              vocab=TINY.vocab)
    w, prefix = _tiny_setup(tpl, seed_cfg=2)
    toks = draw_tokens(2, 6 * 4, TINY.vocab).reshape(6, 4)
    dec = O.OracleDecoder(TINY, w, tpl.prefix_len, tpl.slot_len, tpl.edges)
    dec.prefill_prefix(0, prefix)
    sched, _ = _decode_some(dec, tpl, len(O.schedule(6, tpl.edges, tpl.content_len)) - 1, toks)
    last = sched[-1]
    assert last, "schedule has a final step"
    snap = (dec.K.copy(), dec.V.copy(), dec.valid_len.copy())
    f, o = last[0]

    def run(mutate):
        dec.K, dec.V, dec.valid_len = snap[0].copy(), snap[1].copy(), snap[2].copy()
        mutate()
        return dec.step([[f]], [[o]], tok_in=[[[int(toks[f, o])]]])["logits"][0]
    base = run(lambda: None)
    assert np.isfinite(base).all()          # holes hold NaN: none was read
    vis = O.visible_row(tpl.prefix_len, dec.slot_start, dec.slot_len, dec.anc,
                        np.maximum(snap[2][0], [o + 1 if g == f else 0 for g in range(6)]), f, o)
    hidden_cols = [j for j in range(dec.N) if not vis[j] and j != dec.slot_start[f] + o]

    def poison():
        dec.K[:, :, :, hidden_cols] = 1e30
        dec.V[:, :, :, hidden_cols] = -1e30
    assert np.array_equal(run(poison), base)
    seen_cols = [j for j in range(dec.N) if vis[j] and j != dec.slot_start[f] + o]
    for j in (seen_cols[0], seen_cols[-1]):
        def nudge(j=j):
            dec.V[0, 0, 0, j] += 1.0
        assert not np.array_equal(run(nudge), base)


def test_branch_order_only_permutes_outputs():
    tpl = edgeless_template(4, 3, 5, TINY.vocab)
    w, prefix = _tiny_setup(tpl, seed_cfg=3)
    toks = draw_tokens(3, 4, TINY.vocab)
    perm = [2, 0, 3, 1]
    outs = []
    for order in (list(range(4)), perm):
        dec = O.OracleDecoder(TINY, w, 5, tpl.slot_len, tpl.edges)
        dec.prefill_prefix(0, prefix)
        outs.append(dec.step([order], [[0] * 4], tok_in=toks[order].reshape(1, 4, 1))["logits"])
    assert np.allclose(outs[1], outs[0][perm], rtol=1e-12, atol=1e-12)


def test_multi_token_step_equals_single_token_steps():
    tpl = random_dag_template(4, n_fields=3, prefix_len=4, max_slot=4, edge_prob=1.0, vocab=TINY.vocab)
    tpl.slot_len = [4, 4, 4]
    w, prefix = _tiny_setup(tpl, seed_cfg=4)
    toks = draw_tokens(4, 4, TINY.vocab)
    a = O.OracleDecoder(TINY, w, 4, tpl.slot_len, [])
    a.prefill_prefix(0, prefix)
    one = [a.step([[1]], [[t]], tok_in=[[[int(toks[t])]]])["logits"][0] for t in range(4)]
    b = O.OracleDecoder(TINY, w, 4, tpl.slot_len, [])
    b.prefill_prefix(0, prefix)
    multi = b.step([[1]], [[0]], tok_in=toks.reshape(1, 1, 4), T=4)["logits"]
    assert np.allclose(multi, np.array(one), rtol=1e-11, atol=1e-11)
    assert np.array_equal(a.valid_len, b.valid_len)


def test_two_scenes_are_independent():
    tpl = random_dag_template(8, n_fields=3, prefix_len=3, max_slot=3, edge_prob=0.5, vocab=TINY.vocab)
    w, _ = _tiny_setup(tpl, seed_cfg=5)
    pre = [draw_prefix_embeddings(5, 3, TINY.d_model, extra=i).astype(np.float64) for i in range(2)]
    toks = draw_tokens(5, 2, TINY.vocab)
    both = O.OracleDecoder(TINY, w, 3, tpl.slot_len, tpl.edges, n_scenes=2)
    for b in range(2):
        both.prefill_prefix(b, pre[b])
    out = both.step([[0], [0]], [[0], [0]], tok_in=toks.reshape(2, 1, 1))["logits"]
    for b in range(2):
        solo = O.OracleDecoder(TINY, w, 3, tpl.slot_len, tpl.edges)
        solo.prefill_prefix(0, pre[b])
        want = solo.step([[0]], [[0]], tok_in=[[[int(toks[b])]]])["logits"]
        assert np.allclose(out[b], want[0], rtol=1e-12, atol=1e-12)


# ---------------------------------------------------------------- scheduler
def _critical_path(F, edges, lens):
    cp = [0] * F
    for f in range(F):                      # field order is topological
        cp[f] = lens[f] + max([cp[u] for (u, v) in edges if v == f], default=0)
    return max(cp) if F else 0


@pytest.mark.parametrize("seed", range(12))
def test_schedule_is_optimal_and_respects_dependencies(seed):
    """Sec. 3.2: number of passes = critical-path length; Sec. 3.3: every
    token is decoded exactly once (no recomputation)."""
    tpl = random_dag_template(100 + seed, n_fields=3 + seed, prefix_len=2, max_slot=6,
                              edge_prob=0.3, vocab=10)
    F = tpl.n_fields
    steps = O.schedule(F, tpl.edges, tpl.content_len)
    assert len(steps) == _critical_path(F, tpl.edges, tpl.content_len)
    seen = {}
    for si, st in enumerate(steps):
        for (f, o) in st:
            assert (f, o) not in seen
            seen[(f, o)] = si
    assert sorted(seen) == [(f, o) for f in range(F) for o in range(tpl.content_len[f])]
    for (u, v) in tpl.edges:                # v starts only after u is complete
        assert seen[(v, 0)] > seen[(u, tpl.content_len[u] - 1)]
    for f in range(F):                      # one token per field per pass, in order
        assert [seen[(f, o)] for o in range(tpl.content_len[f])] == \
            list(range(seen[(f, 0)], seen[(f, 0)] + tpl.content_len[f]))
    assert sum(len(s) for s in steps) == sum(tpl.content_len)


def test_workload_templates_are_valid_and_shaped_as_stated():
    t0 = template(0)
    assert t0.edges == [(0, 3), (1, 3), (2, 3)] and t0.slot_len == [8] * 4 and t0.prefix_len == 128
    steps = O.schedule(4, t0.edges, t0.content_len)
    assert len(steps) == 16 and [len(s) for s in steps] == [3] * 8 + [1] * 8
    t1 = template(1)
    assert all(16 <= c <= 48 for c in t1.content_len) and len(t1.edges) == 12
    t2 = template(2)
    O.check_template(12, t2.edges)
    lv = O.levels(12, t2.edges)
    assert lv[:8] == [0] * 8 and lv[8:11] == [1] * 3 and lv[11] == 2
    for f in (8, 9, 10):
        assert 2 <= sum(1 for (_, v) in t2.edges if v == f) <= 4
    for rho in (0.0, 0.1, 0.3, 1.0):
        t3 = template(3, rho=rho)
        O.check_template(16, t3.edges)
    assert len(template(3, rho=1.0).edges) == 120 and template(3, rho=0.0).edges == []
    t4 = template(4)
    O.check_template(32, t4.edges)
    assert O.levels(32, t4.edges) == [f // 8 for f in range(32)]


def test_run_cot_free_running_matches_manual_feedback():
    tpl = random_dag_template(21, n_fields=4, prefix_len=3, max_slot=3, edge_prob=0.5, vocab=TINY.vocab)
    w, prefix = _tiny_setup(tpl, seed_cfg=6)
    dec = O.OracleDecoder(TINY, w, 3, tpl.slot_len, tpl.edges)
    dec.prefill_prefix(0, prefix)
    trace = O.run_cot(dec, tpl.content_len, tpl.start_token)
    assert len(trace) == _critical_path(4, tpl.edges, tpl.content_len)
    first = {}
    for st in trace:
        for i, f in enumerate(st["branch_field"]):
            if f < 0:
                continue
            if f not in first:
                assert st["tok_in"][i] == tpl.start_token[f]
            else:
                assert st["tok_in"][i] == first[f]
            first[f] = int(st["out"]["tok"][i])
    assert list(dec.valid_len[0]) == tpl.content_len


# ------------------------------------- Algorithm 1 with real finishing rules
def _tiny_decoder(tpl, seed_cfg, B=1):
    w, _ = _tiny_setup(tpl, seed_cfg=seed_cfg)
    dec = O.OracleDecoder(TINY, w, tpl.prefix_len, tpl.slot_len, tpl.edges, n_scenes=B)
    for b in range(B):
        dec.prefill_prefix(b, draw_prefix_embeddings(seed_cfg + 31 * b, tpl.prefix_len, TINY.d_model)
                           .astype(np.float64))
    return w, dec


def _texts_from_trace(trace, F):
    text = [[] for _ in range(F)]
    for st in trace:
        for i, f in enumerate(st["branch_field"]):
            if f >= 0:
                text[f].append(int(st["out"]["tok"][i]))
    return text


def test_dynamic_driver_without_end_tokens_fills_every_slot():
    """No end token: every field is truncated at its slot length (Sec. 3.3), so the
    run is the static schedule with content_len = slot_len, pass for pass."""
    tpl = random_dag_template(33, n_fields=5, prefix_len=3, max_slot=4, edge_prob=0.4, vocab=TINY.vocab)
    _, dec = _tiny_decoder(tpl, 9)
    res = O.run_cot_dynamic(dec, tpl.start_token)
    assert [len(t) for t in res["text"][0]] == tpl.slot_len
    assert res["passes"] == _critical_path(5, tpl.edges, tpl.slot_len)
    _, dec2 = _tiny_decoder(tpl, 9)
    assert res["text"][0] == _texts_from_trace(O.run_cot(dec2, tpl.slot_len, tpl.start_token), 5)
    assert list(dec.valid_len[0]) == tpl.slot_len


@pytest.mark.parametrize("seed", range(6))
def test_dynamic_driver_end_tokens_finish_fields_and_passes_are_minimal(seed):
    """A field ends at its first end token or at its slot length; the number of
    passes is the critical path of the lengths that came out (Sec. 3.2:
    optimal), and the tokens are those of the static schedule for those lengths."""
    tpl = random_dag_template(50 + seed, n_fields=6, prefix_len=2, max_slot=5, edge_prob=0.35,
                              vocab=TINY.vocab)
    eos = set(range(0, TINY.vocab, 3))                        # a third of the vocabulary ends a line
    _, dec = _tiny_decoder(tpl, 11 + seed)
    res = O.run_cot_dynamic(dec, tpl.start_token, eos)
    text = res["text"][0]
    lens = [len(t) for t in text]
    for f, t in enumerate(text):
        assert 1 <= len(t) <= tpl.slot_len[f]
        assert not any(x in eos for x in t[:-1])
        assert t[-1] in eos or len(t) == tpl.slot_len[f]
    assert res["passes"] == _critical_path(6, tpl.edges, lens)
    assert list(dec.valid_len[0]) == lens
    _, dec2 = _tiny_decoder(tpl, 11 + seed)
    assert text == _texts_from_trace(O.run_cot(dec2, lens, tpl.start_token), 6)
    if seed == 0:
        assert len(set(lens)) > 1 and any(l < s for l, s in zip(lens, tpl.slot_len))


def test_dynamic_driver_on_a_chain_is_greedy_autoregressive_decoding_with_stop_tokens():
    """Chain-shaped graph = the autoregressive baseline (Sec. 4.1): compared with a
    plain causal decoder that re-reads the whole sequence for every token."""
    F, S, P = 3, 4, 4
    tpl = chain_template(F, S, P, TINY.vocab)
    w, dec = _tiny_decoder(tpl, 13)
    prefix = draw_prefix_embeddings(13, P, TINY.d_model).astype(np.float64)
    eos = set(range(1, TINY.vocab, 4))
    res = O.run_cot_dynamic(dec, tpl.start_token, eos)
    emb = np.asarray(w["emb"], dtype=np.float64)
    rows, pos, want = [r for r in prefix], list(range(P)), []
    for f in range(F):
        tok, out = tpl.start_token[f], []
        for o in range(S):
            rows.append(emb[tok])
            pos.append(P + f * S + o)
            logits, _ = _torch_reference_logits(TINY, w, np.array(rows), np.array(pos))
            tok = int(np.argmax(logits[-1]))
            out.append(tok)
            if tok in eos:
                break
        want.append(out)
    assert res["text"][0] == want
    assert res["passes"] == sum(len(t) for t in want)


def test_dynamic_driver_scenes_diverge_and_stay_independent():
    """Sec. 3.2: field lengths differ from case to case, so scenes sharing a
    pass have different ready sets; each scene's result is that of running it alone."""
    tpl = random_dag_template(77, n_fields=5, prefix_len=3, max_slot=5, edge_prob=0.4, vocab=TINY.vocab)
    eos = set(range(0, TINY.vocab, 3))
    w, dec = _tiny_decoder(tpl, 17, B=2)
    res = O.run_cot_dynamic(dec, tpl.start_token, eos)
    alone = []
    for b in range(2):
        d1 = O.OracleDecoder(TINY, w, tpl.prefix_len, tpl.slot_len, tpl.edges)
        d1.prefill_prefix(0, draw_prefix_embeddings(17 + 31 * b, tpl.prefix_len, TINY.d_model).astype(np.float64))
        alone.append(O.run_cot_dynamic(d1, tpl.start_token, eos))
        assert res["text"][b] == alone[b]["text"][0]
    assert res["text"][0] != res["text"][1]
    assert res["passes"] == max(a["passes"] for a in alone)
    assert any((p["branch_field"][0] != p["branch_field"][1]).any() for p in res["trace"])


def test_dynamic_driver_fixed_text_is_visible_like_a_longer_prefix():
    """Sec. 3.3: fixed template tokens are pre-filled and visible to every later
    token.  A header field that every other field depends on and whose slot it
    fills must act exactly like the same tokens appended to the prefix."""
    P, H = 3, 2
    body = random_dag_template(91, n_fields=4, prefix_len=P + H, max_slot=4, edge_prob=0.4, vocab=TINY.vocab)
    header = [7, 19]
    edges = [(0, v + 1) for v in range(4)] + [(u + 1, v + 1) for (u, v) in body.edges]
    slot_len = [H] + body.slot_len
    start = [0] + body.start_token
    eos = set(range(2, TINY.vocab, 3))
    w, _ = _tiny_setup(body, seed_cfg=19)
    prefix = draw_prefix_embeddings(19, P, TINY.d_model).astype(np.float64)
    dec = O.OracleDecoder(TINY, w, P, slot_len, edges)
    dec.prefill_prefix(0, prefix)
    res = O.run_cot_dynamic(dec, start, eos, fixed={0: header})
    assert res["text"][0][0] == header
    ref = O.OracleDecoder(TINY, w, P + H, body.slot_len, body.edges)
    emb = np.asarray(w["emb"], dtype=np.float64)
    ref.prefill_prefix(0, np.concatenate([prefix, emb[header]]))
    want = O.run_cot_dynamic(ref, body.start_token, eos)
    assert res["text"][0][1:] == want["text"][0]
    assert res["passes"] == want["passes"]
    with pytest.raises(ValueError):
        O.run_cot_dynamic(dec, start, eos, fixed={1: [3]})     # field 1 depends on the unfixed field 0


def test_dynamic_driver_fast_response_and_post_cot_continuation():
    """Two template shapes the paper names (Sec. 3.3 and its discussion): a branch
    decoded alongside the CoT that depends on nothing (a fast response), and a
    final branch after the CoT that sees every non-padding CoT token.  With a
    chain-shaped CoT the final branch must equal ordinary causal decoding over
    prefix + CoT tokens (padding and the fast response skipped, position ids
    kept), and the fast response must equal decoding its field alone."""
    P, S = 4, 4
    slot_len = [S, S, S, 3, 3]                      # CoT fields 0-2 (a chain), 3: fast response, 4: final
    edges = [(0, 1), (1, 2), (0, 4), (1, 4), (2, 4)]
    start = [5, 9, 13, 21, 33]
    eos = set(range(1, TINY.vocab, 4))
    tpl = chain_template(3, S, P, TINY.vocab)       # only for the weight draw
    w, _ = _tiny_setup(tpl, seed_cfg=23)
    prefix = draw_prefix_embeddings(23, P, TINY.d_model).astype(np.float64)
    dec = O.OracleDecoder(TINY, w, P, slot_len, edges)
    dec.prefill_prefix(0, prefix)
    res = O.run_cot_dynamic(dec, start, eos)
    text = res["text"][0]
    first = res["trace"][0]["branch_field"][0]
    assert list(first[first >= 0]) == [0, 3]        # the fast response starts with the first CoT field
    # the fast response alone: a decoder that only ever steps field 3
    alone = O.OracleDecoder(TINY, w, P, slot_len, edges)
    alone.prefill_prefix(0, prefix)
    tok, want = start[3], []
    for o in range(slot_len[3]):
        tok = int(alone.step([[3]], [[o]], tok_in=[[[tok]]])["tok"][0])
        want.append(tok)
        if tok in eos:
            break
    assert text[3] == want
    # the final branch: plain causal decoding over prefix + the CoT's written tokens + its own
    emb = np.asarray(w["emb"], dtype=np.float64)
    slot_start, _ = O.slot_layout(P, slot_len)
    rows, pos = [r for r in prefix], list(range(P))
    for f in range(3):
        inputs = [start[f]] + text[f][:-1]
        for o, t in enumerate(inputs):
            rows.append(emb[t])
            pos.append(slot_start[f] + o)
    tok, want = start[4], []
    for o in range(slot_len[4]):
        rows.append(emb[tok])
        pos.append(slot_start[4] + o)
        logits, _ = _torch_reference_logits(TINY, w, np.array(rows), np.array(pos))
        tok = int(np.argmax(logits[-1]))
        want.append(tok)
        if tok in eos:
            break
    assert text[4] == want
    # it started only after the whole chain had finished
    started = next(i for i, p in enumerate(res["trace"]) if 4 in p["branch_field"][0])
    assert started == sum(len(text[f]) for f in range(3))
