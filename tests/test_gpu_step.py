"""GPU parity of the whole parallel decoding step (Sec. 3.3) through the C
ABI against the fp64 oracle: hidden states within 2e-3 (max |err| / max |ref|
per tensor), greedy ids identical where the oracle's top-2 gap exceeds 1e-2,
valid lengths and inactive rows exact.  Steps are teacher-forced with the
oracle's tokens."""
import numpy as np
import pytest

import oracle.fdc_oracle as O
from synth_inputs import (ModelDims, bf16_round, chain_template, draw_layer_weights,
                          draw_normal_bf16, draw_prefix_embeddings, draw_tokens, draw_weights,
                          model_dims, random_dag_template, template, workload_seed)
from tests.helpers import HIDDEN_TOL, Pair, rel_err, run_schedule

pytestmark = pytest.mark.gpu


def _random_prefix_kv(pair, cfg_id, scene=0):
    d, P = pair.dims, pair.tpl.prefix_len
    rng = workload_seed(cfg_id, "prefix", 50 + scene)
    K = draw_normal_bf16(rng, (d.n_layers, d.n_kv_heads, P, d.head_dim))
    V = draw_normal_bf16(rng, (d.n_layers, d.n_kv_heads, P, d.head_dim))
    pair.install_prefix_kv(scene, K, V)


def test_workload0_whole_schedule():
    """Tiny layer, 4 fields (0-2 independent, 3 depends on all), 8-token slots:
    8 passes of 3 branches, then 8 passes of the dependent field."""
    dims = model_dims(0)
    tpl = template(0)
    w = draw_weights(0, dims, random_gains=True)
    pair = Pair(dims, tpl, w)
    pair.prefill_with_oracle(0, draw_prefix_embeddings(0, tpl.prefix_len, dims.d_model))
    worst, n = run_schedule(pair, tpl.content_len, tpl.start_token, tag="cfg0")
    assert n == 16
    assert list(pair.ctx.get_valid_len()[0]) == [8, 8, 8, 8]
    pair.close()


def _random_model_steps(seed, B, T, R, dims, n_fields=5, max_slot=9, n_steps=6, f16_weights=None):
    tpl = random_dag_template(900 + seed, n_fields=n_fields, prefix_len=19 + seed, max_slot=max_slot,
                              edge_prob=0.4, vocab=dims.vocab)
    tpl.slot_len = [max(s, T) for s in tpl.slot_len]
    w = draw_weights(10 + seed, dims, random_gains=True, std=0.05)
    R = min(R, tpl.n_fields)
    pair = Pair(dims, tpl, w, n_scenes=B, max_branches=R, max_tokens=T, f16_weights=f16_weights)
    for b in range(B):
        pair.prefill_with_oracle(b, draw_prefix_embeddings(10 + seed, tpl.prefix_len, dims.d_model, extra=b))
    rng = np.random.default_rng(seed)
    F = tpl.n_fields
    done = np.zeros((B, F), dtype=int)
    ran = 0
    for step in range(n_steps):
        bf = np.full((B, R), -1, dtype=np.int32)
        bo = np.zeros((B, R), dtype=np.int32)
        for b in range(B):
            # any field whose parents are complete and that still has room may go
            ready = [f for f in range(F) if done[b, f] + T <= tpl.slot_len[f] and
                     all(done[b, u] > 0 for (u, v) in tpl.edges if v == f)]
            rng.shuffle(ready)
            for i, f in enumerate(ready[:int(rng.integers(0, R + 1))]):
                bf[b, i], bo[b, i] = f, done[b, f]
        if (bf < 0).all():
            continue
        tok = rng.integers(0, dims.vocab, size=(B, R, T)).astype(np.int32)
        pair.step_both(bf, bo, tok, T=T, tag=f"seed{seed} step{step}")
        ran += 1
        for b in range(B):
            for i in range(R):
                if bf[b, i] >= 0:
                    done[b, bf[b, i]] += T
    pair.close()
    return ran


@pytest.mark.parametrize("seed,B,T,D", [(0, 2, 1, 64), (1, 1, 2, 128), (2, 3, 1, 128), (3, 2, 3, 64)])
def test_random_small_models_ragged_templates(seed, B, T, D):
    """Ragged slots and prefix, random gains, several scenes in different
    states, inactive branch entries, multi-token steps."""
    dims = ModelDims(n_layers=2, d_model=128, n_q_heads=4, n_kv_heads=2, head_dim=D, d_mlp=160,
                     vocab=500 + 4 * seed)
    assert _random_model_steps(seed, B, T, max(1, 16 // (B * T)), dims) >= 3


@pytest.mark.parametrize("seed,B,T,R,Hq,Hkv,D,F", [(4, 4, 2, 5, 4, 2, 64, 5),      # 40 rows
                                                   (5, 3, 4, 6, 14, 2, 64, 8),     # 72 rows, 168 per kv head
                                                   (6, 8, 4, 5, 8, 2, 128, 6),     # 160 rows: two row blocks
                                                   (7, 2, 3, 3, 4, 4, 128, 4),     # 18 rows: just above 16
                                                   (8, 8, 4, 32, 8, 2, 64, 32)])   # up to 1024 rows: the row limit
@pytest.mark.parametrize("f16", ["all", None])
def test_many_rows_per_step_use_the_tiled_projections(seed, B, T, R, Hq, Hkv, D, F, f16):
    """More than 16 rows in a step (several scenes, several tokens per branch:
    the multi-token masked prefill inside a slot): the projections switch to the
    tiled matrix-core kernels - two-pass (bf16 head + tail activations) on the
    bf16 weights with only the LM head single-pass on its fp16 copy (the default),
    or every projection single-pass on fp16 copies ("all") - and attention to
    several row groups per KV head."""
    dims = ModelDims(n_layers=2, d_model=Hq * 32, n_q_heads=Hq, n_kv_heads=Hkv, head_dim=D, d_mlp=352,
                     vocab=600 + 4 * seed)
    assert _random_model_steps(seed, B, T, R, dims, n_fields=F, max_slot=12, n_steps=5, f16_weights=f16) >= 2


def test_wide_mlp_at_256_rows_uses_the_eight_wavefront_projection():
    """An MLP wide enough (2 x 8320 gate/up features at 256 rows) that the gate/up
    projection takes the wide tile: the eight-wavefront kernel with weights
    straight into registers and the gate/up pair that is split between two
    wavefronts; a vocabulary that makes the LM head take it too."""
    dims = ModelDims(n_layers=2, d_model=64, n_q_heads=2, n_kv_heads=1, head_dim=64, d_mlp=8320, vocab=17000)
    for f16 in ("all", None, False):
        assert _random_model_steps(9, 8, 4, 8, dims, n_fields=8, max_slot=12, n_steps=3, f16_weights=f16) >= 2


@pytest.mark.parametrize("seed,B,P,chunk,D", [(30, 1, 70, 16, 64), (31, 2, 45, 32, 128)])
def test_prefix_prefill_through_the_step(seed, B, P, chunk, D):
    """The prefix as field 0 of a context over the same cache: stepping it with
    `chunk` tokens per pass is the causal prefill.  Its final hidden rows match the
    oracle's plain causal pass, and decoding on top of the prefilled cache matches
    the oracle decoding on top of its own prefill."""
    dims = ModelDims(n_layers=2, d_model=128, n_q_heads=4, n_kv_heads=2, head_dim=D, d_mlp=160, vocab=520)
    tpl = random_dag_template(900 + seed, n_fields=4, prefix_len=P, max_slot=8, edge_prob=0.5, vocab=dims.vocab)
    w = draw_weights(10 + seed, dims, random_gains=True, std=0.05)
    pair = Pair(dims, tpl, w, n_scenes=B, max_branches=tpl.n_fields)
    view = pair.ctx.prefill_view(max_tokens=chunk)
    emb = np.stack([draw_prefix_embeddings(10 + seed, P, dims.d_model, extra=b) for b in range(B)])
    emb = bf16_round(emb.astype(np.float32))
    out = view.prefill(emb, chunk)
    import torch
    torch.cuda.synchronize()
    last = min(chunk, P - (P - 1) // chunk * chunk)          # rows of the last pass
    hid = out["hidden"].cpu().numpy()[dims.n_layers].reshape(B, last, dims.d_model)
    for b in range(B):
        x = pair.dec.prefill_prefix(b, emb[b])
        assert rel_err(hid[b], x[P - last:]) <= HIDDEN_TOL
    # the cache is bf16 storage on both sides
    pair.dec.K[:, :, :, :P] = bf16_round(pair.dec.K[:, :, :, :P].astype(np.float32))
    pair.dec.V[:, :, :, :P] = bf16_round(pair.dec.V[:, :, :, :P].astype(np.float32))
    assert list(view.get_valid_len()[:, 0]) == [P] * B
    roots = [f for f in range(tpl.n_fields) if not any(v == f for _, v in tpl.edges)]
    rng = np.random.default_rng(seed)
    for step in range(3):
        bf = np.full((B, tpl.n_fields), -1, dtype=np.int32)
        bo = np.zeros((B, tpl.n_fields), dtype=np.int32)
        for b in range(B):
            for i, f in enumerate(roots):
                if step < tpl.slot_len[f]:
                    bf[b, i], bo[b, i] = f, step
        if (bf < 0).all():
            break
        tok = rng.integers(0, dims.vocab, size=(B, tpl.n_fields, 1)).astype(np.int32)
        pair.step_both(bf, bo, tok, tag=f"after prefill, step {step}")
    view.close()
    pair.close()


def test_chain_dag_on_gpu_is_causal_decoding():
    """Chain-shaped graph: the GPU path reproduces ordinary autoregressive
    decoding (the oracle is pinned to a plain causal decoder on the CPU)."""
    dims = ModelDims(n_layers=2, d_model=256, n_q_heads=4, n_kv_heads=4, head_dim=64, d_mlp=512, vocab=1000)
    tpl = chain_template(3, 4, 40, dims.vocab)
    w = draw_weights(20, dims, random_gains=True, std=0.04)
    pair = Pair(dims, tpl, w, max_branches=1)
    pair.prefill_with_oracle(0, draw_prefix_embeddings(20, 40, dims.d_model))
    toks = draw_tokens(20, 12, dims.vocab)
    for i in range(12):
        ref, got = pair.step_both([[i // 4]], [[i % 4]], [int(toks[i])], tag=f"chain {i}")
        assert ref["pos"][0] == 40 + i
    pair.close()


def test_workload1_shapes_two_layers():
    """0.5B-class widths (896 / 14 q heads / 2 kv heads / 64 / 4864 / vocab 32000),
    2 layers, the 8-field template, first passes and the dependent fields."""
    dims = model_dims(1, n_layers=2)
    tpl = template(1)
    w = draw_weights(1, dims, random_gains=True)
    pair = Pair(dims, tpl, w)
    _random_prefix_kv(pair, 1)
    lens = [3, 2, 3, 2, 3, 2, 2, 2]            # short contents: reach the dependent fields quickly
    worst, n = run_schedule(pair, lens, tpl.start_token, tag="cfg1")
    assert n == 5
    pair.close()


def test_workload2_shapes_two_layers():
    """7B-class widths (3584 / 28 q / 4 kv / 128 / 18944 / vocab 32000), 2 layers,
    the 12-field 3-level template: 8 roots, then the middle level, then the final field."""
    dims = model_dims(2, n_layers=2)
    tpl = template(2)
    w = {"layers": [draw_layer_weights(2, dims, l, random_gains=True) for l in range(2)]}
    rng = workload_seed(2, "weights", 0)
    w["emb"] = draw_normal_bf16(rng, (dims.vocab, dims.d_model), 0.02)
    w["gf"] = draw_normal_bf16(rng, (dims.d_model,), 0.02, 1.0)
    w["lm"] = draw_normal_bf16(rng, (dims.vocab, dims.d_model), 0.02)
    pair = Pair(dims, tpl, w)
    _random_prefix_kv(pair, 2)
    lens = [2, 1, 2, 1, 2, 1, 2, 1, 2, 1, 2, 2]
    worst, n = run_schedule(pair, lens, tpl.start_token, tag="cfg2")
    assert n == 6
    pair.close()


def test_workload4_shapes_one_layer_256_rows():
    """Workload-4 shapes at full width (7B-class layer, 8 scenes, prefix 8192, 32 fields
    of 32-token slots in 4 levels, 4 tokens per branch per pass = 256 rows): the tiled
    projections and four row groups per KV head in the launch shape the benchmark
    times; one pass of the first level on one layer (the oracle's cost)."""
    dims = model_dims(4, n_layers=1)
    tpl = template(4)
    w = {"layers": [draw_layer_weights(4, dims, 0, random_gains=True)]}
    rng = workload_seed(4, "weights", 0)
    w["emb"] = draw_normal_bf16(rng, (dims.vocab, dims.d_model), 0.02)
    w["gf"] = draw_normal_bf16(rng, (dims.d_model,), 0.02, 1.0)
    w["lm"] = draw_normal_bf16(rng, (dims.vocab, dims.d_model), 0.02)
    B, R, T = 8, 8, 4
    pair = Pair(dims, tpl, w, n_scenes=B, max_branches=R, max_tokens=T)
    for b in range(B):
        _random_prefix_kv(pair, 4, scene=b)
    trng = np.random.default_rng(44)
    bf = np.tile(np.arange(R, dtype=np.int32), (B, 1))
    tok = trng.integers(0, dims.vocab, size=(B, R, T)).astype(np.int32)
    pair.step_both(bf, np.zeros((B, R), dtype=np.int32), tok, T=T, tag="cfg4 level 0")
    pair.close()


def _cfg_head_weights(cfg_id, dims):
    rng = workload_seed(cfg_id, "weights", 0)
    return {"emb": draw_normal_bf16(rng, (dims.vocab, dims.d_model), 0.02),
            "gf": draw_normal_bf16(rng, (dims.d_model,), 0.02, 1.0),
            "lm": draw_normal_bf16(rng, (dims.vocab, dims.d_model), 0.02)}


def test_workload4_three_layers_two_passes_256_rows():
    """Workload 4 at full width beyond one layer: three 7B-class layers, 8 scenes,
    prefix 8192, the first level's 8 fields with 4 tokens per pass (256 rows, the
    launch shape the benchmark times), two passes in a row - the second reads, in
    every layer, the K/V the first one stored.  Mask and positions of all 256 rows
    bit for bit; hidden states after every layer and logits against the oracle on
    two of the eight scenes (scenes are independent)."""
    import torch
    dims = model_dims(4, n_layers=3)
    tpl = template(4)
    w = {"layers": [draw_layer_weights(4, dims, l, random_gains=True) for l in range(dims.n_layers)],
         **_cfg_head_weights(4, dims)}
    B, R, T = 8, 8, 4
    sample = [2, 5]
    pair = Pair(dims, tpl, w, n_scenes=B, max_branches=R, max_tokens=T)
    sub = O.OracleDecoder(dims, w, tpl.prefix_len, tpl.slot_len, tpl.edges, len(sample), kv_bf16=True)
    shp = (dims.n_layers, dims.n_kv_heads, tpl.prefix_len, dims.head_dim)
    for b in range(B):
        prng = workload_seed(4, "prefix", 70 + b)
        K, V = draw_normal_bf16(prng, shp), draw_normal_bf16(prng, shp)
        pair.install_prefix_kv(b, K, V)
        if b in sample:
            sub.set_prefix_kv(sample.index(b), K, V)
    trng = np.random.default_rng(46)
    bf = np.tile(np.arange(R, dtype=np.int32), (B, 1))
    rows_g = np.concatenate([np.arange(b * R * T, (b + 1) * R * T) for b in sample])
    L = dims.n_layers
    for step in range(2):
        bo = np.full((B, R), step * T, dtype=np.int32)
        tok = trng.integers(0, dims.vocab, size=(B, R, T)).astype(np.int32)
        g = pair.ctx.parallel_decode_step(bf, bo, tok_in=tok, T=T, want_logits=True, want_hidden=True)
        torch.cuda.synchronize()
        got = {k: v.cpu().numpy() for k, v in g.items() if not k.startswith("_")}
        pair.dec.valid_len[:, :R] = (step + 1) * T
        assert np.array_equal(pair.ctx.get_valid_len(), pair.dec.valid_len)
        pair.compare_tables(bf, bo, T, f"cfg4 three layers, pass {step}")
        ref = sub.step(bf[sample], bo[sample], tok_in=tok[sample], T=T)
        errs = [rel_err(got["hidden"][l][rows_g], ref["hidden"][l]) for l in range(L + 1)]
        errs.append(rel_err(got["hidden"][L + 1][rows_g], ref["normed"]))
        errs.append(rel_err(got["logits"][rows_g], ref["logits"]))
        assert max(errs) <= ARITH_BOUND, (step, errs)
        sure = np.nonzero(ref["gap"] > 1e-2)[0]
        assert sure.size > 0
        assert np.array_equal(got["tok"][rows_g][sure], ref["tok"][sure])
    pair.close(need_sure=False)


def test_workload4_all_active_1024_rows_full_width():
    """The all-active half of workload 4 at full width, in the launch shape the
    benchmark's stress run times: 8 scenes x 32 fields x 4 tokens = 1024 rows
    through one 7B-class layer, prefix 8192, fourteen row groups per KV head.
    Every slot already holds 12 tokens (history installed as data on both sides),
    so every field attends to 16 tokens of each of its ancestors.  The device's
    mask and positions are compared for all 1024 rows; hidden states and logits
    against the oracle on two of the eight scenes (scenes are independent; the
    oracle takes about a minute per four scenes)."""
    dims = model_dims(4, n_layers=1)
    tpl = template(4)
    w = {"layers": [draw_layer_weights(4, dims, 0, random_gains=True)], **_cfg_head_weights(4, dims)}
    B, R, T, hist = 8, tpl.n_fields, 4, 12
    sample = [1, 6]
    pair = Pair(dims, tpl, w, n_scenes=B, max_branches=R, max_tokens=T)
    sub = O.OracleDecoder(dims, w, tpl.prefix_len, tpl.slot_len, tpl.edges, len(sample), kv_bf16=True)
    shp = (dims.n_layers, dims.n_kv_heads, tpl.prefix_len, dims.head_dim)
    hshp = (dims.n_layers, dims.n_kv_heads, hist, dims.head_dim)
    for b in range(B):
        prng = workload_seed(4, "prefix", 50 + b)
        K, V = draw_normal_bf16(prng, shp), draw_normal_bf16(prng, shp)
        hk = [(draw_normal_bf16(prng, hshp), draw_normal_bf16(prng, hshp)) for _ in range(R)]
        if b in sample:
            i = sample.index(b)
            sub.set_prefix_kv(i, K, V)
            for f, (k, v) in enumerate(hk):
                s0 = sub.slot_start[f]
                sub.K[:, i, :, s0:s0 + hist], sub.V[:, i, :, s0:s0 + hist] = k, v
        # the full-batch oracle object only carries state (valid lengths) for the table check
        for l in range(dims.n_layers):
            pos = np.concatenate([np.arange(tpl.prefix_len)] +
                                 [np.arange(pair.dec.slot_start[f], pair.dec.slot_start[f] + hist) for f in range(R)])
            kk = np.concatenate([K[l]] + [k[l] for k, _ in hk], axis=1)
            vv = np.concatenate([V[l]] + [v[l] for _, v in hk], axis=1)
            pair.ctx.kv_append(l, np.ascontiguousarray(np.transpose(kk, (1, 0, 2)), dtype=np.float32),
                               np.ascontiguousarray(np.transpose(vv, (1, 0, 2)), dtype=np.float32),
                               np.full(pos.size, b, dtype=np.int32), pos.astype(np.int32))
    pair.dec.valid_len[:] = hist
    sub.valid_len[:] = hist
    pair.ctx.set_valid_len(pair.dec.valid_len)
    trng = np.random.default_rng(45)
    bf = np.tile(np.arange(R, dtype=np.int32), (B, 1))
    bo = np.full((B, R), hist, dtype=np.int32)
    tok = trng.integers(0, dims.vocab, size=(B, R, T)).astype(np.int32)
    import torch
    g = pair.ctx.parallel_decode_step(bf, bo, tok_in=tok, T=T, want_logits=True, want_hidden=True)
    torch.cuda.synchronize()
    got = {k: v.cpu().numpy() for k, v in g.items() if not k.startswith("_")}
    pair.dec.valid_len[:] = hist + T                    # what the step leaves behind
    assert np.array_equal(pair.ctx.get_valid_len(), pair.dec.valid_len)
    pair.compare_tables(bf, bo, T, "cfg4 all active")   # all 1024 rows, bit for bit
    assert np.isfinite(got["logits"]).all()
    ref = sub.step(bf[sample], bo[sample], tok_in=tok[sample], T=T)
    rows_g = np.concatenate([np.arange(b * R * T, (b + 1) * R * T) for b in sample])
    L = dims.n_layers
    errs = [rel_err(got["hidden"][l][rows_g], ref["hidden"][l]) for l in range(L + 1)]
    errs.append(rel_err(got["hidden"][L + 1][rows_g], ref["normed"]))
    errs.append(rel_err(got["logits"][rows_g], ref["logits"]))
    assert max(errs) <= HIDDEN_TOL, errs
    sure = np.nonzero(ref["gap"] > 1e-2)[0]
    assert sure.size > 0
    assert np.array_equal(got["tok"][rows_g][sure], ref["tok"][sure])
    pair.close(need_sure=False)


def test_step_error_paths_leave_state_unchanged():
    from paper_2602_02864_amd import FdcError, binding as fb
    dims = model_dims(0)
    tpl = template(0)
    pair = Pair(dims, tpl, draw_weights(0, dims, random_gains=False))
    ctx = pair.ctx
    before = ctx.get_valid_len().copy()
    for args, code in [(([0, 1, 2, 3, 0], [0] * 5), fb.FDC_ECAP),        # R above max_branches
                       (([4], [0]), fb.FDC_ERANGE),                       # field id
                       (([0], [8]), fb.FDC_ERANGE),                       # offset beyond slot
                       (([0], [-1]), fb.FDC_ERANGE),
                       (([0], [3]), fb.FDC_ERANGE),                       # a gap: the slot holds no tokens yet
                       (([1, 1], [0, 0]), fb.FDC_EINVAL)]:                # one field twice in a scene
        with pytest.raises(FdcError) as e:
            ctx.parallel_decode_step(args[0], args[1], tok_in=[0] * len(args[0]))
        assert e.value.code == code
    with pytest.raises(FdcError) as e:
        ctx.parallel_decode_step([0], [0])                                 # neither tokens nor rows
    assert e.value.code == fb.FDC_EINVAL
    with pytest.raises(FdcError) as e:                                     # logits of a pass that runs no head
        ctx.parallel_decode_step([0], [0], tok_in=[0], want_logits=True, want_tokens=False)
    assert e.value.code == fb.FDC_EINVAL
    assert np.array_equal(ctx.get_valid_len(), before)
    pair.close()


def test_pass_without_tokens_fills_the_cache_like_any_other():
    """A pass that asks for no tokens (a prefill pass) skips the LM head and the
    argmax; the residual stream it reports and the K/V it leaves are those of the
    same pass with the head: the next step, which reads that K/V, matches the
    oracle either way."""
    import torch
    dims = model_dims(0)
    tpl = template(0)
    w = draw_weights(0, dims, random_gains=True)
    pair = Pair(dims, tpl, w)
    _random_prefix_kv(pair, 0)
    full = pair.ctx.parallel_decode_step([0, 1, 2], [0, 0, 0], tok_in=[5, 6, 7], want_hidden=True)
    torch.cuda.synchronize()
    h_full = full["hidden"].cpu().numpy()
    pair.ctx.reset()
    quiet = pair.ctx.parallel_decode_step([0, 1, 2], [0, 0, 0], tok_in=[5, 6, 7], want_hidden=True, want_tokens=False)
    torch.cuda.synchronize()
    assert "tok" not in quiet and np.array_equal(quiet["hidden"].cpu().numpy(), h_full)
    # the oracle takes the same first step, then both take a second one on top of it
    pair.dec.step(np.array([[0, 1, 2]], dtype=np.int32), np.array([[0, 0, 0]], dtype=np.int32),
                  tok_in=np.array([5, 6, 7], dtype=np.int32).reshape(1, 3, 1))
    pair.step_both([[0, 1, 2]], [[1, 1, 1]], [9, 10, 11], tag="after a pass without tokens")
    pair.close()


def test_repeated_runs_are_bit_identical():
    """No atomics, fixed merge orders: the same step twice gives the same bits."""
    import torch
    dims = model_dims(0)
    tpl = template(0)
    pair = Pair(dims, tpl, draw_weights(0, dims, random_gains=True))
    _random_prefix_kv(pair, 0)
    outs = []
    for _ in range(2):
        pair.ctx.reset()
        g = pair.ctx.parallel_decode_step([0, 1, 2], [0, 0, 0], tok_in=[5, 6, 7], want_logits=True)
        torch.cuda.synchronize()
        outs.append(g["logits"].cpu().numpy())
    assert np.array_equal(outs[0], outs[1])
    pair.close()


def _curve_rows(errs_by_name):
    """One curve per name as a table: every fourth layer, the last one, the maximum."""
    n = len(next(iter(errs_by_name.values())))
    pick = sorted({l for l in range(4, n, 4)} | {n - 1})
    out = ["   layer " + " ".join(f"{l:>9d}" for l in pick) + "       max"]
    for name, e in errs_by_name.items():
        out.append(f"   {name:<5s} " + " ".join(f"{e[l]:9.2e}" for l in pick) + f" {max(e):9.2e}")
    return out


def _curve_file(name, lines):
    """Per-layer error curves of a full-depth run, kept as a record next to the
    run's other outputs (profiles/parity_error_curve.txt is these files, one after
    the other)."""
    import os
    d = os.environ.get("FDC_RECORD_DIR") or os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "gpurun_out")
    os.makedirs(d, exist_ok=True)
    with open(os.path.join(d, f"parity_error_curve_{name}.txt"), "w") as f:
        f.write("\n".join(lines) + "\n\n")


def _both_oracles_step(pair, plain, bf, bo, ti, tag, curves):
    """One teacher-forced step on the GPU, on the oracle that stores K/V as bf16
    (the graded comparison) and on the oracle that keeps fp64 K/V (what the
    storage format costs).  Appends the three per-layer curves to `curves`."""
    L = pair.dims.n_layers
    ref, got = pair.step_both([bf], [bo], ti, check=False)
    worst = pair.compare(ref, got, tag)
    ref2 = plain.step([bf], [bo], tok_in=np.array(ti).reshape(1, -1, 1))
    rows = ref2["rows"]
    e_store = [rel_err(got["hidden"][l][rows], ref["hidden"][l][rows]) for l in range(L + 1)]
    e_plain = [rel_err(got["hidden"][l][rows], ref2["hidden"][l][rows]) for l in range(L + 1)]
    e_fmt = [rel_err(ref["hidden"][l][rows], ref2["hidden"][l][rows]) for l in range(L + 1)]
    curves.append((tag, e_store, e_plain, e_fmt))
    # what separates the GPU from the fp64-K/V oracle is the storage format: the two
    # oracles differ by as much
    assert max(e_plain) <= 1.1 * max(e_fmt) + ARITH_BOUND, (tag, max(e_plain), max(e_fmt))
    return ref, worst, max(e_plain), max(e_fmt)


def _curve_lines(title, curves):
    out = [title, "rows: A = GPU vs oracle with bf16 K/V storage (the graded comparison), B = GPU vs oracle with fp64 K/V,",
           "      C = oracle bf16-storage vs oracle fp64 (the storage format alone, CPU only)",
           "metric: max|a - b| / max|b| over the residual stream after a layer"]
    for tag, e_store, e_plain, e_fmt in curves:
        out.append(f"-- {tag}")
        out += _curve_rows({"A": e_store, "B": e_plain, "C": e_fmt})
    return out


_CFG2_BITS = []


def _cfg2_full_depth(max_tokens=1, f16_weights=None):
    from synth_inputs import bits_to_f32
    dims = model_dims(2)
    tpl = template(2)
    if not _CFG2_BITS:          # 6.5 GB of bf16 patterns, drawn once for the tests that use them
        _CFG2_BITS.extend(draw_layer_weights(2, dims, l, random_gains=True, bits=True) for l in range(dims.n_layers))
    bits = _CFG2_BITS

    def layer(l):
        return {k: (bits_to_f32(v) if v.dtype == np.uint16 else v) for k, v in bits[l].items()}
    w = {"layers": layer, **_cfg_head_weights(2, dims)}
    pair = Pair(dims, tpl, w, max_branches=8 if max_tokens > 1 else None, max_tokens=max_tokens,
                f16_weights=f16_weights)
    plain = O.OracleDecoder(dims, w, tpl.prefix_len, tpl.slot_len, tpl.edges, kv_bf16=False)
    prng = workload_seed(2, "prefix", 50)
    shp = (dims.n_layers, dims.n_kv_heads, tpl.prefix_len, dims.head_dim)
    K, V = draw_normal_bf16(prng, shp), draw_normal_bf16(prng, shp)
    pair.install_prefix_kv(0, K, V)
    plain.set_prefix_kv(0, K, V)
    return dims, tpl, pair, plain, prng


# Bounds of the full-depth runs.  Against the oracle that stores K/V as bf16 the
# arithmetic alone is compared and must stay far inside the 2e-3 budget.  Against
# the oracle that keeps fp64 K/V the rounding of newly stored K/V to the cache's
# bf16 format is included: that comparison is bounded by what was measured plus
# ten per cent, and the oracles' own difference (CPU only) shows the format
# accounts for it.
ARITH_BOUND = 5e-4
PLAIN_BOUND_CFG2 = 2.3e-3      # measured 2.09e-3 (first pass, layer 27); the oracles differ by the same 2.09e-3
PLAIN_BOUND_CFG1 = 9.0e-4      # measured 7.8e-4 (first pass of the dependent fields, layer 24)


def test_workload2_full_depth_first_passes():
    """The benchmarked configuration at full size: all 28 layers at 7B-class
    widths, prefix 3072, the first two passes of the schedule (8 branches each),
    against both oracles, layer by layer."""
    dims, tpl, pair, plain, _ = _cfg2_full_depth()
    steps = O.schedule(tpl.n_fields, tpl.edges, tpl.content_len)[:2]
    last = list(tpl.start_token)
    curves = []
    for si, st in enumerate(steps):
        bf = [f for f, _ in st]
        ref, worst, e_plain, e_fmt = _both_oracles_step(pair, plain, bf, [o for _, o in st], [last[f] for f in bf],
                                                        f"cfg2 full depth, pass {si}: 8 roots at offset {si}", curves)
        assert worst < ARITH_BOUND, worst
        assert e_plain < PLAIN_BOUND_CFG2, e_plain
        for i, f in enumerate(bf):
            last[f] = int(ref["tok"][i])
    _curve_file("cfg2_first_passes", _curve_lines("workload 2 (28 layers, 7B-class widths), first passes", curves))
    pair.close()


def test_workload2_full_depth_later_passes():
    """Later passes of workload 2 at all 28 layers: the three middle fields (R = 3,
    each seeing 2-4 complete root fields) and the final field (R = 1, seeing all
    eleven others).  The fields they depend on are installed as data (random K/V
    of their content lengths) on both sides; each pass is run twice in a row so
    that the second also reads K/V the first one stored."""
    dims, tpl, pair, plain, prng = _cfg2_full_depth()
    curves = []

    def history(fields):
        for f in fields:
            n = tpl.content_len[f]
            shp = (dims.n_layers, dims.n_kv_heads, n, dims.head_dim)
            Kf, Vf = draw_normal_bf16(prng, shp), draw_normal_bf16(prng, shp)
            pair.install_slot_kv(0, f, Kf, Vf)
            s0 = plain.slot_start[f]
            plain.K[:, 0, :, s0:s0 + n], plain.V[:, 0, :, s0:s0 + n] = Kf, Vf
            plain.valid_len[0, f] = n
    history(range(8))
    last = list(tpl.start_token)
    for fields, name in (([8, 9, 10], "middle fields 8-10"), ([11], "final field 11")):
        for off in range(2):
            ref, worst, e_plain, e_fmt = _both_oracles_step(
                pair, plain, fields, [off] * len(fields), [last[f] for f in fields],
                f"cfg2 full depth, {name} at offset {off}", curves)
            assert worst < ARITH_BOUND, worst
            assert e_plain < PLAIN_BOUND_CFG2, e_plain
            for i, f in enumerate(fields):
                last[f] = int(ref["tok"][i])
        if fields != [11]:
            # the middle fields complete (their two decoded tokens stay, data fills the rest)
            for f in fields:
                n = tpl.content_len[f] - 2
                shp = (dims.n_layers, dims.n_kv_heads, n, dims.head_dim)
                Kf, Vf = draw_normal_bf16(prng, shp), draw_normal_bf16(prng, shp)
                s0 = plain.slot_start[f] + 2
                for dec in (pair.dec, plain):
                    dec.K[:, 0, :, s0:s0 + n], dec.V[:, 0, :, s0:s0 + n] = Kf, Vf
                    dec.valid_len[0, f] = n + 2
                for l in range(dims.n_layers):
                    pair.ctx.kv_append(l, np.ascontiguousarray(np.transpose(Kf[l], (1, 0, 2)), dtype=np.float32),
                                       np.ascontiguousarray(np.transpose(Vf[l], (1, 0, 2)), dtype=np.float32),
                                       np.zeros(n, dtype=np.int32), np.arange(s0, s0 + n, dtype=np.int32))
            pair.ctx.set_valid_len(pair.dec.valid_len)
    _curve_file("cfg2_later_passes", _curve_lines("workload 2 (28 layers, 7B-class widths), later passes", curves))
    pair.close()


def test_workload2_model_full_depth_32_rows_per_step():
    """The 7B-class model at all 28 layers with 32 rows per step (8 root fields x 4
    given tokens): more than 16 rows, so the projections are the tiled matrix-core
    kernels.  First pass as the library runs by default (layer projections two-pass
    with bf16 head + tail activations, LM head single-pass on its fp16 copy): inside
    the 2e-3 budget with room.  Second pass with EVERY projection single-pass on
    fp16 copies (fp16 activations: 11 significant bits): recorded; it is the reason
    that mode is not the default - about 3e-3 at layer 28."""
    dims, tpl, pair, plain, _ = _cfg2_full_depth(max_tokens=4, f16_weights="all")
    pair.ctx.set_f16_projections(16)               # the default set, on a context that has every copy
    L = dims.n_layers
    rng = np.random.default_rng(77)
    lines = ["workload 2 model (28 layers), 8 branches x 4 tokens = 32 rows per step (tiled projections)",
             "row A = GPU vs oracle with bf16 K/V storage (max|a - b| / max|b| over the residual stream after a layer)"]
    for step, (mask, name) in enumerate([(16, "default: layer projections two-pass bf16 head + tail, LM head fp16"),
                                         (31, "every projection single-pass fp16 (opt-in)")]):
        pair.ctx.set_f16_projections(mask)
        bf = list(range(8))
        tok = rng.integers(0, dims.vocab, size=(1, 8, 4)).astype(np.int32)
        ref, got = pair.step_both([bf], [[4 * step] * 8], tok, T=4, check=False)
        rows = ref["rows"]
        errs = [rel_err(got["hidden"][l][rows], ref["hidden"][l][rows]) for l in range(L + 1)]
        e_log = rel_err(got["logits"][rows], ref["logits"][rows])
        lines.append(f"-- pass {step}, offsets {4 * step}..{4 * step + 3}; {name}; logits {e_log:.3e}")
        lines += _curve_rows({"A": errs})
        if mask == 16:
            worst = pair.compare(ref, got, "32 rows per step, default projections")
            assert worst < ARITH_BOUND, worst
        else:
            assert 5e-4 < max(errs) < 6e-3, max(errs)      # a record of what the shortcut costs, not a parity claim
    _curve_file("cfg2_model_32_rows", lines)
    pair.close(need_sure=False)


def test_workload1_full_depth_schedule_prefix():
    """Workload 1 as benchmarked: all 24 layers at 0.5B-class widths, prefix 1536, the
    8-field template, a whole (shortened) schedule: six passes of the independent
    fields, then three of the two dependent fields, which read 33 decoded K/V rows
    of their ancestors.  Against both oracles, layer by layer."""
    dims = model_dims(1)
    tpl = template(1)
    w = draw_weights(1, dims, random_gains=True)
    pair = Pair(dims, tpl, w)
    plain = O.OracleDecoder(dims, w, tpl.prefix_len, tpl.slot_len, tpl.edges, kv_bf16=False)
    prng = workload_seed(1, "prefix", 50)
    shp = (dims.n_layers, dims.n_kv_heads, tpl.prefix_len, dims.head_dim)
    K, V = draw_normal_bf16(prng, shp), draw_normal_bf16(prng, shp)
    pair.install_prefix_kv(0, K, V)
    plain.set_prefix_kv(0, K, V)
    lens = [6, 5, 6, 5, 6, 5, 3, 3]
    steps = O.schedule(tpl.n_fields, tpl.edges, lens)
    assert len(steps) == 9
    last = list(tpl.start_token)
    curves = []
    for si, st in enumerate(steps):
        bf = [f for f, _ in st]
        ref, worst, e_plain, e_fmt = _both_oracles_step(pair, plain, bf, [o for _, o in st], [last[f] for f in bf],
                                                        f"cfg1 full depth, pass {si}: fields {bf}", curves)
        assert worst < 1e-3, worst
        assert e_plain < PLAIN_BOUND_CFG1, e_plain
        for i, f in enumerate(bf):
            last[f] = int(ref["tok"][i])
    _curve_file("cfg1_schedule", _curve_lines("workload 1 (24 layers, 0.5B-class widths), whole shortened schedule",
                                              curves))
    pair.close()


def _driver_case(seed, header, D):
    dims = ModelDims(n_layers=2, d_model=128, n_q_heads=4, n_kv_heads=2, head_dim=D, d_mlp=160, vocab=520)
    body = random_dag_template(1200 + seed, n_fields=6, prefix_len=21 + seed, max_slot=7, edge_prob=0.35,
                               vocab=dims.vocab)
    if header:      # field 0 is fixed template text that every other field depends on
        tpl = random_dag_template(1200 + seed, n_fields=6, prefix_len=21 + seed, max_slot=7, edge_prob=0.35,
                                  vocab=dims.vocab)
        tpl.slot_len = [3] + body.slot_len
        tpl.edges = [(0, v + 1) for v in range(6)] + [(u + 1, v + 1) for (u, v) in body.edges]
        tpl.start_token = [0] + body.start_token
        tpl.content_len = [3] + body.content_len
        fixed = {0: [11, 7 + seed, 401]}
    else:
        tpl, fixed = body, None
    return dims, tpl, fixed, draw_weights(40 + seed, dims, random_gains=True, std=0.05)


@pytest.mark.parametrize("seed,B,header,D", [(57, 2, False, 64), (9, 3, True, 128)])
def test_cot_decode_driver_matches_the_oracle_driver(seed, B, header, D):
    """Algorithm 1 end to end on the GPU (free-running, end-of-line tokens, slot
    truncation, scenes with different ready sets, fixed header text filled by
    multi-token passes) against the oracle's driver: same tokens, same lengths,
    same number of passes.  The seeds are ones where every top-2 gap of the oracle
    run is well above the level at which greedy ids must agree."""
    from tests.helpers import GAP_MIN
    dims, tpl, fixed, w = _driver_case(seed, header, D)
    F = tpl.n_fields
    pair = Pair(dims, tpl, w, n_scenes=B, max_branches=F, max_tokens=2)
    for b in range(B):
        pair.prefill_with_oracle(b, draw_prefix_embeddings(40 + seed, tpl.prefix_len, dims.d_model, extra=b))
    eos = list(range(0, dims.vocab, 3))
    ref = O.run_cot_dynamic(pair.dec, tpl.start_token, eos, fixed)
    assert ref["min_gap"] > 2 * GAP_MIN
    got = pair.ctx.cot_decode(tpl.start_token, eos, fixed)
    assert got["passes"] == ref["passes"]
    assert got["fixed_passes"] == (2 if header else 0)          # 3 header tokens, 2 per pass
    for b in range(B):
        for f in range(F):
            n = len(ref["text"][b][f])
            assert got["len"][b, f] == n, (b, f)
            assert list(got["tok"][b, f, :n]) == ref["text"][b][f], (b, f)
            assert (got["tok"][b, f, n:] == -1).all()
    assert np.array_equal(pair.ctx.get_valid_len(), pair.dec.valid_len)
    lens = got["len"]
    assert len({tuple(lens[b]) for b in range(B)}) > 1          # the scenes did diverge
    # a second run starts from empty slots again and repeats itself
    again = pair.ctx.cot_decode(tpl.start_token, eos, fixed)
    assert np.array_equal(again["tok"], got["tok"]) and again["passes"] == got["passes"]
    # without end tokens every generated field runs to its slot length
    full = pair.ctx.cot_decode(tpl.start_token, (), fixed)
    assert np.array_equal(full["len"], np.tile(np.asarray(tpl.slot_len, dtype=np.int32), (B, 1)))
    cp = [0] * F
    for f in range(F):
        cp[f] = (0 if fixed and f in fixed else tpl.slot_len[f]) + \
            max([cp[u] for (u, v) in tpl.edges if v == f], default=0)
    assert full["passes"] == max(cp)
    pair.close()


def test_cot_decode_driver_error_paths():
    import paper_2602_02864_amd.binding as fb
    dims, tpl, fixed, w = _driver_case(9, True, 64)
    F = tpl.n_fields
    pair = Pair(dims, tpl, w, n_scenes=1, max_branches=F, max_tokens=2)
    pair.prefill_with_oracle(0, draw_prefix_embeddings(49, tpl.prefix_len, dims.d_model))

    def code(*a, **k):
        with pytest.raises(fb.FdcError) as e:
            pair.ctx.cot_decode(*a, **k)
        return e.value.code
    assert code(tpl.start_token, (), fixed, max_passes=2) == fb.FDC_ECAP
    bad = list(tpl.start_token)
    bad[2] = dims.vocab
    assert code(bad, (), fixed) == fb.FDC_ERANGE
    assert code(tpl.start_token, (), {0: [1, 2, 3, 4]}) == fb.FDC_ERANGE       # longer than the slot
    assert code(tpl.start_token, (), {0: [1, dims.vocab]}) == fb.FDC_ERANGE
    assert code(tpl.start_token, (), {1: [5]}) == fb.FDC_EINVAL                # depends on the unfixed field 0
    pair.close()
    narrow = Pair(dims, tpl, w, n_scenes=1, max_branches=1, max_tokens=2)      # ready sets larger than R
    with pytest.raises(fb.FdcError) as e:
        narrow.ctx.cot_decode(tpl.start_token, (), fixed)
    assert e.value.code == fb.FDC_ECAP
    narrow.close()


@pytest.mark.parametrize("what,old,new", [
    ("rotary sign", "x1 * c - x2 * s, x2 * c + x1 * s", "x1 * c + x2 * s, x2 * c - x1 * s"),
    ("padding visible", "slot_start[g] + valid_len[g]] = True", "slot_start[g] + 99] = True"),
    ("gate and up swapped", "h = silu(gu[:, :d.d_mlp]) * gu[:, d.d_mlp:]", "h = silu(gu[:, d.d_mlp:]) * gu[:, :d.d_mlp]"),
    ("own token not visible", "vis[slot_start[f]: slot_start[f] + t + 1] = True",
     "vis[slot_start[f]: slot_start[f] + t] = True"),
])
def test_the_parity_comparison_notices_a_wrong_oracle(monkeypatch, what, old, new):
    """The comparison has teeth: against an oracle with one planted mistake (in a
    copy of its source; the library is untouched) the same steps that pass above
    must fail the 2e-3 check."""
    import os
    import types
    import tests.helpers as H
    src = open(os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "oracle", "fdc_oracle.py")).read()
    assert old in src
    mutant = types.ModuleType("fdc_oracle_mutant")
    exec(compile(src.replace(old, new, 1), "fdc_oracle_mutant.py", "exec"), mutant.__dict__)
    dims = ModelDims(n_layers=2, d_model=128, n_q_heads=4, n_kv_heads=2, head_dim=64, d_mlp=160, vocab=520)
    tpl = random_dag_template(931, n_fields=4, prefix_len=21, max_slot=6, edge_prob=0.6, vocab=dims.vocab)
    tpl.slot_len = [max(3, s) for s in tpl.slot_len]
    w = draw_weights(41, dims, random_gains=True, std=0.05)

    def run(oracle_module):
        monkeypatch.setattr(H, "O", oracle_module)
        pair = Pair(dims, tpl, w, n_scenes=1, max_branches=tpl.n_fields)
        pair.prefill_with_oracle(0, draw_prefix_embeddings(41, tpl.prefix_len, dims.d_model))
        try:
            roots = [f for f in range(tpl.n_fields) if not any(v == f for (_, v) in tpl.edges)]
            for off in range(2):                          # two tokens in every root field
                pair.step_both([roots], [[off] * len(roots)], [7 + off] * len(roots), tag=what)
            rest = [f for f in range(tpl.n_fields) if f not in roots]
            if rest:                                      # then the fields that see them
                pair.step_both([rest], [[0] * len(rest)], [11] * len(rest), tag=what)
        finally:
            pair.close(need_sure=False)
    run(O)                                                # the oracle as it is: passes
    with pytest.raises(AssertionError):
        run(mutant)


@pytest.mark.parametrize("seed", [42, 1])
def test_cot_decode_with_a_fast_response_branch_and_a_post_cot_branch(seed):
    """A root branch that depends on nothing decodes alongside the CoT, and a final
    branch that depends on every CoT field starts when all of them have ended and
    sees their non-padding tokens: through fdc_cot_decode, two scenes with
    different lengths, against the oracle's driver."""
    from tests.helpers import GAP_MIN
    dims = ModelDims(n_layers=2, d_model=128, n_q_heads=4, n_kv_heads=2, head_dim=64, d_mlp=160, vocab=520)
    tpl = random_dag_template(1400 + seed, n_fields=4, prefix_len=30 + seed, max_slot=6, edge_prob=0.4,
                              vocab=dims.vocab)
    tpl.slot_len = tpl.slot_len + [5, 4]                     # field 4: fast response, field 5: final branch
    tpl.edges = list(tpl.edges) + [(f, 5) for f in range(4)]
    tpl.start_token = tpl.start_token + [17, 23]
    tpl.content_len = tpl.content_len + [5, 4]
    w = draw_weights(60 + seed, dims, random_gains=True, std=0.05)
    B, F = 2, 6
    pair = Pair(dims, tpl, w, n_scenes=B, max_branches=F)
    for b in range(B):
        pair.prefill_with_oracle(b, draw_prefix_embeddings(60 + seed, tpl.prefix_len, dims.d_model, extra=b))
    eos = list(range(0, dims.vocab, 3))
    ref = O.run_cot_dynamic(pair.dec, tpl.start_token, eos)
    assert ref["min_gap"] > 2 * GAP_MIN
    got = pair.ctx.cot_decode(tpl.start_token, eos)
    assert got["passes"] == ref["passes"]
    for b in range(B):
        for f in range(F):
            n = len(ref["text"][b][f])
            assert got["len"][b, f] == n and list(got["tok"][b, f, :n]) == ref["text"][b][f], (b, f)
        first = ref["trace"][0]["branch_field"][b]
        assert 4 in first and 5 not in first
    pair.close()
