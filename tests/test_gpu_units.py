"""GPU parity of the single kernels through the C ABI: projections, argmax,
KV append + DAG-masked attention (Sec. 3.3), each against the CPU oracle or
the plain definition in fp64."""
import numpy as np
import pytest

import oracle.fdc_oracle as O
from synth_inputs import (ModelDims, bf16_round, draw_normal_bf16, random_dag_template, template)
from tests.helpers import rel_err

pytestmark = pytest.mark.gpu


def _torch():
    import torch
    return torch


@pytest.mark.parametrize("M,N,K", [(1, 16, 32), (3, 48, 64), (8, 4608, 3584), (16, 896, 4864),
                                   (5, 1000, 256), (8, 3584, 18944), (7, 2048, 128), (16, 32000, 896),
                                   # more than 16 rows: the tiled kernel (ragged rows, ragged
                                   # feature tiles, split and unsplit K)
                                   (17, 48, 64), (40, 1000, 256), (129, 1152, 896), (200, 320, 2048),
                                   (256, 3584, 4864), (64, 37888, 512), (1000, 256, 160),
                                   # wide tiles (the eight-wavefront kernel): ragged rows, a feature count
                                   # that ends inside a tile and inside a workgroup, odd and even k tiles
                                   (130, 20008, 288), (300, 33000, 96), (1000, 9000, 160), (513, 40000, 32),
                                   # the 7B-class projections at 256 and 1024 rows: wide tiles with K split
                                   # nine ways (down), two ways over the 320-wide tile (QKV), two ways (O)
                                   (256, 3584, 18944), (1024, 4608, 3584), (1024, 3584, 3584)])
def test_linear_matches_fp64_matmul(M, N, K):
    """y = x W^T with bf16 weights; x is carried as bf16 head + tail, so the
    result must be fp32-accurate, far inside the 2e-3 budget."""
    torch = _torch()
    from paper_2602_02864_amd import fdc_linear, fdc_pack_weight
    rng = np.random.default_rng(M * 1000 + N + K)
    W = draw_normal_bf16(rng, (N, K), 0.02)
    x = rng.standard_normal((M, K)).astype(np.float32)
    wp = fdc_pack_weight(torch.from_numpy(W).cuda().to(torch.bfloat16).contiguous())
    y = fdc_linear(torch.from_numpy(x).cuda(), wp, N)
    torch.cuda.synchronize()
    ref = x.astype(np.float64) @ W.astype(np.float64).T
    assert rel_err(y.cpu().numpy(), ref) < 2e-5


def test_argmax_lowest_index_and_gap():
    torch = _torch()
    from paper_2602_02864_amd import fdc_argmax
    rng = np.random.default_rng(0)
    V = 32000
    lg = rng.standard_normal((9, V)).astype(np.float32)
    lg[0, [5, 777, 31999]] = 9.0            # three-way tie -> lowest index, gap 0
    lg[1, 31999] = 50.0                     # last element
    lg[2, 0] = 50.0
    lg[3] = -3.0                            # all equal
    idx, gap = fdc_argmax(torch.from_numpy(lg).cuda())
    torch.cuda.synchronize()
    idx, gap = idx.cpu().numpy(), gap.cpu().numpy()
    for m in range(9):
        tok, g = O.greedy(lg[m].astype(np.float64))
        assert idx[m] == tok
        assert abs(gap[m] - g) <= 1e-6 * max(1.0, abs(g))
    assert idx[0] == 5 and gap[0] == 0.0 and idx[3] == 0
    # ragged V with a leading dimension
    idx2, _ = fdc_argmax(torch.from_numpy(lg).cuda(), V=1000)
    assert np.array_equal(idx2.cpu().numpy(), np.argmax(lg[:, :1000], axis=1))


def _attention_case(dims, tpl, B, T, seed, active_prob=0.8, valid_mode="random", ramp=0.0):
    """Random K/V/q of bf16 values, random cache state; returns max rel err.
    ramp > 0: keys and queries share a direction along which the keys grow with their
    position, so the scores rise steadily through the cache (by `ramp` in all): the
    running maximum of the softmax keeps moving, far beyond any fixed head-room."""
    torch = _torch()
    from paper_2602_02864_amd import Context
    rng = np.random.default_rng(seed)
    F, P = tpl.n_fields, tpl.prefix_len
    start, N = O.slot_layout(P, tpl.slot_len)
    Hq, Hkv, D = dims.n_q_heads, dims.n_kv_heads, dims.head_dim
    G = Hq // Hkv
    K = draw_normal_bf16(rng, (B, Hkv, N, D))
    V = draw_normal_bf16(rng, (B, Hkv, N, D))
    u = None
    if ramp:
        from synth_inputs import bf16_round
        u = rng.standard_normal(D)
        u /= np.linalg.norm(u)
        K = bf16_round(K + (ramp * np.sqrt(D) * np.arange(N) / N)[None, None, :, None] * u)
    # cache state: how many tokens of each field exist per scene
    valid = np.zeros((B, F), dtype=np.int32)
    bf = np.full((B, F), -1, dtype=np.int32)
    bo = np.zeros((B, F), dtype=np.int32)
    for b in range(B):
        for f in range(F):
            S = tpl.slot_len[f]
            if valid_mode == "full":
                valid[b, f] = S
            else:
                valid[b, f] = int(rng.integers(0, S + 1))
            if S >= T and rng.random() < active_prob:
                off = int(rng.integers(0, S - T + 1))
                bf[b, f], bo[b, f] = f, off
                valid[b, f] = max(valid[b, f], off + T)
    if (bf < 0).all():
        bf[0, 0], bo[0, 0] = 0, 0
        valid[0, 0] = max(valid[0, 0], T)
    ctx = Context(dims, tpl.slot_len, tpl.edges, P, n_scenes=B, max_branches=F, max_tokens=T)
    # install only what is "written": prefix + valid tokens; the rest keeps NaN
    rs, rp = [], []
    for b in range(B):
        for j in range(N):
            rs.append(b)
            rp.append(j)
    Kin = np.ascontiguousarray(np.transpose(K, (0, 2, 1, 3)).reshape(B * N, Hkv, D))
    Vin = np.ascontiguousarray(np.transpose(V, (0, 2, 1, 3)).reshape(B * N, Hkv, D))
    written = np.zeros((B, N), dtype=bool)
    written[:, :P] = True
    for b in range(B):
        for f in range(F):
            written[b, start[f]:start[f] + valid[b, f]] = True
    # unwritten positions (padding, not yet decoded) hold NaN: reading one shows
    Kin[~written.reshape(-1)] = np.nan
    Vin[~written.reshape(-1)] = np.nan
    ctx.kv_append(0, Kin, Vin, np.array(rs, dtype=np.int32), np.array(rp, dtype=np.int32))
    ctx.set_valid_len(valid)
    M = B * F * T
    q = draw_normal_bf16(rng, (M, Hq, D))
    if ramp:
        q = bf16_round(q + u)
    out = ctx.masked_attention(0, q, bf, bo, T=T)
    torch.cuda.synchronize()
    got = out.cpu().numpy().reshape(M, Hq, D)
    worst = 0.0
    for b in range(B):
        rows, rf, ro = [], [], []
        for r in range(F):
            if bf[b, r] < 0:
                assert np.all(got[(b * F + r) * T:(b * F + r + 1) * T] == 0.0)
                continue
            for t in range(T):
                rows.append((b * F + r) * T + t)
                rf.append(int(bf[b, r]))
                ro.append(int(bo[b, r]) + t)
        if not rows:
            continue
        ref = O.attention_only(q[rows], K[b], V[b], P, tpl.slot_len, tpl.edges, valid[b], rf, ro, G)
        assert np.isfinite(got[rows]).all()
        worst = max(worst, rel_err(got[rows], ref))
    ctx.close()
    return worst


ATT_DIMS = {
    "g1d64": ModelDims(1, 256, 4, 4, 64, 512, 1000),
    "g7d64": ModelDims(1, 896, 14, 2, 64, 512, 1000),
    "g7d128": ModelDims(1, 3584, 28, 4, 128, 512, 1000),
    "g4d128": ModelDims(1, 4096, 32, 8, 128, 512, 1000),
}


@pytest.mark.parametrize("name,seed,F,P,max_slot,p,B,T", [
    ("g1d64", 0, 4, 128, 8, 0.5, 1, 1),
    ("g1d64", 1, 7, 37, 9, 0.3, 2, 1),       # ragged prefix / slots: tiles straddle fields
    ("g7d64", 2, 8, 200, 48, 0.4, 1, 1),
    ("g7d64", 3, 5, 0, 20, 0.6, 2, 2),       # no prefix at all, multi-token
    ("g7d128", 4, 12, 300, 64, 0.3, 1, 1),
    ("g4d128", 5, 16, 260, 33, 0.2, 3, 1),
    ("g4d128", 6, 6, 100, 16, 1.0, 2, 4),    # chain closure, T = 4
    ("g7d128", 7, 3, 31, 5, 0.0, 1, 3),      # edgeless
    ("g4d128", 8, 40, 64, 6, 0.1, 1, 1),     # many fields
])
def test_masked_attention_matches_oracle(name, seed, F, P, max_slot, p, B, T):
    dims = ATT_DIMS[name]
    tpl = random_dag_template(500 + seed, F, P, max_slot, p, dims.vocab)
    err = _attention_case(dims, tpl, B, T, seed)
    assert err < 2e-3, err


@pytest.mark.parametrize("name,seed,F,P,max_slot,p,B,T", [
    ("g1d64", 1, 7, 37, 9, 0.3, 2, 1),
    ("g7d64", 3, 5, 0, 20, 0.6, 2, 2),
    ("g7d128", 4, 12, 300, 64, 0.3, 1, 1),
    ("g4d128", 6, 6, 100, 16, 1.0, 2, 4),
    ("g7d128", 7, 3, 31, 5, 0.0, 1, 3),
    ("g4d128", 8, 40, 64, 6, 0.1, 1, 1),
])
def test_masked_attention_register_variant_on_small_ragged_shapes(monkeypatch, name, seed, F, P, max_slot, p, B, T):
    """The library picks the kernel that keeps K/V tiles in registers only for
    large caches (workloads 3 and 4); here it is forced onto the small ragged
    cases (the context reads FDC_ATTN_VARIANT when it is created), so that both
    kernels see ragged prefixes, inactive rows, T > 1 and unwritten positions."""
    monkeypatch.setenv("FDC_ATTN_VARIANT", "1")
    dims = ATT_DIMS[name]
    tpl = random_dag_template(500 + seed, F, P, max_slot, p, dims.vocab)
    err = _attention_case(dims, tpl, B, T, seed)
    assert err < 2e-3, err


@pytest.mark.parametrize("name,seed,F,P,max_slot,p,B,T,ramp", [
    ("g7d128", 21, 12, 300, 64, 0.3, 2, 4, 0.0),     # 12 x 4 x 7 = 336 rows per KV head: two row groups of eight tiles
    ("g4d128", 22, 16, 2100, 33, 0.2, 3, 2, 0.0),    # 128 rows: four-wavefront workgroups, long ragged prefix
    ("g7d64", 23, 10, 515, 20, 0.6, 2, 2, 0.0),      # head size 64
    ("g7d128", 24, 9, 4000, 40, 0.4, 1, 4, 60.0),    # scores rise by 60 along the cache
    ("g4d128", 25, 6, 1500, 64, 1.0, 2, 8, 25.0),
])
def test_masked_attention_many_rows_kernel_on_ragged_shapes(monkeypatch, name, seed, F, P, max_slot, p, B, T, ramp):
    """The kernel for many rows per KV head (one workgroup shares each K/V tile among
    up to eight row tiles), forced onto ragged cases: inactive rows, unwritten
    positions, T > 1, chunks cut per step; and with scores that keep rising along the
    cache, so that the reference point of its exponentials (moved only when a score
    exceeds it by 2^8) moves many times in every chunk and the weights in between
    are far above 1."""
    monkeypatch.setenv("FDC_ATTN_VARIANT", "2")
    dims = ATT_DIMS[name]
    tpl = random_dag_template(500 + seed, F, P, max_slot, p, dims.vocab)
    err = _attention_case(dims, tpl, B, T, seed, active_prob=0.9, ramp=ramp)
    assert err < 2e-3, err


def _wide_slots_template(n_fields=24, slot=64, prefix_len=100, p=0.2, seed=3):
    """More than 32 tiles past the prefix (24 x 64 = 48 tiles), ragged prefix."""
    from synth_inputs import Template
    rng = np.random.default_rng(seed)
    edges = [(i, j) for j in range(n_fields) for i in range(j) if rng.random() < p]
    return Template(prefix_len, [slot] * n_fields, edges, [slot] * n_fields, [1] * n_fields, name="wide")


@pytest.mark.parametrize("variant", ["0", "1", "2"])
@pytest.mark.parametrize("B,T", [(1, 1), (2, 2)])
def test_masked_attention_with_more_than_32_slot_tiles(monkeypatch, variant, B, T):
    """48 tiles reach past the prefix: more than one workgroup's mask tables hold
    (32), so the chunks are cut shorter; under all three attention kernels (the
    many-row kernel then keeps the context's cut instead of the step's own)."""
    from paper_2602_02864_amd import fdc_attention_plan
    monkeypatch.setenv("FDC_ATTN_VARIANT", variant)
    dims = ATT_DIMS["g4d128"]
    tpl = _wide_slots_template()
    plan = fdc_attention_plan(dims, tpl.slot_len, tpl.edges, tpl.prefix_len, B, tpl.n_fields, T)
    assert plan["tiles"] - plan["prefix_tiles"] > plan["max_masked_tiles"] and plan["variant"] == int(variant)
    err = _attention_case(dims, tpl, B, T, seed=11 + B, active_prob=0.9)
    assert err < 2e-3, err


def _tables_case(tpl, B, T, seed, active_prob):
    """The device's mask words and position table, expanded, against the oracle's
    dense mask: random cache states, random active subsets and offsets."""
    from paper_2602_02864_amd import Context
    dims = ModelDims(1, 64, 1, 1, 64, 32, 8)             # the tables do not depend on the model
    rng = np.random.default_rng(seed)
    F, P = tpl.n_fields, tpl.prefix_len
    ctx = Context(dims, tpl.slot_len, tpl.edges, P, n_scenes=B, max_branches=F, max_tokens=T)
    n_rows = 0
    for rep in range(3):
        valid = np.zeros((B, F), dtype=np.int32)
        bf = np.full((B, F), -1, dtype=np.int32)
        bo = np.zeros((B, F), dtype=np.int32)
        for b in range(B):
            order = rng.permutation(F)                   # branch entries in any order
            for i, f in enumerate(order):
                S = tpl.slot_len[f]
                valid[b, f] = int(rng.integers(0, S + 1))
                if S >= T and rng.random() < active_prob:
                    off = int(rng.integers(0, S - T + 1))
                    bf[b, i], bo[b, i] = f, off
                    valid[b, f] = max(valid[b, f], off + T)
        ctx.set_valid_len(valid)
        mask, pos = ctx.step_tables_dense(F, T, bf, bo)
        assert mask.shape == (B * F * T, P + sum(tpl.slot_len))
        for b in range(B):
            for r in range(F):
                m0 = (b * F + r) * T
                if bf[b, r] < 0:
                    assert not mask[m0:m0 + T].any() and (pos[m0:m0 + T] == -1).all()
                    continue
                want, wpos = O.dense_mask(P, tpl.slot_len, tpl.edges, valid[b], [int(bf[b, r])] * T,
                                          [int(bo[b, r]) + t for t in range(T)])
                assert np.array_equal(mask[m0:m0 + T].astype(bool), want), (rep, b, r)
                assert np.array_equal(pos[m0:m0 + T], wpos), (rep, b, r)
                n_rows += T
    ctx.close()
    return n_rows


@pytest.mark.parametrize("T", [1, 4])
@pytest.mark.parametrize("cfg_id,B,kw", [(0, 1, {}), (1, 2, {}), (2, 1, {}), (3, 3, {"rho": 0.3}), (3, 2, {"rho": 1.0}),
                                         (4, 8, {})])
def test_device_mask_and_positions_are_bit_exact_on_the_workload_templates(cfg_id, B, kw, T):
    """Eq. 1 / Sec. 3.3 on the device: what the kernels consume (one visibility word
    per row and 32-key tile past the prefix, one position id per row) expanded to
    a dense mask equals the oracle's, for the five workload templates, one and
    four tokens per branch, inactive entries included."""
    assert _tables_case(template(cfg_id, **kw), B, T, 100 * cfg_id + T, 0.7) > 0


@pytest.mark.parametrize("seed,F,P,max_slot,p,B,T", [(1, 7, 37, 9, 0.3, 2, 1), (3, 5, 0, 20, 0.6, 2, 4),
                                                     (8, 40, 64, 6, 0.1, 1, 1), (12, 64, 1, 5, 0.05, 3, 2),
                                                     (13, 9, 95, 70, 0.5, 2, 4)])
def test_device_mask_and_positions_are_bit_exact_on_ragged_templates(seed, F, P, max_slot, p, B, T):
    tpl = random_dag_template(500 + seed, F, P, max_slot, p, 100)
    tpl.slot_len = [max(s, T) for s in tpl.slot_len]
    assert _tables_case(tpl, B, T, seed, 0.6) > 0
    assert _tables_case(_wide_slots_template(), 2, T, seed, 0.8) > 0


def test_masked_attention_microbenchmark_shape_sampled():
    """Workload 3 geometry (16 fields x 64 slots, prefix 4096, 32/8 heads, D 128)
    at 2 scenes: every branch active at offset 32, all other slots full."""
    torch = _torch()
    dims = ATT_DIMS["g4d128"]
    for rho in (0.0, 0.3, 1.0):
        tpl = template(3, rho=rho)
        err = _attention_case(dims, tpl, B=2, T=1, seed=int(rho * 10), active_prob=1.1, valid_mode="full")
        assert err < 2e-3, (rho, err)


def test_masked_out_kv_is_never_read_and_visible_kv_is():
    """Perturbing masked-out K/V (other branches, padding) leaves the output
    bit-identical; perturbing a visible key changes it."""
    torch = _torch()
    from paper_2602_02864_amd import Context
    dims = ATT_DIMS["g4d128"]
    tpl = random_dag_template(77, 6, 70, 12, 0.4, dims.vocab)
    F, P = tpl.n_fields, tpl.prefix_len
    start, N = O.slot_layout(P, tpl.slot_len)
    rng = np.random.default_rng(5)
    Hkv, D, Hq = dims.n_kv_heads, dims.head_dim, dims.n_q_heads
    valid = np.array([[max(1, s // 2) for s in tpl.slot_len]], dtype=np.int32)
    bf = np.array([[2, 5]], dtype=np.int32)
    bo = np.array([[valid[0, 2] - 1, valid[0, 5] - 1]], dtype=np.int32)
    K = draw_normal_bf16(rng, (N, Hkv, D))
    V = draw_normal_bf16(rng, (N, Hkv, D))
    q = draw_normal_bf16(rng, (2, Hq, D))
    mask, _ = O.dense_mask(P, tpl.slot_len, tpl.edges, valid[0], [2, 5], list(bo[0]))
    unseen = np.nonzero(~mask.any(axis=0))[0]
    seen = np.nonzero(mask.all(axis=0))[0]
    assert unseen.size > 0 and seen.size > 0

    def run(Kx, Vx):
        ctx = Context(dims, tpl.slot_len, tpl.edges, P, 1, 2, 1)
        ctx.kv_append(0, Kx, Vx, np.zeros(N, dtype=np.int32), np.arange(N, dtype=np.int32))
        ctx.set_valid_len(valid)
        o = ctx.masked_attention(0, q, bf, bo)
        torch.cuda.synchronize()
        o = o.cpu().numpy()
        ctx.close()
        return o
    base = run(K, V)
    K2, V2 = K.copy(), V.copy()
    K2[unseen] = 1.0e30
    V2[unseen] = -1.0e30
    assert np.array_equal(run(K2, V2), base)
    V3 = V.copy()
    V3[seen[-1]] += 1.0
    assert not np.array_equal(run(K, V3), base)


def test_kv_append_skips_bad_rows_and_error_paths():
    torch = _torch()
    from paper_2602_02864_amd import Context, FdcError, binding as fb
    dims = ATT_DIMS["g1d64"]
    ctx = Context(dims, [4, 4], [(0, 1)], 8, 1, 2, 1)
    k = np.ones((3, 4, 64), dtype=np.float32)
    ctx.kv_append(0, k, k, [0, -1, 5], [0, 1, 2])            # rows 1, 2 skipped, no fault
    with pytest.raises(FdcError) as e:
        ctx.kv_append(3, k, k, [0, 0, 0], [0, 1, 2])
    assert e.value.code == fb.FDC_ERANGE
    with pytest.raises(FdcError) as e:
        ctx.masked_attention(0, np.zeros((2, 4, 64), np.float32), [0, 1], [0, 0])
    assert e.value.code == fb.FDC_ERANGE                         # valid_len does not cover the rows
    with pytest.raises(FdcError) as e:
        ctx.parallel_decode_step([0, 1], [0, 0], tok_in=[1, 2])
    assert e.value.code == fb.FDC_ESTATE                         # no weights yet
    with pytest.raises(FdcError) as e:
        ctx.set_valid_len([5, 0])
    assert e.value.code == fb.FDC_ERANGE
    ctx.close()


@pytest.mark.parametrize("rho,dag_seed", [(0.0, 0), (0.3, 0), (0.5, 2), (1.0, 0)])
def test_masked_attention_full_size_benchmark_configuration_sampled(rho, dag_seed):
    """Workload 3 exactly as bench.py times it (16 scenes, 32/8 heads x 128,
    prefix 4096, 16 branches x 64-token slots, every branch active at offset 32,
    all other slots full) at the densities of its sweep - no edges, 0.3, a random
    graph of density 0.5, the full chain closure; the oracle on every row of three
    of the scenes."""
    torch = _torch()
    from paper_2602_02864_amd import Context
    from synth_inputs import model_dims, workload_seed
    dims = model_dims(3)
    tpl = template(3, rho=rho, dag_seed=dag_seed)
    B, F, S, P = 16, tpl.n_fields, tpl.slot_len[0], tpl.prefix_len
    N = P + F * S
    Hq, Hkv, D = dims.n_q_heads, dims.n_kv_heads, dims.head_dim
    rng = workload_seed(3, "prefix", 11)
    ctx = Context(dims, tpl.slot_len, tpl.edges, P, B, F, 1)
    keep = {}
    for b in range(B):                                    # one scene at a time: bounded host memory
        Kb = draw_normal_bf16(rng, (N, Hkv, D))
        Vb = draw_normal_bf16(rng, (N, Hkv, D))
        ctx.kv_append(0, Kb, Vb, np.full(N, b, dtype=np.int32), np.arange(N, dtype=np.int32))
        if b in (0, 7, 15):
            keep[b] = (np.ascontiguousarray(Kb.transpose(1, 0, 2)), np.ascontiguousarray(Vb.transpose(1, 0, 2)))
    ctx.set_valid_len(np.full((B, F), S, dtype=np.int32))
    bf = np.tile(np.arange(F, dtype=np.int32), B)
    bo = np.full(B * F, 32, dtype=np.int32)
    q = draw_normal_bf16(rng, (B * F, Hq, D))
    out = ctx.masked_attention(0, q, bf, bo)
    torch.cuda.synchronize()
    got = out.cpu().numpy().reshape(B * F, Hq, D)
    assert np.isfinite(got).all()
    for b, (Kb, Vb) in keep.items():
        rows = [b * F + f for f in range(F)]
        ref = O.attention_only(q[rows], Kb, Vb, P, tpl.slot_len, tpl.edges, [S] * F, list(range(F)), [32] * F,
                               Hq // Hkv)
        assert rel_err(got[rows], ref) < 2e-3, (rho, b, rel_err(got[rows], ref))
    ctx.close()


def test_stream_copy_and_event_calibration():
    """Measurement helpers: the copy is exact (ragged size), misuse is refused, and
    the event-pair overhead is a small non-negative number of microseconds."""
    import torch
    from paper_2602_02864_amd import FdcError, fdc_profile_calibrate, fdc_stream_copy
    n = (1 << 22) + 16 * 37
    src = torch.randint(0, 255, (n,), dtype=torch.uint8, device="cuda")
    dst = torch.zeros_like(src)
    fdc_stream_copy(dst, src)
    torch.cuda.synchronize()
    assert torch.equal(dst, src)
    with pytest.raises(FdcError):
        fdc_stream_copy(dst[:24], src[:24])          # not a multiple of 16 bytes
    ov, nul = fdc_profile_calibrate(50)
    assert 0.0 <= ov < 100.0 and 0.0 <= nul < 100.0
