"""CPU tests of the C ABI: the library loads without a GPU, exports every symbol
the header declares, and its host-only entry points (mask metadata, Sec. 3.3 /
Eq. 1) agree bit-exactly with the oracle and report errors as documented."""
import itertools
import os
import re

import numpy as np
import pytest

import oracle.fdc_oracle as O
from paper_2602_02864_amd import binding as fb
from paper_2602_02864_amd import fdc_build_mask, fdc_dense_mask, FdcError
from synth_inputs import random_dag_template, template

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "fdc.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = sorted(set(re.findall(r"\b(fdc_[a-z0-9_]+)\s*\(", hdr)))
    assert "fdc_build_mask" in declared and "fdc_kv_append" in declared
    assert "fdc_parallel_decode_step" in declared and "fdc_argmax" in declared
    L = fb.lib()
    for name in declared:
        assert hasattr(L, name), f"{name} declared in fdc.h but not exported"
    assert sorted(fb.EXPORTS) == declared
    assert L.fdc_version() >= 100
    assert L.fdc_strerror(fb.FDC_ECYCLE).decode() != L.fdc_strerror(fb.FDC_EORDER).decode()


def test_header_is_plain_c_and_a_c_program_links_against_the_library(tmp_path):
    """The boundary is a C ABI: the header compiles as strict C99, and a C program
    that knows nothing but the header builds, loads the library and gets the
    ancestor words of a three-field chain from it."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no C compiler")
    src = tmp_path / "use_fdc.c"
    src.write_text(r"""
#include <stdio.h>
#include "fdc.h"
int main(void) {
    int32_t slot[3] = {2, 3, 4}, es[2] = {0, 1}, ed[2] = {1, 2}, start[3], level[3], total = 0;
    uint64_t anc[3];
    int32_t rc = fdc_build_mask(3, slot, 2, es, ed, 5, anc, start, level, &total);
    if (rc != FDC_OK) { printf("error %s\n", fdc_last_error()); return 1; }
    printf("%llu %llu %llu %d %d %d %d\n", (unsigned long long)anc[0], (unsigned long long)anc[1],
           (unsigned long long)anc[2], start[0], start[1], start[2], total);
    return fdc_version() >= 100 ? 0 : 2;
}
""")
    inc = os.path.join(ROOT, "include")
    subprocess.run([gcc, "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-fsyntax-only", "-I", inc, str(src)],
                   check=True)
    exe = tmp_path / "use_fdc"
    libdir = os.path.dirname(fb.LIB_PATH)
    subprocess.run([gcc, "-std=c99", "-I", inc, str(src), "-o", str(exe), "-L", libdir, "-lfdc",
                    "-Wl,-rpath," + libdir], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()
    assert out == ["0", "1", "3", "5", "7", "10", "14"]        # anc: {}, {0}, {0, 1}; starts; N


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2 and "ONE GPU" in r.stderr and r.stdout == ""


@pytest.mark.parametrize("F", [1, 2, 3, 4, 5])
def test_build_mask_matches_oracle_on_all_small_dags(F):
    pairs = [(i, j) for j in range(F) for i in range(j)]
    rng = np.random.default_rng(F)
    for bits in range(1 << len(pairs)):
        edges = [p for k, p in enumerate(pairs) if bits >> k & 1]
        slot = [int(x) for x in rng.integers(1, 6, size=F)]
        P = int(rng.integers(0, 5))
        r = fdc_build_mask(slot, edges, P)
        assert np.array_equal(r["anc_words"], O.ancestor_words(F, edges))
        start, N = O.slot_layout(P, slot)
        assert list(r["slot_start"]) == start and r["total_len"] == N
        assert list(r["level"]) == O.levels(F, edges)


@pytest.mark.parametrize("seed,F,p", [(0, 33, 0.1), (1, 64, 0.05), (2, 64, 0.5), (3, 65, 0.1),
                                      (4, 130, 0.03)])
def test_build_mask_matches_oracle_on_random_dags_incl_multiword(seed, F, p):
    rng = np.random.default_rng(seed)
    edges = [(i, j) for j in range(F) for i in range(j) if rng.random() < p]
    rng.shuffle(edges)                       # edge order must not matter
    edges += edges[:3]                       # nor duplicates
    slot = [int(x) for x in rng.integers(1, 70, size=F)]
    r = fdc_build_mask(slot, edges, 100)
    assert r["anc_words"].shape == (F, (F + 63) // 64)
    assert np.array_equal(r["anc_words"], O.ancestor_words(F, edges))
    assert list(r["level"]) == O.levels(F, edges)


@pytest.mark.parametrize("seed", range(8))
def test_dense_mask_and_positions_match_oracle(seed):
    tpl = random_dag_template(300 + seed, n_fields=3 + 2 * seed, prefix_len=seed, max_slot=7,
                              edge_prob=0.35, vocab=10)
    rng = np.random.default_rng(seed)
    F = tpl.n_fields
    valid = [int(rng.integers(0, s + 1)) for s in tpl.slot_len]
    rf = [int(x) for x in rng.integers(0, F, size=9)]
    ro = [int(rng.integers(0, tpl.slot_len[f])) for f in rf]
    r = fdc_build_mask(tpl.slot_len, tpl.edges, tpl.prefix_len)
    mask, pos = fdc_dense_mask(tpl.slot_len, r["slot_start"], r["anc_words"], tpl.prefix_len, valid, rf, ro)
    want_mask, want_pos = O.dense_mask(tpl.prefix_len, tpl.slot_len, tpl.edges, valid, rf, ro)
    assert np.array_equal(mask.astype(bool), want_mask)
    assert np.array_equal(pos, want_pos)


def test_workload_templates_masks_match_oracle():
    for cfg, kw in [(0, {}), (1, {}), (2, {}), (3, {"rho": 0.3}), (3, {"rho": 1.0}), (4, {})]:
        tpl = template(cfg, **kw)
        F = tpl.n_fields
        r = fdc_build_mask(tpl.slot_len, tpl.edges, tpl.prefix_len)
        assert np.array_equal(r["anc_words"], O.ancestor_words(F, tpl.edges))
        rf = list(range(F))
        ro = [c - 1 for c in tpl.content_len]
        mask, pos = fdc_dense_mask(tpl.slot_len, r["slot_start"], r["anc_words"], tpl.prefix_len,
                                   tpl.content_len, rf, ro)
        want_mask, want_pos = O.dense_mask(tpl.prefix_len, tpl.slot_len, tpl.edges, tpl.content_len, rf, ro)
        assert np.array_equal(mask.astype(bool), want_mask) and np.array_equal(pos, want_pos)


@pytest.mark.parametrize("seed", range(10))
def test_scheduler_matches_oracle_algorithm1(seed):
    """Same passes, same (field, offset) sets as the oracle's Algorithm 1, and
    as many passes as the critical path is long (Sec. 3.2)."""
    from paper_2602_02864_amd import fdc_schedule
    tpl = random_dag_template(700 + seed, n_fields=2 + 2 * seed, prefix_len=0, max_slot=7,
                              edge_prob=0.3, vocab=10)
    F = tpl.n_fields
    want = O.schedule(F, tpl.edges, tpl.content_len)
    got = fdc_schedule(F, tpl.edges + tpl.edges[:2], tpl.content_len)
    assert len(got) == len(want)
    for (bf, bo), st in zip(got, want):
        n = len(st)
        assert [(int(f), int(o)) for f, o in zip(bf[:n], bo[:n])] == st
        assert (bf[n:] == -1).all()
    cp = [0] * F
    for f in range(F):
        cp[f] = tpl.content_len[f] + max([cp[u] for (u, v) in tpl.edges if v == f], default=0)
    assert len(got) == max(cp)
    with pytest.raises(FdcError) as e:
        fdc_schedule(3, [], [1, 1, 1], max_branches=2)
    assert e.value.code == fb.FDC_ECAP
    with pytest.raises(FdcError) as e:
        fdc_schedule(2, [(0, 1), (1, 0)], [1, 1])
    assert e.value.code == fb.FDC_ECYCLE


@pytest.mark.parametrize("seed", range(8))
def test_dynamic_scheduler_follows_algorithm1_under_random_finishing(seed):
    """peek / advance with finishing decided by the caller: the ready sets are
    those of Algorithm 1 written out with in-degree counters and a set, for any
    sequence of finishing decisions; pre-filled fields release their successors."""
    from paper_2602_02864_amd import Scheduler
    rng = np.random.default_rng(900 + seed)
    tpl = random_dag_template(800 + seed, n_fields=3 + 2 * seed, prefix_len=0, max_slot=7,
                              edge_prob=0.3, vocab=10)
    F = tpl.n_fields
    preds = [set(u for (u, v) in tpl.edges if v == f) for f in range(F)]
    fixed = {}
    if seed % 2:                        # roots as fixed text
        fixed = {f: int(rng.integers(1, 5)) for f in range(F) if not preds[f] and rng.random() < 0.6}
    s = Scheduler(F, tpl.edges)
    for f in sorted(fixed):
        s.complete(f, fixed[f])
    d = [len(preds[f] - set(fixed)) for f in range(F)]
    S = {f for f in range(F) if d[f] == 0 and f not in fixed}
    done = [0] * F
    passes = tokens = 0
    while True:
        bf, bo = s.peek()
        assert list(bf) == sorted(S) and list(bo) == [done[f] for f in sorted(S)]
        if not S:
            break
        fin = [int(rng.random() < 0.4) for _ in bf]
        s.advance(fin)
        passes += 1
        tokens += len(bf)
        for f, fl in zip(sorted(S), fin):
            done[f] += 1
            if fl:
                S.discard(f)
                for u in range(F):
                    if f in preds[u]:
                        d[u] -= 1
                        if d[u] == 0:
                            S.add(u)
    assert s.stats() == {"passes": passes, "tokens": tokens, "unfinished": 0}
    with pytest.raises(FdcError) as e:
        s.advance([1])                                   # nothing is ready any more
    assert e.value.code == fb.FDC_EINVAL
    s.close()
    s = Scheduler(3, [(0, 1), (1, 2)])
    with pytest.raises(FdcError) as e:
        s.complete(1, 2)                                 # its prerequisite is not complete
    assert e.value.code == fb.FDC_EINVAL
    with pytest.raises(FdcError) as e:
        s.complete(3, 1)
    assert e.value.code == fb.FDC_ERANGE
    bf, _ = s.peek()
    with pytest.raises(FdcError) as e:
        s.advance([0, 0])                                # one field is ready, two flags
    assert e.value.code == fb.FDC_EINVAL
    with pytest.raises(FdcError) as e:
        fb._check(fb.lib().fdc_sched_next(s._h, 3, fb._p(np.zeros(3, np.int32)), fb._p(np.zeros(3, np.int32)),
                                          fb._p(np.zeros(1, np.int32))))
    assert e.value.code == fb.FDC_EINVAL                 # created without content lengths
    s.close()


def test_build_mask_error_codes():
    def code(*a):
        with pytest.raises(FdcError) as e:
            fdc_build_mask(*a)
        return e.value.code
    assert code([1, 1, 1], [(0, 1), (1, 2), (2, 0)], 0) == fb.FDC_ECYCLE
    assert code([1, 1], [(0, 0)], 0) == fb.FDC_ECYCLE
    assert code([1, 1, 1], [(2, 1)], 0) == fb.FDC_EORDER
    assert code([1, 1, 1], [(0, 3)], 0) == fb.FDC_ERANGE
    assert code([1, 1, 1], [(-1, 2)], 0) == fb.FDC_ERANGE
    assert code([1, 0, 1], [], 0) == fb.FDC_EINVAL
    assert code([1, 1], [], -1) == fb.FDC_EINVAL
    assert code([], [], 0) == fb.FDC_EINVAL
    assert "cycle" in fb.lib().fdc_last_error().decode() or True
    # the oracle rejects the same templates
    for edges in ([(0, 1), (1, 2), (2, 0)], [(2, 1)], [(0, 3)]):
        with pytest.raises(ValueError):
            O.check_template(3, edges)


def test_dense_mask_error_codes():
    r = fdc_build_mask([2, 2], [(0, 1)], 1)
    def code(valid, rf, ro):
        with pytest.raises(FdcError) as e:
            fdc_dense_mask([2, 2], r["slot_start"], r["anc_words"], 1, valid, rf, ro)
        return e.value.code
    assert code([3, 0], [0], [0]) == fb.FDC_ERANGE
    assert code([1, 1], [2], [0]) == fb.FDC_ERANGE
    assert code([1, 1], [1], [2]) == fb.FDC_ERANGE


def test_null_pointers_are_rejected_not_dereferenced():
    L = fb.lib()
    assert L.fdc_build_mask(2, None, 0, None, None, 0, None, None, None, None) == fb.FDC_EINVAL
    assert L.fdc_create(None, 1, None, 0, None, None, 0, 1, 1, 1, None) == fb.FDC_EINVAL
    assert L.fdc_argmax(None, 1, 1, 1, None, None, None) == fb.FDC_EINVAL
    assert L.fdc_kv_append(None, 0, None, None, None, None, 0, None) == fb.FDC_EINVAL
    assert L.fdc_parallel_decode_step(None, 1, 1, None, None, None, None, None, None, None, None, None) == fb.FDC_EINVAL
    assert L.fdc_cot_decode(None, None, None, None, None, 0, 0, None, None, None, None) == fb.FDC_EINVAL
    assert L.fdc_sched_peek(None, 1, None, None, None) == fb.FDC_EINVAL
    assert L.fdc_sched_advance(None, 0, None) == fb.FDC_EINVAL
    assert L.fdc_packed_weight_bytes(16, 32) == 1024 and L.fdc_packed_weight_bytes(1000, 32) == 1008 * 64


def _check_plan(dims, tpl, B, R, T, tag):
    """What the attention kernels assume of a context's launch plan: the chunks
    tile the key range, none exceeds the kernel's tile list, none has more tiles
    past the prefix than the mask tables hold, and a chunk's real tiles never
    outnumber its weighted size (the register kernel lists `cb` candidates)."""
    from paper_2602_02864_amd import fdc_attention_plan
    p = fdc_attention_plan(dims, tpl.slot_len, tpl.edges, tpl.prefix_len, B, R, T)
    first = p["chunk_first_tile"]
    N = tpl.prefix_len + sum(tpl.slot_len)
    assert p["tiles"] == (N + 31) // 32 and p["prefix_tiles"] == tpl.prefix_len // 32, tag
    assert len(first) == p["chunks"] + 1 and first[0] == 0 and first[-1] == p["tiles"], (tag, p)
    assert p["wq"] >= 16 and p["nrt"] in (1, 2, 4, 8) and p["rg_max"] >= 1, (tag, p)
    rows = R * T * (dims.n_q_heads // dims.n_kv_heads)
    assert p["rg_max"] * p["nrt"] * 32 >= rows, (tag, p)
    for c in range(p["chunks"]):
        n = first[c + 1] - first[c]
        assert 0 <= n <= p["max_chunk_tiles"] and n <= p["cb"], (tag, c, p)
        masked = max(0, first[c + 1] - max(first[c], p["prefix_tiles"]))
        assert masked <= p["max_masked_tiles"], (tag, c, p)
        if p["variant"] == 0:
            assert (n + 1) // 2 <= 64, (tag, c, p)        # one tile per lane and stream
    return p


def test_attention_plan_bounds_over_the_admissible_shapes(monkeypatch):
    """plan_attention at the corners: few and many fields, short and long slots,
    no prefix and a long one, one scene and many, the row limit, both kernels."""
    from synth_inputs import ModelDims, Template
    seen = set()
    shapes = []
    for F, S in [(1, 1), (1, 2048), (3, 5), (12, 64), (16, 64), (24, 64), (32, 32), (64, 1), (64, 31), (64, 96),
                 (40, 200), (64, 512)]:
        for P in (0, 1, 31, 32, 100, 3072, 8192, 70000):
            shapes.append((F, S, P))
    for variant in (None, "0", "1", "2"):
        if variant is None:
            monkeypatch.delenv("FDC_ATTN_VARIANT", raising=False)
        else:
            monkeypatch.setenv("FDC_ATTN_VARIANT", variant)
        for (F, S, P) in shapes:
            tpl = Template(P, [S] * F, [(i, i + 1) for i in range(F - 1)], [S] * F, [0] * F)
            for Hq, Hkv, D in [(4, 4, 64), (14, 2, 64), (28, 4, 128), (32, 8, 128)]:
                dims = ModelDims(1, 256, Hq, Hkv, D, 512, 1000)
                for B, R, T in [(1, 1, 1), (1, F, 1), (16, min(F, 16), 1), (8, min(F, 32), 4), (1, 1, min(S, 1024)),
                                (2, min(F, 8), min(S, 64))]:
                    if B * R * T > 1024 or T > S:
                        continue
                    p = _check_plan(dims, tpl, B, R, T, (variant, F, S, P, Hq, Hkv, D, B, R, T))
                    seen.add((p["variant"], p["chunks"] > 1, p["tiles"] - p["prefix_tiles"] > p["max_masked_tiles"]))
    assert len(seen) >= 8          # all three kernels, one and several chunks, few and many slot tiles
    # the five workloads as benchmarked
    from synth_inputs import model_dims
    for cfg, B, R, T in [(0, 1, 3, 1), (1, 1, 6, 1), (2, 1, 8, 1), (3, 16, 16, 1), (4, 8, 8, 4), (4, 8, 32, 4)]:
        t = template(cfg)
        _check_plan(model_dims(cfg), t, B, R, T, f"cfg{cfg}")


def test_attention_plan_of_a_step_balances_the_chunks_and_keeps_the_bounds():
    """With many rows per KV head the key chunks are cut per step.  Workload 4, every
    level of the template and several slot offsets: the cut covers all tiles, keeps
    the kernel's limits, has no more chunks than the context's plan, and the chunk
    that holds the slots has about as many VISIBLE tiles (plus its table set-up) as
    the others - with the context's fixed cut it had as few as a quarter."""
    from paper_2602_02864_amd import fdc_attention_plan
    from synth_inputs import model_dims
    dims, tpl = model_dims(4), template(4)
    F, S, B, T = tpl.n_fields, tpl.slot_len[0], 8, 4
    anc = [set() for _ in range(F)]
    for s, d in tpl.edges:
        anc[d].add(s)
    for _ in range(F):
        for f in range(F):
            for g in list(anc[f]):
                anc[f] |= anc[g]
    for R, levels in [(8, range(F // 8)), (F, [None])]:
        base = fdc_attention_plan(dims, tpl.slot_len, tpl.edges, tpl.prefix_len, B, R, T)
        for lv in levels:
            for off in (0, 12, 28):
                fields = list(range(F)) if lv is None else list(range(8 * lv, 8 * lv + 8))
                vl = np.zeros((B, F), dtype=np.int32)
                if lv is not None:
                    vl[:, :8 * lv] = S
                vl[:, fields] = off + T
                bf = np.tile(np.array(fields, dtype=np.int32), B)
                bo = np.full(bf.size, off, dtype=np.int32)
                p = fdc_attention_plan(dims, tpl.slot_len, tpl.edges, tpl.prefix_len, B, R, T, step=(vl, bf, bo, T))
                first, t0 = p["chunk_first_tile"], p["prefix_tiles"]
                assert p["chunks"] <= base["chunks"] and first[0] == 0 and first[-1] == p["tiles"], (lv, off, p)
                seen = set()
                for f in fields:
                    for g in anc[f] | {f}:
                        n = off + T if g == f else int(vl[0, g])
                        if n > 0:
                            p0 = tpl.prefix_len + sum(tpl.slot_len[:g])
                            seen |= set(range(p0 // 32, (p0 + n - 1) // 32 + 1))
                cost = []
                for c in range(p["chunks"]):
                    n = first[c + 1] - first[c]
                    masked = max(0, first[c + 1] - max(first[c], t0))
                    assert 0 < n <= p["max_chunk_tiles"] and masked <= p["max_masked_tiles"], (lv, off, c, p)
                    vis = sum(1 for t in range(max(first[c], t0), first[c + 1]) if t in seen)
                    cost.append((n - masked) + 1.2 * vis + (1 if vis else 0))
                assert max(cost) <= 1.12 * (sum(cost) / len(cost)) + 1, (lv, off, cost, p)


def test_create_refuses_more_cache_positions_than_the_kernels_index():
    """Tile numbers travel as 16-bit values in the attention kernels: a context
    with more than 65535 tiles of 32 positions is refused (and one just below is
    accepted; nothing is allocated at creation)."""
    import ctypes as C
    from synth_inputs import ModelDims
    dims = ModelDims(1, 64, 1, 1, 64, 32, 8)
    desc = fb.ModelDesc(dims.n_layers, dims.d_model, dims.n_q_heads, dims.n_kv_heads, dims.head_dim,
                        dims.d_mlp, dims.vocab, dims.rope_base, dims.norm_eps)
    sl = np.array([32], dtype=np.int32)
    for P, want in [(65534 * 32, fb.FDC_OK), (65535 * 32, fb.FDC_ECAP)]:
        h = C.c_void_p()
        rc = fb.lib().fdc_create(C.byref(desc), 1, fb._p(sl), 0, None, None, P, 1, 1, 1, C.byref(h))
        assert rc == want, (P, rc)
        if rc == fb.FDC_OK:
            fb.lib().fdc_destroy(h)


def test_linear_static_refuses_oversize_before_touching_the_gpu():
    """The entry point that allocates nothing checks its size limit on the host."""
    import ctypes as C
    buf = (C.c_float * 64)()
    a = C.addressof(buf)
    a += (-a) % 16
    rc = fb.lib().fdc_linear_static(a, a, a, 256, 37888, 3584, None)
    assert rc == fb.FDC_ECAP and b"static" in fb.lib().fdc_last_error()


_SAN_DRIVER = r"""
// Drives every host-only entry point over enumerated and pseudo-random inputs
// (valid and invalid) and prints a hash of everything that came back.  Built
// with AddressSanitizer and UndefinedBehaviorSanitizer: a bad access aborts.
#include <cstdio>
#include <cstdint>
#include <vector>
#include "fdc.h"
static uint64_t H = 1469598103934665603ULL;
static void mix(int64_t v) { for (int i = 0; i < 8; ++i) { H ^= (uint64_t)(v >> (8 * i)) & 0xff; H *= 1099511628211ULL; } }
static uint64_t S = 88172645463325252ULL;
static uint32_t rnd(uint32_t n) { S = S * 6364136223846793005ULL + 1442695040888963407ULL; return (uint32_t)((S >> 33) % n); }
int main() {
    for (int it = 0; it < 400; ++it) {
        const int F = 1 + (int)rnd(it < 200 ? 6 : 130);
        std::vector<int32_t> slot(F), src, dst, start(F), level(F), valid(F);
        for (int f = 0; f < F; ++f) slot[f] = 1 + (int)rnd(9);
        const int E = (int)rnd(3 * F + 1);
        for (int e = 0; e < E; ++e) {
            int u = (int)rnd(F), v = (int)rnd(F);
            if (rnd(8) != 0 && u > v) { int t = u; u = v; v = t; }      // mostly forward edges
            if (rnd(40) == 0) v = F + (int)rnd(3);                      // sometimes out of range
            src.push_back(u); dst.push_back(v);
        }
        const int W = (F + 63) / 64, P = (int)rnd(70);
        std::vector<uint64_t> anc((size_t)F * W);
        int32_t total = -1;
        int32_t rc = fdc_build_mask(F, slot.data(), E, src.data(), dst.data(), P, anc.data(), start.data(),
                                    level.data(), &total);
        mix(rc);
        if (rc != FDC_OK) { mix(fdc_last_error()[0] != 0); continue; }
        for (auto a : anc) mix((int64_t)a);
        for (int f = 0; f < F; ++f) { mix(start[f]); mix(level[f]); }
        mix(total);
        // dense mask of a few rows under a random cache state
        const int nr = 1 + (int)rnd(5);
        std::vector<int32_t> rf(nr), ro(nr), pos(nr);
        for (int f = 0; f < F; ++f) valid[f] = (int)rnd(slot[f] + 1);
        for (int r = 0; r < nr; ++r) { rf[r] = (int)rnd(F); ro[r] = (int)rnd(slot[rf[r]]); }
        if (rnd(25) == 0) ro[0] = slot[rf[0]];                           // an offset past the slot
        std::vector<uint8_t> mask((size_t)nr * total);
        rc = fdc_dense_mask(F, slot.data(), start.data(), anc.data(), P, valid.data(), nr, rf.data(), ro.data(),
                            mask.data(), pos.data());
        mix(rc);
        if (rc == FDC_OK) { for (auto m : mask) mix(m); for (auto p : pos) mix(p); }
        // Algorithm 1 to the end with drawn content lengths, through peek / advance
        std::vector<int32_t> len(F), bf(F), bo(F), fin(F), done(F, 0);
        for (int f = 0; f < F; ++f) len[f] = 1 + (int)rnd(slot[f]);
        fdc_sched* sc = nullptr;
        rc = fdc_sched_create(F, E, src.data(), dst.data(), rnd(2) ? len.data() : nullptr, &sc);
        mix(rc);
        if (rc != FDC_OK) continue;
        for (int guard = 0; guard < 100000; ++guard) {
            int32_t n = 0;
            rc = fdc_sched_peek(sc, F, bf.data(), bo.data(), &n);
            mix(rc); mix(n);
            if (rc != FDC_OK || n == 0) break;
            for (int i = 0; i < n; ++i) { mix(bf[i]); mix(bo[i]); done[bf[i]]++; fin[i] = done[bf[i]] >= len[bf[i]]; }
            mix(fdc_sched_advance(sc, n, fin.data()));
        }
        mix(fdc_sched_advance(sc, 3, fin.data()));                       // wrong count: an error, not a fault
        mix(fdc_sched_complete(sc, F, 1));                               // field out of range
        int64_t ps = 0, tk = 0; int32_t un = 0;
        mix(fdc_sched_stats(sc, &ps, &tk, &un)); mix(ps); mix(tk); mix(un);
        fdc_sched_destroy(sc);
    }
    mix(fdc_build_mask(0, nullptr, 0, nullptr, nullptr, 0, nullptr, nullptr, nullptr, nullptr));
    printf("%llu\n", (unsigned long long)H);
    return 0;
}
"""


def test_host_code_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    """fdc_host.cpp (everything of the library that runs without a GPU) built with
    -fsanitize=address,undefined and driven over valid and invalid inputs; the same
    program built without sanitizers against the regular library must print the
    same hash, so the sanitized run did exercise the shipped code's behaviour."""
    import shutil
    import subprocess
    gxx = shutil.which("g++")
    if gxx is None:
        pytest.skip("no C++ compiler")
    src = tmp_path / "drive_host.cpp"
    src.write_text(_SAN_DRIVER)
    inc = ["-I", os.path.join(ROOT, "include"), "-I", os.path.join(ROOT, "paper_2602_02864_amd", "csrc")]
    host = os.path.join(ROOT, "paper_2602_02864_amd", "csrc", "fdc_host.cpp")
    san = tmp_path / "drive_san"
    subprocess.run([gxx, "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                    "-static-libasan", "-static-libubsan", *inc, str(src), host, "-o", str(san)], check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([str(san)], capture_output=True, text=True, env=env)
    assert r.returncode == 0, r.stderr[-3000:]
    plain = tmp_path / "drive_plain"
    libdir = os.path.dirname(fb.LIB_PATH)
    subprocess.run([gxx, "-std=c++17", "-O1", *inc, str(src), "-o", str(plain), "-L", libdir, "-lfdc",
                    "-Wl,-rpath," + libdir], check=True)
    r2 = subprocess.run([str(plain)], capture_output=True, text=True)
    assert r2.returncode == 0, r2.stderr[-3000:]
    assert r.stdout.strip() == r2.stdout.strip() and int(r.stdout) != 0
