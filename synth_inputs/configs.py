"""Model dimensions and CoT templates of the five synthetic workloads.

A template is what the method takes as given (Sec. 3.1-3.3 of the paper): an
ordered list of fields, a fixed slot length per field, direct-dependency edges
between fields, and the length of the shared prefix that precedes the first
slot.  `content_len` is the synthetic stand-in for "the field is finished":
a random-init model has no meaningful end-of-line token, so every field is
declared finished after a drawn number of tokens (never more than its slot).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Tuple

import numpy as np

BASE_SEED = 2864000

# order of the independent random sub-streams of a workload
_STREAMS = ("weights", "prefix", "dag", "lengths", "tokens")


def workload_seed(cfg_id: int, stream: str, extra: int = 0) -> np.random.Generator:
    """Generator for one named sub-stream of workload `cfg_id`."""
    idx = _STREAMS.index(stream)
    ss = np.random.SeedSequence([BASE_SEED + cfg_id, idx, extra])
    return np.random.Generator(np.random.PCG64(ss))


@dataclass(frozen=True)
class ModelDims:
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_mlp: int
    vocab: int
    rope_base: float = 1.0e6
    norm_eps: float = 1.0e-6

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def qkv_out(self) -> int:
        return (self.n_q_heads + 2 * self.n_kv_heads) * self.head_dim


@dataclass
class Template:
    prefix_len: int
    slot_len: List[int]
    edges: List[Tuple[int, int]]          # (src, dst): dst needs src complete
    content_len: List[int]                # tokens until the field counts as finished
    start_token: List[int]                # token occupying slot offset 0
    name: str = ""
    extra: dict = field(default_factory=dict)

    @property
    def n_fields(self) -> int:
        return len(self.slot_len)


_DIMS = {
    0: ModelDims(1, 256, 4, 4, 64, 512, 1000),
    1: ModelDims(24, 896, 14, 2, 64, 4864, 32000),
    2: ModelDims(28, 3584, 28, 4, 128, 18944, 32000),
    # workload 3 is attention only; the GEMM dimensions are unused placeholders
    3: ModelDims(1, 4096, 32, 8, 128, 4096, 1000),
    4: ModelDims(28, 3584, 28, 4, 128, 18944, 32000),
}


def model_dims(cfg_id: int, n_layers: int | None = None) -> ModelDims:
    d = _DIMS[cfg_id]
    if n_layers is not None:
        d = ModelDims(n_layers, d.d_model, d.n_q_heads, d.n_kv_heads, d.head_dim,
                      d.d_mlp, d.vocab, d.rope_base, d.norm_eps)
    return d


def _tokens(rng, n, vocab):
    return [int(t) for t in rng.integers(0, vocab, size=n)]


def template(cfg_id: int, *, full_slots: bool = False, rho: float = 0.0,
             dag_seed: int = 0) -> Template:
    """Template of workload `cfg_id`.

    full_slots: every field's content length equals its slot length (worst-case
                critical path) instead of the drawn lengths.
    rho, dag_seed: workload 3 only - edge probability of the random DAG and
                which of the DAG draws to use.
    """
    vocab = _DIMS[cfg_id].vocab
    rng_dag = workload_seed(cfg_id, "dag", dag_seed)
    rng_len = workload_seed(cfg_id, "lengths")
    rng_tok = workload_seed(cfg_id, "tokens")
    if cfg_id == 0:
        F, S, P = 4, 8, 128
        edges = [(0, 3), (1, 3), (2, 3)]
        lens = [S] * F
    elif cfg_id == 1:
        F, S, P = 8, 48, 1536
        edges = [(i, j) for j in (6, 7) for i in range(6)]
        lens = [int(x) for x in rng_len.integers(16, 49, size=F)]
    elif cfg_id == 2:
        F, S, P = 12, 64, 3072
        edges = []
        for f in (8, 9, 10):
            k = int(rng_dag.integers(2, 5))
            parents = sorted(int(p) for p in rng_dag.choice(8, size=k, replace=False))
            edges += [(p, f) for p in parents]
        edges += [(p, 11) for p in range(11)]
        lens = [int(x) for x in rng_len.integers(24, 65, size=F)]
    elif cfg_id == 3:
        F, S, P = 16, 64, 4096
        edges = [(i, j) for j in range(F) for i in range(j) if rng_dag.random() < rho] \
            if rho < 1.0 else [(i, j) for j in range(F) for i in range(j)]
        lens = [S] * F
    elif cfg_id == 4:
        F, S, P = 32, 32, 8192
        per = 8
        edges = []
        for v in range(per, F):
            lv = v // per
            got_prev = False
            for u in range(0, lv * per):
                if rng_dag.random() < 0.2:
                    edges.append((u, v))
                    got_prev = got_prev or (u // per == lv - 1)
            if not got_prev:
                u = (lv - 1) * per + int(rng_dag.integers(0, per))
                edges.append((u, v))
        edges = sorted(set(edges), key=lambda e: (e[1], e[0]))
        lens = [S] * F
    else:
        raise ValueError(f"unknown workload {cfg_id}")
    if full_slots:
        lens = [S] * F
    return Template(prefix_len=P, slot_len=[S] * F, edges=edges, content_len=lens,
                    start_token=_tokens(rng_tok, F, vocab), name=f"cfg{cfg_id}",
                    extra={"rho": rho, "dag_seed": dag_seed})


def random_dag_template(seed: int, n_fields: int, prefix_len: int, max_slot: int,
                        edge_prob: float, vocab: int) -> Template:
    """Small random template for tests: ragged slots, ragged content lengths,
    edges only from an earlier field to a later one."""
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([7717, seed])))
    slot = [int(x) for x in rng.integers(1, max_slot + 1, size=n_fields)]
    lens = [int(rng.integers(1, s + 1)) for s in slot]
    edges = [(i, j) for j in range(n_fields) for i in range(j) if rng.random() < edge_prob]
    return Template(prefix_len, slot, edges, lens, _tokens(rng, n_fields, vocab),
                    name=f"rand{seed}")


def chain_template(n_fields: int, slot: int, prefix_len: int, vocab: int,
                   seed: int = 0) -> Template:
    """Field i depends on field i-1; every slot full.  Equivalent to ordinary
    autoregressive decoding of the concatenated sequence."""
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([7718, seed])))
    return Template(prefix_len, [slot] * n_fields,
                    [(i, i + 1) for i in range(n_fields - 1)], [slot] * n_fields,
                    _tokens(rng, n_fields, vocab), name="chain")


def edgeless_template(n_fields: int, slot: int, prefix_len: int, vocab: int,
                      seed: int = 0) -> Template:
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([7719, seed])))
    return Template(prefix_len, [slot] * n_fields, [], [slot] * n_fields,
                    _tokens(rng, n_fields, vocab), name="edgeless")
