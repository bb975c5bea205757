"""CPU oracle for one parallel-decoding step of template-structured CoT.

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain, fp64 definition the
GPU library is checked against.  Nothing in the product path may import it;
only tests, the smoke check and the benchmark's CPU-baseline leg do.  It shares
no code with the HIP path and imports nothing from it.

What it computes follows the paper's Sec. 3.2 (dependency graph, Algorithm 1)
and Sec. 3.3 (single packed sequence, ancestor attention mask of Eq. 1, fixed
slot lengths that fix position ids, invisible and unprocessed padding, fully
reused KV cache).  The method is exact: every decoded row is the output of an
ordinary pre-norm decoder (RMSNorm, GQA attention with rotary embedding,
SwiGLU MLP - the Qwen family named in Sec. 4.1) whose attention set is the
row's visible set.  The oracle is therefore that definition written out with a
dense boolean mask and no blocking, fusion or caching tricks.

Readings the paper does not fix (parity unpinned by the paper; fixed here and
mirrored by the library): strict ancestors plus a separate own-slot causal
clause; rotate-half rotary convention with base 1e6; no biases; eps 1e-6;
untied LM head; softmax scale 1/sqrt(D); append-then-attend inside a step;
first token of a field is a given start token at slot offset 0; lowest index
wins argmax ties.  The workloads hold the KV cache in bf16 ("bf16 weights and
KV"; Sec. 4.1: BFloat16 for most calculations): with kv_bf16=True the oracle
rounds K and V to bf16 at the moment it stores them in its cache - a storage
format, like the bf16 weights - and still computes everything in fp64.  The
default (False) is the unrounded definition the CPU pins use.
"""
from __future__ import annotations

import numpy as np

F64 = np.float64


# --------------------------------------------------------------------------
# Sec. 3.3: fixed slot lengths => every position id is known in advance
# --------------------------------------------------------------------------
def slot_layout(prefix_len, slot_len):
    """slot_start[f] = prefix_len + sum of earlier slots; returns (starts, N)."""
    starts, at = [], int(prefix_len)
    for s in slot_len:
        starts.append(at)
        at += int(s)
    return starts, at


def position_ids(slot_start, row_field, row_off):
    """Position (= cache index) of slot offset `off` of field `f`."""
    return [slot_start[f] + t for f, t in zip(row_field, row_off)]


# --------------------------------------------------------------------------
# Sec. 3.2 / Eq. 1: ancestors = fields from which a path of >= 1 edge leads here
# --------------------------------------------------------------------------
def check_template(n_fields, edges):
    """Raise ValueError unless the edges form a DAG over fields 0..F-1 whose
    field order is a topological order (every edge goes to a later field), so
    that every visible key sits at a smaller position than its query."""
    for (u, v) in edges:
        if not (0 <= u < n_fields and 0 <= v < n_fields):
            raise ValueError(f"edge ({u},{v}) names a field outside 0..{n_fields - 1}")
        if u == v:
            raise ValueError(f"self-loop on field {u}: not a DAG")
    # Kahn's peeling detects cycles independently of the order test below
    indeg = [0] * n_fields
    for (_, v) in set(edges):
        indeg[v] += 1
    ready = [v for v in range(n_fields) if indeg[v] == 0]
    seen = 0
    while ready:
        v = ready.pop()
        seen += 1
        for (a, b) in set(edges):
            if a == v:
                indeg[b] -= 1
                if indeg[b] == 0:
                    ready.append(b)
    if seen != n_fields:
        raise ValueError("dependency graph has a cycle")
    for (u, v) in edges:
        if u > v:
            raise ValueError(f"edge ({u},{v}) points to an earlier field")


def ancestors(n_fields, edges):
    """Strict ancestor set of every field, by depth-first search from the
    field over reversed edges (one search per field)."""
    parents = [[] for _ in range(n_fields)]
    for (u, v) in edges:
        parents[v].append(u)
    out = []
    for f in range(n_fields):
        seen, stack = set(), list(parents[f])
        while stack:
            g = stack.pop()
            if g in seen:
                continue
            seen.add(g)
            stack.extend(parents[g])
        out.append(seen)
    return out


def ancestor_words(n_fields, edges):
    """Ancestor sets as bit words: bit (g % 64) of word g // 64 of row f."""
    W = max(1, (n_fields + 63) // 64)
    words = np.zeros((n_fields, W), dtype=np.uint64)
    for f, s in enumerate(ancestors(n_fields, edges)):
        for g in s:
            words[f, g // 64] |= np.uint64(1) << np.uint64(g % 64)
    return words


def levels(n_fields, edges):
    """Longest-path depth of every field (roots are level 0)."""
    memo = {}
    parents = [[] for _ in range(n_fields)]
    for (u, v) in edges:
        parents[v].append(u)

    def depth(f):
        if f not in memo:
            memo[f] = 0 if not parents[f] else 1 + max(depth(p) for p in parents[f])
        return memo[f]
    return [depth(f) for f in range(n_fields)]


# --------------------------------------------------------------------------
# Sec. 3.3: the attention mask
# --------------------------------------------------------------------------
def visible_row(prefix_len, slot_start, slot_len, anc, valid_len, f, t):
    """Boolean [N]: which cache positions the token at offset t of field f sees.

    A position j is visible iff it is in the shared prefix, or it is an
    already-written (non-padding) token of a strict ancestor field, or it is a
    token of the same field at offset <= t.  `valid_len[g]` is the number of
    tokens of field g in the cache after this step's appends.
    """
    N = slot_start[-1] + slot_len[-1] if len(slot_len) else prefix_len
    vis = np.zeros(N, dtype=bool)
    vis[:prefix_len] = True
    for g in anc[f]:
        vis[slot_start[g]: slot_start[g] + valid_len[g]] = True
    vis[slot_start[f]: slot_start[f] + t + 1] = True
    return vis


def dense_mask(prefix_len, slot_len, edges, valid_len, row_field, row_off):
    """[rows][N] boolean mask and [rows] position ids for one scene."""
    slot_start, N = slot_layout(prefix_len, slot_len)
    anc = ancestors(len(slot_len), edges)
    mask = np.zeros((len(row_field), N), dtype=bool)
    for r, (f, t) in enumerate(zip(row_field, row_off)):
        mask[r] = visible_row(prefix_len, slot_start, slot_len, anc, valid_len, f, t)
    return mask, np.asarray(position_ids(slot_start, row_field, row_off), dtype=np.int32)


# --------------------------------------------------------------------------
# Decoder arithmetic (stock pre-norm decoder, Sec. 4.1 model family)
# --------------------------------------------------------------------------
def rmsnorm(x, g, eps):
    x = np.asarray(x, dtype=F64)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * np.asarray(g, dtype=F64)


def rope(x, pos, base):
    """Rotary embedding, rotate-half convention.  x: [..., D]; pos broadcasts
    over the leading axes.  Pair (i, i + D/2) is rotated by pos * base**(-2i/D)."""
    x = np.asarray(x, dtype=F64)
    D = x.shape[-1]
    half = D // 2
    inv_freq = F64(base) ** (-np.arange(half, dtype=F64) * 2.0 / D)
    ang = np.asarray(pos, dtype=F64)[..., None] * inv_freq
    c, s = np.cos(ang), np.sin(ang)
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


def silu(x):
    return x / (1.0 + np.exp(-x))


def softmax(s):
    e = np.exp(s - np.max(s))
    return e / np.sum(e)


def attend(q, K, V, visible):
    """One query head against the visible keys: softmax(q.K/sqrt(D)) V."""
    idx = np.nonzero(visible)[0]
    s = K[idx] @ q / np.sqrt(F64(q.shape[-1]))
    return softmax(s) @ V[idx]


def greedy(logits):
    """(token, top-2 gap): lowest index among the maxima; gap to the runner-up."""
    tok = int(np.argmax(logits))          # numpy returns the first maximum
    rest = np.delete(logits, tok)
    gap = float(logits[tok] - np.max(rest)) if rest.size else float("inf")
    return tok, gap


def _f64(a):
    return np.asarray(a, dtype=F64)


def to_bf16(x):
    """Nearest bf16 value (ties to even) of every element, returned as fp64.
    bf16 keeps the top 16 bits of the fp32 pattern: round the fp32 value there."""
    f = np.ascontiguousarray(x, dtype=np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    keep = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    out = keep.astype(np.uint32).view(np.float32).astype(F64)
    return np.where(np.isfinite(f), out, f.astype(F64))


class OracleDecoder:
    """fp64 decoder with a position-indexed KV cache and per-scene valid lengths.

    weights: {'emb','gf','lm', 'layers': sequence or callable l -> layer dict};
    layer dict keys g1, wqkv, wo, g2, wgu, wd; matrices are [out][in].
    Cache positions that were never written hold NaN, so any read of padding
    or of a not-yet-decoded token poisons the result instead of hiding.
    """

    def __init__(self, dims, weights, prefix_len, slot_len, edges, n_scenes=1, kv_bf16=False):
        check_template(len(slot_len), edges)
        self.kv_bf16 = bool(kv_bf16)
        self.d = dims
        self.w = weights
        self.prefix_len = int(prefix_len)
        self.slot_len = [int(s) for s in slot_len]
        self.edges = [(int(u), int(v)) for (u, v) in edges]
        self.slot_start, self.N = slot_layout(prefix_len, slot_len)
        self.anc = ancestors(len(slot_len), edges)
        self.B = n_scenes
        L, Hkv, D = dims.n_layers, dims.n_kv_heads, dims.head_dim
        self.K = np.full((L, n_scenes, Hkv, self.N, D), np.nan, dtype=F64)
        self.V = np.full((L, n_scenes, Hkv, self.N, D), np.nan, dtype=F64)
        self.valid_len = np.zeros((n_scenes, len(slot_len)), dtype=np.int64)

    # -- weights ------------------------------------------------------------
    def layer(self, l):
        lw = self.w["layers"]
        lw = lw(l) if callable(lw) else lw[l]
        return {k: _f64(v) for k, v in lw.items()}

    # -- shared per-row pieces ---------------------------------------------
    def _qkv(self, lw, x, pos):
        d = self.d
        a = rmsnorm(x, lw["g1"], d.norm_eps)
        qkv = a @ lw["wqkv"].T
        nq, nk = d.n_q_heads * d.head_dim, d.n_kv_heads * d.head_dim
        q = qkv[:, :nq].reshape(-1, d.n_q_heads, d.head_dim)
        k = qkv[:, nq:nq + nk].reshape(-1, d.n_kv_heads, d.head_dim)
        v = qkv[:, nq + nk:].reshape(-1, d.n_kv_heads, d.head_dim)
        pos = np.asarray(pos)
        q = rope(q, pos[:, None], d.rope_base)
        k = rope(k, pos[:, None], d.rope_base)
        return q, k, v

    def _mlp(self, lw, x):
        d = self.d
        a = rmsnorm(x, lw["g2"], d.norm_eps)
        gu = a @ lw["wgu"].T
        h = silu(gu[:, :d.d_mlp]) * gu[:, d.d_mlp:]
        return x + h @ lw["wd"].T

    # -- prefix -------------------------------------------------------------
    def prefill_prefix(self, scene, x_rows):
        """Ordinary causal pass over the prefix rows (embeddings [P][d]); fills
        cache positions 0..P-1 of `scene` in every layer, returns final x."""
        d = self.d
        P = self.prefix_len
        x = _f64(x_rows)
        assert x.shape == (P, d.d_model)
        causal = np.tril(np.ones((P, P), dtype=bool))
        pos = np.arange(P)
        for l in range(d.n_layers):
            lw = self.layer(l)
            q, k, v = self._qkv(lw, x, pos)
            self.K[l, scene, :, :P] = k.transpose(1, 0, 2)
            self.V[l, scene, :, :P] = v.transpose(1, 0, 2)
            o = np.zeros((P, d.n_q_heads, d.head_dim), dtype=F64)
            for h in range(d.n_q_heads):
                kh = h // d.group
                s = q[:, h] @ k[:, kh].T / np.sqrt(F64(d.head_dim))
                s = np.where(causal, s, -np.inf)
                p = np.exp(s - s.max(axis=1, keepdims=True))
                p /= p.sum(axis=1, keepdims=True)
                o[:, h] = p @ v[:, kh]
            x = x + o.reshape(P, -1) @ lw["wo"].T
            x = self._mlp(lw, x)
        return x

    def set_prefix_kv(self, scene, K, V):
        """Install given prefix K/V ([L][Hkv][P][D], K already rotated)."""
        P = self.prefix_len
        self.K[:, scene, :, :P] = _f64(K)
        self.V[:, scene, :, :P] = _f64(V)

    # -- one parallel decoding step (Sec. 3.3; body of Algorithm 1's loop) ---
    def step(self, branch_field, branch_off, tok_in=None, emb_in=None, T=1):
        """Decode T tokens for every active branch of every scene in one pass.

        branch_field, branch_off: [B][R]; field -1 marks an inactive entry.
        tok_in: [B][R][T] token ids, or emb_in: [B][R][T][d] embedding rows.
        Row order of every output is m = (b*R + r)*T + t; inactive rows hold
        NaN / token -1.  The step appends all K/V first, then attends.
        """
        d = self.d
        bf = np.asarray(branch_field).reshape(self.B, -1)
        bo = np.asarray(branch_off).reshape(self.B, -1)
        R = bf.shape[1]
        M = self.B * R * T
        rows = []                                  # (m, scene, field, offset)
        for b in range(self.B):
            for r in range(R):
                f = int(bf[b, r])
                if f < 0:
                    continue
                if not 0 <= f < len(self.slot_len):
                    raise ValueError("field id out of range")
                if bo[b, r] < 0 or bo[b, r] + T > self.slot_len[f]:
                    raise ValueError("tokens do not fit the field's slot")
                for t in range(T):
                    rows.append(((b * R + r) * T + t, b, f, int(bo[b, r]) + t))
        idx = np.array([m for (m, _, _, _) in rows], dtype=np.int64)
        pos = np.array([self.slot_start[f] + o for (_, _, f, o) in rows], dtype=np.int64)
        if emb_in is not None:
            x = _f64(emb_in).reshape(M, d.d_model)[idx]
        else:
            tok = np.asarray(tok_in).reshape(M)[idx]
            x = _f64(self.w["emb"])[tok]

        # padding is never processed: only offsets actually decoded count
        valid_after = self.valid_len.copy()
        for b in range(self.B):
            for r in range(R):
                if bf[b, r] >= 0:
                    valid_after[b, bf[b, r]] = max(valid_after[b, bf[b, r]], bo[b, r] + T)

        hidden = np.full((d.n_layers + 1, M, d.d_model), np.nan, dtype=F64)
        hidden[0, idx] = x
        for l in range(d.n_layers):
            lw = self.layer(l)
            q, k, v = self._qkv(lw, x, pos)
            if self.kv_bf16:                                 # the cache's storage format
                k, v = to_bf16(k), to_bf16(v)
            for i, (_, b, f, o) in enumerate(rows):          # append ...
                self.K[l, b, :, pos[i]] = k[i]
                self.V[l, b, :, pos[i]] = v[i]
            att = np.zeros((len(rows), d.n_q_heads, d.head_dim), dtype=F64)
            for i, (_, b, f, o) in enumerate(rows):          # ... then attend
                vis = visible_row(self.prefix_len, self.slot_start, self.slot_len,
                                  self.anc, valid_after[b], f, o)
                for h in range(d.n_q_heads):
                    kh = h // d.group
                    att[i, h] = attend(q[i, h], self.K[l, b, kh], self.V[l, b, kh], vis)
            x = x + att.reshape(len(rows), -1) @ lw["wo"].T
            x = self._mlp(lw, x)
            hidden[l + 1, idx] = x
        self.valid_len = valid_after

        xn = rmsnorm(x, self.w["gf"], d.norm_eps)
        logits_rows = xn @ _f64(self.w["lm"]).T
        normed = np.full((M, d.d_model), np.nan, dtype=F64)
        logits = np.full((M, d.vocab), np.nan, dtype=F64)
        tok_out = np.full(M, -1, dtype=np.int32)
        gap = np.full(M, np.nan, dtype=F64)
        normed[idx] = xn
        logits[idx] = logits_rows
        for i, m in enumerate(idx):
            tok_out[m], gap[m] = greedy(logits_rows[i])
        return {"hidden": hidden, "normed": normed, "logits": logits, "tok": tok_out,
                "gap": gap, "pos": pos.astype(np.int32), "rows": idx}


def attention_only(q, K, V, prefix_len, slot_len, edges, valid_len, row_field, row_off, group):
    """Masked GQA attention of one scene on given tensors.
    q: [rows][Hq][D] (already rotated), K, V: [Hkv][N][D]; returns [rows][Hq][D]."""
    q, K, V = _f64(q), _f64(K), _f64(V)
    slot_start, _ = slot_layout(prefix_len, slot_len)
    anc = ancestors(len(slot_len), edges)
    out = np.zeros_like(q)
    for r in range(q.shape[0]):
        vis = visible_row(prefix_len, slot_start, slot_len, anc, valid_len,
                          row_field[r], row_off[r])
        for h in range(q.shape[1]):
            out[r, h] = attend(q[r, h], K[h // group], V[h // group], vis)
    return out


# --------------------------------------------------------------------------
# Algorithm 1: ready-set scheduling over the dependency graph
# --------------------------------------------------------------------------
def schedule(n_fields, edges, content_len):
    """Run Algorithm 1 with "field v is finished" := content_len[v] tokens have
    been decoded.  Returns the list of steps; each step is the list of
    (field, offset) decoded in that forward pass, in field order."""
    indeg = [0] * n_fields
    succ = [[] for _ in range(n_fields)]
    for (u, v) in set(edges):
        indeg[v] += 1
        succ[u].append(v)
    ready = {v for v in range(n_fields) if indeg[v] == 0}
    done = [0] * n_fields
    steps = []
    while ready:
        steps.append([(v, done[v]) for v in sorted(ready)])
        for v in sorted(ready):
            done[v] += 1
            if done[v] >= content_len[v]:
                ready.discard(v)
                for u in succ[v]:
                    indeg[u] -= 1
                    if indeg[u] == 0:
                        ready.add(u)
    return steps


def run_cot(dec, content_len, start_token, forced_tokens=None):
    """Greedy template decoding of scene 0 of `dec` (B == 1) to completion.

    The input of a field's first row is its start token; afterwards it is the
    token the previous step produced for that field (or forced_tokens[step][i]
    when given).  Returns the per-step oracle outputs plus the inputs used."""
    assert dec.B == 1
    F = len(dec.slot_len)
    steps = schedule(F, dec.edges, content_len)
    R = max(len(s) for s in steps)
    last_tok = list(start_token)
    trace = []
    for si, st in enumerate(steps):
        bf = [-1] * R
        bo = [0] * R
        ti = [0] * R
        for i, (f, o) in enumerate(st):
            bf[i], bo[i] = f, o
            ti[i] = last_tok[f] if forced_tokens is None else int(forced_tokens[si][i])
        out = dec.step([bf], [bo], tok_in=np.array(ti, dtype=np.int32).reshape(1, R, 1))
        for i, (f, o) in enumerate(st):
            last_tok[f] = int(out["tok"][i])
        trace.append({"branch_field": bf, "branch_off": bo, "tok_in": ti, "out": out})
    return trace


def run_cot_dynamic(dec, start_token, eos_ids=(), fixed=None):
    """Algorithm 1 with the finishing rules of Sec. 3.3, for every scene of `dec`.

    A field is finished when the token it just produced is in `eos_ids` (the
    model ended the line) or when its slot is full (truncation to the fixed
    length).  The first input of a field is its start token; afterwards the
    token it produced in the previous pass.  `fixed` maps a field to tokens
    known from the start (template text): those fields are written before the
    loop starts and count as finished; who sees them follows from the edges.
    Scenes run Algorithm 1 independently and share each forward pass.

    Returns text[b][v] (tokens recorded for field v of scene b), the number of
    passes of the loop, and per pass what was decoded and the top-2 logit gaps.
    """
    F, B = len(dec.slot_len), dec.B
    eos = set(int(t) for t in eos_ids)
    fixed = {int(f): [int(t) for t in toks] for f, toks in (fixed or {}).items()}
    preds = [set() for _ in range(F)]
    succ = [set() for _ in range(F)]
    for (u, v) in set(dec.edges):
        preds[v].add(u)
        succ[u].add(v)
    dec.valid_len[:] = 0
    text = [[[] for _ in range(F)] for _ in range(B)]
    for f in sorted(fixed):
        toks = fixed[f]
        if not preds[f] <= set(fixed):
            raise ValueError("a fixed field may only depend on fixed fields")
        if not 0 < len(toks) <= dec.slot_len[f]:
            raise ValueError("fixed text does not fit its slot")
        dec.step([[f]] * B, [[0]] * B, tok_in=np.array([toks] * B, dtype=np.int32).reshape(B, 1, len(toks)),
                 T=len(toks))
        for b in range(B):
            text[b][f] = list(toks)
    # d_v and S of Algorithm 1, one copy per scene; fixed fields have signalled already
    d = [[len(preds[v] - set(fixed)) for v in range(F)] for _ in range(B)]
    S = [{v for v in range(F) if d[b][v] == 0 and v not in fixed} for b in range(B)]
    last = [list(start_token) for _ in range(B)]
    trace = []
    while any(S):
        R = max(len(s) for s in S)
        bf = np.full((B, R), -1, dtype=np.int32)
        bo = np.zeros((B, R), dtype=np.int32)
        ti = np.zeros((B, R, 1), dtype=np.int32)
        for b in range(B):
            for i, v in enumerate(sorted(S[b])):
                bf[b, i], bo[b, i], ti[b, i, 0] = v, len(text[b][v]), last[b][v]
        out = dec.step(bf, bo, tok_in=ti)
        gaps = []
        for b in range(B):
            for i, v in enumerate(sorted(S[b])):
                t = int(out["tok"][b * R + i])
                gaps.append(float(out["gap"][b * R + i]))
                text[b][v].append(t)
                last[b][v] = t
                if t in eos or len(text[b][v]) >= dec.slot_len[v]:
                    S[b].discard(v)
                    for u in succ[v]:
                        d[b][u] -= 1
                        if d[b][u] == 0:
                            S[b].add(u)
        trace.append({"branch_field": bf, "branch_off": bo, "tok_in": ti, "gaps": gaps})
    return {"text": text, "passes": len(trace), "trace": trace,
            "min_gap": min((g for p in trace for g in p["gaps"]), default=float("inf"))}
