"""ctypes binding of libfdc.so.

Argument marshalling only: every function here converts Python / numpy /
torch arguments into the plain pointers and sizes of the C ABI declared in
include/fdc.h and calls the entry point of the same name.  torch is used for
device memory and the current HIP stream, nothing else; no step of the decode
path is computed here.  If the library has not been built the import of the
entry points fails loudly - there is no fallback.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libfdc.so")

FDC_OK, FDC_EINVAL, FDC_ECYCLE, FDC_EORDER, FDC_ERANGE, FDC_ECAP, FDC_EHIP, FDC_ESTATE = \
    0, -1, -2, -3, -4, -5, -6, -7
FDC_PACK_PLAIN, FDC_PACK_GATE_UP, FDC_PACK_F16 = 0, 1, 2

EXPORTS = [
    "fdc_strerror", "fdc_last_error", "fdc_version", "fdc_build_mask", "fdc_dense_mask",
    "fdc_packed_weight_bytes", "fdc_pack_weight", "fdc_create", "fdc_destroy",
    "fdc_kv_cache_bytes", "fdc_workspace_bytes", "fdc_set_kv_cache", "fdc_set_workspace",
    "fdc_set_layer_weights", "fdc_set_head_weights", "fdc_reset", "fdc_set_valid_len",
    "fdc_get_valid_len", "fdc_kv_append", "fdc_parallel_decode_step", "fdc_masked_attention",
    "fdc_argmax", "fdc_linear_scratch_bytes", "fdc_linear", "fdc_linear_static",
    "fdc_profile_enable", "fdc_profile_read", "fdc_profile_kind_name",
    "fdc_profile_calibrate", "fdc_stream_copy",
    "fdc_sched_create", "fdc_sched_next", "fdc_sched_destroy",
    "fdc_sched_peek", "fdc_sched_advance", "fdc_sched_complete", "fdc_sched_stats",
    "fdc_cot_decode", "fdc_step_tables_dense", "fdc_attention_plan", "fdc_attention_plan_step",
    "fdc_set_layer_weights_f16", "fdc_set_head_weights_f16", "fdc_set_f16_projections",
]
FDC_PROF_KINDS = 9


class FdcError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"fdc error {code}: {msg}")
        self.code = code


class ModelDesc(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_q_heads", C.c_int32),
                ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("d_mlp", C.c_int32),
                ("vocab", C.c_int32), ("rope_base", C.c_float), ("norm_eps", C.c_float)]


class LayerWeightsF16(C.Structure):
    _fields_ = [("wqkv", C.c_void_p), ("wo", C.c_void_p), ("wgu", C.c_void_p), ("wd", C.c_void_p)]


class LayerWeights(C.Structure):
    _fields_ = [("g1", C.c_void_p), ("wqkv", C.c_void_p), ("wo", C.c_void_p),
                ("g2", C.c_void_p), ("wgu", C.c_void_p), ("wd", C.c_void_p)]


_lib = None


def lib() -> C.CDLL:
    """Loads libfdc.so (once) and declares the signatures."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with "
                           f"`python -m paper_2602_02864_amd.build` (no fallback exists)")
    L = C.CDLL(LIB_PATH)
    i32, i64, vp, sz = C.c_int32, C.c_int64, C.c_void_p, C.c_size_t
    pi32 = C.POINTER(C.c_int32)
    L.fdc_strerror.restype = C.c_char_p
    L.fdc_strerror.argtypes = [i32]
    L.fdc_last_error.restype = C.c_char_p
    L.fdc_last_error.argtypes = []
    L.fdc_version.restype = i32
    L.fdc_build_mask.restype = i32
    L.fdc_build_mask.argtypes = [i32, pi32, i32, pi32, pi32, i32, C.POINTER(C.c_uint64), pi32, pi32, pi32]
    L.fdc_dense_mask.restype = i32
    L.fdc_dense_mask.argtypes = [i32, pi32, pi32, C.POINTER(C.c_uint64), i32, pi32, i32, pi32, pi32,
                                 C.POINTER(C.c_uint8), pi32]
    L.fdc_packed_weight_bytes.restype = sz
    L.fdc_packed_weight_bytes.argtypes = [i64, i64]
    L.fdc_pack_weight.restype = i32
    L.fdc_pack_weight.argtypes = [vp, vp, i64, i64, i32, vp]
    L.fdc_create.restype = i32
    L.fdc_create.argtypes = [C.POINTER(ModelDesc), i32, pi32, i32, pi32, pi32, i32, i32, i32, i32,
                             C.POINTER(vp)]
    L.fdc_destroy.restype = None
    L.fdc_destroy.argtypes = [vp]
    L.fdc_kv_cache_bytes.restype = sz
    L.fdc_kv_cache_bytes.argtypes = [vp]
    L.fdc_workspace_bytes.restype = sz
    L.fdc_workspace_bytes.argtypes = [vp]
    L.fdc_set_kv_cache.restype = i32
    L.fdc_set_kv_cache.argtypes = [vp, vp, vp]
    L.fdc_set_workspace.restype = i32
    L.fdc_set_workspace.argtypes = [vp, vp, sz, vp]
    L.fdc_set_layer_weights.restype = i32
    L.fdc_set_layer_weights.argtypes = [vp, i32, C.POINTER(LayerWeights)]
    L.fdc_set_head_weights.restype = i32
    L.fdc_set_head_weights.argtypes = [vp, vp, vp, vp]
    L.fdc_set_layer_weights_f16.restype = i32
    L.fdc_set_layer_weights_f16.argtypes = [vp, i32, C.POINTER(LayerWeightsF16)]
    L.fdc_set_head_weights_f16.restype = i32
    L.fdc_set_head_weights_f16.argtypes = [vp, vp]
    L.fdc_set_f16_projections.restype = i32
    L.fdc_set_f16_projections.argtypes = [vp, i32]
    L.fdc_reset.restype = i32
    L.fdc_reset.argtypes = [vp]
    L.fdc_set_valid_len.restype = i32
    L.fdc_set_valid_len.argtypes = [vp, pi32]
    L.fdc_get_valid_len.restype = i32
    L.fdc_get_valid_len.argtypes = [vp, pi32]
    L.fdc_kv_append.restype = i32
    L.fdc_kv_append.argtypes = [vp, i32, vp, vp, vp, vp, i32, vp]
    L.fdc_parallel_decode_step.restype = i32
    L.fdc_parallel_decode_step.argtypes = [vp, i32, i32, pi32, pi32, vp, vp, vp, vp, vp, vp, vp]
    L.fdc_masked_attention.restype = i32
    L.fdc_masked_attention.argtypes = [vp, i32, vp, i32, i32, pi32, pi32, vp, vp]
    L.fdc_argmax.restype = i32
    L.fdc_argmax.argtypes = [vp, i32, i32, i64, vp, vp, vp]
    L.fdc_linear_scratch_bytes.restype = sz
    L.fdc_linear_scratch_bytes.argtypes = [i32, i64, i64]
    L.fdc_linear.restype = i32
    L.fdc_linear.argtypes = [vp, vp, vp, i32, i64, i64, vp, vp]
    L.fdc_linear_static.restype = i32
    L.fdc_linear_static.argtypes = [vp, vp, vp, i32, i64, i64, vp]
    L.fdc_profile_enable.restype = i32
    L.fdc_profile_enable.argtypes = [vp, i32]
    L.fdc_profile_read.restype = i32
    L.fdc_profile_read.argtypes = [vp, C.POINTER(C.c_float), pi32]
    L.fdc_profile_kind_name.restype = C.c_char_p
    L.fdc_profile_kind_name.argtypes = [i32]
    L.fdc_profile_calibrate.restype = i32
    L.fdc_profile_calibrate.argtypes = [i32, vp, sz, C.POINTER(C.c_float), C.POINTER(C.c_float), vp]
    L.fdc_stream_copy.restype = i32
    L.fdc_stream_copy.argtypes = [vp, vp, sz, vp]
    L.fdc_sched_create.restype = i32
    L.fdc_sched_create.argtypes = [i32, i32, pi32, pi32, pi32, C.POINTER(vp)]
    L.fdc_sched_next.restype = i32
    L.fdc_sched_next.argtypes = [vp, i32, pi32, pi32, pi32]
    L.fdc_sched_destroy.restype = None
    L.fdc_sched_destroy.argtypes = [vp]
    L.fdc_sched_peek.restype = i32
    L.fdc_sched_peek.argtypes = [vp, i32, pi32, pi32, pi32]
    L.fdc_sched_advance.restype = i32
    L.fdc_sched_advance.argtypes = [vp, i32, pi32]
    L.fdc_sched_complete.restype = i32
    L.fdc_sched_complete.argtypes = [vp, i32, i32]
    L.fdc_sched_stats.restype = i32
    L.fdc_sched_stats.argtypes = [vp, C.POINTER(C.c_int64), C.POINTER(C.c_int64), C.POINTER(i32)]
    L.fdc_cot_decode.restype = i32
    L.fdc_cot_decode.argtypes = [vp, pi32, pi32, pi32, pi32, i32, i32, pi32, pi32, pi32, vp]
    L.fdc_step_tables_dense.restype = i32
    L.fdc_step_tables_dense.argtypes = [vp, i32, i32, pi32, pi32, C.POINTER(C.c_uint8), pi32, vp]
    L.fdc_attention_plan.restype = i32
    L.fdc_attention_plan.argtypes = [vp, pi32, pi32]
    L.fdc_attention_plan_step.restype = i32
    L.fdc_attention_plan_step.argtypes = [vp, i32, i32, pi32, pi32, pi32, pi32]
    _lib = L
    return L


def _check(rc: int) -> None:
    if rc != FDC_OK:
        raise FdcError(rc, lib().fdc_last_error().decode() or lib().fdc_strerror(rc).decode())


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.int32).reshape(-1))


def _p(a: np.ndarray, ty=C.c_int32):
    return a.ctypes.data_as(C.POINTER(ty))


def _edges(edges):
    e = np.asarray(list(edges), dtype=np.int32).reshape(-1, 2)
    return np.ascontiguousarray(e[:, 0]), np.ascontiguousarray(e[:, 1])


def _stream() -> int:
    import torch
    return torch.cuda.current_stream().cuda_stream


# --------------------------------------------------------------------------- host only
def fdc_build_mask(slot_len: Sequence[int], edges, prefix_len: int) -> dict:
    sl = _i32(slot_len)
    F = sl.size
    src, dst = _edges(edges)
    W = max(1, (F + 63) // 64)
    anc = np.zeros((max(F, 1), W), dtype=np.uint64)
    start = np.zeros(max(F, 1), dtype=np.int32)
    level = np.zeros(max(F, 1), dtype=np.int32)
    total = C.c_int32(0)
    _check(lib().fdc_build_mask(F, _p(sl), src.size, _p(src), _p(dst), int(prefix_len),
                                _p(anc, C.c_uint64), _p(start), _p(level), C.byref(total)))
    return {"anc_words": anc, "slot_start": start, "level": level, "total_len": int(total.value)}


def fdc_dense_mask(slot_len, slot_start, anc_words, prefix_len: int, valid_len, row_field, row_off):
    sl, ss, vl = _i32(slot_len), _i32(slot_start), _i32(valid_len)
    rf, ro = _i32(row_field), _i32(row_off)
    anc = np.ascontiguousarray(np.asarray(anc_words, dtype=np.uint64))
    N = int(ss[-1] + sl[-1])
    mask = np.zeros((rf.size, N), dtype=np.uint8)
    pos = np.zeros(rf.size, dtype=np.int32)
    _check(lib().fdc_dense_mask(sl.size, _p(sl), _p(ss), _p(anc, C.c_uint64), int(prefix_len), _p(vl),
                                rf.size, _p(rf), _p(ro), _p(mask, C.c_uint8), _p(pos)))
    return mask, pos


def fdc_schedule(n_fields: int, edges, content_len, max_branches: Optional[int] = None):
    """Runs fdc_sched_* to completion; returns the list of passes, each a pair
    (branch_field, branch_off) of int32 arrays of length max_branches."""
    src, dst = _edges(edges)
    cl = _i32(content_len)
    R = max_branches or n_fields
    h = C.c_void_p()
    _check(lib().fdc_sched_create(n_fields, src.size, _p(src), _p(dst), _p(cl), C.byref(h)))
    passes = []
    try:
        while True:
            bf = np.zeros(R, dtype=np.int32)
            bo = np.zeros(R, dtype=np.int32)
            n = C.c_int32(0)
            _check(lib().fdc_sched_next(h, R, _p(bf), _p(bo), C.byref(n)))
            if n.value == 0:
                break
            passes.append((bf, bo))
    finally:
        lib().fdc_sched_destroy(h)
    return passes


class Scheduler:
    """fdc_sched_* with finishing decided by the caller (peek / advance / complete)."""

    def __init__(self, n_fields: int, edges, content_len=None):
        src, dst = _edges(edges)
        self.F = n_fields
        self._h = C.c_void_p()
        cl = _i32(content_len) if content_len is not None else None
        _check(lib().fdc_sched_create(n_fields, src.size, _p(src), _p(dst),
                                      _p(cl) if cl is not None else None, C.byref(self._h)))

    def close(self):
        if self._h:
            lib().fdc_sched_destroy(self._h)
            self._h = C.c_void_p()

    __del__ = close

    def peek(self, max_branches: Optional[int] = None):
        R = max_branches or self.F
        bf = np.zeros(R, dtype=np.int32)
        bo = np.zeros(R, dtype=np.int32)
        n = C.c_int32(0)
        _check(lib().fdc_sched_peek(self._h, R, _p(bf), _p(bo), C.byref(n)))
        return bf[:n.value].copy(), bo[:n.value].copy()

    def advance(self, finished):
        fin = _i32(finished)
        _check(lib().fdc_sched_advance(self._h, fin.size, _p(fin) if fin.size else None))

    def complete(self, field: int, n_tokens: int):
        _check(lib().fdc_sched_complete(self._h, field, n_tokens))

    def stats(self):
        p, t, u = C.c_int64(0), C.c_int64(0), C.c_int32(0)
        _check(lib().fdc_sched_stats(self._h, C.byref(p), C.byref(t), C.byref(u)))
        return {"passes": p.value, "tokens": t.value, "unfinished": u.value}


# --------------------------------------------------------------------------- device
def fdc_packed_weight_bytes(n_out: int, k_in: int) -> int:
    return int(lib().fdc_packed_weight_bytes(n_out, k_in))


def fdc_pack_weight(src, mode: int = FDC_PACK_PLAIN):
    """src: torch bf16 [n_out][k_in] on the GPU -> packed torch buffer (bf16, 1-D)."""
    import torch
    assert src.is_cuda and src.dtype == torch.bfloat16 and src.is_contiguous() and src.dim() == 2
    n_out, k_in = src.shape
    dst = torch.empty(fdc_packed_weight_bytes(n_out, k_in) // 2, dtype=torch.bfloat16, device=src.device)
    _check(lib().fdc_pack_weight(src.data_ptr(), dst.data_ptr(), n_out, k_in, mode, _stream()))
    return dst


def fdc_argmax(logits, V: Optional[int] = None, want_gap: bool = True):
    import torch
    assert logits.is_cuda and logits.dtype == torch.float32 and logits.dim() == 2 and logits.is_contiguous()
    M, ld = logits.shape
    V = ld if V is None else V
    idx = torch.empty(M, dtype=torch.int32, device=logits.device)
    gap = torch.empty(M, dtype=torch.float32, device=logits.device) if want_gap else None
    _check(lib().fdc_argmax(logits.data_ptr(), M, V, ld, idx.data_ptr(),
                            gap.data_ptr() if want_gap else None, _stream()))
    return idx, gap


def fdc_linear(x, w_packed, n_out: int):
    import torch
    assert x.is_cuda and x.dtype == torch.float32 and x.dim() == 2 and x.is_contiguous()
    M, k_in = x.shape
    nbytes = int(lib().fdc_linear_scratch_bytes(M, n_out, k_in))
    if nbytes == 0:
        raise FdcError(FDC_ECAP, "shape not supported by fdc_linear")
    # scratch arrives as NaN patterns: rows beyond M must never leak into y
    scratch = torch.full((nbytes,), 0xFF, dtype=torch.uint8, device=x.device)
    y = torch.empty(M, n_out, dtype=torch.float32, device=x.device)
    _check(lib().fdc_linear(x.data_ptr(), w_packed.data_ptr(), y.data_ptr(), M, n_out, k_in,
                            scratch.data_ptr(), _stream()))
    return y


def fdc_linear_static(x, w_packed, n_out: int, out=None):
    """fdc_linear without a workspace argument (the library's static scratch array).
    `out`: an existing fp32 [M][n_out] device tensor to write into (then the call
    allocates nothing on the Python side either)."""
    import torch
    assert x.is_cuda and x.dtype == torch.float32 and x.dim() == 2 and x.is_contiguous()
    M, k_in = x.shape
    y = out if out is not None else torch.empty(M, n_out, dtype=torch.float32, device=x.device)
    assert y.is_cuda and y.dtype == torch.float32 and y.shape == (M, n_out) and y.is_contiguous()
    _check(lib().fdc_linear_static(x.data_ptr(), w_packed.data_ptr(), y.data_ptr(), M, n_out, k_in, _stream()))
    return y


def fdc_profile_calibrate(rounds: int = 200, scratch=None):
    """(cost of an event pair around one launch, duration of that launch), microseconds.
    The launch copies half of the device tensor `scratch` onto its other half; without
    scratch it is an empty kernel."""
    ov, nul = C.c_float(0), C.c_float(0)
    ptr = scratch.data_ptr() if scratch is not None else None
    nb = scratch.numel() * scratch.element_size() if scratch is not None else 0
    _check(lib().fdc_profile_calibrate(rounds, ptr, nb, C.byref(ov), C.byref(nul), _stream()))
    return float(ov.value), float(nul.value)


def fdc_stream_copy(dst, src) -> None:
    """dst <- src for two device tensors of equal byte size (multiple of 16)."""
    nb = src.numel() * src.element_size()
    if nb != dst.numel() * dst.element_size() or not (src.is_contiguous() and dst.is_contiguous()):
        raise ValueError("copy needs contiguous tensors of equal byte size")
    _check(lib().fdc_stream_copy(dst.data_ptr(), src.data_ptr(), nb, _stream()))


def fdc_attention_plan(dims, slot_len, edges, prefix_len, n_scenes=1, max_branches=1, max_tokens=1,
                       step=None) -> dict:
    """The attention launch plan of a context of this shape (host only: no GPU needed).
    step = (valid_len [B][F], branch_field, branch_off, T): the cut of that step."""
    desc = ModelDesc(dims.n_layers, dims.d_model, dims.n_q_heads, dims.n_kv_heads, dims.head_dim,
                     dims.d_mlp, dims.vocab, dims.rope_base, dims.norm_eps)
    sl = _i32(slot_len)
    src, dst = _edges(edges)
    h = C.c_void_p()
    _check(lib().fdc_create(C.byref(desc), sl.size, _p(sl), src.size, _p(src), _p(dst), int(prefix_len),
                            n_scenes, max_branches, max_tokens, C.byref(h)))
    try:
        info = np.zeros(10, dtype=np.int32)
        _check(lib().fdc_attention_plan(h, _p(info), None))
        first = np.zeros(int(info[3]) + 1, dtype=np.int32)
        if step is None:
            _check(lib().fdc_attention_plan(h, _p(info), _p(first)))
        else:
            vl, bf, bo, T = step
            vl, bf, bo = _i32(vl), _i32(bf), _i32(bo)
            _check(lib().fdc_set_valid_len(h, _p(vl)))
            _check(lib().fdc_attention_plan_step(h, bf.size // n_scenes, int(T), _p(bf), _p(bo), _p(info), _p(first)))
            first = first[:int(info[3]) + 1]
    finally:
        lib().fdc_destroy(h)
    keys = ("variant", "nrt", "rg_max", "chunks", "cb", "wq", "tiles", "prefix_tiles", "max_chunk_tiles",
            "max_masked_tiles")
    out = {k: int(v) for k, v in zip(keys, info)}
    out["chunk_first_tile"] = [int(x) for x in first]
    return out


class Context:
    """Owns an fdc_ctx plus the torch buffers handed to it (cache, workspace,
    packed weights).  Methods carry the names of the C entry points."""

    def __init__(self, dims, slot_len, edges, prefix_len, n_scenes=1, max_branches=1, max_tokens=1,
                 device="cuda:0", share=None, weights_from=None, f16_weights=None):
        """share: another Context over the same model and the same cache positions
        (same total length) whose KV cache and packed weights this one uses too.
        weights_from: another Context over the same model whose packed weights this
        one uses (its own cache: any template, any batch).
        f16_weights: fp16 copies for the single-pass projections of steps with more
        than 16 rows: "head" = of the LM head only (the default when such steps can
        occur, i.e. n_scenes * max_branches * max_tokens > 16), "all" / True = of
        every matrix (then fdc_set_f16_projections can enable the layer projections
        too), False = none."""
        import torch
        self.torch = torch
        self.device = torch.device(device)
        self.dims = dims
        self.desc = ModelDesc(dims.n_layers, dims.d_model, dims.n_q_heads, dims.n_kv_heads,
                              dims.head_dim, dims.d_mlp, dims.vocab, dims.rope_base, dims.norm_eps)
        self.slot_len = _i32(slot_len)
        self.F = self.slot_len.size
        self.B, self.Rmax, self.Tmax = n_scenes, max_branches, max_tokens
        src, dst = _edges(edges)
        self._h = C.c_void_p()
        _check(lib().fdc_create(C.byref(self.desc), self.F, _p(self.slot_len), src.size, _p(src), _p(dst),
                                int(prefix_len), n_scenes, max_branches, max_tokens, C.byref(self._h)))
        self._keep = []
        self._layer_w, self._head_w = {}, None
        self._layer_w16, self._head_w16 = {}, None
        if f16_weights is None:
            f16_weights = "head" if n_scenes * max_branches * max_tokens > 16 else False
        self.f16_weights = "all" if f16_weights is True else f16_weights
        assert self.f16_weights in ("all", "head", False)
        self.edges = [(int(u), int(v)) for u, v in zip(src, dst)]
        self.prefix_len = int(prefix_len)
        self.total_len = int(prefix_len) + int(self.slot_len.sum())
        with torch.cuda.device(self.device):
            kvb = int(lib().fdc_kv_cache_bytes(self._h))
            if share is not None and weights_from is not None:
                raise ValueError("give share or weights_from, not both")
            if share is not None:
                if share.k_cache.numel() * 2 != kvb:
                    raise ValueError("contexts that share a cache must cover the same positions")
                self.k_cache, self.v_cache = share.k_cache, share.v_cache
            else:
                self.k_cache = torch.zeros(kvb // 2, dtype=torch.bfloat16, device=self.device)
                self.v_cache = torch.zeros(kvb // 2, dtype=torch.bfloat16, device=self.device)
            _check(lib().fdc_set_kv_cache(self._h, self.k_cache.data_ptr(), self.v_cache.data_ptr()))
            wsb = int(lib().fdc_workspace_bytes(self._h))
            self.workspace = torch.empty(wsb, dtype=torch.uint8, device=self.device)
            _check(lib().fdc_set_workspace(self._h, self.workspace.data_ptr(), wsb, _stream()))
        if share is None and weights_from is not None:
            share = weights_from
        if share is not None:
            for layer, lw in share._layer_w.items():
                _check(lib().fdc_set_layer_weights(self._h, layer, C.byref(lw)))
                self._layer_w[layer] = lw
            if share._head_w is not None:
                _check(lib().fdc_set_head_weights(self._h, *share._head_w))
                self._head_w = share._head_w
            # whatever fp16 copies the other context holds come along (pointers only)
            for layer, lw in share._layer_w16.items():
                _check(lib().fdc_set_layer_weights_f16(self._h, layer, C.byref(lw)))
                self._layer_w16[layer] = lw
            if share._head_w16 is not None:
                _check(lib().fdc_set_head_weights_f16(self._h, share._head_w16))
                self._head_w16 = share._head_w16
            self._keep.append(share._keep)

    def prefill_view(self, max_tokens: int):
        """A context over the same cache and weights in which the prefix is field 0
        (a slot of prefix_len tokens that every other field depends on): stepping
        field 0 with T tokens per pass is the causal prefill of the prefix, a
        multi-token masked prefill inside a slot like any other (Sec. 3.3)."""
        P = self.prefix_len
        if P < 1:
            raise ValueError("no prefix to prefill")
        edges = [(0, f + 1) for f in range(self.F)] + [(u + 1, v + 1) for u, v in self.edges]
        return Context(self.dims, [P] + [int(x) for x in self.slot_len], edges, 0, self.B, 1, max_tokens,
                       device=str(self.device), share=self)

    def prefill(self, emb_rows, chunk: int, want_hidden: bool = True):
        """Causal prefill of field 0 of every scene from embedding rows [B][n][d]
        (bf16 values), `chunk` tokens per pass; returns the last pass's outputs (the
        only pass that runs the LM head: the others just fill the cache)."""
        torch = self.torch
        e = self._dev_bf16(emb_rows).reshape(self.B, -1, self.dims.d_model)
        n = e.shape[1]
        out = None
        for t0 in range(0, n, chunk):
            T = min(chunk, n - t0)
            out = self.parallel_decode_step(np.zeros((self.B, 1), dtype=np.int32),
                                            np.full((self.B, 1), t0, dtype=np.int32),
                                            emb_in=e[:, t0:t0 + T].contiguous(), T=T, want_hidden=want_hidden,
                                            want_tokens=t0 + T >= n)
        return out

    def close(self):
        if getattr(self, "_h", None) is not None and self._h.value:
            self.torch.cuda.synchronize(self.device)
            lib().fdc_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- weights -------------------------------------------------------------------
    def _dev_bf16(self, a):
        """numpy uint16 bf16 patterns / fp32 values of bf16-representable numbers /
        torch tensor -> contiguous torch bf16 tensor on the device."""
        torch = self.torch
        if isinstance(a, torch.Tensor):
            return a.to(self.device, torch.bfloat16).contiguous()
        a = np.asarray(a)
        if a.dtype == np.uint16:
            return torch.from_numpy(a.view(np.int16)).to(self.device).view(torch.bfloat16).contiguous()
        return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(self.device).to(torch.bfloat16)

    def _dev_f32(self, a):
        torch = self.torch
        if isinstance(a, torch.Tensor):
            return a.to(self.device, torch.float32).contiguous()
        return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(self.device)

    def set_layer_weights(self, layer: int, w: dict):
        """w: g1, wqkv, wo, g2, wgu, wd in the row-major [out][in] convention."""
        g1, g2 = self._dev_f32(w["g1"]), self._dev_f32(w["g2"])
        packed, packed16 = {}, {}
        for k in ("wqkv", "wo", "wgu", "wd"):
            src = self._dev_bf16(w[k])
            mode = FDC_PACK_GATE_UP if k == "wgu" else FDC_PACK_PLAIN
            packed[k] = fdc_pack_weight(src, mode)
            if self.f16_weights == "all":
                packed16[k] = fdc_pack_weight(src, mode | FDC_PACK_F16)
            del src
        lw = LayerWeights(g1.data_ptr(), packed["wqkv"].data_ptr(), packed["wo"].data_ptr(),
                          g2.data_ptr(), packed["wgu"].data_ptr(), packed["wd"].data_ptr())
        _check(lib().fdc_set_layer_weights(self._h, layer, C.byref(lw)))
        self._layer_w[layer] = lw
        if self.f16_weights == "all":
            lw16 = LayerWeightsF16(packed16["wqkv"].data_ptr(), packed16["wo"].data_ptr(),
                                   packed16["wgu"].data_ptr(), packed16["wd"].data_ptr())
            _check(lib().fdc_set_layer_weights_f16(self._h, layer, C.byref(lw16)))
            self._layer_w16[layer] = lw16
        self._keep.append((g1, g2, packed, packed16))

    def set_head_weights(self, emb, gf, lm):
        e, g = self._dev_bf16(emb), self._dev_f32(gf)
        lms = self._dev_bf16(lm)
        lmp = fdc_pack_weight(lms)
        self._head_w = (e.data_ptr(), g.data_ptr(), lmp.data_ptr())
        _check(lib().fdc_set_head_weights(self._h, *self._head_w))
        lmp16 = None
        if self.f16_weights:
            lmp16 = fdc_pack_weight(lms, FDC_PACK_PLAIN | FDC_PACK_F16)
            self._head_w16 = lmp16.data_ptr()
            _check(lib().fdc_set_head_weights_f16(self._h, self._head_w16))
        self._keep.append((e, g, lmp, lmp16))

    # -- state ---------------------------------------------------------------------
    def reset(self):
        _check(lib().fdc_reset(self._h))

    def set_valid_len(self, v):
        a = _i32(v)
        assert a.size == self.B * self.F
        _check(lib().fdc_set_valid_len(self._h, _p(a)))

    def set_f16_projections(self, mask: int):
        """Which projections run single-pass on the fp16 weights (1 QKV, 2 O, 4 gate/up, 8 down, 16 LM head)."""
        _check(lib().fdc_set_f16_projections(self._h, int(mask)))

    def get_valid_len(self) -> np.ndarray:
        a = np.zeros(self.B * self.F, dtype=np.int32)
        _check(lib().fdc_get_valid_len(self._h, _p(a)))
        return a.reshape(self.B, self.F)

    def kv_append(self, layer: int, k_new, v_new, row_scene, row_pos):
        torch = self.torch
        k = self._dev_bf16(k_new)
        v = self._dev_bf16(v_new)
        rs = torch.as_tensor(np.asarray(row_scene, dtype=np.int32)).to(self.device)
        rp = torch.as_tensor(np.asarray(row_pos, dtype=np.int32)).to(self.device)
        n = rs.numel()
        assert k.numel() == n * self.dims.n_kv_heads * self.dims.head_dim == v.numel()
        _check(lib().fdc_kv_append(self._h, layer, k.data_ptr(), v.data_ptr(), rs.data_ptr(),
                                   rp.data_ptr(), n, _stream()))
        torch.cuda.current_stream().synchronize()      # temporaries die here

    def profile_enable(self, on: bool):
        _check(lib().fdc_profile_enable(self._h, 1 if on else 0))

    def profile_read(self) -> dict:
        ms = np.zeros(FDC_PROF_KINDS, dtype=np.float32)
        n = np.zeros(FDC_PROF_KINDS, dtype=np.int32)
        _check(lib().fdc_profile_read(self._h, _p(ms, C.c_float), _p(n)))
        return {lib().fdc_profile_kind_name(k).decode(): (float(ms[k]), int(n[k]))
                for k in range(FDC_PROF_KINDS)}

    # -- the step -------------------------------------------------------------------
    def parallel_decode_step(self, branch_field, branch_off, tok_in=None, emb_in=None, T: int = 1,
                             want_logits=False, want_hidden=False, want_gap=True, want_tokens=True) -> dict:
        """want_tokens=False (with no logits and no gaps): the rows only fill the cache, the
        LM head and the argmax are not run (prefill passes)."""
        torch = self.torch
        bf, bo = _i32(branch_field), _i32(branch_off)
        assert bf.size == bo.size and bf.size % self.B == 0
        R = bf.size // self.B
        M = self.B * R * T
        d = self.dims
        dev = self.device
        tok_t = emb_t = None
        if tok_in is not None:
            tok_t = tok_in if isinstance(tok_in, torch.Tensor) else \
                torch.as_tensor(np.asarray(tok_in, dtype=np.int32).reshape(-1)).to(dev)
            assert tok_t.numel() == M and tok_t.dtype == torch.int32
        if emb_in is not None:
            emb_t = self._dev_bf16(emb_in)
            assert emb_t.numel() == M * d.d_model
        out = {"tok": torch.empty(M, dtype=torch.int32, device=dev)} if want_tokens else {}
        if want_gap and want_tokens:
            out["gap"] = torch.empty(M, dtype=torch.float32, device=dev)
        if want_logits:
            out["logits"] = torch.empty(M, d.vocab, dtype=torch.float32, device=dev)
        if want_hidden:
            out["hidden"] = torch.zeros(d.n_layers + 2, M, d.d_model, dtype=torch.float32, device=dev)
        ptr = lambda k: out[k].data_ptr() if k in out else None
        _check(lib().fdc_parallel_decode_step(
            self._h, R, T, _p(bf), _p(bo),
            tok_t.data_ptr() if tok_t is not None else None,
            emb_t.data_ptr() if emb_t is not None else None,
            ptr("tok"), ptr("gap"), ptr("logits"), ptr("hidden"), _stream()))
        out["_inputs"] = (tok_t, emb_t)            # keep alive until the caller syncs
        return out

    def cot_decode(self, start_token, eos_ids=(), fixed=None, max_passes: int = 0):
        """fdc_cot_decode.  fixed: {field: token list} of pre-filled fields.  Returns
        {"tok": [B][F][Smax], "len": [B][F], "passes", "fixed_passes"} (numpy, host)."""
        F, B = len(self.slot_len), self.B
        st = _i32(start_token)
        if st.size != F:
            raise ValueError("start_token needs one entry per field")
        fl = np.zeros(F, dtype=np.int32)
        ft = []
        for f in sorted(fixed or {}):
            fl[f] = len(fixed[f])
            ft.extend(int(t) for t in fixed[f])
        ft = _i32(ft)
        eos = _i32(list(eos_ids))
        Smax = int(max(self.slot_len))
        tok = np.empty((B, F, Smax), dtype=np.int32)
        ln = np.empty((B, F), dtype=np.int32)
        ps = np.zeros(2, dtype=np.int32)
        _check(lib().fdc_cot_decode(self._h, _p(st), _p(fl) if fixed else None, _p(ft) if ft.size else None,
                                    _p(eos) if eos.size else None, eos.size, max_passes,
                                    _p(tok), _p(ln), _p(ps), _stream()))
        return {"tok": tok, "len": ln, "passes": int(ps[0]), "fixed_passes": int(ps[1])}

    def step_tables_dense(self, R: int, T: int = 1, branch_field=None, branch_off=None):
        """fdc_step_tables_dense: (mask [B*R*T][N] uint8, pos [B*R*T] int32) expanded from
        the tables on the device; without branch tables, those of the last step."""
        N = int(self.total_len)
        M = self.B * R * T
        mask = np.empty((M, N), dtype=np.uint8)
        pos = np.empty(M, dtype=np.int32)
        bf = _i32(branch_field) if branch_field is not None else None
        bo = _i32(branch_off) if branch_off is not None else None
        _check(lib().fdc_step_tables_dense(self._h, R, T, _p(bf) if bf is not None else None,
                                           _p(bo) if bo is not None else None, _p(mask, C.c_uint8), _p(pos),
                                           _stream()))
        return mask, pos

    def masked_attention(self, layer: int, q, branch_field, branch_off, T: int = 1):
        torch = self.torch
        bf, bo = _i32(branch_field), _i32(branch_off)
        R = bf.size // self.B
        M = self.B * R * T
        d = self.dims
        qt = self._dev_bf16(q)
        assert qt.numel() == M * d.n_q_heads * d.head_dim
        out = torch.empty(M, d.n_q_heads * d.head_dim, dtype=torch.float32, device=self.device)
        _check(lib().fdc_masked_attention(self._h, layer, qt.data_ptr(), R, T, _p(bf), _p(bo),
                                          out.data_ptr(), _stream()))
        out._fdc_q = qt
        return out
