"""Thin ctypes binding of libems_hip.so (C ABI in include/ems.h).

Argument marshalling only: every step of the path runs in the HIP kernels.  PyTorch is used
for device memory and the current stream.  There is no CPU fallback: if the library is not
built, importing the entry points raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libems_hip.so")

EMS_OK = 0
EMS_ERR_INVALID_ARG = -1
EMS_ERR_UNSUPPORTED = -2
EMS_ERR_WORKSPACE = -3
EMS_ERR_LAUNCH = -4
EMS_BF16 = 0
EMS_F32 = 1
EMS_SIM_KEY = 0
EMS_SIM_VALUE = 1
EMS_SIM_KEY_VALUE = 2
EMS_STEP_FROM_STATE = -1

EXPORTS = ("ems_version", "ems_strerror", "ems_partition_sizes", "ems_workspace_bytes",
           "ems_global_local_score", "ems_attention_lse", "ems_global_local_score_from_lse",
           "ems_select", "ems_evict_merge", "ems_evict_merge_variant", "ems_evict_merge_static", "ems_expand",
           "ems_decode_workspace_bytes", "ems_decode_init", "ems_decode_step",
           "ems_sparsity_rate", "ems_redundancy_rate")


class ems_params(C.Structure):
    _fields_ = [("batch", C.c_int32), ("q_heads", C.c_int32), ("kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("seq_len", C.c_int32), ("window", C.c_int32),
                ("budget", C.c_int32), ("merge_ratio", C.c_float), ("tau", C.c_float),
                ("pool_kernel", C.c_int32), ("softmax_scale", C.c_float), ("dtype", C.c_int32)]


STATE_FIELDS = ("k_cache", "v_cache", "row_norm", "entry_count", "entry_tok", "tok_pos", "tok_row",
                "tok_norm", "tok_glo", "tok_past", "tok_cur", "step_count")


class ems_decode_state(C.Structure):
    _fields_ = [(name, C.c_void_p) for name in STATE_FIELDS]


class EmsError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {strerror(status)} ({status})")


@dataclass
class EmsParams:
    batch: int
    q_heads: int
    kv_heads: int
    head_dim: int
    seq_len: int
    window: int
    budget: int = 0
    merge_ratio: float = 0.5
    tau: float = 0.6
    pool_kernel: int = 7
    softmax_scale: float = 0.0
    dtype: int = EMS_BF16

    def c(self) -> ems_params:
        return ems_params(self.batch, self.q_heads, self.kv_heads, self.head_dim, self.seq_len,
                          self.window, self.budget, self.merge_ratio, self.tau,
                          self.pool_kernel, self.softmax_scale, self.dtype)

    @property
    def torch_dtype(self):
        return torch.float32 if self.dtype == EMS_F32 else torch.bfloat16


_lib = None


def lib():
    """Load the built library (never builds, never falls back)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is not built: run `python -m paper_2412_08521_amd.build`")
        l = C.CDLL(LIB_PATH)
        l.ems_version.restype = C.c_int
        l.ems_strerror.restype = C.c_char_p
        l.ems_strerror.argtypes = [C.c_int]
        P = C.POINTER(ems_params)
        l.ems_partition_sizes.argtypes = [P, C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
        l.ems_workspace_bytes.argtypes = [P] + [C.POINTER(C.c_size_t)] * 3
        l.ems_global_local_score.argtypes = [P] + [C.c_void_p] * 6 + [C.c_size_t, C.c_void_p]
        l.ems_attention_lse.argtypes = [P] + [C.c_void_p] * 4 + [C.c_size_t, C.c_void_p]
        l.ems_global_local_score_from_lse.argtypes = [P] + [C.c_void_p] * 6 + [C.c_size_t, C.c_void_p]
        l.ems_select.argtypes = [P] + [C.c_void_p] * 6 + [C.c_size_t, C.c_void_p]
        l.ems_evict_merge.argtypes = [P] + [C.c_void_p] * 12 + [C.c_size_t, C.c_void_p]
        l.ems_evict_merge_variant.argtypes = ([P, C.c_int] + [C.c_void_p] * 13 + [C.c_size_t, C.c_void_p])
        l.ems_evict_merge_static.argtypes = [P] + [C.c_void_p] * 12
        l.ems_expand.argtypes = [P] + [C.c_void_p] * 10
        l.ems_sparsity_rate.argtypes = [P, C.c_float] + [C.c_void_p] * 5
        l.ems_redundancy_rate.argtypes = [P] + [C.c_void_p] * 5
        S = C.POINTER(ems_decode_state)
        l.ems_decode_workspace_bytes.argtypes = [P, C.POINTER(C.c_size_t)]
        l.ems_decode_init.argtypes = [P] + [C.c_void_p] * 7 + [S, C.c_void_p]
        l.ems_decode_step.argtypes = [P, S, C.c_int32] + [C.c_void_p] * 6 + [C.c_void_p, C.c_size_t, C.c_void_p]
        for name in EXPORTS[2:]:
            getattr(l, name).restype = C.c_int
        _lib = l
    return _lib


def strerror(status: int) -> str:
    return lib().ems_strerror(int(status)).decode()


def ems_version() -> int:
    return int(lib().ems_version())


def ems_partition_sizes(p: EmsParams):
    a, b = C.c_int32(0), C.c_int32(0)
    cp = p.c()
    rc = lib().ems_partition_sizes(C.byref(cp), C.byref(a), C.byref(b))
    if rc != EMS_OK:
        raise EmsError(rc, "ems_partition_sizes")
    return int(a.value), int(b.value)


def ems_workspace_bytes(p: EmsParams, full: bool = True):
    s, t, u = C.c_size_t(0), C.c_size_t(0), C.c_size_t(0)
    cp = p.c()
    rc = lib().ems_workspace_bytes(C.byref(cp), C.byref(s), C.byref(t) if full else None,
                                   C.byref(u) if full else None)
    if rc != EMS_OK:
        raise EmsError(rc, "ems_workspace_bytes")
    return int(s.value), int(t.value), int(u.value)


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check_tensor(t, shape, dtype, name):
    if not t.is_cuda:
        raise ValueError(f"{name} must be a device tensor")
    if tuple(t.shape) != tuple(shape) or t.dtype != dtype or not t.is_contiguous():
        raise ValueError(f"{name}: expected contiguous {dtype} {tuple(shape)}, got {t.dtype} {tuple(t.shape)}")


def _workspace(nbytes: int, device, ws=None):
    if ws is None:
        ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)
    return ws


def ems_global_local_score(p: EmsParams, q, k, want_lse: bool = False, ws=None, out=None):
    """-> (s_glo, s_loc[, lse]) device f32 tensors [B,Hkv,N] ([B,Hq,N])."""
    _check_tensor(q, (p.batch, p.q_heads, p.seq_len, p.head_dim), p.torch_dtype, "q")
    _check_tensor(k, (p.batch, p.kv_heads, p.seq_len, p.head_dim), p.torch_dtype, "k")
    dev = q.device
    need = ems_workspace_bytes(p, full=False)[0]
    ws = _workspace(need, dev, ws)
    if out is None:
        s_glo = torch.empty((p.batch, p.kv_heads, p.seq_len), dtype=torch.float32, device=dev)
        s_loc = torch.empty_like(s_glo)
    else:
        s_glo, s_loc = out
    lse = torch.empty((p.batch, p.q_heads, p.seq_len), dtype=torch.float32, device=dev) if want_lse else None
    cp = p.c()
    rc = lib().ems_global_local_score(C.byref(cp), _ptr(q), _ptr(k), _ptr(s_glo), _ptr(s_loc),
                                      _ptr(lse), _ptr(ws), ws.numel(), _stream())
    if rc != EMS_OK:
        raise EmsError(rc, "ems_global_local_score")
    return (s_glo, s_loc, lse) if want_lse else (s_glo, s_loc)


def ems_attention_lse(p: EmsParams, q, k, ws=None, out=None):
    """-> lse device f32 [B,Hq,N] (natural log)."""
    _check_tensor(q, (p.batch, p.q_heads, p.seq_len, p.head_dim), p.torch_dtype, "q")
    _check_tensor(k, (p.batch, p.kv_heads, p.seq_len, p.head_dim), p.torch_dtype, "k")
    ws = _workspace(ems_workspace_bytes(p, full=False)[0], q.device, ws)
    lse = out if out is not None else torch.empty((p.batch, p.q_heads, p.seq_len),
                                                  dtype=torch.float32, device=q.device)
    cp = p.c()
    rc = lib().ems_attention_lse(C.byref(cp), _ptr(q), _ptr(k), _ptr(lse), _ptr(ws), ws.numel(),
                                 _stream())
    if rc != EMS_OK:
        raise EmsError(rc, "ems_attention_lse")
    return lse


def ems_global_local_score_from_lse(p: EmsParams, q, k, lse, ws=None, out=None):
    """-> (s_glo, s_loc) from a caller-supplied natural-log row log-sum-exp."""
    _check_tensor(q, (p.batch, p.q_heads, p.seq_len, p.head_dim), p.torch_dtype, "q")
    _check_tensor(k, (p.batch, p.kv_heads, p.seq_len, p.head_dim), p.torch_dtype, "k")
    _check_tensor(lse, (p.batch, p.q_heads, p.seq_len), torch.float32, "lse")
    dev = q.device
    ws = _workspace(ems_workspace_bytes(p, full=False)[0], dev, ws)
    if out is None:
        s_glo = torch.empty((p.batch, p.kv_heads, p.seq_len), dtype=torch.float32, device=dev)
        s_loc = torch.empty_like(s_glo)
    else:
        s_glo, s_loc = out
    cp = p.c()
    rc = lib().ems_global_local_score_from_lse(C.byref(cp), _ptr(q), _ptr(k), _ptr(lse),
                                               _ptr(s_glo), _ptr(s_loc), _ptr(ws), ws.numel(),
                                               _stream())
    if rc != EMS_OK:
        raise EmsError(rc, "ems_global_local_score_from_lse")
    return s_glo, s_loc


def ems_select(p: EmsParams, s_glo, s_loc, want_pooled: bool = False, ws=None, out=None):
    """-> (imp_idx, tbm_idx[, pooled]) device tensors."""
    shape = (p.batch, p.kv_heads, p.seq_len)
    _check_tensor(s_glo, shape, torch.float32, "s_glo")
    _check_tensor(s_loc, shape, torch.float32, "s_loc")
    dev = s_glo.device
    n_imp, n_tbm = ems_partition_sizes(p)
    need = ems_workspace_bytes(p)[1]
    ws = _workspace(need, dev, ws)
    if out is None:
        imp = torch.empty((p.batch, p.kv_heads, n_imp), dtype=torch.int32, device=dev)
        tbm = torch.empty((p.batch, p.kv_heads, n_tbm), dtype=torch.int32, device=dev)
    else:
        imp, tbm = out
    pooled = torch.empty(shape, dtype=torch.float32, device=dev) if want_pooled else None
    cp = p.c()
    rc = lib().ems_select(C.byref(cp), _ptr(s_glo), _ptr(s_loc), _ptr(pooled), _ptr(imp),
                          _ptr(tbm) if n_tbm else None, _ptr(ws), ws.numel(), _stream())
    if rc != EMS_OK:
        raise EmsError(rc, "ems_select")
    return (imp, tbm, pooled) if want_pooled else (imp, tbm)


def alloc_evict_merge_outputs(p: EmsParams, device):
    n_imp, n_tbm = ems_partition_sizes(p)
    B, H, D, Nb = p.batch, p.kv_heads, p.head_dim, p.budget
    i32, f32 = torch.int32, torch.float32
    return dict(
        k_out=torch.empty((B, H, Nb + 1, D), dtype=p.torch_dtype, device=device),
        v_out=torch.empty((B, H, Nb + 1, D), dtype=p.torch_dtype, device=device),
        kept_pos=torch.empty((B, H, Nb), dtype=i32, device=device),
        tbm_dest=torch.empty((B, H, n_tbm), dtype=i32, device=device),
        tbm_sim=torch.empty((B, H, n_tbm), dtype=f32, device=device),
        k_norm=torch.empty((B, H, n_imp + n_tbm), dtype=f32, device=device),
        slot_count=torch.empty((B, H, n_imp + 1), dtype=i32, device=device),
    )


def ems_evict_merge(p: EmsParams, k, v, imp_idx, tbm_idx, ws=None, out=None):
    """-> dict(k_out, v_out, kept_pos, tbm_dest, tbm_sim, k_norm, slot_count)."""
    shape = (p.batch, p.kv_heads, p.seq_len, p.head_dim)
    _check_tensor(k, shape, p.torch_dtype, "k")
    _check_tensor(v, shape, p.torch_dtype, "v")
    n_imp, n_tbm = ems_partition_sizes(p)
    _check_tensor(imp_idx, (p.batch, p.kv_heads, n_imp), torch.int32, "imp_idx")
    _check_tensor(tbm_idx, (p.batch, p.kv_heads, n_tbm), torch.int32, "tbm_idx")
    dev = k.device
    need = ems_workspace_bytes(p)[2]
    ws = _workspace(need, dev, ws)
    o = out if out is not None else alloc_evict_merge_outputs(p, dev)
    has = n_tbm > 0
    cp = p.c()
    rc = lib().ems_evict_merge(C.byref(cp), _ptr(k), _ptr(v), _ptr(imp_idx),
                               _ptr(tbm_idx) if has else None, _ptr(o["k_out"]), _ptr(o["v_out"]),
                               _ptr(o["kept_pos"]), _ptr(o["tbm_dest"]) if has else None,
                               _ptr(o["tbm_sim"]) if has else None, _ptr(o["k_norm"]),
                               _ptr(o["slot_count"]), _ptr(ws), ws.numel(), _stream())
    if rc != EMS_OK:
        raise EmsError(rc, "ems_evict_merge")
    return o


def ems_evict_merge_static(p: EmsParams, k, v, imp_idx, tbm_idx, out=None, k_norm: bool = True):
    """ems_evict_merge on the library's fixed scratch array: no workspace, nothing allocated by the
    call (pass `out` from alloc_evict_merge_outputs to keep the binding from allocating as well).
    With k_norm=False no key norms are returned and they live in the scratch array."""
    shape = (p.batch, p.kv_heads, p.seq_len, p.head_dim)
    _check_tensor(k, shape, p.torch_dtype, "k")
    _check_tensor(v, shape, p.torch_dtype, "v")
    n_imp, n_tbm = ems_partition_sizes(p)
    _check_tensor(imp_idx, (p.batch, p.kv_heads, n_imp), torch.int32, "imp_idx")
    _check_tensor(tbm_idx, (p.batch, p.kv_heads, n_tbm), torch.int32, "tbm_idx")
    o = dict(out) if out is not None else alloc_evict_merge_outputs(p, k.device)
    if not k_norm:
        o["k_norm"] = None
    has = n_tbm > 0
    cp = p.c()
    rc = lib().ems_evict_merge_static(C.byref(cp), _ptr(k), _ptr(v), _ptr(imp_idx),
                                      _ptr(tbm_idx) if has else None, _ptr(o["k_out"]), _ptr(o["v_out"]),
                                      _ptr(o["kept_pos"]), _ptr(o["tbm_dest"]) if has else None,
                                      _ptr(o["tbm_sim"]) if has else None, _ptr(o["k_norm"]),
                                      _ptr(o["slot_count"]), _stream())
    if rc != EMS_OK:
        raise EmsError(rc, "ems_evict_merge_static")
    return o


def ems_evict_merge_variant(p: EmsParams, similarity: int, k, v, token_weight, imp_idx, tbm_idx,
                            ws=None, out=None):
    """ems_evict_merge with the redundancy of `similarity` (EMS_SIM_*) and, when `token_weight`
    ([B, Hkv, N] f32) is given, the score-weighted merge.  Same outputs."""
    shape = (p.batch, p.kv_heads, p.seq_len, p.head_dim)
    _check_tensor(k, shape, p.torch_dtype, "k")
    _check_tensor(v, shape, p.torch_dtype, "v")
    if token_weight is not None:
        _check_tensor(token_weight, shape[:3], torch.float32, "token_weight")
    n_imp, n_tbm = ems_partition_sizes(p)
    _check_tensor(imp_idx, (p.batch, p.kv_heads, n_imp), torch.int32, "imp_idx")
    _check_tensor(tbm_idx, (p.batch, p.kv_heads, n_tbm), torch.int32, "tbm_idx")
    dev = k.device
    ws = _workspace(ems_workspace_bytes(p)[2], dev, ws)
    o = out if out is not None else alloc_evict_merge_outputs(p, dev)
    has = n_tbm > 0
    cp = p.c()
    rc = lib().ems_evict_merge_variant(
        C.byref(cp), int(similarity), _ptr(k), _ptr(v), _ptr(token_weight), _ptr(imp_idx),
        _ptr(tbm_idx) if has else None, _ptr(o["k_out"]), _ptr(o["v_out"]), _ptr(o["kept_pos"]),
        _ptr(o["tbm_dest"]) if has else None, _ptr(o["tbm_sim"]) if has else None,
        _ptr(o["k_norm"]), _ptr(o["slot_count"]), _ptr(ws), ws.numel(), _stream())
    if rc != EMS_OK:
        raise EmsError(rc, "ems_evict_merge_variant")
    return o


def ems_expand(p: EmsParams, merged: dict, tbm_idx, out=None):
    """Expand the compact cache `merged` (the dict ems_evict_merge returned) back to one
    key / value per kept token -> (k_exp, v_exp, pos_exp)."""
    n_imp, n_tbm = ems_partition_sizes(p)
    n_exp = n_imp + n_tbm + p.window
    dev = merged["k_out"].device
    _check_tensor(merged["k_out"], (p.batch, p.kv_heads, p.budget + 1, p.head_dim), p.torch_dtype, "k_cache")
    _check_tensor(merged["v_out"], (p.batch, p.kv_heads, p.budget + 1, p.head_dim), p.torch_dtype, "v_cache")
    _check_tensor(merged["kept_pos"], (p.batch, p.kv_heads, p.budget), torch.int32, "kept_pos")
    _check_tensor(merged["k_norm"], (p.batch, p.kv_heads, n_imp + n_tbm), torch.float32, "k_norm")
    _check_tensor(merged["tbm_dest"], (p.batch, p.kv_heads, n_tbm), torch.int32, "tbm_dest")
    _check_tensor(tbm_idx, (p.batch, p.kv_heads, n_tbm), torch.int32, "tbm_idx")
    if out is None:
        k_exp = torch.empty((p.batch, p.kv_heads, n_exp, p.head_dim), dtype=p.torch_dtype, device=dev)
        v_exp = torch.empty_like(k_exp)
        pos = torch.empty((p.batch, p.kv_heads, n_exp), dtype=torch.int32, device=dev)
    else:
        k_exp, v_exp, pos = out
    has = n_tbm > 0
    cp = p.c()
    rc = lib().ems_expand(C.byref(cp), _ptr(merged["k_out"]), _ptr(merged["v_out"]),
                          _ptr(merged["kept_pos"]), _ptr(tbm_idx) if has else None,
                          _ptr(merged["tbm_dest"]) if has else None, _ptr(merged["k_norm"]),
                          _ptr(k_exp), _ptr(v_exp), _ptr(pos), _stream())
    if rc != EMS_OK:
        raise EmsError(rc, "ems_expand")
    return k_exp, v_exp, pos


def ems_decode_workspace_bytes(p: EmsParams) -> int:
    n = C.c_size_t(0)
    cp = p.c()
    rc = lib().ems_decode_workspace_bytes(C.byref(cp), C.byref(n))
    if rc != EMS_OK:
        raise EmsError(rc, "ems_decode_workspace_bytes")
    return int(n.value)


class DecodeState:
    """Device tensors of the decode-time state (see ems_decode_state in include/ems.h)."""

    def __init__(self, p: EmsParams, k_cache, v_cache):
        n_imp, n_tbm = ems_partition_sizes(p)
        B, H, Nb = p.batch, p.kv_heads, p.budget
        T = n_imp + n_tbm + p.window
        dev = k_cache.device
        _check_tensor(k_cache, (B, H, Nb + 1, p.head_dim), p.torch_dtype, "k_cache")
        _check_tensor(v_cache, (B, H, Nb + 1, p.head_dim), p.torch_dtype, "v_cache")
        self.n_tokens = T
        self.k_cache, self.v_cache = k_cache, v_cache
        # one slab for the nine small arrays: they are all touched by every step, and sitting in
        # one allocation keeps them on as few pages as possible
        shapes = [("row_norm", (B, H, Nb), torch.float32), ("entry_count", (B, H, n_imp), torch.int32),
                  ("entry_tok", (B, H, n_imp), torch.int32), ("tok_pos", (B, H, T), torch.int32),
                  ("tok_row", (B, H, T), torch.int32), ("tok_norm", (B, H, T), torch.float32),
                  ("tok_glo", (B, H, T), torch.float32), ("tok_past", (B, H, T), torch.float32),
                  ("tok_cur", (B, H, T), torch.float32), ("step_count", (1,), torch.int32)]
        sizes = [(4 * int(torch.Size(shape).numel()) + 255) // 256 * 256 for _, shape, _ in shapes]
        self.slab = torch.zeros(sum(sizes), dtype=torch.uint8, device=dev)
        off = 0
        for (name, shape, dtype), size in zip(shapes, sizes):
            n = int(torch.Size(shape).numel())
            setattr(self, name, self.slab[off:off + 4 * n].view(dtype).view(shape))
            off += size
        self.tok_pos.fill_(-1)
        self.tok_row.fill_(-1)

    def c(self) -> ems_decode_state:
        if getattr(self, "_c", None) is None:                # the tensors never move
            self._c = ems_decode_state(*[getattr(self, name).data_ptr() for name in STATE_FIELDS])
        return self._c


def ems_decode_init(p: EmsParams, merged: dict, tbm_idx, s_glo, s_loc, state=None) -> DecodeState:
    """State for the generation from ems_evict_merge's outputs (`merged`; its k_out / v_out
    become the live cache and are updated in place by ems_decode_step)."""
    n_imp, n_tbm = ems_partition_sizes(p)
    shape = (p.batch, p.kv_heads, p.seq_len)
    _check_tensor(s_glo, shape, torch.float32, "s_glo")
    _check_tensor(s_loc, shape, torch.float32, "s_loc")
    _check_tensor(merged["kept_pos"], (p.batch, p.kv_heads, p.budget), torch.int32, "kept_pos")
    _check_tensor(merged["k_norm"], (p.batch, p.kv_heads, n_imp + n_tbm), torch.float32, "k_norm")
    _check_tensor(merged["tbm_dest"], (p.batch, p.kv_heads, n_tbm), torch.int32, "tbm_dest")
    _check_tensor(merged["slot_count"], (p.batch, p.kv_heads, n_imp + 1), torch.int32, "slot_count")
    _check_tensor(tbm_idx, (p.batch, p.kv_heads, n_tbm), torch.int32, "tbm_idx")
    st = state if state is not None else DecodeState(p, merged["k_out"], merged["v_out"])
    has = n_tbm > 0
    cp, cs = p.c(), st.c()
    rc = lib().ems_decode_init(C.byref(cp), _ptr(s_glo), _ptr(s_loc), _ptr(merged["kept_pos"]),
                               _ptr(tbm_idx) if has else None, _ptr(merged["tbm_dest"]) if has else None,
                               _ptr(merged["k_norm"]), _ptr(merged["slot_count"]), C.byref(cs), _stream())
    if rc != EMS_OK:
        raise EmsError(rc, "ems_decode_init")
    return st


def ems_decode_step(p: EmsParams, st: DecodeState, step: int, q_new, k_new, v_new, want_attn=False,
                    ws=None, out=None):
    """One generated token -> dict(decision [B,Hkv,2], sim [B,Hkv], attn [B,Hq,T+1] or None)."""
    _check_tensor(q_new, (p.batch, p.q_heads, p.head_dim), p.torch_dtype, "q_new")
    _check_tensor(k_new, (p.batch, p.kv_heads, p.head_dim), p.torch_dtype, "k_new")
    _check_tensor(v_new, (p.batch, p.kv_heads, p.head_dim), p.torch_dtype, "v_new")
    dev = q_new.device
    if ws is None:
        ws = _workspace(ems_decode_workspace_bytes(p), dev)
    if out is None:
        out = dict(decision=torch.empty((p.batch, p.kv_heads, 2), dtype=torch.int32, device=dev),
                   sim=torch.empty((p.batch, p.kv_heads), dtype=torch.float32, device=dev),
                   attn=torch.empty((p.batch, p.q_heads, st.n_tokens + 1), dtype=torch.float32, device=dev)
                   if want_attn else None)
    cp, cs = p.c(), st.c()
    rc = lib().ems_decode_step(C.byref(cp), C.byref(cs), int(step), _ptr(q_new), _ptr(k_new), _ptr(v_new),
                               _ptr(out.get("attn")), _ptr(out["decision"]), _ptr(out["sim"]),
                               _ptr(ws), ws.numel(), _stream())
    if rc != EMS_OK:
        raise EmsError(rc, "ems_decode_step")
    return out


def ems_sparsity_rate(p: EmsParams, zeta: float, s_glo, s_loc):
    """Eq. 3 -> (rate [B,Hkv] f32, n_k [B,Hkv] i32)."""
    shape = (p.batch, p.kv_heads, p.seq_len)
    _check_tensor(s_glo, shape, torch.float32, "s_glo")
    _check_tensor(s_loc, shape, torch.float32, "s_loc")
    rate = torch.empty(shape[:2], dtype=torch.float32, device=s_glo.device)
    n_k = torch.empty(shape[:2], dtype=torch.int32, device=s_glo.device)
    cp = p.c()
    rc = lib().ems_sparsity_rate(C.byref(cp), float(zeta), _ptr(s_glo), _ptr(s_loc), _ptr(rate), _ptr(n_k),
                                 _stream())
    if rc != EMS_OK:
        raise EmsError(rc, "ems_sparsity_rate")
    return rate, n_k


def ems_redundancy_rate(p: EmsParams, k, v):
    """Eq. 4 -> (rate [B,Hkv] f32, best [B,Hkv,N] f32)."""
    shape = (p.batch, p.kv_heads, p.seq_len, p.head_dim)
    _check_tensor(k, shape, p.torch_dtype, "k")
    _check_tensor(v, shape, p.torch_dtype, "v")
    rate = torch.empty(shape[:2], dtype=torch.float32, device=k.device)
    best = torch.empty(shape[:3], dtype=torch.float32, device=k.device)
    cp = p.c()
    rc = lib().ems_redundancy_rate(C.byref(cp), _ptr(k), _ptr(v), _ptr(rate), _ptr(best), _stream())
    if rc != EMS_OK:
        raise EmsError(rc, "ems_redundancy_rate")
    return rate, best
