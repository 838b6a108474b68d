"""ctypes front end of the CPU oracle (oracle/ems_ref.c).

TEST INFRASTRUCTURE ONLY: the tests, the smoke check and the benchmark's cpu_baseline leg
may import this module; the HIP package never does.  Argument marshalling only -- all the
arithmetic is in the C file.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ems_ref.c")
_LIB = os.path.join(_HERE, "libems_ref.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (a second or two)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-march=native",
               "-fno-fast-math", "-o", _LIB + ".tmp", _SRC, "-lm"]
        subprocess.run(cmd, check=True, cwd=_HERE)
        os.replace(_LIB + ".tmp", _LIB)
    return _LIB


class _Params(C.Structure):
    _fields_ = [("batch", C.c_int32), ("q_heads", C.c_int32), ("kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("seq_len", C.c_int32), ("window", C.c_int32),
                ("budget", C.c_int32), ("pool_kernel", C.c_int32),
                ("merge_ratio", C.c_double), ("tau", C.c_double),
                ("softmax_scale", C.c_double)]


@dataclass
class RefParams:
    batch: int
    q_heads: int
    kv_heads: int
    head_dim: int
    seq_len: int
    window: int
    budget: int = 0
    merge_ratio: float = 0.0
    tau: float = 0.6
    pool_kernel: int = 1
    softmax_scale: float = 0.0

    def c(self) -> _Params:
        return _Params(self.batch, self.q_heads, self.kv_heads, self.head_dim, self.seq_len,
                       self.window, self.budget, self.pool_kernel, float(self.merge_ratio),
                       float(self.tau), float(self.softmax_scale))


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.ems_ref_threads.restype = C.c_int
    return _lib


def _ptr(a, ctype):
    return None if a is None else a.ctypes.data_as(C.POINTER(ctype))


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _check(rc, what):
    if rc != 0:
        raise ValueError(f"oracle {what}: invalid arguments (rc={rc})")


def threads() -> int:
    return int(lib().ems_ref_threads())


def sizes(p: RefParams):
    n_imp, n_tbm = C.c_int32(0), C.c_int32(0)
    cp = p.c()
    _check(lib().ems_ref_sizes(C.byref(cp), C.byref(n_imp), C.byref(n_tbm)), "sizes")
    return int(n_imp.value), int(n_tbm.value)


def score(p: RefParams, q, k, want_lse: bool = False):
    q, k = _f32(q), _f32(k)
    assert q.shape == (p.batch, p.q_heads, p.seq_len, p.head_dim), q.shape
    assert k.shape == (p.batch, p.kv_heads, p.seq_len, p.head_dim), k.shape
    s_glo = np.empty((p.batch, p.kv_heads, p.seq_len), np.float64)
    s_loc = np.empty_like(s_glo)
    lse = np.empty((p.batch, p.q_heads, p.seq_len), np.float64) if want_lse else None
    cp = p.c()
    _check(lib().ems_ref_score(C.byref(cp), _ptr(q, C.c_float), _ptr(k, C.c_float),
                               _ptr(s_glo, C.c_double), _ptr(s_loc, C.c_double),
                               _ptr(lse, C.c_double)), "score")
    return (s_glo, s_loc, lse) if want_lse else (s_glo, s_loc)


def combine_pool(p: RefParams, s_glo, s_loc):
    s_glo, s_loc = _f64(s_glo), _f64(s_loc)
    shape = (p.batch, p.kv_heads, p.seq_len)
    assert s_glo.shape == shape and s_loc.shape == shape
    out = np.empty(shape, np.float64)
    cp = p.c()
    _check(lib().ems_ref_combine_pool(C.byref(cp), _ptr(s_glo, C.c_double),
                                      _ptr(s_loc, C.c_double), _ptr(out, C.c_double)),
           "combine_pool")
    return out


def partition(p: RefParams, s_pooled):
    s_pooled = _f64(s_pooled)
    assert s_pooled.shape == (p.batch, p.kv_heads, p.seq_len)
    n_imp, n_tbm = sizes(p)
    imp = np.empty((p.batch, p.kv_heads, n_imp), np.int32)
    tbm = np.empty((p.batch, p.kv_heads, n_tbm), np.int32)
    cp = p.c()
    _check(lib().ems_ref_partition(C.byref(cp), _ptr(s_pooled, C.c_double),
                                   _ptr(imp, C.c_int32), _ptr(tbm, C.c_int32)), "partition")
    return imp, tbm


def select(p: RefParams, s_glo, s_loc):
    s_glo, s_loc = _f64(s_glo), _f64(s_loc)
    shape = (p.batch, p.kv_heads, p.seq_len)
    assert s_glo.shape == shape and s_loc.shape == shape
    n_imp, n_tbm = sizes(p)
    pooled = np.empty(shape, np.float64)
    imp = np.empty((p.batch, p.kv_heads, n_imp), np.int32)
    tbm = np.empty((p.batch, p.kv_heads, n_tbm), np.int32)
    cp = p.c()
    _check(lib().ems_ref_select(C.byref(cp), _ptr(s_glo, C.c_double), _ptr(s_loc, C.c_double),
                                _ptr(pooled, C.c_double), _ptr(imp, C.c_int32),
                                _ptr(tbm, C.c_int32)), "select")
    return pooled, imp, tbm


def dest(p: RefParams, k, imp_idx, tbm_idx):
    k, imp_idx, tbm_idx = _f32(k), _i32(imp_idx), _i32(tbm_idx)
    n_imp, n_tbm = sizes(p)
    assert k.shape == (p.batch, p.kv_heads, p.seq_len, p.head_dim)
    assert imp_idx.shape == (p.batch, p.kv_heads, n_imp)
    assert tbm_idx.shape == (p.batch, p.kv_heads, n_tbm)
    d = np.empty((p.batch, p.kv_heads, n_tbm), np.int32)
    sim = np.empty((p.batch, p.kv_heads, n_tbm), np.float64)
    norm = np.empty((p.batch, p.kv_heads, n_imp + n_tbm), np.float64)
    cp = p.c()
    _check(lib().ems_ref_dest(C.byref(cp), _ptr(k, C.c_float), _ptr(imp_idx, C.c_int32),
                              _ptr(tbm_idx, C.c_int32), _ptr(d, C.c_int32),
                              _ptr(sim, C.c_double), _ptr(norm, C.c_double)), "dest")
    return d, sim, norm


def merge(p: RefParams, k, v, imp_idx, tbm_idx, tbm_dest):
    k, v = _f32(k), _f32(v)
    imp_idx, tbm_idx, tbm_dest = _i32(imp_idx), _i32(tbm_idx), _i32(tbm_dest)
    n_imp, n_tbm = sizes(p)
    shape = (p.batch, p.kv_heads, p.seq_len, p.head_dim)
    assert k.shape == shape and v.shape == shape
    assert imp_idx.shape == (p.batch, p.kv_heads, n_imp)
    assert tbm_idx.shape == (p.batch, p.kv_heads, n_tbm)
    assert tbm_dest.shape == (p.batch, p.kv_heads, n_tbm)
    k_out = np.empty((p.batch, p.kv_heads, p.budget + 1, p.head_dim), np.float64)
    v_out = np.empty_like(k_out)
    kept = np.empty((p.batch, p.kv_heads, p.budget), np.int32)
    cnt = np.empty((p.batch, p.kv_heads, n_imp + 1), np.int32)
    cp = p.c()
    _check(lib().ems_ref_merge(C.byref(cp), _ptr(k, C.c_float), _ptr(v, C.c_float),
                               _ptr(imp_idx, C.c_int32), _ptr(tbm_idx, C.c_int32),
                               _ptr(tbm_dest, C.c_int32), _ptr(k_out, C.c_double),
                               _ptr(v_out, C.c_double), _ptr(kept, C.c_int32),
                               _ptr(cnt, C.c_int32)), "merge")
    return k_out, v_out, kept, cnt


def evict_merge(p: RefParams, k, v, imp_idx, tbm_idx):
    k, v = _f32(k), _f32(v)
    imp_idx, tbm_idx = _i32(imp_idx), _i32(tbm_idx)
    n_imp, n_tbm = sizes(p)
    shape = (p.batch, p.kv_heads, p.seq_len, p.head_dim)
    assert k.shape == shape and v.shape == shape
    assert imp_idx.shape == (p.batch, p.kv_heads, n_imp)
    assert tbm_idx.shape == (p.batch, p.kv_heads, n_tbm)
    k_out = np.empty((p.batch, p.kv_heads, p.budget + 1, p.head_dim), np.float64)
    v_out = np.empty_like(k_out)
    kept = np.empty((p.batch, p.kv_heads, p.budget), np.int32)
    d = np.empty((p.batch, p.kv_heads, n_tbm), np.int32)
    sim = np.empty((p.batch, p.kv_heads, n_tbm), np.float64)
    norm = np.empty((p.batch, p.kv_heads, n_imp + n_tbm), np.float64)
    cnt = np.empty((p.batch, p.kv_heads, n_imp + 1), np.int32)
    cp = p.c()
    _check(lib().ems_ref_evict_merge(C.byref(cp), _ptr(k, C.c_float), _ptr(v, C.c_float),
                                     _ptr(imp_idx, C.c_int32), _ptr(tbm_idx, C.c_int32),
                                     _ptr(k_out, C.c_double), _ptr(v_out, C.c_double),
                                     _ptr(kept, C.c_int32), _ptr(d, C.c_int32),
                                     _ptr(sim, C.c_double), _ptr(norm, C.c_double),
                                     _ptr(cnt, C.c_int32)), "evict_merge")
    return dict(k_out=k_out, v_out=v_out, kept_pos=kept, tbm_dest=d, tbm_sim=sim,
                k_norm=norm, slot_count=cnt)


def dest_sim(p: RefParams, similarity: int, k, v, imp_idx, tbm_idx):
    k, v, imp_idx, tbm_idx = _f32(k), _f32(v), _i32(imp_idx), _i32(tbm_idx)
    n_imp, n_tbm = sizes(p)
    shape = (p.batch, p.kv_heads, p.seq_len, p.head_dim)
    assert k.shape == shape and v.shape == shape
    assert imp_idx.shape == (p.batch, p.kv_heads, n_imp)
    assert tbm_idx.shape == (p.batch, p.kv_heads, n_tbm)
    d = np.empty((p.batch, p.kv_heads, n_tbm), np.int32)
    sim = np.empty((p.batch, p.kv_heads, n_tbm), np.float64)
    norm = np.empty((p.batch, p.kv_heads, n_imp + n_tbm), np.float64)
    cp = p.c()
    _check(lib().ems_ref_dest_sim(C.byref(cp), C.c_int(int(similarity)), _ptr(k, C.c_float),
                                  _ptr(v, C.c_float), _ptr(imp_idx, C.c_int32),
                                  _ptr(tbm_idx, C.c_int32), _ptr(d, C.c_int32),
                                  _ptr(sim, C.c_double), _ptr(norm, C.c_double)), "dest_sim")
    return d, sim, norm


def merge_weighted(p: RefParams, k, v, weight, imp_idx, tbm_idx, tbm_dest):
    k, v, weight = _f32(k), _f32(v), _f64(weight)
    imp_idx, tbm_idx, tbm_dest = _i32(imp_idx), _i32(tbm_idx), _i32(tbm_dest)
    n_imp, n_tbm = sizes(p)
    shape = (p.batch, p.kv_heads, p.seq_len, p.head_dim)
    assert k.shape == shape and v.shape == shape and weight.shape == shape[:3]
    assert imp_idx.shape == (p.batch, p.kv_heads, n_imp)
    assert tbm_idx.shape == (p.batch, p.kv_heads, n_tbm)
    assert tbm_dest.shape == (p.batch, p.kv_heads, n_tbm)
    k_out = np.empty((p.batch, p.kv_heads, p.budget + 1, p.head_dim), np.float64)
    v_out = np.empty_like(k_out)
    kept = np.empty((p.batch, p.kv_heads, p.budget), np.int32)
    cnt = np.empty((p.batch, p.kv_heads, n_imp + 1), np.int32)
    cp = p.c()
    _check(lib().ems_ref_merge_weighted(C.byref(cp), _ptr(k, C.c_float), _ptr(v, C.c_float),
                                        _ptr(weight, C.c_double), _ptr(imp_idx, C.c_int32),
                                        _ptr(tbm_idx, C.c_int32), _ptr(tbm_dest, C.c_int32),
                                        _ptr(k_out, C.c_double), _ptr(v_out, C.c_double),
                                        _ptr(kept, C.c_int32), _ptr(cnt, C.c_int32)),
           "merge_weighted")
    return k_out, v_out, kept, cnt


def sparsity(p: RefParams, zeta: float, s_glo, s_loc):
    s_glo, s_loc = _f64(s_glo), _f64(s_loc)
    shape = (p.batch, p.kv_heads, p.seq_len)
    assert s_glo.shape == shape and s_loc.shape == shape
    out = np.empty(shape[:2], np.float64)
    nk = np.empty(shape[:2], np.int32)
    cp = p.c()
    _check(lib().ems_ref_sparsity(C.byref(cp), C.c_double(zeta), _ptr(s_glo, C.c_double),
                                  _ptr(s_loc, C.c_double), _ptr(out, C.c_double), _ptr(nk, C.c_int32)),
           "sparsity")
    return out, nk


def redundancy(p: RefParams, k, v):
    k, v = _f32(k), _f32(v)
    shape = (p.batch, p.kv_heads, p.seq_len, p.head_dim)
    assert k.shape == shape and v.shape == shape
    r = np.empty(shape[:2], np.float64)
    best = np.empty(shape[:3], np.float64)
    cp = p.c()
    _check(lib().ems_ref_redundancy(C.byref(cp), _ptr(k, C.c_float), _ptr(v, C.c_float),
                                    _ptr(r, C.c_double), _ptr(best, C.c_double)), "redundancy")
    return r, best


def redundancy_at(p: RefParams, k, v, tokens):
    k, v, tokens = _f32(k), _f32(v), _i32(tokens)
    shape = (p.batch, p.kv_heads, p.seq_len, p.head_dim)
    assert k.shape == shape and v.shape == shape and tokens.ndim == 1
    best = np.empty((p.batch, p.kv_heads, len(tokens)), np.float64)
    cp = p.c()
    _check(lib().ems_ref_redundancy_at(C.byref(cp), _ptr(k, C.c_float), _ptr(v, C.c_float),
                                       _ptr(tokens, C.c_int32), C.c_int32(len(tokens)),
                                       _ptr(best, C.c_double)), "redundancy_at")
    return best


def expand(p: RefParams, k_cache, v_cache, kept_pos, tbm_idx, tbm_dest, k_norm):
    k_cache, v_cache, k_norm = _f64(k_cache), _f64(v_cache), _f64(k_norm)
    kept_pos, tbm_idx, tbm_dest = _i32(kept_pos), _i32(tbm_idx), _i32(tbm_dest)
    n_imp, n_tbm = sizes(p)
    B, H, D, E = p.batch, p.kv_heads, p.head_dim, n_imp + n_tbm + p.window
    assert k_cache.shape == (B, H, p.budget + 1, D) and v_cache.shape == k_cache.shape
    assert kept_pos.shape == (B, H, p.budget) and k_norm.shape == (B, H, n_imp + n_tbm)
    assert tbm_idx.shape == (B, H, n_tbm) and tbm_dest.shape == (B, H, n_tbm)
    k_exp = np.empty((B, H, E, D), np.float64)
    v_exp = np.empty_like(k_exp)
    pos = np.empty((B, H, E), np.int32)
    cp = p.c()
    _check(lib().ems_ref_expand(C.byref(cp), _ptr(k_cache, C.c_double), _ptr(v_cache, C.c_double),
                                _ptr(kept_pos, C.c_int32), _ptr(tbm_idx, C.c_int32),
                                _ptr(tbm_dest, C.c_int32), _ptr(k_norm, C.c_double),
                                _ptr(k_exp, C.c_double), _ptr(v_exp, C.c_double),
                                _ptr(pos, C.c_int32)), "expand")
    return k_exp, v_exp, pos
