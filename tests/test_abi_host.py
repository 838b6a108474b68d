"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol
the header declares, sizes follow Sec. 4.2, and argument errors are caught before launch."""
import ctypes as C
import os
import re

import pytest

from paper_2412_08521_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        from paper_2412_08521_amd import build
        build.build()
    return B.lib()


def test_exports_match_header(lib):
    text = "".join(open(os.path.join(ROOT, "include", h)).read() for h in sorted(os.listdir(os.path.join(ROOT, "include"))))
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(ems_[a-z_]+)\s*\(", text))
    assert declared == set(B.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name
    assert B.ems_version() >= 100
    assert B.strerror(0) == "ok" and "argument" in B.strerror(-1)


def test_struct_layout_matches_header():
    assert C.sizeof(B.ems_params) == 12 * 4
    assert [n for n, _ in B.ems_params._fields_] == [
        "batch", "q_heads", "kv_heads", "head_dim", "seq_len", "window", "budget",
        "merge_ratio", "tau", "pool_kernel", "softmax_scale", "dtype"]


@pytest.mark.parametrize("n,w,nb,r,exp", [(4096, 32, 256, 0.5, (224, 128)),
                                          (1024, 32, 64, 0.5, (32, 32)),
                                          (131072, 64, 2048, 0.5, (1984, 1024)),
                                          (300, 10, 290, 3.0, (280, 10)),
                                          (100, 10, 20, 0.0, (10, 0))])
def test_partition_sizes(lib, n, w, nb, r, exp):
    p = B.EmsParams(1, 8, 2, 128, n, w, nb, merge_ratio=r)
    assert B.ems_partition_sizes(p) == exp


def test_workspace_sizes(lib):
    p = B.EmsParams(4, 32, 8, 128, 32768, 64, 128)
    s, t, u = B.ems_workspace_bytes(p)
    assert s >= 4 * 32 * 32768 * 4 and s % 256 == 0
    assert t >= 4 * 8 * 32768 * 4 and u >= 4 * 8 * 128 * 4


def _bad(**kw):
    base = dict(batch=1, q_heads=4, kv_heads=2, head_dim=128, seq_len=512, window=16, budget=64)
    base.update(kw)
    return B.EmsParams(**base)


@pytest.mark.parametrize("p,code", [
    (_bad(q_heads=3), B.EMS_ERR_INVALID_ARG), (_bad(window=0), B.EMS_ERR_INVALID_ARG),
    (_bad(window=513), B.EMS_ERR_INVALID_ARG), (_bad(seq_len=0), B.EMS_ERR_INVALID_ARG),
    (_bad(dtype=7), B.EMS_ERR_INVALID_ARG), (_bad(head_dim=96), B.EMS_ERR_UNSUPPORTED),
    (_bad(batch=0), B.EMS_ERR_INVALID_ARG), (_bad(softmax_scale=float("nan")), B.EMS_ERR_INVALID_ARG)])
def test_score_argument_errors(lib, p, code):
    cp = p.c()
    dummy = C.c_void_p(256)
    rc = lib.ems_global_local_score(C.byref(cp), dummy, dummy, dummy, dummy, None, dummy, 1 << 40, None)
    assert rc == code


@pytest.mark.parametrize("p", [_bad(budget=16), _bad(budget=513), _bad(pool_kernel=4),
                               _bad(pool_kernel=0), _bad(merge_ratio=-0.5),
                               _bad(merge_ratio=float("nan")), _bad(tau=float("nan"))])
def test_select_and_merge_argument_errors(lib, p):
    cp = p.c()
    dummy = C.c_void_p(256)
    assert lib.ems_select(C.byref(cp), dummy, dummy, None, dummy, dummy, dummy, 1 << 40, None) \
        == B.EMS_ERR_INVALID_ARG
    assert lib.ems_evict_merge(C.byref(cp), *([dummy] * 12), 1 << 40, None) == B.EMS_ERR_INVALID_ARG
    with pytest.raises(B.EmsError):
        B.ems_partition_sizes(p)


def test_null_pointers_and_workspace_errors(lib):
    p = _bad()
    cp = p.c()
    d = C.c_void_p(256)
    assert lib.ems_global_local_score(None, d, d, d, d, None, d, 1 << 40, None) == B.EMS_ERR_INVALID_ARG
    assert lib.ems_global_local_score(C.byref(cp), None, d, d, d, None, d, 1 << 40, None) == B.EMS_ERR_INVALID_ARG
    assert lib.ems_global_local_score(C.byref(cp), d, d, d, None, None, d, 1 << 40, None) == B.EMS_ERR_INVALID_ARG
    assert lib.ems_global_local_score(C.byref(cp), d, d, d, d, None, None, 1 << 40, None) == B.EMS_ERR_WORKSPACE
    assert lib.ems_global_local_score(C.byref(cp), d, d, d, d, None, d, 16, None) == B.EMS_ERR_WORKSPACE
    assert lib.ems_global_local_score(C.byref(cp), d, d, d, d, None, C.c_void_p(260), 1 << 40, None) == B.EMS_ERR_WORKSPACE
    assert lib.ems_select(C.byref(cp), d, d, None, None, d, d, 1 << 40, None) == B.EMS_ERR_INVALID_ARG
    assert lib.ems_select(C.byref(cp), d, d, None, d, None, d, 1 << 40, None) == B.EMS_ERR_INVALID_ARG
    assert lib.ems_select(C.byref(cp), d, d, None, d, d, d, 8, None) == B.EMS_ERR_WORKSPACE
    args = [d] * 12
    args[3] = None     # tbm_idx missing while N_tbm > 0
    assert lib.ems_evict_merge(C.byref(cp), *args, 1 << 40, None) == B.EMS_ERR_INVALID_ARG
    assert lib.ems_evict_merge(C.byref(cp), *([d] * 12), 8, None) == B.EMS_ERR_WORKSPACE
    # the allocation-free entry point: same argument checks, and a size limit instead of `ws`
    assert lib.ems_evict_merge_static(C.byref(cp), *args, None) == B.EMS_ERR_INVALID_ARG
    assert lib.ems_evict_merge_static(None, *([d] * 12), None) == B.EMS_ERR_INVALID_ARG
    big = B.EmsParams(64, 32, 32, 128, 1 << 20, 32, 1 << 19, merge_ratio=0.5)
    assert B.ems_workspace_bytes(big)[2] > 8 << 20
    cbig = big.c()
    assert lib.ems_evict_merge_static(C.byref(cbig), *([d] * 12), None) == B.EMS_ERR_WORKSPACE
    assert lib.ems_workspace_bytes(None, None, None, None) == B.EMS_ERR_INVALID_ARG
    assert lib.ems_expand(C.byref(cp), d, d, d, d, d, None, d, d, d, None) == B.EMS_ERR_INVALID_ARG
    assert lib.ems_expand(C.byref(cp), d, d, d, None, d, d, d, d, d, None) == B.EMS_ERR_INVALID_ARG
    args = [d] * 13 + [1 << 20, None]
    assert lib.ems_evict_merge_variant(C.byref(cp), 3, *args) == B.EMS_ERR_INVALID_ARG
    assert lib.ems_evict_merge_variant(C.byref(cp), -1, *args) == B.EMS_ERR_INVALID_ARG
    args[0] = None
    assert lib.ems_evict_merge_variant(C.byref(cp), 2, *args) == B.EMS_ERR_INVALID_ARG
    bad = _bad(budget=16).c()
    assert lib.ems_expand(C.byref(bad), d, d, d, d, d, d, d, d, d, None) == B.EMS_ERR_INVALID_ARG


def test_decode_argument_errors(lib):
    p = _bad()
    cp = p.c()
    d = C.c_void_p(256)
    st = B.ems_decode_state(*[256] * len(B.STATE_FIELDS))
    assert C.sizeof(B.ems_decode_state) == 12 * C.sizeof(C.c_void_p)
    need = B.ems_decode_workspace_bytes(p)
    assert need >= 4 * (2 * 2 * 64 + 2 * 48) and need % 256 == 0
    # null state member, null token, negative step, workspace too small
    hole = B.ems_decode_state(*([256] * 5 + [0] + [256] * 6))
    assert lib.ems_decode_step(C.byref(cp), C.byref(hole), 0, d, d, d, None, None, None, d, need, None) == B.EMS_ERR_INVALID_ARG
    assert lib.ems_decode_step(C.byref(cp), C.byref(st), 0, None, d, d, None, None, None, d, need, None) == B.EMS_ERR_INVALID_ARG
    assert lib.ems_decode_step(C.byref(cp), C.byref(st), -2, d, d, d, None, None, None, d, need, None) == B.EMS_ERR_INVALID_ARG
    assert lib.ems_decode_step(C.byref(cp), C.byref(st), 0, d, d, d, None, None, None, d, need - 1, None) == B.EMS_ERR_WORKSPACE
    assert lib.ems_decode_step(C.byref(cp), C.byref(st), 0, d, d, d, None, None, None, C.c_void_p(8), need, None) == B.EMS_ERR_WORKSPACE
    assert lib.ems_decode_init(C.byref(cp), d, d, d, d, d, d, d, None, None) == B.EMS_ERR_INVALID_ARG
    assert lib.ems_decode_init(C.byref(cp), None, d, d, d, d, d, d, C.byref(st), None) == B.EMS_ERR_INVALID_ARG
    # group sizes other than 1, 2, 4, 8 are not built
    odd = _bad(q_heads=6).c()
    assert lib.ems_decode_step(C.byref(odd), C.byref(st), 0, d, d, d, None, None, None, d, 1 << 30, None) == B.EMS_ERR_UNSUPPORTED
    n = C.c_size_t(0)
    assert lib.ems_decode_workspace_bytes(C.byref(odd), C.byref(n)) == B.EMS_ERR_UNSUPPORTED


def test_stats_argument_errors(lib):
    cp = _bad().c()
    d = C.c_void_p(256)
    for zeta in (0.0, -0.1, 1.5, float("nan")):
        assert lib.ems_sparsity_rate(C.byref(cp), zeta, d, d, d, None, None) == B.EMS_ERR_INVALID_ARG
    assert lib.ems_sparsity_rate(C.byref(cp), 0.9, None, d, d, None, None) == B.EMS_ERR_INVALID_ARG
    assert lib.ems_sparsity_rate(C.byref(cp), 0.9, d, d, None, None, None) == B.EMS_ERR_INVALID_ARG
    assert lib.ems_redundancy_rate(C.byref(cp), d, d, d, None, None) == B.EMS_ERR_INVALID_ARG
    assert lib.ems_redundancy_rate(C.byref(cp), None, d, d, d, None) == B.EMS_ERR_INVALID_ARG
    odd = _bad(head_dim=96).c()
    assert lib.ems_redundancy_rate(C.byref(odd), d, d, d, d, None) == B.EMS_ERR_UNSUPPORTED


def test_header_is_plain_c_and_links(lib, tmp_path):
    """include/ems.h compiles as C99 and a C program can call the host-only entry points."""
    import subprocess
    src = tmp_path / "use_ems.c"
    src.write_text(r'''
#include "ems.h"
#include <stdio.h>
int main(void) {
    ems_params p = {1, 8, 2, 128, 4096, 32, 256, 0.5f, 0.6f, 7, 0.0f, EMS_BF16};
    int32_t n_imp = 0, n_tbm = 0;
    size_t a = 0, b = 0, c = 0, d = 0;
    if (ems_partition_sizes(&p, &n_imp, &n_tbm) != EMS_OK) return 1;
    if (ems_workspace_bytes(&p, &a, &b, &c) != EMS_OK) return 2;
    if (ems_decode_workspace_bytes(&p, &d) != EMS_OK) return 3;
    if (ems_global_local_score(&p, 0, 0, 0, 0, 0, 0, 0, 0) != EMS_ERR_INVALID_ARG) return 4;
    printf("%d %d %d %zu %zu %zu %zu %s\n", ems_version(), (int)n_imp, (int)n_tbm, a, b, c, d, ems_strerror(EMS_ERR_WORKSPACE));
    return 0;
}
''')
    exe = tmp_path / "use_ems"
    libdir = os.path.dirname(B.LIB_PATH)
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"), str(src),
                    "-o", str(exe), "-L", libdir, "-lems_hip", f"-Wl,-rpath,{libdir}"], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()
    assert int(out[0]) >= 200 and (int(out[1]), int(out[2])) == (224, 128)
    assert all(int(x) % 256 == 0 for x in out[3:7]) and "workspace" in " ".join(out[7:])


def test_probe_library_is_separate_and_checks_arguments(lib):
    """The benchmark's measurement kernels live in a library of their own."""
    from paper_2412_08521_amd import bench_probe
    assert not hasattr(lib, "ems_probe_mfma") and not hasattr(lib, "ems_probe_copy")
    pl = bench_probe.lib()
    d = C.c_void_p(256)
    assert pl.ems_probe_mfma(0, 10, None, d, None) == -1
    assert pl.ems_probe_mfma(8, 0, None, d, None) == -1
    assert pl.ems_probe_mfma(8, 10, None, None, None) == -1
    assert pl.ems_probe_mfma(8, 10, C.c_void_p(8), d, None) == -1          # misaligned operand buffer
    assert pl.ems_probe_copy(d, d, 24, None) == -1                           # not a multiple of 16
    assert pl.ems_probe_copy(C.c_void_p(8), d, 32, None) == -1
    assert pl.ems_probe_copy(None, d, 32, None) == -1


def test_binding_rejects_host_tensors_and_wrong_shapes(lib):
    """The Python layer only marshals: it refuses anything that is not a contiguous device tensor of
    the documented shape before the library is called (no CPU path exists)."""
    import torch
    p = _bad(budget=64)
    q = torch.zeros((1, 4, 512, 128), dtype=torch.bfloat16)
    k = torch.zeros((1, 2, 512, 128), dtype=torch.bfloat16)
    with pytest.raises(ValueError, match="device tensor"):
        B.ems_global_local_score(p, q, k)
    with pytest.raises(ValueError, match="device tensor"):
        B.ems_select(p, torch.zeros((1, 2, 512)), torch.zeros((1, 2, 512)))
    with pytest.raises(ValueError, match="device tensor"):
        B.ems_evict_merge(p, k, k, torch.zeros((1, 2, 48), dtype=torch.int32), torch.zeros((1, 2, 32), dtype=torch.int32))
    with pytest.raises(ValueError, match="device tensor"):
        B.ems_redundancy_rate(p, k, k)
    with pytest.raises(B.EmsError):
        B.ems_partition_sizes(_bad(budget=8))
