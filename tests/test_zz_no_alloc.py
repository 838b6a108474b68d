"""The allocation-free evict-merge entry point against the one that takes a workspace.

Both run the same kernels, so every output has to be bit-identical.  Two calls in a row on the
same device, the second on a smaller problem, show that nothing left in the library's fixed
scratch array by one call leaks into the next."""
import numpy as np
import pytest
import torch

import ems_inputs
from gpu_util import dev_tensor
from paper_2412_08521_amd import binding as B

pytestmark = pytest.mark.gpu

# (batch, kv heads, head dim, N, window, budget, merge ratio): first the larger, then the smaller
SHAPES = [(2, 4, 128, 3000, 32, 700, 0.5), (1, 2, 128, 777, 16, 150, 0.7)]


def _partition(p, seed):
    rng = np.random.default_rng(seed)
    n_imp, n_tbm = B.ems_partition_sizes(p)
    imp = np.empty((p.batch, p.kv_heads, n_imp), np.int32)
    tbm = np.empty((p.batch, p.kv_heads, n_tbm), np.int32)
    for b in range(p.batch):
        for h in range(p.kv_heads):
            perm = rng.permutation(p.seq_len - p.window)
            imp[b, h] = np.sort(perm[:n_imp])
            tbm[b, h] = np.sort(perm[n_imp:n_imp + n_tbm])
    return imp, tbm


@pytest.mark.parametrize("mode", [B.EMS_BF16, B.EMS_F32])
def test_static_scratch_entry_matches_workspace_entry(mode):
    for call, (b, hkv, d, n, w, nb, r) in enumerate(SHAPES):
        print("evict_merge_static call", call, (b, hkv, d, n, w, nb, r), "mode", mode, flush=True)
        p = B.EmsParams(b, hkv, hkv, d, n, w, nb, merge_ratio=r, tau=0.22, dtype=mode)
        inp = ems_inputs.small(b, hkv, hkv, d, n, seed=40 + call)
        imp, tbm = _partition(p, seed=50 + call)
        k, v = dev_tensor(inp.k, mode), dev_tensor(inp.v, mode)
        imp_d, tbm_d = torch.from_numpy(imp).cuda(), torch.from_numpy(tbm).cuda()
        want = B.ems_evict_merge(p, k, v, imp_d, tbm_d)
        assert (want["tbm_dest"] < nb).any() and (want["tbm_dest"] == nb).any()   # merges and evictions
        # key norms kept inside the library's scratch array ...
        got = B.ems_evict_merge_static(p, k, v, imp_d, tbm_d, k_norm=False)
        # ... and handed back to the caller
        got_n = B.ems_evict_merge_static(p, k, v, imp_d, tbm_d)
        torch.cuda.synchronize()
        for name, ref in want.items():
            assert torch.equal(got_n[name], ref), name
            if name != "k_norm":
                assert torch.equal(got[name], ref), name
        assert got["k_norm"] is None


def test_static_scratch_entry_rejects_oversize():
    # merge_ws beyond the fixed array: refused on the host, nothing is launched
    p = B.EmsParams(64, 32, 32, 128, 1 << 20, 32, 1 << 19, merge_ratio=0.5)
    assert B.ems_workspace_bytes(p)[2] > 8 << 20
    t = torch.zeros(1, device="cuda")
    import ctypes as C
    cp = p.c()
    d = C.c_void_p(t.data_ptr())
    assert B.lib().ems_evict_merge_static(C.byref(cp), *([d] * 12), None) == B.EMS_ERR_WORKSPACE
