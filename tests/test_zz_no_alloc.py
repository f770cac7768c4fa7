"""dsvt_attn_pool_static -- the entry point that allocates nothing -- against dsvt_attn_pool, through the C ABI.

Two calls in a row on the library's built-in scratch, the second with a smaller input (what the first call left in
the scratch must not matter): pooled coordinates, counts and status bit for bit, features to the parity bar (the two
entry points run the same kernels, so the features come out equal bit for bit as well).
"""
import ctypes as C

import numpy as np
import pytest
import torch

import synth

pytestmark = pytest.mark.gpu
dsvt = pytest.importorskip("paper_2301_06051_amd")
from gpu_util import TOL, dev_coords, dev_feats, rel_err  # noqa: E402


def _outs(n, x):
    return (torch.full((n, 4), -7, dtype=torch.int32, device="cuda"), torch.zeros_like(x),
            torch.zeros((1,), dtype=torch.int32, device="cuda"), torch.zeros((1,), dtype=torch.int32, device="cuda"))


def test_static_scratch_entry_point_matches_workspace_entry_point():
    cfg = synth.CONFIGS[4]
    lib = dsvt.lib()
    w = synth.make_pool_weights(91, cfg["C"], cfg["heads"], cfg["dtype"])
    ptr = lambda t: C.c_void_p(t.data_ptr())
    stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    for n_vox, pool, mask_empty in ((20000, (1, 1, 4), 1), (6000, (2, 2, 2), 0)):
        coords = synth.make_frame(4, n=n_vox)
        n = len(coords)
        print(f"[case] dsvt_attn_pool_static vs dsvt_attn_pool: {n} voxels, pool {pool}, mask_empty {mask_empty}", flush=True)
        pw = dsvt.PoolWeights(w, cfg["grid"], pool, cfg["batch"], mask_empty)
        cd = dev_coords(coords)
        x = dev_feats(synth.make_features(35, n, cfg["C"], cfg["dtype"]), cfg["dtype"])
        ws = torch.empty((dsvt.dsvt_attn_pool_workspace_size(pw, n),), dtype=torch.uint8, device="cuda")
        ref, got = _outs(n, x), _outs(n, x)
        torch.cuda.synchronize()
        rc = lib.dsvt_attn_pool(C.byref(pw.struct), ptr(cd), ptr(x), n, ptr(ref[0]), ptr(ref[1]), ptr(ref[2]), ptr(ws),
                                ws.numel(), ptr(ref[3]), stream)
        assert rc == 0
        rc = lib.dsvt_attn_pool_static(C.byref(pw.struct), ptr(cd), ptr(x), n, ptr(got[0]), ptr(got[1]), ptr(got[2]),
                                       ptr(got[3]), stream)
        assert rc == 0
        torch.cuda.synchronize()
        m = int(ref[2].item())
        assert int(got[2].item()) == m and 0 < m < n
        assert int(got[3].item()) == int(ref[3].item()) == 0
        assert torch.equal(got[0], ref[0])                         # pooled coordinates, and the untouched rows past them
        assert rel_err(got[1][:m], ref[1][:m].double().cpu().numpy()) < TOL[cfg["dtype"]]
        assert torch.equal(got[1], ref[1])
    # an input whose scratch would not fit the built-in array is refused, nothing is enqueued
    big = dsvt.PoolWeights(w, (468, 468, 32), (1, 1, 1), 8, 1)       # 56 M pooled cells: bitmap + prefix alone are 14 MB
    assert dsvt.dsvt_attn_pool_workspace_size(big, 1000) > (8 << 20)
    cd = dev_coords(synth.make_frame(4, n=1000))
    x = dev_feats(synth.make_features(35, 1000, cfg["C"], cfg["dtype"]), cfg["dtype"])
    got = _outs(1000, x)
    rc = lib.dsvt_attn_pool_static(C.byref(big.struct), ptr(cd), ptr(x), 1000, ptr(got[0]), ptr(got[1]), ptr(got[2]), ptr(got[3]),
                                   stream)
    assert rc == dsvt.binding.DSVT_ENOSPC
    torch.cuda.synchronize()
    assert int(got[2].item()) == 0 and torch.all(got[0] == -7)
