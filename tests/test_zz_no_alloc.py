"""The entry point for callers that cannot allocate: cqil_group_forward_static keeps its workspace in a static
device array.  Two calls in a row through the C ABI, the second with a smaller input, each compared with
cqil_group_forward on the same state (the same kernels run, so the results must agree bit for bit, which is
inside the parity tolerance by construction), and with the oracle."""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2404_06709_amd import binding as cq
from paper_2404_06709_amd import synth
from parity_util import TOL, Pair, rel_err, say

pytestmark = pytest.mark.gpu

MID = synth.Shape(512, 4, 128, 1024)


def _both(pair, x, d, lens):
    """Runs the step through both entry points from the same cache state; returns the two outputs and caches."""
    g = pair.group
    B, T, _ = x.shape
    k0, v0 = g.k.clone(), g.v.clone()
    out = []
    for static in (False, True):
        g.k.copy_(k0); g.v.copy_(v0)
        g.set_kv_len(list(lens) + [0] * (pair.b_max - len(lens)))
        g.kv.max_kv_len = int(max(lens))
        y = torch.full_like(x, float("nan"))
        if static:
            cq.cqil_group_forward_static(g.dims, g.P, d, g.packed, g.kv, x, y, B, T, True)
        else:
            cq.cqil_group_forward(g.dims, g.P, d, g.packed, g.kv, x, y, B, T, True, g.workspace(B, T))
        torch.cuda.synchronize()
        out.append((y.clone(), g.k.clone(), g.v.clone(), g.kv_len.cpu().tolist(), g.kv.max_kv_len))
    return out


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_static_scratch_entry_point_matches_group_forward(dtype):
    assert cq.cqil_static_scratch_bytes() == 8 << 20
    pair = Pair(MID, 3, dtype, max_seq=96, b_max=3, seed=4100, w_std=0.05, gain_jitter=0.1)
    pair.fill_cache([40, 0, 17], seed=3)
    lens = [40, 0, 17]
    # first call: a chunk of 3 sequences x 5 tokens (token-parallel kernels, split-K scratch in use for bf16);
    # second call: one token of one sequence (single-token kernels, a much smaller part of the same array)
    for (B, T, d, seed) in ((3, 5, 1, 11), (1, 1, 2, 12)):
        assert cq.cqil_workspace_bytes(pair.gd, pair.P, B, T) <= cq.cqil_static_scratch_bytes()
        x = pair.hidden(B, T, seed=seed).cuda()
        (y0, k0, v0, l0, m0), (y1, k1, v1, l1, m1) = _both(pair, x, d, lens[:B])
        assert torch.equal(y0.view(torch.uint8), y1.view(torch.uint8)), f"B={B} T={T}: x_out differs"
        assert torch.equal(k0, k1) and torch.equal(v0, v1), f"B={B} T={T}: caches differ"
        assert l0 == l1 and m0 == m1
        # and against the oracle, to the stated tolerance
        import oracle as orc
        okc, ovc = pair.okc.copy(), pair.ovc.copy()
        ref = orc.group_forward(pair.od, pair.np_layers, d, okc, ovc, np.asarray(lens[:B], dtype=np.int32),
                                synth.widen(x.cpu()))
        e = rel_err(synth.widen(y1.cpu()), ref)
        say(f"  static scratch {dtype} B={B} T={T}: bit-equal to cqil_group_forward, oracle rel err {e:.2e}")
        assert e <= TOL[dtype]


def test_static_scratch_rejects_steps_beyond_its_size():
    pair = Pair(MID, 2, torch.bfloat16, max_seq=4096, b_max=1, seed=4200)
    g = pair.group
    T = 2048
    assert cq.cqil_workspace_bytes(pair.gd, 2, 1, T) > cq.cqil_static_scratch_bytes()
    x = pair.hidden(1, T, seed=1).cuda()
    y = torch.zeros_like(x)
    g.set_kv_len([0])
    rc = cq.lib().cqil_group_forward_static(C.byref(g.dims), 2, 1, g.packed.data_ptr(), C.byref(g.kv), x.data_ptr(),
                                            y.data_ptr(), 1, T, 0, None)
    torch.cuda.synchronize()
    assert rc == cq.CQIL_ESIZE
    assert not y.any()           # nothing was launched
