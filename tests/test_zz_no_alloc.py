"""mdh_custom_reduce_static, the entry point for callers that cannot allocate: its results must equal
those of mdh_custom_reduce (which takes a caller's workspace) bit for bit, on two calls in a row that
share the library's static scratch array, the second with a smaller input."""
import numpy as np
import pytest

import paper_2405_05118_amd as mdh
from paper_2405_05118_amd import workloads as W

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def both(nA, nB, seed):
    cfg = W.PrlCfg(nA, nB, 8, seed)
    A, Bt, wp, wm = (dev(x) for x in W.prl_inputs(cfg))
    sizes = (nA, nB, 8)
    p = mdh.mdh_default_params(mdh.MDH_CUSTOM_REDUCE, sizes)
    assert p.prt[3][1] > 1, "the default must split b over workgroups, or no scratch memory is used"
    n = mdh.mdh_workspace_size(mdh.MDH_CUSTOM_REDUCE, sizes)
    assert 0 < n <= mdh.mdh_static_scratch_bytes()
    ws = torch.empty(n // 4, dtype=torch.int32, device="cuda")
    s0 = torch.full((nA,), -7, dtype=torch.int32, device="cuda")
    i0 = torch.full((nA,), -7, dtype=torch.int32, device="cuda")
    mdh.mdh_custom_reduce(A, Bt, wp, wm, s0, i0, None, ws)
    s1 = torch.full((nA,), -9, dtype=torch.int32, device="cuda")
    i1 = torch.full((nA,), -9, dtype=torch.int32, device="cuda")
    mdh.mdh_custom_reduce_static(A, Bt, wp, wm, s1, i1)
    torch.cuda.synchronize()
    return (s0.cpu().numpy(), i0.cpu().numpy()), (s1.cpu().numpy(), i1.cpu().numpy())


def test_static_scratch_matches_workspace_entry_point_twice():
    # first call: 20000 x 30000 records; second call, right after it on the same array: 3000 x 4100
    for nA, nB, seed in ((20000, 30000, W.SEED_BASE + 201), (3000, 4100, W.SEED_BASE + 202)):
        (s0, i0), (s1, i1) = both(nA, nB, seed)
        assert i0.min() >= 0 and i0.max() < nB
        assert np.array_equal(s0, s1) and np.array_equal(i0, i1), (nA, nB)


def test_static_scratch_limit_is_an_error():
    # 2 * S * nA int32 beyond the 16 MiB array: refused before anything is enqueued
    nA, nB = (1 << 17) + 128, 1 << 18  # the default splits b 16 ways here: 2 * 16 * nA int32 > 16 MiB
    p = mdh.mdh_default_params(mdh.MDH_CUSTOM_REDUCE, (nA, nB, 8))
    assert 2 * p.prt[3][1] * nA * 4 > mdh.mdh_static_scratch_bytes()
    one = torch.zeros(8, dtype=torch.int32, device="cuda")
    big = torch.zeros((nA, 8), dtype=torch.int32, device="cuda")
    bt = torch.zeros((nB, 8), dtype=torch.int32, device="cuda")
    out = torch.full((nA,), -3, dtype=torch.int32, device="cuda")
    with pytest.raises(mdh.MdhError) as e:
        mdh.mdh_custom_reduce_static(big, bt, one, one, out, out.clone())
    assert e.value.status == 8
    torch.cuda.synchronize()
    assert int(out.min()) == -3 and int(out.max()) == -3
