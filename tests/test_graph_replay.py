"""The entry points allocate nothing and synchronise nothing, so a sequence of calls can be captured
into a HIP graph (after one eager call has loaded the kernels) and replayed: launch-bound
sequences then cost one graph launch.  Every replay is checked, bit for bit, against the eager
calls on the same inputs, with eager work and synchronisations between the replays; the eager
path is what the parity tests check against the oracle, and one result is checked against it here
too."""
import numpy as np
import pytest

import oracle
import paper_2405_05118_amd as mdh
from paper_2405_05118_amd import workloads as W

torch = pytest.importorskip("torch")

pytestmark = pytest.mark.gpu


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _ws(inst, sizes, p=None):
    n = mdh.mdh_workspace_size(inst, sizes, p)
    return torch.empty(max(n, 4) // 4, dtype=torch.int32, device="cuda") if n else None


def test_sequence_of_calls_replays_from_a_graph():
    M, N, K = 96, 160, 4096          # split reduction: main kernel + second pass
    n_scan = 1 << 20                 # single-pass scan: workspace initialisation kernel + scan kernel
    n_dot = 1 << 20
    nx = 40
    a = torch.empty((M, K), device="cuda")
    b = torch.empty((K, N), device="cuda")
    xs = torch.empty((1, n_scan), device="cuda")
    xd = torch.empty(n_dot, device="cuda")
    yd = torch.empty(n_dot, device="cuda")
    g3 = torch.empty((nx + 2, nx + 2, nx + 2), device="cuda")
    nA, nB = 300, 5000
    A8 = torch.empty((nA, 8), dtype=torch.int32, device="cuda")
    B8 = torch.empty((nB, 8), dtype=torch.int32, device="cuda")
    wp = dev(np.arange(1, 9, dtype=np.int32))
    wm = dev(-np.arange(1, 9, dtype=np.int32))

    # MatMul with the reduction split over workgroups (the default at this size keeps k inside one launch)
    pm = next(p for p in (mdh.mdh_candidate(mdh.MDH_MATMUL, (M, N, K), i) for i in range(mdh.mdh_num_candidates(mdh.MDH_MATMUL, (M, N, K))))
              if p.prt[3][2] > 1 and p.prt[4][2] == 1)
    ps = mdh.mdh_default_params(mdh.MDH_SCAN, (1, n_scan))
    ws_m, ws_s = _ws(mdh.MDH_MATMUL, (M, N, K), pm), _ws(mdh.MDH_SCAN, (1, n_scan))
    # small-M MatMul and Dot: split reductions folded by the last workgroup part to arrive (arrival
    # counters inside the library that every launch must leave at zero, replay after replay)
    Ms, Ns, Ks = 16, 1000, 2048
    a_s = torch.empty((Ms, Ks), device="cuda")
    b_s = torch.empty((Ks, Ns), device="cuda")
    p_small = mdh.mdh_default_params(mdh.MDH_MATMUL, (Ms, Ns, Ks))
    assert p_small.prt[3][2] > 1 and p_small.out_region == 0
    ws_small = _ws(mdh.MDH_MATMUL, (Ms, Ns, Ks))
    assert mdh.mdh_default_params(mdh.MDH_DOT, (n_dot,)).out_region == 0
    ws_d, ws_p = _ws(mdh.MDH_DOT, (n_dot,)), _ws(mdh.MDH_CUSTOM_REDUCE, (nA, nB, 8))
    assert ws_s is not None and ps.prt[3][1] > 1
    # few-channel MCC with its tiles dealt out by a ticket counter (inside the library, left at zero by every
    # launch): 24 images of 99 x 163 x 3, 5 x 5 filter, stride 2 -- more tiles than resident workgroups
    cN, cH, cW, cC, cK, cR = 24, 99, 163, 3, 40, 5
    cP, cQ = (cH - cR) // 2 + 1, (cW - cR) // 2 + 1
    c_sizes = (cN, cP, cQ, cK, cC, cR, cR, 2, 2)
    pc = next(p for p in (mdh.mdh_candidate(mdh.MDH_MCC, c_sizes, i) for i in range(mdh.mdh_num_candidates(mdh.MDH_MCC, c_sizes)))
              if p.blk[4] == 1 and p.strided == 1)
    cx = torch.empty((cN, cH, cW, cC), device="cuda")
    cf = torch.empty((cK, cR, cR, cC), device="cuda")

    def outputs():
        return [torch.full((M, N), float("nan"), device="cuda"), torch.full((1, n_scan), float("nan"), device="cuda"),
                torch.full((1,), float("nan"), device="cuda"), torch.full((nx, nx, nx), float("nan"), device="cuda"),
                torch.full((nA,), -1, dtype=torch.int32, device="cuda"), torch.full((nA,), -1, dtype=torch.int32, device="cuda"),
                torch.full((Ms, Ns), float("nan"), device="cuda"), torch.full((cN, cP, cQ, cK), float("nan"), device="cuda")]

    def calls(o):
        mdh.mdh_matmul(a, b, o[0], pm, ws_m)
        mdh.mdh_matmul(a_s, b_s, o[6], None, ws_small)
        mdh.mdh_scan(xs, o[1], None, ws_s)
        mdh.mdh_dot(xd, yd, o[2], None, ws_d)
        mdh.mdh_stencil(g3, o[3], 0.5, 1.0 / 12.0)
        mdh.mdh_custom_reduce(A8, B8, wp, wm, o[4], o[5], None, ws_p)
        mdh.mdh_mcc(cx, cf, o[7], (2, 2), pc)

    def fill(seed):
        a.copy_(dev(W.uniform(seed, 1, (M, K), -1, 1)))
        b.copy_(dev(W.uniform(seed, 2, (K, N), -1, 1)))
        xs.copy_(dev(W.uniform(seed, 3, (1, n_scan), -1, 1)))
        xd.copy_(dev(W.uniform(seed, 4, (n_dot,), -1, 1)))
        yd.copy_(dev(W.uniform(seed, 5, (n_dot,), -1, 1)))
        g3.copy_(dev(W.uniform(seed, 6, (nx + 2, nx + 2, nx + 2), 0, 1)))
        a_s.copy_(dev(W.uniform(seed, 9, (Ms, Ks), -1, 1)))
        b_s.copy_(dev(W.uniform(seed, 10, (Ks, Ns), -1, 1)))
        A8.copy_(dev(W.integers(seed, 7, (nA, 8), 0, 3)))
        B8.copy_(dev(W.integers(seed, 8, (nB, 8), 0, 3)))
        cx.copy_(dev(W.uniform(seed, 11, (cN, cH, cW, cC), -1, 1)))
        cf.copy_(dev(W.uniform(seed, 12, (cK, cR, cR, cC), -1, 1)))

    fill(W.SEED_BASE + 90)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    out_g = outputs()
    with torch.cuda.stream(side):
        calls(out_g)  # eager, on the capture stream: loads the kernels, sets their attributes
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        calls(out_g)
    torch.cuda.synchronize()

    for rep in range(4):
        fill(W.SEED_BASE + 91 + rep)
        out_e = outputs()
        calls(out_e)                     # eager, default stream
        torch.cuda.synchronize()
        for t in out_g:
            t.fill_(-1) if t.dtype == torch.int32 else t.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for i, (e, g) in enumerate(zip(out_e, out_g)):
            assert torch.equal(e, g), (rep, i)
        if rep == 0:
            ref, refabs = oracle.matmul(a.cpu().numpy(), b.cpu().numpy(), with_abs=True)
            assert float(np.max(np.abs(out_g[0].cpu().numpy() - ref) / refabs)) <= 1e-4
            ref, refabs = oracle.matmul(a_s.cpu().numpy(), b_s.cpu().numpy(), with_abs=True)
            assert float(np.max(np.abs(out_g[6].cpu().numpy() - ref) / refabs)) <= 1e-4
            ref, refabs = oracle.mcc(cx.cpu().numpy(), cf.cpu().numpy(), (2, 2), with_abs=True)
            assert float(np.max(np.abs(out_g[7].cpu().numpy() - ref) / refabs)) <= 1e-4
