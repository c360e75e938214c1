"""GPU parity for rows wider than 65536 columns (one workgroup per row, the row streamed: once when the pass
for its minimum and maximum can also keep the candidates, else with eight bisection steps per further pass):
indices and values bit-exact against the CPU oracle in every mode."""
import numpy as np
import pytest

import oracle
import workloads

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def _gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2409_00822_amd as R

    R.load_library()
    return R


def bits(a):
    return np.ascontiguousarray(a, dtype=np.float32).view(np.int32)


def check(R, x, k, tag, modes=("exact", "early", "eps", "smallest")):
    xd = torch.from_numpy(x).cuda()
    if "exact" in modes:
        gv, gi = R.rtopk_rowwise_exact(xd, k)
        ov, oi = oracle.topk_exact(x, k)
        assert np.array_equal(gi.cpu().numpy(), oi), f"{tag} exact columns"
        assert np.array_equal(bits(gv.cpu().numpy()), bits(ov)), f"{tag} exact values"
    if "early" in modes:
        for mi in (0, 1, 7, 8, 9, 16, 17, 40):
            gv, gi = R.rtopk_rowwise(xd, k, mi)
            ov, oi = oracle.topk_earlystop(x, k, mi)
            assert np.array_equal(gi.cpu().numpy(), oi), f"{tag} max_iter={mi} columns"
            assert np.array_equal(bits(gv.cpu().numpy()), bits(ov)), f"{tag} max_iter={mi} values"
    if "eps" in modes:
        for eps in (0.0, 1e-4, 1e-2, 0.3, 5.0):
            gv, gi, gt = R.rtopk_rowwise_eps(xd, k, eps, want_iters=True)
            ov, oi, ot = oracle.alg1(x, k, eps_rel=eps, collect=1)
            assert np.array_equal(gi.cpu().numpy(), oi), f"{tag} eps={eps} columns"
            assert np.array_equal(bits(gv.cpu().numpy()), bits(ov)), f"{tag} eps={eps} values"
            assert np.array_equal(gt.cpu().numpy(), ot), f"{tag} eps={eps} exit iterations"
    if "smallest" in modes:
        gv, gi = R.rtopk_rowwise_exact_smallest(xd, k)
        ov, oi = oracle.topk_exact_smallest(x, k)
        assert np.array_equal(gi.cpu().numpy(), oi) and np.array_equal(bits(gv.cpu().numpy()), bits(ov)), f"{tag} smallest exact"
        gv, gi = R.rtopk_rowwise_smallest(xd, k, 9)
        ov, oi = oracle.topk_earlystop_smallest(x, k, 9)
        assert np.array_equal(gi.cpu().numpy(), oi) and np.array_equal(bits(gv.cpu().numpy()), bits(ov)), f"{tag} smallest early"


@pytest.mark.parametrize("N,M,ks", [(3, 65540, (1, 50, 4000)), (2, 70001, (33,)), (4, 131072, (64, 1000)),
                                     (2, 100003, (7, 100003)), (1, 1 << 20, (256, 50000)), (5, 90000, (90000 - 1,))])
def test_streamed_rows_every_mode(N, M, ks):
    R = _gpu()
    x = workloads.normal(N, M, seed=N * 53 + M)
    for k in ks:
        check(R, x, k, f"N={N} M={M} k={k}")


@pytest.mark.parametrize("M", [65600, 200000])
def test_streamed_tie_heavy_rows(M):
    R = _gpu()
    for name, x in (("pool", workloads.from_pool(3, M, 71 + M)), ("ints", workloads.small_ints(3, M, 72 + M, span=20)),
                    ("ties", workloads.normal_ties(3, M, 73 + M, p=0.5))):
        for k in (1, 64, 1000, M // 2):
            check(R, x, k, f"{name} M={M} k={k}", modes=("exact", "early", "eps"))


def test_streamed_constant_rows_signed_zeros_and_unaligned_input():
    R = _gpu()
    M = 70000
    x = np.full((3, M), 2.5, dtype=np.float32)
    x[1, ::3] = -1.0
    x[2, ::2] = 0.0
    x[2, 1::4] = -0.0
    x[2, 5] = 1.0
    x[2, 9] = -1.0
    for k in (1, 100, 23334, M - 1, M):
        check(R, x, k, f"const k={k}", modes=("exact", "early", "eps"))
    # 4-byte aligned input: the scalar-load instance
    y = workloads.normal(2, 65544, seed=99)
    buf = torch.empty(2 * 65544 + 1, dtype=torch.float32, device="cuda")
    yd = buf[1:].view(2, 65544)
    yd.copy_(torch.from_numpy(y))
    gv, gi = R.rtopk_rowwise_exact(yd, 77)
    ov, oi = oracle.topk_exact(y, 77)
    assert np.array_equal(gi.cpu().numpy(), oi) and np.array_equal(bits(gv.cpu().numpy()), bits(ov))


def test_streamed_rows_whose_candidates_crowd_one_part_of_the_row():
    # ascending and descending rows put all k winners into one wavefront's sixteenth of the row: its
    # candidate list overflows and the general ranking pass takes over; 2049 <= k never uses the lists
    R = _gpu()
    M = 80000
    base = np.sort(workloads.normal(1, M, seed=31)[0])
    x = np.stack([base, base[::-1].copy(), np.roll(base, 12345)]).astype(np.float32)
    for k in (100, 129, 2048, 2049):
        check(R, x, k, f"sorted k={k}", modes=("exact", "early"))


def test_streamed_rows_skewed_values_outliers_and_k_near_the_list_capacity():
    # the pass that finds minimum and maximum also keeps the keys above a rising floor, chosen from 256 equal
    # parts of the range seen so far: heavy skew, one huge outlier (every other key in the lowest part) and a
    # range that spans many binades put that choice under stress; k around a thousand fills the lists; every
    # case must come out the same whether the lists are used or the search passes take over
    R = _gpu()
    M = 150000
    rng = np.random.default_rng(2024)
    g = rng.standard_normal((6, M)).astype(np.float32)
    x = np.empty((6, M), dtype=np.float32)
    x[0] = np.exp(8.0 * g[0])            # lognormal over ~28 binades
    x[1] = -np.exp(8.0 * g[1])           # the same, all negative
    x[2] = g[2]
    x[2, 77777] = 3.0e38                 # one outlier near the top of the format
    x[3] = g[3]
    x[3, 5] = -3.0e38                    # and one at the bottom
    x[4] = np.where(g[4] > 0, 1.0e-30 * g[4], g[4])   # positive side squeezed into tiny values
    x[5] = np.floor(g[5] * 2.0) / 2.0    # a few dozen distinct values
    for k in (3, 512, 1000, 1365, 1366, 2047):
        check(R, x, k, f"skewed k={k}", modes=("exact", "early", "eps", "smallest"))


def test_streamed_rows_at_the_maximum_width():
    # M = rtopk_max_m() = 2^24 columns (64 MiB per row): column numbers use 24 bits, a wavefront makes 4096
    # loads, the floor of the first pass is raised 12 times; small k from the lists, k = 5000 through the
    # search passes
    R = _gpu()
    M = 1 << 24
    x = workloads.laplace(2, M, seed=777)
    x[1, M - 1] = 50.0    # the last column must be reachable
    x[1, 0] = 49.0
    for k in (64, 5000):
        check(R, x, k, f"M=2^24 k={k}", modes=("exact", "smallest"))
        xd = torch.from_numpy(x).cuda()
        gv, gi = R.rtopk_rowwise(xd, k, 8)
        ov, oi = oracle.topk_earlystop(x, k, 8)
        assert np.array_equal(gi.cpu().numpy(), oi) and np.array_equal(bits(gv.cpu().numpy()), bits(ov))
        gv, gi, gt = R.rtopk_rowwise_eps(xd, k, 1e-3, want_iters=True)
        ov, oi, ot = oracle.alg1(x, k, eps_rel=1e-3, collect=1)
        assert np.array_equal(gi.cpu().numpy(), oi) and np.array_equal(bits(gv.cpu().numpy()), bits(ov))
        assert np.array_equal(gt.cpu().numpy(), ot)


def test_streamed_rows_many_rows_guard_bands_and_nonfinite_inputs():
    R = _gpu()
    N, M, k = 300, 65600, 128
    x = workloads.laplace(N, M, seed=123)
    pad = 4096
    vbuf = torch.full((N * k + 2 * pad,), 12345.0, dtype=torch.float32, device="cuda")
    ibuf = torch.full((N * k + 2 * pad,), -77, dtype=torch.int32, device="cuda")
    ov, oi = vbuf[pad:pad + N * k].view(N, k), ibuf[pad:pad + N * k].view(N, k)
    xd = torch.from_numpy(x).cuda()
    R.rtopk_rowwise_exact(xd, k, ov, oi)
    torch.cuda.synchronize()
    ev, ei = oracle.topk_exact(x, k)
    assert np.array_equal(oi.cpu().numpy(), ei) and np.array_equal(bits(ov.cpu().numpy()), bits(ev))
    assert (vbuf[:pad] == 12345.0).all() and (vbuf[-pad:] == 12345.0).all()
    assert (ibuf[:pad] == -77).all() and (ibuf[-pad:] == -77).all()
    # non-finite inputs: outside the contract, but the calls terminate and stay inside the outputs
    x[::7, 3] = np.inf
    x[::11, 9] = -np.inf
    x[::13, 100] = np.nan
    x[5] = np.nan
    xd = torch.from_numpy(x).cuda()
    for call in (lambda: R.rtopk_rowwise_exact(xd, k, ov, oi), lambda: R.rtopk_rowwise(xd, k, 8, ov, oi),
                 lambda: R.rtopk_rowwise_eps(xd, k, 1e-3, ov, oi)):
        call()
        torch.cuda.synchronize()
        assert (vbuf[:pad] == 12345.0).all() and (vbuf[-pad:] == 12345.0).all()
        assert (ibuf[:pad] == -77).all() and (ibuf[-pad:] == -77).all()


def test_the_variants_without_a_streamed_form_refuse_wider_rows():
    R = _gpu()
    x = torch.zeros((2, 65540), dtype=torch.float32, device="cuda")
    with pytest.raises(R.RTopKError):
        R.rtopk_maxk_dense(x, 5)
    with pytest.raises(R.RTopKError):
        R.rtopk_rowwise_exact_bf16(x.bfloat16(), 5)
