"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element.

Bar: column indices bit-exact, values bit-exact copies (tolerance 0), in both modes.
"""
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

    R.load_library()  # fails loudly if the HIP library is not built
    return R


def bits(a):
    return np.ascontiguousarray(a, dtype=np.float32).view(np.int32)


def run_gpu(R, x_np, k, mode, max_iter=0, u8=False, x_dev=None):
    x = torch.from_numpy(x_np).cuda() if x_dev is None else x_dev
    if mode == "exact":
        v, i = (R.rtopk_rowwise_exact_u8 if u8 else R.rtopk_rowwise_exact)(x, k)
    else:
        v, i = (R.rtopk_rowwise_u8 if u8 else R.rtopk_rowwise)(x, k, max_iter)
    torch.cuda.synchronize()
    return v.cpu().numpy(), i.cpu().numpy()


def run_oracle(x_np, k, mode, max_iter=0):
    if mode == "exact":
        return oracle.topk_exact(x_np, k)
    return oracle.topk_earlystop(x_np, k, max_iter)


def assert_parity(R, x_np, k, mode, max_iter=0, u8=False, tag=""):
    gv, gi = run_gpu(R, x_np, k, mode, max_iter, u8)
    ov, oi = run_oracle(x_np, k, mode, max_iter)
    gi32 = gi.astype(np.int32)
    if not np.array_equal(gi32, oi):
        bad = np.nonzero((gi32 != oi).any(axis=1))[0]
        r = int(bad[0])
        raise AssertionError(f"{tag} index mismatch in {bad.size} rows; first row {r}: gpu {gi32[r]} oracle {oi[r]}")
    assert np.array_equal(bits(gv), bits(ov)), f"{tag} value bits differ"


# ----------------------------------------------------------------------------------------------
# small shapes: several tiles, ragged tails, every load path
# ----------------------------------------------------------------------------------------------
SHAPES = [
    # (N, M, ks)
    (1, 1, (1,)), (5, 2, (1, 2)), (9, 7, (1, 3, 7)), (33, 63, (1, 8, 63)), (64, 64, (1, 5, 16, 64)),
    (65, 65, (3, 65)), (100, 100, (10, 12)), (257, 128, (1, 16, 20, 128)), (31, 130, (13,)),
    (77, 200, (25, 32)), (4099, 256, (1, 16, 31, 32, 64, 128, 255, 256)), (50, 260, (33, 64)),
    (130, 300, (32,)), (515, 512, (64, 100)), (129, 768, (96,)), (40, 1000, (125, 128)),
    (259, 1024, (128, 1000)), (33, 1500, (200,)), (67, 2048, (256,)), (35, 3000, (64,)),
    (70, 4096, (64, 256, 1024)), (9, 4095, (7, 512)), (17, 1021, (17,)), (21, 6000, (300,)),
    (20, 8192, (64, 512, 4097)), (7, 5001, (33,)), (5, 8191, (8,)),
    (6, 8192, (8191, 8192)),  # the largest staging area: 8192 pairs = 64 KiB of LDS
]


@pytest.mark.parametrize("N,M,ks", SHAPES)
def test_exact_small_shapes(N, M, ks):
    R = _gpu()
    x = workloads.normal(N, M, seed=N * 7919 + M)
    for k in ks:
        assert_parity(R, x, k, "exact", tag=f"N={N} M={M} k={k}")


@pytest.mark.parametrize("N,M,ks", SHAPES)
def test_earlystop_small_shapes(N, M, ks):
    R = _gpu()
    x = workloads.normal(N, M, seed=N * 104729 + M)
    for k in ks:
        for mi in (0, 1, 2, 4, 8, 16, 40):
            assert_parity(R, x, k, "early", mi, tag=f"N={N} M={M} k={k} max_iter={mi}")


@pytest.mark.parametrize("M", [3, 8, 17, 64, 128, 256, 512, 1024])
def test_tie_heavy_rows(M):
    R = _gpu()
    for gen, seed in (("pool", 61), ("ints", 62)):
        x = workloads.from_pool(700, M, seed + M) if gen == "pool" else workloads.small_ints(700, M, seed + M, span=3)
        for k in sorted({1, 2, max(1, M // 8), M // 2 or 1, M - 1 or 1, M}):
            assert_parity(R, x, k, "exact", tag=f"{gen} M={M} k={k}")
            for mi in (0, 3, 8, 30):
                assert_parity(R, x, k, "early", mi, tag=f"{gen} M={M} k={k} mi={mi}")


@pytest.mark.parametrize("M", [1280, 2048, 3000, 4096, 6144, 8192])
def test_tie_heavy_wide_rows(M):
    # wide rows count without keeping masks and select through the converged-search path under ties
    R = _gpu()
    for gen, seed in (("pool", 91), ("ints", 92), ("ties", 93)):
        if gen == "pool":
            x = workloads.from_pool(150, M, seed + M)
        elif gen == "ints":
            x = workloads.small_ints(150, M, seed + M, span=20)
        else:
            x = workloads.normal_ties(150, M, seed + M, p=0.5)
        for k in (1, 64, 257, M // 2, M - 1):
            assert_parity(R, x, k, "exact", tag=f"{gen} M={M} k={k}")
            for mi in (0, 5, 30):
                assert_parity(R, x, k, "early", mi, tag=f"{gen} M={M} k={k} mi={mi}")


def test_all_equal_and_two_valued_rows():
    R = _gpu()
    x = np.full((40, 256), 3.25, dtype=np.float32)
    x[20:, ::3] = -1.5
    x[30:, 5] = 7.0
    for k in (1, 32, 85, 86, 200, 256):
        assert_parity(R, x, k, "exact", tag=f"const k={k}")
        assert_parity(R, x, k, "early", 8, tag=f"const k={k}")


@pytest.mark.parametrize("M,k", [(256, 32), (128, 16), (200, 24), (64, 8), (100, 7), (255, 33)])
def test_uint8_columns(M, k):
    R = _gpu()
    x = workloads.normal_ties(3001, M, seed=70 + M, p=0.2)
    assert_parity(R, x, k, "exact", u8=True, tag=f"u8 M={M} k={k}")
    assert_parity(R, x, k, "early", 8, u8=True, tag=f"u8 M={M} k={k}")


def test_unaligned_input_and_output_pointers_take_the_scalar_paths():
    R = _gpu()
    N, M, k = 300, 256, 32
    x = workloads.normal(N, M, seed=81)
    buf = torch.empty(N * M + 1, dtype=torch.float32, device="cuda")
    xd = buf[1:].view(N, M)  # 4-byte aligned only
    xd.copy_(torch.from_numpy(x))
    ob = torch.empty(N * k + 1, dtype=torch.float32, device="cuda")
    ib = torch.empty(N * k + 1, dtype=torch.int32, device="cuda")
    ov, oi = ob[1:].view(N, k), ib[1:].view(N, k)
    R.rtopk_rowwise_exact(xd, k, ov, oi)
    torch.cuda.synchronize()
    ev, ei = oracle.topk_exact(x, k)
    assert np.array_equal(oi.cpu().numpy(), ei) and np.array_equal(bits(ov.cpu().numpy()), bits(ev))
    R.rtopk_rowwise(xd, k, 5, ov, oi)
    torch.cuda.synchronize()
    sv, si = oracle.topk_earlystop(x, k, 5)
    assert np.array_equal(oi.cpu().numpy(), si) and np.array_equal(bits(ov.cpu().numpy()), bits(sv))


def test_writes_stay_inside_the_outputs_and_nonfinite_inputs_terminate():
    R = _gpu()
    N, M, k = 1000, 256, 32
    x = workloads.normal(N, M, seed=82)
    x[::7, 3] = np.inf
    x[::11, 9] = -np.inf
    x[::13, 100] = np.nan
    x[5] = np.nan
    x[6] = np.inf
    pad = 4096
    vbuf = torch.full((N * k + 2 * pad,), 12345.0, dtype=torch.float32, device="cuda")
    ibuf = torch.full((N * k + 2 * pad,), -77, dtype=torch.int32, device="cuda")
    ov = vbuf[pad:pad + N * k].view(N, k)
    oi = ibuf[pad:pad + N * k].view(N, k)
    xd = torch.from_numpy(x).cuda()
    for call in (lambda: R.rtopk_rowwise_exact(xd, k, ov, oi), lambda: R.rtopk_rowwise(xd, k, 8, ov, oi)):
        call()
        torch.cuda.synchronize()
        assert (vbuf[:pad] == 12345.0).all() and (vbuf[-pad:] == 12345.0).all()
        assert (ibuf[:pad] == -77).all() and (ibuf[-pad:] == -77).all()
    # rows without non-finite values are still exact
    clean = np.isfinite(x).all(axis=1)
    R.rtopk_rowwise_exact(xd, k, ov, oi)
    torch.cuda.synchronize()
    _, ei = oracle.topk_exact(x[clean], k)
    assert np.array_equal(oi.cpu().numpy()[clean], ei)


# ----------------------------------------------------------------------------------------------
# Algorithm 1 with a precision epsilon, and its exit-iteration output
# ----------------------------------------------------------------------------------------------
def assert_eps_parity(R, x_np, k, eps_rel, tag=""):
    xd = torch.from_numpy(x_np).cuda()
    gv, gi, gt = R.rtopk_rowwise_eps(xd, k, eps_rel, want_iters=True)
    torch.cuda.synchronize()
    ov, oi, ot = oracle.alg1(x_np, k, eps_rel=eps_rel, collect=1)
    gi, gt = gi.cpu().numpy(), gt.cpu().numpy()
    if not np.array_equal(gi, oi):
        bad = np.nonzero((gi != oi).any(axis=1))[0]
        raise AssertionError(f"{tag} index mismatch in {bad.size} rows; first {bad[0]}: gpu {gi[bad[0]]} oracle {oi[bad[0]]}")
    assert np.array_equal(bits(gv.cpu().numpy()), bits(ov)), f"{tag} value bits differ"
    assert np.array_equal(gt, ot), f"{tag} exit iterations differ"


@pytest.mark.parametrize("N,M,ks", [(9, 7, (1, 3, 7)), (257, 128, (16, 128)), (4099, 256, (1, 32, 128, 256)),
                                     (130, 300, (32,)), (515, 512, (64,)), (129, 768, (96,)), (259, 1024, (128,)),
                                     (35, 3000, (64,)), (70, 4096, (256,)), (9, 4095, (7,)), (100, 100, (12,)),
                                     (12, 8192, (100,)), (6, 7000, (64,))])
def test_eps_mode_small_shapes(N, M, ks):
    R = _gpu()
    x = workloads.normal(N, M, seed=N * 31 + M)
    for k in ks:
        for eps in (0.0, 1e-6, 1e-4, 1e-2, 0.3, 5.0):
            assert_eps_parity(R, x, k, eps, tag=f"N={N} M={M} k={k} eps={eps}")


@pytest.mark.parametrize("M", [8, 64, 256, 1024, 2048])
def test_eps_mode_tie_heavy_and_negative_rows(M):
    R = _gpu()
    xs = [workloads.from_pool(300, M, 55 + M), workloads.small_ints(300, M, 56 + M, span=4),
          -np.abs(workloads.normal(300, M, 57 + M)) - 1.0]  # all-negative rows: epsilon uses |max|
    for x in xs:
        for k in sorted({1, max(1, M // 8), M // 2, M}):
            for eps in (0.0, 1e-4, 0.05):
                assert_eps_parity(R, x, k, eps, tag=f"M={M} k={k} eps={eps}")


def test_eps_zero_equals_exact_entry_point_and_iters_are_optional():
    R = _gpu()
    x = workloads.normal_ties(6000, 256, seed=58, p=0.2)
    xd = torch.from_numpy(x).cuda()
    ev, ei = R.rtopk_rowwise_exact(xd, 32)
    gv, gi = R.rtopk_rowwise_eps(xd, 32, 0.0)  # no iteration output requested
    torch.cuda.synchronize()
    assert torch.equal(ei, gi) and torch.equal(ev.view(torch.int32), gv.view(torch.int32))


def test_exit_iteration_statistics_of_table1_on_the_gpu():
    # Table 1 (Section 3.1) reproduced by the kernel's own iteration output: eps' = 1e-4, M = 256, N(0,1).
    from conftest import read_table

    R = _gpu()
    header, rows = read_table("table1_exit_cumulative.txt")
    x = workloads.normal(100000, 256, seed=1001)
    xd = torch.from_numpy(x).cuda()
    for col, k in enumerate(int(h[1:]) for h in header[1:]):
        _, _, it = R.rtopk_rowwise_eps(xd, k, 1e-4, want_iters=True)
        it = it.cpu().numpy()
        for row in rows:
            t, paper = int(row[0]), float(row[1 + col])
            assert abs(float((it <= t).mean() * 100.0) - paper) < 1.0, (k, t)


def test_config1_eps_mode_full_size():
    R = _gpu()
    x = workloads.make("c1_maxk")
    assert_eps_parity(R, x, 32, 1e-4, tag="c1 eps=1e-4")
    assert_eps_parity(R, x, 32, 0.0, tag="c1 eps=0")


# ----------------------------------------------------------------------------------------------
# the k smallest
# ----------------------------------------------------------------------------------------------
def assert_smallest_parity(R, x_np, k, mode, max_iter=0, tag=""):
    xd = torch.from_numpy(x_np).cuda()
    if mode == "exact":
        gv, gi = R.rtopk_rowwise_exact_smallest(xd, k)
        ov, oi = oracle.topk_exact_smallest(x_np, k)
    else:
        gv, gi = R.rtopk_rowwise_smallest(xd, k, max_iter)
        ov, oi = oracle.topk_earlystop_smallest(x_np, k, max_iter)
    torch.cuda.synchronize()
    gi = gi.cpu().numpy()
    if not np.array_equal(gi, oi):
        bad = np.nonzero((gi != oi).any(axis=1))[0]
        raise AssertionError(f"{tag} index mismatch in {bad.size} rows; first {bad[0]}: gpu {gi[bad[0]]} oracle {oi[bad[0]]}")
    assert np.array_equal(bits(gv.cpu().numpy()), bits(ov)), f"{tag} value bits differ"


@pytest.mark.parametrize("N,M,ks", [(9, 7, (1, 3, 7)), (257, 128, (16, 128)), (4099, 256, (1, 32, 128, 256)),
                                     (130, 300, (32,)), (515, 512, (64,)), (129, 768, (96,)), (259, 1024, (128,)),
                                     (35, 3000, (64,)), (70, 4096, (256,)), (9, 4095, (7,)), (100, 100, (12,)),
                                     (12, 8192, (100,)), (33, 63, (8,))])
def test_smallest_small_shapes(N, M, ks):
    R = _gpu()
    x = workloads.normal(N, M, seed=N * 37 + M)
    for k in ks:
        assert_smallest_parity(R, x, k, "exact", tag=f"smallest N={N} M={M} k={k}")
        for mi in (0, 2, 8, 30):
            assert_smallest_parity(R, x, k, "early", mi, tag=f"smallest N={N} M={M} k={k} mi={mi}")


@pytest.mark.parametrize("M", [8, 64, 256, 1024, 4096])
def test_smallest_tie_heavy_rows(M):
    R = _gpu()
    for x in (workloads.from_pool(300, M, 65 + M), workloads.small_ints(300, M, 66 + M, span=4)):
        for k in sorted({1, max(1, M // 8), M // 2, M}):
            assert_smallest_parity(R, x, k, "exact", tag=f"smallest ties M={M} k={k}")
            assert_smallest_parity(R, x, k, "early", 5, tag=f"smallest ties M={M} k={k}")


def test_config1_smallest_full_size():
    R = _gpu()
    x = workloads.make("c1_maxk")
    assert_smallest_parity(R, x, 32, "exact", tag="c1 smallest exact")
    assert_smallest_parity(R, x, 32, "early", 8, tag="c1 smallest early")


def test_empty_batch_and_error_codes_on_device():
    R = _gpu()
    x = torch.empty((0, 256), dtype=torch.float32, device="cuda")
    v, i = R.rtopk_rowwise_exact(x, 32)
    assert v.shape == (0, 32) and i.shape == (0, 32)
    y = torch.zeros((4, 8), dtype=torch.float32, device="cuda")
    with pytest.raises(R.RTopKError):
        R.rtopk_rowwise(y, 3, -1)
    with pytest.raises(R.RTopKError):
        R.rtopk_rowwise_eps(y, 3, -0.5)
    with pytest.raises(R.RTopKError):
        R.rtopk_rowwise_eps(y, 3, float("nan"))


def test_hip_graph_capture_and_replay():
    # One launch per call, no allocation, no memset: the entry points can be recorded into a HIP graph.
    # Replays are interleaved with eager work and checked every time.
    R = _gpu()
    N, M, k = 20000, 256, 32
    xs = [workloads.normal(N, M, seed=84 + i) for i in range(3)]
    xd = torch.from_numpy(xs[0]).cuda()
    ov = torch.empty((N, k), dtype=torch.float32, device="cuda")
    oi = torch.empty((N, k), dtype=torch.int32, device="cuda")
    sv = torch.empty((N, k), dtype=torch.float32, device="cuda")
    si = torch.empty((N, k), dtype=torch.int32, device="cuda")
    R.rtopk_rowwise_exact(xd, k, ov, oi)  # warm-up outside capture
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        R.rtopk_rowwise_exact(xd, k, ov, oi)
        R.rtopk_rowwise(xd, k, 6, sv, si)
    for x in xs + xs[:1]:
        xd.copy_(torch.from_numpy(x).cuda())
        ov.fill_(-1.0)
        oi.fill_(-1)
        si.fill_(-1)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        ev, ei = oracle.topk_exact(x, k)
        _, e2 = oracle.topk_earlystop(x, k, 6)
        assert np.array_equal(oi.cpu().numpy(), ei) and np.array_equal(bits(ov.cpu().numpy()), bits(ev))
        assert np.array_equal(si.cpu().numpy(), e2)


def test_other_stream():
    R = _gpu()
    x = workloads.normal(5000, 256, seed=83)
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        xd = torch.from_numpy(x).cuda()
        v, i = R.rtopk_rowwise_exact(xd, 32)
    s.synchronize()
    _, ei = oracle.topk_exact(x, 32)
    assert np.array_equal(i.cpu().numpy(), ei)


# ----------------------------------------------------------------------------------------------
# the five configurations at full size, in the launch configuration the benchmark times
# ----------------------------------------------------------------------------------------------
def _full(name, k, mode, max_iter=0):
    R = _gpu()
    cfg = workloads.CONFIGS[name]
    x = workloads.make(name)
    assert_parity(R, x, k, mode, max_iter, u8=(cfg["idx"] == "uint8"), tag=f"{name} k={k} {mode} {max_iter}")


def test_config0_small():
    _full("c0_small", 32, "exact")
    _full("c0_small", 32, "early", 8)


def test_config1_maxk_full_size():
    R = _gpu()
    x = workloads.make("c1_maxk")
    xd = torch.from_numpy(x).cuda()
    for k in (16, 32, 64, 128):
        gv, gi = run_gpu(R, x, k, "exact", x_dev=xd)
        ov, oi = oracle.topk_exact(x, k)
        assert np.array_equal(gi, oi), f"c1 exact k={k}"
        assert np.array_equal(bits(gv), bits(ov))
        for mi in (4, 8, 16):
            gv, gi = run_gpu(R, x, k, "early", mi, x_dev=xd)
            ov, oi = oracle.topk_earlystop(x, k, mi)
            assert np.array_equal(gi, oi), f"c1 early k={k} max_iter={mi}"
            assert np.array_equal(bits(gv), bits(ov))


@pytest.mark.parametrize("name", ["c2_w128", "c2_w512", "c2_w1024"])
def test_config2_width_sweep_full_size(name):
    _full(name, workloads.CONFIGS[name]["ks"][0], "exact")


def test_config3_ties_uint8_full_size():
    _full("c3_ties", 32, "exact")
    _full("c3_ties", 32, "early", 8)


def test_config4_wide_rows_full_size():
    _full("c4_wide", 64, "exact")
    _full("c4_wide", 256, "exact")


# ----------------------------------------------------------------------------------------------
# dense form (MaxK non-linearity): selected values in place, zero elsewhere
# ----------------------------------------------------------------------------------------------
def assert_dense_parity(R, x_np, k, max_iter, tag="", x_dev=None):
    xd = torch.from_numpy(x_np).cuda() if x_dev is None else x_dev
    g = R.rtopk_maxk_dense(xd, k, max_iter)
    torch.cuda.synchronize()
    o = oracle.maxk_dense(x_np, k, max_iter)
    g = g.cpu().numpy()
    if not np.array_equal(bits(g), bits(o)):
        bad = np.nonzero((bits(g) != bits(o)).any(axis=1))[0]
        r = int(bad[0])
        raise AssertionError(f"{tag} dense rows differ in {bad.size} rows; first row {r}: "
                             f"gpu cols {np.nonzero(g[r])[0]} oracle cols {np.nonzero(o[r])[0]}")


@pytest.mark.parametrize("N,M,ks", SHAPES)
def test_dense_small_shapes(N, M, ks):
    R = _gpu()
    x = workloads.normal(N, M, seed=N * 13 + M)
    xd = torch.from_numpy(x).cuda()
    for k in ks:
        for mi in (-1, 0, 3, 8, 40):
            assert_dense_parity(R, x, k, mi, tag=f"dense N={N} M={M} k={k} max_iter={mi}", x_dev=xd)


@pytest.mark.parametrize("M", [8, 64, 128, 256, 1024, 4096])
def test_dense_tie_heavy_rows(M):
    R = _gpu()
    for x in (workloads.from_pool(300, M, 75 + M), workloads.small_ints(300, M, 76 + M, span=4)):
        for k in sorted({1, max(1, M // 8), M // 2, M - 1, M}):
            for mi in (-1, 0, 5, 30):
                assert_dense_parity(R, x, k, mi, tag=f"dense ties M={M} k={k} mi={mi}")


def test_dense_unaligned_pointers_and_guard_bands():
    R = _gpu()
    N, M, k = 300, 256, 32
    x = workloads.normal(N, M, seed=86)
    pad = 1024
    ibuf = torch.empty(N * M + 1, dtype=torch.float32, device="cuda")
    xd = ibuf[1:].view(N, M)
    xd.copy_(torch.from_numpy(x))
    obuf = torch.full((N * M + 2 * pad + 1,), 777.0, dtype=torch.float32, device="cuda")
    od = obuf[pad + 1:pad + 1 + N * M].view(N, M)
    R.rtopk_maxk_dense(xd, k, -1, od)
    torch.cuda.synchronize()
    assert np.array_equal(bits(od.cpu().numpy()), bits(oracle.maxk_dense(x, k)))
    assert (obuf[:pad + 1] == 777.0).all() and (obuf[pad + 1 + N * M:] == 777.0).all()


def test_dense_headline_shape_full_size():
    R = _gpu()
    x = workloads.make("c1_maxk")
    xd = torch.from_numpy(x).cuda()
    assert_dense_parity(R, x, 32, -1, tag="c1 dense exact", x_dev=xd)
    assert_dense_parity(R, x, 32, 8, tag="c1 dense early", x_dev=xd)


# ----------------------------------------------------------------------------------------------
# rows wider than 8192 columns: one workgroup of 16 wavefronts per row
# ----------------------------------------------------------------------------------------------
WIDE = [(6, 8193, (1, 100)), (5, 8196, (64, 4000)), (7, 9000, (33, 512)), (4, 12288, (1, 1536)),
        (9, 16384, (64, 2048, 16383)), (3, 20000, (500,)), (3, 20001, (77,)), (4, 32768, (1, 4096)),
        (3, 40001, (999,)), (3, 49152, (6144,)), (5, 65536, (64, 8192, 65535, 65536)), (2, 65535, (31,))]


@pytest.mark.parametrize("N,M,ks", WIDE)
def test_very_wide_rows(N, M, ks):
    R = _gpu()
    x = workloads.normal(N, M, seed=N * 4099 + M)
    for k in ks:
        assert_parity(R, x, k, "exact", tag=f"wide N={N} M={M} k={k}")
        for mi in (0, 1, 6, 40):
            assert_parity(R, x, k, "early", mi, tag=f"wide N={N} M={M} k={k} max_iter={mi}")


@pytest.mark.parametrize("M", [8200, 16384, 30000, 65536])
def test_very_wide_tie_heavy_rows(M):
    R = _gpu()
    for x in (workloads.from_pool(12, M, 95 + M), workloads.small_ints(12, M, 96 + M, span=20),
              workloads.normal_ties(12, M, 97 + M, p=0.5)):
        for k in (1, 64, 1000, M // 2, M - 1, M):
            assert_parity(R, x, k, "exact", tag=f"wide ties M={M} k={k}")
            for mi in (0, 5, 30):
                assert_parity(R, x, k, "early", mi, tag=f"wide ties M={M} k={k} mi={mi}")


def test_very_wide_rows_many_rows_and_unaligned_input():
    R = _gpu()
    N, M, k = 3000, 16384, 256
    x = workloads.laplace(N, M, seed=98)
    assert_parity(R, x, k, "exact", tag="wide many rows")
    # 4-byte aligned input takes the scalar-load variant
    buf = torch.empty(64 * M + 1, dtype=torch.float32, device="cuda")
    xd = buf[1:].view(64, M)
    xd.copy_(torch.from_numpy(x[:64]))
    v, i = R.rtopk_rowwise_exact(xd, k)
    torch.cuda.synchronize()
    ev, ei = oracle.topk_exact(x[:64], k)
    assert np.array_equal(i.cpu().numpy(), ei) and np.array_equal(bits(v.cpu().numpy()), bits(ev))


def test_more_than_2_to_31_elements():
    # 64-bit addressing: 2^22 + 5 rows of 512 columns is just over 2^31 input elements (8 GiB)
    R = _gpu()
    N, M, k = (1 << 22) + 5, 512, 64
    x = workloads.uniform(N, M, seed=99)
    xd = torch.from_numpy(x).cuda()
    gv, gi = R.rtopk_rowwise_exact(xd, k)
    torch.cuda.synchronize()
    ov, oi = oracle.topk_exact(x, k)
    assert np.array_equal(gi.cpu().numpy(), oi)
    assert np.array_equal(bits(gv.cpu().numpy()), bits(ov))
    del gv, gi
    d = R.rtopk_maxk_dense(xd, k, 6)
    torch.cuda.synchronize()
    sv, si = oracle.topk_earlystop(x, k, 6)
    tail = slice(N - 4096, N)  # the rows whose addresses lie beyond 2^31 elements
    dt = d[tail].cpu().numpy()
    ref = np.zeros_like(dt)
    rows = np.arange(4096)[:, None]
    ref[rows, si[tail]] = x[tail][rows, si[tail]]
    assert np.array_equal(bits(dt), bits(ref))


def test_nonfinite_inputs_terminate_and_stay_in_bounds_in_every_variant():
    # NaN / infinities are outside the contract; every entry point must still return and write only
    # inside its outputs (guard bands around every output buffer are checked)
    R = _gpu()
    pad = 2048

    def guarded(n, dtype, fill):
        buf = torch.full((n + 2 * pad,), fill, dtype=dtype, device="cuda")
        return buf, buf[pad:pad + n]

    def check(buf, fill):
        assert (buf[:pad] == fill).all() and (buf[-pad:] == fill).all()

    for N, M, k in ((500, 256, 32), (40, 4096, 64), (6, 20000, 300)):
        x = workloads.normal(N, M, seed=87 + M)
        x[::3, 1] = np.inf
        x[1::3, M // 2] = -np.inf
        x[2::3, M - 1] = np.nan
        x[0] = np.nan
        xd = torch.from_numpy(x).cuda()
        vb, ov = guarded(N * k, torch.float32, 4321.0)
        ib, oi = guarded(N * k, torch.int32, -9)
        calls = [lambda: R.rtopk_rowwise_exact(xd, k, ov.view(N, k), oi.view(N, k)),
                 lambda: R.rtopk_rowwise(xd, k, 9, ov.view(N, k), oi.view(N, k))]
        calls += [lambda: R.rtopk_rowwise_exact_smallest(xd, k, ov.view(N, k), oi.view(N, k)),
                  lambda: R.rtopk_rowwise_eps(xd, k, 1e-3, ov.view(N, k), oi.view(N, k))]
        for call in calls:
            call()
            torch.cuda.synchronize()
            check(vb, 4321.0)
            check(ib, -9)
        db, od = guarded(N * M, torch.float32, 4321.0)
        for mi in (-1, 7):
            R.rtopk_maxk_dense(xd, k, mi, od.view(N, M))
            torch.cuda.synchronize()
            check(db, 4321.0)
        for dt in (torch.float16, torch.bfloat16):
            x16 = xd.to(dt)
            hb, oh = guarded(N * k, dt, 7.0)
            name = "f16" if dt == torch.float16 else "bf16"
            getattr(R, f"rtopk_rowwise_exact_{name}")(x16, k, oh.view(N, k), oi.view(N, k))
            getattr(R, f"rtopk_rowwise_{name}")(x16, k, 9, oh.view(N, k), oi.view(N, k))
            torch.cuda.synchronize()
            check(hb, 7.0)
            check(ib, -9)


def test_hip_graph_replay_of_the_other_entry_points():
    # dense, 16-bit and wide-row calls are single launches too: capture once, replay on fresh inputs
    R = _gpu()
    N, M, k = 3000, 256, 32
    xs = [workloads.normal(N, M, seed=120 + i) for i in range(2)]
    ws = [workloads.normal(16, 12288, seed=130 + i) for i in range(2)]
    xd = torch.from_numpy(xs[0]).cuda()
    wd = torch.from_numpy(ws[0]).cuda()
    hd = xd.to(torch.bfloat16)
    dense = torch.empty_like(xd)
    hv = torch.empty((N, k), dtype=torch.bfloat16, device="cuda")
    hi = torch.empty((N, k), dtype=torch.int32, device="cuda")
    wv = torch.empty((16, 100), dtype=torch.float32, device="cuda")
    wi = torch.empty((16, 100), dtype=torch.int32, device="cuda")
    R.rtopk_maxk_dense(xd, k, -1, dense)
    R.rtopk_rowwise_exact_bf16(hd, k, hv, hi)
    R.rtopk_rowwise_exact(wd, 100, wv, wi)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        R.rtopk_maxk_dense(xd, k, -1, dense)
        R.rtopk_rowwise_exact_bf16(hd, k, hv, hi)
        R.rtopk_rowwise_exact(wd, 100, wv, wi)
    for x, w in list(zip(xs, ws)) + [(xs[0], ws[0])]:
        xd.copy_(torch.from_numpy(x).cuda())
        wd.copy_(torch.from_numpy(w).cuda())
        hd.copy_(xd.to(torch.bfloat16))
        dense.fill_(-1.0)
        hi.fill_(-1)
        wi.fill_(-1)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert np.array_equal(bits(dense.cpu().numpy()), bits(oracle.maxk_dense(x, k)))
        b16 = workloads.to_bits16(x, "bf16")
        ev, ei = oracle.topk_exact_16(b16, "bf16", k)
        assert np.array_equal(hi.cpu().numpy(), ei)
        assert np.array_equal(hv.view(torch.int16).cpu().numpy().view(np.uint16), ev)
        _, wei = oracle.topk_exact(w, 100)
        assert np.array_equal(wi.cpu().numpy(), wei)


def test_randomised_shapes_modes_and_entry_points():
    # 300 seeded draws of (N, M, k, mode, entry point, value distribution): every load path, ragged
    # widths, every output form, each compared with the oracle bit for bit
    R = _gpu()
    rng = np.random.Generator(np.random.Philox(20240901))
    widths = [1, 2, 3, 31, 64, 65, 127, 128, 129, 255, 256, 257, 384, 500, 512, 640, 768, 1000, 1024, 1028, 1536, 2047,
              2048, 2500, 3072, 4096, 5000, 6144, 7777, 8192, 8200, 10000, 16384, 24576, 33000]
    for it in range(300):
        M = int(widths[rng.integers(len(widths))]) if rng.random() < 0.7 else int(rng.integers(1, 9000))
        N = int(rng.integers(1, 40 if M > 2048 else 300))
        k = int(rng.integers(1, M + 1)) if rng.random() < 0.5 else int(max(1, min(M, rng.integers(1, 65))))
        gen = rng.integers(4)
        seed = int(rng.integers(1 << 30))
        if gen == 0:
            x = workloads.normal(N, M, seed)
        elif gen == 1:
            x = workloads.normal_ties(N, M, seed, p=0.3)
        elif gen == 2:
            x = workloads.small_ints(N, M, seed, span=int(rng.integers(1, 30)))
        else:
            x = workloads.laplace(N, M, seed)
        mi = int(rng.integers(0, 20))
        kinds = ["exact", "early", "smallest_exact", "smallest_early", "eps", "dense_exact", "dense_early", "f16", "bf16"]
        if M <= 256:
            kinds += ["u8_exact", "u8_early"]
        kind = kinds[rng.integers(len(kinds))]
        tag = f"draw {it}: N={N} M={M} k={k} {kind} max_iter={mi} gen={gen} seed={seed}"
        if kind == "exact":
            assert_parity(R, x, k, "exact", tag=tag)
        elif kind == "early":
            assert_parity(R, x, k, "early", mi, tag=tag)
        elif kind == "u8_exact":
            assert_parity(R, x, k, "exact", u8=True, tag=tag)
        elif kind == "u8_early":
            assert_parity(R, x, k, "early", mi, u8=True, tag=tag)
        elif kind == "smallest_exact":
            assert_smallest_parity(R, x, k, "exact", tag=tag)
        elif kind == "smallest_early":
            assert_smallest_parity(R, x, k, "early", mi, tag=tag)
        elif kind == "eps":
            assert_eps_parity(R, x, k, float(10.0 ** -rng.integers(1, 8)), tag=tag)
        elif kind == "dense_exact":
            assert_dense_parity(R, x, k, -1, tag=tag)
        elif kind == "dense_early":
            assert_dense_parity(R, x, k, mi, tag=tag)
        else:
            b = workloads.to_bits16(x, kind)
            xd = torch.from_numpy(b.view(np.int16)).cuda().view(torch.float16 if kind == "f16" else torch.bfloat16)
            exact = rng.random() < 0.5
            if exact:
                gv, gi = getattr(R, f"rtopk_rowwise_exact_{kind}")(xd, k)
                ov, oi = oracle.topk_exact_16(b, kind, k)
            else:
                gv, gi = getattr(R, f"rtopk_rowwise_{kind}")(xd, k, mi)
                ov, oi = oracle.topk_earlystop_16(b, kind, k, mi)
            torch.cuda.synchronize()
            assert np.array_equal(gi.cpu().numpy(), oi), tag
            assert np.array_equal(gv.view(torch.int16).cpu().numpy().view(np.uint16), ov), tag


def test_exit_iteration_statistics_of_table5_on_the_gpu():
    # Table 5 (Appendix A) reproduced from the kernel's own iteration output at epsilon = 0, including
    # the closed form of Eq. 4 sitting slightly above the measured mean, for rows up to 8192 wide
    from conftest import read_table

    R = _gpu()
    header, rows = read_table("table5_exit_cumulative.txt")
    cols = [tuple(int(a) for a in h.split("_")) for h in header[1:]]
    for col, (M, k) in enumerate(cols):
        x = workloads.normal(10000, M, seed=3000 + col)
        _, _, it = R.rtopk_rowwise_eps(torch.from_numpy(x).cuda(), k, 0.0, want_iters=True)
        it = it.cpu().numpy()
        for row in rows:
            paper = float(row[1 + col])
            if row[0] == "avg":
                assert abs(float(it.mean()) - paper) < 0.12, (M, k, it.mean(), paper)
            elif row[0] == "En":
                assert 0.0 < paper - float(it.mean()) < 0.6, (M, k)
            else:
                assert abs(float((it <= int(row[0])).mean() * 100.0) - paper) < 2.6, (M, k, row[0])


@pytest.mark.parametrize("N,M,ks", [(5, 8196, (64, 4000)), (4, 9001, (33,)), (6, 16384, (1, 2048)), (3, 20000, (500,)),
                                     (3, 32768, (4096,)), (3, 40001, (999,)), (4, 65536, (64, 65535, 65536))])
def test_very_wide_rows_every_variant(N, M, ks):
    # the k smallest, the precision-bounded mode, the dense form and 16-bit rows beyond 8192 columns
    R = _gpu()
    for x in (workloads.normal(N, M, seed=N * 5003 + M), workloads.normal_ties(N, M, seed=N * 5009 + M, p=0.5)):
        xd = torch.from_numpy(x).cuda()
        for k in ks:
            tag = f"wide variants N={N} M={M} k={k}"
            assert_smallest_parity(R, x, k, "exact", tag=tag)
            assert_smallest_parity(R, x, k, "early", 7, tag=tag)
            for eps in (0.0, 1e-4, 0.05):
                assert_eps_parity(R, x, k, eps, tag=tag)
            assert_dense_parity(R, x, k, -1, tag=tag, x_dev=xd)
            assert_dense_parity(R, x, k, 6, tag=tag, x_dev=xd)
            for kind in ("f16", "bf16"):
                b = workloads.to_bits16(x, kind)
                hd = torch.from_numpy(b.view(np.int16)).cuda().view(torch.float16 if kind == "f16" else torch.bfloat16)
                for mode, mi in (("exact", 0), ("early", 6)):
                    if mode == "exact":
                        gv, gi = getattr(R, f"rtopk_rowwise_exact_{kind}")(hd, k)
                        ov, oi = oracle.topk_exact_16(b, kind, k)
                    else:
                        gv, gi = getattr(R, f"rtopk_rowwise_{kind}")(hd, k, mi)
                        ov, oi = oracle.topk_earlystop_16(b, kind, k, mi)
                    torch.cuda.synchronize()
                    assert np.array_equal(gi.cpu().numpy(), oi), f"{tag} {kind} {mode}"
                    assert np.array_equal(gv.view(torch.int16).cpu().numpy().view(np.uint16), ov), f"{tag} {kind} {mode}"


@pytest.mark.parametrize("N,M,k", [(32768 + 5, 256, 32), (32768 + 13, 128, 16), (32768 + 3, 200, 25), (40001, 64, 8)])
def test_many_rows_with_a_ragged_last_wavefront(N, M, k):
    # from 32768 rows on, narrow rows go 8 or 16 to a wavefront; the last wavefront holds fewer
    R = _gpu()
    x = workloads.normal_ties(N, M, seed=N + M, p=0.1)
    assert_parity(R, x, k, "exact", tag=f"N={N} M={M}")
    assert_parity(R, x, k, "early", 6, tag=f"N={N} M={M}")
    assert_parity(R, x, k, "exact", u8=True, tag=f"u8 N={N} M={M}")
    assert_dense_parity(R, x, k, -1, tag=f"dense N={N} M={M}")
    assert_smallest_parity(R, x, k, "exact", tag=f"smallest N={N} M={M}")


def test_results_do_not_depend_on_the_run_or_on_what_the_outputs_held():
    # no atomics on the outputs, no dependence on launch order: repeated calls give identical bytes,
    # whatever the output buffers contained before
    R = _gpu()
    for N, M, k in ((50000, 256, 32), (3000, 4096, 64), (12, 40000, 700)):
        x = torch.from_numpy(workloads.normal_ties(N, M, seed=N + 7, p=0.2)).cuda()
        v0, i0 = R.rtopk_rowwise_exact(x, k)
        d0 = R.rtopk_maxk_dense(x, k, 5)
        torch.cuda.synchronize()
        for fill in (0.0, float("nan")):
            v = torch.full_like(v0, fill)
            i = torch.full_like(i0, -1)
            d = torch.full_like(d0, fill)
            R.rtopk_rowwise_exact(x, k, v, i)
            R.rtopk_maxk_dense(x, k, 5, d)
            torch.cuda.synchronize()
            assert torch.equal(i, i0) and torch.equal(v.view(torch.int32), v0.view(torch.int32))
            assert torch.equal(d.view(torch.int32), d0.view(torch.int32))


def test_huge_max_iter_means_no_early_stop_and_terminates():
    # max_iter above 512 runs as 512 (further steps cannot move a bound: shown on the CPU in
    # test_alg2_is_a_fixed_point_after_at_most_512_steps), so INT32_MAX is a legal way to say "no early
    # stop" even on rows whose k-th place is tied and never count exactly k.
    R = _gpu()
    big = 2 ** 31 - 1
    for x, ks in ((workloads.from_pool(2000, 24, seed=1400), (1, 3, 12)), (workloads.normal_ties(3000, 256, seed=1402, p=0.5), (32,)),
                  (workloads.small_ints(50, 4096, seed=1404, span=3), (100,)), (workloads.small_ints(6, 20000, seed=1405, span=3), (500,))):
        for k in ks:
            ov, oi = oracle.topk_earlystop(x, k, 600)
            gv, gi = run_gpu(R, x, k, "early", big)
            assert np.array_equal(gi, oi) and np.array_equal(bits(gv), bits(ov)), (x.shape, k)
    x = workloads.normal_ties(3000, 256, seed=1406, p=0.5)
    xd = torch.from_numpy(x).cuda()
    d = R.rtopk_maxk_dense(xd, 32, big)
    gv, gi = R.rtopk_rowwise_u8(xd, 32, big)
    sv, si = R.rtopk_rowwise_smallest(xd, 32, big)
    torch.cuda.synchronize()
    assert np.array_equal(bits(d.cpu().numpy()), bits(oracle.maxk_dense(x, 32, 600)))
    assert np.array_equal(gi.cpu().numpy().astype(np.int32), oracle.topk_earlystop(x, 32, 600)[1])
    assert np.array_equal(si.cpu().numpy(), oracle.topk_earlystop_smallest(x, 32, 600)[1])


def test_width_768_full_size():
    # the third width of the paper's sweep (Section 4.1, Table 3): 2^18 x 768, k = 96
    R = _gpu()
    x = workloads.normal(1 << 18, 768, seed=768)
    assert_parity(R, x, 96, "exact", tag="768 exact")
    assert_parity(R, x, 96, "early", 8, tag="768 max_iter=8")


def test_config4_eps_mode_full_size():
    R = _gpu()
    x = workloads.make("c4_wide")
    assert_eps_parity(R, x, 64, 1e-4, tag="c4 eps=1e-4")


@pytest.mark.parametrize("name,ks", [("x_wide8k", (256,)), ("x_wide32k", (256, 2048)), ("x_wide64k", (512,)),
                                     ("x_stream256k", (512,))])
def test_workgroup_per_row_bench_workloads_full_size(name, ks):
    # the workloads the widest one-wavefront shape and the workgroup-per-row kernels (row in registers, row
    # streamed) are timed on, at the size that is timed
    R = _gpu()
    x = workloads.make(name)
    for k in ks:
        assert_parity(R, x, k, "exact", tag=f"{name} k={k} exact")
        assert_parity(R, x, k, "early", 8, tag=f"{name} k={k} max_iter=8")


@pytest.mark.parametrize("N", [1, 100, 4097, 32767])
def test_few_rows_take_the_two_rows_per_wavefront_shape_in_every_variant(N):
    # fewer than 32768 narrow rows: uint8 columns, the k smallest, the precision-bounded mode, 16-bit rows
    # and the dense form all run the 2-rows-per-wavefront instances
    R = _gpu()
    for M, k in ((256, 32), (128, 16), (200, 25)):
        x = workloads.normal_ties(N, M, seed=N + M, p=0.2)
        assert_parity(R, x, k, "exact", u8=True, tag=f"u8 N={N} M={M}")
        assert_parity(R, x, k, "early", 6, u8=True, tag=f"u8 N={N} M={M}")
        assert_smallest_parity(R, x, k, "exact", tag=f"smallest N={N} M={M}")
        assert_smallest_parity(R, x, k, "early", 6, tag=f"smallest N={N} M={M}")
        assert_eps_parity(R, x, k, 1e-3, tag=f"eps N={N} M={M}")
        xd = torch.from_numpy(x).cuda()
        d = R.rtopk_maxk_dense(xd, k)
        torch.cuda.synchronize()
        assert np.array_equal(bits(d.cpu().numpy()), bits(oracle.maxk_dense(x, k)))
        for kind, tdt in (("f16", torch.float16), ("bf16", torch.bfloat16)):
            b16 = workloads.to_bits16(x, kind)
            x16 = torch.from_numpy(b16.view(np.int16)).cuda().view(tdt)
            gv, gi = getattr(R, "rtopk_rowwise_exact_" + kind)(x16, k)
            torch.cuda.synchronize()
            ov, oi = oracle.topk_exact_16(b16, kind, k)
            assert np.array_equal(gi.cpu().numpy(), oi) and np.array_equal(gv.view(torch.int16).cpu().numpy().view(np.uint16), ov)
