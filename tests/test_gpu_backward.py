"""GPU parity of the backward edge of the MaxK non-linearity (scatter and gather forms) against the CPU
oracle, element by element; the values are bit copies, so the tolerance is 0."""
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


def check(R, N, M, k, seed, u8=False, idx=None, tag=""):
    x = workloads.normal(N, M, seed)
    if idx is None:
        _, idx = oracle.topk_exact(x, k)
    g = workloads.normal(N, k, seed + 1)
    w = workloads.normal(N, M, seed + 2)
    idx_d = torch.from_numpy(idx.astype(np.uint8) if u8 else idx).cuda()
    dense = R.rtopk_maxk_backward(torch.from_numpy(g).cuda(), idx_d, M)
    gath = R.rtopk_maxk_backward_gather(torch.from_numpy(w).cuda(), idx_d)
    torch.cuda.synchronize()
    assert np.array_equal(bits(dense.cpu().numpy()), bits(oracle.maxk_backward(g, idx, M))), f"{tag} scatter"
    assert np.array_equal(bits(gath.cpu().numpy()), bits(oracle.maxk_backward_gather(w, idx))), f"{tag} gather"


SHAPES = [(1, 1, (1,)), (5, 2, (1, 2)), (9, 7, (1, 3, 7)), (33, 63, (1, 8, 63)), (64, 64, (1, 5, 16, 64)),
          (100, 100, (10, 12)), (257, 128, (1, 16, 20, 128)), (31, 130, (13,)), (77, 200, (25, 32)),
          (4099, 256, (1, 16, 31, 32, 33, 64, 65, 128, 255, 256)), (50, 260, (33, 64)), (515, 512, (64, 100)),
          (129, 768, (96,)), (40, 1000, (125, 128)), (259, 1024, (128, 1000)), (33, 1500, (200,)), (67, 2048, (256, 2048)),
          (35, 3000, (64,)), (70, 4096, (64, 1024)), (9, 4095, (7, 512)), (20, 8192, (64, 4097)), (7, 10001, (33, 9000)),
          (5, 32768, (256,)), (3, 65536, (512, 65536))]


@pytest.mark.parametrize("N,M,ks", SHAPES)
def test_backward_small_shapes(N, M, ks):
    R = _gpu()
    for k in ks:
        check(R, N, M, k, seed=N * 13 + M + k, tag=f"N={N} M={M} k={k}")
        if M <= 256:
            check(R, N, M, k, seed=N * 17 + M + k, u8=True, tag=f"u8 N={N} M={M} k={k}")


def test_backward_columns_in_any_order_and_out_of_range_columns():
    R = _gpu()
    N, M, k = 3000, 256, 32
    rng = np.random.Generator(np.random.Philox(5))
    idx = np.stack([rng.permutation(M)[:k] for _ in range(N)]).astype(np.int32)  # distinct, unsorted
    check(R, N, M, k, seed=41, idx=idx, tag="unsorted")
    bad = idx.copy()
    bad[::3, 5] = -1
    bad[::5, 7] = M
    bad[::7, 0] = 2 ** 31 - 1
    bad[::11, 31] = -(2 ** 31)
    check(R, N, M, k, seed=43, idx=bad, tag="out-of-range columns")
    # wide rows (workgroup per row) too
    idx = np.stack([rng.permutation(9000)[:100] for _ in range(40)]).astype(np.int32)
    idx[::2, 3] = 9000
    idx[::3, 4] = -5
    check(R, 40, 9000, 100, seed=45, idx=idx, tag="wide, out-of-range columns")


def test_backward_unaligned_pointers_and_guard_bands():
    R = _gpu()
    N, M, k = 777, 256, 32
    x = workloads.normal(N, M, seed=51)
    _, idx = oracle.topk_exact(x, k)
    g = workloads.normal(N, k, seed=52)
    pad = 1024
    buf = torch.full((N * M + 2 * pad + 1,), 7.5, dtype=torch.float32, device="cuda")
    out = buf[pad + 1:pad + 1 + N * M].view(N, M)  # 4-byte aligned only: the scalar store path
    R.rtopk_maxk_backward(torch.from_numpy(g).cuda(), torch.from_numpy(idx).cuda(), M, out)
    torch.cuda.synchronize()
    assert np.array_equal(bits(out.cpu().numpy()), bits(oracle.maxk_backward(g, idx, M)))
    assert (buf[:pad + 1] == 7.5).all() and (buf[pad + 1 + N * M:] == 7.5).all()
    w = workloads.normal(N, M, seed=53)
    wb = torch.empty(N * M + 1, dtype=torch.float32, device="cuda")
    wd = wb[1:].view(N, M)
    wd.copy_(torch.from_numpy(w))
    gbuf = torch.full((N * k + 2 * pad,), 7.5, dtype=torch.float32, device="cuda")
    gv = gbuf[pad:pad + N * k].view(N, k)
    R.rtopk_maxk_backward_gather(wd, torch.from_numpy(idx).cuda(), gv)
    torch.cuda.synchronize()
    assert np.array_equal(bits(gv.cpu().numpy()), bits(oracle.maxk_backward_gather(w, idx)))
    assert (gbuf[:pad] == 7.5).all() and (gbuf[pad + N * k:] == 7.5).all()


def test_backward_round_trip_with_the_forward_pass_full_size():
    # the headline shape, with the columns the forward kernel itself saved (int32 and uint8)
    R = _gpu()
    x = workloads.make("c1_maxk")
    N, M, k = x.shape[0], x.shape[1], 32
    xd = torch.from_numpy(x).cuda()
    for u8 in (False, True):
        vals, idx = (R.rtopk_rowwise_exact_u8 if u8 else R.rtopk_rowwise_exact)(xd, k)
        g = workloads.normal(N, k, seed=61)
        dense = R.rtopk_maxk_backward(torch.from_numpy(g).cuda(), idx, M)
        torch.cuda.synchronize()
        idx_h = idx.cpu().numpy().astype(np.int32)
        assert np.array_equal(bits(dense.cpu().numpy()), bits(oracle.maxk_backward(g, idx_h, M))), f"scatter u8={u8}"
        del dense
        # gathering the forward input at the saved columns returns the forward values
        back = R.rtopk_maxk_backward_gather(xd, idx)
        torch.cuda.synchronize()
        assert torch.equal(back.view(torch.int32), vals.view(torch.int32)), f"gather u8={u8}"
        w = workloads.normal(N, M, seed=62)
        gath = R.rtopk_maxk_backward_gather(torch.from_numpy(w).cuda(), idx)
        torch.cuda.synchronize()
        assert np.array_equal(bits(gath.cpu().numpy()), bits(oracle.maxk_backward_gather(w, idx_h))), f"gather u8={u8}"


def test_backward_empty_batch_and_errors():
    R = _gpu()
    g = torch.empty((0, 32), dtype=torch.float32, device="cuda")
    i = torch.empty((0, 32), dtype=torch.int32, device="cuda")
    assert R.rtopk_maxk_backward(g, i, 256).shape == (0, 256)
    g = torch.zeros((4, 8), dtype=torch.float32, device="cuda")
    i = torch.zeros((4, 8), dtype=torch.int32, device="cuda")
    with pytest.raises(R.RTopKError):
        R.rtopk_maxk_backward(g, i, 4)  # k > M
    with pytest.raises(ValueError):
        R.rtopk_maxk_backward(g, torch.zeros((4, 8), dtype=torch.uint8, device="cuda"), 300)
