"""GPU parity for rows stored as float16 / bfloat16: the HIP path (through the C ABI) against the CPU
oracle.  Bar: columns bit-exact, values bit-exact 16-bit copies of the input, in both modes."""
import numpy as np
import pytest

import oracle
import workloads

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

KINDS = ("f16", "bf16")
TORCH_DT = {"f16": torch.float16, "bf16": torch.bfloat16}


def _gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2409_00822_amd as R

    R.load_library()
    return R


def to_dev(bits16, kind):
    return torch.from_numpy(bits16.view(np.int16)).cuda().view(TORCH_DT[kind])


def from_dev(t):
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def assert_parity16(R, b, kind, k, mode, max_iter=0, tag="", x_dev=None):
    xd = to_dev(b, kind) if x_dev is None else x_dev
    if mode == "exact":
        gv, gi = getattr(R, f"rtopk_rowwise_exact_{kind}")(xd, k)
        ov, oi = oracle.topk_exact_16(b, kind, k)
    else:
        gv, gi = getattr(R, f"rtopk_rowwise_{kind}")(xd, k, max_iter)
        ov, oi = oracle.topk_earlystop_16(b, kind, k, max_iter)
    torch.cuda.synchronize()
    gi = gi.cpu().numpy()
    if not np.array_equal(gi, oi):
        bad = np.nonzero((gi != oi).any(axis=1))[0]
        r = int(bad[0])
        raise AssertionError(f"{tag} index mismatch in {bad.size} rows; first row {r}: gpu {gi[r]} oracle {oi[r]}")
    assert np.array_equal(from_dev(gv), ov), f"{tag} value bits differ"


SHAPES = [
    (1, 1, (1,)), (9, 7, (1, 3, 7)), (33, 63, (8, 63)), (64, 64, (5, 64)), (65, 65, (3,)), (100, 100, (10, 12)),
    (257, 128, (16, 20, 128)), (31, 130, (13,)), (77, 200, (25, 32)), (4099, 256, (1, 16, 31, 32, 64, 128, 256)),
    (50, 260, (33, 64)), (130, 264, (32,)), (515, 512, (64, 100)), (129, 768, (96,)), (40, 1000, (125, 128)),
    (259, 1024, (128, 1000)), (33, 1504, (200,)), (67, 2048, (256,)), (35, 3000, (64,)), (70, 4096, (64, 256, 1024)),
    (9, 4095, (7, 512)), (17, 1021, (17,)), (21, 6000, (300,)), (20, 8192, (64, 512, 4097)), (5, 8191, (8,)),
]


@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("N,M,ks", SHAPES)
def test_16bit_small_shapes(kind, N, M, ks):
    R = _gpu()
    b = workloads.to_bits16(workloads.normal(N, M, seed=N * 7919 + M + 5), kind)
    xd = to_dev(b, kind)
    for k in ks:
        assert_parity16(R, b, kind, k, "exact", tag=f"{kind} N={N} M={M} k={k}", x_dev=xd)
        for mi in (0, 1, 4, 8, 40):
            assert_parity16(R, b, kind, k, "early", mi, tag=f"{kind} N={N} M={M} k={k} max_iter={mi}", x_dev=xd)


@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("M", [8, 64, 128, 256, 512, 1024, 4096])
def test_16bit_tie_heavy_rows(kind, M):
    R = _gpu()
    # a pool of values that both types represent exactly, incl. signed zeros, their smallest subnormals
    # and neighbouring values around 1
    pool = {"f16": np.array([0x0000, 0x8000, 0x3C00, 0x3C01, 0x3BFF, 0xBC00, 0x0001, 0x8001, 0x7BFF, 0xFBFF, 0x4200],
                            dtype=np.uint16),
            "bf16": np.array([0x0000, 0x8000, 0x3F80, 0x3F81, 0x3F7F, 0xBF80, 0x0001, 0x8001, 0x7E7F, 0xFE7F, 0x4040],
                             dtype=np.uint16)}[kind]
    rng = np.random.Generator(np.random.Philox(300 + M))
    rows = []
    for _ in range(300):
        sub = rng.choice(pool, size=int(rng.integers(1, 6)), replace=False)
        rows.append(rng.choice(sub, size=M, replace=True))
    b = np.stack(rows)
    xd = to_dev(b, kind)
    for k in sorted({1, max(1, M // 8), M // 2, M - 1, M}):
        assert_parity16(R, b, kind, k, "exact", tag=f"{kind} pool M={M} k={k}", x_dev=xd)
        for mi in (0, 3, 30):
            assert_parity16(R, b, kind, k, "early", mi, tag=f"{kind} pool M={M} k={k} mi={mi}", x_dev=xd)


@pytest.mark.parametrize("kind", KINDS)
def test_16bit_unaligned_pointers_and_odd_k(kind):
    R = _gpu()
    N, M, k = 300, 256, 30
    b = workloads.to_bits16(workloads.normal(N, M, seed=85), kind)
    buf = torch.empty(N * M + 1, dtype=TORCH_DT[kind], device="cuda")
    xd = buf[1:].view(N, M)  # 2-byte aligned only
    xd.copy_(to_dev(b, kind))
    ob = torch.empty(N * k + 1, dtype=TORCH_DT[kind], device="cuda")
    ov = ob[1:].view(N, k)
    oi = torch.empty((N, k), dtype=torch.int32, device="cuda")
    getattr(R, f"rtopk_rowwise_exact_{kind}")(xd, k, ov, oi)
    torch.cuda.synchronize()
    ev, ei = oracle.topk_exact_16(b, kind, k)
    assert np.array_equal(oi.cpu().numpy(), ei) and np.array_equal(from_dev(ov.contiguous()), ev)


@pytest.mark.parametrize("kind", KINDS)
def test_16bit_headline_shape_full_size(kind):
    # the MaxK-GNN hidden-layer workload stored in 16 bits, in the launch configuration the benchmark times
    R = _gpu()
    b = workloads.to_bits16(workloads.make("c1_maxk"), kind)
    xd = to_dev(b, kind)
    assert_parity16(R, b, kind, 32, "exact", tag=f"c1 {kind} exact", x_dev=xd)
    assert_parity16(R, b, kind, 32, "early", 8, tag=f"c1 {kind} early", x_dev=xd)


@pytest.mark.parametrize("kind,name,k", [("bf16", "c2_w512", 64), ("f16", "c2_w1024", 128), ("bf16", "c4_wide", 256)])
def test_16bit_wider_configs_full_size(kind, name, k):
    R = _gpu()
    b = workloads.to_bits16(workloads.make(name), kind)
    assert_parity16(R, b, kind, k, "exact", tag=f"{name} {kind} exact")
