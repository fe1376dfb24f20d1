"""GPU parity of batchnorm2d_fwd / batchnorm2d_bwd against the CPU oracle, through the C ABI.

Bounds (fp32 tensors; each is 1e-5 times the sum of the absolute values of the terms the result is made of, the
same rule as for the convolution passes).  With s = inv_std, m = mean of channel c and M = N*H*W:
  y        |gpu - ref| <= 1e-5 * (|gamma| (|x| + |m|) s + |beta|)
  mean     |gpu - ref| <= 1e-5 * sum |x| / M
  inv_std  |gpu - ref| <= 1e-5 * s
  dbeta    |gpu - ref| <= 1e-5 * sum |dy|
  dgamma   |gpu - ref| <= 1e-5 * sum |dy| (|x| + |m|) s
  dx       |gpu - ref| <= 1e-5 * |gamma| s (|dy| + sum |dy| / M + (|x| + |m|) s * sum |dy| (|x| + |m|) s / M)
The backward call is fed the oracle's statistics rounded to fp32 (never the GPU forward's), so each call is
checked on its own; one test also chains the two GPU calls.
"""
import numpy as np
import pytest

from oracle import convref as ref
from paper_1912_01703_amd import workloads as wl

pytestmark = pytest.mark.gpu
TOL = 1e-5
EPS = 1e-5

SHAPES = [
    # name      N    C    H    W
    ("bn14", 64, 256, 14, 14),       # a channel fits the registers of a 512-thread workgroup
    ("bn112", 64, 64, 112, 112),     # 98 chunks per channel: partial statistics, merge, apply
    ("bn1", 1, 1, 1, 1),             # a single element: variance 0, y = beta
    ("bn7", 2, 3, 7, 7),             # planes not a multiple of four floats: 4-byte units
    ("bn9x13", 3, 5, 9, 13),
    ("bn7n70", 70, 8, 7, 7),         # 3430 four-byte units: 512 threads x 8
    ("bn7n600", 600, 2, 7, 7),       # 29 400 four-byte units: the split kernels with 4-byte units
    ("bn56", 4, 16, 56, 56),         # 3136 units of 16 bytes
    ("bn56n16", 16, 4, 56, 56),      # 12 544 units: seven chunks, the last one ragged
    ("bn30", 5, 3, 30, 30),
    ("bn4", 2, 2, 4, 4),
    ("bn28", 40, 7, 28, 28),         # 7840 units: 1024 threads x 8
]


def bounds(x, dy, gamma, beta, mean, inv_std):
    """The denominators of the module docstring, float64."""
    x, dy = x.astype(np.float64), dy.astype(np.float64)
    g, b = np.abs(gamma.astype(np.float64))[None, :, None, None], np.abs(beta.astype(np.float64))[None, :, None, None]
    m, s = np.abs(mean)[None, :, None, None], inv_std[None, :, None, None]
    M = x.shape[0] * x.shape[2] * x.shape[3]
    ax = (np.abs(x) + m) * s
    ady = np.abs(dy)
    sum_dy = ady.sum(axis=(0, 2, 3))
    sum_dyx = (ady * ax).sum(axis=(0, 2, 3))
    return dict(y=g * ax + b, mean=np.abs(x).sum(axis=(0, 2, 3)) / M, inv_std=inv_std.copy(), dbeta=sum_dy, dgamma=sum_dyx,
                dx=g * s * (ady + sum_dy[None, :, None, None] / M + ax * sum_dyx[None, :, None, None] / M))


def worst(got, want, den):
    got = np.asarray(got, dtype=np.float64)
    assert np.all(np.isfinite(got))
    live = den > 0
    assert np.all(got[~live] == want[~live])
    return float(np.max(np.abs(got[live] - want[live]) / den[live])) if live.any() else 0.0


def run_case(name, N, C, H, W, seed, offset=0, shift=0.0, eps=EPS):
    import torch
    from paper_1912_01703_amd import binding as mc
    x, dy, gamma, beta = wl.make_bn_inputs(N, C, H, W, seed)
    if shift:
        x = (x + np.float32(shift)).astype(np.float32)
    y_ref, mean_ref, inv_ref = ref.batchnorm2d_fwd(x, gamma, beta, eps)
    dx_ref, dg_ref, db_ref = ref.batchnorm2d_bwd(x, dy, gamma, eps)
    den = bounds(x, dy, gamma, beta, mean_ref, inv_ref)
    dev = "cuda:0"

    def up(a):   # offset > 0: a tensor that starts `offset` floats into its allocation (not 16-byte aligned)
        flat = torch.empty(a.size + offset, dtype=torch.float32, device=dev)
        flat[offset:].copy_(torch.from_numpy(a.reshape(-1)))
        return flat[offset:].view(a.shape)

    xd, dyd, gd, bd = up(x), up(dy), up(gamma), up(beta)
    nan = lambda shape: up(np.full(shape, np.nan, dtype=np.float32))
    y, dx = nan(x.shape), nan(x.shape)
    mean, inv_std, dgamma, dbeta = nan((C,)), nan((C,)), nan((C,)), nan((C,))
    need = max(mc.batchnorm2d_workspace_bytes(p, N, C, H, W) for p in (0, 1))
    ws = torch.empty(max(need, 256), dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream().cuda_stream
    print(f"[batchnorm] case={name} N={N} C={C} H={H} W={W} offset={offset} workspace={need}", flush=True)
    mc.batchnorm2d_fwd(xd, gd, bd, y, mean, inv_std, N, C, H, W, eps, mc.F32, ws, stream)
    stats = (up(mean_ref.astype(np.float32)), up(inv_ref.astype(np.float32)))
    mc.batchnorm2d_bwd(xd, dyd, gd, stats[0], stats[1], dx, dgamma, dbeta, N, C, H, W, mc.F32, ws, stream)
    torch.cuda.synchronize()
    errs = dict(y=worst(y.cpu().numpy(), y_ref, den["y"]), mean=worst(mean.cpu().numpy(), mean_ref, den["mean"]),
                inv_std=worst(inv_std.cpu().numpy(), inv_ref, den["inv_std"]),
                dbeta=worst(dbeta.cpu().numpy(), db_ref, den["dbeta"]), dgamma=worst(dgamma.cpu().numpy(), dg_ref, den["dgamma"]),
                dx=worst(dx.cpu().numpy(), dx_ref, den["dx"]))
    for k, e in errs.items():
        assert e <= TOL, f"{name}: {k} normalised error {e:.3e}"
    assert np.array_equal(xd.cpu().numpy(), x) and np.array_equal(dyd.cpu().numpy(), dy)     # inputs untouched
    return errs


@pytest.mark.parametrize("row", SHAPES, ids=[r[0] for r in SHAPES])
def test_batchnorm_shapes(row):
    name, N, C, H, W = row
    run_case(name, N, C, H, W, seed=9000 + SHAPES.index(row))


@pytest.mark.parametrize("row", [("bn14u", 8, 16, 14, 14), ("bn56u", 16, 4, 56, 56)], ids=["resident", "split"])
def test_batchnorm_unaligned_tensors_take_the_four_byte_path(row):
    name, N, C, H, W = row
    run_case(name, N, C, H, W, seed=9100, offset=1)


@pytest.mark.parametrize("row", [("bn14m", 64, 32, 14, 14), ("bn56m", 16, 4, 56, 56)], ids=["resident", "split"])
def test_batchnorm_with_a_mean_far_from_zero(row):
    """Channels whose mean is a thousand standard deviations away from zero: the variance must come from the centred
    values (a sum of squares minus the squared mean would lose all its digits in fp32)."""
    name, N, C, H, W = row
    run_case(name, N, C, H, W, seed=9400, shift=1000.0)


def test_batchnorm_without_eps():
    run_case("bn0", 8, 16, 14, 14, seed=9410, eps=0.0)


def test_batchnorm_forward_statistics_feed_the_backward_call():
    """The two GPU calls chained as a framework would chain them, on the benchmark's small shape."""
    import torch
    from paper_1912_01703_amd import binding as mc
    N, C, H, W = 64, 256, 14, 14
    x, dy, gamma, beta = wl.make_bn_inputs(N, C, H, W, 9200)
    dx_ref, dg_ref, db_ref = ref.batchnorm2d_bwd(x, dy, gamma, EPS)
    _, mean_ref, inv_ref = ref.batchnorm2d_fwd(x, gamma, beta, EPS)
    den = bounds(x, dy, gamma, beta, mean_ref, inv_ref)
    t = lambda a: torch.from_numpy(a).to("cuda:0")
    xd, dyd, gd, bd = t(x), t(dy), t(gamma), t(beta)
    y, dx = torch.empty_like(xd), torch.empty_like(xd)
    mean, inv_std, dgamma, dbeta = (torch.empty(C, device="cuda:0") for _ in range(4))
    mc.batchnorm2d_fwd(xd, gd, bd, y, mean, inv_std, N, C, H, W, EPS)
    mc.batchnorm2d_bwd(xd, dyd, gd, mean, inv_std, dx, dgamma, dbeta, N, C, H, W)
    torch.cuda.synchronize()
    assert worst(dx.cpu().numpy(), dx_ref, den["dx"]) <= TOL
    assert worst(dgamma.cpu().numpy(), dg_ref, den["dgamma"]) <= TOL
    assert worst(dbeta.cpu().numpy(), db_ref, den["dbeta"]) <= TOL


def test_batchnorm_is_bit_reproducible():
    import torch
    from paper_1912_01703_amd import binding as mc
    N, C, H, W = 16, 4, 56, 56          # the split kernels
    x, dy, gamma, beta = wl.make_bn_inputs(N, C, H, W, 9300)
    t = lambda a: torch.from_numpy(a).to("cuda:0")
    xd, gd, bd = t(x), t(gamma), t(beta)
    ws = torch.empty(max(256, mc.batchnorm2d_workspace_bytes(0, N, C, H, W)), dtype=torch.uint8, device="cuda:0")
    outs = []
    for _ in range(2):
        y, mean, inv_std = torch.empty_like(xd), torch.empty(C, device="cuda:0"), torch.empty(C, device="cuda:0")
        mc.batchnorm2d_fwd(xd, gd, bd, y, mean, inv_std, N, C, H, W, EPS, mc.F32, ws)
        torch.cuda.synchronize()
        outs.append((y, mean, inv_std))
    for u, v in zip(*outs):
        assert torch.equal(u, v)


def test_batchnorm_rejects_bad_arguments():
    import torch
    from paper_1912_01703_amd import binding as mc
    t = torch.zeros(256, device="cuda:0")
    assert mc.batchnorm2d_fwd(t, t, t, t, t, t, 0, 1, 2, 2, EPS, check=False) == mc.ERR_SHAPE
    assert mc.batchnorm2d_fwd(t, t, t, t, t, t, 1, 1, 2, 2, -1.0, check=False) == mc.ERR_SHAPE
    assert mc.batchnorm2d_fwd(t, t, t, t, t, t, 1, 1, 2, 2, EPS, mc.BF16_F32ACC, check=False) == mc.ERR_DTYPE
    assert mc.batchnorm2d_fwd(None, t, t, t, t, t, 1, 1, 2, 2, EPS, check=False) == mc.ERR_NULL
    assert mc.batchnorm2d_bwd(t, t, t, t, t, t, t, None, 1, 1, 2, 2, check=False) == mc.ERR_NULL
    assert mc.batchnorm2d_fwd(t, t, t, t, t, t, 600, 2, 7, 7, EPS, check=False) == mc.ERR_WORKSPACE   # split path, no workspace
    assert "workspace" in mc.last_error()
