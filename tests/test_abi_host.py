"""Host-only checks of the C ABI: the library loads, exports every symbol the
header declares, and rejects invalid arguments before launching anything."""
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "miconv.h")


@pytest.fixture(scope="module")
def mc():
    from paper_1912_01703_amd import binding
    return binding


def declared_symbols():
    text = "\n".join(l for l in open(HEADER).read().splitlines() if not l.startswith("#define"))
    return re.findall(r"MICONV_API\s+[\w\s\*]*?\b(\w+)\s*\(", text)


def test_header_declares_the_three_passes():
    names = declared_symbols()
    for required in ("conv2d_fwd", "conv2d_bwd_data", "conv2d_bwd_weight", "conv2d_workspace_bytes"):
        assert required in names


def test_library_exports_every_declared_symbol(mc):
    for name in declared_symbols():
        assert hasattr(mc._lib, name), name


GOOD = dict(N=1, C=4, H=8, W=8, K=4, R=3, S=3, stride_h=1, stride_w=1, pad_h=1, pad_w=1, groups=1)


def call(mc, fn, ptrs=(0, 0, 0), dtype=0, **over):
    a = dict(GOOD)
    a.update(over)
    return fn(ptrs[0] or None, ptrs[1] or None, ptrs[2] or None, *a.values(), dtype, None, 0, check=False)


@pytest.mark.parametrize("fname", ["conv2d_fwd", "conv2d_bwd_data", "conv2d_bwd_weight"])
def test_invalid_arguments_are_rejected_without_launch(mc, fname):
    fn = getattr(mc, fname)
    assert call(mc, fn, N=0) == mc.ERR_SHAPE
    assert call(mc, fn, R=0) == mc.ERR_SHAPE
    assert call(mc, fn, stride_h=0) == mc.ERR_SHAPE
    assert call(mc, fn, pad_w=-1) == mc.ERR_SHAPE
    assert call(mc, fn, H=2, pad_h=0) == mc.ERR_SHAPE          # filter larger than the padded input
    assert "larger" in mc.last_error()
    assert call(mc, fn, groups=3) == mc.ERR_GROUPS
    assert call(mc, fn, groups=0) == mc.ERR_GROUPS
    assert call(mc, fn, dtype=7) == mc.ERR_DTYPE
    assert call(mc, fn, N=1 << 20, C=1 << 10, H=64, W=64) == mc.ERR_SHAPE   # >= 2^31 elements
    assert call(mc, fn) == mc.ERR_NULL                          # valid shape, NULL tensors
    assert "NULL" in mc.last_error()
    assert call(mc, fn, ptrs=(256, 0, 256)) == mc.ERR_NULL
    assert call(mc, fn, ptrs=(256, 256, 0)) == mc.ERR_NULL


def test_raises_with_message(mc):
    with pytest.raises(mc.MiconvError) as ei:
        mc.conv2d_fwd(None, None, None, 1, 3, 8, 8, 4, 3, 3, 1, 1, 1, 1, 2)
    assert ei.value.code == mc.ERR_GROUPS and "groups" in str(ei.value)


def test_algo_override_codes(mc):
    assert mc.miconv_set_algo(0, 99) == mc.ERR_DTYPE
    assert mc.miconv_set_algo(5, 0) == mc.ERR_DTYPE
    assert mc.miconv_set_algo(0, mc.ALGO_DIRECT) == mc.OK
    assert mc.conv2d_workspace_bytes(0, *GOOD.values()) == 0    # direct kernels need no workspace
    assert mc.miconv_set_algo(0, mc.ALGO_DEPTHWISE) == mc.OK
    assert call(mc, mc.conv2d_fwd, ptrs=(256, 256, 256)) == mc.ERR_UNSUPPORTED   # dense problem, depthwise forced
    assert mc.miconv_set_algo(0, mc.ALGO_AUTO) == mc.OK
    assert mc.miconv_last_algo(0) == mc.ALGO_AUTO               # nothing has run on this thread


def test_workspace_query_is_zero_for_invalid_arguments(mc):
    bad = dict(GOOD, groups=3)
    assert mc.conv2d_workspace_bytes(2, *bad.values()) == 0
    assert mc.conv2d_workspace_bytes(9, *GOOD.values()) == 0


def test_workspace_sizes_of_the_benchmark_layers(mc):
    """Host arithmetic only: which passes of which layers need scratch memory, and how much."""
    from paper_1912_01703_amd import workloads as wl
    L = wl.LAYERS
    # layer 2a backward-weight: 256 workgroups without a split, nothing to reduce
    assert mc.conv2d_workspace_bytes(2, *L["2a"].conv_args(), mc.F32) == 0
    # depthwise: the image ranges of a channel pair are the eight waves of one workgroup and are summed there
    assert mc.conv2d_workspace_bytes(2, *L["5a"].conv_args(), mc.F32) == 0
    for p in (0, 1):
        assert mc.conv2d_workspace_bytes(p, *L["4b"].conv_args(), mc.F32) == 0
    # a split reduction holds one partial dw per split
    ws = mc.conv2d_workspace_bytes(2, *L["2b"].conv_args(), mc.F32)
    dw_bytes = 4 * L["2b"].K * L["2b"].C
    assert ws > 0 and ws % dw_bytes == 0
    # bf16 inputs on the bf16 matrix cores: a channels-innermost copy of the source and the packed filters
    l4 = L["4b"]
    need = l4.N * l4.H * l4.W * l4.C * 2 + 9 * l4.K * l4.C * 2
    got = mc.conv2d_workspace_bytes(0, *l4.conv_args(), mc.BF16_F32ACC)
    assert need <= got <= need + 512
    # ... and for backward-weight images-innermost copies of x and dy (N is a multiple of 8 here) plus the partials
    got2 = mc.conv2d_workspace_bytes(2, *l4.conv_args(), mc.BF16_F32ACC)
    assert got2 >= 2 * l4.N * l4.C * l4.H * l4.W * 2
    # with few channels backward-weight transposes its operands on the way into LDS: only partial sums
    l4a = L["4a"]
    got3 = mc.conv2d_workspace_bytes(2, *l4a.conv_args(), mc.BF16_F32ACC)
    assert 0 < got3 and got3 % (4 * 9 * l4a.K * l4a.C) == 0
    # few channels on wide planes: forward and backward-data read the NCHW source in place, only the packed filters are scratch
    for p in (0, 1):
        assert mc.conv2d_workspace_bytes(p, *l4a.conv_args(), mc.BF16_F32ACC) == 9 * l4a.K * l4a.C * 2
    # 14x14 planes with bf16 inputs: the bf16 matrix cores too (a channels-innermost copy of x and the packed filters)
    l2a = L["2a"]
    assert mc.miconv_kernel_path(0, *l2a.conv_args(), mc.BF16_F32ACC) == "mfma/bf16_tile"
    got4 = mc.conv2d_workspace_bytes(0, *l2a.conv_args(), mc.BF16_F32ACC)
    need4 = l2a.N * l2a.H * l2a.W * l2a.C * 2 + 9 * l2a.K * l2a.C * 2
    assert need4 <= got4 <= need4 + 512
    # planes of an odd number of pixels: bf16 inputs take the fp32 matrix cores on widened values, no layout copies
    assert mc.conv2d_workspace_bytes(0, 4, 64, 7, 7, 64, 3, 3, 1, 1, 1, 1, 1, mc.BF16_F32ACC) == 0


def test_kernel_path_of_the_benchmark_layers(mc):
    """Host arithmetic only: which kernel family each benchmark layer is dispatched to."""
    from paper_1912_01703_amd import workloads as wl
    L = wl.LAYERS
    path = lambda name, p, dt=mc.F32: mc.miconv_kernel_path(p, *L[name].conv_args(), dt)
    for name in ("1", "2a", "2b", "4a", "4b", "5b"):
        assert [path(name, p) for p in range(3)] == ["mfma/tile", "mfma/tile", "mfma/wgrad"], name
    assert [path("2c", p) for p in range(3)] == ["mfma/tile", "mfma/tile_merge2", "mfma/wgrad"]
    assert [path("3", p) for p in range(3)] == ["mfma/smallc"] * 3
    assert [path("5a", p) for p in range(3)] == ["depthwise/strip"] * 3
    for name in ("4a", "4b"):
        assert [path(name, p, mc.BF16_F32ACC) for p in range(3)] == ["mfma/bf16_tile", "mfma/bf16_tile", "mfma/bf16_wgrad"]
    assert mc.miconv_kernel_path(0, 1, 4, 8, 8, 4, 3, 3, 1, 1, 1, 1, 3) == "none"      # invalid groups
    assert mc.miconv_kernel_path(0, 1, 4, 9, 9, 4, 5, 4, 3, 2, 1, 1, 1) == "direct"    # no tuned kernel


# Depthwise problems around the sizes at which individual kernel families bow out (tensors of 2 GiB and more,
# millions of planes, planes too large for LDS): whatever the dispatcher accepts must have a kernel to run on.
DW_LIMITS = [
    # N     C    H    W  stride pad
    (512, 512, 56, 56, 1, 1),       # 3.3 GB of fp32: beyond the 32-bit byte offsets of the strip and row kernels
    (680, 512, 56, 56, 1, 1),       # just under 2^31 elements
    (512, 512, 56, 56, 2, 1),
    (40000, 128, 8, 8, 1, 1),       # 5.1 M planes: beyond the exact range of the strip kernels' channel decode
    (65536, 96, 7, 7, 1, 1),
    (2, 8, 300, 300, 1, 1),         # a plane larger than any LDS budget
    (1, 16, 4000, 4000, 1, 1),
    (3, 16, 2000, 3000, 2, 1),
]


@pytest.mark.parametrize("dtype", [0, 1])
@pytest.mark.parametrize("row", DW_LIMITS, ids=["x".join(map(str, r)) for r in DW_LIMITS])
def test_accepted_depthwise_problems_have_a_kernel(mc, row, dtype):
    N, C, H, W, st, pd = row
    args = (N, C, H, W, C, 3, 3, st, st, pd, pd, C)
    for p in range(3):
        auto = mc.miconv_kernel_path(p, *args, dtype)
        assert auto != "none", (p, row)
        assert mc.miconv_set_algo(p, mc.ALGO_DEPTHWISE) == mc.OK
        try:
            forced = mc.miconv_kernel_path(p, *args, dtype)
        finally:
            mc.miconv_set_algo(p, mc.ALGO_AUTO)
        # AUTO picks the depthwise family exactly when the family says it can run the problem
        assert (forced != "none") == auto.startswith("depthwise/"), (p, row, auto, forced)


def test_backward_weight_declines_stages_beyond_32_bit_offsets(mc):
    """N=2, C=512, 1024x1024 fp32: four images' channels exceed 2 GiB, so the matrix-core backward-weight
    kernel (32-bit offsets within a stage) must not be chosen; the direct kernels take the problem."""
    args = (2, 512, 1024, 1024, 1, 3, 3, 1, 1, 1, 1, 1)
    assert mc.miconv_kernel_path(2, *args, mc.F32) == "direct"
    assert mc.miconv_kernel_path(2, 2, 512, 64, 64, 64, 3, 3, 1, 1, 1, 1, 1, mc.F32) == "mfma/wgrad"


def test_algorithm_override_is_per_thread(mc):
    import threading
    seen = {}
    assert mc.miconv_set_algo(0, mc.ALGO_DIRECT) == mc.OK
    try:
        t = threading.Thread(target=lambda: seen.update(other=mc.miconv_kernel_path(0, *GOOD.values(), 0)))
        t.start()
        t.join()
        seen["mine"] = mc.miconv_kernel_path(0, *GOOD.values(), 0)
    finally:
        mc.miconv_set_algo(0, mc.ALGO_AUTO)
    assert seen == {"other": "mfma/tile", "mine": "direct"}
