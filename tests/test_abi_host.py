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
    # 14x14 planes are not a multiple of 8 elements: bf16 inputs take the widening path, no layout copies
    assert mc.conv2d_workspace_bytes(0, *L["2a"].conv_args(), mc.BF16_F32ACC) == 0
