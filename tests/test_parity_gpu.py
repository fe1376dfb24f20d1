"""GPU parity: every pass through the C ABI against the CPU oracle.

Full tensors for the layers the oracle finishes in seconds.  The two VGG-sized
layers are checked in full for backward-weight and, for forward and
backward-data, on whole images, whole tiles at the structurally delicate places
of the tuned kernels' work decomposition and a seeded random sample.  Bounds
and the error measure are in parity_util.
"""
import numpy as np
import pytest

from paper_1912_01703_amd import workloads as wl

import parity_util as pu

pytestmark = pytest.mark.gpu

ODD = [
    # name   N  C   H   W   K  R  S  stride   pad    groups
    ("odd0", 2, 3, 7, 6, 4, 3, 3, (1, 1), (1, 1), 1),
    ("odd1", 1, 4, 9, 8, 6, 3, 2, (2, 1), (0, 1), 2),
    ("odd2", 2, 6, 8, 11, 6, 1, 3, (1, 3), (0, 2), 3),
    ("odd3", 1, 2, 12, 12, 2, 5, 5, (2, 2), (2, 2), 2),
    ("odd4", 2, 3, 13, 9, 5, 4, 3, (3, 2), (1, 0), 1),
    ("odd5", 1, 8, 6, 6, 8, 3, 3, (1, 1), (1, 1), 8),
    ("odd6", 3, 20, 17, 19, 36, 3, 3, (1, 1), (1, 1), 4),
    ("odd7", 2, 5, 8, 8, 7, 3, 3, (3, 3), (0, 0), 1),     # rows/cols past the last window: dx == 0 there
    ("odd8", 1, 2, 10, 7, 4, 3, 3, (1, 1), (3, 2), 1),    # padding wider than the filter reach
    ("odd9", 5, 1, 1, 1, 3, 1, 1, (1, 1), (0, 0), 1),     # single pixel
]


def odd_layer(row, seed_off=0):
    name, N, C, H, W, K, R, S, st, pd, g = row
    return wl.custom_layer(name, N, C, H, W, K, R, S, st, pd, g, seed=1000 + seed_off)


def test_tiny_config_auto():
    from paper_1912_01703_amd import binding as mc
    errs = pu.check_layer_full(wl.LAYERS["1"], expect_algo=mc.ALGO_MFMA)
    assert set(errs) == set(pu.PASSES)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("row", ODD, ids=[r[0] for r in ODD])
def test_odd_shapes_direct(row, dtype):
    from paper_1912_01703_amd import binding as mc
    pu.check_layer_full(odd_layer(row, ODD.index(row)), dtype, algo=mc.ALGO_DIRECT, expect_algo=mc.ALGO_DIRECT)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("row", ODD, ids=[r[0] for r in ODD])
def test_odd_shapes_auto(row, dtype):
    pu.check_layer_full(odd_layer(row, ODD.index(row)), dtype)


MFMA = [
    # name     N   C   H   W   K  R  S  stride  pad   groups
    ("m3x3a", 2, 32, 14, 14, 64, 3, 3, 1, 1, 1),
    ("m3x3b", 3, 16, 17, 19, 40, 3, 3, 1, 1, 1),      # ragged tiles, K not a multiple of 16
    ("m3x3c", 2, 32, 9, 30, 24, 3, 3, 1, 0, 1),       # no padding
    ("m3x3d", 1, 48, 15, 15, 16, 3, 3, 1, 2, 1),      # padding 2: backward-data sees pad' = 0
    ("m3x3g", 2, 64, 14, 14, 96, 3, 3, 1, 1, 2),      # two groups
    ("m1x1a", 2, 48, 14, 14, 80, 1, 1, 1, 0, 1),
    ("m1x1b", 1, 128, 7, 29, 33, 1, 1, 1, 0, 1),
    ("m3x3t", 2, 3, 20, 20, 10, 3, 3, 1, 1, 1),       # reduction channels not a multiple of the chunk
    ("m3x3u", 2, 21, 14, 14, 35, 3, 3, 1, 1, 1),
    ("m1x1c", 3, 200, 14, 14, 136, 1, 1, 1, 0, 1),    # several 128-wide blocks with ragged edges
    ("m1x1d", 2, 72, 20, 28, 40, 1, 1, 1, 0, 1),      # few filters: 64-wide blocks in backward-weight, two of them along C;
                                                      # 28 pixels wide: bands of 8 full rows, the last one ragged
    ("m1x1e", 1, 72, 9, 56, 40, 1, 1, 1, 0, 1),       # 56 wide: bands of 4 rows, three chunks
    ("m1x1i", 1, 24, 14, 112, 40, 1, 1, 1, 0, 1),     # 112 wide: handled as a plane of 28 x 56 pixels
    ("m1x1j", 2, 72, 8, 21, 136, 1, 1, 1, 0, 1),      # 168 pixels = 3 x 56
    ("m1x1g", 2, 136, 10, 28, 200, 1, 1, 1, 0, 1),    # 28 wide, many channels: backward-weight stages of two full rows
    ("m1x1h", 1, 72, 7, 56, 136, 1, 1, 1, 0, 1),      # 56 wide, many channels: stages of one row
    ("m1x1f", 2, 16, 5, 112, 24, 1, 1, 1, 0, 1),      # 112 wide: bands of 2 rows, a partial chunk
    ("m3x3n", 9, 16, 14, 14, 16, 3, 3, 1, 1, 1),      # more images than one split holds
    ("m3x3p", 5, 16, 210, 210, 24, 3, 3, 1, 1, 1),    # > 1024 work items of one chunk: persistent workgroups
    ("m3x3q", 3, 40, 200, 206, 72, 3, 3, 1, 1, 1),    # ... with two filter blocks, three chunks, ragged tiles
    ("m3x3w", 9, 16, 100, 208, 24, 3, 3, 1, 1, 1),    # > 1024 items, width a multiple of 16: 12 x 16 tiles, last tile row ragged
    ("m3x3s2", 2, 32, 28, 28, 32, 3, 3, 2, 1, 1),     # stride 2: backward-data runs once per output phase
    ("m3x3s2b", 1, 16, 31, 27, 20, 3, 3, 2, 1, 1),    # odd sizes: phases of different extent
    ("m3x3s2c", 2, 16, 16, 16, 24, 3, 3, 2, 0, 1),    # no padding: the last input row/column feeds nothing
    ("m3x3s2g", 1, 32, 14, 14, 32, 3, 3, 2, 1, 2),
    ("m3x3s2d", 2, 24, 57, 60, 40, 3, 3, 2, 1, 1),    # merged-phase backward-data over several ragged tiles
    ("m3x3s2e", 50, 16, 28, 28, 128, 3, 3, 2, 1, 1),  # forward on 7 x 14 half tiles (14 x 14 tiles would leave CUs idle)
    ("m3x3s2f", 56, 8, 26, 25, 72, 3, 3, 2, 1, 1),    # ... ragged: 13 x 13 outputs, a partial second filter block
    ("m3x3s2h", 2, 64, 28, 28, 16, 3, 3, 2, 1, 1),    # backward-data: 64 destination channels on 7 x 14 grid tiles
    ("m3x3s2i", 1, 128, 27, 31, 8, 3, 3, 2, 1, 1),    # ... odd plane, two channel blocks, three ragged grid tiles
    ("m3x3z", 5, 40, 7, 7, 72, 3, 3, 1, 1, 1),        # 7 x 7 planes: tiles of 7 x 7 pixels
    ("m1x1z", 6, 72, 7, 7, 136, 1, 1, 1, 0, 1),
    ("m3x3y", 3, 24, 6, 5, 24, 3, 3, 1, 1, 1),        # ... smaller than the tile
    ("m1x1s2", 3, 40, 28, 28, 72, 1, 1, 2, 0, 1),     # 1x1 stride 2: three of four dx phases receive nothing
    ("m1x1s2b", 2, 136, 15, 19, 24, 1, 1, 2, 0, 1),   # ... odd sizes, more than one 128-channel block
    ("m1x1s2c", 2, 136, 15, 19, 136, 1, 1, 2, 0, 1),  # ... more than 128 channels on both sides: 128 x 128 blocks in backward-weight,
                                                      # 128 filters per workgroup forward
    ("m1x1s2d", 128, 512, 28, 28, 8, 1, 1, 2, 0, 1),  # ... backward-data with 1024 work items: 128 destination channels per workgroup
    # 128 filters (destination channels) per workgroup where the layer has them and the grid stays large enough
    ("m1x1w", 128, 16, 14, 14, 512, 1, 1, 1, 0, 1),   # 1x1 on 14 x 14 planes, forward
    ("m1x1v", 103, 640, 14, 14, 8, 1, 1, 1, 0, 1),    # ... backward-data, five blocks of 128 channels
    ("m1x1y", 3, 136, 7, 7, 40, 1, 1, 1, 0, 1),       # 7 x 7 planes, backward-data, partial second block
    ("m1x1k", 1, 16, 4, 112, 136, 1, 1, 1, 0, 1),     # row bands of a 112-wide plane
    ("m3x3x", 3, 136, 7, 7, 136, 3, 3, 1, 1, 1),      # 3x3 on 7 x 7 planes, both directions
    ("m3x3v", 64, 8, 14, 14, 512, 3, 3, 1, 1, 1),     # 3x3 on 14 x 14 tiles, forward
    ("m3x3v2", 64, 512, 14, 14, 8, 3, 3, 1, 1, 1),    # ... backward-data
    ("m3x3v3", 7, 8, 96, 112, 136, 3, 3, 1, 1, 1),    # ... persistent workgroups on 12 x 16 tiles
    # backward-weight with 32 x 32 channel blocks (enough stages per workgroup)
    ("m3x3wg", 128, 256, 14, 14, 256, 3, 3, 1, 1, 1), # 64 blocks, split four ways
    ("m3x3wh", 228, 64, 30, 30, 64, 3, 3, 1, 1, 1),   # four blocks, nine tiles per image, the outer ones ragged
]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("row", MFMA, ids=[r[0] for r in MFMA])
def test_mfma_shapes(row, dtype):
    from paper_1912_01703_amd import binding as mc
    name, N, C, H, W, K, R, S, st, pd, g = row
    L = wl.custom_layer(name, N, C, H, W, K, R, S, st, pd, g, seed=2000 + MFMA.index(row))
    pu.check_layer_full(L, dtype, algo=mc.ALGO_MFMA, expect_algo=mc.ALGO_MFMA)


BF16MM = [
    # name     N   C    H   W   K   pad    3x3 stride 1, bf16: forward (C % 32 == 0, H*W even) and/or
    #                                      backward-data (K % 32 == 0, P*Q even) run on the bf16 matrix cores
    ("b3x3a", 2, 32, 16, 16, 64, 1),
    ("b3x3b", 3, 64, 20, 18, 48, 1),       # 48 filters: partial filter block; backward-data takes the widened path
    ("b3x3c", 1, 96, 30, 28, 96, 0),       # no padding; backward-data sees pad' = 2
    ("b3x3d", 2, 32, 12, 24, 32, 2),       # padding 2
    ("b3x3e", 1, 160, 28, 28, 128, 1),     # five chunks, four tiles, two filter blocks
    ("b3x3f", 5, 32, 8, 8, 16, 1),         # one partial tile, one partial filter block
    ("b3x3g", 2, 32, 8, 17, 32, 1),        # odd output width: the write-out stores single pixels
    ("b3x3w", 1, 32, 100, 48, 64, 1),      # wide plane: 12 x 16 tiles, the last tile row ragged
    ("b3x3h", 2, 64, 14, 14, 64, 1),       # planes of an even number of pixels that is no multiple of 8: the last group of eight
    ("b3x3i", 3, 32, 9, 6, 32, 1),         # pixels the pre-pass loads runs into the next plane
    # wide planes with at most 128 reduction channels: the kernel reads the NCHW source itself (no copy)
    ("b3x3n", 2, 64, 100, 50, 32, 0),      # no padding: groups of four pixels start at the patch's first column; 98 x 48 outputs
    ("b3x3o", 1, 128, 96, 46, 64, 2),      # padding 2, four chunks, the last tile row ragged (98 rows)
    ("b3x3p", 2, 32, 120, 64, 96, 1),      # four tiles side by side: image borders left and right, interior tiles between
]


@pytest.mark.parametrize("row", BF16MM, ids=[r[0] for r in BF16MM])
def test_bf16_matrix_core_path(row):
    from paper_1912_01703_amd import binding as mc
    name, N, C, H, W, K, pd = row
    L = wl.custom_layer(name, N, C, H, W, K, 3, 3, 1, pd, 1, seed=6000 + BF16MM.index(row))
    # the layout pre-passes of that path are what needs a workspace in a forward pass
    assert mc.conv2d_workspace_bytes(0, *L.conv_args(), mc.BF16_F32ACC) > 0
    pu.check_layer_full(L, "bf16", passes=("fwd", "bwd_data"), algo=mc.ALGO_MFMA, expect_algo=mc.ALGO_MFMA)


BF16WG = [
    # name     N   C    H   W   K   pad    3x3 stride 1, bf16, N*P*Q >= 4096, Q % 4 == 0 and W even (few channels) or planes % 8 == 0:
    #                                      backward-weight on the bf16 matrix cores (rows streamed through LDS)
    ("w3x3a", 16, 32, 16, 16, 64, 1),
    ("w3x3b", 9, 40, 32, 32, 72, 1),       # N not a multiple of 8, partial channel blocks, two strips
    ("w3x3c", 8, 32, 30, 28, 64, 0),       # no padding
    ("w3x3d", 8, 16, 24, 24, 16, 2),       # padding 2
    ("w3x3e", 3, 64, 120, 40, 64, 1),      # three row segments
    # many channels: x and dy are rewritten images-innermost by a pre-pass instead of inside the kernel
    ("w3x3f", 16, 128, 16, 16, 128, 1),
    ("w3x3g", 9, 136, 24, 32, 120, 1),     # N not a multiple of 8, partial channel blocks, two strips
    ("w3x3h", 8, 128, 24, 30, 128, 0),     # no padding
    ("w3x3i", 8, 128, 24, 26, 128, 2),     # padding 2, width not a multiple of 4
    ("w3x3j", 16, 128, 14, 14, 128, 1),    # planes of 196 pixels: the pre-pass's last group of eight runs into the next plane
    ("w3x3k", 9, 136, 10, 13, 120, 1),     # 130 pixels, N not a multiple of 8, partial channel blocks
]


@pytest.mark.parametrize("row", BF16WG, ids=[r[0] for r in BF16WG])
def test_bf16_matrix_core_bwd_weight(row):
    from paper_1912_01703_amd import binding as mc
    name, N, C, H, W, K, pd = row
    L = wl.custom_layer(name, N, C, H, W, K, 3, 3, 1, pd, 1, seed=6100 + BF16WG.index(row))
    pu.check_layer_full(L, "bf16", passes=("bwd_weight",), algo=mc.ALGO_MFMA, expect_algo=mc.ALGO_MFMA)


@pytest.mark.parametrize("shape", [(2, 64, 14, 14, 64), (1, 32, 100, 48, 64), (16, 128, 16, 16, 128)],
                         ids=["copy", "nchw-in-place", "wgrad-prepass"])
def test_bf16_tensors_that_start_on_an_odd_element(shape):
    """The bf16 matrix-core kernels load 4 bytes and more at a time; tensors that are only 2-byte aligned are served by
    the kernels that take any alignment, within the workspace the query reported."""
    import torch
    from paper_1912_01703_amd import binding as mc
    N, C, H, W, K = shape
    L = wl.custom_layer("odd-start", N, C, H, W, K, 3, 3, 1, 1, 1, seed=6200)
    h = pu.prepare(L, "bf16")
    gr = pu.GpuRunner(L, h, "bf16")

    def shifted(t):
        flat = torch.empty(t.numel() + 1, dtype=t.dtype, device=t.device)
        flat[1:].copy_(t.reshape(-1))
        return flat[1:].view(t.shape)

    gr.x, gr.w, gr.dy = shifted(gr.x), shifted(gr.w), shifted(gr.dy)
    assert gr.x.data_ptr() % 4 == 2
    for p in pu.PASSES:
        out = gr.run(p).cpu().numpy()
        refv, den = pu.oracle_full(L, h, p)
        err, ok = pu.max_norm_err(out, refv, den)
        assert ok and err <= pu.TOL["bf16"], (p, err)


BF16GEMM = [
    # name      N    C    H   W    K      1x1, stride 1, bf16: all three passes as matrix products on the bf16 matrix cores
    ("g1x1a", 16, 64, 14, 14, 128),      # one 128 x 128 tile column, 25 pixel tiles, two chunks
    ("g1x1b", 6, 200, 14, 14, 136),      # partial tiles in every dimension, a partial last chunk (200 = 3 * 64 + 8)
    ("g1x1c", 16, 72, 20, 28, 40),       # fewer filters than a tile
    ("g1x1d", 4, 256, 9, 6, 520),        # planes of 54 pixels: backward-weight rows end inside a 16-byte piece
    ("g1x1e", 160, 32, 7, 8, 64),        # half a chunk of channels; backward-weight: 56-pixel rows, 160 images over the splits
    ("g1x1f", 2, 1024, 14, 14, 256),     # sixteen chunks
]


@pytest.mark.parametrize("row", BF16GEMM, ids=[r[0] for r in BF16GEMM])
def test_bf16_matrix_core_1x1(row):
    from paper_1912_01703_amd import binding as mc
    name, N, C, H, W, K = row
    L = wl.custom_layer(name, N, C, H, W, K, 1, 1, 1, 0, 1, seed=6300 + BF16GEMM.index(row))
    for p in range(3):
        assert mc.miconv_kernel_path(p, *L.conv_args(), mc.BF16_F32ACC) == "mfma/bf16_gemm", (name, p)
    pu.check_layer_full(L, "bf16", algo=mc.ALGO_MFMA, expect_algo=mc.ALGO_MFMA)


def test_bf16_1x1_tensors_that_start_on_an_odd_element():
    import torch
    L = wl.custom_layer("g-odd-start", 16, 64, 14, 14, 128, 1, 1, 1, 0, 1, seed=6310)
    h = pu.prepare(L, "bf16")
    gr = pu.GpuRunner(L, h, "bf16")

    def shifted(t):
        flat = torch.empty(t.numel() + 1, dtype=t.dtype, device=t.device)
        flat[1:].copy_(t.reshape(-1))
        return flat[1:].view(t.shape)

    gr.x, gr.w, gr.dy = shifted(gr.x), shifted(gr.w), shifted(gr.dy)
    for p in pu.PASSES:
        out = gr.run(p).cpu().numpy()
        refv, den = pu.oracle_full(L, h, p)
        err, ok = pu.max_norm_err(out, refv, den)
        assert ok and err <= pu.TOL["bf16"], (p, err)


PHASED = [
    # name      N   C   H   W   K   R   S  stride pad groups      backward-data only (per-phase MFMA launches)
    ("p5x5s2", 2, 16, 20, 20, 16, 5, 5, 2, 2, 1),
    ("p11s4", 2, 3, 63, 63, 16, 11, 11, 4, 2, 1),     # AlexNet-like: 16 phases of 3x3 / 3x2 / 2x3 / 2x2 taps
    ("p3x3s3", 1, 8, 17, 15, 8, 3, 3, 3, 1, 1),       # stride == filter size: every phase has one tap
    ("p4x2s2", 2, 8, 12, 13, 12, 4, 2, (2, 1), (1, 0), 1),
]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("row", PHASED, ids=[r[0] for r in PHASED])
def test_strided_bwd_data_phases(row, dtype):
    from paper_1912_01703_amd import binding as mc
    name, N, C, H, W, K, R, S, st, pd, g = row
    L = wl.custom_layer(name, N, C, H, W, K, R, S, st, pd, g, seed=4000 + PHASED.index(row))
    pu.check_layer_full(L, dtype, passes=("bwd_data",), algo=mc.ALGO_MFMA, expect_algo=mc.ALGO_MFMA)


SMALLC = [
    # name      N   H    W    K  pad     3 input channels, 11x11 filter, stride 4 (AlexNet-style first layer)
    ("a11a", 2, 63, 63, 64, 2),
    ("a11b", 3, 51, 75, 40, 2),      # ragged tiles, K not a multiple of 64
    ("a11c", 1, 227, 227, 16, 0),    # no padding, full-width rows
    ("a11f", 1, 35, 243, 16, 2),     # 60 output columns / 61 column positions: two tiles side by side in every pass
]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("row", SMALLC, ids=[r[0] for r in SMALLC])
def test_small_channel_large_filter(row, dtype):
    from paper_1912_01703_amd import binding as mc
    name, N, H, W, K, pd = row
    L = wl.custom_layer(name, N, 3, H, W, K, 11, 11, 4, pd, 1, seed=5000 + SMALLC.index(row))
    pu.check_layer_full(L, dtype, algo=mc.ALGO_MFMA, expect_algo=mc.ALGO_MFMA)


STEM = [
    # name     N   H    W    K  pad     3 input channels, 7x7 filter, stride 2 (ResNet-style first layer): forward and
    #                                   backward-weight on the matrix cores
    ("s7a", 2, 64, 64, 64, 3),
    ("s7b", 3, 51, 75, 40, 3),       # ragged tiles, K not a multiple of 64
    ("s7c", 1, 230, 230, 16, 0),     # no padding, 112 output columns: two tiles side by side
    ("s7d", 2, 37, 33, 72, 2),       # two filter blocks, padding 2
]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("row", STEM, ids=[r[0] for r in STEM])
def test_three_channel_7x7_stride_2(row, dtype):
    from paper_1912_01703_amd import binding as mc
    name, N, H, W, K, pd = row
    L = wl.custom_layer(name, N, 3, H, W, K, 7, 7, 2, pd, 1, seed=5100 + STEM.index(row))
    pu.check_layer_full(L, dtype, passes=("fwd", "bwd_weight"), algo=mc.ALGO_MFMA, expect_algo=mc.ALGO_MFMA)


def test_three_channel_7x7_stride_2_backward_data():
    """Padding 3, fp32: the vector-ALU kernel with a 2 x 2 block of dx pixels per lane."""
    from paper_1912_01703_amd import binding as mc
    for i, (N, H, W, K) in enumerate([(2, 64, 64, 64), (1, 45, 51, 24)]):
        L = wl.custom_layer("s7bd%d" % i, N, 3, H, W, K, 7, 7, 2, 3, 1, seed=5200 + i)
        pu.check_layer_full(L, "f32", passes=("bwd_data",), algo=mc.ALGO_MFMA, expect_algo=mc.ALGO_MFMA)


def test_small_channel_backward_data_with_more_than_64_filters():
    """The matrix-core backward-data kernel keeps all filters of a layer in LDS (K <= 64); with more, fp32
    tensors take the vector-ALU kernel."""
    from paper_1912_01703_amd import binding as mc
    L = wl.custom_layer("a11e", 2, 3, 63, 67, 80, 11, 11, 4, 2, 1, seed=5011)
    pu.check_layer_full(L, "f32", passes=("bwd_data",), algo=mc.ALGO_MFMA, expect_algo=mc.ALGO_MFMA)


def test_small_channel_forward_walks_several_items():
    """Two filter blocks share the 256 persistent workgroups, and 140 work items per block exceed the 128
    workgroups of each: some workgroups run a second item out of the other LDS buffer."""
    from paper_1912_01703_amd import binding as mc
    L = wl.custom_layer("a11d", 5, 3, 227, 227, 128, 11, 11, 4, 2, 1, seed=5010)
    pu.check_layer_full(L, "f32", passes=("fwd",), algo=mc.ALGO_MFMA, expect_algo=mc.ALGO_MFMA)


DW = [
    # name    N   C   H   W  stride pad
    ("dw14", 3, 40, 14, 14, 1, 1),
    ("dw7", 2, 70, 7, 7, 1, 1),        # 49 outputs per plane: ragged groups of four, scalar stores
    ("dw28s2", 2, 24, 28, 28, 2, 1),   # stride 2: backward-data on the row kernel
    ("dw29s2", 2, 6, 29, 31, 2, 1),    # stride 2, odd sizes: the last row and column of dx see fewer taps
    ("dw16s2p0", 1, 5, 16, 18, 2, 0),  # stride 2 without padding: the last input row and column feed nothing
    ("dw112", 1, 3, 112, 112, 1, 1),   # planes too large for the LDS kernels: the row kernels
    ("dw60x70s2", 1, 4, 60, 70, 2, 1), # ... at stride 2, ragged 16 x 64 blocks
    ("dw9x13", 5, 33, 9, 13, 1, 0),    # no padding, non-square
    ("dw15p2", 1, 17, 15, 15, 1, 2),   # padding wider than the filter reach
    ("dw56", 1, 8, 56, 56, 1, 1),
    # backward-weight: 20 batches of 4 images on 4 channels = 8 waves x 2 workgroups per channel, partial sums reduced
    ("dwsplit", 80, 4, 14, 14, 1, 1),
    ("dwc1024", 2, 1024, 14, 14, 1, 1),   # backward-weight: a wave owns 4 consecutive channels
    ("dwc513", 3, 513, 14, 14, 1, 1),     # ... 2 channels, the last pair half empty; 2 images per batch, the last half empty
]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("row", DW, ids=[r[0] for r in DW])
def test_depthwise_shapes(row, dtype):
    from paper_1912_01703_amd import binding as mc
    name, N, C, H, W, st, pd = row
    L = wl.custom_layer(name, N, C, H, W, C, 3, 3, st, pd, C, seed=3000 + DW.index(row))
    pu.check_layer_full(L, dtype, algo=mc.ALGO_DEPTHWISE, expect_algo=mc.ALGO_DEPTHWISE)


# the kernel family of each pass of each benchmark layer (fp32), as miconv_kernel_path names it
FAMILY = {
    "2a": ("mfma/tile", "mfma/tile", "mfma/wgrad"), "2b": ("mfma/tile", "mfma/tile", "mfma/wgrad"),
    "2c": ("mfma/tile", "mfma/tile_merge2", "mfma/wgrad"), "3": ("mfma/smallc",) * 3,
    "4a": ("mfma/tile", "mfma/tile", "mfma/wgrad"), "4b": ("mfma/tile", "mfma/tile", "mfma/wgrad"),
    "5a": ("depthwise/strip",) * 3, "5b": ("mfma/tile", "mfma/tile", "mfma/wgrad"),
}
FAMILY_BF16 = {"4a": ("mfma/bf16_tile", "mfma/bf16_tile", "mfma/bf16_wgrad"),
               "4b": ("mfma/bf16_tile", "mfma/bf16_tile", "mfma/bf16_wgrad")}


def expected_dispatch(name, dtype="f32"):
    """Asserts the tuned family every pass of the layer is dispatched to and returns the algorithm code."""
    from paper_1912_01703_amd import binding as mc
    fam = (FAMILY_BF16 if dtype == "bf16" else FAMILY)[name]
    code = mc.BF16_F32ACC if dtype == "bf16" else mc.F32
    got = tuple(mc.miconv_kernel_path(p, *wl.LAYERS[name].conv_args(), code) for p in range(3))
    assert got == fam, (name, dtype, got)
    return mc.ALGO_DEPTHWISE if fam[0].startswith("depthwise") else mc.ALGO_MFMA


@pytest.mark.parametrize("name", ["2a", "2b", "2c", "3", "5a", "5b"])
def test_full_size_layers_fp32(name):
    pu.check_layer_full(wl.LAYERS[name], expect_algo=expected_dispatch(name))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("name", ["4a", "4b"])
def test_vgg_layers_structured(name, dtype):
    """The two VGG-sized layers: forward and backward-data on whole images, whole tiles at both ends of every
    XCD's range of work, the tiles the persistent workgroups finish on, a mid-batch plane and a random sample;
    backward-weight in full."""
    pu.check_layer_structured(wl.LAYERS[name], dtype, expect_algo=expected_dispatch(name, dtype))


def test_bwd_weight_is_bit_reproducible():
    import torch
    L = wl.LAYERS["2a"]
    h = pu.prepare(L)
    gr = pu.GpuRunner(L, h)
    a = gr.run("bwd_weight").clone()
    b = gr.run("bwd_weight")
    torch.cuda.synchronize()
    assert torch.equal(a, b)


@pytest.mark.parametrize("name,dtype", [("2b", "f32"), ("2c", "f32"), ("5a", "f32"), ("3", "f32"), ("2b", "bf16"), ("2a", "bf16")],
                         ids=["split-1x1", "split-3x3s2", "depthwise", "three-channel", "bf16-product", "bf16-3x3"])
def test_bwd_weight_is_bit_reproducible_on_the_split_paths(name, dtype):
    """Paths that sum partial results (workspace partials, wave shares, register reductions) do so in a fixed order:
    two runs give the same bits."""
    import torch
    L = wl.LAYERS[name]
    h = pu.prepare(L, dtype)
    gr = pu.GpuRunner(L, h, dtype)
    a = gr.run("bwd_weight").clone()
    b = gr.run("bwd_weight")
    torch.cuda.synchronize()
    assert torch.equal(a, b)


def test_inputs_are_not_modified():
    import torch
    L = odd_layer(ODD[6])
    h = pu.prepare(L)
    gr = pu.GpuRunner(L, h)
    for p in pu.PASSES:
        gr.run(p)
    torch.cuda.synchronize()
    assert np.array_equal(gr.x.cpu().numpy(), h["x"])
    assert np.array_equal(gr.w.cpu().numpy(), h["w"])
    assert np.array_equal(gr.dy.cpu().numpy(), h["dy"])


def test_runs_on_a_side_stream():
    import torch
    from paper_1912_01703_amd import binding as mc
    L = wl.LAYERS["1"]
    h = pu.prepare(L)
    gr = pu.GpuRunner(L, h)
    s = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        y = gr.run("fwd")
    s.synchronize()
    refv, den = pu.oracle_full(L, h, "fwd")
    err, ok = pu.max_norm_err(y.cpu().numpy(), refv, den)
    assert ok and err <= 1e-5
    assert mc.miconv_last_algo(0) != mc.ALGO_AUTO
