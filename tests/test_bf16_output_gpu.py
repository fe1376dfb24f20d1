"""GPU parity of the bf16-output variant (MICONV_BF16_BF16OUT): bf16 inputs, fp32 accumulation, y and dx stored as
bf16, dw as float.  The oracle is unchanged (fp64 results of the bf16 inputs); the stored bf16 value is widened and
compared with it under the bf16 bound, |gpu - ref| <= 1e-2 * sum |a||b|: rounding the result to bf16 adds at most
2^-9 |ref| <= 2^-9 * sum |a||b| to the kernel's own error, well inside the bound.  Where the denominator is zero the
stored value must be zero.
"""
import numpy as np
import pytest

from oracle import convref as ref
from paper_1912_01703_amd import workloads as wl

import parity_util as pu

pytestmark = pytest.mark.gpu

SHAPES = [
    # name        N   C    H    W   K  R  S  stride pad groups   what runs
    ("o3x3a", 2, 32, 16, 16, 64, 3, 3, 1, 1, 1),       # bf16 matrix cores, the kernel stores bf16 pairs itself
    ("o3x3g", 2, 32, 8, 17, 32, 3, 3, 1, 1, 1),        # ... odd row length: 2-byte stores
    ("o3x3w", 1, 32, 100, 48, 64, 3, 3, 1, 1, 1),      # ... the instance that reads NCHW in place
    ("o3x3e", 1, 160, 28, 28, 128, 3, 3, 1, 1, 1),     # ... several chunks and filter blocks
    ("o1x1a", 2, 48, 14, 14, 80, 1, 1, 1, 0, 1),       # fp32 matrix cores on widened inputs: float result staged, then converted
    ("o1x1g", 16, 64, 14, 14, 128, 1, 1, 1, 0, 1),     # 1x1 as a matrix product on the bf16 cores: bf16 stored by the kernel
    ("o3x3s2", 2, 32, 28, 28, 32, 3, 3, 2, 1, 1),      # strided: merged-phase backward-data
    ("o7", 2, 64, 7, 7, 64, 3, 3, 1, 1, 1),            # 7x7 planes (an odd number of pixels): not on the bf16 cores
    ("oodd4", 2, 3, 13, 9, 5, 4, 3, (3, 2), (1, 0), 1),   # direct kernels
    ("odw14", 3, 40, 14, 14, 40, 3, 3, 1, 1, 40),      # depthwise
    ("oa11", 2, 3, 63, 63, 64, 11, 11, 4, 2, 1),       # three-channel first layer
]


def run_case(L, which, fused=False):
    import torch
    from paper_1912_01703_amd import binding as mc
    h = pu.prepare(L, "bf16")
    st, pd, g = L.strides, L.pads, L.groups
    dev = "cuda:0"
    up = lambda a: torch.from_numpy(a.view(np.int16) if a.dtype == np.uint16 else a).to(dev)
    pid = 0 if which == "fwd" else 1
    args = L.conv_args()
    need = mc.conv2d_workspace_bytes(pid, *args, mc.BF16_BF16OUT)
    ws = torch.empty(max(need, 256), dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream().cuda_stream
    shape = L.y_shape if which == "fwd" else L.x_shape
    out = torch.full(shape, 0x7FC0, dtype=torch.int16, device=dev)      # bf16 NaN
    bias, act = wl.make_epilogue_inputs(L)
    actb = wl.to_bf16_bits(act)
    print(f"[bf16-out] layer={L.name} call={which} fused={fused} path={mc.miconv_kernel_path(pid, *args, mc.BF16_BF16OUT)} ws={need}", flush=True)
    if which == "fwd":
        if fused:
            mc.conv2d_fwd_bias_relu(up(h["x"]), up(h["w"]), up(bias), out, *args, mc.BF16_BF16OUT, ws, stream)
            want = ref.conv2d_fwd_bias_relu(h["xo"], h["wo"], bias, st, pd, g)
        else:
            mc.conv2d_fwd(up(h["x"]), up(h["w"]), out, *args, mc.BF16_BF16OUT, ws, stream)
            want = ref.conv2d_fwd(h["xo"], h["wo"], st, pd, g)
        den = ref.conv2d_fwd(pu._abs(h["xo"]), pu._abs(h["wo"]), st, pd, g)
        if fused:
            den = den + np.abs(bias.astype(np.float64))[None, :, None, None]
    else:
        if fused:
            mc.conv2d_bwd_data_relu_mask(up(h["dy"]), up(h["w"]), up(actb), out, *args, mc.BF16_BF16OUT, ws, stream)
            want = ref.conv2d_bwd_data_relu(h["dyo"], h["wo"], actb, st, pd, g)
        else:
            mc.conv2d_bwd_data(up(h["dy"]), up(h["w"]), out, *args, mc.BF16_BF16OUT, ws, stream)
            want = ref.conv2d_bwd_data(h["dyo"], h["wo"], L.x_shape, st, pd, g)
        den = ref.conv2d_bwd_data(pu._abs(h["dyo"]), pu._abs(h["wo"]), L.x_shape, st, pd, g)
    torch.cuda.synchronize()
    got = wl.bf16_bits_to_f32(out.cpu().numpy().view(np.uint16)).astype(np.float64)
    err, ok = pu.max_norm_err(got, want, den)
    assert ok, f"{L.name}/{which}: non-finite output or non-zero where nothing reaches"
    assert err <= pu.TOL["bf16"], f"{L.name}/{which}: normalised error {err:.3e}"
    if fused and which == "bwd_data":
        assert np.all(got[~(act > 0)] == 0.0)
    return need


@pytest.mark.parametrize("which", ["fwd", "bwd_data"])
@pytest.mark.parametrize("row", SHAPES, ids=[r[0] for r in SHAPES])
def test_bf16_output_shapes(row, which):
    name, N, C, H, W, K, R, S, st, pd, g = row
    L = wl.custom_layer(name, N, C, H, W, K, R, S, st, pd, g, seed=8500 + SHAPES.index(row))
    run_case(L, which)


@pytest.mark.parametrize("which", ["fwd", "bwd_data"])
@pytest.mark.parametrize("row", [SHAPES[0], SHAPES[2], SHAPES[4], SHAPES[5], SHAPES[9]],
                         ids=["native", "native-nchw", "staged-mfma", "native-1x1", "staged-dw"])
def test_bf16_output_with_fused_epilogues(row, which):
    name, N, C, H, W, K, R, S, st, pd, g = row
    L = wl.custom_layer(name + "e", N, C, H, W, K, R, S, st, pd, g, seed=8600 + SHAPES.index(row))
    run_case(L, which, fused=True)


def test_bf16_output_needs_no_staging_on_the_bf16_matrix_cores():
    from paper_1912_01703_amd import binding as mc
    for name in ("4a", "4b"):
        L = wl.LAYERS[name]
        for p in (0, 1):
            assert mc.conv2d_workspace_bytes(p, *L.conv_args(), mc.BF16_BF16OUT) == mc.conv2d_workspace_bytes(p, *L.conv_args(), mc.BF16_F32ACC)
    L = wl.LAYERS["3"]       # the three-channel first layer: fp32 matrix cores on widened inputs, the float result is staged
    assert mc.conv2d_workspace_bytes(0, *L.conv_args(), mc.BF16_BF16OUT) == 4 * L.N * L.K * L.P * L.Q
    L = wl.LAYERS["2b"]      # 1x1 on the bf16 matrix cores: bf16 written by the kernel, scratch for the channels-innermost copy only
    assert mc.conv2d_workspace_bytes(0, *L.conv_args(), mc.BF16_BF16OUT) == mc.conv2d_workspace_bytes(0, *L.conv_args(), mc.BF16_F32ACC)


def test_bf16_output_backward_weight_is_the_float_result():
    import torch
    from paper_1912_01703_amd import binding as mc
    L = wl.custom_layer("owg", 16, 32, 16, 16, 64, 3, 3, 1, 1, 1, seed=8700)
    h = pu.prepare(L, "bf16")
    gr = pu.GpuRunner(L, h, "bf16")
    a = gr.run("bwd_weight").clone()
    gr.code = mc.BF16_BF16OUT
    b = gr.run("bwd_weight")
    torch.cuda.synchronize()
    assert torch.equal(a, b)


def test_bf16_output_on_layer_4b_sampled():
    """The 28x28 VGG layer with bf16 results, forward, on a seeded sample of 2^16 outputs."""
    import torch
    from paper_1912_01703_amd import binding as mc
    L = wl.LAYERS["4b"]
    h = pu.prepare(L, "bf16")
    gr = pu.GpuRunner(L, h, "bf16")
    need = mc.conv2d_workspace_bytes(0, *L.conv_args(), mc.BF16_BF16OUT)
    ws = torch.empty(need, dtype=torch.uint8, device="cuda:0")
    out = torch.full(L.y_shape, 0x7FC0, dtype=torch.int16, device="cuda:0")
    mc.conv2d_fwd(gr.x, gr.w, out, *L.conv_args(), mc.BF16_BF16OUT, ws, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    idx = wl.sample_indices(L.y_shape, 1 << 16, seed=L.seed + 9)
    sel = wl.bf16_bits_to_f32(out.reshape(-1)[torch.from_numpy(idx).to("cuda:0")].cpu().numpy().view(np.uint16)).astype(np.float64)
    refv, den = pu.oracle_at(L, h, "fwd", idx)
    err, ok = pu.max_norm_err(sel, refv, den)
    assert ok and err <= pu.TOL["bf16"], err
    assert not bool((out == 0x7FC0).any())          # every element was written
