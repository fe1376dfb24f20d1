"""Helpers for the GPU parity tests: run one pass through the C ABI and compare
it, element by element, with the CPU oracle.

Error measure (per output element i): e_i = |gpu_i - ref_i| / D_i, where D_i is
the same reduction evaluated on absolute values (forward: sum |x||w|; backward
data: sum |dy||w|; backward weight: sum |x||dy|), obtained by running the
oracle on |inputs|.  Where D_i == 0 no product reaches the element and the GPU
value must be exactly 0.  Bounds: 1e-5 for fp32 inputs, 1e-2 for bf16 inputs.
"""
from __future__ import annotations

import numpy as np

from oracle import convref as ref
from paper_1912_01703_amd import workloads as wl

TOL = {"f32": 1e-5, "bf16": 1e-2}
PASSES = ("fwd", "bwd_data", "bwd_weight")


def prepare(layer, dtype="f32"):
    """Host inputs for a layer.  Returns dict with the arrays handed to the GPU
    ('x','w','dy': float32 or uint16 bf16 bits) and the float32/float64-exact
    values the oracle is fed ('xo','wo','dyo')."""
    x, w, dy = wl.make_inputs(layer)
    if dtype == "bf16":
        xb, wb, dyb = wl.to_bf16_bits(x), wl.to_bf16_bits(w), wl.to_bf16_bits(dy)
        return dict(x=xb, w=wb, dy=dyb, xo=xb, wo=wb, dyo=dyb)
    return dict(x=x, w=w, dy=dy, xo=x, wo=w, dyo=dy)


def _abs(a):
    if a.dtype == np.uint16:
        return a & np.uint16(0x7FFF)
    return np.abs(a)


def oracle_full(layer, h, pass_name):
    """(reference, denominator) as full float64 tensors."""
    st, pd, g = layer.strides, layer.pads, layer.groups
    if pass_name == "fwd":
        f = lambda a, b: ref.conv2d_fwd(a, b, st, pd, g)
        a, b = h["xo"], h["wo"]
    elif pass_name == "bwd_data":
        f = lambda a, b: ref.conv2d_bwd_data(a, b, layer.x_shape, st, pd, g)
        a, b = h["dyo"], h["wo"]
    else:
        f = lambda a, b: ref.conv2d_bwd_weight(a, b, layer.w_shape, st, pd, g)
        a, b = h["xo"], h["dyo"]
    return f(a, b), f(_abs(a), _abs(b))


def oracle_at(layer, h, pass_name, idx):
    """(reference, denominator) at flat output indices idx."""
    st, pd, g = layer.strides, layer.pads, layer.groups
    if pass_name == "fwd":
        f = lambda a, b: ref.conv2d_fwd_at(a, b, idx, st, pd, g)
        a, b = h["xo"], h["wo"]
    elif pass_name == "bwd_data":
        f = lambda a, b: ref.conv2d_bwd_data_at(a, b, layer.x_shape, idx, st, pd, g)
        a, b = h["dyo"], h["wo"]
    else:
        f = lambda a, b: ref.conv2d_bwd_weight_at(a, b, layer.w_shape, idx, st, pd, g)
        a, b = h["xo"], h["dyo"]
    return f(a, b), f(_abs(a), _abs(b))


def out_shape(layer, pass_name):
    return {"fwd": layer.y_shape, "bwd_data": layer.x_shape, "bwd_weight": layer.w_shape}[pass_name]


def max_norm_err(gpu, refv, den):
    """max_i |gpu_i - ref_i| / D_i over elements with D_i > 0, and whether all
    elements with D_i == 0 are exactly zero on the GPU."""
    gpu = np.asarray(gpu, dtype=np.float64).reshape(-1)
    refv = refv.reshape(-1)
    den = den.reshape(-1)
    finite = bool(np.all(np.isfinite(gpu)))
    dead = den == 0
    zeros_ok = bool(np.all(gpu[dead] == 0))
    live = ~dead
    err = float(np.max(np.abs(gpu[live] - refv[live]) / den[live])) if live.any() else 0.0
    return err, zeros_ok and finite


# ----------------------------------------------------------------- GPU side
class GpuRunner:
    """Owns device copies of one layer's inputs and runs passes through the C ABI."""

    def __init__(self, layer, h, dtype="f32"):
        import torch
        from paper_1912_01703_amd import binding as mc
        self.torch, self.mc = torch, mc
        self.layer, self.dtype = layer, dtype
        self.code = mc.BF16_F32ACC if dtype == "bf16" else mc.F32
        dev = "cuda:0"

        def up(a):
            if a.dtype == np.uint16:
                return torch.from_numpy(a.view(np.int16)).to(dev)
            return torch.from_numpy(a).to(dev)

        self.x, self.w, self.dy = up(h["x"]), up(h["w"]), up(h["dy"])
        self.ws = None

    def _workspace(self, pass_id):
        need = self.mc.conv2d_workspace_bytes(pass_id, *self.layer.conv_args(), self.code)
        if need == 0:
            return None
        if self.ws is None or self.ws.numel() < need:
            self.ws = self.torch.empty(need, dtype=self.torch.uint8, device="cuda:0")
        return self.ws

    def run(self, pass_name, poison=True, out=None):
        torch, mc, L = self.torch, self.mc, self.layer
        pass_id = PASSES.index(pass_name)
        if out is None:
            out = torch.empty(out_shape(L, pass_name), dtype=torch.float32, device="cuda:0")
        if poison:
            out.fill_(float("nan"))
        stream = torch.cuda.current_stream().cuda_stream
        ws = self._workspace(pass_id)
        if pass_name == "fwd":
            mc.conv2d_fwd(self.x, self.w, out, *L.conv_args(), self.code, ws, stream)
        elif pass_name == "bwd_data":
            mc.conv2d_bwd_data(self.dy, self.w, out, *L.conv_args(), self.code, ws, stream)
        else:
            mc.conv2d_bwd_weight(self.x, self.dy, out, *L.conv_args(), self.code, ws, stream)
        return out

    def last_algo(self, pass_name):
        return self.mc.miconv_last_algo(PASSES.index(pass_name))


def check_layer_full(layer, dtype="f32", passes=PASSES, algo=None, expect_algo=None):
    """Full-tensor parity of the listed passes.  Returns {pass: err}."""
    from paper_1912_01703_amd import binding as mc
    h = prepare(layer, dtype)
    gr = GpuRunner(layer, h, dtype)
    errs = {}
    for p in passes:
        pid = PASSES.index(p)
        mc.miconv_set_algo(pid, algo if algo is not None else mc.ALGO_AUTO)
        try:
            print(f"[parity] layer={layer.name} dtype={dtype} pass={p} algo={algo}", flush=True)
            out = gr.run(p).cpu().numpy()
        finally:
            mc.miconv_set_algo(pid, mc.ALGO_AUTO)
        if expect_algo is not None:
            assert gr.last_algo(p) == expect_algo, (p, gr.last_algo(p), expect_algo)
        refv, den = oracle_full(layer, h, p)
        err, ok = max_norm_err(out, refv, den)
        assert ok, f"{layer.name}/{p}: non-finite output or non-zero where no tap reaches"
        assert err <= TOL[dtype], f"{layer.name}/{p}/{dtype}: normalised error {err:.3e} > {TOL[dtype]}"
        errs[p] = err
    return errs


def structured_indices(layer, pass_name, count=1 << 18, tail_units=64, tail_channels=4):
    """Flat output indices for a forward / backward-data check of a layer too large for the full oracle, placed
    where a tiled, persistent, XCD-aware kernel would go wrong rather than uniformly.

    The tuned kernels cut every (image, group) plane of the output into tiles of 12 x 16 pixels (planes at
    least 96 rows high whose width is a multiple of 16) or 14 x 14 pixels otherwise, numbered row-major within
    the plane, planes in image order: these are the "units".  The units are split into 8 equal contiguous
    ranges (one per XCD, ceil(units / 8) each), and persistent workgroups walk the ids of a range in order, so
    the last ids a workgroup walks are the last units of each range.  This function re-derives that map from
    the description above (no kernel code is imported) and returns
      (i)   every element of the first and of the last image (all channels, all tile seams and ragged tiles);
      (ii)  for each of the 8 ranges: the first unit and the last unit as whole tiles over all channels, and the
            last `tail_units` units as whole tiles over `tail_channels` channels (first, last, two seeded ones);
      (iii) one whole plane in the middle of the batch (every seam row and column once more);
      (iv)  wl.sample_indices' corners / edges / uniform random sample.
    """
    d0, d1, d2, d3 = out_shape(layer, pass_name)
    th, tw = (12, 16) if (d3 % 16 == 0 and d2 >= 96) else (14, 14)
    tiles_h, tiles_w = -(-d2 // th), -(-d3 // tw)
    units = d0 * tiles_h * tiles_w            # groups == 1 for the layers this is used on
    assert layer.groups == 1
    per_xcd = -(-units // 8)
    rng = np.random.Generator(np.random.PCG64(layer.seed + 11))
    picks = []

    def block(n, chans, r0, r1, c0, c1):
        n = np.asarray(n).reshape(-1, 1, 1, 1)
        ch = np.asarray(chans).reshape(1, -1, 1, 1)
        rr = np.arange(r0, min(r1, d2)).reshape(1, 1, -1, 1)
        cc = np.arange(c0, min(c1, d3)).reshape(1, 1, 1, -1)
        picks.append((((n * d1 + ch) * d2 + rr) * d3 + cc).reshape(-1))

    all_ch = np.arange(d1)
    for n in sorted({0, d0 - 1}):
        block(n, all_ch, 0, d2, 0, d3)                                    # (i)
    few = np.unique(np.concatenate([[0, d1 - 1], rng.integers(0, d1, size=max(0, tail_channels - 2))]))
    for x in range(8):                                                    # (ii)
        lo, hi = x * per_xcd, min((x + 1) * per_xcd, units)
        if lo >= hi:
            continue
        for u in range(max(lo, hi - tail_units), hi):
            n, t = divmod(u, tiles_h * tiles_w)
            ti, tj = divmod(t, tiles_w)
            block(n, all_ch if u in (lo, hi - 1) else few, ti * th, (ti + 1) * th, tj * tw, (tj + 1) * tw)
        n, t = divmod(lo, tiles_h * tiles_w)
        ti, tj = divmod(t, tiles_w)
        block(n, all_ch, ti * th, (ti + 1) * th, tj * tw, (tj + 1) * tw)
    block(d0 // 2, [d1 // 2], 0, d2, 0, d3)                               # (iii)
    picks.append(wl.sample_indices((d0, d1, d2, d3), count, seed=layer.seed + 7))   # (iv)
    return np.unique(np.concatenate(picks))


def check_layer_structured(layer, dtype="f32", expect_algo=None):
    """Parity of a layer too large for the full oracle in forward and backward-data: outputs at the structured
    places of structured_indices; backward-weight: every element of dw."""
    import torch
    from paper_1912_01703_amd import binding as mc
    h = prepare(layer, dtype)
    gr = GpuRunner(layer, h, dtype)
    errs = {}
    for p in PASSES:
        print(f"[parity-structured] layer={layer.name} dtype={dtype} pass={p}", flush=True)
        out_t = gr.run(p)
        if expect_algo is not None:
            assert gr.last_algo(p) == expect_algo, (p, gr.last_algo(p), expect_algo)
        assert bool(self_finite(out_t)), f"{layer.name}/{p}: non-finite output"
        if p == "bwd_weight":
            sel = out_t.cpu().numpy()
            refv, den = oracle_full(layer, h, p)
        else:
            idx = structured_indices(layer, p)
            sel = out_t.reshape(-1)[torch.from_numpy(idx).to(out_t.device)].cpu().numpy()
            refv, den = oracle_at(layer, h, p, idx)
            print(f"[parity-structured]   {idx.size} of {out_t.numel()} outputs", flush=True)
        err, ok = max_norm_err(sel, refv, den)
        assert ok, f"{layer.name}/{p}: non-zero where no tap reaches"
        assert err <= TOL[dtype], f"{layer.name}/{p}/{dtype}: normalised error {err:.3e} > {TOL[dtype]}"
        errs[p] = err
    return errs


def self_finite(t):
    import torch
    return torch.isfinite(t).all().item()
