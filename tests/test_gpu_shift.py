"""GPU parity of the plain-shift forward (slide_attn_fwd_shift; Sec. 4.2, Eq. 9-13: the shifts
as one-hot depthwise kernels, no learned kernels) against the CPU oracle.

The expected values are the oracle's forward with the kernels the oracle's own
re-parameterisation gives for a zero learned part (the one-hot kernels of Eq. 11), on the same
seeded inputs; tolerances as in test_gpu_parity.py.
"""
import numpy as np
import pytest
import torch

import paper_2304_04237_amd as sa
from paper_2304_04237_amd import synth
from oracle import slide_oracle as oracle

from tests.test_gpu_parity import check, sample_positions, tdtype

pytestmark = pytest.mark.gpu

SHIFT_SHAPES = [
    # B, H, W, C, heads, ksize, dtype, forward variant of the shape (24: streaming kernel in its plain form)
    (3, 8, 56, 64, 2, 3, "bf16", 24),       # stage-1 width, short bands
    (2, 56, 56, 64, 2, 3, "bf16", 24),      # stage-1 planes
    (1, 33, 64, 32, 1, 3, "bf16", 24),      # widest map of the streaming kernel, odd height
    (5, 31, 32, 96, 3, 3, "bf16", 24),      # narrowest, three heads
    (4, 21, 48, 64, 2, 3, "bf16", 24),
    (2, 9, 304, 96, 3, 3, "bf16", 26),      # wide maps: column strips
    (3, 17, 80, 64, 2, 3, "bf16", 26),
    (1, 40, 144, 32, 1, 3, "bf16", 26),
    (2, 9, 40, 64, 2, 3, "bf16", None),     # general kernel from here on
    (1, 14, 14, 64, 2, 3, "f32", None),
    (2, 9, 21, 64, 2, 3, "bf16", None),
    (2, 17, 13, 128, 4, 5, "bf16", None),
    (1, 7, 5, 24, 3, 3, "f32", None),
    (2, 5, 9, 16, 2, 1, "bf16", None),
    (1, 3, 2, 8, 2, 7, "f32", None),
    (1, 1, 1, 32, 1, 3, "bf16", None),
]


def shift_problem(B, H, W, C, heads, ksize, dtype, seed):
    d = synth.make_inputs(B, H, W, C, heads, ksize, dtype, seed=seed)
    dev = torch.device("cuda:0")
    g = {n: d[n].to(dev).to(tdtype(dtype)) for n in ("q", "k", "v")}
    g["bias"] = d["bias"].to(dev)
    n = {x: d[x].double().numpy() for x in ("q", "k", "v", "bias")}
    n["w"] = oracle.reparam(np.zeros((C, ksize * ksize, ksize, ksize)), ksize)
    return g, n


@pytest.mark.parametrize("shape", SHIFT_SHAPES)
def test_shift_forward_matches_oracle(shape):
    B, H, W, C, heads, ksize, dtype, variant = shape
    print("plain-shift case", shape, flush=True)
    if variant is not None:
        assert sa.slide_attn_fwd_variant(B, H, W, C, heads, ksize, dtype == "bf16" and 1 or 0) == variant
    g, n = shift_problem(B, H, W, C, heads, ksize, dtype, seed=300 + H + W)
    out = sa.slide_attn_fwd_shift(g["q"], g["k"], g["v"], g["bias"], heads, ksize)
    torch.cuda.synchronize()
    ref, ref_lse = oracle.fwd(n["q"], n["k"], n["v"], n["w"], n["w"], n["bias"], heads, ksize, return_lse=True)
    check("out", dtype, out, ref)
    out0 = sa.slide_attn_fwd_shift(g["q"], g["k"], g["v"], None, heads, ksize)
    ref0 = oracle.fwd(n["q"], n["k"], n["v"], n["w"], n["w"], None, heads, ksize)
    check("out(no bias)", dtype, out0, ref0)
    lse = torch.full((B, heads, H, W), float("nan"), dtype=torch.float32, device=out.device)
    out1 = sa.slide_attn_fwd_shift(g["q"], g["k"], g["v"], g["bias"], heads, ksize, lse=lse)
    assert torch.equal(out1, out)
    check("lse", dtype, lse, ref_lse)


def test_shift_forward_unaligned_pointers_take_the_general_kernel():
    """Views that start 2 bytes into an allocation: not 16-byte aligned, same results."""
    B, H, W, C, heads, ksize = 2, 8, 56, 64, 2, 3
    g, n = shift_problem(B, H, W, C, heads, ksize, "bf16", seed=11)
    numel = B * C * H * W
    off = {}
    for name in ("q", "k", "v"):
        buf = torch.empty(numel + 8, dtype=torch.bfloat16, device="cuda:0")
        view = buf[1:1 + numel].view(B, C, H, W)
        view.copy_(g[name])
        assert view.data_ptr() % 16 != 0
        off[name] = view
    out = sa.slide_attn_fwd_shift(off["q"], off["k"], off["v"], g["bias"], heads, ksize)
    ref = oracle.fwd(n["q"], n["k"], n["v"], n["w"], n["w"], n["bias"], heads, ksize)
    check("out", "bf16", out, ref)


def test_shift_forward_closed_forms():
    """q = 0, no bias: the 3x3 box mean of v with the zero padding counted (corners 4/9 of the
    in-range mean); a huge bias on one shift: that shifted copy of v, zero at the border."""
    dev = torch.device("cuda:0")
    for (B, H, W, C, heads) in ((2, 12, 56, 64, 2), (1, 10, 23, 64, 2)):
        v = torch.randn(B, C, H, W, device=dev).bfloat16()
        k = torch.randn(B, C, H, W, device=dev).bfloat16()
        q = torch.zeros_like(v)
        out = sa.slide_attn_fwd_shift(q, k, v, None, heads, 3).float()
        want = torch.nn.functional.avg_pool2d(v.float(), 3, stride=1, padding=1, count_include_pad=True)
        assert (out - want).abs().max().item() <= 2e-2
        for s in (0, 5, 8):
            u, w = s // 3 - 1, s % 3 - 1
            bias = torch.zeros(heads, 9, device=dev)
            bias[:, s] = 1.0e4
            got = sa.slide_attn_fwd_shift(torch.randn_like(v), k, v, bias, heads, 3)
            want = torch.zeros_like(v)
            ys = slice(max(0, -u), min(H, H - u))
            xs = slice(max(0, -w), min(W, W - w))
            yd = slice(max(0, u), min(H, H + u))
            xd = slice(max(0, w), min(W, W + w))
            want[:, :, ys, xs] = v[:, :, yd, xd]
            # (the matrix-core path holds v in half precision: exact down to 2^-17, below that
            # low bits are dropped, an error of at most 2^-24)
            assert (got.float() - want.float()).abs().max().item() <= 2.0 ** -24, s


def test_shift_forward_stage1_full_size():
    """The benchmark's stage-1 shape at full size: sampled pixels and two whole batch items."""
    wl = synth.CONFIGS[1]
    assert (wl.B, wl.H, wl.W, wl.C, wl.heads, wl.ksize) == (64, 56, 56, 64, 2, 3)
    g, n = shift_problem(wl.B, wl.H, wl.W, wl.C, wl.heads, wl.ksize, "bf16", seed=1001)
    lse = torch.empty(wl.B, wl.heads, wl.H, wl.W, dtype=torch.float32, device="cuda:0")
    out = sa.slide_attn_fwd_shift(g["q"], g["k"], g["v"], g["bias"], wl.heads, wl.ksize, lse=lse)
    torch.cuda.synchronize()
    out = out.float().cpu().numpy()
    assert np.isfinite(out).all()
    pos = sample_positions(wl.B, wl.heads, wl.H, wl.W, 1500, seed=5)
    ref = oracle.fwd_samples(n["q"], n["k"], n["v"], n["w"], n["w"], n["bias"], wl.heads, wl.ksize, pos)
    dd = wl.C // wl.heads
    got = np.stack([out[b, m * dd:(m + 1) * dd, i, j] for b, m, i, j in pos])
    assert np.abs(got - ref).max() <= 2e-2
    for b in (0, wl.B - 1):
        sl = slice(b, b + 1)
        refp, ref_lse = oracle.fwd(n["q"][sl], n["k"][sl], n["v"][sl], n["w"], n["w"], n["bias"], wl.heads,
                                   wl.ksize, return_lse=True)
        assert np.abs(out[sl] - refp).max() <= 2e-2
        assert np.abs(lse[sl].cpu().numpy() - ref_lse).max() <= 2e-2


def test_traffic_probe_runs_and_rejects_what_it_cannot_do():
    """The measurement aid: both modes run on the stage-1 shape (out = XOR of the inputs in mode
    0), mode 1 is refused where the streaming kernel does not run, bad modes are refused."""
    dev = torch.device("cuda:0")
    B, C, H, W, heads = 2, 64, 56, 56, 2
    q, k, v = (torch.randn(B, C, H, W, device=dev).bfloat16() for _ in range(3))
    out = torch.zeros_like(q)
    sa.slide_attn_fwd_traffic_probe(q, k, v, out, heads, 0)
    torch.cuda.synchronize()
    want = q.view(torch.int16) ^ k.view(torch.int16) ^ v.view(torch.int16)
    assert torch.equal(out.view(torch.int16), want)
    sa.slide_attn_fwd_traffic_probe(q, k, v, out, heads, 1)
    torch.cuda.synchronize()
    with pytest.raises(sa.SlideAttnError):
        sa.slide_attn_fwd_traffic_probe(q, k, v, out, heads, 2)
    wide = torch.zeros(1, 64, 8, 304, device=dev, dtype=torch.bfloat16)
    with pytest.raises(sa.SlideAttnError):
        sa.slide_attn_fwd_traffic_probe(wide, wide, wide, torch.empty_like(wide), heads, 1)


HEAD24_SHAPES = [
    # B, H, W, C, heads: head size 24 (Slide-CSwin-B, App. A) on the streaming matrix-core kernel
    (2, 20, 56, 48, 2),
    (3, 33, 32, 72, 3),
    (1, 9, 64, 24, 1),
    (4, 56, 56, 48, 2),
]


@pytest.mark.parametrize("shape", HEAD24_SHAPES)
def test_head_size_24_on_the_streaming_kernel(shape):
    """Merged-kernel forward (with lse), training form and plain shift at 24 channels per head."""
    B, H, W, C, heads = shape
    ksize, dtype = 3, "bf16"
    print("head size 24 case", shape, flush=True)
    assert sa.slide_attn_fwd_variant(B, H, W, C, heads, ksize, 1) == 24
    assert sa.slide_attn_fwd_variant(B, H, W, C, heads, ksize, 1, aligned16=False) == 10
    d = synth.make_inputs(B, H, W, C, heads, ksize, dtype, seed=700 + H + W)
    dev = torch.device("cuda:0")
    g = {n: d[n].to(dev).to(torch.bfloat16) for n in ("q", "k", "v")}
    wk_l, wv_l = d["wk_learned"].to(dev), d["wv_learned"].to(dev)
    wk, wv = sa.slide_reparam(wk_l), sa.slide_reparam(wv_l)
    bias = d["bias"].to(dev)
    n = {x: d[x].double().numpy() for x in ("q", "k", "v", "bias")}
    lse = torch.full((B, heads, H, W), float("nan"), dtype=torch.float32, device=dev)
    out = sa.slide_attn_fwd(g["q"], g["k"], g["v"], wk, wv, bias, heads, ksize, lse=lse)
    torch.cuda.synchronize()
    ref, ref_lse = oracle.fwd(n["q"], n["k"], n["v"], wk.double().cpu().numpy(), wv.double().cpu().numpy(),
                              n["bias"], heads, ksize, return_lse=True)
    check("out", dtype, out, ref)
    check("lse", dtype, lse, ref_lse)
    out_nolse = sa.slide_attn_fwd(g["q"], g["k"], g["v"], wk, wv, bias, heads, ksize)
    assert torch.equal(out_nolse, out)
    out_tb = sa.slide_attn_fwd_two_branch(g["q"], g["k"], g["v"], wk_l, wv_l, bias, heads, ksize)
    ref_tb = oracle.fwd(n["q"], n["k"], n["v"], d["wk_learned"].double().numpy(), d["wv_learned"].double().numpy(),
                        n["bias"], heads, ksize, two_branch=True)
    check("out(two-branch)", dtype, out_tb, ref_tb)
    w1 = oracle.reparam(np.zeros((C, 9, 3, 3)), 3)
    out_s = sa.slide_attn_fwd_shift(g["q"], g["k"], g["v"], bias, heads, ksize)
    check("out(shift)", dtype, out_s, oracle.fwd(n["q"], n["k"], n["v"], w1, w1, n["bias"], heads, ksize))
    # the general kernel on the same problem (unaligned views) agrees with the oracle as well
    numel = B * C * H * W
    views = {}
    for name in ("q", "k", "v"):
        buf = torch.empty(numel + 8, dtype=torch.bfloat16, device=dev)
        views[name] = buf[1:1 + numel].view(B, C, H, W)
        views[name].copy_(g[name])
    out_g = sa.slide_attn_fwd(views["q"], views["k"], views["v"], wk, wv, bias, heads, ksize)
    check("out(general kernel)", dtype, out_g, ref)
