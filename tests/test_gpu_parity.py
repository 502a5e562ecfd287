"""GPU parity: the HIP library (through the C ABI binding) against the CPU oracle,
element by element on the same seeded inputs.

Tolerances (written here, from the problem statement):
  float32 : max|x - o| <= 1e-5 * max|o|                       per tensor
  bfloat16: max|x - o| <= 2e-2                                out, lse, dq, dk, dv
            max|x - o| <= 2e-2 * max(1, max|o|)               dwk, dwv, dbias
The oracle receives the inputs already rounded to the storage dtype, so both
sides see identical values.
"""
import numpy as np
import pytest
import torch

import paper_2304_04237_amd as sa
from paper_2304_04237_amd import synth
from oracle import slide_oracle as oracle

pytestmark = pytest.mark.gpu

GRAD_NAMES = "dq dk dv dwk dwv dbias".split()


def tdtype(dtype):
    return torch.float32 if dtype == "f32" else torch.bfloat16


def bound_for(name, dtype, want):
    mx = float(np.abs(want).max())
    if dtype == "f32":
        return 1e-5 * mx
    if name in ("dwk", "dwv", "dbias"):
        return 2e-2 * max(1.0, mx)
    return 2e-2


def check(name, dtype, got, want):
    got = got.detach().double().cpu().numpy()
    assert got.shape == want.shape, (name, got.shape, want.shape)
    assert np.isfinite(got).all(), name
    err = float(np.abs(got - want).max())
    bound = bound_for(name, dtype, want)
    assert err <= bound, "%s (%s): max abs err %.3e > %.3e" % (name, dtype, err, bound)
    return err


def gpu_problem(B, H, W, C, heads, ksize, dtype, seed, kernel_std=synth.KERNEL_STD,
                bias_std=synth.BIAS_STD):
    d = synth.make_inputs(B, H, W, C, heads, ksize, dtype, seed=seed, kernel_std=kernel_std,
                          bias_std=bias_std)
    dev = torch.device("cuda:0")
    g = {n: d[n].to(dev).to(tdtype(dtype)) for n in ("q", "k", "v", "dout")}
    g["wk"] = sa.slide_reparam(d["wk_learned"].to(dev))
    g["wv"] = sa.slide_reparam(d["wv_learned"].to(dev))
    g["bias"] = d["bias"].to(dev)
    n = {x: d[x].double().numpy() for x in ("q", "k", "v", "dout", "bias")}
    # the oracle gets the float32 merged kernels the GPU produced, widened
    n["wk"] = g["wk"].double().cpu().numpy()
    n["wv"] = g["wv"].double().cpu().numpy()
    return d, g, n


def test_reparam_matches_oracle_bit_exactly():
    for C, ksize in ((64, 3), (8, 5), (3, 1), (4, 7)):
        w = torch.randn(C, ksize * ksize, ksize, ksize, generator=torch.Generator().manual_seed(1)) * 0.02
        got = sa.slide_reparam(w.cuda()).cpu().numpy()
        want = oracle.reparam(w.double().numpy(), ksize).astype(np.float32)
        assert np.array_equal(got, want)
        # in place
        wd = w.cuda()
        sa.slide_reparam(wd, wd)
        assert np.array_equal(wd.cpu().numpy(), want)


FWD_SHAPES = [
    # B, H, W, C, heads, ksize, dtype
    (1, 14, 14, 64, 2, 3, "f32"),        # benchmark configuration 1
    (2, 9, 21, 64, 2, 3, "bf16"),        # ragged: several tiles and a tail
    (1, 33, 70, 32, 1, 3, "bf16"),       # wider than one tile
    (2, 17, 13, 128, 4, 5, "bf16"),      # 5x5 window
    (1, 7, 5, 24, 3, 3, "f32"),          # head size 8
    (1, 6, 6, 48, 2, 5, "f32"),          # head size 24, 5x5
    (2, 5, 9, 16, 2, 1, "bf16"),         # 1x1 window
    (1, 3, 2, 8, 2, 7, "f32"),           # map smaller than the window
    (1, 1, 1, 32, 1, 3, "bf16"),         # single pixel
    (1, 20, 40, 96, 3, 3, "bf16"),       # three heads
    (3, 8, 56, 64, 2, 3, "bf16"),        # stage-1 width
    (1, 9, 70, 32, 1, 5, "bf16"),        # 5x5, wider than one tile
    (1, 3, 4, 32, 1, 5, "bf16"),         # 5x5, map smaller than the window
    (2, 30, 28, 64, 2, 5, "bf16"),       # 5x5, several tiles per plane, two heads
    (1, 5, 130, 64, 2, 3, "bf16"),       # three column tiles, ragged last one
]


@pytest.mark.parametrize("shape", FWD_SHAPES)
def test_forward_matches_oracle(shape):
    B, H, W, C, heads, ksize, dtype = shape
    print("forward case", shape, flush=True)
    d, g, n = gpu_problem(B, H, W, C, heads, ksize, dtype, seed=100 + H + W)
    out = sa.slide_attn_fwd(g["q"], g["k"], g["v"], g["wk"], g["wv"], g["bias"], heads, ksize)
    torch.cuda.synchronize()
    ref = oracle.fwd(n["q"], n["k"], n["v"], n["wk"], n["wv"], n["bias"], heads, ksize)
    check("out", dtype, out, ref)
    # no bias == zero bias
    out0 = sa.slide_attn_fwd(g["q"], g["k"], g["v"], g["wk"], g["wv"], None, heads, ksize)
    ref0 = oracle.fwd(n["q"], n["k"], n["v"], n["wk"], n["wv"], None, heads, ksize)
    check("out(no bias)", dtype, out0, ref0)
    # with the log of the softmax denominator as a second result: out is unchanged
    lse = torch.full((B, heads, H, W), float("nan"), dtype=torch.float32, device=out.device)
    out1 = sa.slide_attn_fwd(g["q"], g["k"], g["v"], g["wk"], g["wv"], g["bias"], heads, ksize, lse=lse)
    assert torch.equal(out1, out)
    _, ref_lse = oracle.fwd(n["q"], n["k"], n["v"], n["wk"], n["wv"], n["bias"], heads, ksize, return_lse=True)
    check("lse", dtype, lse, ref_lse)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_forward_large_kernels_and_bias(dtype):
    """Kernels and biases far from the synthetic recipe (O(1) entries, peaked softmax)."""
    B, H, W, C, heads, ksize = 1, 12, 18, 64, 2, 3
    d, g, n = gpu_problem(B, H, W, C, heads, ksize, dtype, seed=77, kernel_std=0.5, bias_std=2.0)
    out = sa.slide_attn_fwd(g["q"], g["k"], g["v"], g["wk"], g["wv"], g["bias"], heads, ksize)
    ref = oracle.fwd(n["q"], n["k"], n["v"], n["wk"], n["wv"], n["bias"], heads, ksize)
    got = out.double().cpu().numpy()
    err = np.abs(got - ref).max()
    scale = np.abs(ref).max()
    # values reach O(10) here, so the bf16 bound is taken relative to the largest output
    assert err <= (1e-5 if dtype == "f32" else 2e-2) * max(1.0, scale), (err, scale)


def test_forward_special_cases_on_gpu():
    """Closed forms on the GPU itself: uniform attention = box filter with the padding
    counted; a huge bias selects one shifted copy of v (zero at the border)."""
    dev = torch.device("cuda:0")
    B, H, W, C, heads, ksize = 1, 10, 23, 64, 2, 3
    S = ksize * ksize
    for dtype in (torch.float32, torch.bfloat16):
        v = torch.randn(B, C, H, W, device=dev).to(dtype)
        k = torch.randn(B, C, H, W, device=dev).to(dtype)
        q = torch.zeros(B, C, H, W, device=dev, dtype=dtype)
        w = sa.slide_reparam(torch.zeros(C, S, ksize, ksize, device=dev))
        out = sa.slide_attn_fwd(q, k, v, w, w, None, heads, ksize)
        ref = torch.nn.functional.avg_pool2d(v.float(), ksize, 1, ksize // 2, count_include_pad=True)
        tol = 1e-6 if dtype == torch.float32 else 2e-2
        assert (out.float() - ref).abs().max().item() <= tol
        bias = torch.zeros(heads, S, device=dev)
        bias[:, 0] = 1e4                               # shift (-1,-1): out[i,j] = v[i-1,j-1]
        out = sa.slide_attn_fwd(torch.randn_like(v), k, v, w, w, bias, heads, ksize)
        expect = torch.zeros_like(v)
        expect[:, :, 1:, 1:] = v[:, :, :-1, :-1]
        if dtype == torch.float32:
            assert torch.equal(out, expect)
        else:
            # the bf16 path holds v in half precision inside the kernel: exact down to 2^-17,
            # multiples of 2^-24 below that
            assert (out.float() - expect.float()).abs().max().item() <= 2.0 ** -24


BWD_SHAPES = [
    (1, 14, 14, 64, 2, 3, "f32"),
    (2, 9, 21, 64, 2, 3, "bf16"),
    (1, 6, 7, 24, 3, 5, "f32"),
    (2, 11, 6, 32, 1, 5, "bf16"),
    (2, 5, 9, 16, 2, 1, "f32"),
    (1, 3, 2, 8, 2, 7, "f32"),
    (3, 8, 56, 64, 2, 3, "bf16"),
    (1, 20, 40, 96, 3, 3, "bf16"),       # three heads
    (2, 13, 72, 32, 1, 3, "bf16"),       # two column tiles
    (1, 5, 8, 32, 1, 3, "bf16"),         # tiny
    (1, 1, 16, 32, 1, 3, "bf16"),        # single row
    (2, 31, 24, 64, 2, 3, "bf16"),       # rows not a multiple of the strip height
    # the kernel-gradient kernel gives a block several work units (strips of 3 rows x 56
    # columns, 128 blocks per head): next-unit prefetch, reuse of its LDS slots
    (40, 10, 56, 64, 2, 3, "bf16"),      # 160 units: two per block for some, a one-row last strip
    (20, 10, 112, 64, 2, 3, "bf16"),     # two column tiles, 160 units
    (24, 17, 48, 32, 1, 3, "bf16"),      # one head: 256 blocks; 144 units of width 48
    (50, 20, 40, 96, 3, 3, "bf16"),      # three heads: 85 blocks per head, 350 units, 4-5 per block
    # the streaming dk/dv kernel: bands of one plane, odd heights, the narrowest and widest maps it takes
    (2, 33, 40, 64, 2, 3, "bf16"),
    (1, 57, 56, 32, 1, 3, "bf16"),
    (3, 29, 48, 64, 2, 3, "bf16"),
    (70, 12, 56, 64, 2, 3, "bf16"),      # more planes than half the compute units: one band per plane
    (66, 25, 48, 64, 2, 3, "bf16"),      # one band of 25 rows per plane: ten epochs
    (150, 9, 48, 64, 2, 3, "bf16"),      # 300 planes: more blocks than compute units
    (1, 150, 40, 32, 1, 3, "bf16"),      # a tall map cut into many bands
    (2, 33, 32, 64, 2, 3, "bf16"),       # too narrow for the streaming dk/dv kernel's rings: tiled kernel for that part
    (3, 40, 64, 32, 1, 3, "bf16"),       # the widest map of the streaming per-pixel kernel; tiled dk/dv kernel
    # maps lower than the window's reach or than one epoch in the streaming kernels: a band ends
    # inside the first groups of rows
    (2, 3, 56, 64, 2, 3, "bf16"),
    (3, 5, 48, 32, 1, 3, "bf16"),
    (5, 4, 40, 64, 2, 3, "bf16"),
    (2, 6, 32, 64, 2, 3, "bf16"),
    (1, 1, 56, 32, 1, 3, "bf16"),        # a single row: rings too short for the streaming dk/dv kernel
    (6, 2, 48, 64, 2, 3, "bf16"),
]
# shapes of the list whose three parts all run in the streaming kernels (slide_attn_bwd_variant
# 27), and those where dk/dv do not (26; 22 where the kernel gradients do not either)
BWD_STREAMING = {(3, 8, 56), (1, 20, 40), (40, 10, 56), (24, 17, 48), (2, 33, 40), (1, 57, 56), (3, 29, 48), (70, 12, 56), (66, 25, 48),
                 (150, 9, 48), (1, 150, 40), (2, 3, 56), (3, 5, 48), (5, 4, 40), (2, 6, 32)}
BWD_STREAMING_PIXEL_ONLY = {(2, 33, 32), (3, 40, 64), (1, 1, 56), (6, 2, 48)}


@pytest.mark.parametrize("shape", BWD_SHAPES)
def test_backward_matches_oracle(shape):
    B, H, W, C, heads, ksize, dtype = shape
    print("backward case", shape, flush=True)
    if dtype == "bf16":
        variant = sa.slide_attn_bwd_variant(B, H, W, C, heads, ksize, torch.bfloat16, True)
        want = 27 if (B, H, W) in BWD_STREAMING else ((26 if W <= 56 else 22) if (B, H, W) in BWD_STREAMING_PIXEL_ONLY else None)
        assert variant == want or (want is None and variant in (10, 20, 24)), variant
    d, g, n = gpu_problem(B, H, W, C, heads, ksize, dtype, seed=200 + H + W)
    grads = sa.slide_attn_bwd(g["dout"], g["q"], g["k"], g["v"], g["wk"], g["wv"], g["bias"], heads, ksize)
    torch.cuda.synchronize()
    ref = oracle.bwd(n["dout"], n["q"], n["k"], n["v"], n["wk"], n["wv"], n["bias"], heads, ksize)
    for name, got, want in zip(GRAD_NAMES, grads, ref):
        check(name, dtype, got, want)
    # run to run reproducible (fixed reduction order)
    again = sa.slide_attn_bwd(g["dout"], g["q"], g["k"], g["v"], g["wk"], g["wv"], g["bias"], heads, ksize)
    for a, b in zip(grads, again):
        assert torch.equal(a, b)
    # a caller that kept the forward's results may pass them: same gradients
    lse = torch.empty((B, heads, H, W), dtype=torch.float32, device=g["q"].device)
    out = sa.slide_attn_fwd(g["q"], g["k"], g["v"], g["wk"], g["wv"], g["bias"], heads, ksize, lse=lse)
    kept = sa.slide_attn_bwd(g["dout"], g["q"], g["k"], g["v"], g["wk"], g["wv"], g["bias"], heads, ksize,
                             out=out, lse=lse)
    for a, b in zip(grads, kept):
        assert torch.equal(a, b)


def _random_streaming_shapes(seed, count):
    """Seeded shapes in the range of the streaming kernels (widths 32..64, heights from one row
    to more than one band, one to three heads, up to a few hundred planes)."""
    import random
    rng = random.Random(seed)
    shapes = []
    for _ in range(count):
        W = rng.choice([32, 40, 48, 56, 64])
        H = rng.choice([1, 2, 3, 4, 5, 7, 9, 11, 13, 16, 19, 23, 27, 31, 37, 45, 61])
        heads = rng.choice([1, 2, 3])
        B = rng.choice([1, 2, 3, 5, 8, 13, 21, 40, 70, 130, 260])
        while B * H * W * heads > 250000:
            B = max(1, B // 2)
        shapes.append((B, H, W, 32 * heads, heads))
    return shapes


@pytest.mark.parametrize("shape", _random_streaming_shapes(3, 16))
def test_forward_and_backward_random_streaming_shapes(shape):
    """Forward (with the log of the softmax denominator) and all six gradients against the
    oracle on seeded random shapes, whichever kernels the dispatch picks for them."""
    B, H, W, C, heads = shape
    print("random streaming case", shape, "forward path", sa.slide_attn_fwd_path(B, H, W, C, heads, 3, torch.bfloat16),
          "backward variant", sa.slide_attn_bwd_variant(B, H, W, C, heads, 3, torch.bfloat16, True), flush=True)
    d, g, n = gpu_problem(B, H, W, C, heads, 3, "bf16", seed=7000 + B + 3 * H + 5 * W)
    lse = torch.empty((B, heads, H, W), dtype=torch.float32, device="cuda:0")
    out = sa.slide_attn_fwd(g["q"], g["k"], g["v"], g["wk"], g["wv"], g["bias"], heads, 3, lse=lse)
    grads = sa.slide_attn_bwd(g["dout"], g["q"], g["k"], g["v"], g["wk"], g["wv"], g["bias"], heads, 3)
    torch.cuda.synchronize()
    ref, ref_lse = oracle.fwd(n["q"], n["k"], n["v"], n["wk"], n["wv"], n["bias"], heads, 3, return_lse=True)
    check("out", "bf16", out, ref)
    check("lse", "bf16", lse, ref_lse)
    refg = oracle.bwd(n["dout"], n["q"], n["k"], n["v"], n["wk"], n["wv"], n["bias"], heads, 3)
    for name, got, want in zip(GRAD_NAMES, grads, refg):
        check(name, "bf16", got, want)


# heads narrower than 32 channels (bf16, 3x3): the backward runs the matrix-core kernels on
# copies padded to 32 channels per head (slide_attn_bwd_variant 100 + the variant of the padded problem)
NARROW_HEAD_SHAPES = [
    (2, 9, 40, 48, 2, 127),              # 24 channels per head (the head size of App. A's CSwin-like stages)
    (3, 20, 56, 72, 3, 127),
    (2, 14, 48, 16, 1, 127),             # 16
    (1, 7, 32, 24, 3, 126),              # 8 (too narrow a map for the streaming dk/dv kernel)
    (2, 13, 72, 48, 2, 120),             # wider than the streaming kernels take: tiled kernels
    (5, 3, 56, 24, 1, 127),
    (130, 5, 40, 48, 2, 127),            # 260 planes
    (2, 9, 21, 48, 2, 120),              # W % 8 != 0: not this path's kernel-gradient kernel ... general kernels
]


@pytest.mark.parametrize("shape", NARROW_HEAD_SHAPES)
def test_backward_narrow_heads(shape):
    B, H, W, C, heads, variant = shape
    print("narrow-head backward case", shape, flush=True)
    got_variant = sa.slide_attn_bwd_variant(B, H, W, C, heads, 3, torch.bfloat16, True)
    if W % 8 != 0:
        assert got_variant == 10
    else:
        assert got_variant == variant, got_variant
    assert sa.slide_attn_bwd_variant(B, H, W, C, heads, 3, torch.bfloat16, False) == 10
    d, g, n = gpu_problem(B, H, W, C, heads, 3, "bf16", seed=1200 + H + W + C)
    dev = g["q"].device
    grads = sa.slide_attn_bwd(g["dout"], g["q"], g["k"], g["v"], g["wk"], g["wv"], g["bias"], heads, 3)
    torch.cuda.synchronize()
    ref = oracle.bwd(n["dout"], n["q"], n["k"], n["v"], n["wk"], n["wv"], n["bias"], heads, 3)
    for name, got, want in zip(GRAD_NAMES, grads, ref):
        check(name, "bf16", got, want)
    again = sa.slide_attn_bwd(g["dout"], g["q"], g["k"], g["v"], g["wk"], g["wv"], g["bias"], heads, 3)
    for a, b in zip(grads, again):
        assert torch.equal(a, b)
    # training form with accumulation: learned kernels in, a second call doubles the parameter gradients
    wk_l, wv_l = d["wk_learned"].to(dev), d["wv_learned"].to(dev)
    tb = sa.slide_attn_bwd_two_branch(g["dout"], g["q"], g["k"], g["v"], wk_l, wv_l, g["bias"], heads, 3)
    for name, got, want in zip(GRAD_NAMES, tb, ref):
        check(name, "bf16", got, want)                 # (learned kernels in: the gradients are those of the merged form)
    first = [t.clone() for t in tb]
    acc = sa.slide_attn_bwd_two_branch(g["dout"], g["q"], g["k"], g["v"], wk_l, wv_l, g["bias"], heads, 3,
                                       outputs=tb, accumulate=True)
    for idx in range(3):
        assert torch.equal(acc[idx], first[idx])
    for idx in range(3, 6):
        assert torch.equal(acc[idx], 2 * first[idx])


def test_backward_unaligned_gradient_buffers_take_the_tiled_kernels():
    """dq, dk, dv that start 2 bytes into an allocation: the streaming kernels, which store 16
    bytes per lane, are not used; the results are those of the aligned call."""
    B, H, W, C, heads, ksize = 3, 12, 56, 64, 2, 3
    d, g, n = gpu_problem(B, H, W, C, heads, ksize, "bf16", seed=77)
    assert sa.slide_attn_bwd_variant(B, H, W, C, heads, ksize, torch.bfloat16, True) == 27
    ref = sa.slide_attn_bwd(g["dout"], g["q"], g["k"], g["v"], g["wk"], g["wv"], g["bias"], heads, ksize)
    numel = B * C * H * W
    views = []
    for _ in range(3):
        buf = torch.zeros(numel + 8, dtype=torch.bfloat16, device="cuda:0")
        view = buf[1:1 + numel].view(B, C, H, W)
        assert view.data_ptr() % 16 != 0
        views.append(view)
    outs = (views[0], views[1], views[2], torch.empty_like(g["wk"]), torch.empty_like(g["wv"]), torch.empty_like(g["bias"]))
    got = sa.slide_attn_bwd(g["dout"], g["q"], g["k"], g["v"], g["wk"], g["wv"], g["bias"], heads, ksize, outputs=outs)
    torch.cuda.synchronize()
    want = oracle.bwd(n["dout"], n["q"], n["k"], n["v"], n["wk"], n["wv"], n["bias"], heads, ksize)
    for name, a, b, w in zip(GRAD_NAMES, got, ref, want):
        check(name, "bf16", a, w)
        check(name, "bf16", b, w)


TWO_BRANCH_SHAPES = [
    # B, H, W, C, heads, ksize, dtype
    (1, 14, 14, 64, 2, 3, "f32"),        # general kernels
    (1, 6, 7, 24, 3, 5, "f32"),
    (2, 9, 21, 64, 2, 3, "bf16"),        # matrix-core forward, one tile per block; float32 workspace
    (2, 31, 24, 64, 2, 3, "bf16"),       # all backward kernels on the matrix cores
    (2, 17, 13, 128, 4, 5, "bf16"),      # 5x5 matrix-core forward, general backward
    (3, 21, 48, 64, 2, 3, "bf16"),       # streaming forward and streaming backward kernels
]


@pytest.mark.parametrize("shape", TWO_BRANCH_SHAPES)
def test_two_branch_form_matches_oracle(shape):
    """Training form (Sec. 4.3, Fig. 4(1)): the entry points that take the learned kernels and
    add the shift path themselves, against the oracle's two-branch forward and (the gradient
    with respect to the learned kernel being that with respect to the merged one) its backward."""
    B, H, W, C, heads, ksize, dtype = shape
    print("two-branch case", shape, flush=True)
    d, g, n = gpu_problem(B, H, W, C, heads, ksize, dtype, seed=300 + H + W)
    dev = g["q"].device
    wk_l, wv_l = d["wk_learned"].to(dev), d["wv_learned"].to(dev)
    lse = torch.empty((B, heads, H, W), dtype=torch.float32, device=dev)
    out = sa.slide_attn_fwd_two_branch(g["q"], g["k"], g["v"], wk_l, wv_l, g["bias"], heads, ksize, lse=lse)
    ref, ref_lse = oracle.fwd(n["q"], n["k"], n["v"], d["wk_learned"].double().numpy(),
                              d["wv_learned"].double().numpy(), n["bias"], heads, ksize,
                              two_branch=True, return_lse=True)
    check("out", dtype, out, ref)
    check("lse", dtype, lse, ref_lse)
    grads = sa.slide_attn_bwd_two_branch(g["dout"], g["q"], g["k"], g["v"], wk_l, wv_l, g["bias"], heads, ksize)
    ref_g = oracle.bwd(n["dout"], n["q"], n["k"], n["v"], n["wk"], n["wv"], n["bias"], heads, ksize)
    for name, got, want in zip(GRAD_NAMES, grads, ref_g):
        check(name, dtype, got, want)
    # accumulation over micro-batches: a second call adds the same parameter gradients again
    # (x + x is exact), the activation gradients are overwritten
    first = [t.clone() for t in grads]
    again = sa.slide_attn_bwd_two_branch(g["dout"], g["q"], g["k"], g["v"], wk_l, wv_l, g["bias"], heads, ksize,
                                         outputs=grads, accumulate=True)
    for idx in range(3):
        assert torch.equal(again[idx], first[idx])
    for idx in range(3, 6):
        assert torch.equal(again[idx], 2 * first[idx])


def test_two_branch_full_size_forward():
    """Stage-1 workload through the pipelined kernel, learned kernels in: whole planes of the
    first and last batch item against the oracle's two-branch form."""
    wl, d = synth.make_config_inputs(1)
    dev = torch.device("cuda:0")
    q, k, v = (d[x].to(dev).to(torch.bfloat16) for x in ("q", "k", "v"))
    wk_l, wv_l, bias = d["wk_learned"].to(dev), d["wv_learned"].to(dev), d["bias"].to(dev)
    out = sa.slide_attn_fwd_two_branch(q, k, v, wk_l, wv_l, bias, wl.heads, wl.ksize)
    torch.cuda.synchronize()
    out = out.float().cpu().numpy()
    for b in (0, wl.B - 1):
        sl = slice(b, b + 1)
        ref = oracle.fwd(d["q"][sl].numpy(), d["k"][sl].numpy(), d["v"][sl].numpy(),
                         d["wk_learned"].double().numpy(), d["wv_learned"].double().numpy(),
                         d["bias"].double().numpy(), wl.heads, wl.ksize, two_branch=True)
        assert np.abs(out[sl] - ref).max() <= 2e-2
    # and it is the merged form's result up to the last bf16 bit (1 + w is formed in float32
    # either way; a fused multiply-add in the operand preparation may round it differently)
    merged = sa.slide_attn_fwd(q, k, v, sa.slide_reparam(wk_l), sa.slide_reparam(wv_l), bias, wl.heads, wl.ksize)
    assert np.abs(merged.float().cpu().numpy() - out).max() <= 2.0 ** -7


def test_forward_unaligned_parameters_and_activations():
    """Pointers that are aligned to their element size only (4 bytes for the kernels, 2 for
    the activations): the forward must not take the paths that need 16-byte alignment."""
    B, H, W, C, heads, ksize = 32, 56, 56, 64, 2, 3                  # enough tiles for the pipelined kernel
    d, g, n = gpu_problem(B, H, W, C, heads, ksize, "bf16", seed=321)
    ref = oracle.fwd(n["q"], n["k"], n["v"], n["wk"], n["wv"], n["bias"], heads, ksize)

    def shifted(t, elems):
        buf = torch.empty(t.numel() + elems, dtype=t.dtype, device=t.device)
        view = buf[elems:].view(t.shape)
        view.copy_(t)
        return view

    wk1, wv1 = shifted(g["wk"], 1), shifted(g["wv"], 1)              # 4 bytes past a 16-byte boundary
    assert wk1.data_ptr() % 16 == 4
    out = sa.slide_attn_fwd(g["q"], g["k"], g["v"], wk1, wv1, g["bias"], heads, ksize)
    check("out (kernels at 4-byte alignment)", "bf16", out, ref)
    q1, k1, v1 = shifted(g["q"], 1), shifted(g["k"], 1), shifted(g["v"], 1)   # 2 bytes past
    out = sa.slide_attn_fwd(q1, k1, v1, g["wk"], g["wv"], g["bias"], heads, ksize)
    check("out (activations at 2-byte alignment)", "bf16", out, ref)


PIPELINED_SHAPES = [
    # B, H, W, C, heads, expected variant
    (90, 33, 48, 64, 2, 24),             # streaming kernel: ragged band split, 48 columns
    (100, 30, 40, 64, 2, 21),            # 40 columns: too much LDS for the streaming kernel, pipelined tiles
    (90, 31, 32, 64, 2, 24),             # 32 columns (groups of up to four new rows per epoch)
    (180, 24, 32, 32, 1, 24),            # one head, 32 columns
    (64, 24, 56, 64, 2, 24),             # stage-1 width, short planes
    (5, 9, 64, 96, 3, 24),               # 64 columns, three heads, one band per plane
    (3, 61, 56, 64, 2, 24),              # tall planes cut into many bands
    (256, 2, 64, 64, 2, 24),             # two-row planes: a band shorter than the window's reach
    (1, 1, 56, 32, 1, 24),               # a single row
    (12, 64, 72, 64, 2, 23),             # pipelined tiles of width 64, ragged second column tile
    # maps wider than 64 columns on the streaming kernel: column strips of 48, the last one moved
    # left to end with the map (columns computed twice), edge columns from the neighbouring strips
    (2, 9, 304, 96, 3, 26),
    (1, 20, 96, 32, 1, 26),              # two strips, no overlap
    (3, 5, 144, 64, 2, 26),
    (1, 33, 240, 32, 1, 26),
    (1, 1, 192, 32, 1, 26),              # a single row
    (2, 7, 432, 64, 2, 26),
    (4, 12, 200, 64, 2, 26),             # the last strip overlaps by 40 columns
    (2, 70, 128, 64, 2, 26),             # several bands per strip
    (3, 17, 80, 64, 2, 26),              # strips of 40
    (2, 9, 72, 64, 2, 26),               # two strips of 40 that overlap by 8 columns
    (4, 50, 104, 64, 2, 26),
    (300, 24, 24, 64, 2, 21),            # pipelined tiles, width from the arguments
    (700, 16, 16, 32, 1, 21),
    # enough tiles for the pipelined kernel, but tile buffers too small to build a head's
    # operand image in: must take the one-tile-per-block kernel
    (128, 8, 8, 128, 4, 20),
]


@pytest.mark.parametrize("shape", PIPELINED_SHAPES)
def test_forward_kernel_variants_match_oracle(shape):
    """Every kernel of the 3x3 matrix-core forward, asserted by the variant query, whole output
    and lse against the oracle."""
    B, H, W, C, heads, variant = shape
    print("variant case", shape, flush=True)
    assert sa.slide_attn_fwd_variant(B, H, W, C, heads, 3, torch.bfloat16, True) == variant
    d, g, n = gpu_problem(B, H, W, C, heads, 3, "bf16", seed=400 + H + W)
    for t in (g["q"], g["k"], g["v"], g["wk"], g["wv"]):
        assert t.data_ptr() % 16 == 0
    lse = torch.full((B, heads, H, W), float("nan"), dtype=torch.float32, device=g["q"].device)
    out = sa.slide_attn_fwd(g["q"], g["k"], g["v"], g["wk"], g["wv"], g["bias"], heads, 3, lse=lse)
    out_nl = sa.slide_attn_fwd(g["q"], g["k"], g["v"], g["wk"], g["wv"], g["bias"], heads, 3)
    torch.cuda.synchronize()
    assert torch.equal(out, out_nl)
    ref, ref_lse = oracle.fwd(n["q"], n["k"], n["v"], n["wk"], n["wv"], n["bias"], heads, 3, return_lse=True)
    check("out", "bf16", out, ref)
    check("lse", "bf16", lse, ref_lse)


# heads of 64 channels (the head size of the PVT-style stages of App. A): two launches of the
# streaming forward over half heads (slide_attn_fwd_variant 25)
WIDE_HEAD_SHAPES = [
    (2, 9, 40, 64, 1, 25),
    (3, 20, 56, 128, 2, 25),
    (4, 56, 56, 64, 1, 25),              # the stage-1 map
    (1, 1, 56, 64, 1, 25),
    (5, 33, 32, 128, 2, 25),
    (130, 5, 48, 64, 1, 25),
    (2, 13, 72, 64, 1, 10),              # wider than the streaming kernel takes: general kernel
    (2, 9, 21, 64, 1, 10),
]


@pytest.mark.parametrize("shape", WIDE_HEAD_SHAPES)
def test_forward_heads_of_64_channels(shape):
    B, H, W, C, heads, variant = shape
    print("wide-head forward case", shape, flush=True)
    assert sa.slide_attn_fwd_variant(B, H, W, C, heads, 3, torch.bfloat16, True) == variant
    d, g, n = gpu_problem(B, H, W, C, heads, 3, "bf16", seed=1400 + H + W + C)
    dev = g["q"].device
    lse = torch.full((B, heads, H, W), float("nan"), dtype=torch.float32, device=dev)
    out = sa.slide_attn_fwd(g["q"], g["k"], g["v"], g["wk"], g["wv"], g["bias"], heads, 3, lse=lse)
    out_nl = sa.slide_attn_fwd(g["q"], g["k"], g["v"], g["wk"], g["wv"], g["bias"], heads, 3)
    torch.cuda.synchronize()
    assert torch.equal(out, out_nl)
    ref, ref_lse = oracle.fwd(n["q"], n["k"], n["v"], n["wk"], n["wv"], n["bias"], heads, 3, return_lse=True)
    check("out", "bf16", out, ref)
    check("lse", "bf16", lse, ref_lse)
    # no bias; learned kernels in (training form)
    out0 = sa.slide_attn_fwd(g["q"], g["k"], g["v"], g["wk"], g["wv"], None, heads, 3)
    check("out(no bias)", "bf16", out0, oracle.fwd(n["q"], n["k"], n["v"], n["wk"], n["wv"], None, heads, 3))
    out2 = sa.slide_attn_fwd_two_branch(g["q"], g["k"], g["v"], d["wk_learned"].to(dev), d["wv_learned"].to(dev),
                                        g["bias"], heads, 3)
    check("out(two-branch)", "bf16", out2, ref)
    # a caller without workspace for the partial logits gets the general kernel: same result within the tolerance
    small = torch.empty(16, dtype=torch.uint8, device=dev)
    out_g = sa.slide_attn_fwd(g["q"], g["k"], g["v"], g["wk"], g["wv"], g["bias"], heads, 3, workspace=small)
    check("out(general kernel)", "bf16", out_g, ref)


# forward of heads narrower than 32 channels on padded copies (slide_attn_fwd_variant 100 + the
# variant of the padded problem); head size 24 on the streaming kernel's maps runs there directly
NARROW_HEAD_FWD_SHAPES = [
    (2, 8, 40, 32, 2, 124),              # 16 channels per head
    (3, 20, 56, 24, 3, 124),             # 8
    (2, 12, 72, 48, 2, 126),             # 24 on a map wider than 64 columns: padded, then column strips
    (2, 12, 172, 48, 2, 120),            # ... W % 8 != 0: padded, then one tile per block
    (2, 56, 56, 48, 2, 24),              # 24 on the streaming kernel itself
    (2, 9, 21, 48, 2, 10),               # H * W % 8 != 0: general kernel
]


@pytest.mark.parametrize("shape", NARROW_HEAD_FWD_SHAPES)
def test_forward_narrow_heads(shape):
    B, H, W, C, heads, variant = shape
    print("narrow-head forward case", shape, flush=True)
    assert sa.slide_attn_fwd_variant(B, H, W, C, heads, 3, torch.bfloat16, True) == variant
    d, g, n = gpu_problem(B, H, W, C, heads, 3, "bf16", seed=1600 + H + W + C)
    dev = g["q"].device
    lse = torch.full((B, heads, H, W), float("nan"), dtype=torch.float32, device=dev)
    out = sa.slide_attn_fwd(g["q"], g["k"], g["v"], g["wk"], g["wv"], g["bias"], heads, 3, lse=lse)
    torch.cuda.synchronize()
    ref, ref_lse = oracle.fwd(n["q"], n["k"], n["v"], n["wk"], n["wv"], n["bias"], heads, 3, return_lse=True)
    check("out", "bf16", out, ref)
    check("lse", "bf16", lse, ref_lse)
    out2 = sa.slide_attn_fwd_two_branch(g["q"], g["k"], g["v"], d["wk_learned"].to(dev), d["wv_learned"].to(dev),
                                        g["bias"], heads, 3)
    check("out(two-branch)", "bf16", out2, ref)
    # without the workspace for the padded copies: the general kernel
    small = torch.empty(16, dtype=torch.uint8, device=dev)
    if variant >= 100:
        out_g = sa.slide_attn_fwd(g["q"], g["k"], g["v"], g["wk"], g["wv"], g["bias"], heads, 3, workspace=small)
        check("out(general kernel)", "bf16", out_g, ref)


# backward of heads of 64 channels: half heads through the matrix-core kernels, the per-pixel part in
# two launches that exchange the halves' shares of logits and da (slide_attn_bwd_variant 200 + ...)
WIDE_HEAD_BWD_SHAPES = [
    (2, 9, 40, 64, 1, 227),
    (3, 20, 56, 128, 2, 227),
    (2, 33, 32, 64, 1, 226),             # tiled dk/dv kernel
    (1, 5, 64, 64, 1, 222),              # 64 columns: only the per-pixel part streams
    (130, 5, 48, 64, 1, 227),
    (4, 56, 56, 64, 1, 227),             # the stage-1 map
    (2, 13, 72, 64, 1, 10),              # wider than the streaming per-pixel kernel takes: general kernels
]


@pytest.mark.parametrize("shape", WIDE_HEAD_BWD_SHAPES)
def test_backward_heads_of_64_channels(shape):
    B, H, W, C, heads, variant = shape
    print("wide-head backward case", shape, flush=True)
    assert sa.slide_attn_bwd_variant(B, H, W, C, heads, 3, torch.bfloat16, True) == variant
    assert sa.slide_attn_bwd_variant(B, H, W, C, heads, 3, torch.bfloat16, False) == 10
    d, g, n = gpu_problem(B, H, W, C, heads, 3, "bf16", seed=1500 + H + W + C)
    dev = g["q"].device
    grads = sa.slide_attn_bwd(g["dout"], g["q"], g["k"], g["v"], g["wk"], g["wv"], g["bias"], heads, 3)
    torch.cuda.synchronize()
    ref = oracle.bwd(n["dout"], n["q"], n["k"], n["v"], n["wk"], n["wv"], n["bias"], heads, 3)
    for name, got, want in zip(GRAD_NAMES, grads, ref):
        check(name, "bf16", got, want)
    again = sa.slide_attn_bwd(g["dout"], g["q"], g["k"], g["v"], g["wk"], g["wv"], g["bias"], heads, 3)
    for a, b in zip(grads, again):
        assert torch.equal(a, b)
    wk_l, wv_l = d["wk_learned"].to(dev), d["wv_learned"].to(dev)
    tb = sa.slide_attn_bwd_two_branch(g["dout"], g["q"], g["k"], g["v"], wk_l, wv_l, g["bias"], heads, 3)
    for name, got, want in zip(GRAD_NAMES, tb, ref):
        check(name, "bf16", got, want)
    first = [t.clone() for t in tb]
    acc = sa.slide_attn_bwd_two_branch(g["dout"], g["q"], g["k"], g["v"], wk_l, wv_l, g["bias"], heads, 3,
                                       outputs=tb, accumulate=True)
    for idx in range(3):
        assert torch.equal(acc[idx], first[idx])
    for idx in range(3, 6):
        assert torch.equal(acc[idx], 2 * first[idx])


def test_kernel_selection():
    """Which forward kernel serves which problem (host-side query of the C ABI)."""
    assert sa.slide_attn_fwd_variant(64, 56, 56, 64, 2, 3, torch.bfloat16, True) == 24
    assert sa.slide_attn_fwd_variant(64, 56, 56, 64, 2, 3, torch.bfloat16, False) == 20
    assert sa.slide_attn_fwd_variant(2, 200, 304, 96, 3, 3, torch.bfloat16, True) == 26
    assert sa.slide_attn_fwd_path(64, 56, 56, 64, 2, 3, torch.bfloat16) == 2
    assert sa.slide_attn_fwd_path(64, 28, 28, 128, 4, 5, torch.bfloat16) == 3
    assert sa.slide_attn_fwd_path(1, 14, 14, 64, 2, 3, torch.float32) == 1
    assert sa.slide_attn_fwd_path(1, 14, 14, 48, 2, 3, torch.bfloat16) == 1


def sample_positions(B, heads, H, W, n, seed):
    rng = np.random.default_rng(seed)
    pos = np.stack([rng.integers(0, B, n), rng.integers(0, heads, n),
                    rng.integers(0, H, n), rng.integers(0, W, n)], axis=1)
    # always include the four corners and edge midpoints of the first and last plane
    extra = []
    for b, m in ((0, 0), (B - 1, heads - 1)):
        for i in (0, H // 2, H - 1):
            for j in (0, W // 2, W - 1):
                extra.append((b, m, i, j))
    return np.concatenate([np.array(extra), pos]).astype(np.int32)


@pytest.mark.parametrize("index", [1, 2, 3])
def test_forward_full_size_configs_sampled(index):
    """Benchmark configurations 2-4 at full size, in the launch configuration the
    benchmark times; outputs compared with the oracle at sampled pixels."""
    wl, d = synth.make_config_inputs(index)
    print("full-size forward", wl, flush=True)
    dev = torch.device("cuda:0")
    q, k, v = (d[x].to(dev).to(tdtype(wl.dtype)) for x in ("q", "k", "v"))
    wk = sa.slide_reparam(d["wk_learned"].to(dev))
    wv = sa.slide_reparam(d["wv_learned"].to(dev))
    bias = d["bias"].to(dev)
    out = sa.slide_attn_fwd(q, k, v, wk, wv, bias, wl.heads, wl.ksize)
    torch.cuda.synchronize()
    out = out.float().cpu().numpy()
    assert np.isfinite(out).all()
    pos = sample_positions(wl.B, wl.heads, wl.H, wl.W, 1500, seed=index)
    ref = oracle.fwd_samples(d["q"].numpy(), d["k"].numpy(), d["v"].numpy(),
                             wk.double().cpu().numpy(), wv.double().cpu().numpy(),
                             d["bias"].double().numpy(), wl.heads, wl.ksize, pos)
    dd = wl.C // wl.heads
    got = np.stack([out[b, m * dd:(m + 1) * dd, i, j] for b, m, i, j in pos])
    err = np.abs(got - ref).max()
    assert err <= 2e-2, err
    # the same launch with the log of the softmax denominator as a second result
    lse = torch.full((wl.B, wl.heads, wl.H, wl.W), float("nan"), dtype=torch.float32, device=dev)
    out_l = sa.slide_attn_fwd(q, k, v, wk, wv, bias, wl.heads, wl.ksize, lse=lse)
    torch.cuda.synchronize()
    assert np.array_equal(out_l.float().cpu().numpy(), out)
    lse = lse.cpu().numpy()
    assert np.isfinite(lse).all()
    # whole planes of the first and last batch item, element by element
    for b in (0, wl.B - 1):
        sl = slice(b, b + 1)
        refp, ref_lse = oracle.fwd(d["q"][sl].numpy(), d["k"][sl].numpy(), d["v"][sl].numpy(),
                                   wk.double().cpu().numpy(), wv.double().cpu().numpy(),
                                   d["bias"].double().numpy(), wl.heads, wl.ksize, return_lse=True)
        assert np.abs(out[sl] - refp).max() <= 2e-2
        assert np.abs(lse[sl] - ref_lse).max() <= 2e-2


def test_training_config_full_size():
    """Benchmark configuration 5 (B=128 forward + backward) at full size.  Activation
    gradients of three batch items are compared element by element (batch items are
    independent); parameter gradients are checked through additivity over the batch
    (dW(full) = dW(first half) + dW(second half)) and against the oracle on a
    sub-batch."""
    wl, d = synth.make_config_inputs(4)
    print("full-size training", wl, flush=True)
    assert sa.slide_attn_bwd_variant(wl.B, wl.H, wl.W, wl.C, wl.heads, wl.ksize, torch.bfloat16, True) == 27
    dev = torch.device("cuda:0")
    t = {x: d[x].to(dev).to(torch.bfloat16) for x in ("q", "k", "v", "dout")}
    wk = sa.slide_reparam(d["wk_learned"].to(dev))
    wv = sa.slide_reparam(d["wv_learned"].to(dev))
    bias = d["bias"].to(dev)
    out = sa.slide_attn_fwd(t["q"], t["k"], t["v"], wk, wv, bias, wl.heads, wl.ksize)
    full = sa.slide_attn_bwd(t["dout"], t["q"], t["k"], t["v"], wk, wv, bias, wl.heads, wl.ksize)
    torch.cuda.synchronize()
    wkn, wvn, bn = wk.double().cpu().numpy(), wv.double().cpu().numpy(), d["bias"].double().numpy()
    for b in (0, 77, wl.B - 1):
        sl = slice(b, b + 1)
        n = {x: d[x][sl].double().numpy() for x in ("q", "k", "v", "dout")}
        ref_out = oracle.fwd(n["q"], n["k"], n["v"], wkn, wvn, bn, wl.heads, wl.ksize)
        assert np.abs(out[sl].double().cpu().numpy() - ref_out).max() <= 2e-2
        ref = oracle.bwd(n["dout"], n["q"], n["k"], n["v"], wkn, wvn, bn, wl.heads, wl.ksize)
        for name, got, want in zip(GRAD_NAMES[:3], full[:3], ref[:3]):
            check(name, "bf16", got[sl], want)
    # parameter gradients of the whole batch against the oracle (every block of the
    # kernel-gradient kernel walks through 19 work units here)
    nall = {x: d[x].double().numpy() for x in ("q", "k", "v", "dout")}
    ref_all = oracle.bwd(nall["dout"], nall["q"], nall["k"], nall["v"], wkn, wvn, bn, wl.heads, wl.ksize)
    del nall
    for name, got, want in zip(GRAD_NAMES[3:], full[3:], ref_all[3:]):
        err = check(name, "bf16", got, want)
        print("config 5 %s: strict max abs err %.3e, max |oracle| %.3e" % (name, err, np.abs(want).max()), flush=True)
    del ref_all
    half = wl.B // 2
    parts = []
    for sl in (slice(0, half), slice(half, wl.B)):
        parts.append(sa.slide_attn_bwd(t["dout"][sl].contiguous(), t["q"][sl].contiguous(),
                                       t["k"][sl].contiguous(), t["v"][sl].contiguous(),
                                       wk, wv, bias, wl.heads, wl.ksize))
    for idx in (3, 4, 5):
        total = parts[0][idx].double() + parts[1][idx].double()
        scale = max(1.0, float(total.abs().max()))
        assert float((full[idx].double() - total).abs().max()) <= 1e-4 * scale
    # oracle on the first 4 items against a GPU run on the same 4 items
    sl = slice(0, 4)
    sub = sa.slide_attn_bwd(t["dout"][sl].contiguous(), t["q"][sl].contiguous(),
                            t["k"][sl].contiguous(), t["v"][sl].contiguous(),
                            wk, wv, bias, wl.heads, wl.ksize)
    n = {x: d[x][sl].double().numpy() for x in ("q", "k", "v", "dout")}
    ref = oracle.bwd(n["dout"], n["q"], n["k"], n["v"], wkn, wvn, bn, wl.heads, wl.ksize)
    for name, got, want in zip(GRAD_NAMES, sub, ref):
        check(name, "bf16", got, want)
