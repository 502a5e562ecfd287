"""Seeded sweeps of shapes through every entry point, against the CPU oracle: forward (with
the log of the softmax denominator), the training-form forward, the backward in both forms,
all six gradients.  Shapes are drawn from a fixed seed: window sizes 1, 3, 5, 7, head sizes
8, 16, 24, 32, float32 and bfloat16, ragged and 8-aligned widths, one to three heads.
Tolerances as in test_gpu_parity.py."""
import numpy as np
import pytest
import torch

import paper_2304_04237_amd as sa
from paper_2304_04237_amd import synth
from oracle import slide_oracle as oracle

pytestmark = pytest.mark.gpu

GRAD_NAMES = "dq dk dv dwk dwv dbias".split()


def _bound(dtype, want, relative):
    mx = float(np.abs(want).max())
    if dtype == "f32":
        return 1e-5 * mx
    return 2e-2 * max(1.0, mx) if relative else 2e-2


def _check(case, name, dtype, got, want, relative=False):
    got = got.detach().double().cpu().numpy()
    assert got.shape == want.shape, (case, name)
    assert np.isfinite(got).all(), (case, name)
    err = float(np.abs(got - want).max())
    bound = _bound(dtype, want, relative)
    assert err <= bound, "%s %s: max abs err %.3e > %.3e" % (case, name, err, bound)
    return err / max(bound, 1e-300)


def _random_cases(n, seed):
    rng = np.random.default_rng(seed)
    cases = []
    for it in range(n):
        ks = int(rng.choice([1, 3, 3, 3, 5, 7]))
        dtype = str(rng.choice(["f32", "bf16", "bf16"]))
        heads = int(rng.integers(1, 4))
        d = int(rng.choice([32, 32, 32, 8, 24, 16]))
        H = int(rng.integers(1, 40))
        W = int(rng.choice([int(rng.integers(1, 80)), 8 * int(rng.integers(1, 11))]))
        B = int(rng.integers(1, 4))
        if ks == 7 and H * W * heads * d > 20000:
            H, W = 5, 6
        cases.append((B, H, W, heads * d, heads, ks, dtype, 900 + it))
    return cases


@pytest.mark.parametrize("chunk", range(4))
def test_random_shapes_all_entry_points(chunk):
    dev = torch.device("cuda:0")
    worst = 0.0
    for case in _random_cases(40, seed=7)[10 * chunk:10 * chunk + 10]:
        B, H, W, C, heads, ks, dtype, seed = case
        print("sweep case", case, flush=True)
        dd = synth.make_inputs(B, H, W, C, heads, ks, dtype, seed=seed, with_dout=True)
        tdt = torch.float32 if dtype == "f32" else torch.bfloat16
        g = {n: dd[n].to(dev).to(tdt) for n in ("q", "k", "v", "dout")}
        wk_l, wv_l, bias = dd["wk_learned"].to(dev), dd["wv_learned"].to(dev), dd["bias"].to(dev)
        wk, wv = sa.slide_reparam(wk_l), sa.slide_reparam(wv_l)
        n = {x: dd[x].double().numpy() for x in ("q", "k", "v", "dout", "bias")}
        wkn, wvn = wk.double().cpu().numpy(), wv.double().cpu().numpy()
        lse = torch.empty((B, heads, H, W), dtype=torch.float32, device=dev)
        out = sa.slide_attn_fwd(g["q"], g["k"], g["v"], wk, wv, bias, heads, ks, lse=lse)
        out2 = sa.slide_attn_fwd_two_branch(g["q"], g["k"], g["v"], wk_l, wv_l, bias, heads, ks)
        ref, ref_lse = oracle.fwd(n["q"], n["k"], n["v"], wkn, wvn, n["bias"], heads, ks, return_lse=True)
        worst = max(worst, _check(case, "out", dtype, out, ref), _check(case, "out (two-branch)", dtype, out2, ref),
                    _check(case, "lse", dtype, lse, ref_lse))
        grads = sa.slide_attn_bwd(g["dout"], g["q"], g["k"], g["v"], wk, wv, bias, heads, ks)
        grads2 = sa.slide_attn_bwd_two_branch(g["dout"], g["q"], g["k"], g["v"], wk_l, wv_l, bias, heads, ks)
        refg = oracle.bwd(n["dout"], n["q"], n["k"], n["v"], wkn, wvn, n["bias"], heads, ks)
        for nm, a, b, w in zip(GRAD_NAMES, grads, grads2, refg):
            rel = nm in ("dwk", "dwv", "dbias")
            worst = max(worst, _check(case, nm, dtype, a, w, rel), _check(case, nm + " (two-branch)", dtype, b, w, rel))
    print("worst error / bound = %.3f" % worst, flush=True)


LARGE_SHAPES = [
    # B, H, W, C, heads: bf16, 3x3, head size 32 -- the matrix-core kernels on maps with several
    # column tiles, ragged last columns, tall planes
    (16, 64, 72, 64, 2), (8, 100, 128, 32, 1), (4, 96, 200, 96, 3), (40, 40, 40, 64, 2),
    (3, 333, 64, 32, 1), (2, 131, 264, 64, 2), (64, 24, 56, 64, 2), (6, 77, 136, 64, 2),
]


@pytest.mark.parametrize("shape", LARGE_SHAPES)
def test_large_shapes_forward_and_all_gradients(shape):
    B, H, W, C, heads = shape
    case = shape + (3, "bf16")
    print("large case", case, "variant", sa.slide_attn_fwd_variant(B, H, W, C, heads, 3, torch.bfloat16), flush=True)
    dev = torch.device("cuda:0")
    dd = synth.make_inputs(B, H, W, C, heads, 3, "bf16", seed=700 + H + W, with_dout=True)
    g = {n: dd[n].to(dev).to(torch.bfloat16) for n in ("q", "k", "v", "dout")}
    wk, wv = sa.slide_reparam(dd["wk_learned"].to(dev)), sa.slide_reparam(dd["wv_learned"].to(dev))
    bias = dd["bias"].to(dev)
    lse = torch.empty((B, heads, H, W), dtype=torch.float32, device=dev)
    out = sa.slide_attn_fwd(g["q"], g["k"], g["v"], wk, wv, bias, heads, 3, lse=lse)
    out_nl = sa.slide_attn_fwd(g["q"], g["k"], g["v"], wk, wv, bias, heads, 3)
    grads = sa.slide_attn_bwd(g["dout"], g["q"], g["k"], g["v"], wk, wv, bias, heads, 3)
    torch.cuda.synchronize()
    assert torch.equal(out, out_nl)
    n = {x: dd[x].double().numpy() for x in ("q", "k", "v", "dout", "bias")}
    wkn, wvn = wk.double().cpu().numpy(), wv.double().cpu().numpy()
    ref, ref_lse = oracle.fwd(n["q"], n["k"], n["v"], wkn, wvn, n["bias"], heads, 3, return_lse=True)
    _check(case, "out", "bf16", out, ref)
    _check(case, "lse", "bf16", lse, ref_lse)
    refg = oracle.bwd(n["dout"], n["q"], n["k"], n["v"], wkn, wvn, n["bias"], heads, 3)
    for nm, a, w in zip(GRAD_NAMES, grads, refg):
        _check(case, nm, "bf16", a, w, nm in ("dwk", "dwv", "dbias"))
