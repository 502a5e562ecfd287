"""The number-format contract of the bf16 matrix-core paths (stated in include/slide_attn.h):
inside the kernels activations and kernels are IEEE halves, products are formed from q/16 and
dout/16, sums are float32.  Inside the contract (|x| <= 2^15, |q k| < 2^20) results meet the
bf16 tolerance relative to max(1, |result|); outside it values saturate at +-65504 or flush
to zero, nothing is rejected and nothing becomes infinite or NaN."""
import numpy as np
import pytest
import torch

import paper_2304_04237_amd as sa
from paper_2304_04237_amd import synth
from oracle import slide_oracle as oracle

pytestmark = pytest.mark.gpu

GRAD_NAMES = "dq dk dv dwk dwv dbias".split()
SHAPES = [(2, 12, 24, 64, 2, 3), (1, 9, 16, 32, 1, 5)]


def _scaled_problem(shape, qs, ks, vs, dos, seed):
    B, H, W, C, heads, ksize = shape
    d = synth.make_inputs(B, H, W, C, heads, ksize, "bf16", seed=seed)
    # powers of two: the scaled values are still exactly representable in bf16
    for name, f in (("q", qs), ("k", ks), ("v", vs), ("dout", dos)):
        d[name] = d[name] * f
        assert torch.equal(d[name], d[name].to(torch.bfloat16).float())
    dev = torch.device("cuda:0")
    g = {n: d[n].to(dev).to(torch.bfloat16) for n in ("q", "k", "v", "dout")}
    g["wk"] = sa.slide_reparam(d["wk_learned"].to(dev))
    g["wv"] = sa.slide_reparam(d["wv_learned"].to(dev))
    g["bias"] = d["bias"].to(dev)
    n = {x: d[x].double().numpy() for x in ("q", "k", "v", "dout", "bias")}
    n["wk"], n["wv"] = g["wk"].double().cpu().numpy(), g["wv"].double().cpu().numpy()
    return g, n


def _rel_check(name, got, want):
    got = got.detach().double().cpu().numpy()
    assert np.isfinite(got).all(), name
    err = float(np.abs(got - want).max())
    bound = 2e-2 * max(1.0, float(np.abs(want).max()))
    assert err <= bound, "%s: max abs err %.3e > %.3e" % (name, err, bound)


@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("scales", [
    # q, k, v, dout
    (1.0, 1.0, 64.0, 64.0),          # large values and upstream gradients
    (1.0, 1.0, 1 / 64.0, 1 / 64.0),  # small ones
    (8.0, 1 / 8.0, 4.0, 1.0),        # q and k far apart, logits as in the recipe
    (1 / 64.0, 1 / 64.0, 1.0, 1.0),  # tiny logits: attention close to uniform
    (2.0, 2.0, 512.0, 1 / 512.0),    # peaked softmax (logits x4), big v, small dout
])
def test_inside_the_contract_far_from_unit_scale(shape, scales):
    print("number format case", shape, scales, flush=True)
    B, H, W, C, heads, ksize = shape
    g, n = _scaled_problem(shape, *scales, seed=500 + H)
    out = sa.slide_attn_fwd(g["q"], g["k"], g["v"], g["wk"], g["wv"], g["bias"], heads, ksize)
    ref = oracle.fwd(n["q"], n["k"], n["v"], n["wk"], n["wv"], n["bias"], heads, ksize)
    _rel_check("out", out, ref)
    grads = sa.slide_attn_bwd(g["dout"], g["q"], g["k"], g["v"], g["wk"], g["wv"], g["bias"], heads, ksize)
    refg = oracle.bwd(n["dout"], n["q"], n["k"], n["v"], n["wk"], n["wv"], n["bias"], heads, ksize)
    for name, a, w in zip(GRAD_NAMES, grads, refg):
        _rel_check(name, a, w)


@pytest.mark.parametrize("shape", SHAPES)
def test_values_below_half_precision_normal_range(shape):
    """bf16 values below 2^-17 (v and k scaled by 2^-20): half precision holds them as
    multiples of 2^-24, so each value moves by less than 2^-24; results stay within the
    absolute tolerance and finite."""
    B, H, W, C, heads, ksize = shape
    g, n = _scaled_problem(shape, 1.0, 2.0 ** -20, 2.0 ** -20, 1.0, seed=600 + H)
    assert float(g["v"].float().abs().max()) < 2.0 ** -17
    out = sa.slide_attn_fwd(g["q"], g["k"], g["v"], g["wk"], g["wv"], g["bias"], heads, ksize)
    ref = oracle.fwd(n["q"], n["k"], n["v"], n["wk"], n["wv"], n["bias"], heads, ksize)
    got = out.double().cpu().numpy()
    assert np.isfinite(got).all()
    # every v moved by < 2^-24 and the weights sum to one (plus learned taps of size 0.02)
    assert np.abs(got - ref).max() <= 2.0 ** -23
    grads = sa.slide_attn_bwd(g["dout"], g["q"], g["k"], g["v"], g["wk"], g["wv"], g["bias"], heads, ksize)
    refg = oracle.bwd(n["dout"], n["q"], n["k"], n["v"], n["wk"], n["wv"], n["bias"], heads, ksize)
    for name, a, w in zip(GRAD_NAMES, grads, refg):
        _rel_check(name, a, w)


def test_outside_the_contract_saturates_and_stays_finite():
    """Activations above 65504 are outside the contract: documented behaviour is saturation
    at +-65504 on the way in, no infinity, no NaN, no error."""
    shape = (1, 8, 16, 32, 1, 3)
    B, H, W, C, heads, ksize = shape
    g, n = _scaled_problem(shape, 1.0, 1.0, 2.0 ** 18, 1.0, seed=77)
    assert float(g["v"].float().abs().max()) > 65504
    zero_w = sa.slide_reparam(torch.zeros_like(g["wv"]))
    bias = torch.zeros(heads, 9, device=g["q"].device)
    bias[:, 4] = 1e4                                  # the centre shift takes all the weight: out = v
    out = sa.slide_attn_fwd(g["q"], g["k"], g["v"], zero_w, zero_w, bias, heads, ksize)
    got = out.float()
    assert torch.isfinite(got).all()
    expect = g["v"].float().clamp(-65504.0, 65504.0).to(torch.bfloat16).float()
    assert torch.equal(got, expect)
