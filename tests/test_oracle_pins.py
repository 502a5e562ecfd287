"""Pins of the CPU oracle against things other than itself (no GPU needed).

Each test names what it pins.  Sources of truth: the paper's definitions (column
view of Im2Col, shift as one-hot depthwise convolution, two-branch vs merged
kernels), closed forms, library routines of CPU PyTorch (unfold, grouped
conv2d, avg_pool2d, softmax, float64 autograd) and finite differences.
"""
import math
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import slide_oracle as oracle
from tests.bruteforce_im2col import local_attention as brute_local_attention

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")

SHAPES = [
    # B, H, W, C, heads, ksize
    (1, 4, 5, 4, 2, 3),
    (2, 3, 2, 4, 1, 5),     # H, W smaller than the window
    (1, 1, 1, 2, 1, 3),
    (1, 2, 5, 4, 2, 3),
    (1, 3, 3, 2, 2, 1),
    (1, 5, 3, 2, 1, 5),
]


def rand_problem(B, H, W, C, heads, ksize, seed, w_std=0.3, bias_std=0.5):
    rng = np.random.default_rng(seed)
    S = ksize * ksize
    q, k, v, do = (rng.standard_normal((B, C, H, W)) for _ in range(4))
    wk = rng.standard_normal((C, S, ksize, ksize)) * w_std
    wv = rng.standard_normal((C, S, ksize, ksize)) * w_std
    bias = rng.standard_normal((heads, S)) * bias_std
    return q, k, v, do, wk, wv, bias


def torch_forward(q, k, v, wk_m, wv_m, bias, heads, ksize):
    """Library-routine statement of the operator: grouped conv2d + softmax (float64)."""
    B, C, H, W = q.shape
    S = ksize * ksize
    d = C // heads
    r = ksize // 2
    Ks = F.conv2d(k, wk_m.reshape(C * S, 1, ksize, ksize), padding=r, groups=C)
    Vs = F.conv2d(v, wv_m.reshape(C * S, 1, ksize, ksize), padding=r, groups=C)
    Ks = Ks.reshape(B, heads, d, S, H, W)
    Vs = Vs.reshape(B, heads, d, S, H, W)
    qh = q.reshape(B, heads, d, 1, H, W)
    logits = (qh * Ks).sum(2) / math.sqrt(d) + bias[None, :, :, None, None]
    a = torch.softmax(logits, dim=2)
    out = (a.unsqueeze(2) * Vs).sum(3).reshape(B, C, H, W)
    return out, a


# ---------------------------------------------------------------- P11: Fig. 2 structure
def test_fig2_key_matrix_structure():
    """Row view (Eq. 8-9) of the 3x3 / 2x2 example equals the hand-written matrix."""
    expected = np.loadtxt(os.path.join(GOLDEN, "fig2_key_matrix.txt"))
    assert expected.shape == (9, 4)
    kmap = np.array([[1.0, 2.0], [3.0, 4.0]]).reshape(1, 1, 2, 2)
    zero_w = np.zeros((1, 9, 3, 3))
    rows = oracle.deformed_shift(kmap, zero_w, 3, two_branch=True)      # shift path only
    assert np.array_equal(rows.reshape(9, 4), expected)
    merged = oracle.reparam(zero_w, 3)
    rows_m = oracle.deformed_shift(kmap, merged, 3, two_branch=False)   # one-hot kernels
    assert np.array_equal(rows_m.reshape(9, 4), expected)
    # column view: column (i,j) is the flattened window centred on (i,j)  (Eq. 7)
    assert np.array_equal(expected[:, 0], [0, 0, 0, 0, 1, 2, 0, 3, 4])


# ---------------------------------------------------------------- P1: brute force
@pytest.mark.parametrize("shape", SHAPES)
def test_forward_matches_bruteforce_im2col(shape):
    B, H, W, C, heads, ksize = shape
    q, k, v, _, wk, wv, bias = rand_problem(*shape, seed=11)
    ref_out, ref_attn = brute_local_attention(q, k, v, wk, wv, bias, heads, ksize)
    out2, attn2 = oracle.fwd(q, k, v, wk, wv, bias, heads, ksize, two_branch=True, return_attn=True)
    np.testing.assert_allclose(out2, ref_out, rtol=0, atol=1e-12)
    np.testing.assert_allclose(attn2, ref_attn, rtol=0, atol=1e-12)
    outm = oracle.fwd(q, k, v, oracle.reparam(wk, ksize), oracle.reparam(wv, ksize), bias, heads, ksize)
    np.testing.assert_allclose(outm, ref_out, rtol=0, atol=1e-12)


def test_zero_learned_kernels_is_textbook_neighbourhood_attention():
    """w = 0: keys/values are the unfolded (Im2Col) windows; checked with F.unfold."""
    B, H, W, C, heads, ksize = 2, 5, 4, 6, 3, 3
    q, k, v, _, _, _, bias = rand_problem(B, H, W, C, heads, ksize, seed=5)
    S, d = ksize * ksize, C // heads
    zero = np.zeros((C, S, ksize, ksize))
    out = oracle.fwd(q, k, v, zero, zero, bias, heads, ksize, two_branch=True)
    tq, tk, tv = (torch.from_numpy(x) for x in (q, k, v))
    ku = F.unfold(tk, ksize, padding=ksize // 2).reshape(B, heads, d, S, H, W)
    vu = F.unfold(tv, ksize, padding=ksize // 2).reshape(B, heads, d, S, H, W)
    logits = (tq.reshape(B, heads, d, 1, H, W) * ku).sum(2) / math.sqrt(d)
    logits = logits + torch.from_numpy(bias)[None, :, :, None, None]
    a = torch.softmax(logits, dim=2)
    ref = (a.unsqueeze(2) * vu).sum(3).reshape(B, C, H, W).numpy()
    np.testing.assert_allclose(out, ref, rtol=0, atol=1e-12)


# ---------------------------------------------------------------- P2: two-branch == merged
@pytest.mark.parametrize("shape", SHAPES)
def test_two_branch_equals_merged(shape):
    B, H, W, C, heads, ksize = shape
    q, k, v, _, wk, wv, bias = rand_problem(*shape, seed=3)
    a = oracle.fwd(q, k, v, wk, wv, bias, heads, ksize, two_branch=True)
    b = oracle.fwd(q, k, v, oracle.reparam(wk, ksize), oracle.reparam(wv, ksize), bias, heads, ksize)
    np.testing.assert_allclose(a, b, rtol=0, atol=1e-12)
    ks2 = oracle.deformed_shift(k, wk, ksize, two_branch=True)
    ksm = oracle.deformed_shift(k, oracle.reparam(wk, ksize), ksize, two_branch=False)
    np.testing.assert_allclose(ks2, ksm, rtol=0, atol=1e-12)


def test_reparam_is_onehot_plus_learned():
    C, ksize = 3, 3
    S = ksize * ksize
    w = np.random.default_rng(0).standard_normal((C, S, ksize, ksize))
    m = oracle.reparam(w, ksize)
    diff = (m - w).reshape(C, S, S)
    for c in range(C):
        np.testing.assert_allclose(diff[c], np.eye(S), rtol=0, atol=1e-15)   # (1+w)-w rounds
    # Eq. 11: the kernel that shifts towards (-1,-1) has its 1 at the top-left tap
    onehot = oracle.reparam(np.zeros((1, S, ksize, ksize)), ksize)
    assert onehot[0, 0, 0, 0] == 1.0 and onehot[0, 0].sum() == 1.0
    assert onehot[0, 4, 1, 1] == 1.0 and onehot[0, 8, 2, 2] == 1.0


# ---------------------------------------------------------------- P3: pure shift
@pytest.mark.parametrize("ksize", [3, 5])
def test_zero_learned_kernel_is_pure_shift(ksize):
    B, C, H, W = 1, 2, 4, 6
    r, S = ksize // 2, ksize * ksize
    x = np.random.default_rng(1).standard_normal((B, C, H, W))
    padded = np.pad(x, ((0, 0), (0, 0), (r, r), (r, r)))
    ks = oracle.deformed_shift(x, oracle.reparam(np.zeros((C, S, ksize, ksize)), ksize), ksize, False)
    for u in range(-r, r + 1):
        for v in range(-r, r + 1):
            s = (u + r) * ksize + (v + r)
            expect = padded[:, :, r + u:r + u + H, r + v:r + v + W]       # x[i+u, j+v]
            assert np.array_equal(ks[:, :, s], expect)
    # Eq. 10: the (-1,-1) shift moves the map down-right: out[i,j] = x[i-1,j-1]
    s11 = (r - 1) * ksize + (r - 1)
    assert np.array_equal(ks[0, 0, s11, 1:, 1:], x[0, 0, :-1, :-1])
    assert np.all(ks[0, 0, s11, 0, :] == 0) and np.all(ks[0, 0, s11, :, 0] == 0)


# ---------------------------------------------------------------- P4: huge bias selects one shift
def test_large_bias_selects_shift_direction():
    B, H, W, C, heads, ksize = 1, 5, 4, 4, 2, 3
    q, k, v, _, _, _, _ = rand_problem(B, H, W, C, heads, ksize, seed=9)
    S = ksize * ksize
    zero = np.zeros((C, S, ksize, ksize))
    vp = np.pad(v, ((0, 0), (0, 0), (1, 1), (1, 1)))
    for s0 in range(S):
        u0, v0 = s0 // ksize - 1, s0 % ksize - 1
        bias = np.zeros((heads, S))
        bias[:, s0] = 1e4
        out = oracle.fwd(q, k, v, zero, zero, bias, heads, ksize, two_branch=True)
        expect = vp[:, :, 1 + u0:1 + u0 + H, 1 + v0:1 + v0 + W]
        assert np.array_equal(out, expect)       # includes the zeros at the border


# ---------------------------------------------------------------- P5: box filter closed form
@pytest.mark.parametrize("ksize", [3, 5])
def test_uniform_attention_is_average_pool_with_padding_counted(ksize):
    B, H, W, C, heads = 1, 6, 7, 4, 2
    S, r = ksize * ksize, ksize // 2
    rng = np.random.default_rng(2)
    v = rng.standard_normal((B, C, H, W))
    k = rng.standard_normal((B, C, H, W))
    q = np.zeros((B, C, H, W))
    zero = np.zeros((C, S, ksize, ksize))
    out = oracle.fwd(q, k, v, zero, zero, None, heads, ksize, two_branch=True)
    ref = F.avg_pool2d(torch.from_numpy(v), ksize, stride=1, padding=r, count_include_pad=True).numpy()
    np.testing.assert_allclose(out, ref, rtol=0, atol=1e-13)
    # v == 1: padded positions stay in the softmax, so borders are attenuated
    ones = np.ones((B, C, H, W))
    o1 = oracle.fwd(q, k, ones, zero, zero, None, heads, ksize, two_branch=True)
    assert abs(o1[0, 0, 0, 0] - (r + 1) ** 2 / S) < 1e-14          # corner  (4/9 at k=3)
    assert abs(o1[0, 0, 0, W // 2] - (r + 1) / ksize) < 1e-14      # edge    (6/9 at k=3)
    assert abs(o1[0, 0, H // 2, W // 2] - 1.0) < 1e-14             # interior


# ---------------------------------------------------------------- P6: impulse response
def test_impulse_response_reads_kernel_unflipped():
    C, H, W, ksize = 2, 5, 6, 3
    S, r = 9, 1
    rng = np.random.default_rng(4)
    wm = rng.standard_normal((C, S, ksize, ksize))
    i0, j0 = 2, 3
    x = np.zeros((1, C, H, W))
    x[0, :, i0, j0] = 1.0
    ks = oracle.deformed_shift(x, wm, ksize, two_branch=False)
    for c in range(C):
        for s in range(S):
            for i in range(H):
                for j in range(W):
                    p, q = i0 - i + r, j0 - j + r
                    expect = wm[c, s, p, q] if (0 <= p < ksize and 0 <= q < ksize) else 0.0
                    assert ks[0, c, s, i, j] == expect


# ---------------------------------------------------------------- P7: ksize == 1
def test_ksize_one_degenerates_to_scaled_value():
    B, H, W, C, heads, ksize = 2, 3, 4, 4, 2, 1
    q, k, v, do, wk, wv, bias = rand_problem(B, H, W, C, heads, ksize, seed=6)
    wkm, wvm = oracle.reparam(wk, 1), oracle.reparam(wv, 1)
    out, attn = oracle.fwd(q, k, v, wkm, wvm, bias, heads, 1, return_attn=True)
    np.testing.assert_allclose(out, (1.0 + wv[:, 0, 0, 0])[None, :, None, None] * v, rtol=0, atol=1e-14)
    assert np.array_equal(attn, np.ones_like(attn))
    dq, dk, dv, dwk, dwv, dbias = oracle.bwd(do, q, k, v, wkm, wvm, bias, heads, 1)
    assert np.all(dq == 0) and np.all(dk == 0) and np.all(dwk == 0) and np.all(dbias == 0)
    np.testing.assert_allclose(dv, (1.0 + wv[:, 0, 0, 0])[None, :, None, None] * do, rtol=0, atol=1e-14)
    np.testing.assert_allclose(dwv[:, 0, 0, 0], (do * v).sum((0, 2, 3)), rtol=0, atol=1e-12)


# ---------------------------------------------------------------- P8: invariants
def test_softmax_and_structural_invariants():
    B, H, W, C, heads, ksize = 2, 5, 6, 4, 2, 3
    q, k, v, do, wk, wv, bias = rand_problem(B, H, W, C, heads, ksize, seed=8)
    wkm, wvm = oracle.reparam(wk, ksize), oracle.reparam(wv, ksize)
    out, attn = oracle.fwd(q, k, v, wkm, wvm, bias, heads, ksize, return_attn=True)
    np.testing.assert_allclose(attn.sum(2), 1.0, rtol=0, atol=1e-14)
    assert np.all(attn > 0)
    # a constant added to one head's bias row changes nothing
    b2 = bias.copy(); b2[1] += 3.7
    np.testing.assert_allclose(oracle.fwd(q, k, v, wkm, wvm, b2, heads, ksize), out, rtol=0, atol=1e-13)
    # bias = None means zero bias
    np.testing.assert_array_equal(oracle.fwd(q, k, v, wkm, wvm, None, heads, ksize),
                                  oracle.fwd(q, k, v, wkm, wvm, np.zeros_like(bias), heads, ksize))
    # batch items are independent
    out0 = oracle.fwd(q[1:], k[1:], v[1:], wkm, wvm, bias, heads, ksize)
    np.testing.assert_array_equal(out0[0], out[1])
    # heads are independent: head 1 alone, with its own slices of everything
    d = C // heads
    outh = oracle.fwd(q[:, d:], k[:, d:], v[:, d:], wkm[d:], wvm[d:], bias[1:], 1, ksize)
    np.testing.assert_allclose(outh, out[:, d:], rtol=0, atol=1e-14)
    # translation equivariance away from the border
    qs, ks_, vs = (np.roll(x, (1, 2), axis=(2, 3)) for x in (q, k, v))
    big = [np.pad(x, ((0, 0), (0, 0), (3, 3), (3, 3))) for x in (q, k, v)]
    bigs = [np.roll(x, (1, 2), axis=(2, 3)) for x in big]
    o_big = oracle.fwd(*big, wkm, wvm, bias, heads, ksize)
    o_bigs = oracle.fwd(*bigs, wkm, wvm, bias, heads, ksize)
    np.testing.assert_allclose(np.roll(o_big, (1, 2), axis=(2, 3))[:, :, 2:-2, 3:-2],
                               o_bigs[:, :, 2:-2, 3:-2], rtol=0, atol=1e-13)
    # gradient of the bias sums to zero over the shifts (softmax Jacobian)
    *_, dbias = oracle.bwd(do, q, k, v, wkm, wvm, bias, heads, ksize)
    np.testing.assert_allclose(dbias.sum(1), 0.0, rtol=0, atol=1e-12)


# ---------------------------------------------------------------- log of the softmax denominator
@pytest.mark.parametrize("shape", SHAPES)
def test_lse_matches_bruteforce_logits_and_library_logsumexp(shape):
    """lse = log sum_s exp(logit[s]) (denominator of Eq. 2): against the column-view brute
    force's raw logits (summed naively here: they are O(1)) and torch.logsumexp of the
    grouped-conv statement."""
    B, H, W, C, heads, ksize = shape
    q, k, v, _, wk, wv, bias = rand_problem(*shape, seed=21)
    _, _, logits = brute_local_attention(q, k, v, wk, wv, bias, heads, ksize, return_logits=True)
    wkm, wvm = oracle.reparam(wk, ksize), oracle.reparam(wv, ksize)
    out, attn, lse = oracle.fwd(q, k, v, wkm, wvm, bias, heads, ksize, return_attn=True, return_lse=True)
    assert lse.shape == (B, heads, H, W)
    np.testing.assert_allclose(lse, np.log(np.exp(logits).sum(2)), rtol=0, atol=1e-12)
    # attention weights, logits and lse belong together: a[s] = exp(l[s] - lse)
    np.testing.assert_allclose(attn, np.exp(logits - lse[:, :, None]), rtol=0, atol=1e-12)
    t = [torch.from_numpy(x) for x in (q, k, v, wkm, wvm, bias)]
    d, S = C // heads, ksize * ksize
    Ks = F.conv2d(t[1], t[3].reshape(C * S, 1, ksize, ksize), padding=ksize // 2, groups=C)
    tl = (t[0].reshape(B, heads, d, 1, H, W) * Ks.reshape(B, heads, d, S, H, W)).sum(2) / math.sqrt(d)
    tl = tl + t[5][None, :, :, None, None]
    np.testing.assert_allclose(lse, torch.logsumexp(tl, dim=2).numpy(), rtol=0, atol=1e-12)
    # the two-branch form gives the same lse, and asking for lse does not change out
    out2, lse2 = oracle.fwd(q, k, v, wk, wv, bias, heads, ksize, two_branch=True, return_lse=True)
    np.testing.assert_allclose(lse2, lse, rtol=0, atol=1e-12)
    np.testing.assert_array_equal(out, oracle.fwd(q, k, v, wkm, wvm, bias, heads, ksize))


def test_lse_closed_forms():
    B, H, W, C, heads, ksize = 1, 4, 3, 4, 2, 3
    q, k, v, _, wk, wv, bias = rand_problem(B, H, W, C, heads, ksize, seed=22)
    wkm, wvm = oracle.reparam(wk, ksize), oracle.reparam(wv, ksize)
    # q = 0, no bias: nine equal logits of zero -> lse = log 9 everywhere, borders included
    # (padded neighbours stay in the softmax)
    _, lse = oracle.fwd(np.zeros_like(q), k, v, wkm, wvm, None, heads, ksize, return_lse=True)
    np.testing.assert_allclose(lse, math.log(9.0), rtol=0, atol=1e-14)
    # q = 0 with bias: lse depends on the head's bias row only
    _, lse = oracle.fwd(np.zeros_like(q), k, v, wkm, wvm, bias, heads, ksize, return_lse=True)
    for m in range(heads):
        np.testing.assert_allclose(lse[:, m], math.log(sum(math.exp(x) for x in bias[m])), rtol=0, atol=1e-13)
    # a constant added to a head's bias row moves that head's lse by the constant
    _, lse_a = oracle.fwd(q, k, v, wkm, wvm, bias, heads, ksize, return_lse=True)
    b2 = bias.copy(); b2[1] += 3.7
    _, lse_b = oracle.fwd(q, k, v, wkm, wvm, b2, heads, ksize, return_lse=True)
    np.testing.assert_allclose(lse_b[:, 0], lse_a[:, 0], rtol=0, atol=1e-13)
    np.testing.assert_allclose(lse_b[:, 1], lse_a[:, 1] + 3.7, rtol=0, atol=1e-12)
    # ksize 1: a single logit, lse is that logit: scale * sum_c q[c] (1 + wk[c]) k[c] + bias
    q1, k1, v1, _, wk1, wv1, bias1 = rand_problem(2, 3, 4, 4, 2, 1, seed=23)
    _, lse1 = oracle.fwd(q1, k1, v1, oracle.reparam(wk1, 1), oracle.reparam(wv1, 1), bias1, 2, 1, return_lse=True)
    prod = q1 * k1 * (1.0 + wk1[:, 0, 0, 0])[None, :, None, None]
    expect = prod.reshape(2, 2, 2, 3, 4).sum(2) / math.sqrt(2.0) + bias1[:, 0][None, :, None, None]
    np.testing.assert_allclose(lse1, expect, rtol=0, atol=1e-13)


def test_sampled_forward_equals_full_forward():
    B, H, W, C, heads, ksize = 2, 4, 5, 4, 2, 3
    q, k, v, _, wk, wv, bias = rand_problem(B, H, W, C, heads, ksize, seed=10)
    wkm, wvm = oracle.reparam(wk, ksize), oracle.reparam(wv, ksize)
    out = oracle.fwd(q, k, v, wkm, wvm, bias, heads, ksize)
    pos = np.array([[0, 0, 0, 0], [1, 1, 3, 4], [0, 1, 2, 2], [1, 0, 0, 4]], dtype=np.int32)
    smp = oracle.fwd_samples(q, k, v, wkm, wvm, bias, heads, ksize, pos)
    d = C // heads
    for n, (b, m, i, j) in enumerate(pos):
        np.testing.assert_array_equal(smp[n], out[b, m * d:(m + 1) * d, i, j])


# ---------------------------------------------------------------- P9: library cross-check
@pytest.mark.parametrize("shape", [(2, 4, 5, 4, 2, 3), (1, 3, 2, 4, 1, 5), (1, 6, 6, 6, 3, 3), (1, 3, 3, 2, 2, 1)])
def test_forward_and_backward_match_torch_autograd(shape):
    B, H, W, C, heads, ksize = shape
    q, k, v, do, wk, wv, bias = rand_problem(*shape, seed=12)
    wkm, wvm = oracle.reparam(wk, ksize), oracle.reparam(wv, ksize)
    tq, tk, tv, twk, twv, tb = (torch.tensor(x, dtype=torch.float64, requires_grad=True)
                                for x in (q, k, v, wkm, wvm, bias))
    tout, tattn = torch_forward(tq, tk, tv, twk, twv, tb, heads, ksize)
    tout.backward(torch.from_numpy(do))
    out, attn = oracle.fwd(q, k, v, wkm, wvm, bias, heads, ksize, return_attn=True)
    np.testing.assert_allclose(out, tout.detach().numpy(), rtol=0, atol=1e-12)
    np.testing.assert_allclose(attn, tattn.detach().numpy(), rtol=0, atol=1e-12)
    grads = oracle.bwd(do, q, k, v, wkm, wvm, bias, heads, ksize)
    for g, t, name in zip(grads, (tq, tk, tv, twk, twv, tb), "dq dk dv dwk dwv dbias".split()):
        np.testing.assert_allclose(g, t.grad.numpy(), rtol=0, atol=1e-11, err_msg=name)


# ---------------------------------------------------------------- P10: finite differences
def test_backward_matches_central_differences():
    B, H, W, C, heads, ksize = 1, 3, 4, 4, 2, 3
    q, k, v, do, wk, wv, bias = rand_problem(B, H, W, C, heads, ksize, seed=13)
    wkm, wvm = oracle.reparam(wk, ksize), oracle.reparam(wv, ksize)
    args = [q, k, v, wkm, wvm, bias]

    def loss(a):
        return float((oracle.fwd(a[0], a[1], a[2], a[3], a[4], a[5], heads, ksize) * do).sum())

    grads = oracle.bwd(do, q, k, v, wkm, wvm, bias, heads, ksize)
    rng = np.random.default_rng(0)
    eps = 1e-6
    for idx, g in enumerate(grads):
        flat = args[idx].reshape(-1)
        picks = rng.choice(flat.size, size=min(12, flat.size), replace=False)
        for e in picks:
            plus = [a.copy() for a in args]; minus = [a.copy() for a in args]
            plus[idx].reshape(-1)[e] += eps
            minus[idx].reshape(-1)[e] -= eps
            fd = (loss(plus) - loss(minus)) / (2 * eps)
            assert abs(fd - g.reshape(-1)[e]) < 1e-7 * max(1.0, abs(fd)), (idx, e, fd, g.reshape(-1)[e])
