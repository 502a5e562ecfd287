"""The forward entry point that allocates nothing (its kernels' scratch is a fixed array
inside the library) against slide_attn_fwd on the same inputs: two calls in a row, the second
on a smaller problem, both on kernel paths that use the scratch."""
import ctypes

import pytest
import torch

import paper_2304_04237_amd as sa
from paper_2304_04237_amd import synth


def _problem(B, H, W, C, heads, ksize, seed):
    d = synth.make_inputs(B, H, W, C, heads, ksize, "bf16", seed=seed, with_dout=False)
    dev = torch.device("cuda:0")
    g = {n: d[n].to(dev).to(torch.bfloat16) for n in ("q", "k", "v")}
    g["wk"] = sa.slide_reparam(d["wk_learned"].to(dev))
    g["wv"] = sa.slide_reparam(d["wv_learned"].to(dev))
    g["bias"] = d["bias"].to(dev)
    return g


@pytest.mark.gpu
def test_no_alloc_forward_matches_the_workspace_entry_point():
    # 5x5 window (operand images of 100 KB per head in the scratch), then a smaller 3x3 problem
    # on the one-tile-per-block kernel (18.5 KB per head), then the 5x5 one again
    shapes = [(2, 17, 13, 128, 4, 5), (1, 9, 21, 64, 2, 3), (2, 17, 13, 128, 4, 5)]
    for idx, shape in enumerate(shapes):
        B, H, W, C, heads, ksize = shape
        print("no-alloc case", shape, flush=True)
        assert sa.slide_attn_workspace_bytes(B, H, W, C, heads, ksize, torch.bfloat16, 0) > 0
        g = _problem(*shape, seed=40 + idx)
        lse_ref = torch.empty((B, heads, H, W), dtype=torch.float32, device=g["q"].device)
        ref = sa.slide_attn_fwd(g["q"], g["k"], g["v"], g["wk"], g["wv"], g["bias"], heads, ksize, lse=lse_ref)
        out = torch.full_like(g["q"], float("nan"))
        lse = torch.full_like(lse_ref, float("nan"))
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        sa.slide_attn_fwd_noalloc(g["q"], g["k"], g["v"], g["wk"], g["wv"], g["bias"], heads, ksize, out, lse=lse)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        # same kernels, same inputs: bit-identical (well inside the bf16 tolerance of 2e-2)
        assert torch.equal(out, ref)
        assert torch.equal(lse, lse_ref)


def test_no_alloc_forward_rejects_what_does_not_fit():
    """Host-side: argument and size errors are returned before the device is touched."""
    lib = sa.load_library()
    p = ctypes.c_void_p(0x1000)
    # 5x5, head size 32, 32 heads: 3.2 MB of operand images > the 2 MiB array
    assert sa.slide_attn_workspace_bytes(1, 8, 8, 1024, 32, 5, torch.bfloat16, 0) > (2 << 20)
    st = lib.slide_attn_fwd_noalloc(p, p, p, p, p, p, p, None, 1, 8, 8, 1024, 32, 5, 1, None)
    assert st == 4 and "scratch" in sa.slide_status_string(st)
    assert lib.slide_attn_fwd_noalloc(p, p, p, p, p, p, p, None, 1, 8, 8, 64, 3, 3, 1, None) == 2
    assert lib.slide_attn_fwd_noalloc(None, p, p, p, p, p, p, None, 1, 8, 8, 64, 2, 3, 1, None) == 1
