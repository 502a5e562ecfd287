"""Host-side checks of the C ABI: the library loads without a GPU, exports every
symbol the public header declares, and rejects bad arguments before any HIP call."""
import ctypes
import os
import re

import pytest

import paper_2304_04237_amd as sa

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "slide_attn.h")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(sa.lib_path()):
        from paper_2304_04237_amd import build
        build.build()
    return sa.load_library()


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(slide_[a-z_]+)\s*\(", text)))


def test_header_declares_the_expected_calls():
    names = declared_functions()
    for required in ("slide_reparam", "slide_attn_fwd", "slide_attn_bwd",
                     "slide_attn_fwd_two_branch", "slide_attn_bwd_two_branch",
                     "slide_attn_workspace_bytes", "slide_status_string"):
        assert required in names


def test_library_exports_every_declared_symbol(lib):
    for name in declared_functions():
        assert hasattr(lib, name), name


def test_status_strings(lib):
    assert sa.slide_status_string(0) == "SLIDE_OK"
    for code in range(1, 7):
        assert sa.slide_status_string(code).startswith("SLIDE_ERR_")
    assert "UNKNOWN" in sa.slide_status_string(99)


FWD_OK = dict(B=1, H=14, W=14, C=64, heads=2, ksize=3, dtype=0)


def call_fwd(lib, ptr=0x1000, lse=None, **kw):
    a = dict(FWD_OK); a.update(kw)
    p = ctypes.c_void_p(ptr)
    return lib.slide_attn_fwd(p, p, p, p, p, p, p, lse, a["B"], a["H"], a["W"], a["C"], a["heads"],
                              a["ksize"], a["dtype"], None, 0, None)


def test_forward_rejects_bad_arguments_on_the_host(lib):
    # none of these may reach a kernel launch: the pointers are not real device memory
    assert call_fwd(lib, heads=3) == 2             # C % heads != 0
    assert call_fwd(lib, ksize=4) == 2             # even window
    assert call_fwd(lib, ksize=0) == 2
    assert call_fwd(lib, ksize=9) == 2             # unsupported instantiation
    assert call_fwd(lib, B=0) == 2
    assert call_fwd(lib, H=-1) == 2
    assert call_fwd(lib, dtype=7) == 3
    assert call_fwd(lib, ptr=0) == 1               # NULL pointers
    assert call_fwd(lib, ptr=0x1002) == 6          # misaligned for float32
    assert call_fwd(lib, ptr=0x1001, dtype=1) == 6 # misaligned for bfloat16
    assert call_fwd(lib, heads=3, lse=ctypes.c_void_p(0x1000)) == 2   # lse given: same checks
    assert call_fwd(lib, lse=ctypes.c_void_p(0x1002)) == 6            # lse not 4-byte aligned


def test_variant_query_knows_head_size_24():
    # head size 24 runs on the streaming kernel where the map fits it, else on padded copies
    # through the other matrix-core kernels, else on the general kernel
    assert sa.slide_attn_fwd_variant(2, 56, 56, 48, 2, 3, 1, True) == 24
    assert sa.slide_attn_fwd_variant(2, 56, 56, 48, 2, 3, 1, False) == 10
    assert sa.slide_attn_fwd_variant(2, 56, 72, 48, 2, 3, 1, True) == 126     # wider than the ring takes: padded to 32 channels per head, streaming kernel on column strips
    assert sa.slide_attn_fwd_variant(2, 9, 21, 48, 2, 3, 1, True) == 10       # H * W % 8 != 0: general kernel
    assert sa.slide_attn_fwd_variant(2, 56, 56, 48, 2, 5, 1, True) == 10      # 5x5 window
    assert sa.slide_attn_fwd_variant(2, 56, 56, 48, 2, 3, 0, True) == 10      # float32


def test_shift_forward_rejects_bad_arguments_on_the_host(lib):
    lib.slide_attn_fwd_shift.restype = ctypes.c_int
    lib.slide_attn_fwd_shift.argtypes = [ctypes.c_void_p] * 6 + [ctypes.c_int] * 7 + [ctypes.c_void_p]

    def call(ptr=0x1000, **kw):
        a = dict(FWD_OK); a.update(kw)
        p = ctypes.c_void_p(ptr)
        return lib.slide_attn_fwd_shift(p, p, p, p, p, None, a["B"], a["H"], a["W"], a["C"], a["heads"],
                                        a["ksize"], a["dtype"], None)
    assert call(heads=3) == 2
    assert call(ksize=2) == 2
    assert call(W=0) == 2
    assert call(dtype=2) == 3
    assert call(ptr=0) == 1
    assert call(ptr=0x1002) == 6
    assert call(ptr=0x1001, dtype=1) == 6


def test_backward_rejects_bad_arguments_on_the_host(lib):
    p = ctypes.c_void_p(0x1000)
    # dout q k v wk wv bias | out lse (optional) | dq dk dv dwk dwv dbias
    args13 = [p] * 7 + [None, None] + [p] * 6
    shape = [1, 14, 14, 64, 2, 3, 0]
    need = lib.slide_attn_workspace_bytes(*shape, 1)
    assert need > 0
    assert lib.slide_attn_bwd(*args13, *shape, None, 0, None) == 4            # no workspace
    assert lib.slide_attn_bwd(*args13, *shape, p, need - 1, None) == 4        # too small
    bad = list(args13); bad[11] = None
    assert lib.slide_attn_bwd(*bad, *shape, p, need, None) == 1               # dv NULL
    bad = list(args13); bad[14] = None
    assert lib.slide_attn_bwd(*bad, *shape, p, need, None) == 1               # bias without dbias
    given = list(args13); given[7] = p; given[8] = ctypes.c_void_p(0x1002)
    assert lib.slide_attn_bwd(*given, *shape, p, need, None) == 6             # lse given but misaligned
    given[7] = ctypes.c_void_p(0x1002); given[8] = p
    assert lib.slide_attn_bwd(*given, *shape, p, need, None) == 6             # out given but misaligned
    shape_bad = [1, 14, 14, 64, 5, 3, 0]
    assert lib.slide_attn_bwd(*args13, *shape_bad, p, need, None) == 2
    # the workspace must be 16-byte aligned, as the header says (no silent slow path)
    assert lib.slide_attn_bwd(*args13, *shape, ctypes.c_void_p(0x1004), need + 16, None) == 6
    assert lib.slide_attn_bwd(*args13, *shape, ctypes.c_void_p(0x1008), need + 16, None) == 6


def test_two_branch_entry_points_check_arguments_like_the_merged_ones(lib):
    p = ctypes.c_void_p(0x1000)
    fwd = lib.slide_attn_fwd_two_branch
    # none of these may reach a kernel launch: the pointers are not real device memory
    assert fwd(p, p, p, p, p, p, p, None, 1, 14, 14, 64, 3, 3, 0, None, 0, None) == 2   # C % heads != 0
    assert fwd(p, p, p, None, p, p, p, None, 1, 14, 14, 64, 2, 3, 0, None, 0, None) == 1  # wk_learned NULL
    assert fwd(p, p, p, p, p, p, p, None, 64, 56, 56, 64, 2, 3, 1, None, 0, None) == 4    # needs its workspace
    bwd = lib.slide_attn_bwd_two_branch
    args = [p] * 7 + [None, None] + [p] * 6
    shape = [1, 14, 14, 64, 2, 3, 0]
    need = lib.slide_attn_workspace_bytes(*shape, 1)
    assert bwd(*args, 1, *shape, None, 0, None) == 4                      # no workspace
    assert bwd(*args, 0, *[1, 14, 14, 64, 5, 3, 0], p, need, None) == 2   # bad shape
    bad = list(args); bad[12] = None
    assert bwd(*bad, 1, *shape, p, need, None) == 1                       # dwk NULL


def test_workspace_query(lib):
    assert lib.slide_attn_workspace_bytes(1, 14, 14, 64, 2, 3, 0, 0) == 0     # forward needs none
    assert lib.slide_attn_workspace_bytes(1, 14, 14, 64, 3, 3, 0, 1) == 0     # invalid -> 0
    small = lib.slide_attn_workspace_bytes(1, 14, 14, 64, 2, 3, 0, 1)
    big = lib.slide_attn_workspace_bytes(4, 14, 14, 64, 2, 3, 0, 1)
    assert 0 < small < big


def test_reparam_rejects_bad_arguments(lib):
    p = ctypes.c_void_p(0x1000)
    assert lib.slide_reparam(None, p, 4, 3, None) == 1
    assert lib.slide_reparam(p, p, 0, 3, None) == 2
    assert lib.slide_reparam(p, p, 4, 2, None) == 2


def test_forward_path_selection(lib):
    assert lib.slide_attn_fwd_path(1, 14, 14, 64, 2, 3, 0) == 1     # float32 -> general kernel
    assert lib.slide_attn_fwd_path(1, 14, 14, 64, 3, 3, 0) == 0
    assert lib.slide_attn_fwd_path(64, 56, 56, 64, 2, 3, 1) == 2    # bf16, head size 32, 3x3 -> matrix cores
    assert lib.slide_attn_fwd_path(64, 28, 28, 128, 4, 5, 1) == 3   # 5x5 -> matrix cores, 5x5 kernel
    assert lib.slide_attn_workspace_bytes(64, 56, 56, 64, 2, 3, 1, 0) > 0
    p = ctypes.c_void_p(0x1000)
    # the matrix-core forward needs its workspace
    assert lib.slide_attn_fwd(p, p, p, p, p, p, p, None, 64, 56, 56, 64, 2, 3, 1, None, 0, None) == 4


def test_forward_variant_selection(lib):
    """Which kernel inside the matrix-core forward serves a problem (256 compute units
    assumed when there is no device)."""
    v = lib.slide_attn_fwd_variant
    assert v(1, 14, 14, 64, 3, 3, 0, 1) == 0                       # invalid
    assert v(1, 14, 14, 64, 2, 3, 0, 1) == 10                      # float32: general kernel
    assert v(64, 28, 28, 128, 4, 5, 1, 1) == 30                    # 5x5
    assert v(64, 56, 56, 64, 2, 3, 1, 1) == 24                     # stage 1: streaming kernel
    assert v(64, 56, 56, 64, 2, 3, 1, 0) == 20                     # unaligned pointers: one tile per block
    assert v(2, 200, 304, 96, 3, 3, 1, 1) == 26                    # 200x304: streaming kernel on column strips
    assert v(12, 64, 72, 64, 2, 3, 1, 1) == 23                     # 72 columns in bands of 64 rows: strips of 40 need too deep a ring, strips of 48 overlap by a third: pipelined tiles, width 64
    assert v(12, 20, 72, 64, 2, 3, 1, 1) == 26                     # 72 columns, short bands: two strips of 40
    assert v(96, 48, 48, 64, 2, 3, 1, 1) == 24                     # streaming kernel, 48 columns
    assert v(96, 40, 40, 64, 2, 3, 1, 1) == 21                     # 40 columns need too much LDS there: pipelined tiles
    assert v(300, 24, 24, 64, 2, 3, 1, 1) == 21                    # narrower than 32: pipelined tiles, width from the arguments
    assert v(2, 9, 21, 64, 2, 3, 1, 1) == 20                       # W % 8 != 0
    assert v(8, 100, 128, 32, 1, 3, 1, 1) == 26                    # 128 columns: three strips
    assert v(8, 100, 128, 32, 1, 3, 1, 0) == 20                    # ... not from unaligned pointers: one tile per block
    # many small planes: enough tiles, but a tile buffer too small to build the operand image in
    assert v(128, 8, 8, 128, 4, 3, 1, 1) == 20
    assert v(256, 2, 64, 64, 2, 3, 1, 1) == 24                     # two-row planes: streaming kernel
    assert v(64, 56, 56, 64, 1, 3, 1, 1) == 25                     # one head of 64 channels: two launches over half heads
    assert v(64, 56, 56, 64, 1, 3, 1, 0) == 10                     # ... not from unaligned pointers
    assert v(8, 100, 128, 64, 1, 3, 1, 1) == 10                    # ... nor on a map the streaming kernel does not take
    assert lib.slide_attn_workspace_bytes(64, 56, 56, 64, 1, 3, 1, 0) == 64 * 2 * 9 * 56 * 56 * 4   # the halves' partial logits
    assert lib.slide_attn_fwd_path(64, 56, 56, 64, 1, 3, 1) == 2


def test_backward_variant_selection(lib):
    """Which kernels serve the backward of a problem (256 compute units assumed when there is
    no device)."""
    v = lib.slide_attn_bwd_variant
    assert v(1, 14, 14, 64, 3, 3, 0, 1) == 0                       # invalid
    assert v(1, 14, 14, 64, 2, 3, 0, 1) == 10                      # float32: general kernels
    assert v(64, 28, 28, 128, 4, 5, 1, 1) == 10                    # 5x5
    assert v(128, 56, 56, 64, 2, 3, 1, 1) == 27                    # stage-1 training: all three streaming kernels
    assert v(128, 56, 56, 64, 2, 3, 1, 0) == 10                    # unaligned pointers: general kernels
    assert v(2, 33, 32, 64, 2, 3, 1, 1) == 26                      # too narrow for the dk/dv kernel's record rings
    assert v(3, 40, 64, 32, 1, 3, 1, 1) == 22                      # 64 columns: a dl / a row is more than one load
    assert v(2, 13, 72, 32, 1, 3, 1, 1) == 20                      # wider than 64: tiled kernels
    assert v(50, 20, 40, 96, 3, 3, 1, 1) == 24                     # bands of 20 rows of 40 columns need too deep a ring: only the kernel gradients stream
    assert v(2, 9, 21, 64, 2, 3, 1, 1) == 20                       # W % 8 != 0: tiled kernels, general kernel-gradient part
    assert v(128, 56, 56, 48, 2, 3, 1, 1) == 127                   # 24 channels per head: the streaming kernels on padded copies
    assert v(128, 56, 56, 48, 2, 3, 1, 0) == 10                    # ... not from unaligned pointers
    assert v(4, 13, 72, 16, 2, 3, 1, 1) == 120                     # 8 channels per head, wide map: the tiled kernels on padded copies
    assert v(4, 13, 72, 128, 2, 3, 1, 1) == 10                     # 64 channels per head on a wide map: general kernels
    assert v(128, 56, 56, 64, 1, 3, 1, 1) == 227                   # 64 channels per head: half heads through the streaming kernels
    assert v(128, 56, 56, 64, 1, 3, 1, 0) == 10


def test_binding_rejects_mismatched_parameter_shapes(lib):
    """Shape mistakes are reported by the binding; they must not reach a kernel."""
    import torch
    q = torch.zeros(1, 64, 6, 6)
    w3 = torch.zeros(64, 9, 3, 3)
    w5 = torch.zeros(64, 25, 5, 5)
    bias = torch.zeros(2, 9)
    with pytest.raises(sa.SlideAttnError, match="wk must be"):
        sa.slide_attn_fwd(q, q, q, w3, w3, bias, 2, 5)             # ksize 5 with 3x3 kernels
    with pytest.raises(sa.SlideAttnError, match="wv must be"):
        sa.slide_attn_fwd(q, q, q, w5, w3, None, 2, 5)
    with pytest.raises(sa.SlideAttnError, match="bias must be"):
        sa.slide_attn_fwd(q, q, q, w3, w3, torch.zeros(4, 9), 2, 3)
    with pytest.raises(sa.SlideAttnError, match="out must match"):
        sa.slide_attn_fwd(q, q, q, w3, w3, bias, 2, 3, out=torch.zeros(1, 64, 6, 5))
    with pytest.raises(sa.SlideAttnError, match="dq must match"):
        sa.slide_attn_bwd(q, q, q, q, w3, w3, bias, 2, 3,
                          outputs=(torch.zeros(1, 64, 6, 5), q, q, w3, w3, bias))
    with pytest.raises(sa.SlideAttnError, match="dwk must have"):
        sa.slide_attn_bwd(q, q, q, q, w3, w3, bias, 2, 3, outputs=(q, q, q, w5, w3, bias))
    with pytest.raises(sa.SlideAttnError, match="dbias must have"):
        sa.slide_attn_bwd(q, q, q, q, w3, w3, bias, 2, 3, outputs=(q, q, q, w3, w3, None))
    with pytest.raises(sa.SlideAttnError, match="w_merged"):
        sa.slide_reparam(w3, w5)
