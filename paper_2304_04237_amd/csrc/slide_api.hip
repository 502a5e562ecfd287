// C ABI of libslide_attn.so: argument validation on the host, then dispatch to
// the gfx950 kernels.  Declarations and contracts: include/slide_attn.h.
#include "slide_attn.h"
#include "slide_internal.h"

using slide::Problem;

int slide::device_cu_count()
{
    constexpr int MAX_DEV = 64;
    static std::mutex mu;
    static int cached[MAX_DEV];                 // 0 = not read yet
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEV) {
        (void)hipGetLastError();
        return MAX_CU_PLANNED;
    }
    std::lock_guard<std::mutex> lock(mu);
    if (cached[dev] == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1) {
            (void)hipGetLastError();
            n = MAX_CU_PLANNED;
        }
        cached[dev] = n > MAX_CU_PLANNED ? MAX_CU_PLANNED : n;
    }
    return cached[dev];
}

static bool ksize_supported(int ksize) { return ksize == 1 || ksize == 3 || ksize == 5 || ksize == 7; }

// Validate the shape arguments common to forward and backward.
static int check_problem(int B, int H, int W, int C, int heads, int ksize, int dtype)
{
    if (dtype != SLIDE_F32 && dtype != SLIDE_BF16) return SLIDE_ERR_DTYPE;
    if (B < 1 || H < 1 || W < 1 || C < 1 || heads < 1) return SLIDE_ERR_SHAPE;
    if (C % heads != 0) return SLIDE_ERR_SHAPE;
    if (!ksize_supported(ksize)) return SLIDE_ERR_SHAPE;
    if (B > 65535 || heads > 65535) return SLIDE_ERR_SHAPE;          // grid y/z limits
    if ((long)H * W > 0x7fffffffL / 64) return SLIDE_ERR_SHAPE;       // plane index arithmetic
    return SLIDE_OK;
}

static bool aligned_to(const void* p, size_t a) { return ((uintptr_t)p % a) == 0; }

extern "C" const char* slide_status_string(int status)
{
    switch (status) {
        case SLIDE_OK: return "SLIDE_OK";
        case SLIDE_ERR_NULL: return "SLIDE_ERR_NULL: a required pointer is NULL";
        case SLIDE_ERR_SHAPE: return "SLIDE_ERR_SHAPE: bad dimension, C % heads != 0, or unsupported ksize";
        case SLIDE_ERR_DTYPE: return "SLIDE_ERR_DTYPE: dtype must be SLIDE_F32 or SLIDE_BF16";
        case SLIDE_ERR_WORKSPACE: return "SLIDE_ERR_WORKSPACE: workspace missing or too small (or the problem needs more scratch than slide_attn_fwd_noalloc has)";
        case SLIDE_ERR_HIP: return "SLIDE_ERR_HIP: kernel launch failed";
        case SLIDE_ERR_ALIGN: return "SLIDE_ERR_ALIGN: a pointer is not aligned to its element size (workspace: 16 bytes)";
        default: return "SLIDE_ERR_UNKNOWN";
    }
}

extern "C" int slide_reparam(const float* w_learned, float* w_merged, int C, int ksize, void* stream)
{
    if (!w_learned || !w_merged) return SLIDE_ERR_NULL;
    if (C < 1 || !ksize_supported(ksize)) return SLIDE_ERR_SHAPE;
    hipError_t e = slide::launch_reparam(w_learned, w_merged, C, ksize, (hipStream_t)stream);
    return e == hipSuccess ? SLIDE_OK : SLIDE_ERR_HIP;
}

extern "C" size_t slide_attn_workspace_bytes(int B, int H, int W, int C, int heads, int ksize,
                                             int dtype, int backward)
{
    if (check_problem(B, H, W, C, heads, ksize, dtype) != SLIDE_OK) return 0;
    Problem p{B, H, W, C, heads, ksize, dtype};
    if (backward) return slide::bwd_generic_workspace_bytes(p);
    // heads of 64 channels: what the two-launch streaming forward exchanges (a caller that brings
    // less gets the general kernel, which needs none)
    if (slide::fwd_ring_enabled() && slide::fwd_ring_wide_supported(p, true)) return slide::fwd_ring_wide_workspace_bytes(p);
    // heads narrower than 32 channels: the padded copies (head size 24 on the streaming kernel's maps needs none)
    Problem p32;
    if (!(C == heads * 24 && slide::fwd_ring_enabled() && slide::fwd_ring_supported(p, true)) && slide::fwd_padded_problem(p, p32))
        return slide::fwd_padded_workspace_bytes(p32);
    return slide::fwd_mfma_supported(p) ? slide::fwd_mfma_workspace_bytes(p) : slide::fwd_mfma5_workspace_bytes(p);
}

extern "C" int slide_attn_fwd_path(int B, int H, int W, int C, int heads, int ksize, int dtype)
{
    if (check_problem(B, H, W, C, heads, ksize, dtype) != SLIDE_OK) return 0;
    Problem p{B, H, W, C, heads, ksize, dtype};
    if (slide::fwd_ring_enabled() && slide::fwd_ring_wide_supported(p, true)) return 2;
    Problem p32;
    if (slide::fwd_padded_problem(p, p32) || (C == heads * 24 && slide::fwd_ring_enabled() && slide::fwd_ring_supported(p, true))) return 2;
    return slide::fwd_mfma_supported(p) ? 2 : (slide::fwd_mfma5_supported(p) ? 3 : 1);
}

extern "C" int slide_attn_fwd_variant(int B, int H, int W, int C, int heads, int ksize, int dtype,
                                      int aligned16)
{
    if (check_problem(B, H, W, C, heads, ksize, dtype) != SLIDE_OK) return 0;
    Problem p{B, H, W, C, heads, ksize, dtype};
    if (slide::fwd_mfma_supported(p)) return slide::fwd_mfma_variant(p, aligned16 != 0);
    if (C == heads * 24 && slide::fwd_ring_enabled() && slide::fwd_ring_supported(p, aligned16 != 0)) return 24;
    if (slide::fwd_ring_enabled() && slide::fwd_ring_wide_supported(p, aligned16 != 0)) return 25;
    Problem p32;
    if (aligned16 && slide::fwd_padded_problem(p, p32)) return 100 + slide::fwd_mfma_variant(p32, true);
    return slide::fwd_mfma5_supported(p) ? 30 : 10;
}

extern "C" int slide_attn_bwd_variant(int B, int H, int W, int C, int heads, int ksize, int dtype,
                                      int aligned16)
{
    if (check_problem(B, H, W, C, heads, ksize, dtype) != SLIDE_OK) return 0;
    Problem p{B, H, W, C, heads, ksize, dtype};
    return slide::bwd_variant(p, aligned16 != 0);
}

// ---- scratch of the entry point that allocates nothing ---------------------------------
// One array per GPU (every device that loads the library holds its own copy until the process
// ends).  In host code the array's name is only a handle for hipGetSymbolAddress: kernels and
// copies get the device address looked up below, never the name.
constexpr size_t NOALLOC_SCRATCH_BYTES = SLIDE_NOALLOC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[NOALLOC_SCRATCH_BYTES];

// Device address of `scratch` on the current device, looked up once per device.
static hipError_t noalloc_scratch(void** ptr)
{
    constexpr int MAX_DEV = 64;
    static std::mutex mu;
    static void* addr[MAX_DEV];                 // null = not looked up yet
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= MAX_DEV) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(mu);
    if (!addr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        addr[dev] = p;
    }
    *ptr = addr[dev];
    return hipSuccess;
}

static int forward(const void* q, const void* k, const void* v,
                   const float* wk, const float* wv, const float* bias, void* out, float* lse,
                   int B, int H, int W, int C, int heads, int ksize, int dtype, int two_branch,
                   void* workspace, size_t workspace_bytes, void* stream)
{
    int st = check_problem(B, H, W, C, heads, ksize, dtype);
    if (st != SLIDE_OK) return st;
    if (!q || !k || !v || !wk || !wv || !out) return SLIDE_ERR_NULL;
    const size_t esz = dtype == SLIDE_F32 ? 4 : 2;
    if (!aligned_to(q, esz) || !aligned_to(k, esz) || !aligned_to(v, esz) || !aligned_to(out, esz) ||
        !aligned_to(wk, 4) || !aligned_to(wv, 4) || !aligned_to(bias, 4) || !aligned_to(lse, 4))
        return SLIDE_ERR_ALIGN;
    Problem p{B, H, W, C, heads, ksize, dtype};
    p.two_branch = two_branch;
    hipError_t e;
    const bool aligned16 = aligned_to(q, 16) && aligned_to(k, 16) && aligned_to(v, 16) && aligned_to(out, 16) &&
                           aligned_to(wk, 16) && aligned_to(wv, 16);
    if (C == heads * 24 && slide::fwd_ring_enabled() && slide::fwd_ring_supported(p, aligned16)) {
        // head size 24 on the streaming matrix-core kernel (no workspace); every other problem of
        // that head size runs on the general kernel below
        e = slide::launch_fwd_ring(p, q, k, v, wk, wv, bias, out, lse, false, (hipStream_t)stream);
    } else if (slide::fwd_ring_enabled() && slide::fwd_ring_wide_supported(p, aligned16) && workspace &&
               workspace_bytes >= slide::fwd_ring_wide_workspace_bytes(p) && aligned_to(workspace, 16)) {
        // heads of 64 channels: two launches of the streaming kernel (without that much workspace:
        // the general kernel below)
        e = slide::launch_fwd_ring_wide(p, q, k, v, wk, wv, bias, out, lse, workspace, (hipStream_t)stream);
    } else if (slide::fwd_mfma_supported(p)) {
        if (!workspace || workspace_bytes < slide::fwd_mfma_workspace_bytes(p)) return SLIDE_ERR_WORKSPACE;
        if (!aligned_to(workspace, 16)) return SLIDE_ERR_ALIGN;
        e = slide::launch_fwd_mfma(p, q, k, v, wk, wv, bias, out, lse, workspace, (hipStream_t)stream);
    } else if (slide::fwd_mfma5_supported(p)) {
        if (!workspace || workspace_bytes < slide::fwd_mfma5_workspace_bytes(p)) return SLIDE_ERR_WORKSPACE;
        if (!aligned_to(workspace, 16)) return SLIDE_ERR_ALIGN;
        e = slide::launch_fwd_mfma5(p, q, k, v, wk, wv, bias, out, lse, workspace, (hipStream_t)stream);
    } else {
        // heads narrower than 32 channels through the matrix-core kernels on padded copies, when
        // the caller brought the workspace for them; the general kernel otherwise
        Problem p32;
        if (aligned16 && slide::fwd_padded_problem(p, p32) && workspace && aligned_to(workspace, 16) &&
            workspace_bytes >= slide::fwd_padded_workspace_bytes(p32))
            e = slide::launch_fwd_padded(p, p32, q, k, v, wk, wv, bias, out, lse, workspace, (hipStream_t)stream);
        else
            e = slide::launch_fwd_generic(p, q, k, v, wk, wv, bias, out, lse, (hipStream_t)stream);
    }
    return e == hipSuccess ? SLIDE_OK : SLIDE_ERR_HIP;
}

extern "C" int slide_attn_fwd(const void* q, const void* k, const void* v,
                              const float* wk, const float* wv, const float* bias, void* out,
                              float* lse,
                              int B, int H, int W, int C, int heads, int ksize, int dtype,
                              void* workspace, size_t workspace_bytes, void* stream)
{
    return forward(q, k, v, wk, wv, bias, out, lse, B, H, W, C, heads, ksize, dtype, 0,
                   workspace, workspace_bytes, stream);
}

extern "C" int slide_attn_fwd_noalloc(const void* q, const void* k, const void* v,
                                      const float* wk, const float* wv, const float* bias, void* out,
                                      float* lse,
                                      int B, int H, int W, int C, int heads, int ksize, int dtype,
                                      void* stream)
{
    // argument errors first, as in slide_attn_fwd, before the device is touched
    int st = check_problem(B, H, W, C, heads, ksize, dtype);
    if (st != SLIDE_OK) return st;
    if (!q || !k || !v || !wk || !wv || !out) return SLIDE_ERR_NULL;
    size_t need = slide_attn_workspace_bytes(B, H, W, C, heads, ksize, dtype, 0);
    {   // (heads of 64 channels whose partial logits do not fit the scratch run on the general kernel, which needs none)
        Problem pw{B, H, W, C, heads, ksize, dtype};
        Problem p32;
        if (need > NOALLOC_SCRATCH_BYTES && (slide::fwd_ring_wide_supported(pw, true) || slide::fwd_padded_problem(pw, p32))) need = 0;
    }
    if (need > NOALLOC_SCRATCH_BYTES) return SLIDE_ERR_WORKSPACE;
    void* ws = nullptr;
    if (noalloc_scratch(&ws) != hipSuccess) {
        (void)hipGetLastError();
        return SLIDE_ERR_HIP;
    }
    return forward(q, k, v, wk, wv, bias, out, lse, B, H, W, C, heads, ksize, dtype, 0,
                   ws, NOALLOC_SCRATCH_BYTES, stream);
}

extern "C" int slide_attn_fwd_two_branch(const void* q, const void* k, const void* v,
                                         const float* wk_learned, const float* wv_learned,
                                         const float* bias, void* out, float* lse,
                                         int B, int H, int W, int C, int heads, int ksize, int dtype,
                                         void* workspace, size_t workspace_bytes, void* stream)
{
    return forward(q, k, v, wk_learned, wv_learned, bias, out, lse, B, H, W, C, heads, ksize, dtype, 1,
                   workspace, workspace_bytes, stream);
}

extern "C" int slide_attn_fwd_shift(const void* q, const void* k, const void* v, const float* bias,
                                    void* out, float* lse,
                                    int B, int H, int W, int C, int heads, int ksize, int dtype, void* stream)
{
    int st = check_problem(B, H, W, C, heads, ksize, dtype);
    if (st != SLIDE_OK) return st;
    if (!q || !k || !v || !out) return SLIDE_ERR_NULL;
    const size_t esz = dtype == SLIDE_F32 ? 4 : 2;
    if (!aligned_to(q, esz) || !aligned_to(k, esz) || !aligned_to(v, esz) || !aligned_to(out, esz) ||
        !aligned_to(bias, 4) || !aligned_to(lse, 4))
        return SLIDE_ERR_ALIGN;
    Problem p{B, H, W, C, heads, ksize, dtype};
    const bool aligned16 = aligned_to(q, 16) && aligned_to(k, 16) && aligned_to(v, 16) && aligned_to(out, 16);
    hipError_t e;
    if ((slide::fwd_mfma_supported(p) || C == heads * 24) && slide::fwd_ring_enabled() && slide::fwd_ring_supported(p, aligned16))
        e = slide::launch_fwd_ring(p, q, k, v, nullptr, nullptr, bias, out, lse, true, (hipStream_t)stream);
    else if (slide::fwd_mfma_supported(p) && slide::fwd_ring_enabled() && slide::fwd_ring_strip_supported(p, aligned16))
        e = slide::launch_fwd_ring_strip(p, q, k, v, nullptr, nullptr, bias, out, lse, true, (hipStream_t)stream);
    else
        e = slide::launch_fwd_generic(p, q, k, v, nullptr, nullptr, bias, out, lse, (hipStream_t)stream);
    return e == hipSuccess ? SLIDE_OK : SLIDE_ERR_HIP;
}

extern "C" int slide_attn_fwd_nhwc(const void* q, const void* k, const void* v,
                                   const float* wk, const float* wv, const float* bias, void* out, float* lse,
                                   int B, int H, int W, int C, int heads, int ksize, int dtype, void* stream)
{
    int st = check_problem(B, H, W, C, heads, ksize, dtype);
    if (st != SLIDE_OK) return st;
    if (!q || !k || !v || !wk || !wv || !out) return SLIDE_ERR_NULL;
    const size_t esz = dtype == SLIDE_F32 ? 4 : 2;
    if (!aligned_to(q, esz) || !aligned_to(k, esz) || !aligned_to(v, esz) || !aligned_to(out, esz) ||
        !aligned_to(wk, 4) || !aligned_to(wv, 4) || !aligned_to(bias, 4) || !aligned_to(lse, 4))
        return SLIDE_ERR_ALIGN;
    Problem p{B, H, W, C, heads, ksize, dtype};
    p.nhwc = 1;
    const bool aligned16 = aligned_to(q, 16) && aligned_to(k, 16) && aligned_to(v, 16) && aligned_to(out, 16) &&
                           aligned_to(wk, 16) && aligned_to(wv, 16);
    hipError_t e;
    if (slide::fwd_ring_enabled() && slide::fwd_ring_nhwc_supported(p, aligned16))
        e = slide::launch_fwd_ring_nhwc(p, q, k, v, wk, wv, bias, out, lse, (hipStream_t)stream);
    else
        e = slide::launch_fwd_generic(p, q, k, v, wk, wv, bias, out, lse, (hipStream_t)stream);
    return e == hipSuccess ? SLIDE_OK : SLIDE_ERR_HIP;
}

extern "C" int slide_attn_fwd_traffic_probe(const void* q, const void* k, const void* v, void* out,
                                           int B, int H, int W, int C, int heads, int mode, void* stream)
{
    int st = check_problem(B, H, W, C, heads, 3, SLIDE_BF16);
    if (st != SLIDE_OK) return st;
    if (!q || !k || !v || !out) return SLIDE_ERR_NULL;
    if (mode != 0 && mode != 1) return SLIDE_ERR_SHAPE;
    if (!aligned_to(q, 16) || !aligned_to(k, 16) || !aligned_to(v, 16) || !aligned_to(out, 16)) return SLIDE_ERR_ALIGN;
    Problem p{B, H, W, C, heads, 3, SLIDE_BF16};
    if (((long)B * C * H * W) % 8 != 0) return SLIDE_ERR_SHAPE;
    if (mode == 1 && (C != heads * 32 || !slide::fwd_ring_supported(p, true))) return SLIDE_ERR_SHAPE;
    hipError_t e = slide::launch_fwd_traffic_probe(p, q, k, v, out, mode, (hipStream_t)stream);
    return e == hipSuccess ? SLIDE_OK : SLIDE_ERR_HIP;
}

static int backward(const void* dout, const void* q, const void* k, const void* v,
                    const float* wk, const float* wv, const float* bias,
                    const void* out, const float* lse,
                    void* dq, void* dk, void* dv, float* dwk, float* dwv, float* dbias,
                    int B, int H, int W, int C, int heads, int ksize, int dtype,
                    int two_branch, int accumulate,
                    void* workspace, size_t workspace_bytes, void* stream, bool nhwc = false)
{
    int st = check_problem(B, H, W, C, heads, ksize, dtype);
    if (st != SLIDE_OK) return st;
    if (!dout || !q || !k || !v || !wk || !wv || !dq || !dk || !dv || !dwk || !dwv) return SLIDE_ERR_NULL;
    if (bias && !dbias) return SLIDE_ERR_NULL;
    const size_t esz = dtype == SLIDE_F32 ? 4 : 2;
    // out and lse are optional and not read: the attention weights are recomputed from q and k
    const void* acts[] = {dout, q, k, v, dq, dk, dv, out};
    for (const void* a : acts)
        if (!aligned_to(a, esz)) return SLIDE_ERR_ALIGN;
    if (!aligned_to(wk, 4) || !aligned_to(wv, 4) || !aligned_to(bias, 4) || !aligned_to(dwk, 4) ||
        !aligned_to(dwv, 4) || !aligned_to(dbias, 4) || !aligned_to(workspace, 16) || !aligned_to(lse, 4))
        return SLIDE_ERR_ALIGN;
    Problem p{B, H, W, C, heads, ksize, dtype};
    p.two_branch = two_branch;
    p.accumulate = accumulate != 0;
    if (nhwc) {
        if (!workspace || workspace_bytes < slide::bwd_nhwc_workspace_bytes(p)) return SLIDE_ERR_WORKSPACE;
        hipError_t en = slide::launch_bwd_nhwc(p, dout, q, k, v, wk, wv, bias, dq, dk, dv, dwk, dwv,
                                               dbias, workspace, (hipStream_t)stream);
        return en == hipSuccess ? SLIDE_OK : SLIDE_ERR_HIP;
    }
    if (!workspace || workspace_bytes < slide::bwd_generic_workspace_bytes(p)) return SLIDE_ERR_WORKSPACE;
    hipError_t e = slide::launch_bwd_generic(p, dout, q, k, v, wk, wv, bias, dq, dk, dv, dwk, dwv,
                                             dbias, workspace, (hipStream_t)stream);
    return e == hipSuccess ? SLIDE_OK : SLIDE_ERR_HIP;
}

extern "C" size_t slide_attn_bwd_nhwc_workspace_bytes(int B, int H, int W, int C, int heads, int ksize, int dtype)
{
    if (check_problem(B, H, W, C, heads, ksize, dtype) != SLIDE_OK) return 0;
    Problem p{B, H, W, C, heads, ksize, dtype};
    return slide::bwd_nhwc_workspace_bytes(p);
}

extern "C" int slide_attn_bwd_nhwc(const void* dout, const void* q, const void* k, const void* v,
                                   const float* wk, const float* wv, const float* bias,
                                   void* dq, void* dk, void* dv,
                                   float* dwk, float* dwv, float* dbias, int two_branch, int accumulate,
                                   int B, int H, int W, int C, int heads, int ksize, int dtype,
                                   void* workspace, size_t workspace_bytes, void* stream)
{
    return backward(dout, q, k, v, wk, wv, bias, nullptr, nullptr, dq, dk, dv, dwk, dwv, dbias,
                    B, H, W, C, heads, ksize, dtype, two_branch != 0, accumulate, workspace, workspace_bytes,
                    stream, true);
}

extern "C" int slide_attn_bwd(const void* dout, const void* q, const void* k, const void* v,
                              const float* wk, const float* wv, const float* bias,
                              const void* out, const float* lse,
                              void* dq, void* dk, void* dv, float* dwk, float* dwv, float* dbias,
                              int B, int H, int W, int C, int heads, int ksize, int dtype,
                              void* workspace, size_t workspace_bytes, void* stream)
{
    return backward(dout, q, k, v, wk, wv, bias, out, lse, dq, dk, dv, dwk, dwv, dbias,
                    B, H, W, C, heads, ksize, dtype, 0, 0, workspace, workspace_bytes, stream);
}

extern "C" int slide_attn_bwd_two_branch(const void* dout, const void* q, const void* k, const void* v,
                                         const float* wk_learned, const float* wv_learned,
                                         const float* bias, const void* out, const float* lse,
                                         void* dq, void* dk, void* dv,
                                         float* dwk, float* dwv, float* dbias, int accumulate,
                                         int B, int H, int W, int C, int heads, int ksize, int dtype,
                                         void* workspace, size_t workspace_bytes, void* stream)
{
    return backward(dout, q, k, v, wk_learned, wv_learned, bias, out, lse, dq, dk, dv, dwk, dwv, dbias,
                    B, H, W, C, heads, ksize, dtype, 1, accumulate, workspace, workspace_bytes, stream);
}
