// Internal declarations shared by the translation units of libslide_attn.so.
// Not part of the public ABI (see include/slide_attn.h for that).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>
#include <initializer_list>
#include <cmath>
#include <mutex>

namespace slide {

struct Problem {
    int B, H, W, C, heads, ksize, dtype;
    // the kernels passed in are the LEARNED ones of the two-branch (training) form: the fixed
    // shift path is added where they are used (Sec. 4.3, Fig. 4(1)); 0: merged kernels
    int two_branch = 0;
    // backward: add the kernel and bias gradients to what dwk, dwv, dbias hold (micro-batches)
    int accumulate = 0;
    // activations are stored [B, H, W, C] (channels last) instead of [B, C, H, W]; forward only
    int nhwc = 0;
    // channels per head that the logit scale 1/sqrt(d) is taken from when the tensors handed to
    // the kernels carry heads padded to more channels (backward of heads narrower than 32); 0: d()
    int scale_dim = 0;
    int d() const { return C / heads; }
    float logit_scale() const { return 1.0f / sqrtf((float)(scale_dim ? scale_dim : d())); }
    int S() const { return ksize * ksize; }
    long plane() const { return (long)H * W; }
};

// Compute units of the current device, read from the runtime once per device and process
// (thread-safe).  MAX_CU_PLANNED when the query fails; never more than MAX_CU_PLANNED, which is
// what the host-only workspace query sizes per-block partial results for.
constexpr int MAX_CU_PLANNED = 256;
int device_cu_count();

// Opt-in of a set of kernels to `bytes` of dynamic LDS: the attribute belongs to the device that
// is current, so it is set once per device (safe when several host threads call into the
// library at the same time; the first error on a device sticks for that device).
struct LdsOptIn {
    static constexpr int MAX_DEV = 64;
    std::once_flag once[MAX_DEV];
    hipError_t err[MAX_DEV] = {};
    hipError_t ensure(std::initializer_list<const void*> kernels, int bytes)
    {
        auto set_all = [&]() {
            for (const void* f : kernels) {
                const hipError_t e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
                if (e != hipSuccess) return e;
            }
            return hipSuccess;
        };
        int dev = 0;
        const hipError_t eg = hipGetDevice(&dev);
        if (eg != hipSuccess) return eg;
        if (dev < 0 || dev >= MAX_DEV) return set_all();            // (beyond the table: every call)
        std::call_once(once[dev], [&] { err[dev] = set_all(); });
        return err[dev];
    }
};

// ---- general kernels (slide_generic.hip): any supported ksize / head size / dtype
hipError_t launch_reparam(const float* w_learned, float* w_merged, int C, int ksize, hipStream_t st);
hipError_t launch_fwd_generic(const Problem& p, const void* q, const void* k, const void* v,
                              const float* wk, const float* wv, const float* bias, void* out,
                              float* lse, hipStream_t st);
size_t bwd_generic_workspace_bytes(const Problem& p);
hipError_t launch_bwd_generic(const Problem& p, const void* dout, const void* q, const void* k,
                              const void* v, const float* wk, const float* wv, const float* bias,
                              void* dq, void* dk, void* dv, float* dwk, float* dwv, float* dbias,
                              void* workspace, hipStream_t st);

// forward of heads narrower than 32 channels (bf16, ksize 3, H * W % 8 == 0) through the
// matrix-core kernels on copies padded to 32 channels per head (p32: the padded problem)
bool fwd_padded_problem(const Problem& p, Problem& p32);
size_t fwd_padded_workspace_bytes(const Problem& p32);
hipError_t launch_fwd_padded(const Problem& p, const Problem& p32, const void* q, const void* k, const void* v,
                             const float* wk, const float* wv, const float* bias, void* out, float* lse,
                             void* workspace, hipStream_t st);

// channels-last activations [B, H, W, C]: the backward on copies turned into [B, C, H, W] in the
// workspace (p describes the problem without the layout flag)
size_t bwd_nhwc_workspace_bytes(const Problem& p);
hipError_t launch_bwd_nhwc(const Problem& p, const void* dout, const void* q, const void* k,
                           const void* v, const float* wk, const float* wv, const float* bias,
                           void* dq, void* dk, void* dv, float* dwk, float* dwv, float* dbias,
                           void* workspace, hipStream_t st);

// which kernels launch_bwd_generic runs: 10 general, 20 tiled matrix-core kernels, + 1 with the
// streaming dk/dv kernel, + 2 with the streaming per-pixel kernel, + 4 with the streaming form
// of the kernel-gradient kernel; aligned16: every pointer is 16-byte aligned
int bwd_variant(const Problem& p, bool aligned16);

// adds n_chunks partial sums per entry in a fixed order; bias_partial [n_chunks][nbias] -> dbias
// in the same launch (dbias may be null)
hipError_t launch_bwd_dw_reduce(const float* partial, float* dwk, float* dwv, long side, int n_chunks,
                                const float* bias_partial, float* dbias, int nbias, int accumulate,
                                hipStream_t st);

// ---- matrix-core kernel/bias gradients (slide_bwd_dw.hip): bf16, d == 32, ksize 3, W % 8 == 0
bool bwd_dw_mfma_supported(const Problem& p);
size_t bwd_dw_mfma_partial_floats(const Problem& p);
bool bwd_dw_ring_supported(const Problem& p);         // launch_bwd_dw_mfma runs its streaming form (maps 32..56 columns wide)
hipError_t launch_bwd_dw_mfma(const Problem& p, const void* dout, const void* q, const void* k,
                              const void* v, const void* attn_ws, const void* dl_ws,   // halves
                              float* partial, float* dwk, float* dwv, float* dbias, hipStream_t st);

// ---- matrix-core key/value gradients (slide_bwd16.hip): bf16, d == 32, ksize 3
bool bwd_dkdv_mfma_supported(const Problem& p);
size_t bwd_dkdv_mfma_image_bytes(const Problem& p);
size_t bwd_pixel_mfma_image_bytes(const Problem& p);
hipError_t launch_bwd_pixel_mfma(const Problem& p, const void* dout, const void* q, const void* k,
                                 const void* v, const float* wk, const float* wv, const float* bias,
                                 void* dq, void* attn_ws, void* dl_ws, bool half_ws, void* image_ws,
                                 void* dkdv_image_ws, bool streaming, hipStream_t st, float* part = nullptr);   // also prepares the dk/dv kernel's operand image; streaming: launch_bwd_pixel_ring does the rest; part: the heads are half heads of 64-channel heads (streaming only), see launch_bwd_pixel_ring
hipError_t launch_bwd_dkdv_mfma(const Problem& p, const void* dout, const void* q,
                                const float* wk, const float* wv,
                                const void* attn_ws, const void* dl_ws, bool half_ws,
                                void* dk, void* dv, void* image_ws, hipStream_t st);

// dwords per head of the dk/dv kernels' operand image (side x tap x channel half x lane x 2)
constexpr int BWD_DKDV_IMG_DWORDS = 2 * 9 * 2 * 64 * 2;

// dword offsets inside the per-pixel backward kernels' per-head operand image: merged K kernel
// and merged V kernel as logit-side operands (tap x lane x 4), merged K kernel as value-side
// operand (product x lane x 2), 16 bias words; dwords per head
constexpr int BWD_PX_A1K = 0, BWD_PX_A1V = 2304, BWD_PX_A2K = 4608, BWD_PX_BIAS = 6912, BWD_PX_IMG_DWORDS = 6928;

// the per-pixel backward by the streaming kernel (slide_bwd16_ring.hip): bf16, d == 32, ksize 3,
// 32 <= W <= 64, W % 8 == 0, every pointer 16-byte aligned, a and dl written as halves; reads the
// operand image that launch_bwd_pixel_mfma prepares
bool bwd_pixel_ring_supported(const Problem& p, bool aligned16);
hipError_t launch_bwd_pixel_ring(const Problem& p, const void* dout, const void* q, const void* k,
                                 const void* v, void* dq, void* attn_ws, void* dl_ws,
                                 const void* image_ws, hipStream_t st, int mode = 0, float* part = nullptr);
// (mode 1 / 2 with part [B, heads, 2, 9, H, W] float32: the heads are the half heads of heads of
// 64 channels; launch 1 writes every half's share of the logits and of da to part, launch 2 adds
// the other half's shares in and does the rest)

// the same gradients by the streaming kernel (slide_bwd16_ring.hip): bf16, d == 32, ksize 3,
// 32 <= W <= 56, W % 8 == 0, every pointer 16-byte aligned, a and dl as halves; reads the operand
// image that launch_bwd_pixel_mfma prepared
bool bwd_dkdv_ring_supported(const Problem& p, bool aligned16);
hipError_t launch_bwd_dkdv_ring(const Problem& p, const void* dout, const void* q,
                                const void* attn_ws, const void* dl_ws, void* dk, void* dv,
                                const void* image_ws, hipStream_t st);

// ---- matrix-core forward (slide_fwd16.hip): bf16, d == 32, ksize 3
bool fwd_mfma_supported(const Problem& p);
size_t fwd_mfma_workspace_bytes(const Problem& p);     // prepared weight operands, per head
// 20: one tile per block; 21, 23: pipelined tile kernel with the tile width read from its
// arguments / fixed at 64; 24: streaming kernel.  aligned16: every pointer is 16-byte aligned.
int fwd_mfma_variant(const Problem& p, bool aligned16);
hipError_t launch_fwd_mfma(const Problem& p, const void* q, const void* k, const void* v,
                           const float* wk, const float* wv, const float* bias, void* out,
                           float* lse, void* workspace, hipStream_t st);

// ---- streaming matrix-core forward (slide_fwd16_ring.hip): bf16, d == 32, ksize 3, 32 <= W <= 64,
// W % 8 == 0, every pointer 16-byte aligned; needs no workspace.  plain: the shift without
// learned kernels (Sec. 4.2, Eq. 10-13); wk and wv are not read then.
bool fwd_ring_supported(const Problem& p, bool aligned16);
bool fwd_ring_enabled();                               // false if the environment switches the streaming kernel off
hipError_t launch_fwd_ring(const Problem& p, const void* q, const void* k, const void* v,
                           const float* wk, const float* wv, const float* bias, void* out,
                           float* lse, bool plain, hipStream_t st);

// bands of rows per plane (nbp bands of rows_pb rows, n_blocks blocks in all), ring depth R and
// most new rows per epoch rpg of a streaming kernel with nw pass waves per block and per_cu
// blocks per compute unit; !ok: the map is not one a streaming kernel takes
struct RingRows { int nbp, rows_pb, n_blocks, R, rpg; bool ok; };
RingRows plan_ring_rows(const Problem& p, int nw, int per_cu);

// the streaming forward on maps wider than 64 columns (bf16, d == 32, ksize 3, W % 8 == 0): column
// strips of 48, 40 or 32, each with its neighbours' edge columns; needs no workspace
bool fwd_ring_strip_supported(const Problem& p, bool aligned16);
hipError_t launch_fwd_ring_strip(const Problem& p, const void* q, const void* k, const void* v,
                                 const float* wk, const float* wv, const float* bias, void* out,
                                 float* lse, bool plain, hipStream_t st);

// heads of 64 channels on the streaming forward (bf16, ksize 3, maps the streaming kernel
// takes): two launches over half heads, the halves' shares of the logits exchanged through the
// workspace (fwd_ring_wide_workspace_bytes, 16-byte aligned)
bool fwd_ring_wide_supported(const Problem& p, bool aligned16);
size_t fwd_ring_wide_workspace_bytes(const Problem& p);
hipError_t launch_fwd_ring_wide(const Problem& p, const void* q, const void* k, const void* v,
                                const float* wk, const float* wv, const float* bias, void* out,
                                float* lse, void* workspace, hipStream_t st);

// the streaming kernel for channels-last activations (Problem::nhwc): bf16, d == 32, ksize 3,
// 32 <= W <= 64, W % 8 == 0, every pointer 16-byte aligned; needs no workspace
bool fwd_ring_nhwc_supported(const Problem& p, bool aligned16);
hipError_t launch_fwd_ring_nhwc(const Problem& p, const void* q, const void* k, const void* v,
                                const float* wk, const float* wv, const float* bias, void* out,
                                float* lse, hipStream_t st);

// the forward's bytes without its arithmetic: mode 0 flat copy-like, mode 1 the streaming
// kernel's access pattern (needs fwd_ring_supported)
hipError_t launch_fwd_traffic_probe(const Problem& p, const void* q, const void* k, const void* v, void* out,
                                    int mode, hipStream_t st);

// ---- matrix-core forward, 5x5 window (slide_fwd16_k5.hip): bf16, d == 32, ksize 5
bool fwd_mfma5_supported(const Problem& p);
size_t fwd_mfma5_workspace_bytes(const Problem& p);
hipError_t launch_fwd_mfma5(const Problem& p, const void* q, const void* k, const void* v,
                            const float* wk, const float* wv, const float* bias, void* out,
                            float* lse, void* workspace, hipStream_t st);

}  // namespace slide
