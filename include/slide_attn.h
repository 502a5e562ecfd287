/*
 * slide_attn.h -- C ABI of the MI355X (gfx950) Slide Attention library.
 *
 * The operator is per-pixel local self-attention over a k x k neighbourhood whose
 * keys and values come from a "deformed shift": k*k depthwise convolutions per
 * channel, each the sum of a fixed one-hot shift kernel and a learned kernel.
 *
 * Conventions shared by every entry point
 *   - All tensor pointers are DEVICE pointers owned by the caller.  The library
 *     never allocates, frees or synchronises; work is enqueued on `stream`
 *     (a hipStream_t passed as void*; NULL = the default stream).
 *   - Activations are contiguous NCHW [B, C, H, W]; `dtype` gives their element
 *     type (SLIDE_F32 or SLIDE_BF16).  Kernels, bias and all parameter gradients
 *     are always float32.  Arithmetic accumulates in float32.
 *   - Number format of the SLIDE_BF16 matrix-core paths (head size 32 with ksize 3 or 5; head
 *     size 24 with ksize 3 where slide_attn_fwd_variant says 24):
 *     inside the kernels the bf16 activations (q, k, v, dout) and the kernels wk, wv are held
 *     as IEEE half precision (11 significant bits, more than bf16's 8), products are formed
 *     in half precision from q/16 (dout/16), and every sum is accumulated in float32.  The
 *     conversion is exact for 2^-17 <= |x| <= 65504.  CONTRACT: finite inputs with
 *     |q|, |k|, |v|, |dout| <= 2^15 and |q*k|, |dout*v| < 2^20 per element, |wk|, |wv| < 2^11.
 *     Inside it results meet the bf16 tolerance (2e-2 relative to max(1, |result|)).
 *     Outside it nothing is rejected: magnitudes above 65504 saturate to +-65504
 *     (conversion rounds toward zero, never to infinity), magnitudes below 2^-24 become
 *     zero and those below 2^-17 lose low bits; NaN and infinity propagate.  SLIDE_F32
 *     problems and all other shapes compute in float32 throughout and have no such limits.
 *   - S = ksize*ksize.  Shift index s = (u+r)*ksize + (v+r) for u,v in [-r, r],
 *     r = ksize/2, reads the neighbour at offset (u, v) (row, column).  Tap index
 *     t = p*ksize + q reads offset (p-r, q-r): depthwise cross-correlation, no
 *     kernel flip.  Outside the map the input is zero; padded neighbours are not
 *     masked out of the softmax.
 *   - Head m owns channels [m*d, (m+1)*d), d = C/heads; logits are scaled by
 *     1/sqrt(d) inside the library.
 *   - Return value: SLIDE_OK or an error code.  Argument errors are detected on
 *     the host before any HIP call and leave all outputs untouched.
 */
#ifndef SLIDE_ATTN_H
#define SLIDE_ATTN_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SLIDE_OK = 0,
    SLIDE_ERR_NULL = 1,       /* a required pointer is NULL */
    SLIDE_ERR_SHAPE = 2,      /* a dimension < 1, C % heads != 0, ksize even or not in {1,3,5,7},
                                 or a size product that overflows 31 bits per plane */
    SLIDE_ERR_DTYPE = 3,      /* dtype is not SLIDE_F32 / SLIDE_BF16 */
    SLIDE_ERR_WORKSPACE = 4,  /* workspace NULL or smaller than slide_attn_workspace_bytes() */
    SLIDE_ERR_HIP = 5,        /* a kernel launch failed (hipGetLastError) */
    SLIDE_ERR_ALIGN = 6       /* a pointer is not aligned to its element size (workspace: 16 bytes) */
} slide_status;

typedef enum { SLIDE_F32 = 0, SLIDE_BF16 = 1 } slide_dtype;

/*
 * Re-parameterisation (Sec. 4.3, Fig. 4(2)): merge the fixed shift path and the
 * learned path of the deformed shifting module into one depthwise kernel,
 *     w_merged[c, s, t] = w_learned[c, s, t] + (t == s ? 1 : 0)
 * (the one-hot kernel of Eq. 11 generalised to every shift direction).
 * Both arrays are float32 [C, S, ksize, ksize] on the device; they may alias.
 */
int slide_reparam(const float* w_learned, float* w_merged, int C, int ksize, void* stream);

/*
 * Bytes of device scratch that slide_attn_fwd (backward == 0) or slide_attn_bwd
 * (backward != 0) needs for this problem.  Returns 0 if the arguments are
 * invalid or no scratch is needed.  Launches nothing; reads the compute-unit count of the
 * current device (256 if there is none).
 * For bf16 problems with ksize 3 whose heads have 64 channels or fewer than 32 the figure
 * includes what the matrix-core kernels need to serve that head size (partial sums exchanged
 * between half heads; copies padded to 32 channels per head: several times the size of an
 * activation tensor).  slide_attn_bwd requires it; a forward call that brings less scratch than
 * this (but enough for the general path: none) is served by the general kernel instead.
 */
size_t slide_attn_workspace_bytes(int B, int H, int W, int C, int heads, int ksize,
                                  int dtype, int backward);

/*
 * Forward (Sec. 3.1 Eq. 2 restricted to the local window; Sec. 4.1-4.3):
 *     Ks[c,s] = sum_t wk[c,s,t] * k[c, pixel + offset(t)]        (deformed shift of K)
 *     l[m,s]  = (1/sqrt(d)) * sum_{c in head m} q[c] * Ks[c,s] + bias[m,s]
 *     a       = softmax over s of l
 *     out[c]  = sum_s a[m(c),s] * Vs[c,s],  Vs as Ks with wv and v.
 * q, k, v, out: [B,C,H,W] of `dtype`.  wk, wv: MERGED kernels (output of
 * slide_reparam), float32 [C,S,ksize,ksize].  bias: float32 [heads,S] or NULL
 * (= zero).  out is overwritten and must not alias an input.  The k*k-fold
 * shifted tensors are never written to memory.
 * lse: float32 [B,heads,H,W] or NULL.  When given it receives, per pixel and head,
 * the natural logarithm of the softmax denominator of Eq. 2, log sum_s exp(l[m,s]),
 * so that a[s] = exp(l[m,s] - lse); NULL skips it at no cost.
 * workspace: device scratch of at least slide_attn_workspace_bytes(..., 0) bytes
 * (may be NULL when that is 0); contents are undefined afterwards.
 */
int slide_attn_fwd(const void* q, const void* k, const void* v,
                   const float* wk, const float* wv, const float* bias,
                   void* out, float* lse,
                   int B, int H, int W, int C, int heads, int ksize, int dtype,
                   void* workspace, size_t workspace_bytes, void* stream);

/*
 * slide_attn_fwd for callers that cannot allocate device memory or hand over a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, results and errors as slide_attn_fwd, minus the workspace: the kernels' scratch
 * (the per-head matrix-core operand images) lives in a fixed array of
 * SLIDE_NOALLOC_SCRATCH_BYTES inside the library, one per GPU, held until the process ends.
 * This call allocates and frees nothing.  A problem whose forward scratch
 * (slide_attn_workspace_bytes(..., 0)) exceeds that size returns SLIDE_ERR_WORKSPACE and
 * launches nothing (at head size 32: more than 113 heads at ksize 3, 20 heads at ksize 5).
 * All calls on one GPU share the array: calls that overlap in time on one GPU (different
 * streams or host threads) race on it; calls on the same stream are safe.  Nothing in it has
 * to start at zero (every call rewrites what it reads).
 */
#define SLIDE_NOALLOC_SCRATCH_BYTES (2u << 20)
int slide_attn_fwd_noalloc(const void* q, const void* k, const void* v,
                           const float* wk, const float* wv, const float* bias,
                           void* out, float* lse,
                           int B, int H, int W, int C, int heads, int ksize, int dtype,
                           void* stream);

/*
 * Backward of slide_attn_fwd (chain rule through the definition above; the
 * attention weights are recomputed from q and k):
 *     dq, dk, dv : [B,C,H,W] of `dtype`   (overwritten)
 *     dwk, dwv   : float32 [C,S,ksize,ksize] (overwritten; gradient with respect
 *                  to the merged kernel, which equals the gradient with respect
 *                  to the learned kernel)
 *     dbias      : float32 [heads,S] (overwritten; may be NULL if bias is NULL)
 * dout is the gradient of the loss with respect to `out`, same layout and dtype.
 * out, lse: the forward's results for the same inputs, or NULL.  They are optional
 * so that a caller that kept them can hand them over; this library recomputes the
 * attention weights from q and k in either case (the recomputation costs less than
 * reading them back), checks the two pointers for alignment only and never reads
 * through them.
 * Parameter gradients are accumulated in float32 in a fixed order (results are
 * reproducible run to run).
 * workspace: at least slide_attn_workspace_bytes(..., 1) bytes of device scratch, 16-byte
 * aligned (SLIDE_ERR_ALIGN otherwise).
 */
int slide_attn_bwd(const void* dout, const void* q, const void* k, const void* v,
                   const float* wk, const float* wv, const float* bias,
                   const void* out, const float* lse,
                   void* dq, void* dk, void* dv,
                   float* dwk, float* dwv, float* dbias,
                   int B, int H, int W, int C, int heads, int ksize, int dtype,
                   void* workspace, size_t workspace_bytes, void* stream);

/*
 * Training form (Sec. 4.3, Fig. 4(1)): the deformed shifting module with its two parallel
 * paths, the fixed one-hot shift and the learned depthwise kernel, before they are merged.
 * These two entry points take the LEARNED kernels wk_learned, wv_learned (float32
 * [C,S,ksize,ksize]) and add the shift path where the kernels are used,
 *     Ks[c,s] = k[c, pixel + offset(s)] + sum_t wk_learned[c,s,t] * k[c, pixel + offset(t)],
 * so a training step needs no slide_reparam call.  Results equal slide_attn_fwd /
 * slide_attn_bwd on slide_reparam(wk_learned), slide_reparam(wv_learned) up to rounding
 * (identical where the kernels enter as float32).  All other arguments, the workspace size
 * and the error behaviour are those of slide_attn_fwd / slide_attn_bwd.
 * accumulate != 0: dwk, dwv and dbias are added to what the arrays hold instead of
 * overwriting it (gradient accumulation over micro-batches; the caller zeroes them before
 * the first one); dq, dk, dv are always overwritten.
 */
int slide_attn_fwd_two_branch(const void* q, const void* k, const void* v,
                              const float* wk_learned, const float* wv_learned, const float* bias,
                              void* out, float* lse,
                              int B, int H, int W, int C, int heads, int ksize, int dtype,
                              void* workspace, size_t workspace_bytes, void* stream);
int slide_attn_bwd_two_branch(const void* dout, const void* q, const void* k, const void* v,
                              const float* wk_learned, const float* wv_learned, const float* bias,
                              const void* out, const float* lse,
                              void* dq, void* dk, void* dv,
                              float* dwk, float* dwv, float* dbias, int accumulate,
                              int B, int H, int W, int C, int heads, int ksize, int dtype,
                              void* workspace, size_t workspace_bytes, void* stream);

/*
 * Backward for channels-last activations (the layout of slide_attn_fwd_nhwc; the [B, HW, C]
 * token tensors of window-attention blocks, App. A): dout, q, k, v and dq, dk, dv are
 * [B,H,W,C] of `dtype`; kernels, bias and their gradients as in slide_attn_bwd.  The
 * activations are turned into [B,C,H,W] copies in the workspace, the backward kernels of
 * slide_attn_bwd run on those (same kernels, same results), and the three activation
 * gradients are turned back.  two_branch != 0: wk, wv are the learned kernels (as in
 * slide_attn_bwd_two_branch); accumulate as there.
 * workspace: at least slide_attn_bwd_nhwc_workspace_bytes(...) bytes (0 for invalid
 * arguments; host-only, no HIP call), 16-byte aligned.  Errors as slide_attn_bwd.
 */
size_t slide_attn_bwd_nhwc_workspace_bytes(int B, int H, int W, int C, int heads, int ksize, int dtype);
int slide_attn_bwd_nhwc(const void* dout, const void* q, const void* k, const void* v,
                        const float* wk, const float* wv, const float* bias,
                        void* dq, void* dk, void* dv,
                        float* dwk, float* dwv, float* dbias, int two_branch, int accumulate,
                        int B, int H, int W, int C, int heads, int ksize, int dtype,
                        void* workspace, size_t workspace_bytes, void* stream);

/* Human-readable name of a status code (static storage, never NULL). */
const char* slide_status_string(int status);

/*
 * Which forward implementation slide_attn_fwd would run for this problem:
 * 0 = invalid arguments, 1 = general kernel (any supported ksize / head size /
 * dtype, float32 vector arithmetic), 2 = matrix-core kernel (bf16, ksize 3, d = 32, or
 * d = 64 on maps the streaming kernel takes), 3 = matrix-core kernel for ksize 5 (bf16,
 * d = 32).  For tests and benchmarks.
 */
int slide_attn_fwd_path(int B, int H, int W, int C, int heads, int ksize, int dtype);

/*
 * The kernel inside that implementation, for tests that must know which code ran:
 * 0 = invalid arguments, 10 = general kernel, 20 = ksize-3 matrix-core kernel with one tile
 * per block, 21 / 23 = pipelined ksize-3 tile kernel (persistent blocks, next tile staged
 * during the passes of the current one) with the tile width taken from its arguments / fixed
 * at 64, 24 = streaming ksize-3 kernel (a block walks down a band of rows, K/V rows in an LDS
 * ring; maps 32..64 columns wide; head size 32, or 24 with the fourth channel octet of every
 * head left empty), 26 = the streaming kernel on column strips of 48, 40 or 32 (maps wider than 64
 * columns, W % 8 == 0, strips covering at most 1.25 W), 25 = two launches of the streaming kernel for heads of 64 channels (each
 * head as two halves of 32 whose shares of the logits cross the workspace; a call that brings
 * less workspace than slide_attn_workspace_bytes says runs on the general kernel), 30 = ksize-5
 * matrix-core kernel, 100 + v = heads narrower than 32 channels (bf16, ksize 3, H * W % 8 == 0)
 * through kernel v on copies of q, k, v and the kernels padded to 32 channels per head in the
 * workspace (again the general kernel for a call with less workspace).  aligned16: whether
 * q, k, v, out, wk, wv are all 16-byte aligned (kernels 21, 23, 24 need that).  Launches
 * nothing; reads the compute-unit count of the current device (256 if there is none).
 */
int slide_attn_fwd_variant(int B, int H, int W, int C, int heads, int ksize, int dtype,
                           int aligned16);

/*
 * The kernels slide_attn_bwd would run, for tests that must know which code ran: 0 = invalid
 * arguments, 10 = general kernels (float32 vector arithmetic), 20 = tiled matrix-core kernels
 * (bf16, d = 32, ksize 3; the kernel-gradient kernel also needs W % 8 == 0, else the general
 * one takes that part); 1 is added where the key and value gradients run in the streaming
 * kernel (maps 32..56 columns wide, W % 8 == 0, bands and rings that fit the LDS), 2 where the
 * per-pixel part (attention recompute, logit and query gradients) does (maps 32..64 columns
 * wide), 4 where the kernel and bias gradients do (maps 32..56 columns wide): 21 .. 27.
 * 100 + v: heads narrower than 32 channels (bf16, ksize 3, W % 8 == 0, 16-byte aligned pointers;
 * e.g. 24 channels per head): the kernels of variant v run on copies of q, k, v, dO and the
 * kernels padded with zero channels to 32 per head, made in the workspace (which is that much
 * larger for these shapes), with the logit scale of the true head size.
 * 200 + v: heads of 64 channels (bf16, ksize 3, maps the streaming per-pixel kernel takes, 16-byte
 * aligned pointers): every head runs as two half heads of 32 through the kernels of variant v;
 * the per-pixel part takes two launches, which exchange the halves' shares of the logits and of
 * the attention gradient through the workspace.
 * aligned16: whether every activation, gradient and workspace pointer is 16-byte aligned.
 * Launches nothing; reads the compute-unit count of the current device (256 if there is none).
 */
int slide_attn_bwd_variant(int B, int H, int W, int C, int heads, int ksize, int dtype,
                           int aligned16);

/*
 * Plain-shift forward: local attention over the ksize x ksize window whose keys and values
 * are the fixed shifts alone (Sec. 4.2: Eq. 9 rewritten as one-hot depthwise kernels in
 * Eq. 10-13; the "without deformed shifting" stage of Fig. 1 and Fig. 5).  Computes what
 * slide_attn_fwd computes for wk = wv = slide_reparam(0), i.e.
 *     Ks[c,s] = k[c, pixel + offset(s)],  Vs[c,s] = v[c, pixel + offset(s)]
 * (zero outside the map; those positions stay in the softmax), without reading any kernel
 * and with k*k instead of k^4 multiply-adds per pixel and channel.
 * q, k, v, bias, out, lse, the shape arguments, dtype, the number-format contract and the
 * error codes are those of slide_attn_fwd; there is no workspace.  Where
 * slide_attn_fwd_variant(...) says 24 the streaming matrix-core kernel runs in its plain
 * form; every other problem runs on the general kernel.
 */
int slide_attn_fwd_shift(const void* q, const void* k, const void* v, const float* bias,
                         void* out, float* lse,
                         int B, int H, int W, int C, int heads, int ksize, int dtype, void* stream);

/*
 * Forward for channels-last activations: q, k, v, out are [B, H, W, C] (the layout of the
 * [B, H*W, C] token tensors of window-attention backbones such as Slide-Swin, App. A), C
 * contiguous, head m owning channels [m*d, (m+1)*d) of every pixel.  Everything else -- the
 * operator (Sec. 3.1 Eq. 2, Sec. 4.1-4.3), the merged kernels wk, wv [C,S,ksize,ksize], bias,
 * lse [B,heads,H,W] (planar in either layout), dtype, the number-format contract, the error
 * codes -- is as for slide_attn_fwd; there is no workspace.  SLIDE_BF16 problems with head size
 * 32, ksize 3, 32 <= W <= 64, W % 8 == 0 and 16-byte aligned pointers run on the streaming
 * matrix-core kernel (the 8 channels a lane works on are 16 contiguous bytes in this layout:
 * nothing is transposed); every other problem runs on the general kernel.
 */
int slide_attn_fwd_nhwc(const void* q, const void* k, const void* v,
                        const float* wk, const float* wv, const float* bias,
                        void* out, float* lse,
                        int B, int H, int W, int C, int heads, int ksize, int dtype, void* stream);

/*
 * Measurement aid for benchmarks: moves the bytes of slide_attn_fwd on a SLIDE_BF16 problem
 * (reads q, k, v once, writes out once; ksize 3) with no arithmetic, so that the forward can be
 * held against what the memory system gives for its traffic.  out receives the bitwise XOR
 * of the data read (contents are meaningless).
 *   mode 0: flat copy-like access (every wave reads and writes contiguous kilobytes);
 *   mode 1: the blocks, bands, per-instruction address shapes and barriers of the streaming
 *           forward kernel (only where slide_attn_fwd_variant says 24; SLIDE_ERR_SHAPE
 *           otherwise).
 * All four pointers 16-byte aligned device pointers of B*C*H*W bf16 elements.
 */
int slide_attn_fwd_traffic_probe(const void* q, const void* k, const void* v, void* out,
                                 int B, int H, int W, int C, int heads, int mode, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SLIDE_ATTN_H */
