// General Slide Attention kernels for gfx950: every supported window size, head
// size and element type, float32 vector arithmetic throughout.
//
// These kernels state the operator directly (Sec. 4.1-4.3 of the paper): for each
// pixel the k*k window of every channel is read with zero padding, the merged
// depthwise kernels are applied on the fly (the k*k-fold shifted tensor is never
// written to memory), logits get the per-head bias, a softmax runs over the k*k
// shifts and the shifted values are summed.  They serve float32 problems, head sizes
// other than 32 and window sizes the matrix-core kernel does not cover, and they
// are the whole backward pass.
//
// Thread mapping: one thread per (pixel, head, batch item); threads of a wavefront
// walk along W, so every per-channel read of q, k, v is a coalesced row segment and
// the window re-reads hit the vector L1.  Kernel weights are indexed only by
// block-uniform values, so the compiler fetches them through the scalar cache.
#include "slide_internal.h"
#include "slide_device.h"
#include <initializer_list>

namespace slide {

// ------------------------------------------------------------------ re-parameterisation
__global__ void reparam_kernel(const float* __restrict__ w_learned, float* __restrict__ w_merged,
                               long n, int S)
{
    long e = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= n) return;
    int t = (int)(e % S);
    int s = (int)((e / S) % S);
    w_merged[e] = w_learned[e] + (t == s ? 1.0f : 0.0f);
}

hipError_t launch_reparam(const float* w_learned, float* w_merged, int C, int ksize, hipStream_t st)
{
    int S = ksize * ksize;
    long n = (long)C * S * S;
    int threads = 256;
    long blocks = (n + threads - 1) / threads;
    hipLaunchKernelGGL(reparam_kernel, dim3((unsigned)blocks), dim3(threads), 0, st,
                       w_learned, w_merged, n, S);
    return hipGetLastError();
}

// ------------------------------------------------------------------ shared device pieces
// zero-padded k*k window of one channel plane around pixel (i, j)
template <typename T, int KS>
__device__ __forceinline__ void load_window(const T* __restrict__ plane, int i, int j, int H, int W,
                                            float (&win)[KS * KS], long sp = 1)
{
    constexpr int R = KS / 2;
#pragma unroll
    for (int p = 0; p < KS; ++p) {
        int y = i + p - R;
#pragma unroll
        for (int qq = 0; qq < KS; ++qq) {
            int x = j + qq - R;
            bool in = (y >= 0) && (y < H) && (x >= 0) && (x < W);
            win[p * KS + qq] = in ? Elem<T>::load(plane + ((long)y * W + x) * sp) : 0.0f;
        }
    }
}

// deformed shift of one channel at one pixel: shifted[s] = sum_t w[s][t] * win[t], plus the
// fixed shift path idw * win[s] (idw = 1 when w is the learned kernel of the two-branch form).
// w_c null: the plain shift (one-hot kernels, Eq. 10-13), shifted[s] = win[s].
template <int KS>
__device__ __forceinline__ void apply_kernels(const float* __restrict__ w_c,
                                              const float (&win)[KS * KS],
                                              float (&shifted)[KS * KS], float idw)
{
    constexpr int S = KS * KS;
    if (!w_c) {
#pragma unroll
        for (int s = 0; s < S; ++s) shifted[s] = win[s];
        return;
    }
#pragma unroll
    for (int s = 0; s < S; ++s) {
        float acc = idw * win[s];
#pragma unroll
        for (int t = 0; t < S; ++t) acc = fmaf(w_c[s * S + t], win[t], acc);
        shifted[s] = acc;
    }
}

// sum of x over the LPP adjacent lanes that share a pixel (every one of them gets the sum)
template <int LPP>
__device__ __forceinline__ float pixel_lanes_sum(float x)
{
#pragma unroll
    for (int w = 1; w < LPP; w <<= 1) x += __shfl_xor(x, w, 64);
    return x;
}

// logits over the S shifts for one pixel of one head, then softmax in place; lse receives
// the log of the softmax denominator, log sum_s exp(logit[s]).  LPP adjacent lanes share the
// pixel: lane cg takes the head's channels cg, cg + LPP, ... and the partial logits are
// added across the lanes (small problems get LPP = 8 so that they fill more of the chip).
template <typename T, int KS, int LPP>
__device__ __forceinline__ void attention_weights(const T* __restrict__ q, const T* __restrict__ k,
                                                  const float* __restrict__ wk,
                                                  const float* __restrict__ bias,
                                                  int b, int m, int i, int j, int H, int W, int C,
                                                  int d, int cg, float idw, float (&a)[KS * KS], float& lse,
                                                  long sc, long sp)
{
    constexpr int S = KS * KS;
    const long HW = (long)H * W;
    const long pix = (long)i * W + j;
    float dot[S];
#pragma unroll
    for (int s = 0; s < S; ++s) dot[s] = 0.0f;
    for (int cc = cg; cc < d; cc += LPP) {
        int c = m * d + cc;
        const T* kp = k + (long)b * C * HW + (long)c * sc;
        float win[S], ks[S];
        load_window<T, KS>(kp, i, j, H, W, win, sp);
        apply_kernels<KS>(wk ? wk + (long)c * S * S : nullptr, win, ks, idw);
        float qc = Elem<T>::load(q + (long)b * C * HW + (long)c * sc + pix * sp);
#pragma unroll
        for (int s = 0; s < S; ++s) dot[s] = fmaf(qc, ks[s], dot[s]);
    }
    const float scale = 1.0f / sqrtf((float)d);
    float mx = -INFINITY;
#pragma unroll
    for (int s = 0; s < S; ++s) {
        dot[s] = pixel_lanes_sum<LPP>(dot[s]);
        a[s] = fmaf(scale, dot[s], bias ? bias[m * S + s] : 0.0f);
        mx = fmaxf(mx, a[s]);
    }
    float den = 0.0f;
#pragma unroll
    for (int s = 0; s < S; ++s) { a[s] = expf(a[s] - mx); den += a[s]; }
    float inv = 1.0f / den;
    lse = mx + logf(den);
#pragma unroll
    for (int s = 0; s < S; ++s) a[s] *= inv;
}

// ------------------------------------------------------------------ forward
template <typename T, int KS, int LPP>
__global__ void __launch_bounds__(256)
fwd_generic_kernel(const T* __restrict__ q, const T* __restrict__ k, const T* __restrict__ v,
                   const float* __restrict__ wk, const float* __restrict__ wv,
                   const float* __restrict__ bias, T* __restrict__ out, float* __restrict__ lse,
                   int H, int W, int C, int heads, float idw, long sc, long sp)
{   // element (b, c, pixel) of an activation tensor is at b*C*H*W + c*sc + pixel*sp: sc = H*W,
    // sp = 1 for [B,C,H,W]; sc = 1, sp = C for [B,H,W,C]
    constexpr int S = KS * KS;
    const int d = C / heads;
    const int m = blockIdx.y, b = blockIdx.z;
    const long HW = (long)H * W;
    const long gid = (long)blockIdx.x * blockDim.x + threadIdx.x;
    const int cg = (int)(gid % LPP);
    // lanes past the last pixel work on the last one (they take part in the lane sums) and store nothing
    const bool live = gid / LPP < HW;
    const long pix = live ? gid / LPP : HW - 1;
    const int i = (int)(pix / W), j = (int)(pix % W);

    float a[S], lse_px;
    attention_weights<T, KS, LPP>(q, k, wk, bias, b, m, i, j, H, W, C, d, cg, idw, a, lse_px, sc, sp);
    if (lse && live && cg == 0) lse[((long)b * heads + m) * HW + pix] = lse_px;

    for (int cc = cg; cc < d; cc += LPP) {
        int c = m * d + cc;
        const T* vp = v + (long)b * C * HW + (long)c * sc;
        float win[S], vs[S];
        load_window<T, KS>(vp, i, j, H, W, win, sp);
        apply_kernels<KS>(wv ? wv + (long)c * S * S : nullptr, win, vs, idw);
        float acc = 0.0f;
#pragma unroll
        for (int s = 0; s < S; ++s) acc = fmaf(a[s], vs[s], acc);
        if (live) Elem<T>::store(out + (long)b * C * HW + (long)c * sc + pix * sp, acc);
    }
}

// small problems: 8 lanes per pixel and head
static bool few_pixels(const Problem& p) { return (long)p.B * p.heads * p.plane() < 262144; }

template <typename T, int KS>
static hipError_t launch_fwd_t(const Problem& p, const void* q, const void* k, const void* v,
                               const float* wk, const float* wv, const float* bias, void* out,
                               float* lse, hipStream_t st)
{
    const int lpp = few_pixels(p) ? 8 : 1;
    dim3 grid((unsigned)((p.plane() * lpp + 255) / 256), (unsigned)p.heads, (unsigned)p.B);
    const long sc = p.nhwc ? 1 : p.plane(), sp = p.nhwc ? p.C : 1;
    if (lpp == 8)
        hipLaunchKernelGGL((fwd_generic_kernel<T, KS, 8>), grid, dim3(256), 0, st,
                           (const T*)q, (const T*)k, (const T*)v, wk, wv, bias, (T*)out, lse,
                           p.H, p.W, p.C, p.heads, p.two_branch ? 1.0f : 0.0f, sc, sp);
    else
        hipLaunchKernelGGL((fwd_generic_kernel<T, KS, 1>), grid, dim3(256), 0, st,
                           (const T*)q, (const T*)k, (const T*)v, wk, wv, bias, (T*)out, lse,
                           p.H, p.W, p.C, p.heads, p.two_branch ? 1.0f : 0.0f, sc, sp);
    return hipGetLastError();
}

#define SLIDE_DISPATCH(FN, ...)                                                         \
    do {                                                                                \
        if (p.dtype == 0) {                                                             \
            switch (p.ksize) {                                                          \
                case 1: return FN<float, 1>(__VA_ARGS__);                               \
                case 3: return FN<float, 3>(__VA_ARGS__);                               \
                case 5: return FN<float, 5>(__VA_ARGS__);                               \
                case 7: return FN<float, 7>(__VA_ARGS__);                               \
            }                                                                           \
        } else {                                                                        \
            switch (p.ksize) {                                                          \
                case 1: return FN<bf16_bits, 1>(__VA_ARGS__);                           \
                case 3: return FN<bf16_bits, 3>(__VA_ARGS__);                           \
                case 5: return FN<bf16_bits, 5>(__VA_ARGS__);                           \
                case 7: return FN<bf16_bits, 7>(__VA_ARGS__);                           \
            }                                                                           \
        }                                                                               \
        return hipErrorInvalidValue;                                                    \
    } while (0)

hipError_t launch_fwd_generic(const Problem& p, const void* q, const void* k, const void* v,
                              const float* wk, const float* wv, const float* bias, void* out,
                              float* lse, hipStream_t st)
{
    SLIDE_DISPATCH(launch_fwd_t, p, q, k, v, wk, wv, bias, out, lse, st);
}

// ------------------------------------------------------------------ backward
// Step 1, one thread per (pixel, head, batch item): recompute the attention
// weights a[s]; da[s] = sum_c dO[c] Vs[c,s]; dl[s] = a[s] (da[s] - sum a da);
// dq[c] = scale * sum_s dl[s] Ks[c,s].  a and dl go to scratch as
// [B, heads, S, H, W] float32 for the gather steps below.
template <typename T, int KS, int LPP>
__global__ void __launch_bounds__(256)
bwd_pixel_kernel(const T* __restrict__ dout, const T* __restrict__ q, const T* __restrict__ k,
                 const T* __restrict__ v, const float* __restrict__ wk,
                 const float* __restrict__ wv, const float* __restrict__ bias,
                 T* __restrict__ dq, float* __restrict__ attn_ws, float* __restrict__ dl_ws,
                 int H, int W, int C, int heads, float idw)
{
    constexpr int S = KS * KS;
    const int d = C / heads;
    const int m = blockIdx.y, b = blockIdx.z;
    const long HW = (long)H * W;
    const long gid = (long)blockIdx.x * blockDim.x + threadIdx.x;
    const int cg = (int)(gid % LPP);
    const bool live = gid / LPP < HW;          // see fwd_generic_kernel
    const long pix = live ? gid / LPP : HW - 1;
    const int i = (int)(pix / W), j = (int)(pix % W);

    float a[S], lse_px;
    attention_weights<T, KS, LPP>(q, k, wk, bias, b, m, i, j, H, W, C, d, cg, idw, a, lse_px, (long)H * W, 1);

    float da[S];
#pragma unroll
    for (int s = 0; s < S; ++s) da[s] = 0.0f;
    for (int cc = cg; cc < d; cc += LPP) {
        int c = m * d + cc;
        float win[S], vs[S];
        load_window<T, KS>(v + ((long)b * C + c) * HW, i, j, H, W, win);
        apply_kernels<KS>(wv + (long)c * S * S, win, vs, idw);
        float doc = Elem<T>::load(dout + ((long)b * C + c) * HW + pix);
#pragma unroll
        for (int s = 0; s < S; ++s) da[s] = fmaf(doc, vs[s], da[s]);
    }
    float dsum = 0.0f;
#pragma unroll
    for (int s = 0; s < S; ++s) {
        da[s] = pixel_lanes_sum<LPP>(da[s]);
        dsum = fmaf(a[s], da[s], dsum);
    }
    float dl[S];
    const long ws_base = ((long)b * heads + m) * S * HW + pix;
#pragma unroll
    for (int s = 0; s < S; ++s) {
        dl[s] = a[s] * (da[s] - dsum);
        if (live && cg == 0) {
            attn_ws[ws_base + (long)s * HW] = a[s];
            dl_ws[ws_base + (long)s * HW] = dl[s];
        }
    }
    const float scale = 1.0f / sqrtf((float)d);
    for (int cc = cg; cc < d; cc += LPP) {
        int c = m * d + cc;
        float win[S], ks[S];
        load_window<T, KS>(k + ((long)b * C + c) * HW, i, j, H, W, win);
        apply_kernels<KS>(wk + (long)c * S * S, win, ks, idw);
        float acc = 0.0f;
#pragma unroll
        for (int s = 0; s < S; ++s) acc = fmaf(dl[s], ks[s], acc);
        if (live) Elem<T>::store(dq + ((long)b * C + c) * HW + pix, scale * acc);
    }
}

// Step 2, gather form of the transposed depthwise convolutions, one thread per
// (pixel y, head, batch item):
//   dk[c,y] = scale * sum_t q[c, y - off(t)] * sum_s wk[c,s,t] dl[s, y - off(t)]
//   dv[c,y] =         sum_t dO[c, y - off(t)] * sum_s wv[c,s,t] a[s, y - off(t)]
// over the taps t whose source pixel y - off(t) lies inside the map.  LPP adjacent lanes share
// the pixel and take every LPP-th group of CH channels (small problems: more lanes in flight).
template <typename T, int KS, int CH, int LPP>
__global__ void __launch_bounds__(256)
bwd_dkdv_kernel(const T* __restrict__ dout, const T* __restrict__ q,
                const float* __restrict__ wk, const float* __restrict__ wv,
                const float* __restrict__ attn_ws, const float* __restrict__ dl_ws,
                T* __restrict__ dk, T* __restrict__ dv, int H, int W, int C, int heads, float idw)
{
    constexpr int S = KS * KS, R = KS / 2;
    const int d = C / heads;
    const int m = blockIdx.y, b = blockIdx.z;
    const long HW = (long)H * W;
    const long gid = (long)blockIdx.x * blockDim.x + threadIdx.x;
    const long pix = gid / LPP;
    const int cg = (int)(gid % LPP);
    if (pix >= HW) return;
    const int i = (int)(pix / W), j = (int)(pix % W);
    const float scale = 1.0f / sqrtf((float)d);
    const long ws_head = ((long)b * heads + m) * S * HW;

    for (int c0 = cg * CH; c0 < d; c0 += LPP * CH) {
        float acc_k[CH], acc_v[CH];
#pragma unroll
        for (int e = 0; e < CH; ++e) { acc_k[e] = 0.0f; acc_v[e] = 0.0f; }
#pragma unroll
        for (int p = 0; p < KS; ++p) {
#pragma unroll
            for (int qq = 0; qq < KS; ++qq) {
                const int t = p * KS + qq;
                const int y = i - (p - R), x = j - (qq - R);     // source pixel of tap t
                const bool in = (y >= 0) && (y < H) && (x >= 0) && (x < W);
                const long src = in ? ((long)y * W + x) : 0;
                float dl[S], a[S];
#pragma unroll
                for (int s = 0; s < S; ++s) {
                    dl[s] = in ? dl_ws[ws_head + (long)s * HW + src] : 0.0f;
                    a[s] = in ? attn_ws[ws_head + (long)s * HW + src] : 0.0f;
                }
#pragma unroll
                for (int e = 0; e < CH; ++e) {
                    if (c0 + e < d) {
                        const int c = m * d + c0 + e;
                        const float* wkc = wk + (long)c * S * S + t;
                        const float* wvc = wv + (long)c * S * S + t;
                        float ck = idw * dl[t], cv = idw * a[t];     // the fixed shift path: shift t reads tap t
#pragma unroll
                        for (int s = 0; s < S; ++s) {
                            ck = fmaf(wkc[s * S], dl[s], ck);
                            cv = fmaf(wvc[s * S], a[s], cv);
                        }
                        const long off = ((long)b * C + c) * HW + src;
                        float qs = in ? Elem<T>::load(q + off) : 0.0f;
                        float ds = in ? Elem<T>::load(dout + off) : 0.0f;
                        acc_k[e] = fmaf(ck, qs, acc_k[e]);
                        acc_v[e] = fmaf(cv, ds, acc_v[e]);
                    }
                }
            }
        }
#pragma unroll
        for (int e = 0; e < CH; ++e) {
            if (c0 + e < d) {
                const long off = ((long)b * C + m * d + c0 + e) * HW + pix;
                Elem<T>::store(dk + off, scale * acc_k[e]);
                Elem<T>::store(dv + off, acc_v[e]);
            }
        }
    }
}

// Step 3, kernel gradients.  Block (c*S + s, chunk) sums over its chunk of
// (batch, pixel) items
//   dwk[c,s,t] += scale * dl[s,y] * q[c,y] * k[c, y + off(t)]
//   dwv[c,s,t] +=          a[s,y] * dO[c,y] * v[c, y + off(t)]
// per thread in registers, then across the block through LDS in a fixed tree
// order, and writes one partial per chunk; step 4 adds the chunks in order.
template <typename T, int KS>
__global__ void __launch_bounds__(256)
bwd_dw_partial_kernel(const T* __restrict__ dout, const T* __restrict__ q, const T* __restrict__ k,
                      const T* __restrict__ v, const float* __restrict__ attn_ws,
                      const float* __restrict__ dl_ws, float* __restrict__ partial,
                      int B, int H, int W, int C, int heads, long items_per_chunk)
{
    constexpr int S = KS * KS;
    const int d = C / heads;
    const int c = blockIdx.x / S, s = blockIdx.x % S;
    const int m = c / d;
    const long HW = (long)H * W;
    const long n_items = (long)B * HW;
    const long begin = (long)blockIdx.y * items_per_chunk;
    const long end = min(begin + items_per_chunk, n_items);
    const float scale = 1.0f / sqrtf((float)d);

    float acc_k[S], acc_v[S];
#pragma unroll
    for (int t = 0; t < S; ++t) { acc_k[t] = 0.0f; acc_v[t] = 0.0f; }
    for (long it = begin + threadIdx.x; it < end; it += blockDim.x) {
        const int b = (int)(it / HW);
        const long pix = it % HW;
        const int i = (int)(pix / W), j = (int)(pix % W);
        const long ws = (((long)b * heads + m) * S + s) * HW + pix;
        const long act = ((long)b * C + c) * HW;
        const float gk = scale * dl_ws[ws] * Elem<T>::load(q + act + pix);
        const float gv = attn_ws[ws] * Elem<T>::load(dout + act + pix);
        float win[S];
        load_window<T, KS>(k + act, i, j, H, W, win);
#pragma unroll
        for (int t = 0; t < S; ++t) acc_k[t] = fmaf(gk, win[t], acc_k[t]);
        load_window<T, KS>(v + act, i, j, H, W, win);
#pragma unroll
        for (int t = 0; t < S; ++t) acc_v[t] = fmaf(gv, win[t], acc_v[t]);
    }
    __shared__ float red[256];
    float* outp = partial + ((long)blockIdx.y * 2 * C * S + (long)c * S + s) * S;
    const long side = (long)C * S * S;     // dwv partials follow the dwk partials of a chunk
#pragma unroll
    for (int t = 0; t < 2 * S; ++t) {
        red[threadIdx.x] = (t < S) ? acc_k[t % S] : acc_v[t % S];
        __syncthreads();
        for (int w = 128; w > 0; w >>= 1) {
            if ((int)threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
            __syncthreads();
        }
        if (threadIdx.x == 0) outp[(t < S ? 0 : side) + (t % S)] = red[0];
        __syncthreads();
    }
}

// Step 4: add the per-chunk partials.  A block handles 64 consecutive output entries (the
// loads of a wave are 256 contiguous bytes); its 16 waves each add every 16th chunk in order,
// with 8 loads in flight, and the 16 sums per entry are combined in a fixed order through
// LDS, so the result does not depend on timing.  n = 2 * C*S*S entries.  Blocks past those
// entries add the bias-gradient partials [n_chunks][nbias] the same way (nbias may be 0).
constexpr int RED_GROUPS = 16;
__global__ void __launch_bounds__(64 * RED_GROUPS)
bwd_dw_reduce_kernel(const float* __restrict__ partial, float* __restrict__ dwk,
                     float* __restrict__ dwv, long side, int n_chunks,
                     const float* __restrict__ bias_partial, float* __restrict__ dbias, int nbias,
                     int accumulate)
{
    __shared__ float part[RED_GROUPS][64];
    const int el = threadIdx.x & 63, grp = threadIdx.x >> 6;
    const long dw_blocks = (2 * side + 63) / 64;
    const bool bias_job = blockIdx.x >= dw_blocks;
    const long e = (long)(bias_job ? blockIdx.x - dw_blocks : blockIdx.x) * 64 + el;
    const long n = bias_job ? nbias : 2 * side;
    const float* src = bias_job ? bias_partial : partial;
    const bool live = e < n;
    float acc = 0.0f;
    for (int base = grp; base < n_chunks; base += 8 * RED_GROUPS) {
        float x[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int ch = base + u * RED_GROUPS;
            x[u] = (live && ch < n_chunks) ? src[(long)ch * n + e] : 0.0f;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) acc += x[u];
    }
    part[grp][el] = acc;
    __syncthreads();
    if (grp == 0 && live) {
        float sum = part[0][el];
#pragma unroll
        for (int g2 = 1; g2 < RED_GROUPS; ++g2) sum += part[g2][el];
        float* dst = bias_job ? dbias + e : (e < side ? dwk + e : dwv + (e - side));
        *dst = accumulate ? *dst + sum : sum;
    }
}

// Step 5: dbias[m,s] = sum over batch and pixels of dl; one block per (m,s),
// fixed-order tree reduction.
__global__ void __launch_bounds__(256)
bwd_dbias_kernel(const float* __restrict__ dl_ws, float* __restrict__ dbias,
                 int B, long HW, int heads, int S, int accumulate)
{
    const int m = blockIdx.x / S, s = blockIdx.x % S;
    float acc = 0.0f;
    for (int b = 0; b < B; ++b) {
        const float* p = dl_ws + (((long)b * heads + m) * S + s) * HW;
        for (long x = threadIdx.x; x < HW; x += blockDim.x) acc += p[x];
    }
    __shared__ float red[256];
    red[threadIdx.x] = acc;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) dbias[blockIdx.x] = accumulate ? dbias[blockIdx.x] + red[0] : red[0];
}

static int dw_chunks(const Problem& p)
{
    long n_items = (long)p.B * p.plane();
    long want = 4096 / ((long)p.C * p.S()) + 1;
    long cap = (n_items + 1023) / 1024;          // at least ~1024 items per chunk
    long n = want < cap ? want : cap;
    if (n < 1) n = 1;
    if (n > 64) n = 64;
    return (int)n;
}

hipError_t launch_bwd_dw_reduce(const float* partial, float* dwk, float* dwv, long side, int n_chunks,
                                const float* bias_partial, float* dbias, int nbias, int accumulate,
                                hipStream_t st)
{
    if (!dbias) nbias = 0;
    const unsigned blocks = (unsigned)((2 * side + 63) / 64 + (nbias + 63) / 64);
    hipLaunchKernelGGL(bwd_dw_reduce_kernel, dim3(blocks), dim3(64 * RED_GROUPS),
                       0, st, partial, dwk, dwv, side, n_chunks, bias_partial, dbias, nbias, accumulate);
    return hipGetLastError();
}

// bytes of the partial kernel-gradient region (whichever kernel runs), a multiple of 16
static size_t bwd_partial_bytes(const Problem& p)
{
    size_t part = (size_t)dw_chunks(p) * 2 * (size_t)p.C * p.S() * p.S() * sizeof(float);
    if (bwd_dw_mfma_supported(p)) {
        const size_t part2 = bwd_dw_mfma_partial_floats(p) * sizeof(float);
        if (part2 > part) part = part2;
    }
    return (part + 15) & ~(size_t)15;
}

static size_t bwd_workspace_bytes_as_given(const Problem& p)
{
    size_t per = (size_t)p.B * p.heads * p.S() * (size_t)p.plane() * sizeof(float);
    return 2 * per + bwd_partial_bytes(p) + (bwd_dkdv_mfma_supported(p) ? bwd_dkdv_mfma_image_bytes(p) + bwd_pixel_mfma_image_bytes(p) : 0);
}

// ---- heads narrower than 32 channels (bf16, 3x3 window; e.g. 24 channels per head, App. A)
// The matrix-core backward kernels work on heads of 32 channels.  A narrower head is run
// through them on copies padded with zero channels: q, k, v, dO and the kernels are copied into
// the workspace with every head widened to 32 channels, the kernels run on the padded problem
// with the logit scale of the true head size, and dq, dk, dv, dwk, dwv are copied back without
// the padding (zero channels add nothing to logits, outputs or the other channels' gradients;
// dbias needs no copy).  Costs two more passes over the activations, far less than the
// general fp32 kernels these shapes ran on.
constexpr int PAD_D = 32;
static size_t pad_act_bytes(const Problem& p32)
{
    return (((size_t)p32.B * p32.C * (size_t)p32.plane() * 2) + 255) & ~(size_t)255;
}
static size_t pad_w_bytes(const Problem& p32)
{
    return (((size_t)p32.C * p32.S() * p32.S() * sizeof(float)) + 255) & ~(size_t)255;
}
// the padded problem, if this problem takes that path (decided from the shape alone)
static bool bwd_padded_problem(const Problem& p, Problem& p32)
{
    if (p.dtype != 1 || p.ksize != 3 || p.heads < 1 || p.C % p.heads != 0) return false;
    const int d = p.d();
    if (d < 1 || d >= PAD_D) return false;
    p32 = p;
    p32.C = p.heads * PAD_D;
    p32.scale_dim = d;
    if ((long)p.B * p32.C >= (1L << 31) || (p.plane() * 2 + 4095) / 4096 > 65535) return false;   // grid of the copy kernels
    return bwd_dkdv_mfma_supported(p32) && bwd_dw_mfma_supported(p32);
}
static size_t bwd_padded_workspace_bytes(const Problem& p32)
{
    const size_t inner = (bwd_workspace_bytes_as_given(p32) + 255) & ~(size_t)255;
    return inner + 7 * pad_act_bytes(p32) + 4 * pad_w_bytes(p32);
}

static bool bwd_wide_problem(const Problem& p, Problem& h);      // heads of 64 channels, below
static size_t bwd_wide_workspace_bytes(const Problem& h);

size_t bwd_generic_workspace_bytes(const Problem& p)
{
    size_t need = bwd_workspace_bytes_as_given(p);
    Problem p32;
    if (bwd_padded_problem(p, p32)) {
        const size_t padded = bwd_padded_workspace_bytes(p32);
        if (padded > need) need = padded;       // (pointers that are not 16-byte aligned still take the general kernels)
    }
    Problem h;
    if (bwd_wide_problem(p, h)) {
        const size_t wide = bwd_wide_workspace_bytes(h);
        if (wide > need) need = wide;
    }
    return need;
}

struct PadArgs {
    const uint4* src[4]; uint4* dst[4];         // tensors handled by one launch (blockIdx.z)
    int heads, d_src, d_dst;                    // channels per head in src and dst
    long chunks;                                // 16-byte chunks per channel plane
};
// dst[b][m * d_dst + j] = src[b][m * d_src + j] for j < min(d_src, d_dst); channels of dst past
// d_src are zero.  One thread per 16-byte chunk of a dst channel plane.
__global__ void __launch_bounds__(256)
repack_heads_kernel(const PadArgs a)
{
    const long x = (long)blockIdx.y * 256 + threadIdx.x;
    if (x >= a.chunks) return;
    const int cd = blockIdx.x;                  // channel of dst, over B * heads * d_dst
    const int per_item = a.heads * a.d_dst;
    const int b = cd / per_item, r = cd - b * per_item;
    const int m = r / a.d_dst, j = r - m * a.d_dst;
    const int t = blockIdx.z;
    uint4 val = make_uint4(0u, 0u, 0u, 0u);
    if (j < a.d_src) val = a.src[t][((long)(b * a.heads + m) * a.d_src + j) * a.chunks + x];
    a.dst[t][(long)cd * a.chunks + x] = val;
}
// the same for kernel tensors [C, S, S] float32 (n = S * S entries per channel), two tensors
__global__ void __launch_bounds__(256)
repack_kernels_kernel(const float* __restrict__ src0, const float* __restrict__ src1,
                      float* __restrict__ dst0, float* __restrict__ dst1,
                      int heads, int d_src, int d_dst, int n)
{
    const long e = (long)blockIdx.x * 256 + threadIdx.x;
    const long total = (long)heads * d_dst * n;
    if (e >= total) return;
    const int c = (int)(e / n), i = (int)(e - (long)c * n);
    const int m = c / d_dst, j = c - m * d_dst;
    const float* src = blockIdx.y ? src1 : src0;
    float* dst = blockIdx.y ? dst1 : dst0;
    dst[e] = j < d_src ? src[((long)(m * d_src + j)) * n + i] : 0.0f;
}

// every activation pointer and the workspace are 16-byte aligned (vector loads)
static bool aligned16(std::initializer_list<const void*> ptrs)
{
    for (const void* x : ptrs)
        if ((uintptr_t)x % 16 != 0) return false;
    return true;
}

template <typename T, int KS>
static hipError_t launch_bwd_t(const Problem& p, const void* dout, const void* q, const void* k,
                               const void* v, const float* wk, const float* wv, const float* bias,
                               void* dq, void* dk, void* dv, float* dwk, float* dwv, float* dbias,
                               void* workspace, hipStream_t st)
{
    const int S = p.S();
    const size_t per = (size_t)p.B * p.heads * S * (size_t)p.plane();
    float* attn_ws = (float*)workspace;
    float* dl_ws = attn_ws + per;
    float* partial = dl_ws + per;
    dim3 grid((unsigned)((p.plane() + 255) / 256), (unsigned)p.heads, (unsigned)p.B);
    const bool fast = bwd_dkdv_mfma_supported(p) && aligned16({dout, q, k, v, workspace});
    // when all three kernels are matrix-core kernels a and dl cross the workspace as halves
    // (in the first half of the same two regions)
    const bool half_ws = fast && bwd_dw_mfma_supported(p);
    hipError_t e;
    if (fast) {
        void* image_ws = (char*)partial + bwd_partial_bytes(p) + bwd_dkdv_mfma_image_bytes(p);
        void* dkdv_image_ws = (char*)partial + bwd_partial_bytes(p);
        // (the streaming kernel where it runs: maps of 32..64 columns, a and dl as halves)
        const bool streaming = half_ws && fwd_ring_enabled() && bwd_pixel_ring_supported(p, aligned16({dq}));
        e = launch_bwd_pixel_mfma(p, dout, q, k, v, wk, wv, bias, dq, attn_ws, dl_ws, half_ws, image_ws,
                                  dkdv_image_ws, streaming, st);
    } else {
        if (few_pixels(p)) {
            dim3 grid8((unsigned)((p.plane() * 8 + 255) / 256), (unsigned)p.heads, (unsigned)p.B);
            hipLaunchKernelGGL((bwd_pixel_kernel<T, KS, 8>), grid8, dim3(256), 0, st,
                               (const T*)dout, (const T*)q, (const T*)k, (const T*)v, wk, wv, bias,
                               (T*)dq, attn_ws, dl_ws, p.H, p.W, p.C, p.heads, p.two_branch ? 1.0f : 0.0f);
        } else
            hipLaunchKernelGGL((bwd_pixel_kernel<T, KS, 1>), grid, dim3(256), 0, st,
                               (const T*)dout, (const T*)q, (const T*)k, (const T*)v, wk, wv, bias,
                               (T*)dq, attn_ws, dl_ws, p.H, p.W, p.C, p.heads, p.two_branch ? 1.0f : 0.0f);
        e = hipGetLastError();
    }
    if (e != hipSuccess) return e;
    if (fast) {
        void* image_ws = (char*)partial + bwd_partial_bytes(p);
        // (the streaming kernel where it runs: maps of 32..56 columns, a and dl as halves)
        if (half_ws && fwd_ring_enabled() && bwd_dkdv_ring_supported(p, aligned16({dk, dv})))
            e = launch_bwd_dkdv_ring(p, dout, q, attn_ws, dl_ws, dk, dv, image_ws, st);
        else
            e = launch_bwd_dkdv_mfma(p, dout, q, wk, wv, attn_ws, dl_ws, half_ws, dk, dv, image_ws, st);
    } else {
        if (few_pixels(p)) {
            dim3 grid8((unsigned)((p.plane() * 8 + 255) / 256), (unsigned)p.heads, (unsigned)p.B);
            hipLaunchKernelGGL((bwd_dkdv_kernel<T, KS, 4, 8>), grid8, dim3(256), 0, st,
                               (const T*)dout, (const T*)q, wk, wv, attn_ws, dl_ws, (T*)dk, (T*)dv,
                               p.H, p.W, p.C, p.heads, p.two_branch ? 1.0f : 0.0f);
        } else
            hipLaunchKernelGGL((bwd_dkdv_kernel<T, KS, 8, 1>), grid, dim3(256), 0, st,
                               (const T*)dout, (const T*)q, wk, wv, attn_ws, dl_ws, (T*)dk, (T*)dv,
                               p.H, p.W, p.C, p.heads, p.two_branch ? 1.0f : 0.0f);
        e = hipGetLastError();
    }
    if (e != hipSuccess) return e;
    if (half_ws) {
        // kernel and bias gradients on the matrix cores
        return launch_bwd_dw_mfma(p, dout, q, k, v, attn_ws, dl_ws, partial, dwk, dwv, dbias, st);
    }
    const int n_chunks = dw_chunks(p);
    const long n_items = (long)p.B * p.plane();
    const long per_chunk = (n_items + n_chunks - 1) / n_chunks;
    hipLaunchKernelGGL((bwd_dw_partial_kernel<T, KS>), dim3((unsigned)(p.C * S), (unsigned)n_chunks),
                       dim3(256), 0, st,
                       (const T*)dout, (const T*)q, (const T*)k, (const T*)v, attn_ws, dl_ws,
                       partial, p.B, p.H, p.W, p.C, p.heads, per_chunk);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    const long side = (long)p.C * S * S;
    e = launch_bwd_dw_reduce(partial, dwk, dwv, side, n_chunks, nullptr, nullptr, 0, p.accumulate, st);
    if (e != hipSuccess) return e;
    if (dbias)
        hipLaunchKernelGGL(bwd_dbias_kernel, dim3((unsigned)(p.heads * S)), dim3(256), 0, st,
                           dl_ws, dbias, p.B, p.plane(), p.heads, S, p.accumulate);
    return hipGetLastError();
}

int bwd_variant(const Problem& p, bool all_aligned16)
{
    Problem p32;
    if (all_aligned16 && bwd_padded_problem(p, p32)) return 100 + bwd_variant(p32, true);
    if (all_aligned16 && bwd_wide_problem(p, p32)) return 200 + bwd_variant(p32, true);
    const bool fast = bwd_dkdv_mfma_supported(p) && all_aligned16;
    if (!fast) return 10;
    const bool half_ws = bwd_dw_mfma_supported(p);
    if (!half_ws || !fwd_ring_enabled()) return 20;
    return 20 + (bwd_dkdv_ring_supported(p, all_aligned16) ? 1 : 0) + (bwd_pixel_ring_supported(p, all_aligned16) ? 2 : 0) +
           (bwd_dw_ring_supported(p) ? 4 : 0);
}

// the backward of heads narrower than 32 channels through the matrix-core kernels (see above)
static hipError_t launch_bwd_padded(const Problem& p, const Problem& p32, const void* dout, const void* q,
                                    const void* k, const void* v, const float* wk, const float* wv,
                                    const float* bias, void* dq, void* dk, void* dv, float* dwk,
                                    float* dwv, float* dbias, void* workspace, hipStream_t st)
{
    const size_t inner = (bwd_workspace_bytes_as_given(p32) + 255) & ~(size_t)255;
    const size_t act = pad_act_bytes(p32), wb = pad_w_bytes(p32);
    char* base = (char*)workspace + inner;
    void* pin[4];                               // dO, q, k, v padded
    void* pout[3];                              // dq, dk, dv padded
    for (int i = 0; i < 4; ++i) pin[i] = base + (size_t)i * act;
    for (int i = 0; i < 3; ++i) pout[i] = base + (size_t)(4 + i) * act;
    float* wk32 = (float*)(base + 7 * act);
    float* wv32 = (float*)(base + 7 * act + wb);
    float* dwk32 = (float*)(base + 7 * act + 2 * wb);
    float* dwv32 = (float*)(base + 7 * act + 3 * wb);
    const int d = p.d(), n = p.S() * p.S();
    const long chunks = p.plane() * 2 / 16;     // (W % 8 == 0: a channel plane is whole 16-byte chunks)
    const unsigned gx = (unsigned)((chunks + 255) / 256);
    {
        PadArgs a{};
        const void* src[4] = {dout, q, k, v};
        for (int i = 0; i < 4; ++i) { a.src[i] = (const uint4*)src[i]; a.dst[i] = (uint4*)pin[i]; }
        a.heads = p.heads; a.d_src = d; a.d_dst = PAD_D; a.chunks = chunks;
        hipLaunchKernelGGL(repack_heads_kernel, dim3((unsigned)(p.B * p.heads * PAD_D), gx, 4), dim3(256), 0, st, a);
    }
    const unsigned gw = (unsigned)(((long)p.heads * PAD_D * n + 255) / 256);
    hipLaunchKernelGGL(repack_kernels_kernel, dim3(gw, 2), dim3(256), 0, st, wk, wv, wk32, wv32, p.heads, d, PAD_D, n);
    if (p.accumulate)                           // the sums continue from what dwk, dwv hold
        hipLaunchKernelGGL(repack_kernels_kernel, dim3(gw, 2), dim3(256), 0, st, (const float*)dwk, (const float*)dwv,
                           dwk32, dwv32, p.heads, d, PAD_D, n);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    e = launch_bwd_t<bf16_bits, 3>(p32, pin[0], pin[1], pin[2], pin[3], wk32, wv32, bias, pout[0], pout[1], pout[2],
                                dwk32, dwv32, dbias, workspace, st);
    if (e != hipSuccess) return e;
    {
        PadArgs a{};
        void* dst[3] = {dq, dk, dv};
        for (int i = 0; i < 3; ++i) { a.src[i] = (const uint4*)pout[i]; a.dst[i] = (uint4*)dst[i]; }
        a.heads = p.heads; a.d_src = PAD_D; a.d_dst = d; a.chunks = chunks;
        hipLaunchKernelGGL(repack_heads_kernel, dim3((unsigned)(p.B * p.heads * d), gx, 3), dim3(256), 0, st, a);
    }
    const unsigned gu = (unsigned)(((long)p.heads * d * n + 255) / 256);
    hipLaunchKernelGGL(repack_kernels_kernel, dim3(gu, 2), dim3(256), 0, st, (const float*)dwk32, (const float*)dwv32,
                       dwk, dwv, p.heads, PAD_D, d, n);
    return hipGetLastError();
}

// ---- forward of heads narrower than 32 channels, the same way (head size 24 on maps of the
// streaming kernel runs there directly and never comes here)
bool fwd_padded_problem(const Problem& p, Problem& p32)
{
    if (p.dtype != 1 || p.ksize != 3 || p.heads < 1 || p.C % p.heads != 0) return false;
    const int d = p.d();
    if (d < 1 || d >= PAD_D || p.plane() % 8 != 0) return false;     // (a channel plane is whole 16-byte chunks)
    p32 = p;
    p32.C = p.heads * PAD_D;
    p32.scale_dim = d;
    if ((long)p.B * p32.C >= (1L << 31) || (p.plane() * 2 + 4095) / 4096 > 65535) return false;
    return fwd_mfma_supported(p32);
}
size_t fwd_padded_workspace_bytes(const Problem& p32)
{
    const size_t inner = (fwd_mfma_workspace_bytes(p32) + 255) & ~(size_t)255;
    return inner + 4 * pad_act_bytes(p32) + 2 * pad_w_bytes(p32);
}
hipError_t launch_fwd_padded(const Problem& p, const Problem& p32, const void* q, const void* k, const void* v,
                             const float* wk, const float* wv, const float* bias, void* out, float* lse,
                             void* workspace, hipStream_t st)
{
    const size_t inner = (fwd_mfma_workspace_bytes(p32) + 255) & ~(size_t)255;
    const size_t act = pad_act_bytes(p32), wb = pad_w_bytes(p32);
    char* base = (char*)workspace + inner;
    void* pin[3] = {base, base + act, base + 2 * act};
    void* pout = base + 3 * act;
    float* wk32 = (float*)(base + 4 * act);
    float* wv32 = (float*)(base + 4 * act + wb);
    const int d = p.d(), n = p.S() * p.S();
    const long chunks = p.plane() * 2 / 16;
    const unsigned gx = (unsigned)((chunks + 255) / 256);
    {
        PadArgs a{};
        const void* src[3] = {q, k, v};
        for (int i = 0; i < 3; ++i) { a.src[i] = (const uint4*)src[i]; a.dst[i] = (uint4*)pin[i]; }
        a.heads = p.heads; a.d_src = d; a.d_dst = PAD_D; a.chunks = chunks;
        hipLaunchKernelGGL(repack_heads_kernel, dim3((unsigned)(p.B * p.heads * PAD_D), gx, 3), dim3(256), 0, st, a);
    }
    const unsigned gw = (unsigned)(((long)p.heads * PAD_D * n + 255) / 256);
    hipLaunchKernelGGL(repack_kernels_kernel, dim3(gw, 2), dim3(256), 0, st, wk, wv, wk32, wv32, p.heads, d, PAD_D, n);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    e = launch_fwd_mfma(p32, pin[0], pin[1], pin[2], wk32, wv32, bias, pout, lse, workspace, st);
    if (e != hipSuccess) return e;
    PadArgs a{};
    a.src[0] = (const uint4*)pout; a.dst[0] = (uint4*)out;
    a.heads = p.heads; a.d_src = PAD_D; a.d_dst = d; a.chunks = chunks;
    hipLaunchKernelGGL(repack_heads_kernel, dim3((unsigned)(p.B * p.heads * d), gx, 1), dim3(256), 0, st, a);
    return hipGetLastError();
}

// ---- heads of 64 channels (bf16, 3x3 window, maps the streaming per-pixel kernel takes)
// The matrix-core kernels work on heads of 32 channels.  Given the attention weights a and the
// logit gradients dl, the key, value and kernel gradients are separate per channel, so a head of
// 64 runs through them as two half heads; only the per-pixel part sums over the whole head
// (logits and da), which its streaming kernel does in two launches that exchange the halves'
// shares (launch_bwd_pixel_ring, modes 1 and 2).  Both halves write their own copy of a and dl;
// the bias gradient comes out once per half head and the first of each pair is kept.
static bool bwd_wide_problem(const Problem& p, Problem& h)
{
    if (p.dtype != 1 || p.ksize != 3 || p.C != p.heads * 64 || !fwd_ring_enabled()) return false;
    h = p;
    h.heads = 2 * p.heads;
    h.scale_dim = 64;
    if ((long)p.B * h.heads * 2 * p.S() * p.plane() >= (1L << 31)) return false;
    return bwd_dkdv_mfma_supported(h) && bwd_dw_mfma_supported(h) && bwd_pixel_ring_supported(h, true);
}
static size_t wide_part_bytes(const Problem& h)
{
    return (((size_t)h.B * h.heads * 2 * h.S() * (size_t)h.plane() * sizeof(float)) + 255) & ~(size_t)255;
}
static size_t bwd_wide_workspace_bytes(const Problem& h)
{
    const size_t dbias_tmp = (((size_t)h.heads * h.S() * sizeof(float)) + 255) & ~(size_t)255;
    return ((bwd_workspace_bytes_as_given(h) + 255) & ~(size_t)255) + wide_part_bytes(h) + dbias_tmp;
}
// tmp [2 heads][S] <-> dbias [heads][S]: row 2m of tmp is head m
__global__ void wide_dbias_kernel(float* __restrict__ tmp, float* __restrict__ dbias, int n, int S, int to_tmp)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    const int m = i / S, s = i - m * S;
    if (to_tmp) { tmp[(2 * m) * S + s] = dbias[i]; tmp[(2 * m + 1) * S + s] = 0.0f; }
    else dbias[i] = tmp[(2 * m) * S + s];
}

static hipError_t launch_bwd_wide(const Problem& p, const Problem& h, const void* dout, const void* q,
                                  const void* k, const void* v, const float* wk, const float* wv,
                                  const float* bias, void* dq, void* dk, void* dv, float* dwk,
                                  float* dwv, float* dbias, void* workspace, hipStream_t st)
{
    const int S = h.S();
    const size_t per = (size_t)h.B * h.heads * S * (size_t)h.plane();
    float* attn_ws = (float*)workspace;
    float* dl_ws = attn_ws + per;
    float* partial = dl_ws + per;
    void* dkdv_image_ws = (char*)partial + bwd_partial_bytes(h);
    void* image_ws = (char*)dkdv_image_ws + bwd_dkdv_mfma_image_bytes(h);
    char* extra = (char*)workspace + ((bwd_workspace_bytes_as_given(h) + 255) & ~(size_t)255);
    float* part = (float*)extra;
    float* dbias_tmp = (float*)(extra + wide_part_bytes(h));
    hipError_t e = launch_bwd_pixel_mfma(h, dout, q, k, v, wk, wv, bias, dq, attn_ws, dl_ws, true, image_ws,
                                         dkdv_image_ws, true, st, part);
    if (e != hipSuccess) return e;
    if (bwd_dkdv_ring_supported(h, true))
        e = launch_bwd_dkdv_ring(h, dout, q, attn_ws, dl_ws, dk, dv, dkdv_image_ws, st);
    else
        e = launch_bwd_dkdv_mfma(h, dout, q, wk, wv, attn_ws, dl_ws, true, dk, dv, dkdv_image_ws, st);
    if (e != hipSuccess) return e;
    const int nb = p.heads * S;
    if (dbias && p.accumulate)
        hipLaunchKernelGGL(wide_dbias_kernel, dim3((unsigned)((nb + 255) / 256)), dim3(256), 0, st, dbias_tmp, dbias, nb, S, 1);
    e = launch_bwd_dw_mfma(h, dout, q, k, v, attn_ws, dl_ws, partial, dwk, dwv, dbias ? dbias_tmp : nullptr, st);
    if (e != hipSuccess) return e;
    if (dbias)
        hipLaunchKernelGGL(wide_dbias_kernel, dim3((unsigned)((nb + 255) / 256)), dim3(256), 0, st, dbias_tmp, dbias, nb, S, 0);
    return hipGetLastError();
}

// ---- channels-last backward.  The backward kernels work on [B, C, H, W]; activations stored
// [B, H, W, C] (the [B, HW, C] token tensors of window-attention blocks, App. A) are turned into
// that layout in the workspace, the backward runs on the copies, and dq, dk, dv are turned back.
// Two more passes over the activations, as for the narrow heads above.
struct RelayoutArgs {
    const void* src[4]; void* dst[4];           // tensors of one launch (blockIdx.y)
    int B, C;
    long P;                                     // pixels per batch item
    int c_tiles; long p_tiles;                  // tiles of 64 channels / 64 pixels
};
constexpr int RL_TILE = 64, RL_ROW = RL_TILE + 8;   // (rows of the LDS tile stay 16-byte aligned)
// 2-byte elements, C % 8 == 0, P % 8 == 0, 16-byte aligned pointers: 16 bytes per thread on
// both sides, a 64 x 64 tile transposed through LDS.  TO_PLANAR: [B, P, C] -> [B, C, P].
template <bool TO_PLANAR>
__global__ void __launch_bounds__(256)
relayout16_kernel(const RelayoutArgs a)
{
    __shared__ __align__(16) uint16_t tile[RL_TILE * RL_ROW];
    long tid_tile = blockIdx.x;
    const long pt = tid_tile % a.p_tiles; tid_tile /= a.p_tiles;
    const int ct = (int)(tid_tile % a.c_tiles);
    const int b = (int)(tid_tile / a.c_tiles);
    const long p0 = pt * RL_TILE;
    const int c0 = ct * RL_TILE;
    const uint16_t* src = (const uint16_t*)a.src[blockIdx.y];
    uint16_t* dst = (uint16_t*)a.dst[blockIdx.y];
    const long item = (long)b * a.C * a.P;
#pragma unroll
    for (int it = 0; it < 2; ++it) {
        const int idx = it * 256 + threadIdx.x;
        // loads run along the contiguous axis of src: channels (TO_PLANAR) or pixels
        const int outer = idx >> 3, chunk = idx & 7;
        const long px = TO_PLANAR ? p0 + outer : p0 + 8 * chunk;
        const int ch = TO_PLANAR ? c0 + 8 * chunk : c0 + outer;
        if (px < a.P && ch < a.C) {
            const uint16_t* at = TO_PLANAR ? src + item + px * a.C + ch : src + item + (long)ch * a.P + px;
            const uint4 v = *(const uint4*)at;
            const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int e = 0; e < 8; ++e)           // tile[contiguous index of dst's rows ...][...]: row = the axis dst keeps outermost
                tile[(8 * chunk + e) * RL_ROW + outer] = (uint16_t)(w[e >> 1] >> (16 * (e & 1)));
        }
    }
    __syncthreads();
#pragma unroll
    for (int it = 0; it < 2; ++it) {
        const int idx = it * 256 + threadIdx.x;
        const int row = idx >> 3, chunk = idx & 7;     // row: channel (TO_PLANAR) or pixel of the tile
        const long px = TO_PLANAR ? p0 + 8 * chunk : p0 + row;
        const int ch = TO_PLANAR ? c0 + row : c0 + 8 * chunk;
        if (px < a.P && ch < a.C) {
            const uint4 v = *(const uint4*)(tile + row * RL_ROW + 8 * chunk);
            uint16_t* at = TO_PLANAR ? dst + item + (long)ch * a.P + px : dst + item + px * a.C + ch;
            *(uint4*)at = v;
        }
    }
}
// any element size and shape: one thread per element of dst
template <typename E, bool TO_PLANAR>
__global__ void __launch_bounds__(256)
relayout_elem_kernel(const RelayoutArgs a)
{
    const long n = (long)a.B * a.C * a.P;
    const long i = (long)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    const E* src = (const E*)a.src[blockIdx.y];
    E* dst = (E*)a.dst[blockIdx.y];
    if (TO_PLANAR) {                                     // dst [B, C, P]
        const long px = i % a.P; const long r = i / a.P;
        const int c = (int)(r % a.C); const long b = r / a.C;
        dst[i] = src[(b * a.P + px) * a.C + c];
    } else {                                             // dst [B, P, C]
        const int c = (int)(i % a.C); const long r = i / a.C;
        const long px = r % a.P; const long b = r / a.P;
        dst[i] = src[(b * a.C + c) * a.P + px];
    }
}

static hipError_t launch_relayout(const Problem& p, const void* const* src, void* const* dst, int count,
                                  bool to_planar, hipStream_t st)
{
    RelayoutArgs a{};
    bool fast = p.dtype == 1 && p.C % 8 == 0 && p.plane() % 8 == 0;
    for (int i = 0; i < count; ++i) {
        a.src[i] = src[i]; a.dst[i] = dst[i];
        fast = fast && (uintptr_t)src[i] % 16 == 0 && (uintptr_t)dst[i] % 16 == 0;
    }
    a.B = p.B; a.C = p.C; a.P = p.plane();
    a.c_tiles = (p.C + RL_TILE - 1) / RL_TILE;
    a.p_tiles = (a.P + RL_TILE - 1) / RL_TILE;
    const long tiles = (long)p.B * a.c_tiles * a.p_tiles;
    const long n = (long)p.B * p.C * a.P;
    if (fast && tiles < (1L << 31)) {
        if (to_planar) hipLaunchKernelGGL(relayout16_kernel<true>, dim3((unsigned)tiles, (unsigned)count), dim3(256), 0, st, a);
        else           hipLaunchKernelGGL(relayout16_kernel<false>, dim3((unsigned)tiles, (unsigned)count), dim3(256), 0, st, a);
    } else {
        const long blocks = (n + 255) / 256;
        if (blocks >= (1L << 31)) return hipErrorInvalidValue;
        const dim3 grid((unsigned)blocks, (unsigned)count);
        if (p.dtype == 1) {
            if (to_planar) hipLaunchKernelGGL((relayout_elem_kernel<uint16_t, true>), grid, dim3(256), 0, st, a);
            else           hipLaunchKernelGGL((relayout_elem_kernel<uint16_t, false>), grid, dim3(256), 0, st, a);
        } else {
            if (to_planar) hipLaunchKernelGGL((relayout_elem_kernel<uint32_t, true>), grid, dim3(256), 0, st, a);
            else           hipLaunchKernelGGL((relayout_elem_kernel<uint32_t, false>), grid, dim3(256), 0, st, a);
        }
    }
    return hipGetLastError();
}

static size_t nhwc_act_bytes(const Problem& p)
{
    return (((size_t)p.B * p.C * (size_t)p.plane() * (p.dtype == 0 ? 4 : 2)) + 255) & ~(size_t)255;
}

size_t bwd_nhwc_workspace_bytes(const Problem& p)
{
    return ((bwd_generic_workspace_bytes(p) + 255) & ~(size_t)255) + 7 * nhwc_act_bytes(p);
}

hipError_t launch_bwd_nhwc(const Problem& p, const void* dout, const void* q, const void* k,
                           const void* v, const float* wk, const float* wv, const float* bias,
                           void* dq, void* dk, void* dv, float* dwk, float* dwv, float* dbias,
                           void* workspace, hipStream_t st)
{
    const size_t inner = (bwd_generic_workspace_bytes(p) + 255) & ~(size_t)255;
    const size_t act = nhwc_act_bytes(p);
    char* base = (char*)workspace + inner;
    void* planar[7];                            // dO, q, k, v, dq, dk, dv as [B, C, H, W]
    for (int i = 0; i < 7; ++i) planar[i] = base + (size_t)i * act;
    const void* src[4] = {dout, q, k, v};
    hipError_t e = launch_relayout(p, src, planar, 4, true, st);
    if (e != hipSuccess) return e;
    e = launch_bwd_generic(p, planar[0], planar[1], planar[2], planar[3], wk, wv, bias, planar[4], planar[5],
                           planar[6], dwk, dwv, dbias, workspace, st);
    if (e != hipSuccess) return e;
    void* dst[3] = {dq, dk, dv};
    const void* back[3] = {planar[4], planar[5], planar[6]};
    return launch_relayout(p, back, dst, 3, false, st);
}

hipError_t launch_bwd_generic(const Problem& p, const void* dout, const void* q, const void* k,
                              const void* v, const float* wk, const float* wv, const float* bias,
                              void* dq, void* dk, void* dv, float* dwk, float* dwv, float* dbias,
                              void* workspace, hipStream_t st)
{
    Problem p32;
    if (bwd_padded_problem(p, p32) && aligned16({dout, q, k, v, dq, dk, dv, workspace}))
        return launch_bwd_padded(p, p32, dout, q, k, v, wk, wv, bias, dq, dk, dv, dwk, dwv, dbias, workspace, st);
    if (bwd_wide_problem(p, p32) && aligned16({dout, q, k, v, dq, dk, dv, workspace}))
        return launch_bwd_wide(p, p32, dout, q, k, v, wk, wv, bias, dq, dk, dv, dwk, dwv, dbias, workspace, st);
    SLIDE_DISPATCH(launch_bwd_t, p, dout, q, k, v, wk, wv, bias, dq, dk, dv, dwk, dwv, dbias,
                   workspace, st);
}

}  // namespace slide
