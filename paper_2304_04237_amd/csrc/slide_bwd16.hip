// Matrix-core backward of Slide Attention for gfx950 (bf16 activations, head size 32, 3x3
// window): the gradients of the keys and values.
//
// The paper gives no backward; this is the chain rule through the operator of Sec. 4.1-4.3.
// With a the attention weights and dl the logit gradients of a pixel (both produced by the
// per-pixel backward kernel, [B, heads, 9, H, W] as halves or float32) the deformed shift is a depthwise
// cross-correlation, so its transpose gathers, for a target pixel y, from the 9 source
// pixels p' = y - off(t) that see y through tap t:
//     dk[c,y] = scale * sum_t q[c,p']  * ( dl[p',t] + sum_s wl_k[c,s,t] dl[p',s] )
//     dv[c,y] =         sum_t dO[c,p'] * (  a[p',t] + sum_s wl_v[c,s,t]  a[p',s] )
// (source pixels outside the map contribute nothing; wl = merged kernel minus one-hot).
// The inner sums over s are the dense part: per source pixel a [32 channels x 9] x [9]
// product, run as v_mfma_f32_16x16x16_f16 with the 16 target pixels of a pass as columns.
// Walking the 3x3 window position u around y, the source pixel is y + off(u) and its tap is
// t = 8 - u.
//
// Tiles of q and dO are staged like the forward's k and v tiles; a and dl of the halo pixels
// are staged as 16-half records in the MFMA operand order (slot 4g+r holds shift 4r+g).
#include "slide_tile16.h"

namespace slide {
namespace b16path {
using namespace t16;

constexpr int WAVES = 4, THREADS = WAVES * 64;
constexpr int REC_BYTES = 32;                       // 16 halves per halo pixel and tensor

// Per-head image of the MFMA weight operands (dwords), written by prep_dkdv_weights:
//   side (K: 0, V: 1) x tap t (9) x channel half j (2) x lane (64) x 2 dwords.
// Row i of product (t, j) is channel 8*(i/4) + 4j + (i%4); dword y of lane (i, g) holds the
// merged weights (one-hot shift included) for the shifts of operand slots 4g+2y and 4g+2y+1.
constexpr int IMG_DWORDS = 2 * S * 2 * 64 * 2;      // 4608
static_assert(IMG_DWORDS == BWD_DKDV_IMG_DWORDS, "the streaming dk/dv kernel reads the same image");

// idw = 1: wk, wv are the learned kernels of the two-branch form and the fixed shift path
// (weight 1 where shift and tap coincide) is added here; 0: merged kernels
__device__ __forceinline__ void prep_dkdv_weights(const float* __restrict__ wk, const float* __restrict__ wv,
                                                  uint32_t* __restrict__ image, int t, int m, float idw)
{
    uint32_t* img = image + (long)m * IMG_DWORDS;
    for (int idx = threadIdx.x; idx < 2 * 2 * 128; idx += 256) {
        const int y = idx & 1, lane = (idx >> 1) & 63, j = (idx >> 7) & 1, side = idx >> 8;
        const int i = lane & 15, g = lane >> 4;
        const int c = m * D + 8 * (i >> 2) + 4 * j + (i & 3);
        const float* w = side ? wv : wk;
        float d[2] = {0.0f, 0.0f};
        for (int h = 0; h < 2; ++h) {
            const int s = shift_of_row(4 * g + 2 * y + h);
            if (s >= 0) d[h] = w[((long)c * S + s) * S + t] + ((s == t) ? idw : 0.0f);
        }
        img[((side * S + t) * 2 + j) * 128 + lane * 2 + y] = pack_half(d[0], d[1]);
    }
}

struct DkdvArgs {
    const bf16_bits* q; const bf16_bits* dout;
    const void* attn; const void* dl;         // [B, heads, 9, H, W], float32 or half (HALF_WS)
    bf16_bits* dk; bf16_bits* dv;
    const uint32_t* image;
    TileGrid g;                               // first staged tensor q, second dO
    int rec_dl, rec_a;                        // byte offsets of the dl / a records in LDS
    float scale;
};

// halo pixel record of one tensor (a or dl): 16 halves, slot kk holds shift shift_of_row(kk)
__device__ __forceinline__ void make_record(const float (&x)[S], uint4_t& lo, uint4_t& hi)
{
    lo[0] = pack_half(x[0], x[4]);  lo[1] = pack_half(x[8], 0.0f);   // slots 0..3
    lo[2] = pack_half(x[1], x[5]);  lo[3] = 0u;                      // slots 4..7
    hi[0] = pack_half(x[2], x[6]);  hi[1] = 0u;                      // slots 8..11
    hi[2] = pack_half(x[3], x[7]);  hi[3] = 0u;                      // slots 12..15
}

// the same record from values that are halves already
__device__ __forceinline__ void make_record(const _Float16 (&x)[S], uint4_t& lo, uint4_t& hi)
{
    const _Float16 z = (_Float16)0.0f;
    lo[0] = as_dword(half2_t{x[0], x[4]});  lo[1] = as_dword(half2_t{x[8], z});
    lo[2] = as_dword(half2_t{x[1], x[5]});  lo[3] = 0u;
    hi[0] = as_dword(half2_t{x[2], x[6]});  hi[1] = 0u;
    hi[2] = as_dword(half2_t{x[3], x[7]});  hi[3] = 0u;
}

// HALF_WS: a and dl come as halves (written so by the per-pixel kernel when every kernel of
// the backward is a matrix-core one), else as float32.
template <bool HALF_WS>
__global__ void __launch_bounds__(THREADS, 2)
bwd_dkdv_kernel16(const DkdvArgs a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int p = lane & 15, g = lane >> 4;
    const int HC = a.g.tw + 2;
    const long HW = (long)a.g.H * a.g.W;
    const uint32_t hw2 = (uint32_t)HW * 2u;

    const Tile tcur = decode_tile(a.g, blockIdx.x);

    // ---- stage q and dO halo tiles (loads of up to three items per thread in flight)
    for (int base = 0; base < tcur.n_items; base += 3 * THREADS) {
        uint4_t r[3][8];
#pragma unroll
        for (int u = 0; u < 3; ++u) {
            const int idx = base + u * THREADS + tid;
            if (idx < tcur.n_items) item_load(a.g, tcur, a.q, a.dout, idx, r[u]);
        }
#pragma unroll
        for (int u = 0; u < 3; ++u) {
            const int idx = base + u * THREADS + tid;
            if (idx < tcur.n_items) item_store(a.g, tcur, idx, r[u], smem);
        }
    }
    zero_pad_columns(a.g, tcur, smem, tid, THREADS);

    // ---- stage the dl and a records of every halo pixel (zero outside the map)
    {
        const int hrows = tcur.rows + 2, hcols = tcur.cols + 2;
        const int n_px = hrows * hcols;
        const float inv_hc = 1.0f / (float)hcols;
        const long plane_ws = ((long)(tcur.head_base / (HW * D))) * S * HW;   // (b*heads + m) * 9 * HW
        for (int idx = tid; idx < 2 * n_px; idx += THREADS) {
            const int tsel = idx >= n_px, id = idx - tsel * n_px;
            const int hr = (int)(((float)id + 0.5f) * inv_hc), hc = id - hr * hcols;
            const int gi = tcur.i0 - 1 + hr, gj = tcur.j0 - 1 + hc;
            const bool inside = gi >= 0 && gi < a.g.H && gj >= 0 && gj < a.g.W;
            const long at = plane_ws + (long)gi * a.g.W + gj;
            uint4_t lo, hi;
            if (HALF_WS) {
                _Float16 x[S];
#pragma unroll
                for (int s = 0; s < S; ++s) x[s] = (_Float16)0.0f;
                if (inside) {
                    const _Float16* src = (const _Float16*)(tsel ? a.attn : a.dl) + at;
#pragma unroll
                    for (int s = 0; s < S; ++s) x[s] = src[(long)s * HW];
                }
                make_record(x, lo, hi);
            } else {
                float x[S];
#pragma unroll
                for (int s = 0; s < S; ++s) x[s] = 0.0f;
                if (inside) {
                    const float* src = (const float*)(tsel ? a.attn : a.dl) + at;
#pragma unroll
                    for (int s = 0; s < S; ++s) x[s] = src[(long)s * HW];
                }
                make_record(x, lo, hi);
            }
            unsigned char* dst = smem + (tsel ? a.rec_a : a.rec_dl) + (hr * HC + hc) * REC_BYTES;
            *(uint4_t*)dst = lo;
            *(uint4_t*)(dst + 16) = hi;
        }
    }

    __syncthreads();

    // ---- MFMA weight operands of this head (loaded after the barrier: the staging registers
    // are free by now)
    const uint32_t* img = a.image + (long)tcur.m * IMG_DWORDS;
    half4_t Ak[S][2], Av[S][2];
#pragma unroll
    for (int t = 0; t < S; ++t) {
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const uint2_t wk2 = *(const uint2_t*)(img + ((0 * S + t) * 2 + j) * 128 + lane * 2);
            const uint2_t wv2 = *(const uint2_t*)(img + ((1 * S + t) * 2 + j) * 128 + lane * 2);
            Ak[t][j] = __builtin_bit_cast(half4_t, wk2);
            Av[t][j] = __builtin_bit_cast(half4_t, wv2);
        }
    }

    // ---- passes of 16 target pixels
    const int npix = tcur.rows * tcur.cols;
    const int npass = (npix + 15) >> 4;
    const float inv_tw = 1.0f / (float)tcur.cols;
    const unsigned char* ql = smem;
    const unsigned char* dol = smem + a.g.v_off;
    char* dkb = (char*)(a.dk + tcur.head_base);
    char* dvb = (char*)(a.dv + tcur.head_base);
    const uint32_t lane_chan = (uint32_t)(8 * g) * hw2 + ((uint32_t)tcur.i0 * a.g.W + tcur.j0) * 2u;
    const float4_t zero4 = {0.0f, 0.0f, 0.0f, 0.0f};

    for (int pass = wave; pass < npass; pass += WAVES) {
        int n = pass * 16 + p;
        const bool valid = n < npix;
        n = valid ? n : npix - 1;
        const int ti = (int)(((float)n + 0.5f) * inv_tw);
        const int tj = n - ti * tcur.cols;
        const uint32_t pix_off = lane_chan + ((uint32_t)ti * a.g.W + tj) * 2u;

        float dk[8], dv[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) { dk[e] = 0.0f; dv[e] = 0.0f; }
#pragma unroll
        for (int u = 0; u < S; ++u) {
            const int uy = u / KS, ux = u % KS;
            const int t = S - 1 - u;                               // tap through which y + off(u) sees y
            const int hpix = (ti + uy) * HC + tj + ux;             // halo pixel index of the source
            const unsigned char* rdl = smem + a.rec_dl + hpix * REC_BYTES;
            const unsigned char* ra = smem + a.rec_a + hpix * REC_BYTES;
            const half4_t Bdl = __builtin_bit_cast(half4_t, *(const uint2_t*)(rdl + 8 * g));
            const half4_t Ba = __builtin_bit_cast(half4_t, *(const uint2_t*)(ra + 8 * g));
            const int toff = (ti + uy) * HC * 64 + col_offset(tj + ux, g);
            const uint4_t qd = *(const uint4_t*)(ql + toff);
            const uint4_t dod = *(const uint4_t*)(dol + toff);
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const float4_t Lk = __builtin_amdgcn_mfma_f32_16x16x16f16(Ak[t][j], Bdl, zero4, 0, 0, 0);
                const float4_t Lv = __builtin_amdgcn_mfma_f32_16x16x16f16(Av[t][j], Ba, zero4, 0, 0, 0);
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int e = 4 * j + r;
                    const half2_t qh = as_half2(qd[e >> 1]), dh = as_half2(dod[e >> 1]);
                    dk[e] = fmaf(Lk[r], (float)qh[e & 1], dk[e]);
                    dv[e] = fmaf(Lv[r], (float)dh[e & 1], dv[e]);
                }
            }
            if (ux == KS - 1) {
                // one window row at a time: pin the partial sums here so that the multiply-adds
                // of this row are not all deferred to the end of the pass (which would keep
                // every MFMA result live at once)
#pragma unroll
                for (int e = 0; e < 8; ++e) asm volatile("" : "+v"(dk[e]), "+v"(dv[e]));
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        if (valid) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                *(bf16_bits*)(dkb + (pix_off + (uint32_t)e * hw2)) = f32_to_bf16(dk[e] * a.scale);
                *(bf16_bits*)(dvb + (pix_off + (uint32_t)e * hw2)) = f32_to_bf16(dv[e]);
            }
        }
    }
}

// ------------------------------------------------------------------ per-pixel backward
// For every pixel of a tile: recompute the attention weights a (as the forward does), then
//     da[s] = sum_c dO[c] Vs[c,s]        (same shape as the logits, with dO, v, wv)
//     dl[s] = a[s] (da[s] - sum_s' a[s'] da[s'])
//     dq[c] = scale * sum_t k[c,p+t] * sum_s dl[s] W~k[c,s,t]            (same shape as out)
// a and dl go to the workspace as [B, heads, 9, H, W] for the other two kernels: as halves
// when both of them are matrix-core kernels (which feed them to the matrix cores as halves
// anyway), as float32 when a general kernel reads them.
//
// Per-head operand image (dwords): A1k [0,2304): merged K kernel (times 16), tap t x lane x 4;
// A1v [2304,4608): merged V kernel (times 16), same arrangement; A2k [4608,6912): merged K
// kernel, product u (18) x lane x 2, arranged like the forward's V-side operand; bias rows.
// The kernels enter as halves, one-hot shift included (as in the forward).
constexpr int PX_A1K = 0, PX_A1V = 2304, PX_A2K = 4608, PX_BIAS = 6912, PX_IMG_DWORDS = 6928;
constexpr float G_SCALE = 0.0625f, W_SCALE = 16.0f;

__device__ __forceinline__ void prep_pixel_weights(const float* __restrict__ wk, const float* __restrict__ wv,
                                                   const float* __restrict__ bias, uint32_t* __restrict__ image,
                                                   int t, int m, float idw, int bias_shift)
{
    uint32_t* img = image + (long)m * PX_IMG_DWORDS;
    const int tid = threadIdx.x;
    {
        // A1 arrangement, tap t: dword y of lane (i, g) = merged weights of channels 8g+2y,
        // 8g+2y+1 for the shift of logit row i
        const int y = tid & 3, lane = tid >> 2;
        const int i = lane & 15, g = lane >> 4;
        const int s = shift_of_row(i);
        float k0 = 0.0f, k1 = 0.0f, v0 = 0.0f, v1 = 0.0f;
        if (s >= 0) {
            const int c = m * D + 8 * g + 2 * y;
            const float id = (s == t) ? idw : 0.0f;
            k0 = (wk[((long)c * S + s) * S + t] + id) * W_SCALE;
            k1 = (wk[((long)(c + 1) * S + s) * S + t] + id) * W_SCALE;
            v0 = (wv[((long)c * S + s) * S + t] + id) * W_SCALE;
            v1 = (wv[((long)(c + 1) * S + s) * S + t] + id) * W_SCALE;
        }
        img[PX_A1K + t * 256 + tid] = pack_half(k0, k1);
        img[PX_A1V + t * 256 + tid] = pack_half(v0, v1);
    }
    {
        // A2 arrangement of the K kernel, products u = 2t and 2t+1 (see the forward kernel)
        const int y = tid & 1, lane = (tid >> 1) & 63, u = 2 * t + (tid >> 7);
        const int i = lane & 15, g = lane >> 4;
        int c, tap;
        if (u < 16) { c = 8 * (i >> 2) + (u & 7); tap = 4 * (u >> 3) + (i & 3); }
        else        { c = 8 * (i >> 2) + 4 * (u - 16) + (i & 3); tap = 8; }
        c += m * D;
        float d[2] = {0.0f, 0.0f};
        for (int h = 0; h < 2; ++h) {
            const int s = shift_of_row(4 * g + 2 * y + h);
            if (s >= 0) d[h] = wk[((long)c * S + s) * S + tap] + ((s == tap) ? idw : 0.0f);
        }
        img[PX_A2K + u * 128 + (tid & 127)] = pack_half(d[0], d[1]);
    }
    if (t == 0 && tid < 16) {
        const int s = shift_of_row(tid);
        float b = -INFINITY;
        if (s >= 0) b = bias ? bias[(m >> bias_shift) * S + s] * 1.44269504088896341f : 0.0f;
        img[PX_BIAS + tid] = __float_as_uint(b);
    }
}

// Both operand images in one launch: blocks (t, m, 0) write tap t of head m of the per-pixel
// kernel's image, blocks (t, m, 1) that of the dk/dv kernel's.
__global__ void __launch_bounds__(256)
prep_bwd_weights_kernel(const float* __restrict__ wk, const float* __restrict__ wv,
                        const float* __restrict__ bias, uint32_t* __restrict__ pixel_image,
                        uint32_t* __restrict__ dkdv_image, float idw, int bias_shift)
{
    // (bias_shift 1: the heads are half heads of 64-channel heads, a pair shares a bias row)
    if (blockIdx.z == 0) prep_pixel_weights(wk, wv, bias, pixel_image, blockIdx.x, blockIdx.y, idw, bias_shift);
    else                 prep_dkdv_weights(wk, wv, dkdv_image, blockIdx.x, blockIdx.y, idw);
}

struct PixelArgs {
    const bf16_bits* dout; const bf16_bits* q; const bf16_bits* k; const bf16_bits* v;
    bf16_bits* dq;
    void* attn; void* dl;                     // [B, heads, 9, H, W], float32 or half (HALF_WS)
    const uint32_t* image;
    TileGrid g;                               // first staged tensor k, second v
    float scale, scale_log2e;
};

// x . (deformed shift of y) for the 9 shifts, through the matrix core with the merged kernel
// as half-precision operand (accumulated into acc, rows 4g+r of the 16x16 tile)
__device__ __forceinline__ void window_dots(const uint4_t (&yd)[S], const half2_t (&xs)[4],
                                            const half8_t (&A)[S], float4_t& acc)
{
    // (two accumulation chains, even and odd taps: a product does not wait for the one before it)
    float4_t accb = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int t = 0; t < S; ++t) {
        uint4_t bb;
#pragma unroll
        for (int y = 0; y < 4; ++y) bb[y] = as_dword(xs[y] * as_half2(yd[t][y]));
        if (t & 1) accb = __builtin_amdgcn_mfma_f32_16x16x32_f16(A[t], __builtin_bit_cast(half8_t, bb), accb, 0, 0, 0);
        else       acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(A[t], __builtin_bit_cast(half8_t, bb), acc, 0, 0, 0);
    }
    acc += accb;
}
// 8 channels as bf16 patterns (one per dword) -> halves divided by 16
__device__ __forceinline__ void raw_to_halves(const uint32_t (&raw)[8], half2_t (&sc)[4])
{
#pragma unroll
    for (int y = 0; y < 4; ++y)
        sc[y] = as_half2(pack_half_rtz(__uint_as_float(raw[2 * y] << 16), __uint_as_float(raw[2 * y + 1] << 16))) *
                half2_t{(_Float16)G_SCALE, (_Float16)G_SCALE};
}

template <bool HALF_WS>
__global__ void __launch_bounds__(THREADS, 2)
bwd_pixel_kernel16(const PixelArgs a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int p = lane & 15, g = lane >> 4;
    const int HC = a.g.tw + 2;
    const long HW = (long)a.g.H * a.g.W;
    const uint32_t hw2 = (uint32_t)HW * 2u;

    const Tile tcur = decode_tile(a.g, blockIdx.x);
    for (int base = 0; base < tcur.n_items; base += 3 * THREADS) {
        uint4_t r[3][8];
#pragma unroll
        for (int u = 0; u < 3; ++u) {
            const int idx = base + u * THREADS + tid;
            if (idx < tcur.n_items) item_load(a.g, tcur, a.k, a.v, idx, r[u]);
        }
#pragma unroll
        for (int u = 0; u < 3; ++u) {
            const int idx = base + u * THREADS + tid;
            if (idx < tcur.n_items) item_store(a.g, tcur, idx, r[u], smem);
        }
    }
    zero_pad_columns(a.g, tcur, smem, tid, THREADS);
    __syncthreads();

    const uint32_t* img = a.image + (long)tcur.m * PX_IMG_DWORDS;
    half8_t A1k[S], A1v[S];
    half4_t A2k[2 * S];
#pragma unroll
    for (int t = 0; t < S; ++t) {
        A1k[t] = __builtin_bit_cast(half8_t, *(const uint4_t*)(img + PX_A1K + (t * 64 + lane) * 4));
        A1v[t] = __builtin_bit_cast(half8_t, *(const uint4_t*)(img + PX_A1V + (t * 64 + lane) * 4));
    }
#pragma unroll
    for (int u = 0; u < 2 * S; ++u)
        A2k[u] = __builtin_bit_cast(half4_t, *(const uint2_t*)(img + PX_A2K + (u * 64 + lane) * 2));
    float bias2[3];
#pragma unroll
    for (int r = 0; r < 3; ++r) bias2[r] = __uint_as_float(img[PX_BIAS + 4 * g + r]);

    const int npix = tcur.rows * tcur.cols;
    const int npass = (npix + 15) >> 4;
    const float inv_tw = 1.0f / (float)tcur.cols;
    const unsigned char* kl = smem;
    const unsigned char* vl = smem + a.g.v_off;
    const char* qb = (const char*)(a.q + tcur.head_base);
    const char* dob = (const char*)(a.dout + tcur.head_base);
    char* dqb = (char*)(a.dq + tcur.head_base);
    const uint32_t lane_chan = (uint32_t)(8 * g) * hw2 + ((uint32_t)tcur.i0 * a.g.W + tcur.j0) * 2u;
    const long ws_plane = ((long)(tcur.head_base / (HW * D))) * S * HW + (long)tcur.i0 * a.g.W + tcur.j0;

    auto pixel_of = [&](int pass, int& ti, int& tj) -> bool {
        int n = pass * 16 + p;
        const bool valid = n < npix;
        n = valid ? n : npix - 1;
        ti = (int)(((float)n + 0.5f) * inv_tw);
        tj = n - ti * tcur.cols;
        return valid;
    };

    uint32_t qraw[8], draw[8];
    {
        int ti0, tj0;
        pixel_of(min(wave, npass - 1), ti0, tj0);
        const uint32_t off = lane_chan + ((uint32_t)ti0 * a.g.W + tj0) * 2u;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            qraw[e] = *(const bf16_bits*)(qb + (off + (uint32_t)e * hw2));
            draw[e] = *(const bf16_bits*)(dob + (off + (uint32_t)e * hw2));
        }
    }
    for (int pass = wave; pass < npass; pass += WAVES) {
        int ti, tj;
        const bool valid = pixel_of(pass, ti, tj);
        const uint32_t pix_off = lane_chan + ((uint32_t)ti * a.g.W + tj) * 2u;
        int coff[KS];
#pragma unroll
        for (int tx = 0; tx < KS; ++tx) coff[tx] = col_offset(tj + tx, g);
        const int row0 = ti * HC * 64;

        // ---- attention weights (as in the forward)
        uint4_t xd[S];
#pragma unroll
        for (int t = 0; t < S; ++t) xd[t] = *(const uint4_t*)(kl + row0 + (t / KS) * HC * 64 + coff[t % KS]);
        half2_t xs[4];
        raw_to_halves(qraw, xs);
        float4_t acc = {0.0f, 0.0f, 0.0f, 0.0f};
        window_dots(xd, xs, A1k, acc);
        // next pass's q and dO: issued now, used at the end of this pass
        uint32_t qnext[8], dnext[8];
        {
            int ti2, tj2;
            pixel_of(min(pass + WAVES, npass - 1), ti2, tj2);
            const uint32_t off = lane_chan + ((uint32_t)ti2 * a.g.W + tj2) * 2u;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                qnext[e] = *(const bf16_bits*)(qb + (off + (uint32_t)e * hw2));
                dnext[e] = *(const bf16_bits*)(dob + (off + (uint32_t)e * hw2));
            }
        }
        // v taps for the da step
#pragma unroll
        for (int t = 0; t < S; ++t) xd[t] = *(const uint4_t*)(vl + row0 + (t / KS) * HC * 64 + coff[t % KS]);
        float l[3], pr[3];
#pragma unroll
        for (int r = 0; r < 3; ++r) l[r] = fmaf(acc[r], a.scale_log2e, bias2[r]);
        const float mx = allmax_groups(fmaxf(fmaxf(l[0], l[1]), l[2]));
#pragma unroll
        for (int r = 0; r < 3; ++r) pr[r] = __builtin_amdgcn_exp2f(l[r] - mx);
        const float inv = __builtin_amdgcn_rcpf(allsum_groups(pr[0] + pr[1] + pr[2]));
#pragma unroll
        for (int r = 0; r < 3; ++r) pr[r] *= inv;

        // ---- da[s] = dO . Vs[s], then dl
        raw_to_halves(draw, xs);
        acc = float4_t{0.0f, 0.0f, 0.0f, 0.0f};
        window_dots(xd, xs, A1v, acc);
        // k taps again for the dq step
#pragma unroll
        for (int t = 0; t < S; ++t) xd[t] = *(const uint4_t*)(kl + row0 + (t / KS) * HC * 64 + coff[t % KS]);
        const float dsum = allsum_groups(pr[0] * acc[0] + pr[1] * acc[1] + pr[2] * acc[2]);
        float dl[3];
#pragma unroll
        for (int r = 0; r < 3; ++r) dl[r] = pr[r] * (acc[r] - dsum);
        if (valid) {
            const long wo = ws_plane + (long)ti * a.g.W + tj;
#pragma unroll
            for (int r = 0; r < 3; ++r) {
                if (r < 2 || g == 0) {
                    const long at = wo + (long)(4 * r + g) * HW;
                    if (HALF_WS) {
                        ((_Float16*)a.attn)[at] = (_Float16)pr[r];
                        ((_Float16*)a.dl)[at] = (_Float16)dl[r];
                    } else {
                        ((float*)a.attn)[at] = pr[r];
                        ((float*)a.dl)[at] = dl[r];
                    }
                }
            }
        }

        // ---- dq[c] = scale * sum_t k[c,p+t] * (sum_s dl[s] W~k[c,s,t]): the inner sum on the
        // matrix core, as the forward's V side
        const float4_t c0 = {0.0f, 0.0f, 0.0f, 0.0f}, c1 = c0;
        uint2_t b2;
        b2[0] = pack_half(dl[0], dl[1]);
        b2[1] = pack_half(dl[2], 0.0f);
        const half4_t B2 = __builtin_bit_cast(half4_t, b2);
        // the 18 products, each two products ahead of the multiply-adds that use it (product uu < 16:
        // channel uu % 8 of the lane's octet, taps 4 (uu / 8) .. + 3; 16, 17: tap 8 of channels 0..3, 4..7)
        float o[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = 0.0f;
        float4_t w[2 * S];
        constexpr int AHEAD = 2;
#pragma unroll
        for (int uu = 0; uu < AHEAD; ++uu) w[uu] = __builtin_amdgcn_mfma_f32_16x16x16f16(A2k[uu], B2, c0, 0, 0, 0);
#pragma unroll
        for (int uu = 0; uu < 2 * S; ++uu) {
            if (uu + AHEAD < 2 * S) w[uu + AHEAD] = __builtin_amdgcn_mfma_f32_16x16x16f16(A2k[uu + AHEAD], B2, c1, 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int e = uu < 16 ? (uu & 7) : 4 * (uu - 16) + r;
                const int tap = uu < 16 ? 4 * (uu >> 3) + r : 8;
                o[e] = fmaf(w[uu][r], (float)as_half2(xd[tap][e >> 1])[e & 1], o[e]);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        if (valid) {
#pragma unroll
            for (int e = 0; e < 8; ++e)
                *(bf16_bits*)(dqb + (pix_off + (uint32_t)e * hw2)) = f32_to_bf16(o[e] * a.scale);
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) { qraw[e] = qnext[e]; draw[e] = dnext[e]; }
    }
}

static TilePlan plan_dkdv(const Problem& p)
{
    return plan_tiles(p, LDS_LIMIT / 2, 64, 64, 2 * REC_BYTES);
}

}  // namespace b16path

size_t bwd_pixel_mfma_image_bytes(const Problem& p)
{
    return (size_t)p.heads * b16path::PX_IMG_DWORDS * sizeof(uint32_t);
}

hipError_t launch_bwd_pixel_mfma(const Problem& p, const void* dout, const void* q, const void* k,
                                 const void* v, const float* wk, const float* wv, const float* bias,
                                 void* dq, void* attn_ws, void* dl_ws, bool half_ws, void* image_ws,
                                 void* dkdv_image_ws, bool streaming, hipStream_t st, float* part)
{
    using namespace b16path;
    const TilePlan t = plan_tiles(p, LDS_LIMIT / 2, 64, 64);
    uint32_t* image = (uint32_t*)image_ws;
    hipLaunchKernelGGL(prep_bwd_weights_kernel, dim3(S, (unsigned)p.heads, 2), dim3(256), 0, st,
                       wk, wv, bias, image, (uint32_t*)dkdv_image_ws, p.two_branch ? 1.0f : 0.0f, part ? 1 : 0);
    if (part) {
        // half heads of 64-channel heads: the shares of logits and da first, then the whole kernel
        hipError_t e0 = hipGetLastError();
        if (e0 != hipSuccess || !streaming) return e0 != hipSuccess ? e0 : hipErrorInvalidValue;
        e0 = launch_bwd_pixel_ring(p, dout, q, k, v, dq, attn_ws, dl_ws, image, st, 1, part);
        if (e0 != hipSuccess) return e0;
        return launch_bwd_pixel_ring(p, dout, q, k, v, dq, attn_ws, dl_ws, image, st, 2, part);
    }
    if (streaming) {
        hipError_t e0 = hipGetLastError();
        if (e0 != hipSuccess) return e0;
        return launch_bwd_pixel_ring(p, dout, q, k, v, dq, attn_ws, dl_ws, image, st, 0, nullptr);
    }
    PixelArgs a;
    a.dout = (const bf16_bits*)dout; a.q = (const bf16_bits*)q;
    a.k = (const bf16_bits*)k; a.v = (const bf16_bits*)v;
    a.dq = (bf16_bits*)dq; a.attn = attn_ws; a.dl = dl_ws; a.image = image;
    fill_grid(a.g, p, t, k, v);
    a.scale = p.logit_scale();
    a.scale_log2e = 1.44269504088896341f * p.logit_scale();
    static LdsOptIn opt_in;
    hipError_t e = opt_in.ensure({(const void*)bwd_pixel_kernel16<false>, (const void*)bwd_pixel_kernel16<true>}, LDS_LIMIT);
    if (e != hipSuccess) return e;
    const unsigned grid = (unsigned)((long)t.TA + t.TB);
    if (half_ws) hipLaunchKernelGGL(bwd_pixel_kernel16<true>, dim3(grid), dim3(THREADS), (size_t)t.buf_bytes, st, a);
    else         hipLaunchKernelGGL(bwd_pixel_kernel16<false>, dim3(grid), dim3(THREADS), (size_t)t.buf_bytes, st, a);
    return hipGetLastError();
}

bool bwd_dkdv_mfma_supported(const Problem& p)
{
    if (p.dtype != 1 || p.ksize != 3 || p.C != p.heads * t16::D) return false;
    const long planes = (long)p.B * p.heads * ((p.W + 63) / 64);
    return planes * p.H < (1L << 30);
}

size_t bwd_dkdv_mfma_image_bytes(const Problem& p)
{
    return (size_t)p.heads * b16path::IMG_DWORDS * sizeof(uint32_t);
}

hipError_t launch_bwd_dkdv_mfma(const Problem& p, const void* dout, const void* q,
                                const float* wk, const float* wv,
                                const void* attn_ws, const void* dl_ws, bool half_ws,
                                void* dk, void* dv, void* image_ws, hipStream_t st)
{
    using namespace b16path;
    const TilePlan t = plan_dkdv(p);
    (void)wk; (void)wv;                         // the operand image was written by launch_bwd_pixel_mfma
    uint32_t* image = (uint32_t*)image_ws;
    DkdvArgs a;
    a.q = (const bf16_bits*)q; a.dout = (const bf16_bits*)dout;
    a.attn = attn_ws; a.dl = dl_ws;
    a.dk = (bf16_bits*)dk; a.dv = (bf16_bits*)dv;
    a.image = image;
    fill_grid(a.g, p, t, q, dout);
    a.rec_dl = t.buf_bytes;
    a.rec_a = t.buf_bytes + t.halo_px * REC_BYTES;
    a.scale = p.logit_scale();
    const int lds_bytes = t.buf_bytes + 2 * t.halo_px * REC_BYTES;
    static LdsOptIn opt_in;
    hipError_t e = opt_in.ensure({(const void*)bwd_dkdv_kernel16<false>, (const void*)bwd_dkdv_kernel16<true>}, LDS_LIMIT);
    if (e != hipSuccess) return e;
    const unsigned grid = (unsigned)((long)t.TA + t.TB);
    if (half_ws) hipLaunchKernelGGL(bwd_dkdv_kernel16<true>, dim3(grid), dim3(THREADS), (size_t)lds_bytes, st, a);
    else         hipLaunchKernelGGL(bwd_dkdv_kernel16<false>, dim3(grid), dim3(THREADS), (size_t)lds_bytes, st, a);
    return hipGetLastError();
}

}  // namespace slide
