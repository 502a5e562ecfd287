// Matrix-core forward of Slide Attention for gfx950, 5x5 window: bf16 activations, head
// size 32, 25 shifts and 25 taps.
//
// Same arithmetic arrangement as the 3x3 kernel (Sec. 4.1-4.3 re-associated), with the
// merged kernels W~ = one-hot shift + learned part as half-precision matrix operands:
//     logit[s] = scale * sum_{c,t} (q[c] k[c, p+t]) W~k[c,s,t]
//     out[c]   = sum_t v[c, p+t] * g[c,t],   g[c,t] = sum_s a[s] W~v[c,s,t]
// both contractions (800 x 25 per pixel and head, each side) on v_mfma_f32_16x16x32_f16.
// What differs from 3x3: the kernels of one head are
// 2 x 50 KB of MFMA operands, far too many for registers, so a block keeps them in LDS next
// to the K/V halo tile and reads them as it goes; blocks are persistent and walk the tile
// list, reloading the operands only when the head changes.  The 25 logits of a pixel live
// in two 16-row MFMA tiles; lane group g owns rows 4g..4g+3 of both, i.e. 7 logits.
#include "slide_tile16.h"

namespace slide {
namespace f16k5 {
using namespace t16;

constexpr int K5 = 5, S5 = 25;
constexpr int WAVES = 8, THREADS = WAVES * 64;
constexpr float G_SCALE = 0.0625f, WK_SCALE = 16.0f;

// Per-head operand image (dwords): A1: (tap t (25) x tile (2)) x lane (64) x 4; A2: product u
// (50) x lane (64) x 4; bias: 32 floats (times log2 e, -inf on unused rows).
constexpr int IMG_A1 = 0, IMG_A2 = 50 * 256, IMG_BIAS = 100 * 256, IMG_DWORDS = 100 * 256 + 32;
constexpr int IMG_BYTES = IMG_DWORDS * 4;           // 102528

// row (0..31) of the two logit tiles <-> shift.  Tile A: row 4g+r is shift 4r+g; tile B
// (rows 16..31): row 16+4g+r is shift 16+4r+g for r = 0,1 and shift 24 for r = 2, g = 0.
__host__ __device__ constexpr int shift_of_row5(int row)
{
    const int tile = row >> 4, g = (row >> 2) & 3, r = row & 3;
    if (tile == 0) return 4 * r + g;
    if (r < 2) return 16 + 4 * r + g;
    return (r == 2 && g == 0) ? 24 : -1;
}
// K slot (0..31) of the V-side product <-> shift: lane group g holds slots 8g..8g+7 = its own
// rows 4g..4g+3 of tile A followed by its rows of tile B
__host__ __device__ constexpr int shift_of_slot5(int slot)
{
    const int g = slot >> 3, j = slot & 7;
    return j < 4 ? shift_of_row5(4 * g + j) : shift_of_row5(16 + 4 * g + (j - 4));
}

// grid = (25, heads), block = 256
__global__ void __launch_bounds__(256)
prep_weights5_kernel(const float* __restrict__ wk, const float* __restrict__ wv,
                     const float* __restrict__ bias, uint32_t* __restrict__ image, float idw)
{   // idw = 1: wk, wv are the learned kernels of the two-branch form, the fixed shift path
    // (weight 1 where shift and tap coincide) is added here; 0: merged kernels
    const int t = blockIdx.x, m = blockIdx.y;
    uint32_t* img = image + (long)m * IMG_DWORDS;
    const int tid = threadIdx.x;
    // A1, tap t, both tiles: dword y of lane (i, g) = merged K weights (times 16) of channels
    // 8g+2y, 8g+2y+1 for the shift of row i of the tile
    for (int tile = 0; tile < 2; ++tile) {
        const int y = tid & 3, lane = tid >> 2;
        const int i = lane & 15, g = lane >> 4;
        const int s = shift_of_row5(16 * tile + i);
        float d0 = 0.0f, d1 = 0.0f;
        if (s >= 0) {
            const int c = m * D + 8 * g + 2 * y;
            const float id = (s == t) ? idw : 0.0f;
            d0 = (wk[((long)c * S5 + s) * S5 + t] + id) * WK_SCALE;
            d1 = (wk[((long)(c + 1) * S5 + s) * S5 + t] + id) * WK_SCALE;
        }
        img[IMG_A1 + (t * 2 + tile) * 256 + tid] = pack_half(d0, d1);
    }
    // A2, products u = 2t and 2t+1.  u < 48: channel slot e = u % 8, tap quad tq = u / 8; row i
    // is channel 8*(i/4) + e at tap 4*tq + (i%4).  u = 48 + j: row i is channel
    // 8*(i/4) + 4j + (i%4) at tap 24.  Dword y of lane (i, g) holds the merged V weights for
    // the shifts of slots 8g+2y, 8g+2y+1.
    for (int uu = 0; uu < 2; ++uu) {
        const int u = 2 * t + uu;
        const int y = tid & 3, lane = tid >> 2;
        const int i = lane & 15, g = lane >> 4;
        int c, tap;
        if (u < 48) { c = 8 * (i >> 2) + (u & 7); tap = 4 * (u >> 3) + (i & 3); }
        else        { c = 8 * (i >> 2) + 4 * (u - 48) + (i & 3); tap = 24; }
        c += m * D;
        float d[2] = {0.0f, 0.0f};
        for (int h = 0; h < 2; ++h) {
            const int s = shift_of_slot5(8 * g + 2 * y + h);
            if (s >= 0) d[h] = wv[((long)c * S5 + s) * S5 + tap] + ((s == tap) ? idw : 0.0f);
        }
        img[IMG_A2 + u * 256 + tid] = pack_half(d[0], d[1]);
    }
    if (t == 0 && tid < 32) {
        const int s = shift_of_row5(tid);
        float b = -INFINITY;
        if (s >= 0) b = bias ? bias[m * S5 + s] * 1.44269504088896341f : 0.0f;
        img[IMG_BIAS + tid] = __float_as_uint(b);
    }
}

struct Fwd5Args {
    const bf16_bits* q; const bf16_bits* k; const bf16_bits* v; bf16_bits* out;
    float* lse;              // [B, heads, H, W] log of the softmax denominator, or null
    const uint32_t* image;
    TileGrid g;
    int w_base;              // byte offset of the operand image in LDS
    float scale_log2e;
};

__global__ void __launch_bounds__(THREADS, 2)
fwd16_k5_kernel(const Fwd5Args a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int p = lane & 15, g = lane >> 4;
    const int HC = a.g.tw + 4;
    const uint32_t hw2 = (uint32_t)a.g.H * (uint32_t)a.g.W * 2u;
    const int n_tiles = a.g.TA + a.g.TB;
    const unsigned char* wl = smem + a.w_base;
    int m_loaded = -1;

    for (int cur = blockIdx.x; cur < n_tiles; cur += gridDim.x) {
        const Tile tcur = decode_tile(a.g, cur);
        const int npix = tcur.rows * tcur.cols;
        const int npass = (npix + 15) >> 4;
        const float inv_tw = 1.0f / (float)tcur.cols;
        const char* qb = (const char*)(a.q + tcur.head_base);
        char* ob = (char*)(a.out + tcur.head_base);
        const uint32_t lane_chan = (uint32_t)(8 * g) * hw2 + ((uint32_t)tcur.i0 * a.g.W + tcur.j0) * 2u;
        auto pixel_of = [&](int pass, int& ti, int& tj) -> bool {
            int n = pass * 16 + p;
            const bool valid = n < npix;
            n = valid ? n : npix - 1;
            ti = (int)(((float)n + 0.5f) * inv_tw);
            tj = n - ti * tcur.cols;
            return valid;
        };
        // q of this wave's first pass: in flight while the tile is staged
        uint32_t qraw[8];
        {
            int ti0, tj0;
            pixel_of(min(wave, npass - 1), ti0, tj0);
            const uint32_t off = lane_chan + ((uint32_t)ti0 * a.g.W + tj0) * 2u;
#pragma unroll
            for (int e = 0; e < 8; ++e) qraw[e] = *(const bf16_bits*)(qb + (off + (uint32_t)e * hw2));
        }

        __syncthreads();                                   // the previous tile is no longer read
        if (tcur.m != m_loaded) {                          // operands of a new head: global -> LDS
            const uint4_t* src = (const uint4_t*)(a.image + (long)tcur.m * IMG_DWORDS);
            for (int idx = tid; idx < IMG_BYTES / 16; idx += THREADS)
                *(uint4_t*)(smem + a.w_base + idx * 16) = src[idx];
            m_loaded = tcur.m;
        }
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

        const unsigned char* kl = smem;
        const unsigned char* vl = smem + a.g.v_off;
        float biasA[4], biasB[3];
#pragma unroll
        for (int r = 0; r < 4; ++r) biasA[r] = *(const float*)(wl + (IMG_BIAS + 4 * g + r) * 4);
#pragma unroll
        for (int r = 0; r < 3; ++r) biasB[r] = *(const float*)(wl + (IMG_BIAS + 16 + 4 * g + r) * 4);

        for (int pass = wave; pass < npass; pass += WAVES) {
            int ti, tj;
            const bool valid = pixel_of(pass, ti, tj);
            const uint32_t pix_off = lane_chan + ((uint32_t)ti * a.g.W + tj) * 2u;
            int coff[K5];
#pragma unroll
            for (int tx = 0; tx < K5; ++tx) coff[tx] = col_offset(tj + tx, g);
            const int row0 = ti * HC * 64;

            half2_t qs[4];
#pragma unroll
            for (int y = 0; y < 4; ++y)
                qs[y] = as_half2(pack_half_rtz(__uint_as_float(qraw[2 * y] << 16),
                                               __uint_as_float(qraw[2 * y + 1] << 16))) *
                        half2_t{(_Float16)G_SCALE, (_Float16)G_SCALE};
            // q of this wave's next pass in this tile
            if (pass + WAVES < npass) {
                int ti2, tj2;
                pixel_of(pass + WAVES, ti2, tj2);
                const uint32_t off = lane_chan + ((uint32_t)ti2 * a.g.W + tj2) * 2u;
#pragma unroll
                for (int e = 0; e < 8; ++e) qraw[e] = *(const bf16_bits*)(qb + (off + (uint32_t)e * hw2));
            }

            // ---- K side: 25 logits in two MFMA tiles
            float4_t accA = {0.0f, 0.0f, 0.0f, 0.0f}, accB = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
            for (int t = 0; t < S5; ++t) {
                const uint4_t kd = *(const uint4_t*)(kl + row0 + (t / K5) * HC * 64 + coff[t % K5]);
                const half8_t A1a = __builtin_bit_cast(half8_t, *(const uint4_t*)(wl + ((IMG_A1 + (t * 2) * 256) + lane * 4) * 4));
                const half8_t A1b = __builtin_bit_cast(half8_t, *(const uint4_t*)(wl + ((IMG_A1 + (t * 2 + 1) * 256) + lane * 4) * 4));
                uint4_t bb;
#pragma unroll
                for (int y = 0; y < 4; ++y) bb[y] = as_dword(qs[y] * as_half2(kd[y]));
                const half8_t G = __builtin_bit_cast(half8_t, bb);
                accA = __builtin_amdgcn_mfma_f32_16x16x32_f16(A1a, G, accA, 0, 0, 0);
                accB = __builtin_amdgcn_mfma_f32_16x16x32_f16(A1b, G, accB, 0, 0, 0);
                if (t % K5 == K5 - 1) __builtin_amdgcn_sched_barrier(0);     // one window row at a time
            }
            // ---- softmax over the 25 shifts (7 per lane, 4 lane groups)
            float l[7], pr[7];
#pragma unroll
            for (int r = 0; r < 4; ++r) l[r] = fmaf(accA[r], a.scale_log2e, biasA[r]);
#pragma unroll
            for (int r = 0; r < 3; ++r) l[4 + r] = fmaf(accB[r], a.scale_log2e, biasB[r]);
            float mx = l[0];
#pragma unroll
            for (int r = 1; r < 7; ++r) mx = fmaxf(mx, l[r]);
            mx = allmax_groups(mx);
            float sum = 0.0f;
#pragma unroll
            for (int r = 0; r < 7; ++r) { pr[r] = __builtin_amdgcn_exp2f(l[r] - mx); sum += pr[r]; }
            const float den = allsum_groups(sum);
            const float inv = __builtin_amdgcn_rcpf(den);
            if (a.lse && valid && g == 0)
                a.lse[tcur.head_base / D + (long)(tcur.i0 + ti) * a.g.W + tcur.j0 + tj] =
                    LN2 * (mx + __builtin_amdgcn_logf(den));
#pragma unroll
            for (int r = 0; r < 7; ++r) pr[r] *= inv;
            uint4_t b2;
            b2[0] = pack_half(pr[0], pr[1]); b2[1] = pack_half(pr[2], pr[3]);
            b2[2] = pack_half(pr[4], pr[5]); b2[3] = pack_half(pr[6], 0.0f);
            const half8_t B2 = __builtin_bit_cast(half8_t, b2);

            // ---- V side: product (e, tq) gives the weights g[c,t] of channel e for taps 4tq..4tq+3
            float o[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = 0.0f;
#pragma unroll
            for (int tq = 0; tq < 6; ++tq) {
                const float4_t c4 = {0.0f, 0.0f, 0.0f, 0.0f};
                uint4_t vd[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int t = 4 * tq + r;
                    vd[r] = *(const uint4_t*)(vl + row0 + (t / K5) * HC * 64 + coff[t % K5]);
                }
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const half8_t A2 = __builtin_bit_cast(half8_t, *(const uint4_t*)(wl + ((IMG_A2 + (tq * 8 + e) * 256) + lane * 4) * 4));
                    const float4_t w = __builtin_amdgcn_mfma_f32_16x16x32_f16(A2, B2, c4, 0, 0, 0);
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        o[e] = fmaf(w[r], (float)as_half2(vd[r][e >> 1])[e & 1], o[e]);
                }
#pragma unroll
                for (int e = 0; e < 8; e += 2) asm volatile("" : "+v"(o[e]), "+v"(o[e + 1]));
                __builtin_amdgcn_sched_barrier(0);
            }
            {
                const float4_t c24 = {0.0f, 0.0f, 0.0f, 0.0f};
                const uint4_t vd24 = *(const uint4_t*)(vl + row0 + 4 * HC * 64 + coff[4]);
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    const half8_t A2 = __builtin_bit_cast(half8_t, *(const uint4_t*)(wl + ((IMG_A2 + (48 + j) * 256) + lane * 4) * 4));
                    const float4_t w = __builtin_amdgcn_mfma_f32_16x16x32_f16(A2, B2, c24, 0, 0, 0);
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int e = 4 * j + r;
                        o[e] = fmaf(w[r], (float)as_half2(vd24[e >> 1])[e & 1], o[e]);
                    }
                }
            }
            if (valid) {
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    *(bf16_bits*)(ob + (pix_off + (uint32_t)e * hw2)) = f32_to_bf16(o[e]);
            }
        }
    }
}

constexpr int TILE_BUDGET = LDS_LIMIT - IMG_BYTES - 256;

}  // namespace f16k5

bool fwd_mfma5_supported(const Problem& p)
{
    if (p.dtype != 1 || p.ksize != 5 || p.C != p.heads * t16::D) return false;
    const long planes = (long)p.B * p.heads * ((p.W + 63) / 64);
    return planes * p.H < (1L << 30);
}

size_t fwd_mfma5_workspace_bytes(const Problem& p)
{
    return fwd_mfma5_supported(p) ? (size_t)p.heads * f16k5::IMG_BYTES : 0;
}

hipError_t launch_fwd_mfma5(const Problem& p, const void* q, const void* k, const void* v,
                            const float* wk, const float* wv, const float* bias, void* out,
                            float* lse, void* workspace, hipStream_t st)
{
    using namespace f16k5;
    const TilePlan t = plan_tiles(p, TILE_BUDGET, 64, 64, 0, WAVES);
    uint32_t* image = (uint32_t*)workspace;
    hipLaunchKernelGGL(prep_weights5_kernel, dim3(S5, (unsigned)p.heads), dim3(256), 0, st,
                       wk, wv, bias, image, p.two_branch ? 1.0f : 0.0f);
    Fwd5Args a;
    a.q = (const bf16_bits*)q; a.k = (const bf16_bits*)k; a.v = (const bf16_bits*)v;
    a.out = (bf16_bits*)out; a.lse = lse; a.image = image;
    fill_grid(a.g, p, t, k, v);
    a.w_base = t.buf_bytes;
    a.scale_log2e = 1.44269504088896341f / sqrtf((float)D);
    const int lds_bytes = t.buf_bytes + IMG_BYTES;
    static LdsOptIn opt_in;
    hipError_t e = opt_in.ensure({(const void*)fwd16_k5_kernel}, LDS_LIMIT);
    if (e != hipSuccess) return e;
    const long n_tiles = (long)t.TA + t.TB;
    const int n_cu = device_cu_count();
    const unsigned grid = (unsigned)(n_tiles > n_cu ? n_cu : n_tiles);
    hipLaunchKernelGGL(fwd16_k5_kernel, dim3(grid), dim3(THREADS), (size_t)lds_bytes, st, a);
    return hipGetLastError();
}

}  // namespace slide
