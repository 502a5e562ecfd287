// Matrix-core forward of Slide Attention for gfx950: bf16 activations, head size 32,
// 3x3 window.  One fused kernel: K/V halo tiles staged in LDS, merged depthwise
// kernels applied on the fly, softmax over the 9 shifts, weighted sum of the
// shifted values.  Nothing of size k*k*C ever reaches HBM.
//
// How the arithmetic is arranged (exactly the operator of Sec. 4.1-4.3, re-associated):
//   merged kernel = one-hot shift + learned part (Sec. 4.3, Fig. 4), so
//     logit[s] = scale * ( sum_c q[c] k[c, p+s]                       <- shift path, fp32
//                        + sum_{c,t} (q[c] k[c, p+t]) wl_k[c,s,t] )    <- learned path, MFMA
//     out[c]   = sum_t v[c, p+t] * ( a[t] + sum_s a[s] wl_v[c,s,t] )   <- a[t]: shift path (fp32),
//                                                                        sum_s: learned path, MFMA
//   The learned paths are the only dense contractions (288 x 9 per pixel and head); they
//   run on the matrix cores with 16-bit operands and fp32 accumulation.  The shift paths
//   stay in fp32 so that 1 + w is never rounded to 16 bits.
//
// Number format inside the kernel: the bf16 inputs are converted to IEEE half precision
// while they are staged (k, v) or loaded (q).  A bf16 value has 8 significant bits, a half
// has 11, so the conversion is exact for 2^-17 <= |x| <= 65504; smaller values are
// truncated to a multiple of 2^-24, larger ones saturate at +-65504.  Half precision is what lets the
// vector ALU form two q*k products per instruction (v_pk_mul_f16), accumulate the exact
// dot product with v_dot2c_f32_f16, and feed v halves straight into fp32 FMAs
// (v_fma_mix_f32) with no unpacking.  The q*k products that enter the matrix core are
// formed from q/16 and the learned K kernel is stored times 16, so products up to 2^20
// stay finite.
//
// Lane mapping: a wavefront handles 16 pixels at a time; lane = pixel p (0..15) +
// 16 * channel group g (0..3), group g owning channels 8g..8g+7 of the head.  This is
// the B-operand layout of v_mfma_f32_16x16x32_f16 with the channel as K index, and the
// D layout of v_mfma_f32_16x16x16_f16 with the pixel as column, so no data moves
// between lanes except two small cross-group reductions (v_permlane{16,32}_swap).
#include "slide_tile16.h"

namespace slide {
namespace f16path {
using namespace t16;

constexpr int A_STRIDE = 12;                       // floats per pixel in the attention scratch
constexpr float G_SCALE = 0.0625f;                 // q is divided by 16 for the MFMA products ...
constexpr float WK_SCALE = 16.0f;                  // ... and the learned K kernel multiplied by 16

// Per-head image of the MFMA weight operands, written by prep_weights_kernel (dwords):
//   [0, 2304)      A1: tap t (9) x lane (64) x 4 dwords       -- learned K kernel (times 16)
//   [2304, 4608)   A2: product u (18) x lane (64) x 2 dwords  -- learned V kernel
//   [4608, 4624)   bias row r (16) as float, times log2(e); -inf on unused rows
constexpr int IMG_A1 = 0, IMG_A2 = 2304, IMG_BIAS = 4608, IMG_DWORDS = 4624;

// ------------------------------------------------------------------ weight preparation
// grid = (9, heads), block = 256.  Reads the merged float32 kernels [C, 9, 3, 3] and
// writes the per-head operand image described above (learned part = merged - one-hot).
__global__ void __launch_bounds__(256)
prep_weights_kernel(const float* __restrict__ wk, const float* __restrict__ wv,
                    const float* __restrict__ bias, uint32_t* __restrict__ image)
{
    const int t = blockIdx.x, m = blockIdx.y;
    uint32_t* img = image + (long)m * IMG_DWORDS;
    const int tid = threadIdx.x;
    {
        // A1, tap t: dword y of lane (i, g) = learned K weights of channels 8g+2y, 8g+2y+1
        // for the shift of logit row i.
        const int y = tid & 3, lane = tid >> 2;
        const int i = lane & 15, g = lane >> 4;
        const int s = shift_of_row(i);
        float d0 = 0.0f, d1 = 0.0f;
        if (s >= 0) {
            const float id = (s == t) ? 1.0f : 0.0f;
            const int c = m * D + 8 * g + 2 * y;
            d0 = (wk[((long)c * S + s) * S + t] - id) * WK_SCALE;
            d1 = (wk[((long)(c + 1) * S + s) * S + t] - id) * WK_SCALE;
        }
        img[IMG_A1 + t * 256 + tid] = pack_half(d0, d1);
    }
    {
        // A2, products u = 2t and 2t+1.  Product u < 16: channel slot e = u & 7, tap quad
        // tq = u >> 3; row i of the product is channel 8*(i/4) + e at tap 4*tq + (i%4).
        // Products 16, 17 (j = u - 16): row i is channel 8*(i/4) + 4j + (i%4) at tap 8.
        // Dword y of lane (i, g) holds the learned V weights for the shifts of logit rows
        // 4g+2y and 4g+2y+1.
        const int y = tid & 1, lane = (tid >> 1) & 63, u = 2 * t + (tid >> 7);
        const int i = lane & 15, g = lane >> 4;
        int c, tap;
        if (u < 16) { c = 8 * (i >> 2) + (u & 7); tap = 4 * (u >> 3) + (i & 3); }
        else        { c = 8 * (i >> 2) + 4 * (u - 16) + (i & 3); tap = 8; }
        c += m * D;
        float d[2] = {0.0f, 0.0f};
        for (int h = 0; h < 2; ++h) {
            const int s = shift_of_row(4 * g + 2 * y + h);
            if (s >= 0) d[h] = wv[((long)c * S + s) * S + tap] - (s == tap ? 1.0f : 0.0f);
        }
        img[IMG_A2 + u * 128 + (tid & 127)] = pack_half(d[0], d[1]);
    }
    if (t == 0 && tid < 16) {
        const int s = shift_of_row(tid);
        float b = -INFINITY;
        if (s >= 0) b = bias ? bias[m * S + s] * 1.44269504088896341f : 0.0f;
        img[IMG_BIAS + tid] = __float_as_uint(b);
    }
}

struct FwdArgs {
    const bf16_bits* q; const bf16_bits* k; const bf16_bits* v; bf16_bits* out;
    const uint32_t* image;   // per-head MFMA operand images
    TileGrid g;
    int buf_stride;          // bytes between the two tile buffers
    int a_base;              // byte offset of the attention scratch
    float scale_log2e;
};

// ------------------------------------------------------------------ the fused forward
// Persistent blocks, one per compute unit.  Block b works through tiles b, b + grid, ... of
// the ordered tile list (big tiles first, so the static deal is balanced); while it
// computes one tile out of one LDS buffer, the global loads of the next tile are in flight
// (into registers) and are converted into the other buffer after the first pass, so memory
// traffic and arithmetic overlap.
template <int WAVES, bool PERSIST>
__global__ void __launch_bounds__(WAVES * 64, 2)
fwd16_kernel(const FwdArgs a)
{
    constexpr int THREADS = WAVES * 64;
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int p = lane & 15, g = lane >> 4;
    const int n_tiles = a.g.TA + a.g.TB;
    const int HC = a.g.tw + 2;
    const uint32_t hw2 = (uint32_t)a.g.H * (uint32_t)a.g.W * 2u;

    int cur = blockIdx.x;                               // gridDim.x <= n_tiles
    Tile tcur = decode_tile(a.g, cur);
    // first tile: issue the loads of up to three items per thread before converting any,
    // so that many requests are in flight
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

    half8_t A1[S];
    half4_t A2[2 * S];
    float bias2[3];
    int m_loaded = -1;
    float* ascr = (float*)(smem + a.a_base) + wave * 16 * A_STRIDE + p * A_STRIDE;
    __syncthreads();

    for (int it = 0;; ++it) {
        unsigned char* buf = smem + (it & 1) * a.buf_stride;
        unsigned char* buf_next = smem + ((it + 1) & 1) * a.buf_stride;
        const int nxt = cur + (int)gridDim.x;
        const bool has_next = PERSIST && nxt < n_tiles;
        Tile tnext = tcur;
        uint4_t pre[8];
        if (has_next) {
            tnext = decode_tile(a.g, nxt);
            if (tid < tnext.n_items) item_load(a.g, tnext, a.k, a.v, tid, pre);
        }
        // ---- MFMA weight operands of this head (coalesced reads of the prepared image)
        if (tcur.m != m_loaded) {
            const uint32_t* img = a.image + (long)tcur.m * IMG_DWORDS;
#pragma unroll
            for (int t = 0; t < S; ++t) {
                uint4_t w = *(const uint4_t*)(img + IMG_A1 + (t * 64 + lane) * 4);
                A1[t] = __builtin_bit_cast(half8_t, w);
            }
#pragma unroll
            for (int u = 0; u < 2 * S; ++u) {
                uint2_t w2 = *(const uint2_t*)(img + IMG_A2 + (u * 64 + lane) * 2);
                A2[u] = __builtin_bit_cast(half4_t, w2);
            }
#pragma unroll
            for (int r = 0; r < 3; ++r) bias2[r] = __uint_as_float(img[IMG_BIAS + 4 * g + r]);
            m_loaded = tcur.m;
        }
        bool staged = !has_next;
        auto stage_next = [&]() {
            if (tid < tnext.n_items) item_store(a.g, tnext, tid, pre, buf_next);
            uint4_t r[8];
            // items beyond one per thread go to the last waves first: they have the fewest passes
            for (int idx = THREADS + ((tid + 64) & (THREADS - 1)); idx < tnext.n_items; idx += THREADS) {
                item_load(a.g, tnext, a.k, a.v, idx, r);
                item_store(a.g, tnext, idx, r, buf_next);
            }
            zero_pad_columns(a.g, tnext, buf_next, tid, THREADS);
        };

        // ---- passes of 16 pixels over the current tile
        const int npix = tcur.rows * tcur.cols;
        const int npass = (npix + 15) >> 4;
        const float inv_tw = 1.0f / (float)tcur.cols;
        const unsigned char* kl = buf;
        const unsigned char* vl = buf + a.g.v_off;
        // q and out addressing: one block-uniform base (scalar registers) plus a 32-bit byte
        // offset per lane; a head spans 32 * H * W * 2 bytes, far below 4 GB
        const char* qb = (const char*)(a.q + tcur.head_base);
        char* ob = (char*)(a.out + tcur.head_base);
        const uint32_t lane_chan = (uint32_t)(8 * g) * hw2 + ((uint32_t)tcur.i0 * a.g.W + tcur.j0) * 2u;

        // (tile row, tile column) of this lane's pixel in a pass; lanes past the end repeat
        // the last pixel (they compute but do not store)
        auto pixel_of = [&](int pass, int& ti, int& tj) -> bool {
            int n = pass * 16 + p;
            const bool valid = n < npix;
            n = valid ? n : npix - 1;
            ti = (int)(((float)n + 0.5f) * inv_tw);
            tj = n - ti * tcur.cols;
            return valid;
        };

        uint32_t qraw[8];                               // q of the current pass, one channel per dword
        {
            int ti0, tj0;
            pixel_of(min(wave, npass - 1), ti0, tj0);
            const uint32_t off = lane_chan + ((uint32_t)ti0 * a.g.W + tj0) * 2u;
#pragma unroll
            for (int e = 0; e < 8; ++e) qraw[e] = *(const bf16_bits*)(qb + (off + (uint32_t)e * hw2));
        }
        for (int pass = wave; pass < npass; pass += WAVES) {
            int ti, tj;
            const bool valid = pixel_of(pass, ti, tj);
            const uint32_t pix_off = lane_chan + ((uint32_t)ti * a.g.W + tj) * 2u;
            int coff[KS];
#pragma unroll
            for (int tx = 0; tx < KS; ++tx) coff[tx] = col_offset(tj + tx, g);
            const int row0 = ti * HC * 64;
            uint4_t kd[S];
#pragma unroll
            for (int t = 0; t < S; ++t)
                kd[t] = *(const uint4_t*)(kl + row0 + (t / KS) * HC * 64 + coff[t % KS]);

            half2_t qpk[4], qs[4];  // channel pairs as halves; qs = q / 16
#pragma unroll
            for (int y = 0; y < 4; ++y) {
                const uint32_t pk = pack_half_rtz(__uint_as_float(qraw[2 * y] << 16),
                                                  __uint_as_float(qraw[2 * y + 1] << 16));
                qpk[y] = as_half2(pk);
                qs[y] = qpk[y] * half2_t{(_Float16)G_SCALE, (_Float16)G_SCALE};
            }

            // ---- K side: logits
            float4_t acc1 = {0.0f, 0.0f, 0.0f, 0.0f};
            float idp[S];
#pragma unroll
            for (int t = 0; t < S; ++t) {
                float R = 0.0f;
                uint4_t bb;
#pragma unroll
                for (int y = 0; y < 4; ++y) {
                    const half2_t kw = as_half2(kd[t][y]);
                    R = __builtin_amdgcn_fdot2(qpk[y], kw, R, false);
                    bb[y] = as_dword(qs[y] * kw);
                }
                acc1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(A1[t], __builtin_bit_cast(half8_t, bb),
                                                              acc1, 0, 0, 0);
                idp[t] = R;
            }
            // q of this wave's next pass: issued once the K taps are consumed, used at the end of this pass
            uint32_t qnext[8];
            {
                int ti2, tj2;
                pixel_of(min(pass + WAVES, npass - 1), ti2, tj2);
                const uint32_t off = lane_chan + ((uint32_t)ti2 * a.g.W + tj2) * 2u;
#pragma unroll
                for (int e = 0; e < 8; ++e) qnext[e] = *(const bf16_bits*)(qb + (off + (uint32_t)e * hw2));
            }
            // V taps 0..3: issue the LDS reads now, they land while the softmax runs
            uint4_t vd[S];
#pragma unroll
            for (int t = 0; t < 4; ++t)
                vd[t] = *(const uint4_t*)(vl + row0 + (t / KS) * HC * 64 + coff[t % KS]);

            // shift-path logits: sum the four channel groups, landing shift 4r+g in group g
            {
                float z1 = fold32(idp[0], idp[2]), z2 = fold32(idp[1], idp[3]);
                acc1[0] += fold16(z1, z2);
                z1 = fold32(idp[4], idp[6]); z2 = fold32(idp[5], idp[7]);
                acc1[1] += fold16(z1, z2);
                z1 = fold32(idp[8], 0.0f);
                acc1[2] += fold16(z1, 0.0f);
            }
            // ---- softmax over the 9 shifts (3 per lane, 4 lane groups)
            float l[3];
#pragma unroll
            for (int r = 0; r < 3; ++r) l[r] = fmaf(acc1[r], a.scale_log2e, bias2[r]);
            const float mx = allmax_groups(fmaxf(fmaxf(l[0], l[1]), l[2]));
            float pr[3];
#pragma unroll
            for (int r = 0; r < 3; ++r) pr[r] = __builtin_amdgcn_exp2f(l[r] - mx);
            const float inv = __builtin_amdgcn_rcpf(allsum_groups(pr[0] + pr[1] + pr[2]));
#pragma unroll
            for (int r = 0; r < 3; ++r) pr[r] *= inv;
            // attention weights of this pixel to the wave's scratch so every group can read all 9
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int r = 0; r < 3; ++r) ascr[4 * r + g] = pr[r];      // slots 9..11 are never read
            __builtin_amdgcn_wave_barrier();
            const float4_t at0 = *(const float4_t*)(ascr), at1 = *(const float4_t*)(ascr + 4);
            const float at8 = ascr[8];
            uint2_t b2;
            b2[0] = pack_half(pr[0], pr[1]);
            b2[1] = pack_half(pr[2], 0.0f);
            const half4_t B2 = __builtin_bit_cast(half4_t, b2);

            // ---- V side: out[c] = sum_t v[c, p+t] * (a[t] + learned part); a[t] enters as the
            // MFMA's C operand, so the matrix core adds the two paths.  Product (e, tq) gives,
            // in its four result registers, the weights of channel e for taps 4tq..4tq+3.
            float o[8];
#pragma unroll
            for (int t = 4; t < S; ++t)
                vd[t] = *(const uint4_t*)(vl + row0 + (t / KS) * HC * 64 + coff[t % KS]);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float4_t w0 = __builtin_amdgcn_mfma_f32_16x16x16f16(A2[e], B2, at0, 0, 0, 0);
                float acc = 0.0f;
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    acc = fmaf(w0[r], (float)as_half2(vd[r][e >> 1])[e & 1], acc);
                o[e] = acc;
                if ((e & 3) == 3) {
                    // pin the sums so the multiply-adds are not deferred past later MFMAs
                    // (that would keep every MFMA result live at once)
                    asm volatile("" : "+v"(o[e - 3]), "+v"(o[e - 2]), "+v"(o[e - 1]), "+v"(o[e]));
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float4_t w1 = __builtin_amdgcn_mfma_f32_16x16x16f16(A2[8 + e], B2, at1, 0, 0, 0);
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    o[e] = fmaf(w1[r], (float)as_half2(vd[4 + r][e >> 1])[e & 1], o[e]);
                if ((e & 3) == 3) {
                    asm volatile("" : "+v"(o[e - 3]), "+v"(o[e - 2]), "+v"(o[e - 1]), "+v"(o[e]));
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            {
                const float4_t c8 = {at8, at8, at8, at8};
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    const float4_t w8 = __builtin_amdgcn_mfma_f32_16x16x16f16(A2[16 + j], B2, c8, 0, 0, 0);
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int e = 4 * j + r;
                        o[e] = fmaf(w8[r], (float)as_half2(vd[8][e >> 1])[e & 1], o[e]);
                    }
                }
            }
            // ---- store
            if (valid) {
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    *(bf16_bits*)(ob + (pix_off + (uint32_t)e * hw2)) = f32_to_bf16(o[e]);
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) qraw[e] = qnext[e];
            if (!staged) { stage_next(); staged = true; }
        }
        if (!staged) stage_next();
        __syncthreads();
        if (!has_next) break;
        cur = nxt;
        tcur = tnext;
    }
}

// ------------------------------------------------------------------ host side
constexpr int FWD_WAVES = 4;
constexpr bool PERSISTENT = false;   // false: one tile per block, two blocks per compute unit
constexpr int SCRATCH_BYTES = FWD_WAVES * 16 * A_STRIDE * 4;

static TilePlan plan_fwd(const Problem& p)
{
    const int budget = PERSISTENT ? (LDS_LIMIT - SCRATCH_BYTES) / 2 : LDS_LIMIT / 2 - SCRATCH_BYTES;
    return plan_tiles(p, budget, 64, 64);
}

}  // namespace f16path

bool fwd_mfma_supported(const Problem& p)
{
    if (p.dtype != 1 || p.ksize != 3 || p.C != p.heads * f16path::D) return false;
    const long planes = (long)p.B * p.heads * ((p.W + 63) / 64);
    return planes * p.H < (1L << 30);                    // tile count fits an int
}

// per head: the MFMA operand image
size_t fwd_mfma_workspace_bytes(const Problem& p)
{
    return fwd_mfma_supported(p) ? (size_t)p.heads * f16path::IMG_DWORDS * sizeof(uint32_t) : 0;
}

hipError_t launch_fwd_mfma(const Problem& p, const void* q, const void* k, const void* v,
                           const float* wk, const float* wv, const float* bias, void* out,
                           void* workspace, hipStream_t st)
{
    using namespace f16path;
    const TilePlan t = plan_fwd(p);
    uint32_t* image = (uint32_t*)workspace;
    hipLaunchKernelGGL(prep_weights_kernel, dim3(S, (unsigned)p.heads), dim3(256), 0, st,
                       wk, wv, bias, image);
    FwdArgs a;
    a.q = (const bf16_bits*)q; a.k = (const bf16_bits*)k; a.v = (const bf16_bits*)v;
    a.out = (bf16_bits*)out; a.image = image;
    fill_grid(a.g, p, t, k, v);
    a.buf_stride = t.buf_bytes;
    a.a_base = (PERSISTENT ? 2 : 1) * t.buf_bytes;
    a.scale_log2e = 1.44269504088896341f / sqrtf((float)D);
    const int lds_bytes = a.a_base + SCRATCH_BYTES;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void*)fwd16_kernel<FWD_WAVES, PERSISTENT>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, LDS_LIMIT);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const long n_tiles = (long)t.TA + t.TB;
    const unsigned grid = (unsigned)((PERSISTENT && n_tiles > NUM_CU) ? NUM_CU : n_tiles);
    hipLaunchKernelGGL((fwd16_kernel<FWD_WAVES, PERSISTENT>), dim3(grid), dim3(FWD_WAVES * 64),
                       (size_t)lds_bytes, st, a);
    return hipGetLastError();
}

}  // namespace slide
