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
constexpr int WAVE_SCRATCH = 1152;                 // per wave: attention weights, or 32 channels x 16 pixels of bf16
// byte offset of channel c's 16 pixels in the wave scratch (octets 64 banks apart would collide)
__device__ __forceinline__ int chan_row(int c) { return (c + (c >> 3)) * 32; }
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
    int buf_stride;          // bytes between the two tile buffers (pipelined kernel)
    int a_base;              // byte offset of the per-wave scratch (1 KB per wave)
    float scale_log2e;
};

// The arithmetic of one pass: 16 pixels, lane = (pixel p, channel group g); (ti, tj) is the
// lane's pixel inside the tile, qraw its 8 q channels (bf16 patterns, one per dword).
// Returns the 8 output channels in o.  `ascr` is the lane's row of the wave's scratch.
__device__ __forceinline__ void slide_pass(const unsigned char* kl, const unsigned char* vl, int HC,
                                           int ti, int tj, int g, const uint32_t (&qraw)[8],
                                           const half8_t (&A1)[S], const half4_t (&A2)[2 * S],
                                           const float (&bias2)[3], float scale_log2e, float* ascr,
                                           float (&o)[8])
{
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
        acc1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(A1[t], __builtin_bit_cast(half8_t, bb), acc1, 0, 0, 0);
        idp[t] = R;
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
    for (int r = 0; r < 3; ++r) l[r] = fmaf(acc1[r], scale_log2e, bias2[r]);
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
}

// MFMA weight operands of one head (coalesced reads of the prepared image)
__device__ __forceinline__ void load_operands(const uint32_t* img, int lane, int g, half8_t (&A1)[S],
                                              half4_t (&A2)[2 * S], float (&bias2)[3])
{
#pragma unroll
    for (int t = 0; t < S; ++t)
        A1[t] = __builtin_bit_cast(half8_t, *(const uint4_t*)(img + IMG_A1 + (t * 64 + lane) * 4));
#pragma unroll
    for (int u = 0; u < 2 * S; ++u)
        A2[u] = __builtin_bit_cast(half4_t, *(const uint2_t*)(img + IMG_A2 + (u * 64 + lane) * 2));
#pragma unroll
    for (int r = 0; r < 3; ++r) bias2[r] = __uint_as_float(img[IMG_BIAS + 4 * g + r]);
}

// ------------------------------------------------------------------ forward, one tile per block
// The general form: any width and alignment.  Two blocks per compute unit.
template <int WAVES>
__global__ void __launch_bounds__(WAVES * 64, 2)
fwd16_kernel(const FwdArgs a)
{
    constexpr int THREADS = WAVES * 64;
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int p = lane & 15, g = lane >> 4;
    const int HC = a.g.tw + 2;
    const uint32_t hw2 = (uint32_t)a.g.H * (uint32_t)a.g.W * 2u;

    const Tile tcur = decode_tile(a.g, blockIdx.x);
    // issue the loads of up to three items per thread before converting any, so that many
    // requests are in flight
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
    load_operands(a.image + (long)tcur.m * IMG_DWORDS, lane, g, A1, A2, bias2);
    float* ascr = (float*)(smem + a.a_base + wave * WAVE_SCRATCH) + p * A_STRIDE;
    __syncthreads();

    const int npix = tcur.rows * tcur.cols;
    const int npass = (npix + 15) >> 4;
    const float inv_tw = 1.0f / (float)tcur.cols;
    // q and out addressing: one block-uniform base (scalar registers) plus a 32-bit byte
    // offset per lane; a head spans 32 * H * W * 2 bytes, far below 4 GB
    const char* qb = (const char*)(a.q + tcur.head_base);
    char* ob = (char*)(a.out + tcur.head_base);
    const uint32_t lane_chan = (uint32_t)(8 * g) * hw2 + ((uint32_t)tcur.i0 * a.g.W + tcur.j0) * 2u;
    // (tile row, tile column) of this lane's pixel in a pass; lanes past the end repeat the
    // last pixel (they compute but do not store)
    auto pixel_of = [&](int pass, int& ti, int& tj) -> bool {
        int n = pass * 16 + p;
        const bool valid = n < npix;
        n = valid ? n : npix - 1;
        ti = (int)(((float)n + 0.5f) * inv_tw);
        tj = n - ti * tcur.cols;
        return valid;
    };
    uint32_t qraw[8];                                   // q of the current pass, one channel per dword
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
        // q of this wave's next pass: issued now, used at the end of this pass
        uint32_t qnext[8];
        {
            int ti2, tj2;
            pixel_of(min(pass + WAVES, npass - 1), ti2, tj2);
            const uint32_t off = lane_chan + ((uint32_t)ti2 * a.g.W + tj2) * 2u;
#pragma unroll
            for (int e = 0; e < 8; ++e) qnext[e] = *(const bf16_bits*)(qb + (off + (uint32_t)e * hw2));
        }
        float o[8];
        slide_pass(smem, smem + a.g.v_off, HC, ti, tj, g, qraw, A1, A2, bias2, a.scale_log2e, ascr, o);
        if (valid) {
#pragma unroll
            for (int e = 0; e < 8; ++e)
                *(bf16_bits*)(ob + (pix_off + (uint32_t)e * hw2)) = f32_to_bf16(o[e]);
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) qraw[e] = qnext[e];
    }
}

// ------------------------------------------------------------------ forward, pipelined
// Persistent blocks of 8 waves, one per compute unit, for problems whose rows are 16-byte
// aligned (W % 8 == 0).  Block b works through tiles b, b + grid, ... of the tile list.  Two
// LDS tile buffers: while the passes of one tile run, each pass also fetches a share of the
// next tile (half an item per lane: 4 channels x 8 columns, four 16-byte loads issued at the
// start of the pass, converted into the other buffer at its end), so global loads and
// arithmetic overlap inside the block instead of alternating across the whole chip.
// q comes in and results go out as 16-byte row segments: lane (c = lane/2, h = lane%2) moves
// pixels 16*pass + 8h .. +7 of channel c, and the wave's scratch transposes between that and
// the per-lane (pixel, 8 channels) view.  Vector memory operations retire in order, so the q
// segment is fetched two passes ahead.
constexpr int PIPE_WAVES = 8;

// half item h of a tile: tensor (h & 1), channel quad (h >> 1) & 7, then (halo row, chunk)
__device__ __forceinline__ void half_item_load(const FwdArgs& a, const Tile& t, int h, uint4_t (&r)[4])
{
    const int tsel = h & 1, cq = (h >> 1) & 7, rest = h >> 4;
    const int hr = rest / t.NX, x = rest - hr * t.NX;
    const int gi = t.i0 - 1 + hr, gx = t.gxa + 8 * x;
    const long HW = (long)a.g.H * a.g.W;
    if (gi < 0 || gi >= a.g.H || gx + 8 > a.g.W) {
#pragma unroll
        for (int e = 0; e < 4; ++e) r[e] = uint4_t{0u, 0u, 0u, 0u};
        return;
    }
    const bf16_bits* src = (tsel ? a.v : a.k) + t.head_base + (long)(4 * cq) * HW + (long)gi * a.g.W + gx;
#pragma unroll
    for (int e = 0; e < 4; ++e) r[e] = *(const uint4_t*)(src + e * HW);
}
__device__ __forceinline__ void half_item_store(const FwdArgs& a, const Tile& t, int h,
                                                const uint4_t (&r)[4], unsigned char* buf)
{
    const int tsel = h & 1, cq = (h >> 1) & 7, rest = h >> 4;
    const int hr = rest / t.NX, x = rest - hr * t.NX;
    const int gx = t.gxa + 8 * x;
    const int HC = a.g.tw + 2;
    unsigned char* dst = buf + (tsel ? a.g.v_off : 0) + hr * HC * 64;
#pragma unroll
    for (int px = 0; px < 8; ++px) {
        uint2_t t2;
#pragma unroll
        for (int y = 0; y < 2; ++y) {
            const uint32_t lo = r[2 * y][px >> 1], hi = r[2 * y + 1][px >> 1];
            if (px & 1)
                t2[y] = pack_half_rtz(__uint_as_float(lo & 0xffff0000u), __uint_as_float(hi & 0xffff0000u));
            else
                t2[y] = pack_half_rtz(__uint_as_float(lo << 16), __uint_as_float(hi << 16));
        }
        const int hc = gx + px - (t.j0 - 1);
        if (hc >= 0 && hc < t.cols + 2) *(uint2_t*)(dst + col_offset(hc, cq >> 1) + (cq & 1) * 8) = t2;
    }
}

__global__ void __launch_bounds__(PIPE_WAVES * 64, 2)
fwd16_pipe_kernel(const FwdArgs a)
{
    constexpr int WAVES = PIPE_WAVES, THREADS = WAVES * 64;
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int p = lane & 15, g = lane >> 4;
    const int HC = a.g.tw + 2;
    const uint32_t hw2 = (uint32_t)a.g.H * (uint32_t)a.g.W * 2u;
    const int n_tiles = a.g.TA + a.g.TB;
    unsigned char* wbuf = smem + a.a_base + wave * WAVE_SCRATCH;
    float* ascr = (float*)wbuf + p * A_STRIDE;
    const int seg_c = lane >> 1, seg_h = lane & 1;

    int cur = blockIdx.x;                               // gridDim.x <= n_tiles
    Tile tcur = decode_tile(a.g, cur);
    // the first tile is staged without overlap
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

    for (int it = 0;; ++it) {
        unsigned char* buf = smem + (it & 1) * a.buf_stride;
        unsigned char* buf_next = smem + ((it + 1) & 1) * a.buf_stride;
        const int nxt = cur + (int)gridDim.x;
        const bool has_next = nxt < n_tiles;
        const Tile tnext = decode_tile(a.g, has_next ? nxt : cur);
        const int n_half = has_next ? 2 * tnext.n_items : 0;
        if (tcur.m != m_loaded) {
            load_operands(a.image + (long)tcur.m * IMG_DWORDS, lane, g, A1, A2, bias2);
            m_loaded = tcur.m;
        }
        const int npix = tcur.rows * tcur.cols;
        const int npass = (npix + 15) >> 4;
        const float inv_tw = 1.0f / (float)tcur.cols;
        const char* qb = (const char*)(a.q + tcur.head_base);
        char* ob = (char*)(a.out + tcur.head_base);
        auto seg_offset = [&](int pass, bool& ok) -> uint32_t {
            const int n0 = pass * 16 + 8 * seg_h;
            ok = n0 < npix;
            const int nn = ok ? n0 : 0;
            const int sti = (int)(((float)nn + 0.5f) * inv_tw);
            const int stj = nn - sti * tcur.cols;
            return (uint32_t)seg_c * hw2 + ((uint32_t)(tcur.i0 + sti) * a.g.W + tcur.j0 + stj) * 2u;
        };
        // q segments of this wave's first two passes
        uint4_t qseg = {0u, 0u, 0u, 0u}, qseg1 = {0u, 0u, 0u, 0u};
        {
            bool ok;
            uint32_t off = seg_offset(min(wave, npass - 1), ok);
            if (ok) qseg = *(const uint4_t*)(qb + off);
            off = seg_offset(min(wave + WAVES, npass - 1), ok);
            if (ok) qseg1 = *(const uint4_t*)(qb + off);
        }
        __syncthreads();                                // buf is complete, buf_next is free

        for (int pass = wave; pass < npass; pass += WAVES) {
            int n = pass * 16 + p;
            n = n < npix ? n : npix - 1;
            const int ti = (int)(((float)n + 0.5f) * inv_tw);
            const int tj = n - ti * tcur.cols;
            // q two passes ahead, then this pass's share of the next tile
            uint4_t qseg2 = {0u, 0u, 0u, 0u};
            {
                bool ok;
                const uint32_t off = seg_offset(min(pass + 2 * WAVES, npass - 1), ok);
                if (ok) qseg2 = *(const uint4_t*)(qb + off);
            }
            const int h = pass * 64 + lane;
            uint4_t pre[4];
            if (h < n_half) half_item_load(a, tnext, h, pre);

            // q segment -> per-lane channels through the wave's scratch
            uint32_t qraw[8];
            __builtin_amdgcn_wave_barrier();
            *(uint4_t*)(wbuf + chan_row(seg_c) + seg_h * 16) = qseg;
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int e = 0; e < 8; ++e) qraw[e] = *(const bf16_bits*)(wbuf + chan_row(8 * g + e) + p * 2);
            __builtin_amdgcn_wave_barrier();

            float o[8];
            slide_pass(buf, buf + a.g.v_off, HC, ti, tj, g, qraw, A1, A2, bias2, a.scale_log2e, ascr, o);

            // results -> 16-byte segments through the scratch
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int e = 0; e < 8; ++e) *(bf16_bits*)(wbuf + chan_row(8 * g + e) + p * 2) = f32_to_bf16(o[e]);
            __builtin_amdgcn_wave_barrier();
            {
                bool ok;
                const uint32_t off = seg_offset(pass, ok);
                const uint4_t ov = *(const uint4_t*)(wbuf + chan_row(seg_c) + seg_h * 16);
                if (ok) *(uint4_t*)(ob + off) = ov;
            }
            __builtin_amdgcn_wave_barrier();
            if (h < n_half) half_item_store(a, tnext, h, pre, buf_next);
            qseg = qseg1;
            qseg1 = qseg2;
        }
        // what the passes did not cover of the next tile (short tiles before tall ones)
        for (int h = npass * 64 + tid; h < n_half; h += THREADS) {
            uint4_t pre[4];
            half_item_load(a, tnext, h, pre);
            half_item_store(a, tnext, h, pre, buf_next);
        }
        if (!has_next) break;
        zero_pad_columns(a.g, tnext, buf_next, tid, THREADS);
        cur = nxt;
        tcur = tnext;
    }
}

// ------------------------------------------------------------------ host side
constexpr int FWD_WAVES = 4;

static TilePlan plan_fwd(const Problem& p, bool pipelined)
{
    const int budget = pipelined ? (LDS_LIMIT - PIPE_WAVES * WAVE_SCRATCH) / 2
                                 : LDS_LIMIT / 2 - FWD_WAVES * WAVE_SCRATCH;
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
    // the pipelined kernel needs 16-byte aligned rows everywhere and enough tiles per block
    const bool aligned = (p.W % 8 == 0) &&
                         (((uintptr_t)q | (uintptr_t)k | (uintptr_t)v | (uintptr_t)out) % 16 == 0);
    TilePlan t = plan_fwd(p, true);
    const bool pipelined = aligned && ((long)t.TA + t.TB >= 2L * NUM_CU);
    if (!pipelined) t = plan_fwd(p, false);
    uint32_t* image = (uint32_t*)workspace;
    hipLaunchKernelGGL(prep_weights_kernel, dim3(S, (unsigned)p.heads), dim3(256), 0, st,
                       wk, wv, bias, image);
    FwdArgs a;
    a.q = (const bf16_bits*)q; a.k = (const bf16_bits*)k; a.v = (const bf16_bits*)v;
    a.out = (bf16_bits*)out; a.image = image;
    fill_grid(a.g, p, t, k, v);
    a.buf_stride = t.buf_bytes;
    a.a_base = (pipelined ? 2 : 1) * t.buf_bytes;
    a.scale_log2e = 1.44269504088896341f / sqrtf((float)D);
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void*)fwd16_kernel<FWD_WAVES>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, LDS_LIMIT);
        if (e != hipSuccess) return e;
        e = hipFuncSetAttribute((const void*)fwd16_pipe_kernel,
                                hipFuncAttributeMaxDynamicSharedMemorySize, LDS_LIMIT);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const long n_tiles = (long)t.TA + t.TB;
    if (pipelined) {
        const int lds_bytes = a.a_base + PIPE_WAVES * WAVE_SCRATCH;
        hipLaunchKernelGGL(fwd16_pipe_kernel, dim3(NUM_CU), dim3(PIPE_WAVES * 64), (size_t)lds_bytes, st, a);
    } else {
        const int lds_bytes = a.a_base + FWD_WAVES * WAVE_SCRATCH;
        hipLaunchKernelGGL(fwd16_kernel<FWD_WAVES>, dim3((unsigned)n_tiles), dim3(FWD_WAVES * 64),
                           (size_t)lds_bytes, st, a);
    }
    return hipGetLastError();
}

}  // namespace slide
