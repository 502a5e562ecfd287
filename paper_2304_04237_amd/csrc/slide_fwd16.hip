// Matrix-core forward of Slide Attention for gfx950: bf16 activations, head size 32,
// 3x3 window.  One fused kernel: K/V halo tiles staged in LDS, merged depthwise
// kernels applied on the fly, softmax over the 9 shifts, weighted sum of the
// shifted values.  Nothing of size k*k*C ever reaches HBM.
//
// How the arithmetic is arranged (exactly the operator of Sec. 4.1-4.3, re-associated):
//   with the merged kernel W~ = one-hot shift + learned part (Sec. 4.3, Fig. 4)
//     logit[s] = scale * sum_{c,t} (q[c] k[c, p+t]) W~k[c,s,t]       <- 288 x 9 contraction, MFMA
//     out[c]   = sum_t v[c, p+t] * g[c,t],  g[c,t] = sum_s a[s] W~v[c,s,t]   <- 9 x 288, MFMA
//   Both contractions run on the matrix cores with half-precision operands and fp32
//   accumulation; the merged kernels enter as halves (1 + w keeps 11 significant bits, an
//   absolute error below 5e-4 on a weight near one, which moves a logit by about 1e-4 and an
//   output by less than 1e-3 at unit-scale inputs).
//
// Number format inside the kernel: the bf16 inputs are converted to IEEE half precision
// while they are staged (k, v) or loaded (q).  A bf16 value has 8 significant bits, a half
// has 11, so the conversion is exact for 2^-17 <= |x| <= 65504; smaller values are
// truncated to a multiple of 2^-24, larger ones saturate at +-65504.  Half precision is what lets the
// vector ALU form two q*k products per instruction (v_pk_mul_f16) and feed v halves straight
// into fp32 FMAs (v_fma_mix_f32) with no unpacking.  The q*k products that enter the matrix core are
// formed from q/16 and the K kernel is stored times 16, so products up to 2^20
// stay finite.
//
// Lane mapping: a wavefront handles 16 pixels at a time; lane = pixel p (0..15) +
// 16 * channel group g (0..3), group g owning channels 8g..8g+7 of the head.  This is
// the B-operand layout of v_mfma_f32_16x16x32_f16 with the channel as K index, and the
// D layout of v_mfma_f32_16x16x16_f16 with the pixel as column, so no data moves
// between lanes except two small cross-group reductions (v_permlane{16,32}_swap).
#include "slide_fwd16_ops.h"
#include <stdlib.h>

namespace slide {
namespace f16path {
using namespace t16;
using namespace f16ops;

constexpr int WAVE_SCRATCH = 1152;                 // per wave (pipelined kernel): 32 channels x 16 pixels of bf16
// byte offset of channel c's 16 pixels in the wave scratch (octets 64 banks apart would collide)
__device__ __forceinline__ int chan_row(int c) { return (c + (c >> 3)) * 32; }
// grid = (9, heads), block = 256: the images in global memory, for the one-tile-per-block kernel
__global__ void __launch_bounds__(256)
prep_weights_kernel(const float* __restrict__ wk, const float* __restrict__ wv,
                    const float* __restrict__ bias, uint32_t* __restrict__ image, float idw)
{
    const int m = blockIdx.y;
    uint32_t* img = image + (long)m * IMG_DWORDS;
    for (int idx = blockIdx.x * 256 + threadIdx.x; idx < IMG_BIAS; idx += gridDim.x * 256) {
        const ImageSource r = image_source(m, idx, idw);
        const float* w = r.from_v ? wv : wk;
        img[idx] = image_value(r, w[r.off0], w[r.off1]);
    }
    if (blockIdx.x == 0 && threadIdx.x < IMG_DWORDS - IMG_BIAS)
        img[IMG_BIAS + threadIdx.x] = image_bias(bias, m, threadIdx.x);
}

struct FwdArgs {
    const bf16_bits* q; const bf16_bits* k; const bf16_bits* v; bf16_bits* out;
    float* lse;              // [B, heads, H, W] log of the softmax denominator, or null
    const uint32_t* image;   // per-head MFMA operand images (one-tile-per-block kernel)
    const float* wk; const float* wv; const float* bias;   // merged kernels (pipelined kernel)
    TileGrid g;
    int buf_stride;          // bytes between the two tile buffers (pipelined kernel)
    int a_base;              // byte offset of the per-wave scratch (1 KB per wave)
    float scale_log2e;
    float idw;               // 1: wk, wv are the learned kernels of the two-branch form; 0: merged
};

// q of one pixel: 8 channels as bf16 patterns (one per dword) -> halves divided by 16
__device__ __forceinline__ void q_halves(const uint32_t (&qraw)[8], half2_t (&qs)[4])
{
#pragma unroll
    for (int y = 0; y < 4; ++y) {
        const uint32_t pk = pack_half_rtz(__uint_as_float(qraw[2 * y] << 16),
                                          __uint_as_float(qraw[2 * y + 1] << 16));
        qs[y] = as_half2(pk) * half2_t{(_Float16)G_SCALE, (_Float16)G_SCALE};
    }
}

// The arithmetic of one pass: 16 pixels, lane = (pixel p, channel group g); (ti, tj) is the
// lane's pixel inside the tile, qs its 8 q channels as halves, already divided by 16.
// Returns the 8 output channels in o.  With LSE, lanes whose lse_dst is not null also store
// the natural logarithm of their pixel's softmax denominator there (as soon as it is known,
// so that nothing of it stays live through the V side).
template <bool LSE>
__device__ __forceinline__ void slide_pass(const unsigned char* kl, int RS, int VD,
                                           int ti, int tj, int g, const half2_t (&qs)[4],
                                           const half8_t (&A1)[S], const half4_t (&A2)[2 * S],
                                           const float (&bias2)[3], float scale_log2e, float (&o)[8],
                                           float* lse_dst)
{
    // halo row stride RS bytes; the V pixel sits VD bytes after the K pixel.  With both known
    // at compile time every tap address is one of three registers plus an immediate.
    const unsigned char* cb[KS];
#pragma unroll
    for (int tx = 0; tx < KS; ++tx) cb[tx] = kl + ti * RS + col_offset(tj + tx, g);
    uint4_t kd[S];
#pragma unroll
    for (int t = 0; t < S; ++t) kd[t] = *(const uint4_t*)(cb[t % KS] + (t / KS) * RS);

    // ---- K side: the nine logits, row 4g+r of the product in acc1[r] of lane group g
    float4_t acc1 = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int t = 0; t < S; ++t) {
        uint4_t bb;
#pragma unroll
        for (int y = 0; y < 4; ++y) bb[y] = as_dword(qs[y] * as_half2(kd[t][y]));
        acc1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(A1[t], __builtin_bit_cast(half8_t, bb), acc1, 0, 0, 0);
    }
    // V taps: issue the LDS reads now, they land while the softmax runs
    uint4_t vd[S];
#pragma unroll
    for (int t = 0; t < S; ++t)
        vd[t] = *(const uint4_t*)(cb[t % KS] + (t / KS) * RS + VD);

    // ---- softmax over the 9 shifts (3 per lane, 4 lane groups; unused rows have bias -inf)
    float l[3];
#pragma unroll
    for (int r = 0; r < 3; ++r) l[r] = fmaf(acc1[r], scale_log2e, bias2[r]);
    const float mx = allmax_groups(fmaxf(fmaxf(l[0], l[1]), l[2]));
    float pr[3];
#pragma unroll
    for (int r = 0; r < 3; ++r) pr[r] = __builtin_amdgcn_exp2f(l[r] - mx);
    const float den = allsum_groups(pr[0] + pr[1] + pr[2]);
    const float inv = __builtin_amdgcn_rcpf(den);
    if (LSE && lse_dst) *lse_dst = LN2 * (mx + __builtin_amdgcn_logf(den));
    uint2_t b2;
    b2[0] = pack_half(pr[0] * inv, pr[1] * inv);
    b2[1] = pack_half(pr[2] * inv, 0.0f);
    const half4_t B2 = __builtin_bit_cast(half4_t, b2);

    // ---- V side: out[c] = sum_t v[c, p+t] * g[c,t] with g = W~v^T a from the matrix core.
    // Product u < 16 gives, in its four result registers, the weights of channel u & 7 for
    // taps 4(u >> 3) .. +3; products 16, 17 those of channels 0..3, 4..7 for tap 8.  Two
    // products stay in flight ahead of the multiply-adds that consume them.
    const float4_t zero4 = {0.0f, 0.0f, 0.0f, 0.0f};
    float4_t w[2 * S];
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = 0.0f;
    constexpr int AHEAD = 2;
#pragma unroll
    for (int u = 0; u < AHEAD; ++u) w[u] = __builtin_amdgcn_mfma_f32_16x16x16f16(A2[u], B2, zero4, 0, 0, 0);
#pragma unroll
    for (int u = 0; u < 2 * S; ++u) {
        if (u + AHEAD < 2 * S)
            w[u + AHEAD] = __builtin_amdgcn_mfma_f32_16x16x16f16(A2[u + AHEAD], B2, zero4, 0, 0, 0);
        // scheduling fence: without it the compiler issues all products first and keeps all
        // 72 results live
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int e = u < 16 ? (u & 7) : 4 * (u - 16) + r;
            const int tap = u < 16 ? 4 * (u >> 3) + r : 8;
            o[e] = fmaf(w[u][r], (float)as_half2(vd[tap][e >> 1])[e & 1], o[e]);
        }
        __builtin_amdgcn_sched_barrier(0);
    }
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
        half2_t qs[4];
        q_halves(qraw, qs);
        float* lse_dst = (a.lse && valid && g == 0)
            ? a.lse + tcur.head_base / D + (long)(tcur.i0 + ti) * a.g.W + tcur.j0 + tj : nullptr;
        slide_pass<true>(smem, HC * 64, a.g.v_off, ti, tj, g, qs, A1, A2, bias2, a.scale_log2e, o, lse_dst);
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
// next tile (four 16-byte loads per lane at the start of the pass, converted into the other
// buffer one pass later), so global loads and arithmetic overlap inside the block instead of
// alternating across the whole chip.  The block also builds its head's operand image itself.
// q comes in and results go out as 16-byte row segments: lane (c = lane/2, h = lane%2) moves
// pixels 16*pass + 8h .. +7 of channel c, and the wave's scratch transposes between that and
// the per-lane (pixel, 8 channels) view.  Vector memory operations retire in order, so the q
// segment is fetched two passes ahead.
//
// Tile buffer of this kernel: halo row hr = [K pixels HC x 64 B][V pixels HC x 64 B], pixel
// = 32 channels as halves with the 16-byte channel octets swizzled as in col_offset().
// TW is the tile width when known at compile time (then tap addresses need no arithmetic),
// 0 = read it from the arguments.  LSE: also write the log of the softmax denominator.
constexpr int PIPE_WAVES = 8;

// Staging unit ("share") n of a tile: wave-sized group hb = n / 64 handles tensor hb & 1;
// inside the tensor, unit u = (hb / 2) * 64 + n % 64 is channel quad u & 7 of 16-byte chunk
// u / 8 = (halo row, chunk in row): 4 channels x 8 columns.
struct ShareGeom {
    int n_units;             // units per tensor: 8 * NX * (rows + 2)
    int n_groups;            // wave-sized groups over both tensors
    uint32_t recip_nx;       // ceil(65536 / NX): (x * recip_nx) >> 16 == x / NX for x < 4096
};
__device__ __forceinline__ ShareGeom share_geom(const Tile& t)
{
    ShareGeom s;
    s.n_units = t.n_items;                              // 8 * NX * (rows + 2)
    s.n_groups = 2 * ((s.n_units + 63) >> 6);
    s.recip_nx = (65536u + (uint32_t)t.NX - 1u) / (uint32_t)t.NX;
    return s;
}

__device__ __forceinline__ void share_load(const FwdArgs& a, const Tile& t, const ShareGeom& sg, int hb,
                                           int lane, uint32_t hw2, uint4_t (&r)[4])
{
    const int u = (hb >> 1) * 64 + lane;
    const int cq = u & 7, rest = u >> 3;
    const int hr = (int)(((uint32_t)rest * sg.recip_nx) >> 16), x = rest - hr * t.NX;
    const int gi = t.i0 - 1 + hr;
    if (u >= sg.n_units || gi < 0 || gi >= a.g.H) {
#pragma unroll
        for (int e = 0; e < 4; ++e) r[e] = uint4_t{0u, 0u, 0u, 0u};
        return;
    }
    const char* base = (const char*)(((hb & 1) ? a.v : a.k) + t.head_base);   // wave-uniform
    const uint32_t off = (uint32_t)(4 * cq) * hw2 + (uint32_t)(gi * a.g.W + t.gxa + 8 * x) * 2u;
#pragma unroll
    for (int e = 0; e < 4; ++e) r[e] = *(const uint4_t*)(base + (off + (uint32_t)e * hw2));
}

template <bool EDGE_CHECK>
__device__ __forceinline__ void share_store(const Tile& t, const ShareGeom& sg, int hb, int lane, int HC,
                                            const uint4_t (&r)[4], unsigned char* buf)
{
    const int u = (hb >> 1) * 64 + lane;
    if (u >= sg.n_units) return;
    const int cq = u & 7, rest = u >> 3;
    const int hr = (int)(((uint32_t)rest * sg.recip_nx) >> 16), x = rest - hr * t.NX;
    // first halo column of the chunk: a multiple of 8 plus 1 (the chunk grid is 8-aligned and
    // a tile starts at a multiple of 64), so the swizzle term of column hc0 + px depends on px only
    const int hc0 = t.gxa + 8 * x - (t.j0 - 1);
    unsigned char* dst = buf + (2 * hr + (hb & 1)) * (HC * 64) + hc0 * 64 + (cq & 1) * 8;
    const int o4 = (cq >> 1) << 4;
    unsigned char* dsw[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) dsw[c] = dst + (o4 ^ (c << 4));
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
        const int hc = hc0 + px;
        if (!EDGE_CHECK || (hc >= 0 && hc < t.cols + 2))
            *(uint2_t*)(dsw[((1 + px) >> 1) & 3] + px * 64) = t2;
    }
}

// halo columns outside the map are zero (both tensors, all rows of the tile)
__device__ __forceinline__ void pipe_zero_pad(const TileGrid& a, const Tile& t, int HC, unsigned char* buf,
                                              int tid, int threads)
{
    const bool left = (t.j0 == 0), right = (t.j0 + t.cols == a.W);
    if (!left && !right) return;
    const int n = (t.rows + 2) * 16;                    // row x side x tensor x channel octet
    for (int idx = tid; idx < n; idx += threads) {
        const int o = idx & 3, tsel = (idx >> 2) & 1, side = (idx >> 3) & 1, hr = idx >> 4;
        if (side ? !right : !left) continue;
        const int hc = side ? t.cols + 1 : 0;
        *(uint4_t*)(buf + (2 * hr + tsel) * (HC * 64) + col_offset(hc, o)) = uint4_t{0u, 0u, 0u, 0u};
    }
}

template <int TW, bool LSE>
__global__ void __launch_bounds__(PIPE_WAVES * 64, 2)
fwd16_pipe_kernel(const FwdArgs a)
{
    constexpr int WAVES = PIPE_WAVES, THREADS = WAVES * 64;
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int p = lane & 15, g = lane >> 4;
    const int HC = (TW ? TW : a.g.tw) + 2;
    const bool single_col = a.g.n_tc == 1;              // then no staged column falls outside a tile
    const uint32_t hw2 = (uint32_t)a.g.H * (uint32_t)a.g.W * 2u;
    const int n_tiles = a.g.TA + a.g.TB;
    unsigned char* wbuf = smem + a.a_base + wave * WAVE_SCRATCH;
    const int seg_c = lane >> 1, seg_h = lane & 1;

    int cur = blockIdx.x;                               // gridDim.x <= n_tiles
    Tile tcur = decode_tile(a.g, cur);
    // The block builds the operand image of its head in the second tile buffer, which is
    // free until the first pass (no separate preparation kernel on this path).
    build_image<THREADS>(a.wk, a.wv, a.bias, tcur.m, a.idw, (uint32_t*)(smem + a.buf_stride),
                         (float*)(smem + a.buf_stride + IMG_RAW_AT), tid);
    // the first tile is staged without overlap, two shares per lane in flight
    {
        const ShareGeom sg = share_geom(tcur);
        for (int hb = wave; hb < sg.n_groups; hb += 2 * WAVES) {
            uint4_t r0[4], r1[4];
            share_load(a, tcur, sg, hb, lane, hw2, r0);
            if (hb + WAVES < sg.n_groups) share_load(a, tcur, sg, hb + WAVES, lane, hw2, r1);
            share_store<true>(tcur, sg, hb, lane, HC, r0, smem);
            if (hb + WAVES < sg.n_groups) share_store<true>(tcur, sg, hb + WAVES, lane, HC, r1, smem);
        }
        pipe_zero_pad(a.g, tcur, HC, smem, tid, THREADS);
    }

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
        ShareGeom sg = share_geom(tnext);
        if (!has_next) sg.n_groups = 0;
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
        // q segment of this wave's first pass
        uint4_t qseg;
        {
            bool ok;
            qseg = *(const uint4_t*)(qb + seg_offset(min(wave, npass - 1), ok));
        }
        __syncthreads();                                // buf is complete, buf_next is free
        if (tcur.m != m_loaded) {
            if (it > 0) {                               // the block moves on to another head
                build_image<THREADS>(a.wk, a.wv, a.bias, tcur.m, a.idw, (uint32_t*)buf_next,
                                     (float*)(buf_next + IMG_RAW_AT), tid);
                __syncthreads();
            }
            load_operands((const uint32_t*)buf_next, lane, g, A1, A2, bias2);
            m_loaded = tcur.m;
            __syncthreads();                            // everyone holds the operands: buf_next is free again
        }

        // K and V of the next tile: the loads of a pass's share are issued at its start and
        // converted into buf_next at its end, before the pass's results are stored.  Nothing
        // that a load fills is copied or carried into another iteration: the only wait for
        // vector memory sits before the conversion, where everything it waits for was issued a
        // pass ago or longer (the store of the previous pass included).  A wait placed after a
        // store would expose the store's completion time in every pass.
        auto store_share = [&](int hb, const uint4_t (&r)[4]) {
            if (single_col) share_store<false>(tnext, sg, hb, lane, HC, r, buf_next);
            else            share_store<true>(tnext, sg, hb, lane, HC, r, buf_next);
        };
        asm volatile("" :: "v"(qseg));                  // the first q has arrived before the loop starts
        for (int pass = wave; pass < npass; pass += WAVES) {
            int n = pass * 16 + p;
            n = n < npix ? n : npix - 1;
            const int ti = (int)(((float)n + 0.5f) * inv_tw);
            const int tj = n - ti * tcur.cols;
            // q segment -> per-lane channels through the wave's scratch
            uint32_t qraw[8];
            __builtin_amdgcn_wave_barrier();
            *(uint4_t*)(wbuf + chan_row(seg_c) + seg_h * 16) = qseg;
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int e = 0; e < 8; ++e) qraw[e] = *(const bf16_bits*)(wbuf + chan_row(8 * g + e) + p * 2);
            __builtin_amdgcn_wave_barrier();
            // q of the wave's next pass, then this pass's share of the next tile
            {
                bool ok;
                const uint32_t off = seg_offset(min(pass + WAVES, npass - 1), ok);
                qseg = *(const uint4_t*)(qb + off);     // (the offset is valid even when the segment is not)
            }
            uint4_t pre[4];
            if (pass < sg.n_groups) share_load(a, tnext, sg, pass, lane, hw2, pre);

            float o[8];
            half2_t qs[4];
            q_halves(qraw, qs);
            float* lse_dst = nullptr;
            if (LSE && g == 0 && pass * 16 + p < npix)
                lse_dst = a.lse + tcur.head_base / D + (long)(tcur.i0 + ti) * a.g.W + tcur.j0 + tj;
            slide_pass<LSE>(buf, 2 * HC * 64, HC * 64, ti, tj, g, qs, A1, A2, bias2, a.scale_log2e, o, lse_dst);

            // results -> 16-byte segments through the scratch
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int e = 0; e < 8; ++e) *(bf16_bits*)(wbuf + chan_row(8 * g + e) + p * 2) = f32_to_bf16(o[e]);
            __builtin_amdgcn_wave_barrier();
            const uint4_t ov = *(const uint4_t*)(wbuf + chan_row(seg_c) + seg_h * 16);
            __builtin_amdgcn_wave_barrier();
            if (pass < sg.n_groups) store_share(pass, pre);
            // every load of this pass counts as used here, on every path: the waits sit here,
            // before the store, and nothing is left pending that a later wait would have to cover
            asm volatile("" :: "v"(qseg), "v"(pre[0]), "v"(pre[1]), "v"(pre[2]), "v"(pre[3]));
            {
                bool ok;
                const uint32_t off = seg_offset(pass, ok);
                if (ok) *(uint4_t*)(ob + off) = ov;
            }
        }
        // what the passes did not cover of the next tile (short tiles before tall ones)
        for (int hb = wave + ((npass - wave + WAVES - 1) / WAVES) * WAVES; hb < sg.n_groups; hb += WAVES) {
            uint4_t pre[4];
            share_load(a, tnext, sg, hb, lane, hw2, pre);
            store_share(hb, pre);
            asm volatile("" :: "v"(pre[0]), "v"(pre[1]), "v"(pre[2]), "v"(pre[3]));
        }
        if (!has_next) break;
        pipe_zero_pad(a.g, tnext, HC, buf_next, tid, THREADS);
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
    if ((long)p.H * p.W * 2 * f16path::D >= (1L << 31)) return false;   // 32-bit byte offsets inside a head
    const long planes = (long)p.B * p.heads * ((p.W + 63) / 64);
    return planes * p.H < (1L << 30);                    // tile count fits an int
}

// per head: the MFMA operand image
size_t fwd_mfma_workspace_bytes(const Problem& p)
{
    return fwd_mfma_supported(p) ? (size_t)p.heads * f16path::IMG_DWORDS * sizeof(uint32_t) : 0;
}

namespace f16path {
// Which 3x3 kernel serves a problem.  The pipelined kernel needs 16-byte aligned rows and
// pointers, at least two tiles per persistent block, and a tile buffer large enough to hold a
// head's operand image plus the raw kernels it is gathered from (the block builds the image in
// the tile buffer that is free at that moment).
static bool choose_pipelined(const Problem& p, bool aligned16, TilePlan& t)
{
    t = plan_fwd(p, true);
    const bool pipelined = aligned16 && (p.W % 8 == 0) &&
                           ((long)t.TA + t.TB >= 2L * device_cu_count()) &&
                           t.buf_bytes >= IMG_RAW_AT + IMG_RAW_BYTES;
    if (!pipelined) t = plan_fwd(p, false);
    return pipelined;
}

}  // namespace f16path

// SLIDE_ATTN_DISABLE_RING=1 in the environment keeps the streaming kernel out of the dispatch
// (for side-by-side measurements of the tiled kernels); read once.
bool fwd_ring_enabled()
{
    static const bool on = [] {
        const char* e = getenv("SLIDE_ATTN_DISABLE_RING");
        return !(e && e[0] == '1');
    }();
    return on;
}

int fwd_mfma_variant(const Problem& p, bool aligned16)
{
    using namespace f16path;
    if (fwd_ring_enabled() && fwd_ring_supported(p, aligned16)) return 24;
    if (fwd_ring_enabled() && fwd_ring_strip_supported(p, aligned16)) return 26;
    TilePlan t;
    if (!choose_pipelined(p, aligned16, t)) return 20;
    return t.tw == 64 ? 23 : 21;
}

hipError_t launch_fwd_mfma(const Problem& p, const void* q, const void* k, const void* v,
                           const float* wk, const float* wv, const float* bias, void* out,
                           float* lse, void* workspace, hipStream_t st)
{
    using namespace f16path;
    const bool aligned = (((uintptr_t)q | (uintptr_t)k | (uintptr_t)v | (uintptr_t)out |
                           (uintptr_t)wk | (uintptr_t)wv) % 16 == 0);
    if (fwd_ring_enabled() && fwd_ring_supported(p, aligned))
        return launch_fwd_ring(p, q, k, v, wk, wv, bias, out, lse, false, st);
    if (fwd_ring_enabled() && fwd_ring_strip_supported(p, aligned))
        return launch_fwd_ring_strip(p, q, k, v, wk, wv, bias, out, lse, false, st);
    TilePlan t;
    const bool pipelined = choose_pipelined(p, aligned, t);
    uint32_t* image = (uint32_t*)workspace;
    if (!pipelined)
        hipLaunchKernelGGL(prep_weights_kernel, dim3(S, (unsigned)p.heads), dim3(256), 0, st,
                           wk, wv, bias, image, p.two_branch ? 1.0f : 0.0f);
    FwdArgs a;
    a.q = (const bf16_bits*)q; a.k = (const bf16_bits*)k; a.v = (const bf16_bits*)v;
    a.out = (bf16_bits*)out; a.lse = lse; a.image = image;
    a.wk = wk; a.wv = wv; a.bias = bias;
    fill_grid(a.g, p, t, k, v);
    a.g.small_first = pipelined;
    a.buf_stride = t.buf_bytes;
    a.a_base = (pipelined ? 2 : 1) * t.buf_bytes;
    a.scale_log2e = 1.44269504088896341f * p.logit_scale();
    a.idw = p.two_branch ? 1.0f : 0.0f;
    static LdsOptIn opt_in;
    hipError_t e = opt_in.ensure({(const void*)fwd16_kernel<FWD_WAVES>,
                                  (const void*)fwd16_pipe_kernel<0, false>, (const void*)fwd16_pipe_kernel<64, false>,
                                  (const void*)fwd16_pipe_kernel<0, true>, (const void*)fwd16_pipe_kernel<64, true>},
                                 LDS_LIMIT);
    if (e != hipSuccess) return e;
    const long n_tiles = (long)t.TA + t.TB;
    if (pipelined) {
        const int lds_bytes = a.a_base + PIPE_WAVES * WAVE_SCRATCH;
        const dim3 grid((unsigned)device_cu_count()), block(PIPE_WAVES * 64);
#define SLIDE_PIPE(TWV)                                                                                      \
        do {                                                                                                 \
            if (lse) hipLaunchKernelGGL((fwd16_pipe_kernel<TWV, true>), grid, block, (size_t)lds_bytes, st, a);  \
            else     hipLaunchKernelGGL((fwd16_pipe_kernel<TWV, false>), grid, block, (size_t)lds_bytes, st, a); \
        } while (0)
        if (t.tw == 64) SLIDE_PIPE(64);
        else            SLIDE_PIPE(0);
#undef SLIDE_PIPE
    } else {
        const int lds_bytes = a.a_base + FWD_WAVES * WAVE_SCRATCH;
        hipLaunchKernelGGL(fwd16_kernel<FWD_WAVES>, dim3((unsigned)n_tiles), dim3(FWD_WAVES * 64),
                           (size_t)lds_bytes, st, a);
    }
    return hipGetLastError();
}

}  // namespace slide
