// Matrix-core forward of Slide Attention for gfx950: bf16 activations, head size 32,
// 3x3 window.  One fused kernel: K/V halo tiles staged in LDS, merged depthwise
// kernels applied on the fly, softmax over the 9 shifts, weighted sum of the
// shifted values.  Nothing of size k*k*C ever reaches HBM.
//
// How the arithmetic is arranged (exactly the operator of Sec. 4.1-4.3, re-associated):
//   merged kernel = one-hot shift + learned part (Sec. 4.3, Fig. 4), so
//     logit[s] = scale * ( sum_c q[c] k[c, p+s]                       <- shift path, exact fp32
//                        + sum_{c,t} (q[c] k[c, p+t]) wl_k[c,s,t] )    <- learned path, MFMA
//     out[c]   = sum_t v[c, p+t] * ( a[t] + sum_s a[s] wl_v[c,s,t] )   <- a[t]: shift path (fp32),
//                                                                        sum_s: learned path, MFMA
//   The learned paths are the only dense contractions (288 x 9 per pixel and head); they
//   run on the matrix cores with bf16 operands and fp32 accumulation.  The shift paths
//   stay in fp32 so that 1 + w is never rounded to bf16.
//
// Lane mapping: a wavefront handles 16 pixels at a time; lane = pixel p (0..15) +
// 16 * channel group g (0..3), group g owning channels 8g..8g+7 of the head.  This is
// the B-operand layout of v_mfma_f32_16x16x32_bf16 with the channel as K index, and the
// D layout of v_mfma_f32_16x16x16_bf16 with the pixel as column, so no data moves
// between lanes except two small cross-group reductions (v_permlane{16,32}_swap).
//
// K side, per tap t, with G_e = q[e]*k[e,p+t] for the lane's channels e = 0..7: one
// v_dot2c_f32_bf16 per channel pair y accumulates the running sum R_y = sum_{e <= 2y+1} G_e
// in place, and one multiply gives the odd product O_y = G_{2y+1}.  (R_y, O_y) are rounded
// to bf16 and fed to the MFMA against re-combined learned weights
//     sum_e G_e w_e = sum_y R_y (w_{2y} - w_{2y+2}) + O_y (w_{2y+1} - w_{2y}),   w_8 = 0
// (summation by parts), and the last running sum R_3 is the lane's share of the exact
// shift-path logit for free.
#include "slide_internal.h"
#include "slide_device.h"

namespace slide {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef __attribute__((ext_vector_type(4))) short short4_t;
typedef __attribute__((ext_vector_type(4))) float float4_t;
typedef __attribute__((ext_vector_type(4))) uint32_t uint4_t;
typedef __attribute__((ext_vector_type(2))) uint32_t uint2_t;

constexpr int KS = 3, S = 9, D = 32;
constexpr int WAVES = 4, THREADS = WAVES * 64;
constexpr int A_STRIDE = 17;                       // floats per pixel in the attention scratch
constexpr int A_SCRATCH_BYTES = WAVES * 16 * A_STRIDE * 4;

// Per-head image of the MFMA weight operands, written by prep_weights_kernel (dwords):
//   [0, 2304)      A1: tap t (9) x lane (64) x 4 dwords  -- differenced learned K kernel
//   [2304, 4608)   A2: tap t (9) x half j (2) x lane (64) x 2 dwords -- learned V kernel
//   [4608, 4624)   bias row r (16) as float, times log2(e); -inf on unused rows
constexpr int IMG_A1 = 0, IMG_A2 = 2304, IMG_BIAS = 4608, IMG_DWORDS = 4624;

// MFMA row 4g+r of the logit tile <-> shift index.  Rows are spread so that each lane
// group holds at most three live shifts: rows r=0,1 of every group and row 2 of group 0.
__host__ __device__ constexpr int shift_of_row(int row)
{
    const int g = row >> 2, r = row & 3;
    const int s = 4 * r + g;
    return (r < 2 || (r == 2 && g == 0)) ? s : -1;
}

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi)
{
    bf16x2_t v = {(__bf16)lo, (__bf16)hi};
    return __builtin_bit_cast(uint32_t, v);
}

// ------------------------------------------------------------------ weight preparation
// grid = (9 taps, heads), block = 256.  Reads the merged float32 kernels [C, 9, 3, 3] and
// writes the per-head operand image described above.
__global__ void __launch_bounds__(256)
prep_weights_kernel(const float* __restrict__ wk, const float* __restrict__ wv,
                    const float* __restrict__ bias, uint32_t* __restrict__ image)
{
    const int t = blockIdx.x, m = blockIdx.y;
    uint32_t* img = image + (long)m * IMG_DWORDS;
    const int tid = threadIdx.x;
    {
        // A1: dword y of lane (i, g) = weights met by (R_y, O_y) for shift row i, channels
        // 8g+2y and 8g+2y+1:  (w_{2y} - w_{2y+2},  w_{2y+1} - w_{2y}), learned part only.
        const int y = tid & 3, lane = tid >> 2;
        const int i = lane & 15, g = lane >> 4;
        const int s = shift_of_row(i);
        float d0 = 0.0f, d1 = 0.0f;
        if (s >= 0) {
            const float id = (s == t) ? 1.0f : 0.0f;
            const int c = m * D + 8 * g + 2 * y;
            const float w_even = wk[((long)c * S + s) * S + t] - id;
            const float w_odd = wk[((long)(c + 1) * S + s) * S + t] - id;
            const float w_next = (y < 3) ? wk[((long)(c + 2) * S + s) * S + t] - id : 0.0f;
            d0 = w_even - w_next;
            d1 = w_odd - w_even;
        }
        img[IMG_A1 + t * 256 + tid] = pack_bf16(d0, d1);
    }
    {
        // A2: dword y of lane (i, g) at half j = learned V weights of channel
        // 8*(i/4) + 4j + (i%4) for the shifts of logit rows 4g+2y, 4g+2y+1.
        const int y = tid & 1, lane = (tid >> 1) & 63, j = tid >> 7;
        const int i = lane & 15, g = lane >> 4;
        const int c = m * D + 8 * (i >> 2) + 4 * j + (i & 3);
        float d[2] = {0.0f, 0.0f};
        for (int h = 0; h < 2; ++h) {
            const int s = shift_of_row(4 * g + 2 * y + h);
            if (s >= 0) d[h] = wv[((long)c * S + s) * S + t] - (s == t ? 1.0f : 0.0f);
        }
        img[IMG_A2 + t * 256 + tid] = pack_bf16(d[0], d[1]);
    }
    if (t == 0 && tid < 16) {
        const int s = shift_of_row(tid);
        float b = -INFINITY;
        if (s >= 0) b = bias ? bias[m * S + s] * 1.44269504088896341f : 0.0f;
        img[IMG_BIAS + tid] = __float_as_uint(b);
    }
}

// ------------------------------------------------------------------ cross-group reductions
// lanes l and l+32:  returns a[l] + a[l+32] in lanes 0..31 and b[l-32] + b[l] in lanes 32..63
__device__ __forceinline__ float fold32(float a, float b)
{
    uint2_t r = __builtin_amdgcn_permlane32_swap(__float_as_uint(a), __float_as_uint(b), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
// rows of 16 lanes: returns (a.r0+a.r1, b.r0+b.r1, a.r2+a.r3, b.r2+b.r3)
__device__ __forceinline__ float fold16(float a, float b)
{
    uint2_t r = __builtin_amdgcn_permlane16_swap(__float_as_uint(a), __float_as_uint(b), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
__device__ __forceinline__ float allmax_groups(float x)
{
    uint2_t r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    x = fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
    r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float allsum_groups(float x)
{
    uint2_t r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    x = __uint_as_float(r[0]) + __uint_as_float(r[1]);
    r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

__device__ __forceinline__ float dot2_bf16(uint32_t a, uint32_t b, float c)
{
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a),
                                           __builtin_bit_cast(bf16x2_t, b), c, false);
}

// byte offset of (halo column hc, channel group g) inside a halo row: 64 B per pixel,
// the four 16-byte channel-group slots XOR-swizzled by the column so that 8 consecutive
// pixels of one group fall on 8 different bank quads.
__device__ __forceinline__ int col_offset(int hc, int g)
{
    return hc * 64 + ((g ^ ((hc >> 1) & 3)) << 4);
}

struct FwdArgs {
    const bf16_bits* q; const bf16_bits* k; const bf16_bits* v; bf16_bits* out;
    const uint32_t* image;
    int B, H, W, C, heads;
    int th, tw;              // tile size in pixels
    int n_tr, n_tc;          // tiles per plane (rows, columns)
    int v_base;              // byte offset of the V halo in LDS
    int a_base;              // byte offset of the attention scratch in LDS
    int vec_ok;              // rows are 16-byte aligned: W % 8 == 0 and 16-byte aligned bases
    float scale_log2e;
};

// ------------------------------------------------------------------ the fused forward
__global__ void __launch_bounds__(THREADS, 2)
fwd_mfma_kernel(const FwdArgs a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int p = lane & 15, g = lane >> 4;

    // ---- which tile: consecutive tiles of a plane go to the same XCD (blocks are dealt
    // round-robin over the 8 XCDs, each with its own L2), so halo rows are re-read from L2.
    const int n_blocks = gridDim.x;
    int vid = blockIdx.x;
    if ((n_blocks & 7) == 0) vid = (blockIdx.x & 7) * (n_blocks >> 3) + (blockIdx.x >> 3);
    const int tiles_per_plane = a.n_tr * a.n_tc;
    const int plane_id = vid / tiles_per_plane;
    const int tile_id = vid - plane_id * tiles_per_plane;
    const int tc = tile_id / a.n_tr, tr = tile_id - tc * a.n_tr;
    const int b = plane_id / a.heads, m = plane_id - b * a.heads;
    const int i0 = tr * a.th, j0 = tc * a.tw;
    const int th_eff = min(a.th, a.H - i0), tw_eff = min(a.tw, a.W - j0);
    const int HR = a.th + 2, HC = a.tw + 2;
    const long HW = (long)a.H * a.W;
    const long head_base = ((long)b * a.C + (long)m * D) * HW;     // element offset of channel 0 of the head

    // ---- MFMA weight operands of this head (coalesced reads of the prepared image)
    const uint32_t* img = a.image + (long)m * IMG_DWORDS;
    bf16x8_t A1[S];
    short4_t A2[S][2];
#pragma unroll
    for (int t = 0; t < S; ++t) {
        uint4_t w = *(const uint4_t*)(img + IMG_A1 + (t * 64 + lane) * 4);
        A1[t] = __builtin_bit_cast(bf16x8_t, w);
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            uint2_t w2 = *(const uint2_t*)(img + IMG_A2 + ((t * 2 + j) * 64 + lane) * 2);
            A2[t][j] = __builtin_bit_cast(short4_t, w2);
        }
    }
    float bias2[3];
#pragma unroll
    for (int r = 0; r < 3; ++r) bias2[r] = __uint_as_float(img[IMG_BIAS + 4 * g + r]);

    // ---- stage the K and V halo tiles: global NCHW -> LDS [row][col][32 channels]
    {
        const int gx0 = ((j0 - 1) >= 0 ? (j0 - 1) : (j0 - 8)) & ~7;       // floor to a multiple of 8
        const int NX = (j0 - 1 + HC - gx0 + 7) >> 3;
        const int n_items = 8 * NX * HR;
        for (int idx = tid; idx < n_items; idx += THREADS) {
            // item = 8 channels (group o) x 8 columns (chunk x) of one halo row of K or V
            const int o = idx & 3, tsel = (idx >> 2) & 1;
            const int rest = idx >> 3;
            const int hr = rest / NX, x = rest - hr * NX;
            const int gi = i0 - 1 + hr, gx = gx0 + 8 * x;
            const bool row_ok = (gi >= 0) && (gi < a.H);
            const bool any_in = row_ok && (gx + 8 > 0) && (gx < a.W);
            const bf16_bits* plane0 = (tsel ? a.v : a.k) + head_base + (long)(8 * o) * HW;
            uint4_t r[8];
            if (any_in && a.vec_ok && gx >= 0 && gx + 8 <= a.W) {
                const bf16_bits* src = plane0 + (long)gi * a.W + gx;
#pragma unroll
                for (int e = 0; e < 8; ++e) r[e] = *(const uint4_t*)(src + e * HW);
            } else if (any_in) {
                // ragged chunk: element loads from clamped (always valid) columns, then masked
                const bf16_bits* src = plane0 + (long)gi * a.W;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
#pragma unroll
                    for (int y = 0; y < 4; ++y) {
                        const int c0 = gx + 2 * y, c1 = c0 + 1;
                        const int cc0 = min(max(c0, 0), a.W - 1), cc1 = min(max(c1, 0), a.W - 1);
                        uint32_t lo = src[e * HW + cc0], hi = src[e * HW + cc1];
                        lo = (c0 == cc0) ? lo : 0u;
                        hi = (c1 == cc1) ? hi : 0u;
                        r[e][y] = lo | (hi << 16);
                    }
                }
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) r[e] = uint4_t{0u, 0u, 0u, 0u};
            }
            unsigned char* dst = smem + (tsel ? a.v_base : 0) + hr * HC * 64;
#pragma unroll
            for (int px = 0; px < 8; ++px) {
                uint4_t t4;
#pragma unroll
                for (int y = 0; y < 4; ++y) {
                    const uint32_t lo = r[2 * y][px >> 1], hi = r[2 * y + 1][px >> 1];
                    t4[y] = (px & 1) ? __builtin_amdgcn_perm(hi, lo, 0x07060302u)
                                     : __builtin_amdgcn_perm(hi, lo, 0x05040100u);
                }
                const int hc = gx + px - (j0 - 1);
                if (hc >= 0 && hc < HC) *(uint4_t*)(dst + col_offset(hc, o)) = t4;
            }
        }
    }
    __syncthreads();

    // ---- passes of 16 pixels
    const int npix = th_eff * tw_eff;
    const int npass = (npix + 15) >> 4;
    const float inv_tw = 1.0f / (float)tw_eff;
    float* ascr = (float*)(smem + a.a_base) + wave * 16 * A_STRIDE + p * A_STRIDE;
    const unsigned char* kl = smem;
    const unsigned char* vl = smem + a.v_base;
    const bf16_bits* qbase = a.q + head_base;           // block-uniform bases, 32-bit lane offsets
    bf16_bits* obase = a.out + head_base;
    const uint32_t hw = (uint32_t)HW;
    const uint32_t lane_chan = (uint32_t)(8 * g) * hw + (uint32_t)i0 * a.W + j0;

    // (tile row, tile column) of this lane's pixel in a pass; lanes past the end repeat the
    // last pixel (they compute but do not store)
    auto pixel_of = [&](int pass, int& ti, int& tj) -> bool {
        int n = pass * 16 + p;
        const bool valid = n < npix;
        n = valid ? n : npix - 1;
        ti = (int)(((float)n + 0.5f) * inv_tw);
        tj = n - ti * tw_eff;
        return valid;
    };

    uint32_t qraw[8];                                   // q of the current pass, one channel per dword
    {
        int ti0, tj0;
        pixel_of(min(wave, npass - 1), ti0, tj0);
        const uint32_t off = lane_chan + (uint32_t)ti0 * a.W + tj0;
#pragma unroll
        for (int e = 0; e < 8; ++e) qraw[e] = qbase[off + e * hw];
    }
    for (int pass = wave; pass < npass; pass += WAVES) {
        int ti, tj;
        const bool valid = pixel_of(pass, ti, tj);
        const uint32_t pix_off = lane_chan + (uint32_t)ti * a.W + tj;
        // q of this wave's next pass: issued now, consumed at the end of this pass
        uint32_t qnext[8];
        {
            int ti2, tj2;
            pixel_of(min(pass + WAVES, npass - 1), ti2, tj2);
            const uint32_t off = lane_chan + (uint32_t)ti2 * a.W + tj2;
#pragma unroll
            for (int e = 0; e < 8; ++e) qnext[e] = qbase[off + e * hw];
        }
        int coff[KS];
#pragma unroll
        for (int tx = 0; tx < KS; ++tx) coff[tx] = col_offset(tj + tx, g);
        const int row0 = ti * HC * 64;
        uint4_t kd[S];
#pragma unroll
        for (int t = 0; t < S; ++t)
            kd[t] = *(const uint4_t*)(kl + row0 + (t / KS) * HC * 64 + coff[t % KS]);

        uint32_t qpk[4];        // channel pairs (even low, odd high)
        float qodd[4];          // the odd channel alone, as float
#pragma unroll
        for (int y = 0; y < 4; ++y) {
            qpk[y] = qraw[2 * y] | (qraw[2 * y + 1] << 16);
            qodd[y] = __uint_as_float(qraw[2 * y + 1] << 16);
        }

        // ---- K side: logits.  Three taps (one window row) at a time so that the three
        // running sums interleave.
        float4_t acc1 = {0.0f, 0.0f, 0.0f, 0.0f};
        float idp[S];
#pragma unroll
        for (int ty = 0; ty < KS; ++ty) {
            float R[KS] = {0.0f, 0.0f, 0.0f};
            uint4_t bb[KS];
#pragma unroll
            for (int y = 0; y < 4; ++y) {
#pragma unroll
                for (int tx = 0; tx < KS; ++tx) {
                    const uint32_t kw = kd[ty * KS + tx][y];
                    R[tx] = dot2_bf16(qpk[y], kw, R[tx]);
                    const float O = qodd[y] * __uint_as_float(kw & 0xffff0000u);
                    bb[tx][y] = pack_bf16(R[tx], O);
                }
            }
#pragma unroll
            for (int tx = 0; tx < KS; ++tx) {
                acc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A1[ty * KS + tx],
                                                               __builtin_bit_cast(bf16x8_t, bb[tx]),
                                                               acc1, 0, 0, 0);
                idp[ty * KS + tx] = R[tx];
            }
        }
        // V taps: issue the LDS reads now, they land while the softmax runs
        uint4_t vd[S];
#pragma unroll
        for (int t = 0; t < S; ++t)
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
        for (int r = 0; r < 3; ++r) ascr[4 * r + g] = pr[r];
        __builtin_amdgcn_wave_barrier();
        float at[S];
#pragma unroll
        for (int t = 0; t < S; ++t) at[t] = ascr[t];
        uint2_t b2;
        b2[0] = pack_bf16(pr[0], pr[1]);
        b2[1] = pack_bf16(pr[2], 0.0f);
        const short4_t B2 = __builtin_bit_cast(short4_t, b2);

        // ---- V side: out[c] = sum_t v[c, p+t] * (a[t] + learned part); a[t] enters as the
        // MFMA's C operand, so the matrix core adds the two paths
        float o[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = 0.0f;
#pragma unroll
        for (int ty = 0; ty < KS; ++ty) {
            float4_t w[KS][2];
#pragma unroll
            for (int tx = 0; tx < KS; ++tx) {
                const int t = ty * KS + tx;
                const float4_t c4 = {at[t], at[t], at[t], at[t]};
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    w[tx][j] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(A2[t][j], B2, c4, 0, 0, 0);
            }
#pragma unroll
            for (int tx = 0; tx < KS; ++tx) {
                const int t = ty * KS + tx;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const uint32_t dw = vd[t][e >> 1];
                    const float vf = __uint_as_float((e & 1) ? (dw & 0xffff0000u) : (dw << 16));
                    o[e] = fmaf(w[tx][e >> 2][e & 3], vf, o[e]);
                }
            }
        }
        // ---- store
        if (valid) {
#pragma unroll
            for (int e = 0; e < 8; ++e) obase[pix_off + e * hw] = f32_to_bf16(o[e]);
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) qraw[e] = qnext[e];
    }
}

// ------------------------------------------------------------------ host side
struct TilePlan { int th, tw, n_tr, n_tc, v_base, a_base, lds_bytes; };

static TilePlan plan_tiles(const Problem& p)
{
    TilePlan t;
    const int budget = 77000;                              // bytes of LDS for the two halo tiles
    const int n_tc = p.W <= 64 ? 1 : (p.W + 63) / 64;
    t.tw = (p.W + n_tc - 1) / n_tc;
    int th_max = budget / (128 * (t.tw + 2)) - 2;
    if (th_max < 1) th_max = 1;
    int th = p.H < th_max ? p.H : th_max;
    const int n_tr = (p.H + th - 1) / th;
    t.th = (p.H + n_tr - 1) / n_tr;
    t.n_tr = (p.H + t.th - 1) / t.th;
    t.n_tc = (p.W + t.tw - 1) / t.tw;
    const int halo = (t.th + 2) * (t.tw + 2) * 64;
    t.v_base = halo + ((halo & 127) ? 0 : 64);             // K and V halos start 64 B apart mod 128
    t.a_base = (t.v_base + halo + 15) & ~15;
    t.lds_bytes = t.a_base + A_SCRATCH_BYTES;
    return t;
}

bool fwd_mfma_supported(const Problem& p)
{
    if (p.dtype != 1 || p.ksize != 3 || p.C != p.heads * D) return false;
    const TilePlan t = plan_tiles(p);
    const long n_blocks = (long)p.B * p.heads * t.n_tr * t.n_tc;
    return n_blocks < (1L << 30);
}

size_t fwd_mfma_workspace_bytes(const Problem& p)
{
    return fwd_mfma_supported(p) ? (size_t)p.heads * IMG_DWORDS * sizeof(uint32_t) : 0;
}

hipError_t launch_fwd_mfma(const Problem& p, const void* q, const void* k, const void* v,
                           const float* wk, const float* wv, const float* bias, void* out,
                           void* workspace, hipStream_t st)
{
    const TilePlan t = plan_tiles(p);
    uint32_t* image = (uint32_t*)workspace;
    hipLaunchKernelGGL(prep_weights_kernel, dim3(S, (unsigned)p.heads), dim3(256), 0, st,
                       wk, wv, bias, image);
    FwdArgs a;
    a.q = (const bf16_bits*)q; a.k = (const bf16_bits*)k; a.v = (const bf16_bits*)v;
    a.out = (bf16_bits*)out; a.image = image;
    a.B = p.B; a.H = p.H; a.W = p.W; a.C = p.C; a.heads = p.heads;
    a.th = t.th; a.tw = t.tw; a.n_tr = t.n_tr; a.n_tc = t.n_tc;
    a.v_base = t.v_base; a.a_base = t.a_base;
    a.vec_ok = (p.W % 8 == 0) && (((uintptr_t)k | (uintptr_t)v) % 16 == 0);
    a.scale_log2e = 1.44269504088896341f / sqrtf((float)D);
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void*)fwd_mfma_kernel,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const unsigned n_blocks = (unsigned)((long)p.B * p.heads * t.n_tr * t.n_tc);
    hipLaunchKernelGGL(fwd_mfma_kernel, dim3(n_blocks), dim3(THREADS), (size_t)t.lds_bytes, st, a);
    return hipGetLastError();
}

}  // namespace slide
