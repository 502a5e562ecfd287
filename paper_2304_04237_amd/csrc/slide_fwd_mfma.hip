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
// K side, per tap t: the products q[c]*k[c,p+t] are formed as a running sum over the
// lane's 8 channels with v_dot2_f32_bf16 (one operand masked to a single channel), the
// prefix sums P_0..P_7 are rounded to bf16 and fed to the MFMA against the DIFFERENCED
// learned weights (w_e - w_{e+1}), which gives sum_e G_e w_e by summation by parts; the
// last prefix P_7 is the lane's share of the exact shift-path logit for free.
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
// grid = heads, block = 256.  Reads the merged float32 kernels [C, 9, 3, 3] and writes
// the per-head operand image described above.
__global__ void __launch_bounds__(256)
prep_weights_kernel(const float* __restrict__ wk, const float* __restrict__ wv,
                    const float* __restrict__ bias, uint32_t* __restrict__ image)
{
    const int m = blockIdx.x;
    uint32_t* img = image + (long)m * IMG_DWORDS;
    // A1: dword y of lane (i, g) at tap t = learned K weights of channels 8g+2y, 8g+2y+1,
    // differenced along the lane's channel chain.
    for (int idx = threadIdx.x; idx < 9 * 64 * 4; idx += blockDim.x) {
        const int y = idx & 3, lane = (idx >> 2) & 63, t = idx >> 8;
        const int i = lane & 15, g = lane >> 4;
        const int s = shift_of_row(i);
        float d[2] = {0.0f, 0.0f};
        if (s >= 0) {
            for (int h = 0; h < 2; ++h) {
                const int e = 2 * y + h;
                const int c = m * D + 8 * g + e;
                float w0 = wk[((long)c * S + s) * S + t] - (s == t ? 1.0f : 0.0f);
                float w1 = 0.0f;
                if (e < 7) w1 = wk[((long)(c + 1) * S + s) * S + t] - (s == t ? 1.0f : 0.0f);
                d[h] = w0 - w1;
            }
        }
        img[IMG_A1 + idx] = pack_bf16(d[0], d[1]);
    }
    // A2: dword y of lane (i, g) at (tap t, half j) = learned V weights of channel
    // 8*(i/4) + 4j + (i%4) for the shifts of logit rows 4g+2y, 4g+2y+1.
    for (int idx = threadIdx.x; idx < 9 * 2 * 64 * 2; idx += blockDim.x) {
        const int y = idx & 1, lane = (idx >> 1) & 63, j = (idx >> 7) & 1, t = idx >> 8;
        const int i = lane & 15, g = lane >> 4;
        const int c = m * D + 8 * (i >> 2) + 4 * j + (i & 3);
        float d[2] = {0.0f, 0.0f};
        for (int h = 0; h < 2; ++h) {
            const int s = shift_of_row(4 * g + 2 * y + h);
            if (s >= 0) d[h] = wv[((long)c * S + s) * S + t] - (s == t ? 1.0f : 0.0f);
        }
        img[IMG_A2 + idx] = pack_bf16(d[0], d[1]);
    }
    if (threadIdx.x < 16) {
        const int s = shift_of_row(threadIdx.x);
        float b = -INFINITY;
        if (s >= 0) b = bias ? bias[m * S + s] * 1.44269504088896341f : 0.0f;
        img[IMG_BIAS + threadIdx.x] = __float_as_uint(b);
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
            const int o = idx & 3, tsel = (idx >> 2) & 1;
            const int rest = idx >> 3;
            const int hr = rest / NX, x = rest - hr * NX;
            const int gi = i0 - 1 + hr, gx = gx0 + 8 * x;
            const bool row_ok = (gi >= 0) && (gi < a.H);
            const bf16_bits* src = (tsel ? a.v : a.k) + head_base + ((long)(8 * o) * a.H + gi) * a.W + gx;
            uint4_t r[8];
            if (row_ok && a.vec_ok && gx >= 0 && gx + 8 <= a.W) {
#pragma unroll
                for (int e = 0; e < 8; ++e) r[e] = *(const uint4_t*)(src + e * HW);
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) {
#pragma unroll
                    for (int y = 0; y < 4; ++y) {
                        const int c0 = gx + 2 * y, c1 = c0 + 1;
                        uint32_t lo = (row_ok && c0 >= 0 && c0 < a.W) ? src[e * HW + 2 * y] : 0;
                        uint32_t hi = (row_ok && c1 >= 0 && c1 < a.W) ? src[e * HW + 2 * y + 1] : 0;
                        r[e][y] = lo | (hi << 16);
                    }
                }
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

    // q of the first pass
    auto pixel_of = [&](int pass, int& ti, int& tj) -> bool {
        int n = pass * 16 + p;
        const bool valid = n < npix;
        n = valid ? n : npix - 1;
        ti = (int)(((float)n + 0.5f) * inv_tw);
        tj = n - ti * tw_eff;
        return valid;
    };
    auto load_q = [&](int ti, int tj, uint32_t (&qd)[4]) {
        const bf16_bits* qp = a.q + head_base + ((long)(8 * g) * a.H + (i0 + ti)) * a.W + (j0 + tj);
#pragma unroll
        for (int y = 0; y < 4; ++y) {
            uint32_t lo = qp[(2 * y) * HW], hi = qp[(2 * y + 1) * HW];
            qd[y] = lo | (hi << 16);
        }
    };

    int ti, tj;
    uint32_t qd[4];
    if (wave < npass) {
        pixel_of(wave, ti, tj);
        load_q(ti, tj, qd);
    }
    for (int pass = wave; pass < npass; pass += WAVES) {
        const bool valid = pixel_of(pass, ti, tj);
        // prefetch q of this wave's next pass
        uint32_t qn[4] = {0, 0, 0, 0};
        if (pass + WAVES < npass) {
            int ti2, tj2;
            pixel_of(pass + WAVES, ti2, tj2);
            load_q(ti2, tj2, qn);
        }
        uint32_t qiso[8];
#pragma unroll
        for (int y = 0; y < 4; ++y) {
            qiso[2 * y] = qd[y] & 0x0000ffffu;
            qiso[2 * y + 1] = qd[y] & 0xffff0000u;
        }
        int coff[KS];
#pragma unroll
        for (int tx = 0; tx < KS; ++tx) coff[tx] = col_offset(tj + tx, g);
        const int row0 = ti * HC * 64;

        // ---- K side: logits
        float4_t acc1 = {0.0f, 0.0f, 0.0f, 0.0f};
        float idp[S];
#pragma unroll
        for (int t = 0; t < S; ++t) {
            const int ty = t / KS, tx = t % KS;
            const uint4_t kd = *(const uint4_t*)(kl + row0 + ty * HC * 64 + coff[tx]);
            float P = 0.0f;
            float pre[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                P = dot2_bf16(qiso[e], kd[e >> 1], P);
                pre[e] = P;
            }
            uint4_t bb;
#pragma unroll
            for (int y = 0; y < 4; ++y) bb[y] = pack_bf16(pre[2 * y], pre[2 * y + 1]);
            acc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A1[t], __builtin_bit_cast(bf16x8_t, bb),
                                                           acc1, 0, 0, 0);
            idp[t] = P;
        }
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
        uint2_t b2;
        b2[0] = pack_bf16(pr[0], pr[1]);
        b2[1] = pack_bf16(pr[2], 0.0f);
        const short4_t B2 = __builtin_bit_cast(short4_t, b2);

        // ---- V side: out[c] = sum_t v[c, p+t] * (a[t] + learned part)
        float o[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = 0.0f;
#pragma unroll
        for (int t = 0; t < S; ++t) {
            const int ty = t / KS, tx = t % KS;
            const uint4_t vd = *(const uint4_t*)(vl + row0 + ty * HC * 64 + coff[tx]);
            const float at = ascr[t];
            const float4_t zero = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const float4_t w = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(A2[t][j], B2, zero, 0, 0, 0);
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int e = 4 * j + r;
                    const uint32_t dw = vd[e >> 1];
                    const float vf = __uint_as_float((e & 1) ? (dw & 0xffff0000u) : (dw << 16));
                    o[e] = fmaf(w[r] + at, vf, o[e]);
                }
            }
        }
        // ---- store
        if (valid) {
            bf16_bits* op = a.out + head_base + ((long)(8 * g) * a.H + (i0 + ti)) * a.W + (j0 + tj);
#pragma unroll
            for (int e = 0; e < 8; ++e) op[e * HW] = f32_to_bf16(o[e]);
        }
#pragma unroll
        for (int y = 0; y < 4; ++y) qd[y] = qn[y];
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
    hipLaunchKernelGGL(prep_weights_kernel, dim3((unsigned)p.heads), dim3(256), 0, st,
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
