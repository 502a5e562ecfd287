// Kernel and bias gradients of Slide Attention on the matrix cores (gfx950): bf16
// activations, head size 32, 3x3 window, W a multiple of 8.
//
// What is computed (chain rule through Sec. 4.1-4.3; the paper gives no backward):
//     dwk[c,s,t] = scale * sum_{b,p} dl[b,m,s,p] * q[b,c,p] * k[b,c,p + off(t)]
//     dwv[c,s,t] =         sum_{b,p}  a[b,m,s,p] * dO[b,c,p] * v[b,c,p + off(t)]
//     dbias[m,s] =         sum_{b,p} dl[b,m,s,p]
// with a the attention weights, dl the logit gradients (both produced by the per-pixel
// backward kernel as halves [B, heads, 9, H, W]) and zero padding outside the map.
//
// Per channel this is a (9 taps) x (9 shifts) matrix whose contraction index is the pixel,
// so it runs as v_mfma_f32_16x16x32_f16 with K = 32 consecutive pixels of a row:
//     A[t, p] = q[c,p] * k[c, p + off(t)]      (two packed multiplies per dword, from LDS)
//     B[p, s] = dl[s, p]                        (shared by all channels of the head; 16 contiguous
//                                                bytes of the workspace per lane, read from
//                                                global memory one work unit ahead)
// The 16 rows of one product hold the three taps of one window row for four channels (12
// rows in use), so a wave's four channels take three products per 32 pixels and side, and
// q (dO) of a row is read once for the three window rows.
// Activations keep their natural layout (pixels contiguous), converted to half precision
// once while they are staged in LDS; q and dO are divided by 16 there so that products up
// to 2^20 stay finite, and the factor is restored with the final scale.  The tap windows
// of k and v start one pixel left or right of an aligned 8-pixel run; k and v are therefore
// staged twice, the second copy moved right by one pixel, so that every window is four
// dwords at a dword-aligned address (left: the moved copy at the run, middle: the plain copy
// at the run, right: the moved copy one dword on) and needs no shifting in registers.
// Each wave stages k, v, q, dO of its own four channels in its own part of LDS and shares
// nothing with the other waves of the block, so the loop over work units has no block
// barrier: the waves drift apart and one wave's staging overlaps another's matrix work.
// Accumulation is fp32 in the MFMA accumulators across all pixels a block visits; blocks
// write partial sums that a second kernel adds in a fixed order (reproducible results).
#include "slide_internal.h"
#include "slide_device.h"

namespace slide {
namespace dwpath {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef __attribute__((ext_vector_type(4))) float float4_t;
typedef __attribute__((ext_vector_type(4))) uint32_t uint4_t;

constexpr int S = 9, D = 32;
constexpr int WAVES = 8, THREADS = WAVES * 64;
constexpr int CPW = D / WAVES;        // channels per wave (4)
constexpr int R = 3;                  // rows of one work unit
constexpr int TW = 56;                // columns of one work unit (a multiple of 8)
constexpr int QP = 64;                // halves per staged row of q, dO
constexpr int KP = 96;                // halves per staged row of k, v: 8 margin, 56 data, 8 margin, 24 padding: the
                                      // (R + 2) rows of a channel then take 240 dwords, so the four channels of a
                                      // wave read their windows from four different quarters of the 64 LDS banks
constexpr float IN_SCALE = 0.0625f;   // q and dO are staged divided by 16

// LDS map (bytes)
constexpr int KH_BYTES = D * (R + 2) * KP * 2;            // 30720
constexpr int QH_BYTES = D * R * QP * 2;                  // 12288
constexpr int OFF_K = 0, OFF_V = OFF_K + KH_BYTES, OFF_Q = OFF_V + KH_BYTES,
              OFF_DO = OFF_Q + QH_BYTES, OFF_ZERO = OFF_DO + QH_BYTES,
              // K1, V1: k and v moved right by one pixel; they start 8 bytes off a 16-byte boundary
              // so that a window in them and the window at the same place in K, V use different banks
              OFF_K1 = OFF_ZERO + 256 + 8, OFF_V1 = OFF_K1 + KH_BYTES, LDS_BYTES = OFF_V1 + KH_BYTES + 8;
static_assert(LDS_BYTES <= 160 * 1024, "LDS");

struct Args {
    const bf16_bits* dout; const bf16_bits* q; const bf16_bits* k; const bf16_bits* v;
    const _Float16* attn; const _Float16* dl; // [B, heads, 9, H, W] as halves
    float* partial;                           // [NB][2][C][9][9]
    float* dbias_partial;                     // [NB][heads][9]
    int B, H, W, C, heads;
    int n_strips, n_ct, NB;
    int nbp, rows_pb;                         // streaming kernel: bands of rows per plane, rows per band
    float scale;
};

__device__ __forceinline__ half2_t as_half2(uint32_t x) { return __builtin_bit_cast(half2_t, x); }
__device__ __forceinline__ uint32_t as_dword(half2_t x) { return __builtin_bit_cast(uint32_t, x); }

// 8 consecutive bf16 (one 16-byte load) -> 8 halves, same order, times `mul`
__device__ __forceinline__ uint4_t bf16x8_to_half(uint4_t r, half2_t mul)
{
    uint4_t o;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const uint32_t d = r[j];
        const uint32_t pk = __builtin_bit_cast(uint32_t,
            __builtin_amdgcn_cvt_pkrtz(__uint_as_float(d << 16), __uint_as_float(d & 0xffff0000u)));
        o[j] = as_dword(as_half2(pk) * mul);
    }
    return o;
}

// one bf16 pattern -> half pattern, converted like bf16x8_to_half does (round toward zero)
__device__ __forceinline__ uint32_t bf16_to_half_bits(uint32_t b)
{
    return __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(__uint_as_float(b << 16), 0.0f)) & 0xffffu;
}

// The tap windows of the three window rows for one 32-pixel step: four consecutive dwords at
// rows 0, 1, 2 (KP halves apart) from each of two dword-aligned LDS addresses, as 8-byte
// two-dword reads.  Written in assembly because the compiler fuses such reads into 16-byte
// reads, and a 16-byte LDS read at an address that is not 16-byte aligned stalls the LDS pipe.
typedef __attribute__((ext_vector_type(2))) uint32_t uint2_t;
static_assert(KP * 2 / 4 == 48, "row stride of the k/v tiles in dwords, as spelled in the assembly below");
static_assert(OFF_K % 16 == 0 && OFF_V % 16 == 0 && OFF_K1 % 16 == 8 && OFF_V1 % 16 == 8, "bank phase of the copies");
__device__ __forceinline__ void lds_read_windows(uint32_t addr_k, uint32_t addr_v,
                                                 uint32_t (&k)[3][4], uint32_t (&v)[3][4])
{
    uint2_t k0a, k0b, k1a, k1b, k2a, k2b, v0a, v0b, v1a, v1b, v2a, v2b;
    asm volatile("ds_read2_b32 %0, %12 offset0:0 offset1:1\n\t"
                 "ds_read2_b32 %1, %12 offset0:2 offset1:3\n\t"
                 "ds_read2_b32 %6, %13 offset0:0 offset1:1\n\t"
                 "ds_read2_b32 %7, %13 offset0:2 offset1:3\n\t"
                 "ds_read2_b32 %2, %12 offset0:48 offset1:49\n\t"
                 "ds_read2_b32 %3, %12 offset0:50 offset1:51\n\t"
                 "ds_read2_b32 %8, %13 offset0:48 offset1:49\n\t"
                 "ds_read2_b32 %9, %13 offset0:50 offset1:51\n\t"
                 "ds_read2_b32 %4, %12 offset0:96 offset1:97\n\t"
                 "ds_read2_b32 %5, %12 offset0:98 offset1:99\n\t"
                 "ds_read2_b32 %10, %13 offset0:96 offset1:97\n\t"
                 "ds_read2_b32 %11, %13 offset0:98 offset1:99\n\t"
                 "s_waitcnt lgkmcnt(0)"
                 : "=&v"(k0a), "=&v"(k0b), "=&v"(k1a), "=&v"(k1b), "=&v"(k2a), "=&v"(k2b),
                   "=&v"(v0a), "=&v"(v0b), "=&v"(v1a), "=&v"(v1b), "=&v"(v2a), "=&v"(v2b)
                 : "v"(addr_k), "v"(addr_v)
                 : "memory");
    k[0][0] = k0a[0]; k[0][1] = k0a[1]; k[0][2] = k0b[0]; k[0][3] = k0b[1];
    k[1][0] = k1a[0]; k[1][1] = k1a[1]; k[1][2] = k1b[0]; k[1][3] = k1b[1];
    k[2][0] = k2a[0]; k[2][1] = k2a[1]; k[2][2] = k2b[0]; k[2][3] = k2b[1];
    v[0][0] = v0a[0]; v[0][1] = v0a[1]; v[0][2] = v0b[0]; v[0][3] = v0b[1];
    v[1][0] = v1a[0]; v[1][1] = v1a[1]; v[1][2] = v1b[0]; v[1][3] = v1b[1];
    v[2][0] = v2a[0]; v[2][1] = v2a[1]; v[2][2] = v2b[0]; v[2][3] = v2b[1];
}

__global__ void __launch_bounds__(THREADS, 2)
bwd_dw_kernel(const Args a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int i = lane & 15, g = lane >> 4;
    const int m = blockIdx.x / a.NB, j = blockIdx.x - m * a.NB;
    const long HW = (long)a.H * a.W;
    const int c0 = m * D + wave * CPW;            // first channel of this wave

    // zero all of LDS once: margins and the zero block stay zero for the whole kernel
    for (int o = tid * 16; o < LDS_BYTES; o += THREADS * 16) *(uint4_t*)(smem + o) = uint4_t{0u, 0u, 0u, 0u};

    // Rows of the products: one product covers one window row ty of this wave's four channels,
    // row i < 12 = (channel cc = i / 3, window column tx = i % 3), i.e. tap t = 3 ty + tx; rows
    // 12..15 are masked (zero q), except that row 12 of wave 0's first product sums dl.
    constexpr int ROWS = 3 * CPW;
    const int lcc = (i < ROWS) ? i / 3 : 0, tx = (i < ROWS) ? i - 3 * (i / 3) : 0;
    // The tap window of k (v) is the aligned 8-pixel run moved by tx-1 pixels: four dwords of
    // the moved copy at the run (tx = 0), of the plain copy at the run (tx = 1), or of the moved
    // copy one dword past the run (tx = 2).
    const int kwin_off = (((wave * CPW + lcc) * (R + 2)) * KP + 8 + 8 * g) * 2 + (tx == 2 ? 4 : 0) +
                         (tx == 1 ? 0 : OFF_K1 - OFF_K);          // + (ty + r)*KP*2 + 64*h; the same offset from OFF_V for v
    const int q_off = (i < ROWS) ? (((wave * CPW + lcc) * R) * QP + 8 * g) * 2 : -1;   // + r*QP*2 + 64*h; -1: masked row, read zeros

    float4_t acc_k[3], acc_v[3];                  // one accumulator per window row
#pragma unroll
    for (int ty = 0; ty < 3; ++ty) { acc_k[ty] = float4_t{0, 0, 0, 0}; acc_v[ty] = float4_t{0, 0, 0, 0}; }
    const half2_t one2 = {(_Float16)1.0f, (_Float16)1.0f};
    const half2_t in2 = {(_Float16)IN_SCALE, (_Float16)IN_SCALE};
    const bool bias_lane = (wave == 0) && (i == ROWS);            // row 12 of the first product sums dl

    const int n_units = a.B * a.n_strips * a.n_ct;

    // Geometry of a work unit (uniform): one strip of R rows x TW columns of one batch item.
    struct Unit { int b, i0, j0, rows_eff, cols_eff, nxc; };
    auto unit_of = [&](int u) {
        Unit t;
        const int ct = u % a.n_ct, us = u / a.n_ct;
        const int strip = us % a.n_strips;
        t.b = us / a.n_strips;
        t.i0 = strip * R; t.j0 = ct * TW;
        t.rows_eff = min(R, a.H - t.i0); t.cols_eff = min(TW, a.W - t.j0);
        t.nxc = t.cols_eff >> 3;                                  // 16-byte chunks per row
        return t;
    };

    // Staging registers of one unit.  The loads of the next unit are issued before the
    // current unit is accumulated and are converted into LDS afterwards, so global latency
    // hides behind the matrix work.  Slots: k/v chunks, k/v halo columns, q/dO chunks of this
    // wave's channels (wave-private LDS regions).
    constexpr int N_KV = CPW * (R + 2) * 8, KV_SLOTS = (2 * N_KV + 63) / 64;        // 5
    constexpr int N_HC = CPW * (R + 2) * 2, HC_SLOTS = (2 * N_HC + 63) / 64;        // 2
    constexpr int N_Q = CPW * R * 8, Q_SLOTS = (2 * N_Q + 63) / 64;                 // 3
    uint4_t pre_kv[KV_SLOTS], pre_q[Q_SLOTS];
    uint32_t pre_kp[KV_SLOTS];                  // the pixel left of each k/v chunk (for the moved copy)
    uint32_t pre_hc[HC_SLOTS];

    auto issue_loads = [&](const Unit& t) {
#pragma unroll
        for (int sl = 0; sl < KV_SLOTS; ++sl) {
            const int idx = sl * 64 + lane;
            const int tsel = idx >= N_KV, id = idx - tsel * N_KV;
            const int x = id & 7, rj = id >> 3;
            const int cc = rj / (R + 2), hr = rj - cc * (R + 2);
            const int gi = t.i0 - 1 + hr;
            pre_kv[sl] = uint4_t{0u, 0u, 0u, 0u};
            pre_kp[sl] = 0u;
            if (idx < 2 * N_KV && x < t.nxc && gi >= 0 && gi < a.H) {
                const bf16_bits* src = (tsel ? a.v : a.k) + ((long)t.b * a.C + c0 + cc) * HW + (long)gi * a.W + t.j0 + 8 * x;
                pre_kv[sl] = *(const uint4_t*)src;
                if (t.j0 + 8 * x > 0) pre_kp[sl] = src[-1];
            }
        }
#pragma unroll
        for (int sl = 0; sl < HC_SLOTS; ++sl) {
            const int idx = sl * 64 + lane;
            const int tsel = idx >= N_HC, id = idx - tsel * N_HC;
            const int side = id & 1, rj = id >> 1;
            const int cc = rj / (R + 2), hr = rj - cc * (R + 2);
            const int gi = t.i0 - 1 + hr, gj = side ? t.j0 + t.cols_eff : t.j0 - 1;
            pre_hc[sl] = 0u;
            if (idx < 2 * N_HC && gi >= 0 && gi < a.H && gj >= 0 && gj < a.W)
                pre_hc[sl] = ((tsel ? a.v : a.k) + ((long)t.b * a.C + c0 + cc) * HW)[(long)gi * a.W + gj];
        }
#pragma unroll
        for (int sl = 0; sl < Q_SLOTS; ++sl) {
            const int idx = sl * 64 + lane;
            const int tsel = idx >= N_Q, id = idx - tsel * N_Q;
            const int x = id & 7, rj = id >> 3;
            const int cc = rj / R, r = rj - cc * R;
            pre_q[sl] = uint4_t{0u, 0u, 0u, 0u};
            if (idx < 2 * N_Q && x < t.nxc && r < t.rows_eff) {
                const bf16_bits* src = (tsel ? a.dout : a.q) + ((long)t.b * a.C + c0 + cc) * HW + (long)(t.i0 + r) * a.W + t.j0 + 8 * x;
                pre_q[sl] = *(const uint4_t*)src;
            }
        }
    };

    auto commit_to_lds = [&](const Unit& t) {
#pragma unroll
        for (int sl = 0; sl < KV_SLOTS; ++sl) {
            const int idx = sl * 64 + lane;
            const int tsel = idx >= N_KV, id = idx - tsel * N_KV;
            const int x = id & 7, rj = id >> 3;
            const int cc = rj / (R + 2), hr = rj - cc * (R + 2);
            // slots past the tile keep stale (finite) data: they only ever meet a zero q
            if (idx < 2 * N_KV && x < t.nxc) {
                const uint4_t val = bf16x8_to_half(pre_kv[sl], one2);
                const int at = (((wave * CPW + cc) * (R + 2) + hr) * KP + 8 + 8 * x) * 2;
                *(uint4_t*)(smem + (tsel ? OFF_V : OFF_K) + at) = val;
                // the copy moved right by one pixel: (left neighbour, pixels 0..6) here, pixel 7
                // opens the next chunk (written there by that chunk's lane, or below at the end)
                const uint32_t left = bf16_to_half_bits(pre_kp[sl]);
                uint4_t mv;
                mv[0] = (val[0] << 16) | left;
#pragma unroll
                for (int y = 1; y < 4; ++y) mv[y] = __builtin_amdgcn_alignbit(val[y], val[y - 1], 16);
                *(uint2_t*)(smem + (tsel ? OFF_V1 : OFF_K1) + at) = uint2_t{mv[0], mv[1]};
                *(uint2_t*)(smem + (tsel ? OFF_V1 : OFF_K1) + at + 8) = uint2_t{mv[2], mv[3]};
                if (x == t.nxc - 1)
                    *(uint16_t*)(smem + (tsel ? OFF_V1 : OFF_K1) + at + 16) = (uint16_t)(val[3] >> 16);
            }
        }
#pragma unroll
        for (int sl = 0; sl < HC_SLOTS; ++sl) {
            const int idx = sl * 64 + lane;
            const int tsel = idx >= N_HC, id = idx - tsel * N_HC;
            const int side = id & 1, rj = id >> 1;
            const int cc = rj / (R + 2), hr = rj - cc * (R + 2);
            if (idx < 2 * N_HC) {
                const uint16_t hv = (uint16_t)bf16_to_half_bits(pre_hc[sl]);
                const int at = (((wave * CPW + cc) * (R + 2) + hr) * KP + (side ? 8 + t.cols_eff : 7)) * 2;
                *(uint16_t*)(smem + (tsel ? OFF_V : OFF_K) + at) = hv;
                // moved copy: the right halo column sits one further right; the left one is the
                // "left neighbour" of chunk 0
                if (side) *(uint16_t*)(smem + (tsel ? OFF_V1 : OFF_K1) + at + 2) = hv;
            }
        }
#pragma unroll
        for (int sl = 0; sl < Q_SLOTS; ++sl) {
            const int idx = sl * 64 + lane;
            const int tsel = idx >= N_Q, id = idx - tsel * N_Q;
            const int x = id & 7, rj = id >> 3;
            const int cc = rj / R, r = rj - cc * R;
            if (idx < 2 * N_Q)
                *(uint4_t*)(smem + (tsel ? OFF_DO : OFF_Q) + (((wave * CPW + cc) * R + r) * QP + 8 * x) * 2) =
                    bf16x8_to_half(pre_q[sl], in2);
        }
    };

    // dl and a enter as the B operands straight from global memory: lane (n, g) needs the 8
    // consecutive pixels 32h + 8g .. +7 of shift n, which are 16 contiguous bytes of the planar
    // workspace.  All 8 waves of a block read the same addresses (served by the caches).  The
    // operand of a step is fetched one unit ahead, into the registers that the step has just
    // used, so nothing of a unit is shared between the waves through LDS and they need not
    // wait for each other: no block barrier inside the loop.
    uint4_t Bop[R][2][2];
    // address = one base per (unit, row, half) that is the same for the whole wave + a byte
    // offset per lane that never changes (9 * H * W halves stay far below 2^31 bytes)
    const uint32_t b_lane = (uint32_t)(((long)(i < S ? i : 0) * HW + 8 * g) * 2);
    auto load_B = [&](const Unit& t, int r, int h, uint4_t (&dst)[2]) {
        dst[0] = uint4_t{0u, 0u, 0u, 0u}; dst[1] = uint4_t{0u, 0u, 0u, 0u};
        const long at = ((long)t.b * a.heads + m) * S * HW + (long)(t.i0 + r) * a.W + t.j0 + 32 * h;   // uniform
        if (i < S && r < t.rows_eff && 32 * h + 8 * g < t.cols_eff) {
            dst[0] = *(const uint4_t*)((const char*)(a.dl + at) + b_lane);
            dst[1] = *(const uint4_t*)((const char*)(a.attn + at) + b_lane);
        }
    };

    __syncthreads();                           // LDS is zeroed
    // A block walks through consecutive units (down the strips of a plane): the k/v halo rows
    // that two neighbouring strips share are then read again by the same compute unit one unit
    // later, out of the caches instead of from HBM.
    const int per_block = (n_units + a.NB - 1) / a.NB;
    const int u_begin = j * per_block, u_end = min(u_begin + per_block, n_units);
    if (u_begin < u_end) {
        const Unit t0 = unit_of(u_begin);
        issue_loads(t0);
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int h = 0; h < 2; ++h) load_B(t0, r, h, Bop[r][h]);
    }
    for (int u = u_begin; u < u_end; ++u) {
        const Unit t = unit_of(u);
        const bool has_next = u + 1 < u_end;
        const Unit tn = unit_of(has_next ? u + 1 : u);
        commit_to_lds(t);                      // this wave's own regions: its reads of the previous unit are done
        if (has_next) issue_loads(tn);
        const int rows_eff = t.rows_eff, cols_eff = t.cols_eff;

        // ---- accumulate: for every 32-pixel chunk, one MFMA per window row and side
#pragma unroll
        for (int r = 0; r < R; ++r) {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                if (r < rows_eff && 32 * h < cols_eff) {
                    const half8_t Bdl = __builtin_bit_cast(half8_t, Bop[r][h][0]);
                    const half8_t Ba = __builtin_bit_cast(half8_t, Bop[r][h][1]);
                    // q and dO of the row's channel: the same for the three window rows
                    const int qo = (q_off >= 0) ? q_off + r * QP * 2 + 64 * h : -1;
                    const uint4_t qv = *(const uint4_t*)(smem + (qo >= 0 ? OFF_Q + qo : OFF_ZERO));
                    const uint4_t dv = *(const uint4_t*)(smem + (qo >= 0 ? OFF_DO + qo : OFF_ZERO));
                    uint32_t kw[3][4], vw[3][4];
                    {
                        const int ko = kwin_off + r * KP * 2 + 64 * h;
                        lds_read_windows((uint32_t)(uintptr_t)(smem + OFF_K + ko),
                                         (uint32_t)(uintptr_t)(smem + OFF_V + ko), kw, vw);
                    }
#pragma unroll
                    for (int ty = 0; ty < 3; ++ty) {
                        uint4_t ak, av;
#pragma unroll
                        for (int y = 0; y < 4; ++y) {
                            ak[y] = as_dword(as_half2(qv[y]) * as_half2(kw[ty][y]));
                            av[y] = as_dword(as_half2(dv[y]) * as_half2(vw[ty][y]));
                        }
                        if (ty == 0 && wave == 0) {
#pragma unroll
                            for (int y = 0; y < 4; ++y) ak[y] = bias_lane ? as_dword(one2) : ak[y];
                        }
                        acc_k[ty] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8_t, ak), Bdl, acc_k[ty], 0, 0, 0);
                        acc_v[ty] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8_t, av), Ba, acc_v[ty], 0, 0, 0);
                        if (ty == 1) __builtin_amdgcn_sched_barrier(0);   // keep two products in flight, not three
                    }
                }
                if (has_next) load_B(tn, r, h, Bop[r][h]);    // the same step of the next unit
            }
        }
    }

    // ---- partial sums of this block.  Result register r of lane (n, g) is row 4g + r =
    // (channel, window column), column s = n of the 16x16 product of window row ty.
    const int n = i;
    const float out_scale = 1.0f / IN_SCALE;
    if (n < S) {
        const long side = (long)a.C * S * S;
        float* base = a.partial + (long)j * 2 * side;
#pragma unroll
        for (int ty = 0; ty < 3; ++ty) {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int row = 4 * g + r;
                if (row < ROWS) {
                    const int cc = row / 3, t = 3 * ty + row - 3 * cc;
                    base[((long)(c0 + cc) * S + n) * S + t] = acc_k[ty][r] * (a.scale * out_scale);
                    base[side + ((long)(c0 + cc) * S + n) * S + t] = acc_v[ty][r] * out_scale;
                }
            }
        }
        if (wave == 0 && g == 3)                                   // row 12 = 4*3 + 0
            a.dbias_partial[((long)j * a.heads + m) * S + n] = acc_k[0][0];
    }
}

// ------------------------------------------------------------------ streaming form
// The same products for maps of 32..56 columns (one column tile), with the data movement of the
// streaming forward: a block of 8 product waves (four channels each, as above) and 4 mover
// waves walks down bands of rows of (batch, head) planes, one row per epoch.  The movers stage
// every row once: 16-byte loads into registers two epochs ahead (mover j: channels 8j..8j+7 of
// k, v, q, dO; a lane owns one 8-pixel piece of one channel's row), conversion to halves, and
// the rows go into rings in LDS in the layout of the kernel above (k and v: four row slots per
// channel, plain and moved by one pixel; q and dO: two row slots).  The product waves read
// the three window rows of a step through one address per row (ring slots wrap).  One block
// barrier per row.  Accumulators live across all bands a block visits; partial sums as above.
namespace ring {
constexpr int RK = 4, RQ = 2;                 // ring slots per channel: k, v / q, dO
constexpr int MOVERS = 4, THREADS_R = (WAVES + MOVERS) * 64;
// halves per channel in a ring: its row slots plus 32, so that the channel stride is 16 dwords
// past a multiple of the 64 banks and the four channels of a product wave (and the eight of a
// mover) use different quarters of the banks
constexpr int KCH = RK * KP + 32, QCH = RQ * QP + 32;
constexpr int K_BYTES = D * KCH * 2;          // 26624
constexpr int Q_BYTES = D * QCH * 2;          // 10240
// (the moved copies start 8 banks after a multiple of 64: within the 16 banks of a channel the
// plain windows of two lane groups use the first eight, the moved windows the rest)
constexpr int OFF_K = 0, OFF_V = OFF_K + K_BYTES, OFF_K1 = OFF_V + K_BYTES + 32, OFF_V1 = OFF_K1 + K_BYTES,
              OFF_Q = OFF_V1 + K_BYTES + 32, OFF_DO = OFF_Q + Q_BYTES, OFF_ZERO = OFF_DO + Q_BYTES,
              LDS_BYTES = OFF_ZERO + 256;
static_assert(K_BYTES % 256 == 0 && OFF_K % 256 == 0 && OFF_K1 % 256 == 32 && OFF_V1 % 256 == 32 && OFF_Q % 16 == 0, "bank phase of the copies");
static_assert(LDS_BYTES <= 160 * 1024, "LDS");

// the tap windows of the three window rows of a step: four consecutive dwords from each of
// three dword-aligned LDS addresses per tensor, as 8-byte two-dword reads (see lds_read_windows)
__device__ __forceinline__ void lds_read_windows3(const uint32_t (&ak)[3], const uint32_t (&av)[3],
                                                  uint32_t (&k)[3][4], uint32_t (&v)[3][4])
{
    uint2_t k0a, k0b, k1a, k1b, k2a, k2b, v0a, v0b, v1a, v1b, v2a, v2b;
    asm volatile("ds_read2_b32 %0, %12 offset0:0 offset1:1\n\t"
                 "ds_read2_b32 %1, %12 offset0:2 offset1:3\n\t"
                 "ds_read2_b32 %6, %15 offset0:0 offset1:1\n\t"
                 "ds_read2_b32 %7, %15 offset0:2 offset1:3\n\t"
                 "ds_read2_b32 %2, %13 offset0:0 offset1:1\n\t"
                 "ds_read2_b32 %3, %13 offset0:2 offset1:3\n\t"
                 "ds_read2_b32 %8, %16 offset0:0 offset1:1\n\t"
                 "ds_read2_b32 %9, %16 offset0:2 offset1:3\n\t"
                 "ds_read2_b32 %4, %14 offset0:0 offset1:1\n\t"
                 "ds_read2_b32 %5, %14 offset0:2 offset1:3\n\t"
                 "ds_read2_b32 %10, %17 offset0:0 offset1:1\n\t"
                 "ds_read2_b32 %11, %17 offset0:2 offset1:3\n\t"
                 "s_waitcnt lgkmcnt(0)"
                 : "=&v"(k0a), "=&v"(k0b), "=&v"(k1a), "=&v"(k1b), "=&v"(k2a), "=&v"(k2b),
                   "=&v"(v0a), "=&v"(v0b), "=&v"(v1a), "=&v"(v1b), "=&v"(v2a), "=&v"(v2b)
                 : "v"(ak[0]), "v"(ak[1]), "v"(ak[2]), "v"(av[0]), "v"(av[1]), "v"(av[2])
                 : "memory");
    k[0][0] = k0a[0]; k[0][1] = k0a[1]; k[0][2] = k0b[0]; k[0][3] = k0b[1];
    k[1][0] = k1a[0]; k[1][1] = k1a[1]; k[1][2] = k1b[0]; k[1][3] = k1b[1];
    k[2][0] = k2a[0]; k[2][1] = k2a[1]; k[2][2] = k2b[0]; k[2][3] = k2b[1];
    v[0][0] = v0a[0]; v[0][1] = v0a[1]; v[0][2] = v0b[0]; v[0][3] = v0b[1];
    v[1][0] = v1a[0]; v[1][1] = v1a[1]; v[1][2] = v1b[0]; v[1][3] = v1b[1];
    v[2][0] = v2a[0]; v[2][1] = v2a[1]; v[2][2] = v2b[0]; v[2][3] = v2b[1];
}

// all LDS operations of this wave are done, then the block barrier; loads from global memory
// stay in flight across it (__syncthreads would wait for them: the rows fetched two epochs ahead)
__device__ __forceinline__ void row_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// The tap windows of ONE row for both steps (pixels 0..31 and 32..63) and both tensors: a row's
// windows are read once and serve as the bottom, middle and top window row of three successive
// rows of products.
struct RowWindows { uint32_t k[2][4], v[2][4]; };
__device__ __forceinline__ void lds_read_row_windows(uint32_t ak, uint32_t av, RowWindows& w)
{
    uint2_t k0a, k0b, k1a, k1b, v0a, v0b, v1a, v1b;
    asm volatile("ds_read2_b32 %0, %8 offset0:0 offset1:1\n\t"
                 "ds_read2_b32 %1, %8 offset0:2 offset1:3\n\t"
                 "ds_read2_b32 %4, %9 offset0:0 offset1:1\n\t"
                 "ds_read2_b32 %5, %9 offset0:2 offset1:3\n\t"
                 "ds_read2_b32 %2, %8 offset0:16 offset1:17\n\t"
                 "ds_read2_b32 %3, %8 offset0:18 offset1:19\n\t"
                 "ds_read2_b32 %6, %9 offset0:16 offset1:17\n\t"
                 "ds_read2_b32 %7, %9 offset0:18 offset1:19\n\t"
                 "s_waitcnt lgkmcnt(0)"
                 : "=&v"(k0a), "=&v"(k0b), "=&v"(k1a), "=&v"(k1b), "=&v"(v0a), "=&v"(v0b), "=&v"(v1a), "=&v"(v1b)
                 : "v"(ak), "v"(av)
                 : "memory");
    w.k[0][0] = k0a[0]; w.k[0][1] = k0a[1]; w.k[0][2] = k0b[0]; w.k[0][3] = k0b[1];
    w.k[1][0] = k1a[0]; w.k[1][1] = k1a[1]; w.k[1][2] = k1b[0]; w.k[1][3] = k1b[1];
    w.v[0][0] = v0a[0]; w.v[0][1] = v0a[1]; w.v[0][2] = v0b[0]; w.v[0][3] = v0b[1];
    w.v[1][0] = v1a[0]; w.v[1][1] = v1a[1]; w.v[1][2] = v1b[0]; w.v[1][3] = v1b[1];
}

__global__ void __launch_bounds__(THREADS_R)
bwd_dw_ring_kernel(const Args a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool mover = wave >= WAVES;
    const int i = lane & 15, g = lane >> 4;
    const int m = blockIdx.x / a.NB, j = blockIdx.x - m * a.NB;
    const int H = a.H, W = a.W;
    const long HW = (long)H * W;
    const int NXC = W >> 3;

    // zero all of LDS once: margins and the zero block stay zero for the whole kernel
    for (int o = tid * 16; o < LDS_BYTES; o += THREADS_R * 16) *(uint4_t*)(smem + o) = uint4_t{0u, 0u, 0u, 0u};
    __syncthreads();

    const int n_items = a.B * a.nbp;                               // bands of this head over the batch
    const half2_t one2 = {(_Float16)1.0f, (_Float16)1.0f};
    const half2_t in2 = {(_Float16)IN_SCALE, (_Float16)IN_SCALE};

    if (mover) {
        // ---- movers: lane = (channel mv * 8 + lane / 8, piece lane % 8) of a row of k, v, q, dO
        const int mv = wave - WAVES;
        const int ch = mv * 8 + (lane >> 3), x = lane & 7;
        const bool has = x < NXC;
        const int xs = has ? x : 0;                                // (idle lanes load piece 0 and store nothing)
        struct Stage { uint4_t k, v, q, d; uint32_t kl, vl; };
        __builtin_amdgcn_s_setprio(3);                             // the movers go ahead of the product waves of their SIMD
        for (int item = j; item < n_items; item += a.NB) {
            const int b = item / a.nbp, part = item - b * a.nbp;
            const int y0 = part * a.rows_pb, nr = min(a.rows_pb, H - y0);
            const long ch_base = ((long)b * a.C + m * D + ch) * HW + 8 * xs;
            // stage s: row y0 + s + 2 of k and v into slot (s + 2) % 4, row y0 + s + 1 of q and dO
            // into slot (s + 1) % 2.  Every load is unconditional (rows outside the map are
            // clamped and written as zeros): straight-line code, in which the compiler counts
            // the loads in flight.
            auto load_stage = [&](int s, Stage& r) {
                const int ykv = min(max(y0 + s + 2, 0), H - 1), yq = min(max(y0 + s + 1, 0), H - 1);
                const bf16_bits* pk = a.k + ch_base + (long)ykv * W;
                const bf16_bits* pv = a.v + ch_base + (long)ykv * W;
                r.k = *(const uint4_t*)pk; r.v = *(const uint4_t*)pv;
                r.kl = pk[xs > 0 ? -1 : 0]; r.vl = pv[xs > 0 ? -1 : 0];
                r.q = *(const uint4_t*)(a.q + ch_base + (long)yq * W);
                r.d = *(const uint4_t*)(a.dout + ch_base + (long)yq * W);
            };
            auto write_kv = [&](int off_plain, int off_moved, int slot, bool in_map, uint4_t raw, uint32_t left_raw) {
                uint4_t val = bf16x8_to_half(raw, one2);
                uint32_t left = (x > 0) ? bf16_to_half_bits(left_raw) : 0u;
                if (!in_map) { val = uint4_t{0u, 0u, 0u, 0u}; left = 0u; }
                const int at = (ch * KCH + slot * KP + 8 + 8 * x) * 2;
                *(uint4_t*)(smem + off_plain + at) = val;
                // the copy moved right by one pixel: (left neighbour, pixels 0..6) here, pixel 7
                // opens the next piece (written by that piece's lane, or below at the row's end)
                uint4_t mvd;
                mvd[0] = (val[0] << 16) | left;
#pragma unroll
                for (int y = 1; y < 4; ++y) mvd[y] = __builtin_amdgcn_alignbit(val[y], val[y - 1], 16);
                *(uint2_t*)(smem + off_moved + at) = uint2_t{mvd[0], mvd[1]};
                *(uint2_t*)(smem + off_moved + at + 8) = uint2_t{mvd[2], mvd[3]};
                if (x == NXC - 1) *(uint16_t*)(smem + off_moved + at + 16) = (uint16_t)(val[3] >> 16);
            };
            auto write_stage = [&](int s, const Stage& r) {
                if (!has) return;
                const int ykv = y0 + s + 2, yq = y0 + s + 1;
                const bool kv_in = ykv >= 0 && ykv < H;
                const int slot = (s + 2) & 3;
                write_kv(OFF_K, OFF_K1, slot, kv_in, r.k, r.kl);
                write_kv(OFF_V, OFF_V1, slot, kv_in, r.v, r.vl);
                if (s + 1 >= 0 && s + 1 < nr) {                       // (rows of the band only)
                    const int at = (ch * QCH + ((s + 1) & 1) * QP + 8 * x) * 2;
                    *(uint4_t*)(smem + OFF_Q + at) = bf16x8_to_half(r.q, in2);
                    *(uint4_t*)(smem + OFF_DO + at) = bf16x8_to_half(r.d, in2);
                }
            };
            // Four register sets (stage s in set s % 4): a row is fetched four epochs before it is
            // written.  The epoch loop is unrolled by four and runs a multiple of twelve epochs (the
            // product waves pass the same barriers; a stage past the band writes a slot nobody reads).
            Stage s0_, s1_, s2_, s3_;
            load_stage(-3, s1_); load_stage(-2, s2_); load_stage(-1, s3_); load_stage(0, s0_);
            write_stage(-3, s1_); load_stage(1, s1_);
            write_stage(-2, s2_); load_stage(2, s2_);
            write_stage(-1, s3_); load_stage(3, s3_);
            row_barrier();                                         // rows -1, 0, 1 of k and v, row 0 of q and dO are in place
            const int nr12 = ((nr + 11) / 12) * 12;                  // (a multiple of four and of the product waves' six)
            for (int r = 0; r < nr12; r += 4) {
                write_stage(r, s0_); load_stage(r + 4, s0_);
                row_barrier();
                write_stage(r + 1, s1_); load_stage(r + 5, s1_);
                row_barrier();
                write_stage(r + 2, s2_); load_stage(r + 6, s2_);
                row_barrier();
                write_stage(r + 3, s3_); load_stage(r + 7, s3_);
                row_barrier();
            }
        }
        return;
    }

    // ---- product waves
    const int c0 = m * D + wave * CPW;
    constexpr int ROWS = 3 * CPW;
    const int lcc = (i < ROWS) ? i / 3 : 0, tx = (i < ROWS) ? i - 3 * (i / 3) : 0;
    const int chl = wave * CPW + lcc;                              // channel of the head that row i belongs to
    // byte offset of the lane's tap window inside ring slot 0 of its channel: + slot * KP * 2 + 64 * h
    const uint32_t kwin = (uint32_t)(uintptr_t)smem +
                          (uint32_t)((chl * KCH + 8 + 8 * g) * 2 + (tx == 2 ? 4 : 0) + (tx == 1 ? OFF_K : OFF_K1));
    const int q_off = (i < ROWS) ? (chl * QCH + 8 * g) * 2 : -1;   // + slot * QP * 2 + 64 * h; -1: masked row, read zeros
    float4_t acc_k[3], acc_v[3];
#pragma unroll
    for (int ty = 0; ty < 3; ++ty) { acc_k[ty] = float4_t{0, 0, 0, 0}; acc_v[ty] = float4_t{0, 0, 0, 0}; }
    const bool bias_lane = (wave == 0) && (i == ROWS);            // row 12 of the first product sums dl
    const uint32_t b_lane = (uint32_t)(((long)(i < S ? i : 0) * HW + 8 * g) * 2);
    const bool second_half = W > 32;

    for (int item = j; item < n_items; item += a.NB) {
        const int b = item / a.nbp, part = item - b * a.nbp;
        const int y0 = part * a.rows_pb, nr = min(a.rows_pb, H - y0);
        // dl and a of a row as the B operands, straight from global memory one row ahead: lane
        // (n, g) holds the 8 pixels 32 h + 8 g .. of shift n
        uint4_t Bop[2][2];
        // (unconditional loads, so that the compiler counts them exactly and waits where they are
        // used: lanes and pieces without data read a valid address and are zeroed at use)
        auto load_B = [&](int r, uint4_t (&dst)[2][2]) {
            const int yr = min(y0 + r, H - 1);
            const long at = ((long)b * a.heads + m) * S * HW + (long)yr * W;   // uniform
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int px = (32 * h + 8 * g < W) ? 32 * h : 0;
                dst[h][0] = *(const uint4_t*)((const char*)(a.dl + at + px) + b_lane);
                dst[h][1] = *(const uint4_t*)((const char*)(a.attn + at + px) + b_lane);
            }
        };
        // one row of products: window rows r - 1 (lo) and r (mid) are held from the two rows before,
        // row r + 1 (hi) is read here; against the row's dl / a operands
        auto read_row = [&](int rho, RowWindows& w) {
            const uint32_t ak = kwin + (uint32_t)((rho & 3) * (KP * 2));      // row rho sits in slot rho % 4
            lds_read_row_windows(ak, ak + (OFF_V - OFF_K), w);
        };
        auto row_products = [&](int r, const RowWindows& lo, const RowWindows& mid, RowWindows& hi, const uint4_t (&Bq)[2][2]) {
            read_row(r + 1, hi);
            const int qs = q_off >= 0 ? q_off + (r & 1) * (QP * 2) : -1;
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                if (h == 0 || second_half) {
                    const bool b_ok = i < S && 32 * h + 8 * g < W;
                    const uint4_t z4 = {0u, 0u, 0u, 0u};
                    const half8_t Bdl = __builtin_bit_cast(half8_t, b_ok ? Bq[h][0] : z4);
                    const half8_t Ba = __builtin_bit_cast(half8_t, b_ok ? Bq[h][1] : z4);
                    const uint4_t qv = *(const uint4_t*)(smem + (qs >= 0 ? OFF_Q + qs + 64 * h : OFF_ZERO));
                    const uint4_t dv = *(const uint4_t*)(smem + (qs >= 0 ? OFF_DO + qs + 64 * h : OFF_ZERO));
#pragma unroll
                    for (int ty = 0; ty < 3; ++ty) {
                        const RowWindows& w = ty == 0 ? lo : (ty == 1 ? mid : hi);
                        uint4_t pk, pv;
#pragma unroll
                        for (int y = 0; y < 4; ++y) {
                            pk[y] = as_dword(as_half2(qv[y]) * as_half2(w.k[h][y]));
                            pv[y] = as_dword(as_half2(dv[y]) * as_half2(w.v[h][y]));
                        }
                        if (ty == 0 && wave == 0) {
#pragma unroll
                            for (int y = 0; y < 4; ++y) pk[y] = bias_lane ? as_dword(one2) : pk[y];
                        }
                        acc_k[ty] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8_t, pk), Bdl, acc_k[ty], 0, 0, 0);
                        acc_v[ty] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8_t, pv), Ba, acc_v[ty], 0, 0, 0);
                    }
                }
            }
        };
        // Two operand sets (even rows in Bop, odd rows in B1, fetched one row ahead) and three sets
        // of window rows that rotate: the loop is unrolled by six and runs a multiple of twelve
        // epochs (the movers' loop is unrolled by four; both pass the same barriers).
        uint4_t B1[2][2];
        RowWindows wa, wb, wc;
        load_B(0, Bop);
        row_barrier();                                             // (the movers' first rows)
        read_row(-1, wa); read_row(0, wb);
        const int nr12 = ((nr + 11) / 12) * 12;
        for (int r = 0; r < nr12; r += 6) {
            load_B(r + 1, B1);
            if (r < nr) row_products(r, wa, wb, wc, Bop);
            row_barrier();
            load_B(r + 2, Bop);
            if (r + 1 < nr) row_products(r + 1, wb, wc, wa, B1);
            row_barrier();
            load_B(r + 3, B1);
            if (r + 2 < nr) row_products(r + 2, wc, wa, wb, Bop);
            row_barrier();
            load_B(r + 4, Bop);
            if (r + 3 < nr) row_products(r + 3, wa, wb, wc, B1);
            row_barrier();
            load_B(r + 5, B1);
            if (r + 4 < nr) row_products(r + 4, wb, wc, wa, Bop);
            row_barrier();
            load_B(r + 6, Bop);
            if (r + 5 < nr) row_products(r + 5, wc, wa, wb, B1);
            row_barrier();
        }
    }

    // ---- partial sums of this block (as in bwd_dw_kernel)
    const int n = i;
    const float out_scale = 1.0f / IN_SCALE;
    if (n < S) {
        const long side = (long)a.C * S * S;
        float* base = a.partial + (long)j * 2 * side;
#pragma unroll
        for (int ty = 0; ty < 3; ++ty) {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int row = 4 * g + r;
                if (row < ROWS) {
                    const int cc = row / 3, t = 3 * ty + row - 3 * cc;
                    base[((long)(c0 + cc) * S + n) * S + t] = acc_k[ty][r] * (a.scale * out_scale);
                    base[side + ((long)(c0 + cc) * S + n) * S + t] = acc_v[ty][r] * out_scale;
                }
            }
        }
        if (wave == 0 && g == 3)                                   // row 12 = 4*3 + 0
            a.dbias_partial[((long)j * a.heads + m) * S + n] = acc_k[0][0];
    }
}

// bands per plane: enough work items for the blocks of a head, bands of at least 4 rows
static int bands_per_plane(const Problem& p, int n_cu)
{
    long want = n_cu / p.heads;
    if (want < 1) want = 1;
    long nbp = (want + p.B - 1) / p.B;
    const long most = p.H >= 8 ? p.H / 4 : 1;
    if (nbp > most) nbp = most;
    if (nbp < 1) nbp = 1;
    // every band has rows
    while (nbp > 1 && ((p.H + nbp - 1) / nbp) * (nbp - 1) >= p.H) --nbp;
    return (int)nbp;
}
}  // namespace ring

// n_cu: compute units to fill (the workspace query passes the upper bound MAX_CU_PLANNED)
static int blocks_per_head(const Problem& p, int n_cu)
{
    const long units = (long)p.B * ((p.H + R - 1) / R) * ((p.W + TW - 1) / TW);
    long nb = n_cu / p.heads;                // one block per compute unit
    if (nb < 1) nb = 1;
    if (nb > units) nb = units;
    return (int)nb;
}

}  // namespace dwpath

bool bwd_dw_mfma_supported(const Problem& p)
{
    return p.dtype == 1 && p.ksize == 3 && p.C == p.heads * dwpath::D && (p.W % 8) == 0;
}

// the streaming form of the kernel: one column tile, rows of at least four 8-pixel pieces
bool bwd_dw_ring_supported(const Problem& p)
{
    return bwd_dw_mfma_supported(p) && p.W >= 32 && p.W <= dwpath::TW;
}

// floats: per-block kernel-gradient partials, then per-block bias partials
size_t bwd_dw_mfma_partial_floats(const Problem& p)
{
    const size_t nb = (size_t)dwpath::blocks_per_head(p, MAX_CU_PLANNED);
    return nb * 2 * (size_t)p.C * 81 + nb * (size_t)p.heads * 9;
}

hipError_t launch_bwd_dw_mfma(const Problem& p, const void* dout, const void* q, const void* k,
                              const void* v, const void* attn_ws, const void* dl_ws,
                              float* partial, float* dwk, float* dwv, float* dbias, hipStream_t st)
{
    using namespace dwpath;
    Args a;
    a.dout = (const bf16_bits*)dout; a.q = (const bf16_bits*)q; a.k = (const bf16_bits*)k; a.v = (const bf16_bits*)v;
    a.attn = (const _Float16*)attn_ws; a.dl = (const _Float16*)dl_ws;
    a.NB = blocks_per_head(p, device_cu_count());
    a.partial = partial;
    a.dbias_partial = partial + (size_t)a.NB * 2 * p.C * 81;
    a.B = p.B; a.H = p.H; a.W = p.W; a.C = p.C; a.heads = p.heads;
    a.n_strips = (p.H + R - 1) / R; a.n_ct = (p.W + TW - 1) / TW;
    a.scale = p.logit_scale();
    if (bwd_dw_ring_supported(p) && fwd_ring_enabled()) {
        // the streaming form: work items are bands of rows of one batch item's head plane
        const int n_cu = device_cu_count();
        a.nbp = ring::bands_per_plane(p, n_cu);
        a.rows_pb = (p.H + a.nbp - 1) / a.nbp;
        long nb = n_cu / p.heads;
        if (nb < 1) nb = 1;
        if (nb > (long)p.B * a.nbp) nb = (long)p.B * a.nbp;
        if (nb > a.NB) nb = a.NB;                               // (never more partials than the workspace was sized for)
        a.NB = (int)nb;
        a.dbias_partial = partial + (size_t)a.NB * 2 * p.C * 81;
        static LdsOptIn opt_in_ring;
        hipError_t er = opt_in_ring.ensure({(const void*)ring::bwd_dw_ring_kernel}, ring::LDS_BYTES);
        if (er != hipSuccess) return er;
        hipLaunchKernelGGL(ring::bwd_dw_ring_kernel, dim3((unsigned)(a.NB * p.heads)), dim3(ring::THREADS_R),
                           (size_t)ring::LDS_BYTES, st, a);
    } else {
        static LdsOptIn opt_in;
        hipError_t e = opt_in.ensure({(const void*)bwd_dw_kernel}, LDS_BYTES);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(bwd_dw_kernel, dim3((unsigned)(a.NB * p.heads)), dim3(THREADS), (size_t)LDS_BYTES, st, a);
    }
    const long side = (long)p.C * 81;
    return launch_bwd_dw_reduce(partial, dwk, dwv, side, a.NB, a.dbias_partial, dbias, p.heads * 9,
                                p.accumulate, st);
}

}  // namespace slide
