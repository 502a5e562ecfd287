// Streaming matrix-core kernels of the backward of Slide Attention on gfx950 (bf16 activations,
// head size 32, 3x3 window, rows and pointers 16-byte aligned): the key and value gradients
// (maps of 32..56 columns, a multiple of 8; first part of this file) and the per-pixel part,
// attention recompute, logit and query gradients (maps of 32..64 columns; second part).
//
// Key and value gradients.  The paper gives no backward; this is the chain rule through
// the operator of Sec. 4.1-4.3, in the gather form of slide_bwd16.hip:
//     dk[c,y] = scale * sum_u q[c,p']  * sum_s W~k[c,s,t] dl[p',s]
//     dv[c,y] =         sum_u dO[c,p'] * sum_s W~v[c,s,t]  a[p',s]      p' = y + off(u), t = 8 - u
// with a the attention weights and dl the logit gradients of the source pixel p' (written by
// the per-pixel backward kernel as halves, [B, heads, 9, H, W]).  The inner sums are
// v_mfma_f32_16x16x16_f16 products (32 channels x 16 shift slots, times 16 slots x 16 target
// pixels), the outer ones fp32 multiply-adds, exactly as in the tiled kernel; what differs is
// how data moves, which follows the streaming forward (slide_fwd16_ring.hip):
//
//   - a block owns a band of rows of one (batch, head) plane; q and dO rows live in LDS in a
//     ring of R rows, eight planes (tensor x channel octet) of [ring row][column][8 channels as
//     halves]; a and dl live in two more rings, each two planes of [ring row][column][8 shift
//     slots as halves] (slot 4g + r holds shift 4r + g: the matrix operand of lane group g is 8
//     contiguous bytes; slots 0..7 in the first plane, 8..15 in the second, so that the 32 lanes
//     of two groups read 256 contiguous bytes);
//   - epochs of 128 target pixels: eight pass waves run one 16-pixel pass each, four mover waves
//     stage the rows two epochs ahead with loads that write straight into LDS landing slots,
//     read them back with the transposing LDS read and fill the rings; movers 0 and 1 also
//     stage the dl and a rows.  One block barrier per epoch;
//   - a pass wave turns its results (pixel-major in registers) into 16-byte pieces of 8 pixels
//     of one channel through a private LDS slot and stores them itself.
#include "slide_fwd16_ops.h"

namespace slide {
namespace b16ring {
using namespace t16;
using namespace f16ops;

constexpr int WAVES = 8, MOVERS = 4, THREADS = (WAVES + MOVERS) * 64;
constexpr int PX_EPOCH = WAVES * 16;
constexpr int SLOT = 1024;                     // bytes of a landing slot: 8 channels x 64 pixels, or 9 shifts x 56 pixels
constexpr int REC = 32;                        // bytes of a pixel's 16 shift slots
constexpr int REC_ZERO_AT = SLOT - 16;         // a dl / a row fills at most 9 * 112 = 1008 bytes of its landing slot

struct Args {
    const bf16_bits* q; const bf16_bits* dout;
    const _Float16* attn; const _Float16* dl;  // [B, heads, 9, H, W]
    bf16_bits* dk; bf16_bits* dv;
    const uint32_t* image;                     // per head BWD_DKDV_IMG_DWORDS, written by the per-pixel kernel's launcher
    int B, H, W, C, heads;
    int nbp, rows_pb, n_blocks;                // bands per plane, rows per band, blocks
    int R, RS, PS;                             // ring rows, bytes per ring row of a q/dO plane = (W + 2) * 16, bytes per plane = R * RS
    int off_raw, off_rraw, off_dummy, off_rec, off_out;   // LDS byte offsets: q/dO landing slots, dl/a landing slots, dump slot, dl/a rings, result slots (1 KB per pass wave)
    uint32_t magic_w, magic_r;                 // ceil(2^32 / W), ceil(2^32 / R)
    float scale;
};

// RPG: most rows a group of new rows can have (rows that one epoch is the first to read).
template <int RPG>
__global__ void __launch_bounds__(THREADS)
bwd16_ring_dkdv_kernel(const Args a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool mover = wave >= WAVES;
    const int mv = wave - WAVES;                                       // mover index 0 .. 3
    const bool rec_mover = mover && mv < 2;                            // also stages dl (mover 0) or a (mover 1)
    const int p = lane & 15, g = lane >> 4;
    const int W = a.W, H = a.H, R = a.R;
    const int RS = a.RS, PS = a.PS, RW = W + 2;
    const int RR = R * RW * REC;                                       // bytes of one record ring
    const uint32_t hw2 = (uint32_t)H * (uint32_t)W * 2u;             // bytes of one channel (or shift) plane
    const uint32_t w2 = (uint32_t)W * 2u;
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem;

    // block -> band of rows of one plane; the bands of a plane run on the same XCD
    int u_blk = blockIdx.x;
    {
        const int per = a.n_blocks >> 3;
        if (u_blk < 8 * per) u_blk = (u_blk & 7) * per + (u_blk >> 3);
    }
    const int plane = u_blk / a.nbp, part = u_blk - plane * a.nbp;
    const int b = plane / a.heads, m = plane - b * a.heads;
    const int y0 = part * a.rows_pb;
    const int nr = min(a.rows_pb, H - y0);
    const long HW = (long)H * W;
    const long head_base = ((long)b * a.C + (long)m * D) * HW;         // element offset of channel 0 of the head
    const int npix = nr * W, npass = (npix + 15) >> 4, E = (npass + WAVES - 1) / WAVES;

    auto div_w = [&](int x) { return (int)__umulhi((uint32_t)x, a.magic_w); };
    auto mod_r = [&](int x) { return x - (int)__umulhi((uint32_t)x, a.magic_r) * R; };
    auto srn = [&](int j) {
        const int rb = min(div_w(PX_EPOCH * j + PX_EPOCH - 1), nr - 1);
        return j >= E ? nr + 1 : min(rb + 2, nr + 1);
    };

    // ---- movers.  Ten units of staging work per epoch: q and dO, four channel octets each, and the
    // dl and a rows (about as much work as two and a half of the others).  Movers 0 and 1 take dl
    // resp. a and octet 0 of q resp. dO; movers 2 and 3 take octets 1..3 of q resp. dO.
    const int mj = mv & 1;                                             // the mover's tensor: q (and dl) or dO (and a)
    const int NU = rec_mover ? 1 : 3;                                  // its channel octets
    auto unit_id = [&](int u) { return 4 * mj + (rec_mover ? 0 : 1 + u); };   // plane of the ring / set of landing slots
    const bf16_bits* kv_base = (mj ? a.dout : a.q) + head_base;
    const int NXC = W >> 3;
    const int kv_cc = lane / NXC, kv_x = lane - kv_cc * NXC;           // channel (or shift) and 16-byte chunk of the lane
    const uint32_t kv_lane_off = (uint32_t)kv_cc * hw2 + (uint32_t)kv_x * 16u;
    // landing slots of a unit: two sets of RPG; at start-up two more, which lie where the dl / a
    // rings will be (they are fetched before the first ring row is written)
    auto slot_off = [&](int u, int s) {
        const int raw = a.off_raw + unit_id(u) * (2 * RPG * SLOT);
        return s < 2 * RPG ? raw + s * SLOT : a.off_rec + (2 * unit_id(u) + (s - 2 * RPG)) * SLOT;
    };
    auto load_row = [&](int u, uint32_t row_off, int off) {
        const bf16_bits* src = kv_base + (long)(8 * (unit_id(u) & 3)) * HW;
        if (lane < W) load_to_lds(src, kv_lane_off + row_off, lds0 + off);
    };
    // dl (mover 0) / a (mover 1): nine shift planes of the head, landing as [shift][W] halves; the
    // last 16 bytes of their landing slots stay zero
    const _Float16* rec_src = (mj ? a.attn : a.dl) + (long)plane * S * HW;
    auto rslot = [&](int s) { return a.off_rraw + mj * ((2 * RPG + 2) * SLOT) + s * SLOT; };
    auto load_rec = [&](uint32_t row_off, int off) {
        if (lane < S * NXC) load_to_lds(rec_src, kv_lane_off + row_off, lds0 + off);
    };
    const int cv_src_off = ((lane & 15) >> 2) * (W * 2) + (16 * (lane >> 4) + 4 * (lane & 3)) * 2;
    struct RawRow { uint2_t lo, hi; };
    auto read_row = [&](int off) {
        RawRow r;
        const unsigned char* src = smem + off + cv_src_off;
        r.lo = lds_read_tr(src);
        r.hi = lds_read_tr(src + 4 * (W * 2));
        return r;
    };
    auto write_row = [&](int u, uint32_t ring_off, bool in_map, const RawRow& r) {
        uint4_t h4 = {0u, 0u, 0u, 0u};
        if (in_map) {                                                  // (uniform)
            h4[0] = bf16x2_to_half2(r.lo[0]); h4[1] = bf16x2_to_half2(r.lo[1]);
            h4[2] = bf16x2_to_half2(r.hi[0]); h4[3] = bf16x2_to_half2(r.hi[1]);
        }
        if (lane < W) *(uint4_t*)(smem + unit_id(u) * PS + (lane + 1) * 16 + ring_off) = h4;
    };
    // A landed dl / a row -> records.  In the 16-lane group g, lane n of piece q16 gets the
    // shifts g, 4 + g, 8 + g, 12 + g of pixel 16 q16 + n (slots 4g .. 4g + 3): lane s of the group
    // addresses the four pixels 4 (s % 4) .. of shift 4 (s / 4) + g, or, for a shift past 8 or a
    // piece past the row, the zero bytes at the end of the slot.
    const int rc_shift = 4 * ((lane & 15) >> 2) + g;
    int rc_off[4];
#pragma unroll
    for (int q16 = 0; q16 < 4; ++q16)
        rc_off[q16] = (rc_shift < S && 16 * q16 < W) ? rc_shift * (W * 2) + 4 * (lane & 3) * 2 + 32 * q16 : REC_ZERO_AT;
    struct RecRow { uint2_t x[4]; };
    auto read_rec = [&](int off) {
        RecRow r;
#pragma unroll
        for (int q16 = 0; q16 < 4; ++q16) r.x[q16] = lds_read_tr(smem + off + rc_off[q16]);
        return r;
    };
    auto write_rec = [&](uint32_t ring_pos, bool in_map, const RecRow& r) {
        unsigned char* dst = smem + a.off_rec + mj * RR + (g >> 1) * (RR / 2) + (ring_pos + 1 + p) * 16 + 8 * (g & 1);
#pragma unroll
        for (int q16 = 0; q16 < 4; ++q16) {
            const uint2_t v = in_map ? r.x[q16] : uint2_t{0u, 0u};     // (uniform)
            if (16 * q16 + 16 <= W) *(uint2_t*)(dst + 16 * q16 * 16) = v;
            else if (16 * q16 < W) { if (p < W - 16 * q16) *(uint2_t*)(dst + 16 * q16 * 16) = v; }
        }
    };

    // ---- start-up: the movers issue groups 0 and 1, the pass waves fetch their matrix operands
    const int v0 = srn(0), v1 = srn(1), v2 = srn(2);
    int n_after_g0 = 0;                                                // mover: loads issued after group 0
    half4_t Ak[S][2], Av[S][2];
    if (mover) {
        for (int k = 0; k <= v0; ++k) {                                // group 0 (at most RPG + 2 rows)
            const int gy = y0 - 1 + k;
            const int sl = k < RPG ? k : 2 * RPG + (k - RPG);
            if (gy >= 0 && gy < H) {
                for (int u = 0; u < NU; ++u) load_row(u, (uint32_t)gy * w2, slot_off(u, sl));
                if (rec_mover) load_rec((uint32_t)gy * w2, rslot(sl));
            }
        }
        for (int k = 0; k < v1 - v0; ++k) {                            // group 1 into set 1
            const int gy = y0 + v0 + k;
            if (gy >= 0 && gy < H) {
                for (int u = 0; u < NU; ++u) load_row(u, (uint32_t)gy * w2, slot_off(u, RPG + k));
                n_after_g0 += NU;
                if (rec_mover) { load_rec((uint32_t)gy * w2, rslot(RPG + k)); n_after_g0 += 1; }
            }
        }
    } else {
        const uint32_t* img = a.image + (long)m * BWD_DKDV_IMG_DWORDS;
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
    }

    // ---- the schedule, lane e of the table registers holding epoch e (E <= 64); ring positions
    // in pixels (10 bits), as in the streaming forward
    uint32_t t_cvA, t_cvB, t_ld, t_p0, t_p1, t_p2;
    {
        const int e = lane;
        const int s0 = srn(e), s1 = srn(e + 1), s2 = srn(e + 2), s3 = srn(e + 3);
        auto ring_of = [&](int sr) { return (uint32_t)(mod_r(sr) * RW); };
        t_cvA = ring_of(s0 + 1) | ring_of(s0 + 2) << 10 | ring_of(s0 + 3) << 20;
        uint32_t outside = 0, ldm = 0;
#pragma unroll
        for (int k = 0; k < RPG; ++k) {
            const int gy = y0 + s0 + k, gl = y0 + s2 + k;
            outside |= (gy < 0 || gy >= H) ? 1u << k : 0u;
            ldm |= (k < s3 - s2 && gl >= 0 && gl < H) ? 1u << k : 0u;
        }
        t_cvB = ring_of(s0 + 4) | (uint32_t)(s1 - s0) << 10 | outside << 13 | ldm << 17;
        t_ld = (uint32_t)(min(max(y0 + s2, 0), H - 1) * W) * 2u;
        const int nbe = PX_EPOCH * e + 16 * (mover ? 0 : wave);
        const int ra = div_w(nbe), c0 = nbe - ra * W;
        t_p0 = ring_of(ra) | ring_of(ra + 1) << 10 | ring_of(ra + 2) << 20;
        t_p1 = ring_of(ra + 1) | ring_of(ra + 2) << 10 | ring_of(ra + 3) << 20;
        t_p2 = (uint32_t)c0 | (nbe < npix ? 256u : 0u);
    }

    // the padding columns of the q / dO ring stay zero; so do the last 16 bytes of the dl / a landing slots
    for (int idx = tid; idx < R * 16; idx += THREADS) {
        const int unit = idx & 7, side = (idx >> 3) & 1, row = idx >> 4;
        *(uint4_t*)(smem + unit * PS + row * RS + (side ? W + 1 : 0) * 16) = uint4_t{0u, 0u, 0u, 0u};
    }
    if (tid < 2 * (2 * RPG + 2)) *(uint4_t*)(smem + a.off_rraw + tid * SLOT + REC_ZERO_AT) = uint4_t{0u, 0u, 0u, 0u};
    block_barrier();                                                   // (those zeros are read by the conversions below)

    auto zero_rec_pads = [&]() {                                       // the padding columns of the dl / a rings (all threads)
        for (int idx = tid; idx < R * 8; idx += THREADS) {
            const int half16 = idx & 1, side = (idx >> 1) & 1, tsel = (idx >> 2) & 1, row = idx >> 3;
            *(uint4_t*)(smem + a.off_rec + tsel * RR + half16 * (RR / 2) + (row * RW + (side ? W + 1 : 0)) * 16) = uint4_t{0u, 0u, 0u, 0u};
        }
    };
    // The two kinds of waves part here (their registers never coexist); both pass two more
    // start-up barriers and one barrier per epoch.
    if (mover) {
        // only the epoch's own round of loads is still in flight: 2 RPG (a record mover: one octet
        // and dl / a) or 3 RPG (three octets)
        auto wait_round = [&]() {
            if (rec_mover) {
                if (RPG == 2) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
                else if (RPG == 3) asm volatile("s_waitcnt vmcnt(6)" ::: "memory");
                else asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
            } else {
                if (RPG == 2) asm volatile("s_waitcnt vmcnt(6)" ::: "memory");
                else if (RPG == 3) asm volatile("s_waitcnt vmcnt(9)" ::: "memory");
                else asm volatile("s_waitcnt vmcnt(12)" ::: "memory");
            }
        };
        // group 0 -> ring rows 0 .. v0 (v0 <= RPG + 1).  The rows in the two extra landing slots
        // of every unit, which lie in the dl / a rings, are fetched before the barrier; no ring row
        // is written before it.
        RawRow gx[2][3];
        wait_vmem(n_after_g0);                                         // group 0 has landed
#pragma unroll
        for (int x = 0; x < 2; ++x)
            if (RPG + x <= v0)
#pragma unroll
                for (int u = 0; u < 3; ++u)
                    if (u < NU) gx[x][u] = read_row(slot_off(u, 2 * RPG + x));
        block_barrier();
        zero_rec_pads();
        for (int k = 0; k <= v0; ++k) {
            const bool in_map = y0 - 1 + k >= 0 && y0 - 1 + k < H;
            const int sl = k < RPG ? k : 2 * RPG + (k - RPG);
            if (k < RPG) {
                RawRow r0[3];
#pragma unroll
                for (int u = 0; u < 3; ++u)
                    if (u < NU) r0[u] = read_row(slot_off(u, k));
#pragma unroll
                for (int u = 0; u < 3; ++u)
                    if (u < NU) write_row(u, (uint32_t)(k * RS), in_map, r0[u]);
            } else {
#pragma unroll
                for (int u = 0; u < 3; ++u)
                    if (u < NU) write_row(u, (uint32_t)(k * RS), in_map, k == RPG ? gx[0][u] : gx[1][u]);
            }
            if (rec_mover) {
                const RecRow rr = read_rec(rslot(sl));
                write_rec((uint32_t)(k * RW), in_map, rr);
            }
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");             // set 0 has been read before it is loaded again
        // group 2 into set 0, as a full round of loads
#pragma unroll
        for (int k = 0; k < RPG; ++k) {
            const int gy = y0 + v1 + k;
            const bool real = k < v2 - v1 && gy >= 0 && gy < H;
            const uint32_t ro = (uint32_t)min(max(gy, 0), H - 1) * w2;
#pragma unroll
            for (int u = 0; u < 3; ++u)
                if (u < NU) load_row(u, ro, real ? slot_off(u, k) : a.off_dummy);
            if (rec_mover) load_rec(ro, real ? rslot(k) : a.off_dummy);
        }
        wait_round();                                                  // everything but that round: group 1 has landed
        block_barrier();

        __builtin_amdgcn_s_setprio(3);                                 // the movers go ahead of the pass waves of their SIMD
        int set_rd = RPG * SLOT;                                       // offset of the set that holds group e + 1
        for (int e = 0; e < E; ++e) {
            const uint32_t cvA = __builtin_amdgcn_readlane(t_cvA, e), cvB = __builtin_amdgcn_readlane(t_cvB, e);
            const uint32_t ldo = __builtin_amdgcn_readlane(t_ld, e);
            // group e + 1 has landed (waited for at the end of the previous epoch): fetch it
            RawRow raw[3][RPG];
            RecRow rec[RPG];
#pragma unroll
            for (int u = 0; u < 3; ++u)
                if (u < NU)
#pragma unroll
                    for (int k = 0; k < RPG; ++k) raw[u][k] = read_row(slot_off(u, 0) + set_rd + k * SLOT);
            if (rec_mover) {
#pragma unroll
                for (int k = 0; k < RPG; ++k) rec[k] = read_rec(rslot(0) + set_rd + k * SLOT);
            }
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            // the epoch's round of loads: group e + 3 into the slots just read
#pragma unroll
            for (int k = 0; k < RPG; ++k) {
                const bool real = (cvB >> (17 + k)) & 1u;
                const uint32_t ro = real ? ldo + (uint32_t)k * w2 : ldo;
#pragma unroll
                for (int u = 0; u < 3; ++u)
                    if (u < NU) load_row(u, ro, real ? slot_off(u, 0) + set_rd + k * SLOT : a.off_dummy);
                if (rec_mover) load_rec(ro, real ? rslot(0) + set_rd + k * SLOT : a.off_dummy);
            }
            // group e + 1 into the rings
            const int cnt = (cvB >> 10) & 7;
#pragma unroll
            for (int k = 0; k < RPG; ++k) {
                const uint32_t pos = k < 3 ? (cvA >> (10 * k)) & 1023u : cvB & 1023u;
                if (k < cnt) {
                    const bool in_map = !((cvB >> (13 + k)) & 1u);
#pragma unroll
                    for (int u = 0; u < 3; ++u)
                        if (u < NU) write_row(u, pos * 16, in_map, raw[u][k]);
                    if (rec_mover) write_rec(pos, in_map, rec[k]);
                }
            }
            set_rd = RPG * SLOT - set_rd;
            wait_round();
            block_barrier();
        }
        wait_vmem(0);                                                  // no load into this block's LDS outlives it
        return;
    }

    // ---- pass waves
    block_barrier();
    zero_rec_pads();
    block_barrier();
    unsigned char* o_slot = smem + a.off_out + wave * SLOT;
    const int VD = 4 * PS;
    const unsigned char* tap_base = smem + g * PS;
    const unsigned char* rec_base = smem + a.off_rec + (g >> 1) * (RR / 2) + 8 * (g & 1);
    const int st_c = 16 * ((lane >> 4) & 1) + (lane & 15), st_hh = lane >> 5;
    char* dk_base = (char*)(a.dk + head_base + (long)y0 * W) + (uint32_t)st_c * hw2;
    char* dv_base = (char*)(a.dv + head_base + (long)y0 * W) + (uint32_t)st_c * hw2;
    const float4_t zero4 = {0.0f, 0.0f, 0.0f, 0.0f};
    int nb = 16 * wave;
    for (int e = 0; e < E; ++e) {
        const uint32_t p2 = __builtin_amdgcn_readlane(t_p2, e);
        if (p2 & 256u) {
            const uint32_t p0 = __builtin_amdgcn_readlane(t_p0, e), p1 = __builtin_amdgcn_readlane(t_p1, e);
            const int cx0 = (int)(p2 & 255u) + p;
            const bool next_row = cx0 >= W;
            const uint32_t cx = next_row ? cx0 - W : cx0;
            const uint32_t rows = next_row ? p1 : p0;
            float dk[8], dv[8];
#pragma unroll
            for (int x = 0; x < 8; ++x) { dk[x] = 0.0f; dv[x] = 0.0f; }
#pragma unroll
            for (int uy = 0; uy < KS; ++uy) {
                const uint32_t pos = ((rows >> (10 * uy)) & 1023u) + cx;   // ring position of the window's left column
                const unsigned char* qrow = tap_base + (pos << 4);
                const unsigned char* rrow = rec_base + (pos << 4);
                uint4_t qd[KS], dod[KS];
                uint2_t bdl[KS], ba[KS];
#pragma unroll
                for (int ux = 0; ux < KS; ++ux) {
                    qd[ux] = *(const uint4_t*)(qrow + ux * 16);
                    dod[ux] = *(const uint4_t*)(qrow + VD + ux * 16);
                    bdl[ux] = *(const uint2_t*)(rrow + ux * 16);
                    ba[ux] = *(const uint2_t*)(rrow + RR + ux * 16);
                }
                // the row's twelve matrix products (tap x channel half x side), each two products ahead
                // of the multiply-adds that use it
                float4_t w[4 * KS];
                auto product = [&](int i) {
                    const int ux = i >> 2, j = (i >> 1) & 1;
                    const int t = S - 1 - (uy * KS + ux);                 // tap through which the source sees the target
                    return (i & 1) ? __builtin_amdgcn_mfma_f32_16x16x16f16(Av[t][j], __builtin_bit_cast(half4_t, ba[ux]), zero4, 0, 0, 0)
                                   : __builtin_amdgcn_mfma_f32_16x16x16f16(Ak[t][j], __builtin_bit_cast(half4_t, bdl[ux]), zero4, 0, 0, 0);
                };
                constexpr int AHEAD = 2;
#pragma unroll
                for (int i = 0; i < AHEAD; ++i) w[i] = product(i);
#pragma unroll
                for (int i = 0; i < 4 * KS; ++i) {
                    if (i + AHEAD < 4 * KS) w[i + AHEAD] = product(i + AHEAD);
                    __builtin_amdgcn_sched_barrier(0);
                    const int ux = i >> 2, j = (i >> 1) & 1;
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int x = 4 * j + r;
                        if (i & 1) dv[x] = fmaf(w[i][r], (float)as_half2(dod[ux][x >> 1])[x & 1], dv[x]);
                        else       dk[x] = fmaf(w[i][r], (float)as_half2(qd[ux][x >> 1])[x & 1], dk[x]);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            uint4_t ovk, ovv;
#pragma unroll
            for (int y = 0; y < 4; ++y) {
                typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
                typedef float float2_t __attribute__((ext_vector_type(2)));
                const float2_t fk = {dk[2 * y] * a.scale, dk[2 * y + 1] * a.scale};
                const float2_t fv = {dv[2 * y], dv[2 * y + 1]};
                ovk[y] = __builtin_bit_cast(uint32_t, __builtin_convertvector(fk, bf16x2_t));
                ovv[y] = __builtin_bit_cast(uint32_t, __builtin_convertvector(fv, bf16x2_t));
            }
            // pixel-major -> 8 pixels of one channel per lane, through the wave's own slot: dk, then
            // dv (the LDS unit serves a wave's accesses in the order of their issue)
            const int wr = p * 64 + ((g ^ ((p >> 2) & 3)) << 4);
            const int grp = lane >> 4, nn = lane & 15;
            const int sa = nn & 3, sj = nn >> 2;
            const int oct_s = 2 * (grp & 1) + (sa >> 1);
            const int P0 = 8 * st_hh + sj, P1 = P0 + 4;
            const int rd0 = P0 * 64 + ((oct_s ^ ((P0 >> 2) & 3)) << 4) + (sa & 1) * 8;
            const int rd1 = P1 * 64 + ((oct_s ^ ((P1 >> 2) & 3)) << 4) + (sa & 1) * 8;
            *(uint4_t*)(o_slot + wr) = ovk;
            asm volatile("" ::: "memory");
            const uint2_t ka = lds_read_tr(o_slot + rd0), kb = lds_read_tr(o_slot + rd1);
            asm volatile("" ::: "memory");
            *(uint4_t*)(o_slot + wr) = ovv;
            asm volatile("" ::: "memory");
            const uint2_t va = lds_read_tr(o_slot + rd0), vb = lds_read_tr(o_slot + rd1);
            const int n0 = nb + 8 * st_hh;
            if (n0 < npix) {
                *(uint4_t*)(dk_base + (uint32_t)n0 * 2u) = uint4_t{ka[0], ka[1], kb[0], kb[1]};
                *(uint4_t*)(dv_base + (uint32_t)n0 * 2u) = uint4_t{va[0], va[1], vb[0], vb[1]};
            }
        }
        nb += PX_EPOCH;
        block_barrier();
    }
}

struct Plan {
    RingRows rr;
    int RS, PS, off_raw, off_rraw, off_dummy, off_rec, off_out, lds_bytes;
    bool ok;
};

static Plan plan(const Problem& p)
{
    Plan r{};
    r.ok = false;
    if (p.W > 56) return r;                                            // a dl / a row (9 shifts x W / 8 pieces) is one load of 64 lanes
    r.rr = plan_ring_rows(p, WAVES, 1);
    if (!r.rr.ok) return r;
    const int W = p.W, rpg = r.rr.rpg, R = r.rr.R;
    r.RS = (W + 2) * 16;
    r.PS = R * r.RS;
    r.off_raw = (8 * r.PS + 1023) & ~1023;
    r.off_rraw = r.off_raw + 8 * 2 * rpg * SLOT;
    r.off_dummy = r.off_rraw + 2 * (2 * rpg + 2) * SLOT;
    r.off_rec = r.off_dummy + SLOT;
    r.off_out = (r.off_rec + 2 * R * (W + 2) * REC + 1023) & ~1023;
    r.lds_bytes = r.off_out + WAVES * SLOT;
    if (4 * r.PS > 65535 - 64) return r;                               // dO taps are read at an immediate offset
    if (2 * R * (W + 2) * REC < 16 * SLOT) return r;                   // the start-up's extra landing slots lie in the dl / a rings
    r.ok = r.lds_bytes <= LDS_LIMIT;
    return r;
}


// ------------------------------------------------------------------ per-pixel backward
// For every pixel: recompute the attention weights a as the forward does, then
//     da[s] = sum_c dO[c] Vs[c,s]        (same shape as the logits, with dO, v, W~v)
//     dl[s] = a[s] (da[s] - sum_s' a[s'] da[s'])
//     dq[c] = scale * sum_t k[c,p+t] * sum_s dl[s] W~k[c,s,t]            (same shape as out)
// a and dl go to the workspace as halves [B, heads, 9, H, W] for the other two kernels.
// Same arithmetic as the tiled bwd_pixel_kernel16; data moves as in the streaming forward: K
// and V rows in an LDS ring staged by four mover waves, q and dO of a pass loaded into slots of
// the pass wave one epoch ahead (two slots per wave and tensor), the matrix operands of the two
// K-kernel products resident in registers and those of the V-kernel product read from a copy
// of the image in LDS (three resident sets would leave no registers for the taps).
struct PixelArgs {
    const bf16_bits* q; const bf16_bits* k; const bf16_bits* v; const bf16_bits* dout;
    bf16_bits* dq;
    _Float16* attn; _Float16* dl;              // [B, heads, 9, H, W]
    const uint32_t* image;                     // per head BWD_PX_IMG_DWORDS
    int B, H, W, C, heads;
    int nbp, rows_pb, n_blocks;
    int R, RS, PS;
    int off_raw, off_dummy, off_q, off_do, off_out, off_a1v;   // LDS byte offsets: K/V landing slots, dump slot, q slots and dO slots (2 KB per pass wave each), result slots, V-kernel operands
    uint32_t magic_w, magic_r;
    float scale, scale_log2e;
    float* part;                               // heads of 64 channels (MODE 1, 2): every half head's share of the logits (times scale_log2e) and of da, [B, 2 heads, 2, 9, H, W]
};

// MODE: heads of 64 channels run as two half heads of 32 (the arguments describe twice as many
// heads).  Logits and da are sums over the channels of the whole head: MODE 1 forms each half's
// share of both and writes them to `part`, nothing else; MODE 2 is the rest: it adds the two
// halves' shares (no q, dO or value rows are staged, no products formed for them), so both
// halves arrive at the same a and dl (each writes its copy, which the other two backward kernels
// read per half head), and each forms dq of its own 32 channels from its key rows.  MODE 0:
// heads of 32 channels, one launch.
template <int RPG, int MODE = 0>
__global__ void __launch_bounds__(THREADS)
bwd16_ring_pixel_kernel(const PixelArgs a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool mover = wave >= WAVES;
    const int mv = wave - WAVES;
    const int p = lane & 15, g = lane >> 4;
    const int W = a.W, H = a.H, R = a.R;
    const int RS = a.RS, PS = a.PS, RW = W + 2;
    const uint32_t hw2 = (uint32_t)H * (uint32_t)W * 2u;
    const uint32_t w2 = (uint32_t)W * 2u;
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem;

    int u_blk = blockIdx.x;
    {
        const int per = a.n_blocks >> 3;
        if (u_blk < 8 * per) u_blk = (u_blk & 7) * per + (u_blk >> 3);
    }
    const int plane = u_blk / a.nbp, part = u_blk - plane * a.nbp;
    const int b = plane / a.heads, m = plane - b * a.heads;
    const int y0 = part * a.rows_pb;
    const int nr = min(a.rows_pb, H - y0);
    const long HW = (long)H * W;
    const long head_base = ((long)b * a.C + (long)m * D) * HW;
    const int npix = nr * W, npass = (npix + 15) >> 4, E = (npass + WAVES - 1) / WAVES;

    auto div_w = [&](int x) { return (int)__umulhi((uint32_t)x, a.magic_w); };
    auto mod_r = [&](int x) { return x - (int)__umulhi((uint32_t)x, a.magic_r) * R; };
    auto srn = [&](int j) {
        const int rb = min(div_w(PX_EPOCH * j + PX_EPOCH - 1), nr - 1);
        return j >= E ? nr + 1 : min(rb + 2, nr + 1);
    };

    // ---- mover: units j = 0 (K), 1 (V) of octet mv; q and dO of pass waves 2 mv, 2 mv + 1
    const int oct = mover ? mv : 0;
    const bf16_bits* kv_src[2] = {a.k + head_base + (long)(8 * oct) * HW, a.v + head_base + (long)(8 * oct) * HW};
    const int NXC = W >> 3;
    const int kv_cc = lane / NXC, kv_x = lane - kv_cc * NXC;
    const uint32_t kv_lane_off = (uint32_t)kv_cc * hw2 + (uint32_t)kv_x * 16u;
    // landing slots of unit j: two sets of RPG; at start-up also the second q slot and the second
    // dO slot of pass wave 2 mv + j (not loaded into before the first epoch)
    auto slot_off = [&](int j, int s) {
        const int raw = a.off_raw + (4 * j + oct) * (2 * RPG * SLOT);
        const int pw = 2 * oct + j;
        return s < 2 * RPG ? raw + s * SLOT : (s == 2 * RPG ? a.off_q : a.off_do) + pw * (2 * SLOT) + SLOT;
    };
    auto load_row = [&](int j, uint32_t row_off, int off) {
        if (lane < W) load_to_lds(kv_src[j], kv_lane_off + row_off, lds0 + off);
    };
    const int cv_src_off = ((lane & 15) >> 2) * (W * 2) + (16 * (lane >> 4) + 4 * (lane & 3)) * 2;
    struct RawRow { uint2_t lo, hi; };
    auto read_row = [&](int off) {
        RawRow r;
        const unsigned char* src = smem + off + cv_src_off;
        r.lo = lds_read_tr(src);
        r.hi = lds_read_tr(src + 4 * (W * 2));
        return r;
    };
    auto write_row = [&](int j, uint32_t ring_off, bool in_map, const RawRow& r) {
        uint4_t h4 = {0u, 0u, 0u, 0u};
        if (in_map) {                                                  // (uniform)
            h4[0] = bf16x2_to_half2(r.lo[0]); h4[1] = bf16x2_to_half2(r.lo[1]);
            h4[2] = bf16x2_to_half2(r.hi[0]); h4[3] = bf16x2_to_half2(r.hi[1]);
        }
        if (lane < W) *(uint4_t*)(smem + (4 * j + oct) * PS + (lane + 1) * 16 + ring_off) = h4;
    };
    // q (x = 0) or dO (x = 1) of pass wave pw, pass starting at band pixel n_first, into slot sl of that wave
    const bf16_bits* qd_src[2] = {a.q + head_base + (long)y0 * W, a.dout + head_base + (long)y0 * W};
    const uint32_t q_lane_off = (uint32_t)(lane >> 1) * hw2 + (uint32_t)(lane & 1) * 16u;
    auto load_qd = [&](int x, int pw, int n_first, int sl) {
        const bool real = n_first < npix;
        const int nf = real ? n_first : 0;
        const int off = real ? (x ? a.off_do : a.off_q) + pw * (2 * SLOT) + sl * SLOT : a.off_dummy;
        if (nf + 8 * (lane & 1) < npix) load_to_lds(qd_src[x], q_lane_off + (uint32_t)nf * 2u, lds0 + off);
    };

    // ---- start-up
    // MODE 2 takes logits and da whole from the workspace: no q, dO or value rows, only key rows for dq
    constexpr int J1 = MODE == 2 ? 1 : 2;                              // tensors a mover stages: K (j = 0), V (j = 1)
    constexpr bool HAS_QD = MODE != 2;
    const int v0 = srn(0), v1 = srn(1), v2 = srn(2);
    int n_after_g0 = 0;
    half8_t A1k[S];
    half4_t A2k[2 * S];
    float bias2[3];
    const uint32_t* img = a.image + (long)m * BWD_PX_IMG_DWORDS;
    if (mover) {
        for (int k = 0; k <= v0; ++k) {                                // group 0 (at most RPG + 2 rows)
            const int gy = y0 - 1 + k;
            if (gy >= 0 && gy < H)
                for (int j = 0; j < J1; ++j) load_row(j, (uint32_t)gy * w2, slot_off(j, k < RPG ? k : 2 * RPG + (k - RPG)));
        }
        if (HAS_QD) {
            for (int i = 0; i < 2; ++i)
                for (int x = 0; x < 2; ++x) load_qd(x, 2 * mv + i, 16 * (2 * mv + i), 0);
            n_after_g0 = 4;
        }
        for (int k = 0; k < v1 - v0; ++k) {                            // group 1 into set 1
            const int gy = y0 + v0 + k;
            if (gy >= 0 && gy < H) {
                for (int j = 0; j < J1; ++j) load_row(j, (uint32_t)gy * w2, slot_off(j, RPG + k));
                n_after_g0 += J1;
            }
        }
    } else {
#pragma unroll
        for (int t = 0; t < S; ++t) A1k[t] = __builtin_bit_cast(half8_t, *(const uint4_t*)(img + BWD_PX_A1K + (t * 64 + lane) * 4));
#pragma unroll
        for (int u = 0; u < 2 * S; ++u) A2k[u] = __builtin_bit_cast(half4_t, *(const uint2_t*)(img + BWD_PX_A2K + (u * 64 + lane) * 2));
#pragma unroll
        for (int r = 0; r < 3; ++r) bias2[r] = __uint_as_float(img[BWD_PX_BIAS + 4 * g + r]);
        // the V-kernel operands (9 taps x 64 lanes x 16 bytes) into LDS
        for (int i = tid; i < S * 64; i += WAVES * 64)
            *(uint4_t*)(smem + a.off_a1v + i * 16) = *(const uint4_t*)(img + BWD_PX_A1V + i * 4);
    }

    uint32_t t_cvA, t_cvB, t_ld, t_p0, t_p1, t_p2;
    {
        const int e = lane;
        const int s0 = srn(e), s1 = srn(e + 1), s2 = srn(e + 2), s3 = srn(e + 3);
        auto ring_of = [&](int sr) { return (uint32_t)(mod_r(sr) * RW); };
        t_cvA = ring_of(s0 + 1) | ring_of(s0 + 2) << 10 | ring_of(s0 + 3) << 20;
        uint32_t outside = 0, ldm = 0;
#pragma unroll
        for (int k = 0; k < RPG; ++k) {
            const int gy = y0 + s0 + k, gl = y0 + s2 + k;
            outside |= (gy < 0 || gy >= H) ? 1u << k : 0u;
            ldm |= (k < s3 - s2 && gl >= 0 && gl < H) ? 1u << k : 0u;
        }
        t_cvB = ring_of(s0 + 4) | (uint32_t)(s1 - s0) << 10 | outside << 13 | ldm << 17;
        t_ld = (uint32_t)(min(max(y0 + s2, 0), H - 1) * W) * 2u;
        const int nbe = PX_EPOCH * e + 16 * (mover ? 0 : wave);
        const int ra = div_w(nbe), c0 = nbe - ra * W;
        t_p0 = ring_of(ra) | ring_of(ra + 1) << 10 | ring_of(ra + 2) << 20;
        t_p1 = ring_of(ra + 1) | ring_of(ra + 2) << 10 | ring_of(ra + 3) << 20;
        t_p2 = (uint32_t)c0 | (nbe < npix ? 256u : 0u);
    }
    for (int idx = tid; idx < R * 16; idx += THREADS) {                // the padding columns of the ring stay zero
        const int unit = idx & 7, side = (idx >> 3) & 1, row = idx >> 4;
        *(uint4_t*)(smem + unit * PS + row * RS + (side ? W + 1 : 0) * 16) = uint4_t{0u, 0u, 0u, 0u};
    }

    if (mover) {
        // only the row loads of the epoch are still in flight (they follow its q and dO loads)
        auto wait_rows = [&]() {
            constexpr int NR = J1 * RPG;                                // row loads per epoch
            if (NR == 2) asm volatile("s_waitcnt vmcnt(2)" ::: "memory");
            else if (NR == 3) asm volatile("s_waitcnt vmcnt(3)" ::: "memory");
            else if (NR == 4) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
            else if (NR == 6) asm volatile("s_waitcnt vmcnt(6)" ::: "memory");
            else asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
        };
        wait_vmem(n_after_g0);                                         // group 0 has landed
        for (int k = 0; k <= v0; ++k) {                                // group 0 -> ring rows 0 .. v0
            RawRow r0[2];
            for (int j = 0; j < J1; ++j) r0[j] = read_row(slot_off(j, k < RPG ? k : 2 * RPG + (k - RPG)));
            for (int j = 0; j < J1; ++j) write_row(j, (uint32_t)(k * RS), y0 - 1 + k >= 0 && y0 - 1 + k < H, r0[j]);
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");             // set 0 has been read before it is loaded again
#pragma unroll
        for (int k = 0; k < RPG; ++k) {                                // group 2 into set 0, as a full round of row loads
            const int gy = y0 + v1 + k;
            const bool real = k < v2 - v1 && gy >= 0 && gy < H;
            for (int j = 0; j < J1; ++j)
                load_row(j, (uint32_t)min(max(gy, 0), H - 1) * w2, real ? slot_off(j, k) : a.off_dummy);
        }
        wait_rows();                                                   // group 1, q and dO of epoch 0 have landed
        block_barrier();

        __builtin_amdgcn_s_setprio(3);                                 // the movers go ahead of the pass waves of their SIMD
        int set_rd = RPG * SLOT;
        for (int e = 0; e < E; ++e) {
            const uint32_t cvA = __builtin_amdgcn_readlane(t_cvA, e), cvB = __builtin_amdgcn_readlane(t_cvB, e);
            const uint32_t ldo = __builtin_amdgcn_readlane(t_ld, e);
            RawRow raw[2][RPG];
#pragma unroll
            for (int j = 0; j < J1; ++j)
#pragma unroll
                for (int k = 0; k < RPG; ++k) raw[j][k] = read_row(slot_off(j, 0) + set_rd + k * SLOT);
            // q and dO of the next epoch, into the slots that the epoch before this one read
            if (HAS_QD) {
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int x = 0; x < 2; ++x) load_qd(x, 2 * mv + i, PX_EPOCH * (e + 1) + 16 * (2 * mv + i), (e + 1) & 1);
            }
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            // group e + 3 into the slots just read
#pragma unroll
            for (int k = 0; k < RPG; ++k) {
                const bool real = (cvB >> (17 + k)) & 1u;
#pragma unroll
                for (int j = 0; j < J1; ++j)
                    load_row(j, real ? ldo + (uint32_t)k * w2 : ldo, real ? slot_off(j, 0) + set_rd + k * SLOT : a.off_dummy);
            }
            const int cnt = (cvB >> 10) & 7;
#pragma unroll
            for (int k = 0; k < RPG; ++k) {
                const uint32_t pos = (k < 3 ? (cvA >> (10 * k)) & 1023u : cvB & 1023u) * 16;
                if (k < cnt) {
                    const bool in_map = !((cvB >> (13 + k)) & 1u);
#pragma unroll
                    for (int j = 0; j < J1; ++j) write_row(j, pos, in_map, raw[j][k]);
                }
            }
            set_rd = RPG * SLOT - set_rd;
            wait_rows();
            block_barrier();
        }
        wait_vmem(0);                                                  // no load into this block's LDS outlives it
        return;
    }

    // ---- pass waves
    block_barrier();
    unsigned char* o_slot = smem + a.off_out + wave * SLOT;
    const int VD = 4 * PS;
    const unsigned char* tap_base = smem + g * PS;
    const unsigned char* a1v = smem + a.off_a1v + lane * 16;
    const int st_c = 16 * ((lane >> 4) & 1) + (lane & 15), st_hh = lane >> 5;
    char* dq_base = (char*)(a.dq + head_base + (long)y0 * W) + (uint32_t)st_c * hw2;
    _Float16* a_base = a.attn + (long)plane * S * HW + (long)y0 * W;
    _Float16* dl_base = a.dl + (long)plane * S * HW + (long)y0 * W;
    const int q_rd = (8 * g + (p >> 2)) * 32 + (p & 3) * 8;            // the lane's piece of a [32 channels][16 pixels] slot
    const float4_t zero4 = {0.0f, 0.0f, 0.0f, 0.0f};
    // lane (p, g) holds the shifts g, 4 + g, 8 + g of pixel p
    float* part_out = MODE == 1 ? a.part + (long)plane * 2 * S * HW + (long)y0 * W : nullptr;
    const float* part_own = MODE == 2 ? a.part + (long)plane * 2 * S * HW + (long)y0 * W : nullptr;
    const float* part_in = MODE == 2 ? a.part + (long)(plane ^ 1) * 2 * S * HW + (long)y0 * W : nullptr;
    int nb = 16 * wave;
    for (int e = 0; e < E; ++e) {
        const uint32_t p2 = __builtin_amdgcn_readlane(t_p2, e);
        if (p2 & 256u) {
            float sh_l[3] = {0.0f, 0.0f, 0.0f}, sh_da[3] = {0.0f, 0.0f, 0.0f};   // MODE 2: the two halves' shares, added
            if (MODE == 2) {
#pragma unroll
                for (int r = 0; r < 3; ++r) {
                    const bool has = nb + p < npix && (r < 2 || g == 0);
                    const long at = (long)(4 * r + g) * HW + nb + p;
                    sh_l[r] = has ? part_own[at] + part_in[at] : 0.0f;
                    sh_da[r] = has ? part_own[at + (long)S * HW] + part_in[at + (long)S * HW] : 0.0f;
                }
            }
            const uint32_t p0 = __builtin_amdgcn_readlane(t_p0, e), p1 = __builtin_amdgcn_readlane(t_p1, e);
            const int cx0 = (int)(p2 & 255u) + p;
            const bool next_row = cx0 >= W;
            const uint32_t cx = next_row ? cx0 - W : cx0;
            const uint32_t rows = next_row ? p1 : p0;
            const unsigned char* kb[KS];
#pragma unroll
            for (int ty = 0; ty < KS; ++ty) kb[ty] = tap_base + ((((rows >> (10 * ty)) & 1023u) + cx) << 4);
            const int slot = wave * (2 * SLOT) + (e & 1) * SLOT + q_rd;
            uint2_t q0 = {0u, 0u}, q1 = {0u, 0u}, d0 = {0u, 0u}, d1 = {0u, 0u};
            uint4_t xd[S];
            const half2_t sc = {(_Float16)G_SCALE, (_Float16)G_SCALE};
            half2_t xs[4];
            float4_t acc = zero4, accb = zero4;
            if (MODE != 2) {
            q0 = lds_read_tr(smem + a.off_q + slot); q1 = lds_read_tr(smem + a.off_q + slot + 4 * 32);
            d0 = lds_read_tr(smem + a.off_do + slot); d1 = lds_read_tr(smem + a.off_do + slot + 4 * 32);
#pragma unroll
            for (int t = 0; t < S; ++t) xd[t] = *(const uint4_t*)(kb[t / KS] + (t % KS) * 16);
            xs[0] = as_half2(bf16x2_to_half2(q0[0])) * sc; xs[1] = as_half2(bf16x2_to_half2(q0[1])) * sc;
            xs[2] = as_half2(bf16x2_to_half2(q1[0])) * sc; xs[3] = as_half2(bf16x2_to_half2(q1[1])) * sc;
            // ---- attention weights (as in the forward)
#pragma unroll
            for (int t = 0; t < S; ++t) {
                uint4_t bb;
#pragma unroll
                for (int y = 0; y < 4; ++y) bb[y] = as_dword(xs[y] * as_half2(xd[t][y]));
                if (t & 1) accb = __builtin_amdgcn_mfma_f32_16x16x32_f16(A1k[t], __builtin_bit_cast(half8_t, bb), accb, 0, 0, 0);
                else       acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(A1k[t], __builtin_bit_cast(half8_t, bb), acc, 0, 0, 0);
            }
            acc += accb;
            // v taps for the da step (not before the K products are formed: the two sets of taps
            // do not fit into the registers together)
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int t = 0; t < S; ++t) xd[t] = *(const uint4_t*)(kb[t / KS] + VD + (t % KS) * 16);
            }
            float l[3], pr[3];
#pragma unroll
            for (int r = 0; r < 3; ++r) l[r] = MODE == 2 ? sh_l[r] + bias2[r] : fmaf(acc[r], a.scale_log2e, bias2[r]);
            const float lg_own[3] = {acc[0] * a.scale_log2e, acc[1] * a.scale_log2e, acc[2] * a.scale_log2e};
            const float mx = allmax_groups(fmaxf(fmaxf(l[0], l[1]), l[2]));
#pragma unroll
            for (int r = 0; r < 3; ++r) pr[r] = __builtin_amdgcn_exp2f(l[r] - mx);
            const float inv = __builtin_amdgcn_rcpf(allsum_groups(pr[0] + pr[1] + pr[2]));
#pragma unroll
            for (int r = 0; r < 3; ++r) pr[r] *= inv;
            // ---- da[s] = dO . Vs[s], then dl
            if (MODE != 2) {
            xs[0] = as_half2(bf16x2_to_half2(d0[0])) * sc; xs[1] = as_half2(bf16x2_to_half2(d0[1])) * sc;
            xs[2] = as_half2(bf16x2_to_half2(d1[0])) * sc; xs[3] = as_half2(bf16x2_to_half2(d1[1])) * sc;
            acc = zero4; accb = zero4;
#pragma unroll
            for (int t = 0; t < S; ++t) {
                const half8_t A1v = __builtin_bit_cast(half8_t, *(const uint4_t*)(a1v + t * 1024));
                uint4_t bb;
#pragma unroll
                for (int y = 0; y < 4; ++y) bb[y] = as_dword(xs[y] * as_half2(xd[t][y]));
                if (t & 1) accb = __builtin_amdgcn_mfma_f32_16x16x32_f16(A1v, __builtin_bit_cast(half8_t, bb), accb, 0, 0, 0);
                else       acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(A1v, __builtin_bit_cast(half8_t, bb), acc, 0, 0, 0);
            }
            acc += accb;
            }
            if (MODE == 1) {
                if (nb + p < npix) {
#pragma unroll
                    for (int r = 0; r < 3; ++r) {
                        if (r < 2 || g == 0) {
                            part_out[(long)(4 * r + g) * HW + nb + p] = lg_own[r];
                            part_out[(long)(S + 4 * r + g) * HW + nb + p] = acc[r];
                        }
                    }
                }
            } else {
            if (MODE == 2) {
#pragma unroll
                for (int r = 0; r < 3; ++r) acc[r] = sh_da[r];
            }
            // k taps again for the dq step
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int t = 0; t < S; ++t) xd[t] = *(const uint4_t*)(kb[t / KS] + (t % KS) * 16);
            const float dsum = allsum_groups(pr[0] * acc[0] + pr[1] * acc[1] + pr[2] * acc[2]);
            float dl[3];
#pragma unroll
            for (int r = 0; r < 3; ++r) dl[r] = pr[r] * (acc[r] - dsum);
            if (nb + p < npix) {
#pragma unroll
                for (int r = 0; r < 3; ++r) {
                    if (r < 2 || g == 0) {
                        const long at = (long)(4 * r + g) * HW + nb + p;
                        a_base[at] = (_Float16)pr[r];
                        dl_base[at] = (_Float16)dl[r];
                    }
                }
            }
            // ---- dq[c] = scale * sum_t k[c,p+t] * (sum_s dl[s] W~k[c,s,t]): the inner sum on the
            // matrix core, each product two products ahead of the multiply-adds that use it
            uint2_t b2;
            b2[0] = pack_half(dl[0], dl[1]);
            b2[1] = pack_half(dl[2], 0.0f);
            const half4_t B2 = __builtin_bit_cast(half4_t, b2);
            float o[8];
#pragma unroll
            for (int x = 0; x < 8; ++x) o[x] = 0.0f;
            float4_t w[2 * S];
            constexpr int AHEAD = 2;
#pragma unroll
            for (int uu = 0; uu < AHEAD; ++uu) w[uu] = __builtin_amdgcn_mfma_f32_16x16x16f16(A2k[uu], B2, zero4, 0, 0, 0);
#pragma unroll
            for (int uu = 0; uu < 2 * S; ++uu) {
                if (uu + AHEAD < 2 * S) w[uu + AHEAD] = __builtin_amdgcn_mfma_f32_16x16x16f16(A2k[uu + AHEAD], B2, zero4, 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int x = uu < 16 ? (uu & 7) : 4 * (uu - 16) + r;
                    const int tap = uu < 16 ? 4 * (uu >> 3) + r : 8;
                    o[x] = fmaf(w[uu][r], (float)as_half2(xd[tap][x >> 1])[x & 1], o[x]);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            uint4_t ov;
#pragma unroll
            for (int y = 0; y < 4; ++y) {
                typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
                typedef float float2_t __attribute__((ext_vector_type(2)));
                const float2_t f2 = {o[2 * y] * a.scale, o[2 * y + 1] * a.scale};
                ov[y] = __builtin_bit_cast(uint32_t, __builtin_convertvector(f2, bf16x2_t));
            }
            *(uint4_t*)(o_slot + p * 64 + ((g ^ ((p >> 2) & 3)) << 4)) = ov;
            const int grp = lane >> 4, nn = lane & 15;
            const int sa = nn & 3, sj = nn >> 2;
            const int oct_s = 2 * (grp & 1) + (sa >> 1);
            const int P0 = 8 * st_hh + sj, P1 = P0 + 4;
            const uint2_t ra2 = lds_read_tr(o_slot + P0 * 64 + ((oct_s ^ ((P0 >> 2) & 3)) << 4) + (sa & 1) * 8);
            const uint2_t rb2 = lds_read_tr(o_slot + P1 * 64 + ((oct_s ^ ((P1 >> 2) & 3)) << 4) + (sa & 1) * 8);
            const int n0 = nb + 8 * st_hh;
            if (n0 < npix) *(uint4_t*)(dq_base + (uint32_t)n0 * 2u) = uint4_t{ra2[0], ra2[1], rb2[0], rb2[1]};
            }
        }
        nb += PX_EPOCH;
        block_barrier();
    }
}

struct PixelPlan {
    RingRows rr;
    int RS, PS, off_raw, off_dummy, off_q, off_do, off_out, off_a1v, lds_bytes;
    bool ok;
};

static PixelPlan plan_pixel(const Problem& p)
{
    PixelPlan r{};
    r.ok = false;
    r.rr = plan_ring_rows(p, WAVES, 1);
    if (!r.rr.ok) return r;
    const int W = p.W, rpg = r.rr.rpg, R = r.rr.R;
    r.RS = (W + 2) * 16;
    r.PS = R * r.RS;
    r.off_raw = (8 * r.PS + 1023) & ~1023;
    r.off_dummy = r.off_raw + 8 * 2 * rpg * SLOT;
    r.off_q = r.off_dummy + SLOT;
    r.off_do = r.off_q + WAVES * 2 * SLOT;
    r.off_out = r.off_do + WAVES * 2 * SLOT;
    r.off_a1v = r.off_out + WAVES * SLOT;
    r.lds_bytes = r.off_a1v + S * 64 * 16;
    if (4 * r.PS > 65535 - 64) return r;                               // V taps are read at an immediate offset
    r.ok = r.lds_bytes <= LDS_LIMIT;
    return r;
}

}  // namespace b16ring

bool bwd_dkdv_ring_supported(const Problem& p, bool aligned16)
{
    if (!aligned16 || p.dtype != 1 || p.ksize != 3 || p.C != p.heads * t16::D) return false;
    if ((long)p.H * p.W * 2 * t16::D >= (1L << 31)) return false;     // 32-bit byte offsets inside a head
    return b16ring::plan(p).ok;
}

hipError_t launch_bwd_dkdv_ring(const Problem& p, const void* dout, const void* q,
                                const void* attn_ws, const void* dl_ws, void* dk, void* dv,
                                const void* image_ws, hipStream_t st)
{
    using namespace b16ring;
    const Plan r = plan(p);
    if (!r.ok) return hipErrorInvalidValue;
    Args a;
    a.q = (const bf16_bits*)q; a.dout = (const bf16_bits*)dout;
    a.attn = (const _Float16*)attn_ws; a.dl = (const _Float16*)dl_ws;
    a.dk = (bf16_bits*)dk; a.dv = (bf16_bits*)dv;
    a.image = (const uint32_t*)image_ws;
    a.B = p.B; a.H = p.H; a.W = p.W; a.C = p.C; a.heads = p.heads;
    a.nbp = r.rr.nbp; a.rows_pb = r.rr.rows_pb; a.n_blocks = r.rr.n_blocks;
    a.R = r.rr.R; a.RS = r.RS; a.PS = r.PS;
    a.off_raw = r.off_raw; a.off_rraw = r.off_rraw; a.off_dummy = r.off_dummy; a.off_rec = r.off_rec;
    a.off_out = r.off_out;
    a.magic_w = (uint32_t)(((1ULL << 32) + p.W - 1) / p.W);
    a.magic_r = (uint32_t)(((1ULL << 32) + r.rr.R - 1) / r.rr.R);
    a.scale = p.logit_scale();
    static LdsOptIn opt_in;
    hipError_t e = opt_in.ensure({(const void*)bwd16_ring_dkdv_kernel<2>, (const void*)bwd16_ring_dkdv_kernel<3>,
                                  (const void*)bwd16_ring_dkdv_kernel<4>}, t16::LDS_LIMIT);
    if (e != hipSuccess) return e;
    const dim3 grid((unsigned)r.rr.n_blocks), block(THREADS);
    if (r.rr.rpg == 2) hipLaunchKernelGGL(bwd16_ring_dkdv_kernel<2>, grid, block, (size_t)r.lds_bytes, st, a);
    else if (r.rr.rpg == 3) hipLaunchKernelGGL(bwd16_ring_dkdv_kernel<3>, grid, block, (size_t)r.lds_bytes, st, a);
    else hipLaunchKernelGGL(bwd16_ring_dkdv_kernel<4>, grid, block, (size_t)r.lds_bytes, st, a);
    return hipGetLastError();
}


bool bwd_pixel_ring_supported(const Problem& p, bool aligned16)
{
    if (!aligned16 || p.dtype != 1 || p.ksize != 3 || p.C != p.heads * t16::D) return false;
    if ((long)p.H * p.W * 2 * t16::D >= (1L << 31)) return false;     // 32-bit byte offsets inside a head
    return b16ring::plan_pixel(p).ok;
}

hipError_t launch_bwd_pixel_ring(const Problem& p, const void* dout, const void* q, const void* k,
                                 const void* v, void* dq, void* attn_ws, void* dl_ws,
                                 const void* image_ws, hipStream_t st, int mode, float* part)
{
    using namespace b16ring;
    const PixelPlan r = plan_pixel(p);
    if (!r.ok) return hipErrorInvalidValue;
    PixelArgs a;
    a.q = (const bf16_bits*)q; a.k = (const bf16_bits*)k; a.v = (const bf16_bits*)v; a.dout = (const bf16_bits*)dout;
    a.dq = (bf16_bits*)dq; a.attn = (_Float16*)attn_ws; a.dl = (_Float16*)dl_ws;
    a.image = (const uint32_t*)image_ws;
    a.B = p.B; a.H = p.H; a.W = p.W; a.C = p.C; a.heads = p.heads;
    a.nbp = r.rr.nbp; a.rows_pb = r.rr.rows_pb; a.n_blocks = r.rr.n_blocks;
    a.R = r.rr.R; a.RS = r.RS; a.PS = r.PS;
    a.off_raw = r.off_raw; a.off_dummy = r.off_dummy; a.off_q = r.off_q; a.off_do = r.off_do;
    a.off_out = r.off_out; a.off_a1v = r.off_a1v;
    a.magic_w = (uint32_t)(((1ULL << 32) + p.W - 1) / p.W);
    a.magic_r = (uint32_t)(((1ULL << 32) + r.rr.R - 1) / r.rr.R);
    a.scale = p.logit_scale();
    a.scale_log2e = 1.44269504088896341f * p.logit_scale();
    a.part = part;
    if (mode < 0 || mode > 2 || (mode != 0 && !part)) return hipErrorInvalidValue;
    static LdsOptIn opt_in;
#define SLIDE_PX_KERNELS(RPGV) (const void*)bwd16_ring_pixel_kernel<RPGV, 0>, (const void*)bwd16_ring_pixel_kernel<RPGV, 1>, \
                               (const void*)bwd16_ring_pixel_kernel<RPGV, 2>
    hipError_t e = opt_in.ensure({SLIDE_PX_KERNELS(2), SLIDE_PX_KERNELS(3), SLIDE_PX_KERNELS(4)}, t16::LDS_LIMIT);
#undef SLIDE_PX_KERNELS
    if (e != hipSuccess) return e;
    const dim3 grid((unsigned)r.rr.n_blocks), block(THREADS);
#define SLIDE_PX_LAUNCH(RPGV)                                                                                      \
    do {                                                                                                           \
        if (mode == 0)      hipLaunchKernelGGL((bwd16_ring_pixel_kernel<RPGV, 0>), grid, block, (size_t)r.lds_bytes, st, a); \
        else if (mode == 1) hipLaunchKernelGGL((bwd16_ring_pixel_kernel<RPGV, 1>), grid, block, (size_t)r.lds_bytes, st, a); \
        else                hipLaunchKernelGGL((bwd16_ring_pixel_kernel<RPGV, 2>), grid, block, (size_t)r.lds_bytes, st, a); \
    } while (0)
    if (r.rr.rpg == 2) SLIDE_PX_LAUNCH(2);
    else if (r.rr.rpg == 3) SLIDE_PX_LAUNCH(3);
    else SLIDE_PX_LAUNCH(4);
#undef SLIDE_PX_LAUNCH
    return hipGetLastError();
}

}  // namespace slide
