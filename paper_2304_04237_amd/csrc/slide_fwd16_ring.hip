// Streaming matrix-core forward of Slide Attention for gfx950: bf16 activations, head size
// 32, 3x3 window, maps of 32..64 columns (a multiple of 8) whose rows and pointers are
// 16-byte aligned; wider maps as column strips of up to 48 (template argument STRIP), heads of 24
// channels with an empty fourth octet (DH), heads of 64 as two half heads (MODE).  Same arithmetic as the tiled kernels (operator of Sec. 4.1-4.3 with the
// merged kernel W~ of Sec. 4.3 / Fig. 4 as matrix-core operands, see slide_fwd16_ops.h); what
// differs is how data moves:
//
//   - A block owns a band of consecutive rows of one (batch, head) plane and walks down it.
//     K and V rows live in LDS in a ring of R rows: eight planes (tensor x channel octet),
//     each [ring row][column][8 channels as halves], 16 B per pixel, so the nine taps of a
//     pixel are three row addresses plus constant offsets and neighbouring lanes read
//     neighbouring 16-byte slots.  Every row is staged exactly once per block; the zero
//     padding left and right of the map are two ring columns that are cleared once, the rows
//     above and below the map are staged as zeros (Fig. 2).
//   - Work is cut into epochs of 128 pixels: eight pass waves run one 16-pixel pass each, four
//     mover waves do the data movement around them.  One block barrier ends the epoch.  The
//     ring is deep enough that rows written during an epoch are never among those read
//     during it.
//   - Global memory is read with 16-byte loads that write straight into LDS
//     (global_load_lds_dwordx4): the raw bf16 rows of a K/V unit (tensor x channel octet) land
//     channel-major in the landing slots of the mover that owns the unit and use no registers
//     while in flight.  Two epochs later the mover reads the slots back with the transposing
//     LDS read (ds_read_b64_tr_b16: a lane gets four channels of one pixel), converts
//     bf16 -> half, writes the ring rows that the next epoch reads first, and re-issues loads
//     into the slots for the epoch after that.  The head's kernels arrive the same way and
//     are turned into the operand image in LDS.
//   - q is private to the pass that uses it: one direct-to-LDS load per pass (issued by a
//     mover two epochs ahead) into a slot of the pass wave, read back transposed.  Results go
//     the other way: a lane writes its pixel's 8 channels to a per-wave slot, reads 8 pixels
//     of one channel back transposed, and puts them into a buffer of the block from which,
//     one barrier later, the movers store 256 contiguous bytes per channel.
//
// Vector-memory waits are placed by hand: the direct-to-LDS loads are issued from inline
// assembly (the compiler would otherwise make every LDS read wait for them), and every epoch
// issues the same number of them per mover, so "all but the latest round have landed" is one
// constant wait.
#include "slide_fwd16_ops.h"

namespace slide {
namespace f16ring {
using namespace t16;
using namespace f16ops;

constexpr int MIN_W = 32, MAX_W = 64;
constexpr int WAVES = 8, THREADS = WAVES * 64;
constexpr int PX_EPOCH = WAVES * 16;           // pixels per epoch
constexpr int SLOT = 1024;                     // bytes of a landing slot: 8 channels x 64 pixels or 32 channels x 16 pixels

struct RingArgs {
    const bf16_bits* q; const bf16_bits* k; const bf16_bits* v; bf16_bits* out;
    float* lse;                                // [B, heads, H, W] or null
    const float* wk; const float* wv; const float* bias;
    int B, H, W, C, heads;
    int d;                                     // channels per head: 32, or 24 (the fourth octet of every unit is then empty: zeros in, nothing out)
    int nbp, rows_pb, n_blocks;                // bands per plane, rows per band, blocks
    int R, RS, PS;                             // ring rows, bytes per ring row = (W + 2) * 16, bytes per unit plane = R * RS
    int off_raw, off_dummy, off_q, off_out, off_out2;   // LDS byte offsets: K/V landing slots, dump slot, q slots, per-wave result slots, the block's two result buffers
    uint32_t magic_w, magic_r;                 // ceil(2^32 / W), ceil(2^32 / R): x / W == umulhi(x, magic_w) for x < 2^26
    float scale_log2e, idw;
    float* part;                               // heads of 64 channels (MODE 1, 2): partial logits of every half head, [B, 2 heads, 9, H, W], times scale_log2e
    int Wf, n_strips;                          // STRIP: columns of the whole map (W is the strip's width), strips per plane
};

// RPG: most rows a group of new K/V rows can have (rows that one epoch is the first to read).
// Twelve waves per block: waves 0 .. 7 ("pass waves") only run passes; waves 8 .. 11 ("movers")
// do all of the data movement around them.  Mover j stages octet j of K and of V (fetch of the
// landed rows, conversion, ring rows, loads of later groups), issues the q loads of pass waves
// 2j and 2j + 1 and stores channels 8j .. 8j + 7 of the previous epoch's results.  A pass wave
// issues about 280 instructions per epoch, and three waves share a SIMD (under 168 registers).
// The epoch loops have no data-dependent control flow beyond "this wave has a pass": a mover
// issues exactly 2 RPG + 2 loads per epoch (rows a group does not have, rows outside the map
// and passes past the end of the band are loaded from a valid address into a dump slot), its
// stores go out before them, and it waits at the END of an epoch until only the loads of that
// epoch are in flight: what the next epoch reads -- q in the pass waves, rows in the mover --
// has landed before the barrier.
//
// PLAIN: the shift without learned kernels (Sec. 4.2, Eq. 10-13: every shift is a one-hot
// depthwise kernel, so the shifted keys and values are the taps themselves).  No kernels are
// read and no operand image is built; the matrix core only adds the 32 channel products of a
// tap, and every lane holds all nine logits of its pixel.
//
// MODE: heads of 64 channels run as two half heads of 32 (the arguments then describe twice as
// many heads; bias and lse are indexed by the pair) in two launches.  The logit of Eq. 2 is a
// sum over the channels of the head, so MODE 1 only forms each half head's share of the nine
// logits (key side; nothing else is computed or stored, no value rows are staged) and writes it
// to `part`; MODE 2 is the rest of the kernel (no q, no key rows, no key-side products): a pass
// adds the two halves' shares, so both halves get the same attention weights, and applies them
// to its own 32 value channels.  MODE 0: heads of DH channels, one launch.
constexpr int MOVERS = 4, WAVES12 = WAVES + MOVERS, THREADS12 = WAVES12 * 64;

template <int RPG, bool LSE, bool PLAIN, int DH, int MODE = 0, bool STRIP = false>
__global__ void __launch_bounds__(THREADS12)
fwd16_ring_kernel(const RingArgs a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool mover = wave >= WAVES;
    const int mv = wave - WAVES;                                       // mover index 0 .. 3
    const int p = lane & 15, g = lane >> 4;
    // W: columns a block works on, the whole row, or (STRIP) a strip of a wider map of Wf columns
    const int W = a.W, H = a.H, R = a.R;
    const int Wf = STRIP ? a.Wf : W;
    const int RS = a.RS, PS = a.PS;
    const uint32_t hw2 = (uint32_t)H * (uint32_t)Wf * 2u;            // bytes of one channel plane
    const uint32_t w2 = (uint32_t)Wf * 2u;
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem;

    // ---- block -> band of rows of one plane.  Consecutive block indices are dealt round-robin to
    // the XCDs by the hardware; the bands of a plane (which share two halo rows) get indices
    // 8 apart, so they run on the same XCD and the shared rows come out of its L2.
    int u = blockIdx.x;
    {
        const int per = a.n_blocks >> 3;
        if (u < 8 * per) u = (u & 7) * per + (u >> 3);
    }
    const int plane_s = u / a.nbp, part = u - plane_s * a.nbp;        // (plane, strip) and band
    const int plane = STRIP ? plane_s / a.n_strips : plane_s;
    // first column of the strip; the last strip is moved left so that it ends with the map (the
    // columns it shares with the strip before it are computed twice, with identical results)
    const int x0 = STRIP ? min((plane_s - plane * a.n_strips) * W, Wf - W) : 0;
    const int b = plane / a.heads, m = plane - b * a.heads;
    const int y0 = part * a.rows_pb;
    const int nr = min(a.rows_pb, H - y0);
    const long HW = (long)H * Wf;
    const long head_base = ((long)b * a.C + (long)m * DH) * HW;   // element offset of channel 0 of the head
    const bool oct_empty = DH < D && mover && 8 * mv >= DH;         // this mover's octet does not exist
    const int npix = nr * W, npass = (npix + 15) >> 4, E = (npass + WAVES - 1) / WAVES;

    auto div_w = [&](int x) { return (int)__umulhi((uint32_t)x, a.magic_w); };
    auto mod_r = [&](int x) { return x - (int)__umulhi((uint32_t)x, a.magic_r) * R; };
    auto srn = [&](int j) {
        const int rb = min(div_w(PX_EPOCH * j + PX_EPOCH - 1), nr - 1);
        return j >= E ? nr + 1 : min(rb + 2, nr + 1);
    };

    // ---- mover: K/V staging of units j = 0 (K), 1 (V), octet mv
    const int oct = mover ? mv : 0;
    const int src_oct = oct_empty ? 0 : oct;
    const bf16_bits* kv_src[2] = {a.k + head_base + (long)(8 * src_oct) * HW, a.v + head_base + (long)(8 * src_oct) * HW};
    // a row of a unit lands as [8 channels][WL pixels]; STRIP: the strip and the 8 pixels either
    // side of it (WL = W + 16 <= 64), of which the ring takes one column left and right
    const int WL = STRIP ? W + 16 : W;
    const int NXC = WL >> 3;
    const int kv_cc = lane / NXC, kv_x = lane - kv_cc * NXC;
    const int kv_col = x0 - 8 + 8 * kv_x;                            // STRIP: first map column of the lane's 16 bytes
    const bool kv_lane = STRIP ? (lane < 8 * NXC && kv_col >= 0 && kv_col < Wf) : lane < W;
    const uint32_t kv_lane_off = STRIP ? (uint32_t)kv_cc * hw2 + (uint32_t)max(kv_col, 0) * 2u
                                       : (uint32_t)kv_cc * hw2 + (uint32_t)kv_x * 16u;
    // ring column that the lane's landed pixel goes to: lane + 1, or (STRIP) lane - 7
    const bool ring_lane = STRIP ? (lane >= 7 && lane <= W + 8) : lane < W;
    const bool ring_zero = STRIP && (x0 - 8 + lane < 0 || x0 - 8 + lane >= Wf);   // a column outside the map
    // landing slots of unit j: two sets of RPG; at start-up also the third q slot and the result
    // slot of pass wave 2 mv + j
    auto slot_off = [&](int j, int s) {
        const int raw = a.off_raw + (4 * j + oct) * (2 * RPG * SLOT);
        const int pw = 2 * oct + j;
        return s < 2 * RPG ? raw + s * SLOT : (s == 2 * RPG ? a.off_q + pw * (3 * SLOT) + 2 * SLOT : a.off_out + pw * SLOT);
    };
    // (an empty octet reads channel 0 of the head's first octet into the dump slot)
    auto load_row = [&](int j, uint32_t row_off, int off) {
        if (kv_lane) load_to_lds(kv_src[j], kv_lane_off + row_off, lds0 + (oct_empty ? a.off_dummy : off));
    };
    const int cv_src_off = ((lane & 15) >> 2) * (WL * 2) + (16 * (lane >> 4) + 4 * (lane & 3)) * 2;
    struct RawRow { uint2_t lo, hi; };
    auto read_row = [&](int off) {
        RawRow r;
        const unsigned char* src = smem + off + cv_src_off;
        r.lo = lds_read_tr(src);
        r.hi = lds_read_tr(src + 4 * (WL * 2));
        return r;
    };
    auto write_row = [&](int j, uint32_t ring_off, bool in_map, const RawRow& r) {
        uint4_t h4;
        h4[0] = bf16x2_to_half2(r.lo[0]); h4[1] = bf16x2_to_half2(r.lo[1]);
        h4[2] = bf16x2_to_half2(r.hi[0]); h4[3] = bf16x2_to_half2(r.hi[1]);
#pragma unroll
        for (int y = 0; y < 4; ++y) h4[y] = (in_map && !oct_empty && !ring_zero) ? h4[y] : 0u;
        if (ring_lane) *(uint4_t*)(smem + (4 * j + oct) * PS + (STRIP ? lane - 7 : lane + 1) * 16 + ring_off) = h4;
    };
    auto write_row_in_map = [&](int j, uint32_t ring_off, const RawRow& r) {
        uint4_t h4;
        h4[0] = bf16x2_to_half2(r.lo[0]); h4[1] = bf16x2_to_half2(r.lo[1]);
        h4[2] = bf16x2_to_half2(r.hi[0]); h4[3] = bf16x2_to_half2(r.hi[1]);
        if (STRIP) {
#pragma unroll
            for (int y = 0; y < 4; ++y) h4[y] = ring_zero ? 0u : h4[y];
        }
        if (ring_lane) *(uint4_t*)(smem + (4 * j + oct) * PS + (STRIP ? lane - 7 : lane + 1) * 16 + ring_off) = h4;
    };
    // q of pass wave pw, pass starting at band pixel n_first, into slot offset qo of that wave
    // band pixel n (a multiple of 8) -> byte offset inside a channel plane, from the band's first row
    auto px_off = [&](int n) {
        if (!STRIP) return (uint32_t)n * 2u;
        const int r = div_w(n);
        return (uint32_t)(r * Wf + x0 + (n - r * W)) * 2u;
    };
    const bf16_bits* q_src = a.q + head_base + (long)y0 * Wf;
    const uint32_t q_lane_off = (uint32_t)(lane >> 1) * hw2 + (STRIP ? 0u : (uint32_t)(lane & 1) * 16u);
    auto load_q = [&](int pw, int n_first, int qo) {
        const bool real = n_first < npix;
        const int nf = real ? n_first : 0;
        const int off = real ? a.off_q + pw * (3 * SLOT) + qo : a.off_dummy;
        if (nf + 8 * (lane & 1) < npix && (lane >> 1) < DH)
            load_to_lds(q_src, q_lane_off + (STRIP ? px_off(nf + 8 * (lane & 1)) : (uint32_t)nf * 2u), lds0 + off);
    };

    // ---- start-up.  The first access to a tensor takes microseconds (cold translation): the
    // bias is fetched first thing, next to the kernels, not where it is used.
    float bias_early = 0.0f;                                           // PLAIN: bias of shift `lane`; else the image's bias word of logit row `tid`
    const int mb = MODE ? m >> 1 : m;                                  // head that the bias and lse belong to
    if (a.bias && !mover && MODE != 1) {
        if (PLAIN) { if (lane < S) bias_early = a.bias[mb * S + lane]; }
        else if (tid < IMG_DWORDS - IMG_BIAS && shift_of_row(tid) >= 0) bias_early = a.bias[mb * S + shift_of_row(tid)];
    }
    // tensors a mover stages: K (j = 0) unless the logits come in whole, V (j = 1) unless only logits are formed
    constexpr int J0 = MODE == 2 ? 1 : 0, J1 = MODE == 1 ? 1 : 2, NJ = J1 - J0;
    constexpr bool HAS_Q = MODE != 2;                                  // q is loaded (the key side is computed)
    const int v0 = srn(0), v1 = srn(1), v2 = srn(2);
    int n_after_g0 = 0;                                                // mover: loads issued after group 0
    if (!PLAIN && !mover) {
        // 2 x 32 x 81 floats = 1296 chunks of 16 bytes, K kernels then V kernels; with 24 channels
        // per head the chunks of channels 24 .. 31 are zeros
        constexpr int CHUNKS = HEAD_W / 4;
        const int head_w = DH * S * S, chunks_d = head_w / 4;
        for (int L = wave; L * 64 < 2 * CHUNKS; L += WAVES) {
            const int c = L * 64 + lane;
            const int cc = c >= CHUNKS ? c - CHUNKS : c;
            const float* src = (c >= CHUNKS ? a.wv : a.wk) + (long)m * head_w + 4 * cc;
            if (c < 2 * CHUNKS) {
                if (DH == D || cc < chunks_d) load_to_lds_addr(src, lds0 + IMG_RAW_AT + L * 1024);
                else *(uint4_t*)(smem + IMG_RAW_AT + c * 16) = uint4_t{0u, 0u, 0u, 0u};
            }
        }
    }
    if (mover) {
        for (int k = 0; k <= v0; ++k) {                                // group 0 (at most RPG + 2 rows)
            const int gy = y0 - 1 + k;
            if (gy >= 0 && gy < H)
                for (int j = J0; j < J1; ++j) load_row(j, (uint32_t)gy * w2, slot_off(j, k < RPG ? k : 2 * RPG + (k - RPG)));
        }
        if (HAS_Q) {
            for (int i = 0; i < 2; ++i) {
                load_q(2 * mv + i, 16 * (2 * mv + i), 0);
                load_q(2 * mv + i, 16 * (2 * mv + i) + PX_EPOCH, SLOT);
            }
            n_after_g0 = 4;
        }
        for (int k = 0; k < v1 - v0; ++k) {                            // group 1 into set 1
            const int gy = y0 + v0 + k;
            if (gy >= 0 && gy < H) {
                for (int j = J0; j < J1; ++j) load_row(j, (uint32_t)gy * w2, slot_off(j, RPG + k));
                n_after_g0 += NJ;
            }
        }
    }
    half8_t A1[S];
    half4_t A2[2 * S];
    float bias2[3];
    float bias9[S];
    if (!PLAIN) {
        if (!mover) wait_vmem(0);                                      // the kernels have landed
        block_barrier();
        if (tid < THREADS) {
            image_from_raw<THREADS>((const float*)(smem + IMG_RAW_AT), nullptr, m, a.idw, (uint32_t*)smem, tid);
            if (tid < IMG_DWORDS - IMG_BIAS)                           // (overwrites the zero-bias words that image_from_raw wrote)
                ((uint32_t*)smem)[IMG_BIAS + tid] = __float_as_uint(shift_of_row(tid) >= 0 ? bias_early * 1.44269504088896341f : -INFINITY);
        }
        block_barrier();
        if (!mover) load_operands((const uint32_t*)smem, lane, g, A1, A2, bias2);
        block_barrier();
    } else if (!mover) {
#pragma unroll
        for (int t = 0; t < S; ++t) bias9[t] = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(bias_early), t)) * 1.44269504088896341f;
    }
    for (int idx = tid; idx < R * 16; idx += THREADS12) {              // the padding columns of the ring stay zero
        const int unit = idx & 7, side = (idx >> 3) & 1, row = idx >> 4;
        *(uint4_t*)(smem + unit * PS + row * RS + (side ? W + 1 : 0) * 16) = uint4_t{0u, 0u, 0u, 0u};
    }
    // q slots: the rows of channels the head does not have stay zero (the first two slots of every
    // pass wave here; the third, which holds start-up rows first, by its mover below)
    auto zero_q_rows = [&](int idx0, int n, int stride, int slot_lo, int slots_per_wave) {
        constexpr int per_slot = DH < D ? (D - DH) * 2 : 1;             // 16-byte chunks per slot
        for (int idx = idx0; idx < n * per_slot; idx += stride) {
            const int sl = idx / per_slot, ch = idx - sl * per_slot;
            const int pw = sl / slots_per_wave, s3 = slot_lo + sl % slots_per_wave;
            *(uint4_t*)(smem + a.off_q + pw * (3 * SLOT) + s3 * SLOT + DH * 32 + ch * 16) = uint4_t{0u, 0u, 0u, 0u};
        }
    };
    if (DH < D) zero_q_rows(tid, 2 * WAVES, THREADS12, 0, 2);
    constexpr int NL = NJ * RPG + (HAS_Q ? 2 : 0);                     // loads of a mover per epoch
    if (mover) {
        wait_vmem(n_after_g0);                                         // group 0 has landed
        for (int k = 0; k <= v0; ++k) {                                // group 0 -> ring rows 0 .. v0
            RawRow r0[2];
            for (int j = J0; j < J1; ++j) r0[j] = read_row(slot_off(j, k < RPG ? k : 2 * RPG + (k - RPG)));
            for (int j = J0; j < J1; ++j) write_row(j, (uint32_t)(k * RS), y0 - 1 + k >= 0 && y0 - 1 + k < H, r0[j]);
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");             // set 0 has been read before it is loaded again
        if (DH < D) {                                                 // third q slots of pass waves 2 mv, 2 mv + 1
            constexpr int per_slot = DH < D ? (D - DH) * 2 : 1;
            if (lane < 2 * per_slot) {
                const int pw = 2 * mv + lane / per_slot, ch = lane % per_slot;
                *(uint4_t*)(smem + a.off_q + pw * (3 * SLOT) + 2 * SLOT + DH * 32 + ch * 16) = uint4_t{0u, 0u, 0u, 0u};
            }
        }
        // group 2 into set 0, as a full round of NL loads
#pragma unroll
        for (int k = 0; k < RPG; ++k) {
            const int gy = y0 + v1 + k;
            const bool real = k < v2 - v1 && gy >= 0 && gy < H;
            for (int j = J0; j < J1; ++j)
                load_row(j, (uint32_t)min(max(gy, 0), H - 1) * w2, real ? slot_off(j, k) : a.off_dummy);
        }
        if (HAS_Q) {
            load_q(0, npix, 0);
            load_q(0, npix, 0);                                        // (two dump loads complete the round)
        }
        wait_vmem(NL);                                                 // everything but that round: group 1, q of epochs 0 and 1
    }
    block_barrier();

    // ---- the schedule: everything uniform that an epoch needs, worked out once, lane e of the
    // table registers holding epoch e (E <= 64).  Ring positions are in 16-byte units (10 bits).
    //   t_cvA, t_cvB: ring positions of the rows of group e + 1 (converted during epoch e), their
    //                 number, which of them lie outside the map (written as zeros), and which
    //                 loads of group e + 3 are real
    //   t_ld:         byte offset of the first row of group e + 3 inside a channel plane
    //   t_p0, t_p1:   ring positions of the three tap rows of this wave's pass, for lanes that stay
    //                 in the pass's first row / that run into the next row
    //   t_p2:         column of the pass's first pixel; bit 8: the wave has a pass
    uint32_t t_cvA, t_cvB, t_ld, t_p0, t_p1, t_p2;
    {
        const int e = lane;
        const int s0 = srn(e), s1 = srn(e + 1), s2 = srn(e + 2), s3 = srn(e + 3);
        const int RW = W + 2;
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
        t_ld = (uint32_t)(min(max(y0 + s2, 0), H - 1) * Wf) * 2u;
        const int nbe = PX_EPOCH * e + 16 * (mover ? 0 : wave);
        const int ra = div_w(nbe), c0 = nbe - ra * W;
        t_p0 = ring_of(ra) | ring_of(ra + 1) << 10 | ring_of(ra + 2) << 20;
        t_p1 = ring_of(ra + 1) | ring_of(ra + 2) << 10 | ring_of(ra + 3) << 20;
        t_p2 = (uint32_t)c0 | (nbe < npix ? 256u : 0u);
    }

    constexpr int OUT_ROW = 2 * PX_EPOCH + 16;
    char* out_base = (char*)(a.out + head_base + (long)y0 * Wf);
    int out2_wr = a.off_out2, out2_rd = a.off_out2 + 32 * OUT_ROW;     // buffer written this epoch / stored this epoch
    int qo_cur = 0, qo_1 = SLOT, qo_2 = 2 * SLOT;                      // slot offsets of q(e), q(e+1), q(e+2)
    // mover: store channels 8 mv .. 8 mv + 7 of the epoch whose first pixel is e0 from buffer rd
    auto store_results = [&](int e0, int rd) {
        uint4_t val[2];
        const int n0 = e0 + 8 * (lane & 15);
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int c = 8 * mv + 4 * i + (lane >> 4);
            if (n0 < npix && (DH == D || c < DH)) val[i] = *(const uint4_t*)(smem + rd + c * OUT_ROW + (lane & 15) * 16);
        }
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int c = 8 * mv + 4 * i + (lane >> 4);
            if (n0 < npix && (DH == D || c < DH)) *(uint4_t*)(out_base + ((uint32_t)c * hw2 + px_off(n0))) = val[i];
        }
    };

    if (mover) {
        // A mover has few instructions per epoch, each waiting for the one before (LDS read, store,
        // load, conversion): they go ahead of the two pass waves on its SIMD, or the pass waves
        // finish their epoch first and then wait for the mover at the barrier.
        __builtin_amdgcn_s_setprio(3);
        int set_rd = RPG * SLOT;                                       // offset of the set that holds group e + 1
        for (int e = 0; e < E; ++e) {
            const uint32_t cvA = __builtin_amdgcn_readlane(t_cvA, e), cvB = __builtin_amdgcn_readlane(t_cvB, e);
            const uint32_t ldo = __builtin_amdgcn_readlane(t_ld, e);
            // group e + 1 has landed (waited for at the end of the previous epoch): fetch it
            RawRow raw[2][RPG];
#pragma unroll
            for (int j = J0; j < J1; ++j)
#pragma unroll
                for (int k = 0; k < RPG; ++k) raw[j][k] = read_row(slot_off(j, 0) + set_rd + k * SLOT);
            if (MODE != 1 && e > 0) store_results(PX_EPOCH * (e - 1), out2_rd);   // (contains the wait for its LDS reads)
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            // the epoch's round of loads: group e + 3 into the slots just read, q(e + 2) of two pass waves
#pragma unroll
            for (int k = 0; k < RPG; ++k) {
                const bool real = (cvB >> (17 + k)) & 1u;
#pragma unroll
                for (int j = J0; j < J1; ++j)
                    load_row(j, real ? ldo + (uint32_t)k * w2 : ldo, real ? slot_off(j, 0) + set_rd + k * SLOT : a.off_dummy);
            }
            if (HAS_Q) {
#pragma unroll
                for (int i = 0; i < 2; ++i) load_q(2 * mv + i, PX_EPOCH * (e + 2) + 16 * (2 * mv + i), qo_2);
            }
            // conversion of group e + 1 into the ring
            const int cnt = (cvB >> 10) & 7;
            if (((cvB >> 13) & 15u) == 0 && !oct_empty) {              // every row inside the map: the usual case
#pragma unroll
                for (int k = 0; k < RPG; ++k) {
                    const uint32_t pos = (k < 3 ? (cvA >> (10 * k)) & 1023u : cvB & 1023u) * 16;
                    if (k < cnt) {
#pragma unroll
                        for (int j = J0; j < J1; ++j) write_row_in_map(j, pos, raw[j][k]);
                    }
                }
            } else {
#pragma unroll
                for (int k = 0; k < RPG; ++k) {
                    const uint32_t pos = (k < 3 ? (cvA >> (10 * k)) & 1023u : cvB & 1023u) * 16;
                    if (k < cnt) {
#pragma unroll
                        for (int j = J0; j < J1; ++j) write_row(j, pos, !((cvB >> (13 + k)) & 1u), raw[j][k]);
                    }
                }
            }
            set_rd = RPG * SLOT - set_rd;
            { const int t = out2_wr; out2_wr = out2_rd; out2_rd = t; }
            { const int t = qo_cur; qo_cur = qo_1; qo_1 = qo_2; qo_2 = t; }
            if (NL == 2) asm volatile("s_waitcnt vmcnt(2)" ::: "memory");
            else if (NL == 3) asm volatile("s_waitcnt vmcnt(3)" ::: "memory");
            else if (NL == 4) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
            else if (NL == 5) asm volatile("s_waitcnt vmcnt(5)" ::: "memory");
            else if (NL == 6) asm volatile("s_waitcnt vmcnt(6)" ::: "memory");
            else if (NL == 8) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
            else asm volatile("s_waitcnt vmcnt(10)" ::: "memory");
            block_barrier();
        }
        if (MODE != 1) store_results(PX_EPOCH * (E - 1), out2_rd);
        wait_vmem(0);                                                  // no load into this block's LDS outlives it
        return;
    }

    // ---- pass waves
    const int q_slots = a.off_q + wave * (3 * SLOT);
    unsigned char* o_slot = smem + a.off_out + wave * SLOT;
    const int VD = 4 * PS;
    const unsigned char* tap_base = smem + g * PS;
    const int st_c = 16 * ((lane >> 4) & 1) + (lane & 15), st_hh = lane >> 5;
    int nb = 16 * wave;
    float* lse_ptr = LSE ? a.lse + ((long)(MODE ? plane >> 1 : plane) * H + y0) * Wf : nullptr;
    auto lse_at = [&](int n) {                                         // band pixel -> index from the band's first row
        if (!STRIP) return n;
        const int r = div_w(n);
        return r * Wf + x0 + (n - r * W);
    };
    // MODE 1: this half head's share of the logits goes out; MODE 2: the other half's comes in,
    // fetched one epoch ahead (lane (p, g) holds the shifts g, 4 + g, 8 + g of pixel p)
    float* part_out = MODE == 1 ? a.part + (long)plane * S * HW + (long)y0 * W : nullptr;
    const float* part_own = MODE == 2 ? a.part + (long)plane * S * HW + (long)y0 * W : nullptr;
    const float* part_in = MODE == 2 ? a.part + (long)(plane ^ 1) * S * HW + (long)y0 * W : nullptr;
    float oth[3] = {0.0f, 0.0f, 0.0f};                                 // the two halves' shares, added
    auto fetch_shares = [&](int n_first) {
#pragma unroll
        for (int r = 0; r < 3; ++r) {
            const bool has = n_first + p < npix && (r < 2 || g == 0);
            const long at = (long)(4 * r + g) * HW + n_first + p;
            oth[r] = has ? part_own[at] + part_in[at] : 0.0f;
        }
    };
    if (MODE == 2) fetch_shares(nb);
    for (int e = 0; e < E; ++e) {
        const uint32_t p2 = __builtin_amdgcn_readlane(t_p2, e);
        if (p2 & 256u) {
            const uint32_t p0 = __builtin_amdgcn_readlane(t_p0, e), p1 = __builtin_amdgcn_readlane(t_p1, e);
            const int cx0 = (int)(p2 & 255u) + p;
            const bool next_row = cx0 >= W;
            const uint32_t cx = next_row ? cx0 - W : cx0;
            const uint32_t rows = next_row ? p1 : p0;
            const unsigned char* kb[KS];
#pragma unroll
            for (int ty = 0; ty < KS; ++ty) kb[ty] = tap_base + ((((rows >> (10 * ty)) & 1023u) + cx) << 4);
            const unsigned char* qsrc = smem + q_slots + qo_cur + (8 * g + (p >> 2)) * 32 + (p & 3) * 8;
            uint2_t q0 = {0u, 0u}, q1 = {0u, 0u};
            uint4_t kd[S];
            if (HAS_Q) {
                q0 = lds_read_tr(qsrc); q1 = lds_read_tr(qsrc + 4 * 32);
#pragma unroll
                for (int t = 0; t < S; ++t) kd[t] = *(const uint4_t*)(kb[t / KS] + (t % KS) * 16);
            }
            half2_t qs[4];
            if (HAS_Q) {
                const half2_t sc = {(_Float16)G_SCALE, (_Float16)G_SCALE};
                qs[0] = as_half2(bf16x2_to_half2(q0[0])) * sc; qs[1] = as_half2(bf16x2_to_half2(q0[1])) * sc;
                qs[2] = as_half2(bf16x2_to_half2(q1[0])) * sc; qs[3] = as_half2(bf16x2_to_half2(q1[1])) * sc;
            }
            float o[8];
#pragma unroll
            for (int x = 0; x < 8; ++x) o[x] = 0.0f;
            if (PLAIN) {
                const uint32_t c16 = 0x4c004c00u;
                const half8_t ones = __builtin_bit_cast(half8_t, uint4_t{c16, c16, c16, c16});
                const float4_t zero4 = {0.0f, 0.0f, 0.0f, 0.0f};
                float l[S];
#pragma unroll
                for (int t = 0; t < S; ++t) {
                    uint4_t bb;
#pragma unroll
                    for (int y = 0; y < 4; ++y) bb[y] = as_dword(qs[y] * as_half2(kd[t][y]));
                    const float4_t dsum = __builtin_amdgcn_mfma_f32_16x16x32_f16(ones, __builtin_bit_cast(half8_t, bb), zero4, 0, 0, 0);
                    l[t] = dsum[0];
                }
                uint4_t vd[S];
#pragma unroll
                for (int t = 0; t < S; ++t) vd[t] = *(const uint4_t*)(kb[t / KS] + VD + (t % KS) * 16);
                float mx = -INFINITY;
#pragma unroll
                for (int t = 0; t < S; ++t) { l[t] = fmaf(l[t], a.scale_log2e, bias9[t]); mx = fmaxf(mx, l[t]); }
                float den = 0.0f;
#pragma unroll
                for (int t = 0; t < S; ++t) { l[t] = __builtin_amdgcn_exp2f(l[t] - mx); den += l[t]; }
                const float inv = __builtin_amdgcn_rcpf(den);
                if (LSE) { if (g == 0 && nb + p < npix) lse_ptr[lse_at(nb + p)] = LN2 * (mx + __builtin_amdgcn_logf(den)); }
#pragma unroll
                for (int t = 0; t < S; ++t)
#pragma unroll
                    for (int x = 0; x < 8; ++x) o[x] = fmaf(l[t], (float)as_half2(vd[t][x >> 1])[x & 1], o[x]);
#pragma unroll
                for (int x = 0; x < 8; ++x) o[x] *= inv;
            } else {
                // (two accumulation chains, even and odd taps: a product does not wait for the one before it)
                float4_t acc1 = {0.0f, 0.0f, 0.0f, 0.0f}, acc1b = {0.0f, 0.0f, 0.0f, 0.0f};
                if (HAS_Q) {
#pragma unroll
                for (int t = 0; t < S; ++t) {
                    uint4_t bb;
#pragma unroll
                    for (int y = 0; y < 4; ++y) bb[y] = as_dword(qs[y] * as_half2(kd[t][y]));
                    if (t & 1) acc1b = __builtin_amdgcn_mfma_f32_16x16x32_f16(A1[t], __builtin_bit_cast(half8_t, bb), acc1b, 0, 0, 0);
                    else       acc1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(A1[t], __builtin_bit_cast(half8_t, bb), acc1, 0, 0, 0);
                }
                acc1 += acc1b;
                }
                if (MODE == 1) {
                    if (nb + p < npix) {
#pragma unroll
                        for (int r = 0; r < 3; ++r)
                            if (r < 2 || g == 0) part_out[(long)(4 * r + g) * HW + nb + p] = acc1[r] * a.scale_log2e;
                    }
                } else {
                uint4_t vd[S];
#pragma unroll
                for (int t = 0; t < S; ++t) vd[t] = *(const uint4_t*)(kb[t / KS] + VD + (t % KS) * 16);
                float l[3];
#pragma unroll
                for (int r = 0; r < 3; ++r) l[r] = MODE == 2 ? oth[r] + bias2[r] : fmaf(acc1[r], a.scale_log2e, bias2[r]);
                if (MODE == 2) fetch_shares(nb + PX_EPOCH);
                const float mx = allmax_groups(fmaxf(fmaxf(l[0], l[1]), l[2]));
                float pr[3];
#pragma unroll
                for (int r = 0; r < 3; ++r) pr[r] = __builtin_amdgcn_exp2f(l[r] - mx);
                const float den = allsum_groups(pr[0] + pr[1] + pr[2]);
                const float inv = __builtin_amdgcn_rcpf(den);
                if (LSE) { if (g == 0 && nb + p < npix && (MODE != 2 || (m & 1) == 0)) lse_ptr[lse_at(nb + p)] = LN2 * (mx + __builtin_amdgcn_logf(den)); }
                uint2_t b2;
                b2[0] = pack_half(pr[0] * inv, pr[1] * inv);
                b2[1] = pack_half(pr[2] * inv, 0.0f);
                const half4_t B2 = __builtin_bit_cast(half4_t, b2);
                const float4_t zero4 = {0.0f, 0.0f, 0.0f, 0.0f};
                float4_t w[2 * S];
                constexpr int AHEAD = 2;
#pragma unroll
                for (int uu = 0; uu < AHEAD; ++uu) w[uu] = __builtin_amdgcn_mfma_f32_16x16x16f16(A2[uu], B2, zero4, 0, 0, 0);
#pragma unroll
                for (int uu = 0; uu < 2 * S; ++uu) {
                    if (uu + AHEAD < 2 * S)
                        w[uu + AHEAD] = __builtin_amdgcn_mfma_f32_16x16x16f16(A2[uu + AHEAD], B2, zero4, 0, 0, 0);
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int x = uu < 16 ? (uu & 7) : 4 * (uu - 16) + r;
                        const int tap = uu < 16 ? 4 * (uu >> 3) + r : 8;
                        o[x] = fmaf(w[uu][r], (float)as_half2(vd[tap][x >> 1])[x & 1], o[x]);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
                }
            }
            if (MODE != 1) {
            uint4_t ov;
#pragma unroll
            for (int y = 0; y < 4; ++y) {
                typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
                typedef float float2_t __attribute__((ext_vector_type(2)));
                const float2_t f2 = {o[2 * y], o[2 * y + 1]};
                ov[y] = __builtin_bit_cast(uint32_t, __builtin_convertvector(f2, bf16x2_t));
            }
            *(uint4_t*)(o_slot + p * 64 + ((g ^ ((p >> 2) & 3)) << 4)) = ov;
            const int grp = lane >> 4, nn = lane & 15;
            const int sa = nn & 3, sj = nn >> 2;
            const int oct_s = 2 * (grp & 1) + (sa >> 1);
            const int P0 = 8 * st_hh + sj, P1 = P0 + 4;
            const uint2_t ra2 = lds_read_tr(o_slot + P0 * 64 + ((oct_s ^ ((P0 >> 2) & 3)) << 4) + (sa & 1) * 8);
            const uint2_t rb2 = lds_read_tr(o_slot + P1 * 64 + ((oct_s ^ ((P1 >> 2) & 3)) << 4) + (sa & 1) * 8);
            *(uint4_t*)(smem + out2_wr + st_c * OUT_ROW + (16 * wave + 8 * st_hh) * 2) = uint4_t{ra2[0], ra2[1], rb2[0], rb2[1]};
            }
        }
        { const int t = out2_wr; out2_wr = out2_rd; out2_rd = t; }
        { const int t = qo_cur; qo_cur = qo_1; qo_1 = qo_2; qo_2 = t; }
        nb += PX_EPOCH;
        block_barrier();
    }
}

// ------------------------------------------------------------------ channels-last activations
// The same kernel for q, k, v, out stored [B, H, W, C] (NHWC, the layout of [B, HW, C] token
// tensors): the 8 channels of a pixel that a lane works on are 16 contiguous bytes, so nothing
// is transposed.  A mover loads the K/V rows of its 16-column group (lane = pixel x channel
// octet, 64 contiguous bytes per pixel and head) and a quarter of every epoch's q into
// registers two epochs ahead; it converts the rows into the ring and passes q on through a
// small LDS buffer in the order the pass waves read it (16 bytes per lane, no transposition).
// A pass wave stores its results straight from its registers.  LDS holds the ring and the q
// buffer only.  All loads are ordinary loads whose waits the compiler places; the movers'
// epoch loop is unrolled by two so that the two register sets in flight alternate by name.
// NW pass waves and NM movers per block.  8 + 4 is what is launched (one block per compute unit,
// epochs of 128 pixels); 4 + 2 with two blocks per compute unit and epochs of 64 pixels was
// measured slower (39 against 30 us at stage 1: twice the epochs, barriers and halo rows).
template <int RPG, bool LSE, int NW, int NM>
__global__ void __launch_bounds__((NW + NM) * 64, 3)
fwd16_ring_nhwc_kernel(const RingArgs a)
{
    constexpr int PXE = 16 * NW;                                       // pixels per epoch
    constexpr int CG = 4 / NM;                                         // 16-column groups per mover
    constexpr int NTH = (NW + NM) * 64, PTH = NW * 64;                 // threads of the block, of its pass waves
    static_assert(NW == 2 * NM && (NM == 4 || NM == 2), "q is dealt two items per mover lane and epoch");
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool mover = wave >= NW;
    const int mv = wave - NW;                                          // mover index
    const int p = lane & 15, g = lane >> 4;
    const int W = a.W, H = a.H, R = a.R, C = a.C;
    const int RS = a.RS, PS = a.PS;

    int u = blockIdx.x;                                                // block -> band of a plane, as above
    {
        const int per = a.n_blocks >> 3;
        if (u < 8 * per) u = (u & 7) * per + (u >> 3);
    }
    const int plane = u / a.nbp, part = u - plane * a.nbp;
    const int b = plane / a.heads, m = plane - b * a.heads;
    const int y0 = part * a.rows_pb;
    const int nr = min(a.rows_pb, H - y0);
    const int npix = nr * W, npass = (npix + 15) >> 4, E = (npass + NW - 1) / NW;
    // byte offset of channel 0 of the head at pixel 0 of batch item b; a pixel is 2 C bytes on
    const size_t img_base = ((size_t)b * H * W * C + (size_t)m * D) * 2;
    const uint32_t px2 = (uint32_t)C * 2u, row2 = (uint32_t)W * px2;

    auto div_w = [&](int x) { return (int)__umulhi((uint32_t)x, a.magic_w); };
    auto mod_r = [&](int x) { return x - (int)__umulhi((uint32_t)x, a.magic_r) * R; };
    auto srn = [&](int j) {
        const int rb = min(div_w(PXE * j + PXE - 1), nr - 1);
        return j >= E ? nr + 1 : min(rb + 2, nr + 1);
    };

    // ---- the schedule, lane e of the table registers holding epoch e (see fwd16_ring_kernel)
    uint32_t t_cvA, t_cvB, t_ld, t_p0, t_p1, t_p2;
    {
        const int e = lane;
        const int s0 = srn(e), s1 = srn(e + 1), s2 = srn(e + 2);
        const int RW = W + 2;
        auto ring_of = [&](int sr) { return (uint32_t)(mod_r(sr) * RW); };
        t_cvA = ring_of(s0 + 1) | ring_of(s0 + 2) << 10 | ring_of(s0 + 3) << 20;
        uint32_t outside = 0;
#pragma unroll
        for (int k = 0; k < RPG; ++k) {
            const int gy = y0 + s0 + k;
            outside |= (gy < 0 || gy >= H) ? 1u << k : 0u;
        }
        t_cvB = ring_of(s0 + 4) | (uint32_t)(s1 - s0) << 10 | outside << 13 | (uint32_t)(srn(e + 3) - s2) << 17;
        t_ld = (uint32_t)max(y0 + s2, 0);                              // map row of the first row of group e + 3
        const int nbe = PXE * e + 16 * (mover ? 0 : wave);
        const int ra = div_w(nbe), c0 = nbe - ra * W;
        t_p0 = ring_of(ra) | ring_of(ra + 1) << 10 | ring_of(ra + 2) << 20;
        t_p1 = ring_of(ra + 1) | ring_of(ra + 2) << 10 | ring_of(ra + 3) << 20;
        t_p2 = (uint32_t)c0 | (nbe < npix ? 256u : 0u);
    }
    const int v0 = srn(0), v1 = srn(1), v2 = srn(2);
    const int E2 = (E + 1) & ~1;                                       // both loops run an even number of epochs (the last may be empty)

    // The two kinds of waves part here for good (their registers never coexist); both pass the same
    // four start-up barriers and one barrier per epoch.
    if (mover) {
        __builtin_amdgcn_s_setprio(3);                                 // (as in fwd16_ring_kernel: the movers go first)
        // columns 16 mv .. 16 mv + 15, lane = pixel (lane / 4) x octet (lane % 4)
        // Every load is unconditional (lanes and rows that have nothing to fetch read a valid
        // address and get zeros afterwards): straight-line code, in which the compiler counts the
        // loads in flight exactly and waits only for the ones it uses.
        // (a mover owns CG groups of 16 columns; item (j, c): tensor j, its c-th group)
        const int m_oct = lane & 3;
        const int m_px0 = 16 * CG * mv + (lane >> 2);                  // the lane's column in the mover's first group
        const char* kv_base[2] = {(const char*)a.k + img_base + m_oct * 16, (const char*)a.v + img_base + m_oct * 16};
        // map row gy (clamped into the map) of item (j, c): the lane's 8 channels.  Nothing is done to
        // the value here: whatever touches it would wait for the load.
        auto load_item = [&](int jc, int gy) {
            const int px = min(m_px0 + 16 * (jc % CG), W - 1);
            return *(const uint4_t*)(kv_base[jc / CG] + (size_t)min(max(gy, 0), H - 1) * row2 + (size_t)px * px2);
        };
        // (in_map false: the row lies above or below the map and is written as zeros, Fig. 2)
        auto write_item = [&](int jc, uint32_t ring_off, bool in_map, const uint4_t& r) {
            const int px = m_px0 + 16 * (jc % CG);
            uint4_t h4;
#pragma unroll
            for (int y = 0; y < 4; ++y) h4[y] = in_map ? bf16x2_to_half2(r[y]) : 0u;
            if (px < W) *(uint4_t*)(smem + (4 * (jc / CG) + m_oct) * PS + (px + 1) * 16 + ring_off) = h4;
        };
        // q: pixels 32 mv .. 32 mv + 31 of every epoch, two items per lane
        const char* q_base = (const char*)a.q + img_base + (size_t)y0 * row2 + m_oct * 16;
        auto load_q = [&](int e, int i) {                              // (zeros past the band)
            const int n = PXE * e + 32 * mv + 16 * i + (lane >> 2);
            return *(const uint4_t*)(q_base + (size_t)min(n, npix - 1) * px2);   // (past the band: some pixel; nothing of it is stored)
        };
        auto write_q = [&](int e, int i, const uint4_t& r) {
            *(uint4_t*)(smem + a.off_q + (e & 1) * (PXE * 64) + ((32 * mv + 16 * i) * 4 + lane) * 16) = r;
        };
        // q of epochs 0 and 1, group 0 (at most RPG + 2 rows) and group 1 are issued before anything is
        // used; q of epoch 2 and group 2 take the place of what the start-up has consumed
        uint4_t q0[2], qa[2], qb[2];
#pragma unroll
        for (int i = 0; i < 2; ++i) { q0[i] = load_q(0, i); qa[i] = load_q(1, i); }
        uint4_t g0[RPG + 2][2 * CG], ga[RPG][2 * CG], gb[RPG][2 * CG];
#pragma unroll
        for (int k = 0; k < RPG + 2; ++k) {
            const int gy = y0 - 1 + k;
#pragma unroll
            for (int j = 0; j < 2 * CG; ++j) g0[k][j] = load_item(j, gy);
        }
#pragma unroll
        for (int k = 0; k < RPG; ++k) {
            const int gy = y0 + v0 + k;
#pragma unroll
            for (int j = 0; j < 2 * CG; ++j) ga[k][j] = load_item(j, gy);
        }
        block_barrier();                                               // (the head's kernels are in LDS)
        block_barrier();                                               // (the operand image is built)
        block_barrier();                                               // (the operands are in registers: the ring's memory is free)
#pragma unroll
        for (int k = 0; k < RPG + 2; ++k)
            if (k <= v0) {
#pragma unroll
                for (int j = 0; j < 2 * CG; ++j) write_item(j, (uint32_t)(k * RS), y0 - 1 + k >= 0 && y0 - 1 + k < H, g0[k][j]);
            }
#pragma unroll
        for (int i = 0; i < 2; ++i) write_q(0, i, q0[i]);
#pragma unroll
        for (int k = 0; k < RPG; ++k) {
            const int gy = y0 + v1 + k;
#pragma unroll
            for (int j = 0; j < 2 * CG; ++j) gb[k][j] = load_item(j, gy);
        }
#pragma unroll
        for (int i = 0; i < 2; ++i) qb[i] = load_q(2, i);
        block_barrier();
        // epoch e: the rows of group e + 1 and q of epoch e + 1 (loaded two epochs ago) go into LDS,
        // the loads of group e + 3 and of q of epoch e + 3 take their registers
        auto mover_epoch = [&](int e, uint4_t (&cur)[RPG][2 * CG], uint4_t (&qcur)[2]) {
            const uint32_t cvA = __builtin_amdgcn_readlane(t_cvA, e), cvB = __builtin_amdgcn_readlane(t_cvB, e);
            const int gy0 = (int)__builtin_amdgcn_readlane(t_ld, e);
            const int cnt = (cvB >> 10) & 7;
#pragma unroll
            for (int k = 0; k < RPG; ++k) {
                const uint32_t pos = (k < 3 ? (cvA >> (10 * k)) & 1023u : cvB & 1023u) * 16;
                if (k < cnt) {
#pragma unroll
                    for (int j = 0; j < 2 * CG; ++j) write_item(j, pos, !((cvB >> (13 + k)) & 1u), cur[k][j]);
                }
            }
            const int n_new = (int)((cvB >> 17) & 7u);                 // rows of group e + 3; loads beyond it read its first row again (cache hits)
#pragma unroll
            for (int k = 0; k < RPG; ++k)
#pragma unroll
                for (int j = 0; j < 2 * CG; ++j) cur[k][j] = load_item(j, gy0 + (k < n_new ? k : 0));
#pragma unroll
            for (int i = 0; i < 2; ++i) { write_q(e + 1, i, qcur[i]); qcur[i] = load_q(e + 3, i); }
            block_barrier();
        };
        for (int e = 0; e < E2; e += 2) {
            mover_epoch(e, ga, qa);
            mover_epoch(e + 1, gb, qb);
        }
        return;
    }

    // ---- pass waves: the bias and q of the first two epochs first (the first access to a tensor
    // takes microseconds), then the head's kernels into LDS (behind where the operand image
    // goes), the image, the operands
    float bias_early = 0.0f;                                           // the image's bias word of logit row `tid`
    if (a.bias && tid < IMG_DWORDS - IMG_BIAS && shift_of_row(tid) >= 0) bias_early = a.bias[m * S + shift_of_row(tid)];
    char* o_base = (char*)a.out + img_base + (size_t)y0 * row2 + g * 16;
    {
        constexpr int CHUNKS = HEAD_W / 4;
        for (int c = tid; c < 2 * CHUNKS; c += PTH) {
            const float* src = (c >= CHUNKS ? a.wv + (long)m * HEAD_W + 4 * (c - CHUNKS) : a.wk + (long)m * HEAD_W + 4 * c);
            *(float4_t*)(smem + IMG_RAW_AT + c * 16) = *(const float4_t*)src;
        }
    }
    block_barrier();
    // (image_from_raw is written for 512 threads: 256 threads run it twice)
    for (int t512 = tid; t512 < THREADS; t512 += PTH)
        image_from_raw<THREADS>((const float*)(smem + IMG_RAW_AT), nullptr, m, a.idw, (uint32_t*)smem, t512);
    if (tid < IMG_DWORDS - IMG_BIAS)
        ((uint32_t*)smem)[IMG_BIAS + tid] = __float_as_uint(shift_of_row(tid) >= 0 ? bias_early * 1.44269504088896341f : -INFINITY);
    block_barrier();
    half8_t A1[S];
    half4_t A2[2 * S];
    float bias2[3];
    load_operands((const uint32_t*)smem, lane, g, A1, A2, bias2);
    block_barrier();
    for (int idx = tid; idx < R * 16; idx += PTH) {                    // the padding columns of the ring stay zero
        const int unit = idx & 7, side = (idx >> 3) & 1, row = idx >> 4;
        *(uint4_t*)(smem + unit * PS + row * RS + (side ? W + 1 : 0) * 16) = uint4_t{0u, 0u, 0u, 0u};
    }
    block_barrier();

    // ---- pass waves
    const int VD = 4 * PS;
    const unsigned char* tap_base = smem + g * PS;
    float* lse_ptr = LSE ? a.lse + ((long)plane * H + y0) * W : nullptr;
    const unsigned char* q_lds = smem + a.off_q + ((16 * wave + p) * 4 + g) * 16;
    for (int e = 0; e < E2; ++e) {
        const uint32_t p2 = __builtin_amdgcn_readlane(t_p2, e);
        const int nb = PXE * e + 16 * wave;
        if (p2 & 256u) {
            const uint4_t qraw = *(const uint4_t*)(q_lds + (e & 1) * (PXE * 64));
            const uint32_t p0 = __builtin_amdgcn_readlane(t_p0, e), p1 = __builtin_amdgcn_readlane(t_p1, e);
            const int cx0 = (int)(p2 & 255u) + p;
            const bool next_row = cx0 >= W;
            const uint32_t cx = next_row ? cx0 - W : cx0;
            const uint32_t rows = next_row ? p1 : p0;
            const unsigned char* kb[KS];
#pragma unroll
            for (int ty = 0; ty < KS; ++ty) kb[ty] = tap_base + ((((rows >> (10 * ty)) & 1023u) + cx) << 4);
            uint4_t kd[S];
#pragma unroll
            for (int t = 0; t < S; ++t) kd[t] = *(const uint4_t*)(kb[t / KS] + (t % KS) * 16);
            half2_t qs[4];
            {
                const half2_t sc = {(_Float16)G_SCALE, (_Float16)G_SCALE};
#pragma unroll
                for (int y = 0; y < 4; ++y) qs[y] = as_half2(bf16x2_to_half2(qraw[y])) * sc;
            }
            float4_t acc1 = {0.0f, 0.0f, 0.0f, 0.0f}, acc1b = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
            for (int t = 0; t < S; ++t) {
                uint4_t bb;
#pragma unroll
                for (int y = 0; y < 4; ++y) bb[y] = as_dword(qs[y] * as_half2(kd[t][y]));
                if (t & 1) acc1b = __builtin_amdgcn_mfma_f32_16x16x32_f16(A1[t], __builtin_bit_cast(half8_t, bb), acc1b, 0, 0, 0);
                else       acc1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(A1[t], __builtin_bit_cast(half8_t, bb), acc1, 0, 0, 0);
            }
            acc1 += acc1b;
            uint4_t vd[S];
#pragma unroll
            for (int t = 0; t < S; ++t) vd[t] = *(const uint4_t*)(kb[t / KS] + VD + (t % KS) * 16);
            float l[3];
#pragma unroll
            for (int r = 0; r < 3; ++r) l[r] = fmaf(acc1[r], a.scale_log2e, bias2[r]);
            const float mx = allmax_groups(fmaxf(fmaxf(l[0], l[1]), l[2]));
            float pr[3];
#pragma unroll
            for (int r = 0; r < 3; ++r) pr[r] = __builtin_amdgcn_exp2f(l[r] - mx);
            const float den = allsum_groups(pr[0] + pr[1] + pr[2]);
            const float inv = __builtin_amdgcn_rcpf(den);
            if (LSE) { if (g == 0 && nb + p < npix) lse_ptr[nb + p] = LN2 * (mx + __builtin_amdgcn_logf(den)); }
            uint2_t b2;
            b2[0] = pack_half(pr[0] * inv, pr[1] * inv);
            b2[1] = pack_half(pr[2] * inv, 0.0f);
            const half4_t B2 = __builtin_bit_cast(half4_t, b2);
            const float4_t zero4 = {0.0f, 0.0f, 0.0f, 0.0f};
            float4_t w[2 * S];
            float o[8];
#pragma unroll
            for (int x = 0; x < 8; ++x) o[x] = 0.0f;
            constexpr int AHEAD = 2;
#pragma unroll
            for (int uu = 0; uu < AHEAD; ++uu) w[uu] = __builtin_amdgcn_mfma_f32_16x16x16f16(A2[uu], B2, zero4, 0, 0, 0);
#pragma unroll
            for (int uu = 0; uu < 2 * S; ++uu) {
                if (uu + AHEAD < 2 * S)
                    w[uu + AHEAD] = __builtin_amdgcn_mfma_f32_16x16x16f16(A2[uu + AHEAD], B2, zero4, 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int x = uu < 16 ? (uu & 7) : 4 * (uu - 16) + r;
                    const int tap = uu < 16 ? 4 * (uu >> 3) + r : 8;
                    o[x] = fmaf(w[uu][r], (float)as_half2(vd[tap][x >> 1])[x & 1], o[x]);
                }
                // (pins the multiply-adds here: otherwise they sink below all the products, whose 72 results then live at once)
                if (uu < 16) asm volatile("" : "+v"(o[uu & 7]));
                else asm volatile("" : "+v"(o[4 * (uu - 16)]), "+v"(o[4 * (uu - 16) + 1]), "+v"(o[4 * (uu - 16) + 2]), "+v"(o[4 * (uu - 16) + 3]));
                __builtin_amdgcn_sched_barrier(0);
            }
            uint4_t ov;
#pragma unroll
            for (int y = 0; y < 4; ++y) {
                typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
                typedef float float2_t __attribute__((ext_vector_type(2)));
                const float2_t f2 = {o[2 * y], o[2 * y + 1]};
                ov[y] = __builtin_bit_cast(uint32_t, __builtin_convertvector(f2, bf16x2_t));
            }
            if (nb + p < npix) *(uint4_t*)(o_base + (size_t)(nb + p) * px2) = ov;
        }
        block_barrier();
    }
}

// ------------------------------------------------------------------ host side
struct RingPlan {
    int rpg, nbp, rows_pb, n_blocks, R, RS, PS, off_raw, off_dummy, off_q, off_out, off_out2, lds_bytes;
    bool ok;
};

// nw: pass waves per block (epochs of 16 nw pixels); per_cu: blocks that share a compute unit;
// nhwc: the channels-last kernel (LDS: the ring and two q buffers only)
}  // namespace f16ring

// Bands of rows per plane, ring depth and rows per group of a streaming kernel with nw pass
// waves per block (epochs of 16 nw pixels) and per_cu blocks per compute unit.
RingRows plan_ring_rows(const Problem& p, int nw, int per_cu)
{
    using namespace f16ring;
    RingRows r{};
    r.ok = false;
    const int W = p.W, H = p.H;
    const int pxe = 16 * nw;
    if (W < MIN_W || W > MAX_W || (W % 8) != 0) return r;
    const long planes = (long)p.B * p.heads;
    const int n_cu = device_cu_count() * per_cu;
    // bands per plane: fewest rounds of blocks over the compute units, each round costing a
    // band's rows plus a start-up share
    double best = 1e300;
    int best_nbp = 1;
    for (int nbp = 1; nbp <= H; ++nbp) {
        const int rows = (H + nbp - 1) / nbp;
        if ((long)rows * (nbp - 1) >= H) continue;                      // every band has rows
        if (rows < 4 && nbp > 1) break;
        if (((rows * W + 15) / 16 + nw - 1) / nw > 64) continue;        // the kernel's schedule table holds 64 epochs
        const long blocks = planes * nbp;
        const long rounds = (blocks + n_cu - 1) / n_cu;
        const double cost = (double)rounds * (rows + 6.0);
        if (cost < best - 1e-9) { best = cost; best_nbp = nbp; }
    }
    r.nbp = best_nbp;
    r.rows_pb = (H + r.nbp - 1) / r.nbp;
    if (planes * r.nbp >= (1L << 30)) return r;
    r.n_blocks = (int)(planes * r.nbp);
    // Ring depth: the rows read during epoch e and the rows written during it (group e + 1)
    // must be distinct ring rows: R >= (last row epoch e + 1 reads) - (first row epoch e reads) + 1.
    const int nr = r.rows_pb;
    const int E = ((nr * W + 15) / 16 + nw - 1) / nw;
    if (E > 64) return r;
    auto srn = [&](int e) {
        if (e < 0) return -1;
        if (e >= E) return nr + 1;
        int rb = (pxe * e + pxe - 1) / W;
        if (rb > nr - 1) rb = nr - 1;
        return rb + 2 < nr + 1 ? rb + 2 : nr + 1;
    };
    int need = 3, rpg = 2;
    for (int e = 0; e < E; ++e) {
        const int first = (pxe * e) / W;
        const int cnt = srn(e + 1) - first + 1;
        if (cnt > need) need = cnt;
        if (e >= 1 && srn(e) - srn(e - 1) > rpg) rpg = srn(e) - srn(e - 1);
    }
    if (rpg < srn(0) - 1) rpg = srn(0) - 1;                             // group 0 (srn(0) + 1 rows) fits the rpg + 2 start-up slots
    if (rpg > 4) return r;
    if (need < srn(0) + 2) need = srn(0) + 2;
    r.rpg = rpg;
    r.R = need;
    r.ok = true;
    return r;
}

namespace f16ring {

static RingPlan plan_ring(const Problem& p, int nw = WAVES, int per_cu = 1, bool nhwc = false)
{
    RingPlan r{};
    r.ok = false;
    const RingRows rr = plan_ring_rows(p, nw, per_cu);
    if (!rr.ok) return r;
    const int W = p.W;
    const int pxe = 16 * nw;
    const int rpg = rr.rpg, need = rr.R;
    r.nbp = rr.nbp; r.rows_pb = rr.rows_pb; r.n_blocks = rr.n_blocks;
    r.rpg = rpg;
    r.R = need;
    r.RS = (W + 2) * 16;
    r.PS = r.R * r.RS;
    int ring_bytes = 8 * r.PS;
    if (ring_bytes < IMG_RAW_AT + 21 * 1024) ring_bytes = IMG_RAW_AT + 21 * 1024;   // the raw kernels land in whole 1 KB loads
    r.off_raw = (ring_bytes + 1023) & ~1023;
    r.off_dummy = r.off_raw + WAVES * 2 * rpg * SLOT;
    r.off_q = r.off_dummy + SLOT;
    r.off_out = r.off_q + WAVES * 3 * SLOT;
    r.off_out2 = r.off_out + WAVES * SLOT;
    r.lds_bytes = r.off_out2 + 2 * 32 * (2 * PX_EPOCH + 16);
    if (4 * r.PS > 65535 - 64) return r;                                // V taps are read at an immediate offset
    if (nhwc) {
        int bytes = 8 * r.PS;                                           // the ring (at start-up the operand image and the raw kernels) ...
        if (bytes < IMG_RAW_AT + IMG_RAW_BYTES) bytes = IMG_RAW_AT + IMG_RAW_BYTES;
        r.off_q = (bytes + 255) & ~255;                                 // ... and two q buffers of one epoch's pixels x 64 bytes
        r.lds_bytes = r.off_q + 2 * pxe * 64;
        r.ok = r.lds_bytes * per_cu <= LDS_LIMIT;
        return r;
    }
    r.ok = r.lds_bytes <= LDS_LIMIT;
    return r;
}

// ------------------------------------------------------------------ traffic probes
// The bytes of the forward without its arithmetic, to measure what the memory system gives
// for them.  Results are the bitwise XOR of what was read (so nothing is optimised away).
typedef __attribute__((ext_vector_type(4))) uint32_t probe_u4;

// flat: every thread reads 16 bytes of q, k, v and writes 16 bytes of out, consecutive lanes
// consecutive addresses, persistent blocks striding over the tensors
__global__ void __launch_bounds__(512)
probe_flat_kernel(const probe_u4* __restrict__ q, const probe_u4* __restrict__ k, const probe_u4* __restrict__ v,
                  probe_u4* __restrict__ out, long n16)
{
    for (long i = (long)blockIdx.x * 512 + threadIdx.x; i < n16; i += (long)gridDim.x * 512)
        out[i] = q[i] ^ k[i] ^ v[i];
}

// streaming pattern: the blocks, bands, epochs and per-instruction address shapes of
// fwd16_ring_kernel (a wave loads the new rows of its K/V unit as 8 channels x one row, its
// pass's q as 32 channels x 32 bytes, and stores 4 channels x 256 bytes of the previous
// epoch's pixels), one block barrier per epoch, loads consumed one epoch after their issue
__global__ void __launch_bounds__(THREADS)
probe_stream_kernel(const RingArgs a)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int W = a.W, H = a.H;
    const uint32_t hw2 = (uint32_t)H * (uint32_t)W * 2u;
    int u = blockIdx.x;
    {
        const int per = a.n_blocks >> 3;
        if (u < 8 * per) u = (u & 7) * per + (u >> 3);
    }
    const int plane = u / a.nbp, part = u - plane * a.nbp;
    const int b = plane / a.heads, m = plane - b * a.heads;
    const int y0 = part * a.rows_pb;
    const int nr = min(a.rows_pb, H - y0);
    const long HW = (long)H * W;
    const long head_base = ((long)b * a.C + (long)m * D) * HW;
    const int npix = nr * W, npass = (npix + 15) >> 4, E = (npass + WAVES - 1) / WAVES;
    auto srn = [&](int j) {
        if (j < 0) return -1;
        const int rb = min((int)__umulhi((uint32_t)(PX_EPOCH * j + PX_EPOCH - 1), a.magic_w), nr - 1);
        return j >= E ? nr + 1 : min(rb + 2, nr + 1);
    };
    const char* kv_src = (const char*)(((wave >> 2) ? a.v : a.k) + head_base + (long)(8 * (wave & 3)) * HW);
    const int NXC = W >> 3;
    const int kv_cc = lane / NXC, kv_x = lane - kv_cc * NXC;
    const uint32_t kv_lane_off = (uint32_t)kv_cc * hw2 + (uint32_t)kv_x * 16u;
    const char* q_src = (const char*)(a.q + head_base + (long)y0 * W);
    char* out_base = (char*)(a.out + head_base + (long)y0 * W);
    probe_u4 acc = {0u, 0u, 0u, 0u};
    probe_u4 pend[5];
#pragma unroll
    for (int j = 0; j < 5; ++j) pend[j] = probe_u4{0u, 0u, 0u, 0u};
    for (int e = -1; e < E; ++e) {
#pragma unroll
        for (int j = 0; j < 5; ++j) { acc ^= pend[j]; pend[j] = probe_u4{0u, 0u, 0u, 0u}; }
        // rows that epoch e + 1 is the first to read
        const int lo = srn(e), hi = srn(e + 1);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int gy = y0 + lo + j;
            if (lo + 1 + j <= hi && gy >= 0 && gy < H && lane < W)
                pend[j] = *(const probe_u4*)(kv_src + kv_lane_off + (uint32_t)(gy * W) * 2u);
        }
        for (int sr = lo + 5; sr <= hi; ++sr) {                        // (start-up group: more than four rows)
            const int gy = y0 - 1 + sr;
            if (gy >= 0 && gy < H && lane < W) acc ^= *(const probe_u4*)(kv_src + kv_lane_off + (uint32_t)(gy * W) * 2u);
        }
        const int nq = PX_EPOCH * (e + 1) + 16 * wave + 8 * (lane & 1);
        if (nq < npix) pend[4] = *(const probe_u4*)(q_src + (uint32_t)(lane >> 1) * hw2 + (uint32_t)nq * 2u);
        const int no = PX_EPOCH * e + 8 * (lane & 15);
        if (e >= 0 && no < npix)
            *(probe_u4*)(out_base + (uint32_t)(4 * wave + (lane >> 4)) * hw2 + (uint32_t)no * 2u) = acc;
        __builtin_amdgcn_s_barrier();
    }
}

}  // namespace f16ring

bool fwd_ring_supported(const Problem& p, bool aligned16)
{
    if (!aligned16 || p.dtype != 1 || p.ksize != 3) return false;
    if (p.C != p.heads * f16ring::D && p.C != p.heads * 24) return false;   // head size 32 or 24
    if ((long)p.H * p.W * 2 * f16ring::D >= (1L << 31)) return false;  // 32-bit byte offsets inside a head
    return f16ring::plan_ring(p).ok;
}

hipError_t launch_fwd_ring(const Problem& p, const void* q, const void* k, const void* v,
                           const float* wk, const float* wv, const float* bias, void* out,
                           float* lse, bool plain, hipStream_t st)
{
    using namespace f16ring;
    const RingPlan r = plan_ring(p);
    if (!r.ok) return hipErrorInvalidValue;
    RingArgs a;
    a.q = (const bf16_bits*)q; a.k = (const bf16_bits*)k; a.v = (const bf16_bits*)v;
    a.out = (bf16_bits*)out; a.lse = lse;
    a.wk = wk; a.wv = wv; a.bias = bias;
    a.B = p.B; a.H = p.H; a.W = p.W; a.C = p.C; a.heads = p.heads; a.d = p.C / p.heads;
    a.nbp = r.nbp; a.rows_pb = r.rows_pb; a.n_blocks = r.n_blocks;
    a.R = r.R; a.RS = r.RS; a.PS = r.PS; a.off_raw = r.off_raw; a.off_dummy = r.off_dummy; a.off_q = r.off_q; a.off_out = r.off_out; a.off_out2 = r.off_out2;
    a.magic_w = (uint32_t)(((1ULL << 32) + p.W - 1) / p.W);
    a.magic_r = (uint32_t)(((1ULL << 32) + r.R - 1) / r.R);
    a.scale_log2e = 1.44269504088896341f * p.logit_scale();
    a.idw = p.two_branch ? 1.0f : 0.0f;
    a.part = nullptr; a.Wf = p.W; a.n_strips = 1;
    static LdsOptIn opt_in;
#define SLIDE_RING_KERNELS2(RPGV, DHV)                                                                              \
    (const void*)fwd16_ring_kernel<RPGV, false, false, DHV>, (const void*)fwd16_ring_kernel<RPGV, true, false, DHV>, \
    (const void*)fwd16_ring_kernel<RPGV, false, true, DHV>, (const void*)fwd16_ring_kernel<RPGV, true, true, DHV>
#define SLIDE_RING_KERNELS(RPGV) SLIDE_RING_KERNELS2(RPGV, 32), SLIDE_RING_KERNELS2(RPGV, 24)
    hipError_t e = opt_in.ensure({SLIDE_RING_KERNELS(2), SLIDE_RING_KERNELS(3), SLIDE_RING_KERNELS(4)}, LDS_LIMIT);
#undef SLIDE_RING_KERNELS
#undef SLIDE_RING_KERNELS2
    if (e != hipSuccess) return e;
    const dim3 grid((unsigned)r.n_blocks), block12(THREADS12);
    // (the head size is a compile-time constant of the kernel: 32 pays nothing for the empty octet of 24)
#define SLIDE_RING_LAUNCH4(RPGV, LSEV, PLAINV, DHV)                                                                 \
    hipLaunchKernelGGL((fwd16_ring_kernel<RPGV, LSEV, PLAINV, DHV>), grid, block12, (size_t)r.lds_bytes, st, a)
#define SLIDE_RING_LAUNCH3(RPGV, LSEV, PLAINV)                                                                      \
    do {                                                                                                            \
        if (a.d == 24) SLIDE_RING_LAUNCH4(RPGV, LSEV, PLAINV, 24);                                                  \
        else           SLIDE_RING_LAUNCH4(RPGV, LSEV, PLAINV, 32);                                                  \
    } while (0)
#define SLIDE_RING_LAUNCH2(RPGV, LSEV)                                                                              \
    do {                                                                                                            \
        if (plain) SLIDE_RING_LAUNCH3(RPGV, LSEV, true);                                                            \
        else       SLIDE_RING_LAUNCH3(RPGV, LSEV, false);                                                           \
    } while (0)
#define SLIDE_RING_LAUNCH(RPGV)                                                                                     \
    do {                                                                                                            \
        if (lse) SLIDE_RING_LAUNCH2(RPGV, true);                                                                    \
        else     SLIDE_RING_LAUNCH2(RPGV, false);                                                                   \
    } while (0)
    if (a.d != 24 && a.d != 32) return hipErrorInvalidValue;
    if (r.rpg == 2) SLIDE_RING_LAUNCH(2);
    else if (r.rpg == 3) SLIDE_RING_LAUNCH(3);
    else SLIDE_RING_LAUNCH(4);
#undef SLIDE_RING_LAUNCH2
#undef SLIDE_RING_LAUNCH3
#undef SLIDE_RING_LAUNCH4
#undef SLIDE_RING_LAUNCH
    return hipGetLastError();
}

// ---- maps wider than 64 columns: column strips (the last one moved left to end with the map)
// A strip of Ws columns is loaded as Ws + 16 (at most 64: one landing slot), so Ws is 48, 40 or
// 32; the width that moves the fewest bytes per map column is taken (strips that together cover
// more than 1.25 x the map, or whose ring does not fit, are left to the tile kernels).
static bool strip_problem(const Problem& p, Problem& s, int& n_strips)
{
    double best = 1e300;
    bool found = false;
    for (int ws = 48; ws >= 32; ws -= 8) {
        if (p.W < ws) continue;
        const int n = (p.W + ws - 1) / ws;
        if ((long)n * ws * 100 > (long)p.W * 125) continue;
        const double cost = (double)(ws + 16) / ws * ((double)n * ws / p.W);
        if (cost >= best - 1e-9) continue;
        Problem c = p;
        c.W = ws;
        if ((long)p.B * n * p.heads >= (1L << 24)) continue;
        c.B = p.B * n;                          // (plane, strip) pairs take the place of planes
        if (!f16ring::plan_ring(c).ok) continue;
        best = cost; s = c; n_strips = n; found = true;
    }
    return found;
}

bool fwd_ring_strip_supported(const Problem& p, bool aligned16)
{
    if (!aligned16 || p.dtype != 1 || p.ksize != 3 || p.C != p.heads * f16ring::D) return false;
    if (p.W <= f16ring::MAX_W || p.W % 8 != 0) return false;
    if ((long)p.H * p.W * 2 * f16ring::D >= (1L << 31)) return false;
    int n_strips;
    Problem s;
    return strip_problem(p, s, n_strips);
}

hipError_t launch_fwd_ring_strip(const Problem& p, const void* q, const void* k, const void* v,
                                 const float* wk, const float* wv, const float* bias, void* out,
                                 float* lse, bool plain, hipStream_t st)
{
    using namespace f16ring;
    int n_strips;
    Problem s;
    if (!strip_problem(p, s, n_strips)) return hipErrorInvalidValue;
    const RingPlan r = plan_ring(s);
    if (!r.ok) return hipErrorInvalidValue;
    const int STRIP_W = s.W;
    RingArgs a;
    a.q = (const bf16_bits*)q; a.k = (const bf16_bits*)k; a.v = (const bf16_bits*)v;
    a.out = (bf16_bits*)out; a.lse = lse;
    a.wk = wk; a.wv = wv; a.bias = bias;
    a.B = p.B; a.H = p.H; a.W = STRIP_W; a.C = p.C; a.heads = p.heads; a.d = D;
    a.Wf = p.W; a.n_strips = n_strips;
    a.nbp = r.nbp; a.rows_pb = r.rows_pb; a.n_blocks = r.n_blocks;
    a.R = r.R; a.RS = r.RS; a.PS = r.PS; a.off_raw = r.off_raw; a.off_dummy = r.off_dummy; a.off_q = r.off_q; a.off_out = r.off_out; a.off_out2 = r.off_out2;
    a.magic_w = (uint32_t)(((1ULL << 32) + STRIP_W - 1) / STRIP_W);
    a.magic_r = (uint32_t)(((1ULL << 32) + r.R - 1) / r.R);
    a.scale_log2e = 1.44269504088896341f * p.logit_scale();
    a.idw = p.two_branch ? 1.0f : 0.0f;
    a.part = nullptr;
    static LdsOptIn opt_in;
#define SLIDE_STRIP_KERNELS(RPGV) (const void*)fwd16_ring_kernel<RPGV, false, false, 32, 0, true>, (const void*)fwd16_ring_kernel<RPGV, true, false, 32, 0, true>, \
                                  (const void*)fwd16_ring_kernel<RPGV, false, true, 32, 0, true>, (const void*)fwd16_ring_kernel<RPGV, true, true, 32, 0, true>
    hipError_t e = opt_in.ensure({SLIDE_STRIP_KERNELS(2), SLIDE_STRIP_KERNELS(3), SLIDE_STRIP_KERNELS(4)}, LDS_LIMIT);
#undef SLIDE_STRIP_KERNELS
    if (e != hipSuccess) return e;
    const dim3 grid((unsigned)r.n_blocks), block12(THREADS12);
#define SLIDE_STRIP_LAUNCH(RPGV)                                                                                      \
    do {                                                                                                              \
        if (plain) {                                                                                                  \
            if (lse) hipLaunchKernelGGL((fwd16_ring_kernel<RPGV, true, true, 32, 0, true>), grid, block12, (size_t)r.lds_bytes, st, a);  \
            else     hipLaunchKernelGGL((fwd16_ring_kernel<RPGV, false, true, 32, 0, true>), grid, block12, (size_t)r.lds_bytes, st, a); \
        } else if (lse) hipLaunchKernelGGL((fwd16_ring_kernel<RPGV, true, false, 32, 0, true>), grid, block12, (size_t)r.lds_bytes, st, a);  \
        else     hipLaunchKernelGGL((fwd16_ring_kernel<RPGV, false, false, 32, 0, true>), grid, block12, (size_t)r.lds_bytes, st, a); \
    } while (0)
    if (r.rpg == 2) SLIDE_STRIP_LAUNCH(2);
    else if (r.rpg == 3) SLIDE_STRIP_LAUNCH(3);
    else SLIDE_STRIP_LAUNCH(4);
#undef SLIDE_STRIP_LAUNCH
    return hipGetLastError();
}

// ---- heads of 64 channels (bf16, 3x3): two launches of the streaming kernel over half heads
static Problem half_head_problem(const Problem& p)
{
    Problem h = p;
    h.heads = 2 * p.heads;                      // same C: 32 channels per (half) head
    return h;
}

bool fwd_ring_wide_supported(const Problem& p, bool aligned16)
{
    if (!aligned16 || p.dtype != 1 || p.ksize != 3 || p.C != p.heads * 64) return false;
    if ((long)p.H * p.W * 2 * f16ring::D >= (1L << 31)) return false;
    if ((long)p.B * p.heads * 2 * 9 * p.H * p.W >= (1L << 31)) return false;   // index arithmetic of the partial logits
    return f16ring::plan_ring(half_head_problem(p)).ok;
}

size_t fwd_ring_wide_workspace_bytes(const Problem& p)
{
    return (size_t)p.B * p.heads * 2 * 9 * (size_t)p.plane() * sizeof(float);
}

hipError_t launch_fwd_ring_wide(const Problem& p, const void* q, const void* k, const void* v,
                                const float* wk, const float* wv, const float* bias, void* out,
                                float* lse, void* workspace, hipStream_t st)
{
    using namespace f16ring;
    const Problem h = half_head_problem(p);
    const RingPlan r = plan_ring(h);
    if (!r.ok) return hipErrorInvalidValue;
    RingArgs a;
    a.q = (const bf16_bits*)q; a.k = (const bf16_bits*)k; a.v = (const bf16_bits*)v;
    a.out = (bf16_bits*)out; a.lse = lse;
    a.wk = wk; a.wv = wv; a.bias = bias;
    a.B = h.B; a.H = h.H; a.W = h.W; a.C = h.C; a.heads = h.heads; a.d = D;
    a.nbp = r.nbp; a.rows_pb = r.rows_pb; a.n_blocks = r.n_blocks;
    a.R = r.R; a.RS = r.RS; a.PS = r.PS; a.off_raw = r.off_raw; a.off_dummy = r.off_dummy; a.off_q = r.off_q; a.off_out = r.off_out; a.off_out2 = r.off_out2;
    a.magic_w = (uint32_t)(((1ULL << 32) + h.W - 1) / h.W);
    a.magic_r = (uint32_t)(((1ULL << 32) + r.R - 1) / r.R);
    a.scale_log2e = 1.44269504088896341f / sqrtf(64.0f);               // (the head has 64 channels)
    a.idw = p.two_branch ? 1.0f : 0.0f;
    a.part = (float*)workspace; a.Wf = h.W; a.n_strips = 1;
    static LdsOptIn opt_in;
#define SLIDE_WIDE_KERNELS(RPGV)                                                                                    \
    (const void*)fwd16_ring_kernel<RPGV, false, false, 32, 1>, (const void*)fwd16_ring_kernel<RPGV, false, false, 32, 2>, \
    (const void*)fwd16_ring_kernel<RPGV, true, false, 32, 2>
    hipError_t e = opt_in.ensure({SLIDE_WIDE_KERNELS(2), SLIDE_WIDE_KERNELS(3), SLIDE_WIDE_KERNELS(4)}, LDS_LIMIT);
#undef SLIDE_WIDE_KERNELS
    if (e != hipSuccess) return e;
    const dim3 grid((unsigned)r.n_blocks), block12(THREADS12);
#define SLIDE_WIDE_LAUNCH(RPGV)                                                                                     \
    do {                                                                                                            \
        hipLaunchKernelGGL((fwd16_ring_kernel<RPGV, false, false, 32, 1>), grid, block12, (size_t)r.lds_bytes, st, a); \
        if (lse) hipLaunchKernelGGL((fwd16_ring_kernel<RPGV, true, false, 32, 2>), grid, block12, (size_t)r.lds_bytes, st, a);  \
        else     hipLaunchKernelGGL((fwd16_ring_kernel<RPGV, false, false, 32, 2>), grid, block12, (size_t)r.lds_bytes, st, a); \
    } while (0)
    if (r.rpg == 2) SLIDE_WIDE_LAUNCH(2);
    else if (r.rpg == 3) SLIDE_WIDE_LAUNCH(3);
    else SLIDE_WIDE_LAUNCH(4);
#undef SLIDE_WIDE_LAUNCH
    return hipGetLastError();
}

bool fwd_ring_nhwc_supported(const Problem& p, bool aligned16)
{
    if (!aligned16 || p.dtype != 1 || p.ksize != 3 || p.C != p.heads * f16ring::D) return false;
    if ((long)p.H * p.W * p.C * 2 >= (1L << 31)) return false;        // 32-bit byte offsets inside a batch item
    return f16ring::plan_ring(p, f16ring::WAVES, 1, true).ok;
}

hipError_t launch_fwd_ring_nhwc(const Problem& p, const void* q, const void* k, const void* v,
                                const float* wk, const float* wv, const float* bias, void* out,
                                float* lse, hipStream_t st)
{
    using namespace f16ring;
    const RingPlan r = plan_ring(p, WAVES, 1, true);
    if (!r.ok) return hipErrorInvalidValue;
    RingArgs a{};
    a.q = (const bf16_bits*)q; a.k = (const bf16_bits*)k; a.v = (const bf16_bits*)v;
    a.out = (bf16_bits*)out; a.lse = lse;
    a.wk = wk; a.wv = wv; a.bias = bias;
    a.B = p.B; a.H = p.H; a.W = p.W; a.C = p.C; a.heads = p.heads; a.d = D;
    a.nbp = r.nbp; a.rows_pb = r.rows_pb; a.n_blocks = r.n_blocks;
    a.R = r.R; a.RS = r.RS; a.PS = r.PS; a.off_q = r.off_q;
    a.magic_w = (uint32_t)(((1ULL << 32) + p.W - 1) / p.W);
    a.magic_r = (uint32_t)(((1ULL << 32) + r.R - 1) / r.R);
    a.scale_log2e = 1.44269504088896341f / sqrtf((float)D);
    a.idw = p.two_branch ? 1.0f : 0.0f;
    static LdsOptIn opt_in;
#define SLIDE_NHWC_KERNELS(RPGV)                                                                                     \
    (const void*)fwd16_ring_nhwc_kernel<RPGV, false, 8, 4>, (const void*)fwd16_ring_nhwc_kernel<RPGV, true, 8, 4>
    hipError_t e = opt_in.ensure({SLIDE_NHWC_KERNELS(2), SLIDE_NHWC_KERNELS(3), SLIDE_NHWC_KERNELS(4)}, LDS_LIMIT);
#undef SLIDE_NHWC_KERNELS
    if (e != hipSuccess) return e;
    const dim3 grid((unsigned)r.n_blocks);
#define SLIDE_NHWC_LAUNCH(RPGV, NWV, NMV)                                                                            \
    do {                                                                                                             \
        if (lse) hipLaunchKernelGGL((fwd16_ring_nhwc_kernel<RPGV, true, NWV, NMV>), grid, dim3((NWV + NMV) * 64), (size_t)r.lds_bytes, st, a);  \
        else     hipLaunchKernelGGL((fwd16_ring_nhwc_kernel<RPGV, false, NWV, NMV>), grid, dim3((NWV + NMV) * 64), (size_t)r.lds_bytes, st, a); \
    } while (0)
    if (r.rpg == 2) SLIDE_NHWC_LAUNCH(2, 8, 4);
    else if (r.rpg == 3) SLIDE_NHWC_LAUNCH(3, 8, 4);
    else SLIDE_NHWC_LAUNCH(4, 8, 4);
#undef SLIDE_NHWC_LAUNCH
    return hipGetLastError();
}

hipError_t launch_fwd_traffic_probe(const Problem& p, const void* q, const void* k, const void* v, void* out,
                                    int mode, hipStream_t st)
{
    using namespace f16ring;
    if (mode == 0) {
        const long n16 = (long)p.B * p.C * p.H * p.W * 2 / 16;
        hipLaunchKernelGGL(probe_flat_kernel, dim3((unsigned)(8 * device_cu_count())), dim3(512), 0, st,
                           (const probe_u4*)q, (const probe_u4*)k, (const probe_u4*)v, (probe_u4*)out, n16);
        return hipGetLastError();
    }
    const RingPlan r = plan_ring(p);
    if (!r.ok) return hipErrorInvalidValue;
    RingArgs a{};
    a.q = (const bf16_bits*)q; a.k = (const bf16_bits*)k; a.v = (const bf16_bits*)v; a.out = (bf16_bits*)out;
    a.B = p.B; a.H = p.H; a.W = p.W; a.C = p.C; a.heads = p.heads;
    a.nbp = r.nbp; a.rows_pb = r.rows_pb; a.n_blocks = r.n_blocks;
    a.magic_w = (uint32_t)(((1ULL << 32) + p.W - 1) / p.W);
    hipLaunchKernelGGL(probe_stream_kernel, dim3((unsigned)r.n_blocks), dim3(THREADS), 0, st, a);
    return hipGetLastError();
}

}  // namespace slide
