// Shared pieces of the half-precision matrix-core kernels (forward and backward) for
// gfx950: bf16 activations, head size 32, 3x3 window.
//
//  - lane mapping: a wavefront handles 16 pixels at a time; lane = pixel p (0..15) +
//    16 * channel group g (0..3), group g owning channels 8g..8g+7 of the head;
//  - tiles: a (batch, head) plane is cut into tiles of th x tw pixels; two activation
//    tensors are staged per tile as halo tiles in LDS, [row][col][32 channels] in half
//    precision, 64 B per pixel with the four 16-byte channel-group slots XOR-swizzled by
//    the column;
//  - the ordered tile list (full-height tiles first) that blocks work through.
#pragma once
#include "slide_internal.h"
#include "slide_device.h"

namespace slide {
namespace t16 {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef __attribute__((ext_vector_type(4))) float float4_t;
typedef __attribute__((ext_vector_type(4))) uint32_t uint4_t;
typedef __attribute__((ext_vector_type(2))) uint32_t uint2_t;

constexpr int KS = 3, S = 9, D = 32;
constexpr float LN2 = 0.693147180559945309f;


// MFMA row 4g+r of the logit tile <-> shift index.  Rows are spread so that each lane
// group holds at most three live shifts: rows r=0,1 of every group and row 2 of group 0.
__host__ __device__ constexpr int shift_of_row(int row)
{
    const int g = row >> 2, r = row & 3;
    const int s = 4 * r + g;
    return (r < 2 || (r == 2 && g == 0)) ? s : -1;
}

__device__ __forceinline__ uint32_t pack_half(float lo, float hi)
{
    half2_t v = {(_Float16)lo, (_Float16)hi};
    return __builtin_bit_cast(uint32_t, v);
}
// Reinterpret a dword as two halves.  Taking the dword by value matters: a bit cast applied
// directly to an element of a vector variable picks element 0 with this compiler.
__device__ __forceinline__ half2_t as_half2(uint32_t x) { return __builtin_bit_cast(half2_t, x); }
__device__ __forceinline__ uint32_t as_dword(half2_t x) { return __builtin_bit_cast(uint32_t, x); }
// round toward zero: saturates instead of overflowing to infinity
__device__ __forceinline__ uint32_t pack_half_rtz(float lo, float hi)
{
    return __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(lo, hi));
}

// ------------------------------------------------------------------ cross-group reductions
// maximum / sum of x over the four lane groups (lanes l, l+16, l+32, l+48); every lane gets it
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

// byte offset of (halo column hc, channel group g) inside a halo row: 64 B per pixel,
// the four 16-byte channel-group slots XOR-swizzled by the column so that 8 consecutive
// pixels of one group fall on 8 different bank quads.
__device__ __forceinline__ int col_offset(int hc, int g)
{
    return hc * 64 + ((g ^ ((hc >> 1) & 3)) << 4);
}

// Uniform description of the tiling of a problem (part of the kernel arguments).
struct TileGrid {
    int B, H, W, C, heads;
    int th, tw, n_tc;        // full tile height, tile width, column tiles per plane
    int nA;                  // full-height row tiles per plane column (class A)
    int nB, hb;              // remainder rows: nB tiles of height hb (class B)
    int TA, TB;              // tiles in each class; the list holds class A first
    int v_off;               // byte offset of the second halo tensor inside a tile buffer
    int vec_ok;              // rows are 16-byte aligned: W % 8 == 0 and 16-byte aligned bases
    int r;                   // halo radius (ksize / 2)
    int small_first;         // the tile list starts with the remainder tiles (class B)
};

// One tile of one (batch, head) plane; every field is wavefront-uniform.
struct Tile {
    int i0, j0, rows, cols, m;
    int gxa, NX, n_items;    // first chunk column, chunks per halo row, staging items
    long head_base;          // element offset of channel 0 of the head
};

// List index -> tile.  Class A (full-height tiles) comes first so that dealing the list
// round-robin to the blocks balances them (a persistent kernel may ask for class B first: its
// blocks then start on a small tile, which shortens the part of the run where nothing
// overlaps the first staging); inside a class tiles are ordered head, batch, row tile, column tile,
// and consecutive queue indices are dealt to the 8 XCDs (blocks are dealt round-robin over
// XCDs too), so tiles adjacent in a plane are staged through the same L2 at about the same
// time and a block rarely changes head.
__device__ __forceinline__ Tile decode_tile(const TileGrid& a, int i)
{
    int k, n_r, hgt, row_base, cnt;
    const bool cls_a = a.small_first ? i >= a.TB : i < a.TA;
    if (cls_a) { k = a.small_first ? i - a.TB : i; n_r = a.nA; hgt = a.th; row_base = 0; cnt = a.TA; }
    else       { k = a.small_first ? i : i - a.TA; n_r = a.nB; hgt = a.hb; row_base = a.nA * a.th; cnt = a.TB; }
    // (the last cnt % 8 tiles of a class keep their place)
    const int per_xcd = cnt >> 3;
    if (k < 8 * per_xcd) k = (k & 7) * per_xcd + (k >> 3);
    const int per_plane = a.n_tc * n_r;
    const int plane = k / per_plane;
    const int rem = k - plane * per_plane;
    const int tr = rem / a.n_tc, tcx = rem - tr * a.n_tc;
    Tile t;
    t.m = plane / a.B;
    const int b = plane - t.m * a.B;
    t.i0 = row_base + tr * hgt;
    t.rows = min(hgt, a.H - t.i0);
    t.j0 = tcx * a.tw;
    t.cols = min(a.tw, a.W - t.j0);
    t.head_base = ((long)b * a.C + (long)t.m * D) * ((long)a.H * a.W);
    t.gxa = max(t.j0 - a.r, 0) & ~7;
    const int gxb = min((t.j0 + t.cols + a.r + 7) & ~7, (a.W + 7) & ~7);
    t.NX = (gxb - t.gxa) >> 3;
    t.n_items = 8 * t.NX * (t.rows + 2 * a.r);
    return t;
}

// Staging item idx of a tile = 8 channels (group o) x 8 columns (chunk x) of one halo row of
// the first or second tensor.  item_load fetches it from global memory (zeros outside the map); item_store
// transposes it to 8 pixels x 8 channels, converts to half and writes it to the tile buffer.
__device__ __forceinline__ void item_load(const TileGrid& a, const Tile& t, const bf16_bits* src_a,
                                          const bf16_bits* src_b, int idx, uint4_t (&r)[8])
{
    const int o = idx & 3, tsel = (idx >> 2) & 1;
    const int rest = idx >> 3;
    const int hr = rest / t.NX, x = rest - hr * t.NX;
    const int gi = t.i0 - a.r + hr, gx = t.gxa + 8 * x;
    const long HW = (long)a.H * a.W;
    if (gi < 0 || gi >= a.H) {
#pragma unroll
        for (int e = 0; e < 8; ++e) r[e] = uint4_t{0u, 0u, 0u, 0u};
        return;
    }
    const bf16_bits* plane0 = (tsel ? src_b : src_a) + t.head_base + (long)(8 * o) * HW;
    if (a.vec_ok && gx + 8 <= a.W) {
        const bf16_bits* src = plane0 + (long)gi * a.W + gx;
#pragma unroll
        for (int e = 0; e < 8; ++e) r[e] = *(const uint4_t*)(src + e * HW);
    } else {
        // ragged chunk: element loads from clamped (always valid) columns, then masked
        const bf16_bits* src = plane0 + (long)gi * a.W;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
#pragma unroll
            for (int y = 0; y < 4; ++y) {
                const int c0 = gx + 2 * y, c1 = c0 + 1;
                const int cc0 = min(c0, a.W - 1), cc1 = min(c1, a.W - 1);
                uint32_t lo = src[e * HW + cc0], hi = src[e * HW + cc1];
                lo = (c0 == cc0) ? lo : 0u;
                hi = (c1 == cc1) ? hi : 0u;
                r[e][y] = lo | (hi << 16);
            }
        }
    }
}

__device__ __forceinline__ void item_store(const TileGrid& a, const Tile& t, int idx,
                                           const uint4_t (&r)[8], unsigned char* buf)
{
    const int o = idx & 3, tsel = (idx >> 2) & 1;
    const int rest = idx >> 3;
    const int hr = rest / t.NX, x = rest - hr * t.NX;
    const int gx = t.gxa + 8 * x;
    const int HC = a.tw + 2 * a.r;
    unsigned char* dst = buf + (tsel ? a.v_off : 0) + hr * HC * 64;
    // Even columns sit in the low half of a dword, odd columns in the high half; either way the
    // float is the bf16 pattern in the upper 16 bits.  The conversion to half is exact for
    // every bf16 value whose last bit weighs at least 2^-24 (round toward zero below that).
#pragma unroll
    for (int px = 0; px < 8; ++px) {
        uint4_t t4;
#pragma unroll
        for (int y = 0; y < 4; ++y) {
            const uint32_t lo = r[2 * y][px >> 1], hi = r[2 * y + 1][px >> 1];
            if (px & 1)
                t4[y] = pack_half_rtz(__uint_as_float(lo & 0xffff0000u), __uint_as_float(hi & 0xffff0000u));
            else
                t4[y] = pack_half_rtz(__uint_as_float(lo << 16), __uint_as_float(hi << 16));
        }
        const int hc = gx + px - (t.j0 - a.r);
        if (hc >= 0 && hc < t.cols + 2 * a.r) *(uint4_t*)(dst + col_offset(hc, o)) = t4;
    }
}

// halo columns that lie outside the map (left of column 0, right of column W-1) are zero
__device__ __forceinline__ void zero_pad_columns(const TileGrid& a, const Tile& t, unsigned char* buf,
                                                 int tid, int threads)
{
    const bool left = (t.j0 == 0), right = (t.j0 + t.cols == a.W);
    if (!left && !right) return;
    const int HC = a.tw + 2 * a.r;
    const int n = (t.rows + 2 * a.r) * a.r * 16;        // row x radius x side x tensor x channel group
    for (int idx = tid; idx < n; idx += threads) {
        const int o = idx & 3, tsel = (idx >> 2) & 1, side = (idx >> 3) & 1;
        const int rest = idx >> 4;
        const int k = rest % a.r, hr = rest / a.r;
        if (side ? !right : !left) continue;
        const int hc = side ? t.cols + a.r + k : k;
        *(uint4_t*)(buf + (tsel ? a.v_off : 0) + hr * HC * 64 + col_offset(hc, o)) = uint4_t{0u, 0u, 0u, 0u};
    }
}

// ------------------------------------------------------------------ host side
constexpr int LDS_LIMIT = 160 * 1024;

struct TilePlan {
    int th, tw, n_tc, nA, nB, hb, TA, TB;
    int v_off, buf_bytes;    // the two halo tensors of a tile occupy buf_bytes of LDS
    int halo_px;             // halo pixels of a full tile: (th + 2r) * (tw + 2r)
};

// makespan of dealing big-first: TA tiles of cost cA first, then TB tiles of cost cB, G blocks
inline double queue_makespan(long TA, double cA, long TB, double cB, int G)
{
    const long qa = TA / G, ra = TA % G;
    const double lo = qa * cA, hi = (ra ? qa + 1 : qa) * cA;
    if (TB == 0) return hi;
    // smallest M with sum_b floor((M - L_b) / cB) >= TB, tried on the grid lo + j*cB, hi + j*cB
    double best = 1e300;
    for (long j = 0; j <= TB / G + 2; ++j) {
        for (int w = 0; w < 2; ++w) {
            const double M = (w ? hi : lo) + j * cB;
            if (M < hi) continue;
            const long cap = (G - ra) * (long)((M - lo) / cB + 1e-9) + ra * (long)((M - hi) / cB + 1e-9);
            if (cap >= TB && M < best) best = M;
        }
    }
    return best;
}

// Tile heights for a kernel that may spend lds_budget bytes on one tile buffer holding two
// halo tensors of px_bytes per halo pixel each (64 for a staged activation tensor).
// px_bytes_extra: further LDS bytes per halo pixel that the kernel places after the buffer.
// pass_waves > 0: the kernel deals the 16-pixel passes of a tile to that many waves and does
// not overlap the staging of a tile with its passes; a tile then costs the rounds of passes
// its busiest wave runs plus a staging share, instead of its rows.
inline TilePlan plan_tiles(const Problem& p, int lds_budget, int px_bytes_a, int px_bytes_b,
                           int px_bytes_extra = 0, int pass_waves = 0)
{
    const int r2 = 2 * (p.ksize / 2);
    const int n_cu = device_cu_count();
    TilePlan t;
    t.tw = p.W <= 64 ? p.W : 64;
    t.n_tc = (p.W + t.tw - 1) / t.tw;
    const int px_bytes = px_bytes_a + px_bytes_b + px_bytes_extra;
    int th_max = (lds_budget - 256) / (px_bytes * (t.tw + r2)) - r2;
    if (th_max < 1) th_max = 1;
    if (th_max > p.H) th_max = p.H;
    const long planes = (long)p.B * p.heads * t.n_tc;
    // choose the tile heights that minimise the makespan of dealing the tiles to one block
    // per compute unit slot (cost of a tile: its rows plus a fixed share for the halo rows
    // and the per-tile overhead)
    double best = 1e300;
    t.th = th_max; t.nA = p.H / th_max; t.nB = (p.H % th_max) ? 1 : 0; t.hb = p.H % th_max;
    for (int th = th_max; th >= 1 && th >= th_max / 2; --th) {
        for (int drop = 0; drop < 2; ++drop) {
            const int nA = p.H / th - drop;
            if (nA < 0) continue;
            const int rem = p.H - nA * th;
            for (int nB = (rem + th - 1) / th; nB <= (rem + th - 1) / th + 2; ++nB) {
                if ((rem == 0) != (nB == 0)) continue;
                const int hb = nB ? (rem + nB - 1) / nB : 0;
                if (nB && (hb < 1 || (long)hb * (nB - 1) >= rem)) continue;
                auto cost = [&](int rows) {
                    if (pass_waves <= 0) return rows + 1.5;
                    const int passes = (rows * t.tw + 15) / 16;
                    return (double)((passes + pass_waves - 1) / pass_waves) + 0.35 + 0.035 * (rows + r2);
                };
                const double ms = queue_makespan(planes * nA, cost(th), planes * nB, cost(hb), n_cu);
                if (ms < best - 1e-9) { best = ms; t.th = th; t.nA = nA; t.nB = nB; t.hb = hb; }
            }
        }
    }
    t.TA = (int)(planes * t.nA);
    t.TB = (int)(planes * t.nB);
    const int halo_px = (t.th + r2) * (t.tw + r2);
    t.halo_px = halo_px;
    t.v_off = halo_px * px_bytes_a;
    if ((t.v_off & 127) == 0) t.v_off += 64;             // the two tensors start 64 B apart mod 128
    t.buf_bytes = (t.v_off + halo_px * px_bytes_b + 127) & ~127;
    return t;
}

inline void fill_grid(TileGrid& g, const Problem& p, const TilePlan& t, const void* src_a, const void* src_b)
{
    g.B = p.B; g.H = p.H; g.W = p.W; g.C = p.C; g.heads = p.heads;
    g.th = t.th; g.tw = t.tw; g.n_tc = t.n_tc; g.nA = t.nA; g.nB = t.nB; g.hb = t.hb;
    g.TA = t.TA; g.TB = t.TB; g.v_off = t.v_off; g.r = p.ksize / 2;
    g.small_first = 0;
    g.vec_ok = (p.W % 8 == 0) && (((uintptr_t)src_a | (uintptr_t)src_b) % 16 == 0);
}

}  // namespace t16
}  // namespace slide
