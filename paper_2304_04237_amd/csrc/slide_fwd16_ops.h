// Pieces shared by the 3x3 matrix-core forward kernels (bf16, head size 32): the per-head
// image of MFMA weight operands (layout, how it is built from the float32 kernels, how a
// wavefront loads it into registers).
//
// Arithmetic the image serves (the operator of Sec. 4.1-4.3, re-associated), with the merged
// kernel W~ = one-hot shift + learned part (Sec. 4.3, Fig. 4):
//     logit[s] = scale * sum_{c,t} (q[c] k[c, p+t]) W~k[c,s,t]       <- 288 x 9 contraction
//     out[c]   = sum_t v[c, p+t] * g[c,t],  g[c,t] = sum_s a[s] W~v[c,s,t]   <- 9 x 288
#pragma once
#include "slide_tile16.h"

namespace slide {
namespace f16ops {
using namespace t16;

constexpr float G_SCALE = 0.0625f;                 // q is divided by 16 for the MFMA products ...
constexpr float WK_SCALE = 16.0f;                  // ... and the learned K kernel multiplied by 16

// Per-head image of the MFMA weight operands, written by prep_weights_kernel (dwords):
//   [0, 2304)      A1: tap t (9) x lane (64) x 4 dwords       -- learned K kernel (times 16)
//   [2304, 4608)   A2: product u (18) x lane (64) x 2 dwords  -- learned V kernel
//   [4608, 4624)   bias row r (16) as float, times log2(e); -inf on unused rows
constexpr int IMG_A1 = 0, IMG_A2 = 2304, IMG_BIAS = 4608, IMG_DWORDS = 4624;

// ------------------------------------------------------------------ weight preparation
// Dword idx < IMG_BIAS of a head's operand image is pack_half(f(w[off0]), f(w[off1])) with
// f(x) = ok ? (x - sub) * scale : 0 and w the K (A1 part) or V (A2 part) kernel [C, 9, 3, 3]
// of float32.  sub is 0 for merged kernels; for the learned kernels of the two-branch form
// it is -1 where shift and tap coincide (idw = 1: the fixed shift path joins the operand).
// The loads are unconditional so that a caller can issue many of them before using any.
struct ImageSource {
    int off0, off1;          // element offsets into the kernel tensor
    float sub0, sub1, scale;
    bool ok0, ok1, from_v;
};
__device__ __forceinline__ ImageSource image_source(int m, int idx, float idw)
{
    ImageSource r;
    if (idx < IMG_A2) {
        // A1, tap t: dword y of lane (i, g) = learned K weights of channels 8g+2y, 8g+2y+1
        // for the shift of logit row i.
        const int t = idx >> 8, y = idx & 3, lane = (idx >> 2) & 63;
        const int i = lane & 15, g = lane >> 4;
        const int s = shift_of_row(i);
        const int c = m * D + 8 * g + 2 * y;
        r.off0 = (c * S + max(s, 0)) * S + t;
        r.off1 = r.off0 + S * S;
        r.sub0 = r.sub1 = (s == t) ? -idw : 0.0f;
        r.ok0 = r.ok1 = s >= 0;
        r.scale = WK_SCALE;
        r.from_v = false;
    } else {
        // A2, product u.  u < 16: channel slot e = u & 7, tap quad tq = u >> 3; row i of the
        // product is channel 8*(i/4) + e at tap 4*tq + (i%4).  Products 16, 17 (j = u - 16):
        // row i is channel 8*(i/4) + 4j + (i%4) at tap 8.  Dword y of lane (i, g) holds the
        // learned V weights for the shifts of logit rows 4g+2y and 4g+2y+1.
        const int q = idx - IMG_A2;
        const int u = q >> 7, y = q & 1, lane = (q >> 1) & 63;
        const int i = lane & 15, g = lane >> 4;
        const int c = m * D + 8 * (i >> 2) + (u < 16 ? (u & 7) : 4 * (u - 16) + (i & 3));
        const int tap = u < 16 ? 4 * (u >> 3) + (i & 3) : 8;
        const int s0 = shift_of_row(4 * g + 2 * y), s1 = shift_of_row(4 * g + 2 * y + 1);
        r.off0 = (c * S + max(s0, 0)) * S + tap;
        r.off1 = (c * S + max(s1, 0)) * S + tap;
        r.sub0 = (s0 == tap) ? -idw : 0.0f;
        r.sub1 = (s1 == tap) ? -idw : 0.0f;
        r.ok0 = s0 >= 0;
        r.ok1 = s1 >= 0;
        r.scale = 1.0f;
        r.from_v = true;
    }
    return r;
}
__device__ __forceinline__ uint32_t image_value(const ImageSource& r, float w0, float w1)
{
    return pack_half(r.ok0 ? (w0 - r.sub0) * r.scale : 0.0f, r.ok1 ? (w1 - r.sub1) * r.scale : 0.0f);
}
// dwords IMG_BIAS .. IMG_DWORDS-1: bias of logit row r times log2(e); -inf on unused rows
__device__ __forceinline__ uint32_t image_bias(const float* __restrict__ bias, int m, int row)
{
    const int s = shift_of_row(row);
    float b = -INFINITY;
    if (s >= 0) b = bias ? bias[m * S + s] * 1.44269504088896341f : 0.0f;
    return __float_as_uint(b);
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

// One block builds a head's operand image in LDS (THREADS threads, every weight load issued
// before the first use).
// The head's kernels (2 x 32 x 81 floats, contiguous) come in as coalesced 16-byte loads and
// are gathered from LDS: `raw` is IMG_RAW_BYTES of LDS that does not overlap dst.  Contains a
// block barrier; every thread of the block must call it.
constexpr int IMG_RAW_AT = 20480;                         // byte offset of `raw` behind an image (IMG_DWORDS * 4 = 18496)
constexpr int HEAD_W = D * S * S;                         // floats of one head in a kernel tensor
constexpr int IMG_RAW_BYTES = 2 * HEAD_W * 4;             // 20736
// the gather: raw (the head's K kernels, then its V kernels, as float32 in LDS) -> operand image.
// 512 threads; the same dwords as image_source() / image_value() describe, with a thread's
// part of the index arithmetic taken out of its loop: thread (lane, y, th) writes dwords y of
// that lane for every second tap (A1 part) and for every fourth product (A2 part).
template <int THREADS>
__device__ __forceinline__ void image_from_raw(const float* raw, const float* __restrict__ bias, int m, float idw,
                                               uint32_t* dst, int tid)
{
    static_assert(THREADS == 512, "thread-to-dword mapping below");
    const int lane = tid & 63, i = lane & 15, g = lane >> 4;
    {
        // A1: dword (t * 64 + lane) * 4 + y = K weights of channels 8g + 2y, 8g + 2y + 1 for the shift of logit row i at tap t
        const int y = (tid >> 6) & 3, th = tid >> 8;
        const int s = shift_of_row(i);
        const bool ok = s >= 0;
        const float* w = raw + ((8 * g + 2 * y) * S + max(s, 0)) * S;
#pragma unroll
        for (int k = 0; k < 5; ++k) {
            const int t = th + 2 * k;
            if (t < S) {
                const float sub = (s == t) ? -idw : 0.0f;
                const float w0 = w[t], w1 = w[t + S * S];
                dst[IMG_A1 + (t * 64 + lane) * 4 + y] = ok ? pack_half((w0 - sub) * WK_SCALE, (w1 - sub) * WK_SCALE) : 0u;
            }
        }
    }
    {
        // A2: dword (u * 64 + lane) * 2 + y = V weights of the product's row i (a channel and a tap) for the shifts of logit rows 4g + 2y, 4g + 2y + 1
        const int y = (tid >> 6) & 1, uh = tid >> 7;
        const int s0 = shift_of_row(4 * g + 2 * y), s1 = shift_of_row(4 * g + 2 * y + 1);
        const float* wv = raw + HEAD_W;
#pragma unroll
        for (int k = 0; k < 5; ++k) {
            const int u = uh + 4 * k;
            if (k < 4 || uh < 2) {
                const int c = 8 * (i >> 2) + (k < 4 ? uh + 4 * (k & 1) : 4 * uh + (i & 3));
                const int tap = k < 4 ? 4 * (k >> 1) + (i & 3) : 8;
                const float w0 = wv[(c * S + max(s0, 0)) * S + tap], w1 = wv[(c * S + max(s1, 0)) * S + tap];
                const float sub0 = (s0 == tap) ? -idw : 0.0f, sub1 = (s1 == tap) ? -idw : 0.0f;
                dst[IMG_A2 + (u * 64 + lane) * 2 + y] = pack_half(s0 >= 0 ? w0 - sub0 : 0.0f, s1 >= 0 ? w1 - sub1 : 0.0f);
            }
        }
    }
    if (tid < IMG_DWORDS - IMG_BIAS) dst[IMG_BIAS + tid] = image_bias(bias, m, tid);
}

template <int THREADS>
__device__ __forceinline__ void build_image(const float* __restrict__ wk, const float* __restrict__ wv,
                                            const float* __restrict__ bias, int m, float idw, uint32_t* dst,
                                            float* raw, int tid)
{
    constexpr int CHUNKS = HEAD_W / 4;
    static_assert(CHUNKS * 4 == HEAD_W, "16-byte chunks");
    for (int i = tid; i < 2 * CHUNKS; i += THREADS) {
        const bool is_v = i >= CHUNKS;
        const float* src = (is_v ? wv : wk) + (long)m * HEAD_W;               // 16-byte aligned: HEAD_W % 4 == 0
        *(float4_t*)(raw + 4 * i) = *(const float4_t*)(src + 4 * (i - (is_v ? CHUNKS : 0)));
    }
    __syncthreads();
    image_from_raw<THREADS>(raw, bias, m, idw, dst, tid);
}

// ------------------------------------------------------------------ data movement of the streaming kernels
typedef short short4_t __attribute__((ext_vector_type(4)));

// 16 bytes per active lane from global memory (uniform base + per-lane byte offset) straight
// into LDS: lane l's bytes land at lds_base + 16 l.  Counts as one vector-memory operation.
__device__ __forceinline__ void load_to_lds(const void* base, uint32_t voff, uint32_t lds_base)
{
    asm volatile("s_mov_b32 m0, %2\n\t"
                 "s_nop 0\n\t"
                 "global_load_lds_dwordx4 %1, %0"
                 :: "s"(base), "v"(voff), "s"(lds_base) : "memory");
}

// the same with a full 64-bit address per lane
__device__ __forceinline__ void load_to_lds_addr(const void* vaddr, uint32_t lds_base)
{
    asm volatile("s_mov_b32 m0, %1\n\t"
                 "s_nop 0\n\t"
                 "global_load_lds_dwordx4 %0, off"
                 :: "v"(vaddr), "s"(lds_base) : "memory");
}

// wait until at most n vector-memory operations of this wave are in flight (n uniform;
// above 12 the wait is for 12, which is stricter)
__device__ __forceinline__ void wait_vmem(int n)
{
    switch (n) {
        case 0: asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); break;
        case 1: asm volatile("s_waitcnt vmcnt(1)" ::: "memory"); break;
        case 2: asm volatile("s_waitcnt vmcnt(2)" ::: "memory"); break;
        case 3: asm volatile("s_waitcnt vmcnt(3)" ::: "memory"); break;
        case 4: asm volatile("s_waitcnt vmcnt(4)" ::: "memory"); break;
        case 5: asm volatile("s_waitcnt vmcnt(5)" ::: "memory"); break;
        case 6: asm volatile("s_waitcnt vmcnt(6)" ::: "memory"); break;
        case 7: asm volatile("s_waitcnt vmcnt(7)" ::: "memory"); break;
        case 8: asm volatile("s_waitcnt vmcnt(8)" ::: "memory"); break;
        case 9: asm volatile("s_waitcnt vmcnt(9)" ::: "memory"); break;
        case 10: asm volatile("s_waitcnt vmcnt(10)" ::: "memory"); break;
        case 11: asm volatile("s_waitcnt vmcnt(11)" ::: "memory"); break;
        default: asm volatile("s_waitcnt vmcnt(12)" ::: "memory"); break;
    }
}

// all LDS operations of this wave are done, then the block barrier; memory operations are not
// moved across it by the compiler
__device__ __forceinline__ void block_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// Transposing LDS read: within each group of 16 lanes, lane n receives element (n % 4) of the
// 8-byte pieces addressed by lanes n / 4, n / 4 + 4, n / 4 + 8, n / 4 + 12.  With lane s
// addressing four consecutive pixels 4 (s % 4) .. + 3 of row s / 4 of a [row][pixel] array,
// lane n gets pixel n of rows 0..3 (and vice versa with rows and pixels exchanged).
__device__ __forceinline__ uint2_t lds_read_tr(const unsigned char* p)
{
    const short4_t r = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) short4_t*)p);
    return __builtin_bit_cast(uint2_t, r);
}

// two bf16 in a dword -> two halves in a dword (exact for 2^-17 <= |x| <= 65504, round toward
// zero below, saturating above)
__device__ __forceinline__ uint32_t bf16x2_to_half2(uint32_t d)
{
    return pack_half_rtz(__uint_as_float(d << 16), __uint_as_float(d & 0xffff0000u));
}

}  // namespace f16ops
}  // namespace slide
