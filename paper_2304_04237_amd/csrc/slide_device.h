// Small device helpers: element load/store with float32 conversion.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace slide {

typedef uint16_t bf16_bits;   // storage of one bfloat16 element

__device__ __forceinline__ float bf16_to_f32(bf16_bits x) {
    return __uint_as_float(((uint32_t)x) << 16);
}

// round to nearest even; the compiler emits the gfx950 hardware conversion for this cast
__device__ __forceinline__ bf16_bits f32_to_bf16(float x) {
    __bf16 h = (__bf16)x;
    return __builtin_bit_cast(bf16_bits, h);
}

template <typename T> struct Elem;
template <> struct Elem<float> {
    static __device__ __forceinline__ float load(const float* p) { return *p; }
    static __device__ __forceinline__ void store(float* p, float x) { *p = x; }
};
template <> struct Elem<bf16_bits> {
    static __device__ __forceinline__ float load(const bf16_bits* p) { return bf16_to_f32(*p); }
    static __device__ __forceinline__ void store(bf16_bits* p, float x) { *p = f32_to_bf16(x); }
};

}  // namespace slide
