// Device-side types shared by the HIP kernels of the segmented base+adapter layer.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace symb {

typedef __bf16 bf16;
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float floatx4;
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short shortx4;

enum : int32_t { KIND_NONE = 0, KIND_LORA = 1, KIND_IA3 = 2, KIND_IA3_IN = 3 };

// Per-segment descriptor as the kernels see it (device memory, one per segment).
struct SegDesc {
    int32_t kind;
    int32_t rank;      // LoRA rank r_i (0 otherwise)
    int32_t rpad;      // r_i rounded up to a multiple of 16 (MFMA K granularity)
    float scale;       // s_i
    const bf16* A;     // LoRA A [r][d_in] / IA3 l[d_out]
    const bf16* B;     // LoRA B [d_out][r]
    float* dA;         // fp32 grads (may be null)
    float* dB;
};

// A segment's noise (or noise-effect) rows: rows == 1 broadcasts, else one row per token of the segment.
struct NoiseDesc {
    const bf16* ptr;   // null: none for this segment
    int32_t rows;
    int32_t pad;
};

// Round-to-nearest-even fp32 -> bf16 (finite inputs; NaN stays NaN).
__device__ __forceinline__ unsigned short f32_to_bf16_bits(float f) {
    unsigned int u = __builtin_bit_cast(unsigned int, f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (unsigned short)((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (unsigned short)(u >> 16);
}
__device__ __forceinline__ float bf16_bits_to_f32(unsigned short b) {
    return __builtin_bit_cast(float, ((unsigned int)b) << 16);
}
// Two fp32 -> packed bf16 pair, round-to-nearest-even in hardware (v_cvt_pk_bf16_f32).
__device__ __forceinline__ unsigned int pack2_bf16(float lo, float hi) {
    typedef float f32x2_t __attribute__((ext_vector_type(2)));
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    const f32x2_t v = {lo, hi};
    return __builtin_bit_cast(unsigned int, __builtin_convertvector(v, bf16x2_t));
}

// Segment of row t among segments [lo, hi], off[lo] <= t < off[hi + 1]: the one with off[i] <= t < off[i+1]
// (empty segments never match).  Bisection: a row tile of decode steps holds dozens of one-row segments,
// and every probe is a memory access.
__device__ __forceinline__ int seg_of_row(const int32_t* __restrict__ off, int lo, int hi, int t) {
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (t >= off[mid]) lo = mid;       // the largest i with off[i] <= t
        else hi = mid - 1;
    }
    return lo;
}

}  // namespace symb
