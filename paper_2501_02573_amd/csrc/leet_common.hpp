// Shared device/host definitions for the gfx950 kernels of the decayed causal
// linear attention library.  gfx950 only: wave64, MFMA, 160 KiB LDS per CU.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace leet {

constexpr int kChunk = 64;  // tokens per chunk (the block size B_c of Alg. 2; B_c = O(d))

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Arguments of the chunk-walk kernels (prefill).  One workgroup walks the chunks
// of one segment of one (batch, head) sequence.
struct FwdParams {
    const void* q;          // [BH][N][D]
    const void* k;
    const void* v;
    const float* gamma;     // [H]
    float* out;             // [BH][N][D]
    const float* state_in;  // [BH][D][D] or null: state before token 0
    float* state_out;       // [BH][D][D] or null: state after token N-1
    float* seg_state;       // [BH][nseg-1][D][D]: slot s-1 holds the state entering segment s
    int H;
    int N;
    int nseg;        // segments per sequence
    int seg_chunks;  // chunks per segment (all but the last segment)
};

// gamma^n for integer n >= 0 in fp64 by binary exponentiation; 0^0 = 1.
__device__ __forceinline__ double pow_int(double g, int n) {
    double r = 1.0;
    while (n > 0) {
        if (n & 1) r *= g;
        g *= g;
        n >>= 1;
    }
    return r;
}

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t bits16) {
    return __uint_as_float(bits16 << 16);
}

// Round-to-nearest-even fp32 -> bf16 bit pattern (finite inputs).
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float x) {
    uint32_t u = __float_as_uint(x);
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    return f32_to_bf16_bits(lo) | (f32_to_bf16_bits(hi) << 16);
}

}  // namespace leet
