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
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Arguments of the chunk-walk kernels (prefill).  One workgroup walks the chunks
// of one segment of one (batch, head) sequence.
struct FwdParams {
    const void* q;          // [BH][N][D]
    const void* k;
    const void* v;
    const float* gamma;     // [H]; not read when no_decay
    void* out;              // [BH][N][D], fp32 or the 16-bit input type
    const float* state_in;  // [BH][D][D] or null: state before token 0
    float* state_out;       // [BH][D][D] or null: state after token N-1
    float* seg_state;       // [BH][state_slots][D][DV]: slot s*state_step-1 holds the state entering segment s
    int H;
    int N;
    int nseg;        // segments per sequence
    int seg_chunks;  // chunks per segment (all but the last segment)
    int state_slots; // boundary-state slots per sequence (nseg-1, or more when the pre-pass runs on finer segments)
    int state_step;  // slots per segment
    int no_decay;    // non-zero: 0/1 causal mask, i.e. gamma = 1 for every head
    int stream_loads;  // non-zero: q, k, v exceed the last-level cache; load them with the nontemporal hint
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

// The two 16-bit input types of the MFMA kernels.  Operands travel as raw 128-bit
// registers (eight elements); only the conversions and the MFMA opcode differ.
struct ElemBf16 {
    static __device__ __forceinline__ float lo(uint32_t word) { return __uint_as_float(word << 16); }
    static __device__ __forceinline__ float hi(uint32_t word) { return __uint_as_float(word & 0xffff0000u); }
    static __device__ __forceinline__ uint32_t pack2(float a, float b) {
        bf16x2 r = {(__bf16)a, (__bf16)b};
        return __builtin_bit_cast(uint32_t, r);
    }
    static __device__ __forceinline__ f32x16 mfma32(u32x4 a, u32x4 b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    }
};

struct ElemF16 {
    static __device__ __forceinline__ float lo(uint32_t word) {
        return (float)__builtin_bit_cast(_Float16, (uint16_t)(word & 0xffffu));
    }
    static __device__ __forceinline__ float hi(uint32_t word) {
        return (float)__builtin_bit_cast(_Float16, (uint16_t)(word >> 16));
    }
    static __device__ __forceinline__ uint32_t pack2(float a, float b) {
        f16x2 r = {(_Float16)a, (_Float16)b};
        return __builtin_bit_cast(uint32_t, r);
    }
    static __device__ __forceinline__ f32x16 mfma32(u32x4 a, u32x4 b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    }
};

}  // namespace leet
