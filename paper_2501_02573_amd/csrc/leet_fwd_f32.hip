// Chunk-walk kernel for fp32 inputs (gfx950, v_mfma_f32_32x32x2_f32: true fp32 products).
//
// Same algorithm and work split as the bf16 kernel: one workgroup per segment of a
// (batch, head) sequence walks 64-token chunks (Alg. 2, Appendix B.2, with the decaying
// mask of Eq. "BCMV" and the weight split of Alg. 4); wave w owns value columns
// [32w, 32w+32) of O and of the state S.
//
// The fp32 MFMA takes one contraction index per lane (lane l: row/column l%32,
// contraction index l/32), so no operand needs a transposed copy: Q, K, V sit
// row-major in LDS, and both the score accumulators (as P) and the state accumulators
// (as S) feed the next MFMA straight from registers, one register per instruction.
#include "leet_common.hpp"

namespace leet {

template <int D>
struct F32Smem {
    static constexpr int RS = D + 4;  // padded row stride (floats)
    float q[kChunk * RS];
    float k[kChunk * RS];
    float v[kChunk * RS];
    float pw[kChunk + 4];
};

template <int D, bool kOut>
__global__ __launch_bounds__(D * 2) void fwd_f32_kernel(FwdParams p) {
    constexpr int NT = D * 2;
    constexpr int DT = D / 32;
    constexpr int RS = F32Smem<D>::RS;
    constexpr int PR = D / 4;                  // 16-byte pieces per row
    constexpr int NLOAD = kChunk * PR / NT;    // pieces per thread per tensor (= 8)
    __shared__ __attribute__((aligned(16))) F32Smem<D> sm;

    const int tid = threadIdx.x;
    const int w = tid >> 6, l = tid & 63, ln = l & 31, g = l >> 5;
    const int nseg_launch = kOut ? p.nseg : p.nseg - 1;
    const int bh = blockIdx.x / nseg_launch;
    const int seg = blockIdx.x % nseg_launch;
    const int h = bh % p.H;

    const int tok_begin = seg * p.seg_chunks * kChunk;
    const int tok_end = (seg == p.nseg - 1) ? p.N : tok_begin + p.seg_chunks * kChunk;
    const int nchunks = (tok_end - tok_begin + kChunk - 1) / kChunk;

    const size_t seq_off = (size_t)bh * p.N * D;
    const float* qb = reinterpret_cast<const float*>(p.q) + seq_off;
    const float* kb = reinterpret_cast<const float*>(p.k) + seq_off;
    const float* vb = reinterpret_cast<const float*>(p.v) + seq_off;
    float* ob = p.out + seq_off;

    {
        const double gd = (double)p.gamma[h];
        for (int n = tid; n <= kChunk; n += NT) sm.pw[n] = (float)pow_int(gd, n);
    }

    f32x16 S[DT];
    const int c_own = 32 * w + ln;
    {
        const float* src = nullptr;
        if (kOut) {
            if (seg == 0) src = p.state_in ? p.state_in + (size_t)bh * D * D : nullptr;
            else src = p.seg_state + ((size_t)bh * (p.nseg - 1) + (seg - 1)) * D * D;
        }
#pragma unroll
        for (int t = 0; t < DT; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                int dk = 32 * t + 8 * (r >> 2) + 4 * g + (r & 3);
                S[t][r] = src ? src[dk * D + c_own] : 0.0f;
            }
    }

    for (int t = 0; t < nchunks; ++t) {
        const int tok0 = tok_begin + t * kChunk;
        const int Lc = min(kChunk, tok_end - tok0);

        __syncthreads();  // previous chunk fully consumed (and pw written, first time round)
#pragma unroll
        for (int r = 0; r < NLOAD; ++r) {
            int piece = r * NT + tid;
            int j = piece / PR, cc = piece % PR;
            bool ok = tok0 + j < tok_end;
            size_t off = (size_t)(tok0 + j) * D + cc * 4;
            f32x4 z = {0.f, 0.f, 0.f, 0.f};
            if (kOut) *reinterpret_cast<f32x4*>(&sm.q[j * RS + cc * 4]) = ok ? *reinterpret_cast<const f32x4*>(qb + off) : z;
            *reinterpret_cast<f32x4*>(&sm.k[j * RS + cc * 4]) = ok ? *reinterpret_cast<const f32x4*>(kb + off) : z;
            *reinterpret_cast<f32x4*>(&sm.v[j * RS + cc * 4]) = ok ? *reinterpret_cast<const f32x4*>(vb + off) : z;
        }
        __syncthreads();

        if (kOut) {
            f32x16 o[2];
#pragma unroll
            for (int it = 0; it < 2; ++it)
#pragma unroll
                for (int r = 0; r < 16; ++r) o[it][r] = 0.0f;

            // ---- inter-chunk term O = Q_t S_t (register r of S[dt] is contraction step r), rows * gamma^(i+1)
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                for (int rq = 0; rq < 4; ++rq)
#pragma unroll
                    for (int it = 0; it < 2; ++it) {
                        f32x4 a = *reinterpret_cast<const f32x4*>(&sm.q[(32 * it + ln) * RS + 32 * dt + 8 * rq + 4 * g]);
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            o[it] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[e], S[dt][4 * rq + e], o[it], 0, 0, 0);
                    }
#pragma unroll
            for (int it = 0; it < 2; ++it)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    int i = 32 * it + 8 * (r >> 2) + 4 * g + (r & 3);
                    o[it][r] *= sm.pw[i + 1];
                }

            // ---- intra-chunk term: P^T = K Q^T, decay mask, O += P V
#pragma unroll
            for (int it = 0; it < 2; ++it)
#pragma unroll
                for (int jt = 0; jt <= it; ++jt) {
                    f32x16 acc;
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
#pragma unroll
                    for (int u = 0; u < D / 8; ++u) {
                        f32x4 a = *reinterpret_cast<const f32x4*>(&sm.k[(32 * jt + ln) * RS + 8 * u + 4 * g]);
                        f32x4 b = *reinterpret_cast<const f32x4*>(&sm.q[(32 * it + ln) * RS + 8 * u + 4 * g]);
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[e], b[e], acc, 0, 0, 0);
                    }
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        int n = 32 * (it - jt) + ln - (8 * (r >> 2) + 4 * g + (r & 3));  // i - j
                        float wgt = sm.pw[max(n, 0)];
                        acc[r] = (n >= 0) ? acc[r] * wgt : 0.0f;
                    }
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        int j = 32 * jt + 8 * (r >> 2) + 4 * g + (r & 3);
                        o[it] = __builtin_amdgcn_mfma_f32_32x32x2f32(acc[r], sm.v[j * RS + c_own], o[it], 0, 0, 0);
                    }
                }

#pragma unroll
            for (int it = 0; it < 2; ++it)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    int i = 32 * it + 8 * (r >> 2) + 4 * g + (r & 3);
                    if (i < Lc) ob[(size_t)(tok0 + i) * D + c_own] = o[it][r];
                }
        }

        // ---- state update: S = gamma^L S + (Gam K)^T V ; contraction step u covers tokens 2u, 2u+1
        {
            const float gl = sm.pw[Lc];
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                for (int r = 0; r < 16; ++r) S[dt][r] *= gl;
#pragma unroll 8
            for (int u = 0; u < kChunk / 2; ++u) {
                const int j = 2 * u + g;
                const float sc = sm.pw[max(Lc - 1 - j, 0)];
                const float b = sm.v[j * RS + c_own];
#pragma unroll
                for (int dt = 0; dt < DT; ++dt) {
                    float a = sm.k[j * RS + 32 * dt + ln] * sc;
                    S[dt] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, S[dt], 0, 0, 0);
                }
            }
        }
    }

    float* dst = nullptr;
    if (kOut) {
        if (seg == p.nseg - 1 && p.state_out) dst = p.state_out + (size_t)bh * D * D;
    } else {
        dst = p.seg_state + ((size_t)bh * (p.nseg - 1) + seg) * D * D;
    }
    if (dst) {
#pragma unroll
        for (int t = 0; t < DT; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                int dk = 32 * t + 8 * (r >> 2) + 4 * g + (r & 3);
                dst[dk * D + c_own] = S[t][r];
            }
    }
}

hipError_t launch_fwd_f32_states(const FwdParams& p, int BH, int D, hipStream_t stream) {
    if (p.nseg <= 1) return hipSuccess;
    if (D == 64) hipLaunchKernelGGL((fwd_f32_kernel<64, false>), dim3(BH * (p.nseg - 1)), dim3(128), 0, stream, p);
    else hipLaunchKernelGGL((fwd_f32_kernel<128, false>), dim3(BH * (p.nseg - 1)), dim3(256), 0, stream, p);
    return hipGetLastError();
}

hipError_t launch_fwd_f32_walk(const FwdParams& p, int BH, int D, hipStream_t stream) {
    if (D == 64) hipLaunchKernelGGL((fwd_f32_kernel<64, true>), dim3(BH * p.nseg), dim3(128), 0, stream, p);
    else hipLaunchKernelGGL((fwd_f32_kernel<128, true>), dim3(BH * p.nseg), dim3(256), 0, stream, p);
    return hipGetLastError();
}

}  // namespace leet
