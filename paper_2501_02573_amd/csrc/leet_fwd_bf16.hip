// Chunk-walk kernel for bf16 inputs (gfx950, v_mfma_f32_32x32x16_bf16, fp32 accumulate).
//
// One workgroup walks the 64-token chunks of one segment of one (batch, head)
// sequence in order (the loop of Alg. 2, Appendix B.2), carrying the d x d state S
// in MFMA accumulators.  With the decaying mask (Section 2.2, Eq. "BCMV"), chunk t of
// length L computes, using the row/column weight split of Alg. 4 (Appendix B.3):
//
//     O_t     = ((Q_t K_t^T) .* D) V_t + Lam (Q_t S_t)       D[i][j] = gamma^(i-j), i >= j
//     S_{t+1} = gamma^L S_t + (Gam K_t)^T V_t                Lam = diag(gamma^(i+1)), Gam = diag(gamma^(L-1-j))
//
// Work split: wave w owns value columns [32w, 32w+32).  It keeps S[:, cols] (D x 32
// fp32) in accumulators for the whole walk and computes O_t[:, cols]; every wave
// recomputes the 64 x 64 score tile, which keeps the waves independent of one
// another between the two barriers that stage a chunk into LDS.
//
// Register-level chaining (no LDS round trip for P or S):
//  * scores are produced transposed, P^T = K Q^T, so that the accumulator layout of
//    P^T (lane = query row, registers = keys) is already the A-operand layout of P
//    for P V, up to a fixed permutation of the contraction index that the V operand
//    read applies as well;
//  * S accumulators (lane = value column, registers = key rows) are the B-operand
//    layout for Q S, again up to a permutation of the contraction index that the Q
//    operand read applies.
// Accumulator layout of a 32x32 tile: lane l holds column l%32 and, in register r,
// row 8*(r/4) + 4*(l/32) + r%4.  A/B operand layout: lane l holds row (A) or column
// (B) l%32 and contraction indices 8*(l/32) .. 8*(l/32)+7.
#include "leet_common.hpp"

namespace leet {

template <int D>
struct Bf16Smem {
    static constexpr int QS = D + 8;  // padded row stride (elements): 16-byte reads of 32 rows spread over all banks
    uint16_t q[kChunk * QS];          // Q_t   [i][dk]
    uint16_t k[kChunk * QS];          // K_t   [j][dk]
    uint16_t kt[D * kChunk];          // (Gam K_t)^T [dk][j], 16-byte slots XOR-swizzled
    uint16_t vt[D * kChunk];          // V_t^T [c][j], same swizzle
    float pw[kChunk + 4];             // gamma^n, n = 0..64
};

// Element offset of (row, j) inside a transposed tile: rows are 64 elements (128 B,
// eight 16-byte slots); the slot index is XORed with a row hash so that both the
// column-wise staging writes and the row-wise operand reads spread over the banks.
__device__ __forceinline__ int tr_off(int row, int j) {
    int slot = (j >> 3) ^ ((row ^ (row >> 3)) & 7);
    return row * kChunk + slot * 8 + (j & 7);
}

__device__ __forceinline__ bf16x8 frag16(const uint16_t* p) {
    return __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(p));
}

__device__ __forceinline__ bf16x8 frag8x2(const uint16_t* p0, const uint16_t* p1) {
    u32x2 a = *reinterpret_cast<const u32x2*>(p0);
    u32x2 b = *reinterpret_cast<const u32x2*>(p1);
    u32x4 r = {a.x, a.y, b.x, b.y};
    return __builtin_bit_cast(bf16x8, r);
}

// registers 8h .. 8h+7 of an accumulator tile -> bf16 operand
__device__ __forceinline__ bf16x8 pack_half(const f32x16& acc, int h) {
    bf16x8 r;
#pragma unroll
    for (int e = 0; e < 8; ++e) r[e] = (__bf16)acc[8 * h + e];
    return r;
}

template <int D>
struct StageMap {
    static constexpr int PR = D / 8;       // 16-byte pieces per row
    static constexpr int RW = 64 / PR;     // rows covered by one wave-wide load
    int cc;                                // piece index within the row
    int jbase;                             // row of load r is jbase + (r&1) + 2*RW*(r>>1)
    __device__ StageMap(int tid) {
        int w = tid >> 6, l = tid & 63;
        cc = l % PR;
        jbase = w * (4 * RW) + 2 * (l / PR);
    }
    __device__ __forceinline__ int row(int r) const { return jbase + (r & 1) + 2 * RW * (r >> 1); }
};

// kOut = true : full walk (outputs + state).   kOut = false : state only (segment
// pre-pass: the end state of a segment started from zero).
template <int D, bool kOut>
__global__ __launch_bounds__(D * 2) void fwd_bf16_kernel(FwdParams p) {
    constexpr int NW = D / 32;   // waves = 32-column slices
    constexpr int DT = D / 32;   // 32-row tiles of the key dimension
    constexpr int QS = Bf16Smem<D>::QS;
    __shared__ __attribute__((aligned(16))) Bf16Smem<D> sm;

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
    const uint16_t* qb = reinterpret_cast<const uint16_t*>(p.q) + seq_off;
    const uint16_t* kb = reinterpret_cast<const uint16_t*>(p.k) + seq_off;
    const uint16_t* vb = reinterpret_cast<const uint16_t*>(p.v) + seq_off;
    float* ob = p.out + seq_off;

    // decay table, fp64 -> fp32 once per workgroup
    {
        const double gd = (double)p.gamma[h];
        for (int n = tid; n <= kChunk; n += D * 2) sm.pw[n] = (float)pow_int(gd, n);
    }

    // state slice S[:, 32w .. 32w+31]
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

    const StageMap<D> sm_map(tid);
    u32x4 rq[4], rk[4], rv[4];
    auto prefetch = [&](int tok0) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            int j = sm_map.row(r);
            bool ok = tok0 + j < tok_end;
            size_t off = (size_t)(tok0 + j) * D + sm_map.cc * 8;
            u32x4 z = {0u, 0u, 0u, 0u};
            if (kOut) rq[r] = ok ? *reinterpret_cast<const u32x4*>(qb + off) : z;
            rk[r] = ok ? *reinterpret_cast<const u32x4*>(kb + off) : z;
            rv[r] = ok ? *reinterpret_cast<const u32x4*>(vb + off) : z;
        }
    };

    prefetch(tok_begin);
    __syncthreads();  // pw visible

    for (int t = 0; t < nchunks; ++t) {
        const int tok0 = tok_begin + t * kChunk;
        const int Lc = min(kChunk, tok_end - tok0);

        if (t > 0) __syncthreads();  // everyone is done reading the previous chunk's tiles
        // ---- registers -> LDS (row-major Q, K; transposed, Gam-scaled K; transposed V)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int j = sm_map.row(r);
            const int cc = sm_map.cc;
            if (kOut) {
                *reinterpret_cast<u32x4*>(&sm.q[j * QS + cc * 8]) = rq[r];
                *reinterpret_cast<u32x4*>(&sm.k[j * QS + cc * 8]) = rk[r];
            }
            const float sc = sm.pw[max(Lc - 1 - j, 0)];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                uint32_t kw = rk[r][e >> 1], vw = rv[r][e >> 1];
                uint32_t kbits = (e & 1) ? (kw >> 16) : (kw & 0xffffu);
                uint32_t vbits = (e & 1) ? (vw >> 16) : (vw & 0xffffu);
                __bf16 ks = (__bf16)(bf16_bits_to_f32(kbits) * sc);
                sm.kt[tr_off(cc * 8 + e, j)] = __builtin_bit_cast(uint16_t, ks);
                sm.vt[tr_off(cc * 8 + e, j)] = (uint16_t)vbits;
            }
        }
        __syncthreads();
        if (t + 1 < nchunks) prefetch(tok0 + kChunk);  // in flight during the MFMA work below

        if (kOut) {
            f32x16 o[2];
#pragma unroll
            for (int it = 0; it < 2; ++it)
#pragma unroll
                for (int r = 0; r < 16; ++r) o[it][r] = 0.0f;

            // ---- inter-chunk term: O = Q_t S_t, then rows scaled by gamma^(i+1)
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                for (int hh = 0; hh < 2; ++hh) {
                    const bf16x8 sb = pack_half(S[dt], hh);
                    const int dk0 = 32 * dt + 16 * hh + 4 * g;
#pragma unroll
                    for (int it = 0; it < 2; ++it) {
                        const uint16_t* row = &sm.q[(32 * it + ln) * QS + dk0];
                        o[it] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag8x2(row, row + 8), sb, o[it], 0, 0, 0);
                    }
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
                    for (int s = 0; s < D / 16; ++s) {
                        bf16x8 a = frag16(&sm.k[(32 * jt + ln) * QS + 16 * s + 8 * g]);
                        bf16x8 b = frag16(&sm.q[(32 * it + ln) * QS + 16 * s + 8 * g]);
                        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc, 0, 0, 0);
                    }
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        int n = 32 * (it - jt) + ln - (8 * (r >> 2) + 4 * g + (r & 3));  // i - j
                        float wgt = sm.pw[max(n, 0)];
                        acc[r] = (n >= 0) ? acc[r] * wgt : 0.0f;
                    }
#pragma unroll
                    for (int hh = 0; hh < 2; ++hh) {
                        const int j0 = 32 * jt + 16 * hh + 4 * g;
                        bf16x8 b = frag8x2(&sm.vt[tr_off(c_own, j0)], &sm.vt[tr_off(c_own, j0 + 8)]);
                        o[it] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pack_half(acc, hh), b, o[it], 0, 0, 0);
                    }
                }

            // ---- store O_t[:, cols]: per register, 32 lanes write 128 contiguous bytes of one row
#pragma unroll
            for (int it = 0; it < 2; ++it)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    int i = 32 * it + 8 * (r >> 2) + 4 * g + (r & 3);
                    if (i < Lc) ob[(size_t)(tok0 + i) * D + c_own] = o[it][r];
                }
        }

        // ---- state update: S = gamma^L S + (Gam K)^T V
        {
            const float gl = sm.pw[Lc];
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                for (int r = 0; r < 16; ++r) S[dt][r] *= gl;
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const int j0 = 16 * s + 8 * g;
                bf16x8 b = frag16(&sm.vt[tr_off(c_own, j0)]);
#pragma unroll
                for (int dt = 0; dt < DT; ++dt) {
                    bf16x8 a = frag16(&sm.kt[tr_off(32 * dt + ln, j0)]);
                    S[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, S[dt], 0, 0, 0);
                }
            }
        }
    }

    // ---- hand the state on
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

hipError_t launch_fwd_bf16_states(const FwdParams& p, int BH, int D, hipStream_t stream) {
    if (p.nseg <= 1) return hipSuccess;
    if (D == 64) hipLaunchKernelGGL((fwd_bf16_kernel<64, false>), dim3(BH * (p.nseg - 1)), dim3(128), 0, stream, p);
    else hipLaunchKernelGGL((fwd_bf16_kernel<128, false>), dim3(BH * (p.nseg - 1)), dim3(256), 0, stream, p);
    return hipGetLastError();
}

hipError_t launch_fwd_bf16_walk(const FwdParams& p, int BH, int D, hipStream_t stream) {
    if (D == 64) hipLaunchKernelGGL((fwd_bf16_kernel<64, true>), dim3(BH * p.nseg), dim3(128), 0, stream, p);
    else hipLaunchKernelGGL((fwd_bf16_kernel<128, true>), dim3(BH * p.nseg), dim3(256), 0, stream, p);
    return hipGetLastError();
}

}  // namespace leet
