// Chunk-walk kernel for fp32 inputs (gfx950, v_mfma_f32_16x16x4_f32: true fp32 products).
//
// Same algorithm as the wide 16-bit kernel: one workgroup per segment of a (batch, head) sequence
// walks 64-token chunks (Alg. 2, Appendix B.2, with the decaying mask of Eq. "BCMV" and the
// weight split of Alg. 4, Appendix B.3):
//
//     O_t     = ((Q_t K_t^T) .* D) V_t + Lam (Q_t S_t)       D[i][j] = gamma^(i-j), i >= j
//     S_{t+1} = gamma^L S_t + (Gam K_t)^T V_t                Lam = diag(gamma^(i+1)), Gam = diag(gamma^(L-1-j))
//
// fp32 MFMA is 16 times slower than bf16 MFMA, so this kernel is bound by MFMA issue and
// latency, not by HBM; the work is therefore cut finer than in the 16-bit kernels: wave w owns
// 16 value columns [16w, 16w+16) of O and of the state S (d/16 waves per workgroup), and all
// products are 16x16x4 tiles.
//
// MFMA conventions (16x16x4 fp32): an A (B) operand is one float per lane: lane l holds row
// (column) l%16 and contraction slot q = l/16; an accumulator holds, in lane l, column l%16
// and, in register r, row 4q + r.  A contraction may assign indices to slots in any way, as
// long as A and B agree.  Everything is computed transposed (lane = token), so that an
// accumulator register of one product is directly an operand of the next:
//   G1  P^T[j][i]  = sum_dk K[j][dk] Q[i][dk]        A, B: 16-byte LDS reads, 4 MFMAs each
//       P^T       *= D^T                             per-lane weights, fixed for the kernel
//   G3  O^T[c][i]  = sum_dk S^T[c][dk] Q^T[dk][i]    A = S accumulator registers, B = Q rows
//       O^T       *= gamma^(i+1)                     one scalar per lane, since lane = token
//   G2  O^T[c][i] += sum_j V^T[c][j] P^T[j][i]       A = V[j][c] for j = 16jt + 4q + r, B = P^T registers
//   G4  S[dk][c]  += sum_j K^T[dk][j] (Gam V)[j][c]  A = K[j][dk], B = the V registers of G2 times Gam
// The 64 x 64 score matrix has ten non-zero 16 x 16 tiles; each is computed once per workgroup
// (tile n by wave n mod #waves), masked, and handed to the other waves through LDS in
// operand-register order.
//
// A ragged last chunk (L < 64) is right-aligned in the tile: rows 64-L.. hold the tokens,
// rows above are zero, so the intra-chunk weights (functions of i-j and of 63-j) stay valid;
// only Lam and gamma^L depend on L.
#include "leet_common.hpp"

namespace leet {

// The pre-pass (kOut = false) reads no Q and forms no scores: without those two members its
// workgroups are small enough for two to share a compute unit at d = 128.
template <int D, bool kOut>
struct F32Smem {
    static constexpr int RS = D + 4;  // padded row stride (floats)
    float q[kOut ? kChunk * RS : 4];
    float k[kChunk * RS];
    float v[kChunk * RS];
    f32x4 pfrag[kOut ? 10 : 1][64];   // masked P^T tiles: [tile][lane], registers 0..3
    float pw[kChunk + 4];             // gamma^n, n = 0..64
};

// The ten score tiles (it >= jt) in production order.
__device__ __forceinline__ constexpr int f32_tile_it(int n) { return n < 1 ? 0 : n < 3 ? 1 : n < 6 ? 2 : 3; }
__device__ __forceinline__ constexpr int f32_tile_jt(int n) { return n - (f32_tile_it(n) * (f32_tile_it(n) + 1)) / 2; }

// kOut = true : full walk (outputs + state).   kOut = false : state only (segment pre-pass).
template <int D, bool kOut>
__global__ __launch_bounds__(D * 4, (kOut || D < 128) ? 2 : 4) void fwd_f32_kernel(FwdParams p) {
    constexpr int NT = D * 4;                  // threads: one wave per 16 value columns
    constexpr int NW = D / 16;                 // waves
    constexpr int DT = D / 16;                 // 16-row tiles of the key dimension
    constexpr int RS = F32Smem<D, kOut>::RS;
    constexpr int PR = D / 4;                  // 16-byte pieces per row
    constexpr int NLOAD = kChunk * PR / NT;    // pieces per thread per tensor (= 4)
    constexpr int ROWS_PER_PASS = NT / PR;     // rows one pass of all threads covers (= 16)
    constexpr int NSLOT = (10 + NW - 1) / NW;  // score tiles per wave, at most
    __shared__ __attribute__((aligned(16))) F32Smem<D, kOut> sm;

    const int tid = threadIdx.x;
    const int w = tid >> 6, l = tid & 63, ln = l & 15, qd = l >> 4;
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
    float* ob = static_cast<float*>(p.out) + seq_off;

    {
        const double gd = p.no_decay ? 1.0 : (double)p.gamma[h];
        for (int n = tid; n <= kChunk; n += NT) sm.pw[n] = (float)pow_int(gd, n);
    }

    // state slice: S[t][r] = S[dk = 16t + 4q + r][c = 16w + ln]
    f32x4 S[DT];
    const int c_own = 16 * w + ln;
    {
        const float* src = nullptr;
        if (kOut) {
            if (seg == 0) src = p.state_in ? p.state_in + (size_t)bh * D * D : nullptr;
            else src = p.seg_state + ((size_t)bh * p.state_slots + (seg * p.state_step - 1)) * D * D;
        }
#pragma unroll
        for (int t = 0; t < DT; ++t)
#pragma unroll
            for (int r = 0; r < 4; ++r) S[t][r] = src ? src[(16 * t + 4 * qd + r) * D + c_own] : 0.0f;
    }

    __syncthreads();  // table visible

    // per-lane constants of the walk
    f32x4 wgt[NSLOT];   // decay weights of the score tiles this wave produces
    float gam[16];      // gamma^(63-j) for the keys j = 16jt + 4q + r this lane feeds to G2 and G4
#pragma unroll
    for (int n = 0; n < 10; ++n) {
        if (n % NW != w) continue;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int d = 16 * (f32_tile_it(n) - f32_tile_jt(n)) + ln - (4 * qd + r);  // i - j
            wgt[n / NW][r] = (d >= 0) ? sm.pw[max(d, 0)] : 0.0f;
        }
    }
#pragma unroll
    for (int e = 0; e < 16; ++e) gam[e] = sm.pw[kChunk - 1 - (16 * (e >> 2) + 4 * qd + (e & 3))];

    // staging: piece r of this thread is row ROWS_PER_PASS*r + tid/PR, floats 4(tid%PR)..+3
    const int j0 = tid / PR, cc = tid % PR;
    f32x4 rq[NLOAD], rk[NLOAD], rv[NLOAD];
    auto prefetch = [&](int tok0) {
        const int shift = max(0, tok0 + kChunk - tok_end);  // rows [0, shift) of the tile stay zero
#pragma unroll
        for (int r = 0; r < NLOAD; ++r) {
            const int j = ROWS_PER_PASS * r + j0;
            const bool ok = j >= shift;
            const size_t off = (size_t)(tok0 - shift + j) * D + cc * 4;
            const f32x4 z = {0.f, 0.f, 0.f, 0.f};
            if (kOut) rq[r] = ok ? *reinterpret_cast<const f32x4*>(qb + off) : z;
            rk[r] = ok ? *reinterpret_cast<const f32x4*>(kb + off) : z;
            rv[r] = ok ? *reinterpret_cast<const f32x4*>(vb + off) : z;
        }
    };

    prefetch(tok_begin);

    for (int t = 0; t < nchunks; ++t) {
        const int tok0 = tok_begin + t * kChunk;
        const int Lc = min(kChunk, tok_end - tok0);
        const int shift = kChunk - Lc;

        if (t > 0) __syncthreads();  // everyone is done reading the previous chunk's tiles and P fragments
#pragma unroll
        for (int r = 0; r < NLOAD; ++r) {
            const int j = ROWS_PER_PASS * r + j0;
            if (kOut) *reinterpret_cast<f32x4*>(&sm.q[j * RS + cc * 4]) = rq[r];
            *reinterpret_cast<f32x4*>(&sm.k[j * RS + cc * 4]) = rk[r];
            *reinterpret_cast<f32x4*>(&sm.v[j * RS + cc * 4]) = rv[r];
        }
        __syncthreads();
        if (t + 1 < nchunks) prefetch(tok0 + kChunk);  // in flight during the MFMA work below

        f32x4 o[4];
        if (kOut) {
            // G1 + mask for the score tiles this wave produces
#pragma unroll
            for (int n = 0; n < 10; ++n) {
                if (n % NW != w) continue;
                f32x4 acc = {0.f, 0.f, 0.f, 0.f};
                const float* krow = &sm.k[(16 * f32_tile_jt(n) + ln) * RS + 4 * qd];
                const float* qrow = &sm.q[(16 * f32_tile_it(n) + ln) * RS + 4 * qd];
#pragma unroll
                for (int s = 0; s < D / 16; ++s) {
                    const f32x4 a = *reinterpret_cast<const f32x4*>(krow + 16 * s);
                    const f32x4 b = *reinterpret_cast<const f32x4*>(qrow + 16 * s);
#pragma unroll
                    for (int e = 0; e < 4; ++e) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a[e], b[e], acc, 0, 0, 0);
                }
                sm.pfrag[n][l] = acc * wgt[n / NW];
            }

            // G3: O^T = S^T Q^T, rows of O scaled by gamma^(i+1)
#pragma unroll
            for (int it = 0; it < 4; ++it) {
                f32x4 acc = {0.f, 0.f, 0.f, 0.f};
                const float* qrow = &sm.q[(16 * it + ln) * RS + 4 * qd];
#pragma unroll
                for (int dt = 0; dt < DT; ++dt) {
                    const f32x4 b = *reinterpret_cast<const f32x4*>(qrow + 16 * dt);
#pragma unroll
                    for (int e = 0; e < 4; ++e) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(S[dt][e], b[e], acc, 0, 0, 0);
                }
                o[it] = acc * sm.pw[max(16 * it + ln + 1 - shift, 0)];
            }
        }

        // V registers: va[4jt + r] = V[j = 16jt + 4q + r][c_own]
        float va[16];
#pragma unroll
        for (int e = 0; e < 16; ++e) va[e] = sm.v[(16 * (e >> 2) + 4 * qd + (e & 3)) * RS + c_own];

        if (kOut) {
            __syncthreads();  // P fragments visible
            // G2: O^T += V^T P^T over the tiles (jt <= it)
#pragma unroll
            for (int n = 0; n < 10; ++n) {
                const f32x4 pt = sm.pfrag[n][l];
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    o[f32_tile_it(n)] = __builtin_amdgcn_mfma_f32_16x16x4f32(va[4 * f32_tile_jt(n) + r], pt[r],
                                                                            o[f32_tile_it(n)], 0, 0, 0);
            }
            // store O^T: lane = token 16it + ln, registers = columns 16w + 4q + (0..3)
#pragma unroll
            for (int it = 0; it < 4; ++it) {
                const int i = 16 * it + ln;
                if (i >= shift)  // written once, not read again here: nontemporal
                    __builtin_nontemporal_store(o[it], reinterpret_cast<f32x4*>(ob + (size_t)(tok0 - shift + i) * D + 16 * w + 4 * qd));
            }
        }

        // G4: S = gamma^L S + K^T (Gam V); contraction slot q of step (jt, r) is key 16jt + 4q + r
        {
            const float gl = sm.pw[Lc];
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) S[dt] *= gl;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const float b = va[e] * gam[e];
                const float* krow = &sm.k[(16 * (e >> 2) + 4 * qd + (e & 3)) * RS + ln];
#pragma unroll
                for (int dt = 0; dt < DT; ++dt)
                    S[dt] = __builtin_amdgcn_mfma_f32_16x16x4f32(krow[16 * dt], b, S[dt], 0, 0, 0);
            }
        }
    }

    float* dst = nullptr;
    if (kOut) {
        if (seg == p.nseg - 1 && p.state_out) dst = p.state_out + (size_t)bh * D * D;
    } else {
        dst = p.seg_state + ((size_t)bh * p.state_slots + seg) * D * D;
    }
    if (dst) {
#pragma unroll
        for (int t = 0; t < DT; ++t)
#pragma unroll
            for (int r = 0; r < 4; ++r) dst[(16 * t + 4 * qd + r) * D + c_own] = S[t][r];
    }
}

hipError_t launch_fwd_f32_states(const FwdParams& p, int BH, int D, hipStream_t stream) {
    if (p.nseg <= 1) return hipSuccess;
    if (D == 64) hipLaunchKernelGGL((fwd_f32_kernel<64, false>), dim3(BH * (p.nseg - 1)), dim3(256), 0, stream, p);
    else hipLaunchKernelGGL((fwd_f32_kernel<128, false>), dim3(BH * (p.nseg - 1)), dim3(512), 0, stream, p);
    return hipGetLastError();
}

hipError_t launch_fwd_f32_walk(const FwdParams& p, int BH, int D, hipStream_t stream) {
    if (D == 64) hipLaunchKernelGGL((fwd_f32_kernel<64, true>), dim3(BH * p.nseg), dim3(256), 0, stream, p);
    else hipLaunchKernelGGL((fwd_f32_kernel<128, true>), dim3(BH * p.nseg), dim3(512), 0, stream, p);
    return hipGetLastError();
}

}  // namespace leet
