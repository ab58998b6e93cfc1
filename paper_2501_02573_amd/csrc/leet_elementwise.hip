// The two element-wise (MFMA-free) prefill kernels: the in-library comparison points for the
// chunked kernels.  Both evaluate, per (batch, head) and value column c, for every rank index j
//
//     run_j <- lambda run_j + k_ij v_i[c]          (one entry of the state / carried vector)
//     o_i[c] += q_ij run_j
//
// -- 3 N r d multiply-adds on the vector ALUs, bound by fp32 VALU issue, not by memory -- and
// differ in the order of the loops, which is what distinguishes the two methods in the paper:
//
// Row-based (Alg. 1, Appendix B.1, with the discounted update of Appendix C.1): token by token,
//     S <- gamma S + k_i^T v_i ;  o_i = q_i S,
// the decode step iterated over N with the state on chip.  The paper's fastest method at batch
// 16 is of this kind (Section 5.1).
//
// FleetAttention (Section 3, Eq. "p"; decayed form Appendix C.1; blocked form Alg. 5, Appendix
// B.4): the operator as a sum over the rank of discounted cumulative sums,
//     O = sum_j diag(b_j) . lambda-cumsum( diag(c_j) V ),        b_j, c_j = columns j of Q and K,
// block by block as Alg. 5 lays it out: V is cut into column blocks that are computed in
// parallel and into row blocks that are taken in order; for every rank index j a vector l^j (one
// entry per column of the block) carries the discounted sum over all earlier row blocks,
//     O_blk  += diag(b_j,blk) ( lambda-cumsum( diag(c_j,blk) V_blk ), seeded with l^j )
//     l^j    <- the last row of that seeded cumsum.
// All of it is Hadamard work, no matrix product, which is the paper's point about this form (end
// of Section 3).  The vectors l^j are the rows of the state S of the other form.
//
// Mapping (both).  One workgroup per (batch, head) and block of 32 value columns (B_c = 32); row
// blocks of 32 tokens (B_r = 32) staged through LDS as fp32 with the next block's loads in
// flight.  The rank is split over G groups of threads: thread (column c, group g) owns ranks
// g r/G .. (g+1) r/G - 1 and keeps their state entries in registers for the whole sequence.
// Per row block the row-based order walks the tokens and, for each, its ranks four at a time;
// the FleetAttention order takes four ranks at a time and runs their seeded cumsums down the 32
// tokens (four independent chains).  Either way a thread ends the block with 32 partial outputs.
// The sum over the rank that the paper's FleetAttention performs with atomic additions into O
// (Appendix E) is here a sum of the G groups' partial outputs through LDS when the block is
// stored: one workgroup owns its column block, so nothing is shared between workgroups and no
// atomics are needed.  G = 16 (512 threads): with the 4 groups of an earlier version a
// 64-sequence job left half of the SIMDs empty and the rest with a single wave each.
#include <type_traits>

#include "leet_common.hpp"

namespace leet {

struct RowParams {
    const void* q;          // [BH][N][D]   (B in the paper's notation)
    const void* k;          // [BH][N][D]   (C)
    const void* v;          // [BH][N][DV]
    const float* gamma;     // [H] or null (lambda = 1: plain cumsum)
    float* out;             // [BH][N][DV] fp32
    const float* state_in;  // [BH][D][DV] or null: the state (the vectors l^j) entering the first row block
    float* state_out;       // [BH][D][DV] or null: l^j after the last
    int BH;                 // number of (batch, head) pairs
    int H;
    int N;
};

constexpr int kRowBlock = 32;  // tokens per staged row block (B_r)
constexpr int kColBlock = 32;  // value columns per workgroup (B_c)

// D: rank; DV: width of v and out rows; kElem: 0 = fp32, 1 = bf16, 2 = fp16 inputs; G: rank groups;
// kRankMajor: FleetAttention's loop order (ranks outside, tokens inside) instead of the row-based one
template <int D, int DV, int kElem, int G, bool kRankMajor>
__global__ __launch_bounds__(32 * G) void elementwise_kernel(RowParams p) {
    constexpr int NT = 32 * G;
    constexpr int R = D / G;                              // ranks per thread
    constexpr int PR = D / 8;                             // 8-element pieces per row of q or k
    constexpr int QK_PIECES = kRowBlock * PR / NT;       // pieces per thread per block (0 if NT is larger)
    constexpr int QK_TOTAL = kRowBlock * PR;
    static_assert(R % 4 == 0, "four ranks at a time");
    __shared__ __attribute__((aligned(16))) float sq[kRowBlock][D];
    __shared__ __attribute__((aligned(16))) float sk[kRowBlock][D];
    __shared__ __attribute__((aligned(16))) float sv[kRowBlock][kColBlock];
    __shared__ __attribute__((aligned(16))) float so[G][kRowBlock][kColBlock + 1];  // per rank group

    const int tid = threadIdx.x;
    const int c = tid & 31, g = tid >> 5;
    // Block -> (sequence, column block).  Consecutive block ids go round-robin over the 8 XCDs; the
    // column blocks of one sequence take ids that are equal modulo 8, so they share one L2 and
    // Q and K come from HBM once (671 MB fetched per launch on config 3 with consecutive ids).
    constexpr int SLICES = DV / kColBlock;
    const int gx = blockIdx.x & 7, rest = blockIdx.x >> 3;
    const int bh = (rest / SLICES) * 8 + gx;
    if (bh >= p.BH) return;
    const int c0 = (rest % SLICES) * kColBlock;
    const float lam = p.gamma ? p.gamma[bh % p.H] : 1.0f;
    const size_t seq_off = (size_t)bh * p.N * D, seq_off_v = (size_t)bh * p.N * DV;
    float* ob = p.out + seq_off_v;

    float L[R];  // S[j][c] = l^j[c] for this thread's ranks
    {
        const float* src = p.state_in ? p.state_in + (size_t)bh * D * DV : nullptr;
#pragma unroll
        for (int e = 0; e < R; ++e) L[e] = src ? src[(size_t)(g * R + e) * DV + c0 + c] : 0.0f;
    }

    // eight consecutive elements of a tensor as fp32 (zeros past the end of the sequence)
    auto fetch8 = [&](const void* base, size_t elem_off, bool ok, float* dst) {
        if (!ok) {
#pragma unroll
            for (int e = 0; e < 8; ++e) dst[e] = 0.0f;
        } else if (kElem == 0) {
            const f32x4* src = reinterpret_cast<const f32x4*>(static_cast<const float*>(base) + elem_off);
            const f32x4 a = src[0], b = src[1];
#pragma unroll
            for (int e = 0; e < 4; ++e) { dst[e] = a[e]; dst[4 + e] = b[e]; }
        } else {
            const u32x4 x = *reinterpret_cast<const u32x4*>(static_cast<const uint16_t*>(base) + elem_off);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                dst[2 * e] = kElem == 1 ? ElemBf16::lo(x[e]) : ElemF16::lo(x[e]);
                dst[2 * e + 1] = kElem == 1 ? ElemBf16::hi(x[e]) : ElemF16::hi(x[e]);
            }
        }
    };
    // staging: q and k pieces m NT + tid (row = piece / PR); v: the first 128 threads, row tid/4, columns 8 (tid%4)
    constexpr int NP = QK_PIECES > 0 ? QK_PIECES : 1;
    float rq[NP][8], rk[NP][8], rv[8];
    const int vrow = tid >> 2, vcol = 8 * (tid & 3);
    const bool v_thread = tid < kRowBlock * 4;
    auto prefetch = [&](int tok0) {
#pragma unroll
        for (int m = 0; m < NP; ++m) {
            const int piece = m * NT + tid;
            if (piece < QK_TOTAL) {
                const int row = piece / PR;
                const bool ok = tok0 + row < p.N;
                const size_t off = seq_off + (size_t)(tok0 + row) * D + (size_t)(piece % PR) * 8;
                fetch8(p.q, off, ok, rq[m]);
                fetch8(p.k, off, ok, rk[m]);
            }
        }
        if (v_thread) fetch8(p.v, seq_off_v + (size_t)(tok0 + vrow) * DV + c0 + vcol, tok0 + vrow < p.N, rv);
    };

    prefetch(0);
    for (int tok0 = 0; tok0 < p.N; tok0 += kRowBlock) {
        const int nt = min(kRowBlock, p.N - tok0);
        __syncthreads();  // the previous block's so[] has been stored, its sq/sk/sv consumed
#pragma unroll
        for (int m = 0; m < NP; ++m) {
            const int piece = m * NT + tid;
            if (piece < QK_TOTAL) {
                float* dq = &sq[piece / PR][(piece % PR) * 8];
                float* dk = &sk[piece / PR][(piece % PR) * 8];
#pragma unroll
                for (int e = 0; e < 8; e += 4) {
                    *reinterpret_cast<f32x4*>(dq + e) = f32x4{rq[m][e], rq[m][e + 1], rq[m][e + 2], rq[m][e + 3]};
                    *reinterpret_cast<f32x4*>(dk + e) = f32x4{rk[m][e], rk[m][e + 1], rk[m][e + 2], rk[m][e + 3]};
                }
            }
        }
        if (v_thread) {
#pragma unroll
            for (int e = 0; e < 8; e += 4)
                *reinterpret_cast<f32x4*>(&sv[vrow][vcol + e]) = f32x4{rv[e], rv[e + 1], rv[e + 2], rv[e + 3]};
        }
        __syncthreads();
        if (tok0 + kRowBlock < p.N) prefetch(tok0 + kRowBlock);

        // V_blk[:, c] and the partial outputs of this thread's ranks
        float vv[kRowBlock], o[kRowBlock];
#pragma unroll
        for (int i = 0; i < kRowBlock; ++i) { vv[i] = sv[i][c]; o[i] = 0.0f; }
        // ragged: the block holds fewer than B_r tokens; rows past the end must not discount the state
        auto rank_sweep = [&](auto ragged) {
            if (kRankMajor) {
#pragma unroll
                for (int e4 = 0; e4 < R; e4 += 4) {
                    f32x4 run = {L[e4], L[e4 + 1], L[e4 + 2], L[e4 + 3]};  // seeded with l^j
#pragma unroll
                    for (int i = 0; i < kRowBlock; ++i) {
                        if (!decltype(ragged)::value || i < nt) {
                            const f32x4 cc = *reinterpret_cast<const f32x4*>(&sk[i][g * R + e4]);
                            const f32x4 bb = *reinterpret_cast<const f32x4*>(&sq[i][g * R + e4]);
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                run[e] = fmaf(lam, run[e], cc[e] * vv[i]);   // lambda-cumsum of diag(c_j) V
                                o[i] = fmaf(bb[e], run[e], o[i]);            // diag(b_j) times it, summed over j
                            }
                        }
                    }
#pragma unroll
                    for (int e = 0; e < 4; ++e) L[e4 + e] = run[e];          // l^j for the next row block
                }
            } else {
#pragma unroll
                for (int i = 0; i < kRowBlock; ++i) {
                    if (!decltype(ragged)::value || i < nt) {
                        f32x4 acc = {0.f, 0.f, 0.f, 0.f};  // four independent chains
#pragma unroll
                        for (int e4 = 0; e4 < R; e4 += 4) {
                            const f32x4 kk = *reinterpret_cast<const f32x4*>(&sk[i][g * R + e4]);
                            const f32x4 qq = *reinterpret_cast<const f32x4*>(&sq[i][g * R + e4]);
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                L[e4 + e] = fmaf(lam, L[e4 + e], kk[e] * vv[i]);   // S <- gamma S + k_i^T v_i
                                acc[e] = fmaf(qq[e], L[e4 + e], acc[e]);           // o_i = q_i S
                            }
                        }
                        o[i] = (acc[0] + acc[1]) + (acc[2] + acc[3]);
                    }
                }
            }
        };
        if (nt == kRowBlock) rank_sweep(std::false_type{});
        else rank_sweep(std::true_type{});
#pragma unroll
        for (int i = 0; i < kRowBlock; ++i) so[g][i][c] = o[i];
        __syncthreads();
        // the rank groups are summed on the way out: thread -> (row, four columns), 128-byte row pieces
        for (int item = tid; item < kRowBlock * (kColBlock / 4); item += NT) {
            const int row = item >> 3, col = 4 * (item & 7);
            if (row < nt) {
                f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int gg = 0; gg < G; ++gg)
#pragma unroll
                    for (int e = 0; e < 4; ++e) acc[e] += so[gg][row][col + e];
                __builtin_nontemporal_store(acc, reinterpret_cast<f32x4*>(ob + (size_t)(tok0 + row) * DV + c0 + col));
            }
        }
    }

    if (p.state_out) {
        float* dst = p.state_out + (size_t)bh * D * DV;
#pragma unroll
        for (int e = 0; e < R; ++e) dst[(size_t)(g * R + e) * DV + c0 + c] = L[e];
    }
}

constexpr int kRankGroups = 16;  // 512 threads per workgroup

template <int D, int DV, bool kRankMajor>
static void launch_elementwise_d(const RowParams& p, int BH, int elem, hipStream_t stream) {
    dim3 grid(8 * (DV / kColBlock) * ((BH + 7) / 8)), block(32 * kRankGroups);
    if (elem == 0) hipLaunchKernelGGL((elementwise_kernel<D, DV, 0, kRankGroups, kRankMajor>), grid, block, 0, stream, p);
    else if (elem == 1) hipLaunchKernelGGL((elementwise_kernel<D, DV, 1, kRankGroups, kRankMajor>), grid, block, 0, stream, p);
    else hipLaunchKernelGGL((elementwise_kernel<D, DV, 2, kRankGroups, kRankMajor>), grid, block, 0, stream, p);
}

template <bool kRankMajor>
static hipError_t launch_elementwise(const void* q, const void* k, const void* v, const float* gamma, float* out,
                                     const float* state_in, float* state_out, int BH, int H, int N, int D, int DV,
                                     int elem, hipStream_t stream) {
    RowParams p;
    p.q = q; p.k = k; p.v = v; p.gamma = gamma; p.out = out;
    p.state_in = state_in; p.state_out = state_out; p.BH = BH; p.H = H; p.N = N;
    if (D == 64) launch_elementwise_d<64, 64, kRankMajor>(p, BH, elem, stream);
    else if (DV == 128) launch_elementwise_d<128, 128, kRankMajor>(p, BH, elem, stream);
    else launch_elementwise_d<128, 256, kRankMajor>(p, BH, elem, stream);
    return hipGetLastError();
}

// elem: 0 = fp32, 1 = bf16, 2 = fp16 inputs; gamma null means gamma = 1;
// (D, DV) one of (64, 64), (128, 128), (128, 256)
hipError_t launch_recurrent(const void* q, const void* k, const void* v, const float* gamma, float* out,
                            const float* state_in, float* state_out, int BH, int H, int N, int D, int DV,
                            int elem, hipStream_t stream) {
    return launch_elementwise<false>(q, k, v, gamma, out, state_in, state_out, BH, H, N, D, DV, elem, stream);
}

hipError_t launch_fleet(const void* q, const void* k, const void* v, const float* gamma, float* out,
                        const float* state_in, float* state_out, int BH, int H, int N, int D, int DV,
                        int elem, hipStream_t stream) {
    return launch_elementwise<true>(q, k, v, gamma, out, state_in, state_out, BH, H, N, D, DV, elem, stream);
}

}  // namespace leet
