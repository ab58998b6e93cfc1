// Row-based prefill: the token-by-token recursion of Alg. 1 (Appendix B.1) with the
// discounted update of Appendix C.1,
//
//     S <- gamma S + k_i^T v_i ;   o_i = q_i S          for i = 0 .. N-1, per (batch, head),
//
// run on the GPU as it is written, with the d x d fp32 state held in registers for the whole
// sequence.  This is the decode step iterated over N with S on chip: no MFMA, parallel only over
// (batch, head) and the value columns, sequential in the token index.  It exists as the
// in-library comparison point for the chunked kernels (the paper's fastest method at batch 16
// is of this kind, Section 5.1) and as a second GPU route to the same result.
//
// One workgroup of two waves per (batch, head) and 32 value columns, one wave per 16 columns;
// the d/32 workgroups of a sequence are independent (columns of S never mix).  Lane l of wave w
// owns column c = c0 + 16w + l%16 and the key rows dk = (l/16) d/4 .. +d/4-1 of S (d/4
// registers).  Tokens are staged through LDS in blocks of 32, converted to fp32, with the next
// block's global loads in flight; per token a lane reads its d/4 entries of k_i and q_i (16-byte
// broadcast reads) and v_i[c], updates its S entries and sums its share of o_i[c]; the four row
// groups' partial sums go to LDS and are added up when the block's outputs are stored, in
// 128-byte row pieces, so that nothing in the token loop waits on another lane.
#include "leet_common.hpp"

namespace leet {

struct RecParams {
    const void* q;          // [BH][N][D]
    const void* k;
    const void* v;          // [BH][N][DV]
    const float* gamma;     // [H] or null (gamma = 1)
    float* out;             // [BH][N][DV] fp32
    const float* state_in;  // [BH][D][DV] or null
    float* state_out;       // [BH][D][DV] or null
    int H;
    int N;
};

constexpr int kRecBlock = 32;  // tokens per staged block

constexpr int kRecCols = 32;   // value columns per workgroup

// D: width of q and k rows (rank); DV: width of v and out rows.  kElem: 0 = fp32, 1 = bf16, 2 = fp16 inputs
template <int D, int DV, int kElem>
__global__ __launch_bounds__(128) void recurrent_kernel(RecParams p) {
    constexpr int NT = 128;
    constexpr int R = D / 4;                         // state rows per lane
    constexpr int QK_PIECES = kRecBlock * D / 8 / NT;  // 8-element pieces per thread per block of q or k
    constexpr int PR = D / 8;                        // pieces per row of q or k
    __shared__ __attribute__((aligned(16))) float sq[kRecBlock][D];
    __shared__ __attribute__((aligned(16))) float sk[kRecBlock][D];
    __shared__ __attribute__((aligned(16))) float sv[kRecBlock][kRecCols];
    __shared__ __attribute__((aligned(16))) float so[4][kRecBlock][kRecCols];  // per row group

    const int tid = threadIdx.x;
    const int w = tid >> 6, l = tid & 63, c = l & 15, rg = l >> 4;
    constexpr int SLICES = DV / kRecCols;
    const int bh = blockIdx.x / SLICES;
    const int c0 = (blockIdx.x % SLICES) * kRecCols;
    const int cl = 16 * w + c;                       // column within the slice
    const float gm = p.gamma ? p.gamma[bh % p.H] : 1.0f;
    const size_t seq_off = (size_t)bh * p.N * D, seq_off_v = (size_t)bh * p.N * DV;
    float* ob = p.out + seq_off_v;

    float S[R];
    {
        const float* src = p.state_in ? p.state_in + (size_t)bh * D * DV : nullptr;
#pragma unroll
        for (int e = 0; e < R; ++e) S[e] = src ? src[(size_t)(rg * R + e) * DV + c0 + cl] : 0.0f;
    }

    // eight consecutive elements of a tensor, converted to fp32 (zeros past the end of the sequence)
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
    // staging: q and k pieces m*NT + tid (row = piece / PR); v and o: row tid/4, columns 8(tid%4)..+7
    float rq[QK_PIECES][8], rk[QK_PIECES][8], rv[8];
    const int vrow = tid >> 2, vcol = 8 * (tid & 3);
    auto prefetch = [&](int tok0) {
#pragma unroll
        for (int m = 0; m < QK_PIECES; ++m) {
            const int piece = m * NT + tid;
            const int row = piece / PR;
            const bool ok = tok0 + row < p.N;
            const size_t off = seq_off + (size_t)(tok0 + row) * D + (size_t)(piece % PR) * 8;
            fetch8(p.q, off, ok, rq[m]);
            fetch8(p.k, off, ok, rk[m]);
        }
        fetch8(p.v, seq_off_v + (size_t)(tok0 + vrow) * DV + c0 + vcol, tok0 + vrow < p.N, rv);
    };

    prefetch(0);
    for (int tok0 = 0; tok0 < p.N; tok0 += kRecBlock) {
        const int nt = min(kRecBlock, p.N - tok0);
        __syncthreads();  // the previous block's so[] has been stored, its sq/sk/sv consumed
#pragma unroll
        for (int m = 0; m < QK_PIECES; ++m) {
            const int piece = m * NT + tid;
            float* dq = &sq[piece / PR][(piece % PR) * 8];
            float* dk = &sk[piece / PR][(piece % PR) * 8];
#pragma unroll
            for (int e = 0; e < 8; e += 4) {
                *reinterpret_cast<f32x4*>(dq + e) = f32x4{rq[m][e], rq[m][e + 1], rq[m][e + 2], rq[m][e + 3]};
                *reinterpret_cast<f32x4*>(dk + e) = f32x4{rk[m][e], rk[m][e + 1], rk[m][e + 2], rk[m][e + 3]};
            }
        }
#pragma unroll
        for (int e = 0; e < 8; e += 4)
            *reinterpret_cast<f32x4*>(&sv[vrow][vcol + e]) = f32x4{rv[e], rv[e + 1], rv[e + 2], rv[e + 3]};
        __syncthreads();
        if (tok0 + kRecBlock < p.N) prefetch(tok0 + kRecBlock);

#pragma unroll 2
        for (int i = 0; i < nt; ++i) {
            const float vv = sv[i][cl];
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};  // four independent chains
#pragma unroll
            for (int e4 = 0; e4 < R; e4 += 4) {
                const f32x4 kk = *reinterpret_cast<const f32x4*>(&sk[i][rg * R + e4]);
                const f32x4 qq = *reinterpret_cast<const f32x4*>(&sq[i][rg * R + e4]);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    S[e4 + e] = fmaf(gm, S[e4 + e], kk[e] * vv);
                    acc[e] = fmaf(qq[e], S[e4 + e], acc[e]);
                }
            }
            so[rg][i][cl] = (acc[0] + acc[1]) + (acc[2] + acc[3]);
        }
        __syncthreads();
        // the four row groups are summed on the way out
        if (vrow < nt) {
            float* dst = ob + (size_t)(tok0 + vrow) * DV + c0 + vcol;
#pragma unroll
            for (int e = 0; e < 8; e += 4) {
                const f32x4 a = *reinterpret_cast<const f32x4*>(&so[0][vrow][vcol + e]);
                const f32x4 b = *reinterpret_cast<const f32x4*>(&so[1][vrow][vcol + e]);
                const f32x4 cc = *reinterpret_cast<const f32x4*>(&so[2][vrow][vcol + e]);
                const f32x4 dd = *reinterpret_cast<const f32x4*>(&so[3][vrow][vcol + e]);
                __builtin_nontemporal_store((a + b) + (cc + dd), reinterpret_cast<f32x4*>(dst + e));
            }
        }
    }

    if (p.state_out) {
        float* dst = p.state_out + (size_t)bh * D * DV;
#pragma unroll
        for (int e = 0; e < R; ++e) dst[(size_t)(rg * R + e) * DV + c0 + cl] = S[e];
    }
}

template <int D, int DV>
static void launch_recurrent_d(const RecParams& p, int BH, int elem, hipStream_t stream) {
    dim3 grid(BH * (DV / kRecCols)), block(128);
    if (elem == 0) hipLaunchKernelGGL((recurrent_kernel<D, DV, 0>), grid, block, 0, stream, p);
    else if (elem == 1) hipLaunchKernelGGL((recurrent_kernel<D, DV, 1>), grid, block, 0, stream, p);
    else hipLaunchKernelGGL((recurrent_kernel<D, DV, 2>), grid, block, 0, stream, p);
}

// elem: 0 = fp32, 1 = bf16, 2 = fp16 inputs; gamma null means gamma = 1;
// (D, DV) one of (64, 64), (128, 128), (128, 256)
hipError_t launch_recurrent(const void* q, const void* k, const void* v, const float* gamma, float* out,
                            const float* state_in, float* state_out, int BH, int H, int N, int D, int DV,
                            int elem, hipStream_t stream) {
    RecParams p;
    p.q = q; p.k = k; p.v = v; p.gamma = gamma; p.out = out;
    p.state_in = state_in; p.state_out = state_out; p.H = H; p.N = N;
    if (D == 64) launch_recurrent_d<64, 64>(p, BH, elem, stream);
    else if (DV == 128) launch_recurrent_d<128, 128>(p, BH, elem, stream);
    else launch_recurrent_d<128, 256>(p, BH, elem, stream);
    return hipGetLastError();
}

}  // namespace leet
