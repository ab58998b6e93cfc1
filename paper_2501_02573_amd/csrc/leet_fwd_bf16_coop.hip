// Column-split chunk-walk kernel for bf16 inputs (gfx950, v_mfma_f32_16x16x32_bf16).
//
// Same mathematics as the wide kernel in leet_fwd_bf16.hip -- Alg. 2 (Appendix B.2) with the
// decaying mask of Eq. "BCMV" (Section 2.2) and the weight split of Alg. 4 (Appendix B.3):
//
//     O_t     = ((Q_t K_t^T) .* D) V_t + Lam (Q_t S_t)       D[i][j] = gamma^(i-j), i >= j
//     S_{t+1} = gamma^L S_t + (Gam K_t)^T V_t
//
// but a different split of the work, made for few, long sequences.  Value columns are
// independent of one another (O[:, c] and S[:, c] need only V[:, c]), so a sequence is
// handled by D/32 workgroups, one per 32-column slice, on D/32 compute units; each reads
// all of Q and K (the copies of one sequence are placed on one XCD so that three of the
// four reads hit its L2) and its own 32 columns of V, and writes its 32 columns of O.
// Inside a workgroup every product is cut into 16x16 tiles that are dealt out to the eight
// waves (two per SIMD, so that one hides the LDS and MFMA latency of the other); what one
// wave produces for the others goes through LDS in operand order:
//
//   G1  P^T tile (jq, iq) = K[16jq..][:] Q[16iq..][:]^T, masked, -> LDS P[i][j] (bf16)
//       ten tiles on and below the diagonal, one or two per wave
//   G3  O^T tile (ch, iq) = S^T[16ch..][:] Q^T[:][16iq..]      wave w does ch = w%2, iq = w/2;
//       S^T comes from LDS ST[c][dk] (bf16), written by the state owners after G4
//   G2  O^T tile (ch, iq) += V^T[16ch..][keys] P^T[keys][16iq..]   V through transposing reads
//   G4  S tile (dk block, ch) = gamma^L S + K^T (Gam V)         the (D/16) x 2 tiles dealt D/64 per wave
//
// MFMA conventions (16x16x32): an A (B) operand holds, in lane l, row (column) l%16 and the
// eight contraction slots 8(l/16)..8(l/16)+7; an accumulator holds, in lane l, column l%16
// and rows 4(l/16)..4(l/16)+3.  Outputs are accumulated transposed (lane = token), so Lam is
// one scalar per lane and a lane stores 16 contiguous bytes.
//
// Q, K, the V slice and its Gam-scaled copy are double-buffered in LDS: chunk t+1 is written
// from registers while chunk t is consumed and chunk t+2 is in flight from HBM, with two
// workgroup barriers per chunk.  A ragged last chunk is right-aligned in the tile (rows
// 64-L.. hold the tokens), which keeps every decay weight chunk-independent.
#include <stdlib.h>

#include <type_traits>

#include "leet_common.hpp"

namespace leet {

typedef short s16x4 __attribute__((ext_vector_type(4)));

template <int D>
struct CoopSmem {
    static constexpr int RSQ = D + 8;   // Q, K row stride (elements): 16-byte row reads spread over the banks
    static constexpr int RSV = 48;      // V slice: 32 columns + pad; 4 rows x 32 B of a transposing read stay apart
    static constexpr int RSP = 72;      // P[i][j]: 64 keys + pad
    static constexpr int RST = D + 8;   // S^T[c][dk]
    uint16_t q[2][kChunk * RSQ];
    uint16_t k[2][kChunk * RSQ];
    uint16_t v[2][kChunk * RSV];
    uint16_t vs[2][kChunk * RSV];       // Gam V: row j scaled by gamma^(63-j)
    uint16_t p[kChunk * RSP];
    uint16_t st[32 * RST];
    float pw[kChunk + 4];               // gamma^n, n = 0..64
};

namespace coop {

__device__ __forceinline__ bf16x8 frag16(const uint16_t* p) {
    return __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(p));
}

// ds_read_b64_tr_b16: within each group of 16 lanes, lane i receives element i%4 of the
// 8-byte rows addressed by lanes i/4, 4+i/4, 8+i/4, 12+i/4 of the group.
__device__ __forceinline__ u32x2 lds_tr(const uint16_t* p) {
    s16x4 r = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (__attribute__((address_space(3))) s16x4*)(const_cast<uint16_t*>(p)));
    return __builtin_bit_cast(u32x2, r);
}

// eight consecutive keys (two transposing reads, four rows apart) of this lane's column
__device__ __forceinline__ bf16x8 frag_tr(const uint16_t* p, int row_stride) {
    u32x2 a = lds_tr(p), b = lds_tr(p + 4 * row_stride);
    u32x4 r = {a.x, a.y, b.x, b.y};
    return __builtin_bit_cast(bf16x8, r);
}

__device__ __forceinline__ u32x2 pack4(const f32x4& x) {
    typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
    bf16x4 r;
#pragma unroll
    for (int e = 0; e < 4; ++e) r[e] = (__bf16)x[e];
    return __builtin_bit_cast(u32x2, r);
}

__device__ __forceinline__ f32x4 mfma16(bf16x8 a, bf16x8 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

// One score tile: P^T[16JQ.., 16IQ..] = K rows x Q rows, masked by gamma^(i-j), to LDS P[i][j].
template <int D, int JQ, int IQ>
__device__ __forceinline__ void score_tile(const uint16_t* k_row, const uint16_t* q_row, uint16_t* p_wr,
                                           const f32x4 (&wgt)[4]) {
    constexpr int RSQ = CoopSmem<D>::RSQ, RSP = CoopSmem<D>::RSP;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < D / 32; ++s)
        acc = mfma16(frag16(k_row + 16 * JQ * RSQ + 32 * s), frag16(q_row + 16 * IQ * RSQ + 32 * s), acc);
    acc *= wgt[IQ - JQ];
    *reinterpret_cast<u32x2*>(p_wr + 16 * IQ * RSP + 16 * JQ) = pack4(acc);
}

}  // namespace coop

// kOut = true : full walk (outputs + state).   kOut = false : state only (segment pre-pass).
template <int D, bool kOut>
__global__ __launch_bounds__(512) void fwd_bf16_coop_kernel(FwdParams p, int ngroups, int map_mode) {
    using namespace coop;
    constexpr int NT = 512;       // threads: eight waves
    constexpr int SL = D / 32;    // column slices (workgroups) per sequence segment
    constexpr int NS = D / 32;    // contraction steps over the key dimension
    constexpr int TPW = D / 64;   // state tiles (16 key rows x 16 columns) per wave
    constexpr int PR = D / 8;     // 16-byte pieces per Q/K row
    constexpr int QPT = D / 64;   // Q (and K) pieces per thread per chunk
    constexpr int RPP = NT / PR;  // rows covered by one piece index
    constexpr int RSQ = CoopSmem<D>::RSQ, RSV = CoopSmem<D>::RSV, RSP = CoopSmem<D>::RSP, RST = CoopSmem<D>::RST;
    __shared__ __attribute__((aligned(16))) CoopSmem<D> sm;

    // Block -> (sequence segment, column slice).  Consecutive block ids go round-robin over
    // the 8 XCDs; the SL slices of one segment take ids that are equal modulo 8, so they share
    // one L2 (map_mode 1 numbers them consecutively instead; measurement only).
    const int gx = blockIdx.x & 7, rest = blockIdx.x >> 3;
    int slice = rest % SL, group = (rest / SL) * 8 + gx;
    if (map_mode == 1) { slice = blockIdx.x % SL; group = blockIdx.x / SL; }
    if (group >= ngroups) return;
    const int nseg_launch = kOut ? p.nseg : p.nseg - 1;
    const int bh = group / nseg_launch, seg = group % nseg_launch;
    const int h = bh % p.H;

    const int tid = threadIdx.x;
    const int w = tid >> 6, l = tid & 63, r16 = l & 15, q4 = l >> 4;
    const int c0 = 32 * slice;
    const int o_ch = w & 1, o_iq = w >> 1;  // the output tile of this wave

    const int tok_begin = seg * p.seg_chunks * kChunk;
    const int tok_end = (seg == p.nseg - 1) ? p.N : tok_begin + p.seg_chunks * kChunk;
    const int nchunks = (tok_end - tok_begin + kChunk - 1) / kChunk;

    const size_t seq_off = (size_t)bh * p.N * D;
    const uint16_t* qg = reinterpret_cast<const uint16_t*>(p.q) + seq_off;
    const uint16_t* kg = reinterpret_cast<const uint16_t*>(p.k) + seq_off;
    const uint16_t* vg = reinterpret_cast<const uint16_t*>(p.v) + seq_off;
    float* og = p.out + seq_off;

    {
        const double gd = (double)p.gamma[h];
        for (int n = tid; n <= kChunk; n += NT) sm.pw[n] = (float)pow_int(gd, n);
        if (kOut) {  // P above the diagonal is read by G2 as part of 32-key steps and must stay zero
            u32x4 z = {0u, 0u, 0u, 0u};
            for (int n = tid; n < kChunk * RSP / 8; n += NT) reinterpret_cast<u32x4*>(sm.p)[n] = z;
        }
    }

    // ---- state tiles of this wave: tile k covers key rows 16 dkb(k) .. +15 and columns 16 ch(k) .. +15
    // of the slice; S[k][r] = S[dk = 16 dkb + 4 q4 + r][c = c0 + 16 ch + r16].
    auto tile_dkb = [&](int k) { return (w * TPW + k) >> 1; };
    auto tile_ch = [&](int k) { return (w * TPW + k) & 1; };
    f32x4 S[TPW];
    {
        const float* src = nullptr;
        if (kOut) {
            if (seg == 0) src = p.state_in ? p.state_in + (size_t)bh * D * D : nullptr;
            else src = p.seg_state + ((size_t)bh * (p.nseg - 1) + (seg - 1)) * D * D;
        }
#pragma unroll
        for (int k = 0; k < TPW; ++k)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                int dk = 16 * tile_dkb(k) + 4 * q4 + r;
                S[k][r] = src ? src[dk * D + c0 + 16 * tile_ch(k) + r16] : 0.0f;
            }
    }
    // S^T[c][dk] in LDS, 4 consecutive dk per lane and tile
    int st_wr_off[TPW], k_tr_off[TPW], vs_tr_off[TPW];
#pragma unroll
    for (int k = 0; k < TPW; ++k) {
        st_wr_off[k] = (16 * tile_ch(k) + r16) * RST + 16 * tile_dkb(k) + 4 * q4;
        k_tr_off[k] = (8 * q4 + (r16 >> 2)) * RSQ + 16 * tile_dkb(k) + 4 * (r16 & 3);
        vs_tr_off[k] = (8 * q4 + (r16 >> 2)) * RSV + 16 * tile_ch(k) + 4 * (r16 & 3);
    }
    auto publish_state = [&]() {
#pragma unroll
        for (int k = 0; k < TPW; ++k) *reinterpret_cast<u32x2*>(&sm.st[st_wr_off[k]]) = pack4(S[k]);
    };
    if (kOut) publish_state();

    // ---- staging: thread -> pieces.  Q, K: QPT pieces of 16 bytes; V slice: one piece, fetched
    // by both halves of the workgroup (so that every thread issues the same loads) and written
    // to LDS by the first half.
    const int qk_row = tid / PR, qk_cc = tid % PR;  // piece r is RPP rows further down
    const int v_row = (tid & 255) >> 2, v_cc = tid & 3;
    const int qk_loff = qk_row * RSQ + qk_cc * 8;
    const int v_loff = v_row * RSV + v_cc * 8;

    // Register ring of kStages chunks: chunk c travels in stage c % kStages from the moment its
    // loads are issued (kStages chunks ahead of its use) until it is written to LDS.
    struct Stage {
        u32x4 q[QPT], k[QPT], v;
    };
    constexpr int kStages = 3;
    Stage stg[kStages];
    // Loads are unconditional (rows above a ragged chunk's first token re-read that token and
    // are zeroed when the stage is written to LDS), so that the wait for one stage can leave
    // the loads of the younger stages in flight.
    auto prefetch = [&](Stage& st, int tok0) {
        const int shift = max(0, tok0 + kChunk - tok_end);  // rows [0, shift) of the tile hold no token
        const size_t base = (size_t)(tok0 - shift) * D;     // wave-uniform
        const uint16_t* qc = qg + base;
        const uint16_t* kc = kg + base;
        const uint16_t* vc = vg + base;
#pragma unroll
        for (int r = 0; r < QPT; ++r) {
            const int row = max(qk_row + r * RPP, shift);
            const unsigned off = (unsigned)(row * D + qk_cc * 8);
            if (kOut) st.q[r] = *reinterpret_cast<const u32x4*>(qc + off);
            st.k[r] = *reinterpret_cast<const u32x4*>(kc + off);
        }
        st.v = *reinterpret_cast<const u32x4*>(vc + (unsigned)(max(v_row, shift) * D + c0 + v_cc * 8));
    };

    __syncthreads();  // tables, zeroed P, S^T visible

    const float v_scale = sm.pw[kChunk - 1 - v_row];  // gamma^(63-j) for this thread's V row
    auto store_tiles = [&](Stage& st, int buf, int tok0) {
        const int shift = max(0, tok0 + kChunk - tok_end);
        if (shift) {  // ragged last chunk: zero the rows that hold no token
            const u32x4 z = {0u, 0u, 0u, 0u};
#pragma unroll
            for (int r = 0; r < QPT; ++r)
                if (qk_row + r * RPP < shift) {
                    if (kOut) st.q[r] = z;
                    st.k[r] = z;
                }
            if (v_row < shift) st.v = z;
        }
#pragma unroll
        for (int r = 0; r < QPT; ++r) {
            if (kOut) *reinterpret_cast<u32x4*>(&sm.q[buf][qk_loff + r * RPP * RSQ]) = st.q[r];
            *reinterpret_cast<u32x4*>(&sm.k[buf][qk_loff + r * RPP * RSQ]) = st.k[r];
        }
        if (tid < 256) {
            if (kOut) *reinterpret_cast<u32x4*>(&sm.v[buf][v_loff]) = st.v;
            typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
            u32x4 sc;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                bf16x2 pr;
                pr[0] = (__bf16)(__uint_as_float(st.v[e] << 16) * v_scale);
                pr[1] = (__bf16)(__uint_as_float(st.v[e] & 0xffff0000u) * v_scale);
                sc[e] = __builtin_bit_cast(uint32_t, pr);
            }
            *reinterpret_cast<u32x4*>(&sm.vs[buf][v_loff]) = sc;
        }
    };

    // ---- per-lane constants
    f32x4 wgt[4];  // wgt[diff][r] = gamma^(16 diff + r16 - 4 q4 - r), zero above the diagonal
    if (kOut) {
#pragma unroll
        for (int diff = 0; diff < 4; ++diff)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                int n = 16 * diff + r16 - 4 * q4 - r;
                wgt[diff][r] = (n >= 0) ? sm.pw[max(n, 0)] : 0.0f;
            }
    }
    const float lam_full = sm.pw[16 * o_iq + r16 + 1];  // gamma^(i+1) in a full chunk
    const float gl_full = sm.pw[kChunk];                // gamma^64
    const int row_off = r16 * RSQ + 8 * q4;             // 16-byte row fragments of Q, K
    const int tr_off_v = (8 * q4 + (r16 >> 2)) * RSV + 16 * o_ch + 4 * (r16 & 3);
    const uint16_t* st_rd = &sm.st[(16 * o_ch + r16) * RST + 8 * q4];  // + 32 s
    const uint16_t* p_rd = &sm.p[(16 * o_iq + r16) * RSP + 8 * q4];    // + 32 u
    uint16_t* p_wr = &sm.p[r16 * RSP + 4 * q4];                        // + 16 IQ RSP + 16 JQ

    // ---- the work of one chunk.  kRagged = false: a full chunk inside the steady-state loop,
    // where every global load and store is issued unconditionally, so that the wait for the
    // oldest register stage leaves the younger stages in flight; kRagged = true: the last,
    // partial chunk (rows [0, shift) of the tile hold no token and are not stored).
    auto chunk_body = [&](auto ragged_tag, int t, Stage& nxt) {
        constexpr bool kRagged = decltype(ragged_tag)::value;
        const int buf = t & 1;
        const int tok0 = tok_begin + t * kChunk;
        const int Lc = kRagged ? tok_end - tok0 : kChunk;
        const int shift = kChunk - Lc;

        if (!kRagged) {
            // chunk t+1 from its register stage into the other buffer (free since the barrier that
            // ended chunk t-1); the stage is refilled with chunk t+1+kStages.  Past the end the
            // last chunk is fetched again and never used.
            store_tiles(nxt, buf ^ 1, tok_begin + min(t + 1, nchunks - 1) * kChunk);
            prefetch(nxt, tok_begin + min(t + 1 + kStages, nchunks - 1) * kChunk);
        }

        const uint16_t* q_row = &sm.q[buf][row_off];
        const uint16_t* k_row = &sm.k[buf][row_off];

        f32x4 o;
        if (kOut) {
            // G1: ten score tiles (jq <= iq) dealt over the waves
            switch (w) {
                case 0: score_tile<D, 0, 0>(k_row, q_row, p_wr, wgt); score_tile<D, 0, 3>(k_row, q_row, p_wr, wgt); break;
                case 1: score_tile<D, 1, 1>(k_row, q_row, p_wr, wgt); score_tile<D, 1, 3>(k_row, q_row, p_wr, wgt); break;
                case 2: score_tile<D, 0, 1>(k_row, q_row, p_wr, wgt); break;
                case 3: score_tile<D, 2, 2>(k_row, q_row, p_wr, wgt); break;
                case 4: score_tile<D, 0, 2>(k_row, q_row, p_wr, wgt); break;
                case 5: score_tile<D, 1, 2>(k_row, q_row, p_wr, wgt); break;
                case 6: score_tile<D, 2, 3>(k_row, q_row, p_wr, wgt); break;
                default: score_tile<D, 3, 3>(k_row, q_row, p_wr, wgt); break;
            }

            // G3: O^T tile (o_ch, o_iq) = S^T Q^T, scaled by gamma^(i+1)
            const uint16_t* q_own = q_row + 16 * o_iq * RSQ;
            o = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s = 0; s < NS; ++s) o = mfma16(frag16(st_rd + 32 * s), frag16(q_own + 32 * s), o);
            o *= kRagged ? sm.pw[max(16 * o_iq + r16 + 1 - shift, 0)] : lam_full;

            __syncthreads();  // P visible; every wave is done reading S^T

            // G2: O^T += V^T P^T over the keys up to this row block, 32 keys per step
            const uint16_t* v_tr = &sm.v[buf][tr_off_v];
            const int nu = (o_iq >> 1) + 1;
            for (int u = 0; u < nu; ++u) o = mfma16(frag_tr(v_tr + 32 * u * RSV, RSV), frag16(p_rd + 32 * u), o);

            // store: lane = token 16 o_iq + r16, registers = columns c0 + 16 o_ch + 4 q4 + (0..3)
            const int i = 16 * o_iq + r16;
            if (!kRagged || i >= shift) {
                float* oc = og + (size_t)(tok0 - shift) * D;  // wave-uniform
                *reinterpret_cast<f32x4*>(oc + (unsigned)(i * D + c0 + 16 * o_ch + 4 * q4)) = o;
            }
        }

        // G4: S = gamma^L S + K^T (Gam V) for this wave's state tiles
        {
            const float gl = kRagged ? sm.pw[Lc] : gl_full;
#pragma unroll
            for (int k = 0; k < TPW; ++k) S[k] *= gl;
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                // with two tiles per wave both share the key rows (dkb) and differ in the column half
                const bf16x8 ka = frag_tr(&sm.k[buf][k_tr_off[0]] + 32 * u * RSQ, RSQ);
#pragma unroll
                for (int k = 0; k < TPW; ++k)
                    S[k] = mfma16(ka, frag_tr(&sm.vs[buf][vs_tr_off[k]] + 32 * u * RSV, RSV), S[k]);
            }
            if (kOut) publish_state();
        }
        __syncthreads();  // chunk t+1 tiles and S^T visible; P and this chunk's tiles free
    };

    // ---- prologue: chunks 0..kStages-1 in flight, chunk 0 into buffer 0, its stage refilled
    const int nfull = (tok_end - tok_begin) / kChunk;  // the steady-state loop walks the full chunks
#pragma unroll
    for (int c = 0; c < kStages; ++c) prefetch(stg[c], tok_begin + min(c, nchunks - 1) * kChunk);
    store_tiles(stg[0], 0, tok_begin);
    prefetch(stg[0], tok_begin + min(kStages, nchunks - 1) * kChunk);
    __syncthreads();

    for (int tb = 0; tb < nfull; tb += kStages) {
#pragma unroll
        for (int ss = 0; ss < kStages; ++ss) {
            const int t = tb + ss;
            if (t >= nfull) break;
            chunk_body(std::false_type{}, t, stg[(ss + 1) % kStages]);
        }
    }
    if (nfull < nchunks) chunk_body(std::true_type{}, nfull, stg[0]);

    // ---- hand the state on
    float* dst = nullptr;
    if (kOut) {
        if (seg == p.nseg - 1 && p.state_out) dst = p.state_out + (size_t)bh * D * D;
    } else {
        dst = p.seg_state + ((size_t)bh * (p.nseg - 1) + seg) * D * D;
    }
    if (dst) {
#pragma unroll
        for (int k = 0; k < TPW; ++k)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                int dk = 16 * tile_dkb(k) + 4 * q4 + r;
                dst[dk * D + c0 + 16 * tile_ch(k) + r16] = S[k][r];
            }
    }
}

namespace {
template <int D, bool kOut>
hipError_t launch_coop(const FwdParams& p, int BH, hipStream_t stream) {
    const int ngroups = BH * (kOut ? p.nseg : p.nseg - 1);
    if (ngroups <= 0) return hipSuccess;
    const int blocks = 8 * (D / 32) * ((ngroups + 7) / 8);
    static const int map_mode = [] { const char* e = getenv("LEET_ATTN_COOP_MAP"); return e ? atoi(e) : 0; }();
    hipLaunchKernelGGL((fwd_bf16_coop_kernel<D, kOut>), dim3(blocks), dim3(512), 0, stream, p, ngroups, map_mode);
    return hipGetLastError();
}
}  // namespace

hipError_t launch_fwd_bf16_coop_states(const FwdParams& p, int BH, int D, hipStream_t stream) {
    if (p.nseg <= 1) return hipSuccess;
    return D == 64 ? launch_coop<64, false>(p, BH, stream) : launch_coop<128, false>(p, BH, stream);
}

hipError_t launch_fwd_bf16_coop_walk(const FwdParams& p, int BH, int D, hipStream_t stream) {
    return D == 64 ? launch_coop<64, true>(p, BH, stream) : launch_coop<128, true>(p, BH, stream);
}

}  // namespace leet
