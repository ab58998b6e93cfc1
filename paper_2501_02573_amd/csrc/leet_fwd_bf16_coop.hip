// Column-split chunk-walk kernel for bf16 inputs (gfx950, v_mfma_f32_32x32x16_bf16).
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
// all of Q and K (the copies of one sequence are placed on one XCD so that all but one of
// the reads hit its L2) and its own 32 columns of V, and writes its 32 columns of O.
//
// Inside a workgroup the waves are specialised, one 32x32 output tile per task, and hand
// their products to one another through LDS in operand-register order:
//
//   waves 0..2   G1  score tile n: P^T = K rows x Q rows, decay mask, pack -> pfrag[n]
//                    (tiles (jt,it) = (0,0), (1,1), (0,1)); after that G4 for state tile n
//   waves 3, 4   G3  O^T[c][i] = S^T Q^T for row block it = w-3 (S^T from LDS st[c][dk]),
//                    rows scaled by gamma^(i+1); then G2: O^T += V^T P^T (V through
//                    transposing LDS reads, P from pfrag); store
//   wave  5      G4  for state tile 3 (d = 128 only)
//   waves 6, 7   staging only
//   G4  S[dk tile][c] = gamma^L S + K^T (Gam V), A = K through transposing reads, B = the
//       Gam-scaled V copy; the owner keeps its 32x32 fp32 tile in accumulators for the whole
//       walk and publishes it as bf16 S^T[c][dk] for the G3 waves of the next chunk.
//
// MFMA conventions (32x32x16): an A (B) operand holds, in lane l, row (column) l%32 and the
// eight contraction slots of group g = l/32; an accumulator holds, in lane l, column l%32
// and, in register r, row m(r, g) = 8(r/4) + 4g + r%4.  A contraction may use any assignment
// of indices to slots as long as A and B agree.  P^T accumulators (lane = query, registers =
// keys) are a B operand as they are; the V fragments are read in the matching key order.  G4
// assigns key-dimension index dk = 32t + pi(m) to accumulator row m (pi swaps bits 2 and 3 of
// m), so registers 8h..8h+7 hold eight consecutive dk and S^T is published 16 bytes at a time.
// Outputs are accumulated transposed (lane = token): Lam is one scalar per lane and a lane
// stores 16 contiguous bytes.
//
// Q, K, the V slice and its Gam-scaled copy are double-buffered in LDS: chunk t+1 is written
// from registers while chunk t is consumed, and a ring of register stages keeps the loads of
// three further chunks in flight; two workgroup barriers per chunk.  A ragged last chunk is
// right-aligned in the tile (rows 64-L.. hold the tokens), which keeps every decay weight
// chunk-independent.
#include <type_traits>

#include "leet_common.hpp"

namespace leet {

typedef short s16x4 __attribute__((ext_vector_type(4)));

template <int D>
struct CoopSmem {
    static constexpr int RSQ = D + 8;   // Q, K row stride (elements): 16-byte row reads spread over the banks
    static constexpr int RSV = 48;      // V slice: 32 columns + pad; 4 rows x 32 B of a transposing read stay apart
    static constexpr int RST = D + 8;   // S^T[c][dk]
    uint16_t q[2][kChunk * RSQ];
    uint16_t k[2][kChunk * RSQ];
    uint16_t v[2][kChunk * RSV];
    uint16_t vs[2][kChunk * RSV];       // Gam V: row j scaled by gamma^(63-j)
    u32x4 pfrag[3][2][64];              // masked P^T tiles as B operands: [tile][register half][lane]
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

// keys {k0..k0+3} and {k0+8..k0+11} of this lane's column: the order in which a 32x32
// accumulator holds its rows (k0 = 16 f + 4 g)
__device__ __forceinline__ bf16x8 frag_tr(const uint16_t* p, int row_stride) {
    u32x2 a = lds_tr(p), b = lds_tr(p + 8 * row_stride);
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

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ f32x16 zero16() {
    f32x16 z;
#pragma unroll
    for (int r = 0; r < 16; ++r) z[r] = 0.0f;
    return z;
}

}  // namespace coop

// kOut = true : full walk (outputs + state).   kOut = false : state only (segment pre-pass).
template <int D, bool kOut>
__global__ __launch_bounds__(512) void fwd_bf16_coop_kernel(FwdParams p, int ngroups, int map_mode) {
    using namespace coop;
    constexpr int NT = 512;       // threads: eight waves
    constexpr int SL = D / 32;    // column slices (workgroups) per sequence segment
    constexpr int DT = D / 32;    // 32-row state tiles of the slice
    constexpr int PR = D / 8;     // 16-byte pieces per Q/K row
    constexpr int QPT = D / 64;   // Q (and K) pieces per thread per chunk
    constexpr int RPP = NT / PR;  // rows covered by one piece index
    constexpr int RSQ = CoopSmem<D>::RSQ, RSV = CoopSmem<D>::RSV, RST = CoopSmem<D>::RST;
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
    const int w = tid >> 6, l = tid & 63, ln = l & 31, g = l >> 5;
    const int s16 = l & 15, half = (l >> 4) & 1;
    const int c0 = 32 * slice;

    // ---- roles
    const bool score_wave = kOut && w < 3;                       // G1 tile n = w
    const bool out_wave = kOut && (w == 3 || w == 4);            // output row block it = w - 3
    const int st_tile = (w < 3) ? w : (w == 5 ? 3 : -1);         // state tile owned (G4), if it exists
    const bool state_wave = st_tile >= 0 && st_tile < DT;
    const int it_own = w - 3;

    const int tok_begin = seg * p.seg_chunks * kChunk;
    const int tok_end = (seg == p.nseg - 1) ? p.N : tok_begin + p.seg_chunks * kChunk;
    const int nchunks = (tok_end - tok_begin + kChunk - 1) / kChunk;

    const size_t seq_off = (size_t)bh * p.N * D;
    const uint16_t* qg = reinterpret_cast<const uint16_t*>(p.q) + seq_off;
    const uint16_t* kg = reinterpret_cast<const uint16_t*>(p.k) + seq_off;
    const uint16_t* vg = reinterpret_cast<const uint16_t*>(p.v) + seq_off;
    float* og = static_cast<float*>(p.out) + seq_off;

    {
        const double gd = (double)p.gamma[h];
        for (int n = tid; n <= kChunk; n += NT) sm.pw[n] = (float)pow_int(gd, n);
    }

    // ---- state tile of this wave: S[r] = S[dk = 32 t + pi(m(r, g))][c = c0 + ln]
    auto dk_of = [&](int r) {
        // m = 8(r/4) + 4g + r%4 ; pi swaps the 4- and 8-bits: dk = 16(r/8) + 8g + 4((r/4)&1) + r%4
        return 32 * st_tile + 16 * (r >> 3) + 8 * g + 4 * ((r >> 2) & 1) + (r & 3);
    };
    f32x16 S = zero16();
    if (state_wave) {
        const float* src = nullptr;
        if (kOut) {
            if (seg == 0) src = p.state_in ? p.state_in + (size_t)bh * D * D : nullptr;
            else src = p.seg_state + ((size_t)bh * (p.nseg - 1) + (seg - 1)) * D * D;
        }
        if (src) {
#pragma unroll
            for (int r = 0; r < 16; ++r) S[r] = src[dk_of(r) * D + c0 + ln];
        }
    }
    // S^T[c][dk] in LDS: registers 8h..8h+7 are dk = 32 t + 16 h + 8 g + (0..7)
    u32x4* st_wr = reinterpret_cast<u32x4*>(&sm.st[ln * RST + 32 * max(st_tile, 0) + 8 * g]);  // + 2h (16 elements)
    auto publish_state = [&]() {
        st_wr[0] = __builtin_bit_cast(u32x4, pack_half(S, 0));
        st_wr[2] = __builtin_bit_cast(u32x4, pack_half(S, 1));
    };
    if (kOut && state_wave) publish_state();

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

    __syncthreads();  // tables, S^T visible

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
    // decay weights of the score tile this wave produces: i - j = 32 (it - jt) + ln - jr
    f32x16 wgt = zero16();
    if (score_wave) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            int n = ln - (8 * (r >> 2) + 4 * g + (r & 3));
            float diag = (n >= 0) ? sm.pw[max(n, 0)] : 0.0f;
            wgt[r] = (w == 2) ? sm.pw[32 + n] : diag;
        }
    }
    const float lam_full = sm.pw[min(32 * max(it_own, 0) + ln + 1, kChunk)];  // gamma^(i+1) in a full chunk
    const float gl_full = sm.pw[kChunk];                                       // gamma^64
    const int row_off = ln * RSQ + 8 * g;  // 16-byte row fragments of Q, K: + 32 tile RSQ + 16 s
    // transposing reads: lane supplies row 4g + s16/4 (+ 16 f, + 8 for the second half) and four columns
    const int tr_off_v = (4 * g + (s16 >> 2)) * RSV + 16 * half + 4 * (s16 & 3);
    const int tr_off_k = (4 * g + (s16 >> 2)) * RSQ + 32 * max(st_tile, 0) + 16 * half + 8 * (s16 & 1) + 4 * ((s16 >> 1) & 1);
    const uint16_t* st_rd = &sm.st[ln * RST + 8 * g];  // + 16 s

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

        // G4 math: S = gamma^L S + K^T (Gam V) for the tile this wave owns
        auto state_update = [&]() {
            const float gl = kRagged ? sm.pw[Lc] : gl_full;
#pragma unroll
            for (int r = 0; r < 16; ++r) S[r] *= gl;
            const uint16_t* k_tr = &sm.k[buf][tr_off_k];
            const uint16_t* vs_tr = &sm.vs[buf][tr_off_v];
#pragma unroll
            for (int f = 0; f < 4; ++f)
                S = mfma32(frag_tr(k_tr + 16 * f * RSQ, RSQ), frag_tr(vs_tr + 16 * f * RSV, RSV), S);
        };

        if (kOut) {
            f32x16 o = zero16();
            if (score_wave) {
                // G1: score tile n = w, (jt, it) = (0,0), (1,1), (0,1)
                const int jt = (w == 1) ? 1 : 0, it = (w == 0) ? 0 : 1;
                const uint16_t* ka = k_row + 32 * jt * RSQ;
                const uint16_t* qa = q_row + 32 * it * RSQ;
                f32x16 acc = zero16();
#pragma unroll
                for (int s = 0; s < D / 16; ++s) acc = mfma32(frag16(ka + 16 * s), frag16(qa + 16 * s), acc);
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[r] *= wgt[r];
                sm.pfrag[w][0][l] = __builtin_bit_cast(u32x4, pack_half(acc, 0));
                sm.pfrag[w][1][l] = __builtin_bit_cast(u32x4, pack_half(acc, 1));
            } else if (out_wave) {
                // G3: O^T = S^T Q^T for row block it_own, rows scaled by gamma^(i+1)
                const uint16_t* qa = q_row + 32 * it_own * RSQ;
#pragma unroll
                for (int s = 0; s < D / 16; ++s) o = mfma32(frag16(st_rd + 16 * s), frag16(qa + 16 * s), o);
                const float lam = kRagged ? sm.pw[max(32 * it_own + ln + 1 - shift, 0)] : lam_full;
#pragma unroll
                for (int r = 0; r < 16; ++r) o[r] *= lam;
            } else if (state_wave) {
                state_update();
            }

            __syncthreads();  // P visible; the output waves are done reading S^T

            if (score_wave) {
                if (state_wave) {
                    state_update();
                    publish_state();
                }
            } else if (out_wave) {
                // G2: O^T += V^T P^T over the score tiles of this row block
                const uint16_t* v_tr = &sm.v[buf][tr_off_v];
                if (it_own == 0) {
#pragma unroll
                    for (int hh = 0; hh < 2; ++hh)
                        o = mfma32(frag_tr(v_tr + 16 * hh * RSV, RSV), __builtin_bit_cast(bf16x8, sm.pfrag[0][hh][l]), o);
                } else {
#pragma unroll
                    for (int hh = 0; hh < 2; ++hh) {
                        o = mfma32(frag_tr(v_tr + 16 * hh * RSV, RSV), __builtin_bit_cast(bf16x8, sm.pfrag[2][hh][l]), o);
                        o = mfma32(frag_tr(v_tr + 16 * (2 + hh) * RSV, RSV), __builtin_bit_cast(bf16x8, sm.pfrag[1][hh][l]), o);
                    }
                }
                // store: lane = token 32 it + ln, registers 4q..4q+3 = columns c0 + 8q + 4g + (0..3)
                const int i = 32 * it_own + ln;
                if (!kRagged || i >= shift) {
                    float* oc = og + (size_t)(tok0 - shift) * D;  // wave-uniform
                    const unsigned ooff = (unsigned)(i * D + c0 + 4 * g);
#pragma unroll
                    for (int qd = 0; qd < 4; ++qd) {
                        f32x4 val = {o[4 * qd], o[4 * qd + 1], o[4 * qd + 2], o[4 * qd + 3]};
                        *reinterpret_cast<f32x4*>(oc + ooff + 8 * qd) = val;
                    }
                }
            } else if (state_wave) {
                publish_state();
            }
        } else {
            if (state_wave) state_update();
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
    if (dst && state_wave) {
#pragma unroll
        for (int r = 0; r < 16; ++r) dst[dk_of(r) * D + c0 + ln] = S[r];
    }
}

// Measurement switch: number the slices of a segment consecutively (spreading them over the
// XCDs) instead of placing them on one XCD.  Off by default.
bool g_coop_consecutive_ids = false;

namespace {
template <int D, bool kOut>
hipError_t launch_coop(const FwdParams& p, int BH, hipStream_t stream) {
    const int ngroups = BH * (kOut ? p.nseg : p.nseg - 1);
    if (ngroups <= 0) return hipSuccess;
    const int blocks = 8 * (D / 32) * ((ngroups + 7) / 8);
    const int map_mode = g_coop_consecutive_ids ? 1 : 0;
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
