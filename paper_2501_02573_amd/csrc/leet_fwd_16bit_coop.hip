// Column-split chunk-walk kernel for bf16 or fp16 inputs (gfx950, v_mfma_f32_32x32x16_bf16 / _f16),
// fp32 output or output in the input type.
//
// Same mathematics as the wide kernel in leet_fwd_16bit.hip -- Alg. 2 (Appendix B.2) with the
// decaying mask of Eq. "BCMV" (Section 2.2) and the weight split of Alg. 4 (Appendix B.3):
//
//     O_t     = ((Q_t K_t^T) .* D) V_t + Lam (Q_t S_t)       D[i][j] = gamma^(i-j), i >= j
//     S_{t+1} = gamma^L S_t + (Gam K_t)^T V_t
//
// but a different split of the work, made for few, long sequences.  Value columns are
// independent of one another (O[:, c] and S[:, c] need only V[:, c]), so a sequence is
// handled by DV/32 workgroups, one per 32-column slice, on DV/32 compute units; each reads
// all of Q and K (the copies of one sequence are placed on one XCD so that all but one of
// the reads hit its L2) and its own 32 columns of V, and writes its 32 columns of O.
//
// Inside a workgroup the waves are specialised and hand their products to one another through
// LDS in operand-register order.  What bounds an iteration is the LDS: every MFMA of a 32x32
// tile takes 2 KB of operands from it, so the roles are cut such that operands shared by two
// products are read once and stay in registers:
//
//   waves 0, 1   row block it = w of the chunk (32 tokens):
//                G1  the masked score tiles of the row block, P^T = K rows x Q rows: the diagonal
//                    tile (it, it) and, for it = 1, the tile (0, 1) below the diagonal
//                G3  O^T[c][i] = S^T Q^T (S^T from LDS st[c][dk]), rows scaled by gamma^(i+1)
//                G2  O^T += V^T P^T (V through transposing LDS reads, P^T straight from the G1
//                    accumulators: a P^T accumulator, lane = query, registers = keys, is a B operand
//                    as it is); the finished tile goes to LDS for the store wave.
//                The Q rows of a row block are used by this wave alone, so they never enter LDS:
//                the wave loads its own operand fragments from global memory into registers, one
//                chunk ahead, and uses them for all three products.
//   waves 2, 3   G4  S[dk tile][c] = gamma^L S + K^T (Gam V) for two of the four 32-row state tiles
//                    each (one of two at d = 64), A = K through transposing reads, B = the Gam-scaled
//                    V copy, read once for both tiles; the owner keeps its fp32 tiles in accumulators
//                    for the whole walk and publishes them in the input type as S^T[c][dk] for the
//                    row waves of the next chunk
//   waves 4, 5   store the finished O tile of row block w - 4 in whole row pieces (and nothing else:
//                    their stores queue behind the loaders' loads in the compute unit's one
//                    vector-memory pipeline)
//   waves 6, 7   loaders: the global loads of K and V and the LDS writes of their tiles
//
// A compute unit accepts only so many outstanding vector-memory requests, and a wave that
// issues one more stalls at that instruction until there is room; a wave that both loads and
// computes therefore spends the delivery time of its loads unable to compute.  Hence the
// loader waves: they sit in that stall (and in the wait for the oldest register stage) while
// the compute waves run, and the only thing that ties the two together is one workgroup
// barrier per chunk.  The chunk is software-pipelined over that barrier: in iteration t the row
// waves produce O(t), the state waves S(t+1), the store waves write chunk t-1 to memory, and
// the loaders write chunk t+1 to LDS and issue the loads of chunk t+3.  The K tile, S^T and the
// output tiles are double-buffered in LDS, the V slice and its scaled copy triple-buffered.
//
// MFMA conventions (32x32x16): an A (B) operand holds, in lane l, row (column) l%32 and the
// eight contraction slots of group g = l/32; an accumulator holds, in lane l, column l%32
// and, in register r, row m(r, g) = 8(r/4) + 4g + r%4.  A contraction may use any assignment
// of indices to slots as long as A and B agree.  P^T accumulators (lane = query, registers =
// keys) are a B operand as they are; the V fragments are read in the matching key order.  G4
// assigns key-dimension index dk = 32t + pi(m) to accumulator row m (pi swaps bits 2 and 3 of
// m), so registers 8h..8h+7 hold eight consecutive dk and S^T is published 16 bytes at a time.
// Outputs are accumulated transposed (lane = token): Lam is one scalar per lane and a lane
// stores 16 contiguous bytes.  A ragged last chunk is right-aligned in the tile (rows 64-L..
// hold the tokens), which keeps every decay weight chunk-independent.
#include <type_traits>

#include "leet_common.hpp"

namespace leet {

typedef short s16x4 __attribute__((ext_vector_type(4)));

template <int D>
struct CoopSmem {
    static constexpr int RSQ = D + 8;   // Q, K row stride (elements): 16-byte row reads spread over the banks
    // V slice, 32 columns, unpadded: the 4 rows x 32 B that 32 lanes of a transposing read touch
    // are then consecutive (4 x 16 banks).  The Gam-scaled copy is read four rows apart (G4), so its
    // rows are padded to 40 elements: rows 0, 4, 8, 12 start 16 banks apart.
    static constexpr int RSV = 32;
    static constexpr int RSVS = 40;
    static constexpr int RST = D + 8;   // S^T[c][dk]
    uint16_t k[2][kChunk * RSQ];
    uint16_t v[3][kChunk * RSV];
    uint16_t vs[3][kChunk * RSVS];      // Gam V: row j scaled by gamma^(63-j)
    uint16_t st[2][32 * RST];
    float obuf[2][2][32 * 36];          // finished O tiles on their way out: [buffer][row block][row][column], padded rows
    float pw[kChunk + 4];               // gamma^n, n = 0..64
};

namespace coop {

// MFMA operands travel as raw 128-bit registers (eight 16-bit elements)
__device__ __forceinline__ u32x4 frag16(const uint16_t* p) {
    return *reinterpret_cast<const u32x4*>(p);
}

// ds_read_b64_tr_b16: within each group of 16 lanes, lane i receives element i%4 of the
// 8-byte rows addressed by lanes i/4, 4+i/4, 8+i/4, 12+i/4 of the group.
__device__ __forceinline__ u32x2 lds_tr(const uint16_t* p) {
    s16x4 r = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (__attribute__((address_space(3))) s16x4*)(const_cast<uint16_t*>(p)));
    return __builtin_bit_cast(u32x2, r);
}

// Two transposing reads make one operand.  G2 pairs V with P^T accumulators and so reads keys
// {k0..k0+3} and {k0+8..k0+11} of this lane's column, the order in which a 32x32 accumulator
// holds its rows (k0 = 16 f + 4 g; second_off = 8 rows).  G4 takes both operands from such reads
// and may order the keys as it likes: it reads rows four apart (second_off = 32 rows).
__device__ __forceinline__ u32x4 frag_tr(const uint16_t* p, int second_off) {
    u32x2 a = lds_tr(p), b = lds_tr(p + second_off);
    u32x4 r = {a.x, a.y, b.x, b.y};
    return r;
}

// registers 8h .. 8h+7 of an accumulator tile -> 16-bit operand
template <typename E>
__device__ __forceinline__ u32x4 pack_half(const f32x16& acc, int h) {
    u32x4 r;
#pragma unroll
    for (int e = 0; e < 4; ++e) r[e] = E::pack2(acc[8 * h + 2 * e], acc[8 * h + 2 * e + 1]);
    return r;
}

__device__ __forceinline__ f32x16 zero16() {
    f32x16 z;
#pragma unroll
    for (int r = 0; r < 16; ++r) z[r] = 0.0f;
    return z;
}

}  // namespace coop

// kOut = true : full walk (outputs + state).   kOut = false : state only (segment pre-pass).
// E: ElemBf16 or ElemF16 (input type).  kOut16: outputs in the input type instead of fp32.
// Two loader waves with two register stages each: more of either measured no faster (four waves,
// three stages), the loads are bound by what one compute unit keeps in flight, not by issue.
constexpr int kCoopLoaderWaves = 2;
constexpr int kCoopStages = 2;
constexpr int kCoopThreads = 384 + 64 * kCoopLoaderWaves;

// D: width of q and k rows (rank); DV: width of v and out rows (DV / 32 slices per sequence).
template <int D, int DV, bool kOut, typename E, bool kOut16>
__global__ __launch_bounds__(kCoopThreads) void fwd_16bit_coop_kernel(FwdParams p, int ngroups) {
    using namespace coop;
    auto mfma32 = [](u32x4 a, u32x4 b, f32x16 c) { return E::mfma32(a, b, c); };
    constexpr int NT = kCoopThreads;            // two row waves, two state waves, two store waves and the loader waves
    constexpr int NL = 64 * kCoopLoaderWaves;   // loader threads (waves 6 and up)
    constexpr int NS = kCoopStages;             // register stages of the loaders
    constexpr int VPL = kChunk * 4 / NL;        // V pieces per loader thread per chunk
    constexpr int VRS = NL / 4;                 // rows between two V pieces of one loader thread
    constexpr int SL = DV / 32;    // column slices (workgroups) per sequence segment
    constexpr int DT = D / 32;     // 32-row state tiles of the slice
    constexpr int PR = D / 8;      // 16-byte pieces per Q/K row
    constexpr int QPL = kChunk * PR / NL;  // Q (and K) pieces per loader thread per chunk
    constexpr int RPL = NL / PR;   // rows between two pieces of one loader thread
    constexpr int RSQ = CoopSmem<D>::RSQ, RSV = CoopSmem<D>::RSV, RSVS = CoopSmem<D>::RSVS, RST = CoopSmem<D>::RST;
    __shared__ __attribute__((aligned(16))) CoopSmem<D> sm;

    // Block -> (sequence segment, column slice).  Consecutive block ids go round-robin over
    // the 8 XCDs; the SL slices of one segment take ids that are equal modulo 8, so they share
    // one L2 (measured on config 3 with FETCH_SIZE: 201.5 MB fetched per launch, the compulsory
    // Q + K + V, against 671 MB with the slices numbered consecutively).
    const int gx = blockIdx.x & 7, rest = blockIdx.x >> 3;
    const int slice = rest % SL, group = (rest / SL) * 8 + gx;
    if (group >= ngroups) return;
    const int nseg_launch = kOut ? p.nseg : p.nseg - 1;
    const int bh = group / nseg_launch, seg = group % nseg_launch;
    const int h = bh % p.H;

    const int tid = threadIdx.x;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform, so the role branches are scalar
    const int l = tid & 63, ln = l & 31, g = l >> 5;
    const int s16 = l & 15, half = (l >> 4) & 1;
    const int c0 = 32 * slice;

    // ---- roles
    // state tiles per state wave: the walk has two state waves (2, 3); the pre-pass, in which nothing
    // else computes, spreads the tiles over waves 0 .. DT-1, one each
    constexpr int TPW = kOut ? ((DT >= 2) ? DT / 2 : 1) : 1;
    const bool row_wave = kOut && w < 2;                         // scores, G3 and G2 of row block it_own = w
    const int it_own = w & 1;
    const int tw = kOut ? w - 2 : w;                             // state wave number
    const bool state_wave = tw >= 0 && tw * TPW < DT && (!kOut || w < 4);   // G4 for state tiles tw TPW .. tw TPW + TPW - 1
    const int tile0 = max(tw, 0) * TPW;
    const bool store_wave = kOut && (w == 4 || w == 5);          // writes the finished O tile of row block w - 4 to global memory
    const bool loader = w >= 6;
    const int lt = tid - (NT - NL);                              // loader thread index

    const int tok_begin = seg * p.seg_chunks * kChunk;
    const int tok_end = (seg == p.nseg - 1) ? p.N : tok_begin + p.seg_chunks * kChunk;
    const int n = (tok_end - tok_begin + kChunk - 1) / kChunk;   // chunks of this segment
    const int last_shift = n * kChunk - (tok_end - tok_begin);   // empty rows at the top of the last chunk's tile

    const size_t seq_off = (size_t)bh * p.N * D, seq_off_v = (size_t)bh * p.N * DV;
    const uint16_t* qg = reinterpret_cast<const uint16_t*>(p.q) + seq_off;
    const uint16_t* kg = reinterpret_cast<const uint16_t*>(p.k) + seq_off;
    const uint16_t* vg = reinterpret_cast<const uint16_t*>(p.v) + seq_off_v;
    float* og = static_cast<float*>(p.out) + seq_off_v;                     // fp32 output
    uint16_t* og16 = static_cast<uint16_t*>(p.out) + seq_off_v;             // output in the input type

    // ---- state tiles of this wave: S[u][r] = S[dk = 32 (tile0 + u) + pi(m(r, g))][c = c0 + ln]
    auto dk_of = [&](int u, int r) {
        // m = 8(r/4) + 4g + r%4 ; pi swaps the 4- and 8-bits: dk = 16(r/8) + 8g + 4((r/4)&1) + r%4
        return 32 * (tile0 + u) + 16 * (r >> 3) + 8 * g + 4 * ((r >> 2) & 1) + (r & 3);
    };
    f32x16 S[TPW];
#pragma unroll
    for (int u = 0; u < TPW; ++u) S[u] = zero16();
    if (state_wave) {
        const float* src = nullptr;
        if (kOut) {
            if (seg == 0) src = p.state_in ? p.state_in + (size_t)bh * D * DV : nullptr;
            else src = p.seg_state + ((size_t)bh * (p.nseg - 1) + (seg - 1)) * D * DV;
        }
        if (src) {
#pragma unroll
            for (int u = 0; u < TPW; ++u)
#pragma unroll
                for (int r = 0; r < 16; ++r) S[u][r] = src[dk_of(u, r) * DV + c0 + ln];
        }
    }
    // S^T[c][dk] in LDS: registers 8h..8h+7 of tile t are dk = 32 t + 16 h + 8 g + (0..7)
    const int st_wr_off = ln * RST + 32 * tile0 + 8 * g;  // + 32 u + 16 h
    auto publish_state = [&](int buf) {
#pragma unroll
        for (int u = 0; u < TPW; ++u) {
            *reinterpret_cast<u32x4*>(&sm.st[buf][st_wr_off + 32 * u]) = pack_half<E>(S[u], 0);
            *reinterpret_cast<u32x4*>(&sm.st[buf][st_wr_off + 32 * u + 16]) = pack_half<E>(S[u], 1);
        }
    };
    if (kOut && state_wave) publish_state(0);

    // ---- loaders: thread -> pieces.  Q, K: piece m is row m RPL + lt/PR, 16 bytes at column
    // 8 (lt%PR); V slice: piece m is row 32 m + lt/4, 16 bytes at column c0 + 8 (lt%4).
    const int qk_row = lt / PR, qk_cc = lt % PR;
    const int v_row = lt >> 2, v_cc = lt & 3;
    const int qk_loff = qk_row * RSQ + qk_cc * 8;
    const int v_loff = v_row * RSV + v_cc * 8, vs_loff = v_row * RSVS + v_cc * 8;

    // Two register stages: chunk c travels in stage c & 1 from the moment its loads are issued
    // (two chunks ahead of the iteration that writes it to LDS) until it is written.  (A third
    // stage measured no faster: the loaders are bound by the rate at which one compute unit
    // can pull data through its vector memory path, not by latency.)
    struct Stage {
        u32x4 k[QPL], v[VPL];
    };
    // Loads are unconditional (rows above a ragged chunk's first token re-read that token and
    // are zeroed when the stage is written to LDS; chunks past the end re-read the last one), so
    // that the wait for one stage can leave the loads of the other in flight.
    auto prefetch = [&](Stage& st, int c) {
        c = min(c, n - 1);
        const int shift = (c == n - 1) ? last_shift : 0;
        // Base = the chunk's first token (tile row `shift`), offsets count rows from there: every
        // address formed lies inside the sequence, also for a ragged first chunk (N < 64), whose
        // tile begins before token 0.
        const size_t tok0 = (size_t)(tok_begin + c * kChunk);  // wave-uniform
        const uint16_t* qc = qg + tok0 * D;
        const uint16_t* kc = kg + tok0 * D;
        const uint16_t* vc = vg + tok0 * DV;
#pragma unroll
        for (int m = 0; m < QPL; ++m) {
            const int row = max(qk_row + m * RPL - shift, 0);
            const unsigned off = (unsigned)(row * D + qk_cc * 8);
            st.k[m] = *reinterpret_cast<const u32x4*>(kc + off);
        }
#pragma unroll
        for (int m = 0; m < VPL; ++m)
            st.v[m] = *reinterpret_cast<const u32x4*>(vc + (unsigned)(max(v_row + VRS * m - shift, 0) * DV + c0 + v_cc * 8));
    };

    // The table of decay weights gamma^n and everything derived from it are filled in behind the
    // first workgroup barrier, which each role executes in its own branch below: the loaders put
    // the first chunks' loads in flight before they wait there, so that the arrival of gamma from
    // memory, the table and the first tile's way from memory overlap.
    float v_scale[VPL];  // gamma^(63-j) for this loader thread's V rows
#pragma unroll
    for (int m = 0; m < VPL; ++m) v_scale[m] = 0.0f;
    auto store_tiles = [&](Stage& st, int c) {
        const int shift = (c == n - 1) ? last_shift : 0;
        const int qb = c & 1, vb = c % 3;
        if (shift) {  // ragged last chunk: zero the rows that hold no token
            const u32x4 z = {0u, 0u, 0u, 0u};
#pragma unroll
            for (int m = 0; m < QPL; ++m)
                if (qk_row + m * RPL < shift) st.k[m] = z;
#pragma unroll
            for (int m = 0; m < VPL; ++m)
                if (v_row + VRS * m < shift) st.v[m] = z;
        }
#pragma unroll
        for (int m = 0; m < QPL; ++m) {
            *reinterpret_cast<u32x4*>(&sm.k[qb][qk_loff + m * RPL * RSQ]) = st.k[m];
        }
#pragma unroll
        for (int m = 0; m < VPL; ++m) {
            if (kOut) *reinterpret_cast<u32x4*>(&sm.v[vb][v_loff + VRS * m * RSV]) = st.v[m];
            u32x4 sc;
#pragma unroll
            for (int e = 0; e < 4; ++e)
                sc[e] = E::pack2(E::lo(st.v[m][e]) * v_scale[m], E::hi(st.v[m][e]) * v_scale[m]);
            *reinterpret_cast<u32x4*>(&sm.vs[vb][vs_loff + VRS * m * RSVS]) = sc;
        }
    };

    // ---- per-lane constants of the compute waves
    // decay weights of the two kinds of score tile, i - j = 32 (it - jt) + ln - jr: the diagonal
    // tiles (jt = it) and the one below the diagonal (jt = 0, it = 1; row wave 1 only)
    f32x16 wgt_d = zero16(), wgt_o = zero16();
    float lam_full = 0.0f;   // gamma^(i+1) in a full chunk
    float gl_full = 0.0f;    // gamma^64
    auto read_tables = [&]() {   // after the first barrier
        if (row_wave) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                int d = ln - (8 * (r >> 2) + 4 * g + (r & 3));
                wgt_d[r] = (d >= 0) ? sm.pw[max(d, 0)] : 0.0f;
                wgt_o[r] = sm.pw[32 + d];
            }
        }
        lam_full = sm.pw[min(32 * it_own + ln + 1, kChunk)];
        gl_full = sm.pw[kChunk];
    };
    const int row_off = ln * RSQ + 8 * g;  // 16-byte row fragments of Q, K: + 32 tile RSQ + 16 s
    // transposing reads: lane supplies row 4g + s16/4 (+ 16 f, + 8 for the second half) and four columns
    const int tr_off_v = (4 * g + (s16 >> 2)) * RSV + 16 * half + 4 * (s16 & 3);
    // G4 contracts keys f + 4u (u = 0..15) in its MFMA number f: one transposing read then touches
    // rows four apart, which the Q/K row stride (4 banks per row) spreads over all banks; with
    // consecutive rows the 64-byte pieces of eight rows would overlap four deep.
    const int tr_row4 = 16 * g + 4 * (s16 >> 2);
    const int tr_off_k = tr_row4 * RSQ + 32 * tile0 + 16 * half + 8 * (s16 & 1) + 4 * ((s16 >> 1) & 1);  // + 32 u
    const int tr_off_vs = tr_row4 * RSVS + 16 * half + 4 * (s16 & 3);
    const int st_rd_off = ln * RST + 8 * g;  // + 16 s

    // ---- iteration t, one body per role.  Each body is straight-line code that first issues every
    // LDS read the iteration needs and then runs its MFMAs back to back; operands that two products
    // share are read once and stay in registers (the Q rows of a row block serve its score tiles and
    // its S^T Q^T product; the Gam V fragments serve both state tiles of a state wave), and the
    // masked scores go from the accumulators straight into the next product as its B operand.

    // State waves, chunk t: S = gamma^L S + K^T (Gam V) for the tiles this wave owns (G4).
    auto state_tiles = [&](int t) {
        const int qb = t & 1;
        const int shift = (t == n - 1) ? last_shift : 0;
        u32x4 ak[TPW][4], bv[4];
        const uint16_t* k_tr = &sm.k[qb][tr_off_k];
        const uint16_t* vs_tr = &sm.vs[t % 3][tr_off_vs];
#pragma unroll
        for (int f = 0; f < 4; ++f) {
            bv[f] = frag_tr(vs_tr + f * RSVS, 32 * RSVS);
#pragma unroll
            for (int u = 0; u < TPW; ++u) ak[u][f] = frag_tr(k_tr + 32 * u + f * RSQ, 32 * RSQ);
        }
        const float gl = shift ? sm.pw[kChunk - shift] : gl_full;
#pragma unroll
        for (int u = 0; u < TPW; ++u) {
#pragma unroll
            for (int r = 0; r < 16; ++r) S[u][r] *= gl;
#pragma unroll
            for (int f = 0; f < 4; ++f) S[u] = mfma32(ak[u][f], bv[f], S[u]);
        }
        if (kOut) publish_state((t + 1) & 1);  // S^T(t+1) for the row waves
    };

    // Row waves, chunk t, row block it_own (compile-time kLower = it_own == 1):
    //   G1  P^T tiles = K rows x Q rows, decay mask: the diagonal tile (it, it) and, for the lower
    //       row block, the tile (0, 1) under the diagonal
    //   G3  O^T = S^T Q^T, rows scaled by gamma^(i+1)
    //   G2  O^T += V^T P^T over the keys of the tiles, then the tile goes to LDS for the store wave
    // Q rows of a row block are used by that block's row wave only, so they do not pass through LDS:
    // the wave loads its own B-operand fragments (lane = query row, 16 bytes at column 16 s + 8 g)
    // straight from global memory into registers, one chunk ahead.
    auto load_q = [&](u32x4 (&qn)[D / 16], int c, int it) {
        c = min(c, n - 1);
        const int shift = (c == n - 1) ? last_shift : 0;
        const uint16_t* qrow = qg + ((size_t)(tok_begin + c * kChunk) + max(32 * it + ln - shift, 0)) * D + 8 * g;
#pragma unroll
        for (int s = 0; s < D / 16; ++s) qn[s] = *reinterpret_cast<const u32x4*>(qrow + 16 * s);
    };
    auto row_block = [&](int t, auto lower, u32x4 (&qf)[D / 16], u32x4 (&qn)[D / 16]) {
        constexpr bool kLower = decltype(lower)::value;
        constexpr int IT = kLower ? 1 : 0;
        const int qb = t & 1;
        const int shift = (t == n - 1) ? last_shift : 0;
        load_q(qn, t + 1, IT);   // the next chunk's fragments
        if (shift && 32 * IT + ln < shift) {   // ragged last chunk: rows above its first token are zero
            const u32x4 z = {0u, 0u, 0u, 0u};
#pragma unroll
            for (int s = 0; s < D / 16; ++s) qf[s] = z;
        }
        u32x4 kd[D / 16], ko[D / 16], sf[D / 16], vt[4];
        const uint16_t* ka = &sm.k[qb][row_off];
        const uint16_t* st_rd = &sm.st[qb][st_rd_off];
        const uint16_t* v_tr = &sm.v[t % 3][tr_off_v];
        // The LDS operands are read in items of two to four LDS instructions, in the order in which the MFMAs
        // take them, and each item is issued kAhead items before it is used: the reads of the next
        // items are then in flight under the MFMAs of this one (the counter of outstanding LDS
        // operations holds 15, so everything cannot be issued up front, and reading an item just
        // before its MFMAs puts one LDS round trip in front of every pair of them).
        //   lower row block: NP items of K rows 0..31 for the tile under the diagonal, NQ items of
        //   K rows 32..63 for the diagonal tile, NQ items of S^T, two items of V^T
        //   upper row block: NP items of K rows 0..31 for the diagonal tile, NQ items of S^T, one of V^T
        constexpr int NP = D / 32, NQ = D / 64, kAhead = 3;
        constexpr int NM = kLower ? NP + 2 * NQ : NP + NQ;   // items with MFMAs of their own
        constexpr int NR = NM + (kLower ? 2 : 1);            // all items
        auto issue = [&](int i) {
            if (i >= NR) return;
            if (i < NP) {
#pragma unroll
                for (int s = 2 * i; s < 2 * i + 2; ++s) {
                    if (kLower) ko[s] = frag16(ka + 16 * s);
                    else kd[s] = frag16(ka + 16 * s);
                }
            } else if (kLower && i < NP + NQ) {
#pragma unroll
                for (int s = 4 * (i - NP); s < 4 * (i - NP) + 4; ++s) kd[s] = frag16(ka + 32 * RSQ + 16 * s);
            } else if (i < NM) {
#pragma unroll
                for (int s = 4 * (i - (NM - NQ)); s < 4 * (i - (NM - NQ)) + 4; ++s) sf[s] = frag16(st_rd + 16 * s);
            } else {
#pragma unroll
                for (int hh = 2 * (i - NM); hh < 2 * (i - NM) + 2; ++hh) vt[hh] = frag_tr(v_tr + 16 * hh * RSV, 8 * RSV);
            }
        };
        f32x16 po = zero16(), pd = zero16(), os = zero16(), o = zero16();
        u32x4 pfo[2], pfd[2];
#pragma unroll
        for (int i = 0; i < kAhead; ++i) issue(i);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < NM; ++i) {
            if (i < NP) {
#pragma unroll
                for (int s = 2 * i; s < 2 * i + 2; ++s) {
                    if (kLower) po = mfma32(ko[s], qf[s], po);
                    else pd = mfma32(kd[s], qf[s], pd);
                }
            } else if (kLower && i < NP + NQ) {
#pragma unroll
                for (int s = 4 * (i - NP); s < 4 * (i - NP) + 4; ++s) pd = mfma32(kd[s], qf[s], pd);
            } else {
#pragma unroll
                for (int s = 4 * (i - (NM - NQ)); s < 4 * (i - (NM - NQ)) + 4; ++s) os = mfma32(sf[s], qf[s], os);
            }
            issue(i + kAhead);
            // mask and pack a score tile once the MFMAs of the next product have been issued behind it
            if (kLower && i == NP + NQ - 1) {
#pragma unroll
                for (int r = 0; r < 16; ++r) po[r] *= wgt_o[r];
                pfo[0] = pack_half<E>(po, 0);
                pfo[1] = pack_half<E>(po, 1);
            }
            if (i == NM - 1) {
#pragma unroll
                for (int r = 0; r < 16; ++r) pd[r] *= wgt_d[r];
                pfd[0] = pack_half<E>(pd, 0);
                pfd[1] = pack_half<E>(pd, 1);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        // V^T P^T into an accumulator of its own, so that it does not wait for the scaling of S^T Q^T
        if (kLower) {
            o = mfma32(vt[0], pfo[0], o);
            o = mfma32(vt[1], pfo[1], o);
        }
        o = mfma32(vt[kLower ? 2 : 0], pfd[0], o);
        o = mfma32(vt[kLower ? 3 : 1], pfd[1], o);
        const float lam = shift ? sm.pw[max(32 * IT + ln + 1 - shift, 0)] : lam_full;
#pragma unroll
        for (int r = 0; r < 16; ++r) o[r] = __builtin_fmaf(os[r], lam, o[r]);
        // hand the tile to the store wave: lane = token 32 it + ln, registers 4q..4q+3 = columns 8q + 4g + (0..3)
        float* ot = &sm.obuf[qb][IT][ln * 36 + 4 * g];
#pragma unroll
        for (int qd = 0; qd < 4; ++qd) {
            f32x4 val = {o[4 * qd], o[4 * qd + 1], o[4 * qd + 2], o[4 * qd + 3]};
            *reinterpret_cast<f32x4*>(ot + 8 * qd) = val;
        }
    };

    // Store waves: row block rb = w - 4 of chunk t-1, finished in iteration t-1: whole row pieces
    // per lane group.  Nontemporal: the output is written once and must not displace Q and K, which
    // the sibling slices re-read, from L2.
    auto store_chunk = [&](int t) {
        const int c = t - 1, rb = w - 4;
        const int cshift = (c == n - 1) ? last_shift : 0;
        // offset of the chunk's first token (tile row cshift); rows are counted from there
        const size_t tile_off = (size_t)(tok_begin + c * kChunk) * DV + c0;
        // All LDS reads of the tile are issued before the first store (a read placed under its row's
        // condition would make every store wait for its own read: LDS round trips in a row);
        // a full chunk, the common case, stores without any per-row condition.
        if (!kOut16) {
            // 128-byte row pieces: lane -> (row l/8 of eight rows, 16 bytes l%8)
            float* oc = og + tile_off + 4 * (l & 7);
            const float* ot = &sm.obuf[c & 1][rb][(l >> 3) * 36 + 4 * (l & 7)];
            f32x4 val[4];
#pragma unroll
            for (int m = 0; m < 4; ++m) val[m] = *reinterpret_cast<const f32x4*>(ot + (8 * m) * 36);
            if (cshift == 0) {
#pragma unroll
                for (int m = 0; m < 4; ++m)   // row 32 rb + 8 m + l/8 of the 64-row chunk tile
                    __builtin_nontemporal_store(val[m], reinterpret_cast<f32x4*>(oc + (size_t)(32 * rb + 8 * m + (l >> 3)) * DV));
            } else {
#pragma unroll
                for (int m = 0; m < 4; ++m) {
                    const int row = 32 * rb + 8 * m + (l >> 3);
                    if (row >= cshift) __builtin_nontemporal_store(val[m], reinterpret_cast<f32x4*>(oc + (size_t)(row - cshift) * DV));
                }
            }
        } else {
            // 64-byte row pieces: lane -> (row l/4 of sixteen rows, eight columns l%4)
            uint16_t* oc = og16 + tile_off + 8 * (l & 3);
            const float* ot = &sm.obuf[c & 1][rb][(l >> 2) * 36 + 8 * (l & 3)];
            u32x4 val[2];
#pragma unroll
            for (int m = 0; m < 2; ++m) {
                const float* src = ot + (16 * m) * 36;
                const f32x4 a = *reinterpret_cast<const f32x4*>(src);
                const f32x4 b = *reinterpret_cast<const f32x4*>(src + 4);
                const u32x4 v8 = {E::pack2(a[0], a[1]), E::pack2(a[2], a[3]), E::pack2(b[0], b[1]), E::pack2(b[2], b[3])};
                val[m] = v8;
            }
            if (cshift == 0) {
#pragma unroll
                for (int m = 0; m < 2; ++m)   // row 32 rb + 16 m + l/4
                    __builtin_nontemporal_store(val[m], reinterpret_cast<u32x4*>(oc + (size_t)(32 * rb + 16 * m + (l >> 2)) * DV));
            } else {
#pragma unroll
                for (int m = 0; m < 2; ++m) {
                    const int row = 32 * rb + 16 * m + (l >> 2);
                    if (row >= cshift) __builtin_nontemporal_store(val[m], reinterpret_cast<u32x4*>(oc + (size_t)(row - cshift) * DV));
                }
            }
        }
    };

    // The loaders and the compute waves run separate loops (so that the register stages are live
    // in the loaders only) that execute the same number of workgroup barriers: one after the
    // prologue and one per iteration t = 0 .. t_end.
    const int t_end = kOut ? n : n - 1;  // the walk needs one more iteration to store the last chunk
    if (loader) {
        // prologue: chunks 0 .. NS-1 in flight, chunk 0 into its buffers, its stage refilled with chunk NS
        Stage stg[NS];
#pragma unroll
        for (int s = 0; s < NS; ++s) prefetch(stg[s], s);
        __syncthreads();  // tables, S^T(0) visible
#pragma unroll
        for (int m = 0; m < VPL; ++m) v_scale[m] = sm.pw[kChunk - 1 - min(max(v_row, 0) + VRS * m, kChunk - 1)];
        store_tiles(stg[0], 0);
        prefetch(stg[0], NS);
        __syncthreads();
        // iteration t (t = 0 .. n-2): chunk t+1 from its stage (number (t+1) % NS) into LDS, the
        // stage refilled with chunk t+1+NS.  The steady-state loop takes the stages in turn with
        // nothing conditional inside: the compiler counts outstanding loads along every path that
        // reaches a wait, and a path on which the other stages' loads had not been issued would
        // make it wait for all of them, which drains the prefetch once per chunk.
        auto step = [&](int t, Stage& nxt) {
            store_tiles(nxt, t + 1);
            prefetch(nxt, t + 1 + NS);
            __syncthreads();
        };
        int t = 0;
        for (; t + NS - 1 <= n - 2; t += NS) {
#pragma unroll
            for (int s = 0; s < NS; ++s) step(t + s, stg[(s + 1) % NS]);
        }
#pragma unroll
        for (int s = 0; s < NS - 1; ++s)
            if (t <= n - 2) {
                step(t, stg[(s + 1) % NS]);
                ++t;
            }
        for (; t <= t_end; ++t) __syncthreads();  // iterations that load nothing
    } else {
        const std::true_type yes;
        const std::false_type no;
        u32x4 qa[D / 16], qb2[D / 16];
        if (row_wave) load_q(qa, 0, it_own);   // in flight before the table's barrier, like the loaders' first loads
        {
            const double gd = p.no_decay ? 1.0 : (double)p.gamma[h];  // 0/1 causal mask: every weight is 1
            for (int i = tid; i <= kChunk; i += NT) sm.pw[i] = (float)pow_int(gd, i);   // threads 0 .. 64: waves 0 and 1
        }
        __syncthreads();  // tables, S^T(0) visible
        read_tables();
        __syncthreads();
        // every branch below executes one barrier per iteration t = 0 .. t_end
        if (row_wave) {
            // qa, qb2: the Q fragments of the chunk in progress and of the next one, in turn (qa holds
            // chunk 0, loaded before the first barrier)
            if (it_own == 0) {
                for (int t = 0; t <= t_end; t += 2) {
                    if (t < n) row_block(t, no, qa, qb2);
                    __syncthreads();  // chunk t+1 tiles, S^T(t+1), O(t) visible; everything read in this iteration is free
                    if (t + 1 <= t_end) {
                        if (t + 1 < n) row_block(t + 1, no, qb2, qa);
                        __syncthreads();
                    }
                }
            } else {
                for (int t = 0; t <= t_end; t += 2) {
                    if (t < n) row_block(t, yes, qa, qb2);
                    __syncthreads();
                    if (t + 1 <= t_end) {
                        if (t + 1 < n) row_block(t + 1, yes, qb2, qa);
                        __syncthreads();
                    }
                }
            }
        } else {
            // the state waves, the store waves of the walk, and waves with nothing to do in this launch
            for (int t = 0; t <= t_end; ++t) {
                if (state_wave && t < n) state_tiles(t);
                if (store_wave && t >= 1) store_chunk(t);
                __syncthreads();
            }
        }
    }

    // ---- hand the state on
    float* dst = nullptr;
    if (kOut) {
        if (seg == p.nseg - 1 && p.state_out) dst = p.state_out + (size_t)bh * D * DV;
    } else {
        dst = p.seg_state + ((size_t)bh * (p.nseg - 1) + seg) * D * DV;
    }
    if (dst && state_wave) {
#pragma unroll
        for (int u = 0; u < TPW; ++u)
#pragma unroll
            for (int r = 0; r < 16; ++r) dst[dk_of(u, r) * DV + c0 + ln] = S[u][r];
    }
}

namespace {
template <int D, int DV, bool kOut, typename E, bool kOut16>
hipError_t launch_coop(const FwdParams& p, int BH, hipStream_t stream) {
    const int ngroups = BH * (kOut ? p.nseg : p.nseg - 1);
    if (ngroups <= 0) return hipSuccess;
    const int blocks = 8 * (DV / 32) * ((ngroups + 7) / 8);
    hipLaunchKernelGGL((fwd_16bit_coop_kernel<D, DV, kOut, E, kOut16>), dim3(blocks), dim3(kCoopThreads), 0, stream, p, ngroups);
    return hipGetLastError();
}

template <bool kOut, typename E, bool kOut16>
hipError_t launch_coop_d(const FwdParams& p, int BH, int D, int DV, hipStream_t stream) {
    if (D == 64) return launch_coop<64, 64, kOut, E, kOut16>(p, BH, stream);
    if (DV == 128) return launch_coop<128, 128, kOut, E, kOut16>(p, BH, stream);
    return launch_coop<128, 256, kOut, E, kOut16>(p, BH, stream);
}
}  // namespace

// (D, DV) one of (64, 64), (128, 128), (128, 256); f16: fp16 instead of bf16 inputs; out16: output in the input type
hipError_t launch_fwd_16bit_coop_states(const FwdParams& p, int BH, int D, int DV, bool f16, hipStream_t stream) {
    if (p.nseg <= 1) return hipSuccess;
    return f16 ? launch_coop_d<false, ElemF16, false>(p, BH, D, DV, stream) : launch_coop_d<false, ElemBf16, false>(p, BH, D, DV, stream);
}

hipError_t launch_fwd_16bit_coop_walk(const FwdParams& p, int BH, int D, int DV, bool f16, bool out16, hipStream_t stream) {
    if (f16) return out16 ? launch_coop_d<true, ElemF16, true>(p, BH, D, DV, stream) : launch_coop_d<true, ElemF16, false>(p, BH, D, DV, stream);
    return out16 ? launch_coop_d<true, ElemBf16, true>(p, BH, D, DV, stream) : launch_coop_d<true, ElemBf16, false>(p, BH, D, DV, stream);
}

}  // namespace leet
