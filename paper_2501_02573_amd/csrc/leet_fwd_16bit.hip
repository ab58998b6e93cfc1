// Chunk-walk kernel for 16-bit inputs, bf16 or fp16 (gfx950, v_mfma_f32_32x32x16_{bf16,f16},
// fp32 accumulate), with fp32 output or output in the input type, and with the decaying mask
// or, as a compile-time special case that drops all decay arithmetic, the 0/1 causal mask
// (gamma = 1, the plain causal linear attention of Section 2.2).
//
// One workgroup walks the 64-token chunks of one segment of one (batch, head)
// sequence in order (the loop of Alg. 2, Appendix B.2), carrying the D x DV state S
// in MFMA accumulators (D = width of the q and k rows, the paper's rank r; DV = width of
// the v and out rows; DV = D except for rank 128 with width 256).  With the decaying mask (Section 2.2, Eq. "BCMV"), chunk t of
// length L computes, using the row/column weight split of Alg. 4 (Appendix B.3):
//
//     O_t     = ((Q_t K_t^T) .* D) V_t + Lam (Q_t S_t)       D[i][j] = gamma^(i-j), i >= j
//     S_{t+1} = gamma^L S_t + (Gam K_t)^T V_t                Lam = diag(gamma^(i+1)), Gam = diag(gamma^(L-1-j))
//
// Work split: wave w owns value columns [32w, 32w+32): it keeps S[:, cols] (D x 32
// fp32) in accumulators for the whole walk and computes O_t[:, cols].  The 64 x 64
// score matrix has three non-zero 32 x 32 tiles; each is computed once per workgroup
// (tile n by wave n mod #waves), masked, packed to 16 bits and handed to the other waves
// through a small LDS buffer laid out in operand-register order.
//
// MFMA conventions (32x32x16): an A (B) operand register set holds, in lane l, row
// (column) l%32 and the eight contraction slots of group g = l/32; an accumulator
// holds, in lane l, column l%32 and, in register r, row m(r, g) = 8(r/4) + 4g + r%4.
// A contraction may use any assignment of indices to slots as long as A and B agree.
//
// Data flow per chunk; Q, K, V sit row-major in LDS and are never transposed in memory:
//   G1  P^T[j][i]  = sum_dk K[j][dk] Q[i][dk]        A = K rows, B = Q rows (16-byte LDS reads)
//       P^T       *= D^T                             per-lane weights, fixed for the kernel
//   G3  O^T[c][i]  = sum_dk S^T[c][dk] Q^T[dk][i]    A = S accumulators (packed to 16 bits), B = Q rows
//       O^T       *= gamma^(i+1)                     one scalar per lane, since lane = token
//   G2  O^T[c][i] += sum_j V^T[c][j] P^T[j][i]       A = V through transposing LDS reads
//                                                    (ds_read_b64_tr_b16), B = packed P^T
//   G4  S[dk][c]  += sum_j K^T[dk][j] (Gam V)[j][c]  A = K through transposing LDS reads,
//                                                    B = the V fragments of G2, scaled by Gam
// P^T accumulators (lane = query, registers = keys) are already a B operand, and S
// accumulators (lane = value column, registers = key rows) are already an A operand,
// so neither is ever re-laid out.  G4 assigns key-dimension index dk = 32t + pi(m) to
// accumulator row m of tile t, pi swapping bits 2 and 3 of m; then registers 8h..8h+7
// of a lane hold the eight consecutive dk = 32t + 16h + 8g + e that G3 contracts
// against one 16-byte Q fragment.
//
// A ragged last chunk (L < 64) is right-aligned in the tile: rows 64-L.. hold the
// tokens, rows above are zero.  The intra-chunk weights depend on i-j only and Gam on
// 63-j', so both stay valid; only Lam and gamma^L are taken from the table.
//
// Memory policy: chunk tiles are fetched one chunk ahead into registers (16-byte loads; with
// the nontemporal hint when the inputs exceed the last-level cache); O leaves through a
// wave-private LDS tile in whole row pieces with nontemporal stores, since nothing here reads
// it again and written normally it displaces the inputs from the caches.
#include "leet_common.hpp"

namespace leet {

typedef short s16x4 __attribute__((ext_vector_type(4)));

// D: rank (width of q and k rows, the paper's r); DV: width of v and out rows (the paper's d).
template <int D, int DV>
struct Bf16Smem {
    static constexpr int RSQ = D + 8;   // row strides (elements): 16-byte row reads of 32 rows spread over the banks
    static constexpr int RSK = D + 8;
    // V is only read through ds_read_b64_tr_b16 (4 rows x 32 B per 16 lanes).  Its tile doubles as
    // the output scratch (DV/32 waves x 32 rows x 36 floats), which fixes the padding at DV = 256.
    static constexpr int RSV = DV + (DV > 128 ? 32 : 16);
    uint16_t q[kChunk * RSQ];           // Q_t [i][dk]
    uint16_t k[kChunk * RSK];           // K_t [j][dk]
    uint16_t v[kChunk * RSV];           // V_t [j][c]
    u32x4 pfrag[3][2][64];              // masked P^T tiles as B operands: [tile][register half][lane]
    float pw[kChunk + 4];               // gamma^n, n = 0..64
    float gw[kChunk];                   // gamma^(63-j)
};

__device__ __forceinline__ u32x4 frag16(const uint16_t* p) { return *reinterpret_cast<const u32x4*>(p); }

// ds_read_b64_tr_b16: within each group of 16 lanes, lane i receives element i%4 of
// the 8-byte rows addressed by lanes i/4, 4+i/4, 8+i/4, 12+i/4 of the group.
__device__ __forceinline__ u32x2 lds_tr(const uint16_t* p) {
    s16x4 r = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (__attribute__((address_space(3))) s16x4*)(const_cast<uint16_t*>(p)));
    return __builtin_bit_cast(u32x2, r);
}

__device__ __forceinline__ u32x4 join(u32x2 a, u32x2 b) {
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

// eight 16-bit values times eight fp32 weights -> 16-bit
template <typename E>
__device__ __forceinline__ u32x4 scale8(u32x4 x, f32x4 w0, f32x4 w1) {
    u32x4 r;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const float wl = (e < 2) ? w0[2 * e] : w1[2 * e - 4];
        const float wh = (e < 2) ? w0[2 * e + 1] : w1[2 * e - 3];
        r[e] = E::pack2(E::lo(x[e]) * wl, E::hi(x[e]) * wh);
    }
    return r;
}

// Score tiles in production order: tile 0 = (jt 0, it 0), tile 1 = (jt 1, it 1), tile 2 = (jt 0, it 1).
__device__ __forceinline__ constexpr int tile_jt(int n) { return n == 1 ? 1 : 0; }
__device__ __forceinline__ constexpr int tile_it(int n) { return n == 0 ? 0 : 1; }

// kOut = true : full walk (outputs + state).   kOut = false : state only (segment
// pre-pass: the end state of a segment started from zero).
// E: input element type.  kOut16: O is stored in the input type instead of fp32.
// kDecay = false: every gamma is 1, so the tables, Lam, Gam and gamma^L all drop out.
// kStream: q, k, v are loaded with the nontemporal hint (inputs larger than the last-level cache).
template <int D, int DV, bool kOut, typename E, bool kOut16, bool kDecay, bool kStream>
__global__ __launch_bounds__(DV * 2, DV > 128 ? 1 : 2) void fwd_16bit_kernel(FwdParams p) {
    constexpr int NT = DV * 2;   // threads: one wave per 32 value columns
    constexpr int NW = DV / 32;  // waves
    constexpr int DT = D / 32;   // 32-row tiles of the key dimension
    constexpr int PR = D / 8;    // 16-byte pieces per q or k row
    constexpr int PRV = DV / 8;  // 16-byte pieces per v row
    constexpr int QP = kChunk * PR / NT;   // q (and k) pieces per thread per chunk
    constexpr int VP = kChunk * PRV / NT;  // v pieces per thread per chunk (= 4)
    constexpr int RSQ = Bf16Smem<D, DV>::RSQ, RSK = Bf16Smem<D, DV>::RSK, RSV = Bf16Smem<D, DV>::RSV;
    static_assert(kChunk * RSV * 2 >= NW * 32 * 36 * 4, "the V tile must hold the output scratch");
    __shared__ __attribute__((aligned(16))) Bf16Smem<D, DV> sm;

    const int tid = threadIdx.x;
    const int w = tid >> 6, l = tid & 63, ln = l & 31, g = l >> 5;
    const int nseg_launch = kOut ? p.nseg : p.nseg - 1;
    const int bh = blockIdx.x / nseg_launch;
    const int seg = blockIdx.x % nseg_launch;
    const int h = bh % p.H;

    const int tok_begin = seg * p.seg_chunks * kChunk;
    const int tok_end = (seg == p.nseg - 1) ? p.N : tok_begin + p.seg_chunks * kChunk;
    const int nchunks = (tok_end - tok_begin + kChunk - 1) / kChunk;

    const size_t seq_off = (size_t)bh * p.N * D, seq_off_v = (size_t)bh * p.N * DV;
    const uint16_t* qb = reinterpret_cast<const uint16_t*>(p.q) + seq_off;
    const uint16_t* kb = reinterpret_cast<const uint16_t*>(p.k) + seq_off;
    const uint16_t* vb = reinterpret_cast<const uint16_t*>(p.v) + seq_off_v;
    float* ob = static_cast<float*>(p.out) + seq_off_v;            // kOut16 = false
    uint16_t* ob16 = static_cast<uint16_t*>(p.out) + seq_off_v;    // kOut16 = true

    // decay tables, fp64 -> fp32 once per workgroup
    if (kDecay) {
        const double gd = (double)p.gamma[h];
        for (int n = tid; n <= kChunk; n += NT) {
            float x = (float)pow_int(gd, n);
            sm.pw[n] = x;
            if (n < kChunk) sm.gw[kChunk - 1 - n] = x;
        }
    }

    // state slice: S[t][r] = S[dk = 32t + pi(m(r, g))][c = 32w + ln]
    f32x16 S[DT];
    const int c_own = 32 * w + ln;
    auto dk_of = [&](int t, int r) {
        // m = 8(r/4) + 4g + r%4 ; pi swaps the 4- and 8-bits: dk = 16(r/8) + 8g + 4((r/4)&1) + r%4
        return 32 * t + 16 * (r >> 3) + 8 * g + 4 * ((r >> 2) & 1) + (r & 3);
    };
    {
        const float* src = nullptr;
        if (kOut) {
            if (seg == 0) src = p.state_in ? p.state_in + (size_t)bh * D * DV : nullptr;
            else src = p.seg_state + ((size_t)bh * p.state_slots + (seg * p.state_step - 1)) * D * DV;
        }
        if (src) {
#pragma unroll
            for (int t = 0; t < DT; ++t)
#pragma unroll
                for (int r = 0; r < 16; ++r) S[t][r] = src[dk_of(t, r) * DV + c_own];
        } else {
#pragma unroll
            for (int t = 0; t < DT; ++t)
#pragma unroll
                for (int r = 0; r < 16; ++r) S[t][r] = 0.0f;
        }
    }

    // ---- per-lane LDS bases; every fragment address below is one of these plus a constant
    const int s16 = l & 15, half = (l >> 4) & 1;
    const uint16_t* q_row = &sm.q[ln * RSQ + 8 * g];   // + 32*it*RSQ + 16*s
    const uint16_t* k_row = &sm.k[ln * RSK + 8 * g];   // + 32*jt*RSK + 16*s
    // transposing reads: lane supplies row 4g + s16/4 (+ 8*rd + 16*f) and four consecutive columns
    const uint16_t* v_tr = &sm.v[(4 * g + (s16 >> 2)) * RSV + 32 * w + 16 * half + 4 * (s16 & 3)];
    const uint16_t* k_tr = &sm.k[(4 * g + (s16 >> 2)) * RSK + 16 * half + 8 * (s16 & 1) + 4 * ((s16 >> 1) & 1)];

    __syncthreads();  // tables visible

    // ---- per-lane constants of the walk: decay weights of the score tiles this wave produces.
    // wgt[0]: a tile on the diagonal (i - j = ln - jr, zero above the diagonal);
    // wgt[1]: the tile below it (i - j = 32 + ln - jr).  With four waves each wave needs one set.
    constexpr bool kBothSets = NW < 3;
    f32x16 wgt[kBothSets ? 2 : 1];
    float lam_full[2];  // gamma^(i+1) for a full chunk
    if (kOut) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            int n = ln - (8 * (r >> 2) + 4 * g + (r & 3));
            float diag = (n >= 0) ? (kDecay ? sm.pw[max(n, 0)] : 1.0f) : 0.0f;
            float below = kDecay ? sm.pw[32 + n] : 1.0f;
            if (kBothSets) {
                wgt[0][r] = diag;
                wgt[kBothSets ? 1 : 0][r] = below;
            } else {
                wgt[0][r] = (w == 2) ? below : diag;
            }
        }
        lam_full[0] = kDecay ? sm.pw[ln + 1] : 1.0f;
        lam_full[1] = kDecay ? sm.pw[32 + ln + 1] : 1.0f;
    }

    u32x4 rq[QP], rk[QP], rv[VP];
    auto prefetch = [&](int tok0) {
        const int shift = max(0, tok0 + kChunk - tok_end);  // rows [0, shift) of the tile stay zero
        const u32x4 z = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int r = 0; r < QP; ++r) {
            int piece = r * NT + tid;
            int j = piece / PR, cc = piece % PR;
            bool ok = j >= shift;
            size_t off = (size_t)(tok0 - shift + j) * D + cc * 8;
            if (kStream) {  // inputs larger than the last-level cache: do not allocate there
                if (kOut) rq[r] = ok ? __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(qb + off)) : z;
                rk[r] = ok ? __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(kb + off)) : z;
            } else {
                if (kOut) rq[r] = ok ? *reinterpret_cast<const u32x4*>(qb + off) : z;
                rk[r] = ok ? *reinterpret_cast<const u32x4*>(kb + off) : z;
            }
        }
#pragma unroll
        for (int r = 0; r < VP; ++r) {
            int piece = r * NT + tid;
            int j = piece / PRV, cc = piece % PRV;
            bool ok = j >= shift;
            size_t off = (size_t)(tok0 - shift + j) * DV + cc * 8;
            if (kStream) rv[r] = ok ? __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(vb + off)) : z;
            else rv[r] = ok ? *reinterpret_cast<const u32x4*>(vb + off) : z;
        }
    };

    prefetch(tok_begin);

    for (int t = 0; t < nchunks; ++t) {
        const int tok0 = tok_begin + t * kChunk;
        const int Lc = min(kChunk, tok_end - tok0);
        const int shift = kChunk - Lc;

        if (t > 0) __syncthreads();  // everyone is done reading the previous chunk's tiles and P fragments
#pragma unroll
        for (int r = 0; r < QP; ++r) {
            int piece = r * NT + tid;
            int j = piece / PR, cc = piece % PR;
            if (kOut) *reinterpret_cast<u32x4*>(&sm.q[j * RSQ + cc * 8]) = rq[r];
            *reinterpret_cast<u32x4*>(&sm.k[j * RSK + cc * 8]) = rk[r];
        }
#pragma unroll
        for (int r = 0; r < VP; ++r) {
            int piece = r * NT + tid;
            int j = piece / PRV, cc = piece % PRV;
            *reinterpret_cast<u32x4*>(&sm.v[j * RSV + cc * 8]) = rv[r];
        }
        __syncthreads();
        if (t + 1 < nchunks) prefetch(tok0 + kChunk);  // in flight during the MFMA work below

        f32x16 o[2];
        if (kOut) {
            // G1 + mask for the score tiles this wave produces
#pragma unroll
            for (int n = 0; n < 3; ++n) {
                if (n % NW != w) continue;
                f32x16 acc;
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
#pragma unroll
                for (int s = 0; s < D / 16; ++s)
                    acc = E::mfma32(frag16(k_row + 32 * tile_jt(n) * RSK + 16 * s),
                                    frag16(q_row + 32 * tile_it(n) * RSQ + 16 * s), acc);
                if (kDecay || n != 2) {  // without decay the tile below the diagonal needs no weights
                    const f32x16& wt = wgt[(kBothSets && n == 2) ? 1 : 0];
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[r] *= wt[r];
                }
                sm.pfrag[n][0][l] = pack_half<E>(acc, 0);
                sm.pfrag[n][1][l] = pack_half<E>(acc, 1);
            }

            // G3: O^T = S^T Q^T, rows of O scaled by gamma^(i+1)
            float lam[2] = {lam_full[0], lam_full[1]};
            if (kDecay && shift) {
                lam[0] = sm.pw[max(ln + 1 - shift, 0)];
                lam[1] = sm.pw[max(32 + ln + 1 - shift, 0)];
            }
#pragma unroll
            for (int it = 0; it < 2; ++it)
#pragma unroll
                for (int r = 0; r < 16; ++r) o[it][r] = 0.0f;
#pragma unroll
            for (int s = 0; s < D / 16; ++s) {
                const u32x4 sa = pack_half<E>(S[s >> 1], s & 1);
#pragma unroll
                for (int it = 0; it < 2; ++it) o[it] = E::mfma32(sa, frag16(q_row + 32 * it * RSQ + 16 * s), o[it]);
            }
            if (kDecay) {
#pragma unroll
                for (int it = 0; it < 2; ++it)
#pragma unroll
                    for (int r = 0; r < 16; ++r) o[it][r] *= lam[it];
            }
        }

        // V fragments: vf[f], f = 2*jt + hh, holds keys 16f + {4g..4g+3, 8+4g..8+4g+3} of column c_own
        u32x4 vf[4];
#pragma unroll
        for (int f = 0; f < 4; ++f)
            vf[f] = join(lds_tr(v_tr + (16 * f) * RSV), lds_tr(v_tr + (16 * f + 8) * RSV));

        if (kOut) {
            __syncthreads();  // P fragments visible
            // G2: O^T += V^T P^T over the tiles (jt <= it)
#pragma unroll
            for (int n = 0; n < 3; ++n)
#pragma unroll
                for (int hh = 0; hh < 2; ++hh)
                    o[tile_it(n)] = E::mfma32(vf[2 * tile_jt(n) + hh], sm.pfrag[n][hh][l], o[tile_it(n)]);

            // store O^T: lane = token 32it + ln, registers 4q..4q+3 = columns 32w + 8q + 4g + (0..3)
            if (kOut16) {
                // 16-bit output: through the same wave-private LDS tile, packed, so that a store
                // instruction covers whole 64-byte row pieces: lane -> (row l/4, 16 bytes l%4).
                uint32_t* scr = reinterpret_cast<uint32_t*>(sm.v) + w * (32 * 36);
#pragma unroll
                for (int it = 0; it < 2; ++it) {
#pragma unroll
                    for (int qd = 0; qd < 4; ++qd) {
                        u32x2 val = {E::pack2(o[it][4 * qd], o[it][4 * qd + 1]), E::pack2(o[it][4 * qd + 2], o[it][4 * qd + 3])};
                        *reinterpret_cast<u32x2*>(scr + ln * 20 + 4 * qd + 2 * g) = val;
                    }
                    // both reads before the first store; a full chunk stores without per-row conditions
                    u32x4 val[2];
#pragma unroll
                    for (int m = 0; m < 2; ++m) val[m] = *reinterpret_cast<const u32x4*>(scr + (16 * m + (l >> 2)) * 20 + 4 * (l & 3));
                    uint16_t* orow = ob16 + (size_t)tok0 * DV + 32 * w + 8 * (l & 3);
                    if (shift == 0) {
#pragma unroll
                        for (int m = 0; m < 2; ++m)
                            __builtin_nontemporal_store(val[m], reinterpret_cast<u32x4*>(orow + (size_t)(32 * it + 16 * m + (l >> 2)) * DV));
                    } else {
#pragma unroll
                        for (int m = 0; m < 2; ++m) {
                            const int i = 32 * it + 16 * m + (l >> 2);
                            if (i >= shift) __builtin_nontemporal_store(val[m], reinterpret_cast<u32x4*>(orow + (size_t)(i - shift) * DV));
                        }
                    }
                }
            } else {
                // The output is written once and not read again by this library: nontemporal stores, so
                // that it does not displace the inputs from the caches (10 % on the walk).
                // Through a wave-private LDS tile (the V tile is dead: its fragments are in registers)
                // so that a store instruction covers whole 128-byte row pieces: lane -> (row l/8, 16 bytes l%8).
                float* scr = reinterpret_cast<float*>(sm.v) + w * (32 * 36);
#pragma unroll
                for (int it = 0; it < 2; ++it) {
#pragma unroll
                    for (int qd = 0; qd < 4; ++qd) {
                        f32x4 val = {o[it][4 * qd], o[it][4 * qd + 1], o[it][4 * qd + 2], o[it][4 * qd + 3]};
                        *reinterpret_cast<f32x4*>(scr + ln * 36 + 8 * qd + 4 * g) = val;
                    }
                    // All four reads before the first store (a read placed under its row's condition makes
                    // every store wait for its own LDS round trip); a full chunk, the common case, stores
                    // without per-row conditions.
                    f32x4 val[4];
#pragma unroll
                    for (int m = 0; m < 4; ++m) val[m] = *reinterpret_cast<const f32x4*>(scr + (8 * m + (l >> 3)) * 36 + 4 * (l & 7));
                    float* orow = ob + (size_t)tok0 * DV + 32 * w + 4 * (l & 7);
                    if (shift == 0) {
#pragma unroll
                        for (int m = 0; m < 4; ++m)
                            __builtin_nontemporal_store(val[m], reinterpret_cast<f32x4*>(orow + (size_t)(32 * it + 8 * m + (l >> 3)) * DV));
                    } else {
#pragma unroll
                        for (int m = 0; m < 4; ++m) {
                            const int i = 32 * it + 8 * m + (l >> 3);
                            if (i >= shift) __builtin_nontemporal_store(val[m], reinterpret_cast<f32x4*>(orow + (size_t)(i - shift) * DV));
                        }
                    }
                }
            }
        }

        // G4: S = gamma^L S + K^T (Gam V)
        {
            if (kDecay) {
                const float gl = sm.pw[Lc];
#pragma unroll
                for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                    for (int r = 0; r < 16; ++r) S[dt][r] *= gl;
            }
#pragma unroll
            for (int f = 0; f < 4; ++f) {
                u32x4 vs = vf[f];
                if (kDecay) {
                    const f32x4 w0 = *reinterpret_cast<const f32x4*>(&sm.gw[16 * f + 4 * g]);
                    const f32x4 w1 = *reinterpret_cast<const f32x4*>(&sm.gw[16 * f + 8 + 4 * g]);
                    vs = scale8<E>(vf[f], w0, w1);
                }
#pragma unroll
                for (int dt = 0; dt < DT; ++dt) {
                    u32x4 a = join(lds_tr(k_tr + (16 * f) * RSK + 32 * dt), lds_tr(k_tr + (16 * f + 8) * RSK + 32 * dt));
                    S[dt] = E::mfma32(a, vs, S[dt]);
                }
            }
        }
    }

    // ---- hand the state on
    float* dst = nullptr;
    if (kOut) {
        if (seg == p.nseg - 1 && p.state_out) dst = p.state_out + (size_t)bh * D * DV;
    } else {
        dst = p.seg_state + ((size_t)bh * p.state_slots + seg) * D * DV;
    }
    if (dst) {
#pragma unroll
        for (int t = 0; t < DT; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) dst[dk_of(t, r) * DV + c_own] = S[t][r];
    }
}

namespace {

template <int D, int DV, bool kOut, typename E, bool kOut16>
void launch_one(const FwdParams& p, int blocks, hipStream_t stream) {
    const dim3 grid(blocks), block(DV * 2);
    if (p.no_decay) {
        if (p.stream_loads) hipLaunchKernelGGL((fwd_16bit_kernel<D, DV, kOut, E, kOut16, false, true>), grid, block, 0, stream, p);
        else hipLaunchKernelGGL((fwd_16bit_kernel<D, DV, kOut, E, kOut16, false, false>), grid, block, 0, stream, p);
    } else {
        if (p.stream_loads) hipLaunchKernelGGL((fwd_16bit_kernel<D, DV, kOut, E, kOut16, true, true>), grid, block, 0, stream, p);
        else hipLaunchKernelGGL((fwd_16bit_kernel<D, DV, kOut, E, kOut16, true, false>), grid, block, 0, stream, p);
    }
}

template <int D, int DV, typename E>
void launch_elem(const FwdParams& p, int BH, bool walk, bool out16, hipStream_t stream) {
    if (!walk) launch_one<D, DV, false, E, false>(p, BH * (p.nseg - 1), stream);
    else if (out16) launch_one<D, DV, true, E, true>(p, BH * p.nseg, stream);
    else launch_one<D, DV, true, E, false>(p, BH * p.nseg, stream);
}

// (D, DV) is one of (64, 64), (128, 128), (128, 256); the host has checked it
void launch_any(const FwdParams& p, int BH, int D, int DV, bool f16, bool walk, bool out16, hipStream_t stream) {
    if (D == 64) {
        if (f16) launch_elem<64, 64, ElemF16>(p, BH, walk, out16, stream);
        else launch_elem<64, 64, ElemBf16>(p, BH, walk, out16, stream);
    } else if (DV == 128) {
        if (f16) launch_elem<128, 128, ElemF16>(p, BH, walk, out16, stream);
        else launch_elem<128, 128, ElemBf16>(p, BH, walk, out16, stream);
    } else {
        if (f16) launch_elem<128, 256, ElemF16>(p, BH, walk, out16, stream);
        else launch_elem<128, 256, ElemBf16>(p, BH, walk, out16, stream);
    }
}

}  // namespace

// D: width of q and k rows (rank); DV: width of v and out rows.  f16: IEEE binary16 inputs instead of bfloat16.
hipError_t launch_fwd_16bit_states(const FwdParams& p, int BH, int D, int DV, bool f16, hipStream_t stream) {
    if (p.nseg <= 1) return hipSuccess;
    launch_any(p, BH, D, DV, f16, false, false, stream);
    return hipGetLastError();
}

// out16: p.out receives the input element type instead of fp32.
hipError_t launch_fwd_16bit_walk(const FwdParams& p, int BH, int D, int DV, bool f16, bool out16, hipStream_t stream) {
    launch_any(p, BH, D, DV, f16, true, out16, stream);
    return hipGetLastError();
}

}  // namespace leet
