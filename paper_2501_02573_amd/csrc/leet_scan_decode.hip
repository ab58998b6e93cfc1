// Two small HBM-bound kernels: the scan over segment boundary states, and the
// single-token decode step.
#include "leet_common.hpp"

namespace leet {

// ---------------------------------------------------------------------------------
// Segment scan.  On entry slot s of seg_state holds the end state of segment s run
// from a zero state, T_s = sum_j gamma^(L-1-j) k_j^T v_j (L = segment length in
// tokens).  On exit slot s holds the true state entering segment s+1:
//     S_in(0) = state_in or 0 ;  S_in(s+1) = gamma^L S_in(s) + T_s
// (the block recurrence of Alg. 2 with the decay of Appendix C.1, over segments).
// Only every `step`-th boundary is written back (slots step-1, 2 step-1, ...): the pre-pass may
// run on segments `step` times finer than the walk's, which reads no other boundary.
// One thread per four state elements; the loop over segments is sequential.
// gamma == nullptr means gamma = 1 for every head (0/1 causal mask).
// state_copy (null, or [BH][D][DV]) receives state_in unchanged: the walk's first segments read the
// entering state from there, so that the caller's buffer is read only by this kernel, which has
// finished before any workgroup of the walk can write the leaving state to an aliased state_out.
// ---------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void seg_scan_kernel(float* seg_state, const float* state_in,
                                                       float* state_copy, const float* gamma, int H, int nseg,
                                                       int seg_tokens, int step, int DD4, size_t total4) {
    size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total4) return;
    int bh = (int)(idx / DD4);
    int e4 = (int)(idx % DD4);
    const float gl = gamma ? (float)pow_int((double)gamma[bh % H], seg_tokens) : 1.0f;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    if (state_in) {
        acc = reinterpret_cast<const f32x4*>(state_in)[idx];
        if (state_copy) reinterpret_cast<f32x4*>(state_copy)[idx] = acc;
    }
    f32x4* slot = reinterpret_cast<f32x4*>(seg_state) + (size_t)bh * (nseg - 1) * DD4 + e4;
    // eight slots at a time: their loads are independent and go out together
    constexpr int kBatch = 8;
    for (int s0 = 0; s0 < nseg - 1; s0 += kBatch) {
        f32x4 t[kBatch];
#pragma unroll
        for (int u = 0; u < kBatch; ++u)
            if (s0 + u < nseg - 1) t[u] = slot[(size_t)(s0 + u) * DD4];
#pragma unroll
        for (int u = 0; u < kBatch; ++u)
            if (s0 + u < nseg - 1) {
                acc = gl * acc + t[u];
                if ((s0 + u) % step == step - 1) slot[(size_t)(s0 + u) * DD4] = acc;
            }
    }
}

// D x DV: shape of one state (rank x value width)
hipError_t launch_seg_scan(float* seg_state, const float* state_in, float* state_copy, const float* gamma, int BH, int H,
                           int nseg, int seg_tokens, int step, int D, int DV, hipStream_t stream) {
    if (nseg <= 1) return hipSuccess;
    int DD4 = D * DV / 4;
    size_t total4 = (size_t)BH * DD4;
    unsigned blocks = (unsigned)((total4 + 255) / 256);
    hipLaunchKernelGGL(seg_scan_kernel, dim3(blocks), dim3(256), 0, stream, seg_state, state_in, state_copy, gamma, H,
                       nseg, seg_tokens, step, DD4, total4);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------
// A prefill over no tokens: the loop of Alg. 1 / Alg. 2 does not run, so the state leaves as it
// entered (zero when none is given).  One thread per four state elements.
// ---------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void state_pass_kernel(const float* state_in, float* state_out, size_t total4) {
    size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total4) return;
    f32x4 s = {0.f, 0.f, 0.f, 0.f};
    if (state_in) s = reinterpret_cast<const f32x4*>(state_in)[idx];
    reinterpret_cast<f32x4*>(state_out)[idx] = s;
}

hipError_t launch_state_pass(const float* state_in, float* state_out, int BH, int D, int DV, hipStream_t stream) {
    if (!state_out || state_out == state_in) return hipSuccess;
    size_t total4 = (size_t)BH * D * DV / 4;
    unsigned blocks = (unsigned)((total4 + 255) / 256);
    hipLaunchKernelGGL(state_pass_kernel, dim3(blocks), dim3(256), 0, stream, state_in, state_out, total4);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------
// Decode step (Alg. 1, Appendix B.1, with the discounted update of Appendix C.1):
//     S <- gamma S + k^T v ;  o = q S        per (batch, head), S is D x DV fp32
// (D = width of q and k, DV = width of v and o; D = DV except for rank 128 / width 256).
// One workgroup of 256 threads streams one state once: every thread issues all of
// its 16-byte loads up front (D*DV*4/256/16 of them), updates in registers, stores
// back to the same addresses and accumulates its share of o = q S; the partial sums
// are combined with wave shuffles and one pass through LDS.
// Thread t: columns 4*(t % (DV/4)) .. +3, rows (t / (DV/4)) + RP*m, RP = 1024/DV.
// ---------------------------------------------------------------------------------
// kElem: 0 = fp32, 1 = bf16, 2 = fp16 inputs.  gamma == nullptr means gamma = 1.
// kStreamStore: the updated state is stored with the nontemporal hint -- right when it will not
// be read again before it has left the last-level cache (states larger than that cache, or many
// layers' states taking turns), wrong when the next step finds it there.
template <int D, int DV, int kElem, bool kStreamStore>
__global__ __launch_bounds__(256) void decode_kernel(const void* q, const void* k, const void* v,
                                                     const float* gamma, float* state, float* out, int H) {
    constexpr int CP = DV / 4;       // threads per state row
    constexpr int RP = 256 / CP;     // rows per pass
    constexpr int NPASS = D / RP;    // passes (= 16-byte loads per thread)
    __shared__ float sq[D], sk[D], sv[DV];
    __shared__ f32x4 red[4][CP];

    const int tid = threadIdx.x;
    const int bh = blockIdx.x;
    const int c4 = tid % CP, r0 = tid / CP;
    f32x4* Sg = reinterpret_cast<f32x4*>(state + (size_t)bh * D * DV);

    f32x4 s[NPASS];
#pragma unroll
    for (int m = 0; m < NPASS; ++m) s[m] = Sg[(size_t)(r0 + RP * m) * CP + c4];

    auto elem = [&](const void* base, size_t off) -> float {
        if (kElem == 1) return ElemBf16::lo(reinterpret_cast<const uint16_t*>(base)[off]);
        if (kElem == 2) return ElemF16::lo(reinterpret_cast<const uint16_t*>(base)[off]);
        return reinterpret_cast<const float*>(base)[off];
    };
    if (tid < D) {
        sq[tid] = elem(q, (size_t)bh * D + tid);
        sk[tid] = elem(k, (size_t)bh * D + tid);
    }
    if (tid < DV) sv[tid] = elem(v, (size_t)bh * DV + tid);
    const float gm = gamma ? gamma[bh % H] : 1.0f;
    __syncthreads();

    const f32x4 vv = *reinterpret_cast<const f32x4*>(&sv[4 * c4]);
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int m = 0; m < NPASS; ++m) {
        const int row = r0 + RP * m;
        const float kr = sk[row], qr = sq[row];
        f32x4 x = s[m];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            x[e] = fmaf(gm, x[e], kr * vv[e]);
            acc[e] = fmaf(qr, x[e], acc[e]);
        }
        if (kStreamStore) __builtin_nontemporal_store(x, &Sg[(size_t)row * CP + c4]);
        else Sg[(size_t)row * CP + c4] = x;
    }

    // combine the row groups: inside a wave (lanes CP apart), then across the four waves
#pragma unroll
    for (int off = CP; off < 64; off <<= 1)
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[e] += __shfl_xor(acc[e], off, 64);
    const int wv = tid >> 6, ln = tid & 63;
    if (ln < CP) red[wv][ln] = acc;
    __syncthreads();
    if (tid < CP) {
        f32x4 r = red[0][tid] + red[1][tid] + red[2][tid] + red[3][tid];
        reinterpret_cast<f32x4*>(out + (size_t)bh * DV)[tid] = r;
    }
}

template <int D, int DV, bool kStreamStore>
static void launch_decode_s(const void* q, const void* k, const void* v, const float* gamma, float* state,
                            float* out, int BH, int H, int elem, hipStream_t stream) {
    dim3 grid(BH), block(256);
    if (elem == 0) hipLaunchKernelGGL((decode_kernel<D, DV, 0, kStreamStore>), grid, block, 0, stream, q, k, v, gamma, state, out, H);
    else if (elem == 1) hipLaunchKernelGGL((decode_kernel<D, DV, 1, kStreamStore>), grid, block, 0, stream, q, k, v, gamma, state, out, H);
    else hipLaunchKernelGGL((decode_kernel<D, DV, 2, kStreamStore>), grid, block, 0, stream, q, k, v, gamma, state, out, H);
}

template <int D, int DV>
static void launch_decode_d(const void* q, const void* k, const void* v, const float* gamma, float* state,
                            float* out, int BH, int H, int elem, bool stream_store, hipStream_t stream) {
    if (stream_store) launch_decode_s<D, DV, true>(q, k, v, gamma, state, out, BH, H, elem, stream);
    else launch_decode_s<D, DV, false>(q, k, v, gamma, state, out, BH, H, elem, stream);
}

// elem: 0 = fp32, 1 = bf16, 2 = fp16 inputs; (D, DV) one of (64, 64), (128, 128), (128, 256)
hipError_t launch_decode(const void* q, const void* k, const void* v, const float* gamma, float* state,
                         float* out, int BH, int H, int D, int DV, int elem, bool stream_store,
                         hipStream_t stream) {
    if (D == 64) launch_decode_d<64, 64>(q, k, v, gamma, state, out, BH, H, elem, stream_store, stream);
    else if (DV == 128) launch_decode_d<128, 128>(q, k, v, gamma, state, out, BH, H, elem, stream_store, stream);
    else launch_decode_d<128, 256>(q, k, v, gamma, state, out, BH, H, elem, stream_store, stream);
    return hipGetLastError();
}

}  // namespace leet
