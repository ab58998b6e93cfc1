// C ABI of the library: argument validation, segment planning, workspace, launches.
// Every step of the computation runs in the HIP kernels; nothing here touches tensor data.
#include <atomic>
#include <math.h>
#include <mutex>
#include <stdlib.h>
#include <string.h>
#include <vector>

#include "../../include/leet_attn.h"
#include "../../include/leet_attn_bench.h"
#include "leet_common.hpp"

namespace leet {
hipError_t launch_fwd_16bit_states(const FwdParams& p, int BH, int D, int DV, bool f16, hipStream_t stream);
hipError_t launch_fwd_16bit_walk(const FwdParams& p, int BH, int D, int DV, bool f16, bool out16, hipStream_t stream);
hipError_t launch_state_pass(const float* state_in, float* state_out, int BH, int D, int DV, hipStream_t stream);
hipError_t launch_fwd_16bit_coop_states(const FwdParams& p, int BH, int D, int DV, bool f16, hipStream_t stream);
hipError_t launch_fwd_16bit_coop_walk(const FwdParams& p, int BH, int D, int DV, bool f16, bool out16, hipStream_t stream);
hipError_t launch_fwd_f32_states(const FwdParams& p, int BH, int D, hipStream_t stream);
hipError_t launch_fwd_f32_walk(const FwdParams& p, int BH, int D, hipStream_t stream);
hipError_t launch_seg_scan(float* seg_state, const float* state_in, float* state_copy, const float* gamma, int BH, int H,
                           int nseg, int seg_tokens, int step, int D, int DV, hipStream_t stream);
hipError_t launch_recurrent(const void* q, const void* k, const void* v, const float* gamma, float* out,
                            const float* state_in, float* state_out, int BH, int H, int N, int D, int DV,
                            int elem, hipStream_t stream);
hipError_t launch_fleet(const void* q, const void* k, const void* v, const float* gamma, float* out,
                        const float* state_in, float* state_out, int BH, int H, int N, int D, int DV,
                        int elem, hipStream_t stream);
hipError_t launch_decode(const void* q, const void* k, const void* v, const float* gamma, float* state,
                         float* out, int BH, int H, int D, int DV, int elem, bool stream_store,
                         hipStream_t stream);
}  // namespace leet

namespace {

using leet::kChunk;

// fp32: sequences are cut into segments so that about this many
// workgroups exist (one per compute unit of a 256-CU device measured best), but no segment is
// shorter than a minimum number of chunks: each extra segment costs one D x DV fp32 state written,
// scanned and re-read, and every segment but the last has its K and V read twice.  The fp32
// kernel is bound by MFMA latency per chunk, not by HBM, so it takes much shorter segments.
constexpr int kTargetWorkgroups = 256;
constexpr int kMinSegChunksF32 = 2;
constexpr int kMaxDevices = 64;
constexpr size_t kLastLevelCacheBytes = (size_t)256 << 20;  // MI355X Infinity Cache

// Process-wide defaults of the two tuning knobs, used by every entry point that does not take the
// choice as an argument (and by the _v3 ones when they are passed LEET_CHOICE_DEFAULT).
// Kernel choice for 16-bit prefill (bf16 and fp16; the name is historical): a leet_bf16_kernel value.
std::atomic<int> g_bf16_kernel{LEET_KERNEL_AUTO};

// Decode-state store policy: a leet_decode_store value.
std::atomic<int> g_decode_store{LEET_DECODE_STORE_AUTO};

// The state buffer of the previous decode call on each device (what AUTO's store policy looks at).
std::atomic<const void*> g_last_decode_state[kMaxDevices];

bool kernel_choice_ok(int c) { return c == LEET_KERNEL_WIDE || c == LEET_KERNEL_COLUMN_SPLIT || c == LEET_KERNEL_AUTO; }
bool decode_store_ok(int m) { return m == LEET_DECODE_STORE_AUTO || m == LEET_DECODE_STORE_CACHED || m == LEET_DECODE_STORE_STREAM; }

struct Plan {
    int nseg;
    int seg_chunks;
    int pre_split;  // the pre-pass and the scan run on segments this many times finer than the walk's
    size_t ws_bytes;
    bool coop;  // the column-split kernel runs this call
};

// The pre-pass is a pure read stream and runs faster with two workgroups per compute unit
// (config 4: 6.2 against 4.7 TB/s), the walk does not (more boundary states to carry); so the
// 16-bit wide path computes the segment states on half-segments and the walk takes every
// second boundary.  Same K and V bytes read, one more state per segment scanned.
int wide_pre_split(long BH, int nseg, int seg_chunks) {
    return (nseg > 1 && seg_chunks >= 16 && seg_chunks % 2 == 0 && BH * (nseg - 1) <= 256) ? 2 : 1;
}

// The fp32 pre-pass is bound by fp32 MFMA issue, so what counts is how evenly its workgroups fill
// the 256 compute units: it runs on segments `split` times finer than the walk's, with the split
// (1, 2, 4 or 8 parts of at least two chunks) that needs the fewest chunk-times -- rounds of 256
// workgroups x chunks per workgroup, a tenth less once two workgroups share a compute unit and
// overlap -- plus half a chunk-time per part for the longer scan (B4 H16 N4096 d128 in fp32: 192
// workgroups of 16 chunks take 93 us, 384 of 8 chunks 85 us, 768 of 4 chunks 73 us).
int f32_pre_split(long BH, int nseg, int seg_chunks) {
    if (nseg <= 1) return 1;
    const long units = BH * (nseg - 1);
    int best = 1;
    double best_cost = 0.0;
    for (int split = 1; split <= 8; split *= 2) {
        if (seg_chunks % split != 0 || (split > 1 && seg_chunks / split < 2)) break;
        const double cost = (double)((units * split + 255) / 256) * (seg_chunks / split) * (split > 1 ? 0.9 : 1.0) + 0.5 * split;
        if (split == 1 || cost < best_cost) { best = split; best_cost = cost; }
    }
    return best;
}

// Cost model of the 16-bit shapes, in microseconds, for one (kernel, segment
// count) pair.  Each kernel is priced as the smooth maximum (x^p + y^p)^(1/p) of its dependent
// chain (rounds of resident workgroups x chunks per segment x the per-chunk time of a lone
// workgroup) and of its HBM/last-level-cache transfer time; a call is the sum of its kernels plus
// a fixed cost per call.  The constants are a least-squares fit (5 % rms) to event-timed runs of
// both kernels at 1 to 64 segments over B*H in 1..768 and N in 256..65536 (each of the three shapes); the tabulated runs are
// kept with the profiles, and a host test checks the planner's picks against them.
struct CostModel {
    double wide_chunk_us, wide_pre_chunk_us;    // lone wide workgroup: walk and pre-pass per chunk
    double coop_chunk_us, coop_pre_chunk_us;    // column-split workgroups of one sequence, likewise
    double wide_bw_cached, wide_bw_streamed;    // bytes per us: inputs within / beyond the last-level cache
    double coop_bw_cached, coop_bw_streamed;
    double one_kernel_us, three_kernel_us;      // fixed cost of a call without / with pre-pass and scan
    double scan_state_us;                       // scan latency per segment state
    double wide_p, coop_p;                      // smooth-maximum exponents
    double wide_crowded;                        // transfer-time factor with more wide workgroups than CUs
    int wide_slots;                             // wide workgroups resident on the device
};
constexpr CostModel kCost128 = {2.718, 0.935, 0.776, 0.391, 8.0e6, 6.734e6, 7.699e6, 5.352e6,
                                3.62, 10.26, 0.341, 2.270, 2.0, 1.256, 512};
constexpr CostModel kCost64 = {1.839, 0.516, 0.546, 0.287, 7.540e6, 6.094e6, 8.0e6, 5.553e6,
                               3.01, 9.10, 0.351, 3.085, 2.567, 1.167, 1024};
// rank 128, value width 256: one wide workgroup per compute unit (512 threads)
constexpr CostModel kCost128x256 = {3.172, 1.643, 0.733, 0.427, 8.0e6, 6.706e6, 6.553e6, 4.692e6,
                                    4.32, 10.17, 0.426, 2.229, 2.0, 1.158, 256};
constexpr double kOneKernelFloorUs = 11.0;    // shortest call seen end to end, one and three kernels
constexpr double kThreeKernelFloorUs = 17.0;
constexpr int kCoopSlots = 256;               // one column-split workgroup per compute unit

double smooth_max(double a, double b, double p) { return pow(pow(a, p) + pow(b, p), 1.0 / p); }

// nseg is a segment count that make_plan has already rounded (nseg = ceil(nchunks / seg_chunks))
double predicted_us(bool coop, long BH, int N, int D, int DV, int nseg, int seg_chunks) {
    const CostModel& m = D == 64 ? kCost64 : DV == 128 ? kCost128 : kCost128x256;
    const double in_bytes = (double)BH * N * (2 * D + DV) * 2, out_bytes = (double)BH * N * DV * 4;
    // share of the inputs that no longer stays in the last-level cache: none up to 0.6 of its size
    // (the outputs pass through it too), all from 1.2
    const double spill = fmin(1.0, fmax(0.0, (in_bytes / (double)kLastLevelCacheBytes - 0.6) / 0.6));
    const double pre_bytes = (double)BH * N * (D + DV) * 2 * (nseg - 1) / nseg;  // K and V of all segments but the last
    double scan = nseg > 1 ? nseg * fmax(m.scan_state_us, (double)BH * D * DV * 8 / 5e6) : 0.0;
    if (coop) {
        const long per_seg = BH * (DV / 32);
        const double bw = m.coop_bw_cached * (1.0 - spill) + m.coop_bw_streamed * spill;
        const long rounds = (per_seg * nseg + kCoopSlots - 1) / kCoopSlots;
        // the walk's software pipeline runs one iteration beyond the chunks of a segment
        const double walk = smooth_max(rounds * (seg_chunks + 1) * m.coop_chunk_us, (in_bytes + out_bytes) / bw, m.coop_p);
        if (nseg == 1) return fmax(kOneKernelFloorUs, m.one_kernel_us + walk);
        const long pre_rounds = (per_seg * (nseg - 1) + kCoopSlots - 1) / kCoopSlots;
        const double pre = smooth_max(pre_rounds * seg_chunks * m.coop_pre_chunk_us, pre_bytes / bw, m.coop_p);
        return fmax(kThreeKernelFloorUs, m.three_kernel_us + walk + pre + scan);
    }
    const double bw = m.wide_bw_cached * (1.0 - spill) + m.wide_bw_streamed * spill;
    const long W = BH * nseg;
    const long rounds = (W + m.wide_slots - 1) / m.wide_slots;
    const double walk = smooth_max(rounds * seg_chunks * m.wide_chunk_us,
                                   (in_bytes + out_bytes) / bw * (W > 256 ? m.wide_crowded : 1.0), m.wide_p);
    if (nseg == 1) return fmax(kOneKernelFloorUs, m.one_kernel_us + walk);
    const int split = wide_pre_split(BH, nseg, seg_chunks);
    const long pre_rounds = (BH * (nseg - 1) * split + m.wide_slots - 1) / m.wide_slots;
    const double pre = smooth_max(pre_rounds * (seg_chunks / split) * m.wide_pre_chunk_us, pre_bytes / bw, m.wide_p);
    return fmax(kThreeKernelFloorUs, m.three_kernel_us + walk + pre + scan * split);
}

// D: width of q and k rows (rank); DV: width of v and out rows
//
// 16-bit inputs: every eligible (kernel, segment count) pair is priced with the cost model
// and the cheapest taken (near-ties go to fewer segments, then to the column-split kernel while its
// grid fits one round of workgroups, else to the wide kernel).  A caller's
// segment count or kernel choice narrows the candidates.  fp32 keeps the rule of
// about one workgroup per compute unit with a minimum segment length.  The plan depends on the
// shape, the input type, the segment request and the kernel knob only -- not on the output type or
// the mask -- so that leet_attn_workspace_bytes always sizes the workspace the call will ask for.
// choice: a leet_bf16_kernel value, or LEET_CHOICE_DEFAULT for the process-wide setting.
bool make_plan(long BH, int N, int D, int DV, int dtype, int segments, int choice, Plan* plan) {
    const int nchunks = (N + kChunk - 1) / kChunk;
    if (choice == LEET_CHOICE_DEFAULT) choice = g_bf16_kernel.load(std::memory_order_relaxed);
    const bool coop_able = dtype != LEET_F32;  // the column-split kernel: 16-bit inputs, every supported shape
    auto finish = [&](bool coop, int nseg, int seg_chunks) {
        const long per_seg = coop ? BH * (DV / 32) : BH;  // workgroups one segment of every sequence gives
        if (per_seg * (long)nseg >= (1L << 28)) return false;
        plan->coop = coop;
        plan->nseg = nseg;
        plan->seg_chunks = seg_chunks;
        plan->pre_split = coop ? 1 : dtype != LEET_F32 ? wide_pre_split(BH, nseg, seg_chunks) : f32_pre_split(BH, nseg, seg_chunks);
        // one state per boundary the pre-pass computes, and, with segments, one more per sequence:
        // the scan's copy of the entering state, which the walk reads instead of the caller's buffer
        const size_t slots = nseg > 1 ? (size_t)(nseg - 1) * plan->pre_split + 1 : 0;
        plan->ws_bytes = (size_t)BH * slots * D * DV * sizeof(float);
        return true;
    };
    auto round_segments = [&](long want, int* nseg, int* seg_chunks) {
        if (want < 1) want = 1;
        if (want > nchunks) want = nchunks;
        *seg_chunks = (int)((nchunks + want - 1) / want);
        *nseg = (nchunks + *seg_chunks - 1) / *seg_chunks;
    };

    if (dtype != LEET_F32) {
        // the column-split kernel needs four chunks to fill its pipeline and is not offered below
        const bool try_coop = coop_able && choice != LEET_KERNEL_WIDE && (nchunks >= 4 || choice == LEET_KERNEL_COLUMN_SPLIT);
        const bool try_wide = !(coop_able && choice == LEET_KERNEL_COLUMN_SPLIT);
        static const int kCounts[] = {1, 2, 3, 4, 6, 8, 12, 16, 24, 32, 48, 64};
        double best = 0.0;
        bool have = false, best_coop = false;
        int best_nseg = 1, best_chunks = nchunks;
        for (int want : kCounts) {
            if (segments > 0) want = segments;
            int nseg, seg_chunks;
            round_segments(want, &nseg, &seg_chunks);
            if (segments == 0 && nseg > 1 && seg_chunks < 2) break;
            // A later candidate must be 2 % cheaper to replace an earlier one, so the order decides
            // near-ties: fewer segments first, and at one segment count the column-split kernel first
            // unless its grid exceeds one round of workgroups (there the model is least sure of it).
            const bool coop_first = BH * (DV / 32) * nseg <= kCoopSlots;
            for (int turn = 0; turn < 2; ++turn) {
                const bool c = (turn == 0) == coop_first;
                if (c ? !try_coop : !try_wide) continue;
                const double t = predicted_us(c, BH, N, D, DV, nseg, seg_chunks);
                if (!have || t < best * 0.98) {
                    have = true; best = t; best_coop = c; best_nseg = nseg; best_chunks = seg_chunks;
                }
            }
            if (segments > 0) break;
        }
        return finish(best_coop, best_nseg, best_chunks);
    }

    // fp32
    long want;
    if (segments > 0) {
        want = segments;
    } else {
        want = (kTargetWorkgroups + BH - 1) / BH;
        // short sequences (up to 32 chunks) are cut down to single chunks: the pre-pass and the scan
        // cost less than a second chunk's MFMA latency in every workgroup (N = 512, d = 128: 28 against 43 us)
        long cap = nchunks <= 32 ? nchunks : nchunks / kMinSegChunksF32;
        if (cap < 1) cap = 1;
        if (want > cap) want = cap;
    }
    int nseg, seg_chunks;
    round_segments(want, &nseg, &seg_chunks);
    return finish(false, nseg, seg_chunks);
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// d: width of q and k rows; dv: width of v and out rows.  Square shapes for every type; rank 128 with
// value width 256 (the shape of the paper's usage example) for the 16-bit types.
bool shape_ok(int d, int dv, int dtype, int* status) {
    if (dtype != LEET_F32 && dtype != LEET_BF16 && dtype != LEET_F16) { *status = LEET_ERR_UNSUPPORTED; return false; }
    const bool square = d == dv && (d == 64 || d == 128);
    const bool wide_v = d == 128 && dv == 256 && dtype != LEET_F32;
    if (!square && !wide_v) { *status = LEET_ERR_UNSUPPORTED; return false; }
    return true;
}
bool shape_ok(int d, int dtype, int* status) { return shape_ok(d, d, dtype, status); }

// Library-owned workspace, one per device, grown on demand.  A block that a call has handed to
// a launch is never freed behind the caller's back: work still in flight, or a captured graph that
// is replayed later, may hold its address.  When a later call needs more, a larger block is
// allocated and the old one is retired until leet_attn_release_workspace.
std::mutex g_ws_mutex;
void* g_ws_ptr[kMaxDevices] = {nullptr};
size_t g_ws_size[kMaxDevices] = {0};
std::vector<void*> g_ws_retired[kMaxDevices];
int g_arch_ok[kMaxDevices] = {0};  // 0 unknown, 1 gfx950, -1 other

// Scratch of the entry point that allocates nothing: segment boundary states, in device memory
// that exists from the moment the library is loaded (every device that loads it holds its own copy
// until the process ends).  The array's name is a host-side handle only; the device address of
// each device's copy is looked up once per device and kept.
constexpr size_t kStaticScratchBytes = (size_t)32 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
void* g_scratch_ptr[kMaxDevices] = {nullptr};

int current_device(int* dev) {
    if (hipGetDevice(dev) != hipSuccess) return LEET_ERR_LAUNCH;
    if (*dev < 0 || *dev >= kMaxDevices) return LEET_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_ws_mutex);
    if (g_arch_ok[*dev] == 0) {
        hipDeviceProp_t prop;
        if (hipGetDeviceProperties(&prop, *dev) != hipSuccess) return LEET_ERR_LAUNCH;
        g_arch_ok[*dev] = (strncmp(prop.gcnArchName, "gfx950", 6) == 0) ? 1 : -1;
    }
    return g_arch_ok[*dev] == 1 ? LEET_OK : LEET_ERR_UNSUPPORTED;
}

// Device address of this device's copy of the static scratch (device `dev` is current).
int static_scratch(int dev, void** out) {
    std::lock_guard<std::mutex> lock(g_ws_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
            (void)hipGetLastError();
            return LEET_ERR_LAUNCH;
        }
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return LEET_OK;
}

int own_workspace(int dev, size_t bytes, hipStream_t stream, void** out) {
    std::lock_guard<std::mutex> lock(g_ws_mutex);
    if (g_ws_size[dev] < bytes) {
        // Growing means hipMalloc, which must not happen inside a stream capture (and the graph
        // would keep an address that only this capture's call ever sized).
        if (stream) {
            hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
            if (hipStreamIsCapturing(stream, &cs) != hipSuccess) {
                (void)hipGetLastError();
                return LEET_ERR_LAUNCH;
            }
            if (cs != hipStreamCaptureStatusNone) return LEET_ERR_CAPTURE;
        }
        // at least double, so that a run of growing shapes retires few blocks
        size_t want = bytes > 2 * g_ws_size[dev] ? bytes : 2 * g_ws_size[dev];
        void* p = nullptr;
        if (hipMalloc(&p, want) != hipSuccess) {
            (void)hipGetLastError();
            want = bytes;
            if (hipMalloc(&p, want) != hipSuccess) {
                (void)hipGetLastError();
                return LEET_ERR_LAUNCH;
            }
        }
        if (g_ws_ptr[dev]) g_ws_retired[dev].push_back(g_ws_ptr[dev]);
        g_ws_ptr[dev] = p;
        g_ws_size[dev] = want;
    }
    *out = g_ws_ptr[dev];
    return LEET_OK;
}

enum WorkspaceKind { kWsCallerOrOwned = 0, kWsStatic = 1 };

// A prefill over no tokens (N = 0): nothing to compute and no output rows; the state leaves as it
// entered, zero when none was given.  Touches the device only when a state has to be written.
int empty_forward(const float* state_in, float* state_out, long BH, int d, int dv, void* stream, float* kernel_ms) {
    if (kernel_ms) kernel_ms[0] = kernel_ms[1] = kernel_ms[2] = 0.0f;
    if (!state_out || state_out == state_in) return LEET_OK;
    int dev = 0;
    const int status = current_device(&dev);
    if (status != LEET_OK) return status;
    const hipError_t e = leet::launch_state_pass(state_in, state_out, (int)BH, d, dv, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? LEET_OK : LEET_ERR_LAUNCH;
}

int forward_impl(const void* q, const void* k, const void* v, const float* gamma, void* out,
                 const float* state_in, float* state_out, void* workspace, size_t workspace_bytes,
                 int segments, int B, int H, int N, int d, int dv, int dtype, int out_dtype, int mask,
                 void* stream, float* kernel_ms, int kernel_choice = LEET_CHOICE_DEFAULT,
                 WorkspaceKind ws_kind = kWsCallerOrOwned) {
    if (mask != LEET_MASK_DECAY && mask != LEET_MASK_CAUSAL) return LEET_ERR_INVALID_ARG;
    if (kernel_choice != LEET_CHOICE_DEFAULT && !kernel_choice_ok(kernel_choice)) return LEET_ERR_INVALID_ARG;
    const bool no_decay = mask == LEET_MASK_CAUSAL;
    if (B <= 0 || H <= 0 || N < 0 || d <= 0 || dv <= 0 || segments < 0) return LEET_ERR_INVALID_ARG;
    // no tokens: q, k, v, out are empty and may be null
    if ((N > 0 && (!q || !k || !v || !out)) || (!gamma && !no_decay)) return LEET_ERR_INVALID_ARG;
    int status = LEET_OK;
    if (!shape_ok(d, dv, dtype, &status)) return status;
    // the output is fp32, or, for 16-bit inputs, the input type
    if (out_dtype != LEET_F32 && (out_dtype != dtype || dtype == LEET_F32)) return LEET_ERR_UNSUPPORTED;
    if (no_decay) gamma = nullptr;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out) || !aligned16(state_in) ||
        !aligned16(state_out) || (reinterpret_cast<uintptr_t>(gamma) & 3u))
        return LEET_ERR_INVALID_ARG;
    if (workspace && (reinterpret_cast<uintptr_t>(workspace) & 255u)) return LEET_ERR_INVALID_ARG;
    const long BH = (long)B * H;
    if (BH >= (1L << 31) || (long)N > (1L << 30)) return LEET_ERR_TOO_LARGE;
    // the timing aid relaunches the walk: with the state handed on in place, later launches would
    // start from the state the first one left
    if (kernel_ms && state_in && state_in == state_out) return LEET_ERR_INVALID_ARG;
    if (N == 0) return empty_forward(state_in, state_out, BH, d, dv, stream, kernel_ms);

    Plan plan;
    if (!make_plan(BH, N, d, dv, dtype, segments, kernel_choice, &plan)) return LEET_ERR_TOO_LARGE;
    if (ws_kind == kWsStatic && plan.ws_bytes > kStaticScratchBytes) return LEET_ERR_SCRATCH_LIMIT;
    int dev = 0;
    status = current_device(&dev);
    if (status != LEET_OK) return status;
    hipStream_t s = static_cast<hipStream_t>(stream);

    void* ws = nullptr;
    if (plan.nseg > 1) {
        if (ws_kind == kWsStatic) {
            status = static_scratch(dev, &ws);
            if (status != LEET_OK) return status;
        } else if (workspace) {
            if (workspace_bytes < plan.ws_bytes) return LEET_ERR_INVALID_ARG;
            ws = workspace;
        } else {
            status = own_workspace(dev, plan.ws_bytes, s, &ws);
            if (status != LEET_OK) return status;
        }
    }

    leet::FwdParams p;
    p.q = q; p.k = k; p.v = v; p.gamma = gamma; p.out = out;
    p.state_in = state_in; p.state_out = state_out;
    p.seg_state = static_cast<float*>(ws);
    p.H = H; p.N = N; p.nseg = plan.nseg; p.seg_chunks = plan.seg_chunks;
    p.state_slots = (plan.nseg - 1) * plan.pre_split;
    p.state_step = plan.pre_split;
    // With segments, the first segments of the walk read the entering state from the scan's copy
    // of it (the slots after all boundary states), never from the caller's buffer: state_out may
    // alias state_in, and the last segment of a sequence may finish, and write it, before the
    // first segment of the same sequence has started.
    float* state_copy = nullptr;
    if (plan.nseg > 1 && state_in) {
        state_copy = p.seg_state + (size_t)BH * p.state_slots * d * dv;
        p.state_in = state_copy;
    }
    p.no_decay = no_decay ? 1 : 0;
    // Inputs that fit the 256 MB last-level cache are left to it (a pre-pass reads K and V before
    // the walk does, and a caller's next layer may reuse them); larger ones are streamed.
    p.stream_loads = (size_t)BH * N * (2 * d + dv) * (dtype == LEET_F32 ? 4 : 2) > kLastLevelCacheBytes ? 1 : 0;
    leet::FwdParams pre = p;  // geometry of the pre-pass and of the scan
    pre.nseg = p.state_slots + 1;
    pre.seg_chunks = plan.seg_chunks / plan.pre_split;
    const bool in16 = dtype != LEET_F32;
    const bool f16 = dtype == LEET_F16;
    const bool out16 = out_dtype != LEET_F32;

    const bool coop = plan.coop;
    auto launch_states = [&]() {
        return coop   ? leet::launch_fwd_16bit_coop_states(p, (int)BH, d, dv, f16, s)
               : in16 ? leet::launch_fwd_16bit_states(pre, (int)BH, d, dv, f16, s)
                      : leet::launch_fwd_f32_states(pre, (int)BH, d, s);
    };
    auto launch_scan = [&]() {
        return leet::launch_seg_scan(p.seg_state, state_in, state_copy, gamma, (int)BH, H, pre.nseg, pre.seg_chunks * kChunk,
                                     p.state_step, d, dv, s);
    };
    auto launch_walk = [&]() {
        return coop   ? leet::launch_fwd_16bit_coop_walk(p, (int)BH, d, dv, f16, out16, s)
               : in16 ? leet::launch_fwd_16bit_walk(p, (int)BH, d, dv, f16, out16, s)
                      : leet::launch_fwd_f32_walk(p, (int)BH, d, s);
    };

    if (!kernel_ms) {
        hipError_t e = launch_states();
        if (e == hipSuccess) e = launch_scan();
        if (e == hipSuccess) e = launch_walk();
        return e == hipSuccess ? LEET_OK : LEET_ERR_LAUNCH;
    }

    // Per-kernel timing: HIP events on the launch stream around each kernel.  The pre-pass and
    // the walk write the same values every time they run, so each is launched kProfileRepeat
    // times back to back between its two events and the time divided, which takes the event and
    // launch overhead out of the figure; the scan rewrites its input in place and runs once.
    constexpr int kProfileRepeat = 5;
    hipEvent_t ev[6] = {nullptr, nullptr, nullptr, nullptr, nullptr, nullptr};
    for (int i = 0; i < 6; ++i)
        if (hipEventCreate(&ev[i]) != hipSuccess) {
            for (int j = 0; j < i; ++j) (void)hipEventDestroy(ev[j]);
            return LEET_ERR_LAUNCH;
        }
    hipError_t e = hipSuccess;
    (void)hipEventRecord(ev[0], s);
    for (int r = 0; r < kProfileRepeat && e == hipSuccess; ++r) e = launch_states();
    (void)hipEventRecord(ev[1], s);
    (void)hipEventRecord(ev[2], s);
    if (e == hipSuccess) e = launch_scan();
    (void)hipEventRecord(ev[3], s);
    (void)hipEventRecord(ev[4], s);
    for (int r = 0; r < kProfileRepeat && e == hipSuccess; ++r) e = launch_walk();
    (void)hipEventRecord(ev[5], s);
    int rc = (e == hipSuccess) ? LEET_OK : LEET_ERR_LAUNCH;
    if (hipEventSynchronize(ev[5]) != hipSuccess) rc = LEET_ERR_LAUNCH;
    for (int i = 0; i < 3 && rc == LEET_OK; ++i)
        if (hipEventElapsedTime(&kernel_ms[i], ev[2 * i], ev[2 * i + 1]) != hipSuccess) rc = LEET_ERR_LAUNCH;
    if (rc == LEET_OK) {
        kernel_ms[0] /= kProfileRepeat;
        kernel_ms[2] /= kProfileRepeat;
        if (plan.nseg <= 1) kernel_ms[0] = kernel_ms[1] = 0.0f;  // nothing was launched in those slots
    }
    for (int i = 0; i < 6; ++i) (void)hipEventDestroy(ev[i]);
    return rc;
}

// the two comparison kernels (row-based, FleetAttention) take the same arguments
int forward_elementwise(bool fleet, const void* q, const void* k, const void* v, const float* gamma, float* out,
                        const float* state_in, float* state_out, int B, int H, int N, int d, int dv,
                        int dtype, int mask, void* stream) {
    if (mask != LEET_MASK_DECAY && mask != LEET_MASK_CAUSAL) return LEET_ERR_INVALID_ARG;
    if (mask == LEET_MASK_CAUSAL) gamma = nullptr;
    if (B <= 0 || H <= 0 || N < 0 || d <= 0 || dv <= 0) return LEET_ERR_INVALID_ARG;
    if ((N > 0 && (!q || !k || !v || !out)) || (!gamma && mask == LEET_MASK_DECAY)) return LEET_ERR_INVALID_ARG;
    int status = LEET_OK;
    if (!shape_ok(d, dv, dtype, &status)) return status;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out) || !aligned16(state_in) ||
        !aligned16(state_out) || (reinterpret_cast<uintptr_t>(gamma) & 3u))
        return LEET_ERR_INVALID_ARG;
    const long BH = (long)B * H;
    if (BH >= (1L << 31) / 8 || (long)N > (1L << 30)) return LEET_ERR_TOO_LARGE;
    if (N == 0) return empty_forward(state_in, state_out, BH, d, dv, stream, nullptr);
    int dev = 0;
    status = current_device(&dev);
    if (status != LEET_OK) return status;
    const int elem = dtype == LEET_F32 ? 0 : dtype == LEET_BF16 ? 1 : 2;
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipError_t e = fleet ? leet::launch_fleet(q, k, v, gamma, out, state_in, state_out, (int)BH, H, N, d, dv, elem, s)
                         : leet::launch_recurrent(q, k, v, gamma, out, state_in, state_out, (int)BH, H, N, d, dv, elem, s);
    return e == hipSuccess ? LEET_OK : LEET_ERR_LAUNCH;
}

}  // namespace

extern "C" {

int leet_attn_forward(const void* q, const void* k, const void* v, const float* gamma, float* out,
                      int B, int H, int N, int d, int dtype, void* stream) {
    if (dtype == LEET_F16) return LEET_ERR_UNSUPPORTED;  // fp16 inputs go through leet_attn_forward_v2
    return forward_impl(q, k, v, gamma, out, nullptr, nullptr, nullptr, 0, 0, B, H, N, d, d, dtype, LEET_F32,
                        LEET_MASK_DECAY, stream, nullptr);
}

int leet_attn_forward_ex(const void* q, const void* k, const void* v, const float* gamma, float* out,
                         const float* state_in, float* state_out, void* workspace, size_t workspace_bytes,
                         int segments, int B, int H, int N, int d, int dtype, void* stream) {
    if (dtype == LEET_F16) return LEET_ERR_UNSUPPORTED;
    return forward_impl(q, k, v, gamma, out, state_in, state_out, workspace, workspace_bytes, segments,
                        B, H, N, d, d, dtype, LEET_F32, LEET_MASK_DECAY, stream, nullptr);
}

int leet_attn_forward_v2(const void* q, const void* k, const void* v, const float* gamma, void* out,
                         const float* state_in, float* state_out, void* workspace, size_t workspace_bytes,
                         int segments, int B, int H, int N, int d, int in_dtype, int out_dtype, int mask,
                         void* stream) {
    return forward_impl(q, k, v, gamma, out, state_in, state_out, workspace, workspace_bytes, segments,
                        B, H, N, d, d, in_dtype, out_dtype, mask, stream, nullptr);
}

int leet_attn_forward_profile(const void* q, const void* k, const void* v, const float* gamma, float* out,
                              const float* state_in, float* state_out, void* workspace, size_t workspace_bytes,
                              int segments, int B, int H, int N, int d, int dtype, void* stream,
                              float* kernel_ms) {
    if (!kernel_ms) return LEET_ERR_INVALID_ARG;
    if (dtype == LEET_F16) return LEET_ERR_UNSUPPORTED;
    return forward_impl(q, k, v, gamma, out, state_in, state_out, workspace, workspace_bytes, segments,
                        B, H, N, d, d, dtype, LEET_F32, LEET_MASK_DECAY, stream, kernel_ms);
}

int leet_attn_forward_rd(const void* q, const void* k, const void* v, const float* gamma, void* out,
                         const float* state_in, float* state_out, void* workspace, size_t workspace_bytes,
                         int segments, int B, int H, int N, int r, int dv, int in_dtype, int out_dtype,
                         int mask, void* stream) {
    return forward_impl(q, k, v, gamma, out, state_in, state_out, workspace, workspace_bytes, segments,
                        B, H, N, r, dv, in_dtype, out_dtype, mask, stream, nullptr);
}

int leet_attn_forward_v3(const void* q, const void* k, const void* v, const float* gamma, void* out,
                         const float* state_in, float* state_out, void* workspace, size_t workspace_bytes,
                         int segments, int kernel, int B, int H, int N, int r, int dv, int in_dtype,
                         int out_dtype, int mask, void* stream) {
    return forward_impl(q, k, v, gamma, out, state_in, state_out, workspace, workspace_bytes, segments,
                        B, H, N, r, dv, in_dtype, out_dtype, mask, stream, nullptr, kernel);
}

int leet_attn_forward_static(const void* q, const void* k, const void* v, const float* gamma, float* out,
                             const float* state_in, float* state_out, int segments,
                             int B, int H, int N, int d, int dtype, void* stream) {
    if (dtype == LEET_F16) return LEET_ERR_UNSUPPORTED;
    return forward_impl(q, k, v, gamma, out, state_in, state_out, nullptr, 0, segments, B, H, N, d, d, dtype,
                        LEET_F32, LEET_MASK_DECAY, stream, nullptr, LEET_CHOICE_DEFAULT, kWsStatic);
}

size_t leet_attn_static_scratch_bytes(void) { return kStaticScratchBytes; }

size_t leet_attn_workspace_bytes_v3(int B, int H, int N, int r, int dv, int dtype, int segments, int kernel) {
    int status = LEET_OK;
    if (B <= 0 || H <= 0 || N <= 0 || segments < 0 || !shape_ok(r, dv, dtype, &status)) return 0;  // N = 0 needs none
    if (kernel != LEET_CHOICE_DEFAULT && !kernel_choice_ok(kernel)) return 0;
    Plan plan;
    if (!make_plan((long)B * H, N, r, dv, dtype, segments, kernel, &plan)) return 0;
    return plan.ws_bytes;
}

size_t leet_attn_workspace_bytes_rd(int B, int H, int N, int r, int dv, int dtype, int segments) {
    return leet_attn_workspace_bytes_v3(B, H, N, r, dv, dtype, segments, LEET_CHOICE_DEFAULT);
}

size_t leet_attn_workspace_bytes(int B, int H, int N, int d, int dtype, int segments) {
    return leet_attn_workspace_bytes_rd(B, H, N, d, d, dtype, segments);
}

int leet_attn_forward_recurrent_rd(const void* q, const void* k, const void* v, const float* gamma, float* out,
                                   const float* state_in, float* state_out, int B, int H, int N, int d, int dv,
                                   int dtype, int mask, void* stream) {
    return forward_elementwise(false, q, k, v, gamma, out, state_in, state_out, B, H, N, d, dv, dtype, mask, stream);
}

int leet_attn_forward_fleet(const void* q, const void* k, const void* v, const float* gamma, float* out,
                            const float* state_in, float* state_out, int B, int H, int N, int r, int dv,
                            int dtype, int mask, void* stream) {
    return forward_elementwise(true, q, k, v, gamma, out, state_in, state_out, B, H, N, r, dv, dtype, mask, stream);
}

int leet_attn_forward_recurrent(const void* q, const void* k, const void* v, const float* gamma, float* out,
                                const float* state_in, float* state_out, int B, int H, int N, int d,
                                int dtype, int mask, void* stream) {
    return leet_attn_forward_recurrent_rd(q, k, v, gamma, out, state_in, state_out, B, H, N, d, d, dtype, mask,
                                          stream);
}

int leet_attn_query_plan_v3(int B, int H, int N, int r, int dv, int dtype, int segments, int kernel_choice,
                            int* nseg, int* kernel) {
    int status = LEET_OK;
    if (B <= 0 || H <= 0 || N < 0 || segments < 0) return LEET_ERR_INVALID_ARG;
    if (kernel_choice != LEET_CHOICE_DEFAULT && !kernel_choice_ok(kernel_choice)) return LEET_ERR_INVALID_ARG;
    if (!shape_ok(r, dv, dtype, &status)) return status;
    if (N == 0) {  // no tokens: no segment, no chunk kernel
        if (nseg) *nseg = 0;
        if (kernel) *kernel = LEET_KERNEL_WIDE;
        return LEET_OK;
    }
    Plan plan;
    if (!make_plan((long)B * H, N, r, dv, dtype, segments, kernel_choice, &plan)) return LEET_ERR_TOO_LARGE;
    if (nseg) *nseg = plan.nseg;
    if (kernel) *kernel = plan.coop ? LEET_KERNEL_COLUMN_SPLIT : LEET_KERNEL_WIDE;
    return LEET_OK;
}

int leet_attn_query_plan_rd(int B, int H, int N, int r, int dv, int dtype, int segments, int* nseg, int* kernel) {
    return leet_attn_query_plan_v3(B, H, N, r, dv, dtype, segments, LEET_CHOICE_DEFAULT, nseg, kernel);
}

int leet_attn_query_plan(int B, int H, int N, int d, int dtype, int segments, int* nseg, int* kernel) {
    return leet_attn_query_plan_rd(B, H, N, d, d, dtype, segments, nseg, kernel);
}

int leet_attn_decode_step_v3(const void* q, const void* k, const void* v, const float* gamma,
                             float* state_inout, float* out, int B, int H, int d, int dv, int dtype, int mask,
                             int store, void* stream) {
    if (mask != LEET_MASK_DECAY && mask != LEET_MASK_CAUSAL) return LEET_ERR_INVALID_ARG;
    if (store != LEET_CHOICE_DEFAULT && !decode_store_ok(store)) return LEET_ERR_INVALID_ARG;
    if (mask == LEET_MASK_CAUSAL) gamma = nullptr;
    if (!q || !k || !v || (!gamma && mask == LEET_MASK_DECAY) || !state_inout || !out) return LEET_ERR_INVALID_ARG;
    if (B <= 0 || H <= 0 || d <= 0 || dv <= 0) return LEET_ERR_INVALID_ARG;
    int status = LEET_OK;
    if (!shape_ok(d, dv, dtype, &status)) return status;
    if (!aligned16(state_inout) || !aligned16(out) || (reinterpret_cast<uintptr_t>(gamma) & 3u) ||
        (reinterpret_cast<uintptr_t>(q) & 3u) || (reinterpret_cast<uintptr_t>(k) & 3u) ||
        (reinterpret_cast<uintptr_t>(v) & 3u))
        return LEET_ERR_INVALID_ARG;
    const long BH = (long)B * H;
    if (BH >= (1L << 31)) return LEET_ERR_TOO_LARGE;
    int dev = 0;
    status = current_device(&dev);
    if (status != LEET_OK) return status;
    const int elem = dtype == LEET_F32 ? 0 : dtype == LEET_BF16 ? 1 : 2;
    // AUTO.  A small state (under a quarter of the last-level cache) is stored normally: it survives
    // there next to a few neighbours.  A larger one is worth caching only if nothing displaces it
    // before its next step -- 5 % gained (128 MiB stepped alone: 39.9 against 41.8 us), against 20 %
    // lost when it is displaced (three 128 MiB states in turn: 53 against 44 us; 512 MiB: 5.1 against
    // 6.4 TB/s).  The library cannot see the caller's other work, but it can see its own: if the
    // previous decode call on this device stepped this very buffer, and the state fits half of the
    // cache, it is being stepped alone and is cached; in every other case (another layer's state
    // came in between, or this is the first step) it is streamed.
    const size_t state_bytes = (size_t)BH * d * dv * sizeof(float);
    const void* prev_state = g_last_decode_state[dev].exchange(state_inout, std::memory_order_relaxed);
    const int store_mode = store == LEET_CHOICE_DEFAULT ? g_decode_store.load(std::memory_order_relaxed) : store;
    bool stream_store = store_mode == LEET_DECODE_STORE_STREAM;
    if (store_mode == LEET_DECODE_STORE_AUTO && state_bytes >= kLastLevelCacheBytes / 4)
        stream_store = !(prev_state == state_inout && state_bytes <= kLastLevelCacheBytes / 2);
    hipError_t e = leet::launch_decode(q, k, v, gamma, state_inout, out, (int)BH, H, d, dv, elem, stream_store,
                                       static_cast<hipStream_t>(stream));
    return e == hipSuccess ? LEET_OK : LEET_ERR_LAUNCH;
}

int leet_attn_decode_step_rd(const void* q, const void* k, const void* v, const float* gamma,
                             float* state_inout, float* out, int B, int H, int d, int dv, int dtype, int mask,
                             void* stream) {
    return leet_attn_decode_step_v3(q, k, v, gamma, state_inout, out, B, H, d, dv, dtype, mask, LEET_CHOICE_DEFAULT,
                                    stream);
}

int leet_attn_decode_step_v2(const void* q, const void* k, const void* v, const float* gamma,
                             float* state_inout, float* out, int B, int H, int d, int dtype, int mask,
                             void* stream) {
    return leet_attn_decode_step_rd(q, k, v, gamma, state_inout, out, B, H, d, d, dtype, mask, stream);
}

int leet_attn_decode_step_ex(const void* q, const void* k, const void* v, const float* gamma,
                             float* state_inout, float* out, int B, int H, int d, int dtype, void* stream) {
    return leet_attn_decode_step_v2(q, k, v, gamma, state_inout, out, B, H, d, dtype, LEET_MASK_DECAY, stream);
}

int leet_attn_decode_step(const void* q, const void* k, const void* v, const float* gamma,
                          float* state_inout, float* out, int B, int H, int d, void* stream) {
    return leet_attn_decode_step_ex(q, k, v, gamma, state_inout, out, B, H, d, LEET_BF16, stream);
}

int leet_attn_release_workspace(void) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return LEET_ERR_LAUNCH;
    std::lock_guard<std::mutex> lock(g_ws_mutex);
    int rc = LEET_OK;
    if (g_ws_ptr[dev]) {
        if (hipFree(g_ws_ptr[dev]) != hipSuccess) rc = LEET_ERR_LAUNCH;
        g_ws_ptr[dev] = nullptr;
        g_ws_size[dev] = 0;
    }
    for (void* old : g_ws_retired[dev])
        if (hipFree(old) != hipSuccess) rc = LEET_ERR_LAUNCH;
    g_ws_retired[dev].clear();
    return rc;
}

const char* leet_attn_strerror(int status) {
    switch (status) {
        case LEET_OK: return "ok";
        case LEET_ERR_INVALID_ARG: return "invalid argument (null pointer, non-positive size, misaligned pointer or workspace too small)";
        case LEET_ERR_UNSUPPORTED: return "unsupported (d must be 64 or 128, or rank 128 with value width 256 for 16-bit inputs; dtype f32, bf16 or f16; output fp32 or the 16-bit input type; device gfx950)";
        case LEET_ERR_LAUNCH: return "HIP runtime error (launch or allocation failed)";
        case LEET_ERR_TOO_LARGE: return "sizes exceed the library's index range";
        case LEET_ERR_CAPTURE: return "the library-owned workspace would have to be allocated or grown while the stream is capturing (make one eager call of this size first, or pass a caller-owned workspace)";
        case LEET_ERR_SCRATCH_LIMIT: return "the segment states of this call exceed the static scratch of leet_attn_forward_static (32 MiB; request fewer segments, or use leet_attn_forward_ex with a workspace)";
        default: return "unknown status";
    }
}

int leet_attn_set_bf16_kernel(int which) {
    if (!kernel_choice_ok(which)) return LEET_ERR_INVALID_ARG;
    g_bf16_kernel.store(which, std::memory_order_relaxed);
    return LEET_OK;
}

int leet_attn_get_bf16_kernel(void) { return g_bf16_kernel.load(std::memory_order_relaxed); }

int leet_attn_set_decode_store(int mode) {
    if (!decode_store_ok(mode)) return LEET_ERR_INVALID_ARG;
    g_decode_store.store(mode, std::memory_order_relaxed);
    return LEET_OK;
}

int leet_attn_get_decode_store(void) { return g_decode_store.load(std::memory_order_relaxed); }

const char* leet_attn_version(void) { return "0.7.0"; }

}  // extern "C"
