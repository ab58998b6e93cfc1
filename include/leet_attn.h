/*
 * leet_attn.h -- C ABI of the MI355X (gfx950) library for exponentially decaying
 * causal linear attention.
 *
 * Operator (Section 2.2, Eq. "BCMV", with B = Q and C = K):
 *
 *     O = ((Q K^T) .* M) V,      M[i][j] = gamma^(i-j) if i >= j, else 0,
 *
 * one gamma per head, 0 <= gamma <= 1, 0^0 = 1 (so M[i][i] = 1 always).  There is
 * no softmax, no row normalisation and no 1/sqrt(d) factor inside the operator.
 * The library evaluates it in chunked ("block-based") form -- Appendix B.2, Alg. 2,
 * carried over to the decaying mask with the row/column weight split of
 * Appendix B.3, Alg. 4 -- and continues it token by token with the row-based
 * recursion of Appendix B.1, Alg. 1 and the discounted update of Appendix C.1:
 *
 *     S <- gamma S + k^T v ;   o = q S            (S is d x d, rows = key index).
 *
 * Conventions shared by every entry point
 *   - Every tensor pointer is a DEVICE pointer (HIP global memory on the current
 *     device), 16-byte aligned, densely packed, row-major in the stated shape.
 *   - `stream` is a hipStream_t passed as void*; NULL means the default stream.
 *     Calls are asynchronous: they enqueue kernels on `stream` and return.  The
 *     caller keeps every buffer alive and unmodified until the stream has
 *     finished the work.
 *   - The caller owns all buffers.  The library keeps no pointer after the work
 *     is done.  `out` must not overlap any input.
 *   - The return value is a leet_status.  Arguments are validated on the host
 *     before anything is enqueued: on every status but LEET_OK and
 *     LEET_ERR_LAUNCH no buffer has been written.  LEET_ERR_LAUNCH means the HIP
 *     runtime failed part-way; the contents of the output buffers are then undefined.
 *   - d must be 64 or 128 (the _rd entry points also take rank 128 with value width
 *     256).  B, H >= 1.  N need not be a multiple of the chunk length (64
 *     tokens); the last chunk may be ragged.
 *   - A prefill over no tokens is legal (N = 0; N < 0 is LEET_ERR_INVALID_ARG): the loop over
 *     chunks (Alg. 2) does not run, so nothing is written to `out`, and `state_out`, when
 *     given, receives the entering state unchanged (zero if `state_in` is NULL).  q, k, v and
 *     out are then empty and may be NULL.  It needs no workspace; the plan query reports zero
 *     segments.  The decode step has no length and always processes one token.
 *   - Outputs that the library will not read again (prefill `out`) are written
 *     with nontemporal stores, so that they do not displace the inputs from the
 *     caches; this changes no value.
 *   - gamma outside [0, 1] is not diagnosed (the values live in device memory).
 */
#ifndef LEET_ATTN_H
#define LEET_ATTN_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    LEET_F32 = 0,  /* q, k, v are IEEE binary32; products on fp32 MFMA              */
    LEET_BF16 = 1, /* q, k, v are bfloat16; products on bf16 MFMA, fp32 accumulate  */
    LEET_F16 = 2   /* q, k, v are IEEE binary16; products on fp16 MFMA, fp32 accumulate
                      (accepted by the _v2, _rd and _recurrent entry points)       */
} leet_dtype;

/*
 * Which mask M the operator uses (Section 2.2: the decaying mask of Eq. "BCMV", or the 0/1
 * causal mask of plain causal linear attention, which is the same operator with gamma = 1).
 */
typedef enum {
    LEET_MASK_DECAY = 0, /* M[i][j] = gamma_h^(i-j), i >= j; `gamma` is read                  */
    LEET_MASK_CAUSAL = 1 /* M[i][j] = 1, i >= j; `gamma` is ignored and may be NULL; kernels
                            specialised to skip every decay multiplication                 */
} leet_mask;

typedef enum {
    LEET_OK = 0,
    LEET_ERR_INVALID_ARG = 1, /* NULL required pointer, non-positive size, misaligned pointer, workspace too small */
    LEET_ERR_UNSUPPORTED = 2, /* d not in {64, 128}, unknown dtype or dtype combination, no gfx950 device */
    LEET_ERR_LAUNCH = 3,      /* the HIP runtime refused a launch or an allocation */
    LEET_ERR_TOO_LARGE = 4,   /* sizes overflow the library's index range */
    LEET_ERR_CAPTURE = 5,     /* `stream` is capturing and the library-owned workspace would have to be
                                 allocated or grown; nothing was enqueued */
    LEET_ERR_SCRATCH_LIMIT = 6 /* leet_attn_forward_static: the call's segment states exceed the static
                                 scratch; nothing was enqueued */
} leet_status;

/*
 * Chunked prefill (Eq. "BCMV" via Alg. 2 + the Alg. 4 weight split), zero initial state.
 *   q, k, v  [B][H][N][d], element type `dtype`
 *   gamma    [H] float
 *   out      [B][H][N][d] float (fp32 for both input types)
 * Long sequences are cut into segments that run in parallel; the segment
 * boundary states live in a per-device workspace that the library allocates
 * with hipMalloc on first need.  When a later call needs more, a larger block
 * is allocated and the old one is kept (work in flight or a captured graph may
 * still use it) until leet_attn_release_workspace.  Because that workspace is
 * shared, calls on one device must not run concurrently on different streams;
 * use leet_attn_forward_ex with caller-owned workspaces for that.
 * Under stream capture the library never allocates: if the workspace it owns
 * is too small for the call the status is LEET_ERR_CAPTURE and nothing is
 * recorded.  Make one eager call of the same shape before capturing (the graph
 * then holds an address that stays valid until leet_attn_release_workspace), or
 * capture leet_attn_forward_ex with a caller-owned workspace.
 */
int leet_attn_forward(const void *q, const void *k, const void *v, const float *gamma, float *out,
                      int B, int H, int N, int d, int dtype, void *stream);

/*
 * One decode step (Alg. 1 with the discounted update of Appendix C.1):
 *     S <- gamma_h S + k^T v ;  o = q S     for each (b, h).
 *   q, k, v      [B][H][d] bfloat16
 *   gamma        [H] float
 *   state_inout  [B][H][d][d] float, rows = key index, cols = value index; updated in place
 *   out          [B][H][d] float
 */
int leet_attn_decode_step(const void *q, const void *k, const void *v, const float *gamma,
                          float *state_inout, float *out, int B, int H, int d, void *stream);

/* As leet_attn_decode_step, with q, k, v of element type `dtype` (LEET_F32 or LEET_BF16). */
int leet_attn_decode_step_ex(const void *q, const void *k, const void *v, const float *gamma,
                             float *state_inout, float *out, int B, int H, int d, int dtype,
                             void *stream);

/*
 * Chunked prefill with state hand-off (the state that Alg. 1 carries from token to token,
 * entering and leaving the call), so that a prompt can be processed in pieces and
 * continued by decode steps.
 *   state_in   [B][H][d][d] float or NULL (zero state); the state before token 0
 *   state_out  [B][H][d][d] float or NULL; receives the state after token N-1.
 *              May alias state_in (when the sequences are cut into segments the kernels read
 *              the entering state from a copy in the workspace, so the order in which the
 *              segments run does not matter).
 *   workspace  device buffer of at least leet_attn_workspace_bytes(B, H, N, d, dtype)
 *              bytes, 256-byte aligned, or NULL to use the library's own per-device
 *              workspace as leet_attn_forward does.  Its contents are scratch.
 *   workspace_bytes  size of `workspace` (ignored when workspace is NULL)
 *   segments   0 = let the library choose how many parallel segments to cut each
 *              sequence into; > 0 = request that many (clamped to the number of
 *              chunks).  The result does not depend on it beyond rounding.
 */
int leet_attn_forward_ex(const void *q, const void *k, const void *v, const float *gamma, float *out,
                         const float *state_in, float *state_out,
                         void *workspace, size_t workspace_bytes, int segments,
                         int B, int H, int N, int d, int dtype, void *stream);

/*
 * Chunked prefill with every option: as leet_attn_forward_ex, and additionally
 *   in_dtype   LEET_F32, LEET_BF16 or LEET_F16 (the paper's methods take fp16 and fp32 inputs,
 *              Section 4; bf16 is this library's headline type)
 *   out_dtype  LEET_F32, or, for 16-bit inputs, the input type: `out` is then [B][H][N][d] of
 *              that type, rounded to nearest even from the fp32 accumulators (halves the
 *              output traffic of an HBM-bound kernel)
 *   mask       a leet_mask
 * Any other combination returns LEET_ERR_UNSUPPORTED.  States stay fp32.
 */
int leet_attn_forward_v2(const void *q, const void *k, const void *v, const float *gamma, void *out,
                         const float *state_in, float *state_out,
                         void *workspace, size_t workspace_bytes, int segments,
                         int B, int H, int N, int d, int in_dtype, int out_dtype, int mask, void *stream);

/*
 * For callers that cannot allocate device memory (code under HIP graph capture that has not made
 * an eager call first, tight serving loops, harnesses that forbid hipMalloc): leet_attn_forward_ex
 * with the segment states in a fixed scratch array that is part of the library's device image
 * (leet_attn_static_scratch_bytes() = 32 MiB, held by every GPU that loads the library until the
 * process ends).  The call allocates and frees nothing; q, k, v, gamma, out and the states are
 * the caller's as everywhere else.  Same kernels and same plan as leet_attn_forward_ex, hence
 * bit-identical results.
 *   segments   as for leet_attn_forward_ex.  If the plan's segment states need more than the
 *              scratch holds (leet_attn_workspace_bytes tells), the status is
 *              LEET_ERR_SCRATCH_LIMIT and nothing is enqueued; ask for fewer segments (one
 *              segment needs no scratch at all) or use leet_attn_forward_ex.
 *   dtype      LEET_F32 or LEET_BF16; fp32 output; decaying mask.
 * All calls on one GPU share that GPU's scratch, which keeps the previous call's contents
 * (nothing in it needs clearing: every slot a call reads is first written by that call's own
 * kernels).  Calls that overlap on one GPU -- different streams, or a graph replay beside an
 * eager call -- race on it; serialise them.
 */
int leet_attn_forward_static(const void *q, const void *k, const void *v, const float *gamma, float *out,
                             const float *state_in, float *state_out, int segments,
                             int B, int H, int N, int d, int dtype, void *stream);
size_t leet_attn_static_scratch_bytes(void);

/*
 * Row-based prefill: the same operator evaluated token by token as Alg. 1 (Appendix B.1) states
 * it, with the discounted update of Appendix C.1 -- the decode step iterated over N with the
 * state kept on chip.  No MFMA, sequential in N, parallel over (batch, head) and value columns
 * only.  It is the in-library comparison point for the chunked kernels (the paper's fastest
 * method at batch 16 is of this kind, Section 5.1); the chunked entry points are the fast path.
 *   q, k, v    [B][H][N][d] of `dtype` (LEET_F32, LEET_BF16 or LEET_F16)
 *   out        [B][H][N][d] float
 *   state_in   [B][H][d][d] float or NULL;  state_out  [B][H][d][d] float or NULL (may alias)
 *   mask       a leet_mask (gamma may be NULL for LEET_MASK_CAUSAL)
 * Needs no workspace.
 */
int leet_attn_forward_recurrent(const void *q, const void *k, const void *v, const float *gamma, float *out,
                                const float *state_in, float *state_out,
                                int B, int H, int N, int d, int dtype, int mask, void *stream);

/*
 * Rank different from the value width.  The operator is defined for B, C in R^(N x r) and
 * V in R^(N x d) (Section 2.2); the entry points above take r = d.  These take them apart:
 *   q, k   [B][H][N][r]      v, out   [B][H][N][dv]      states   [B][H][r][dv] float
 * Supported: r = dv in {64, 128} for every input type, and r = 128, dv = 256 (the shape of the
 * paper's usage example, Section 4) for LEET_BF16 and LEET_F16 inputs; anything else returns
 * LEET_ERR_UNSUPPORTED.  All other arguments as in leet_attn_forward_v2,
 * leet_attn_forward_recurrent, leet_attn_decode_step_v2 and leet_attn_workspace_bytes.
 */
int leet_attn_forward_rd(const void *q, const void *k, const void *v, const float *gamma, void *out,
                         const float *state_in, float *state_out,
                         void *workspace, size_t workspace_bytes, int segments,
                         int B, int H, int N, int r, int dv, int in_dtype, int out_dtype, int mask, void *stream);
int leet_attn_forward_recurrent_rd(const void *q, const void *k, const void *v, const float *gamma, float *out,
                                   const float *state_in, float *state_out,
                                   int B, int H, int N, int r, int dv, int dtype, int mask, void *stream);
int leet_attn_decode_step_rd(const void *q, const void *k, const void *v, const float *gamma,
                             float *state_inout, float *out, int B, int H, int r, int dv, int dtype, int mask,
                             void *stream);
size_t leet_attn_workspace_bytes_rd(int B, int H, int N, int r, int dv, int dtype, int segments);

/*
 * FleetAttention prefill: the operator as the sum over the rank of discounted cumulative sums,
 * O = sum_j diag(b_j) lambda-cumsum(diag(c_j) V) (Section 3, Eq. "p"; Appendix C.1 for the decay),
 * evaluated in column blocks (parallel) and row blocks (in order) with one carried vector per
 * rank index, as Alg. 5 (Appendix B.4) lays it out.  Element-wise work on the vector ALUs only,
 * no MFMA: like the row-based kernel it is an in-library comparison point (the paper's own
 * measurements, Section 5.1 and Appendix E, have it slowest), not the fast path.
 *   q, k   [B][H][N][r] of `dtype` (the paper's B and C)      v   [B][H][N][dv] of `dtype`
 *   out    [B][H][N][dv] float
 *   state_in, state_out   [B][H][r][dv] float or NULL: the carried vectors l^j entering the first
 *          row block and leaving the last; they are the rows of the state the other kernels use
 *   mask   a leet_mask (gamma may be NULL for LEET_MASK_CAUSAL: plain cumsum)
 * Shapes as for leet_attn_forward_recurrent_rd.  Needs no workspace and no atomics.
 */
int leet_attn_forward_fleet(const void *q, const void *k, const void *v, const float *gamma, float *out,
                            const float *state_in, float *state_out,
                            int B, int H, int N, int r, int dv, int dtype, int mask, void *stream);

/* As leet_attn_decode_step_ex, with `dtype` also LEET_F16 and with a leet_mask. */
int leet_attn_decode_step_v2(const void *q, const void *k, const void *v, const float *gamma,
                             float *state_inout, float *out, int B, int H, int d, int dtype, int mask,
                             void *stream);

/*
 * Bytes of workspace leet_attn_forward_ex needs for this shape with `segments`
 * as above (0 = library's choice) under the process-wide kernel choice: one d x d
 * fp32 state per segment boundary the library computes, plus one per sequence for
 * the copy of the entering state.  Returns 0 when no workspace is needed (one
 * segment) or the arguments are invalid.
 */
size_t leet_attn_workspace_bytes(int B, int H, int N, int d, int dtype, int segments);

/*
 * Frees the library-owned workspace of the current device, including blocks retired
 * when it grew (synchronises the device first).  Optional; the workspace is
 * otherwise kept until process exit.  A graph captured from a call that used the
 * library-owned workspace must not be replayed after this.
 */
int leet_attn_release_workspace(void);

/*
 * Tuning knob: which kernel a bf16 or fp16 prefill uses.  Both compute the same chunked form (Alg. 2
 * with the decaying mask) and pass the same parity tests; they differ in how the work is split.
 *   LEET_KERNEL_WIDE          one workgroup per (sequence, segment), all d value columns
 *   LEET_KERNEL_COLUMN_SPLIT  dv/32 workgroups per (sequence, segment), 32 value columns each,
 *                             placed on one XCD; fewer segments needed to fill the device
 *                             (16-bit inputs, every supported shape; fp32 runs wide)
 *   LEET_KERNEL_AUTO          (default) the library prices both kernels at each candidate segment
 *                             count with a cost model fitted to measurements and takes the
 *                             cheapest pair; leet_attn_query_plan reports the outcome
 * With WIDE or COLUMN_SPLIT set, only the segment count is chosen that way.
 * The setter changes the process-wide default, which every entry point without a `kernel`
 * argument uses; a thread that must not depend on what other threads set between its workspace
 * query and its call passes the choice per call (the _v3 entry points below).  Returns
 * LEET_ERR_INVALID_ARG for any other value.
 */
typedef enum { LEET_KERNEL_WIDE = 0, LEET_KERNEL_COLUMN_SPLIT = 1, LEET_KERNEL_AUTO = 2 } leet_bf16_kernel;
int leet_attn_set_bf16_kernel(int which);
int leet_attn_get_bf16_kernel(void);

/*
 * Tuning knob: how a decode step stores the updated state.
 *   LEET_DECODE_STORE_AUTO    (default) a state under a quarter of the 256 MB last-level cache is
 *                             cached.  A larger one is cached only when it is being stepped alone --
 *                             the previous decode call on this device updated this very buffer, and
 *                             it fits half of the cache -- and streamed otherwise (another state came
 *                             in between, or this is its first step).  Streaming a state that would
 *                             have stayed cached costs about 5 %, caching one that is displaced
 *                             before its next step about 20 %
 *   LEET_DECODE_STORE_CACHED  ordinary stores: best when the next step on the same state finds it
 *                             in the cache (one small model stepping alone)
 *   LEET_DECODE_STORE_STREAM  nontemporal stores: best when other states are touched before this one
 *                             is used again (many layers taking turns), whatever its size
 * The results are identical; only the memory traffic differs.  The setter changes the
 * process-wide default; leet_attn_decode_step_v3 takes the policy per call.
 */
typedef enum { LEET_DECODE_STORE_AUTO = 0, LEET_DECODE_STORE_CACHED = 1, LEET_DECODE_STORE_STREAM = 2 } leet_decode_store;
int leet_attn_set_decode_store(int mode);
int leet_attn_get_decode_store(void);

/*
 * Every choice per call.  `kernel` is a leet_bf16_kernel value and `store` a leet_decode_store
 * value, or LEET_CHOICE_DEFAULT for the process-wide setting; everything else as in
 * leet_attn_forward_rd, leet_attn_workspace_bytes_rd, leet_attn_query_plan_rd and
 * leet_attn_decode_step_rd.  A caller that passes the same `kernel` and `segments` to
 * leet_attn_workspace_bytes_v3 and to leet_attn_forward_v3 gets a workspace size that matches
 * the call whatever other threads do with the setters.
 */
#define LEET_CHOICE_DEFAULT (-1)
int leet_attn_forward_v3(const void *q, const void *k, const void *v, const float *gamma, void *out,
                         const float *state_in, float *state_out,
                         void *workspace, size_t workspace_bytes, int segments, int kernel,
                         int B, int H, int N, int r, int dv, int in_dtype, int out_dtype, int mask, void *stream);
size_t leet_attn_workspace_bytes_v3(int B, int H, int N, int r, int dv, int dtype, int segments, int kernel);
int leet_attn_query_plan_v3(int B, int H, int N, int r, int dv, int dtype, int segments, int kernel_choice,
                            int *nseg, int *kernel);
int leet_attn_decode_step_v3(const void *q, const void *k, const void *v, const float *gamma,
                             float *state_inout, float *out, int B, int H, int r, int dv, int dtype, int mask,
                             int store, void *stream);

/*
 * What leet_attn_forward_ex would do for this shape under the current kernel choice (fp32
 * output, decaying mask; the plan depends on neither): *nseg receives the number of segments per
 * sequence, *kernel LEET_KERNEL_WIDE or LEET_KERNEL_COLUMN_SPLIT (fp32 inputs always run WIDE;
 * both 16-bit types have both kernels).  Either pointer may be NULL.  Host-only; touches no device.
 */
int leet_attn_query_plan(int B, int H, int N, int d, int dtype, int segments, int *nseg, int *kernel);
/* The same for rank r and value width dv given separately (shapes as for leet_attn_forward_rd). */
int leet_attn_query_plan_rd(int B, int H, int N, int r, int dv, int dtype, int segments, int *nseg, int *kernel);

/* Static, never-NULL description of a leet_status value. */
const char *leet_attn_strerror(int status);

/* Library version as "major.minor.patch". */
const char *leet_attn_version(void);

#ifdef __cplusplus
}
#endif
#endif /* LEET_ATTN_H */
