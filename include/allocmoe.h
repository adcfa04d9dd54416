/*
 * allocmoe.h — C ABI of the budget-constrained MoE layer forward of Alloc-MoE
 * for one AMD MI355X (gfx950).
 *
 * One call of allocmoe_moe_forward computes, for the T tokens of one MoE layer,
 *   1. routing scores  s[t,:] = Softmax(x_t W_gate)            (Section 3.1, Eq. (1))
 *   2. the candidate set: each token's Top-K_orig scores, sorted descending
 *                                                              (Section 3.3, Eq. (6))
 *   3. Alloc-T: keep every token's Top-K_base, then the globally largest
 *      B - T*K_base of the remaining candidates of the whole batch
 *                                  (Section 3.3, Eqs. (7)-(9) and the procedure after them)
 *   4. an expert-sorted dispatch of the selected (token, expert) pairs
 *   5. the SwiGLU expert networks over only the selected pairs, plus the
 *      always-on shared expert of the workload                 (Section 3.1: a
 *      feed-forward execution per activation)
 *   6. y_t = sum_i w_{t,i} E_i(x_t), w = retained score or 0   (Section 3.1, Eq. (2))
 * The per-layer budget B is an input: it is what Alloc-L's offline dynamic
 * programme (Section 3.2, Eqs. (3)-(5)) hands to the layer, as T*K_l.
 *
 * Conventions for every entry point
 *   - Pointers named in a comment as "device" are device (HBM) addresses owned
 *     by the caller; the library allocates nothing, frees nothing and keeps no
 *     pointer after a call returns.  Descriptor structs are host memory.
 *   - All matrices are dense row-major.  X [T,d]; W_gate [d,E]; expert e:
 *     W1[e], W3[e] are [d,I], W2[e] is [I,d], E_e(x) = (silu(x W1) * (x W3)) W2;
 *     shared expert Ws1, Ws3 [d,I_shared], Ws2 [I_shared,d].
 *   - Work is enqueued on the given stream (a hipStream_t passed as void*, NULL
 *     = the null stream); no call synchronises with the host or copies to it.
 *   - Arguments are validated on the host before anything is enqueued; on an
 *     error nothing was launched and outputs are untouched.  Return value: an
 *     allocmoe_status; the library never aborts or throws across this boundary.
 *   - Same inputs give bit-identical outputs from run to run (no atomics on
 *     floating-point data, fixed summation orders).
 *   - Scores, routing weights and all accumulation are fp32 whatever `dtype`.
 *   - Ties (equal scores) go to the lower expert id inside a token and to the
 *     lower token, then lower rank, across the batch.  NaN scores are not
 *     supported.
 */
#ifndef ALLOCMOE_H
#define ALLOCMOE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef void *allocmoe_stream; /* hipStream_t */

typedef enum {
    ALLOCMOE_OK = 0,
    ALLOCMOE_EINVAL = -1,     /* null pointer, bad enum, K_base > K, K > E, ...         */
    ALLOCMOE_EBUDGET = -2,    /* budget < T*K_base (Eq. (9) infeasible) or > T*K        */
    ALLOCMOE_ESHAPE = -3,     /* a size outside what the kernels support (see desc)     */
    ALLOCMOE_EWORKSPACE = -4, /* workspace / packed buffer too small or misaligned      */
    ALLOCMOE_EHIP = -5        /* a HIP runtime call (kernel launch) reported an error   */
} allocmoe_status;

typedef enum { ALLOCMOE_F32 = 0, ALLOCMOE_BF16 = 1 } allocmoe_dtype;

/* One layer call.  Supported sizes: 1 <= T, T*K < 2^31; 1 <= E <= 64;
 * 1 <= K <= min(E,16); 0 <= K_base <= K; d, I >= 1.  With dtype BF16
 * additionally d, I and I_shared must be multiples of 64. */
typedef struct {
    int32_t T, d, E, I;   /* tokens, hidden size H, routed experts N, expert width      */
    int32_t K, K_base;    /* K_orig candidates per token; guaranteed minimum per token  */
    int64_t budget;       /* B = T*K_l routed activations, T*K_base <= B <= T*K          */
    int32_t I_shared;     /* 0 = no shared expert; else its (fused) intermediate width  */
    int32_t shared_gate;  /* 0: y += Shared(x);  1: y += sigmoid(x . w_sg) * Shared(x)  */
    int32_t dtype;        /* allocmoe_dtype of X, Y and every weight matrix             */
    int32_t flags;        /* allocmoe_selector | optional ALLOCMOE_WEIGHTS_FP8; rest 0  */
} allocmoe_layer_desc;

/* Token-level selector (desc->flags).  All of them keep every token's first K_base
 * candidates and then the B - T*K_base pool entries with the largest key (ties: lower
 * token, then lower rank), i.e. they spend exactly the layer budget; they differ in
 * the key of candidate j of token t (formed in fp32, non-increasing along the sorted
 * row, so a token's kept candidates are a prefix):
 *   SCORE    s[t,j]                              Alloc-T (Section 3.3)
 *   TOP_P    -(s[t,0] + ... + s[t,j-1])          Top-P routing (Dynamic-MoE baseline,
 *            Appendix A.1): kept while the mass before j is below p, the threshold p
 *            being the one that meets the budget on this batch
 *   RELATIVE s[t,j] / s[t,0] (0 if s[t,0] <= 0)  expert skipping relative to the Top-1
 *            score (NAEE baseline extended to Top-K, Appendix A.1): kept iff >= beta,
 *            beta being the one that meets the budget on this batch
 * Uniform Top-K_l is SCORE with K_base = K_l and budget = T*K_l.  TOP_P and RELATIVE
 * need T*K*4 bytes of device scratch in the calls that take `ws`. */
typedef enum {
    ALLOCMOE_SELECT_SCORE = 0,
    ALLOCMOE_SELECT_TOP_P = 1,
    ALLOCMOE_SELECT_RELATIVE = 2
} allocmoe_selector;

/* Expert-weight format flag, OR-ed into desc->flags (dtype BF16 only; d, I and I_shared
 * multiples of 128).  The paper treats weight quantisation as orthogonal to budget
 * allocation (Section 6); this is the variant for the weight-bound regimes (decode,
 * small budgets), where the layer's time is the bytes of the active experts' weights.
 * allocmoe_pack_weights then stores every expert matrix W[k][n] (routed and shared; the
 * gate stays bf16) as one byte per element plus one fp32 scale per output column n:
 *     scale[n] = max_k |W[k][n]| / 448          (fp32; 1 if the column is all zero)
 *     q[k][n]  = the E4M3 code (OCP 8-bit floating point: 1 sign, 4 exponent bits with
 *                bias 7, 3 mantissa bits, subnormals, no infinities, largest finite
 *                magnitude 448) nearest to W[k][n] / scale[n] (fp32 division), ties to
 *                the even mantissa, larger magnitudes saturating to 448
 * standing for decode(q[k][n]) * scale[n].  The expert networks widen the codes to bf16
 * in registers (exact), multiply on the bf16 matrix cores with fp32 accumulation and
 * multiply the sum by the column's scale (both expert-network kernels read either
 * format; the kernel choice does not depend on it).  Packed buffer (byte offsets, each region 256-byte aligned, in this order):
 * codes of W1|W3 [E], of W2 [E], of Ws1|Ws3, of Ws2 (same element order as the bf16
 * buffer, a fragment of 32 k x 32 columns being 64 lanes x 16 bytes: lane l holds
 * k = 32 kb + 8 (l/32) + i in byte i and k = 32 kb + 16 + 8 (l/32) + i in byte 8 + i,
 * i = 0..7, column 32 nb + l%32; per expert and column block the W1 fragments along k,
 * then the W3 fragments), the re-tiled bf16 gate, then the scales fp32 [E][2][I]
 * (W1, W3), [E][d] (W2), [2][I_shared], [d]. */
#define ALLOCMOE_WEIGHTS_FP8 0x100

/* Weights, all device pointers, read-only.  gate_bias (fp32 [E], added to the
 * logits before the softmax) and the shared-expert fields may be NULL.
 * `packed` is the buffer written by allocmoe_pack_weights; with dtype BF16 the
 * expert networks read only `packed` (W1..Ws2 may then be NULL), with dtype F32
 * they read the row-major matrices and `packed` is ignored. */
typedef struct {
    const void *Wg;         /* [d,E]                                  */
    const float *gate_bias; /* [E] or NULL                            */
    const void *W1, *W3;    /* [E,d,I]                                */
    const void *W2;         /* [E,I,d]                                */
    const void *Ws1, *Ws3;  /* [d,I_shared] or NULL                   */
    const void *Ws2;        /* [I_shared,d] or NULL                   */
    const void *w_sg;       /* [d] or NULL (needed iff shared_gate)   */
    const void *packed;     /* allocmoe_packed_bytes() bytes or NULL  */
} allocmoe_weights;

/* Byte offsets, inside the workspace of allocmoe_moe_forward, of the
 * intermediates it leaves behind (for inspection and tests).  Types and shapes:
 * scores f32 [T,E]; topk_ids i32 [T,K]; topk_s f32 [T,K]; keep_count i32 [T];
 * shared_gate f32 [T]; expert_offsets i32 [E+1]; row_token, row_rank i32 [B];
 * inv_row i32 [T,K]; H dtype [B,I]; Hs dtype [T,I_shared]; O dtype [B,d];
 * Os dtype [T,d] (the experts' outputs are kept in the layer's dtype; Eq. (2)'s
 * weighted sum over them is formed in fp32). */
typedef struct {
    size_t scores, topk_ids, topk_s, keep_count, shared_gate;
    size_t expert_offsets, row_token, row_rank, inv_row;
    size_t H, Hs, O, Os;
    size_t scratch; /* selection/dispatch scratch and tile map */
    size_t sel_keys; /* f32 [T,K] selector keys (TOP_P / RELATIVE only)                  */
    size_t total;   /* == allocmoe_workspace_bytes                                      */
} allocmoe_ws_layout;

/* Size in bytes of the workspace allocmoe_moe_forward needs for this
 * descriptor.  The workspace is device memory, 256-byte aligned, contents
 * undefined on entry, reusable across calls on the same stream.
 * allocmoe_dispatch uses only its first allocmoe_ws_layout.scores bytes (the
 * scratch region, which starts the workspace).  allocmoe_route and
 * allocmoe_route_from_scores need none (ws may be NULL: one workgroup then does the
 * selection, whatever T); given a workspace of at least allocmoe_ws_layout.scores
 * bytes they spread the selection over many workgroups from 4096 tokens on (same
 * result, bit for bit). */
allocmoe_status allocmoe_workspace_bytes(const allocmoe_layer_desc *desc, size_t *bytes);
allocmoe_status allocmoe_workspace_layout(const allocmoe_layer_desc *desc,
                                          allocmoe_ws_layout *layout);

/* One-time re-tiling of the static expert weights (bf16 only) into the
 * fragment order the matrix-core kernels stream: same bytes, same values, a
 * different order.  `canonical` holds the row-major device matrices (W1, W3,
 * W2 and, if I_shared > 0, Ws1, Ws3, Ws2); `packed` is a device buffer of
 * packed_bytes >= allocmoe_packed_bytes(), 256-byte aligned.  Not part of the
 * per-batch path: call once per layer at load time. */
allocmoe_status allocmoe_packed_bytes(const allocmoe_layer_desc *desc, size_t *bytes);
allocmoe_status allocmoe_pack_weights(const allocmoe_layer_desc *desc,
                                      const allocmoe_weights *canonical, void *packed,
                                      size_t packed_bytes, allocmoe_stream stream);

/* Steps 1-3.  X: device [T,d] of desc->dtype; reads w->Wg, w->gate_bias.
 * Outputs (device): scores f32 [T,E] (may be NULL), topk_ids i32 [T,K] and
 * topk_s f32 [T,K] (each token's K largest scores, descending, ties by lower
 * expert id), keep_count i32 [T]: token t keeps ranks 0..keep_count[t]-1, with
 * K_base <= keep_count[t] <= K and sum_t keep_count[t] == budget. */
allocmoe_status allocmoe_route(const allocmoe_layer_desc *desc, const void *X,
                               const allocmoe_weights *w, float *scores, int32_t *topk_ids,
                               float *topk_s, int32_t *keep_count, void *ws, size_t ws_bytes,
                               allocmoe_stream stream);

/* Steps 2-3 from caller-supplied scores (device f32 [T,E], finite): the entry
 * point whose integer outputs are bit-exact functions of its input.  Uses T, E,
 * K, K_base, budget of the descriptor. */
allocmoe_status allocmoe_route_from_scores(const allocmoe_layer_desc *desc, const float *scores,
                                           int32_t *topk_ids, float *topk_s,
                                           int32_t *keep_count, void *ws, size_t ws_bytes,
                                           allocmoe_stream stream);

/* Step 4.  From topk_ids [T,K] and keep_count [T] (device) build the rows of
 * the selected pairs ordered by (expert ascending, token ascending):
 * expert_offsets i32 [E+1] (rows of expert e are offsets[e]..offsets[e+1]),
 * row_token / row_rank i32 [budget] (the pair behind each row), inv_row i32
 * [T,K] (row of pair (t,j), -1 if not kept).  sum_t keep_count[t] must equal
 * desc->budget (it lives on the device and is not checked on the host).  If it is
 * larger, nothing is written past the budget: pairs whose row would be >= budget get
 * inv_row -1 and no row, and every expert_offsets entry is capped at budget. */
allocmoe_status allocmoe_dispatch(const allocmoe_layer_desc *desc, const int32_t *topk_ids,
                                  const int32_t *keep_count, int32_t *expert_offsets,
                                  int32_t *row_token, int32_t *row_rank, int32_t *inv_row,
                                  void *ws, size_t ws_bytes, allocmoe_stream stream);

/* Steps 1-6.  X device [T,d], Y device [T,d], both desc->dtype (with BF16: both
 * 16-byte aligned, else ALLOCMOE_EINVAL).  The
 * intermediates stay in the workspace at the offsets of
 * allocmoe_workspace_layout.  All work is ordered after what `stream` holds at
 * the call and before what is enqueued on it afterwards.  For prefill-shaped
 * calls with a shared expert the library runs that expert's GEMMs on a
 * stream of its own (one extra stream and two events per device, created on
 * first use, default priority) beside the selection; both ends are tied to
 * `stream` with events, no host synchronisation.  Calls on one device from
 * several host threads are serialised by a per-device lock for the duration of
 * the enqueue (they share that stream and its events).  The call only enqueues kernels
 * and those two events (no allocation, no memset, no host wait), so it may be
 * captured into a HIP graph and replayed; make the first call on a device outside
 * a capture (it creates the side stream). */
allocmoe_status allocmoe_moe_forward(const allocmoe_layer_desc *desc, const void *X,
                                     const allocmoe_weights *w, void *Y, void *ws,
                                     size_t ws_bytes, allocmoe_stream stream);

/* Intervals reported by allocmoe_moe_forward_timed (indices into stage_ms). */
typedef enum {
    ALLOCMOE_STAGE_ROUTE = 0,   /* steps 1-2: gate, softmax, sorted candidates              */
    ALLOCMOE_STAGE_PLAN = 1,    /* steps 3-4: Alloc-T selection, dispatch, tile map          */
    ALLOCMOE_STAGE_FFN1 = 2,    /* step 5 on `stream`: H = silu(x W1) * (x W3); the selected */
                                /* rows, and the shared expert where it shares the launch    */
    ALLOCMOE_STAGE_FFN2 = 3,    /* step 5 on `stream`: O = H W2; then the wait for the       */
                                /* library's own stream, if it was used                      */
    ALLOCMOE_STAGE_COMBINE = 4, /* step 6: Eq. (2)                                           */
    ALLOCMOE_STAGE_SHARED_FFN1 = 5, /* the shared expert's first GEMM on the library's stream */
    ALLOCMOE_STAGE_SHARED_FFN2 = 6, /* its second GEMM there (both 0 if that stream was idle) */
    ALLOCMOE_STAGE_EXPERT_SPAN = 7, /* start of PLAN to start of COMBINE: the region in which */
                                /* every expert GEMM of the layer runs, on either stream     */
    ALLOCMOE_STAGE_TOTAL = 8,   /* start of ROUTE to the end of COMBINE                      */
    ALLOCMOE_N_STAGES = 9
} allocmoe_stage;

/* Measurement variant of allocmoe_moe_forward: the same kernels in the same launch
 * structure (the shared expert on the library's own stream where allocmoe_moe_forward
 * puts it there), with a HIP event recorded on the stream concerned around every
 * launch; the call then WAITS for the last events (the one exception to the
 * no-synchronisation rule) and writes the durations in milliseconds to
 * stage_ms[ALLOCMOE_N_STAGES] (host memory).  Intervals of kernels that run beside each
 * other on the two streams overlap in time: EXPERT_SPAN is the wall-clock figure for
 * them.  The events are host objects the library creates per device on first use and
 * keeps.  For benchmarking. */
allocmoe_status allocmoe_moe_forward_timed(const allocmoe_layer_desc *desc, const void *X,
                                           const allocmoe_weights *w, void *Y, void *ws,
                                           size_t ws_bytes, allocmoe_stream stream,
                                           float *stage_ms);

/* Ceiling probes (measurement utilities, not on the layer's path; both WAIT for their
 * kernels and copy a few bytes back).  The rooflines of the layer's kernels are quoted
 * against the published peaks; these re-measure what the device at hand sustains.
 *
 * allocmoe_probe_mfma: the matrix-core instruction the expert GEMMs use
 * (32x32x16 bf16, fp32 accumulate) issued back to back on eight independent
 * accumulators per wave, `waves_per_simd` (1 or 2) waves on every SIMD of every compute
 * unit (a grid of 256 workgroups), `iters` passes of 8 instructions.  The operand
 * fragments come from `operands` (device, allocmoe_probe_mfma_operand_bytes() bytes of
 * bf16, 16-byte aligned, filled by the caller: zeros or random values - the clock the
 * device sustains, and so the rate, depends on the data).  Writes the achieved TFLOP/s
 * and the shader clock in MHz (core-clock counter against the constant 100 MHz counter
 * around the loop).  sink: device scratch of allocmoe_probe_sink_bytes() bytes.
 *
 * allocmoe_probe_hbm_read: reads `bytes` (a multiple of 256 KiB is used) of `buf` with
 * 16-byte loads per lane, eight in flight, `repeats` times, with (1) or without (0) the
 * non-temporal hint; writes the achieved GB/s.  Use a buffer much larger than the
 * 256 MiB memory-side cache. */
size_t allocmoe_probe_mfma_operand_bytes(void);
size_t allocmoe_probe_sink_bytes(void);
allocmoe_status allocmoe_probe_mfma(const void *operands, size_t operand_bytes,
                                    int waves_per_simd, int iters, void *sink, size_t sink_bytes,
                                    float *tflops, float *shader_mhz, allocmoe_stream stream);
allocmoe_status allocmoe_probe_hbm_read(const void *buf, size_t bytes, int nontemporal,
                                        int repeats, void *sink, size_t sink_bytes,
                                        float *gbytes_per_s, allocmoe_stream stream);

/* Summary numbers of allocmoe_routing_stats (device memory, 5 floats in this order). */
typedef struct {
    float spearman_load;   /* Spearman rank correlation of the per-expert loads, original vs budgeted */
    float entropy_orig;    /* normalised entropy of the score-weighted load distribution, original */
    float entropy_kept;    /* the same under the budgeted routing                                    */
    float js_divergence;   /* Jensen-Shannon divergence between the two distributions (nats)         */
    float spearman_tokens; /* Spearman correlation: token routing entropy vs experts kept            */
} allocmoe_routing_metrics;

/* Routing analytics of one layer (Section 5, "Analysis of Expert Load Balance" and
 * "Analysis of Budget Allocation in Alloc-L and Alloc-T"), from a routing result as
 * allocmoe_route leaves it: scores f32 [T,E], topk_ids i32 [T,K], topk_s f32 [T,K],
 * keep_count i32 [T] (all device).  "Original" routing = all K candidates of every
 * token, budgeted = the first keep_count[t].  Outputs (device): load_orig, load_kept
 * i32 [E] (pairs per expert), wload_orig, wload_kept f32 [E] (sum of their routing
 * scores), token_entropy f32 [T] (H_t = -sum_e s ln s over all E experts), metrics.
 * Entropies are normalised by ln E, logarithms are natural, rank correlations use
 * average ranks for ties and are 0 when one side is constant (the paper names the
 * statistics only).  ws: device scratch of at least 4*T bytes, 256-byte aligned.
 * Deterministic: no floating-point atomics; the rank correlations come from exact
 * integer sums.  Only desc->T, E, K are used (after the usual validation). */
allocmoe_status allocmoe_routing_stats(const allocmoe_layer_desc *desc, const float *scores,
                                       const int32_t *topk_ids, const float *topk_s,
                                       const int32_t *keep_count, int32_t *load_orig,
                                       int32_t *load_kept, float *wload_orig, float *wload_kept,
                                       float *token_entropy, allocmoe_routing_metrics *metrics,
                                       void *ws, size_t ws_bytes, allocmoe_stream stream);

/* Alloc-L's layer-wise allocation (Section 3.2, Eqs. (3)-(5)), the offline step that
 * produces the per-layer budgets: given the sensitivity matrix S [L, K_orig] (host,
 * row-major, S[i*K_orig + k-1] = loss of layer i with k experts per token) and the
 * global budget B (expert activations per token summed over the layers), writes to
 * K_out[L] (host) the allocation 1 <= K_i <= K_orig with sum K_i <= B that minimises
 * sum_i S[i][K_i] (summed in fp64 in layer order), found exactly by the grouped-knapsack
 * dynamic programme of Eq. (5) with backtracking, O(L * B * K_orig).  Of several
 * minimisers: the one that spends less, then the one with the smaller K at the deepest
 * layer, then at the layer before, and so on.  cost_out (host, may be NULL) receives the
 * minimum.  A layer call then takes budget = T * K_i.  Host-only: touches no device,
 * uses host heap for the table.  Errors: B < L -> ALLOCMOE_EBUDGET; NaN in S, L < 1,
 * K_orig < 1 -> ALLOCMOE_EINVAL; L * K_orig > 2^24 -> ALLOCMOE_ESHAPE. */
allocmoe_status allocmoe_alloc_l(const double *S, int32_t L, int32_t K_orig, int64_t B,
                                 int32_t *K_out, double *cost_out);

/* The heuristic layer-level schedules Alloc-L is compared with (appendix
 * "Implementation Details of Baselines", layer-level baseline).  Ascending: an integer
 * vector by rounded (halves up) linear interpolation from K_min at the first layer to
 * K_max at the last, made non-decreasing with steps of at most one by a forward and a
 * backward pass, then moved to the exact total B by sweeps over the internal layers
 * (shallow to deep, one unit per layer and sweep, only where the vector stays
 * non-decreasing, inside [K_min, K_max] and with steps of at most one).  K_min = 1 and
 * K_max = K_orig; a B above their reach raises K_min, a B below it lowers K_max, until
 * B fits.  Descending: the same vector in reverse layer order.  Writes K_out[L] (host)
 * with sum K_i == B exactly, 1 <= K_i <= K_orig.  A single layer gets K = B.  Host-only.
 * Errors: B < L or B > L * K_orig -> ALLOCMOE_EBUDGET; L < 1, K_orig < 1, unknown kind,
 * K_out NULL -> ALLOCMOE_EINVAL. */
typedef enum allocmoe_schedule {
    ALLOCMOE_SCHEDULE_ASCENDING = 0,
    ALLOCMOE_SCHEDULE_DESCENDING = 1
} allocmoe_schedule;
allocmoe_status allocmoe_layer_schedule(allocmoe_schedule kind, int32_t L, int32_t K_orig,
                                        int64_t B, int32_t *K_out);

/* allocmoe_dispatch for callers that cannot allocate device memory or pass a workspace
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc):
 * the same kernels and the same outputs, but the scratch (ballot words and prefixes,
 * 768 bytes per 64 tokens) lives in a buffer of ALLOCMOE_STATIC_SCRATCH_BYTES that is
 * part of the library's device image (every GPU the library runs on holds its own copy
 * until the process ends).  Sizes beyond ALLOCMOE_STATIC_MAX_TOKENS tokens are rejected
 * with ALLOCMOE_ESHAPE.  Allocates nothing, frees nothing and calls no allocating
 * routine.  Every call on a GPU shares that GPU's buffer (nothing in it has to start at
 * zero: each call writes what it reads), so calls that overlap in time on one GPU (two
 * streams, two threads) race; calls on one stream are ordered and safe. */
#define ALLOCMOE_STATIC_MAX_TOKENS 65536
#define ALLOCMOE_STATIC_SCRATCH_BYTES (ALLOCMOE_STATIC_MAX_TOKENS / 64 * 768)
allocmoe_status allocmoe_dispatch_static(const allocmoe_layer_desc *desc, const int32_t *topk_ids,
                                         const int32_t *keep_count, int32_t *expert_offsets,
                                         int32_t *row_token, int32_t *row_rank, int32_t *inv_row,
                                         allocmoe_stream stream);

const char *allocmoe_status_string(allocmoe_status status);

#ifdef __cplusplus
}
#endif
#endif /* ALLOCMOE_H */
