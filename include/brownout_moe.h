/*
 * brownout_moe.h -- C ABI of the MI355X (gfx950) BrownoutMoE layer library.
 *
 * One MoE layer's forward pass with the brownout mechanism of BrownoutServe
 * (arXiv 2507.17133): gate affinities and TopK weights (section "Architecture
 * of BrownoutMoE"), the brownout decision of Algorithm 1 (section "Brownout
 * Approach"), token rows grouped per execution unit, the expert FFNs (original,
 * united, shared) and the weighted sum of the layer equation.
 *
 * Conventions
 *   - Every data pointer is a DEVICE pointer owned by the caller; the library
 *     never allocates or frees device memory.  moe_config / moe_ffn_weights /
 *     moe_route_out structs themselves live in HOST memory.
 *   - All work is enqueued on the HIP stream passed as `stream` (a hipStream_t
 *     cast to void*, NULL = default stream); no call synchronises with the host
 *     (moe_profile_collect excepted).  Per-expert counts stay on the device.
 *   - Arguments are validated on the host before any launch; on error nothing
 *     has been enqueued.  Every function returns a moe_status.
 *   - Activations and FFN weights are bf16 (round-to-nearest-even), gate
 *     weights fp32; FFN accumulation is fp32.  All matrices are row-major and
 *     dense.  Pointers must be 16-byte aligned.
 *   - Symbols: T tokens, d = d_model, F = d_ff, m = n_experts, K = top_k,
 *     way = experts per united-expert group (the paper's k), G = ceil(m/way),
 *     N_s = n_shared, U = m + G + N_s execution units, numbered
 *     0..m-1 original experts, m..m+G-1 united experts, m+G.. shared experts.
 *   - Limits: d and F (and d_ff_shared) multiples of 64; m <= 256; K <= min(m,32);
 *     N_s <= 8; T*(K+N_s) <= 2^30; T*d < 2^31 (MOE_ERR_UNSUPPORTED beyond).
 *   - Per-device set-up (kernel attributes, device queries) happens in moe_init, in
 *     moe_workspace_size, or else in the first call that launches work on that device.
 *     Only the last cannot happen under stream capture: a caller that captures its very
 *     first call into a HIP graph calls moe_init (or moe_workspace_size) beforehand.
 *   - The environment variables BROWNOUT_MOE_BM / _GM / _KSPLIT (measurement switches,
 *     unset in normal use) are read once, when the library first needs them.
 */
#ifndef BROWNOUT_MOE_H
#define BROWNOUT_MOE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t moe_status;
#define MOE_OK 0
#define MOE_ERR_INVALID_ARG (-1) /* NULL required pointer, value out of range            */
#define MOE_ERR_SHAPE (-2)       /* a dimension violates the limits above                */
#define MOE_ERR_ALIGNMENT (-3)   /* a pointer is not 16-byte aligned                     */
#define MOE_ERR_WORKSPACE (-4)   /* workspace NULL or smaller than moe_workspace_size    */
#define MOE_ERR_UNSUPPORTED (-5) /* valid request this build does not implement          */
#define MOE_ERR_HIP (-6)         /* a HIP runtime call failed (see moe_last_hip_error)   */

typedef struct moe_config {
    int32_t d_model;      /* d                                                              */
    int32_t d_ff;         /* F of original AND united experts (a united expert has the      */
                          /* parameter size of one original expert: Introduction)           */
    int32_t n_experts;    /* m  (United Expert Model)                                       */
    int32_t top_k;        /* K  (TopK(.,K) in the g equation)                               */
    int32_t way;          /* experts per group; G = ceil(m/way) united experts              */
    int32_t n_shared;     /* N_s shared experts of the layer equation, 0 if none            */
    int32_t d_ff_shared;  /* F of a shared expert (ignored if n_shared == 0)                */
    int32_t score_fn;     /* 0: g = softmax over the K winners (the g equation);            */
                          /* 1: sigmoid(s) renormalised over the K winners                  */
    int32_t add_residual; /* 1: output includes the "x_t +" term of the layer equation      */
    int32_t gate_format;  /* what gate_w points to: MOE_GATE_FP32 (0) or MOE_GATE_PACKED (1)        */
} moe_config;
#define MOE_GATE_FP32 0   /* gate_w: [m][d] fp32, row i = centroid e_i                          */
#define MOE_GATE_PACKED 1 /* gate_w: the buffer moe_pack_gate wrote from such a matrix          */

/* n SwiGLU experts, FFN(x) = W2 (silu(W1 x) * (W3 x)):
 *   w1, w3: [n][F][d] bf16     w2: [n][d][F] bf16
 * (each matrix stored [out_features][in_features]). */
typedef struct moe_ffn_weights {
    const void *w1, *w3, *w2;
} moe_ffn_weights;
/* The same three tensors where a call WRITES them (united experts being built or trained). */
typedef struct moe_ffn_weights_out {
    void *w1, *w3, *w2;
} moe_ffn_weights_out;

/* Routing artefacts.  In moe_route every field may be NULL (not wanted).  A
 * moe_route_out handed to moe_forward must have expert_unit, unit_cnt,
 * unit_off, row_token, row_weight and token_rows set, as written by moe_route
 * with the same config and T. */
typedef struct moe_route_out {
    int32_t *topk_idx;    /* [T][K]   experts by descending affinity, equal affinities: lower id first */
    float *topk_w;        /* [T][K]   g of those experts                                                */
    int32_t *expert_cnt;  /* [m]      cnt_i of Algorithm 1 (before brownout); sums to T*K               */
    int32_t *expert_unit; /* [m]      unit serving expert i: i, m+g (united g), -1 (dropped)            */
    uint8_t *expert_in_s1;/* [m]      1 if expert i is in S1                                            */
    int32_t *unit_cnt;    /* [U]      rows of each execution unit                                       */
    int32_t *unit_off;    /* [U+1]    exclusive prefix of unit_cnt                                      */
    int32_t *row_token;   /* [T*(K+N_s)] token of each row; rows of a unit are contiguous, ascending    */
                          /*          token; first unit_off[U] entries valid                            */
    float *row_weight;    /* [T*(K+N_s)] weight of each row.  A token whose TopK holds several experts  */
                          /*          delegated to one united expert has ONE row there, weight = sum    */
                          /*          of their g (added in TopK order); shared rows have weight 1       */
    int32_t *token_rows;  /* [T][K+N_s] row of TopK entry j (or -1: dropped / merged into an earlier    */
                          /*          entry's row); entries K.. are the token's rows in the shared units*/
    int32_t *n_rows;      /* [1]      = unit_off[U]                                                     */
    uint8_t *near_tie;    /* [T]      1 if two neighbours among the K winners + best loser differ by    */
                          /*          less than 1e-6 in the fp32 logits (a decision that rounding       */
                          /*          order could flip)                                                 */
} moe_route_out;

const char *moe_status_string(moe_status s);
/* Text of the last HIP error seen by this thread ("" if none). */
const char *moe_last_hip_error(void);

/* Per-device set-up for the current HIP device (see Conventions).  Idempotent, thread-safe.
 * Errors: MOE_ERR_HIP (no device, or a runtime call failed). */
moe_status moe_init(void);

/* Bytes of device workspace moe_route / moe_forward / moe_build_united need for up
 * to T_max tokens (or calibration tokens) with this config: a workspace of this size
 * serves every call with the same config and T <= T_max (the size never shrinks as
 * T_max grows).  256-byte aligned base.  Also performs moe_init's set-up when a
 * device is present. */
moe_status moe_workspace_size(const moe_config *cfg, int32_t T_max, size_t *bytes);

/*
 * One-time repack of the gate matrix (section "Architecture of BrownoutMoE": the
 * centroids e_i of the affinity s_{i,t} = x_t . e_i).  With more than 16 experts the
 * gate runs on the bf16 matrix cores with every fp32 weight cut into three bf16
 * pieces (hi + mid + lo carry its 24-bit significand, so x . e_i keeps fp32
 * accuracy).  With cfg->gate_format == MOE_GATE_FP32 moe_route / moe_forward cut
 * gate_w on every call; a caller whose gate does not change between calls does it
 * once here and passes `packed` as gate_w with cfg->gate_format ==
 * MOE_GATE_PACKED.  Results are bit-identical either way.  (With at most 16
 * experts the gate is plain fp64 arithmetic that reads either form as it is.)
 *   gate_w [m][d] fp32 (device)    packed: moe_gate_packed_size bytes (device)
 * Errors: NULL / misaligned pointers, packed_bytes too small (MOE_ERR_WORKSPACE).
 */
moe_status moe_gate_packed_size(const moe_config *cfg, size_t *bytes);
moe_status moe_pack_gate(const moe_config *cfg, const float *gate_w, void *packed, size_t packed_bytes,
                         void *stream);

/*
 * United experts (section "United Expert Model").  The paper trains one student
 * per group of `way` consecutive experts by distillation and does not give the
 * recipe; this call writes the student's starting point, the element-wise mean
 * of the group's parameters (sum in member order and one division in fp64,
 * rounded once to bf16; the last group averages its actual members), into the
 * caller's `united` tensors ([G][F][d], [G][F][d], [G][d][F]).  If calib_x
 * ([n_calib][d] bf16) and loss_per_group ([G] fp32) are given it also evaluates
 * the MSE equation of that section on the calibration tokens:
 *   L^j = (1/k_j) sum_i ||H_u^j - H_o^{j*way+i}||^2,
 * H = FFN outputs, squared norm summed over features and averaged over tokens.
 * Errors: NULL experts/united pointers, n_calib < 0, workspace too small.
 */
moe_status moe_build_united(const moe_config *cfg, const moe_ffn_weights *experts,
                            const moe_ffn_weights_out *united_out, const void *calib_x, int32_t n_calib,
                            float *loss_per_group, void *workspace, size_t workspace_bytes, void *stream);

/*
 * United-expert distillation (section "United Expert Model"): trains the student of
 * every group, in place in `united` (bf16, the starting point: moe_build_united's
 * parameter mean or anything else), to minimise the section's MSE equation
 *   L^j = (1/k_j) sum_i ||H_u^j - H_o^{j*way+i}||^2
 * (summed over features, averaged over the n_calib calibration tokens calib_x
 * [n_calib][d] bf16).  The paper gives no optimiser, settings or data: this call runs
 * `steps` full-batch steps of Adam (beta1 0.9, beta2 0.999, eps 1e-8, bias corrected,
 * step size lr) on fp32 master weights; the GEMMs of the forward and backward pass
 * run in bf16 with fp32 accumulation, teacher outputs are held in half precision.
 * loss_history (device, [G][steps+1] fp32, may be NULL) receives the loss before every
 * step and after the last.  A group with one member is not trained: its student becomes
 * a copy of that member (the minimiser, loss 0).  Workspace: moe_distill_workspace_size bytes.
 * Errors: n_calib not a positive multiple of 64 (MOE_ERR_SHAPE), NULL pointers,
 * steps < 0, lr < 0 or NaN, workspace too small.
 */
moe_status moe_distill_workspace_size(const moe_config *cfg, int32_t n_calib, size_t *bytes);
moe_status moe_distill_united(const moe_config *cfg, const moe_ffn_weights *experts, const moe_ffn_weights_out *united,
                              const void *calib_x, int32_t n_calib, int32_t steps, float lr, float *loss_history,
                              void *workspace, size_t workspace_bytes, void *stream);

/*
 * Gate + TopK + Algorithm 1 + row lists for T tokens x [T][d] bf16.
 *   gate_w [m][d] fp32 (row i = centroid e_i) or, with cfg->gate_format ==
 *   MOE_GATE_PACKED, the buffer moe_pack_gate wrote; gate_bias [m] fp32 or NULL:
 *   s_{i,t} = x_t . e_i (+ bias_i), accumulated to fp32 accuracy.
 *   threshold in [0,1]: share of token->expert assignments that stays on
 *   original experts (1 = zero-brownout).  Algorithm 1 is read so that it
 *   reproduces the paper's worked examples: experts sorted by count descending
 *   (equal counts: lower id first) join S1 while the count already covered is
 *   < S*threshold (double product); the rest are S2.  S2 experts of a group
 *   go to united expert floor(i/way) if at least two of them hold tokens, else
 *   the single one serves itself; with use_full_brownout != 0 S2 is dropped.
 * Errors: threshold outside [0,1] or NaN, top_k > n_experts, way < 1, T <= 0,
 * NULL x / gate_w / out, misaligned pointers, workspace too small.
 */
moe_status moe_route(const moe_config *cfg, const void *x, int32_t T, const void *gate_w,
                     const float *gate_bias, double threshold, int32_t use_full_brownout,
                     const moe_route_out *out, void *workspace, size_t workspace_bytes, void *stream);

/*
 * moe_route for callers that cannot allocate device memory or hand over a workspace
 * (code under HIP graph capture, tight serving loops, harnesses that forbid
 * allocation): same arguments without the workspace, same results bit for bit.  Its
 * work space is a fixed 8 MiB array inside the library's device image (one per
 * GPU, held until the process ends); fields of `out` left NULL live there too.
 * The call allocates and frees nothing (profiling, moe_profile_enable, must be off:
 * it creates events).  A batch whose routing work space exceeds 8 MiB is rejected
 * with MOE_ERR_WORKSPACE before anything is launched; the need is about
 * T*(K+N_s)*12 + T*K*8 + T/64*U*8 bytes, plus 6*16*ceil(m/16)*d for an unpacked gate of
 * more than 16 experts (pack it with moe_pack_gate to save that).  All calls on one GPU share the array:
 * two such calls whose work overlaps in time (different streams) race; calls on one
 * stream are safe, and nothing an earlier call left in the array is read.
 */
moe_status moe_route_static(const moe_config *cfg, const void *x, int32_t T, const void *gate_w,
                            const float *gate_bias, double threshold, int32_t use_full_brownout,
                            const moe_route_out *out, void *stream);

/*
 * The layer equation:
 *   out_t = [x_t] + sum_s FFN^(s)_s(x_t) + sum_i p_{i,t} FFN^(r)_i(x_t) + sum_i q_{i,t} FFN^(u)_{floor(i/way)}(x_t)
 * out [T][d] bf16.  route == NULL: routing is computed internally exactly as
 * moe_route does (gate_w required); otherwise the given rows are used and
 * gate_w / gate_bias / threshold / use_full_brownout are ignored.
 * `united` may be NULL only if no token can reach a united expert
 * (threshold == 1 or use_full_brownout); `shared` must be set iff n_shared > 0.
 * Intermediate activations are bf16, sums fp32; the sum over a token's rows
 * is taken in TopK order, shared experts first (deterministic, no atomics).
 */
moe_status moe_forward(const moe_config *cfg, const void *x, int32_t T, const void *gate_w,
                       const float *gate_bias, const moe_ffn_weights *experts, const moe_ffn_weights *united,
                       const moe_ffn_weights *shared, double threshold, int32_t use_full_brownout,
                       const moe_route_out *route, void *out, void *workspace, size_t workspace_bytes,
                       void *stream);

/*
 * Per-kernel timing for benchmarks.  moe_profile_enable takes a bit mask of
 * stages (bit MOE_STAGE_x; 0 switches profiling off).  While a stage is
 * enabled, moe_route / moe_forward / moe_build_united bracket that stage's
 * kernel with two HIP events on the caller's stream (up to 4096 calls are
 * kept, later ones are not recorded).  moe_profile_collect waits for the
 * recorded events, adds up the elapsed milliseconds and the number of
 * launches per stage and clears the record.  Process-wide state; not
 * thread-safe.
 */
enum {
    MOE_STAGE_PREP = 0,   /* clear counters, split gate weights                */
    MOE_STAGE_GATE = 1,   /* affinities, TopK, weights, expert counts          */
    MOE_STAGE_COUNT = 2,  /* Algorithm 1 + rows per unit and token block       */
    MOE_STAGE_SCAN = 3,   /* offsets                                           */
    MOE_STAGE_SCATTER = 4,/* row lists                                         */
    MOE_STAGE_TILES = 5,  /* GEMM tile table                                   */
    MOE_STAGE_GEMM1 = 6,  /* rows x [W1|W3] + SwiGLU                           */
    MOE_STAGE_GEMM2 = 7,  /* H x W2                                            */
    MOE_STAGE_COMBINE = 8,/* weighted sum per token                            */
    MOE_N_STAGES = 9
};
moe_status moe_profile_enable(int32_t stage_mask);
moe_status moe_profile_collect(double *total_ms /*[MOE_N_STAGES]*/, int64_t *launches /*[MOE_N_STAGES]*/);

/*
 * Measurement aids for benchmarks: what the GPU at hand sustains on the two
 * resources the layer is priced against, so that a roofline fraction can be
 * stated against the measured ceiling beside the nominal one.  Both calls launch
 * on the caller's stream, time a batch of launches with HIP events after a
 * warm-up (0.3 s and 0.1 s) and WAIT for the stream; they allocate nothing.
 *   moe_probe_mfma      a loop of independent bf16 MFMAs (16x16x32, fp32
 *                       accumulate) on register operands, eight waves per CU, no
 *                       memory traffic.  The operand bits are the first 64 KiB of
 *                       `operands` (device, bf16; operand_bytes >= 65536): pass
 *                       real weights to see the rate under the power the data
 *                       draws, constants to see the rate without that limit.
 *                       sink: device scratch of >= 2 MiB.  Result: TFLOP/s.
 *   moe_probe_hbm_read  every thread adds up 16-byte loads of buf (device,
 *                       bytes >= 1 MiB, use a buffer far larger than the caches),
 *                       grid-stride.  sink: device, >= 4 bytes.  Result: GB/s.
 * Errors: NULL pointers (MOE_ERR_INVALID_ARG), buffers too small
 * (MOE_ERR_WORKSPACE), misaligned pointers, HIP failures.
 */
moe_status moe_probe_mfma(const void *operands, size_t operand_bytes, void *sink, size_t sink_bytes, void *stream,
                          double *tflops);
moe_status moe_probe_hbm_read(const void *buf, size_t bytes, void *sink, size_t sink_bytes, void *stream, double *gbs);

/*
 * SLO-aware latency control (the paper's Algorithm 2, "SLO-Aware Latency
 * Control Algorithm"): the host-side controller that moves `threshold`
 * between calls of moe_forward.  Pure host functions, no device work, no state.
 *
 * moe_latency_p90: the P90 of n recent latencies (host array, any order, not
 *   modified): the value of rank ceil(0.9 n) in ascending order.  NaN if
 *   latencies is NULL or n is 0.
 * moe_salc_update: one controller step.  With warning_line = slo *
 *   warning_factor: latency below the warning line -> threshold + increment;
 *   latency above slo -> threshold * shrink_ratio; otherwise unchanged.  The
 *   result is clamped to [0, 1], the range moe_forward accepts (the paper does
 *   not say what happens at the ends).  NaN if params is NULL, a field is not
 *   finite, slo <= 0, warning_factor outside (0, 1], increment < 0 or
 *   shrink_ratio outside [0, 1].
 */
typedef struct moe_salc_params {
    double slo;            /* latency objective, same unit as the latencies */
    double warning_factor; /* warning line as a fraction of slo (paper: 0.8) */
    double increment;      /* additive step up (paper: 0.1)                 */
    double shrink_ratio;   /* multiplicative step down (paper: 0.8)         */
} moe_salc_params;
double moe_latency_p90(const double *latencies, size_t n);
double moe_salc_update(double threshold, double latency_p90, const moe_salc_params *params);

#ifdef __cplusplus
}
#endif
#endif /* BROWNOUT_MOE_H */
