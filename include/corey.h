/*
 * corey.h -- C ABI of libcorey: the COREY hot path on one AMD MI355X (gfx950).
 *
 * Three operations, named after the paper's statement of the problem (its inline scheduling hook runs
 * them in this order on every Mamba layer: statistic of the post-convolution tensor u -> chunk -> scan
 * with that chunk, "Active-Mode Overhead Budget", steps (2)-(4)):
 *
 *   corey_entropy_hist   fixed-bin histogram of a tensor, its Shannon entropy H (Eq. 1) and the
 *                        normalised signal r = H / log K (Method, Preliminaries).
 *   corey_select_chunk   the entropy-to-chunk rule (Eq. 2) and the scheduler family around it
 *                        (sequence-length table, guarded fallback, static chunk).
 *   selective_scan_fwd   the Mamba-1 selective-scan forward with a run-time chunk (the
 *                        recurrence-preserving runtime-chunk scan of "End-to-End Routed Inference").
 *
 * Conventions common to all calls
 *   - Plain C: no C++ types, no exceptions cross the boundary.  Every function returns a corey_status;
 *     0 is success.  corey_last_error() gives a thread-local message for the last failure.
 *   - Pointers marked DEVICE point to GPU global memory owned by the caller; HOST pointers to ordinary
 *     memory.  The library never frees or keeps caller memory and allocates nothing itself.
 *   - GPU work is enqueued on the HIP stream passed as `hip_stream` (a hipStream_t cast to void*; NULL is
 *     the default stream) and the call returns without synchronising.  Argument errors are detected on
 *     the host before anything is launched; outputs are then untouched.
 *   - Tensors are dense and row-major with the last index contiguous.  Activation tensors (x, u, delta,
 *     z, y) are [B, D, L] (batch, channel, time); Bm and Cm are [B, N, L]; A is [D, N].
 *   - The library keeps no settings between calls: every option is an argument.  Calls are thread-safe; two calls that share an output or workspace buffer must be ordered by the
 *     caller (same stream, or events).
 */
#ifndef COREY_H
#define COREY_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    COREY_F32 = 0,   /* IEEE binary32 storage                                 */
    COREY_BF16 = 1,  /* bfloat16 storage; all arithmetic and the state are fp32 */
    COREY_F16 = 2    /* IEEE binary16 storage (the paper's kernel-level benchmarks run in FP16); arithmetic and state fp32 */
} corey_dtype;

typedef enum {
    COREY_OK = 0,
    COREY_EINVAL = 1,       /* a size, flag or enum is out of range                          */
    COREY_ENULL = 2,        /* a required pointer is NULL                                    */
    COREY_ESHAPE = 3,       /* sizes are inconsistent or exceed what the kernels index       */
    COREY_ENONFINITE = 4,   /* r is NaN (the statistic saw a non-finite range)               */
    COREY_EUNSUPPORTED = 5, /* valid request the library does not implement                  */
    COREY_EHIP = 6,         /* a HIP runtime call failed (message in corey_last_error)       */
    COREY_EWORKSPACE = 7    /* workspace missing or smaller than the query call says         */
} corey_status;

/* Limits the kernels are written for. */
#define COREY_MAX_BINS 4096      /* K                      */
#define COREY_MAX_STATE 256      /* N (d_state)            */
#define COREY_MIN_CHUNK 16
#define COREY_MAX_CHUNK 2048
#define COREY_CHUNK_SLOTS 12     /* chunk-distribution counters: slot log2(chunk), chunk = 1 .. 2048 */
#define COREY_MAX_CONV 4         /* taps of the causal convolution that produces u */
#define COREY_RANGE_PARTS 1024   /* partial ranges a producer of u hands to corey_entropy_hist (16 bytes each) */
#define COREY_HANDOFF_BYTES (COREY_RANGE_PARTS * 16 + 16 * COREY_MAX_BINS * 4)   /* the buffer a producer of u hands to the statistic */

/* -------------------------------------------------------------------------------------------------------
 * corey_entropy_hist -- Eq. 1 and r = H / log K.
 *
 * For one histogram over a set S of values: lo = min S, hi = max S (binary32); K equal-width bins on
 * [lo, hi], half open, the last closed; p_k = count_k / |S|; H = -sum_k p_k log(p_k + eps) in nats;
 * r = clamp(H / log K, 0, 1).  Bin index of a value v, stated to the rounding because counts are integers:
 *     scale = (float)(K / ((double)hi - (double)lo));  k = min((int)((v - lo) * scale), K - 1)
 * with the subtraction and the multiplication each one binary32 operation (no fused multiply-add).
 * An empty bin contributes nothing to H (p log(p + eps) is 0 at p = 0; for eps = 0 this is the usual 0 log 0 = 0).
 * hi == lo puts every sample in bin 0.  If S is empty or its range is not finite (NaN or infinity in the
 * input) the counts are zero and H and r are NaN.  binary32 subnormal inputs are outside the contract.
 *
 *   x           DEVICE, [B, D, L] in `dt`.
 *   seqlens     DEVICE int32[B] or NULL.  NULL: one histogram over all B*D*L values (nh = 1).  Otherwise one
 *               histogram per sequence b over the positions t < seqlens[b] of its D channels (nh = B);
 *               0 <= seqlens[b] <= L is the caller's responsibility (values are clamped to [0, L]).
 *   K           number of bins, 2 <= K <= COREY_MAX_BINS.   eps >= 0 (the paper's hook uses 1e-8).
 *   stride, block   >= 1.  Number the values of one histogram in memory order j = 0, 1, ... and cut them into blocks
 *               of `block` consecutive values; value j is used iff (j / block) % stride == 0 (every stride-th block).
 *               stride 1 is the exact statistic.  stride 8 with block 1 is the paper's sampled variant (its routed
 *               ablation's "sampled histogram (stride 8)"), which thins the arithmetic but still touches every cache
 *               line; with a block of a few hundred values (a power-of-two number of 16-byte words, e.g. 512) only
 *               the sampled runs of memory are fetched, so the statistic costs 1/stride of the traffic.
 *   counts_out  DEVICE uint32[nh * K].   H_out, r_out: DEVICE double[nh].
 *   range_out   DEVICE float[nh * 2] (lo, hi per histogram) or NULL.
 *   range_parts DEVICE, COREY_HANDOFF_BYTES as written by causal_conv1d_silu_fwd for this same tensor, or NULL.  With
 *               it the range sweep is skipped (the producer of x already saw every value) and so is the launch that
 *               clears the partial histograms (the producer cleared the ones inside this buffer; the call leaves them
 *               cleared again, so the buffer serves any number of calls): only the count sweep reads x.  The buffer
 *               is read and written.  Requires seqlens == NULL (COREY_EINVAL otherwise).  With stride > 1 the bins are
 *               then bounded by the minimum and maximum of ALL values while the counts are those of the sampled
 *               blocks (without range_parts a sampled statistic takes the range of the sampled values; the paper
 *               does not say which its sampled variant uses): the cheapest statistic the library offers, one read
 *               of 1/stride of x.
 *   workspace   DEVICE, at least corey_entropy_hist_workspace(B, K) bytes, 256-byte aligned; scratch only,
 *               contents are undefined afterwards.
 * The work is two sweeps over the sampled values of x (range, then counts) plus an O(K) reduction, as the paper's
 * protocol states; H is summed in double.  Counts are exact integers; H and r agree with a sequential double
 * evaluation to summation-order rounding (about 1e-15 relative).
 * ----------------------------------------------------------------------------------------------------- */
int corey_entropy_hist(const void* x, corey_dtype dt, int64_t B, int64_t D, int64_t L,
                       const int32_t* seqlens, int32_t K, double eps, int64_t stride, int64_t block,
                       uint32_t* counts_out, double* H_out, double* r_out, float* range_out,
                       void* range_parts, void* workspace, size_t workspace_bytes, void* hip_stream);

/* Bytes of workspace corey_entropy_hist needs for batch B and K bins (0 if the arguments are invalid). */
size_t corey_entropy_hist_workspace(int64_t B, int32_t K);

/* -------------------------------------------------------------------------------------------------------
 * corey_entropy_hist_static -- corey_entropy_hist for callers that cannot allocate device memory and have no
 * workspace to pass: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, results and errors as corey_entropy_hist, minus the workspace: the scratch memory is a buffer of
 * COREY_STATIC_SCRATCH_BYTES built into the library's GPU code (each GPU the library runs on holds one copy until the
 * process ends).  The call allocates and frees nothing, on the host or on the GPU.
 *   Limit: corey_entropy_hist_workspace(B, K) <= COREY_STATIC_SCRATCH_BYTES (e.g. B = 1 with any K, B <= 60 at
 *   K = 256); beyond it COREY_EWORKSPACE, nothing launched.
 *   Every call on one GPU uses that GPU's one buffer: calls that may overlap on a GPU (different streams, different
 *   threads) race on it and must be ordered by the caller.  The buffer keeps the last call's contents; the kernels
 *   clear what has to start at zero, as they do for a caller's workspace.
 *   Errors besides those of corey_entropy_hist: COREY_EHIP if the buffer's address cannot be obtained,
 *   COREY_EUNSUPPORTED for a device index of 64 or more.
 * ----------------------------------------------------------------------------------------------------- */
#define COREY_STATIC_SCRATCH_BYTES (1 << 20)
int corey_entropy_hist_static(const void* x, corey_dtype dt, int64_t B, int64_t D, int64_t L,
                              const int32_t* seqlens, int32_t K, double eps, int64_t stride, int64_t block,
                              uint32_t* counts_out, double* H_out, double* r_out, float* range_out,
                              void* range_parts, void* hip_stream);

/* -------------------------------------------------------------------------------------------------------
 * corey_select_chunk -- Eq. 2:  C = clip(2^round(log2(c_min + r (c_max - c_min))), c_min, c_max).
 *
 * Pure host function (HOST pointers, no GPU work), evaluated in double; round(v) = floor(v + 0.5).
 *   mode 0  entropy rule.
 *   mode 1  sequence-length gate, then entropy rule: L <= short_len returns short_chunk.
 *   mode 2  sequence-length table only: L <= short_len -> short_chunk, else long_chunk
 *           (the paper's learned table: <= 50 tokens -> 128, otherwise 512).
 *   mode 3  static_chunk.
 *   mode 4  guarded entropy rule: the prediction is kept only if it is at least guard_buckets powers of
 *           two away from safe_chunk, else safe_chunk (the paper's guard: 512, two buckets).
 * r is first multiplied by h_ref_scale and clamped to [0, 1]: 1.0 is the calibrated reference
 * H_ref = log K; log(K)/8 gives the legacy H_ref = 8 nats.
 * Eq. 2's own result is finally capped at the smallest power of two >= L (never below c_min), since a
 * larger tile cannot be filled; table and static values are returned as given.
 * Errors: COREY_ENULL; COREY_EINVAL for L < 1, a chunk field that is not a power of two, c_min > c_max or
 * an unknown mode; COREY_ENONFINITE if r is NaN in an entropy mode.
 * ----------------------------------------------------------------------------------------------------- */
typedef struct {
    int32_t mode;
    int32_t c_min, c_max;        /* library default 64, 2048; Eq. 2 as printed uses 32, 512 */
    double  h_ref_scale;
    int32_t short_len, short_chunk, long_chunk;   /* 50, 128, 512 */
    int32_t static_chunk;
    int32_t safe_chunk, guard_buckets;            /* 512, 2 */
} corey_policy;

/* Fill *p with the defaults named above (mode 0). */
int corey_policy_default(corey_policy* p);

int corey_select_chunk(double r, int64_t L, const corey_policy* p, int32_t* chunk_out);

/* -------------------------------------------------------------------------------------------------------
 * corey_select_chunk_device -- the same rule, evaluated on the GPU for nh values of r that are still in
 * device memory, so that a routed scan needs no host round trip (the paper names the synchronisation around
 * runtime feature collection as one of the costs of routing).
 *
 *   r_dev        DEVICE double[nh]   (r_out of corey_entropy_hist).
 *   seqlens      DEVICE int32[nh] or NULL: the sequence length each decision is taken for; NULL uses L for all.
 *   p            HOST policy (copied at call time).
 *   chunks_out   DEVICE int32[nh]: the chunk per histogram, directly usable as `chunks_dev` of selective_scan_fwd.
 *                An entry whose r is NaN in an entropy mode is written as 0, which selective_scan_fwd treats as
 *                "use the host chunk".
 * Same arithmetic as corey_select_chunk (double precision, round = floor(v + 0.5)); the device log2 can differ
 * from the host's in the last bit, which matters only within ~1e-15 of a rounding tie of Eq. 2.
 * Errors (host side, before the launch): COREY_ENULL, COREY_EINVAL as for corey_select_chunk, nh < 1, or a policy
 * whose mode can select a chunk above COREY_MAX_CHUNK (the scan could not run it).
 * ----------------------------------------------------------------------------------------------------- */
int corey_select_chunk_device(const double* r_dev, const int32_t* seqlens, int64_t L, int32_t nh,
                              const corey_policy* p, int32_t* chunks_out, void* hip_stream);

/* -------------------------------------------------------------------------------------------------------
 * corey_ema_update -- the exponential moving average of the entropy estimate across calls ("Entropy Estimation
 * Protocol"):  H^_t = lambda * H^_{t-1} + (1 - lambda) * H_t,  0 <= lambda < 1  (the paper's prototype: 0.85, an
 * effective horizon of about 1 / (1 - lambda) = 6.7 calls).  Host function on a HOST state: *state = NaN means "no
 * estimate yet" and the first observation is taken as it is (the paper does not state the initial value); a NaN
 * observation leaves the state unchanged.  Errors: COREY_ENULL, COREY_EINVAL for lambda outside [0, 1).
 * ----------------------------------------------------------------------------------------------------- */
int corey_ema_update(double lambda, double* state, double H);

/* -------------------------------------------------------------------------------------------------------
 * corey_route_device -- corey_entropy_hist followed by corey_select_chunk_device in one call: the statistic of x,
 * then the chunk rule applied to each r by the kernel that reduces the histogram (one launch fewer on the routed
 * path; the paper counts scheduler dispatch among the costs of routing).  Arguments as for those two calls; the
 * sequence length each decision is taken for is seqlens[h] when seqlens is given, else L.  Without the two optional
 * arguments below the results are identical to calling the two one after the other.
 *   ema_lambda, ema_state   ema_state: DEVICE double[nh] or NULL.  With a state, the rule is applied to the smoothed
 *               entropy: ema_state[h] is updated as in corey_ema_update (NaN = no estimate yet) and r for the rule
 *               is clamp(ema_state[h] / log K, 0, 1); H_out and r_out still hold the raw values of this call.
 *   chunk_calls DEVICE uint32[COREY_CHUNK_SLOTS] or NULL: chunk-distribution counters (the paper logs, per run, how
 *               many scheduler calls chose each chunk); slot log2(chunk) is incremented for every decision taken
 *               (not for NaN decisions).  The caller clears them.
 * Errors: as for both calls; COREY_EINVAL for ema_lambda outside [0, 1) when ema_state is given.
 * ----------------------------------------------------------------------------------------------------- */
int corey_route_device(const void* x, corey_dtype dt, int64_t B, int64_t D, int64_t L,
                       const int32_t* seqlens, int32_t K, double eps, int64_t stride, int64_t block,
                       const corey_policy* p, double ema_lambda, double* ema_state, uint32_t* chunk_calls,
                       uint32_t* counts_out, double* H_out, double* r_out, float* range_out, void* range_parts,
                       int32_t* chunks_out, void* workspace, size_t workspace_bytes, void* hip_stream);

/* -------------------------------------------------------------------------------------------------------
 * corey_route_device_deferred / selective_scan_fwd_routed -- the routed path with one launch fewer.  The paper names
 * "histogram construction, synchronization boundaries around runtime feature collection, and scheduler dispatch
 * overhead" as the costs that make routing lose end to end: each dependent launch between the producer of u and the
 * scan is such a cost.  corey_route_device_deferred runs the sweeps of corey_route_device but not its O(K) reduction;
 * it fills *route (HOST, caller-owned, opaque) instead.  selective_scan_fwd_routed is selective_scan_fwd with the
 * reduction and the chunk rule evaluated at the start of its own first kernel: every result corey_route_device
 * would have written (counts, H, r, range, chunk, chunk counters) is written then, bit for bit the same, and the scan
 * runs with the chunk so selected (per sequence when the statistic was per sequence, else one chunk for all).
 * With range_parts from the producer the whole routed path is: producer, one count sweep, scan.
 *   Arguments as for corey_route_device and selective_scan_fwd (which has no chunks_dev here).  ema_state must be NULL
 *   (COREY_EUNSUPPORTED: the smoothed rule needs the reduction in a launch of its own).  *route is valid for ONE
 *   selective_scan_fwd_routed call on the same stream, with the buffers it names still alive; `chunk` of that call is
 *   the launch-shape hint and the fallback when r is NaN.
 * ----------------------------------------------------------------------------------------------------- */
typedef struct { uint64_t opaque[40]; } corey_deferred_route;
int corey_route_device_deferred(const void* x, corey_dtype dt, int64_t B, int64_t D, int64_t L,
                                const int32_t* seqlens, int32_t K, double eps, int64_t stride, int64_t block,
                                const corey_policy* p, uint32_t* chunk_calls,
                                uint32_t* counts_out, double* H_out, double* r_out, float* range_out, void* range_parts,
                                int32_t* chunks_out, void* workspace, size_t workspace_bytes,
                                corey_deferred_route* route, void* hip_stream);

/* -------------------------------------------------------------------------------------------------------
 * corey_entropy_hist_onesweep -- Eq. 1 and r = H / log K for a 16-bit tensor from ONE pass over it.
 *
 * The paper's estimator reads the tensor twice (a min/max pass, then a bin-count pass: "Entropy Estimation Protocol";
 * its overhead budget counts 2 * N * sizeof bytes, "Active-Mode Overhead Budget").  For 16-bit storage one pass
 * suffices: count how often each of the 65536 bit patterns occurs, then take the range and the K bin counts from
 * that table.  A value's bin depends on the value and the range only, so the counts, H and r are exactly those of
 * corey_entropy_hist (same binary32 bin expression, applied once per occurring pattern with its multiplicity).
 * Whole-tensor statistic, every value (no seqlens, no sampling).
 *
 *   x           DEVICE, [B, D, L] in `dt`; dt must be COREY_BF16 or COREY_F16 (COREY_F32: COREY_EUNSUPPORTED).
 *   p, chunks_out   HOST policy and DEVICE int32[1], or both NULL: with a policy the chunk rule is applied to r on
 *               the GPU as by corey_route_device (sequence length L).
 *   counts_out  DEVICE uint32[K].   H_out, r_out: DEVICE double[1].   range_out: DEVICE float[2] or NULL.
 *   table_ws    DEVICE, corey_pattern_table_workspace() bytes (about 33 MiB: one 128 KiB table per compute unit),
 *               256-byte aligned; scratch, contents undefined afterwards.
 * Errors: COREY_ENULL, COREY_EINVAL, COREY_ESHAPE (B*D*L >= 2^32), COREY_EUNSUPPORTED, COREY_EWORKSPACE, COREY_EHIP.
 *
 * corey_entropy_hist_from_table -- the same statistic from a table that causal_conv1d_silu_fwd filled while it wrote
 * the tensor (its `pattern_table` argument): no pass over the tensor at all, which is how the paper proposes to make
 * routing cheap ("fuse the entropy statistic more deeply").  Arguments as above; L is only the sequence length the
 * rule is applied for.  The table is left as it is: further calls (another K, another policy) give the statistic of
 * the same tensor again.
 * ----------------------------------------------------------------------------------------------------- */
size_t corey_pattern_table_workspace(void);
int corey_entropy_hist_onesweep(const void* x, corey_dtype dt, int64_t B, int64_t D, int64_t L, int32_t K, double eps,
                                const corey_policy* p, int32_t* chunks_out, uint32_t* counts_out, double* H_out,
                                double* r_out, float* range_out, void* table_ws, size_t table_ws_bytes, void* hip_stream);
int corey_entropy_hist_from_table(corey_dtype dt, int64_t L, int32_t K, double eps, const corey_policy* p,
                                  int32_t* chunks_out, uint32_t* counts_out, double* H_out, double* r_out,
                                  float* range_out, void* table_ws, size_t table_ws_bytes, void* hip_stream);

/* -------------------------------------------------------------------------------------------------------
 * causal_conv1d_silu_fwd -- the step before the path: the causal depthwise convolution and SiLU that produce the
 * scan input u (step (1) of the paper's inline hook, "Active-Mode Overhead Budget": convolution, then the entropy of
 * the post-convolution tensor, then the rule, then the scan), with the range of u taken in the same pass (the paper
 * names fusing the statistic more deeply into the layer as the way to make routing cheaper):
 *
 *     v[b,d,t] = bias[d] + sum_{k=0}^{W-1} weight[d,k] * x[b,d,t-(W-1)+k]       (x before t = 0: state_in, else 0)
 *     u[b,d,t] = v * sigmoid(v)                                                   stored in `dt`
 *
 * evaluated in binary32 (taps accumulated oldest first with fused multiply-adds).
 *   x, u        DEVICE [B, D, L] in `dt`; u may not overlap x (only u == x is detected: COREY_EINVAL).
 *   weight      DEVICE float[D, W], 1 <= W <= COREY_MAX_CONV.     bias: DEVICE float[D] or NULL.
 *   state_in    DEVICE [B, D, W-1] in `dt` or NULL: the W-1 inputs that precede t = 0 (oldest first).
 *   state_out   DEVICE [B, D, W-1] in `dt` or NULL: the last W-1 inputs (for continuing the sequence); may not
 *               overlap state_in.
 *   range_parts DEVICE, COREY_HANDOFF_BYTES, or NULL: partial minima / maxima (and a NaN flag) of the values of u *as
 *               stored*, followed by cleared partial histograms, for corey_entropy_hist / corey_route_device on this u.
 *   pattern_table, pattern_table_bytes   DEVICE, corey_pattern_table_workspace() bytes, 256-byte aligned, or NULL / 0
 *               (16-bit storage only): the kernel also counts the bit patterns of the values of u it stores, so that
 *               corey_entropy_hist_from_table gives the exact statistic of u without reading u at all.
 * Errors: COREY_ENULL, COREY_EINVAL (dtype, W), COREY_ESHAPE, COREY_EUNSUPPORTED (pattern_table with fp32 storage),
 * COREY_EWORKSPACE (pattern_table too small or misaligned).
 * ----------------------------------------------------------------------------------------------------- */
int causal_conv1d_silu_fwd(const void* x, const float* weight, const float* bias, const void* state_in,
                           void* u, void* state_out, void* range_parts, void* pattern_table, size_t pattern_table_bytes,
                           corey_dtype dt, int64_t B, int64_t D, int64_t L, int32_t W, void* hip_stream);

/* -------------------------------------------------------------------------------------------------------
 * selective_scan_fwd -- the recurrence h_t = A_t h_{t-1} + B_t x_t, y_t = C_t h_t + D_t x_t (Method,
 * Preliminaries) in its Mamba-1 form, for every sequence b and channel d independently:
 *
 *     dl_t = delta[b,d,t] + delta_bias[d];   if delta_softplus: dl_t = log(1 + exp(dl_t))
 *     h_t[n] = exp(dl_t * A[d,n]) * h_{t-1}[n] + dl_t * Bm[b,n,t] * u[b,d,t]          (h_{-1} = h0 or 0)
 *     y[b,d,t] = sum_n Cm[b,n,t] * h_t[n] + Dv[d] * u[b,d,t];   if z: y *= z * sigmoid(z)
 *
 * The sequence is processed in tiles of `chunk` time steps per workgroup iteration with the fp32 state
 * carried on chip from tile to tile; the result does not depend on `chunk` beyond floating-point
 * reassociation (the paper's patched kernel is "recurrence-preserving").
 *
 *   u, delta, z, y   DEVICE [B, D, L] in `dt`; z may be NULL (no gate).
 *   A                DEVICE float[D, N].     Bm, Cm: DEVICE [B, N, L] in `dt`.
 *   Dv, delta_bias   DEVICE float[D] or NULL (treated as zeros).
 *   h0               DEVICE float[B, D, N] or NULL (zero initial state).
 *   seqlens          DEVICE int32[B] or NULL.  With seqlens, sequence b is scanned over t < seqlens[b];
 *                    y is written as 0 for the padded positions and last_state is the state after the
 *                    last valid step.
 *   chunk            HOST value: power of two in [COREY_MIN_CHUNK, COREY_MAX_CHUNK].  chunk > L is legal.
 *   chunks_dev       DEVICE int32[B] (int32[1] with COREY_SCAN_ONE_CHUNK) or NULL: per-sequence chunk (same
 *                    constraints) that overrides `chunk` without a host round trip; out-of-range or
 *                    non-power-of-two entries fall back to `chunk`.
 *   last_state       DEVICE float[B, D, N], required.
 *   workspace        DEVICE, at least selective_scan_fwd_workspace(B, N, L) bytes, 16-byte aligned; scratch only
 *                    (the call first rewrites B and C there as fp32 in the order, or the two orders, the scan reads
 *                    them in).
 *   1 <= N <= COREY_MAX_STATE;  B*D*L and B*N*L must fit in int64 and B*D in int32.
 *   flags            bitwise OR of COREY_SCAN_* options, 0 for the defaults.
 *                    COREY_SCAN_GENERAL_A: never take the fast path for structured A.  By default, when
 *                    A[d, n] = (n + 1) * A[d, 0] holds exactly for the channels of a workgroup -- Mamba's S4D-real
 *                    initialisation, A = -(1 .. N), which the benchmark layers use; trained weights in general do
 *                    not -- and the storage type is 16-bit, exp(dl * A[d, n]) is formed as exp(dl * A[d, 0])^(n + 1)
 *                    by repeated multiplication: one exponential per time step instead of one per (time step,
 *                    state).  The result differs from the general path only by the chain's roundings (at most about
 *                    (n + 1) * 2^-24 relative per decay factor).  The test is made on the GPU per workgroup; any
 *                    other A takes the general path whatever the flag.
 *                    COREY_SCAN_ONE_CHUNK: chunks_dev holds ONE entry that applies to every sequence (the chunk
 *                    routed from a whole-tensor statistic of a batch: corey_route_device without seqlens writes one).
 *                    COREY_SCAN_WHOLE_ROWS: never share the states of a channel between two rows of lanes (see
 *                    selective_scan_fwd_plan_split; for tests and measurements of the other launch shape).
 *                    Unknown bits: COREY_EINVAL.
 * y and last_state may not alias any input.  Accuracy against a double-precision evaluation of the same
 * bits: about 1e-6 relative to the row's scale for fp32 storage; for bf16 storage y carries one bf16
 * rounding (half an ulp: up to 2^-8 relative) on top, for fp16 storage 2^-11.
 * ----------------------------------------------------------------------------------------------------- */
#define COREY_SCAN_GENERAL_A 1u
#define COREY_SCAN_ONE_CHUNK 2u
#define COREY_SCAN_WHOLE_ROWS 4u
int selective_scan_fwd(const void* u, const void* delta, const float* A, const void* Bm, const void* Cm,
                       const float* Dv, const void* z, const float* delta_bias, int delta_softplus,
                       const float* h0, const int32_t* seqlens, int32_t chunk, const int32_t* chunks_dev,
                       void* y, float* last_state, corey_dtype dt,
                       int64_t B, int64_t D, int64_t N, int64_t L, uint32_t flags,
                       void* workspace, size_t workspace_bytes, void* hip_stream);

int selective_scan_fwd_routed(const void* u, const void* delta, const float* A, const void* Bm, const void* Cm,
                              const float* Dv, const void* z, const float* delta_bias, int delta_softplus,
                              const float* h0, const int32_t* seqlens, int32_t chunk, const corey_deferred_route* route,
                              void* y, float* last_state, corey_dtype dt,
                              int64_t B, int64_t D, int64_t N, int64_t L, uint32_t flags,
                              void* workspace, size_t workspace_bytes, void* hip_stream);

/* Bytes of workspace selective_scan_fwd needs (0 if the arguments are invalid): room for B and C as fp32, padded
 * along L to whole tiles and in N to a multiple of 4, in the two orders a launch may read them in (one launch can run
 * some channels with 16 and the others with 8 or 4 time steps per lane):
 * 4 * B * roundup(N, 4) * roundup(L + 2048, 4) * 4. */
size_t selective_scan_fwd_workspace(int64_t B, int64_t N, int64_t L);

/* How selective_scan_fwd shapes its launch for these sizes (host functions, no GPU work; for inspection and tests).
 * selective_scan_fwd_plan: the number d16 of leading channels of every sequence that are processed with 16 time steps
 * per lane; the remaining D - d16 channels take selective_scan_fwd_plan_steps time steps per lane: 8, or 4 when the
 * launch would otherwise leave most of the GPU without a wave (short tiles, few channels).  d16 = 0 or D means one lane
 * geometry for all channels.  The shape never changes results beyond floating-point reassociation (each channel is an
 * independent recurrence; the steps of a tile are combined by an associative scan).  -1 if the arguments are invalid.
 * selective_scan_fwd_plan_split: 1 when the launch gives every channel two rows of lanes, each with half of the N states
 * (launches of one lane geometry that would leave most SIMDs with at most one wave: small layers, short tiles; tiles of
 * at most 1024 steps, N >= 4): the two partial sums over states of the read-out y_t = C_t h_t (Method, Preliminaries) are added
 * once per tile.  0 otherwise, and always 0 under COREY_SCAN_WHOLE_ROWS. */
int64_t selective_scan_fwd_plan(int64_t B, int64_t D, int64_t N, int32_t chunk);
int32_t selective_scan_fwd_plan_steps(int64_t B, int64_t D, int64_t N, int32_t chunk);
int32_t selective_scan_fwd_plan_split(int64_t B, int64_t D, int64_t N, int32_t chunk);

/* Message for the most recent failing call on this thread ("" if none).  Static storage; do not free. */
const char* corey_last_error(void);

/* Library version, "major.minor". */
const char* corey_version(void);

/* -------------------------------------------------------------------------------------------------------
 * selective_state_update -- one generated token: the recurrence of selective_scan_fwd (Method, Preliminaries) taken
 * for a single step from the carried state, as in the greedy-generation steps that follow the prompt in the paper's
 * quality check ("Output Quality Preservation").  For every sequence b and channel d:
 *
 *     dl = delta[b,d] + delta_bias[d];   if delta_softplus: dl = log(1 + exp(dl))
 *     state[b,d,n] <- exp(dl * A[d,n]) * state[b,d,n] + dl * Bt[b,n] * x[b,d]
 *     y[b,d] = sum_n Ct[b,n] * state[b,d,n] + Dv[d] * x[b,d];   if z: y *= z * sigmoid(z)
 *
 *   state       DEVICE float[B, D, N], read and overwritten in place (the layout of selective_scan_fwd's last_state
 *               and h0, so a prompt's final state can be carried straight into generation).
 *   x, delta, z DEVICE [B, D] in `dt` (z may be NULL).   Bt, Ct: DEVICE [B, N] in `dt`.   y: DEVICE [B, D] in `dt`.
 *   A float[D, N], Dv and delta_bias float[D] or NULL, DEVICE.
 * y may not alias an input; state is the only tensor that is both read and written.
 * Arithmetic in binary32 as in the scan; y is rounded once to `dt`.  Asynchronous on hip_stream; needs no workspace.
 * Errors: COREY_ENULL, COREY_EINVAL (dtype, misaligned state), COREY_ESHAPE (B, D < 1, N outside
 * [1, COREY_MAX_STATE], B*D >= 2^25), COREY_EHIP.
 * ----------------------------------------------------------------------------------------------------- */
int selective_state_update(void* state, const void* x, const void* delta, const float* A, const void* Bt,
                           const void* Ct, const float* Dv, const void* z, const float* delta_bias,
                           int32_t delta_softplus, void* y, corey_dtype dt, int64_t B, int64_t D, int64_t N,
                           void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* COREY_H */
