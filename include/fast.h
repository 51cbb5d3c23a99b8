/*
 * fast.h - C ABI of the MI355X (gfx950) batched All-to-All(v) schedule synthesiser.
 *
 * For each of B GPU-to-GPU traffic matrices of a two-tier cluster of S servers x G
 * GPUs (N = S*G GPUs, GPU g = a*G + i is GPU i of server a), the library computes,
 * entirely on the device:
 *   1. the intra-server sender balancing of every cross-server tile and the
 *      resulting lane-routing matrix (paper Section 4.1 "Mitigating sender skew",
 *      Section 4.2 Step 1), together with the merged peer transfer that collapses
 *      each tile to one per-lane server-level entry (Section 4.1 "Mitigating
 *      receiver skew", Section 4.2 / Fig. 6);
 *   2. the embedding of the server-level matrix into a scaled doubly stochastic
 *      matrix and its Birkhoff decomposition into balanced, one-to-one scale-out
 *      stages (Section 4.4 "Adapting an arbitrary matrix to a valid form" and
 *      "Birkhoff's decomposition: overview"; Section 4.2);
 *   3. the analytical two-tier completion time of the plan (Section 5.4 simulator;
 *      Appendix, Theorems 1 and 2).
 *
 * Conventions.  All byte counts are int64 and non-negative; indices are int32;
 * times are double seconds; bandwidths are double bytes/second per GPU
 * (full duplex).  "device" pointers are HIP device memory on the device that was
 * current when the plan was created; "host" pointers are ordinary host memory.
 * No function takes or returns ownership of a caller's buffer.
 *
 * Return codes: 0 on success, otherwise one of the negative FAST_ERR_* values;
 * on error nothing has been enqueued.
 */
#ifndef FAST_H_
#define FAST_H_

#include <stdint.h>
#include <hip/hip_runtime_api.h>

#ifdef __cplusplus
extern "C" {
#endif

#define FAST_OK                0
#define FAST_ERR_INVALID_ARG  -1   /* NULL pointer, B < 0, S < 1, G < 1, bandwidth not finite or <= 0,
                                      or the plan's device is not the current HIP device */
#define FAST_ERR_UNSUPPORTED  -2   /* S > FAST_MAX_SERVERS, G > FAST_MAX_GPUS_PER_SERVER, or a batch of
                                      more than FAST_MAX_BATCH matrices (or selections) in one call */
#define FAST_ERR_HIP          -3   /* a HIP runtime call failed */
#define FAST_ERR_OOM          -4   /* the plan's device workspace could not be allocated */

#define FAST_MAX_SERVERS          128
#define FAST_MAX_GPUS_PER_SERVER  8
#define FAST_MAX_BATCH            65535   /* matrices per call (a launch-grid dimension) */

/* Per-matrix status values stored in out_num_stages[b] instead of a stage count. */
#define FAST_STATUS_NEGATIVE_ENTRY  -1  /* an off-diagonal traffic entry is negative */
#define FAST_STATUS_STAGE_OVERFLOW  -2  /* more than fast_plan_max_stages() stages (cannot happen
                                           while the Birkhoff bound S*S-2S+2 holds; a tripwire) */
#define FAST_STATUS_INTERNAL        -3  /* no augmenting path found (impossible for a doubly
                                           stochastic residual; a tripwire) */

typedef struct fast_plan fast_plan_t;   /* opaque; owns a device workspace */

/*
 * Creates a plan for clusters of S servers x G GPUs with per-GPU scale-up bandwidth
 * link_bw_up ("B_1" of the Appendix) and scale-out bandwidth link_bw_out ("B_2").
 * The plan is bound to the HIP device current at this call.  *out_plan receives the
 * plan; free it with fast_plan_destroy.  Requires 1 <= S <= FAST_MAX_SERVERS and
 * 1 <= G <= FAST_MAX_GPUS_PER_SERVER.
 */
int fast_plan_create(int S, int G, double link_bw_up, double link_bw_out, fast_plan_t **out_plan);

/* Stage capacity per matrix that the output buffers must provide: S*S (a safe
 * bound; Section 4.4 "Number of stages" gives S*S - 2S + 2).  -1 if plan is NULL. */
int fast_plan_max_stages(const fast_plan_t *plan);

/*
 * Allocates every part of the plan's workspace for batches of up to B matrices (B <=
 * FAST_MAX_BATCH), so that no later call of any entry point with a batch of at most B
 * allocates, frees or synchronises: for callers that capture the calls into a HIP graph or must
 * keep allocation out of their steady state.  Sizes at 128 servers: about 0.5 MB per matrix
 * for the synthesis, 0.3 MB for the SpreadOut pass, 0.2 MB for the stage order, plus at most
 * 34 MB for the chunked stage walk.  The plan's device must be current.  May synchronise the
 * device (it frees what it replaces); a smaller B than already reserved changes nothing.
 * FAST_ERR_OOM leaves the plan usable with what it had or has got so far.
 */
int fast_plan_reserve(fast_plan_t *plan, int B);

/*
 * Synthesises the schedules of B traffic matrices (B <= FAST_MAX_BATCH).  All work is
 * enqueued on `stream` (the plan's device must be current: FAST_ERR_INVALID_ARG otherwise)
 * and the call returns without synchronising; outputs are valid once the stream has
 * drained.  The plan's workspace is reused by the next call, so calls on one plan must be
 * stream-ordered.  It is grown on demand, the only allocation this call may make: a call
 * with a larger B than any before on this plan (the first call included) frees the old
 * workspace and allocates a new one, which synchronises the device, must not happen while
 * a stream is being captured, and leaves any HIP graph captured from earlier calls on this
 * plan pointing at freed memory.  Make one call with the largest B first to avoid all three;
 * the analysis entry points below treat their own parts of the workspace the same way.
 *
 *  traffic            device, [B][N][N] row-major; traffic[b][g][h] = bytes GPU g sends to
 *                     GPU h (row = sender, Section 4.1 "Example setup").  The GPU diagonal
 *                     g == h is ignored.  Read only.
 *  out_rebalance      device, [B][N][N]; lane-routing matrix X of the sender balancing
 *                     (Section 4.1): X[(a,i)][(d,k)] = bytes of GPU (a,i)'s traffic for server
 *                     d that cross scale-out on lane k, i.e. leave from GPU (a,k) and arrive
 *                     at its peer (d,k).  k == i: kept by the GPU; k != i: handed to (a,k)
 *                     over scale-up first.  Lane loads are floor/ceil(T[a][d]/G) with the
 *                     remainder on the lowest lanes; surplus is poured into deficit in
 *                     ascending GPU index.  Intra-server tiles (d == a) are zero.
 *  out_stages         device, [B][max_stages][S]; out_stages[b][s][a] = destination server of
 *                     source server a in scale-out stage s, or -1 if a sends no real bytes in
 *                     that stage.  In a stage, destinations of active servers are distinct
 *                     (one-to-one) and GPU (a,k) talks only to GPU (dest,k) (Section 4.2,
 *                     Step 2).  Rows s >= K are left untouched.
 *  out_stage_bytes    device, [B][max_stages][S]; real bytes per lane that server a sends to
 *                     out_stages[b][s][a] in stage s (0 where the destination is -1).
 *  out_num_stages     device, [B]; number of stages K >= 0 of matrix b, or a negative
 *                     FAST_STATUS_* value, in which case the other outputs of that matrix
 *                     are unspecified.
 *  out_predicted_time device, [B][4] = { T_pred, t0, t2, t_opt } in seconds:
 *                     t0 = balancing, t2 = scale-out stages (sum of stage weights / B_out),
 *                     T_pred = t0 + t1 + t2 + t3 (+ exposed redistribution when
 *                     link_bw_up < (G-1)*link_bw_out) with t1 = intra-server portion and
 *                     t3 = last stage's redistribution (Appendix, proof of Theorem 2, the
 *                     four terms evaluated on the actual plan); t_opt = Theorem 1.
 *                     t3 = (G-1) * largest stage weight / link_bw_up: step (i) of that proof
 *                     prices a stage's redistribution at (m-1) l / B_1 (every GPU of the
 *                     destination server forwards all it received to one GPU) while the t3
 *                     printed after it has lost the (m-1); the factor of step (i) is kept.
 *                     The exposed part is sum over i >= 1 of max(0, (G-1) l_{i-1} / link_bw_up
 *                     - l_i / link_bw_out) on the stage weights in ascending order: pipeline
 *                     step i (stage i on scale-out, stage i-1 redistributed) ends when both
 *                     have ended.
 *
 * Results are a deterministic function of each matrix alone: independent of B, of the
 * position in the batch and of launch geometry.  B == 0 is valid and does nothing.
 */
int fast_synthesize_batched(fast_plan_t *plan, int B,
                            const int64_t *traffic,
                            int64_t *out_rebalance,
                            int32_t *out_stages,
                            int64_t *out_stage_bytes,
                            int32_t *out_num_stages,
                            double *out_predicted_time,
                            hipStream_t stream);

/*
 * fast_synthesize_batched for callers that cannot allocate device memory: code under HIP graph
 * capture, serving loops, harnesses that forbid hipMalloc.  Same arguments, same outputs, same
 * kernels; the workspace is a fixed array of FAST_NOALLOC_SCRATCH_BYTES in the library's device
 * image instead of the plan's grown-on-demand allocation, and the call makes no hipMalloc,
 * hipFree or any other allocating call (it records no timing events either:
 * fast_plan_set_timing does not apply to it).  Limit: B * (24 * S * S + 32 * S) bytes must fit
 * the array (B <= 84 at 128 servers, <= 5400 at 16), otherwise FAST_ERR_UNSUPPORTED and nothing
 * is enqueued.  Every call on a GPU, from any plan, uses that GPU's one array: calls that may
 * overlap on one GPU (different streams, different plans, different threads) race; order them.
 * The array keeps the last call's contents; nothing in it needs clearing between calls.
 * fast_plan_summary_batched keeps describing the last fast_synthesize_batched call, not this one.
 */
#define FAST_NOALLOC_SCRATCH_BYTES (32 * 1024 * 1024)
int fast_synthesize_batched_noalloc(fast_plan_t *plan, int B,
                                    const int64_t *traffic,
                                    int64_t *out_rebalance,
                                    int32_t *out_stages,
                                    int64_t *out_stage_bytes,
                                    int32_t *out_num_stages,
                                    double *out_predicted_time,
                                    hipStream_t stream);

/*
 * Link wake-up delay of the completion-time model (Section 5.4: every transfer step
 * costs a fixed wake-up delay plus size / bandwidth).  `seconds` >= 0 is added to T_pred
 * once per executed step - the balance (if anything is handed off), the intra-server
 * portion (if any), each stage, the last redistribution (if G > 1 and there is a stage)
 * - and to every non-empty SpreadOut stage.  The paper gives no value; the default 0
 * reproduces the Appendix.  FAST_ERR_INVALID_ARG if plan is NULL or seconds is negative
 * or not finite.
 */
int fast_plan_set_wakeup_delay(fast_plan_t *plan, double seconds);

/*
 * Which perfect matching a stage of the decomposition takes.  The paper (Section 4.4
 * "Birkhoff's decomposition: overview") accepts any perfect matching on the support of
 * the residual; Section 4.4 "Number of stages" adds that fewer stages are preferable
 * (each costs a synchronisation) and that the minimum is NP-hard to find.
 *   FAST_MATCHING_SUPPORT (default): the matching is repaired from stage to stage on the
 *     support of the residual (the paper's rule; canonical choices stated at
 *     fast_synthesize_batched).  Fastest synthesis, about (S-1)^2 stages on dense matrices.
 *   FAST_MATCHING_BOTTLENECK: a greedy rule that is not in the paper.  Every stage takes a
 *     bottleneck assignment: with t* = the largest t for which the cells of the residual
 *     holding at least t contain a perfect matching, the stage's matching is the canonical
 *     matching (same search rules, rows 0..S-1 augmented in order from nothing) of the
 *     cells holding at least t*, and its weight is t*.  Stage weights never increase from
 *     one stage to the next.  Far fewer stages on skewed matrices (about 14 times fewer at
 *     128 servers), slower synthesis.  Same outputs, same stage-count bound, same status
 *     codes; every other entry point works on the stages whichever rule made them.
 * Takes effect from the next fast_synthesize_batched call on this plan.
 * FAST_ERR_INVALID_ARG if plan is NULL or matching is neither constant.
 */
#define FAST_MATCHING_SUPPORT 0
#define FAST_MATCHING_BOTTLENECK 1
int fast_plan_set_matching(fast_plan_t *plan, int matching);

/*
 * SpreadOut baseline (Section 4.2 "SpreadOut: one-to-one but not optimal"; the
 * comparison schedule of the Section 5.4 simulation): stage i pairs endpoint s with
 * endpoint (s+i) mod n, every stage lasts as long as its largest transfer.  For each of
 * the B matrices (device, [B][N][N], as for fast_synthesize_batched) writes to
 *   out_spreadout_time  device, [B][2] seconds:
 *     [0] SpreadOut over the N GPUs on the raw matrix: sum over i = 1..N-1 of the
 *         non-empty stages' (delay + max over g of traffic[g][(g+i) mod N] / bandwidth of
 *         that pair), a pair inside a server moving at link_bw_up, across servers at
 *         link_bw_out;
 *     [1] SpreadOut over the S servers on the balanced per-lane matrix Q = ceil(T/G):
 *         sum over i = 1..S-1 of (delay + max over a of Q[a][(a+i) mod S] / link_bw_out);
 *     both are -1 for a matrix with a negative off-diagonal entry.
 * Enqueued on `stream`, asynchronous, same ownership and ordering rules as
 * fast_synthesize_batched; uses its own part of the plan's workspace.
 */
int fast_spreadout_batched(fast_plan_t *plan, int B, const int64_t *traffic,
                           double *out_spreadout_time, hipStream_t stream);

/*
 * Execution order of the stages of synthesised plans (Appendix, proof of Theorem 2: stages
 * are executed in ascending order of their transfer size, so that each stage's
 * redistribution hides under the next one; the completion-time model assumes this order).
 *   stage_bytes      device, [B][max_stages][S], as written by fast_synthesize_batched
 *   num_stages       device, [B], as written by fast_synthesize_batched
 *   out_stage_order  device, [B][max_stages] int32; entries 0..K-1 receive the stage indices
 *                    by ascending stage weight (largest per-lane byte count of the stage),
 *                    equal weights in extraction order; entries >= K, and all entries of a
 *                    matrix whose num_stages is negative, are left untouched
 * Enqueued on `stream`, asynchronous; uses its own part of the plan's workspace.
 */
int fast_stage_order_batched(fast_plan_t *plan, int B, const int64_t *stage_bytes,
                             const int32_t *num_stages, int32_t *out_stage_order,
                             hipStream_t stream);

/*
 * Builds traffic matrices from per-expert token counts (Section 5 "Integration into MoE
 * systems": the all-gathered counts that MoE frameworks hold before every dispatch).
 *   tokens_per_expert  device, [B][N][E] int64; [b][src][e] = tokens GPU src routes to expert e
 *   expert_to_gpu      device, [B][E] int32; GPU (0..N-1) that hosts expert e in matrix b
 *   token_bytes        bytes per routed token (> 0)
 *   out_traffic        device, [B][N][N]; out_traffic[b][src][h] = token_bytes * sum of the
 *                      counts of the experts placed on GPU h; the diagonal holds what stays
 *                      on the GPU (fast_synthesize_batched ignores it)
 *   out_status         device, [B] int32; 0, or -1 if a count is negative or an expert is
 *                      placed outside 0..N-1 (out_traffic of that matrix is unspecified)
 * E >= 1.  Enqueued on `stream`, asynchronous; needs no workspace.
 */
int fast_build_traffic_batched(fast_plan_t *plan, int B, int E, const int64_t *tokens_per_expert,
                               const int32_t *expert_to_gpu, int64_t token_bytes,
                               int64_t *out_traffic, int32_t *out_status, hipStream_t stream);

/*
 * Per-stage send offsets (Section 4.2 Step 2 / Step 3: a server pair's bytes are delivered over
 * several stages; this says where in each lane's send queue a stage's bytes start).  The stages
 * are walked in execution order: stage_order[b][e] = e-th stage to run, as written by
 * fast_stage_order_batched, or NULL for the order in which they were extracted.
 *   stages, stage_bytes, num_stages  device, as written by fast_synthesize_batched
 *   out_stage_offset   device, [B][max_stages][S] int64; [b][s][a] = bytes per lane that server a
 *                      has sent to server stages[b][s][a] in the stages executed before s (0 where
 *                      a is idle in s); rows s >= K and matrices with negative num_stages are
 *                      left untouched
 * stage_order[b][0..K) has to be a permutation of 0..K-1; entries outside that range are clamped
 * into it (no out-of-bounds access), and the offsets of such a matrix are unspecified.
 * Enqueued on `stream`, asynchronous.  When the batch alone would not fill the chip the walk over
 * the stages is cut into up to 16 chunks that run side by side; their per-pair totals go through
 * a part of the plan's workspace (at most 15 * 512 * S * ceil(S / 64) bytes per matrix),
 * allocated at the first call and whenever more is needed.
 */
int fast_stage_offsets_batched(fast_plan_t *plan, int B, const int32_t *stages,
                               const int64_t *stage_bytes, const int32_t *num_stages,
                               const int32_t *stage_order, int64_t *out_stage_offset,
                               hipStream_t stream);

/*
 * Exact scale-up volume of every stage's redistribution (Section 4.1 "Redistribution",
 * Section 4.2 Step 3; the Appendix bounds it by (G-1) * stage weight, the case where all bytes
 * of a stage are for one GPU).  Which bytes a stage carries follows from this byte-identity
 * policy (the paper fixes none): the bytes a GPU holds for a server form one region ordered by
 * destination GPU; balancing keeps the head of the region on the GPU and hands off the tail, cut
 * into the pieces of out_rebalance in ascending receiver index; a lane sends what its GPU kept,
 * then the pieces it was handed in ascending donor index; every stage takes the next
 * stage_bytes[s][a] bytes of each lane's queue.
 *   traffic, rebalance, stages, stage_bytes, num_stages   device, input and outputs of
 *                      fast_synthesize_batched for the same B matrices
 *   stage_order        device, [B][max_stages], or NULL = extraction order
 *   out_stage_offset   device, [B][max_stages][S], as for fast_stage_offsets_batched
 *   out_redis_bytes    device, [B][max_stages] int64; [b][s] = largest, over the GPUs of all
 *                      servers that receive in stage s, of max(bytes the GPU forwards to other
 *                      GPUs of its server, bytes other GPUs forward to it); entries s >= K are 0
 * Enqueued on `stream`, asynchronous; uses its own part of the plan's workspace (4 * S bytes
 * per matrix: one flag per source server, plus what fast_stage_offsets_batched uses), allocated
 * at the first call and whenever B grows.
 */
int fast_redistribution_batched(fast_plan_t *plan, int B, const int64_t *traffic,
                                const int64_t *rebalance, const int32_t *stages,
                                const int64_t *stage_bytes, const int32_t *num_stages,
                                const int32_t *stage_order, int64_t *out_stage_offset,
                                int64_t *out_redis_bytes, hipStream_t stream);

/*
 * The G x G redistribution matrices of selected stages (same policy and inputs as
 * fast_redistribution_batched; stage_offset as written by it or by fast_stage_offsets_batched).
 *   n_sel              number of selected stages (>= 0)
 *   sel                device, [n_sel][2] int32 = (matrix b, stage s)
 *   out_matrices       device, [n_sel][S][G][G] int64; [q][d][k][j] = bytes that arrive at server d
 *                      on lane k (at GPU (d,k)) in stage sel[q] and belong to GPU (d,j); the tile
 *                      of a server that receives nothing in that stage is zero, and so is every
 *                      tile of a selection that names no stage (b or s out of range)
 * Enqueued on `stream`, asynchronous; needs no workspace.
 */
int fast_redistribution_matrices(fast_plan_t *plan, int B, const int64_t *traffic,
                                 const int64_t *rebalance, const int32_t *stages,
                                 const int64_t *stage_bytes, const int32_t *num_stages,
                                 const int64_t *stage_offset, int n_sel, const int32_t *sel,
                                 int64_t *out_matrices, hipStream_t stream);

/*
 * Completion time of the overlapped pipeline (Section 4.3 "Pipeline structure"): balancing
 * first; the scale-out stages back to back in execution order; the intra-server portion on the
 * scale-up fabric alongside the first stage; a stage's redistribution starts when its scale-out
 * has ended and the scale-up fabric is free (one transfer at a time: the intra-server portion,
 * then the redistributions in stage order); the last redistribution is exposed.  Each step that
 * moves bytes costs the wake-up delay plus bytes / bandwidth.
 * Everything it evaluates is passed in; the plan contributes S, G, the bandwidths and the delay.
 *   stage_weight       device, [B][max_stages] int64; [b][s] = weight of stage s (largest per-lane
 *                      byte count of the stage), as written by fast_plan_summary_batched
 *   scaleup_bytes      device, [B][2] int64 = { balancing volume, intra-server volume } (the
 *                      numerators of t0 and t1), as written by fast_plan_summary_batched
 *   num_stages         device, [B], as written by fast_synthesize_batched; a count above
 *                      max_stages is read as max_stages
 *   stage_order        device, [B][max_stages], or NULL = extraction order
 *   redis_bytes        device, [B][max_stages] as written by fast_redistribution_batched, or NULL
 *                      = the Appendix's worst case (G-1) * stage weight
 *   out_pipeline_time  device, [B][2] seconds = { completion time, end of the last scale-out
 *                      stage }; both 0 for a matrix with negative num_stages
 */
int fast_pipeline_time_batched(fast_plan_t *plan, int B, const int64_t *stage_weight,
                               const int64_t *scaleup_bytes, const int32_t *num_stages,
                               const int32_t *stage_order, const int64_t *redis_bytes,
                               double *out_pipeline_time, hipStream_t stream);

/*
 * Copies out what the completion-time models need of the plans of the most recent
 * fast_synthesize_batched call on this plan (Appendix, proof of Theorem 2: the balancing and
 * intra-server volumes behind t0 and t1 and the stage sizes l_i), so that
 * fast_pipeline_time_batched can be given them explicitly.  Call it on the same stream right
 * after the synthesis call whose plans it describes: B has to be that call's B
 * (FAST_ERR_INVALID_ARG otherwise), and a later synthesis call on the plan replaces what it
 * would copy.
 *   out_stage_weight   device, [B][max_stages] int64; entries 0..K-1 = stage weights in
 *                      extraction order, entries >= K unspecified
 *   out_scaleup_bytes  device, [B][2] int64 = { largest over the GPUs of max(bytes handed off,
 *                      bytes handed in) by the balancing, largest over the GPUs of
 *                      max(intra-server bytes out, in) }
 * Unspecified for a matrix whose num_stages is negative.  Enqueued on `stream`, asynchronous.
 */
int fast_plan_summary_batched(fast_plan_t *plan, int B, int64_t *out_stage_weight,
                              int64_t *out_scaleup_bytes, hipStream_t stream);

/*
 * Per-kernel timing for measurement.  fast_plan_set_timing(plan, 1) starts a new
 * recording (dropping any earlier one): each following fast_synthesize_batched call,
 * up to FAST_MAX_TIMED_CALLS of them, records HIP events on its stream around its
 * three kernels (aggregation + balancing, decomposition, cost); further calls run
 * untimed.  fast_plan_set_timing(plan, 0) stops recording and keeps what was recorded.
 * fast_plan_timed_calls returns how many calls have been recorded (-1 if plan is NULL).
 * fast_plan_kernel_ms waits for recorded call `call` (0-based) to finish and writes its
 * three kernel durations in milliseconds to host array out_ms[3]; FAST_ERR_INVALID_ARG
 * if there is no such recorded call.  Up to 32 servers, with a scale-up bandwidth of at
 * least (G-1) times the scale-out bandwidth and the default matching rule, the cost model
 * is evaluated by the decomposition kernel itself (one launch less): its time is then part
 * of out_ms[1] and out_ms[2] is the few microseconds between two event records.
 */
#define FAST_MAX_TIMED_CALLS 256
int fast_plan_set_timing(fast_plan_t *plan, int enable);
int fast_plan_timed_calls(const fast_plan_t *plan);
int fast_plan_kernel_ms(fast_plan_t *plan, int call, float *out_ms);

/* Frees the plan and its workspace.  Work enqueued with it must have finished.
 * NULL is a no-op. */
void fast_plan_destroy(fast_plan_t *plan);

#ifdef __cplusplus
}
#endif
#endif /* FAST_H_ */
