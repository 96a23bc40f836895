/*
 * kfkb.h - C boundary of the single-GPU kFkB stage engine (gfx950 / MI355X).
 *
 * One process owns one GPU and one pipeline stage (the paper's worker model, Section 6.1:
 * one stage per device).  A stage is a stack of `layers` pre-LN GPT blocks.  The library
 * runs the stage's forward and backward task nodes (paper Section 2.4) for micro-batches in
 * the order of a kFkB plan (Sections 1 and 3.2.1: k forwards, then k backwards, units
 * alternating, early backward between units; k = 1 is 1F1B, k = M is GPipe), accumulates
 * parameter gradients across micro-batches in fp32 (Section 2.4, gradient-accumulation
 * nodes), and moves stage inputs / outputs over side streams with an injected per-transfer
 * delay (Section 5.3: send and receive on streams of their own, successive transfers of a
 * direction serialised).
 *
 * Conventions
 *   - every function returns 0 on success or a negative KFKB_E_* code; kfkb_last_error()
 *     gives a message for the calling thread's last failure.  No exception crosses the boundary.
 *   - "device" pointers are HIP device memory, "host" pointers are ordinary or pinned host
 *     memory, as stated per argument.  The library never takes ownership: every buffer
 *     handed in is borrowed until stage_destroy() and is freed by the caller.
 *   - stage_forward / stage_backward / run_kFkB only enqueue work; stage_sync() waits.
 *   - all matrices are row-major.  Activations are [tokens, features] with
 *     tokens = micro_batch * seq and token index = sample * seq + position.
 *   - not thread-safe: one stage per process, driven from one host thread.
 */
#ifndef KFKB_H
#define KFKB_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  KFKB_OK = 0,
  KFKB_E_ARG = -1,       /* bad argument (shape, k, null pointer) */
  KFKB_E_STATE = -2,     /* call out of order: backward before forward, forward of a live micro-batch, not bound */
  KFKB_E_MEMLIMIT = -3,  /* the plan's peak activation bytes exceed mem_limit, or the workspace is too small */
  KFKB_E_HIP = -4,       /* a HIP runtime call failed */
  KFKB_E_TIMEOUT = -5    /* stage_sync_timeout() gave up */
};

enum { KFKB_F32 = 0, KFKB_BF16 = 1, KFKB_F16 = 2 };   /* fp16: the paper's own precision; same kernels as bf16 */
enum { KFKB_OP_F = 0, KFKB_OP_B = 1 };

/* Options fixed before stage_init().  Zero-initialise, then set what differs from the default. */
typedef struct kfkb_config {
  int dtype;             /* KFKB_F32, KFKB_BF16 or KFKB_F16: storage type of weights and activations; all
                            reductions, statistics and gradient accumulators are fp32 either way */
  int micro_batch;       /* b: samples per micro-batch (>= 1) */
  int mlp_ratio;         /* MLP width F = mlp_ratio * hidden; 0 means 4 */
  int causal;            /* 1: causal attention mask, 0: none */
  float ln_eps;          /* LayerNorm epsilon; 0 means 1e-5 */
  int num_stages;        /* S: pipeline depth this stage pretends to sit in; 0 means 1 */
  int stage_index;       /* s in [0, S): the stage runs w = min(S-1-s, ceil(M/k)) warm-up groups */
  int max_microbatches;  /* upper bound on num_microbatches of any later run_kFkB (>= 1) */
  int recompute;         /* 1: activation recomputation (paper Section 2.2: with it more micro-batches fit, i.e. a
                            larger k under the same limit).  The two LayerNorm outputs and the GELU output of a block
                            are not kept from forward to backward; the backward forms them again from the kept
                            block input, x1 and pre-activation with the same kernels (same bits): 6 b*T*H + b*T*F
                            stashed elements per block instead of 8 b*T*H + 2 b*T*F.  Results do not change. */
} kfkb_config_t;

typedef struct kfkb_op {
  int op;                /* KFKB_OP_F or KFKB_OP_B */
  int mb;                /* micro-batch index */
  double t_start_ms;     /* start / end of the op's kernels on the compute stream, in ms since  */
  double t_end_ms;       /* the start of the run that logged it                                 */
} kfkb_op_t;

const char* kfkb_last_error(void);

/* ---- host-only planning (no GPU needed) ------------------------------------------------- */

/* kFkB order of one stage (paper Sections 1, 3.2.1, 5.4).  Writes 2*M ops into out (cap >= 2*M)
 * and returns 2*M, or a negative error.  w = number of warm-up forward groups (0 for the
 * last stage).  Inside a group micro-batches run in ascending index. */
int kfkb_schedule(int k, int num_microbatches, int warmup_groups, kfkb_op_t* out, int cap);

/* Largest number of micro-batches whose activations are alive at once under that plan. */
int kfkb_peak_live(int k, int num_microbatches, int warmup_groups);

/* Activation bytes one micro-batch holds from its forward to its backward (paper Section 4.1),
 * for a stage of the given shape; elem_bytes = 4 (fp32) or 2 (bf16). */
size_t kfkb_activation_bytes_per_microbatch(int layers, int micro_batch, int seq, int hidden, int heads,
                                            int mlp_width, int elem_bytes);
/* The same with the choice of kfkb_config_t.recompute (0: as above). */
size_t kfkb_activation_bytes_per_microbatch_ex(int layers, int micro_batch, int seq, int hidden, int heads,
                                               int mlp_width, int elem_bytes, int recompute);

/* Candidate plans (k, b) on the memory-limit curve at a fixed global batch (paper Section 4.2, pruning of the
 * candidate set): for k = 1, 2, ... the LARGEST micro-batch size b that divides global_batch, leaves at least k
 * micro-batches and whose plan fits: peak live micro-batches (stage position as in kfkb_config_t) x b x
 * bytes_per_sample <= mem_limit.  Stops at the first k for which b = 1 does not fit, or after k_max (0 = none).
 * Writes out_k[i], out_b[i] for up to cap candidates; returns their number. */
int kfkb_enumerate_candidates(int global_batch, size_t mem_limit, size_t bytes_per_sample, int num_stages,
                              int stage_index, int k_max, int* out_k, int* out_b, int cap);

/* ---- cost model and online choice of k (paper Sections 3.2.2 "auto tunner", 4.3, 5.2, 5.4) -------- *
 * The pipeline length of a candidate plan is estimated from stage computation times, profiled once *
 * per plan, and from communication times measured end to end and averaged over a moving window;    *
 * at regular intervals the admissible candidate with the shortest estimate is taken (ties: the      *
 * smaller k), and the switch costs nothing because no parameter moves.  The calls of this block are *
 * host-only; times are in milliseconds.                                                            */

/* Estimated iteration time of plan (k, M, w) on one stage whose neighbours do no compute: a discrete-event
 * run of the transfer rules (three FIFO resources compute / receive / send; send Y_mb after F(mb), send dX_mb
 * after B(mb), dY_mb arrives only after Y_mb has been sent, receives are issued in the order
 * kfkb_set_inputs_ahead describes as far ahead as the slot pools allow, a slot returns to its pool when the backward that read it ends).  Every op takes t_fwd / t_bwd and
 * every transfer of a direction its t_*.  x_slots / dy_slots: pool sizes, 0 = peak live + k and 2k.
 * Returns a negative error code for an invalid plan. */
double kfkb_predict_iteration_ms(int k, int num_microbatches, int warmup_groups, double t_fwd, double t_bwd,
                                 double t_recv_x, double t_recv_dy, double t_send_y, double t_send_dx,
                                 int x_slots, int dy_slots);

/* Candidates (1..8 group sizes), window = samples of the moving averages, interval = iterations between
 * evaluations.  Clears the windows, the computation profile and the iteration count; the current k becomes
 * the smallest candidate. */
int kfkb_tuner_config(int window, int interval, const int* candidates, int num_candidates);
/* Stage computation time of one forward / backward under plan k (profiled once, reused afterwards). */
int kfkb_tuner_set_compute_profile(int k, double t_fwd, double t_bwd);
/* One sample per direction (the mean transfer time of one iteration) into the windows; counts an iteration. */
int kfkb_tuner_push_sample(double t_recv_x, double t_recv_dy, double t_send_y, double t_send_dx);
/* Group size of the next iteration: re-evaluated when the number of samples pushed so far is a positive
 * multiple of `interval`, otherwise unchanged.  Candidates above num_microbatches, without a profile, or whose
 * peak of live micro-batches times bytes_per_microbatch exceeds mem_limit (0 = no limit) are skipped.
 * estimates (may be NULL): the estimate of every candidate at the last evaluation, in candidate order,
 * -1 where skipped. */
int kfkb_tuner_next_k(int num_microbatches, int warmup_groups, size_t mem_limit, size_t bytes_per_microbatch,
                      double* estimates, int cap);

/* ---- the stage ------------------------------------------------------------------------- */

/* Optional; must precede stage_init.  Copies *cfg. */
int stage_config(const kfkb_config_t* cfg);

/* Creates the process-global stage.  `weights`: device pointer, one flat buffer in the stage's
 * dtype holding, per block and in this order,
 *   ln1_gamma[H] ln1_beta[H] W_qkv[H,3H] b_qkv[3H] W_o[H,H] b_o[H]
 *   ln2_gamma[H] ln2_beta[H] W_1[H,F] b_1[F] W_2[F,H] b_2[H]
 * matrices [in, out]; QKV columns ordered [Q | K | V], head j owning columns j*d..(j+1)*d of
 * each third, d = hidden / heads.  Borrowed until stage_destroy.
 * Errors: KFKB_E_ARG for a null pointer, a size < 1, hidden % heads != 0, stage_index outside [0, num_stages), or
 * an unsupported shape: hidden > 8192 (any dtype); 16-bit storage needs hidden % 128 == 0, d in {64, 128} and
 * seq * 3 * hidden * 2 bytes < 2 GiB (the attention kernels address a sample's rows with 32-bit byte offsets);
 * fp32 needs hidden % 8 == 0, d <= 128 and seq <= 4096; activation recomputation needs
 * micro_batch * seq * mlp_width % 8 == 0.  KFKB_E_STATE if a stage exists. */
int stage_init(const void* weights, int layers, int hidden, int heads, int seq);

/* Number of parameters of the stage (elements of `weights` and of `grad_accum`). */
size_t stage_param_count(void);

/* Activation bytes of a plan with group size k over num_microbatches (the memory model that
 * run_kFkB admits plans against): peak_live * bytes per micro-batch. */
size_t stage_activation_bytes(int k, int num_microbatches);

/* Device bytes the caller must provide to stage_bind for plans up to group size k_max
 * (activation stash for the peak live count, transfer slots, backward scratch, the
 * re-laid-out weight copy the bf16 kernels read, and, for k_max >= 2, the operands of a
 * W-step window: min(k_max, 8) * layers * 9 b*T*H output-gradient elements). */
size_t stage_workspace_bytes(int k_max);

/* Hands the library its memory.  workspace: device, >= stage_workspace_bytes(k_max) bytes,
 * 256-byte aligned.  grad_accum: device, fp32, stage_param_count() elements, same layout as
 * weights.  host_inputs / host_upstream_grads: pinned host, [max_microbatches][b*T*H] in the
 * stage dtype, read by the receive stream.  host_outputs / host_input_grads: pinned host, same
 * shape, written by the send stream.  All borrowed until stage_destroy. */
int stage_bind(void* workspace, size_t workspace_bytes, float* grad_accum,
               const void* host_inputs, const void* host_upstream_grads,
               void* host_outputs, void* host_input_grads);

/* Injected delay before each transfer of the next runs, nanoseconds, indexed by micro-batch;
 * each array has max_microbatches entries (host memory, copied) or is NULL for no delay.
 * Random delays are drawn by the caller and passed in: the library draws nothing. */
int stage_set_delays(const int64_t* recv_input_ns, const int64_t* recv_upstream_grad_ns,
                     const int64_t* send_output_ns, const int64_t* send_input_grad_ns);

/* Rebuilds the library's re-laid-out weight copy after the caller changed `weights`. */
int stage_refresh_weights(void);

/* Forward task node of micro-batch mb: receive X_mb (if not already received), run the blocks,
 * stash activations, send Y_mb.  KFKB_E_STATE if mb is live or no stash slot is free. */
int stage_forward(int mb);

/* Backward task node of micro-batch mb: receive dY_mb, run the blocks in reverse, add the
 * parameter gradients into grad_accum, send dX_mb, release mb's stash.  KFKB_E_STATE if mb has
 * no live forward. */
int stage_backward(int mb);

/* One iteration: builds the kFkB plan for (k, num_microbatches, this stage's warm-up), checks
 * its activation bytes against mem_limit (bytes of stashed activations; 0 = no limit), then
 * enqueues every op in plan order with receives issued ahead and sends behind.  k <= 0 picks
 * the largest k dividing num_microbatches that fits mem_limit and the bound workspace; the
 * value used is returned by stage_last_k().  Gradients are added to grad_accum (call
 * stage_zero_grads first for a fresh iteration).
 * Errors: KFKB_E_ARG (k > M, M > max_microbatches), KFKB_E_MEMLIMIT (before any GPU work). */
int run_kFkB(int k, int num_microbatches, size_t mem_limit);

int stage_last_k(void);

/* 1 if the library's compute, send and receive streams really run side by side, 0 if the HIP runtime
 * mapped two of them onto one hardware queue (it has 4 per process; every stream the process creates
 * takes a share), in which case delayed transfers serialise and timings, not results, are affected.
 * Measures three 1 ms delay kernels, one per stream; call while the stage is idle. */
int stage_side_streams_overlap(void);
int stage_zero_grads(void);               /* enqueues a fill of grad_accum on the compute stream */
/* Compute lanes.  Default: 2 where one block's matrix products are small enough to leave the chip partly idle
 * (24 * tokens * hidden^2 < 2e12 flops per block forward), 1 above that, where kernels of two streams only take
 * each other's CUs.  run_kFkB admits ops in schedule order, up to `lanes` at a time and only while
 * an activation slot is free, so the plan's peak of live micro-batches (paper sections 3.1, 4.2: larger k holds
 * more activations) is never exceeded; the blocks of the ops in flight are enqueued in turn on one stream per
 * lane.  Independent micro-batches of a group then fill each other's idle phases; k = 1 on the last stage
 * (one live micro-batch) still runs one op at a time.  Results do not depend on the setting: every
 * accumulation into a block's gradients stays in micro-batch order.  With 2 lanes ops overlap in time in
 * stage_get_order.  Call while no micro-batch is live.  Returns the previous setting. */
int stage_set_compute_lanes(int lanes);
/* W steps (beside the chain by default exactly where the default number of lanes is 2): the weight, bias and LayerNorm parameter gradients of a block (the
 * gradient-accumulation task nodes of paper section 2.4) are enqueued on the other lane's stream while that
 * lane has no op of its own, and run beside the chain of input gradients of the following blocks and of the
 * next op; the accumulation order, hence every result bit, is unchanged.  An op's end time in
 * stage_get_order is the end of its chain (dX is complete then).  0 keeps them on the op's own stream.
 * Call while no micro-batch is live.  Returns the previous setting. */
int stage_set_wgrad_stream(int enable);
/* The small reductions of a W step (bias column sums, finishing pass of the LayerNorm parameter sums) ride in the
 * grouped weight-gradient launch on the CUs its tiles leave idle (1, the default) or run as launches of their own
 * (0).  16-bit storage only; the sums are formed in a fixed order either way, but not the same one: results of
 * the two settings agree to fp32 rounding, each is bit-reproducible.  Call while no micro-batch is live.
 * Returns the previous setting. */
int stage_set_fused_w_reductions(int enable);
/* W-step windows.  The backwards of one kFkB schedule unit run back to back, so a 16-bit stage whose shapes allow it
 * (hidden % 128 == 0, tokens per micro-batch % 32 == 0) accumulates the gradients of a block ONCE for up to
 * `max_microbatches` of them (at most 8, the default; never more than the k_max the workspace was sized for): the
 * fp32 gradients are then read and written once per window instead of once per micro-batch, which is what a larger k
 * buys on the compute side.  Every gradient keeps its bits: a weight-gradient tile starts from the accumulator and
 * adds the products of every token on top in token order, whatever the window.  The micro-batches of a window give
 * their activation and input slots back when the window's last W step has been enqueued, not one by one.  1 switches
 * the windows off; a stage with activation recomputation has none (the recomputed tensors would have to be kept for
 * the whole window).  Call while no micro-batch is live.  Returns the previous setting. */
int stage_set_wstep_window(int max_microbatches);
/* Order in which the receive stream is fed (paper Section 5.3: receives of one stream complete one after the other,
 * so the order decides which transfer waits behind which; Section 4.4: inputs sent ahead wait in a queue).
 * 0: the plan's consumption order: the upstream gradients of a schedule unit, then the inputs of the next forward
 * unit.  1: every forward unit's inputs ahead of the upstream gradients of the backward unit before it.  2 (the
 * default): 1 for k = 1, 0 for k >= 2.  Changes timing, never a result.  Process-wide, host-only, also read by
 * kfkb_predict_iteration_ms and the tuner; takes effect at the next run_kFkB.  Returns the previous mode, or
 * KFKB_E_ARG for a mode outside 0 .. 2. */
int kfkb_set_inputs_ahead(int mode);
/* How an output (Y_mb, dX_mb) is copied to the caller's pinned host array once its injected delay has passed (the
 * "send" of paper Section 5.3 on this one GPU): by a copy kernel of the library with `blocks` workgroups (1 .. 4096,
 * default 8) that writes the array through its device view, or, with 0, by the runtime's device-to-host copy.  Arrays
 * that have no device view (not pinned) always take the runtime's copy.  Changes timing, never a result.  Takes
 * effect at the next send.  Returns the previous setting; KFKB_E_STATE before stage_init, KFKB_E_ARG outside the range. */
int stage_set_send_copy_blocks(int blocks);
/* Tile choice of the 16-bit matrix products: 256 x 256 tiles are used where the product divides into at least
 * `tiles` of them (default 192: three quarters of the 256 CUs get a tile), 128 x 128 tiles otherwise.  Process-wide,
 * host-only; returns the previous value.  A product's result does not depend on the tile shape beyond fp32
 * rounding order.  KFKB_E_ARG for tiles < 1. */
int kfkb_set_big_tile_min(int tiles);
/* 128 x 256 tiles for NT products whose B operand is chunk-major (the stage's forward and input-gradient products;
 * K % 64 == 0, N % 256 == 0): mode 0 never, 1 (default) where the shape rates best — share of the CU slots its tiles
 * fill over whole rounds of 256, times `rate_percent` / 100, the rate such a tile reaches of a 256 x 256 tile's (default
 * 90; 128 x 128 tiles count 84) —, 2 wherever they fit.  Process-wide, host-only; returns the previous mode.  A
 * product's result does not depend on the tile shape beyond fp32 rounding order.  KFKB_E_ARG outside the ranges. */
int kfkb_set_mid_tiles(int mode, int rate_percent);
int stage_sync(void);                     /* waits for both compute lanes, the send and the receive stream */
int stage_sync_timeout(double seconds);   /* same, polling; KFKB_E_TIMEOUT if not done in time */
int stage_destroy(void);

/* Executed-order log of the ops enqueued since the last run_kFkB began (or since bind): up to
 * cap entries, returns the count.  Times are resolved from HIP events: call after stage_sync. */
int stage_get_order(kfkb_op_t* out, int cap);

/* Measured transfer times (ms, injected delay + copy, from the moment the stream was free to start it) of the
 * micro-batches of the last iteration: direction 0 receive X, 1 receive dY, 2 send Y, 3 send dX.  Fills
 * out[mb]; returns the number of micro-batches.  Call after stage_sync. */
int stage_get_transfer_ms(int direction, double* out, int cap);

/* Profiles the stage computation of every tuner candidate (paper Section 5.2): `repeats` iterations of
 * `num_microbatches` per candidate with the injected delays switched off, mean forward / backward op times
 * scaled so that they add up to the measured iteration (ops of two lanes overlap).  Accumulates into
 * grad_accum: zero it afterwards.  Blocks until done. */
int stage_tuner_calibrate(int num_microbatches, int repeats);

/* One iteration under the tuner: waits for the previous adaptive iteration, pushes its mean transfer times
 * into the windows, asks kfkb_tuner_next_k (mem_limit as in run_kFkB) and enqueues run_kFkB with that k.
 * Returns the k used, or a negative error. */
int run_kFkB_adaptive(int num_microbatches, size_t mem_limit);

/* Milliseconds from the start of the last run_kFkB to the completion of its last op or
 * transfer, measured with HIP events on the library's streams.  Call after stage_sync. */
double stage_last_run_ms(void);

/* ---- per-kernel timing ------------------------------------------------------------------------ *
 * While enabled, every kernel launch of the library carries a start and a stop HIP event on the     *
 * stream it is launched on (the kernel's own begin / end timestamps).  kfkb_profile(1) clears the   *
 * record and starts collecting, kfkb_profile(0) stops; kfkb_profile_report, called after the work   *
 * has been synchronised, sums launches, milliseconds and algorithmic work per kernel instantiation.  */
typedef struct kfkb_kernel_stat {
  char name[80];        /* kernel template instantiation */
  int bound;            /* what `work` counts: 0 = matrix-core flops, 1 = HBM bytes, 2 = vector-ALU flops */
  long long launches;
  double total_ms;
  double work;          /* summed over the launches */
} kfkb_kernel_stat_t;
int kfkb_profile(int enable);
int kfkb_profile_report(kfkb_kernel_stat_t* out, int cap);

/* ---- the pipeline of S stages, rehearsed on the one GPU (paper Sections 2.2, 3.2.1, 5) ------------------- *
 * The bound stage's L blocks are cut into S consecutive virtual stages of L / S blocks.  Virtual stage v runs
 * its own kFkB plan with w = min(S-1-v, ceil(M/k)) warm-up groups (so earlier stages hold more live
 * micro-batches), forwards a micro-batch after stage v-1 has and backwards it after stage v+1 has.  An
 * activation crosses a boundary as a delayed device-to-device copy on the send stream, a gradient on the
 * receive stream; the delay counts from the moment the producing op finished.  Stage 0 receives X and sends dX,
 * stage S-1 sends Y and receives dY exactly as the single stage does (stage_set_delays).  The result (Y, dX,
 * gradient accumulators) equals that of run_kFkB on the whole stage bit for bit.
 * The GPU issues the ops of all stages in list-schedule order: every stage imagined on a device of its own,
 * forward 1 time unit, backward 2, transfers free; the op that would start earliest goes next, ties go to
 * the later stage (the paper does not say how one executor should order S stages; this is this library's rule). */
typedef struct kfkb_pipe_op {
  int stage;             /* virtual stage, 0 .. S-1 */
  int op;                /* KFKB_OP_F or KFKB_OP_B */
  int mb;                /* micro-batch index */
  double t_start_ms;     /* as in kfkb_op_t; zero from kfkb_pipeline_schedule */
  double t_end_ms;
} kfkb_pipe_op_t;

/* Host only: the 2*S*M ops of one iteration in the order they are issued.  Returns their number or < 0. */
int kfkb_pipeline_schedule(int num_stages, int k, int num_microbatches, kfkb_pipe_op_t* out, int cap);

/* Bytes of device memory the boundary tensors of S stages and M micro-batches need (3 (S-1) M tensors of
 * b*T*H elements and their clock stamps); 0 before stage_init. */
size_t stage_pipeline_bytes(int num_stages, int num_microbatches);

/* Borrows `buffer` (device, 256-byte aligned, >= stage_pipeline_bytes) until the next stage_bind,
 * stage_pipeline_bind or stage_destroy.  Needs stage_bind with a workspace that holds one activation slot per
 * micro-batch (stage_workspace_bytes(M) on a stage configured as the last one), L % S == 0, M <= the
 * configured maximum.  KFKB_E_STATE / _ARG / _MEMLIMIT otherwise. */
int stage_pipeline_bind(void* buffer, size_t bytes, int num_stages, int num_microbatches);

/* Injected delay in ns per boundary crossing: forward_ns[v * M + mb] for the activation of micro-batch mb
 * from stage v to v+1, backward_ns[v * M + mb] for its gradient from v+1 to v, v < S-1; NULL = none.
 * Host arrays, copied. */
int stage_set_pipeline_delays(const int64_t* forward_ns, const int64_t* backward_ns);

/* Enqueues one iteration of the S-stage pipeline with group size k (1 <= k <= M) and returns; stage_sync waits.
 * Accumulates into grad_accum, writes host_outputs and host_input_grads like run_kFkB. */
int run_pipeline_kFkB(int k);

/* The ops of the last run_pipeline_kFkB in the order they were issued, with their measured times.  Call after
 * stage_sync.  Returns the number written. */
int stage_get_pipeline_order(kfkb_pipe_op_t* out, int cap);

/* ---- per-kernel entry points (building blocks, used by unit tests and kernel benchmarks) -- *
 * All pointers are device pointers; dtype is KFKB_F32, KFKB_BF16 or KFKB_F16 (which follows every  *
 * rule stated for bf16) and names the storage type                                            *
 * of every "T" buffer; `stream` is a hipStream_t (NULL = default stream).  Calls enqueue only. */

enum { KFKB_GEMM_NN = 0,   /* C[M,N] = A[M,K] . B[K,N]                       (forward, fp32 only)   */
       KFKB_GEMM_NT = 1,   /* C[M,N] = A[M,K] . B[N,K]^T                     (forward bf16, dgrad)  */
       KFKB_GEMM_TN = 2 }; /* C[M,N] = A[K,M]^T . B[K,N], K = token axis      (wgrad)                */
enum { KFKB_EPI_NONE = 0,       /* C = acc                                                       */
       KFKB_EPI_BIAS = 1,       /* C = acc + bias[n]                                             */
       KFKB_EPI_BIAS_GELU = 2,  /* C = acc + bias[n] (pre-activation), C2 = gelu_tanh(C)         */
       KFKB_EPI_BIAS_RES = 3,   /* C = acc + bias[n] + residual[m,n]                             */
       KFKB_EPI_ACCUM = 4,      /* Cacc[m,n] += acc   (fp32 accumulator, fused gradient add)     */
       KFKB_EPI_GELU_BWD = 5 }; /* C = acc * gelu_tanh'(residual[m,n])   (residual = pre-activation) */

/* bf16: N % 128 == 0, K % 64 == 0 (NT) / M,N % 128 == 0 (TN), any token count. */
int kfkb_op_gemm(int dtype, int kind, int epilogue, int M, int N, int K, const void* A, const void* B,
                 const void* bias, const void* residual, void* C, void* C2, float* Cacc, void* stream);

/* The layout the stage keeps its bf16 weight copies in, and the NT product that reads it (bf16 only).
 * kfkb_op_tile_weights: dst[kc][n][kk] = B[n][32 kc + kk], kc < K / 32, kk < 32, where B[N, K] is src itself
 * (transposed == 0) or the transpose of src[K, N] (transposed != 0); N % 8 == 0, K % 32 == 0; src and dst are
 * distinct device buffers of N * K bf16 values.
 * kfkb_op_gemm_nt_tiled: kfkb_op_gemm(KFKB_BF16, KFKB_GEMM_NT, ...) with B given in that layout (Bt);
 * N % 128 == 0, K % 64 == 0, any M.  Both enqueue only; a bad argument returns KFKB_E_ARG and launches nothing. */
int kfkb_op_tile_weights(const void* src, void* dst, int N, int K, int transposed, void* stream);
int kfkb_op_gemm_nt_tiled(int epilogue, int M, int N, int K, const void* A, const void* Bt, const void* bias,
                          const void* residual, void* C, void* C2, float* Cacc, void* stream);

/* y = LN(x) over H per row; mean, rstd: fp32 [rows]. */
int kfkb_op_layernorm_fwd(int dtype, const void* x, const void* gamma, const void* beta, void* y,
                          float* mean, float* rstd, int rows, int H, float eps, void* stream);

/* dx = LN-backward(dy) + dres (dres may be NULL); dgamma += sum_rows dy*xhat, dbeta += sum_rows dy.
 * scratch: fp32, kfkb_op_reduce_scratch_floats(H) elements. */
int kfkb_op_layernorm_bwd(int dtype, const void* dy, const void* x, const float* mean, const float* rstd,
                          const void* gamma, const void* dres, void* dx, float* dgamma, float* dbeta,
                          float* scratch, int rows, int H, void* stream);

/* out[n] += sum_rows dy[rows, N]  (bias gradient).  scratch as above with H = N. */
int kfkb_op_colsum_accum(int dtype, const void* dy, float* out, float* scratch, int rows, int N, void* stream);
size_t kfkb_op_reduce_scratch_floats(int width);

/* kfkb_op_colsum_accum for callers that cannot allocate device memory: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  The same two kernels; the partial sums of the first pass go to a
 * 16 MiB array built into the library (one copy per GPU, held until the process ends) instead of a buffer of the
 * caller's.  dy: device, [rows, N] in `dtype`; out: device, fp32 [N], added to.  N % 8 == 0 and N <= 32768,
 * otherwise KFKB_E_ARG and nothing is launched.  Calls no hipMalloc / hipFree (kfkb_profile must be off: timing
 * creates events).  Nothing has to be cleared between calls (the first pass rewrites every entry the second
 * reads), but all calls on one GPU share the one array: two calls whose kernels may overlap on that GPU (different
 * streams, no ordering between them) race.  Enqueues only. */
int kfkb_op_colsum_accum_static(int dtype, const void* dy, float* out, int rows, int N, void* stream);

/* du = dg * gelu_tanh'(u), n elements. */
int kfkb_op_gelu_bwd(int dtype, const void* dg, const void* u, void* du, size_t n, void* stream);

/* Attention over qkv [b*T, 3H] (columns [Q|K|V], head-major inside each third):
 * o [b*T, H], lse fp32 [b, heads, T] = log-sum-exp of the scaled, masked scores.  16-bit storage: head size 64 or
 * 128 and T * 3 * H * 2 bytes < 2 GiB; fp32: head size <= 128, T <= 4096; otherwise KFKB_E_ARG. */
int kfkb_op_attention_fwd(int dtype, const void* qkv, void* o, float* lse, int b, int T, int H, int heads,
                          int causal, void* stream);

/* dqkv [b*T, 3H] from do [b*T, H]; needs o and lse of the forward; dsum: fp32 scratch [b, heads, T]. */
int kfkb_op_attention_bwd(int dtype, const void* qkv, const void* o, const void* d_o, const float* lse,
                          float* dsum, void* dqkv, int b, int T, int H, int heads, int causal, void* stream);

/* out[c, r] = in[r, c] for a [rows, cols] matrix of the given dtype. */
int kfkb_op_transpose(int dtype, const void* in, void* out, int rows, int cols, void* stream);

/* One-wave kernel that returns after `ns` nanoseconds of device wall clock (transfer delay). */
int kfkb_op_delay(int64_t ns, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* KFKB_H */
