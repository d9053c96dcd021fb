/*
 * pmc.h - C ABI of the pipeline-stage library ("pipeline parallelism with controllable memory").
 *
 * One pipeline stage's work for one microbatch is split, as in Section 2.1 of the paper, into
 *   F  forward pass,
 *   B  backward for the activations (gradient w.r.t. the stage input),
 *   W  backward for the weights (may be deferred),
 * and a schedule is the per-device order of such passes obtained by repeating a building block
 * (Section 2).  This library runs F, B and W of a chunk of pre-LayerNorm GPT layers as HIP kernels
 * for gfx950, generates the 1F1B / V-ZB / V-Half / V-Min orders (Section 3, Table 1, Appendix F),
 * and replays a whole schedule on one GPU stream while an activation pool does the lifetime
 * bookkeeping of Section 2.2 (a unit is allocated when F starts and retained until both B and W
 * have consumed it).
 *
 * Conventions
 *  - Every function returns PMC_OK (0) or a negative pmc_status; nothing throws or aborts.
 *    pmc_last_error() returns a thread-local, human-readable description of the last failure.
 *  - Pointers named "device" are GPU memory, BORROWED from the caller: the library never allocates
 *    or frees device memory.  Everything else is host memory.
 *  - Work is enqueued on the HIP stream given to pmc_create and is asynchronous unless stated.
 *    One exception inside a call: the bf16 W pass runs every second weight-gradient product and the
 *    bias-gradient column sums on a second, non-blocking stream of default priority that the
 *    context owns (created at first use).  The pass forks it from the context's stream with an
 *    event when it starts and joins it back before it returns (also when a launch fails), so
 *    everything the caller enqueues on the context's stream before or after the call is ordered
 *    against all of the pass's work; nothing is ever left running on the second stream between
 *    calls.  pmc_tuning_set("w_streams", 1) keeps the whole pass on the context's stream, and so
 *    does tracing (pmc_trace_begin), whose per-operation events assume one stream: traced W times
 *    are therefore those of the one-stream configuration.
 *  - Tensors are row-major.  Activations are [tokens, hidden] with tokens = microbatch * seq
 *    (sequences of one microbatch stored back to back).  Storage type is float (PMC_F32) or
 *    bfloat16 (PMC_BF16; all accumulation in fp32).  Gradients of parameters are always fp32.
 *  - Layer (Section 4.1 says GPT-like; details are this library's stated reading): pre-LN block,
 *    LayerNorm with biased variance and eps inside the root, tanh-form GeLU, biases on the four
 *    linear maps, optional causal mask, no dropout.  Packed qkv columns are [q | k | v], each with
 *    the heads' slices side by side.
 *  - Parameter order per layer (PMC_PARAMS_PER_LAYER pointers, layer after layer):
 *      0 ln1_gain[h] 1 ln1_bias[h] 2 w_qkv[h,3h] 3 b_qkv[3h] 4 w_o[h,h] 5 b_o[h]
 *      6 ln2_gain[h] 7 ln2_bias[h] 8 w_1[h,ffn] 9 b_1[ffn] 10 w_2[ffn,h] 11 b_2[h]
 *    Weights are stored [in, out].  Gradient buffers have the same shapes in fp32 and are
 *    ACCUMULATED into (never cleared) by B (LayerNorm gain/bias) and W (weights and biases).
 */
#ifndef PMC_H
#define PMC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PMC_PARAMS_PER_LAYER 12

typedef enum pmc_status {
  PMC_OK = 0,
  PMC_ERR_INVALID = -1,     /* bad argument or unsupported shape                              */
  PMC_ERR_STATE = -2,       /* pass order violated: B before F, W before B, live id reused    */
  PMC_ERR_NOMEM = -3,       /* activation pool or workspace too small / exhausted             */
  PMC_ERR_HIP = -4,         /* a HIP runtime call failed                                      */
  PMC_ERR_ILLEGAL_BLOCK = -5 /* building block collides when repeated (Section 2.3)           */
} pmc_status;

typedef enum pmc_dtype { PMC_F32 = 0, PMC_BF16 = 1 } pmc_dtype;
typedef enum pmc_kind {
  PMC_1F1B = 0, PMC_VZB = 1, PMC_VHALF = 2, PMC_VMIN = 3,
  PMC_1F1BV = 4 /* Appendix H: V-shape placement with B and W fused; about 2/3 of 1F1B's peak */
} pmc_kind;
typedef enum pmc_op { PMC_F = 0, PMC_B = 1, PMC_W = 2 } pmc_op;

typedef struct pmc_ctx pmc_ctx;
typedef struct pmc_chunk pmc_chunk;
typedef struct pmc_schedule pmc_schedule;

typedef struct pmc_chunk_cfg {
  int32_t layers, hidden, heads, ffn, seq, microbatch;
  int32_t dtype;  /* pmc_dtype */
  int32_t causal; /* 1 = causal mask */
  float ln_eps;
} pmc_chunk_cfg;

/* One pass of a schedule.  `chunk` is 0 or 1 (which of the device's two chunks), `model_chunk`
 * its position in the model (0 .. 2d-1), `time` its cell in the repeated, unsqueezed grid. */
typedef struct pmc_pass {
  int32_t time, device, op, chunk, mb, model_chunk;
} pmc_pass;

typedef struct pmc_device_peak {
  int64_t peak_live_units;   /* paper's unit count (Section 2.2)                               */
  int64_t peak_live_bytes;   /* pool bytes: units * unit size                                  */
  int64_t peak_tensor_bytes; /* bytes of tensors alive at pass boundaries (fp32 statistics die
                                when B ends, the rest when W ends)                             */
} pmc_device_peak;

typedef struct pmc_replay_report {
  double ms_total;          /* wall time of the replayed iteration on the stream               */
  double ms_f, ms_b, ms_w;  /* summed per-pass times (only with PMC_REPLAY_TIME_PASSES)        */
  int32_t passes;           /* number of chunk passes executed                                 */
  int32_t devices;          /* d                                                               */
  int64_t transit_peak_bytes; /* inter-chunk activation/gradient buffers in flight (workspace) */
} pmc_replay_report;

#define PMC_REPLAY_TIME_PASSES 1u

const char* pmc_last_error(void);

/* Tuning switches, process-wide (tests, kernel tuning): value -1 = the library decides.
 *   "gemm_tile" 0..4 (256x256, 256x128, 128x128, 64x128, 256x320)   "gemm_group" 1..64 (tile walk)
 *   "gemm_wgrad" 0..2 (W product: plain tiles, persistent 256x256 walk, two 256x128 workgroups per unit)
 *   "attn_shape" 0..2 (launch family)   "w_streams" 1|2
 * The environment variables PMC_GEMM_TILE, PMC_GEMM_GROUP, PMC_GEMM_WGRAD, PMC_ATTN_SHAPE,
 * PMC_W_STREAMS give the initial values; they are read once, at the first use of any switch, never
 * on a launch path.  PMC_ERR_INVALID for an unknown name or a
 * value out of range. */
int pmc_tuning_set(const char* name, int32_t value);
int pmc_tuning_get(const char* name, int32_t* value);

/* ---- context, pool, workspace --------------------------------------------------------------- */

/* Creates a context bound to `hip_stream` (a hipStream_t, borrowed; NULL = default stream) on
 * the current device.  Host-only call. */
int pmc_create(void* hip_stream, pmc_ctx** out);
void pmc_destroy(pmc_ctx* ctx);

/* Attaches the activation pool: `arena` (device, >= 256-byte aligned, borrowed) of `bytes` bytes is
 * cut into slabs of `slab_bytes` (rounded up to 256).  One slab holds everything one
 * (chunk, microbatch) keeps between its F and its W (Section 2.2's activation unit, Section 3.1's
 * m).  Fails with PMC_ERR_STATE if slabs are in use. */
int pmc_pool_attach(pmc_ctx* ctx, void* arena, size_t bytes, size_t slab_bytes);
/* Slabs in use / high-water mark since attach (or since the last pmc_pool_reset_peak). */
int64_t pmc_pool_live_slabs(const pmc_ctx* ctx);
int64_t pmc_pool_peak_slabs(const pmc_ctx* ctx);
void pmc_pool_reset_peak(pmc_ctx* ctx);

/* Attaches scratch memory (device, 256-byte aligned, borrowed) used for transient tensors inside
 * a pass and for the replayer's inter-chunk buffers.  Contents are undefined between calls. */
int pmc_workspace_attach(pmc_ctx* ctx, void* workspace, size_t bytes);

/* ---- chunks ------------------------------------------------------------------------------- */

/* m: bytes one (chunk, microbatch) unit holds from F to W: per layer 16 [tokens, hidden] tensors of
 * the storage type plus fp32 statistics (4 + heads values per token).  Returns 0 on a bad cfg. */
size_t pmc_activation_bytes(const pmc_chunk_cfg* cfg);
/* The fp32-statistics part of the above (dead once B has run). */
size_t pmc_activation_stats_bytes(const pmc_chunk_cfg* cfg);
/* Scratch bytes one pass of such a chunk needs in the workspace. */
size_t pmc_pass_workspace_bytes(const pmc_chunk_cfg* cfg);

/* Creates a chunk of cfg->layers identical layers.  Constraints: hidden % heads == 0, head size
 * <= 128 (multiples of 8 take the matrix-core attention kernels in bf16 mode); hidden, ffn and tokens
 * multiples of 8 with hidden <= 12288 in bf16 mode, multiples of 4 with hidden <= 4096 in fp32
 * mode.  Host-only call. */
int pmc_chunk_create(pmc_ctx* ctx, const pmc_chunk_cfg* cfg, pmc_chunk** out);
void pmc_chunk_destroy(pmc_chunk* chunk);
/* Binds parameters and gradient accumulators: arrays of layers * PMC_PARAMS_PER_LAYER device
 * pointers (params in the storage type, grads fp32), both borrowed until the chunk is destroyed. */
int pmc_chunk_bind(pmc_chunk* chunk, const void* const* params, void* const* grads_fp32);

/* F (Section 2.1): y = chunk(x) for microbatch id `mb`; takes one slab from the pool at its start.
 * x, y: device, [tokens, hidden], storage type.  PMC_ERR_STATE if `mb` is already live in this
 * chunk, PMC_ERR_NOMEM if the pool has no free slab. */
int stage_forward(pmc_chunk* chunk, int32_t mb, const void* x, void* y);
/* As stage_forward, but the caller names the simulated device the slab is charged to. */
int stage_forward_on(pmc_chunk* chunk, int32_t mb, const void* x, void* y, int32_t device);

/* B (Section 2.1): dx = d loss / d x given dy = d loss / d y, for a microbatch whose F has run.
 * Adds the LayerNorm gain/bias gradients into the bound accumulators and leaves in the slab what
 * W needs.  PMC_ERR_STATE if F has not run or B already has. */
int stage_backward_input(pmc_chunk* chunk, int32_t mb, const void* dy, void* dx);

/* W (Section 2.1): adds the weight and bias gradients of the `count` listed microbatches (each
 * must have had its B) into the bound fp32 accumulators and returns their slabs to the pool.
 * count > 1 is the deferred, queued case (Section 2.1: W "can be deferred").  In bf16 mode queued
 * microbatches are contracted together, PMC_MAX_QUEUED_W at a time in list order: each weight
 * gradient is ONE product dW += [X_1; X_2; ...]^T . [dY_1; dY_2; ...] over the concatenated token
 * axis, so the fp32 accumulator is read and written once per group instead of once per
 * microbatch.  The sum is the same up to fp32 summation order (the microbatches are added inside
 * the matrix-core accumulators before the one addition into dW), so a queued W and `count` single
 * ones agree to rounding, not bit for bit; fp32 mode runs the microbatches one after the other. */
#define PMC_MAX_QUEUED_W 8
int stage_backward_weight(pmc_chunk* chunk, const int32_t* mbs, int32_t count);

/* Gives up a live microbatch of the chunk in whatever state it is (after F, after B, or reserved)
 * and returns its slab to the pool: the way back to a clean pool after a pass has failed part-way.
 * A pass that fails never leaves a half-taken unit behind by itself: stage_forward returns the
 * slab it took, stage_backward_input and stage_backward_weight leave the microbatch in the state
 * it had (its slab contents are then undefined: abandon it).  A failed schedule_replay returns
 * every unit it still held.  Host-only; work already enqueued for the microbatch still runs, in
 * stream order, before anything that reuses the slab.  PMC_ERR_STATE if `mb` is not live. */
int stage_abandon(pmc_chunk* chunk, int32_t mb);

/* ---- schedules (host only; no GPU needed) --------------------------------------------------- */

/* Builds the pass orders of `kind` for d devices and n microbatches by laying out the building
 * block (Table 1 offsets; Appendix F same-device offsets; V-ZB's same-device offsets, which the
 * paper finds by brute force and does not print, are (1,1,1)), checking that it repeats every 6
 * cells without collision (Section 2.3) and repeating it n times (Section 2).  d >= 1, n >= 1.
 * PMC_1F1BV (Appendix H's 1F1B-V: the V-shape placement with a chunk's B and W run as one pass) is
 * this library's construction, the paper prints no offsets for it: every pass sits at the first
 * cell at or after the end of the pass it depends on that is free modulo 6 on its device and leaves
 * room for the device's remaining passes; the forward's turn on the last device is delayed by the
 * 0..5 cells that give the least peak, then the least unit-time makespan.  Its peak is
 * ceil((4d + 2) / 3) units per device against 1F1B's 2d, at 1F1B's bubble count. */
int pmc_schedule_build(int32_t kind, int32_t d, int32_t n, pmc_schedule** out);
/* As above for an arbitrary V-shape block: cross-device offsets delta0, delta1 (Section 3.1) and
 * the three same-device offsets (F turn on the last device, F->B turn on the first device, B turn
 * on the last device).  PMC_ERR_ILLEGAL_BLOCK if it collides. */
int pmc_schedule_build_vshape(int32_t d, int32_t n, int32_t delta0, int32_t delta1, int32_t turn_f,
                              int32_t turn_fb, int32_t turn_b, pmc_schedule** out);
void pmc_schedule_destroy(pmc_schedule* s);
int32_t pmc_schedule_devices(const pmc_schedule* s);
int32_t pmc_schedule_microbatches(const pmc_schedule* s);
int32_t pmc_schedule_num_passes(const pmc_schedule* s); /* 6 * n * d */
/* Cell index of each pass of microbatch 0: out[6][d] in the row order F0, F1, B1, B0, W1, W0. */
int pmc_schedule_block(const pmc_schedule* s, int32_t* out, int32_t capacity);
/* The optional third step of the construction (Section 2 "Reordering", Appendix C): a new schedule
 * in which, on the squeezed grid at unit pass times, warm-up bubbles before a device's first B are
 * filled with later passes of that device (refused where the device's peak of live units would
 * rise) and the W passes after a device's last F are re-placed into the bubbles of the cool-down,
 * each after its own B.  The `time` of the result's passes is their cell in the final squeezed
 * grid; per-device and global orders, accounting, makespan and replay take it like any schedule.
 * A 1F1B schedule (fused B and W) is returned squeezed, its orders unchanged.  Host-only; the
 * caller destroys *out. */
int pmc_schedule_reorder(const pmc_schedule* s, pmc_schedule** out);
/* Adaptive V-shape scheduler (Appendix A): minimises the finish time under an activation-memory
 * limit.  Search space: the split K (first K devices / the rest), the four offsets
 * delta^0_{<K}, delta^1_{<=K}, delta^0_{>=K}, delta^1_{>K} in 1..max_delta, and the three
 * same-device offsets in 1..6 (the residues of the first device's passes).  A block is dropped if
 * it collides when repeated or if some device's peak of live units over the n microbatches exceeds
 * limit_units (units of one chunk's activation, m = M / 2d); the others are squeezed, reordered if
 * `reorder` is non-zero, and timed with t_f, t_b, t_w; the first block (loops nested in the order
 * of pmc_search_result's fields) with the least finish time wins.  Host-only, allocates host memory
 * only; cost grows as d * max_delta^4 * 216 blocks.  Returns PMC_ERR_ILLEGAL_BLOCK if no block
 * fits the limit.  result may be NULL; the caller destroys *out. */
typedef struct pmc_search_result {
  int32_t split, delta0_lo, delta1_lo, delta0_hi, delta1_hi, turn_f, turn_fb, turn_b;
  int64_t peak_units;   /* largest per-device peak of the winning block                        */
  double makespan;      /* its finish time with the given pass times                            */
  int64_t candidates;   /* blocks visited                                                       */
  int64_t feasible;     /* of those: collision-free and within the limit                        */
} pmc_search_result;
int pmc_schedule_search(int32_t d, int32_t n, int64_t limit_units, double t_f, double t_b, double t_w,
                        int32_t max_delta, int32_t reorder, pmc_search_result* result, pmc_schedule** out);
/* One device's order (6n passes), sorted by cell; squeezing keeps this order (Section 2). */
int pmc_schedule_device_order(const pmc_schedule* s, int32_t device, pmc_pass* out, int32_t capacity);
/* The one-stream replay order: all passes by (cell, device). */
int pmc_schedule_global_order(const pmc_schedule* s, pmc_pass* out, int32_t capacity);
/* Lifetime accounting without running anything (Section 2.2): out[d]. */
int pmc_schedule_account(const pmc_schedule* s, int64_t unit_bytes, int64_t stats_bytes,
                         pmc_device_peak* out, int32_t capacity);
/* Finish time when every device runs its order as early as dependencies allow, with the given
 * pass durations (Section 2 "squeezing"; Appendix E). */
int pmc_schedule_makespan(const pmc_schedule* s, double t_f, double t_b, double t_w, double* out);

/* ---- replay ---------------------------------------------------------------------------------- */

/* Workspace bytes schedule_replay needs for chunks of this shape (pass scratch + the largest
 * number of inter-chunk buffers the order ever has in flight). */
size_t pmc_replay_workspace_bytes(const pmc_schedule* s, const pmc_chunk_cfg* cfg);

/* Runs one training iteration of the schedule on the context's stream: every pass of the global
 * order, chunk by chunk, with activations handed from chunk to chunk through workspace buffers.
 *   chunks     2d chunks in model order, all of one shape, bound to their parameters
 *   x          n device pointers: input of model chunk 0 per microbatch
 *   dy_last    n device pointers: gradient w.r.t. the last chunk's output per microbatch
 *   y_last     n device pointers or NULL: receives the last chunk's output
 *   dx_first   n device pointers or NULL: receives the gradient w.r.t. x
 *   peaks      d entries: per simulated device, measured from the pool's own alloc/free calls
 * Synchronises the stream before returning.  A 1F1B stage takes both its chunks' slabs when its F
 * starts and returns them when its fused backward ends. */
int schedule_replay(pmc_ctx* ctx, const pmc_schedule* s, pmc_chunk* const* chunks,
                    const void* const* x, const void* const* dy_last, void* const* y_last,
                    void* const* dx_first, uint32_t flags, pmc_replay_report* report,
                    pmc_device_peak* peaks, int32_t peaks_capacity);

/* ---- per-operation timing (profiling the passes, as the paper profiles F/B/W for its
 *      scheduler, Appendix D.1) -------------------------------------------------------------- */

typedef enum pmc_trace_op {
  PMC_OP_GEMM = 0, PMC_OP_LN_FWD = 1, PMC_OP_LN_BWD = 2, PMC_OP_ATTN_FWD = 3, PMC_OP_ATTN_BWD = 4,
  PMC_OP_COLSUM = 5, PMC_OP_COPY = 6
} pmc_trace_op;

typedef struct pmc_trace_rec {
  int32_t op;        /* pmc_trace_op                                                          */
  int32_t pass;      /* pmc_op of the pass that launched it                                    */
  int32_t m, n, k;   /* GEMM: problem size; attention: tokens, heads, head size; else rows, cols, 0 */
  int32_t variant;   /* GEMM: trans_a | trans_b << 1 | epilogue << 2; else 0                   */
  float ms;          /* elapsed time between HIP events recorded around the operation          */
} pmc_trace_rec;

/* From this call on, every operation the passes launch is bracketed by a pair of HIP events on
 * the context's stream (up to `capacity` operations; later ones are not recorded). */
int pmc_trace_begin(pmc_ctx* ctx, int32_t capacity);
/* Synchronises the stream, writes up to `capacity` records to `out`, stores the number recorded in
 * *count, and stops tracing. */
int pmc_trace_end(pmc_ctx* ctx, pmc_trace_rec* out, int32_t capacity, int32_t* count);

/* ---- single operations (unit parity tests and kernel timing) --------------------------------- */

typedef enum pmc_epilogue {
  PMC_EPI_NONE = 0,        /* C = A.B                                                         */
  PMC_EPI_BIAS = 1,        /* C = A.B + bias[n]                                               */
  PMC_EPI_BIAS_RESID = 2,  /* C = A.B + bias[n] + resid[m,n]                                  */
  PMC_EPI_BIAS_GELU = 3,   /* C = A.B + bias[n]; aux = gelu(C)                                */
  PMC_EPI_DGELU = 4,       /* C = (A.B) * gelu'(aux[m,n])  (C may alias aux)                  */
  PMC_EPI_ACCUM_F32 = 5,   /* C(fp32) += A.B                                                  */
  PMC_EPI_BIAS_GELU_GRAD = 6, /* u = A.B + bias[n]; C = gelu'(u); aux = gelu(u)  (what F keeps of FC1) */
  PMC_EPI_MUL = 7          /* C = (A.B) * aux[m,n]  (C may alias aux)                         */
} pmc_epilogue;

/* C[M,N] = op(A)[M,K] . op(B)[K,N] with the epilogue above.  trans_a = 0: A stored [M,K]
 * (row pitch lda); 1: stored [K,M].  trans_b = 0: B stored [K,N]; 1: stored [N,K].  All device.
 * bf16 mode needs M, N, K multiples of 64 and pitches multiples of 8. */
int pmc_gemm(pmc_ctx* ctx, int32_t dtype, int32_t trans_a, int32_t trans_b, int32_t M, int32_t N,
             int32_t K, const void* A, int32_t lda, const void* B, int32_t ldb, void* C, int32_t ldc,
             int32_t epilogue, const void* bias, const void* resid, void* aux);

/* C[M,N] (fp32) += sum over i < count of A_i^T . B_i, with A_i stored [K,M] (row pitch lda) and
 * B_i stored [K,N] (row pitch ldb), bf16, all device; a, b: host arrays of `count` device pointers
 * (1 <= count <= PMC_MAX_QUEUED_W).  One product over the concatenated K axis: the kernel behind
 * the queued W pass.  M, N multiples of 8, K (of one piece) a multiple of 64. */
int pmc_gemm_grouped_wgrad(pmc_ctx* ctx, int32_t M, int32_t N, int32_t K, int32_t count,
                           const void* const* a, int32_t lda, const void* const* b, int32_t ldb,
                           float* C, int32_t ldc);

/* y = LayerNorm(x) over rows of length h (a multiple of 4 up to 6144 in fp32, of 8 up to 12288 in
 * bf16); mean and rstd are fp32 [rows]; x_copy (may be NULL) receives a copy of x. */
int pmc_layernorm_forward(pmc_ctx* ctx, int32_t dtype, int32_t rows, int32_t h, const void* x,
                          const void* gain, const void* bias, float eps, void* y, float* mean,
                          float* rstd, void* x_copy);
/* dx = resid + LayerNorm input-gradient of dy (resid may be NULL); dgain/dbias (fp32 [h]) are
 * accumulated into.  Uses the attached workspace.  dx may alias x. */
int pmc_layernorm_backward(pmc_ctx* ctx, int32_t dtype, int32_t rows, int32_t h, const void* dy,
                           const void* x, const void* gain, const float* mean, const float* rstd,
                           const void* resid, void* dx, float* dgain, float* dbias);
/* For callers that cannot allocate device memory or attach a workspace (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): pmc_layernorm_backward with its
 * scratch (one row of 2h fp32 partial sums per workgroup, at most 512 workgroups) in a 32 MiB
 * device array built into the library, PMC_LAYERNORM_STATIC_SCRATCH_BYTES; each GPU the library
 * runs on holds its own copy until the process ends.  Same arguments, same kernels, same results
 * bit for bit; needs no workspace and calls no allocating routine.  Returns PMC_ERR_NOMEM, and
 * launches nothing, when min(rows, 512) * 2h * 4 bytes exceed the array (h > 8192 with 512 or
 * more rows).  All calls on one GPU share the array, so two calls that overlap in time on one GPU
 * (different streams or host threads) race; calls on one stream are ordered and safe. */
#define PMC_LAYERNORM_STATIC_SCRATCH_BYTES ((size_t)32 << 20)
int pmc_layernorm_backward_static(pmc_ctx* ctx, int32_t dtype, int32_t rows, int32_t h, const void* dy,
                                  const void* x, const void* gain, const float* mean, const float* rstd,
                                  const void* resid, void* dx, float* dgain, float* dbias);
/* Fused attention on packed qkv [batch*seq, 3h]: o [batch*seq, h], lse fp32 [batch, heads, seq].
 * In bf16 with a head size that is a multiple of 8 (the matrix-core kernels) one sequence's rows, seq * 3h * 2
 * bytes, must stay below 2 GB; larger shapes return PMC_ERR_INVALID (also from pmc_chunk_create). */
int pmc_attention_forward(pmc_ctx* ctx, int32_t dtype, int32_t batch, int32_t seq, int32_t heads,
                          int32_t head_dim, int32_t causal, const void* qkv, void* o, float* lse);
/* dqkv (same layout as qkv; may alias qkv) from d_o; uses the workspace. */
int pmc_attention_backward(pmc_ctx* ctx, int32_t dtype, int32_t batch, int32_t seq, int32_t heads,
                           int32_t head_dim, int32_t causal, const void* qkv, const void* o,
                           const float* lse, const void* d_o, void* dqkv);
/* out[n] += column sums of a [rows, n] (fp32 out). */
int pmc_column_sum(pmc_ctx* ctx, int32_t dtype, int32_t rows, int32_t n, const void* a, int32_t lda,
                   float* out);

#ifdef __cplusplus
}
#endif
#endif /* PMC_H */
