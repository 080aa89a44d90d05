/*
 * ccfused — fused gradient-reduce + mixed-precision Adam / LAMB step on one GPU's parameter shard
 * (MI355X, gfx950).  C ABI: plain pointers and sizes, no C++ or framework types.
 *
 * The operation is the data-parallel parameter update of the paper (Fig. 4a: all-reduce of the
 * gradients with "+", then the Adam moments, bias corrections and parameter update) after the
 * schedule of Fig. 4b has been applied: the all-reduce is split into reduce-scatter + all-gather,
 * the all-gather is moved behind the update, m and v live only on the owning rank, and the
 * reduce, the update and the emission of the new fp16 parameters are fused into one kernel
 * (Section 3.3 "AllReduce Fuse", Section 5.2).  This library is the compute side of that fused
 * kernel on ONE rank: the R incoming fp16 gradient slices are R device buffers, the reduced value
 * never goes through memory, and the new parameters are written once as fp32 master weights and
 * once as the fp16 values that would be all-gathered.  Tensors are scattered (one buffer per
 * layer) and indexed through a chunk table built once on the host (Section 5.4).
 *
 * Conventions
 *   - "device" pointers are HIP device memory on the current device, owned by the caller.
 *   - fp16 data is passed as uint16_t bit patterns (IEEE binary16).
 *   - Every call returns CC_OK (0) or a negative cc_status; nothing throws.  cc_last_error() gives a
 *     thread-local message for the last failing call on this thread.
 *   - Step calls are asynchronous: they enqueue kernels on `hip_stream` (a hipStream_t passed as
 *     void*, NULL = the default stream); they never synchronise and never allocate, so every step
 *     call can be captured into a HIP graph.  Arguments are validated on the host before anything
 *     is enqueued; a rejected call enqueues nothing.
 *   - A plan may be used by one stream at a time: its scratch buffers are shared by all of its calls.
 */
#ifndef CCFUSED_H
#define CCFUSED_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif
#if defined(__GNUC__)
#pragma GCC visibility push(default)   /* the library itself is built with hidden visibility: only these are exported */
#endif

#define CC_MAX_R 16            /* most gradient slices one element can be reduced from */
#define CC_VERSION 200

typedef enum cc_status {
    CC_OK = 0,
    CC_ERR_NULL = -1,          /* a required pointer is NULL */
    CC_ERR_ARG = -2,           /* a count, size or hyper-parameter is out of range */
    CC_ERR_ALIGN = -3,         /* a tensor base pointer is not 16-byte aligned */
    CC_ERR_ALIAS = -4,         /* in/out buffers alias in a mode that forbids it */
    CC_ERR_HIP = -5,           /* a HIP runtime call failed (no device, out of memory, launch error) */
    CC_ERR_NOMEM = -6          /* host allocation failed */
} cc_status;

/*
 * One tensor of the shard (the p, g, m, v of Fig. 4, restricted to this rank's slice).
 * All pointers are device pointers to `numel` elements and must be 16-byte aligned (numel == 0:
 * pointers are ignored).  w/m/v outputs may be the same buffers as the inputs (in place) or
 * different ones (out of place, so that a skipped step leaves the inputs untouched).  Any other
 * overlap that involves an output is an error (CC_ERR_ALIAS), within a tensor and across the
 * tensors of a plan: two output buffers, or an output with w_in/m_in/v_in/grad[r] other than its
 * own in-place input.  Inputs may overlap inputs.  Only grad[0..R-1] are read.
 */
typedef struct cc_tensor {
    uint64_t        numel;
    const float    *w_in;              /* fp32 master weights before the step */
    const float    *m_in;              /* first moment  */
    const float    *v_in;              /* second moment */
    float          *w_out;             /* fp32 master weights after the step */
    float          *m_out;
    float          *v_out;
    uint16_t       *w16_out;           /* fp16 copy of w_out, round to nearest even (what is all-gathered) */
    const void     *grad[CC_MAX_R];    /* R gradient slices, one per contributing rank: fp16 bit patterns, or fp32
                                          values when the plan is created with CC_GRAD_F32 */
    float           weight_decay;      /* per tensor (0 for bias / LayerNorm) */
} cc_tensor;

/*
 * Scalars of one step (lr, beta1, beta2, t of Fig. 4a; epsilon, decay, loss scale as in standard
 * mixed-precision training).  The fp32 values given here are the definition: bias corrections
 * 1 - beta^step are formed from them in double on the host.
 */
typedef struct cc_hparams {
    float   lr;
    float   beta1;             /* in [0, 1) */
    float   beta2;             /* in [0, 1) */
    float   eps;               /* >= 0; added to the root of the bias-corrected second moment */
    float   loss_scale;        /* > 0, finite; the reduced gradient is divided by it once */
    int32_t step;              /* t, 1-based */
    int32_t grad_average;      /* 0: sum of the R slices; 1: also divide by R */
    int32_t adam_mode;         /* 1: decoupled weight decay (u += wd*w); 0: L2 (g += wd*w). LAMB: 1 only */
    int32_t skip_mode;         /* 0: whole-step skip on overflow, needs out buffers distinct from in
                                     buffers; the caller adopts the out buffers only if the flag is 0.
                                  1: per-element guard: an element whose reduced gradient is inf/NaN
                                     keeps its w, m, v; allowed in place.  LAMB: 0 only */
} cc_hparams;

/* Element type of the incoming gradient slices.  fp16 is the mixed-precision case the paper evaluates; fp32 is
 * its "Float 32" case (Section 6.1.1).  With fp32 slices the flag also rises when a finite sum overflows fp32. */
typedef enum cc_grad_dtype { CC_GRAD_F16 = 0, CC_GRAD_F32 = 1 } cc_grad_dtype;

typedef struct cc_plan cc_plan;   /* opaque: device copy of the tensor list, chunk table, scratch */

/* ---- host-only helpers of the chunk table (Section 5.4); no device is touched ---- */

/* Number of chunks a tensor list needs: sum over tensors of ceil(numel / chunk_elems).
 * chunk_elems must be a positive multiple of 1024 (0 selects the default). Returns < 0 on error. */
int64_t cc_chunk_count(const uint64_t *numels, int32_t T, int32_t chunk_elems);

/* Fills `table` (host memory, capacity entries of 2 x uint32: tensor index, chunk index inside the
 * tensor) in tensor order.  Returns the number of entries written, or < 0 on error / too small. */
int64_t cc_chunk_table_fill(const uint64_t *numels, int32_t T, int32_t chunk_elems,
                            uint32_t *table, int64_t capacity);

/* The same entries in the order the ordered schedule (cc_plan_set_schedule) works through them: every full chunk
 * first, in tensor order, then the tensors' short last chunks.  *full_chunks (may be NULL) receives the number of
 * full chunks.  Returns the number of entries written, or < 0 on error / too small. */
int64_t cc_ordered_table_fill(const uint64_t *numels, int32_t T, int32_t chunk_elems,
                              uint32_t *table, int64_t capacity, int64_t *full_chunks);

/* Default chunk size in elements for large shards (a tuning choice of this library; the paper's buckets hold
 * 2^10, Section 5.4).  Shards below 64 Mi elements default to 1024-element chunks (faster there in the size sweep). */
int32_t cc_default_chunk_elems(void);

/* ---- plan ---- */

/*
 * Validates the T tensors (host array, copied) and builds the device-side descriptor array and chunk
 * table once, like the paper's wrapper pre-computes bucket pointers (Section 5.5).  R = number of
 * gradient slices per tensor, 1..CC_MAX_R.  chunk_elems: a positive multiple of 1024 up to 2^24 (chunks of 4096
 * and more run in 512-thread workgroups, smaller ones in 128-thread workgroups), or 0: the plan is then prepared for
 * chunks of 1024, 4096 and 16384 elements (8 bytes of table per chunk each), starts with the one the size rule picks
 * (1024 below 64 Mi elements, else 4096), and cc_plan_set_chunk_elems / cc_plan_autotune can switch between them.
 * The plan owns only its own tables and scratch; it keeps raw copies of the caller's pointers, which
 * must stay valid while the plan is used.  Tensors with numel == 0 are legal and produce no chunks.
 */
int cc_plan_create(const cc_tensor *tensors, int32_t T, int32_t R, int32_t chunk_elems, cc_plan **out);

/* The same with the gradient element type stated (cc_plan_create is the CC_GRAD_F16 case). */
int cc_plan_create_ex(const cc_tensor *tensors, int32_t T, int32_t R, int32_t chunk_elems, int32_t grad_dtype,
                      cc_plan **out);
int cc_plan_destroy(cc_plan *plan);

/*
 * How a plan's kernels are laid over the device (a tuning choice like the protocol and the number of channels that
 * the paper's standalone experiments sweep, Section 6.1.1; results do not depend on it beyond the order of LAMB's
 * per-chunk partial sums, which both schedules keep identical).
 *   CC_SCHEDULE_PER_CHUNK  one workgroup per chunk, launched as a grid of that many workgroups.
 *   CC_SCHEDULE_ORDERED    `workgroups` persistent workgroups (0 = one per compute unit) take the chunks in table
 *                          order from a counter and keep the next chunk's loads in flight; needs the default
 *                          chunk size of large shards (cc_default_chunk_elems()).
 *   CC_SCHEDULE_AUTO       (default) ordered for large shards, per chunk for small ones.
 * cc_plan_schedule reports what the plan will use (schedule: ORDERED or PER_CHUNK; workgroups per launch).
 */
typedef enum cc_schedule { CC_SCHEDULE_AUTO = 0, CC_SCHEDULE_PER_CHUNK = 1, CC_SCHEDULE_ORDERED = 2 } cc_schedule;
int cc_plan_set_schedule(cc_plan *plan, int32_t schedule, int32_t workgroups);
int cc_plan_schedule(const cc_plan *plan, int32_t *schedule, int32_t *workgroups);

/*
 * Chunk size of the step calls: one of the sizes the plan was prepared for (see cc_plan_create), or 0 for the size
 * rule.  Adam results do not depend on it; LAMB's norms are summed chunk by chunk, so they move in the last bits.
 * cc_plan_layout reports what the plan will use (each pointer may be NULL): chunk size, threads per workgroup,
 * cache policy (CC_CACHE_STREAMING, CC_CACHE_RESIDENT or CC_CACHE_WRITE_THROUGH).
 */
int cc_plan_set_chunk_elems(cc_plan *plan, int32_t chunk_elems);
int cc_plan_layout(const cc_plan *plan, int32_t *chunk_elems, int32_t *block_threads, int32_t *cache_policy);

/*
 * Cache policy of the streaming kernels' accesses.  STREAMING marks every access non-temporal (right for shards far
 * beyond what the chip holds).  RESIDENT uses plain loads and write-through stores, so that a shard whose whole step
 * fits the 256 MB Infinity Cache finds its inputs on chip in the next step.  WRITE_THROUGH keeps the non-temporal loads
 * and writes the stores through, for shards of which one launch's output still about fits that cache.  The last two
 * exist for 128-thread workgroups (chunks below 4096 elements) and are ignored otherwise.  Results do not depend on
 * the policy.  AUTO (default): STREAMING while the step's buffers total less than 4 MiB (1-6 % faster there); else
 * RESIDENT while they total less than 200 MiB (4-24 % faster than STREAMING between 2^18 and 2^22 elements in the size
 * sweep); else WRITE_THROUGH while a launch stores less than
 * 288 MiB (the Adam step stores 14 bytes per element: up to 20.5 Mi elements, 8-12 % faster at 2^23 and 2^24; LAMB's
 * sweeps store 8 and 6: up to 36 Mi elements, and cc_plan_layout reports the Adam step's policy); else STREAMING.
 * cc_plan_autotune tries all three.
 */
typedef enum cc_cache_policy { CC_CACHE_AUTO = 0, CC_CACHE_STREAMING = 1, CC_CACHE_RESIDENT = 2, CC_CACHE_WRITE_THROUGH = 3 } cc_cache_policy;
int cc_plan_set_cache_policy(cc_plan *plan, int32_t policy);

/*
 * Picks chunk size, workgroup size, cache policy, schedule and workgroup count by measurement instead of by the size
 * rule, as the paper's autotuner keeps the fastest schedule per workload (Section 3.5): runs the plan's own fused
 * step (optimizer 0 = Adam, 1 = LAMB) a few times under each candidate (one workgroup per chunk for every chunk size
 * the plan was prepared for, with every cache policy that exists for it; ordered with compute units / 2, x 1 and x 2
 * workgroups on the 4096-element chunks), timed with events on `hip_stream`, and leaves the plan set to the fastest.  The
 * trial steps are ordinary steps on the caller's buffers: they write the out buffers and the flag, never the in
 * buffers, so the plan must be out of place (CC_ERR_ALIAS otherwise) and the caller must not have adopted the out
 * buffers' contents.  Synchronises the stream.  best_ms / per_chunk_ms (each may be NULL) receive the time per step
 * of the schedule kept and of one workgroup per chunk.
 */
int cc_plan_autotune(cc_plan *plan, const cc_hparams *hp, int32_t optimizer, int32_t *d_overflow_flag,
                     void *hip_stream, float *best_ms, float *per_chunk_ms);

/* Totals of a plan: elements, chunks and bytes of table memory on the device. */
int cc_plan_info(const cc_plan *plan, uint64_t *numel, int64_t *chunks, uint64_t *table_bytes);

/* ---- fused steps (one pass over HBM per sweep) ---- */

/*
 * Adam (Fig. 4a with the schedule of Fig. 4b).  Per element i of every tensor (the slices are added in double and S is
 * rounded to fp32; gh, m' and v' are formed in double from S, m and v, and m' and v' rounded to fp32 once each; u and w'
 * are computed in fp32 from the rounded moments):
 *   S = g_0[i] + g_1[i] + ... + g_{R-1}[i]   (fixed rank order)     gh = S / (loss_scale * (avg ? R : 1))
 *   m' = beta1 m + (1-beta1) gh      v' = beta2 v + (1-beta2) gh^2
 *   u  = (m'/(1-beta1^t)) / (sqrt(v'/(1-beta2^t)) + eps) + wd w     w' = w - lr u     w16 = fp16(w')
 * *d_overflow_flag (device int32) is written by the call: 1 if any S is inf or NaN, else 0 (the same launch that
 * does the update writes it; there is no separate clearing launch).
 * skip_mode 0: outputs are written unconditionally to the (distinct) out buffers; they are valid only
 * if the flag reads 0 afterwards.  skip_mode 1: see cc_hparams.
 */
int cc_fused_adam_step(cc_plan *plan, const cc_hparams *hp, int32_t *d_overflow_flag, void *hip_stream);

/*
 * For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops, harnesses that
 * forbid it): the fused Adam step of cc_fused_adam_step on ONE tensor with fp16 gradient slices, without a plan.
 * The call allocates nothing on the host or the device and creates no plan: the descriptor travels in the kernel
 * arguments, and the kernel's only scratch memory, the counting words of the overflow flag (16.6 KB), lives in a
 * static device array of the library that every GPU the library runs on holds until the process ends.  Same kernel,
 * same results bit for bit as cc_fused_adam_step on a single-tensor plan with 1024-element chunks.
 * `tensor` is a host pointer to one cc_tensor (device buffers as for a plan, same alignment and overlap rules).
 * numel may be 0 (the flag is cleared) and at most 2^26 (64 Mi) elements: larger tensors are rejected with CC_ERR_ARG,
 * they belong to a plan and the ordered schedule.  All calls on one GPU share that GPU's array, which keeps its
 * contents from call to call (the counting words leave every launch in the state the next one expects, whatever
 * the two sizes); calls that overlap in time on one GPU race on it, so they must be ordered (one stream, or events).
 */
int cc_fused_adam_step_static(const cc_tensor *tensor, int32_t R, const cc_hparams *hp, int32_t *d_overflow_flag,
                              void *hip_stream);

/*
 * LAMB, two sweeps around a per-tensor reduction (Section 5.2 "Tensor Reduction": each rank reduces
 * locally).  Phase 1 reduces the gradients, writes m', v' and accumulates sum(w^2), sum(u^2) per tensor
 * (u as above, w before the update).  Phase 2 forms ratio = ||w||/||u|| (1 if either norm is 0) and
 * writes w' = w - lr ratio u and w16.  On overflow phase 2 leaves w_out and w16_out untouched.
 * cc_fused_lamb_step = phase 1 then phase 2.  The two phases are exported separately so that a
 * cross-rank sum of the per-tensor norms can be placed between them.  The single call gives the same bits in two
 * launches instead of three when no tensor has more than 512 chunks: the workgroups of phase 2 then add up their own
 * tensor's partial sums (same additions, same order) instead of a per-tensor launch between the phases.
 */
int cc_fused_lamb_step(cc_plan *plan, const cc_hparams *hp, int32_t *d_overflow_flag, void *hip_stream);
int cc_fused_lamb_phase1(cc_plan *plan, const cc_hparams *hp, int32_t *d_overflow_flag, void *hip_stream);
int cc_fused_lamb_phase2(cc_plan *plan, const cc_hparams *hp, const int32_t *d_overflow_flag, void *hip_stream);

/* Device pointer to the plan's T x 2 doubles {sum w^2, sum u^2}, valid after phase 1 has run. */
int cc_lamb_norm_buffer(cc_plan *plan, double **d_sums);

/* Waits for `hip_stream`, then copies those T x 2 doubles to host memory `h_sums` (synchronous). */
int cc_lamb_norms_read(cc_plan *plan, double *h_sums, void *hip_stream);

/* ---- unfused reference pipelines (the AR-Opt shape of Section 6.1.1: reduce, then optimizer, then cast) ---- */

/*
 * Same results as the fused calls, computed by separate kernels with the reduced gradient stored to and
 * re-read from an fp32 buffer owned by the plan: reduce R slices -> fp32, optimizer kernel(s) on the reduced
 * gradient, fp32 -> fp16 cast.  The flag is known after the reduce kernel, so in skip_mode 0 the later kernels
 * leave every output untouched on overflow.
 * cc_plan_reserve_unfused allocates that buffer (4 bytes per element; synchronous; once per plan, further calls do
 * nothing).  The unfused step calls return CC_ERR_ARG until it has been called: a step call never allocates.
 */
int cc_plan_reserve_unfused(cc_plan *plan);
int cc_unfused_adam_step(cc_plan *plan, const cc_hparams *hp, int32_t *d_overflow_flag, void *hip_stream);
int cc_unfused_lamb_step(cc_plan *plan, const cc_hparams *hp, int32_t *d_overflow_flag, void *hip_stream);

/*
 * The unfused Adam pipeline with the element type of the intermediate stated.  CC_GRAD_F32 is cc_unfused_adam_step.
 * CC_GRAD_F16 is the baseline as a framework runs it over an fp16 all-reduce (Section 6.1.1, AR-Opt): the reduce
 * kernel hands fp16(fp32(sum)) to the optimizer kernel, which changes the numerics (the fused kernel keeps the
 * sum in fp32 registers for free) and raises the flag when a finite sum leaves the fp16 range.  fp16 slices only.
 */
int cc_unfused_adam_step_ex(cc_plan *plan, const cc_hparams *hp, int32_t *d_overflow_flag, void *hip_stream,
                            int32_t sum_dtype);

/* ---- model-parallel epilogue (the paper's running example) ---- */

/*
 * Fig. 3: sum = AllReduce("+", layer); out = Dropout(sum + b, p) + r, all fp16, with the schedule of Fig. 5
 * program 3 applied (reduce-scatter + pointwise work on the slice + all-gather fused, Section 3.3).  This is the
 * compute side on ONE rank's slice of the flattened [B*S, H] tensor: element i of the slice is element first + i
 * of the full tensor, its bias column is (first + i) % hidden.
 *   out[i] = keep(first + i) ? (partial_0[i] + ... + partial_{R-1}[i] + bias[col]) / (1 - p) : 0,  plus residual[i]
 * in fp32, rounded once to fp16.  keep() is Philox4x32-10 (counter = global index / 4, key = seed; the element
 * takes word index % 4) >= floor(p 2^32): the mask depends only on (seed, global index), never on the slicing.
 * Device pointers, 16-byte aligned; first and hidden must be multiples of 8; 0 <= p < 1; R in 1..CC_MAX_R.
 */
typedef struct cc_epilogue {
    uint64_t        numel;                 /* elements of this rank's slice */
    uint64_t        first;                 /* global index of its first element */
    uint32_t        hidden;                /* H */
    int32_t         R;                     /* number of partial outputs */
    const uint16_t *partial[CC_MAX_R];     /* R fp16 partial outputs of the local MatMul, numel each */
    const uint16_t *bias;                  /* hidden fp16 */
    const uint16_t *residual;              /* numel fp16 */
    uint16_t       *out;                   /* numel fp16 */
    float           dropout_p;
    uint64_t        seed;
} cc_epilogue;

/* One pass: 2R + 4 bytes per element. */
int cc_fused_epilogue(const cc_epilogue *args, void *hip_stream);

/* Reference pipeline with the same result: reduce the R partial outputs into `d_sum_scratch` (numel floats, device,
 * 16-byte aligned, owned by the caller), then the pointwise kernel: 2R + 4 and 4 + 4 bytes per element. */
int cc_unfused_epilogue(const cc_epilogue *args, float *d_sum_scratch, void *hip_stream);

/* ---- measurement aid ---- */

/* Plain streaming copy of `bytes` (multiple of 16, both pointers 16-byte aligned) device to device with
 * the same launch shape as the fused kernels; gives the practical HBM ceiling and calibrates counters. */
int cc_copy_probe(void *d_dst, const void *d_src, uint64_t bytes, void *hip_stream);

/* The memory pattern of the small-shard fused Adam step on one tensor (R = 4 or 8 fp16 slices, numel a multiple of
 * 1024, one 128-thread workgroup per 1024 elements) with parts taken away, to show where a launch-bound step's time
 * goes: what = 0 empty workgroups, 1 the loads only, 2 the stores only (w_out, m_out, v_out, w16_out receive filler
 * values), 3 loads and stores without the update arithmetic and without the flag (outputs are not an Adam step).
 * cache_policy: CC_CACHE_STREAMING, CC_CACHE_RESIDENT or CC_CACHE_WRITE_THROUGH.  d_sink: one device int32 (never written in practice). */
int cc_pattern_probe(const cc_tensor *tensor, int32_t R, int32_t what, int32_t cache_policy, int32_t *d_sink,
                     void *hip_stream);

/* Waits for `hip_stream`, then reads the ordered schedule's ticket counter and finished-workgroup word of the plan
 * (both are zero between launches; a test aid). */
int cc_plan_queue_state(cc_plan *plan, uint32_t *next_ticket, uint64_t *done_word, void *hip_stream);

/* What the current device reports about itself (any output pointer may be NULL): compute units, memory clock in
 * kHz and memory bus width in bits as hipDeviceGetAttribute gives them, total device memory in bytes. */
int cc_device_info(int32_t *compute_units, int32_t *memory_clock_khz, int32_t *memory_bus_bits, uint64_t *total_bytes);

const char *cc_last_error(void);
int cc_version(void);

#if defined(__GNUC__)
#pragma GCC visibility pop
#endif
#ifdef __cplusplus
}
#endif
#endif /* CCFUSED_H */
