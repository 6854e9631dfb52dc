/*
 * ps_step.h -- C ABI of the placement-sharded optimizer step for MI355X (gfx950).
 *
 * One device's share of a ZeRO/FSDP training step under the paper's placement
 * semantics: gradients G and optimizer state Omega are sharded (mode S), the
 * 16-bit parameters Theta are replicated (R) or sharded-with-gather (S*).
 * Device i reduces the N per-device gradient contributions for its shard in a
 * fixed order, applies mixed-precision Adam with decoupled weight decay to its
 * FP32 master/m/v shard, and writes the updated parameters in their 16-bit
 * format (bf16 or IEEE binary16) into the buffer the following All-Gather reads.
 *
 * Conventions
 *   - Plain C types only.  Every pointer below is marked HOST or DEVICE.
 *   - DEVICE buffers are owned by the caller, must be 16-byte aligned and must
 *     stay alive until the work queued on the given stream has finished.  No
 *     step, scan or copy call allocates, frees or keeps device memory; the one
 *     call that allocates is ps_arena_create, for callers who want their flat
 *     buffers laid out for this part's HBM.  (Speed, not correctness: the
 *     kernels run 3-7 % faster on MI355X when all buffers of a call start on
 *     4 KiB boundaries, as separate allocations do, and 5 % faster when the
 *     operands of a launch lie close together physically, see ps_arena_create.)
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).
 *     Calls that take a stream only enqueue work and return; they never
 *     synchronise the device.
 *   - No exceptions and no aborts cross this boundary.  Every call returns a
 *     ps_status_t; validation happens before the first HIP call, so argument
 *     errors are reported identically with or without a GPU.
 *   - The library keeps no state of the optimisation between calls: the step
 *     count t and all buffers belong to the caller, so a checkpoint is a copy of
 *     the flat shard buffers plus t.  What it does keep: a thread-local error
 *     string, per device the address of its static partial-sum array
 *     (ps_step_reduce_sumsq_static), and the measurement override of
 *     ps_probe_set_update_residency.
 *   - Sizes are element counts unless the name says bytes.  GB = 1e9 bytes in
 *     the cost figures, as in the paper's examples.
 */
#ifndef PS_STEP_H
#define PS_STEP_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PS_ABI_VERSION 5u
/* Largest number of gradient contributions one call can reduce. */
#define PS_MAX_CONTRIB 16u

/* Largest elem_count of one ps_step_reduce_sumsq_static call. */
#define PS_STATIC_MAX_ELEMS (1ull << 30)

/* Placement modes (Definition 1, Eq. 1-5). */
enum { PS_R = 0, PS_S = 1, PS_SG = 2 /* S*: sharded with gather */, PS_M = 3, PS_O = 4 };
/* Element types.  Gradient contributions: any of the three.  Parameters (the
 * 16-bit image of the master weights): PS_BF16 or PS_F16, the "FP16" of the
 * paper's Table 1 and Remark 1 being either 2-byte format.  PS_F16 is IEEE
 * binary16; with it a loss scale usually rides on ps_adamw_t.grad_scale. */
enum { PS_BF16 = 0, PS_F32 = 1, PS_F16 = 2 };

typedef enum {
    PS_OK = 0,
    PS_EINVAL = 1,       /* NULL pointer, bad enum, count mismatch                 */
    PS_EUNSUPPORTED = 2, /* placement this path does not execute                   */
    PS_EALIGN = 3,       /* pointer or offset not 16-byte aligned                  */
    PS_ERANGE = 4,       /* index/size out of range, or N does not divide a size   */
    PS_ENODEVICE = 5,    /* no HIP device present                                  */
    PS_EHIP = 6          /* a HIP call failed; text in ps_last_error()             */
} ps_status_t;

/* Placement specification Pi = (pi_Theta, pi_Omega, pi_G, pi_A) over N devices
 * (Definition 2) plus what is needed to turn it into bytes and index ranges. */
typedef struct ps_spec_t {
    int32_t theta, omega, grad, act; /* PS_R .. PS_O                                       */
    uint32_t n_devices;              /* N >= 1                                             */
    uint32_t shard_index;            /* i in [0, N)                                        */
    uint64_t psi;                    /* parameter count (the paper's P)                    */
    uint32_t align_elems;            /* 0/1: Eq. 2 exactly (N must divide psi); k > 1: pad
                                        psi up to a multiple of N*k, pad at the flat end  */
    uint32_t reserved;               /* must be 0                                          */
    uint64_t s_unit_bytes;           /* reconstruction unit (Definition 3); 0 reproduces the
                                        paper's worked examples, which drop the term      */
    uint64_t act_bytes;              /* |A| accounted to one device before mu is applied   */
} ps_spec_t;

/* Result of the derivation rules.  Fields ending in _xN hold bytes * N so that
 * the (N-1)/N factors of the ring cost models stay exact integers. */
typedef struct ps_cost_t {
    /* Theorem 1, Eq. 6-11: persistent GPU bytes per device and state. */
    uint64_t theta_bytes, omega_bytes, grad_bytes, act_bytes;
    uint64_t transient_bytes;  /* s_unit terms of S* and M                           */
    uint64_t persistent_total; /* sum of the four persistent parts                   */
    uint64_t peak_total;       /* persistent_total + transient_bytes = M(Pi)          */
    /* Theorem 2, Eq. 12-14: bytes per device per step, times N. */
    uint64_t comm_grad_sync_xN;    /* 2(N-1)|G| for pi_G=R, (N-1)|G| for pi_G=S      */
    uint64_t comm_param_gather_xN; /* 2(N-1)|Theta| for pi_Theta=S*, else 0          */
    double comm_total_bytes;       /* (sum of the two above) / N                     */
    /* Not a term of Theorem 2: the All-Gather of updated parameters that pi_Theta=R
     * with pi_Omega=S implies ((N-1)|Theta|).  Never included in comm_total_bytes. */
    uint64_t implied_update_gather_xN;
    /* Shard geometry (Eq. 2 with the padding rule of align_elems), in elements. */
    uint64_t psi_padded, shard_offset, shard_len, valid_len;
} ps_cost_t;

/* AdamW hyper-parameters.  All scalars the kernels use are formed from these in
 * binary64 on the host and rounded once to binary32. */
typedef struct ps_adamw_t {
    double lr, beta1, beta2, eps, weight_decay;
    uint64_t step;     /* t >= 1, the step being taken (bias correction 1-beta^t)     */
    double grad_scale; /* <= 0: 1/N, the mean over devices (proof of Theorem 5)       */
    double clip_coef;  /* <= 0: 1 (no clipping); else multiplies the mean gradient    */
    const float *clip_coef_device; /* DEVICE, optional (NULL: use clip_coef).  When set,
                          the kernels read the coefficient from this address when they
                          run (so it may be written earlier on the same stream, e.g. by
                          ps_step_clip_coef, with no host round trip), clip_coef must be
                          0, and a NaN found there makes the launch a no-op: nothing is
                          read or written (the step is skipped).                       */
} ps_adamw_t;

/* This device's shard of Omega and its output slot.  All DEVICE pointers. */
typedef struct ps_shard_t {
    float *master;     /* DEVICE, len floats: FP32 master weights, updated in place   */
    float *m;          /* DEVICE, len floats: Adam first moment, updated in place     */
    float *v;          /* DEVICE, len floats: Adam second moment, updated in place    */
    void *gather_out;  /* DEVICE, 16-bit elements of type param_dtype.  pi_Theta = S*:
                          the persistent parameter shard (len elements) that the
                          All-Gather reads.  pi_Theta = R: the full replicated parameter
                          buffer (psi_padded elements); the library writes this shard's
                          slice at shard_offset.                                      */
    uint64_t len;      /* shard length n = psi_padded / N, in elements                */
    uint64_t valid_len;/* elements [valid_len, len) are padding and are never written */
    int32_t param_dtype; /* PS_BF16 (0, the default of a zeroed field) or PS_F16.  16-bit
                          gradient contributions must be of the same type            */
    int32_t reserved;  /* must be 0                                                   */
} ps_shard_t;

/* The N gradient contributions for this shard (the inputs of the Reduce-Scatter
 * whose result device i owns; Section 2.3, Theorem 2 part 2). */
typedef struct ps_grads_t {
    const void *const *contrib; /* HOST array of n_contrib DEVICE pointers; contrib[r]
                                   is element 0 of device r's contribution for the range
                                   being processed (the shard, or the current bucket)  */
    uint32_t n_contrib;         /* = n_devices, or 1 for an already reduced gradient   */
    int32_t dtype;              /* PS_BF16, PS_F16 or PS_F32, one type for all
                                   (Theorem 4)                                         */
    const float *accum;         /* DEVICE or NULL, shard-based like ps_shard_t.master: the
                                   FP32 accumulator of earlier micro-batches
                                   (ps_step_accumulate).  ps_step_update adds it to the
                                   contributions' sum before the mean, so the last
                                   micro-batch needs no accumulation pass of its own;
                                   every other call wants it NULL (PS_EUNSUPPORTED)    */
} ps_grads_t;

/* How ps_step_update_bucketed moves a bucket into its staging slot. */
enum {
    PS_COPY_KERNEL = 0, /* the library's copy kernel; the source must be readable by
                           device code (device memory, or pinned host memory)        */
    PS_COPY_MEMCPY = 1, /* hipMemcpyAsync per contribution (DMA engines for host
                           sources); needs source_elems % bucket_elems == 0          */
    PS_COPY_REDUCE = 3, /* the library's reduce kernel in place of a copy: it reads the
                           bucket's N contributions from the source (memory device code
                           can read: device, peer-mapped or pinned host) and leaves their
                           fixed-order FP32 sum in the staging slot; the update takes that
                           sum as its one contribution (same bits as reducing inside the
                           update).  Slots of bucket_elems FP32 values suffice.  Moves
                           2N + 4 bytes per element on the copy stream instead of 4N and
                           leaves the update 4 bytes to read instead of 2N: the form for a
                           source that is read over a link                             */
    PS_COPY_NONE = 2    /* no copy: the source is memory of THIS device and the update
                           reads every bucket where it lies, one kernel per bucket on
                           compute_stream (one per contiguous piece where a repeating
                           source wraps inside a bucket).  staging, copy_stream and
                           schedule are not used and may be zero.  The source must stay
                           unchanged until the work queued on compute_stream is done */
};

/* How the staging copy of bucket b+1 and the update of bucket b share the device. */
enum {
    PS_SCHED_AUTO = 0,     /* PS_COPY_KERNEL, PS_COPY_REDUCE: alternate; PS_COPY_MEMCPY: overlap */
    PS_SCHED_OVERLAP = 1,  /* both run as soon as their inputs are ready                    */
    PS_SCHED_ALTERNATE = 2 /* the copy of bucket b+1 starts when the update of bucket b has
                              finished; still enqueued ahead on its own stream, no host wait */
};

/* Gradients that arrive in buckets: bucket b of a shard covers elements
 * [b*bucket_elems, min((b+1)*bucket_elems, len)).  Where the contributions have
 * to be moved first (PS_COPY_KERNEL, PS_COPY_MEMCPY) the library copies each
 * bucket from `source` into one of two staging slots on `copy_stream` and
 * updates it on `compute_stream`; events order the two streams, the host never
 * waits.  In a multi-device job such a source is wherever the other devices'
 * contributions arrive (peer-mapped or host memory).  A copy that runs on DMA
 * engines is bound by its link and overlaps the update of the previous bucket.
 * A copy kernel reading local memory is bound by HBM like the update itself;
 * measured on MI355X the two then finish sooner taking turns than side by side
 * (77.9 vs 82.9 ms for the 70B shard), which is what PS_SCHED_AUTO does.
 * Contributions that already lie in this device's memory need no copy at all:
 * staging them writes 2N bytes per element to HBM only to read them back (the
 * memory-side cache writes through), so PS_COPY_NONE updates each bucket straight
 * from the source (56.5 ms for the same shard in arena buffers, 60 ms with one
 * plain allocation per buffer).  Where staging is unavoidable, PS_COPY_REDUCE
 * stages the bucket's FP32 sum instead of its N contributions (70 ms against 105
 * ms from a source in HBM). */
typedef struct ps_bucket_plan_t {
    const void *const *source;  /* HOST array of n_contrib pointers (DEVICE or pinned HOST
                                   memory), each holding source_elems elements of that
                                   contribution.  Shard element e of contribution r is
                                   read from source[r][e % source_elems]: a source as
                                   long as the shard holds every bucket, a shorter one is
                                   a pool that repeats                                 */
    uint32_t n_contrib;
    int32_t dtype;
    uint64_t bucket_elems;      /* multiple of 8                                        */
    uint64_t source_elems;      /* >= 1, multiple of 512                                */
    void *staging[2];           /* DEVICE, each n_contrib * bucket_elems elements; slot
                                   layout: contribution r at element r * bucket_elems
                                   (PS_COPY_REDUCE: bucket_elems floats; unused with
                                   PS_COPY_NONE)                                       */
    void *copy_stream;          /* hipStream_t (unused with PS_COPY_NONE)               */
    void *compute_stream;       /* hipStream_t, must differ from copy_stream            */
    int32_t copy_engine;        /* PS_COPY_KERNEL, PS_COPY_MEMCPY, PS_COPY_REDUCE, PS_COPY_NONE */
    int32_t schedule;           /* PS_SCHED_AUTO, PS_SCHED_OVERLAP or PS_SCHED_ALTERNATE */
    float *kernel_ms;           /* HOST, optional (may be NULL): receives, per bucket,
                                   the update kernel's duration in ms from HIP events
                                   on compute_stream.  When non-NULL the call waits for
                                   the streams to drain before returning.              */
    uint64_t kernel_ms_len;     /* capacity of kernel_ms                                */
} ps_bucket_plan_t;

/* Where ps_step_update_offloaded finds the state on the host. */
enum { PS_HOST_FLAT = 0, PS_HOST_PACKED = 1 };

/* Offloaded optimizer state (Table 2, ZeRO-Offload: Theta and Omega in mode O,
 * G sharded): master, m, v and the 16-bit parameters of this shard live in pinned
 * HOST memory and stream through the device in buckets. */
typedef struct ps_offload_plan_t {
    float *host_master;     /* pinned HOST, len floats, updated in place (PS_HOST_FLAT)  */
    float *host_m;          /* pinned HOST, len floats                                   */
    float *host_v;          /* pinned HOST, len floats                                   */
    void *host_param_out;   /* pinned HOST, len 16-bit elements of type param_dtype:
                               the updated parameters                                    */
    uint64_t len;           /* shard length n = psi_padded / N                           */
    uint64_t valid_len;     /* elements [valid_len, len) are never read or written       */
    uint64_t bucket_elems;  /* multiple of 8.  On MI355X copies of 0.4-0.5 GB (2^25
                               elements) keep the host link at its full-duplex rate run
                               after run; half that size has measured up to twice the
                               step time, the DMA engines then being shared unevenly    */
    uint32_t n_slots;       /* 2 or 3 DEVICE slots; 3 lets upload, update and download
                               of neighbouring buckets run at the same time             */
    int32_t param_dtype;    /* PS_BF16 (0) or PS_F16, as in ps_shard_t                   */
    void *slot[3];          /* DEVICE, each 14 * bucket_elems bytes, 16-byte aligned:
                               master | m | v (FP32) | 16-bit parameters of one bucket  */
    void *h2d_stream;       /* hipStream_t; the three streams must differ                */
    void *compute_stream;
    void *d2h_stream;
    int32_t host_layout;    /* PS_HOST_FLAT (0, a zeroed field): the four host_* arrays above.
                               PS_HOST_PACKED: host_packed below, the four host_* are unused */
    int32_t reserved;       /* must be 0                                                 */
    void *host_packed;      /* pinned HOST, ceil(len / bucket_elems) * 14 * bucket_elems
                               bytes, 16-byte aligned: bucket b occupies the 14 *
                               bucket_elems bytes from byte b * 14 * bucket_elems on, laid
                               out like a DEVICE slot: master | m | v (FP32, bucket_elems
                               each) | 16-bit parameters (bucket_elems).  A whole bucket
                               then moves as ONE copy per direction (12 bucket_elems bytes
                               up, 14 bucket_elems bytes down) instead of three and four */
} ps_offload_plan_t;

typedef struct ps_device_info_t {
    char name[128];
    char arch[64];
    int32_t compute_units;
    int32_t wavefront_size;
    int32_t clock_khz, memory_clock_khz, memory_bus_bits;
    int32_t l2_bytes;
    uint64_t total_bytes, free_bytes;
} ps_device_info_t;

/* ---- host-only calls (no GPU needed) ---- */

uint32_t ps_abi_version(void);
const char *ps_status_string(ps_status_t st);
/* Text of the last error on the calling thread ("" if none). */
const char *ps_last_error(void);

/* Fills *spec with a named row of the paper's Table 2: "dp", "zero1", "zero2",
 * "zero3" (also "fsdp"), "zero_offload", "tp", "pp".  align_elems, s_unit_bytes
 * and act_bytes are set to 0.  Unknown name: PS_EINVAL. */
ps_status_t ps_spec_preset(const char *name, uint32_t n_devices, uint32_t shard_index,
                           uint64_t psi, ps_spec_t *spec);

/* Derivation rules: per-device memory (Theorem 1), per-step communication
 * (Theorem 2, with the ring cost models of Section 2.3) and the shard geometry
 * (Eq. 2), with the byte accounting of Remark 1 (|Theta| = 2 psi, |Omega| =
 * 12 psi, |G| = 2 psi).  Sizes are taken on psi_padded, the length the flat
 * buffers hold (= psi whenever N divides psi).  Pure function of *spec.
 * PS_ERANGE if a division by N is not exact or a result overflows 64 bits. */
ps_status_t ps_cost_eval(const ps_spec_t *spec, ps_cost_t *cost);

/* Global-norm clip coefficient (gradient clipping is not in the paper; the named
 * 13B workload asks for it), in binary64: min(1, max_norm / (sqrt(sumsq_local
 * + sumsq_others) + 1e-6)), the sums being those of the squared mean gradient
 * over this device's shard and over all other devices' shards.  A non-finite
 * or negative sum, or max_norm <= 0, gives NaN (the caller should skip the
 * step).  Pass the result as ps_adamw_t.clip_coef. */
double ps_clip_coef(double sumsq_local, double sumsq_others, double max_norm);

/* The same coefficient (again not in the paper) formed on the device, for callers that keep the two
 * phases of a clipped step on the stream: *coef_out (DEVICE float) =
 * ps_clip_coef(*sumsq_local, sumsq_others ? *sumsq_others : 0, max_norm) rounded
 * to binary32, NaN where ps_clip_coef gives NaN.  sumsq_local and sumsq_others
 * are DEVICE doubles (the result of ps_step_reduce_sumsq; the other devices'
 * total as an all-reduce leaves it; NULL: none).  Enqueued on `stream`; pass
 * coef_out as ps_adamw_t.clip_coef_device of the following ps_step_update. */
ps_status_t ps_step_clip_coef(const double *sumsq_local, const double *sumsq_others,
                              double max_norm, float *coef_out, void *stream);

/* Illustrative strategy selection (Algorithm 1) with its printed thresholds:
 * 16 psi < 0.7 device_mem_bytes -> data parallel (R,R,R,R); else ZeRO-3
 * (S*,S,S,R).  *fits is set to whether the chosen placement's model state stays
 * below 0.7 device_mem_bytes per device.  *add_tp is set when ZeRO-3 alone does
 * not fit, a single layer (layer_bytes) exceeds 0.3 device_mem_bytes and the
 * interconnect is fast: tensor parallelism is then to be added within a node
 * (the composed specification itself is left to the caller).  Comparisons are
 * exact (integers, strict inequalities as printed).  spec receives n_devices,
 * psi and shard_index 0. */
ps_status_t ps_select_strategy(uint64_t psi, uint64_t device_mem_bytes, uint32_t n_devices,
                               uint64_t layer_bytes, int32_t fast_interconnect, ps_spec_t *spec,
                               int32_t *fits, int32_t *add_tp);

/* Composition calculus (Definition 5): where device `device` of n = inner * outer
 * devices sits when one strategy is applied within groups of `inner` consecutive
 * devices and another across the groups.
 *   Tensor x data parallel (Theorem 6): inner = T; TP group i = {iT..(i+1)T-1};
 *     data-parallel sync runs across groups between equal positions.
 *   Pipeline x data parallel (Theorem 7): inner = D; stage k is replicated on
 *     {kD..(k+1)D-1} (gradient sync inside); activations move across groups
 *     between equal positions (device +- D).
 * Outputs: inner_group = device / inner, inner_rank = device % inner; the outer
 * group is the set {inner_rank + j * inner}, indexed by outer_group = inner_rank,
 * with outer_rank = inner_group. */
ps_status_t ps_compose_index(uint32_t inner, uint32_t outer, uint32_t device,
                             uint32_t *inner_group, uint32_t *inner_rank,
                             uint32_t *outer_group, uint32_t *outer_rank);

/* Cost of a composed strategy as one device sees it (Definition 5; Theorems 6
 * and 7; the remark on three-way composition).  The inner strategy (tensor
 * parallelism of degree T, a pipeline of K stages, or both: inner = T, K or
 * T * K) leaves each device 1/inner of the model; *outer is a data-parallel
 * family specification (a row of Table 2) over the outer->n_devices devices
 * that hold the same share, its psi being the parameter count of the WHOLE
 * model.  The result is Theorems 1 and 2 applied inside that group: memory per
 * device and the bytes one device moves per step for gradient sync and
 * parameter gathers among its outer->n_devices peers.  What the inner strategy
 * itself communicates (per-layer collectives on activations, stage-to-stage
 * activation transfers) is not quantified by the paper and is not included.
 * Shard geometry in *cost refers to the group's flat buffers of psi / inner
 * elements.  PS_ERANGE if inner does not divide psi, else as ps_cost_eval. */
ps_status_t ps_compose_cost(const ps_spec_t *outer, uint32_t inner, ps_cost_t *cost);

/* ---- device calls ---- */

/* Properties of the current HIP device as hipGetDeviceProperties and
 * hipMemGetInfo report them (name, architecture, compute units, clocks, memory
 * bus, L2 size, total and free memory); recorded next to every measurement.
 * info is HOST memory owned by the caller.  PS_ENODEVICE without a GPU. */
ps_status_t ps_device_info(ps_device_info_t *info);

/* One optimizer step on elements [elem_offset, elem_offset + elem_count) of the
 * shard (the whole shard, or one bucket of it).
 *
 *   acc = ((g_0 + g_1) + g_2) + ...          binary32, contribution index ascending
 *   acc = accum + acc                        only with grads->accum (see below)
 *   g   = (acc * grad_scale) * clip_coef     the global-batch mean (Theorem 3)
 *   m'  = fma(beta1, m, (1-beta1) * g)
 *   v'  = fma(beta2, v, ((1-beta2) * g) * g)
 *   u   = m' / fma(sqrt(v'), 1/sqrt(1-beta2^t), eps)
 *   th' = fma(-lr/(1-beta1^t), u, fma(-lr*wd, th, th))
 *   out = th' rounded to nearest even in the parameters' 16-bit format (bf16:
 *         NaN -> 0x7FC0 with the sign; binary16: NaN -> 0x7E00 with the sign,
 *         |th'| >= 65520 -> infinity, subnormals kept)
 *
 * each line one correctly rounded binary32 operation.  State pointers in *shard
 * are shard-based (element 0 of the shard); grads->contrib[r] points at element
 * elem_offset of contribution r.  Only elements below shard->valid_len are read
 * or written.  Placements executed (rows of Table 2):
 *   ZeRO-2 / ZeRO-3 (omega S, grad S, theta R or S*): n_contrib == n_devices, or
 *     1 with PS_F32 for a gradient reduced (or accumulated) beforehand;
 *   ZeRO-1 (omega S, grad R, theta R): the gradient has already been all-reduced
 *     into one full-length replicated buffer (psi_padded elements, PS_BF16 or
 *     PS_F32); n_contrib == 1, contrib[0] points at element 0 of that buffer and
 *     the library reads this shard's slice at shard_offset, as it writes the
 *     parameters' slice.  grad_scale <= 0 still means 1/N: the all-reduce sums.
 *   Data parallelism (all four modes R): nothing is sharded, so every device
 *     updates the whole state from the all-reduced gradient: shard->len ==
 *     psi_padded, valid_len <= psi, all buffers full length and element-0 based,
 *     n_contrib == 1 as for ZeRO-1.  (ps_cost_eval still reports the Eq. 2
 *     geometry of shard_index; the step does not use it here.)
 * Anything else: PS_EUNSUPPORTED.  elem_offset must be a multiple of 8.
 * With grads->accum (pi_G = S only, 16-byte aligned) the contributions are the
 * LAST of k micro-batches and accum holds the sum of the k - 1 before it: the
 * result is bit for bit that of ps_step_accumulate on these contributions
 * followed by an update from the accumulator alone, without writing the
 * accumulator and reading it back (8 bytes per element less).  accum is only
 * read.  grad_scale is then the caller's to set, 1 / (N k).
 * Deterministic: no atomics, results do not depend on launch shape (Theorem 5,
 * assumption 1).  The call only enqueues kernels on hip_stream: it allocates
 * nothing and waits for nothing, so it may be recorded into a HIP graph by a
 * stream capture (the scalars derived from *hp are then fixed in the graph). */
ps_status_t ps_step_update(const ps_spec_t *spec, const ps_adamw_t *hp,
                           const ps_shard_t *shard, const ps_grads_t *grads,
                           uint64_t elem_offset, uint64_t elem_count, void *stream);

/* The same step over a whole shard whose gradient contributions arrive in
 * buckets (see ps_bucket_plan_t).  Enqueues every copy and kernel without a
 * host wait (unless plan->kernel_ms asks for timings).  With PS_COPY_NONE the
 * call only enqueues kernels on compute_stream and creates nothing (when
 * kernel_ms is NULL), so it may be recorded by a stream capture. */
ps_status_t ps_step_update_bucketed(const ps_spec_t *spec, const ps_adamw_t *hp,
                                    const ps_shard_t *shard, const ps_bucket_plan_t *plan);

/* Gradient accumulation (Limitations: several micro-batches per synchronisation,
 * communication amortised by their number).  Adds one micro-batch to this
 * shard's FP32 accumulator: accum[e] = accum[e] + ((g_0[e] + g_1[e]) + ...), the
 * contributions summed first in the fixed order, each `+` one binary32
 * operation; overwrite != 0 stores the sum instead (first micro-batch).  accum
 * is DEVICE, shard-based, 16-byte aligned; contrib[r] points at element
 * elem_offset.  After k micro-batches pass accum to ps_step_update as a single
 * PS_F32 contribution with grad_scale = 1 / (N k).  Requires omega S, grad S. */
ps_status_t ps_step_accumulate(const ps_spec_t *spec, const ps_grads_t *grads, float *accum,
                               int32_t overwrite, uint64_t elem_offset, uint64_t elem_count,
                               uint64_t valid_len, void *stream);

/* The same step with the optimizer state offloaded to pinned host memory
 * (Definition 1, Eq. 5: mode O holds nothing on the GPU).  Requires theta ==
 * PS_O, omega == PS_O, grad == PS_S.  grads->contrib[r] points at element 0 of
 * this shard's slice of contribution r in DEVICE memory (n_contrib ==
 * n_devices, or 1 with PS_F32).  Per bucket: three host-to-device copies on
 * h2d_stream, the update kernel on compute_stream, four device-to-host copies on
 * d2h_stream, ordered by events; nothing waits on the host.  Before it returns the
 * call makes h2d_stream wait for its own last downloads, so a following call with
 * the same streams may be enqueued right away: its uploads (which reuse the slots
 * and read the host ranges this call writes) start only when this step's results
 * have landed.  The caller synchronises d2h_stream before reading the host buffers
 * itself.  The path is bound by the host link (12 bytes in, 14 bytes out per
 * element), not by HBM. */
ps_status_t ps_step_update_offloaded(const ps_spec_t *spec, const ps_adamw_t *hp,
                                     const ps_offload_plan_t *plan, const ps_grads_t *grads);

/* Bytes of DEVICE workspace ps_step_reduce_sumsq needs for a call over
 * elem_count elements (about elem_count / 128 bytes; host-only query). */
uint64_t ps_workspace_bytes(uint64_t elem_count);

/* First phase of a step with global-norm clipping: reduce the contributions
 * for [elem_offset, elem_offset + elem_count), form the mean g = acc *
 * grad_scale (grad_scale <= 0: 1/N), store it as FP32 at reduced_out +
 * elem_offset (reduced_out DEVICE, shard-based, may be NULL), and write the sum
 * of g*g over the valid elements of the range, accumulated in binary64 in a
 * fixed tree, to *sumsq_out (DEVICE double).  accumulate != 0 adds to the value
 * already there, so several buckets called in order give a reproducible total.
 * The caller combines it with the other devices' sums, forms the clip
 * coefficient and calls ps_step_update with the reduced gradient as a single
 * PS_F32 contribution, grad_scale = 1 and that coefficient.  Under pi_G = R
 * (ZeRO-1, data parallelism) contrib[0] is the all-reduced full-length buffer
 * and this device's range of it is read; reduced_out is still based at the
 * first element of that range, i.e. the mean leaves this call in sharded form,
 * so under ZeRO-1 the second phase is a pi_G = S call on the same geometry (the
 * ZeRO-2 row of Table 2).  Like
 * ps_step_update the call only enqueues kernels (the partial sums live in the
 * caller's workspace, which a later call on another stream must not share while
 * this one is in flight) and may be recorded by a stream capture. */
ps_status_t ps_step_reduce_sumsq(const ps_spec_t *spec, const ps_grads_t *grads,
                                 double grad_scale, float *reduced_out, double *sumsq_out,
                                 int32_t accumulate, void *workspace,
                                 uint64_t workspace_bytes, uint64_t elem_offset,
                                 uint64_t elem_count, uint64_t valid_len, void *stream);

/* ps_step_reduce_sumsq for callers that cannot allocate device memory and so have
 * no workspace to pass: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, results and error behaviour
 * (bit for bit: same kernels, same reduction tree), minus the workspace: the
 * partial sums live in an array of the library's own, a file-scope __device__
 * array of 8 MiB + 8 KiB that every device the library runs on holds until the
 * process ends.  The call allocates and frees nothing.  elem_count may be at most
 * PS_STATIC_MAX_ELEMS (2^30) per call, else PS_ERANGE and nothing is enqueued; a
 * longer range goes out as several calls in order, accumulate != 0 from the second
 * on.  Nothing in the array has to start at zero (every partial sum is written
 * before it is read), so it is never cleared.  All calls on one device share that
 * device's array: calls whose work overlaps on one device (two streams, two
 * threads) race on it; calls on one stream, or ordered by events, do not.  The first
 * call on each device looks the array up with the runtime (no allocation either);
 * make that call outside a stream capture. */
ps_status_t ps_step_reduce_sumsq_static(const ps_spec_t *spec, const ps_grads_t *grads,
                                        double grad_scale, float *reduced_out, double *sumsq_out,
                                        int32_t accumulate, uint64_t elem_offset,
                                        uint64_t elem_count, uint64_t valid_len, void *stream);

/* ---- verification protocol (Section 7.1) ---- */

/* Bytes of DEVICE workspace the two verification scans need for a buffer of
 * buffer_bytes bytes (16 KiB + about buffer_bytes / 2048; host-only query). */
uint64_t ps_verify_workspace_bytes(uint64_t buffer_bytes);

/* Gradient integrity check: writes out2[0] = sum (a-b)^2 and out2[1] = sum a^2
 * over elem_count elements of the DEVICE buffers a and b (PS_BF16, PS_F16 or PS_F32,
 * one type for both), accumulated in binary64 in a fixed tree (reproducible bit
 * for bit).  The caller forms ||a-b|| / ||a|| = sqrt(out2[0] / out2[1]) and
 * compares it with the protocol's 1e-5.  accumulate != 0 adds to the values
 * already in out2 (DEVICE, two doubles). */
ps_status_t ps_verify_diff_sumsq(const void *a, const void *b, int32_t dtype, uint64_t elem_count,
                                 double *out2, int32_t accumulate, void *workspace,
                                 uint64_t workspace_bytes, void *stream);

/* State consistency check: a position-sensitive 64-bit checksum of `bytes` bytes
 * (a multiple of 8) of a DEVICE buffer, for comparing copies across devices
 * after a collective.  Word i (8 bytes, little endian, index first_word_index +
 * i) contributes the splitmix64 output function of
 * w_i + (index + 1) * 0x9E3779B97F4A7C15; contributions add modulo 2^64, so the
 * value does not depend on summation order and checksums of consecutive pieces
 * add up (accumulate != 0 adds to *out, DEVICE). */
ps_status_t ps_verify_checksum(const void *buf, uint64_t bytes, uint64_t first_word_index,
                               uint64_t *out, int32_t accumulate, void *workspace,
                               uint64_t workspace_bytes, void *stream);

/* ---- memory layout for a working set of hundreds of GB ---- */

/* Flat DEVICE buffers with interleaved physical backing.  The step walks its
 * operands in lock step (element e of every contribution, of master, m, v and of
 * the 16-bit parameters at the same time).  Measured on MI355X: the physical HBM
 * address space falls into regions of 32-64 GiB of three kinds, and a streaming
 * kernel runs 4-6 % faster when all its operands lie in regions of one kind.
 * Flat buffers of a 70B shard's working set (262 GB) allocated one after the
 * other cannot: element 0 of master lies 100 GB from element 0 of the last
 * contribution.  The arena reserves n_buffers flat virtual ranges (buffer k:
 * len elements of elem_bytes[k] bytes; the one pointer per buffer that the step's
 * interface takes) and creates the physical memory chunk by chunk (chunk c of
 * buffer 0, of buffer 1, ... then chunk c+1), mapping each piece in place, so
 * that what the kernel touches at any moment lies within a few GiB.  chunk_elems
 * is the bucket size where gradients arrive in buckets; chunk_elems *
 * elem_bytes[k] must be a multiple of 2 MiB.  This is the one call that
 * allocates device memory, and it does so only for the caller who asks: the step
 * itself never allocates.  Results never depend on it; where the driver places
 * consecutive physical allocations is its own business (in address order on a
 * device with free memory).  PS_EHIP with the runtime's text if the memory cannot
 * be had (everything is released again), PS_ENODEVICE without a GPU. */
typedef struct ps_arena_t ps_arena_t;
ps_status_t ps_arena_create(uint64_t len, uint64_t chunk_elems, const uint32_t *elem_bytes,
                            uint32_t n_buffers, ps_arena_t **arena);
/* DEVICE pointer to element 0 of buffer k (2 MiB aligned); NULL if k is out of range. */
void *ps_arena_buffer(const ps_arena_t *arena, uint32_t k);
/* Unmaps and releases everything.  All work that uses the buffers must have
 * finished.  NULL is allowed. */
ps_status_t ps_arena_destroy(ps_arena_t *arena);

/* Plain streaming copy of `bytes` bytes (multiple of 16) between DEVICE buffers
 * with the same launch shape as the update kernel.  A yardstick for achievable
 * HBM bandwidth and for calibrating hardware byte counters; not part of the
 * step. */
ps_status_t ps_probe_copy(void *dst, const void *src, uint64_t bytes, void *stream);

/* Measurement aid, not part of the step: overrides how many single-wave workgroups
 * of the update kernel may be resident per compute unit (the library chooses 8 to
 * 12 by operand mix; the launch shape decides the speed of a pure stream, never
 * its results).  0 restores the library's choice, 3..32 sets the cap, a larger
 * value removes it.  1 and 2: PS_ERANGE.  Process-wide (the one piece of global
 * state besides the error string); used by the benchmark's launch-shape sweep. */
ps_status_t ps_probe_set_update_residency(uint32_t waves_per_cu);

#ifdef __cplusplus
}
#endif
#endif /* PS_STEP_H */
