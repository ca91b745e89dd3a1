/*
 * came.h -- C ABI of the MI355X (gfx950) CAME optimizer-step library.
 *
 * One call, came_step, applies one step of the CAME optimizer (Luo et al.,
 * "CAME: Confidence-guided Adaptive Memory Efficient Optimization",
 * Algorithm 2) to every tensor of a parameter list on one GPU.  For an n x m
 * weight matrix theta with gradient g (Section 3.1 notation; n = rows,
 * m = columns, row-major contiguous):
 *
 *   r <- beta2 r + (1-beta2) rowsum(g^2 + eps1)        c <- ... colsum(...)
 *   v  = r c^T / sum(r)                                u  = g / sqrt(v)
 *   u^ = u / max(1, RMS(u)/d)                          (Eq. 1)
 *   M <- beta1 M + (1-beta1) u^
 *   U  = (u^ - M)^2
 *   R <- beta3 R + (1-beta3) rowsum(U + eps2)          C <- ... colsum(...)
 *   S  = R C^T / sum(R)                                theta <- theta - eta M / sqrt(S)
 *
 * Row/column reductions are sums (as printed), RMS is over the n*m entries of
 * that tensor, all state starts at zero, and the step counter never enters
 * the arithmetic (no bias correction in Algorithm 2).  A 1-D parameter of
 * length n is treated as the n x 1 special case of Algorithm 2, which
 * degenerates to the unfactored update: v (length n) replaces r c^T / sum r and
 * s (length n) replaces R C^T / sum R.
 *
 * Memory and ownership.  ALL device memory belongs to the caller: the
 * parameter tensors, the gradient tensors, one `state` blob and one `scratch`
 * blob whose sizes came_state_size reports.  The library never allocates or
 * frees device memory.  came_ctx is a host object owned by the library from
 * came_init_state until came_destroy.  Pointers marked "device" must be
 * device-accessible addresses on the GPU that is current when the call is
 * made; pointers marked "host" are ordinary process memory.
 *
 * Threading / ordering.  came_step only enqueues kernels (and, when the
 * parameter/gradient addresses differ from the previous call, one small
 * host-to-device copy) on the given HIP stream and returns without
 * synchronising.  Calls on one context must be issued from one thread at a
 * time and on streams ordered with respect to each other.
 *
 * Errors.  Every function returning int gives 0 (CAME_OK) or a negative
 * came_status.  No exceptions cross this boundary.  On error nothing has been
 * enqueued unless the code is CAME_EHIP (a HIP runtime call failed part-way).
 */
#ifndef CAME_H
#define CAME_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    CAME_OK = 0,
    CAME_EINVAL = -1, /* null pointer, count <= 0, rows/cols <= 0, ndim not 1 or 2, bad dtype,
                         beta outside [0,1), eps < 0, clip_d <= 0, weight_decay < 0, non-finite lr, step < 1,
                         option out of range */
    CAME_ESIZE = -2,  /* state or scratch blob smaller than came_state_size reports */
    CAME_EALIGN = -3, /* a device pointer is not aligned as documented */
    CAME_EHIP = -4,   /* a HIP runtime call failed; see came_last_hip_error */
    CAME_ENOMEM = -5, /* host allocation failed */
    CAME_ETIMEOUT = -6 /* a wait inside the on-chip kernel of an earlier step ran into its time limit
                          (came_options.resident_wait_us): the workgroups gave up waiting and ran to
                          their end, so nothing hangs, but the state and parameters of the matrices
                          that take the on-chip path are undefined from that step on.  Sticky until
                          came_destroy */
} came_status;

typedef enum {
    CAME_GRAD_F32 = 0, /* gradient stored as IEEE binary32 */
    CAME_GRAD_BF16 = 1 /* gradient stored as bfloat16 (upper 16 bits of binary32); widened exactly */
} came_grad_dtype;

typedef enum {
    CAME_ALGO_CAME = 0,     /* Algorithm 2 */
    CAME_ALGO_ADAFACTOR = 1 /* Algorithm 1 (Adafactor with momentum): Algorithm 2 without the
                               instability/confidence lines, theta <- theta - eta M; R, C stay zero */
} came_algo;

typedef enum {
    CAME_MOMENTUM_F32 = 0, /* M kept as binary32 (Algorithm 2 evaluated in binary32 throughout) */
    CAME_MOMENTUM_BF16 = 1 /* M kept as bfloat16 BETWEEN steps: a step widens the stored M_{t-1}
                              exactly, forms M_t, U_t and theta_t from it in binary32 as printed in
                              Algorithm 2, and stores M_t rounded to nearest even.  The paper does
                              not say in what precision states are kept; this halves M's bytes
                              (state rows*cols*2 + ..., step traffic 14 + 3*grad_bytes per
                              parameter instead of 20 + 3*grad_bytes) at the cost of a relative
                              storage error of at most 2^-9 in M */
} came_momentum_dtype;

typedef enum {
    CAME_VECTOR_ALGORITHM2 = 0,   /* 1-D parameters: Algorithm 2 on the n x 1 matrix (unfactored v and s) */
    CAME_VECTOR_MOMENTUM_ONLY = 1 /* 1-D parameters move by -eta M_t (Algorithm 1's update: no instability,
                                     no confidence; their s stays zero); matrices are unaffected.  A
                                     convention of some trainers, not the paper's */
} came_vector_rule;

typedef enum {
    CAME_RESIDENT_AUTO = 0, /* the planner's default: CAME_RESIDENT_OFF (on MI355X the on-chip path measures
                               slower than the streaming sweeps: see CAME_RESIDENT_ON) */
    CAME_RESIDENT_OFF = 1,  /* every matrix takes the three streaming sweeps */
    CAME_RESIDENT_ON = 2    /* matrices small enough take the on-chip path: their gradient and
                               momentum tiles stay in LDS across the two whole-tensor
                               dependencies of Algorithm 2 (r_t, c_t before any u_t; RMS(u_t) of
                               Eq. 1 before any u^_t), so g, M and theta cross the memory bus once
                               per step instead of three, two and one times.  Same arithmetic per
                               element; the partial sums are added in a different (fixed) order, so
                               results agree with the streaming path to rounding, not bit for bit.
                               The workgroups of a matrix meet four times per step through device
                               memory; with at most 512 tiles of 8192 elements on the chip and about
                               45 microseconds from a tile's first load to its last store, the path
                               tops out near 9e10 parameters per second, below the streaming sweeps */
} came_resident_mode;

/* One parameter tensor.  ndim == 2: rows x cols matrix (factored statistics).
 * ndim == 1: vector of `rows` entries, cols must be 1 (unfactored statistics).
 * Parameters (theta) and the factored statistics are binary32; the gradient dtype is
 * per tensor, the momentum dtype per context (came_options). */
typedef struct {
    int64_t rows;
    int64_t cols;
    int32_t ndim;
    int32_t grad_dtype; /* came_grad_dtype */
} came_tensor_desc;

/* Hyper-parameters of Algorithm 2's input list, passed per call so that the
 * caller can schedule them.  Doubles, so that 1-beta is formed without first
 * rounding beta to binary32 (1-0.9999f is off by 1e-3 relative). */
typedef struct {
    double beta1;  /* EMA coefficient of the momentum M,          [0,1) */
    double beta2;  /* EMA coefficient of r, c (second moment),    [0,1) */
    double beta3;  /* EMA coefficient of R, C (confidence),       [0,1) */
    double eps1;   /* added to g^2 inside the row/column sums,    >= 0  */
    double eps2;   /* added to U inside the row/column sums,      >= 0  */
    double clip_d; /* RMS clipping threshold d of Eq. 1,          > 0   */
    double weight_decay; /* lambda >= 0 of a decoupled weight decay (not in the paper): theta
                            shrinks by eta*lambda*theta before the update, i.e.
                            theta_t = (1 - eta lambda) theta_{t-1} - eta M_t / sqrt(S_t);
                            0 = Algorithm 2 as printed */
} came_hyper;

/* Planner knobs; pass NULL for defaults.  Zero in a field means "default". */
typedef struct {
    int32_t tile_rows;       /* rows of a matrix one workgroup sweeps per tile in the two sweeps
                                that form sums (r_t, c_t; the statistics of u_t): multiple of 4,
                                4..1024; 0 = chosen from the list so the launch fills the GPU */
    int32_t algo;            /* came_algo */
    int64_t group_elements;  /* 0 = all tensors in one launch group; otherwise consecutive
                                tensors are packed into groups of at most about this many
                                elements and the phases run group after group, so that a
                                group's gradient and momentum can stay in the on-package cache
                                between phases */
    int32_t momentum_dtype;  /* came_momentum_dtype, for every tensor of the context */
    int32_t vector_rule;     /* came_vector_rule */
    int32_t resident;        /* came_resident_mode.  A matrix takes the on-chip path when its columns
                                are a multiple of 8, Algorithm 2 is selected and its
                                ceil(rows/16) * ceil(cols/512) tiles fit the co-resident grid (512
                                workgroups on MI355X); came_plan_traffic reports what was chosen */
    int32_t resident_wait_us; /* upper bound, in microseconds, of any single wait of a workgroup of
                                the on-chip kernel for the others of its matrix; 0 = 2 000 000.  When
                                it runs out the kernel flags the failure, every workgroup stops
                                waiting and the launch ends normally; the next came_step or
                                came_device_status on the context returns CAME_ETIMEOUT */
    int32_t tile_rows3;      /* rows per tile of the update sweep (M_t, theta_t), which forms no
                                sums and so has no per-tile results to pay for: multiple of 4,
                                4..1024; 0 = 12 (16 under CAME_MOMENTUM_BF16).  Short tiles keep the addresses that are read and
                                written at any one time close together, which is what the memory
                                system wants of a stream pair that reads and writes the same
                                arrays (tall tiles: up to 20 % slower, depending on where the
                                arrays lie) */
    int32_t reserved;        /* must be 0 */
} came_options;

/* Device addresses of one tensor's state inside the caller's state blob.
 * Matrix: m = M (rows*cols), r, R (rows), c, C (cols).
 * Vector: m = M, r = v, R = s (rows each); c = C = NULL.   All binary32, except m under
 * CAME_MOMENTUM_BF16: rows*cols bfloat16. */
typedef struct {
    void *m, *r, *c, *R, *C;
} came_state_view;

typedef struct came_ctx came_ctx;

/*
 * Bytes the caller must provide for the optimizer state (Algorithm 2's M, r,
 * c, R, C for every tensor: rows*cols + 2(rows+cols) floats per matrix, 3*rows
 * per vector, each array padded to 256 B; M takes 2 bytes per entry instead of 4
 * under CAME_MOMENTUM_BF16) and for the library's scratch
 * (tile/descriptor tables, per-tile partial sums, per-tensor scalars).
 * Host-only: touches no device.  descs: host, `count` entries.
 */
int came_state_size(const came_tensor_desc *descs, int32_t count, const came_options *opts,
                    size_t *state_bytes, size_t *scratch_bytes);

/*
 * Creates a context for the tensor list, uploads the launch plan into
 * `scratch_dev` and zero-fills `state_dev` (M_0 = r_0 = c_0 = 0 from
 * Algorithm 2's input list; R_0 = C_0 = 0 likewise) on `hip_stream`
 * (a hipStream_t, or NULL for the default stream).  state_dev / scratch_dev:
 * device, 256-byte aligned, at least the sizes came_state_size reports; they
 * must stay valid and untouched by others (except through came_state_view)
 * until came_destroy.  *out receives the context.
 */
int came_init_state(came_ctx **out, const came_tensor_desc *descs, int32_t count,
                    const came_options *opts, void *state_dev, size_t state_bytes,
                    void *scratch_dev, size_t scratch_bytes, void *hip_stream);

/*
 * One optimizer step over the whole list (Algorithm 2, one iteration of the
 * loop; Algorithm 1 if the context was created with CAME_ALGO_ADAFACTOR).
 * theta_dev / grad_dev: host arrays of `count` device pointers, one per
 * tensor in descriptor order; theta[i] (binary32, updated in place) and
 * grad[i] (dtype of the descriptor, read only) are contiguous and 16-byte
 * aligned.  No parameter may overlap any other buffer of the call or the
 * state/scratch blobs (CAME_EINVAL, checked whenever an address differs from
 * the previous call's); gradients are only read and may share memory with
 * each other.
 * lr is the learning rate eta; step is the 1-based iteration number t, which
 * is validated (must be >= 1) and recorded but, as in Algorithm 2, never used
 * in the arithmetic.  Asynchronous on hip_stream.
 * On lists of at most 2^29 parameters the update sweep walks its tiles forwards on a
 * context's 1st, 3rd, ... call and backwards on the others (it then starts on the
 * entries the previous call left in the on-package cache); that sweep forms no sums,
 * so results do not depend on the order, bit for bit.
 * Stream capture: a call whose parameter/gradient addresses are those of the previous call
 * on this context only enqueues kernels and may be captured into a HIP graph (no memset
 * nodes).  A call with a changed address has to wait for a free slot of the pointer table
 * and copy from host staging memory; issued while hip_stream is capturing it is refused
 * with CAME_EINVAL and nothing is recorded -- make one eager call with the final
 * addresses first.  The phase timer must be off during capture.
 */
int came_step(came_ctx *ctx, void *const *theta_dev, const void *const *grad_dev,
              const came_hyper *hyper, double lr, int64_t step, void *hip_stream);

/*
 * came_step that also leaves a bfloat16 copy of the updated parameters, for trainers that
 * keep fp32 master weights and compute in bf16: the copy is written by the same sweep
 * that updates theta (2 more bytes per parameter written instead of a separate 6-byte
 * cast pass).  theta_bf16_dev: host array of `count` device pointers; entry i is NULL
 * (no copy for tensor i) or a contiguous, 16-byte aligned buffer of rows*cols bfloat16
 * that aliases nothing else.  The copy is theta_t rounded to nearest even, NaN kept NaN.
 * Everything else as came_step.
 */
int came_step_bf16_copy(came_ctx *ctx, void *const *theta_dev, const void *const *grad_dev,
                        void *const *theta_bf16_dev, const came_hyper *hyper, double lr,
                        int64_t step, void *hip_stream);

/*
 * came_step for callers that cannot allocate device memory or keep a context: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  One call does what
 * came_init_state + came_step do, with the library's OWN scratch: a 16 MiB array that is part
 * of the loaded code object (one copy per GPU, held until the process ends) takes the place
 * of the caller's scratch blob.  The call allocates and frees no device or pinned memory,
 * creates no event and copies nothing with a copy engine: the launch plan is rebuilt on the
 * host (a few KB of ordinary heap) and reaches the GPU inside kernel argument blocks, then
 * the streaming kernels of came_step run on hip_stream (never the on-chip path of
 * came_options.resident, which needs a context to report to: CAME_RESIDENT_ON is refused with
 * CAME_EINVAL, CAME_RESIDENT_AUTO means off here).  Results are bit-identical to
 * came_init_state + came_step with the same options and CAME_RESIDENT_OFF.
 *   descs, count, opts: as for came_init_state; at most 64 tensors, and came_state_size's
 *     scratch_bytes for them must not exceed 16 MiB (roughly: the matrices' row counts times
 *     their number of 512-column blocks plus their column counts times their number of row
 *     blocks, times 24 bytes) and the tile tables 256 KiB -- otherwise CAME_ESIZE and nothing
 *     is enqueued.
 *   state_dev, state_bytes: the caller's state blob (device, 256-byte aligned, at least
 *     came_state_size's state_bytes), input and output; zero_state != 0 zero-fills it first
 *     (Algorithm 2's M_0 = r_0 = c_0 = 0), which is how the first step starts.
 *   theta_dev, grad_dev, hyper, lr, step, hip_stream: as for came_step.
 * Every call on a GPU uses that GPU's one array, which keeps the previous call's contents:
 * each call rewrites the tables and clears the scalars it needs, so calls of any sizes may
 * follow each other on one stream (or on streams ordered with each other), but calls that
 * overlap in time on one GPU race on it.  The first call on a device resolves the array's
 * device address (which may load the code object there): make it outside stream capture.
 * A failed HIP call gives CAME_EHIP; came_last_hip_error(NULL) then returns the hipError_t of
 * the last such failure on the calling thread.
 */
int came_step_noalloc(const came_tensor_desc *descs, int32_t count, const came_options *opts,
                      void *state_dev, size_t state_bytes, int32_t zero_state, void *const *theta_dev,
                      const void *const *grad_dev, const came_hyper *hyper, double lr, int64_t step,
                      void *hip_stream);

/*
 * Waits for hip_stream and reports whether the on-chip kernel of any step so far gave up a wait
 * (CAME_ETIMEOUT, see there), else CAME_OK.  came_step itself reports the same condition as soon
 * as it is visible on the host, without waiting.  Must not be called while the stream is
 * capturing.
 */
int came_device_status(came_ctx *ctx, void *hip_stream);

/* Device addresses of tensor i's state arrays, for checkpointing and tests: the quantities
 * Algorithm 2 carries from one iteration to the next -- m, r, c of its input list and the
 * confidence statistics R, C of its last lines (both start at zero like r, c). */
int came_state_view_get(const came_ctx *ctx, int32_t i, came_state_view *view);

/*
 * Plan introspection (host only, no device): fills out[0..7] with
 * { tile_rows chosen, tile_cols, number of work items (matrix tiles + vectors),
 *   number of finalize workgroups per phase, number of launch groups,
 *   number of matrices, number of vectors, total elements }.
 */
int came_plan_query(const came_tensor_desc *descs, int32_t count, const came_options *opts,
                    int64_t out[8]);

/*
 * What the planner chose for the list and what one step then moves (host only, no device):
 * out[0] = matrices on the on-chip path, out[1] = their elements,
 * out[2] = algorithmic HBM bytes of one step of the whole list as planned (streaming matrices
 *          came_algorithmic_bytes(.., 0) per element, on-chip ones came_algorithmic_bytes(.., 4),
 *          1-D parameters 24 + grad_bytes + 2*momentum_bytes),
 * out[3] = the same if every matrix took the streaming path.
 */
int came_plan_traffic(const came_tensor_desc *descs, int32_t count, const came_options *opts,
                      double out[4]);

/*
 * Algorithmic HBM bytes per parameter of the shipped three-sweep design (the count the
 * roofline fraction is priced with; derived from the dependency chain of Algorithm 2:
 * r_t, c_t complete before any u_t, RMS(u_t) of Eq. 1 complete before any u^_t, m_t).
 * grad_bytes 4 or 2 (came_grad_dtype), momentum_bytes 4 or 2 (came_momentum_dtype), algo a
 * came_algo (Algorithm 1's sweep 2 does not read M).  Sweep 1 reads g; sweep 2 reads g
 * and M; sweep 3 reads g, M, theta and writes M, theta:
 *   8 + 3*grad_bytes + 3*momentum_bytes   (Algorithm 1: ... + 2*momentum_bytes),
 * i.e. 20 + 3*grad_bytes with a binary32 momentum.
 * which: 0 = whole step, 1/2/3 = that sweep alone, 4 = whole step of a matrix on the on-chip
 * path (came_options.resident): g, M and theta read once, M and theta written once,
 *   8 + grad_bytes + 2*momentum_bytes,
 * the compulsory count.  Returns 0 for arguments out of range.
 */
double came_algorithmic_bytes(int32_t grad_bytes, int32_t momentum_bytes, int32_t algo, int32_t which);

/*
 * Placement probe.  On MI355X the time of a sweep that streams from two or three arrays at
 * once -- above all the one sweep that both reads and writes (sweep 3: theta and M in
 * place) -- depends on WHERE the caller's buffers sit physically: when theta and the state
 * blob share one of the HBM's three 96 GB address regions the mixed read/write stream runs
 * at about 5.4 TB/s, when they sit in different regions at about 6.2 TB/s (pure reads
 * of one array and pure writes do not care; sweep 2's two read streams g and M gain 2.5-5 %).
 * Measured cost of not caring, state blob wherever a fresh allocator puts it (directly behind
 * the parameters and gradients): a whole step takes about 10 % longer on a
 * 6.7-billion-parameter list and 0-9 % longer on lists of 0.1-0.4 billion parameters.
 * The library owns no memory, so it can only measure: this call runs the memory traffic of
 * sweep 3 over every matrix (theta and M read and written back with their own bits; nothing
 * changes) and, when grad_dev is given, also reads g in that pass and first runs the traffic
 * of sweep 2 (g and M read), `repeats` times on hip_stream, waits, and reports the achieved
 * GB/s over all of it (0 if the list has no matrix).  A caller can allocate its state blob at
 * several addresses, probe each against its parameters (and gradient buffers, if those are
 * long-lived) and keep the fastest.  theta_dev: host array of `count` device pointers as for
 * came_step; grad_dev: the same for the gradients, or NULL.  Synchronises the stream; must
 * not be called while the stream is capturing.  Valid any time after came_init_state.
 */
int came_probe_placement(came_ctx *ctx, void *const *theta_dev, const void *const *grad_dev,
                         void *hip_stream, int32_t repeats, double *gbytes_per_s);

/*
 * Built-in phase timer.  While enabled, came_step brackets each of its
 * launches with HIP events on the step's stream.  came_profile_read waits for
 * the recorded events, adds the elapsed milliseconds and launch counts per
 * phase { sweep 1, finalize 1, sweep 2, finalize 2, sweep 3, vectors, on-chip kernel } since
 * the previous read into phase_ms[7] / phase_launches[7], and forgets them.
 * "vectors" counts only launches of their own (long 1-D parameters, groups
 * without a matrix); ordinary 1-D parameters are updated by the first workgroups
 * of the sweep-3 launch and count there.
 * At most 65536 launches are kept between reads; further ones go untimed.
 */
int came_profile_enable(came_ctx *ctx, int32_t on);
int came_profile_read(came_ctx *ctx, double phase_ms[7], int64_t phase_launches[7]);

/* hipError_t of the last failed HIP call on this context (0 if none); with ctx == NULL, of the
 * last failed HIP call inside came_step_noalloc on the calling thread. */
int came_last_hip_error(const came_ctx *ctx);

/* Releases the host context.  Does not touch or free any device memory and
 * does not synchronise: the caller must keep the blobs alive until work
 * already enqueued has finished. */
void came_destroy(came_ctx *ctx);

/* Static, never NULL. */
const char *came_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* CAME_H */
