/*
 * lagom.h -- C ABI of the MI355X (gfx950) hot path of Lagom: one GPU's share of an
 * overlapped training step, and the host-side model and search that tune it.
 *
 * Conventions common to every call
 *   - Plain C types only.  "device pointer" = address in this GPU's HBM (hipMalloc or
 *     a torch tensor's data_ptr); "host pointer" = ordinary process memory.
 *   - The caller owns every buffer and both streams.  The library allocates no device
 *     memory.  Host structs and host pointer arrays are read during the call only.
 *   - Return value: LAGOM_OK (0) or a negative LAGOM_E* code; lagom_last_error()
 *     gives the text for the calling thread.  Nothing is thrown across the boundary.
 *   - Times are microseconds (double), bandwidths bytes per microsecond, sizes bytes.
 */
#ifndef LAGOM_H
#define LAGOM_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define LAGOM_OK          0
#define LAGOM_EINVAL    (-1)  /* bad argument (null, out of range, inconsistent)          */
#define LAGOM_EALIGN    (-2)  /* a device pointer is not 16-byte aligned                  */
#define LAGOM_EHIP      (-3)  /* the HIP runtime reported an error                        */
#define LAGOM_ECALLBACK (-4)  /* the profile callback failed; outputs hold best-so-far    */

#define LAGOM_MAX_SRCS     16
#define LAGOM_MAX_DSTS      4
#define LAGOM_MAX_LAUNCHES 256  /* kernel launches per stream in one overlap group        */
#define LAGOM_MAX_COMMS    64   /* tunable communications in one overlap group            */
#define LAGOM_MAX_STEPS    32   /* local steps in one lagom_comm_steps launch             */
#define LAGOM_MAX_STEP_PTRS 96  /* sources and destinations of all its steps together     */

/* The three resource-related parameters of a communication (Sec. 2.2 and Sec. 3.2):
 * number of channels NC (= workgroups), threads per block NT, chunk size C in bytes. */
typedef struct {
    int32_t nc;
    int32_t nt;
    int64_t chunk_bytes;
} lagom_cfg;

typedef enum { LAGOM_F32 = 0, LAGOM_BF16 = 1 } lagom_dtype;
typedef enum { LAGOM_REDUCE_COPY = 0, LAGOM_GATHER_COPY = 1 } lagom_op;

const char* lagom_strerror(int code);   /* static text for a LAGOM_E* code              */
const char* lagom_last_error(void);     /* detail of the calling thread's last failure  */

/* ---------------------------------------------------------------------------------
 * lagom_comm_kernel -- the local data-movement step of a chunked collective
 * (Sec. 3.2, "Global Resource Competition": a communication launches NC thread blocks
 * that move data at granularity C; Sec. 2.1 names the collectives).
 *
 *   LAGOM_REDUCE_COPY: for every element i < count and every destination d
 *       dsts[d][i] = round_dt(((src0[i] + src1[i]) + src2[i]) + ...)
 *     fp32 additions in source order, bf16 widened exactly, one round-to-nearest-even
 *     at the store.  Every source and destination holds `count` elements.
 *   LAGOM_GATHER_COPY: dsts[d][r*count + i] = srcs[r][i]; every destination holds
 *     nsrc*count elements (concatenation in rank order).
 *
 * The grid is cfg->nc workgroups of cfg->nt threads; chunk g (cfg->chunk_bytes bytes,
 * numbered shard by shard, the last one of a shard may be short) is moved by
 * workgroup g mod nc.  The result does not depend on cfg.
 *
 *   srcs, dsts : HOST arrays of DEVICE pointers, 16-byte aligned.  Buffers must not overlap in part;
 *                a reduce-copy destination may be exactly one of its sources (in-place
 *                accumulation: every element is read before the same lane writes it).
 *   nsrc 1..LAGOM_MAX_SRCS, ndst 1..LAGOM_MAX_DSTS, count >= 0 (0 launches nothing).
 *   cfg        : nc >= 1; nt a multiple of 64 in 64..1024; chunk_bytes a positive
 *                multiple of 16.
 *   hip_stream : a hipStream_t (0 = the null stream).  Enqueue only: no synchronisation.
 * Errors: LAGOM_EINVAL, LAGOM_EALIGN, LAGOM_EHIP.  Byte counts that are not multiples
 * of 16 are handled (a short tail), not rejected.
 */
int lagom_comm_kernel(lagom_op op, lagom_dtype dt,
                      const void* const* srcs, int nsrc,
                      void* const* dsts, int ndst,
                      int64_t count, const lagom_cfg* cfg, void* hip_stream);

/* lagom_comm_kernel_lds -- lagom_comm_kernel with every source vector staged through LDS: direct-to-LDS
 * loads of 16 bytes per lane fill a ring of stages per wavefront (8 KiB per wavefront), the next stages in
 * flight while the current one is read back and folded, in source order.  Same arguments, same result bit
 * for bit, same chunk-to-channel assignment; a workgroup holds (nt / 64) * 8 KiB of LDS, so it shares a
 * compute unit only with workgroups that leave that much (lagom_gemm's leave none).  A gather-copy whose
 * shards are not multiples of 16 bytes is passed on to lagom_comm_kernel.  Slower than the register path
 * on gfx950 (measured); kept for comparison. */
int lagom_comm_kernel_lds(lagom_op op, lagom_dtype dt,
                          const void* const* srcs, int nsrc,
                          void* const* dsts, int ndst,
                          int64_t count, const lagom_cfg* cfg, void* hip_stream);

/* ---------------------------------------------------------------------------------
 * lagom_comm_steps -- several local steps of ONE collective in one kernel launch (Sec. 2.1: a ring
 * all-reduce is P-1 reduce steps followed by P-1 copy steps; Sec. 3.2: the collective's NC thread
 * blocks stay for the whole operator).  The cfg->nc channels are persistent: every channel walks
 * the steps in order and takes chunks k, k+nc, ... of each, with no synchronisation between
 * channels, exactly as nsteps calls of lagom_comm_kernel would assign them, without the nsteps-1
 * launch boundaries in between.
 *
 *   steps[nsteps] : host array; step i is a reduce-copy of nsrc sources into ndst destinations, or
 *                   a gather-copy of ONE source (a plain copy, e.g. store-and-forward) into ndst
 *                   destinations.  Every buffer of every step holds `count` elements of dt, so a given
 *                   element is moved by the same lane in every step.
 *   Ordering      : a location that one step writes and a later step reads or overwrites THROUGH
 *                   THE SAME POINTER is handled in step order (same lane, program order).  Buffers
 *                   of different steps that overlap only in part are refused (LAGOM_EINVAL).
 *   nsteps 1..LAGOM_MAX_STEPS, at most LAGOM_MAX_STEP_PTRS buffers in all steps together;
 *   pointers 16-byte aligned; cfg as for lagom_comm_kernel.  Enqueue only.
 * The result equals that of the nsteps separate launches in order, bit for bit.
 * Errors: LAGOM_EINVAL, LAGOM_EALIGN, LAGOM_EHIP.
 */
typedef struct {
    int32_t op;                 /* lagom_op                                             */
    const void* const* srcs;    /* host array of device pointers                        */
    int32_t nsrc;
    void* const* dsts;          /* host array of device pointers                        */
    int32_t ndst;
} lagom_comm_step;
int lagom_comm_steps(lagom_dtype dt, const lagom_comm_step* steps, int nsteps, int64_t count,
                     const lagom_cfg* cfg, void* hip_stream);

/* ---------------------------------------------------------------------------------
 * lagom_gemm -- the computation whose slow-down under contention is studied
 * (Sec. 3.2, Fig. 3: an FFN matrix multiply next to a collective).
 *
 *   C[M,N] = A[M,K] . B, bf16 inputs, fp32 accumulation on the matrix cores.
 *   A : device, row-major [M,K] bf16.
 *   B : device, bf16, row-major [N,K] when b_is_nk != 0 (weight layout), else [K,N].
 *   C : device, row-major [M,N], bf16 (round-to-nearest-even) or fp32 per out_dt.
 *   M, N, K >= 1; K a multiple of 8 (16-byte rows); [K,N] also needs N a multiple of 8;
 *   pointers 16-byte aligned.  Fastest when K is a multiple of 64; K < 64 takes a slow path.
 * Enqueue only on hip_stream.  Errors: LAGOM_EINVAL, LAGOM_EALIGN, LAGOM_EHIP.
 */
int lagom_gemm(const void* A, const void* B, void* C, int64_t M, int64_t N, int64_t K,
               int b_is_nk, lagom_dtype out_dt, void* hip_stream);

/* Workgroup geometry of lagom_gemm for a problem size, as the cost model needs it
 * (Eq. 5-6: mu = total workgroups, TB = workgroups resident per compute unit,
 * D = bytes each workgroup reads and writes).  The tiling depends on the size only: the smallest
 * of 128 x 128, 256 x 128 and 256 x 256 of which at most 256 tiles cover C (256 x 256 whenever
 * K < 64 or K > 2^22).  Host only. */
typedef struct {
    int64_t mu;
    int32_t tb;
    double  d_bytes;
    int32_t tile_m, tile_n, tile_k, threads;
    double  d_bytes_past_l2;    /* estimate of the bytes of d_bytes that leave an XCD's L2: the kernel's
                                   tile order gives the n (up to 32) workgroups an XCD runs at a time a
                                   block of r x c tiles that share r A panels and c B panels, so a
                                   workgroup's share is (r*tile_m + c*tile_n)*K*2/n + tile_m*tile_n*out_size */
} lagom_gemm_geometry;
int lagom_gemm_describe(int64_t M, int64_t N, int64_t K, lagom_dtype out_dt, lagom_gemm_geometry* out);

/* ---------------------------------------------------------------------------------
 * lagom_overlap_run -- execute one overlap group and time it (Sec. 3.1, Eq. 1:
 * communications serialized on one stream, computations on another, makespan
 * Z = time until both have drained; this is also Alg. 2's ProfileTime).
 */
typedef struct {
    int32_t op;                 /* lagom_op                                             */
    int32_t dtype;              /* lagom_dtype                                          */
    const void* const* srcs;    /* host array of device pointers                        */
    int32_t nsrc;
    void* const* dsts;          /* host array of device pointers                        */
    int32_t ndst;
    int64_t count;
    int32_t comm_id;            /* the tunable communication this launch belongs to:
                                   index into cfgs; launches of one id are contiguous  */
    int32_t after_comp;         /* index of a computation that must have finished before this
                                   launch starts, or -1 (honoured in LAGOM_CORUN only)  */
    int32_t lds_staged;         /* non-zero: issue this launch through lagom_comm_kernel_lds (not
                                   together with fuse_with_prev: LAGOM_EINVAL)                  */
    int32_t fuse_with_prev;     /* non-zero: issue this launch in the same kernel launch as the
                                   previous one (lagom_comm_steps).  Needs the same comm_id, dtype
                                   and count as the previous launch, after_comp == -1, and the
                                   shape rules of lagom_comm_steps; otherwise LAGOM_EINVAL      */
} lagom_comm_desc;

typedef struct {
    const void* A; const void* B; void* C;
    int64_t M, N, K;
    int32_t b_is_nk;
    int32_t out_dtype;
    int32_t after_comm_id;      /* communication (comm_id) whose last launch must have finished
                                   before this GEMM starts, or -1 (LAGOM_CORUN only)    */
} lagom_gemm_desc;

typedef enum { LAGOM_ALONE_COMM = 0, LAGOM_ALONE_COMP = 1, LAGOM_CORUN = 2 } lagom_run_mode;

typedef struct {
    double X_us;      /* communication stream: first kernel start to last kernel end    */
    double Y_us;      /* computation stream: likewise                                   */
    double Z_us;      /* common start to the later of the two ends                      */
    double* x_us;     /* host [ncfg]  per communication (nullable)                      */
    double* y_us;     /* host [ncomp] per computation   (nullable)                      */
    /* Spread over the `iters` repetitions, as median absolute deviations (outputs; a caller that
     * does not want x_mad_us sets it to null before the call):                             */
    double* x_mad_us; /* host [ncfg]  per communication (nullable)                      */
    double Ysum_us;   /* median over repetitions of sum_i y_i of that repetition        */
    double Ysum_mad_us;
    double Z_mad_us;
    /* Release of each stream: common start to the start of its first kernel.  The common start is the earlier of
     * the two (so one of them is 0, as is that of a stream that did not run); in a co-run without cross-stream
     * dependencies they differ by a microsecond or so.                                                            */
    double comm_start_us;
    double comp_start_us;
} lagom_timing;

/*   launches[nlaunch] : communication kernels in stream order; cfgs[ncfg] their
 *                       parameters, selected by comm_id.
 *   comps[ncomp]      : GEMMs in stream order.
 *   comm_stream, comp_stream : two distinct hipStream_t of default priority.
 *   Each of warmup + iters repetitions starts both streams together behind a gate and
 *   drains both before the next; every value reported is the median over `iters`.  In LAGOM_CORUN
 *   the gate is a bounded delay kernel on either stream; the two agree on the instant of release
 *   through 16 bytes of pinned host memory that the library allocates once per device and keeps
 *   (calls that overlap in time on one device share it and may delay each other's release).
 *   Cross-stream dependencies (after_comp / after_comm_id) are enforced with events in
 *   LAGOM_CORUN; the two enqueue orders are merged on the host so that every awaited event
 *   has been recorded first, and a dependency cycle is LAGOM_EINVAL.  With dependencies X and
 *   Y still run from a stream's first kernel start to its last kernel end (waits included).
 *   The call synchronises both streams and owns its events.
 * Errors: LAGOM_EINVAL, LAGOM_EALIGN, LAGOM_EHIP.
 */
int lagom_overlap_run(const lagom_comm_desc* launches, int nlaunch,
                      const lagom_cfg* cfgs, int ncfg,
                      const lagom_gemm_desc* comps, int ncomp,
                      void* comm_stream, void* comp_stream,
                      int warmup, int iters, int mode, lagom_timing* out);

/* Sustained rate of an overlap group (the executor path of a training loop): `steps` repetitions of
 * the group of lagom_overlap_run(LAGOM_CORUN) are enqueued back to back; between repetitions the two
 * streams wait for each other through events, with no host synchronisation and no start gate, so a
 * repetition starts when the previous one has ended on both streams while the host is already
 * enqueueing later ones.  *us_per_step = device time from the start of the first repetition to the
 * end of the last, divided by steps.  Cross-stream dependencies inside the group are honoured as
 * in lagom_overlap_run.  Synchronises both streams before it returns.
 * Errors: as lagom_overlap_run (a pair of streams that does not overlap is LAGOM_EINVAL). */
int lagom_overlap_steps(const lagom_comm_desc* launches, int nlaunch,
                        const lagom_cfg* cfgs, int ncfg,
                        const lagom_gemm_desc* comps, int ncomp,
                        void* comm_stream, void* comp_stream, int steps, double* us_per_step);

/* As lagom_overlap_steps, replayed from a HIP graph: after one eager repetition, one repetition is
 * captured from both streams (the computation stream forks from and joins the communication stream
 * through events) and the graph is launched `steps` times on the communication stream.  The host
 * enqueues one graph launch per step instead of every kernel.  Neither stream may be capturing when
 * the call is made; both are synchronised before it returns.  Errors: as lagom_overlap_steps. */
int lagom_overlap_steps_graph(const lagom_comm_desc* launches, int nlaunch,
                              const lagom_cfg* cfgs, int ncfg,
                              const lagom_gemm_desc* comps, int ncomp,
                              void* comm_stream, void* comp_stream, int steps, double* us_per_step);

/* Whether kernels enqueued on the two streams can run at the same time.  HIP multiplexes streams
 * onto a few hardware queues (4 per process by default); two streams that share a queue run their
 * kernels in submission order, and an overlap measured on them is a serial run.  Probes with two
 * bounded delay kernels (0.3 ms; 3 ms more before it answers 0) and synchronises both streams.  *overlap = 1 or 0; 0 for
 * stream_a == stream_b.  lagom_overlap_run(LAGOM_CORUN) makes this check itself and returns
 * LAGOM_EINVAL for a pair that does not overlap.  Errors: LAGOM_EINVAL (null output), LAGOM_EHIP. */
int lagom_streams_overlap(void* stream_a, void* stream_b, int* overlap);

/* ---------------------------------------------------------------------------------
 * lagom_contention_sweep -- the contention profiler (the experiment of Fig. 3,
 * Sec. 3.2): for every configuration of a list, applied to all communications of
 * the group, time the communications alone, the computations alone (once), and both
 * together, and derive the communication's global-memory bandwidth V (Eq. 6).  The computations
 * alone are re-timed every eighth point (the clock held under load drifts over a long sweep).
 */
typedef struct {
    lagom_cfg cfg;
    double comm_alone_us, comm_corun_us;     /* X = sum of the x_j (Eq. 1)              */
    double comp_alone_us, comp_corun_us;     /* Y = sum of the y_i (waits not included) */
    double z_corun_us;
    double v_alone, v_corun;                 /* algorithmic bytes / X, bytes per us     */
} lagom_sweep_point;

int lagom_contention_sweep(const lagom_comm_desc* launches, int nlaunch, int ncfg,
                           const lagom_gemm_desc* comps, int ncomp,
                           const lagom_cfg* points, int npoints,
                           void* comm_stream, void* comp_stream,
                           int warmup, int iters, lagom_sweep_point* out /* [npoints] */);

/* Algorithmic bytes of one launch: (S + D) * count * element size for a reduce-copy,
 * (1 + D) * S * count * element size for a gather-copy.  Host only; -1 on bad input. */
int64_t lagom_comm_bytes(int op, int dtype, int nsrc, int ndst, int64_t count);

/* ---------------------------------------------------------------------------------
 * lagom_cost_model -- the unified overlap cost model (Eq. 1) over the contention wave
 * model (Eq. 4-6, notation of Table 1).  Host only; no GPU is touched.
 *
 *   y_i = sum_j f_ij * g_ij,  g_ij = ceil(mu_i / ((lambda - NC_j) * TB_i)),
 *   f_ij = theta_i + (lambda - NC_j) * TB_i * D_i / (B - V(NC_j, C_j)),
 *   X = sum_j x_j, Y = sum_i y_i, Z = max(X, Y).
 * x_j and V come from per-communication tables keyed by the exact (NC, NT, C).
 * With several communications the two serialized queues are stepped wave by wave:
 * communication j is active on [sum_{<j} x, sum_{<=j} x); a wave that starts under j
 * (or after the last one: NC = 0, V = 0) retires min(remaining, (lambda-NC_j)*TB_i)
 * workgroups and lasts f_ij; g_ij counts the waves issued under j.
 * With dependencies each stream stays serial, an operator starts at the later of its stream
 * being free and its dependency having ended, the wave stepping is unchanged, and Z is the later
 * of the two stream ends (X and Y remain the sums of the x_j and y_i).  A dependency cycle is
 * LAGOM_EINVAL.
 */
typedef struct { lagom_cfg cfg; double x_us; double v; } lagom_table_entry;
typedef struct { const lagom_table_entry* entries; int32_t n; } lagom_comm_table;
typedef struct { int64_t mu; int32_t tb; double d_bytes; double theta_us; } lagom_comp_model;
typedef struct { int32_t nt; double rho; } lagom_penalty;
typedef struct {
    int32_t lambda;                  /* compute units                                   */
    double  bw_peak;                 /* B, bytes per microsecond                        */
    const lagom_comp_model* comps;   /* host [ncomp]                                    */
    int32_t ncomp;
    const lagom_comm_table* tables;  /* host [ncomm]                                    */
    int32_t ncomm;
    /* Optional cross-stream dependencies (both nullable = none, the literal Eq. 1).  The overlap
     * patterns of Sec. 2.1 have them: an FSDP layer's GEMM needs its all-gathered weights, a
     * pipelined TP batch's all-reduce needs that batch's GEMM.                                  */
    const int32_t* comp_after_comm;  /* host [ncomp]: communication that must have ended before
                                        computation i starts, or -1                              */
    const int32_t* comm_after_comp;  /* host [ncomm]: computation that must have ended before
                                        communication j starts, or -1                            */
    /* Not in the paper; 0 gives Eq. 5-6 exactly.  Fraction sigma in [0, 1] of a compute unit that
     * stays available to the computation while a channel runs on it: the workgroups in flight
     * become floor((lambda - NC*(1 - sigma)) * TB) in Eq. 5 and Eq. 6.  On this part a channel's
     * wavefronts fit beside the GEMM's on the same compute unit (sigma near 1): the channel then
     * costs the computation bandwidth (V), not compute units.                                  */
    double corun_share;
    /* Not in the paper either; null / 0 gives Eq. 6 exactly.  A wave of a computation issued while a
     * communication whose channels have nt threads is active lasts f_ij * (1 + rho) for the entry with that
     * nt (first match; no entry: rho = 0).  On this part the computation is slowed for as long as channels
     * are resident, by an amount that depends on how heavy one channel is and hardly on how many there are:
     * neither (lambda - NC) nor B - V can express that.                                             */
    const lagom_penalty* penalty;    /* host [npenalty], nullable                                   */
    int32_t npenalty;
} lagom_model;
typedef struct {
    double X_us, Y_us, Z_us;
    double*  x_us;   /* host [ncomm] (nullable)                                         */
    double*  y_us;   /* host [ncomp] (nullable)                                         */
    int32_t* g;      /* host [ncomp * (ncomm + 1)] wave counts, last column = no
                        communication active (nullable)                                 */
} lagom_pred;

/* Errors: LAGOM_EINVAL for a null pointer, ncomm != model ncomm, a configuration that
 * is not in its table, NC < 1 or NC >= lambda, V < 0 or V >= B, x < 0, mu < 0, TB < 1,
 * corun_share outside [0, 1], a negative rho. */
int lagom_cost_model(const lagom_model* m, const lagom_cfg* cfgs, int ncomm, lagom_pred* out);

/* ---------------------------------------------------------------------------------
 * lagom_model_fill, lagom_model_calibrate -- the contention wave model (Eq. 4-6) filled from a
 * sweep of the contention profiler.  The paper measures x_j (Sec. 3.4, ProfileTime) and names
 * theta and V(NC, C) in Eq. 6 without printing how they are obtained; this is the reading:
 *   t_alone = median over the points (not held out) of comp_alone_us, divided by ncomp;
 *   theta   = t_alone / g0 - lambda*TB*D/B, g0 = ceil(mu / (lambda*TB)), floored at 0
 *             (Eq. 5-6 with no communication active, solved for theta);
 *   per communication j and swept configuration: x_j = (bytes_j / sum bytes) * comm_corun_us,
 *   V = min(v_corun, v_cap_frac * B).
 * Host only.
 */
typedef struct {
    int32_t lambda;             /* compute units                                            */
    double  bw_peak;            /* B, bytes per microsecond                                 */
    int64_t mu; int32_t tb; double d_bytes;   /* geometry shared by the group's computations
                                                 (lagom_gemm_describe)                      */
    int32_t ncomp;
    int32_t ncomm;
    const double* comm_bytes;   /* host [ncomm]: algorithmic bytes of each communication    */
    double  v_cap_frac;         /* V is capped at this fraction of B (Eq. 6 needs V < B);
                                   0 selects 0.99                                           */
} lagom_fill_desc;

/*   pts[npts]     : sweep points (lagom_contention_sweep); held_out[npts] nullable, non-zero =
 *                   the point's standalone time is not used for theta.
 *   entries       : out, host [ncomm * npts]; tables[ncomm] out, pointing into entries;
 *   comps[ncomp]  : out; t_alone_us out, nullable.
 * The caller assembles a lagom_model from tables and comps (and sets dependencies, corun_share).
 * Errors: LAGOM_EINVAL (null, npts < 1, bad description, negative times, all points held out). */
int lagom_model_fill(const lagom_sweep_point* pts, int npts, const uint8_t* held_out, const lagom_fill_desc* d,
                     lagom_table_entry* entries, lagom_comm_table* tables, lagom_comp_model* comps, double* t_alone_us);

/* Picks the co-run share sigma (lagom_model.corun_share) among sigmas[nsigma]: the model is filled
 * as by lagom_model_fill, every candidate is scored by the mean of |Y_model - Y_measured| /
 * Y_measured over the points that are not held out (all communications at the point's
 * configuration), the first smallest mean wins; the same error over the held-out points is
 * reported beside it.  x and V of every point stay in the tables: they are measured inputs of
 * Eq. 1, not predictions.  comp_after_comm / comm_after_comp as in lagom_model (nullable).
 * With nrho > 0 the resident penalty (lagom_model.penalty) is calibrated after sigma: for every thread count
 * among the points not held out, in ascending order, the candidate rho with the smallest mean error over the
 * fitted points of that thread count (first smallest) is written to penalty_out; the errors reported are then
 * those with sigma and every rho in place.  penalty_out needs room for every distinct thread count
 * (LAGOM_EINVAL if penalty_capacity is too small). */
typedef struct {
    double  sigma, theta_us;
    double  fit_mean, fit_max;      /* over the points not held out                         */
    double  held_mean, held_max;    /* over the held-out points (0 when there are none)     */
    int32_t n_fit, n_held;
    int32_t npenalty;               /* entries written to penalty_out                       */
} lagom_calibration;
int lagom_model_calibrate(const lagom_sweep_point* pts, int npts, const uint8_t* held_out, const lagom_fill_desc* d,
                          const int32_t* comp_after_comm, const int32_t* comm_after_comp,
                          const double* sigmas, int nsigma,
                          const double* rhos, int nrho, lagom_penalty* penalty_out, int penalty_capacity,
                          lagom_calibration* out);

/* ---------------------------------------------------------------------------------
 * lagom_tune -- priority-based parameter search (Sec. 3.3-3.4: metric H of Eq. 7,
 * the cost-effectiveness loop of Alg. 1, resource-efficient tuning of Alg. 2), or
 * exhaustive search over the same space.  Host only; all measuring is done by the
 * callback.
 *
 * Space: communication j moves on a ladder of levels 0..K_j-1; level l stands for
 * (nc[min(l,n_nc-1)], nt[min(l,n_nt-1)], chunk[min(l,n_chunk-1)]) over strictly
 * ascending grids, K_j = the longest grid (Alg. 2 raises NC, NT and C together).
 *
 * LAGOM_PRIORITY: all communications start at level 0 and are profiled once; if
 * X < Y the search ends there.  Otherwise, repeatedly: take the not-done
 * communication with the smallest H (initially 0.01; ties to the lowest index), raise
 * it to the lowest level at which every parameter reached min(p*(1+lr), p_max) (one
 * level when it has no lr yet), profile.  If its x rose: done, previous level kept.
 * Else if X' < Y': done, and the new level is kept only if its Z is smaller.  Else the
 * step is accepted, H_j = (Y'-Y)/(x_j-x_j') (+inf for a zero denominator),
 * lr = (x_j-x_j')/x_j', and a communication that reached its top level is done.
 * At most 1 + sum_j K_j profile calls.
 * LAGOM_EXHAUSTIVE: every level vector in lexicographic order; the smallest Z wins,
 * ties to the smallest level sum, then to the lexicographically smallest vector.
 * Refused (LAGOM_EINVAL) above 2^20 vectors.
 * LAGOM_COMM_OPTIMAL: the communication-bound regime (Eq. 2), where Z = sum_j x_j separates:
 * each x_j is minimised on its own over the full (NC, NT, C) product by coordinate descent with
 * measured feedback -- communications in index order, the others staying where they are; start
 * at the minimum of every grid, sweep the coordinates NC, C, NT: one grid step up while x_j falls
 * strictly, else down while it falls strictly; repeat until a sweep changes nothing.  This is
 * the point a tuner that looks at communication time only would pick.  trace->levels receives
 * the NC grid index of every communication; no steps are recorded.
 * LAGOM_HIDE_COMM: the computation-bound objective (Sec. 3.1, Eq. 3: once communication is hidden
 * the makespan is Y, which the communications' resources inflate): the least Y subject to
 * X <= Y.  The loop of LAGOM_PRIORITY with two changes: the baseline ends the search when
 * X <= Y; a trial with X' <= Y' is kept and ends the search for every communication (the lowest
 * resources on the path that hide the communication; raising anything further only adds
 * contention).  If no visited vector hides the communication the result is the priority
 * search's last accepted vector.
 * LAGOM_PRIORITY_FREE: LAGOM_PRIORITY, except that a trial with X' < Y' which also lowered Y (H of Eq. 7
 * negative: the step made the communication faster at no cost to the computation) is accepted like any
 * other step and does not end the communication.  Alg. 2 stops at X' < Y' because more resources can only
 * lengthen the computation (Sec. 3.2); this variant is for hardware on which that does not hold.
 * LAGOM_EXHAUSTIVE_HIDE: every level vector; among those with X <= Y the smallest Y wins (ties:
 * smallest level sum, then lexicographic); if none has X <= Y, the smallest Z as in
 * LAGOM_EXHAUSTIVE.
 */
typedef int (*lagom_profile_fn)(void* user, const lagom_cfg* cfgs, int ncomm,
                                double* x_us /* out [ncomm] */, double* Y_us /* out */);

typedef struct {
    const int32_t* nc;    int32_t n_nc;
    const int32_t* nt;    int32_t n_nt;
    const int64_t* chunk; int32_t n_chunk;
} lagom_tune_space;

typedef struct {
    int32_t comm;         /* -1 for the baseline profile                                */
    int32_t level_from, level_to;
    int32_t accepted, done;
    double  xj_prev, xj_new;     /* NaN on the baseline step                            */
    double  X, Y, Z;             /* of the profiled (trial) configuration               */
    double  H, lr;               /* of `comm` after the step; lr NaN while undefined    */
} lagom_trace_step;

typedef struct {
    lagom_trace_step* steps;     /* host [capacity] (nullable: then only counters)      */
    int32_t capacity;
    int32_t n;                   /* out: steps written (priority mode)                  */
    int32_t calls;               /* out: profile calls made                             */
    double  X, Y, Z;             /* out: of the returned configuration                  */
    int32_t* levels;             /* host [ncomm] out (nullable)                         */
} lagom_trace;

typedef enum { LAGOM_PRIORITY = 0, LAGOM_EXHAUSTIVE = 1, LAGOM_COMM_OPTIMAL = 2,
               LAGOM_HIDE_COMM = 3, LAGOM_EXHAUSTIVE_HIDE = 4, LAGOM_PRIORITY_FREE = 5 } lagom_tune_mode;

/*   spaces[ncomm], out_cfgs[ncomm] host arrays; trace nullable.
 * Errors: LAGOM_EINVAL (null, ncomm < 1 or > LAGOM_MAX_COMMS, empty or non-ascending
 * grid, trace too small), LAGOM_ECALLBACK (callback returned non-zero or a
 * non-finite/negative time: out_cfgs holds the best configuration so far). */
int lagom_tune(const lagom_tune_space* spaces, int ncomm, lagom_profile_fn profile, void* user,
               int mode, lagom_cfg* out_cfgs, lagom_trace* trace);

/* The chunk grid of a ladder.  Chunk g of a launch goes to channel g mod NC, so once
 * chunk * nc_max exceeds the bytes a launch moves per source, some channels of every launch have
 * no chunk; and on a ladder NC and C rise together (Alg. 2).
 *   LAGOM_LADDER_FULL        : the grid as given;
 *   LAGOM_LADDER_CUT         : the chunks with chunk * nc_max <= bytes_per_source (at least the smallest);
 *   LAGOM_LADDER_FIXED_CHUNK : one chunk, the one with the smallest standalone communication time
 *                              among the sweep points with nc == nc_max and nt == nt_ref (first
 *                              smallest in grid order; the ladder then raises NC and NT only).
 * chunk_grid strictly ascending; out_chunks has room for n_chunk values; pts may be null unless
 * kind is LAGOM_LADDER_FIXED_CHUNK.  Host only.  Errors: LAGOM_EINVAL. */
typedef enum { LAGOM_LADDER_FULL = 0, LAGOM_LADDER_CUT = 1, LAGOM_LADDER_FIXED_CHUNK = 2 } lagom_ladder_kind;
int lagom_ladder_chunks(const int64_t* chunk_grid, int n_chunk, int32_t nc_max, int32_t nt_ref, int64_t bytes_per_source,
                        int kind, const lagom_sweep_point* pts, int npts, int64_t* out_chunks, int32_t* out_n);

/* Ready-made callbacks for lagom_tune. */
/* user = const lagom_model*: x_j from the tables, Y from lagom_cost_model.             */
int lagom_model_profile(void* user, const lagom_cfg* cfgs, int ncomm, double* x_us, double* Y_us);
/* user = const lagom_overlap_ctx*: one measured co-run of the group (ProfileTime); x_j per
 * communication and Y = sum of the per-GEMM times y_i, as in Eq. 1.                      */
/* What every call of lagom_overlap_profile measured, in call order (optional). */
typedef struct {
    int32_t capacity;            /* calls the arrays have room for                          */
    int32_t ncomm;               /* row length of cfgs / x_us / x_mad_us                    */
    int32_t n;                   /* out: calls made (recording stops at capacity)           */
    lagom_cfg* cfgs;             /* host [capacity * ncomm]                                 */
    double* x_us;  double* x_mad_us;    /* host [capacity * ncomm]                          */
    double* Y_us;  double* Y_mad_us;    /* host [capacity]: Y as returned, spread of sum y_i */
    double* Z_us;  double* Z_mad_us;    /* host [capacity]                                  */
    int32_t* iters;              /* host [capacity]: repetitions the call measured          */
} lagom_profile_log;

typedef struct {
    const lagom_comm_desc* launches; int32_t nlaunch;
    const lagom_gemm_desc* comps;    int32_t ncomp;
    void* comm_stream; void* comp_stream;
    int32_t warmup, iters;
    /* A short group is noisy at a fixed repetition count: when min_total_us > 0 and
     * iters * Z < min_total_us after the first measurement, the group is measured again with
     * ceil(min_total_us / Z) repetitions (at most max_iters) and that result is returned.   */
    double  min_total_us;
    int32_t max_iters;
    lagom_profile_log* log;      /* nullable                                                */
} lagom_overlap_ctx;
int lagom_overlap_profile(void* user, const lagom_cfg* cfgs, int ncomm, double* x_us, double* Y_us);

#ifdef __cplusplus
}
#endif
#endif /* LAGOM_H */
