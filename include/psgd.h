/*
 * psgd.h - C ABI of the MI355X (gfx950) PowerSGD step library.
 *
 * The library runs, for every gradient matrix of a model and for W simulated
 * workers resident on one GPU, one step of the rank-r PowerSGD compressor with
 * error feedback (Vogels, Karimireddy, Jaggi, "PowerSGD", arXiv 1905.13727):
 *
 *   Algorithm 2, "Delta_w <- g_w + e_w"            error-feedback add
 *   Algorithm 1, compress+aggregate                P <- M Q ; mean over workers ;
 *                                                  P_hat <- orthogonalize(P) ;
 *                                                  Q <- M^T P_hat ; mean over workers
 *   Algorithm 1, decompress                        Delta' <- P_hat Q^T
 *   Algorithm 2 / eq. (ef-sgd), last line          e_w <- Delta_w - Delta'
 *   Algorithm 1 line 1, Section 3                  tensors with >= 2 dims are seen as
 *                                                  matrices d0 x prod(d1..); vector-shaped
 *                                                  tensors are aggregated uncompressed
 *   Section 3, "warm start"                        the Q written by one step is the
 *                                                  starting Q of the next
 *
 * All data buffers are DEVICE pointers owned by the caller (allocate them with
 * any allocator; the tests use PyTorch).  The library owns only the plan and
 * its small device-side descriptor tables.  No entry point throws or aborts;
 * every failure is a psgd_status.
 *
 * Flat layout (all offsets in elements, reported by psgd_plan_sizes /
 * psgd_plan_offsets):
 *   matrix region   [0, N): the matrices in the order given to
 *                   psgd_plan_create, each row-major n x m, each starting at a
 *                   multiple of 64 elements (padding elements are never read or
 *                   written);
 *   vector region   [N, N+L): the 1-D tensors back to back, same order.
 *   grad   [W][grad_stride]  gradients g_w, dtype grad_dtype, grad_stride >= N+L
 *   err    [W][N]            error memory e_w, float
 *   out    [N+L]             Delta' (matrices) and the worker mean (vectors), out_dtype
 *   p      [p_elems]         per matrix n x r_i row-major, float
 *   q      [q_elems]         per matrix m x r_i row-major, float
 *   r_i = min(rank, n, m) is the effective rank of matrix i.
 */
#ifndef PSGD_H
#define PSGD_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PSGD_API __attribute__((visibility("default")))

typedef struct psgd_plan psgd_plan; /* opaque, library-owned */

typedef enum {
    PSGD_OK = 0,
    PSGD_EINVAL = 1,       /* bad argument (null pointer, non-positive size, ...) */
    PSGD_ENOMEM = 2,       /* host or device allocation failed */
    PSGD_EHIP = 3,         /* a HIP runtime call or kernel launch failed */
    PSGD_EUNSUPPORTED = 4  /* valid request the library does not implement */
} psgd_status;

typedef enum { PSGD_F32 = 0, PSGD_BF16 = 1 } psgd_dtype;

/* One tensor of the model as the compressor sees it (Algorithm 1 line 1).
 * cols >= 2: a rows x cols matrix (conv kernels o,i,k,k are passed as rows=o,
 * cols=i*k*k).  cols == 1: a vector-shaped tensor of `rows` elements, not
 * compressed. */
typedef struct {
    int64_t rows;
    int64_t cols;
} psgd_shape;

typedef struct {
    int64_t n_mat_elems;     /* N, including alignment padding */
    int64_t n_vec_elems;     /* L */
    int64_t grad_stride;     /* elements between consecutive workers in grad */
    int64_t err_stride;      /* elements between consecutive workers in err (= N) */
    int64_t out_elems;       /* N + L */
    int64_t p_elems;         /* sum n_i r_i */
    int64_t q_elems;         /* sum m_i r_i */
    int64_t workspace_bytes; /* scratch the caller must provide to compress/decompress/step */
    int64_t n_matrices;
    int64_t n_vectors;
    int64_t payload_elems;   /* sum of n_i*m_i + L without padding: what SGD would exchange */
    int64_t compressed_elems;/* sum r_i (n_i + m_i) + L: what PowerSGD exchanges (Appendix F tables) */
    int64_t bytes_min;       /* algorithmic HBM bytes per step if every M element moved once:
                                read g, read e, write e' per worker, write Delta' once */
    int64_t bytes_stream;    /* same with the two extra reads of M forced by the two global
                                reductions (after P, after Q) */
    int64_t kept_elems;      /* Random Block / Random K baselines (Appendix G): sum over the matrices of
                                min((n_i + m_i) * rank, n_i * m_i), the length of their packed value / index buffers */
} psgd_sizes;

/* Build a plan.  Host only: makes no HIP call, so it works without a GPU.
 *   shapes[n_tensors]  tensors in model order (see psgd_shape)
 *   rank               r >= 1; clipped per matrix to min(r, n, m)
 *   workers            W >= 1 simulated workers whose P and Q are averaged
 *                      (the two "all reduce mean" lines of Algorithm 1)
 *   grad_dtype         PSGD_F32, or PSGD_BF16 (upcast exactly; error memory,
 *                      P and Q stay float)
 *   out_dtype          dtype of `out`
 * Errors: PSGD_EINVAL for null pointers, n_tensors < 1, rank < 1, workers < 1,
 * a non-positive dimension; PSGD_EUNSUPPORTED for rank > PSGD_MAX_RANK, or,
 * when rank > 8 (the matrix-core kernels), a matrix whose column count is not a
 * multiple of 4 or exceeds 2^20, or with more than 2^22 rows; on the other kernels
 * (rank <= 8, fp32 or bf16 data, any row length) for a matrix with more than about
 * 64 M columns (a strip of 8 rows is addressed with 31-bit byte offsets); PSGD_ENOMEM. */
#define PSGD_MAX_RANK 64
PSGD_API psgd_status psgd_plan_create(const psgd_shape* shapes, int32_t n_tensors, int32_t rank,
                             int32_t workers, psgd_dtype grad_dtype, psgd_dtype out_dtype,
                             psgd_plan** out_plan);

/* Frees the plan and its device tables (if any were uploaded).  NULL is allowed. */
PSGD_API void psgd_plan_destroy(psgd_plan* plan);

/* Sizes of every buffer of the flat layout, and the traffic model. */
PSGD_API psgd_status psgd_plan_sizes(const psgd_plan* plan, psgd_sizes* out_sizes);

/* Placement of tensor `tensor` (index into the shapes array).
 *   flat_off   offset in the flat [N+L] layout (matrix region or vector region)
 *   p_off, q_off, eff_rank   for matrices (offsets are multiples of 4 floats: each
 *                            factor is padded to a 16-byte boundary); -1, -1, 0 for vectors
 * Any output pointer may be NULL. */
PSGD_API psgd_status psgd_plan_offsets(const psgd_plan* plan, int32_t tensor, int64_t* flat_off,
                              int64_t* p_off, int64_t* q_off, int32_t* eff_rank);

/* Tuning knob for experiments; must be called before the plan's first GPU call.
 * Unknown keys and values out of range give PSGD_EINVAL.  Keys:
 *   resident      1 (default): psgd_step keeps M on chip when the model qualifies; 0: always stream;
 *                 2 (TEST ONLY): as 1, but the grid is not checked against what the device holds at once
 *   res_rows      forced strip height of the resident tiling (0: chosen by the planner)
 *   res_trace     1: the resident kernel records phase timestamps (psgd_plan_read_trace)
 *   res_spin      polls before a wait of the resident kernel gives up, 1 .. 2^30 (default 2^21)
 *   res_max_blocks  TEST ONLY: most workgroups the resident tiling may use (0, the default: what the device
 *                 holds at once, found when the plan's tables are uploaded)
 *   k1_rows, k1_nv / k3_rows, k3_nv / k4_rows, k4_nv
 *                 rows per workgroup tile and column vectors per lane of the three sweeps of the
 *                 streaming path (P = M Q; Q = M^T P_hat; decompression); rows 0 (default):
 *                 chosen per matrix by the planner
 *   hr_k1_rows, hr_k1_cols, hr_k3_rows, hr_k4_rows   tile shapes of the matrix-core path
 *                 (hr_k4_rows 0, the default: 64, 256 or 512 rows by rank <= 16, <= 32, <= 64)
 *   xcd_order     order of the tile lists over the accelerator dies: 0 plain, 1 one contiguous range
 *                 of the whole list per die, k >= 2 the same within groups of consecutive matrices
 *                 of at least k tiles, -1 (default) the planner's choice: groups of 4096 / workers
 *                 tiles (128 .. 2048); the whole list for one worker and a set beyond the cache
 *   stream_hints  cache policy of the second and third sweep: -1 (default) by the size of M over all
 *                 workers (non-temporal accesses to M and the error memory above 320 MB), 0 never,
 *                 1 always
 *   gram_fused    orthogonalisation over row blocks: 1 (default) Gram matrices and factorisation in one launch where the
 *                 device holds all row blocks of the launch at once, 0 in two launches, 2 (TEST ONLY) in one
 *                 launch unconditionally: its waits may then time out, see psgd_plan_check
 *   gram_spin     polls before a wait in that launch gives up, 1 .. 2^24 (default 2^18)
 *   ortho_rows    panels of at most this many rows (0 .. 1024) are orthogonalised by one workgroup with modified
 *                 Gram-Schmidt in LDS instead of Cholesky-QR over row blocks; default 0: none
 *   bf16_valu     bf16 gradients / output at rank <= 8: 1 streaming kernels, 0 matrix-core kernels, -1 (default) the
 *                 matrix-core kernels at rank >= 4 when the update matrices of all workers exceed 320 MB and every
 *                 row length is a multiple of 4, the streaming kernels otherwise
 *                 (then every row length must be a multiple of 4, else PSGD_EUNSUPPORTED) */
PSGD_API psgd_status psgd_plan_set_tuning(psgd_plan* plan, const char* key, int64_t value);

/* Algorithm 2 "Delta_w <- g_w + e_w" followed by Algorithm 1 compress+aggregate.
 *   grad (device, const)  g_w                          [W][grad_stride] grad_dtype
 *   err  (device, in/out) in: e_w ; out: M_w = g_w+e_w [W][N] float
 *   q    (device, in/out) in: previous Q (warm start; iid N(0,1) before the
 *                         first step) ; out: Q = mean_w M_w^T P_hat
 *   p    (device, out)    P_hat (orthonormal columns)
 *   workspace (device)    workspace_bytes of scratch, 256-byte aligned, contents
 *                         ignored on entry and undefined on exit
 *   hip_stream            a hipStream_t (NULL = the default stream)
 * Everything is enqueued on hip_stream; the call does not synchronise, allocate
 * or read back, except that a plan's first GPU call allocates and uploads its
 * descriptor tables (one hipMalloc, one synchronous copy).
 * Vector-shaped tensors are not touched by this call. */
PSGD_API psgd_status psgd_compress(psgd_plan* plan, const void* grad, float* err, float* q, float* p,
                          void* workspace, void* hip_stream);

/* Algorithm 1 decompress and the error-memory update of Algorithm 2.
 *   p, q (device, const)  the pair produced by psgd_compress
 *   err  (device, in/out) in: M_w as left by psgd_compress ; out: e_w = M_w - P_hat Q^T
 *   grad (device, const)  read only for the vector-shaped tensors
 *   out  (device, out)    [N+L] out_dtype: Delta' = P_hat Q^T for matrices, the
 *                         mean over workers of g_w for vectors
 * Same stream / workspace rules as psgd_compress. */
PSGD_API psgd_status psgd_decompress(psgd_plan* plan, const float* p, const float* q, float* err,
                            const void* grad, void* out, void* workspace, void* hip_stream);

/* One whole step: the same quantities as psgd_compress followed by
 * psgd_decompress.  For W = 1, rank <= 4 and a model whose matrices fit the
 * register files of the chip (every matrix at most 512 rows, about 16 M
 * elements in total) the plan runs in RESIDENT mode: one kernel keeps
 * M = g + e on chip for the whole step, so each element is read and written
 * once.  Its sums run in another (fixed) order than the split calls, so the
 * two agree to rounding, not bit for bit; each is reproducible from run to
 * run.  Otherwise psgd_step is exactly the two calls in sequence.  Resident
 * mode, and the one-launch orthogonalisation over row blocks (tuning key
 * gram_fused), keep hand-over words in plan-owned device memory: do not run
 * two calls of the same plan concurrently on different streams.  Both are
 * kernels whose workgroups wait for each other inside one ordinary launch:
 * THEY NEED THE GPU TO THEMSELVES for the length of the kernel (no other
 * stream or process holding compute units).  Their waits are bounded; if one
 * gives up (the GPU was shared), the kernel still ends, that step's outputs -
 * err and q included, which are updated in place - are invalid, and
 * psgd_plan_check (below) reports it and moves the plan to the kernels that
 * need no co-residency.  A caller that may share the GPU checks every step,
 * or sets the tuning keys resident = 0 and gram_fused = 0.
 * The plan's first GPU call (any entry point) uploads its tables (one device
 * allocation and copy).  After that this call, psgd_compress and psgd_decompress
 * only launch kernels on hip_stream: no allocation, no memset, no host
 * synchronisation, so they may be captured into a HIP graph and replayed. */
PSGD_API psgd_status psgd_step(psgd_plan* plan, const void* grad, float* err, float* q, float* p,
                      void* out, void* workspace, void* hip_stream);

/* One more subspace iteration of Algorithm 1 on the update already held in `err`
 * (M_w = g_w + e_w as left there by psgd_compress): P = mean_w M_w Q, orthogonalise,
 * Q = mean_w M_w^T P_hat.  Nothing is added to err and err is not written.
 * psgd_compress followed by k-1 calls of psgd_iterate, then psgd_decompress, is the
 * compressor with k iterations per step of Appendix G.7 ("best approximation" as k
 * grows; started from a fresh random Q it is the variant without warm start of
 * Table 2).  Always the streaming or matrix-core kernels; psgd_step_iterations is the
 * one-call form that can stay on chip.
 *   err (device, const in effect)  M_w  [W][N] float
 *   q   (device, in/out), p (device, out), workspace, hip_stream: as psgd_compress */
PSGD_API psgd_status psgd_iterate(psgd_plan* plan, float* err, float* q, float* p, void* workspace,
                         void* hip_stream);

/* psgd_step for callers that cannot allocate device memory (code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc): the workspace is not an argument but an array the library itself holds on
 * every GPU it is loaded on (PSGD_STATIC_WORKSPACE_BYTES, part of the code object, kept until the process
 * ends).  The call allocates and frees nothing and otherwise behaves exactly like psgd_step with that workspace.
 * Conditions: the plan's tables are on the device already (psgd_plan_check, or any earlier GPU call on the plan,
 * puts them there; that upload is the one allocation a plan makes) - else PSGD_EINVAL; the plan's
 * workspace_bytes fit - else PSGD_EUNSUPPORTED (the ResNet18-shaped set up to 16 workers and the LSTM-shaped set
 * fit, the 24-layer transformer-shaped set does not); the current device is the plan's.  All plans on a GPU share
 * the one array and it keeps whatever the last call left there (the kernels read nothing of it that they have
 * not written in the same call): calls that overlap in time on one GPU, from any plan or stream, race. */
#define PSGD_STATIC_WORKSPACE_BYTES (32u << 20)
PSGD_API psgd_status psgd_step_static(psgd_plan* plan, const void* grad, float* err, float* q, float* p, void* out,
                                      void* hip_stream);

/* One whole step with `iterations` subspace iterations (Appendix G.7, "best-approximation PowerSGD"; Table 2):
 * the same quantities as psgd_compress, iterations - 1 calls of psgd_iterate, psgd_decompress.  iterations = 1 is
 * psgd_step.  A plan in resident mode (see psgd_step) keeps M on chip through all the iterations: one kernel, each
 * element of g, e read once and of e', Delta' written once whatever the count; otherwise the calls above in
 * sequence.  Start it from a fresh random Q for the variants without warm start.
 * Errors: PSGD_EINVAL also for iterations outside 1 .. 64. */
PSGD_API psgd_status psgd_step_iterations(psgd_plan* plan, const void* grad, float* err, float* q, float* p,
                                          void* out, void* workspace, void* hip_stream, int32_t iterations);

/* The step fused with the last two lines of Algorithm 2 (error-feedback SGD with
 * momentum): m <- lambda m + Delta' ; x <- x - gamma (Delta' + m).  Delta' is not
 * stored: the decompression pass reads and writes the momentum and parameter
 * buffers instead (8 bytes per element less traffic than psgd_step followed by a
 * separate update).  Vector-shaped tensors take Delta' = mean over workers of g_w.
 *   mom   (device, in/out) m [N+L] float, laid out like `out` of psgd_decompress
 *   param (device, in/out) x [N+L] float, same layout
 *   lr, momentum           gamma and lambda
 * All other arguments, the resident / streaming choice and the stream rules are
 * those of psgd_step / psgd_decompress; a plan's out_dtype is not used here.
 * Errors: PSGD_EINVAL for null pointers or NaN step sizes. */
PSGD_API psgd_status psgd_step_update(psgd_plan* plan, const void* grad, float* err, float* q, float* p,
                             float* mom, float* param, float lr, float momentum, void* workspace,
                             void* hip_stream);
PSGD_API psgd_status psgd_decompress_update(psgd_plan* plan, const float* p, const float* q, float* err,
                                   const void* grad, float* mom, float* param, float lr, float momentum,
                                   void* workspace, void* hip_stream);

/* ---- The two linear baselines of Appendix G that share the error-feedback loop of Algorithm 2 -------------
 *
 * "Random Block compression" and "Random K compression": the update M_w = g_w + e_w of a matrix is seen as a
 * vector of length n m; every worker keeps the same b = (n + m) rank entries of it (PowerSGD's budget; at most
 * n m): a contiguous block M(s : s+b) from a sampled start s, or a sampled set I of b distinct positions.  The
 * kept values are averaged over the workers, Delta' is zero everywhere else, and e_w <- M_w - Delta'.  The
 * library draws nothing: the samples are arguments (the appendix samples them on the CPU with the same seed on
 * every worker).  A block that would run past the end of the vector stops there.  Vector-shaped tensors are
 * averaged uncompressed, as in psgd_step.  fp32 plans only (else PSGD_EUNSUPPORTED); the plan's workspace and
 * its P / Q buffers are not used.
 *
 *   grad   (device, const)   as psgd_step
 *   err    (device, in/out)  in: e_w ; out: e_w <- g_w + e_w - Delta'
 *   starts (device, const)   Random Block: int64 [n_tensors], starts[t] = s of tensor t in [0, n m) (values
 *                            outside are clamped into the range; entries of vector tensors are ignored)
 *   indices (device, const)  Random K: int64 [kept_elems], the positions of matrix i at kept_off_i .. + kept_i
 *                            (psgd_plan_kept), each in [0, n m) and distinct within a matrix; a position outside
 *                            the range is skipped (its value slot is zero); repeated positions race
 *   vals   (device, out)     [kept_elems] float: the averaged kept values in block / index order (what the
 *                            workers would all-reduce); zero past the end of a block cut short
 *   out    (device, out)     [N+L] float: Delta'
 * Enqueued on hip_stream; no allocation (after the plan's first GPU call), no synchronisation. */
PSGD_API psgd_status psgd_random_block_step(psgd_plan* plan, const void* grad, float* err, const int64_t* starts,
                                            float* vals, void* out, void* hip_stream);
PSGD_API psgd_status psgd_random_k_step(psgd_plan* plan, const void* grad, float* err, const int64_t* indices,
                                        float* vals, void* out, void* hip_stream);
/* Placement of tensor `tensor` in the packed value / index buffers of the baselines: offset and count
 * (-1 and 0 for vector tensors).  Either output may be NULL. */
PSGD_API psgd_status psgd_plan_kept(const psgd_plan* plan, int32_t tensor, int64_t* kept_off, int64_t* kept);

/* Per-kernel timing for benchmarks.  With profiling enabled, psgd_compress and
 * psgd_decompress record HIP events on the caller's stream around each of their
 * kernels, and psgd_decompress (hence psgd_step) WAITS for the stream at its
 * end to accumulate the elapsed times: use it for measurement runs only.
 * psgd_plan_kernel_times copies the accumulated milliseconds per kernel (array
 * of PSGD_N_KERNELS doubles, order given by psgd_kernel_name) and the number of
 * accumulated steps, then clears the accumulators.  A plan in resident mode
 * (see psgd_step) runs one kernel per step, index PSGD_KERNEL_RESIDENT; the
 * baseline steps (psgd_random_block_step, psgd_random_k_step) fill the last two
 * entries and wait for the stream at their end like psgd_decompress. */
#define PSGD_N_KERNELS 8
#define PSGD_KERNEL_RESIDENT 5
#define PSGD_KERNEL_EF_ADD_ZERO 6   /* the two launches of the Appendix G baselines */
#define PSGD_KERNEL_KEPT_ENTRIES 7
PSGD_API psgd_status psgd_plan_set_profiling(psgd_plan* plan, int32_t enable);
PSGD_API psgd_status psgd_plan_kernel_times(psgd_plan* plan, double* ms_sum, int64_t* steps);
/* Name of kernel `index` in [0, PSGD_N_KERNELS) as it appears in a profiler's
 * kernel trace (prefix of the symbol); NULL if out of range. */
PSGD_API const char* psgd_kernel_name(int32_t index);

/* A plan that has made no GPU call yet: uploads its tables (the plan's one device allocation) and returns.
 * Otherwise waits for hip_stream, then returns PSGD_EHIP if a kernel of this plan whose
 * workgroups wait for each other (resident mode; the one-launch orthogonalisation
 * over row blocks) gave up waiting since the last check, PSGD_OK otherwise.
 * After PSGD_EHIP the outputs of the steps since the last check are invalid
 * (restore err and q from a copy, or restart them), the plan's hand-over words
 * are reset, and the mode that failed is switched off for this plan: later
 * steps run on the streaming kernels / the two-launch factorisation.
 * is_resident (may be NULL) receives 1 if psgd_step runs in resident mode (a
 * plan that has made no GPU call yet answers with the planner's provisional
 * choice; the device's capacity is known once its tables are uploaded). */
PSGD_API psgd_status psgd_plan_check(psgd_plan* plan, void* hip_stream, int32_t* is_resident);

/* Diagnostic.  After psgd_plan_set_tuning(plan, "res_trace", 1), every resident
 * step records 16 values per wavefront: device timestamps (100 MHz clock) of start,
 * partial P posted, reducer work done, P_hat received, partial Q posted, Q received,
 * end; 7..11 are written by a wavefront that orthogonalises (own partial posted,
 * strip sum posted, mean P received, Gram-Schmidt done, P_hat posted); 12..15 name
 * the tile: matrix, column chunk (upper half: the hardware id register of the
 * wavefront), first row (upper half: accelerator die), partial-Q slot or -1.
 * Synchronises the device and copies at most
 * `capacity` values of the last step to `out` (host); *n_written = count. */
PSGD_API psgd_status psgd_plan_read_trace(psgd_plan* plan, uint64_t* out, int64_t capacity, int64_t* n_written);

/* Which kernels psgd_step runs for this plan (Algorithm 1 and the loop of Algorithm 2 are the same on all of
 * them; the choice is the planner's, from rank, data types, shapes and set size, see psgd_plan_set_tuning):
 * *path = PSGD_PATH_STREAMING, PSGD_PATH_RESIDENT or PSGD_PATH_MATRIX_CORES.  For a plan that has made no GPU call
 * yet "resident" is the planner's provisional choice (see psgd_plan_check).  PSGD_EINVAL for NULL arguments. */
#define PSGD_PATH_STREAMING 0
#define PSGD_PATH_RESIDENT 1
#define PSGD_PATH_MATRIX_CORES 2
PSGD_API psgd_status psgd_plan_path(const psgd_plan* plan, int32_t* path);

/* Static, never NULL. */
PSGD_API const char* psgd_status_string(psgd_status status);

/* Text of the last HIP error seen by this plan ("" if none).  The pointer is
 * valid until the next failing call on the plan or its destruction. */
PSGD_API const char* psgd_plan_last_error(const psgd_plan* plan);

#ifdef __cplusplus
}
#endif
#endif /* PSGD_H */
