/*
 * dad.h - C ABI of libdad: the single-GPU hot path of distributed
 * auto-differentiation (dAD, arXiv 2102.09631) for AMD MI355X (gfx950).
 *
 * One linear layer with input width h_in = h_{i-1} and output width
 * h_out = h_i contributes a factor pair, one row per sample or token
 * (Section 3.3; Algorithm 2, INPUT):
 *
 *     A     N x h_in    input activations  A_{i-1}
 *     Delta N x h_out   back-propagated errors  Delta_i
 *
 * whose product M = A^T Delta (h_in x h_out) is the layer's weight gradient
 * (Section 3.1, Eq. 4).  The library stacks the pairs of S sites, compresses
 * the implicit product to rank r without forming it, and rebuilds the gradient
 * from either form.
 *
 * Conventions for every call
 *   - All matrices are dense, row-major, with no padding between rows.
 *   - Every pointer named "device" is a HIP device pointer on the current
 *     device and is owned by the caller; the library allocates and frees no
 *     device memory.  Scratch space comes in through `workspace` (size from
 *     the matching *_workspace_bytes query).  Nothing computed is kept from
 *     one call to the next; the only process-wide state is per device: a
 *     "set-up done" flag (see dad_init), seven side streams and their events
 *     for dad_compress_rank_grouped, the static scratch array of
 *     dad_compress_rank_noalloc, and, when switched on, the timing records of
 *     dad_profile_*; all are safe to use from several host threads.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls enqueue work and return; they do not synchronise.
 *   - Argument errors are detected on the host and returned before anything
 *     is enqueued (so they can be exercised without a GPU).  A numerical
 *     breakdown found on the device is latched in the workspace and reported
 *     by dad_poll_numeric_status.
 *   - Device pointers must be 16-byte aligned.  Any 1 <= N <= DAD_MAX_ROWS and
 *     1 <= h_in, h_out <= DAD_MAX_WIDTH is accepted (DAD_ERR_SHAPE beyond: the
 *     launch grids do not hold more); shapes whose widths are multiples of the
 *     MFMA tile take the fast kernels, others a slower guarded path with
 *     identical results up to rounding order.
 *   - Overlapping calls that share a workspace race; use one workspace per
 *     stream.
 *   - Every call but dad_poll_numeric_status (which copies one word to the host
 *     and waits for it) and dad_init may be recorded into a HIP graph: nothing
 *     is allocated, copied or cleared by memset.  The first call on a device
 *     sets kernel attributes (several kernels ask for more than 64 KB of LDS):
 *     call dad_init() on that device before the first capture, or make any
 *     first call outside a capture.
 */
#ifndef DAD_H
#define DAD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Element type of the factor matrices.  Accumulation is always fp32. */
typedef enum { DAD_F32 = 0, DAD_BF16 = 1 } dad_dtype;

typedef enum {
    DAD_OK = 0,
    DAD_ERR_NULL = 1,      /* a required pointer is NULL                              */
    DAD_ERR_SHAPE = 2,     /* a size is < 1, r > DAD_MAX_RANK or r > min(N,h_in,h_out) */
    DAD_ERR_ALIGN = 3,     /* a device pointer is not 16-byte aligned                 */
    DAD_ERR_WORKSPACE = 4, /* ws_bytes is smaller than the matching query returns     */
    DAD_ERR_DTYPE = 5,     /* unknown dad_dtype                                       */
    DAD_ERR_NUMERIC = 6,   /* orthonormalisation met a non-positive or NaN pivot      */
    DAD_ERR_HIP = 7        /* a HIP runtime call failed (launch, copy, sync)          */
} dad_status;

#define DAD_MAX_RANK 64    /* largest r accepted by dad_compress_rank */
#define DAD_GRAM_MAX_ROWS 1024 /* largest N accepted by dad_compress_rank_gram */
#define DAD_MAX_SITES 4096 /* largest S accepted by dad_stack_factors */
#define DAD_MAX_GROUP 4096 /* largest n accepted by the *_grouped calls */
#define DAD_MAX_ROWS ((int64_t)1 << 36)  /* largest N (or K) accepted */
#define DAD_MAX_WIDTH ((int64_t)1 << 21) /* largest h_in, h_out accepted */

/* Human-readable name of a status code; static storage, never NULL. */
const char* dad_status_string(dad_status s);

/*
 * One-time set-up of the current device (kernel attributes, address of the static scratch).  Optional: every entry point does the
 * same on its first call on a device, guarded by a mutex, and after that only reads a flag.  Call
 * it explicitly, once per device with that device current, when the first real call would fall
 * inside a HIP graph capture.  Returns DAD_OK or DAD_ERR_HIP.
 */
dad_status dad_init(void);

/*
 * dad_stack_factors - Section 3.2 (concatenate the sites' factors along the
 * batch dimension) and Algorithm 1 (the aggregator's vertcat of the rank-r
 * pairs): A_out = [A_1; ...; A_S], D_out = [Delta_1; ...; Delta_S].
 *
 *   S         number of sites, 1..DAD_MAX_SITES
 *   A_sites   HOST array of S device pointers; A_sites[s] is rows[s] x h_in
 *   D_sites   HOST array of S device pointers; D_sites[s] is rows[s] x h_out
 *   rows      HOST array of S row counts, each >= 0 (an empty site is skipped)
 *   dt        element type of all inputs and outputs (a bit-exact copy)
 *   A_out     device, (sum rows) x h_in ;  D_out  device, (sum rows) x h_out
 * Site s lands at row offset rows[0]+...+rows[s-1].  Outputs must not overlap
 * inputs.  Returns DAD_ERR_SHAPE if S, h_in, h_out < 1 or any rows[s] < 0.
 */
dad_status dad_stack_factors(int S, const void* const* A_sites, const void* const* D_sites,
                             const int64_t* rows, int64_t h_in, int64_t h_out, dad_dtype dt,
                             void* A_out, void* D_out, void* stream);

/* Bytes of device workspace dad_compress_rank needs for these sizes (0 on invalid sizes). */
size_t dad_compress_workspace_bytes(int64_t N, int64_t h_in, int64_t h_out, int r, dad_dtype dt);

/*
 * dad_compress_rank - Algorithm 2 (structured power iteration, Section 3.3.1,
 * Eq. 5-6) applied to all r start vectors at once.  n_iter times the block
 * G (h_out x r) is replaced by an orthonormal basis of
 *     M^T M G = Delta^T ( A ( A^T ( Delta G ) ) ),
 * evaluated right to left so that neither M nor A A^T is formed; the
 * orthonormalisation (Cholesky QR: one round for the intermediate iterates,
 * of which only the span is used; for the last one a second round unless the
 * first factor shows cond(Y) <= 4 r through the upper bound ||R||_F ||R^-1||_F,
 * decided on the device) stands in for
 * the peeling of Eq. 7.  Then the left factor P = A^T (Delta G) is formed with the singular values left
 * inside it (footnote to Section 3.3.1), so that  M ~ P G^T = M G G^T.
 *
 *   A, D      device, N x h_in and N x h_out, element type dt
 *   r         target rank, 1 <= r <= min(N, h_in, h_out, DAD_MAX_RANK)
 *   n_iter    number of applications of M^T M, >= 1
 *   G0        device, r x h_out fp32: row j is the start vector g_0^j
 *   Pt        device out, r x h_in  fp32: row j is the left vector p_j = M g_j
 *   Gt        device out, r x h_out fp32: rows orthonormal
 *   workspace device, ws_bytes >= dad_compress_workspace_bytes(...)
 * Outputs have the factor layout (one row per component), so S such pairs can
 * be stacked and compressed again (Algorithm 1).  For dt = DAD_BF16 on shapes
 * the MFMA kernels serve (N >= 256, widths multiples of 128, r a multiple of
 * 8) the two N x r intermediates travel as bf16 between contractions: Delta G
 * rounded once, A U as two bf16 terms (value and rounding remainder, 16
 * significand bits: activations with a non-zero mean make one rounding of it
 * too coarse); with N a multiple of 256 the h x r panels enter the next
 * contraction rounded to bf16 as well.  On other shapes and for fp32 factors
 * the intermediates are fp32.  The panels themselves, the outputs and
 * everything r x r stay fp32 (Gram matrix and r x r factorisation in fp64).
 * If the iterate loses rank (r > rank(M)) the outputs are unspecified and
 * DAD_ERR_NUMERIC is latched for dad_poll_numeric_status.
 */
dad_status dad_compress_rank(const void* A, const void* D, int64_t N, int64_t h_in, int64_t h_out,
                             dad_dtype dt, int r, int n_iter, const float* G0, float* Pt, float* Gt,
                             void* workspace, size_t ws_bytes, void* stream);

/*
 * dad_compress_rank_noalloc - dad_compress_rank for callers that cannot allocate device memory or
 * carry a workspace: code recorded into a HIP graph whose owner has no buffer to hand over, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, kernels and results (bit for bit)
 * as dad_compress_rank, but the scratch space is a static array of DAD_STATIC_SCRATCH_BYTES that the
 * library's code object holds on every device it is loaded on until the process ends; the call
 * allocates and frees nothing.
 *   numeric_flag  device out, one int (4-byte aligned), or NULL: receives 0, or 1 when the
 *                 orthonormalisation broke down (what dad_poll_numeric_status reports for the
 *                 workspace variant); the pointer may also be handed to dad_poll_numeric_status
 * Sizes whose dad_compress_workspace_bytes exceeds DAD_STATIC_SCRATCH_BYTES are rejected with
 * DAD_ERR_WORKSPACE before anything is enqueued (every benchmark shape up to N = 65536 rows at
 * r = 32 and every per-site reduction fits; N = 262144 at r = 64 does not).  All calls on one
 * device share that device's array: calls that overlap in time on one device (two streams, two
 * threads) race; calls on one stream, or ordered by events, do not.  The first call on a device
 * resolves the array's address (see dad_init for calls under capture).
 */
#define DAD_STATIC_SCRATCH_BYTES (32u << 20)
dad_status dad_compress_rank_noalloc(const void* A, const void* D, int64_t N, int64_t h_in, int64_t h_out,
                                     dad_dtype dt, int r, int n_iter, const float* G0, float* Pt, float* Gt,
                                     int* numeric_flag, void* stream);

/*
 * dad_compress_rank_grouped - dad_compress_rank for n layers in one call (Algorithm 1 reduces every
 * layer's pair in the same step).  Layer i gets exactly the launches of dad_compress_rank on its own
 * region of the workspace, so its Pt, Gt are bit-identical to a single call's; up to `lanes` layers
 * are in flight at once (layer i on lane i mod lanes), so that the short, latency-bound launches of
 * one layer's orthonormalisation run while another layer streams its factors.  A run of consecutive
 * stacked layers of equal N that the bf16 direct-to-LDS kernels serve (N a multiple of 256, widths
 * multiples of 128, r in {16, 32, 64}) is executed as a batch of up to 32: every launch does the
 * same step of all its layers, so the run costs the launches of one layer.  Batched are layers of
 * equal widths with at most 256 MiB of factors each (typically the S site reductions of one layer
 * in Algorithm 1, each site's block passed as a layer), and layers of unequal widths, all multiples
 * of 256, with at most 64 MiB each (the layers of a small block).  A batch takes one lane and as
 * many workspace regions as it has layers (the size query accounts for that); its results are still
 * bit-identical to single calls.
 *   descs     HOST array of n layers, 1 <= n <= DAD_MAX_GROUP; every pointer is a device pointer with
 *             the meaning and alignment of dad_compress_rank's.  A layer with S > 0 gives its factors
 *             as the S site blocks of dad_stack_factors (A_sites, D_sites, rows: HOST arrays read
 *             during the call; A, D and N are then ignored, N = sum of rows) and is reduced as
 *             dad_compress_rank_sites reduces it
 *   dt, r, n_iter   common to all layers
 *   lanes     1 .. DAD_MAX_LANES; lane 0 is `stream` itself, the others are streams of default
 *             priority that the library keeps per device; they start after the work already enqueued
 *             on `stream`, and `stream` waits for them before the call's successors (fork and join by
 *             events, so the call can be recorded into a HIP graph after dad_init)
 *   workspace device, ws_bytes >= dad_compress_grouped_workspace_bytes(n, descs, dt, r, lanes)
 * dad_poll_numeric_status(workspace, stream) reports DAD_ERR_NUMERIC if ANY layer of the call broke
 * down.  Calls on one device are serialised on the host by a mutex while they enqueue.
 */
typedef struct {
    const void* A;   /* N x h_in  */
    const void* D;   /* N x h_out */
    const float* G0; /* r x h_out */
    float* Pt;       /* r x h_in,  out */
    float* Gt;       /* r x h_out, out */
    int64_t N, h_in, h_out;
    int S;                       /* 0: stacked factors A, D with N rows; > 0: S site blocks */
    const void* const* A_sites;  /* S device pointers, rows[s] x h_in  */
    const void* const* D_sites;  /* S device pointers, rows[s] x h_out */
    const int64_t* rows;         /* S row counts */
} dad_compress_desc;
#define DAD_MAX_LANES 8
size_t dad_compress_grouped_workspace_bytes(int n, const dad_compress_desc* descs, dad_dtype dt, int r, int lanes);
dad_status dad_compress_rank_grouped(int n, const dad_compress_desc* descs, dad_dtype dt, int r, int n_iter, int lanes,
                                     void* workspace, size_t ws_bytes, void* stream);

/*
 * dad_compress_rank_sites, dad_reconstruct_grad_sites - dad_compress_rank and the full rebuild
 * G = A^T D (Eq. 4) on factors that are given as the S site blocks of dad_stack_factors instead of
 * the stacked matrices (Section 3.2: stacking only orders the rows; Algorithm 1's vertcat).  The
 * results are bit-identical to dad_stack_factors followed by dad_compress_rank /
 * dad_reconstruct_grad, because the same kernels do the same work in the same order and only
 * fetch their rows from the blocks.
 *   S, A_sites, D_sites, rows   as for dad_stack_factors (HOST arrays of device pointers and row
 *             counts, read during the call; empty sites allowed); N = sum of rows must satisfy the
 *             stacked call's limits
 *   the other arguments as in dad_compress_rank / dad_reconstruct_grad (L = A, R = D, K = N)
 *   workspace ws_bytes >= dad_compress_sites_workspace_bytes / dad_reconstruct_sites_workspace_bytes
 * The blocks are read in place, without any copy, when the stacked call would run its
 * direct-to-LDS bf16 kernels (bf16, N a multiple of 256, widths multiples of 128, for the
 * reduction r in {16, 32, 64}), there are at most 32 non-empty sites and every site's row count is a
 * multiple of 256.  Otherwise the call stacks the blocks into its own workspace first (the size
 * query accounts for that) and proceeds as the stacked call.  dad_poll_numeric_status(workspace,
 * stream) works as for dad_compress_rank.  Errors as for the stacked calls and dad_stack_factors.
 */
size_t dad_compress_sites_workspace_bytes(int S, const int64_t* rows, int64_t h_in, int64_t h_out, int r, dad_dtype dt);
dad_status dad_compress_rank_sites(int S, const void* const* A_sites, const void* const* D_sites, const int64_t* rows,
                                   int64_t h_in, int64_t h_out, dad_dtype dt, int r, int n_iter, const float* G0,
                                   float* Pt, float* Gt, void* workspace, size_t ws_bytes, void* stream);
size_t dad_reconstruct_sites_workspace_bytes(int S, const int64_t* rows, int64_t h_in, int64_t h_out, dad_dtype dt);
dad_status dad_reconstruct_grad_sites(int S, const void* const* A_sites, const void* const* D_sites, const int64_t* rows,
                                      int64_t h_in, int64_t h_out, dad_dtype dt, float* G, void* workspace,
                                      size_t ws_bytes, void* stream);

/* Bytes of device workspace dad_compress_rank_gram needs (0 on invalid sizes, N > DAD_GRAM_MAX_ROWS included). */
size_t dad_compress_gram_workspace_bytes(int64_t N, int64_t h_in, int64_t h_out, int r, dad_dtype dt);

/*
 * dad_compress_rank_gram - the few-rows form of dad_compress_rank (Algorithm 2 with its
 * precomputation C = A A^T, Eq. 6; the regime N << h of Section 3.3.1).  C = A A^T, E = D D^T and
 * H0 = D G0^T are formed once in fp64; with every iterate written as G_k = D^T T_k the block power
 * iteration and its Cholesky orthonormalisation (one round per iterate; a second one for the returned
 * iterate unless the first factor shows cond(Y) <= 1e3 r through the bound ||R||_F ||R^-1||_F) run on
 * N x N and N x r fp64 matrices:
 *     Z_1 = C H0,  Z_k = C (E T_{k-1}),  Z_k^T E Z_k = R^T R,  T_k = Z_k R^-1,
 * and the pair is Gt = T_n^T D, Pt = (E T_n)^T A.  Each factor is read twice instead of
 * 2 n_iter + 1 times and the call is 9 launches for n_iter = 2.
 *
 * Arguments, outputs and errors are those of dad_compress_rank, with 1 <= N <= DAD_GRAM_MAX_ROWS
 * (else DAD_ERR_SHAPE) and workspace >= dad_compress_gram_workspace_bytes(...).  Pt^T Gt is the same
 * matrix as dad_compress_rank's up to rounding (the span of the iterate is the same); Pt and Gt
 * themselves agree with it whenever the iterate is well conditioned (both come from Cholesky
 * factors with a positive diagonal).  Squared conditioning is the price of the Gram form: the
 * orthonormalisation holds to about 1e-16 cond(Y)^2 per round, and a non-positive pivot latches
 * DAD_ERR_NUMERIC for dad_poll_numeric_status.  It is the faster call for N <= 256 (0.6 to 0.75 of
 * dad_compress_rank's time) and even with it at N = 512; with more rows the N^2 (h_in + h_out) flops
 * of the two Gram matrices cost more than the thin passes they replace.
 */
dad_status dad_compress_rank_gram(const void* A, const void* D, int64_t N, int64_t h_in, int64_t h_out, dad_dtype dt,
                                  int r, int n_iter, const float* G0, float* Pt, float* Gt, void* workspace,
                                  size_t ws_bytes, void* stream);

/* Bytes of device workspace dad_compress_rank_sequential needs (0 on invalid sizes). */
size_t dad_compress_sequential_workspace_bytes(int64_t N, int64_t h_in, int64_t h_out, dad_dtype dt);

/*
 * dad_compress_rank_sequential - Algorithm 2 as printed (Section 3.3.1, Eq. 5-7): one singular
 * pair at a time, with peeling.  Component j starts from g = G0[j] / ||G0[j]|| and applies
 *     g <- normalise( M^T M g - sum_{i<j} sigma_i^2 g_i (g_i^T g) )
 * exactly n_iter times (the deflation of M^T M by the pairs already found stands in for the printed
 * Q (G^T g), whose vectors have two different lengths; for the threshold theta of the listing see
 * dad_compress_rank_adaptive).  Then v = Delta g, sigma_j = ||A^T v||, q_j = A^T v / sigma_j.
 *
 *   A, D, N, h_in, h_out, dt, r, n_iter, G0   as for dad_compress_rank
 *   Qt        device out, r x h_in fp32: row j = q_j, unit length
 *   sGt       device out, r x h_out fp32: row j = sigma_j g_j, so that M ~ Qt^T sGt and the pair can
 *             be passed to dad_reconstruct_grad or stacked like the pair of dad_compress_rank
 *   sigma     device out, r fp32 singular-value estimates, or NULL
 *   workspace device, ws_bytes >= dad_compress_sequential_workspace_bytes(...)
 * Every thin pass over a factor costs the same for one vector as for r of them, so this call costs
 * about r times dad_compress_rank; it exists as the paper's own recurrence.  A vanishing iterate
 * (rank exhausted) latches DAD_ERR_NUMERIC for dad_poll_numeric_status.
 */
dad_status dad_compress_rank_sequential(const void* A, const void* D, int64_t N, int64_t h_in, int64_t h_out,
                                        dad_dtype dt, int r, int n_iter, const float* G0, float* Qt, float* sGt,
                                        float* sigma, void* workspace, size_t ws_bytes, void* stream);

/*
 * dad_compress_rank_adaptive - dad_compress_rank_sequential with the stop tests of Algorithm 2 and the
 * effective rank of Section 3.3.1 (last paragraph), under this reading of the ambiguous listing:
 *   - component j applies M^T M at most max_iter times and stops once two successive unit iterates
 *     differ by at most theta (sign aligned);
 *   - component j > 0 is dropped, and no further component is computed, when sigma_j < theta sigma_0
 *     or when an application leaves nothing to normalise (||y|| < (theta sigma_0)^2 after the found
 *     vectors are projected out);
 *   - the peel of Eq. 7 is applied as a projection (the start vector and every iterate are kept
 *     orthogonal to the vectors already found).  For exact singular pairs that is the printed
 *     subtraction; for pairs converged only to theta the subtraction leaves a first-order residual
 *     whose "component" has ||M g|| of the order of sigma_0, and no threshold on sigma_j / sigma_0
 *     could detect an exhausted gradient.
 * Everything is decided on the device: the launch sequence is that of r components x max_iter
 * applications, and the launches of skipped work return at once on a flag in the workspace, so the
 * call can be recorded into a HIP graph.
 *   A .. G0, Qt, sGt, sigma, workspace   as for dad_compress_rank_sequential (same workspace size);
 *             rows of Qt, sGt and entries of sigma beyond the effective rank are zero
 *   max_iter  >= 1;  theta  0 <= theta < 1 (the paper uses 1e-3)
 *   effective_rank  device out, one int: number of components kept (1 .. r)
 *   iterations      device out, r ints, or NULL: applications spent on each component
 * Near the thresholds fp32 arithmetic may decide differently from exact arithmetic by one
 * application or one component; both outcomes are valid results of the method.
 */
dad_status dad_compress_rank_adaptive(const void* A, const void* D, int64_t N, int64_t h_in, int64_t h_out,
                                      dad_dtype dt, int r, int max_iter, float theta, const float* G0, float* Qt,
                                      float* sGt, float* sigma, int* effective_rank, int* iterations,
                                      void* workspace, size_t ws_bytes, void* stream);

/* Bytes of device workspace dad_reconstruct_grad needs (may be 0 for small K; 0 on invalid sizes). */
size_t dad_reconstruct_workspace_bytes(int64_t K, int64_t h_in, int64_t h_out, dad_dtype dt);

/*
 * dad_reconstruct_grad - Section 3.1, Eq. 4:  G = L^T R,  G[p][q] = sum_k L[k][p] R[k][q].
 *   full gradient  : L = A (N x h_in), R = Delta (N x h_out), K = N, dt = factor type
 *   rank-r gradient: L = Pt (r x h_in), R = Gt (r x h_out), K = r, dt = DAD_F32
 *                    (Algorithm 1, the sites' local rebuild)
 *   G         device out, h_in x h_out fp32, overwritten
 *   workspace device, may be NULL when the query returns 0
 */
dad_status dad_reconstruct_grad(const void* L, const void* R, int64_t K, int64_t h_in, int64_t h_out,
                                dad_dtype dt, float* G, void* workspace, size_t ws_bytes, void* stream);

/*
 * dad_reconstruct_grad_grouped - dad_reconstruct_grad for n layers in one call (Algorithm 1 rebuilds
 * every layer's gradient from its broadcast pair in the same step): G_i = L_i^T R_i.
 *   descs     HOST array of n jobs, 1 <= n <= DAD_MAX_GROUP; pointers are device pointers with the
 *             meaning and alignment of dad_reconstruct_grad's
 *   dt        element type of every L_i, R_i
 *   workspace device, ws_bytes >= dad_reconstruct_grouped_workspace_bytes(n, descs, dt) (may be NULL
 *             when that is 0)
 * fp32 jobs (the rank-r pairs, K = r) share launches, up to 32 jobs per launch: one layer's rank-r
 * gradient is a few MB and launch bound on its own; their results are bit-identical to n separate
 * dad_reconstruct_grad calls.  Runs of consecutive bf16 jobs with K a multiple of 32 and widths
 * multiples of 256 (the full gradients of a block's layers) share launches too, up to 16 per launch,
 * with ONE number of K chunks chosen for the run as a whole: gradients with few output tiles then
 * fill the chip together instead of each splitting K finely.  Such a job is summed in another chunk
 * order than a call of its own would use: equal to it within fp32 summation error (the parity bar
 * against the oracle is the same), bit-identical from run to run.  Other bf16 jobs run one after the
 * other exactly as dad_reconstruct_grad runs them.
 */
typedef struct {
    const void* L; /* K x h_in  */
    const void* R; /* K x h_out */
    float* G;      /* h_in x h_out, overwritten */
    int64_t K, h_in, h_out;
} dad_rebuild_desc;
size_t dad_reconstruct_grouped_workspace_bytes(int n, const dad_rebuild_desc* descs, dad_dtype dt);
dad_status dad_reconstruct_grad_grouped(int n, const dad_rebuild_desc* descs, dad_dtype dt, void* workspace,
                                        size_t ws_bytes, void* stream);

/* Activation functions phi whose derivative dad_backprop_delta applies. */
typedef enum {
    DAD_ACT_IDENTITY = 0,
    DAD_ACT_RELU = 1,
    DAD_ACT_TANH = 2,
    DAD_ACT_SIGMOID = 3
} dad_activation;

/*
 * dad_backprop_delta - Section 3.1, Eq. 3, one step of the delta recursion (the step that
 * produces the factor Delta_i the calls above consume):
 *     D_out[n][p] = ( sum_q D_next[n][q] * W_next[p][q] ) * phi'(Z[n][p])
 *   D_next    device, N x h_next, element type dt: Delta_{i+1}
 *   W_next    device, h x h_next, dt: W_{i+1} in the orientation of Eq. 1 (row p holds the
 *             weights leaving unit p of layer i)
 *   Z         device, N x h, dt: pre-activations Z_i
 *   act       phi_i
 *   D_out     device out, N x h, dt, dense rows of pitch h, overwritten.  Rows are independent,
 *             so a site passes the address of its first row inside the stacked buffer and its
 *             own row count N, and the delta is born in the stacked layout of Section 3.2.
 * For dt = DAD_BF16 the contraction accumulates in fp32 and the result is rounded once.
 * No workspace.  Errors: DAD_ERR_NULL, DAD_ERR_DTYPE, DAD_ERR_SHAPE (sizes or act out of range),
 * DAD_ERR_ALIGN (bf16 shapes served by the MFMA kernel need 16-byte aligned pointers).
 */
dad_status dad_backprop_delta(const void* D_next, const void* W_next, const void* Z, int64_t N, int64_t h,
                              int64_t h_next, dad_dtype dt, dad_activation act, void* D_out, void* stream);

/*
 * Synchronises `stream`, reads the flag a previous dad_compress_rank latched in
 * `workspace` and returns DAD_OK or DAD_ERR_NUMERIC (DAD_ERR_HIP if the sync or
 * copy fails).  The flag is cleared at the start of every dad_compress_rank.
 */
dad_status dad_poll_numeric_status(const void* workspace, void* stream);

/*
 * Optional per-kernel timing (instrumentation, not part of the method).  While enabled, every
 * kernel the library launches is bracketed by two HIP events on its launch stream.
 * dad_profile_get synchronises with the recorded events and returns, for kernel `id` in
 * [0, dad_profile_kernel_count()), the summed duration in milliseconds and the number of launches
 * since the last dad_profile_reset.  dad_profile_kernel_name gives the kernel's function name as a
 * profiler shows it.  Process-wide state, guarded by a mutex; disabled by default.
 */
dad_status dad_profile_enable(int on);
dad_status dad_profile_reset(void);
int dad_profile_kernel_count(void);
const char* dad_profile_kernel_name(int id);
dad_status dad_profile_get(int id, double* total_ms, int64_t* launches);

/*
 * In-process ceilings (instrumentation, not part of the method; bench.py reports them beside the
 * published peaks).  Both calls time their own launches with events, synchronise `stream` and
 * cannot be recorded into a graph.  `sink` is one caller-owned device word (4-byte aligned) that the
 * kernels may write.
 *
 * dad_probe_mfma_loop: one workgroup of eight waves per compute unit; every wave loads 4 + 2 operand
 * fragments once from `operands` (device, >= 48 KiB of bf16 values, 16-byte aligned; workgroup b
 * takes the b-th 48 KiB piece, modulo the pieces available) and issues iters * 8 independent
 * v_mfma_f32_32x32x16_bf16 with no memory access inside the loop.  *tflops = sustained rate.  The
 * matrix cores' clock under load depends on the operand values, hence real data as input.
 *
 * dad_probe_read_stream: one pass over `bytes` bytes of `src` with non-temporal 16-byte loads,
 * averaged over five launches.  *gbps = bytes / time.
 */
dad_status dad_probe_mfma_loop(const void* operands, size_t operand_bytes, int iters, void* sink, void* stream,
                               double* tflops);
dad_status dad_probe_read_stream(const void* src, size_t bytes, void* sink, void* stream, double* gbps);

#ifdef __cplusplus
}
#endif
#endif /* DAD_H */
