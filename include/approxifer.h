/*
 * approxifer.h -- C ABI of the ApproxIFER coding layer for AMD MI355X (gfx950).
 *
 * ApproxIFER (arXiv 2109.09868) serves K queries of a group with N workers that all
 * host the same model f: the K queries are encoded into N coded queries, every worker
 * runs f on one coded query, and the K predictions are rebuilt from whichever workers
 * answer, after workers that answered wrongly have been located and dropped.
 *
 * Naming.  N here is the NUMBER OF WORKERS.  The paper indexes its workers 0..N and so
 * has N+1 of them (Section 2, "System Architecture"); this library's N is the paper's
 * N+1.  S is the number of stragglers, A the number of Byzantine workers (the paper's E).
 * alpha[K] are the query nodes, beta[N] the worker nodes (Section 3, "ApproxIFER
 * Encoding").
 *
 * Conventions common to all entry points
 *   - d_* arguments are DEVICE pointers owned by the caller; h_* arguments are HOST
 *     pointers that are read before the call returns and may be freed afterwards.
 *   - All tensors are dense, row-major, with the last index contiguous.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Work is
 *     enqueued on it and the call returns without synchronising.  The library allocates
 *     no device memory and keeps no state between calls; the one kind of scratch memory
 *     it uses (the Byzantine decoders' workspace) is the caller's.
 *   - Return value: APPROXIFER_OK when the kernels were enqueued; a negative
 *     APPROXIFER_ERR_* code otherwise.  Every code but APPROXIFER_ERR_LAUNCH is decided on
 *     the host before anything is enqueued: no output is touched.  APPROXIFER_ERR_LAUNCH is
 *     the HIP runtime's refusal of a launch; a call that consists of two launches (see the
 *     individual entry points) may then have enqueued the first.  approxifer_strerror()
 *     turns a code into text.
 *   - G = 0, D = 0 or C = 0 is a valid empty call: nothing is enqueued, OK is returned.
 *   - Limits: 1 <= K <= APPROXIFER_MAX_K, 2 <= N <= APPROXIFER_MAX_N; the Byzantine
 *     decoder additionally needs N - S <= APPROXIFER_MAX_AVAIL_BYZ.
 *   - Nodes must be finite and pairwise distinct within each set.  A query node may
 *     coincide with a worker node; the interpolant then passes through the data there.
 */
#ifndef APPROXIFER_H
#define APPROXIFER_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define APPROXIFER_MAX_K 64
#define APPROXIFER_MAX_N 128
#define APPROXIFER_MAX_AVAIL_BYZ 64

#define APPROXIFER_OK 0
#define APPROXIFER_ERR_NULL_POINTER (-1)   /* a required pointer is NULL */
#define APPROXIFER_ERR_BAD_SHAPE (-2)      /* negative size, K < 1, N < 2, S < -1, S >= N, A < 1 ... */
#define APPROXIFER_ERR_LIMIT (-3)          /* K, N or N-S above the compiled limits */
#define APPROXIFER_ERR_BAD_NODES (-4)      /* a node is not finite, or two nodes of one set are equal */
#define APPROXIFER_ERR_TOO_FEW_WORKERS (-5)/* N - S < 2 (K + A): Algorithm 2's system would be under-determined */
#define APPROXIFER_ERR_BAD_SIGN_MODE (-6)  /* sign_mode is neither 0 nor 1 */
#define APPROXIFER_ERR_LAUNCH (-7)         /* the HIP runtime refused the launch */
#define APPROXIFER_ERR_WORKSPACE_LIMIT (-8)/* approxifer_decode_byzantine_static(): the built-in workspace is too small */

/* Decoder sign conventions, see approxifer_decode(). */
#define APPROXIFER_SIGN_WORKER_INDEX 0
#define APPROXIFER_SIGN_SURVIVOR_RANK 1

/* Passed as S to the decoders: every group has its own number of stragglers, read off its mask. */
#define APPROXIFER_S_FROM_MASK (-1)

/* Per-group status values written to d_status. */
#define APPROXIFER_GROUP_OK 0
#define APPROXIFER_GROUP_BAD_MASK 1        /* the group's mask does not hold an acceptable number of ones */

/*
 * Chebyshev nodes of Section 3, "ApproxIFER Encoding":
 *   h_alpha[j] = cos((2j+1) pi / (2K)), j = 0..K-1   (first kind, query nodes)
 *   h_beta[i]  = cos(i pi / (N-1)),     i = 0..N-1   (second kind, worker nodes)
 * Both arrays are host memory written by the call.  Returns OK, ERR_NULL_POINTER or
 * ERR_BAD_SHAPE (K < 1 or N < 2).
 */
int approxifer_chebyshev_nodes(int K, int N, double *h_alpha, double *h_beta);

/*
 * Encoder (Section 3, "ApproxIFER Encoding").  For every group g and worker i
 *     d_coded[g][i][:] = u_g(beta_i) = sum_j l_j(beta_i) d_queries[g][j][:],
 *     l_j(z) = ((-1)^j / (z - alpha_j)) / sum_j' ((-1)^j' / (z - alpha_j')),
 * Berrut's rational interpolant through the K queries, read at the worker nodes.
 * If beta_i equals some alpha_j exactly, coded query i is query j.
 *
 *   d_queries  [G][K][D] float32, device, read only
 *   d_coded    [G][N][D] float32, device, written; must not overlap d_queries
 *   h_alpha    [K] float64, host;  h_beta [N] float64, host
 * The basis functions are evaluated in float64 on the device and rounded to float32;
 * the contraction over j accumulates in float32.
 */
int approxifer_encode(const float *d_queries, float *d_coded,
                      int64_t G, int K, int N, int64_t D,
                      const double *h_alpha, const double *h_beta, void *stream);

/*
 * Forming groups out of a stream of queries (Section 2, "System Architecture": the K queries of a group are
 * encoded together).  With the [G][K][D] layout of approxifer_encode() a stream of Q queries stored row by row,
 * [Q][D], IS its groups: queries g K .. g K + K - 1 are group g, no copy is made.  approxifer_group_count()
 * returns G = ceil(Q / K) (-1 for Q < 0 or K < 1).  When K does not divide Q the last group is short; the paper
 * has no rule for it, this library completes it by repeating the stream's last query (the interpolant then passes
 * through that query at every added node -- for a group of one query this is the replication the encoder reduces
 * to at K = 1 -- and the added answers are simply not read back).
 *
 * approxifer_pad_last_group(): d_queries is a device buffer of at least G K rows of D floats whose first Q rows
 * hold the stream; rows Q .. G K - 1 are overwritten with copies of row Q - 1.  Nothing is enqueued when K
 * divides Q, or when Q = 0 or D = 0.  Ungrouping needs no call: row q of the decoded [G][K][C] tensor (of the
 * [G][K] top-1 tensor) is query q's answer, rows Q and up belong to the repeated query.
 * Returns OK, ERR_NULL_POINTER, ERR_BAD_SHAPE (Q < 0, D < 0, K < 1), ERR_LIMIT (K > APPROXIFER_MAX_K) or ERR_LAUNCH.
 */
int64_t approxifer_group_count(int64_t Q, int K);
int approxifer_pad_last_group(float *d_queries, int64_t Q, int K, int64_t D, void *stream);

/*
 * Decoder (Section 3, "ApproxIFER Decoding", step 2).  For every group g, with F the
 * set of workers whose mask byte is non-zero, in ascending order,
 *     d_out[g][j][:] = r_g(alpha_j)
 *                    = sum_{i in F} w_i d_preds[g][i][:] / sum_{i in F} w_i,
 *     w_i = s_i / (alpha_j - beta_i).
 * sign_mode APPROXIFER_SIGN_WORKER_INDEX takes s_i = (-1)^i with i the worker index,
 * as that formula is printed; APPROXIFER_SIGN_SURVIVOR_RANK takes s_i = (-1)^rank(i in F),
 * which is Berrut's interpolant (Section 3, eq. (2)) on the surviving nodes.  The two are
 * equal when no worker is missing.
 *
 *   d_preds   [G][N][C] float32, device; rows of workers with mask 0 are never read
 *   d_mask    [G][N] uint8, device; non-zero = the worker returned
 *   d_out     [G][K][C] float32, device, written
 *   d_status  [G] int32, device, written, or NULL.  A group whose mask does not hold
 *             exactly N-S non-zero bytes gets APPROXIFER_GROUP_BAD_MASK and its d_out
 *             rows are left untouched; every other group gets APPROXIFER_GROUP_OK.
 *   S         number of stragglers of every group, 0 <= S < N, or APPROXIFER_S_FROM_MASK:
 *             groups may then differ in how many workers returned (the formula of Section 3
 *             holds for any non-empty F); only a group with no survivor at all is a bad mask.
 * Weights and accumulation are float64; each output is rounded to float32 once.
 */
int approxifer_decode(const float *d_preds, const uint8_t *d_mask, float *d_out, int32_t *d_status,
                      int64_t G, int K, int N, int S, int64_t C,
                      const double *h_alpha, const double *h_beta, int sign_mode, void *stream);

/*
 * Byzantine decoder (Section 3, "ApproxIFER Decoding", steps 1-2, Algorithm 2).
 * For every group: among the N-S available workers locate A adversaries, drop them,
 * decode over the rest as approxifer_decode() does.
 * Location, per class c = 0..C-1 (Algorithm 2): with M = K + A and x_i = beta_i,
 * y_i = d_preds[g][i][c] for the available i, find P (degree M-1) and
 * Q = 1 + Q_1 x + .. + Q_{M-1} x^{M-1} minimising sum_i (P(x_i) - y_i Q(x_i))^2
 * (ordinary least squares, float64 Householder QR), set a_i = Q(x_i), and note the A
 * workers of smallest |a_i| (equal magnitudes: smaller worker index first).  The A workers
 * noted most often over the C classes (equal counts: smaller worker index first) are the
 * adversaries.
 *
 *   d_adv     [G][A] int32, device, written: located workers in ascending order
 *   d_workspace, workspace_bytes
 *             device scratch memory owned by the caller, 8-byte aligned, or NULL / 0; contents on entry and exit
 *             are meaningless, the call initialises what it uses.  Two things live there.
 *             (1) The vote of Algorithm 2's return step is the one place where the classes of a group meet.  With
 *             few groups and many classes the library spreads a group's classes over several workgroups, which
 *             pool their per-class picks in N vote counters and an arrival counter per group.
 *             (2) Without stragglers (S = 0, the setting of the paper's Byzantine experiments, or
 *             APPROXIFER_S_FROM_MASK) every group whose mask is full fits the same node set: the part of
 *             Algorithm 2's system that does not depend on the predictions is then factorised once per call
 *             instead of once per group, and kept in the workspace.
 *             approxifer_workspace_bytes() gives the size that allows both.  With NULL, fewer bytes or a
 *             misaligned pointer the call uses what fits and is just as correct: d_out, d_adv and d_status hold
 *             the same bits; only time is lost (every group stays with one workgroup and repeats the
 *             factorisation).  Nothing but the workspace is ever used as scratch: output rows are written
 *             once, with their final values.  The workspace must not be shared with a call that may run
 *             concurrently.
 *   other arguments as approxifer_decode(); groups with a bad mask leave d_out and
 *   d_adv rows untouched.
 * On APPROXIFER_ERR_LAUNCH the kernels that prepare the workspace may have been enqueued; no output
 * is touched.
 * Requires A >= 1, N - S >= 2 (K + A) (Section 3, eq. (3), the decoding condition) and
 * N - S <= APPROXIFER_MAX_AVAIL_BYZ.  With S = APPROXIFER_S_FROM_MASK a group is decoded when its
 * own number of available workers n satisfies 2 (K + A) <= n <= APPROXIFER_MAX_AVAIL_BYZ and gets
 * APPROXIFER_GROUP_BAD_MASK otherwise.  A worker whose node is exactly 0 can never be
 * located, since Q(0) = 1 by construction; the Chebyshev worker nodes contain 0 only
 * when N is odd.
 */
int approxifer_decode_byzantine(const float *d_preds, const uint8_t *d_mask, float *d_out,
                                int32_t *d_adv, int32_t *d_status,
                                int64_t G, int K, int N, int S, int A, int64_t C,
                                const double *h_alpha, const double *h_beta, int sign_mode,
                                void *d_workspace, size_t workspace_bytes, void *stream);

/*
 * Size in bytes of the workspace with which approxifer_decode_byzantine() and
 * approxifer_decode_byzantine_homogeneous() run fastest for this shape (Algorithm 2, return step: the
 * per-class picks of a group are pooled there when its classes are spread over several workgroups).
 * 0 when the shape needs none -- a fixed number S > 0 of stragglers with enough groups to fill the GPU with one
 * workgroup each, or few classes -- and for shapes the decoders refuse.  Host arithmetic only; at most
 * 4 (N + 1) bytes per group plus 13 KiB, each part rounded up to a multiple of 256.
 */
size_t approxifer_workspace_bytes(int64_t G, int K, int N, int S, int A, int64_t C);

/*
 * approxifer_decode_byzantine() for callers that cannot allocate device memory, not even a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The same call with
 * the workspace arguments left out; the scratch memory is an array of APPROXIFER_STATIC_WORKSPACE_BYTES
 * bytes built into the library's device code (every GPU the library runs on holds one copy until the
 * process ends).  The call allocates and frees nothing and calls no allocating routine; inputs and outputs
 * are still the caller's.
 *   - A shape for which approxifer_workspace_bytes() exceeds APPROXIFER_STATIC_WORKSPACE_BYTES is refused
 *     with APPROXIFER_ERR_WORKSPACE_LIMIT before anything is enqueued (4 (N + 1) G bytes are needed when
 *     few groups bring hundreds of classes or more, up to 13 KiB when no stragglers are asked for; shapes
 *     that need no workspace are never refused).
 *   - The device of `stream` must be the current device.  The first call on a device looks up the address
 *     of that device's copy of the array (no allocation, no synchronisation).
 *   - All calls on one GPU share that GPU's array.  Each call clears the part it uses with a kernel of
 *     its own, so what an earlier call left there does not matter; two calls whose work OVERLAPS on one
 *     GPU (different streams, or graphs replayed concurrently) race on it and give undefined results.
 *     Calls on one stream, one after the other, are safe.
 * Results, other arguments, requirements and error codes are those of approxifer_decode_byzantine().
 */
#define APPROXIFER_STATIC_WORKSPACE_BYTES 65536
int approxifer_decode_byzantine_static(const float *d_preds, const uint8_t *d_mask, float *d_out,
                                       int32_t *d_adv, int32_t *d_status,
                                       int64_t G, int K, int N, int S, int A, int64_t C,
                                       const double *h_alpha, const double *h_beta, int sign_mode, void *stream);

/*
 * Byzantine decoder with the locator of Section 2, Algorithm 1, in place of Algorithm 2: the
 * same call, the same picks, vote and decode, but per class the fit leaves Q_0 free.  With
 * M = K + A, P and Q both of degree M-1, the coefficient vector (P_0..P_{M-1}, Q_0..Q_{M-1})
 * is the unit vector minimising sum_i (P(x_i) - y_i Q(x_i))^2 over the available workers: the
 * right singular vector of the smallest singular value of the n x 2M matrix of the
 * homogeneous system (float64 Householder QR, then inverse iteration on the triangular
 * factor and, for a class whose iteration does not settle, one-sided Jacobi rotations
 * until every pair of its columns is orthogonal to rounding).  a_i = Q(x_i) is
 * defined up to one factor, which the order of the |a_i| does not see.  Unlike Algorithm 2
 * this locator can find a worker whose node is exactly 0.  It costs a singular value
 * decomposition per class where Algorithm 2 costs a least-squares solve.
 * The iterations are bounded (24 rounds of inverse iteration, then at most 30 Jacobi sweeps); a
 * class whose columns are still not orthogonal to rounding after that -- not observed on finite
 * data -- votes with the shortest column found so far, best effort, and no status reports it.
 * Arguments, requirements and error behaviour as approxifer_decode_byzantine().
 */
int approxifer_decode_byzantine_homogeneous(const float *d_preds, const uint8_t *d_mask, float *d_out,
                                            int32_t *d_adv, int32_t *d_status,
                                            int64_t G, int K, int N, int S, int A, int64_t C,
                                            const double *h_alpha, const double *h_beta, int sign_mode,
                                            void *d_workspace, size_t workspace_bytes, void *stream);

/*
 * Decoder by rational reconstruction (Appendix A, Algorithm 3 and Theorem 2).  For every group, class c and
 * query j: with (P, Q) the least-squares fit of Algorithm 2 (degrees K + A - 1, Q_0 = 1) to the class's
 * values on the available workers,
 *     d_out[g][j][c] = P(alpha_j) / Q(alpha_j).
 * No worker is located or dropped and Berrut's interpolant is not used: when the hosted model makes the
 * coded predictions exactly rational in the node and at most A workers lie, P / Q is that rational function
 * (Theorem 2).  The paper sets this decoder aside because the quotient is fragile under round-off -- P and Q
 * share the error-locator factor -- and so does this library: it is here to make the comparison possible,
 * approxifer_decode_byzantine() is the decoder to use.  On float32 data of the paper's sizes single groups lose
 * several digits; the fit's condition number, not the arithmetic (float64 Householder QR), bounds the accuracy.
 *   arguments, requirements, status values and error codes as approxifer_decode_byzantine(), without
 *   d_adv, sign_mode and workspace; groups with a bad mask leave their d_out rows untouched.  Q can vanish
 *   at a query node only by accident of the data; the quotient is then non-finite.
 */
int approxifer_decode_rational(const float *d_preds, const uint8_t *d_mask, float *d_out, int32_t *d_status,
                               int64_t G, int K, int N, int S, int A, int64_t C,
                               const double *h_alpha, const double *h_beta, void *stream);

/*
 * Fused decoder + top-1 (Section 4.1, "Performance metric": the paper scores the class of the
 * largest decoded soft label).  Decodes exactly as approxifer_decode() does, in float64, and for
 * every group g and query j writes only
 *     d_top1[g][j]  = argmax_c r_g(alpha_j)[c]      (equal values: the smallest c)
 *     d_score[g][j] = that largest decoded value, rounded to float32 (d_score may be NULL)
 * The [G][K][C] prediction tensor is never written.  The argmax is taken on the float64
 * accumulators, before any rounding.
 *
 *   d_top1    [G][K] int32, device, written
 *   d_score   [G][K] float32, device, written, or NULL
 *   other arguments, status values and errors as approxifer_decode(); groups with a bad mask
 *   leave their d_top1 / d_score rows untouched.
 */
int approxifer_decode_top1(const float *d_preds, const uint8_t *d_mask, int32_t *d_top1, float *d_score,
                           int32_t *d_status, int64_t G, int K, int N, int S, int64_t C,
                           const double *h_alpha, const double *h_beta, int sign_mode, void *stream);

/*
 * Top-1 of an already decoded tensor (Section 4.1, "Performance metric"): for every row of d_values [rows][C]
 * the class of the largest value (equal values: the smallest class) and, optionally, that value.  For the
 * outputs of approxifer_decode_byzantine(), whose [G][K][C] tensor is [G K][C] row by row;
 * approxifer_decode_top1() fuses the same decision into the plain decoder.  The decision is taken on the
 * float32 values as stored.  NaN never wins; a row without any ordinary value gives class 0.
 *   d_values  [rows][C] float32, device, read only
 *   d_top1    [rows] int32, device, written;  d_score [rows] float32, device, written, or NULL
 * Returns OK, ERR_NULL_POINTER, ERR_BAD_SHAPE (rows < 0 or C < 0), ERR_LIMIT (C >= 2^31) or ERR_LAUNCH.
 */
int approxifer_top1(const float *d_values, int32_t *d_top1, float *d_score, int64_t rows, int64_t C, void *stream);

/*
 * Wait rule (Section 3, "ApproxIFER Decoding", step 1: the decoder waits for the results of the
 * fastest workers -- K of them without adversaries, 2 (K + E) with E of them).  Turns arrival times
 * into the survivor mask the decoders take: for every group g the `wait_for` workers with the
 * smallest arrival time get mask 1, all others 0.  Equal times: the smaller worker index first.
 * A time that is not finite (NaN, +-inf) means the worker never answers; a group in which fewer
 * than `wait_for` workers answer has all of those marked, and its count says so.
 *
 *   d_arrival  [G][N] float32, device, read only: arrival time of every worker's result, any unit
 *   d_mask     [G][N] uint8, device, written (0 or 1)
 *   d_count    [G] int32, device, written, or NULL: number of ones in the group's mask
 *   wait_for   1 <= wait_for <= N
 * Returns OK, ERR_NULL_POINTER, ERR_BAD_SHAPE (G < 0, N < 1, wait_for out of range) or ERR_LIMIT
 * (N > APPROXIFER_MAX_N).
 */
int approxifer_wait_mask(const float *d_arrival, uint8_t *d_mask, int32_t *d_count,
                         int64_t G, int N, int wait_for, void *stream);

/* Text for a return code; never NULL.  The string is static. */
const char *approxifer_strerror(int code);

/* Library version, major*10000 + minor*100 + patch. */
int approxifer_version(void);

#ifdef __cplusplus
}
#endif
#endif /* APPROXIFER_H */
