// ApproxIFER Byzantine decoder for gfx950: Algorithm 2 (error locator) followed by the decoder of
// Section 3, "ApproxIFER Decoding", one workgroup per group.
//
// Algorithm 2 fits, per class c, polynomials P (degree M-1) and Q (degree M-1, Q_0 = 1), M = K+A, to
//     P(x_r) - y_rc Q(x_r) = 0        over the n available workers (x_r their nodes),
// in the least-squares sense, reads a_r = Q(x_r), lets the A smallest |a_r| of every class vote and
// returns the A most voted workers.  The system is  V p + C_c q = y_c  with V the n x M Vandermonde
// matrix of the nodes and C_c = -diag(y_c) V[:, 1:].
//
// Two kernels compute the same thing:
//
//  * decode_byzantine_proj_kernel (K+A <= 16, at most 48 available workers, n-M <= 32).  V is the
//    same for every class of a group, so its Householder QR is done ONCE per group, by one wave
//    with one lane per column of [V | I] held in registers (pivot columns travel by v_readlane):
//    that leaves U = the last n-M rows of Q^T, an orthonormal basis of range(V)'s complement, in
//    LDS.  Eliminating p exactly, class c only has to solve the (n-M) x (M-1) problem
//        min_q || U C_c q - U y_c ||,
//    so a class needs 16 lanes (lane = column, 15 = right-hand side), four classes share a wave, the
//    four projected systems are formed by the float64 matrix cores (operands read from LDS, result
//    directly in the lane layout of the factorisation), and the Householder QR runs entirely in
//    registers: the pivot column reaches the other lanes of the class through DPP row broadcasts.
//    No LDS traffic and no barrier inside either factorisation.
//
//  * decode_byzantine_general_kernel (everything else up to 64 available workers).  A class owns
//    2M neighbouring lanes, lane j owns COLUMN j of the full n x (2M-1) system, which sits in LDS
//    row-major; a Householder step walks down the pivot column (an LDS broadcast).
//
// Both finish the same way: Q by back substitution, a_r = Q(x_r) by Horner's rule, the A smallest
// |a_r| (equal magnitudes: smaller worker index first; by counting ranks in the general kernel, by A
// rounds of a DPP arg-min in the projected one) vote in an LDS histogram, the A most voted workers
// (equal counts: smaller index first) leave the available list, and the workgroup decodes the group
// over the rest.
#include <mutex>

#include "decode_common.h"

// Built-in workspace of approxifer_decode_byzantine_static(): one copy per GPU the library runs on, held until
// the process ends.  In host code this name only stands for the symbol; its device address comes from
// hipGetSymbolAddress (see static_workspace below) and kernels receive that address as an argument.
static __device__ __align__(256) unsigned char scratch[APPROXIFER_STATIC_WORKSPACE_BYTES];

namespace approxifer {
namespace {

// ------------------------------------------------------------------------------------------------
// shared tail: vote -> located adversaries -> F -> decode
// ------------------------------------------------------------------------------------------------
// Decoder contraction of one group over every column tile, predictions read from global memory.
template <int VEC>
__device__ __forceinline__ void contract_group(const float *__restrict__ pg, float *__restrict__ og, const int *F, int nF,
                                               int K, int KP, int64_t C, int64_t Cv, const double *WdT) {
    for (int64_t cv0 = 0; cv0 < Cv; cv0 += kColsPerTile) {
        const int64_t cv1 = (cv0 + kColsPerTile < Cv) ? cv0 + kColsPerTile : Cv;
        typename PredVec<VEC>::type unused[kRowChunk];
        contract_tile<VEC, false>(pg, og, F, nF, K, KP, C, cv0, cv1, WdT, unused);
    }
}

// The A most voted workers (equal counts: smaller index first) go to adv_g in ascending order; F = the
// available workers without them (ascending), Fpos = their positions in `avail`.  n <= 64, N <= 128.
// One wave does it in registers: lane i ranks workers i and i + 64 by counting against the vote counts
// (broadcast reads of LDS), ballots turn ranks into the ascending lists.
// select_adversaries_wave: called by one whole wave after every vote has been added and a barrier; the lists are
// visible after the next barrier.
__device__ __forceinline__ void select_adversaries_wave(int32_t *__restrict__ adv_g, const int *avail, int n, int N,
                                                        int A, const int *votes, int *F, int *Fpos) {
    {
        const int lane = lane_id();
        const int mine0 = lane < N ? votes[lane] : -1;
        const int mine1 = lane + kWave < N ? votes[lane + kWave] : -1;
        int rank0 = 0, rank1 = 0;
#pragma unroll 8
        for (int o = 0; o < N; ++o) {
            const int v = votes[o];
            rank0 += (v > mine0 || (v == mine0 && o < lane)) ? 1 : 0;
            rank1 += (v > mine1 || (v == mine1 && o < lane + kWave)) ? 1 : 0;
        }
        const bool s0 = lane < N && rank0 < A;
        const bool s1 = lane + kWave < N && rank1 < A;
        const unsigned long long m0 = __ballot(s0), m1 = __ballot(s1);
        const unsigned long long below = (1ull << lane) - 1ull;
        if (s0) adv_g[__popcll(m0 & below)] = lane;
        if (s1) adv_g[__popcll(m0) + __popcll(m1 & below)] = lane + kWave;
        const int w = lane < n ? avail[lane] : 0;
        const bool dropped = ((w < kWave ? m0 >> w : m1 >> (w - kWave)) & 1ull) != 0ull;
        const bool keep = lane < n && !dropped;
        const unsigned long long mk = __ballot(keep);
        if (keep) {
            const int pos = __popcll(mk & below);
            F[pos] = w;
            Fpos[pos] = lane;
        }
    }
}

// Called by the whole workgroup after every vote has been added and a barrier; ends with a barrier.
__device__ __forceinline__ void select_adversaries(int32_t *__restrict__ adv_g, const int *avail, int n, int N, int A,
                                                   const int *votes, int *F, int *Fpos) {
    if (wave_id() == 0) select_adversaries_wave(adv_g, avail, n, N, A, votes, F, Fpos);
    __syncthreads();
}

// Several workgroups share a group (few groups, many classes: each takes part of the classes).  They meet in the
// group's N+1 words of the caller's workspace -- N vote counters and an arrival counter, cleared by
// clear_workspace_kernel before the launch.  These words are touched by device-scope atomic read-modify-writes only,
// which are carried out at the one place all workgroups of the device share.  A part's additions have been carried
// out once their old values are back; only then does it count itself in, and the part that counts itself in last
// reads the votes with the same kind of operation: no cache write-back or invalidation (a fence) is needed, and none
// of the part's other memory traffic has to be ordered with this.  No part waits for another: whichever arrives last
// gets every vote (into `votes`, LDS) and true, and finishes the group.
// Called by the whole workgroup after a barrier that follows its last vote; ends with a barrier when it returns true.
__device__ __forceinline__ bool pool_votes_last_arrival(int *gvotes, int *votes, int N, int splits, int *flag) {
    const int tid = threadIdx.x;
    int seen = 0;
    for (int i = tid; i < N; i += blockDim.x)
        if (votes[i] != 0) seen |= __hip_atomic_fetch_add(&gvotes[i], votes[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    asm volatile("" ::"v"(seen));                         // the returned values are waited for
    __syncthreads();
    if (tid == 0)
        *flag = __hip_atomic_fetch_add(&gvotes[N], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == splits - 1 ? 1 : 0;
    __syncthreads();
    if (*flag == 0) return false;
    for (int i = tid; i < N; i += blockDim.x)
        votes[i] = __hip_atomic_fetch_add(&gvotes[i], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    return true;
}

// vec4: prediction rows are 16-byte aligned and C % 4 == 0, Cv = C / 4; else Cv = C.
__device__ __forceinline__ void finish_group(const float *__restrict__ pg, float *__restrict__ og,
                                             int32_t *__restrict__ adv_g, const int *avail, int n, int N, int A, int K,
                                             int KP, int64_t C, int64_t Cv, bool vec4, int sign_mode,
                                             const double *alpha_s, const double *beta_s, const int *votes,
                                             int *F, int *Fpos, double *WdT) {
    select_adversaries(adv_g, avail, n, N, A, votes, F, Fpos);
    const int nF = n - A;
    decoder_weights(alpha_s, beta_s, F, nF, K, KP, sign_mode, WdT);
    __syncthreads();
    if (vec4) contract_group<4>(pg, og, F, nF, K, KP, C, Cv, WdT);
    else contract_group<1>(pg, og, F, nF, K, KP, C, Cv, WdT);
}

// Rank of |a_r| among the n rows of one class (LDS key[n]); the A smallest vote for their worker.
// Called by the lanes of one class, lane j of `width` handling rows j, j+width, ..
__device__ __forceinline__ void pick_and_vote(const double *key, const int *avail, int n, int A, int j, int width,
                                              int *votes) {
    for (int r = j; r < n; r += width) {
        const double mine = key[r];
        int rank = 0;                                  // equal magnitudes keep ascending worker order
        for (int o = 0; o < n; ++o) {
            const double other = key[o];
            rank += (other < mine || (other == mine && o < r)) ? 1 : 0;
        }
        if (rank < A) atomicAdd(&votes[avail[r]], 1);
    }
}

// ------------------------------------------------------------------------------------------------
// projected kernel: shared QR of the Vandermonde block, per-class QR in registers
// ------------------------------------------------------------------------------------------------
constexpr int kClsLanes = 16;      // lanes per class (one DPP row)
constexpr int kClsPerWave = 4;
constexpr int kPwStride = 16;      // powers table row: x^0 .. x^15
constexpr int kProjMaxM = 16;      // M - 1 <= 15 unknown columns in lanes 0..14, right-hand side in lane 15
// U in LDS: rows padded to a multiple of four (the matrix-core tiles below take four rows of U at a time), row
// stride chosen so that the sixteen (row, column) pairs one operand load touches fall in distinct banks.
// Register-array bound of Algorithm 1's locator for a tile of NB rows: eq. (3) gives M <= n / 2 <= NB / 2.
constexpr int hom_mt(int NB) { return NB / 2 < kProjMaxM ? NB / 2 : kProjMaxM; }
constexpr int ush_rows(int RM) { return (RM + 3) & ~3; }
constexpr int ush_stride(int NB) { return NB % 16 == 0 ? NB + 4 : NB; }

template <int LANE>
__device__ __forceinline__ double row_bcast(double v) {   // lane LANE of every 16-lane row, to the whole row
    // all rows and banks enabled and every source lane exists: the 'old' operand is never used, and with
    // bound_ctrl set the compiler knows it and does not materialise it
    const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(v), 0x150 + LANE, 0xF, 0xF, true);
    const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(v), 0x150 + LANE, 0xF, 0xF, true);
    return __hiloint2double(hi, lo);
}

// The same for a lane index that is only known after unrolling.
__device__ __forceinline__ double row_bcast_dyn(double v, int lane_in_row) {
    switch (lane_in_row) {
        case 0: return row_bcast<0>(v);
        case 1: return row_bcast<1>(v);
        case 2: return row_bcast<2>(v);
        case 3: return row_bcast<3>(v);
        case 4: return row_bcast<4>(v);
        case 5: return row_bcast<5>(v);
        case 6: return row_bcast<6>(v);
        case 7: return row_bcast<7>(v);
        case 8: return row_bcast<8>(v);
        case 9: return row_bcast<9>(v);
        case 10: return row_bcast<10>(v);
        case 11: return row_bcast<11>(v);
        case 12: return row_bcast<12>(v);
        case 13: return row_bcast<13>(v);
        case 14: return row_bcast<14>(v);
        default: return row_bcast<15>(v);
    }
}

// Reciprocal and square root of a normal, positive-or-negative (rcp) / positive (sqrt) double to full
// double precision: the hardware estimate refined by two Newton (Goldschmidt) steps and, for the root, one
// residual correction.  No scaling for denormals or infinities and no final correctly-rounded fix-up, which
// the factorisations here do not need: their operands are column norms and pivots, and a zero norm is
// handled by the caller.
__device__ __forceinline__ double rcp_normal(double x) {
    double r = __builtin_amdgcn_rcp(x);
    r = fma(fma(-x, r, 1.0), r, r);
    r = fma(fma(-x, r, 1.0), r, r);
    return r;
}
__device__ __forceinline__ double sqrt_normal(double s) {
    const double y = __builtin_amdgcn_rsq(s);
    double g = s * y, h = 0.5 * y;
    double r = fma(-h, g, 0.5);
    g = fma(g, r, g);
    h = fma(h, r, h);
    r = fma(-h, g, 0.5);
    g = fma(g, r, g);
    h = fma(h, r, h);
    return fma(fma(-g, g, s), h, g);
}

// Householder reflector of a pivot column x (rows k..): returns alpha = -sign(x_k) ||x|| and the factor
// f = 2 v^T a / (v^T v) for a column a, v = x - alpha e_k, given sigma = x^T x, d = x^T a.
struct Reflector {
    double alpha, f;
    bool degenerate;
};
__device__ __forceinline__ Reflector reflector(double sigma, double d, double xkk, double akj) {
    Reflector h;
    h.degenerate = !(sigma > 0.0);
    // a zero (or NaN) column: the caller applies no reflection; alpha and f stay finite so that a factor 0 times
    // them is 0 and not NaN (an exactly singular system must keep its exact zero on the diagonal)
    const double s = h.degenerate ? 1.0 : sigma;
    const double nrm = sqrt_normal(s);
    h.alpha = (xkk >= 0.0) ? -nrm : nrm;
    const double scale = rcp_normal(fma(-h.alpha, xkk, s));   // 2 / (v^T v) = 1 / (sigma + |x_k| ||x||)
    h.f = scale * fma(-h.alpha, akj, d);
    return h;
}

// ---- once per group: U = rows M..n-1 of Q^T, V = Q R (one wave; lane = column of [V | I]) ----------
template <int K0, int NB>
struct SharedQrSteps {
    static __device__ __forceinline__ void run(double (&col)[NB], int lane, int M) {
        if (K0 < M) {
            double dt[2] = {0.0, 0.0};                       // two partial sums: shorter dependency chains
#pragma unroll
            for (int r = K0; r < NB; ++r) dt[(r - K0) & 1] = fma(read_lane(col[r], K0), col[r], dt[(r - K0) & 1]);
            const double d = dt[0] + dt[1];                  // x^T a for this lane's column a ..
            const double sigma = read_lane(d, K0);           // .. which in the pivot lane is x^T x
            const double xkk = read_lane(col[K0], K0);
            const Reflector h = reflector(sigma, d, xkk, col[K0]);
            // no branch: columns up to the pivot (and every column of a degenerate step) take the factor 0, so the
            // pivot values read for the dot products serve the update as well
            const double nf = (!h.degenerate && lane > K0) ? -h.f : 0.0;
            const double ckk = fma(nf, xkk - h.alpha, col[K0]);
            col[K0] = (!h.degenerate && lane == K0) ? h.alpha : ckk;      // R[k][k] in the pivot lane
#pragma unroll
            for (int r = K0 + 1; r < NB; ++r) col[r] = fma(nf, read_lane(col[r], K0), col[r]);
            SharedQrSteps<K0 + 1, NB>::run(col, lane, M);
        }
    }
};
template <int NB>
struct SharedQrSteps<kProjMaxM, NB> {
    static __device__ __forceinline__ void run(double (&)[NB], int, int) {}
};

// Pw[r][e] = x_r^e (LDS), n rows, M <= 16 columns.  Writes Ush[i][r] = U[i][r], i < RM, row stride ush_stride(NB).
// WITH_RANGE (Algorithm 1's locator needs the whole factorisation): also Q1sh[i][r] = row i < M of Q^T (16 rows of
// the same stride, rows from M on left as they are) and Rv[i][j] = R[i][j], the M x M triangular factor of V (row
// stride 16, zero below the diagonal).
template <int NB, int RM, bool WITH_RANGE = false>
__device__ __forceinline__ void shared_complement_basis(const double *Pw, int n, int M, double *Ush, double *Q1sh = nullptr,
                                                        double *Rv = nullptr) {
    const int lane = lane_id();
    double col[NB];
    const bool vandermonde = lane < M;                // lanes 0..M-1: V; lanes M..M+n-1: the identity
    const int e = vandermonde ? lane : 0;
#pragma unroll
    for (int r = 0; r < NB; ++r) {
        const double p = Pw[(r < n ? r : 0) * kPwStride + e];
        col[r] = (r < n) ? (vandermonde ? p : (lane - M == r ? 1.0 : 0.0)) : 0.0;
    }
    SharedQrSteps<0, NB>::run(col, lane, M);
    const int r_out = lane - M;                     // this lane holds column r_out of Q^T
    if (r_out >= 0 && r_out < n) {
#pragma unroll
        for (int row = 2; row < NB; ++row) {        // M >= 2 always
            const int i = row - M;
            if (i >= 0 && i < RM) Ush[i * ush_stride(NB) + r_out] = col[row];
        }
        if (WITH_RANGE) {
#pragma unroll
            for (int row = 0; row < kProjMaxM && row < NB; ++row)
                if (row < M) Q1sh[row * ush_stride(NB) + r_out] = col[row];
        }
    }
    if (WITH_RANGE && lane < M) {
#pragma unroll
        for (int row = 0; row < kProjMaxM && row < NB; ++row)
            if (row < M) Rv[row * kProjMaxM + lane] = row <= lane ? col[row] : 0.0;
    }
}

// ---- per class: Householder QR of the projected system, in registers ----------------------------
// Steps K0 .. KEND-1 (those below `cols`); KEND = min(15, RM - 1) bounds the unrolling: cols <= R - 1 <= RM - 1.
template <int K0, int KEND, int RM>
struct ClassQrSteps {
    static __device__ __forceinline__ void run(double (&a)[RM], int j, int cols) {
        if (K0 < cols) {
            double v[RM];
            double dt[2] = {0.0, 0.0};                       // two partial sums: shorter dependency chains
#pragma unroll
            for (int r = K0; r < RM; ++r) {
                v[r] = row_bcast<K0>(a[r]);
                dt[(r - K0) & 1] = fma(v[r], a[r], dt[(r - K0) & 1]);
            }
            const double d = dt[0] + dt[1];                  // x^T a for this lane's column a ..
            const double sigma = row_bcast<K0>(d);           // .. which in the pivot lane is x^T x
            const Reflector h = reflector(sigma, d, v[K0], a[K0]);
            const double nf = (!h.degenerate && j > K0) ? -h.f : 0.0;       // no branch: other columns take the factor 0
            const double akk = fma(nf, v[K0] - h.alpha, a[K0]);
            a[K0] = (!h.degenerate && j == K0) ? h.alpha : akk;           // R[k][k] in the pivot lane
#pragma unroll
            for (int r = K0 + 1; r < RM; ++r) a[r] = fma(nf, v[r], a[r]);
            ClassQrSteps<K0 + 1, KEND, RM>::run(a, j, cols);
        }
    }
};
template <int KEND, int RM>
struct ClassQrSteps<KEND, KEND, RM> {
    static __device__ __forceinline__ void run(double (&)[RM], int, int) {}
};

// Back substitution R q = rhs over the first `cols` rows; column t of R sits in lane t of the row, the
// transformed right-hand side in lane 15.  Every lane of the class ends with the whole solution.
template <int T, int NS, int RM>
struct BackSubst {
    // s enters as the transformed right-hand side and leaves as the solution: entry T is final once solved
    static __device__ __forceinline__ void run(const double (&a)[RM], double (&s)[NS], int cols) {
        if (T < cols) {
            s[T] = s[T] * rcp_normal(row_bcast<T>(a[T]));
#pragma unroll
            for (int i = 0; i < T; ++i) s[i] = fma(-row_bcast<T>(a[i]), s[T], s[i]);
        } else {
            s[T] = 0.0;                                   // no such unknown
        }
        BackSubst<T - 1, NS, RM>::run(a, s, cols);
    }
};
template <int NS, int RM>
struct BackSubst<-1, NS, RM> {
    static __device__ __forceinline__ void run(const double (&)[RM], double (&)[NS], int) {}
};

// (value, row) minimum over the 16 lanes of a class: smaller value first, equal values: smaller row.
template <int CTRL>
__device__ __forceinline__ void row_min_step(double &v, int &i) {
    const double ov = dpp_exchange<CTRL>(v);
    const int oi = __builtin_amdgcn_update_dpp(0, i, CTRL, 0xF, 0xF, true);
    const bool take = ov < v || (ov == v && oi < i);
    v = take ? ov : v;
    i = take ? oi : i;
}

// Algorithm 2, steps 1-5, for four classes at a time, by one wave.
//   ycol (per lane): the staged predictions of class slot (lane % 16) & 3 of this round, ycol[r * CW] = prediction of
//   the r-th available worker for that class, float, zero past n (an empty slot points at zeros);
//   live, votes (per lane): class slot lane / 16 holds a class, and the vote counters of its group;
//   Ush[ush_rows(RM)][ush_stride(NB)] (zero past row n-M and column n), Pw[NB][16] (rows past n zero), xs[n]: LDS.
template <int NB, int RM>
__device__ __forceinline__ void locate_classes_proj(const float *ycol, int CW, bool live, const int *avail,
                                                    const double *xs, const double *Pw, const double *Ush, int n,
                                                    int M, int A, int *votes) {
    typedef double v4d __attribute__((ext_vector_type(4)));
    const int lane = lane_id();
    const int j = lane % kClsLanes;
    const int cols = M - 1;                               // unknowns Q_1 .. Q_{M-1}

    // column of this lane: -y x^(j+1) for the unknown Q_(j+1), y for the right-hand side, 0 on idle lanes
    const int e = j < cols ? j + 1 : 0;
    const double sgn = j < cols ? -1.0 : (j == kClsLanes - 1 ? 1.0 : 0.0);

    // ---- the projected systems of the four classes, B_c = U diag(y_c) [x^e], on the float64 matrix cores -------
    // v_mfma_f64_16x16x4_f64 computes D[16x16] += A[16x4] * B[4x16]; lane l holds A[l%16][l/16], B[l/16][l%16] and, in
    // register t of D, D[4t + l/16][l%16].  With
    //     A[4t + c][k] = U[4b + t][r] * y_{r, class c}      B[k][j] = sgn_j * x_r^{e_j}      (r = 4s + k)
    // summed over the k-steps s, register t of lane (c, j) receives B_c[4b + t][j]: exactly the layout the
    // factorisation below wants (lane = class and column, rows in registers), with no lane exchange at all.
    // Rows past n of Ysh and Pw and columns past n of Ush are zero, so the k-steps need no bound.
    constexpr int kKSteps = NB / 4;
    constexpr int kRowBlocks = ush_rows(RM) / 4;
    static_assert(NB % 4 == 0, "k-steps take four available workers at a time");
    double bop[kKSteps], yop[kKSteps];
    {
        const int k = lane / kClsLanes;
#pragma unroll
        for (int s = 0; s < kKSteps; ++s) {
            const int r = 4 * s + k;
            bop[s] = sgn * Pw[r * kPwStride + e];
            yop[s] = static_cast<double>(ycol[r * CW]);
        }
    }
    double a[RM];
    {
        const double *urow = Ush + ((lane % kClsLanes) >> 2) * ush_stride(NB) + lane / kClsLanes;
        v4d acc[kRowBlocks];
#pragma unroll
        for (int b = 0; b < kRowBlocks; ++b) acc[b] = v4d{0.0, 0.0, 0.0, 0.0};
#pragma unroll
        for (int s = 0; s < kKSteps; ++s)                 // the row blocks are independent accumulation chains
#pragma unroll
            for (int b = 0; b < kRowBlocks; ++b)
                acc[b] = __builtin_amdgcn_mfma_f64_16x16x4f64(urow[4 * b * ush_stride(NB) + 4 * s] * yop[s], bop[s], acc[b],
                                                              0, 0, 0);
#pragma unroll
        for (int b = 0; b < kRowBlocks; ++b)
#pragma unroll
            for (int t = 0; t < 4; ++t)
                if (4 * b + t < RM) a[4 * b + t] = acc[b][t];
    }

    constexpr int kSteps = RM - 1 < kProjMaxM - 1 ? RM - 1 : kProjMaxM - 1;   // most unknowns this tile can hold
    ClassQrSteps<0, kSteps, RM>::run(a, j, cols);

    double q[kSteps];                                     // right-hand side in, Q_1 .. Q_{M-1} out
#pragma unroll
    for (int i = 0; i < kSteps; ++i) q[i] = row_bcast<kClsLanes - 1>(a[i]);
    BackSubst<kSteps - 1, kSteps, RM>::run(a, q, cols);

    // a_r = Q(x_r) = 1 + sum_t q[t] x^(t+1) (q[t] = 0 for t >= cols), rows j, j+16, .. of this lane
    constexpr int PR = (NB + kClsLanes - 1) / kClsLanes;
    double kv[PR];
    int ki[PR];
#pragma unroll
    for (int p = 0; p < PR; ++p) {
        const int r = j + p * kClsLanes;
        const double x = xs[r < n ? r : 0];
        double av = 0.0;
#pragma unroll
        for (int t = kSteps - 1; t >= 0; --t) av = fma(av, x, q[t]);
        av = fma(av, x, 1.0);
        kv[p] = (r < n && av == av) ? fabs(av) : __builtin_inf();
        ki[p] = r;
    }
    // the A smallest |a_r| (equal magnitudes: smaller worker index, i.e. smaller row, first) vote
    for (int pick = 0; pick < A; ++pick) {
        double bv = kv[0];
        int bi = ki[0];
#pragma unroll
        for (int p = 1; p < PR; ++p) {
            const bool take = kv[p] < bv || (kv[p] == bv && ki[p] < bi);
            bv = take ? kv[p] : bv;
            bi = take ? ki[p] : bi;
        }
        row_min_step<kDppQuadXor1>(bv, bi);
        row_min_step<kDppQuadXor2>(bv, bi);
        row_min_step<kDppRowHalfMirror>(bv, bi);
        row_min_step<kDppRowMirror>(bv, bi);
        if (live && j == 0) atomicAdd(&votes[avail[bi]], 1);   // bi < n: at least A < n rows are real
#pragma unroll
        for (int p = 0; p < PR; ++p) {
            if (ki[p] == bi) {
                kv[p] = __builtin_inf();
                ki[p] = 0x7fffffff;
            }
        }
    }
}

__device__ __forceinline__ void homogeneous_q(double *mat, int LD, double *coef, double *key, int W2, int M, int j,
                                              bool live, bool jacobi_only);

constexpr int kInverseRounds = 24;      // inverse-iteration rounds before a class goes to the Jacobi iteration
constexpr int kJacobiSweeps = 30;
constexpr int kRegisterRounds = 64;     // .. and of the register form, whose rounds are cheap next to that fallback

// Smallest right singular vector of the 2M x 2M factor R = [[R_V, B1], [0, R2]] of one class, by inverse iteration
// z <- (R^T R)^-1 z, entirely in the registers of the class's 16-lane row (lane j = index j of both halves of
// z = (p, q), M <= 15).  The four triangular solves of a round,
//     w1 = R_V^-T p,   w2 = R2^-T (q - B1^T w1),   q' = R2^-1 w2,   p' = R_V^-1 (w1 - B1 q'),
// are column sweeps: the entry that has just become final is broadcast along the row (DPP) and every lane subtracts
// its multiple.  The two forward sweeps need the lane's COLUMN of R_V, B1, R2, the two backward ones its ROW; the
// rows of B1 and R2 come through one transposition in the wave's LDS scratch (T: 4 classes x MT x (MT + 1) doubles), those
// of R_V from the group's LDS copy.  Start vector, settling rule, extrapolation of a slowly decaying error mode and
// the floor under vanishing pivots are those of homogeneous_q (the LDS form, which stays the fallback for a class
// that has not settled after kRegisterRounds: it also holds the Jacobi iteration).
//   r2c[i] = R2[i][j] (i <= j), b1c[i] = B1[i][j]: this lane's columns; Rv: LDS, row stride 16.
//   MT >= M bounds the unrolling and the register arrays (the register tile of the kernel bounds M: M <= NB / 2).
// `live`: the row holds a class.  Returns q_j in `qv` and whether the class settled (the same value in all lanes of
// the row).
template <int MT>
__device__ __forceinline__ bool singular_vector_rows(const double (&r2c)[MT], const double (&b1c)[MT],
                                                     const double *Rv, double *T, int M, int j, int cl, bool live,
                                                     double &qv) {
    constexpr int LDT = MT + 1;
    const bool act = j < M;
    double *Tc = T + cl * MT * LDT;                        // M <= MT: lanes j >= MT hold no column and read no row
    // rows of R2 and B1 by transposition through LDS
    double r2r[MT], b1r[MT];
#pragma unroll
    for (int i = 0; i < MT; ++i)
        if (j < MT) Tc[i * LDT + j] = (act && i < M && i <= j) ? r2c[i] : 0.0;
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int k = 0; k < MT; ++k) r2r[k] = Tc[(j < MT ? j : 0) * LDT + k];
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int i = 0; i < MT; ++i)
        if (j < MT) Tc[i * LDT + j] = (act && i < M) ? b1c[i] : 0.0;
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int k = 0; k < MT; ++k) b1r[k] = act ? Tc[j * LDT + k] : 0.0;
    __builtin_amdgcn_wave_barrier();
    // R_V's column and row are read from the group's LDS copy inside the sweeps (they are the same for the wave's
    // four classes); Rv is zero below its diagonal and outside M x M.
    constexpr int LDV = kProjMaxM;
    const double *rv_col = Rv + j;                         // rv_col[i * LDV] = R_V[i][j]
    const double *rv_row = Rv + j * LDV;                   // rv_row[k] = R_V[j][k]
    // reciprocal pivots; a pivot below 1e-24 of its column of R is raised to that (an exactly singular system keeps
    // its null vector to 1e-24, and the solves stay finite)
    double csv = 0.0, cs2 = 0.0;
#pragma unroll
    for (int i = 0; i < MT; ++i) {
        const double rv = rv_col[i * LDV];
        csv = fma(rv, rv, csv);
        cs2 = fma(b1c[i], b1c[i], fma((i < M && i <= j) ? r2c[i] : 0.0, (i < M && i <= j) ? r2c[i] : 0.0, cs2));
    }
    double dv = rv_row[j], d2 = 0.0;
#pragma unroll
    for (int i = 0; i < MT; ++i) d2 = (i == j && i < M) ? r2c[i] : d2;
    const double fv = 1e-24 * sqrt(csv), f2 = 1e-24 * sqrt(cs2);
    if (fabs(dv) < fv) dv = dv < 0.0 ? -fv : fv;
    if (fabs(d2) < f2) d2 = d2 < 0.0 ? -f2 : f2;
    const double rdv = act ? 1.0 / dv : 0.0, rd2 = act ? 1.0 / d2 : 0.0;   // a zero column: inf, the class does not settle
    // strictly upper parts: the multiples a sweep subtracts
#pragma unroll
    for (int i = 0; i < MT; ++i) r2r[i] = (act && i > j) ? r2r[i] : 0.0;
    double r2u[MT];
#pragma unroll
    for (int i = 0; i < MT; ++i) r2u[i] = (act && i < M && i < j) ? r2c[i] : 0.0;

    double p = act ? 1.0 + 0.25 * (j % 3) : 0.0;
    double q = act ? 1.0 + 0.25 * ((M + j) % 3) : 0.0;
    double dd_prev = __builtin_inf();
    int since_jump = 0;
    bool settled = false;
    for (int round = 0; round < kRegisterRounds; ++round) {
        // forward: w1 = R_V^-T p, t = q - B1^T w1, then w2 = R2^-T t
        double s1 = p, t = q;
#pragma unroll
        for (int i = 0; i < MT; ++i) {
            if (i < M) {
                const double wi = row_bcast_dyn(s1 * rdv, i);
                s1 = fma(i < j ? -rv_col[i * LDV] : 0.0, wi, s1);
                t = fma(-b1c[i], wi, t);
            }
        }
        const double w1 = s1 * rdv;
        double s2 = t;
#pragma unroll
        for (int i = 0; i < MT; ++i) {
            if (i < M) {
                const double wi = row_bcast_dyn(s2 * rd2, i);
                s2 = fma(-r2u[i], wi, s2);
            }
        }
        // backward: q' = R2^-1 w2, u = w1 - B1 q', then p' = R_V^-1 u
        double s3 = s2 * rd2, u = w1;
#pragma unroll
        for (int k = MT - 1; k >= 0; --k) {
            if (k < M) {
                const double qk = row_bcast_dyn(s3 * rd2, k);
                s3 = fma(-r2r[k], qk, s3);
                u = fma(-b1r[k], qk, u);
            }
        }
        const double qn_raw = s3 * rd2;
        double s4 = u;
#pragma unroll
        for (int k = MT - 1; k >= 0; --k) {
            if (k < M) {
                const double pk = row_bcast_dyn(s4 * rdv, k);
                s4 = fma(k > j ? -rv_row[k] : 0.0, pk, s4);
            }
        }
        const double pn_raw = s4 * rdv;
        const double nn = row16_sum(act ? fma(pn_raw, pn_raw, qn_raw * qn_raw) : 0.0);
        const double inv = rcp_normal(sqrt_normal(nn));       // nn = 0, inf or NaN: NaN, the class does not settle
        const double pn = act ? pn_raw * inv : 0.0, qn = act ? qn_raw * inv : 0.0;
        const double dp = pn - p, dq = qn - q;                // z' . z > 0 always: no sign to align
        const double dd = row16_sum(fma(dp, dp, dq * dq));
        const double dd_before = dd_prev;
        settled = settled || dd <= 1e-22 || (dd_prev <= 1e-16 && dd >= 0.25 * dd_prev);
        p = pn;
        q = qn;
        dd_prev = dd;
        ++since_jump;
        if (!settled && since_jump >= 3 && dd < 1e-4 && dd_before < __builtin_inf()) {
            const double r = sqrt(dd / dd_before);
            if (r > 0.05 && r < 0.97) {
                p = fma(r / (1.0 - r), dp, pn);
                q = fma(r / (1.0 - r), dq, qn);
                since_jump = 0;
                dd_prev = __builtin_inf();
            }
        }
        if (__all((settled || !live) ? 1 : 0)) break;     // rows without a class (all zeros) never settle: not waited for
    }
    qv = q;
    return settled;
}

// Algorithm 1 (the homogeneous fit, Q_0 free) for the four classes c_rel..c_rel+3 of the staged tile, by one wave, on
// the shared factorisation V = Q [R_V; 0] of the group.  With H_c = [V | diag(y_c) V] (the sign of the second block
// only flips the sign of Q),
//     Q^T H_c = [ R_V   Q1^T diag(y_c) V ]      Q1^T = rows 0..M-1 of Q^T,
//               [  0     U  diag(y_c) V ]      U    = rows M..n-1,
// so the 2M x 2M triangular factor of H_c is [[R_V, B1], [0, R2]] with B1 = Q1^T diag(y_c) V (M x M) and
// R2 the triangular factor of B2 = U diag(y_c) V ((n-M) x M; n - M >= M by eq. (3)).  B1 and B2 come from the
// float64 matrix cores exactly as the projected system of Algorithm 2 does (Q1 sits in the 16 rows that follow U in
// LDS), R2 from the same register Householder QR, run over all M columns.  The smallest right singular vector of
// the assembled factor is found in registers (singular_vector_rows); a class that does not settle there is assembled
// in this wave's scratch, mat[2M][2M+1] | coef[M] | key[n], and goes through the LDS form (homogeneous_q), as many
// classes at a time as the scratch holds (one, as the host sizes it).
template <int NB, int RM>
__device__ __forceinline__ void locate_classes_hom_proj(const float *Ysh, int CW, int c_rel, int tile_classes,
                                                        const int *avail, const double *xs, const double *Pw,
                                                        const double *Ush, const double *Rv, int n, int M, int A,
                                                        double *scratch, int scratch_doubles, int *votes) {
    typedef double v4d __attribute__((ext_vector_type(4)));
    const int lane = lane_id();
    const int j = lane % kClsLanes;
    const int e = j < M ? j : 0;                          // column of this lane: y x^j; idle lanes hold zeros
    const double sgn = j < M ? 1.0 : 0.0;
    constexpr int MT = hom_mt(NB);
    constexpr int kKSteps = NB / 4;
    constexpr int kUBlocks = ush_rows(RM) / 4;
    constexpr int kBlocks = kUBlocks + (MT + 3) / 4;      // then the rows of Q1 (16 of them in LDS, the first MT used)
    double bop[kKSteps], yop[kKSteps];
    {
        const int k = lane / kClsLanes, cm = (lane % kClsLanes) & 3;
#pragma unroll
        for (int s = 0; s < kKSteps; ++s) {
            const int r = 4 * s + k;
            bop[s] = sgn * Pw[r * kPwStride + e];
            yop[s] = static_cast<double>(Ysh[r * CW + c_rel + cm]);
        }
    }
    double a[RM], b1[MT];
    {
        const double *urow = Ush + ((lane % kClsLanes) >> 2) * ush_stride(NB) + lane / kClsLanes;
        v4d acc[kBlocks];
#pragma unroll
        for (int b = 0; b < kBlocks; ++b) acc[b] = v4d{0.0, 0.0, 0.0, 0.0};
#pragma unroll
        for (int s = 0; s < kKSteps; ++s)
#pragma unroll
            for (int b = 0; b < kBlocks; ++b)
                acc[b] = __builtin_amdgcn_mfma_f64_16x16x4f64(urow[4 * b * ush_stride(NB) + 4 * s] * yop[s], bop[s], acc[b],
                                                              0, 0, 0);
#pragma unroll
        for (int b = 0; b < kUBlocks; ++b)
#pragma unroll
            for (int t = 0; t < 4; ++t)
                if (4 * b + t < RM) a[4 * b + t] = acc[b][t];
#pragma unroll
        for (int i = 0; i < MT; ++i) b1[i] = acc[kUBlocks + i / 4][i % 4];
    }

    // R2: steps 0 .. min(M, RM - 1) - 1; when M == RM the last diagonal entry is the one row that is left
    constexpr int kSteps = RM - 1 < kProjMaxM - 1 ? RM - 1 : kProjMaxM - 1;
    ClassQrSteps<0, kSteps, RM>::run(a, j, M);

    // ---- the singular vector: in registers; classes that do not settle there go through the LDS form below ---------
    const int cl16 = lane / kClsLanes;                    // class slot of this lane in the register layout
    double r2c[MT];
#pragma unroll
    for (int i = 0; i < MT; ++i) r2c[i] = i < RM ? a[i < RM ? i : 0] : 0.0;
    double qv;
    const bool class_live = c_rel + cl16 < tile_classes;
    const bool settled = singular_vector_rows<MT>(r2c, b1, Rv, scratch, M, j, cl16, class_live, qv);
    // a_r = Q(x_r) = sum_k q_k x_r^k, rows j, j+16, .. of this lane; the A smallest |a_r| vote
    {
        double qk[MT];
#pragma unroll
        for (int k = 0; k < MT; ++k) qk[k] = row_bcast_dyn(qv, k);              // zero from idle lanes
        constexpr int PR = (NB + kClsLanes - 1) / kClsLanes;
        double kv[PR];
        int ki[PR];
#pragma unroll
        for (int pr = 0; pr < PR; ++pr) {
            const int r = j + pr * kClsLanes;
            const double x = xs[r < n ? r : 0];
            double av = 0.0;
#pragma unroll
            for (int k = MT - 1; k >= 0; --k) av = fma(av, x, qk[k]);
            kv[pr] = (r < n && av == av) ? fabs(av) : __builtin_inf();
            ki[pr] = r;
        }
        for (int pick = 0; pick < A; ++pick) {
            double bv = kv[0];
            int bi = ki[0];
#pragma unroll
            for (int pr = 1; pr < PR; ++pr) {
                const bool take = kv[pr] < bv || (kv[pr] == bv && ki[pr] < bi);
                bv = take ? kv[pr] : bv;
                bi = take ? ki[pr] : bi;
            }
            row_min_step<kDppQuadXor1>(bv, bi);
            row_min_step<kDppQuadXor2>(bv, bi);
            row_min_step<kDppRowHalfMirror>(bv, bi);
            row_min_step<kDppRowMirror>(bv, bi);
            if (class_live && settled && j == 0) atomicAdd(&votes[avail[bi]], 1);
#pragma unroll
            for (int pr = 0; pr < PR; ++pr) {
                if (ki[pr] == bi) {
                    kv[pr] = __builtin_inf();
                    ki[pr] = 0x7fffffff;
                }
            }
        }
    }
    const unsigned long long open_lanes = __ballot(class_live && !settled);
    if (open_lanes == 0ull) return;

    // ---- fallback: assemble the factor in LDS and find the vector there (inverse iteration again, then Jacobi) -----
    const int W2 = 2 * M;
    const int LD = W2 + 1;
    const int per_class = W2 * LD + M + n;
    const int fit = scratch_doubles / per_class;          // >= 1 (hom_scratch_doubles)
    const int cpw = kWave / W2 < fit ? kWave / W2 : fit;  // classes per pass: what the lanes and the scratch hold
    const int clw = lane / W2, jw = lane - clw * W2;      // the layout of homogeneous_q (lane jw owns row jw)
    __builtin_amdgcn_wave_barrier();                      // the transposition scratch is free again
    for (int p0 = 0; p0 < kClsPerWave; p0 += cpw) {
        if (cl16 >= p0 && cl16 < p0 + cpw && j < M) {
            double *mat = scratch + (cl16 - p0) * per_class;
#pragma unroll
            for (int i = 0; i < MT; ++i) {
                if (i < M) {
                    mat[i * LD + j] = Rv[i * kProjMaxM + j];                    // R_V (zero below its diagonal)
                    mat[(M + i) * LD + j] = 0.0;
                    mat[i * LD + M + j] = b1[i];                                // B1
                    mat[(M + i) * LD + M + j] = (i <= j) ? r2c[i] : 0.0;        // R2
                }
            }
        }
        __builtin_amdgcn_wave_barrier();
        const bool in_pass = clw < cpw && p0 + clw < kClsPerWave;
        const bool live = in_pass && ((open_lanes >> ((p0 + (in_pass ? clw : 0)) * kClsLanes)) & 1ull) != 0ull;
        double *mat = scratch + (live ? clw : 0) * per_class;
        double *coef = mat + W2 * LD;
        double *key = coef + M;
        homogeneous_q(mat, LD, coef, key, W2, M, jw, live, true);
        if (live) {
            for (int r = jw; r < n; r += W2) {            // a_r = Q(x_r), Q_k = coef[k]
                const double x = xs[r];
                double av = 0.0;
                for (int t = M - 1; t >= 0; --t) av = fma(av, x, coef[t]);
                key[r] = (av != av) ? __builtin_inf() : fabs(av);
            }
        }
        __builtin_amdgcn_wave_barrier();
        if (live) pick_and_vote(key, avail, n, A, jw, W2, votes);
        __builtin_amdgcn_wave_barrier();
    }
}

// Per-wave LDS scratch of Algorithm 1's locator: the transposition tiles of singular_vector_rows (4 classes x MT x
// (MT + 1)) or, for a class that falls back to homogeneous_q, ONE assembled factor with its coefficient and key
// arrays.  Kept this small on purpose: LDS, not registers, decides how many groups a CU holds (at K = 8, A = 2 with
// three factors per wave seven workgroups fitted a CU where eight were due, and the launch took two rounds).
__host__ __device__ constexpr int hom_scratch_doubles(int M, int n_cap, int MT) {
    const int fallback = 2 * M * (2 * M + 1) + M + n_cap;
    const int transpose = kClsPerWave * MT * (MT + 1);
    return fallback > transpose ? fallback : transpose;
}

// Doubles of the shared factorisation as the kernel keeps it in LDS (and as full_basis_kernel writes it out):
// Ush[ush_rows(RM)][ush_stride(NB)], and for Algorithm 1's locator also Q1sh[16][ush_stride(NB)] | Rv[16][16].
template <int NB, int RM, bool HOMOG>
constexpr int basis_doubles() {
    return ush_rows(RM) * ush_stride(NB) + (HOMOG ? kProjMaxM * ush_stride(NB) + kProjMaxM * kProjMaxM : 0);
}

// HOMOG: Algorithm 1's fit as the per-class locator (locate_classes_hom_proj) instead of Algorithm 2's.
// dynamic LDS (doubles): basis (see basis_doubles) | Pw[NB*16] | xs[NB] | WdT[(n_cap-A)*KP] | alpha_s[K] | beta_s[N]
//               | HOMOG: scratch[nw][hom_scratch_doubles(M, n_cap, NB / 2)]
//               then float Ysh[NB*CW], then ints: avail[N] | F[N] | Fpos[N] | votes[N] | n | flag
template <int NB, int RM, bool HOMOG>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(!HOMOG && RM <= 16 && NB <= 28 ? 3 : 2))) void decode_byzantine_proj_kernel(
    const float *__restrict__ preds, const uint8_t *__restrict__ mask, float *__restrict__ out,
    int32_t *__restrict__ adv, int32_t *__restrict__ status, int K, int N, int S, int A, int64_t C, int64_t Cv,
    int vec4, int sign_mode, int n_cap, int cw_log2, int splits, int32_t *__restrict__ workspace,
    const double *__restrict__ full_basis, const Nodes nodes) {
    extern __shared__ __align__(16) double lds_d[];
    const int KP = round_up4(K);
    const int M = K + A;
    const int nw = blockDim.x / kWave;
    const int CW = 1 << cw_log2;                          // classes per staged tile (16, 32 or 64)
    double *Ush = lds_d;
    constexpr int kUshDoubles = basis_doubles<NB, RM, HOMOG>();
    double *Q1sh = Ush + ush_rows(RM) * ush_stride(NB);   // HOMOG only: the 16 rows after U, then R_V
    double *Rv = Q1sh + kProjMaxM * ush_stride(NB);
    double *Pw = Ush + kUshDoubles;
    double *xs = Pw + NB * kPwStride;
    double *WdT = xs + NB;
    double *alpha_s = WdT + (n_cap - A) * KP;
    double *beta_s = alpha_s + K;
    const int hom_wave_doubles = HOMOG ? hom_scratch_doubles(M, n_cap, hom_mt(NB)) : 0;
    double *hom_scratch = beta_s + N;
    float *Ysh = reinterpret_cast<float *>(hom_scratch + static_cast<size_t>(nw) * hom_wave_doubles);
    int *avail = reinterpret_cast<int *>(Ysh + NB * CW);
    int *F = avail + N;
    int *Fpos = F + N;
    int *votes = Fpos + N;
    int *n_sh = votes + N;

    // splits > 1: `splits` workgroups share a group, workgroup `part` taking the class tiles part, part + splits, ..
    const int64_t g = blockIdx.x / splits;
    const int part = static_cast<int>(blockIdx.x - g * splits);
    const int wv = wave_id();
    const int tid = threadIdx.x;
    const float *pg = preds + static_cast<size_t>(g) * N * C;

    stage_nodes(nodes, K, N, alpha_s, beta_s);
    for (int e = tid; e < (n_cap - A) * KP; e += blockDim.x) WdT[e] = 0.0;
    for (int e = tid; e < N; e += blockDim.x) votes[e] = 0;
    if (wv == 0) {
        const int cnt = survivors_from_mask(mask + g * N, N, avail);
        if (lane_id() == 0) *n_sh = cnt;
    }
    __syncthreads();
    const int n = *n_sh;
    const bool good = S < 0 ? (n >= 2 * M && n <= n_cap) : n == n_cap;
    if (tid == 0 && status != nullptr) status[g] = good ? APPROXIFER_GROUP_OK : APPROXIFER_GROUP_BAD_MASK;
    if (!good) return;
    // A group in which every worker answered has the node set of the whole call: its complement basis was
    // factorised once, ahead of this launch (full_basis_kernel), and is only copied here.
    const bool preloaded = full_basis != nullptr && n == N;
    for (int e = tid; e < kUshDoubles; e += blockDim.x) Ush[e] = preloaded ? full_basis[e] : 0.0;

    // first class tile: the loads are issued now and land in LDS after the shared factorisation
    constexpr int kPrefetch = 8;
    const int64_t cb_first = static_cast<int64_t>(part) * CW;
    const int slots = NB * CW;                            // slot = (row r, class c) = (slot >> cw_log2, slot & (CW-1))
    float pf[kPrefetch];
#pragma unroll
    for (int u = 0; u < kPrefetch; ++u) {
        const int slot = tid + u * blockDim.x;
        const int r = slot >> cw_log2, c = slot & (CW - 1);
        pf[u] = (slot < slots && r < n && cb_first + c < C) ? pg[static_cast<size_t>(avail[r]) * C + cb_first + c] : 0.0f;
    }

    // powers of the available workers' nodes, x^e by repeated multiplication; rows past n are zero
    for (int r = tid; r < NB; r += blockDim.x) {
        const double x = r < n ? beta_s[avail[r]] : 0.0;
        if (r < n) xs[r] = x;
        double p = r < n ? 1.0 : 0.0;
        for (int e = 0; e < kPwStride; ++e) {
            Pw[r * kPwStride + e] = p;
            p *= x;
        }
    }
    __syncthreads();
    if (wv == 0 && !preloaded) shared_complement_basis<NB, RM, HOMOG>(Pw, n, M, Ush, Q1sh, Rv);

    for (int64_t cb = cb_first; cb < C; cb += static_cast<int64_t>(splits) * CW) {   // class tiles of this part
        if (cb == cb_first) {
#pragma unroll
            for (int u = 0; u < kPrefetch; ++u) {
                const int slot = tid + u * blockDim.x;
                if (slot < slots) Ysh[slot] = pf[u];
            }
            for (int slot = tid + kPrefetch * blockDim.x; slot < slots; slot += blockDim.x) {
                const int r = slot >> cw_log2, c = slot & (CW - 1);
                Ysh[slot] = (r < n && cb + c < C) ? pg[static_cast<size_t>(avail[r]) * C + cb + c] : 0.0f;
            }
        } else {
            __syncthreads();                              // every wave is done with the previous tile
            for (int slot = tid; slot < slots; slot += blockDim.x) {
                const int r = slot >> cw_log2, c = slot & (CW - 1);
                Ysh[slot] = (r < n && cb + c < C) ? pg[static_cast<size_t>(avail[r]) * C + cb + c] : 0.0f;
            }
        }
        __syncthreads();
        const int tile_classes = (C - cb < CW) ? static_cast<int>(C - cb) : CW;
        for (int c_rel = wv * kClsPerWave; c_rel < tile_classes; c_rel += nw * kClsPerWave) {
            if (HOMOG)
                locate_classes_hom_proj<NB, RM>(Ysh, CW, c_rel, tile_classes, avail, xs, Pw, Ush, Rv, n, M, A,
                                                hom_scratch + static_cast<size_t>(wv) * hom_wave_doubles, hom_wave_doubles,
                                                votes);
            else
                locate_classes_proj<NB, RM>(Ysh + c_rel + ((lane_id() % kClsLanes) & 3), CW,
                                            c_rel + lane_id() / kClsLanes < tile_classes, avail, xs, Pw, Ush, n, M, A, votes);
        }
    }
    __syncthreads();

    float *og = out + static_cast<size_t>(g) * K * C;
    if (splits > 1 && !pool_votes_last_arrival(workspace + g * (N + 1), votes, N, splits, n_sh + 1)) return;
    const bool staged = C <= CW;                          // the one tile holds every prediction of the group
    select_adversaries(adv + g * A, avail, n, N, A, votes, F, Fpos);
    const int nF = n - A;
    decoder_weights(alpha_s, beta_s, F, nF, K, KP, sign_mode, WdT);
    __syncthreads();
    if (staged) {
        // out[j][c] = sum_r WdT[r][j] * Y[F_r][c] straight from the staged tile
        const int Ci = static_cast<int>(C);
        for (int o = tid; o < K * Ci; o += blockDim.x) {
            const int jq = o / Ci, c = o - jq * Ci;
            double acc = 0.0;
#pragma unroll 6
            for (int r = 0; r < nF; ++r)
                acc = fma(WdT[r * KP + jq], static_cast<double>(Ysh[(Fpos[r] << cw_log2) + c]), acc);
            og[o] = static_cast<float>(acc);
        }
    } else if (vec4) {
        contract_group<4>(pg, og, F, nF, K, KP, C, Cv, WdT);
    } else {
        contract_group<1>(pg, og, F, nF, K, KP, C, Cv, WdT);
    }
}

// Algorithm 2 for the paper's Byzantine operating points (Section 4.2, "Byzantine-Robustness": no stragglers, ten
// classes): every group answers in full, so all groups share the factorisation that full_basis_kernel wrote, and
// nothing ties a wave's four class slots to one group any more.  A workgroup takes GPW consecutive groups and walks
// their GPW * C classes four at a time: with C = 10 four groups fill ten rounds where each alone needs three (twelve
// slots for ten classes); nodes, powers and the basis are staged once for all of them.  Per class the arithmetic is
// that of decode_byzantine_proj_kernel (same functions, same operands in the same order): the outputs are the same bits.
// Host guarantees: S = 0 (a group whose mask is not full is marked bad and skipped), C <= 16, N <= 48.
// dynamic LDS (doubles): Ush | Pw[NB*16] | xs[NB] | WdT[GPW][(N-A)*KP] | alpha_s[K] | beta_s[N]
//               then float Ysh[GPW + 1][NB*16] (the last tile stays zero: empty class slots read it),
//               then ints: ident[N] | F[GPW][N] | Fpos[GPW][N] | votes[GPW][N] | good[GPW]
template <int NB, int RM, int GPW>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(RM <= 16 && NB <= 28 ? 3 : 2))) void decode_byzantine_shared_basis_kernel(
    const float *__restrict__ preds, const uint8_t *__restrict__ mask, float *__restrict__ out,
    int32_t *__restrict__ adv, int32_t *__restrict__ status, int64_t G, int K, int N, int A, int C, int sign_mode,
    const double *__restrict__ full_basis, const Nodes nodes) {
    extern __shared__ __align__(16) double lds_d[];
    constexpr int CW = kClsLanes;                         // staged tile: sixteen class columns per row
    constexpr int kTile = NB * CW;
    constexpr int kUshDoubles = basis_doubles<NB, RM, false>();
    const int KP = round_up4(K);
    const int M = K + A;
    const int nF = N - A;
    const int nw = blockDim.x / kWave;
    double *Ush = lds_d;
    double *Pw = Ush + kUshDoubles;
    double *xs = Pw + NB * kPwStride;
    double *WdT = xs + NB;
    double *alpha_s = WdT + GPW * nF * KP;
    double *beta_s = alpha_s + K;
    float *Ysh = reinterpret_cast<float *>(beta_s + N);
    int *ident = reinterpret_cast<int *>(Ysh + (GPW + 1) * kTile);
    int *F = ident + N;
    int *Fpos = F + GPW * N;
    int *votes = Fpos + GPW * N;
    int *good_sh = votes + GPW * N;
    const int64_t g0 = static_cast<int64_t>(blockIdx.x) * GPW;
    const int here = G - g0 < GPW ? static_cast<int>(G - g0) : GPW;   // groups of this workgroup
    const int tid = threadIdx.x;
    const int wv = wave_id();
    const int lane = lane_id();

    stage_nodes(nodes, K, N, alpha_s, beta_s);
    for (int e = tid; e < GPW * nF * KP; e += blockDim.x) WdT[e] = 0.0;
    for (int e = tid; e < GPW * N; e += blockDim.x) votes[e] = 0;
    for (int e = tid; e < N; e += blockDim.x) ident[e] = e;
    for (int e = tid; e < (GPW + 1) * kTile; e += blockDim.x) Ysh[e] = 0.0f;
    for (int e = tid; e < kUshDoubles; e += blockDim.x) Ush[e] = full_basis[e];
    for (int q = wv; q < GPW; q += nw) {                  // N <= 48: one ballot counts a mask row
        bool ok = q < here;
        if (ok) {
            const bool b = lane < N && mask[(g0 + q) * N + lane] != 0;
            ok = static_cast<int>(__popcll(__ballot(b))) == N;
            if (lane == 0 && status != nullptr) status[g0 + q] = ok ? APPROXIFER_GROUP_OK : APPROXIFER_GROUP_BAD_MASK;
        }
        if (lane == 0) good_sh[q] = ok ? 1 : 0;
    }
    __syncthreads();
    for (int r = tid; r < NB; r += blockDim.x) {
        const double x = r < N ? beta_s[r] : 0.0;
        if (r < N) xs[r] = x;
        double pw = r < N ? 1.0 : 0.0;
        for (int e = 0; e < kPwStride; ++e) {
            Pw[r * kPwStride + e] = pw;
            pw *= x;
        }
    }
    // the predictions of the workgroup's groups are one contiguous run of here * N * C floats
    {
        const float *pg = preds + static_cast<size_t>(g0) * N * C;
        const int per_group = N * C;
        for (int idx = tid; idx < here * per_group; idx += blockDim.x) {
            const int q = idx / per_group, rem = idx - q * per_group;
            const int r = rem / C, c = rem - r * C;
            if (good_sh[q] != 0) Ysh[q * kTile + r * CW + c] = pg[idx];
        }
    }
    __syncthreads();

    const int total = GPW * C;
    for (int c0 = wv * kClsPerWave; c0 < total; c0 += nw * kClsPerWave) {
        const int s_op = c0 + ((lane % kClsLanes) & 3);   // the slot whose predictions this lane feeds to the matrix cores
        const int q_op = s_op / C, c_op = s_op - q_op * C;
        const bool op_ok = s_op < total && good_sh[s_op < total ? q_op : 0] != 0;
        const int s_res = c0 + lane / kClsLanes;          // the slot whose system this lane's row then holds
        const int q_res = s_res < total ? s_res / C : 0;
        const bool live = s_res < total && good_sh[q_res] != 0;
        locate_classes_proj<NB, RM>(Ysh + (op_ok ? q_op * kTile + c_op : GPW * kTile), CW, live, ident, xs, Pw, Ush, N, M,
                                    A, votes + q_res * N);
    }
    __syncthreads();

    for (int q = wv; q < here; q += nw)                   // a wave per group
        if (good_sh[q] != 0)
            select_adversaries_wave(adv + (g0 + q) * A, ident, N, N, A, votes + q * N, F + q * N, Fpos + q * N);
    __syncthreads();
    for (int q = 0; q < here; ++q)
        if (good_sh[q] != 0) decoder_weights(alpha_s, beta_s, F + q * N, nF, K, KP, sign_mode, WdT + q * nF * KP);
    __syncthreads();
    // out[g][j][c] = sum_r WdT[r][j] * Y[F_r][c] straight from the staged tiles
    {
        float *og = out + static_cast<size_t>(g0) * K * C;
        const int per_group = K * C;
        for (int o = tid; o < here * per_group; o += blockDim.x) {
            const int q = o / per_group, rem = o - q * per_group;
            if (good_sh[q] == 0) continue;
            const int jq = rem / C, c = rem - jq * C;
            const double *w = WdT + q * nF * KP + jq;
            const float *y = Ysh + q * kTile + c;
            const int *fp = Fpos + q * N;
            double acc = 0.0;
#pragma unroll 6
            for (int r = 0; r < nF; ++r) acc = fma(w[r * KP], static_cast<double>(y[fp[r] << 4]), acc);
            og[o] = static_cast<float>(acc);
        }
    }
}

// The complement basis of the node set of ALL N workers, once per call, for the groups whose mask is full (the
// paper's Byzantine experiments have no stragglers: every group then shares this one factorisation).  One wave;
// writes Ush as the kernel above lays it out, ush_rows(RM) * ush_stride(NB) doubles, to `basis`.
template <int NB, int RM, bool HOMOG>
__global__ __launch_bounds__(kWave) void full_basis_kernel(double *__restrict__ basis, int N, int M, const Nodes nodes) {
    constexpr int kUshDoubles = basis_doubles<NB, RM, HOMOG>();
    __shared__ double Ush[kUshDoubles];
    __shared__ double Pw[NB * kPwStride];
    const int tid = threadIdx.x;
    for (int e = tid; e < kUshDoubles; e += kWave) Ush[e] = 0.0;
    for (int r = tid; r < NB; r += kWave) {
        const double x = r < N ? nodes.beta[r] : 0.0;
        double p = r < N ? 1.0 : 0.0;
        for (int e = 0; e < kPwStride; ++e) {
            Pw[r * kPwStride + e] = p;
            p *= x;
        }
    }
    __syncthreads();
    shared_complement_basis<NB, RM, HOMOG>(Pw, N, M, Ush, Ush + ush_rows(RM) * ush_stride(NB),
                                           Ush + (ush_rows(RM) + kProjMaxM) * ush_stride(NB));
    __syncthreads();
    for (int e = tid; e < kUshDoubles; e += kWave) basis[e] = Ush[e];
}

// ------------------------------------------------------------------------------------------------
// general kernel: the full system per class, in LDS
// ------------------------------------------------------------------------------------------------
// Algorithm 1's fit needs a null vector of the homogeneous system: the right singular vector of the smallest
// singular value of its triangular factor R (rows 0..W2-1 of mat, row stride LD, lane j owns row j).  Writes the Q
// half of that vector to coef[0..M-1] (coefficients of columns M..W2-1); its length and sign are immaterial.
//
//  1. Inverse iteration z <- (R^T R)^-1 z, two triangular solves per round.  When the data are rational up to
//     rounding -- the case the locator is built for -- the smallest singular value is orders of magnitude below the
//     next and two to four rounds settle z: successive iterates within 1e-11, or no longer approaching each other.
//     A steady slow decay (two close smallest singular values) is extrapolated to its limit, Aitken's way.
//  2. Classes that have not settled after kInverseRounds (no gap: data that fit no rational function; or a zero on
//     the diagonal) get the full answer from one-sided Jacobi on G = R^T: lane j owns column j of G, which is row j
//     of mat; a step rotates W2/2 disjoint pairs of columns (round-robin pairing, W2 - 1 steps per sweep) until all
//     are orthogonal to rounding; the columns then are sigma_i v_i, v_i the right singular vectors of R, and the
//     shortest is the one wanted.  Both lanes of a pair read both columns and write their own: the new value of
//     element t depends on both reads of element t, and the lanes of a wave run in lock step, so no lane sees a
//     half-rotated pair.
// jacobi_only (wave-uniform): the caller's own inverse iteration has already failed to settle; go to step 2.
__device__ __forceinline__ void homogeneous_q(double *mat, int LD, double *coef, double *key, int W2, int M, int j,
                                              bool live, bool jacobi_only = false) {
    double *own = mat + j * LD;
    // ---- 1. inverse iteration; R mirrored into the lower triangle so that both solves read rows ----------------
    double colsq = 0.0;                                   // |column j of R|^2 = |column j of the system|^2
    for (int t = 0; t <= j; ++t) colsq = fma(mat[t * LD + j], mat[t * LD + j], colsq);
    if (live) {
        for (int t = 0; t < j; ++t) own[t] = mat[t * LD + j];
        // An exactly singular system (K = 1: the good workers return one and the same number) leaves a zero on the
        // diagonal.  Its null vector is the answer, but a zero pivot stops the solves and, in the Jacobi fallback, a
        // zero singular value wipes out its own vector (the columns there are sigma_i v_i).  A pivot below 1e-24 of
        // its column is raised to that: the null vector moves by 1e-24, far below the rounding of everything else.
        const double floor = 1e-24 * sqrt(colsq);
        if (fabs(own[j]) < floor) own[j] = own[j] < 0.0 ? -floor : floor;
    }
    __builtin_amdgcn_wave_barrier();
    const double rd = 1.0 / own[j];                     // still zero (a zero column): nothing settles, nor matters
    double z = 1.0 + 0.25 * (j % 3);
    double dd_prev = __builtin_inf();
    int since_jump = 0;
    bool settled = false;
    for (int round = jacobi_only ? kInverseRounds : 0; round < kInverseRounds; ++round) {
        double s = z;                                     // R^T w = z, forward
        for (int t = 0; t < W2; ++t) {
            const double rtj = mat[t * LD + j];           // issued ahead of the write -> read chain through key
            if (live && j == t) key[t] = s * rd;
            __builtin_amdgcn_wave_barrier();
            const double wt = key[t];
            if (j > t) s = fma(-rtj, wt, s);
        }
        __builtin_amdgcn_wave_barrier();
        s = key[j];                                       // R z' = w, backward
        for (int t = W2 - 1; t >= 0; --t) {
            const double rjt = mat[t * LD + j];           // the mirrored R[j][t]
            if (live && j == t) key[t] = s * rd;
            __builtin_amdgcn_wave_barrier();
            const double zt = key[t];
            if (j < t) s = fma(-rjt, zt, s);
        }
        __builtin_amdgcn_wave_barrier();
        double nn = 0.0;
        for (int t = 0; t < W2; ++t) nn = fma(key[t], key[t], nn);
        const double zn = key[j] * rcp_normal(sqrt_normal(nn));   // nn = 0, inf or NaN: NaN, and the class goes to Jacobi
        const double dz = zn - z;                         // z' . z > 0 always: no sign to align
        __builtin_amdgcn_wave_barrier();
        if (live) key[j] = dz * dz;
        __builtin_amdgcn_wave_barrier();
        double dd = 0.0;
        for (int t = 0; t < W2; ++t) dd += key[t];
        __builtin_amdgcn_wave_barrier();
        const double dd_before = dd_prev;
        // settled: the step is below 1e-11, or it has stopped shrinking at the level rounding allows (false for NaN)
        settled = settled || dd <= 1e-22 || (dd_prev <= 1e-16 && dd >= 0.25 * dd_prev);
        z = zn;
        dd_prev = dd;
        // Two close smallest singular values leave one slowly decaying error mode: z_k = v + r^k e.  Once the steps are
        // small and shrink by a steady factor r, jump to the limit of that sequence, z + r/(1-r) (z - z_previous); the
        // next two steps are no longer part of it, so at most every third round.
        ++since_jump;
        if (!settled && since_jump >= 3 && dd < 1e-4 && dd_before < __builtin_inf()) {
            const double r = sqrt(dd / dd_before);
            if (r > 0.05 && r < 0.97) {
                z = fma(r / (1.0 - r), dz, zn);
                since_jump = 0;
                dd_prev = __builtin_inf();
            }
        }
        if (__all((settled || !live) ? 1 : 0)) break;
    }
    if (live && settled && j >= M) coef[j - M] = z;
    const bool need = live && !settled;
    if (!__any(need ? 1 : 0)) {
        __builtin_amdgcn_wave_barrier();
        return;
    }

    // ---- 2. one-sided Jacobi for the classes that did not settle ----------------------------------------------
    if (need)
        for (int t = 0; t < j; ++t) own[t] = 0.0;
    __builtin_amdgcn_wave_barrier();
    const int m = W2 - 1;
    const double tol2 = (W2 * 2.220446049250313e-16) * (W2 * 2.220446049250313e-16);
    for (int sweep = 0; sweep < kJacobiSweeps; ++sweep) {
        bool rotated = false;
        for (int s = 0; s < m; ++s) {
            int k;                                        // this lane's partner: lane m plays s, the others mirror about s
            if (j == m) {
                k = s;
            } else if (j == s) {
                k = m;
            } else {
                k = 2 * s - j;
                if (k < 0) k += m;
                if (k >= m) k -= m;
            }
            const double *oth = mat + k * LD;
            double al = 0.0, be = 0.0, ga = 0.0;
            if (need) {
#pragma unroll 4
                for (int t = 0; t < W2; ++t) {
                    const double a = own[t], b = oth[t];
                    al = fma(a, a, al);
                    be = fma(b, b, be);
                    ga = fma(a, b, ga);
                }
            }
            const bool first = j < k;                     // the pair is (p, q), p < q; both lanes compute the same angle
            const double ap = first ? al : be, aq = first ? be : al;
            // rotate unless |g_p . g_q| <= tol |g_p| |g_q| (also skipped: NaN, and products that underflow to zero)
            const bool rot = need && ga * ga > tol2 * (ap * aq);
            if (rot) {
                // zeta = cot(2 phi), clamped so that its square stays finite (beyond 1e150 the rotation is the identity
                // to more digits than a double holds)
                const double zeta = fmin(fmax((aq - ap) * rcp_normal(2.0 * ga), -1e150), 1e150);
                const double tn = (zeta >= 0.0 ? 1.0 : -1.0) * rcp_normal(fabs(zeta) + sqrt_normal(fma(zeta, zeta, 1.0)));
                const double cs = rcp_normal(sqrt_normal(fma(tn, tn, 1.0)));
                const double so = first ? -cs * tn : cs * tn;      // g_p' = c g_p - s g_q,  g_q' = s g_p + c g_q
#pragma unroll 4
                for (int t = 0; t < W2; ++t) own[t] = fma(so, oth[t], cs * own[t]);
                rotated = true;
            }
            __builtin_amdgcn_wave_barrier();
        }
        if (!__any(rotated ? 1 : 0)) break;
    }
    double nrm = 0.0;
    for (int t = 0; t < W2; ++t) nrm = fma(own[t], own[t], nrm);
    if (need) key[j] = (nrm == nrm) ? nrm : __builtin_inf();
    __builtin_amdgcn_wave_barrier();
    int jmin = 0;
    double best = key[0];
    for (int t = 1; t < W2; ++t) {
        const double v = key[t];
        if (v < best) {
            best = v;
            jmin = t;
        }
    }
    if (need && j >= M) coef[j - M] = mat[jmin * LD + j];
    __builtin_amdgcn_wave_barrier();                      // key is reused by the caller
}

// Algorithm 2, steps 1-2, for one class: row r of the n x 2M matrix  [x^0 .. x^(M-1) | -y x^1 .. -y x^(M-1) | y]
// (the last column is the right-hand side), written by lane j of the class's `width` lanes for rows j, j+width, ..
__device__ __forceinline__ void build_class_system(const float *__restrict__ pg, int64_t C, int64_t c, const int *avail,
                                                   const double *xs, int n, int M, double *mat, int LD, int j, int width,
                                                   bool live) {
    if (live) {
        for (int r = j; r < n; r += width) {
            const double x = xs[r];
            const double y = static_cast<double>(pg[static_cast<size_t>(avail[r]) * C + c]);
            double *row = mat + r * LD;
            double p = 1.0;
            for (int k = 0; k < M; ++k) {
                row[k] = p;                               // x^k
                if (k >= 1) row[M - 1 + k] = -y * p;      // -y x^k
                p *= x;
            }
            row[2 * M - 1] = y;
        }
    }
    __builtin_amdgcn_wave_barrier();
}

// Householder QR in least-squares form, one lane per column: step k reflects column k onto e_k over rows k..n-1
// and applies the reflector to the columns right of it (and to the right-hand side).
__device__ __forceinline__ void factor_class_system(double *mat, int LD, int n, int j, int qr_steps, bool live) {
    for (int k = 0; k < qr_steps; ++k) {
        double sigma = 0.0, d = 0.0;
#pragma unroll 4
        for (int r = k; r < n; ++r) {
            const double vr = mat[r * LD + k];            // broadcast inside the class
            const double arj = mat[r * LD + j];
            sigma = fma(vr, vr, sigma);
            d = fma(vr, arj, d);
        }
        const double xkk = mat[k * LD + k];
        const double akj = mat[k * LD + j];
        const Reflector h = reflector(sigma, d, xkk, akj);
        __builtin_amdgcn_wave_barrier();
        if (live && !h.degenerate) {
            if (j > k) {
#pragma unroll 4
                for (int r = k; r < n; ++r) {
                    const double vr = (r == k) ? xkk - h.alpha : mat[r * LD + k];
                    mat[r * LD + j] = fma(-h.f, vr, mat[r * LD + j]);
                }
            } else if (j == k) {
                mat[k * LD + k] = h.alpha;                // R[k][k]
            }
        }
        __builtin_amdgcn_wave_barrier();
    }
}

// Algorithm 2, steps 1-5, for the classes c0 .. c0+cpw-1 of one group, by one wave.
//   n        available workers (rows), M = K + A, W2 = 2M columns including the right-hand side
//   xs[n]    worker nodes of the available workers (LDS, shared by the workgroup)
//   scratch  this wave's LDS: per class  mat[n][W2] | coef[M] | key[n]
// Lane (cl, j) = (lane / W2, lane % W2) works on class c0 + cl; lanes beyond cpw classes idle.
// HOMOG: Algorithm 1's fit instead (Q_0 free).  The last column, y, then is one more column of the homogeneous
// system [V | -y x^1 .. -y x^(M-1) | y] whose coefficient is -Q_0; (P, Q) is its null vector of unit length.
template <bool HOMOG>
__device__ __forceinline__ void locate_classes_wave(const float *__restrict__ pg, int64_t C, int64_t c0, int cpw,
                                                    const int *avail, const double *xs, int n, int M, int A,
                                                    double *scratch, int *votes) {
    const int lane = lane_id();
    const int W2 = 2 * M;
    const int cols = W2 - 1;                 // unknowns P_0..P_{M-1}, Q_1..Q_{M-1}; column `cols` is the rhs
    const int cl = lane / W2;
    const int j = lane - cl * W2;
    const int64_t c = c0 + cl;
    const bool live = cl < cpw && c < C;     // this lane's class exists
    const int LD = HOMOG ? W2 + 1 : W2;     // row stride of mat; odd for the column rotations of Algorithm 1's fit
    const int per_class = n * LD + M + n;
    double *mat = scratch + (live ? cl : 0) * per_class;
    double *coef = mat + n * LD;
    double *key = coef + M;

    build_class_system(pg, C, c, avail, xs, n, M, mat, LD, j, W2, live);
    factor_class_system(mat, LD, n, j, HOMOG ? W2 : cols, live);

    if (HOMOG) {
        // ---- the null vector, then a_r = Q(x_r): Q_k = coef[k-1] for k >= 1, Q_0 = -coef[M-1] ----------------------
        homogeneous_q(mat, LD, coef, key, W2, M, j, live);
        if (live) {
            for (int r = j; r < n; r += W2) {
                const double x = xs[r];
                double a = 0.0;
                for (int t = M - 2; t >= 0; --t) a = fma(a, x, coef[t]);
                a = fma(a, x, -coef[M - 1]);
                key[r] = (a != a) ? __builtin_inf() : fabs(a);
            }
        }
    } else {
        // ---- back substitution for Q_{M-1} .. Q_1 (unknowns cols-1 .. M); P is not needed ----
        // lane j holds the transformed right-hand side entry of row j.
        double s = (live && j < cols) ? mat[j * LD + cols] : 0.0;
        const double diag = (live && j < cols) ? mat[j * LD + j] : 1.0;
        for (int t = cols - 1; t >= M; --t) {
            if (live && j == t) coef[t - M] = s / diag;   // Q_{t-M+1}
            __builtin_amdgcn_wave_barrier();
            const double sol = coef[t - M];
            if (live && j < t) s = fma(-mat[j * LD + t], sol, s);
            __builtin_amdgcn_wave_barrier();
        }

        // ---- step 3: a_r = Q(x_r), Horner, one lane per row; steps 4-5: the A smallest |a_r| ----
        if (live) {
            for (int r = j; r < n; r += W2) {
                const double x = xs[r];
                double a = 0.0;
                for (int t = cols - 1; t >= M; --t) a = fma(a, x, coef[t - M]);
                a = fma(a, x, 1.0);                       // Q_0 = 1
                key[r] = (a != a) ? __builtin_inf() : fabs(a);
            }
        }
    }
    __builtin_amdgcn_wave_barrier();
    if (live) pick_and_vote(key, avail, n, A, j, W2, votes);
    __builtin_amdgcn_wave_barrier();
}

// Appendix A, Algorithm 3, for the classes c0 .. c0+cpw-1 of one group, by one wave: the same least-squares fit of
// (P, Q) as Algorithm 2, then the K values r(alpha_j) = P(alpha_j) / Q(alpha_j) instead of an error locator.
// Layout as locate_classes_wave (per class  mat[n][2M] | sol[2M-1] in the coef and key slots); lane j of a class
// evaluates query j, so K <= 2M lanes always suffice.
__device__ __forceinline__ void reconstruct_classes_wave(const float *__restrict__ pg, float *__restrict__ og, int64_t C,
                                                         int64_t c0, int cpw, const int *avail, const double *xs,
                                                         const double *alpha_s, int n, int K, int M, double *scratch) {
    const int lane = lane_id();
    const int W2 = 2 * M;
    const int cols = W2 - 1;                 // unknowns P_0..P_{M-1}, Q_1..Q_{M-1}; column `cols` is the rhs
    const int cl = lane / W2;
    const int j = lane - cl * W2;
    const int64_t c = c0 + cl;
    const bool live = cl < cpw && c < C;
    const int per_class = n * W2 + M + n;    // M + n >= 3M > cols doubles follow the matrix
    double *mat = scratch + (live ? cl : 0) * per_class;
    double *sol = mat + n * W2;

    build_class_system(pg, C, c, avail, xs, n, M, mat, W2, j, W2, live);
    factor_class_system(mat, W2, n, j, cols, live);

    // back substitution for every unknown; lane j holds the transformed right-hand side entry of row j
    double s = (live && j < cols) ? mat[j * W2 + cols] : 0.0;
    const double diag = (live && j < cols) ? mat[j * W2 + j] : 1.0;
    for (int t = cols - 1; t >= 0; --t) {
        if (live && j == t) sol[t] = s / diag;
        __builtin_amdgcn_wave_barrier();
        const double v = sol[t];
        if (live && j < t) s = fma(-mat[j * W2 + t], v, s);
        __builtin_amdgcn_wave_barrier();
    }
    if (live && j < K) {
        const double z = alpha_s[j];
        double num = 0.0, den = 0.0;
        for (int k = M - 1; k >= 0; --k) num = fma(num, z, sol[k]);              // P_0 .. P_{M-1}
        for (int k = M - 1; k >= 1; --k) den = fma(den, z, sol[M - 1 + k]);      // Q_1 .. Q_{M-1}
        den = fma(den, z, 1.0);                                                  // Q_0 = 1
        og[static_cast<size_t>(j) * C + c] = static_cast<float>(num / den);
    }
    __builtin_amdgcn_wave_barrier();
}

// One workgroup per group; waves take the classes cpw at a time.
// dynamic LDS: double scratch[nw][cpw * (n*2M + M + n)] | double xs[n] | double alpha_s[K] | double beta_s[N] | int avail[N] | int n
__global__ void decode_rational_kernel(const float *__restrict__ preds, const uint8_t *__restrict__ mask,
                                       float *__restrict__ out, int32_t *__restrict__ status, int K, int N, int S, int A,
                                       int64_t C, int cpw, int n_cap, const Nodes nodes) {
    extern __shared__ __align__(16) double lds_d[];
    const int M = K + A;
    const int nw = blockDim.x / kWave;
    const int wave_doubles = cpw * (n_cap * 2 * M + M + n_cap);
    double *scratch = lds_d;
    double *xs = scratch + static_cast<size_t>(nw) * wave_doubles;
    double *alpha_s = xs + n_cap;
    double *beta_s = alpha_s + K;
    int *avail = reinterpret_cast<int *>(beta_s + N);
    int *n_sh = avail + N;
    const int64_t g = blockIdx.x;
    const int wv = wave_id();

    stage_nodes(nodes, K, N, alpha_s, beta_s);
    if (wv == 0) {
        const int cnt = survivors_from_mask(mask + g * N, N, avail);
        if (lane_id() == 0) *n_sh = cnt;
    }
    __syncthreads();
    const int n = *n_sh;
    const bool good = S < 0 ? (n >= 2 * M && n <= n_cap) : n == n_cap;
    if (threadIdx.x == 0 && status != nullptr) status[g] = good ? APPROXIFER_GROUP_OK : APPROXIFER_GROUP_BAD_MASK;
    if (!good) return;
    for (int r = threadIdx.x; r < n; r += blockDim.x) xs[r] = beta_s[avail[r]];
    __syncthreads();
    const float *pg = preds + static_cast<size_t>(g) * N * C;
    float *og = out + static_cast<size_t>(g) * K * C;
    for (int64_t c0 = static_cast<int64_t>(wv) * cpw; c0 < C; c0 += static_cast<int64_t>(nw) * cpw)
        reconstruct_classes_wave(pg, og, C, c0, cpw, avail, xs, alpha_s, n, K, M, scratch + static_cast<size_t>(wv) * wave_doubles);
}

// dynamic LDS: double scratch[nw][cpw * (n*LD + M + n)] (LD = 2M, 2M+1 for Algorithm 1) | double WdT[(n-A) * KP] | double xs[n]
//              | double alpha_s[K] | double beta_s[N]
//              | int avail[N] | int F[N] | int Fpos[N] | int votes[N] | int n | int flag
template <bool HOMOG>
__global__ void decode_byzantine_general_kernel(const float *__restrict__ preds, const uint8_t *__restrict__ mask,
                                                float *__restrict__ out, int32_t *__restrict__ adv,
                                                int32_t *__restrict__ status, int K, int N, int S, int A, int64_t C,
                                                int64_t Cv, int vec4, int sign_mode, int cpw, int n_cap,
                                                int splits, int32_t *__restrict__ workspace, const Nodes nodes) {
    extern __shared__ __align__(16) double lds_d[];
    const int KP = round_up4(K);
    const int M = K + A;
    const int nF_cap = n_cap - A;
    const int nw = blockDim.x / kWave;
    const int wave_doubles = cpw * (n_cap * (HOMOG ? 2 * M + 1 : 2 * M) + M + n_cap);

    double *scratch = lds_d;
    double *WdT = scratch + static_cast<size_t>(nw) * wave_doubles;
    double *xs = WdT + nF_cap * KP;
    double *alpha_s = xs + n_cap;
    double *beta_s = alpha_s + K;
    int *avail = reinterpret_cast<int *>(beta_s + N);
    int *F = avail + N;
    int *Fpos = F + N;
    int *votes = Fpos + N;
    int *n_sh = votes + N;

    // splits > 1: `splits` workgroups share a group, see pool_votes_last_arrival
    const int64_t g = blockIdx.x / splits;
    const int part = static_cast<int>(blockIdx.x - g * splits);
    const int wv = wave_id();
    const float *pg = preds + static_cast<size_t>(g) * N * C;

    stage_nodes(nodes, K, N, alpha_s, beta_s);
    for (int e = threadIdx.x; e < nF_cap * KP; e += blockDim.x) WdT[e] = 0.0;
    for (int e = threadIdx.x; e < N; e += blockDim.x) votes[e] = 0;
    if (wv == 0) {
        const int cnt = survivors_from_mask(mask + g * N, N, avail);
        if (lane_id() == 0) *n_sh = cnt;
    }
    __syncthreads();
    const int n = *n_sh;
    const bool good = S < 0 ? (n >= 2 * M && n <= n_cap) : n == n_cap;
    if (threadIdx.x == 0 && status != nullptr) status[g] = good ? APPROXIFER_GROUP_OK : APPROXIFER_GROUP_BAD_MASK;
    if (!good) return;

    for (int r = threadIdx.x; r < n; r += blockDim.x) xs[r] = beta_s[avail[r]];
    __syncthreads();
    for (int64_t c0 = (static_cast<int64_t>(part) * nw + wv) * cpw; c0 < C; c0 += static_cast<int64_t>(splits) * nw * cpw)
        locate_classes_wave<HOMOG>(pg, C, c0, cpw, avail, xs, n, M, A, scratch + static_cast<size_t>(wv) * wave_doubles,
                                   votes);
    __syncthreads();
    if (splits > 1 && !pool_votes_last_arrival(workspace + g * (N + 1), votes, N, splits, n_sh + 1)) return;

    finish_group(pg, out + static_cast<size_t>(g) * K * C, adv + g * A, avail, n, N, A, K, KP, C, Cv, vec4 != 0, sign_mode,
                 alpha_s, beta_s, votes, F, Fpos, WdT);
}

// Before a launch in which several workgroups share a group: zero the workspace words through which they meet.
// (A kernel, not a memset: the call may be recorded into a HIP graph.)
__global__ void clear_workspace_kernel(int32_t *__restrict__ workspace, int64_t words) {
    const int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i < words) workspace[i] = 0;
}

// ---- launch shapes (host) --------------------------------------------------------------------------
constexpr int64_t kFillWaves = 4096;     // waves that put about four on every SIMD of the chip (256 CUs x 4 SIMDs)

bool proj_domain(int M, int n) { return M <= kProjMaxM && n <= 48 && n - M <= 32; }

struct ProjShape {
    int cw_log2, nw, splits;
};
// `may_split`: the caller brought a workspace for the workgroups of a group to meet in.
ProjShape proj_shape(int64_t G, int64_t C, bool may_split, int64_t fill_waves = kFillWaves) {
    ProjShape p;
    p.cw_log2 = C <= 16 ? 4 : (C <= 32 ? 5 : 6);           // classes per staged tile: 16, 32 or 64
    const int CW = 1 << p.cw_log2;
    // waves per workgroup: one per four classes of a tile, at most four -- but no more than it takes to put
    // about four waves on every SIMD of the chip: beyond that, extra waves of a group only
    // idle through the shared factorisation (measured at G = 2048, C = 10: 1 wave 44.7 us, 2 waves 42.7, 3 waves 53.0)
    int nw = static_cast<int>(((C < CW ? C : CW) + kClsPerWave - 1) / kClsPerWave);
    if (nw > 4) nw = 4;
    const int64_t fill = (fill_waves + G - 1) / G;
    if (nw > fill) nw = static_cast<int>(fill);
    p.nw = nw;
    // Few groups with many classes: one workgroup per group would leave most of the chip idle while each group walks
    // through its class tiles.  Then several workgroups share a group, each repeating the shared factorisation and
    // taking every splits-th tile, up to about 4096 waves in all.  From four tiles on: with fewer the repeated
    // factorisation and the extra launch cost what the split saves (G = 512, C = 100: 51 us whole, 59 us split).
    const int64_t tiles = (C + CW - 1) / CW;
    p.splits = 1;
    if (may_split && tiles >= 4) {
        const int64_t want = fill_waves / (G * nw);
        p.splits = static_cast<int>(want < tiles ? want : tiles);
        if (p.splits < 1) p.splits = 1;
    }
    return p;
}

struct GeneralShape {
    int cpw, nw, splits;
    size_t lds;                                            // 0: the shape does not fit the workgroup's LDS
};
GeneralShape general_shape(int64_t G, int K, int N, int n, int A, int64_t C, bool homogeneous, bool may_split) {
    GeneralShape s;
    const int KP = (K + 3) & ~3;
    const int M = K + A;
    // classes per wave: a class takes 2M lanes; waves per workgroup: enough for all classes, at most 4
    int cpw = kWave / (2 * M);
    if (cpw < 1) cpw = 1;
    if (cpw > C) cpw = static_cast<int>(C);
    const size_t fixed = sizeof(double) * (static_cast<size_t>(n - A) * KP + n + K + N) + sizeof(int) * (4 * static_cast<size_t>(N) + 2);
    const size_t per_class = sizeof(double) * (static_cast<size_t>(n) * (homogeneous ? 2 * M + 1 : 2 * M) + M + n);
    const size_t budget = 64 * 1024;
    while (cpw > 1 && fixed + cpw * per_class > budget) --cpw;
    const size_t per_wave = cpw * per_class;
    s.cpw = cpw;
    s.nw = 1;
    s.splits = 1;
    s.lds = 0;
    if (fixed + per_wave > budget) return s;
    int nw = static_cast<int>((C + cpw - 1) / cpw);
    if (nw > 4) nw = 4;
    if (nw > static_cast<int>((budget - fixed) / per_wave)) nw = static_cast<int>((budget - fixed) / per_wave);
    if (nw < 1) nw = 1;
    s.nw = nw;
    s.lds = fixed + nw * per_wave;
    // few groups, many classes: several workgroups share a group, as in the projected kernel (from four passes of a
    // workgroup over its classes on)
    const int64_t passes = (C + static_cast<int64_t>(nw) * cpw - 1) / (static_cast<int64_t>(nw) * cpw);
    if (may_split && passes >= 4) {
        const int64_t want = kFillWaves / (G * nw);
        s.splits = static_cast<int>(want < passes ? want : passes);
        if (s.splits < 1) s.splits = 1;
    }
    return s;
}

// most available workers a group can bring (S < 0: read off each mask)
int avail_capacity(int N, int S) { return S < 0 ? (N < APPROXIFER_MAX_AVAIL_BYZ ? N : APPROXIFER_MAX_AVAIL_BYZ) : N - S; }

int clear_workspace(int32_t *ws, int64_t G, int N, hipStream_t stream) {
    const int64_t words = G * (N + 1);
    const int threads = 256;
    return launch_status(launch_kernel(clear_workspace_kernel, dim3(static_cast<unsigned>((words + threads - 1) / threads)),
                                       dim3(threads), 0, stream, ws, words));
}

// Register tiles <rows of [V | I], rows of the projected system> of the projected kernel, smallest first.
struct ProjTile {
    int nb, rm;
};
constexpr ProjTile kProjTiles[] = {
    {20, 10},                 // n = 2M, the minimum of eq. (3), up to K + A = 10
    {20, 12}, {24, 12},       // n = 2M up to K + A = 12
    {24, 16}, {28, 14},       // n = 2M up to K + A = 14
    {32, 16}, {32, 32}, {48, 16}, {48, 32},
};
constexpr int kProjTileCount = sizeof(kProjTiles) / sizeof(kProjTiles[0]);
int proj_tile(int n, int M) {         // the smallest tile that holds (n, n - M); inside proj_domain one always does
    for (int t = 0; t < kProjTileCount; ++t)
        if (n <= kProjTiles[t].nb && n - M <= kProjTiles[t].rm) return t;
    return -1;
}
size_t basis_bytes(int tile, bool homogeneous) {
    const int stride = ush_stride(kProjTiles[tile].nb);
    const size_t b = sizeof(double) * (ush_rows(kProjTiles[tile].rm) * stride +
                                       (homogeneous ? kProjMaxM * stride + kProjMaxM * kProjMaxM : 0));
    return (b + 255) & ~static_cast<size_t>(255);
}
// Algorithm 1 on the shared factorisation: the register QR runs min(M, RM - 1) <= 15 steps.  Below K + A = 6 the LDS
// kernel, which packs 64 / 2M classes into a wave, is the faster one (measured, 10 classes, 4096 groups: K + A = 3:
// 33 us against 77; K + A = 6: 105 against 101; K + A = 10: 233 against 124; K + A = 12: 830 against 214;
// K + A = 14, 8192 groups: 2651 against 548).
bool hom_proj_domain(int M, int n) { return proj_domain(M, n) && M >= 6 && M <= kProjMaxM - 1; }
size_t votes_bytes(int64_t G, int N) {
    return (sizeof(int32_t) * static_cast<size_t>(G) * (N + 1) + 255) & ~static_cast<size_t>(255);
}
// Groups with a full mask exist only when no fixed number of stragglers is asked for; the shared basis serves the
// projected kernel (Algorithm 2).
bool full_basis_applies(int N, int S, int M) { return S <= 0 && proj_domain(M, N); }

// The caller's workspace, carved: first the basis of the full node set (8-byte aligned), then the vote words.
struct Carved {
    double *basis;
    int32_t *votes;
};
Carved carve_workspace(void *d_workspace, size_t bytes, size_t need_basis, size_t need_votes) {
    Carved c = {nullptr, nullptr};
    unsigned char *p = static_cast<unsigned char *>(d_workspace);
    if (p == nullptr) return c;
    if (need_basis != 0 && reinterpret_cast<uintptr_t>(p) % sizeof(double) == 0 && bytes >= need_basis) {
        c.basis = reinterpret_cast<double *>(p);
        p += need_basis;
        bytes -= need_basis;
    }
    if (need_votes != 0 && reinterpret_cast<uintptr_t>(p) % sizeof(int32_t) == 0 && bytes >= need_votes)
        c.votes = reinterpret_cast<int32_t *>(p);
    return c;
}

// kNoFit: the shape does not fit this kernel's LDS (Algorithm 1 with many workers): the caller falls back.
constexpr int kNoFit = 1;

// Whether decode_byzantine_shared_basis_kernel takes the call: the classes of a group leave class slots empty (C is
// not a multiple of four), a group is staged in one sixteen-class tile, and there are enough groups to fill the chip
// four to a workgroup (with fewer, a workgroup per group spreads them over more CUs).  Measured at K = 12, A = 2,
// 28 workers, 10 classes, 8192 groups (kernel time): one group per workgroup 132 us; 2 groups, 2 waves 137; 4 groups,
// 4 waves 126; 8 groups, 4 waves 125; one wave per workgroup of 2 / 4 groups 159 / 208.
constexpr int kSharedBasisGroups = 4;
bool shared_basis_applies(int64_t G, int64_t C) {
    if (C > kClsLanes || C % kClsPerWave == 0) return false;
    return G * ((C + kClsPerWave - 1) / kClsPerWave) >= kFillWaves;
}

template <int NB, int RM, int GPW>
int run_shared_basis(const float *d_preds, const uint8_t *d_mask, float *d_out, int32_t *d_adv, int32_t *d_status,
                     int64_t G, int K, int N, int A, int64_t C, const Nodes &nodes, int sign_mode, const double *basis,
                     hipStream_t stream) {
    const int KP = (K + 3) & ~3;
    const int64_t blocks = (G + GPW - 1) / GPW;
    int nw = static_cast<int>((GPW * C + kClsPerWave - 1) / kClsPerWave);   // a wave per round of four classes, up to four
    if (nw > 4) nw = 4;
    const size_t lds = sizeof(double) * (static_cast<size_t>(basis_doubles<NB, RM, false>()) + NB * kPwStride + NB +
                                         static_cast<size_t>(GPW) * (N - A) * KP + K + N) +
                       sizeof(float) * (static_cast<size_t>(GPW + 1) * NB * kClsLanes) +
                       sizeof(int) * (static_cast<size_t>(N) * (1 + 3 * GPW) + GPW);
    if (lds > 64 * 1024) return kNoFit;                   // the caller goes on with a workgroup per group
    if (blocks > 0x7fffffffLL) return APPROXIFER_ERR_LIMIT;
    return launch_status(launch_kernel(decode_byzantine_shared_basis_kernel<NB, RM, GPW>, dim3(static_cast<unsigned>(blocks)),
                                       dim3(nw * kWave), lds, stream, d_preds, d_mask, d_out, d_adv, d_status, G, K, N, A,
                                       static_cast<int>(C), sign_mode, basis, nodes));
}

template <int NB, int RM, bool HOMOG>
int run_proj(const float *d_preds, const uint8_t *d_mask, float *d_out, int32_t *d_adv, int32_t *d_status, int64_t G,
             int K, int N, int S, int A, int64_t C, int n_cap, bool vec4, const Nodes &nodes, int sign_mode,
             void *d_workspace, size_t workspace_bytes, int tile, hipStream_t stream) {
    const int KP = (K + 3) & ~3;
    const int M = K + A;
    const int64_t Cv = vec4 ? C / 4 : C;
    const size_t need_basis = full_basis_applies(N, S, M) ? basis_bytes(tile, HOMOG) : 0;
    const Carved ws = carve_workspace(d_workspace, workspace_bytes, need_basis, votes_bytes(G, N));
    // Algorithm 1's locator runs two waves to a SIMD (registers): half as many waves fill the chip
    ProjShape p = proj_shape(G, C, ws.votes != nullptr, HOMOG ? kFillWaves / 2 : kFillWaves);
    const int CW = 1 << p.cw_log2;
    const size_t hom_wave = HOMOG ? sizeof(double) * hom_scratch_doubles(M, n_cap, hom_mt(NB)) : 0;
    const size_t fixed = sizeof(double) * (static_cast<size_t>(basis_doubles<NB, RM, HOMOG>()) + NB * kPwStride + NB +
                                           static_cast<size_t>(n_cap - A) * KP + K + N) +
                         sizeof(float) * (static_cast<size_t>(NB) * CW) + sizeof(int) * (4 * static_cast<size_t>(N) + 2);
    while (p.nw > 1 && fixed + p.nw * hom_wave > 64 * 1024) --p.nw;
    const size_t lds = fixed + p.nw * hom_wave;
    if (lds > 64 * 1024) return HOMOG ? kNoFit : APPROXIFER_ERR_LIMIT;   // Algorithm 2: cannot happen inside the domain
    if (G * p.splits > 0x7fffffffLL) return APPROXIFER_ERR_LIMIT;
    if (ws.basis != nullptr) {
        const hipError_t e = launch_kernel(full_basis_kernel<NB, RM, HOMOG>, dim3(1), dim3(kWave), 0, stream, ws.basis, N, M, nodes);
        if (e != hipSuccess) return APPROXIFER_ERR_LAUNCH;
        if constexpr (!HOMOG) {
            // no stragglers by contract (S = 0): every good group shares this factorisation, and groups whose classes
            // do not fill whole rounds of four are packed several to a workgroup
            if (S == 0 && shared_basis_applies(G, C)) {
                const int rc = run_shared_basis<NB, RM, kSharedBasisGroups>(d_preds, d_mask, d_out, d_adv, d_status, G, K, N,
                                                                            A, C, nodes, sign_mode, ws.basis, stream);
                if (rc != kNoFit) return rc;
            }
        }
    }
    if (p.splits > 1) {
        const int rc = clear_workspace(ws.votes, G, N, stream);
        if (rc != APPROXIFER_OK) return rc;
    }
    const dim3 grid(static_cast<unsigned>(G * p.splits)), block(p.nw * kWave);
    return launch_status(launch_kernel(decode_byzantine_proj_kernel<NB, RM, HOMOG>, grid, block, lds, stream, d_preds, d_mask, d_out,
                                       d_adv, d_status, K, N, S, A, C, Cv, vec4 ? 1 : 0, sign_mode, n_cap, p.cw_log2,
                                       p.splits, ws.votes, static_cast<const double *>(ws.basis), nodes));
}

}  // namespace

// Device address of this GPU's copy of the built-in workspace.  Looked up once per device, with that device current
// (every GPU has its own copy at its own address), and kept for the life of the process.
int static_workspace(void **d_ptr) {
    constexpr int kMaxDevices = 64;
    static std::mutex lock;
    static void *per_device[kMaxDevices] = {};
    int device = -1;
    if (hipGetDevice(&device) != hipSuccess || device < 0 || device >= kMaxDevices) return APPROXIFER_ERR_LAUNCH;
    std::lock_guard<std::mutex> hold(lock);
    if (per_device[device] == nullptr) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) return APPROXIFER_ERR_LAUNCH;
        per_device[device] = p;
    }
    *d_ptr = per_device[device];
    return APPROXIFER_OK;
}

int launch_decode_rational(const float *d_preds, const uint8_t *d_mask, float *d_out, int32_t *d_status, int64_t G, int K,
                           int N, int S, int A, int64_t C, const Nodes &nodes, hipStream_t stream) {
    const int n = avail_capacity(N, S);
    const int M = K + A;
    if (G > 0x7fffffffLL) return APPROXIFER_ERR_LIMIT;
    int cpw = kWave / (2 * M);
    if (cpw < 1) cpw = 1;
    if (cpw > C) cpw = static_cast<int>(C);
    const size_t fixed = sizeof(double) * (static_cast<size_t>(n) + K + N) + sizeof(int) * (static_cast<size_t>(N) + 2);
    const size_t per_class = sizeof(double) * (static_cast<size_t>(n) * 2 * M + M + n);
    const size_t budget = 64 * 1024;
    while (cpw > 1 && fixed + cpw * per_class > budget) --cpw;
    const size_t per_wave = cpw * per_class;
    if (fixed + per_wave > budget) return APPROXIFER_ERR_LIMIT;
    int nw = static_cast<int>((C + cpw - 1) / cpw);
    if (nw > 4) nw = 4;
    if (nw > static_cast<int>((budget - fixed) / per_wave)) nw = static_cast<int>((budget - fixed) / per_wave);
    if (nw < 1) nw = 1;
    return launch_status(launch_kernel(decode_rational_kernel, dim3(static_cast<unsigned>(G)), dim3(nw * kWave),
                                       fixed + nw * per_wave, stream, d_preds, d_mask, d_out, d_status, K, N, S, A, C, cpw, n,
                                       nodes));
}

size_t byzantine_workspace_bytes(int64_t G, int K, int N, int S, int A, int64_t C) {
    const int n = avail_capacity(N, S);
    const int M = K + A;
    bool splits = false;
    size_t basis = 0;
    if (proj_domain(M, n)) {
        splits = proj_shape(G, C, true).splits > 1;
        if (full_basis_applies(N, S, M)) basis = basis_bytes(proj_tile(n, M), hom_proj_domain(M, n));
    } else {
        splits = general_shape(G, K, N, n, A, C, false, true).splits > 1;
    }
    splits = splits || general_shape(G, K, N, n, A, C, true, true).splits > 1;       // Algorithm 1's locator
    return basis + (splits ? votes_bytes(G, N) : 0);
}

int launch_decode_byzantine(const float *d_preds, const uint8_t *d_mask, float *d_out, int32_t *d_adv,
                            int32_t *d_status, int64_t G, int K, int N, int S, int A, int64_t C, const Nodes &nodes,
                            int sign_mode, bool homogeneous, void *d_workspace, size_t workspace_bytes,
                            hipStream_t stream) {
    const int n = avail_capacity(N, S);
    const int M = K + A;
    const bool vec4 = (C % 4 == 0) && aligned16(d_preds) && aligned16(d_out);
    const int64_t Cv = vec4 ? C / 4 : C;
    if (G > 0x7fffffffLL) return APPROXIFER_ERR_LIMIT;

    if (homogeneous ? hom_proj_domain(M, n) : proj_domain(M, n)) {
        int rc = kNoFit;
#define APPROXIFER_PROJ(T, NB, RM)                                                                                     \
    case T:                                                                                                            \
        static_assert(kProjTiles[T].nb == NB && kProjTiles[T].rm == RM, "tile table");                                 \
        rc = homogeneous ? run_proj<NB, RM, true>(d_preds, d_mask, d_out, d_adv, d_status, G, K, N, S, A, C, n, vec4,     \
                                                  nodes, sign_mode, d_workspace, workspace_bytes, T, stream)            \
                         : run_proj<NB, RM, false>(d_preds, d_mask, d_out, d_adv, d_status, G, K, N, S, A, C, n, vec4,    \
                                                   nodes, sign_mode, d_workspace, workspace_bytes, T, stream);          \
        break;
        switch (proj_tile(n, M)) {
            APPROXIFER_PROJ(0, 20, 10)
            APPROXIFER_PROJ(1, 20, 12)
            APPROXIFER_PROJ(2, 24, 12)
            APPROXIFER_PROJ(3, 24, 16)
            APPROXIFER_PROJ(4, 28, 14)
            APPROXIFER_PROJ(5, 32, 16)
            APPROXIFER_PROJ(6, 32, 32)
            APPROXIFER_PROJ(7, 48, 16)
            APPROXIFER_PROJ(8, 48, 32)
            default: return APPROXIFER_ERR_LIMIT;          // cannot happen inside the projected kernel's domain
        }
#undef APPROXIFER_PROJ
        if (rc != kNoFit) return rc;
    }

    // the workgroups of a group meet in the workspace: without one that holds N + 1 words per group, and is aligned
    // for them, every group stays with one workgroup
    const Carved ws = carve_workspace(d_workspace, workspace_bytes, 0, votes_bytes(G, N));
    const GeneralShape sh = general_shape(G, K, N, n, A, C, homogeneous, ws.votes != nullptr);
    if (sh.lds == 0) return APPROXIFER_ERR_LIMIT;
    if (G * sh.splits > 0x7fffffffLL) return APPROXIFER_ERR_LIMIT;
    if (sh.splits > 1) {
        const int rc = clear_workspace(ws.votes, G, N, stream);
        if (rc != APPROXIFER_OK) return rc;
    }
    const dim3 grid(static_cast<unsigned>(G * sh.splits)), block(sh.nw * kWave);
    return launch_status(launch_kernel(homogeneous ? decode_byzantine_general_kernel<true> : decode_byzantine_general_kernel<false>,
                                       grid, block, sh.lds, stream, d_preds, d_mask, d_out, d_adv, d_status, K, N, S, A, C, Cv,
                                       vec4 ? 1 : 0, sign_mode, sh.cpw, n, sh.splits, ws.votes, nodes));
}

}  // namespace approxifer
