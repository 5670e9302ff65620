// ApproxIFER decoder and Byzantine decoder for gfx950 (Section 3, "ApproxIFER Decoding").
//
// Decoder: one workgroup per (group, tile of prediction columns).  The group's mask is
// turned into the ascending survivor list F with wavefront ballots, the K x |F| matrix of
// basis functions is evaluated in float64 (one wave per query node, the denominator by a
// wavefront reduction) and kept transposed in LDS, and the contraction over F accumulates
// in float64 with the weights broadcast from LDS.  Rows of missing workers are never read.
//
// Byzantine decoder: one workgroup per group.  Algorithm 2 runs on several classes per wave:
// a class owns 2(K+A) neighbouring lanes, lane j of a class owns COLUMN j of its
// (N-S) x (2(K+A)-1) system (the last lane owns the right-hand side), and the matrix sits in
// LDS row-major so that the lanes of a class touch consecutive addresses.  A Householder step
// then needs no cross-lane reduction at all: every lane walks down the pivot column (an LDS
// broadcast) accumulating the column norm and its own dot product, and updates its own
// column.  The Q coefficients come out of a back substitution restricted to the trailing
// block, a_r = Q(x_r) is evaluated by Horner's rule with one lane per row, the A smallest
// |a_r| vote; after the vote the adversaries are removed from the available list and the
// workgroup decodes the group as above.
#include "common.h"

namespace approxifer {
namespace {

constexpr int kColsPerTile = 64;   // vector columns handled by one wave-wide item row

__device__ __forceinline__ int round_up4(int v) { return (v + 3) & ~3; }

// Ascending list of the workers whose mask byte is non-zero.  Called by ONE whole wave.
// Returns the number of survivors; list[0..n) is written (visible after the next barrier).
__device__ __forceinline__ int survivors_from_mask(const uint8_t *__restrict__ mask_row, int N, int *list) {
    const int lane = lane_id();
    const bool b0 = (lane < N) && (mask_row[lane] != 0);
    const bool b1 = (lane + kWave < N) && (mask_row[lane + kWave] != 0);
    const unsigned long long m0 = __ballot(b0);
    const unsigned long long m1 = __ballot(b1);
    const unsigned long long below = (1ull << lane) - 1ull;
    const int n0 = __popcll(m0);
    if (b0) list[__popcll(m0 & below)] = lane;
    if (b1) list[n0 + __popcll(m1 & below)] = lane + kWave;
    return n0 + __popcll(m1);
}

// Transposed decoder weights WdT[r*KP + j] = l_{F_r}(alpha_j), Section 3 "ApproxIFER Decoding"
// step 2.  Called by the whole workgroup after F is visible; the caller provides a barrier
// afterwards.  WdT must have been zeroed for the pad columns j in [K, KP).
// Up to 64 survivors: a group of LPR = 16/32/64 lanes per query node, several nodes per pass.
template <int LPR>
__device__ __forceinline__ void decoder_weights_grouped(const double *alpha_s, const double *beta_s, const int *F, int nF, int K, int KP,
                                                        int sign_mode, double *WdT) {
    const int tid = threadIdx.x;
    const int r = tid % LPR;
    const int sub = tid / LPR;
    const int rows_per_pass = blockDim.x / LPR;
    const bool valid = r < nF;
    const int i = valid ? F[r] : 0;
    const double xb = beta_s[i];
    const int parity = (sign_mode == APPROXIFER_SIGN_WORKER_INDEX) ? (i & 1) : (r & 1);
    const double sign = parity ? -1.0 : 1.0;
    const unsigned long long group_mask =
        (LPR == 64) ? ~0ull : ((1ull << (LPR & 63)) - 1ull) << ((tid & 63) / LPR * LPR);
    for (int j0 = 0; j0 < K; j0 += rows_per_pass) {
        const int j = j0 + sub;
        const bool row = j < K;
        const BerrutTerm bt = berrut_term(alpha_s[row ? j : 0], xb, sign, valid && row);
        const double rden = 1.0 / group_sum<LPR>(bt.t);
        const bool any_hit = (__ballot(bt.hit) & group_mask) != 0ull;
        if (valid && row) WdT[r * KP + j] = any_hit ? (bt.hit ? 1.0 : 0.0) : bt.t * rden;
    }
}

// More than 64 survivors: one wave per query node, two lanes-worth of survivors per lane.
__device__ __forceinline__ void decoder_weights_wide(const double *alpha_s, const double *beta_s, const int *F, int nF, int K, int KP,
                                                     int sign_mode, double *WdT) {
    const int lane = lane_id();
    const int nwaves = blockDim.x / kWave;
    for (int j = wave_id(); j < K; j += nwaves) {
        const double z = alpha_s[j];
        BerrutTerm bt[2];
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            const int r = p * kWave + lane;
            const bool valid = r < nF;
            const int i = valid ? F[r] : 0;
            const int parity = (sign_mode == APPROXIFER_SIGN_WORKER_INDEX) ? (i & 1) : (r & 1);
            bt[p] = berrut_term(z, beta_s[i], parity ? -1.0 : 1.0, valid);
        }
        const double rden = 1.0 / wave_sum(bt[0].t + bt[1].t);
        const bool any_hit = (__ballot(bt[0].hit) | __ballot(bt[1].hit)) != 0ull;
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            const int r = p * kWave + lane;
            if (r < nF) WdT[r * KP + j] = any_hit ? (bt[p].hit ? 1.0 : 0.0) : bt[p].t * rden;
        }
    }
}

__device__ __forceinline__ void decoder_weights(const double *alpha_s, const double *beta_s, const int *F, int nF, int K, int KP,
                                                int sign_mode, double *WdT) {
    if (nF <= 16) decoder_weights_grouped<16>(alpha_s, beta_s, F, nF, K, KP, sign_mode, WdT);
    else if (nF <= 32) decoder_weights_grouped<32>(alpha_s, beta_s, F, nF, K, KP, sign_mode, WdT);
    else if (nF <= 64) decoder_weights_grouped<64>(alpha_s, beta_s, F, nF, K, KP, sign_mode, WdT);
    else decoder_weights_wide(alpha_s, beta_s, F, nF, K, KP, sign_mode, WdT);
}

// The nodes arrive in the kernel-argument segment; the decoders index them per lane, so every
// workgroup first copies them to LDS (alpha_s[K], beta_s[N]) with one load per thread, issued
// together with the mask load instead of later in the dependency chain.
__device__ __forceinline__ void stage_nodes(const Nodes &nodes, int K, int N, double *alpha_s, double *beta_s) {
    for (int t = threadIdx.x; t < K + N; t += blockDim.x) {
        if (t < K) alpha_s[t] = nodes.alpha[t];
        else beta_s[t - K] = nodes.beta[t - K];
    }
}

template <int VEC> struct PredVec;
template <> struct PredVec<4> { typedef v4f type; };
template <> struct PredVec<1> { typedef float type; };

template <int VEC> __device__ __forceinline__ float vec_get(typename PredVec<VEC>::type v, int e);
template <> __device__ __forceinline__ float vec_get<4>(v4f v, int e) { return v[e]; }
template <> __device__ __forceinline__ float vec_get<1>(float v, int) { return v; }

template <int VEC> __device__ __forceinline__ void store_row(float *dst, const double *acc);
template <> __device__ __forceinline__ void store_row<4>(float *dst, const double *acc) {
    v4f v;
    v[0] = static_cast<float>(acc[0]);
    v[1] = static_cast<float>(acc[1]);
    v[2] = static_cast<float>(acc[2]);
    v[3] = static_cast<float>(acc[3]);
    *reinterpret_cast<v4f *>(dst) = v;
}
template <> __device__ __forceinline__ void store_row<1>(float *dst, const double *acc) {
    *dst = static_cast<float>(acc[0]);
}

constexpr int kRowChunk = 8;   // prediction rows a lane keeps in flight at once

// Loads of one chunk of surviving rows for one vector column.  Rows past the end of F are
// clamped to the last survivor (always a valid address); their values are never used.
template <int VEC>
__device__ __forceinline__ void load_row_chunk(const float *__restrict__ pg, const int *F, int nF, int r0, int64_t C,
                                               int64_t cv, typename PredVec<VEC>::type (&y)[kRowChunk]) {
    typedef typename PredVec<VEC>::type V;
#pragma unroll
    for (int u = 0; u < kRowChunk; ++u) {
        const int r = (r0 + u < nF) ? r0 + u : nF - 1;
        y[u] = *reinterpret_cast<const V *>(pg + static_cast<size_t>(F[r]) * C + cv * VEC);
    }
}

// out[g][j][c] = sum_r WdT[r][j] * preds[g][F_r][c] for the vector columns [cv0, cv1) of one
// group.  Work items are (quad of query rows, vector column); a wave shares its quad, so the
// weight reads are LDS broadcasts.  Rows are fetched kRowChunk at a time so that a lane has
// that many loads in flight; float64 accumulation, one rounding on store.
// PREFETCHED: the caller already issued the first chunk of this lane's first item into `first`
// (before it evaluated the weights, to overlap the two).
template <int VEC, bool PREFETCHED>
__device__ __forceinline__ void contract_tile(const float *__restrict__ pg, float *__restrict__ og, const int *F,
                                              int nF, int K, int KP, int64_t C, int64_t cv0, int64_t cv1,
                                              const double *WdT, typename PredVec<VEC>::type (&first)[kRowChunk]) {
    typedef typename PredVec<VEC>::type V;
    const int KQ = KP / 4;
    const int items = KQ * kColsPerTile;
    for (int it = threadIdx.x; it < items; it += blockDim.x) {
        const int q = it / kColsPerTile;
        const int64_t cv = cv0 + (it % kColsPerTile);
        if (cv >= cv1) continue;
        double acc[4][VEC];
#pragma unroll
        for (int jj = 0; jj < 4; ++jj)
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc[jj][e] = 0.0;
        for (int r0 = 0; r0 < nF; r0 += kRowChunk) {
            V y[kRowChunk];
            if (PREFETCHED && r0 == 0 && it == static_cast<int>(threadIdx.x)) {
#pragma unroll
                for (int u = 0; u < kRowChunk; ++u) y[u] = first[u];
            } else {
                load_row_chunk<VEC>(pg, F, nF, r0, C, cv, y);
            }
#pragma unroll
            for (int u = 0; u < kRowChunk; ++u) {
                if (r0 + u < nF) {
                    const double *w = WdT + (r0 + u) * KP + 4 * q;
#pragma unroll
                    for (int jj = 0; jj < 4; ++jj) {
                        const double wj = w[jj];
#pragma unroll
                        for (int e = 0; e < VEC; ++e)
                            acc[jj][e] = fma(wj, static_cast<double>(vec_get<VEC>(y[u], e)), acc[jj][e]);
                    }
                }
            }
        }
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
            const int j = 4 * q + jj;
            if (j < K) store_row<VEC>(og + static_cast<size_t>(j) * C + cv * VEC, acc[jj]);
        }
    }
}

// ------------------------------------------------------------------------------------
// decoder kernel
// ------------------------------------------------------------------------------------
// dynamic LDS: double WdT[(N-S) * KP] | double alpha_s[K] | double beta_s[N] | int F[N] | int n
template <int VEC>
__global__ void decode_kernel(const float *__restrict__ preds, const uint8_t *__restrict__ mask,
                              float *__restrict__ out, int32_t *__restrict__ status, int K, int N, int S,
                              int64_t C, int64_t Cv, int64_t ctiles, int sign_mode, const Nodes nodes) {
    extern __shared__ double lds_d[];
    const int KP = round_up4(K);
    const int nF_cap = S < 0 ? N : N - S;          // S < 0: every group brings its own straggler count
    double *WdT = lds_d;
    double *alpha_s = WdT + nF_cap * KP;
    double *beta_s = alpha_s + K;
    int *F = reinterpret_cast<int *>(beta_s + N);
    int *n_sh = F + N;

    const int64_t g = blockIdx.x / ctiles;
    const int64_t ct = blockIdx.x - g * ctiles;

    stage_nodes(nodes, K, N, alpha_s, beta_s);
    for (int e = threadIdx.x; e < nF_cap * KP; e += blockDim.x) WdT[e] = 0.0;
    if (wave_id() == 0) {
        const int n = survivors_from_mask(mask + g * N, N, F);
        if (lane_id() == 0) *n_sh = n;
    }
    __syncthreads();
    const int nF = *n_sh;
    const bool good = S < 0 ? nF >= 1 : nF == nF_cap;
    if (ct == 0 && threadIdx.x == 0 && status != nullptr)
        status[g] = good ? APPROXIFER_GROUP_OK : APPROXIFER_GROUP_BAD_MASK;
    if (!good) return;

    // first chunk of this lane's prediction rows: issued now, consumed after the weights exist
    const int64_t cv0 = ct * kColsPerTile;
    const int64_t cv1 = (cv0 + kColsPerTile < Cv) ? cv0 + kColsPerTile : Cv;
    const float *pg = preds + static_cast<size_t>(g) * N * C;
    typename PredVec<VEC>::type first[kRowChunk];
    {
        const int64_t cv = cv0 + (threadIdx.x % kColsPerTile);
        load_row_chunk<VEC>(pg, F, nF, 0, C, cv < cv1 ? cv : cv0, first);
    }

    decoder_weights(alpha_s, beta_s, F, nF, K, KP, sign_mode, WdT);
    __syncthreads();

    contract_tile<VEC, true>(pg, out + static_cast<size_t>(g) * K * C, F, nF, K, KP, C, cv0, cv1, WdT, first);
}

// ------------------------------------------------------------------------------------
// fused decoder + top-1 kernel
// ------------------------------------------------------------------------------------
struct Best {
    double v;
    int i;
};
__device__ __forceinline__ bool better(double v, int i, const Best &b) { return v > b.v || (v == b.v && i < b.i); }

// One workgroup per group, one wave per quad of query rows.  A lane walks vector columns
// lane, lane+64, .. of its quad, decodes them in float64 exactly as contract_tile does and
// keeps the largest value (smallest class on equal values) per query row; a wavefront
// butterfly merges the 64 candidates; when the workgroup has more waves than quads, the waves
// of a quad split its columns and their winners are merged through LDS.  Nothing but [K] class
// indices (and scores) is written.
// dynamic LDS: as decode_kernel, then pad to 16 bytes | Best merged[KP][slices].
template <int VEC>
__global__ void decode_top1_kernel(const float *__restrict__ preds, const uint8_t *__restrict__ mask,
                                   int32_t *__restrict__ top1, float *__restrict__ score,
                                   int32_t *__restrict__ status, int K, int N, int S, int64_t C, int64_t Cv,
                                   int sign_mode, const Nodes nodes) {
    typedef typename PredVec<VEC>::type V;
    extern __shared__ double lds_d[];
    const int KP = round_up4(K);
    const int nF_cap = S < 0 ? N : N - S;          // S < 0: every group brings its own straggler count
    double *WdT = lds_d;
    double *alpha_s = WdT + nF_cap * KP;
    double *beta_s = alpha_s + K;
    int *F = reinterpret_cast<int *>(beta_s + N);
    int *n_sh = F + N;
    const int64_t g = blockIdx.x;

    stage_nodes(nodes, K, N, alpha_s, beta_s);
    for (int e = threadIdx.x; e < nF_cap * KP; e += blockDim.x) WdT[e] = 0.0;
    if (wave_id() == 0) {
        const int n = survivors_from_mask(mask + g * N, N, F);
        if (lane_id() == 0) *n_sh = n;
    }
    __syncthreads();
    const int nF = *n_sh;
    const bool good = S < 0 ? nF >= 1 : nF == nF_cap;
    if (threadIdx.x == 0 && status != nullptr) status[g] = good ? APPROXIFER_GROUP_OK : APPROXIFER_GROUP_BAD_MASK;
    if (!good) return;
    decoder_weights(alpha_s, beta_s, F, nF, K, KP, sign_mode, WdT);
    __syncthreads();

    const float *pg = preds + static_cast<size_t>(g) * N * C;
    const int lane = lane_id();
    const int KQ = KP / 4;
    const int nwaves = blockDim.x / kWave;
    const int slices = nwaves >= KQ ? nwaves / KQ : 1;          // waves that share one quad split its columns
    const int qwaves = nwaves >= KQ ? KQ : nwaves;              // quads processed concurrently
    const int slice = wave_id() / qwaves;
    Best *merged = reinterpret_cast<Best *>((reinterpret_cast<uintptr_t>(n_sh + 1) + 15) & ~static_cast<uintptr_t>(15));   // [KP][slices]
    for (int q = wave_id() % qwaves; q < KQ && slice < slices; q += qwaves) {
        Best best[4];
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
            best[jj].v = -__builtin_inf();
            best[jj].i = 0x7fffffff;
        }
        for (int64_t cv = static_cast<int64_t>(slice) * kWave + lane; cv < Cv; cv += static_cast<int64_t>(slices) * kWave) {
            double acc[4][VEC];
#pragma unroll
            for (int jj = 0; jj < 4; ++jj)
#pragma unroll
                for (int e = 0; e < VEC; ++e) acc[jj][e] = 0.0;
            for (int r0 = 0; r0 < nF; r0 += kRowChunk) {
                V y[kRowChunk];
                load_row_chunk<VEC>(pg, F, nF, r0, C, cv, y);
#pragma unroll
                for (int u = 0; u < kRowChunk; ++u) {
                    if (r0 + u < nF) {
                        const double *w = WdT + (r0 + u) * KP + 4 * q;
#pragma unroll
                        for (int jj = 0; jj < 4; ++jj) {
                            const double wj = w[jj];
#pragma unroll
                            for (int e = 0; e < VEC; ++e)
                                acc[jj][e] = fma(wj, static_cast<double>(vec_get<VEC>(y[u], e)), acc[jj][e]);
                        }
                    }
                }
            }
#pragma unroll
            for (int jj = 0; jj < 4; ++jj)
#pragma unroll
                for (int e = 0; e < VEC; ++e) {
                    const int idx = static_cast<int>(cv * VEC + e);
                    if (better(acc[jj][e], idx, best[jj])) {
                        best[jj].v = acc[jj][e];
                        best[jj].i = idx;
                    }
                }
        }
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) {
                const double ov = __shfl_xor(best[jj].v, off, kWave);
                const int oi = __shfl_xor(best[jj].i, off, kWave);
                if (better(ov, oi, best[jj])) {
                    best[jj].v = ov;
                    best[jj].i = oi;
                }
            }
            if (lane == 0) merged[(4 * q + jj) * slices + slice] = best[jj];
        }
    }
    __syncthreads();
    for (int j = threadIdx.x; j < K; j += blockDim.x) {
        Best b = merged[j * slices];
        for (int sl = 1; sl < slices; ++sl) {
            const Best o = merged[j * slices + sl];
            if (better(o.v, o.i, b)) b = o;
        }
        top1[g * K + j] = b.i == 0x7fffffff ? 0 : b.i;
        if (score != nullptr) score[g * K + j] = static_cast<float>(b.v);
    }
}

// ------------------------------------------------------------------------------------
// Byzantine decoder kernel
// ------------------------------------------------------------------------------------
// Algorithm 2, steps 1-5, for the classes c0 .. c0+cpw-1 of one group, by one wave.
//   n        available workers (rows), M = K + A, W2 = 2M columns including the right-hand side
//   xs[n]    worker nodes of the available workers (LDS, shared by the workgroup)
//   scratch  this wave's LDS: per class  mat[n][W2] | coef[M] | key[n]
// Lane (cl, j) = (lane / W2, lane % W2) works on class c0 + cl; lanes beyond cpw classes idle.
// Votes for the A smallest |Q(x_r)| of every class are added to votes[worker].
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
    const int per_class = n * W2 + M + n;
    double *mat = scratch + (live ? cl : 0) * per_class;
    double *coef = mat + n * W2;
    double *key = coef + M;

    // ---- steps 1-2: the system, one lane per row (rows j, j+W2, ..) -------------------
    if (live) {
        for (int r = j; r < n; r += W2) {
            const double x = xs[r];
            const double y = static_cast<double>(pg[static_cast<size_t>(avail[r]) * C + c]);
            double *row = mat + r * W2;
            double p = 1.0;
            for (int k = 0; k < M; ++k) {
                row[k] = p;                               // x^k
                if (k >= 1) row[M - 1 + k] = -y * p;      // -y x^k
                p *= x;
            }
            row[cols] = y;
        }
    }
    __builtin_amdgcn_wave_barrier();

    // ---- Householder QR in least-squares form, one lane per column ---------------------
    // Step k reflects column k onto e_k over rows k..n-1 and applies the reflector to the
    // columns right of it (and to the right-hand side).
    for (int k = 0; k < cols; ++k) {
        double sigma = 0.0, d = 0.0;
#pragma unroll 4
        for (int r = k; r < n; ++r) {
            const double vr = mat[r * W2 + k];            // broadcast inside the class
            const double arj = mat[r * W2 + j];
            sigma = fma(vr, vr, sigma);
            d = fma(vr, arj, d);
        }
        const double xkk = mat[k * W2 + k];
        const double akj = mat[k * W2 + j];
        const bool degenerate = !(sigma > 0.0);
        const double nrm = sqrt(sigma);
        const double alpha = (xkk >= 0.0) ? -nrm : nrm;
        const double scale = 1.0 / (sigma - alpha * xkk);   // 2 / (v^T v), v = x - alpha e_k
        const double f = scale * (d - alpha * akj);          // 2 v^T a_j / (v^T v)
        __builtin_amdgcn_wave_barrier();
        if (live && !degenerate) {
            if (j > k) {
#pragma unroll 4
                for (int r = k; r < n; ++r) {
                    const double vr = (r == k) ? xkk - alpha : mat[r * W2 + k];
                    mat[r * W2 + j] = fma(-f, vr, mat[r * W2 + j]);
                }
            } else if (j == k) {
                mat[k * W2 + k] = alpha;                  // R[k][k]
            }
        }
        __builtin_amdgcn_wave_barrier();
    }

    // ---- back substitution for Q_{M-1} .. Q_1 (unknowns cols-1 .. M); P is not needed ----
    // lane j holds the transformed right-hand side entry of row j.
    double s = (live && j < cols) ? mat[j * W2 + cols] : 0.0;
    const double diag = (live && j < cols) ? mat[j * W2 + j] : 1.0;
    for (int t = cols - 1; t >= M; --t) {
        if (live && j == t) coef[t - M] = s / diag;       // Q_{t-M+1}
        __builtin_amdgcn_wave_barrier();
        const double sol = coef[t - M];
        if (live && j < t) s = fma(-mat[j * W2 + t], sol, s);
        __builtin_amdgcn_wave_barrier();
    }

    // ---- step 3: a_r = Q(x_r), Horner, one lane per row; steps 4-5: the A smallest |a_r| ----
    if (live) {
        for (int r = j; r < n; r += W2) {
            const double x = xs[r];
            double a = 0.0;
            for (int t = cols - 1; t >= M; --t) a = fma(a, x, coef[t - M]);
            a = fma(a, x, 1.0);                           // Q_0 = 1
            key[r] = (a != a) ? __builtin_inf() : fabs(a);
        }
    }
    __builtin_amdgcn_wave_barrier();
    if (live) {
        for (int r = j; r < n; r += W2) {
            const double mine = key[r];
            int rank = 0;                                  // equal magnitudes keep ascending worker order
            for (int o = 0; o < n; ++o) {
                const double other = key[o];
                rank += (other < mine || (other == mine && o < r)) ? 1 : 0;
            }
            if (rank < A) atomicAdd(&votes[avail[r]], 1);
        }
    }
    __builtin_amdgcn_wave_barrier();
}

// dynamic LDS: double scratch[nw][cpw * (n*2M + M + n)] | double WdT[(n-A) * KP] | double xs[n]
//              | double alpha_s[K] | double beta_s[N]
//              | int avail[N] | int F[N] | int votes[N] | int sel[N] | int n
template <int VEC>
__global__ void decode_byzantine_kernel(const float *__restrict__ preds, const uint8_t *__restrict__ mask,
                                        float *__restrict__ out, int32_t *__restrict__ adv,
                                        int32_t *__restrict__ status, int K, int N, int S, int A, int64_t C,
                                        int64_t Cv, int sign_mode, int cpw, const Nodes nodes) {
    extern __shared__ double lds_d[];
    const int KP = round_up4(K);
    const int M = K + A;
    const int n_cap = S < 0 ? (N < APPROXIFER_MAX_AVAIL_BYZ ? N : APPROXIFER_MAX_AVAIL_BYZ) : N - S;   // layout capacity
    const int nF_cap = n_cap - A;
    const int nw = blockDim.x / kWave;
    const int wave_doubles = cpw * (n_cap * 2 * M + M + n_cap);

    double *scratch = lds_d;
    double *WdT = scratch + static_cast<size_t>(nw) * wave_doubles;
    double *xs = WdT + nF_cap * KP;
    double *alpha_s = xs + n_cap;
    double *beta_s = alpha_s + K;
    int *avail = reinterpret_cast<int *>(beta_s + N);
    int *F = avail + N;
    int *votes = F + N;
    int *sel = votes + N;
    int *n_sh = sel + N;

    const int64_t g = blockIdx.x;
    const int lane = lane_id();
    const int wv = wave_id();
    const float *pg = preds + static_cast<size_t>(g) * N * C;

    stage_nodes(nodes, K, N, alpha_s, beta_s);
    for (int e = threadIdx.x; e < nF_cap * KP; e += blockDim.x) WdT[e] = 0.0;
    for (int e = threadIdx.x; e < N; e += blockDim.x) votes[e] = 0;
    if (wv == 0) {
        const int n = survivors_from_mask(mask + g * N, N, avail);
        if (lane == 0) *n_sh = n;
    }
    __syncthreads();
    const int n = *n_sh;
    const bool good = S < 0 ? (n >= 2 * M && n <= n_cap) : n == n_cap;
    const int nF = n - A;
    if (threadIdx.x == 0 && status != nullptr) status[g] = good ? APPROXIFER_GROUP_OK : APPROXIFER_GROUP_BAD_MASK;
    if (!good) return;

    // ---- Algorithm 2: per-class fit, pick, vote ---------------------------------------
    for (int r = threadIdx.x; r < n; r += blockDim.x) xs[r] = beta_s[avail[r]];
    __syncthreads();
    for (int64_t c0 = static_cast<int64_t>(wv) * cpw; c0 < C; c0 += static_cast<int64_t>(nw) * cpw)
        locate_classes_wave(pg, C, c0, cpw, avail, xs, n, M, A, scratch + static_cast<size_t>(wv) * wave_doubles, votes);
    __syncthreads();

    // ---- the A most voted workers (equal counts: smaller index first), ascending -------
    for (int i = threadIdx.x; i < N; i += blockDim.x) {
        const int mine = votes[i];
        int rank = 0;
        for (int o = 0; o < N; ++o) {
            const int v = votes[o];
            rank += (v > mine || (v == mine && o < i)) ? 1 : 0;
        }
        sel[i] = rank < A ? 1 : 0;
    }
    __syncthreads();
    for (int i = threadIdx.x; i < N; i += blockDim.x) {
        if (sel[i]) {
            int pos = 0;
            for (int o = 0; o < i; ++o) pos += sel[o];
            adv[g * A + pos] = i;
        }
    }
    if (wv == 0) {   // F = available workers minus the located ones (n <= 64: one pass)
        const bool keep = (lane < n) && !sel[avail[lane]];
        const unsigned long long m = __ballot(keep);
        if (keep) F[__popcll(m & ((1ull << lane) - 1ull))] = avail[lane];
    }
    __syncthreads();

    // ---- decode over F -------------------------------------------------------------------
    decoder_weights(alpha_s, beta_s, F, nF, K, KP, sign_mode, WdT);
    __syncthreads();
    float *og = out + static_cast<size_t>(g) * K * C;
    for (int64_t cv0 = 0; cv0 < Cv; cv0 += kColsPerTile) {
        const int64_t cv1 = (cv0 + kColsPerTile < Cv) ? cv0 + kColsPerTile : Cv;
        typename PredVec<VEC>::type unused[kRowChunk];
        contract_tile<VEC, false>(pg, og, F, nF, K, KP, C, cv0, cv1, WdT, unused);
    }
}

bool aligned16(const void *p) { return reinterpret_cast<uintptr_t>(p) % 16 == 0; }

}  // namespace

int launch_decode(const float *d_preds, const uint8_t *d_mask, float *d_out, int32_t *d_status, int64_t G, int K,
                  int N, int S, int64_t C, const Nodes &nodes, int sign_mode, hipStream_t stream) {
    const int KP = (K + 3) & ~3;
    const bool vec4 = (C % 4 == 0) && aligned16(d_preds) && aligned16(d_out);
    const int64_t Cv = vec4 ? C / 4 : C;
    const int64_t ctiles = (Cv + kColsPerTile - 1) / kColsPerTile;
    const int64_t blocks = G * ctiles;
    if (blocks > 0x7fffffffLL) return APPROXIFER_ERR_LIMIT;
    int waves = KP / 4;
    if (waves > 4) waves = 4;
    const size_t lds = sizeof(double) * (static_cast<size_t>(S < 0 ? N : N - S) * KP + K + N) + sizeof(int) * (static_cast<size_t>(N) + 2);
    const dim3 grid(static_cast<unsigned>(blocks)), block(waves * kWave);
    if (lds > 64 * 1024) {   // only K = 64 with more than 127 survivors; gfx950 has 160 KB of LDS per CU
        const void *fn = vec4 ? reinterpret_cast<const void *>(decode_kernel<4>)
                              : reinterpret_cast<const void *>(decode_kernel<1>);
        if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds)) != hipSuccess)
            return APPROXIFER_ERR_LAUNCH;
    }
    if (vec4)
        hipLaunchKernelGGL(decode_kernel<4>, grid, block, lds, stream, d_preds, d_mask, d_out, d_status, K, N, S, C,
                           Cv, ctiles, sign_mode, nodes);
    else
        hipLaunchKernelGGL(decode_kernel<1>, grid, block, lds, stream, d_preds, d_mask, d_out, d_status, K, N, S, C,
                           Cv, ctiles, sign_mode, nodes);
    return hipGetLastError() == hipSuccess ? APPROXIFER_OK : APPROXIFER_ERR_LAUNCH;
}

int launch_decode_top1(const float *d_preds, const uint8_t *d_mask, int32_t *d_top1, float *d_score,
                       int32_t *d_status, int64_t G, int K, int N, int S, int64_t C, const Nodes &nodes,
                       int sign_mode, hipStream_t stream) {
    const int KP = (K + 3) & ~3;
    const bool vec4 = (C % 4 == 0) && aligned16(d_preds);
    const int64_t Cv = vec4 ? C / 4 : C;
    if (G > 0x7fffffffLL) return APPROXIFER_ERR_LIMIT;
    const int KQ = KP / 4;
    int slices = static_cast<int>((Cv + kWave - 1) / kWave);     // column slices worth a wave of their own
    if (slices > 4) slices = 4;
    if (slices * KQ > 16) slices = 16 / KQ;
    if (slices < 1) slices = 1;
    const int waves = KQ <= 16 ? KQ * slices : 16;
    // int F[N] | int n | 1 pad int  keeps the Best array that follows 16-byte aligned when N is even; round up
    size_t lds = sizeof(double) * (static_cast<size_t>(S < 0 ? N : N - S) * KP + K + N) + sizeof(int) * (static_cast<size_t>(N) + 3);
    lds += 16 + sizeof(double) * 2 * static_cast<size_t>(KP) * (waves >= KQ ? waves / KQ : 1);
    const dim3 grid(static_cast<unsigned>(G)), block(waves * kWave);
    if (lds > 64 * 1024) {
        const void *fn = vec4 ? reinterpret_cast<const void *>(decode_top1_kernel<4>)
                              : reinterpret_cast<const void *>(decode_top1_kernel<1>);
        if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds)) != hipSuccess)
            return APPROXIFER_ERR_LAUNCH;
    }
    if (vec4)
        hipLaunchKernelGGL(decode_top1_kernel<4>, grid, block, lds, stream, d_preds, d_mask, d_top1, d_score, d_status,
                           K, N, S, C, Cv, sign_mode, nodes);
    else
        hipLaunchKernelGGL(decode_top1_kernel<1>, grid, block, lds, stream, d_preds, d_mask, d_top1, d_score, d_status,
                           K, N, S, C, Cv, sign_mode, nodes);
    return hipGetLastError() == hipSuccess ? APPROXIFER_OK : APPROXIFER_ERR_LAUNCH;
}

int launch_decode_byzantine(const float *d_preds, const uint8_t *d_mask, float *d_out, int32_t *d_adv,
                            int32_t *d_status, int64_t G, int K, int N, int S, int A, int64_t C, const Nodes &nodes,
                            int sign_mode, hipStream_t stream) {
    const int KP = (K + 3) & ~3;
    const int n = S < 0 ? (N < APPROXIFER_MAX_AVAIL_BYZ ? N : APPROXIFER_MAX_AVAIL_BYZ) : N - S;   // capacity
    const int M = K + A;
    const bool vec4 = (C % 4 == 0) && aligned16(d_preds) && aligned16(d_out);
    const int64_t Cv = vec4 ? C / 4 : C;
    if (G > 0x7fffffffLL) return APPROXIFER_ERR_LIMIT;

    // classes per wave: a class takes 2M lanes; waves per workgroup: enough for all classes, at most 4
    int cpw = kWave / (2 * M);
    if (cpw < 1) cpw = 1;
    if (cpw > C) cpw = static_cast<int>(C);
    const size_t fixed = sizeof(double) * (static_cast<size_t>(n - A) * KP + n + K + N) + sizeof(int) * (4 * static_cast<size_t>(N) + 2);
    const size_t per_class = sizeof(double) * (static_cast<size_t>(n) * 2 * M + M + n);
    const size_t budget = 64 * 1024;
    while (cpw > 1 && fixed + cpw * per_class > budget) --cpw;
    const size_t per_wave = cpw * per_class;
    if (fixed + per_wave > budget) return APPROXIFER_ERR_LIMIT;
    int nw = static_cast<int>((C + cpw - 1) / cpw);
    if (nw > 4) nw = 4;
    if (nw > static_cast<int>((budget - fixed) / per_wave)) nw = static_cast<int>((budget - fixed) / per_wave);
    if (nw < 1) nw = 1;
    const size_t lds = fixed + nw * per_wave;
    const dim3 grid(static_cast<unsigned>(G)), block(nw * kWave);
    if (vec4)
        hipLaunchKernelGGL(decode_byzantine_kernel<4>, grid, block, lds, stream, d_preds, d_mask, d_out, d_adv,
                           d_status, K, N, S, A, C, Cv, sign_mode, cpw, nodes);
    else
        hipLaunchKernelGGL(decode_byzantine_kernel<1>, grid, block, lds, stream, d_preds, d_mask, d_out, d_adv,
                           d_status, K, N, S, A, C, Cv, sign_mode, cpw, nodes);
    return hipGetLastError() == hipSuccess ? APPROXIFER_OK : APPROXIFER_ERR_LAUNCH;
}

}  // namespace approxifer
