// Device helpers shared by the decoder, the fused top-1 decoder and the Byzantine decoder
// (Section 3, "ApproxIFER Decoding"): mask -> survivor list, decoder weights, node staging and
// the float64-accumulating contraction over the surviving workers.
#pragma once

#include "common.h"

namespace approxifer {

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
    __builtin_nontemporal_store(v, reinterpret_cast<v4f *>(dst));     // written once, not read again by this call
}
template <> __device__ __forceinline__ void store_row<1>(float *dst, const double *acc) {
    __builtin_nontemporal_store(static_cast<float>(acc[0]), dst);
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
        y[u] = __builtin_nontemporal_load(reinterpret_cast<const V *>(pg + static_cast<size_t>(F[r]) * C + cv * VEC));
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

inline bool aligned16(const void *p) { return reinterpret_cast<uintptr_t>(p) % 16 == 0; }

}  // namespace approxifer
