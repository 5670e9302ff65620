// ApproxIFER decoder and fused decoder + top-1 for gfx950 (Section 3, "ApproxIFER Decoding").
//
// One workgroup per (group, tile of prediction columns).  The group's mask is turned into the
// ascending survivor list F with wavefront ballots, the K x |F| matrix of basis functions is
// evaluated in float64 (a group of lanes per query node, the denominator by a wavefront
// reduction) and kept transposed in LDS, and the contraction over F accumulates in float64
// with the weights broadcast from LDS.  Rows of missing workers are never read.
#include "decode_common.h"

namespace approxifer {
namespace {

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

}  // namespace approxifer
