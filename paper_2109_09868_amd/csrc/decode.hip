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
// decoder kernel with all K accumulator rows in one wave (K <= 16, 16-byte rows)
// ------------------------------------------------------------------------------------
// decode_kernel gives every quad of queries a wave of its own, so each wave moves only a third or a quarter of a
// tile's bytes, and with the registers it needs four waves fit a SIMD, which bounds the bytes in flight.  Here ONE wave
// keeps the accumulators of all K <= 4 KQ queries for its 64 vector columns, as the encoder keeps its K inputs: it
// reads every surviving row once and writes all K output rows, three to four times the bytes in flight per wave, and
// a group's tile costs one wave's worth of prologue instead of K/4.  16-byte-aligned rows, K <= 16, up to 64
// survivors; measured against decode_kernel: 512 x 12 x 1000 classes 23.1 -> 20.7 us, 4096 x 8 x 100 classes
// 17.3 -> 13.8 us, 1.1 GB (K = 16, 4096 classes) 336 -> 235 us.
// UNAL: rows are only 4-byte aligned (C % 4 != 0 or offset tensors): the same 128-bit accesses through a
// 4-byte-aligned vector type, and the lane that holds a row's last, partial vector (C % 4 floats) moves it float
// by float.  Cv = ceil(C / 4) then counts that partial vector.
// dynamic LDS: as decode_kernel.
typedef v4f v4f_dword_aligned __attribute__((aligned(4)));

template <bool UNAL>
__device__ __forceinline__ v4f load_pred_vector(const float *p, int floats) {
    // every prediction is read once and every output written once: non-temporal accesses keep them out of the way of
    // the caches (measured on the streaming kernel: 49 MB cold 21.4 -> 17.5 us, 0.4 GB 105 -> 73 us, 1.1 GB +7..9 %)
    if (!UNAL) return __builtin_nontemporal_load(reinterpret_cast<const v4f *>(p));
    if (floats >= 4) return __builtin_nontemporal_load(reinterpret_cast<const v4f_dword_aligned *>(p));
    v4f v = v4f(0.0f);
    v[0] = p[0];
    if (floats > 1) v[1] = p[1];
    if (floats > 2) v[2] = p[2];
    return v;
}

template <int KQ, bool UNAL>
__global__ __launch_bounds__(kWave) void decode_stream_kernel(const float *__restrict__ preds,
                                                              const uint8_t *__restrict__ mask, float *__restrict__ out,
                                                              int32_t *__restrict__ status, int K, int N, int S, int64_t C,
                                                              int64_t Cv, int64_t ctiles, int sign_mode, const Nodes nodes) {
    constexpr int KP = 4 * KQ;
    extern __shared__ double lds_d[];
    const int nF_cap = S < 0 ? N : N - S;
    double *WdT = lds_d;
    double *alpha_s = WdT + nF_cap * KP;
    double *beta_s = alpha_s + K;
    int *F = reinterpret_cast<int *>(beta_s + N);

    const int64_t g = blockIdx.x / ctiles;
    const int64_t ct = blockIdx.x - g * ctiles;
    const int lane = threadIdx.x;

    stage_nodes(nodes, K, N, alpha_s, beta_s);
    for (int e = lane; e < nF_cap * KP; e += kWave) WdT[e] = 0.0;
    const int nF = survivors_from_mask(mask + g * N, N, F);
    __syncthreads();
    const bool good = S < 0 ? nF >= 1 : nF == nF_cap;
    if (ct == 0 && lane == 0 && status != nullptr) status[g] = good ? APPROXIFER_GROUP_OK : APPROXIFER_GROUP_BAD_MASK;
    if (!good) return;

    const int64_t cv_raw = ct * kColsPerTile + lane;
    const bool ok = cv_raw < Cv;
    const int64_t cv = ok ? cv_raw : ct * kColsPerTile;    // lanes past the ragged end read the tile's first column
    const int floats = (UNAL && C - 4 * cv < 4) ? static_cast<int>(C - 4 * cv) : 4;   // of this lane's vector
    const float *pg = preds + static_cast<size_t>(g) * N * C + 4 * cv;
    v4f y[kRowChunk];
#pragma unroll
    for (int u = 0; u < kRowChunk; ++u)                    // in flight while the weights are evaluated
        y[u] = load_pred_vector<UNAL>(pg + static_cast<size_t>(F[u < nF ? u : nF - 1]) * C, floats);

    decoder_weights(alpha_s, beta_s, F, nF, K, KP, sign_mode, WdT);
    __syncthreads();

    double acc[KP][4];
#pragma unroll
    for (int j = 0; j < KP; ++j)
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[j][e] = 0.0;
    for (int r0 = 0; r0 < nF; r0 += kRowChunk) {
        if (r0 > 0) {
#pragma unroll
            for (int u = 0; u < kRowChunk; ++u)
                y[u] = load_pred_vector<UNAL>(pg + static_cast<size_t>(F[r0 + u < nF ? r0 + u : nF - 1]) * C, floats);
        }
#pragma unroll
        for (int u = 0; u < kRowChunk; ++u) {
            if (r0 + u < nF) {
                const double *w = WdT + (r0 + u) * KP;
                const double y0 = y[u][0], y1 = y[u][1], y2 = y[u][2], y3 = y[u][3];
#pragma unroll
                for (int j = 0; j < KP; ++j) {
                    const double wj = w[j];
                    acc[j][0] = fma(wj, y0, acc[j][0]);
                    acc[j][1] = fma(wj, y1, acc[j][1]);
                    acc[j][2] = fma(wj, y2, acc[j][2]);
                    acc[j][3] = fma(wj, y3, acc[j][3]);
                }
            }
        }
    }
    if (!ok) return;
    float *og = out + static_cast<size_t>(g) * K * C + cv * 4;
#pragma unroll
    for (int j = 0; j < KP; ++j) {
        if (j < K) {
            float *dst = og + static_cast<size_t>(j) * C;
            if (!UNAL) {
                store_row<4>(dst, acc[j]);
            } else if (floats >= 4) {
                v4f v;
                v[0] = static_cast<float>(acc[j][0]);
                v[1] = static_cast<float>(acc[j][1]);
                v[2] = static_cast<float>(acc[j][2]);
                v[3] = static_cast<float>(acc[j][3]);
                __builtin_nontemporal_store(static_cast<v4f_dword_aligned>(v), reinterpret_cast<v4f_dword_aligned *>(dst));
            } else {
                dst[0] = static_cast<float>(acc[j][0]);
                if (floats > 1) dst[1] = static_cast<float>(acc[j][1]);
                if (floats > 2) dst[2] = static_cast<float>(acc[j][2]);
            }
        }
    }
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
                                   int sign_mode, int qsplit, const Nodes nodes) {
    typedef typename PredVec<VEC>::type V;
    extern __shared__ double lds_d[];
    const int KP = round_up4(K);
    const int nF_cap = S < 0 ? N : N - S;          // S < 0: every group brings its own straggler count
    double *WdT = lds_d;
    double *alpha_s = WdT + nF_cap * KP;
    double *beta_s = alpha_s + K;
    int *F = reinterpret_cast<int *>(beta_s + N);
    int *n_sh = F + N;
    // qsplit > 1 (few groups, very many classes): qsplit = KP/4 workgroups share a group, one quad of queries each
    const int64_t g = blockIdx.x / qsplit;
    const int qpart = static_cast<int>(blockIdx.x - g * qsplit);

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
    const bool one_quad = qsplit > 1;                           // this workgroup: quad qpart only, every wave a slice
    const int slices = one_quad ? nwaves : (nwaves >= KQ ? nwaves / KQ : 1);   // waves that share one quad split its columns
    const int qwaves = one_quad ? 1 : (nwaves >= KQ ? KQ : nwaves);            // quads processed concurrently
    const int slice = wave_id() / qwaves;
    Best *merged = reinterpret_cast<Best *>((reinterpret_cast<uintptr_t>(n_sh + 1) + 15) & ~static_cast<uintptr_t>(15));   // [KP][slices]
    for (int q = one_quad ? qpart : wave_id() % qwaves; q < KQ && slice < slices; q += one_quad ? KQ : qwaves) {
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
    const int j_first = one_quad ? 4 * qpart : 0;
    const int j_end = one_quad ? (4 * qpart + 4 < K ? 4 * qpart + 4 : K) : K;
    for (int j = j_first + threadIdx.x; j < j_end; j += blockDim.x) {
        Best b = merged[j * slices];
        for (int sl = 1; sl < slices; ++sl) {
            const Best o = merged[j * slices + sl];
            if (better(o.v, o.i, b)) b = o;
        }
        top1[g * K + j] = b.i == 0x7fffffff ? 0 : b.i;
        if (score != nullptr) score[g * K + j] = static_cast<float>(b.v);
    }
}

// one step of a (value, class) maximum inside the 16-lane rows: larger value first, equal values: smaller class
template <int CTRL>
__device__ __forceinline__ void best_step(Best &b) {
    const double ov = dpp_exchange<CTRL>(b.v);
    const int oi = __builtin_amdgcn_update_dpp(0, b.i, CTRL, 0xF, 0xF, true);
    if (better(ov, oi, b)) {
        b.v = ov;
        b.i = oi;
    }
}

// ------------------------------------------------------------------------------------
// fused decoder + top-1 with all K accumulator rows in one wave (K <= 16, up to 64 survivors)
// ------------------------------------------------------------------------------------
// One workgroup per group; its waves take the column tiles wave, wave + nwaves, .. and each keeps, per lane, the
// float64 accumulators of all K queries for four columns and the best (value, class) seen so far for every query.
// Nothing is stored inside the tile loop, so the next tile's loads are not held up by stores.  At the end a
// butterfly merges the lanes, LDS merges the waves.  Ties: the smaller class index.
// dynamic LDS: as decode_kernel, then pad to 16 bytes | Best merged[KP][nwaves].
template <int KQ, bool UNAL>
__global__ __launch_bounds__(256) void decode_top1_stream_kernel(const float *__restrict__ preds,
                                                                  const uint8_t *__restrict__ mask,
                                                                  int32_t *__restrict__ top1, float *__restrict__ score,
                                                                  int32_t *__restrict__ status, int K, int N, int S,
                                                                  int64_t C, int64_t Cv, int64_t ctiles, int sign_mode,
                                                                  const Nodes nodes) {
    constexpr int KP = 4 * KQ;
    extern __shared__ double lds_d[];
    const int nF_cap = S < 0 ? N : N - S;
    double *WdT = lds_d;
    double *alpha_s = WdT + nF_cap * KP;
    double *beta_s = alpha_s + K;
    int *F = reinterpret_cast<int *>(beta_s + N);
    int *n_sh = F + N;
    Best *merged = reinterpret_cast<Best *>((reinterpret_cast<uintptr_t>(n_sh + 1) + 15) & ~static_cast<uintptr_t>(15));
    const int64_t g = blockIdx.x;
    const int lane = lane_id();
    const int wv = wave_id();
    const int nwaves = blockDim.x / kWave;

    stage_nodes(nodes, K, N, alpha_s, beta_s);
    for (int e = threadIdx.x; e < nF_cap * KP; e += blockDim.x) WdT[e] = 0.0;
    if (wv == 0) {
        const int n = survivors_from_mask(mask + g * N, N, F);
        if (lane == 0) *n_sh = n;
    }
    __syncthreads();
    const int nF = *n_sh;
    const bool good = S < 0 ? nF >= 1 : nF == nF_cap;
    if (threadIdx.x == 0 && status != nullptr) status[g] = good ? APPROXIFER_GROUP_OK : APPROXIFER_GROUP_BAD_MASK;
    if (!good) return;

    const float *pgroup = preds + static_cast<size_t>(g) * N * C;
    // first tile of this wave: its first rows are in flight while the weights are evaluated
    v4f y[kRowChunk];
    {
        const int64_t cv_raw = static_cast<int64_t>(wv) * kColsPerTile + lane;
        const int64_t cv = cv_raw < Cv ? cv_raw : 0;
        const int floats = (UNAL && C - 4 * cv < 4) ? static_cast<int>(C - 4 * cv) : 4;
#pragma unroll
        for (int u = 0; u < kRowChunk; ++u)
            y[u] = load_pred_vector<UNAL>(pgroup + 4 * cv + static_cast<size_t>(F[u < nF ? u : nF - 1]) * C, floats);
    }
    decoder_weights(alpha_s, beta_s, F, nF, K, KP, sign_mode, WdT);
    __syncthreads();

    Best best[KP];
#pragma unroll
    for (int j = 0; j < KP; ++j) {
        best[j].v = -__builtin_inf();
        best[j].i = 0x7fffffff;
    }
    for (int64_t ct = wv; ct < ctiles; ct += nwaves) {
        const int64_t cv_raw = ct * kColsPerTile + lane;
        const bool ok = cv_raw < Cv;
        const int64_t cv = ok ? cv_raw : 0;
        const int floats = (UNAL && C - 4 * cv < 4) ? static_cast<int>(C - 4 * cv) : 4;
        const float *pg = pgroup + 4 * cv;
        double acc[KP][4];
#pragma unroll
        for (int j = 0; j < KP; ++j)
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[j][e] = 0.0;
        for (int r0 = 0; r0 < nF; r0 += kRowChunk) {
            if (r0 > 0 || ct != wv) {
#pragma unroll
                for (int u = 0; u < kRowChunk; ++u)
                    y[u] = load_pred_vector<UNAL>(pg + static_cast<size_t>(F[r0 + u < nF ? r0 + u : nF - 1]) * C, floats);
            }
#pragma unroll
            for (int u = 0; u < kRowChunk; ++u) {
                if (r0 + u < nF) {
                    const double *w = WdT + (r0 + u) * KP;
                    const double y0 = y[u][0], y1 = y[u][1], y2 = y[u][2], y3 = y[u][3];
#pragma unroll
                    for (int j = 0; j < KP; ++j) {
                        const double wj = w[j];
                        acc[j][0] = fma(wj, y0, acc[j][0]);
                        acc[j][1] = fma(wj, y1, acc[j][1]);
                        acc[j][2] = fma(wj, y2, acc[j][2]);
                        acc[j][3] = fma(wj, y3, acc[j][3]);
                    }
                }
            }
        }
        if (ok) {
#pragma unroll
            for (int j = 0; j < KP; ++j)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int idx = static_cast<int>(cv * 4 + e);
                    if (e < floats && better(acc[j][e], idx, best[j])) {
                        best[j].v = acc[j][e];
                        best[j].i = idx;
                    }
                }
        }
    }
#pragma unroll
    for (int j = 0; j < KP; ++j) {
        // the wave's best: four DPP steps inside each row of 16 lanes, then the four rows by v_readlane
        best_step<kDppQuadXor1>(best[j]);
        best_step<kDppQuadXor2>(best[j]);
        best_step<kDppRowHalfMirror>(best[j]);
        best_step<kDppRowMirror>(best[j]);
        Best b = best[j];
        b.v = read_lane(best[j].v, 0);
        b.i = __builtin_amdgcn_readlane(best[j].i, 0);
#pragma unroll
        for (int row = 1; row < 4; ++row) {
            const double ov = read_lane(best[j].v, 16 * row);
            const int oi = __builtin_amdgcn_readlane(best[j].i, 16 * row);
            if (better(ov, oi, b)) {
                b.v = ov;
                b.i = oi;
            }
        }
        if (lane == 0) merged[j * nwaves + wv] = b;
    }
    __syncthreads();
    for (int j = threadIdx.x; j < K; j += blockDim.x) {
        Best b = merged[j * nwaves];
        for (int w2 = 1; w2 < nwaves; ++w2) {
            const Best o = merged[j * nwaves + w2];
            if (better(o.v, o.i, b)) b = o;
        }
        top1[g * K + j] = b.i == 0x7fffffff ? 0 : b.i;
        if (score != nullptr) score[g * K + j] = static_cast<float>(b.v);
    }
}

// ------------------------------------------------------------------------------------
// packed kernel for the small shapes of the image-classification operating points
// ------------------------------------------------------------------------------------
// K <= KT queries, at most RT surviving workers, C <= 16 classes, (KT, RT) = (16, 16), (16, 32) or (32, 64) (e.g.
// K = 8..12, one to three stragglers, ten classes; K = 16 with 18 of 24 workers and K = 32 with 36 of 48, two classes).  A group is then a few hundred bytes, and a workgroup per group spends its time on launch
// and barrier latency.  Here ONE WAVE decodes a group on its own -- four (two for the largest tile) groups per workgroup, the only
// workgroup barrier is the one after the nodes are staged -- with everything in 16 x 16 tiles in the wave's
// own LDS: survivors from one ballot, predictions Y[r][c], weights W[j][r] (RT lanes per query node, 64 / RT
// nodes per pass), then one lane per output (j, c).  TOP1 adds the argmax over classes.
constexpr int kPk = 16;                 // tile edge for C (and for K in the smaller tiles)

template <bool TOP1, int KT, int RT, int GROUPS>
__global__ __launch_bounds__(GROUPS *kWave) void decode_packed_kernel(
    const float *__restrict__ preds, const uint8_t *__restrict__ mask, float *__restrict__ out,
    int32_t *__restrict__ top1, float *__restrict__ score, int32_t *__restrict__ status, int64_t G, int K, int N,
    int S, int C, int sign_mode, const Nodes nodes) {
    static_assert((KT == 16 && (RT == 16 || RT == 32)) || (KT == 32 && RT == 64), "tile");
    __shared__ double alpha_s[KT];
    __shared__ double beta_s[kWave];
    __shared__ double W_s[GROUPS][KT * RT];            // W[j][r]
    __shared__ double O_s[TOP1 ? GROUPS : 1][KT * kPk];
    __shared__ float Y_s[GROUPS][RT * kPk];            // Y[r][c]
    __shared__ int F_s[GROUPS][RT];

    const int lane = lane_id();
    const int wv = wave_id();
    for (int t = threadIdx.x; t < K + N; t += blockDim.x) {
        if (t < K) alpha_s[t] = nodes.alpha[t];
        else beta_s[t - K] = nodes.beta[t - K];
    }
    __syncthreads();
    const int64_t g = static_cast<int64_t>(blockIdx.x) * GROUPS + wv;
    if (g >= G) return;

    double *W = W_s[wv];
    float *Y = Y_s[wv];
    int *F = F_s[wv];

    // survivors: N <= 64, one ballot
    const bool mine = lane < N && mask[g * N + lane] != 0;
    const unsigned long long m = __ballot(mine);
    const int nF = __popcll(m);
    const bool good = S < 0 ? (nF >= 1 && nF <= RT) : nF == N - S;
    if (lane == 0 && status != nullptr) status[g] = good ? APPROXIFER_GROUP_OK : APPROXIFER_GROUP_BAD_MASK;
    if (!good) return;
    if (mine) F[__popcll(m & ((1ull << lane) - 1ull))] = lane;
    __builtin_amdgcn_wave_barrier();

    // predictions of the survivors: slot (r, c) = (slot / 16, slot % 16), RT / 4 slots per lane
    constexpr int kYSlots = RT / 4;
    const float *pg = preds + static_cast<size_t>(g) * N * C;
    float yv[kYSlots];
#pragma unroll
    for (int u = 0; u < kYSlots; ++u) {
        const int slot = lane + u * kWave;
        const int r = slot / kPk, c = slot % kPk;
        yv[u] = (r < nF && c < C) ? pg[static_cast<size_t>(F[r]) * C + c] : 0.0f;
    }

    // weights, Section 3 "ApproxIFER Decoding" step 2: lanes (jsub, r) = (lane / RT, lane % RT)
    {
        constexpr int kRowsPerPass = kWave / RT;
        const int r = lane % RT, jsub = lane / RT;
        const bool valid = r < nF;
        const int i = valid ? F[r] : 0;
        const double xb = beta_s[i];
        const int parity = (sign_mode == APPROXIFER_SIGN_WORKER_INDEX) ? (i & 1) : (r & 1);
        const double sign = parity ? -1.0 : 1.0;
        const unsigned long long group_mask = RT == 64 ? ~0ull : (RT == 16 ? 0xFFFFull : 0xFFFFFFFFull) << (jsub * (RT & 63));
#pragma unroll
        for (int p = 0; p < KT / kRowsPerPass; ++p) {
            if (kRowsPerPass * p < K) {
                const int j = kRowsPerPass * p + jsub;
                const bool row = j < K;
                const BerrutTerm bt = berrut_term(alpha_s[row ? j : 0], xb, sign, valid && row);
                const double rden = 1.0 / group_sum<RT>(bt.t);
                const bool any_hit = (__ballot(bt.hit) & group_mask) != 0ull;
                W[j * RT + r] = (valid && row) ? (any_hit ? (bt.hit ? 1.0 : 0.0) : bt.t * rden) : 0.0;
            }
        }
    }
#pragma unroll
    for (int u = 0; u < kYSlots; ++u) Y[lane + u * kWave] = yv[u];
    __builtin_amdgcn_wave_barrier();

    // one lane per output (j, c) = (slot / 16, slot % 16); float64 accumulation, one rounding
    const int nF4 = (nF + 3) & ~3;                       // rows nF.. of W and Y are zero
    float *og = out + static_cast<size_t>(g) * K * C;
#pragma unroll
    for (int u = 0; u < KT / 4; ++u) {
        if (u * 4 < K) {
            const int slot = lane + u * kWave;
            const int j = slot / kPk, c = slot % kPk;
            double acc = 0.0;
#pragma unroll
            for (int r0 = 0; r0 < RT; r0 += 4) {
                if (r0 < nF4) {
#pragma unroll
                    for (int r = r0; r < r0 + 4; ++r)
                        acc = fma(W[j * RT + r], static_cast<double>(Y[r * kPk + c]), acc);
                }
            }
            if (TOP1) O_s[TOP1 ? wv : 0][slot] = acc;
            else if (j < K && c < C) og[j * C + c] = static_cast<float>(acc);
        }
    }
    if (TOP1) {
        __builtin_amdgcn_wave_barrier();
        if (lane < K) {                                   // largest value, smallest class on equal values
            const double *o = O_s[TOP1 ? wv : 0] + lane * kPk;
            double bv = o[0];
            int bi = 0;
            for (int c = 1; c < C; ++c) {
                const double v = o[c];
                if (v > bv) {
                    bv = v;
                    bi = c;
                }
            }
            top1[g * K + lane] = bi;
            if (score != nullptr) score[g * K + lane] = static_cast<float>(bv);
        }
    }
}

// ------------------------------------------------------------------------------------
// wait rule: arrival times -> survivor mask
// ------------------------------------------------------------------------------------
// One wave per group, four groups per workgroup; a lane owns workers lane and lane + 64.  The rank of a
// worker is the number of workers that answer before it (equal times: smaller index first), counted
// against the group's times broadcast from the wave's LDS; the wait_for lowest ranks are the survivors.
constexpr int kWaitGroups = 4;

__global__ __launch_bounds__(kWaitGroups *kWave) void wait_mask_kernel(const float *__restrict__ arrival,
                                                                         uint8_t *__restrict__ mask,
                                                                         int32_t *__restrict__ count, int64_t G, int N,
                                                                         int wait_for) {
    __shared__ float t_s[kWaitGroups][APPROXIFER_MAX_N];
    const int lane = lane_id();
    const int wv = wave_id();
    const int64_t g = static_cast<int64_t>(blockIdx.x) * kWaitGroups + wv;
    if (g >= G) return;
    float *t = t_s[wv];
    const float never = __builtin_inff();
    float mine[2];
#pragma unroll
    for (int p = 0; p < 2; ++p) {
        const int i = lane + p * kWave;
        float v = never;
        if (i < N) {
            v = arrival[g * N + i];
            if (!(fabsf(v) < never)) v = never;           // NaN and both infinities: never answers
            t[i] = v;
        }
        mine[p] = v;
    }
    __builtin_amdgcn_wave_barrier();
    int total = 0;
#pragma unroll
    for (int p = 0; p < 2; ++p) {
        const int i = lane + p * kWave;
        int rank = 0;
#pragma unroll 8
        for (int o = 0; o < N; ++o) {
            const float other = t[o];
            rank += (other < mine[p] || (other == mine[p] && o < i)) ? 1 : 0;
        }
        const bool in = i < N && mine[p] < never && rank < wait_for;
        if (i < N) mask[g * N + i] = in ? 1 : 0;
        total += __popcll(__ballot(in));
    }
    if (lane == 0 && count != nullptr) count[g] = total;
}

// ------------------------------------------------------------------------------------
// top-1 of an already decoded tensor
// ------------------------------------------------------------------------------------
// LPR lanes per row of [rows][C] float32 (a wave for long rows, sixteen lanes for rows of up to 32 classes, so that a
// wave takes four rows of a ten-class output instead of idling 54 lanes on one): largest value, smallest class on
// equal values (NaN never wins; a row of NaNs gives class 0).  Four waves per workgroup.
constexpr int kArgmaxWaves = 4;

template <int LPR>
__global__ __launch_bounds__(kArgmaxWaves *kWave) void argmax_rows_kernel(const float *__restrict__ values,
                                                                           int32_t *__restrict__ top1,
                                                                           float *__restrict__ score, int64_t rows,
                                                                           int64_t C) {
    constexpr int kRowsPerWave = kWave / LPR;
    const int lane = lane_id();
    const int64_t row = (static_cast<int64_t>(blockIdx.x) * kArgmaxWaves + wave_id()) * kRowsPerWave + lane / LPR;
    const bool live = row < rows;
    const float *v = values + (live ? row : 0) * C;
    float bv = -__builtin_inff();
    int bi = 0x7fffffff;
    for (int64_t c = lane % LPR; c < C; c += LPR) {
        const float x = v[c];
        if (x > bv) {                                       // ascending c: the first occurrence stays
            bv = x;
            bi = static_cast<int>(c);
        }
    }
#pragma unroll
    for (int off = LPR / 2; off >= 1; off >>= 1) {
        const float ov = __shfl_xor(bv, off, kWave);
        const int oi = __shfl_xor(bi, off, kWave);
        if (ov > bv || (ov == bv && oi < bi)) {
            bv = ov;
            bi = oi;
        }
    }
    if (live && lane % LPR == 0) {
        const bool none = bi == 0x7fffffff;                 // every value NaN or -inf
        top1[row] = none ? 0 : bi;
        if (score != nullptr) score[row] = none ? v[0] : bv;
    }
}

bool packed_shape(int K, int N, int64_t C) {
    return K <= 32 && N <= kWave && C <= kPk;             // N <= 64: the survivors fit the largest tile
}

int run_packed(bool top1_variant, const float *d_preds, const uint8_t *d_mask, float *d_out, int32_t *d_top1,
               float *d_score, int32_t *d_status, int64_t G, int K, int N, int S, int64_t C, const Nodes &nodes,
               int sign_mode, hipStream_t stream) {
    const int most_survivors = S < 0 ? N : N - S;
    // the smallest tile (queries, survivors) that holds the shape; the largest takes two groups per workgroup
    const int tile = (K <= 16 && most_survivors <= 16) ? 0 : ((K <= 16 && most_survivors <= 32) ? 1 : 2);
    const int groups = tile == 2 ? 2 : 4;
    const int64_t blocks = (G + groups - 1) / groups;
    if (blocks > 0x7fffffffLL) return APPROXIFER_ERR_LIMIT;
    const dim3 grid(static_cast<unsigned>(blocks)), block(groups * kWave);
#define APPROXIFER_PACKED(TOP1, KT, RT, GROUPS)                                                                        \
    launch_status(launch_kernel(decode_packed_kernel<TOP1, KT, RT, GROUPS>, grid, block, 0, stream, d_preds, d_mask,     \
                                d_out, d_top1, d_score, d_status, G, K, N, S, static_cast<int>(C), sign_mode, nodes))
    if (top1_variant) {
        if (tile == 0) return APPROXIFER_PACKED(true, 16, 16, 4);
        if (tile == 1) return APPROXIFER_PACKED(true, 16, 32, 4);
        return APPROXIFER_PACKED(true, 32, 64, 2);
    }
    if (tile == 0) return APPROXIFER_PACKED(false, 16, 16, 4);
    if (tile == 1) return APPROXIFER_PACKED(false, 16, 32, 4);
    return APPROXIFER_PACKED(false, 32, 64, 2);
#undef APPROXIFER_PACKED
}

}  // namespace

int launch_decode(const float *d_preds, const uint8_t *d_mask, float *d_out, int32_t *d_status, int64_t G, int K,
                  int N, int S, int64_t C, const Nodes &nodes, int sign_mode, hipStream_t stream) {
    if (packed_shape(K, N, C))
        return run_packed(false, d_preds, d_mask, d_out, nullptr, nullptr, d_status, G, K, N, S, C, nodes, sign_mode, stream);
    const int KP = (K + 3) & ~3;
    const bool vec4 = (C % 4 == 0) && aligned16(d_preds) && aligned16(d_out);
    const int64_t Cv = vec4 ? C / 4 : C;
    const int64_t ctiles = (Cv + kColsPerTile - 1) / kColsPerTile;
    const int64_t blocks = G * ctiles;
    if (blocks > 0x7fffffffLL) return APPROXIFER_ERR_LIMIT;
    int waves = KP / 4;
    if (waves > 4) waves = 4;
    const size_t lds = sizeof(double) * (static_cast<size_t>(S < 0 ? N : N - S) * KP + K + N) + sizeof(int) * (static_cast<size_t>(N) + 2);
    // K <= 16, up to 64 survivors: one wave per tile with all K accumulator rows (faster at every size measured, 26 MB
    // to 1.1 GB; capping its residency as in the encoder changes nothing: 4 to 12 waves per CU +-3 %)
    const int most_survivors = S < 0 ? N : N - S;
    if (K <= 16 && most_survivors <= 64 && C >= 4) {
        const int64_t sCv = (C + 3) / 4;                  // counts a partial last vector
        const int64_t stiles = (sCv + kColsPerTile - 1) / kColsPerTile;
        if (G * stiles > 0x7fffffffLL) return APPROXIFER_ERR_LIMIT;
        const dim3 sgrid(static_cast<unsigned>(G * stiles)), sblock(kWave);
#define APPROXIFER_STREAM(KQ, UNAL)                                                                                    \
    launch_status(launch_kernel(decode_stream_kernel<KQ, UNAL>, sgrid, sblock, lds, stream, d_preds, d_mask, d_out,       \
                                d_status, K, N, S, C, sCv, stiles, sign_mode, nodes))
        switch (KP / 4) {
            case 1: return vec4 ? APPROXIFER_STREAM(1, false) : APPROXIFER_STREAM(1, true);
            case 2: return vec4 ? APPROXIFER_STREAM(2, false) : APPROXIFER_STREAM(2, true);
            case 3: return vec4 ? APPROXIFER_STREAM(3, false) : APPROXIFER_STREAM(3, true);
            default: return vec4 ? APPROXIFER_STREAM(4, false) : APPROXIFER_STREAM(4, true);
        }
#undef APPROXIFER_STREAM
    }
    const dim3 grid(static_cast<unsigned>(blocks)), block(waves * kWave);
    if (lds > 64 * 1024) {   // only K = 64 with more than 127 survivors; gfx950 has 160 KB of LDS per CU
        const void *fn = vec4 ? reinterpret_cast<const void *>(decode_kernel<4>)
                              : reinterpret_cast<const void *>(decode_kernel<1>);
        if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds)) != hipSuccess)
            return APPROXIFER_ERR_LAUNCH;
    }
    return launch_status(launch_kernel(vec4 ? decode_kernel<4> : decode_kernel<1>, grid, block, lds, stream, d_preds, d_mask,
                                       d_out, d_status, K, N, S, C, Cv, ctiles, sign_mode, nodes));
}

int launch_decode_top1(const float *d_preds, const uint8_t *d_mask, int32_t *d_top1, float *d_score,
                       int32_t *d_status, int64_t G, int K, int N, int S, int64_t C, const Nodes &nodes,
                       int sign_mode, hipStream_t stream) {
    if (packed_shape(K, N, C))
        return run_packed(true, d_preds, d_mask, nullptr, d_top1, d_score, d_status, G, K, N, S, C, nodes, sign_mode, stream);
    const int KP = (K + 3) & ~3;
    const bool vec4 = (C % 4 == 0) && aligned16(d_preds);
    const int64_t Cv = vec4 ? C / 4 : C;
    if (G > 0x7fffffffLL) return APPROXIFER_ERR_LIMIT;
    const int KQ = KP / 4;
    // K <= 16, up to 64 survivors, enough groups to fill the chip: a workgroup per group whose waves keep all K
    // accumulator rows (few groups with very many classes stay with the quad-per-workgroup split below)
    if (K <= 16 && (S < 0 ? N : N - S) <= 64 && C >= 4 && !(G * KQ <= 512 && (C + 3) / 4 >= 64 * 16)) {
        const int64_t sCv = (C + 3) / 4;
        const int64_t stiles = (sCv + kColsPerTile - 1) / kColsPerTile;
        const int nwaves = stiles < 4 ? static_cast<int>(stiles) : 4;
        size_t slds = sizeof(double) * (static_cast<size_t>(S < 0 ? N : N - S) * KP + K + N) + sizeof(int) * (static_cast<size_t>(N) + 3);
        slds += 16 + sizeof(double) * 2 * static_cast<size_t>(KP) * nwaves;
        const dim3 sgrid(static_cast<unsigned>(G)), sblock(nwaves * kWave);
#define APPROXIFER_TOP1_STREAM(KQV, UNAL)                                                                              \
    launch_status(launch_kernel(decode_top1_stream_kernel<KQV, UNAL>, sgrid, sblock, slds, stream, d_preds, d_mask,       \
                                d_top1, d_score, d_status, K, N, S, C, sCv, stiles, sign_mode, nodes))
        switch (KQ) {
            case 1: return vec4 ? APPROXIFER_TOP1_STREAM(1, false) : APPROXIFER_TOP1_STREAM(1, true);
            case 2: return vec4 ? APPROXIFER_TOP1_STREAM(2, false) : APPROXIFER_TOP1_STREAM(2, true);
            case 3: return vec4 ? APPROXIFER_TOP1_STREAM(3, false) : APPROXIFER_TOP1_STREAM(3, true);
            default: return vec4 ? APPROXIFER_TOP1_STREAM(4, false) : APPROXIFER_TOP1_STREAM(4, true);
        }
#undef APPROXIFER_TOP1_STREAM
    }
    int slices = static_cast<int>((Cv + kWave - 1) / kWave);     // column slices worth a wave of their own
    const int most = G >= 512 ? 4 : 16;                          // few groups: all sixteen waves of a workgroup
    if (slices > most) slices = most;
    if (slices * KQ > 16) slices = 16 / KQ;
    if (slices < 1) slices = 1;
    int waves = KQ <= 16 ? KQ * slices : 16;
    // Few groups and very many classes (vocabulary-sized predictions in a small batch): a workgroup per quad of
    // queries, all sixteen waves slicing the columns.  Every workgroup reads all surviving rows; with so few
    // groups they come from the cache.
    int qsplit = 1;
    if (G * KQ <= 512 && KQ >= 2 && Cv >= 64 * 16) {
        qsplit = KQ;
        waves = 16;
    }
    const int lds_slices = qsplit > 1 ? waves : (waves >= KQ ? waves / KQ : 1);
    // int F[N] | int n | 1 pad int  keeps the Best array that follows 16-byte aligned when N is even; round up
    size_t lds = sizeof(double) * (static_cast<size_t>(S < 0 ? N : N - S) * KP + K + N) + sizeof(int) * (static_cast<size_t>(N) + 3);
    lds += 16 + sizeof(double) * 2 * static_cast<size_t>(KP) * lds_slices;
    const dim3 grid(static_cast<unsigned>(G * qsplit)), block(waves * kWave);
    if (lds > 64 * 1024) {
        const void *fn = vec4 ? reinterpret_cast<const void *>(decode_top1_kernel<4>)
                              : reinterpret_cast<const void *>(decode_top1_kernel<1>);
        if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds)) != hipSuccess)
            return APPROXIFER_ERR_LAUNCH;
    }
    return launch_status(launch_kernel(vec4 ? decode_top1_kernel<4> : decode_top1_kernel<1>, grid, block, lds, stream,
                                       d_preds, d_mask, d_top1, d_score, d_status, K, N, S, C, Cv, sign_mode, qsplit, nodes));
}

int launch_argmax_rows(const float *d_values, int32_t *d_top1, float *d_score, int64_t rows, int64_t C,
                       hipStream_t stream) {
    const bool narrow = C <= 32;
    const int64_t per_block = kArgmaxWaves * (narrow ? kWave / 16 : 1);
    const int64_t blocks = (rows + per_block - 1) / per_block;
    if (blocks > 0x7fffffffLL) return APPROXIFER_ERR_LIMIT;
    const dim3 grid(static_cast<unsigned>(blocks)), block(kArgmaxWaves * kWave);
    if (narrow) return launch_status(launch_kernel(argmax_rows_kernel<16>, grid, block, 0, stream, d_values, d_top1, d_score, rows, C));
    return launch_status(launch_kernel(argmax_rows_kernel<kWave>, grid, block, 0, stream, d_values, d_top1, d_score, rows, C));
}

int launch_wait_mask(const float *d_arrival, uint8_t *d_mask, int32_t *d_count, int64_t G, int N, int wait_for,
                     hipStream_t stream) {
    const int64_t blocks = (G + kWaitGroups - 1) / kWaitGroups;
    if (blocks > 0x7fffffffLL) return APPROXIFER_ERR_LIMIT;
    return launch_status(launch_kernel(wait_mask_kernel, dim3(static_cast<unsigned>(blocks)), dim3(kWaitGroups * kWave), 0,
                                       stream, d_arrival, d_mask, d_count, G, N, wait_for));
}

}  // namespace approxifer
