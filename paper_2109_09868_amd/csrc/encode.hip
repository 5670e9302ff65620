// ApproxIFER encoder for gfx950 (Section 3, "ApproxIFER Encoding").
//
//   coded[g][i][d] = sum_j l_j(beta_i) * queries[g][j][d]
//
// One workgroup per (group, tile of 256 vector columns).  Each lane first issues the loads of
// its vector column of all K queries (they stay in registers), and while those are in flight
// the workgroup evaluates the N x K matrix l_j(beta_i) -- it depends on the nodes only --
// in float64 (one 16/32/64-lane group per worker row, the row's denominator by a DPP
// reduction) and keeps it in LDS as float32.  The N coded values of the column are then formed
// one worker at a time with the weights broadcast from LDS and stored as soon as complete.
// Every query element is read from HBM exactly once and every coded element written exactly
// once: the kernel is an HBM stream of 4*D*(K+N) bytes per group with 2*K*N flops per
// 4*(K+N) bytes on top.  Workgroups do not loop over tiles: a wave that has issued its
// stores retires at once instead of waiting for them before its next loads, which measured
// 9 % faster than a persistent grid.
#include "common.h"

namespace approxifer {
namespace {

constexpr int kEncodeThreads = 256;

template <int VEC> struct VecOf;
template <> struct VecOf<4> { typedef v4f type; };
template <> struct VecOf<2> { typedef v2f type; };
template <> struct VecOf<1> { typedef float type; };

template <int VEC>
__device__ __forceinline__ typename VecOf<VEC>::type load_stream(const float *p) {
    typedef typename VecOf<VEC>::type V;
    return __builtin_nontemporal_load(reinterpret_cast<const V *>(p));
}
template <int VEC>
__device__ __forceinline__ void store_stream(float *p, typename VecOf<VEC>::type v) {
    typedef typename VecOf<VEC>::type V;
    __builtin_nontemporal_store(v, reinterpret_cast<V *>(p));
}

// K: queries per group (compile time so that the K input columns stay in registers).
// VEC: floats per lane per access.
template <int K, int VEC>
__global__ __launch_bounds__(kEncodeThreads) void encode_kernel(
    const float *__restrict__ queries, float *__restrict__ coded, int N, int64_t D, int64_t Dv,
    int64_t chunks, const Nodes nodes) {
    typedef typename VecOf<VEC>::type V;
    constexpr int KP = (K + 3) & ~3;       // weight row padded to whole float4s
    constexpr int LPR = K <= 16 ? 16 : (K <= 32 ? 32 : 64);   // lanes per weight row
    constexpr int ROWS_PER_PASS = kEncodeThreads / LPR;
    extern __shared__ float wl[];          // [N][KP]

    const int tid = threadIdx.x;
    const int64_t g = blockIdx.x / chunks;
    const int64_t ch = blockIdx.x - g * chunks;
    const int64_t col = ch * kEncodeThreads + tid;
    const bool ok = col < Dv;
    // lanes past the ragged end read column 0 of the group (always in bounds) and store nothing
    const float *xg = queries + static_cast<size_t>(g) * K * D + (ok ? col : 0) * VEC;
    float *og = coded + static_cast<size_t>(g) * N * D + col * VEC;

    // ---- this lane's column of the K queries: issue every load before anything else ----
    V x[K];
#pragma unroll
    for (int j = 0; j < K; ++j) x[j] = load_stream<VEC>(xg + static_cast<size_t>(j) * D);

    // ---- l_j(beta_i) in float64, one group of LPR lanes per worker row ---------------------
    {
        const int j = tid % LPR;
        const bool valid = j < K;
        const double xa = valid ? nodes.alpha[j] : 0.0;
        const double sign = (j & 1) ? -1.0 : 1.0;
        for (int i0 = 0; i0 < N; i0 += ROWS_PER_PASS) {
            const int i = i0 + tid / LPR;
            const bool row = i < N;
            const BerrutTerm bt = berrut_term(row ? nodes.beta[i] : 2.0, xa, sign, valid && row);
            const double den = group_sum<LPR>(bt.t);
            const bool any_hit = group_sum<LPR>(bt.hit ? 1.0 : 0.0) != 0.0;
            const double w = any_hit ? (bt.hit ? 1.0 : 0.0) : bt.t * (1.0 / den);
            if (row && j < KP) wl[i * KP + j] = valid ? static_cast<float>(w) : 0.0f;
        }
    }
    __syncthreads();

    const v4f *wl4 = reinterpret_cast<const v4f *>(wl);
    for (int i = 0; i < N; ++i) {
        V acc = V(0.0f);
#pragma unroll
        for (int j4 = 0; j4 < KP / 4; ++j4) {
            const v4f w = wl4[i * (KP / 4) + j4];
#pragma unroll
            for (int jj = 0; jj < 4; ++jj)
                if (4 * j4 + jj < K) acc = w[jj] * x[4 * j4 + jj] + acc;
        }
        if (ok) store_stream<VEC>(og + static_cast<size_t>(i) * D, acc);
    }
}

template <int K, int VEC>
int run_encode(const float *d_queries, float *d_coded, int64_t G, int N, int64_t D, const Nodes &nodes,
               hipStream_t stream) {
    constexpr int KP = (K + 3) & ~3;
    const int64_t Dv = D / VEC;
    const int64_t chunks = (Dv + kEncodeThreads - 1) / kEncodeThreads;
    const int64_t tiles = G * chunks;
    if (tiles > 0x7fffffffLL) return APPROXIFER_ERR_LIMIT;
    const size_t lds = static_cast<size_t>(N) * KP * sizeof(float);
    hipLaunchKernelGGL((encode_kernel<K, VEC>), dim3(static_cast<unsigned>(tiles)), dim3(kEncodeThreads), lds,
                       stream, d_queries, d_coded, N, D, Dv, chunks, nodes);
    return hipGetLastError() == hipSuccess ? APPROXIFER_OK : APPROXIFER_ERR_LAUNCH;
}

template <int K>
int run_encode_k(const float *d_queries, float *d_coded, int64_t G, int N, int64_t D, const Nodes &nodes,
                 hipStream_t stream) {
    const bool aligned16 = (reinterpret_cast<uintptr_t>(d_queries) % 16 == 0) &&
                           (reinterpret_cast<uintptr_t>(d_coded) % 16 == 0) && (D % 4 == 0);
    if (aligned16) return run_encode<K, 4>(d_queries, d_coded, G, N, D, nodes, stream);
    return run_encode<K, 1>(d_queries, d_coded, G, N, D, nodes, stream);
}

}  // namespace

#define APPROXIFER_K_CASE(k) \
    case k: return run_encode_k<k>(d_queries, d_coded, G, N, D, nodes, stream);
#define APPROXIFER_K_CASE8(b)                                                                        \
    APPROXIFER_K_CASE(b + 1) APPROXIFER_K_CASE(b + 2) APPROXIFER_K_CASE(b + 3) APPROXIFER_K_CASE(b + 4) \
    APPROXIFER_K_CASE(b + 5) APPROXIFER_K_CASE(b + 6) APPROXIFER_K_CASE(b + 7) APPROXIFER_K_CASE(b + 8)

int launch_encode(const float *d_queries, float *d_coded, int64_t G, int K, int N, int64_t D, const Nodes &nodes,
                  hipStream_t stream) {
    static_assert(APPROXIFER_MAX_K == 64, "the K dispatch below covers 1..64");
    switch (K) {
        APPROXIFER_K_CASE8(0)
        APPROXIFER_K_CASE8(8)
        APPROXIFER_K_CASE8(16)
        APPROXIFER_K_CASE8(24)
        APPROXIFER_K_CASE8(32)
        APPROXIFER_K_CASE8(40)
        APPROXIFER_K_CASE8(48)
        APPROXIFER_K_CASE8(56)
        default: return APPROXIFER_ERR_LIMIT;
    }
}

}  // namespace approxifer
