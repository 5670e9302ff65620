// ApproxIFER encoder for gfx950 (Section 3, "ApproxIFER Encoding").
//
//   coded[g][i][d] = sum_j l_j(beta_i) * queries[g][j][d]
//
// The N x K matrix l_j(beta_i) depends on the nodes only, so every workgroup evaluates it
// once (float64, one wave per row, the row's denominator by a wavefront reduction), keeps
// it in LDS as float32 and then streams tiles of the query tensor: each lane holds one
// vector column of all K queries of a group in registers, forms the N coded values of that
// column one worker at a time with the weights broadcast from LDS, and stores each as soon
// as it is complete.  Every query element is read from HBM exactly once and every coded
// element written exactly once; the kernel is a pure HBM stream of 4*D*(K+N) bytes per
// group with 2*K*N flops per 4*(K+N) bytes on top.
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
// VEC: floats per lane per access.  UN: vector columns per lane per tile.
template <int K, int VEC, int UN>
__global__ __launch_bounds__(kEncodeThreads) void encode_kernel(
    const float *__restrict__ queries, float *__restrict__ coded, int N, int64_t D, int64_t Dv,
    int64_t chunks, int64_t tiles, const Nodes nodes) {
    typedef typename VecOf<VEC>::type V;
    constexpr int KP = (K + 3) & ~3;       // weight row padded to whole float4s
    extern __shared__ float wl[];          // [N][KP]

    // ---- l_j(beta_i), float64, one wave per worker row ------------------------------
    {
        const int lane = lane_id();
        const bool valid = lane < K;
        const double x = valid ? nodes.alpha[lane] : 0.0;
        const double sign = (lane & 1) ? -1.0 : 1.0;
        for (int i = wave_id(); i < N; i += kEncodeThreads / kWave) {
            const BerrutTerm bt = berrut_term(nodes.beta[i], x, sign, valid);
            const double den = wave_sum(bt.t);
            const bool any_hit = __ballot(bt.hit) != 0ull;
            const double w = any_hit ? (bt.hit ? 1.0 : 0.0) : bt.t / den;
            if (lane < KP) wl[i * KP + lane] = valid ? static_cast<float>(w) : 0.0f;
        }
    }
    __syncthreads();

    const v4f *wl4 = reinterpret_cast<const v4f *>(wl);
    const int tid = threadIdx.x;

    for (int64_t t = blockIdx.x; t < tiles; t += gridDim.x) {
        const int64_t g = t / chunks;
        const int64_t ch = t - g * chunks;
        const float *xg = queries + static_cast<size_t>(g) * K * D;
        float *og = coded + static_cast<size_t>(g) * N * D;

        int64_t col[UN];
        bool ok[UN];
        V x[UN][K];
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            col[u] = (ch * UN + u) * kEncodeThreads + tid;
            ok[u] = col[u] < Dv;
#pragma unroll
            for (int j = 0; j < K; ++j) {
                if (ok[u]) x[u][j] = load_stream<VEC>(xg + static_cast<size_t>(j) * D + col[u] * VEC);
                else x[u][j] = V(0.0f);
            }
        }

        for (int i = 0; i < N; ++i) {
            V acc[UN];
#pragma unroll
            for (int u = 0; u < UN; ++u) acc[u] = V(0.0f);
#pragma unroll
            for (int j4 = 0; j4 < KP / 4; ++j4) {
                const v4f w = wl4[i * (KP / 4) + j4];
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) {
                    if (4 * j4 + jj < K) {
#pragma unroll
                        for (int u = 0; u < UN; ++u) acc[u] = w[jj] * x[u][4 * j4 + jj] + acc[u];
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < UN; ++u)
                if (ok[u]) store_stream<VEC>(og + static_cast<size_t>(i) * D + col[u] * VEC, acc[u]);
        }
    }
}

struct EncodeGeometry {
    int num_cus;
};

int device_cu_count() {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    int cus = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
    return cus;
}

template <int K, int VEC, int UN>
int run_encode(const float *d_queries, float *d_coded, int64_t G, int N, int64_t D, const Nodes &nodes,
               hipStream_t stream) {
    constexpr int KP = (K + 3) & ~3;
    const int64_t Dv = D / VEC;
    const int64_t chunks = (Dv + int64_t(kEncodeThreads) * UN - 1) / (int64_t(kEncodeThreads) * UN);
    const int64_t tiles = G * chunks;
    const size_t lds = static_cast<size_t>(N) * KP * sizeof(float);

    int per_cu = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, encode_kernel<K, VEC, UN>, kEncodeThreads, lds) !=
            hipSuccess || per_cu < 1)
        per_cu = 1;
    const int cus = device_cu_count();
    if (cus < 1) return APPROXIFER_ERR_LAUNCH;
    int64_t grid = int64_t(cus) * per_cu;
    if (grid > tiles) grid = tiles;

    hipLaunchKernelGGL((encode_kernel<K, VEC, UN>), dim3(static_cast<unsigned>(grid)), dim3(kEncodeThreads), lds,
                       stream, d_queries, d_coded, N, D, Dv, chunks, tiles, nodes);
    return hipGetLastError() == hipSuccess ? APPROXIFER_OK : APPROXIFER_ERR_LAUNCH;
}

template <int K>
int run_encode_k(const float *d_queries, float *d_coded, int64_t G, int N, int64_t D, const Nodes &nodes,
                 hipStream_t stream) {
    const bool aligned16 = (reinterpret_cast<uintptr_t>(d_queries) % 16 == 0) &&
                           (reinterpret_cast<uintptr_t>(d_coded) % 16 == 0) && (D % 4 == 0);
    if (aligned16) return run_encode<K, 4, 1>(d_queries, d_coded, G, N, D, nodes, stream);
    return run_encode<K, 1, 1>(d_queries, d_coded, G, N, D, nodes, stream);
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
