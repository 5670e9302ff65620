// ApproxIFER encoder for gfx950 (Section 3, "ApproxIFER Encoding").
//
//   coded[g][i][d] = sum_j l_j(beta_i) * queries[g][j][d]
//
// One workgroup per (group, tile of vector columns): a single wave (64 columns) for K <= 16,
// four waves (256 columns) above.  Each lane first issues the loads of its vector column of
// all K queries (they stay in registers), and while those are in flight the workgroup
// evaluates the N x K matrix l_j(beta_i) -- it depends on the nodes only -- in float64 (one
// 16/32/64-lane group per worker row, the row's denominator by a DPP reduction) and keeps it
// in LDS as float32.  The N coded values of the column are then formed one worker at a time
// with the weights broadcast from LDS and stored as soon as complete.
// Every query element is read from HBM exactly once and every coded element written exactly
// once: the kernel is an HBM stream of 4*D*(K+N) bytes per group with 2*K*N flops per
// 4*(K+N) bytes on top.
//
// Two launch-shape facts, both measured on MI355X at the 3x224x224, K=12, N=20 shape:
//  * Workgroups do not loop over tiles.  On gfx9 one counter orders a wave's loads and stores,
//    so a looping wave waits for its previous stores before it can use its next loads; a wave
//    that retires after issuing its stores does not (1.92 ms persistent, 1.76 ms one-shot).
//  * HBM efficiency falls with the number of row streams that are open at once (a plain copy
//    reaches 6.6 TB/s walked sequentially, 5.2 TB/s walked as 12+12 interleaved rows), i.e.
//    with the number of tiles in flight.  The kernel therefore caps residency at a few waves
//    per CU by reserving LDS it does not use: each wave has all K of its 128-bit loads in flight,
//    which is enough to cover latency (1.76 ms uncapped, 1.62 ms at 7 waves per CU).
#include "common.h"

namespace approxifer {
namespace {

// Residency caps (workgroups per CU), found by sweeping 4..32 on the five benchmark shapes.
#ifndef APPROXIFER_ENCODE_WAVES_PER_CU_SMALL_K
#define APPROXIFER_ENCODE_WAVES_PER_CU_SMALL_K 7     // K <= 16: one-wave workgroups
#endif
#ifndef APPROXIFER_ENCODE_BLOCKS_PER_CU_LARGE_K
#define APPROXIFER_ENCODE_BLOCKS_PER_CU_LARGE_K 2    // K > 16: four-wave workgroups
#endif
constexpr int kLdsPerCu = 160 * 1024;                // gfx950

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
// VEC: floats per lane per access.  THREADS: workgroup size.
template <int K, int VEC, int THREADS>
__global__ __launch_bounds__(THREADS) void encode_kernel(
    const float *__restrict__ queries, float *__restrict__ coded, int N, int64_t D, int64_t Dv,
    int64_t chunks, const Nodes nodes) {
    typedef typename VecOf<VEC>::type V;
    constexpr int KP = (K + 3) & ~3;       // weight row padded to whole float4s
    constexpr int LPR = K <= 16 ? 16 : (K <= 32 ? 32 : 64);   // lanes per weight row
    constexpr int ROWS_PER_PASS = THREADS / LPR;
    extern __shared__ float wl[];          // [N][KP]

    const int tid = threadIdx.x;
    const int64_t g = blockIdx.x / chunks;
    const int64_t ch = blockIdx.x - g * chunks;
    const int64_t col = ch * THREADS + tid;
    const bool ok = col < Dv;
    // lanes past the ragged end read column 0 of the group (always in bounds) and store nothing
    const float *xg = queries + static_cast<size_t>(g) * K * D + (ok ? col : 0) * VEC;
    float *og = coded + static_cast<size_t>(g) * N * D + col * VEC;

    // ---- this lane's column of the K queries: issue every load before anything else ----
    V x[K];
#pragma unroll
    for (int j = 0; j < K; ++j) x[j] = load_stream<VEC>(xg + static_cast<size_t>(j) * D);

    // ---- l_j(beta_i) in float64, one group of LPR lanes per worker row ---------------------
    // The nodes are read with compile-time or wave-uniform indices only, i.e. through scalar
    // loads: a vector load here would queue behind the query loads above and make the wave
    // wait for all of them before it could evaluate a single weight.
    {
        const int j = tid % LPR;
        const int sub = tid / LPR;
        const bool valid = j < K;
        double xa = 0.0;
#pragma unroll
        for (int jj = 0; jj < K; ++jj) {
            const double a = wave_uniform(nodes.alpha[jj]);
            if (j == jj) xa = a;
        }
        const double sign = (j & 1) ? -1.0 : 1.0;
        for (int i0 = 0; i0 < N; i0 += ROWS_PER_PASS) {   // i0 + ROWS_PER_PASS <= APPROXIFER_MAX_N always
            double z = wave_uniform(nodes.beta[i0]);
#pragma unroll
            for (int r = 1; r < ROWS_PER_PASS; ++r) {
                const double zr = wave_uniform(nodes.beta[i0 + r]);
                if (sub == r) z = zr;
            }
            const int i = i0 + sub;
            const bool row = i < N;
            const BerrutTerm bt = berrut_term(z, xa, sign, valid && row);
            const double den = group_sum<LPR>(bt.t);
            const unsigned long long hits = __ballot(bt.hit);
            const unsigned long long group_mask = (LPR == 64) ? ~0ull : ((1ull << (LPR & 63)) - 1ull) << ((tid & 63) / LPR * LPR);
            const bool any_hit = (hits & group_mask) != 0ull;
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
    constexpr int THREADS = K <= 16 ? 64 : 256;
    constexpr int PER_CU = K <= 16 ? APPROXIFER_ENCODE_WAVES_PER_CU_SMALL_K : APPROXIFER_ENCODE_BLOCKS_PER_CU_LARGE_K;
    const int64_t Dv = D / VEC;
    const int64_t chunks = (Dv + THREADS - 1) / THREADS;
    const int64_t tiles = G * chunks;
    if (tiles > 0x7fffffffLL) return APPROXIFER_ERR_LIMIT;
    const size_t lds_used = static_cast<size_t>(N) * KP * sizeof(float);
    // reserve 1/PER_CU of the CU's LDS so that at most PER_CU workgroups are resident
    size_t lds = (static_cast<size_t>(kLdsPerCu / PER_CU) / 512) * 512;
    if (lds < lds_used) lds = lds_used;
    if (lds > 64 * 1024 &&
        hipFuncSetAttribute(reinterpret_cast<const void *>(encode_kernel<K, VEC, THREADS>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds)) != hipSuccess)
        return APPROXIFER_ERR_LAUNCH;
    hipLaunchKernelGGL((encode_kernel<K, VEC, THREADS>), dim3(static_cast<unsigned>(tiles)), dim3(THREADS), lds,
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
