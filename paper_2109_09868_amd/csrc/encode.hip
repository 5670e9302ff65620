// ApproxIFER encoder for gfx950 (Section 3, "ApproxIFER Encoding").
//
//   coded[g][i][d] = sum_j l_j(beta_i) * queries[g][j][d]
//
// One workgroup per (group, tile of vector columns): a single wave (64 columns) for K <= 16,
// four waves (256 columns) above; short ragged rows are tiled over the flattened (group, column)
// index instead, so that no lane idles at a row end.  Each lane first issues the loads of its vector column of
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
//    which is enough to cover latency (1.76 ms uncapped, 1.60 ms at 6 waves per CU).
#include "common.h"

namespace approxifer {
namespace {

// Residency caps (workgroups per CU), from sweeps on the benchmark shapes and on a K x N x D grid.
// K <= 16, one-wave workgroups: enough waves to keep about 48 KB of query loads in flight per CU (a wave
// has K loads of 1 KB each), never fewer than six and never more than 24: measured optima are 20+ at K = 1,
// 12..16 at K = 2, 8..12 at K = 4..6, 6 at K = 8..16 (7 and up lose 1..4 % there: more row streams open).
constexpr int kWavesPerCuMin = 6;
constexpr int kLoadKbPerCu = 48;
constexpr int kBlocksPerCuLargeK = 2;   // K > 16: four-wave workgroups
constexpr int kMfmaMinK = 17;   // from this K on the matrix-core variant serves every shape
constexpr int kMfmaWideMinK = 8;   // .. and from this K on the shapes with N >= 2K + 4
constexpr int kMfmaBlocksPerCu = 4;   // matrix-core variant (four waves of 64 columns)
constexpr int kScalarRowsMaxD = 128;   // ragged rows (D % 4 != 0) this short: 64-bit or 4-byte accesses only
constexpr int kLdsPerCu = 160 * 1024;                // gfx950

// Register type of VEC floats, and the type a lane loads and stores it through.  Rows that are only
// 4-byte aligned (a row length that is not a multiple of 4 floats, or an offset base pointer) are still
// moved 128 bits at a time: gfx950 serves dword-aligned 128-bit global accesses, and the compiler emits them
// for a vector type declared with 4-byte alignment.
template <int VEC> struct VecOf;
template <> struct VecOf<4> { typedef v4f type; };
template <> struct VecOf<2> { typedef v2f type; };
template <> struct VecOf<1> { typedef float type; };
typedef v4f v4f_align4 __attribute__((aligned(4)));
template <int VEC, bool UNAL> struct MemOf { typedef typename VecOf<VEC>::type type; };
template <> struct MemOf<4, true> { typedef v4f_align4 type; };

template <int VEC, bool UNAL = false>
__device__ __forceinline__ typename VecOf<VEC>::type load_stream(const float *p) {
    typedef typename MemOf<VEC, UNAL>::type M;
    const M v = __builtin_nontemporal_load(reinterpret_cast<const M *>(p));
    return v;
}
template <int VEC, bool UNAL = false>
__device__ __forceinline__ void store_stream(float *p, typename VecOf<VEC>::type v) {
    typedef typename MemOf<VEC, UNAL>::type M;
    __builtin_nontemporal_store(static_cast<M>(v), reinterpret_cast<M *>(p));
}

// K: queries per group (compile time so that the K input columns stay in registers).
// VEC: floats per lane per access.  THREADS: workgroup size.
// FLAT: false -- a workgroup covers THREADS consecutive vector columns of ONE group (`chunks` workgroups per
//       group; the last one of a group may be partly idle);  true -- the (group, vector column) pairs of the
//       whole batch are numbered consecutively and a workgroup takes THREADS of them, so lanes never idle at a
//       row end.  Used when rows are short and ragged (28 x 28 queries: 196 vector columns, 23 % idle lanes
//       otherwise); `chunks` then carries the total number of pairs.
// UNAL: rows are only 4-byte aligned (VEC == 4 accesses then go through the 4-byte-aligned vector type).
// col0: first float column served; columns col0 + VEC * [0, Dv) are produced.
template <int K, int VEC, int THREADS, bool FLAT, bool UNAL>
__global__ __launch_bounds__(THREADS) void encode_kernel(
    const float *__restrict__ queries, float *__restrict__ coded, int N, int64_t D, int64_t Dv,
    int64_t chunks, int64_t col0, const Nodes nodes) {
    typedef typename VecOf<VEC>::type V;
    constexpr int KP = (K + 3) & ~3;       // weight row padded to whole float4s
    constexpr int LPR = K <= 16 ? 16 : (K <= 32 ? 32 : 64);   // lanes per weight row
    constexpr int ROWS_PER_PASS = THREADS / LPR;
    extern __shared__ float wl[];          // [N][KP]

    const int tid = threadIdx.x;
    int64_t g, col;
    bool ok;
    if (FLAT) {
        const int64_t q = static_cast<int64_t>(blockIdx.x) * THREADS + tid;
        ok = q < chunks;
        const int64_t qq = ok ? q : 0;
        if (chunks <= 0xffffffffLL) {      // the usual case: one 32-bit division per lane
            const uint32_t g32 = static_cast<uint32_t>(qq) / static_cast<uint32_t>(Dv);
            g = g32;
            col = static_cast<uint32_t>(qq) - g32 * static_cast<uint32_t>(Dv);
        } else {
            g = qq / Dv;
            col = qq - g * Dv;
        }
    } else {
        g = blockIdx.x / chunks;
        col = (blockIdx.x - g * chunks) * THREADS + tid;
        ok = col < Dv;
        if (!ok) col = 0;                  // lanes past the ragged end read column 0 of the group and store nothing
    }
    const float *xg = queries + static_cast<size_t>(g) * K * D + col0 + col * VEC;
    float *og = coded + static_cast<size_t>(g) * N * D + col0 + col * VEC;

    // ---- this lane's column of the K queries: issue every load before anything else ----
    V x[K];
#pragma unroll
    for (int j = 0; j < K; ++j) x[j] = load_stream<VEC, UNAL>(xg + static_cast<size_t>(j) * D);

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
        if (ok) store_stream<VEC, UNAL>(og + static_cast<size_t>(i) * D, acc);
    }
}

// ---- matrix-core variant for K > 16 -----------------------------------------------------
// At K = 32, N = 48 the vector kernel above issues VALU instructions on 95 % of all cycles
// (SQ_INSTS_VALU x 4 against SIMD-cycles): the contraction, not HBM, bounds it there.  This
// variant forms coded = W (N x K) * X (K x columns) with v_mfma_f32_16x16x4_f32, whose fp32 rate is
// twice the plain vector FMA rate, and leaves the vector ALUs to address arithmetic.
//
// Operand layout of v_mfma_f32_16x16x4_f32 (D[16x16] += A[16x4] * B[4x16]), lane l of the wave:
//   A: element (row l%16, k l/16)       B: element (k l/16, column l%16)
//   D: register r holds element (row 4*(l/16) + r, column l%16)
// A wave owns 64 consecutive columns of a group.  One 128-bit load gives lane l the four columns
// 4*(l%16)..+3 of query row 4s + l/16, so component e of that register IS the B operand of k-step
// s for the column set {4c + e}: no shuffles.  The four column sets give, in register r of their
// accumulators, four consecutive columns of worker row 16*mt + 4*(l/16) + r: one 128-bit store.
// The weights sit in LDS already in A-operand order, wA[(mt*KS + s)*64 + l].
constexpr int kMfmaThreads = 256;

// KS = ceil(K / 4) k-steps; UNAL: rows only 4-byte aligned; FLAT: the 16-column wave tiles run over the flattened
// (group, vector column) numbering of the batch (`chunks` = number of pairs), as in encode_kernel.
template <int KS, bool UNAL, bool FLAT>
__global__ __launch_bounds__(kMfmaThreads) void encode_mfma_kernel(
    const float *__restrict__ queries, float *__restrict__ coded, int K, int N, int64_t D, int64_t Dv,
    int64_t chunks, const Nodes nodes) {
    constexpr int LPR = KS <= 8 ? 32 : 64;                    // lanes per weight row (K <= 32 / K <= 64)
    constexpr int ROWS_PER_PASS = kMfmaThreads / LPR;
    extern __shared__ float wA[];                             // [ceil(N/16)][KS][64]

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wv = tid >> 6;
    int64_t g, col;                                           // this lane's group and vector column
    bool ok;
    if (FLAT) {
        const int64_t q = (static_cast<int64_t>(blockIdx.x) * (kMfmaThreads / 64) + wv) * 16 + (lane & 15);
        ok = q < chunks;
        const int64_t qq = ok ? q : 0;
        if (chunks <= 0xffffffffLL) {
            const uint32_t g32 = static_cast<uint32_t>(qq) / static_cast<uint32_t>(Dv);
            g = g32;
            col = static_cast<uint32_t>(qq) - g32 * static_cast<uint32_t>(Dv);
        } else {
            g = qq / Dv;
            col = qq - g * Dv;
        }
    } else {
        g = blockIdx.x / chunks;
        col = ((blockIdx.x - g * chunks) * (kMfmaThreads / 64) + wv) * 16 + (lane & 15);
        ok = col < Dv;
        if (!ok) col = 0;
    }
    const int krow = lane >> 4;                               // row offset inside a k-step
    const float *xg = queries + static_cast<size_t>(g) * K * D + col * 4;
    float *og = coded + static_cast<size_t>(g) * N * D + col * 4;

    // ---- query rows 4s + krow, columns 4*col..+3; rows past K are clamped (their weights are 0) ----
    v4f x[KS];
#pragma unroll
    for (int s = 0; s < KS; ++s) {
        const int row = (4 * s + krow < K) ? 4 * s + krow : K - 1;
        x[s] = load_stream<4, UNAL>(xg + static_cast<size_t>(row) * D);
    }

    // ---- l_j(beta_i) in float64 (scalar node loads only, see encode_kernel), stored in A order ----
    {
        const int j = tid % LPR;
        const int sub = tid / LPR;
        const bool valid = j < K;
        double xa = 0.0;
#pragma unroll
        for (int jj = 0; jj < 4 * KS; ++jj) {
            const double a = wave_uniform(nodes.alpha[jj]);   // entries past K are zero-filled by the host
            if (j == jj) xa = a;
        }
        const double sign = (j & 1) ? -1.0 : 1.0;
        const int n16 = (N + 15) & ~15;
        for (int i0 = 0; i0 < n16; i0 += ROWS_PER_PASS) {     // n16 <= 128 = APPROXIFER_MAX_N: reads stay in bounds
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
            const unsigned long long group_mask =
                (LPR == 64) ? ~0ull : ((1ull << (LPR & 63)) - 1ull) << ((tid & 63) / LPR * LPR);
            const bool any_hit = (hits & group_mask) != 0ull;
            const double w = any_hit ? (bt.hit ? 1.0 : 0.0) : bt.t * (1.0 / den);
            if (j < 4 * KS)   // rows N..n16-1 and columns K..4KS-1 hold zeros
                wA[((i >> 4) * KS + (j >> 2)) * 64 + (j & 3) * 16 + (i & 15)] = (valid && row) ? static_cast<float>(w) : 0.0f;
        }
    }
    __syncthreads();

    const int mtiles = (N + 15) >> 4;
    for (int mt = 0; mt < mtiles; ++mt) {
        v4f acc[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[e] = v4f(0.0f);
        const float *wmt = wA + mt * KS * 64 + lane;
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            const float a = wmt[s * 64];
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[e] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, x[s][e], acc[e], 0, 0, 0);
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int i = 16 * mt + 4 * krow + r;
            if (ok && i < N) {
                v4f v;
                v[0] = acc[0][r];
                v[1] = acc[1][r];
                v[2] = acc[2][r];
                v[3] = acc[3][r];
                store_stream<4, UNAL>(og + static_cast<size_t>(i) * D, v);
            }
        }
    }
}

template <int KS, bool UNAL, bool FLAT>
int run_encode_mfma_shape(const float *d_queries, float *d_coded, int64_t tiles, int64_t chunks, int K, int N, int64_t D,
                          int64_t Dv, const Nodes &nodes, hipStream_t stream) {
    if (tiles > 0x7fffffffLL) return APPROXIFER_ERR_LIMIT;
    const size_t lds_used = static_cast<size_t>((N + 15) / 16) * KS * 64 * sizeof(float);
    size_t lds = (static_cast<size_t>(kLdsPerCu / kMfmaBlocksPerCu) / 512) * 512;
    if (lds < lds_used) lds = lds_used;
    if (lds > 64 * 1024 &&
        hipFuncSetAttribute(reinterpret_cast<const void *>(encode_mfma_kernel<KS, UNAL, FLAT>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds)) != hipSuccess)
        return APPROXIFER_ERR_LAUNCH;
    return launch_status(launch_kernel(encode_mfma_kernel<KS, UNAL, FLAT>, dim3(static_cast<unsigned>(tiles)),
                                       dim3(kMfmaThreads), lds, stream, d_queries, d_coded, K, N, D, Dv, chunks, nodes));
}

template <int KS, bool UNAL>
int run_encode_mfma(const float *d_queries, float *d_coded, int64_t G, int K, int N, int64_t D, const Nodes &nodes,
                    hipStream_t stream) {
    const int64_t Dv = D / 4;
    const int64_t cols_per_block = (kMfmaThreads / 64) * 16;           // vector columns per workgroup
    const int64_t chunks = (Dv + cols_per_block - 1) / cols_per_block;
    const int64_t idle = chunks * cols_per_block - Dv;                  // columns without data at the row ends
    if (idle * 100 > 3 * chunks * cols_per_block) {
        const int64_t pairs = G * Dv;
        return run_encode_mfma_shape<KS, UNAL, true>(d_queries, d_coded, (pairs + cols_per_block - 1) / cols_per_block,
                                                     pairs, K, N, D, Dv, nodes, stream);
    }
    return run_encode_mfma_shape<KS, UNAL, false>(d_queries, d_coded, G * chunks, chunks, K, N, D, Dv, nodes, stream);
}

template <int K, int VEC, bool FLAT, bool UNAL>
int run_encode_shape(const float *d_queries, float *d_coded, int64_t tiles, int64_t chunks, int N, int64_t D,
                     int64_t Dv, int64_t col0, const Nodes &nodes, hipStream_t stream) {
    constexpr int KP = (K + 3) & ~3;
    constexpr int THREADS = K <= 16 ? 64 : 256;
    int per_cu = kBlocksPerCuLargeK;
    if (K <= 16) {
        per_cu = (kLoadKbPerCu + K - 1) / K;     // K loads of 1 KB per wave
        if (per_cu < kWavesPerCuMin) per_cu = kWavesPerCuMin;
        if (per_cu > 24) per_cu = 24;
        if (VEC == 1) per_cu = 7;       // 4-byte accesses (the last D % 4 columns, or D < 4): a sliver of the work
    }
    if (tiles > 0x7fffffffLL) return APPROXIFER_ERR_LIMIT;
    const size_t lds_used = static_cast<size_t>(N) * KP * sizeof(float);
    // reserve 1/per_cu of the CU's LDS so that at most per_cu workgroups are resident
    size_t lds = (static_cast<size_t>(kLdsPerCu / per_cu) / 512) * 512;
    if (lds < lds_used) lds = lds_used;
    if (lds > 64 * 1024 &&
        hipFuncSetAttribute(reinterpret_cast<const void *>(encode_kernel<K, VEC, THREADS, FLAT, UNAL>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds)) != hipSuccess)
        return APPROXIFER_ERR_LAUNCH;
    return launch_status(launch_kernel(encode_kernel<K, VEC, THREADS, FLAT, UNAL>, dim3(static_cast<unsigned>(tiles)),
                                       dim3(THREADS), lds, stream, d_queries, d_coded, N, D, Dv, chunks, col0, nodes));
}

// Vector columns [0, Dv) of width VEC floats, starting at float column col0.
template <int K, int VEC, bool UNAL>
int run_encode(const float *d_queries, float *d_coded, int64_t G, int N, int64_t D, int64_t Dv, int64_t col0,
               const Nodes &nodes, hipStream_t stream) {
    constexpr int THREADS = K <= 16 ? 64 : 256;
    const int64_t chunks = (Dv + THREADS - 1) / THREADS;
    // lanes left idle at the row ends by the per-group tiling; above 3 % the flattened numbering pays for its
    // per-lane division and addresses
    const int64_t idle = chunks * THREADS - Dv;
    if (idle * 100 > 3 * chunks * THREADS) {
        const int64_t pairs = G * Dv;
        return run_encode_shape<K, VEC, true, UNAL>(d_queries, d_coded, (pairs + THREADS - 1) / THREADS, pairs, N, D, Dv,
                                                    col0, nodes, stream);
    }
    return run_encode_shape<K, VEC, false, UNAL>(d_queries, d_coded, G * chunks, chunks, N, D, Dv, col0, nodes, stream);
}

// 128-bit columns: the matrix-core kernel or the vector kernel, by shape.
template <int K, bool UNAL>
int run_encode_wide(const float *d_queries, float *d_coded, int64_t G, int N, int64_t D, const Nodes &nodes,
                    hipStream_t stream) {
    if constexpr (K >= kMfmaMinK) {
        return run_encode_mfma<(K + 3) / 4, UNAL>(d_queries, d_coded, G, K, N, D, nodes, stream);
    } else {
        if constexpr (K >= kMfmaWideMinK) {
            // Many more coded than plain queries (the Byzantine worker counts, N = 2 (K + A) + S): a one-wave
            // tile would keep K + N >= 3K + 4 row streams open, and the matrix-core variant, whose waves work on
            // 256-byte row segments, measures 4..14 % faster (K=8, N=24: 5.7 -> 6.2 TB/s; K=12, N=36: 5.5 -> 6.0).
            if (N >= 2 * K + 4)
                return run_encode_mfma<(K + 3) / 4, UNAL>(d_queries, d_coded, G, K, N, D, nodes, stream);
        }
        return run_encode<K, 4, UNAL>(d_queries, d_coded, G, N, D, D / 4, 0, nodes, stream);
    }
}

template <int K>
int run_encode_k(const float *d_queries, float *d_coded, int64_t G, int N, int64_t D, const Nodes &nodes,
                 hipStream_t stream) {
    const bool aligned16 = (reinterpret_cast<uintptr_t>(d_queries) % 16 == 0) &&
                           (reinterpret_cast<uintptr_t>(d_coded) % 16 == 0) && (D % 4 == 0);
    if (aligned16) return run_encode_wide<K, false>(d_queries, d_coded, G, N, D, nodes, stream);
    // rows only 4-byte aligned: 128-bit accesses on the first 4 * (D / 4) columns, 4-byte accesses on the rest;
    // short ragged rows: aligned 64-bit accesses throughout where the rows allow them, else 4-byte accesses
    const int64_t tail = D % 4;
    if (tail != 0 && D <= kScalarRowsMaxD) {
        if (D % 2 == 0 && reinterpret_cast<uintptr_t>(d_queries) % 8 == 0 && reinterpret_cast<uintptr_t>(d_coded) % 8 == 0)
            return run_encode<K, 2, false>(d_queries, d_coded, G, N, D, D / 2, 0, nodes, stream);
        return run_encode<K, 1, false>(d_queries, d_coded, G, N, D, D, 0, nodes, stream);
    }
    if (D >= 4) {
        const int rc = run_encode_wide<K, true>(d_queries, d_coded, G, N, D, nodes, stream);
        if (rc != APPROXIFER_OK) return rc;
    }
    if (tail == 0) return APPROXIFER_OK;
    return run_encode<K, 1, false>(d_queries, d_coded, G, N, D, tail, D - tail, nodes, stream);
}

}  // namespace

// Rows Q .. Q + fill - 1 of a [rows][D] query buffer become copies of row Q - 1 (a stream whose length is not a
// multiple of K: the last group is completed by repeating its last query).  One float per thread.
__global__ void pad_last_group_kernel(float *__restrict__ queries, int64_t Q, int64_t D, int64_t fill) {
    const int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i >= fill * D) return;
    const int64_t d = i % D;
    queries[Q * D + i] = queries[(Q - 1) * D + d];
}

int launch_pad_last_group(float *d_queries, int64_t Q, int K, int64_t D, hipStream_t stream) {
    const int64_t fill = (K - Q % K) % K;
    if (fill == 0 || D == 0) return APPROXIFER_OK;
    const int threads = 256;
    const int64_t blocks = (fill * D + threads - 1) / threads;
    if (blocks > 0x7fffffffLL) return APPROXIFER_ERR_LIMIT;
    return launch_status(launch_kernel(pad_last_group_kernel, dim3(static_cast<unsigned>(blocks)), dim3(threads), 0, stream,
                                       d_queries, Q, D, fill));
}

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
