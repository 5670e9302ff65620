// Shared device helpers of the ApproxIFER coding-layer kernels (gfx950, wave64).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "approxifer.h"

namespace approxifer {

constexpr int kWave = 64;

// Query and worker nodes travel by value in the kernel-argument segment: the library
// owns no device memory, and K + N doubles always fit.
struct Nodes {
    double alpha[APPROXIFER_MAX_K];
    double beta[APPROXIFER_MAX_N];
};

typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v2f __attribute__((ext_vector_type(2)));

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, kWave);
    return v;
}

__device__ __forceinline__ int lane_id() { return threadIdx.x & (kWave - 1); }
__device__ __forceinline__ int wave_id() { return threadIdx.x >> 6; }

// One row of Berrut basis functions, Section 3 eq. (2): given this lane's node x (valid
// lanes only), its sign and the evaluation point z, returns
//   (sign/(z-x)) / sum over valid lanes of (sign/(z-x)),
// or the unit vector of the node that equals z exactly.  Called by a whole wave; a row of
// more than 64 nodes is covered by two calls sharing one denominator (see callers).
struct BerrutTerm {
    double t;      // sign/(z-x), 0 on invalid lanes
    bool hit;      // z == x on this lane
};

__device__ __forceinline__ BerrutTerm berrut_term(double z, double x, double sign, bool valid) {
    BerrutTerm r;
    r.hit = valid && (z == x);
    r.t = (valid && !r.hit) ? sign / (z - x) : 0.0;
    return r;
}

// Host-side launchers (defined in encode.hip / decode.hip).
int launch_encode(const float *d_queries, float *d_coded, int64_t G, int K, int N, int64_t D,
                  const Nodes &nodes, hipStream_t stream);
int launch_decode(const float *d_preds, const uint8_t *d_mask, float *d_out, int32_t *d_status,
                  int64_t G, int K, int N, int S, int64_t C, const Nodes &nodes, int sign_mode,
                  hipStream_t stream);
int launch_decode_byzantine(const float *d_preds, const uint8_t *d_mask, float *d_out, int32_t *d_adv,
                            int32_t *d_status, int64_t G, int K, int N, int S, int A, int64_t C,
                            const Nodes &nodes, int sign_mode, hipStream_t stream);

}  // namespace approxifer
