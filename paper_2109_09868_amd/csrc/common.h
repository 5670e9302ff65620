// Shared device helpers of the ApproxIFER coding-layer kernels (gfx950, wave64).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <tuple>
#include <type_traits>
#include <utility>

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

// ---- wavefront reductions -------------------------------------------------------------
// Data-parallel-primitive (DPP) lane exchanges inside a row of 16 lanes; no LDS round trip.
constexpr int kDppQuadXor1 = 0xB1;       // quad_perm:[1,0,3,2]
constexpr int kDppQuadXor2 = 0x4E;       // quad_perm:[2,3,0,1]
constexpr int kDppRowHalfMirror = 0x141; // lane i <-> 7-i inside each half row
constexpr int kDppRowMirror = 0x140;     // lane i <-> 15-i inside each row

template <int CTRL>
__device__ __forceinline__ double dpp_exchange(double v) {
    // every pattern used here reads an existing lane of the same row, all rows and banks are enabled:
    // the 'old' operand is dead, and bound_ctrl tells the compiler so (no extra move per exchange)
    const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(v), CTRL, 0xF, 0xF, true);
    const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(v), CTRL, 0xF, 0xF, true);
    return __hiloint2double(hi, lo);
}

__device__ __forceinline__ double read_lane(double v, int lane) {
    const int lo = __builtin_amdgcn_readlane(__double2loint(v), lane);
    const int hi = __builtin_amdgcn_readlane(__double2hiint(v), lane);
    return __hiloint2double(hi, lo);
}

// Marks a wave-uniform value as such (it then lives in scalar registers, and a load that
// produces it stays a scalar load instead of being merged into a per-lane address select).
__device__ __forceinline__ double wave_uniform(double v) {
    const int lo = __builtin_amdgcn_readfirstlane(__double2loint(v));
    const int hi = __builtin_amdgcn_readfirstlane(__double2hiint(v));
    return __hiloint2double(hi, lo);
}

// Sum of v over each aligned group of 16 lanes, returned in every lane of the group.
// Fixed association: ((x0+x1)+(x2+x3)) + ((x4+x5)+(x6+x7)) ... as a butterfly.
__device__ __forceinline__ double row16_sum(double v) {
    v += dpp_exchange<kDppQuadXor1>(v);
    v += dpp_exchange<kDppQuadXor2>(v);
    v += dpp_exchange<kDppRowHalfMirror>(v);   // quads are uniform by now: adds the other quad of the half row
    v += dpp_exchange<kDppRowMirror>(v);       // half rows are uniform: adds the other half row
    return v;
}

// Sum over each aligned group of WIDTH lanes (16, 32 or 64), returned in every lane of the group.
template <int WIDTH>
__device__ __forceinline__ double group_sum(double v) {
    static_assert(WIDTH == 16 || WIDTH == 32 || WIDTH == 64, "group width");
    v = row16_sum(v);
    if (WIDTH == 16) return v;
    const double r0 = read_lane(v, 0), r1 = read_lane(v, 16), r2 = read_lane(v, 32), r3 = read_lane(v, 48);
    if (WIDTH == 32) return (threadIdx.x & 32) ? (r2 + r3) : (r0 + r1);
    return (r0 + r1) + (r2 + r3);
}

__device__ __forceinline__ double wave_sum(double v) { return group_sum<64>(v); }

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

// Enqueues `kernel` and returns the status of THIS launch.  An error that an earlier, unrelated HIP call left in the
// calling thread's error state is neither taken for a failure of the launch nor cleared from the caller's view.
template <typename... Params, size_t... I>
inline hipError_t launch_kernel_indexed(void (*kernel)(Params...), dim3 grid, dim3 block, size_t lds, hipStream_t stream,
                                        std::tuple<std::remove_cv_t<Params>...> &vals, std::index_sequence<I...>) {
    void *ptrs[] = {static_cast<void *>(&std::get<I>(vals))...};
    return hipLaunchKernel(reinterpret_cast<const void *>(kernel), grid, block, ptrs, lds, stream);
}
template <typename... Params, typename... Args>
inline hipError_t launch_kernel(void (*kernel)(Params...), dim3 grid, dim3 block, size_t lds, hipStream_t stream,
                                Args &&...args) {
    static_assert(sizeof...(Params) == sizeof...(Args), "one argument per kernel parameter");
    std::tuple<std::remove_cv_t<Params>...> vals(static_cast<std::remove_cv_t<Params>>(args)...);
    return launch_kernel_indexed(kernel, grid, block, lds, stream, vals, std::index_sequence_for<Params...>{});
}
inline int launch_status(hipError_t e) { return e == hipSuccess ? APPROXIFER_OK : APPROXIFER_ERR_LAUNCH; }

// Host-side launchers (defined in encode.hip / decode.hip / byzantine.hip).
int launch_encode(const float *d_queries, float *d_coded, int64_t G, int K, int N, int64_t D,
                  const Nodes &nodes, hipStream_t stream);
int launch_pad_last_group(float *d_queries, int64_t Q, int K, int64_t D, hipStream_t stream);
int launch_decode(const float *d_preds, const uint8_t *d_mask, float *d_out, int32_t *d_status,
                  int64_t G, int K, int N, int S, int64_t C, const Nodes &nodes, int sign_mode,
                  hipStream_t stream);
int launch_decode_top1(const float *d_preds, const uint8_t *d_mask, int32_t *d_top1, float *d_score,
                       int32_t *d_status, int64_t G, int K, int N, int S, int64_t C, const Nodes &nodes,
                       int sign_mode, hipStream_t stream);
int launch_decode_byzantine(const float *d_preds, const uint8_t *d_mask, float *d_out, int32_t *d_adv,
                            int32_t *d_status, int64_t G, int K, int N, int S, int A, int64_t C,
                            const Nodes &nodes, int sign_mode, bool homogeneous, void *d_workspace,
                            size_t workspace_bytes, hipStream_t stream);
int launch_decode_rational(const float *d_preds, const uint8_t *d_mask, float *d_out, int32_t *d_status, int64_t G, int K,
                           int N, int S, int A, int64_t C, const Nodes &nodes, hipStream_t stream);
size_t byzantine_workspace_bytes(int64_t G, int K, int N, int S, int A, int64_t C);
int static_workspace(void **d_ptr);

int launch_argmax_rows(const float *d_values, int32_t *d_top1, float *d_score, int64_t rows, int64_t C,
                       hipStream_t stream);
int launch_wait_mask(const float *d_arrival, uint8_t *d_mask, int32_t *d_count, int64_t G, int N, int wait_for,
                     hipStream_t stream);

}  // namespace approxifer
