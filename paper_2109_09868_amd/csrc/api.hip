// C ABI of the ApproxIFER coding layer: argument validation on the host, then one kernel
// launch on the caller's stream.  See include/approxifer.h for the contract.
#include <cmath>

#include "common.h"

using approxifer::Nodes;

namespace {

constexpr double kPi = 3.14159265358979323846264338327950288;

int check_nodes(const double *h, int n) {
    for (int i = 0; i < n; ++i) {
        if (!std::isfinite(h[i])) return APPROXIFER_ERR_BAD_NODES;
        for (int k = 0; k < i; ++k)
            if (h[k] == h[i]) return APPROXIFER_ERR_BAD_NODES;
    }
    return APPROXIFER_OK;
}

int check_common(int K, int N, const double *h_alpha, const double *h_beta, Nodes *nodes) {
    if (h_alpha == nullptr || h_beta == nullptr) return APPROXIFER_ERR_NULL_POINTER;
    if (K < 1 || N < 2) return APPROXIFER_ERR_BAD_SHAPE;
    if (K > APPROXIFER_MAX_K || N > APPROXIFER_MAX_N) return APPROXIFER_ERR_LIMIT;
    int rc = check_nodes(h_alpha, K);
    if (rc != APPROXIFER_OK) return rc;
    rc = check_nodes(h_beta, N);
    if (rc != APPROXIFER_OK) return rc;
    for (int j = 0; j < APPROXIFER_MAX_K; ++j) nodes->alpha[j] = j < K ? h_alpha[j] : 0.0;
    for (int i = 0; i < APPROXIFER_MAX_N; ++i) nodes->beta[i] = i < N ? h_beta[i] : 0.0;
    return APPROXIFER_OK;
}

}  // namespace

extern "C" {

int approxifer_version(void) { return 300; }   // 0.3.0: workspace arguments of the Byzantine decoders

const char *approxifer_strerror(int code) {
    switch (code) {
        case APPROXIFER_OK: return "ok";
        case APPROXIFER_ERR_NULL_POINTER: return "a required pointer is NULL";
        case APPROXIFER_ERR_BAD_SHAPE: return "bad shape: need G,D,C >= 0, K >= 1, N >= 2, -1 <= S < N, A >= 1";
        case APPROXIFER_ERR_LIMIT: return "size above the compiled limits (K <= 64, N <= 128, N-S <= 64 for the Byzantine decoder)";
        case APPROXIFER_ERR_BAD_NODES: return "nodes must be finite and pairwise distinct within each set";
        case APPROXIFER_ERR_TOO_FEW_WORKERS: return "the Byzantine decoder needs N - S >= 2 (K + A) available workers";
        case APPROXIFER_ERR_BAD_SIGN_MODE: return "sign_mode must be 0 (worker index) or 1 (survivor rank)";
        case APPROXIFER_ERR_LAUNCH: return "the HIP runtime refused the kernel launch";
        case APPROXIFER_ERR_WORKSPACE_LIMIT:
            return "the shape needs more scratch memory than the built-in workspace holds (APPROXIFER_STATIC_WORKSPACE_BYTES); "
                   "use approxifer_decode_byzantine with a workspace of approxifer_workspace_bytes()";
        default: return "unknown approxifer error code";
    }
}

int approxifer_chebyshev_nodes(int K, int N, double *h_alpha, double *h_beta) {
    if (h_alpha == nullptr || h_beta == nullptr) return APPROXIFER_ERR_NULL_POINTER;
    if (K < 1 || N < 2) return APPROXIFER_ERR_BAD_SHAPE;
    for (int j = 0; j < K; ++j) h_alpha[j] = std::cos((2.0 * j + 1.0) * kPi / (2.0 * K));
    for (int i = 0; i < N; ++i) h_beta[i] = std::cos(i * kPi / (N - 1.0));
    return APPROXIFER_OK;
}

int approxifer_encode(const float *d_queries, float *d_coded, int64_t G, int K, int N, int64_t D,
                      const double *h_alpha, const double *h_beta, void *stream) {
    if (G < 0 || D < 0) return APPROXIFER_ERR_BAD_SHAPE;
    Nodes nodes;
    const int rc = check_common(K, N, h_alpha, h_beta, &nodes);
    if (rc != APPROXIFER_OK) return rc;
    if (G == 0 || D == 0) return APPROXIFER_OK;
    if (d_queries == nullptr || d_coded == nullptr) return APPROXIFER_ERR_NULL_POINTER;
    return approxifer::launch_encode(d_queries, d_coded, G, K, N, D, nodes, static_cast<hipStream_t>(stream));
}

int64_t approxifer_group_count(int64_t Q, int K) {
    if (Q < 0 || K < 1) return -1;
    return (Q + K - 1) / K;
}

int approxifer_pad_last_group(float *d_queries, int64_t Q, int K, int64_t D, void *stream) {
    if (Q < 0 || D < 0 || K < 1) return APPROXIFER_ERR_BAD_SHAPE;
    if (K > APPROXIFER_MAX_K) return APPROXIFER_ERR_LIMIT;
    if (Q == 0 || D == 0 || Q % K == 0) return APPROXIFER_OK;
    if (d_queries == nullptr) return APPROXIFER_ERR_NULL_POINTER;
    return approxifer::launch_pad_last_group(d_queries, Q, K, D, static_cast<hipStream_t>(stream));
}

int approxifer_decode(const float *d_preds, const uint8_t *d_mask, float *d_out, int32_t *d_status, int64_t G, int K,
                      int N, int S, int64_t C, const double *h_alpha, const double *h_beta, int sign_mode,
                      void *stream) {
    if (G < 0 || C < 0) return APPROXIFER_ERR_BAD_SHAPE;
    Nodes nodes;
    const int rc = check_common(K, N, h_alpha, h_beta, &nodes);
    if (rc != APPROXIFER_OK) return rc;
    if (S < APPROXIFER_S_FROM_MASK || S >= N) return APPROXIFER_ERR_BAD_SHAPE;
    if (sign_mode != APPROXIFER_SIGN_WORKER_INDEX && sign_mode != APPROXIFER_SIGN_SURVIVOR_RANK)
        return APPROXIFER_ERR_BAD_SIGN_MODE;
    if (G == 0 || C == 0) return APPROXIFER_OK;
    if (d_mask == nullptr || d_preds == nullptr || d_out == nullptr) return APPROXIFER_ERR_NULL_POINTER;
    return approxifer::launch_decode(d_preds, d_mask, d_out, d_status, G, K, N, S, C, nodes, sign_mode,
                                     static_cast<hipStream_t>(stream));
}

int approxifer_decode_top1(const float *d_preds, const uint8_t *d_mask, int32_t *d_top1, float *d_score,
                           int32_t *d_status, int64_t G, int K, int N, int S, int64_t C, const double *h_alpha,
                           const double *h_beta, int sign_mode, void *stream) {
    if (G < 0 || C < 0) return APPROXIFER_ERR_BAD_SHAPE;
    Nodes nodes;
    const int rc = check_common(K, N, h_alpha, h_beta, &nodes);
    if (rc != APPROXIFER_OK) return rc;
    if (S < APPROXIFER_S_FROM_MASK || S >= N) return APPROXIFER_ERR_BAD_SHAPE;
    if (sign_mode != APPROXIFER_SIGN_WORKER_INDEX && sign_mode != APPROXIFER_SIGN_SURVIVOR_RANK)
        return APPROXIFER_ERR_BAD_SIGN_MODE;
    if (C > 0x7fffffffLL) return APPROXIFER_ERR_LIMIT;   // class indices are int32
    if (G == 0 || C == 0) return APPROXIFER_OK;
    if (d_mask == nullptr || d_preds == nullptr || d_top1 == nullptr) return APPROXIFER_ERR_NULL_POINTER;
    return approxifer::launch_decode_top1(d_preds, d_mask, d_top1, d_score, d_status, G, K, N, S, C, nodes,
                                          sign_mode, static_cast<hipStream_t>(stream));
}

static int decode_byzantine_checked(const float *d_preds, const uint8_t *d_mask, float *d_out, int32_t *d_adv,
                                    int32_t *d_status, int64_t G, int K, int N, int S, int A, int64_t C,
                                    const double *h_alpha, const double *h_beta, int sign_mode, bool homogeneous,
                                    void *d_workspace, size_t workspace_bytes, void *stream) {
    if (G < 0 || C < 0) return APPROXIFER_ERR_BAD_SHAPE;
    Nodes nodes;
    const int rc = check_common(K, N, h_alpha, h_beta, &nodes);
    if (rc != APPROXIFER_OK) return rc;
    if (S < APPROXIFER_S_FROM_MASK || S >= N || A < 1) return APPROXIFER_ERR_BAD_SHAPE;
    if (sign_mode != APPROXIFER_SIGN_WORKER_INDEX && sign_mode != APPROXIFER_SIGN_SURVIVOR_RANK)
        return APPROXIFER_ERR_BAD_SIGN_MODE;
    const int most_available = S < 0 ? N : N - S;
    if (most_available < 2 * (K + A)) return APPROXIFER_ERR_TOO_FEW_WORKERS;
    if (S >= 0 && N - S > APPROXIFER_MAX_AVAIL_BYZ) return APPROXIFER_ERR_LIMIT;
    if (G == 0 || C == 0) return APPROXIFER_OK;
    if (d_mask == nullptr || d_adv == nullptr || d_preds == nullptr || d_out == nullptr)
        return APPROXIFER_ERR_NULL_POINTER;
    return approxifer::launch_decode_byzantine(d_preds, d_mask, d_out, d_adv, d_status, G, K, N, S, A, C, nodes,
                                               sign_mode, homogeneous, d_workspace, workspace_bytes,
                                               static_cast<hipStream_t>(stream));
}

int approxifer_decode_byzantine(const float *d_preds, const uint8_t *d_mask, float *d_out, int32_t *d_adv,
                                int32_t *d_status, int64_t G, int K, int N, int S, int A, int64_t C,
                                const double *h_alpha, const double *h_beta, int sign_mode, void *d_workspace,
                                size_t workspace_bytes, void *stream) {
    return decode_byzantine_checked(d_preds, d_mask, d_out, d_adv, d_status, G, K, N, S, A, C, h_alpha, h_beta,
                                    sign_mode, false, d_workspace, workspace_bytes, stream);
}

int approxifer_decode_byzantine_homogeneous(const float *d_preds, const uint8_t *d_mask, float *d_out,
                                            int32_t *d_adv, int32_t *d_status, int64_t G, int K, int N, int S,
                                            int A, int64_t C, const double *h_alpha, const double *h_beta,
                                            int sign_mode, void *d_workspace, size_t workspace_bytes, void *stream) {
    return decode_byzantine_checked(d_preds, d_mask, d_out, d_adv, d_status, G, K, N, S, A, C, h_alpha, h_beta,
                                    sign_mode, true, d_workspace, workspace_bytes, stream);
}

int approxifer_decode_rational(const float *d_preds, const uint8_t *d_mask, float *d_out, int32_t *d_status, int64_t G,
                               int K, int N, int S, int A, int64_t C, const double *h_alpha, const double *h_beta,
                               void *stream) {
    if (G < 0 || C < 0) return APPROXIFER_ERR_BAD_SHAPE;
    Nodes nodes;
    const int rc = check_common(K, N, h_alpha, h_beta, &nodes);
    if (rc != APPROXIFER_OK) return rc;
    if (S < APPROXIFER_S_FROM_MASK || S >= N || A < 1) return APPROXIFER_ERR_BAD_SHAPE;
    const int most_available = S < 0 ? N : N - S;
    if (most_available < 2 * (K + A)) return APPROXIFER_ERR_TOO_FEW_WORKERS;
    if (S >= 0 && N - S > APPROXIFER_MAX_AVAIL_BYZ) return APPROXIFER_ERR_LIMIT;
    if (G == 0 || C == 0) return APPROXIFER_OK;
    if (d_mask == nullptr || d_preds == nullptr || d_out == nullptr) return APPROXIFER_ERR_NULL_POINTER;
    return approxifer::launch_decode_rational(d_preds, d_mask, d_out, d_status, G, K, N, S, A, C, nodes,
                                              static_cast<hipStream_t>(stream));
}

int approxifer_decode_byzantine_static(const float *d_preds, const uint8_t *d_mask, float *d_out, int32_t *d_adv,
                                       int32_t *d_status, int64_t G, int K, int N, int S, int A, int64_t C,
                                       const double *h_alpha, const double *h_beta, int sign_mode, void *stream) {
    // shapes the decoder refuses are refused by the checked call below with their own codes (need is 0 for them)
    const size_t need = approxifer_workspace_bytes(G, K, N, S, A, C);
    if (need > APPROXIFER_STATIC_WORKSPACE_BYTES) return APPROXIFER_ERR_WORKSPACE_LIMIT;
    void *d_scratch = nullptr;
    if (need > 0) {
        const int rc = approxifer::static_workspace(&d_scratch);
        if (rc != APPROXIFER_OK) return rc;
    }
    return decode_byzantine_checked(d_preds, d_mask, d_out, d_adv, d_status, G, K, N, S, A, C, h_alpha, h_beta,
                                    sign_mode, false, d_scratch, need, stream);
}

size_t approxifer_workspace_bytes(int64_t G, int K, int N, int S, int A, int64_t C) {
    // the shapes the Byzantine decoders accept; anything else needs no workspace because the call is refused
    if (G <= 0 || C <= 0 || K < 1 || K > APPROXIFER_MAX_K || N < 2 || N > APPROXIFER_MAX_N) return 0;
    if (S < APPROXIFER_S_FROM_MASK || S >= N || A < 1) return 0;
    const int most_available = S < 0 ? N : N - S;
    if (most_available < 2 * (K + A) || (S >= 0 && N - S > APPROXIFER_MAX_AVAIL_BYZ)) return 0;
    return approxifer::byzantine_workspace_bytes(G, K, N, S, A, C);
}

int approxifer_top1(const float *d_values, int32_t *d_top1, float *d_score, int64_t rows, int64_t C, void *stream) {
    if (rows < 0 || C < 0) return APPROXIFER_ERR_BAD_SHAPE;
    if (C > 0x7fffffffLL) return APPROXIFER_ERR_LIMIT;   // class indices are int32
    if (rows == 0 || C == 0) return APPROXIFER_OK;
    if (d_values == nullptr || d_top1 == nullptr) return APPROXIFER_ERR_NULL_POINTER;
    return approxifer::launch_argmax_rows(d_values, d_top1, d_score, rows, C, static_cast<hipStream_t>(stream));
}

int approxifer_wait_mask(const float *d_arrival, uint8_t *d_mask, int32_t *d_count, int64_t G, int N, int wait_for,
                         void *stream) {
    if (G < 0 || N < 1 || wait_for < 1 || wait_for > N) return APPROXIFER_ERR_BAD_SHAPE;
    if (N > APPROXIFER_MAX_N) return APPROXIFER_ERR_LIMIT;
    if (G == 0) return APPROXIFER_OK;
    if (d_arrival == nullptr || d_mask == nullptr) return APPROXIFER_ERR_NULL_POINTER;
    return approxifer::launch_wait_mask(d_arrival, d_mask, d_count, G, N, wait_for, static_cast<hipStream_t>(stream));
}

}  // extern "C"
