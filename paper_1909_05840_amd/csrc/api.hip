// Host-only entry points of the C ABI: status strings and buffer sizes.
#include "qb_common.hpp"

using namespace qb;

extern "C" const char *qb_status_string(qb_status s)
{
    switch (s) {
        case QB_OK: return "ok";
        case QB_ERR_NULL: return "a required pointer is NULL";
        case QB_ERR_BITS: return "bits must be 2, 3, 4 or 8";
        case QB_ERR_SHAPE: return "invalid shape (dims must be positive, K a multiple of 64 and <= 32768, N divisible by groups)";
        case QB_ERR_CLIP: return "activation range must be a positive finite number";
        case QB_ERR_WORKSPACE: return "workspace missing or not 256-byte aligned";
        case QB_ERR_HIP: return "the HIP runtime refused a kernel launch";
    }
    return "unknown status";
}

extern "C" size_t qb_packed_nbytes(int64_t N, int64_t K, int bits)
{
    if (!bits_ok(bits) || N <= 0 || N > (1 << 24) || !k_ok(K)) return 0;
    return (size_t)padded_rows(N) * (size_t)K * (size_t)bits / 8;
}

// declared in bwd_bf16.hip and hessian.hip
extern "C" size_t qb_bwd_workspace_nbytes(int64_t T, int64_t N, int64_t K);
extern "C" size_t qb_power_iteration_scratch_floats(void);

extern "C" size_t qb_workspace_nbytes(int op, int64_t T, int64_t N, int64_t K, int bits)
{
    switch (op) {
        case QB_OP_QLINEAR_BWD_STE:
            return bits_ok(bits) ? qb_bwd_workspace_nbytes(T, N, K) : 0;
        case QB_OP_POWER_ITERATION:
            return qb_power_iteration_scratch_floats() * sizeof(float);
        default:  // the quantizers, the forward calls and the embedding calls work in their inputs and outputs only
            return 0;
    }
}
