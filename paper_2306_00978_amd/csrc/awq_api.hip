// Version, status strings and size queries of the C ABI (host only).
#include "awq_common.h"

extern "C" int awq_version(void) { return 1; }

extern "C" const char *awq_status_string(int status)
{
    switch (status) {
    case AWQ_OK: return "ok";
    case AWQ_ERR_NULL_POINTER: return "null pointer";
    case AWQ_ERR_BAD_SHAPE: return "bad shape (sizes must be positive, K % 128 == 0, N % 16 == 0)";
    case AWQ_ERR_UNSUPPORTED_GROUP: return "unsupported group size (only 128)";
    case AWQ_ERR_MISALIGNED: return "tensor pointer is not 16-byte aligned";
    case AWQ_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
    case AWQ_ERR_HIP: return "HIP runtime refused the launch";
    case AWQ_ERR_BAD_ARGUMENT: return "scalar argument out of range";
    default: return "unknown status";
    }
}

extern "C" int awq_packed_sizes(int64_t N, int64_t K, int group, size_t *qweight_bytes,
                                size_t *scales_bytes, size_t *zeros_bytes)
{
    int st = awq_check_weight_shape(N, K, group);
    if (st != AWQ_OK) return st;
    const int64_t G = K / AWQ_GROUP;
    if (qweight_bytes) *qweight_bytes = (size_t)(N * K / 2);
    if (scales_bytes) *scales_bytes = (size_t)(N * G * 2);
    if (zeros_bytes) *zeros_bytes = (size_t)(N * G / 2);
    return AWQ_OK;
}
