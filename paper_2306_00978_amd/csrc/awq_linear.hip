// awq_w4a16_linear: validation and dispatch between the decode (M <= 16) and the
// prefill (M > 16) kernels.  AWQ Sec. 4.2: the same fused dequantization is used
// by the matrix-vector and the matrix-matrix kernel.
#include "awq_common.h"

int awq_gemv_launch(const void *x, const void *qweight, const void *scales, const void *zeros,
                    void *y, int M, int N, int K, hipStream_t stream);
int awq_gemm_launch(const void *x, const void *qweight, const void *scales, const void *zeros,
                    void *y, int M, int N, int K, hipStream_t stream);

extern "C" size_t awq_linear_workspace_bytes(int64_t M, int64_t N, int64_t K, int group)
{
    (void)M; (void)N; (void)K; (void)group;
    return 0;   // both paths reduce inside the workgroup; no global scratch
}

extern "C" int awq_w4a16_linear(const void *x_f16, const void *qweight, const void *scales,
                                const void *zeros, void *y_f16, int64_t M, int64_t N,
                                int64_t K, int group, void *workspace, size_t workspace_bytes,
                                void *stream)
{
    if (!x_f16 || !qweight || !scales || !zeros || !y_f16) return AWQ_ERR_NULL_POINTER;
    int st = awq_check_weight_shape(N, K, group);
    if (st != AWQ_OK) return st;
    if (M <= 0 || M > (int64_t)1 << 22) return AWQ_ERR_BAD_SHAPE;
    if (!awq_aligned16(x_f16) || !awq_aligned16(qweight) || !awq_aligned16(scales) ||
        !awq_aligned16(zeros) || !awq_aligned16(y_f16))
        return AWQ_ERR_MISALIGNED;
    const size_t need = awq_linear_workspace_bytes(M, N, K, group);
    if (need > 0) {
        if (!workspace) return AWQ_ERR_NULL_POINTER;
        if (workspace_bytes < need) return AWQ_ERR_WORKSPACE_TOO_SMALL;
        if (!awq_aligned16(workspace)) return AWQ_ERR_MISALIGNED;
    }
    if (M <= 16)
        return awq_gemv_launch(x_f16, qweight, scales, zeros, y_f16, (int)M, (int)N, (int)K,
                               (hipStream_t)stream);
    return awq_gemm_launch(x_f16, qweight, scales, zeros, y_f16, (int)M, (int)N, (int)K,
                           (hipStream_t)stream);
}
