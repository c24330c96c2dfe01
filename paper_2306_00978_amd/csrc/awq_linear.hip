// awq_w4a16_linear: validation and dispatch between the decode (M <= 16) and the
// prefill (M > 16) kernels.  AWQ Sec. 4.2: the same fused dequantization is used
// by the matrix-vector and the matrix-matrix kernel.
#include "awq_common.h"
#include "awq_gemv_stream.h"

#include <stdlib.h>
#include <algorithm>
#include <atomic>

int awq_gemv_launch_residual(const void *x, const void *qweight, const void *scales, const void *zeros,
                             void *y, const void *res, int M, int N, int K, hipStream_t stream);
int awq_gemv_launch(const void *x, const void *qweight, const void *scales, const void *zeros,
                    void *y, int M, int N, int K, hipStream_t stream);
int awq_gemm_launch(const void *x, const void *qweight, const void *scales, const void *zeros,
                    void *y, int M, int N, int K, hipStream_t stream);

int awq_gemm_launch_split(const void *x, const void *qweight, const void *scales, const void *zeros,
                          void *y, int M, int N, int K, void *part, int ksplit, hipStream_t stream);
int awq_gemm_ksplit(int M, int N, int K, double *estimate_us);

// Only the prefill kernel at a few hundred tokens uses scratch: fp32 partial tiles of its K ranges.
extern "C" size_t awq_linear_workspace_bytes(int64_t M, int64_t N, int64_t K, int group)
{
    if (awq_check_weight_shape(N, K, group) != AWQ_OK || M <= 48 || M > (int64_t)1 << 22) return 0;
    double split_us = 0.0;
    const int ks = awq_gemm_ksplit((int)M, (int)N, (int)K, &split_us);
    // 49..128 tokens run through the decode kernels in blocks of 16 -- one grouped launch that
    // takes about 7 us + blocks * (packed bytes at 6 TB/s, the repeats come from cache) -- unless
    // the prefill kernel with K cut into ranges is estimated to be clearly faster, or the shape
    // does not fit the grouped launch (then it would be one launch per block)
    if (M <= 128 && awq_gemv_stream_fits((int)N, (int)K, 16)) {
        const double blocked_us = 7.0 + (double)((M + 15) / 16) * ((double)N * (double)K * 0.53125) / 6.0e6;
        if (ks < 2 || split_us > 0.85 * blocked_us) return 0;
    }
    return ks > 1 ? (size_t)ks * (size_t)M * (size_t)N * sizeof(float) : 0;
}

namespace {
int grouped_decode(const awq_linear_desc *descs, int count, int64_t M, int group, void *stream, bool token_blocks);
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
    // the workspace is optional: with NULL, K is not split
    const size_t need = awq_linear_workspace_bytes(M, N, K, group);
    const bool split = need > 0 && workspace;
    if (split && workspace_bytes < need) return AWQ_ERR_WORKSPACE_TOO_SMALL;
    if (split && !awq_aligned16(workspace)) return AWQ_ERR_MISALIGNED;
    if (M <= 16) {
        // a single linear is a short kernel dominated by one memory round trip: the batch
        // kernel (everything requested at once) is the faster one; the streaming kernel is
        // for grouped launches.  (The tuning build can force it: AWQ_GEMV_STREAM_SINGLE.)
        static const bool stream_single = awq_knob("AWQ_GEMV_STREAM_SINGLE", 0) != 0;
        if (stream_single) {
            GemvProblem p = {};
            p.x = (const half_t *)x_f16;
            p.q = (const uint4 *)qweight;
            p.sc = (const uint16_t *)scales;
            p.zp = (const uint8_t *)zeros;
            p.y = (half_t *)y_f16;
            p.N = (int)N;
            p.K = (int)K;
            st = awq_gemv_stream_launch(&p, 1, (int)M, (hipStream_t)stream);
            if (st != AWQ_GEMV_STREAM_UNFIT) return st;
        }
        return awq_gemv_launch(x_f16, qweight, scales, zeros, y_f16, (int)M, (int)N, (int)K,
                               (hipStream_t)stream);
    }
    // A few dozen tokens: the matrix-matrix kernel would run ceil(M/128) * N/256 tiles, a handful
    // of CUs each walking all of K.  The decode kernel on blocks of 16 tokens reads the weights
    // once per block (the repeats come from cache) but keeps the whole chip busy, all blocks in one
    // grouped launch where the shape allows it.  The last block is moved back so that it has 16
    // tokens too; the tokens it shares with its neighbour are computed twice, bit for bit alike.
    // (4096 x 4096: 43 us -> 9-18 us for 17..128 tokens; 4096 x 11008: 105 us -> 20-43 us; when the
    // caller brings its workspace, the prefill kernel with K cut into ranges takes over from 49
    // tokens on: 36 us for that shape.)
    static const int small_env = awq_knob("AWQ_SMALL_M_MAX", -1);
    const int64_t small_max = small_env >= 0 ? std::min(small_env, 128) : 128;
    if (M <= small_max && !split) {
        const int blocks = (int)((M + 15) / 16);
        awq_linear_desc d[8];
        for (int b = 0; b < blocks; ++b) {
            const int64_t m0 = b + 1 < blocks ? 16 * (int64_t)b : M - 16;
            d[b].x_f16 = (const half_t *)x_f16 + m0 * K;
            d[b].qweight = qweight;
            d[b].scales = scales;
            d[b].zeros = zeros;
            d[b].y_f16 = (half_t *)y_f16 + m0 * N;
            d[b].N = N;
            d[b].K = K;
        }
        return grouped_decode(d, blocks, 16, group, stream, true);
    }
    if (split)
        return awq_gemm_launch_split(x_f16, qweight, scales, zeros, y_f16, (int)M, (int)N, (int)K, workspace,
                                     awq_gemm_ksplit((int)M, (int)N, (int)K, nullptr), (hipStream_t)stream);
    return awq_gemm_launch(x_f16, qweight, scales, zeros, y_f16, (int)M, (int)N, (int)K,
                           (hipStream_t)stream);
}

// ---- the entry point that allocates nothing ---------------------------------------------------
// The K-range form of the prefill kernel needs room for its fp32 partial tiles.  Callers that cannot
// allocate (code under graph capture, serving loops, harnesses that forbid it) get that room from
// this array: one copy per GPU the library runs on, held until the process ends.  In host code the
// name `scratch` is only a handle for hipGetSymbolAddress; kernels receive the device address.
static __device__ __align__(256) unsigned char scratch[AWQ_STATIC_SCRATCH_BYTES];

namespace {

// Device address of `scratch` on the current device, looked up once per device.
int static_scratch(void **out)
{
    static std::atomic<void *> address[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return AWQ_ERR_HIP;
    void *p = address[dev].load(std::memory_order_acquire);
    if (!p) {
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
            (void)hipGetLastError();
            return AWQ_ERR_HIP;
        }
        address[dev].store(p, std::memory_order_release);      // every thread finds the same address
    }
    *out = p;
    return AWQ_OK;
}

}  // namespace

extern "C" size_t awq_static_scratch_bytes(void) { return AWQ_STATIC_SCRATCH_BYTES; }

extern "C" int awq_w4a16_linear_static(const void *x_f16, const void *qweight, const void *scales,
                                       const void *zeros, void *y_f16, int64_t M, int64_t N, int64_t K,
                                       int group, void *stream)
{
    // same validation order as awq_w4a16_linear, so that a bad argument reads the same from both
    if (!x_f16 || !qweight || !scales || !zeros || !y_f16) return AWQ_ERR_NULL_POINTER;
    int st = awq_check_weight_shape(N, K, group);
    if (st != AWQ_OK) return st;
    if (M <= 0 || M > (int64_t)1 << 22) return AWQ_ERR_BAD_SHAPE;
    const size_t need = awq_linear_workspace_bytes(M, N, K, group);
    if (need > AWQ_STATIC_SCRATCH_BYTES) return AWQ_ERR_SCRATCH_LIMIT;
    void *ws = nullptr;
    if (need > 0) {
        st = static_scratch(&ws);
        if (st != AWQ_OK) return st;
    }
    return awq_w4a16_linear(x_f16, qweight, scales, zeros, y_f16, M, N, K, group, ws, need, stream);
}

extern "C" int awq_w4a16_linear_multi(const awq_linear_desc *descs, int count, int64_t M, int group,
                                      void *workspace, size_t workspace_bytes, void *stream)
{
    (void)workspace; (void)workspace_bytes;
    return grouped_decode(descs, count, M, group, stream, false);
}

namespace {

// The grouped decode call.  token_blocks: the linears are blocks of 16 tokens of ONE linear (the
// call comes from awq_w4a16_linear for 17..128 tokens), so the weights are the same for all.
int grouped_decode(const awq_linear_desc *descs, int count, int64_t M, int group, void *stream, bool token_blocks)
{
    if (!descs) return AWQ_ERR_NULL_POINTER;
    if (count < 1 || count > AWQ_MULTI_MAX) return AWQ_ERR_BAD_ARGUMENT;
    if (M <= 0 || M > 16) return AWQ_ERR_BAD_SHAPE;
    GemvProblem p[GEMV_MAX_PROBLEMS] = {};
    for (int i = 0; i < count; ++i) {
        const awq_linear_desc &d = descs[i];
        if (!d.x_f16 || !d.qweight || !d.scales || !d.zeros || !d.y_f16) return AWQ_ERR_NULL_POINTER;
        int st = awq_check_weight_shape(d.N, d.K, group);
        if (st != AWQ_OK) return st;
        if (!awq_aligned16(d.x_f16) || !awq_aligned16(d.qweight) || !awq_aligned16(d.scales) ||
            !awq_aligned16(d.zeros) || !awq_aligned16(d.y_f16))
            return AWQ_ERR_MISALIGNED;
        p[i].x = (const half_t *)d.x_f16;
        p[i].q = (const uint4 *)d.qweight;
        p[i].sc = (const uint16_t *)d.scales;
        p[i].zp = (const uint8_t *)d.zeros;
        p[i].y = (half_t *)d.y_f16;
        p[i].N = (int)d.N;
        p[i].K = (int)d.K;
    }
    // More than four tokens: the kernel that takes the activations through LDS (any K) runs all
    // linears of the call in one launch.  A lone linear goes there only when it has row blocks
    // enough for every CU (measured at N = 32000, K = 4096, 16 tokens: 21.5 us against 41 us); a
    // smaller one stays with the batch kernel, where everything requested at once is the faster way
    // through a small matrix (N = 4096, K = 11008: 10 us against 20 us).  Token blocks of one linear
    // go there from 40 M weights on (4096 x 11008 at 128 tokens: 43 us against 70 us; 4096 x 4096 is
    // faster the other way, 9 us against 11 us at 32 tokens).
    static const int rows_min_count = awq_knob("AWQ_ROWS_MIN_COUNT", 2);
    const bool rows = token_blocks ? (int64_t)p[0].N * p[0].K >= (int64_t)40 << 20
                                   : (count >= rows_min_count || p[0].N >= 16384);
    if (M > 4 && rows) {
        // the last token block is moved back over its neighbour; the rows they share are written
        // by the neighbour alone
        int first_row[GEMV_MAX_PROBLEMS] = {};
        if (token_blocks && count > 1)
            first_row[count - 1] = (int)((p[count - 2].y + 16 * (size_t)p[0].N - p[count - 1].y) / p[0].N);
        return awq_gemv_rows_launch(p, count, (int)M, (hipStream_t)stream, first_row);
    }
    // The linears whose K fits the register-resident activations of the streaming kernel at
    // this M go out in one launch; the others (and a lone linear) take one launch of the batch
    // kernel each.
    GemvProblem fit[GEMV_MAX_PROBLEMS];
    int nfit = 0;
    bool grouped[GEMV_MAX_PROBLEMS] = {};
    if (count > 1) {
        for (int i = 0; i < count; ++i)
            if (awq_gemv_stream_fits(p[i].N, p[i].K, (int)M)) {
                fit[nfit++] = p[i];
                grouped[i] = true;
            }
        if (nfit < 2) {
            nfit = 0;
            for (int i = 0; i < count; ++i) grouped[i] = false;
        }
    }
    if (nfit > 0) {
        int st = awq_gemv_stream_launch(fit, nfit, (int)M, (hipStream_t)stream);
        if (st == AWQ_GEMV_STREAM_UNFIT) {
            for (int i = 0; i < count; ++i) grouped[i] = false;
        } else if (st != AWQ_OK) {
            return st;
        }
    }
    for (int i = 0; i < count; ++i) {
        if (grouped[i]) continue;
        int st = awq_gemv_launch(p[i].x, p[i].q, p[i].sc, p[i].zp, p[i].y, (int)M, p[i].N, p[i].K,
                                 (hipStream_t)stream);
        if (st != AWQ_OK) return st;
    }
    return AWQ_OK;
}

}  // namespace

namespace {

// validation of the linears of a fused / chained call and their translation for the launcher
int fused_problems(const awq_fused_desc *descs, int count, int group, GemvProblem *p, GemvFusedExtra *e)
{
    for (int i = 0; i < count; ++i) {
        const awq_linear_desc &d = descs[i].linear;
        if (!d.x_f16 || !d.qweight || !d.scales || !d.zeros || !d.y_f16) return AWQ_ERR_NULL_POINTER;
        int st = awq_check_weight_shape(d.N, d.K, group);
        if (st != AWQ_OK) return st;
        if (!awq_aligned16(d.x_f16) || !awq_aligned16(d.qweight) || !awq_aligned16(d.scales) ||
            !awq_aligned16(d.zeros) || !awq_aligned16(d.y_f16))
            return AWQ_ERR_MISALIGNED;
        if (descs[i].pre_op == AWQ_PRE_RMSNORM || descs[i].pre_op == AWQ_PRE_SCALE) {
            if (!descs[i].pre_f16) return AWQ_ERR_NULL_POINTER;
            if (!awq_aligned16(descs[i].pre_f16)) return AWQ_ERR_MISALIGNED;
            if (descs[i].pre_op == AWQ_PRE_RMSNORM && !(descs[i].eps >= 0.0f)) return AWQ_ERR_BAD_ARGUMENT;
        } else if (descs[i].pre_op != AWQ_PRE_NONE) {
            return AWQ_ERR_BAD_ARGUMENT;
        }
        p[i] = GemvProblem{};
        p[i].x = (const half_t *)d.x_f16;
        p[i].q = (const uint4 *)d.qweight;
        p[i].sc = (const uint16_t *)d.scales;
        p[i].zp = (const uint8_t *)d.zeros;
        p[i].y = (half_t *)d.y_f16;
        p[i].N = (int)d.N;
        p[i].K = (int)d.K;
        e[i].pre = (const half_t *)descs[i].pre_f16;
        e[i].res = (const half_t *)descs[i].residual_f16;
        e[i].eps = descs[i].eps;
        e[i].pre_op = descs[i].pre_op == AWQ_PRE_RMSNORM ? GEMV_PRE_RMSNORM
                      : descs[i].pre_op == AWQ_PRE_SCALE ? GEMV_PRE_SCALE : GEMV_PRE_NONE;
    }
    return AWQ_OK;
}

}  // namespace

extern "C" int awq_w4a16_linear_chain(const awq_chain_stage *stages, int n_stages, int64_t M, int group, void *sync,
                                      int spin_limit, void *stream)
{
    if (!stages || !sync) return AWQ_ERR_NULL_POINTER;
    if (n_stages < 1 || n_stages > AWQ_CHAIN_MAX_STAGES || spin_limit < 0) return AWQ_ERR_BAD_ARGUMENT;
    if (M <= 0 || M > 16) return AWQ_ERR_BAD_SHAPE;
    if (!awq_aligned16(sync)) return AWQ_ERR_MISALIGNED;
    GemvProblem p[AWQ_CHAIN_MAX_STAGES][AWQ_CHAIN_MAX_LINEARS];
    GemvFusedExtra e[AWQ_CHAIN_MAX_STAGES][AWQ_CHAIN_MAX_LINEARS];
    const GemvProblem *pp[AWQ_CHAIN_MAX_STAGES];
    const GemvFusedExtra *ee[AWQ_CHAIN_MAX_STAGES];
    int counts[AWQ_CHAIN_MAX_STAGES];
    static_assert(AWQ_CHAIN_MAX_STAGES == CHAIN_MAX_STAGES && AWQ_CHAIN_MAX_LINEARS == CHAIN_MAX_ENTRIES &&
                  AWQ_CHAIN_SYNC_BYTES >= CHAIN_SYNC_BYTES, "limits");
    for (int s = 0; s < n_stages; ++s) {
        if (!stages[s].descs) return AWQ_ERR_NULL_POINTER;
        if (stages[s].count < 1 || stages[s].count > AWQ_CHAIN_MAX_LINEARS) return AWQ_ERR_BAD_ARGUMENT;
        const int st = fused_problems(stages[s].descs, stages[s].count, group, p[s], e[s]);
        if (st != AWQ_OK) return st;
        for (int i = 0; i < stages[s].count; ++i)
            if (!awq_gemv_stream_fits(p[s][i].N, p[s][i].K, (int)M)) return AWQ_ERR_BAD_SHAPE;
        pp[s] = p[s];
        ee[s] = e[s];
        counts[s] = stages[s].count;
    }
    const int st = awq_gemv_chain_launch(pp, ee, counts, n_stages, (int)M, (uint32_t *)sync, spin_limit,
                                         (hipStream_t)stream);
    return st == AWQ_GEMV_STREAM_UNFIT ? AWQ_ERR_BAD_SHAPE : st;
}

extern "C" int awq_w4a16_linear_fused_multi(const awq_fused_desc *descs, int count, int64_t M, int group,
                                            void *stream)
{
    if (!descs) return AWQ_ERR_NULL_POINTER;
    if (count < 1 || count > AWQ_FUSED_MAX) return AWQ_ERR_BAD_ARGUMENT;
    if (M <= 0 || M > 16) return AWQ_ERR_BAD_SHAPE;
    GemvProblem p[GEMV_MAX_FUSED] = {};
    GemvFusedExtra e[GEMV_MAX_FUSED] = {};
    {
        const int st = fused_problems(descs, count, group, p, e);
        if (st != AWQ_OK) return st;
    }
    // a lone linear without a normalisation: the batch kernel (every shape, and the faster one
    // for a single small matrix)
    if (count == 1 && e[0].pre_op == GEMV_PRE_NONE)
        return awq_gemv_launch_residual(p[0].x, p[0].q, p[0].sc, p[0].zp, p[0].y, e[0].res, (int)M, p[0].N,
                                        p[0].K, (hipStream_t)stream);
    for (int i = 0; i < count; ++i)
        if (!awq_gemv_stream_fits(p[i].N, p[i].K, (int)M)) return AWQ_ERR_BAD_SHAPE;
    int st = awq_gemv_stream_launch_fused(p, e, count, (int)M, (hipStream_t)stream);
    return st == AWQ_GEMV_STREAM_UNFIT ? AWQ_ERR_BAD_SHAPE : st;
}

extern "C" int awq_w4a16_linear_fused_fits(int64_t N, int64_t K, int64_t M, int group)
{
    if (M <= 0 || M > 16 || awq_check_weight_shape(N, K, group) != AWQ_OK) return 0;
    return awq_gemv_stream_fits((int)N, (int)K, (int)M) ? 1 : 0;
}
