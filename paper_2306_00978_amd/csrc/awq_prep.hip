// awq_act_scale / awq_apply_inv_scale for gfx950.
//
// AWQ Sec. 3.2: the saliency of a weight channel is decided by the magnitude of
// its input activation; Eq. 5 takes s = s_X^alpha with s_X the per-input-channel
// mean |X| over the calibration rows, and Eq. 4 moves diag(s)^-1 onto the
// activations.  Both are plain streaming passes over X (HBM-bound).
#include "awq_common.h"

#include <algorithm>

namespace {

constexpr int ACT_COLS = 64;     // columns per workgroup (8 lanes x 8 halves = one 128-byte line per row)
constexpr int ACT_PHASES = 128;  // row phases per workgroup (1024 threads)
constexpr int ACT_MAX = 16;      // matrices per launch

struct ActProblem {
    const uint4 *X;
    float *s;
    int64_t T, K;
    int wg_begin, pad;
};
struct ActArgs {
    ActProblem p[ACT_MAX];
    int count;
    float alpha;
};

// Up to 16 matrices per launch.  A workgroup (1024 threads) owns 64 columns of one matrix and walks
// all its T rows; thread (phase, oct) sums |x| of rows phase, phase + 128, ... for its eight
// columns.  The 128 partial sums per column are then added in a fixed tree order, so the result is
// deterministic and does not depend on what else the launch holds.  RAW: store the (floored) mean
// itself instead of its power.
// The sums are per column, so the workgroups divide the columns, and a matrix gives K / 64 of
// them: 172 for K = 11008 (5.2 TB/s at 65 536 rows) but 64 for K = 4096, a quarter of the chip --
// a CU alone takes in about 33 GB/s whatever the number of loads in flight (2.1-2.2 TB/s).
// Narrower column blocks (16 columns, the workgroups that share a 128-byte line on one XCD) reach
// 2.5 TB/s for K = 4096 and are slower for wide K; dividing the rows over workgroups would need
// a place for partial sums, which the call does not have.  What fills the chip is several
// matrices per launch (awq_act_scale_multi): a decoder layer has four distinct inputs to calibrate.
template <bool RAW>
__global__ __launch_bounds__(1024) void act_scale_kernel(const ActArgs A)
{
    __shared__ float red[ACT_PHASES][ACT_COLS];
    int pi = 0;
    for (int i = 1; i < A.count; ++i)
        if ((int)blockIdx.x >= A.p[i].wg_begin) pi = i;
    const uint4 *__restrict__ X = A.p[pi].X;
    float *__restrict__ s = A.p[pi].s;
    const int64_t T = A.p[pi].T, K = A.p[pi].K;
    const int cb = (int)blockIdx.x - A.p[pi].wg_begin;
    const float alpha = A.alpha;
    const int oct = threadIdx.x & 7;
    const int phase = threadIdx.x >> 3;
    const int64_t col0 = (int64_t)cb * ACT_COLS + oct * 8;
    float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    if (col0 < K) {
        const int64_t K8 = K / 8;
        const uint4 *p = X + col0 / 8;
        // eight rows requested before the first is added; the additions keep the order of the rows
        constexpr int AHEAD = 8;
        int64_t t = phase;
        for (; t + (AHEAD - 1) * ACT_PHASES < T; t += AHEAD * ACT_PHASES) {
            uint4 raw[AHEAD];
#pragma unroll
            for (int a = 0; a < AHEAD; ++a) raw[a] = p[(t + a * ACT_PHASES) * K8];
#pragma unroll
            for (int a = 0; a < AHEAD; ++a) {
                const half_t *h = reinterpret_cast<const half_t *>(&raw[a]);
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[e] += __builtin_fabsf((float)h[e]);
            }
        }
        for (; t < T; t += ACT_PHASES) {
            uint4 raw = p[t * K8];
            const half_t *h = reinterpret_cast<const half_t *>(&raw);
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[e] += __builtin_fabsf((float)h[e]);
        }
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) red[phase][oct * 8 + e] = acc[e];
    __syncthreads();
    for (int half = ACT_PHASES / 2; half >= 1; half >>= 1) {
        for (int i = threadIdx.x; i < half * ACT_COLS; i += 1024) {
            const int p = i / ACT_COLS, cidx = i % ACT_COLS;
            red[p][cidx] += red[p + half][cidx];
        }
        __syncthreads();
    }
    if (threadIdx.x < ACT_COLS) {
        const int64_t col = (int64_t)cb * ACT_COLS + threadIdx.x;
        if (col < K) {
            float mean = red[0][threadIdx.x] / (float)T;
            mean = fmaxf(mean, 1e-4f);
            s[col] = RAW ? mean : powf(mean, alpha);
        }
    }
}

template <bool RAW>
int act_scale_launch(const ActProblem *probs, int count, float alpha, hipStream_t stream)
{
    ActArgs A = {};
    int wg = 0;
    for (int i = 0; i < count; ++i) {
        A.p[i] = probs[i];
        A.p[i].wg_begin = wg;
        wg += (int)((probs[i].K + ACT_COLS - 1) / ACT_COLS);
    }
    A.count = count;
    A.alpha = alpha;
    act_scale_kernel<RAW><<<dim3(wg), dim3(1024), 0, stream>>>(A);
    return awq_launch_status();
}

int act_scale_check(const void *X_f16, int64_t T, int64_t K, const float *s)
{
    if (!X_f16 || !s) return AWQ_ERR_NULL_POINTER;
    if (T <= 0 || K <= 0 || (K % 8) != 0 || K > (int64_t)1 << 30) return AWQ_ERR_BAD_SHAPE;
    if (!awq_aligned16(X_f16) || !awq_aligned16(s)) return AWQ_ERR_MISALIGNED;
    return AWQ_OK;
}

__global__ __launch_bounds__(256) void apply_inv_scale_kernel(const uint4 *__restrict__ x,
                                                              const float4 *__restrict__ s,
                                                              int64_t runs_total, int64_t K8,
                                                              uint4 *__restrict__ xs)
{
    // all arguments fetched in one round (otherwise one scalar-cache miss per first use)
    asm volatile("" ::"s"(x), "s"(s), "s"(runs_total), "s"(K8), "s"(xs));
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= runs_total) return;
    const int64_t run = i % K8;
    uint4 raw = x[i];
    const half_t *h = reinterpret_cast<const half_t *>(&raw);
    const float4 a = s[2 * run], b = s[2 * run + 1];
    const float sv[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
    uint4 out;
    half_t *o = reinterpret_cast<half_t *>(&out);
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = (half_t)((float)h[e] / sv[e]);
    xs[i] = out;
}

// RMS normalisation with the 1/s factor of Eq. 4 folded in (Sec. 4.2: the operators of the
// normalisation in one kernel; Sec. 3.2, Eq. 4: the diag(s)^-1 factor belongs to the producer
// of x).  One workgroup per row: sum of squares with 16-byte loads (the row is read a second
// time from cache for the output), wave shuffles and one pass through LDS, then
// x * rsqrt(mean + eps) * gamma / s in fp32, rounded once to fp16.
__global__ __launch_bounds__(256) void rmsnorm_inv_scale_kernel(const uint4 *__restrict__ x,
                                                                const uint4 *__restrict__ gamma,
                                                                const float4 *__restrict__ s,
                                                                int64_t K8, float inv_k, float eps,
                                                                uint4 *__restrict__ xs)
{
    // all arguments fetched in one round (otherwise one scalar-cache miss per first use)
    asm volatile("" ::"s"(x), "s"(gamma), "s"(s), "s"(K8), "s"(inv_k), "s"(eps), "s"(xs));
    __shared__ float part[4];
    const uint4 *row = x + (int64_t)blockIdx.x * K8;
    // The first KEEP x 256 runs of the row (K <= 8192: all of it) stay in registers, and their
    // gamma and s are requested in the same round, before the reduction: a decode call is one
    // short row, and every further round trip to memory would be a third of its time.
    constexpr int KEEP = 4;
    uint4 raw[KEEP], graw[KEEP];
    float4 sa[KEEP], sb[KEEP];
#pragma unroll
    for (int j = 0; j < KEEP; ++j) {
        const int64_t i = threadIdx.x + 256 * j, ic = i < K8 ? i : K8 - 1;
        raw[j] = row[ic];
        graw[j] = gamma[ic];
        if (s) {
            sa[j] = s[2 * ic];
            sb[j] = s[2 * ic + 1];
        } else {
            sa[j] = sb[j] = make_float4(1.f, 1.f, 1.f, 1.f);
        }
    }
    float ss = 0.f;
#pragma unroll
    for (int j = 0; j < KEEP; ++j) {
        const half_t *h = reinterpret_cast<const half_t *>(&raw[j]);
        float t = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) t += (float)h[e] * (float)h[e];
        ss += threadIdx.x + 256 * j < K8 ? t : 0.f;
    }
    for (int64_t i = threadIdx.x + 256 * KEEP; i < K8; i += 256) {
        const uint4 r = row[i];
        const half_t *h = reinterpret_cast<const half_t *>(&r);
#pragma unroll
        for (int e = 0; e < 8; ++e) ss += (float)h[e] * (float)h[e];
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) ss += __shfl_xor(ss, d);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = ss;
    __syncthreads();
    const float total = (part[0] + part[1]) + (part[2] + part[3]);
    const float inv = 1.0f / sqrtf(total * inv_k + eps);
    uint4 *out = xs + (int64_t)blockIdx.x * K8;
    auto emit = [&](int64_t i, const uint4 &r, const uint4 &g, const float4 &a, const float4 &b) {
        const half_t *h = reinterpret_cast<const half_t *>(&r);
        const half_t *gm = reinterpret_cast<const half_t *>(&g);
        const float sv[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
        uint4 o;
        half_t *oh = reinterpret_cast<half_t *>(&o);
#pragma unroll
        for (int e = 0; e < 8; ++e) oh[e] = (half_t)(((float)h[e] * inv) * (float)gm[e] / sv[e]);
        out[i] = o;
    };
#pragma unroll
    for (int j = 0; j < KEEP; ++j) {
        const int64_t i = threadIdx.x + 256 * j;
        if (i < K8) emit(i, raw[j], graw[j], sa[j], sb[j]);
    }
    for (int64_t i = threadIdx.x + 256 * KEEP; i < K8; i += 256) {
        const float4 one = make_float4(1.f, 1.f, 1.f, 1.f);
        emit(i, row[i], gamma[i], s ? s[2 * i] : one, s ? s[2 * i + 1] : one);
    }
}

// silu(gate) * up, element-wise (the gated activation between gate/up and down): fp32, one rounding
__global__ __launch_bounds__(256) void silu_mul_kernel(const uint4 *__restrict__ gate,
                                                       const uint4 *__restrict__ up, int64_t n8,
                                                       uint4 *__restrict__ out)
{
    // all arguments fetched in one round (otherwise one scalar-cache miss per first use)
    asm volatile("" ::"s"(gate), "s"(up), "s"(n8), "s"(out));
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n8) return;
    const uint4 graw = gate[i], uraw = up[i];
    const half_t *g = reinterpret_cast<const half_t *>(&graw);
    const half_t *u = reinterpret_cast<const half_t *>(&uraw);
    uint4 o;
    half_t *oh = reinterpret_cast<half_t *>(&o);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const float x = (float)g[e];
        oh[e] = (half_t)(x / (1.0f + expf(-x)) * (float)u[e]);
    }
    out[i] = o;
}

}  // namespace

extern "C" int awq_silu_mul(const void *gate_f16, const void *up_f16, int64_t n, void *out_f16,
                            void *stream)
{
    if (!gate_f16 || !up_f16 || !out_f16) return AWQ_ERR_NULL_POINTER;
    if (n <= 0 || (n % 8) != 0 || n > (int64_t)1 << 40) return AWQ_ERR_BAD_SHAPE;
    if (!awq_aligned16(gate_f16) || !awq_aligned16(up_f16) || !awq_aligned16(out_f16))
        return AWQ_ERR_MISALIGNED;
    const int64_t n8 = n / 8, blocks = (n8 + 255) / 256;
    if (blocks > 0x7fffffff) return AWQ_ERR_BAD_SHAPE;
    silu_mul_kernel<<<dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream>>>(
        (const uint4 *)gate_f16, (const uint4 *)up_f16, n8, (uint4 *)out_f16);
    return awq_launch_status();
}

extern "C" int awq_rmsnorm_inv_scale(const void *x_f16, const void *gamma_f16, const float *s,
                                     int64_t M, int64_t K, float eps, void *xs_f16, void *stream)
{
    if (!x_f16 || !gamma_f16 || !xs_f16) return AWQ_ERR_NULL_POINTER;
    if (M <= 0 || K <= 0 || (K % 8) != 0 || M > 0x7fffffff || K > (int64_t)1 << 30)
        return AWQ_ERR_BAD_SHAPE;
    if (!(eps >= 0.0f)) return AWQ_ERR_BAD_ARGUMENT;
    if (!awq_aligned16(x_f16) || !awq_aligned16(gamma_f16) || !awq_aligned16(xs_f16) ||
        (s && !awq_aligned16(s)))
        return AWQ_ERR_MISALIGNED;
    rmsnorm_inv_scale_kernel<<<dim3((unsigned)M), dim3(256), 0, (hipStream_t)stream>>>(
        (const uint4 *)x_f16, (const uint4 *)gamma_f16, (const float4 *)s, K / 8, 1.0f / (float)K, eps,
        (uint4 *)xs_f16);
    return awq_launch_status();
}

extern "C" int awq_act_scale(const void *X_f16, int64_t T, int64_t K, float alpha, float *s,
                             void *stream)
{
    const int st = act_scale_check(X_f16, T, K, s);
    if (st != AWQ_OK) return st;
    if (!(alpha >= 0.0f && alpha <= 1.0f)) return AWQ_ERR_BAD_ARGUMENT;
    const ActProblem p = {(const uint4 *)X_f16, s, T, K, 0, 0};
    return act_scale_launch<false>(&p, 1, alpha, (hipStream_t)stream);
}

extern "C" int awq_act_scale_multi(const awq_act_scale_desc *descs, int count, float alpha, void *stream)
{
    if (!descs) return AWQ_ERR_NULL_POINTER;
    if (count < 1 || count > AWQ_ACT_SCALE_MULTI_MAX) return AWQ_ERR_BAD_ARGUMENT;
    if (!(alpha >= 0.0f && alpha <= 1.0f)) return AWQ_ERR_BAD_ARGUMENT;
    static_assert(AWQ_ACT_SCALE_MULTI_MAX % ACT_MAX == 0, "whole launches");
    for (int i = 0; i < count; ++i) {
        const int st = act_scale_check(descs[i].X_f16, descs[i].T, descs[i].K, descs[i].s);
        if (st != AWQ_OK) return st;
    }
    for (int first = 0; first < count; first += ACT_MAX) {
        ActProblem p[ACT_MAX];
        const int n = std::min(ACT_MAX, count - first);
        for (int i = 0; i < n; ++i)
            p[i] = {(const uint4 *)descs[first + i].X_f16, descs[first + i].s, descs[first + i].T, descs[first + i].K, 0, 0};
        const int st = act_scale_launch<false>(p, n, alpha, (hipStream_t)stream);
        if (st != AWQ_OK) return st;
    }
    return AWQ_OK;
}

// s_X itself: max(mean_t |X[t,k]|, 1e-4), the base of Eq. 5 (used by the scale search, which
// raises it to every alpha of its grid).  Arguments validated by the caller.
int awq_act_mean_launch(const void *X_f16, int64_t T, int64_t K, float *mean, hipStream_t stream)
{
    const ActProblem p = {(const uint4 *)X_f16, mean, T, K, 0, 0};
    return act_scale_launch<true>(&p, 1, 1.0f, stream);
}

extern "C" int awq_apply_inv_scale(const void *x_f16, const float *s, int64_t M, int64_t K,
                                   void *xs_f16, void *stream)
{
    if (!x_f16 || !s || !xs_f16) return AWQ_ERR_NULL_POINTER;
    if (M <= 0 || K <= 0 || (K % 8) != 0 || M * (K / 8) > (int64_t)1 << 38)
        return AWQ_ERR_BAD_SHAPE;
    if (!awq_aligned16(x_f16) || !awq_aligned16(s) || !awq_aligned16(xs_f16))
        return AWQ_ERR_MISALIGNED;
    const int64_t runs = M * (K / 8);
    const int64_t blocks = (runs + 255) / 256;
    if (blocks > 0x7fffffff) return AWQ_ERR_BAD_SHAPE;
    apply_inv_scale_kernel<<<dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream>>>(
        (const uint4 *)x_f16, (const float4 *)s, runs, K / 8, (uint4 *)xs_f16);
    return awq_launch_status();
}
