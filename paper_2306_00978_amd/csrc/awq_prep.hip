// awq_act_scale / awq_apply_inv_scale for gfx950.
//
// AWQ Sec. 3.2: the saliency of a weight channel is decided by the magnitude of
// its input activation; Eq. 5 takes s = s_X^alpha with s_X the per-input-channel
// mean |X| over the calibration rows, and Eq. 4 moves diag(s)^-1 onto the
// activations.  Both are plain streaming passes over X (HBM-bound).
#include "awq_common.h"

namespace {

// A workgroup (1024 threads) owns COLS columns and walks all T rows; thread (phase, oct) sums |x|
// of rows phase, phase + PHASES, ... for its eight columns (PHASES = 1024 / (COLS / 8)).  The
// PHASES partial sums per column are then added in a fixed tree order, so the result is
// deterministic.  RAW: store the (floored) mean itself instead of its power.
// COLS: 64 columns (128 B per row) give K / 64 workgroups: 172 for K = 11008 (5.2 TB/s at 65 536
// rows) but only 64 for K = 4096, a quarter of the chip (2.1 TB/s).  Below K = 8192 a workgroup
// therefore takes 16 columns (2.5 TB/s for K = 4096; 32 columns: 2.4); so that a 128-byte line is
// still fetched from memory once, the workgroups are numbered so that each XCD (own L2;
// workgroups go to the XCDs round-robin by their id) gets a contiguous range of column blocks:
// the workgroups that share a line sit on one XCD and start one after the other.  For wide K
// the narrow blocks are slower (K = 11008: 3.2 TB/s).  More loads in flight per thread than eight change nothing: a CU
// alone takes in about 33 GB/s.  Splitting the rows over workgroups would need a place for partial
// sums, which the call does not have.
template <bool RAW, int COLS>
__global__ __launch_bounds__(1024) void act_scale_kernel(const uint4 *__restrict__ X,
                                                         int64_t T, int64_t K, float alpha,
                                                         float *__restrict__ s, int nblocks)
{
    constexpr int OCTS = COLS / 8, PHASES = 1024 / OCTS;
    // all arguments fetched in one round (otherwise one scalar-cache miss per first use)
    asm volatile("" ::"s"(X), "s"(T), "s"(K), "s"(alpha), "s"(s), "s"(nblocks));
    __shared__ float red[PHASES][COLS];
    const int per_xcd = (nblocks + 7) >> 3;
    const int cb = ((int)blockIdx.x & 7) * per_xcd + ((int)blockIdx.x >> 3);
    if (cb >= nblocks) return;
    const int oct = threadIdx.x % OCTS;
    const int phase = threadIdx.x / OCTS;
    const int64_t col0 = (int64_t)cb * COLS + oct * 8;
    float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    if (col0 < K) {
        const int64_t K8 = K / 8;
        const uint4 *p = X + col0 / 8;
        // eight rows requested before the first is added (the requests in flight per thread decide
        // the rate of a CU); the additions keep the order of the rows
        constexpr int AHEAD = 8;
        int64_t t = phase;
        for (; t + (AHEAD - 1) * PHASES < T; t += AHEAD * PHASES) {
            uint4 raw[AHEAD];
#pragma unroll
            for (int a = 0; a < AHEAD; ++a) raw[a] = p[(t + a * PHASES) * K8];
#pragma unroll
            for (int a = 0; a < AHEAD; ++a) {
                const half_t *h = reinterpret_cast<const half_t *>(&raw[a]);
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[e] += __builtin_fabsf((float)h[e]);
            }
        }
        for (; t < T; t += PHASES) {
            uint4 raw = p[t * K8];
            const half_t *h = reinterpret_cast<const half_t *>(&raw);
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[e] += __builtin_fabsf((float)h[e]);
        }
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) red[phase][oct * 8 + e] = acc[e];
    __syncthreads();
    for (int half = PHASES / 2; half >= 1; half >>= 1) {
        for (int i = threadIdx.x; i < half * COLS; i += 1024) {
            const int p = i / COLS, cidx = i % COLS;
            red[p][cidx] += red[p + half][cidx];
        }
        __syncthreads();
    }
    if (threadIdx.x < COLS) {
        const int64_t col = (int64_t)cb * COLS + threadIdx.x;
        if (col < K) {
            float mean = red[0][threadIdx.x] / (float)T;
            mean = fmaxf(mean, 1e-4f);
            s[col] = RAW ? mean : powf(mean, alpha);
        }
    }
}

// Column-block width by K (the same for the plain and the RAW form, whose results must agree bit
// for bit).
template <bool RAW>
int act_scale_launch(const void *X_f16, int64_t T, int64_t K, float alpha, float *s, hipStream_t stream)
{
    const int cols = K >= 8192 ? 64 : 16;
    const int nblocks = (int)((K + cols - 1) / cols);
    const dim3 grid(8 * ((nblocks + 7) / 8)), block(1024);
    const uint4 *X = (const uint4 *)X_f16;
    if (cols == 64) act_scale_kernel<RAW, 64><<<grid, block, 0, stream>>>(X, T, K, alpha, s, nblocks);
    else act_scale_kernel<RAW, 16><<<grid, block, 0, stream>>>(X, T, K, alpha, s, nblocks);
    return awq_launch_status();
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
    if (!X_f16 || !s) return AWQ_ERR_NULL_POINTER;
    if (T <= 0 || K <= 0 || (K % 8) != 0 || K > (int64_t)1 << 30) return AWQ_ERR_BAD_SHAPE;
    if (!(alpha >= 0.0f && alpha <= 1.0f)) return AWQ_ERR_BAD_ARGUMENT;
    if (!awq_aligned16(X_f16) || !awq_aligned16(s)) return AWQ_ERR_MISALIGNED;
    return act_scale_launch<false>(X_f16, T, K, alpha, s, (hipStream_t)stream);
}

// s_X itself: max(mean_t |X[t,k]|, 1e-4), the base of Eq. 5 (used by the scale search, which
// raises it to every alpha of its grid).  Arguments validated by the caller.
int awq_act_mean_launch(const void *X_f16, int64_t T, int64_t K, float *mean, hipStream_t stream)
{
    return act_scale_launch<true>(X_f16, T, K, 1.0f, mean, stream);
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
