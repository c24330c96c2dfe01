// awq_search_scale for gfx950: the grid search for the activation-aware scale.
//
// AWQ Sec. 3.2, the search for the scale.  Eq. 4 asks for the per-input-channel scale s that
// minimises the output difference of one layer after quantization,
//     L(s) = || Q(W diag(s)) (diag(s)^-1 X) - W X ||,
// on calibration rows X cached for that layer; Eq. 5 restricts s to s_X^alpha (s_X = mean |X|
// per channel) and picks alpha on a grid over [0, 1].
//
// Every candidate is evaluated with the kernels that serve the layer afterwards, so the loss is
// the loss of the deployed arithmetic: quantize_pack(W, s_X^alpha) -> x' = X / s ->
// awq_w4a16_linear(x') -> sum of squared differences to the fp16 layer X W^T (one dense fp16
// MFMA product, computed once).  Sums of squares are kept in fp64 and reduced in a fixed order;
// the argmin and s* = s_X^alpha* are taken on the device, so the call neither synchronises nor
// copies to the host.
#include "awq_common.h"

int awq_act_mean_launch(const void *X_f16, int64_t T, int64_t K, float *mean, hipStream_t stream);

namespace {

constexpr int LOSS_BLOCKS = 1024;
constexpr int MAX_ALPHAS = 64;

struct AlphaList {
    float a[MAX_ALPHAS];
};

__global__ __launch_bounds__(256) void pow_kernel(const float *__restrict__ mean, float alpha, int K,
                                                  float *__restrict__ s)
{
    asm volatile("" ::"s"(mean), "s"(alpha), "s"(K), "s"(s));           // arguments in one round
    const int k = blockIdx.x * 256 + threadIdx.x;
    if (k < K) s[k] = powf(mean[k], alpha);
}

// Y[T,N] = X[T,K] W[N,K]^T, fp16 operands, fp32 accumulation, fp16 result: the unquantized layer
// of Eq. 4.  128 x 128 tile per workgroup, four waves of 64 x 64 (2 x 2 tiles of
// v_mfma_f32_32x32x16_f16), 64 columns of K per step staged through LDS (rows padded to 144
// bytes: the 16-byte fragment reads of 16 consecutive rows fall into 16 different bank groups),
// next step prefetched into registers.  It runs once per search, next to one quantized product
// per grid point.
constexpr int DT = 128;
constexpr int DROW = 144;

__global__ __launch_bounds__(256) void dense_gemm_kernel(const half_t *__restrict__ X,
                                                         const half_t *__restrict__ W,
                                                         half_t *__restrict__ Y, int T, int N, int K)
{
    __shared__ __align__(16) unsigned char lds[2 * DT * DROW];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, hi = lane >> 5;
    const int t0 = blockIdx.y * DT, n0 = blockIdx.x * DT;
    const int lrow = tid >> 3, lchunk = tid & 7;
    const uint4 *asrc[4], *bsrc[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        int ra = t0 + lrow + 32 * j;
        ra = ra < T ? ra : T - 1;                       // ragged edge: repeat the last row
        int rb = n0 + lrow + 32 * j;
        rb = rb < N ? rb : N - 1;
        asrc[j] = reinterpret_cast<const uint4 *>(X + (size_t)ra * K) + lchunk;
        bsrc[j] = reinterpret_cast<const uint4 *>(W + (size_t)rb * K) + lchunk;
    }
    uint4 pa[4], pb[4];
    floatx16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
    const int wm = wave >> 1, wn = wave & 1;
    const int steps = K / 64;
#pragma unroll
    for (int j = 0; j < 4; ++j) { pa[j] = asrc[j][0]; pb[j] = bsrc[j][0]; }
    for (int ks = 0; ks < steps; ++ks) {
        __syncthreads();                                 // everyone has read the previous step
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            *reinterpret_cast<uint4 *>(lds + (lrow + 32 * j) * DROW + lchunk * 16) = pa[j];
            *reinterpret_cast<uint4 *>(lds + (DT + lrow + 32 * j) * DROW + lchunk * 16) = pb[j];
        }
        __syncthreads();
        if (ks + 1 < steps) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                pa[j] = asrc[j][(size_t)(ks + 1) * 8];
                pb[j] = bsrc[j][(size_t)(ks + 1) * 8];
            }
        }
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            half8_t a[2], b[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                a[i] = *reinterpret_cast<const half8_t *>(lds + (64 * wm + 32 * i + l32) * DROW + (2 * s + hi) * 16);
                b[i] = *reinterpret_cast<const half8_t *>(lds + (DT + 64 * wn + 32 * i + l32) * DROW + (2 * s + hi) * 16);
            }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[i], b[j], acc[i][j], 0, 0, 0);
        }
    }
    // accumulator v of tile (i, j): row 8 (v/4) + 4 hi + v%4, column l32
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int col = n0 + 64 * wn + 32 * j + l32;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = t0 + 64 * wm + 32 * i + 8 * (v >> 2) + 4 * hi + (v & 3);
                if (row < T && col < N) Y[(size_t)row * N + col] = (half_t)acc[i][j][v];
            }
        }
}

// partial[b] = sum over the 16-byte chunks of workgroup b of (Yq - Y)^2: eight differences are
// squared and added in fp32, the chunk sums are added in fp64; the workgroup's 256 sums are
// folded in a fixed tree, so the result does not depend on timing.
__global__ __launch_bounds__(256) void loss_kernel(const uint4 *__restrict__ Yq,
                                                   const uint4 *__restrict__ Y, int64_t chunks,
                                                   double *__restrict__ partial)
{
    asm volatile("" ::"s"(Yq), "s"(Y), "s"(chunks), "s"(partial));     // arguments in one round
    __shared__ double red[256];
    double acc = 0.0;
    // four chunk pairs requested together (a chunk past the end re-reads the last one and is not
    // counted); the order of the additions is the order of the chunks either way
    const int64_t stride = (int64_t)LOSS_BLOCKS * 256;
    for (int64_t i0 = (int64_t)blockIdx.x * 256 + threadIdx.x; i0 < chunks; i0 += 4 * stride) {
        uint4 a[4], b[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int64_t i = i0 + u * stride, ic = i < chunks ? i : chunks - 1;
            a[u] = Yq[ic];
            b[u] = Y[ic];
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const half_t *ha = reinterpret_cast<const half_t *>(&a[u]);
            const half_t *hb = reinterpret_cast<const half_t *>(&b[u]);
            float c = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float d = (float)ha[e] - (float)hb[e];
                c += d * d;
            }
            if (i0 + u * stride < chunks) acc += (double)c;
        }
    }
    red[threadIdx.x] = acc;
    __syncthreads();
    for (int half = 128; half >= 1; half >>= 1) {
        if ((int)threadIdx.x < half) red[threadIdx.x] += red[threadIdx.x + half];
        __syncthreads();
    }
    if (threadIdx.x == 0) partial[blockIdx.x] = red[0];
}

// losses[i] = sum of the partial sums of grid point i (fixed tree); best = first index of the
// smallest loss (a loss that is not a number never wins); s_best = s_X^alpha[best].
__global__ __launch_bounds__(1024) void finalize_kernel(const double *__restrict__ partial, int n_alpha,
                                                        AlphaList alphas, const float *__restrict__ mean,
                                                        int K, double *__restrict__ losses,
                                                        int32_t *__restrict__ best, float *__restrict__ s_best)
{
    __shared__ double red[LOSS_BLOCKS];
    __shared__ double total[MAX_ALPHAS];
    __shared__ int chosen;
    const int tid = threadIdx.x;
    for (int i = 0; i < n_alpha; ++i) {
        red[tid] = partial[(size_t)i * LOSS_BLOCKS + tid];
        __syncthreads();
        for (int half = LOSS_BLOCKS / 2; half >= 1; half >>= 1) {
            if (tid < half) red[tid] += red[tid + half];
            __syncthreads();
        }
        if (tid == 0) total[i] = red[0];
        __syncthreads();
    }
    if (tid == 0) {
        int b = 0;
        double lb = total[0] == total[0] ? total[0] : __builtin_inf();
        for (int i = 1; i < n_alpha; ++i) {
            const double li = total[i] == total[i] ? total[i] : __builtin_inf();
            if (li < lb) { lb = li; b = i; }
        }
        chosen = b;
        *best = b;
    }
    if (tid < n_alpha) losses[tid] = total[tid];
    __syncthreads();
    const float alpha = alphas.a[chosen];
    for (int k = tid; k < K; k += 1024) s_best[k] = powf(mean[k], alpha);
}

struct SearchLayout {
    size_t mean, s, xs, q, sc, zp, y, yq, partial, total;
};

inline size_t up256(size_t v) { return (v + 255) & ~(size_t)255; }

SearchLayout search_layout(int64_t T, int64_t N, int64_t K, int n_alpha)
{
    SearchLayout L;
    const int64_t G = K / AWQ_GROUP;
    size_t o = 0;
    L.mean = o; o = up256(o + (size_t)K * 4);
    L.s = o; o = up256(o + (size_t)K * 4);
    L.xs = o; o = up256(o + (size_t)T * K * 2);
    L.q = o; o = up256(o + (size_t)N * K / 2);
    L.sc = o; o = up256(o + (size_t)N * G * 2);
    L.zp = o; o = up256(o + (size_t)N * G / 2);
    L.y = o; o = up256(o + (size_t)T * N * 2);
    L.yq = o; o = up256(o + (size_t)T * N * 2);
    L.partial = o; o = up256(o + (size_t)n_alpha * LOSS_BLOCKS * 8);
    L.total = o;
    return L;
}

int check_search_shape(int64_t T, int64_t N, int64_t K, int n_alpha, int group)
{
    int st = awq_check_weight_shape(N, K, group);
    if (st != AWQ_OK) return st;
    if (T <= 0 || T > (int64_t)1 << 22) return AWQ_ERR_BAD_SHAPE;
    if (n_alpha < 1 || n_alpha > MAX_ALPHAS) return AWQ_ERR_BAD_ARGUMENT;
    return AWQ_OK;
}

}  // namespace

extern "C" size_t awq_search_scale_workspace_bytes(int64_t T, int64_t N, int64_t K, int n_alpha,
                                                   int group)
{
    if (check_search_shape(T, N, K, n_alpha, group) != AWQ_OK) return 0;
    return search_layout(T, N, K, n_alpha).total;
}

extern "C" int awq_search_scale(const void *W_f16, const void *X_f16, int64_t T, int64_t N, int64_t K,
                                const float *alphas, int n_alpha, int group, void *workspace,
                                size_t workspace_bytes, double *losses, int32_t *best, float *s_best,
                                void *stream)
{
    if (!W_f16 || !X_f16 || !alphas || !workspace || !losses || !best || !s_best)
        return AWQ_ERR_NULL_POINTER;
    int st = check_search_shape(T, N, K, n_alpha, group);
    if (st != AWQ_OK) return st;
    AlphaList al = {};
    for (int i = 0; i < n_alpha; ++i) {
        if (!(alphas[i] >= 0.0f && alphas[i] <= 1.0f)) return AWQ_ERR_BAD_ARGUMENT;
        al.a[i] = alphas[i];
    }
    if (!awq_aligned16(W_f16) || !awq_aligned16(X_f16) || !awq_aligned16(s_best) ||
        (reinterpret_cast<uintptr_t>(workspace) & 255u) != 0 ||
        (reinterpret_cast<uintptr_t>(losses) & 7u) != 0 || (reinterpret_cast<uintptr_t>(best) & 3u) != 0)
        return AWQ_ERR_MISALIGNED;
    const SearchLayout L = search_layout(T, N, K, n_alpha);
    if (workspace_bytes < L.total) return AWQ_ERR_WORKSPACE_TOO_SMALL;
    unsigned char *ws = static_cast<unsigned char *>(workspace);
    float *mean = reinterpret_cast<float *>(ws + L.mean);
    float *s = reinterpret_cast<float *>(ws + L.s);
    void *xs = ws + L.xs, *q = ws + L.q, *sc = ws + L.sc, *zp = ws + L.zp;
    half_t *Y = reinterpret_cast<half_t *>(ws + L.y);
    half_t *Yq = reinterpret_cast<half_t *>(ws + L.yq);
    double *partial = reinterpret_cast<double *>(ws + L.partial);
    hipStream_t hs = (hipStream_t)stream;

    st = awq_act_mean_launch(X_f16, T, K, mean, hs);
    if (st != AWQ_OK) return st;
    {
        const dim3 grid((unsigned)((N + DT - 1) / DT), (unsigned)((T + DT - 1) / DT));
        dense_gemm_kernel<<<grid, dim3(256), 0, hs>>>((const half_t *)X_f16, (const half_t *)W_f16, Y,
                                                      (int)T, (int)N, (int)K);
        st = awq_launch_status();
        if (st != AWQ_OK) return st;
    }
    const int64_t chunks = T * N / 8;                    // N % 16 == 0
    for (int i = 0; i < n_alpha; ++i) {
        pow_kernel<<<dim3((unsigned)((K + 255) / 256)), dim3(256), 0, hs>>>(mean, al.a[i], (int)K, s);
        st = awq_launch_status();
        if (st != AWQ_OK) return st;
        st = awq_quantize_pack(W_f16, s, N, K, group, q, sc, zp, stream);
        if (st != AWQ_OK) return st;
        st = awq_apply_inv_scale(X_f16, s, T, K, xs, stream);
        if (st != AWQ_OK) return st;
        st = awq_w4a16_linear(xs, q, sc, zp, Yq, T, N, K, group, nullptr, 0, stream);
        if (st != AWQ_OK) return st;
        loss_kernel<<<dim3(LOSS_BLOCKS), dim3(256), 0, hs>>>((const uint4 *)Yq, (const uint4 *)Y, chunks,
                                                             partial + (size_t)i * LOSS_BLOCKS);
        st = awq_launch_status();
        if (st != AWQ_OK) return st;
    }
    finalize_kernel<<<dim3(1), dim3(1024), 0, hs>>>(partial, n_alpha, al, mean, (int)K, losses, best, s_best);
    return awq_launch_status();
}
