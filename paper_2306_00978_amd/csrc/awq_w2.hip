// INT2-g64 variant of the path for gfx950: quantize/pack, unpack and the decode kernel.
//
// AWQ Sec. 5 (the extreme low-bit table) quantizes to INT2 with group size 64.  The quantizer is
// the 4-level form of Sec. 3.2, Eq. 1-2, over groups of 64 input channels:
//   scale = fp16(clamp((max-min)/3, 2^-14, 65504)); zero = clamp(rint(-min/scale), 0, 3);
//   q = clamp(rint(w*s/scale) + zero, 0, 3),   binary32, one rounding per operation.
//
// Packed layout.  The unit is a block of 16 rows x 256 columns = four groups, 1 KB, so that a lane
// still fetches 16 bytes and a wave 1 KB of contiguous codes per load.  Lane l = (row l%16, column
// block c = l/16) owns, in word t of its 16-byte slot, the 16 codes of group t of the block:
// columns 64 t + 32 j + 8 c + e (j = 0..1, e = 0..7).  Code i = 8 j + e is member h = i%2 of pair
// p = i/2 and sits at bits [2p, 2p+2) of the low (h = 0) or high (h = 1) half of the word, so
// that (word >> 2p) & 0x00030003 is the pair as two fp16 SUBNORMALS q * 2^-24 -- the B-operand
// register of v_mfma_f32_16x16x32_f16 for columns (k, k+1), with no integer-to-float conversion.
// A row's four steps of a block are stored together (one 8-byte load per lane), its four zero
// points share a byte.
//
// Decode kernel (M <= 16): a workgroup owns one 16-row block of one linear, its waves split the
// K/256 blocks.  Per block a wave copies the 256-column slice of x it needs into its own LDS
// area (two rows per pass of 16-byte loads, no workgroup barrier), requests the next block's
// loads, and runs eight MFMA steps against the codes and eight against the constant code 1:
//   sum_k x_k (q_k - z) = 2^24 * (MFMA(x, q 2^-24) - z * MFMA(x, 2^-24)),  per group of 64,
// then applies the group's step in fp32.  Partial sums of the waves are combined through LDS in
// a fixed order.  Several linears (different shapes, same M) can share one launch.
//
// This file is compiled with -ffp-contract=off (integer decisions in the quantizer).
#include "awq_common.h"

namespace {

constexpr int W2_GROUP = AWQ_GROUP_W2;
constexpr int W2_BLOCK_COLS = 256;
constexpr int W2_MAX_PROBLEMS = 8;        // linears per launch

int check_shape_w2(int64_t N, int64_t K, int group)
{
    if (group != W2_GROUP) return AWQ_ERR_UNSUPPORTED_GROUP;
    if (N <= 0 || K <= 0 || (K % W2_BLOCK_COLS) != 0 || (N % AWQ_TILE_ROWS) != 0) return AWQ_ERR_BAD_SHAPE;
    if (N > (int64_t)1 << 24 || K > (int64_t)1 << 24 || (N / 16) * (K / 256) > (int64_t)1 << 30)
        return AWQ_ERR_BAD_SHAPE;
    return AWQ_OK;
}

__device__ __forceinline__ float clamp2(float v, float lo, float hi)
{
    if (v < lo) v = lo;
    if (v > hi) v = hi;
    return v;
}

// one wave per block of 16 rows x 256 columns
__global__ __launch_bounds__(256) void quantize_pack_w2_kernel(
    const uint4 *__restrict__ W, const float4 *__restrict__ s, uint4 *__restrict__ qweight,
    uint2 *__restrict__ scales, uint8_t *__restrict__ zeros, int B, int num_blocks)
{
    asm volatile("" ::"s"(W), "s"(s), "s"(qweight), "s"(scales), "s"(zeros), "s"(B), "s"(num_blocks));
    const int lane = threadIdx.x & 63;
    const int block = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (block >= num_blocks) return;               // whole wave leaves together
    const int rb = block / B, b = block - rb * B;
    const int r = lane & 15, c = lane >> 4;
    const int64_t K8 = (int64_t)B * 32;            // 16-byte runs per row
    const int64_t n = (int64_t)rb * 16 + r;

    uint4 raw[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) raw[i] = W[n * K8 + b * 32 + 4 * i + c];     // i = 2 t + j

    uint32_t words[4], zbyte = 0;
    uint16_t sc_bits[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        float wp[16];
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int run = b * 32 + 8 * t + 4 * j + c;
            const half_t *h = reinterpret_cast<const half_t *>(&raw[2 * t + j]);
            float sv[8] = {1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f};
            if (s) {
                const float4 a = s[2 * run], bb = s[2 * run + 1];
                sv[0] = a.x; sv[1] = a.y; sv[2] = a.z; sv[3] = a.w;
                sv[4] = bb.x; sv[5] = bb.y; sv[6] = bb.z; sv[7] = bb.w;
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) wp[8 * j + e] = (float)h[e] * sv[e];
        }
        float mx = wp[0], mn = wp[0];
#pragma unroll
        for (int i = 1; i < 16; ++i) {
            mx = fmaxf(mx, wp[i]);
            mn = fminf(mn, wp[i]);
        }
        mx = fmaxf(mx, __shfl_xor(mx, 16));
        mn = fminf(mn, __shfl_xor(mn, 16));
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        mn = fminf(mn, __shfl_xor(mn, 32));

        const float range = mx - mn;
        float sc32 = range / 3.0f;
        sc32 = clamp2(sc32, 6.103515625e-05f, 65504.0f);
        const half_t sc_h = (half_t)sc32;
        const float scale = (float)sc_h;
        const float nmn = -mn;
        const float zr = nmn / scale;
        const float zero = clamp2(__builtin_rintf(zr), 0.0f, 3.0f);

        uint32_t word = 0;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            float v = __builtin_rintf(wp[i] / scale);
            v = v + zero;
            v = clamp2(v, 0.0f, 3.0f);
            word |= (uint32_t)v << (16 * (i % 2) + 2 * (i / 2));
        }
        words[t] = word;
        sc_bits[t] = __builtin_bit_cast(uint16_t, sc_h);
        zbyte |= (uint32_t)zero << (2 * t);
    }
    qweight[(int64_t)block * 64 + lane] = make_uint4(words[0], words[1], words[2], words[3]);
    if (c == 0) {
        scales[(int64_t)block * 16 + r] = make_uint2((uint32_t)sc_bits[0] | ((uint32_t)sc_bits[1] << 16),
                                                     (uint32_t)sc_bits[2] | ((uint32_t)sc_bits[3] << 16));
        zeros[(int64_t)block * 16 + r] = (uint8_t)zbyte;
    }
}

// the eight codes (four subnormal fp16 pairs) of MFMA step j (0..1) of a group's word
__device__ __forceinline__ uint4 w2_fragment(uint32_t w, int j)
{
    const uint32_t v = w >> (8 * j);
    return make_uint4(v & 0x00030003u, (v >> 2) & 0x00030003u, (v >> 4) & 0x00030003u, (v >> 6) & 0x00030003u);
}

__global__ __launch_bounds__(256) void unpack_w2_kernel(
    const uint4 *__restrict__ qweight, const uint16_t *__restrict__ scales,
    const uint8_t *__restrict__ zeros, uint8_t *__restrict__ codes,
    uint16_t *__restrict__ scales_out, uint8_t *__restrict__ zeros_out, int B, int num_blocks)
{
    const int lane = threadIdx.x & 63;
    const int block = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (block >= num_blocks) return;
    const int rb = block / B, b = block - rb * B;
    const int r = lane & 15, c = lane >> 4;
    const int64_t n = (int64_t)rb * 16 + r;
    const int64_t K = (int64_t)B * 256, G = (int64_t)B * 4;
    if (codes) {
        const uint4 q = qweight[(int64_t)block * 64 + lane];
        const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const uint4 f = w2_fragment(w[t], j);
                const uint32_t pr[4] = {f.x, f.y, f.z, f.w};
                uint32_t lo = 0, hi = 0;               // bytes e = 0..3 and 4..7
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const uint32_t two = (pr[i] & 0xFFu) | ((pr[i] >> 16) << 8);     // codes 2i, 2i+1
                    if (i < 2) lo |= two << (16 * i);
                    else hi |= two << (16 * (i - 2));
                }
                uint2 *dst = reinterpret_cast<uint2 *>(codes + n * K + b * 256 + 64 * t + 32 * j + 8 * c);
                *dst = make_uint2(lo, hi);
            }
    }
    // lane (r, c) takes group c of the block
    if (scales_out) scales_out[n * G + 4 * b + c] = scales[((int64_t)block * 16 + r) * 4 + c];
    if (zeros_out) zeros_out[n * G + 4 * b + c] = (zeros[(int64_t)block * 16 + r] >> (2 * c)) & 0x3;
}

struct W2Problem {
    const half_t *x;
    const uint4 *q;
    const uint2 *sc;
    const uint8_t *zp;
    half_t *y;
    int N, K;
};

struct W2Args {
    W2Problem p[W2_MAX_PROBLEMS];
    int wg_begin[W2_MAX_PROBLEMS];     // first workgroup of each problem (wg_begin[0] = 0)
    int count, M, logW;
};

// MS = rows of x a wave stages per block (M <= MS, one of 1, 2, 4, 8, 16); rows >= M repeat row
// M-1 (row m of the MFMA result depends on row m of A only, and rows >= M are never stored).
// Dynamic LDS: [W][MS rows x 528 bytes], then 16*M outputs x 16 wave slots of fp32.
template <int MS>
__global__ __launch_bounds__(1024) void gemv_w2_kernel(const W2Args a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    constexpr int NS = (MS + 1) / 2;               // 32 lanes x 16 B cover one row: two rows per pass
    constexpr int ROW_BYTES = 512 + 16;            // +16: rows land on different banks
    constexpr int WAVE_BYTES = MS * ROW_BYTES;
    // the linear this workgroup works on: scalar selects over the argument table
    W2Problem P = a.p[0];
    int first = 0;
#pragma unroll
    for (int i = 1; i < W2_MAX_PROBLEMS; ++i)
        if (i < a.count && (int)blockIdx.x >= a.wg_begin[i]) {
            P = a.p[i];
            first = a.wg_begin[i];
        }
    const int M = a.M, logW = a.logW;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int W = 1 << logW;
    const int rb = blockIdx.x - first;
    const int r = lane & 15, c = lane >> 4;
    const int K = P.K, N = P.N;
    const int B = K >> 8;
    const int b0 = (B * wave) >> logW, b1 = (B * (wave + 1)) >> logW;

    const uint4 *qt = P.q + (int64_t)rb * B * 64 + lane;
    const uint2 *sc = P.sc + (int64_t)rb * B * 16 + r;
    const uint8_t *zp = P.zp + (int64_t)rb * B * 16 + r;
    const int mrow = r < M ? r : M - 1;
    unsigned char *xw = smem + (size_t)wave * WAVE_BYTES;
    const uint4 *xl = reinterpret_cast<const uint4 *>(xw + mrow * ROW_BYTES) + c;
    const int srow = lane >> 5, schunk = lane & 31;
    const uint4 *xstage = reinterpret_cast<const uint4 *>(P.x) + schunk;
    const int64_t K8 = (int64_t)K >> 3;

    // One block as loaded from global memory: the staging rows of x (requested first, so that
    // they return first), the row's four steps and zero points, the codes.
    uint4 xs[NS], q_cur;
    uint2 s_cur;
    uint32_t z_cur;
#pragma unroll
    for (int i = 0; i < NS; ++i) xs[i] = make_uint4(0, 0, 0, 0);
    q_cur = make_uint4(0, 0, 0, 0);
    s_cur = make_uint2(0, 0);
    z_cur = 0;
    if (b0 < b1) {
#pragma unroll
        for (int i = 0; i < NS; ++i) {
            const int m = 2 * i + srow;
            xs[i] = xstage[(int64_t)(m < M ? m : M - 1) * K8 + b0 * 32];
        }
        s_cur = sc[b0 * 16];
        z_cur = zp[b0 * 16];
        q_cur = qt[b0 * 64];
    }
    const half8_t ones = __builtin_bit_cast(half8_t, make_uint4(0x00010001u, 0x00010001u, 0x00010001u, 0x00010001u));
    floatx4 total = {0.f, 0.f, 0.f, 0.f};
    for (int b = b0; b < b1; ++b) {
        // LDS operations of one wave execute in order: these stores follow the previous block's reads
#pragma unroll
        for (int i = 0; i < NS; ++i) {
            const int m = 2 * i + srow;
            if (m < MS) reinterpret_cast<uint4 *>(xw + m * ROW_BYTES)[schunk] = xs[i];
        }
        const uint32_t w[4] = {q_cur.x, q_cur.y, q_cur.z, q_cur.w};
        const uint32_t sraw[4] = {s_cur.x & 0xFFFFu, s_cur.x >> 16, s_cur.y & 0xFFFFu, s_cur.y >> 16};
        const uint32_t z = z_cur;
        // the next block is requested before this one is consumed (the last block of a wave
        // requests itself again: an unconditional load from an address that is in bounds)
        const int bn = b + 1 < b1 ? b + 1 : b;
#pragma unroll
        for (int i = 0; i < NS; ++i) {
            const int m = 2 * i + srow;
            xs[i] = xstage[(int64_t)(m < M ? m : M - 1) * K8 + bn * 32];
        }
        s_cur = sc[bn * 16];
        z_cur = zp[bn * 16];
        q_cur = qt[bn * 64];
        uint4 xa[8];
#pragma unroll
        for (int jj = 0; jj < 8; ++jj) xa[jj] = xl[4 * jj];      // k = 32 jj + 8 c + 0..7
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            floatx4 acc = {0.f, 0.f, 0.f, 0.f}, xsum = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const half8_t av = __builtin_bit_cast(half8_t, xa[2 * t + j]);
                const half8_t bv = __builtin_bit_cast(half8_t, w2_fragment(w[t], j));
                acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(av, bv, acc, 0, 0, 0);
                xsum = __builtin_amdgcn_mfma_f32_16x16x32_f16(av, ones, xsum, 0, 0, 0);
            }
            const float zf = (float)((z >> (2 * t)) & 3u);
            const float s24 = (float)__builtin_bit_cast(half_t, (uint16_t)sraw[t]) * 16777216.f;
#pragma unroll
            for (int v = 0; v < 4; ++v) total[v] += s24 * (acc[v] - zf * xsum[v]);
        }
    }

    // lane holds the partial y[m = 4c + v][n = 16 rb + r]; combine the waves in fixed order.
    // red[t][w], t = 16 m + n: the 16 partials of one output are contiguous.
    float *red = reinterpret_cast<float *>(smem + (size_t)W * WAVE_BYTES);
    if (4 * c < M) {
#pragma unroll
        for (int v = 0; v < 4; ++v) red[((4 * c + v) * 16 + r) * 16 + wave] = total[v];
    }
    __syncthreads();
    for (int t = threadIdx.x; t < 16 * M; t += blockDim.x) {
        const float4 *p = reinterpret_cast<const float4 *>(red + t * 16);
        const float4 a0 = p[0], a1 = p[1], a2 = p[2], a3 = p[3];
        const float part[16] = {a0.x, a0.y, a0.z, a0.w, a1.x, a1.y, a1.z, a1.w,
                                a2.x, a2.y, a2.z, a2.w, a3.x, a3.y, a3.z, a3.w};
        float sum = 0.f;
#pragma unroll
        for (int w2 = 0; w2 < 16; ++w2) sum += (w2 < W) ? part[w2] : 0.f;
        P.y[(int64_t)(t >> 4) * N + rb * 16 + (t & 15)] = (half_t)sum;
    }
}

template <int MS>
int launch_w2_one(const W2Args &a, int total_wgs, size_t lds, hipStream_t stream)
{
    static AwqOncePerDevice once;
    bool &raised = once.here();
    if (lds > 64 * 1024 && !raised) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(gemv_w2_kernel<MS>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess)
            return AWQ_ERR_HIP;
        raised = true;
    }
    gemv_w2_kernel<MS><<<dim3(total_wgs), dim3(64 << a.logW), lds, stream>>>(a);
    return awq_launch_status();
}

// up to W2_MAX_PROBLEMS validated linears in one launch; the ones with the longest rows first
// (their workgroups run longest, so they should not start last)
int launch_w2(const W2Problem *probs, int count, int M, hipStream_t stream)
{
    W2Args a = {};
    int order[W2_MAX_PROBLEMS];
    for (int i = 0; i < count; ++i) order[i] = i;
    for (int i = 1; i < count; ++i)                       // insertion sort, stable, K descending
        for (int j = i; j > 0 && probs[order[j]].K > probs[order[j - 1]].K; --j) {
            const int t = order[j];
            order[j] = order[j - 1];
            order[j - 1] = t;
        }
    int total = 0, maxB = 0;
    for (int i = 0; i < count; ++i) {
        a.p[i] = probs[order[i]];
        a.wg_begin[i] = total;
        total += a.p[i].N / 16;
        if (a.p[i].K / 256 > maxB) maxB = a.p[i].K / 256;
    }
    a.count = count;
    a.M = M;
    const int MS = M == 1 ? 1 : (M == 2 ? 2 : (M <= 4 ? 4 : (M <= 8 ? 8 : 16)));
    // about two blocks per wave, 1..16 waves; 16 rows x 16 waves of staging would leave no LDS
    int logW = maxB >= 32 ? 4 : (maxB >= 16 ? 3 : (maxB >= 8 ? 2 : (maxB >= 4 ? 1 : 0)));
    if (MS == 16 && logW > 3) logW = 3;
    a.logW = logW;
    const size_t lds = (size_t)((M + 3) / 4 * 4) * 1024 + (size_t)(1 << logW) * MS * 528;
    if (lds > (size_t)160 * 1024) return AWQ_ERR_BAD_SHAPE;
    switch (MS) {
    case 1: return launch_w2_one<1>(a, total, lds, stream);
    case 2: return launch_w2_one<2>(a, total, lds, stream);
    case 4: return launch_w2_one<4>(a, total, lds, stream);
    case 8: return launch_w2_one<8>(a, total, lds, stream);
    default: return launch_w2_one<16>(a, total, lds, stream);
    }
}

int fill_problem(W2Problem &p, const void *x, const void *q, const void *sc, const void *zp, void *y,
                 int64_t N, int64_t K, int group)
{
    if (!x || !q || !sc || !zp || !y) return AWQ_ERR_NULL_POINTER;
    int st = check_shape_w2(N, K, group);
    if (st != AWQ_OK) return st;
    if (!awq_aligned16(x) || !awq_aligned16(q) || !awq_aligned16(sc) || !awq_aligned16(zp) || !awq_aligned16(y))
        return AWQ_ERR_MISALIGNED;
    p.x = (const half_t *)x;
    p.q = (const uint4 *)q;
    p.sc = (const uint2 *)sc;
    p.zp = (const uint8_t *)zp;
    p.y = (half_t *)y;
    p.N = (int)N;
    p.K = (int)K;
    return AWQ_OK;
}

}  // namespace

extern "C" int awq_packed_sizes_w2(int64_t N, int64_t K, int group, size_t *qweight_bytes,
                                   size_t *scales_bytes, size_t *zeros_bytes)
{
    int st = check_shape_w2(N, K, group);
    if (st != AWQ_OK) return st;
    const int64_t G = K / W2_GROUP;
    if (qweight_bytes) *qweight_bytes = (size_t)(N * K / 4);
    if (scales_bytes) *scales_bytes = (size_t)(N * G * 2);
    if (zeros_bytes) *zeros_bytes = (size_t)(N * G / 4);
    return AWQ_OK;
}

extern "C" int awq_quantize_pack_w2(const void *W_f16, const float *s, int64_t N, int64_t K,
                                    int group, void *qweight, void *scales, void *zeros,
                                    void *stream)
{
    if (!W_f16 || !qweight || !scales || !zeros) return AWQ_ERR_NULL_POINTER;
    int st = check_shape_w2(N, K, group);
    if (st != AWQ_OK) return st;
    if (!awq_aligned16(W_f16) || !awq_aligned16(qweight) || !awq_aligned16(scales) ||
        !awq_aligned16(zeros) || (s && !awq_aligned16(s)))
        return AWQ_ERR_MISALIGNED;
    const int B = (int)(K / W2_BLOCK_COLS);
    const int num_blocks = (int)(N / 16) * B;
    quantize_pack_w2_kernel<<<dim3((num_blocks + 3) / 4), dim3(256), 0, (hipStream_t)stream>>>(
        (const uint4 *)W_f16, (const float4 *)s, (uint4 *)qweight, (uint2 *)scales, (uint8_t *)zeros, B,
        num_blocks);
    return awq_launch_status();
}

extern "C" int awq_unpack_w2(const void *qweight, const void *scales, const void *zeros,
                             int64_t N, int64_t K, int group, uint8_t *codes, void *scales_f16,
                             uint8_t *zeros_u8, void *stream)
{
    if (!qweight || !scales || !zeros) return AWQ_ERR_NULL_POINTER;
    int st = check_shape_w2(N, K, group);
    if (st != AWQ_OK) return st;
    if (!awq_aligned16(qweight) || !awq_aligned16(scales) || !awq_aligned16(zeros) ||
        (codes && !awq_aligned16(codes)) || (scales_f16 && !awq_aligned16(scales_f16)) ||
        (zeros_u8 && !awq_aligned16(zeros_u8)))
        return AWQ_ERR_MISALIGNED;
    const int B = (int)(K / W2_BLOCK_COLS);
    const int num_blocks = (int)(N / 16) * B;
    unpack_w2_kernel<<<dim3((num_blocks + 3) / 4), dim3(256), 0, (hipStream_t)stream>>>(
        (const uint4 *)qweight, (const uint16_t *)scales, (const uint8_t *)zeros, codes,
        (uint16_t *)scales_f16, zeros_u8, B, num_blocks);
    return awq_launch_status();
}

extern "C" int awq_w2a16_linear(const void *x_f16, const void *qweight, const void *scales,
                                const void *zeros, void *y_f16, int64_t M, int64_t N, int64_t K,
                                int group, void *stream)
{
    W2Problem p;
    int st = fill_problem(p, x_f16, qweight, scales, zeros, y_f16, N, K, group);
    if (st != AWQ_OK) return st;
    if (M <= 0 || M > 128) return AWQ_ERR_BAD_SHAPE;
    if (M <= 16) return launch_w2(&p, 1, (int)M, (hipStream_t)stream);
    // a few dozen tokens: blocks of 16 rows through the decode kernel, eight blocks per launch; the
    // last block is moved back to end at row M (its overlap is computed twice, same values)
    const int blocks = (int)((M + 15) / 16);
    W2Problem d[W2_MAX_PROBLEMS];
    for (int b = 0; b < blocks; ++b) {
        const int64_t m0 = b + 1 < blocks ? 16 * (int64_t)b : M - 16;
        d[b] = p;
        d[b].x = p.x + m0 * K;
        d[b].y = p.y + m0 * N;
    }
    return launch_w2(d, blocks, 16, (hipStream_t)stream);
}

extern "C" int awq_w2a16_linear_multi(const awq_linear_desc *descs, int count, int64_t M, int group,
                                      void *stream)
{
    if (!descs) return AWQ_ERR_NULL_POINTER;
    if (count < 1 || count > AWQ_MULTI_MAX) return AWQ_ERR_BAD_ARGUMENT;
    if (M <= 0 || M > 16) return AWQ_ERR_BAD_SHAPE;
    W2Problem p[AWQ_MULTI_MAX];
    for (int i = 0; i < count; ++i) {
        const awq_linear_desc &d = descs[i];
        int st = fill_problem(p[i], d.x_f16, d.qweight, d.scales, d.zeros, d.y_f16, d.N, d.K, group);
        if (st != AWQ_OK) return st;
    }
    for (int i = 0; i < count; i += W2_MAX_PROBLEMS) {
        const int n = count - i < W2_MAX_PROBLEMS ? count - i : W2_MAX_PROBLEMS;
        int st = launch_w2(p + i, n, (int)M, (hipStream_t)stream);
        if (st != AWQ_OK) return st;
    }
    return AWQ_OK;
}
