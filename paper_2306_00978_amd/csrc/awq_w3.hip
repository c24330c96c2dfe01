// INT3-g128 variant of the path for gfx950: quantize/pack, unpack and the decode kernel.
//
// AWQ Sec. 5 studies INT4 and INT3 with group size 128 (its ablation table uses INT3-g128).
// The quantizer is the 8-level form of Sec. 3.2, Eq. 1-2:
//   scale = fp16(clamp((max-min)/7, 2^-14, 65504)); zero = clamp(rint(-min/scale), 0, 7);
//   q = clamp(rint(w*s/scale) + zero, 0, 7),   binary32, one rounding per operation.
//
// Packed layout.  Three bits do not divide a 128-bit load; the unit here is 96 bits.  A tile is
// still 16 rows x 128 columns (768 B) and lane l = (row l%16, column block c = l/16) still owns
// the 32 codes of columns 32 j + 8 c + e, now as three 32-bit words (a 12-byte slot, one
// global_load_dwordx3 per lane, 768 contiguous bytes per wave).  Code i = 8 j + e is member
// h = i%2 of pair p = i/2; pairs 0..14 sit in word p/5 at bits [3f, 3f+3), f = p%5, of the low
// (h = 0) or high (h = 1) half, so that (word >> 3f) & 0x00070007 is the pair as two fp16
// SUBNORMALS q * 2^-24 -- the B-operand register of v_mfma_f32_16x16x32_f16 for columns
// (k, k+1), with no integer-to-float conversion.  Pair 15 is spread over the spare top bits of
// the six halves.  Steps and zero points are stored as in the 4-bit layout.
//
// The decode kernel (M <= 16) is the BITS = 3 form of the batch decode kernel of the 4-bit path.
//
// This file is compiled with -ffp-contract=off (integer decisions in the quantizer).
#include "awq_common.h"
#include "awq_gemv_stream.h"

int awq_gemv_launch_w3(const void *x, const void *qweight, const void *scales, const void *zeros,
                       void *y, int M, int N, int K, hipStream_t stream);

namespace {

__device__ __forceinline__ float clamp3(float v, float lo, float hi)
{
    if (v < lo) v = lo;
    if (v > hi) v = hi;
    return v;
}

// one wave per tile
__global__ __launch_bounds__(256) void quantize_pack_w3_kernel(
    const uint4 *__restrict__ W, const float4 *__restrict__ s, uint32_t *__restrict__ qweight,
    uint16_t *__restrict__ scales, uint8_t *__restrict__ zeros, int G, int num_tiles)
{
    const int lane = threadIdx.x & 63;
    const int tile = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (tile >= num_tiles) return;                 // whole wave leaves together
    const int rb = tile / G, g = tile - rb * G;
    const int r = lane & 15, c = lane >> 4;
    const int64_t K8 = (int64_t)G * 16;
    const int64_t n = (int64_t)rb * 16 + r;

    float wp[32];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int run = g * 16 + 4 * j + c;
        const uint4 raw = W[n * K8 + run];
        const half_t *h = reinterpret_cast<const half_t *>(&raw);
        float sv[8] = {1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f};
        if (s) {
            const float4 a = s[2 * run], b = s[2 * run + 1];
            sv[0] = a.x; sv[1] = a.y; sv[2] = a.z; sv[3] = a.w;
            sv[4] = b.x; sv[5] = b.y; sv[6] = b.z; sv[7] = b.w;
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) wp[8 * j + e] = (float)h[e] * sv[e];
    }
    float mx = wp[0], mn = wp[0];
#pragma unroll
    for (int i = 1; i < 32; ++i) {
        mx = fmaxf(mx, wp[i]);
        mn = fminf(mn, wp[i]);
    }
    mx = fmaxf(mx, __shfl_xor(mx, 16));
    mn = fminf(mn, __shfl_xor(mn, 16));
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    mn = fminf(mn, __shfl_xor(mn, 32));

    const float range = mx - mn;
    float sc32 = range / 7.0f;
    sc32 = clamp3(sc32, 6.103515625e-05f, 65504.0f);
    const half_t sc_h = (half_t)sc32;
    const float scale = (float)sc_h;
    const float nmn = -mn;
    const float zr = nmn / scale;
    const float zero = clamp3(__builtin_rintf(zr), 0.0f, 7.0f);

    uint32_t q[32];
#pragma unroll
    for (int i = 0; i < 32; ++i) {
        float v = __builtin_rintf(wp[i] / scale);
        v = v + zero;
        v = clamp3(v, 0.0f, 7.0f);
        q[i] = (uint32_t)v;
    }
    uint32_t words[3] = {0u, 0u, 0u};
#pragma unroll
    for (int p = 0; p < 15; ++p)
        words[p / 5] |= (q[2 * p] << (3 * (p % 5))) | (q[2 * p + 1] << (16 + 3 * (p % 5)));
#pragma unroll
    for (int b = 0; b < 3; ++b)
        words[b] |= (((q[30] >> b) & 1u) << 15) | (((q[31] >> b) & 1u) << 31);
    uint32_t *dst = qweight + (int64_t)tile * 192 + lane * 3;
    dst[0] = words[0];
    dst[1] = words[1];
    dst[2] = words[2];

    const uint32_t z = (uint32_t)zero;
    const uint32_t z_hi = __shfl_xor(z, 1);
    if (c == 0) {
        scales[(int64_t)tile * 16 + r] = __builtin_bit_cast(uint16_t, sc_h);
        if ((r & 1) == 0) zeros[(int64_t)tile * 8 + (r >> 1)] = (uint8_t)(z | (z_hi << 4));
    }
}

// the eight codes (as four subnormal fp16 pairs) of MFMA step j from the three words of a slot
__device__ __forceinline__ uint4 w3_fragment(const uint32_t (&w)[3], uint32_t last_pair, int j)
{
    uint32_t t[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int p = 4 * j + i;
        t[i] = p < 15 ? ((w[p / 5] >> (3 * (p % 5))) & 0x00070007u) : last_pair;
    }
    return make_uint4(t[0], t[1], t[2], t[3]);
}

// pair 15 from the top bits of the six halves
__device__ __forceinline__ uint32_t w3_last_pair(const uint32_t (&w)[3])
{
    return ((w[0] >> 15) & 0x00010001u) | ((w[1] >> 14) & 0x00020002u) | ((w[2] >> 13) & 0x00040004u);
}

__global__ __launch_bounds__(256) void unpack_w3_kernel(
    const uint32_t *__restrict__ qweight, const uint16_t *__restrict__ scales,
    const uint8_t *__restrict__ zeros, uint8_t *__restrict__ codes,
    uint16_t *__restrict__ scales_out, uint8_t *__restrict__ zeros_out, int G, int num_tiles)
{
    const int lane = threadIdx.x & 63;
    const int tile = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (tile >= num_tiles) return;
    const int rb = tile / G, g = tile - rb * G;
    const int r = lane & 15, c = lane >> 4;
    const int64_t n = (int64_t)rb * 16 + r;
    const int64_t K = (int64_t)G * 128;
    if (codes) {
        const uint32_t *src = qweight + (int64_t)tile * 192 + lane * 3;
        const uint32_t w[3] = {src[0], src[1], src[2]};
        const uint32_t last = w3_last_pair(w);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint4 f = w3_fragment(w, last, j);
            const uint32_t pr[4] = {f.x, f.y, f.z, f.w};
            uint32_t lo = 0, hi = 0;               // bytes e = 0..3 and 4..7
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint32_t two = (pr[i] & 0xFFu) | ((pr[i] >> 16) << 8);     // codes 2i, 2i+1
                if (i < 2) lo |= two << (16 * i);
                else hi |= two << (16 * (i - 2));
            }
            uint2 *dst = reinterpret_cast<uint2 *>(codes + n * K + g * 128 + 32 * j + 8 * c);
            *dst = make_uint2(lo, hi);
        }
    }
    if (c == 0) {
        if (scales_out) scales_out[n * G + g] = scales[(int64_t)tile * 16 + r];
        if (zeros_out)
            zeros_out[n * G + g] = (zeros[(int64_t)tile * 8 + (r >> 1)] >> (4 * (r & 1))) & 0xF;
    }
}

// 3-bit slots -> 4-bit slots of the same tile: lane l owns the same 32 codes in both layouts, and
// a pair read as (q, q') in the two halves goes to nibble i of both halves of word j
__global__ __launch_bounds__(256) void repack_w3_to_w4_kernel(const uint32_t *__restrict__ q3,
                                                              uint4 *__restrict__ q4, int num_tiles)
{
    const int lane = threadIdx.x & 63;
    const int tile = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (tile >= num_tiles) return;
    const uint32_t *src = q3 + (int64_t)tile * 192 + lane * 3;
    const uint32_t w[3] = {src[0], src[1], src[2]};
    const uint32_t last = w3_last_pair(w);
    uint32_t out[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const uint4 f = w3_fragment(w, last, j);
        out[j] = f.x | (f.y << 4) | (f.z << 8) | (f.w << 12);
    }
    q4[(int64_t)tile * 64 + lane] = make_uint4(out[0], out[1], out[2], out[3]);
}

}  // namespace

int awq_gemm_launch(const void *x, const void *qweight, const void *scales, const void *zeros,
                    void *y, int M, int N, int K, hipStream_t stream);
int awq_gemm_launch_split(const void *x, const void *qweight, const void *scales, const void *zeros,
                          void *y, int M, int N, int K, void *part, int ksplit, hipStream_t stream);
int awq_gemm_ksplit(int M, int N, int K, double *estimate_us);

extern "C" int awq_repack_w3_to_w4(const void *qweight_w3, int64_t N, int64_t K, int group,
                                   void *qweight_w4, void *stream)
{
    if (!qweight_w3 || !qweight_w4) return AWQ_ERR_NULL_POINTER;
    int st = awq_check_weight_shape(N, K, group);
    if (st != AWQ_OK) return st;
    if (!awq_aligned16(qweight_w3) || !awq_aligned16(qweight_w4)) return AWQ_ERR_MISALIGNED;
    const int num_tiles = (int)(N / 16) * (int)(K / AWQ_GROUP);
    repack_w3_to_w4_kernel<<<dim3((num_tiles + 3) / 4), dim3(256), 0, (hipStream_t)stream>>>(
        (const uint32_t *)qweight_w3, (uint4 *)qweight_w4, num_tiles);
    return awq_launch_status();
}

extern "C" size_t awq_w3a16_prefill_workspace_bytes(int64_t N, int64_t K, int group)
{
    if (awq_check_weight_shape(N, K, group) != AWQ_OK) return 0;
    return (size_t)(N * K / 2);
}

extern "C" int awq_w3a16_linear_prefill(const void *x_f16, const void *qweight, const void *scales,
                                        const void *zeros, void *y_f16, int64_t M, int64_t N, int64_t K,
                                        int group, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!x_f16 || !qweight || !scales || !zeros || !y_f16 || !workspace) return AWQ_ERR_NULL_POINTER;
    int st = awq_check_weight_shape(N, K, group);
    if (st != AWQ_OK) return st;
    if (M <= 16 || M > 0x7fffffff) return AWQ_ERR_BAD_SHAPE;   // M <= 16: awq_w3a16_linear
    if (!awq_aligned16(x_f16) || !awq_aligned16(qweight) || !awq_aligned16(scales) ||
        !awq_aligned16(zeros) || !awq_aligned16(y_f16) || !awq_aligned16(workspace))
        return AWQ_ERR_MISALIGNED;
    if (workspace_bytes < (size_t)(N * K / 2)) return AWQ_ERR_WORKSPACE_TOO_SMALL;
    if (M <= 128) {
        // a few dozen tokens: blocks of 16 through the 3-bit decode kernels in one grouped call
        // (see awq_w4a16_linear); the workspace is not touched
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
        return awq_w3a16_linear_multi(d, blocks, 16, group, stream);
    }
    st = awq_repack_w3_to_w4(qweight, N, K, group, workspace, stream);
    if (st != AWQ_OK) return st;
    // a few hundred tokens: with room behind the re-packed codes (rounded up to 256 bytes) for the
    // fp32 partial tiles, the prefill kernel cuts K into ranges as in awq_w4a16_linear
    const size_t repacked = ((size_t)(N * K / 2) + 255) & ~(size_t)255;
    const size_t partials = awq_linear_workspace_bytes(M, N, K, group);
    if (partials > 0 && workspace_bytes >= repacked + partials)
        return awq_gemm_launch_split(x_f16, workspace, scales, zeros, y_f16, (int)M, (int)N, (int)K,
                                     (unsigned char *)workspace + repacked,
                                     awq_gemm_ksplit((int)M, (int)N, (int)K, nullptr), (hipStream_t)stream);
    return awq_gemm_launch(x_f16, workspace, scales, zeros, y_f16, (int)M, (int)N, (int)K, (hipStream_t)stream);
}

extern "C" int awq_packed_sizes_w3(int64_t N, int64_t K, int group, size_t *qweight_bytes,
                                   size_t *scales_bytes, size_t *zeros_bytes)
{
    int st = awq_check_weight_shape(N, K, group);
    if (st != AWQ_OK) return st;
    const int64_t G = K / AWQ_GROUP;
    if (qweight_bytes) *qweight_bytes = (size_t)(N * K * 3 / 8);
    if (scales_bytes) *scales_bytes = (size_t)(N * G * 2);
    if (zeros_bytes) *zeros_bytes = (size_t)(N * G / 2);
    return AWQ_OK;
}

extern "C" int awq_quantize_pack_w3(const void *W_f16, const float *s, int64_t N, int64_t K,
                                    int group, void *qweight, void *scales, void *zeros,
                                    void *stream)
{
    if (!W_f16 || !qweight || !scales || !zeros) return AWQ_ERR_NULL_POINTER;
    int st = awq_check_weight_shape(N, K, group);
    if (st != AWQ_OK) return st;
    if (!awq_aligned16(W_f16) || !awq_aligned16(qweight) || !awq_aligned16(scales) ||
        !awq_aligned16(zeros) || (s && !awq_aligned16(s)))
        return AWQ_ERR_MISALIGNED;
    const int G = (int)(K / AWQ_GROUP);
    const int num_tiles = (int)(N / 16) * G;
    quantize_pack_w3_kernel<<<dim3((num_tiles + 3) / 4), dim3(256), 0, (hipStream_t)stream>>>(
        (const uint4 *)W_f16, (const float4 *)s, (uint32_t *)qweight, (uint16_t *)scales,
        (uint8_t *)zeros, G, num_tiles);
    return awq_launch_status();
}

extern "C" int awq_unpack_w3(const void *qweight, const void *scales, const void *zeros,
                             int64_t N, int64_t K, int group, uint8_t *codes, void *scales_f16,
                             uint8_t *zeros_u8, void *stream)
{
    if (!qweight || !scales || !zeros) return AWQ_ERR_NULL_POINTER;
    int st = awq_check_weight_shape(N, K, group);
    if (st != AWQ_OK) return st;
    if (!awq_aligned16(qweight) || !awq_aligned16(scales) || !awq_aligned16(zeros) ||
        (codes && !awq_aligned16(codes)) || (scales_f16 && !awq_aligned16(scales_f16)) ||
        (zeros_u8 && !awq_aligned16(zeros_u8)))
        return AWQ_ERR_MISALIGNED;
    const int G = (int)(K / AWQ_GROUP);
    const int num_tiles = (int)(N / 16) * G;
    unpack_w3_kernel<<<dim3((num_tiles + 3) / 4), dim3(256), 0, (hipStream_t)stream>>>(
        (const uint32_t *)qweight, (const uint16_t *)scales, (const uint8_t *)zeros, codes,
        (uint16_t *)scales_f16, zeros_u8, G, num_tiles);
    return awq_launch_status();
}

extern "C" int awq_w3a16_linear(const void *x_f16, const void *qweight, const void *scales,
                                const void *zeros, void *y_f16, int64_t M, int64_t N, int64_t K,
                                int group, void *stream)
{
    if (!x_f16 || !qweight || !scales || !zeros || !y_f16) return AWQ_ERR_NULL_POINTER;
    int st = awq_check_weight_shape(N, K, group);
    if (st != AWQ_OK) return st;
    if (M <= 0 || M > 16) return AWQ_ERR_BAD_SHAPE;          // decode path only
    if (!awq_aligned16(x_f16) || !awq_aligned16(qweight) || !awq_aligned16(scales) ||
        !awq_aligned16(zeros) || !awq_aligned16(y_f16))
        return AWQ_ERR_MISALIGNED;
    return awq_gemv_launch_w3(x_f16, qweight, scales, zeros, y_f16, (int)M, (int)N, (int)K,
                              (hipStream_t)stream);
}

// Sec. 4.2 kernel fusion for the 3-bit layout: as awq_w4a16_linear_multi.
extern "C" int awq_w3a16_linear_multi(const awq_linear_desc *descs, int count, int64_t M, int group,
                                      void *stream)
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
        int st = awq_gemv_stream_launch_w3(fit, nfit, (int)M, (hipStream_t)stream);
        if (st == AWQ_GEMV_STREAM_UNFIT) {
            for (int i = 0; i < count; ++i) grouped[i] = false;
        } else if (st != AWQ_OK) {
            return st;
        }
    }
    for (int i = 0; i < count; ++i) {
        if (grouped[i]) continue;
        int st = awq_gemv_launch_w3(p[i].x, p[i].q, p[i].sc, p[i].zp, p[i].y, (int)M, p[i].N, p[i].K,
                                    (hipStream_t)stream);
        if (st != AWQ_OK) return st;
    }
    return AWQ_OK;
}
