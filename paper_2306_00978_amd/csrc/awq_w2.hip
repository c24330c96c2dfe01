// INT2-g64 variant of the path for gfx950: quantize/pack, unpack and the decode kernel.
//
// AWQ Sec. 5 (the extreme low-bit table) quantizes to INT2 with group size 64.  The quantizer is
// the 4-level form of Sec. 3.2, Eq. 1-2, over groups of 64 input channels:
//   scale = fp16(clamp((max-min)/3, 2^-14, 65504)); zero = clamp(rint(-min/scale), 0, 3);
//   q = clamp(rint(w*s/scale) + zero, 0, 3),   binary32, one rounding per operation.
//
// Packed layout.  The unit is a block of 16 rows x 256 columns = four groups, 1 KB, so that a lane
// still fetches 16 bytes and a wave 1 KB of contiguous codes per load.  Lane l = (row l%16, column
// block c = l/16) owns the 64 codes of columns 64 t + 32 j + 8 c + 2 i + h (group t, half of the
// group j, i = 0..3, h = 0..1).  Word i of its 16-byte slot holds the codes with that i: the code
// of (t, j, h) in field f = t + 4 j, bits [2f, 2f+2), of the low (h = 0) or high (h = 1) half.
// Then  (word >> 8 j) & (0x00030003 << 2 t)  -- one AND, and one shift per word for j = 1 -- is
// the pair of columns (2i, 2i+1) of MFMA step (t, j) as two fp16 SUBNORMALS q * 4^t * 2^-24: the
// B-operand register i of v_mfma_f32_16x16x32_f16, with no integer-to-float conversion and no
// shift to the low bits.  The factor 4^t is the same for the whole group and is divided out
// together with the group's step.  A row's four steps of a block are stored together (one 8-byte
// load per lane), its four zero points share a byte, zero point t at bits [2t, 2t+2) -- the same
// place as the codes of group t, so the zero point needs no shift either.
//
// Decode kernel (M <= 16): a wave owns a 16-row block of one linear, or a slice of its K/256
// blocks where rows are long.  Per batch of up to four blocks a wave requests everything at once,
// copies the slice of x it needs into its own LDS area (16-byte loads, no workgroup barrier),
// requests the next batch, and runs per block eight MFMA steps against the codes and eight
// against the constant -z 4^t 2^-24 of the lane's row (a negative subnormal), all in one
// accumulator per group:
//   sum_k x_k (q_k - z) = 2^24 4^-t * (MFMA(x, q 4^t 2^-24) + MFMA(x, -z 4^t 2^-24)),  per group,
// then adds step * accumulator to the running sum of group position t with one mixed-precision
// FMA per output; the factors 2^(24 - 2t) are applied once after the loop.  Partial sums of the
// slices of a row block are combined through LDS in a fixed order.  Several linears (different
// shapes, same M) can share one launch.
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

    uint32_t words[4] = {0u, 0u, 0u, 0u}, zbyte = 0;
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

#pragma unroll
        for (int i = 0; i < 16; ++i) {             // i = 8 j + e, e = 2 (word) + h
            float v = __builtin_rintf(wp[i] / scale);
            v = v + zero;
            v = clamp2(v, 0.0f, 3.0f);
            words[(i % 8) / 2] |= (uint32_t)v << (16 * (i % 2) + 2 * (t + 4 * (i / 8)));
        }
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

// register i of the B fragment of MFMA step (t, j): the column pair (2i, 2i+1) as two fp16
// subnormals q * 4^t * 2^-24
__device__ __forceinline__ uint32_t w2_pair(uint32_t word, int t, int j)
{
    return (word >> (8 * j)) & (0x00030003u << (2 * t));
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
                uint32_t lo = 0, hi = 0;               // bytes e = 0..3 and 4..7
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const uint32_t pr = w2_pair(w[i], t, j) >> (2 * t);
                    const uint32_t two = (pr & 0xFFu) | ((pr >> 16) << 8);           // codes 2i, 2i+1
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

constexpr int W2_WAVES = 4;               // waves per workgroup

struct W2Args {
    W2Problem p[W2_MAX_PROBLEMS];
    int wg_begin[W2_MAX_PROBLEMS];     // first workgroup of each problem (wg_begin[0] = 0)
    int logS[W2_MAX_PROBLEMS];         // log2 of the K slices per row block: 0, 1 or 2
    int count, M;
};

// A workgroup has four waves; for a linear with S = 2^logS slices of K per row block it owns 4/S
// row blocks, wave w taking slice w % S of row block w / S.  Short rows (S = 1) give every wave a
// row block of its own and no exchange between waves at all; long rows are cut so that the waves
// of all linears of a launch have about the same number of blocks.
// MS = rows of x a wave stages (M <= MS, one of 1, 2, 4, 8, 16); rows >= M repeat row M-1 (row m
// of the MFMA result depends on row m of A only, and rows >= M are never stored).
// U = blocks per batch: all loads of a batch (its slice of x first, then steps, zero points and
// codes) are requested before anything is consumed, so a wave has U KB of codes in flight.  The
// blocks of a batch past the end of the wave's range repeat the range's last block (loads from
// addresses that are in bounds) and are skipped by a wave-uniform branch.
// Dynamic LDS: [4 waves][MS rows x (U*512 + 16) bytes], then [4/S row blocks][16*M outputs][4
// slots] of fp32 for the sum over the slices.
template <int MS, int U>
__global__ __launch_bounds__(256, 3) void gemv_w2_kernel(const W2Args a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    constexpr int CHUNKS = MS * U * 32;            // 16-byte chunks of x per batch
    constexpr int NS = (CHUNKS + 63) / 64;         // passes of one load per lane
    constexpr int ROW_BYTES = U * 512 + 16;        // +16: rows land on different banks
    constexpr int WAVE_BYTES = MS * ROW_BYTES;
    // the linear this workgroup works on: scalar selects over the argument table
    W2Problem P = a.p[0];
    int first = 0, logS = a.logS[0];
#pragma unroll
    for (int i = 1; i < W2_MAX_PROBLEMS; ++i)
        if (i < a.count && (int)blockIdx.x >= a.wg_begin[i]) {
            P = a.p[i];
            first = a.wg_begin[i];
            logS = a.logS[i];
        }
    const int M = a.M;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int S = 1 << logS, RBW = W2_WAVES >> logS;
    const int slice = wave & (S - 1), rbi = wave >> logS;
    const int K = P.K, N = P.N;
    const int B = K >> 8;
    const int rb_raw = ((int)blockIdx.x - first) * RBW + rbi;
    const bool active = rb_raw < (N >> 4);         // the last workgroup of a linear may have spare waves
    const int rb = active ? rb_raw : 0;
    const int r = lane & 15, c = lane >> 4;
    const int b0 = active ? (B * slice) >> logS : 0, b1 = active ? (B * (slice + 1)) >> logS : 0;

    const uint4 *qt = P.q + (int64_t)rb * B * 64 + lane;
    const uint2 *sc = P.sc + (int64_t)rb * B * 16 + r;
    const uint8_t *zp = P.zp + (int64_t)rb * B * 16 + r;
    const int mrow = r < M ? r : M - 1;
    unsigned char *xw = smem + (size_t)wave * WAVE_BYTES;
    const uint4 *xl = reinterpret_cast<const uint4 *>(xw + mrow * ROW_BYTES) + c;
    const uint4 *xg = reinterpret_cast<const uint4 *>(P.x);
    const int64_t K8 = (int64_t)K >> 3;

    // opaque to the optimizer, so that (v & mask) | sign is selected as one v_and_or_b32
    uint32_t kmask = 0x00030003u, ksign = 0x80008000u;
    asm("" : "+s"(kmask));
    asm("" : "+v"(ksign));
    float tot[4][4] = {};                          // [group of the block][output]: sums of step * acc
    // chunk ci = 64 i + lane of a batch's slice of x: row ci / (32 U), block (ci / 32) % U,
    // 16-byte chunk ci % 32 of the block
    uint4 xs[NS], q[U];
    uint2 sv[U];
    uint32_t z[U];
    auto request = [&](int b) {
#pragma unroll
        for (int i = 0; i < NS; ++i) {
            const int ci = 64 * i + lane;
            const int m = ci / (32 * U), u = (ci >> 5) % U;
            const int bu = b + u < b1 ? b + u : b1 - 1;
            xs[i] = xg[(int64_t)(m < M ? m : M - 1) * K8 + bu * 32 + (ci & 31)];
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int bu = b + u < b1 ? b + u : b1 - 1;
            sv[u] = sc[bu * 16];
            z[u] = zp[bu * 16];
            q[u] = qt[bu * 64];
        }
    };
#pragma unroll
    for (int i = 0; i < NS; ++i) xs[i] = make_uint4(0, 0, 0, 0);
#pragma unroll
    for (int u = 0; u < U; ++u) {
        q[u] = make_uint4(0, 0, 0, 0);
        sv[u] = make_uint2(0, 0);
        z[u] = 0;
    }
    if (b0 < b1) request(b0);
    for (int b = b0; b < b1; b += U) {
        // LDS operations of one wave execute in order: these stores follow the previous batch's reads
#pragma unroll
        for (int i = 0; i < NS; ++i) {
            const int ci = 64 * i + lane;
            const int m = ci / (32 * U), cc = ci % (32 * U);
            reinterpret_cast<uint4 *>(xw + m * ROW_BYTES)[cc] = xs[i];
        }
        // this batch's codes move to registers of their own and the next batch is requested
        // before this one is consumed (three waves per SIMD leave the registers for that)
        uint4 qc[U];
        uint2 svc[U];
        uint32_t zc[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            qc[u] = q[u];
            svc[u] = sv[u];
            zc[u] = z[u];
        }
        if (b + U < b1) request(b + U);            // wave-uniform
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (b + u < b1) {                      // wave-uniform
                uint4 xa[8];
#pragma unroll
                for (int jj = 0; jj < 8; ++jj) xa[jj] = xl[u * 32 + 4 * jj];      // k = 256 u + 32 jj + 8 c + 0..7
                const uint32_t w[4] = {qc[u].x, qc[u].y, qc[u].z, qc[u].w};
                const uint32_t wh[4] = {w[0] >> 8, w[1] >> 8, w[2] >> 8, w[3] >> 8};
                const half2_t s01 = __builtin_bit_cast(half2_t, svc[u].x), s23 = __builtin_bit_cast(half2_t, svc[u].y);
                const half_t sh[4] = {s01[0], s01[1], s23[0], s23[1]};
                const uint32_t zz = zc[u] * 0x00010001u;            // the zero-point byte in both halves
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const uint32_t mt = kmask << (2 * t);          // wave-uniform
                    // -z * 4^t * 2^-24 in every column of this lane's row: a negative fp16 subnormal
                    const uint32_t nz = (zz & mt) | ksign;
                    const half8_t zv = __builtin_bit_cast(half8_t, make_uint4(nz, nz, nz, nz));
                    const half8_t b0v = __builtin_bit_cast(half8_t, make_uint4(w[0] & mt, w[1] & mt, w[2] & mt, w[3] & mt));
                    const half8_t b1v = __builtin_bit_cast(half8_t, make_uint4(wh[0] & mt, wh[1] & mt, wh[2] & mt, wh[3] & mt));
                    const half8_t a0v = __builtin_bit_cast(half8_t, xa[2 * t]);
                    const half8_t a1v = __builtin_bit_cast(half8_t, xa[2 * t + 1]);
                    floatx4 acc = {0.f, 0.f, 0.f, 0.f};
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(a0v, b0v, acc, 0, 0, 0);
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(a0v, zv, acc, 0, 0, 0);
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(a1v, b1v, acc, 0, 0, 0);
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(a1v, zv, acc, 0, 0, 0);
                    // the group's step; the factor 2^24 / 4^t is applied after the loop
                    const float st = (float)sh[t];
#pragma unroll
                    for (int v = 0; v < 4; ++v) tot[t][v] = __builtin_fmaf(st, acc[v], tot[t][v]);
                }
            }
        }
    }

    floatx4 total;
#pragma unroll
    for (int v = 0; v < 4; ++v)
        total[v] = (tot[0][v] * 16777216.f + tot[1][v] * 4194304.f) + (tot[2][v] * 1048576.f + tot[3][v] * 262144.f);
    // lane holds y[m = 4c + v][n = 16 rb + r], complete (S = 1) or one slice's share of it
    if (logS == 0) {                               // uniform over the workgroup: no barrier below
        if (active) {
#pragma unroll
            for (int v = 0; v < 4; ++v)
                if (4 * c + v < M) P.y[(int64_t)(4 * c + v) * N + rb * 16 + r] = (half_t)total[v];
        }
        return;
    }
    // red[rbi][t][slot], t = 16 m + n: the partials of one output are contiguous, summed in fixed order
    const int MP = (M + 3) & ~3;
    float *red = reinterpret_cast<float *>(smem + (size_t)W2_WAVES * WAVE_BYTES);
    if (4 * c < M) {
#pragma unroll
        for (int v = 0; v < 4; ++v) red[((rbi * MP + 4 * c + v) * 16 + r) * 4 + slice] = total[v];
    }
    __syncthreads();
    for (int t = threadIdx.x; t < RBW * 16 * M; t += blockDim.x) {
        const int ri = t / (16 * M), o = t - ri * 16 * M;       // row block of the workgroup, output in it
        const int rbo = ((int)blockIdx.x - first) * RBW + ri;
        if (rbo < (N >> 4)) {
            const float4 pr = *reinterpret_cast<const float4 *>(red + ((ri * MP + (o >> 4)) * 16 + (o & 15)) * 4);
            const float sum = S == 2 ? pr.x + pr.y : (pr.x + pr.y) + (pr.z + pr.w);
            P.y[(int64_t)(o >> 4) * N + rbo * 16 + (o & 15)] = (half_t)sum;
        }
    }
}

template <int MS, int U>
int launch_w2_one(const W2Args &a, int total_wgs, size_t lds, hipStream_t stream)
{
    gemv_w2_kernel<MS, U><<<dim3(total_wgs), dim3(64 * W2_WAVES), lds, stream>>>(a);
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
    int64_t row_blocks = 0;
    for (int i = 0; i < count; ++i) row_blocks += probs[i].N / 16;
    // enough row blocks to give every CU several waves: at most 8..11 blocks (two or three batches)
    // per wave, which keeps the waves of short and long rows alike; otherwise K is cut as far as it
    // goes so that the launch has more waves
    const bool wide = row_blocks > 1024;
    int total = 0;
    for (int i = 0; i < count; ++i) {
        a.p[i] = probs[order[i]];
        const int B = a.p[i].K / 256;
        const int logS = wide ? (B <= 8 ? 0 : (B <= 16 ? 1 : 2)) : (B >= 4 ? 2 : (B >= 2 ? 1 : 0));
        a.logS[i] = logS;
        a.wg_begin[i] = total;
        const int rbw = W2_WAVES >> logS;
        total += (a.p[i].N / 16 + rbw - 1) / rbw;
    }
    a.count = count;
    a.M = M;
    const int MS = M == 1 ? 1 : (M == 2 ? 2 : (M <= 4 ? 4 : (M <= 8 ? 8 : 16)));
    // blocks per batch: at most eight passes of staging loads per lane
    const int U = MS <= 4 ? 4 : (MS == 8 ? 2 : 1);
    const size_t lds = (size_t)W2_WAVES * MS * (U * 512 + 16) + (size_t)W2_WAVES * ((M + 3) / 4 * 4) * 256;
    switch (MS) {
    case 1: return launch_w2_one<1, 4>(a, total, lds, stream);
    case 2: return launch_w2_one<2, 4>(a, total, lds, stream);
    case 4: return launch_w2_one<4, 4>(a, total, lds, stream);
    case 8: return launch_w2_one<8, 2>(a, total, lds, stream);
    default: return launch_w2_one<16, 1>(a, total, lds, stream);
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
    if (M <= 0 || M > 0x7fffffff) return AWQ_ERR_BAD_SHAPE;
    // up to 16 rows: one launch.  More: blocks of 16 rows through the same kernel, eight blocks
    // (128 rows) per launch; the last block of a launch is moved back to end at its last row (the
    // overlap is computed twice, same values)
    for (int64_t r0 = 0; r0 < M; r0 += 128) {
        const int64_t rows = M - r0 < 128 ? M - r0 : 128;
        W2Problem c = p;
        c.x = p.x + r0 * K;
        c.y = p.y + r0 * N;
        if (rows <= 16) {
            st = launch_w2(&c, 1, (int)rows, (hipStream_t)stream);
        } else {
            const int blocks = (int)((rows + 15) / 16);
            W2Problem d[W2_MAX_PROBLEMS];
            for (int b = 0; b < blocks; ++b) {
                const int64_t m0 = b + 1 < blocks ? 16 * (int64_t)b : rows - 16;
                d[b] = c;
                d[b].x = c.x + m0 * K;
                d[b].y = c.y + m0 * N;
            }
            st = launch_w2(d, blocks, 16, (hipStream_t)stream);
        }
        if (st != AWQ_OK) return st;
    }
    return AWQ_OK;
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
