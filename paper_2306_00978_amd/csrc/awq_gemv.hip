// Decode path of awq_w4a16_linear (M <= 16) for gfx950.
//
// AWQ Sec. 4.2: generation is memory-bound and weight traffic dominates, so the
// 4-bit weights are streamed once and dequantized on the fly inside the
// matrix-vector kernel; nothing dequantized is written back to memory.
//
// Mapping.  A workgroup owns one 16-row block of W (its tiles are contiguous along
// K); its waves split the K/128 groups between them.  Per tile a lane issues one
// 16-byte load (the wave reads the 1 KB tile fully coalesced) and receives, in
// word j, eight codes that are its B-operand fragment of the j-th
// v_mfma_f32_16x16x32_f16 step (n = lane%16, k = 32j + 8*(lane/16) + 0..7).  The
// activations are the A operand (m = lane%16), so one MFMA chain handles up to 16
// tokens at the cost of one, and the k-reduction across lanes happens inside the
// matrix core instead of through shuffles.
//
// Dequantization in registers: the nibble order of a word makes
// (w >> {0,8}) & 0x000F000F | 0x6400.. the half pair (1024+q, 1024+q') and
// & 0x00F000F0 | 0x5400.. the pair (64+q, 64+q'); subtracting (1024+z) / (64+z)
// with one packed-half add each gives q - z exactly.  The MFMA accumulates
// sum_k x*(q-z) per group in fp32 and the group's step is applied once per group
// in fp32, so the only roundings are those of the fp32 accumulation.
//
// The partial sums of the waves are combined through LDS in a fixed order
// (deterministic output), rounded once to fp16 and stored.
#include "awq_common.h"

#include <stdlib.h>

namespace {

__device__ __forceinline__ half8_t expand_word(uint32_t w, uint32_t zA, uint32_t zB)
{
    const uint32_t w8 = w >> 8;
    const uint32_t t0 = (w & 0x000F000Fu) | 0x64006400u;
    const uint32_t t1 = (w & 0x00F000F0u) | 0x54005400u;
    const uint32_t t2 = (w8 & 0x000F000Fu) | 0x64006400u;
    const uint32_t t3 = (w8 & 0x00F000F0u) | 0x54005400u;
    const half2_t a = __builtin_bit_cast(half2_t, zA), b = __builtin_bit_cast(half2_t, zB);
    const half2_t d0 = __builtin_bit_cast(half2_t, t0) - a;
    const half2_t d1 = __builtin_bit_cast(half2_t, t1) - b;
    const half2_t d2 = __builtin_bit_cast(half2_t, t2) - a;
    const half2_t d3 = __builtin_bit_cast(half2_t, t3) - b;
    half8_t out;
    out[0] = d0[0]; out[1] = d0[1]; out[2] = d1[0]; out[3] = d1[1];
    out[4] = d2[0]; out[5] = d2[1]; out[6] = d3[0]; out[7] = d3[1];
    return out;
}

// U = tiles (groups) a wave keeps in flight per loop trip.
template <int U>
__global__ __launch_bounds__(1024) void gemv_kernel(
    const half_t *__restrict__ x, const uint4 *__restrict__ qweight,
    const uint16_t *__restrict__ scales, const uint8_t *__restrict__ zeros,
    half_t *__restrict__ y, int M, int N, int K, int G)
{
    __shared__ float red[16][4][64];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave-uniform
    const int W = blockDim.x >> 6;
    const int rb = blockIdx.x;
    const int r = lane & 15, c = lane >> 4;

    const int g0 = (G * wave) / W, g1 = (G * (wave + 1)) / W;
    const uint4 *qt = qweight + (int64_t)rb * G * 64 + lane;
    const uint16_t *sc = scales + (int64_t)rb * G * 16 + r;
    const uint8_t *zp = zeros + (int64_t)rb * G * 8 + (r >> 1);
    const int zshift = (r & 1) * 4;
    // A-operand row m = lane%16.  Rows >= M read a valid row instead of zeros: row m of
    // the MFMA result depends on row m of A only, and rows >= M are never stored.
    const uint4 *xr = reinterpret_cast<const uint4 *>(x + (int64_t)(r < M ? r : M - 1) * K + 8 * c);

    floatx4 total = {0.f, 0.f, 0.f, 0.f};
    for (int base = g0; base < g1; base += U) {
        uint4 q[U];
        float sv[U];
        uint32_t zv[U];
        int gi[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int g = base + u;
            gi[u] = g < g1 ? g : g1 - 1;
            q[u] = qt[(int64_t)gi[u] * 64];
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const half_t sh = __builtin_bit_cast(half_t, sc[gi[u] * 16]);
            sv[u] = (base + u < g1) ? (float)sh : 0.0f;
            zv[u] = (zp[gi[u] * 8] >> zshift) & 0xFu;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            uint4 xa[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                // k = 128*g + 32*j + 8*c + 0..7  ->  16-byte run index 16*g + 4*j (+c folded in xr)
                xa[j] = xr[gi[u] * 16 + 4 * j];
            }
            const uint32_t zA = 0x64006400u | (zv[u] * 0x00010001u);
            const uint32_t zB = 0x54005400u | (zv[u] * 0x00100010u);
            const uint32_t words[4] = {q[u].x, q[u].y, q[u].z, q[u].w};
            floatx4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const half8_t b = expand_word(words[j], zA, zB);
                const half8_t a = __builtin_bit_cast(half8_t, xa[j]);
                acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, acc, 0, 0, 0);
            }
#pragma unroll
            for (int v = 0; v < 4; ++v) total[v] += sv[u] * acc[v];
        }
    }

    // lane holds y[m = 4*c + v][n = 16*rb + r] partials; combine the waves in order
#pragma unroll
    for (int v = 0; v < 4; ++v) red[wave][v][lane] = total[v];
    __syncthreads();
    for (int t = threadIdx.x; t < 256; t += blockDim.x) {
        const int v = t >> 6, l = t & 63;
        float sum = 0.f;
        for (int w = 0; w < W; ++w) sum += red[w][v][l];
        const int m = 4 * (l >> 4) + v;
        if (m < M) y[(int64_t)m * N + rb * 16 + (l & 15)] = (half_t)sum;
    }
}

int pick_waves(int G)
{
    static const int forced = [] {
        const char *e = getenv("AWQ_GEMV_WAVES");
        return e ? atoi(e) : 0;
    }();
    if (forced >= 1 && forced <= 16) return forced;
    int w = (G + 3) / 4;
    if (w < 4) w = 4;
    if (w > 16) w = 16;
    return w;
}

int pick_unroll(int G, int W)
{
    static const int forced = [] {
        const char *e = getenv("AWQ_GEMV_UNROLL");
        return e ? atoi(e) : 0;
    }();
    if (forced >= 2 && forced <= 4) return forced;
    const int cnt = (G + W - 1) / W;
    int best = 4, waste = 1 << 30;
    for (int u = 4; u >= 2; --u) {
        const int wst = (cnt + u - 1) / u * u - cnt;
        if (wst < waste) { waste = wst; best = u; }
    }
    return best;
}

}  // namespace

// Host side of the decode path; arguments were validated by awq_w4a16_linear.
int awq_gemv_launch(const void *x, const void *qweight, const void *scales, const void *zeros,
                    void *y, int M, int N, int K, hipStream_t stream)
{
    const int G = K / AWQ_GROUP;
    const int W = pick_waves(G);
    const int U = pick_unroll(G, W);
    const dim3 grid(N / 16), block(W * 64);
#define AWQ_GEMV_ARGS (const half_t *)x, (const uint4 *)qweight, (const uint16_t *)scales, \
                      (const uint8_t *)zeros, (half_t *)y, M, N, K, G
    switch (U) {
    case 2: gemv_kernel<2><<<grid, block, 0, stream>>>(AWQ_GEMV_ARGS); break;
    case 3: gemv_kernel<3><<<grid, block, 0, stream>>>(AWQ_GEMV_ARGS); break;
    default: gemv_kernel<4><<<grid, block, 0, stream>>>(AWQ_GEMV_ARGS); break;
    }
#undef AWQ_GEMV_ARGS
    return awq_launch_status();
}
