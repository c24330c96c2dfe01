// Prefill path of awq_w4a16_linear (M > 16) for gfx950.
//
// AWQ Sec. 4.2: with 4-bit storage and 16-bit compute the dequantization has to
// sit inside the main loop of the matrix-matrix kernel (it cannot be moved to the
// epilogue as with W8A8), and dequantized weights are never written to memory.
//
// Mapping.  A workgroup computes a 128 (tokens) x 128 (out-features) tile of y with
// four waves side by side along N (wave tile 128 x 32), looping over K one
// quantization group (128) at a time.
//   * x tile (128 x 128 fp16, 32 KB) goes through LDS, stored in MFMA fragment
//     order so that every A-operand read is one conflict-free ds_read_b128.
//   * weights never touch LDS: the packed layout is already the B-operand layout of
//     v_mfma_f32_16x16x32_f16, so a lane loads its 16 bytes per 16x128 tile straight
//     from global memory, expands them in registers to fp16 (q - z) * scale and
//     feeds the matrix core.  Each wave owns its own two 16-row weight tiles, so no
//     weight is dequantized twice inside a workgroup.
//   * fp32 accumulators (8 x 2 MFMA tiles per wave), one rounding to fp16 at the end.
#include "awq_common.h"

namespace {

constexpr int BM = 128, BN = 128;

__device__ __forceinline__ half8_t dequant_word(uint32_t w, uint32_t zA, uint32_t zB, half2_t s2)
{
    const uint32_t w8 = w >> 8;
    const uint32_t t0 = (w & 0x000F000Fu) | 0x64006400u;
    const uint32_t t1 = (w & 0x00F000F0u) | 0x54005400u;
    const uint32_t t2 = (w8 & 0x000F000Fu) | 0x64006400u;
    const uint32_t t3 = (w8 & 0x00F000F0u) | 0x54005400u;
    const half2_t a = __builtin_bit_cast(half2_t, zA), b = __builtin_bit_cast(half2_t, zB);
    const half2_t d0 = (__builtin_bit_cast(half2_t, t0) - a) * s2;
    const half2_t d1 = (__builtin_bit_cast(half2_t, t1) - b) * s2;
    const half2_t d2 = (__builtin_bit_cast(half2_t, t2) - a) * s2;
    const half2_t d3 = (__builtin_bit_cast(half2_t, t3) - b) * s2;
    half8_t out;
    out[0] = d0[0]; out[1] = d0[1]; out[2] = d1[0]; out[3] = d1[1];
    out[4] = d2[0]; out[5] = d2[1]; out[6] = d3[0]; out[7] = d3[1];
    return out;
}

__global__ __launch_bounds__(256, 2) void gemm_kernel(
    const half_t *__restrict__ x, const uint4 *__restrict__ qweight,
    const uint16_t *__restrict__ scales, const uint8_t *__restrict__ zeros,
    half_t *__restrict__ y, int M, int N, int K, int G)
{
    __shared__ uint4 a_lds[8 * 4 * 64];            // [i][j][lane] fragments, 32 KB
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int r = lane & 15, c = lane >> 4;
    const int m0 = blockIdx.y * BM;
    const int NT = N / 16;                         // number of 16-row weight tiles rows
    const int nt0 = blockIdx.x * (BN / 16) + wave * 2;

    // per-lane weight streams of the wave's two 16-row blocks (clamped when ragged)
    const uint4 *qt[2];
    const uint16_t *sc[2];
    const uint8_t *zp[2];
    bool nvalid[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        nvalid[t] = nt0 + t < NT;
        const int64_t rb = nvalid[t] ? nt0 + t : 0;
        qt[t] = qweight + rb * G * 64 + lane;
        sc[t] = scales + rb * G * 16 + r;
        zp[t] = zeros + rb * G * 8 + (r >> 1);
    }
    const int zshift = (r & 1) * 4;

    // x tile copy: unit u = tid + 256*p -> row u/16, 16-byte run u%16
    const uint4 *xg[8];
    int ldst[8];
    bool avalid[8];
#pragma unroll
    for (int p = 0; p < 8; ++p) {
        const int u = tid + 256 * p;
        const int row = u >> 4, oct = u & 15;
        avalid[p] = m0 + row < M;
        xg[p] = reinterpret_cast<const uint4 *>(x + (int64_t)(avalid[p] ? m0 + row : 0) * K) + oct;
        ldst[p] = ((row >> 4) * 4 + (oct >> 2)) * 64 + (row & 15) + 16 * (oct & 3);
    }

    floatx4 acc[8][2];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int t = 0; t < 2; ++t) acc[i][t] = floatx4{0.f, 0.f, 0.f, 0.f};

    uint4 areg[8], breg[2];
    uint16_t sreg[2];
    uint32_t zreg[2];
    auto load_tiles = [&](int g) {
#pragma unroll
        for (int p = 0; p < 8; ++p)
            areg[p] = avalid[p] ? xg[p][g * 16] : make_uint4(0, 0, 0, 0);
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            breg[t] = qt[t][(int64_t)g * 64];
            sreg[t] = sc[t][g * 16];
            zreg[t] = (zp[t][g * 8] >> zshift) & 0xFu;
        }
    };

    load_tiles(0);
#pragma unroll
    for (int p = 0; p < 8; ++p) a_lds[ldst[p]] = areg[p];
    __syncthreads();

    for (int g = 0; g < G; ++g) {
        // this group's weights, expanded to fp16 (q - z) * scale
        half8_t bf[2][4];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const half_t sh = __builtin_bit_cast(half_t, sreg[t]);
            const half2_t s2 = {sh, sh};
            const uint32_t zA = 0x64006400u | (zreg[t] * 0x00010001u);
            const uint32_t zB = 0x54005400u | (zreg[t] * 0x00100010u);
            const uint32_t words[4] = {breg[t].x, breg[t].y, breg[t].z, breg[t].w};
#pragma unroll
            for (int j = 0; j < 4; ++j) bf[t][j] = dequant_word(words[j], zA, zB, s2);
        }
        if (g + 1 < G) load_tiles(g + 1);          // prefetch into registers

#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const half8_t a = __builtin_bit_cast(half8_t, a_lds[(i * 4 + j) * 64 + lane]);
                acc[i][0] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, bf[0][j], acc[i][0], 0, 0, 0);
                acc[i][1] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, bf[1][j], acc[i][1], 0, 0, 0);
            }
        __syncthreads();
        if (g + 1 < G) {
#pragma unroll
            for (int p = 0; p < 8; ++p) a_lds[ldst[p]] = areg[p];
        }
        __syncthreads();
    }

    // epilogue: lane holds y[m0 + 16i + 4c + v][16*(nt0+t) + r]
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        if (!nvalid[t]) continue;
        const int n = (nt0 + t) * 16 + r;
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int m = m0 + 16 * i + 4 * c + v;
                if (m < M) y[(int64_t)m * N + n] = (half_t)acc[i][t][v];
            }
    }
}

}  // namespace

// Host side of the prefill path; arguments were validated by awq_w4a16_linear.
int awq_gemm_launch(const void *x, const void *qweight, const void *scales, const void *zeros,
                    void *y, int M, int N, int K, hipStream_t stream)
{
    const int G = K / AWQ_GROUP;
    const dim3 grid((N + BN - 1) / BN, (M + BM - 1) / BM), block(256);
    gemm_kernel<<<grid, block, 0, stream>>>((const half_t *)x, (const uint4 *)qweight,
                                            (const uint16_t *)scales, (const uint8_t *)zeros,
                                            (half_t *)y, M, N, K, G);
    return awq_launch_status();
}
