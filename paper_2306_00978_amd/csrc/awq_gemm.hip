// Prefill path of awq_w4a16_linear (M > 16) for gfx950.
//
// AWQ Sec. 4.2: with 4-bit storage and 16-bit compute the dequantization has to
// sit inside the main loop of the matrix-matrix kernel (it cannot be moved to the
// epilogue as with W8A8), and dequantized weights are never written to memory.
//
// Mapping.  A workgroup computes a 128 (tokens) x 256 (out-features) tile of y with
// four waves side by side along N (wave tile 128 x 64 = 8 x 4 MFMA tiles, 128 fp32
// accumulators per lane), looping over K one quantization group (128) at a time.
//   * x tile (128 x 128 fp16, 32 KB) goes through LDS, double-buffered, stored in MFMA
//     fragment order so that every A-operand read is one conflict-free ds_read_b128;
//     each fragment read feeds four MFMAs, which keeps LDS traffic at half its peak.
//   * weights never touch LDS: the packed layout is already the B-operand layout of
//     v_mfma_f32_16x16x32_f16, so a lane loads its 16 bytes per 16x128 tile straight
//     from global memory (prefetched one group ahead), expands them in registers to
//     fp16 (q - z) * scale and feeds the matrix core.  Each wave owns its own four
//     16-row weight tiles, so no weight is dequantized twice inside a workgroup.
//   * one rounding to fp16 at the end.
#include "awq_common.h"

namespace {

constexpr int BM = 128, BN = 256;
constexpr int WN_TILES = 4;                 // 16-row weight tiles per wave
constexpr int A_FRAGS = 8 * 4;              // (m-tile, k-step) fragments of 1 KB per buffer

struct DqConsts {
    uint32_t mask_lo, mask_hi;   // SGPR
    uint32_t magA, magB;         // VGPR
};

__device__ __forceinline__ DqConsts dq_consts()
{
    DqConsts k = {0x000F000Fu, 0x00F000F0u, 0x64006400u, 0x54005400u};
    asm("" : "+s"(k.mask_lo));
    asm("" : "+s"(k.mask_hi));
    asm("" : "+v"(k.magA));
    asm("" : "+v"(k.magB));
    return k;
}

// eight codes of one packed word -> (q - z) * scale in fp16, k order.
// (w & mask) | magic is 1024+q or 64+q as a half pair; subtracting 1024+z / 64+z is exact.
__device__ __forceinline__ half8_t dequant_word(uint32_t w, const DqConsts &k, half2_t zA,
                                                half2_t zB, half2_t s2)
{
    const uint32_t w8 = w >> 8;
    const uint32_t t0 = (w & k.mask_lo) | k.magA;
    const uint32_t t1 = (w & k.mask_hi) | k.magB;
    const uint32_t t2 = (w8 & k.mask_lo) | k.magA;
    const uint32_t t3 = (w8 & k.mask_hi) | k.magB;
    const half2_t d0 = (__builtin_bit_cast(half2_t, t0) - zA) * s2;
    const half2_t d1 = (__builtin_bit_cast(half2_t, t1) - zB) * s2;
    const half2_t d2 = (__builtin_bit_cast(half2_t, t2) - zA) * s2;
    const half2_t d3 = (__builtin_bit_cast(half2_t, t3) - zB) * s2;
    half8_t out;
    out[0] = d0[0]; out[1] = d0[1]; out[2] = d1[0]; out[3] = d1[1];
    out[4] = d2[0]; out[5] = d2[1]; out[6] = d3[0]; out[7] = d3[1];
    return out;
}

__global__ __launch_bounds__(256, 1) void gemm_kernel(
    const half_t *__restrict__ x, const uint4 *__restrict__ qweight,
    const uint16_t *__restrict__ scales, const uint8_t *__restrict__ zeros,
    half_t *__restrict__ y, int M, int N, int K, int G)
{
    __shared__ uint4 a_lds[2][A_FRAGS * 64];       // [buffer][m-tile i][k-step j][lane], 2 x 32 KB
    const DqConsts kc = dq_consts();
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r = lane & 15, c = lane >> 4;
    const int m0 = blockIdx.y * BM;
    const int NT = N / 16;                         // 16-row weight tiles in the matrix
    const int nt0 = blockIdx.x * (BN / 16) + wave * WN_TILES;

    // per-lane weight streams of the wave's four 16-row blocks (clamped when ragged)
    const uint4 *qt[WN_TILES];
    const uint16_t *sc[WN_TILES];
    const uint8_t *zp[WN_TILES];
#pragma unroll
    for (int t = 0; t < WN_TILES; ++t) {
        const int64_t rb = nt0 + t < NT ? nt0 + t : NT - 1;
        qt[t] = qweight + rb * G * 64 + lane;
        sc[t] = scales + rb * G * 16 + r;
        zp[t] = zeros + rb * G * 8 + (r >> 1);
    }
    const int zshift = (r & 1) * 4;

    // x tile copy: unit u = tid + 256*p -> row u/16, 16-byte run u%16 of the 128-wide k slab
    const uint4 *xg[8];
    int ldst[8];
#pragma unroll
    for (int p = 0; p < 8; ++p) {
        const int u = tid + 256 * p;
        const int row = u >> 4, oct = u & 15;
        const int mr = m0 + row < M ? m0 + row : M - 1;          // rows >= M repeat a valid row
        xg[p] = reinterpret_cast<const uint4 *>(x + (int64_t)mr * K) + oct;
        ldst[p] = ((row >> 4) * 4 + (oct >> 2)) * 64 + (row & 15) + 16 * (oct & 3);
    }

    floatx4 acc[8][WN_TILES];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int t = 0; t < WN_TILES; ++t) acc[i][t] = floatx4{0.f, 0.f, 0.f, 0.f};

    uint4 areg[8], breg[WN_TILES];
    uint32_t sreg[WN_TILES], zreg[WN_TILES];
#define AWQ_GEMM_LOAD(g_)                                                        \
    {                                                                            \
        _Pragma("unroll") for (int p = 0; p < 8; ++p) areg[p] = xg[p][(g_) * 16]; \
        _Pragma("unroll") for (int t = 0; t < WN_TILES; ++t) {                   \
            breg[t] = qt[t][(g_) * 64];                                          \
            sreg[t] = sc[t][(g_) * 16];                                          \
            zreg[t] = zp[t][(g_) * 8];                                           \
        }                                                                        \
    }

    AWQ_GEMM_LOAD(0)
#pragma unroll
    for (int p = 0; p < 8; ++p) a_lds[0][ldst[p]] = areg[p];
    __syncthreads();

    for (int g = 0; g < G; ++g) {
        const uint4 *abuf = a_lds[g & 1];
        // this group's weights; next group's operands are requested right away
        uint4 bcur[WN_TILES];
        half2_t s2[WN_TILES], zA[WN_TILES], zB[WN_TILES];
#pragma unroll
        for (int t = 0; t < WN_TILES; ++t) {
            bcur[t] = breg[t];
            const half_t sh = __builtin_bit_cast(half_t, (uint16_t)sreg[t]);
            s2[t] = half2_t{sh, sh};
            const uint32_t z = (zreg[t] >> zshift) & 0xFu;
            zA[t] = __builtin_bit_cast(half2_t, 0x64006400u | (z * 0x00010001u));
            zB[t] = __builtin_bit_cast(half2_t, 0x54005400u | (z * 0x00100010u));
        }
        // unconditional (the last trip re-reads its own group): keeps the staging registers
        // out of control flow.  The fence keeps the requests at the top of the trip, a whole
        // trip ahead of their use.
        const int gn = g + 1 < G ? g + 1 : g;
        AWQ_GEMM_LOAD(gn)
        asm volatile("" ::: "memory");

        // A fragments are fetched two steps ahead of the MFMAs that use them
        const uint4 *ap = abuf + lane;
        uint4 a0 = ap[0 * 64], a1 = ap[4 * 64];           // (i=0,j=0), (i=1,j=0)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            half8_t bf[WN_TILES];
#pragma unroll
            for (int t = 0; t < WN_TILES; ++t) {
                const uint32_t w = j == 0 ? bcur[t].x : j == 1 ? bcur[t].y : j == 2 ? bcur[t].z : bcur[t].w;
                bf[t] = dequant_word(w, kc, zA[t], zB[t], s2[t]);
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const half8_t a = __builtin_bit_cast(half8_t, a0);
                a0 = a1;
                const int nx = j * 8 + i + 2;              // step index of the fragment to fetch
                if (nx < 32) a1 = ap[((nx & 7) * 4 + (nx >> 3)) * 64];
#pragma unroll
                for (int t = 0; t < WN_TILES; ++t)
                    acc[i][t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, bf[t], acc[i][t], 0, 0, 0);
            }
        }
        {
            // the other buffer was last read in iteration g-1, which every wave has left
            uint4 *nbuf = a_lds[(g + 1) & 1];
#pragma unroll
            for (int p = 0; p < 8; ++p) nbuf[ldst[p]] = areg[p];
        }
        __syncthreads();
    }
#undef AWQ_GEMM_LOAD

    // epilogue: lane holds y[m0 + 16i + 4c + v][16*(nt0+t) + r]
#pragma unroll
    for (int t = 0; t < WN_TILES; ++t) {
        if (nt0 + t >= NT) continue;
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
    if (grid.y > 65535) return AWQ_ERR_BAD_SHAPE;
    gemm_kernel<<<grid, block, 0, stream>>>((const half_t *)x, (const uint4 *)qweight,
                                            (const uint16_t *)scales, (const uint8_t *)zeros,
                                            (half_t *)y, M, N, K, G);
    return awq_launch_status();
}
