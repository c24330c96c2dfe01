// Prefill path of awq_w4a16_linear (M > 16) for gfx950.
//
// AWQ Sec. 4.2: with 4-bit storage and 16-bit compute the dequantization has to
// sit inside the main loop of the matrix-matrix kernel (it cannot be moved to the
// epilogue as with W8A8), and dequantized weights are never written to memory.
//
// Mapping.  A workgroup computes a 128 (tokens) x 256 (out-features) tile of y with
// four waves side by side along N; a wave owns 128 x 64 = 4 x 2 tiles of
// v_mfma_f32_32x32x16_f16 (128 fp32 accumulators per lane) and loops over K one
// quantization group (128 columns = 8 MFMA steps) at a time.  The 32x32x16 shape is
// chosen for its issue budget: one MFMA keeps the matrix pipe busy for 32 cycles, and in
// that shadow the wave has to issue everything else (operand reads, dequantization).
//
// Operands.  Nothing is staged through registers on the way in: both operands are
// fetched with global_load_lds (memory -> LDS, 16 bytes per lane landing in lane order),
// two groups ahead of the one being computed, into a ring of three stages.
//   * x: one load instruction fetches 8 rows x 128 contiguous bytes (whole cache lines) and
//     lands as 8 LDS rows of 128 bytes.  Which 16-byte chunk of the row a lane fetches is
//     XOR-swizzled with the row index, so that the A fragment of any MFMA step (lane l: row
//     l%32, 16 bytes at columns 16 s + 8 (l/32)) is read back with one conflict-free
//     ds_read_b128.  The four waves share the x tile (each loads its own 32 rows, all read
//     all four row blocks); one barrier per group.
//   * weights: the packed layout is already the B-operand layout.  For a block of 32
//     out-features (two 16-row tiles), lane l takes slot (l%16) + 16 (2h + l/32) of tile
//     (l%32)/16: its word j is the fragment of MFMA step k = 32 j + 16 h.  A wave's
//     weights are private to it (4 KB + steps + zero points per group).
//   Each fragment word is expanded in registers to fp16 (q - z) * scale and feeds four
//   MFMAs (the four token blocks), so dequantization costs about three vector
//   instructions per MFMA.
// fp32 accumulation, one rounding to fp16 at the end.
#include "awq_common.h"

namespace {

typedef __attribute__((address_space(3))) void lds_void_t;
typedef const __attribute__((address_space(1))) void gbl_void_t;

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int BM = 128, BN = 256;
constexpr int NSTAGE = 3;
constexpr int A_STAGE = 32 * 1024;               // 4 row blocks x 2 column halves x (32 rows x 128 B)
constexpr int B_STAGE = 4096 + 256 + 128;        // 2 blocks x 2 halves x 1 KB, 64 steps, 32 zero bytes
constexpr int B_SC = 4096, B_ZP = 4352;
constexpr int LDS_BYTES = NSTAGE * A_STAGE + 4 * NSTAGE * B_STAGE;
constexpr int LOADS_PER_GROUP = 8 + 4 + 2;       // per wave

__device__ __forceinline__ void dma16(const void *g, uint32_t lds_addr)
{
    __builtin_amdgcn_global_load_lds((gbl_void_t *)(uintptr_t)g, (lds_void_t *)(uintptr_t)lds_addr,
                                     16, 0, 0);
}
__device__ __forceinline__ void dma2(const void *g, uint32_t lds_addr)
{
    __builtin_amdgcn_global_load_lds((gbl_void_t *)(uintptr_t)g, (lds_void_t *)(uintptr_t)lds_addr,
                                     2, 0, 0);
}
__device__ __forceinline__ void dma1(const void *g, uint32_t lds_addr)
{
    __builtin_amdgcn_global_load_lds((gbl_void_t *)(uintptr_t)g, (lds_void_t *)(uintptr_t)lds_addr,
                                     1, 0, 0);
}

// LDS reads are written as asm so that the compiler does not tie them to the outstanding
// memory->LDS loads of later groups; the waits are placed by hand.
__device__ __forceinline__ u32x4 lds_read16(uint32_t addr)
{
    u32x4 v;
    asm volatile("ds_read_b128 %0, %1" : "=v"(v) : "v"(addr));
    return v;
}
template <int OFF>
__device__ __forceinline__ u32x4 lds_read16_off(uint32_t addr)
{
    u32x4 v;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
    return v;
}
__device__ __forceinline__ uint32_t lds_read4(uint32_t addr)
{
    uint32_t v;
    asm volatile("ds_read_b32 %0, %1" : "=v"(v) : "v"(addr));
    return v;
}
__device__ __forceinline__ void lds_wait(u32x4 &a, u32x4 &b, u32x4 &c, u32x4 &d)
{
    asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(a), "+v"(b), "+v"(c), "+v"(d));
}

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
    uint4 out;
    out.x = __builtin_bit_cast(uint32_t, d0);
    out.y = __builtin_bit_cast(uint32_t, d1);
    out.z = __builtin_bit_cast(uint32_t, d2);
    out.w = __builtin_bit_cast(uint32_t, d3);
    return __builtin_bit_cast(half8_t, out);
}

__device__ __forceinline__ uint32_t word_of(const u32x4 &v, int j)
{
    return v[j];
}

__global__ __launch_bounds__(256, 1) void gemm_kernel(
    const half_t *__restrict__ x, const unsigned char *__restrict__ qweight,
    const unsigned char *__restrict__ scales, const unsigned char *__restrict__ zeros,
    half_t *__restrict__ y, int M, int N, int K, int G)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const DqConsts kc = dq_consts();
    const uint32_t lds0 = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)smem);
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, hi = lane >> 5;
    const int m0 = blockIdx.y * BM;
    const int NT = N >> 4;                                   // 16-row weight tiles in the matrix
    const int nt0 = blockIdx.x * (BN / 16) + wave * 4;      // first of the wave's four tiles

    // ---- sources of this lane's memory->LDS loads (group 0), advanced by constant strides
    // x: load instruction d of a group (d = 0..7) covers rows 8 (d%4) .. +8 of the wave's 32
    // rows and columns 64 (d/4) .. +64; lane l takes row 8 (d%4) + l/8 (rows >= M repeat row
    // M-1) and chunk (l%8) ^ f, f = (l/16)%4 = ((row in block)/2)%4, and lands at chunk l%8
    const unsigned char *xsrc[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        int xr = m0 + 32 * wave + 8 * q + (lane >> 3);
        xr = xr < M ? xr : M - 1;
        const int chunk = (lane & 7) ^ ((lane >> 4) & 3);
        xsrc[q] = reinterpret_cast<const unsigned char *>(x) + ((size_t)xr * K + 8 * chunk) * 2;
    }
    // weights: block b (32 out-features = tiles nt0+2b, nt0+2b+1), half h
    const unsigned char *qsrc[2];
#pragma unroll
    for (int b = 0; b < 2; ++b) {
        int t = nt0 + 2 * b + (l32 >> 4);
        t = t < NT ? t : NT - 1;                             // ragged N: repeat the last tile
        qsrc[b] = qweight + ((size_t)t * G * 64 + (l32 & 15) + 16 * hi) * 16;
    }
    // steps: lane -> block lane/32, row l32; zero points: lane < 32 -> block lane/16, byte lane%16
    const unsigned char *ssrc, *zsrc;
    {
        int t = nt0 + 2 * hi + (l32 >> 4);
        t = t < NT ? t : NT - 1;
        ssrc = scales + ((size_t)t * G * 16 + (l32 & 15)) * 2;
        int tz = nt0 + 2 * ((lane >> 4) & 1) + ((lane >> 3) & 1);
        tz = tz < NT ? tz : NT - 1;
        zsrc = zeros + (size_t)tz * G * 8 + (lane & 7);
    }

    const uint32_t a_ring = lds0;
    const uint32_t b_ring = lds0 + NSTAGE * A_STAGE + (uint32_t)wave * (NSTAGE * B_STAGE);

    auto issue_group = [&](int g, int stage) {
        g = g < G ? g : G - 1;                               // past the end: a harmless repeat
        // LDS: [row block 4][column half 2][32 rows x 128 B]
        const uint32_t adst = a_ring + (uint32_t)stage * A_STAGE + (uint32_t)wave * 8192;
#pragma unroll
        for (int d = 0; d < 8; ++d)
            dma16(xsrc[d & 3] + (size_t)g * 256 + (d >> 2) * 128, adst + (d >> 2) * 4096 + (d & 3) * 1024);
        const uint32_t bdst = b_ring + (uint32_t)stage * B_STAGE;
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            const unsigned char *qs = qsrc[b] + (size_t)g * 1024;
            dma16(qs, bdst + (2 * b) * 1024);
            dma16(qs + 512, bdst + (2 * b + 1) * 1024);
        }
        dma2(ssrc + (size_t)g * 32, bdst + B_SC);
        if (lane < 32) dma1(zsrc + (size_t)g * 8, bdst + B_ZP);
    };

    floatx16 acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][b][v] = 0.f;

    issue_group(0, 0);
    issue_group(1, 1);
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(LOADS_PER_GROUP) : "memory");
    __builtin_amdgcn_s_barrier();

    const uint32_t lane16 = (uint32_t)lane << 4;
    // byte offset of this lane's A fragment inside a (row block, column half) area, for the
    // four steps of the half: row l32, chunk (2 s' + hi) ^ ((l32/2)%4)
    uint32_t aoff[4];
#pragma unroll
    for (int sp = 0; sp < 4; ++sp)
        aoff[sp] = (uint32_t)l32 * 128 + (uint32_t)(((2 * sp + hi) ^ ((l32 >> 1) & 3)) * 16);
    int stage = 0;
    for (int g = 0; g < G; ++g) {
        // two groups ahead; the stage it overwrites was last read in group g-1, which every
        // wave left before the barrier at its end
        int nstage = stage + 2;
        nstage = nstage >= NSTAGE ? nstage - NSTAGE : nstage;
        issue_group(g + 2, nstage);

        const uint32_t abase = a_ring + (uint32_t)stage * A_STAGE;
        const uint32_t bbase = b_ring + (uint32_t)stage * B_STAGE;
        // this group's packed words, steps and zero points
        u32x4 braw[2][2];
        braw[0][0] = lds_read16(bbase + lane16);
        braw[0][1] = lds_read16_off<1024>(bbase + lane16);
        braw[1][0] = lds_read16_off<2048>(bbase + lane16);
        braw[1][1] = lds_read16_off<3072>(bbase + lane16);
        uint32_t sraw[2], zraw[2];
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            sraw[b] = lds_read4(bbase + B_SC + 4 * (32 * b + l32));
            zraw[b] = lds_read4(bbase + B_ZP + 4 * (16 * b + (l32 >> 1)));
        }
        u32x4 a[4];
        a[0] = lds_read16_off<0>(abase + aoff[0]);
        a[1] = lds_read16_off<8192>(abase + aoff[0]);
        a[2] = lds_read16_off<16384>(abase + aoff[0]);
        a[3] = lds_read16_off<24576>(abase + aoff[0]);
        asm volatile("s_waitcnt lgkmcnt(0)"
                     : "+v"(braw[0][0]), "+v"(braw[0][1]), "+v"(braw[1][0]), "+v"(braw[1][1]),
                       "+v"(sraw[0]), "+v"(sraw[1]), "+v"(zraw[0]), "+v"(zraw[1]), "+v"(a[0]),
                       "+v"(a[1]), "+v"(a[2]), "+v"(a[3]));
        half2_t s2[2], zA[2], zB[2];
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            const half_t sh = __builtin_bit_cast(half_t, (uint16_t)sraw[b]);
            s2[b] = half2_t{sh, sh};
            const uint32_t z = (zraw[b] >> ((l32 & 1) * 4)) & 0xFu;
            zA[b] = __builtin_bit_cast(half2_t, 0x64006400u | (z * 0x00010001u));
            zB[b] = __builtin_bit_cast(half2_t, 0x54005400u | (z * 0x00100010u));
        }

#pragma unroll
        for (int s = 0; s < 8; ++s) {
            const int j = s >> 1, h = s & 1;
            // fragments of the next step are requested before this step's MFMAs
            u32x4 an[4];
            if (s < 7) {
                const uint32_t ad = abase + aoff[(s + 1) & 3] + ((s + 1) >> 2) * 4096;
                an[0] = lds_read16_off<0>(ad);
                an[1] = lds_read16_off<8192>(ad);
                an[2] = lds_read16_off<16384>(ad);
                an[3] = lds_read16_off<24576>(ad);
            }
            half8_t bf[2];
#pragma unroll
            for (int b = 0; b < 2; ++b)
                bf[b] = dequant_word(word_of(braw[b][h], j), kc, zA[b], zB[b], s2[b]);
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int b = 0; b < 2; ++b)
                    acc[i][b] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8_t, a[i]),
                                                                       bf[b], acc[i][b], 0, 0, 0);
            if (s < 7) {
                lds_wait(an[0], an[1], an[2], an[3]);
#pragma unroll
                for (int i = 0; i < 4; ++i) a[i] = an[i];
            }
        }

        // group g+1 has landed once only the loads of group g+2 are outstanding
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(LOADS_PER_GROUP) : "memory");
        __builtin_amdgcn_s_barrier();
        stage = stage + 1 == NSTAGE ? 0 : stage + 1;
    }
    // drain the two harmless repeats before the LDS is released
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");

    // epilogue: accumulator v of tile (i, b) is y[m0 + 32 i + 8 (v/4) + 4 hi + v%4][16 nt0 + 32 b + l32]
#pragma unroll
    for (int b = 0; b < 2; ++b) {
        const int n = (nt0 + 2 * b) * 16 + l32;
        if (n >= N) continue;
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = m0 + 32 * i + 8 * (v >> 2) + 4 * hi + (v & 3);
                if (m < M) y[(size_t)m * N + n] = (half_t)acc[i][b][v];
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
    static bool attr_set = false;
    if (!attr_set) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(gemm_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES) != hipSuccess)
            return AWQ_ERR_HIP;
        attr_set = true;
    }
    gemm_kernel<<<grid, block, LDS_BYTES, stream>>>(
        (const half_t *)x, (const unsigned char *)qweight, (const unsigned char *)scales,
        (const unsigned char *)zeros, (half_t *)y, M, N, K, G);
    return awq_launch_status();
}
