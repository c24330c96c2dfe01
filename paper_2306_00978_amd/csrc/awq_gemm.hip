// Prefill path of awq_w4a16_linear (M > 16) for gfx950.
//
// AWQ Sec. 4.2: with 4-bit storage and 16-bit compute the dequantization has to
// sit inside the main loop of the matrix-matrix kernel (it cannot be moved to the
// epilogue as with W8A8), and dequantized weights are never written to memory.
//
// Mapping.  A workgroup computes a 128 (tokens) x 256 (out-features) tile of y with
// eight waves: four side by side along N (128 x 64 = 4 x 2 tiles of
// v_mfma_f32_32x32x16_f16, 128 fp32 accumulators per lane), each of them twice, the two
// copies sharing a SIMD and splitting K between them: of the eight MFMA steps of a
// quantization group (128 columns) one wave takes the even ones, the other the odd ones, and
// the two partial tiles are added through LDS at the end.  A single wave per SIMD cannot keep
// the matrix pipe busy (loop overhead, waits, the change of group all stall it); with two,
// one computes while the other does that work, and no weight is dequantized twice.  The
// 32x32x16 shape is chosen for its issue budget: one MFMA occupies the matrix pipe for 32
// cycles, and in that shadow the wave issues everything else (operand reads, dequantization).
//
// Operands.  Nothing is staged through registers on the way in: both operands are
// fetched with global_load_lds (memory -> LDS, 16 bytes per lane landing in lane order),
// two groups ahead of the one being computed, into a ring of three stages.
//   * x: one load instruction fetches 8 rows x 128 contiguous bytes (whole cache lines) and
//     lands as 8 LDS rows of 128 bytes.  Which 16-byte chunk of the row a lane fetches is
//     XOR-swizzled with the row index, so that the A fragment of any MFMA step (lane l: row
//     l%32, 16 bytes at columns 16 s + 8 (l/32)) is read back with one conflict-free
//     ds_read_b128.  All waves share the x tile (wave (n-quarter q, k-half h) loads row block
//     q, column half h of every group); one barrier per group.
//   * weights: the packed layout is already the B-operand layout.  For a block of 32
//     out-features (two 16-row tiles), lane l takes slot (l%16) + 16 (2h + l/32) of tile
//     (l%32)/16: its word j is the fragment of MFMA step 2 j + h, i.e. half h of a tile holds
//     exactly the steps of k-half h.  A wave loads and reads only its own half.
//   Each fragment word is expanded in registers to fp16 (q - z) * scale and feeds four
//   MFMAs (the four token blocks), so dequantization costs about three vector
//   instructions per MFMA.
// fp32 accumulation, one rounding to fp16 at the end.
#include "awq_common.h"

#include <type_traits>

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
constexpr int LOADS_PER_GROUP = 4 + 2 + 1;       // per wave

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

// Dequantization of one packed word (eight codes) to fp16 (q - z) * scale, k order, cut into
// 13 single-instruction steps so that the main loop can place them one by one in the issue
// shadow of the MFMAs:  (w & mask) | magic is 1024+q or 64+q as a half pair; subtracting
// 1024+z / 64+z is exact; one rounding in the multiplication by the step.
struct DqWord {
    uint32_t w, w8;
    uint32_t t[4];
};

template <int OP>
__device__ __forceinline__ void dq_step(DqWord &d, const DqConsts &k, half2_t zA, half2_t zB,
                                        half2_t s2)
{
    if (OP == 0) d.w8 = d.w >> 8;
    if (OP == 1) d.t[0] = (d.w & k.mask_lo) | k.magA;
    if (OP == 2) d.t[1] = (d.w & k.mask_hi) | k.magB;
    if (OP == 3) d.t[2] = (d.w8 & k.mask_lo) | k.magA;
    if (OP == 4) d.t[3] = (d.w8 & k.mask_hi) | k.magB;
    if (OP >= 5 && OP <= 8) {
        const int i = OP - 5;
        d.t[i] = __builtin_bit_cast(uint32_t, __builtin_bit_cast(half2_t, d.t[i]) - ((i & 1) ? zB : zA));
    }
    if (OP >= 9 && OP <= 12) {
        const int i = OP - 9;
        d.t[i] = __builtin_bit_cast(uint32_t, __builtin_bit_cast(half2_t, d.t[i]) * s2);
    }
}

// steps [26 SLOT / 8, 26 (SLOT + 1) / 8) of the 26 that dequantize the two words of an MFMA step
template <int SLOT>
__device__ __forceinline__ void dq_slice(DqWord (&d)[2], const DqConsts &k, const half2_t (&zA)[2],
                                         const half2_t (&zB)[2], const half2_t (&s2)[2])
{
#define AWQ_DQ_ONE(I)                                                                           \
    if ((I) >= 26 * SLOT / 8 && (I) < 26 * (SLOT + 1) / 8) {                                    \
        constexpr int b_ = (I) / 13, op_ = (I) % 13;                                            \
        dq_step<op_>(d[b_], k, zA[b_], zB[b_], s2[b_]);                                         \
    }
    AWQ_DQ_ONE(0) AWQ_DQ_ONE(1) AWQ_DQ_ONE(2) AWQ_DQ_ONE(3) AWQ_DQ_ONE(4) AWQ_DQ_ONE(5) AWQ_DQ_ONE(6)
    AWQ_DQ_ONE(7) AWQ_DQ_ONE(8) AWQ_DQ_ONE(9) AWQ_DQ_ONE(10) AWQ_DQ_ONE(11) AWQ_DQ_ONE(12)
    AWQ_DQ_ONE(13) AWQ_DQ_ONE(14) AWQ_DQ_ONE(15) AWQ_DQ_ONE(16) AWQ_DQ_ONE(17) AWQ_DQ_ONE(18)
    AWQ_DQ_ONE(19) AWQ_DQ_ONE(20) AWQ_DQ_ONE(21) AWQ_DQ_ONE(22) AWQ_DQ_ONE(23) AWQ_DQ_ONE(24)
    AWQ_DQ_ONE(25)
#undef AWQ_DQ_ONE
}

__device__ __forceinline__ half8_t dq_result(const DqWord &d)
{
    return __builtin_bit_cast(half8_t, make_uint4(d.t[0], d.t[1], d.t[2], d.t[3]));
}

__device__ __forceinline__ uint32_t word_of(const u32x4 &v, int j)
{
    return v[j];
}

// SPLIT: K is cut into `ksplit` ranges of whole groups, one workgroup per (tile, range); each
// writes its partial tile in fp32 to part[range][M][N] and a second kernel adds the ranges.  For
// a few hundred tokens there are far fewer tiles than CUs (ceil(M/128) * N/256), and a workgroup
// per tile would leave most of the chip idle while a handful of CUs walk all of K.
template <bool SPLIT>
__global__ __launch_bounds__(512, 1) void gemm_kernel(
    const half_t *__restrict__ x, const unsigned char *__restrict__ qweight,
    const unsigned char *__restrict__ scales, const unsigned char *__restrict__ zeros,
    half_t *__restrict__ y, int M, int N, int K, int G, int tiles_n, int tiles_total,
    float *__restrict__ part, int ksplit)
{
    extern __shared__ __align__(16) unsigned char smem[];
    // all arguments fetched in one round (otherwise one scalar-cache miss per first use)
    asm volatile("" ::"s"(x), "s"(qweight), "s"(scales), "s"(zeros), "s"(y), "s"(M), "s"(N), "s"(K), "s"(G),
                 "s"(tiles_n), "s"(tiles_total), "s"(part), "s"(ksplit));
    // Workgroups are handed to the eight XCDs round-robin by their linear id, and each XCD has
    // its own L2.  The tile a workgroup computes is therefore chosen so that an XCD gets a
    // contiguous range of tiles in token-block-major order: its workgroups then share a few x
    // row blocks and sweep the same weight groups at about the same time, which keeps the
    // operand traffic inside that L2.
    const int units_total = SPLIT ? tiles_total * ksplit : tiles_total;      // (tile, K range) pairs
    const int per_xcd = (units_total + 7) >> 3;
    const int unit = ((int)blockIdx.x & 7) * per_xcd + ((int)blockIdx.x >> 3);
    if (unit >= units_total) return;
    const int tile = SPLIT ? unit / ksplit : unit;
    const int ks = SPLIT ? unit - tile * ksplit : 0;
    // groups [gofs, gofs + GL) of the G of a row
    const int gofs = SPLIT ? (int)(((int64_t)G * ks) / ksplit) : 0;
    const int GL = SPLIT ? (int)(((int64_t)G * (ks + 1)) / ksplit) - gofs : G;
    const int tile_m = tile / tiles_n, tile_n = tile - tile_m * tiles_n;
    const DqConsts kc = dq_consts();
    const uint32_t lds0 = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)smem);
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // waves w and w+4 run on the same SIMD: they form a pair on the same 128 x 64 sub-tile
    const int nq = wave & 3;                                 // which 64 out-features
    const int kh = wave >> 2;                                // which MFMA steps: 2 t + kh
    const int l32 = lane & 31, hi = lane >> 5;
    const int m0 = tile_m * BM;
    const int NT = N >> 4;                                   // 16-row weight tiles in the matrix
    const int nt0 = tile_n * (BN / 16) + nq * 4;            // first of the pair's four tiles

    // ---- sources of this lane's memory->LDS loads (group 0), advanced by constant strides
    // x: the wave fetches rows 32 nq .. +32, columns 64 kh .. +64 of the group; load q (0..3)
    // covers rows 8 q .. +8 of them; lane l takes row 8 q + l/8 (rows >= M repeat row M-1) and
    // chunk (l%8) ^ f, f = ((row in block)/2)%8, and lands at chunk l%8: sixteen consecutive
    // rows then hold any given chunk in sixteen different bank groups
    const unsigned char *xsrc[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        int xr = m0 + 32 * nq + 8 * q + (lane >> 3);
        xr = xr < M ? xr : M - 1;
        const int chunk = (lane & 7) ^ (((8 * q + (lane >> 3)) >> 1) & 7);
        xsrc[q] = reinterpret_cast<const unsigned char *>(x) + ((size_t)xr * K + 8 * chunk) * 2 + kh * 128 +
                  (size_t)gofs * 256;
    }
    // weights: block b (32 out-features = tiles nt0+2b, nt0+2b+1), half kh
    const unsigned char *qsrc[2];
#pragma unroll
    for (int b = 0; b < 2; ++b) {
        int t = nt0 + 2 * b + (l32 >> 4);
        t = t < NT ? t : NT - 1;                             // ragged N: repeat the last tile
        qsrc[b] = qweight + ((size_t)t * G * 64 + (l32 & 15) + 16 * hi) * 16 + kh * 512 + (size_t)gofs * 1024;
    }
    // steps (fetched by the kh = 0 wave): lane -> block lane/32, row l32;
    // zero points (kh = 1 wave): lane < 32 -> block lane/16, byte lane%16
    const unsigned char *msrc;
    if (kh == 0) {
        int t = nt0 + 2 * hi + (l32 >> 4);
        t = t < NT ? t : NT - 1;
        msrc = scales + ((size_t)t * G * 16 + (l32 & 15)) * 2 + (size_t)gofs * 32;
    } else {
        int tz = nt0 + 2 * ((lane >> 4) & 1) + ((lane >> 3) & 1);
        tz = tz < NT ? tz : NT - 1;
        msrc = zeros + (size_t)tz * G * 8 + (lane & 7) + (size_t)gofs * 8;
    }

    const uint32_t a_ring = lds0;
    const uint32_t b_ring = lds0 + NSTAGE * A_STAGE + (uint32_t)nq * (NSTAGE * B_STAGE);

    // One of the 7 loads of a group (PIECE 0..3: x, 4..5: weights, 6: steps or zero points).
    // They are issued one at a time from the issue shadow of the MFMAs.
    auto issue_piece = [&](auto piece_tag, int g, int stage) {
        constexpr int PIECE = decltype(piece_tag)::value;
        g = g < GL ? g : GL - 1;                             // past the end: a harmless repeat
        if constexpr (PIECE < 4) {
            // LDS: [row block 4][column half 2][32 rows x 128 B]
            const uint32_t adst = a_ring + (uint32_t)stage * A_STAGE + (uint32_t)nq * 8192 + (uint32_t)kh * 4096;
            dma16(xsrc[PIECE] + (size_t)g * 256, adst + PIECE * 1024);
        } else {
            const uint32_t bdst = b_ring + (uint32_t)stage * B_STAGE;
            if constexpr (PIECE < 6) {
                constexpr int b = PIECE - 4;
                dma16(qsrc[b] + (size_t)g * 1024, bdst + (2 * b) * 1024 + (uint32_t)kh * 1024);
            } else if (kh == 0) {
                dma2(msrc + (size_t)g * 32, bdst + B_SC);
            } else {
                if (lane < 32) dma1(msrc + (size_t)g * 8, bdst + B_ZP);
            }
        }
    };
#define AWQ_PIECE(P, G_, ST_) issue_piece(std::integral_constant<int, (P)>{}, (G_), (ST_))
    auto issue_group = [&](int g, int stage) {
        AWQ_PIECE(0, g, stage); AWQ_PIECE(1, g, stage); AWQ_PIECE(2, g, stage); AWQ_PIECE(3, g, stage);
        AWQ_PIECE(4, g, stage); AWQ_PIECE(5, g, stage); AWQ_PIECE(6, g, stage);
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
    // byte offset of this lane's A fragment inside a row block for the wave's four steps
    // S = 2 t + kh of a group: column half S/4, row l32, chunk (2 (S%4) + hi) ^ ((l32/2)%8)
    uint32_t aoff[4];
#pragma unroll
    for (int t = 0; t < 4; ++t)
        aoff[t] = (uint32_t)(t >> 1) * 4096 + (uint32_t)l32 * 128 +
                  (uint32_t)(((4 * (t & 1) + 2 * kh + hi) ^ ((l32 >> 1) & 7)) * 16);

    // ---- what a wave holds in registers for the group it is computing
    u32x4 braw[2];               // packed words of its k-half: [block], word t = its step t
    half2_t s2[2], zA[2], zB[2]; // per block: step, 1024 + z, 64 + z (as half pairs)
    u32x4 a[4];                  // A fragments of the current step
    DqWord dq[2];                // dequantization in flight (current or next step)

    // request the packed words, steps, zero points and the first A fragments of a stage
    u32x4 nbraw[2], na[4];
    uint32_t nsraw[2], nzraw[2];
    auto read_group = [&](int st) {
        const uint32_t bb = b_ring + (uint32_t)st * B_STAGE;
        const uint32_t bk = bb + (uint32_t)kh * 1024 + lane16;
        const uint32_t ab = a_ring + (uint32_t)st * A_STAGE + aoff[0];
        nbraw[0] = lds_read16_off<0>(bk);
        nbraw[1] = lds_read16_off<2048>(bk);
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            nsraw[b] = lds_read4(bb + B_SC + 4 * (32 * b + l32));
            nzraw[b] = lds_read4(bb + B_ZP + 4 * (16 * b + (l32 >> 1)));
        }
        na[0] = lds_read16_off<0>(ab);
        na[1] = lds_read16_off<8192>(ab);
        na[2] = lds_read16_off<16384>(ab);
        na[3] = lds_read16_off<24576>(ab);
    };
    auto wait_group = [&]() {
        asm volatile("s_waitcnt lgkmcnt(0)"
                     : "+v"(nbraw[0]), "+v"(nbraw[1]), "+v"(nsraw[0]), "+v"(nsraw[1]), "+v"(nzraw[0]),
                       "+v"(nzraw[1]), "+v"(na[0]), "+v"(na[1]), "+v"(na[2]), "+v"(na[3]));
    };
    // the group's constants from what was read, and step 0 of its dequantization set up
    half2_t ns2[2], nzA[2], nzB[2];
    DqWord ndq[2];
    auto group_consts = [&]() {
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            const half_t sh = __builtin_bit_cast(half_t, (uint16_t)nsraw[b]);
            ns2[b] = half2_t{sh, sh};
            const uint32_t z = (nzraw[b] >> ((l32 & 1) * 4)) & 0xFu;
            nzA[b] = __builtin_bit_cast(half2_t, 0x64006400u | (z * 0x00010001u));
            nzB[b] = __builtin_bit_cast(half2_t, 0x54005400u | (z * 0x00100010u));
            ndq[b].w = nbraw[b][0];
        }
    };
    auto adopt_group = [&]() {
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            braw[b] = nbraw[b];
            s2[b] = ns2[b]; zA[b] = nzA[b]; zB[b] = nzB[b];
            dq[b] = ndq[b];
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) a[i] = na[i];
    };

    // group 0: nothing to overlap with yet
    read_group(0);
    wait_group();
    group_consts();
    dq_slice<0>(ndq, kc, nzA, nzB, ns2); dq_slice<1>(ndq, kc, nzA, nzB, ns2);
    dq_slice<2>(ndq, kc, nzA, nzB, ns2); dq_slice<3>(ndq, kc, nzA, nzB, ns2);
    dq_slice<4>(ndq, kc, nzA, nzB, ns2); dq_slice<5>(ndq, kc, nzA, nzB, ns2);
    dq_slice<6>(ndq, kc, nzA, nzB, ns2); dq_slice<7>(ndq, kc, nzA, nzB, ns2);
    adopt_group();

    // One MFMA and, in its issue shadow, EXTRA.  The scheduling barrier pins the interleaving.
#define AWQ_MFMA_SLOT(I, B, EXTRA)                                                                 \
    acc[I][B] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8_t, a[I]),          \
                                                       (B) ? bf1 : bf0, acc[I][B], 0, 0, 0);       \
    EXTRA;                                                                                         \
    __builtin_amdgcn_sched_barrier(0);

    int stage = 0;
    for (int g = 0; g < GL; ++g) {
        int nstage = stage + 1 == NSTAGE ? 0 : stage + 1;    // stage of group g+1
        int fstage = nstage + 1 == NSTAGE ? 0 : nstage + 1;  // stage to fill with group g+2; it was
                                                             // last read in group g-1, which every
                                                             // wave left before the previous barrier
        const uint32_t abase = a_ring + (uint32_t)stage * A_STAGE;
        // the wave's steps 0..2: every MFMA is followed by a slice of the dequantization of its
        // next step; the first four also by a fragment read of that step, later ones by a load
        // of group g+2
#pragma unroll
        for (int t = 0; t < 3; ++t) {
            const half8_t bf0 = dq_result(dq[0]), bf1 = dq_result(dq[1]);
            u32x4 an[4];
            const uint32_t ad = abase + aoff[t + 1];
#pragma unroll
            for (int b = 0; b < 2; ++b) dq[b].w = word_of(braw[b], t + 1);
            __builtin_amdgcn_sched_barrier(0);
            AWQ_MFMA_SLOT(0, 0, an[0] = lds_read16_off<0>(ad); dq_slice<0>(dq, kc, zA, zB, s2))
            AWQ_MFMA_SLOT(0, 1, an[1] = lds_read16_off<8192>(ad); dq_slice<1>(dq, kc, zA, zB, s2))
            AWQ_MFMA_SLOT(1, 0, an[2] = lds_read16_off<16384>(ad); dq_slice<2>(dq, kc, zA, zB, s2))
            AWQ_MFMA_SLOT(1, 1, an[3] = lds_read16_off<24576>(ad); dq_slice<3>(dq, kc, zA, zB, s2))
            AWQ_MFMA_SLOT(2, 0, if (t == 0) AWQ_PIECE(0, g + 2, fstage); if (t == 1) AWQ_PIECE(2, g + 2, fstage);
                                if (t == 2) AWQ_PIECE(4, g + 2, fstage);
                                dq_slice<4>(dq, kc, zA, zB, s2))
            AWQ_MFMA_SLOT(2, 1, if (t == 0) AWQ_PIECE(1, g + 2, fstage); if (t == 1) AWQ_PIECE(3, g + 2, fstage);
                                if (t == 2) AWQ_PIECE(5, g + 2, fstage);
                                dq_slice<5>(dq, kc, zA, zB, s2))
            AWQ_MFMA_SLOT(3, 0, if (t == 2) AWQ_PIECE(6, g + 2, fstage); dq_slice<6>(dq, kc, zA, zB, s2))
            AWQ_MFMA_SLOT(3, 1, dq_slice<7>(dq, kc, zA, zB, s2))
            lds_wait(an[0], an[1], an[2], an[3]);
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = an[i];
        }

        // group g+1 has landed once only the loads of group g+2 are outstanding; after the barrier
        // every wave's part of it is visible.  The wave's last step of this group has all its
        // operands in registers already: its MFMAs cover the reads and the set-up of group g+1.
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(LOADS_PER_GROUP) : "memory");
        __builtin_amdgcn_s_barrier();
        {
            const half8_t bf0 = dq_result(dq[0]), bf1 = dq_result(dq[1]);
            read_group(nstage);
            __builtin_amdgcn_sched_barrier(0);
            AWQ_MFMA_SLOT(0, 0, (void)0)
            AWQ_MFMA_SLOT(0, 1, (void)0)
            AWQ_MFMA_SLOT(1, 0, (void)0)
            AWQ_MFMA_SLOT(1, 1, (void)0)
            wait_group();
            group_consts();
            __builtin_amdgcn_sched_barrier(0);
            AWQ_MFMA_SLOT(2, 0, dq_slice<0>(ndq, kc, nzA, nzB, ns2); dq_slice<1>(ndq, kc, nzA, nzB, ns2))
            AWQ_MFMA_SLOT(2, 1, dq_slice<2>(ndq, kc, nzA, nzB, ns2); dq_slice<3>(ndq, kc, nzA, nzB, ns2))
            AWQ_MFMA_SLOT(3, 0, dq_slice<4>(ndq, kc, nzA, nzB, ns2); dq_slice<5>(ndq, kc, nzA, nzB, ns2))
            AWQ_MFMA_SLOT(3, 1, dq_slice<6>(ndq, kc, nzA, nzB, ns2); dq_slice<7>(ndq, kc, nzA, nzB, ns2))
            adopt_group();
        }
        stage = nstage;
    }
#undef AWQ_MFMA_SLOT
#undef AWQ_PIECE
    // drain the two harmless repeats; after the barrier nobody reads the rings any more
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();

    // The two waves of a pair hold partial sums of the same 128 x 64 sub-tile.  Wave kh keeps
    // token blocks 2 kh, 2 kh + 1 and hands the other two to its partner through the now idle
    // LDS: 64 accumulators per lane, stored as [wave][accumulator][lane] (consecutive lanes in
    // consecutive words).
    {
        float *xch = reinterpret_cast<float *>(smem);
        float *mine = xch + (size_t)wave * (64 * 64);
        const float *theirs = xch + (size_t)(wave ^ 4) * (64 * 64);
#pragma unroll
        for (int ii = 0; ii < 2; ++ii)
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    // the block this wave gives away: kh = 0 gives 2, 3; kh = 1 gives 0, 1
                    const float give = kh ? acc[ii][b][v] : acc[2 + ii][b][v];
                    mine[((ii * 2 + b) * 16 + v) * 64 + lane] = give;
                }
        __syncthreads();
#pragma unroll
        for (int ii = 0; ii < 2; ++ii)
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const float got = theirs[((ii * 2 + b) * 16 + v) * 64 + lane];
                    if (kh) acc[2 + ii][b][v] += got;
                    else acc[ii][b][v] += got;
                }
        __syncthreads();
    }

    if (SPLIT) {
        // partial sums leave in fp32, 32 consecutive columns per half-wave and accumulator
        float *dst = part + (size_t)ks * M * N;
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int ii = 0; ii < 2; ++ii)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int m = m0 + 64 * kh + 32 * ii + 8 * (v >> 2) + 4 * hi + (v & 3);
                    const int n = nt0 * 16 + 32 * b + l32;
                    const float val = kh ? acc[2 + ii][b][v] : acc[ii][b][v];
                    if (m < M && n < N) dst[(size_t)m * N + n] = val;
                }
        return;
    }
    // Epilogue.  Accumulator v of tile (i, b) is y[m0 + 32 i + 8 (v/4) + 4 hi + v%4][16 nt0 + 32 b
    // + l32]: a lane holds single columns, which would leave as 2-byte stores.  Each wave turns
    // its 64 x 64 part around through its own 9 KB of LDS (rows of 128 + 16 bytes: the padding
    // spreads the banks) and stores 16 bytes per lane, 8 rows x 128 contiguous bytes per
    // instruction.
    {
        constexpr int ROWB = 144;
        unsigned char *mine = smem + (size_t)wave * (64 * ROWB);
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int ii = 0; ii < 2; ++ii)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int row = 32 * ii + 8 * (v >> 2) + 4 * hi + (v & 3);
                    const float val = kh ? acc[2 + ii][b][v] : acc[ii][b][v];
                    *reinterpret_cast<half_t *>(mine + row * ROWB + (32 * b + l32) * 2) = (half_t)val;
                }
        // wave-private area: the compiler orders these LDS reads after the writes above
        const int n = nt0 * 16 + (lane & 7) * 8;
#pragma unroll
        for (int it = 0; it < 8; ++it) {
            const int row = it * 8 + (lane >> 3);
            const uint4 v = *reinterpret_cast<const uint4 *>(mine + row * ROWB + (lane & 7) * 16);
            const int m = m0 + 64 * kh + row;
            if (m < M && n < N) *reinterpret_cast<uint4 *>(y + (size_t)m * N + n) = v;
        }
    }
}

// y = fp16(sum over the K ranges of the fp32 partial tiles), four outputs per thread
__global__ __launch_bounds__(256) void gemm_reduce_kernel(const float4 *__restrict__ part, uint2 *__restrict__ y,
                                                          int64_t quads, int ksplit)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= quads) return;
    float4 a = part[i];
    for (int k = 1; k < ksplit; ++k) {
        const float4 b = part[(int64_t)k * quads + i];
        a.x += b.x; a.y += b.y; a.z += b.z; a.w += b.w;
    }
    const half2_t lo = {(half_t)a.x, (half_t)a.y}, hi = {(half_t)a.z, (half_t)a.w};
    y[i] = make_uint2(__builtin_bit_cast(uint32_t, lo), __builtin_bit_cast(uint32_t, hi));
}

}  // namespace

// How many K ranges the prefill launch of this shape is cut into when a workspace is given: the
// count (1..8, at least four groups per range) with the smallest estimated time.  A workgroup
// takes about 4 us + 1.4 us per group, workgroups run in rounds of 256 (one per CU), and the
// second kernel moves (ranges + 1/2) * M * N * 4 bytes at about 3.5 TB/s after a launch of
// 2.5 us -- figures measured on the three Llama-2-7B shapes at 160..2048 tokens.  Cutting K pays
// while the tiles (ceil(M/128) * N/256) are fewer than the CUs, or just over a multiple of them.
int awq_gemm_ksplit(int M, int N, int K, double *estimate_us)
{
    const int G = K / AWQ_GROUP;
    const int64_t tiles = (int64_t)((N + BN - 1) / BN) * ((M + BM - 1) / BM);
    int best = 1;
    double best_us = 0.0;
    for (int ks = 1; ks <= 8 && (ks == 1 || G / ks >= 4); ++ks) {
        const double rounds = (double)((tiles * ks + 255) / 256);
        const double gl = (double)((G + ks - 1) / ks);
        double us = rounds * (4.0 + 1.4 * gl);
        if (ks > 1) us += 2.5 + (ks + 0.5) * (double)M * (double)N * 4.0 / 3.5e6;
        if (ks == 1 || us < 0.95 * best_us) {       // a split has to win by a margin
            best = ks;
            best_us = us;
        }
    }
    if (estimate_us) *estimate_us = best_us;
    return best;
}

namespace {

template <bool SPLIT>
int gemm_launch_any(const void *x, const void *qweight, const void *scales, const void *zeros,
                    void *y, int M, int N, int K, float *part, int ksplit, hipStream_t stream)
{
    const int G = K / AWQ_GROUP;
    const int tiles_n = (N + BN - 1) / BN;
    const int64_t tiles_total = (int64_t)tiles_n * ((M + BM - 1) / BM);
    if (tiles_total * ksplit > (1 << 30)) return AWQ_ERR_BAD_SHAPE;
    const dim3 grid((unsigned)((tiles_total * ksplit + 7) / 8 * 8)), block(512);
    static AwqOncePerDevice once;
    std::atomic<bool> &attr_set = once.here();
    if (!attr_set.load(std::memory_order_relaxed)) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(gemm_kernel<SPLIT>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES) != hipSuccess)
            return AWQ_ERR_HIP;
        attr_set.store(true, std::memory_order_relaxed);
    }
    gemm_kernel<SPLIT><<<grid, block, LDS_BYTES, stream>>>(
        (const half_t *)x, (const unsigned char *)qweight, (const unsigned char *)scales,
        (const unsigned char *)zeros, (half_t *)y, M, N, K, G, tiles_n, (int)tiles_total, part, ksplit);
    return awq_launch_status();
}

}  // namespace

// Host side of the prefill path; arguments were validated by awq_w4a16_linear.
int awq_gemm_launch(const void *x, const void *qweight, const void *scales, const void *zeros,
                    void *y, int M, int N, int K, hipStream_t stream)
{
    return gemm_launch_any<false>(x, qweight, scales, zeros, y, M, N, K, nullptr, 1, stream);
}

// The same with K cut into awq_gemm_ksplit() ranges; part: ksplit * M * N floats, 16-byte aligned.
int awq_gemm_launch_split(const void *x, const void *qweight, const void *scales, const void *zeros,
                          void *y, int M, int N, int K, void *part, int ksplit, hipStream_t stream)
{
    int st = gemm_launch_any<true>(x, qweight, scales, zeros, y, M, N, K, (float *)part, ksplit, stream);
    if (st != AWQ_OK) return st;
    const int64_t quads = (int64_t)M * N / 4;
    gemm_reduce_kernel<<<dim3((unsigned)((quads + 255) / 256)), dim3(256), 0, stream>>>(
        (const float4 *)part, (uint2 *)y, quads, ksplit);
    return awq_launch_status();
}
