// Decode path of awq_w4a16_linear (M <= 16) for gfx950.
//
// AWQ Sec. 4.2: generation is memory-bound and weight traffic dominates, so the
// 4-bit weights are streamed once and dequantized on the fly inside the
// matrix-vector kernel; nothing dequantized is written back to memory.  The same
// passage warns that dequantization (shift, AND, FMA per weight) costs more ALU
// work than the product it feeds; the scheme below brings it to 5 vector
// instructions per 8 weights.
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
// Dequantization.  The nibble order of a word makes
//   (w >> {0,8}) & 0x000F000F | 0x64006400  the half pair (1024+q, 1024+q')  and
//   (w >> {0,8}) & 0x00F000F0 | 0x54005400  the half pair (  64+q,   64+q'),
// one v_and_or_b32 each.  These biased halves go to the matrix core as they are, and
// a second MFMA with the constant fragment -(1024+z), -(64+z) takes the bias and the
// zero point out again:  sum_k x_k (1024 + q_k) - sum_k x_k (1024 + z) = sum_k x_k (q_k - z).
// All products are exact in fp32; the two chains alternate so the running sum stays
// small.  The group's step is applied once per group in fp32.
//
// The partial sums of the waves are combined through LDS in a fixed order
// (deterministic output), rounded once to fp16 and stored.
#include "awq_common.h"

#include <stdlib.h>

namespace {

// The four constants of the expansion, held in registers.  They are made opaque to the
// optimizer so that (w & mask) | bits is selected as ONE v_and_or_b32 (mask in an SGPR,
// bits in a VGPR) instead of a v_and_b32 and a v_or_b32 with literal operands.
struct ExpandConsts {
    uint32_t mask_lo, mask_hi;   // 0x000F000F, 0x00F000F0  (SGPR)
    uint32_t magA, magB;         // 0x64006400, 0x54005400  (VGPR)
};

__device__ __forceinline__ ExpandConsts expand_consts()
{
    ExpandConsts k = {0x000F000Fu, 0x00F000F0u, 0x64006400u, 0x54005400u};
    asm("" : "+s"(k.mask_lo));
    asm("" : "+s"(k.mask_hi));
    asm("" : "+v"(k.magA));
    asm("" : "+v"(k.magB));
    return k;
}

// Eight codes of one packed word -> eight biased halves, in k order.
__device__ __forceinline__ half8_t biased_halves(uint32_t w, const ExpandConsts &k)
{
    const uint32_t w8 = w >> 8;
    uint4 t;
    t.x = (w & k.mask_lo) | k.magA;    // 1024 + (e0, e1)
    t.y = (w & k.mask_hi) | k.magB;    //   64 + (e2, e3)
    t.z = (w8 & k.mask_lo) | k.magA;   // 1024 + (e4, e5)
    t.w = (w8 & k.mask_hi) | k.magB;   //   64 + (e6, e7)
    return __builtin_bit_cast(half8_t, t);
}

// One batch of U consecutive tiles (groups) of a wave, as loaded from global memory.  The
// tiles of a row block are contiguous along K, so the U loads differ by a constant 1 KB.
// The step and zero point are fetched with ONE 2-byte and ONE 1-byte load per lane for the
// whole batch: lane (r, c) fetches those of row r of group base + min(c, U-1), turns them
// into the three per-tile constants, and tile u later takes them from lane r + 16u with
// cross-lane permutes.
// BITS = 4: a tile is 64 slots of 16 bytes; BITS = 3 (the INT3-g128 variant of Sec. 5): 64 slots
// of 12 bytes, three words per lane.
template <int BITS, int U>
struct TileBatch {
    uint32_t q[U][BITS];
    uint32_t s_raw, z_raw;
};

template <int BITS, int U>
__device__ __forceinline__ void load_batch(TileBatch<BITS, U> &b, const uint32_t *qt, const uint16_t *sc,
                                           const uint8_t *zp, int base)
{
    // the two small loads go first: loads return in order, and the first tile can only be
    // consumed once its step and zero point are there
    b.s_raw = sc[base * 16];
    b.z_raw = zp[base * 8];
    const uint32_t *p = qt + base * (64 * BITS);          // qt already points at this lane's slot
#pragma unroll
    for (int u = 0; u < U; ++u) {
        if (BITS == 4) {
            const uint4 v = *reinterpret_cast<const uint4 *>(p + u * 256);
            b.q[u][0] = v.x; b.q[u][1] = v.y; b.q[u][2] = v.z; b.q[u][BITS - 1] = v.w;
        } else {
#pragma unroll
            for (int i = 0; i < BITS; ++i) b.q[u][i] = p[u * 192 + i];
        }
    }
}

// INT3 slot: pair p = 0..14 of the 16 code pairs sits in word p/5 at bits [3f, 3f+3), f = p%5,
// of both halves; pair 15 in the top bits of the six halves.  (word >> 3f) & 0x00070007 is the
// pair as two fp16 subnormals q * 2^-24, which the matrix core takes at full precision.
__device__ __forceinline__ half8_t w3_halves(const uint32_t (&w)[3], uint32_t last_pair, int j)
{
    uint32_t t[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int p = 4 * j + i;
        t[i] = p < 15 ? ((w[p / 5] >> (3 * (p % 5))) & 0x00070007u) : last_pair;
    }
    return __builtin_bit_cast(half8_t, make_uint4(t[0], t[1], t[2], t[3]));
}

constexpr int GEMV_STAGE_MAX_M = 16;  // activations of up to this many rows go through LDS

// Decode kernel.
// U     = tiles (groups) per batch, a divisor of G: 1, 2 or 4.  A wave owns whole batches.
// PIPE  = double-buffer the batches (only worth its registers when a wave has several).
// MS > 0 (M <= MS <= 16): each wave copies the slice of x that its batch needs (MS rows x
//   U*128 halves; rows >= M repeat row M-1) into a private LDS area with one coalesced
//   16-byte load per lane for every 64/(16 U) rows, issued before the weight loads so that it returns first,
//   and then reads its A fragments from LDS.  No workgroup barrier is involved, so a wave
//   starts computing as soon as its own weights arrive.  With few rows most lanes of an A
//   fragment are duplicates, which is why this is cheaper than loading fragments from
//   global memory.
// MS == 0: A fragments are loaded straight from global memory (L2 hits); kept for reference,
//   the launcher stages every decode M (fragment loads at the point of use are round trips
//   to L2 in the middle of a batch).
//
// The workgroup has W = 2^logW waves; wave w owns batches [NB*w/W, NB*(w+1)/W), NB = G/U.
// Dynamic LDS: [W][MS rows x (U*256 + 16) bytes], then 16*M outputs x 16 wave slots of
// fp32 for the cross-wave reduction.
template <int BITS, int U, int MS, bool PIPE>
__global__ __launch_bounds__(1024, (MS >= 8 || (U == 4 && (PIPE || MS == 0 || (BITS == 3 && MS == 4)))) ? 4 : 6) void gemv_kernel(
    const half_t *__restrict__ x, const uint32_t *__restrict__ qweight,
    const uint16_t *__restrict__ scales, const uint8_t *__restrict__ zeros,
    half_t *y, int M, int N, int K, int G, int logW, const half_t *res)
{
    extern __shared__ __align__(16) unsigned char smem[];
    // all arguments are fetched in one round, before the first branch: left to itself the
    // compiler sinks the pointer loads below it, a second scalar-cache miss in front of the
    // first request of a kernel that lives for a few microseconds
    asm volatile("" ::"s"(x), "s"(qweight), "s"(scales), "s"(zeros), "s"(y), "s"(M), "s"(N), "s"(K), "s"(G),
                 "s"(logW), "s"(res));
    const ExpandConsts kc = expand_consts();
    constexpr bool STAGE = MS > 0;
    // staging: a row of the batch is U*16 lanes wide, so one 16-byte load per lane covers
    // RPP = 64 / (U*16) rows; NS passes cover the MS rows
    constexpr int LPR = U * 16, RPP = 64 / LPR;
    constexpr int NS = STAGE ? (MS + RPP - 1) / RPP : 1;
    constexpr int ROW_BYTES = U * 256 + 16;           // +16: rows land on different banks
    constexpr int WAVE_BYTES = MS * ROW_BYTES;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave-uniform
    const int W = 1 << logW;
    const int rb = blockIdx.x;
    const int r = lane & 15, c = lane >> 4;
    const int cu = c < U ? c : U - 1;                 // group of the batch this lane fetches meta for

    const int NB = G / U;
    const int g0 = ((NB * wave) >> logW) * U, g1 = ((NB * (wave + 1)) >> logW) * U;
    const uint32_t *qt = qweight + ((int64_t)rb * G * 64 + lane) * BITS;
    const uint16_t *sc = scales + (int64_t)rb * G * 16 + cu * 16 + r;
    const uint8_t *zp = zeros + (int64_t)rb * G * 8 + cu * 8 + (r >> 1);
    const int zshift = (r & 1) * 4;

    // A-operand row m = lane%16.  Rows >= M use row M-1 instead of zeros: row m of the MFMA
    // result depends on row m of A only, and rows >= M are never stored.
    const int mrow = r < M ? r : M - 1;
    unsigned char *xw = smem + (size_t)wave * WAVE_BYTES;                 // this wave's x slice
    const uint4 *xl = reinterpret_cast<const uint4 *>(xw + mrow * ROW_BYTES) + c;
    const uint4 *xg = reinterpret_cast<const uint4 *>(x + (int64_t)mrow * K) + c;
    // staging source of this lane in pass i: row i*RPP + lane/LPR (clamped to M-1 for the load,
    // not stored when >= MS), 16-byte chunk lane%LPR of the batch
    const int srow = lane / LPR, schunk = lane % LPR;
    const uint4 *xstage = reinterpret_cast<const uint4 *>(x) + schunk;
    const int64_t K8 = (int64_t)K >> 3;
    auto stage_src = [&](int i, int g) -> const uint4 & {
        const int m = i * RPP + srow;
        return xstage[(int64_t)(m < M ? m : M - 1) * K8 + g * 16];
    };
    auto stage_store = [&](int i, const uint4 &v) {
        const int m = i * RPP + srow;
        if (MS % RPP == 0 || m < MS) reinterpret_cast<uint4 *>(xw + m * ROW_BYTES)[schunk] = v;
    };
    constexpr bool stager = STAGE;

    TileBatch<BITS, U> cur;
    uint4 xs[NS];
#pragma unroll
    for (int m = 0; m < NS; ++m) xs[m] = make_uint4(0, 0, 0, 0);
    if (g0 < g1) {
        if (stager) {                              // first: it must not wait for the weights
#pragma unroll
            for (int m = 0; m < NS; ++m) xs[m] = stage_src(m, g0);
        }
        load_batch<BITS, U>(cur, qt, sc, zp, g0);
    }

    floatx4 total = {0.f, 0.f, 0.f, 0.f};
    for (int base = g0; base < g1; base += U) {
        if (stager) {                              // LDS ops of one wave execute in order
#pragma unroll
            for (int m = 0; m < NS; ++m) stage_store(m, xs[m]);
        }
        // PIPE: the next batch is requested before this one is consumed
        TileBatch<BITS, U> nxt;
        const bool more = base + U < g1;
        if (PIPE && more) {
            if (stager) {
#pragma unroll
                for (int m = 0; m < NS; ++m) xs[m] = stage_src(m, base + U);
            }
            load_batch<BITS, U>(nxt, qt, sc, zp, base + U);
        }
        // constants of (group base + cu, row r), computed once per batch by their owner lane
        const uint32_t z = (cur.z_raw >> zshift) & 0xFu;
        const uint32_t own_nzA = 0xE400E400u | (z * 0x00010001u);      // -(1024 + z) twice
        const uint32_t own_nzB = 0xD400D400u | (z * 0x00100010u);      // -(  64 + z) twice
        const float own_sv = (float)__builtin_bit_cast(half_t, (uint16_t)cur.s_raw);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            uint4 xa[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                // k = 128g + 32j + 8c + 0..7 -> 16-byte chunk 16g + 4j (+c folded into xl/xg)
                xa[j] = STAGE ? xl[u * 16 + 4 * j] : xg[(base + u) * 16 + 4 * j];
            }
            const int src = r + 16 * u;
            const uint32_t nzA = __shfl(own_nzA, src);
            const uint32_t nzB = __shfl(own_nzB, src);
            const float sv = __shfl(own_sv, src);
            if (BITS == 4) {
                const half8_t nb = __builtin_bit_cast(half8_t, make_uint4(nzA, nzB, nzA, nzB));
                floatx4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const half8_t a = __builtin_bit_cast(half8_t, xa[j]);
                    const half8_t b = biased_halves(cur.q[u][j & (BITS - 1)], kc);
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, acc, 0, 0, 0);
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, nb, acc, 0, 0, 0);
                }
#pragma unroll
                for (int v = 0; v < 4; ++v) total[v] += sv * acc[v];
            } else {
                // codes as subnormals q * 2^-24; the zero point leaves in fp32 through
                // S = 2^-24 * sum_k x_k (a second chain against the constant code 1)
                const uint32_t w3[3] = {cur.q[u][0], cur.q[u][1], cur.q[u][2]};
                const uint32_t last = ((w3[0] >> 15) & 0x00010001u) | ((w3[1] >> 14) & 0x00020002u) |
                                      ((w3[2] >> 13) & 0x00040004u);
                const half8_t ones = __builtin_bit_cast(half8_t, make_uint4(0x00010001u, 0x00010001u, 0x00010001u, 0x00010001u));
                floatx4 acc = {0.f, 0.f, 0.f, 0.f}, xsum = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const half8_t a = __builtin_bit_cast(half8_t, xa[j]);
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, w3_halves(w3, last, j), acc, 0, 0, 0);
                    xsum = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, ones, xsum, 0, 0, 0);
                }
                const float zf = __shfl((float)z, src);
                const float s24 = sv * 16777216.f;
#pragma unroll
                for (int v = 0; v < 4; ++v) total[v] += s24 * (acc[v] - zf * xsum[v]);
            }
        }
        if (PIPE) {
            if (more) cur = nxt;
        } else if (more) {
            if (stager) {
#pragma unroll
                for (int m = 0; m < NS; ++m) xs[m] = stage_src(m, base + U);
            }
            load_batch<BITS, U>(cur, qt, sc, zp, base + U);
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
        for (int w = 0; w < 16; ++w) sum += (w < W) ? part[w] : 0.f;
        // `res` (may be y itself): a residual added in fp32 before the one rounding
        const int64_t at = (int64_t)(t >> 4) * N + rb * 16 + (t & 15);
        y[at] = (half_t)(res ? sum + (float)res[at] : sum);
    }
}

// log2 of the waves per workgroup: about four tiles per wave, 4..16 waves
int pick_log_waves(int G)
{
    static const int forced = awq_knob("AWQ_GEMV_WAVES", 0);
    if (forced == 1 || forced == 2 || forced == 4 || forced == 8 || forced == 16)
        return forced == 1 ? 0 : forced == 2 ? 1 : forced == 4 ? 2 : forced == 8 ? 3 : 4;
    if (G >= 64) return 4;
    if (G >= 24) return 3;
    return 2;
}

// tiles per batch: the largest of 4, 2, 1 that divides G
int pick_unroll(int G)
{
    static const int forced = awq_knob("AWQ_GEMV_UNROLL", 0);
    if ((forced == 1 || forced == 2 || forced == 4) && G % forced == 0) return forced;
    return G % 4 == 0 ? 4 : (G % 2 == 0 ? 2 : 1);
}

}  // namespace

namespace {

// one instantiation: raises its dynamic-LDS limit once if the launch needs more than 64 KB
template <int BITS, int U, int MS, bool PIPE>
int gemv_launch_one(dim3 grid, dim3 block, size_t lds, hipStream_t stream, const half_t *x,
                    const uint32_t *qweight, const uint16_t *scales, const uint8_t *zeros, half_t *y, int M,
                    int N, int K, int G, int logW, const half_t *res)
{
    static AwqOncePerDevice once;
    std::atomic<bool> &raised = once.here();
    if (lds > 64 * 1024 && !raised.load(std::memory_order_relaxed)) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(gemv_kernel<BITS, U, MS, PIPE>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess)
            return AWQ_ERR_HIP;
        raised.store(true, std::memory_order_relaxed);
    }
    gemv_kernel<BITS, U, MS, PIPE><<<grid, block, lds, stream>>>(x, qweight, scales, zeros, y, M, N, K, G, logW, res);
    return awq_launch_status();
}

template <int BITS>
int gemv_launch_bits(const void *x, const void *qweight, const void *scales, const void *zeros,
                     void *y, int M, int N, int K, hipStream_t stream, const void *res = nullptr)
{
    const int G = K / AWQ_GROUP;
    const int logW = pick_log_waves(G);
    const int W = 1 << logW;
    // every decode M stages its activations through LDS: 1, 2, 4, 8 or 16 rows per wave
    const int MS = M == 1 ? 1 : (M == 2 ? 2 : (M <= 4 ? 4 : (M <= 8 ? 8 : 16)));
    int U = pick_unroll(G);
    if (MS == 16 && U == 4) U = 2;                  // 16 waves x 16 rows x 4 groups would not fit in LDS
    const dim3 grid(N / 16), block(W * 64);
    const bool pipe = (G / U + W - 1) / W > 1;      // some wave has more than one batch
    // reduction area: 16*M outputs x 16 wave slots x 4 bytes, after the staging areas
    // (a lane parks four token rows at once: the area covers M rounded up to a multiple of 4)
    const size_t lds = (size_t)((M + 3) / 4 * 4) * 1024 + (size_t)W * MS * (U * 256 + 16);
    if (lds > (size_t)160 * 1024) return AWQ_ERR_BAD_SHAPE;
#define AWQ_GEMV_LAUNCH(UU, MM, PP)                                                                   \
    return gemv_launch_one<BITS, UU, MM, PP>(grid, block, lds, stream, (const half_t *)x,             \
                                             (const uint32_t *)qweight, (const uint16_t *)scales,     \
                                             (const uint8_t *)zeros, (half_t *)y, M, N, K, G, logW,   \
                                             (const half_t *)res)
#define AWQ_GEMV_ROWS(UU, PP)                                                               \
    switch (MS) {                                                                           \
    case 1: AWQ_GEMV_LAUNCH(UU, 1, PP);                                                     \
    case 2: AWQ_GEMV_LAUNCH(UU, 2, PP);                                                     \
    case 4: AWQ_GEMV_LAUNCH(UU, 4, PP);                                                     \
    case 8: AWQ_GEMV_LAUNCH(UU, 8, PP);                                                     \
    default: break;                                                                         \
    }
    switch (U) {
    case 1:
        if (pipe) { AWQ_GEMV_ROWS(1, true) AWQ_GEMV_LAUNCH(1, 16, true); }
        else { AWQ_GEMV_ROWS(1, false) AWQ_GEMV_LAUNCH(1, 16, false); }
    case 2:
        if (pipe) { AWQ_GEMV_ROWS(2, true) AWQ_GEMV_LAUNCH(2, 16, true); }
        else { AWQ_GEMV_ROWS(2, false) AWQ_GEMV_LAUNCH(2, 16, false); }
    default:                                        // U == 4: never with 16 rows
        if (pipe) { AWQ_GEMV_ROWS(4, true) }
        else { AWQ_GEMV_ROWS(4, false) }
    }
#undef AWQ_GEMV_ROWS
#undef AWQ_GEMV_LAUNCH
    return AWQ_ERR_BAD_SHAPE;
}

}  // namespace

// Host side of the decode path; arguments were validated by awq_w4a16_linear / awq_w3a16_linear.
int awq_gemv_launch(const void *x, const void *qweight, const void *scales, const void *zeros,
                    void *y, int M, int N, int K, hipStream_t stream)
{
    return gemv_launch_bits<4>(x, qweight, scales, zeros, y, M, N, K, stream);
}

int awq_gemv_launch_w3(const void *x, const void *qweight, const void *scales, const void *zeros,
                       void *y, int M, int N, int K, hipStream_t stream)
{
    return gemv_launch_bits<3>(x, qweight, scales, zeros, y, M, N, K, stream);
}

// the 4-bit decode launch with a residual [M,N] (may be y) added to the output
int awq_gemv_launch_residual(const void *x, const void *qweight, const void *scales, const void *zeros,
                             void *y, const void *res, int M, int N, int K, hipStream_t stream)
{
    return gemv_launch_bits<4>(x, qweight, scales, zeros, y, M, N, K, stream, res);
}
