// Streaming decode kernel of awq_w4a16_linear / awq_w4a16_linear_multi (M <= 16) for gfx950.
//
// AWQ Sec. 4.2: generation is memory-bound, the weights are the traffic, and each
// decode kernel is so short that launch overhead is comparable to its run time;
// the paper's answer is on-the-fly dequantization inside the matrix-vector kernel
// plus kernel fusion (e.g. one kernel for the Q, K and V projections).  This kernel
// does both: it dequantizes in registers, and one launch can run a list of
// independent linears (a "grouped" launch), each on its own share of the grid.
//
// Work decomposition of one linear (W[N,K], G = K/128 groups, tiles of 16 rows x 128
// columns = 1 KB, all tiles of a 16-row block contiguous along K):
//   * a batch is four consecutive tiles of one row block (4 KB) plus their 128 B of
//     steps and 32 B of zero points; NBT = ceil(G/4) batches per row block;
//   * a workgroup has W = KS * RW waves: wave w works on K-slice ks = w % KS (a
//     contiguous range of batches, the same for its whole life) of row block
//     ri = w / KS of the RW row blocks the workgroup handles per iteration, for
//     `iters` iterations over consecutive row blocks.  The jobs (iteration, batch) of a
//     wave form one flat pipeline.
//
// Memory pipeline.  Weights never pass through registers on their way in: every job is
// fetched with global_load_lds (HBM -> LDS directly, 16 bytes per lane, a 1 KB tile lands
// contiguously) into one of STAGES private ring slots of the wave, STAGES-1 jobs ahead of
// the job being consumed.  That keeps (STAGES-1) * 4.2 KB in flight per wave at no
// register cost; a job is read back with one ds_read_b128 per tile when its turn comes.
// vmcnt counts these loads in order, so "at most 6*(STAGES-1) outstanding" means the
// oldest job has landed.  The ring is private to a wave: no barrier is involved.
//
// Activations.  x stays in registers for the whole kernel.  A-operand row r of the MFMA
// is token (r % Mpad) of "slot" r / Mpad (Mpad = M rounded up to a power of two), and
// slot s carries the activations of batch b0 + s of the wave's K-slice.  A tile of batch
// b0 + s therefore yields its valid sums in output rows s * Mpad + m; the other rows are
// finite garbage and are masked out when the batch is added to the running sums.  With
// M = 1 one wave covers 16 batches (K = 8192) with 64 registers and no per-tile
// activation traffic of any kind.
//
// Arithmetic per tile.  (w & 0x000F000F) and (w & 0x00F000F0) read as fp16 pairs are the
// SUBNORMAL halves q * 2^-24 and q * 2^-20: exact, no bias, one v_and_b32 per pair.  The matrix
// core of gfx950 takes subnormal inputs at full precision, so the codes go to
// v_mfma_f32_16x16x32_f16 as they are.  The 2^-20 positions are evened out on the activation
// side (those fragment elements are multiplied by 2^-4 once, when the fragments are loaded),
// and the zero point is taken out per tile in fp32:
//     sum_k x_k (q_k - z) = acc - z * S,   S = sum_k x_k  (once per wave, by an MFMA of the
// fragments against the constant code 1).  The step and the common factor 2^24 are applied
// once per group in fp32.  Every product and, for integer-valued data, every sum is exact.
//
// Output.  The running sums are folded across slots with cross-lane permutes; waves that
// share a row block (KS > 1) meet in LDS (one barrier per iteration), are added in a
// fixed order (deterministic), rounded once to fp16 and stored.
//
// Start-up.  A launch lives for 10-25 us, so the microsecond before the first weight request
// counts: the linear's entry of the kernel-argument block is fetched with vector loads (lane l
// takes entry l, a ballot and readlanes pick the workgroup's), and the activation fragments
// with unconditional loads from clamped addresses, so that everything is in flight in two
// rounds instead of a chain of misses.
//
// FUSED form (Sec. 4.2, fusion of the small operators around a linear).  The activations of a
// wave are already in its registers, so an RMS normalisation in front of the linear is a sum of
// squares over them (lanes of one token by shuffles, waves that split K through LDS) and one
// rescaling pass with mixed-precision fma instructions; a residual is added to the fp32 sums
// right before the one rounding to fp16.  Neither needs a launch or a pass over memory.
#include "awq_common.h"
#include "awq_gemv_stream.h"

#include <stdlib.h>
#include <algorithm>
#include <cmath>

namespace {

typedef __attribute__((address_space(3))) void lds_void_t;
typedef const __attribute__((address_space(1))) void gbl_void_t;

// Ring slot of one job: 4 tiles, 256 B of steps, 128 B of zero points.  BITS = 4: tiles of 1 KB;
// BITS = 3 (INT3-g128 variant, Sec. 5): tiles of 768 B, the four of a batch are 3 KB contiguous
// and arrive with three full-wave 16-byte loads.
template <int BITS> struct Slot {
    static constexpr int TILE = BITS == 4 ? 1024 : 768;
    static constexpr int SC = 4 * TILE, ZP = SC + 256, BYTES = ZP + 128;
    static constexpr int LOADS = (BITS == 4 ? 4 : 3) + 2;
};

// HBM -> LDS without a register in between.  Lane l's 16 bytes land at lds + OFF + 16 l (OFF is
// added to the global address as well); 2- and 1-byte loads land zero-extended at lds + 4 l.
template <int OFF>
__device__ __forceinline__ void dma16_to_lds(const void *g, uint32_t lds_addr)
{
    __builtin_amdgcn_global_load_lds((gbl_void_t *)(uintptr_t)g, (lds_void_t *)(uintptr_t)lds_addr,
                                     16, OFF, 0);
}
__device__ __forceinline__ void dma2_to_lds(const void *g, uint32_t lds_addr)
{
    __builtin_amdgcn_global_load_lds((gbl_void_t *)(uintptr_t)g, (lds_void_t *)(uintptr_t)lds_addr,
                                     2, 0, 0);
}
__device__ __forceinline__ void dma1_to_lds(const void *g, uint32_t lds_addr)
{
    __builtin_amdgcn_global_load_lds((gbl_void_t *)(uintptr_t)g, (lds_void_t *)(uintptr_t)lds_addr,
                                     1, 0, 0);
}

// What a wave reads back from a landed ring slot: the four tiles (one 16-byte word group
// per lane and tile) and, for its row r, the four steps (fp16 bits) and the four zero-point
// bytes (rows 2*(r/2) and 2*(r/2)+1 in the low and high nibble).
struct Landed {
    uint4 q[4];          // BITS = 3: .x .y .z are the three words of the lane's slot
    uint4 s, z;
};

// Workgroup barrier for data exchanged through LDS with ordinary ds_write / ds_read: waits for
// this wave's LDS operations only.  __syncthreads() also waits for every outstanding memory
// request, and here those are the weight jobs on their way into the wave's private ring,
// which no other wave reads: waiting for them at each meeting of the waves would undo the
// prefetch.
__device__ __forceinline__ void lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

template <int PENDING>
__device__ __forceinline__ void wait_loads()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(PENDING) : "memory");
}

// BITS = 3: lane l's 12 bytes of tile u sit at 768 u + 12 l (4-byte aligned): three ds_read_b32
__device__ __forceinline__ void read_slot_w3(Landed &d, uint32_t tile_addr, uint32_t sc_addr,
                                             uint32_t zp_addr)
{
    asm volatile(
        "ds_read_b128 %12, %15 offset:3072\n"
        "ds_read_b128 %13, %16 offset:3328\n"
        "ds_read_b32 %0, %14\n"
        "ds_read_b32 %1, %14 offset:4\n"
        "ds_read_b32 %2, %14 offset:8\n"
        "ds_read_b32 %3, %14 offset:768\n"
        "ds_read_b32 %4, %14 offset:772\n"
        "ds_read_b32 %5, %14 offset:776\n"
        "ds_read_b32 %6, %14 offset:1536\n"
        "ds_read_b32 %7, %14 offset:1540\n"
        "ds_read_b32 %8, %14 offset:1544\n"
        "ds_read_b32 %9, %14 offset:2304\n"
        "ds_read_b32 %10, %14 offset:2308\n"
        "ds_read_b32 %11, %14 offset:2312\n"
        "s_waitcnt lgkmcnt(0)"
        : "=&v"(d.q[0].x), "=&v"(d.q[0].y), "=&v"(d.q[0].z), "=&v"(d.q[1].x), "=&v"(d.q[1].y), "=&v"(d.q[1].z),
          "=&v"(d.q[2].x), "=&v"(d.q[2].y), "=&v"(d.q[2].z), "=&v"(d.q[3].x), "=&v"(d.q[3].y), "=&v"(d.q[3].z),
          "=&v"(d.s), "=&v"(d.z)
        : "v"(tile_addr), "v"(sc_addr), "v"(zp_addr)
        : "memory");
}

__device__ __forceinline__ void read_slot(Landed &d, uint32_t tile_addr, uint32_t sc_addr,
                                          uint32_t zp_addr)
{
    asm volatile(
        "ds_read_b128 %4, %7 offset:4096\n"
        "ds_read_b128 %5, %8 offset:4352\n"
        "ds_read_b128 %0, %6\n"
        "ds_read_b128 %1, %6 offset:1024\n"
        "ds_read_b128 %2, %6 offset:2048\n"
        "ds_read_b128 %3, %6 offset:3072\n"
        "s_waitcnt lgkmcnt(0)"
        : "=&v"(d.q[0]), "=&v"(d.q[1]), "=&v"(d.q[2]), "=&v"(d.q[3]), "=&v"(d.s), "=&v"(d.z)
        : "v"(tile_addr), "v"(sc_addr), "v"(zp_addr)
        : "memory");
}

// (w & mask) as fp16 pairs: q * 2^-24 for the low-nibble mask, q * 2^-20 for the high one
__device__ __forceinline__ half8_t subnormal_halves(uint32_t w, uint32_t mask_lo, uint32_t mask_hi)
{
    const uint32_t w8 = w >> 8;
    return __builtin_bit_cast(half8_t, make_uint4(w & mask_lo, w & mask_hi, w8 & mask_lo, w8 & mask_hi));
}

// One batch (four tiles) against the register-resident activation fragments xa[4u + j];
// xsum[u] is 2^-24 * (sum of the activations of tile u) per output row.  Returns, per lane,
// the four partial sums of output rows 4c + v for column r.
__device__ __forceinline__ floatx4 consume_batch(const Landed &b, const uint4 (&xa)[16],
                                                 const floatx4 (&xsum)[4], uint32_t mask_lo,
                                                 uint32_t mask_hi, int zshift)
{
    floatx4 bacc = {0.f, 0.f, 0.f, 0.f};
    const uint32_t sraw[4] = {b.s.x, b.s.y, b.s.z, b.s.w};
    const uint32_t zraw[4] = {b.z.x, b.z.y, b.z.z, b.z.w};
#pragma unroll
    for (int u = 0; u < 4; u += 2) {
        // two tiles at a time: their accumulation chains interleave in the matrix pipe
        const uint32_t wa[4] = {b.q[u].x, b.q[u].y, b.q[u].z, b.q[u].w};
        const uint32_t wb[4] = {b.q[u + 1].x, b.q[u + 1].y, b.q[u + 1].z, b.q[u + 1].w};
        floatx4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            acc0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8_t, xa[4 * u + j]),
                                                          subnormal_halves(wa[j], mask_lo, mask_hi), acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8_t, xa[4 * u + 4 + j]),
                                                          subnormal_halves(wb[j], mask_lo, mask_hi), acc1, 0, 0, 0);
        }
        const float z0 = (float)((zraw[u] >> zshift) & 0xFu), z1 = (float)((zraw[u + 1] >> zshift) & 0xFu);
        const float s0 = (float)__builtin_bit_cast(half_t, (uint16_t)sraw[u]) * 16777216.f;
        const float s1 = (float)__builtin_bit_cast(half_t, (uint16_t)sraw[u + 1]) * 16777216.f;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            bacc[v] += s0 * (acc0[v] - z0 * xsum[u][v]);
            bacc[v] += s1 * (acc1[v] - z1 * xsum[u + 1][v]);
        }
    }
    return bacc;
}

// INT3: pair p = 4 j + i of a slot (MFMA step j, halves 2i, 2i+1) sits in word p/5 at field
// f = p%5 (bits [3f, 3f+3) of both halves); pair 15 in the top bits of the six halves.  Fields 0..2
// are taken where they are, fields 3, 4 after one shift by 9: the pair then reads as the fp16
// subnormals q * 2^(3 cls - 24), cls = w3_cls(p), and the activation it meets carries 2^(-3 cls).
__host__ __device__ constexpr int w3_cls(int p) { return p == 15 ? 0 : ((p % 5) % 3); }

__device__ __forceinline__ half8_t w3_subnormal_halves(const uint32_t (&w)[3], const uint32_t (&w9)[3],
                                                       uint32_t last_pair, int j)
{
    uint32_t t[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int p = 4 * j + i, f = p % 5;
        const uint32_t mask = 0x00070007u << (3 * (f % 3));
        t[i] = p == 15 ? last_pair : ((f < 3 ? w[p / 5] : w9[p / 5]) & mask);
    }
    return __builtin_bit_cast(half8_t, make_uint4(t[0], t[1], t[2], t[3]));
}

__device__ __forceinline__ floatx4 consume_batch_w3(const Landed &b, const uint4 (&xa)[16],
                                                    const floatx4 (&xsum)[4], int zshift)
{
    floatx4 bacc = {0.f, 0.f, 0.f, 0.f};
    const uint32_t sraw[4] = {b.s.x, b.s.y, b.s.z, b.s.w};
    const uint32_t zraw[4] = {b.z.x, b.z.y, b.z.z, b.z.w};
#pragma unroll
    for (int u = 0; u < 4; u += 2) {
        const uint32_t wa[3] = {b.q[u].x, b.q[u].y, b.q[u].z};
        const uint32_t wb[3] = {b.q[u + 1].x, b.q[u + 1].y, b.q[u + 1].z};
        const uint32_t wa9[3] = {wa[0] >> 9, wa[1] >> 9, wa[2] >> 9};
        const uint32_t wb9[3] = {wb[0] >> 9, wb[1] >> 9, wb[2] >> 9};
        const uint32_t la = ((wa[0] >> 15) & 0x00010001u) | ((wa[1] >> 14) & 0x00020002u) | ((wa[2] >> 13) & 0x00040004u);
        const uint32_t lb = ((wb[0] >> 15) & 0x00010001u) | ((wb[1] >> 14) & 0x00020002u) | ((wb[2] >> 13) & 0x00040004u);
        floatx4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            acc0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8_t, xa[4 * u + j]),
                                                          w3_subnormal_halves(wa, wa9, la, j), acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8_t, xa[4 * u + 4 + j]),
                                                          w3_subnormal_halves(wb, wb9, lb, j), acc1, 0, 0, 0);
        }
        const float z0 = (float)((zraw[u] >> zshift) & 0xFu), z1 = (float)((zraw[u + 1] >> zshift) & 0xFu);
        const float s0 = (float)__builtin_bit_cast(half_t, (uint16_t)sraw[u]) * 16777216.f;
        const float s1 = (float)__builtin_bit_cast(half_t, (uint16_t)sraw[u + 1]) * 16777216.f;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            bacc[v] += s0 * (acc0[v] - z0 * xsum[u][v]);
            bacc[v] += s1 * (acc1[v] - z1 * xsum[u + 1][v]);
        }
    }
    return bacc;
}

// Mixed-precision helpers of the fused normalisation (fp16 operands taken from a packed pair,
// fp32 arithmetic, no separate conversions): acc + lo(h2)^2 + hi(h2)^2, and the pair
// fp16(lo(x2) * f * lo(w2)), fp16(hi(x2) * f * hi(w2)).
__device__ __forceinline__ float mix_sum_squares(uint32_t h2, float acc)
{
    asm("v_fma_mix_f32 %0, %1, %1, %0 op_sel_hi:[1,1,0]\n\t"
        "v_fma_mix_f32 %0, %1, %1, %0 op_sel:[1,1,0] op_sel_hi:[1,1,0]"
        : "+v"(acc)
        : "v"(h2));
    return acc;
}

__device__ __forceinline__ uint32_t mix_scale_pair(uint32_t x2, float f, uint32_t w2)
{
    float lo, hi;
    uint32_t out;
    asm("v_fma_mix_f32 %1, %3, %4, 0 op_sel_hi:[1,0,0]\n\t"
        "v_fma_mix_f32 %2, %3, %4, 0 op_sel:[1,0,0] op_sel_hi:[1,0,0]\n\t"
        "v_fma_mixlo_f16 %0, %1, %5, 0 op_sel_hi:[0,1,0]\n\t"
        "v_fma_mixhi_f16 %0, %2, %5, 0 op_sel:[0,1,0] op_sel_hi:[0,1,0]"
        : "=&v"(out), "=&v"(lo), "=&v"(hi)
        : "v"(x2), "v"(f), "v"(w2));
    return out;
}

// What a stage of a chained launch waits for before it may read its activations: a counter in
// global memory that every workgroup of the launch increments when it has finished the stage
// before, the value it has to reach, and the give-up flag of the launch.
struct ChainWait {
    const uint32_t *counter;      // nullptr: nothing to wait for
    uint32_t target;
    uint32_t *gave_up;            // set (never cleared here) by a workgroup whose wait ran out
    int spin_limit;
};

// The work of one workgroup of a grouped launch.  `ka` points at a launch table inside the
// kernel-argument block: int wg_begin[MAXP] at OFF_BEGIN, GemvProblem p[MAXP] at OFF_P and, FUSED,
// GemvFusedExtra e[MAXF] at OFF_E; `vwg` is the workgroup's index within that table's launch.
// CHAIN: the table is one stage of a chained launch (see chain_kernel); the first weight jobs are
// requested before the wait for the stage in front, the activations are read after it.  Returns
// false if that wait ran out (the workgroup then leaves the launch).
template <int STAGES, int BITS, bool FUSED, bool CHAIN, int OFF_BEGIN, int OFF_P, int OFF_E, int MAXP, int MAXF>
__device__ __forceinline__ bool stream_body(const unsigned char *ka, const int M, const int mlog, const int logW,
                                            const int vwg, unsigned char *smem, const ChainWait cw)
{
    constexpr int STAGE_BYTES = Slot<BITS>::BYTES, STAGE_SC = Slot<BITS>::SC, STAGE_ZP = Slot<BITS>::ZP;
    constexpr int TILE_BYTES = Slot<BITS>::TILE, LOADS_PER_JOB = Slot<BITS>::LOADS;
    uint32_t mask_lo = 0x000F000Fu, mask_hi = 0x00F000F0u;      // kept in SGPRs
    asm("" : "+s"(mask_lo));
    asm("" : "+s"(mask_hi));

    // Which linear of the list this workgroup belongs to, and that linear's entry.  Read through
    // the scalar cache this is a chain of dependent misses (table, then entry) in front of the
    // first weight request of every wave; instead lane l fetches wg_begin[l] and entry l of the
    // kernel-argument block with vector loads, all in flight together, and the wave picks its
    // entry with a ballot and readlanes: one memory round trip.  (Entries and table slots beyond
    // `count` hold INT_MAX / unused bytes; they lie inside the argument block.)
    typedef const __attribute__((address_space(1))) half_t gbl_half_t;
    typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
    typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
    typedef const __attribute__((address_space(1))) u32x2_t gbl_u32x2_t;
    typedef const __attribute__((address_space(1))) u32x4_t gbl_u32x4_t;
    GemvProblem P;
    gbl_half_t *px;                                     // activations and outputs of this linear,
    __attribute__((address_space(1))) half_t *py;       // known to the compiler as global memory
    int wg0;                                            // first workgroup of this linear
    gbl_half_t *ppre = nullptr, *pres = nullptr;        // FUSED: normalisation factors, residual
    float eps = 0.f;
    int pre_op = GEMV_PRE_NONE;
    {
        const int l = threadIdx.x & 63, le = l < MAXP ? l : MAXP - 1;
        typedef const __attribute__((address_space(1))) int gbl_int_t;
        const int begin = *(gbl_int_t *)(uintptr_t)(ka + OFF_BEGIN + 4 * le);
        gbl_u32x2_t *pe = (gbl_u32x2_t *)(uintptr_t)(ka + OFF_P + sizeof(GemvProblem) * le);
        uint32_t f[14];
#pragma unroll
        for (int d = 0; d < 7; ++d) {
            const u32x2_t t = pe[d];
            f[2 * d] = t.x;
            f[2 * d + 1] = t.y;
        }
        uint32_t fe[6] = {};
        if (FUSED) {
            const int lf = l < MAXF ? l : MAXF - 1;
            gbl_u32x2_t *ee = (gbl_u32x2_t *)(uintptr_t)(ka + OFF_E + sizeof(GemvFusedExtra) * lf);
#pragma unroll
            for (int d = 0; d < 3; ++d) {
                const u32x2_t t = ee[d];
                fe[2 * d] = t.x;
                fe[2 * d + 1] = t.y;
            }
        }
        const uint64_t mine = __ballot(l < MAXP && vwg >= begin);
        const int pi = __builtin_amdgcn_readfirstlane(__popcll(mine) - 1);     // wg_begin is ascending from 0
        uint32_t g[14];
#pragma unroll
        for (int d = 0; d < 14; ++d) g[d] = __builtin_amdgcn_readlane(f[d], pi);
        static_assert(sizeof(GemvProblem) == 56 && offsetof(GemvProblem, N) == 40, "entry layout");
        px = (gbl_half_t *)(uintptr_t)(((uint64_t)g[1] << 32) | g[0]);
        py = (__attribute__((address_space(1))) half_t *)(uintptr_t)(((uint64_t)g[9] << 32) | g[8]);
        P.x = nullptr;
        P.y = nullptr;
        P.q = reinterpret_cast<const uint4 *>(((uint64_t)g[3] << 32) | g[2]);
        P.sc = reinterpret_cast<const uint16_t *>(((uint64_t)g[5] << 32) | g[4]);
        P.zp = reinterpret_cast<const uint8_t *>(((uint64_t)g[7] << 32) | g[6]);
        P.N = (int)g[10];
        P.K = (int)g[11];
        P.plan = (int)g[12];
        P.nrb = (int)g[13];
        wg0 = __builtin_amdgcn_readlane(begin, pi);
        if (FUSED) {
            static_assert(sizeof(GemvFusedExtra) == 24, "layout");
            uint32_t ge[6];
#pragma unroll
            for (int d = 0; d < 6; ++d) ge[d] = __builtin_amdgcn_readlane(fe[d], pi);
            ppre = (gbl_half_t *)(uintptr_t)(((uint64_t)ge[1] << 32) | ge[0]);
            pres = (gbl_half_t *)(uintptr_t)(((uint64_t)ge[3] << 32) | ge[2]);
            eps = __builtin_bit_cast(float, ge[4]);
            pre_op = (int)ge[5];
        }
    }

    const int Mpad = 1 << mlog;
    const int K = P.K, N = P.N;
    const int G = K >> 7, NRB = P.nrb, NBT = (G + 3) >> 2;
    const int ksl = P.plan & 15, KS = 1 << ksl;
    const int W = 1 << logW, RW = W >> ksl;
    const int iters = P.plan >> 4;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int ks = wave & (KS - 1), ri = wave >> ksl;
    const int b0 = (NBT * ks) >> ksl, b1 = (NBT * (ks + 1)) >> ksl;      // 1..16/Mpad batches (host)
    const int unit = vwg - wg0;
    const int rb_wg = unit * iters * RW;                                 // first row block of the WG
    const int r = lane & 15, c = lane >> 4;
    const int zshift = (r & 1) * 4;

    // LDS: [W][STAGES] ring slots, then the cross-wave reduction area (two buffers)
    const uint32_t lds0 = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)smem);
    const uint32_t ring = lds0 + (uint32_t)wave * (STAGES * STAGE_BYTES);
    float *red = reinterpret_cast<float *>(smem + (size_t)W * STAGES * STAGE_BYTES);
    const int red_floats = W * Mpad * 16;           // [ri][ks][token][column]

    const unsigned char *qbase = reinterpret_cast<const unsigned char *>(P.q);
    const unsigned char *scbase = reinterpret_cast<const unsigned char *>(P.sc);
    const unsigned char *zpbase = reinterpret_cast<const unsigned char *>(P.zp);
    const uint32_t lane16 = (uint32_t)lane << 4;

    // per-lane parts of the source addresses: tile bytes; step of (row lane/4, group lane%4);
    // zero-point byte of (row pair lane/4, group lane%4)
    const uint32_t sc_lane = (uint32_t)(lane & 3) * 32 + (uint32_t)(lane >> 2) * 2;
    const uint32_t zp_lane = (uint32_t)(lane & 3) * 8 + (uint32_t)((lane >> 2) & 7);
    const bool ragged = (G & 3) != 0;

    // request one job: 4 tiles (all lanes, 16 B each), 64 steps (all lanes, 2 B each), 32
    // zero-point bytes (lanes 0..31).  Groups beyond G-1 (ragged last batch) re-read group
    // G-1; their activation fragments are zero, so they contribute nothing.
    auto issue = [&](int it, int b, int slot) {
        int rb = rb_wg + it * RW + ri;
        rb = rb < NRB ? rb : NRB - 1;                       // surplus waves redo the last block
        const size_t t0 = (size_t)rb * G + (size_t)b * 4;   // first tile of the batch
        const uint32_t dst = ring + (uint32_t)slot * STAGE_BYTES;
        const unsigned char *tq = qbase + t0 * TILE_BYTES, *ts = scbase + t0 * 32, *tz = zpbase + t0 * 8;
        if (!ragged || b * 4 + 4 <= G) {
            dma16_to_lds<0>(tq + lane16, dst);
            dma16_to_lds<1024>(tq + lane16, dst);
            dma16_to_lds<2048>(tq + lane16, dst);
            if (BITS == 4) dma16_to_lds<3072>(tq + lane16, dst);
            dma2_to_lds(ts + sc_lane, dst + STAGE_SC);
            if (lane < 32) dma1_to_lds(tz + zp_lane, dst + STAGE_ZP);
        } else {
            const int last = G - 1 - b * 4;                 // last valid group of this batch (0..2)
            if (BITS == 4) {
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    dma16_to_lds<0>(tq + ((size_t)min(u, last) << 10) + lane16, dst + u * 1024);
            } else {
                // the same three loads; a 16-byte chunk that belongs to a tile beyond the last
                // valid one re-reads that last tile instead (never past the end of the array)
#pragma unroll
                for (int i = 0; i < 3; ++i) {
                    const int ch = lane + 64 * i, tl = ch / 48, off = 16 * (ch - 48 * tl);
                    dma16_to_lds<0>(tq + min(tl, last) * 768 + off, dst + i * 1024);
                }
            }
            const int gl = min(lane & 3, last);
            dma2_to_lds(ts + gl * 32 + (lane >> 2) * 2, dst + STAGE_SC);
            if (lane < 32) dma1_to_lds(tz + gl * 8 + ((lane >> 2) & 7), dst + STAGE_ZP);
        }
    };

    // CHAIN: what one stage writes another workgroup reads within the same launch, and the L2
    // caches of the eight XCDs are not kept coherent for ordinary accesses.  Outputs are therefore
    // written, and activations and residuals read, as device-scope atomic accesses (they go to the
    // memory side instead of staying in one XCD's L2); with that no cache has to be written back or
    // invalidated as a whole between stages, which was measured at about 30 us per stage.
    auto coherent_load16 = [](gbl_half_t *p) -> uint4 {
        const uint64_t *q = (const uint64_t *)(uintptr_t)p;
        const uint64_t lo = __hip_atomic_load(q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const uint64_t hi = __hip_atomic_load(q + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return make_uint4((uint32_t)lo, (uint32_t)(lo >> 32), (uint32_t)hi, (uint32_t)(hi >> 32));
    };
    auto load_res = [](gbl_half_t *p) -> float {
        if (CHAIN) {
            const uint16_t b = __hip_atomic_load((const uint16_t *)(uintptr_t)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            return (float)__builtin_bit_cast(half_t, b);
        }
        return (float)*p;
    };
    auto store_out = [](__attribute__((address_space(1))) half_t *p, float v) {
        const half_t h = (half_t)v;
        if (CHAIN) __hip_atomic_store((uint16_t *)(uintptr_t)p, __builtin_bit_cast(uint16_t, h), __ATOMIC_RELAXED,
                                      __HIP_MEMORY_SCOPE_AGENT);
        else *p = h;
    };

    // activation fragments (see the header comment), loaded once.  Their loads go out first:
    // they are tiny, and behind the first weight requests of the whole grid they would wait
    // for megabytes that are of no use before the fragments are there.  (CHAIN: the other way
    // round -- the weights do not depend on the stage in front, the activations do.)
    uint4 xa[16];
    uint4 wn[16];                // FUSED: normalisation factors, alive until the fragments are final
    bool okx[4];                 // whether tile u of the lane's slot exists (else its fragments are 0)
    auto load_fragments = [&]() {
        const int slot = r >> mlog;
        int m = r & (Mpad - 1);
        m = m < M ? m : M - 1;
        const int bl = b0 + slot;
        gbl_half_t *xrow = px + (size_t)m * K + 8 * c;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int g = 4 * bl + u;
            okx[u] = bl < b1 && g < G;
            const int gs = okx[u] ? g : 0;          // always a valid address: no branch, no wait
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (CHAIN) xa[4 * u + j] = coherent_load16(xrow + gs * 128 + 32 * j);
                else xa[4 * u + j] = __builtin_bit_cast(uint4, *(gbl_u32x4_t *)(xrow + gs * 128 + 32 * j));
        }
        if (FUSED && pre_op != GEMV_PRE_NONE) {      // the factors of the same columns
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int gs = okx[u] ? 4 * bl + u : 0;
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    wn[4 * u + j] = __builtin_bit_cast(uint4, *(gbl_u32x4_t *)(ppre + 8 * c + gs * 128 + 32 * j));
            }
        }
    };
    if (!CHAIN) load_fragments();

    // the first weight requests
    const int nbw = b1 - b0;
    const int J = iters * nbw;                               // jobs of this wave
    int nit = 0, nb = b0, nslot = 0, nj = 0;                 // next job to request
    auto issue_next = [&]() {
        issue(nit, nb, nslot);
        ++nj;
        if (++nslot == STAGES) nslot = 0;
        if (++nb == b1) { nb = b0; ++nit; }
    };
#pragma unroll
    for (int s = 0; s < STAGES - 1; ++s)
        if (nj < J) issue_next();

    if (CHAIN) {
        // Wait (bounded) until every workgroup of the launch has finished the stage in front: its
        // outputs are this stage's activations.  The weights requested above travel meanwhile.
        // The decision to go on or to give up is taken by the workgroup as a whole, since its
        // waves meet at barriers later on.
        if (cw.counter) {
            // one wave polls for the workgroup (2048 waves polling one address slow down the very
            // atomics they wait for); lane h reads shard h of the counter
            uint32_t *vote = reinterpret_cast<uint32_t *>(red + 2 * red_floats + W * 16);
            if (wave == 0) {
                bool ok = true;
                int spins = 0;
                for (;;) {
                    uint32_t part = 0;
                    if (lane < CHAIN_SHARDS)
                        part = __hip_atomic_load(cw.counter + CHAIN_SHARD_STRIDE * lane, __ATOMIC_RELAXED,
                                                 __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
                    for (int d = 1; d < CHAIN_SHARDS; d <<= 1) part += __shfl_xor(part, d);
                    // the flag first: once it is set no wait of the launch succeeds any more
                    const uint32_t stop = __builtin_amdgcn_readfirstlane(
                        __hip_atomic_load(cw.gave_up, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
                    const uint32_t seen = __builtin_amdgcn_readfirstlane(part);
                    if (stop != 0) { ok = false; break; }
                    if (seen >= cw.target) break;
                    if (++spins > cw.spin_limit) { ok = false; break; }
                    __builtin_amdgcn_s_sleep(8);
                }
                if (lane == 0) vote[0] = ok ? 1u : 0u;
            }
            lds_barrier();
            const bool all_ok = vote[0] != 0;
            if (!all_ok) {
                if (tid == 0) __hip_atomic_store(cw.gave_up, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                wait_loads<0>();                   // nothing may still be on its way into this LDS
                return false;
            }
            // the counter was read at device scope and so are the activations below; the fence keeps
            // the compiler from moving them in front of the wait (no cache operation at this scope)
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        }
        load_fragments();
    }

#pragma unroll
    for (int i = 0; i < 16; ++i)
        if (!okx[i >> 2]) xa[i] = make_uint4(0, 0, 0, 0);

    // FUSED, RMS normalisation in front of the linear: x' = fp16(x * rsqrt(mean_k x^2 + eps) * w_k).
    // The fragments of a wave hold its K-slice of token r % Mpad once (lanes of the same token
    // differ in c and in the slot bits of r); the waves that split K meet in LDS.
    // (SCALE: the rescaling pass alone, x' = fp16(x * w_k).)
    if (FUSED && pre_op != GEMV_PRE_NONE) {
        float rinv = 1.0f;
        if (pre_op == GEMV_PRE_RMSNORM) {
            float ss = 0.f;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                ss = mix_sum_squares(xa[i].x, ss);
                ss = mix_sum_squares(xa[i].y, ss);
                ss = mix_sum_squares(xa[i].z, ss);
                ss = mix_sum_squares(xa[i].w, ss);
            }
            ss += __shfl_xor(ss, 16);
            ss += __shfl_xor(ss, 32);
            if (mlog < 4) ss += __shfl_xor(ss, 8);
            if (mlog < 3) ss += __shfl_xor(ss, 4);
            if (mlog < 2) ss += __shfl_xor(ss, 2);
            if (mlog < 1) ss += __shfl_xor(ss, 1);
            if (KS > 1) {
                float *nred = red + 2 * red_floats;                 // [wave][16]
                if (c == 0) nred[wave * 16 + r] = ss;
                lds_barrier();
                ss = 0.f;
                for (int k = 0; k < KS; ++k) ss += nred[((ri << ksl) + k) * 16 + r];
            }
            rinv = rsqrtf(ss / (float)K + eps);
        }
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            xa[i].x = mix_scale_pair(xa[i].x, rinv, wn[i].x);
            xa[i].y = mix_scale_pair(xa[i].y, rinv, wn[i].y);
            xa[i].z = mix_scale_pair(xa[i].z, rinv, wn[i].z);
            xa[i].w = mix_scale_pair(xa[i].w, rinv, wn[i].w);
        }
    }

    // halves 2,3,6,7 of every fragment meet the 2^-20 codes and are scaled by 2^-4 to match the
    // 2^-24 ones
    if (BITS == 4) {
        const half2_t sixteenth = {(half_t)0.0625f, (half_t)0.0625f};
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            xa[i].y = __builtin_bit_cast(uint32_t, __builtin_bit_cast(half2_t, xa[i].y) * sixteenth);
            xa[i].w = __builtin_bit_cast(uint32_t, __builtin_bit_cast(half2_t, xa[i].w) * sixteenth);
        }
    } else {
        // INT3: halves 2i, 2i+1 of step j meet the codes of pair 4j + i, which read as
        // q * 2^(3 cls - 24): the activations carry 2^(-3 cls)
        const half2_t down[3] = {{(half_t)1.0f, (half_t)1.0f}, {(half_t)0.125f, (half_t)0.125f},
                                 {(half_t)0.015625f, (half_t)0.015625f}};
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                uint32_t *h = reinterpret_cast<uint32_t *>(&xa[4 * u + j]);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int cls = w3_cls(4 * j + i);
                    if (cls) h[i] = __builtin_bit_cast(uint32_t, __builtin_bit_cast(half2_t, h[i]) * down[cls]);
                }
            }
    }
    // 2^-24 * sum of the activations of each tile, per output row: the fragments against the
    // constant code 1 (halves 2^-24, 2^-24, 2^-20, 2^-20, ...)
    floatx4 xsum[4];
    {
        const half8_t ones = __builtin_bit_cast(half8_t, make_uint4(0x00010001u, 0x00100010u, 0x00010001u, 0x00100010u));
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            floatx4 t = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                half8_t one_j = ones;
                if (BITS == 3)   // the code 1 at the position of every pair of step j
                    one_j = __builtin_bit_cast(half8_t, make_uint4(0x00010001u << (3 * w3_cls(4 * j)),
                                                                   0x00010001u << (3 * w3_cls(4 * j + 1)),
                                                                   0x00010001u << (3 * w3_cls(4 * j + 2)),
                                                                   0x00010001u << (3 * w3_cls(4 * j + 3))));
                t = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8_t, xa[4 * u + j]), one_j, t, 0, 0, 0);
            }
            xsum[u] = t;
        }
    }

    // slot of output row 4c + v
    int slotv[4];
#pragma unroll
    for (int v = 0; v < 4; ++v) slotv[v] = (4 * c + v) >> mlog;

    const uint32_t rd_tile = ring + (BITS == 4 ? lane16 : (uint32_t)lane * 12), rd_sc = ring + 16 * r,
                   rd_zp = ring + 16 * (r >> 1);
    floatx4 total = {0.f, 0.f, 0.f, 0.f};
    int cit = 0, cb = b0, cslot = 0;                         // job being consumed

    // fold the running sums over the slots: afterwards lanes with c < max(1, Mpad/4) hold
    // token m = 4c + v (v < min(4, Mpad)) of column r
    auto fold = [&]() {
        if (mlog < 2) { total[0] += total[2]; total[1] += total[3]; }
        if (mlog < 1) total[0] += total[1];
        if (mlog < 4) {
#pragma unroll
            for (int v = 0; v < 4; ++v) total[v] += __shfl_xor(total[v], 32);
        }
        if (mlog < 3) {
#pragma unroll
            for (int v = 0; v < 4; ++v) total[v] += __shfl_xor(total[v], 16);
        }
    };
    const int cmax = Mpad >= 4 ? Mpad >> 2 : 1;

    auto finish_block = [&](int it) {
        fold();
        if (KS == 1) {
            const int rbo = rb_wg + it * RW + ri;
            if (rbo < NRB && c < cmax) {
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int m = 4 * c + v;
                    if (v < Mpad && m < M) {
                        const size_t at = (size_t)m * N + rbo * 16 + r;
                        store_out(py + at, FUSED && pres ? total[v] + load_res(pres + at) : total[v]);
                    }
                }
            }
            total = floatx4{0.f, 0.f, 0.f, 0.f};
            return;
        }
        float *rbuf = red + (it & 1) * red_floats;
        if (c < cmax) {
#pragma unroll
            for (int v = 0; v < 4; ++v)
                if (v < Mpad) rbuf[((ri * KS + ks) * Mpad + 4 * c + v) * 16 + r] = total[v];
        }
        total = floatx4{0.f, 0.f, 0.f, 0.f};
        lds_barrier();
        // one output per thread and pass: (row block tri, token m, column n) = bits of t
        for (int t = tid; t < (RW << (mlog + 4)); t += W * 64) {
            const int tri = t >> (mlog + 4), rem = t & ((16 << mlog) - 1), m = rem >> 4;
            const float *p = rbuf + ((tri * KS) << (mlog + 4)) + rem;
            float sum = 0.f;
            for (int k = 0; k < KS; ++k) sum += p[k << (mlog + 4)];
            const int rbo = rb_wg + it * RW + tri;
            if (rbo < NRB && m < M) {
                const size_t at = (size_t)m * N + rbo * 16 + (rem & 15);
                store_out(py + at, FUSED && pres ? sum + load_res(pres + at) : sum);
            }
        }
    };

    for (int j = 0; j < J; ++j) {
        if (nj < J) issue_next();
        // jobs requested after job j: min(STAGES-1, J-1-j); job j has landed once at most that
        // many jobs' loads are outstanding
        const int later = nj - j - 1;
        if (later >= STAGES - 1) wait_loads<LOADS_PER_JOB *(STAGES - 1)>();
        else if (STAGES > 2 && later == 2) wait_loads<LOADS_PER_JOB * 2>();
        else if (later == 1) wait_loads<LOADS_PER_JOB>();
        else wait_loads<0>();
        Landed cur;
        const uint32_t off = (uint32_t)cslot * STAGE_BYTES;
        if (BITS == 4) read_slot(cur, rd_tile + off, rd_sc + off, rd_zp + off);
        else read_slot_w3(cur, rd_tile + off, rd_sc + off, rd_zp + off);
        if (++cslot == STAGES) cslot = 0;
        const floatx4 bacc = BITS == 4 ? consume_batch(cur, xa, xsum, mask_lo, mask_hi, zshift)
                                       : consume_batch_w3(cur, xa, xsum, zshift);
        const int slot = cb - b0;
#pragma unroll
        for (int v = 0; v < 4; ++v) total[v] += slotv[v] == slot ? bacc[v] : 0.f;
        if (++cb == b1) { finish_block(cit); cb = b0; ++cit; }
    }
    return true;
}

template <int STAGES, int BITS, bool FUSED>
__global__ __launch_bounds__(512, 2) void gemv_stream_kernel(const GemvArgs<FUSED> A)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const unsigned char *ka = (const unsigned char *)__builtin_amdgcn_kernarg_segment_ptr();
    static_assert(!FUSED || offsetof(GemvArgs<true>, e) == sizeof(GemvLaunch), "layout");
    stream_body<STAGES, BITS, FUSED, false, offsetof(GemvLaunch, wg_begin), offsetof(GemvLaunch, p), sizeof(GemvLaunch),
                GEMV_MAX_PROBLEMS, GEMV_MAX_FUSED>(ka, A.L.M, A.L.mlog, A.L.logW, (int)blockIdx.x, smem,
                                                   ChainWait{});
}

// Chained launch (Sec. 4.2, kernel fusion carried across the data dependences of a decoder layer).
// A decode step orders its linears (Q,K,V | o | gate,up | down); as separate launches each of them
// pays a launch, a ramp-up of the memory pipeline and a run-out, which together exceed the time
// the weights need.  Here ONE launch of resident workgroups runs the stages one after the other.
// What makes that pay: the weights of a stage do not depend on the stage in front, so a workgroup
// that has finished its share of stage s requests its first jobs of stage s + 1 at once and only
// then waits until every workgroup has finished stage s (a counter in global memory, incremented
// by each workgroup once its outputs have been acknowledged, polled with a bounded number of spins).  Every
// workgroup must be resident for that (the launcher checks the occupancy); a wait that runs out
// sets the give-up flag, on which all others leave as well, so the launch always ends.
//   sync (32-bit words): [0] give-up flag, [1] workgroups that finished the launch (the last of
//   those sets all counters back to zero); the count of the workgroups that finished stage s is
//   kept in CHAIN_SHARDS parts, part h in word 32 (1 + CHAIN_SHARDS s + h), each in a cache line of
//   its own: a workgroup adds to part blockIdx % CHAIN_SHARDS, so that the atomics of the 512
//   workgroups do not all queue at one address, and the polling wave sums the parts.
// Ring slots per wave in a chained launch: CHAIN_RING - 1 jobs (4.2 KB each) are on their way while
// a workgroup waits for the stage in front, so that the memory system keeps working through the
// wait (the round trips of a wait go to a memory that is busy with the weights and take
// several microseconds).
#ifndef AWQ_CHAIN_RING
#define AWQ_CHAIN_RING 2
#endif
constexpr int CHAIN_RING = AWQ_CHAIN_RING;

struct ChainStage {
    int wg_begin[CHAIN_MAX_ENTRIES];
    int count, wgs;
    GemvProblem p[CHAIN_MAX_ENTRIES];
    GemvFusedExtra e[CHAIN_MAX_ENTRIES];
};
struct ChainArgs {
    ChainStage st[CHAIN_MAX_STAGES];
    uint32_t *sync;
    int nstages, M, mlog, logW, spin_limit, pad;
};
static_assert(sizeof(ChainArgs) <= 4096, "kernel arguments are limited to 4 KB");

__global__ __launch_bounds__(512, 2) void chain_kernel(const ChainArgs A)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const unsigned char *ka = (const unsigned char *)__builtin_amdgcn_kernarg_segment_ptr();
    uint32_t *sync = A.sync;
    const uint32_t workgroups = gridDim.x;
    for (int s = 0; s < A.nstages; ++s) {
        if ((int)blockIdx.x < A.st[s].wgs) {
            const ChainWait cw = {s > 0 ? sync + CHAIN_SHARD_STRIDE * (1 + CHAIN_SHARDS * (s - 1)) : nullptr, workgroups,
                                  sync, A.spin_limit};
            const bool ok = stream_body<CHAIN_RING, 4, true, true, offsetof(ChainStage, wg_begin), offsetof(ChainStage, p),
                                        offsetof(ChainStage, e), CHAIN_MAX_ENTRIES, CHAIN_MAX_ENTRIES>(
                ka + offsetof(ChainArgs, st) + (size_t)s * sizeof(ChainStage), A.M, A.mlog, A.logW, (int)blockIdx.x,
                smem, cw);
            if (!ok) return;                                   // the whole workgroup, see stream_body
        }
        if (s + 1 < A.nstages) {
            // every wave's outputs (device-scope stores) have been acknowledged, then the count
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();
            if (threadIdx.x == 0)
                __hip_atomic_fetch_add(sync + CHAIN_SHARD_STRIDE * (1 + CHAIN_SHARDS * s + (blockIdx.x % CHAIN_SHARDS)), 1u,
                                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    if (threadIdx.x == 0) {
        // every workgroup that arrives here has passed its last wait: the last one may reset
        const uint32_t before = __hip_atomic_fetch_add(sync + 1, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (before == workgroups - 1) {
            for (int i = 0; i < CHAIN_SHARDS * (CHAIN_MAX_STAGES - 1); ++i)
                __hip_atomic_store(sync + CHAIN_SHARD_STRIDE * (1 + i), 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(sync + 1, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}


// ---- decode kernel for more than four tokens (gemv_rows_kernel) -------------------------------------
// With 5..16 tokens the register-resident activations of stream_body hold one or two batches per
// wave, so eight waves have to share a row block and meet in LDS after every job, and K beyond
// eight batches (the down projection) does not fit at all.  Here the activations go through LDS
// instead, one chunk of 512 columns (= one batch of four groups) at a time:
//   * a workgroup is two units of three compute waves and one loader wave, one workgroup per CU.
//     A compute wave owns `iters` row blocks and keeps their sums in its registers;
//   * the loader wave of a unit keeps the next two chunks of x (16 token rows x 1 KB each; rows
//     beyond M repeat row M - 1) in its registers and writes chunk c + 1 into the other of the unit's
//     two LDS buffers (rows 1040 bytes apart, so that the 16 lanes of a fragment read hit 16
//     different bank groups) as soon as every compute wave of the unit has copied chunk c - 1 into
//     its own registers; it also applies the factor 2^-4 to the halves that meet the codes in the
//     high nibble positions and zeroes columns beyond K, so that the compute waves use the same
//     fragments, the same constant-code MFMA for the row sums and the same consume_batch as
//     stream_body;
//   * a linear is planned in one of two ways.  Whole rows: the two units work on different row
//     blocks (six per step of the workgroup) and each walks all chunks of K.  Split rows (for long
//     K, where a whole row would be more jobs than a wave's share of the launch): both units work on
//     the same three row blocks per step, unit 0 on the first half of the chunks and unit 1 on the
//     rest; at the end unit 1 hands its sums over through LDS, behind the only barrier of the kernel;
//   * the chunks of a unit are taken in cyclic order from a start that differs from workgroup to
//     workgroup;
//   * no barrier in the steady state: the loader publishes the number of the newest chunk in place
//     in an LDS word and every compute wave the newest chunk whose fragments it has read into its
//     registers; the loader overwrites a buffer once all three have read it, a compute wave reads a
//     chunk once it is published.  The compute waves therefore never wait for each other, only
//     (rarely) for the loader; a barrier per chunk held all of them to the pace of the slowest
//     memory response.  The weight jobs run through each compute wave's private ring exactly as
//     in stream_body (requested ahead, across chunk boundaries).
// A-operand row m of the MFMA is token m.  Any K (a multiple of 128), 1 <= M <= 16.
constexpr int ROWS_X_ROW = 1024 + 16;                  // bytes of one token row of a chunk in LDS
constexpr int ROWS_MAX_ITERS = 8;
constexpr int ROWS_CW = 3;                             // compute waves of a unit
constexpr int ROWS_UNITS = 2;
constexpr int ROWS_THREADS = 64 * ROWS_UNITS * (ROWS_CW + 1);
// MR = token rows kept in LDS (8 or 16; tokens beyond M repeat token M - 1, and with MR = 8 the
// MFMA rows 8..15 read the LDS rows 0..7 again).  Half the rows leave room for a fourth ring slot.
template <int MR>
struct RowsShape {
    static constexpr int X_BUF = MR * ROWS_X_ROW;
    static constexpr int RING = MR == 8 ? 4 : 3;       // ring slots per compute wave
    static constexpr int UNIT_LDS = ROWS_CW * RING * Slot<4>::BYTES + 2 * X_BUF + 64;   // + the progress words
    static constexpr int LDS = ROWS_UNITS * UNIT_LDS;
    static_assert(ROWS_MAX_ITERS * 1024 <= RING * Slot<4>::BYTES, "the hand-over of the sums uses a wave's ring");
    static_assert(LDS <= 160 * 1024, "one workgroup per CU");
};

template <int MR>
__global__ __launch_bounds__(ROWS_THREADS) void gemv_rows_kernel(const GemvArgs<false> A)
{
    extern __shared__ __align__(16) unsigned char smem[];
    constexpr int ROWS_X_BUF = RowsShape<MR>::X_BUF, ROWS_RING = RowsShape<MR>::RING;
    constexpr int ROWS_UNIT_LDS = RowsShape<MR>::UNIT_LDS;
    constexpr int STAGE_BYTES = Slot<4>::BYTES, STAGE_SC = Slot<4>::SC, STAGE_ZP = Slot<4>::ZP;
    constexpr int LOADS_PER_JOB = Slot<4>::LOADS;
    typedef const __attribute__((address_space(1))) half_t gbl_half_t;
    typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
    typedef const __attribute__((address_space(1))) u32x4_t gbl_u32x4_t;
    uint32_t mask_lo = 0x000F000Fu, mask_hi = 0x00F000F0u;
    asm("" : "+s"(mask_lo));
    asm("" : "+s"(mask_hi));
    const GemvLaunch &L = A.L;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int unit = wave >> 2, role = wave & 3;           // role 3 = loader
    // the workgroup's entry of the launch table, fetched as in stream_body: lane l reads wg_begin[l]
    // and entry l with vector loads, a ballot and readlanes pick the right one (one round trip)
    GemvProblem P;
    int wg0;
    {
        typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
        typedef const __attribute__((address_space(1))) u32x2_t gbl_u32x2_t;
        typedef const __attribute__((address_space(1))) int gbl_int_t;
        const unsigned char *ka = (const unsigned char *)__builtin_amdgcn_kernarg_segment_ptr();
        const int le = lane < GEMV_MAX_PROBLEMS ? lane : GEMV_MAX_PROBLEMS - 1;
        const int begin = *(gbl_int_t *)(uintptr_t)(ka + offsetof(GemvLaunch, wg_begin) + 4 * le);
        gbl_u32x2_t *pe = (gbl_u32x2_t *)(uintptr_t)(ka + offsetof(GemvLaunch, p) + sizeof(GemvProblem) * le);
        uint32_t f[14], g[14];
#pragma unroll
        for (int d = 0; d < 7; ++d) {
            const u32x2_t t = pe[d];
            f[2 * d] = t.x;
            f[2 * d + 1] = t.y;
        }
        const uint64_t mine = __ballot(lane < GEMV_MAX_PROBLEMS && (int)blockIdx.x >= begin);
        const int pi = __builtin_amdgcn_readfirstlane(__popcll(mine) - 1);
#pragma unroll
        for (int d = 0; d < 14; ++d) g[d] = __builtin_amdgcn_readlane(f[d], pi);
        P.x = reinterpret_cast<const half_t *>(((uint64_t)g[1] << 32) | g[0]);
        P.q = reinterpret_cast<const uint4 *>(((uint64_t)g[3] << 32) | g[2]);
        P.sc = reinterpret_cast<const uint16_t *>(((uint64_t)g[5] << 32) | g[4]);
        P.zp = reinterpret_cast<const uint8_t *>(((uint64_t)g[7] << 32) | g[6]);
        P.y = reinterpret_cast<half_t *>(((uint64_t)g[9] << 32) | g[8]);
        P.N = (int)g[10];
        P.K = (int)g[11];
        P.plan = (int)g[12];
        P.nrb = (int)g[13];
        wg0 = __builtin_amdgcn_readlane(begin, pi);
    }
    const int M = L.M, K = P.K, N = P.N, G = K >> 7, NRB = P.nrb, NB = (G + 3) >> 2;
    const int iters = P.plan >> 8;
    const bool split = (P.plan & 15) != 0;                 // rows split over the two units
    const int m_first = (P.plan >> 4) & 15;                // token rows below this one are not written
    const int rows_per_step = split ? ROWS_CW : ROWS_UNITS * ROWS_CW;
    const int rb_first = ((int)blockIdx.x - wg0) * iters * rows_per_step + (split ? 0 : unit * ROWS_CW);
    // the unit's chunks [c0, c0 + NC)
    const int half_chunks = (NB + 1) >> 1;
    const int c0 = split && unit ? half_chunks : 0;
    const int NC = split ? (unit ? NB - half_chunks : half_chunks) : NB;
    unsigned char *const usmem = smem + unit * ROWS_UNIT_LDS;
    const uint32_t lds0 = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)usmem);
    const uint32_t xbuf = lds0 + ROWS_CW * ROWS_RING * STAGE_BYTES;
    gbl_half_t *px = (gbl_half_t *)(uintptr_t)P.x;
    // Every workgroup walks its chunks of K in the same cyclic order but starts at a chunk of its
    // own.  Started together at chunk 0 all workgroups would read, at any moment, the same 4 KB
    // window of every row block (addresses a multiple of the row-block size apart), i.e. keep a
    // fraction of the memory channels busy and leave the rest idle.
    const int rot = NC > 0 ? (int)blockIdx.x % NC : 0;

    // progress words: [0] newest chunk in place, [1 + w] newest chunk compute wave w has read
    volatile int *flags = reinterpret_cast<volatile int *>(usmem + ROWS_CW * ROWS_RING * STAGE_BYTES + 2 * ROWS_X_BUF);
    if (lane == 0) flags[role == ROWS_CW ? 0 : 1 + role] = -1;
    lds_barrier();

    floatx4 acc[ROWS_MAX_ITERS];
#pragma unroll
    for (int i = 0; i < ROWS_MAX_ITERS; ++i) acc[i] = floatx4{0.f, 0.f, 0.f, 0.f};
    const int r = lane & 15, c4 = lane >> 4;
    const uint32_t lane16 = (uint32_t)lane << 4;
    const uint32_t ring = lds0 + (uint32_t)role * (ROWS_RING * STAGE_BYTES);

    if (role == ROWS_CW) {
        // ---- loader wave: lane l owns the 16 bytes at column 8 l of a chunk, for the 16 token rows
        uint4 regA[MR], regB[MR];
        const half2_t sixteenth = {(half_t)0.0625f, (half_t)0.0625f};
        auto fetch = [&](uint4 (&reg)[MR], int step) {
            const int chunk = c0 + (step + rot < NC ? step + rot : step + rot - NC);
            int col = chunk * 512 + lane * 8;
            col = col < K ? col : K - 8;                           // beyond K: any valid address
#pragma unroll
            for (int m = 0; m < MR; ++m) {
                const int row = m < M ? m : M - 1;
                reg[m] = __builtin_bit_cast(uint4, *(gbl_u32x4_t *)(px + (size_t)row * K + col));
            }
        };
        auto store = [&](const uint4 (&reg)[MR], int step) {
            const int chunk = c0 + (step + rot < NC ? step + rot : step + rot - NC);
            // step goes where step - 2 was: every compute wave must have read step - 2
            for (;;) {
                int slowest = flags[1];
#pragma unroll
                for (int w = 1; w < ROWS_CW; ++w) slowest = min(slowest, flags[1 + w]);
                if (slowest >= step - 2) break;
                __builtin_amdgcn_s_sleep(1);
            }
            const bool valid = chunk * 512 + lane * 8 < K;
            unsigned char *dst = usmem + ROWS_CW * ROWS_RING * STAGE_BYTES + (step & 1) * ROWS_X_BUF + lane * 16;
#pragma unroll
            for (int m = 0; m < MR; ++m) {
                uint4 v = reg[m];
                v.y = __builtin_bit_cast(uint32_t, __builtin_bit_cast(half2_t, v.y) * sixteenth);
                v.w = __builtin_bit_cast(uint32_t, __builtin_bit_cast(half2_t, v.w) * sixteenth);
                if (!valid) v = make_uint4(0, 0, 0, 0);
                *reinterpret_cast<uint4 *>(dst + m * ROWS_X_ROW) = v;
            }
            // LDS operations of a wave are carried out in order: the word follows the data
            asm volatile("" ::: "memory");
            if (lane == 0) flags[0] = step;
        };
        if (NC > 0) fetch(regA, 0);
        if (NC > 1) fetch(regB, 1);
        for (int c = 0; c < NC; c += 2) {
            store(regA, c);
            if (c + 2 < NC) fetch(regA, c + 2);
            if (c + 1 < NC) {
                store(regB, c + 1);
                if (c + 3 < NC) fetch(regB, c + 3);
            }
        }
    } else {
        // ---- compute waves
        const int zshift = (r & 1) * 4;
        const unsigned char *qbase = reinterpret_cast<const unsigned char *>(P.q);
        const unsigned char *scbase = reinterpret_cast<const unsigned char *>(P.sc);
        const unsigned char *zpbase = reinterpret_cast<const unsigned char *>(P.zp);
        const uint32_t sc_lane = (uint32_t)(lane & 3) * 32 + (uint32_t)(lane >> 2) * 2;
        const uint32_t zp_lane = (uint32_t)(lane & 3) * 8 + (uint32_t)((lane >> 2) & 7);
        const bool ragged = (G & 3) != 0;
        auto issue = [&](int it, int b, int slot) {
            int rb = rb_first + it * rows_per_step + role;
            rb = rb < NRB ? rb : NRB - 1;                       // surplus waves redo the last block
            const size_t t0 = (size_t)rb * G + (size_t)b * 4;
            const uint32_t dst = ring + (uint32_t)slot * STAGE_BYTES;
            const unsigned char *tq = qbase + t0 * 1024, *ts = scbase + t0 * 32, *tz = zpbase + t0 * 8;
            if (!ragged || b * 4 + 4 <= G) {
                dma16_to_lds<0>(tq + lane16, dst);
                dma16_to_lds<1024>(tq + lane16, dst);
                dma16_to_lds<2048>(tq + lane16, dst);
                dma16_to_lds<3072>(tq + lane16, dst);
                dma2_to_lds(ts + sc_lane, dst + STAGE_SC);
                if (lane < 32) dma1_to_lds(tz + zp_lane, dst + STAGE_ZP);
            } else {
                const int last = G - 1 - b * 4;                 // last valid group of this batch (0..2)
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    dma16_to_lds<0>(tq + ((size_t)min(u, last) << 10) + lane16, dst + u * 1024);
                const int gl = min(lane & 3, last);
                dma2_to_lds(ts + gl * 32 + (lane >> 2) * 2, dst + STAGE_SC);
                if (lane < 32) dma1_to_lds(tz + gl * 8 + ((lane >> 2) & 7), dst + STAGE_ZP);
            }
        };
        // jobs in the order (chunk, row block): job j = chunk j / iters, row block j % iters
        const int J = NC * iters;
        int nj = 0, nit = 0, nb = 0, nslot = 0;
        auto issue_next = [&]() {
            issue(nit, c0 + (nb + rot < NC ? nb + rot : nb + rot - NC), nslot);
            ++nj;
            if (++nslot == ROWS_RING) nslot = 0;
            if (++nit == iters) { nit = 0; ++nb; }
        };
#pragma unroll
        for (int t = 0; t < ROWS_RING - 1; ++t)
            if (nj < J) issue_next();

        const half8_t ones = __builtin_bit_cast(half8_t, make_uint4(0x00010001u, 0x00100010u, 0x00010001u, 0x00100010u));
        const uint32_t rd_tile = ring + lane16, rd_sc = ring + 16 * r, rd_zp = ring + 16 * (r >> 1);
        const uint32_t rd_x = xbuf + (uint32_t)(r & (MR - 1)) * ROWS_X_ROW + (uint32_t)c4 * 16;
        int cslot = 0, j = 0;
        for (int c = 0; c < NC; ++c) {
            while (flags[0] < c) __builtin_amdgcn_s_sleep(1);
            // fragments of this chunk: token r, columns 128 u + 32 j + 8 c4 + 0..7
            uint4 xa[16];
            {
                const uint32_t xaddr = rd_x + (uint32_t)(c & 1) * ROWS_X_BUF;
                asm volatile(
                    "ds_read_b128 %0, %16\n\tds_read_b128 %1, %16 offset:64\n\tds_read_b128 %2, %16 offset:128\n\t"
                    "ds_read_b128 %3, %16 offset:192\n\tds_read_b128 %4, %16 offset:256\n\tds_read_b128 %5, %16 offset:320\n\t"
                    "ds_read_b128 %6, %16 offset:384\n\tds_read_b128 %7, %16 offset:448\n\tds_read_b128 %8, %16 offset:512\n\t"
                    "ds_read_b128 %9, %16 offset:576\n\tds_read_b128 %10, %16 offset:640\n\tds_read_b128 %11, %16 offset:704\n\t"
                    "ds_read_b128 %12, %16 offset:768\n\tds_read_b128 %13, %16 offset:832\n\tds_read_b128 %14, %16 offset:896\n\t"
                    "ds_read_b128 %15, %16 offset:960\n\ts_waitcnt lgkmcnt(0)"
                    : "=&v"(xa[0]), "=&v"(xa[1]), "=&v"(xa[2]), "=&v"(xa[3]), "=&v"(xa[4]), "=&v"(xa[5]), "=&v"(xa[6]),
                      "=&v"(xa[7]), "=&v"(xa[8]), "=&v"(xa[9]), "=&v"(xa[10]), "=&v"(xa[11]), "=&v"(xa[12]), "=&v"(xa[13]),
                      "=&v"(xa[14]), "=&v"(xa[15])
                    : "v"(xaddr)
                    : "memory");
                if (lane == 0) flags[1 + role] = c;             // read: the loader may reuse the buffer
            }
            floatx4 xsum[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                floatx4 t = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int jj = 0; jj < 4; ++jj)
                    t = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8_t, xa[4 * u + jj]), ones, t, 0, 0, 0);
                xsum[u] = t;
            }
#pragma unroll
            for (int it = 0; it < ROWS_MAX_ITERS; ++it) {
                if (it < iters) {
                    if (nj < J) issue_next();
                    const int later = nj - j - 1;               // jobs requested after the one now due
                    if (ROWS_RING > 3 && later >= 3) wait_loads<3 * LOADS_PER_JOB>();
                    else if (later >= 2) wait_loads<2 * LOADS_PER_JOB>();
                    else if (later == 1) wait_loads<LOADS_PER_JOB>();
                    else wait_loads<0>();
                    Landed cur;
                    const uint32_t off = (uint32_t)cslot * STAGE_BYTES;
                    read_slot(cur, rd_tile + off, rd_sc + off, rd_zp + off);
                    if (++cslot == ROWS_RING) cslot = 0;
                    const floatx4 b = consume_batch(cur, xa, xsum, mask_lo, mask_hi, zshift);
#pragma unroll
                    for (int v = 0; v < 4; ++v) acc[it][v] += b[v];
                    ++j;
                }
            }
        }
    }
    if (split) {
        // unit 1 hands its sums to the wave of unit 0 with the same row blocks; every job of the ring
        // has been consumed, so the ring is free to carry them
        if (unit == 1 && role < ROWS_CW) {
#pragma unroll
            for (int it = 0; it < ROWS_MAX_ITERS; ++it)
                if (it < iters) *reinterpret_cast<floatx4 *>(usmem + role * (ROWS_RING * STAGE_BYTES) + it * 1024 + lane * 16) = acc[it];
        }
        lds_barrier();
        if (unit == 1) return;
        if (role < ROWS_CW) {
            const unsigned char *other = smem + ROWS_UNIT_LDS + role * (ROWS_RING * STAGE_BYTES);
#pragma unroll
            for (int it = 0; it < ROWS_MAX_ITERS; ++it)
                if (it < iters) {
                    const floatx4 o = *reinterpret_cast<const floatx4 *>(other + it * 1024 + lane * 16);
#pragma unroll
                    for (int v = 0; v < 4; ++v) acc[it][v] += o[v];
                }
        }
    }
    if (role == ROWS_CW) return;
    // lane (r, c4) holds tokens 4 c4 + v of column r of each of its row blocks
    __attribute__((address_space(1))) half_t *py = (__attribute__((address_space(1))) half_t *)(uintptr_t)P.y;
#pragma unroll
    for (int it = 0; it < ROWS_MAX_ITERS; ++it) {
        const int rbo = rb_first + it * rows_per_step + role;
        if (it < iters && rbo < NRB) {
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int m = 4 * c4 + v;
                if (m >= m_first && m < M) py[(size_t)m * N + rbo * 16 + r] = (half_t)acc[it][v];
            }
        }
    }
}

int ceil_log2(int v) { int l = 0; while ((1 << l) < v) ++l; return l; }

}  // namespace

// Plans and launches one grouped decode launch.  Returns AWQ_OK, an error, or
// AWQ_GEMV_STREAM_UNFIT when some linear has more batches along K than the waves of a
// workgroup can hold as register-resident activations (the caller then uses the batch
// kernel).
//
// Plan.  The kernel is bound by how evenly the memory requests of all resident waves cover
// the run time, so every wave should get about the same number of jobs T = (all batches) /
// (waves wanted on the chip), with a floor of one job.  Per linear, K is split over the fewest
// waves the register slots allow, and a workgroup takes `iters` consecutive row-block steps
// so that iters * (batches per wave and row block) comes as close to T as possible.
bool awq_gemv_stream_fits(int N, int K, int M)
{
    (void)N;
    const int bpr = 16 >> ceil_log2(M);
    const int NBT = (K / 128 + 3) / 4;
    const int ksl_min = ceil_log2((NBT + bpr - 1) / bpr);
    return ksl_min <= 3 && (1 << ksl_min) <= NBT;
}

namespace {

// Paired plan of a grouped launch.
//
// All workgroups of a launch are resident at once (two fit on a CU), and the hardware places
// workgroup w and workgroup w + 256 on the same CU.  With one size of workgroup per linear their
// number is whatever the row-block steps give (428 for a Llama-2-7B layer): 172 CUs then carry
// two workgroups and 84 one, and the launch ends with a run-out in which only the loaded CUs
// still stream.  Here every linear is cut into workgroups of two sizes (lo or lo + 1 steps) so
// that 512 come out, the 256 largest first and the rest in ascending order behind them: each
// CU gets a large and a small one.  A run of equal workgroups of one linear becomes one entry of
// the launch table: a range of row blocks of a linear is a linear of its own (its packed arrays
// are contiguous, its outputs a column range of y).
struct PairedRun {
    int lin, iters, count, load;
};

std::atomic<int> g_last_plan{0};   // diagnostic: 1 = one size of workgroup per linear, 2 = paired plan

template <int BITS>
bool plan_paired(const GemvProblem *problems, int count, const int *ksl_of, int W, GemvLaunch &L, int &wg_total)
{
    constexpr int TARGET = 512, ROUND = 256;
    int S[GEMV_MAX_PROBLEMS], nbw[GEMV_MAX_PROBLEMS], RW[GEMV_MAX_PROBLEMS], lo[GEMV_MAX_PROBLEMS];
    int hN[GEMV_MAX_PROBLEMS], lN[GEMV_MAX_PROBLEMS], removable[GEMV_MAX_PROBLEMS], rem[GEMV_MAX_PROBLEMS];
    long long U = 0;
    for (int i = 0; i < count; ++i) {
        const int NBT = (problems[i].K / 128 + 3) / 4;
        nbw[i] = (NBT + (1 << ksl_of[i]) - 1) >> ksl_of[i];
        RW[i] = W >> ksl_of[i];
        S[i] = (problems[i].N / 16 + RW[i] - 1) / RW[i];
        U += (long long)S[i] * nbw[i];
    }
    const double tstar = (double)U / TARGET;
    if (tstar < 6.0) return false;                        // too small a launch for two workgroups per CU
    int w_lo = 0, w_hi = 0;
    for (int i = 0; i < count; ++i) {
        lo[i] = std::max(1, (int)(tstar / nbw[i]));
        const int a = (S[i] + lo[i] - 1) / lo[i], b = (S[i] + lo[i]) / (lo[i] + 1);
        removable[i] = a - b;
        rem[i] = 0;
        w_lo += a;
        w_hi += b;
    }
    if (w_hi > TARGET || w_lo < TARGET) return false;
    // take the surplus workgroups away where the larger size is smallest (equal sizes share in
    // proportion to what they can give)
    int R = w_lo - TARGET;
    bool done[GEMV_MAX_PROBLEMS] = {};
    while (R > 0) {
        int best = -1;
        for (int i = 0; i < count; ++i)
            if (!done[i] && removable[i] > 0 && (best < 0 || (lo[i] + 1) * nbw[i] < (lo[best] + 1) * nbw[best])) best = i;
        if (best < 0) return false;
        const int load = (lo[best] + 1) * nbw[best];
        int cap = 0;
        for (int i = 0; i < count; ++i)
            if (!done[i] && (lo[i] + 1) * nbw[i] == load) cap += removable[i];
        const int take = std::min(R, cap);
        int given = 0;
        for (int i = 0; i < count; ++i)
            if (!done[i] && (lo[i] + 1) * nbw[i] == load) {
                rem[i] = (int)((long long)take * removable[i] / cap);
                given += rem[i];
            }
        for (int i = 0; i < count && given < take; ++i)
            if (!done[i] && (lo[i] + 1) * nbw[i] == load && rem[i] < removable[i]) {
                ++rem[i];
                ++given;
            }
        for (int i = 0; i < count; ++i)
            if ((lo[i] + 1) * nbw[i] == load) done[i] = true;
        R -= take;
    }
    int total = 0;
    for (int i = 0; i < count; ++i) {
        hN[i] = std::min(rem[i] * lo[i], S[i] / (lo[i] + 1));
        const int left = S[i] - hN[i] * (lo[i] + 1);
        lN[i] = left > 0 ? (left + lo[i] - 1) / lo[i] : 0;
        total += hN[i] + lN[i];
    }
    if (total > TARGET || total <= ROUND) return false;

    // runs of equal workgroups, largest first
    PairedRun runs[2 * GEMV_MAX_PROBLEMS];
    int nruns = 0;
    for (int i = 0; i < count; ++i) {
        if (hN[i] > 0) runs[nruns++] = {i, lo[i] + 1, hN[i], (lo[i] + 1) * nbw[i]};
        if (lN[i] > 0) runs[nruns++] = {i, lo[i], lN[i], lo[i] * nbw[i]};
    }
    std::stable_sort(runs, runs + nruns, [](const PairedRun &a, const PairedRun &b) { return a.load > b.load; });
    // the first 256 in this order, then the others smallest first
    PairedRun order[2 * GEMV_MAX_PROBLEMS + 2];
    int norder = 0, seen = 0, split_at = -1;
    PairedRun tail[2 * GEMV_MAX_PROBLEMS + 1];
    int ntail = 0;
    for (int r = 0; r < nruns; ++r) {
        if (seen >= ROUND) {
            tail[ntail++] = runs[r];
        } else if (seen + runs[r].count <= ROUND) {
            order[norder++] = runs[r];
        } else {
            PairedRun first = runs[r], second = runs[r];
            first.count = ROUND - seen;
            second.count = runs[r].count - first.count;
            order[norder++] = first;
            tail[ntail++] = second;
            split_at = r;
        }
        seen += runs[r].count;
    }
    (void)split_at;
    for (int r = ntail - 1; r >= 0; --r) order[norder++] = tail[r];
    if (norder > GEMV_MAX_PROBLEMS) return false;

    // entries: consecutive row-block ranges of their linear
    int cursor[GEMV_MAX_PROBLEMS] = {};
    int wg = 0, ne = 0;
    for (int r = 0; r < norder; ++r) {
        const PairedRun &run = order[r];
        const GemvProblem &src = problems[run.lin];
        const int NRB = src.N / 16, G = src.K / 128;
        const int rb0 = cursor[run.lin];
        const int nrb = std::min(run.count * run.iters * RW[run.lin], NRB - rb0);
        if (nrb <= 0) continue;
        cursor[run.lin] += nrb;
        GemvProblem p = src;
        p.q = reinterpret_cast<const uint4 *>(reinterpret_cast<const unsigned char *>(src.q) +
                                              (size_t)rb0 * G * Slot<BITS>::TILE);
        p.sc = src.sc + (size_t)rb0 * G * 16;
        p.zp = src.zp + (size_t)rb0 * G * 8;
        p.y = src.y + (size_t)rb0 * 16;
        p.plan = ksl_of[run.lin] | (run.iters << 4);
        p.nrb = nrb;
        const int steps = (nrb + RW[run.lin] - 1) / RW[run.lin];
        L.wg_begin[ne] = wg;
        L.p[ne] = p;
        wg += (steps + run.iters - 1) / run.iters;
        ++ne;
    }
    for (int i = 0; i < count; ++i)
        if (cursor[i] != problems[i].N / 16) return false;          // every row block exactly once
    L.count = ne;
    wg_total = wg;
    return true;
}

template <int BITS, bool FUSED>
int stream_launch_bits(const GemvProblem *problems, const GemvFusedExtra *extra, int count, int M,
                       hipStream_t stream)
{
    constexpr int STAGE_BYTES = Slot<BITS>::BYTES;
    static const int f_logw = awq_knob("AWQ_GEMV_LOGW", -1);
    static const int f_iters = awq_knob("AWQ_GEMV_ITERS", -1);
    static const int f_ksl = awq_knob("AWQ_GEMV_KSL", -1);
    static const int f_stages = awq_knob("AWQ_GEMV_STAGES", 2);
    static const int f_slots = awq_knob("AWQ_GEMV_SLOTS", 1792);
    static const int f_jobs = awq_knob("AWQ_GEMV_JOBS", -1);
    if (count < 1 || count > (FUSED ? GEMV_MAX_FUSED : GEMV_MAX_PROBLEMS)) return AWQ_ERR_BAD_ARGUMENT;

    GemvArgs<FUSED> A{};          // the kernel fetches whole table rows: no uninitialised bytes in them
    if constexpr (FUSED)
        for (int i = 0; i < count; ++i) A.e[i] = extra[i];
    GemvLaunch &L = A.L;
    for (int i = 0; i < GEMV_MAX_PROBLEMS; ++i) L.wg_begin[i] = 0x7fffffff;   // beyond the grid
    L.count = count;
    L.M = M;
    L.mlog = ceil_log2(M);
    const int bpr = 16 >> L.mlog;                  // batches one wave can hold activations for
    double total_batches = 0;
    for (int i = 0; i < count; ++i)
        total_batches += (double)(problems[i].N / 16) * ((problems[i].K / 128 + 3) / 4);
    double T = f_jobs > 0 ? f_jobs : std::max(1.0, total_batches / f_slots);

    int ksl_of[GEMV_MAX_PROBLEMS], iters_of[GEMV_MAX_PROBLEMS];
    int logW = 2;
    for (int i = 0; i < count; ++i) {
        const int NBT = (problems[i].K / 128 + 3) / 4;
        const int ksl_min = ceil_log2((NBT + bpr - 1) / bpr);
        if (ksl_min > 3) return AWQ_GEMV_STREAM_UNFIT;
        // K is split over as few waves as the register slots allow (splitting costs a pass
        // through LDS and a barrier per row block)
        int best_ksl = ksl_min;
        // ... unless the launch is so small that a wave would then have far more jobs than its
        // share T (a single projection): more waves along K put the whole matrix in flight
        while (best_ksl < 3 && (2 << best_ksl) <= NBT && ((NBT + (1 << best_ksl) - 1) >> best_ksl) > 1.5 * T)
            ++best_ksl;
        if (f_ksl > ksl_min) best_ksl = std::min(3, f_ksl);
        while ((1 << best_ksl) > NBT && best_ksl > ksl_min) --best_ksl;
        if ((1 << best_ksl) > NBT) return AWQ_GEMV_STREAM_UNFIT;
        ksl_of[i] = best_ksl;
        logW = std::max(logW, best_ksl);
    }
    if (f_logw >= 0) logW = std::min(3, std::max(f_logw, logW));
    L.logW = logW;
    const int W = 1 << logW;
    const int stages = f_stages == 3 ? 3 : (f_stages == 4 ? 4 : 2);
    const size_t lds = (size_t)W * stages * STAGE_BYTES + 2 * (size_t)W * (16 << L.mlog) * 4 +
                       (FUSED ? (size_t)W * 16 * 4 : 0);

    // The row-block steps per workgroup bring the jobs of a wave as close to T as they get.
    // Workgroups of eight waves take more than half of a CU's LDS, so only one is resident per
    // CU: their number must not exceed the CUs (a second round would run nearly alone), and T
    // is raised until it does not.
    const int wg_cap = lds * 2 > 160 * 1024 ? 256 : (1 << 30);
    int wg = 0;
    static const int f_paired = awq_knob("AWQ_GEMV_PAIRED", 1);
    bool paired = false;
    if (!FUSED && logW == 2 && stages == 2 && f_paired && f_logw < 0 && f_iters < 0 && f_ksl < 0 &&
        f_jobs < 0 && f_slots == 1792 && count * 3 <= GEMV_MAX_PROBLEMS) {
        paired = plan_paired<BITS>(problems, count, ksl_of, W, L, wg);
        if (!paired) {                                  // the table may be half written: start again
            for (int i = 0; i < GEMV_MAX_PROBLEMS; ++i) L.wg_begin[i] = 0x7fffffff;
            L.count = count;
            wg = 0;
        }
    }
    g_last_plan.store(paired ? 2 : 1, std::memory_order_relaxed);
    for (int attempt = 0; attempt < 64 && !paired; ++attempt) {
        wg = 0;
        for (int i = 0; i < count; ++i) {
            GemvProblem p = problems[i];
            const int NBT = (p.K / 128 + 3) / 4;
            const int nbw = (NBT + (1 << ksl_of[i]) - 1) >> ksl_of[i];
            int it = std::max(1, (int)(T / nbw + 0.5));
            if (f_iters > 0) it = f_iters;
            const int NRB = p.N / 16;
            const int RW = W >> ksl_of[i];
            const int steps = (NRB + RW - 1) / RW;            // row-block steps of the whole linear
            const int iters = std::min(it, steps);
            iters_of[i] = iters;
            p.plan = ksl_of[i] | (iters << 4);
            p.nrb = NRB;
            L.wg_begin[i] = wg;
            wg += (steps + iters - 1) / iters;
            L.p[i] = p;
        }
        if (wg <= wg_cap || f_iters > 0 || f_jobs > 0) break;
        T *= 1.04;
    }
    static AwqOncePerDevice once;
    std::atomic<bool> &attr_set = once.here();
    if (!attr_set.load(std::memory_order_relaxed)) {
        const int cap = 160 * 1024;
        const void *kernels[] = {reinterpret_cast<const void *>(gemv_stream_kernel<2, BITS, FUSED>),
                                 reinterpret_cast<const void *>(gemv_stream_kernel<3, BITS, FUSED>),
                                 reinterpret_cast<const void *>(gemv_stream_kernel<4, BITS, FUSED>)};
        for (int k = 0; k < (FUSED ? 1 : 3); ++k)
            if (hipFuncSetAttribute(kernels[k], hipFuncAttributeMaxDynamicSharedMemorySize, cap) != hipSuccess)
                return AWQ_ERR_HIP;
        attr_set.store(true, std::memory_order_relaxed);
    }
    if (lds > (size_t)160 * 1024) return AWQ_GEMV_STREAM_UNFIT;
    if (stages == 4 && !FUSED) gemv_stream_kernel<4, BITS, FUSED><<<dim3(wg), dim3(W * 64), lds, stream>>>(A);
    else if (stages == 3 && !FUSED) gemv_stream_kernel<3, BITS, FUSED><<<dim3(wg), dim3(W * 64), lds, stream>>>(A);
    else gemv_stream_kernel<2, BITS, FUSED><<<dim3(wg), dim3(W * 64), lds, stream>>>(A);
    return awq_launch_status();
}

}  // namespace

// Plans and launches a chained decode launch (chain_kernel).  Every stage is planned like a grouped
// launch of its own with one size of workgroup per linear; all stages share the workgroup size, and
// no stage may need more workgroups than the chip holds at once, because a workgroup that is not
// resident cannot report the end of a stage the others wait for.
int awq_gemv_chain_launch(const GemvProblem *const *problems, const GemvFusedExtra *const *extras, const int *counts,
                          int nstages, int M, uint32_t *sync, int spin_limit, hipStream_t stream)
{
    constexpr int STAGE_BYTES = Slot<4>::BYTES;
    if (nstages < 1 || nstages > CHAIN_MAX_STAGES) return AWQ_ERR_BAD_ARGUMENT;
    ChainArgs A{};
    A.sync = sync;
    A.nstages = nstages;
    A.M = M;
    A.mlog = ceil_log2(M);
    A.spin_limit = spin_limit > 0 ? spin_limit : 2000000;      // a few seconds of polling
    const int bpr = 16 >> A.mlog;
    int ksl_of[CHAIN_MAX_STAGES][CHAIN_MAX_ENTRIES];
    double T_of[CHAIN_MAX_STAGES];
    int logW = 2;
    for (int s = 0; s < nstages; ++s) {
        if (counts[s] < 1 || counts[s] > CHAIN_MAX_ENTRIES) return AWQ_ERR_BAD_ARGUMENT;
        double total_batches = 0;
        for (int i = 0; i < counts[s]; ++i)
            total_batches += (double)(problems[s][i].N / 16) * ((problems[s][i].K / 128 + 3) / 4);
        const double T = std::max(1.0, total_batches / 1792);
        T_of[s] = T;
        for (int i = 0; i < counts[s]; ++i) {
            const int NBT = (problems[s][i].K / 128 + 3) / 4;
            const int ksl_min = ceil_log2((NBT + bpr - 1) / bpr);
            if (ksl_min > 3) return AWQ_GEMV_STREAM_UNFIT;
            // a small stage spreads its rows over more waves along K -- but over four at most unless
            // the registers force eight: all stages share the workgroup size, and with eight waves
            // per workgroup the wide stages (gate, up) would fill only part of the chip
            int ksl = ksl_min;
            while (ksl < 2 && (2 << ksl) <= NBT && ((NBT + (1 << ksl) - 1) >> ksl) > 1.5 * T) ++ksl;
            while ((1 << ksl) > NBT && ksl > ksl_min) --ksl;
            if ((1 << ksl) > NBT) return AWQ_GEMV_STREAM_UNFIT;
            ksl_of[s][i] = ksl;
            logW = std::max(logW, ksl);
        }
    }
    A.logW = logW;
    const int W = 1 << logW;
    const size_t lds = (size_t)W * CHAIN_RING * STAGE_BYTES + 2 * (size_t)W * (16 << A.mlog) * 4 + (size_t)W * 16 * 4 + 64;
    if (lds > (size_t)160 * 1024) return AWQ_GEMV_STREAM_UNFIT;

    // workgroups the chip holds at once (per device and workgroup size; the query is not free)
    static std::atomic<int> resident[64][2];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return AWQ_ERR_HIP;
    static AwqOncePerDevice once;
    std::atomic<bool> &attr_set = once.here();
    if (!attr_set.load(std::memory_order_relaxed)) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(chain_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                160 * 1024) != hipSuccess)
            return AWQ_ERR_HIP;
        attr_set.store(true, std::memory_order_relaxed);
    }
    int cap = resident[dev][logW - 2].load(std::memory_order_relaxed);
    if (cap == 0) {
        int per_cu = 0, cus = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, reinterpret_cast<const void *>(chain_kernel), W * 64,
                                                         lds) != hipSuccess ||
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
            return AWQ_ERR_HIP;
        cap = std::min(per_cu, 2) * cus;             // two per CU at most: the layout the plans are made for
        if (cap < 1) return AWQ_GEMV_STREAM_UNFIT;
        resident[dev][logW - 2].store(cap, std::memory_order_relaxed);
    }

    int grid = 0;
    for (int s = 0; s < nstages; ++s) {
        ChainStage &S = A.st[s];
        double T = T_of[s];
        int wg = 0;
        for (int attempt = 0; attempt < 400; ++attempt) {
            wg = 0;
            for (int i = 0; i < counts[s]; ++i) {
                GemvProblem p = problems[s][i];
                const int NBT = (p.K / 128 + 3) / 4;
                const int nbw = (NBT + (1 << ksl_of[s][i]) - 1) >> ksl_of[s][i];
                const int NRB = p.N / 16, RW = W >> ksl_of[s][i];
                const int steps = (NRB + RW - 1) / RW;
                const int iters = std::min(std::max(1, (int)(T / nbw + 0.5)), steps);
                p.plan = ksl_of[s][i] | (iters << 4);
                p.nrb = NRB;
                S.wg_begin[i] = wg;
                S.p[i] = p;
                S.e[i] = extras[s][i];
                wg += (steps + iters - 1) / iters;
            }
            if (wg <= cap) break;
            T *= 1.04;
        }
        if (wg > cap) return AWQ_GEMV_STREAM_UNFIT;
        for (int i = counts[s]; i < CHAIN_MAX_ENTRIES; ++i) S.wg_begin[i] = 0x7fffffff;
        S.count = counts[s];
        S.wgs = wg;
        grid = std::max(grid, wg);
    }
    chain_kernel<<<dim3(grid), dim3(W * 64), lds, stream>>>(A);
    return awq_launch_status();
}


// Plans and launches gemv_rows_kernel for `count` linears (any K).  One workgroup per CU, so at most
// 256 workgroups; per linear one way of cutting it (whole or split rows, 1..ROWS_MAX_ITERS row-block
// steps per workgroup).  A wave's run time is
// about (jobs) x (time per job), and the time per job falls with the steps per workgroup, because
// the cost of taking a chunk of x out of LDS is shared by that many jobs (measured: 1.5 us per job
// with one step, 0.9 us with three).  The plan is the one with the smallest largest such estimate
// among those with at most 256 workgroups.
//
// first_row (optional): per linear, the first token row whose outputs are written.  The sums are
// taken chunk by chunk in an order that differs between workgroups, so two linears that share
// weights and tokens need not agree in the last bit: a caller that lets token blocks overlap names
// here the rows that the block in front has already written.
int awq_gemv_rows_launch(const GemvProblem *problems, int count, int M, hipStream_t stream, const int *first_row)
{
    if (count < 1 || count > GEMV_MAX_PROBLEMS || M < 1 || M > 16) return AWQ_ERR_BAD_ARGUMENT;
    struct Option {
        int split, iters, wgs;
        double cost;
    };
    constexpr int MAX_OPTIONS = 2 * ROWS_MAX_ITERS;
    static const double per_job = awq_knob("AWQ_ROWS_COST_JOB", 850) * 1e-3;
    static const double per_chunk = awq_knob("AWQ_ROWS_COST_CHUNK", 650) * 1e-3;
    Option options[GEMV_MAX_PROBLEMS][MAX_OPTIONS];
    int n_options[GEMV_MAX_PROBLEMS];
    double caps[GEMV_MAX_PROBLEMS * MAX_OPTIONS];
    int n_caps = 0;
    for (int i = 0; i < count; ++i) {
        const int NB = (problems[i].K / 128 + 3) / 4, NRB = problems[i].N / 16;
        n_options[i] = 0;
        for (int split = 0; split < (NB >= 2 ? 2 : 1); ++split) {
            const int rows = split ? ROWS_CW : ROWS_UNITS * ROWS_CW;
            const int steps = (NRB + rows - 1) / rows;
            const int chunks = split ? (NB + 1) / 2 : NB;
            for (int iters = 1; iters <= std::min(ROWS_MAX_ITERS, steps); ++iters) {
                const Option o = {split, iters, (steps + iters - 1) / iters, chunks * (iters * per_job + per_chunk)};
                options[i][n_options[i]++] = o;
                caps[n_caps++] = o.cost;
            }
        }
    }
    std::sort(caps, caps + n_caps);
    Option chosen[GEMV_MAX_PROBLEMS];
    for (int c = 0; c < n_caps; ++c) {
        int total = 0;
        bool ok = true;
        for (int i = 0; i < count && ok; ++i) {
            int best = -1;
            for (int o = 0; o < n_options[i]; ++o) {
                const Option &t = options[i][o];
                if (t.cost > caps[c]) continue;
                if (best < 0 || t.wgs < options[i][best].wgs ||
                    (t.wgs == options[i][best].wgs && t.cost < options[i][best].cost))
                    best = o;
            }
            if (best < 0) ok = false;
            else {
                chosen[i] = options[i][best];
                total += chosen[i].wgs;
            }
        }
        // beyond one workgroup per CU the rest waits for a second round; the last candidate (the
        // fewest workgroups there are) is taken whatever their number
        if (ok && (total <= 256 || c == n_caps - 1)) break;
    }
    GemvArgs<false> A{};
    GemvLaunch &L = A.L;
    for (int i = 0; i < GEMV_MAX_PROBLEMS; ++i) L.wg_begin[i] = 0x7fffffff;
    L.count = count;
    L.M = M;
    L.mlog = 4;
    L.logW = 2;
    int order[GEMV_MAX_PROBLEMS];
    for (int i = 0; i < count; ++i) order[i] = i;
    std::stable_sort(order, order + count, [&](int a, int b) { return chosen[a].cost > chosen[b].cost; });
    int wg = 0;
    for (int e = 0; e < count; ++e) {
        GemvProblem p = problems[order[e]];
        const int skip = first_row ? std::max(0, std::min(15, first_row[order[e]])) : 0;
        p.plan = chosen[order[e]].split | (skip << 4) | (chosen[order[e]].iters << 8);
        p.nrb = p.N / 16;
        L.wg_begin[e] = wg;
        L.p[e] = p;
        wg += chosen[order[e]].wgs;
    }
    static AwqOncePerDevice once;
    std::atomic<bool> &attr_set = once.here();
    if (!attr_set.load(std::memory_order_relaxed)) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(gemv_rows_kernel<8>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, RowsShape<8>::LDS) != hipSuccess ||
            hipFuncSetAttribute(reinterpret_cast<const void *>(gemv_rows_kernel<16>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, RowsShape<16>::LDS) != hipSuccess)
            return AWQ_ERR_HIP;
        attr_set.store(true, std::memory_order_relaxed);
    }
    if (M <= 8) gemv_rows_kernel<8><<<dim3(wg), dim3(ROWS_THREADS), RowsShape<8>::LDS, stream>>>(A);
    else gemv_rows_kernel<16><<<dim3(wg), dim3(ROWS_THREADS), RowsShape<16>::LDS, stream>>>(A);
    return awq_launch_status();
}

int awq_gemv_stream_launch(const GemvProblem *problems, int count, int M, hipStream_t stream)
{
    return stream_launch_bits<4, false>(problems, nullptr, count, M, stream);
}

int awq_gemv_stream_launch_w3(const GemvProblem *problems, int count, int M, hipStream_t stream)
{
    return stream_launch_bits<3, false>(problems, nullptr, count, M, stream);
}

int awq_gemv_stream_launch_fused(const GemvProblem *problems, const GemvFusedExtra *extra, int count,
                                 int M, hipStream_t stream)
{
    return stream_launch_bits<4, true>(problems, extra, count, M, stream);
}

extern "C" int awq_last_grouped_plan(void)
{
    return g_last_plan.load(std::memory_order_relaxed);
}
