// awq_quantize_pack / awq_unpack for gfx950.
//
// AWQ Sec. 3.2, Eq. 1-2: the group quantizer applied to w*s, in the asymmetric
// 16-level min/max form; Sec. 4.2: the codes are written directly in the packed
// order the linear kernels consume.
//
// A wavefront works on one tile at a time (16 rows x 128 columns = one quantization group
// for 16 rows).  Lane l works on row l%16 and on the four 8-column runs
// 32*j + 8*(l/16) + 0..7, which is exactly the 16-byte slot it will write, so the
// packed tile leaves the wave as a single coalesced 1 KB store.  The four lanes
// l, l^16, l^32, l^48 share a row; its min/max are combined with two xor-shuffles.
//
// This file must be compiled with -ffp-contract=off: the integer decisions
// (zero point, codes) are taken in IEEE binary32 with one rounding per operation,
// correctly rounded division and round-half-even, bit for bit.
#include "awq_common.h"

#include <algorithm>

namespace {

// clamp of a finite value (weights must be finite): one v_med3_f32
__device__ __forceinline__ float clampf(float v, float lo, float hi)
{
    return __builtin_amdgcn_fmed3f(v, lo, hi);
}

// nibble position of element e inside a packed word: {0,4,1,5,2,6,3,7}
__device__ __forceinline__ int nib_shift(int e) { return 4 * ((e >> 1) + 4 * (e & 1)); }

// rint(n / d) for a divisor d shared by many numerators, with the IEEE quotient deciding.
//
// The codes are rint(fl(n / d)) with fl the correctly rounded binary32 division (what the CPU side
// computes).  A full IEEE division costs about ten instructions per weight and this kernel is
// bound by instruction issue, so the quotient is first formed as q0 = fl(n * r) with r the
// reciprocal of d refined once (r depends on d only).  With the hardware reciprocal within one ulp,
// |r - 1/d| <= 2^-23 / d, so |q0 - n/d| <= |n/d| (2^-24 + 2^-23 + 2^-47) and, with the rounding of
// the IEEE quotient itself, |q0 - fl(n/d)| < 2^-22 |n/d|: for |q0| < 32 that is below 2^-17.
// rint(q0) can therefore differ from rint(fl(n/d)) only if q0 lies within 2^-17 of a half-integer,
// i.e. if |q0 - rint(q0)| > 1/2 - 2^-17; `off` collects the largest |q0 - rint(q0)| over a lane's
// weights (the difference is exact), and when any lane of the wave exceeds 1/2 - 2^-16 the whole
// tile is redone with the plain `/`.  (For |q0| >= 32 both roundings end up clamped to the same end
// code, whatever their difference.)  About 6 % of the tiles of a Gaussian matrix take the second
// pass.  tests/quotient_filter_check.c proves the claim exhaustively on the CPU.
struct Reciprocal {
    float d, r;
};
__device__ __forceinline__ Reciprocal make_reciprocal(float d)
{
    const float r0 = __builtin_amdgcn_rcpf(d);
    const float e0 = __builtin_fmaf(-d, r0, 1.0f);
    return {d, __builtin_fmaf(e0, r0, r0)};
}
constexpr float AWQ_TIE_BAND = 1.52587890625e-05f;          // 2^-16
__device__ __forceinline__ float fast_rint_quotient(float n, const Reciprocal &k, float &off)
{
    const float q0 = n * k.r;
    const float kq = __builtin_rintf(q0);
    off = fmaxf(off, fabsf(q0 - kq));
    return kq;
}
__device__ __forceinline__ bool near_tie(float off) { return off > 0.5f - AWQ_TIE_BAND; }

// fl(fp32(h) * s) for the two halves of a packed pair: the conversion is exact, so the mixed-
// precision multiply-add with a zero addend rounds once, exactly like convert-then-multiply
__device__ __forceinline__ void scaled_pair(uint32_t h2, float s_lo, float s_hi, float &lo, float &hi)
{
    asm("v_fma_mix_f32 %0, %2, %3, 0 op_sel_hi:[1,0,0]\n\t"
        "v_fma_mix_f32 %1, %2, %4, 0 op_sel:[1,0,0] op_sel_hi:[1,0,0]"
        : "=&v"(lo), "=&v"(hi)
        : "v"(h2), "v"(s_lo), "v"(s_hi));
}

// Range ratios of the clipping search (Sec. 3.2, weight clipping; objective and grid not
// specified there: per group, squared error of the weights or of the outputs on given rows).
struct ClipRatios {
    float v[AWQ_CLIP_MAX_RATIOS];
    int n;
};

// One wave owns group g of a range of consecutive row blocks: the 128 scale factors s of the
// group stay in registers, and the loads of the next tile are in flight while the current one
// is quantized.
// CLIP: before a group is quantized, its range [min, max] is tried shrunk by every ratio of
// the grid; the ratio with the smallest sum of squared differences between dequantized and
// scaled weights (differences in fp32, one rounding per operation; their squares summed in
// fp64) is used, the first one on ties.  choice[n*G+g] (optional) receives its index.
// ACT (with CLIP): the error of a trial is not that of the weights but the group's contribution
// to the layer output on up to 64 rows xs = x/s: sum_t (sum_k e[k] xs[t,k])^2.  That is a
// 16 x 128 by 128 x T product per tile and trial, and the lane layout of this kernel is the
// B-operand layout of v_mfma_f32_16x16x32_f16 (row l%16, columns 32 j + 8 (l/16) + 0..7 in
// step j): the errors go to the matrix core as they are, scaled by a power of two into fp16
// range, against the rows of xs held in registers as A operands for the wave's whole life (its
// group never changes).  Lane l receives the sums of its own row for tokens 4 (l/16) + 0..3 of
// every block of 16 rows; squares are added in fp64 and combined over the four lanes of the row.
// One matrix of a launch.  A launch quantizes up to QUANT_MAX_PROBLEMS matrices: its waves are
// numbered through all of them (`unit_begin` = first wave of a matrix), so that a pass over many
// small matrices (one decoder layer is seven) pays one launch and one run-out instead of one each.
struct QuantProblem {
    const uint4 *W;        // [N, K/8] runs of eight fp16
    const float4 *s;       // [K/4] or nullptr
    uint4 *qweight;
    uint16_t *scales;
    uint8_t *zeros;
    uint8_t *choice;       // CLIP: [N, G] or nullptr
    const uint4 *xs;       // ACT: [T, K/8]
    int G, NRB, rb_per_wave, unit_begin;
    int T, pad;
};
constexpr int QUANT_MAX_PROBLEMS = 16;
struct QuantArgs {
    QuantProblem p[QUANT_MAX_PROBLEMS];
    int count, num_units;
};

// Waves per SIMD the plain kernel is compiled for.  It needs about 130 registers, i.e. three waves
// per SIMD; forced into 128 for a fourth wave it spills four values per tile and the 224-matrix
// pass was measured slower (4.4 against 4.8 TB/s), so no minimum is requested.
#ifndef AWQ_QUANT_MIN_WAVES
#define AWQ_QUANT_MIN_WAVES 1
#endif

template <bool CLIP, bool ACT>
__global__ __launch_bounds__(256, CLIP ? 1 : AWQ_QUANT_MIN_WAVES) void quantize_pack_kernel(const QuantArgs A, const ClipRatios ratios)
{
    const int lane = threadIdx.x & 63;
    const int unit = __builtin_amdgcn_readfirstlane(blockIdx.x * 4 + (threadIdx.x >> 6));
    if (unit >= A.num_units) return;               // whole wave leaves together
    int pi = 0;
    for (int i = 1; i < A.count; ++i)
        if (unit >= A.p[i].unit_begin) pi = i;
    const QuantProblem &P = A.p[pi];
    const uint4 *__restrict__ W = P.W;
    const float4 *__restrict__ s = P.s;
    uint4 *__restrict__ qweight = P.qweight;
    uint16_t *__restrict__ scales = P.scales;
    uint8_t *__restrict__ zeros = P.zeros;
    uint8_t *__restrict__ choice = P.choice;
    const uint4 *__restrict__ xs = P.xs;
    const int G = P.G, NRB = P.NRB, rb_per_wave = P.rb_per_wave, T = P.T;
    const int local = unit - P.unit_begin;
    const int g = local % G, part = local / G;
    const int rb0 = part * rb_per_wave;
    const int rb1 = min(NRB, rb0 + rb_per_wave);
    const int r = lane & 15, c = lane >> 4;
    const int64_t K8 = (int64_t)G * 16;            // row length in 8-element runs

    // s for this lane's four runs (columns 32 j + 8 c + 0..7 of the group)
    float sv[4][8];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int run = g * 16 + 4 * j + c;
        if (s) {
            const float4 a = s[2 * run], b = s[2 * run + 1];
            sv[j][0] = a.x; sv[j][1] = a.y; sv[j][2] = a.z; sv[j][3] = a.w;
            sv[j][4] = b.x; sv[j][5] = b.y; sv[j][6] = b.z; sv[j][7] = b.w;
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) sv[j][e] = 1.0f;
        }
    }

    // A operands of the activation rows: token 16 tb + l%16, columns 32 j + 8 (l/16) + 0..7
    uint4 xa[ACT ? 4 : 1][4];
    const int tblocks = ACT ? (T + 15) >> 4 : 0;
    if (ACT) {
#pragma unroll
        for (int tb = 0; tb < 4; ++tb) {
            const int t = 16 * tb + r;
#pragma unroll
            for (int j = 0; j < 4; ++j)
                xa[tb][j] = t < T ? xs[(int64_t)t * K8 + g * 16 + 4 * j + c] : make_uint4(0, 0, 0, 0);
        }
    }

    auto load_tile = [&](uint4 (&raw)[4], int rb) {
        const int64_t n = (int64_t)rb * 16 + r;
#pragma unroll
        for (int j = 0; j < 4; ++j) raw[j] = W[n * K8 + g * 16 + 4 * j + c];
    };

    uint4 cur[4], nxt[4];
    if (rb0 < rb1) load_tile(cur, rb0);
    for (int rb = rb0; rb < rb1; ++rb) {
        if (rb + 1 < rb1) load_tile(nxt, rb + 1);

        float wp[4][8];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t h2[4] = {cur[j].x, cur[j].y, cur[j].z, cur[j].w};
#pragma unroll
            for (int e = 0; e < 8; e += 2) scaled_pair(h2[e >> 1], sv[j][e], sv[j][e + 1], wp[j][e], wp[j][e + 1]);
        }

        float mx = wp[0][0], mn = wp[0][0];
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                mx = fmaxf(mx, wp[j][e]);
                mn = fminf(mn, wp[j][e]);
            }
        mx = fmaxf(mx, __shfl_xor(mx, 16));
        mn = fminf(mn, __shfl_xor(mn, 16));
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        mn = fminf(mn, __shfl_xor(mn, 32));

        int best = 0;
        if (CLIP) {
            double best_err = 0.0;
            for (int i = 0; i < ratios.n; ++i) {
                const float mxr = mx * ratios.v[i], mnr = mn * ratios.v[i];
                float t32 = (mxr - mnr) / 15.0f;
                t32 = clampf(t32, 6.103515625e-05f, 65504.0f);
                const float tscale = (float)(half_t)t32;
                const float tzero = clampf(__builtin_rintf((-mnr) / tscale), 0.0f, 15.0f);
                const Reciprocal trc = make_reciprocal(tscale);
                double err = 0.0;
                // ACT: errors times 2^-e, e the exponent of the step, fit fp16 (|e[k]| <= 16 steps)
                const uint32_t sbits = __builtin_bit_cast(uint32_t, tscale);
                const float down = __builtin_bit_cast(float, (254u - ((sbits >> 23) & 255u)) << 23);
                half_t eh[4][8];
                // q - zero = clamp(rint(w'/step), -zero, 15 - zero): the same integers as
                // clamp(rint(w'/step) + zero, 0, 15) - zero
                const float tlo = -tzero, thi = 15.0f - tzero;
                auto accumulate = [&](auto rint_quotient) {
                    err = 0.0;
#pragma unroll
                    for (int j = 0; j < 4; ++j)
#pragma unroll
                        for (int e = 0; e < 8; ++e) {
                            const float lv = clampf(rint_quotient(wp[j][e]), tlo, thi);
                            const float dq = lv * tscale;
                            const float d = dq - wp[j][e];
                            if (ACT) eh[j][e] = (half_t)(d * down);
                            else err += (double)d * (double)d;
                        }
                };
                float toff = 0.0f;
                accumulate([&](float n) { return fast_rint_quotient(n, trc, toff); });
                if (__any(near_tie(toff))) accumulate([&](float n) { return __builtin_rintf(n / tscale); });
                if (ACT) {
                    for (int tb = 0; tb < tblocks; ++tb) {
                        floatx4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            half8_t b;
#pragma unroll
                            for (int e = 0; e < 8; ++e) b[e] = eh[j][e];
                            // tb is wave-uniform; the four A operands of a block are picked by it
                            const uint4 a = tb == 0 ? xa[0][j] : tb == 1 ? xa[1][j] : tb == 2 ? xa[2][j] : xa[3][j];
                            acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8_t, a), b, acc, 0, 0, 0);
                        }
#pragma unroll
                        for (int v = 0; v < 4; ++v) err += (double)acc[v] * (double)acc[v];
                    }
                    const double up = 1.0 / (double)down;          // a power of two
                    err = err * up * up;
                }
                // the four lanes of a row: every one of them ends up with the same bits
                err += __shfl_xor(err, 16);
                err += __shfl_xor(err, 32);
                if (i == 0 || err < best_err) {
                    best = i;
                    best_err = err;
                }
            }
            mx = mx * ratios.v[best];
            mn = mn * ratios.v[best];
        }

        const float range = mx - mn;
        float sc32 = range / 15.0f;
        sc32 = clampf(sc32, 6.103515625e-05f, 65504.0f);
        const half_t sc_h = (half_t)sc32;              // v_cvt_f16_f32, round-half-even
        const float scale = (float)sc_h;
        const float nmn = -mn;
        const float zr = nmn / scale;
        const float zero = clampf(__builtin_rintf(zr), 0.0f, 15.0f);
        const Reciprocal rc = make_reciprocal(scale);

        // a word is assembled as two exact fp32 integers of 16 bits (four nibbles each): the sums
        // of (q - zero) 16^i, with q - zero = clamp(rint(w'/step), -zero, 15 - zero) (the same
        // integers as clamp(rint(w'/step) + zero, 0, 15) - zero), plus zero * 0x1111 at the end
        uint32_t words[4];
        const float klo = -zero, khi = 15.0f - zero, zfill = zero * 4369.0f;
        auto assemble = [&](auto rint_quotient) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                float lo = zfill, hi = zfill;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float k = clampf(rint_quotient(wp[j][e]), klo, khi);
                    const int sh = nib_shift(e);            // 0,16,4,20,8,24,12,28
                    const float weight = (float)(1u << (sh & 15));
                    if (sh < 16) lo = __builtin_fmaf(k, weight, lo);
                    else hi = __builtin_fmaf(k, weight, hi);
                }
                words[j] = (uint32_t)lo | ((uint32_t)hi << 16);
            }
        };
        float off = 0.0f;
        assemble([&](float n) { return fast_rint_quotient(n, rc, off); });
        if (__any(near_tie(off))) assemble([&](float n) { return __builtin_rintf(n / scale); });
        const int64_t tile = (int64_t)rb * G + g;
        qweight[tile * 64 + lane] = make_uint4(words[0], words[1], words[2], words[3]);

        const uint32_t z = (uint32_t)zero;
        const uint32_t z_hi = __shfl_xor(z, 1);        // the odd row of the pair
        if (c == 0) {
            scales[tile * 16 + r] = __builtin_bit_cast(uint16_t, sc_h);
            if ((r & 1) == 0) zeros[tile * 8 + (r >> 1)] = (uint8_t)(z | (z_hi << 4));
            if (CLIP && choice) choice[((int64_t)rb * 16 + r) * G + g] = (uint8_t)best;
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) cur[j] = nxt[j];
    }
}

__global__ __launch_bounds__(256) void unpack_kernel(
    const uint4 *__restrict__ qweight, const uint16_t *__restrict__ scales,
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
        const uint4 q = qweight[(int64_t)tile * 64 + lane];
        const uint32_t words[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            uint32_t lo = 0, hi = 0;               // bytes e = 0..3 and 4..7
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                lo |= ((words[j] >> nib_shift(e)) & 0xFu) << (8 * e);
                hi |= ((words[j] >> nib_shift(e + 4)) & 0xFu) << (8 * e);
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

}  // namespace

namespace {

// One matrix as the host sees it.
struct QuantJob {
    const void *W;
    const float *s;
    int64_t N, K;
    void *qweight, *scales, *zeros;
    uint8_t *choice;
    const void *xs;
    int64_t T;
};

int quantize_check(const QuantJob &j, int group)
{
    if (!j.W || !j.qweight || !j.scales || !j.zeros) return AWQ_ERR_NULL_POINTER;
    int st = awq_check_weight_shape(j.N, j.K, group);
    if (st != AWQ_OK) return st;
    if (!awq_aligned16(j.W) || !awq_aligned16(j.qweight) || !awq_aligned16(j.scales) ||
        !awq_aligned16(j.zeros) || (j.s && !awq_aligned16(j.s)))
        return AWQ_ERR_MISALIGNED;
    return AWQ_OK;
}

// Launches for `count` validated matrices, QUANT_MAX_PROBLEMS per launch.  A wave keeps one group
// and walks down `rb_per_wave` row blocks; that number is chosen so that the waves of a launch
// about fill the chip once (three waves per SIMD, the kernel's register budget): more waves
// would queue behind the resident ones as a second, nearly empty round.
int quantize_launch(const QuantJob *jobs, int count, const ClipRatios *ratios, hipStream_t stream)
{
    const int RESIDENT_WAVES = 256 * 4 * (ratios ? 3 : AWQ_QUANT_MIN_WAVES == 4 ? 4 : 3);
    for (int first = 0; first < count; first += QUANT_MAX_PROBLEMS) {
        const int n = std::min(QUANT_MAX_PROBLEMS, count - first);
        int64_t tiles = 0;
        for (int i = 0; i < n; ++i) tiles += (jobs[first + i].N / 16) * (jobs[first + i].K / AWQ_GROUP);
        const int64_t per_wave = std::max<int64_t>(1, (tiles + RESIDENT_WAVES - 1) / RESIDENT_WAVES);
        QuantArgs A = {};
        int units = 0;
        bool act = false;
        for (int i = 0; i < n; ++i) {
            const QuantJob &j = jobs[first + i];
            QuantProblem &P = A.p[i];
            P.W = (const uint4 *)j.W;
            P.s = (const float4 *)j.s;
            P.qweight = (uint4 *)j.qweight;
            P.scales = (uint16_t *)j.scales;
            P.zeros = (uint8_t *)j.zeros;
            P.choice = j.choice;
            P.xs = (const uint4 *)j.xs;
            P.T = (int)j.T;
            P.G = (int)(j.K / AWQ_GROUP);
            P.NRB = (int)(j.N / 16);
            P.rb_per_wave = (int)std::min<int64_t>(per_wave, P.NRB);
            P.unit_begin = units;
            units += ((P.NRB + P.rb_per_wave - 1) / P.rb_per_wave) * P.G;
            act = act || j.xs;
        }
        A.count = n;
        A.num_units = units;
        const dim3 grid((unsigned)((units + 3) / 4)), block(256);
        if (ratios && act) quantize_pack_kernel<true, true><<<grid, block, 0, stream>>>(A, *ratios);
        else if (ratios) quantize_pack_kernel<true, false><<<grid, block, 0, stream>>>(A, *ratios);
        else quantize_pack_kernel<false, false><<<grid, block, 0, stream>>>(A, ClipRatios{});
        const int st = awq_launch_status();
        if (st != AWQ_OK) return st;
    }
    return AWQ_OK;
}

}  // namespace

extern "C" int awq_quantize_pack(const void *W_f16, const float *s, int64_t N, int64_t K,
                                 int group, void *qweight, void *scales, void *zeros,
                                 void *stream)
{
    const QuantJob j = {W_f16, s, N, K, qweight, scales, zeros, nullptr, nullptr, 0};
    const int st = quantize_check(j, group);
    return st != AWQ_OK ? st : quantize_launch(&j, 1, nullptr, (hipStream_t)stream);
}

extern "C" int awq_quantize_pack_multi(const awq_quantize_desc *descs, int count, int group, void *stream)
{
    if (!descs) return AWQ_ERR_NULL_POINTER;
    if (count < 1 || count > AWQ_QUANTIZE_MULTI_MAX) return AWQ_ERR_BAD_ARGUMENT;
    QuantJob jobs[AWQ_QUANTIZE_MULTI_MAX];
    for (int i = 0; i < count; ++i) {
        jobs[i] = {descs[i].W_f16, descs[i].s, descs[i].N, descs[i].K, descs[i].qweight, descs[i].scales,
                   descs[i].zeros, nullptr, nullptr, 0};
        const int st = quantize_check(jobs[i], group);
        if (st != AWQ_OK) return st;
    }
    return quantize_launch(jobs, count, nullptr, (hipStream_t)stream);
}

extern "C" int awq_quantize_pack_clip(const void *W_f16, const float *s, int64_t N, int64_t K,
                                      int group, const float *ratios, int n_ratios,
                                      const void *xs_f16, int64_t T, void *qweight, void *scales,
                                      void *zeros, uint8_t *choice, void *stream)
{
    if (!ratios) return AWQ_ERR_NULL_POINTER;
    if (xs_f16 && (T < 1 || T > AWQ_CLIP_MAX_ROWS)) return AWQ_ERR_BAD_SHAPE;
    if (xs_f16 && !awq_aligned16(xs_f16)) return AWQ_ERR_MISALIGNED;
    if (n_ratios < 1 || n_ratios > AWQ_CLIP_MAX_RATIOS) return AWQ_ERR_BAD_ARGUMENT;
    ClipRatios r = {};
    r.n = n_ratios;
    for (int i = 0; i < n_ratios; ++i) {
        if (!(ratios[i] > 0.0f && ratios[i] <= 1.0f)) return AWQ_ERR_BAD_ARGUMENT;
        r.v[i] = ratios[i];
    }
    const QuantJob j = {W_f16, s, N, K, qweight, scales, zeros, choice, xs_f16, T};
    const int st = quantize_check(j, group);
    return st != AWQ_OK ? st : quantize_launch(&j, 1, &r, (hipStream_t)stream);
}

extern "C" int awq_unpack(const void *qweight, const void *scales, const void *zeros,
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
    const int blocks = (num_tiles + 3) / 4;
    unpack_kernel<<<dim3(blocks), dim3(256), 0, (hipStream_t)stream>>>(
        (const uint4 *)qweight, (const uint16_t *)scales, (const uint8_t *)zeros, codes,
        (uint16_t *)scales_f16, zeros_u8, G, num_tiles);
    return awq_launch_status();
}
