// awq_decode_attention for gfx950: one decode step of the attention layer.
//
// Sec. 4.2, kernel fusion: the attention kernel evaluates the position embedding itself and
// writes the new key and value into caches that were allocated ahead.  One call
// takes the q, k, v rows the (fused) QKV projection produced for the current token, rotates q
// and k by the rotary embedding of the token's position, stores the rotated key and the value
// in the caches, and returns softmax(q K^T / sqrt(D)) V over all positions so far.
//
// The step is bound by reading the caches once (2 * L * Hkv * D * 2 bytes).  They are laid out
// [kv head][position][D], so the keys of a head are one contiguous stream.  A workgroup handles
// one query head and one slice of the positions; a wave takes four positions per step: lane
// l = 16 g + u holds dimensions 8 u .. 8 u + 7 (one 16-byte load) of position 4 i + g, the
// partial dot products are folded over the 16 lanes of a group with four xor-shuffles, and each
// group keeps a running (max, sum, weighted values) of its own positions, merged at the end
// (groups by shuffles, waves through LDS).  Slices are merged by a second, tiny kernel.
// The current token's key and value are taken from the inputs, not from the cache row that is
// written in the same launch, so no workgroup depends on another one's stores.
#include "awq_common.h"

#include <cmath>

namespace {

constexpr int AD = 128;                 // head dimension
constexpr int ATT_WAVES = 4;

// theta^(-2 i / 128), i = 0..63, computed once per call on the host in fp64
struct RopeTable {
    double inv_freq[AD / 2];
};

// q (or k) of one head, rotated: pairs (i, i + 64), angle pos * theta^(-2 i / 128).  The angle (a
// few thousand radians at long contexts) is formed and reduced to [-pi, pi] in fp64, sine and
// cosine of the reduced angle in fp32.  (a, b) are elements t and t + 64, inv_freq is entry t.
__device__ __forceinline__ void rope_pair(float a, float b, double inv_freq, int pos, float &lo, float &hi)
{
    const double ang = (double)pos * inv_freq;
    const double turns = __builtin_rint(ang * 0.15915494309189535);        // 1 / (2 pi)
    const float red = (float)(ang - turns * 6.283185307179586);
    const float sn = sinf(red), cs = cosf(red);
    lo = a * cs - b * sn;
    hi = b * cs + a * sn;
}

struct Running {
    float m, l;          // running maximum of the scores and sum of exp(score - m)
    float acc[8];        // sum of exp(score - m) * value, this lane's eight dimensions
};

__device__ __forceinline__ void absorb(Running &r, float score, const float (&val)[8])
{
    const float m_new = fmaxf(r.m, score);
    const float keep = __expf(r.m - m_new), add = __expf(score - m_new);
    r.l = r.l * keep + add;
#pragma unroll
    for (int e = 0; e < 8; ++e) r.acc[e] = r.acc[e] * keep + add * val[e];
    r.m = m_new;
}

__device__ __forceinline__ void merge(Running &r, float m2, float l2, const float (&acc2)[8])
{
    const float m_new = fmaxf(r.m, m2);
    // an empty side has m = -inf and l = 0: exp(-inf - finite) = 0, and two empty sides stay empty
    const float k1 = r.m == m_new ? 1.0f : __expf(r.m - m_new), k2 = m2 == m_new ? 1.0f : __expf(m2 - m_new);
    r.l = r.l * k1 + l2 * k2;
#pragma unroll
    for (int e = 0; e < 8; ++e) r.acc[e] = r.acc[e] * k1 + acc2[e] * k2;
    r.m = m_new;
}

// grid (H, splits); 256 threads.  partial: [H][splits][AD + 2] floats = (acc[128], m, l).
__global__ __launch_bounds__(256) void attention_partial_kernel(
    const half_t *__restrict__ q, const half_t *__restrict__ k, const half_t *__restrict__ v,
    half_t *__restrict__ k_cache, half_t *__restrict__ v_cache, int H, int Hkv, int Lmax, int pos,
    RopeTable tab, int chunk, float *__restrict__ partial)
{
    __shared__ float qs[AD];                         // rotated query times 1/sqrt(D)
    __shared__ float ks[AD];                         // rotated key of the current token (fp32)
    __shared__ float wave_state[ATT_WAVES][AD + 2];
    // all pointer arguments fetched in one round (the compiler would otherwise fetch each where
    // it is first needed, one scalar-cache miss after the other)
    asm volatile("" ::"s"(q), "s"(k), "s"(v), "s"(k_cache), "s"(v_cache), "s"(partial), "s"(H), "s"(Hkv),
                 "s"(Lmax), "s"(pos), "s"(chunk));
    const int h = blockIdx.x, split = blockIdx.y;
    const int g_kv = h / (H / Hkv);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int grp = lane >> 4, u = lane & 15;
    // what the rotary prologue needs (wave 0: the query, wave 1: the key; elements lane and
    // lane + 64), requested before the cache rows so that it is not waited for behind them
    const half_t *rsrc = wave == 1 ? k + (size_t)g_kv * AD : q + (size_t)h * AD;
    const half_t ra_h = rsrc[lane], rb_h = rsrc[lane + 64];
    const double rfreq = tab.inv_freq[lane];
    const int L = pos + 1;
    const int p0 = split * chunk, p1 = min(L, p0 + chunk);
    const uint4 *kbase = reinterpret_cast<const uint4 *>(k_cache + (size_t)g_kv * Lmax * AD) + u;
    const uint4 *vbase = reinterpret_cast<const uint4 *>(v_cache + (size_t)g_kv * Lmax * AD) + u;
    // positions of this lane group: p, p + 16, ...; the loads of the next four are in flight while
    // one is folded in.  The first ones go out before anything else: they do not depend on the
    // query, and the rotary prologue below runs while they travel.
    constexpr int AHEAD = 4;
    uint4 kq[AHEAD + 1], vq[AHEAD + 1];
    const int first = p0 + 4 * wave + grp;
#pragma unroll
    for (int a = 0; a < AHEAD; ++a) {
        // unconditional (a row that is not needed reads row 0 and is ignored): a predicated
        // load would be waited for on the spot
        const int pa = first + 16 * a, pe = pa < p1 ? pa : 0;
        kq[a] = kbase[(size_t)pe * (AD / 8)];
        vq[a] = vbase[(size_t)pe * (AD / 8)];
    }

    {
        // every wave rotates what it fetched (waves 2 and 3 discard the result): a rotation
        // only some waves need would have its loads moved down behind the cache rows
        float lo, hi;
        rope_pair((float)ra_h, (float)rb_h, rfreq, pos, lo, hi);
        if (wave == 0) {
            qs[lane] = lo * 0.08838834764831845f;    // 1 / sqrt(128)
            qs[lane + 64] = hi * 0.08838834764831845f;
        } else if (wave == 1) {
            ks[lane] = lo;
            ks[lane + 64] = hi;
            // the first query head of a kv group (first slice) files the token into the caches
            if (split == 0 && h % (H / Hkv) == 0) {
                half_t *kd = k_cache + ((size_t)g_kv * Lmax + pos) * AD;
                half_t *vd = v_cache + ((size_t)g_kv * Lmax + pos) * AD;
                kd[lane] = (half_t)lo;
                kd[lane + 64] = (half_t)hi;
                vd[lane] = v[(size_t)g_kv * AD + lane];
                vd[lane + 64] = v[(size_t)g_kv * AD + lane + 64];
            }
        }
    }
    __syncthreads();

    float qf[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) qf[e] = qs[8 * u + e];
    Running r;
    r.m = -__builtin_inff();
    r.l = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) r.acc[e] = 0.f;

    for (int p = first; p < p1; p += 16 * (AHEAD + 1)) {
#pragma unroll
        for (int a = 0; a <= AHEAD; ++a) {
            const int pc = p + 16 * a;                       // position folded in now
            const int pn = pc + 16 * AHEAD;                  // position requested now
            const int pne = pn < p1 ? pn : 0;
            kq[(a + AHEAD) % (AHEAD + 1)] = kbase[(size_t)pne * (AD / 8)];
            vq[(a + AHEAD) % (AHEAD + 1)] = vbase[(size_t)pne * (AD / 8)];
            if (pc < p1) {
                float kf[8], vf[8];
                if (pc == pos) {                             // the token of this call: from the inputs
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        kf[e] = ks[8 * u + e];
                        vf[e] = (float)v[(size_t)g_kv * AD + 8 * u + e];
                    }
                } else {
                    const half_t *kh = reinterpret_cast<const half_t *>(&kq[a]);
                    const half_t *vh = reinterpret_cast<const half_t *>(&vq[a]);
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        kf[e] = (float)kh[e];
                        vf[e] = (float)vh[e];
                    }
                }
                float s = 0.f;
#pragma unroll
                for (int e = 0; e < 8; ++e) s += qf[e] * kf[e];
                s += __shfl_xor(s, 1);
                s += __shfl_xor(s, 2);
                s += __shfl_xor(s, 4);
                s += __shfl_xor(s, 8);
                absorb(r, s, vf);
            }
        }
    }
    // the four groups of the wave (lanes u, u+16, u+32, u+48 hold the same dimensions)
#pragma unroll
    for (int d = 16; d <= 32; d <<= 1) {
        const float m2 = __shfl_xor(r.m, d), l2 = __shfl_xor(r.l, d);
        float a2[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) a2[e] = __shfl_xor(r.acc[e], d);
        merge(r, m2, l2, a2);
    }
    if (grp == 0) {
#pragma unroll
        for (int e = 0; e < 8; ++e) wave_state[wave][8 * u + e] = r.acc[e];
        if (u == 0) {
            wave_state[wave][AD] = r.m;
            wave_state[wave][AD + 1] = r.l;
        }
    }
    __syncthreads();
    if (tid < AD) {
        float m = wave_state[0][AD];
#pragma unroll
        for (int w = 1; w < ATT_WAVES; ++w) m = fmaxf(m, wave_state[w][AD]);
        float l = 0.f, a = 0.f;
#pragma unroll
        for (int w = 0; w < ATT_WAVES; ++w) {
            const float mw = wave_state[w][AD];
            const float kf = mw == m ? 1.0f : __expf(mw - m);
            l += wave_state[w][AD + 1] * kf;
            a += wave_state[w][tid] * kf;
        }
        float *dst = partial + ((size_t)h * gridDim.y + split) * (AD + 2);
        dst[tid] = a;
        if (tid == 0) {
            dst[AD] = m;
            dst[AD + 1] = l;
        }
    }
}

// grid H, 256 threads: merge the slices of a head in a fixed order.  The head's partial results
// (at most 64 x 130 floats) are first copied to LDS with coalesced loads: read one by one from
// memory they would be a chain of dependent round trips.
__global__ __launch_bounds__(256) void attention_merge_kernel(const float *__restrict__ partial,
                                                              int splits, half_t *__restrict__ out)
{
    __shared__ float ps[64 * (AD + 2)];
    const int h = blockIdx.x, t = threadIdx.x;
    const float *p = partial + (size_t)h * splits * (AD + 2);
    asm volatile("" ::"s"(partial), "s"(splits), "s"(out));       // arguments in one round
    const int n = splits * (AD + 2);
    for (int base = 0; base < n; base += 256 * 9) {               // nine loads in flight: 16 slices in one round
        float tmp[9];
#pragma unroll
        for (int e = 0; e < 9; ++e) {
            const int i = base + 256 * e + t;
            tmp[e] = p[i < n ? i : n - 1];
        }
#pragma unroll
        for (int e = 0; e < 9; ++e) {
            const int i = base + 256 * e + t;
            if (i < n) ps[i] = tmp[e];
        }
    }
    __syncthreads();
    if (t >= AD) return;
    float m = -__builtin_inff();
    for (int s = 0; s < splits; ++s) m = fmaxf(m, ps[s * (AD + 2) + AD]);
    float l = 0.f, a = 0.f;
    for (int s = 0; s < splits; ++s) {
        const float ms = ps[s * (AD + 2) + AD];
        const float kf = ms == m ? 1.0f : __expf(ms - m);
        l += ps[s * (AD + 2) + AD + 1] * kf;
        a += ps[s * (AD + 2) + t] * kf;
    }
    out[(size_t)h * AD + t] = (half_t)(a / l);
}

int attention_splits(int64_t H, int64_t L)
{
    // about two workgroups per CU (the best of 256, 512 and 1024 at 32 heads x 2048 positions),
    // at least 64 positions each
    int64_t s = (512 + H - 1) / H;
    const int64_t most = (L + 63) / 64;
    if (s > most) s = most;
    if (s < 1) s = 1;
    if (s > 64) s = 64;
    return (int)s;
}

}  // namespace

extern "C" size_t awq_decode_attention_workspace_bytes(int64_t H, int64_t D, int64_t L)
{
    if (H <= 0 || D != AD || L <= 0) return 0;
    return (size_t)H * attention_splits(H, L) * (AD + 2) * sizeof(float);
}

extern "C" int awq_decode_attention(const void *q_f16, const void *k_f16, const void *v_f16,
                                    void *k_cache_f16, void *v_cache_f16, int64_t H, int64_t Hkv,
                                    int64_t D, int64_t Lmax, int64_t pos, float rope_theta,
                                    void *out_f16, void *workspace, size_t workspace_bytes,
                                    void *stream)
{
    if (!q_f16 || !k_f16 || !v_f16 || !k_cache_f16 || !v_cache_f16 || !out_f16 || !workspace)
        return AWQ_ERR_NULL_POINTER;
    if (D != AD || H <= 0 || Hkv <= 0 || H % Hkv != 0 || H > 65535 || Lmax <= 0 || Lmax > (int64_t)1 << 24 ||
        pos < 0 || pos >= Lmax)
        return AWQ_ERR_BAD_SHAPE;
    if (!(rope_theta > 1.0f)) return AWQ_ERR_BAD_ARGUMENT;
    if (!awq_aligned16(q_f16) || !awq_aligned16(k_f16) || !awq_aligned16(v_f16) ||
        !awq_aligned16(k_cache_f16) || !awq_aligned16(v_cache_f16) || !awq_aligned16(out_f16) ||
        !awq_aligned16(workspace))
        return AWQ_ERR_MISALIGNED;
    const int64_t L = pos + 1;
    if (workspace_bytes < awq_decode_attention_workspace_bytes(H, D, L)) return AWQ_ERR_WORKSPACE_TOO_SMALL;
    const int splits = attention_splits(H, L);
    int chunk = (int)((L + splits - 1) / splits);
    chunk = (chunk + 15) / 16 * 16;                  // whole steps of the four waves
    RopeTable tab;
    for (int i = 0; i < AD / 2; ++i) tab.inv_freq[i] = pow((double)rope_theta, -2.0 * i / AD);
    attention_partial_kernel<<<dim3((unsigned)H, (unsigned)splits), dim3(256), 0, (hipStream_t)stream>>>(
        (const half_t *)q_f16, (const half_t *)k_f16, (const half_t *)v_f16, (half_t *)k_cache_f16,
        (half_t *)v_cache_f16, (int)H, (int)Hkv, (int)Lmax, (int)pos, tab, chunk, (float *)workspace);
    int st = awq_launch_status();
    if (st != AWQ_OK) return st;
    attention_merge_kernel<<<dim3((unsigned)H), dim3(256), 0, (hipStream_t)stream>>>(
        (const float *)workspace, splits, (half_t *)out_f16);
    return awq_launch_status();
}
