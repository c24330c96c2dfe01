// Host/device interface of the streaming decode kernel (awq_gemv_stream.hip).
#pragma once

#include "awq_common.h"

constexpr int GEMV_MAX_PROBLEMS = 56;     // 56 x 64 B of kernel arguments (limit: 4 KB)
constexpr int AWQ_GEMV_STREAM_UNFIT = 1;    // internal: shape not covered, use the batch kernel

// One linear of a grouped decode launch.  The caller fills the pointers and N, K; the
// launcher fills the planning fields.
struct GemvProblem {
    const half_t *x;          // [M,K]
    const uint4 *q;           // packed codes
    const uint16_t *sc;       // steps
    const uint8_t *zp;        // zero points
    half_t *y;                // [M,N]
    int N, K;                 // N: features of the whole linear = row stride of y
    int plan;                 // log2 of the waves that split K for one row block, and
                              // (<< 4) the row-block iterations per workgroup
    int nrb;                  // 16-row blocks of this entry (q, sc, zp, y point at its first one)
};

struct GemvLaunch {
    // first workgroup of each linear in the grid; kept together (and first) so that finding the
    // linear of a workgroup touches one or two cache lines of the kernel arguments, not one per
    // linear
    int wg_begin[GEMV_MAX_PROBLEMS];
    GemvProblem p[GEMV_MAX_PROBLEMS];
    int count;
    int M;
    int logW;                 // log2 of the waves per workgroup
    int mlog;                 // log2 of M rounded up to a power of two
};

static_assert(sizeof(GemvLaunch) <= 4096, "kernel arguments are limited to 4 KB");

// Operators fused into a linear of a grouped launch (Sec. 4.2, kernel fusion).
constexpr int GEMV_MAX_FUSED = 24;        // linears per fused launch (24 more bytes each)
constexpr int GEMV_PRE_NONE = 0, GEMV_PRE_RMSNORM = 1, GEMV_PRE_SCALE = 2;
struct GemvFusedExtra {
    const half_t *pre;        // RMSNORM, SCALE: [K] fp16 factors (gamma / s, 1 / s); else unused
    const half_t *res;        // [M,N] fp16 added to the output, or null
    float eps;
    int pre_op;
};

template <bool FUSED> struct GemvArgs {
    GemvLaunch L;
};
template <> struct GemvArgs<true> {
    GemvLaunch L;
    GemvFusedExtra e[GEMV_MAX_FUSED];
};
static_assert(sizeof(GemvArgs<true>) <= 4096, "kernel arguments are limited to 4 KB");

// Chained launch: up to CHAIN_MAX_STAGES stages of up to CHAIN_MAX_ENTRIES linears each, a stage
// may read what earlier stages wrote.  sync: CHAIN_SYNC_BYTES of zeroed device memory.
constexpr int CHAIN_MAX_STAGES = 4, CHAIN_MAX_ENTRIES = 10;
#ifndef AWQ_CHAIN_SHARDS
#define AWQ_CHAIN_SHARDS 16
#endif
constexpr int CHAIN_SHARDS = AWQ_CHAIN_SHARDS, CHAIN_SHARD_STRIDE = 32;            // words: one cache line per shard
constexpr int CHAIN_SYNC_BYTES = 4 * CHAIN_SHARD_STRIDE * (1 + CHAIN_SHARDS * (CHAIN_MAX_STAGES - 1));
int awq_gemv_chain_launch(const GemvProblem *const *problems, const GemvFusedExtra *const *extras, const int *counts,
                          int nstages, int M, uint32_t *sync, int spin_limit, hipStream_t stream);

int awq_gemv_stream_launch(const GemvProblem *problems, int count, int M, hipStream_t stream);
// grouped decode launch for more than four tokens: activations through LDS, any K
int awq_gemv_rows_launch(const GemvProblem *problems, int count, int M, hipStream_t stream,
                         const int *first_row = nullptr);
// the same for linears in the 3-bit packed layout (q then points at 12-byte slots)
int awq_gemv_stream_launch_w3(const GemvProblem *problems, int count, int M, hipStream_t stream);
// the 4-bit launch with a normalisation in front of and/or a residual behind each linear; every
// linear must fit (awq_gemv_stream_fits), count <= GEMV_MAX_FUSED
int awq_gemv_stream_launch_fused(const GemvProblem *problems, const GemvFusedExtra *extra, int count,
                                 int M, hipStream_t stream);
// whether a linear of this shape can be part of a grouped launch at this M
bool awq_gemv_stream_fits(int N, int K, int M);
