/*
 * awq_mi355x.h -- C ABI of the MI355X (gfx950) W4A16 group-quantized linear library.
 *
 * Method: AWQ, arXiv 2306.00978.  Weights W[N,K] (out-features x in-features) are
 * quantized to 4-bit codes in groups of 128 consecutive input channels with one
 * fp16 step ("scale") and one uint4 zero point per group, after folding the
 * per-input-channel activation-aware scale s into them (Sec. 3.2, Eq. 1-2).  The
 * layer is evaluated as y = x' * dequant(q)^T with dequantization fused into the
 * matrix-vector / matrix-matrix kernel (Sec. 4.2), where x' = x / s (Eq. 4).
 *
 * Conventions for every call below
 *   - Tensor pointers are DEVICE pointers (HIP global memory) owned by the caller;
 *     size/out-parameter pointers (size_t*) are HOST pointers.  The library never
 *     allocates, frees or synchronises.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All
 *     work is enqueued on it and may still be running when the call returns.
 *   - Shapes: N % 16 == 0, K % 128 == 0, group == 128, all sizes > 0.
 *     Tensor pointers must be 16-byte aligned.
 *   - Return value: AWQ_OK (0) or a negative awq_status.  Arguments are validated
 *     before anything is launched, so on a validation error no output is touched.
 *   - Calls on distinct streams, from one or several host threads, may run concurrently as
 *     long as their outputs (and workspaces) do not overlap.  The library keeps no state between
 *     calls except per-device "kernel attribute already raised" flags and the diagnostic of
 *     awq_last_grouped_plan (relaxed atomics), and the built-in scratch of
 *     awq_w4a16_linear_static, whose calls must not overlap on one GPU.  It reads no environment
 *     variable.
 *
 * Packed layout, version 1 (what awq_quantize_pack writes and awq_w4a16_linear reads)
 *   qweight : N*K/2 bytes; tiles of 16 rows x 128 columns (1024 B), tile index
 *             (n/16)*(K/128) + k/128.  A tile is 64 slots of 16 B; slot
 *             (n%16) + 16*c holds, in its little-endian 32-bit word j (0..3), the
 *             codes of columns 32*j + 8*c + e (e = 0..7), element e in nibble
 *             {0,4,1,5,2,6,3,7}[e].
 *   scales  : [N/16][K/128][16] fp16, row (n%16) innermost.
 *   zeros   : [N/16][K/128][8] bytes, byte b = row 2b (low nibble), row 2b+1 (high).
 */
#ifndef AWQ_MI355X_H
#define AWQ_MI355X_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum awq_status {
    AWQ_OK = 0,
    AWQ_ERR_NULL_POINTER = -1,
    AWQ_ERR_BAD_SHAPE = -2,         /* size <= 0, K % 128 != 0, N % 16 != 0 */
    AWQ_ERR_UNSUPPORTED_GROUP = -3, /* group != 128 */
    AWQ_ERR_MISALIGNED = -4,        /* a tensor pointer is not 16-byte aligned */
    AWQ_ERR_WORKSPACE_TOO_SMALL = -5,
    AWQ_ERR_HIP = -6,               /* the HIP runtime refused a launch */
    AWQ_ERR_BAD_ARGUMENT = -7,      /* a scalar argument is out of range (e.g. alpha) */
    AWQ_ERR_SCRATCH_LIMIT = -8      /* awq_w4a16_linear_static: the shape needs more than the built-in scratch */
} awq_status;

/* Version of the packed layout / ABI (currently 1). */
int awq_version(void);

/* Static, human-readable name of a status code (never NULL). */
const char *awq_status_string(int status);

/* Export aid, not part of the method: a 64-byte header for a file that stores packed arrays
 * (magic, version of the packed layout, bit width, group size, shape, bytes of the three arrays).
 * awq_blob_header_init fills it for bits in {4, 3, 2} (the layouts of awq_quantize_pack, _w3, _w2),
 * with the shape rules of that layout; awq_blob_header_check accepts exactly what init would have
 * written for the header's own bits / N / K / group with this library's layout version, and
 * returns AWQ_ERR_BAD_ARGUMENT for anything else (another version, a damaged field).  HOST
 * pointers; nothing is launched. */
typedef struct awq_blob_header {
    char magic[8];                  /* "AWQgfx95" */
    uint32_t layout_version, bits, group, reserved;
    int64_t N, K;
    uint64_t qweight_bytes, scales_bytes, zeros_bytes;
} awq_blob_header;
int awq_blob_header_init(awq_blob_header *h, int bits, int64_t N, int64_t K, int group);
int awq_blob_header_check(const awq_blob_header *h);

/* Measurement aid, not part of the method: streams `bytes` (rounded down to a multiple of 16) of
 * a device buffer with 128-bit loads and discards them -- the read bandwidth this machine
 * reaches on a buffer of that size, against which the decode kernels are stated.  sink: device
 * word, written only in a one-in-2^32 case. */
int awq_read_probe(const void *buffer, size_t bytes, uint32_t *sink, void *stream);

/* Bytes of the three packed arrays for an [N,K] weight.  Host pointers; any of
 * the three may be NULL. */
int awq_packed_sizes(int64_t N, int64_t K, int group, size_t *qweight_bytes,
                     size_t *scales_bytes, size_t *zeros_bytes);

/* Sec. 3.2, Eq. 5: s[k] = max(mean_t |X[t,k]|, 1e-4)^alpha, the activation-aware
 * per-input-channel scale.  X [T,K] fp16 row-major (device), s [K] fp32 (device,
 * written).  0 <= alpha <= 1.  K % 8 == 0.  fp32 arithmetic. */
int awq_act_scale(const void *X_f16, int64_t T, int64_t K, float alpha, float *s,
                  void *stream);

/* The same computation for up to AWQ_ACT_SCALE_MULTI_MAX matrices in one call (16 per launch),
 * each result bit for bit that of awq_act_scale on its own.  The sums are per column, so a
 * launch has K / 64 workgroups per matrix: one matrix of K = 4096 occupies a quarter of the
 * chip, the four distinct inputs of a decoder layer (Sec. 3.2 calibrates every linear on its own
 * input) fill it.  The matrices may differ in T and K; outputs must not overlap.  `descs` is a
 * HOST array, read before the call returns. */
typedef struct awq_act_scale_desc {
    const void *X_f16;     /* [T,K] fp16 row-major, device */
    int64_t T, K;
    float *s;              /* [K] fp32, device, written */
} awq_act_scale_desc;
#define AWQ_ACT_SCALE_MULTI_MAX 64
int awq_act_scale_multi(const awq_act_scale_desc *descs, int count, float alpha, void *stream);

/* Sec. 3.2, Eq. 4: the diag(s)^-1 X factor, applied once by the producer of x:
 * xs[m,k] = fp16(fp32(x[m,k]) / s[k]) (correctly rounded).  x, xs [M,K] fp16
 * (device; xs may alias x), s [K] fp32 (device).  K % 8 == 0. */
int awq_apply_inv_scale(const void *x_f16, const float *s, int64_t M, int64_t K,
                        void *xs_f16, void *stream);

/* Sec. 4.2 (kernel fusion: the operators of the normalisation in one kernel) with the 1/s factor
 * of Eq. 4 folded in (Sec. 3.2: that factor belongs to the producer of x): RMS form,
 *   xs[m,k] = fp16( x[m,k] / sqrt(mean_k x[m,k]^2 + eps) * gamma[k] / s[k] ),  fp32 inside.
 * x, xs [M,K] fp16 (device; xs may alias x), gamma [K] fp16 (device), s [K] fp32 (device) or
 * NULL (= ones), eps >= 0.  K % 8 == 0.  The result feeds awq_w4a16_linear directly. */
int awq_rmsnorm_inv_scale(const void *x_f16, const void *gamma_f16, const float *s, int64_t M,
                          int64_t K, float eps, void *xs_f16, void *stream);

/* The gated activation between the gate/up and the down projection of a Llama-style MLP (one
 * of the element-wise operators that Sec. 4.2 fuses): out[i] = fp16(silu(gate[i]) * up[i]),
 * fp32 inside.  gate, up, out: n fp16 elements (device; out may alias either), n % 8 == 0. */
int awq_silu_mul(const void *gate_f16, const void *up_f16, int64_t n, void *out_f16, void *stream);

/* Sec. 3.2, Eq. 1-2 and Sec. 4.2 (weight packing): quantize W*diag(s) per group of
 * 128 input channels and write the packed layout.
 *   w' = fp32(W)*s;  scale = fp16(clamp((max-min)/15, 2^-14, 65504));
 *   zero = clamp(rint(-min/scale), 0, 15);  q = clamp(rint(w'/scale)+zero, 0, 15)
 * in IEEE binary32, round-half-even, no contraction.
 * W_f16 [N,K] fp16 row-major (device, read); s [K] fp32 (device) or NULL (= ones);
 * qweight/scales/zeros: device buffers of awq_packed_sizes() bytes (written). */
int awq_quantize_pack(const void *W_f16, const float *s, int64_t N, int64_t K, int group,
                      void *qweight, void *scales, void *zeros, void *stream);

/* One matrix of awq_quantize_pack_multi: the arguments of awq_quantize_pack. */
typedef struct awq_quantize_desc {
    const void *W_f16;     /* [N,K] fp16 row-major, device */
    const float *s;        /* [K] fp32, device, or NULL (= ones) */
    int64_t N, K;
    void *qweight;         /* device buffers of awq_packed_sizes(N, K) bytes, written */
    void *scales;
    void *zeros;
} awq_quantize_desc;

#define AWQ_QUANTIZE_MULTI_MAX 64

/* The same computation as `count` calls of awq_quantize_pack (Sec. 3.2, Eq. 1-2; Sec. 4.2 packing),
 * bit for bit, in one kernel launch per 16 matrices: quantizing a 4096 x 4096 matrix takes about
 * as long as a launch, so a pass over a model's matrices (seven per decoder layer) runs faster
 * grouped.  The matrices may differ in shape; outputs must not overlap.  `descs` is a HOST array
 * of 1..AWQ_QUANTIZE_MULTI_MAX entries, read before the call returns. */
int awq_quantize_pack_multi(const awq_quantize_desc *descs, int count, int group, void *stream);

#define AWQ_CLIP_MAX_RATIOS 32
#define AWQ_CLIP_MAX_ROWS 64

/* Sec. 3.2, weight clipping (named there in one sentence as a second step that lowers the squared
 * quantization error; objective, grid and granularity are not given, this is the reading taken): awq_quantize_pack with a
 * search per quantization group.  The group's range [min, max] of w' = W*s is shrunk to
 * [r*min, r*max] for every r of `ratios`, the group is quantized with that range by the
 * formulas of awq_quantize_pack (values outside it saturate at code 0 or 15), and the r with
 * the smallest sum over the group of ((q - zero)*scale - w')^2 is used (differences in
 * binary32, one rounding per operation; squares summed in binary64; the first r wins a tie).
 * With xs_f16 != NULL the error of a trial is instead the group's contribution to the layer
 * output on the rows xs = x/s [T,K] fp16 (device, 1 <= T <= AWQ_CLIP_MAX_ROWS; take a sample
 * of a larger calibration set): sum_t (sum_k ((q - zero)*scale - w')[k] * xs[t,k])^2, the
 * counterpart of Eq. 4 for one group.  Here the inner sums run on the matrix cores from
 * errors rounded to fp16 (relative 2^-11), so among trials whose errors agree to about 1e-3
 * the choice is not unique; the codes are always exactly those of the chosen ratio.
 *   ratios: HOST array of 1..AWQ_CLIP_MAX_RATIOS values in (0, 1], read before the call
 *   returns; choice: device [N, K/128] bytes, row-major, receives the index of the winning
 *   ratio of every group, or NULL.  Everything else as awq_quantize_pack. */
int awq_quantize_pack_clip(const void *W_f16, const float *s, int64_t N, int64_t K, int group,
                           const float *ratios, int n_ratios, const void *xs_f16, int64_t T,
                           void *qweight, void *scales, void *zeros, uint8_t *choice,
                           void *stream);

/* Inverse of the packing (export / test path): codes [N,K] one code per byte,
 * scales_f16 [N,K/128] fp16, zeros_u8 [N,K/128] one zero point per byte, all
 * device, row-major, written.  Any of the three outputs may be NULL (skipped). */
int awq_unpack(const void *qweight, const void *scales, const void *zeros, int64_t N,
               int64_t K, int group, uint8_t *codes, void *scales_f16, uint8_t *zeros_u8,
               void *stream);

/* Bytes of scratch awq_w4a16_linear can use for this shape (0 if none; 0 for invalid shapes as
 * well, awq_w4a16_linear reports those).  Only a prefill of a few hundred tokens uses it: there the
 * matrix-matrix kernel has far fewer output tiles (ceil(M/128) * N/256) than the chip has CUs, and
 * with the workspace it cuts K into 2..8 ranges, one workgroup per tile and range, whose fp32
 * partial tiles (ranges * M * N * 4 bytes) a second kernel adds.  The workspace is optional: with
 * NULL the call runs without it (1.2 to 2.9 times slower at 50..1000 tokens). */
size_t awq_linear_workspace_bytes(int64_t M, int64_t N, int64_t K, int group);

/* Sec. 4.2 (on-the-fly dequantization fused into the MV / MM kernel):
 *   y[m,n] = fp16( sum_k fp32(x[m,k]) * (q[n,k] - zero[n,k/128]) * scale[n,k/128] )
 * with fp32 accumulation.  x_f16 [M,K] fp16 row-major, already divided by s;
 * qweight/scales/zeros as written by awq_quantize_pack; y_f16 [M,N] fp16 row-major
 * (written).  M <= 16 takes the decode path (streams the packed weights once), 17..128 tokens
 * go through the decode kernels in blocks of 16 (one grouped launch where the shape allows it;
 * the last block is moved back to hold 16 tokens, so a few tokens are computed twice with
 * identical results), larger M the prefill path (MFMA tiles; with the workspace also from 49 tokens on where that
 * is estimated to be faster).  `workspace` may be NULL; if it is given where
 * awq_linear_workspace_bytes() is not 0 it must hold that many bytes (AWQ_ERR_WORKSPACE_TOO_SMALL)
 * and be 16-byte aligned (AWQ_ERR_MISALIGNED); its contents are undefined afterwards.  Results with and without the workspace
 * differ by the order of the fp32 sums only. */
int awq_w4a16_linear(const void *x_f16, const void *qweight, const void *scales,
                     const void *zeros, void *y_f16, int64_t M, int64_t N, int64_t K,
                     int group, void *workspace, size_t workspace_bytes, void *stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): awq_w4a16_linear with the scratch of its K-range prefill
 * form taken from an array built into the library instead of a caller's workspace.  Same kernels,
 * same results bit for bit as awq_w4a16_linear with a workspace of awq_linear_workspace_bytes().
 * The call allocates and frees nothing and calls no allocating routine.
 *   - The array is AWQ_STATIC_SCRATCH_BYTES (32 MiB, awq_static_scratch_bytes()) of device memory
 *     per GPU the library is used on, held until the process ends; it covers the Llama-2-7B
 *     shapes up to 1024 tokens.  A shape whose awq_linear_workspace_bytes() exceeds it is refused
 *     with AWQ_ERR_SCRATCH_LIMIT before anything is launched (use awq_w4a16_linear, with or
 *     without a workspace).  Shapes that need no scratch (decode, M = 2048) never touch it.
 *   - All calls on one GPU share that one array.  Nothing in it has to start at zero (every word
 *     a launch reads was written by the same call before), so calls in sequence on one stream
 *     need no clearing in between; calls that OVERLAP on one GPU (two streams, two threads) race
 *     on it and give undefined results: serialise them, or use awq_w4a16_linear with workspaces
 *     of your own.
 *   - The array's device address is looked up on the first call on each device (with that device
 *     current); make that first call outside a graph capture.
 * Arguments, layouts and every other error as for awq_w4a16_linear. */
#define AWQ_STATIC_SCRATCH_BYTES ((size_t)32 << 20)
size_t awq_static_scratch_bytes(void);
int awq_w4a16_linear_static(const void *x_f16, const void *qweight, const void *scales,
                            const void *zeros, void *y_f16, int64_t M, int64_t N, int64_t K,
                            int group, void *stream);

/* One linear of a grouped decode call: the arguments of awq_w4a16_linear without M. */
typedef struct awq_linear_desc {
    const void *x_f16;     /* [M,K] fp16 row-major, device */
    const void *qweight;   /* packed arrays of this linear, device */
    const void *scales;
    const void *zeros;
    void *y_f16;           /* [M,N] fp16 row-major, device, written */
    int64_t N, K;
} awq_linear_desc;

#define AWQ_MULTI_MAX 56

/* Sec. 4.2 (kernel fusion: several projections in one kernel, because a decode
 * kernel is about as short as a launch): the same computation as `count` calls of
 * awq_w4a16_linear with the same M <= 16, in ONE kernel launch (up to four tokens a linear whose
 * K is too long for the register-resident activations takes a launch of its own; from five
 * tokens on the activations go through LDS and any K is in the one launch).  The linears are
 * independent (none may read another's output; outputs must not overlap); they may
 * share x (Q/K/V, gate/up) or not.  `descs` is a HOST array of 1..AWQ_MULTI_MAX
 * entries, read before the call returns.  Workspace as for awq_w4a16_linear
 * (currently none needed).  Results obey the same tolerance as the single calls but
 * need not be bit-identical to them (the summation order differs); a given call is
 * deterministic. */
int awq_w4a16_linear_multi(const awq_linear_desc *descs, int count, int64_t M, int group,
                           void *workspace, size_t workspace_bytes, void *stream);

/* Sec. 4.2 (kernel fusion of the operators around a linear): a grouped decode call whose linears
 * may carry a normalisation in front and a residual behind, so that a decoder layer needs no
 * launch of its own for either:
 *   pre_op == AWQ_PRE_RMSNORM: the linear runs on
 *       x'[m,k] = fp16( x[m,k] * rsqrt(mean_k x[m,k]^2 + eps) * pre[k] ),
 *     pre_f16 [K] fp16 (device, 16-byte aligned) = norm weight / AWQ scale s of Eq. 4 (the
 *     composition awq_rmsnorm_inv_scale computes with gamma and s apart), fp32 inside;
 *   pre_op == AWQ_PRE_SCALE: the division by s of Eq. 4 as a multiplication inside the launch,
 *       x'[m,k] = fp16( x[m,k] * pre[k] ),  pre_f16 [K] fp16 = 1/s (for a linear whose input
 *     comes from an operator the factor cannot be folded into);
 *   residual_f16 != NULL: y[m,n] = fp16( residual[m,n] + sum ), [M,N] fp16 (device); it may be
 *     y_f16 itself (in-place accumulation into the hidden state).
 * A call with one linear and pre_op == AWQ_PRE_NONE runs at every decode shape.  Otherwise every
 * linear must fit the streaming decode kernel at this M: its activations stay in the
 * registers of the at most eight waves that share a row block, 8192 / M' columns per wave with
 * M' = M rounded up to a power of two (so K <= 65536 / M', and K not so short that a wave would
 * be left without columns).  awq_w4a16_linear_fused_fits() returns 1 for a shape that does, 0
 * otherwise; the call returns AWQ_ERR_BAD_SHAPE for one that does not (use the separate calls).
 * M <= 16, count <= AWQ_FUSED_MAX.  `descs` is a HOST array, read before the call returns. */
#define AWQ_PRE_NONE 0
#define AWQ_PRE_RMSNORM 1
#define AWQ_PRE_SCALE 2
#define AWQ_FUSED_MAX 24
typedef struct awq_fused_desc {
    awq_linear_desc linear;
    const void *pre_f16;        /* AWQ_PRE_RMSNORM, AWQ_PRE_SCALE: [K] fp16 factors; else ignored */
    const void *residual_f16;   /* [M,N] fp16 or NULL */
    float eps;
    int pre_op;
} awq_fused_desc;
int awq_w4a16_linear_fused_multi(const awq_fused_desc *descs, int count, int64_t M, int group,
                                 void *stream);
int awq_w4a16_linear_fused_fits(int64_t N, int64_t K, int64_t M, int group);

/* Sec. 4.2 (kernel fusion; the generation stage is memory-bound and its kernels are as short as a
 * launch): the linears of a decode step in the order their data dependences impose, in ONE launch.
 * A chain is 1..AWQ_CHAIN_MAX_STAGES stages; a stage is a list of 1..AWQ_CHAIN_MAX_LINEARS linears
 * that do not depend on each other (described as for awq_w4a16_linear_fused_multi: optional
 * normalisation or column scale in front, optional residual behind); a linear of stage s may read,
 * as x or as residual, anything a linear of a stage before s writes.  Example: {o (+residual, in
 * place into the hidden state)} -> {gate, up (RMS normalisation of that hidden state in front)}.
 * The results obey the tolerance of the separate calls (they equal those of
 * awq_w4a16_linear_fused_multi on the same stage wherever that call runs the streaming kernel); a
 * given call is deterministic.
 *   How: every workgroup of the launch is resident; one that has finished its share of a stage
 *   requests its first weights of the next stage at once (they do not depend on the stage) and
 *   then waits, for a bounded number of polls, until all workgroups have finished the stage.
 *   sync: AWQ_CHAIN_SYNC_BYTES of device memory, 16-byte aligned, ZERO before the first use; a
 *     call that ends normally leaves it zero again, so consecutive calls on one stream (and
 *     replays of a captured graph) can share it.  Calls that may overlap need one each.
 *   spin_limit: polls a workgroup spends on one wait before it gives up (0 = default, some
 *     seconds).  A wait can only run out if the launch's workgroups are not all resident, i.e. if
 *     another kernel occupies the GPU at the same time; then, or when sync was not zero, word 0 of
 *     sync is set to a non-zero value, every workgroup leaves, the outputs are undefined and sync
 *     must be zeroed again.  The launch always ends.
 *   M <= 16; every linear must fit the streaming decode kernel (awq_w4a16_linear_fused_fits),
 *   AWQ_ERR_BAD_SHAPE otherwise, also when a stage would need more workgroups than the GPU holds
 *   at once.  `stages` and the arrays it points to are HOST memory, read before the call returns. */
#define AWQ_CHAIN_MAX_STAGES 4
#define AWQ_CHAIN_MAX_LINEARS 10
#define AWQ_CHAIN_SYNC_BYTES 8192
typedef struct awq_chain_stage {
    const awq_fused_desc *descs;
    int count;
} awq_chain_stage;
int awq_w4a16_linear_chain(const awq_chain_stage *stages, int n_stages, int64_t M, int group, void *sync,
                           int spin_limit, void *stream);

/* Diagnostic: how the last grouped decode launch of this process (awq_w4a16_linear_multi,
 * awq_w3a16_linear_multi, awq_w4a16_linear_fused_multi through the streaming kernel) laid out its
 * workgroups: 0 = none yet, 1 = one size of workgroup per linear, 2 = two sizes per linear, paired
 * large with small on every CU.  Not synchronised between threads. */
int awq_last_grouped_plan(void);

/* ---- INT3-g128 variant (Sec. 5: INT4/INT3 with group size 128) ----------------------------
 * The 8-level form of the quantizer (15 -> 7 in the formulas of awq_quantize_pack) and its own
 * packed layout, version 1:
 *   qweight : N*K*3/8 bytes; tiles of 16 rows x 128 columns (768 B), tile index as above.  A
 *             tile is 64 slots of 12 B = three little-endian 32-bit words; slot (n%16) + 16*c
 *             holds the 32 codes of columns 32*j + 8*c + e (j = 0..3, e = 0..7).  Code
 *             i = 8*j + e is member h = i%2 of pair p = i/2; pairs 0..14 sit in word p/5 at bits
 *             [3f, 3f+3), f = p%5, of the low (h = 0) or high (h = 1) 16-bit half; bit b of a
 *             code of pair 15 is bit 15 (h = 0) or bit 31 (h = 1) of word b.
 *   scales, zeros : as in the 4-bit layout (zero points 0..7 in nibbles).
 * Arguments, ownership and errors as for the 4-bit calls of the same name. */
int awq_packed_sizes_w3(int64_t N, int64_t K, int group, size_t *qweight_bytes,
                        size_t *scales_bytes, size_t *zeros_bytes);
int awq_quantize_pack_w3(const void *W_f16, const float *s, int64_t N, int64_t K, int group,
                         void *qweight, void *scales, void *zeros, void *stream);
int awq_unpack_w3(const void *qweight, const void *scales, const void *zeros, int64_t N,
                  int64_t K, int group, uint8_t *codes, void *scales_f16, uint8_t *zeros_u8,
                  void *stream);
/* Sec. 4.2 decode kernel for the 3-bit layout: y = x' * dequant(q)^T, fp32 accumulation,
 * 1 <= M <= 16 (AWQ_ERR_BAD_SHAPE otherwise: larger M goes through awq_w3a16_linear_prefill). */
int awq_w3a16_linear(const void *x_f16, const void *qweight, const void *scales,
                     const void *zeros, void *y_f16, int64_t M, int64_t N, int64_t K, int group,
                     void *stream);
/* Prefill (M > 16) for the 3-bit layout.  There is no 3-bit matrix-matrix kernel: the codes are
 * re-packed into the 4-bit layout (the steps and zero points are stored identically in both, and
 * a code 0..7 is a valid 4-bit code), then the prefill kernel of the 4-bit path runs on them --
 * one extra pass over the packed weights, about a tenth of the GEMM's time at M = 2048.
 *   awq_repack_w3_to_w4: qweight_w3 (N*K*3/8 bytes) -> qweight_w4 (N*K/2 bytes, written), both
 *     device, 16-byte aligned; a caller with the memory can keep the result and use the 4-bit
 *     calls with the 3-bit linear's scales and zeros.
 *   awq_w3a16_linear_prefill: the two steps in one call; workspace (device, 16-byte aligned,
 *     awq_w3a16_prefill_workspace_bytes() = N*K/2 bytes) holds the re-packed codes, contents
 *     undefined afterwards.  With N*K/2 rounded up to a multiple of 256, plus
 *     awq_linear_workspace_bytes(M, N, K, group) bytes, the prefill kernel also cuts K into
 *     ranges for a few hundred tokens, as awq_w4a16_linear does with its workspace.
 *     M <= 16 returns AWQ_ERR_BAD_SHAPE (use awq_w3a16_linear). */
int awq_repack_w3_to_w4(const void *qweight_w3, int64_t N, int64_t K, int group, void *qweight_w4,
                        void *stream);
size_t awq_w3a16_prefill_workspace_bytes(int64_t N, int64_t K, int group);
int awq_w3a16_linear_prefill(const void *x_f16, const void *qweight, const void *scales,
                             const void *zeros, void *y_f16, int64_t M, int64_t N, int64_t K,
                             int group, void *workspace, size_t workspace_bytes, void *stream);
/* As awq_w4a16_linear_multi for linears in the 3-bit layout (no workspace). */
int awq_w3a16_linear_multi(const awq_linear_desc *descs, int count, int64_t M, int group,
                           void *stream);

/* ---- INT2-g64 variant (Sec. 5, the extreme low-bit table: INT2 with group size 64) ----------
 * The 4-level form of the quantizer (15 -> 3 in the formulas of awq_quantize_pack) over groups of
 * AWQ_GROUP_W2 = 64 input channels, and its own packed layout, version 1.  `group` must be 64, N a
 * multiple of 16, K a multiple of 256 (AWQ_ERR_UNSUPPORTED_GROUP / AWQ_ERR_BAD_SHAPE otherwise):
 *   qweight : N*K/4 bytes; blocks of 16 rows x 256 columns (four groups, 1 KB), block index
 *             (n/16)*(K/256) + k/256.  A block is 64 slots of 16 B = four little-endian 32-bit
 *             words; slot (n%16) + 16*c holds the 64 codes of columns 64*t + 32*j + 8*c + 2*i + h
 *             of the block (group t = 0..3, half of the group j = 0..1, i = 0..3, h = 0..1): word
 *             i holds the codes with that i, the code of (t, j, h) in field f = t + 4*j, bits
 *             [2f, 2f+2), of the low (h = 0) or high (h = 1) 16-bit half.
 *   scales  : N*(K/64)*2 bytes; [N/16][K/256][16 rows][4 groups] binary16.
 *   zeros   : N*(K/64)/4 bytes; [N/16][K/256][16 rows]; the byte of a row holds the zero point of
 *             group t of the block at bits [2t, 2t+2).
 * Arguments, ownership and errors as for the 4-bit calls of the same name.  awq_unpack_w2 returns
 * codes u8[N,K], scales f16[N,K/64], zeros u8[N,K/64] (each optional).
 * awq_w2a16_linear: y = x' * dequant(q)^T with fp32 accumulation, any M >= 1, through the decode
 * kernel: more than 16 rows run as blocks of 16 rows, 128 rows per launch.  There is no 2-bit
 * matrix-matrix kernel, so the time grows with M/128 launches that each read the packed weights
 * again (sized for prompts of a few hundred tokens).  awq_w2a16_linear_multi: as awq_w4a16_linear_multi
 * (1 <= M <= 16, up to AWQ_MULTI_MAX linears, eight per launch). */
#define AWQ_GROUP_W2 64
int awq_packed_sizes_w2(int64_t N, int64_t K, int group, size_t *qweight_bytes,
                        size_t *scales_bytes, size_t *zeros_bytes);
int awq_quantize_pack_w2(const void *W_f16, const float *s, int64_t N, int64_t K, int group,
                         void *qweight, void *scales, void *zeros, void *stream);
int awq_unpack_w2(const void *qweight, const void *scales, const void *zeros, int64_t N,
                  int64_t K, int group, uint8_t *codes, void *scales_f16, uint8_t *zeros_u8,
                  void *stream);
int awq_w2a16_linear(const void *x_f16, const void *qweight, const void *scales,
                     const void *zeros, void *y_f16, int64_t M, int64_t N, int64_t K, int group,
                     void *stream);
int awq_w2a16_linear_multi(const awq_linear_desc *descs, int count, int64_t M, int group,
                           void *stream);

/* ---- decode attention (Sec. 4.2, kernel fusion: the kernel evaluates the position embedding
 * itself and writes the new key and value into caches allocated ahead) -------------------
 * One decode step of one sequence.  q [H,D], k, v [Hkv,D] fp16: the projections of the token at
 * position pos (0-based).  k_cache, v_cache [Hkv][Lmax][D] fp16, pre-allocated by the caller,
 * rows < pos filled by earlier calls.  The call rotates q and k by the rotary embedding of pos
 * (pairs (i, i + D/2), angle pos * rope_theta^(-2i/D)), writes fp16(k_rot) and v into row pos of
 * the caches and out [H,D] fp16 = softmax(q_rot K^T / sqrt(D)) V over rows 0..pos; query head h
 * reads kv head h / (H/Hkv).  fp32 arithmetic (fp64 for the angles).  D == 128, H % Hkv == 0,
 * 0 <= pos < Lmax, rope_theta > 1.  workspace: device, 16-byte aligned,
 * awq_decode_attention_workspace_bytes(H, D, pos + 1) bytes (partial results of the slices of
 * the positions), contents undefined afterwards.  Calls for consecutive positions on one stream
 * are ordered by the stream. */
size_t awq_decode_attention_workspace_bytes(int64_t H, int64_t D, int64_t L);
int awq_decode_attention(const void *q_f16, const void *k_f16, const void *v_f16, void *k_cache_f16,
                         void *v_cache_f16, int64_t H, int64_t Hkv, int64_t D, int64_t Lmax,
                         int64_t pos, float rope_theta, void *out_f16, void *workspace,
                         size_t workspace_bytes, void *stream);

#define AWQ_SEARCH_MAX_ALPHAS 64

/* Bytes of scratch awq_search_scale needs (0 for an invalid shape): the packed candidate,
 * x / s, the fp16 layer output and the candidate's output ([T,N] fp16 each) and the partial
 * sums. */
size_t awq_search_scale_workspace_bytes(int64_t T, int64_t N, int64_t K, int n_alpha, int group);

/* Sec. 3.2 (the search for the scale), Eq. 4-5: for every alpha of the grid, s = s_X^alpha with
 * s_X[k] = max(mean_t |X[t,k]|, 1e-4), and
 *   loss(alpha) = sum_{t,n} ( y_q[t,n] - y[t,n] )^2,
 *   y_q = awq_w4a16_linear(awq_apply_inv_scale(X, s), awq_quantize_pack(W, s)),  y = fp16(X W^T)
 * (the squared Frobenius norm of Eq. 4, both outputs as the fp16 arrays the layers produce,
 * squares summed in fp64 in a fixed order).  best = first index of the smallest loss;
 * s_best = s_X^alphas[best], bit-identical to awq_act_scale(X, alphas[best]).
 *   W_f16 [N,K], X_f16 [T,K] fp16 row-major (device, read); alphas: HOST array of n_alpha
 *   values in [0,1], 1 <= n_alpha <= AWQ_SEARCH_MAX_ALPHAS, read before the call returns;
 *   workspace: device, 256-byte aligned, awq_search_scale_workspace_bytes() bytes, contents
 *   undefined afterwards; losses [n_alpha] fp64, best [1] int32, s_best [K] fp32: device,
 *   written.  Like every other call it only enqueues work on `stream`. */
int awq_search_scale(const void *W_f16, const void *X_f16, int64_t T, int64_t N, int64_t K,
                     const float *alphas, int n_alpha, int group, void *workspace,
                     size_t workspace_bytes, double *losses, int32_t *best, float *s_best,
                     void *stream);

#ifdef __cplusplus
}
#endif
#endif /* AWQ_MI355X_H */
