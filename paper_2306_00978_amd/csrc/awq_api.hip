// Version, status strings and size queries of the C ABI (host only).
#include "awq_common.h"

extern "C" int awq_version(void) { return 1; }

extern "C" const char *awq_status_string(int status)
{
    switch (status) {
    case AWQ_OK: return "ok";
    case AWQ_ERR_NULL_POINTER: return "null pointer";
    case AWQ_ERR_BAD_SHAPE: return "bad shape (sizes must be positive, K % 128 == 0, N % 16 == 0)";
    case AWQ_ERR_UNSUPPORTED_GROUP: return "unsupported group size (only 128)";
    case AWQ_ERR_MISALIGNED: return "tensor pointer is not 16-byte aligned";
    case AWQ_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
    case AWQ_ERR_HIP: return "HIP runtime refused the launch";
    case AWQ_ERR_BAD_ARGUMENT: return "scalar argument out of range";
    case AWQ_ERR_SCRATCH_LIMIT: return "shape needs more scratch than the library's built-in array holds";
    default: return "unknown status";
    }
}

extern "C" int awq_packed_sizes(int64_t N, int64_t K, int group, size_t *qweight_bytes,
                                size_t *scales_bytes, size_t *zeros_bytes)
{
    int st = awq_check_weight_shape(N, K, group);
    if (st != AWQ_OK) return st;
    const int64_t G = K / AWQ_GROUP;
    if (qweight_bytes) *qweight_bytes = (size_t)(N * K / 2);
    if (scales_bytes) *scales_bytes = (size_t)(N * G * 2);
    if (zeros_bytes) *zeros_bytes = (size_t)(N * G / 2);
    return AWQ_OK;
}

// Header of a packed blob (export / checkpoint aid).  Three layouts exist (4-, 3-, 2-bit); a file that
// stores packed arrays should say which one it holds and for what shape, so that a reader built
// for another layout version refuses it instead of computing with reshuffled codes.
extern "C" int awq_blob_header_init(awq_blob_header *h, int bits, int64_t N, int64_t K, int group)
{
    if (!h) return AWQ_ERR_NULL_POINTER;
    size_t q = 0, s = 0, z = 0;
    int st;
    if (bits == 4) st = awq_packed_sizes(N, K, group, &q, &s, &z);
    else if (bits == 3) st = awq_packed_sizes_w3(N, K, group, &q, &s, &z);
    else if (bits == 2) st = awq_packed_sizes_w2(N, K, group, &q, &s, &z);
    else return AWQ_ERR_BAD_ARGUMENT;
    if (st != AWQ_OK) return st;
    const char magic[8] = {'A', 'W', 'Q', 'g', 'f', 'x', '9', '5'};
    for (int i = 0; i < 8; ++i) h->magic[i] = magic[i];
    h->layout_version = (uint32_t)awq_version();
    h->bits = (uint32_t)bits;
    h->group = (uint32_t)group;
    h->reserved = 0;
    h->N = N;
    h->K = K;
    h->qweight_bytes = q;
    h->scales_bytes = s;
    h->zeros_bytes = z;
    return AWQ_OK;
}

extern "C" int awq_blob_header_check(const awq_blob_header *h)
{
    if (!h) return AWQ_ERR_NULL_POINTER;
    awq_blob_header want;
    const int st = awq_blob_header_init(&want, (int)h->bits, h->N, h->K, (int)h->group);
    if (st != AWQ_OK) return st;
    for (int i = 0; i < 8; ++i)
        if (h->magic[i] != want.magic[i]) return AWQ_ERR_BAD_ARGUMENT;
    if (h->layout_version != want.layout_version || h->reserved != 0 || h->qweight_bytes != want.qweight_bytes ||
        h->scales_bytes != want.scales_bytes || h->zeros_bytes != want.zeros_bytes)
        return AWQ_ERR_BAD_ARGUMENT;
    return AWQ_OK;
}

namespace {

// Read-only reference of the benchmark: every lane streams 16-byte words with a grid stride and
// folds them into one word; nothing is written unless the fold hits a magic value.
__global__ __launch_bounds__(512) void read_probe_kernel(const uint4 *__restrict__ p, int64_t n16,
                                                         uint32_t *__restrict__ sink)
{
    uint32_t acc = 0;
    const int64_t stride = (int64_t)gridDim.x * 512;
    int64_t i = (int64_t)blockIdx.x * 512 + threadIdx.x;
    for (; i + 3 * stride < n16; i += 4 * stride) {
        const uint4 a = p[i], b = p[i + stride], c = p[i + 2 * stride], d = p[i + 3 * stride];
        acc ^= a.x ^ a.y ^ a.z ^ a.w ^ b.x ^ b.y ^ b.z ^ b.w ^ c.x ^ c.y ^ c.z ^ c.w ^ d.x ^ d.y ^ d.z ^ d.w;
    }
    for (; i < n16; i += stride) {
        const uint4 a = p[i];
        acc ^= a.x ^ a.y ^ a.z ^ a.w;
    }
    if (acc == 0x9E3779B9u) sink[0] = acc;
}

}  // namespace

extern "C" int awq_read_probe(const void *buffer, size_t bytes, uint32_t *sink, void *stream)
{
    if (!buffer || !sink) return AWQ_ERR_NULL_POINTER;
    if (bytes < 16) return AWQ_ERR_BAD_SHAPE;
    if (!awq_aligned16(buffer)) return AWQ_ERR_MISALIGNED;
    // one workgroup of eight waves per CU: the fastest of the launch shapes tried on ~100 MB
    read_probe_kernel<<<dim3(256), dim3(512), 0, (hipStream_t)stream>>>((const uint4 *)buffer,
                                                                         (int64_t)(bytes / 16), sink);
    return awq_launch_status();
}
