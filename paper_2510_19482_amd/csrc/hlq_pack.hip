// hlq_pack / hlq_unpack: the offline bit-plane decomposition (App. B) and weight
// re-arrangement (App. D, Weight-Rearrange) for the CDNA4 layout described in
// hlq_internal.h.  Integer work only; pack and unpack are exact inverses.
#include "hlq_internal.h"

namespace {

// One thread per (chunk c, column n): gathers the 128 codes of that column slice and emits
// one 16-byte word per bit-plane.  Threads of a wavefront own adjacent columns, so both the
// byte reads (row k, columns n..n+63) and the 16-byte writes are contiguous.
__global__ void __launch_bounds__(256)
hlq_pack_bits_kernel(const uint8_t *__restrict__ codes, uint4 *__restrict__ bits, int N,
                     int nchunks, int q)
{
    const int n = blockIdx.x * 256 + threadIdx.x;
    const int c = blockIdx.y;
    if (n >= N) return;
    uint32_t w[4][4];   // [plane][word]
    for (int j = 0; j < 4; ++j)
        for (int d = 0; d < 4; ++d) w[j][d] = 0u;
    const uint8_t *src = codes + (size_t)c * HLQ_CHUNK_K * N + n;
    for (int d = 0; d < 4; ++d) {
        for (int b = 0; b < 32; ++b) {
            const uint32_t code = src[(size_t)(32 * d + b) * N];
#pragma unroll
            for (int j = 0; j < 4; ++j) w[j][d] |= ((code >> j) & 1u) << b;
        }
    }
    for (int j = 0; j < q; ++j)
        bits[((size_t)j * nchunks + c) * N + n] = make_uint4(w[j][0], w[j][1], w[j][2], w[j][3]);
}

__global__ void __launch_bounds__(256)
hlq_unpack_bits_kernel(const uint4 *__restrict__ bits, uint8_t *__restrict__ codes, int N,
                       int nchunks, int q)
{
    const int n = blockIdx.x * 256 + threadIdx.x;
    const int c = blockIdx.y;
    if (n >= N) return;
    uint32_t w[4][4];
    for (int j = 0; j < 4; ++j) {
        uint4 v = make_uint4(0u, 0u, 0u, 0u);
        if (j < q) v = bits[((size_t)j * nchunks + c) * N + n];
        w[j][0] = v.x; w[j][1] = v.y; w[j][2] = v.z; w[j][3] = v.w;
    }
    uint8_t *dst = codes + (size_t)c * HLQ_CHUNK_K * N + n;
    for (int d = 0; d < 4; ++d) {
        for (int b = 0; b < 32; ++b) {
            uint32_t code = 0u;
#pragma unroll
            for (int j = 0; j < 4; ++j) code |= ((w[j][d] >> b) & 1u) << j;
            dst[(size_t)(32 * d + b) * N] = (uint8_t)code;
        }
    }
}

// meta[g][r][n] <- r < q ? scales[r][g][n] : zeros[g][n]   (and the inverse)
__global__ void __launch_bounds__(256)
hlq_pack_meta_kernel(const uint16_t *__restrict__ scales, const uint16_t *__restrict__ zeros,
                     uint16_t *__restrict__ meta, int N, int ngroups, int q)
{
    const int n = blockIdx.x * 256 + threadIdx.x;
    const int g = blockIdx.y;
    if (n >= N) return;
    for (int r = 0; r < q; ++r)
        meta[((size_t)g * (q + 1) + r) * N + n] = scales[((size_t)r * ngroups + g) * N + n];
    meta[((size_t)g * (q + 1) + q) * N + n] = zeros[(size_t)g * N + n];
}

__global__ void __launch_bounds__(256)
hlq_unpack_meta_kernel(const uint16_t *__restrict__ meta, uint16_t *__restrict__ scales,
                       uint16_t *__restrict__ zeros, int N, int ngroups, int q)
{
    const int n = blockIdx.x * 256 + threadIdx.x;
    const int g = blockIdx.y;
    if (n >= N) return;
    if (scales)
        for (int r = 0; r < q; ++r)
            scales[((size_t)r * ngroups + g) * N + n] = meta[((size_t)g * (q + 1) + r) * N + n];
    if (zeros) zeros[(size_t)g * N + n] = meta[((size_t)g * (q + 1) + q) * N + n];
}

} // namespace

hlq_status hlq_launch_pack(const HlqDims &dm, const uint8_t *codes, const uint16_t *scales,
                           const uint16_t *zeros, void *packed, hipStream_t st)
{
    const unsigned ntiles = (unsigned)((dm.N + 255) / 256);
    uint4 *bits = (uint4 *)packed;
    uint16_t *meta = (uint16_t *)((char *)packed + dm.bits_bytes);
    hlq_pack_bits_kernel<<<dim3(ntiles, dm.nchunks), 256, 0, st>>>(codes, bits, dm.N, dm.nchunks, dm.q);
    hlq_pack_meta_kernel<<<dim3(ntiles, dm.ngroups), 256, 0, st>>>(scales, zeros, meta, dm.N, dm.ngroups, dm.q);
    return hlq_hip_status(hipGetLastError());
}

hlq_status hlq_launch_unpack(const HlqDims &dm, const void *packed, uint8_t *codes,
                             uint16_t *scales, uint16_t *zeros, hipStream_t st)
{
    const unsigned ntiles = (unsigned)((dm.N + 255) / 256);
    const uint4 *bits = (const uint4 *)packed;
    const uint16_t *meta = (const uint16_t *)((const char *)packed + dm.bits_bytes);
    if (codes)
        hlq_unpack_bits_kernel<<<dim3(ntiles, dm.nchunks), 256, 0, st>>>(bits, codes, dm.N, dm.nchunks, dm.q);
    if (scales || zeros)
        hlq_unpack_meta_kernel<<<dim3(ntiles, dm.ngroups), 256, 0, st>>>(meta, scales, zeros, dm.N, dm.ngroups, dm.q);
    return hlq_hip_status(hipGetLastError());
}
