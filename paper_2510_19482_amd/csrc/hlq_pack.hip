// hlq_pack / hlq_unpack: the offline bit-plane decomposition (App. B) and weight
// re-arrangement (App. D, Weight-Rearrange) for the CDNA4 layout described in
// hlq_internal.h.  Integer work only; pack and unpack are exact inverses.
#include "hlq_internal.h"

namespace {

// One thread per (chunk c, column n): gathers the 128 codes of that column slice and emits
// one 16-byte word per bit-plane into record (tile, c).  Threads of a wavefront own adjacent
// columns, so both the byte reads (row k, columns n..n+63) and the 16-byte writes are contiguous.
__global__ void __launch_bounds__(256)
hlq_pack_bits_kernel(const uint8_t *__restrict__ codes, char *__restrict__ packed, int N,
                     size_t col_bytes, int q, int G)
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
            for (int j = 0; j < 4; ++j) w[j][d] |= ((code >> j) & 1u) << hlq_bit_pos(b);
        }
    }
    const int tile = n / HLQ_TILE_N, lane = n % HLQ_TILE_N, tw = hlq_tile_width(tile, N);
    uint4 *rec = (uint4 *)(packed + hlq_rec_off(col_bytes, tile, tw, c, q, G));
    for (int j = 0; j < q; ++j) rec[j * tw + lane] = make_uint4(w[j][0], w[j][1], w[j][2], w[j][3]);
}

__global__ void __launch_bounds__(256)
hlq_unpack_bits_kernel(const char *__restrict__ packed, uint8_t *__restrict__ codes, int N,
                       size_t col_bytes, int q, int G)
{
    const int n = blockIdx.x * 256 + threadIdx.x;
    const int c = blockIdx.y;
    if (n >= N) return;
    uint32_t w[4][4];
    const int tile = n / HLQ_TILE_N, lane = n % HLQ_TILE_N, tw = hlq_tile_width(tile, N);
    const uint4 *rec = (const uint4 *)(packed + hlq_rec_off(col_bytes, tile, tw, c, q, G));
    for (int j = 0; j < 4; ++j) {
        uint4 v = make_uint4(0u, 0u, 0u, 0u);
        if (j < q) v = rec[j * tw + lane];
        w[j][0] = v.x; w[j][1] = v.y; w[j][2] = v.z; w[j][3] = v.w;
    }
    uint8_t *dst = codes + (size_t)c * HLQ_CHUNK_K * N + n;
    for (int d = 0; d < 4; ++d) {
        for (int b = 0; b < 32; ++b) {
            uint32_t code = 0u;
#pragma unroll
            for (int j = 0; j < 4; ++j) code |= ((w[j][d] >> hlq_bit_pos(b)) & 1u) << j;
            dst[(size_t)(32 * d + b) * N] = (uint8_t)code;
        }
    }
}

// Address of the fp16 slot (group g, row r, column n) inside the record of the chunk in which
// group g starts.
__device__ __forceinline__ size_t meta_slot(size_t col_bytes, int N, int q, int G, int g, int r, int n)
{
    const int tile = n / HLQ_TILE_N, lane = n % HLQ_TILE_N, tw = hlq_tile_width(tile, N);
    const int c = (int)(((long)g * G) / HLQ_CHUNK_K);
    const int s = g - hlq_groups_before(c, G);
    return hlq_rec_off(col_bytes, tile, tw, c, q, G) + (size_t)tw * q * 16 +
           ((size_t)(s * (q + 1) + r) * tw + lane) * 2;
}

// record meta <- r < q ? scales[r][g][n] : zeros[g][n]   (and the inverse)
__global__ void __launch_bounds__(256)
hlq_pack_meta_kernel(const uint16_t *__restrict__ scales, const uint16_t *__restrict__ zeros,
                     char *__restrict__ packed, int N, size_t col_bytes, int ngroups, int q, int G)
{
    const int n = blockIdx.x * 256 + threadIdx.x;
    const int g = blockIdx.y;
    if (n >= N) return;
    for (int r = 0; r < q; ++r)
        *(uint16_t *)(packed + meta_slot(col_bytes, N, q, G, g, r, n)) = scales[((size_t)r * ngroups + g) * N + n];
    *(uint16_t *)(packed + meta_slot(col_bytes, N, q, G, g, q, n)) = zeros[(size_t)g * N + n];
}

__global__ void __launch_bounds__(256)
hlq_unpack_meta_kernel(const char *__restrict__ packed, uint16_t *__restrict__ scales,
                       uint16_t *__restrict__ zeros, int N, size_t col_bytes, int ngroups, int q, int G)
{
    const int n = blockIdx.x * 256 + threadIdx.x;
    const int g = blockIdx.y;
    if (n >= N) return;
    if (scales)
        for (int r = 0; r < q; ++r)
            scales[((size_t)r * ngroups + g) * N + n] =
                *(const uint16_t *)(packed + meta_slot(col_bytes, N, q, G, g, r, n));
    if (zeros) zeros[(size_t)g * N + n] = *(const uint16_t *)(packed + meta_slot(col_bytes, N, q, G, g, q, n));
}

} // namespace

hlq_status hlq_launch_pack(const HlqDims &dm, const uint8_t *codes, const uint16_t *scales,
                           const uint16_t *zeros, void *packed, hipStream_t st)
{
    hlq_clear_stale_error();
    const unsigned ntiles = (unsigned)((dm.N + 255) / 256);
    hlq_pack_bits_kernel<<<dim3(ntiles, dm.nchunks), 256, 0, st>>>(codes, (char *)packed, dm.N, dm.col_bytes, dm.q, dm.G);
    hlq_pack_meta_kernel<<<dim3(ntiles, dm.ngroups), 256, 0, st>>>(scales, zeros, (char *)packed, dm.N, dm.col_bytes,
                                                                   dm.ngroups, dm.q, dm.G);
    return hlq_hip_status(hipGetLastError());
}

hlq_status hlq_launch_unpack(const HlqDims &dm, const void *packed, uint8_t *codes,
                             uint16_t *scales, uint16_t *zeros, hipStream_t st)
{
    hlq_clear_stale_error();
    const unsigned ntiles = (unsigned)((dm.N + 255) / 256);
    if (codes)
        hlq_unpack_bits_kernel<<<dim3(ntiles, dm.nchunks), 256, 0, st>>>((const char *)packed, codes, dm.N, dm.col_bytes,
                                                                         dm.q, dm.G);
    if (scales || zeros)
        hlq_unpack_meta_kernel<<<dim3(ntiles, dm.ngroups), 256, 0, st>>>((const char *)packed, scales, zeros, dm.N,
                                                                         dm.col_bytes, dm.ngroups, dm.q, dm.G);
    return hlq_hip_status(hipGetLastError());
}
