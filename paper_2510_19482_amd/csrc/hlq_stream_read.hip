// Measurement helper: a plain streaming read of device memory with 128-bit loads.  It does nothing
// of the method; benchmarks time it on the same number of bytes as a GEMV launch to see what part
// of the 8 TB/s figure a read-only kernel of that size reaches on the machine at hand.
#include <hip/hip_runtime.h>

#include "hlq_internal.h"

typedef unsigned rd_uint4 __attribute__((ext_vector_type(4)));

namespace {

// Every lane reads 16-byte units lane, lane + stride, ... of its workgroup's contiguous share and
// folds them into one word; one word per workgroup is stored so that no load can be dropped.
template <int UNROLL, bool NT>
__global__ __launch_bounds__(256) void hlq_stream_read_kernel(const rd_uint4 *__restrict__ src, size_t units,
                                                              size_t units_per_block, uint32_t *__restrict__ sink)
{
    const size_t b0 = (size_t)blockIdx.x * units_per_block;
    size_t b1 = b0 + units_per_block;
    if (b1 > units) b1 = units;
    auto ld = [](const rd_uint4 *p) -> rd_uint4 { return NT ? __builtin_nontemporal_load(p) : *p; };
    rd_uint4 acc = {0u, 0u, 0u, 0u};
    size_t i = b0 + threadIdx.x;
    for (; i + (size_t)(UNROLL - 1) * 256 < b1; i += (size_t)UNROLL * 256) {
        rd_uint4 v[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) v[u] = ld(src + i + (size_t)u * 256);
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) acc ^= v[u];
    }
    for (; i < b1; i += 256) acc ^= ld(src + i);
    uint32_t r = acc.x ^ acc.y ^ acc.z ^ acc.w;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) r ^= __shfl_xor(r, o);
    __shared__ uint32_t part[4];
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = r;
    __syncthreads();
    if (threadIdx.x == 0) sink[blockIdx.x] = part[0] ^ part[1] ^ part[2] ^ part[3];
}

template <bool NT>
void launch_read(int unroll, int blocks, hipStream_t st, const rd_uint4 *src, size_t units, size_t upb, uint32_t *sink)
{
    switch (unroll) {
    case 1: hipLaunchKernelGGL((hlq_stream_read_kernel<1, NT>), dim3(blocks), dim3(256), 0, st, src, units, upb, sink); break;
    case 2: hipLaunchKernelGGL((hlq_stream_read_kernel<2, NT>), dim3(blocks), dim3(256), 0, st, src, units, upb, sink); break;
    case 8: hipLaunchKernelGGL((hlq_stream_read_kernel<8, NT>), dim3(blocks), dim3(256), 0, st, src, units, upb, sink); break;
    case 16: hipLaunchKernelGGL((hlq_stream_read_kernel<16, NT>), dim3(blocks), dim3(256), 0, st, src, units, upb, sink); break;
    default: hipLaunchKernelGGL((hlq_stream_read_kernel<4, NT>), dim3(blocks), dim3(256), 0, st, src, units, upb, sink); break;
    }
}

}  // namespace

static hlq_status stream_read(const void *src, size_t bytes, int blocks, int unroll, int temporal, void *sink,
                              size_t sink_bytes, void *stream)
{
    if (!src || !sink) return HLQ_ERR_NULL;
    if (((uintptr_t)src & 15u) || (bytes & 15u) || ((uintptr_t)sink & 3u)) return HLQ_ERR_BAD_STRIDE;
    if (blocks < 0 || blocks > 65536) return HLQ_ERR_UNSUPPORTED;
    if (unroll != 1 && unroll != 2 && unroll != 4 && unroll != 8 && unroll != 16) return HLQ_ERR_UNSUPPORTED;
    if (bytes == 0) return HLQ_OK;
    const size_t units = bytes / 16;
    if (blocks == 0) blocks = 2048;
    if ((size_t)blocks > (units + 255) / 256) blocks = (int)((units + 255) / 256);
    if (sink_bytes < (size_t)blocks * 4) return HLQ_ERR_BUFFER_TOO_SMALL;
    const size_t upb = (units + blocks - 1) / blocks;
    hlq_clear_stale_error();
    if (temporal) launch_read<false>(unroll, blocks, (hipStream_t)stream, (const rd_uint4 *)src, units, upb, (uint32_t *)sink);
    else launch_read<true>(unroll, blocks, (hipStream_t)stream, (const rd_uint4 *)src, units, upb, (uint32_t *)sink);
    return hlq_hip_status(hipGetLastError());
}

extern "C" HLQ_API hlq_status hlq_stream_read(const void *src, size_t bytes, int blocks, void *sink, size_t sink_bytes,
                                              void *stream)
{
    return stream_read(src, bytes, blocks, 4, 0, sink, sink_bytes, stream);
}

extern "C" HLQ_API hlq_status hlq_stream_read_shaped(const void *src, size_t bytes, int blocks, int unroll, int temporal,
                                                     void *sink, size_t sink_bytes, void *stream)
{
    return stream_read(src, bytes, blocks, unroll, temporal, sink, sink_bytes, stream);
}
