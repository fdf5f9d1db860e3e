// Measurement helper: a loop of nothing but v_mfma_f32_32x32x16_f16 on register operands, the instruction
// the tiled prefill kernel is built on.  It does nothing of the method; benchmarks time it beside the
// prefill GEMM to see what the matrix cores sustain on the machine at hand with the operand data they are
// given (the sustained matrix-core clock depends on how many operand bits toggle), at the prefill kernel's
// occupancy of two wavefronts per SIMD.
#include <hip/hip_runtime.h>

#include "hlq_internal.h"

namespace {

typedef _Float16 probe_half8 __attribute__((ext_vector_type(8)));
typedef float probe_float16 __attribute__((ext_vector_type(16)));

constexpr int PROBE_CHAINS = 4;    // independent accumulator tiles per wavefront: 64 accumulator registers
constexpr int PROBE_OPERANDS = 4;  // operand pairs a wavefront rotates through

// Every wavefront loads PROBE_OPERANDS operand pairs (8 fp16 per lane each) once, then issues
// iters x PROBE_OPERANDS x PROBE_CHAINS MFMAs; the accumulators are folded into one float per lane at the end.
__global__ __launch_bounds__(256) void hlq_mfma_probe_kernel(const probe_half8 *__restrict__ operands, int units, int iters,
                                                             float *__restrict__ sink)
{
    const int wave = (int)((blockIdx.x * 256u + threadIdx.x) >> 6), lane = (int)(threadIdx.x & 63u);
    probe_half8 a[PROBE_OPERANDS], b[PROBE_OPERANDS];
#pragma unroll
    for (int o = 0; o < PROBE_OPERANDS; ++o) {
        a[o] = operands[(unsigned)((wave * 2 * PROBE_OPERANDS + 2 * o) * 64 + lane) % (unsigned)units];
        b[o] = operands[(unsigned)((wave * 2 * PROBE_OPERANDS + 2 * o + 1) * 64 + lane) % (unsigned)units];
    }
    probe_float16 acc[PROBE_CHAINS];
#pragma unroll
    for (int c = 0; c < PROBE_CHAINS; ++c)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[c][r] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int o = 0; o < PROBE_OPERANDS; ++o)
#pragma unroll
            for (int c = 0; c < PROBE_CHAINS; ++c)
                acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[(o + c) % PROBE_OPERANDS], b[o], acc[c], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int c = 0; c < PROBE_CHAINS; ++c)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[c][r];
    sink[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}

}  // namespace

extern "C" HLQ_API hlq_status hlq_mfma_probe(const void *operands, size_t operand_bytes, int iters, int blocks, void *sink,
                                             size_t sink_bytes, double *flop, void *stream)
{
    if (!operands || !sink) return HLQ_ERR_NULL;
    if (((uintptr_t)operands & 15u) || ((uintptr_t)sink & 3u)) return HLQ_ERR_BAD_STRIDE;
    if (operand_bytes < 16 || (operand_bytes & 15u) || operand_bytes > ((size_t)1 << 30)) return HLQ_ERR_BAD_STRIDE;
    if (iters < 1 || iters > (1 << 20) || blocks < 1 || blocks > 65536) return HLQ_ERR_UNSUPPORTED;
    if (sink_bytes < (size_t)blocks * 256 * 4) return HLQ_ERR_BUFFER_TOO_SMALL;
    if (flop) *flop = (double)blocks * 4.0 * (double)iters * PROBE_OPERANDS * PROBE_CHAINS * (2.0 * 32 * 32 * 16);
    hlq_clear_stale_error();
    hipLaunchKernelGGL(hlq_mfma_probe_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream, (const probe_half8 *)operands,
                       (int)(operand_bytes / 16), iters, (float *)sink);
    return hlq_hip_status(hipGetLastError());
}
