// Measurement helper: a loop of nothing but one matrix-core instruction on register operands -- kind 0:
// v_mfma_f32_32x32x16_f16, the instruction the tiled prefill kernel is built on; kind 1:
// v_mfma_f32_16x16x128_f8f6f4 with a bf8 and an fp4 operand, the instruction of the bit-plane GEMV kernels.  It does nothing of the method; benchmarks time it beside the
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

typedef int probe_int8 __attribute__((ext_vector_type(8)));
typedef int probe_int4 __attribute__((ext_vector_type(4)));
typedef float probe_float4 __attribute__((ext_vector_type(4)));
constexpr int PROBE_MX_CHAINS = 8;

// kind 1: the operand units are taken as they are (32 bytes of bf8 codes, 16 bytes of fp4 codes per lane);
// iters x PROBE_OPERANDS x PROBE_MX_CHAINS instructions per wavefront, eight independent accumulators.
__global__ __launch_bounds__(256) void hlq_mfma_probe_mx_kernel(const probe_half8 *__restrict__ operands, int units, int iters,
                                                                float *__restrict__ sink)
{
    const int wave = (int)((blockIdx.x * 256u + threadIdx.x) >> 6), lane = (int)(threadIdx.x & 63u);
    probe_int8 a[PROBE_OPERANDS], b[PROBE_OPERANDS];
#pragma unroll
    for (int o = 0; o < PROBE_OPERANDS; ++o) {
        const probe_half8 lo = operands[(unsigned)((wave * 3 * PROBE_OPERANDS + 3 * o) * 64 + lane) % (unsigned)units];
        const probe_half8 hi = operands[(unsigned)((wave * 3 * PROBE_OPERANDS + 3 * o + 1) * 64 + lane) % (unsigned)units];
        const probe_half8 bb = operands[(unsigned)((wave * 3 * PROBE_OPERANDS + 3 * o + 2) * 64 + lane) % (unsigned)units];
        const probe_int4 l4 = __builtin_bit_cast(probe_int4, lo), h4 = __builtin_bit_cast(probe_int4, hi), b4 = __builtin_bit_cast(probe_int4, bb);
        // bf8 codes with the top exponent bit cleared: finite, moderate magnitudes
        a[o] = (probe_int8){l4.x & 0x3f3f3f3f, l4.y & 0x3f3f3f3f, l4.z & 0x3f3f3f3f, l4.w & 0x3f3f3f3f,
                            h4.x & 0x3f3f3f3f, h4.y & 0x3f3f3f3f, h4.z & 0x3f3f3f3f, h4.w & 0x3f3f3f3f};
        b[o] = (probe_int8){b4.x, b4.y, b4.z, b4.w, 0, 0, 0, 0};
    }
    probe_float4 acc[PROBE_MX_CHAINS];
#pragma unroll
    for (int c = 0; c < PROBE_MX_CHAINS; ++c) acc[c] = (probe_float4){0.f, 0.f, 0.f, 0.f};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int o = 0; o < PROBE_OPERANDS; ++o)
#pragma unroll
            for (int c = 0; c < PROBE_MX_CHAINS; ++c)
                acc[c] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a[(o + c) % PROBE_OPERANDS], b[o], acc[c], 1, 4, 0, 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int c = 0; c < PROBE_MX_CHAINS; ++c) s += acc[c][0] + acc[c][1] + acc[c][2] + acc[c][3];
    sink[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}

}  // namespace

extern "C" HLQ_API hlq_status hlq_mfma_probe(int kind, const void *operands, size_t operand_bytes, int iters, int blocks,
                                             void *sink, size_t sink_bytes, double *flop, void *stream)
{
    if (kind != 0 && kind != 1) return HLQ_ERR_UNSUPPORTED;
    if (!operands || !sink) return HLQ_ERR_NULL;
    if (((uintptr_t)operands & 15u) || ((uintptr_t)sink & 3u)) return HLQ_ERR_BAD_STRIDE;
    if (operand_bytes < 16 || (operand_bytes & 15u) || operand_bytes > ((size_t)1 << 30)) return HLQ_ERR_BAD_STRIDE;
    if (iters < 1 || iters > (1 << 20) || blocks < 1 || blocks > 65536) return HLQ_ERR_UNSUPPORTED;
    if (sink_bytes < (size_t)blocks * 256 * 4) return HLQ_ERR_BUFFER_TOO_SMALL;
    hlq_clear_stale_error();
    if (kind == 0) {
        if (flop) *flop = (double)blocks * 4.0 * (double)iters * PROBE_OPERANDS * PROBE_CHAINS * (2.0 * 32 * 32 * 16);
        hipLaunchKernelGGL(hlq_mfma_probe_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream, (const probe_half8 *)operands,
                           (int)(operand_bytes / 16), iters, (float *)sink);
    } else {
        if (flop) *flop = (double)blocks * 4.0 * (double)iters * PROBE_OPERANDS * PROBE_MX_CHAINS * (2.0 * 16 * 16 * 128);
        hipLaunchKernelGGL(hlq_mfma_probe_mx_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream, (const probe_half8 *)operands,
                           (int)(operand_bytes / 16), iters, (float *)sink);
    }
    return hlq_hip_status(hipGetLastError());
}
