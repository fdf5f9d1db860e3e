// hlq_lut_gemv: M = 1 bit-serial LUT GEMV (Sec. 2 "Bit-Serial LUT-Based GEMM", App. B).
//
// Work split: a workgroup of 256 lanes owns 256 adjacent output columns and a slice of U
// chunks (U*128 consecutive k).  Lane <-> column, so every lane of a wavefront indexes the
// SAME 16-entry table at the same time: the 16 fp32 entries sit in 16 different LDS banks
// and equal addresses broadcast, hence no bank conflicts by construction.
//
//   1. every lane issues its 128-bit plane loads and its scale/zero loads (HBM latency
//      starts first),
//   2. lanes 0 .. 32U-1 each build one table (15 adds, four 128-bit LDS writes) and the
//      per-segment activation sums (wave shuffles),
//   3. one barrier,
//   4. per plane and 4-bit slice: one LDS lookup + one fp32 add; per (plane, quant group)
//      one FMA with s_j; per quant group one FMA  z * sum(x)           (Eq. 3 by linearity),
//   5. the slice's partial sum goes to y (one slice) or to the workspace, which a second
//      small kernel reduces in a fixed order (deterministic; no float atomics).
#include "hlq_internal.h"

namespace {

__device__ __forceinline__ float h2f(uint16_t h) { return (float)__builtin_bit_cast(_Float16, h); }

__device__ __forceinline__ void store_out(void *y, size_t idx, float v, int out_f32)
{
    if (out_f32) ((float *)y)[idx] = v;
    else ((_Float16 *)y)[idx] = (_Float16)v;   // round-to-nearest-even
}

template <int Q, int G, int U>
__global__ void __launch_bounds__(256)
hlq_gemv_kernel(const uint4 *__restrict__ bits, const uint16_t *__restrict__ meta,
                const uint16_t *__restrict__ x, void *__restrict__ y, float *__restrict__ ws,
                int N, int nchunks, int nslices, int out_f32)
{
    constexpr int GS = G < 128 ? G : 128;   // k covered by one scale inside a chunk
    constexpr int SEG = 128 / GS;           // scale segments per chunk
    constexpr int TPS = GS / 4;             // tables per segment
    __shared__ __attribute__((aligned(16))) float T[U * 32 * 16];
    __shared__ float XS[U * SEG];

    const int tid = threadIdx.x;
    const int n = blockIdx.x * 256 + tid;
    const int c0 = blockIdx.y * U;
    const bool col_ok = n < N;

    // ---- 1. weight and scale loads ------------------------------------------------------
    uint4 w[U][Q];
    uint16_t mt[U][SEG][Q + 1];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int c = c0 + u;
        const bool ok = col_ok && c < nchunks;
#pragma unroll
        for (int j = 0; j < Q; ++j)
            w[u][j] = ok ? bits[((size_t)j * nchunks + c) * N + n] : make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
        for (int s = 0; s < SEG; ++s) {
            const int g = (G >= 128) ? (c * 128) / G : c * SEG + s;
#pragma unroll
            for (int r = 0; r <= Q; ++r)
                mt[u][s][r] = ok ? meta[((size_t)g * (Q + 1) + r) * N + n] : (uint16_t)0;
        }
    }

    // ---- 2. tables: T[t][i] = sum_r bit_r(i) * x[4t + r]  (App. B) --------------------------
    if (tid < 32 * U) {
        const int k = c0 * 128 + 4 * tid;
        float xv[4] = {0.f, 0.f, 0.f, 0.f};
        if (k < nchunks * 128) {
            const uint2 raw = *(const uint2 *)(x + k);
            xv[0] = h2f((uint16_t)(raw.x & 0xffffu));
            xv[1] = h2f((uint16_t)(raw.x >> 16));
            xv[2] = h2f((uint16_t)(raw.y & 0xffffu));
            xv[3] = h2f((uint16_t)(raw.y >> 16));
        }
        float e[16];
        e[0] = 0.f;
#pragma unroll
        for (int i = 1; i < 16; ++i) e[i] = e[i & (i - 1)] + xv[__builtin_ctz(i)];
        float4 *dst = (float4 *)(T + tid * 16);
#pragma unroll
        for (int v = 0; v < 4; ++v) dst[v] = make_float4(e[4 * v], e[4 * v + 1], e[4 * v + 2], e[4 * v + 3]);
        // sum of the segment's activations = sum of its tables' last entries
        float tot = e[15];
#pragma unroll
        for (int off = TPS / 2; off >= 1; off >>= 1) tot += __shfl_xor(tot, off);
        if (tid % TPS == 0) XS[tid / TPS] = tot;
    }
    __syncthreads();

    // ---- 4. lookups ---------------------------------------------------------------------------
    float acc = 0.f;
#pragma unroll
    for (int u = 0; u < U; ++u) {
#pragma unroll
        for (int s = 0; s < SEG; ++s) {
#pragma unroll
            for (int j = 0; j < Q; ++j) {
                const uint32_t wd[4] = {w[u][j].x, w[u][j].y, w[u][j].z, w[u][j].w};
                float p0 = 0.f, p1 = 0.f;
#pragma unroll
                for (int tt = 0; tt < TPS; tt += 2) {
                    const int t0 = s * TPS + tt, t1 = t0 + 1;
                    const uint32_t i0 = (wd[t0 >> 3] >> (4 * (t0 & 7))) & 15u;
                    const uint32_t i1 = (wd[t1 >> 3] >> (4 * (t1 & 7))) & 15u;
                    p0 += T[(u * 32 + t0) * 16 + i0];
                    p1 += T[(u * 32 + t1) * 16 + i1];
                }
                acc += h2f(mt[u][s][j]) * (p0 + p1);
            }
            acc += h2f(mt[u][s][Q]) * XS[u * SEG + s];
        }
    }

    // ---- 5. store ---------------------------------------------------------------------------
    if (!col_ok) return;
    if (nslices == 1) store_out(y, n, acc, out_f32);
    else ws[(size_t)blockIdx.y * N + n] = acc;
}

__global__ void __launch_bounds__(256)
hlq_splitk_reduce_kernel(const float *__restrict__ ws, void *__restrict__ y, int total, int nslices,
                         int out_f32)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    float acc = 0.f;
    for (int s = 0; s < nslices; ++s) acc += ws[(size_t)s * total + i];
    store_out(y, i, acc, out_f32);
}

template <int Q, int G>
hlq_status launch_qg(const HlqDims &dm, const HlqPlan &pl, const uint4 *bits, const uint16_t *meta,
                     const uint16_t *x, void *y, float *ws, int out_f32, hipStream_t st)
{
    const dim3 grid((unsigned)((dm.N + 255) / 256), (unsigned)pl.nslices);
    switch (pl.chunks_per_wg) {
    case 1: hlq_gemv_kernel<Q, G, 1><<<grid, 256, 0, st>>>(bits, meta, x, y, ws, dm.N, dm.nchunks, pl.nslices, out_f32); break;
    case 2: hlq_gemv_kernel<Q, G, 2><<<grid, 256, 0, st>>>(bits, meta, x, y, ws, dm.N, dm.nchunks, pl.nslices, out_f32); break;
    case 4: hlq_gemv_kernel<Q, G, 4><<<grid, 256, 0, st>>>(bits, meta, x, y, ws, dm.N, dm.nchunks, pl.nslices, out_f32); break;
    default: return HLQ_ERR_UNSUPPORTED;
    }
    return HLQ_OK;
}

template <int Q>
hlq_status launch_q(const HlqDims &dm, const HlqPlan &pl, const uint4 *bits, const uint16_t *meta,
                    const uint16_t *x, void *y, float *ws, int out_f32, hipStream_t st)
{
    switch (dm.G) {
    case 32: return launch_qg<Q, 32>(dm, pl, bits, meta, x, y, ws, out_f32, st);
    case 64: return launch_qg<Q, 64>(dm, pl, bits, meta, x, y, ws, out_f32, st);
    case 128: return launch_qg<Q, 128>(dm, pl, bits, meta, x, y, ws, out_f32, st);
    case 256: return launch_qg<Q, 256>(dm, pl, bits, meta, x, y, ws, out_f32, st);
    }
    return HLQ_ERR_UNSUPPORTED;
}

} // namespace

HlqPlan hlq_plan_gemv(const HlqDims &dm)
{
    // Enough workgroups to cover 256 CUs a few times over, as few split-K partials as that allows.
    const int ntiles = (dm.N + 255) / 256;
    int U = 4;
    if (dm.q >= 3) U = 2;
    while (U > 1 && (long)ntiles * ((dm.nchunks + U - 1) / U) < 1024) U >>= 1;
    HlqPlan pl;
    pl.chunks_per_wg = U;
    pl.nslices = (dm.nchunks + U - 1) / U;
    return pl;
}

size_t hlq_gemv_ws_bytes(const HlqDims &dm)
{
    const HlqPlan pl = hlq_plan_gemv(dm);
    return pl.nslices > 1 ? (size_t)pl.nslices * (size_t)dm.N * sizeof(float) : 0;
}

hlq_status hlq_launch_gemv(const HlqDims &dm, const void *packed, const uint16_t *x, void *y,
                           hlq_out_dtype out, void *ws, hipStream_t st)
{
    const HlqPlan pl = hlq_plan_gemv(dm);
    const uint4 *bits = (const uint4 *)packed;
    const uint16_t *meta = (const uint16_t *)((const char *)packed + dm.bits_bytes);
    const int out_f32 = out == HLQ_OUT_F32;
    hlq_status s;
    switch (dm.q) {
    case 1: s = launch_q<1>(dm, pl, bits, meta, x, y, (float *)ws, out_f32, st); break;
    case 2: s = launch_q<2>(dm, pl, bits, meta, x, y, (float *)ws, out_f32, st); break;
    case 3: s = launch_q<3>(dm, pl, bits, meta, x, y, (float *)ws, out_f32, st); break;
    case 4: s = launch_q<4>(dm, pl, bits, meta, x, y, (float *)ws, out_f32, st); break;
    default: return HLQ_ERR_UNSUPPORTED;
    }
    if (s != HLQ_OK) return s;
    if (pl.nslices > 1) {
        const unsigned nb = (unsigned)((dm.N + 255) / 256);
        hlq_splitk_reduce_kernel<<<nb, 256, 0, st>>>((const float *)ws, y, dm.N, pl.nslices, out_f32);
    }
    return hlq_hip_status(hipGetLastError());
}
