// hlq_lut_gemm: M > 1 bit-serial LUT GEMM (Sec. 2 "Bit-Serial LUT-Based GEMM", App. B),
// table-lookup formulation with one table set per activation row.
//
// A workgroup owns 256 adjacent columns, MB rows and a slice of K that it walks in steps of
// U = 2 chunks (256 k).  Table entries of the MB rows are interleaved, T[t][i][r], so one LDS
// read of MB floats serves all rows for a decoded 4-bit slice: the weight words are loaded
// and decoded once per step and shared by the rows, as in the batched reading of App. B.
#include <atomic>

#include "hlq_internal.h"

namespace {

__device__ __forceinline__ float h2f(uint16_t h) { return (float)__builtin_bit_cast(_Float16, h); }

__device__ __forceinline__ void store_out(void *y, size_t idx, float v, int out_f32)
{
    if (out_f32) ((float *)y)[idx] = v;
    else ((_Float16 *)y)[idx] = (_Float16)v;   // round-to-nearest-even
}

template <int MB> struct RowVec;
template <> struct RowVec<1> { float v[1]; };
template <> struct RowVec<2> { float v[2]; };
template <> struct RowVec<4> { float v[4]; };

template <int Q, int G, int MB>
__global__ void __launch_bounds__(256)
hlq_gemm_lut_kernel(const char *__restrict__ packed, size_t col_bytes,
                    const uint16_t *__restrict__ X, long ldx, int M, void *__restrict__ Y, long ldy,
                    float *__restrict__ ws, int N, int nchunks, int chunks_per_slice, int nslices,
                    int out_f32)
{
    constexpr int U = 2;
    constexpr int GS = G < 128 ? G : 128;
    constexpr int SEG = 128 / GS;
    constexpr int TPS = GS / 4;
    constexpr int NT = 32 * U;              // tables per step
    static_assert(NT * MB <= 256, "one table-build item per lane");
    __shared__ __attribute__((aligned(16))) float T[NT * 16 * MB];
    __shared__ float XS[U * SEG * MB];

    const int tid = threadIdx.x;
    const int n = blockIdx.x * 256 + tid;
    const bool col_ok = n < N;
    const int tile = n / HLQ_TILE_N, lane = n % HLQ_TILE_N;   // wavefront <-> column tile
    const int tw = col_ok ? hlq_tile_width(tile, N) : 0;
    const char *tile_base = packed + (size_t)tile * HLQ_TILE_N * col_bytes;
    const int m0 = blockIdx.z * MB;
    const int cbeg = blockIdx.y * chunks_per_slice;
    const int cend = min(cbeg + chunks_per_slice, nchunks);

    float acc[MB];
#pragma unroll
    for (int r = 0; r < MB; ++r) acc[r] = 0.f;

    for (int c0 = cbeg; c0 < cend; c0 += U) {
        uint4 w[U][Q];
        uint16_t mt[U][SEG][Q + 1];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int c = c0 + u;
            const bool ok = col_ok && c < cend;
            const char *rec = tile_base + hlq_rec_in_tile(tw, c, Q, G);
#pragma unroll
            for (int j = 0; j < Q; ++j)
                w[u][j] = ok ? ((const uint4 *)rec)[j * tw + lane] : make_uint4(0u, 0u, 0u, 0u);
            const char *mrec = rec;
            if (G > 128) {   // the group's meta sits in the record of its first (even) chunk
                const int ce = c & ~1;
                mrec = tile_base + hlq_rec_in_tile(tw, ce, Q, G);
            }
            const uint16_t *mp = (const uint16_t *)(mrec + (size_t)tw * Q * 16);
#pragma unroll
            for (int s = 0; s < SEG; ++s)
#pragma unroll
                for (int r = 0; r <= Q; ++r)
                    mt[u][s][r] = ok ? mp[(s * (Q + 1) + r) * tw + lane] : (uint16_t)0;
        }

        __syncthreads();   // readers of the previous step's tables are done
        if (tid < NT * MB) {
            const int r = tid / NT, tl = tid % NT;   // a wavefront builds one row's 64 tables
            // table tl = word (tl / 8), 4-bit slice i = tl % 8: the four even (i < 4) or odd (i >= 4)
            // activations of the 8-k window 4 * (tl / 8) + (i & 3)
            const int wnd = 4 * (tl >> 3) + (tl & 3), par = (tl >> 2) & 1;
            const int k = c0 * 128 + 8 * wnd;
            const int m = m0 + r;
            float xv[4] = {0.f, 0.f, 0.f, 0.f};
            if (m < M && k < cend * 128) {
                const uint4 raw = *(const uint4 *)(X + (size_t)m * ldx + k);
                const uint32_t xd[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
                for (int v = 0; v < 4; ++v) xv[v] = h2f((uint16_t)(xd[v] >> (16 * par)));
            }
            float e[16];
            e[0] = 0.f;
#pragma unroll
            for (int i = 1; i < 16; ++i) e[i] = e[i & (i - 1)] + xv[__builtin_ctz(i)];
#pragma unroll
            for (int i = 0; i < 16; ++i) T[(tl * 16 + i) * MB + r] = e[i];
            float tot = e[15];
#pragma unroll
            for (int off = TPS / 2; off >= 1; off >>= 1) tot += __shfl_xor(tot, off);
            if (tl % TPS == 0) XS[(tl / TPS) * MB + r] = tot;
        }
        __syncthreads();

#pragma unroll
        for (int u = 0; u < U; ++u) {
#pragma unroll
            for (int s = 0; s < SEG; ++s) {
#pragma unroll
                for (int j = 0; j < Q; ++j) {
                    const uint32_t wd[4] = {w[u][j].x, w[u][j].y, w[u][j].z, w[u][j].w};
                    float p[MB];
#pragma unroll
                    for (int r = 0; r < MB; ++r) p[r] = 0.f;
#pragma unroll
                    for (int tt = 0; tt < TPS; ++tt) {
                        const int t = s * TPS + tt;
                        const uint32_t idx = (wd[t >> 3] >> (4 * (t & 7))) & 15u;
                        const RowVec<MB> e = *(const RowVec<MB> *)(T + ((u * 32 + t) * 16 + idx) * MB);
#pragma unroll
                        for (int r = 0; r < MB; ++r) p[r] += e.v[r];
                    }
                    const float sj = h2f(mt[u][s][j]);
#pragma unroll
                    for (int r = 0; r < MB; ++r) acc[r] += sj * p[r];
                }
                const float z = h2f(mt[u][s][Q]);
#pragma unroll
                for (int r = 0; r < MB; ++r) acc[r] += z * XS[(u * SEG + s) * MB + r];
            }
        }
    }

    if (!col_ok) return;
#pragma unroll
    for (int r = 0; r < MB; ++r) {
        const int m = m0 + r;
        if (m >= M) break;
        if (nslices == 1) store_out(Y, (size_t)m * ldy + n, acc[r], out_f32);
        else ws[((size_t)blockIdx.y * M + m) * N + n] = acc[r];
    }
}

__global__ void __launch_bounds__(256)
hlq_gemm_reduce_kernel(const float *__restrict__ ws, void *__restrict__ Y, long ldy, int M, int N,
                       int nslices, int out_f32)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    const size_t total = (size_t)M * N;
    if (i >= total) return;
    float acc = 0.f;
    for (int s = 0; s < nslices; ++s) acc += ws[(size_t)s * total + i];
    const size_t m = i / N, n = i % N;
    store_out(Y, m * ldy + n, acc, out_f32);
}

struct GemmPlan {
    int MB, chunks_per_slice, nslices, rowblocks;
};

GemmPlan plan_gemm(const HlqDims &dm, int64_t M)
{
    GemmPlan p;
    p.MB = M >= 3 ? 4 : 2;
    p.rowblocks = (int)((M + p.MB - 1) / p.MB);
    const long ntiles = (dm.N + 255) / 256;
    const long wg_cols = ntiles * p.rowblocks;
    long want = (1024 + wg_cols - 1) / wg_cols;          // slices wanted to fill the chip
    const long max_slices = (dm.nchunks + 1) / 2;        // a slice is at least one step (2 chunks)
    if (want > max_slices) want = max_slices;
    if (want < 1) want = 1;
    int cps = (int)((dm.nchunks + want - 1) / want);
    cps = (cps + 1) & ~1;                                 // whole steps
    p.chunks_per_slice = cps;
    p.nslices = (dm.nchunks + cps - 1) / cps;
    return p;
}

template <int Q, int G, int MB>
void launch_one(const HlqDims &dm, const GemmPlan &p, const char *bits, size_t meta,
                const uint16_t *X, long ldx, int M, void *Y, long ldy, float *ws, int out_f32,
                hipStream_t st)
{
    const dim3 grid((unsigned)((dm.N + 255) / 256), (unsigned)p.nslices, (unsigned)p.rowblocks);
    hlq_gemm_lut_kernel<Q, G, MB><<<grid, 256, 0, st>>>(bits, meta, X, ldx, M, Y, ldy, ws, dm.N, dm.nchunks,
                                                        p.chunks_per_slice, p.nslices, out_f32);
}

template <int Q, int G>
void launch_qg(const HlqDims &dm, const GemmPlan &p, const char *bits, size_t meta,
               const uint16_t *X, long ldx, int M, void *Y, long ldy, float *ws, int out_f32,
               hipStream_t st)
{
    if (p.MB == 2) launch_one<Q, G, 2>(dm, p, bits, meta, X, ldx, M, Y, ldy, ws, out_f32, st);
    else launch_one<Q, G, 4>(dm, p, bits, meta, X, ldx, M, Y, ldy, ws, out_f32, st);
}

template <int Q>
hlq_status launch_q(const HlqDims &dm, const GemmPlan &p, const char *bits, size_t meta,
                    const uint16_t *X, long ldx, int M, void *Y, long ldy, float *ws, int out_f32,
                    hipStream_t st)
{
    switch (dm.G) {
    case 32: launch_qg<Q, 32>(dm, p, bits, meta, X, ldx, M, Y, ldy, ws, out_f32, st); return HLQ_OK;
    case 64: launch_qg<Q, 64>(dm, p, bits, meta, X, ldx, M, Y, ldy, ws, out_f32, st); return HLQ_OK;
    case 128: launch_qg<Q, 128>(dm, p, bits, meta, X, ldx, M, Y, ldy, ws, out_f32, st); return HLQ_OK;
    case 256: launch_qg<Q, 256>(dm, p, bits, meta, X, ldx, M, Y, ldy, ws, out_f32, st); return HLQ_OK;
    }
    return HLQ_ERR_UNSUPPORTED;
}

} // namespace

size_t hlq_gemm_lut_partial_bytes(const HlqDims &dm, int64_t M)
{
    const GemmPlan p = plan_gemm(dm, M);
    return p.nslices > 1 ? (size_t)p.nslices * (size_t)M * (size_t)dm.N * sizeof(float) : 0;
}

hlq_status hlq_launch_gemm_lut(const HlqDims &dm, const void *packed, const uint16_t *X, int64_t M,
                           int64_t ldx, void *Y, int64_t ldy, hlq_out_dtype out, void *ws,
                           hipStream_t st)
{
    hlq_clear_stale_error();
    if (M > (int64_t)65535 * 2) return HLQ_ERR_UNSUPPORTED;   // grid.z limit
    const GemmPlan p = plan_gemm(dm, M);
    const char *bits = (const char *)packed;
    const size_t meta = dm.col_bytes;
    const int out_f32 = out == HLQ_OUT_F32;
    ws = (char *)ws + HLQ_WS_COUNTER_BYTES;   // partial sums follow the counter block
    hlq_status s;
    switch (dm.q) {
    case 1: s = launch_q<1>(dm, p, bits, meta, X, (long)ldx, (int)M, Y, (long)ldy, (float *)ws, out_f32, st); break;
    case 2: s = launch_q<2>(dm, p, bits, meta, X, (long)ldx, (int)M, Y, (long)ldy, (float *)ws, out_f32, st); break;
    case 3: s = launch_q<3>(dm, p, bits, meta, X, (long)ldx, (int)M, Y, (long)ldy, (float *)ws, out_f32, st); break;
    case 4: s = launch_q<4>(dm, p, bits, meta, X, (long)ldx, (int)M, Y, (long)ldy, (float *)ws, out_f32, st); break;
    default: return HLQ_ERR_UNSUPPORTED;
    }
    if (s != HLQ_OK) return s;
    if (p.nslices > 1) {
        const size_t total = (size_t)M * dm.N;
        const unsigned nb = (unsigned)((total + 255) / 256);
        hlq_gemm_reduce_kernel<<<nb, 256, 0, st>>>((const float *)ws, Y, (long)ldy, (int)M, dm.N, p.nslices, out_f32);
    }
    return hlq_hip_status(hipGetLastError());
}

// ---- formulation choice ---------------------------------------------------------------------------
// 0 = automatic (by M), 1 = table lookups (this file), 2 = matrix cores (hlq_gemm_mfma.hip)
static std::atomic<int> g_gemm_path{0};

hlq_status hlq_gemm_path_override(int path)
{
    if (path < 0 || path > 4) return HLQ_ERR_UNSUPPORTED;
    g_gemm_path = path;
    return HLQ_OK;
}

static bool use_mfma(int64_t M)
{
    const int path = g_gemm_path.load(std::memory_order_relaxed);
    if (path == 1) return false;
    if (path >= 2) return true;
    // measured on MI355X (8B shapes, q = 2..4, HIP-graph timing): the matrix-core kernels are faster
    // than the lookup kernel from M = 2 on, and the gap grows with M
    return M >= 2;
}

// true if hlq_launch_gemm sends M rows (that fit one pass) to the few-rows matrix-core GEMV kernel
bool hlq_gemm_uses_mx_rows(int64_t M) { return use_mfma(M) && g_gemm_path.load(std::memory_order_relaxed) != 3; }

// true if the many-rows kernel is to take all the rows it can carry (hlq_set_gemm_path(4))
bool hlq_gemm_rows_all() { return g_gemm_path.load(std::memory_order_relaxed) == 4; }

// true if hlq_launch_gemm computes M rows on the matrix cores (either kernel)
bool hlq_gemm_uses_matrix_cores(int64_t M) { return use_mfma(M); }

size_t hlq_gemm_partial_bytes(const HlqDims &dm, int64_t M)
{
    size_t a = hlq_gemm_lut_partial_bytes(dm, M);
    const size_t b = hlq_gemm_mfma_partial_bytes(dm, M);
    const size_t e = hlq_gemm_mx_partial_bytes(dm, M);
    if (b > a) a = b;
    if (e > a) a = e;
    return a;
}

hlq_status hlq_launch_gemm(const HlqDims &dm, const void *packed, const uint16_t *X, int64_t M, int64_t ldx,
                           void *Y, int64_t ldy, hlq_out_dtype out, void *ws, hipStream_t st)
{
    if (use_mfma(M)) {
        // up to one row set of the matrix-core GEMV kernel (several activation rows per operand): measured
        // faster than the tiled kernel there; from the second row set on the tiled kernel, whose time
        // hardly depends on M up to 32 rows, is as fast or faster for a single call
        if (g_gemm_path.load(std::memory_order_relaxed) != 3 && M <= hlq_gemv_mx_rows_per_set(dm.G))
            return hlq_launch_gemm_mx_rows(dm, packed, X, M, ldx, Y, ldy, out, ws, st);
        // 5..16 rows on a large matrix: the many-rows kernel (same rule as for grouped launches)
        if (g_gemm_path.load(std::memory_order_relaxed) != 3 && M <= hlq_gemm_rows_max(dm.G) &&
            (hlq_gemm_rows_all() || hlq_gemm_rows_wins((long)dm.ntiles * dm.nchunks, dm.q, M)))
            return hlq_launch_gemm_mx_rows(dm, packed, X, M, ldx, Y, ldy, out, ws, st);
        return hlq_launch_gemm_mfma(dm, packed, X, M, ldx, Y, ldy, out, ws, st);
    }
    return hlq_launch_gemm_lut(dm, packed, X, M, ldx, Y, ldy, out, ws, st);
}
