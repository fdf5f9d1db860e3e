// hlq_lut_gemm for a few rows (2 <= M <= 32: small-batch decode), matrix-core formulation with the
// work split of the GEMV kernel: weights are streamed once at GEMV speed, the rows ride along.
//
//   Y[M,N] = X[M,K] @ W^,   W^ = sum_j s_j b_j + z   (Eq. 3 / Eq. 6)
//
// A wavefront owns one column tile (64 columns, lane <-> column) and a run of consecutive chunks
// of that tile's record stream.  Per 32-k plane word it rebuilds the 32 fp16 weights of its column
// in registers (mask + packed FMA, see hlq_mfma_common.h), transposes them across the four
// 16-lane groups with v_permlane16_swap / v_permlane32_swap so that each group holds one 8-k
// block of 16 columns -- the B operand of v_mfma_f32_16x16x32_f16 -- and issues four MFMAs (one per
// 16-column block) per block of 16 rows.  A fragments (16 rows x 8 k per lane group) are read
// straight from X, which is small enough to stay in L2.  The W wavefronts of a workgroup take W
// consecutive K ranges of the same tile and add their 16*RB x 64 results through LDS; K can also
// be split across workgroups with the workspace/arrival-counter scheme of the GEMV kernel.
#include "hlq_mfma_common.h"

namespace {

struct SkinnyArgs {
    const char *packed;
    const uint16_t *X;
    void *Y;
    float *part;   // [nslices][M][N]
    int *cnt;      // [ntiles]
    size_t col_bytes;
    long ldx, ldy;
    int M, N, nchunks, ntiles, nslices, cps, out_f32;
};

template <int Q, int G, int RB>
struct SkinnyRegs {
    static constexpr int GS = G < 128 ? G : 128;
    static constexpr int SEG = 128 / GS;
    uint32_t w[Q][4];
    uint16_t mt[SEG][Q + 1];
    uint4v a[RB][4];   // A fragments: row block rb, word d
};

template <int Q, int G, int RB>
__global__ void __launch_bounds__(256)
hlq_gemm_skinny_kernel(const SkinnyArgs P)
{
    using Regs = SkinnyRegs<Q, G, RB>;
    constexpr int GS = Regs::GS, SEG = Regs::SEG;
    constexpr int NACC = 16 * RB;          // accumulator floats per lane
    extern __shared__ float red[];         // [W-1][NACC][64]
    const int W = (int)(blockDim.x >> 6);

    const int tile = (int)blockIdx.x / P.nslices, slice = (int)blockIdx.x % P.nslices;
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int sbeg = slice * P.cps;
    const int send = min(sbeg + P.cps, P.nchunks);
    const int len = send - sbeg;
    const int cbeg = sbeg + (len * wave) / W;
    const int cend = sbeg + (len * (wave + 1)) / W;

    const int tw = hlq_tile_width(tile, P.N);
    const int lane_c = lane < tw ? lane : tw - 1;   // clamped: loads stay in bounds, results dropped
    const char *tile_base = P.packed + (size_t)tile * HLQ_TILE_N * P.col_bytes;
    // A-fragment role of this lane: row (lane % 16) of each row block, k-block lane / 16 of a word
    const int arow = lane & 15, akb = lane >> 4;

    auto load_chunk = [&](int c, Regs &R) {
        const char *rec = tile_base + (size_t)tw * ((size_t)c * Q * 16 + (size_t)hlq_groups_before(c, G) * (Q + 1) * 2);
#pragma unroll
        for (int j = 0; j < Q; ++j) {
            const uint4 v = ((const uint4 *)rec)[j * tw + lane_c];
            R.w[j][0] = v.x; R.w[j][1] = v.y; R.w[j][2] = v.z; R.w[j][3] = v.w;
        }
        const char *mrec = rec;
        if (G > 128) {
            const int c0 = c & ~1;
            mrec = tile_base + (size_t)tw * ((size_t)c0 * Q * 16 + (size_t)hlq_groups_before(c0, G) * (Q + 1) * 2);
        }
        const uint16_t *m = (const uint16_t *)(mrec + (size_t)tw * Q * 16);
#pragma unroll
        for (int sg = 0; sg < SEG; ++sg)
#pragma unroll
            for (int r = 0; r <= Q; ++r) R.mt[sg][r] = m[(sg * (Q + 1) + r) * tw + lane_c];
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
            const int m_ = rb * 16 + arow;
            const uint16_t *xr = P.X + (size_t)(m_ < P.M ? m_ : 0) * P.ldx + (size_t)c * 128 + akb * 8;
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                const uint4v v = *(const uint4v *)(xr + d * 32);
                R.a[rb][d] = m_ < P.M ? v : (uint4v){0u, 0u, 0u, 0u};
            }
        }
    };

    float4v acc[RB][4];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int cb = 0; cb < 4; ++cb) acc[rb][cb] = (float4v){0.f, 0.f, 0.f, 0.f};

    auto step = [&](const Regs &R) {
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            HlqSegScales<Q> sc;
            sc.set(R.mt[(d * 32) / GS]);
            uint32_t wd[Q];
#pragma unroll
            for (int j = 0; j < Q; ++j) wd[j] = R.w[j][d];
            uint32_t wp[16];   // wp[4b + v]: register v of k-block b (8 k) of this lane's column
            hlq_rebuild_word<Q>(wd, sc, wp);
            // 4 x 4 transpose over (16-lane group, k-block): afterwards register set cb of lane group g
            // holds k-block g of the 16 columns of column block cb
            uint4v bop[4];
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const uint2v s01 = __builtin_amdgcn_permlane16_swap(wp[0 + v], wp[4 + v], false, false);
                const uint2v s23 = __builtin_amdgcn_permlane16_swap(wp[8 + v], wp[12 + v], false, false);
                const uint2v t02 = __builtin_amdgcn_permlane32_swap(s01.x, s23.x, false, false);
                const uint2v t13 = __builtin_amdgcn_permlane32_swap(s01.y, s23.y, false, false);
                bop[0][v] = t02.x;
                bop[2][v] = t02.y;
                bop[1][v] = t13.x;
                bop[3][v] = t13.y;
            }
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) {
                const half8v a = __builtin_bit_cast(half8v, R.a[rb][d]);
#pragma unroll
                for (int cb = 0; cb < 4; ++cb)
                    acc[rb][cb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, __builtin_bit_cast(half8v, bop[cb]), acc[rb][cb], 0, 0, 0);
            }
        }
    };

    // ---- chunk loop: two register sets, the next chunk's loads in flight -----------------------------
    if (cbeg < cend) {
        Regs RA, RB_;
        load_chunk(cbeg, RA);
        load_chunk(min(cbeg + 1, cend - 1), RB_);
        for (int c = cbeg; c < cend; c += 2) {
            step(RA);
            load_chunk(min(c + 2, cend - 1), RA);
            if (c + 1 < cend) step(RB_);
            load_chunk(min(c + 3, cend - 1), RB_);
        }
    }

    // ---- add the W wavefronts' K ranges ------------------------------------------------------------------
    if (wave > 0) {
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
#pragma unroll
            for (int cb = 0; cb < 4; ++cb)
#pragma unroll
                for (int r = 0; r < 4; ++r) red[((wave - 1) * NACC + (rb * 4 + cb) * 4 + r) * 64 + lane] = acc[rb][cb][r];
    }
    __syncthreads();
    if (wave > 0) return;
    for (int w2 = 1; w2 < W; ++w2) {
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
#pragma unroll
            for (int cb = 0; cb < 4; ++cb)
#pragma unroll
                for (int r = 0; r < 4; ++r) acc[rb][cb][r] += red[((w2 - 1) * NACC + (rb * 4 + cb) * 4 + r) * 64 + lane];
    }

    // element (rb, cb, r) of lane l: row 16 rb + 4 (l / 16) + r, column 16 cb + l % 16 of the tile
    const int col0 = lane & 15, row0 = 4 * (lane >> 4);
    if (P.nslices == 1) {
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
#pragma unroll
            for (int cb = 0; cb < 4; ++cb) {
                const int col = cb * 16 + col0;
                if (col >= tw) continue;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int m = rb * 16 + row0 + r;
                    if (m >= P.M) continue;
                    const size_t off = (size_t)m * P.ldy + (size_t)tile * HLQ_TILE_N + col;
                    if (P.out_f32) ((float *)P.Y)[off] = acc[rb][cb][r];
                    else ((_Float16 *)P.Y)[off] = (_Float16)acc[rb][cb][r];
                }
            }
        return;
    }
    // ---- split-K across workgroups: device-scope write-through partials, arrival counter, the last
    // workgroup adds the partials in slice order (same scheme as the GEMV kernel) -----------------------
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int cb = 0; cb < 4; ++cb) {
            const int col = cb * 16 + col0;
            if (col >= tw) continue;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int m = rb * 16 + row0 + r;
                if (m >= P.M) continue;
                __hip_atomic_store(&P.part[((size_t)slice * P.M + m) * P.N + (size_t)tile * HLQ_TILE_N + col], acc[rb][cb][r],
                                   __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    int old = 0;
    if (lane == 0) old = __hip_atomic_fetch_add(&P.cnt[tile], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    old = __builtin_amdgcn_readfirstlane(old);
    if (old != P.nslices - 1) return;
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int cb = 0; cb < 4; ++cb) {
            const int col = cb * 16 + col0;
            if (col >= tw) continue;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int m = rb * 16 + row0 + r;
                if (m >= P.M) continue;
                const size_t e = (size_t)m * P.N + (size_t)tile * HLQ_TILE_N + col;
                float a = 0.f;
                for (int sl = 0; sl < P.nslices; ++sl)
                    a += __hip_atomic_load(&P.part[(size_t)sl * P.M * P.N + e], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                const size_t off = (size_t)m * P.ldy + (size_t)tile * HLQ_TILE_N + col;
                if (P.out_f32) ((float *)P.Y)[off] = a;
                else ((_Float16 *)P.Y)[off] = (_Float16)a;
            }
        }
    if (lane == 0) __hip_atomic_store(&P.cnt[tile], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

struct SkinnyPlan {
    int RB, W, cps, nslices;
};

SkinnyPlan plan_skinny(const HlqDims &dm, int64_t M)
{
    SkinnyPlan p;
    p.RB = M > 16 ? 2 : 1;
    p.W = 4;
    // about four chunks per wavefront, as for the GEMV; fewer K slices once the tiles alone fill the chip
    const long units = (long)dm.ntiles * dm.nchunks;
    const int cpw = units >= 65536 ? 8 : 4;
    int cps = (p.W * cpw + 1) & ~1;
    p.nslices = (dm.nchunks + cps - 1) / cps;
    p.cps = ((dm.nchunks + p.nslices - 1) / p.nslices + 1) & ~1;
    return p;
}

template <int Q, int G>
void launch_qg(const SkinnyArgs &a, const SkinnyPlan &p, unsigned nblocks, hipStream_t st)
{
    const dim3 blk(64 * p.W);
    const size_t lds = (size_t)(p.W - 1) * 16 * p.RB * 64 * sizeof(float);
    if (p.RB == 1) hlq_gemm_skinny_kernel<Q, G, 1><<<nblocks, blk, lds, st>>>(a);
    else hlq_gemm_skinny_kernel<Q, G, 2><<<nblocks, blk, lds, st>>>(a);
}

template <int Q>
hlq_status launch_q(int G, const SkinnyArgs &a, const SkinnyPlan &p, unsigned nblocks, hipStream_t st)
{
    switch (G) {
    case 32: launch_qg<Q, 32>(a, p, nblocks, st); return HLQ_OK;
    case 64: launch_qg<Q, 64>(a, p, nblocks, st); return HLQ_OK;
    case 128: launch_qg<Q, 128>(a, p, nblocks, st); return HLQ_OK;
    case 256: launch_qg<Q, 256>(a, p, nblocks, st); return HLQ_OK;
    }
    return HLQ_ERR_UNSUPPORTED;
}

} // namespace

size_t hlq_gemm_skinny_partial_bytes(const HlqDims &dm, int64_t M)
{
    if (M > 32) return 0;
    const SkinnyPlan p = plan_skinny(dm, M);
    return p.nslices > 1 ? (size_t)p.nslices * (size_t)M * (size_t)dm.N * sizeof(float) : 0;
}

hlq_status hlq_launch_gemm_skinny(const HlqDims &dm, const void *packed, const uint16_t *X, int64_t M, int64_t ldx,
                                  void *Y, int64_t ldy, hlq_out_dtype out, void *ws, hipStream_t st)
{
    hlq_clear_stale_error();
    if (M < 1 || M > 32) return HLQ_ERR_UNSUPPORTED;
    const SkinnyPlan p = plan_skinny(dm, M);
    if (p.nslices > 1 && (long)dm.ntiles > HLQ_WS_COUNTER_BYTES / 4) return HLQ_ERR_UNSUPPORTED;
    SkinnyArgs a;
    a.packed = (const char *)packed;
    a.X = X;
    a.Y = Y;
    a.cnt = (int *)ws;
    a.part = (float *)((char *)ws + HLQ_WS_COUNTER_BYTES);
    a.col_bytes = dm.col_bytes;
    a.ldx = (long)ldx;
    a.ldy = (long)ldy;
    a.M = (int)M;
    a.N = dm.N;
    a.nchunks = dm.nchunks;
    a.ntiles = dm.ntiles;
    a.nslices = p.nslices;
    a.cps = p.cps;
    a.out_f32 = out == HLQ_OUT_F32;
    const unsigned nblocks = (unsigned)((long)dm.ntiles * p.nslices);
    hlq_status s;
    switch (dm.q) {
    case 1: s = launch_q<1>(dm.G, a, p, nblocks, st); break;
    case 2: s = launch_q<2>(dm.G, a, p, nblocks, st); break;
    case 3: s = launch_q<3>(dm.G, a, p, nblocks, st); break;
    case 4: s = launch_q<4>(dm.G, a, p, nblocks, st); break;
    default: return HLQ_ERR_UNSUPPORTED;
    }
    if (s != HLQ_OK) return s;
    return hlq_hip_status(hipGetLastError());
}
