// hlq_lut_gemv: M = 1 bit-serial LUT GEMV (Sec. 2 "Bit-Serial LUT-Based GEMM", App. B),
// one launch for one or several independent GEMVs.
//
// Work split.  The unit of work is a wavefront: it owns one column tile (64 columns, lane <->
// column) and a run of consecutive chunks (128 k each), i.e. one contiguous byte stream of the
// packed blob.  Per chunk it
//
//   build    makes its OWN 32 tables in LDS (T[t][i] = sum_r bit_r(i) x[4t+r], App. B): lane
//            (t, h) computes entries 8h .. 8h+7 of table t and stores them with two 128-bit LDS
//            writes; the per-quant-group activation sums come from a shuffle reduction;
//   consume  per plane and 4-bit slice one LDS lookup + one fp32 add; per (plane, quant group)
//            one FMA with s_j; per quant group one FMA z * sum(x)   (Eq. 3 by linearity).
//
// All lanes of the wavefront index the same 16-entry fp32 table at the same time: its entries
// lie in 16 different LDS banks and equal addresses broadcast, so lookups are conflict-free by
// construction.  Because tables are private to the wavefront and LDS operations of one
// wavefront execute in order, the chunk loop has no barrier at all; the weight loads of chunk
// c+1 are in flight while chunk c is consumed (two register sets).
//
// The four wavefronts of a workgroup take four consecutive K ranges of the SAME tile and add
// their results through LDS.  If K is also split across workgroups ("slices"), each workgroup
// writes its partial sums to the workspace and bumps an arrival counter; the last one to arrive
// adds the partials in slice order, so the result does not depend on arrival order.
#include <stdlib.h>

#include "hlq_internal.h"

namespace {

struct GemvProb {
    const char *packed;
    const uint16_t *x;
    void *y;
    float *part;       // [nslices][N] partial sums (nslices > 1)
    int *cnt;          // [ntiles] arrival counters, zero between launches
    size_t col_bytes;
    int N, nchunks, ntiles, nslices, cps, blk_begin;
};

struct GemvBatch {
    GemvProb p[HLQ_MAX_BATCH];
    int count;
    int out_f32;
};

__device__ __forceinline__ float h2f(uint16_t h) { return (float)__builtin_bit_cast(_Float16, h); }

__device__ __forceinline__ void store_out(void *y, size_t idx, float v, int out_f32)
{
    if (out_f32) ((float *)y)[idx] = v;
    else ((_Float16 *)y)[idx] = (_Float16)v;   // round-to-nearest-even
}

template <int Q, int G>
struct ChunkRegs {
    static constexpr int GS = G < 128 ? G : 128;   // k covered by one scale inside a chunk
    static constexpr int SEG = 128 / GS;           // scale segments per chunk
    uint32_t w[Q][4];
    uint16_t mt[SEG][Q + 1];
    uint2 x;                                       // this lane's four activations (table build)
};

// ---- hand-scheduled lookup blocks -----------------------------------------------------------------
// One block serves NW consecutive 32-bit plane words (8 * NW lookups) of one (plane, quant
// segment).  For 4-bit slice i of a word the LDS byte address is  base + 64*table + 4*slice.
// Per word: two shifts put slice*4 into bits [5:2] of a byte ((w << 2) for even slices, (w >> 2)
// for odd ones); one sub-dword AND per slice picks that byte, masks it with 0x3c and writes it
// into byte 0 of an address register whose upper bytes keep the wavefront's 256-aligned table
// base; one ds_read_b32 (table number in the immediate offset) fetches the entry; one v_add_f32
// accumulates it: 2.25 VALU ops per lookup.  The LDS reads of word k+1 are issued before the
// adds of word k.  The block drains the LDS queue on entry, so its own lgkmcnt arithmetic is
// exact, and on exit, so every output is valid for the compiler.
#define HLQ_LK1(R, AD, SRC, BYTE, T)                                                                          \
    "v_and_b32_sdwa " AD ", " SRC ", 60 dst_sel:BYTE_0 dst_unused:UNUSED_PRESERVE src0_sel:BYTE_" #BYTE        \
    " src1_sel:DWORD\n"                                                                                        \
    "ds_read_b32 " R ", " AD " offset:%[off]+" #T "*64\n"
#define HLQ_LK_WORD(W, S, T0, T1, T2, T3, T4, T5, T6, T7)                                                     \
    "v_lshlrev_b32 %[sa], 2, " W "\n"                                                                         \
    "v_lshrrev_b32 %[sb], 2, " W "\n"                                                                         \
    HLQ_LK1("%[" S "0]", "%[d0]", "%[sa]", 0, T0) HLQ_LK1("%[" S "1]", "%[d1]", "%[sb]", 0, T1)               \
    HLQ_LK1("%[" S "2]", "%[d2]", "%[sa]", 1, T2) HLQ_LK1("%[" S "3]", "%[d3]", "%[sb]", 1, T3)               \
    HLQ_LK1("%[" S "4]", "%[d0]", "%[sa]", 2, T4) HLQ_LK1("%[" S "5]", "%[d1]", "%[sb]", 2, T5)               \
    HLQ_LK1("%[" S "6]", "%[d2]", "%[sa]", 3, T6) HLQ_LK1("%[" S "7]", "%[d3]", "%[sb]", 3, T7)
#define HLQ_LK_ADD(S)                                                                                         \
    "v_add_f32 %[p0], %[p0], %[" S "0]\n" "v_add_f32 %[p1], %[p1], %[" S "1]\n"                               \
    "v_add_f32 %[p0], %[p0], %[" S "2]\n" "v_add_f32 %[p1], %[p1], %[" S "3]\n"                               \
    "v_add_f32 %[p0], %[p0], %[" S "4]\n" "v_add_f32 %[p1], %[p1], %[" S "5]\n"                               \
    "v_add_f32 %[p0], %[p0], %[" S "6]\n" "v_add_f32 %[p1], %[p1], %[" S "7]\n"
#define HLQ_LK_OUTS                                                                                           \
    [p0] "+v"(p0), [p1] "+v"(p1), [d0] "+v"(ad[0]), [d1] "+v"(ad[1]), [d2] "+v"(ad[2]), [d3] "+v"(ad[3]),      \
        [sa] "=&v"(sa), [sb] "=&v"(sb), [a0] "=&v"(a0), [a1] "=&v"(a1), [a2] "=&v"(a2), [a3] "=&v"(a3),        \
        [a4] "=&v"(a4), [a5] "=&v"(a5), [a6] "=&v"(a6), [a7] "=&v"(a7)
#define HLQ_LK_OUTS_B                                                                                         \
    , [b0] "=&v"(b0), [b1] "=&v"(b1), [b2] "=&v"(b2), [b3] "=&v"(b3), [b4] "=&v"(b4), [b5] "=&v"(b5),          \
        [b6] "=&v"(b6), [b7] "=&v"(b7)

// `ad`: four address registers holding the wavefront's table base (a multiple of 256) in
// bytes 1..3; OFF: byte offset of the block's first table from that base.
template <int OFF>
__device__ __forceinline__ void lookup_words(const uint32_t (&w)[4], uint32_t (&ad)[4], float &p0, float &p1)
{
    uint32_t sa, sb;
    float a0, a1, a2, a3, a4, a5, a6, a7, b0, b1, b2, b3, b4, b5, b6, b7;
    asm volatile("s_waitcnt lgkmcnt(0)\n"
                 HLQ_LK_WORD("%[w0]", "a", 0, 1, 2, 3, 4, 5, 6, 7)
                 HLQ_LK_WORD("%[w1]", "b", 8, 9, 10, 11, 12, 13, 14, 15)
                 "s_waitcnt lgkmcnt(8)\n"
                 HLQ_LK_ADD("a")
                 HLQ_LK_WORD("%[w2]", "a", 16, 17, 18, 19, 20, 21, 22, 23)
                 "s_waitcnt lgkmcnt(8)\n"
                 HLQ_LK_ADD("b")
                 HLQ_LK_WORD("%[w3]", "b", 24, 25, 26, 27, 28, 29, 30, 31)
                 "s_waitcnt lgkmcnt(8)\n"
                 HLQ_LK_ADD("a")
                 "s_waitcnt lgkmcnt(0)\n"
                 HLQ_LK_ADD("b")
                 : HLQ_LK_OUTS HLQ_LK_OUTS_B
                 : [w0] "v"(w[0]), [w1] "v"(w[1]), [w2] "v"(w[2]), [w3] "v"(w[3]), [off] "n"(OFF)
                 : "memory");
}

template <int OFF>
__device__ __forceinline__ void lookup_words(const uint32_t (&w)[2], uint32_t (&ad)[4], float &p0, float &p1)
{
    uint32_t sa, sb;
    float a0, a1, a2, a3, a4, a5, a6, a7, b0, b1, b2, b3, b4, b5, b6, b7;
    asm volatile("s_waitcnt lgkmcnt(0)\n"
                 HLQ_LK_WORD("%[w0]", "a", 0, 1, 2, 3, 4, 5, 6, 7)
                 HLQ_LK_WORD("%[w1]", "b", 8, 9, 10, 11, 12, 13, 14, 15)
                 "s_waitcnt lgkmcnt(8)\n"
                 HLQ_LK_ADD("a")
                 "s_waitcnt lgkmcnt(0)\n"
                 HLQ_LK_ADD("b")
                 : HLQ_LK_OUTS HLQ_LK_OUTS_B
                 : [w0] "v"(w[0]), [w1] "v"(w[1]), [off] "n"(OFF)
                 : "memory");
}

template <int OFF>
__device__ __forceinline__ void lookup_words(const uint32_t (&w)[1], uint32_t (&ad)[4], float &p0, float &p1)
{
    uint32_t sa, sb;
    float a0, a1, a2, a3, a4, a5, a6, a7;
    asm volatile("s_waitcnt lgkmcnt(0)\n"
                 HLQ_LK_WORD("%[w0]", "a", 0, 1, 2, 3, 4, 5, 6, 7)
                 "s_waitcnt lgkmcnt(0)\n"
                 HLQ_LK_ADD("a")
                 : HLQ_LK_OUTS
                 : [w0] "v"(w[0]), [off] "n"(OFF)
                 : "memory");
}

// All lookups of one chunk, then scales and zeros: compile-time recursion over (segment sg,
// plane j) so that every LDS offset is an immediate.  xs[sg] = sum of the segment's activations.
template <int Q, int G, int I = 0>
struct Consume {
    using Regs = ChunkRegs<Q, G>;
    static constexpr int SEG = Regs::SEG, WPS = Regs::GS / 32;
    static constexpr int sg = I / Q, j = I % Q;
    __device__ __forceinline__ static void run(const Regs &R, const float (&xs)[SEG], uint32_t (&ad)[4], float &acc)
    {
        uint32_t w[WPS];
#pragma unroll
        for (int d = 0; d < WPS; ++d) w[d] = R.w[j][sg * WPS + d];
        float p0 = 0.f, p1 = 0.f;
        lookup_words<sg * WPS * 8 * 64>(w, ad, p0, p1);
        acc += h2f(R.mt[sg][j]) * (p0 + p1);
        if (j == Q - 1) acc += h2f(R.mt[sg][Q]) * xs[sg];
        Consume<Q, G, I + 1>::run(R, xs, ad, acc);
    }
};
template <int Q, int G>
struct Consume<Q, G, (128 / (G < 128 ? G : 128)) * Q> {
    __device__ __forceinline__ static void run(const ChunkRegs<Q, G> &, const float (&)[128 / (G < 128 ? G : 128)],
                                               uint32_t (&)[4], float &) {}
};

#define HLQ_GEMV_WAVES 4
#define HLQ_GEMV_TABLE_BYTES 2048   // 32 tables x 16 entries x fp32, per wavefront

// Register budget: two chunks of planes and scales are live at once; with many planes and many
// small quant groups that needs more than the 128 VGPRs four wavefronts per SIMD leave each.
template <int Q, int G>
constexpr int gemv_min_waves() { return Q * (G < 128 ? 128 / G : 1) <= 6 ? 4 : 2; }

template <int Q, int G>
__global__ void __launch_bounds__(64 * HLQ_GEMV_WAVES) __attribute__((amdgpu_waves_per_eu(gemv_min_waves<Q, G>(), 8)))
hlq_gemv_kernel(const GemvBatch b)
{
    using Regs = ChunkRegs<Q, G>;
    constexpr int GS = Regs::GS, SEG = Regs::SEG;
    constexpr int TPS = GS / 4;          // tables per segment
    // LDS (dynamic segment only): [waves][32 tables][16] fp32 | reduction scratch
    extern __shared__ __attribute__((aligned(256))) float lds[];
    float *red = lds + HLQ_GEMV_WAVES * (HLQ_GEMV_TABLE_BYTES / 4);   // [waves-1][64]

    // ---- which problem, which column tile, which K slice --------------------------------------
    int pi = 0;
    for (int i = 1; i < b.count; ++i)
        if ((int)blockIdx.x >= b.p[i].blk_begin) pi = i;
    const GemvProb &P = b.p[pi];
    const int local = (int)blockIdx.x - P.blk_begin;
    const int tile = local / P.nslices, slice = local % P.nslices;

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int tw = hlq_tile_width(tile, P.N);
    const bool col_ok = lane < tw;
    const int lane_c = col_ok ? lane : tw - 1;   // clamped: loads stay in bounds, results of
    const int n = tile * HLQ_TILE_N + lane;      // invalid lanes are dropped
    // this wavefront's run of chunks: the slice is cut into HLQ_GEMV_WAVES near-equal parts
    const int sbeg = slice * P.cps;
    const int send = min(sbeg + P.cps, P.nchunks);
    const int len = send - sbeg;
    const int cbeg = sbeg + (len * wave) / HLQ_GEMV_WAVES;
    const int cend = sbeg + (len * (wave + 1)) / HLQ_GEMV_WAVES;
    const char *tile_base = P.packed + (size_t)tile * HLQ_TILE_N * P.col_bytes;

    // table-build role of this lane: entries 8h .. 8h+7 of table t of the current chunk
    const int bt = lane >> 1, bh = lane & 1;
    float *Tw = lds + wave * (HLQ_GEMV_TABLE_BYTES / 4);
    // LDS byte address of this wavefront's tables, a multiple of 256
    const uint32_t tbase = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) float *)Tw;
    uint32_t ad[4] = {tbase, tbase, tbase, tbase};

    auto load_chunk = [&](int c, Regs &R) {
        const char *rec = tile_base + (size_t)tw * ((size_t)c * Q * 16 + (size_t)hlq_groups_before(c, G) * (Q + 1) * 2);
#pragma unroll
        for (int j = 0; j < Q; ++j) {
            const uint4 v = ((const uint4 *)rec)[j * tw + lane_c];
            R.w[j][0] = v.x; R.w[j][1] = v.y; R.w[j][2] = v.z; R.w[j][3] = v.w;
        }
        const char *mrec = rec;
        if (G > 128) {   // the group's meta sits in the record of its first (even) chunk
            const int c0 = c & ~1;
            mrec = tile_base + (size_t)tw * ((size_t)c0 * Q * 16 + (size_t)hlq_groups_before(c0, G) * (Q + 1) * 2);
        }
        const uint16_t *m = (const uint16_t *)(mrec + (size_t)tw * Q * 16);
#pragma unroll
        for (int sg = 0; sg < SEG; ++sg)
#pragma unroll
            for (int r = 0; r <= Q; ++r) R.mt[sg][r] = m[(sg * (Q + 1) + r) * tw + lane_c];
        R.x = *(const uint2 *)(P.x + (size_t)c * 128 + 4 * bt);
    };

    float acc = 0.f;
    auto step = [&](const Regs &R) {
        // build: entries 8h .. 8h+7 of table bt;  entry i = sum_r bit_r(i) x_r
        const float x0 = h2f((uint16_t)(R.x.x & 0xffffu)), x1 = h2f((uint16_t)(R.x.x >> 16));
        const float x2 = h2f((uint16_t)(R.x.y & 0xffffu)), x3 = h2f((uint16_t)(R.x.y >> 16));
        const float e0 = bh ? x3 : 0.f;
        const float e1 = e0 + x0, e2 = e0 + x1, e3 = e1 + x1;
        float4 *dst = (float4 *)(Tw + bt * 16 + bh * 8);
        dst[0] = make_float4(e0, e1, e2, e3);
        dst[1] = make_float4(e0 + x2, e1 + x2, e2 + x2, e3 + x2);
        // sums of the segments' activations (both lanes of a table hold the table's total)
        float tot = (x0 + x1) + (x2 + x3);
#pragma unroll
        for (int off = 2; off < 2 * TPS; off <<= 1) tot += __shfl_xor(tot, off);
        float xs[SEG];
#pragma unroll
        for (int sg = 0; sg < SEG; ++sg)
            xs[sg] = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, tot), sg * TPS * 2));
        Consume<Q, G>::run(R, xs, ad, acc);
    };

    // ---- chunk loop: two register sets, loads of chunk c+1 in flight while c is consumed ----------
    Regs RA, RB;
    if (cbeg < cend) load_chunk(cbeg, RA);
    if (cbeg + 1 < cend) load_chunk(cbeg + 1, RB);
    for (int c = cbeg; c < cend; c += 2) {
        step(RA);
        if (c + 2 < cend) load_chunk(c + 2, RA);
        if (c + 1 < cend) {
            step(RB);
            if (c + 3 < cend) load_chunk(c + 3, RB);
        }
    }

    // ---- add the four wavefronts' K ranges ------------------------------------------------------------
    if (wave > 0) red[(wave - 1) * 64 + lane] = acc;
    __syncthreads();
    if (wave > 0) return;
#pragma unroll
    for (int w2 = 1; w2 < HLQ_GEMV_WAVES; ++w2) acc += red[(w2 - 1) * 64 + lane];

    if (P.nslices == 1) {
        if (col_ok) store_out(P.y, n, acc, b.out_f32);
        return;
    }
    // ---- split-K across workgroups -----------------------------------------------------------------------
    // Partial sums and the counter live at device scope: the store below writes through the
    // XCD-local L2, the wavefront waits for its acknowledgement, and only then is the arrival
    // counted.  The last workgroup reads the partials with device-scope loads, which bypass its
    // own L2.  No cache-wide write-back or invalidate (as a device-scope fence would issue) is
    // needed, and none is used: it costs tens of microseconds per launch on this part.
    if (col_ok)
        __hip_atomic_store(&P.part[(size_t)slice * P.N + n], acc, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    int old = 0;
    if (lane == 0) old = __hip_atomic_fetch_add(&P.cnt[tile], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    old = __builtin_amdgcn_readfirstlane(old);
    if (old != P.nslices - 1) return;
    if (col_ok) {
        float a = 0.f;
        int sl = 0;
        for (; sl + 4 <= P.nslices; sl += 4) {   // four independent loads in flight, added in slice order
            const float v0 = __hip_atomic_load(&P.part[(size_t)(sl + 0) * P.N + n], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const float v1 = __hip_atomic_load(&P.part[(size_t)(sl + 1) * P.N + n], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const float v2 = __hip_atomic_load(&P.part[(size_t)(sl + 2) * P.N + n], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const float v3 = __hip_atomic_load(&P.part[(size_t)(sl + 3) * P.N + n], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            a = (((a + v0) + v1) + v2) + v3;
        }
        for (; sl < P.nslices; ++sl)
            a += __hip_atomic_load(&P.part[(size_t)sl * P.N + n], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        store_out(P.y, n, a, b.out_f32);
    }
    if (lane == 0) __hip_atomic_store(&P.cnt[tile], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__global__ void __launch_bounds__(256) hlq_ws_init_kernel(int *p, int n)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < n) p[i] = 0;
}

constexpr size_t gemv_lds_bytes() { return HLQ_GEMV_WAVES * HLQ_GEMV_TABLE_BYTES + (HLQ_GEMV_WAVES - 1) * 64 * 4; }

template <int Q>
hlq_status launch_q(int G, const GemvBatch &b, unsigned nblocks, hipStream_t st)
{
    const dim3 blk(64 * HLQ_GEMV_WAVES);
    switch (G) {
    case 32: hlq_gemv_kernel<Q, 32><<<nblocks, blk, gemv_lds_bytes(), st>>>(b); return HLQ_OK;
    case 64: hlq_gemv_kernel<Q, 64><<<nblocks, blk, gemv_lds_bytes(), st>>>(b); return HLQ_OK;
    case 128: hlq_gemv_kernel<Q, 128><<<nblocks, blk, gemv_lds_bytes(), st>>>(b); return HLQ_OK;
    case 256: hlq_gemv_kernel<Q, 256><<<nblocks, blk, gemv_lds_bytes(), st>>>(b); return HLQ_OK;
    }
    return HLQ_ERR_UNSUPPORTED;
}

int env_int(const char *name, int dflt)
{
    const char *v = getenv(name);
    return v && *v ? atoi(v) : dflt;
}

// Chunks per workgroup (= per K slice) for a launch whose problems hold `units` (tile, chunk)
// pairs in total: aim at a few workgroups per CU; a workgroup takes at least one chunk per
// wavefront, and slice boundaries stay even (with G = 256 a group spans two chunks).
int plan_cps(long units)
{
    static const int target_wgs = env_int("HLQ_TARGET_WGS", 1536);
    long cps = units / target_wgs;
    if (cps < HLQ_GEMV_WAVES) cps = HLQ_GEMV_WAVES;
    return (int)((cps + 1) & ~1L);
}

int slices_for(const HlqDims &dm, int cps) { return (dm.nchunks + cps - 1) / cps; }

} // namespace

size_t hlq_gemv_partial_bytes(const HlqDims &dm)
{
    // A launch with more problems only raises chunks-per-slice, so the slice count of the
    // single-problem plan bounds what any batch containing this problem uses.
    const long units = (long)dm.ntiles * dm.nchunks;
    const int ns = slices_for(dm, plan_cps(units));
    return ns > 1 ? (size_t)ns * (size_t)dm.N * sizeof(float) : 0;
}

hlq_status hlq_launch_ws_init(void *ws, size_t bytes, hipStream_t st)
{
    if (bytes < HLQ_WS_COUNTER_BYTES) return HLQ_ERR_BUFFER_TOO_SMALL;
    const int n = HLQ_WS_COUNTER_BYTES / 4;
    hlq_ws_init_kernel<<<(n + 255) / 256, 256, 0, st>>>((int *)ws, n);
    return hlq_hip_status(hipGetLastError());
}

hlq_status hlq_launch_gemv_batch(int count, const HlqGemvItem *items, hlq_out_dtype out, void *ws,
                                 hipStream_t st)
{
    if (count < 1 || count > HLQ_MAX_BATCH) return HLQ_ERR_UNSUPPORTED;
    long units = 0;
    for (int i = 0; i < count; ++i) units += (long)items[i].dm.ntiles * items[i].dm.nchunks;
    const int cps = plan_cps(units);

    GemvBatch b;
    b.count = count;
    b.out_f32 = out == HLQ_OUT_F32;
    int *cnt = (int *)ws;
    float *part = (float *)((char *)ws + HLQ_WS_COUNTER_BYTES);
    long blk = 0;
    long cnt_used = 0;
    for (int i = 0; i < count; ++i) {
        const HlqDims &dm = items[i].dm;
        GemvProb &p = b.p[i];
        p.packed = (const char *)items[i].packed;
        p.x = items[i].x;
        p.y = items[i].y;
        p.col_bytes = dm.col_bytes;
        p.N = dm.N;
        p.nchunks = dm.nchunks;
        p.ntiles = dm.ntiles;
        p.nslices = slices_for(dm, cps);
        p.cps = ((dm.nchunks + p.nslices - 1) / p.nslices + 1) & ~1;   // even split, even boundaries
        p.blk_begin = (int)blk;
        p.cnt = cnt + cnt_used;
        p.part = part;
        blk += (long)p.ntiles * p.nslices;
        if (p.nslices > 1) {
            cnt_used += p.ntiles;
            part += (size_t)p.nslices * dm.N;
        }
    }
    for (int i = count; i < HLQ_MAX_BATCH; ++i) b.p[i] = b.p[0];
    if (cnt_used > HLQ_WS_COUNTER_BYTES / 4 || blk > 0x7fffffffL) return HLQ_ERR_UNSUPPORTED;

    const int q = items[0].dm.q, G = items[0].dm.G;
    hlq_status s;
    switch (q) {
    case 1: s = launch_q<1>(G, b, (unsigned)blk, st); break;
    case 2: s = launch_q<2>(G, b, (unsigned)blk, st); break;
    case 3: s = launch_q<3>(G, b, (unsigned)blk, st); break;
    case 4: s = launch_q<4>(G, b, (unsigned)blk, st); break;
    default: return HLQ_ERR_UNSUPPORTED;
    }
    if (s != HLQ_OK) return s;
    return hlq_hip_status(hipGetLastError());
}
