// hlq_lut_gemv, table-lookup formulation: M = 1 bit-serial LUT GEMV (Sec. 2 "Bit-Serial LUT-Based
// GEMM", App. B), one launch for one or several independent GEMVs; plus the host side (launch
// plans, grouped launches) of both GEMV formulations -- the matrix-core kernel is in hlq_gemv_mx.hip.
//
// Work split.  The unit of work is a wavefront: it owns TN adjacent column tiles (64 columns
// each, lane <-> column) and a run of consecutive chunks (128 k each), i.e. TN contiguous byte
// streams of the packed blob.  Per chunk it
//
//   build    makes its OWN 32 tables in LDS (T[t][i] = sum_r bit_r(i) x_r over the four even or
//            four odd activations of one 8-k window, App. B; fp32 entries): each lane loads its
//            8-k window (quad of lanes <-> window), takes the even or the odd four and stores
//            entries 0..7 or 8..15 of that table with two 128-bit LDS writes; the per-quant-group
//            activation sums come from a DPP reduction of exact fp32 dot products;
//   consume  per plane and 4-bit slice one LDS lookup + one fp32 add; per (plane, quant group)
//            one FMA with s_j; per quant group one FMA  z * sum(x)       (Eq. 3 by linearity).
//
// All lanes of the wavefront index the same 16-entry table at the same time: its entries lie in
// different LDS banks and equal addresses broadcast, so lookups are conflict-free by
// construction.  Because tables are private to the wavefront and LDS operations of one
// wavefront execute in order, the chunk loop has no barrier at all; the weight loads of the next
// NBUF-1 chunks are in flight while a chunk is consumed (NBUF register sets).
//
// The W wavefronts of a workgroup take W consecutive K ranges of the SAME tiles and add their
// results through LDS.  If K is also split across workgroups ("slices"), each workgroup writes
// its partial sums to the workspace and bumps an arrival counter; the last one to arrive adds
// the partials in slice order, so the result does not depend on arrival order.
#include <stdlib.h>

#include <atomic>

#include "hlq_gemv_common.h"

namespace {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));

// v + (v moved across lanes by DPP control CTRL), rows outside ROWMASK unchanged
template <int CTRL, int ROWMASK = 0xf>
__device__ __forceinline__ float add_dpp(float v)
{
    const int moved = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, ROWMASK, 0xf, false);
    return v + __builtin_bit_cast(float, moved);
}

__device__ __forceinline__ float lane_value(float v, int lane)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), lane));
}

template <int Q, int G, int TN>
struct ChunkRegs {
    static constexpr int GS = G < 128 ? G : 128;   // k covered by one scale inside a chunk
    static constexpr int SEG = 128 / GS;           // scale segments per chunk
    uint32_t w[TN][Q][4];
    uint16_t mt[TN][SEG][Q + 1];
    uint4 x;                                       // this lane's 8-k activation window (table build)
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
// (fp16 entries fetched pairwise into the halves of one register would save adds, but on this
// part 16-bit LDS loads clear the other half of their destination, so the pairing is lost.)
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

// All lookups of one chunk, then scales and zeros: compile-time recursion over (tile tn,
// segment sg, plane j) so that every LDS offset is an immediate.  xs[sg] = sum of the
// segment's activations.
template <int Q, int G, int TN, int I = 0>
struct Consume {
    using Regs = ChunkRegs<Q, G, TN>;
    static constexpr int SEG = Regs::SEG, WPS = Regs::GS / 32;
    static constexpr int tn = I / (SEG * Q), sg = (I / Q) % SEG, j = I % Q;
    __device__ __forceinline__ static void run(const Regs &R, const float (&xs)[SEG], uint32_t (&ad)[4],
                                               float (&acc)[TN])
    {
        uint32_t w[WPS];
#pragma unroll
        for (int d = 0; d < WPS; ++d) w[d] = R.w[tn][j][sg * WPS + d];
        float p0 = 0.f, p1 = 0.f;
        lookup_words<sg * WPS * 8 * 64>(w, ad, p0, p1);
        acc[tn] += h2f(R.mt[tn][sg][j]) * (p0 + p1);
        if (j == Q - 1) acc[tn] += h2f(R.mt[tn][sg][Q]) * xs[sg];
        Consume<Q, G, TN, I + 1>::run(R, xs, ad, acc);
    }
};
template <int Q, int G, int TN>
struct Consume<Q, G, TN, TN *(128 / (G < 128 ? G : 128)) * Q> {
    __device__ __forceinline__ static void run(const ChunkRegs<Q, G, TN> &, const float (&)[128 / (G < 128 ? G : 128)],
                                               uint32_t (&)[4], float (&)[TN]) {}
};

#ifndef HLQ_DEBUG_MODE
#define HLQ_DEBUG_MODE 0   // 1: loads only (no lookups), 2: lookups only (no reloads) -- timing experiments
#endif
#define HLQ_GEMV_TABLE_BYTES 2048   // 32 tables x 16 entries x fp32, per wavefront

// Register budget: two chunks of planes and scales are live at once.  A 1024-lane workgroup
// leaves 128 VGPRs per lane; the heaviest shapes (many planes and many small quant groups)
// need more and are limited to 512 lanes (8 wavefronts) per workgroup.
constexpr int gemv_weight(int Q, int G, int TN) { return TN * Q * (G < 128 ? 128 / G : 1); }
constexpr int gemv_max_threads(int Q, int G, int TN) { return gemv_weight(Q, G, TN) <= 12 ? 1024 : 512; }
constexpr bool gemv_two_tiles_ok(int Q, int G) { return gemv_weight(Q, G, 2) <= 6; }
// register sets (chunks in flight + 1): deeper where a set is small
constexpr int gemv_nbuf(int Q, int G, int TN) { return gemv_weight(Q, G, TN) <= 2 ? 4 : gemv_weight(Q, G, TN) <= 4 ? 3 : 2; }

template <int Q, int G, int TN>
__global__ void __launch_bounds__(gemv_max_threads(Q, G, TN))
hlq_gemv_kernel(const int4v bb_lo, const int4v bb_hi, const int out_f32_flag, const GemvProbs probs)
{
    struct { int out_f32; } b = {out_f32_flag};
    using Regs = ChunkRegs<Q, G, TN>;
    constexpr int GS = Regs::GS, SEG = Regs::SEG;
    constexpr int NBUF = gemv_nbuf(Q, G, TN);
    const int W = (int)(blockDim.x >> 6);   // wavefronts per workgroup
    // LDS (dynamic segment only): [W][32 tables][16] fp32 | reduction scratch [W-1][TN][64] fp32
    extern __shared__ __attribute__((aligned(256))) float lds[];
    float *red = lds + W * (HLQ_GEMV_TABLE_BYTES / 4);

    // ---- which problem, which column tile group, which K slice ---------------------------------
    const GemvProb P = probs.p[gemv_problem_of(bb_lo, bb_hi, (int)blockIdx.x)];   // a copy: one burst of scalar loads
    int tg, slice;
    gemv_split_block(P, (int)blockIdx.x - P.blk_begin, tg, slice);

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    // this wavefront's run of chunks: the slice is cut into W near-equal parts
    // (the host plans every slice to start inside K; the clamp keeps every address inside the tile and x)
    const int sbeg = min(slice * P.cps, P.nchunks - 1);
    const int send = min(sbeg + P.cps, P.nchunks);
    const int len = send - sbeg;
    const int cbeg = sbeg + (len * wave) / W;
    const int cend = sbeg + (len * (wave + 1)) / W;

    // per tile: width, validity, clamped lane (loads stay in bounds; results of invalid lanes and
    // tiles are dropped), stream base
    int tw[TN], lane_c[TN];
    bool col_ok[TN];
    const char *tile_base[TN];
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) {
        const int tile = tg * TN + tn;
        const int tile_c = tile < P.ntiles ? tile : P.ntiles - 1;
        tw[tn] = hlq_tile_width(tile_c, P.N);
        col_ok[tn] = tile < P.ntiles && lane < tw[tn];
        lane_c[tn] = lane < tw[tn] ? lane : tw[tn] - 1;
        tile_base[tn] = P.packed + (size_t)tile_c * HLQ_TILE_N * P.col_bytes;
    }

    // table-build role of this lane: 8-k window bw of the chunk, parity bp (even / odd k of the
    // window, i.e. the table of word bw/4, 4-bit slice (bw & 3) + 4*bp), entries 8*bh .. 8*bh+7
    const int bw = lane >> 2, bp = (lane >> 1) & 1, bh = lane & 1;
    const int bt = 8 * (bw >> 2) + (bw & 3) + 4 * bp;
    char *Tw = (char *)lds + wave * HLQ_GEMV_TABLE_BYTES;
    // LDS byte address of this wavefront's tables, a multiple of 256
    const uint32_t tbase = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)Tw;
    uint32_t ad[4] = {tbase, tbase, tbase, tbase};

    auto load_chunk = [&](int c, Regs &R) {
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) {
            const int w_ = tw[tn];
            const char *rec = tile_base[tn] + hlq_rec_in_tile(w_, c, Q, G);
#pragma unroll
            for (int j = 0; j < Q; ++j) {
                // default cache policy: non-temporal loads, which help the matrix-core kernel, cost this one 2 us per layer
                const int4v v = *((const int4v *)rec + (j * w_ + lane_c[tn]));
                R.w[tn][j][0] = v.x; R.w[tn][j][1] = v.y; R.w[tn][j][2] = v.z; R.w[tn][j][3] = v.w;
            }
            const char *mrec = rec;
            if (G > 128) {   // the group's meta sits in the record of its first (even) chunk
                const int c0 = c & ~1;
                mrec = tile_base[tn] + hlq_rec_in_tile(w_, c0, Q, G);
            }
            const uint16_t *m = (const uint16_t *)(mrec + (size_t)w_ * Q * 16);
#pragma unroll
            for (int sg = 0; sg < SEG; ++sg)
#pragma unroll
                for (int r = 0; r <= Q; ++r) R.mt[tn][sg][r] = m[(sg * (Q + 1) + r) * w_ + lane_c[tn]];
        }
        R.x = *(const uint4 *)(P.x + (size_t)c * 128 + 8 * bw);
    };

    float acc[TN];
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) acc[tn] = 0.f;

    auto step = [&](const Regs &R) {
        // build: entries 8h .. 8h+7 of table bt;  entry i = sum_r bit_r(i) x_r  (fp32), where
        // x_r is the r-th even (bp = 0) or odd (bp = 1) activation of the window
        const uint32_t xd[4] = {R.x.x, R.x.y, R.x.z, R.x.w};
        float xv[4];
#pragma unroll
        for (int r = 0; r < 4; ++r)
            xv[r] = (float)__builtin_bit_cast(_Float16, (uint16_t)(xd[r] >> (16 * bp)));
        const float e0 = bh ? xv[3] : 0.f;
        const float e1 = e0 + xv[0], e2 = e0 + xv[1], e3 = e1 + xv[1];
        float4 *dst = (float4 *)(Tw + bt * 64 + bh * 32);
        dst[0] = make_float4(e0, e1, e2, e3);
        dst[1] = make_float4(e0 + xv[2], e1 + xv[2], e2 + xv[2], e3 + xv[2]);
        // sums of the segments' activations: exact fp32 dot products of the window with (1, 1)
        // (the four lanes of a quad share a window), then a DPP reduction over the four windows
        // (32 k) of a 16-lane row and, for larger groups, over rows
        const half2_t ones = {(_Float16)1.0f, (_Float16)1.0f};
        float tot = 0.f;
#pragma unroll
        for (int r = 0; r < 4; ++r) tot = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, xd[r]), ones, tot, false);
        tot = add_dpp<0x124>(tot);   // row_ror:4
        tot = add_dpp<0x128>(tot);   // row_ror:8   -> every lane holds its row's 32-k sum
        float xs[SEG];
        if (GS == 32) {
#pragma unroll
            for (int sg = 0; sg < SEG; ++sg) xs[sg] = lane_value(tot, 16 * sg);
        } else if (GS == 64) {
            tot = add_dpp<0x142, 0xa>(tot);   // row_bcast15: rows 1, 3 += rows 0, 2
            xs[0] = lane_value(tot, 31);
            xs[SEG - 1] = lane_value(tot, 63);
        } else {
            tot = add_dpp<0x142, 0xa>(tot);
            tot = add_dpp<0x143, 0xc>(tot);   // row_bcast31: rows 2, 3 += row 1
            xs[0] = lane_value(tot, 63);
        }
        if (HLQ_DEBUG_MODE == 1) {
#pragma unroll
            for (int tn = 0; tn < TN; ++tn) {
                uint32_t m = 0;
#pragma unroll
                for (int j = 0; j < Q; ++j) m ^= R.w[tn][j][0] ^ R.w[tn][j][1] ^ R.w[tn][j][2] ^ R.w[tn][j][3];
                acc[tn] += (float)m * h2f(R.mt[tn][0][0]) + xs[0];
            }
        } else {
            Consume<Q, G, TN>::run(R, xs, ad, acc);
        }
    };

    // ---- chunk loop: NBUF register sets, loads of the next NBUF-1 chunks in flight ----------------------
    // A register set is reloaded only while the run has a further chunk for it (the branch sits between
    // steps, not inside one).
    if (cbeg < cend) {
        Regs R[NBUF];
#pragma unroll
        for (int i = 0; i < NBUF; ++i) load_chunk(min(cbeg + i, cend - 1), R[i]);
        for (int c = cbeg; c < cend; c += NBUF) {
#pragma unroll
            for (int i = 0; i < NBUF; ++i) {
                if (c + i < cend) step(R[i]);
                if (HLQ_DEBUG_MODE != 2 && c + i + NBUF < cend) load_chunk(c + i + NBUF, R[i]);
            }
        }
    }

    // ---- add the W wavefronts' K ranges ------------------------------------------------------------------
    if (wave > 0) {
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) red[((wave - 1) * TN + tn) * 64 + lane] = acc[tn];
    }
    __syncthreads();
    if (wave > 0) return;
    for (int w2 = 1; w2 < W; ++w2) {
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) acc[tn] += red[((w2 - 1) * TN + tn) * 64 + lane];
    }

    if (P.nslices == 1) {
#pragma unroll
        for (int tn = 0; tn < TN; ++tn)
            if (col_ok[tn]) store_out(P.y, (size_t)(tg * TN + tn) * HLQ_TILE_N + lane, acc[tn], b.out_f32);
        return;
    }
    // ---- split-K across workgroups -----------------------------------------------------------------------
    // Partial sums and the counter live at device scope: the stores below write through the
    // XCD-local L2, the wavefront waits for their acknowledgement, and only then is the arrival
    // counted.  The last workgroup reads the partials with device-scope loads, which bypass its
    // own L2.  No cache-wide write-back or invalidate (as a device-scope fence would issue) is
    // needed, and none is used: it costs tens of microseconds per launch on this part.
#pragma unroll
    for (int tn = 0; tn < TN; ++tn)
        if (col_ok[tn])
            __hip_atomic_store(&P.part[(size_t)slice * P.N + (size_t)(tg * TN + tn) * HLQ_TILE_N + lane], acc[tn],
                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    int old = 0;
    if (lane == 0) old = __hip_atomic_fetch_add(&P.cnt[tg], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    old = __builtin_amdgcn_readfirstlane(old);
    if (old != P.nslices - 1) return;
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) {
        if (!col_ok[tn]) continue;
        const size_t n = (size_t)(tg * TN + tn) * HLQ_TILE_N + lane;
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
    if (lane == 0) __hip_atomic_store(&P.cnt[tg], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__global__ void __launch_bounds__(256) hlq_ws_init_kernel(int *p, int n)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < n) p[i] = 0;
}

size_t gemv_lds_bytes(int W, int TN) { return (size_t)W * HLQ_GEMV_TABLE_BYTES + (size_t)(W - 1) * TN * 64 * 4; }

template <int Q, int G>
void launch_qg(const GemvBatch &b, unsigned nblocks, int W, int TN, hipStream_t st)
{
    const dim3 blk(64 * W);
    const GemvKernelArgs a = gemv_kernel_args(b);
    if (TN == 2) {
        if constexpr (gemv_two_tiles_ok(Q, G))
            hlq_gemv_kernel<Q, G, 2><<<nblocks, blk, gemv_lds_bytes(W, 2), st>>>(a.lo, a.hi, a.out_f32, a.probs);
    } else {
        hlq_gemv_kernel<Q, G, 1><<<nblocks, blk, gemv_lds_bytes(W, 1), st>>>(a.lo, a.hi, a.out_f32, a.probs);
    }
}

template <int Q>
hlq_status launch_q(int G, const GemvBatch &b, unsigned nblocks, int W, int TN, hipStream_t st)
{
    switch (G) {
    case 32: launch_qg<Q, 32>(b, nblocks, W, TN, st); return HLQ_OK;
    case 64: launch_qg<Q, 64>(b, nblocks, W, TN, st); return HLQ_OK;
    case 128: launch_qg<Q, 128>(b, nblocks, W, TN, st); return HLQ_OK;
    case 256: launch_qg<Q, 256>(b, nblocks, W, TN, st); return HLQ_OK;
    }
    return HLQ_ERR_UNSUPPORTED;
}

int env_int(const char *name, int dflt)
{
    const char *v = getenv(name);
    return v && *v ? atoi(v) : dflt;
}

// Launch shape for a batch holding `units` (tile, chunk) pairs in total.
struct GemvPlan {
    int TN;    // column tiles per wavefront (1 or 2)
    int W;     // wavefronts per workgroup (K ranges added through LDS)
    int cpw;   // target chunks per wavefront; a slice is W * cpw chunks (rounded to even)
};

// process-wide overrides set by hlq_set_gemv_plan (0 = automatic).  Atomic, so that a launch on one
// thread reads a whole value while another thread sets a knob; a launch that overlaps a change of the
// three plan values may still see some old and some new ones (each combination is a valid plan).
std::atomic<int> g_plan_tn{0}, g_plan_w{0}, g_plan_cpw{0};
// formulation: 0 automatic, 1 table lookup, 2 matrix core (hlq_set_gemv_path)
std::atomic<int> g_gemv_path{0};

bool use_mx()
{
    static const int env_path = env_int("HLQ_GEMV_PATH", 0);
    const int knob = g_gemv_path.load(std::memory_order_relaxed);
    const int path = knob ? knob : env_path;
    return path == 0 || path == 2;   // automatic: the matrix-core kernel is the faster one on every measured shape
}

// table-storage variant of the lookup formulation (hlq_gemv_variants.hip): -1 = none (the hand-scheduled kernel)
int table_variant()
{
    const int knob = g_gemv_path.load(std::memory_order_relaxed);
    return knob >= 3 ? knob - 3 : -1;
}

GemvPlan plan_gemv(long units)
{
    static const int env_tn = env_int("HLQ_GEMV_TN", 0);
    static const int env_w = env_int("HLQ_GEMV_W", 0);
    static const int env_cpw = env_int("HLQ_GEMV_CPW", 0);
    GemvPlan pl;
    // Measured on MI355X (sweeps over TN x W x cpw on the 8B / 70B shapes): one tile per
    // wavefront, four wavefronts per workgroup; short runs for launches that would otherwise
    // not fill the wavefront slots, longer runs (fewer split-K partials) for large ones.
    pl.TN = 1;
    pl.W = 4;
    pl.cpw = units >= 65536 ? 8 : 4;
    if (use_mx()) {
        // matrix-core kernel (sweeps on the same shapes): short runs on many wavefronts while the
        // launch is small, longer runs once the chip is full
        pl.W = 8;
        pl.cpw = units < 12000 ? 4 : 7;
    }
    if (env_tn) pl.TN = env_tn;
    if (env_w) pl.W = env_w;
    if (env_cpw) pl.cpw = env_cpw;
    if (const int v = g_plan_tn.load(std::memory_order_relaxed)) pl.TN = v;
    if (const int v = g_plan_w.load(std::memory_order_relaxed)) pl.W = v;
    if (const int v = g_plan_cpw.load(std::memory_order_relaxed)) pl.cpw = v;
    return pl;
}

// chunks per K slice: a multiple of two (with G = 256 a group spans two chunks)
int slice_chunks(const GemvPlan &pl) { return (pl.W * pl.cpw + 1) & ~1; }
int slices_for(const HlqDims &dm, int cps) { return (dm.nchunks + cps - 1) / cps; }

// Work split of one problem for the matrix-core kernel: runs of about cpw chunks for every problem
// of a launch (wavefronts with longer runs would finish alone, with the memory system half idle):
// K is cut inside the workgroup first (kw wavefronts per tile), then across workgroups.
void plan_mx_problem(const HlqDims &dm, int W, int cpw, GemvProb &p)
{
    p.kw = 1;
    while (p.kw * 2 <= W && dm.nchunks / (p.kw * 2) >= cpw) p.kw *= 2;
    int per_slice = p.kw * cpw;
    if (per_slice < 4) per_slice = 4;
    p.nslices = (dm.nchunks + per_slice / 2) / per_slice;   // nearest
    if (p.nslices < 1) p.nslices = 1;
    const int tiles_per_wg = W / p.kw;
    p.ntg = (dm.ntiles + tiles_per_wg - 1) / tiles_per_wg;
    p.cps = ((dm.nchunks + p.nslices - 1) / p.nslices + 1) & ~1;   // even split, even boundaries
    // rounding the slice length up can leave trailing slices without a chunk: count the slices again, so
    // that every slice starts inside K ((nslices - 1) * cps < nchunks)
    p.nslices = (dm.nchunks + p.cps - 1) / p.cps;
}

} // namespace

hlq_status hlq_gemv_path_override(int path)
{
    if (path < 0 || path > 6) return HLQ_ERR_UNSUPPORTED;
    g_gemv_path = path;
    return HLQ_OK;
}

hlq_status hlq_gemv_plan_override(int tn, int w, int cpw)
{
    if (tn < 0 || tn > 2 || w < 0 || w > 16 || cpw < 0) return HLQ_ERR_UNSUPPORTED;
    g_plan_tn = tn;
    g_plan_w = w;
    g_plan_cpw = cpw;
    return HLQ_OK;
}

size_t hlq_gemv_partial_bytes(const HlqDims &dm)
{
    // Upper bound over every plan: slices are never shorter than 4 chunks.
    const int ns = (dm.nchunks + 3) / 4;
    return ns > 1 ? (size_t)ns * (size_t)dm.N * sizeof(float) : 0;
}

hlq_status hlq_launch_ws_init(void *ws, size_t bytes, hipStream_t st)
{
    hlq_clear_stale_error();
    if (bytes < HLQ_WS_COUNTER_BYTES) return HLQ_ERR_BUFFER_TOO_SMALL;
    const int n = HLQ_WS_COUNTER_BYTES / 4;
    hlq_ws_init_kernel<<<(n + 255) / 256, 256, 0, st>>>((int *)ws, n);
    return hlq_hip_status(hipGetLastError());
}

// The work split of a grouped launch: everything the host decides (formulation, workgroup shape, K
// slices and runs per problem, block ranges, workspace carving).  Touches no device memory, so the
// plan can also be inspected without a GPU (hlq_gemv_plan_query).
struct GemvLaunchShape {
    bool mx;
    bool rowsk;       // the many-rows kernel (hlq_gemm_rows.hip) instead of the few-rows instantiation of the GEMV kernel
    int W, TN, rows;
    long nblocks;
    size_t ws_used;   // bytes of the workspace this plan touches: the counter block and its partial sums
};

static hlq_status plan_gemv_batch(int count, const HlqGemvItem *items, hlq_out_dtype out, void *ws, GemvBatch &b,
                                  GemvLaunchShape &ls)
{
    if (count < 1 || count > HLQ_MAX_BATCH) return HLQ_ERR_UNSUPPORTED;
    long units = 0;
    for (int i = 0; i < count; ++i) units += (long)items[i].dm.ntiles * items[i].dm.nchunks;
    GemvPlan pl = plan_gemv(units);
    const int rows = items[0].M;
    for (int i = 1; i < count; ++i)
        if (items[i].M != rows) return HLQ_ERR_UNSUPPORTED;
    if (rows < 1 || rows > hlq_gemm_mx_rows_per_pass(items[0].dm.G)) return HLQ_ERR_UNSUPPORTED;
    const bool mx = use_mx() || rows > 1;   // several activation rows exist in the matrix-core kernels only
    // more rows than one operand of the GEMV kernel holds: the many-rows kernel (terms chained through the
    // accumulator, activations converted once per workgroup), where it exists for this group size
    bool rowsk = rows > hlq_gemv_mx_rows_per_set(items[0].dm.G) && rows <= hlq_gemm_rows_max(items[0].dm.G) &&
                 rows <= hlq_gemm_mx_rows_per_pass(items[0].dm.G);
    // three or four rows (which the GEMV kernel's one row set also holds): the one-operand instantiation of the
    // many-rows kernel where its pre-pass pays
    if (!rowsk && rows >= 3 && rows <= hlq_gemm_rows_max(items[0].dm.G) &&
        (hlq_gemm_rows_all() || hlq_gemm_rows_wins_few(units, items[0].dm.q, rows)))
        rowsk = true;
    if (rowsk) {
        pl.W = 4;
        // chunks per K slice: long enough that the partial sums (rows x columns x slices) stay a small part of the
        // traffic, short enough that the launch has several workgroups per compute unit
        pl.cpw = units < 12000 ? 4 : 16;   // measured on the 8B layer at q = 4: 16 beats 8 (one round of workgroups instead of two)
        if (const int v = g_plan_cpw.load(std::memory_order_relaxed)) pl.cpw = v < 4 ? 4 : v;
    } else if (rows > 1) {
        // measured (8B shapes, q = 4, M = 2..8): short runs on few wavefronts per workgroup for narrow
        // launches, longer runs and eight wavefronts once there are enough tiles
        pl.W = units < 4096 ? 4 : 8;
        pl.cpw = units < 4096 ? 2 : units < 12000 ? 4 : 6;
        if (const int v = g_plan_w.load(std::memory_order_relaxed)) pl.W = v;
        if (const int v = g_plan_cpw.load(std::memory_order_relaxed)) pl.cpw = v;
    }
    {
        const int q0 = items[0].dm.q, G0 = items[0].dm.G;
        if (mx || !gemv_two_tiles_ok(q0, G0) || table_variant() >= 0) pl.TN = 1;
        const int maxw = mx ? hlq_gemv_mx_max_waves(q0, G0) : gemv_max_threads(q0, G0, pl.TN) / 64;
        if (pl.W > maxw) pl.W = maxw;
        if (!mx && table_variant() >= 0 && pl.W > 8) pl.W = 8;   // the plain variant kernels: up to 512 lanes
        if (rowsk) {
            pl.W = 4;
            if (const int v = g_plan_w.load(std::memory_order_relaxed)) pl.W = v >= 8 ? 8 : v >= 4 ? 4 : 2;
        }
        if (mx)   // a power of two
            while (pl.W & (pl.W - 1)) pl.W &= pl.W - 1;
    }
    if (pl.W < 1 || pl.W > 16 || (pl.TN != 1 && pl.TN != 2) || pl.cpw < 1) return HLQ_ERR_UNSUPPORTED;
    // chunks per K slice of the lookup kernel: each of its W wavefronts takes cpw chunks of one tile
    int cps = slice_chunks(pl);
    if (cps < 4) cps = 4;

    b.count = count;
    b.out_f32 = out == HLQ_OUT_F32;
    int *cnt = (int *)ws;
    float *part = (float *)((char *)ws + HLQ_WS_COUNTER_BYTES);
    long blk = 0;
    long cnt_used = 0;
    // Workgroups start in block order: problems with long K (long runs, or K split across workgroups
    // with extra trips to memory at the end) go first.
    int order[HLQ_MAX_BATCH];
    for (int i = 0; i < count; ++i) order[i] = i;
    for (int i = 1; i < count; ++i)
        for (int j = i; j > 0 && items[order[j]].dm.nchunks > items[order[j - 1]].dm.nchunks; --j) {
            const int t = order[j];
            order[j] = order[j - 1];
            order[j - 1] = t;
        }
    for (int i = 0; i < count; ++i) {
        const HlqDims &dm = items[order[i]].dm;
        GemvProb &p = b.p[i];
        p.packed = (const char *)items[order[i]].packed;
        p.x = items[order[i]].x;
        p.y = items[order[i]].y;
        p.col_bytes = dm.col_bytes;
        p.N = dm.N;
        p.nchunks = dm.nchunks;
        p.ntiles = dm.ntiles;
        p.kw = 1;
        p.M = rows;
        p.ldx = items[order[i]].ldx;
        p.ldy = items[order[i]].ldy;
        if (rowsk) {
            plan_mx_problem(dm, pl.W, pl.cpw, p);
        } else if (mx) {
            plan_mx_problem(dm, pl.W, pl.cpw, p);
        } else {
            p.ntg = (dm.ntiles + pl.TN - 1) / pl.TN;
            p.nslices = slices_for(dm, cps);
            p.cps = ((dm.nchunks + p.nslices - 1) / p.nslices + 1) & ~1;   // even split, even boundaries
            p.nslices = slices_for(dm, p.cps);
        }
        // every K slice must start inside K: the kernels form addresses from a slice's first chunk
        if (p.nslices < 1 || p.cps < 1 || (long)(p.nslices - 1) * p.cps >= dm.nchunks) return HLQ_ERR_UNSUPPORTED;
        p.kw_shift = 0;
        while ((1 << p.kw_shift) < p.kw) ++p.kw_shift;
        // exact for local * nslices < 2^32, far above any grid this library launches (checked below)
        p.slice_magic = p.nslices > 1 ? (unsigned)((0x100000000ULL + (unsigned)p.nslices - 1) / (unsigned)p.nslices) : 0u;
        if ((unsigned long long)p.ntg * p.nslices * p.nslices >= 0x100000000ULL) return HLQ_ERR_UNSUPPORTED;
        p.blk_begin = (int)blk;
        b.blk_begin[i] = (int)blk;
        p.cnt = cnt + cnt_used;
        p.part = part;
        blk += (long)p.ntg * p.nslices;
        if (p.nslices > 1) {
            cnt_used += mx ? dm.ntiles : p.ntg;
            part += (size_t)p.nslices * dm.N * rows;
        }
    }
    if (rowsk) {
        // behind all partial sums: every problem's activations in operand form, then its row exponents
        char *xt = (char *)(((uintptr_t)part + 255u) & ~(uintptr_t)255u);
        for (int i = 0; i < count; ++i) {
            const size_t nb = hlq_gemm_rows_xt_bytes(items[order[i]].dm, rows);
            b.p[i].xt = xt;
            b.p[i].xexp = (int *)(xt + nb - 256);
            xt += nb;
        }
        part = (float *)xt;
    } else {
        for (int i = 0; i < count; ++i) {
            b.p[i].xt = nullptr;
            b.p[i].xexp = nullptr;
        }
    }
    for (int i = count; i < HLQ_MAX_BATCH; ++i) {
        b.p[i] = b.p[0];
        b.blk_begin[i] = 0x7fffffff;
    }
    if (cnt_used > HLQ_WS_ARRIVAL_COUNTERS || blk > 0x7fffffffL) return HLQ_ERR_UNSUPPORTED;
    ls.mx = mx;
    ls.rowsk = rowsk;
    ls.W = pl.W;
    ls.TN = pl.TN;
    ls.rows = rows;
    ls.nblocks = blk;
    ls.ws_used = HLQ_WS_COUNTER_BYTES + (size_t)(part - (float *)((char *)ws + HLQ_WS_COUNTER_BYTES)) * sizeof(float);
    return HLQ_OK;
}

hlq_status hlq_launch_gemv_batch(int count, const HlqGemvItem *items, hlq_out_dtype out, void *ws,
                                 hipStream_t st, size_t ws_cap)
{
    hlq_clear_stale_error();
    GemvBatch b;
    GemvLaunchShape ls;
    hlq_status s = plan_gemv_batch(count, items, out, ws, b, ls);
    if (s != HLQ_OK) return s;
    if (ws_cap && ls.ws_used > ws_cap) return HLQ_ERR_BUFFER_TOO_SMALL;   // checked on the plan that is launched
    const int q = items[0].dm.q, G = items[0].dm.G;
    const unsigned blk = (unsigned)ls.nblocks;
    if (ls.rowsk) {
        s = hlq_launch_gemm_rows(b, blk, ls.W, ls.rows, q, G, st);
        if (s != HLQ_OK) return s;
        return hlq_hip_status(hipGetLastError());
    }
    if (ls.mx) {
        const int nsets = ls.rows == 1 ? 0 : ls.rows <= hlq_gemv_mx_rows_per_set(G) ? 1 : 2;
        s = hlq_launch_gemv_mx(b, blk, ls.W, nsets, ls.rows, q, G, st);
        if (s != HLQ_OK) return s;
        return hlq_hip_status(hipGetLastError());
    }
    if (table_variant() >= 0 && ls.TN == 1) {
        s = hlq_launch_gemv_variant(table_variant(), b, blk, ls.W, q, G, st);
        if (s != HLQ_OK) return s;
        return hlq_hip_status(hipGetLastError());
    }
    switch (q) {
    case 1: s = launch_q<1>(G, b, blk, ls.W, ls.TN, st); break;
    case 2: s = launch_q<2>(G, b, blk, ls.W, ls.TN, st); break;
    case 3: s = launch_q<3>(G, b, blk, ls.W, ls.TN, st); break;
    case 4: s = launch_q<4>(G, b, blk, ls.W, ls.TN, st); break;
    default: return HLQ_ERR_UNSUPPORTED;
    }
    if (s != HLQ_OK) return s;
    return hlq_hip_status(hipGetLastError());
}

// Workspace bytes the GEMV of one matrix touches with the plan it would get now (at most the bound
// hlq_workspace_bytes reports, usually far less: most plans cut K inside a workgroup only).
hlq_status hlq_gemv_ws_used(const HlqDims &dm, size_t *bytes)
{
    HlqGemvItem it;
    it.dm = dm;
    it.packed = nullptr;
    it.x = nullptr;
    it.y = nullptr;
    GemvBatch b;
    GemvLaunchShape ls;
    const hlq_status s = plan_gemv_batch(1, &it, HLQ_OUT_F16, nullptr, b, ls);
    if (s == HLQ_OK) *bytes = ls.ws_used;
    return s;
}

// The plan of a launch of `count` problems with M rows each, as hlq_launch_gemv_batch would make it now
// (current knobs).  Host arithmetic only.
hlq_status hlq_gemv_plan_describe(int count, const HlqDims *dms, int M, hlq_gemv_plan_info *out)
{
    HlqGemvItem items[HLQ_MAX_BATCH];
    if (count < 1 || count > HLQ_MAX_BATCH) return HLQ_ERR_UNSUPPORTED;
    for (int i = 0; i < count; ++i) {
        items[i].dm = dms[i];
        items[i].packed = nullptr;
        items[i].x = nullptr;
        items[i].y = nullptr;
        items[i].M = M;
        items[i].ldx = dms[i].K;
        items[i].ldy = dms[i].N;
    }
    GemvBatch b;
    GemvLaunchShape ls;
    const hlq_status s = plan_gemv_batch(count, items, HLQ_OUT_F16, nullptr, b, ls);
    if (s != HLQ_OK) return s;
    bool taken[HLQ_MAX_BATCH] = {};
    for (int i = 0; i < count; ++i) {
        // problems are planned in launch order (long K first); report them in the caller's order
        int at = -1;
        for (int k = 0; k < count && at < 0; ++k)
            if (!taken[k] && b.p[k].nchunks == dms[i].nchunks && b.p[k].N == dms[i].N && b.p[k].col_bytes == dms[i].col_bytes) at = k;
        if (at < 0) return HLQ_ERR_UNSUPPORTED;
        taken[at] = true;
        const GemvProb &p = b.p[at];
        out[i].formulation = ls.mx ? 2 : 1;
        out[i].waves_per_workgroup = ls.W;
        out[i].waves_per_tile = ls.mx ? p.kw : ls.W;
        out[i].chunks_per_slice = p.cps;
        out[i].slices = p.nslices;
        out[i].tile_groups = p.ntg;
        out[i].first_block = p.blk_begin;
        out[i].blocks = (int32_t)((long)p.ntg * p.nslices);
    }
    return HLQ_OK;
}

// Rows an MX launch can carry for group size G: two row sets of the GEMV kernel, or what the many-rows kernel holds.
int hlq_gemm_mx_rows_per_pass(int G)
{
    const int two_sets = 2 * hlq_gemv_mx_rows_per_set(G);
    const int many = hlq_gemm_rows_max(G);
    return many > two_sets ? many : two_sets;
}

// Many-rows kernel or tiled kernel for 5..16 rows (G >= 128)?  Measured on 8B / 70B layer shapes, single calls and
// grouped launches, in microseconds (many-rows against tiled).  The many-rows kernel pays per MFMA (q planes x four
// activation terms per row, twice the instructions from 9 rows on) and needs a launch large enough to spread its
// wavefronts; the tiled kernel pays for rebuilding the weights, whatever M.
//   q = 4, up to 8 rows:  2048 chunk-tiles 15.1 / 12.3,  7168: 19.3 / 23.6 and 21.6 / 27.6,  28672: 41 / 64, 8B layer 40 / 68
//   q = 4, 9..16 rows:    2048: 17.1 / 12.6,  2560 (two matrices) 18.1 / 19.6,  7168: 24.2 / 23.8 and 26.5 / 28.2,  8B layer 60 / 69
//   q = 2, up to 8 rows:  2048: 13.9 / 10.5,  7168: 16.6 / 16.4 and 19.3 / 17.9,  28672: 29 / 41
//   q = 2, 9..16 rows:    7168: 20.8 / 16.8 and 23.2 / 18.3,  28672: 43.4 / 42.5,  8B layer 47 / 49
// The same question for 3 or 4 rows, where the alternative is the few-rows instantiation of the GEMV kernel
// (which converts the activations in every wavefront and needs no pre-pass).  Measured, many-rows against few-rows:
//   8B layer (27648 chunk-tiles)  q = 4: 33.3 / 36.4 (3 rows), 33.2 / 39.5 (4 rows);  q = 3: 28.8 / 27.0, 28.7 / 30.1;
//                                 q = 2: 25.6 / 22.5, 26.0 / 26.0
//   70B layer (104448), q = 2: 66.3 / 68.3, 67.0 / 77.6;   one 4096 x 14336 (7168), q = 4: 18.5 / 13.0, 18.5 / 14.3
bool hlq_gemm_rows_wins_few(long units, int q, int rows)
{
    if (q >= 4) return units >= 20000;
    if (rows < 4) return false;
    return units >= (q == 3 ? 40000 : 60000);
}

bool hlq_gemm_rows_wins(long units, int q, int64_t M)
{
    if (M <= 8) return units >= (q >= 3 ? 4096 : 12000);
    return units >= (q >= 3 ? 2400 : 20000);
}

// Whether a grouped launch of M rows goes to the matrix-core GEMV-shaped kernels (few-rows / many-rows) rather
// than to the tiled kernel: up to one row set (four rows at G >= 128) and whatever the second row set of the
// GEMV kernel carries at G <= 64 always; 5..16 rows at G >= 128 by the rule above; hlq_set_gemm_path(4) sends all of
// them here.
bool hlq_gemm_batch_on_mx(int count, const HlqGemvItem *items, int64_t M)
{
    if (count < 1 || M < 1) return false;
    const int G = items[0].dm.G;
    if (M > hlq_gemm_mx_rows_per_pass(G)) return false;
    if (M <= hlq_gemv_mx_rows_per_set(G) || hlq_gemm_rows_max(G) == 0 || hlq_gemm_rows_all()) return true;
    long units = 0;
    for (int i = 0; i < count; ++i) units += (long)items[i].dm.ntiles * items[i].dm.nchunks;
    return hlq_gemm_rows_wins(units, items[0].dm.q, M);
}

size_t hlq_gemm_mx_partial_bytes(const HlqDims &dm, int64_t M)
{
    const int cap = hlq_gemm_mx_rows_per_pass(dm.G);
    const int64_t rows = M < cap ? M : cap;
    // slices are never shorter than 4 chunks here either; the many-rows kernel adds the operand form of the activations
    return (size_t)rows * hlq_gemv_partial_bytes(dm) + hlq_gemm_rows_xt_bytes(dm, 16) + 256;
}

// Y[M, N] = X[M, K] @ W^ for as many rows as one pass of the matrix-core GEMV kernel carries.
hlq_status hlq_launch_gemm_mx_rows(const HlqDims &dm, const void *packed, const uint16_t *X, int64_t M, int64_t ldx,
                                   void *Y, int64_t ldy, hlq_out_dtype out, void *ws, hipStream_t st)
{
    if (M < 1 || M > hlq_gemm_mx_rows_per_pass(dm.G)) return HLQ_ERR_UNSUPPORTED;
    HlqGemvItem it;
    it.dm = dm;
    it.packed = packed;
    it.x = X;
    it.y = Y;
    it.M = (int)M;
    it.ldx = (long)ldx;
    it.ldy = (long)ldy;
    return hlq_launch_gemv_batch(1, &it, out, ws, st);
}
