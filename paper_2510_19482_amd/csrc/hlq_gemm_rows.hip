// hlq_lut_gemm for a handful of rows (small-batch decode, 5 <= M <= 16, quant groups of 128 or 256):
// the bit-serial product of Sec. 2 "Bit-Serial LUT-Based GEMM" / App. B with the per-plane dot products
// on the MX matrix cores, as in hlq_gemv_mx.hip, arranged for many activation rows:
//
//   Y[m,n] = sum_groups ( sum_j s_j[g,n] * <b_j[.,n], X[m,.]>_g  +  z[g,n] * sum_g(X[m,.]) )
//
// Planes become fp4 codes by AND masks; an activation is an exact sum of four bf8 terms (each the
// running remainder cut to three significant bits).  In the GEMV kernel the four terms sit in four
// ROWS of the 16-row operand and meet again as four scaled results per (row, column, plane).  Here the
// terms lie along the ACCUMULATION: operand o holds terms [o TPO, (o + 1) TPO) of 16 / TPO activation
// rows, the NT = 4 / TPO matrix-core instructions of an item (plane j, block of 16 columns) chain
// through their accumulator, and what comes out is the finished dot product of every row -- one scale
// multiplication per (row, column, plane).  NT = 2 carries up to 8 rows, NT = 4 up to 16.  NT = 1 is the other
// end: all four terms of up to 4 rows in one operand, one matrix-core instruction per item, the four terms of a
// result in the four 16-lane groups, added by two cross-lane adds at the very end (the arrangement of the GEMV
// kernel, but with the activations converted once per call by the pre-pass instead of once per column tile).
//
// Two kernels.  hlq_rows_split_kernel runs once per call: the workgroups of a (problem, activation row) find
// the row's largest magnitude, which fixes a power-of-two scale that puts the row high in the bf8 range
// (removed again at the end), cuts every activation into its four terms and writes them to the workspace
// exactly as the matrix core wants its 8-bit operand: [chunk][operand][row][128 codes in matrix-core k
// order] -- 2 KiB per operand and chunk, rows the call does not have as zeros.  hlq_gemm_rows_kernel then
// has no activation work at all: a lane loads its 32 bytes of every operand straight into registers,
// one chunk ahead.
//
// Work split of the main kernel.  A workgroup of W wavefronts owns W / kw adjacent column tiles and one
// K slice; the kw wavefronts of a tile take consecutive runs of chunks and add their results through LDS
// at the end (as in hlq_gemv_mx.hip); nothing is shared before that, so there is no barrier in the chunk
// loop.  K slices of different workgroups meet in the workspace (partial sums, one arrival counter per
// tile, the last arriver adds in slice order).
#include "hlq_gemv_common.h"

#ifndef HLQ_ROWS_SKIP
#define HLQ_ROWS_SKIP 0    // timing experiments (wrong results), bit mask -- 1: no scale multiplications, 2: no word transpose, 4: no plane expansion
#endif
#ifndef HLQ_ROWS_DEBUG
#define HLQ_ROWS_DEBUG 0   // timing experiments -- 1: loads only (no matrix-core work), 2: no weight reloads (compute only), 3: nor operand reloads
#endif

namespace {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef unsigned short ushort2_t __attribute__((ext_vector_type(2)));
typedef int int8v __attribute__((ext_vector_type(8)));
typedef unsigned int uint2v __attribute__((ext_vector_type(2)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef uint16_t __attribute__((may_alias)) u16_alias;
typedef uint32_t __attribute__((may_alias)) u32_alias;

constexpr int rows_meta_stride(int Q) { return ((Q + 1) * 2 + 7) & ~7; }
// LDS per wavefront: scales [64][stride] | results [16][64] fp32 for the sum over the tile's kw runs
constexpr int rows_wave_lds(int Q) { return 64 * rows_meta_stride(Q) + 16 * 64 * 4; }
constexpr int rows_lds_bytes(int Q, int W) { return W * rows_wave_lds(Q); }
// bytes of one operand of one chunk in the workspace: 16 rows x 128 codes
constexpr int ROWS_OPERAND_BYTES = 16 * 128;

template <int CTRL, int ROWMASK = 0xf>
__device__ __forceinline__ uint32_t max_dpp(uint32_t v)
{
    const uint32_t moved = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, ROWMASK, 0xf, false);
    return max(v, moved);
}

// Workgroup = (activation row m = blockIdx.x, problem blockIdx.y, share blockIdx.z of the row's chunks).  Term t of row m goes to operand t / TPO,
// operand row (t % TPO) * RPO + m; a row the call does not have is written as zeros.
// Word cd = 8 gg + 2 rr + hh of an operand row holds the matrix-core k indices 32 gg + 8 rr + 4 hh + n, n = 0..3,
// i.e. the activations k = 32 gg + 8 n + 2 rr + hh of the chunk: weight k0 = 2 p + hh of block gg is plane bit
// p = 4 n + rr, which the plane expansion puts into nibble n + 4 hh of register rr.
template <int NT>
__global__ void __launch_bounds__(256) hlq_rows_split_kernel(const GemvProbs probs)
{
    constexpr int TPO = 4 / NT, RPO = 16 / TPO;
    const GemvProb &P = probs.p[blockIdx.y];
    const int m = (int)blockIdx.x, tid = (int)threadIdx.x;
    const int K = P.nchunks * 128;
    __shared__ uint32_t wmax[4];
    const bool have = m < P.M;
    const uint16_t *xrow = P.x + (size_t)min(m, P.M - 1) * P.ldx;

    // ---- largest magnitude of the row (as an fp16 bit pattern; the ordering of magnitudes is that of the patterns).
    // Every workgroup of the row scans the whole row (a few tens of KB): cheaper than a second launch or a hand-over.
    uint32_t mxv = 0;
    if (have) {
        for (int k0 = 0; k0 < K; k0 += 256 * 8 * 8) {   // eight independent 128-bit loads in flight per thread
            uint4 v[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int k = k0 + (i * 256 + tid) * 8;
                v[i] = k < K ? *(const uint4 *)(xrow + k) : make_uint4(0u, 0u, 0u, 0u);
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const uint32_t u[4] = {v[i].x, v[i].y, v[i].z, v[i].w};
#pragma unroll
                for (int d = 0; d < 4; ++d)
                    mxv = __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(ushort2_t, mxv),
                                                                                __builtin_bit_cast(ushort2_t, u[d] & 0x7fff7fffu)));
            }
        }
    }
    mxv = max(mxv & 0xffffu, mxv >> 16);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) mxv = max(mxv, (uint32_t)__shfl_xor((int)mxv, o));
    if ((tid & 63) == 0) wmax[tid >> 6] = mxv;
    __syncthreads();
    mxv = max(max(wmax[0], wmax[1]), max(wmax[2], wmax[3]));
    // biased fp16 exponent e of the largest magnitude: |x| < 2^(e-14); scaling by 2^(29-e) gives |x| < 2^15.  Plane
    // codes are worth 1/2, 1, 2, 2 by expansion register rr: weights 1/2, 1/4, 1/8, 1/8 make every product
    // bit x activation / 4.  The factor (<= 2^29) is applied as two fp16 multiplications.
    const int e = (int)(mxv >> 10);
    if (tid == 0 && m < RPO && blockIdx.z == 0) P.xexp[m] = e;

    // ---- the terms: item = (chunk, word cd); this workgroup converts the chunks [c0, c1) of its row
    const int per = (P.nchunks + (int)gridDim.z - 1) / (int)gridDim.z;
    const int c0 = (int)blockIdx.z * per, c1 = min(c0 + per, P.nchunks);
    for (int item = c0 * 32 + tid; item < c1 * 32; item += 256) {
        const int ch = item >> 5, cd = item & 31;
        const int rr = (cd >> 1) & 3;
        char *dst = P.xt + (size_t)ch * (NT * ROWS_OPERAND_BYTES) + 4 * cd;
        uint32_t word[4] = {0u, 0u, 0u, 0u};
        if (have) {
            const uint16_t *src = xrow + (size_t)ch * 128 + 32 * (cd >> 3) + 2 * rr + (cd & 1);
            const uint32_t x0 = src[0], x1 = src[8], x2 = src[16], x3 = src[24];
            const int k1 = (29 - e) / 2, k2 = (29 - e) - k1 - (rr == 0 ? 1 : rr == 1 ? 2 : 3);   // -4 <= k2 <= 14
            const _Float16 f1 = __builtin_bit_cast(_Float16, (uint16_t)((15 + k1) << 10));
            const _Float16 f2 = __builtin_bit_cast(_Float16, (uint16_t)((15 + k2) << 10));
            const half2_t sw1 = {f1, f1}, sw2 = {f2, f2};
            half2_t p0 = __builtin_bit_cast(half2_t, x0 | (x1 << 16));
            half2_t p1 = __builtin_bit_cast(half2_t, x2 | (x3 << 16));
            p0 = (p0 * sw1) * sw2;   // exact: powers of two, in range
            p1 = (p1 * sw1) * sw2;
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                // cut to three significant bits: the high byte of an fp16 is a bf8 code; the remainder is exact
                const uint32_t u0 = __builtin_bit_cast(uint32_t, p0) & 0xff00ff00u, u1 = __builtin_bit_cast(uint32_t, p1) & 0xff00ff00u;
                word[t] = __builtin_amdgcn_perm(u1, u0, 0x07050301u);   // the four codes in k order
                p0 = p0 - __builtin_bit_cast(half2_t, u0);
                p1 = p1 - __builtin_bit_cast(half2_t, u1);
            }
        }
        if (m < RPO) {
#pragma unroll
            for (int t = 0; t < 4; ++t)
                *(u32_alias *)(dst + ((t / TPO) * 16 + (t % TPO) * RPO + m) * 128) = word[t];
        }
    }
}

template <int Q>
struct RowsRegs {
    uint32_t w[Q][4];      // plane j: the four words (32 k each) of column `lane`
    uint16_t mt[Q + 1];    // scales and zero of column `lane` for the chunk's quant group
};

template <int Q, int G, int NT>
__global__ void __launch_bounds__(512)
hlq_gemm_rows_kernel(const int4v bb_lo, const int4v bb_hi, const int out_f32_flag, const GemvProbs probs)
{
    static_assert(G >= 128, "one quant segment per chunk");
    static_assert(NT == 1 || NT == 2 || NT == 4, "one operand, or two or four chained ones");
    constexpr int TPO = 4 / NT;            // terms per operand
    constexpr int RPO = 16 / TPO;          // activation rows an operand carries
    constexpr int MSTR = rows_meta_stride(Q);
    using Regs = RowsRegs<Q>;
    const int W = (int)(blockDim.x >> 6);
    extern __shared__ __attribute__((aligned(256))) char lds[];

    const GemvProb P = probs.p[gemv_problem_of(bb_lo, bb_hi, (int)blockIdx.x)];
    int tg, slice;
    gemv_split_block(P, (int)blockIdx.x - P.blk_begin, tg, slice);

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int KW = P.kw, KSH = P.kw_shift, part = wave & (KW - 1);   // W and KW are powers of two
    const int tile = tg * (W >> KSH) + (wave >> KSH);
    const bool tile_ok = tile < P.ntiles;             // a surplus wavefront gets an empty run
    const int tile_c = tile_ok ? tile : P.ntiles - 1;
    const int M = P.M;
    // this wavefront's run of chunks: the workgroup's K slice is cut into KW near-equal parts
    const int sbeg = min(slice * P.cps, P.nchunks - 1);
    const int send = min(sbeg + P.cps, P.nchunks);
    const int len = send - sbeg;
    const int cbeg = sbeg + ((len * part) >> KSH);
    const int cend = tile_ok ? sbeg + ((len * (part + 1)) >> KSH) : cbeg;

    const int tw = hlq_tile_width(tile_c, P.N);
    const char *tile_base = P.packed + (size_t)tile_c * HLQ_TILE_N * P.col_bytes;
    const int c = lane & 15, g = lane >> 4;
    const uint32_t moff = (uint32_t)(lane < tw ? lane : tw - 1) * 2u;   // clamped column: loads stay in bounds
    const uint32_t woff = moff * 8u;
    char *meta = lds + wave * rows_wave_lds(Q);           // this wavefront's scales [64][MSTR]
    float *red = (float *)(meta + 64 * MSTR);             // and results [16][64] for the sum over the tile's KW runs

    // ---- weights: range-checked loads through a descriptor over [tile start, end of the run's last record) ----
    const uint32_t run_end = tile_ok ? hlq_rec_in_tile(tw, cend, Q, G) : 0u;
    const __amdgpu_buffer_rsrc_t wrsrc = __builtin_amdgcn_make_buffer_rsrc((void *)tile_base, 0, (int)run_end, 0x00020000);
    auto load_plane = [&](int ch, Regs &R, int j) {
        const uint32_t vo = woff + hlq_rec_in_tile(tw, ch, Q, G);
        const int4v v = __builtin_bit_cast(int4v, __builtin_amdgcn_raw_buffer_load_b128(wrsrc, (int)vo, j * tw * 16, 2));
        R.w[j][0] = v.x; R.w[j][1] = v.y; R.w[j][2] = v.z; R.w[j][3] = v.w;
    };
    auto load_meta = [&](int ch, Regs &R) {
        const int cm = G > 128 ? (ch & ~1) : ch;      // a 256-wide group keeps its scales in its first (even) chunk
        const uint32_t vo = moff + hlq_rec_in_tile(tw, cm, Q, G);
#pragma unroll
        for (int r = 0; r <= Q; ++r) R.mt[r] = __builtin_amdgcn_raw_buffer_load_b16(wrsrc, (int)vo, tw * Q * 16 + r * tw * 2, 0);
    };

    // first loads: the weights of the first two chunks
    Regs R[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
#pragma unroll
        for (int j = 0; j < Q; ++j) load_plane(cbeg + i, R[i], j);
        load_meta(cbeg + i, R[i]);
    }

    // ---- activation operands: made by hlq_rows_split_kernel, [chunk][operand][row][128 codes].  Lane (row = lane & 15,
    // g) holds the 16-k runs [16 g, 16 g + 16) and [64 + 16 g, ...) of its row: two 128-bit loads per operand.
    const char *a_src = P.xt + (lane & 15) * 128 + 16 * g;
    struct Ops {
        int8v A[NT];
    };
    auto load_ops = [&](int ch, Ops &o) {
        if (HLQ_ROWS_DEBUG == 3 && ch > cbeg + 1) return;   // timing experiment: operands of the first two chunks only
        const int chx = max(min(ch, cend - 1), sbeg);   // stays inside K also past the end of the run
        const char *src = a_src + (size_t)chx * (NT * ROWS_OPERAND_BYTES);
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const uint4 lo = *(const uint4 *)(src + t * ROWS_OPERAND_BYTES);
            const uint4 hi = *(const uint4 *)(src + t * ROWS_OPERAND_BYTES + 64);
            o.A[t] = (int8v){(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, (int)hi.z, (int)hi.w};
        }
    };
    // scales: lane <-> column to LDS, read back per column block (this lane's column 16 cb + c)
    struct Sc {
        uint32_t m[4][MSTR / 4];
    };
    auto stage_scales = [&](const Regs &Rn, Sc &s) {
#pragma unroll
        for (int r = 0; r <= Q; ++r) ((u16_alias *)(meta + lane * MSTR))[r] = Rn.mt[r];
#pragma unroll
        for (int cb = 0; cb < 4; ++cb)
#pragma unroll
            for (int i = 0; i < MSTR / 4; ++i) s.m[cb][i] = ((const u32_alias *)(meta + (16 * cb + c) * MSTR))[i];
    };
    auto scale_of = [](const uint32_t (&m)[MSTR / 4], int i) -> float {
        const half2_t h = __builtin_bit_cast(half2_t, m[i >> 1]);
        return (float)((i & 1) ? h.y : h.x);
    };
    auto expand = [](uint32_t w) -> int8v {   // plane word -> 32 fp4 codes (bit 4p+r -> nibble p of register r)
        if (HLQ_ROWS_SKIP & 4) return (int8v){(int)w, 0x22222222, 0x44444444, 0x11111111, 0, 0, 0, 0};
        return (int8v){(int)(w & 0x11111111u), (int)(w & 0x22222222u), (int)(w & 0x44444444u),
                       (int)((w >> 1) & 0x44444444u), 0, 0, 0, 0};
    };
    const float4v zero4 = {0.f, 0.f, 0.f, 0.f};
    auto chain = [&](const Ops &o, const int8v &B) -> float4v {
        float4v d = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(o.A[0], B, zero4, 1, 4, 0, 0, 0, 0);
#pragma unroll
        for (int t = 1; t < NT; ++t) d = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(o.A[t], B, d, 1, 4, 0, 0, 0, 0);
        return d;
    };

    // acc[sl][cb]: output (operand row 4 g + sl, column 16 cb + c) -- for NT = 2 still split by term half
    float acc[4][4];
#pragma unroll
    for (int sl = 0; sl < 4; ++sl)
#pragma unroll
        for (int cb = 0; cb < 4; ++cb) acc[sl][cb] = 0.f;

    // One chunk: the items (plane j, column block cb) as a software pipeline -- matrix-core chain of item n |
    // expansion of the word of item n + 1, scales applied to the result of item n - 1.  R's planes are reloaded
    // (chunk two ahead) right after their last item; past the end of the slice the range check answers with zeros.
    auto step = [&](Regs &R, const Ops &o, const Sc &s, int ch_reload) {
        constexpr int NI = 4 * Q;
        if (HLQ_ROWS_DEBUG == 1) {   // timing experiment: loads only
            uint32_t m = 0;
#pragma unroll
            for (int j = 0; j < Q; ++j) m ^= R.w[j][0] ^ R.w[j][1] ^ R.w[j][2] ^ R.w[j][3];
            acc[0][0] += (float)m + (float)o.A[0][0] + (float)s.m[0][0];
            load_meta(ch_reload, R);
#pragma unroll
            for (int j = 0; j < Q; ++j) load_plane(ch_reload, R, j);
            return;
        }
        auto apply = [&](const float4v &d, int cb, int which) {
            if (HLQ_ROWS_SKIP & 1) {
                acc[0][cb] += d[which & 3];
                return;
            }
            const float sc = scale_of(s.m[cb], which);
#pragma unroll
            for (int sl = 0; sl < 4; ++sl) acc[sl][cb] += sc * d[sl];
        };
        const int8v ones = {0x11111111, 0x22222222, 0x44444444, 0x44444444, 0, 0, 0, 0};
        const float4v xs = chain(o, ones);   // the chunk's activation sums per row, for the zero points
        uint32_t wt[Q][4];
#pragma unroll
        for (int j = 0; j < Q; ++j) {        // 4 x 4 transpose over (16-lane group, word)
            const uint2v s01 = __builtin_amdgcn_permlane16_swap(R.w[j][0], R.w[j][1], false, false);
            const uint2v s23 = __builtin_amdgcn_permlane16_swap(R.w[j][2], R.w[j][3], false, false);
            const uint2v t02 = __builtin_amdgcn_permlane32_swap(s01.x, s23.x, false, false);
            const uint2v t13 = __builtin_amdgcn_permlane32_swap(s01.y, s23.y, false, false);
            wt[j][0] = t02.x; wt[j][2] = t02.y; wt[j][1] = t13.x; wt[j][3] = t13.y;
            if (HLQ_ROWS_SKIP & 2) { wt[j][0] = R.w[j][0]; wt[j][1] = R.w[j][1]; wt[j][2] = R.w[j][2]; wt[j][3] = R.w[j][3]; }
        }
        if (HLQ_ROWS_DEBUG < 2) load_meta(ch_reload, R);             // its scales were staged one chunk ahead
        // Items go through the matrix core two at a time: the chains of a pair are independent, so the second
        // instruction of one never waits for the first of the same chain, and the vector work of the stage (expansion
        // of the next pair's words, scales on the previous pair's results) is dealt out between the matrix-core
        // instructions instead of queueing behind them.
        constexpr int NP = NI / 2;
        int8v B0 = expand(wt[0][0]), B1 = expand(wt[0][1]);
        float4v pA = zero4, pB = zero4;
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int pr = 0; pr < NP; ++pr) {
            const int n0 = 2 * pr, n1 = 2 * pr + 1;
            float4v dA = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(o.A[0], B0, zero4, 1, 4, 0, 0, 0, 0);
            float4v dB = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(o.A[0], B1, zero4, 1, 4, 0, 0, 0, 0);
#pragma unroll
            for (int t = 1; t < NT; ++t) {
                dA = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(o.A[t], B0, dA, 1, 4, 0, 0, 0, 0);
                dB = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(o.A[t], B1, dB, 1, 4, 0, 0, 0, 0);
            }
            int8v nB0 = B0, nB1 = B1;
            if (pr + 1 < NP) {
                nB0 = expand(wt[(n0 + 2) / 4][(n0 + 2) % 4]);
                nB1 = expand(wt[(n1 + 2) / 4][(n1 + 2) % 4]);
            }
            if (n1 % 4 == 3 && HLQ_ROWS_DEBUG < 2) load_plane(ch_reload, R, n1 / 4);   // the plane's last item is in this pair
            if (pr >= 1) {
                apply(pA, (n0 - 2) % 4, (n0 - 2) / 4);
                apply(pB, (n1 - 2) % 4, (n1 - 2) / 4);
            }
            // 2 NT matrix-core instructions, each followed by its share of the stage's vector instructions
#pragma unroll
            for (int i = 0; i < 2 * NT; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x002, NT == 1 ? 9 : NT == 2 ? 6 : 3, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
            pA = dA; pB = dB; B0 = nB0; B1 = nB1;
        }
        apply(pA, (NI - 2) % 4, (NI - 2) / 4);
        apply(pB, (NI - 1) % 4, (NI - 1) / 4);
#pragma unroll
        for (int cb = 0; cb < 4; ++cb) apply(xs, cb, Q);
    };

    // ---- chunk loop: no barrier; weights two chunks ahead, activation operands and staged scales one chunk ahead -----
    Ops oA, oB;
    load_ops(cbeg, oA);
    Sc sc0, sc1;
    stage_scales(R[0], sc0);
    for (int ch = cbeg; ch < cend; ch += 2) {   // two chunks per trip: register sets are named at compile time
        load_ops(ch + 1, oB);
        stage_scales(R[1], sc1);
        step(R[0], oA, sc0, ch + 2);
        if (ch + 1 < cend) {
            load_ops(ch + 2, oA);
            stage_scales(R[0], sc0);
            step(R[1], oB, sc1, ch + 3);
        }
    }

    // ---- undo the rows' scaling, add the two term halves (NT = 2) and the tile's KW runs, store --------------------
    float y[4][4];
#pragma unroll
    for (int sl = 0; sl < 4; ++sl) {
        const int row = (NT == 1 ? 0 : NT == 2 ? 4 * (g & 1) : 4 * g) + sl;
        const float f = __builtin_bit_cast(float, (uint32_t)(127 + 2 - 29 + P.xexp[row]) << 23);   // 4 * 2^(e-29)
#pragma unroll
        for (int cb = 0; cb < 4; ++cb) {
            float v = acc[sl][cb];
            if (NT == 1) v += __shfl_xor(v, 16);   // one term per 16-lane group
            if (NT <= 2) v += __shfl_xor(v, 32);   // NT = 2: lanes 32..63 hold terms 2, 3 of the same rows
            y[sl][cb] = v * f;
        }
    }
    if (KW > 1) {
#pragma unroll
        for (int sl = 0; sl < 4; ++sl)
#pragma unroll
            for (int cb = 0; cb < 4; ++cb) red[(sl * 4 + cb) * 64 + lane] = y[sl][cb];
        __syncthreads();
        if (part == 0) {
            constexpr int RSTR = rows_wave_lds(Q) / 4;   // floats between wavefronts' blocks
#pragma unroll
            for (int sl = 0; sl < 4; ++sl)
#pragma unroll
                for (int cb = 0; cb < 4; ++cb)
                    for (int w2 = 1; w2 < KW; ++w2) y[sl][cb] += red[w2 * RSTR + (sl * 4 + cb) * 64 + lane];
        }
    }
    if (!tile_ok || part != 0) return;
    if ((NT == 2 && g >= 2) || (NT == 1 && g >= 1)) return;
    const int row0 = (NT == 1 ? 0 : NT == 2 ? 4 * (g & 1) : 4 * g);
    const size_t n0 = (size_t)tile * HLQ_TILE_N;
    const size_t ldy = (size_t)P.ldy;
    const int out_f32 = out_f32_flag;

    if (P.nslices == 1) {
#pragma unroll
        for (int sl = 0; sl < 4; ++sl)
#pragma unroll
            for (int cb = 0; cb < 4; ++cb)
                if (row0 + sl < M && 16 * cb + c < tw) store_out(P.y, (size_t)(row0 + sl) * ldy + n0 + 16 * cb + c, y[sl][cb], out_f32);
        return;
    }
    // ---- split-K across workgroups: write-through partials [slice][row][N], arrival counter per tile, the last
    // workgroup to arrive adds in slice order
    const size_t MN = (size_t)M * P.N;
#pragma unroll
    for (int sl = 0; sl < 4; ++sl)
#pragma unroll
        for (int cb = 0; cb < 4; ++cb)
            if (row0 + sl < M && 16 * cb + c < tw)
                __hip_atomic_store(&P.part[(size_t)slice * MN + (size_t)(row0 + sl) * P.N + n0 + 16 * cb + c], y[sl][cb],
                                   __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    // every lane that stored has its writes acknowledged once the whole wavefront is past the wait above
    int old = 0;
    if (lane == 0) old = __hip_atomic_fetch_add(&P.cnt[tile], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    old = __builtin_amdgcn_readfirstlane(old);
    if (old != P.nslices - 1) return;
    // all sixteen outputs of a lane, of four slices, are read before any is added (64 loads in flight); the sums
    // still run in slice order
    {
        float a[4][4];
        const float *src[4][4];
        bool on[4][4];
#pragma unroll
        for (int sl = 0; sl < 4; ++sl)
#pragma unroll
            for (int cb = 0; cb < 4; ++cb) {
                a[sl][cb] = 0.f;
                on[sl][cb] = row0 + sl < M && 16 * cb + c < tw;
                // lanes without an output re-read a valid one (row 0 of this tile's first column) and drop it
                src[sl][cb] = &P.part[on[sl][cb] ? (size_t)(row0 + sl) * P.N + n0 + 16 * cb + c : n0];
            }
        for (int s2 = 0; s2 < P.nslices; s2 += 4) {   // four slices per trip; slices past the last re-read it and add zero
            float v[4][4][4];
#pragma unroll
            for (int k = 0; k < 4; ++k)
#pragma unroll
                for (int sl = 0; sl < 4; ++sl)
#pragma unroll
                    for (int cb = 0; cb < 4; ++cb)
                        v[k][sl][cb] = __hip_atomic_load(src[sl][cb] + (size_t)min(s2 + k, P.nslices - 1) * MN, __ATOMIC_RELAXED,
                                                         __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
            for (int k = 0; k < 4; ++k)
#pragma unroll
                for (int sl = 0; sl < 4; ++sl)
#pragma unroll
                    for (int cb = 0; cb < 4; ++cb) a[sl][cb] += s2 + k < P.nslices ? v[k][sl][cb] : 0.f;
        }
#pragma unroll
        for (int sl = 0; sl < 4; ++sl)
#pragma unroll
            for (int cb = 0; cb < 4; ++cb)
                if (on[sl][cb]) store_out(P.y, (size_t)(row0 + sl) * ldy + n0 + 16 * cb + c, a[sl][cb], out_f32);
    }
    if (lane == 0) __hip_atomic_store(&P.cnt[tile], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

template <int Q, int G>
void launch_qg(const GemvBatch &b, unsigned nblocks, int W, int rows, hipStream_t st)
{
    const dim3 blk(64 * W);
    const GemvKernelArgs a = gemv_kernel_args(b);
    if constexpr (G >= 128) {
        if (rows <= 4) {
            hlq_rows_split_kernel<1><<<dim3(4, b.count, 8), 256, 0, st>>>(a.probs);
            hlq_gemm_rows_kernel<Q, G, 1><<<nblocks, blk, (size_t)rows_lds_bytes(Q, W), st>>>(a.lo, a.hi, a.out_f32, a.probs);
        } else if (rows <= 8) {
            hlq_rows_split_kernel<2><<<dim3(8, b.count, 8), 256, 0, st>>>(a.probs);
            hlq_gemm_rows_kernel<Q, G, 2><<<nblocks, blk, (size_t)rows_lds_bytes(Q, W), st>>>(a.lo, a.hi, a.out_f32, a.probs);
        } else {
            hlq_rows_split_kernel<4><<<dim3(16, b.count, 8), 256, 0, st>>>(a.probs);
            hlq_gemm_rows_kernel<Q, G, 4><<<nblocks, blk, (size_t)rows_lds_bytes(Q, W), st>>>(a.lo, a.hi, a.out_f32, a.probs);
        }
    }
}

template <int Q>
hlq_status launch_q(int G, const GemvBatch &b, unsigned nblocks, int W, int rows, hipStream_t st)
{
    switch (G) {
    case 128: launch_qg<Q, 128>(b, nblocks, W, rows, st); return HLQ_OK;
    case 256: launch_qg<Q, 256>(b, nblocks, W, rows, st); return HLQ_OK;
    }
    return HLQ_ERR_UNSUPPORTED;
}

} // namespace

size_t hlq_gemm_rows_xt_bytes(const HlqDims &dm, int64_t M)
{
    if (M < 1 || M > hlq_gemm_rows_max(dm.G)) return 0;
    const size_t nt = M <= 4 ? 1 : M <= 8 ? 2 : 4;
    return (size_t)dm.nchunks * nt * ROWS_OPERAND_BYTES + 256;   // operands + the row exponents, kept 256-byte aligned
}

// rows this kernel carries for group size G (0: no instantiation)
int hlq_gemm_rows_max(int G) { return G >= 128 ? 16 : 0; }

hlq_status hlq_launch_gemm_rows(const GemvBatch &b, unsigned nblocks, int W, int rows, int q, int G, hipStream_t st)
{
    if ((W != 2 && W != 4 && W != 8) || rows < 1 || rows > hlq_gemm_rows_max(G)) return HLQ_ERR_UNSUPPORTED;
    switch (q) {
    case 1: return launch_q<1>(G, b, nblocks, W, rows, st);
    case 2: return launch_q<2>(G, b, nblocks, W, rows, st);
    case 3: return launch_q<3>(G, b, nblocks, W, rows, st);
    case 4: return launch_q<4>(G, b, nblocks, W, rows, st);
    }
    return HLQ_ERR_UNSUPPORTED;
}
