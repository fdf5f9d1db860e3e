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
// multiplication per (row, column, plane).  NT = 2 carries up to 8 rows, NT = 4 up to 16.
//
// Work split.  A workgroup of W wavefronts owns W adjacent column tiles (wavefront <-> tile, lane <->
// column when loading, as in the GEMV kernels) and one K slice; every wavefront walks the slice on its
// own -- after one barrier at the start nothing is shared, so the wavefronts of a SIMD drift apart and
// one's vector phases (word transpose, activation conversion) run under the other's matrix-core phases.
// Per chunk a wavefront converts the activations of all rows itself: a lane takes eight activations of
// a row (four pairs of neighbours), cuts them into the four terms and writes two packed words per term
// to its LDS block (matrix-core k order); the operands are read back once per chunk.  Per row a
// power-of-two scale taken from the largest magnitude of the row's slice (found once per workgroup)
// puts the activations high in the bf8 range; it is removed at the end.  K slices of different
// workgroups meet in the workspace (partial sums, one arrival counter per tile, last arriver adds in
// slice order).
#include "hlq_gemv_common.h"

#ifndef HLQ_ROWS_DEBUG
#define HLQ_ROWS_DEBUG 0   // timing experiments -- 1: loads only (no matrix-core work), 2: no reloads (compute only)
#endif

namespace {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef unsigned short ushort2_t __attribute__((ext_vector_type(2)));
typedef int int8v __attribute__((ext_vector_type(8)));
typedef unsigned int uint2v __attribute__((ext_vector_type(2)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef uint16_t __attribute__((may_alias)) u16_alias;
typedef uint32_t __attribute__((may_alias)) u32_alias;

constexpr int ROWS_XROW = 144;   // bytes per operand row in LDS: 128 codes + 16 of padding, so that the 16 rows a
                                 // quarter-wave reads side by side fall into different banks
constexpr int rows_meta_stride(int Q) { return ((Q + 1) * 2 + 7) & ~7; }
constexpr int rows_xt_bytes(int NT) { return NT * 16 * ROWS_XROW; }   // NT operands x 16 rows
// LDS per wavefront: operands | scales [64][stride] | row exponents (16 ints) | results [16][64] fp32
constexpr int rows_wave_lds(int Q, int NT) { return rows_xt_bytes(NT) + 64 * rows_meta_stride(Q) + 64 + 16 * 64 * 4; }
constexpr int rows_lds_bytes(int Q, int NT, int W) { return W * rows_wave_lds(Q, NT); }

template <int CTRL, int ROWMASK = 0xf>
__device__ __forceinline__ uint32_t max_dpp(uint32_t v)
{
    const uint32_t moved = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, ROWMASK, 0xf, false);
    return max(v, moved);
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
    static_assert(NT == 2 || NT == 4, "two or four chained operands");
    constexpr int TPO = 4 / NT;            // terms per operand
    constexpr int RPO = 16 / TPO;          // activation rows an operand carries
    constexpr int MSTR = rows_meta_stride(Q);
    constexpr int XTB = rows_xt_bytes(NT);
    using Regs = RowsRegs<Q>;
    const int W = (int)(blockDim.x >> 6);
    extern __shared__ __attribute__((aligned(256))) char lds[];

#ifdef HLQ_ROWS_TS
    const long long ts0 = wall_clock64();
    long long ts1 = 0, ts2 = 0, ts3 = 0;
#endif
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
    char *xt = lds + wave * rows_wave_lds(Q, NT);        // this wavefront's operands [NT][16][ROWS_XROW],
    char *meta = xt + XTB;                                // scales [64][MSTR],
    int *exps = (int *)(meta + 64 * MSTR);                // row exponents [16]
    float *red = (float *)(meta + 64 * MSTR + 64);        // and results [16][64] for the sum over the tile's KW runs

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

    // ---- activations.  A conversion item is (row, 32-k block gg, register rr): the eight activations
    // k = 32 gg + 8 n + 2 rr + hh (n = 0..3, hh = 0, 1), i.e. four pairs of neighbours, which end up as the two words
    // cd = 8 gg + 2 rr + hh of the row -- matrix-core k indices 32 gg + 8 rr + 4 hh + n (weight k0 = 2 p + hh of block
    // gg is plane bit p = 4 n + rr, which the expansion puts into nibble n + 4 hh of register rr).  Lane l takes
    // items (row 4 i + (l >> 4), gg = (l >> 2) & 3, rr = l & 3), i < NIT: a row of sixteen lanes covers a chunk row.
    constexpr int NIT = RPO / 4;
    int rowexp[NIT];
    const int rr = lane & 3, cw = 8 * ((lane >> 2) & 3) + 2 * rr;   // first of the item's two words
    const uint32_t *xsrc[NIT];
    bool conv_on[NIT];
#pragma unroll
    for (int i = 0; i < NIT; ++i) {
        const int row = 4 * i + g;
        conv_on[i] = row < M;
        xsrc[i] = (const uint32_t *)(P.x + (size_t)min(row, M - 1) * P.ldx) + (16 * ((lane >> 2) & 3) + rr);
    }
    uint32_t xv[NIT][4];
    auto load_x = [&](int ch) {
        const int chx = max(min(ch, cend - 1), sbeg);   // stays inside the slice also for an empty run
#pragma unroll
        for (int i = 0; i < NIT; ++i)
#pragma unroll
            for (int n = 0; n < 4; ++n) xv[i][n] = xsrc[i][(size_t)chx * 64 + 4 * n];
    };

    // first loads: activations of the first chunk, then the weights of the first two chunks
    load_x(cbeg);
    Regs R[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
#pragma unroll
        for (int j = 0; j < Q; ++j) load_plane(cbeg + i, R[i], j);
        load_meta(cbeg + i, R[i]);
    }

    // clear the operand block (rows past M and the padding are never written)
    for (int i = lane; i < XTB / 4; i += 64) ((uint32_t *)xt)[i] = 0u;

    // ---- per row: largest magnitude of this wavefront's run -> power-of-two scale.  The sixteen lanes of a lane
    // row scan an activation row, one 128-bit load per lane and chunk, eight chunks in flight.
#pragma unroll
    for (int i = 0; i < NIT; ++i) {
        const int row = 4 * i + g;
        const uint4 *xr = (const uint4 *)(P.x + (size_t)min(row, M - 1) * P.ldx) + c;
        uint32_t mxv = 0;
        for (int base = cbeg; base < cend; base += 8) {   // chunks past the end re-read the last one
            uint4 v[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) v[k] = xr[(size_t)min(base + k, cend - 1) * 16];
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const uint32_t u[4] = {v[k].x, v[k].y, v[k].z, v[k].w};
#pragma unroll
                for (int d = 0; d < 4; ++d)
                    mxv = __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(ushort2_t, mxv),
                                                                                __builtin_bit_cast(ushort2_t, u[d] & 0x7fff7fffu)));
            }
        }
        mxv = max(mxv & 0xffffu, mxv >> 16);
        mxv = max_dpp<0xB1>(mxv);          // quad_perm [1,0,3,2]
        mxv = max_dpp<0x4E>(mxv);          // quad_perm [2,3,0,1]
        mxv = max_dpp<0x124>(mxv);         // row_ror:4
        mxv = max_dpp<0x128>(mxv);         // row_ror:8: every lane holds the maximum of its sixteen lanes = of its row
        if (c == 0) exps[row] = (int)(mxv >> 10);   // for the lanes that hold this row's results at the end
        rowexp[i] = (int)(mxv >> 10);
    }
    // biased fp16 exponent e of the largest magnitude: |x| < 2^(e-14); scaling by 2^(29-e) gives |x| < 2^15.  Plane
    // codes are worth 1/2, 1, 2, 2 by expansion register rr: lane weights 1/2, 1/4, 1/8, 1/8 make every product
    // bit x activation / 4.  The factor (<= 2^29) is applied as two fp16 multiplications.
    half2_t sw1[NIT], sw2[NIT];
#pragma unroll
    for (int i = 0; i < NIT; ++i) {
        const int e = rowexp[i];
        const int k1 = (29 - e) / 2, k2 = (29 - e) - k1 - (rr == 0 ? 1 : rr == 1 ? 2 : 3);
        const _Float16 f1 = __builtin_bit_cast(_Float16, (uint16_t)((15 + k1) << 10));
        const _Float16 f2 = __builtin_bit_cast(_Float16, (uint16_t)((15 + k2) << 10));
        sw1[i] = (half2_t){f1, f1};
        sw2[i] = (half2_t){f2, f2};
    }

    // Converts the activations in xv into their four terms and stores them in the operand block.  Term t of row m goes
    // to operand t / TPO, operand row (t % TPO) * RPO + m.
    auto convert = [&]() {
#pragma unroll
        for (int i = 0; i < NIT; ++i) {
            if (!conv_on[i]) continue;
            // xv[i][n] = (x[.. + 8 n + hh]) for hh = 0 (low half), 1 (high half): separate the two hh
            half2_t p0[2], p1[2];
            p0[0] = __builtin_bit_cast(half2_t, __builtin_amdgcn_perm(xv[i][1], xv[i][0], 0x05040100u));   // n = 0, 1, hh = 0
            p1[0] = __builtin_bit_cast(half2_t, __builtin_amdgcn_perm(xv[i][3], xv[i][2], 0x05040100u));   // n = 2, 3, hh = 0
            p0[1] = __builtin_bit_cast(half2_t, __builtin_amdgcn_perm(xv[i][1], xv[i][0], 0x07060302u));   // hh = 1
            p1[1] = __builtin_bit_cast(half2_t, __builtin_amdgcn_perm(xv[i][3], xv[i][2], 0x07060302u));
            char *dst = xt + (4 * i + g) * ROWS_XROW + 4 * cw;
#pragma unroll
            for (int hh = 0; hh < 2; ++hh) {
                p0[hh] = (p0[hh] * sw1[i]) * sw2[i];   // exact: powers of two, in range
                p1[hh] = (p1[hh] * sw1[i]) * sw2[i];
            }
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                uint32_t word[2];
#pragma unroll
                for (int hh = 0; hh < 2; ++hh) {
                    const uint32_t u0 = __builtin_bit_cast(uint32_t, p0[hh]) & 0xff00ff00u;
                    const uint32_t u1 = __builtin_bit_cast(uint32_t, p1[hh]) & 0xff00ff00u;
                    word[hh] = __builtin_amdgcn_perm(u1, u0, 0x07050301u);   // the four codes (high bytes) in k order
                    if (t < 3) {
                        p0[hh] = p0[hh] - __builtin_bit_cast(half2_t, u0);   // exact remainders
                        p1[hh] = p1[hh] - __builtin_bit_cast(half2_t, u1);
                    }
                }
                *(uint2v *)(dst + ((t / TPO) * 16 + (t % TPO) * RPO) * ROWS_XROW) = (uint2v){word[0], word[1]};
            }
        }
    };

    // ---- operand role: row (lane & 15) of every operand, 16-k runs [16 g, 16 g + 16) and [64 + 16 g, ...) ----------
    const char *a_src = xt + (lane & 15) * ROWS_XROW + 16 * g;
    struct Ops {
        int8v A[NT];
    };
    auto read_ops = [&](Ops &o) {
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const uint4 lo = *(const uint4 *)(a_src + t * 16 * ROWS_XROW);
            const uint4 hi = *(const uint4 *)(a_src + t * 16 * ROWS_XROW + 64);
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
        }
        if (HLQ_ROWS_DEBUG != 2) load_meta(ch_reload, R);             // its scales were staged one chunk ahead
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
            if (n1 % 4 == 3 && HLQ_ROWS_DEBUG != 2) load_plane(ch_reload, R, n1 / 4);   // the plane's last item is in this pair
            if (pr >= 1) {
                apply(pA, (n0 - 2) % 4, (n0 - 2) / 4);
                apply(pB, (n1 - 2) % 4, (n1 - 2) / 4);
            }
            // 2 NT matrix-core instructions, each followed by its share of the stage's vector instructions
#pragma unroll
            for (int i = 0; i < 2 * NT; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x002, NT == 2 ? 6 : 3, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
            pA = dA; pB = dB; B0 = nB0; B1 = nB1;
        }
        apply(pA, (NI - 2) % 4, (NI - 2) / 4);
        apply(pB, (NI - 1) % 4, (NI - 1) / 4);
#pragma unroll
        for (int cb = 0; cb < 4; ++cb) apply(xs, cb, Q);
    };

    // ---- chunk loop: no barrier; LDS operations of a wavefront execute in order, so the conversion of the next chunk
    // may overwrite the operand block as soon as this chunk's operands have been asked for -------------------------
    convert();                  // chunk cbeg
    load_x(cbeg + 1);
    Sc sc0, sc1;
    stage_scales(R[0], sc0);
#ifdef HLQ_ROWS_TS
    ts1 = wall_clock64();
#endif
    for (int ch = cbeg; ch < cend; ch += 2) {   // two chunks per trip: register sets are named at compile time
#ifdef HLQ_ROWS_TS
        if (ch == cbeg + 2) ts2 = wall_clock64();
#endif
        {
            Ops o;
            read_ops(o);
            convert();          // next chunk's operands (xv holds its activations)
            load_x(ch + 2);
            stage_scales(R[1], sc1);
            step(R[0], o, sc0, ch + 2);
        }
        if (ch + 1 < cend) {
            Ops o;
            read_ops(o);
            convert();
            load_x(ch + 3);
            stage_scales(R[0], sc0);
            step(R[1], o, sc1, ch + 3);
        }
    }

#ifdef HLQ_ROWS_TS
    ts3 = wall_clock64();
    if (threadIdx.x == 0 && blockIdx.x < 1000) {
        long long *t = (long long *)((char *)probs.p[0].cnt + 65536) + 8 * blockIdx.x;
        t[0] = ts0; t[1] = ts1; t[2] = ts2; t[3] = ts3; t[5] = cend - cbeg; t[6] = (long long)(&P.cnt[0] - probs.p[0].cnt);
    }
#endif
    // ---- undo the rows' scaling, add the two term halves (NT = 2) and the tile's KW runs, store --------------------
    float y[4][4];
#pragma unroll
    for (int sl = 0; sl < 4; ++sl) {
        const int row = (NT == 2 ? 4 * (g & 1) : 4 * g) + sl;
        const float f = __builtin_bit_cast(float, (uint32_t)(127 + 2 - 29 + exps[row]) << 23);   // 4 * 2^(e-29)
#pragma unroll
        for (int cb = 0; cb < 4; ++cb) {
            float v = acc[sl][cb];
            if (NT == 2) v += __shfl_xor(v, 32);   // lanes 32..63 hold terms 2, 3 of the same rows
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
            constexpr int RSTR = rows_wave_lds(Q, NT) / 4;   // floats between wavefronts' blocks
#pragma unroll
            for (int sl = 0; sl < 4; ++sl)
#pragma unroll
                for (int cb = 0; cb < 4; ++cb)
                    for (int w2 = 1; w2 < KW; ++w2) y[sl][cb] += red[w2 * RSTR + (sl * 4 + cb) * 64 + lane];
        }
    }
#ifdef HLQ_ROWS_TS
    if (threadIdx.x == 0 && blockIdx.x < 1000) ((long long *)((char *)probs.p[0].cnt + 65536))[8 * blockIdx.x + 4] = wall_clock64();
#endif
    if (!tile_ok || part != 0) return;
    if (NT == 2 && g >= 2) return;
    const int row0 = (NT == 2 ? 4 * (g & 1) : 4 * g);
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
        if (rows <= 8)
            hlq_gemm_rows_kernel<Q, G, 2><<<nblocks, blk, (size_t)rows_lds_bytes(Q, 2, W), st>>>(a.lo, a.hi, a.out_f32, a.probs);
        else
            hlq_gemm_rows_kernel<Q, G, 4><<<nblocks, blk, (size_t)rows_lds_bytes(Q, 4, W), st>>>(a.lo, a.hi, a.out_f32, a.probs);
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
