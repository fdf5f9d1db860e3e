// hlq_lut_gemv, matrix-core formulation of the bit-serial product (Sec. 2, paragraph
// "Bit-Serial LUT-Based GEMM", and App. B; weights in the format of Eq. 3):
//
//   y[n] = sum_groups ( sum_j s_j[g,n] * <b_j[.,n], x>_g  +  z[g,n] * sum_g(x) )
//
// The inner bit-plane dot product <b_j, x> over a group -- the quantity the lookup tables of App. B
// deliver four activations at a time -- is taken here by v_mfma_f32_16x16x128_f8f6f4, which
// multiplies 4-bit by 8-bit floating-point operands:
//
//   planes       a 32-bit plane word becomes 32 fp4 (e2m1) values with four AND masks: bit 4p+r of
//                the word lands in nibble p of register r as the code 1, 2, 4 or 4 (value 0.5, 1,
//                2, 2).  No table, no LDS traffic, 5 VALU operations per 32 weights.
//   activations  x (fp16) is written as an exact sum of four bf8 (e5m2) terms, x = t0+t1+t2+t3
//                (each term is the running remainder cut to three significant bits, so after
//                four terms all eleven bits of an fp16 significand are covered), after a power-of-
//                two weight (1/2, 1/4, 1/8, 1/8 by register r) that evens out the plane codes.  The
//                four terms occupy four ROWS of the 16-row operand; with quant groups shorter than
//                a chunk the rows are further split by segment (row 4t + sg holds term t, zero
//                outside segment sg), so one MFMA returns every (term, segment) dot product of 16
//                columns x 128 k of one plane.
//   zero point   the same MFMA with an all-ones plane gives the segment sums of x.
//
// The matrix core adds the products of an 8-element run in fixed point aligned to the run's largest
// product and keeps 13 bits below it (measured); every bf8 x fp4 product has three significant
// bits, so a product loses bits only if it is more than 2^10 times smaller than its largest
// neighbour, and then less than 2^-13 of that neighbour.  Everything else is exact fp32 work.
//
// Work split.  A workgroup of W wavefronts owns W / kw adjacent column tiles and one K slice; the kw
// wavefronts of a tile take kw consecutive runs of chunks of the slice and add their results through
// LDS (kw is chosen per problem, so that short and long K in one grouped launch get runs of similar
// length).  Slices of different workgroups meet in the workspace as in the lookup kernel
// (hlq_gemv.hip: partial sums, one arrival counter per tile, the last workgroup adds in slice
// order); that costs three dependent trips to device memory at the end of a workgroup, so the host
// splits K inside the workgroup first.  Everything up to the final sum is private to the wavefront,
// so the chunk loop has no barrier:
//
//   scale     the largest |x| of the wavefront's run fixes a power-of-two scale that puts the
//             activations high in the bf8 range; it is removed from the result at the end, so
//             activations of any magnitude keep their precision;
//   convert   per chunk, lane l turns x[2l], x[2l+1] into four bf8 terms each and stores the codes
//             in the wavefront's LDS block in matrix-core k order, one chunk ahead of the MFMAs;
//   contract  per chunk and column block one MFMA per plane, plus one with the all-ones plane.
//
// A few rows at once (small-batch decode, hlq_lut_gemm with M <= 16).  At M = 1 only four of the 16
// operand rows are in use when a quant group spans the chunk (G >= 128).  The batched instantiation
// fills them: row 4t + (r * SEG + sg) holds term t of activation row r restricted to segment sg, so
// one operand carries 4 / SEG activation rows, NS operands ("row sets") carry NS * 4 / SEG rows,
// and every expanded plane word is used NS times.  Weights are still read once.
//
// Lane l loads the four plane words of column l (one 128-bit load per plane, as the lookup kernel
// does); a 4 x 4 transpose over (16-lane group, word) by v_permlane16_swap / v_permlane32_swap then
// gives lane l = c + 16 g word g (32 k) of column 16 cb + c for the four column blocks cb -- the
// plane operand.  As result the lane holds, for column 16 cb + c, the dot products of term g
// (register = segment).
#include <type_traits>

#include "hlq_gemv_common.h"

#ifndef HLQ_MX_DEBUG
#define HLQ_MX_DEBUG 0   // timing experiments -- 1: loads only (no MFMA work), 2: no reloads (compute only)
#endif

namespace {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef unsigned short ushort2_t __attribute__((ext_vector_type(2)));
typedef int int8v __attribute__((ext_vector_type(8)));
typedef unsigned int uint2v __attribute__((ext_vector_type(2)));
typedef float float4v __attribute__((ext_vector_type(4)));
// the scale block in LDS is written as 16-bit values and read back as 32-bit words
typedef uint16_t __attribute__((may_alias)) u16_alias;
typedef uint32_t __attribute__((may_alias)) u32_alias;

// Cuts the pair v to three significant bits (the high byte of each fp16 is a bf8 code: sign, exponent,
// two mantissa bits), stores the two codes at LDS bytes addr + 128 T and addr + 128 T + 4, returns
// the remainder (exact).  Each term strips at least three leading bits of the significand, so four
// terms hold all eleven bits of an fp16 value.
template <int T>
__device__ __forceinline__ half2_t put_term(uint32_t addr, half2_t v)
{
    const uint32_t u = __builtin_bit_cast(uint32_t, v);
    // after one shift the codes sit where the two byte stores read them (bits 7:0 and 23:16)
    const uint32_t sh = u >> 8;
    asm volatile("ds_write_b8 %0, %1 offset:%2\n\tds_write_b8_d16_hi %0, %1 offset:%3"
                 :: "v"(addr), "v"(sh), "n"(128 * T), "n"(128 * T + 4) : "memory");
    return v - __builtin_bit_cast(half2_t, u & 0xff00ff00u);
}

// max(v, v moved across lanes by DPP control CTRL); rows outside ROWMASK keep v
template <int CTRL, int ROWMASK = 0xf>
__device__ __forceinline__ uint32_t max_dpp(uint32_t v)
{
    const uint32_t moved = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, ROWMASK, 0xf, false);
    return max(v, moved);
}

template <int Q, int G, int NROW>
struct MxRegs {
    static constexpr int GS = G < 128 ? G : 128;
    static constexpr int SEG = 128 / GS;
    uint32_t w[Q][4];          // plane j: the four words (32 k each) of column l
    uint16_t mt[SEG][Q + 1];   // lane <-> column l of the tile
    uint32_t x[NROW];          // activations 2l, 2l+1 of the chunk, per activation row
};

// bytes per column of the transposed scale block in LDS (a multiple of 8)
constexpr int mx_meta_stride(int Q, int G) { return ((128 / (G < 128 ? G : 128)) * (Q + 1) * 2 + 7) & ~7; }
// activation rows a kernel instantiation handles: one (GEMV), or NS row sets of 4 / SEG rows
constexpr int mx_rows(int G, int NS, bool batched) { return batched ? NS * (4 / (128 / (G < 128 ? G : 128))) : 1; }
// per wavefront: activation codes (per row four terms x 128 bf8; then 16 zero bytes, padded to 64) |
// scales [64][stride] | sums [row][4][64] fp32
constexpr int mx_xt_bytes(int nrow) { return nrow * 512 + 64; }
constexpr int mx_wave_lds(int Q, int G, int nrow) { return mx_xt_bytes(nrow) + 64 * mx_meta_stride(Q, G) + nrow * 4 * 64 * 4; }
// Instantiations whose chunk loop ends in steps without reloads (several copies of the step: they cost
// registers).  The plain GEMV at one or two planes stays within 128 registers, i.e. two workgroups of
// eight wavefronts per CU; the others would lose a resident workgroup or spill, so they drop the loads
// past the end of a run through the range check of a buffer descriptor instead (measured a few per
// cent slower than the peeled loop where both are possible: a dropped load still takes its issue slot).
constexpr bool mx_peeled_tail(int Q, int G, int NR) { return NR == 0 && G >= 128 && Q <= 2; }
// Register sets of chunk loads per wavefront (chunks in flight + 1).  Two: launches of this kernel
// have thousands of wavefronts, which together keep far more than the bandwidth-delay product in
// flight; deeper prefetch only costs registers, i.e. resident wavefronts (measured: 2 beats 3, 4, 6, 8).
#ifdef HLQ_MX_NBUF
constexpr int mx_nbuf(int, int) { return HLQ_MX_NBUF; }
#else
constexpr int mx_nbuf(int, int) { return 2; }
#endif

// NR: activation rows the instantiation carries (0: the GEMV, one row per problem and no row stride);
// NR <= NS * (rows per set).  Fewer rows than the sets could hold means fewer loads, conversions and
// scale multiplications per chunk, so a launch picks the smallest instantiation that holds its M.
template <int Q, int G, int NS, int NR>
__global__ void __launch_bounds__(512)
hlq_gemv_mx_kernel(const int4v bb_lo, const int4v bb_hi, const int out_f32_flag, const GemvProbs probs)
{
    struct { int out_f32; } b = {out_f32_flag};
    constexpr bool BATCHED = NR > 0;
    constexpr int NROW = BATCHED ? NR : 1;
    static_assert(NROW <= mx_rows(G, NS, true), "more rows than the row sets hold");
    using Regs = MxRegs<Q, G, NROW>;
    constexpr int GS = Regs::GS, SEG = Regs::SEG;
    constexpr int RPS = 4 / SEG;   // activation rows one operand can carry
    constexpr int MSTR = mx_meta_stride(Q, G);
    constexpr int PERW = mx_wave_lds(Q, G, NROW);
    constexpr int NBUF = mx_nbuf(Q, G);
    const int W = (int)(blockDim.x >> 6);
    extern __shared__ __attribute__((aligned(256))) char lds[];

    const int pi = gemv_problem_of(bb_lo, bb_hi, (int)blockIdx.x);
    const GemvProb P = probs.p[pi];   // a copy: one burst of scalar loads
    int tg, slice;
    gemv_split_block(P, (int)blockIdx.x - P.blk_begin, tg, slice);

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int KW = P.kw, KSH = P.kw_shift, part = wave & (KW - 1);   // W and KW are powers of two
    const int tile = tg * (W >> KSH) + (wave >> KSH);
    const bool tile_ok = tile < P.ntiles;               // a surplus wavefront gets an empty run
    const int tile_c = tile_ok ? tile : P.ntiles - 1;
    // this wavefront's run of chunks: the slice is cut into KW near-equal parts
    // (the host plans every slice to start inside K; the clamp keeps every address formed below inside the
    // tile and inside x whatever the plan says)
    const int sbeg = min(slice * P.cps, P.nchunks - 1);
    const int send = min(sbeg + P.cps, P.nchunks);
    const int len = send - sbeg;
    const int cbeg = sbeg + ((len * part) >> KSH);
    const int cend = tile_ok ? sbeg + ((len * (part + 1)) >> KSH) : cbeg;

    const int tw = hlq_tile_width(tile_c, P.N);
    const char *tile_base = P.packed + (size_t)tile_c * HLQ_TILE_N * P.col_bytes;
    const int c = lane & 15, g = lane >> 4;
    // clamped column: loads stay in bounds, results of lanes past the tile's width are dropped
    uint32_t moff = (uint32_t)(lane < tw ? lane : tw - 1) * 2u;
    uint32_t woff = moff * 8u;   // this lane's 16 bytes inside a plane of a record
    uint32_t xoff = (uint32_t)lane * 4u;

    char *xt = lds + wave * PERW;                     // [row][term][128] bf8 in matrix-core k order, 16 zero bytes
    char *meta = xt + mx_xt_bytes(NROW);              // [column][SEG][Q+1] fp16
    float *red = (float *)(meta + 64 * MSTR);         // [row][4][64]
    constexpr int RSTR = PERW / 4;                    // floats between wavefronts' sums
    const int M = BATCHED ? P.M : 1;

    // Loads of one chunk, in two parts: the plane words (one 128-bit load per plane) and the rest (scales,
    // zero points, activations).  Two forms of the weight loads:
    //  * PEELED instantiations (their chunk loop ends in steps without loads): plain loads.  The lane
    //    offsets pass through an empty asm: they are re-extended to 64 bits at each use, which lets the
    //    loads take the form "scalar base + 32-bit lane offset" instead of one 64-bit vector add each.
    //  * the others, whose every step asks for "the chunk two ahead": loads through a buffer descriptor
    //    over this wavefront's part of the tile, [tile_base, first byte after the run's last record).
    //    The hardware's range check returns zero for anything beyond it without touching memory, so
    //    past the end of a run nothing is fetched -- no branch, no clamping.
    // Plane words are read exactly once per call: streaming (non-temporal) loads, which measurably
    // shorten the launch.  The 16-bit scale loads keep the default policy: a wavefront's 128-byte row
    // reaches the L2 as several requests.  The activations, shared by all workgroups, stay cached.
    constexpr bool PEELED = mx_peeled_tail(Q, G, NR);
    const uint32_t run_end = (!PEELED && tile_ok) ? hlq_rec_in_tile(tw, cend, Q, G) : 0u;
    const __amdgpu_buffer_rsrc_t wrsrc = __builtin_amdgcn_make_buffer_rsrc((void *)tile_base, 0, (int)run_end, 0x00020000);
    auto record_of = [&](int ch) -> const char * {
        return tile_base + hlq_rec_in_tile(tw, ch, Q, G);
    };
    auto load_chunk_plane = [&](int ch, Regs &R, int j) {
        int4v v;
        if constexpr (PEELED) {
            asm volatile("" : "+v"(woff));
            v = __builtin_nontemporal_load((const int4v *)(record_of(ch) + (size_t)(j * tw * 16) + woff));
        } else {
            // The record's offset goes into the per-lane offset, which the range check certainly covers;
            // only the position inside the record is a scalar offset.  A record that starts inside the
            // run lies inside it entirely, so the check on its start decides for all of its loads.
            const uint32_t vo = woff + hlq_rec_in_tile(tw, ch, Q, G);
            v = __builtin_bit_cast(int4v, __builtin_amdgcn_raw_buffer_load_b128(wrsrc, (int)vo, j * tw * 16, 2));   // aux 2: non-temporal
        }
        R.w[j][0] = v.x; R.w[j][1] = v.y; R.w[j][2] = v.z; R.w[j][3] = v.w;
    };
    auto load_chunk_rest = [&](int ch, Regs &R) {
        asm volatile("" : "+v"(moff), "+v"(xoff));
        // with G > 128 the group's scales sit in the record of its first (even) chunk
        const int cm = G > 128 ? (ch & ~1) : ch;
#pragma unroll
        for (int sg = 0; sg < SEG; ++sg)
#pragma unroll
            for (int r = 0; r <= Q; ++r) {
                if constexpr (PEELED) {
                    asm volatile("" : "+v"(moff));   // per load, or the compiler adds lane offset and base once, in vector registers
                    R.mt[sg][r] = *(const uint16_t *)(record_of(cm) + (size_t)tw * Q * 16 + (size_t)((sg * (Q + 1) + r) * tw * 2) + moff);
                } else {
                    const uint32_t vo = moff + hlq_rec_in_tile(tw, cm, Q, G);
                    R.mt[sg][r] = __builtin_amdgcn_raw_buffer_load_b16(wrsrc, (int)vo, tw * Q * 16 + (sg * (Q + 1) + r) * tw * 2, 0);
                }
            }
        // activations: plain loads; the chunk index stays inside the run (rows past M re-read the last row and are ignored)
        const int chx = PEELED ? ch : max(min(ch, cend - 1), sbeg);
#pragma unroll
        for (int m = 0; m < NROW; ++m)
            R.x[m] = *(const uint32_t *)((const char *)(P.x + (size_t)min(m, M - 1) * P.ldx + (size_t)chx * 128) + xoff);
    };
    auto load_chunk = [&](int ch, Regs &R) {
#pragma unroll
        for (int j = 0; j < Q; ++j) load_chunk_plane(ch, R, j);
        load_chunk_rest(ch, R);
    };

    // ---- scale: largest magnitude of the run's activations (as fp16 bit patterns) --------------------------
    // The activation loads go out BEFORE the weight loads: memory returns a wavefront's loads in
    // order, so the scale is known as soon as x is there, long before the first chunk.
    const int nrun = cend - cbeg;
    uint32_t xu[NROW][8];
#pragma unroll
    for (int m = 0; m < NROW; ++m) {
        const uint32_t *xr = (const uint32_t *)(P.x + (size_t)min(m, M - 1) * P.ldx + (size_t)cbeg * 128) + lane;
#pragma unroll
        for (int i = 0; i < 8; ++i)
            xu[m][i] = xr[(size_t)max(min(i, nrun - 1), 0) * 64];
    }

    // weight loads of the first chunks (an empty run re-reads the slice's first chunk and drops it, or
    // gets zeros from the range check)
    Regs R[NBUF];
#pragma unroll
    for (int i = 0; i < NBUF; ++i) load_chunk(PEELED ? max(min(cbeg + i, cend - 1), sbeg) : cbeg + i, R[i]);

    // with the first loads on their way: clear the operand area (rows past M are never converted, their
    // codes stay zero)
    for (int i = lane; i < mx_xt_bytes(NROW) / 4; i += 64) ((uint32_t *)xt)[i] = 0u;

    // per activation row: largest magnitude -> power-of-two scale.  Biased fp16 exponent e of the largest
    // magnitude: |x| < 2^(e-14); scaling by 2^(29-e) gives |x| < 2^15.  Plane codes are worth 1/2, 1, 2, 2
    // by register: lane weights 1/2, 1/4, 1/8, 1/8 make every product bit x activation / 4.  The factor
    // 2^(29-e) (<= 2^29) is applied as two fp16 multiplications.
    const int r_ = lane & 3;
    half2_t sw1[NROW], sw2[NROW];
    float yscale[NROW];
#pragma unroll
    for (int m = 0; m < NROW; ++m) {
        uint32_t mx = 0;
#pragma unroll
        for (int i = 0; i < 8; ++i)
            mx = __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(ushort2_t, mx),
                                                                        __builtin_bit_cast(ushort2_t, xu[m][i] & 0x7fff7fffu)));
        if (m < M)
            for (int ci = 8; ci < nrun; ++ci) {   // runs longer than eight chunks
                const uint32_t u = ((const uint32_t *)(P.x + (size_t)m * P.ldx + (size_t)(cbeg + ci) * 128))[lane] & 0x7fff7fffu;
                mx = __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(ushort2_t, mx), __builtin_bit_cast(ushort2_t, u)));
            }
        mx = max(mx & 0xffffu, mx >> 16);
        mx = max_dpp<0xB1>(mx);          // quad_perm [1,0,3,2]
        mx = max_dpp<0x4E>(mx);          // quad_perm [2,3,0,1]
        mx = max_dpp<0x124>(mx);         // row_ror:4
        mx = max_dpp<0x128>(mx);         // row_ror:8: every lane holds its row's maximum
        mx = max_dpp<0x142, 0xa>(mx);    // row_bcast15: rows 1, 3 take rows 0, 2 in
        mx = max_dpp<0x143, 0xc>(mx);    // row_bcast31: row 3 takes row 1 in
        const uint32_t top = (uint32_t)__builtin_amdgcn_readlane((int)mx, 63);
        const int e = (int)(top >> 10);
        const int k1 = (29 - e) / 2, k2 = (29 - e) - k1 - (r_ == 0 ? 1 : r_ == 1 ? 2 : 3);   // -4 <= k2 <= 14
        const _Float16 f1 = __builtin_bit_cast(_Float16, (uint16_t)((15 + k1) << 10));
        const _Float16 f2 = __builtin_bit_cast(_Float16, (uint16_t)((15 + k2) << 10));
        sw1[m] = (half2_t){f1, f1};
        sw2[m] = (half2_t){f2, f2};
        yscale[m] = __builtin_bit_cast(float, (uint32_t)(127 + 2 - 29 + e) << 23);   // 4 * 2^(e-29)
    }

    // ---- activation role: this lane converts x[2l], x[2l+1] of a chunk.  Weight k0 = 2 (l & 15) + h of
    // block g is plane bit (l & 15) + 16 h, i.e. register r = l & 3, nibble ((l >> 2) & 3) + 4 h of the
    // expanded word: matrix-core k index 32 g + 8 r + nibble.
    const uint32_t xt_wa = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)xt +
                           (uint32_t)(32 * g + 8 * r_ + ((lane >> 2) & 3));
    // ---- operand role: row (lane & 15) = 4 t + s of the activation operand, s = r * SEG + sg (activation
    // row r of the set, segment sg); 16-k runs [16 g, 16 g + 16) and [64 + 16 g, ...) of the chunk; a run
    // outside segment sg -- or a row the instantiation does not carry -- reads the zero bytes
    const int at = (lane & 15) >> 2, as = lane & 3;
    const char *a_src[NS][2];
#pragma unroll
    for (int set = 0; set < NS; ++set)
#pragma unroll
        for (int hh = 0; hh < 2; ++hh) {
            const int blk = 2 * hh + (g >> 1);       // 32-k block the run lies in
            const int r = as / SEG, sg = as % SEG;
            const bool on = set * RPS + r < NROW && (blk * 32) / GS == sg;
            a_src[set][hh] = xt + (on ? (set * RPS + r) * 512 + 128 * at + 64 * hh + 16 * g : NROW * 512);
        }

    float acc[NROW][4];
#pragma unroll
    for (int m = 0; m < NROW; ++m)
#pragma unroll
        for (int cb = 0; cb < 4; ++cb) acc[m][cb] = 0.f;
    const float4v zero4 = {0.f, 0.f, 0.f, 0.f};

    // Operands that come through LDS, fetched one chunk ahead: the activation operand and, per column
    // block, the scales of this lane's column (MSTR bytes, fp16).
    struct Pre {
        int8v A[NS];
        uint32_t m[4][MSTR / 4];
    };
    auto scale_of = [](const uint32_t (&m)[MSTR / 4], int i) -> float {   // i-th fp16 of a scale record
        const half2_t h = __builtin_bit_cast(half2_t, m[i >> 1]);
        return (float)((i & 1) ? h.y : h.x);
    };
    auto prefetch = [&](const Regs &Rn, Pre &pn) {
        // activations -> four bf8 terms (bytes = high bytes of fp16 values with three significant bits)
#pragma unroll
        for (int m = 0; m < NROW; ++m) {
            if (m >= M) break;
            half2_t v = (__builtin_bit_cast(half2_t, Rn.x[m]) * sw1[m]) * sw2[m];   // exact: powers of two, in range
            const uint32_t addr = xt_wa + (uint32_t)(m * 512);
            v = put_term<0>(addr, v);
            v = put_term<1>(addr, v);
            v = put_term<2>(addr, v);
            (void)put_term<3>(addr, v);
        }
        // scales: lane <-> column to LDS, read back per column block
#pragma unroll
        for (int sg = 0; sg < SEG; ++sg)
#pragma unroll
            for (int r = 0; r <= Q; ++r) ((u16_alias *)(meta + lane * MSTR))[sg * (Q + 1) + r] = Rn.mt[sg][r];
#pragma unroll
        for (int set = 0; set < NS; ++set) {
            const uint4 alo = *(const uint4 *)a_src[set][0];
            const uint4 ahi = *(const uint4 *)a_src[set][1];
            pn.A[set] = (int8v){(int)alo.x, (int)alo.y, (int)alo.z, (int)alo.w, (int)ahi.x, (int)ahi.y, (int)ahi.z, (int)ahi.w};
        }
#pragma unroll
        for (int cb = 0; cb < 4; ++cb)
#pragma unroll
            for (int i = 0; i < MSTR / 4; ++i) pn.m[cb][i] = ((const u32_alias *)(meta + (16 * cb + c) * MSTR))[i];
    };
    auto expand = [](uint32_t w) -> int8v {   // plane word -> 32 fp4 codes (bit 4p+r -> nibble p of register r)
        return (int8v){(int)(w & 0x11111111u), (int)(w & 0x22222222u), (int)(w & 0x44444444u),
                       (int)((w >> 1) & 0x44444444u), 0, 0, 0, 0};
    };

    // One chunk.  The matrix core takes ~32 cycles per MFMA and the wavefront issues in order, so the
    // step is written as a software pipeline: each stage issues the MFMA of item n (plane j of column
    // block cb), expands the plane word of item n+1 and applies the scales to the result of item
    // n-1; scheduling barriers keep the stages apart.  The LDS operands of the NEXT chunk are fetched
    // in the middle of the step.
    auto step = [&](auto reload_tag, Regs &R, const Pre &p, const Regs &Rn, Pre &pn, int ch_reload) {
        constexpr bool reload = decltype(reload_tag)::value;   // false: nothing left to load into this register set
        if (HLQ_MX_DEBUG == 1) {   // timing experiment: loads only
            uint32_t m = 0;
#pragma unroll
            for (int j = 0; j < Q; ++j) m ^= R.w[j][0] ^ R.w[j][1] ^ R.w[j][2] ^ R.w[j][3];
#pragma unroll
            for (int r = 0; r <= Q; ++r) m ^= R.mt[0][r];
            acc[0][0] += (float)m;
            if (reload) load_chunk(ch_reload, R);
            return;
        }
        constexpr int NI = 4 * Q;   // items; item n: plane n / 4, column block n % 4
        // result register s of an MFMA belongs to activation row s / SEG of the set and segment s % SEG
        auto apply = [&](int set, const float4v &d, int cb, int which) {
#pragma unroll
            for (int sl = 0; sl < 4; ++sl) {
                const int r = sl / SEG, sg = sl % SEG;
                if (set * RPS + r < NROW) acc[set * RPS + r][cb] += scale_of(p.m[cb], sg * (Q + 1) + which) * d[sl];
            }
        };
        // segment sums of x for the zero points: all-ones plane
        const int8v ones = {0x11111111, 0x22222222, 0x44444444, 0x44444444, 0, 0, 0, 0};
        float4v xs[NS];
#pragma unroll
        for (int set = 0; set < NS; ++set) xs[set] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(p.A[set], ones, zero4, 1, 4, 0, 0, 0, 0);
        // 4 x 4 transpose over (16-lane group, word): afterwards wt[j][cb] of lane (c, g) is word g of
        // column 16 cb + c
        uint32_t wt[Q][4];
#pragma unroll
        for (int j = 0; j < Q; ++j) {
            const uint2v s01 = __builtin_amdgcn_permlane16_swap(R.w[j][0], R.w[j][1], false, false);
            const uint2v s23 = __builtin_amdgcn_permlane16_swap(R.w[j][2], R.w[j][3], false, false);
            const uint2v t02 = __builtin_amdgcn_permlane32_swap(s01.x, s23.x, false, false);
            const uint2v t13 = __builtin_amdgcn_permlane32_swap(s01.y, s23.y, false, false);
            wt[j][0] = t02.x; wt[j][2] = t02.y; wt[j][1] = t13.x; wt[j][3] = t13.y;
        }
        // This register set's scales and activations were consumed one chunk ahead: refill them now.
        // The lane swaps above work in place, so a plane's registers hold its transposed words until its
        // four items are done; they are reloaded right then (one load per plane, spread over the step)
        // -- later than "as early as possible", but reloading everything here would cost a copy of
        // every word (the loads would need the registers the swapped words sit in).
        if (HLQ_MX_DEBUG != 2 && reload) load_chunk_rest(ch_reload, R);
        int8v B = expand(wt[0][0]);
        float4v d[NS][3];
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int n = 0; n < NI; ++n) {
#pragma unroll
            for (int set = 0; set < NS; ++set)
                d[set][n % 3] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(p.A[set], B, zero4, 1, 4, 0, 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            if (n + 1 < NI) B = expand(wt[(n + 1) / 4][(n + 1) % 4]);
            if ((n + 1) % 4 == 0 && HLQ_MX_DEBUG != 2 && reload) load_chunk_plane(ch_reload, R, n / 4);
            if (n >= 1) {
#pragma unroll
                for (int set = 0; set < NS; ++set) {
                    apply(set, d[set][(n - 1) % 3], (n - 1) % 4, (n - 1) / 4);
                    // keeps all four result registers allocated up to here: if the unused ones were handed
                    // to the next operand while the MFMA is in flight, every write to them would have to
                    // wait for it
                    asm volatile("" ::"v"(d[set][(n - 1) % 3]));
                }
            }
            if (n == 1) prefetch(Rn, pn);
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int set = 0; set < NS; ++set) {
            apply(set, d[set][(NI - 1) % 3], (NI - 1) % 4, (NI - 1) / 4);
#pragma unroll
            for (int cb = 0; cb < 4; ++cb) apply(set, xs[set], cb, Q);
        }
    };

    // ---- chunk loop: NBUF register sets, loads of the next NBUF-1 chunks in flight ----------------------
    Pre pre[2];
    if (cbeg < cend && HLQ_MX_DEBUG != 1) prefetch(R[0], pre[0]);
    static_assert(NBUF == 2, "the loops below alternate two register sets");
    const std::true_type more;
    const std::false_type last;
    if constexpr (PEELED) {
        // Steps whose register set has a further chunk to fetch reload it; the last two of a run do not.
        // The choice is made between steps, at compile time inside them: a branch around the loads inside
        // a step breaks its schedule and costs more than the loads it saves.
        int ch = cbeg;
        for (; ch + 3 < cend; ch += 2) {
            step(more, R[0], pre[0], R[1], pre[1], ch + 2);
            step(more, R[1], pre[1], R[0], pre[0], ch + 3);
        }
        const int left = cend - ch;   // 0 (empty run), 1, 2 or 3
        if (left == 3) {
            step(more, R[0], pre[0], R[1], pre[1], ch + 2);
            step(last, R[1], pre[1], R[0], pre[0], 0);
            step(last, R[0], pre[0], R[1], pre[1], 0);
        } else if (left == 2) {
            step(last, R[0], pre[0], R[1], pre[1], 0);
            step(last, R[1], pre[1], R[0], pre[0], 0);
        } else if (left == 1) {
            step(last, R[0], pre[0], R[1], pre[1], 0);
        }
    } else {
        // every step asks for the chunk NBUF ahead; past the end of the run the range check answers with zeros
        for (int ch = cbeg; ch < cend; ch += NBUF) {
#pragma unroll
            for (int i = 0; i < NBUF; ++i) {
                if (ch + i < cend) step(more, R[i], pre[i & 1], R[(i + 1) % NBUF], pre[(i + 1) & 1], ch + i + NBUF);
            }
        }
    }

    // ---- undo the run's scaling; add the four terms (lane groups) and the tile's KW runs ---------------------
#pragma unroll
    for (int m = 0; m < NROW; ++m)
#pragma unroll
        for (int cb = 0; cb < 4; ++cb) red[(m * 4 + cb) * 64 + lane] = acc[m][cb] * yscale[m];
    __syncthreads();
    if (part != 0 || !tile_ok) return;
    float y[NROW];
#pragma unroll
    for (int m = 0; m < NROW; ++m) {
        y[m] = 0.f;
        for (int w2 = 0; w2 < KW; ++w2)
#pragma unroll
            for (int g2 = 0; g2 < 4; ++g2) y[m] += red[w2 * RSTR + (m * 4 + (lane >> 4)) * 64 + (lane & 15) + 16 * g2];
    }
    const bool col_ok = lane < tw;
    const size_t n = (size_t)tile * HLQ_TILE_N + lane;
    const size_t ldy = BATCHED ? (size_t)P.ldy : 0;

    if (P.nslices == 1) {
#pragma unroll
        for (int m = 0; m < NROW; ++m)
            if (col_ok && m < M) store_out(P.y, m * ldy + n, y[m], b.out_f32);
        return;
    }
    // ---- split-K across workgroups: write-through partials [slice][row][N], arrival counter, last one adds
    // in slice order
    const size_t MN = (size_t)M * P.N;
#pragma unroll
    for (int m = 0; m < NROW; ++m)
        if (col_ok && m < M)
            __hip_atomic_store(&P.part[(size_t)slice * MN + (size_t)m * P.N + n], y[m], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    int old = 0;
    if (lane == 0) old = __hip_atomic_fetch_add(&P.cnt[tile], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    old = __builtin_amdgcn_readfirstlane(old);
    if (old != P.nslices - 1) return;
    if (col_ok) {
#pragma unroll
        for (int m = 0; m < NROW; ++m) {
            if (m >= M) break;
            const float *src = &P.part[(size_t)m * P.N + n];
            float a = 0.f;
            int sl = 0;
            for (; sl + 4 <= P.nslices; sl += 4) {
                const float v0 = __hip_atomic_load(src + (size_t)(sl + 0) * MN, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                const float v1 = __hip_atomic_load(src + (size_t)(sl + 1) * MN, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                const float v2 = __hip_atomic_load(src + (size_t)(sl + 2) * MN, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                const float v3 = __hip_atomic_load(src + (size_t)(sl + 3) * MN, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                a = (((a + v0) + v1) + v2) + v3;
            }
            for (; sl < P.nslices; ++sl) a += __hip_atomic_load(src + (size_t)sl * MN, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            store_out(P.y, m * ldy + n, a, b.out_f32);
        }
    }
    if (lane == 0) __hip_atomic_store(&P.cnt[tile], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

template <int Q, int G>
void launch_qg(const GemvBatch &b, unsigned nblocks, int W, int nsets, int rows, hipStream_t st)
{
    const dim3 blk(64 * W);
    const GemvKernelArgs a = gemv_kernel_args(b);
    constexpr int RPS = mx_rows(G, 1, true);   // rows per set
#define HLQ_MX_LAUNCH(NS_, NR_) \
    hlq_gemv_mx_kernel<Q, G, NS_, NR_><<<nblocks, blk, (size_t)W * mx_wave_lds(Q, G, (NR_) > 0 ? (NR_) : 1), st>>>(a.lo, a.hi, a.out_f32, a.probs)
    // the smallest instantiation that holds `rows` (rows <= nsets * RPS is checked by the caller)
    if (nsets == 0) {
        HLQ_MX_LAUNCH(1, 0);
    } else if (nsets == 1) {
        switch (rows < RPS ? rows : RPS) {
        case 1: HLQ_MX_LAUNCH(1, 1); break;
        case 2: HLQ_MX_LAUNCH(1, (RPS >= 2 ? 2 : RPS)); break;
        case 3: HLQ_MX_LAUNCH(1, (RPS >= 3 ? 3 : RPS)); break;
        default: HLQ_MX_LAUNCH(1, RPS); break;
        }
    } else {
        switch (rows < 2 * RPS ? rows - RPS : RPS) {   // rows of the second set
        case 1: HLQ_MX_LAUNCH(2, RPS + 1); break;
        case 2: HLQ_MX_LAUNCH(2, (RPS >= 2 ? RPS + 2 : 2 * RPS)); break;
        case 3: HLQ_MX_LAUNCH(2, (RPS >= 3 ? RPS + 3 : 2 * RPS)); break;
        default: HLQ_MX_LAUNCH(2, 2 * RPS); break;
        }
    }
#undef HLQ_MX_LAUNCH
}

template <int Q>
hlq_status launch_q(int G, const GemvBatch &b, unsigned nblocks, int W, int nsets, int rows, hipStream_t st)
{
    switch (G) {
    case 32: launch_qg<Q, 32>(b, nblocks, W, nsets, rows, st); return HLQ_OK;
    case 64: launch_qg<Q, 64>(b, nblocks, W, nsets, rows, st); return HLQ_OK;
    case 128: launch_qg<Q, 128>(b, nblocks, W, nsets, rows, st); return HLQ_OK;
    case 256: launch_qg<Q, 256>(b, nblocks, W, nsets, rows, st); return HLQ_OK;
    }
    return HLQ_ERR_UNSUPPORTED;
}

} // namespace

int hlq_gemv_mx_max_waves(int, int) { return 8; }
int hlq_gemv_mx_rows_per_set(int G) { return mx_rows(G, 1, true); }

// nsets: 0 = GEMV (one activation row per problem), 1 / 2 = batched rows with that many row sets
// (every problem's M must fit nsets * hlq_gemv_mx_rows_per_set(G)).
hlq_status hlq_launch_gemv_mx(const GemvBatch &b, unsigned nblocks, int W, int nsets, int rows, int q, int G, hipStream_t st)
{
    if (W < 1 || W > 8 || (W & (W - 1)) || nsets < 0 || nsets > 2) return HLQ_ERR_UNSUPPORTED;
    if (rows < 1 || rows > (nsets ? nsets : 1) * hlq_gemv_mx_rows_per_set(G)) return HLQ_ERR_UNSUPPORTED;
    switch (q) {
    case 1: return launch_q<1>(G, b, nblocks, W, nsets, rows, st);
    case 2: return launch_q<2>(G, b, nblocks, W, nsets, rows, st);
    case 3: return launch_q<3>(G, b, nblocks, W, nsets, rows, st);
    case 4: return launch_q<4>(G, b, nblocks, W, nsets, rows, st);
    }
    return HLQ_ERR_UNSUPPORTED;
}
