// Table-storage variants of the bit-serial LUT GEMV (App. D, "Mirror Storage" and "Table Quantization"),
// M = 1.  Same method as hlq_gemv.hip -- per chunk every wavefront builds its own 32 tables of four
// activations each in LDS, every 4-bit slice of every plane word looks its entry up, looked-up entries
// are added, s_j and z enter once per (plane, quant segment) -- with the table held in one of four ways:
//
//   FULL32    16 entries, fp32            the reference of this file (what hlq_gemv_kernel stores)
//   MIRROR32   8 entries, fp32            +-1 form: b^ = 2 b - 1, s^_j = s_j / 2, z^ = z + 1/2 sum_j s_j;
//                                         entry i < 8 = sum_r (+-) x_r with + where bit r of i is set and the
//                                         fourth activation always -, index i >= 8 reads entry 15 - i and
//                                         negates it.  Lossless (up to fp32 rounding order).
//   FULL16    16 entries, fp16            entries rounded to nearest even from the fp32 sums (the paper's
//                                         NEON tables); lossy.
//   FULL8     16 entries, int8            one fp32 scale per table, max|entry| / 127, entries rounded to the
//                                         nearest integer in [-127, 127]; lossy.
//
// This file is written for comparison, in plain HIP without the hand-scheduled lookup blocks of
// hlq_gemv_kernel: FULL32 here against FULL32 there shows what the hand scheduling is worth, the other
// three against FULL32 here show what the storage form is worth.  Work split, workspace protocol and
// launch plan are those of hlq_gemv_kernel with one tile per wavefront.
#include "hlq_gemv_common.h"

namespace {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));

enum { FULL32 = 0, MIRROR32 = 1, FULL16 = 2, FULL8 = 3 };

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

template <int Q, int G>
struct VRegs {
    static constexpr int GS = G < 128 ? G : 128;
    static constexpr int SEG = 128 / GS;
    uint32_t w[Q][4];
    uint16_t mt[SEG][Q + 1];
    uint4 x;   // this lane's 8-k activation window (table build)
};

constexpr int VAR_TABLE_BYTES = 2048;   // per wavefront, the largest form (32 tables x 16 fp32); the others use less

template <int Q, int G, int V>
__global__ void __launch_bounds__(512)
hlq_gemv_variant_kernel(const int4v bb_lo, const int4v bb_hi, const int out_f32_flag, const GemvProbs probs)
{
    using Regs = VRegs<Q, G>;
    constexpr int GS = Regs::GS, SEG = Regs::SEG, WPS = GS / 32;
    const int W = (int)(blockDim.x >> 6);
    extern __shared__ __attribute__((aligned(256))) float lds[];
    float *red = lds + W * (VAR_TABLE_BYTES / 4);

    const GemvProb P = probs.p[gemv_problem_of(bb_lo, bb_hi, (int)blockIdx.x)];
    int tg, slice;
    gemv_split_block(P, (int)blockIdx.x - P.blk_begin, tg, slice);
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int sbeg = min(slice * P.cps, P.nchunks - 1);
    const int send = min(sbeg + P.cps, P.nchunks);
    const int len = send - sbeg;
    const int cbeg = sbeg + (len * wave) / W;
    const int cend = sbeg + (len * (wave + 1)) / W;

    const int tile = tg;
    const int tw = hlq_tile_width(tile, P.N);
    const bool col_ok = lane < tw;
    const int lane_c = col_ok ? lane : tw - 1;
    const char *tile_base = P.packed + (size_t)tile * HLQ_TILE_N * P.col_bytes;

    // table-build role of this lane: 8-k window bw of the chunk, parity bp (even / odd k of the window: the table of
    // word bw / 4, 4-bit slice (bw & 3) + 4 bp), half bh of the table's entries
    const int bw = lane >> 2, bp = (lane >> 1) & 1, bh = lane & 1;
    const int bt = 8 * (bw >> 2) + (bw & 3) + 4 * bp;
    char *Tw = (char *)lds + wave * VAR_TABLE_BYTES;

    auto load_chunk = [&](int c, Regs &R) {
        const char *rec = tile_base + hlq_rec_in_tile(tw, c, Q, G);
#pragma unroll
        for (int j = 0; j < Q; ++j) {
            const uint4 v = *((const uint4 *)rec + (j * tw + lane_c));
            R.w[j][0] = v.x; R.w[j][1] = v.y; R.w[j][2] = v.z; R.w[j][3] = v.w;
        }
        const char *mrec = G > 128 ? tile_base + hlq_rec_in_tile(tw, c & ~1, Q, G) : rec;
        const uint16_t *m = (const uint16_t *)(mrec + (size_t)tw * Q * 16);
#pragma unroll
        for (int sg = 0; sg < SEG; ++sg)
#pragma unroll
            for (int r = 0; r <= Q; ++r) R.mt[sg][r] = m[(sg * (Q + 1) + r) * tw + lane_c];
        R.x = *(const uint4 *)(P.x + (size_t)c * 128 + 8 * bw);
    };

    // one looked-up entry of table t for index idx (0..15), as fp32
    auto lookup = [&](int t, uint32_t idx) -> float {
        if (V == FULL32) return *(const float *)(Tw + t * 64 + idx * 4);
        if (V == MIRROR32) {
            const bool hi = idx >= 8u;
            const float v = *(const float *)(Tw + t * 32 + (hi ? 15u - idx : idx) * 4);
            return hi ? -v : v;
        }
        if (V == FULL16) return (float)*(const _Float16 *)(Tw + t * 32 + idx * 2);
        return (float)*(const signed char *)(Tw + t * 16 + idx);   // FULL8: times the table's scale, applied by the caller
    };

    float acc = 0.f;
    auto step = [&](const Regs &R) {
        // ---- build: the lane's four activations x_r (fp32), then its half of the table's entries -----------------
        const uint32_t xd[4] = {R.x.x, R.x.y, R.x.z, R.x.w};
        float xv[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) xv[r] = (float)__builtin_bit_cast(_Float16, (uint16_t)(xd[r] >> (16 * bp)));
        if (V == MIRROR32) {
            // entries 4 bh .. 4 bh + 3 of the eight stored: index i has bit 2 = bh, bit 3 = 0 (x_3 enters with -)
            const float base = (bh ? xv[2] : -xv[2]) - xv[3];
            const float4 e = make_float4(base - xv[0] - xv[1], base + xv[0] - xv[1], base - xv[0] + xv[1], base + xv[0] + xv[1]);
            *(float4 *)(Tw + bt * 32 + bh * 16) = e;
        } else {
            // entries 8 bh .. 8 bh + 7 of the sixteen: index i has bit 3 = bh
            const float e0 = bh ? xv[3] : 0.f;
            const float e1 = e0 + xv[0], e2 = e0 + xv[1], e3 = e1 + xv[1];
            const float e[8] = {e0, e1, e2, e3, e0 + xv[2], e1 + xv[2], e2 + xv[2], e3 + xv[2]};
            if (V == FULL32) {
                float4 *dst = (float4 *)(Tw + bt * 64 + bh * 32);
                dst[0] = make_float4(e[0], e[1], e[2], e[3]);
                dst[1] = make_float4(e[4], e[5], e[6], e[7]);
            } else if (V == FULL16) {
                uint32_t pk[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const half2_t h = {(_Float16)e[2 * i], (_Float16)e[2 * i + 1]};   // round to nearest even
                    pk[i] = __builtin_bit_cast(uint32_t, h);
                }
                *(uint4 *)(Tw + bt * 32 + bh * 16) = make_uint4(pk[0], pk[1], pk[2], pk[3]);
            } else {
                // largest magnitude among all sixteen entries = the larger of the sum of the positive and of the
                // negative activations; both lanes of the table compute it from the same four values
                float pos = 0.f, neg = 0.f;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    pos += fmaxf(xv[r], 0.f);
                    neg -= fminf(xv[r], 0.f);
                }
                const float scale = fmaxf(pos, neg) / 127.0f;
                const float inv = scale > 0.f ? 1.0f / scale : 0.f;
                uint32_t pk[2] = {0u, 0u};
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const int qv = (int)fminf(fmaxf(rintf(e[i] * inv), -127.f), 127.f);
                    pk[i >> 2] |= (uint32_t)(qv & 0xff) << (8 * (i & 3));
                }
                *(uint2 *)(Tw + bt * 16 + bh * 8) = make_uint2(pk[0], pk[1]);
                if (bh == 0) *(float *)(Tw + 512 + bt * 4) = scale;
            }
        }
        // ---- sums of the segments' activations (exact fp32 dot products with (1, 1), DPP reduction) -----------------
        const half2_t ones = {(_Float16)1.0f, (_Float16)1.0f};
        float tot = 0.f;
#pragma unroll
        for (int r = 0; r < 4; ++r) tot = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, xd[r]), ones, tot, false);
        tot = add_dpp<0x124>(tot);
        tot = add_dpp<0x128>(tot);
        float xs[SEG];
        if (GS == 32) {
#pragma unroll
            for (int sg = 0; sg < SEG; ++sg) xs[sg] = lane_value(tot, 16 * sg);
        } else if (GS == 64) {
            tot = add_dpp<0x142, 0xa>(tot);
            xs[0] = lane_value(tot, 31);
            xs[SEG - 1] = lane_value(tot, 63);
        } else {
            tot = add_dpp<0x142, 0xa>(tot);
            tot = add_dpp<0x143, 0xc>(tot);
            xs[0] = lane_value(tot, 63);
        }
        // ---- lookups: per quant segment and plane the sum of the looked-up entries, then the scale ------------------
#pragma unroll
        for (int sg = 0; sg < SEG; ++sg) {
            float ssum = 0.f;
#pragma unroll
            for (int j = 0; j < Q; ++j) {
                float p = 0.f;
#pragma unroll
                for (int dd = 0; dd < WPS; ++dd) {
                    const int d = sg * WPS + dd;
                    const uint32_t w = R.w[j][d];
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        const int t = 8 * d + i;
                        const float v = lookup(t, (w >> (4 * i)) & 15u);
                        if (V == FULL8) p += v * *(const float *)(Tw + 512 + t * 4);   // the table's scale (same address in every lane)
                        else p += v;
                    }
                }
                const float sj = h2f(R.mt[sg][j]);
                if (V == MIRROR32) {
                    acc += (0.5f * sj) * p;
                    ssum += sj;
                } else {
                    acc += sj * p;
                }
            }
            const float z = h2f(R.mt[sg][Q]);
            acc += (V == MIRROR32 ? z + 0.5f * ssum : z) * xs[sg];
        }
    };

    if (cbeg < cend) {
        Regs R[2];
        load_chunk(cbeg, R[0]);
        load_chunk(min(cbeg + 1, cend - 1), R[1]);
        for (int c = cbeg; c < cend; c += 2) {
            step(R[0]);
            if (c + 2 < cend) load_chunk(c + 2, R[0]);
            if (c + 1 < cend) {
                step(R[1]);
                if (c + 3 < cend) load_chunk(c + 3, R[1]);
            }
        }
    }

    // ---- add the W wavefronts' K ranges, then the K slices of other workgroups (as in hlq_gemv_kernel) -------------
    if (wave > 0) red[(wave - 1) * 64 + lane] = acc;
    __syncthreads();
    if (wave > 0) return;
    for (int w2 = 1; w2 < W; ++w2) acc += red[(w2 - 1) * 64 + lane];
    const size_t n = (size_t)tile * HLQ_TILE_N + lane;
    if (P.nslices == 1) {
        if (col_ok) store_out(P.y, n, acc, out_f32_flag);
        return;
    }
    if (col_ok) __hip_atomic_store(&P.part[(size_t)slice * P.N + n], acc, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    int old = 0;
    if (lane == 0) old = __hip_atomic_fetch_add(&P.cnt[tg], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    old = __builtin_amdgcn_readfirstlane(old);
    if (old != P.nslices - 1) return;
    if (col_ok) {
        float a = 0.f;
        for (int sl = 0; sl < P.nslices; ++sl)
            a += __hip_atomic_load(&P.part[(size_t)sl * P.N + n], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        store_out(P.y, n, a, out_f32_flag);
    }
    if (lane == 0) __hip_atomic_store(&P.cnt[tg], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

template <int Q, int G>
void launch_qg(int variant, const GemvBatch &b, unsigned nblocks, int W, hipStream_t st)
{
    const dim3 blk(64 * W);
    const size_t lds = (size_t)W * VAR_TABLE_BYTES + (size_t)(W - 1) * 64 * 4;
    const GemvKernelArgs a = gemv_kernel_args(b);
    switch (variant) {
    case FULL32: hlq_gemv_variant_kernel<Q, G, FULL32><<<nblocks, blk, lds, st>>>(a.lo, a.hi, a.out_f32, a.probs); break;
    case MIRROR32: hlq_gemv_variant_kernel<Q, G, MIRROR32><<<nblocks, blk, lds, st>>>(a.lo, a.hi, a.out_f32, a.probs); break;
    case FULL16: hlq_gemv_variant_kernel<Q, G, FULL16><<<nblocks, blk, lds, st>>>(a.lo, a.hi, a.out_f32, a.probs); break;
    default: hlq_gemv_variant_kernel<Q, G, FULL8><<<nblocks, blk, lds, st>>>(a.lo, a.hi, a.out_f32, a.probs); break;
    }
}

template <int Q>
hlq_status launch_q(int G, int variant, const GemvBatch &b, unsigned nblocks, int W, hipStream_t st)
{
    switch (G) {
    case 32: launch_qg<Q, 32>(variant, b, nblocks, W, st); return HLQ_OK;
    case 64: launch_qg<Q, 64>(variant, b, nblocks, W, st); return HLQ_OK;
    case 128: launch_qg<Q, 128>(variant, b, nblocks, W, st); return HLQ_OK;
    case 256: launch_qg<Q, 256>(variant, b, nblocks, W, st); return HLQ_OK;
    }
    return HLQ_ERR_UNSUPPORTED;
}

} // namespace

// variant: 0 = 16 fp32 entries, 1 = mirror form (8 fp32 entries), 2 = 16 fp16 entries, 3 = 16 int8 entries + a scale
// per table.  The batch must be planned as for hlq_gemv_kernel with one tile per wavefront.
hlq_status hlq_launch_gemv_variant(int variant, const GemvBatch &b, unsigned nblocks, int W, int q, int G, hipStream_t st)
{
    if (variant < 0 || variant > 3 || W < 1 || W > 8) return HLQ_ERR_UNSUPPORTED;
    switch (q) {
    case 1: return launch_q<1>(G, variant, b, nblocks, W, st);
    case 2: return launch_q<2>(G, variant, b, nblocks, W, st);
    case 3: return launch_q<3>(G, variant, b, nblocks, W, st);
    case 4: return launch_q<4>(G, variant, b, nblocks, W, st);
    }
    return HLQ_ERR_UNSUPPORTED;
}
