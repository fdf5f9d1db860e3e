// hlq_lut_gemm, dense-contraction formulation for larger M (the alternative the batched rows of
// App. B allow once table construction no longer amortises: one table set per row costs
// M*q*K*N/4 lookup-adds, a matrix-core contraction costs M*K*N MACs at ~60x the rate).
//
//   Y[M,N] = X[M,K] @ W^,   W^ = sum_j s_j b_j + z   (Eq. 3 / Eq. 6)
//
// W^ is rebuilt tile by tile IN REGISTERS as fp16 and fed straight to v_mfma_f32_32x32x16_f16;
// it never goes through LDS or HBM.
//
// Work split.  A workgroup (4 wavefronts) owns 32*MW rows x 256 columns x a K slice; wavefront w
// owns column tile 4*blockIdx.x + w (lane <-> column, the same records the GEMV reads) and keeps
// MW x 2 accumulator tiles of 32x32.  The X tile of the current chunk (32*MW rows x 128 k) is
// staged in LDS once per workgroup, double-buffered, one barrier per chunk.  It gets there by
// global_load_lds_dwordx4: memory -> LDS without passing through registers, 16 bytes per lane,
// lane L of an instruction landing at (base in M0) + 16 L.  A staged row is 16 such units with no
// padding; unit u of row r sits at position u ^ (r & 7), which spreads the eight rows that one
// 128-bit fragment read touches per cycle over all banks.  Each lane picks the global address
// whose data belongs at its LDS position, so one instruction still reads four whole 256-byte rows.
//
// Rebuilding weights.  A lane holds, per plane, the 128 bits of its column for the chunk; in a
// 32-bit plane word bits p and p+16 are the adjacent weights k0 = 2p, 2p+1 of the word's 32-k
// block.  (w << t) & 0x20002000 isolates such a pair at bit 13 of the two 16-bit halves: read as
// packed fp16 that is (2^-7 * b[2p], 2^-7 * b[2p+1]); with mask 0x40004000 (bit 14) it is
// (2 * b, 2 * b).  One v_pk_fma_f16 per plane with the pre-scaled scale (s * 2^7 or s / 2) adds
// s_j * b_j for two weights; the chain starts from (z, z).  Cost: 8 shifts + 16 ANDs per word and
// plane, 16*q packed FMAs per word: about 2.3 VALU lane-ops per weight at q = 2.
// Range of this path: |s_j| < 512 (pre-scaling by 2^7 must stay finite in fp16) -- HLQ scales are
// weight magnitudes, orders of magnitude below that.  The kernel checks every scale and zero it
// loads; if one is outside, it raises a flag and the fp32 fallback launched behind it
// (hlq_gemm_safe.hip) computes the call again, so any finite fp16 parameters give a right result.
//
// Contraction order.  Register pair p of a word holds k0 = 2p, 2p+1, so registers 8ks .. 8ks+7
// hold the 16 consecutive k of k-step ks in natural order and every A fragment is one aligned
// 16-byte LDS read of the staged X tile.  A k-step of the MFMA takes 8 registers of a lane: 4
// for k-slots 0..7, 4 for slots 8..15.  The matrix core wants slots 0..7 in lanes 0..31 and slots
// 8..15 in lanes 32..63 for the SAME 32 columns; one v_permlane32_swap per register hands the
// upper k-slots of columns 0..31 to lanes 32..63 and the lower k-slots of columns 32..63 to
// lanes 0..31, giving the B operands of both 32-column halves of the tile.
#include "hlq_mfma_common.h"

namespace {

__device__ __forceinline__ void store_out(void *y, size_t idx, float v, int out_f32)
{
    if (out_f32) ((float *)y)[idx] = v;
    else ((_Float16 *)y)[idx] = (_Float16)v;   // round-to-nearest-even
}

constexpr int XROW = 128;   // halfs per staged X row: the 128 k of a chunk as 16 swizzled 16-byte units

// vmcnt(0) with the other counters left alone (expcnt 7, lgkmcnt 15)
constexpr int WAIT_VM0 = (7 << 4) | (15 << 8);

// 16 bytes per lane from global memory straight into LDS at lds_base + 16 * lane.  Issued as inline
// assembly so that the compiler's wait-count bookkeeping does not tie later LDS reads (of the other
// buffer) to it; completion is awaited explicitly (vmcnt) before the barrier that publishes the tile.
__device__ __forceinline__ void dma_16B_per_lane(const void *gptr, uint32_t lds_base)
{
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(gptr), "s"(lds_base) : "memory", "m0");
}

template <int Q, int G>
struct WRegs {
    static constexpr int GS = G < 128 ? G : 128;
    static constexpr int SEG = 128 / GS;
    uint32_t w[Q][4];
    uint32_t mt[SEG][Q + 1];   // fp16 bit patterns, one register each: a 16-bit load then needs no merge (and
                               // no wait for the load) before its first real use
};

// The work of one workgroup: column group bx (four 64-column tiles), K slice by, row block bz of one problem.
template <int Q, int G, int MW>
__device__ __forceinline__ void gemm_mfma_block(const char *__restrict__ packed, size_t col_bytes,
                                                const uint16_t *__restrict__ X, long ldx, int M, void *__restrict__ Y,
                                                long ldy, float *__restrict__ ws, int N, int ntiles, int nchunks, int cps,
                                                int nslices, int out_f32, int bx, int by, int bz, int *range_flag)
{
    using Regs = WRegs<Q, G>;
    constexpr int GS = Regs::GS, SEG = Regs::SEG;
    constexpr int ROWS = 32 * MW;
    extern __shared__ __attribute__((aligned(16))) _Float16 Xs[];   // [2][ROWS][XROW]

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int tile = bx * 4 + wave;
    const int tile_c = tile < ntiles ? tile : ntiles - 1;          // clamped: loads stay in bounds
    const int tw = hlq_tile_width(tile_c, N);
    const bool col_ok = tile < ntiles && lane < tw;
    const int lane_c = lane < tw ? lane : tw - 1;
    const char *tile_base = packed + (size_t)tile_c * HLQ_TILE_N * col_bytes;
    const int m0 = bz * ROWS;
    const int cbeg = by * cps;
    const int cend = min(cbeg + cps, nchunks);

    auto load_w = [&](int c, Regs &R) {
        const char *rec = tile_base + hlq_rec_in_tile(tw, c, Q, G);
#pragma unroll
        for (int j = 0; j < Q; ++j) {
            const uint4 v = ((const uint4 *)rec)[j * tw + lane_c];
            R.w[j][0] = v.x; R.w[j][1] = v.y; R.w[j][2] = v.z; R.w[j][3] = v.w;
        }
        const char *mrec = rec;
        if (G > 128) {
            const int c0 = c & ~1;
            mrec = tile_base + hlq_rec_in_tile(tw, c0, Q, G);
        }
        const uint16_t *m = (const uint16_t *)(mrec + (size_t)tw * Q * 16);
#pragma unroll
        for (int sg = 0; sg < SEG; ++sg)
#pragma unroll
            for (int r = 0; r <= Q; ++r) R.mt[sg][r] = m[(sg * (Q + 1) + r) * tw + lane_c];
    };

    // X staging: wavefront w fills rows [w ROWS/4, (w+1) ROWS/4) of the tile, four rows per instruction;
    // lane L writes position L & 15 of row 4 i + (L >> 4), i.e. it fetches unit (L & 15) ^ (row & 7).
    // Rows past M re-read row M - 1: they only feed accumulator rows that are never stored.
    constexpr int RPW = ROWS / 4, NDMA = RPW / 4;
    const _Float16 *xsrc[NDMA];
#pragma unroll
    for (int i = 0; i < NDMA; ++i) {
        const int row = wave * RPW + 4 * i + (lane >> 4);
        const int u = (lane & 15) ^ (row & 7);
        const int m = min(m0 + row, M - 1);
        xsrc[i] = (const _Float16 *)X + (size_t)m * ldx + u * 8;
    }
    // LDS byte address of this wavefront's rows in buffer 0 (wave-uniform: it goes to M0)
    const uint32_t lds_wave = (uint32_t)__builtin_amdgcn_readfirstlane(
        (int)(uint32_t)(uintptr_t)(__attribute__((address_space(3))) _Float16 *)(Xs + (size_t)wave * RPW * XROW));
    auto dma_x = [&](int c, int buf) {
#pragma unroll
        for (int i = 0; i < NDMA; ++i)
            dma_16B_per_lane(xsrc[i] + (size_t)c * 128, lds_wave + (uint32_t)((buf * ROWS + 4 * i) * XROW * 2));
    };

    float16v acc[MW][2];
#pragma unroll
    for (int mb = 0; mb < MW; ++mb)
#pragma unroll
        for (int cb = 0; cb < 2; ++cb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mb][cb][r] = 0.f;

    // A fragments: lane l reads row l & 31 of a row block, logical unit 4 d + 2 ks + (l >> 5), stored at
    // that number ^ (l & 7): four per-lane origins cover the low bits, bit 3 is an immediate offset
    const _Float16 *xrow[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) xrow[k] = Xs + (size_t)(lane & 31) * XROW + (((2 * k) | (lane >> 5)) ^ (lane & 7)) * 8;

    // One chunk = 8 MW steps; step s = ((word d, k-step ks), row block mb) issues the two MFMAs of row
    // block mb against the two 32-column halves of the tile.  The wavefront issues in order and an
    // MFMA occupies the matrix core for 32 cycles (and the vector issue port for about 8; up to six
    // plain vector instructions per MFMA issue for free), so everything else is spread between the
    // MFMAs as side work of a step,
    // one stage ahead of its use (scheduling barriers keep the stages apart):
    //   - the A fragment of step s + 1 (one 128-bit LDS read) is requested before the MFMAs of step s;
    //   - the 16 weight pairs of word d + 1 are rebuilt 16 / (2 MW) per step during word d;
    //   - the four lane exchanges that form the B operands of the next k-step are spread over the MW
    //     steps of the current one.
    // largest magnitude (as an fp16 bit pattern) among the scales and zeros this lane has used: the rebuild below is
    // only valid while s * 2^7 and the partial sums of z + sum s_j b_j stay finite in fp16
    uint32_t meta_max = 0;
    auto compute = [&](const Regs &R, int buf) {
#pragma unroll
        for (int sg = 0; sg < SEG; ++sg)
#pragma unroll
            for (int r = 0; r <= Q; ++r) meta_max = max(meta_max, R.mt[sg][r] & 0x7fffu);
        const size_t xb = (size_t)buf * ROWS * XROW;
        constexpr int STEPS = 8 * MW, SPW = 2 * MW, PPS = 16 / SPW, XPS = (4 + MW - 1) / MW;
        auto frag = [&](int s) -> half8v {
            const int mb = s % MW, ks = (s / MW) & 1, d = s / SPW;
            return *(const half8v *)(xrow[(d & 1) * 2 + ks] + xb + (size_t)mb * 32 * XROW + (d >> 1) * 64);
        };
        uint32_t wp[2][16];   // rebuilt pairs of the current / next word: wp[d & 1][p] = k 32d + 2p, 2p + 1
        HlqSegScales<Q> sc;
        uint32_t wd[Q];
        auto word_setup = [&](int d) {
            sc.set(R.mt[(d * 32) / GS]);
#pragma unroll
            for (int j = 0; j < Q; ++j) wd[j] = R.w[j][d];
        };
        // B operands of a k-step: after the exchange lo = columns 0..31 of the tile (lanes 0..31 hold
        // k-slots 0..7, lanes 32..63 slots 8..15), hi = columns 32..63
        uint4v lo_c, hi_c, lo_n, hi_n;
        auto exchange = [&](int d, int ks, int v, uint4v &lo, uint4v &hi) {
            const uint2v r = __builtin_amdgcn_permlane32_swap(wp[d & 1][ks * 8 + v], wp[d & 1][ks * 8 + 4 + v], false, false);
            lo[v] = r.x;
            hi[v] = r.y;
        };
        // prologue: word 0 in full, operands of its first k-step, first fragment
        word_setup(0);
#pragma unroll
        for (int p = 0; p < 16; ++p) wp[0][p] = hlq_rebuild_pair<Q>(wd, sc, p);
#pragma unroll
        for (int v = 0; v < 4; ++v) exchange(0, 0, v, lo_c, hi_c);
        half8v a_cur = frag(0);
        word_setup(1);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int s = 0; s < STEPS; ++s) {
            const int mb = s % MW, ks = (s / MW) & 1, d = s / SPW, i = s % SPW;
            const half8v a_nxt = frag(s + 1 < STEPS ? s + 1 : s);
            acc[mb][0] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a_cur, __builtin_bit_cast(half8v, lo_c), acc[mb][0], 0, 0, 0);
            acc[mb][1] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a_cur, __builtin_bit_cast(half8v, hi_c), acc[mb][1], 0, 0, 0);
            a_cur = a_nxt;
            __builtin_amdgcn_sched_barrier(0);
            if (d < 3) {
#pragma unroll
                for (int p = i * PPS; p < (i + 1) * PPS; ++p) wp[(d + 1) & 1][p] = hlq_rebuild_pair<Q>(wd, sc, p);
            }
            // operands of the next k-step: (d, 1) during (d, 0), (d + 1, 0) during (d, 1)
            const int nd = ks == 0 ? d : d + 1, nks = ks ^ 1;
            if (nd < 4) {
#pragma unroll
                for (int v = mb * XPS; v < (mb + 1) * XPS && v < 4; ++v) exchange(nd, nks, v, lo_n, hi_n);
            }
            if (mb == MW - 1) {
                lo_c = lo_n;
                hi_c = hi_n;
                if (i == SPW - 1 && d + 2 < 4) word_setup(d + 2);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // ---- chunk loop: weights (registers) and X (LDS) of chunk c + 2 are requested right after the barrier
    //      that ends chunk c and have the whole of chunk c + 1 to arrive ------------------------------------
    if (cbeg < cend) {
        Regs RA, RB;
        load_w(cbeg, RA);
        load_w(min(cbeg + 1, cend - 1), RB);
        dma_x(cbeg, 0);
        if (cbeg + 1 < cend) dma_x(cbeg + 1, 1);
        __builtin_amdgcn_s_waitcnt(WAIT_VM0);
        __syncthreads();
        for (int c = cbeg; c < cend; c += 2) {
            compute(RA, 0);
            __builtin_amdgcn_s_waitcnt(WAIT_VM0);   // own share of chunk c + 1 has landed
            __syncthreads();                        // everyone's has; buffer 0 is free
            if (c + 2 < cend) {
                load_w(c + 2, RA);
                dma_x(c + 2, 0);
            }
            if (c + 1 < cend) {
                compute(RB, 1);
                __builtin_amdgcn_s_waitcnt(WAIT_VM0);
                __syncthreads();
                if (c + 3 < cend) {
                    load_w(c + 3, RB);
                    dma_x(c + 3, 1);
                }
            }
        }
    }

    // a scale of magnitude >= 512 (or a zero that large, or a non-finite value): raise the flag that makes the fallback
    // kernel behind this launch compute the call again in fp32
    if (__builtin_amdgcn_ballot_w64(meta_max >= 0x6000u) != 0 && lane == 0)
        __hip_atomic_store(range_flag, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    // ---- store: D tile register r of lane l is row 8*(r/4) + 4*(l/32) + r%4, column l%32 ----------------
    if (tile >= ntiles) return;
    const int rbase = m0 + 4 * (lane >> 5);
    const bool rows_full = m0 + ROWS <= M;
    auto store_tiles = [&](auto *dst, long rstride) {   // dst points at (row rbase, column 0 of the tile)
#pragma unroll
        for (int cb = 0; cb < 2; ++cb) {
            const int col_in_tile = cb * 32 + (lane & 31);
            if (col_in_tile >= tw) continue;
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) {
                auto *p = dst + col_in_tile + (long)rr * rstride;
#pragma unroll
                for (int blk = 0; blk < 4 * MW; ++blk) {   // rows rbase + rr + 8*blk
                    const float v = acc[blk >> 2][cb][(blk & 3) * 4 + rr];
                    if (rows_full || rbase + rr + 8 * blk < M) *p = (decltype(*p + 0))v;
                    p += 8 * rstride;
                }
            }
        }
    };
    const size_t n0 = (size_t)tile * HLQ_TILE_N;
    if (nslices > 1) store_tiles(ws + ((size_t)by * M + rbase) * (size_t)N + n0, (long)N);
    else if (out_f32) store_tiles((float *)Y + (size_t)rbase * ldy + n0, ldy);
    else store_tiles((_Float16 *)Y + (size_t)rbase * ldy + n0, ldy);
    (void)col_ok;
}


template <int Q, int G, int MW>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2)))
hlq_gemm_mfma_kernel(const char *__restrict__ packed, size_t col_bytes, const uint16_t *__restrict__ X, long ldx,
                     int M, void *__restrict__ Y, long ldy, float *__restrict__ ws, int N, int ntiles, int nchunks,
                     int cps, int nslices, int out_f32, int *range_flag)
{
    gemm_mfma_block<Q, G, MW>(packed, col_bytes, X, ldx, M, Y, ldy, ws, N, ntiles, nchunks, cps, nslices, out_f32,
                              (int)blockIdx.x, (int)blockIdx.y, (int)blockIdx.z, range_flag);
}

// Several problems with the same q, G and M in one launch (hlq_lut_gemm_batch): workgroups are numbered
// problem by problem, long-K problems first; inside a problem the column group runs fastest, then
// the K slice, then the row block.  The table of first blocks arrives in preloaded scalar
// registers, as in the GEMV kernel.  Problems whose K is split leave fp32 partial sums that
// hlq_gemm_mfma_group_reduce_kernel adds, again in one launch for all of them.
struct GemmProb {
    const char *packed;
    size_t col_bytes;
    const uint16_t *X;
    long ldx;
    void *Y;
    long ldy;
    float *part;         // [nslices][M][N] partial sums (nslices > 1)
    int N, ntiles, nchunks, colgroups, blk_begin, cps, nslices;
    unsigned cg_magic;   // ceil(2^32 / colgroups): local / colgroups = umulhi(local, cg_magic)
    unsigned ns_magic;   // the same for nslices
};
struct GemmProbs {
    GemmProb p[HLQ_MAX_BATCH];
};
typedef int int4v __attribute__((ext_vector_type(4)));

// index of the problem that owns block `blk`: the table is ascending, unused entries INT_MAX
__device__ __forceinline__ int group_problem_of(const int4v &bb_lo, const int4v &bb_hi, int blk)
{
    return blk >= bb_hi.w ? 7 : blk >= bb_hi.z ? 6 : blk >= bb_hi.y ? 5 : blk >= bb_hi.x ? 4
         : blk >= bb_lo.w ? 3 : blk >= bb_lo.z ? 2 : blk >= bb_lo.y ? 1 : 0;
}

template <int Q, int G, int MW>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2)))
hlq_gemm_mfma_group_kernel(const int4v bb_lo, const int4v bb_hi, const int M, const int out_f32, int *range_flag,
                           const GemmProbs probs)
{
    const int blk = (int)blockIdx.x;
    const GemmProb P = probs.p[group_problem_of(bb_lo, bb_hi, blk)];
    const int local = blk - P.blk_begin;
    const int t = P.colgroups > 1 ? (int)__umulhi((unsigned)local, P.cg_magic) : local;
    const int cg = local - t * P.colgroups;
    const int rb = P.nslices > 1 ? (int)__umulhi((unsigned)t, P.ns_magic) : t;
    const int sl = t - rb * P.nslices;
    gemm_mfma_block<Q, G, MW>(P.packed, P.col_bytes, P.X, P.ldx, M, P.Y, P.ldy, P.part, P.N, P.ntiles, P.nchunks,
                              P.cps, P.nslices, out_f32, cg, sl, rb, range_flag);
}

// adds the partial sums of all problems of a grouped launch whose K was split; 256 outputs per block
struct GemmRedProb {
    const float *part;
    void *Y;
    long ldy;
    int N, nslices, blk_begin;
};
struct GemmRedProbs {
    GemmRedProb p[HLQ_MAX_BATCH];
};

__global__ void __launch_bounds__(256)
hlq_gemm_mfma_group_reduce_kernel(const int4v bb_lo, const int4v bb_hi, const int M, const int out_f32,
                                  const GemmRedProbs probs)
{
    const int blk = (int)blockIdx.x;
    const GemmRedProb P = probs.p[group_problem_of(bb_lo, bb_hi, blk)];
    const size_t i = (size_t)(blk - P.blk_begin) * 256 + threadIdx.x;
    const size_t total = (size_t)M * P.N;
    if (i >= total) return;
    float a = 0.f;
    for (int s = 0; s < P.nslices; ++s) a += P.part[(size_t)s * total + i];
    const size_t m = i / P.N, n = i % P.N;
    store_out(P.Y, m * P.ldy + n, a, out_f32);
}

__global__ void __launch_bounds__(256)
hlq_gemm_mfma_reduce_kernel(const float *__restrict__ ws, void *__restrict__ Y, long ldy, int M, int N,
                            int nslices, int out_f32)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    const size_t total = (size_t)M * N;
    if (i >= total) return;
    float a = 0.f;
    for (int s = 0; s < nslices; ++s) a += ws[(size_t)s * total + i];
    const size_t m = i / N, n = i % N;
    store_out(Y, m * ldy + n, a, out_f32);
}

struct MfmaPlan {
    int MW, cps, nslices, rowblocks;
};

// K split.  A workgroup takes cps chunks; nslices = ceil(nchunks / cps) slices leave fp32 partials that
// a second kernel adds.  The choice minimises a small cost model fitted to measurements on MI355X
// (M = 16 .. 2048, the 8B layer shapes): a chunk costs a workgroup t1 when it has its CU to itself
// and t2 = 1.65 t1 when two workgroups share the CU (two per CU is the occupancy limit), workgroups
// run in rounds of 512, and the reduction costs a launch plus reading the partials back.
MfmaPlan plan_mfma(const HlqDims &dm, int64_t M)
{
    MfmaPlan p;
    p.MW = M > 64 ? 4 : (M > 32 ? 2 : 1);
    p.rowblocks = (int)((M + 32 * p.MW - 1) / (32 * p.MW));
    const long colgroups = (dm.ntiles + 3) / 4;
    const long wgs = colgroups * p.rowblocks;
    // us per chunk and workgroup: rebuilding the weights (per plane) + MFMAs and fragment reads (per row block)
    const double t1 = 0.275 * dm.q + 0.5 * p.MW, t2 = 1.65 * t1;
    const double mn = (double)M * (double)dm.N;
    double best = 0.0;
    const int top = (dm.nchunks + 1) & ~1;   // cps is even: the chunk loop alternates two register sets
    p.cps = top;
    p.nslices = 1;
    for (int cps = top;; cps -= 2) {
        const int ns = (dm.nchunks + cps - 1) / cps;
        const long total = wgs * ns;
        const long full = total / 512, rem = total % 512;
        double t = cps * (full * t2 + (rem == 0 ? 0.0 : (rem <= 256 ? t1 : t2)));
        if (ns > 1) t += 5.0 + ns * mn * 4.0 / 4.0e6;
        if (best == 0.0 || t < best) {
            best = t;
            p.cps = cps;
            p.nslices = ns;
        }
        if (cps - 2 < 2) break;
    }
    return p;
}

template <int Q, int G, int MW>
void launch_one(const HlqDims &dm, const MfmaPlan &p, const char *packed, const uint16_t *X, long ldx, int M,
                void *Y, long ldy, float *ws, int out_f32, hipStream_t st)
{
    const dim3 grid((unsigned)((dm.ntiles + 3) / 4), (unsigned)p.nslices, (unsigned)p.rowblocks);
    const size_t lds = (size_t)2 * 32 * MW * XROW * sizeof(_Float16);
    // ws points at the partial sums, which follow the counter block
    int *range_flag = hlq_ws_range_flag((char *)ws - HLQ_WS_COUNTER_BYTES);
    hlq_gemm_mfma_kernel<Q, G, MW><<<grid, 256, lds, st>>>(packed, dm.col_bytes, X, ldx, M, Y, ldy, ws, dm.N, dm.ntiles,
                                                          dm.nchunks, p.cps, p.nslices, out_f32, range_flag);
}

template <int Q, int G>
void launch_qg(const HlqDims &dm, const MfmaPlan &p, const char *packed, const uint16_t *X, long ldx, int M,
               void *Y, long ldy, float *ws, int out_f32, hipStream_t st)
{
    switch (p.MW) {
    case 1: launch_one<Q, G, 1>(dm, p, packed, X, ldx, M, Y, ldy, ws, out_f32, st); break;
    case 2: launch_one<Q, G, 2>(dm, p, packed, X, ldx, M, Y, ldy, ws, out_f32, st); break;
    default: launch_one<Q, G, 4>(dm, p, packed, X, ldx, M, Y, ldy, ws, out_f32, st); break;
    }
}

template <int Q>
hlq_status launch_q(const HlqDims &dm, const MfmaPlan &p, const char *packed, const uint16_t *X, long ldx, int M,
                    void *Y, long ldy, float *ws, int out_f32, hipStream_t st)
{
    switch (dm.G) {
    case 32: launch_qg<Q, 32>(dm, p, packed, X, ldx, M, Y, ldy, ws, out_f32, st); return HLQ_OK;
    case 64: launch_qg<Q, 64>(dm, p, packed, X, ldx, M, Y, ldy, ws, out_f32, st); return HLQ_OK;
    case 128: launch_qg<Q, 128>(dm, p, packed, X, ldx, M, Y, ldy, ws, out_f32, st); return HLQ_OK;
    case 256: launch_qg<Q, 256>(dm, p, packed, X, ldx, M, Y, ldy, ws, out_f32, st); return HLQ_OK;
    }
    return HLQ_ERR_UNSUPPORTED;
}

template <int Q, int G>
void launch_group_qg(int MW, unsigned nblocks, const int4v &lo, const int4v &hi, int M, int out_f32, int *flag,
                     const GemmProbs &pr, hipStream_t st)
{
    const size_t lds = (size_t)2 * 32 * MW * XROW * sizeof(_Float16);
    switch (MW) {
    case 1: hlq_gemm_mfma_group_kernel<Q, G, 1><<<nblocks, 256, lds, st>>>(lo, hi, M, out_f32, flag, pr); break;
    case 2: hlq_gemm_mfma_group_kernel<Q, G, 2><<<nblocks, 256, lds, st>>>(lo, hi, M, out_f32, flag, pr); break;
    default: hlq_gemm_mfma_group_kernel<Q, G, 4><<<nblocks, 256, lds, st>>>(lo, hi, M, out_f32, flag, pr); break;
    }
}

template <int Q>
hlq_status launch_group_q(int G, int MW, unsigned nblocks, const int4v &lo, const int4v &hi, int M, int out_f32,
                          int *flag, const GemmProbs &pr, hipStream_t st)
{
    switch (G) {
    case 32: launch_group_qg<Q, 32>(MW, nblocks, lo, hi, M, out_f32, flag, pr, st); return HLQ_OK;
    case 64: launch_group_qg<Q, 64>(MW, nblocks, lo, hi, M, out_f32, flag, pr, st); return HLQ_OK;
    case 128: launch_group_qg<Q, 128>(MW, nblocks, lo, hi, M, out_f32, flag, pr, st); return HLQ_OK;
    case 256: launch_group_qg<Q, 256>(MW, nblocks, lo, hi, M, out_f32, flag, pr, st); return HLQ_OK;
    }
    return HLQ_ERR_UNSUPPORTED;
}

} // namespace

size_t hlq_gemm_mfma_partial_bytes(const HlqDims &dm, int64_t M)
{
    const MfmaPlan p = plan_mfma(dm, M);
    return p.nslices > 1 ? (size_t)p.nslices * (size_t)M * (size_t)dm.N * sizeof(float) : 0;
}

hlq_status hlq_launch_gemm_mfma(const HlqDims &dm, const void *packed, const uint16_t *X, int64_t M, int64_t ldx,
                                void *Y, int64_t ldy, hlq_out_dtype out, void *ws, hipStream_t st)
{
    hlq_clear_stale_error();
    const MfmaPlan p = plan_mfma(dm, M);
    if (p.rowblocks > 65535) return HLQ_ERR_UNSUPPORTED;
    const int out_f32 = out == HLQ_OUT_F32;
    float *part = (float *)((char *)ws + HLQ_WS_COUNTER_BYTES);
    hlq_status s;
    switch (dm.q) {
    case 1: s = launch_q<1>(dm, p, (const char *)packed, X, (long)ldx, (int)M, Y, (long)ldy, part, out_f32, st); break;
    case 2: s = launch_q<2>(dm, p, (const char *)packed, X, (long)ldx, (int)M, Y, (long)ldy, part, out_f32, st); break;
    case 3: s = launch_q<3>(dm, p, (const char *)packed, X, (long)ldx, (int)M, Y, (long)ldy, part, out_f32, st); break;
    case 4: s = launch_q<4>(dm, p, (const char *)packed, X, (long)ldx, (int)M, Y, (long)ldy, part, out_f32, st); break;
    default: return HLQ_ERR_UNSUPPORTED;
    }
    if (s != HLQ_OK) return s;
    if (p.nslices > 1) {
        const size_t total = (size_t)M * dm.N;
        hlq_gemm_mfma_reduce_kernel<<<(unsigned)((total + 255) / 256), 256, 0, st>>>(part, Y, (long)ldy, (int)M, dm.N,
                                                                                    p.nslices, out_f32);
    }
    // behind it, the fp32 fallback for weights outside the range of the fp16 rebuild (a no-op unless the flag went up)
    HlqGemvItem it;
    it.dm = dm;
    it.packed = packed;
    it.x = X;
    it.y = Y;
    it.ldx = (long)ldx;
    it.ldy = (long)ldy;
    s = hlq_launch_gemm_safe(1, &it, M, out, ws, st);
    if (s != HLQ_OK) return s;
    return hlq_hip_status(hipGetLastError());
}

// Work split of a grouped launch.  Every problem is cut along K into slices of about the same number of
// chunks, chosen so that the launch has about 512 workgroups (one round at two workgroups per CU);
// with many rows nothing is cut.  Used by the launch and by the workspace size.
struct GroupPlan {
    int MW;
    long rowblocks;
    int cps[HLQ_MAX_BATCH], nslices[HLQ_MAX_BATCH];
};

static GroupPlan plan_group(int count, const HlqDims *dms, int64_t M)
{
    GroupPlan g;
    g.MW = M > 64 ? 4 : (M > 32 ? 2 : 1);
    g.rowblocks = (long)((M + 32 * g.MW - 1) / (32 * g.MW));
    double units = 0.0;   // workgroup-chunks of the whole launch
    for (int i = 0; i < count; ++i) units += (double)((dms[i].ntiles + 3) / 4) * g.rowblocks * dms[i].nchunks;
    long target = (long)(units / 512.0 + 0.999);
    if (target < 2) target = 2;
    for (int i = 0; i < count; ++i) {
        int ns = (int)((dms[i].nchunks + target - 1) / target);
        if (ns < 1) ns = 1;
        int cps = (dms[i].nchunks + ns - 1) / ns;
        cps = (cps + 1) & ~1;   // the chunk loop alternates two register sets
        g.cps[i] = cps;
        g.nslices[i] = (dms[i].nchunks + cps - 1) / cps;
    }
    return g;
}

size_t hlq_gemm_mfma_batch_partial_bytes(int count, const HlqDims *dms, int64_t M)
{
    if (count < 2 || M < 1) return 0;
    const GroupPlan g = plan_group(count, dms, M);
    size_t b = 0;
    for (int i = 0; i < count; ++i)
        if (g.nslices[i] > 1) b += (size_t)g.nslices[i] * (size_t)M * (size_t)dms[i].N * sizeof(float);
    return b;
}

// One launch for several problems of the same q, G and M.  HLQ_ERR_UNSUPPORTED if the launch cannot be
// formed (the caller then runs the problems one after the other).
hlq_status hlq_launch_gemm_mfma_batch(int count, const HlqGemvItem *items, int64_t M, hlq_out_dtype out, void *ws,
                                      hipStream_t st)
{
    static_assert(HLQ_MAX_BATCH == 8, "the grouped kernels take the first blocks of eight problems");
    hlq_clear_stale_error();
    if (count < 1 || count > HLQ_MAX_BATCH || M < 1 || M > 0x7fffffff) return HLQ_ERR_UNSUPPORTED;
    // workgroups start in block order: long-K problems first, so that the longest workgroups do not end alone
    int order[HLQ_MAX_BATCH];
    for (int i = 0; i < count; ++i) order[i] = i;
    for (int i = 1; i < count; ++i)
        for (int j = i; j > 0 && items[order[j]].dm.nchunks > items[order[j - 1]].dm.nchunks; --j) {
            const int t = order[j];
            order[j] = order[j - 1];
            order[j - 1] = t;
        }
    HlqDims dms[HLQ_MAX_BATCH];
    for (int i = 0; i < count; ++i) dms[i] = items[order[i]].dm;
    const GroupPlan g = plan_group(count, dms, M);
    GemmProbs pr;
    GemmRedProbs rp;
    int begin[HLQ_MAX_BATCH], rbegin[HLQ_MAX_BATCH];
    long blk = 0, rblk = 0;
    int nred = 0;
    float *part = (float *)((char *)ws + HLQ_WS_COUNTER_BYTES);
    auto magic = [](int d) { return d > 1 ? (unsigned)((0x100000000ULL + (unsigned)d - 1) / (unsigned)d) : 0u; };
    for (int i = 0; i < count; ++i) {
        const HlqGemvItem &it = items[order[i]];
        if (it.dm.q != items[0].dm.q || it.dm.G != items[0].dm.G) return HLQ_ERR_UNSUPPORTED;
        GemmProb &p = pr.p[i];
        p.packed = (const char *)it.packed;
        p.col_bytes = it.dm.col_bytes;
        p.X = it.x;
        p.ldx = it.ldx;
        p.Y = it.y;
        p.ldy = it.ldy;
        p.part = part;
        p.N = it.dm.N;
        p.ntiles = it.dm.ntiles;
        p.nchunks = it.dm.nchunks;
        p.colgroups = (it.dm.ntiles + 3) / 4;
        p.cps = g.cps[i];
        p.nslices = g.nslices[i];
        p.cg_magic = magic(p.colgroups);
        p.ns_magic = magic(p.nslices);
        const unsigned long long blocks = (unsigned long long)p.colgroups * p.nslices * g.rowblocks;
        // the reciprocals are exact while (largest dividend) * divisor < 2^32
        if (blocks * p.colgroups >= 0x100000000ULL || blocks * p.nslices >= 0x100000000ULL) return HLQ_ERR_UNSUPPORTED;
        p.blk_begin = (int)blk;
        begin[i] = (int)blk;
        blk += (long)blocks;
        if (blk > 0x7fffffffL) return HLQ_ERR_UNSUPPORTED;
        if (p.nslices > 1) {
            GemmRedProb &r = rp.p[nred];
            r.part = part;
            r.Y = it.y;
            r.ldy = it.ldy;
            r.N = it.dm.N;
            r.nslices = p.nslices;
            r.blk_begin = (int)rblk;
            rbegin[nred++] = (int)rblk;
            rblk += (long)(((size_t)M * it.dm.N + 255) / 256);
            if (rblk > 0x7fffffffL) return HLQ_ERR_UNSUPPORTED;
            part += (size_t)p.nslices * (size_t)M * (size_t)it.dm.N;
        }
    }
    for (int i = count; i < HLQ_MAX_BATCH; ++i) {
        pr.p[i] = pr.p[0];
        begin[i] = 0x7fffffff;
    }
    const int4v lo = {begin[0], begin[1], begin[2], begin[3]}, hi = {begin[4], begin[5], begin[6], begin[7]};
    const int out_f32 = out == HLQ_OUT_F32;
    hlq_status s;
    switch (items[0].dm.q) {
    case 1: s = launch_group_q<1>(items[0].dm.G, g.MW, (unsigned)blk, lo, hi, (int)M, out_f32, hlq_ws_range_flag(ws), pr, st); break;
    case 2: s = launch_group_q<2>(items[0].dm.G, g.MW, (unsigned)blk, lo, hi, (int)M, out_f32, hlq_ws_range_flag(ws), pr, st); break;
    case 3: s = launch_group_q<3>(items[0].dm.G, g.MW, (unsigned)blk, lo, hi, (int)M, out_f32, hlq_ws_range_flag(ws), pr, st); break;
    case 4: s = launch_group_q<4>(items[0].dm.G, g.MW, (unsigned)blk, lo, hi, (int)M, out_f32, hlq_ws_range_flag(ws), pr, st); break;
    default: return HLQ_ERR_UNSUPPORTED;
    }
    if (s != HLQ_OK) return s;
    if (nred > 0) {
        for (int i = nred; i < HLQ_MAX_BATCH; ++i) {
            rp.p[i] = rp.p[0];
            rbegin[i] = 0x7fffffff;
        }
        const int4v rlo = {rbegin[0], rbegin[1], rbegin[2], rbegin[3]}, rhi = {rbegin[4], rbegin[5], rbegin[6], rbegin[7]};
        hlq_gemm_mfma_group_reduce_kernel<<<(unsigned)rblk, 256, 0, st>>>(rlo, rhi, (int)M, out_f32, rp);
    }
    s = hlq_launch_gemm_safe(count, items, M, out, ws, st);
    if (s != HLQ_OK) return s;
    return hlq_hip_status(hipGetLastError());
}
