// Kernel argument block and epilogue pieces shared by the two GEMV formulations (table lookup and
// matrix core).  Both use the same work split: a workgroup owns one group of column tiles and one
// K slice, its wavefronts take consecutive K ranges, K slices of different workgroups meet in the
// workspace.
#pragma once

#include "hlq_internal.h"

struct GemvProb {
    const char *packed;
    const uint16_t *x;
    void *y;
    float *part;       // [nslices][N] partial sums (nslices > 1)
    int *cnt;          // [ntg] arrival counters, zero between launches
    size_t col_bytes;
    int N, nchunks, ntiles, ntg, nslices, cps, blk_begin;
    int kw;            // matrix-core kernel: wavefronts per tile (runs a slice is cut into), a power of two
    int kw_shift;      // log2(kw)
    unsigned slice_magic;   // ceil(2^32 / nslices) for nslices > 1: local / nslices = umulhi(local, slice_magic)
    int M;             // matrix-core kernel, batched rows: activation rows; x / y row strides in elements
    long ldx, ldy;
    char *xt;          // many-rows kernel: the activations as matrix-core operands [chunk][operand][16 rows][128] (workspace)
    int *xexp;         //                   and the exponent of every row's scale [16]
};

// Host-side description of a launch.
struct GemvBatch {
    int blk_begin[HLQ_MAX_BATCH];   // first block of every problem, ascending; unused entries INT_MAX
    int count;
    int out_f32;
    GemvProb p[HLQ_MAX_BATCH];
};

// What the kernels take: the first blocks of the problems and the flag as leading scalar arguments --
// they are preloaded into scalar registers when a wavefront starts (kernarg preload, a per-file
// compiler option), so a workgroup finds its problem without a trip to memory -- and the problem
// records, of which the workgroup copies its own with one burst of scalar loads.
typedef int int4v __attribute__((ext_vector_type(4)));
struct GemvProbs {
    GemvProb p[HLQ_MAX_BATCH];
};
struct GemvKernelArgs {
    int4v lo, hi;
    int out_f32;
    GemvProbs probs;
};
inline GemvKernelArgs gemv_kernel_args(const GemvBatch &b)
{
    static_assert(HLQ_MAX_BATCH == 8, "the kernels take the first blocks of eight problems");
    GemvKernelArgs a;
    a.lo = (int4v){b.blk_begin[0], b.blk_begin[1], b.blk_begin[2], b.blk_begin[3]};
    a.hi = (int4v){b.blk_begin[4], b.blk_begin[5], b.blk_begin[6], b.blk_begin[7]};
    a.out_f32 = b.out_f32;
    for (int i = 0; i < HLQ_MAX_BATCH; ++i) a.probs.p[i] = b.p[i];
    return a;
}

// index of the problem that owns workgroup `blk`: the table is ascending, unused entries INT_MAX
__device__ __forceinline__ int gemv_problem_of(const int4v &bb_lo, const int4v &bb_hi, int blk)
{
    return blk >= bb_hi.w ? 7 : blk >= bb_hi.z ? 6 : blk >= bb_hi.y ? 5 : blk >= bb_hi.x ? 4
         : blk >= bb_lo.w ? 3 : blk >= bb_lo.z ? 2 : blk >= bb_lo.y ? 1 : 0;
}

// (tile group, K slice) of workgroup `local` of a problem: local = tg * nslices + slice, without an
// integer division (emulated ones cost some 30 dependent instructions at the head of every workgroup)
__device__ __forceinline__ void gemv_split_block(const GemvProb &P, int local, int &tg, int &slice)
{
    tg = P.nslices > 1 ? (int)__umulhi((unsigned)local, P.slice_magic) : local;
    slice = local - tg * P.nslices;
}


__device__ __forceinline__ float h2f(uint16_t h) { return (float)__builtin_bit_cast(_Float16, h); }

__device__ __forceinline__ void store_out(void *y, size_t idx, float v, int out_f32)
{
    if (out_f32) ((float *)y)[idx] = v;
    else ((_Float16 *)y)[idx] = (_Float16)v;   // round-to-nearest-even
}

// matrix-core formulation (hlq_gemv_mx.hip): W (a power of two) wavefronts per workgroup, kw of them
// per tile: ntg = ceil(ntiles / (W / kw)) tile groups, one arrival counter per TILE
hlq_status hlq_launch_gemv_mx(const GemvBatch &b, unsigned nblocks, int W, int nsets, int rows, int q, int G, hipStream_t st);
int hlq_gemv_mx_max_waves(int q, int G);

// many-rows kernel (hlq_gemm_rows.hip): W = 2, 4 or 8 wavefronts, one tile each, all on the workgroup's K slice
hlq_status hlq_launch_gemm_rows(const GemvBatch &b, unsigned nblocks, int W, int rows, int q, int G, hipStream_t st);
int hlq_gemm_rows_max(int G);

// table-storage variants of the lookup formulation (hlq_gemv_variants.hip); batch planned as for hlq_gemv_kernel, TN = 1
hlq_status hlq_launch_gemv_variant(int variant, const GemvBatch &b, unsigned nblocks, int W, int q, int G, hipStream_t st);

// workspace bytes the many-rows kernel needs beyond the partial sums, for one problem with M rows: the operand
// form of the activations and the row exponents (0 if M rows do not go to that kernel)
size_t hlq_gemm_rows_xt_bytes(const HlqDims &dm, int64_t M);
