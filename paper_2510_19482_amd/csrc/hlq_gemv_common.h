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
};

// The head of the block (first blocks of all problems, flags) is what every workgroup needs before it
// knows its problem: kept together so that one scalar load fetches it, a second one the problem.
struct GemvBatch {
    int blk_begin[HLQ_MAX_BATCH];   // ascending; unused entries INT_MAX
    int count;
    int out_f32;
    GemvProb p[HLQ_MAX_BATCH];
};

// (tile group, K slice) of workgroup `local` of a problem: local = tg * nslices + slice, without an
// integer division (emulated ones cost some 30 dependent instructions at the head of every workgroup)
__device__ __forceinline__ void gemv_split_block(const GemvProb &P, int local, int &tg, int &slice)
{
    tg = P.nslices > 1 ? (int)__umulhi((unsigned)local, P.slice_magic) : local;
    slice = local - tg * P.nslices;
}

// index of the problem that owns workgroup `blk` (branch-free: the table is sorted)
__device__ __forceinline__ int gemv_problem_of(const GemvBatch &b, int blk)
{
    int pi = 0;
#pragma unroll
    for (int i = 1; i < HLQ_MAX_BATCH; ++i) pi += blk >= b.blk_begin[i] ? 1 : 0;
    return pi;
}

__device__ __forceinline__ float h2f(uint16_t h) { return (float)__builtin_bit_cast(_Float16, h); }

__device__ __forceinline__ void store_out(void *y, size_t idx, float v, int out_f32)
{
    if (out_f32) ((float *)y)[idx] = v;
    else ((_Float16 *)y)[idx] = (_Float16)v;   // round-to-nearest-even
}

// matrix-core formulation (hlq_gemv_mx.hip): W (a power of two) wavefronts per workgroup, kw of them
// per tile: ntg = ceil(ntiles / (W / kw)) tile groups, one arrival counter per TILE
hlq_status hlq_launch_gemv_mx(const GemvBatch &b, unsigned nblocks, int W, int nsets, int q, int G, hipStream_t st);
int hlq_gemv_mx_max_waves(int q, int G);
