// Internal declarations shared by the translation units of libhlq (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include "hlq.h"

// ---------------------------------------------------------------------------------------
// Packed layout "HLQ3" (designed for 128-bit coalesced loads by 64-wide wavefronts):
//
// The matrix is cut into column tiles of 64 columns (the last tile holds N - 64*tile
// columns, a multiple of 8) and into chunks of 128 consecutive k.  Everything one
// wavefront needs for (tile, chunk) is one contiguous record, and the records of a tile
// follow each other in chunk order, so a wavefront that walks K for its 64 columns reads
// one contiguous byte stream:
//
//   blob      = tile 0 | tile 1 | ...                 tile t starts at 64*t*col_bytes
//   col_bytes = (K/128)*q*16 + (K/G)*(q+1)*2          bytes per column
//   tile      = record(c=0) | record(c=1) | ...
//   record(c) = bits[j<q][lane<w][16 bytes]           w = tile width
//               meta[s][r<=q][lane<w] fp16             for the quant groups g that START in
//                                                      chunk c (s = their index in the chunk):
//                                                      r < q scale s_r[g, n], r == q zero z[g, n]
//
//   The 16 bytes of (plane j, lane) are four little-endian 32-bit words, word d covering the
//   32-k block k = 128c + 32d .. +31 of column n = 64*tile + lane.  Inside a word the even k of
//   the block sit in the low half and the odd k in the high half: weight k0 (0 <= k0 < 32) is
//   bit (k0 >> 1) + 16 * (k0 & 1).  Consequences the kernels rely on:
//     - a 4-bit slice [4i+3:4i] of a word indexes the table of the four activations
//       k0 = 8*(i & 3) + 2r + (i >> 2), r = 0..3 (bit r <-> r): four even or four odd k of one
//       8-k window -- any grouping of four activations serves the lookup method;
//     - bits p and p+16 of a word are the ADJACENT weights k0 = 2p, 2p+1, so one AND with a
//       two-bit mask yields a packed pair in natural k order for the matrix-core path.
//   With G = 256 a group spans two chunks; its meta sits in the even one.
//
// Total size is exactly K*N*q/8 + 2*(q+1)*(K/G)*N bytes: no padding anywhere.
// ---------------------------------------------------------------------------------------
#define HLQ_LAYOUT_V3 0x484c5133u /* "HLQ3" */
#define HLQ_CHUNK_K 128
#define HLQ_TILE_N 64
#define HLQ_MAX_K (1 << 21)
#define HLQ_MAX_N (1 << 20)

struct HlqDims {
    int K, N, q, G;
    int nchunks;   // K / 128
    int ngroups;   // K / G
    int ntiles;    // ceil(N / 64)
    size_t col_bytes;
    size_t bits_bytes;
    size_t meta_bytes;
};

// bit position inside a plane word of weight k0 (0..31) of the word's 32-k block
__host__ __device__ __forceinline__ int hlq_bit_pos(int k0) { return (k0 >> 1) + 16 * (k0 & 1); }

// groups whose meta is stored before chunk c of a tile
// (c >= 0; written so that with a constant G it is one multiplication or one shift)
__host__ __device__ __forceinline__ int hlq_groups_before(int c, int G)
{
    return G <= HLQ_CHUNK_K ? c * (HLQ_CHUNK_K / G) : (int)(((unsigned)c * HLQ_CHUNK_K + (unsigned)G - 1u) / (unsigned)G);
}

__host__ __device__ __forceinline__ int hlq_tile_width(int tile, int N)
{
    const int w = N - tile * HLQ_TILE_N;
    return w < HLQ_TILE_N ? w : HLQ_TILE_N;
}

// byte offset of record c inside its tile; w = tile width.  Fits 32 bits: at most 64 columns x 2^14 chunks x 104 bytes.
__host__ __device__ __forceinline__ uint32_t hlq_rec_in_tile(int w, int c, int q, int G)
{
    return (uint32_t)w * ((uint32_t)c * (uint32_t)(q * 16) + (uint32_t)hlq_groups_before(c, G) * (uint32_t)((q + 1) * 2));
}

// byte offset of record (tile, c); w = tile width
__host__ __device__ __forceinline__ size_t hlq_rec_off(size_t col_bytes, int tile, int w, int c, int q, int G)
{
    return (size_t)tile * HLQ_TILE_N * col_bytes +
           (size_t)w * ((size_t)c * q * 16 + (size_t)hlq_groups_before(c, G) * (q + 1) * 2);
}

hlq_status hlq_check_desc(const hlq_desc *d, HlqDims *out);

hlq_status hlq_launch_pack(const HlqDims &dm, const uint8_t *codes, const uint16_t *scales,
                           const uint16_t *zeros, void *packed, hipStream_t st);
hlq_status hlq_launch_unpack(const HlqDims &dm, const void *packed, uint8_t *codes,
                             uint16_t *scales, uint16_t *zeros, hipStream_t st);

hlq_status hlq_launch_quantize(const HlqDims &dm, const float *W, int t_max, uint8_t *codes, uint16_t *scales,
                               uint16_t *zeros, float *group_err, hipStream_t st);

// One GEMV of a grouped launch (all problems of a launch share q and G).
struct HlqGemvItem {
    HlqDims dm;
    const void *packed;
    const uint16_t *x;
    void *y;
    int M = 1;              // activation rows (all items of a launch carry the same number)
    long ldx = 0, ldy = 0;  // row strides of x and y in elements (M > 1)
};
#define HLQ_MAX_BATCH 8
// ws_cap: size of the workspace behind `ws` if the launch is to be refused when its plan needs more
// (HLQ_ERR_BUFFER_TOO_SMALL); 0 = the caller has checked the documented bound already
hlq_status hlq_launch_gemv_batch(int count, const HlqGemvItem *items, hlq_out_dtype out, void *ws,
                                 hipStream_t st, size_t ws_cap = 0);
hlq_status hlq_launch_gemm(const HlqDims &dm, const void *packed, const uint16_t *X, int64_t M,
                           int64_t ldx, void *Y, int64_t ldy, hlq_out_dtype out, void *ws,
                           hipStream_t st);
hlq_status hlq_launch_ws_init(void *ws, size_t bytes, hipStream_t st);
hlq_status hlq_gemv_plan_override(int tn, int w, int cpw);
hlq_status hlq_gemv_ws_used(const HlqDims &dm, size_t *bytes);
hlq_status hlq_gemv_plan_describe(int count, const HlqDims *dms, int M, hlq_gemv_plan_info *out);
hlq_status hlq_gemv_path_override(int path);

// Workspace = [HLQ_WS_COUNTER_BYTES of split-K arrival counters][fp32 partial sums].
// Counters are zero between calls (hlq_workspace_init zeroes them; kernels re-zero them).
#define HLQ_WS_COUNTER_BYTES 131072
// The last two counters are not arrival counters: [0] is raised by the tiled matrix-core GEMM when it meets a
// scale or zero outside the range its fp16 weight rebuild can represent, [1] counts the fallback kernel's
// workgroups out (hlq_gemm_safe.hip).  Both are zero between calls, like the arrival counters.
#define HLQ_WS_ARRIVAL_COUNTERS (HLQ_WS_COUNTER_BYTES / 4 - 2)
static inline int *hlq_ws_range_flag(void *ws) { return (int *)ws + HLQ_WS_ARRIVAL_COUNTERS; }

// one problem of the fallback launch
struct HlqSafeProb {
    const char *packed;
    size_t col_bytes;
    const uint16_t *X;
    long ldx;
    void *Y;
    long ldy;
    int N, ntiles, nchunks, q, G;
    long item_begin;
};
struct HlqSafeProbs {
    HlqSafeProb p[8];
    int count;
    long items_total;
};
size_t hlq_gemv_partial_bytes(const HlqDims &dm);
size_t hlq_gemm_partial_bytes(const HlqDims &dm, int64_t M);
size_t hlq_gemm_lut_partial_bytes(const HlqDims &dm, int64_t M);
size_t hlq_gemm_mfma_partial_bytes(const HlqDims &dm, int64_t M);
hlq_status hlq_launch_gemm_lut(const HlqDims &dm, const void *packed, const uint16_t *X, int64_t M,
                               int64_t ldx, void *Y, int64_t ldy, hlq_out_dtype out, void *ws, hipStream_t st);
hlq_status hlq_launch_gemm_mfma(const HlqDims &dm, const void *packed, const uint16_t *X, int64_t M,
                                int64_t ldx, void *Y, int64_t ldy, hlq_out_dtype out, void *ws, hipStream_t st);
hlq_status hlq_gemm_path_override(int path);
bool hlq_gemm_uses_matrix_cores(int64_t M);
hlq_status hlq_launch_gemm_mfma_batch(int count, const HlqGemvItem *items, int64_t M, hlq_out_dtype out, void *ws,
                                      hipStream_t st);
size_t hlq_gemm_mfma_batch_partial_bytes(int count, const HlqDims *dms, int64_t M);
hlq_status hlq_launch_gemm_safe(int count, const HlqGemvItem *items, int64_t M, hlq_out_dtype out, void *ws, hipStream_t st);
int hlq_gemv_mx_rows_per_set(int G);
int hlq_gemm_mx_rows_per_pass(int G);
bool hlq_gemm_batch_on_mx(int count, const HlqGemvItem *items, int64_t M);
bool hlq_gemm_rows_wins(long units, int q, int64_t M);
bool hlq_gemm_rows_wins_few(long units, int q, int rows);
int hlq_gemm_rows_max(int G);
bool hlq_gemm_uses_mx_rows(int64_t M);
bool hlq_gemm_rows_all();
size_t hlq_gemm_mx_partial_bytes(const HlqDims &dm, int64_t M);
hlq_status hlq_launch_gemm_mx_rows(const HlqDims &dm, const void *packed, const uint16_t *X, int64_t M, int64_t ldx,
                                   void *Y, int64_t ldy, hlq_out_dtype out, void *ws, hipStream_t st);

// HLQ_VERBOSE=1 in the environment prints the runtime's message for a failed launch to stderr.
static inline hlq_status hlq_hip_status(hipError_t e)
{
    if (e == hipSuccess) return HLQ_OK;
    const char *v = getenv("HLQ_VERBOSE");
    if (v && *v && *v != '0') fprintf(stderr, "libhlq: HIP error %d: %s\n", (int)e, hipGetErrorString(e));
    return HLQ_ERR_HIP;
}
// The runtime's "last error" is sticky per thread: drop whatever an earlier caller left there, so
// that the check after our own launches reports our launches only.
static inline void hlq_clear_stale_error() { (void)hipGetLastError(); }
