// Internal declarations shared by the translation units of libhlq (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "hlq.h"

// ---------------------------------------------------------------------------------------
// Packed layout, version 1 (designed for 128-bit coalesced loads on CDNA4):
//
//   bits region, q*K*N/8 bytes, as 16-byte words  bits[j][c][n]:
//       j < q       bit-plane
//       c < K/128   "chunk" = 128 consecutive k (k = 128c .. 128c+127)
//       n < N       output column
//     The 16 bytes are four little-endian 32-bit words; bit b of word d is the plane-j bit
//     of weight (k = 128c + 32d + b, n).  A 4-bit slice [4i+3:4i] of word d is therefore
//     the table index for activations k = 128c + 32d + 4i .. +3 (bit r <-> k + r).
//     Consecutive n are consecutive 16-byte words: a wavefront whose lanes own 64
//     adjacent columns reads 1 KiB contiguous per load instruction.
//
//   meta region, 2*(q+1)*(K/G)*N bytes, fp16  meta[g][r][n]:
//       g < K/G, r < q: scale s_r[g, n];  r == q: zero z[g, n].
//     Consecutive n are consecutive halfs.
// ---------------------------------------------------------------------------------------
#define HLQ_LAYOUT_V1 0x484c5131u /* "HLQ1" */
#define HLQ_CHUNK_K 128

struct HlqDims {
    int K, N, q, G;
    int nchunks;   // K / 128
    int ngroups;   // K / G
    size_t bits_bytes;
    size_t meta_bytes;
};

hlq_status hlq_check_desc(const hlq_desc *d, HlqDims *out);

// Split-K plan for the LUT kernels: every workgroup owns `chunks_per_wg` consecutive chunks
// of K for a tile of columns; `nslices` partial results per output are then reduced.
struct HlqPlan {
    int chunks_per_wg;
    int nslices;
};
HlqPlan hlq_plan_gemv(const HlqDims &dm);

hlq_status hlq_launch_pack(const HlqDims &dm, const uint8_t *codes, const uint16_t *scales,
                           const uint16_t *zeros, void *packed, hipStream_t st);
hlq_status hlq_launch_unpack(const HlqDims &dm, const void *packed, uint8_t *codes,
                             uint16_t *scales, uint16_t *zeros, hipStream_t st);
hlq_status hlq_launch_gemv(const HlqDims &dm, const void *packed, const uint16_t *x, void *y,
                           hlq_out_dtype out, void *ws, hipStream_t st);
hlq_status hlq_launch_gemm(const HlqDims &dm, const void *packed, const uint16_t *X, int64_t M,
                           int64_t ldx, void *Y, int64_t ldy, hlq_out_dtype out, void *ws,
                           hipStream_t st);
size_t hlq_gemv_ws_bytes(const HlqDims &dm);
size_t hlq_gemm_ws_bytes(const HlqDims &dm, int64_t M);

static inline hlq_status hlq_hip_status(hipError_t e) { return e == hipSuccess ? HLQ_OK : HLQ_ERR_HIP; }
