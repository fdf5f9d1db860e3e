// Fallback of the tiled matrix-core GEMM for weights it cannot represent.  That kernel rebuilds
// W^ = sum_j s_j b_j + z (Eq. 3) in fp16 registers with pre-scaled scales (s_j * 2^7), which is only
// finite for |s_j| < 512; any finite fp16 scale is a valid HLQ parameter, though.  The tiled kernel
// therefore looks at every scale and zero it loads and raises a flag in the workspace if one lies
// outside its range; this kernel is launched behind it in every call, leaves at once if the flag
// is down (the normal case: one scalar load per workgroup), and otherwise computes the whole
// product again the plain way -- W^ element by element in fp32 from the plane bits, fp32
// accumulation -- and overwrites Y.  Slow, exact to fp32 rounding, valid for every finite fp16
// parameter.  The last workgroup to finish lowers the flag again.
#include "hlq_internal.h"

namespace {

constexpr int SAFE_ROWS = 8;   // activation rows per work item

__device__ __forceinline__ float half_bits_to_float(uint16_t h) { return (float)__builtin_bit_cast(_Float16, h); }

__global__ void __launch_bounds__(64)
hlq_gemm_safe_kernel(const HlqSafeProbs pr, const int M, const int out_f32, int *flag, int *done)
{
    // an ordinary load: the flag was written by the launch before this one, and a kernel boundary makes that visible
    if (*(const int *)flag == 0) return;
    const int lane = threadIdx.x;
    for (long item = blockIdx.x; item < pr.items_total; item += gridDim.x) {
        int pi = 0;
        while (pi + 1 < pr.count && item >= pr.p[pi + 1].item_begin) ++pi;
        const HlqSafeProb &P = pr.p[pi];
        const long local = item - P.item_begin;
        const int tile = (int)(local % P.ntiles), m0 = (int)(local / P.ntiles) * SAFE_ROWS;
        const int tw = hlq_tile_width(tile, P.N);
        const bool col_ok = lane < tw;
        const int lane_c = col_ok ? lane : tw - 1;
        const char *tile_base = P.packed + (size_t)tile * HLQ_TILE_N * P.col_bytes;
        const int q = P.q, G = P.G;
        float acc[SAFE_ROWS];
#pragma unroll
        for (int r = 0; r < SAFE_ROWS; ++r) acc[r] = 0.f;
        for (int c = 0; c < P.nchunks; ++c) {
            const char *rec = tile_base + hlq_rec_in_tile(tw, c, q, G);
            uint32_t w[4][4];
            for (int j = 0; j < q; ++j) {
                const uint4 v = ((const uint4 *)rec)[j * tw + lane_c];
                w[j][0] = v.x; w[j][1] = v.y; w[j][2] = v.z; w[j][3] = v.w;
            }
            // scales of the chunk's quant segments; a 256-wide group keeps them in the record of its even chunk
            const int cm = G > 128 ? (c & ~1) : c;
            const uint16_t *mp = (const uint16_t *)(tile_base + hlq_rec_in_tile(tw, cm, q, G) + (size_t)tw * q * 16);
            const int gs = G < 128 ? G : 128;
            for (int sg = 0; sg < 128 / gs; ++sg) {
                float s[4] = {0.f, 0.f, 0.f, 0.f};
                for (int j = 0; j < q; ++j) s[j] = half_bits_to_float(mp[(sg * (q + 1) + j) * tw + lane_c]);
                const float z = half_bits_to_float(mp[(sg * (q + 1) + q) * tw + lane_c]);
                for (int k0 = sg * gs; k0 < (sg + 1) * gs; ++k0) {
                    const int bit = hlq_bit_pos(k0 & 31), d = k0 >> 5;
                    float wv = z;
                    for (int j = 0; j < q; ++j)
                        if ((w[j][d] >> bit) & 1u) wv += s[j];
                    const size_t k = (size_t)c * 128 + k0;
#pragma unroll
                    for (int r = 0; r < SAFE_ROWS; ++r) {
                        const int m = min(m0 + r, M - 1);   // rows past M repeat the last one and are dropped
                        acc[r] += half_bits_to_float(P.X[(size_t)m * P.ldx + k]) * wv;
                    }
                }
            }
        }
        if (col_ok) {
            const size_t n = (size_t)tile * HLQ_TILE_N + lane;
#pragma unroll
            for (int r = 0; r < SAFE_ROWS; ++r) {
                if (m0 + r >= M) break;
                if (out_f32) ((float *)P.Y)[(size_t)(m0 + r) * P.ldy + n] = acc[r];
                else ((_Float16 *)P.Y)[(size_t)(m0 + r) * P.ldy + n] = (_Float16)acc[r];
            }
        }
    }
    // every workgroup that saw the flag up counts itself out; the last one lowers the flag for the next call
    if (lane == 0) {
        const int old = __hip_atomic_fetch_add(done, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (old == (int)gridDim.x - 1) {
            __hip_atomic_store(done, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(flag, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

} // namespace

// Launches the fallback behind a tiled-kernel launch over the same problems.  `ws` is the call's workspace.
hlq_status hlq_launch_gemm_safe(int count, const HlqGemvItem *items, int64_t M, hlq_out_dtype out, void *ws, hipStream_t st)
{
    if (count < 1 || count > HLQ_MAX_BATCH || M < 1 || M > 0x7fffffff) return HLQ_ERR_UNSUPPORTED;
    HlqSafeProbs pr;
    long total = 0;
    for (int i = 0; i < count; ++i) {
        HlqSafeProb &p = pr.p[i];
        p.packed = (const char *)items[i].packed;
        p.col_bytes = items[i].dm.col_bytes;
        p.X = items[i].x;
        p.ldx = items[i].ldx;
        p.Y = items[i].y;
        p.ldy = items[i].ldy;
        p.N = items[i].dm.N;
        p.ntiles = items[i].dm.ntiles;
        p.nchunks = items[i].dm.nchunks;
        p.q = items[i].dm.q;
        p.G = items[i].dm.G;
        p.item_begin = total;
        total += (long)items[i].dm.ntiles * (long)((M + SAFE_ROWS - 1) / SAFE_ROWS);
    }
    for (int i = count; i < HLQ_MAX_BATCH; ++i) pr.p[i] = pr.p[0];
    pr.count = count;
    pr.items_total = total;
    // few workgroups: in the normal case all of them only look at the flag and leave, and that costs per workgroup
    const unsigned grid = (unsigned)(total < 512 ? total : 512);
    hlq_gemm_safe_kernel<<<grid, 64, 0, st>>>(pr, (int)M, out == HLQ_OUT_F32, hlq_ws_range_flag(ws), hlq_ws_range_flag(ws) + 1);
    return HLQ_OK;
}
