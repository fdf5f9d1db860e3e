// Host side of the C ABI: argument validation, size arithmetic, dispatch.
// Everything that can be decided without a GPU is decided here, before any launch.
#include "hlq_internal.h"

hlq_status hlq_check_desc(const hlq_desc *d, HlqDims *out)
{
    if (!d) return HLQ_ERR_NULL;
    if (d->layout != HLQ_LAYOUT_V1) return HLQ_ERR_BAD_DESC;
    if (d->q < 1 || d->q > 4) return HLQ_ERR_BAD_DESC;
    if (d->G != 32 && d->G != 64 && d->G != 128 && d->G != 256) return HLQ_ERR_BAD_DESC;
    if (d->K < 1 || d->N < 1) return HLQ_ERR_BAD_DESC;
    if (d->K % HLQ_CHUNK_K != 0 || d->K % d->G != 0 || d->N % 8 != 0) return HLQ_ERR_BAD_DESC;
    if (out) {
        out->K = d->K;
        out->N = d->N;
        out->q = d->q;
        out->G = d->G;
        out->nchunks = d->K / HLQ_CHUNK_K;
        out->ngroups = d->K / d->G;
        out->bits_bytes = (size_t)d->q * (size_t)out->nchunks * (size_t)d->N * 16u;
        out->meta_bytes = (size_t)(d->q + 1) * (size_t)out->ngroups * (size_t)d->N * 2u;
    }
    return HLQ_OK;
}

extern "C" {

const char *hlq_status_string(hlq_status s)
{
    switch (s) {
    case HLQ_OK: return "ok";
    case HLQ_ERR_NULL: return "a required pointer is NULL";
    case HLQ_ERR_BAD_DESC:
        return "bad descriptor (need 1<=q<=4, G in {32,64,128,256}, K%128==0, K%G==0, N%8==0, "
               "layout==hlq_layout_version())";
    case HLQ_ERR_UNSUPPORTED: return "request not supported by this build";
    case HLQ_ERR_BUFFER_TOO_SMALL: return "packed or workspace buffer too small";
    case HLQ_ERR_BAD_STRIDE: return "bad leading dimension or row count";
    case HLQ_ERR_HIP: return "HIP runtime error at launch";
    }
    return "unknown status";
}

uint32_t hlq_layout_version(void) { return HLQ_LAYOUT_V1; }

hlq_status hlq_packed_bytes(const hlq_desc *d, size_t *total, size_t *bits, size_t *meta)
{
    HlqDims dm;
    hlq_status s = hlq_check_desc(d, &dm);
    if (s != HLQ_OK) return s;
    if (!total) return HLQ_ERR_NULL;
    *total = dm.bits_bytes + dm.meta_bytes;
    if (bits) *bits = dm.bits_bytes;
    if (meta) *meta = dm.meta_bytes;
    return HLQ_OK;
}

hlq_status hlq_workspace_bytes(const hlq_desc *d, int64_t M, size_t *bytes)
{
    HlqDims dm;
    hlq_status s = hlq_check_desc(d, &dm);
    if (s != HLQ_OK) return s;
    if (!bytes) return HLQ_ERR_NULL;
    if (M < 0) return HLQ_ERR_BAD_STRIDE;
    size_t b = M <= 1 ? hlq_gemv_ws_bytes(dm) : hlq_gemm_ws_bytes(dm, M);
    size_t b1 = hlq_gemv_ws_bytes(dm);
    if (b1 > b) b = b1;
    *bytes = (b + 255u) & ~(size_t)255u;
    return HLQ_OK;
}

hlq_status hlq_pack(const hlq_desc *d, const uint8_t *codes, const uint16_t *scales,
                    const uint16_t *zeros, void *packed, size_t packed_bytes, void *stream)
{
    HlqDims dm;
    hlq_status s = hlq_check_desc(d, &dm);
    if (s != HLQ_OK) return s;
    if (!codes || !scales || !zeros || !packed) return HLQ_ERR_NULL;
    if (packed_bytes < dm.bits_bytes + dm.meta_bytes) return HLQ_ERR_BUFFER_TOO_SMALL;
    return hlq_launch_pack(dm, codes, scales, zeros, packed, (hipStream_t)stream);
}

hlq_status hlq_unpack(const hlq_desc *d, const void *packed, uint8_t *codes, uint16_t *scales,
                      uint16_t *zeros, void *stream)
{
    HlqDims dm;
    hlq_status s = hlq_check_desc(d, &dm);
    if (s != HLQ_OK) return s;
    if (!packed) return HLQ_ERR_NULL;
    return hlq_launch_unpack(dm, packed, codes, scales, zeros, (hipStream_t)stream);
}

hlq_status hlq_lut_gemv(const hlq_desc *d, const void *packed, const uint16_t *x, void *y,
                        hlq_out_dtype out, void *ws, size_t ws_bytes, void *stream)
{
    HlqDims dm;
    hlq_status s = hlq_check_desc(d, &dm);
    if (s != HLQ_OK) return s;
    if (!packed || !x || !y) return HLQ_ERR_NULL;
    if (out != HLQ_OUT_F16 && out != HLQ_OUT_F32) return HLQ_ERR_UNSUPPORTED;
    size_t need = hlq_gemv_ws_bytes(dm);
    if (need > 0 && !ws) return HLQ_ERR_NULL;
    if (ws_bytes < need) return HLQ_ERR_BUFFER_TOO_SMALL;
    return hlq_launch_gemv(dm, packed, x, y, out, ws, (hipStream_t)stream);
}

hlq_status hlq_lut_gemm(const hlq_desc *d, const void *packed, const uint16_t *X, int64_t M,
                        int64_t ldx, void *Y, int64_t ldy, hlq_out_dtype out, void *ws,
                        size_t ws_bytes, void *stream)
{
    HlqDims dm;
    hlq_status s = hlq_check_desc(d, &dm);
    if (s != HLQ_OK) return s;
    if (M < 0 || ldx < dm.K || ldy < dm.N) return HLQ_ERR_BAD_STRIDE;
    if (out != HLQ_OUT_F16 && out != HLQ_OUT_F32) return HLQ_ERR_UNSUPPORTED;
    if (M == 0) return HLQ_OK;
    if (!packed || !X || !Y) return HLQ_ERR_NULL;
    if (M == 1) {
        size_t need1 = hlq_gemv_ws_bytes(dm);
        if (need1 > 0 && !ws) return HLQ_ERR_NULL;
        if (ws_bytes < need1) return HLQ_ERR_BUFFER_TOO_SMALL;
        return hlq_launch_gemv(dm, packed, X, Y, out, ws, (hipStream_t)stream);
    }
    size_t need = hlq_gemm_ws_bytes(dm, M);
    if (need > 0 && !ws) return HLQ_ERR_NULL;
    if (ws_bytes < need) return HLQ_ERR_BUFFER_TOO_SMALL;
    return hlq_launch_gemm(dm, packed, X, M, ldx, Y, ldy, out, ws, (hipStream_t)stream);
}

} // extern "C"
