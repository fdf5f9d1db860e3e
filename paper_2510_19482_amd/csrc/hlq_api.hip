// Host side of the C ABI: argument validation, size arithmetic, dispatch.
// Everything that can be decided without a GPU is decided here, before any launch.
#include "hlq_internal.h"

hlq_status hlq_check_desc(const hlq_desc *d, HlqDims *out)
{
    if (!d) return HLQ_ERR_NULL;
    if (d->layout != HLQ_LAYOUT_V3) return HLQ_ERR_BAD_DESC;
    if (d->q < 1 || d->q > 4) return HLQ_ERR_BAD_DESC;
    if (d->G != 32 && d->G != 64 && d->G != 128 && d->G != 256) return HLQ_ERR_BAD_DESC;
    if (d->K < 1 || d->N < 1) return HLQ_ERR_BAD_DESC;
    if (d->K % HLQ_CHUNK_K != 0 || d->K % d->G != 0 || d->N % 8 != 0) return HLQ_ERR_BAD_DESC;
    if (d->K > HLQ_MAX_K || d->N > HLQ_MAX_N) return HLQ_ERR_UNSUPPORTED;
    if (out) {
        out->K = d->K;
        out->N = d->N;
        out->q = d->q;
        out->G = d->G;
        out->nchunks = d->K / HLQ_CHUNK_K;
        out->ngroups = d->K / d->G;
        out->ntiles = (d->N + HLQ_TILE_N - 1) / HLQ_TILE_N;
        out->col_bytes = (size_t)out->nchunks * d->q * 16u + (size_t)out->ngroups * (d->q + 1) * 2u;
        out->bits_bytes = (size_t)d->q * (size_t)out->nchunks * (size_t)d->N * 16u;
        out->meta_bytes = (size_t)(d->q + 1) * (size_t)out->ngroups * (size_t)d->N * 2u;
    }
    return HLQ_OK;
}

// counters + the larger of the GEMV and GEMM partial-sum areas, rounded to 256 bytes
static size_t ws_need(const HlqDims &dm, int64_t M)
{
    size_t part = hlq_gemv_partial_bytes(dm);
    if (M > 1) {
        const size_t pm = hlq_gemm_partial_bytes(dm, M);
        if (pm > part) part = pm;
    }
    return (HLQ_WS_COUNTER_BYTES + part + 255u) & ~(size_t)255u;
}

static bool misaligned(const void *p, unsigned a) { return ((uintptr_t)p & (a - 1u)) != 0; }

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

uint32_t hlq_layout_version(void) { return HLQ_LAYOUT_V3; }

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
    *bytes = ws_need(dm, M);
    return HLQ_OK;
}

hlq_status hlq_batch_workspace_bytes(int count, const hlq_desc *descs, size_t *bytes)
{
    if (!descs || !bytes) return HLQ_ERR_NULL;
    if (count < 1 || count > HLQ_MAX_BATCH) return HLQ_ERR_UNSUPPORTED;
    size_t b = HLQ_WS_COUNTER_BYTES;
    for (int i = 0; i < count; ++i) {
        HlqDims dm;
        hlq_status s = hlq_check_desc(&descs[i], &dm);
        if (s != HLQ_OK) return s;
        b += hlq_gemv_partial_bytes(dm);
    }
    *bytes = (b + 255u) & ~(size_t)255u;
    return HLQ_OK;
}

static size_t batch_partial_bytes(int count, const HlqDims *dms, int64_t M)
{
    return M > 1 ? hlq_gemm_mfma_batch_partial_bytes(count, dms, M) : 0;
}

hlq_status hlq_gemm_batch_workspace_bytes(int count, const hlq_desc *descs, int64_t M, size_t *bytes)
{
    if (!descs || !bytes) return HLQ_ERR_NULL;
    if (count < 1 || count > HLQ_MAX_BATCH) return HLQ_ERR_UNSUPPORTED;
    if (M < 0) return HLQ_ERR_BAD_STRIDE;
    size_t b = HLQ_WS_COUNTER_BYTES;
    HlqDims dms[HLQ_MAX_BATCH];
    for (int i = 0; i < count; ++i) {
        hlq_status s = hlq_check_desc(&descs[i], &dms[i]);
        if (s != HLQ_OK) return s;
        b += M <= 1 ? hlq_gemv_partial_bytes(dms[i]) : hlq_gemm_partial_bytes(dms[i], M);
    }
    // the grouped launch of the tiled kernel splits K on its own terms
    const size_t grouped = HLQ_WS_COUNTER_BYTES + batch_partial_bytes(count, dms, M);
    if (grouped > b) b = grouped;
    *bytes = (b + 255u) & ~(size_t)255u;
    return HLQ_OK;
}

hlq_status hlq_workspace_init(void *ws, size_t ws_bytes, void *stream)
{
    if (!ws) return HLQ_ERR_NULL;
    if (ws_bytes < HLQ_WS_COUNTER_BYTES) return HLQ_ERR_BUFFER_TOO_SMALL;
    if (((uintptr_t)ws & 15u) != 0) return HLQ_ERR_BAD_STRIDE;
    return hlq_launch_ws_init(ws, ws_bytes, (hipStream_t)stream);
}

hlq_status hlq_set_gemv_plan(int tiles_per_wave, int waves_per_workgroup, int chunks_per_wave)
{
    return hlq_gemv_plan_override(tiles_per_wave, waves_per_workgroup, chunks_per_wave);
}

hlq_status hlq_gemv_plan_query(int count, const hlq_desc *descs, int64_t M, hlq_gemv_plan_info *out)
{
    if (!descs || !out) return HLQ_ERR_NULL;
    if (count < 1 || count > HLQ_MAX_BATCH) return HLQ_ERR_UNSUPPORTED;
    if (M < 1 || M > 64) return HLQ_ERR_UNSUPPORTED;
    HlqDims dms[HLQ_MAX_BATCH];
    for (int i = 0; i < count; ++i) {
        hlq_status s = hlq_check_desc(&descs[i], &dms[i]);
        if (s != HLQ_OK) return s;
        if (descs[i].q != descs[0].q || descs[i].G != descs[0].G) return HLQ_ERR_UNSUPPORTED;
    }
    return hlq_gemv_plan_describe(count, dms, (int)M, out);
}

hlq_status hlq_set_gemm_path(int path) { return hlq_gemm_path_override(path); }

hlq_status hlq_set_gemv_path(int path) { return hlq_gemv_path_override(path); }

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

hlq_status hlq_quantize(const hlq_desc *d, const float *W, int t_max, uint8_t *codes, uint16_t *scales,
                        uint16_t *zeros, float *group_err, void *stream)
{
    HlqDims dm;
    hlq_status s = hlq_check_desc(d, &dm);
    if (s != HLQ_OK) return s;
    if (!W || !codes || !scales || !zeros) return HLQ_ERR_NULL;
    if (t_max < 1 || t_max > 1000) return HLQ_ERR_UNSUPPORTED;
    if (misaligned(W, 4) || misaligned(scales, 2) || misaligned(zeros, 2) || (group_err && misaligned(group_err, 4)))
        return HLQ_ERR_BAD_STRIDE;
    return hlq_launch_quantize(dm, W, t_max, codes, scales, zeros, group_err, (hipStream_t)stream);
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
    if (!packed || !x || !y || !ws) return HLQ_ERR_NULL;
    if (out != HLQ_OUT_F16 && out != HLQ_OUT_F32) return HLQ_ERR_UNSUPPORTED;
    if (misaligned(packed, 16) || misaligned(x, 16) || misaligned(ws, 16) || misaligned(y, out == HLQ_OUT_F32 ? 4 : 2))
        return HLQ_ERR_BAD_STRIDE;
    if (ws_bytes < HLQ_WS_COUNTER_BYTES + hlq_gemv_partial_bytes(dm)) return HLQ_ERR_BUFFER_TOO_SMALL;
    HlqGemvItem it;
    it.dm = dm;
    it.packed = packed;
    it.x = x;
    it.y = y;
    return hlq_launch_gemv_batch(1, &it, out, ws, (hipStream_t)stream);
}

hlq_status hlq_lut_gemv_batch(int count, const hlq_desc *descs, const void *const *packed,
                              const uint16_t *const *x, void *const *y, hlq_out_dtype out, void *ws,
                              size_t ws_bytes, void *stream)
{
    if (!descs || !packed || !x || !y || !ws) return HLQ_ERR_NULL;
    if (count < 1 || count > HLQ_MAX_BATCH) return HLQ_ERR_UNSUPPORTED;
    if (out != HLQ_OUT_F16 && out != HLQ_OUT_F32) return HLQ_ERR_UNSUPPORTED;
    if (misaligned(ws, 16)) return HLQ_ERR_BAD_STRIDE;
    HlqGemvItem items[HLQ_MAX_BATCH];
    size_t need = HLQ_WS_COUNTER_BYTES;
    for (int i = 0; i < count; ++i) {
        hlq_status s = hlq_check_desc(&descs[i], &items[i].dm);
        if (s != HLQ_OK) return s;
        if (descs[i].q != descs[0].q || descs[i].G != descs[0].G) return HLQ_ERR_UNSUPPORTED;
        if (!packed[i] || !x[i] || !y[i]) return HLQ_ERR_NULL;
        if (misaligned(packed[i], 16) || misaligned(x[i], 16) || misaligned(y[i], out == HLQ_OUT_F32 ? 4 : 2))
            return HLQ_ERR_BAD_STRIDE;
        items[i].packed = packed[i];
        items[i].x = x[i];
        items[i].y = y[i];
        need += hlq_gemv_partial_bytes(items[i].dm);
    }
    if (ws_bytes < need) return HLQ_ERR_BUFFER_TOO_SMALL;
    return hlq_launch_gemv_batch(count, items, out, ws, (hipStream_t)stream);
}

hlq_status hlq_lut_gemm_batch(int count, const hlq_desc *descs, const void *const *packed,
                              const uint16_t *const *X, int64_t M, const int64_t *ldx, void *const *Y,
                              const int64_t *ldy, hlq_out_dtype out, void *ws, size_t ws_bytes, void *stream)
{
    if (!descs || !packed || !X || !Y || !ldx || !ldy || !ws) return HLQ_ERR_NULL;
    if (count < 1 || count > HLQ_MAX_BATCH) return HLQ_ERR_UNSUPPORTED;
    if (out != HLQ_OUT_F16 && out != HLQ_OUT_F32) return HLQ_ERR_UNSUPPORTED;
    if (M < 0) return HLQ_ERR_BAD_STRIDE;
    if (misaligned(ws, 16)) return HLQ_ERR_BAD_STRIDE;
    HlqGemvItem items[HLQ_MAX_BATCH];
    size_t need = HLQ_WS_COUNTER_BYTES;
    for (int i = 0; i < count; ++i) {
        hlq_status s = hlq_check_desc(&descs[i], &items[i].dm);
        if (s != HLQ_OK) return s;
        if (descs[i].q != descs[0].q || descs[i].G != descs[0].G) return HLQ_ERR_UNSUPPORTED;
        if (ldx[i] < items[i].dm.K || ldy[i] < items[i].dm.N || (M > 1 && ldx[i] % 8 != 0)) return HLQ_ERR_BAD_STRIDE;
        if (M == 0) continue;
        if (!packed[i] || !X[i] || !Y[i]) return HLQ_ERR_NULL;
        if (misaligned(packed[i], 16) || misaligned(X[i], 16) || misaligned(Y[i], out == HLQ_OUT_F32 ? 4 : 2))
            return HLQ_ERR_BAD_STRIDE;
        items[i].packed = packed[i];
        items[i].x = X[i];
        items[i].y = Y[i];
        items[i].M = (int)(M < 1024 ? M : 1024);
        items[i].ldx = (long)ldx[i];
        items[i].ldy = (long)ldy[i];
        need += M <= 1 ? hlq_gemv_partial_bytes(items[i].dm) : hlq_gemm_partial_bytes(items[i].dm, M);
    }
    if (M == 0) return HLQ_OK;
    {
        HlqDims dms[HLQ_MAX_BATCH];
        for (int i = 0; i < count; ++i) dms[i] = items[i].dm;
        const size_t grouped = HLQ_WS_COUNTER_BYTES + batch_partial_bytes(count, dms, M);
        if (grouped > need) need = grouped;
    }
    if (ws_bytes < need) return HLQ_ERR_BUFFER_TOO_SMALL;
    // one launch when the few-rows kernel carries M rows and the lookup formulation is not forced
    if (M == 1 || (hlq_gemm_batch_on_mx(count, items, M) && hlq_gemm_uses_mx_rows(M)))
        return hlq_launch_gemv_batch(count, items, out, ws, (hipStream_t)stream);
    // more rows on the matrix cores: one launch of the tiled kernel over all problems (and one for the partial
    // sums where K is split)
    if (count > 1 && hlq_gemm_uses_matrix_cores(M)) {
        const hlq_status s = hlq_launch_gemm_mfma_batch(count, items, M, out, ws, (hipStream_t)stream);
        if (s != HLQ_ERR_UNSUPPORTED) return s;
    }
    for (int i = 0; i < count; ++i) {
        hlq_status s = hlq_launch_gemm(items[i].dm, packed[i], X[i], M, ldx[i], Y[i], ldy[i], out, ws, (hipStream_t)stream);
        if (s != HLQ_OK) return s;
    }
    return HLQ_OK;
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
    if (!packed || !X || !Y || !ws) return HLQ_ERR_NULL;
    if (misaligned(packed, 16) || misaligned(X, 16) || misaligned(ws, 16) || misaligned(Y, out == HLQ_OUT_F32 ? 4 : 2))
        return HLQ_ERR_BAD_STRIDE;
    if (M > 1 && ldx % 8 != 0) return HLQ_ERR_BAD_STRIDE;   // rows are read as 16-byte words
    if (ws_bytes < ws_need(dm, M)) return HLQ_ERR_BUFFER_TOO_SMALL;
    if (M == 1) {
        HlqGemvItem it;
        it.dm = dm;
        it.packed = packed;
        it.x = X;
        it.y = Y;
        return hlq_launch_gemv_batch(1, &it, out, ws, (hipStream_t)stream);
    }
    return hlq_launch_gemm(dm, packed, X, M, ldx, Y, ldy, out, ws, (hipStream_t)stream);
}

} // extern "C"
