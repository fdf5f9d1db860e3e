/* hlq.h -- C ABI of libhlq: bit-serial LUT GEMV/GEMM over HLQ weights on MI355X (gfx950).
 *
 * The operation (paper: Sec. 2 "Bit-Serial LUT-Based GEMM", App. B, App. D; format: Eq. 3):
 *
 *     W^[k,n] = sum_{j<q} s_j[k/G, n] * b_j[k,n] + z[k/G, n],   b_j in {0,1}      (Eq. 3)
 *     Y[m,n]  = sum_k X[m,k] * W^[k,n]
 *
 * computed without reconstructing W^: activations are taken four at a time, each group
 * of four gets a 16-entry table of the partial sums sum_r bit_r(i) * x[4t+r], and every
 * 4-bit slice of every bit-plane indexes that table; looked-up entries are added in
 * fp32, multiplied once per (plane, quant group) by s_j, and z enters as
 * z * (sum of the group's activations).  By default the per-plane binary dot products are
 * taken on the matrix cores instead of through tables (same sums, see hlq_set_gemv_path),
 * and for many rows W^ is rebuilt tile by tile in registers (see hlq_set_gemm_path).
 * hlq_quantize produces the codes, scales and zeros from real-valued weights (Alg. 1).
 *
 * Conventions
 *   - Every pointer below is a DEVICE pointer unless it is marked "host".
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *   - Calls are asynchronous on `stream`; the library never allocates, frees or
 *     synchronises, and keeps no pointer after a call returns.  All buffers stay owned by
 *     the caller and must stay alive until the stream has run the call.
 *   - Argument errors are found on the host before anything is launched and are reported
 *     through the return code; nothing aborts or throws across this boundary.
 *   - Supported descriptors: 1 <= q <= 4, G in {32, 64, 128, 256}, K % 128 == 0,
 *     K % G == 0, N % 8 == 0, K, N >= 1, layout == hlq_layout_version()
 *     (anything else: HLQ_ERR_BAD_DESC); K <= 2^21 and N <= 2^20 (beyond: HLQ_ERR_UNSUPPORTED).
 *   - Alignment: packed blobs, workspaces and activations 16 bytes, outputs their element
 *     size; ldx a multiple of 8 when M > 1 (violations: HLQ_ERR_BAD_STRIDE).
 */
#ifndef HLQ_H
#define HLQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    HLQ_OK = 0,
    HLQ_ERR_NULL = 1,             /* a required pointer is NULL                              */
    HLQ_ERR_BAD_DESC = 2,         /* q, G, K, N or layout outside the supported set          */
    HLQ_ERR_UNSUPPORTED = 3,      /* valid request this build has no kernel for              */
    HLQ_ERR_BUFFER_TOO_SMALL = 4, /* packed / workspace buffer smaller than required         */
    HLQ_ERR_BAD_STRIDE = 5,       /* ldx < K, ldy < N, M < 0, or a misaligned pointer / ldx  */
    HLQ_ERR_HIP = 6               /* the HIP runtime refused a launch                        */
} hlq_status;

#define HLQ_API __attribute__((visibility("default")))

typedef enum { HLQ_OUT_F16 = 0, HLQ_OUT_F32 = 1 } hlq_out_dtype;

/* One HLQ weight matrix W[K, N] (K = input features, N = output columns; the paper's
 * W in R^{n x k} of Alg. 1 with n = out-channels and groups along k is the same thing):
 * q bit-planes, quantisation groups of G consecutive k.  `layout` is the version tag
 * of the packed byte layout and must equal hlq_layout_version(). */
typedef struct {
    int32_t K, N, q, G;
    uint32_t layout;
} hlq_desc;

/* Static, NUL-terminated description of a status code (never NULL). */
HLQ_API const char *hlq_status_string(hlq_status s);

/* Version tag of the packed layout this library reads and writes. */
HLQ_API uint32_t hlq_layout_version(void);

/* Size of the packed weight blob.  Equals K*N*(q/8 + 2*(q+1)/G) bytes: q one-bit planes
 * plus q fp16 scales and one fp16 zero per (group, column) -- the bits-per-weight
 * accounting of Table 1 (q + 16(q+1)/G); the layout adds no padding.  `bits` / `meta`
 * (optional, host) receive the byte counts of the two parts (they are interleaved in the
 * blob).  Host-only, no GPU needed. */
HLQ_API hlq_status hlq_packed_bytes(const hlq_desc *d, size_t *total, size_t *bits, size_t *meta);

/* Bytes of caller-provided workspace hlq_lut_gemv / hlq_lut_gemm need for M rows (host-only).
 * The workspace holds split-K arrival counters and partial sums.  It must be passed once
 * through hlq_workspace_init after allocation; every call leaves it initialised, so one
 * workspace can serve any number of successive calls (also of different shapes, if large
 * enough for each).  Two calls that may run concurrently need separate workspaces.
 * The size is that of a call with exactly M rows and is not monotone in M (the split of K is
 * planned per M): a workspace meant for several M must cover the largest of their sizes. */
HLQ_API hlq_status hlq_workspace_bytes(const hlq_desc *d, int64_t M, size_t *bytes);

/* Workspace size for hlq_lut_gemv_batch over `count` descriptors (host array). */
HLQ_API hlq_status hlq_batch_workspace_bytes(int count, const hlq_desc *descs, size_t *bytes);

/* Zero the arrival counters of a freshly allocated workspace (asynchronous on `stream`).
 * REQUIRED once per workspace before its first use.  The kernels cannot tell a counter that was
 * never cleared from one that counts arrivals: with K split across workgroups, a workgroup adds the
 * partial sums when the counter of its column tile reaches (slices - 1), so on memory that does not
 * start at zero that moment never comes, or comes early: the affected outputs are then not written
 * at all (they keep what y held) or are sums over the slices that happened to be there.  No fault, no
 * error code -- wrong numbers.  Launches whose plan does not split K across workgroups do not
 * touch the workspace.  hlq_lut_gemv_static needs no such call. */
HLQ_API hlq_status hlq_workspace_init(void *ws, size_t ws_bytes, void *stream);

/* Alg. 1 (Sec. 4.1; its steps "Bit-Pattern Selection" and "Linear Reconstruction" are defined in
 * Sec. 4.2), the alternating optimisation for HLQ: quantizes W[K, N] group by group (G
 * consecutive k of a column) into the tensors hlq_pack consumes.  Start: uniform grid over the
 * group's [min, max]; then t_max times (the paper uses 10): per weight the nearest of the 2^q
 * values sum_j s_j bit_j(c) + z (ties: smallest code), then (s, z) by least squares given the
 * bits.  fp64 arithmetic.  If the least-squares system of a group is rank deficient (a plane
 * constant over the group, equal or complementary planes, all weights equal), columns are taken in
 * the order 1, b_0, b_1, ... and a column that depends on the earlier ones keeps its previous
 * parameter.  Plane j of the codes belongs to scale j (initially 2^j * Delta).
 *   W         fp32 [K, N] row-major, finite
 *   codes     u8   [K, N]      out; the codes chosen in the last iteration
 *   scales    fp16 [q, K/G, N] out; zeros fp16 [K/G, N] out (rounded to nearest from fp64)
 *   group_err fp32 [K/G, N]    out, may be NULL: squared reconstruction error of each group with
 *                              the unrounded parameters (Eq. 7)
 * 1 <= t_max <= 1000 and K/G <= 65535, else HLQ_ERR_UNSUPPORTED.  Integer codes and fp16
 * parameters only: no workspace. */
HLQ_API hlq_status hlq_quantize(const hlq_desc *d, const float *W, int t_max, uint8_t *codes,
                                uint16_t *scales, uint16_t *zeros, float *group_err, void *stream);

/* Offline step of App. B ("decomposed into q single-bit matrices offline") and of
 * App. D, Weight-Rearrange: split codes into bit-planes and store them so the runtime
 * kernel reads contiguous 128-bit words along the output-column dimension.
 *   codes  u8   [K, N] row-major, bit j of codes[k,n] = plane j (bits >= q must be 0)
 *   scales fp16 [q, K/G, N]  (raw IEEE binary16 bits)
 *   zeros  fp16 [K/G, N]
 *   packed out, packed_bytes >= hlq_packed_bytes().  Integer work only; bijective. */
HLQ_API hlq_status hlq_pack(const hlq_desc *d, const uint8_t *codes, const uint16_t *scales,
                    const uint16_t *zeros, void *packed, size_t packed_bytes, void *stream);

/* Exact inverse of hlq_pack (any of codes / scales / zeros may be NULL to skip it). */
HLQ_API hlq_status hlq_unpack(const hlq_desc *d, const void *packed, uint8_t *codes,
                      uint16_t *scales, uint16_t *zeros, void *stream);

/* y[N] = x[K] @ W^  (M = 1 decode; Sec. 2 "Bit-Serial LUT-Based GEMM" and App. B on weights in the format
 * of Eq. 3: per plane and quant group the dot product
 * <b_j, x>, times s_j, plus z times the group's activation sum).  The per-plane dot products are
 * taken either on the matrix cores (default) or with the 16-entry tables of App. B, see
 * hlq_set_gemv_path; W^ is never formed.
 *   x fp16 [K], finite; y fp16 or fp32 [N] per `out`, overwritten (beta = 0), fp16 by
 *   round-to-nearest-even from the fp32 accumulator.
 *   ws / ws_bytes: workspace of at least hlq_workspace_bytes(d, 1). */
HLQ_API hlq_status hlq_lut_gemv(const hlq_desc *d, const void *packed, const uint16_t *x, void *y,
                        hlq_out_dtype out, void *ws, size_t ws_bytes, void *stream);

/* hlq_lut_gemv for callers that cannot allocate device memory and therefore have no workspace to
 * pass: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * kernels and results as hlq_lut_gemv; the split-K counters and partial sums live in a fixed
 * array of HLQ_STATIC_SCRATCH_BYTES inside the library, one copy per GPU, held until the
 * process ends.  The call allocates nothing and needs no hlq_workspace_init.
 *   - the device that owns `stream` must be the current device of the calling thread;
 *   - a GEMV whose launch plan needs more partial sums than the array holds is refused with
 *     HLQ_ERR_BUFFER_TOO_SMALL before anything is launched (every LLaMA-3.1-8B / 70B layer shape
 *     and the 128256-wide head fit with the built-in plans; forced plans with many K slices on very
 *     wide matrices may not);
 *   - all calls on one GPU share that GPU's array: calls that may overlap in time on one GPU
 *     (different streams, or graphs replayed concurrently) race on it and must use hlq_lut_gemv
 *     with separate workspaces instead.  Calls in stream order are fine, also mixed shapes. */
#define HLQ_STATIC_SCRATCH_BYTES ((size_t)131072 + ((size_t)4 << 20))
HLQ_API hlq_status hlq_lut_gemv_static(const hlq_desc *d, const void *packed, const uint16_t *x, void *y,
                                       hlq_out_dtype out, void *stream);

/* `count` (1..8) independent GEMVs y_i = x_i @ W^_i in ONE launch (the decode GEMVs of a
 * layer that do not depend on each other, e.g. q/k/v or gate/up).  All descriptors must share
 * q and G.  descs, packed, x, y are HOST arrays of length count; packed[i], x[i], y[i] are
 * device pointers with the meaning they have in hlq_lut_gemv.  Results are identical to
 * `count` separate hlq_lut_gemv calls up to fp32 summation order.
 *   ws / ws_bytes: workspace of at least hlq_batch_workspace_bytes(count, descs). */
HLQ_API hlq_status hlq_lut_gemv_batch(int count, const hlq_desc *descs, const void *const *packed,
                                      const uint16_t *const *x, void *const *y, hlq_out_dtype out,
                                      void *ws, size_t ws_bytes, void *stream);

/* Several independent products Y_i[M, N_i] = X_i[M, K_i] @ W^_i in one launch (the GEMMs of a
 * decoder layer: Sec. 2, batched rows).  All problems share q, G and M; X_i row-major with
 * leading dimension ldx[i] >= K_i (a multiple of 8 for M > 1), Y_i with ldy[i] >= N_i; descs,
 * packed, X, ldx, Y, ldy are host arrays of `count` (1..8) entries.  One launch of the few-rows
 * kernel takes all problems up to 4 rows at G >= 128 (4 at G = 64, 2 at G = 32: two row sets);
 * 5..16 rows at G >= 128 go to the many-rows kernel (a small pre-pass that writes the activations in
 * matrix-core operand form into the workspace, then one launch) when the launch is large enough
 * for it to win, see hlq_set_gemm_path; everything else to one launch of the tiled matrix-core
 * kernel (plus one that adds the partial sums when K is cut: the seven GEMMs of an 8B layer run
 * 1.3x faster than as seven calls at M = 2048).  If the
 * lookup formulation is forced the problems run one after the other on the stream.  M = 0 is a
 * no-op.
 *   ws / ws_bytes: workspace of at least hlq_gemm_batch_workspace_bytes(count, descs, M). */
HLQ_API hlq_status hlq_gemm_batch_workspace_bytes(int count, const hlq_desc *descs, int64_t M, size_t *bytes);
HLQ_API hlq_status hlq_lut_gemm_batch(int count, const hlq_desc *descs, const void *const *packed,
                                      const uint16_t *const *X, int64_t M, const int64_t *ldx, void *const *Y,
                                      const int64_t *ldy, hlq_out_dtype out, void *ws, size_t ws_bytes,
                                      void *stream);

/* Tuning knob (process-wide; for benchmarks and tests.  Each of the knobs below is one atomic value:
 * setting it while another thread launches is safe, and that launch uses the old or the new value;
 * there is no per-call or per-thread setting): force the launch shape
 * of the GEMV kernel -- column tiles per wavefront (1 or 2), wavefronts per workgroup (1..16),
 * chunks of 128 k per wavefront -- instead of the built-in choice.  0 leaves a value automatic.
 * Results stay within the documented tolerance for every setting; only speed changes.
 * Values outside the ranges above: HLQ_ERR_UNSUPPORTED. */
HLQ_API hlq_status hlq_set_gemv_plan(int tiles_per_wave, int waves_per_workgroup, int chunks_per_wave);

/* Host-only: the work split hlq_lut_gemv_batch (M = 1) or the few-rows / many-rows launch of
 * hlq_lut_gemm_batch (2 <= M <= rows one pass carries: 16 at G >= 128, 4 at G = 64, 2 at G = 32) would use for these `count` problems with the knobs as they
 * are now; nothing is launched and no GPU is needed.  For tests and tools: every K slice of a
 * plan starts inside K, i.e. (slices - 1) * chunks_per_slice < K / 128.
 *   descs host array of `count` (1..8) descriptors sharing q and G; out host array of `count`.
 * M outside that range: HLQ_ERR_UNSUPPORTED. */
typedef struct {
    int32_t formulation;          /* 1 = table lookups, 2 = matrix cores                             */
    int32_t waves_per_workgroup;  /* wavefronts of a workgroup                                       */
    int32_t waves_per_tile;       /* of those, the wavefronts that share one column tile's K slice   */
    int32_t chunks_per_slice;     /* chunks of 128 k per K slice (a slice = one workgroup's share)   */
    int32_t slices;               /* K slices, i.e. partial sums per output in the workspace         */
    int32_t tile_groups;          /* groups of column tiles, one workgroup per (group, slice)        */
    int32_t first_block, blocks;  /* this problem's range of workgroups in the launch                */
} hlq_gemv_plan_info;
HLQ_API hlq_status hlq_gemv_plan_query(int count, const hlq_desc *descs, int64_t M, hlq_gemv_plan_info *out);

/* Tuning knob (process-wide, atomic): formulation of the per-plane dot products in
 * hlq_lut_gemv / hlq_lut_gemv_batch.  0 = automatic, 1 = table lookups (App. B), 2 = matrix
 * cores (plane words expanded to 4-bit floats, activations as an exact sum of four 8-bit
 * floats; the matrix core keeps 13 bits below the largest product of an 8-element run, so a
 * result can differ from exact fp32 accumulation by about 1e-4 of the products' magnitude).
 * 3..6 = table lookups with the table stored as App. D discusses ("Mirror Storage", "Table
 * Quantization"), in a plain kernel written for the comparison: 3 = sixteen fp32 entries (the
 * reference of the comparison), 4 = mirror form, eight fp32 entries of the +-1 re-parametrisation,
 * the other eight by negation (lossless), 5 = sixteen fp16 entries (lossy: entries rounded to
 * nearest even), 6 = sixteen int8 entries with one fp32 scale per table (lossy; outside the 2e-3 bar
 * on layer-sized problems with outlier activations).
 * Other values: HLQ_ERR_UNSUPPORTED.  Activations must be finite. */
HLQ_API hlq_status hlq_set_gemv_path(int path);

/* Tuning knob (process-wide, atomic): formulation used by hlq_lut_gemm for M > 1.
 * 0 = automatic (matrix cores from M = 2 on: the lookup kernel for M > 1 is a plain first version --
 *     tables shared per workgroup, two barriers per step -- and is kept as the method's own formulation
 *     for reference, not as a tuned competitor),
 * 1 = table lookups always,
 * 2 = matrix cores always: for a few rows (M <= 4 at G >= 128, <= 2 at G = 64, 1 at G = 32) the
 *     GEMV kernel of hlq_set_gemv_path(2) with several activation rows per operand, for 5..16 rows on large
 *     problems (G >= 128) the many-rows kernel, otherwise the tiled kernel that rebuilds W^ in fp16 registers
 *     (hlq_lut_gemm_batch keeps up to twice as many rows on the GEMV kernel at G <= 64),
 * 3 = as 2 but never the few-rows GEMV kernel,
 * 4 = as 2, and 3..16 rows (G >= 128) always go to the many-rows kernel (by default only when the call or grouped
 *     launch is large enough for it to win: from 4096 chunk-tiles of 64 columns x 128 k at q >= 3 and 12000 at
 *     q <= 2 for 5..8 rows, from 2400 resp. 20000 for 9..16 rows, smaller ones going to the tiled kernel; 3 and 4
 *     rows from 20000 chunk-tiles at q = 4, 4 rows from 40000 at q = 3 and 60000 at q <= 2, otherwise they stay
 *     on the few-rows GEMV kernel).
 * Other values: HLQ_ERR_UNSUPPORTED.  The fp16-rebuild kernel represents scales up to |s_j| < 512 (and
 * zeros of that size); it checks what it loads, and a call whose weights lie outside is computed again
 * by an fp32 kernel launched behind it (slow, but right for every finite fp16 parameter). */
HLQ_API hlq_status hlq_set_gemm_path(int path);

/* Y[M, N] = X[M, K] @ W^  (same procedure with one table set per row, the decoded
 * weight words shared by all rows; by default, from M = 2 on, the per-plane products run on the
 * matrix cores, and from a few rows on the same product is
 * computed as a dense contraction on the matrix cores with W^ rebuilt tile by tile in
 * registers -- see hlq_set_gemm_path).  X row-major with leading dimension ldx >= K (in
 * elements), Y row-major with ldy >= N.  M = 0 is a no-op.
 *   ws / ws_bytes: workspace of at least hlq_workspace_bytes(d, M). */
HLQ_API hlq_status hlq_lut_gemm(const hlq_desc *d, const void *packed, const uint16_t *X, int64_t M,
                        int64_t ldx, void *Y, int64_t ldy, hlq_out_dtype out, void *ws,
                        size_t ws_bytes, void *stream);

/* Measurement helper, no part of the method: read `bytes` of device memory once with 128-bit
 * loads, `blocks` workgroups of 256 lanes each taking one contiguous share (0 = 2048), and store
 * one checksum word per workgroup to `sink`.  Benchmarks time it on as many bytes as a GEMV launch
 * reads, as the read-only reference beside the published bandwidth figure.
 *   src 16-byte aligned, bytes a multiple of 16 (else HLQ_ERR_BAD_STRIDE); 0 <= blocks <= 65536
 *   (else HLQ_ERR_UNSUPPORTED); sink_bytes >= 4 * (workgroups launched) <= 4 * max(blocks, 1) resp.
 *   8192 for blocks = 0 (else HLQ_ERR_BUFFER_TOO_SMALL). */
HLQ_API hlq_status hlq_stream_read(const void *src, size_t bytes, int blocks, void *sink, size_t sink_bytes,
                                   void *stream);

/* The same read with its shape as arguments, for sweeps that look for the fastest plain read the
 * machine does on a given footprint: `unroll` independent 128-bit loads in flight per lane and loop
 * trip (1, 2, 4, 8 or 16; else HLQ_ERR_UNSUPPORTED), `temporal` != 0 for default-policy loads
 * instead of streaming (non-temporal) ones.  hlq_stream_read is unroll 4, streaming. */
HLQ_API hlq_status hlq_stream_read_shaped(const void *src, size_t bytes, int blocks, int unroll, int temporal,
                                          void *sink, size_t sink_bytes, void *stream);

/* Measurement helper, no part of the method: a loop of nothing but one matrix-core instruction on register
 * operands.  kind 0: the fp16 instruction the tiled prefill kernel uses (v_mfma_f32_32x32x16_f16), 16 * iters
 * instructions per wavefront in four accumulator chains; kind 1: the 8-bit x 4-bit instruction of the bit-plane
 * GEMV kernels (v_mfma_f32_16x16x128_f8f6f4 with bf8 and fp4 operands), 32 * iters instructions per wavefront in
 * eight chains; other kinds HLQ_ERR_UNSUPPORTED.  `blocks` workgroups of four
 * wavefronts each load four operand sets from `operands` (device, 16-byte aligned,
 * operand_bytes a multiple of 16, between 16 bytes and 1 GiB, else HLQ_ERR_BAD_STRIDE; fp16 values for kind 0,
 * any bytes for kind 1, where the top exponent bit of every bf8 code is cleared; wavefronts take
 * successive 1 KiB units, wrapping around);
 * one float per lane goes to `sink` (sink_bytes >= blocks * 1024, else
 * HLQ_ERR_BUFFER_TOO_SMALL).  *flop (host, may be NULL) receives the floating-point operations of the
 * launch.  1 <= iters <= 2^20, 1 <= blocks <= 65536 (else HLQ_ERR_UNSUPPORTED).  Benchmarks time it with
 * constant and with random operand data as the matrix-core ceiling beside the prefill GEMM. */
HLQ_API hlq_status hlq_mfma_probe(int kind, const void *operands, size_t operand_bytes, int iters, int blocks, void *sink,
                                  size_t sink_bytes, double *flop, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* HLQ_H */
