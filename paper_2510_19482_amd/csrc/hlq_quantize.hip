// hlq_quantize: Alg. 1 (Sec. 3.2, "Alternating Optimization for Hierarchical Linear Quantization") --
// produces the codes, per-plane scales and zero points that hlq_pack consumes.
//
//   per group of G consecutive k of a column:  Delta = (max - min) / (2^q - 1),
//   s = [Delta, 2 Delta, ...], z = min;  then T_max times
//     bit-pattern selection   code = argmin_c | (w - z) - sum_j s_j bit_j(c) |      (Eq. 9)
//     linear reconstruction   (s, z) = least squares of w ~ sum_j s_j b_j + z        (Eq. 10)
//
// Groups are independent (App. C), so the unit of work is one lane = one (group, column): the lane
// walks its G weights once for the range and once per iteration; lanes of a wavefront hold adjacent
// columns, so every step of the walk is one coalesced 256-byte read of a row of W (11 passes over
// W in all, served by L2 / the memory-side cache after the first).  Within a pass a weight's code is
// chosen and immediately folded into the sums the least-squares step needs -- the integer Gram
// matrix of [1 b_0 .. b_{q-1}] and the fp64 right-hand side -- so nothing per weight is stored
// until the last iteration writes the codes.  All arithmetic is fp64: the step is offline, and
// decisions (the argmin) then agree with an fp64 reference except at exact ties.
//
// Rank-deficient systems (a plane constant over the group, equal or complementary planes, all
// weights equal): columns are taken in the order 1, b_0, b_1, ...; a column that depends linearly on
// the earlier ones keeps its previous parameter, whose contribution moves to the right-hand side.
// Dependence among the columns is a property of the SET of codes present in the group, so it is
// decided exactly on the small integer Gram matrix of the distinct rows [1 bits(c)] (entries <= 16,
// 64-bit fraction-free elimination cannot overflow).
#include "hlq_internal.h"

#pragma clang fp contract(off)

namespace {

constexpr int QMAX = 4, NP = QMAX + 1;

// exact determinant of the leading n x n part of a small integer matrix given by an index list
// (fraction-free elimination; |entries| <= 16, n <= 5: every intermediate is a minor < 2^31)
__device__ long long det_sub(const int (&gram)[NP][NP], const int (&idx)[NP], int n)
{
    long long m[NP][NP];
    for (int i = 0; i < n; ++i)
        for (int j = 0; j < n; ++j) m[i][j] = gram[idx[i]][idx[j]];
    long long prev = 1;
    int sign = 1;
    for (int k = 0; k + 1 < n; ++k) {
        if (m[k][k] == 0) {
            int sw = -1;
            for (int i = k + 1; i < n; ++i)
                if (m[i][k] != 0) { sw = i; break; }
            if (sw < 0) return 0;
            for (int j = 0; j < n; ++j) { const long long t = m[k][j]; m[k][j] = m[sw][j]; m[sw][j] = t; }
            sign = -sign;
        }
        for (int i = k + 1; i < n; ++i)
            for (int j = k + 1; j < n; ++j) m[i][j] = (m[i][j] * m[k][k] - m[i][k] * m[k][j]) / prev;
        prev = m[k][k];
    }
    return sign * m[n - 1][n - 1];
}

template <int Q>
__global__ void __launch_bounds__(256)
hlq_quantize_kernel(const float *__restrict__ W, int K, int N, int G, int t_max, uint8_t *__restrict__ codes,
                    uint16_t *__restrict__ scales, uint16_t *__restrict__ zeros, float *__restrict__ group_err)
{
    constexpr int NC = 1 << Q, P = Q + 1;
    const int n = (int)(blockIdx.x * 256 + threadIdx.x);
    const int gi = (int)blockIdx.y;
    if (n >= N) return;
    const int ngroups = K / G;
    const float *w0 = W + (size_t)gi * G * N + n;
    uint8_t *c0 = codes + (size_t)gi * G * N + n;

    // Alg. 1 steps 2-3
    double lo = (double)w0[0], hi = lo;
    for (int i = 1; i < G; ++i) {
        const double v = (double)w0[(size_t)i * N];
        lo = v < lo ? v : lo;
        hi = v > hi ? v : hi;
    }
    const double delta = (hi - lo) / (double)(NC - 1);
    double theta[P];   // theta[0] = z, theta[1 + j] = s_j
    theta[0] = lo;
#pragma unroll
    for (int j = 0; j < Q; ++j) theta[1 + j] = delta * (double)(1 << j);

    for (int t = 0; t < t_max; ++t) {
        // candidate values V_c = sum_j s_j bit_j(c)   (step 7)
        double V[NC];
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            double v = 0.0;
#pragma unroll
            for (int j = 0; j < Q; ++j) v += theta[1 + j] * (double)((c >> j) & 1);
            V[c] = v;
        }
        const double z = theta[0];
        int nb[Q], nbb[Q][Q];
        double rb[Q], rw = 0.0;
        unsigned present = 0u;
#pragma unroll
        for (int j = 0; j < Q; ++j) {
            nb[j] = 0;
            rb[j] = 0.0;
#pragma unroll
            for (int k = 0; k < Q; ++k) nbb[j][k] = 0;
        }
        const bool last = t == t_max - 1;
#pragma unroll 8
        for (int i = 0; i < G; ++i) {   // G is a multiple of 32: eight independent loads in flight
            const double w = (double)w0[(size_t)i * N];
            const double what = w - z;
            int best = 0;
            double bd = fabs(what - V[0]);
#pragma unroll
            for (int c = 1; c < NC; ++c) {   // first minimum wins ties
                const double d = fabs(what - V[c]);
                if (d < bd) {
                    bd = d;
                    best = c;
                }
            }
            present |= 1u << best;
            rw += w;
#pragma unroll
            for (int j = 0; j < Q; ++j) {
                const int bj = (best >> j) & 1;
                nb[j] += bj;
                rb[j] += bj ? w : 0.0;
#pragma unroll
                for (int k = j + 1; k < Q; ++k) nbb[j][k] += bj & (best >> k);
            }
            if (last) c0[(size_t)i * N] = (uint8_t)best;
        }

        // ---- linear reconstruction: normal equations of [1 b_0 .. b_{Q-1}] ---------------------------------
        double M[NP][NP], rhs[NP];
        M[0][0] = (double)G;
        rhs[0] = rw;
#pragma unroll
        for (int j = 0; j < Q; ++j) {
            M[0][1 + j] = M[1 + j][0] = (double)nb[j];
            M[1 + j][1 + j] = (double)nb[j];
            rhs[1 + j] = rb[j];
#pragma unroll
            for (int k = j + 1; k < Q; ++k) M[1 + j][1 + k] = M[1 + k][1 + j] = (double)nbb[j][k];
        }
        // which columns are independent: Gram matrix of the distinct rows [1 bits(c)], c present
        int gram[NP][NP];
        for (int a = 0; a < P; ++a)
            for (int bq = 0; bq < P; ++bq) gram[a][bq] = 0;
        for (int c = 0; c < NC; ++c) {
            if (!((present >> c) & 1u)) continue;
            int row[NP];
            row[0] = 1;
            for (int j = 0; j < Q; ++j) row[1 + j] = (c >> j) & 1;
            for (int a = 0; a < P; ++a)
                for (int bq = 0; bq < P; ++bq) gram[a][bq] += row[a] * row[bq];
        }
        int act[NP], nact = 0;
        bool is_act[NP];
        for (int col = 0; col < P; ++col) {
            act[nact] = col;
            is_act[col] = det_sub(gram, act, nact + 1) != 0;
            if (is_act[col]) ++nact;
        }
        // move the dependent columns' contribution (previous parameters) to the right-hand side
        double A[NP][NP], r[NP];
        for (int a = 0; a < nact; ++a) {
            double v = rhs[act[a]];
            for (int col = 0; col < P; ++col)
                if (!is_act[col]) v -= M[act[a]][col] * theta[col];
            r[a] = v;
            for (int bq = 0; bq < nact; ++bq) A[a][bq] = M[act[a]][act[bq]];
        }
        // Gaussian elimination with partial pivoting (the active Gram matrix is positive definite)
        for (int k = 0; k < nact; ++k) {
            int piv = k;
            for (int i = k + 1; i < nact; ++i)
                if (fabs(A[i][k]) > fabs(A[piv][k])) piv = i;
            if (piv != k) {
                for (int j = 0; j < nact; ++j) { const double tt = A[k][j]; A[k][j] = A[piv][j]; A[piv][j] = tt; }
                const double tt = r[k]; r[k] = r[piv]; r[piv] = tt;
            }
            for (int i = k + 1; i < nact; ++i) {
                const double f = A[i][k] / A[k][k];
                for (int j = k; j < nact; ++j) A[i][j] -= f * A[k][j];
                r[i] -= f * r[k];
            }
        }
        for (int k = nact - 1; k >= 0; --k) {
            double v = r[k];
            for (int j = k + 1; j < nact; ++j) v -= A[k][j] * theta[act[j]];
            theta[act[k]] = v / A[k][k];
        }
    }

    // ---- outputs: parameters rounded to fp16 (nearest even); error with the unrounded ones ---------------
    zeros[(size_t)gi * N + n] = __builtin_bit_cast(uint16_t, (_Float16)theta[0]);
#pragma unroll
    for (int j = 0; j < Q; ++j) scales[((size_t)j * ngroups + gi) * N + n] = __builtin_bit_cast(uint16_t, (_Float16)theta[1 + j]);
    if (group_err) {
        double e = 0.0;
        for (int i = 0; i < G; ++i) {
            const int c = c0[(size_t)i * N];
            double v = theta[0];
#pragma unroll
            for (int j = 0; j < Q; ++j) v += theta[1 + j] * (double)((c >> j) & 1);
            const double dlt = (double)w0[(size_t)i * N] - v;
            e += dlt * dlt;
        }
        group_err[(size_t)gi * N + n] = (float)e;
    }
}

} // namespace

hlq_status hlq_launch_quantize(const HlqDims &dm, const float *W, int t_max, uint8_t *codes, uint16_t *scales,
                               uint16_t *zeros, float *group_err, hipStream_t st)
{
    hlq_clear_stale_error();
    if (t_max < 1 || t_max > 1000) return HLQ_ERR_UNSUPPORTED;
    if (dm.ngroups > 65535) return HLQ_ERR_UNSUPPORTED;
    const dim3 grid((unsigned)((dm.N + 255) / 256), (unsigned)dm.ngroups);
    switch (dm.q) {
    case 1: hlq_quantize_kernel<1><<<grid, 256, 0, st>>>(W, dm.K, dm.N, dm.G, t_max, codes, scales, zeros, group_err); break;
    case 2: hlq_quantize_kernel<2><<<grid, 256, 0, st>>>(W, dm.K, dm.N, dm.G, t_max, codes, scales, zeros, group_err); break;
    case 3: hlq_quantize_kernel<3><<<grid, 256, 0, st>>>(W, dm.K, dm.N, dm.G, t_max, codes, scales, zeros, group_err); break;
    case 4: hlq_quantize_kernel<4><<<grid, 256, 0, st>>>(W, dm.K, dm.N, dm.G, t_max, codes, scales, zeros, group_err); break;
    default: return HLQ_ERR_UNSUPPORTED;
    }
    return hlq_hip_status(hipGetLastError());
}
