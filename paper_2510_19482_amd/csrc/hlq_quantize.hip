// hlq_quantize: Alg. 1 (Sec. 4.1, "Alternating Optimization for Hierarchical Linear Quantization"; its two steps are
// defined in Sec. 4.2 under "Bit-Pattern Selection" and "Linear Reconstruction") --
// produces the codes, per-plane scales and zero points that hlq_pack consumes.
//
//   per group of G consecutive k of a column:  Delta = (max - min) / (2^q - 1),
//   s = [Delta, 2 Delta, ...], z = min;  then T_max times
//     bit-pattern selection   code = argmin_c | (w - z) - sum_j s_j bit_j(c) |      (Bit-Pattern Selection)
//     linear reconstruction   (s, z) = least squares of w ~ sum_j s_j b_j + z        (Linear Reconstruction, LSE)
//
// Groups are independent (App. C), so the unit of work is one lane = one (group, column).  The lane
// reads its G weights once, into registers (G fp32 values; lanes of a wavefront hold adjacent
// columns, so each of the G loads is one coalesced 256-byte read of a row of W and all G are in
// flight together), and every later step works from there: W is read from HBM exactly once and the
// kernel is bound by fp64 arithmetic (2^q candidate distances per weight and iteration).  Within
// a pass a weight's code is chosen and immediately folded into the sums the least-squares step
// needs -- the integer Gram matrix of [1 b_0 .. b_{q-1}] and the fp64 right-hand side -- so nothing
// per weight is stored until the last iteration writes the codes.  All arithmetic is fp64: the
// step is offline, and decisions (the argmin) then agree with an fp64 reference except at exact
// ties.
//
// Rank-deficient systems (a plane constant over the group, equal or complementary planes, all
// weights equal): columns are taken in the order 1, b_0, b_1, ...; a column that depends linearly on
// the earlier ones keeps its previous parameter, whose contribution moves to the right-hand side.
// Dependence among the columns is a property of the SET of codes present in the group, so it is
// decided exactly on the small integer Gram matrix of the distinct rows [1 bits(c)] (entries <= 16):
// fraction-free elimination in column order, in which a zero pivot (the Gram determinant of the
// independent columns so far plus this one) marks a dependent column, which is then skipped.
// Every loop below has compile-time bounds and indices, so all of this lives in registers.
#include "hlq_internal.h"
#include <type_traits>

#pragma clang fp contract(off)

namespace {

template <int Q, int G>
__global__ void __launch_bounds__(256)
hlq_quantize_kernel(const float *__restrict__ W, int K, int N, int t_max, uint8_t *__restrict__ codes,
                    uint16_t *__restrict__ scales, uint16_t *__restrict__ zeros, float *__restrict__ group_err)
{
    constexpr int NC = 1 << Q, P = Q + 1;
    const int n = (int)(blockIdx.x * 256 + threadIdx.x);
    const int gi = (int)blockIdx.y;
    if (n >= N) return;
    const int ngroups = K / G;
    const float *w0 = W + (size_t)gi * G * N + n;
    uint8_t *c0 = codes + (size_t)gi * G * N + n;

    // groups of up to 128 weights stay in registers; longer ones are re-read (from L2) every pass
    constexpr bool RESIDENT = G <= 128;
    constexpr int GR = RESIDENT ? G : 1;
    float wv[GR];
    float lof, hif;   // Alg. 1 steps 2-3 (min / max are exact in fp32)
    if constexpr (RESIDENT) {
#pragma unroll
        for (int i = 0; i < G; ++i) wv[i] = w0[(size_t)i * N];
        lof = hif = wv[0];
#pragma unroll
        for (int i = 1; i < G; ++i) {
            lof = wv[i] < lof ? wv[i] : lof;
            hif = wv[i] > hif ? wv[i] : hif;
        }
    } else {
        lof = hif = w0[0];
#pragma unroll 8
        for (int i = 1; i < G; ++i) {
            const float v = w0[(size_t)i * N];
            lof = v < lof ? v : lof;
            hif = v > hif ? v : hif;
        }
    }
    auto weight = [&](int i) -> float {
        if constexpr (RESIDENT) {
            // opaque to the optimiser, so the fp64 copies are made per use instead of being kept
            // for the whole kernel (which would double the registers held)
            asm volatile("" : "+v"(wv[i]));
            return wv[i];
        } else {
            return w0[(size_t)i * N];
        }
    };
    const double lo = (double)lof, hi = (double)hif;
    const double delta = (hi - lo) / (double)(NC - 1);
    double theta[P];   // theta[0] = z, theta[1 + j] = s_j
    theta[0] = lo;
#pragma unroll
    for (int j = 0; j < Q; ++j) theta[1 + j] = delta * (double)(1 << j);

    // one iteration of Alg. 1; the last one also stores the codes (a separate instantiation, so that
    // the G store addresses are not kept in registers across the other iterations)
    auto iteration = [&](auto last_c) {
        constexpr bool last = decltype(last_c)::value;
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
#pragma unroll(RESIDENT ? G : 8)
        for (int i = 0; i < G; ++i) {
            const double w = (double)weight(i);
            const double what = w - z;
            int best = 0;
            double bd = fabs(what - V[0]);
#pragma unroll
            for (int c = 1; c < NC; ++c) {   // first minimum wins ties
                const double d = fabs(what - V[c]);
                best = d < bd ? c : best;
                bd = __builtin_fmin(bd, d);
            }
            present |= 1u << best;
            rw += w;
#pragma unroll
            for (int j = 0; j < Q; ++j) {
                const int bj = (best >> j) & 1;
                nb[j] += bj;
                rb[j] = __builtin_fma((double)bj, w, rb[j]);   // bj * w is exact: same rounding as an add
#pragma unroll
                for (int k = j + 1; k < Q; ++k) nbb[j][k] += bj & (best >> k);
            }
            if constexpr (last) c0[(size_t)i * N] = (uint8_t)best;
            // keep the instruction scheduler from converting many weights ahead (register pressure)
            if (RESIDENT && (i & 3) == 3) __builtin_amdgcn_sched_barrier(0);
        }

        // the sums are complete here; without this the optimiser postpones them past the branches
        // below and keeps every weight's code in a register until then
#pragma unroll
        for (int j = 0; j < Q; ++j) {
            asm volatile("" : "+v"(rb[j]), "+v"(nb[j]));
#pragma unroll
            for (int k = j + 1; k < Q; ++k) asm volatile("" : "+v"(nbb[j][k]));
        }
        asm volatile("" : "+v"(rw), "+v"(present));

        // ---- which columns of [1 b_0 .. b_{Q-1}] are independent ---------------------------------------------
        // Fraction-free elimination on the Gram matrix of the distinct rows present.  Every
        // intermediate is a minor of that matrix: a sum over at most C(16,5) row subsets of squared
        // determinants of 0/1 matrices of order <= 5 (each <= 5), so below 2^17; products and their
        // differences stay below 2^35 and the divisions are exact, hence fp64 computes them exactly.
        double gm[P][P];
#pragma unroll
        for (int a = 0; a < P; ++a)
#pragma unroll
            for (int b = 0; b < P; ++b) {
                int cnt = 0;
#pragma unroll
                for (int c = 0; c < NC; ++c) {
                    const int ra = a == 0 ? 1 : (c >> (a - 1)) & 1, rc = b == 0 ? 1 : (c >> (b - 1)) & 1;
                    if (ra & rc) cnt += (int)((present >> c) & 1u);
                }
                gm[a][b] = (double)cnt;
            }
        bool is_act[P];
        double prev = 1.0;
#pragma unroll
        for (int k = 0; k < P; ++k) {
            const double pv = gm[k][k];
            is_act[k] = pv != 0.0;
            if (is_act[k]) {
#pragma unroll
                for (int i = k + 1; i < P; ++i)
#pragma unroll
                    for (int j = k + 1; j < P; ++j) gm[i][j] = (gm[i][j] * pv - gm[i][k] * gm[k][j]) / prev;
                prev = pv;
            }
        }

        // ---- linear reconstruction: normal equations; a dependent column becomes the identity equation
        //      theta = previous value and its contribution moves to the right-hand side ----------------------
        double A[P][P], r[P];
        A[0][0] = (double)G;
        r[0] = rw;
#pragma unroll
        for (int j = 0; j < Q; ++j) {
            A[0][1 + j] = A[1 + j][0] = (double)nb[j];
            A[1 + j][1 + j] = (double)nb[j];
            r[1 + j] = rb[j];
#pragma unroll
            for (int k = j + 1; k < Q; ++k) A[1 + j][1 + k] = A[1 + k][1 + j] = (double)nbb[j][k];
        }
#pragma unroll
        for (int a = 0; a < P; ++a) {
            double v = r[a];
#pragma unroll
            for (int col = 0; col < P; ++col)
                if (col != a && !is_act[col]) v -= A[a][col] * theta[col];
            r[a] = is_act[a] ? v : theta[a];
        }
#pragma unroll
        for (int a = 0; a < P; ++a)
#pragma unroll
            for (int b = 0; b < P; ++b)
                if (!is_act[a] || !is_act[b]) A[a][b] = a == b ? 1.0 : 0.0;
        // elimination without pivoting: the matrix is symmetric positive definite
#pragma unroll
        for (int k = 0; k < P; ++k) {
            const double inv = 1.0 / A[k][k];
#pragma unroll
            for (int i = k + 1; i < P; ++i) {
                const double f = A[i][k] * inv;
#pragma unroll
                for (int j = k + 1; j < P; ++j) A[i][j] -= f * A[k][j];
                r[i] -= f * r[k];
            }
        }
#pragma unroll
        for (int k = P - 1; k >= 0; --k) {
            double v = r[k];
#pragma unroll
            for (int j = k + 1; j < P; ++j) v -= A[k][j] * theta[j];
            theta[k] = v / A[k][k];
        }
    };
    for (int t = 0; t + 1 < t_max; ++t) iteration(std::false_type{});
    iteration(std::true_type{});

    // ---- outputs: parameters rounded to fp16 (nearest even); error with the unrounded ones ---------------
    zeros[(size_t)gi * N + n] = __builtin_bit_cast(uint16_t, (_Float16)theta[0]);
#pragma unroll
    for (int j = 0; j < Q; ++j) scales[((size_t)j * ngroups + gi) * N + n] = __builtin_bit_cast(uint16_t, (_Float16)theta[1 + j]);
    if (group_err) {
        double e = 0.0;
#pragma unroll(RESIDENT ? G : 8)
        for (int i = 0; i < G; ++i) {
            const int c = c0[(size_t)i * N];
            double v = theta[0];
#pragma unroll
            for (int j = 0; j < Q; ++j) v += theta[1 + j] * (double)((c >> j) & 1);
            const double dlt = (double)weight(i) - v;
            e += dlt * dlt;
        }
        group_err[(size_t)gi * N + n] = (float)e;
    }
}

template <int Q>
void launch_q(const HlqDims &dm, const float *W, int t_max, uint8_t *codes, uint16_t *scales, uint16_t *zeros,
              float *group_err, hipStream_t st)
{
    const dim3 grid((unsigned)((dm.N + 255) / 256), (unsigned)dm.ngroups);
    switch (dm.G) {
    case 32: hlq_quantize_kernel<Q, 32><<<grid, 256, 0, st>>>(W, dm.K, dm.N, t_max, codes, scales, zeros, group_err); break;
    case 64: hlq_quantize_kernel<Q, 64><<<grid, 256, 0, st>>>(W, dm.K, dm.N, t_max, codes, scales, zeros, group_err); break;
    case 128: hlq_quantize_kernel<Q, 128><<<grid, 256, 0, st>>>(W, dm.K, dm.N, t_max, codes, scales, zeros, group_err); break;
    default: hlq_quantize_kernel<Q, 256><<<grid, 256, 0, st>>>(W, dm.K, dm.N, t_max, codes, scales, zeros, group_err); break;
    }
}

} // namespace

hlq_status hlq_launch_quantize(const HlqDims &dm, const float *W, int t_max, uint8_t *codes, uint16_t *scales,
                               uint16_t *zeros, float *group_err, hipStream_t st)
{
    hlq_clear_stale_error();
    if (t_max < 1 || t_max > 1000) return HLQ_ERR_UNSUPPORTED;
    if (dm.ngroups > 65535) return HLQ_ERR_UNSUPPORTED;
    if (dm.G != 32 && dm.G != 64 && dm.G != 128 && dm.G != 256) return HLQ_ERR_UNSUPPORTED;
    switch (dm.q) {
    case 1: launch_q<1>(dm, W, t_max, codes, scales, zeros, group_err, st); break;
    case 2: launch_q<2>(dm, W, t_max, codes, scales, zeros, group_err, st); break;
    case 3: launch_q<3>(dm, W, t_max, codes, scales, zeros, group_err, st); break;
    case 4: launch_q<4>(dm, W, t_max, codes, scales, zeros, group_err, st); break;
    default: return HLQ_ERR_UNSUPPORTED;
    }
    return hlq_hip_status(hipGetLastError());
}
