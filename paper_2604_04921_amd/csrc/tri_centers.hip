// Offline calibration (Section 4.1; Appendix B.5): per (layer, query head, band) the complex mean
// of the pre-RoPE query samples and the mean of their moduli.
#include "tri_internal.h"

namespace tri {

namespace {

struct CentersArgs {
    const void *q;  // [T][L][Hq][d]
    float *out;     // [L][Hq][F][3], or NULL: leave the sums in `sums`
    double *sums;   // [L][Hq][F][3] running sums (streaming calibration), or NULL
    int64_t T;
    int32_t L, Hq, pairs, is_bf16;
    int32_t first;  // sums: 1 = overwrite, 0 = add to what is there
};

constexpr int kCenterParts = 16;

__device__ __forceinline__ double load_q(const CentersArgs &a, int64_t i)
{
    if (a.is_bf16) return (double)__uint_as_float((uint32_t)((const uint16_t *)a.q)[i] << 16);
    return (double)((const float *)a.q)[i];
}

// grid (Hq, L), block F * 16: thread = (band, token residue mod 16); double sums, fixed order.
__global__ __launch_bounds__(kBands *kCenterParts) void centers_kernel(CentersArgs a)
{
    __shared__ double part[kCenterParts][kBands][3];
    const int f = threadIdx.x % kBands, r = threadIdx.x / kBands;
    const int h = blockIdx.x, l = blockIdx.y;
    const int ire = a.pairs == TRI_PAIR_HALF ? f : 2 * f;
    const int iim = a.pairs == TRI_PAIR_HALF ? f + kBands : 2 * f + 1;
    double sre = 0.0, sim = 0.0, sab = 0.0;
    for (int64_t t = r; t < a.T; t += kCenterParts) {
        const int64_t row = ((t * a.L + l) * a.Hq + h) * kHeadDim;
        const double re = load_q(a, row + ire), im = load_q(a, row + iim);
        sre += re;
        sim += im;
        sab += sqrt(re * re + im * im);
    }
    part[r][f][0] = sre;
    part[r][f][1] = sim;
    part[r][f][2] = sab;
    __syncthreads();
    if (r == 0) {
        double t0 = 0.0, t1 = 0.0, t2 = 0.0;
        for (int k = 0; k < kCenterParts; ++k) {
            t0 += part[k][f][0];
            t1 += part[k][f][1];
            t2 += part[k][f][2];
        }
        const int64_t e = (((int64_t)l * a.Hq + h) * kBands + f) * 3;
        if (a.sums) {   // one thread owns the entry: a plain read-modify-write, chunks arrive in stream order
            double *o = a.sums + e;
            o[0] = a.first ? t0 : o[0] + t0;
            o[1] = a.first ? t1 : o[1] + t1;
            o[2] = a.first ? t2 : o[2] + t2;
        } else {
            float *o = a.out + e;
            o[0] = (float)(t0 / (double)a.T);
            o[1] = (float)(t1 / (double)a.T);
            o[2] = (float)(t2 / (double)a.T);
        }
    }
}

// sums / total tokens -> the statistics table
__global__ __launch_bounds__(256) void centers_finalize_kernel(const double *sums, double total, int64_t n, float *out)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) out[i] = (float)(sums[i] / total);
}

struct DiagArgs {
    const float *q;      // [L][Hq][F][3]
    const float *k;      // [L][Hkv][F][3] or NULL
    float *mrl;          // [L][Hq][F]
    float *contrib;      // [L][Hq][F] or NULL
    int32_t *top;        // [L][Hq][K] or NULL
    int32_t Hq, Hkv, K;
};

// Appendix B.5: R_f = ||E[q_f]|| / E||q_f||.  Appendix B.7: C_f = E||q_f|| E||k_f|| and the K bands with the
// largest C_f (equal contributions: the lower band first).  grid (Hq, L), block F: thread = band.
__global__ __launch_bounds__(kBands) void diagnostics_kernel(DiagArgs a)
{
    __shared__ float cf[kBands];
    const int f = threadIdx.x, h = blockIdx.x, l = blockIdx.y;
    const int64_t e = ((int64_t)l * a.Hq + h) * kBands + f;
    const float *q = a.q + e * 3;
    const double ab = (double)q[2];
    a.mrl[e] = ab > 0.0 ? (float)(hypot((double)q[0], (double)q[1]) / ab) : 0.f;
    if (!a.k) return;
    const int G = a.Hq / a.Hkv;
    const float *k = a.k + (((int64_t)l * a.Hkv + h / G) * kBands + f) * 3;
    const float c = (float)(ab * (double)k[2]);
    if (a.contrib) a.contrib[e] = c;
    if (!a.top) return;
    cf[f] = c;
    __syncthreads();
    int rank = 0;
    for (int o = 0; o < kBands; ++o) rank += (cf[o] > c || (cf[o] == c && o < f)) ? 1 : 0;
    if (rank < a.K) a.top[((int64_t)l * a.Hq + h) * a.K + rank] = f;
}

}  // namespace

tri_status launch_centers(const tri_model &m, const void *q, int32_t q_dtype, int64_t n_tokens, float *out,
                          double *sums, int32_t first, hipStream_t st)
{
    CentersArgs a{q, out, sums, n_tokens, m.n_layers, m.n_q_heads, m.pairs, q_dtype == TRI_BF16 ? 1 : 0, first};
    hipLaunchKernelGGL(centers_kernel, dim3(m.n_q_heads, m.n_layers), dim3(kBands * kCenterParts), 0, st, a);
    return hip_status("centers_kernel");
}

tri_status launch_centers_finalize(const tri_model &m, const double *sums, int64_t total_tokens, float *out,
                                   hipStream_t st)
{
    const int64_t n = (int64_t)m.n_layers * m.n_q_heads * kBands * 3;
    hipLaunchKernelGGL(centers_finalize_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, sums,
                       (double)total_tokens, n, out);
    return hip_status("centers_finalize_kernel");
}

tri_status launch_diagnostics(const tri_model &m, const float *q_centers, const float *k_centers, float *mrl,
                              float *contrib, int32_t top_k, int32_t *top, hipStream_t st)
{
    DiagArgs a{q_centers, k_centers, mrl, contrib, top, m.n_q_heads, m.n_kv_heads, top_k};
    hipLaunchKernelGGL(diagnostics_kernel, dim3(m.n_q_heads, m.n_layers), dim3(kBands), 0, st, a);
    return hip_status("diagnostics_kernel");
}

}  // namespace tri
