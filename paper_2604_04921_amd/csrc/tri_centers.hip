// Offline calibration (Section 4.1; Appendix B.5): per (layer, query head, band) the complex mean
// of the pre-RoPE query samples and the mean of their moduli.
#include "tri_internal.h"

namespace tri {

namespace {

struct CentersArgs {
    const void *q;  // [T][L][Hq][d]
    float *out;     // [L][Hq][F][3]
    int64_t T;
    int32_t L, Hq, pairs, is_bf16;
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
        float *o = a.out + (((int64_t)l * a.Hq + h) * kBands + f) * 3;
        o[0] = (float)(t0 / (double)a.T);
        o[1] = (float)(t1 / (double)a.T);
        o[2] = (float)(t2 / (double)a.T);
    }
}

}  // namespace

tri_status launch_centers(const tri_model &m, const void *q, int32_t q_dtype, int64_t n_tokens, float *out,
                          hipStream_t st)
{
    CentersArgs a{q, out, n_tokens, m.n_layers, m.n_q_heads, m.pairs, q_dtype == TRI_BF16 ? 1 : 0};
    hipLaunchKernelGGL(centers_kernel, dim3(m.n_q_heads, m.n_layers), dim3(kBands * kCenterParts), 0, st, a);
    return hip_status("centers_kernel");
}

}  // namespace tri
