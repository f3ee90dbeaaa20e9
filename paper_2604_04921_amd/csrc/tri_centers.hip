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

constexpr int kCenterThreads = 512;   // 8 band octets x 64 token residues
constexpr int kCenterWaves = kCenterThreads / 64;

// The (re, im) of bands 8q..8q+7 of the head vector that starts at element `row`: 32 contiguous bytes (bf16,
// interleaved pairs), two 16-byte pieces 128 bytes apart (bf16, half-split), or the fp32 counterparts.
__device__ __forceinline__ void load_octet(const CentersArgs &a, int64_t row, int q, float (&re)[8], float (&im)[8])
{
    const bool half = a.pairs == TRI_PAIR_HALF;
    if (a.is_bf16) {
        const uint16_t *p = (const uint16_t *)a.q + row;
        const uint4 u0 = *reinterpret_cast<const uint4 *>(p + (half ? 8 * q : 16 * q));
        const uint4 u1 = *reinterpret_cast<const uint4 *>(p + (half ? kBands + 8 * q : 16 * q + 8));
        const uint32_t w0[4] = {u0.x, u0.y, u0.z, u0.w}, w1[4] = {u1.x, u1.y, u1.z, u1.w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            if (half) {   // u0 = 8 real parts, u1 = 8 imaginary parts
                re[2 * k] = __uint_as_float(w0[k] << 16);
                re[2 * k + 1] = __uint_as_float(w0[k] & 0xffff0000u);
                im[2 * k] = __uint_as_float(w1[k] << 16);
                im[2 * k + 1] = __uint_as_float(w1[k] & 0xffff0000u);
            } else {      // u0 = bands 0-3 as (re, im) pairs, u1 = bands 4-7
                re[k] = __uint_as_float(w0[k] << 16);
                im[k] = __uint_as_float(w0[k] & 0xffff0000u);
                re[4 + k] = __uint_as_float(w1[k] << 16);
                im[4 + k] = __uint_as_float(w1[k] & 0xffff0000u);
            }
        }
    } else {
        const float *p = (const float *)a.q + row;
#pragma unroll
        for (int k = 0; k < 2; ++k) {
            if (half) {
                const float4 r4 = *reinterpret_cast<const float4 *>(p + 8 * q + 4 * k);
                const float4 i4 = *reinterpret_cast<const float4 *>(p + kBands + 8 * q + 4 * k);
                re[4 * k] = r4.x, re[4 * k + 1] = r4.y, re[4 * k + 2] = r4.z, re[4 * k + 3] = r4.w;
                im[4 * k] = i4.x, im[4 * k + 1] = i4.y, im[4 * k + 2] = i4.z, im[4 * k + 3] = i4.w;
            } else {
                const float4 a4 = *reinterpret_cast<const float4 *>(p + 16 * q + 8 * k);
                const float4 b4 = *reinterpret_cast<const float4 *>(p + 16 * q + 8 * k + 4);
                re[4 * k] = a4.x, im[4 * k] = a4.y, re[4 * k + 1] = a4.z, im[4 * k + 1] = a4.w;
                re[4 * k + 2] = b4.x, im[4 * k + 2] = b4.y, re[4 * k + 3] = b4.z, im[4 * k + 3] = b4.w;
            }
        }
    }
}

// grid (Hq, L), block 512: thread = (token residue r mod 64, band octet q); eight neighbouring threads read one
// whole head vector with 16-byte loads.  Double sums in a fixed order: per thread over its tokens, then a
// butterfly over the 8 residues of a wave, then the 8 waves in order.
__global__ __launch_bounds__(kCenterThreads) void centers_kernel(CentersArgs a)
{
    __shared__ double part[kCenterWaves][kBands][3];
    const int q = threadIdx.x & 7, r = threadIdx.x >> 3, wave = threadIdx.x >> 6;
    const int h = blockIdx.x, l = blockIdx.y;
    double sre[8], sim[8], sab[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) sre[k] = sim[k] = sab[k] = 0.0;
    for (int64_t t = r; t < a.T; t += kCenterThreads / 8) {
        float re[8], im[8];
        load_octet(a, ((t * a.L + l) * a.Hq + h) * kHeadDim, q, re, im);
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const double x = (double)re[k], y = (double)im[k];
            sre[k] += x;
            sim[k] += y;
            sab[k] += sqrt(x * x + y * y);
        }
    }
#pragma unroll
    for (int k = 0; k < 8; ++k) {
#pragma unroll
        for (int o = 8; o < 64; o <<= 1) {   // lanes that differ in the residue only
            sre[k] += __shfl_xor(sre[k], o, 64);
            sim[k] += __shfl_xor(sim[k], o, 64);
            sab[k] += __shfl_xor(sab[k], o, 64);
        }
        if ((threadIdx.x & 63) < 8) {
            part[wave][8 * q + k][0] = sre[k];
            part[wave][8 * q + k][1] = sim[k];
            part[wave][8 * q + k][2] = sab[k];
        }
    }
    __syncthreads();
    if (threadIdx.x < kBands) {
        const int f = threadIdx.x;
        double t0 = 0.0, t1 = 0.0, t2 = 0.0;
        for (int k = 0; k < kCenterWaves; ++k) {
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
    hipLaunchKernelGGL(centers_kernel, dim3(m.n_q_heads, m.n_layers), dim3(kCenterThreads), 0, st, a);
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
