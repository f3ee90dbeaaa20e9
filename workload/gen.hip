// Device-side synthetic workload generator (inputs only: no scoring arithmetic lives here).
// Counter-based: every value is a pure function of (seed, tag, element index), so any slice
// can be regenerated independently.  Built into its own library, apart from libtri.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

__device__ __forceinline__ uint64_t mix64(uint64_t z)
{
    z += 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

__device__ __forceinline__ uint64_t stream_key(uint64_t seed, uint64_t tag)
{
    return mix64(mix64(seed) ^ (tag * 0xD6E8FEB86659FD93ull));
}

// two independent standard normals from one 64-bit hash (Box-Muller)
__device__ __forceinline__ void normal_pair(uint64_t h, float *a, float *b)
{
    const float u1 = ((float)(h >> 40) + 0.5f) * (1.0f / 16777216.0f);
    const float u2 = ((float)(h & 0xFFFFFFull) + 0.5f) * (1.0f / 16777216.0f);
    const float r = sqrtf(-2.0f * logf(u1));
    float s, c;
    sincosf(6.28318530717958647692f * u2, &s, &c);
    *a = r * c;
    *b = r * s;
}

__device__ __forceinline__ uint32_t bf16_rne(float x)
{
    uint32_t u = __float_as_uint(x);
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

struct SampleArgs {
    void *out;             // [rows][128], dense
    const float *centres;  // [n_centres][64][2]
    int64_t rows;
    int64_t B, C, Dn;      // row = ((a*B + b)*C + c)*Dn + dn; centre index = a*C + c
    float noise, outlier_p, outlier_scale;
    uint64_t key_noise, key_outlier;
    int32_t is_bf16;
};

// thread = (row, group of 4 bands)
__global__ __launch_bounds__(256) void sample_kernel(SampleArgs a)
{
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t row = t >> 4;
    const int fg = (int)(t & 15);
    if (row >= a.rows) return;
    const int64_t c = (row / a.Dn) % a.C;
    const int64_t aa = row / (a.Dn * a.C * a.B);
    const float *ct = a.centres + ((aa * a.C + c) * 64 + fg * 4) * 2;
    float scale = 1.0f;
    if (a.outlier_p > 0.f) {
        const uint64_t h = mix64(a.key_outlier + (uint64_t)row);
        if (((float)(h >> 40) + 0.5f) * (1.0f / 16777216.0f) < a.outlier_p) scale = a.outlier_scale;
    }
    float v[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float cr = ct[2 * i], ci = ct[2 * i + 1];
        const float sd = a.noise * sqrtf(cr * cr + ci * ci) * 0.70710678118654752440f;
        float n1, n2;
        normal_pair(mix64(a.key_noise + (uint64_t)(row * 64 + fg * 4 + i)), &n1, &n2);
        v[2 * i] = (cr + sd * n1) * scale;
        v[2 * i + 1] = (ci + sd * n2) * scale;
    }
    if (a.is_bf16) {
        uint4 o;
        o.x = bf16_rne(v[0]) | (bf16_rne(v[1]) << 16);
        o.y = bf16_rne(v[2]) | (bf16_rne(v[3]) << 16);
        o.z = bf16_rne(v[4]) | (bf16_rne(v[5]) << 16);
        o.w = bf16_rne(v[6]) | (bf16_rne(v[7]) << 16);
        reinterpret_cast<uint4 *>(a.out)[row * 16 + fg] = o;
    } else {
        float4 *o = reinterpret_cast<float4 *>(a.out) + (row * 32 + fg * 2);
        o[0] = make_float4(v[0], v[1], v[2], v[3]);
        o[1] = make_float4(v[4], v[5], v[6], v[7]);
    }
}

struct NormalArgs {
    void *out;
    int64_t n8;  // number of 8-element groups
    uint64_t key;
    int32_t is_bf16;
};

__global__ __launch_bounds__(256) void normal_kernel(NormalArgs a)
{
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= a.n8) return;
    float v[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) normal_pair(mix64(a.key + (uint64_t)(t * 4 + i)), &v[2 * i], &v[2 * i + 1]);
    if (a.is_bf16) {
        uint4 o;
        o.x = bf16_rne(v[0]) | (bf16_rne(v[1]) << 16);
        o.y = bf16_rne(v[2]) | (bf16_rne(v[3]) << 16);
        o.z = bf16_rne(v[4]) | (bf16_rne(v[5]) << 16);
        o.w = bf16_rne(v[6]) | (bf16_rne(v[7]) << 16);
        reinterpret_cast<uint4 *>(a.out)[t] = o;
    } else {
        float4 *o = reinterpret_cast<float4 *>(a.out) + t * 2;
        o[0] = make_float4(v[0], v[1], v[2], v[3]);
        o[1] = make_float4(v[4], v[5], v[6], v[7]);
    }
}

// Streaming probe: every wave reads its own contiguous range 4 KB at a time (16 bytes per lane and load) and,
// every `write_every` reads (0 = never), writes 256 bytes.  Measures what the HBM delivers for a pure read
// stream and for a read stream with a thin write stream mixed in -- the two regimes of the score kernel.
typedef unsigned int probe_u4 __attribute__((ext_vector_type(4)));

template <bool NT>   // NT: loads carry the non-temporal hint (data read once)
__global__ __launch_bounds__(512) void stream_probe_kernel(const uint4 *__restrict__ in, uint32_t *__restrict__ out,
                                                           uint32_t *sink, int64_t per_wave16, int write_every)
{
    const int lane = threadIdx.x & 63;
    const int64_t wave = (int64_t)blockIdx.x * 8 + (threadIdx.x >> 6);
    const uint4 *p = in + wave * per_wave16;
    uint32_t *w = out + wave * (per_wave16 / 16);
    uint32_t acc = 0;
    int64_t it = 0, wofs = 0;
    for (int64_t i = 0; i + 256 <= per_wave16; i += 256, ++it) {
        uint4 a[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if constexpr (NT) {
                const probe_u4 t = __builtin_nontemporal_load(reinterpret_cast<const probe_u4 *>(p + i + u * 64 + lane));
                a[u] = make_uint4(t.x, t.y, t.z, t.w);
            } else {
                a[u] = p[i + u * 64 + lane];
            }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) acc ^= a[u].x ^ a[u].y ^ a[u].z ^ a[u].w;
        if (write_every > 0 && (it % write_every) == write_every - 1) {
            w[wofs + lane] = acc;
            wofs += 64;
        }
    }
    if (acc == 0x12345678u) sink[0] = acc;
}

}  // namespace

extern "C" {

// Launch the streaming probe over `bytes` of `in` (device); `out` needs bytes/16 + 4 bytes.  Returns the number
// of bytes the launch reads, or a negative value on error.
int64_t wl_stream_probe(const void *in, int64_t bytes, void *out, int write_every, int nontemporal, void *stream)
{
    if (!in || !out || bytes < (1 << 24)) return -1;
    const int wgs = 4096;
    const int64_t waves = (int64_t)wgs * 8;
    const int64_t per = (bytes / 16 / waves) / 256 * 256;
    uint32_t *o = reinterpret_cast<uint32_t *>(out);
    if (nontemporal)
        hipLaunchKernelGGL(stream_probe_kernel<true>, dim3(wgs), dim3(512), 0, (hipStream_t)stream,
                           reinterpret_cast<const uint4 *>(in), o, o + bytes / 64, per, write_every);
    else
        hipLaunchKernelGGL(stream_probe_kernel<false>, dim3(wgs), dim3(512), 0, (hipStream_t)stream,
                           reinterpret_cast<const uint4 *>(in), o, o + bytes / 64, per, write_every);
    return hipGetLastError() == hipSuccess ? per * waves * 16 : -4;
}

// Samples around per-head centres (keys, calibration queries).  All pointers are device pointers.
int wl_fill_samples(void *out, int is_bf16, const float *centres, int64_t rows, int64_t B, int64_t C, int64_t Dn,
                    float noise, float outlier_p, float outlier_scale, uint64_t seed, uint64_t tag, void *stream)
{
    if (!out || !centres || rows < 0 || B < 1 || C < 1 || Dn < 1) return -1;
    if (rows == 0) return 0;
    const int64_t blocks = (rows * 16 + 255) / 256;
    if (blocks > 0x7FFFFFFF) return -1;
    SampleArgs a{out, centres, rows, B, C, Dn, noise, outlier_p, outlier_scale, 0, 0, is_bf16};
    // host copies of the device hash so that the stream keys are computed once
    auto hmix = [](uint64_t z) {
        z += 0x9E3779B97F4A7C15ull;
        z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
        z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
        return z ^ (z >> 31);
    };
    a.key_noise = hmix(hmix(seed) ^ (tag * 0xD6E8FEB86659FD93ull));
    a.key_outlier = hmix(hmix(seed) ^ ((tag + 1000) * 0xD6E8FEB86659FD93ull));
    hipLaunchKernelGGL(sample_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream, a);
    return hipGetLastError() == hipSuccess ? 0 : -4;
}

// Unit Gaussians (values).  n must be a multiple of 8.
int wl_fill_normal(void *out, int is_bf16, int64_t n, uint64_t seed, uint64_t tag, void *stream)
{
    if (!out || n < 0 || (n & 7)) return -1;
    if (n == 0) return 0;
    const int64_t n8 = n / 8, blocks = (n8 + 255) / 256;
    if (blocks > 0x7FFFFFFF) return -1;
    auto hmix = [](uint64_t z) {
        z += 0x9E3779B97F4A7C15ull;
        z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
        z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
        return z ^ (z >> 31);
    };
    NormalArgs a{out, n8, hmix(hmix(seed) ^ (tag * 0xD6E8FEB86659FD93ull)), is_bf16};
    hipLaunchKernelGGL(normal_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream, a);
    return hipGetLastError() == hipSuccess ? 0 : -4;
}

}  // extern "C"
