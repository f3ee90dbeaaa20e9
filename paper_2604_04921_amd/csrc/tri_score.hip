// Scoring kernels: table fold, per-key score, moments, z-score + max over the GQA group.
//
// Algebra (Sections 4.1-4.2, Appendix B.2).  With q = E[q_f], k = k_f complex, x = p_q + delta - p_k:
//   ||q|| ||k|| cos(omega x + arg q - arg k) = Re( q conj(k) e^{i omega x} )
// and the average over the offsets delta in D is linear, so
//   S~_trig(k) = Re sum_f  Qhat_f * conj( k_f e^{i omega_f p_k} ),
//   Qhat_f = E[q_f] * (1/|D|) sum_delta e^{i omega_f delta} * e^{i omega_f p_q}.
// The norm term does not depend on the offset: S_norm(k) = sum_f c_f |k_f|, c_f = E||q_f|| - ||E[q_f]||.
// The fold kernel builds (Re Qhat, Im Qhat, c) per (layer, sequence, query head, band) in double;
// the score kernel then needs, per key and band, one rotation of the key by its own position,
// one modulus, and three FMAs per query head -- independent of |D|.
#include <atomic>

#include "tri_score_common.h"

namespace tri {

namespace {

constexpr double kTwoPi = 6.283185307179586476925286766559;

struct FoldArgs {
    const float *centers;   // [L][Hq][F][3]
    float *table;           // [L][S][Hkv][F][3][G]
    double *band_rev;       // [F]
    double *phasors;        // [1 + S][F][2]: (0) mean over the offsets of e^{i w delta}; (1 + s) e^{i w cur_pos[s]}
    const int32_t *cur_pos; // [S]
    const int32_t *seq_len; // [S]
    int32_t *work;          // work list of the MFMA score kernel, or NULL when the generic kernel runs
    int32_t chunk_keys;     // keys per entry of that list
    float4 *lane_table;     // relative-position phasor table of the one-key-per-lane kernel to fill in, or NULL
    int32_t max_seq_len;
    int32_t S, Hq, Hkv, G;
    double theta;
    int32_t n_off;
    int32_t variant;        // tri_score_variant
    int64_t offsets[kMaxOffsets];
};

// exp(2 pi i * frac(t * rev)) in double; t * rev is exact enough for |t| < 2^62 * 2^-53 relative
__device__ __forceinline__ void unit_phasor(double t, double rev, double *c, double *s)
{
    double x = t * rev;
    x -= floor(x);
    sincos(kTwoPi * x, s, c);
}

// The phasors the fold needs depend on the band and, for the query position, on the sequence only: they
// are evaluated once here (double-precision pow / sincos are long software routines) instead of once per
// query head and layer.  grid (2 + S), block F: thread = band.  Workgroup S + 1 has nothing to do with phasors:
// it lists the chunks of the MFMA score kernel (a launch of its own would cost more than the list); nor have the
// kLaneTableEntries / F workgroups after it, which fill the one-key-per-lane kernel's table when it is asked for.
__global__ __launch_bounds__(kBands) void fold_phasor_kernel(FoldArgs a)
{
    if ((int)blockIdx.x > a.S + 1) {
        lane_phasor_entry(a.theta, ((int)blockIdx.x - a.S - 2) * kBands + (int)threadIdx.x, a.lane_table);
        return;
    }
    if ((int)blockIdx.x == a.S + 1) {   // uniform over the workgroup
        if (a.work) build_work_list(a.seq_len, a.S, a.max_seq_len, a.chunk_keys, a.work);
        return;
    }
    const int f = threadIdx.x;
    // Section 2.1: omega_f = theta^(-2f/d); kept as revolutions per position
    const double rev = pow(a.theta, -2.0 * (double)f / (double)kHeadDim) / kTwoPi;
    double *out = a.phasors + ((int64_t)blockIdx.x * kBands + f) * 2;
    if (blockIdx.x == 0) {
        a.band_rev[f] = rev;
        double er = 0.0, ei = 0.0;
        for (int j = 0; j < a.n_off; ++j) {
            double c, s;
            unit_phasor((double)a.offsets[j], rev, &c, &s);
            er += c;
            ei += s;
        }
        out[0] = er / (double)a.n_off;
        out[1] = ei / (double)a.n_off;
    } else {
        double c, s;
        unit_phasor((double)a.cur_pos[blockIdx.x - 1], rev, &c, &s);
        out[0] = c;
        out[1] = s;
    }
}

constexpr int kFoldSeqs = 8;   // sequences per workgroup

// grid (Hkv, L, ceil(S / kFoldSeqs)), block F * G: thread = (band, query head of the group), so that a
// wave's stores fill whole stretches of the [F][3][G] table of its head-instance
__global__ __launch_bounds__(kBands *kMaxGroup) void fold_kernel(FoldArgs a)
{
    const int f = threadIdx.x / a.G, g = threadIdx.x % a.G, h = blockIdx.x, l = blockIdx.y;
    const int qh = h * a.G + g;
    const double er = a.phasors[f * 2], ei = a.phasors[f * 2 + 1];
    const float *ct = a.centers + (((int64_t)l * a.Hq + qh) * kBands + f) * 3;
    const double qr = (double)ct[0], qi = (double)ct[1], qa = (double)ct[2];
    // the ablation variants (Section 5) only change the table: no trig part, no norm part, or the norm
    // part without its (1 - R_f) weight, i.e. S_norm^(0) of Section 4.1
    const bool trig_on = a.variant != TRI_SCORE_NORM_ONLY, norm_on = a.variant != TRI_SCORE_TRIG_ONLY;
    const double ar = trig_on ? qr * er - qi * ei : 0.0, ai = trig_on ? qr * ei + qi * er : 0.0;
    const double cn = !norm_on ? 0.0 : a.variant == TRI_SCORE_NORM_UNWEIGHTED ? qa : qa - hypot(qr, qi);
    const int s_end = min(a.S, ((int)blockIdx.z + 1) * kFoldSeqs);
    for (int s = blockIdx.z * kFoldSeqs; s < s_end; ++s) {
        const double c = a.phasors[((int64_t)(1 + s) * kBands + f) * 2], sn = a.phasors[((int64_t)(1 + s) * kBands + f) * 2 + 1];
        float *t = a.table + (((((int64_t)l * a.S + s) * a.Hkv + h) * kBands + f) * 3) * a.G;
        t[0 * a.G + g] = (float)(ar * c - ai * sn);
        t[1 * a.G + g] = (float)(ar * sn + ai * c);
        t[2 * a.G + g] = (float)cn;
    }
}

template <typename T>
struct Elem;
template <>
struct Elem<float> {
    static constexpr int kRow16 = 32;  // 16-byte chunks per key row
};
template <>
struct Elem<uint16_t> {
    static constexpr int kRow16 = 16;
};

// One band of one key: rotate the key by its own position, take its modulus, and add the
// three products per query head.  tb points at this band's [3][G] table entries (wave-uniform).
template <int G>
__device__ __forceinline__ void band_update(float (&acc)[G], const float *__restrict__ tb, double pd,
                                            double rev, float re, float im)
{
    double xr = pd * rev;
    float x = (float)__builtin_amdgcn_fract(xr);   // phase in revolutions, [0, 1]
    float sn = __builtin_amdgcn_sinf(x);           // v_sin_f32 / v_cos_f32 take revolutions
    float cs = __builtin_amdgcn_cosf(x);
    float kr = re * cs - im * sn;
    float ki = re * sn + im * cs;
    float m = __builtin_amdgcn_sqrtf(re * re + im * im);
#pragma unroll
    for (int g = 0; g < G; ++g)
        acc[g] = fmaf(tb[0 * G + g], kr, fmaf(tb[1 * G + g], ki, fmaf(tb[2 * G + g], m, acc[g])));
}

// grid (n_tiles, S*Hkv, L), block 256: one key per thread, staged through LDS so that global
// loads are coalesced 16-byte accesses while each thread ends up owning one whole key.
template <int G, typename T, int PAIRS>
__global__ __launch_bounds__(kScoreTile) void score_kernel(ScoreArgs a)
{
    constexpr int ROW16 = Elem<T>::kRow16;
    constexpr int STRIDE16 = ROW16 + 1;   // odd number of 16-byte units: conflict-free row reads
    extern __shared__ uint4 lds[];
    __shared__ int64_t row_off[kScoreTile];
    __shared__ double red[4][2 * G];

    const CacheView &c = a.c;
    const int tid = threadIdx.x;
    const int tile = blockIdx.x;
    const int s = blockIdx.y / c.n_kv_heads, h = blockIdx.y % c.n_kv_heads;
    const int l = blockIdx.z;
    const int N = clamp_len(c.seq_len[s], c.max_seq_len);
    const int n0 = tile * kScoreTile;
    if (n0 >= N) return;
    const int n = n0 + tid;
    const bool valid = n < N;

    row_off[tid] = valid ? kv_offset(c, l, s, h, n) : (int64_t)-1;
    int p = 0;
    if (valid && !c.k_rotated) p = c.pos[pos_offset(c, l, s, h, n)];   // a post-RoPE key needs no rotation
    __syncthreads();

    const T *kbase = (const T *)c.k;
#pragma unroll 4
    for (int i = 0; i < ROW16; ++i) {
        int ci = i * kScoreTile + tid;
        int key = ci / ROW16, part = ci % ROW16;
        int64_t off = row_off[key];
        uint4 v = make_uint4(0u, 0u, 0u, 0u);
        if (off >= 0) v = reinterpret_cast<const uint4 *>(kbase + off)[part];
        lds[key * STRIDE16 + part] = v;
    }
    __syncthreads();

    const int64_t inst = ((int64_t)l * c.n_seqs + s) * c.n_kv_heads + h;
    const float *__restrict__ tb = a.table + inst * (kBands * 3 * G);
    const double *__restrict__ rev = a.band_rev;
    const double pd = (double)p;
    float acc[G];
#pragma unroll
    for (int g = 0; g < G; ++g) acc[g] = 0.f;
    const uint4 *row = lds + tid * STRIDE16;

    if constexpr (sizeof(T) == 2 && PAIRS == TRI_PAIR_INTERLEAVED) {
#pragma unroll 2
        for (int j = 0; j < 16; ++j) {
            uint4 q = row[j];
            const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                int f = 4 * j + i;
                band_update<G>(acc, tb + f * 3 * G, pd, rev[f], bf16_lo(w[i]), bf16_hi(w[i]));
            }
        }
    } else if constexpr (sizeof(T) == 2) {
#pragma unroll 2
        for (int j = 0; j < 8; ++j) {
            uint4 qr = row[j], qi = row[j + 8];
            const uint32_t wr[4] = {qr.x, qr.y, qr.z, qr.w}, wi[4] = {qi.x, qi.y, qi.z, qi.w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                int f = 8 * j + 2 * i;
                band_update<G>(acc, tb + f * 3 * G, pd, rev[f], bf16_lo(wr[i]), bf16_lo(wi[i]));
                band_update<G>(acc, tb + (f + 1) * 3 * G, pd, rev[f + 1], bf16_hi(wr[i]), bf16_hi(wi[i]));
            }
        }
    } else if constexpr (PAIRS == TRI_PAIR_INTERLEAVED) {
#pragma unroll 2
        for (int j = 0; j < 32; ++j) {
            uint4 q = row[j];
            int f = 2 * j;
            band_update<G>(acc, tb + f * 3 * G, pd, rev[f], __uint_as_float(q.x), __uint_as_float(q.y));
            band_update<G>(acc, tb + (f + 1) * 3 * G, pd, rev[f + 1], __uint_as_float(q.z), __uint_as_float(q.w));
        }
    } else {
#pragma unroll 2
        for (int j = 0; j < 16; ++j) {
            uint4 qr = row[j], qi = row[j + 16];
            const uint32_t wr[4] = {qr.x, qr.y, qr.z, qr.w}, wi[4] = {qi.x, qi.y, qi.z, qi.w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                int f = 4 * j + i;
                band_update<G>(acc, tb + f * 3 * G, pd, rev[f], __uint_as_float(wr[i]), __uint_as_float(wi[i]));
            }
        }
    }

    // raw scores out, and this tile's sum / sum of squares per query head (double, fixed order)
    const int Hq = c.n_kv_heads * G;
    float *rw = a.raw + (((int64_t)l * c.n_seqs + s) * Hq + (int64_t)h * G) * c.max_seq_len + n;
    double mom[2 * G];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        if (valid) rw[(int64_t)g * c.max_seq_len] = acc[g];
        double v = valid ? (double)acc[g] : 0.0;
        mom[g] = v;
        mom[G + g] = v * v;
    }
#pragma unroll
    for (int i = 0; i < 2 * G; ++i) {
        double v = mom[i];
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
        mom[i] = v;
    }
    if ((tid & 63) == 0) {
#pragma unroll
        for (int i = 0; i < 2 * G; ++i) red[tid >> 6][i] = mom[i];
    }
    __syncthreads();
    if (tid < 2 * G) {
        double v = red[0][tid] + red[1][tid] + red[2][tid] + red[3][tid];
        a.partials[(inst * a.n_tiles + tile) * (2 * G) + tid] = v;
    }
}

struct StatsArgs {
    const double *partials;
    double *stats;  // [inst][G][2] = (mean, 1/sigma)
    const int32_t *seq_len;
    int32_t n_seqs, n_kv_heads, n_tiles, G, tile_keys, max_seq_len;
};

// grid (instances), block 256: Section 4.3, mu_g and sigma_g over the N keys (population sigma).
__global__ __launch_bounds__(256) void stats_kernel(StatsArgs a)
{
    __shared__ double part[16][16];
    const int inst = blockIdx.x;
    const int s = (inst / a.n_kv_heads) % a.n_seqs;
    const int N = clamp_len(a.seq_len[s], a.max_seq_len);
    const int tiles = (N + a.tile_keys - 1) / a.tile_keys;
    const int i = threadIdx.x & 15, r = threadIdx.x >> 4;
    const int W = 2 * a.G;
    double acc = 0.0;
    if (i < W)
        for (int t = r; t < tiles; t += 16) acc += a.partials[((int64_t)inst * a.n_tiles + t) * W + i];
    part[r][i] = acc;
    __syncthreads();
    if (threadIdx.x < a.G) {   // (the same order of additions as block_stats)
        const int g = threadIdx.x;
        double s1 = 0.0, s2 = 0.0;
        for (int k = 0; k < 16; ++k) {
            s1 += part[k][g];
            s2 += part[k][a.G + g];
        }
        double mean, rsig;
        moments_to_stats(s1, s2, N, &mean, &rsig);
        a.stats[((int64_t)inst * a.G + g) * 2 + 0] = mean;
        a.stats[((int64_t)inst * a.G + g) * 2 + 1] = rsig;
    }
}

struct FinalArgs {
    const float *raw;     // [inst][G][Nmax]  (instance-major because Hq = Hkv * G)
    const double *stats;  // [inst][G][2]
    float *final_;        // [inst][Nmax]
    const int32_t *seq_len;
    int32_t n_seqs, n_kv_heads, max_seq_len;
    int32_t key_blocks;   // workgroups per head-instance
};

// grid (instances * ceil(Nmax/1024)), block 256: S_final(k) = max_g (S~(g)(k) - mu_g) / sigma_g.
template <int G>
__global__ __launch_bounds__(256) void final_kernel(FinalArgs a)
{
    const int inst = blockIdx.x / a.key_blocks, kb = blockIdx.x - inst * a.key_blocks;
    const int s = (inst / a.n_kv_heads) % a.n_seqs;
    const int N = clamp_len(a.seq_len[s], a.max_seq_len);
    const int n = (kb * 256 + threadIdx.x) * 4;
    if (n >= N) return;
    const float *rw = a.raw + (int64_t)inst * G * a.max_seq_len + n;
    const double *st = a.stats + (int64_t)inst * G * 2;
    float best[4];
    if (n + 3 < N && (a.max_seq_len & 3) == 0) {
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const float4 v = *reinterpret_cast<const float4 *>(rw + (int64_t)g * a.max_seq_len);
            const ZParams zp = z_params(st[2 * g], st[2 * g + 1]);
            const float z[4] = {z_score(v.x, zp), z_score(v.y, zp), z_score(v.z, zp), z_score(v.w, zp)};
#pragma unroll
            for (int k = 0; k < 4; ++k) best[k] = (g == 0) ? z[k] : fmaxf(best[k], z[k]);
        }
        *reinterpret_cast<float4 *>(a.final_ + (int64_t)inst * a.max_seq_len + n) =
            make_float4(best[0], best[1], best[2], best[3]);
    } else {
        for (int k = 0; k < 4 && n + k < N; ++k) {
            float b = 0.f;
#pragma unroll
            for (int g = 0; g < G; ++g) {
                float z = z_score(rw[(int64_t)g * a.max_seq_len + k], z_params(st[2 * g], st[2 * g + 1]));
                b = (g == 0) ? z : fmaxf(b, z);
            }
            a.final_[(int64_t)inst * a.max_seq_len + n + k] = b;
        }
    }
}

template <int G, typename T>
tri_status launch_score_kernel(const tri_model &m, const ScoreArgs &sa, dim3 grid, hipStream_t st)
{
    const size_t lds = (size_t)kScoreTile * (Elem<T>::kRow16 + 1) * 16;
    if (m.pairs == TRI_PAIR_INTERLEAVED) {
        auto kern = score_kernel<G, T, TRI_PAIR_INTERLEAVED>;
        if (lds > 48 * 1024 &&
            hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
            return hip_status("hipFuncSetAttribute(score_kernel)");
        hipLaunchKernelGGL(kern, grid, dim3(kScoreTile), lds, st, sa);
    } else {
        auto kern = score_kernel<G, T, TRI_PAIR_HALF>;
        if (lds > 48 * 1024 &&
            hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
            return hip_status("hipFuncSetAttribute(score_kernel)");
        hipLaunchKernelGGL(kern, grid, dim3(kScoreTile), lds, st, sa);
    }
    return hip_status("score_kernel");
}

// MFMA kernel: bf16, a group of 16 slots never straddling a block, 32-bit row offsets
bool mfma_path(const tri_cache &c, int G)
{
    return c.dtype == TRI_BF16 && (c.block_size == 0 || c.block_size >= 16) &&
           c.stride_slot * 2 * 16 < ((int64_t)1 << 31) && ((int64_t)G * c.max_seq_len + 16) * 4 < ((int64_t)1 << 32);
}

template <int G>
tri_status launch_score_g(const tri_model &m, const tri_cache &c, ScoreArgs sa, const FinalArgs &fa,
                          float *final_out, MomentLayout *moments, bool lane_kernel, hipStream_t st)
{
    const int n_inst = m.n_layers * c.n_seqs * m.n_kv_heads;
    const bool fast = mfma_path(c, G);
    const int tile_keys = fast ? sa.chunk_keys : kScoreTile;
    sa.n_tiles = (c.max_seq_len + tile_keys - 1) / tile_keys;
    tri_status rc = TRI_OK;
    if (fast && !lane_kernel && !c.k_rotated) {   // (the one-key-per-lane kernel's table came with the fold's phasors)
        rc = launch_phasor_table(m.rope_theta, const_cast<uint4 *>(sa.phasors), st);
        if (rc != TRI_OK) return rc;
    }
    hipEvent_t ev0, ev1;
    const bool timed = timing_next(&ev0, &ev1);
    if (timed) (void)hipEventRecord(ev0, st);
    if (lane_kernel) {
        rc = launch_score_lane(G, sa, st);
    } else if (fast) {
        rc = launch_score_fast(G, sa, m.pairs == TRI_PAIR_HALF, st);
    } else {
        dim3 grid(sa.n_tiles, c.n_seqs * m.n_kv_heads, m.n_layers);
        rc = (c.dtype == TRI_BF16) ? launch_score_kernel<G, uint16_t>(m, sa, grid, st)
                                   : launch_score_kernel<G, float>(m, sa, grid, st);
    }
    if (timed) (void)hipEventRecord(ev1, st);
    if (rc != TRI_OK) return rc;
    if (moments) {
        moments->n_tiles = sa.n_tiles;
        moments->tile_keys = tile_keys;
    }
    if (!final_out) return rc;   // fused step: the selection forms the statistics from the moments itself
    StatsArgs ta{sa.partials, const_cast<double *>(fa.stats), c.seq_len, c.n_seqs, m.n_kv_heads, sa.n_tiles, G,
                 tile_keys, c.max_seq_len};
    hipLaunchKernelGGL(stats_kernel, dim3(n_inst), dim3(256), 0, st, ta);
    if ((rc = hip_status("stats_kernel")) != TRI_OK) return rc;
    if (final_out) {
        FinalArgs fb = fa;
        fb.key_blocks = (c.max_seq_len + 1023) / 1024;
        if ((int64_t)fb.key_blocks * n_inst > (int64_t)0x7fffffff) {
            set_error("tri_score: %d head-instances x %d key blocks exceed the grid", n_inst, fb.key_blocks);
            return TRI_ERR_UNSUPPORTED;
        }
        hipLaunchKernelGGL(final_kernel<G>, dim3((uint32_t)((int64_t)fb.key_blocks * n_inst)), dim3(256), 0, st, fb);
        rc = hip_status("final_kernel");
    }
    return rc;
}

}  // namespace

// Compute units of the current GPU (asked once per GPU).
tri_status device_cus(int *n_cu)
{
    constexpr int kDevices = 64;
    static std::atomic<int> cached[kDevices];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kDevices) {
        (void)hipGetLastError();
        set_error("score: no current device below %d", kDevices);
        return TRI_ERR_HIP;
    }
    int n = cached[dev].load(std::memory_order_relaxed);
    if (n == 0) {
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) {
            (void)hipGetLastError();
            set_error("score: compute-unit count not available");
            return TRI_ERR_HIP;
        }
        cached[dev].store(n, std::memory_order_relaxed);
    }
    *n_cu = n;
    return TRI_OK;
}

tri_status launch_score(const tri_model &m, const float *centers, const tri_cache &c, float *final_out,
                        float *raw_out, char *ws, const Workspace &wl, MomentLayout *moments, hipStream_t st)
{
    const int G = m.n_q_heads / m.n_kv_heads;
    if (moments) *moments = MomentLayout{1, 1};
    if (c.max_seq_len <= 0 || c.n_seqs <= 0) return TRI_OK;
    FoldArgs fo{};
    fo.centers = centers;
    fo.table = reinterpret_cast<float *>(ws + wl.table);
    fo.band_rev = reinterpret_cast<double *>(ws + wl.band_rev);
    fo.phasors = reinterpret_cast<double *>(ws + wl.fold_phasors);
    fo.cur_pos = c.cur_pos;
    fo.seq_len = c.seq_len;
    fo.work = mfma_path(c, G) ? reinterpret_cast<int32_t *>(ws + wl.work) : nullptr;
    // keys per work item: small batches on the one-key-per-lane kernel are cut finer
    int chunk_keys = kFastChunk;
    if (fo.work && m.pairs == TRI_PAIR_INTERLEAVED) {
        int n_cu = 0;
        tri_status rcu = device_cus(&n_cu);
        if (rcu != TRI_OK) return rcu;
        chunk_keys = lane_chunk_keys(G, (int64_t)m.n_layers * c.n_seqs * m.n_kv_heads, c.max_seq_len, n_cu);
    }
    fo.chunk_keys = chunk_keys;
    fo.max_seq_len = c.max_seq_len;
    fo.S = c.n_seqs;
    fo.Hq = m.n_q_heads;
    fo.Hkv = m.n_kv_heads;
    fo.G = G;
    fo.theta = m.rope_theta;
    fo.n_off = m.n_offsets;
    fo.variant = m.score_variant;
    for (int j = 0; j < m.n_offsets; ++j) fo.offsets[j] = m.offsets[j];
    // Interleaved pairs: the kernel with one key per lane.  Paged caches go there only as small batches (work items
    // below kFastChunk, which only that kernel takes): on large paged batches the kernel that spreads a key over
    // sixteen lanes is 3 % faster (config 4: 12.2 ms against 12.5 ms per 12-layer slab), as it is the only one for
    // half-split pairs.
    const bool lane_kernel = fo.work && m.pairs == TRI_PAIR_INTERLEAVED && (c.block_size == 0 || chunk_keys < kFastChunk);
    const bool lane_table = lane_kernel && !c.k_rotated;
    fo.lane_table = lane_table ? reinterpret_cast<float4 *>(ws + wl.phasors) : nullptr;
    hipLaunchKernelGGL(fold_phasor_kernel, dim3(2 + c.n_seqs + (lane_table ? kLaneTableEntries / kBands : 0)),
                       dim3(kBands), 0, st, fo);
    tri_status rc0 = hip_status("fold_phasor_kernel");
    if (rc0 != TRI_OK) return rc0;
    hipLaunchKernelGGL(fold_kernel, dim3(m.n_kv_heads, m.n_layers, (c.n_seqs + kFoldSeqs - 1) / kFoldSeqs),
                       dim3(kBands * G), 0, st, fo);
    tri_status rc = hip_status("fold_kernel");
    if (rc != TRI_OK) return rc;

    ScoreArgs sa{};
    sa.c = make_view(m, c);
    sa.table = fo.table;
    sa.band_rev = fo.band_rev;
    sa.raw = raw_out ? raw_out : reinterpret_cast<float *>(ws + wl.raw);
    sa.partials = reinterpret_cast<double *>(ws + wl.partials);
    sa.phasors = reinterpret_cast<const uint4 *>(ws + wl.phasors);
    sa.work = reinterpret_cast<int32_t *>(ws + wl.work);
    sa.n_layers = m.n_layers;
    sa.chunk_keys = chunk_keys;
    FinalArgs fa{sa.raw, reinterpret_cast<double *>(ws + wl.stats), final_out, c.seq_len, c.n_seqs,
                 m.n_kv_heads, c.max_seq_len, 0};
    switch (G) {
        case 1: return launch_score_g<1>(m, c, sa, fa, final_out, moments, lane_kernel, st);
        case 2: return launch_score_g<2>(m, c, sa, fa, final_out, moments, lane_kernel, st);
        case 3: return launch_score_g<3>(m, c, sa, fa, final_out, moments, lane_kernel, st);
        case 4: return launch_score_g<4>(m, c, sa, fa, final_out, moments, lane_kernel, st);
        case 5: return launch_score_g<5>(m, c, sa, fa, final_out, moments, lane_kernel, st);
        case 6: return launch_score_g<6>(m, c, sa, fa, final_out, moments, lane_kernel, st);
        case 7: return launch_score_g<7>(m, c, sa, fa, final_out, moments, lane_kernel, st);
        case 8: return launch_score_g<8>(m, c, sa, fa, final_out, moments, lane_kernel, st);
    }
    set_error("group size %d not built (1 to 8)", G);
    return TRI_ERR_UNSUPPORTED;
}

}  // namespace tri
