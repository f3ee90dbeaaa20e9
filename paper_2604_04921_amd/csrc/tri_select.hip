// Top-B selection per head-instance (Section 4.3): exact radix select on an order-preserving
// integer image of the float score, then an ordered emit so that the kept slots come out
// ascending and equal scores at the threshold go to the lower slots.
//
// The kernel either takes final scores (tri_select_topk) or takes the raw per-head scores and the
// per-head mean / 1/sigma and forms S_final = max_g (S~(g) - mu_g) / sigma_g itself (fused step:
// the final scores then never travel through memory).  The integer keys of a head-instance are
// kept in LDS when they fit (32768 keys = 128 KB); longer sequences re-read them from memory.
#include "tri_internal.h"

namespace tri {

namespace {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / 64;
constexpr int kSelBins = 2048;          // 11-bit digits: bits 31..21, 20..10, then the low 10 bits
constexpr int kSelLdsKeys = 32768;      // keys held in LDS at most

// Monotone map float -> uint32 (larger float <=> larger key); -0.0 is folded onto +0.0.
__device__ __forceinline__ uint32_t order_key(float x)
{
    uint32_t b = __float_as_uint(x);
    if (b == 0x80000000u) b = 0u;
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

struct SelectArgs {
    const float *final_;   // [inst][Nmax] final scores, or NULL when raw + stats are given
    const float *raw;      // [inst][G][Nmax]
    const double *stats;   // [inst][G][2] = (mean, 1/sigma)
    uint32_t *scratch;     // [inst][Nmax] keys of sequences too long for LDS (raw mode only)
    const int32_t *seq_len;
    int32_t *kept_idx;     // [inst][B]
    int32_t *kept_cnt;     // [inst]
    int32_t n_seqs, n_kv_heads, max_seq_len, budget, lds_keys;
};

// grid (instances), block 1024.  G = 0: final scores given; G > 0: raw scores of G query heads given.
template <int G>
__global__ __launch_bounds__(kSelThreads) void select_kernel(SelectArgs a)
{
    extern __shared__ uint32_t lds_keys[];
    __shared__ uint32_t hist[kSelBins];
    __shared__ uint32_t wave_tot[kSelWaves];
    __shared__ uint32_t sel[2];
    __shared__ uint32_t wg[2][kSelWaves], we[2][kSelWaves];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int inst = blockIdx.x;
    const int s = (inst / a.n_kv_heads) % a.n_seqs;
    const int N = a.seq_len[s];
    const int B = a.budget;
    int32_t *out = a.kept_idx + (int64_t)inst * B;
    if (tid == 0) a.kept_cnt[inst] = N < B ? N : B;
    if (N <= B) {  // nothing to evict: keep every slot
        for (int n = tid; n < N; n += kSelThreads) out[n] = n;
        return;
    }
    const bool in_lds = N <= a.lds_keys;
    const float *fs = G == 0 ? a.final_ + (int64_t)inst * a.max_seq_len : nullptr;
    const float *rw = G > 0 ? a.raw + (int64_t)inst * (G > 0 ? G : 1) * a.max_seq_len : nullptr;
    uint32_t *gk = (G > 0 && !in_lds) ? a.scratch + (int64_t)inst * a.max_seq_len : nullptr;

    double mu[G > 0 ? G : 1], rs[G > 0 ? G : 1];
    if constexpr (G > 0) {
#pragma unroll
        for (int g = 0; g < G; ++g) {
            mu[g] = a.stats[((int64_t)inst * G + g) * 2];
            rs[g] = a.stats[((int64_t)inst * G + g) * 2 + 1];
        }
    }
    // key of slot n from its source (first touch)
    auto make_key = [&](int n) {
        float f;
        if constexpr (G > 0) {
#pragma unroll
            for (int g = 0; g < G; ++g) {
                const float z = (float)(((double)rw[(int64_t)g * a.max_seq_len + n] - mu[g]) * rs[g]);
                f = g == 0 ? z : fmaxf(f, z);
            }
        } else {
            f = fs[n];
        }
        return order_key(f);
    };
    // key of slot n on later passes
    auto get_key = [&](int n) {
        if (in_lds) return lds_keys[n];
        if constexpr (G > 0) return gk[n];
        else return order_key(fs[n]);
    };

    // ---- threshold: the B-th largest key, one 11-bit digit at a time from the top
    uint32_t prefix = 0u, mask = 0u;
    uint32_t need = (uint32_t)B;
#pragma unroll 1
    for (int pass = 0; pass < 3; ++pass) {
        const int shift = pass == 0 ? 21 : (pass == 1 ? 10 : 0);
        const uint32_t dmask = pass == 2 ? 1023u : 2047u;
        for (int k = tid; k < kSelBins; k += kSelThreads) hist[k] = 0u;
        __syncthreads();
        if (pass == 0) {
            for (int n = tid; n < N; n += kSelThreads) {
                const uint32_t u = make_key(n);
                if (in_lds) lds_keys[n] = u;
                else if constexpr (G > 0) gk[n] = u;
                atomicAdd(&hist[u >> 21], 1u);
            }
        } else {
            for (int n = tid; n < N; n += kSelThreads) {
                const uint32_t u = get_key(n);
                if ((u & mask) == prefix) atomicAdd(&hist[(u >> shift) & dmask], 1u);
            }
        }
        __syncthreads();
        // thread t owns bins 2047-2t and 2046-2t: running count from the top bin down
        const uint32_t v0 = hist[kSelBins - 1 - 2 * tid], v1 = hist[kSelBins - 2 - 2 * tid];
        uint32_t cum = v0 + v1;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const uint32_t t = __shfl_up(cum, o, 64);
            if (lane >= o) cum += t;
        }
        if (lane == 63) wave_tot[wave] = cum;
        __syncthreads();
        for (int w = 0; w < wave; ++w) cum += wave_tot[w];
        const uint32_t excl = cum - v0 - v1;
        if (excl < need && need <= excl + v0) {          // exactly one thread and bin holds the B-th key
            sel[0] = (uint32_t)(kSelBins - 1 - 2 * tid);
            sel[1] = need - excl;
        } else if (excl + v0 < need && need <= cum) {
            sel[0] = (uint32_t)(kSelBins - 2 - 2 * tid);
            sel[1] = need - excl - v0;
        }
        __syncthreads();
        prefix |= sel[0] << shift;
        mask |= dmask << shift;
        need = sel[1];
        __syncthreads();
    }
    const uint32_t thr = prefix;  // keys > thr are kept; of the keys == thr the first `need` slots

    // ---- ordered emit
    uint32_t g_run = 0u, e_run = 0u;
    int buf = 0;
    for (int n0 = 0; n0 < N; n0 += kSelThreads, buf ^= 1) {
        const int n = n0 + tid;
        uint32_t u = 0u;
        const bool in = n < N;
        if (in) u = get_key(n);
        const bool gt = in && u > thr, eq = in && u == thr;
        const uint64_t gm = __ballot(gt), em = __ballot(eq);
        const uint64_t below = (1ull << lane) - 1ull;
        const uint32_t g_lt = __popcll(gm & below), e_lt = __popcll(em & below);
        if (lane == 0) {
            wg[buf][wave] = __popcll(gm);
            we[buf][wave] = __popcll(em);
        }
        __syncthreads();
        uint32_t g_before = 0u, e_before = 0u, g_tot = 0u, e_tot = 0u;
#pragma unroll
        for (int w = 0; w < kSelWaves; ++w) {
            const uint32_t a_ = wg[buf][w], b_ = we[buf][w];
            if (w < wave) {
                g_before += a_;
                e_before += b_;
            }
            g_tot += a_;
            e_tot += b_;
        }
        const uint32_t e_rank = e_run + e_before + e_lt;
        if (gt || (eq && e_rank < need)) {
            const uint32_t dst = g_run + g_before + g_lt + (e_rank < need ? e_rank : need);
            out[dst] = n;
        }
        g_run += g_tot;
        e_run += e_tot;
    }
}

template <int G>
tri_status launch_select_g(const SelectArgs &sa, int n_inst, hipStream_t st)
{
    auto kern = select_kernel<G>;
    const size_t lds = (size_t)sa.lds_keys * sizeof(uint32_t);
    if (hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
        return hip_status("hipFuncSetAttribute(select_kernel)");
    hipLaunchKernelGGL(kern, dim3(n_inst), dim3(kSelThreads), lds, st, sa);
    return hip_status("select_kernel");
}

}  // namespace

tri_status launch_select(const tri_model &m, const float *final_scores, const float *raw, const double *stats,
                         uint32_t *scratch, const tri_cache &c, int32_t budget, int32_t *kept_idx,
                         int32_t *kept_cnt, hipStream_t st)
{
    const int n_inst = m.n_layers * c.n_seqs * m.n_kv_heads;
    if (n_inst <= 0) return TRI_OK;
    SelectArgs sa{final_scores, raw, stats, scratch, c.seq_len, kept_idx, kept_cnt, c.n_seqs, m.n_kv_heads,
                  c.max_seq_len, budget, c.max_seq_len < kSelLdsKeys ? (c.max_seq_len > 0 ? c.max_seq_len : 1) : kSelLdsKeys};
    if (final_scores) return launch_select_g<0>(sa, n_inst, st);
    switch (m.n_q_heads / m.n_kv_heads) {
        case 1: return launch_select_g<1>(sa, n_inst, st);
        case 2: return launch_select_g<2>(sa, n_inst, st);
        case 4: return launch_select_g<4>(sa, n_inst, st);
        case 8: return launch_select_g<8>(sa, n_inst, st);
    }
    set_error("group size not built (1, 2, 4, 8)");
    return TRI_ERR_UNSUPPORTED;
}

}  // namespace tri
