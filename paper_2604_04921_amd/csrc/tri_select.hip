// Top-B selection per head-instance (Section 4.3): exact radix select on an order-preserving
// integer image of the float score, then an ordered emit so that the kept slots come out
// ascending and equal scores at the threshold go to the lower slots.
#include "tri_internal.h"

namespace tri {

namespace {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / 64;

// Monotone map float -> uint32 (larger float <=> larger key); -0.0 is folded onto +0.0.
__device__ __forceinline__ uint32_t order_key(float x)
{
    uint32_t b = __float_as_uint(x);
    if (b == 0x80000000u) b = 0u;
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

struct SelectArgs {
    const float *final_;  // [inst][Nmax]
    const int32_t *seq_len;
    int32_t *kept_idx;    // [inst][B]
    int32_t *kept_cnt;    // [inst]
    int32_t n_seqs, n_kv_heads, max_seq_len, budget;
};

// grid (instances), block 1024
__global__ __launch_bounds__(kSelThreads) void select_kernel(SelectArgs a)
{
    __shared__ uint32_t hist[256];
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
    const float *fs = a.final_ + (int64_t)inst * a.max_seq_len;

    // ---- threshold: the B-th largest key, 8 bits at a time from the top
    uint32_t prefix = 0u, mask = 0u;
    uint32_t need = (uint32_t)B;
    for (int shift = 24; shift >= 0; shift -= 8) {
        if (tid < 256) hist[tid] = 0u;
        __syncthreads();
        for (int n = tid; n < N; n += kSelThreads) {
            uint32_t u = order_key(fs[n]);
            if ((u & mask) == prefix) atomicAdd(&hist[(u >> shift) & 255u], 1u);
        }
        __syncthreads();
        // counts of bins 255, 254, ... as an inclusive running sum over threads 0..255
        uint32_t v = 0u, cum = 0u;
        if (tid < 256) {
            v = hist[255 - tid];
            cum = v;
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                uint32_t t = __shfl_up(cum, o, 64);
                if (lane >= o) cum += t;
            }
            if (lane == 63) wave_tot[wave] = cum;
        }
        __syncthreads();
        if (tid < 256) {
            for (int w = 0; w < wave; ++w) cum += wave_tot[w];
            if (cum >= need && cum - v < need) {  // exactly one thread: the bin holding the B-th key
                sel[0] = 255u - (uint32_t)tid;
                sel[1] = need - (cum - v);
            }
        }
        __syncthreads();
        prefix |= sel[0] << shift;
        mask |= 255u << shift;
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
        if (in) u = order_key(fs[n]);
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

}  // namespace

tri_status launch_select(const tri_model &m, const float *final_scores, const tri_cache &c, int32_t budget,
                         int32_t *kept_idx, int32_t *kept_cnt, hipStream_t st)
{
    const int n_inst = m.n_layers * c.n_seqs * m.n_kv_heads;
    if (n_inst <= 0) return TRI_OK;
    SelectArgs sa{final_scores, c.seq_len, kept_idx, kept_cnt, c.n_seqs, m.n_kv_heads, c.max_seq_len, budget};
    hipLaunchKernelGGL(select_kernel, dim3(n_inst), dim3(kSelThreads), 0, st, sa);
    return hip_status("select_kernel");
}

}  // namespace tri
