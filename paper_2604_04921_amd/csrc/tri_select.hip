// Top-B selection per head-instance (Section 4.3): an exact select on an order-preserving integer
// image of the float score, then an ordered emit so that the kept slots come out ascending and equal
// scores at the threshold go to the lower slots.
//
// Either kernel takes final scores (tri_select_topk) or takes the raw per-head scores and their
// per-chunk moments (or ready-made mean / 1/sigma), forms the statistics and S_final = max_g (S~(g) - mu_g) /
// sigma_g itself (fused step: neither statistics nor final scores then travel through memory).  Sequences of up to 32768 keys keep their
// integer keys in registers (select_reg_kernel: one histogram over linear score bins, exact ranking of
// the threshold bin); longer ones use select_kernel (the same steps over keys held in LDS or, beyond
// 32768 keys, in a workspace area).
#include "tri_fill.h"

namespace tri {

namespace {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / 64;
constexpr int kSelBins = 2048;          // linear score bins of the histogram pass
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
    const double *stats;   // [inst][G][2] = (mean, 1/sigma); unused when partials is given
    const double *partials;   // [inst][n_tiles][2G] per-tile sum and sum of squares of the raw scores, or NULL
    int32_t n_tiles, tile_keys;
    uint32_t *scratch;     // [inst][Nmax] keys of sequences too long for LDS (raw mode only)
    const int32_t *seq_len;
    int32_t *kept_idx;     // [inst][B]
    int32_t *kept_cnt;     // [inst]
    int32_t n_seqs, n_kv_heads, max_seq_len, budget, lds_keys;
    const int32_t *head_budgets;   // [L][Hkv] or NULL: budget of each (layer, KV head), at most `budget`
    int32_t n_above, n_upto;       // select_kernel: this launch handles the head-instances with n_above < N <= n_upto
    // 256-thread select_reg_kernel, fill != 0: the workgroup goes on to evict its head-instance in place (fill_block)
    FillArgs fa;
    int32_t fill;
};

// The budget of head-instance `inst`: the common one, or the head's own (read into [0, budget]).
__device__ __forceinline__ int instance_budget(const SelectArgs &a, int inst)
{
    if (!a.head_budgets) return a.budget;
    const int h = inst % a.n_kv_heads, l = inst / (a.n_kv_heads * a.n_seqs);
    return min(max(a.head_budgets[l * a.n_kv_heads + h], 0), a.budget);
}

constexpr int kSelCand = 2048;   // keys of the threshold bin ranked in LDS

__device__ __forceinline__ float key_to_float(uint32_t u)
{
    return __uint_as_float((u & 0x80000000u) ? (u & 0x7fffffffu) : ~u);
}
__device__ __forceinline__ int linear_bin(uint32_t u)
{
    const float x = (key_to_float(u) + 4.0f) * 128.0f;   // 2048 bins over [-4, 12)
    return (int)fminf(fmaxf(x, 0.0f), 2047.0f);
}

// grid (instances), block 1024.  G = 0: final scores given; G > 0: raw scores of G query heads given.
template <int G>
__global__ __launch_bounds__(kSelThreads) void select_kernel(SelectArgs a)
{
    extern __shared__ uint32_t lds_keys[];
    __shared__ uint32_t hist[kSelBins];
    __shared__ uint32_t cand_key[kSelCand];
    __shared__ int32_t cand_idx[kSelCand];
    __shared__ uint32_t wave_tot[kSelWaves];
    __shared__ uint32_t sh[36];   // 0: selected bin, 1: need inside it, 2: candidate count, 3: threshold key, 4..35: bit counters / tie count
    __shared__ uint32_t wg[2][kSelWaves], we[2][kSelWaves];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int inst = blockIdx.x;
    const int s = (inst / a.n_kv_heads) % a.n_seqs;
    const int N = clamp_len(a.seq_len[s], a.max_seq_len);
    if (N <= a.n_above || N > a.n_upto) return;   // the other launch's head-instance (uniform over the workgroup)
    const int B = instance_budget(a, inst);
    int32_t *out = a.kept_idx + (int64_t)inst * a.budget;
    if (tid == 0) a.kept_cnt[inst] = N < B ? N : B;
    if (B == 0) return;   // a head whose own budget is 0 keeps nothing
    if (N <= B) {  // nothing to evict: keep every slot
        for (int n = tid; n < N; n += kSelThreads) out[n] = n;
        return;
    }
    const bool in_lds = N <= a.lds_keys;
    const float *fs = G == 0 ? a.final_ + (int64_t)inst * a.max_seq_len : nullptr;
    const float *rw = G > 0 ? a.raw + (int64_t)inst * (G > 0 ? G : 1) * a.max_seq_len : nullptr;
    uint32_t *gk = (G > 0 && !in_lds) ? a.scratch + (int64_t)inst * a.max_seq_len : nullptr;

    ZParams zp[G > 0 ? G : 1];
    if constexpr (G > 0) {
        __shared__ double zst[2 * (G > 0 ? G : 1)], zpart[32 * (G > 0 ? G : 1)];
        if (a.partials)   // statistics from the moments (uniform over the launch)
            block_stats<G>(a.partials + (int64_t)inst * a.n_tiles * (2 * G), (N + a.tile_keys - 1) / a.tile_keys, N, tid,
                           zpart, zst);
#pragma unroll
        for (int g = 0; g < G; ++g)
            zp[g] = a.partials ? z_params(zst[2 * g], zst[2 * g + 1])
                               : z_params(a.stats[((int64_t)inst * G + g) * 2], a.stats[((int64_t)inst * G + g) * 2 + 1]);
    }
    // key of slot n from its source (first touch)
    auto make_key = [&](int n) {
        float f;
        if constexpr (G > 0) {
#pragma unroll
            for (int g = 0; g < G; ++g) {
                const float z = z_score(__builtin_nontemporal_load(&rw[(int64_t)g * a.max_seq_len + n]), zp[g]);
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

    // ---- keys to LDS / scratch, histogram of their linear score bins (see select_reg_kernel: the same three
    // steps, with the keys in memory instead of registers).  Four rows of loads are issued before their updates.
    for (int k = tid; k < kSelBins; k += kSelThreads) hist[k] = 0u;
    if (tid < 36) sh[tid] = 0u;
    __syncthreads();
    for (int n0 = tid; n0 < N; n0 += 4 * kSelThreads) {
        uint32_t u[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) u[j] = make_key(min(n0 + j * kSelThreads, N - 1));
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int n = n0 + j * kSelThreads;
            if (n < N) {
                if (in_lds) lds_keys[n] = u[j];
                else if constexpr (G > 0) gk[n] = u[j];
                atomicAdd(&hist[linear_bin(u[j])], 1u);
            }
        }
    }
    __syncthreads();

    // ---- the bin holding the B-th largest: thread t owns bins 2047-2t and 2046-2t, running count from the top
    {
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
        const uint32_t excl = cum - v0 - v1, want = (uint32_t)B;
        if (excl < want && want <= excl + v0) {          // exactly one thread and bin holds the B-th key
            sh[0] = (uint32_t)(kSelBins - 1 - 2 * tid);
            sh[1] = want - excl;
        } else if (excl + v0 < want && want <= cum) {
            sh[0] = (uint32_t)(kSelBins - 2 - 2 * tid);
            sh[1] = want - excl - v0;
        }
    }
    __syncthreads();
    const int sel_bin = (int)sh[0];
    uint32_t need = sh[1];   // how many keys of the selected bin are kept (>= 1)

    // ---- gather the selected bin's keys (any order; the ranks below do not depend on it)
    for (int n0 = 0; n0 < N; n0 += kSelThreads) {
        const int n = n0 + tid;
        const uint32_t u = n < N ? get_key(n) : 0u;
        const bool hit = n < N && linear_bin(u) == sel_bin;
        const uint64_t hm = __ballot(hit);
        if (hm) {
            uint32_t base = 0u;
            if (lane == 0) base = atomicAdd(&sh[2], (uint32_t)__popcll(hm));
            base = __builtin_amdgcn_readfirstlane(base);
            const uint32_t pos = base + (uint32_t)__popcll(hm & ((1ull << lane) - 1ull));
            if (hit && pos < (uint32_t)kSelCand) {
                cand_key[pos] = u;
                cand_idx[pos] = n;
            }
        }
    }
    __syncthreads();
    const uint32_t m = sh[2];
    uint32_t thr;
    if (m <= (uint32_t)kSelCand) {
        // exact rank of every candidate among the candidates: key descending, slot ascending
        for (uint32_t c = tid; c < m; c += kSelThreads) {
            const uint32_t kc = cand_key[c];
            const int32_t ic = cand_idx[c];
            uint32_t rank = 0u;
            for (uint32_t o = 0; o < m; ++o) {
                const uint32_t ko = cand_key[o];
                rank += (ko > kc || (ko == kc && cand_idx[o] < ic)) ? 1u : 0u;
            }
            if (rank == need - 1u) sh[3] = kc;   // the last kept candidate defines the threshold
        }
        __syncthreads();
        thr = sh[3];
        // threshold ties kept = need - (candidates strictly above the threshold)
        uint32_t above = 0u;
        for (uint32_t c = tid; c < m; c += kSelThreads) above += cand_key[c] > thr ? 1u : 0u;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) above += __shfl_xor(above, o, 64);
        if (lane == 0 && above) atomicAdd(&sh[4], above);
        __syncthreads();
        need -= sh[4];
    } else {
        // too many keys in one bin (many equal scores): one bit at a time, keys of the bin only
        uint32_t prefix = 0u, mask = 0u;
#pragma unroll 1
        for (int bit = 31; bit >= 0; --bit) {
            const uint32_t bm = 1u << bit;
            uint32_t c = 0u;
            for (int n0 = 0; n0 < N; n0 += kSelThreads) {
                const int n = n0 + tid;
                const uint32_t u = n < N ? get_key(n) : 0u;
                const bool in = n < N && linear_bin(u) == sel_bin;
                c += (uint32_t)__popcll(__ballot(in && (u & mask) == prefix && (u & bm) != 0u));
            }
            if (lane == 0 && c) atomicAdd(&sh[4 + bit], c);
            __syncthreads();
            const uint32_t ones = sh[4 + bit];
            if (ones >= need) prefix |= bm;
            else need -= ones;
            mask |= bm;
        }
        thr = prefix;
    }
    // keys > thr are kept; of the keys == thr the first `need` slots

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

// Register-resident variant for sequences of at most THREADS * KPT keys: every thread keeps KPT keys
// (slot n = j * THREADS + tid) in registers.  Built as 256 x 16 (up to 4096 keys: small workgroups, cheap
// barriers, eight per CU), 1024 x 8 and 1024 x 32.
//   1. One histogram pass over 2048 *linear* bins of the score on [-4, 12) (monotone in the score, so
//      a valid coarse partition; z-scores spread over hundreds of bins, whereas the top bits of their
//      float image share a handful of values and would serialise the LDS atomics).
//   2. The bin holding the B-th largest score is found with one scan; its few keys are gathered in LDS
//      and ranked exactly (key descending, slot ascending), which gives the threshold key and the number
//      of threshold ties to keep.  A bin with more keys than the LDS list holds (many equal scores)
//      is resolved one bit at a time from the registers instead.
//   3. Ordered emit with three barriers: per-(row, wave) counts from ballots, one scan, the stores.
template <int G, int KPT, int THREADS>
__global__ __launch_bounds__(THREADS) void select_reg_kernel(SelectArgs a)
{
    constexpr int kWaves = THREADS / 64;
    constexpr int kBinsPerThread = kSelBins / THREADS;
    __shared__ uint32_t hist[kSelBins];
    __shared__ uint32_t cand_store[2 * kSelCand];   // candidate keys, then their slots (later the fill's move list)
    uint32_t *const cand_key = cand_store;
    int32_t *const cand_idx = reinterpret_cast<int32_t *>(cand_store + kSelCand);
    __shared__ uint32_t row_g[KPT * kWaves], row_e[KPT * kWaves];   // [row j][wave], then exclusive prefixes
    __shared__ uint32_t scan_tot[2][kWaves];
    __shared__ uint32_t sh[36];   // 0: selected bin, 1: need inside it, 2: candidate count, 3: threshold key, 4..35: bit counters / tie count

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int inst = blockIdx.x;
    const int s = (inst / a.n_kv_heads) % a.n_seqs;
    const int N = clamp_len(a.seq_len[s], a.max_seq_len);
    const int B = instance_budget(a, inst);
    int32_t *out = a.kept_idx + (int64_t)inst * a.budget;
    if (tid == 0) a.kept_cnt[inst] = N < B ? N : B;
    // the eviction in place that may follow: the histogram and the candidate arrays are free by then
    auto fill_tail = [&](int cnt) {
        if constexpr (THREADS == kFillThreads) {
            if (a.fill) {
                __syncthreads();   // out[] is complete and nobody reads hist or the candidates any more
                fill_block(a.fa, inst, cnt, out, reinterpret_cast<int32_t *>(cand_store), hist, scan_tot[0],
                           reinterpret_cast<int32_t *>(&sh[0]));
            }
        }
    };
    if (B == 0) {   // a head whose own budget is 0 keeps nothing
        fill_tail(0);
        return;
    }
    if (N <= B) {  // nothing to evict: keep every slot
        for (int n = tid; n < N; n += THREADS) out[n] = n;
        fill_tail(N);
        return;
    }
    for (int k = tid; k < kSelBins; k += THREADS) hist[k] = 0u;
    if (tid < 36) sh[tid] = 0u;
    __shared__ double zst[2 * (G > 0 ? G : 1)], zpart[32 * (G > 0 ? G : 1)];
    if constexpr (G > 0) {
        if (a.partials)   // statistics from the moments (uniform over the launch)
            block_stats<G>(a.partials + (int64_t)inst * a.n_tiles * (2 * G), (N + a.tile_keys - 1) / a.tile_keys, N, tid,
                           zpart, zst);
    }
    __syncthreads();

    // ---- keys into registers, histogram of their linear bins.  A slot past the end holds key 0, which no finite
    // score maps to (the smallest, -inf, is 0x007fffff) and which lies below every threshold: the later phases
    // need no bounds test, only "key != 0" where a bin is recomputed.
    uint32_t key[KPT];
    {
        const float *rw = G > 0 ? a.raw + (int64_t)inst * (G > 0 ? G : 1) * a.max_seq_len : nullptr;
        const float *fs = G == 0 ? a.final_ + (int64_t)inst * a.max_seq_len : nullptr;
        ZParams zp[G > 0 ? G : 1];
        if constexpr (G > 0) {
#pragma unroll
            for (int g = 0; g < G; ++g)
                zp[g] = a.partials ? z_params(zst[2 * g], zst[2 * g + 1])
                                   : z_params(a.stats[((int64_t)inst * G + g) * 2], a.stats[((int64_t)inst * G + g) * 2 + 1]);
        }
        // Rows are taken 16 at a time (fewer with many query heads, and in the 256-thread variant, whose occupancy
        // depends on its register count; measured: 16 rows 729 us on config 3, was 940; 8 rows 216 us at steady state,
        // was 240): first the keys of the chunk with unconditional loads (a slot past the end
        // re-reads the last one), so that the compiler may issue the loads of many rows before it waits for the
        // first -- one row at a time the phase is bound by load latency --, then the chunk's histogram updates,
        // whose branches also keep the next chunk's loads from being hoisted (registers).
        constexpr int kChunkMax = THREADS == 256 ? (G > 4 ? 4 : 8) : G > 6 ? 4 : G > 4 ? 8 : 16;
        constexpr int kChunk = KPT < kChunkMax ? KPT : kChunkMax;
#pragma unroll
        for (int j0 = 0; j0 < KPT; j0 += kChunk) {
#pragma unroll
            for (int j = j0; j < j0 + kChunk; ++j) {
                const int n = j * THREADS + tid;
                const int nc = min(n, N - 1);
                float f;
                if constexpr (G > 0) {
#pragma unroll
                    for (int g = 0; g < G; ++g) {
                        // raw scores are read exactly once
                        const float z = z_score(__builtin_nontemporal_load(&rw[(int64_t)g * a.max_seq_len + nc]), zp[g]);
                        f = g == 0 ? z : fmaxf(f, z);
                    }
                } else {
                    f = __builtin_nontemporal_load(&fs[nc]);
                }
                key[j] = n < N ? order_key(f) : 0u;
            }
#pragma unroll
            for (int j = j0; j < j0 + kChunk; ++j)
                if (key[j] != 0u) atomicAdd(&hist[linear_bin(key[j])], 1u);
        }
    }
    __syncthreads();

    // ---- the bin holding the B-th largest: thread t owns bins 2047 - t*kBinsPerThread and the ones just below
    {
        uint32_t v[kBinsPerThread];
        uint32_t cum = 0u;
#pragma unroll
        for (int k = 0; k < kBinsPerThread; ++k) {
            v[k] = hist[kSelBins - 1 - kBinsPerThread * tid - k];
            cum += v[k];
        }
        const uint32_t own = cum;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const uint32_t t = __shfl_up(cum, o, 64);
            if (lane >= o) cum += t;
        }
        if (lane == 63) scan_tot[0][wave] = cum;
        __syncthreads();
        for (int w = 0; w < wave; ++w) cum += scan_tot[0][w];
        uint32_t excl = cum - own;
        const uint32_t need = (uint32_t)B;
#pragma unroll
        for (int k = 0; k < kBinsPerThread; ++k) {
            if (excl < need && need <= excl + v[k]) {
                sh[0] = (uint32_t)(kSelBins - 1 - kBinsPerThread * tid - k);
                sh[1] = need - excl;
            }
            excl += v[k];
        }
    }
    __syncthreads();
    const int sel_bin = (int)sh[0];
    uint32_t need = sh[1];   // how many keys of the selected bin are kept (>= 1)

    // ---- gather the selected bin's keys (any order; ranks below do not depend on it)
#pragma unroll
    for (int j = 0; j < KPT; ++j) {
        const int n = j * THREADS + tid;
        const bool hit = key[j] != 0u && linear_bin(key[j]) == sel_bin;
        const uint64_t hm = __ballot(hit);
        if (hm) {
            uint32_t base = 0u;
            if (lane == 0) base = atomicAdd(&sh[2], (uint32_t)__popcll(hm));
            base = __builtin_amdgcn_readfirstlane(base);
            const uint32_t pos = base + (uint32_t)__popcll(hm & ((1ull << lane) - 1ull));
            if (hit && pos < (uint32_t)kSelCand) {
                cand_key[pos] = key[j];
                cand_idx[pos] = n;
            }
        }
    }
    __syncthreads();
    const uint32_t m = sh[2];
    uint32_t thr;
    if (m <= (uint32_t)kSelCand) {
        // exact rank of every candidate among the candidates: key descending, slot ascending
        for (uint32_t c = tid; c < m; c += THREADS) {
            const uint32_t kc = cand_key[c];
            const int32_t ic = cand_idx[c];
            uint32_t rank = 0u;
            for (uint32_t o = 0; o < m; ++o) {
                const uint32_t ko = cand_key[o];
                rank += (ko > kc || (ko == kc && cand_idx[o] < ic)) ? 1u : 0u;
            }
            if (rank == need - 1u) sh[3] = kc;   // the last kept candidate defines the threshold
        }
        __syncthreads();
        thr = sh[3];
        // threshold ties kept = need - (candidates strictly above the threshold)
        uint32_t above = 0u;
        for (uint32_t c = tid; c < m; c += THREADS) above += cand_key[c] > thr ? 1u : 0u;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) above += __shfl_xor(above, o, 64);
        if (lane == 0 && above) atomicAdd(&sh[4], above);
        __syncthreads();
        need -= sh[4];
    } else {
        // too many keys in one bin (many equal scores): one bit at a time, keys of the bin only
        uint32_t prefix = 0u, mask = 0u;
#pragma unroll 1
        for (int bit = 31; bit >= 0; --bit) {
            const uint32_t bm = 1u << bit;
            uint32_t c = 0u;
#pragma unroll
            for (int j = 0; j < KPT; ++j) {
                const bool in = key[j] != 0u && linear_bin(key[j]) == sel_bin;
                c += (uint32_t)__popcll(__ballot(in && (key[j] & mask) == prefix && (key[j] & bm) != 0u));
            }
            if (lane == 0 && c) atomicAdd(&sh[4 + bit], c);
            __syncthreads();
            const uint32_t ones = sh[4 + bit];
            if (ones >= need) prefix |= bm;
            else need -= ones;
            mask |= bm;
        }
        thr = prefix;
    }
    // keys > thr are kept; of the keys == thr the first `need` slots

    // ---- ordered emit: slot order is row-major (row j, then wave, then lane)
#pragma unroll
    for (int j = 0; j < KPT; ++j) {
        const uint64_t gm = __ballot(key[j] > thr), em = __ballot(key[j] == thr);
        if (lane == 0) {
            row_g[j * kWaves + wave] = (uint32_t)__popcll(gm);
            row_e[j * kWaves + wave] = (uint32_t)__popcll(em);
        }
    }
    __syncthreads();
    {   // exclusive scan over the KPT*16 (row, wave) counts: thread t owns entry t
        constexpr int kEntries = KPT * kWaves;
        static_assert(kEntries <= THREADS, "one thread per (row, wave) entry");
        uint32_t vg = tid < kEntries ? row_g[tid] : 0u, ve = tid < kEntries ? row_e[tid] : 0u;
        uint32_t cg = vg, ce = ve;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const uint32_t tg = __shfl_up(cg, o, 64), te = __shfl_up(ce, o, 64);
            if (lane >= o) {
                cg += tg;
                ce += te;
            }
        }
        if (lane == 63) {
            scan_tot[0][wave] = cg;
            scan_tot[1][wave] = ce;
        }
        __syncthreads();
        for (int w = 0; w < wave; ++w) {
            cg += scan_tot[0][w];
            ce += scan_tot[1][w];
        }
        if (tid < kEntries) {
            row_g[tid] = cg - vg;
            row_e[tid] = ce - ve;
        }
    }
    __syncthreads();
    const uint64_t below = (1ull << lane) - 1ull;
#pragma unroll
    for (int j = 0; j < KPT; ++j) {
        const int n = j * THREADS + tid;
        const bool gt = key[j] > thr, eq = key[j] == thr;
        const uint64_t gm = __ballot(gt), em = __ballot(eq);
        const uint32_t g_before = row_g[j * kWaves + wave] + (uint32_t)__popcll(gm & below);
        const uint32_t e_before = row_e[j * kWaves + wave] + (uint32_t)__popcll(em & below);
        if (gt || (eq && e_before < need)) out[g_before + (e_before < need ? e_before : need)] = n;
    }
    fill_tail(B);
}

template <int G>
tri_status launch_select_g(const SelectArgs &sa, int n_inst, hipStream_t st)
{
    if (sa.max_seq_len <= 16 * 256) {   // short sequences: small workgroups, cheap barriers, many per CU
        hipLaunchKernelGGL((select_reg_kernel<G, 16, 256>), dim3(n_inst), dim3(256), 0, st, sa);
        return hip_status("select_reg_kernel");
    }
    if (sa.max_seq_len <= 8 * kSelThreads) {
        hipLaunchKernelGGL((select_reg_kernel<G, 8, kSelThreads>), dim3(n_inst), dim3(kSelThreads), 0, st, sa);
        return hip_status("select_reg_kernel");
    }
    if (sa.max_seq_len <= 32 * kSelThreads) {
        hipLaunchKernelGGL((select_reg_kernel<G, 32, kSelThreads>), dim3(n_inst), dim3(kSelThreads), 0, st, sa);
        return hip_status("select_reg_kernel");
    }
    // Longer than the register-resident kernel takes.  Two launches split the head-instances by length on the
    // device: those whose keys fit LDS, and the rest, whose keys go through the workspace -- that launch asks for no
    // dynamic LDS, so two workgroups share a CU and one's load phase overlaps the other's ranking and emit.
    auto kern = select_kernel<G>;
    const size_t lds = (size_t)kSelLdsKeys * sizeof(uint32_t);
    if (hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
        return hip_status("hipFuncSetAttribute(select_kernel)");
    SelectArgs lo = sa, hi = sa;
    lo.lds_keys = kSelLdsKeys;
    lo.n_above = -1;
    lo.n_upto = kSelLdsKeys;
    hi.lds_keys = 0;
    hi.n_above = kSelLdsKeys;
    hi.n_upto = sa.max_seq_len;
    hipLaunchKernelGGL(kern, dim3(n_inst), dim3(kSelThreads), lds, st, lo);
    tri_status rc = hip_status("select_kernel");
    if (rc != TRI_OK) return rc;
    hipLaunchKernelGGL(kern, dim3(n_inst), dim3(kSelThreads), 0, st, hi);
    return hip_status("select_kernel");
}

}  // namespace

tri_status launch_select(const tri_model &m, const float *final_scores, const float *raw, const double *stats,
                         const double *partials, MomentLayout moments, uint32_t *scratch, const tri_cache &c,
                         int32_t budget, int32_t *kept_idx, int32_t *kept_cnt, hipStream_t st, const FillTail *fill,
                         bool *fill_taken)
{
    if (fill_taken) *fill_taken = false;
    const int n_inst = m.n_layers * c.n_seqs * m.n_kv_heads;
    if (n_inst <= 0) return TRI_OK;
    SelectArgs sa{final_scores, raw, stats, partials, moments.n_tiles, moments.tile_keys, scratch, c.seq_len, kept_idx,
                  kept_cnt, c.n_seqs, m.n_kv_heads,
                  c.max_seq_len, budget, c.max_seq_len < kSelLdsKeys ? (c.max_seq_len > 0 ? c.max_seq_len : 1) : kSelLdsKeys,
                  m.head_budgets, -1, c.max_seq_len};
    sa.fill = 0;
    // Sequences short enough for the 256-thread kernel, whose workgroup is the fill's: the eviction in place rides
    // along (its move list takes the candidate arrays' place, so the budget may not exceed their length) -- on small
    // batches, whose workgroups are all resident at once (eight per CU): there the launch saved counts (one sequence
    // of 288 head-instances: 0.147 -> 0.142 ms per step, four: 0.299 -> 0.291), whereas 18432 head-instances take
    // 0.74 ms this way against 0.21 + 0.44 ms as two launches.
    int n_cu = 0;
    if (fill && fill_taken && c.max_seq_len <= 16 * kFillThreads && budget <= kSelCand) {
        const tri_status rcu = device_cus(&n_cu);
        if (rcu != TRI_OK) return rcu;
    }
    if (n_cu > 0 && n_inst <= 8 * n_cu) {
        sa.fa = FillArgs{make_view(m, c), fill->new_seq_len, budget, c.dtype == TRI_BF16 ? 2 : 4,
                         kHeadDim * (c.dtype == TRI_BF16 ? 2 : 4) / 16};
        sa.fill = 1;
        *fill_taken = true;
    }
    if (final_scores) return launch_select_g<0>(sa, n_inst, st);
    switch (m.n_q_heads / m.n_kv_heads) {
        case 1: return launch_select_g<1>(sa, n_inst, st);
        case 2: return launch_select_g<2>(sa, n_inst, st);
        case 3: return launch_select_g<3>(sa, n_inst, st);
        case 4: return launch_select_g<4>(sa, n_inst, st);
        case 5: return launch_select_g<5>(sa, n_inst, st);
        case 6: return launch_select_g<6>(sa, n_inst, st);
        case 7: return launch_select_g<7>(sa, n_inst, st);
        case 8: return launch_select_g<8>(sa, n_inst, st);
    }
    set_error("group size not built (1 to 8)");
    return TRI_ERR_UNSUPPORTED;
}

}  // namespace tri
