// Internal declarations shared by the HIP translation units of libtri (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "tri.h"

namespace tri {

constexpr int kHeadDim = 128;
constexpr int kBands = 64;        // F = head_dim / 2
constexpr int kScoreTile = 256;   // keys scored by one workgroup
constexpr int kMaxOffsets = 64;
constexpr int kMaxGroup = 8;

// Bytes of the library's own scratch array (tri_compress_step_static), one copy per GPU.
#ifndef TRI_STATIC_SCRATCH_BYTES
#define TRI_STATIC_SCRATCH_BYTES (64u << 20)
#endif

// Device-side view of a tri_cache (plain copy of the descriptor's fields).
struct CacheView {
    const void *k;
    const void *v;
    const int32_t *pos;
    const int32_t *seq_len;
    const int32_t *cur_pos;
    const int32_t *block_table;
    int64_t stride_layer, stride_sb, stride_head, stride_slot;
    int64_t pos_stride_layer, pos_stride_sb, pos_stride_head;
    int32_t n_seqs, n_kv_heads;
    int32_t max_seq_len;
    int32_t block_shift;   // log2(block_size), -1 = contiguous
    int32_t max_blocks;
    int32_t k_rotated;     // keys stored post-RoPE: no rotation in the score kernel
};

// A sequence length as read from device memory, forced into [0, max_seq_len]: grids, score-array strides and
// workspace areas are sized by the host's max_seq_len, so a larger value must never reach an index.
__device__ __forceinline__ int clamp_len(int n, int max_seq_len) { return min(max(n, 0), max_seq_len); }

// Section 4.3, z-score of one raw score: (s - mu) / sigma with mu held as two floats (the double split into hi + lo)
// and 1/sigma as one.  Three fp32 operations that agree with the double-precision expression to about two units in
// the last place (raw - mu_hi is exact when the two are within a factor of two).  Every kernel that forms a final
// score goes through this one function, so the fused step and tri_score + tri_select_topk agree bit for bit.
struct ZParams {
    float mu_hi, mu_lo, rs;
};
__device__ __forceinline__ ZParams z_params(double mu, double inv_sigma)
{
    ZParams p;
    p.mu_hi = (float)mu;
    p.mu_lo = (float)(mu - (double)p.mu_hi);
    p.rs = (float)inv_sigma;
    return p;
}
__device__ __forceinline__ float z_score(float raw, const ZParams &p) { return ((raw - p.mu_hi) - p.mu_lo) * p.rs; }

// Section 4.3, mu_g and 1/sigma_g of one query head from the per-tile sums of its raw scores and of their squares.
// The tiles are added in sixteen interleaved groups (one thread each) and the groups in order, in stats_kernel and
// in the selection kernels (block_stats) alike, so both get the same bits.
__device__ __forceinline__ void moments_to_stats(double s1, double s2, int N, double *mean_out, double *rsig_out)
{
    double mean = 0.0, rsig = 0.0;
    if (N > 0) {
        mean = s1 / (double)N;
        const double msq = s2 / (double)N;
        const double var = msq - mean * mean;
        // sigma = 0: the head contributes 0.  The raw scores are fp32 sums of 192 products, so scores that are equal
        // in exact arithmetic may differ in their last bits (the same key scored against two different table
        // bases), and the moments carry that noise: a spread below 3e-6 of the root mean square is not
        // distinguishable from zero and is read as zero.
        if (var > 1e-11 * msq) rsig = 1.0 / sqrt(var);
    }
    *mean_out = mean;
    *rsig_out = rsig;
}

// Statistics of a head-instance's G query heads inside a workgroup of at least 32 G threads: pt = the
// head-instance's [tiles][2G] moments, part = 32 G doubles and zst = 2 G doubles of LDS; on return (after a barrier)
// zst[2g], zst[2g + 1] = mean and 1/sigma of head g.
template <int G>
__device__ __forceinline__ void block_stats(const double *pt, int tiles, int N, int tid, double *part, double *zst)
{
    if (tid < 2 * G * 16) {
        const int col = tid >> 4, k = tid & 15;
        double acc = 0.0;
        for (int t = k; t < tiles; t += 16) acc += pt[(int64_t)t * (2 * G) + col];
        part[col * 16 + k] = acc;
    }
    __syncthreads();
    if (tid < G) {
        double s1 = 0.0, s2 = 0.0;
        for (int k = 0; k < 16; ++k) {
            s1 += part[tid * 16 + k];
            s2 += part[(G + tid) * 16 + k];
        }
        moments_to_stats(s1, s2, N, &zst[2 * tid], &zst[2 * tid + 1]);
    }
    __syncthreads();
}

typedef unsigned int uint4v __attribute__((ext_vector_type(4)));
// 16 bytes that a step reads once / writes and does not read again: non-temporal hint (measured on this GPU: a
// streaming read reaches 7.0 TB/s with it and 6.2 TB/s without; the gather runs 10 % faster with such stores)
__device__ __forceinline__ uint4 load_stream16(const char *p)
{
    const uint4v t = __builtin_nontemporal_load(reinterpret_cast<const uint4v *>(p));
    return make_uint4(t.x, t.y, t.z, t.w);
}
__device__ __forceinline__ void store_stream16(char *p, const uint4 &v)
{
    __builtin_nontemporal_store(uint4v{v.x, v.y, v.z, v.w}, reinterpret_cast<uint4v *>(p));
}

// Element offset of slot n of (layer, seq, head) in k / v.
// The slot stride is below 2^31 (checked on the host) and n >= 0, so the per-lane product is one 32 x 32 -> 64
// bit multiply; everything else is uniform over a workgroup and stays in scalar registers.
__device__ __forceinline__ int64_t slot_offset(const CacheView &c, int n)
{
    return (int64_t)((uint64_t)(uint32_t)n * (uint32_t)c.stride_slot);
}
__device__ __forceinline__ int64_t kv_offset(const CacheView &c, int l, int s, int h, int n)
{
    int64_t base = (int64_t)l * c.stride_layer + (int64_t)h * c.stride_head;
    if (c.block_shift < 0) return base + (int64_t)s * c.stride_sb + slot_offset(c, n);
    int b = c.block_table[(int64_t)s * c.max_blocks + (n >> c.block_shift)];
    return base + (int64_t)b * c.stride_sb + slot_offset(c, n & ((1 << c.block_shift) - 1));
}

// Element offset of slot n of (layer, seq, head) in pos.
__device__ __forceinline__ int64_t pos_offset(const CacheView &c, int l, int s, int h, int n)
{
    int64_t base = (int64_t)l * c.pos_stride_layer + (int64_t)h * c.pos_stride_head;
    if (c.block_shift < 0) return base + (int64_t)s * c.pos_stride_sb + n;
    int b = c.block_table[(int64_t)s * c.max_blocks + (n >> c.block_shift)];
    return base + (int64_t)b * c.pos_stride_sb + (n & ((1 << c.block_shift) - 1));
}

// Workspace carve-up (all offsets 256-byte aligned).
struct Workspace {
    size_t band_rev;   // double [F]: omega_f / 2pi
    size_t fold_phasors;   // double [1 + S][F][2]: mean over the offsets of e^{i w delta}; e^{i w cur_pos[s]}
    size_t phasors;    // relative-position phasor table of the MFMA score kernel
    size_t table;      // float  [L][S][Hkv][F][3][G]: folded centre table
    size_t work;       // int32: item counter and work list of the MFMA score kernel
    size_t partials;   // double [L][S][Hkv][n_tiles][2G]: per-tile sum and sum of squares
    size_t stats;      // double [L][S][Hkv][G][2]: mean and 1/sigma
    size_t raw;        // float  [L][S][Hq][Nmax] (used when the caller passes no raw_out)
    size_t final_;     // float  [L][S][Hkv][Nmax] (tri_compress_step only)
    size_t total;
};
Workspace workspace_layout(const tri_model &m, const tri_cache &c, int32_t budget);

void set_error(const char *fmt, ...);
tri_status check_model(const tri_model *m);
tri_status check_cache(const tri_model *m, const tri_cache *c, bool need_v, const char *what);
tri_status check_limits(const tri_model &m, const tri_cache &c, int32_t budget, const char *what);
tri_status check_fill_budget(int32_t budget);   // tri_compact_fill's own limit on the budget
CacheView make_view(const tri_model &m, const tri_cache &c);
tri_status hip_status(const char *what);
tri_status device_cus(int *n_cu);   // compute units of the current GPU (asked once per GPU)
// timing hook: the next event pair to record around a score-kernel launch, if any is attached
bool timing_next(hipEvent_t *start, hipEvent_t *stop);

// launchers (each validates nothing; the entry points in tri_api.hip do)
tri_status launch_centers(const tri_model &m, const void *q, int32_t q_dtype, int64_t n_tokens,
                          float *out, double *sums, int32_t first, hipStream_t st);
tri_status launch_centers_finalize(const tri_model &m, const double *sums, int64_t total_tokens, float *out,
                                   hipStream_t st);
tri_status launch_diagnostics(const tri_model &m, const float *q_centers, const float *k_centers, float *mrl,
                              float *contrib, int32_t top_k, int32_t *top, hipStream_t st);
// final_out == NULL (fused step): the moments stay in the workspace's `partials` (layout returned through
// moments) and no statistics are formed here: the selection does that itself.
struct MomentLayout {
    int32_t n_tiles;     // entries per head-instance
    int32_t tile_keys;   // keys per entry
};
tri_status launch_score(const tri_model &m, const float *centers, const tri_cache &c, float *final_out,
                        float *raw_out, char *ws, const Workspace &wl, MomentLayout *moments, hipStream_t st);
// final_scores given: select on them; else form them from the raw scores and either stats (mean, 1/sigma) or, when
// partials is given, the per-tile moments (scratch: keys of long sequences)
// fill given and taken (*fill_taken set): the selection's workgroups also evict their head-instances in place, as
// launch_compact_fill would afterwards (short sequences only; else the caller launches the fill itself)
struct FillTail {
    int32_t *new_seq_len;   // [S] or NULL
};
tri_status launch_select(const tri_model &m, const float *final_scores, const float *raw, const double *stats,
                         const double *partials, MomentLayout moments, uint32_t *scratch, const tri_cache &c,
                         int32_t budget, int32_t *kept_idx, int32_t *kept_cnt, hipStream_t st,
                         const FillTail *fill = nullptr, bool *fill_taken = nullptr);
tri_status launch_compact(const tri_model &m, const tri_cache &src, const tri_cache &dst, int32_t budget,
                          const int32_t *kept_idx, const int32_t *kept_cnt, int32_t *new_seq_len,
                          hipStream_t st);

tri_status launch_compact_fill(const tri_model &m, const tri_cache &c, int32_t budget, const int32_t *kept_idx,
                               const int32_t *kept_cnt, int32_t *new_seq_len, hipStream_t st);

}  // namespace tri
