// Declarations shared by the two score kernels (generic and MFMA).
#pragma once
#include "tri_internal.h"

namespace tri {

struct ScoreArgs {
    CacheView c;
    const float *table;      // [L][S][Hkv][F][3][G]: folded centre table
    const double *band_rev;  // [F]: omega_f / 2pi
    const uint4 *phasors;    // relative-position phasor table (MFMA kernel only)
    float *raw;              // [L][S][Hq][Nmax]
    double *partials;        // [L][S][Hkv][n_tiles][2G]: per-tile sum and sum of squares
    int32_t n_tiles;         // tiles per head-instance in `partials`
    int32_t n_layers;
    int32_t *work;           // MFMA kernel only: item counter and work list (kFastWorkInts(S, Nmax) ints)
};

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// Keys per workgroup of the MFMA score kernel (= keys per entry of `partials` on that path).
constexpr int kFastChunk = 8192;
// Relative positions covered by the phasor table.
constexpr int kPhasorRange = 128;
constexpr int kPhasorBlockStride = kPhasorRange * 16 + 64;      // bytes per 4-band chunk (64 B skew)
constexpr int kPhasorHalfStride = 16 * kPhasorBlockStride;      // bytes per half (bands 0-1 / 2-3 of a chunk)
constexpr int kPhasorBytes = 2 * kPhasorHalfStride;

tri_status launch_phasor_table(double theta, uint4 *phasors, hipStream_t st);
// bf16 keys; G in 1..8
tri_status launch_score_fast(int G, const ScoreArgs &sa, bool half_split, hipStream_t st);
// ints the MFMA kernel's work list takes: a header and one (sequence, chunk) pair per possible chunk
inline size_t fast_work_ints(int64_t n_seqs, int64_t max_seq_len)
{
    return 4 + 2 * (size_t)n_seqs * (size_t)((max_seq_len + kFastChunk - 1) / kFastChunk);
}

}  // namespace tri
