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
    int32_t first_mult;      // MFMA kernel only: workgroup b starts on item (b * first_mult) mod grid size
    int32_t *work;           // MFMA kernel only: item counter and work list (kFastWorkInts(S, Nmax) ints)
    int32_t chunk_keys;      // MFMA kernels only: keys per work item (= keys per entry of `partials`)
};

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// Keys per work item of the MFMA score kernels (= keys per entry of `partials` on that path): kFastChunk, or for
// the one-key-per-lane kernel on a small batch a few rounds of its waves (see lane_chunk_keys), kMinChunk at least.
constexpr int kFastChunk = 8192;
constexpr int kMinChunk = 512;
constexpr int lane_waves(int G) { return G > 4 ? 8 : 12; }      // waves per workgroup of the one-key-per-lane kernel
// A batch with few tiles per CU is cut into items of r rounds (one tile per wave and round) so that every CU gets
// about four items or more; r = 1 is the smallest item.
inline int lane_chunk_keys(int G, int64_t instances, int max_seq_len, int n_cu)
{
    const int round_keys = lane_waves(G) * 64;
    const int64_t tiles = instances * (((int64_t)max_seq_len + 63) / 64);
    const int64_t r = tiles / (4 * (int64_t)(n_cu > 0 ? n_cu : 1) * lane_waves(G));
    if (r * round_keys >= kFastChunk) return kFastChunk;
    return (int)(r > 1 ? r : 1) * round_keys;
}
// Relative positions covered by the phasor table.
constexpr int kPhasorRange = 128;
constexpr int kPhasorBlockStride = kPhasorRange * 16 + 64;      // bytes per 4-band chunk (64 B skew)
constexpr int kPhasorHalfStride = 16 * kPhasorBlockStride;      // bytes per half (bands 0-1 / 2-3 of a chunk)
constexpr int kPhasorBytes = 2 * kPhasorHalfStride;

// Work list of the MFMA score kernel, built on the device from the sequence lengths by one workgroup of any size
// (kWorkThreads at most): [0] the kernel's shared item counter (zeroed here), [1] entries per (layer, KV head), from
// kWorkHeader on one (sequence, chunk) pair per chunk of chunk_keys keys that exists.
constexpr int kWorkHeader = 4;
constexpr int kWorkThreads = 256;
__device__ __forceinline__ void build_work_list(const int32_t *seq_len, int n_seqs, int max_seq_len, int chunk_keys,
                                                int32_t *work)
{
    __shared__ int start[kWorkThreads + 1];
    const int tid = threadIdx.x, nt = blockDim.x;
    const int seg = (n_seqs + nt - 1) / nt, s0 = min(n_seqs, tid * seg), s1 = min(n_seqs, s0 + seg);
    int cnt = 0;
    for (int s = s0; s < s1; ++s) cnt += (clamp_len(seq_len[s], max_seq_len) + chunk_keys - 1) / chunk_keys;
    start[tid + 1] = cnt;
    __syncthreads();
    if (tid == 0) {
        start[0] = 0;
        for (int k = 1; k <= nt; ++k) start[k] += start[k - 1];
        work[0] = 0;
        work[1] = start[nt];
    }
    __syncthreads();
    int o = start[tid];
    for (int s = s0; s < s1; ++s) {
        const int n = (clamp_len(seq_len[s], max_seq_len) + chunk_keys - 1) / chunk_keys;
        for (int ch = 0; ch < n; ++ch, ++o) {
            work[kWorkHeader + 2 * o] = s;
            work[kWorkHeader + 2 * o + 1] = ch;
        }
    }
}

tri_status launch_phasor_table(double theta, uint4 *phasors, hipStream_t st);
// bf16 keys; G in 1..8
tri_status launch_score_fast(int G, const ScoreArgs &sa, bool half_split, hipStream_t st);
// bf16 keys with interleaved pairs, one key per lane (tri_score_lane.hip); its own phasor table layout
// Its table of e^{i w r}: entry (band pair bp, r) = (cos, sin) of bands 2bp and 2bp+1 at relative position r, at byte
// bp * kLanePairStride + 16 r.  The fold's phasor kernel writes it with kLaneTableEntries extra threads.
constexpr int kLaneRange = 64;                                  // relative positions 0 .. 63
constexpr int kLanePairStride = kLaneRange * 16 + 16;           // bytes per band pair (16 bytes of skew)
constexpr int kLanePhasorBytes = (kBands / 2) * kLanePairStride;
constexpr int kLaneTableEntries = (kBands / 2) * kLaneRange;
__device__ __forceinline__ void lane_phasor_entry(double theta, int t, float4 *out)
{
    constexpr double kTwoPiD = 6.283185307179586476925286766559;
    const int r = t % kLaneRange, bp = t / kLaneRange;
    float v[4];
    for (int k = 0; k < 2; ++k) {
        const int f = 2 * bp + k;
        double x = (double)r * (pow(theta, -2.0 * (double)f / (double)kHeadDim) / kTwoPiD);
        x -= floor(x);
        double s, c;
        sincos(kTwoPiD * x, &s, &c);
        v[2 * k] = (float)c;
        v[2 * k + 1] = (float)s;
    }
    out[bp * (kLanePairStride / 16) + r] = make_float4(v[0], v[1], v[2], v[3]);
}
tri_status launch_score_lane(int G, const ScoreArgs &sa, hipStream_t st);
// ints the MFMA kernel's work list takes: a header and one (sequence, chunk) pair per possible chunk
inline size_t fast_work_ints(int64_t n_seqs, int64_t max_seq_len)
{
    return kWorkHeader + 2 * (size_t)n_seqs * (size_t)((max_seq_len + kMinChunk - 1) / kMinChunk);
}

}  // namespace tri
