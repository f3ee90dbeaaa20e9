// Score kernel for bf16 keys with a key spread over sixteen lanes: fp32 MFMA for the contraction over
// (band, component) x query head, a phasor table in LDS for the rotation of the key.  It takes interleaved or
// half-split pairs; the launcher in tri_score.hip sends it the half-split caches and the large paged batches
// (the one-key-per-lane kernel of tri_score_lane.hip takes the rest).
//
// Lane layout (wave64): lane = 4*b + i.  In one step a wave scores 4 keys; lane (b, i) loads the
// 16 bytes holding bands 4b..4b+3 of key i -- exactly the operand layout of
// v_mfma_f32_4x4x1_16b_f32, whose block b multiplies a 4x1 column (rows = keys i) by a 1x4 row
// (columns = query heads j).  Per band the lane produces the rotated key (Re, Im) and the modulus
// and feeds each as an A operand; the B operand is the lane's own table entry (band, component,
// head j = lane % 4), held in registers.  Twelve MFMAs accumulate the lane's four bands; the sixteen
// blocks are then summed with two lane swaps per step and two row rotations shared by the four steps of a
// group (each halving keeps only the lanes whose result survives, so the group's 16 keys x 4 heads end up
// in one register, one value per lane, ready for a single coalesced store).
//
// Rotation of the key (Sections 4.1-4.2, Appendix B.2): k e^{i w p} = (k e^{i w r}) e^{i w base}
// with r = p - base in [0, R).  e^{i w r} comes from a table in LDS (one 16-byte read per two
// bands); e^{-i w base} is folded into the lane's table registers whenever the wave moves its base.
// A step whose four keys span R positions or more takes the direct path instead (phase in double,
// v_sin_f32 / v_cos_f32), so any position layout is handled.
#include <algorithm>
#include <atomic>
#include <type_traits>

#include "tri_score_common.h"

namespace tri {

namespace {

constexpr double kTwoPi = 6.283185307179586476925286766559;
constexpr int kMaxDevices = 64;   // GPUs of one process the occupancy cache distinguishes
// Workgroup size of the score kernel: with more than four query heads per KV head a wave needs more than 128
// registers, so only three waves fit a SIMD; 12-wave workgroups fill them (8-wave ones would leave one of three unused).
constexpr int fast_threads(int G) { return G > 4 ? 768 : 512; }

typedef float float4v __attribute__((ext_vector_type(4)));

// grid (2*16*R / 256), block 256: entry (half hf, chunk b, r) = (cos, sin) of bands 4b+2hf, 4b+2hf+1
// at relative position r, in double, stored at byte hf*HalfStride + b*BlockStride + 16*r.
__global__ __launch_bounds__(256) void phasor_table_kernel(double theta, float4 *out)
{
    const int t = blockIdx.x * 256 + threadIdx.x;
    const int r = t % kPhasorRange, b = (t / kPhasorRange) % 16, hf = t / (kPhasorRange * 16);
    if (hf >= 2) return;
    float v[4];
    for (int k = 0; k < 2; ++k) {
        const int f = 4 * b + 2 * hf + k;
        double x = (double)r * (pow(theta, -2.0 * (double)f / (double)kHeadDim) / kTwoPi);
        x -= floor(x);
        double s, c;
        sincos(kTwoPi * x, &s, &c);
        v[2 * k] = (float)c;
        v[2 * k + 1] = (float)s;
    }
    out[(hf * kPhasorHalfStride + b * kPhasorBlockStride) / 16 + r] = make_float4(v[0], v[1], v[2], v[3]);
}

__device__ __forceinline__ float row_ror_add(float c, int ctrl_is_8)
{
    const int v = __float_as_int(c);
    const int r = ctrl_is_8 ? __builtin_amdgcn_update_dpp(0, v, 0x128, 0xf, 0xf, false)
                            : __builtin_amdgcn_update_dpp(0, v, 0x124, 0xf, 0xf, false);
    return c + __int_as_float(r);
}

// Sum the 16 blocks of a 4x4x1 accumulator.  In: lane (b, j) reg i = partial of (key i, head j) over
// the lane's 4 bands.  Out: lane q of row r (lanes 16r..16r+15) holds the sum over blocks q/4, q/4+4, q/4+8,
// q/4+12 of (key r, head q % 4); merge_steps() adds the four lanes of a row that share a head.
__device__ __forceinline__ float reduce_blocks(float4v acc)
{
    auto s02 = __builtin_amdgcn_permlane32_swap(__float_as_uint(acc[0]), __float_as_uint(acc[2]), false, false);
    auto s13 = __builtin_amdgcn_permlane32_swap(__float_as_uint(acc[1]), __float_as_uint(acc[3]), false, false);
    // lanes < 32: keys 0 / 1 summed over both halves; lanes >= 32: keys 2 / 3
    const float a0 = __uint_as_float(s02[0]) + __uint_as_float(s02[1]);
    const float a1 = __uint_as_float(s13[0]) + __uint_as_float(s13[1]);
    auto sw = __builtin_amdgcn_permlane16_swap(__float_as_uint(a0), __float_as_uint(a1), false, false);
    return __uint_as_float(sw[0]) + __uint_as_float(sw[1]);   // row r now holds key r, still split over its 4 blocks
}

// Finishes the block sums of four steps at once.  In: c0..c3 = reduce_blocks() of four steps (lane q of a
// row = block q / 4 of that row, head q % 4).  Out: lane q holds the total of step q / 4, head q % 4 -- the
// last two halvings write only the lanes that keep their result (DPP bank mask), so the four steps end up
// side by side in one register without a select.
__device__ __forceinline__ float merge_steps(float c0, float c1, float c2, float c3)
{
    // blocks (q/4, q/4 ^ 2): lanes 0-7 of a row take the first step of the pair, lanes 8-15 the second
    float m01 = row_ror_add(c3, 1), m23 = row_ror_add(c2, 1);
    // a VALU result needs two wait states before a DPP read; the compiler does not see into the statement
    asm("s_nop 1\n\tv_add_f32_dpp %0, %1, %1 row_ror:8 row_mask:0xf bank_mask:0x3" : "+v"(m01) : "v"(c1));
    asm("s_nop 1\n\tv_add_f32_dpp %0, %1, %1 row_ror:8 row_mask:0xf bank_mask:0x3" : "+v"(m23) : "v"(c0));
    // m01 = (step 1 | step 3), m23 = (step 0 | step 2), each still split over blocks (q/4, q/4 ^ 1).
    // lanes 4-7 and 12-15 of m01 + (m01 from 4 lanes below) are the totals of steps 1 and 3 ...
    const int v = __float_as_int(m01);
    float f = m01 + __int_as_float(__builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, true));
    // ... and lanes 0-3 and 8-11 of m23 + (m23 from 4 lanes above) those of steps 0 and 2
    asm("s_nop 1\n\tv_add_f32_dpp %0, %1, %1 row_shl:4 row_mask:0xf bank_mask:0x5" : "+v"(f) : "v"(m23));
    return f;
}

// The lane's slice of the folded centre table for one group of four query heads, rotated by
// e^{-i w base}: what the MFMAs consume.
struct LaneTable {
    float rr[4], ri[4];   // Re / Im of Qhat e^{-i w base} for bands 4b..4b+3
    float cn[4];          // norm-term weight
};

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
// (K rows are read exactly once: load_stream16, the 16-byte load with the non-temporal hint.)

// ROTATE = false: the key is stored post-RoPE, already k e^{i w p}.
// HALF = false: kd holds the (re, im) pairs of the lane's four bands; HALF = true (half-split layout):
// kd = (re of bands 0-1, re of bands 2-3, im of bands 0-1, im of bands 2-3), two bf16 per dword.
template <int NG, bool ROTATE, bool HALF>
__device__ __forceinline__ void score_step(const uint4 kd, const float (&cs)[4], const float (&sn)[4],
                                           const LaneTable (&tb)[NG], float (&out)[NG])
{
    const uint32_t w[4] = {kd.x, kd.y, kd.z, kd.w};
    // First everything the vector ALU does for the four bands, then the twelve matrix instructions in one run: a
    // wave that alternates between the two kinds pays about 3.5 cycles per matrix instruction for it (measured with
    // four waves per SIMD: 16 x (one 4x4x1 + two additions) take 115 ns per SIMD, 20 of the former followed by 32 of
    // the latter 107 ns, which is the sum of their separate rates).
    float kr[4], ki[4], m[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        float re, im;
        if constexpr (HALF) {
            re = (k & 1) ? bf16_hi(w[k >> 1]) : bf16_lo(w[k >> 1]);
            im = (k & 1) ? bf16_hi(w[2 + (k >> 1)]) : bf16_lo(w[2 + (k >> 1)]);
        } else {
            re = bf16_lo(w[k]);
            im = bf16_hi(w[k]);
        }
        // |k_f|^2 from the unpacked pair: fp32 multiplications and fused multiply-adds run at twice the rate of the
        // packed bf16 dot product (and of every integer, conversion or cross-lane instruction) on this GPU
        m[k] = __builtin_amdgcn_sqrtf(fmaf(re, re, im * im));
        kr[k] = ROTATE ? re * cs[k] - im * sn[k] : re;
        ki[k] = ROTATE ? re * sn[k] + im * cs[k] : im;
    }
    __builtin_amdgcn_sched_barrier(0);
    // the wave's priority drops for its matrix run and rises again for the vector work that follows, so that a wave
    // in its vector part outranks those in their matrix runs (ragged paged batch of 6144 head-instances 12.23 -> 12.03 ms,
    // half-split pairs on 36 x 16 x 8 x 32768 keys 7.86 -> 7.60 ms, in one process each)
    __builtin_amdgcn_s_setprio(0);
    float4v acc[NG];
#pragma unroll
    for (int q = 0; q < NG; ++q) acc[q] = float4v{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int k = 0; k < 4; ++k) {
#pragma unroll
        for (int q = 0; q < NG; ++q) acc[q] = __builtin_amdgcn_mfma_f32_4x4x1f32(kr[k], tb[q].rr[k], acc[q], 0, 0, 0);
#pragma unroll
        for (int q = 0; q < NG; ++q) acc[q] = __builtin_amdgcn_mfma_f32_4x4x1f32(ki[k], tb[q].ri[k], acc[q], 0, 0, 0);
#pragma unroll
        for (int q = 0; q < NG; ++q) acc[q] = __builtin_amdgcn_mfma_f32_4x4x1f32(m[k], tb[q].cn[k], acc[q], 0, 0, 0);
    }
    __builtin_amdgcn_s_setprio(2);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int q = 0; q < NG; ++q) out[q] = reduce_blocks(acc[q]);
}

// grid = as many workgroups as the GPU holds at once, block 512 (768 for G > 4).  A workgroup stays for the whole launch and
// takes items -- one (layer, KV head, sequence, chunk of 8192 keys) each, listed by build_work_list() -- from a
// shared counter until they run out; the phasor table is loaded once per workgroup, and neither empty chunks of short sequences nor the order
// in which the hardware hands workgroups to the XCDs cost anything (with one workgroup per chunk slot of the
// longest sequence, ragged batches lost up to a quarter of the kernel's throughput to the empty ones).  The item's
// keys are split evenly over the waves; each wave walks its contiguous share in groups of 16 (4 steps).
// PAGED: block_size >= 16, so a group never straddles a block.
template <int G, bool PAGED, bool ROTATED, bool HALF>
// (the second launch bound keeps every variant at four waves per SIMD for G <= 4, three above: two workgroups per CU)
__global__ __launch_bounds__(fast_threads(G), G > 4 ? 3 : 4) void score_mfma_kernel(ScoreArgs a)
{
    constexpr int NG = (G + 3) / 4;
    constexpr int kFastThreads = fast_threads(G), kFastWaves = kFastThreads / 64;
    extern __shared__ uint4 lds_phasors[];
    __shared__ double red[kFastWaves][2 * 4 * NG];
    __shared__ double lds_rev[kBands];          // omega_f / 2pi
    __shared__ float lds_tab[kBands * 3 * G];   // this head-instance's folded table (no base)
    __shared__ int lds_item;

    const CacheView &c = a.c;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: keeps loop control scalar
    const int b = lane >> 2, i = lane & 3;

    if constexpr (!ROTATED)
        for (int k = tid; k < kPhasorBytes / 16; k += kFastThreads) lds_phasors[k] = a.phasors[k];
    if (tid < kBands) lds_rev[tid] = a.band_rev[tid];
    const int per_lh = __builtin_amdgcn_readfirstlane(a.work[1]);   // items per (layer, KV head)
    const int n_items = per_lh * a.n_layers * c.n_kv_heads;       // below 2^31: checked on the host
    // The first item needs no trip to the shared counter (hundreds of workgroups asking at once queue up on that one
    // address for tens of microseconds, which is what a small batch takes in all): workgroup b starts on item
    // (b * first_mult) mod gridDim.x, a permutation (first_mult is coprime to the grid size); later items are
    // gridDim.x + the counter's value.  The identity (item b) was measured 4 to 11 % slower on the large
    // configurations than this or than a counter-only start; why is not understood -- workgroups go to the XCDs
    // in turn by index, so the identity ties neighbouring items to neighbouring XCDs for the first items and, with
    // equal item durations, for every later one.
    int next_item = (int)(((uint32_t)blockIdx.x * (uint32_t)a.first_mult) % gridDim.x);

  for (;;) {
    // every wave has finished the previous item when it arrives here: lds_tab, red and lds_item are free
    if (tid == 0) lds_item = next_item;
    __syncthreads();
    const int item = __builtin_amdgcn_readfirstlane(lds_item);
    if (item >= n_items) break;   // uniform over the workgroup; the counter only grows, so every workgroup gets here
    if (tid == 0) next_item = (int)gridDim.x + atomicAdd(&a.work[0], 1);   // in flight while this item is scored
    const int lh = item / per_lh, wi = item - lh * per_lh;
    const int l = lh / c.n_kv_heads, h = lh - l * c.n_kv_heads;
    const int s = __builtin_amdgcn_readfirstlane(a.work[kWorkHeader + 2 * wi]);
    const int chunk = __builtin_amdgcn_readfirstlane(a.work[kWorkHeader + 2 * wi + 1]);
    const int N = clamp_len(c.seq_len[s], c.max_seq_len);   // chunk * chunk_keys < N by construction of the list

    const int64_t inst = ((int64_t)l * c.n_seqs + s) * c.n_kv_heads + h;
    for (int k = tid; k < kBands * 3 * G; k += kFastThreads) lds_tab[k] = a.table[inst * (kBands * 3 * G) + k];
    __syncthreads();

    LaneTable tb[NG];
#pragma unroll
    for (int k = 0; k < 4; ++k)
#pragma unroll
        for (int q = 0; q < NG; ++q) {
            const int f = 4 * b + k, g = 4 * q + i;
            const bool on = g < G;
            tb[q].rr[k] = on ? lds_tab[(f * 3 + 0) * G + g] : 0.f;
            tb[q].ri[k] = on ? lds_tab[(f * 3 + 1) * G + g] : 0.f;
            tb[q].cn[k] = on ? lds_tab[(f * 3 + 2) * G + g] : 0.f;
        }

    const int c0 = chunk * a.chunk_keys, c_len = min(N - c0, a.chunk_keys);
    const int wave_keys = ((c_len + kFastWaves - 1) / kFastWaves + 15) & ~15;   // multiple of 16: groups stay aligned
    const int w0 = c0 + wave * wave_keys;
    const int w1 = min(w0 + wave_keys, c0 + c_len);
    const char *ph0 = (const char *)lds_phasors + b * kPhasorBlockStride;
    const int Hq = c.n_kv_heads * G;
    float *rw = a.raw + (((int64_t)l * c.n_seqs + s) * Hq + (int64_t)h * G) * c.max_seq_len;

    double s1[NG], s2[NG];
#pragma unroll
    for (int q = 0; q < NG; ++q) s1[q] = s2[q] = 0.0;

    int base = 0;                      // base = 0 with the unrotated table is a valid state
    const int sub = (lane >> 2) & 3;   // which of 4 consecutive steps this lane keeps for the store
    const int row = lane >> 4;         // key of the step this lane holds after the reduction
    // byte offset of the lane's raw score inside its group's rows: head 4q + i, key 4*sub + row (below 2^32: checked
    // on the host)
    uint32_t st_off[NG];
#pragma unroll
    for (int q = 0; q < NG; ++q)
        st_off[q] = ((uint32_t)(4 * q + i) * (uint32_t)c.max_seq_len + (uint32_t)(4 * sub + row)) * 4u;

    // Addresses.  Everything that depends on the group is wave-uniform (scalar registers); a lane
    // adds its own constant offset: key (4t + i) of the group, 16-byte piece b of the row.
    const uint32_t slot_bytes = (uint32_t)c.stride_slot * 2u;
    const char *krow = (const char *)c.k + ((int64_t)l * c.stride_layer + (int64_t)h * c.stride_head) * 2 +
                       (PAGED ? 0 : (int64_t)s * c.stride_sb * 2);
    const int32_t *prow = c.pos + (int64_t)l * c.pos_stride_layer + (int64_t)h * c.pos_stride_head +
                          (PAGED ? 0 : (int64_t)s * c.pos_stride_sb);
    const int32_t *bt = PAGED ? c.block_table + (int64_t)s * c.max_blocks : nullptr;
    const int bmask = PAGED ? (1 << c.block_shift) - 1 : 0;
    // Loads are issued in the coalesced lane order (lane = 16*key + piece: a wave instruction reads
    // four whole 256-byte rows front to back) and handed to the consumer lane (b, i) = piece b of
    // key i with one cross-lane permute per dword.  Loading straight in consumer order costs the
    // texture-address unit four cache-line lookups per lane quad and makes it the bottleneck.
    const int ld_key = lane >> 4, ld_piece = lane & 15;
    uint32_t koff[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) koff[t] = (uint32_t)(4 * t + ld_key) * slot_bytes + (uint32_t)ld_piece * 16u;
    uint32_t pos_off = (uint32_t)ld_piece * 4u;   // the lane's position inside a group's 16 (same addressing trick)
    const int perm_k = (16 * i + b) * 4;   // ds_bpermute address: source lane of this lane's K piece
    const int perm_p = i * 4;              // source lane (4t + i) of this lane's position at step t, plus 16*t

    // Paged: the wave's share (at most 1024 keys) spans at most 64 blocks plus one; their ids are read once,
    // one per lane, so that no group's addresses wait on a block-table load behind the K loads in flight.
    const int blk0 = PAGED ? (w0 >> c.block_shift) : 0;
    int blk_ids = 0, blk_ids_hi = 0;
    if constexpr (PAGED) {
        blk_ids = bt[min(blk0 + lane, c.max_blocks - 1)];
        blk_ids_hi = bt[min(blk0 + 64, c.max_blocks - 1)];
    }

    // group starting at key n (a multiple of 16): uniform base pointers of its K rows and positions
    auto group_ptrs = [&](int n, const char *&kp, const int32_t *&pq) {
        if constexpr (PAGED) {
            const int rel = (n >> c.block_shift) - blk0;
            const int blk = rel < 64 ? __builtin_amdgcn_readlane(blk_ids, rel) : __builtin_amdgcn_readfirstlane(blk_ids_hi);
            const int slot = n & bmask;
            kp = krow + (int64_t)blk * c.stride_sb * 2 + (int64_t)slot * slot_bytes;
            pq = prow + (int64_t)blk * c.pos_stride_sb + slot;
        } else {
            kp = krow + (int64_t)n * slot_bytes;
            pq = prow + n;
        }
    };

    // all 16 keys of the group exist: no per-lane address arithmetic at all.  kd[t] = rows 4t..4t+3 in
    // load order, pp = the 16 positions (lane l holds key l % 16).
    auto load_full = [&](int n, uint4(&kd)[4], int &pp) {
        const char *kp;
        const int32_t *pq;
        group_ptrs(n, kp, pq);
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            // the offset stays an opaque 32-bit register here: widened once outside the loop it would turn every
            // load address into a 64-bit vector add instead of (scalar base + 32-bit vector offset)
            asm volatile("" : "+v"(koff[t]));
            kd[t] = load_stream16(kp + koff[t]);
        }
        if constexpr (ROTATED) {
            pp = 0;
        } else {
            asm volatile("" : "+v"(pos_off));
            pp = *reinterpret_cast<const int32_t *>(reinterpret_cast<const char *>(pq) + pos_off);
        }
    };

    // last, partial group: keys past the end repeat the last one (their results are discarded)
    auto load_tail = [&](int n, int cnt, uint4(&kd)[4], int &pp) {
        const char *kp;
        const int32_t *pq;
        group_ptrs(n, kp, pq);
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int j = min(4 * t + ld_key, cnt - 1);
            kd[t] = load_stream16(kp + (uint32_t)j * slot_bytes + (uint32_t)ld_piece * 16u);
        }
        pp = ROTATED ? 0 : pq[min(ld_piece, cnt - 1)];
    };

    // Half-split layout: a row is 64 real parts followed by 64 imaginary parts, so piece p < 8 holds the
    // real parts of bands 8p..8p+7 and piece 8 + p their imaginary parts.  Consumer (b, i) needs dwords
    // 2(b&1), 2(b&1)+1 of pieces b>>1 and 8 + (b>>1) of key i.  Four permutes still do: in each, the real
    // pieces offer one dword and the imaginary pieces another, and even / odd consumers read opposite kinds.
    const bool ld_im = ld_piece >= 8, odd_b = (b & 1) != 0;
    const int perm_re = (16 * i + (b >> 1)) * 4, perm_im = perm_re + 8 * 4;
    const int perm_a = odd_b ? perm_im : perm_re, perm_b = odd_b ? perm_re : perm_im;

    // load order -> consumer order
    auto to_consumer = [&](const uint4 &raw) {
        uint4 v;
        if constexpr (HALF) {
            const int r1 = __builtin_amdgcn_ds_bpermute(perm_a, (int)(ld_im ? raw.z : raw.x));
            const int r2 = __builtin_amdgcn_ds_bpermute(perm_b, (int)(ld_im ? raw.x : raw.z));
            const int r3 = __builtin_amdgcn_ds_bpermute(perm_a, (int)(ld_im ? raw.w : raw.y));
            const int r4 = __builtin_amdgcn_ds_bpermute(perm_b, (int)(ld_im ? raw.y : raw.w));
            v.x = (uint32_t)(odd_b ? r2 : r1);   // re of bands 4b, 4b+1
            v.y = (uint32_t)(odd_b ? r4 : r3);   // re of bands 4b+2, 4b+3
            v.z = (uint32_t)(odd_b ? r1 : r2);   // im of bands 4b, 4b+1
            v.w = (uint32_t)(odd_b ? r3 : r4);   // im of bands 4b+2, 4b+3
        } else {
            v.x = (uint32_t)__builtin_amdgcn_ds_bpermute(perm_k, (int)raw.x);
            v.y = (uint32_t)__builtin_amdgcn_ds_bpermute(perm_k, (int)raw.y);
            v.z = (uint32_t)__builtin_amdgcn_ds_bpermute(perm_k, (int)raw.z);
            v.w = (uint32_t)__builtin_amdgcn_ds_bpermute(perm_k, (int)raw.w);
        }
        return v;
    };

    // fold e^{-i w base} into the lane's table registers
    auto move_base = [&](int new_base) {
        base = new_base;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int f = 4 * b + k;
            const float x = (float)__builtin_amdgcn_fract((double)base * lds_rev[f]);
            const float bs = __builtin_amdgcn_sinf(x), bc = __builtin_amdgcn_cosf(x);
#pragma unroll
            for (int q = 0; q < NG; ++q) {
                const int g = 4 * q + i;
                const float qr = g < G ? lds_tab[(f * 3 + 0) * G + g] : 0.f;
                const float qi = g < G ? lds_tab[(f * 3 + 1) * G + g] : 0.f;
                tb[q].rr[k] = qr * bc + qi * bs;
                tb[q].ri[k] = qi * bc - qr * bs;
            }
        }
    };

    // one step with the key's phasors read from the table (0 <= r < R)
    auto step_table = [&](const uint4 &kd, int r, float(&out)[NG]) {
        const float4 e0 = *reinterpret_cast<const float4 *>(ph0 + r * 16);
        const float4 e1 = *reinterpret_cast<const float4 *>(ph0 + kPhasorHalfStride + r * 16);
        const float cs[4] = {e0.x, e0.z, e1.x, e1.z}, sn[4] = {e0.y, e0.w, e1.y, e1.w};
        score_step<NG, true, HALF>(kd, cs, sn, tb, out);
    };

    // one step for any four positions: move the base if that brings them into the table, else
    // evaluate the phasors directly (phase in double, relative to the base in force)
    auto step_general = [&](const uint4 &kd, int p, float(&out)[NG]) {
        int r = p - base;
        if (__builtin_amdgcn_ballot_w64((unsigned)r >= (unsigned)kPhasorRange) != 0ull) {
            const int p0 = __builtin_amdgcn_readlane(p, 0), p1 = __builtin_amdgcn_readlane(p, 1);
            const int p2 = __builtin_amdgcn_readlane(p, 2), p3 = __builtin_amdgcn_readlane(p, 3);
            const int lo = min(min(p0, p1), min(p2, p3)), hi = max(max(p0, p1), max(p2, p3));
            if ((int64_t)hi - (int64_t)lo < kPhasorRange) {
                move_base(lo);
                r = p - base;
            } else {
                const double pd = (double)((int64_t)p - (int64_t)base);
                float cs[4], sn[4];
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const float x = (float)__builtin_amdgcn_fract(pd * lds_rev[4 * b + k]);
                    sn[k] = __builtin_amdgcn_sinf(x);
                    cs[k] = __builtin_amdgcn_cosf(x);
                }
                score_step<NG, true, HALF>(kd, cs, sn, tb, out);
                return;
            }
        }
        step_table(kd, r, out);
    };

    auto process_group = [&](int n, const uint4(&kraw)[4], int praw, auto full_tag) {
        constexpr bool kFull = decltype(full_tag)::value;   // all 16 keys of the group exist
        uint4 kd[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) kd[t] = to_consumer(kraw[t]);
        float out[4][NG];   // per step, block sums not yet finished (reduce_blocks)
        if constexpr (ROTATED) {   // post-RoPE keys: straight into the contraction
            const float one[4] = {1.f, 1.f, 1.f, 1.f}, zero[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int t = 0; t < 4; ++t) score_step<NG, false, HALF>(kd[t], one, zero, tb, out[t]);
        } else {
            // common case: all 16 positions of the group fall in the table around the current base.  The test
            // and the table index are formed on the positions in load order (every lane holds one of the 16),
            // before they go to the consumer lanes.
            int rraw = praw - base;
            bool fast = __builtin_amdgcn_ballot_w64((unsigned)rraw >= (unsigned)kPhasorRange) == 0ull;
            if (!fast) {
                // span of the 16 positions: lanes 0..15 hold one each (one DPP row)
                int lo = praw, hi = praw;
#pragma unroll
                for (int o = 8; o >= 1; o >>= 1) {
                    lo = min(lo, __shfl_xor(lo, o, 16));
                    hi = max(hi, __shfl_xor(hi, o, 16));
                }
                lo = __builtin_amdgcn_readfirstlane(lo);
                hi = __builtin_amdgcn_readfirstlane(hi);
                if ((int64_t)hi - (int64_t)lo < kPhasorRange) {
                    move_base(lo);
                    rraw = praw - base;
                    fast = true;
                }
            }
            if (fast) {
#pragma unroll
                for (int t = 0; t < 4; ++t)
                    step_table(kd[t], __builtin_amdgcn_ds_bpermute(perm_p + 16 * t, rraw), out[t]);
            } else {
#pragma unroll
                for (int t = 0; t < 4; ++t)
                    step_general(kd[t], __builtin_amdgcn_ds_bpermute(perm_p + 16 * t, praw), out[t]);
            }
        }
        float kept[NG];   // the lane's own result: step sub
#pragma unroll
        for (int q = 0; q < NG; ++q) kept[q] = merge_steps(out[0][q], out[1][q], out[2][q], out[3][q]);
        // lane (row, sub, j) now holds key n + 4*sub + row for head j (+4q): 16 keys x 4 heads per wave
        const int key = n + 4 * sub + row;
        char *rw_group = reinterpret_cast<char *>(rw + n);   // uniform; the lane adds its constant 32-bit offset
        if (kFull || key < w1) {
#pragma unroll
            for (int q = 0; q < NG; ++q) {
                const int g = 4 * q + i;
                if (g < G) {
                    asm volatile("" : "+v"(st_off[q]));   // keeps (scalar base + 32-bit vector offset), as for the loads
                    *reinterpret_cast<float *>(rw_group + st_off[q]) = kept[q];
                    const double v = (double)kept[q];
                    s1[q] += v;
                    s2[q] += v * v;
                }
            }
        }
    };

    // Two register buffers: the loads of the next group are in flight while one is scored.  Inside the
    // main loop every load is unconditional (a group index past the last full group is clamped to it
    // and its data ignored), so the loop is straight-line code and the compiler can count
    // outstanding loads exactly.
    const int n_full = (w1 - w0) >> 4, rem = (w1 - w0) & 15;
    if (w0 < w1) {
        uint4 kdA[4], kdB[4];
        int ppA, ppB;
        int g = 0;
        if (n_full > 0) {
            const int last = n_full - 1;
            load_full(w0, kdA, ppA);
            for (; g + 2 <= n_full; g += 2) {
                load_full(w0 + 16 * (g + 1), kdB, ppB);
                process_group(w0 + 16 * g, kdA, ppA, std::true_type{});
                load_full(w0 + 16 * min(g + 2, last), kdA, ppA);
                process_group(w0 + 16 * (g + 1), kdB, ppB, std::true_type{});
            }
            if (g < n_full) process_group(w0 + 16 * g, kdA, ppA, std::true_type{});
        }
        if (rem) {
            load_tail(w0 + 16 * n_full, rem, kdB, ppB);
            process_group(w0 + 16 * n_full, kdB, ppB, std::false_type{});
        }
    }

    // per-head sums over the wave's keys: lanes with equal lane % 4 hold the same head
#pragma unroll
    for (int q = 0; q < NG; ++q) {
#pragma unroll
        for (int o = 4; o < 64; o <<= 1) {
            s1[q] += __shfl_xor(s1[q], o, 64);
            s2[q] += __shfl_xor(s2[q], o, 64);
        }
        if (lane < 4) {
            red[wave][(4 * q + lane) * 2 + 0] = s1[q];
            red[wave][(4 * q + lane) * 2 + 1] = s2[q];
        }
    }
    __syncthreads();
    if (tid < 2 * G) {
        const int g = tid % G, which = tid / G;
        double v = 0.0;
        for (int w = 0; w < kFastWaves; ++w) v += red[w][g * 2 + which];
        a.partials[(inst * a.n_tiles + chunk) * (2 * G) + tid] = v;
    }
  }   // next item
}

template <int G>
tri_status launch_fast_g(const ScoreArgs &sa, bool half_split, hipStream_t st)
{
    const bool paged = sa.c.block_shift >= 0;
    auto pick = [&](auto half) {
        constexpr bool H = decltype(half)::value;
        return sa.c.k_rotated ? (paged ? score_mfma_kernel<G, true, true, H> : score_mfma_kernel<G, false, true, H>)
                              : (paged ? score_mfma_kernel<G, true, false, H> : score_mfma_kernel<G, false, false, H>);
    };
    auto kern = half_split ? pick(std::true_type{}) : pick(std::false_type{});
    const int lds = sa.c.k_rotated ? 0 : kPhasorBytes;   // no phasor table for post-RoPE keys
    if (lds && hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds) != hipSuccess)
        return hip_status("hipFuncSetAttribute(score_mfma_kernel)");
    // as many workgroups as are resident at once (they stay until the work list is empty), no more than items can exist.
    // The answer is kept per kernel and per GPU; threads that ask at the same time compute the same number.
    static std::atomic<int> resident[2][2][2][kMaxDevices];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        (void)hipGetLastError();
        set_error("score: no current device below %d", kMaxDevices);
        return TRI_ERR_HIP;
    }
    std::atomic<int> &cached = resident[sa.c.k_rotated ? 1 : 0][paged ? 1 : 0][half_split ? 1 : 0][dev];
    int slots = cached.load(std::memory_order_relaxed);
    if (slots == 0) {
        int n_cu = 0, per_cu = 0;
        if (hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
            hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, (const void *)kern, fast_threads(G), lds) != hipSuccess ||
            n_cu <= 0 || per_cu <= 0) {
            (void)hipGetLastError();
            set_error("score: occupancy query failed");
            return TRI_ERR_HIP;
        }
        slots = n_cu * per_cu;
        cached.store(slots, std::memory_order_relaxed);
    }
    const int64_t max_items = (int64_t)sa.n_tiles * sa.c.n_seqs * sa.c.n_kv_heads * sa.n_layers;
    if (max_items > (int64_t)0x7fff0000) {   // the item counter is a 32-bit integer
        set_error("score: %lld chunks of %d keys exceed the 32-bit work counter", (long long)max_items, kFastChunk);
        return TRI_ERR_UNSUPPORTED;
    }
    const int grid = (int)std::min<int64_t>((int64_t)slots, max_items);
    ScoreArgs sb = sa;
    sb.first_mult = 1;
    for (int p : {197, 199, 211, 223})   // a prime that does not divide the grid size
        if (grid % p != 0) {
            sb.first_mult = p;
            break;
        }
    hipLaunchKernelGGL(kern, dim3(grid), dim3(fast_threads(G)), lds, st, sb);
    return hip_status("score_mfma_kernel");
}

}  // namespace

tri_status launch_phasor_table(double theta, uint4 *phasors, hipStream_t st)
{
    hipLaunchKernelGGL(phasor_table_kernel, dim3(2 * 16 * kPhasorRange / 256), dim3(256), 0, st, theta,
                       reinterpret_cast<float4 *>(phasors));
    return hip_status("phasor_table_kernel");
}

tri_status launch_score_fast(int G, const ScoreArgs &sa, bool half_split, hipStream_t st)
{
    switch (G) {
        case 1: return launch_fast_g<1>(sa, half_split, st);
        case 2: return launch_fast_g<2>(sa, half_split, st);
        case 3: return launch_fast_g<3>(sa, half_split, st);
        case 4: return launch_fast_g<4>(sa, half_split, st);
        case 5: return launch_fast_g<5>(sa, half_split, st);
        case 6: return launch_fast_g<6>(sa, half_split, st);
        case 7: return launch_fast_g<7>(sa, half_split, st);
        case 8: return launch_fast_g<8>(sa, half_split, st);
    }
    set_error("group size %d not built (1 to 8)", G);
    return TRI_ERR_UNSUPPORTED;
}

}  // namespace tri
