// Score kernel for bf16 keys with interleaved pairs, one key per lane (Sections 4.1-4.2).
//
// A wave takes 64 consecutive slots of a head-instance -- a tile -- and every lane scores one of them against all
// query heads of the group.  The contraction over (band, component) x query head runs on v_mfma_f32_4x4x1_16b_f32:
// block b of the instruction holds lanes 4b..4b+3, its rows are those four lanes' keys (operand A: the lane's own
// rotated component or modulus of the band in turn), its columns four query heads (operand B: lane 4b+j supplies the
// folded table entry of head j, the same in every block).  The accumulator of lane (b, j) therefore ends up with the
// scores of keys 4b..4b+3 for head j: no cross-lane reduction, and one 16-byte store per lane writes them.
//
// What it takes to get there:
//   * K rows reach their lanes through LDS: the wave loads half rows (128 bytes per key, whole cache lines) with
//     coalesced 16-byte loads, writes them to its own staging area and each lane reads its key back 16 bytes (four
//     bands) at a time.  The area is XOR-swizzled so that both the writes (16 lanes = 2 keys x 8 pieces) and the reads
//     (16 lanes = 16 keys, one piece) touch every bank once.
//   * Rotation of the key (Appendix B.2): k e^{i w p} = (k e^{i w r}) e^{i w base} with base a position in the middle of
//     the tile's positions and |r| < 64.  e^{i w |r|} comes from a table in LDS (one 16-byte read per two bands; a
//     negative r flips the sign of the sine), e^{-i w base} is folded into the wave's copy of the head-instance's table,
//     which it rewrites for every tile (lane = band: one sine / cosine pair and 2 G complex products per lane).  A tile
//     whose positions span 127 or more takes the direct path (phase in double, v_sin_f32 / v_cos_f32 per lane and band).
//   * Operand B is read from that copy in LDS, four bands per read.
// The vector instructions of four bands are issued first and their twelve (24) matrix instructions in one run after
// them: a wave that alternates between the two kinds loses about 3.5 clocks per matrix instruction.
#include <algorithm>
#include <atomic>
#include <type_traits>

#include "tri_score_common.h"

namespace tri {

namespace {

constexpr int kMaxDevices = 64;

typedef float float4v __attribute__((ext_vector_type(4)));

constexpr int kTileKeys = 64;
constexpr int kStageBytes = kTileKeys * 128;                    // one half row per key, swizzled, no padding
constexpr int kTabRow = kBands + 4;                             // floats per (component, head) row: 16 bytes of skew

// (lane_waves(G): LDS decides -- 33 KB of phasors + a stage and a table per wave)
constexpr int lane_heads(int G) { return 4 * ((G + 3) / 4); }   // table rows: query heads rounded up to whole quads
constexpr int lane_wave_bytes(int G) { return kStageBytes + 2 * lane_heads(G) * kTabRow * 4; }   // stage + (re, im) rows
constexpr int lane_lds_bytes(int G, bool rotated)
{
    return (rotated ? 0 : kLanePhasorBytes) + lane_heads(G) * kTabRow * 4 + lane_waves(G) * lane_wave_bytes(G);
}

// Byte offset of (key k, 16-byte piece p of its half row) in a wave's staging area.  Rows k and k ^ 1 swap places when
// bit 3 of k is set and the piece index is XORed with k & 7: 16 lanes that hold 2 keys x 8 pieces (the writes) or 16
// keys x 1 piece (the reads) then fall into 16 different groups of four banks.
__device__ __forceinline__ int stage_offset(int k, int p) { return ((k ^ ((k >> 3) & 1)) << 7) + ((p ^ (k & 7)) << 4); }

// ROTATED: the keys are stored post-RoPE (no rotation, no positions).  PAGED: block_size >= 16.
template <int G, bool PAGED, bool ROTATED>
__global__ __launch_bounds__(lane_waves(G) * 64) void score_lane_kernel(ScoreArgs a)
{
    constexpr int NG = (G + 3) / 4, HR = lane_heads(G), W = lane_waves(G), kThreads = W * 64;
    constexpr int kTabBytes = HR * kTabRow * 4;          // one component's rows
    extern __shared__ __align__(16) char lds[];
    __shared__ double red[W][2 * 4 * NG];
    __shared__ double lds_rev[kBands];                    // omega_f / 2pi
    __shared__ float q_tab[2][G][kBands];                 // E[q] e^{..} of the head-instance, (re, im) x head x band
    __shared__ int lds_item;

    const CacheView &c = a.c;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int j = lane & 3, b = lane >> 2;                // column (query head within a quad) and block of the lane

    char *const ph_base = lds;                                                  // phasor table (absent when ROTATED)
    char *const cn_base = lds + (ROTATED ? 0 : kLanePhasorBytes);               // norm-term rows, shared by the waves
    char *const my_base = cn_base + kTabBytes + wave * lane_wave_bytes(G);
    char *const stage = my_base;                                                // this wave's half rows
    char *const tab_re = my_base + kStageBytes, *const tab_im = tab_re + kTabBytes;

    if constexpr (!ROTATED)
        for (int k = tid; k < kLanePhasorBytes / 16; k += kThreads)
            reinterpret_cast<uint4 *>(ph_base)[k] = a.phasors[k];
    if (tid < kBands) lds_rev[tid] = a.band_rev[tid];
    // rows of heads that do not exist (G not a multiple of four) stay zero for the whole launch
    for (int k = lane; k < 2 * HR * kTabRow; k += 64) reinterpret_cast<float *>(tab_re)[k] = 0.f;
    for (int k = tid; k < HR * kTabRow; k += kThreads) reinterpret_cast<float *>(cn_base)[k] = 0.f;

    const int per_lh = __builtin_amdgcn_readfirstlane(a.work[1]);
    const int n_items = per_lh * a.n_layers * c.n_kv_heads;
    int next_item = (int)(((uint32_t)blockIdx.x * (uint32_t)a.first_mult) % gridDim.x);

    const uint32_t slot_bytes = (uint32_t)c.stride_slot * 2u;
    // loads: instruction t of a half row brings keys 8t .. 8t+7, eight lanes (128 contiguous bytes) per key
    const int ld_key = lane >> 3, ld_piece = lane & 7;
    const int bmask = PAGED ? (1 << c.block_shift) - 1 : 0;
    uint32_t ld_off = (uint32_t)ld_key * slot_bytes + (uint32_t)ld_piece * 16u;   // the lane's part of a load address
    // where the lane writes its loaded pieces and reads its own key's pieces in the staging area
    // (load t is written at 1024 t plus one of two offsets, by the parity of t: see stage_offset)
    const int st_wr0 = stage_offset(ld_key, ld_piece), st_wr1 = stage_offset(8 + ld_key, ld_piece) - 1024;
    const int st_rd0 = stage_offset(lane, 0);   // piece p of the lane's key lies at st_rd0 ^ (p << 4)
    const int tab_lane = j * kTabRow * 4;   // byte offset of the lane's head row inside a quad of table rows

    for (;;) {
        if (tid == 0) lds_item = next_item;
        __syncthreads();
        const int item = __builtin_amdgcn_readfirstlane(lds_item);
        if (item >= n_items) break;
        if (tid == 0) next_item = (int)gridDim.x + atomicAdd(&a.work[0], 1);
        const int lh = item / per_lh, wi = item - lh * per_lh;
        const int l = lh / c.n_kv_heads, h = lh - l * c.n_kv_heads;
        const int s = __builtin_amdgcn_readfirstlane(a.work[kWorkHeader + 2 * wi]);
        const int chunk = __builtin_amdgcn_readfirstlane(a.work[kWorkHeader + 2 * wi + 1]);
        const int N = clamp_len(c.seq_len[s], c.max_seq_len);
        const int64_t inst = ((int64_t)l * c.n_seqs + s) * c.n_kv_heads + h;
        const float *tbl = a.table + inst * (kBands * 3 * G);   // [F][3][G]

        const int c0 = chunk * a.chunk_keys, c_len = min(N - c0, a.chunk_keys);
        const int n_tiles = (c_len + kTileKeys - 1) / kTileKeys;
        const int Hq = c.n_kv_heads * G;
        float *rw = a.raw + (((int64_t)l * c.n_seqs + s) * Hq + (int64_t)h * G) * c.max_seq_len;
        const bool vec_store = (c.max_seq_len & 3) == 0 && ((uintptr_t)a.raw & 15) == 0;

        const char *krow = (const char *)c.k + ((int64_t)l * c.stride_layer + (int64_t)h * c.stride_head) * 2 +
                           (PAGED ? 0 : (int64_t)s * c.stride_sb * 2);
        const int32_t *prow = c.pos + (int64_t)l * c.pos_stride_layer + (int64_t)h * c.pos_stride_head +
                              (PAGED ? 0 : (int64_t)s * c.pos_stride_sb);
        const int32_t *bt = PAGED ? c.block_table + (int64_t)s * c.max_blocks : nullptr;

        // half row `half` of the tile at slot n0 (cnt keys exist): eight 16-byte loads per lane.  For a whole tile every
        // address is a wave-uniform pointer (a group of eight keys never straddles a block) plus the lane's constant
        // offset; in the last, partial tile a key past the end repeats the last one.
        // Paged caches: lane j of `btv` holds the physical block of keys n0 + 16 j .. + 15 (load_blocks; a block holds
        // 16 slots or more), asked for a tile ahead like the positions, so that no load here waits for a block-table
        // entry.
        auto load_half = [&](int n0, int cnt, int half, uint4(&kd)[8], int btv) {
            if (cnt == kTileKeys) {
#pragma unroll
                for (int t = 0; t < 8; t += 2) {
                    const int n = n0 + 8 * t;
                    const char *p;
                    if constexpr (PAGED) {
                        const int blk = __builtin_amdgcn_readlane(btv, t / 2);
                        p = krow + (int64_t)blk * c.stride_sb * 2 + (int64_t)(n & bmask) * slot_bytes;
                    } else {
                        p = krow + (int64_t)n * slot_bytes;
                    }
                    asm volatile("" : "+v"(ld_off));   // keeps (scalar base + 32-bit lane offset) addressing
                    kd[t] = load_stream16(p + half * 128 + ld_off);
                    asm volatile("" : "+v"(ld_off));
                    kd[t + 1] = load_stream16(p + 8 * (int64_t)slot_bytes + half * 128 + ld_off);
                }
            } else {
#pragma unroll
                for (int t = 0; t < 8; ++t) {
                    const int n = n0 + min(8 * t + ld_key, cnt - 1);
                    const char *p;
                    if constexpr (PAGED) {
                        const int blk = bt[n >> c.block_shift];
                        p = krow + (int64_t)blk * c.stride_sb * 2 + (int64_t)(n & bmask) * slot_bytes;
                    } else {
                        p = krow + (int64_t)n * slot_bytes;
                    }
                    kd[t] = load_stream16(p + half * 128 + ld_piece * 16);
                }
            }
        };
        auto load_blocks = [&](int n0, int cnt) -> int {
            if constexpr (!PAGED) return 0;
            return bt[(n0 + min(16 * (lane & 3), cnt - 1)) >> c.block_shift];
        };
        auto load_pos = [&](int n0, int cnt) -> int {
            if constexpr (ROTATED) return 0;
            const int n = n0 + min(lane, cnt - 1);
            if constexpr (PAGED) {
                const int blk = bt[n >> c.block_shift];
                return prow[(int64_t)blk * c.pos_stride_sb + (n & bmask)];
            } else {
                return prow[n];
            }
        };
        auto stage_half = [&](const uint4(&kd)[8]) {
#pragma unroll
            for (int t = 0; t < 8; ++t) *reinterpret_cast<uint4 *>(stage + ((t & 1) ? st_wr1 : st_wr0) + 1024 * t) = kd[t];
        };

        double s1[NG], s2[NG];
#pragma unroll
        for (int q = 0; q < NG; ++q) s1[q] = s2[q] = 0.0;

        int t_idx = wave;
        // Item i takes its tiles in an order rotated by 5 i: workgroups that run side by side work on neighbouring
        // chunks and would otherwise read the same offset of their chunk (addresses one chunk apart) at the same
        // time, all the way through.  Measured on 36 x 16 x 8 head-instances of 32768 keys in one process: 8.13 ->
        // 7.97 ms and 7.74 -> 7.53 ms (steps of 2 to 6 tiles alike, 1, 11 to 37 less, 7 and 9 little or nothing); with more
        // than four query heads the kernel is bound by its arithmetic and the rotation costs 0.7 %, so it stays off.
        const int rot = G <= 4 && n_tiles > 0 ? (int)(((unsigned)item * 5u) % (unsigned)n_tiles) : 0;
        auto tile_at = [&](int t) { const int u = t + rot; return u >= n_tiles ? u - n_tiles : u; };
        uint4 kd[8];
        int pos_next = 0, bt_cur = 0, bt_next = 0;
        if (t_idx < n_tiles) {
            const int n0 = c0 + tile_at(t_idx) * kTileKeys;
            bt_cur = load_blocks(n0, min(kTileKeys, c0 + c_len - n0));
            load_half(n0, min(kTileKeys, c0 + c_len - n0), 0, kd, bt_cur);
            pos_next = load_pos(n0, min(kTileKeys, c0 + c_len - n0));
        }
        // (the first tile's loads are on their way)  Norm-term rows of this head-instance, shared by the waves, and the
        // folded table per band
        for (int k = tid; k < kBands * G; k += kThreads) {
            const int f = k / G, g = k - f * G;
            reinterpret_cast<float *>(cn_base)[g * kTabRow + f] = tbl[(f * 3 + 2) * G + g];
        }
        for (int k = tid; k < kBands * G; k += kThreads) {
            const int f = k / G, g = k - f * G;
            const float re = tbl[(f * 3 + 0) * G + g], im = tbl[(f * 3 + 1) * G + g];
            q_tab[0][g][f] = re;
            q_tab[1][g][f] = im;
            if constexpr (ROTATED) {   // no base to fold in: every wave's copy is written once per item
                for (int w = 0; w < W; ++w) {
                    char *const wb = cn_base + kTabBytes + w * lane_wave_bytes(G) + kStageBytes;
                    reinterpret_cast<float *>(wb)[g * kTabRow + f] = re;
                    reinterpret_cast<float *>(wb + kTabBytes)[g * kTabRow + f] = im;
                }
            }
        }
        __syncthreads();

        for (; t_idx < n_tiles; t_idx += W) {
            const int n0 = c0 + tile_at(t_idx) * kTileKeys;
            const int cnt = min(kTileKeys, c0 + c_len - n0);
            const int p_key = pos_next;
            if (t_idx + W < n_tiles) {   // the next tile's blocks: needed when its first loads go out, half a tile from now
                const int m0 = c0 + tile_at(t_idx + W) * kTileKeys;
                bt_next = load_blocks(m0, min(kTileKeys, c0 + c_len - m0));
            }

            // ---- the tile's base and the lane's relative position
            int r = 0;
            bool in_table = true, mirrored = false;   // wave-uniform
            float sgn = 1.f;
            double rel_d = 0.0;
            if constexpr (!ROTATED) {
                int lo = p_key, hi = p_key;
#pragma unroll
                for (int o = 32; o >= 1; o >>= 1) {
                    lo = min(lo, __shfl_xor(lo, o, 64));
                    hi = max(hi, __shfl_xor(hi, o, 64));
                }
                lo = __builtin_amdgcn_readfirstlane(lo);
                hi = __builtin_amdgcn_readfirstlane(hi);
                const int64_t span = (int64_t)hi - (int64_t)lo;
                // positions within 64 of the lowest: base = the lowest, r >= 0.  Else base = the middle and the table
                // serves |r| (a negative r flips the sine), as long as the span stays below 127.
                mirrored = span >= kLaneRange;
                in_table = span < 2 * kLaneRange - 1;
                const int base = mirrored ? (int)((int64_t)lo + (span >> 1)) : lo;
                const int64_t rel = (int64_t)p_key - (int64_t)base;
                rel_d = (double)rel;
                sgn = rel < 0 ? -1.f : 1.f;
                r = in_table ? (int)(rel < 0 ? -rel : rel) : 0;   // (0 keeps the unused table address in range)
                // fold e^{-i w base} into the wave's table: lane = band
                const float x = (float)__builtin_amdgcn_fract((double)base * lds_rev[lane]);
                const float bs = __builtin_amdgcn_sinf(x), bc = __builtin_amdgcn_cosf(x);
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    const float qr = q_tab[0][g][lane], qi = q_tab[1][g][lane];
                    reinterpret_cast<float *>(tab_re)[g * kTabRow + lane] = qr * bc + qi * bs;
                    reinterpret_cast<float *>(tab_im)[g * kTabRow + lane] = qi * bc - qr * bs;
                }
            }
            const char *ph_lane = ph_base + r * 16;

            float4v acc[NG], acc2[NG];   // two chains, so that consecutive matrix instructions do not depend on each other
#pragma unroll
            for (int q = 0; q < NG; ++q) acc[q] = acc2[q] = float4v{0.f, 0.f, 0.f, 0.f};

            // Everything a piece (four bands of the lane's key) needs from LDS: the key's 16 bytes, the phasors of its
            // four bands at the lane's relative position, the lane's table entries.  Pieces are fetched one ahead of
            // the piece being scored, in straight-line code, so that the LDS latency hides behind the arithmetic.
            struct Piece {
                uint4 kq;
                float4 e0, e1;
                float4 br[NG], bi[NG], bc[NG];
            };
            auto fetch = [&](int half, int pc, auto table_tag) {
                constexpr bool TABLE = decltype(table_tag)::value;
                const int f0 = 32 * half + 4 * pc;   // first of the piece's four bands
                Piece o;
                o.kq = *reinterpret_cast<const uint4 *>(stage + (st_rd0 ^ (pc << 4)));
                if constexpr (TABLE) {
                    o.e0 = *reinterpret_cast<const float4 *>(ph_lane + (f0 / 2) * kLanePairStride);
                    o.e1 = *reinterpret_cast<const float4 *>(ph_lane + (f0 / 2 + 1) * kLanePairStride);
                }
#pragma unroll
                for (int q = 0; q < NG; ++q) {
                    const int off = tab_lane + (4 * q * kTabRow + f0) * 4;
                    o.br[q] = *reinterpret_cast<const float4 *>(tab_re + off);
                    o.bi[q] = *reinterpret_cast<const float4 *>(tab_im + off);
                    o.bc[q] = *reinterpret_cast<const float4 *>(cn_base + off);
                }
                return o;
            };
            // The vector instructions of the piece first, then its matrix instructions in one run.
            auto score_piece = [&](const Piece &pz, int half, int pc, auto table_tag, auto mirror_tag) {
                constexpr bool TABLE = decltype(table_tag)::value, MIRROR = decltype(mirror_tag)::value;
                const int f0 = 32 * half + 4 * pc;
                const uint32_t w[4] = {pz.kq.x, pz.kq.y, pz.kq.z, pz.kq.w};
                float cs[4] = {1.f, 1.f, 1.f, 1.f}, sn[4] = {0.f, 0.f, 0.f, 0.f};
                if constexpr (!ROTATED) {
                    if constexpr (TABLE) {
                        cs[0] = pz.e0.x, sn[0] = pz.e0.y, cs[1] = pz.e0.z, sn[1] = pz.e0.w;
                        cs[2] = pz.e1.x, sn[2] = pz.e1.y, cs[3] = pz.e1.z, sn[3] = pz.e1.w;
                        if constexpr (MIRROR) {
#pragma unroll
                            for (int k = 0; k < 4; ++k) sn[k] *= sgn;
                        }
                    } else {
#pragma unroll
                        for (int k = 0; k < 4; ++k) {
                            const float x = (float)__builtin_amdgcn_fract(rel_d * lds_rev[f0 + k]);
                            sn[k] = __builtin_amdgcn_sinf(x);
                            cs[k] = __builtin_amdgcn_cosf(x);
                        }
                    }
                }
                float kr[4], ki[4], m[4];
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const float re = bf16_lo(w[k]), im = bf16_hi(w[k]);
                    m[k] = __builtin_amdgcn_sqrtf(fmaf(re, re, im * im));
                    kr[k] = ROTATED ? re : re * cs[k] - im * sn[k];
                    ki[k] = ROTATED ? im : re * sn[k] + im * cs[k];
                }
                // memory instructions may move across; vector and matrix instructions stay apart
                __builtin_amdgcn_sched_barrier(0x4 | 0x20 | 0x100);
                // A wave in its vector part outranks the waves that are in their matrix runs (whose instructions each
                // hold the pipe for eight cycles and leave issue slots between them): measured in one process, 36 x 16 x 8
                // head-instances of 32768 keys 7.90 -> 7.60 ms, sparse positions 8.51 -> 8.01, G = 8 (64 x 8 of 131072 keys)
                // 4.63 -> 4.38; the other way round gains half of that, the levels themselves (1 / 0, 3 / 0, 2 / 1) nothing.
                __builtin_amdgcn_s_setprio(0);
#pragma unroll
                for (int k = 0; k < 4; ++k) {
#pragma unroll
                    for (int q = 0; q < NG; ++q) {
                        const float t_[4] = {pz.br[q].x, pz.br[q].y, pz.br[q].z, pz.br[q].w};
                        acc[q] = __builtin_amdgcn_mfma_f32_4x4x1f32(kr[k], t_[k], acc[q], 0, 0, 0);
                    }
#pragma unroll
                    for (int q = 0; q < NG; ++q) {
                        const float t_[4] = {pz.bi[q].x, pz.bi[q].y, pz.bi[q].z, pz.bi[q].w};
                        acc2[q] = __builtin_amdgcn_mfma_f32_4x4x1f32(ki[k], t_[k], acc2[q], 0, 0, 0);
                    }
#pragma unroll
                    for (int q = 0; q < NG; ++q) {
                        const float t_[4] = {pz.bc[q].x, pz.bc[q].y, pz.bc[q].z, pz.bc[q].w};
                        acc[q] = __builtin_amdgcn_mfma_f32_4x4x1f32(m[k], t_[k], acc[q], 0, 0, 0);
                    }
                }
                __builtin_amdgcn_s_setprio(2);
                __builtin_amdgcn_sched_barrier(0x4 | 0x20 | 0x100);
            };
            auto score_tile = [&](auto table_tag, auto mirror_tag) {
#pragma unroll
                for (int half = 0; half < 2; ++half) {
                    stage_half(kd);   // waits for the half row's loads, then 8 LDS writes
                    // the next loads go out while this half row is scored
                    if (half == 0) {
                        load_half(n0, cnt, 1, kd, bt_cur);
                    } else if (t_idx + W < n_tiles) {
                        const int m0 = c0 + tile_at(t_idx + W) * kTileKeys, mc = min(kTileKeys, c0 + c_len - m0);
                        load_half(m0, mc, 0, kd, bt_next);
                        pos_next = load_pos(m0, mc);
                    }
                    Piece cur = fetch(half, 0, table_tag);
#pragma unroll
                    for (int pc = 0; pc < 8; ++pc) {
                        Piece nxt = cur;
                        if (pc + 1 < 8) nxt = fetch(half, pc + 1, table_tag);
                        score_piece(cur, half, pc, table_tag, mirror_tag);
                        cur = nxt;
                    }
                }
            };
            if (ROTATED || !in_table) score_tile(std::false_type{}, std::false_type{});
            else if (mirrored) score_tile(std::true_type{}, std::true_type{});
            else score_tile(std::true_type{}, std::false_type{});

            bt_cur = bt_next;
#pragma unroll
            for (int q = 0; q < NG; ++q) acc[q] += acc2[q];
            // ---- lane (b, j) holds keys n0 + 4b .. + 3 for head 4q + j
#pragma unroll
            for (int q = 0; q < NG; ++q) {
                const int g = 4 * q + j;
                if (g < G) {
                    float *dst = rw + (int64_t)g * c.max_seq_len + n0 + 4 * b;
                    const int live = min(4, cnt - 4 * b);   // keys of this lane that exist
                    if (live == 4 && vec_store) {
                        // the selection reads the raw scores from HBM whatever the cache policy of this store; with
                        // the non-temporal hint the launch is 1 % faster (36 x 16 x 8 x 32768 keys: 7.71 -> 7.63 ms where
                        // the stores hurt most, equal where they hurt least; post-RoPE keys 6.80 -> 6.60).  Four-byte
                        // stores do not take the hint well: the sixteen-lane kernel is 3 - 4 % slower with it.
                        __builtin_nontemporal_store(acc[q], reinterpret_cast<float4v *>(dst));
                    } else {
#pragma unroll
                        for (int k = 0; k < 4; ++k)
                            if (k < live) dst[k] = acc[q][k];
                    }
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        const double v = k < live ? (double)acc[q][k] : 0.0;
                        s1[q] += v;
                        s2[q] += v * v;
                    }
                }
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
            for (int w_ = 0; w_ < W; ++w_) v += red[w_][g * 2 + which];
            a.partials[(inst * a.n_tiles + chunk) * (2 * G) + tid] = v;
        }
    }
}

template <int G>
tri_status launch_lane_g(const ScoreArgs &sa, hipStream_t st)
{
    const bool paged = sa.c.block_shift >= 0, rotated = sa.c.k_rotated != 0;
    auto kern = rotated ? (paged ? score_lane_kernel<G, true, true> : score_lane_kernel<G, false, true>)
                        : (paged ? score_lane_kernel<G, true, false> : score_lane_kernel<G, false, false>);
    const int lds = lane_lds_bytes(G, rotated);
    if (hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds) != hipSuccess)
        return hip_status("hipFuncSetAttribute(score_lane_kernel)");
    static std::atomic<int> resident[2][2][kMaxDevices];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        (void)hipGetLastError();
        set_error("score: no current device below %d", kMaxDevices);
        return TRI_ERR_HIP;
    }
    std::atomic<int> &cached = resident[rotated ? 1 : 0][paged ? 1 : 0][dev];
    int slots = cached.load(std::memory_order_relaxed);
    if (slots == 0) {
        int n_cu = 0, per_cu = 0;
        if (hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
            hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, (const void *)kern, lane_waves(G) * 64, lds) != hipSuccess ||
            n_cu <= 0 || per_cu <= 0) {
            (void)hipGetLastError();
            set_error("score: occupancy query failed");
            return TRI_ERR_HIP;
        }
        slots = n_cu * per_cu;
        cached.store(slots, std::memory_order_relaxed);
    }
    const int64_t max_items = (int64_t)sa.n_tiles * sa.c.n_seqs * sa.c.n_kv_heads * sa.n_layers;
    if (max_items > (int64_t)0x7fff0000) {
        set_error("score: %lld chunks of %d keys exceed the 32-bit work counter", (long long)max_items, sa.chunk_keys);
        return TRI_ERR_UNSUPPORTED;
    }
    const int grid = (int)std::min<int64_t>((int64_t)slots, max_items);
    ScoreArgs sb = sa;
    sb.first_mult = 1;
    for (int p : {197, 199, 211, 223})
        if (grid % p != 0) {
            sb.first_mult = p;
            break;
        }
    hipLaunchKernelGGL(kern, dim3(grid), dim3(lane_waves(G) * 64), lds, st, sb);
    return hip_status("score_lane_kernel");
}

}  // namespace

tri_status launch_score_lane(int G, const ScoreArgs &sa, hipStream_t st)
{
    switch (G) {
        case 1: return launch_lane_g<1>(sa, st);
        case 2: return launch_lane_g<2>(sa, st);
        case 3: return launch_lane_g<3>(sa, st);
        case 4: return launch_lane_g<4>(sa, st);
        case 5: return launch_lane_g<5>(sa, st);
        case 6: return launch_lane_g<6>(sa, st);
        case 7: return launch_lane_g<7>(sa, st);
        case 8: return launch_lane_g<8>(sa, st);
    }
    set_error("group size %d not built (1 to 8)", G);
    return TRI_ERR_UNSUPPORTED;
}

}  // namespace tri
