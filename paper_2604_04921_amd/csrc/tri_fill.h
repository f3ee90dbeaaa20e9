// In-place eviction that moves as few slots as possible (Section 4.3 fixes no slot order), as a routine of one
// 256-thread workgroup: the kernel of tri_compact_fill calls it, and so does the selection kernel of short sequences at
// the end of the fused step, on the kept slots it has just written.
#pragma once
#include "tri_internal.h"

namespace tri {

constexpr int kFillThreads = 256;
constexpr int kFillMaxWords = 2048;   // budget <= 65536

struct FillArgs {
    CacheView c;               // the cache, evicted in place
    int32_t *new_seq_len;      // [S] or NULL
    int32_t budget;            // row length of kept_idx and half the length of `moves`
    int32_t elem_bytes, row16; // bytes per element, 16-byte chunks per K (or V) row
};

// Kept keys already in slots [0, cnt) stay; the i-th free slot below cnt (ascending) receives the i-th kept key stored
// at or beyond cnt (ascending).  Sources (>= cnt) and destinations (< cnt) are disjoint, so the moves need no ordering.
// idx: the head-instance's kept slots, ascending (read into [0, max_seq_len - 1]: device memory the host cannot check).
// LDS handed in: moves [2][budget] (destination slots, source slots), kept_bits [ceil(cnt / 32)] at least,
// wave_tot [4], n_tail [1].  Every thread of the workgroup must call it; it starts with a barrier of its own only
// after its first LDS writes, so the caller synchronises before if the LDS was in other use.
__device__ __forceinline__ void fill_block(const FillArgs &a, int inst, int cnt, const int32_t *idx, int32_t *moves,
                                           uint32_t *kept_bits, uint32_t *wave_tot, int32_t *n_tail)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int ls = inst / a.c.n_kv_heads, h = inst - ls * a.c.n_kv_heads;
    const int l = ls / a.c.n_seqs, s = ls - l * a.c.n_seqs;
    if (a.new_seq_len && l == 0 && h == 0 && tid == 0) a.new_seq_len[s] = cnt;
    auto slot = [&](int j) { return min(max(idx[j], 0), a.c.max_seq_len - 1); };
    const int n_words = (cnt + 31) >> 5;
    for (int w = tid; w < n_words; w += kFillThreads) kept_bits[w] = 0u;
    if (tid == 0) *n_tail = 0;
    __syncthreads();
    int my_tail = 0;
    for (int j = tid; j < cnt; j += kFillThreads) {
        const int n = slot(j);
        if (n < cnt) atomicOr(&kept_bits[n >> 5], 1u << (n & 31));
        else ++my_tail;
    }
    if (my_tail) atomicAdd(n_tail, my_tail);
    __syncthreads();
    const int tail = *n_tail;
    const int first_tail = cnt - tail;   // idx is ascending: its last `tail` entries lie at or beyond cnt
    // free slots below cnt, in ascending order, paired with the tail survivors
    int done = 0;
    for (int w0 = 0; w0 < n_words; w0 += kFillThreads) {
        const int w = w0 + tid;
        uint32_t free_bits = 0u;
        if (w < n_words) {
            free_bits = ~kept_bits[w];
            if (w == n_words - 1 && (cnt & 31)) free_bits &= (1u << (cnt & 31)) - 1u;
        }
        const uint32_t c = (uint32_t)__popc(free_bits);
        uint32_t cum = c;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const uint32_t t = __shfl_up(cum, o, 64);
            if (lane >= o) cum += t;
        }
        if (lane == 63) wave_tot[wave] = cum;
        __syncthreads();
        uint32_t before = cum - c, total = 0u;
        for (int k = 0; k < kFillThreads / 64; ++k) {
            if (k < wave) before += wave_tot[k];
            total += wave_tot[k];
        }
        int o = done + (int)before;
        while (free_bits) {
            const int bit = __ffs(free_bits) - 1;
            free_bits &= free_bits - 1u;
            if (o < tail) {   // always true for an ascending duplicate-free kept_idx; guards the reads otherwise
                moves[o] = (w << 5) + bit;
                moves[a.budget + o] = slot(first_tail + o);
            }
            ++o;
        }
        done = min(done + (int)total, tail);
        __syncthreads();
    }
    // done == tail moves; 16 bytes of K and of V per thread and move
    const int rows_per_pass = kFillThreads / a.row16;
    const int r = tid / a.row16, part = tid % a.row16;
    char *kb = (char *)a.c.k, *vb = (char *)a.c.v;
    int32_t *pb = const_cast<int32_t *>(a.c.pos);
    for (int m0 = 0; m0 < done; m0 += rows_per_pass) {
        const int m = m0 + r;
        if (m >= done) continue;
        const int dj = moves[m], sn = moves[a.budget + m];
        const int64_t so = kv_offset(a.c, l, s, h, sn) * a.elem_bytes + part * 16;
        const int64_t d_o = kv_offset(a.c, l, s, h, dj) * a.elem_bytes + part * 16;
        const uint4 kv = load_stream16(kb + so);
        const uint4 vv = load_stream16(vb + so);
        store_stream16(kb + d_o, kv);
        store_stream16(vb + d_o, vv);
        if (part == 0) pb[pos_offset(a.c, l, s, h, dj)] = pb[pos_offset(a.c, l, s, h, sn)];
    }
}

}  // namespace tri
