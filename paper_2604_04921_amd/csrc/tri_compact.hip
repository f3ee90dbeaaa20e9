// Eviction as compaction (Section 4.3, "evict the rest"): slot j <- slot kept_idx[j] for K, V
// and the key positions.  Pure byte moves, 16 bytes per lane.
#include "tri_internal.h"

namespace tri {

namespace {

struct CompactArgs {
    CacheView src, dst;
    const int32_t *kept_idx;  // [inst][B]
    const int32_t *kept_cnt;  // [inst]
    int32_t *new_seq_len;     // [S] or NULL
    int32_t budget;
    int32_t row16;            // 16-byte chunks per K (or V) row
    int32_t elem_bytes;
    int32_t row_blocks;       // gather kernel: workgroups per head-instance
};

__device__ __forceinline__ void decode_inst(const CacheView &c, int inst, int &l, int &s, int &h)
{
    h = inst % c.n_kv_heads;
    s = (inst / c.n_kv_heads) % c.n_seqs;
    l = inst / (c.n_kv_heads * c.n_seqs);
}

__device__ __forceinline__ void write_new_len(const CompactArgs &a, int l, int s, int h, int cnt)
{
    if (a.new_seq_len && l == 0 && h == 0 && threadIdx.x == 0) a.new_seq_len[s] = cnt;
}

// kept_cnt and kept_idx live in device memory where the host cannot check them: a count is read into
// [0, budget] and a slot index into [0, max_seq_len - 1], so that nothing outside the caches is touched.
__device__ __forceinline__ int read_cnt(const CompactArgs &a, int inst) { return min(max(a.kept_cnt[inst], 0), a.budget); }
__device__ __forceinline__ int read_slot(const CompactArgs &a, const int32_t *idx, int j)
{
    return min(max(idx[j], 0), a.src.max_seq_len - 1);
}

typedef unsigned int uint4v __attribute__((ext_vector_type(4)));

// the compacted cache is not read again by this step: non-temporal stores (the gather runs 10 % faster with them)
__device__ __forceinline__ void store_stream16(char *p, const uint4 &v)
{
    __builtin_nontemporal_store(uint4v{v.x, v.y, v.z, v.w}, reinterpret_cast<uint4v *>(p));
}

// 128 threads, one pass over 8 bf16 rows: small workgroups keep the most independent row fetches in flight
// (measured on 9.4 M scattered rows: 64 threads 1.64 ms, 128: 1.63, 256: 1.71, 512: 1.68, 1024: 1.72)
constexpr int kGatherThreads = 128;
constexpr int kRowsPerBlock = kGatherThreads / 16;


// the evicted cache is read once: non-temporal hint (a streaming read is 13 % faster with it on this GPU)
__device__ __forceinline__ uint4 load_stream16(const char *p)
{
    const uint4v t = __builtin_nontemporal_load(reinterpret_cast<const uint4v *>(p));
    return make_uint4(t.x, t.y, t.z, t.w);
}

// dst and src are different memory: a plain gather.  grid (instances * ceil(B / rows per block)), block 128: the
// row block is the fastest part of the index, so workgroups that run together write neighbouring rows.
// The workgroups are so small (one 16-byte piece of one row per thread) that their fixed cost matters -- the
// kernel is bound by instruction issue, much of it integer division and 64-bit index arithmetic: two
// divisions decode the instance, row16 is a power of two, and everything uniform stays in scalar registers.
__global__ __launch_bounds__(kGatherThreads) void gather_kernel(CompactArgs a)
{
    // x = instance * row_blocks + row block (x reaches 2^31 - 1; y and z stop at 65535)
    const int inst = blockIdx.x / a.row_blocks, rb = blockIdx.x - inst * a.row_blocks;
    const int ls = inst / a.src.n_kv_heads, h = inst - ls * a.src.n_kv_heads;
    const int l = ls / a.src.n_seqs, s = ls - l * a.src.n_seqs;
    const int cnt = read_cnt(a, inst);
    if (rb == 0) write_new_len(a, l, s, h, cnt);
    const int row_shift = a.row16 == 16 ? 4 : 5;   // bf16 rows are 16 pieces of 16 bytes, fp32 rows 32
    const int rows_per_pass = kGatherThreads >> row_shift;
    const int r = threadIdx.x >> row_shift, part = threadIdx.x & (a.row16 - 1);
    const int32_t *idx = a.kept_idx + (int64_t)inst * a.budget;
    const char *sk = (const char *)a.src.k, *sv = (const char *)a.src.v;
    char *dk = (char *)a.dst.k, *dv = (char *)a.dst.v;
    for (int j0 = rb * kRowsPerBlock; j0 < (rb + 1) * kRowsPerBlock; j0 += rows_per_pass) {
        const int j = j0 + r;
        if (j >= cnt) continue;
        const int n = read_slot(a, idx, j);
        const int64_t so = kv_offset(a.src, l, s, h, n) * a.elem_bytes + part * 16;
        const int64_t d_o = kv_offset(a.dst, l, s, h, j) * a.elem_bytes + part * 16;
        const uint4 kv = load_stream16(sk + so);
        const uint4 vv = load_stream16(sv + so);
        store_stream16(dk + d_o, kv);
        store_stream16(dv + d_o, vv);
        if (part == 0) const_cast<int32_t *>(a.dst.pos)[pos_offset(a.dst, l, s, h, j)] = a.src.pos[pos_offset(a.src, l, s, h, n)];
    }
}

constexpr int kInplaceThreads = 1024;
constexpr int kInplaceUnroll = 4;

// dst is src: an overlapping move with dst row j <= src row kept_idx[j].  One workgroup walks the
// survivors of a head-instance in ascending chunks: load a chunk into registers, wait for the data,
// barrier, store.  A chunk's destinations [j0, j0+R) are never the source of a later chunk (those
// sources are >= j0+R), and all of its own sources have been read before the barrier.
// grid (instances), block 1024.
__global__ __launch_bounds__(kInplaceThreads) void inplace_kernel(CompactArgs a)
{
    const int inst = blockIdx.x;
    int l, s, h;
    decode_inst(a.src, inst, l, s, h);
    const int cnt = read_cnt(a, inst);
    write_new_len(a, l, s, h, cnt);
    const int rows_per_pass = kInplaceThreads / a.row16;
    const int r = threadIdx.x / a.row16, part = threadIdx.x % a.row16;
    const int32_t *idx = a.kept_idx + (int64_t)inst * a.budget;
    char *kb = (char *)a.dst.k, *vb = (char *)a.dst.v;
    int32_t *pb = const_cast<int32_t *>(a.dst.pos);
    for (int j0 = 0; j0 < cnt; j0 += rows_per_pass * kInplaceUnroll) {
        uint4 kv[kInplaceUnroll], vv[kInplaceUnroll];
        int32_t pp[kInplaceUnroll];
        int src_n[kInplaceUnroll];
#pragma unroll
        for (int u = 0; u < kInplaceUnroll; ++u) {
            const int j = j0 + u * rows_per_pass + r;
            src_n[u] = j < cnt ? read_slot(a, idx, j) : -1;
        }
#pragma unroll
        for (int u = 0; u < kInplaceUnroll; ++u) {
            const int j = j0 + u * rows_per_pass + r;
            if (src_n[u] >= 0 && src_n[u] != j) {
                const int64_t so = kv_offset(a.src, l, s, h, src_n[u]) * a.elem_bytes + part * 16;
                kv[u] = load_stream16(kb + so);
                vv[u] = load_stream16(vb + so);
                if (part == 0) pp[u] = pb[pos_offset(a.src, l, s, h, src_n[u])];
            }
        }
        // the loads must have returned before any thread of the group may overwrite their sources
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
#pragma unroll
        for (int u = 0; u < kInplaceUnroll; ++u) {
            const int j = j0 + u * rows_per_pass + r;
            if (src_n[u] >= 0 && src_n[u] != j) {
                const int64_t d_o = kv_offset(a.dst, l, s, h, j) * a.elem_bytes + part * 16;
                store_stream16(kb + d_o, kv[u]);
                store_stream16(vb + d_o, vv[u]);
                if (part == 0) pb[pos_offset(a.dst, l, s, h, j)] = pp[u];
            }
        }
    }
}

constexpr int kFillThreads = 256;
constexpr int kFillMaxWords = 2048;   // budget <= 65536

// In-place eviction that moves as few slots as possible (Section 4.3 fixes no slot order): kept keys already in
// slots [0, cnt) stay; the i-th free slot below cnt (ascending) receives the i-th kept key stored at or beyond
// cnt (ascending).  Sources (>= cnt) and destinations (< cnt) are disjoint, so the moves need no ordering.
// grid (instances), block 256, dynamic LDS 8 * budget bytes (the move list).
__global__ __launch_bounds__(kFillThreads) void fill_kernel(CompactArgs a)
{
    extern __shared__ int32_t moves[];   // [2][budget]: destination slots, source slots
    __shared__ uint32_t kept_bits[kFillMaxWords];
    __shared__ uint32_t wave_tot[kFillThreads / 64];
    __shared__ int32_t n_tail;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int inst = blockIdx.x;
    int l, s, h;
    decode_inst(a.src, inst, l, s, h);
    const int cnt = read_cnt(a, inst);
    write_new_len(a, l, s, h, cnt);
    const int32_t *idx = a.kept_idx + (int64_t)inst * a.budget;
    const int n_words = (cnt + 31) >> 5;
    for (int w = tid; w < n_words; w += kFillThreads) kept_bits[w] = 0u;
    if (tid == 0) n_tail = 0;
    __syncthreads();
    int my_tail = 0;
    for (int j = tid; j < cnt; j += kFillThreads) {
        const int n = read_slot(a, idx, j);
        if (n < cnt) atomicOr(&kept_bits[n >> 5], 1u << (n & 31));
        else ++my_tail;
    }
    if (my_tail) atomicAdd(&n_tail, my_tail);
    __syncthreads();
    const int first_tail = cnt - n_tail;   // idx is ascending: its last n_tail entries lie at or beyond cnt
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
            if (o < n_tail) {   // always true for an ascending duplicate-free kept_idx; guards the reads otherwise
                moves[o] = (w << 5) + bit;
                moves[a.budget + o] = read_slot(a, idx, first_tail + o);
            }
            ++o;
        }
        done = min(done + (int)total, n_tail);
        __syncthreads();
    }
    // done == n_tail moves; 16 bytes of K and of V per thread and move
    const int rows_per_pass = kFillThreads / a.row16;
    const int r = tid / a.row16, part = tid % a.row16;
    char *kb = (char *)a.dst.k, *vb = (char *)a.dst.v;
    int32_t *pb = const_cast<int32_t *>(a.dst.pos);
    for (int m0 = 0; m0 < done; m0 += rows_per_pass) {
        const int m = m0 + r;
        if (m >= done) continue;
        const int dj = moves[m], sn = moves[a.budget + m];
        const int64_t so = kv_offset(a.src, l, s, h, sn) * a.elem_bytes + part * 16;
        const int64_t d_o = kv_offset(a.dst, l, s, h, dj) * a.elem_bytes + part * 16;
        const uint4 kv = load_stream16(kb + so);
        const uint4 vv = load_stream16(vb + so);
        store_stream16(kb + d_o, kv);
        store_stream16(vb + d_o, vv);
        if (part == 0) pb[pos_offset(a.dst, l, s, h, dj)] = pb[pos_offset(a.src, l, s, h, sn)];
    }
}

}  // namespace

tri_status check_fill_budget(int32_t budget)
{
    if (budget > kFillMaxWords * 32) {
        set_error("tri_compact_fill: budget %d above %d", budget, kFillMaxWords * 32);
        return TRI_ERR_UNSUPPORTED;
    }
    return TRI_OK;
}

tri_status launch_compact_fill(const tri_model &m, const tri_cache &c, int32_t budget, const int32_t *kept_idx,
                               const int32_t *kept_cnt, int32_t *new_seq_len, hipStream_t st)
{
    const int n_inst = m.n_layers * c.n_seqs * m.n_kv_heads;
    if (n_inst <= 0) return TRI_OK;
    tri_status rc = check_fill_budget(budget);
    if (rc != TRI_OK) return rc;
    CompactArgs a{};
    a.src = make_view(m, c);
    a.dst = a.src;
    a.kept_idx = kept_idx;
    a.kept_cnt = kept_cnt;
    a.new_seq_len = new_seq_len;
    a.budget = budget;
    a.elem_bytes = c.dtype == TRI_BF16 ? 2 : 4;
    a.row16 = kHeadDim * a.elem_bytes / 16;
    const size_t lds = (size_t)budget * 8;
    if (lds > 48 * 1024 &&
        hipFuncSetAttribute((const void *)fill_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
        return hip_status("hipFuncSetAttribute(fill_kernel)");
    hipLaunchKernelGGL(fill_kernel, dim3(n_inst), dim3(kFillThreads), lds, st, a);
    return hip_status("fill_kernel");
}

tri_status launch_compact(const tri_model &m, const tri_cache &src, const tri_cache &dst, int32_t budget,
                          const int32_t *kept_idx, const int32_t *kept_cnt, int32_t *new_seq_len,
                          hipStream_t st)
{
    const int n_inst = m.n_layers * src.n_seqs * m.n_kv_heads;
    if (n_inst <= 0) return TRI_OK;
    CompactArgs a{};
    a.src = make_view(m, src);
    a.dst = make_view(m, dst);
    a.dst.n_seqs = a.src.n_seqs;
    a.kept_idx = kept_idx;
    a.kept_cnt = kept_cnt;
    a.new_seq_len = new_seq_len;
    a.budget = budget;
    a.elem_bytes = src.dtype == TRI_BF16 ? 2 : 4;
    a.row16 = kHeadDim * a.elem_bytes / 16;
    const bool same = dst.k == src.k || dst.v == src.v || dst.pos == src.pos;
    if (same) {
        hipLaunchKernelGGL(inplace_kernel, dim3(n_inst), dim3(kInplaceThreads), 0, st, a);
        return hip_status("inplace_kernel");
    }
    a.row_blocks = (budget + kRowsPerBlock - 1) / kRowsPerBlock;
    if ((int64_t)a.row_blocks * n_inst > (int64_t)0x7fffffff) {
        set_error("tri_compact: %d head-instances x %d row blocks exceed the grid", n_inst, a.row_blocks);
        return TRI_ERR_UNSUPPORTED;
    }
    hipLaunchKernelGGL(gather_kernel, dim3((uint32_t)(a.row_blocks * (int64_t)n_inst)), dim3(kGatherThreads), 0, st, a);
    return hip_status("gather_kernel");
}

}  // namespace tri
