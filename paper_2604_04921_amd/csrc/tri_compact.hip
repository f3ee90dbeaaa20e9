// Eviction as compaction (Section 4.3, "evict the rest"): slot j <- slot kept_idx[j] for K, V
// and the key positions.  Pure byte moves, 16 bytes per lane.
#include "tri_fill.h"

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

// 128 threads, one pass over 8 bf16 rows: small workgroups keep the most independent row fetches in flight
// (measured on 9.4 M scattered rows: 64 threads 1.64 ms, 128: 1.63, 256: 1.71, 512: 1.68, 1024: 1.72)
constexpr int kGatherThreads = 128;
constexpr int kRowsPerBlock = kGatherThreads / 16;


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

// tri_compact_fill: grid (instances), block 256, dynamic LDS 8 * budget bytes (the move list); see fill_block.
__global__ __launch_bounds__(kFillThreads) void fill_kernel(CompactArgs a)
{
    extern __shared__ int32_t moves[];   // [2][budget]: destination slots, source slots
    __shared__ uint32_t kept_bits[kFillMaxWords];
    __shared__ uint32_t wave_tot[kFillThreads / 64];
    __shared__ int32_t n_tail;
    const int inst = blockIdx.x;
    const FillArgs f{a.src, a.new_seq_len, a.budget, a.elem_bytes, a.row16};
    fill_block(f, inst, read_cnt(a, inst), a.kept_idx + (int64_t)inst * a.budget, moves, kept_bits, wave_tot, &n_tail);
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
