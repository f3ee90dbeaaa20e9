// C-ABI entry points: host-side validation and dispatch.  See include/tri.h for the contract.
#include <cstdarg>
#include <cstdio>
#include <algorithm>
#include <mutex>

#include "tri_internal.h"
#include "tri_score_common.h"

namespace tri {

static thread_local char g_error[512] = "";

void set_error(const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_error, sizeof g_error, fmt, ap);
    va_end(ap);
}

static thread_local void **g_events = nullptr;
static thread_local int32_t g_event_pairs = 0, g_event_next = 0;

bool timing_next(hipEvent_t *start, hipEvent_t *stop)
{
    if (!g_events || g_event_next >= g_event_pairs) return false;
    *start = (hipEvent_t)g_events[2 * g_event_next];
    *stop = (hipEvent_t)g_events[2 * g_event_next + 1];
    ++g_event_next;
    return true;
}

tri_status hip_status(const char *what)
{
    hipError_t e = hipGetLastError();
    if (e == hipSuccess) return TRI_OK;
    set_error("%s: %s", what, hipGetErrorString(e));
    return TRI_ERR_HIP;
}

tri_status check_model(const tri_model *m)
{
    if (!m) {
        set_error("model is NULL");
        return TRI_ERR_INVALID_ARG;
    }
    if (m->n_layers < 1 || m->n_q_heads < 1 || m->n_kv_heads < 1 || m->n_q_heads % m->n_kv_heads != 0) {
        set_error("bad geometry: layers %d, q heads %d, kv heads %d", m->n_layers, m->n_q_heads, m->n_kv_heads);
        return TRI_ERR_INVALID_ARG;
    }
    if (m->head_dim != kHeadDim) {
        set_error("head_dim %d not built (128 only)", m->head_dim);
        return TRI_ERR_UNSUPPORTED;
    }
    const int G = m->n_q_heads / m->n_kv_heads;
    if (G < 1 || G > kMaxGroup) {
        set_error("group size %d not built (1 to 8)", G);
        return TRI_ERR_UNSUPPORTED;
    }
    if (!(m->rope_theta > 1.0)) {
        set_error("rope_theta must be > 1");
        return TRI_ERR_INVALID_ARG;
    }
    if (m->pairs != TRI_PAIR_INTERLEAVED && m->pairs != TRI_PAIR_HALF) {
        set_error("unknown pair layout %d", m->pairs);
        return TRI_ERR_INVALID_ARG;
    }
    if (m->score_variant < TRI_SCORE_FULL || m->score_variant > TRI_SCORE_NORM_UNWEIGHTED) {
        set_error("unknown score variant %d", m->score_variant);
        return TRI_ERR_INVALID_ARG;
    }
    if (m->n_offsets < 1 || m->n_offsets > kMaxOffsets || !m->offsets) {
        set_error("n_offsets must be in [1, %d] with a host offsets array", kMaxOffsets);
        return TRI_ERR_INVALID_ARG;
    }
    for (int j = 0; j < m->n_offsets; ++j)
        if (m->offsets[j] > ((int64_t)1 << 61) || m->offsets[j] < -((int64_t)1 << 61)) {
            set_error("offset %d out of range", j);
            return TRI_ERR_INVALID_ARG;
        }
    return TRI_OK;
}

static bool pow2(int x) { return x > 0 && (x & (x - 1)) == 0; }

tri_status check_cache(const tri_model *m, const tri_cache *c, bool need_v, const char *what)
{
    (void)m;
    if (!c) {
        set_error("%s cache is NULL", what);
        return TRI_ERR_INVALID_ARG;
    }
    if (!c->k || !c->pos || (need_v && !c->v)) {
        set_error("%s cache: k, pos%s must not be NULL", what, need_v ? ", v" : "");
        return TRI_ERR_INVALID_ARG;
    }
    if (c->dtype != TRI_F32 && c->dtype != TRI_BF16) {
        set_error("%s cache: unknown dtype %d", what, c->dtype);
        return TRI_ERR_INVALID_ARG;
    }
    if (c->n_seqs < 1 || c->max_seq_len < 0 || !c->seq_len || !c->cur_pos) {
        set_error("%s cache: n_seqs >= 1, max_seq_len >= 0, seq_len and cur_pos required", what);
        return TRI_ERR_INVALID_ARG;
    }
    if (c->block_size != 0 && (!pow2(c->block_size) || !c->block_table || c->max_blocks_per_seq < 1 ||
                               (int64_t)c->max_blocks_per_seq * c->block_size < c->max_seq_len)) {
        set_error("%s cache: paged layout needs a power-of-two block_size, a block table and "
                  "max_blocks_per_seq * block_size >= max_seq_len", what);
        return TRI_ERR_INVALID_ARG;
    }
    const int eb = c->dtype == TRI_BF16 ? 2 : 4;
    const int64_t a16 = 16 / eb;
    if (c->stride_slot < kHeadDim || c->stride_slot > 0x7fffffff || c->stride_slot % a16 || c->stride_head % a16 || c->stride_layer % a16 ||
        c->stride_seq_or_block % a16 || ((uintptr_t)c->k & 15) || ((uintptr_t)c->v & 15)) {
        set_error("%s cache: slots must be 16-byte aligned, at least head_dim and less than 2^31 elements apart", what);
        return TRI_ERR_INVALID_ARG;
    }
    if (c->stride_head < 0 || c->stride_layer < 0 || c->stride_seq_or_block < 0 || c->pos_stride_head < 0 ||
        c->pos_stride_layer < 0 || c->pos_stride_seq_or_block < 0) {
        set_error("%s cache: negative stride", what);
        return TRI_ERR_INVALID_ARG;
    }
    return TRI_OK;
}

CacheView make_view(const tri_model &m, const tri_cache &c)
{
    CacheView v{};
    v.k = c.k;
    v.v = c.v;
    v.pos = c.pos;
    v.seq_len = c.seq_len;
    v.cur_pos = c.cur_pos;
    v.block_table = c.block_table;
    v.stride_layer = c.stride_layer;
    v.stride_sb = c.stride_seq_or_block;
    v.stride_head = c.stride_head;
    v.stride_slot = c.stride_slot;
    v.pos_stride_layer = c.pos_stride_layer;
    v.pos_stride_sb = c.pos_stride_seq_or_block;
    v.pos_stride_head = c.pos_stride_head;
    v.n_seqs = c.n_seqs;
    v.n_kv_heads = m.n_kv_heads;
    v.max_seq_len = c.max_seq_len;
    v.block_shift = -1;
    if (c.block_size > 0) {
        v.block_shift = 0;
        while ((1 << v.block_shift) < c.block_size) ++v.block_shift;
    }
    v.max_blocks = c.max_blocks_per_seq;
    v.k_rotated = c.k_rotated != 0;
    return v;
}

static size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

Workspace workspace_layout(const tri_model &m, const tri_cache &c, int32_t budget)
{
    (void)budget;
    Workspace w{};
    const size_t G = (size_t)(m.n_q_heads / m.n_kv_heads);
    const size_t inst = (size_t)m.n_layers * c.n_seqs * m.n_kv_heads;
    const size_t tiles = ((size_t)c.max_seq_len + kScoreTile - 1) / kScoreTile;
    size_t o = 0;
    w.band_rev = o;
    o = align256(o + kBands * sizeof(double));
    w.fold_phasors = o;
    o = align256(o + ((size_t)c.n_seqs + 1) * kBands * 2 * sizeof(double));
    w.phasors = o;
    o = align256(o + 128 * 1024);
    w.table = o;
    o = align256(o + inst * kBands * 3 * G * sizeof(float));
    w.work = o;
    o = align256(o + fast_work_ints(c.n_seqs, c.max_seq_len) * sizeof(int32_t));
    w.partials = o;
    o = align256(o + inst * tiles * 2 * G * sizeof(double));
    w.stats = o;
    o = align256(o + inst * G * 2 * sizeof(double));
    w.raw = o;
    o = align256(o + inst * G * (size_t)c.max_seq_len * sizeof(float));
    w.final_ = o;
    o = align256(o + inst * (size_t)c.max_seq_len * sizeof(float));
    w.total = o;
    return w;
}

// Sizes that the launch grids cannot take are refused here, before anything is enqueued.  Head-instances (times the
// workgroups each of them gets) are a grid's x index, below 2^31; the score kernel for fp32 keys and small blocks puts
// (sequence, KV head) on y and the layer on z, below 65536 each.
tri_status check_limits(const tri_model &m, const tri_cache &c, int32_t budget, const char *what)
{
    const int64_t inst = (int64_t)m.n_layers * c.n_seqs * m.n_kv_heads;
    const int64_t per_inst = std::max<int64_t>(((int64_t)c.max_seq_len + 255) / 256, ((int64_t)budget + 7) / 8);
    if (inst * std::max<int64_t>(per_inst, 1) > (int64_t)0x7fffffff) {
        set_error("%s: %lld head-instances of up to %d keys (budget %d) exceed what one call takes; split the batch",
                  what, (long long)inst, c.max_seq_len, budget);
        return TRI_ERR_UNSUPPORTED;
    }
    if ((int64_t)c.n_seqs * m.n_kv_heads > 65535 || m.n_layers > 65535) {
        set_error("%s: n_seqs * n_kv_heads and n_layers must each be below 65536", what);
        return TRI_ERR_UNSUPPORTED;
    }
    return TRI_OK;
}

// The checks of tri_compact on its two caches; *d receives dst completed with the fields it borrows from src.
static tri_status check_compact(const tri_model *model, const tri_cache *src, const tri_cache *dst, int32_t budget,
                                tri_cache *d, const char *what)
{
    if (!dst || !dst->k || !dst->v || !dst->pos) {
        set_error("%s: dst with k, v, pos required", what);
        return TRI_ERR_INVALID_ARG;
    }
    *d = *dst;
    d->n_seqs = src->n_seqs;
    d->dtype = src->dtype;
    d->seq_len = src->seq_len;
    d->cur_pos = src->cur_pos;
    // only the first min(N_s, budget) slots of dst are ever written
    d->max_seq_len = budget < src->max_seq_len ? budget : src->max_seq_len;
    tri_status rc = check_cache(model, d, true, what);
    if (rc != TRI_OK) return rc;
    if (dst->k == src->k || dst->v == src->v || dst->pos == src->pos) {
        // In place: the ordered move relies on dst slot j and src slot j being the same memory, so the two
        // descriptors must map slots identically.
        const bool same_map = dst->k == src->k && dst->v == src->v && dst->pos == src->pos &&
                              dst->block_size == src->block_size && dst->block_table == src->block_table &&
                              (dst->block_size == 0 || dst->max_blocks_per_seq == src->max_blocks_per_seq) &&
                              dst->stride_layer == src->stride_layer && dst->stride_seq_or_block == src->stride_seq_or_block &&
                              dst->stride_head == src->stride_head && dst->stride_slot == src->stride_slot &&
                              dst->pos_stride_layer == src->pos_stride_layer &&
                              dst->pos_stride_seq_or_block == src->pos_stride_seq_or_block &&
                              dst->pos_stride_head == src->pos_stride_head;
        if (!same_map) {
            set_error("%s: dst shares memory with src but maps slots differently (in-place compaction needs the same "
                      "k, v, pos, strides and block table)", what);
            return TRI_ERR_INVALID_ARG;
        }
    }
    return check_limits(*model, *src, budget, what);
}

static tri_status check_workspace(const Workspace &wl, void *ws, size_t ws_bytes)
{
    if (!ws || ((uintptr_t)ws & 255) || ws_bytes < wl.total) {
        set_error("workspace must be 256-byte aligned and hold %zu bytes (got %zu)", wl.total, ws_bytes);
        return TRI_ERR_WORKSPACE;
    }
    return TRI_OK;
}

// ---- scratch memory of tri_compress_step_static(): owned by the library, one copy per GPU, kept until the process ends
constexpr size_t kStaticScratchBytes = TRI_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static void *g_scratch_ptr[kMaxDevices];   // device address of `scratch` on each GPU, asked once per GPU

// The array's name is a host-side stand-in, not a device address: the address on the current GPU comes from the
// runtime (no allocation: the array is part of the loaded code object).
static tri_status static_scratch(void **ptr)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        (void)hipGetLastError();
        set_error("tri_compress_step_static: no current device below %d", kMaxDevices);
        return TRI_ERR_HIP;
    }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) {
            (void)hipGetLastError();
            set_error("tri_compress_step_static: hipGetSymbolAddress(scratch): %s", hipGetErrorString(e));
            return TRI_ERR_HIP;
        }
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return TRI_OK;
}

}  // namespace tri

using namespace tri;

extern "C" {

const char *tri_last_error(void) { return g_error; }

tri_status tri_timing_attach(void **events, int32_t n_pairs)
{
    if (n_pairs < 0 || (n_pairs > 0 && !events)) {
        set_error("tri_timing_attach: events required for n_pairs > 0");
        return TRI_ERR_INVALID_ARG;
    }
    g_events = n_pairs > 0 ? events : nullptr;
    g_event_pairs = n_pairs;
    g_event_next = 0;
    return TRI_OK;
}

int32_t tri_timing_detach(void)
{
    const int32_t n = g_event_next;
    g_events = nullptr;
    g_event_pairs = g_event_next = 0;
    return n;
}

tri_status tri_build_centers(const tri_model *model, const void *q_samples, int32_t q_dtype, int64_t n_tokens,
                             float *centers_out, void *stream)
{
    tri_status rc = check_model(model);
    if (rc != TRI_OK) return rc;
    if (!q_samples || ((uintptr_t)q_samples & 15) || !centers_out || n_tokens < 1 ||
        (q_dtype != TRI_F32 && q_dtype != TRI_BF16)) {
        set_error("tri_build_centers: q_samples (16-byte aligned), centers_out, n_tokens >= 1 and a known dtype required");
        return TRI_ERR_INVALID_ARG;
    }
    return launch_centers(*model, q_samples, q_dtype, n_tokens, centers_out, nullptr, 0, (hipStream_t)stream);
}

tri_status tri_centers_accumulate(const tri_model *model, const void *q_samples, int32_t q_dtype, int64_t n_tokens,
                                  double *sums, int32_t first, void *stream)
{
    tri_status rc = check_model(model);
    if (rc != TRI_OK) return rc;
    if (!q_samples || ((uintptr_t)q_samples & 15) || !sums || n_tokens < 1 || (q_dtype != TRI_F32 && q_dtype != TRI_BF16)) {
        set_error("tri_centers_accumulate: q_samples (16-byte aligned), sums, n_tokens >= 1 and a known dtype required");
        return TRI_ERR_INVALID_ARG;
    }
    return launch_centers(*model, q_samples, q_dtype, n_tokens, nullptr, sums, first ? 1 : 0, (hipStream_t)stream);
}

tri_status tri_centers_finalize(const tri_model *model, const double *sums, int64_t total_tokens, float *centers_out,
                                void *stream)
{
    tri_status rc = check_model(model);
    if (rc != TRI_OK) return rc;
    if (!sums || !centers_out || total_tokens < 1) {
        set_error("tri_centers_finalize: sums, centers_out and total_tokens >= 1 required");
        return TRI_ERR_INVALID_ARG;
    }
    return launch_centers_finalize(*model, sums, total_tokens, centers_out, (hipStream_t)stream);
}

tri_status tri_band_diagnostics(const tri_model *model, const float *q_centers, const float *k_centers,
                                float *mrl_out, float *contrib_out, int32_t top_k, int32_t *top_bands_out,
                                void *stream)
{
    tri_status rc = check_model(model);
    if (rc != TRI_OK) return rc;
    if (!q_centers || !mrl_out) {
        set_error("tri_band_diagnostics: q_centers and mrl_out required");
        return TRI_ERR_INVALID_ARG;
    }
    if ((contrib_out || top_bands_out) && !k_centers) {
        set_error("tri_band_diagnostics: the band contributions need k_centers");
        return TRI_ERR_INVALID_ARG;
    }
    if (top_bands_out && (top_k < 1 || top_k > kBands)) {
        set_error("tri_band_diagnostics: top_k must be in [1, %d]", kBands);
        return TRI_ERR_INVALID_ARG;
    }
    return launch_diagnostics(*model, q_centers, k_centers, mrl_out, contrib_out, top_k, top_bands_out,
                              (hipStream_t)stream);
}

size_t tri_workspace_size(const tri_model *model, const tri_cache *cache, int32_t budget)
{
    if (check_model(model) != TRI_OK || !cache || cache->n_seqs < 1 || cache->max_seq_len < 0 || budget < 1)
        return 0;
    return workspace_layout(*model, *cache, budget).total;
}

tri_status tri_score(const tri_model *model, const float *centers, const tri_cache *cache, float *final_out,
                     float *raw_out, void *workspace, size_t ws_bytes, void *stream)
{
    tri_status rc = check_model(model);
    if (rc != TRI_OK) return rc;
    if ((rc = check_cache(model, cache, false, "tri_score")) != TRI_OK) return rc;
    if (!centers || !final_out) {
        set_error("tri_score: centers and final_out required");
        return TRI_ERR_INVALID_ARG;
    }
    if ((rc = check_limits(*model, *cache, 0, "tri_score")) != TRI_OK) return rc;
    const Workspace wl = workspace_layout(*model, *cache, 1);
    if ((rc = check_workspace(wl, workspace, ws_bytes)) != TRI_OK) return rc;
    return launch_score(*model, centers, *cache, final_out, raw_out, (char *)workspace, wl, nullptr, (hipStream_t)stream);
}

tri_status tri_select_topk(const tri_model *model, const float *final_scores, const tri_cache *cache,
                           int32_t budget, int32_t *kept_idx, int32_t *kept_cnt, void *workspace,
                           size_t ws_bytes, void *stream)
{
    (void)workspace;
    (void)ws_bytes;
    tri_status rc = check_model(model);
    if (rc != TRI_OK) return rc;
    if (!cache || cache->n_seqs < 1 || !cache->seq_len || cache->max_seq_len < 0) {
        set_error("tri_select_topk: cache with n_seqs, seq_len and max_seq_len required");
        return TRI_ERR_INVALID_ARG;
    }
    if (!final_scores || !kept_idx || !kept_cnt || budget < 1) {
        set_error("tri_select_topk: final_scores, kept_idx, kept_cnt and budget >= 1 required");
        return TRI_ERR_INVALID_ARG;
    }
    if ((rc = check_limits(*model, *cache, budget, "tri_select_topk")) != TRI_OK) return rc;
    return launch_select(*model, final_scores, nullptr, nullptr, nullptr, MomentLayout{1, 1}, nullptr, *cache, budget,
                         kept_idx, kept_cnt,
                         (hipStream_t)stream);
}

tri_status tri_compact(const tri_model *model, const tri_cache *src, const tri_cache *dst, int32_t budget,
                       const int32_t *kept_idx, const int32_t *kept_cnt, int32_t *new_seq_len, void *stream)
{
    tri_status rc = check_model(model);
    if (rc != TRI_OK) return rc;
    if ((rc = check_cache(model, src, true, "tri_compact src")) != TRI_OK) return rc;
    if (!kept_idx || !kept_cnt || budget < 1) {
        set_error("tri_compact: kept_idx, kept_cnt and budget >= 1 required");
        return TRI_ERR_INVALID_ARG;
    }
    tri_cache d;
    if ((rc = check_compact(model, src, dst, budget, &d, "tri_compact")) != TRI_OK) return rc;
    return launch_compact(*model, *src, d, budget, kept_idx, kept_cnt, new_seq_len, (hipStream_t)stream);
}

tri_status tri_compact_fill(const tri_model *model, const tri_cache *cache, int32_t budget,
                            const int32_t *kept_idx, const int32_t *kept_cnt, int32_t *new_seq_len, void *stream)
{
    tri_status rc = check_model(model);
    if (rc != TRI_OK) return rc;
    if ((rc = check_cache(model, cache, true, "tri_compact_fill")) != TRI_OK) return rc;
    if (!kept_idx || !kept_cnt || budget < 1) {
        set_error("tri_compact_fill: kept_idx, kept_cnt and budget >= 1 required");
        return TRI_ERR_INVALID_ARG;
    }
    if ((rc = check_limits(*model, *cache, budget, "tri_compact_fill")) != TRI_OK) return rc;
    if ((rc = check_fill_budget(budget)) != TRI_OK) return rc;
    return launch_compact_fill(*model, *cache, budget, kept_idx, kept_cnt, new_seq_len, (hipStream_t)stream);
}

// Everything tri_compress_step checks, so that an invalid call enqueues nothing at all: the source cache, the
// destination (as tri_compact or tri_compact_fill will check it again, on the same arguments) and the grid limits.
static tri_status check_step(const tri_model *model, const float *centers, const tri_cache *src, const tri_cache *dst,
                             int32_t budget, const int32_t *kept_idx, const int32_t *kept_cnt)
{
    tri_status rc = check_model(model);
    if (rc != TRI_OK) return rc;
    if ((rc = check_cache(model, src, true, "tri_compress_step src")) != TRI_OK) return rc;
    if (!centers || !kept_idx || !kept_cnt || budget < 1) {
        set_error("tri_compress_step: centers, kept_idx, kept_cnt and budget >= 1 required");
        return TRI_ERR_INVALID_ARG;
    }
    if ((rc = check_limits(*model, *src, budget, "tri_compress_step")) != TRI_OK) return rc;
    if (!dst) return check_fill_budget(budget);
    tri_cache d;
    return check_compact(model, src, dst, budget, &d, "tri_compress_step dst");
}

static tri_status run_step(const tri_model *model, const float *centers, const tri_cache *src, const tri_cache *dst,
                           int32_t budget, int32_t *kept_idx, int32_t *kept_cnt, int32_t *new_seq_len, char *ws,
                           const Workspace &wl, void *stream)
{
    tri_status rc;
    // raw scores and their moments stay in the workspace; the selection forms statistics and final scores itself
    MomentLayout moments{1, 1};
    if ((rc = launch_score(*model, centers, *src, nullptr, nullptr, ws, wl, &moments, (hipStream_t)stream)) != TRI_OK)
        return rc;
    // evicting in place with the fewest moves, the selection's workgroups do the moves themselves where they can
    const FillTail fill{new_seq_len};
    bool filled = false;
    if ((rc = launch_select(*model, nullptr, reinterpret_cast<const float *>(ws + wl.raw), nullptr,
                            reinterpret_cast<const double *>(ws + wl.partials), moments,
                            reinterpret_cast<uint32_t *>(ws + wl.final_), *src, budget, kept_idx, kept_cnt,
                            (hipStream_t)stream, dst ? nullptr : &fill, &filled)) != TRI_OK)
        return rc;
    if (filled) return TRI_OK;
    if (!dst) return tri_compact_fill(model, src, budget, kept_idx, kept_cnt, new_seq_len, stream);
    return tri_compact(model, src, dst, budget, kept_idx, kept_cnt, new_seq_len, stream);
}

tri_status tri_compress_step(const tri_model *model, const float *centers, const tri_cache *src,
                             const tri_cache *dst, int32_t budget, int32_t *kept_idx, int32_t *kept_cnt,
                             int32_t *new_seq_len, void *workspace, size_t ws_bytes, void *stream)
{
    tri_status rc = check_step(model, centers, src, dst, budget, kept_idx, kept_cnt);
    if (rc != TRI_OK) return rc;
    const Workspace wl = workspace_layout(*model, *src, budget);
    if ((rc = check_workspace(wl, workspace, ws_bytes)) != TRI_OK) return rc;
    return run_step(model, centers, src, dst, budget, kept_idx, kept_cnt, new_seq_len, (char *)workspace, wl, stream);
}

size_t tri_static_scratch_size(void) { return kStaticScratchBytes; }

tri_status tri_compress_step_static(const tri_model *model, const float *centers, const tri_cache *src,
                                    const tri_cache *dst, int32_t budget, int32_t *kept_idx, int32_t *kept_cnt,
                                    int32_t *new_seq_len, void *stream)
{
    tri_status rc = check_step(model, centers, src, dst, budget, kept_idx, kept_cnt);
    if (rc != TRI_OK) return rc;
    const Workspace wl = workspace_layout(*model, *src, budget);
    if (wl.total > kStaticScratchBytes) {
        set_error("tri_compress_step_static: this call needs %zu bytes of scratch, the library's own array holds %zu; "
                  "use tri_compress_step with a workspace", wl.total, kStaticScratchBytes);
        return TRI_ERR_WORKSPACE;
    }
    void *ws = nullptr;
    if ((rc = static_scratch(&ws)) != TRI_OK) return rc;
    return run_step(model, centers, src, dst, budget, kept_idx, kept_cnt, new_seq_len, (char *)ws, wl, stream);
}

}  // extern "C"
