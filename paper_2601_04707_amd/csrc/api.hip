// Host side of the C ABI: contexts, argument checks, profiling, dispatch to the kernel launchers.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>

#include "common.h"

namespace {
thread_local std::string g_create_error = "";

bool valid_itype(int32_t t) { return t == MQG_I32 || t == MQG_I64; }
bool valid_dtype(int32_t t) { return t == MQG_F32 || t == MQG_F16; }

template <typename T>
hipError_t dev_alloc(T **p, int64_t n) {
    return hipMalloc(reinterpret_cast<void **>(p), static_cast<size_t>(std::max<int64_t>(n, 1)) * sizeof(T));
}
}  // namespace

namespace mqg {

int fail(mqg_ctx *ctx, int code, const std::string &msg) {
    if (ctx) ctx->last_error = msg; else g_create_error = msg;
    return code;
}

int prof_name_id(mqg_ctx *ctx, const char *name) {
    for (size_t i = 0; i < ctx->prof_names.size(); ++i)
        if (ctx->prof_names[i] == name) return static_cast<int>(i);
    ctx->prof_names.emplace_back(name);
    ctx->prof_total_ms.push_back(0.0);
    ctx->prof_launches.push_back(0);
    return static_cast<int>(ctx->prof_names.size()) - 1;
}

static hipEvent_t take_event(mqg_ctx *ctx) {
    if (!ctx->event_pool.empty()) {
        hipEvent_t e = ctx->event_pool.back();
        ctx->event_pool.pop_back();
        return e;
    }
    hipEvent_t e = nullptr;
    (void)hipEventCreate(&e);
    return e;
}

void prof_begin(mqg_ctx *ctx, const char *name, hipStream_t s) {
    ProfRec r;
    r.name_id = prof_name_id(ctx, name);
    r.start = take_event(ctx);
    r.stop = take_event(ctx);
    (void)hipEventRecord(r.start, s);
    ctx->prof_recs.push_back(r);
}

// A record whose two events the launch itself fills in (hipExtLaunchKernelGGL): the kernel's own
// start and end, without the latency of separate event packets around it.
void prof_begin_ext(mqg_ctx *ctx, const char *name, hipEvent_t *start, hipEvent_t *stop) {
    ProfRec r;
    r.name_id = prof_name_id(ctx, name);
    r.start = take_event(ctx);
    r.stop = take_event(ctx);
    ctx->prof_recs.push_back(r);
    *start = r.start;
    *stop = r.stop;
}

void prof_end(mqg_ctx *ctx, hipStream_t s) {
    (void)hipEventRecord(ctx->prof_recs.back().stop, s);
}

// Fold finished event pairs into the per-kernel totals and recycle the events.
static int prof_collect(mqg_ctx *ctx) {
    for (auto &r : ctx->prof_recs) {
        hipError_t e = hipEventSynchronize(r.stop);
        if (e != hipSuccess) return fail(ctx, MQG_ERR_HIP, std::string("hipEventSynchronize: ") + hipGetErrorString(e));
        float ms = 0.f;
        e = hipEventElapsedTime(&ms, r.start, r.stop);
        if (e != hipSuccess) return fail(ctx, MQG_ERR_HIP, std::string("hipEventElapsedTime: ") + hipGetErrorString(e));
        ctx->prof_total_ms[r.name_id] += ms;
        ctx->prof_launches[r.name_id] += 1;
        ctx->event_pool.push_back(r.start);
        ctx->event_pool.push_back(r.stop);
    }
    ctx->prof_recs.clear();
    return MQG_OK;
}

void free_backward_scratch(mqg_ctx *ctx) {
    (void)hipFree(ctx->bwd.keys[0]);
    (void)hipFree(ctx->bwd.keys[1]);
    (void)hipFree(ctx->bwd.vals[0]);
    (void)hipFree(ctx->bwd.vals[1]);
    (void)hipFree(ctx->bwd.hist);
    (void)hipFree(ctx->bwd.tile_sums);
    (void)hipFree(ctx->bwd_dst_row);
    (void)hipFree(ctx->bwd_col_ptr);
    (void)hipFree(ctx->bwd_w_sorted);
    ctx->bwd_w_sorted = nullptr;
    ctx->bwd = RadixBufs{};
    ctx->bwd_dst_row = ctx->bwd_col_ptr = nullptr;
    ctx->bwd_nnz_cap = ctx->bwd_src_cap = 0;
}

}  // namespace mqg

using mqg::fail;

extern "C" {

int32_t mqg_version(void) { return 100; }

const char *mqg_last_error(const mqg_ctx *ctx) {
    return ctx ? ctx->last_error.c_str() : g_create_error.c_str();
}

int mqg_ctx_create(mqg_ctx **out, const mqg_graph *g, int32_t max_seeds, const int32_t *max_fanouts,
                   int32_t L) {
    if (!out) return fail(nullptr, MQG_ERR_INVALID_ARG, "mqg_ctx_create: out is NULL");
    *out = nullptr;
    if (!g || !max_fanouts) return fail(nullptr, MQG_ERR_INVALID_ARG, "mqg_ctx_create: NULL graph or fanouts");
    if (g->num_nodes < 0 || g->num_edges < 0 || !valid_itype(g->ptr_type) || !valid_itype(g->idx_type))
        return fail(nullptr, MQG_ERR_INVALID_ARG, "mqg_ctx_create: bad graph descriptor");
    if (g->num_nodes >= (int64_t(1) << 31))
        return fail(nullptr, MQG_ERR_UNSUPPORTED, "mqg_ctx_create: num_nodes must be below 2^31");
    if (L < 1 || L > MQG_MAX_LAYERS) return fail(nullptr, MQG_ERR_INVALID_ARG, "mqg_ctx_create: num_layers out of range");
    if (max_seeds < 0) return fail(nullptr, MQG_ERR_INVALID_ARG, "mqg_ctx_create: negative max_seeds");
    for (int l = 0; l < L; ++l)
        if (max_fanouts[l] < 1 || max_fanouts[l] > MQG_MAX_FANOUT)
            return fail(nullptr, MQG_ERR_UNSUPPORTED, "mqg_ctx_create: fanout outside 1..MQG_MAX_FANOUT");

    mqg_ctx *c = new (std::nothrow) mqg_ctx();
    if (!c) return fail(nullptr, MQG_ERR_HIP, "mqg_ctx_create: out of host memory");
    hipError_t e = hipGetDevice(&c->device);
    if (e != hipSuccess) {
        delete c;
        return fail(nullptr, MQG_ERR_HIP, std::string("hipGetDevice: ") + hipGetErrorString(e));
    }
    c->num_nodes = g->num_nodes;
    c->ptr_type = g->ptr_type;
    c->idx_type = g->idx_type;
    c->max_seeds = max_seeds;
    c->num_layers = L;
    int64_t dst = max_seeds;
    for (int l = L - 1; l >= 0; --l) {
        c->max_fanouts[l] = max_fanouts[l];
        c->bound_dst[l] = dst;
        c->bound_nnz[l] = dst * max_fanouts[l];
        c->bound_src[l] = std::max(dst, std::min<int64_t>(g->num_nodes, dst + c->bound_nnz[l]));
        c->max_dst = std::max(c->max_dst, c->bound_dst[l]);
        c->max_nnz = std::max(c->max_nnz, c->bound_nnz[l]);
        c->max_src = std::max(c->max_src, c->bound_src[l]);
        dst = c->bound_src[l];
    }
    if (c->max_nnz >= (int64_t(1) << 31)) {
        delete c;
        return fail(nullptr, MQG_ERR_UNSUPPORTED, "mqg_ctx_create: more than 2^31 sampled edges per block");
    }
    c->bitmap_words = std::max<int64_t>(1, mqg::ceil_div(mqg::ceil_div(g->num_nodes, 32), mqg::kBitmapTileWords)) * mqg::kBitmapTileWords;
    c->max_tiles = std::max<int64_t>(mqg::ceil_div(c->max_dst, mqg::kBlock), c->bitmap_words / mqg::kBlock) + 1;

    bool ok = true;
    ok = ok && dev_alloc(&c->local_of, c->num_nodes) == hipSuccess;
    ok = ok && dev_alloc(&c->bitmap, c->bitmap_words) == hipSuccess;
    ok = ok && dev_alloc(&c->tile_vals, c->max_tiles) == hipSuccess;
    ok = ok && dev_alloc(&c->bitmap_tile_vals, c->max_tiles) == hipSuccess;
    ok = ok && dev_alloc(&c->row_start, c->max_dst) == hipSuccess;
    ok = ok && dev_alloc(&c->row_deg, c->max_dst) == hipSuccess;
    ok = ok && dev_alloc(reinterpret_cast<int32_t **>(&c->nbr), c->max_nnz) == hipSuccess;
    ok = ok && dev_alloc(&c->heavy_rows, c->max_dst) == hipSuccess;
    ok = ok && dev_alloc(&c->heavy_count, MQG_MAX_LAYERS + 1) == hipSuccess;
    ok = ok && dev_alloc(&c->hit_list, c->max_src) == hipSuccess;
    ok = ok && dev_alloc(&c->miss_list, c->max_src) == hipSuccess;
    ok = ok && dev_alloc(&c->counters, 8) == hipSuccess;
    if (ok) ok = hipMemset(c->local_of, 0xFF, std::max<int64_t>(c->num_nodes, 1) * sizeof(int32_t)) == hipSuccess;
    if (ok) ok = hipMemset(c->bitmap, 0, std::max<int64_t>(c->bitmap_words, 1) * sizeof(uint32_t)) == hipSuccess;
    if (ok) ok = hipMemset(c->counters, 0, 8 * sizeof(unsigned long long)) == hipSuccess;
    if (ok) ok = hipMemset(c->heavy_count, 0, (MQG_MAX_LAYERS + 1) * sizeof(int32_t)) == hipSuccess;
    if (ok) ok = hipDeviceSynchronize() == hipSuccess;
    if (!ok) {
        std::string msg = std::string("mqg_ctx_create: scratch allocation failed: ") + hipGetErrorString(hipGetLastError());
        mqg_ctx_destroy(c);
        return fail(nullptr, MQG_ERR_HIP, msg);
    }
    *out = c;
    return MQG_OK;
}

int mqg_ctx_destroy(mqg_ctx *c) {
    if (!c) return MQG_OK;
    (void)hipFree(c->local_of);
    (void)hipFree(c->bitmap);
    (void)hipFree(c->tile_vals);
    (void)hipFree(c->bitmap_tile_vals);
    (void)hipFree(c->row_start);
    (void)hipFree(c->row_deg);
    (void)hipFree(c->nbr);
    (void)hipFree(c->heavy_rows);
    (void)hipFree(c->heavy_count);
    (void)hipFree(c->hit_list);
    (void)hipFree(c->miss_list);
    (void)hipFree(c->counters);
    mqg::free_backward_scratch(c);
    mqg::free_hash_scratch(c);
    mqg::free_layerwise_scratch(c);
    (void)hipFree(c->prio_bitmap);
    (void)hipFree(c->prio_count);
    (void)hipFree(c->cache_arena);
    for (auto &r : c->prof_recs) {
        (void)hipEventDestroy(r.start);
        (void)hipEventDestroy(r.stop);
    }
    for (auto e : c->event_pool) (void)hipEventDestroy(e);
    delete c;
    return MQG_OK;
}

int mqg_ctx_set_option(mqg_ctx *ctx, int32_t option, int64_t value) {
    if (!ctx) return MQG_ERR_INVALID_ARG;
    switch (option) {
        case MQG_OPT_FORCE_SLOW_SELECT: ctx->force_slow_select = value != 0; return MQG_OK;
        case MQG_OPT_PROFILE: ctx->profile = value != 0; return MQG_OK;
        case MQG_OPT_DEDUP_HASH:
            if (value != 0) {
                int rc = mqg::ensure_hash_scratch(ctx);
                if (rc != MQG_OK) return rc;
            }
            ctx->dedup_hash = value != 0;
            return MQG_OK;
        case MQG_OPT_HEAVY_DEGREE:
            if (value < 64 || value > 0x7FFFFFFF) return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_ctx_set_option: MQG_OPT_HEAVY_DEGREE outside 64..2^31-1");
            ctx->heavy_degree = static_cast<int>(value);
            return MQG_OK;
        case MQG_OPT_MISS_INFLIGHT_BYTES:
            if (value < 1024 || value > (int64_t(1) << 30)) return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_ctx_set_option: MQG_OPT_MISS_INFLIGHT_BYTES outside 1 KiB..1 GiB");
            ctx->miss_inflight_bytes = value;
            return MQG_OK;
        case MQG_OPT_LAYERWISE_CANDIDATES:
            if (value < 0 || value > 3) return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_ctx_set_option: MQG_OPT_LAYERWISE_CANDIDATES outside 0..3");
            ctx->layerwise_candidates = static_cast<int>(value);
            return MQG_OK;
        default: return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_ctx_set_option: unknown option");
    }
}

int mqg_ctx_reserve(mqg_ctx *ctx, int32_t what, int64_t layerwise_rows) {
    if (!ctx) return MQG_ERR_INVALID_ARG;
    const int32_t all = MQG_RESERVE_BACKWARD | MQG_RESERVE_LAYERWISE | MQG_RESERVE_DEDUP_HASH | MQG_RESERVE_SAMPLING_PRIORITY |
                        MQG_RESERVE_CACHE_BUILD;
    if (what < 0 || (what & ~all) != 0 || layerwise_rows < 0)
        return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_ctx_reserve: unknown flag or negative row count");
    int rc = MQG_OK;
    if (rc == MQG_OK && (what & MQG_RESERVE_BACKWARD))
        rc = mqg::ensure_backward_scratch(ctx, ctx->max_nnz, ctx->max_src, nullptr, "mqg_ctx_reserve: ");
    if (rc == MQG_OK && (what & MQG_RESERVE_LAYERWISE))
        rc = mqg::ensure_layerwise_scratch(ctx, std::max<int64_t>(std::max<int64_t>(layerwise_rows, ctx->max_seeds), 1), nullptr);
    if (rc == MQG_OK && (what & MQG_RESERVE_DEDUP_HASH)) rc = mqg::ensure_hash_scratch(ctx);
    if (rc == MQG_OK && (what & MQG_RESERVE_SAMPLING_PRIORITY)) rc = mqg::ensure_priority_scratch(ctx);
    if (rc == MQG_OK && (what & MQG_RESERVE_CACHE_BUILD)) rc = mqg::ensure_cache_build_scratch(ctx);
    return rc;
}

int mqg_ctx_kernel_time(mqg_ctx *ctx, const char *name, double *total_ms, int64_t *launches) {
    if (!ctx || !name || !total_ms || !launches) return MQG_ERR_INVALID_ARG;
    int rc = mqg::prof_collect(ctx);
    if (rc != MQG_OK) return rc;
    *total_ms = 0.0;
    *launches = 0;
    for (size_t i = 0; i < ctx->prof_names.size(); ++i)
        if (ctx->prof_names[i] == name) {
            *total_ms = ctx->prof_total_ms[i];
            *launches = ctx->prof_launches[i];
        }
    return MQG_OK;
}

int mqg_ctx_reset_profile(mqg_ctx *ctx) {
    if (!ctx) return MQG_ERR_INVALID_ARG;
    int rc = mqg::prof_collect(ctx);
    if (rc != MQG_OK) return rc;
    std::fill(ctx->prof_total_ms.begin(), ctx->prof_total_ms.end(), 0.0);
    std::fill(ctx->prof_launches.begin(), ctx->prof_launches.end(), 0);
    return MQG_OK;
}

int mqg_ctx_kernel_names(mqg_ctx *ctx, char *buf, int64_t buf_len) {
    if (!ctx || !buf || buf_len < 1) return MQG_ERR_INVALID_ARG;
    std::string all;
    for (auto &n : ctx->prof_names) {
        if (!all.empty()) all += "\n";
        all += n;
    }
    if (static_cast<int64_t>(all.size()) + 1 > buf_len) return fail(ctx, MQG_ERR_CAPACITY, "mqg_ctx_kernel_names: buffer too small");
    std::memcpy(buf, all.c_str(), all.size() + 1);
    return MQG_OK;
}

static int check_graph(mqg_ctx *ctx, const mqg_graph *g, const char *who) {
    if (!g) return fail(ctx, MQG_ERR_INVALID_ARG, std::string(who) + ": graph is NULL");
    if (!valid_itype(g->ptr_type) || !valid_itype(g->idx_type))
        return fail(ctx, MQG_ERR_INVALID_ARG, std::string(who) + ": bad index type");
    if (g->num_nodes != ctx->num_nodes || g->ptr_type != ctx->ptr_type || g->idx_type != ctx->idx_type)
        return fail(ctx, MQG_ERR_INVALID_ARG, std::string(who) + ": graph does not match the context");
    if (!g->row_ptr || (g->num_edges > 0 && !g->col_idx))
        return fail(ctx, MQG_ERR_INVALID_ARG, std::string(who) + ": NULL graph arrays");
    return MQG_OK;
}

int mqg_build_cache_ex(mqg_ctx *ctx, const mqg_graph *g, mqg_cache *cache, const mqg_cache_plan *plan, mqg_stream stream) {
    if (!ctx) return MQG_ERR_INVALID_ARG;
    int rc = check_graph(ctx, g, "mqg_build_cache");
    if (rc != MQG_OK) return rc;
    if (!cache) return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_build_cache: cache is NULL");
    if (cache->num_nodes != g->num_nodes) return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_build_cache: cache->num_nodes differs from the graph");
    if (cache->num_cached < 0 || cache->num_cached > cache->num_nodes)
        return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_build_cache: num_cached outside [0, num_nodes]");
    if (!valid_dtype(cache->dtype) || cache->dim < 1) return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_build_cache: bad dtype or dim");
    if (!cache->slot_of || !cache->feats || (cache->num_cached > 0 && !cache->cache_rows))
        return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_build_cache: NULL cache buffers");
    if (cache->feat_stride < cache->dim || cache->cache_stride < cache->dim)
        return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_build_cache: stride below dim");
    if (plan) {
        if (plan->policy != MQG_CACHE_TOP_DEGREE && plan->policy != MQG_CACHE_DEGREE_SAMPLED && plan->policy != MQG_CACHE_RANDOM_WALK &&
            plan->policy != MQG_CACHE_RANDOM_WALK_SAMPLED)
            return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_build_cache_ex: unknown policy");
        if (plan->policy == MQG_CACHE_RANDOM_WALK || plan->policy == MQG_CACHE_RANDOM_WALK_SAMPLED) {
            if (plan->num_steps < 0 || plan->num_steps > MQG_MAX_LAYERS) return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_build_cache_ex: num_steps outside 0..MQG_MAX_LAYERS");
            if (plan->num_train < 0 || (plan->num_train > 0 && !plan->train_ids)) return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_build_cache_ex: bad training set");
            if (plan->num_steps > 0 && !plan->step_fanouts) return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_build_cache_ex: step_fanouts is NULL");
            for (int l = 0; l < plan->num_steps; ++l)
                if (plan->step_fanouts[l] < 1) return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_build_cache_ex: step fanout below 1");
            if (g->num_edges > 0 && !g->col_idx) return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_build_cache_ex: col_idx is NULL");
            if (plan->walk_form != MQG_WALK_PUSH && plan->walk_form != MQG_WALK_PRINTED)
                return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_build_cache_ex: unknown walk_form");
            if (plan->walk_form == MQG_WALK_PUSH && !plan->graph_symmetric && g->num_edges >= (int64_t(1) << 31))
                return fail(ctx, MQG_ERR_UNSUPPORTED, "mqg_build_cache_ex: the push form transposes the adjacency, which is built for "
                                                      "fewer than 2^31 edges (set graph_symmetric if the graph equals its transpose)");
        }
    }
    return mqg::run_build_cache(ctx, g, cache, plan, static_cast<hipStream_t>(stream));
}

int mqg_ctx_set_sampling_priority(mqg_ctx *ctx, const mqg_graph *g, const mqg_cache *cache, mqg_stream stream) {
    if (!ctx) return MQG_ERR_INVALID_ARG;
    if (cache) {
        int rc = check_graph(ctx, g, "mqg_ctx_set_sampling_priority");
        if (rc != MQG_OK) return rc;
        if (!cache->slot_of) return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_ctx_set_sampling_priority: cache->slot_of is NULL");
        if (cache->num_nodes != ctx->num_nodes)
            return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_ctx_set_sampling_priority: cache->num_nodes differs from the context's graph");
    }
    return mqg::run_set_sampling_priority(ctx, g, cache, static_cast<hipStream_t>(stream));
}

int mqg_build_cache(mqg_ctx *ctx, const mqg_graph *g, mqg_cache *cache, mqg_stream stream) {
    return mqg_build_cache_ex(ctx, g, cache, nullptr, stream);
}

static int sample_blocks_checked(mqg_ctx *ctx, const mqg_graph *g, const void *seeds_dev, int32_t num_seeds,
                                 const int32_t *fanouts, int32_t L, uint64_t rng_seed, const uint64_t *seed_dev,
                                 mqg_block *blocks, mqg_stream stream) {
    if (!ctx) return MQG_ERR_INVALID_ARG;
    int rc = check_graph(ctx, g, "mqg_sample_blocks");
    if (rc != MQG_OK) return rc;
    if (!fanouts || !blocks) return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_sample_blocks: NULL fanouts or blocks");
    if (L != ctx->num_layers) return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_sample_blocks: num_layers differs from the context");
    if (num_seeds < 0) return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_sample_blocks: negative num_seeds");
    if (num_seeds > ctx->max_seeds) return fail(ctx, MQG_ERR_CAPACITY, "mqg_sample_blocks: num_seeds above the context's max_seeds");
    if (num_seeds > 0 && !seeds_dev) return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_sample_blocks: seeds_dev is NULL");
    if (num_seeds > 0 && g->num_nodes == 0) return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_sample_blocks: seeds given for an empty graph");
    int64_t dst = num_seeds;
    for (int l = L - 1; l >= 0; --l) {
        if (fanouts[l] < 1 || fanouts[l] > MQG_MAX_FANOUT)
            return fail(ctx, MQG_ERR_UNSUPPORTED, "mqg_sample_blocks: fanout outside 1..MQG_MAX_FANOUT");
        if (fanouts[l] > ctx->max_fanouts[l])
            return fail(ctx, MQG_ERR_CAPACITY, "mqg_sample_blocks: fanout above the context's max_fanouts");
        const mqg_block &b = blocks[l];
        if (!b.src_ids || !b.indptr || !b.indices || !b.sizes)
            return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_sample_blocks: NULL block buffer");
        int64_t nnz = dst * fanouts[l];
        int64_t src = std::max(dst, std::min<int64_t>(g->num_nodes, dst + nnz));
        if (b.cap_dst < dst || b.cap_nnz < nnz || b.cap_src < src)
            return fail(ctx, MQG_ERR_CAPACITY, "mqg_sample_blocks: block " + std::to_string(l) +
                        " needs cap_dst>=" + std::to_string(dst) + " cap_nnz>=" + std::to_string(nnz) +
                        " cap_src>=" + std::to_string(src));
        dst = src;
    }
    return mqg::run_sample_blocks(ctx, g, seeds_dev, num_seeds, fanouts, L, rng_seed, seed_dev, blocks,
                                  static_cast<hipStream_t>(stream));
}

int mqg_sample_blocks(mqg_ctx *ctx, const mqg_graph *g, const void *seeds_dev, int32_t num_seeds,
                      const int32_t *fanouts, int32_t L, uint64_t rng_seed, mqg_block *blocks,
                      mqg_stream stream) {
    return sample_blocks_checked(ctx, g, seeds_dev, num_seeds, fanouts, L, rng_seed, nullptr, blocks, stream);
}

int mqg_sample_blocks_seed_dev(mqg_ctx *ctx, const mqg_graph *g, const void *seeds_dev, int32_t num_seeds,
                               const int32_t *fanouts, int32_t L, const uint64_t *rng_seed_dev, mqg_block *blocks,
                               mqg_stream stream) {
    if (!ctx) return MQG_ERR_INVALID_ARG;
    if (!rng_seed_dev) return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_sample_blocks_seed_dev: rng_seed_dev is NULL");
    return sample_blocks_checked(ctx, g, seeds_dev, num_seeds, fanouts, L, 0, rng_seed_dev, blocks, stream);
}

int mqg_sample_layerwise(mqg_ctx *ctx, const mqg_graph *g, const void *seeds_dev, int32_t num_seeds,
                         const int32_t *layer_sizes, int32_t L, uint64_t rng_seed, int32_t normalise, int32_t method,
                         mqg_block *blocks, float *const *edge_w, mqg_stream stream) {
    if (!ctx) return MQG_ERR_INVALID_ARG;
    int rc = check_graph(ctx, g, "mqg_sample_layerwise");
    if (rc != MQG_OK) return rc;
    if (!layer_sizes || !blocks || !edge_w) return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_sample_layerwise: NULL layer_sizes, blocks or edge_w");
    if (L < 1 || L > MQG_MAX_LAYERS) return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_sample_layerwise: num_layers outside 1..MQG_MAX_LAYERS");
    if (method < 0 || method > (MQG_LAYERWISE_FASTGCN | MQG_LAYERWISE_DEBIAS | MQG_LAYERWISE_FLAT))
        return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_sample_layerwise: unknown method");
    if (num_seeds < 0) return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_sample_layerwise: negative num_seeds");
    if (num_seeds > 0 && !seeds_dev) return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_sample_layerwise: seeds_dev is NULL");
    if (num_seeds > 0 && g->num_nodes == 0) return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_sample_layerwise: seeds given for an empty graph");
    int64_t rows = num_seeds;
    for (int l = L - 1; l >= 0; --l) {
        if (layer_sizes[l] < 1) return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_sample_layerwise: layer size below 1");
        const mqg_block &b = blocks[l];
        if (!b.src_ids || !b.indptr || !b.indices || !b.sizes || !edge_w[l])
            return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_sample_layerwise: NULL block buffer");
        const int64_t src = std::min<int64_t>(g->num_nodes, layer_sizes[l]);
        if (rows * (src + 1) >= (int64_t(1) << 31))         // edge positions are 32-bit: rows x drawn nodes bounds the edges
            return fail(ctx, MQG_ERR_UNSUPPORTED, "mqg_sample_layerwise: block " + std::to_string(l) + " could hold 2^31 edges or more");
        if (b.cap_dst < rows || b.cap_src < src || b.cap_nnz < 0 || b.cap_nnz >= (int64_t(1) << 31))
            return fail(ctx, MQG_ERR_CAPACITY, "mqg_sample_layerwise: block " + std::to_string(l) + " needs cap_dst>=" +
                        std::to_string(rows) + " cap_src>=" + std::to_string(src) + " and 0 <= cap_nnz < 2^31");
        rows = src;
    }
    return mqg::run_sample_layerwise(ctx, g, seeds_dev, num_seeds, layer_sizes, L, rng_seed, normalise, method, blocks, edge_w,
                                     static_cast<hipStream_t>(stream));
}

int mqg_select_smallest_keys(mqg_ctx *ctx, const uint64_t *keys_dev, int64_t n, int64_t k, uint32_t *out_bitmap_dev,
                             mqg_stream stream) {
    if (!ctx) return MQG_ERR_INVALID_ARG;
    if (n < 0 || k < 0 || n >= (int64_t(1) << 31)) return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_select_smallest_keys: n or k out of range");
    if (n > 0 && (!keys_dev || !out_bitmap_dev)) return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_select_smallest_keys: NULL keys or bitmap");
    if (n == 0) return MQG_OK;
    return mqg::run_select_smallest_keys(ctx, keys_dev, n, k, out_bitmap_dev, static_cast<hipStream_t>(stream));
}

int mqg_select_row_candidates(mqg_ctx *ctx, const uint64_t *keys_dev, const uint32_t *slot_words_dev, int32_t count,
                              int32_t k, int32_t prioritised, int32_t ordered, uint32_t *out_mask_dev, mqg_stream stream) {
    if (!ctx) return MQG_ERR_INVALID_ARG;
    if (count < 1 || count > 256 || k < 1 || k > count)
        return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_select_row_candidates: need 1 <= k <= count <= 256");
    if (!keys_dev || !slot_words_dev || !out_mask_dev)
        return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_select_row_candidates: NULL argument");
    return mqg::run_select_row_candidates(ctx, keys_dev, slot_words_dev, count, k, prioritised ? 1 : 0, ordered ? 1 : 0,
                                          out_mask_dev, static_cast<hipStream_t>(stream));
}

int mqg_exp_tickets(mqg_ctx *ctx, uint64_t seed, int64_t tag, int64_t first, int64_t n, uint64_t *tickets_dev,
                    mqg_stream stream) {
    if (!ctx) return MQG_ERR_INVALID_ARG;
    if (n < 0 || n >= (int64_t(1) << 31) * mqg::kBlock) return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_exp_tickets: n out of range");
    if (n > 0 && !tickets_dev) return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_exp_tickets: tickets_dev is NULL");
    if (n == 0) return MQG_OK;
    return mqg::run_exp_tickets(ctx, seed, tag, first, n, tickets_dev, static_cast<hipStream_t>(stream));
}

static int gather_checked(mqg_ctx *ctx, const mqg_cache *cache, int32_t idx_type, const void *ids_dev,
                          const int64_t *num_ids_dev, int64_t cap_ids, void *out_dev, int64_t out_stride,
                          int64_t *stats_dev, int phases, mqg_stream stream) {
    if (!ctx) return MQG_ERR_INVALID_ARG;
    int rc = mqg::check_gather_args(ctx, cache, idx_type, ids_dev, num_ids_dev, cap_ids, out_dev, out_stride, ctx->max_src,
                                    "the context's largest source list");
    if (rc != MQG_OK) return rc;
    return mqg::run_gather(ctx, cache, idx_type, ids_dev, num_ids_dev, cap_ids, out_dev, out_stride,
                           stats_dev, phases, static_cast<hipStream_t>(stream));
}

int mqg_gather_features(mqg_ctx *ctx, const mqg_cache *cache, int32_t idx_type, const void *ids_dev,
                        const int64_t *num_ids_dev, int64_t cap_ids, void *out_dev, int64_t out_stride,
                        int64_t *stats_dev, mqg_stream stream) {
    return gather_checked(ctx, cache, idx_type, ids_dev, num_ids_dev, cap_ids, out_dev, out_stride, stats_dev,
                          mqg::kGatherCached | mqg::kGatherMissed, stream);
}

int mqg_gather_features_cached(mqg_ctx *ctx, const mqg_cache *cache, int32_t idx_type, const void *ids_dev,
                               const int64_t *num_ids_dev, int64_t cap_ids, void *out_dev, int64_t out_stride,
                               int64_t *stats_dev, mqg_stream stream) {
    return gather_checked(ctx, cache, idx_type, ids_dev, num_ids_dev, cap_ids, out_dev, out_stride, stats_dev,
                          mqg::kGatherCached, stream);
}

int mqg_gather_features_missed(mqg_ctx *ctx, const mqg_cache *cache, int32_t idx_type, const void *ids_dev,
                               const int64_t *num_ids_dev, int64_t cap_ids, void *out_dev, int64_t out_stride,
                               int64_t *stats_dev, mqg_stream stream) {
    return gather_checked(ctx, cache, idx_type, ids_dev, num_ids_dev, cap_ids, out_dev, out_stride, stats_dev,
                          mqg::kGatherMissed, stream);
}

int mqg_sage_mean_aggregate(mqg_ctx *ctx, const mqg_block *block, const void *x_src, int64_t x_stride,
                            void *out, int64_t out_stride, int32_t dim, int32_t dtype, mqg_stream stream) {
    if (!ctx) return MQG_ERR_INVALID_ARG;
    if (!block || !block->indptr || !block->indices || !block->sizes)
        return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_sage_mean_aggregate: NULL block buffers");
    if (!valid_dtype(dtype) || dim < 1) return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_sage_mean_aggregate: bad dtype or dim");
    if (block->cap_dst < 0) return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_sage_mean_aggregate: negative cap_dst");
    if (block->cap_dst > 0 && (!x_src || !out)) return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_sage_mean_aggregate: NULL x_src or out");
    if (x_stride < dim || out_stride < dim) return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_sage_mean_aggregate: stride below dim");
    return mqg::run_mean_aggregate(ctx, block, x_src, x_stride, out, out_stride, dim, dtype,
                                   static_cast<hipStream_t>(stream));
}

int mqg_sage_mean_aggregate_backward(mqg_ctx *ctx, const mqg_block *block, const void *grad_out, int64_t go_stride,
                                     void *grad_x, int64_t gx_stride, int32_t dim, int32_t dtype, mqg_stream stream) {
    if (!ctx) return MQG_ERR_INVALID_ARG;
    if (!block || !block->indptr || !block->indices || !block->sizes)
        return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_sage_mean_aggregate_backward: NULL block buffers");
    if (!valid_dtype(dtype) || dim < 1) return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_sage_mean_aggregate_backward: bad dtype or dim");
    if (block->cap_dst < 0 || block->cap_src < 0 || block->cap_nnz < 0 || block->cap_nnz >= (int64_t(1) << 31))
        return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_sage_mean_aggregate_backward: bad block capacities");
    if (block->cap_src > 0 && (!grad_out || !grad_x)) return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_sage_mean_aggregate_backward: NULL grad_out or grad_x");
    if (go_stride < dim || gx_stride < dim) return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_sage_mean_aggregate_backward: stride below dim");
    return mqg::run_aggregate_backward(ctx, block, nullptr, nullptr, grad_out, go_stride, grad_x, gx_stride, dim, dtype,
                                       static_cast<hipStream_t>(stream));
}

int mqg_gcn_edge_weights(mqg_ctx *ctx, const mqg_graph *graph, const mqg_block *block, float *edge_w, float *self_w,
                         mqg_stream stream) {
    if (!ctx) return MQG_ERR_INVALID_ARG;
    int rc = check_graph(ctx, graph, "mqg_gcn_edge_weights");
    if (rc != MQG_OK) return rc;
    if (!block || !block->indptr || !block->indices || !block->sizes || !block->src_ids)
        return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_gcn_edge_weights: NULL block buffers");
    if (block->cap_dst < 0) return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_gcn_edge_weights: negative cap_dst");
    if (!edge_w || !self_w) return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_gcn_edge_weights: NULL edge_w or self_w");
    return mqg::run_gcn_edge_weights(ctx, graph, block, edge_w, self_w, static_cast<hipStream_t>(stream));
}

int mqg_weighted_aggregate(mqg_ctx *ctx, const mqg_block *block, const float *edge_w, const float *self_w, const void *x_src,
                           int64_t x_stride, void *out, int64_t out_stride, int32_t dim, int32_t dtype, mqg_stream stream) {
    if (!ctx) return MQG_ERR_INVALID_ARG;
    if (!block || !block->indptr || !block->indices || !block->sizes)
        return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_weighted_aggregate: NULL block buffers");
    if (!edge_w) return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_weighted_aggregate: NULL edge_w");
    if (!valid_dtype(dtype) || dim < 1) return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_weighted_aggregate: bad dtype or dim");
    if (block->cap_dst < 0) return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_weighted_aggregate: negative cap_dst");
    if (block->cap_dst > 0 && (!x_src || !out)) return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_weighted_aggregate: NULL x_src or out");
    if (x_stride < dim || out_stride < dim) return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_weighted_aggregate: stride below dim");
    return mqg::run_weighted_aggregate(ctx, block, edge_w, self_w, x_src, x_stride, out, out_stride, dim, dtype,
                                       static_cast<hipStream_t>(stream));
}

int mqg_weighted_aggregate_backward(mqg_ctx *ctx, const mqg_block *block, const float *edge_w, const float *self_w,
                                    const void *grad_out, int64_t go_stride, void *grad_x, int64_t gx_stride, int32_t dim,
                                    int32_t dtype, mqg_stream stream) {
    if (!ctx) return MQG_ERR_INVALID_ARG;
    if (!block || !block->indptr || !block->indices || !block->sizes)
        return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_weighted_aggregate_backward: NULL block buffers");
    if (!edge_w) return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_weighted_aggregate_backward: NULL edge_w");
    if (!valid_dtype(dtype) || dim < 1) return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_weighted_aggregate_backward: bad dtype or dim");
    if (block->cap_dst < 0 || block->cap_src < 0 || block->cap_nnz < 0 || block->cap_nnz >= (int64_t(1) << 31))
        return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_weighted_aggregate_backward: bad block capacities");
    if (block->cap_src > 0 && (!grad_out || !grad_x))
        return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_weighted_aggregate_backward: NULL grad_out or grad_x");
    if (go_stride < dim || gx_stride < dim) return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_weighted_aggregate_backward: stride below dim");
    return mqg::run_aggregate_backward(ctx, block, edge_w, self_w, grad_out, go_stride, grad_x, gx_stride, dim, dtype,
                                       static_cast<hipStream_t>(stream));
}

int mqg_queue_size(double max_prepare_ms, double mean_compute_ms, int64_t total_mem_bytes, int64_t peak_mem_bytes,
                   int32_t margin_percent, int64_t mem_per_batch_bytes, int64_t *cap_out, int64_t *queue_size_out) {
    if (!queue_size_out) return MQG_ERR_INVALID_ARG;
    if (!(max_prepare_ms > 0.0) || !(mean_compute_ms > 0.0) || total_mem_bytes <= 0 || peak_mem_bytes < 0 ||
        mem_per_batch_bytes <= 0 || margin_percent < 0 || margin_percent > 100)
        return fail(nullptr, MQG_ERR_INVALID_ARG, "mqg_queue_size: non-positive time or size, or margin outside 0..100");
    // peak * (1 + margin/100) in integers, rounded up so that the margin is never short
    const int64_t reserved = peak_mem_bytes + (peak_mem_bytes / 100) * margin_percent +
                             ((peak_mem_bytes % 100) * margin_percent + 99) / 100;
    if (reserved > total_mem_bytes) return fail(nullptr, MQG_ERR_INVALID_ARG, "mqg_queue_size: peak memory (with margin) above the total");
    const int64_t cap = (total_mem_bytes - reserved) / mem_per_batch_bytes;
    const double ratio = std::ceil(max_prepare_ms / mean_compute_ms);
    int64_t want = ratio >= 9.0e18 ? INT64_MAX : static_cast<int64_t>(ratio);
    if (want < 2) want = 2;
    if (cap_out) *cap_out = cap;
    *queue_size_out = std::min(cap, want);
    return MQG_OK;
}

}  // extern "C"
