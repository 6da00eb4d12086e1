// Internal declarations shared by the library's translation units (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>
#include <vector>

#include "mqg.h"

namespace mqg {

constexpr int kWave = 64;                // CDNA wavefront width
constexpr int kBlock = 256;              // default workgroup: 4 wavefronts
constexpr int kWavesPerBlock = kBlock / kWave;
constexpr int kBitmapTileWords = 1024;   // the frontier bitmap is padded to a multiple of this many words
constexpr int kCandidates = 256;         // per-wavefront candidate slots of the threshold selection

// Ping-pong buffers of the radix sort (see radix.h)
struct RadixBufs {
    uint32_t *keys[2] = {nullptr, nullptr};     // [n_cap] each
    int32_t *vals[2] = {nullptr, nullptr};      // [n_cap] each
    int32_t *hist = nullptr;                    // [radix_hist_len(n_cap)]
    int32_t *tile_sums = nullptr;               // [radix_scan_tiles(n_cap)]
};

struct ProfRec {
    int name_id;
    hipEvent_t start, stop;
};

}  // namespace mqg

// scratch of the layer-wise sampler (layerwise.hip), sized by the graph
struct LayerwiseScratch {
    unsigned long long *mass = nullptr;  // [num_nodes] integer column masses, zero between calls
    int32_t *cand = nullptr;             // [num_nodes] candidates, ascending
    uint64_t *key64 = nullptr;           // [num_nodes] race keys (double bit patterns)
    uint64_t *bkey = nullptr;            // [num_nodes] keys that share the threshold's leading bits ...
    int32_t *bpos = nullptr;             // ... and their positions
    uint64_t *xkey = nullptr;            // the same for a selection on its own over more keys than the graph has nodes
    int32_t *xpos = nullptr;
    int64_t xcap = 0;
    unsigned long long *sel_state = nullptr;   // [18] radix select: prefix and wanted count per pass
    int32_t *sel_hist = nullptr;         // [passes][digits] counts of the radix select
    int32_t *chunk_offs = nullptr;       // [rows_cap * 16 + 1] edges per (row, chunk), then their scan
    int32_t *chunk_scan = nullptr;       // the scan of a small chunk_offs table (one-launch scan, out of place)
    double *chunk_sum = nullptr;         // [rows_cap * 16] raw weight sums per (row, chunk)
    int32_t *word_offs = nullptr;        // [bitmap_words + 1] set bits per tile of the bitmap
    int32_t *scan_tiles = nullptr;
    double *q_part = nullptr;            // per-workgroup partial sums of q
    int64_t *counters = nullptr;         // [0]: number of candidates, [1]: keys of a selection on its own, [2]: nodes, [3]: boundary keys
    double *q_total = nullptr;
    int64_t *seeds_copy = nullptr;       // [rows_cap] the checked seeds
    int32_t *flags = nullptr;
    uint64_t *dkey = nullptr;            // [rows_cap] race keys of the drawn nodes (debiased coefficients)
    double *dq = nullptr, *beta = nullptr;
    int32_t *order = nullptr;            // [rows_cap] source positions in draw order
    unsigned long long *fg_mass = nullptr;     // [num_nodes] masses over all rows of the graph (FastGCN)
    bool fg_ready = false;
    int64_t rows_cap = 0;
};

struct mqg_ctx {
    int device = 0;
    int64_t num_nodes = 0;
    int32_t ptr_type = 0, idx_type = 0;
    int32_t max_seeds = 0, num_layers = 0;
    int32_t max_fanouts[MQG_MAX_LAYERS] = {0};
    int64_t bound_dst[MQG_MAX_LAYERS] = {0};   // worst-case sizes per block for this context
    int64_t bound_src[MQG_MAX_LAYERS] = {0};
    int64_t bound_nnz[MQG_MAX_LAYERS] = {0};
    int64_t max_dst = 0, max_src = 0, max_nnz = 0;

    // scratch (device)
    int32_t *local_of = nullptr;         // [num_nodes] position of a node in the current source list, -1 if absent
    uint32_t *bitmap = nullptr;          // [bitmap_words] nodes first seen in the current layer
    int64_t bitmap_words = 0;            // padded to a multiple of kBitmapTileWords
    int32_t *tile_vals = nullptr;        // [max_tiles] per-tile sums of the rows, then their exclusive scan
    int32_t *bitmap_tile_vals = nullptr; // [max_tiles] the same for the tiles of the bitmap
    int64_t max_tiles = 0;
    int64_t *row_start = nullptr;        // [max_dst] first adjacency slot of each destination
    int32_t *row_deg = nullptr;          // [max_dst] degree of each destination
    void *nbr = nullptr;                 // [max_nnz] sampled neighbours, global ids, 32-bit
    int32_t *heavy_rows = nullptr;       // [max_dst] destinations whose degree exceeds heavy_degree
    int32_t *heavy_count = nullptr;      // [MQG_MAX_LAYERS] their number, per block; [MQG_MAX_LAYERS] seed-check flags
    int2 *hit_list = nullptr;            // [max_src] (output row, cache slot)
    int2 *miss_list = nullptr;           // [max_src] (output row, node id)
    unsigned long long *counters = nullptr;  // [8] hits, misses, finished workgroups of the miss launch; zero between gathers
    // backward aggregation: edges ordered by source; allocated at the first backward call
    mqg::RadixBufs bwd;
    int32_t *bwd_dst_row = nullptr;      // [bwd_nnz_cap] destination row of every edge
    float *bwd_w_sorted = nullptr;       // [bwd_nnz_cap] edge weights in the by-source order (weighted backward)
    int32_t *bwd_col_ptr = nullptr;      // [bwd_src_cap + 2] offsets of every source in the sorted edge list
    int64_t bwd_nnz_cap = 0, bwd_src_cap = 0;
    LayerwiseScratch lw;
    // cache-prioritised neighbour sampling (mqg_ctx_set_sampling_priority)
    bool prio_enabled = false;
    uint32_t *prio_bitmap = nullptr;     // [bitmap_words] bit v = node v is cached
    int32_t *prio_count = nullptr;       // [num_nodes] number of cached neighbours of every node
    // temporaries of the cache build, reserved by mqg_ctx_reserve (otherwise allocated and freed per call)
    char *cache_arena = nullptr;
    int64_t cache_arena_bytes = 0;
    // hash-table dedup (MQG_OPT_DEDUP_HASH); allocated when the option is first used
    bool dedup_hash = false;
    unsigned long long *hash_table = nullptr;      // [hash_capacity] (id << 32 | position), all ones = empty
    int64_t hash_capacity = 0;
    uint32_t *hash_new_keys = nullptr;             // [max_nnz] ids first seen in the current block
    unsigned long long *hash_new_count = nullptr;  // their number
    mqg::RadixBufs hash_sort;

    // options
    bool force_slow_select = false;
    int layerwise_candidates = 0;        // MQG_OPT_LAYERWISE_CANDIDATES
    bool profile = false;
    int64_t miss_inflight_bytes = 1024 * 1024;  // read bytes the host-link gather keeps outstanding
    int heavy_degree = 2048;             // rows longer than this get a whole workgroup in sampling

    // profiling
    std::vector<std::string> prof_names;
    std::vector<mqg::ProfRec> prof_recs;
    std::vector<hipEvent_t> event_pool;
    std::vector<double> prof_total_ms;
    std::vector<int64_t> prof_launches;

    std::string last_error;
};

namespace mqg {

int fail(mqg_ctx *ctx, int code, const std::string &msg);
int prof_name_id(mqg_ctx *ctx, const char *name);
void prof_begin(mqg_ctx *ctx, const char *name, hipStream_t s);
void prof_end(mqg_ctx *ctx, hipStream_t s);
void prof_begin_ext(mqg_ctx *ctx, const char *name, hipEvent_t *start, hipEvent_t *stop);

// Launch wrapper: optional event bracketing, error check.  Usage:
//   MQG_LAUNCH(ctx, "k_name", stream, (k_name<<<grid, block, 0, stream>>>(args...)));
#define MQG_LAUNCH(ctx, name, stream, launch_expr)                                  \
    do {                                                                            \
        if ((ctx)->profile) mqg::prof_begin((ctx), (name), (stream));               \
        launch_expr;                                                                \
        if ((ctx)->profile) mqg::prof_end((ctx), (stream));                         \
        hipError_t _e = hipGetLastError();                                          \
        if (_e != hipSuccess)                                                       \
            return mqg::fail((ctx), MQG_ERR_HIP,                                    \
                             std::string(name) + ": " + hipGetErrorString(_e));     \
    } while (0)

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// ---- steps implemented in the other translation units ----------------------------------
int run_sample_blocks(mqg_ctx *ctx, const mqg_graph *g, const void *seeds, int32_t num_seeds, const int32_t *fanouts,
                      int32_t L, uint64_t rng_seed, const uint64_t *seed_dev, mqg_block *blocks, hipStream_t s);
constexpr int kGatherCached = 1, kGatherMissed = 2;   // the two halves of a gather
int run_gather(mqg_ctx *ctx, const mqg_cache *c, int32_t idx_type, const void *ids,
               const int64_t *num_ids, int64_t cap_ids, void *out, int64_t out_stride,
               int64_t *stats, int phases, hipStream_t s);
int check_gather_args(mqg_ctx *ctx, const mqg_cache *cache, int32_t idx_type, const void *ids_dev,
                      const int64_t *num_ids_dev, int64_t cap_ids, const void *out_dev, int64_t out_stride,
                      int64_t max_ids, const char *what_max);
int run_mean_aggregate(mqg_ctx *ctx, const mqg_block *b, const void *x, int64_t x_stride, void *out,
                       int64_t out_stride, int32_t dim, int32_t dtype, hipStream_t s);
int run_build_cache(mqg_ctx *ctx, const mqg_graph *g, mqg_cache *c, const mqg_cache_plan *plan, hipStream_t s);
int run_aggregate_backward(mqg_ctx *ctx, const mqg_block *b, const float *edge_w, const float *self_w, const void *grad_out,
                           int64_t go_stride, void *grad_x, int64_t gx_stride, int32_t dim, int32_t dtype, hipStream_t s);
int run_gcn_edge_weights(mqg_ctx *ctx, const mqg_graph *g, const mqg_block *b, float *edge_w, float *self_w, hipStream_t s);
int run_weighted_aggregate(mqg_ctx *ctx, const mqg_block *b, const float *edge_w, const float *self_w, const void *x,
                           int64_t x_stride, void *out, int64_t out_stride, int32_t dim, int32_t dtype, hipStream_t s);
void free_backward_scratch(mqg_ctx *ctx);
int ensure_backward_scratch(mqg_ctx *ctx, int64_t nnz_cap, int64_t src_cap, hipStream_t s, const char *who);
int ensure_layerwise_scratch(mqg_ctx *ctx, int64_t rows_cap, hipStream_t s);
int ensure_priority_scratch(mqg_ctx *ctx);
int ensure_cache_build_scratch(mqg_ctx *ctx);
int run_sample_layerwise(mqg_ctx *ctx, const mqg_graph *g, const void *seeds, int32_t num_seeds, const int32_t *layer_sizes,
                         int32_t L, uint64_t rng_seed, int32_t normalise, int32_t method, mqg_block *blocks,
                         float *const *edge_w, hipStream_t s);
void free_layerwise_scratch(mqg_ctx *ctx);
int run_select_smallest_keys(mqg_ctx *ctx, const uint64_t *keys, int64_t n, int64_t k, uint32_t *out_bitmap, hipStream_t s);
int run_select_row_candidates(mqg_ctx *ctx, const uint64_t *keys, const uint32_t *slot_words, int32_t cnt, int32_t k,
                              int32_t prioritised, int32_t ordered, uint32_t *out_mask, hipStream_t s);
int run_exp_tickets(mqg_ctx *ctx, uint64_t seed, int64_t tag, int64_t first, int64_t n, uint64_t *tickets, hipStream_t s);
int run_set_sampling_priority(mqg_ctx *ctx, const mqg_graph *g, const mqg_cache *cache, hipStream_t s);
// hash-table dedup (dedup_hash.hip)
int ensure_hash_scratch(mqg_ctx *ctx);
void free_hash_scratch(mqg_ctx *ctx);
int hash_put_seeds(mqg_ctx *ctx, const void *seeds, int idx_type, int64_t need_dst, const int64_t *sizes, hipStream_t s);
int hash_dedup_block(mqg_ctx *ctx, const int32_t *nbr, int64_t need_nnz, int64_t num_nodes, int idx_type, void *src_ids,
                     int64_t *sizes, int64_t *sizes_next, int32_t *indices, hipStream_t s);
int hash_clear(mqg_ctx *ctx, hipStream_t s);

// Exclusive scan of vals[0..n) in place by one workgroup; the total (plus *addend if given) is
// stored to *total_a and *total_b where non-null.
int launch_scan_tiles(mqg_ctx *ctx, int32_t *vals, int64_t n, const int64_t *addend,
                      int64_t *total_a, int64_t *total_b, hipStream_t s, const char *name = "k_scan_tiles");

}  // namespace mqg
