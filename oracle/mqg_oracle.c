/*
 * CPU oracle for mini-batch generation in sampled GNN training.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, single-threaded,
 * plainly written statement of what the GPU library must compute.  It is
 * used by the tests, by the smoke check and by the benchmark's CPU-baseline
 * leg; no product code path may call it.  It shares no code, header, table
 * or helper with the GPU implementation.
 *
 * All node ids, offsets and counts are int64 here; every floating-point
 * reduction is carried out in double.
 *
 * What each function follows in the paper (MQ-GNN):
 *   - orc_build_cache      : Sec. III "Feature Cache" (node cache C of
 *                            high-degree nodes whose features are preloaded
 *                            on the GPU; Eq. 13 ranks by in-degree).  Read
 *                            deterministically: the num_cached nodes of
 *                            highest degree, ties to the lower id.
 *   - orc_build_cache_sampled : the same section, Eq. 13 read as the paper
 *                            states it: cache membership is *drawn* with
 *                            probability proportional to in-degree (weighted
 *                            sampling without replacement, redrawn per epoch).
 *   - orc_random_walk_scores / orc_build_cache_by_score : Eq. 14-15, the
 *                            short-random-walk probabilities P^(L) used when
 *                            the training set is a small part of the graph;
 *                            Eq. 15 as printed, and the same matrix applied
 *                            along the direction in which sampling moves.
 *   - orc_exp_ticket / orc_build_cache_drawn_by_score : the text after
 *                            Eq. 15 takes P^(L) as the probability with
 *                            which the cache is sampled; taken literally:
 *                            membership
 *                            is drawn with probability proportional to the
 *                            score, by weighted sampling with random keys
 *                            (Efraimidis and Spirakis, cited in Sec. III-B).
 *   - orc_sample_blocks    : Sec. III-A "Node-wise Sampling", GraphSAGE
 *                            paragraph: for every node of a layer a fixed
 *                            number s_node of its neighbours is drawn
 *                            uniformly at random; the sampled set carries a
 *                            layer superscript (text after Eq. 3), so a node
 *                            is re-sampled in every layer it appears in.
 *                            Sec. IV "Mini-Batch Transfer": a mini-batch
 *                            carries topology and features.
 *   - orc_sample_block_prioritised : Sec. I on global neighbour sampling: the
 *                            sampler gives neighbours held in the cache
 *                            precedence, so that fewer distinct uncached
 *                            nodes enter a mini-batch.  Read as: a row's cached neighbours
 *                            are drawn before its uncached ones.  The paper
 *                            prints no rule, so this function is "parity
 *                            unpinned" against the paper; the reading itself
 *                            is pinned by its invariants.
 *   - orc_ladies_probabilities / orc_ladies_block : Sec. III-B "Layer-wise
 *                            sampling", LADIES paragraph (Eq. 6-9): the nodes
 *                            of the next layer are drawn from the neighbours
 *                            of the current layer's nodes with probability
 *                            proportional to the squared column norm of the
 *                            row-selected normalised adjacency; a sampled
 *                            node's column is scaled by 1 / (s p).  The
 *                            "flat" variants (Sec. III-B "Calibrate and
 *                            Debias LS", Eq. 10) draw in proportion to the
 *                            column norm itself, not its square: the
 *                            variance of the sampled product P (H W) is
 *                            least for p_i proportional to |P_{*,i}| |(HW)_i|
 *                            and the row norms of H W are taken as uniform.
 *   - orc_gather           : Sec. IV "Mini-Batch Transfer To GPU": features
 *                            of nodes absent from the GPU cache come from
 *                            host memory, the rest from the cache; the
 *                            result is the feature rows of the block's
 *                            source nodes.
 *   - orc_mean_aggregate   : Eq. 16, Z_agg(v) = Mean(H(v)) over the sampled
 *                            neighbours of v (the GA step, "AH").
 *   - orc_gcn_edge_weights / orc_weighted_aggregate : Eq. 1-3, the sampled
 *                            estimator of the graph convolution P H with
 *                            P = D^-1/2 (A + I) D^-1/2 (Eq. 2): a sampled
 *                            neighbour j of v_i carries |N(v_i)|/s_node * P_ij
 *                            (Eq. 3).
 *   - orc_mean_aggregate_backward : Sec. IV "Computation", backward pass: the
 *                            gradient of the GA step is the transposed
 *                            product ("AG" with G the gradient matrix), here
 *                            the transpose of the row-mean operator.
 *
 * Randomness is a pure function of its coordinates: the key of slot j in
 * the adjacency row of node v at block l under seed s is
 *     key = mix(mix(mix(mix(s + GOLDEN) ^ l) ^ v) ^ j)
 * where mix is the 64-bit finaliser of the SplitMix64 generator (Steele,
 * Lea, Flood 2014).  A row of d > k entries keeps the k slots with the
 * smallest (key, slot) pairs - a uniform k-subset when keys are i.i.d.
 * uniform, the equal-weights case of sampling by random keys (Efraimidis
 * and Spirakis, cited by the paper in Sec. III-B).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_GOLDEN 0x9E3779B97F4A7C15ULL

uint64_t orc_mix(uint64_t z)
{
    z ^= z >> 30;
    z *= 0xBF58476D1CE4E5B9ULL;
    z ^= z >> 27;
    z *= 0x94D049BB133111EBULL;
    z ^= z >> 31;
    return z;
}

uint64_t orc_key(uint64_t rng_seed, int64_t layer, int64_t node, int64_t slot)
{
    uint64_t h = orc_mix(rng_seed + ORC_GOLDEN);
    h = orc_mix(h ^ (uint64_t)layer);
    h = orc_mix(h ^ (uint64_t)node);
    return orc_mix(h ^ (uint64_t)slot);
}

/* ---------------------------------------------------------------- cache */

typedef struct { int64_t deg; int64_t id; } orc_deg_id;

static int cmp_deg_desc_id_asc(const void *a, const void *b)
{
    const orc_deg_id *x = a, *y = b;
    if (x->deg != y->deg) return x->deg > y->deg ? -1 : 1;
    if (x->id != y->id) return x->id < y->id ? -1 : 1;
    return 0;
}

/* Rank all nodes by (degree descending, id ascending); the first num_cached
 * are cached, slot s holding the s-th ranked node.  slot_of[v] = s or -1. */
int orc_build_cache(int64_t num_nodes, const int64_t *row_ptr, int64_t num_cached,
                    int64_t *cached_ids, int32_t *slot_of)
{
    if (num_cached < 0 || num_cached > num_nodes) return -1;
    orc_deg_id *all = malloc((size_t)(num_nodes > 0 ? num_nodes : 1) * sizeof *all);
    if (!all) return -2;
    for (int64_t v = 0; v < num_nodes; ++v) {
        all[v].deg = row_ptr[v + 1] - row_ptr[v];
        all[v].id = v;
    }
    qsort(all, (size_t)num_nodes, sizeof *all, cmp_deg_desc_id_asc);
    for (int64_t v = 0; v < num_nodes; ++v) slot_of[v] = -1;
    for (int64_t s = 0; s < num_cached; ++s) {
        cached_ids[s] = all[s].id;
        slot_of[all[s].id] = (int32_t)s;
    }
    free(all);
    return 0;
}

/* cache_rows[s] = feats[cached_ids[s]] as bytes */
void orc_fill_cache_rows(const int64_t *cached_ids, int64_t num_cached, const uint8_t *feats,
                         int64_t feat_stride_bytes, int64_t row_bytes, uint8_t *cache_rows,
                         int64_t cache_stride_bytes)
{
    for (int64_t s = 0; s < num_cached; ++s)
        memcpy(cache_rows + s * cache_stride_bytes, feats + cached_ids[s] * feat_stride_bytes,
               (size_t)row_bytes);
}

/* ------------------------------------------------------------- sampling */

typedef struct { uint64_t key; int64_t slot; } orc_key_slot;

static int cmp_key_slot(const void *a, const void *b)
{
    const orc_key_slot *x = a, *y = b;
    if (x->key != y->key) return x->key < y->key ? -1 : 1;
    if (x->slot != y->slot) return x->slot < y->slot ? -1 : 1;
    return 0;
}

static int cmp_i64(const void *a, const void *b)
{
    int64_t x = *(const int64_t *)a, y = *(const int64_t *)b;
    return x < y ? -1 : (x > y ? 1 : 0);
}

/* Chosen slots of one adjacency row of length d, ascending; returns their
 * number min(k, d).  out_slots has room for k entries. */
int64_t orc_sample_row(uint64_t rng_seed, int64_t layer, int64_t node, int64_t d, int64_t k,
                       int64_t *out_slots)
{
    if (d <= k) {
        for (int64_t j = 0; j < d; ++j) out_slots[j] = j;
        return d;
    }
    orc_key_slot *ks = malloc((size_t)d * sizeof *ks);
    for (int64_t j = 0; j < d; ++j) {
        ks[j].key = orc_key(rng_seed, layer, node, j);
        ks[j].slot = j;
    }
    qsort(ks, (size_t)d, sizeof *ks, cmp_key_slot);
    for (int64_t j = 0; j < k; ++j) out_slots[j] = ks[j].slot;
    free(ks);
    qsort(out_slots, (size_t)k, sizeof *out_slots, cmp_i64);
    return k;
}

typedef struct { int uncached; uint64_t key; int64_t slot; } orc_prio_key_slot;

static int cmp_prio_key_slot(const void *a, const void *b)
{
    const orc_prio_key_slot *x = a, *y = b;
    if (x->uncached != y->uncached) return x->uncached < y->uncached ? -1 : 1;
    if (x->key != y->key) return x->key < y->key ? -1 : 1;
    if (x->slot != y->slot) return x->slot < y->slot ? -1 : 1;
    return 0;
}

/*
 * Cache-prioritised choice for one adjacency row nbrs[0..d): as orc_sample_row,
 * but the k slots are the first k in the order (not cached, key, slot) - every
 * cached neighbour (slot_of >= 0) goes before every uncached one, and within
 * each class the draw is the uniform one.  With c cached neighbours the row
 * keeps min(k, c) of them, uniformly, and fills up with k - c uncached ones,
 * uniformly.  Chosen slots ascending; returns min(k, d).
 */
int64_t orc_sample_row_prioritised(uint64_t rng_seed, int64_t layer, int64_t node, int64_t d, int64_t k,
                                   const int64_t *nbrs, const int32_t *slot_of, int64_t *out_slots)
{
    if (d <= k) {
        for (int64_t j = 0; j < d; ++j) out_slots[j] = j;
        return d;
    }
    orc_prio_key_slot *ks = malloc((size_t)d * sizeof *ks);
    for (int64_t j = 0; j < d; ++j) {
        ks[j].uncached = slot_of[nbrs[j]] < 0;
        ks[j].key = orc_key(rng_seed, layer, node, j);
        ks[j].slot = j;
    }
    qsort(ks, (size_t)d, sizeof *ks, cmp_prio_key_slot);
    for (int64_t j = 0; j < k; ++j) out_slots[j] = ks[j].slot;
    free(ks);
    qsort(out_slots, (size_t)k, sizeof *out_slots, cmp_i64);
    return k;
}

typedef struct { int64_t id; int64_t pos; } orc_id_pos;

static int cmp_id_pos(const void *a, const void *b)
{
    const orc_id_pos *x = a, *y = b;
    if (x->id != y->id) return x->id < y->id ? -1 : 1;
    return x->pos < y->pos ? -1 : (x->pos > y->pos ? 1 : 0);
}

/* position of id in a sorted orc_id_pos array, or -1 */
static int64_t find_id(const orc_id_pos *a, int64_t n, int64_t id)
{
    int64_t lo = 0, hi = n;
    while (lo < hi) {
        int64_t mid = lo + (hi - lo) / 2;
        if (a[mid].id < id) lo = mid + 1; else hi = mid;
    }
    return (lo < n && a[lo].id == id) ? lo : -1;
}

static int64_t find_i64(const int64_t *a, int64_t n, int64_t x)
{
    int64_t lo = 0, hi = n;
    while (lo < hi) {
        int64_t mid = lo + (hi - lo) / 2;
        if (a[mid] < x) lo = mid + 1; else hi = mid;
    }
    return (lo < n && a[lo] == x) ? lo : -1;
}

/*
 * One block: destination nodes dst[0..num_dst) with fanout k at block index
 * `layer`.  Outputs:
 *   indptr[num_dst+1]   running count of sampled neighbours per destination
 *   nbr[nnz]            sampled neighbours (global ids), rows in destination
 *                       order, within a row in ascending adjacency slot
 *   src[num_src]        dst, followed by the sampled neighbours that are not
 *                       in dst, each once, ascending
 *   indices[nnz]        position of nbr[e] in src
 * Returns num_src, or a negative value on capacity overflow / no memory.
 */
static int64_t sample_block(const int64_t *row_ptr, const int64_t *col_idx, const int64_t *dst,
                            int64_t num_dst, int64_t k, int64_t layer, uint64_t rng_seed,
                            int64_t cap_nnz, int64_t cap_src, int64_t *indptr, int64_t *nbr,
                            int64_t *src, int32_t *indices, const int32_t *prio_slot_of);

int64_t orc_sample_block(const int64_t *row_ptr, const int64_t *col_idx, const int64_t *dst,
                         int64_t num_dst, int64_t k, int64_t layer, uint64_t rng_seed,
                         int64_t cap_nnz, int64_t cap_src, int64_t *indptr, int64_t *nbr,
                         int64_t *src, int32_t *indices)
{
    return sample_block(row_ptr, col_idx, dst, num_dst, k, layer, rng_seed, cap_nnz, cap_src, indptr, nbr,
                        src, indices, NULL);
}

/* The same block with every row drawn by orc_sample_row_prioritised against the cache table slot_of. */
int64_t orc_sample_block_prioritised(const int64_t *row_ptr, const int64_t *col_idx, const int64_t *dst,
                                     int64_t num_dst, int64_t k, int64_t layer, uint64_t rng_seed,
                                     int64_t cap_nnz, int64_t cap_src, int64_t *indptr, int64_t *nbr,
                                     int64_t *src, int32_t *indices, const int32_t *slot_of)
{
    return sample_block(row_ptr, col_idx, dst, num_dst, k, layer, rng_seed, cap_nnz, cap_src, indptr, nbr,
                        src, indices, slot_of);
}

static int64_t sample_block(const int64_t *row_ptr, const int64_t *col_idx, const int64_t *dst,
                            int64_t num_dst, int64_t k, int64_t layer, uint64_t rng_seed,
                            int64_t cap_nnz, int64_t cap_src, int64_t *indptr, int64_t *nbr,
                            int64_t *src, int32_t *indices, const int32_t *prio_slot_of)
{
    int64_t *slots = malloc((size_t)(k > 0 ? k : 1) * sizeof *slots);
    int64_t nnz = 0;
    indptr[0] = 0;
    for (int64_t i = 0; i < num_dst; ++i) {
        int64_t v = dst[i];
        int64_t start = row_ptr[v], d = row_ptr[v + 1] - start;
        int64_t c = prio_slot_of
                        ? orc_sample_row_prioritised(rng_seed, layer, v, d, k, col_idx + start, prio_slot_of, slots)
                        : orc_sample_row(rng_seed, layer, v, d, k, slots);
        if (nnz + c > cap_nnz) { free(slots); return -2; }
        for (int64_t j = 0; j < c; ++j) nbr[nnz + j] = col_idx[start + slots[j]];
        nnz += c;
        indptr[i + 1] = nnz;
    }
    free(slots);

    /* destination nodes sorted by id, remembering their position */
    orc_id_pos *dsorted = malloc((size_t)(num_dst > 0 ? num_dst : 1) * sizeof *dsorted);
    for (int64_t i = 0; i < num_dst; ++i) { dsorted[i].id = dst[i]; dsorted[i].pos = i; }
    qsort(dsorted, (size_t)num_dst, sizeof *dsorted, cmp_id_pos);

    /* the set of sampled neighbours, ascending, minus the destinations */
    int64_t *uniq = malloc((size_t)(nnz > 0 ? nnz : 1) * sizeof *uniq);
    memcpy(uniq, nbr, (size_t)nnz * sizeof *uniq);
    qsort(uniq, (size_t)nnz, sizeof *uniq, cmp_i64);
    int64_t num_new = 0;
    for (int64_t e = 0; e < nnz; ++e) {
        if (e > 0 && uniq[e] == uniq[e - 1]) continue;
        if (find_id(dsorted, num_dst, uniq[e]) >= 0) continue;
        uniq[num_new++] = uniq[e];
    }
    if (num_dst + num_new > cap_src) { free(uniq); free(dsorted); return -2; }
    for (int64_t i = 0; i < num_dst; ++i) src[i] = dst[i];
    for (int64_t r = 0; r < num_new; ++r) src[num_dst + r] = uniq[r];

    for (int64_t e = 0; e < nnz; ++e) {
        int64_t p = find_id(dsorted, num_dst, nbr[e]);
        if (p >= 0) {
            indices[e] = (int32_t)dsorted[p].pos;
        } else {
            int64_t r = find_i64(uniq, num_new, nbr[e]);
            indices[e] = (int32_t)(num_dst + r);
        }
    }
    free(uniq);
    free(dsorted);
    return num_dst + num_new;
}

/* ---------------------------------------------------------------- gather */

/* out[i] = F[ids[i]] byte for byte.  A row with slot_of[id] >= 0 is read
 * from cache_rows (a hit), otherwise from feats (a miss).  slot_of may be
 * NULL: then every row is read from feats and counted as a miss. */
void orc_gather(const int64_t *ids, int64_t n, const uint8_t *feats, int64_t feat_stride_bytes,
                const int32_t *slot_of, const uint8_t *cache_rows, int64_t cache_stride_bytes,
                int64_t row_bytes, uint8_t *out, int64_t out_stride_bytes, int64_t *hits,
                int64_t *misses)
{
    int64_t h = 0, m = 0;
    for (int64_t i = 0; i < n; ++i) {
        int64_t id = ids[i];
        const uint8_t *srcrow;
        if (slot_of && slot_of[id] >= 0) {
            srcrow = cache_rows + (int64_t)slot_of[id] * cache_stride_bytes;
            ++h;
        } else {
            srcrow = feats + id * feat_stride_bytes;
            ++m;
        }
        memcpy(out + i * out_stride_bytes, srcrow, (size_t)row_bytes);
    }
    *hits = h;
    *misses = m;
}

/* --------------------------------------------------------- fp16 helpers */

/* IEEE 754 binary16 -> double, exact */
double orc_half_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1F;
    int m = h & 0x3FF;
    double v;
    if (e == 0) {
        v = (double)m * (1.0 / 16777216.0);            /* m * 2^-24 (subnormal or zero) */
    } else if (e == 31) {
        if (m == 0) { union { uint64_t u; double d; } inf = { 0x7FF0000000000000ULL }; v = inf.d; }
        else { union { uint64_t u; double d; } nan = { 0x7FF8000000000000ULL }; v = nan.d; }
    } else {
        double scale = 1.0;
        int p = e - 15;
        if (p >= 0) for (int i = 0; i < p; ++i) scale *= 2.0;
        else for (int i = 0; i < -p; ++i) scale *= 0.5;
        v = (1.0 + (double)m / 1024.0) * scale;
    }
    return sign ? -v : v;
}

/* float -> IEEE 754 binary16, round to nearest, ties to even */
uint16_t orc_float_to_half(float f)
{
    union { float f; uint32_t u; } in = { f };
    uint32_t x = in.u;
    uint16_t sign = (uint16_t)((x >> 16) & 0x8000u);
    uint32_t expo = (x >> 23) & 0xFFu;
    uint32_t mant = x & 0x7FFFFFu;
    if (expo == 0xFFu) return (uint16_t)(sign | 0x7C00u | (mant ? 0x200u : 0u));
    int32_t e = (int32_t)expo - 127 + 15;
    if (e >= 31) return (uint16_t)(sign | 0x7C00u);                 /* overflow -> inf */
    if (e <= 0) {
        if (e < -10) return sign;                                   /* below half of min subnormal */
        mant |= 0x800000u;                                          /* implicit one */
        int shift = 14 - e;                                         /* 14..24 */
        uint32_t q = mant >> shift;
        uint32_t rem = mant & ((1u << shift) - 1u);
        uint32_t halfway = 1u << (shift - 1);
        if (rem > halfway || (rem == halfway && (q & 1u))) ++q;
        return (uint16_t)(sign | q);
    }
    uint32_t q = ((uint32_t)e << 10) | (mant >> 13);
    uint32_t rem = mant & 0x1FFFu;
    if (rem > 0x1000u || (rem == 0x1000u && (q & 1u))) ++q;         /* carry may reach inf: correct */
    return (uint16_t)(sign | q);
}

/* ------------------------------------------------------------ aggregate */

/*
 * out[i, :] = mean over e in [indptr[i], indptr[i+1]) of x[indices[e], :]
 * accumulated in double in row order, divided by the count, rounded once to
 * float (and then once to half for is_half).  An empty row gives zeros.
 * Strides are in elements.
 */
void orc_mean_aggregate(const int64_t *indptr, const int32_t *indices, int64_t num_dst,
                        const void *x, int64_t x_stride, void *out, int64_t out_stride,
                        int64_t dim, int is_half)
{
    double *acc = malloc((size_t)(dim > 0 ? dim : 1) * sizeof *acc);
    for (int64_t i = 0; i < num_dst; ++i) {
        int64_t b = indptr[i], e = indptr[i + 1], n = e - b;
        for (int64_t c = 0; c < dim; ++c) acc[c] = 0.0;
        for (int64_t p = b; p < e; ++p) {
            int64_t r = indices[p];
            if (is_half) {
                const uint16_t *row = (const uint16_t *)x + r * x_stride;
                for (int64_t c = 0; c < dim; ++c) acc[c] += orc_half_to_double(row[c]);
            } else {
                const float *row = (const float *)x + r * x_stride;
                for (int64_t c = 0; c < dim; ++c) acc[c] += (double)row[c];
            }
        }
        for (int64_t c = 0; c < dim; ++c) {
            double m = n > 0 ? acc[c] / (double)n : 0.0;
            if (is_half) ((uint16_t *)out)[i * out_stride + c] = orc_float_to_half((float)m);
            else ((float *)out)[i * out_stride + c] = (float)m;
        }
    }
    free(acc);
}

/*
 * Backward of the mean aggregation: with out = M x, M[i, s] = (number of edges
 * of row i that point to s) / n_i, this computes grad_x = M^T grad_out, i.e.
 *   grad_x[s, :] = sum over rows i and edges e of row i with indices[e] == s
 *                  of grad_out[i, :] / n_i,
 * accumulated in double in row order and rounded once to float (and then once
 * to half for is_half).  Sources without an incoming edge get zeros.
 */
int orc_mean_aggregate_backward(const int64_t *indptr, const int32_t *indices, int64_t num_dst,
                                int64_t num_src, const void *grad_out, int64_t go_stride,
                                void *grad_x, int64_t gx_stride, int64_t dim, int is_half)
{
    size_t total = (size_t)(num_src > 0 ? num_src : 1) * (size_t)(dim > 0 ? dim : 1);
    double *acc = calloc(total, sizeof *acc);
    if (!acc) return -2;
    for (int64_t i = 0; i < num_dst; ++i) {
        int64_t b = indptr[i], e = indptr[i + 1], n = e - b;
        for (int64_t p = b; p < e; ++p) {
            int64_t s = indices[p];
            for (int64_t c = 0; c < dim; ++c) {
                double g = is_half ? orc_half_to_double(((const uint16_t *)grad_out)[i * go_stride + c])
                                   : (double)((const float *)grad_out)[i * go_stride + c];
                acc[s * dim + c] += g / (double)n;
            }
        }
    }
    for (int64_t s = 0; s < num_src; ++s)
        for (int64_t c = 0; c < dim; ++c) {
            double v = acc[s * dim + c];
            if (is_half) ((uint16_t *)grad_x)[s * gx_stride + c] = orc_float_to_half((float)v);
            else ((float *)grad_x)[s * gx_stride + c] = (float)v;
        }
    free(acc);
    return 0;
}

/* ------------------------------------------------ weighted (GCN) aggregation */

/*
 * Weights of the sampled estimator of the graph convolution (Eq. 1-3).
 *
 * P = D^-1/2 (A + I) D^-1/2 with D_ii = deg(v_i) + 1 (Eq. 2), so for an edge
 * (v_i, v_j) of the graph P_ij = 1 / sqrt((deg(v_i)+1) (deg(v_j)+1)) and the
 * diagonal is P_ii = 1 / (deg(v_i)+1).  Eq. 3 scales a sampled neighbour's
 * entry by |N(v_i)| / s_node.
 *
 * Readings.  N(v_i) is the adjacency row of v_i (no self loop: rows hold
 * none), s_node is the number of neighbours actually drawn for v_i,
 * n_i = min(fanout, deg(v_i)) - so a row that was kept whole has factor 1 and
 * reproduces its row of P exactly.  The diagonal term of A + I is not part of
 * the sampled set; it is returned separately (self_w) and applied to the
 * node's own row, which a block always carries as source i.
 *
 * src_ids: global ids of the block's sources (the first num_dst are the
 * destinations).  edge_w[p] for block edge p, self_w[i] for destination i.
 */
void orc_gcn_edge_weights(const int64_t *row_ptr, const int64_t *src_ids, const int64_t *indptr,
                          const int32_t *indices, int64_t num_dst, double *edge_w, double *self_w)
{
    for (int64_t i = 0; i < num_dst; ++i) {
        int64_t v = src_ids[i];
        double deg_i = (double)(row_ptr[v + 1] - row_ptr[v]);
        int64_t b = indptr[i], e = indptr[i + 1];
        double s_node = (double)(e - b);
        self_w[i] = 1.0 / (deg_i + 1.0);
        for (int64_t p = b; p < e; ++p) {
            int64_t u = src_ids[indices[p]];
            double deg_j = (double)(row_ptr[u + 1] - row_ptr[u]);
            double P_ij = 1.0 / sqrt((deg_i + 1.0) * (deg_j + 1.0));
            edge_w[p] = deg_i / s_node * P_ij;
        }
    }
}

/*
 * out[i, :] = self_w[i] * x[i, :] + sum over the edges p of row i of
 * edge_w[p] * x[indices[p], :]  (self_w may be NULL: no diagonal term),
 * accumulated in double in row order (the diagonal term first), rounded once
 * to float (and then once to half for is_half).
 */
void orc_weighted_aggregate(const int64_t *indptr, const int32_t *indices, int64_t num_dst,
                            const double *edge_w, const double *self_w, const void *x, int64_t x_stride,
                            void *out, int64_t out_stride, int64_t dim, int is_half)
{
    double *acc = malloc((size_t)(dim > 0 ? dim : 1) * sizeof *acc);
    for (int64_t i = 0; i < num_dst; ++i) {
        for (int64_t c = 0; c < dim; ++c) acc[c] = 0.0;
        for (int64_t p = indptr[i] - (self_w ? 1 : 0); p < indptr[i + 1]; ++p) {
            int64_t r = p < indptr[i] ? i : indices[p];
            double w = p < indptr[i] ? self_w[i] : edge_w[p];
            for (int64_t c = 0; c < dim; ++c) {
                double xv = is_half ? orc_half_to_double(((const uint16_t *)x)[r * x_stride + c])
                                    : (double)((const float *)x)[r * x_stride + c];
                acc[c] += w * xv;
            }
        }
        for (int64_t c = 0; c < dim; ++c) {
            if (is_half) ((uint16_t *)out)[i * out_stride + c] = orc_float_to_half((float)acc[c]);
            else ((float *)out)[i * out_stride + c] = (float)acc[c];
        }
    }
    free(acc);
}

/*
 * Backward of orc_weighted_aggregate: grad_x = M^T grad_out for the operator
 * M[i, s] = sum of edge_w over the edges of row i that point to s, plus
 * self_w[i] at s == i.  Accumulated in double in row order, rounded once.
 */
int orc_weighted_aggregate_backward(const int64_t *indptr, const int32_t *indices, int64_t num_dst,
                                    int64_t num_src, const double *edge_w, const double *self_w,
                                    const void *grad_out, int64_t go_stride, void *grad_x,
                                    int64_t gx_stride, int64_t dim, int is_half)
{
    size_t total = (size_t)(num_src > 0 ? num_src : 1) * (size_t)(dim > 0 ? dim : 1);
    double *acc = calloc(total, sizeof *acc);
    if (!acc) return -2;
    for (int64_t i = 0; i < num_dst; ++i)
        for (int64_t p = indptr[i] - (self_w ? 1 : 0); p < indptr[i + 1]; ++p) {
            int64_t s = p < indptr[i] ? i : indices[p];
            double w = p < indptr[i] ? self_w[i] : edge_w[p];
            for (int64_t c = 0; c < dim; ++c) {
                double g = is_half ? orc_half_to_double(((const uint16_t *)grad_out)[i * go_stride + c])
                                   : (double)((const float *)grad_out)[i * go_stride + c];
                acc[s * dim + c] += w * g;
            }
        }
    for (int64_t s = 0; s < num_src; ++s)
        for (int64_t c = 0; c < dim; ++c) {
            double v = acc[s * dim + c];
            if (is_half) ((uint16_t *)grad_x)[s * gx_stride + c] = orc_float_to_half((float)v);
            else ((float *)grad_x)[s * gx_stride + c] = (float)v;
        }
    free(acc);
    return 0;
}

/* --------------------------------------------- sampled / random-walk cache */

typedef struct { uint64_t key; int64_t id; } orc_key_id;

static int cmp_key_id(const void *a, const void *b)
{
    const orc_key_id *x = a, *y = b;
    if (x->key != y->key) return x->key < y->key ? -1 : 1;
    if (x->id != y->id) return x->id < y->id ? -1 : 1;
    return 0;
}

/* Domain tag that keeps the cache draw apart from every block's neighbour draw. */
#define ORC_CACHE_LAYER (-1)

/*
 * Cache membership drawn with probability proportional to in-degree (Eq. 13),
 * without replacement.  Every adjacency slot of a node is a ticket with an
 * independent uniform 64-bit key; a node's key is the smallest of its tickets
 * (nodes without neighbours get the largest possible key); the num_cached
 * nodes with the smallest (key, id) are cached, slot s holding the s-th
 * smallest.  The minimum of d independent uniforms is distributed as an
 * exponential race with rate d, so this is weighted sampling without
 * replacement with weight = degree (Efraimidis and Spirakis 2006), in integer
 * arithmetic only.
 */
int orc_build_cache_sampled(int64_t num_nodes, const int64_t *row_ptr, int64_t num_cached,
                            uint64_t seed, int64_t *cached_ids, int32_t *slot_of)
{
    if (num_cached < 0 || num_cached > num_nodes) return -1;
    orc_key_id *all = malloc((size_t)(num_nodes > 0 ? num_nodes : 1) * sizeof *all);
    if (!all) return -2;
    for (int64_t v = 0; v < num_nodes; ++v) {
        int64_t d = row_ptr[v + 1] - row_ptr[v];
        uint64_t best = ~(uint64_t)0;
        for (int64_t j = 0; j < d; ++j) {
            uint64_t k = orc_key(seed, ORC_CACHE_LAYER, v, j);
            if (k < best) best = k;
        }
        all[v].key = best;
        all[v].id = v;
    }
    qsort(all, (size_t)num_nodes, sizeof *all, cmp_key_id);
    for (int64_t v = 0; v < num_nodes; ++v) slot_of[v] = -1;
    for (int64_t s = 0; s < num_cached; ++s) {
        cached_ids[s] = all[s].id;
        slot_of[all[s].id] = (int32_t)s;
    }
    free(all);
    return 0;
}

/*
 * Short-random-walk scores (Eq. 14-15): P^(0) = 1/|V_t| on the training
 * nodes, 0 elsewhere, then L propagation steps with the sampling ratio
 * d_v = min(fanout_l, deg_v) / deg_v (Eq. 14: the share of node v's
 * neighbours that sampling keeps; 0 for a node without neighbours), deg_v the
 * length of v's adjacency row.  Row v lists the nodes that v samples from,
 * and A is that adjacency as a matrix: A[v][u] = 1 for u in row(v).  D A
 * therefore scales row v - the list v samples from - by v's own ratio.
 *
 * form ORC_WALK_PRINTED: Eq. 15 exactly as printed, with P a column vector,
 *   P^(l) = (D A + I) P^(l-1):   P'[i] = P[i] + d_i * sum_{j in row(i)} P[j].
 *   Node i collects the mass of the nodes it samples from, scaled by its own
 *   ratio.  The row is summed in adjacency order, then multiplied by d_i.
 *
 * form ORC_WALK_PUSH: the same matrix applied along the direction in which
 * sampling moves, P^(l) = (D A + I)^T P^(l-1):
 *   P'[u] = P[u] + sum over v with u in row(v) of d_v * P[v].
 *   A node v that holds mass P[v] reaches each of the nodes it samples from
 *   with probability d_v, so after l steps P[u] is the expected number of
 *   times u has entered the sampled frontier (a frontier keeps its nodes and
 *   adds the sampled neighbours of each, as the blocks of node-wise sampling
 *   do), started from a uniformly chosen training node.  This is "reached
 *   from the training set with high probability", the property the cache
 *   section asks for; the printed form moves mass against the sampling
 *   direction and, on a directed graph, scores nodes that sampling never
 *   reaches.  Written as the plain scatter: v ascending, the slots of row(v)
 *   in order, so the terms of a node u are added in ascending order of v.
 *
 * On a graph that equals its transpose the push form is
 * P'[u] = P[u] + sum_{v in row(u)} d_v * P[v], i.e. (A D + I) P.
 * Double precision; every product is rounded on its own (no fused
 * multiply-add).  step_fanouts[l-1] is the fanout of step l.
 */
#define ORC_WALK_PUSH 0
#define ORC_WALK_PRINTED 1

int orc_random_walk_scores(int64_t num_nodes, const int64_t *row_ptr, const int64_t *col_idx,
                           const int64_t *train_ids, int64_t num_train, const int64_t *step_fanouts,
                           int64_t num_steps, int64_t form, double *scores)
{
    if (form != ORC_WALK_PUSH && form != ORC_WALK_PRINTED) return -1;
    size_t cnt = (size_t)(num_nodes > 0 ? num_nodes : 1);
    double *cur = calloc(cnt, sizeof *cur);
    double *next = calloc(cnt, sizeof *next);
    if (!cur || !next) { free(cur); free(next); return -2; }
    for (int64_t t = 0; t < num_train; ++t) cur[train_ids[t]] = 1.0 / (double)num_train;
    for (int64_t l = 0; l < num_steps; ++l) {
        for (int64_t i = 0; i < num_nodes; ++i) next[i] = cur[i];              /* the "+ I" term */
        for (int64_t v = 0; v < num_nodes; ++v) {
            int64_t deg = row_ptr[v + 1] - row_ptr[v];
            double keep = deg < step_fanouts[l] ? (double)deg : (double)step_fanouts[l];
            double d = deg > 0 ? keep / (double)deg : 0.0;
            if (form == ORC_WALK_PRINTED) {
                double acc = 0.0;
                for (int64_t p = row_ptr[v]; p < row_ptr[v + 1]; ++p) acc += cur[col_idx[p]];
                double scaled = d * acc;                                      /* rounded before the addition */
                next[v] = cur[v] + scaled;
            } else {
                double share = d * cur[v];                                    /* what v hands to each node it samples from */
                for (int64_t p = row_ptr[v]; p < row_ptr[v + 1]; ++p) next[col_idx[p]] += share;
            }
        }
        double *t = cur; cur = next; next = t;
    }
    for (int64_t i = 0; i < num_nodes; ++i) scores[i] = cur[i];
    free(cur);
    free(next);
    return 0;
}

typedef struct { double score; int64_t id; } orc_score_id;

static int cmp_score_desc_id_asc(const void *a, const void *b)
{
    const orc_score_id *x = a, *y = b;
    if (x->score != y->score) return x->score > y->score ? -1 : 1;
    if (x->id != y->id) return x->id < y->id ? -1 : 1;
    return 0;
}

/* The num_cached nodes of highest score, ties to the lower id; slot s = s-th ranked. */
int orc_build_cache_by_score(int64_t num_nodes, const double *scores, int64_t num_cached,
                             int64_t *cached_ids, int32_t *slot_of)
{
    if (num_cached < 0 || num_cached > num_nodes) return -1;
    orc_score_id *all = malloc((size_t)(num_nodes > 0 ? num_nodes : 1) * sizeof *all);
    if (!all) return -2;
    for (int64_t v = 0; v < num_nodes; ++v) { all[v].score = scores[v]; all[v].id = v; }
    qsort(all, (size_t)num_nodes, sizeof *all, cmp_score_desc_id_asc);
    for (int64_t v = 0; v < num_nodes; ++v) slot_of[v] = -1;
    for (int64_t s = 0; s < num_cached; ++s) {
        cached_ids[s] = all[s].id;
        slot_of[all[s].id] = (int32_t)s;
    }
    free(all);
    return 0;
}

/* ------------------------------------------- weighted draws with real weights */

/*
 * An exponential variate from 64 random bits, in integers: -log2(r / 2^64)
 * with 32 fractional bits, for r in [1, 2^64) (r = 0 is treated as 1), in
 * (0, 64 * 2^32].  With m = r * 2^lz in [2^63, 2^64) (lz = leading zeros) the
 * integer part is lz + 1 and the fraction's complement comes from the binary
 * logarithm of m / 2^63 in [1, 2) by repeated squaring: square, and if the
 * square reached 2 emit a one bit and halve.  Squares are truncated to 64
 * bits, so the last bits of the fraction are approximate (error < 2^-30 of
 * one unit); what matters is that the function is a fixed integer
 * function of r.  Times ln 2 / 2^32 this is Exp(1) distributed.
 */
uint64_t orc_exp_ticket(uint64_t r)
{
    if (r == 0) r = 1;
    int lz = 0;
    while (!(r >> 63)) { r <<= 1; ++lz; }
    uint64_t m = r, frac = 0;
    for (int b = 0; b < 32; ++b) {
        unsigned __int128 sq = (unsigned __int128)m * m;      /* (m/2^63)^2 * 2^126 */
        uint64_t hi = (uint64_t)(sq >> 64), lo = (uint64_t)sq;
        if (hi >> 63) {                                       /* square >= 2 */
            frac = (frac << 1) | 1;
            m = hi;
        } else {
            frac <<= 1;
            m = (hi << 1) | (lo >> 63);
        }
    }
    return ((uint64_t)(lz + 1) << 32) - frac;
}

/* tickets[i] = orc_exp_ticket(orc_key(seed, layer, first + i, 0)): a stretch of the ticket stream of one draw. */
void orc_exp_tickets(uint64_t seed, int64_t layer, int64_t first, int64_t n, uint64_t *tickets)
{
    for (int64_t i = 0; i < n; ++i) tickets[i] = orc_exp_ticket(orc_key(seed, layer, first + i, 0));
}

/* Domain tag of the draw below (apart from the blocks' and from the degree-proportional draw). */
#define ORC_SCORE_DRAW_LAYER (-2)

typedef struct { double key; int64_t id; } orc_dkey_id;

static int cmp_dkey_id(const void *a, const void *b)
{
    const orc_dkey_id *x = a, *y = b;
    if (x->key != y->key) return x->key < y->key ? -1 : 1;
    if (x->id != y->id) return x->id < y->id ? -1 : 1;
    return 0;
}

/*
 * Cache membership drawn with probability proportional to a non-negative
 * score (the P^(L) of Eq. 14-15), without replacement: node i races with the
 * exponential clock key_i = ticket_i / score_i, ticket_i =
 * orc_exp_ticket(orc_key(seed, -2, i, 0)) (one IEEE double division; +inf for
 * a score of 0); the num_cached smallest (key, id) are cached, slot s = the
 * s-th smallest.
 */
int orc_build_cache_drawn_by_score(int64_t num_nodes, const double *scores, int64_t num_cached,
                                   uint64_t seed, int64_t *cached_ids, int32_t *slot_of)
{
    if (num_cached < 0 || num_cached > num_nodes) return -1;
    orc_dkey_id *all = malloc((size_t)(num_nodes > 0 ? num_nodes : 1) * sizeof *all);
    if (!all) return -2;
    for (int64_t v = 0; v < num_nodes; ++v) {
        double t = (double)orc_exp_ticket(orc_key(seed, ORC_SCORE_DRAW_LAYER, v, 0));
        all[v].key = scores[v] > 0.0 ? t / scores[v] : INFINITY;
        all[v].id = v;
    }
    qsort(all, (size_t)num_nodes, sizeof *all, cmp_dkey_id);
    for (int64_t v = 0; v < num_nodes; ++v) slot_of[v] = -1;
    for (int64_t s = 0; s < num_cached; ++s) {
        cached_ids[s] = all[s].id;
        slot_of[all[s].id] = (int32_t)s;
    }
    free(all);
    return 0;
}

/* ------------------------------------------------- layer-wise sampling (LADIES) */

/*
 * Eq. 7 in double precision: p_i = ||R P_{*,i}||_2^2 / ||R P||_F^2 for the rows
 * R = dst[0..num_dst) of P = D^-1/2 (A + I) D^-1/2 (Eq. 2), i.e.
 *   q_i = sum over v in dst with i in N(v) or i == v of 1 / ((deg_v+1)(deg_i+1)),
 *   p_i = q_i / sum_j q_j.
 * p has num_nodes entries; nodes outside the union of Eq. 6 get 0.  dst == NULL
 * stands for all rows (R = I): FastGCN's probabilities (Sec. III-B, FastGCN
 * paragraph), the squared column norms of P itself.
 */
void orc_ladies_probabilities(const int64_t *row_ptr, const int64_t *col_idx, int64_t num_nodes,
                              const int64_t *dst, int64_t num_dst, int flat, double *p)
{
    for (int64_t i = 0; i < num_nodes; ++i) p[i] = 0.0;
    if (!dst) num_dst = num_nodes;                 /* every row: the batch-independent norms of FastGCN */
    for (int64_t t = 0; t < num_dst; ++t) {
        int64_t v = dst ? dst[t] : t;
        double dv = (double)(row_ptr[v + 1] - row_ptr[v]) + 1.0;
        p[v] += 1.0 / (dv * dv);
        for (int64_t e = row_ptr[v]; e < row_ptr[v + 1]; ++e) {
            int64_t i = col_idx[e];
            double di = (double)(row_ptr[i + 1] - row_ptr[i]) + 1.0;
            p[i] += 1.0 / (dv * di);
        }
    }
    if (flat)                                      /* the norm itself instead of its square */
        for (int64_t i = 0; i < num_nodes; ++i) p[i] = sqrt(p[i]);
    double total = 0.0;
    for (int64_t i = 0; i < num_nodes; ++i) total += p[i];
    if (total > 0.0)
        for (int64_t i = 0; i < num_nodes; ++i) p[i] /= total;
}

/*
 * Debiased coefficients for draws without replacement (the recursion printed
 * as Eq. 12, Sec. III-B "Calibrate and Debias LS"): with the items in the
 * order they were drawn, p[i] the probability of the i-th drawn item in the
 * whole population of n items (sum over the population = 1),
 *   Y_0 = 0,  Y_{i+1} = (1 - a_{i+1}) Y_i + a_{i+1} Pi_{i+1},
 *   Pi_{i+1} = sum_{j drawn before} X_j + X_{i+1} / p^i_{i+1},
 *   a_1 = 1,  a_{k+1} = n / ((n - k)(k + 1)),
 * where p^i_{i+1} = p[i] / (1 - sum of the p drawn before) is the probability
 * of that draw given the earlier ones.  Y_s = sum_j beta[j] X_j estimates the
 * total sum_j X_j over the population without bias; beta is what is returned.
 * The recursion is carried out literally, O(s^2).
 */
void orc_debias_coefficients(const double *p, int64_t s, int64_t n, double *beta)
{
    double drawn = 0.0;
    for (int64_t i = 0; i < s; ++i) {
        double alpha = (double)n / ((double)(n - i) * (double)(i + 1));
        for (int64_t j = 0; j < i; ++j) beta[j] = (1.0 - alpha) * beta[j] + alpha;
        double p_cond = p[i] / (1.0 - drawn);
        beta[i] = alpha / p_cond;
        drawn += p[i];
    }
}

/* Domain tag of the layer-wise draw at block `layer` (the node-wise draw uses `layer` itself). */
#define ORC_LAYERWISE_TAG 64

/*
 * One LADIES block (Eq. 6-9).  Rows: dst[0..num_dst) (distinct nodes).
 *
 * Probabilities.  So that a CPU and a GPU agree on every decision, the column
 * masses are accumulated in integers: mass_i = sum over v in dst with i in
 * N(v) or i == v of floor(2^40 / (deg_v + 1)), and q_i = mass_i / (deg_i + 1)
 * stands for the q_i of orc_ladies_probabilities times 2^40 (relative error
 * below 2^-40 * (deg_v + 1) per term).  Candidates (Eq. 6, with the self loops
 * of A + I): the nodes with mass_i > 0.
 *
 * Draw: s_layer candidates without replacement with probability proportional
 * to q_i (all of them if there are at most s_layer), by an exponential race:
 * key_i = ticket_i * (deg_i + 1) / mass_i in doubles (one multiplication, one
 * division, each rounded once; mass converted to double first), ticket_i =
 * orc_exp_ticket(orc_key(seed, 64 + layer, i, 0)); the smallest (key, id) win.
 *
 * Block: sources = the drawn nodes in ascending id order (the next layer's
 * rows); row t lists the drawn nodes among v's neighbours and v itself: the
 * self edge first, then the adjacency row in slot order.  Weight of edge
 * (v, i) (Eq. 8): P_vi / (s * p_i) with s the number of drawn nodes and p_i =
 * q_i / sum_j q_j (sum over the candidates in ascending id order); with
 * `normalise` every row is then divided by its sum (the paper's normalisation
 * of the sampled Laplacian; rows without an edge stay empty).
 *
 * fastgcn != 0: the FastGCN variant (Eq. 4): the masses are taken over all rows
 * of the graph instead of the block's rows, so every node is a candidate and
 * the draw does not depend on the mini-batch; everything else is the same (the
 * draw is without replacement here too, and the weights are the importance
 * weights P_vu / (s p_u) of the estimator the paper states before Eq. 12).
 *
 * debias != 0 (the "+debias" variants, Eq. 12): a drawn node's column is scaled
 * by its debiased coefficient beta (orc_debias_coefficients over the drawn
 * nodes in the order of the race, population = the candidates) instead of
 * 1 / (s p): weight = P_vi * beta_i.  When every candidate is drawn beta is 1.
 *
 * flat != 0 (the "+flat" variants, Eq. 10): nodes are drawn with probability
 * proportional to sqrt(q_i), the column norm itself.  In the race the ticket is
 * squared instead of the rate being rooted - key_i = ((ticket_i * ticket_i) *
 * (deg_i + 1)) / mass_i, the same order as ticket_i / sqrt(q_i) - so that the
 * keys need multiplications and one division only; p_i = sqrt(q_i) / sum_j
 * sqrt(q_j) in the weights and in the debiased coefficients.
 *
 * mass_out (may be NULL): num_nodes masses.  Returns the number of sources,
 * -2 when cap_nnz or cap_src is too small or memory runs out.
 */
int64_t orc_ladies_block(const int64_t *row_ptr, const int64_t *col_idx, int64_t num_nodes,
                         const int64_t *dst, int64_t num_dst, int64_t s_layer, int64_t layer,
                         uint64_t rng_seed, int normalise, int fastgcn, int debias, int flat,
                         int64_t cap_src, int64_t cap_nnz, int64_t *src, int64_t *indptr,
                         int32_t *indices, double *edge_w, uint64_t *mass_out)
{
    size_t cnt = (size_t)(num_nodes > 0 ? num_nodes : 1);
    uint64_t *mass = calloc(cnt, sizeof *mass);
    int64_t *pos = malloc(cnt * sizeof *pos);
    orc_dkey_id *cand = malloc(cnt * sizeof *cand);
    if (!mass || !pos || !cand) { free(mass); free(pos); free(cand); return -2; }

    for (int64_t t = 0; t < (fastgcn ? num_nodes : num_dst); ++t) {
        int64_t v = fastgcn ? t : dst[t];
        uint64_t add = ((uint64_t)1 << 40) / (uint64_t)(row_ptr[v + 1] - row_ptr[v] + 1);
        mass[v] += add;
        for (int64_t e = row_ptr[v]; e < row_ptr[v + 1]; ++e) mass[col_idx[e]] += add;
    }
    if (mass_out) memcpy(mass_out, mass, (size_t)num_nodes * sizeof *mass);

    int64_t num_cand = 0;
    double q_total = 0.0;
    for (int64_t i = 0; i < num_nodes; ++i) {
        if (!mass[i]) continue;
        double deg1 = (double)(row_ptr[i + 1] - row_ptr[i] + 1);
        double ticket = (double)orc_exp_ticket(orc_key(rng_seed, ORC_LAYERWISE_TAG + layer, i, 0));
        cand[num_cand].key = flat ? ((ticket * ticket) * deg1) / (double)mass[i] : (ticket * deg1) / (double)mass[i];
        cand[num_cand].id = i;
        ++num_cand;
        q_total += flat ? sqrt((double)mass[i] / deg1) : (double)mass[i] / deg1;
    }
    int64_t num_src = num_cand < s_layer ? num_cand : s_layer;
    if (num_src > cap_src) { free(mass); free(pos); free(cand); return -2; }
    if (num_cand > s_layer) qsort(cand, (size_t)num_cand, sizeof *cand, cmp_dkey_id);
    for (int64_t r = 0; r < num_src; ++r) src[r] = cand[r].id;
    qsort(src, (size_t)num_src, sizeof *src, cmp_i64);
    for (int64_t i = 0; i < num_nodes; ++i) pos[i] = -1;
    for (int64_t r = 0; r < num_src; ++r) pos[src[r]] = r;

    double *beta_of_pos = NULL;
    if (debias) {
        size_t ns = (size_t)(num_src > 0 ? num_src : 1);
        double *p_drawn = malloc(ns * sizeof *p_drawn);
        double *beta = malloc(ns * sizeof *beta);
        beta_of_pos = malloc(ns * sizeof *beta_of_pos);
        if (!p_drawn || !beta || !beta_of_pos) { free(p_drawn); free(beta); free(beta_of_pos); free(mass); free(pos); free(cand); return -2; }
        if (num_src == num_cand) {
            for (int64_t r = 0; r < num_src; ++r) beta_of_pos[r] = 1.0;
        } else {
            for (int64_t r = 0; r < num_src; ++r) {              /* cand[0..num_src) is in draw order */
                int64_t i = cand[r].id;
                double q_i = (double)mass[i] / (double)(row_ptr[i + 1] - row_ptr[i] + 1);
                p_drawn[r] = (flat ? sqrt(q_i) : q_i) / q_total;
            }
            orc_debias_coefficients(p_drawn, num_src, num_cand, beta);
            for (int64_t r = 0; r < num_src; ++r) beta_of_pos[pos[cand[r].id]] = beta[r];
        }
        free(p_drawn);
        free(beta);
    }

    int64_t nnz = 0;
    indptr[0] = 0;
    for (int64_t t = 0; t < num_dst; ++t) {
        int64_t v = dst[t];
        double dv = (double)(row_ptr[v + 1] - row_ptr[v] + 1);
        int64_t row_begin = nnz;
        for (int64_t e = row_ptr[v] - 1; e < row_ptr[v + 1]; ++e) {      /* e == row_ptr[v] - 1: the self edge */
            int64_t i = e < row_ptr[v] ? v : col_idx[e];
            if (pos[i] < 0) continue;
            if (nnz >= cap_nnz) { free(mass); free(pos); free(cand); free(beta_of_pos); return -2; }
            double di = (double)(row_ptr[i + 1] - row_ptr[i] + 1);
            double P_vi = 1.0 / sqrt(dv * di);
            double p_i = (flat ? sqrt((double)mass[i] / di) : (double)mass[i] / di) / q_total;
            indices[nnz] = (int32_t)pos[i];
            edge_w[nnz] = debias ? P_vi * beta_of_pos[pos[i]] : P_vi / ((double)num_src * p_i);
            ++nnz;
        }
        if (normalise) {
            double row_sum = 0.0;
            for (int64_t e = row_begin; e < nnz; ++e) row_sum += edge_w[e];
            for (int64_t e = row_begin; e < nnz; ++e) edge_w[e] /= row_sum;
        }
        indptr[t + 1] = nnz;
    }
    free(mass);
    free(pos);
    free(cand);
    free(beta_of_pos);
    return num_src;
}
