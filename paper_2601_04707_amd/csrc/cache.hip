// Hot-node feature cache construction (paper Sec. III "Feature Cache": the features of a small
// set of high-degree nodes are preloaded on the GPU).  Three ways to rank the nodes; the first
// num_cached of the ranking are cached, slot s holding the s-th ranked node:
//   top degree       (degree descending, id ascending) - deterministic reading of Eq. 13
//   degree-sampled   Eq. 13 as stated: membership drawn with probability proportional to in-degree,
//                    without replacement.  Every adjacency slot is a ticket with a uniform 64-bit
//                    key, a node's key is the minimum over its tickets (k_ticket_keys), nodes are
//                    ranked by (key, id) ascending - an exponential race in integer arithmetic
//   random walk      Eq. 14-15: L propagation steps from the training set, ranked by (P^(L) descending,
//                    id ascending).  Push form: every node hands d_v * P[v] to the nodes of its
//                    row, the terms of a node added in ascending order of v - computed as a sum
//                    over the rows of the transposed adjacency (k_edge_pairs, a stable radix sort
//                    by column, k_in_ptr), or over the adjacency itself when the caller states
//                    that the graph equals its transpose.  Printed form: a node collects
//                    d_i * sum of P over its row.  k_rw_pass, k_rw_step: double precision, every
//                    row summed in order, so the result does not depend on the schedule
// 64-bit keys are ordered by two stable 32-bit radix sorts (low word, then high word).
//
// The ranking is a stable least-significant-digit radix sort of (max_degree - degree) with the
// node id as payload: ids start ascending, stable passes keep them ascending inside equal
// degrees.  Only as many 8-bit passes run as max_degree has bytes.
//   k_degrees        degree per node, running maximum
//   k_sort_keys      key = max_degree - degree, payload = id
//   (radix passes)   see radix.hip
//   k_assign_slots   slot_of / cached_ids
// then the cached rows are copied with the direct gather kernel.
#include <algorithm>
#include <vector>

#include "common.h"
#include "device_utils.h"
#include "radix.h"

namespace mqg {

int gather_direct_i32(mqg_ctx *ctx, const int32_t *ids, const int64_t *num_ids, int64_t cap, int64_t src_rows, const void *src,
                      int64_t src_stride_bytes, void *dst, int64_t dst_stride_bytes, int64_t row_bytes, hipStream_t s);

namespace {


template <typename PtrT>
__global__ void __launch_bounds__(kBlock)
k_degrees(const PtrT *__restrict__ row_ptr, int64_t n, uint32_t *__restrict__ deg, uint32_t *__restrict__ max_deg) {
    int64_t v = int64_t(blockIdx.x) * kBlock + threadIdx.x;
    uint32_t d = 0;
    if (v < n) {
        d = static_cast<uint32_t>(row_ptr[v + 1] - row_ptr[v]);
        deg[v] = d;
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        uint32_t o = __shfl_xor(d, off, 64);
        d = o > d ? o : d;
    }
    // a plain read first: once the running maximum is high almost no wavefront needs the atomic
    if (lane_id() == 0 && d > *reinterpret_cast<volatile uint32_t *>(max_deg)) atomicMax(max_deg, d);
}

__global__ void __launch_bounds__(kBlock)
k_sort_keys(uint32_t *__restrict__ keys, int32_t *__restrict__ vals, int64_t n, uint32_t max_deg) {
    int64_t v = int64_t(blockIdx.x) * kBlock + threadIdx.x;
    if (v < n) {
        keys[v] = max_deg - keys[v];                 // in: degree, out: sort key
        vals[v] = static_cast<int32_t>(v);
    }
}

constexpr uint64_t kGolden = 0x9E3779B97F4A7C15ULL;

uint64_t host_mix64(uint64_t z) {
    z ^= z >> 30;
    z *= 0xBF58476D1CE4E5B9ULL;
    z ^= z >> 27;
    z *= 0x94D049BB133111EBULL;
    z ^= z >> 31;
    return z;
}

__device__ __forceinline__ uint64_t wave_min_u64(uint64_t v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        uint64_t o = __shfl_xor(v, off, 64);
        v = o < v ? o : v;
    }
    return v;
}

// key64[v] = min over the adjacency slots j of node v of mix(mix(tag_hash ^ v) ^ j); all ones for
// a node without neighbours.  A lane owns a node; rows of up to 32 slots are walked by their
// lane, longer rows by the whole wavefront, one after the other.
template <typename PtrT>
__global__ void __launch_bounds__(kBlock)
k_ticket_keys(const PtrT *__restrict__ row_ptr, int64_t n, uint64_t tag_hash, uint64_t *__restrict__ key64) {
    const int lane = lane_id();
    const int64_t v = int64_t(blockIdx.x) * kBlock + threadIdx.x;
    int d = 0;
    if (v < n) d = static_cast<int>(row_ptr[v + 1] - row_ptr[v]);
    const uint64_t hv = mix64(tag_hash ^ static_cast<uint64_t>(v));
    uint64_t best = ~uint64_t(0);
    if (d <= 32)
        for (int j = 0; j < d; ++j) {
            uint64_t k = mix64(hv ^ static_cast<uint64_t>(j));
            best = k < best ? k : best;
        }
    uint64_t big = ballot64(d > 32);
    while (big) {
        const int l = __ffsll(static_cast<long long>(big)) - 1;
        big &= big - 1;
        const int dl = static_cast<int>(readlane32(static_cast<uint32_t>(d), l));
        const uint64_t hl = readlane64(hv, l);
        uint64_t m = ~uint64_t(0);
        for (int j = lane; j < dl; j += kWave) {
            uint64_t k = mix64(hl ^ static_cast<uint64_t>(j));
            m = k < m ? k : m;
        }
        m = wave_min_u64(m);
        if (lane == l) best = m;
    }
    if (v < n) key64[v] = best;
}

template <typename IdxT>
__global__ void __launch_bounds__(kBlock)
k_rw_seed(const IdxT *__restrict__ train_ids, int64_t num_train, int64_t n, double *__restrict__ p,
          uint32_t *__restrict__ flags) {
    int64_t t = int64_t(blockIdx.x) * kBlock + threadIdx.x;
    if (t >= num_train) return;
    const int64_t id = static_cast<int64_t>(train_ids[t]);
    if (id < 0 || id >= n) atomicOr(flags, 1u);            // reported by the host; never used as an index
    else p[id] = 1.0 / static_cast<double>(num_train);
}

// The adjacency as (column, row) pairs in row order: keys[e] = col_idx[e], vals[e] = the row that
// holds slot e.  Sorted stably by key they are the transposed adjacency with every in-list in
// ascending order of the row.  Rows of up to 16 slots are written by their lane, longer rows by
// the wavefront.
template <typename PtrT, typename IdxT>
__global__ void __launch_bounds__(kBlock)
k_edge_pairs(const PtrT *__restrict__ row_ptr, const IdxT *__restrict__ col_idx, int64_t n,
             uint32_t *__restrict__ keys, int32_t *__restrict__ vals) {
    const int lane = lane_id();
    const int64_t i = int64_t(blockIdx.x) * kBlock + threadIdx.x;
    int64_t b = 0;
    int deg = 0;
    if (i < n) {
        b = static_cast<int64_t>(row_ptr[i]);
        deg = static_cast<int>(static_cast<int64_t>(row_ptr[i + 1]) - b);
    }
    if (deg <= 16)
        for (int p = 0; p < deg; ++p) {
            keys[b + p] = static_cast<uint32_t>(col_idx[b + p]);
            vals[b + p] = static_cast<int32_t>(i);
        }
    uint64_t big = ballot64(deg > 16);
    while (big) {
        const int l = __ffsll(static_cast<long long>(big)) - 1;
        big &= big - 1;
        const int dl = static_cast<int>(readlane32(static_cast<uint32_t>(deg), l));
        const int64_t bl = static_cast<int64_t>(readlane64(static_cast<uint64_t>(b), l));
        const int32_t row = static_cast<int32_t>(readlane64(static_cast<uint64_t>(i), l));
        for (int c = lane; c < dl; c += kWave) {
            keys[bl + c] = static_cast<uint32_t>(col_idx[bl + c]);
            vals[bl + c] = row;
        }
    }
}

// in_ptr[u] = first position in the sorted column array whose column is >= u (bisection), u = 0..n
__global__ void __launch_bounds__(kBlock)
k_in_ptr(const uint32_t *__restrict__ sorted_cols, int64_t num_edges, int64_t n, int32_t *__restrict__ in_ptr) {
    const int64_t u = int64_t(blockIdx.x) * kBlock + threadIdx.x;
    if (u > n) return;
    int64_t lo = 0, hi = num_edges;
    while (lo < hi) {
        const int64_t mid = (lo + hi) >> 1;
        if (static_cast<int64_t>(sorted_cols[mid]) < u) lo = mid + 1; else hi = mid;
    }
    in_ptr[u] = static_cast<int32_t>(lo);
}

// A step of the random-walk scores.
//   k_rw_pass   share[v] = d_v * P[v], d_v = min(fanout, deg_v) / deg_v: what a node that holds mass
//               P[v] hands to each node of its row (push form)
//   k_rw_step   P_next[i] = P[i] + scale_i * sum_{j in list(i)} val[j], every list added strictly in
//               order (push form: onto P[i], term by term; printed form: from zero, then scaled) (lists of up to 16 entries by their lane, longer ones by the wavefront: 64
//               values are fetched in parallel and then added one after the other) - bit for bit
//               the plain sequential loop, whatever the schedule.
//               Push form: list = the in-list of i in ascending order of the source (the
//               transposed adjacency, or the adjacency itself on a graph that equals its
//               transpose), val = share, no scale.  Printed form (scale_fanout > 0): list = the
//               row of i, val = P, scale_i = d_i, the product rounded before the addition.
template <typename PtrT>
__global__ void __launch_bounds__(kBlock)
k_rw_pass(const PtrT *__restrict__ row_ptr, int64_t n, int fanout, const double *__restrict__ cur,
          double *__restrict__ pass) {
#pragma clang fp contract(off)
    const int64_t j = int64_t(blockIdx.x) * kBlock + threadIdx.x;
    if (j < n) {
        const int64_t deg = static_cast<int64_t>(row_ptr[j + 1]) - static_cast<int64_t>(row_ptr[j]);
        const double keep = deg < fanout ? static_cast<double>(deg) : static_cast<double>(fanout);
        const double d = deg > 0 ? keep / static_cast<double>(deg) : 0.0;
        pass[j] = d * cur[j];
    }
}

template <typename PtrT, typename IdxT>
__global__ void __launch_bounds__(kBlock)
k_rw_step(const PtrT *__restrict__ row_ptr, const IdxT *__restrict__ col_idx, int64_t n,
          const double *__restrict__ cur, const double *__restrict__ pass, double *__restrict__ next,
          int scale_fanout) {
#pragma clang fp contract(off)
    const int lane = lane_id();
    const int64_t i = int64_t(blockIdx.x) * kBlock + threadIdx.x;
    int64_t b = 0;
    int deg = 0;
    if (i < n) {
        b = static_cast<int64_t>(row_ptr[i]);
        deg = static_cast<int>(static_cast<int64_t>(row_ptr[i + 1]) - b);
    }
    // push form: the terms are added onto the node's own mass, one after the other; printed form: the
    // row is summed from zero, scaled, and added to the node's mass
    const double own = i < n ? cur[i] : 0.0;
    const double start = scale_fanout > 0 ? 0.0 : own;
    double acc = start;
    if (deg <= 16)
        for (int p = 0; p < deg; ++p) acc = acc + pass[col_idx[b + p]];
    uint64_t big = ballot64(deg > 16);
    while (big) {
        const int l = __ffsll(static_cast<long long>(big)) - 1;
        big &= big - 1;
        const int dl = static_cast<int>(readlane32(static_cast<uint32_t>(deg), l));
        const int64_t bl = static_cast<int64_t>(readlane64(static_cast<uint64_t>(b), l));
        double a = __longlong_as_double(static_cast<long long>(readlane64(static_cast<uint64_t>(__double_as_longlong(start)), l)));
        for (int c0 = 0; c0 < dl; c0 += kWave) {
            const int m = dl - c0 < kWave ? dl - c0 : kWave;
            double val = 0.0;
            if (lane < m) val = pass[col_idx[bl + c0 + lane]];
            const uint64_t bits = static_cast<uint64_t>(__double_as_longlong(val));
            for (int t = 0; t < m; ++t) a = a + __longlong_as_double(static_cast<long long>(readlane64(bits, t)));
        }
        if (lane == l) acc = a;
    }
    if (i < n) {
        if (scale_fanout > 0) {
            const double keep = deg < scale_fanout ? static_cast<double>(deg) : static_cast<double>(scale_fanout);
            const double d = deg > 0 ? keep / static_cast<double>(deg) : 0.0;
            const double scaled = d * acc;
            next[i] = own + scaled;
        } else {
            next[i] = acc;
        }
    }
}

// ascending radix order of ~bits(score) = descending score (scores are non-negative)
__global__ void __launch_bounds__(kBlock)
k_score_keys(const double *__restrict__ score, int64_t n, uint64_t *__restrict__ key64) {
    int64_t v = int64_t(blockIdx.x) * kBlock + threadIdx.x;
    if (v < n) key64[v] = ~static_cast<uint64_t>(__double_as_longlong(score[v]));
}

// Exponential race for a draw in proportion to the score: key = ticket / score as a double (one IEEE
// division; +inf for a score of 0), ticket = exp_ticket64 of the node's random bits.  Positive
// doubles order like their bit patterns.
__global__ void __launch_bounds__(kBlock)
k_draw_keys(const double *__restrict__ score, int64_t n, uint64_t tag_hash, uint64_t *__restrict__ key64) {
    int64_t v = int64_t(blockIdx.x) * kBlock + threadIdx.x;
    if (v >= n) return;
    const uint64_t r = mix64(mix64(tag_hash ^ static_cast<uint64_t>(v)));     // slot 0 of node v
    const double t = static_cast<double>(exp_ticket64(r));
    const double sc = score[v];
    const double key = sc > 0.0 ? t / sc : __longlong_as_double(0x7FF0000000000000LL);
    key64[v] = static_cast<uint64_t>(__double_as_longlong(key));
}

// tickets[i] = exp_ticket64 of the random bits of (seed, tag, first + i, slot 0): the ticket stream on its own
__global__ void __launch_bounds__(kBlock)
k_exp_tickets(uint64_t tag_hash, int64_t first, int64_t n, uint64_t *__restrict__ tickets) {
    const int64_t i = int64_t(blockIdx.x) * kBlock + threadIdx.x;
    if (i >= n) return;
    const uint64_t r = mix64(mix64(tag_hash ^ static_cast<uint64_t>(first + i)));
    tickets[i] = exp_ticket64(r);
}

__global__ void __launch_bounds__(kBlock)
k_split_low(const uint64_t *__restrict__ key64, int64_t n, uint32_t *__restrict__ lo, int32_t *__restrict__ ids) {
    int64_t v = int64_t(blockIdx.x) * kBlock + threadIdx.x;
    if (v < n) {
        lo[v] = static_cast<uint32_t>(key64[v]);
        ids[v] = static_cast<int32_t>(v);
    }
}

__global__ void __launch_bounds__(kBlock)
k_gather_high(const uint64_t *__restrict__ key64, const int32_t *__restrict__ ids_in, int64_t n,
              uint32_t *__restrict__ hi, int32_t *__restrict__ ids_out) {
    int64_t p = int64_t(blockIdx.x) * kBlock + threadIdx.x;
    if (p < n) {
        int32_t v = ids_in[p];
        hi[p] = static_cast<uint32_t>(key64[v] >> 32);
        ids_out[p] = v;
    }
}

template <typename IdxT>
__global__ void __launch_bounds__(kBlock)
k_assign_slots(const int32_t *__restrict__ ranked, int64_t num_cached, int32_t *__restrict__ slot_of,
               IdxT *__restrict__ cached_ids) {
    int64_t s = int64_t(blockIdx.x) * kBlock + threadIdx.x;
    if (s < num_cached) {
        int32_t v = ranked[s];
        slot_of[v] = static_cast<int32_t>(s);
        if (cached_ids) cached_ids[s] = static_cast<IdxT>(v);
    }
}

__global__ void k_store_i64(int64_t *p, int64_t v) {
    if (blockIdx.x == 0 && threadIdx.x == 0) *p = v;
}

// Temporaries of one build.  With a reserved arena (mqg_ctx_reserve) they are carved out of it and
// nothing is allocated; what does not fit - the transposed adjacency of the push walk, sized by the
// edges - and everything on a context without an arena is hipMalloc'ed and freed on return.
struct Temp {
    char *arena = nullptr;
    int64_t arena_bytes = 0, used = 0;
    std::vector<void *> ptrs;
    explicit Temp(mqg_ctx *ctx) : arena(ctx->cache_arena), arena_bytes(ctx->cache_arena_bytes) {}
    ~Temp() {
        for (void *p : ptrs) (void)hipFree(p);
    }
    bool allocated_any() const { return !ptrs.empty(); }
    template <typename T>
    bool alloc(T **p, int64_t n) {
        const int64_t bytes = (std::max<int64_t>(n, 1) * int64_t(sizeof(T)) + 255) & ~int64_t(255);
        if (arena && used + bytes <= arena_bytes) {
            *p = reinterpret_cast<T *>(arena + used);
            used += bytes;
            return true;
        }
        void *q = nullptr;
        if (hipMalloc(&q, static_cast<size_t>(bytes)) != hipSuccess) return false;
        ptrs.push_back(q);
        *p = static_cast<T *>(q);
        return true;
    }
};

}  // namespace

// node ids ranked by ascending 64-bit key (ties: ascending id), into *ranked (a buffer owned by tmp)
static int rank_by_key64(mqg_ctx *ctx, Temp &tmp, const uint64_t *key64, int64_t n, const int32_t **ranked, hipStream_t s) {
    uint32_t *lo, *hi;
    int32_t *ids0, *ids1;
    RadixBufs rb;
    bool ok = tmp.alloc(&lo, n) && tmp.alloc(&hi, n) && tmp.alloc(&ids0, n) && tmp.alloc(&ids1, n) &&
              tmp.alloc(&rb.keys[0], n) && tmp.alloc(&rb.keys[1], n) && tmp.alloc(&rb.vals[0], n) && tmp.alloc(&rb.vals[1], n) &&
              tmp.alloc(&rb.hist, radix_hist_len_max(n)) && tmp.alloc(&rb.tile_sums, radix_scan_tiles_max(n));
    if (!ok) return fail(ctx, MQG_ERR_HIP, "mqg_build_cache: temporary allocation failed");
    const int ngrid = static_cast<int>(ceil_div(n, kBlock));
    MQG_LAUNCH(ctx, "k_split_low", s, (k_split_low<<<ngrid, kBlock, 0, s>>>(key64, n, lo, ids0)));
    int which = -1;
    int rc = radix_sort_pairs(ctx, lo, ids0, rb, n, nullptr, 32, s, &which);
    if (rc != MQG_OK) return rc;
    MQG_LAUNCH(ctx, "k_gather_high", s, (k_gather_high<<<ngrid, kBlock, 0, s>>>(key64, rb.vals[which], n, hi, ids1)));
    rc = radix_sort_pairs(ctx, hi, ids1, rb, n, nullptr, 32, s, &which);
    if (rc != MQG_OK) return rc;
    *ranked = rb.vals[which];
    return MQG_OK;
}

int run_build_cache(mqg_ctx *ctx, const mqg_graph *g, mqg_cache *c, const mqg_cache_plan *plan, hipStream_t s) {
    const int64_t n = g->num_nodes;
    const int64_t elt = c->dtype == MQG_F16 ? 2 : 4;
    const int policy = plan ? plan->policy : MQG_CACHE_TOP_DEGREE;
    hipError_t e = hipMemsetAsync(c->slot_of, 0xFF, static_cast<size_t>(std::max<int64_t>(n, 1)) * sizeof(int32_t), s);
    if (e != hipSuccess) return fail(ctx, MQG_ERR_HIP, std::string("hipMemsetAsync: ") + hipGetErrorString(e));
    const bool walk = policy == MQG_CACHE_RANDOM_WALK || policy == MQG_CACHE_RANDOM_WALK_SAMPLED;
    const bool want_scores = walk && plan->scores_out;
    if (n == 0 || (c->num_cached == 0 && !want_scores)) {
        e = hipStreamSynchronize(s);
        return e == hipSuccess ? MQG_OK : fail(ctx, MQG_ERR_HIP, hipGetErrorString(e));
    }

    Temp tmp(ctx);
    const int ngrid = static_cast<int>(ceil_div(n, kBlock));
    const int32_t *ranked = nullptr;
    uint32_t *walk_flags = nullptr;                  // bit 0: a training id outside the graph

    if (policy == MQG_CACHE_TOP_DEGREE) {
        uint32_t *keys_a, *max_deg_dev;
        int32_t *vals_a;
        RadixBufs rb;
        bool ok = tmp.alloc(&keys_a, n) && tmp.alloc(&vals_a, n) && tmp.alloc(&rb.keys[0], n) && tmp.alloc(&rb.keys[1], n) &&
                  tmp.alloc(&rb.vals[0], n) && tmp.alloc(&rb.vals[1], n) && tmp.alloc(&rb.hist, radix_hist_len_max(n)) &&
                  tmp.alloc(&rb.tile_sums, radix_scan_tiles_max(n)) && tmp.alloc(&max_deg_dev, 1);
        if (!ok) return fail(ctx, MQG_ERR_HIP, "mqg_build_cache: temporary allocation failed");
        e = hipMemsetAsync(max_deg_dev, 0, sizeof(uint32_t), s);
        if (e != hipSuccess) return fail(ctx, MQG_ERR_HIP, hipGetErrorString(e));
        if (g->ptr_type == MQG_I64)
            MQG_LAUNCH(ctx, "k_degrees", s, (k_degrees<int64_t><<<ngrid, kBlock, 0, s>>>(static_cast<const int64_t *>(g->row_ptr), n, keys_a, max_deg_dev)));
        else
            MQG_LAUNCH(ctx, "k_degrees", s, (k_degrees<int32_t><<<ngrid, kBlock, 0, s>>>(static_cast<const int32_t *>(g->row_ptr), n, keys_a, max_deg_dev)));
        uint32_t max_deg = 0;
        e = hipMemcpyAsync(&max_deg, max_deg_dev, sizeof(uint32_t), hipMemcpyDeviceToHost, s);
        if (e == hipSuccess) e = hipStreamSynchronize(s);
        if (e != hipSuccess) return fail(ctx, MQG_ERR_HIP, std::string("mqg_build_cache: ") + hipGetErrorString(e));
        MQG_LAUNCH(ctx, "k_sort_keys", s, (k_sort_keys<<<ngrid, kBlock, 0, s>>>(keys_a, vals_a, n, max_deg)));
        const int bits = radix_key_bits(max_deg);
        int which = -1;
        int rc0 = radix_sort_pairs(ctx, keys_a, vals_a, rb, n, nullptr, bits, s, &which);
        if (rc0 != MQG_OK) return rc0;
        ranked = which < 0 ? vals_a : rb.vals[which];
    } else if (policy == MQG_CACHE_DEGREE_SAMPLED) {
        uint64_t *key64;
        if (!tmp.alloc(&key64, n)) return fail(ctx, MQG_ERR_HIP, "mqg_build_cache: temporary allocation failed");
        // the tag keeps this draw apart from every block's neighbour draw (block index -1)
        const uint64_t tag_hash = host_mix64(host_mix64(plan->seed + kGolden) ^ ~uint64_t(0));
        if (g->ptr_type == MQG_I64)
            MQG_LAUNCH(ctx, "k_ticket_keys", s, (k_ticket_keys<int64_t><<<ngrid, kBlock, 0, s>>>(static_cast<const int64_t *>(g->row_ptr), n, tag_hash, key64)));
        else
            MQG_LAUNCH(ctx, "k_ticket_keys", s, (k_ticket_keys<int32_t><<<ngrid, kBlock, 0, s>>>(static_cast<const int32_t *>(g->row_ptr), n, tag_hash, key64)));
        int rc0 = rank_by_key64(ctx, tmp, key64, n, &ranked, s);
        if (rc0 != MQG_OK) return rc0;
    } else {  // MQG_CACHE_RANDOM_WALK, MQG_CACHE_RANDOM_WALK_SAMPLED
        double *pa, *pb, *pass;
        uint64_t *key64;
        if (!(tmp.alloc(&pa, n) && tmp.alloc(&pb, n) && tmp.alloc(&pass, n) && tmp.alloc(&key64, n) && tmp.alloc(&walk_flags, 1)))
            return fail(ctx, MQG_ERR_HIP, "mqg_build_cache: temporary allocation failed");
        e = hipMemsetAsync(pa, 0, static_cast<size_t>(n) * sizeof(double), s);
        if (e == hipSuccess) e = hipMemsetAsync(walk_flags, 0, sizeof(uint32_t), s);
        if (e != hipSuccess) return fail(ctx, MQG_ERR_HIP, hipGetErrorString(e));
        if (plan->num_train > 0) {
            const int tgrid = static_cast<int>(ceil_div(plan->num_train, kBlock));
            if (g->idx_type == MQG_I64)
                MQG_LAUNCH(ctx, "k_rw_seed", s, (k_rw_seed<int64_t><<<tgrid, kBlock, 0, s>>>(static_cast<const int64_t *>(plan->train_ids), plan->num_train, n, pa, walk_flags)));
            else
                MQG_LAUNCH(ctx, "k_rw_seed", s, (k_rw_seed<int32_t><<<tgrid, kBlock, 0, s>>>(static_cast<const int32_t *>(plan->train_ids), plan->num_train, n, pa, walk_flags)));
        }
        const bool p64 = g->ptr_type == MQG_I64, i64 = g->idx_type == MQG_I64;
        const bool printed = plan->walk_form == MQG_WALK_PRINTED;
        // push form on a graph that is not known to equal its transpose: the in-lists, sources ascending
        const int32_t *in_ptr = nullptr, *in_src = nullptr;
        if (!printed && !plan->graph_symmetric && plan->num_steps > 0) {
            const int64_t ne = g->num_edges;
            const int bits = radix_key_bits(static_cast<uint64_t>(n - 1));
            uint32_t *cols;
            int32_t *rows_of, *ptr_t;
            RadixBufs rb;
            bool ok = tmp.alloc(&cols, ne) && tmp.alloc(&rows_of, ne) && tmp.alloc(&ptr_t, n + 1) && tmp.alloc(&rb.keys[0], ne) &&
                      tmp.alloc(&rb.keys[1], ne) && tmp.alloc(&rb.vals[0], ne) && tmp.alloc(&rb.vals[1], ne) &&
                      tmp.alloc(&rb.hist, radix_hist_len(ne, bits)) && tmp.alloc(&rb.tile_sums, radix_scan_tiles(ne, bits));
            if (!ok) return fail(ctx, MQG_ERR_HIP, "mqg_build_cache: temporary allocation failed (transposed adjacency)");
            if (ne > 0) {
                if (p64 && i64)
                    MQG_LAUNCH(ctx, "k_edge_pairs", s, (k_edge_pairs<int64_t, int64_t><<<ngrid, kBlock, 0, s>>>(static_cast<const int64_t *>(g->row_ptr), static_cast<const int64_t *>(g->col_idx), n, cols, rows_of)));
                else if (p64)
                    MQG_LAUNCH(ctx, "k_edge_pairs", s, (k_edge_pairs<int64_t, int32_t><<<ngrid, kBlock, 0, s>>>(static_cast<const int64_t *>(g->row_ptr), static_cast<const int32_t *>(g->col_idx), n, cols, rows_of)));
                else if (i64)
                    MQG_LAUNCH(ctx, "k_edge_pairs", s, (k_edge_pairs<int32_t, int64_t><<<ngrid, kBlock, 0, s>>>(static_cast<const int32_t *>(g->row_ptr), static_cast<const int64_t *>(g->col_idx), n, cols, rows_of)));
                else
                    MQG_LAUNCH(ctx, "k_edge_pairs", s, (k_edge_pairs<int32_t, int32_t><<<ngrid, kBlock, 0, s>>>(static_cast<const int32_t *>(g->row_ptr), static_cast<const int32_t *>(g->col_idx), n, cols, rows_of)));
            }
            int which = -1;
            int rc0 = radix_sort_pairs(ctx, cols, rows_of, rb, ne, nullptr, bits, s, &which);
            if (rc0 != MQG_OK) return rc0;
            const uint32_t *sorted_cols = which < 0 ? cols : rb.keys[which];
            in_src = which < 0 ? rows_of : rb.vals[which];
            MQG_LAUNCH(ctx, "k_in_ptr", s, (k_in_ptr<<<static_cast<int>(ceil_div(n + 1, kBlock)), kBlock, 0, s>>>(sorted_cols, ne, n, ptr_t)));
            in_ptr = ptr_t;
        }
        double *cur = pa, *next = pb;
        for (int l = 0; l < plan->num_steps; ++l) {
            const int fo = plan->step_fanouts[l];
            if (!printed) {
                if (p64)
                    MQG_LAUNCH(ctx, "k_rw_pass", s, (k_rw_pass<int64_t><<<ngrid, kBlock, 0, s>>>(static_cast<const int64_t *>(g->row_ptr), n, fo, cur, pass)));
                else
                    MQG_LAUNCH(ctx, "k_rw_pass", s, (k_rw_pass<int32_t><<<ngrid, kBlock, 0, s>>>(static_cast<const int32_t *>(g->row_ptr), n, fo, cur, pass)));
            }
            const double *val = printed ? cur : pass;
            const int scale = printed ? fo : 0;
            if (in_ptr)
                MQG_LAUNCH(ctx, "k_rw_step", s, (k_rw_step<int32_t, int32_t><<<ngrid, kBlock, 0, s>>>(in_ptr, in_src, n, cur, val, next, scale)));
            else if (p64 && i64)
                MQG_LAUNCH(ctx, "k_rw_step", s, (k_rw_step<int64_t, int64_t><<<ngrid, kBlock, 0, s>>>(static_cast<const int64_t *>(g->row_ptr), static_cast<const int64_t *>(g->col_idx), n, cur, val, next, scale)));
            else if (p64)
                MQG_LAUNCH(ctx, "k_rw_step", s, (k_rw_step<int64_t, int32_t><<<ngrid, kBlock, 0, s>>>(static_cast<const int64_t *>(g->row_ptr), static_cast<const int32_t *>(g->col_idx), n, cur, val, next, scale)));
            else if (i64)
                MQG_LAUNCH(ctx, "k_rw_step", s, (k_rw_step<int32_t, int64_t><<<ngrid, kBlock, 0, s>>>(static_cast<const int32_t *>(g->row_ptr), static_cast<const int64_t *>(g->col_idx), n, cur, val, next, scale)));
            else
                MQG_LAUNCH(ctx, "k_rw_step", s, (k_rw_step<int32_t, int32_t><<<ngrid, kBlock, 0, s>>>(static_cast<const int32_t *>(g->row_ptr), static_cast<const int32_t *>(g->col_idx), n, cur, val, next, scale)));
            std::swap(cur, next);
        }
        if (plan->scores_out) {
            e = hipMemcpyAsync(plan->scores_out, cur, static_cast<size_t>(n) * sizeof(double), hipMemcpyDeviceToDevice, s);
            if (e != hipSuccess) return fail(ctx, MQG_ERR_HIP, hipGetErrorString(e));
        }
        if (c->num_cached > 0) {
            if (policy == MQG_CACHE_RANDOM_WALK_SAMPLED) {
                const uint64_t tag_hash = host_mix64(host_mix64(plan->seed + kGolden) ^ static_cast<uint64_t>(int64_t(-2)));
                MQG_LAUNCH(ctx, "k_draw_keys", s, (k_draw_keys<<<ngrid, kBlock, 0, s>>>(cur, n, tag_hash, key64)));
            } else {
                MQG_LAUNCH(ctx, "k_score_keys", s, (k_score_keys<<<ngrid, kBlock, 0, s>>>(cur, n, key64)));
            }
            int rc0 = rank_by_key64(ctx, tmp, key64, n, &ranked, s);
            if (rc0 != MQG_OK) return rc0;
        }
    }

    if (c->num_cached > 0) {
        int64_t *count_dev;
        if (!tmp.alloc(&count_dev, 1)) return fail(ctx, MQG_ERR_HIP, "mqg_build_cache: temporary allocation failed");
        const int cgrid = static_cast<int>(ceil_div(c->num_cached, kBlock));
        if (g->idx_type == MQG_I64)
            MQG_LAUNCH(ctx, "k_assign_slots", s, (k_assign_slots<int64_t><<<cgrid, kBlock, 0, s>>>(ranked, c->num_cached, c->slot_of, static_cast<int64_t *>(c->cached_ids))));
        else
            MQG_LAUNCH(ctx, "k_assign_slots", s, (k_assign_slots<int32_t><<<cgrid, kBlock, 0, s>>>(ranked, c->num_cached, c->slot_of, static_cast<int32_t *>(c->cached_ids))));
        MQG_LAUNCH(ctx, "k_store_i64", s, (k_store_i64<<<1, 64, 0, s>>>(count_dev, c->num_cached)));
        int rc = gather_direct_i32(ctx, ranked, count_dev, c->num_cached, n, c->feats, c->feat_stride * elt, c->cache_rows,
                                   c->cache_stride * elt, int64_t(c->dim) * elt, s);
        if (rc != MQG_OK) return rc;
    }
    // With every temporary in the reserved arena and nothing to report back, the call ends here: the
    // work is enqueued and the arena stays the context's (the next build on it follows on the stream).
    if (!walk_flags && !tmp.allocated_any() && ctx->cache_arena && policy != MQG_CACHE_TOP_DEGREE) return MQG_OK;
    uint32_t flags = 0;
    if (walk_flags) {
        e = hipMemcpyAsync(&flags, walk_flags, sizeof(uint32_t), hipMemcpyDeviceToHost, s);
        if (e != hipSuccess) return fail(ctx, MQG_ERR_HIP, std::string("mqg_build_cache: ") + hipGetErrorString(e));
    }
    e = hipStreamSynchronize(s);                     // temporaries are freed on return
    if (e != hipSuccess) return fail(ctx, MQG_ERR_HIP, std::string("mqg_build_cache: ") + hipGetErrorString(e));
    if (flags & 1u)
        return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_build_cache_ex: a training id lies outside [0, num_nodes); it was skipped and the "
                                               "cache was filled from the remaining ones");
    return MQG_OK;
}

int run_exp_tickets(mqg_ctx *ctx, uint64_t seed, int64_t tag, int64_t first, int64_t n, uint64_t *tickets, hipStream_t s) {
    const uint64_t tag_hash = host_mix64(host_mix64(seed + kGolden) ^ static_cast<uint64_t>(tag));
    MQG_LAUNCH(ctx, "k_exp_tickets", s, (k_exp_tickets<<<static_cast<int>(ceil_div(n, kBlock)), kBlock, 0, s>>>(tag_hash, first, n, tickets)));
    return MQG_OK;
}

// The arena that holds a build's temporaries: room for the largest policy that does not transpose
// the adjacency (scores drawn from a random walk: three score vectors, 64-bit keys, two 32-bit
// sorts and their counter tables), about 75 bytes per node.
int ensure_cache_build_scratch(mqg_ctx *ctx) {
    if (ctx->cache_arena) return MQG_OK;
    const int64_t n = std::max<int64_t>(ctx->num_nodes, 1);
    const int64_t bytes = n * (3 * 8 + 8 + 4 * 4 + 4 * 4 + 2 * 4) + (radix_hist_len_max(n) + radix_scan_tiles_max(n)) * 4 + 64 * 256;
    void *p = nullptr;
    if (hipMalloc(&p, static_cast<size_t>(bytes)) != hipSuccess) {
        (void)hipGetLastError();
        return fail(ctx, MQG_ERR_HIP, "mqg_ctx_reserve: cache-build scratch allocation failed");
    }
    ctx->cache_arena = static_cast<char *>(p);
    ctx->cache_arena_bytes = bytes;
    return MQG_OK;
}

}  // namespace mqg
