// Frontier dedup and relabel with a global open-addressing hash table plus a sort - the
// alternative to the node-indexed bitmap/local_of[] path of sample.hip, selected per context with
// MQG_OPT_DEDUP_HASH.  It needs memory proportional to the mini-batch instead of the graph (16
// bytes per potential source node of the largest block instead of 4.2 bytes per graph node) and
// produces exactly the same blocks; it exists for graphs whose node count makes the node-indexed
// tables unaffordable, and to measure one design against the other.
//
// The table maps a global node id to its position in the current source list.  After block l it
// holds exactly S_l, which is D_{l-1}: only the seeds are ever inserted as destinations.
//   k_hash_put_dst   seeds -> (id, position); a repeated seed is flagged
//   k_hash_put_nbr   every sampled neighbour: found -> nothing; absent -> inserted as "new", and the
//                    winner of the insertion appends the id to the list of new nodes (ballot
//                    compaction, one atomic per wavefront)
//   (radix sort)     the new ids, ascending
//   k_hash_assign    new id r gets position num_dst + r, in the source list and in the table
//   k_hash_relabel   indices[e] = table[neighbour e]
// The table is cleared with one memset at the end of the call.
#include <algorithm>

#include "common.h"
#include "device_utils.h"
#include "radix.h"

namespace mqg {

namespace {

constexpr unsigned long long kEmpty = ~0ull;
constexpr uint32_t kNewMark = 0xFFFFFFFEu;

__device__ __forceinline__ uint32_t slot_of_key(uint32_t key, uint32_t mask) {
    key *= 0x9E3779B1u;                                    // Fibonacci hashing
    key ^= key >> 15;
    return key & mask;
}
__device__ __forceinline__ unsigned long long pack(uint32_t key, uint32_t val) {
    return (static_cast<unsigned long long>(key) << 32) | val;
}

template <typename IdxT>
__global__ void __launch_bounds__(kBlock)
k_hash_put_dst(const IdxT *__restrict__ dst, const int64_t *__restrict__ sizes, unsigned long long *__restrict__ table,
               uint32_t mask, int32_t *__restrict__ seed_flags) {
    const int64_t n = sizes[0];
    const int64_t i = int64_t(blockIdx.x) * kBlock + threadIdx.x;
    if (i >= n) return;
    const uint32_t key = static_cast<uint32_t>(dst[i]);
    uint32_t slot = slot_of_key(key, mask);
    for (uint32_t probes = 0; probes <= mask; ++probes) {  // the table is at most half full: ends early
        unsigned long long old = atomicCAS(&table[slot], kEmpty, pack(key, static_cast<uint32_t>(i)));
        if (old == kEmpty) return;
        if (static_cast<uint32_t>(old >> 32) == key) {     // the same seed twice
            atomicOr(seed_flags, 2);
            return;
        }
        slot = (slot + 1) & mask;
    }
}

__global__ void __launch_bounds__(kBlock)
k_hash_put_nbr(const int32_t *__restrict__ nbr, const int64_t *__restrict__ sizes, unsigned long long *__restrict__ table,
               uint32_t mask, uint32_t *__restrict__ new_keys, unsigned long long *__restrict__ new_count) {
    const int64_t nnz = sizes[2];
    const int lane = lane_id();
    const int64_t stride = int64_t(gridDim.x) * kBlock;
    for (int64_t base = int64_t(blockIdx.x) * kBlock + (threadIdx.x & ~63); base < nnz; base += stride) {
        const int64_t e = base + lane;
        bool won = false;
        uint32_t key = 0;
        if (e < nnz) {
            key = static_cast<uint32_t>(nbr[e]);
            uint32_t slot = slot_of_key(key, mask);
            for (uint32_t probes = 0; probes <= mask; ++probes) {
                unsigned long long cur = __hip_atomic_load(&table[slot], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (cur == kEmpty) {
                    cur = atomicCAS(&table[slot], kEmpty, pack(key, kNewMark));
                    if (cur == kEmpty) {
                        won = true;
                        break;
                    }
                }
                if (static_cast<uint32_t>(cur >> 32) == key) break;
                slot = (slot + 1) & mask;
            }
        }
        const uint64_t m = ballot64(won);
        if (m) {
            unsigned long long b = 0;
            if (lane == 0) b = atomicAdd(new_count, static_cast<unsigned long long>(popc64(m)));
            b = __shfl(b, 0, 64);
            if (won) new_keys[b + popc64(m & lanes_below(lane))] = key;
        }
    }
}

template <typename IdxT>
__global__ void __launch_bounds__(kBlock)
k_hash_assign(const uint32_t *__restrict__ sorted_keys, const unsigned long long *__restrict__ new_count,
              int64_t *sizes, int64_t *sizes_next, IdxT *__restrict__ src_ids,
              unsigned long long *__restrict__ table, uint32_t mask) {
    const int64_t cnt = static_cast<int64_t>(*new_count);
    const int64_t nd = sizes[0];
    const int64_t stride = int64_t(gridDim.x) * kBlock;
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        sizes[1] = nd + cnt;
        if (sizes_next) sizes_next[0] = nd + cnt;
    }
    for (int64_t r = int64_t(blockIdx.x) * kBlock + threadIdx.x; r < cnt; r += stride) {
        const uint32_t key = sorted_keys[r];
        src_ids[nd + r] = static_cast<IdxT>(key);
        uint32_t slot = slot_of_key(key, mask);
        for (uint32_t probes = 0; probes <= mask; ++probes) {
            if (static_cast<uint32_t>(table[slot] >> 32) == key) {
                table[slot] = pack(key, static_cast<uint32_t>(nd + r));
                break;
            }
            slot = (slot + 1) & mask;
        }
    }
}

__global__ void __launch_bounds__(kBlock)
k_hash_relabel(const int32_t *__restrict__ nbr, const int64_t *__restrict__ sizes,
               const unsigned long long *__restrict__ table, uint32_t mask, int32_t *__restrict__ indices) {
    const int64_t nnz = sizes[2];
    const int64_t stride = int64_t(gridDim.x) * kBlock;
    for (int64_t e = int64_t(blockIdx.x) * kBlock + threadIdx.x; e < nnz; e += stride) {
        const uint32_t key = static_cast<uint32_t>(nbr[e]);
        uint32_t slot = slot_of_key(key, mask);
        int32_t pos = -1;
        for (uint32_t probes = 0; probes <= mask; ++probes) {
            const unsigned long long cur = table[slot];
            if (static_cast<uint32_t>(cur >> 32) == key) {
                pos = static_cast<int32_t>(static_cast<uint32_t>(cur));
                break;
            }
            if (cur == kEmpty) break;                      // cannot happen: every neighbour was inserted
            slot = (slot + 1) & mask;
        }
        indices[e] = pos;
    }
}

__global__ void k_zero_u64(unsigned long long *p) {
    if (blockIdx.x == 0 && threadIdx.x == 0) *p = 0;
}

}  // namespace

void free_hash_scratch(mqg_ctx *ctx) {
    (void)hipFree(ctx->hash_table);
    (void)hipFree(ctx->hash_new_keys);
    (void)hipFree(ctx->hash_new_count);
    (void)hipFree(ctx->hash_sort.keys[0]);
    (void)hipFree(ctx->hash_sort.keys[1]);
    (void)hipFree(ctx->hash_sort.vals[0]);
    (void)hipFree(ctx->hash_sort.vals[1]);
    (void)hipFree(ctx->hash_sort.hist);
    (void)hipFree(ctx->hash_sort.tile_sums);
    ctx->hash_table = nullptr;
    ctx->hash_new_keys = nullptr;
    ctx->hash_new_count = nullptr;
    ctx->hash_sort = RadixBufs{};
    ctx->hash_capacity = 0;
}

// Scratch of the hash path, sized by the context's bounds; allocated when the option is first used.
int ensure_hash_scratch(mqg_ctx *ctx) {
    if (ctx->hash_table) return MQG_OK;
    int64_t cap = 1024;
    while (cap < 2 * (ctx->max_src + 1)) cap <<= 1;        // at most half full
    if (cap > (int64_t(1) << 31)) return fail(ctx, MQG_ERR_UNSUPPORTED, "hash dedup: source lists too large");
    const int64_t nn = std::max<int64_t>(ctx->max_nnz, 1);
    auto alloc = [&](void **p, int64_t bytes) { return hipMalloc(p, static_cast<size_t>(std::max<int64_t>(bytes, 8))) == hipSuccess; };
    bool ok = alloc(reinterpret_cast<void **>(&ctx->hash_table), cap * 8) &&
              alloc(reinterpret_cast<void **>(&ctx->hash_new_keys), nn * 4) &&
              alloc(reinterpret_cast<void **>(&ctx->hash_new_count), 8) &&
              alloc(reinterpret_cast<void **>(&ctx->hash_sort.keys[0]), nn * 4) &&
              alloc(reinterpret_cast<void **>(&ctx->hash_sort.keys[1]), nn * 4) &&
              alloc(reinterpret_cast<void **>(&ctx->hash_sort.vals[0]), nn * 4) &&
              alloc(reinterpret_cast<void **>(&ctx->hash_sort.vals[1]), nn * 4) &&
              alloc(reinterpret_cast<void **>(&ctx->hash_sort.hist), radix_hist_len_max(nn) * 4) &&
              alloc(reinterpret_cast<void **>(&ctx->hash_sort.tile_sums), radix_scan_tiles_max(nn) * 4);
    if (ok) ok = hipMemset(ctx->hash_table, 0xFF, static_cast<size_t>(cap) * 8) == hipSuccess;
    if (ok) ok = hipDeviceSynchronize() == hipSuccess;
    if (!ok) {
        free_hash_scratch(ctx);
        return fail(ctx, MQG_ERR_HIP, "hash dedup: scratch allocation failed");
    }
    ctx->hash_capacity = cap;
    return MQG_OK;
}

template <typename IdxT>
int hash_put_seeds_t(mqg_ctx *ctx, const IdxT *seeds, int64_t need_dst, const int64_t *sizes, hipStream_t s) {
    const int grid = static_cast<int>(std::max<int64_t>(1, ceil_div(need_dst, kBlock)));
    MQG_LAUNCH(ctx, "k_hash_put_dst", s,
               (k_hash_put_dst<IdxT><<<grid, kBlock, 0, s>>>(seeds, sizes, ctx->hash_table, static_cast<uint32_t>(ctx->hash_capacity - 1),
                                                             ctx->heavy_count + MQG_MAX_LAYERS)));
    return MQG_OK;
}

int hash_put_seeds(mqg_ctx *ctx, const void *seeds, int idx_type, int64_t need_dst, const int64_t *sizes, hipStream_t s) {
    if (idx_type == MQG_I64) return hash_put_seeds_t(ctx, static_cast<const int64_t *>(seeds), need_dst, sizes, s);
    return hash_put_seeds_t(ctx, static_cast<const int32_t *>(seeds), need_dst, sizes, s);
}

// One block's dedup + relabel: nbr[0..nnz) -> new source ids (ascending) appended to src_ids, indices.
int hash_dedup_block(mqg_ctx *ctx, const int32_t *nbr, int64_t need_nnz, int64_t num_nodes, int idx_type, void *src_ids,
                     int64_t *sizes, int64_t *sizes_next, int32_t *indices, hipStream_t s) {
    const uint32_t mask = static_cast<uint32_t>(ctx->hash_capacity - 1);
    const int egrid = static_cast<int>(std::min<int64_t>(std::max<int64_t>(1, ceil_div(need_nnz, kBlock)), 4096));
    MQG_LAUNCH(ctx, "k_zero_u64", s, (k_zero_u64<<<1, 64, 0, s>>>(ctx->hash_new_count)));
    MQG_LAUNCH(ctx, "k_hash_put_nbr", s,
               (k_hash_put_nbr<<<egrid, kBlock, 0, s>>>(nbr, sizes, ctx->hash_table, mask, ctx->hash_new_keys, ctx->hash_new_count)));
    const int bits = radix_key_bits(static_cast<uint64_t>(std::max<int64_t>(num_nodes, 1) - 1));
    int which = -1;
    int rc = radix_sort_pairs(ctx, ctx->hash_new_keys, reinterpret_cast<const int32_t *>(ctx->hash_new_keys), ctx->hash_sort,
                              std::min<int64_t>(std::max<int64_t>(need_nnz, 1), std::max<int64_t>(ctx->max_nnz, 1)), reinterpret_cast<const int64_t *>(ctx->hash_new_count), bits, s, &which);
    if (rc != MQG_OK) return rc;
    const uint32_t *sorted = which < 0 ? ctx->hash_new_keys : ctx->hash_sort.keys[which];
    if (idx_type == MQG_I64)
        MQG_LAUNCH(ctx, "k_hash_assign", s,
                   (k_hash_assign<int64_t><<<egrid, kBlock, 0, s>>>(sorted, ctx->hash_new_count, sizes, sizes_next,
                                                                    static_cast<int64_t *>(src_ids), ctx->hash_table, mask)));
    else
        MQG_LAUNCH(ctx, "k_hash_assign", s,
                   (k_hash_assign<int32_t><<<egrid, kBlock, 0, s>>>(sorted, ctx->hash_new_count, sizes, sizes_next,
                                                                    static_cast<int32_t *>(src_ids), ctx->hash_table, mask)));
    MQG_LAUNCH(ctx, "k_hash_relabel", s, (k_hash_relabel<<<egrid, kBlock, 0, s>>>(nbr, sizes, ctx->hash_table, mask, indices)));
    return MQG_OK;
}

int hash_clear(mqg_ctx *ctx, hipStream_t s) {
    hipError_t e = hipMemsetAsync(ctx->hash_table, 0xFF, static_cast<size_t>(ctx->hash_capacity) * 8, s);
    if (e != hipSuccess) return fail(ctx, MQG_ERR_HIP, std::string("hash dedup: ") + hipGetErrorString(e));
    return MQG_OK;
}

}  // namespace mqg
