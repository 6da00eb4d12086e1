// Feature gather through the hot-node cache (paper Sec. III "Feature Cache", Sec. IV
// "Mini-Batch Transfer To GPU"): out[i] = F[ids[i]], a row coming from the HBM cache when the
// node is cached and from the full feature matrix (pinned host memory, read over the host link
// by the kernel itself) when it is not.
//
//   k_classify        slot_of lookup, ballot-compacted (output row, source row) lists for hits and
//                     misses, one atomic per wavefront and list
//   k_gather_rows<.,0> hits:   HBM cache -> HBM output, one wavefront per row, widest aligned loads
//   k_gather_rows<.,1> misses: feature matrix -> HBM output (same code, separate symbol so that
//                     profiles tell the HBM-bound from the link-bound launch)
//   k_gather_direct   no cache: every row straight from the feature matrix
#include <algorithm>

#include "common.h"
#include "device_utils.h"

namespace mqg {

namespace {

__global__ void k_fill_u64(unsigned long long *p, int n, unsigned long long v) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

__global__ void k_direct_stats(unsigned long long *counters, const int64_t *num_ids, int64_t cap) {
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        int64_t n = *num_ids;
        if (n > cap) n = cap;
        counters[0] = 0;
        counters[1] = static_cast<unsigned long long>(n < 0 ? 0 : n);
    }
}

template <typename IdxT>
__global__ void __launch_bounds__(kBlock)
k_classify(const IdxT *__restrict__ ids, const int64_t *__restrict__ num_ids, int64_t cap,
           const int32_t *__restrict__ slot_of, int2 *__restrict__ hit_list, int2 *__restrict__ miss_list,
           unsigned long long *__restrict__ counters) {
    int64_t n = *num_ids;
    if (n > cap) n = cap;
    const int lane = lane_id();
    const int64_t stride = int64_t(gridDim.x) * kBlock;
    // the loop bound is the same for every lane of a wavefront, so ballots see all 64 lanes
    for (int64_t base = int64_t(blockIdx.x) * kBlock + (threadIdx.x & ~63); base < n; base += stride) {
        int64_t i = base + lane;
        bool valid = i < n;
        int32_t id = 0, slot = -1;
        if (valid) {
            id = static_cast<int32_t>(ids[i]);
            slot = slot_of[id];
        }
        bool hit = valid && slot >= 0, miss = valid && slot < 0;
        uint64_t mh = ballot64(hit), mm = ballot64(miss);
        unsigned long long bh = 0, bm = 0;
        if (lane == 0) {
            if (mh) bh = atomicAdd(&counters[0], static_cast<unsigned long long>(popc64(mh)));
            if (mm) bm = atomicAdd(&counters[1], static_cast<unsigned long long>(popc64(mm)));
        }
        bh = __shfl(bh, 0, 64);
        bm = __shfl(bm, 0, 64);
        if (hit) hit_list[bh + popc64(mh & lanes_below(lane))] = make_int2(static_cast<int>(i), slot);
        if (miss) miss_list[bm + popc64(mm & lanes_below(lane))] = make_int2(static_cast<int>(i), id);
    }
}

template <typename VecT>
__device__ __forceinline__ void copy_row(const VecT *__restrict__ src, VecT *__restrict__ dst, int vecs, int lane) {
    int c = lane;
    for (; c + 3 * kWave < vecs; c += 4 * kWave) {          // four loads in flight per lane
        VecT a = src[c], b = src[c + kWave], d = src[c + 2 * kWave], e = src[c + 3 * kWave];
        dst[c] = a;
        dst[c + kWave] = b;
        dst[c + 2 * kWave] = d;
        dst[c + 3 * kWave] = e;
    }
    for (; c < vecs; c += kWave) dst[c] = src[c];
}

// One wavefront per listed row; list entries are (output row, source row).
template <typename VecT, int MISS>
__global__ void __launch_bounds__(kBlock)
k_gather_rows(const int2 *__restrict__ list, const unsigned long long *__restrict__ count,
              const char *__restrict__ src, int64_t src_stride_bytes, char *__restrict__ dst,
              int64_t dst_stride_bytes, int vecs) {
    const int64_t n = static_cast<int64_t>(*count);
    const int lane = lane_id();
    const int64_t wave0 = int64_t(blockIdx.x) * kWavesPerBlock + (threadIdx.x >> 6);
    const int64_t nwaves = int64_t(gridDim.x) * kWavesPerBlock;
    for (int64_t r = wave0; r < n; r += nwaves) {
        int2 e = list[r];
        copy_row(reinterpret_cast<const VecT *>(src + int64_t(e.y) * src_stride_bytes),
                 reinterpret_cast<VecT *>(dst + int64_t(e.x) * dst_stride_bytes), vecs, lane);
    }
}

template <typename VecT, typename IdxT>
__global__ void __launch_bounds__(kBlock)
k_gather_direct(const IdxT *__restrict__ ids, const int64_t *__restrict__ num_ids, int64_t cap,
                const char *__restrict__ src, int64_t src_stride_bytes, char *__restrict__ dst,
                int64_t dst_stride_bytes, int vecs) {
    int64_t n = *num_ids;
    if (n > cap) n = cap;
    const int lane = lane_id();
    const int64_t wave0 = int64_t(blockIdx.x) * kWavesPerBlock + (threadIdx.x >> 6);
    const int64_t nwaves = int64_t(gridDim.x) * kWavesPerBlock;
    for (int64_t r = wave0; r < n; r += nwaves) {
        int64_t id = static_cast<int64_t>(ids[r]);
        copy_row(reinterpret_cast<const VecT *>(src + id * src_stride_bytes),
                 reinterpret_cast<VecT *>(dst + r * dst_stride_bytes), vecs, lane);
    }
}

// Widest power-of-two access (16, 8, 4 or 2 bytes) that keeps every row of both sides aligned.
int pick_vec_bytes(int64_t row_bytes, int64_t a_stride, int64_t b_stride, const void *a, const void *b) {
    uint64_t bits = static_cast<uint64_t>(row_bytes) | static_cast<uint64_t>(a_stride) | static_cast<uint64_t>(b_stride) |
                    reinterpret_cast<uintptr_t>(a) | reinterpret_cast<uintptr_t>(b);
    for (int v = 16; v > 2; v >>= 1)
        if ((bits & static_cast<uint64_t>(v - 1)) == 0) return v;
    return 2;
}

int gather_grid(int64_t rows) {
    // persistent-style grid: enough wavefronts to fill 256 CUs several times over
    return static_cast<int>(std::min<int64_t>(std::max<int64_t>(1, ceil_div(rows, kWavesPerBlock)), 256 * 16));
}

template <int MISS>
int launch_rows(mqg_ctx *ctx, const char *name, const int2 *list, const unsigned long long *count, int64_t cap,
                const void *src, int64_t src_stride_bytes, void *dst, int64_t dst_stride_bytes,
                int64_t row_bytes, hipStream_t s) {
    const int vb = pick_vec_bytes(row_bytes, src_stride_bytes, dst_stride_bytes, src, dst);
    const int vecs = static_cast<int>(row_bytes / vb);
    const int grid = gather_grid(cap);
    const char *sp = static_cast<const char *>(src);
    char *dp = static_cast<char *>(dst);
    switch (vb) {
        case 16: MQG_LAUNCH(ctx, name, s, (k_gather_rows<uint4, MISS><<<grid, kBlock, 0, s>>>(list, count, sp, src_stride_bytes, dp, dst_stride_bytes, vecs))); break;
        case 8: MQG_LAUNCH(ctx, name, s, (k_gather_rows<uint2, MISS><<<grid, kBlock, 0, s>>>(list, count, sp, src_stride_bytes, dp, dst_stride_bytes, vecs))); break;
        case 4: MQG_LAUNCH(ctx, name, s, (k_gather_rows<uint32_t, MISS><<<grid, kBlock, 0, s>>>(list, count, sp, src_stride_bytes, dp, dst_stride_bytes, vecs))); break;
        default: MQG_LAUNCH(ctx, name, s, (k_gather_rows<uint16_t, MISS><<<grid, kBlock, 0, s>>>(list, count, sp, src_stride_bytes, dp, dst_stride_bytes, vecs))); break;
    }
    return MQG_OK;
}

template <typename IdxT>
int launch_direct(mqg_ctx *ctx, const IdxT *ids, const int64_t *num_ids, int64_t cap, const void *src,
                  int64_t src_stride_bytes, void *dst, int64_t dst_stride_bytes, int64_t row_bytes, hipStream_t s) {
    const int vb = pick_vec_bytes(row_bytes, src_stride_bytes, dst_stride_bytes, src, dst);
    const int vecs = static_cast<int>(row_bytes / vb);
    const int grid = gather_grid(cap);
    const char *sp = static_cast<const char *>(src);
    char *dp = static_cast<char *>(dst);
    switch (vb) {
        case 16: MQG_LAUNCH(ctx, "k_gather_direct", s, (k_gather_direct<uint4, IdxT><<<grid, kBlock, 0, s>>>(ids, num_ids, cap, sp, src_stride_bytes, dp, dst_stride_bytes, vecs))); break;
        case 8: MQG_LAUNCH(ctx, "k_gather_direct", s, (k_gather_direct<uint2, IdxT><<<grid, kBlock, 0, s>>>(ids, num_ids, cap, sp, src_stride_bytes, dp, dst_stride_bytes, vecs))); break;
        case 4: MQG_LAUNCH(ctx, "k_gather_direct", s, (k_gather_direct<uint32_t, IdxT><<<grid, kBlock, 0, s>>>(ids, num_ids, cap, sp, src_stride_bytes, dp, dst_stride_bytes, vecs))); break;
        default: MQG_LAUNCH(ctx, "k_gather_direct", s, (k_gather_direct<uint16_t, IdxT><<<grid, kBlock, 0, s>>>(ids, num_ids, cap, sp, src_stride_bytes, dp, dst_stride_bytes, vecs))); break;
    }
    return MQG_OK;
}

}  // namespace

// Rows listed by 32-bit ids straight from `src` (used by the cache build to fill the cache).
int gather_direct_i32(mqg_ctx *ctx, const int32_t *ids, const int64_t *num_ids, int64_t cap, const void *src,
                      int64_t src_stride_bytes, void *dst, int64_t dst_stride_bytes, int64_t row_bytes,
                      hipStream_t s) {
    return launch_direct<int32_t>(ctx, ids, num_ids, cap, src, src_stride_bytes, dst, dst_stride_bytes, row_bytes, s);
}

int run_gather(mqg_ctx *ctx, const mqg_cache *c, int32_t idx_type, const void *ids, const int64_t *num_ids,
               int64_t cap_ids, void *out, int64_t out_stride, int64_t *stats, hipStream_t s) {
    const int64_t elt = c->dtype == MQG_F16 ? 2 : 4;
    const int64_t row_bytes = int64_t(c->dim) * elt;
    unsigned long long *counters = stats ? reinterpret_cast<unsigned long long *>(stats) : ctx->counters;
    MQG_LAUNCH(ctx, "k_fill_u64", s, (k_fill_u64<<<1, 64, 0, s>>>(counters, 2, 0ull)));
    if (cap_ids == 0) return MQG_OK;

    if (!c->slot_of) {                                   // no cache: everything from feats
        int rc;
        if (idx_type == MQG_I64)
            rc = launch_direct<int64_t>(ctx, static_cast<const int64_t *>(ids), num_ids, cap_ids, c->feats,
                                        c->feat_stride * elt, out, out_stride * elt, row_bytes, s);
        else
            rc = launch_direct<int32_t>(ctx, static_cast<const int32_t *>(ids), num_ids, cap_ids, c->feats,
                                        c->feat_stride * elt, out, out_stride * elt, row_bytes, s);
        if (rc != MQG_OK) return rc;
        // every row counts as served from feats
        MQG_LAUNCH(ctx, "k_direct_stats", s, (k_direct_stats<<<1, 64, 0, s>>>(counters, num_ids, cap_ids)));
        return MQG_OK;
    }

    const int cgrid = static_cast<int>(std::min<int64_t>(std::max<int64_t>(1, ceil_div(cap_ids, kBlock)), 2048));
    if (idx_type == MQG_I64)
        MQG_LAUNCH(ctx, "k_classify", s, (k_classify<int64_t><<<cgrid, kBlock, 0, s>>>(static_cast<const int64_t *>(ids), num_ids, cap_ids, c->slot_of, ctx->hit_list, ctx->miss_list, counters)));
    else
        MQG_LAUNCH(ctx, "k_classify", s, (k_classify<int32_t><<<cgrid, kBlock, 0, s>>>(static_cast<const int32_t *>(ids), num_ids, cap_ids, c->slot_of, ctx->hit_list, ctx->miss_list, counters)));

    int rc = launch_rows<0>(ctx, "k_gather_hit", ctx->hit_list, &counters[0], cap_ids, c->cache_rows,
                            c->cache_stride * elt, out, out_stride * elt, row_bytes, s);
    if (rc != MQG_OK) return rc;
    return launch_rows<1>(ctx, "k_gather_miss", ctx->miss_list, &counters[1], cap_ids, c->feats,
                          c->feat_stride * elt, out, out_stride * elt, row_bytes, s);
}

}  // namespace mqg
