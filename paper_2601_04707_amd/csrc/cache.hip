// Hot-node feature cache construction (paper Sec. III "Feature Cache": the features of a small
// set of high-degree nodes are preloaded on the GPU; Eq. 13 weights nodes by in-degree).
// Deterministic reading: rank all nodes by (degree descending, id ascending) and cache the first
// num_cached; slot s holds the s-th ranked node.
//
// The ranking is a stable least-significant-digit radix sort of (max_degree - degree) with the
// node id as payload: ids start ascending, stable passes keep them ascending inside equal
// degrees.  Only as many 8-bit passes run as max_degree has bytes.
//   k_degrees        degree per node, running maximum
//   k_sort_keys      key = max_degree - degree, payload = id
//   k_radix_hist     per-workgroup digit histogram, laid out [digit][workgroup]
//   k_scan_*         exclusive scan of that table (reduce / one-workgroup scan / apply)
//   k_radix_scatter  stable scatter: ballot match inside a wavefront, LDS counts across the four
//                    wavefronts and across the rounds of a tile
//   k_assign_slots   slot_of / cached_ids
// then the cached rows are copied with the direct gather kernel.
#include <algorithm>
#include <vector>

#include "common.h"
#include "device_utils.h"

namespace mqg {

int gather_direct_i32(mqg_ctx *ctx, const int32_t *ids, const int64_t *num_ids, int64_t cap, const void *src,
                      int64_t src_stride_bytes, void *dst, int64_t dst_stride_bytes, int64_t row_bytes, hipStream_t s);

namespace {

constexpr int kRadixItems = 8;                       // rounds per tile
constexpr int kRadixTile = kBlock * kRadixItems;     // keys per workgroup
constexpr int kScanTile = 1024;                      // elements per workgroup in the generic scan

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
    if (lane_id() == 0 && d > 0) atomicMax(max_deg, d);
}

__global__ void __launch_bounds__(kBlock)
k_sort_keys(uint32_t *__restrict__ keys, int32_t *__restrict__ vals, int64_t n, uint32_t max_deg) {
    int64_t v = int64_t(blockIdx.x) * kBlock + threadIdx.x;
    if (v < n) {
        keys[v] = max_deg - keys[v];                 // in: degree, out: sort key
        vals[v] = static_cast<int32_t>(v);
    }
}

__global__ void __launch_bounds__(kBlock)
k_radix_hist(const uint32_t *__restrict__ keys, int64_t n, int shift, int32_t *__restrict__ hist, int nblocks) {
    __shared__ int h[256];
    h[threadIdx.x] = 0;
    __syncthreads();
    const int64_t base = int64_t(blockIdx.x) * kRadixTile;
#pragma unroll
    for (int r = 0; r < kRadixItems; ++r) {
        int64_t i = base + r * kBlock + threadIdx.x;
        if (i < n) atomicAdd(&h[(keys[i] >> shift) & 255], 1);
    }
    __syncthreads();
    hist[int64_t(threadIdx.x) * nblocks + blockIdx.x] = h[threadIdx.x];
}

__global__ void __launch_bounds__(kBlock)
k_scan_reduce(const int32_t *__restrict__ in, int64_t n, int32_t *__restrict__ tile_sums) {
    __shared__ int lds[kWavesPerBlock];
    const int64_t base = int64_t(blockIdx.x) * kScanTile + threadIdx.x * 4;
    int c = 0;
#pragma unroll
    for (int q = 0; q < 4; ++q)
        if (base + q < n) c += in[base + q];
    int s = wave_sum(c);
    if (lane_id() == 0) lds[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) tile_sums[blockIdx.x] = lds[0] + lds[1] + lds[2] + lds[3];
}

__global__ void __launch_bounds__(kBlock)
k_scan_apply(int32_t *__restrict__ data, int64_t n, const int32_t *__restrict__ tile_base) {
    __shared__ int lds[kWavesPerBlock];
    const int64_t base = int64_t(blockIdx.x) * kScanTile + threadIdx.x * 4;
    int v[4];
    int c = 0;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        v[q] = base + q < n ? data[base + q] : 0;
        c += v[q];
    }
    int total;
    int ex = block_excl_scan<kWavesPerBlock>(c, &total, lds) + tile_base[blockIdx.x];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        if (base + q < n) data[base + q] = ex;
        ex += v[q];
    }
}

__global__ void __launch_bounds__(kBlock)
k_radix_scatter(const uint32_t *__restrict__ keys_in, const int32_t *__restrict__ vals_in, int64_t n, int shift,
                const int32_t *__restrict__ offsets, int nblocks, uint32_t *__restrict__ keys_out,
                int32_t *__restrict__ vals_out) {
    __shared__ int run[256];                         // keys of this digit placed in earlier rounds
    __shared__ int wcnt[kWavesPerBlock][256];        // per wavefront, this round
    __shared__ int gbase[256];                       // first output position of this workgroup per digit
    const int tid = threadIdx.x;
    const int lane = lane_id();
    const int wave = tid >> 6;
    run[tid] = 0;
    gbase[tid] = offsets[int64_t(tid) * nblocks + blockIdx.x];
#pragma unroll
    for (int w = 0; w < kWavesPerBlock; ++w) wcnt[w][tid] = 0;
    __syncthreads();
    const int64_t base = int64_t(blockIdx.x) * kRadixTile;
    for (int r = 0; r < kRadixItems; ++r) {
        const int64_t i = base + r * kBlock + tid;
        const bool valid = i < n;
        uint32_t key = 0;
        int32_t val = 0;
        if (valid) {
            key = keys_in[i];
            val = vals_in[i];
        }
        const int digit = (key >> shift) & 255;
        // lanes of this wavefront holding the same digit
        uint64_t peers = ballot64(valid);
#pragma unroll
        for (int bit = 0; bit < 8; ++bit) {
            uint64_t m = ballot64((digit >> bit) & 1);
            peers &= ((digit >> bit) & 1) ? m : ~m;
        }
        const int rank_in_wave = popc64(peers & lanes_below(lane));
        if (valid && rank_in_wave == 0) wcnt[wave][digit] = popc64(peers);
        __syncthreads();
        if (valid) {
            int before = run[digit];
            for (int w = 0; w < wave; ++w) before += wcnt[w][digit];
            int64_t o = int64_t(gbase[digit]) + before + rank_in_wave;
            keys_out[o] = key;
            vals_out[o] = val;
        }
        __syncthreads();
        {
            int add = 0;
#pragma unroll
            for (int w = 0; w < kWavesPerBlock; ++w) {
                add += wcnt[w][tid];
                wcnt[w][tid] = 0;
            }
            run[tid] += add;
        }
        __syncthreads();
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

struct Temp {
    std::vector<void *> ptrs;
    ~Temp() {
        for (void *p : ptrs) (void)hipFree(p);
    }
    template <typename T>
    bool alloc(T **p, int64_t n) {
        void *q = nullptr;
        if (hipMalloc(&q, static_cast<size_t>(std::max<int64_t>(n, 1)) * sizeof(T)) != hipSuccess) return false;
        ptrs.push_back(q);
        *p = static_cast<T *>(q);
        return true;
    }
};

// exclusive scan of data[0..n) in place
int device_scan(mqg_ctx *ctx, int32_t *data, int64_t n, int32_t *tile_sums, hipStream_t s) {
    const int tiles = static_cast<int>(std::max<int64_t>(1, ceil_div(n, kScanTile)));
    MQG_LAUNCH(ctx, "k_scan_reduce", s, (k_scan_reduce<<<tiles, kBlock, 0, s>>>(data, n, tile_sums)));
    int rc = launch_scan_tiles(ctx, tile_sums, tiles, nullptr, nullptr, nullptr, s);
    if (rc != MQG_OK) return rc;
    MQG_LAUNCH(ctx, "k_scan_apply", s, (k_scan_apply<<<tiles, kBlock, 0, s>>>(data, n, tile_sums)));
    return MQG_OK;
}

}  // namespace

int run_build_cache(mqg_ctx *ctx, const mqg_graph *g, mqg_cache *c, hipStream_t s) {
    const int64_t n = g->num_nodes;
    const int64_t elt = c->dtype == MQG_F16 ? 2 : 4;
    hipError_t e = hipMemsetAsync(c->slot_of, 0xFF, static_cast<size_t>(std::max<int64_t>(n, 1)) * sizeof(int32_t), s);
    if (e != hipSuccess) return fail(ctx, MQG_ERR_HIP, std::string("hipMemsetAsync: ") + hipGetErrorString(e));
    if (n == 0 || c->num_cached == 0) {
        e = hipStreamSynchronize(s);
        return e == hipSuccess ? MQG_OK : fail(ctx, MQG_ERR_HIP, hipGetErrorString(e));
    }

    Temp tmp;
    uint32_t *keys_a, *keys_b, *max_deg_dev;
    int32_t *vals_a, *vals_b, *hist, *tile_sums;
    int64_t *count_dev;
    const int nblocks = static_cast<int>(ceil_div(n, kRadixTile));
    const int64_t hist_len = int64_t(256) * nblocks;
    bool ok = tmp.alloc(&keys_a, n) && tmp.alloc(&keys_b, n) && tmp.alloc(&vals_a, n) && tmp.alloc(&vals_b, n) &&
              tmp.alloc(&hist, hist_len) && tmp.alloc(&tile_sums, ceil_div(hist_len, kScanTile) + 1) &&
              tmp.alloc(&max_deg_dev, 1) && tmp.alloc(&count_dev, 1);
    if (!ok) return fail(ctx, MQG_ERR_HIP, "mqg_build_cache: temporary allocation failed");

    const int ngrid = static_cast<int>(ceil_div(n, kBlock));
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
    int passes = 0;
    while (passes < 4 && (max_deg >> (8 * passes)) != 0) ++passes;
    uint32_t *kin = keys_a, *kout = keys_b;
    int32_t *vin = vals_a, *vout = vals_b;
    for (int p = 0; p < passes; ++p) {
        const int shift = 8 * p;
        MQG_LAUNCH(ctx, "k_radix_hist", s, (k_radix_hist<<<nblocks, kBlock, 0, s>>>(kin, n, shift, hist, nblocks)));
        int rc = device_scan(ctx, hist, hist_len, tile_sums, s);
        if (rc != MQG_OK) return rc;
        MQG_LAUNCH(ctx, "k_radix_scatter", s,
                   (k_radix_scatter<<<nblocks, kBlock, 0, s>>>(kin, vin, n, shift, hist, nblocks, kout, vout)));
        std::swap(kin, kout);
        std::swap(vin, vout);
    }
    // vin: node ids by (degree descending, id ascending)
    const int cgrid = static_cast<int>(ceil_div(c->num_cached, kBlock));
    if (g->idx_type == MQG_I64)
        MQG_LAUNCH(ctx, "k_assign_slots", s, (k_assign_slots<int64_t><<<cgrid, kBlock, 0, s>>>(vin, c->num_cached, c->slot_of, static_cast<int64_t *>(c->cached_ids))));
    else
        MQG_LAUNCH(ctx, "k_assign_slots", s, (k_assign_slots<int32_t><<<cgrid, kBlock, 0, s>>>(vin, c->num_cached, c->slot_of, static_cast<int32_t *>(c->cached_ids))));
    MQG_LAUNCH(ctx, "k_store_i64", s, (k_store_i64<<<1, 64, 0, s>>>(count_dev, c->num_cached)));
    int rc = gather_direct_i32(ctx, vin, count_dev, c->num_cached, c->feats, c->feat_stride * elt, c->cache_rows,
                               c->cache_stride * elt, int64_t(c->dim) * elt, s);
    if (rc != MQG_OK) return rc;
    e = hipStreamSynchronize(s);                     // temporaries are freed on return
    if (e != hipSuccess) return fail(ctx, MQG_ERR_HIP, std::string("mqg_build_cache: ") + hipGetErrorString(e));
    return MQG_OK;
}

}  // namespace mqg
