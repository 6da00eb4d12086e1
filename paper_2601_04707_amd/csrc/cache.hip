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
//   (radix passes)   see radix.hip
//   k_assign_slots   slot_of / cached_ids
// then the cached rows are copied with the direct gather kernel.
#include <algorithm>
#include <vector>

#include "common.h"
#include "device_utils.h"
#include "radix.h"

namespace mqg {

int gather_direct_i32(mqg_ctx *ctx, const int32_t *ids, const int64_t *num_ids, int64_t cap, const void *src,
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
    uint32_t *keys_a, *max_deg_dev;
    int32_t *vals_a;
    int64_t *count_dev;
    RadixBufs rb;
    bool ok = tmp.alloc(&keys_a, n) && tmp.alloc(&vals_a, n) && tmp.alloc(&rb.keys[0], n) && tmp.alloc(&rb.keys[1], n) &&
              tmp.alloc(&rb.vals[0], n) && tmp.alloc(&rb.vals[1], n) && tmp.alloc(&rb.hist, radix_hist_len(n)) &&
              tmp.alloc(&rb.tile_sums, radix_scan_tiles(n)) && tmp.alloc(&max_deg_dev, 1) && tmp.alloc(&count_dev, 1);
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
    int bits = 0;
    while (bits < 32 && (max_deg >> bits) != 0) bits += 8;
    int which = -1;
    int rc0 = radix_sort_pairs(ctx, keys_a, vals_a, rb, n, nullptr, bits, s, &which);
    if (rc0 != MQG_OK) return rc0;
    const int32_t *vin = which < 0 ? vals_a : rb.vals[which];
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
