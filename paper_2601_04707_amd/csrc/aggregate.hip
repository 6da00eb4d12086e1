// GraphSAGE mean aggregation over one block and its backward (paper Eq. 16: Z_agg(v) =
// Mean(H(v)), the GA step "AH" of Sec. IV "Computation"; the backward of GA is the transposed
// product "AG").  Both are segmented reductions over rows of a sparse operator: HBM-bound, no
// dense contraction, hence no matrix cores.
//
// One wavefront per output row.
//   k_segment_reduce       rows of at most 64*VEC columns: the 64 lanes are split into G groups of
//                          LPR lanes; the lanes of a group cover the feature columns with VEC-wide
//                          loads and group g takes the row's entries g, g+G, ...; the G partial
//                          sums are then folded across groups.  (Also the generic fallback: one
//                          group, one column pass after the other.)
//   k_segment_reduce_wide  wider rows: a lane owns PASSES column chunks and keeps all of them in
//                          registers, so every input row is fetched with PASSES independent loads
//                          in flight; the row's entries are loaded 64 at a time, one per lane, and
//                          broadcast with v_readlane.
// Forward: output row i reduces x[indices[e]] over the edges e of destination i and divides by
// their number.  Backward: output row s reduces grad_out[i] / n_i over the edges that point to
// source s, taken from the block's edge list sorted by source (stable radix sort, so a row's terms
// are always added in ascending destination order: the result is reproducible bit for bit).
// Sums are fp32; fp16 output is rounded once (to nearest even) at the store.
#include <hip/hip_fp16.h>

#include <algorithm>

#include "common.h"
#include "device_utils.h"
#include "radix.h"

namespace mqg {

namespace {

template <typename T, int VEC>
struct alignas(sizeof(T) * VEC) Pack {
    T v[VEC];
};

__device__ __forceinline__ float to_f32(float x) { return x; }
__device__ __forceinline__ float to_f32(_Float16 x) { return static_cast<float>(x); }
__device__ __forceinline__ void from_f32(float x, float *o) { *o = x; }
__device__ __forceinline__ void from_f32(float x, _Float16 *o) { *o = static_cast<_Float16>(x); }

// Forward: entries of output row i are the block's edges of destination i.
struct ForwardRows {
    static constexpr bool kWeighted = false;
    static constexpr bool kSelf = false;
    __device__ __forceinline__ float self_weight(int64_t) const { return 0.f; }
    const int32_t *indptr;
    const int32_t *indices;
    __device__ __forceinline__ int begin(int64_t i) const { return indptr[i]; }
    __device__ __forceinline__ int end(int64_t i) const { return indptr[i + 1]; }
    __device__ __forceinline__ int input_row(int p) const { return indices[p]; }
    __device__ __forceinline__ float weight(int) const { return 1.f; }
    __device__ __forceinline__ float finish(float acc, int count) const { return count > 0 ? acc / static_cast<float>(count) : 0.f; }
};

// Backward: entries of output row s are the edges pointing to source s; each contributes the
// gradient row of its destination scaled by one over that destination's edge count.
struct BackwardRows {
    static constexpr bool kWeighted = true;
    static constexpr bool kSelf = false;
    __device__ __forceinline__ float self_weight(int64_t) const { return 0.f; }
    const int32_t *col_ptr;     // [num_src + 1] offsets into dst_rows
    const int32_t *dst_rows;    // [nnz] destination row of every edge, edges ordered by source
    const int32_t *indptr;      // the block's forward offsets, for the edge counts
    __device__ __forceinline__ int begin(int64_t s) const { return col_ptr[s]; }
    __device__ __forceinline__ int end(int64_t s) const { return col_ptr[s + 1]; }
    __device__ __forceinline__ int input_row(int p) const { return dst_rows[p]; }
    __device__ __forceinline__ float weight(int p) const {
        const int i = dst_rows[p];
        return 1.f / static_cast<float>(indptr[i + 1] - indptr[i]);
    }
    __device__ __forceinline__ float finish(float acc, int) const { return acc; }
};

// Weighted forward (the sampled estimator of the graph convolution, paper Eq. 1-3, or any other
// per-edge weights): out[i] = self_w[i] x[i] + sum over the edges p of row i of edge_w[p] x[indices[p]].
struct WeightedRows {
    static constexpr bool kWeighted = true;
    static constexpr bool kSelf = true;
    const int32_t *indptr;
    const int32_t *indices;
    const float *edge_w;
    const float *self_w;        // may be null: no diagonal term
    __device__ __forceinline__ int begin(int64_t i) const { return indptr[i]; }
    __device__ __forceinline__ int end(int64_t i) const { return indptr[i + 1]; }
    __device__ __forceinline__ int input_row(int p) const { return indices[p]; }
    __device__ __forceinline__ float weight(int p) const { return edge_w[p]; }
    __device__ __forceinline__ float self_weight(int64_t i) const { return self_w ? self_w[i] : 0.f; }
    __device__ __forceinline__ float finish(float acc, int) const { return acc; }
};

// Its transpose: output row s reduces edge_w * grad_out[destination] over the edges pointing to
// source s (ordered by source, stable), plus self_w[s] * grad_out[s] where s is a destination.
struct WeightedBackwardRows {
    static constexpr bool kWeighted = true;
    static constexpr bool kSelf = true;
    const int32_t *col_ptr;
    const int32_t *dst_rows;
    const float *w_sorted;      // edge weights in the by-source order
    const float *self_w;
    const int64_t *sizes;
    __device__ __forceinline__ int begin(int64_t s) const { return col_ptr[s]; }
    __device__ __forceinline__ int end(int64_t s) const { return col_ptr[s + 1]; }
    __device__ __forceinline__ int input_row(int p) const { return dst_rows[p]; }
    __device__ __forceinline__ float weight(int p) const { return w_sorted[p]; }
    __device__ __forceinline__ float self_weight(int64_t s) const { return (self_w && s < sizes[0]) ? self_w[s] : 0.f; }
    __device__ __forceinline__ float finish(float acc, int) const { return acc; }
};

template <typename T, int VEC, typename Rows>
__global__ void __launch_bounds__(kBlock)
k_segment_reduce(Rows rows, const int64_t *__restrict__ n_rows, const T *__restrict__ x, int64_t x_stride,
                 T *__restrict__ out, int64_t out_stride, int dim, int log2_lpr) {
    using P = Pack<T, VEC>;
    const int lane = lane_id();
    const int lpr = 1 << log2_lpr;
    const int groups = kWave >> log2_lpr;
    const int g = lane >> log2_lpr;
    const int gl = lane & (lpr - 1);
    const int64_t n = *n_rows;
    const int64_t wave0 = int64_t(blockIdx.x) * kWavesPerBlock + (threadIdx.x >> 6);
    const int64_t nwaves = int64_t(gridDim.x) * kWavesPerBlock;
    for (int64_t i = wave0; i < n; i += nwaves) {
        const int b = rows.begin(i), e = rows.end(i);
        // every lane of the wavefront runs the same number of column passes (shuffles below)
        const int passes = (dim + lpr * VEC - 1) / (lpr * VEC);
        for (int ps = 0; ps < passes; ++ps) {
            const int col0 = (ps * lpr + gl) * VEC;
            const bool live = col0 < dim;
            float acc[VEC];
#pragma unroll
            for (int q = 0; q < VEC; ++q) acc[q] = 0.f;
            if (Rows::kSelf) {                             // the diagonal term: the row's own input row
                const float ws = rows.self_weight(i);
                if (ws != 0.f && live && g == 0) {
                    P v = *reinterpret_cast<const P *>(x + i * x_stride + col0);
#pragma unroll
                    for (int q = 0; q < VEC; ++q) acc[q] = ws * to_f32(v.v[q]);
                }
            }
#pragma unroll 4
            for (int p = b + g; p < e; p += groups) {
                const int64_t r = rows.input_row(p);
                const float w = rows.weight(p);
                if (live) {
                    P v = *reinterpret_cast<const P *>(x + r * x_stride + col0);
#pragma unroll
                    for (int q = 0; q < VEC; ++q) {
                        if (Rows::kWeighted) acc[q] += w * to_f32(v.v[q]);
                        else acc[q] += to_f32(v.v[q]);
                    }
                }
            }
            for (int off = lpr; off < kWave; off <<= 1) {
#pragma unroll
                for (int q = 0; q < VEC; ++q) acc[q] += __shfl_xor(acc[q], off, 64);
            }
            if (live && g == 0) {
                P o;
#pragma unroll
                for (int q = 0; q < VEC; ++q) from_f32(rows.finish(acc[q], e - b), &o.v[q]);
                *reinterpret_cast<P *>(out + i * out_stride + col0) = o;
            }
        }
    }
}

template <typename T, int VEC, int PASSES, typename Rows>
__global__ void __launch_bounds__(kBlock)
k_segment_reduce_wide(Rows rows, const int64_t *__restrict__ n_rows, const T *__restrict__ x, int64_t x_stride,
                      T *__restrict__ out, int64_t out_stride, int dim) {
    using P = Pack<T, VEC>;
    const int lane = lane_id();
    const int64_t n = *n_rows;
    const int64_t wave0 = int64_t(blockIdx.x) * kWavesPerBlock + (threadIdx.x >> 6);
    const int64_t nwaves = int64_t(gridDim.x) * kWavesPerBlock;
    bool live[PASSES];
#pragma unroll
    for (int ps = 0; ps < PASSES; ++ps) live[ps] = (ps * kWave + lane) * VEC < dim;
    for (int64_t i = wave0; i < n; i += nwaves) {
        const int b = rows.begin(i), e = rows.end(i);
        float acc[PASSES][VEC];
#pragma unroll
        for (int ps = 0; ps < PASSES; ++ps)
#pragma unroll
            for (int q = 0; q < VEC; ++q) acc[ps][q] = 0.f;
        if (Rows::kSelf) {
            const float ws = rows.self_weight(i);
            if (ws != 0.f) {
                const T *row = x + i * x_stride + lane * VEC;
#pragma unroll
                for (int ps = 0; ps < PASSES; ++ps)
                    if (live[ps]) {
                        P v = *reinterpret_cast<const P *>(row + ps * kWave * VEC);
#pragma unroll
                        for (int q = 0; q < VEC; ++q) acc[ps][q] = ws * to_f32(v.v[q]);
                    }
            }
        }
        for (int c0 = b; c0 < e; c0 += kWave) {            // entries 64 at a time, one per lane
            const int m = e - c0 < kWave ? e - c0 : kWave;
            const int my_row = lane < m ? rows.input_row(c0 + lane) : 0;
            const float my_w = lane < m ? rows.weight(c0 + lane) : 0.f;
            auto load_row = [&](int t, P *v) {
                const int64_t r = static_cast<int>(readlane32(static_cast<uint32_t>(my_row), t));
                const T *row = x + r * x_stride + lane * VEC;
#pragma unroll
                for (int ps = 0; ps < PASSES; ++ps)
                    if (live[ps]) v[ps] = *reinterpret_cast<const P *>(row + ps * kWave * VEC);
            };
            auto add_row = [&](int t, const P *v) {
                const float w = __uint_as_float(readlane32(__float_as_uint(my_w), t));
#pragma unroll
                for (int ps = 0; ps < PASSES; ++ps)
                    if (live[ps]) {
#pragma unroll
                        for (int q = 0; q < VEC; ++q) {
                            if (Rows::kWeighted) acc[ps][q] += w * to_f32(v[ps].v[q]);
                            else acc[ps][q] += to_f32(v[ps].v[q]);
                        }
                    }
            };
            int t = 0;
            for (; t + 1 < m; t += 2) {                    // two input rows (2*PASSES loads) in flight
                P v0[PASSES], v1[PASSES];
                load_row(t, v0);
                load_row(t + 1, v1);
                add_row(t, v0);
                add_row(t + 1, v1);
            }
            if (t < m) {
                P v0[PASSES];
                load_row(t, v0);
                add_row(t, v0);
            }
        }
        T *orow = out + i * out_stride + lane * VEC;
#pragma unroll
        for (int ps = 0; ps < PASSES; ++ps)
            if (live[ps]) {
                P o;
#pragma unroll
                for (int q = 0; q < VEC; ++q) from_f32(rows.finish(acc[ps][q], e - b), &o.v[q]);
                *reinterpret_cast<P *>(orow + ps * kWave * VEC) = o;
            }
    }
}

template <typename T, typename Rows>
int launch(mqg_ctx *ctx, const char *name, const Rows &rows, const int64_t *n_rows, int64_t cap_rows, const T *x,
           int64_t x_stride, T *out, int64_t out_stride, int dim, hipStream_t s) {
    // widest vector (<= 16 bytes) that divides dim and both strides and keeps the bases aligned.
    // When both strides leave room, dim is first rounded up to whole 16-byte words: the extra
    // columns are read from the input rows' padding and written to the output rows' padding.
    int vec = 16 / static_cast<int>(sizeof(T));
    {
        const int dim16 = static_cast<int>(ceil_div(dim, vec)) * vec;
        if (dim16 <= x_stride && dim16 <= out_stride && x_stride % vec == 0 && out_stride % vec == 0) dim = dim16;
    }
    auto ok = [&](int v) {
        int64_t bytes = int64_t(v) * sizeof(T);
        return dim % v == 0 && x_stride % v == 0 && out_stride % v == 0 &&
               reinterpret_cast<uintptr_t>(x) % bytes == 0 && reinterpret_cast<uintptr_t>(out) % bytes == 0;
    };
    while (vec > 1 && !ok(vec)) vec >>= 1;
    int lanes = static_cast<int>(ceil_div(dim, vec));
    int log2_lpr = 0;
    while ((1 << log2_lpr) < lanes && log2_lpr < 6) ++log2_lpr;
    const int grid = static_cast<int>(std::min<int64_t>(std::max<int64_t>(1, ceil_div(cap_rows, kWavesPerBlock)), 256 * 32));
    const int passes = static_cast<int>(ceil_div(lanes, kWave));
#define MQG_AGG(V)                                                                                              \
    MQG_LAUNCH(ctx, name, s,                                                                                    \
               (k_segment_reduce<T, V, Rows><<<grid, kBlock, 0, s>>>(rows, n_rows, x, x_stride, out, out_stride, dim, log2_lpr)))
#define MQG_AGG_WIDE(V, PS)                                                                                     \
    MQG_LAUNCH(ctx, name, s,                                                                                    \
               (k_segment_reduce_wide<T, V, PS, Rows><<<grid, kBlock, 0, s>>>(rows, n_rows, x, x_stride, out, out_stride, dim)))
#define MQG_AGG_PICK(V)                        \
    switch (passes) {                          \
        case 1: MQG_AGG(V); break;             \
        case 2: MQG_AGG_WIDE(V, 2); break;     \
        case 3: MQG_AGG_WIDE(V, 3); break;     \
        case 4: MQG_AGG_WIDE(V, 4); break;     \
        case 5: MQG_AGG_WIDE(V, 5); break;     \
        case 6: MQG_AGG_WIDE(V, 6); break;     \
        default: MQG_AGG(V); break;            \
    }
    constexpr int kWidest = 16 / static_cast<int>(sizeof(T));
    if (vec == kWidest) {
        MQG_AGG_PICK(kWidest);
    } else if (vec == kWidest / 2) {
        MQG_AGG_PICK(kWidest / 2);
    } else if (vec == 2 && kWidest == 8) {
        MQG_AGG(2);
    } else {
        MQG_AGG(1);
    }
#undef MQG_AGG_PICK
#undef MQG_AGG_WIDE
#undef MQG_AGG
    return MQG_OK;
}

// ---------------------------------------------------------------- edges ordered by source

// payload of edge e = its destination row, found by bisection of indptr (the keys are `indices`)
__global__ void __launch_bounds__(kBlock)
k_edge_dst_rows(const int32_t *__restrict__ indptr, const int64_t *__restrict__ sizes, int32_t *__restrict__ dst_row) {
    const int64_t num_dst = sizes[0], nnz = sizes[2];
    const int64_t stride = int64_t(gridDim.x) * kBlock;
    for (int64_t e = int64_t(blockIdx.x) * kBlock + threadIdx.x; e < nnz; e += stride) {
        int64_t lo = 0, hi = num_dst;                      // largest i with indptr[i] <= e
        while (hi - lo > 1) {
            int64_t mid = (lo + hi) >> 1;
            if (indptr[mid] <= e) lo = mid; else hi = mid;
        }
        dst_row[e] = static_cast<int32_t>(lo);
    }
}

// col_ptr[s] = first position in the sorted key array whose source is >= s (bisection), s = 0..num_src
__global__ void __launch_bounds__(kBlock)
k_col_ptr(const uint32_t *__restrict__ sorted_src, const int64_t *__restrict__ sizes, int32_t *__restrict__ col_ptr) {
    const int64_t num_src = sizes[1], nnz = sizes[2];
    const int64_t stride = int64_t(gridDim.x) * kBlock;
    for (int64_t k = int64_t(blockIdx.x) * kBlock + threadIdx.x; k <= num_src; k += stride) {
        int64_t lo = 0, hi = nnz;
        while (lo < hi) {
            int64_t mid = (lo + hi) >> 1;
            if (static_cast<int64_t>(sorted_src[mid]) < k) lo = mid + 1; else hi = mid;
        }
        col_ptr[k] = static_cast<int32_t>(lo);
    }
}

// destination row and weight of every edge in the by-source order
__global__ void __launch_bounds__(kBlock)
k_permute_edges(const int32_t *__restrict__ perm, const int32_t *__restrict__ indptr, const float *__restrict__ edge_w,
                const int64_t *__restrict__ sizes, int32_t *__restrict__ dst_row, float *__restrict__ w_sorted) {
    const int64_t num_dst = sizes[0], nnz = sizes[2];
    const int64_t stride = int64_t(gridDim.x) * kBlock;
    for (int64_t q = int64_t(blockIdx.x) * kBlock + threadIdx.x; q < nnz; q += stride) {
        const int32_t e = perm[q];
        int64_t lo = 0, hi = num_dst;                      // largest i with indptr[i] <= e
        while (hi - lo > 1) {
            int64_t mid = (lo + hi) >> 1;
            if (indptr[mid] <= e) lo = mid; else hi = mid;
        }
        dst_row[q] = static_cast<int32_t>(lo);
        w_sorted[q] = edge_w[e];
    }
}

// Weights of the sampled estimator of P H, P = D^-1/2 (A + I) D^-1/2 (paper Eq. 1-3): one wavefront
// per destination row; edge p = (v_i, v_j) gets deg(v_i)/n_i / sqrt((deg(v_i)+1)(deg(v_j)+1)), the
// row's diagonal term is 1/(deg(v_i)+1).  Computed in double, rounded once to float.
template <typename PtrT, typename IdxT>
__global__ void __launch_bounds__(kBlock)
k_gcn_edge_weights(const PtrT *__restrict__ row_ptr, const IdxT *__restrict__ src_ids, const int32_t *__restrict__ indptr,
                   const int32_t *__restrict__ indices, const int64_t *__restrict__ sizes, float *__restrict__ edge_w,
                   float *__restrict__ self_w) {
    const int lane = lane_id();
    const int64_t n = sizes[0];
    const int64_t wave0 = int64_t(blockIdx.x) * kWavesPerBlock + (threadIdx.x >> 6);
    const int64_t nwaves = int64_t(gridDim.x) * kWavesPerBlock;
    for (int64_t i = wave0; i < n; i += nwaves) {
        const int64_t v = static_cast<int64_t>(src_ids[i]);
        const double deg_i = static_cast<double>(static_cast<int64_t>(row_ptr[v + 1]) - static_cast<int64_t>(row_ptr[v]));
        const int b = indptr[i], e = indptr[i + 1];
        const double scale = deg_i / static_cast<double>(e - b);
        if (lane == 0) self_w[i] = static_cast<float>(1.0 / (deg_i + 1.0));
        for (int p = b + lane; p < e; p += kWave) {
            const int64_t u = static_cast<int64_t>(src_ids[indices[p]]);
            const double deg_j = static_cast<double>(static_cast<int64_t>(row_ptr[u + 1]) - static_cast<int64_t>(row_ptr[u]));
            edge_w[p] = static_cast<float>(scale * (1.0 / sqrt((deg_i + 1.0) * (deg_j + 1.0))));
        }
    }
}

}  // namespace

int run_gcn_edge_weights(mqg_ctx *ctx, const mqg_graph *g, const mqg_block *b, float *edge_w, float *self_w, hipStream_t s) {
    const int grid = static_cast<int>(std::min<int64_t>(std::max<int64_t>(1, ceil_div(b->cap_dst, kWavesPerBlock)), 256 * 32));
#define MQG_GCNW(PT, IT)                                                                                              \
    MQG_LAUNCH(ctx, "k_gcn_edge_weights", s,                                                                          \
               (k_gcn_edge_weights<PT, IT><<<grid, kBlock, 0, s>>>(static_cast<const PT *>(g->row_ptr),                \
                                                                   static_cast<const IT *>(b->src_ids), b->indptr,    \
                                                                   b->indices, b->sizes, edge_w, self_w)))
    if (g->ptr_type == MQG_I64 && g->idx_type == MQG_I64) MQG_GCNW(int64_t, int64_t);
    else if (g->ptr_type == MQG_I64) MQG_GCNW(int64_t, int32_t);
    else if (g->idx_type == MQG_I64) MQG_GCNW(int32_t, int64_t);
    else MQG_GCNW(int32_t, int32_t);
#undef MQG_GCNW
    return MQG_OK;
}

int run_weighted_aggregate(mqg_ctx *ctx, const mqg_block *b, const float *edge_w, const float *self_w, const void *x,
                           int64_t x_stride, void *out, int64_t out_stride, int32_t dim, int32_t dtype, hipStream_t s) {
    WeightedRows rows{b->indptr, b->indices, edge_w, self_w};
    if (dtype == MQG_F16)
        return launch<_Float16>(ctx, "k_weighted_aggregate", rows, &b->sizes[0], b->cap_dst, static_cast<const _Float16 *>(x),
                                x_stride, static_cast<_Float16 *>(out), out_stride, dim, s);
    return launch<float>(ctx, "k_weighted_aggregate", rows, &b->sizes[0], b->cap_dst, static_cast<const float *>(x), x_stride,
                         static_cast<float *>(out), out_stride, dim, s);
}

int run_mean_aggregate(mqg_ctx *ctx, const mqg_block *b, const void *x, int64_t x_stride, void *out,
                       int64_t out_stride, int32_t dim, int32_t dtype, hipStream_t s) {
    ForwardRows rows{b->indptr, b->indices};
    if (dtype == MQG_F16)
        return launch<_Float16>(ctx, "k_mean_aggregate", rows, &b->sizes[0], b->cap_dst, static_cast<const _Float16 *>(x),
                                x_stride, static_cast<_Float16 *>(out), out_stride, dim, s);
    return launch<float>(ctx, "k_mean_aggregate", rows, &b->sizes[0], b->cap_dst, static_cast<const float *>(x), x_stride,
                         static_cast<float *>(out), out_stride, dim, s);
}

// Scratch of the backward: room for blocks of nnz_cap edges and src_cap sources (never less than the
// context's own bounds).  Growing it waits for the stream first: earlier work may still use the old one.
int ensure_backward_scratch(mqg_ctx *ctx, int64_t nnz_cap, int64_t src_cap, hipStream_t s, const char *who) {
    if (nnz_cap <= ctx->bwd_nnz_cap && src_cap <= ctx->bwd_src_cap) return MQG_OK;
    hipError_t e = hipStreamSynchronize(s);
    if (e != hipSuccess) return fail(ctx, MQG_ERR_HIP, std::string(who) + hipGetErrorString(e));
    free_backward_scratch(ctx);
    const int64_t nn = std::max<int64_t>(std::max(nnz_cap, ctx->max_nnz), 1);
    const int64_t ns = std::max<int64_t>(std::max(src_cap, ctx->max_src), 1);
    auto alloc = [&](void **p, int64_t bytes) { return hipMalloc(p, static_cast<size_t>(std::max<int64_t>(bytes, 4))) == hipSuccess; };
    bool ok = alloc(reinterpret_cast<void **>(&ctx->bwd.keys[0]), nn * 4) && alloc(reinterpret_cast<void **>(&ctx->bwd.keys[1]), nn * 4) &&
              alloc(reinterpret_cast<void **>(&ctx->bwd.vals[0]), nn * 4) && alloc(reinterpret_cast<void **>(&ctx->bwd.vals[1]), nn * 4) &&
              alloc(reinterpret_cast<void **>(&ctx->bwd.hist), radix_hist_len_max(nn) * 4) &&
              alloc(reinterpret_cast<void **>(&ctx->bwd.tile_sums), radix_scan_tiles_max(nn) * 4) &&
              alloc(reinterpret_cast<void **>(&ctx->bwd_dst_row), nn * 4) &&
              alloc(reinterpret_cast<void **>(&ctx->bwd_w_sorted), nn * 4) &&
              alloc(reinterpret_cast<void **>(&ctx->bwd_col_ptr), (ns + 2) * 4);
    if (!ok) {
        free_backward_scratch(ctx);
        return fail(ctx, MQG_ERR_HIP, std::string(who) + "scratch allocation failed");
    }
    ctx->bwd_nnz_cap = nn;
    ctx->bwd_src_cap = ns;
    return MQG_OK;
}

// edge_w == nullptr: the mean aggregation's backward; otherwise the weighted one (self_w may be null)
int run_aggregate_backward(mqg_ctx *ctx, const mqg_block *b, const float *edge_w, const float *self_w, const void *grad_out,
                           int64_t go_stride, void *grad_x, int64_t gx_stride, int32_t dim, int32_t dtype, hipStream_t s) {
    const char *who = edge_w ? "mqg_weighted_aggregate_backward: " : "mqg_sage_mean_aggregate_backward: ";
    // scratch for the by-source ordering of the edges (reserved, or allocated at the first backward call)
    const int64_t nnz_cap = b->cap_nnz, src_cap = b->cap_src;
    int rc0 = ensure_backward_scratch(ctx, nnz_cap, src_cap, s, who);
    if (rc0 != MQG_OK) return rc0;

    const int egrid = static_cast<int>(std::min<int64_t>(std::max<int64_t>(1, ceil_div(nnz_cap, kBlock)), 8192));
    // Edges by source, stably.  An edge carries its destination row along, or (weighted) its own
    // position, which the sort's first pass makes itself - at least one pass, for that.
    if (!edge_w) MQG_LAUNCH(ctx, "k_edge_dst_rows", s, (k_edge_dst_rows<<<egrid, kBlock, 0, s>>>(b->indptr, b->sizes, ctx->bwd_dst_row)));
    const int bits = std::max(1, radix_key_bits(static_cast<uint64_t>(std::max<int64_t>(src_cap, 1) - 1)));
    int which = -1;
    int rc = radix_sort_pairs(ctx, reinterpret_cast<const uint32_t *>(b->indices), edge_w ? nullptr : ctx->bwd_dst_row, ctx->bwd, nnz_cap,
                              &b->sizes[2], bits, s, &which);
    if (rc != MQG_OK) return rc;
    const uint32_t *sorted_src = ctx->bwd.keys[which];
    const int32_t *sorted_dst = ctx->bwd.vals[which];
    const int cgrid = static_cast<int>(std::min<int64_t>(std::max<int64_t>(1, ceil_div(src_cap + 1, kBlock)), 8192));
    MQG_LAUNCH(ctx, "k_col_ptr", s, (k_col_ptr<<<cgrid, kBlock, 0, s>>>(sorted_src, b->sizes, ctx->bwd_col_ptr)));

    if (edge_w) {
        // the sort's payload was the edge position: turn it into (destination row, weight)
        int32_t *dst_sorted = ctx->bwd_dst_row;
        MQG_LAUNCH(ctx, "k_permute_edges", s,
                   (k_permute_edges<<<egrid, kBlock, 0, s>>>(sorted_dst, b->indptr, edge_w, b->sizes, dst_sorted, ctx->bwd_w_sorted)));
        WeightedBackwardRows rows{ctx->bwd_col_ptr, dst_sorted, ctx->bwd_w_sorted, self_w, b->sizes};
        if (dtype == MQG_F16)
            return launch<_Float16>(ctx, "k_weighted_aggregate_backward", rows, &b->sizes[1], src_cap,
                                    static_cast<const _Float16 *>(grad_out), go_stride, static_cast<_Float16 *>(grad_x), gx_stride, dim, s);
        return launch<float>(ctx, "k_weighted_aggregate_backward", rows, &b->sizes[1], src_cap, static_cast<const float *>(grad_out),
                             go_stride, static_cast<float *>(grad_x), gx_stride, dim, s);
    }
    BackwardRows rows{ctx->bwd_col_ptr, sorted_dst, b->indptr};
    if (dtype == MQG_F16)
        return launch<_Float16>(ctx, "k_mean_aggregate_backward", rows, &b->sizes[1], src_cap,
                                static_cast<const _Float16 *>(grad_out), go_stride, static_cast<_Float16 *>(grad_x), gx_stride, dim, s);
    return launch<float>(ctx, "k_mean_aggregate_backward", rows, &b->sizes[1], src_cap, static_cast<const float *>(grad_out),
                         go_stride, static_cast<float *>(grad_x), gx_stride, dim, s);
}

}  // namespace mqg
