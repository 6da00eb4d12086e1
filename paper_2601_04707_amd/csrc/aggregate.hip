// GraphSAGE mean aggregation over one block (paper Eq. 16: Z_agg(v) = Mean(H(v)); the GA step,
// "AH", of Sec. IV "Computation").  A segmented reduction over the block's CSR rows: HBM-bound,
// no dense contraction, hence no matrix cores.
//
// One wavefront per destination row.
//   k_mean_aggregate       rows of at most 64*VEC columns: the 64 lanes are split into G groups of
//                          LPR lanes; the lanes of a group cover the feature columns with VEC-wide
//                          loads and group g takes the row's edges g, g+G, ...; the G partial sums
//                          are then folded across groups.  (Also the generic fallback: one group,
//                          one column pass after the other.)
//   k_mean_aggregate_wide  wider rows: a lane owns PASSES column chunks and keeps all of them in
//                          registers, so every source row is fetched with PASSES independent loads
//                          in flight; the row's (at most 64) indices are loaded once, one per lane,
//                          and broadcast with v_readlane.
// Sums are fp32, the mean is one fp32 division, fp16 output is rounded once (to nearest even) at
// the store.
#include <hip/hip_fp16.h>

#include <algorithm>

#include "common.h"
#include "device_utils.h"

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

template <typename T, int VEC>
__global__ void __launch_bounds__(kBlock)
k_mean_aggregate(const int32_t *__restrict__ indptr, const int32_t *__restrict__ indices,
                 const int64_t *__restrict__ sizes, const T *__restrict__ x, int64_t x_stride,
                 T *__restrict__ out, int64_t out_stride, int dim, int log2_lpr) {
    using P = Pack<T, VEC>;
    const int lane = lane_id();
    const int lpr = 1 << log2_lpr;
    const int groups = kWave >> log2_lpr;
    const int g = lane >> log2_lpr;
    const int gl = lane & (lpr - 1);
    const int64_t n_dst = sizes[0];
    const int64_t wave0 = int64_t(blockIdx.x) * kWavesPerBlock + (threadIdx.x >> 6);
    const int64_t nwaves = int64_t(gridDim.x) * kWavesPerBlock;
    for (int64_t i = wave0; i < n_dst; i += nwaves) {
        const int b = indptr[i], e = indptr[i + 1];
        const float cnt = static_cast<float>(e - b);
        // every lane of the wavefront runs the same number of column passes (shuffles below)
        const int passes = (dim + lpr * VEC - 1) / (lpr * VEC);
        for (int ps = 0; ps < passes; ++ps) {
            const int col0 = (ps * lpr + gl) * VEC;
            const bool live = col0 < dim;
            float acc[VEC];
#pragma unroll
            for (int q = 0; q < VEC; ++q) acc[q] = 0.f;
#pragma unroll 4
            for (int p = b + g; p < e; p += groups) {
                const int64_t r = indices[p];
                if (live) {
                    P v = *reinterpret_cast<const P *>(x + r * x_stride + col0);
#pragma unroll
                    for (int q = 0; q < VEC; ++q) acc[q] += to_f32(v.v[q]);
                }
            }
            for (int off = lpr; off < kWave; off <<= 1) {
#pragma unroll
                for (int q = 0; q < VEC; ++q) acc[q] += __shfl_xor(acc[q], off, 64);
            }
            if (live && g == 0) {
                P o;
#pragma unroll
                for (int q = 0; q < VEC; ++q) from_f32(e > b ? acc[q] / cnt : 0.f, &o.v[q]);
                *reinterpret_cast<P *>(out + i * out_stride + col0) = o;
            }
        }
    }
}

template <typename T, int VEC, int PASSES>
__global__ void __launch_bounds__(kBlock)
k_mean_aggregate_wide(const int32_t *__restrict__ indptr, const int32_t *__restrict__ indices,
                      const int64_t *__restrict__ sizes, const T *__restrict__ x, int64_t x_stride,
                      T *__restrict__ out, int64_t out_stride, int dim) {
    using P = Pack<T, VEC>;
    const int lane = lane_id();
    const int64_t n_dst = sizes[0];
    const int64_t wave0 = int64_t(blockIdx.x) * kWavesPerBlock + (threadIdx.x >> 6);
    const int64_t nwaves = int64_t(gridDim.x) * kWavesPerBlock;
    bool live[PASSES];
#pragma unroll
    for (int ps = 0; ps < PASSES; ++ps) live[ps] = (ps * kWave + lane) * VEC < dim;
    for (int64_t i = wave0; i < n_dst; i += nwaves) {
        const int b = indptr[i], e = indptr[i + 1];
        float acc[PASSES][VEC];
#pragma unroll
        for (int ps = 0; ps < PASSES; ++ps)
#pragma unroll
            for (int q = 0; q < VEC; ++q) acc[ps][q] = 0.f;
        for (int c0 = b; c0 < e; c0 += kWave) {            // one chunk: a row has at most 64 edges
            const int m = e - c0 < kWave ? e - c0 : kWave;
            const int my_idx = lane < m ? indices[c0 + lane] : 0;
            auto load_row = [&](int t, P *v) {
                const int64_t r = static_cast<int>(readlane32(static_cast<uint32_t>(my_idx), t));
                const T *row = x + r * x_stride + lane * VEC;
#pragma unroll
                for (int ps = 0; ps < PASSES; ++ps)
                    if (live[ps]) v[ps] = *reinterpret_cast<const P *>(row + ps * kWave * VEC);
            };
            auto add_row = [&](const P *v) {
#pragma unroll
                for (int ps = 0; ps < PASSES; ++ps)
                    if (live[ps]) {
#pragma unroll
                        for (int q = 0; q < VEC; ++q) acc[ps][q] += to_f32(v[ps].v[q]);
                    }
            };
            int t = 0;
            for (; t + 1 < m; t += 2) {                    // two source rows (2*PASSES loads) in flight
                P v0[PASSES], v1[PASSES];
                load_row(t, v0);
                load_row(t + 1, v1);
                add_row(v0);
                add_row(v1);
            }
            if (t < m) {
                P v0[PASSES];
                load_row(t, v0);
                add_row(v0);
            }
        }
        const float cnt = static_cast<float>(e - b);
        T *orow = out + i * out_stride + lane * VEC;
#pragma unroll
        for (int ps = 0; ps < PASSES; ++ps)
            if (live[ps]) {
                P o;
#pragma unroll
                for (int q = 0; q < VEC; ++q) from_f32(e > b ? acc[ps][q] / cnt : 0.f, &o.v[q]);
                *reinterpret_cast<P *>(orow + ps * kWave * VEC) = o;
            }
    }
}

template <typename T>
int launch(mqg_ctx *ctx, const mqg_block *b, const T *x, int64_t x_stride, T *out, int64_t out_stride, int dim,
           hipStream_t s) {
    // widest vector (<= 16 bytes) that divides dim and both strides and keeps the bases aligned.
    // When both strides leave room, dim is first rounded up to whole 16-byte words: the extra
    // columns are read from the source rows' padding and written to the output rows' padding.
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
    const int grid = static_cast<int>(std::min<int64_t>(std::max<int64_t>(1, ceil_div(b->cap_dst, kWavesPerBlock)), 256 * 32));
    const int passes = static_cast<int>(ceil_div(lanes, kWave));
#define MQG_AGG(V)                                                                                            \
    MQG_LAUNCH(ctx, "k_mean_aggregate", s,                                                                    \
               (k_mean_aggregate<T, V><<<grid, kBlock, 0, s>>>(b->indptr, b->indices, b->sizes, x, x_stride, out, \
                                                               out_stride, dim, log2_lpr)))
#define MQG_AGG_WIDE(V, PS)                                                                                   \
    MQG_LAUNCH(ctx, "k_mean_aggregate", s,                                                                    \
               (k_mean_aggregate_wide<T, V, PS><<<grid, kBlock, 0, s>>>(b->indptr, b->indices, b->sizes, x,    \
                                                                        x_stride, out, out_stride, dim)))
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

}  // namespace

int run_mean_aggregate(mqg_ctx *ctx, const mqg_block *b, const void *x, int64_t x_stride, void *out,
                       int64_t out_stride, int32_t dim, int32_t dtype, hipStream_t s) {
    if (dtype == MQG_F16)
        return launch<_Float16>(ctx, b, static_cast<const _Float16 *>(x), x_stride, static_cast<_Float16 *>(out),
                                out_stride, dim, s);
    return launch<float>(ctx, b, static_cast<const float *>(x), x_stride, static_cast<float *>(out), out_stride, dim, s);
}

}  // namespace mqg
