// Feature gather through the hot-node cache (paper Sec. III "Feature Cache", Sec. IV
// "Mini-Batch Transfer To GPU"): out[i] = F[ids[i]], a row coming from the HBM cache when the
// node is cached and from the full feature matrix (pinned host memory, read over the host link
// by the kernel itself) when it is not.
//
//   k_classify        slot_of lookup, ballot-compacted (output row, source row) lists for hits and
//                     misses, one atomic per wavefront and list
//   k_gather_rows<.,0> hits:   HBM cache -> HBM output, widest aligned loads; rows of up to 64 vectors
//                     as one flat sequence of vectors (every lane carries one), longer rows two at a
//                     time by a wavefront
//   k_gather_rows<.,1> misses: feature matrix -> HBM output (same code, separate symbol so that
//                     profiles tell the HBM-bound from the link-bound launch)
//   k_gather_direct   no cache: every row straight from the feature matrix
#include <hip/hip_ext.h>

#include <algorithm>
#include <mutex>

#include "common.h"
#include "device_utils.h"

namespace mqg {

namespace {

// Stats of a gather without a cache: every valid id is a row served from feats.  counters[3] holds
// the number of ids outside the graph that the copy skipped; it is left at zero for the next call.
__global__ void k_direct_stats(int64_t *stats, const int64_t *num_ids, int64_t cap, unsigned long long *counters) {
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        int64_t n = *num_ids;
        if (n > cap) n = cap;
        if (n < 0) n = 0;
        if (counters) {
            n -= static_cast<int64_t>(counters[3]);
            counters[3] = 0;
        }
        if (stats) {
            stats[0] = 0;
            stats[1] = n;
        }
    }
}

constexpr int kClassifyItems = 4;                       // ids per thread and tile
constexpr int kClassifyTile = kBlock * kClassifyItems;

// Splits the ids into a hit list (output row, cache slot) and a miss list (output row, node id).
// A workgroup classifies a tile of 1024 ids, scans its hit and miss counts together (packed in
// one int) and reserves its share of both lists with one atomic each, so the two counters see
// about a hundred atomics per mini-batch instead of one per wavefront.  The order of the list
// entries is arbitrary; the gather does not depend on it.  An id outside [0, num_nodes) is never
// used as an index: it goes on neither list, so its output row stays untouched and hits + misses
// fall short of the number of ids.
template <typename IdxT>
__global__ void __launch_bounds__(kBlock)
k_classify(const IdxT *__restrict__ ids, const int64_t *__restrict__ num_ids, int64_t cap,
           const int32_t *__restrict__ slot_of, int64_t num_nodes, int2 *__restrict__ hit_list,
           int2 *__restrict__ miss_list, unsigned long long *__restrict__ counters) {
    __shared__ int lds[kWavesPerBlock];
    __shared__ unsigned long long base[2];
    int64_t n = *num_ids;
    if (n > cap) n = cap;
    for (int64_t t0 = int64_t(blockIdx.x) * kClassifyTile; t0 < n; t0 += int64_t(gridDim.x) * kClassifyTile) {
        int32_t id[kClassifyItems], slot[kClassifyItems];
        int h = 0, m = 0;
#pragma unroll
        for (int q = 0; q < kClassifyItems; ++q) {
            int64_t i = t0 + q * kBlock + threadIdx.x;
            id[q] = -1;
            slot[q] = -1;
            if (i < n) {
                const int64_t raw = static_cast<int64_t>(ids[i]);
                if (raw >= 0 && raw < num_nodes) {          // an id outside the graph is on neither list
                    id[q] = static_cast<int32_t>(raw);
                    slot[q] = slot_of[id[q]];
                    if (slot[q] >= 0) ++h; else ++m;
                }
            }
        }
        int total;
        int ex = block_excl_scan<kWavesPerBlock>(h | (m << 16), &total, lds);
        if (threadIdx.x == 0) {
            base[0] = atomicAdd(&counters[0], static_cast<unsigned long long>(total & 0xFFFF));
            base[1] = atomicAdd(&counters[1], static_cast<unsigned long long>(total >> 16));
        }
        __syncthreads();
        unsigned long long ph = base[0] + (ex & 0xFFFF), pm = base[1] + (ex >> 16);
#pragma unroll
        for (int q = 0; q < kClassifyItems; ++q) {
            int i = static_cast<int>(t0 + q * kBlock + threadIdx.x);
            if (slot[q] >= 0) hit_list[ph++] = make_int2(i, slot[q]);
            else if (id[q] >= 0) miss_list[pm++] = make_int2(i, id[q]);
        }
        __syncthreads();                                // base[] is rewritten by the next tile
    }
}

// Which rows to copy: entry r of a (output row, source row) list, or row ids[r] to output row r.
// get() returns false for a row that must not be written (an id outside the feature matrix); the
// source row is then 0, so that a load issued before the check stays inside the matrix.  skipped()
// is called once per such row.
struct ListRows {
    const int2 *list;
    __device__ __forceinline__ bool get(int64_t r, int64_t *src_row, int64_t *dst_row) const {
        int2 e = list[r];
        *src_row = e.y;
        *dst_row = e.x;
        return true;
    }
    __device__ __forceinline__ void skipped() const {}
};
template <typename IdxT>
struct DirectRows {
    const IdxT *ids;
    int64_t num_rows;                    // rows of the source matrix
    unsigned long long *bad;             // counter of skipped rows, may be null
    __device__ __forceinline__ bool get(int64_t r, int64_t *src_row, int64_t *dst_row) const {
        const int64_t id = static_cast<int64_t>(ids[r]);
        const bool ok = id >= 0 && id < num_rows;
        *src_row = ok ? id : 0;
        *dst_row = r;
        return ok;
    }
    __device__ __forceinline__ void skipped() const {
        if (bad) atomicAdd(bad, 1ull);
    }
};

// A 16-byte load that is not kept in the caches on its way (STREAM: read-once data of a launch too
// large for the last-level cache); narrower vectors are loaded normally.
typedef unsigned int uint4_native __attribute__((ext_vector_type(4)));
template <bool STREAM, typename VecT>
__device__ __forceinline__ VecT load_vec(const VecT *p) {
    if constexpr (STREAM && sizeof(VecT) == 16) {
        const uint4_native v = __builtin_nontemporal_load(reinterpret_cast<const uint4_native *>(p));
        VecT out;
        __builtin_memcpy(&out, &v, 16);
        return out;
    } else {
        return *p;
    }
}

constexpr int kRowUnroll = 4;                            // row loads in flight per lane (rows of up to 64 vectors)
// Longer rows: all 64 lanes walk WR rows at a time, NCH 64-vector chunks of each, so that up to
// eight loads per lane are issued before the first store (a row's last, partial chunk rides along
// instead of trailing alone).  NCH is the number of chunks a row needs, at most four; loads are
// unconditional (an index past the row re-reads its last vector), only the stores are predicated.
template <typename VecT, int NCH, int WR, bool STREAM, typename Rows>
__device__ __forceinline__ void copy_rows_wide(const Rows &rows, int64_t n, const char *__restrict__ src,
                                               int64_t src_stride_bytes, char *__restrict__ dst,
                                               int64_t dst_stride_bytes, int vecs) {
    const int lane = lane_id();
    const int64_t wave0 = int64_t(blockIdx.x) * kWavesPerBlock + (threadIdx.x >> 6);
    const int64_t nwaves = int64_t(gridDim.x) * kWavesPerBlock;
    for (int64_t r0 = wave0 * WR; r0 < n; r0 += nwaves * WR) {
        const VecT *sp[WR];
        VecT *dp[WR];
        bool rok[WR];
#pragma unroll
        for (int q = 0; q < WR; ++q) {
            const int64_t r = r0 + q;
            int64_t srow, drow;
            const bool valid = rows.get(r < n ? r : n - 1, &srow, &drow);          // a row past the end re-reads the last one
            if (r < n && !valid && lane == 0) rows.skipped();
            rok[q] = r < n && valid;
            sp[q] = reinterpret_cast<const VecT *>(src + srow * src_stride_bytes);
            dp[q] = reinterpret_cast<VecT *>(dst + drow * dst_stride_bytes);
        }
        for (int c0 = lane; c0 < vecs; c0 += NCH * kWave) {
            VecT v[WR][NCH];
#pragma unroll
            for (int q = 0; q < WR; ++q)
#pragma unroll
                for (int k = 0; k < NCH; ++k) {
                    const int c = c0 + k * kWave;
                    v[q][k] = load_vec<STREAM>(&sp[q][c < vecs ? c : vecs - 1]);
                }
#pragma unroll
            for (int q = 0; q < WR; ++q)
#pragma unroll
                for (int k = 0; k < NCH; ++k) {
                    const int c = c0 + k * kWave;
                    if (rok[q] && c < vecs) dp[q][c] = v[q][k];
                }
        }
    }
}

// chunks per row and rows per wavefront of the long-row copy
inline __host__ __device__ int wide_chunks(int vecs) { return vecs > 3 * kWave ? 4 : (vecs > 2 * kWave ? 3 : 2); }
inline __host__ __device__ int wide_rows(int vecs) { return vecs > 2 * kWave ? 2 : 4; }

// Row copies by one wavefront (the grouped copy).  Rows of up to 64 vectors: the wavefront is split
// into 64/LPR groups of LPR lanes (LPR = 2^log2_lpr >= vecs), every group copies one row per step
// and kRowUnroll steps are in flight, so a wavefront moves 4*64/LPR short rows at a time.  Longer
// rows: copy_rows_wide.
template <typename VecT, bool STREAM, typename Rows>
__device__ __forceinline__ void copy_rows(const Rows &rows, int64_t n, const char *__restrict__ src,
                                          int64_t src_stride_bytes, char *__restrict__ dst,
                                          int64_t dst_stride_bytes, int vecs, int log2_lpr) {
    if (vecs > kWave) {
        switch (wide_chunks(vecs)) {
            case 2: copy_rows_wide<VecT, 2, 4, STREAM>(rows, n, src, src_stride_bytes, dst, dst_stride_bytes, vecs); break;
            case 3: copy_rows_wide<VecT, 3, 2, STREAM>(rows, n, src, src_stride_bytes, dst, dst_stride_bytes, vecs); break;
            default: copy_rows_wide<VecT, 4, 2, STREAM>(rows, n, src, src_stride_bytes, dst, dst_stride_bytes, vecs); break;
        }
        return;
    }
    const int lane = lane_id();
    const int64_t wave0 = int64_t(blockIdx.x) * kWavesPerBlock + (threadIdx.x >> 6);
    const int64_t nwaves = int64_t(gridDim.x) * kWavesPerBlock;
    const int groups = kWave >> log2_lpr;
    const int g = lane >> log2_lpr;
    const int gl = lane & ((1 << log2_lpr) - 1);
    const int64_t per_wave = int64_t(groups) * kRowUnroll;
    for (int64_t base = wave0 * per_wave; base < n; base += nwaves * per_wave) {
        const VecT *sp[kRowUnroll];
        VecT *dp[kRowUnroll];
        bool ok[kRowUnroll];
        VecT v[kRowUnroll];
#pragma unroll
        for (int u = 0; u < kRowUnroll; ++u) {
            const int64_t r = base + u * groups + g;
            int64_t srow = 0, drow = 0;
            bool valid = false;
            if (r < n) {
                valid = rows.get(r, &srow, &drow);
                if (!valid && gl == 0) rows.skipped();
            }
            ok[u] = valid && gl < vecs;
            sp[u] = reinterpret_cast<const VecT *>(src + srow * src_stride_bytes) + gl;
            dp[u] = reinterpret_cast<VecT *>(dst + drow * dst_stride_bytes) + gl;
        }
#pragma unroll
        for (int u = 0; u < kRowUnroll; ++u)
            if (ok[u]) v[u] = *sp[u];
#pragma unroll
        for (int u = 0; u < kRowUnroll; ++u)
            if (ok[u]) *dp[u] = v[u];
    }
}

// The rows of a launch as one flat sequence of vectors: vector t belongs to row t / vecs (a
// multiplication by magic = ceil(2^64 / vecs), exact for t < 2^32).  Every lane carries a vector
// whatever the row length - no idle lanes in a row's last, partial chunk - and kFlatUnroll
// consecutive 256-vector spans are in flight per workgroup.

constexpr int kFlatUnroll = 4;
// Read plus written bytes of one hit-gather launch above which the source rows are loaded with the
// non-temporal hint: the chip's last-level cache holds 256 MB; measured on 512-byte rows, 453 MB per
// launch 77.5 -> 72.0 us and 889 MB 159.7 -> 139.2 us with the hint, while launches of 125-180 MB
// lose 5-15 % with it.
constexpr int64_t kStreamingBytes = int64_t(320) << 20;

template <typename VecT, bool STREAM, typename Rows>
__device__ __forceinline__ void copy_rows_flat(const Rows &rows, int64_t n, const char *__restrict__ src,
                                               int64_t src_stride_bytes, char *__restrict__ dst,
                                               int64_t dst_stride_bytes, int vecs, unsigned long long magic) {
    const int64_t total = n * vecs;
    const int64_t span = int64_t(kBlock) * kFlatUnroll;
    for (int64_t b0 = int64_t(blockIdx.x) * span; b0 < total; b0 += int64_t(gridDim.x) * span) {
        const VecT *sp[kFlatUnroll];
        VecT *dp[kFlatUnroll];
        bool ok[kFlatUnroll];
        VecT v[kFlatUnroll];
#pragma unroll
        for (int u = 0; u < kFlatUnroll; ++u) {
            const int64_t t = b0 + u * kBlock + threadIdx.x;
            ok[u] = t < total;
            const unsigned long long tc = static_cast<unsigned long long>(ok[u] ? t : total - 1);   // past the end: re-read the last vector
            const int64_t row = static_cast<int64_t>(__umul64hi(tc, magic));
            const int64_t col = static_cast<int64_t>(tc) - row * vecs;
            int64_t srow, drow;
            const bool valid = rows.get(row, &srow, &drow);
            if (ok[u] && !valid && col == 0) rows.skipped();
            ok[u] = ok[u] && valid;
            sp[u] = reinterpret_cast<const VecT *>(src + srow * src_stride_bytes) + col;
            dp[u] = reinterpret_cast<VecT *>(dst + drow * dst_stride_bytes) + col;
        }
#pragma unroll
        for (int u = 0; u < kFlatUnroll; ++u) v[u] = load_vec<STREAM>(sp[u]);
#pragma unroll
        for (int u = 0; u < kFlatUnroll; ++u)
            if (ok[u]) *dp[u] = v[u];
    }
}

// MISS names the launch: 0 = rows from the HBM cache, 1 = rows from the feature matrix in pinned
// host memory.  The copy is the same; profiles tell the two apart by symbol.  The miss launch is
// the last kernel of a gather and leaves the (hits, misses) counters at zero for the next one: the
// workgroup that finishes last - every workgroup has read its count by then - clears them, so the
// call is self-contained and can be replayed from a recorded graph.  counters[2] counts the
// finished workgroups.
template <typename VecT, int MISS>
__global__ void __launch_bounds__(kBlock)
k_gather_rows(const int2 *__restrict__ list, const unsigned long long *count,
              const char *__restrict__ src, int64_t src_stride_bytes, char *__restrict__ dst,
              int64_t dst_stride_bytes, int vecs, int log2_lpr, int64_t *__restrict__ stats,
              unsigned long long *counters, unsigned long long magic) {
    if (stats && blockIdx.x == 0 && threadIdx.x < 2) stats[threadIdx.x] = static_cast<int64_t>(counters[threadIdx.x]);
    const int64_t n = static_cast<int64_t>(*count);
    // a launch that moves more than the last-level cache holds reads its source rows past the caches
    const bool streaming = !MISS && sizeof(VecT) == 16 && 2 * n * vecs * int64_t(sizeof(VecT)) > kStreamingBytes;
    const ListRows rows{list};
    if (streaming) {                                       // one uniform branch; the copies themselves are straight code
        if (magic) copy_rows_flat<VecT, true>(rows, n, src, src_stride_bytes, dst, dst_stride_bytes, vecs, magic);
        else copy_rows<VecT, true>(rows, n, src, src_stride_bytes, dst, dst_stride_bytes, vecs, log2_lpr);
    } else {
        if (magic) copy_rows_flat<VecT, false>(rows, n, src, src_stride_bytes, dst, dst_stride_bytes, vecs, magic);
        else copy_rows<VecT, false>(rows, n, src, src_stride_bytes, dst, dst_stride_bytes, vecs, log2_lpr);
    }
    if (MISS) {
        __syncthreads();                                   // every thread of the workgroup has read its count
        if (threadIdx.x == 0) {
            __threadfence();
            const unsigned long long done = atomicAdd(&counters[2], 1ull);
            if (done == gridDim.x - 1) {
                counters[0] = 0;
                counters[1] = 0;
                counters[2] = 0;
            }
        }
    }
}

template <typename VecT, typename IdxT>
__global__ void __launch_bounds__(kBlock)
k_gather_direct(const IdxT *__restrict__ ids, const int64_t *__restrict__ num_ids, int64_t cap, int64_t src_rows,
                unsigned long long *bad, const char *__restrict__ src, int64_t src_stride_bytes, char *__restrict__ dst,
                int64_t dst_stride_bytes, int vecs, int log2_lpr, unsigned long long magic) {
    int64_t n = *num_ids;
    if (n > cap) n = cap;
    const DirectRows<IdxT> rows{ids, src_rows, bad};
    if (magic) copy_rows_flat<VecT, false>(rows, n, src, src_stride_bytes, dst, dst_stride_bytes, vecs, magic);
    else copy_rows<VecT, false>(rows, n, src, src_stride_bytes, dst, dst_stride_bytes, vecs, log2_lpr);
}

// Widest power-of-two access (16, 8, 4 or 2 bytes) that keeps every row of both sides aligned.
int pick_vec_bytes(int64_t row_bytes, int64_t a_stride, int64_t b_stride, const void *a, const void *b) {
    uint64_t bits = static_cast<uint64_t>(row_bytes) | static_cast<uint64_t>(a_stride) | static_cast<uint64_t>(b_stride) |
                    reinterpret_cast<uintptr_t>(a) | reinterpret_cast<uintptr_t>(b);
    for (int v = 16; v > 2; v >>= 1)
        if ((bits & static_cast<uint64_t>(v - 1)) == 0) return v;
    return 2;
}

// Bytes to move per row.  When both sides keep rows 16-byte aligned and have room for it, the row
// is rounded up to whole 16-byte words so that 128-bit accesses can be used; an HBM-to-HBM copy
// (whole_lines) whose rows are 64-byte aligned on both sides is rounded up to whole 64-byte lines,
// so that no line of the destination is written in part (2,408-byte rows: 47.7 -> 46.7 us).  The
// few bytes past the row that are then copied come from the source row's own padding and land in
// the destination row's own padding.  Copies over the host link move no more than they must.
int64_t copy_bytes(int64_t row_bytes, int64_t a_stride, int64_t b_stride, const void *a, const void *b,
                   bool whole_lines) {
    uint64_t bits = static_cast<uint64_t>(a_stride) | static_cast<uint64_t>(b_stride) |
                    reinterpret_cast<uintptr_t>(a) | reinterpret_cast<uintptr_t>(b);
    int64_t r64 = (row_bytes + 63) & ~int64_t(63);
    if (whole_lines && (bits & 63) == 0 && r64 <= a_stride && r64 <= b_stride) return r64;
    int64_t r16 = (row_bytes + 15) & ~int64_t(15);
    if ((bits & 15) == 0 && r16 <= a_stride && r16 <= b_stride) return r16;
    return row_bytes;
}

// Geometry of a row-copy launch.
struct RowGeom {
    int vb;          // bytes per vector
    int vecs;        // vectors per row
    int log2_lpr;    // lanes per row group (rows of at most 64 vectors)
    int64_t rows_per_wave;       // rows a wavefront has in flight
    int64_t bytes_per_wave;      // bytes a wavefront has in flight
};

RowGeom row_geom(int64_t row_bytes, int64_t a_stride, int64_t b_stride, const void *a, const void *b) {
    RowGeom g;
    g.vb = pick_vec_bytes(row_bytes, a_stride, b_stride, a, b);
    g.vecs = static_cast<int>(row_bytes / g.vb);
    g.log2_lpr = 0;
    while ((1 << g.log2_lpr) < g.vecs && g.log2_lpr < 6) ++g.log2_lpr;
    if (g.vecs <= kWave) {
        g.rows_per_wave = int64_t(kWave >> g.log2_lpr) * kRowUnroll;
        g.bytes_per_wave = g.rows_per_wave * row_bytes;
    } else {
        g.rows_per_wave = wide_rows(g.vecs);
        g.bytes_per_wave = g.rows_per_wave * std::min<int64_t>(row_bytes, int64_t(wide_chunks(g.vecs)) * kWave * g.vb);
    }
    return g;
}

// HBM-side copies: enough wavefronts to cover the rows, capped at several per SIMD of 256 CUs.
int hbm_grid(int64_t rows, const RowGeom &g) {
    int64_t waves = ceil_div(rows, g.rows_per_wave);
    // measured on "medium": the copy rate stops rising at about 2,048 workgroups
    return static_cast<int>(std::min<int64_t>(std::max<int64_t>(1, ceil_div(waves, kWavesPerBlock)), 256 * 16));
}

// Which HBM-side copies go flat: rows of 2..64 vectors, where the grouped copy leaves lanes idle
// (25 vectors occupy a 32-lane group) and keeps fewer bytes in flight; measured 3.8 -> 5.1 TB/s for
// 400-byte rows, 4.0 -> 5.4 for 256-byte rows, 4.4 -> 5.7 for 512-byte rows.  Longer rows stay with
// the two-rows-at-a-time copy (2,408-byte rows: 49.3 us grouped, 50.1 us flat inside the whole
// step).  Copies over the host link stay grouped too: with 1 MiB of reads outstanding the grouped
// copy is as fast or faster on its own (256-byte rows 54.6 vs 54.2 GB/s flat, 400-byte rows 43.8 vs
// 42.6) and the flat one slows the pipelined step (0.69 -> 0.84 ms per "xlarge" mini-batch).
// Returns ceil(2^64 / vecs), or 0 for the grouped copy.
unsigned long long flat_magic(int64_t rows, const RowGeom &g) {
    if (g.vecs < 2 || g.vecs > kWave || rows * g.vecs >= (int64_t(1) << 32)) return 0;
    return ~0ull / static_cast<unsigned long long>(g.vecs) + 1;
}
// one workgroup per span of 4 x 256 vectors, up to 32 K workgroups (measured: no difference between
// 8 K and 128 K, and between 2, 4 and 8 spans in flight)
int flat_grid(int64_t rows, const RowGeom &g) {
    const int64_t spans = ceil_div(rows * g.vecs, int64_t(kBlock) * kFlatUnroll);
    return static_cast<int>(std::min<int64_t>(std::max<int64_t>(1, spans), 32 * 1024));
}

// Host-link copies: only as many wavefronts as keep `inflight_bytes` of reads outstanding.  The
// link is saturated by little more than a hundred kilobytes in flight; more only queues up in
// the memory system in front of the HBM traffic of whatever runs beside this kernel.
int link_grid(int64_t rows, const RowGeom &g, int64_t inflight_bytes) {
    int64_t waves = std::max<int64_t>(1, ceil_div(inflight_bytes, g.bytes_per_wave));
    int64_t blocks = ceil_div(waves, kWavesPerBlock);
    return static_cast<int>(std::min<int64_t>(blocks, hbm_grid(rows, g)));
}

template <int MISS>
int launch_rows(mqg_ctx *ctx, const char *name, const int2 *list, const unsigned long long *count, int64_t cap,
                const void *src, int64_t src_stride_bytes, void *dst, int64_t dst_stride_bytes,
                int64_t row_bytes, int64_t *stats, unsigned long long *counters, hipStream_t s) {
    row_bytes = copy_bytes(row_bytes, src_stride_bytes, dst_stride_bytes, src, dst, !MISS);
    const RowGeom g = row_geom(row_bytes, src_stride_bytes, dst_stride_bytes, src, dst);
    int grid = MISS ? link_grid(cap, g, ctx->miss_inflight_bytes) : hbm_grid(cap, g);   // the grouped copy's
    const unsigned long long magic = MISS ? 0 : flat_magic(cap, g);
    if (magic) grid = flat_grid(cap, g);
    const char *sp = static_cast<const char *>(src);
    char *dp = static_cast<char *>(dst);
    if (ctx->profile && g.vb == 16) {
        // the two kernels the rooflines are quoted on: timed by the dispatch's own start and end
        hipEvent_t e0, e1;
        prof_begin_ext(ctx, name, &e0, &e1);
        hipExtLaunchKernelGGL((k_gather_rows<uint4, MISS>), dim3(grid), dim3(kBlock), 0, s, e0, e1, 0, list, count, sp, src_stride_bytes, dp,
                              dst_stride_bytes, g.vecs, g.log2_lpr, stats, counters, magic);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return fail(ctx, MQG_ERR_HIP, std::string(name) + ": " + hipGetErrorString(e));
        return MQG_OK;
    }
    switch (g.vb) {
        case 16: MQG_LAUNCH(ctx, name, s, (k_gather_rows<uint4, MISS><<<grid, kBlock, 0, s>>>(list, count, sp, src_stride_bytes, dp, dst_stride_bytes, g.vecs, g.log2_lpr, stats, counters, magic))); break;
        case 8: MQG_LAUNCH(ctx, name, s, (k_gather_rows<uint2, MISS><<<grid, kBlock, 0, s>>>(list, count, sp, src_stride_bytes, dp, dst_stride_bytes, g.vecs, g.log2_lpr, stats, counters, magic))); break;
        case 4: MQG_LAUNCH(ctx, name, s, (k_gather_rows<uint32_t, MISS><<<grid, kBlock, 0, s>>>(list, count, sp, src_stride_bytes, dp, dst_stride_bytes, g.vecs, g.log2_lpr, stats, counters, magic))); break;
        default: MQG_LAUNCH(ctx, name, s, (k_gather_rows<uint16_t, MISS><<<grid, kBlock, 0, s>>>(list, count, sp, src_stride_bytes, dp, dst_stride_bytes, g.vecs, g.log2_lpr, stats, counters, magic))); break;
    }
    return MQG_OK;
}

// from_host: the source is host memory, so the launch is sized for the link
template <typename IdxT>
int launch_direct(mqg_ctx *ctx, const IdxT *ids, const int64_t *num_ids, int64_t cap, int64_t src_rows,
                  unsigned long long *bad, const void *src, int64_t src_stride_bytes, void *dst,
                  int64_t dst_stride_bytes, int64_t row_bytes, bool from_host, hipStream_t s) {
    row_bytes = copy_bytes(row_bytes, src_stride_bytes, dst_stride_bytes, src, dst, !from_host);
    const RowGeom g = row_geom(row_bytes, src_stride_bytes, dst_stride_bytes, src, dst);
    int grid = from_host ? link_grid(cap, g, ctx->miss_inflight_bytes) : hbm_grid(cap, g);
    const unsigned long long magic = from_host ? 0 : flat_magic(cap, g);
    if (magic) grid = flat_grid(cap, g);
    const char *sp = static_cast<const char *>(src);
    char *dp = static_cast<char *>(dst);
    switch (g.vb) {
        case 16: MQG_LAUNCH(ctx, "k_gather_direct", s, (k_gather_direct<uint4, IdxT><<<grid, kBlock, 0, s>>>(ids, num_ids, cap, src_rows, bad, sp, src_stride_bytes, dp, dst_stride_bytes, g.vecs, g.log2_lpr, magic))); break;
        case 8: MQG_LAUNCH(ctx, "k_gather_direct", s, (k_gather_direct<uint2, IdxT><<<grid, kBlock, 0, s>>>(ids, num_ids, cap, src_rows, bad, sp, src_stride_bytes, dp, dst_stride_bytes, g.vecs, g.log2_lpr, magic))); break;
        case 4: MQG_LAUNCH(ctx, "k_gather_direct", s, (k_gather_direct<uint32_t, IdxT><<<grid, kBlock, 0, s>>>(ids, num_ids, cap, src_rows, bad, sp, src_stride_bytes, dp, dst_stride_bytes, g.vecs, g.log2_lpr, magic))); break;
        default: MQG_LAUNCH(ctx, "k_gather_direct", s, (k_gather_direct<uint16_t, IdxT><<<grid, kBlock, 0, s>>>(ids, num_ids, cap, src_rows, bad, sp, src_stride_bytes, dp, dst_stride_bytes, g.vecs, g.log2_lpr, magic))); break;
    }
    return MQG_OK;
}

// Is p host memory (as opposed to memory of a GPU)?  Unknown pointers count as host.
bool is_host_memory(const void *p) {
    hipPointerAttribute_t attr;
    hipError_t e = hipPointerGetAttributes(&attr, p);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return true;
    }
    return attr.type != hipMemoryTypeDevice;
}

}  // namespace

// Rows listed by 32-bit ids straight from `src` (used by the cache build to fill the cache).
int gather_direct_i32(mqg_ctx *ctx, const int32_t *ids, const int64_t *num_ids, int64_t cap, int64_t src_rows,
                      const void *src, int64_t src_stride_bytes, void *dst, int64_t dst_stride_bytes, int64_t row_bytes,
                      hipStream_t s) {
    return launch_direct<int32_t>(ctx, ids, num_ids, cap, src_rows, nullptr, src, src_stride_bytes, dst, dst_stride_bytes,
                                  row_bytes, is_host_memory(src), s);
}

// Host-side argument checks shared by the gather entry points.  max_ids bounds cap_ids when the
// rows go through the cache (the hit and miss lists hold one entry per id); what_max names it.
int check_gather_args(mqg_ctx *ctx, const mqg_cache *cache, int32_t idx_type, const void *ids_dev,
                      const int64_t *num_ids_dev, int64_t cap_ids, const void *out_dev, int64_t out_stride,
                      int64_t max_ids, const char *what_max) {
    if (!cache || !num_ids_dev) return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_gather_features: NULL cache or num_ids_dev");
    if ((idx_type != MQG_I32 && idx_type != MQG_I64) || (cache->dtype != MQG_F32 && cache->dtype != MQG_F16) || cache->dim < 1)
        return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_gather_features: bad idx_type, dtype or dim");
    if (cap_ids < 0) return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_gather_features: negative cap_ids");
    if (cap_ids > 0 && (!ids_dev || !out_dev)) return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_gather_features: NULL ids or out");
    if (!cache->feats) return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_gather_features: feats is NULL");
    if (out_stride < cache->dim || cache->feat_stride < cache->dim)
        return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_gather_features: stride below dim");
    if (cache->slot_of != nullptr) {
        if (cache->num_cached > 0 && !cache->cache_rows) return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_gather_features: slot_of without cache_rows");
        if (cache->cache_stride < cache->dim) return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_gather_features: cache_stride below dim");
        if (cap_ids > max_ids)
            return fail(ctx, MQG_ERR_CAPACITY, std::string("mqg_gather_features: cap_ids above ") + what_max + " (" +
                        std::to_string(max_ids) + ")");
    } else if (cache->cache_rows) {
        return fail(ctx, MQG_ERR_INVALID_ARG, "mqg_gather_features: cache_rows without slot_of");
    }
    return MQG_OK;
}

// phases: bit 0 = classify the ids and copy the rows found in the cache, bit 1 = copy the others
// from the feature matrix.  Without a cache every row counts as one of the others.
int run_gather(mqg_ctx *ctx, const mqg_cache *c, int32_t idx_type, const void *ids, const int64_t *num_ids,
               int64_t cap_ids, void *out, int64_t out_stride, int64_t *stats, int phases, hipStream_t s) {
    const int64_t elt = c->dtype == MQG_F16 ? 2 : 4;
    const int64_t row_bytes = int64_t(c->dim) * elt;
    if (cap_ids == 0) {
        if (stats && (phases & kGatherMissed)) MQG_LAUNCH(ctx, "k_direct_stats", s, (k_direct_stats<<<1, 64, 0, s>>>(stats, num_ids, 0, nullptr)));
        return MQG_OK;
    }

    if (!c->slot_of) {                                   // no cache: everything from feats
        if (!(phases & kGatherMissed)) return MQG_OK;
        int rc;
        const bool from_host = is_host_memory(c->feats);
        if (idx_type == MQG_I64)
            rc = launch_direct<int64_t>(ctx, static_cast<const int64_t *>(ids), num_ids, cap_ids, c->num_nodes, &ctx->counters[3],
                                        c->feats, c->feat_stride * elt, out, out_stride * elt, row_bytes, from_host, s);
        else
            rc = launch_direct<int32_t>(ctx, static_cast<const int32_t *>(ids), num_ids, cap_ids, c->num_nodes, &ctx->counters[3],
                                        c->feats, c->feat_stride * elt, out, out_stride * elt, row_bytes, from_host, s);
        if (rc != MQG_OK) return rc;
        // every valid id counts as served from feats; the launch also clears the count of skipped ids
        MQG_LAUNCH(ctx, "k_direct_stats", s, (k_direct_stats<<<1, 64, 0, s>>>(stats, num_ids, cap_ids, ctx->counters)));
        return MQG_OK;
    }

    // (hits, misses) counters: zero between gathers (the miss launch clears them when it is done)
    unsigned long long *counters = ctx->counters;
    if (phases & kGatherCached) {
        const int cgrid = static_cast<int>(std::min<int64_t>(std::max<int64_t>(1, ceil_div(cap_ids, kClassifyTile)), 1024));
        if (idx_type == MQG_I64)
            MQG_LAUNCH(ctx, "k_classify", s, (k_classify<int64_t><<<cgrid, kBlock, 0, s>>>(static_cast<const int64_t *>(ids), num_ids, cap_ids, c->slot_of, c->num_nodes, ctx->hit_list, ctx->miss_list, counters)));
        else
            MQG_LAUNCH(ctx, "k_classify", s, (k_classify<int32_t><<<cgrid, kBlock, 0, s>>>(static_cast<const int32_t *>(ids), num_ids, cap_ids, c->slot_of, c->num_nodes, ctx->hit_list, ctx->miss_list, counters)));
        int rc = launch_rows<0>(ctx, "k_gather_hit", ctx->hit_list, &counters[0], cap_ids, c->cache_rows,
                                c->cache_stride * elt, out, out_stride * elt, row_bytes, stats, counters, s);
        if (rc != MQG_OK) return rc;
    }
    if (phases & kGatherMissed)
        return launch_rows<1>(ctx, "k_gather_miss", ctx->miss_list, &counters[1], cap_ids, c->feats,
                              c->feat_stride * elt, out, out_stride * elt, row_bytes, nullptr, counters, s);
    return MQG_OK;
}

}  // namespace mqg

// ---- the gather for callers that cannot allocate ------------------------------------------------
//
// mqg_gather_features keeps its hit and miss lists and its counters in a context, and a context is
// hipMalloc'ed.  The entry point below needs no context: the same lists live in a device array of
// fixed size that is part of the code object, so nothing is allocated when it is called (or ever).
// Layout of the array, in 8-byte words: [0, kMax) hit list, [kMax, 2 kMax) miss list, then the
// eight counter words of run_gather.

namespace mqg {
namespace {

constexpr int64_t kStaticMaxIds = MQG_GATHER_STATIC_MAX_IDS;
constexpr int kStaticMaxDevices = 64;

static __device__ __align__(256) unsigned long long scratch[2 * kStaticMaxIds + 8];

// What the host knows about a device's copy of the array: its address there, and a context object
// (host memory only) that points run_gather at it.  Filled at the first call on the device.
struct StaticGather {
    bool ready = false;
    unsigned long long *ptr = nullptr;
    mqg_ctx ctx;
};
StaticGather g_static[kStaticMaxDevices];
std::mutex g_static_mutex;

__global__ void k_clear_words(unsigned long long *p, int n) {
    if (static_cast<int>(threadIdx.x) < n) p[threadIdx.x] = 0;
}

}  // namespace
}  // namespace mqg

extern "C" int mqg_gather_features_static(const mqg_cache *cache, int32_t idx_type, const void *ids_dev,
                                          const int64_t *num_ids_dev, int64_t cap_ids, void *out_dev,
                                          int64_t out_stride, int64_t *stats_dev, mqg_stream stream) {
    using namespace mqg;
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(nullptr, MQG_ERR_HIP, std::string("mqg_gather_features_static: hipGetDevice: ") + hipGetErrorString(e));
    if (dev < 0 || dev >= kStaticMaxDevices)
        return fail(nullptr, MQG_ERR_UNSUPPORTED, "mqg_gather_features_static: device index above 63");
    StaticGather &sg = g_static[dev];
    {
        std::lock_guard<std::mutex> lock(g_static_mutex);
        if (!sg.ready) {
            // `scratch` is a host-side stand-in here; the device's copy of the array is at the
            // address this call returns, with that device current
            void *p = nullptr;
            e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
            if (e != hipSuccess || !p)
                return fail(nullptr, MQG_ERR_HIP, std::string("mqg_gather_features_static: hipGetSymbolAddress: ") + hipGetErrorString(e));
            sg.ptr = static_cast<unsigned long long *>(p);
            sg.ctx.device = dev;
            sg.ctx.max_src = kStaticMaxIds;
            sg.ctx.hit_list = reinterpret_cast<int2 *>(sg.ptr);
            sg.ctx.miss_list = reinterpret_cast<int2 *>(sg.ptr + kStaticMaxIds);
            sg.ctx.counters = sg.ptr + 2 * kStaticMaxIds;
            sg.ready = true;
        }
    }
    mqg_ctx *ctx = &sg.ctx;
    int rc = check_gather_args(ctx, cache, idx_type, ids_dev, num_ids_dev, cap_ids, out_dev, out_stride, kStaticMaxIds,
                               "MQG_GATHER_STATIC_MAX_IDS");
    if (rc == MQG_OK) {
        hipStream_t s = static_cast<hipStream_t>(stream);
        // the array keeps what the last call left; the counters have to start at zero (a fill
        // kernel rather than a memset, so that the call can also be recorded into a graph)
        if (cap_ids > 0) {
            k_clear_words<<<1, 64, 0, s>>>(ctx->counters, 8);
            e = hipGetLastError();
            if (e != hipSuccess) return fail(nullptr, MQG_ERR_HIP, std::string("mqg_gather_features_static: k_clear_words: ") + hipGetErrorString(e));
        }
        rc = run_gather(ctx, cache, idx_type, ids_dev, num_ids_dev, cap_ids, out_dev, out_stride, stats_dev, kGatherCached | kGatherMissed, s);
    }
    if (rc != MQG_OK) return fail(nullptr, rc, ctx->last_error);      // no context handle: the message goes where mqg_last_error(NULL) reads
    return MQG_OK;
}
