// Stable least-significant-digit radix sort of (32-bit key, 32-bit payload) pairs, 8 bits per pass,
// and the exclusive scan it needs.  Used to rank nodes by degree for the cache and to order a
// block's edges by source node for the backward aggregation.  The element count may live on the
// device (n_dev): grids are sized by the host-side bound n_cap and every kernel clamps.
//   k_radix_hist     per-workgroup digit histogram, laid out [digit][workgroup]
//   k_scan_reduce / k_scan_apply   exclusive scan of that table (k_scan_tiles between them only
//                    above 2,048 tiles; a single tile needs no reduce)
//   k_radix_scatter  stable scatter: ballot match inside a wavefront, LDS counts across the four
//                    wavefronts and across the rounds of a tile
// Sorts of up to 32 tiles (65,536 keys: the inner blocks of a mini-batch) need no scan launch at
// all: the histogram table is laid out [tile][digit] and every workgroup of the scatter adds up, per
// digit, the counts of all tiles (for the digit's base) and of the tiles before its own - two
// launches per pass instead of four.  (With 138 tiles the adding-up made the scatter 25 us instead of
// 8: more than the two scan launches it saved.)
#include <algorithm>

#include "common.h"
#include "device_utils.h"
#include "radix.h"

namespace mqg {

namespace {

// tile_major: the table is [tile][digit] (for the scatter that adds the counts up itself), otherwise
// [digit][tile] (so that one exclusive scan over the flat table gives every tile its bases)
__global__ void __launch_bounds__(kBlock)
k_radix_hist(const uint32_t *__restrict__ keys, int64_t n, const int64_t *__restrict__ n_dev, int shift,
             int32_t *__restrict__ hist, int nblocks, int items, int tile_major) {
    __shared__ int h[256];
    if (n_dev && *n_dev < n) n = *n_dev;
    h[threadIdx.x] = 0;
    __syncthreads();
    const int64_t base = int64_t(blockIdx.x) * kBlock * items;
    for (int r = 0; r < items; ++r) {
        int64_t i = base + r * kBlock + threadIdx.x;
        if (i < n) atomicAdd(&h[(keys[i] >> shift) & 255], 1);
    }
    __syncthreads();
    if (tile_major) hist[int64_t(blockIdx.x) * 256 + threadIdx.x] = h[threadIdx.x];
    else hist[int64_t(threadIdx.x) * nblocks + blockIdx.x] = h[threadIdx.x];
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

// scanned: tile_vals holds the exclusive scan of the tile sums; otherwise the sums themselves, and
// every workgroup adds up the ones before its own
__global__ void __launch_bounds__(kBlock)
k_scan_apply(int32_t *__restrict__ data, int64_t n, const int32_t *__restrict__ tile_vals, int scanned) {
    __shared__ int lds[kWavesPerBlock];
    const int tile_base = scanned ? tile_vals[blockIdx.x] : tiles_before(tile_vals, lds);
    const int64_t base = int64_t(blockIdx.x) * kScanTile + threadIdx.x * 4;
    int v[4];
    int c = 0;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        v[q] = base + q < n ? data[base + q] : 0;
        c += v[q];
    }
    int total;
    int ex = block_excl_scan<kWavesPerBlock>(c, &total, lds) + tile_base;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        if (base + q < n) data[base + q] = ex;
        ex += v[q];
    }
}

// SELF: `offsets` is the [tile][digit] table of counts and the bases are added up here; otherwise it
// is the scanned [digit][tile] table.
template <bool SELF>
__global__ void __launch_bounds__(kBlock)
k_radix_scatter(const uint32_t *__restrict__ keys_in, const int32_t *__restrict__ vals_in, int64_t n,
                const int64_t *__restrict__ n_dev, int shift,
                const int32_t *__restrict__ offsets, int nblocks, int items, uint32_t *__restrict__ keys_out,
                int32_t *__restrict__ vals_out) {
    __shared__ int run[256];                         // keys of this digit placed in earlier rounds
    __shared__ int wcnt[kWavesPerBlock][256];        // per wavefront, this round
    __shared__ int gbase[256];                       // first output position of this workgroup per digit
    __shared__ int scan_lds[kWavesPerBlock];
    const int tid = threadIdx.x;
    const int lane = lane_id();
    const int wave = tid >> 6;
    if (n_dev && *n_dev < n) n = *n_dev;
    run[tid] = 0;
    if (SELF) {
        // digit tid: keys with a smaller digit in any tile, plus keys with this digit in earlier tiles
        int all = 0, before = 0;
        const int me = static_cast<int>(blockIdx.x);
#pragma unroll 8
        for (int w = 0; w < nblocks; ++w) {
            const int c = offsets[int64_t(w) * 256 + tid];
            all += c;
            before += w < me ? c : 0;
        }
        int total;
        gbase[tid] = block_excl_scan<kWavesPerBlock>(all, &total, scan_lds) + before;
    } else {
        gbase[tid] = offsets[int64_t(tid) * nblocks + blockIdx.x];
    }
#pragma unroll
    for (int w = 0; w < kWavesPerBlock; ++w) wcnt[w][tid] = 0;
    __syncthreads();
    const int64_t base = int64_t(blockIdx.x) * kBlock * items;
    for (int r = 0; r < items; ++r) {
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


}  // namespace

int64_t radix_blocks(int64_t n_cap) { return std::max<int64_t>(1, ceil_div(n_cap, kRadixTile)); }
int64_t radix_hist_len(int64_t n_cap) { return 256 * radix_blocks(n_cap); }
int64_t radix_scan_tiles(int64_t n_cap) { return ceil_div(radix_hist_len(n_cap), kScanTile) + 1; }

// exclusive scan of data[0..n) in place
int device_scan(mqg_ctx *ctx, int32_t *data, int64_t n, int32_t *tile_sums, hipStream_t s) {
    const int tiles = static_cast<int>(std::max<int64_t>(1, ceil_div(n, kScanTile)));
    const int scanned = tiles > kSelfPrefixTiles ? 1 : 0;     // few tiles: k_scan_apply adds the sums up itself
    if (tiles > 1) MQG_LAUNCH(ctx, "k_scan_reduce", s, (k_scan_reduce<<<tiles, kBlock, 0, s>>>(data, n, tile_sums)));
    if (scanned) {
        int rc = launch_scan_tiles(ctx, tile_sums, tiles, nullptr, nullptr, nullptr, s, "k_scan_tiles(radix)");
        if (rc != MQG_OK) return rc;
    }
    MQG_LAUNCH(ctx, "k_scan_apply", s, (k_scan_apply<<<tiles, kBlock, 0, s>>>(data, n, tile_sums, scanned)));
    return MQG_OK;
}

static int radix_items(int64_t) { return kRadixItems; }

int radix_sort_pairs(mqg_ctx *ctx, const uint32_t *keys_in, const int32_t *vals_in, const RadixBufs &b,
                     int64_t n_cap, const int64_t *n_dev, int bits, hipStream_t s, int *result) {
    const int items = radix_items(n_cap);
    const int nblocks = static_cast<int>(std::max<int64_t>(1, ceil_div(n_cap, int64_t(kBlock) * items)));
    const bool self = nblocks <= kRadixSelfBlocks;
    const int64_t hist_len = int64_t(256) * nblocks;         // never more than radix_hist_len(n_cap)
    const uint32_t *kin = keys_in;
    const int32_t *vin = vals_in;
    int out = 0;
    *result = -1;
    for (int shift = 0; shift < bits; shift += 8) {
        MQG_LAUNCH(ctx, "k_radix_hist", s, (k_radix_hist<<<nblocks, kBlock, 0, s>>>(kin, n_cap, n_dev, shift, b.hist, nblocks, items, self ? 1 : 0)));
        if (self) {
            MQG_LAUNCH(ctx, "k_radix_scatter", s,
                       (k_radix_scatter<true><<<nblocks, kBlock, 0, s>>>(kin, vin, n_cap, n_dev, shift, b.hist, nblocks, items, b.keys[out],
                                                                         b.vals[out])));
        } else {
            int rc = device_scan(ctx, b.hist, hist_len, b.tile_sums, s);
            if (rc != MQG_OK) return rc;
            MQG_LAUNCH(ctx, "k_radix_scatter", s,
                       (k_radix_scatter<false><<<nblocks, kBlock, 0, s>>>(kin, vin, n_cap, n_dev, shift, b.hist, nblocks, items, b.keys[out],
                                                                          b.vals[out])));
        }
        kin = b.keys[out];
        vin = b.vals[out];
        *result = out;
        out ^= 1;
    }
    return MQG_OK;
}

}  // namespace mqg
