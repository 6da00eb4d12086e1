// Stable least-significant-digit radix sort of (32-bit key, 32-bit payload) pairs and the exclusive
// scan it needs.  Used to rank nodes by degree for the cache, to transpose an adjacency and to order a
// block's edges by source node for the backward aggregation.  The element count may live on the
// device (n_dev): grids are sized by the host-side bound n_cap and every kernel clamps.  Keys of b
// significant bits take ceil(b / 11) passes (ceil(b / 9) for more than 2 M keys) with digits of
// ceil(b / passes) bits (8 at least): the 18-bit source positions of a 230 k-node block sort in two
// 9-bit passes.
//   k_radix_hist     per-workgroup digit histogram, laid out [digit][workgroup]
//   k_scan_reduce / k_scan_apply   exclusive scan of that table (k_scan_tiles between them only
//                    above 8,192 tiles; a single tile needs no reduce)
//   k_radix_scatter  stable scatter: ballot match inside a wavefront, LDS counts across the four
//                    wavefronts and across the rounds of a tile
// Sorts of up to 32 tiles (65,536 keys: the inner blocks of a mini-batch) need no scan launch:
// the histogram table is laid out [tile][digit] and every workgroup of the scatter adds up, per
// digit, the counts of all tiles (for the digit's base) and of the tiles before its own.  (With 138
// tiles the adding-up made the scatter 25 us instead of 8: more than the two scan launches it
// saved.)  Small inputs are cut into tiles of fewer rounds, so that about 32 workgroups share them.
#include <algorithm>

#include "common.h"
#include "device_utils.h"
#include "radix.h"

namespace mqg {

namespace {

// tile_major: the table is [tile][digit] (for the scatter that adds the counts up itself), otherwise
// [digit][tile] (so that one exclusive scan over the flat table gives every tile its bases).
// DB = bits per digit.
template <int DB>
__global__ void __launch_bounds__(kBlock)
k_radix_hist(const uint32_t *__restrict__ keys, int64_t n, const int64_t *__restrict__ n_dev, int shift,
             int32_t *__restrict__ hist, int nblocks, int items, int tile_major) {
    constexpr int D = 1 << DB, PER = D / kBlock;
    __shared__ int h[D];
    if (n_dev && *n_dev < n) n = *n_dev;
#pragma unroll
    for (int q = 0; q < PER; ++q) h[q * kBlock + threadIdx.x] = 0;
    __syncthreads();
    const int64_t base = int64_t(blockIdx.x) * kBlock * items;
    for (int r = 0; r < items; ++r) {
        int64_t i = base + r * kBlock + threadIdx.x;
        if (i < n) atomicAdd(&h[(keys[i] >> shift) & (D - 1)], 1);
    }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < PER; ++q) {
        const int d = q * kBlock + threadIdx.x;
        if (tile_major) hist[int64_t(blockIdx.x) * D + d] = h[d];
        else hist[int64_t(d) * nblocks + blockIdx.x] = h[d];
    }
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

// Exclusive scan of up to kScanSelfTiles tiles in one launch, out of place: every workgroup adds up
// the elements of the tiles before its own (at most 31 x 4 KB, from L2) and scans its tile.
__global__ void __launch_bounds__(kBlock)
k_scan_self(const int32_t *__restrict__ in, int64_t n, int32_t *__restrict__ out) {
    __shared__ int lds[kWavesPerBlock];
    const int64_t tile0 = int64_t(blockIdx.x) * kScanTile;
    int part = 0;
    for (int64_t i = int64_t(threadIdx.x) * 4; i < tile0; i += kBlock * 4) {    // tile0 is a multiple of kBlock * 4
        const int4 x = *reinterpret_cast<const int4 *>(in + i);
        part += x.x + x.y + x.z + x.w;
    }
    part = wave_sum(part);
    if (lane_id() == 0) lds[threadIdx.x >> 6] = part;
    __syncthreads();
    int tile_base = 0;
#pragma unroll
    for (int k = 0; k < kWavesPerBlock; ++k) tile_base += lds[k];
    const int64_t base = tile0 + threadIdx.x * 4;
    int v[4];
    int c = 0;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        v[q] = base + q < n ? in[base + q] : 0;
        c += v[q];
    }
    int total;
    int ex = block_excl_scan<kWavesPerBlock>(c, &total, lds) + tile_base;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        if (base + q < n) out[base + q] = ex;
        ex += v[q];
    }
}

// What a key carries along: vals_in[i], or (vals_in == nullptr, first pass only) its own position i.
struct RadixPayload {
    const int32_t *vals_in;
    __device__ __forceinline__ int32_t get(int64_t i) const { return vals_in ? vals_in[i] : static_cast<int32_t>(i); }
};

// SELF: `offsets` is the [tile][digit] table of counts and the bases are added up here; otherwise it
// is the scanned [digit][tile] table.
template <bool SELF, int DB>
__global__ void __launch_bounds__(kBlock)
k_radix_scatter(const uint32_t *__restrict__ keys_in, RadixPayload payload, int64_t n,
                const int64_t *__restrict__ n_dev, int shift,
                const int32_t *__restrict__ offsets, int nblocks, int items, uint32_t *__restrict__ keys_out,
                int32_t *__restrict__ vals_out) {
    constexpr int D = 1 << DB, PER = D / kBlock;
    __shared__ int run[D];                           // keys of this digit placed in earlier rounds
    __shared__ int wcnt[kWavesPerBlock][D];          // per wavefront, this round
    __shared__ int gbase[D];                         // first output position of this workgroup per digit
    __shared__ int scan_lds[kWavesPerBlock];
    const int tid = threadIdx.x;
    const int lane = lane_id();
    const int wave = tid >> 6;
    if (n_dev && *n_dev < n) n = *n_dev;
    const int me = static_cast<int>(blockIdx.x);
    const int64_t base = int64_t(blockIdx.x) * kBlock * items;
    if (!SELF) {
#pragma unroll
        for (int q = 0; q < PER; ++q) {
            const int d = q * kBlock + tid;
            gbase[d] = offsets[int64_t(d) * nblocks + me];
            run[d] = 0;
        }
    } else {
        // thread t owns the digits t * PER .. t * PER + PER - 1: keys with a smaller digit in any tile,
        // plus keys with the same digit in earlier tiles
        int all[PER], before[PER];
#pragma unroll
        for (int q = 0; q < PER; ++q) all[q] = before[q] = 0;
#pragma unroll 4
        for (int w = 0; w < nblocks; ++w) {
#pragma unroll
            for (int q = 0; q < PER; ++q) {
                const int c = offsets[int64_t(w) * D + tid * PER + q];
                all[q] += c;
                before[q] += w < me ? c : 0;
            }
        }
        int mine = 0;
#pragma unroll
        for (int q = 0; q < PER; ++q) mine += all[q];
        int total;
        int ex = block_excl_scan<kWavesPerBlock>(mine, &total, scan_lds);
#pragma unroll
        for (int q = 0; q < PER; ++q) {
            gbase[tid * PER + q] = ex + before[q];
            run[tid * PER + q] = 0;
            ex += all[q];
        }
    }
#pragma unroll
    for (int w = 0; w < kWavesPerBlock; ++w)
#pragma unroll
        for (int q = 0; q < PER; ++q) wcnt[w][q * kBlock + tid] = 0;
    __syncthreads();
    for (int r = 0; r < items; ++r) {
        const int64_t i = base + r * kBlock + tid;
        const bool valid = i < n;
        uint32_t key = 0;
        int32_t val = 0;
        if (valid) {
            key = keys_in[i];
            val = payload.get(i);
        }
        const int digit = (key >> shift) & (D - 1);
        // lanes of this wavefront holding the same digit
        uint64_t peers = ballot64(valid);
#pragma unroll
        for (int bit = 0; bit < DB; ++bit) {
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
#pragma unroll
        for (int q = 0; q < PER; ++q) {
            const int d = q * kBlock + tid;
            int add = 0;
#pragma unroll
            for (int w = 0; w < kWavesPerBlock; ++w) {
                add += wcnt[w][d];
                wcnt[w][d] = 0;
            }
            run[d] += add;
        }
        __syncthreads();
    }
}

}  // namespace

// Digits: as few passes as the widest digit allows, then the digit just wide enough for them (8 bits
// at least).  The widest digit is 11 bits for inputs of up to kRadixWideKeys keys, where a pass is
// mostly its launches, and 9 bits above, where it is mostly its per-key work (the LDS counters to
// clear and add up per round grow with the digit: the 4.5 M edges of a "stress" block sorted faster
// in three 8-bit passes than in two of 11 bits).
static int max_digit_bits(int64_t n_cap) { return n_cap <= kRadixWideKeys ? kRadixMaxDigitBits : 9; }
int radix_passes(int bits, int64_t n_cap) { return bits <= 0 ? 0 : (bits + max_digit_bits(n_cap) - 1) / max_digit_bits(n_cap); }
int radix_digit_bits(int bits, int64_t n_cap) {
    const int p = radix_passes(bits, n_cap);
    return p == 0 ? 8 : std::max(8, (bits + p - 1) / p);
}
int radix_key_bits(uint64_t max_key) {
    int bits = 0;
    while (bits < 32 && (max_key >> bits) != 0) ++bits;
    return bits;
}
int64_t radix_blocks(int64_t n_cap) { return std::max<int64_t>(1, ceil_div(n_cap, kRadixTile)); }
// (small inputs have up to kRadixSelfBlocks tiles whatever their size)
int64_t radix_hist_len(int64_t n_cap, int bits) {
    return (int64_t(1) << radix_digit_bits(bits, n_cap)) * std::max<int64_t>(radix_blocks(n_cap), kRadixSelfBlocks);
}
int64_t radix_scan_tiles(int64_t n_cap, int bits) { return ceil_div(radix_hist_len(n_cap, bits), kScanTile) + 1; }
// The largest table any sort of at most n_cap keys of at most 32 bits needs: the widest digit on the
// largest input that still takes it, or the 9-bit digit on all of n_cap.
int64_t radix_hist_len_max(int64_t n_cap) {
    const int64_t wide = (int64_t(1) << kRadixMaxDigitBits) * std::max<int64_t>(radix_blocks(std::min(n_cap, kRadixWideKeys)), kRadixSelfBlocks);
    const int64_t narrow = (int64_t(1) << 9) * radix_blocks(n_cap);
    return std::max(wide, narrow);
}
int64_t radix_scan_tiles_max(int64_t n_cap) { return ceil_div(radix_hist_len_max(n_cap), kScanTile) + 1; }

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

int device_scan_copy(mqg_ctx *ctx, const int32_t *in, int32_t *out, int64_t n, hipStream_t s) {
    const int tiles = static_cast<int>(std::max<int64_t>(1, ceil_div(n, kScanTile)));
    if (tiles > kScanSelfTiles || in == out) return fail(ctx, MQG_ERR_INVALID_ARG, "device_scan_copy: too many tiles, or in place");
    MQG_LAUNCH(ctx, "k_scan_self", s, (k_scan_self<<<tiles, kBlock, 0, s>>>(in, n, out)));
    return MQG_OK;
}

// rounds per tile: 8, fewer for small inputs (a round is a serial step of a workgroup; 32 tiles of
// one round sort 8 k keys faster than 4 tiles of eight)
static int radix_items(int64_t n_cap) {
    return static_cast<int>(std::min<int64_t>(kRadixItems, std::max<int64_t>(1, ceil_div(n_cap, int64_t(kBlock) * kRadixSelfBlocks))));
}

template <int DB>
static int radix_sort_pairs_t(mqg_ctx *ctx, const uint32_t *keys_in, RadixPayload first, const RadixBufs &b, int64_t n_cap,
                              const int64_t *n_dev, int bits, hipStream_t s, int *result) {
    constexpr int D = 1 << DB;
    const int items = radix_items(n_cap);
    const int nblocks = static_cast<int>(std::max<int64_t>(1, ceil_div(n_cap, int64_t(kBlock) * items)));
    const bool self = nblocks <= kRadixSelfBlocks;
    const int64_t hist_len = int64_t(D) * nblocks;           // never more than radix_hist_len(n_cap, bits)
    const uint32_t *kin = keys_in;
    RadixPayload pay = first;
    int out = 0;
    *result = -1;
    const int passes = radix_passes(bits, n_cap);
    for (int p = 0; p < passes; ++p) {
        const int shift = p * DB;
        MQG_LAUNCH(ctx, "k_radix_hist", s, (k_radix_hist<DB><<<nblocks, kBlock, 0, s>>>(kin, n_cap, n_dev, shift, b.hist, nblocks, items, self ? 1 : 0)));
        if (self) {
            MQG_LAUNCH(ctx, "k_radix_scatter", s,
                       (k_radix_scatter<true, DB><<<nblocks, kBlock, 0, s>>>(kin, pay, n_cap, n_dev, shift, b.hist, nblocks, items, b.keys[out], b.vals[out])));
        } else {
            int rc = device_scan(ctx, b.hist, hist_len, b.tile_sums, s);
            if (rc != MQG_OK) return rc;
            MQG_LAUNCH(ctx, "k_radix_scatter", s,
                       (k_radix_scatter<false, DB><<<nblocks, kBlock, 0, s>>>(kin, pay, n_cap, n_dev, shift, b.hist, nblocks, items, b.keys[out], b.vals[out])));
        }
        kin = b.keys[out];
        pay = RadixPayload{b.vals[out]};
        *result = out;
        out ^= 1;
    }
    return MQG_OK;
}

int radix_sort_pairs(mqg_ctx *ctx, const uint32_t *keys_in, const int32_t *vals_in, const RadixBufs &b,
                     int64_t n_cap, const int64_t *n_dev, int bits, hipStream_t s, int *result) {
    const RadixPayload first{vals_in};
    switch (radix_digit_bits(bits, n_cap)) {
        case 8: return radix_sort_pairs_t<8>(ctx, keys_in, first, b, n_cap, n_dev, bits, s, result);
        case 9: return radix_sort_pairs_t<9>(ctx, keys_in, first, b, n_cap, n_dev, bits, s, result);
        case 10: return radix_sort_pairs_t<10>(ctx, keys_in, first, b, n_cap, n_dev, bits, s, result);
        default: return radix_sort_pairs_t<11>(ctx, keys_in, first, b, n_cap, n_dev, bits, s, result);
    }
}

}  // namespace mqg
