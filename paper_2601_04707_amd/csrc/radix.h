// Radix sort of (key, payload) pairs and the device-wide exclusive scan (internal).
#pragma once

#include "common.h"

namespace mqg {

constexpr int kRadixItems = 8;                       // rounds per tile
constexpr int kRadixTile = kBlock * kRadixItems;     // keys per workgroup
constexpr int kScanTile = 1024;                      // elements per workgroup in the generic scan
constexpr int kRadixSelfBlocks = 32;                 // up to this many tiles the scatter adds the tile counts up itself
constexpr int kRadixMaxDigitBits = 11;

constexpr int kScanSelfTiles = 32;                   // up to this many tiles device_scan_copy scans in one launch

constexpr int64_t kRadixWideKeys = int64_t(2) << 20;  // inputs above this many keys use digits of at most 9 bits
// n_cap keys of `bits` significant bits are sorted in radix_passes passes of radix_digit_bits bits.
int radix_passes(int bits, int64_t n_cap);
int radix_digit_bits(int bits, int64_t n_cap);
int radix_key_bits(uint64_t max_key);                // significant bits of the largest key (at most 32)
int64_t radix_blocks(int64_t n_cap);
int64_t radix_hist_len(int64_t n_cap, int bits);     // table of one sort of exactly this shape
int64_t radix_scan_tiles(int64_t n_cap, int bits);
int64_t radix_hist_len_max(int64_t n_cap);            // enough for every sort of at most n_cap keys, any key width
int64_t radix_scan_tiles_max(int64_t n_cap);

// exclusive scan of data[0..n) in place; tile_sums needs ceil(n / kScanTile) + 1 ints
int device_scan(mqg_ctx *ctx, int32_t *data, int64_t n, int32_t *tile_sums, hipStream_t s);

// exclusive scan of in[0..n) into out[0..n) (out != in), one launch; n <= kScanSelfTiles * kScanTile
int device_scan_copy(mqg_ctx *ctx, const int32_t *in, int32_t *out, int64_t n, hipStream_t s);

// Sorts the first min(n_cap, *n_dev) pairs by the low `bits` bits of the key, stably.  The input
// arrays are only read; *result tells which of b.keys/b.vals holds the output (-1: bits == 0,
// nothing was moved and the input is the output).  b.hist needs radix_hist_len(n_cap, bits) entries,
// b.tile_sums radix_scan_tiles(n_cap, bits).
// vals_in == nullptr: the payload of key i is i itself, made in the first pass (bits > 0 then).
int radix_sort_pairs(mqg_ctx *ctx, const uint32_t *keys_in, const int32_t *vals_in, const RadixBufs &b,
                     int64_t n_cap, const int64_t *n_dev, int bits, hipStream_t s, int *result);

}  // namespace mqg
