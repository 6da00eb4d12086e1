// Radix sort of (key, payload) pairs and the device-wide exclusive scan (internal).
#pragma once

#include "common.h"

namespace mqg {

constexpr int kRadixItems = 8;                       // rounds per tile
constexpr int kRadixTile = kBlock * kRadixItems;     // keys per workgroup
constexpr int kScanTile = 1024;                      // elements per workgroup in the generic scan
constexpr int kRadixSelfBlocks = 32;                 // up to this many tiles the scatter adds the tile counts up itself

int64_t radix_blocks(int64_t n_cap);
int64_t radix_hist_len(int64_t n_cap);
int64_t radix_scan_tiles(int64_t n_cap);

// exclusive scan of data[0..n) in place; tile_sums needs ceil(n / kScanTile) + 1 ints
int device_scan(mqg_ctx *ctx, int32_t *data, int64_t n, int32_t *tile_sums, hipStream_t s);

// Sorts the first min(n_cap, *n_dev) pairs by the low `bits` bits of the key, stably.  The input
// arrays are only read; *result tells which of b.keys/b.vals holds the output (-1: bits == 0,
// nothing was moved and the input is the output).
int radix_sort_pairs(mqg_ctx *ctx, const uint32_t *keys_in, const int32_t *vals_in, const RadixBufs &b,
                     int64_t n_cap, const int64_t *n_dev, int bits, hipStream_t s, int *result);

}  // namespace mqg
