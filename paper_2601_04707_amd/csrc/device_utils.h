// Wavefront- and workgroup-level building blocks for gfx950 (64-wide wavefronts).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mqg {

__device__ __forceinline__ int lane_id() { return static_cast<int>(threadIdx.x) & 63; }

__device__ __forceinline__ uint64_t lanes_below(int lane) { return (uint64_t(1) << lane) - 1; }

__device__ __forceinline__ uint64_t ballot64(bool p) { return __ballot(p); }

__device__ __forceinline__ int popc64(uint64_t m) { return __popcll(m); }

// Value of v in lane `l`; l must be the same in every lane.
__device__ __forceinline__ uint32_t readlane32(uint32_t v, int l) {
    return static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(v), l));
}
__device__ __forceinline__ uint64_t readlane64(uint64_t v, int l) {
    uint32_t lo = readlane32(static_cast<uint32_t>(v), l);
    uint32_t hi = readlane32(static_cast<uint32_t>(v >> 32), l);
    return (uint64_t(hi) << 32) | lo;
}

// Orders LDS traffic of one wavefront: writes before, reads after.
__device__ __forceinline__ void wave_lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// The lowest n lanes.
__device__ __forceinline__ uint64_t low_lanes(int n) { return n >= 64 ? ~uint64_t(0) : (uint64_t(1) << n) - 1; }

// Selection of the `need` smallest among the candidates a wavefront holds, NCH per lane: candidate
// c*64+lane has key[c], cand[c] is the set of lanes that hold one.  The order is (late bit, key,
// tie, candidate index), where late[c] marks candidates that come after every unmarked one (PRIO
// only) and tie[c] is a second, 32-bit key (TIE only; for candidates not stored in the order that
// breaks ties between equal keys).
// Binary radix select from the top bit down: one ballot per chunk and bit splits the undecided
// candidates into those with a zero (smaller) and those with a one; either the zeros are still
// too many and the ones drop out, or all zeros are taken and the ones compete for the rest.  It
// stops as soon as the undecided candidates are exactly as many as are still needed, after about
// log2(candidates) bits for random keys.  Masks and counters live in scalar registers.  Every lane
// of the wavefront must call it; need must be at least 1 and at most the number of candidates.
// On return sel[c] holds the chosen lanes of chunk c.
template <int NCH, bool PRIO, bool TIE>
__device__ __forceinline__ void wave_select_smallest(const uint64_t (&key)[NCH], const uint64_t (&late)[NCH],
                                                     const uint32_t (&tie)[NCH], uint64_t (&cand)[NCH], int need,
                                                     uint64_t (&sel)[NCH]) {
#pragma unroll
    for (int c = 0; c < NCH; ++c) sel[c] = 0;
    auto settled = [&]() -> bool {
        int total = 0;
#pragma unroll
        for (int c = 0; c < NCH; ++c) total += popc64(cand[c]);
        if (total != need) return false;
#pragma unroll
        for (int c = 0; c < NCH; ++c) sel[c] |= cand[c];
        return true;
    };
    auto split = [&](const uint64_t (&zeros)[NCH]) {
        int c0 = 0;
#pragma unroll
        for (int c = 0; c < NCH; ++c) c0 += popc64(zeros[c]);
        if (c0 >= need) {
#pragma unroll
            for (int c = 0; c < NCH; ++c) cand[c] = zeros[c];
        } else {
#pragma unroll
            for (int c = 0; c < NCH; ++c) {
                sel[c] |= zeros[c];
                cand[c] &= ~zeros[c];
            }
            need -= c0;
        }
    };
    if (settled()) return;
    uint64_t zeros[NCH];
    if (PRIO) {
#pragma unroll
        for (int c = 0; c < NCH; ++c) zeros[c] = cand[c] & ~late[c];
        split(zeros);
        if (settled()) return;
    }
    for (int part = 0; part < (TIE ? 3 : 2); ++part) {
        uint32_t w[NCH];
#pragma unroll
        for (int c = 0; c < NCH; ++c)
            w[c] = part == 0 ? static_cast<uint32_t>(key[c] >> 32) : part == 1 ? static_cast<uint32_t>(key[c]) : tie[c];
        for (int b = 31; b >= 0; --b) {
            const uint32_t bit = uint32_t(1) << b;
#pragma unroll
            for (int c = 0; c < NCH; ++c) zeros[c] = ballot64((w[c] & bit) == 0) & cand[c];
            split(zeros);
            if (settled()) return;
        }
    }
    // the undecided candidates are equal in every word: lowest candidate index first
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        while (need > 0 && cand[c] != 0) {
            const uint64_t low = cand[c] & (~cand[c] + 1);
            sel[c] |= low;
            cand[c] ^= low;
            --need;
        }
    }
}

// Inclusive prefix sum over the 64 lanes of a wavefront.
__device__ __forceinline__ int wave_incl_scan(int v) {
    const int lane = lane_id();
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        int t = __shfl_up(v, off, 64);
        if (lane >= off) v += t;
    }
    return v;
}

__device__ __forceinline__ int wave_sum(int v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// Exclusive prefix sum over a workgroup of NWAVES*64 threads; *total gets the workgroup sum.
// `lds` needs NWAVES ints.  Every thread of the workgroup must call it.
template <int NWAVES>
__device__ __forceinline__ int block_excl_scan(int v, int *total, int *lds) {
    const int lane = lane_id();
    const int wave = static_cast<int>(threadIdx.x) >> 6;
    int incl = wave_incl_scan(v);
    __syncthreads();                       // lds may still be read from a previous call
    if (lane == 63) lds[wave] = incl;
    __syncthreads();
    int base = 0, sum = 0;
#pragma unroll
    for (int w = 0; w < NWAVES; ++w) {
        int t = lds[w];
        if (w < wave) base += t;
        sum += t;
    }
    *total = sum;
    return base + incl - v;
}

// Sum of tile_sums[0 .. tile): what a tile's own workgroup adds up instead of a separate scan
// launch when the tiles are few (kSelfPrefixTiles at most, i.e. at most 32 loads per thread).
// Every thread of the workgroup (256 threads) must call it; `lds` needs 4 ints.
constexpr int kSelfPrefixTiles = 8192;
constexpr int kSelfPrefixBlock = 256, kSelfPrefixWaves = kSelfPrefixBlock / 64;
__device__ __forceinline__ int tiles_before(const int32_t *__restrict__ tile_sums, int *lds, int tile) {
    int part = 0;
    for (int t = threadIdx.x; t < tile; t += kSelfPrefixBlock) part += tile_sums[t];
    part = wave_sum(part);
    __syncthreads();                                       // lds may still be read from an earlier use
    if (lane_id() == 0) lds[threadIdx.x >> 6] = part;
    __syncthreads();
    int sum = 0;
#pragma unroll
    for (int k = 0; k < kSelfPrefixWaves; ++k) sum += lds[k];
    return sum;
}
__device__ __forceinline__ int tiles_before(const int32_t *__restrict__ tile_sums, int *lds) {
    return tiles_before(tile_sums, lds, static_cast<int>(blockIdx.x));
}

// SplitMix64 finaliser (Steele, Lea, Flood 2014): the mixing function of the sampling keys.
__device__ __forceinline__ uint64_t mix64(uint64_t z) {
    z ^= z >> 30;
    z *= 0xBF58476D1CE4E5B9ULL;
    z ^= z >> 27;
    z *= 0x94D049BB133111EBULL;
    z ^= z >> 31;
    return z;
}

// An exponential variate from 64 random bits in integer arithmetic: -log2(r / 2^64) with 32
// fractional bits (r = 0 counts as 1).  With m = r << lz in [2^63, 2^64) the integer part is
// lz + 1; the fraction of log2(m / 2^63) comes bit by bit from repeated squaring (a square that
// reaches 2 emits a one and is halved), squares truncated to 64 bits.  The step is written without
// a data-dependent branch (the renormalising shift is 0 or 1) so that the loop compiles to straight
// vector code: with a branch the compiler wraps the low product in an exec-mask save/restore, and
// one build of a kernel around that form returned wrong tickets, different from run to run, in
// every workgroup but the first of a compute unit.
__device__ __forceinline__ uint64_t exp_ticket64(uint64_t r) {
    if (r == 0) r = 1;
    const int lz = __clzll(static_cast<long long>(r));
    uint64_t m = r << lz, frac = 0;
#pragma unroll 4
    for (int b = 0; b < 32; ++b) {
        const uint64_t hi = __umul64hi(m, m), lo = m * m;
        const uint64_t one = hi >> 63;
        frac = (frac << 1) | one;
        const uint64_t sh = one ^ 1;                       // not yet at 2: renormalise by one bit
        m = (hi << sh) | ((lo >> 63) & sh);
    }
    return (static_cast<uint64_t>(lz + 1) << 32) - frac;
}

}  // namespace mqg
