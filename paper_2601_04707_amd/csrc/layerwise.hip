// Layer-wise sampling after LADIES (paper Sec. III-B, Eq. 6-9): the nodes of the next layer are
// drawn from the neighbours of the current layer's nodes (and these nodes themselves: A + I) with
// probability proportional to the squared column norm of the row-selected normalised adjacency
// P = D^-1/2 (A + I) D^-1/2, and a drawn node's column is scaled by 1 / (s p) (Eq. 8).
//
// Per block, for the rows D (the seeds, then the previous block's drawn nodes):
//   k_lw_mass        mass[i] += floor(2^40 / (deg_v + 1)) for every row v and every i in N(v) or
//                    i == v: integer atomics, so the sums do not depend on the schedule.
//                    q_i = mass[i] / (deg_i + 1) is 2^40 times the squared column norm of Eq. 7.
//                    Touched nodes are marked in the context's node bitmap - slot by slot on graphs
//                    above kMassScanNodes nodes, otherwise by k_lw_mass_bits from the masses.
//   bitmap -> list   the candidates (Eq. 6), ascending: set bits counted per tile (by k_lw_mass_bits
//                    itself, else k_lw_tile_counts), then k_lw_emit, whose workgroups add up the
//                    counts of the tiles before their own
//   k_lw_keys        exponential race: key = ticket * (deg_i + 1) / mass[i] in doubles (the "flat"
//                    variants, Eq. 10, draw in proportion to sqrt(q_i): ticket^2 in place of ticket), ticket from
//                    exp_ticket64; partial sums of q per workgroup, added up in a fixed order
//   k_lw_select      radix select of the s-th smallest 64-bit key pattern, most significant digit
//                    first: the leading 12 bits are counted by k_lw_keys itself, the next 13 by
//                    this launch, whose workgroups derive the digit found so far from the
//                    histogram before
//   k_lw_mark        derives the threshold's 25 leading bits; keys below them are marked in the
//                    bitmap, keys that share them (a few dozen) are listed (all candidates are
//                    marked if there are at most s)
//   k_lw_finish      one workgroup ranks the listed keys by (key, id) and marks as many as are
//                    still wanted (a long list - many equal keys - by a radix select of its own)
//   bitmap -> list   the drawn nodes ascending = the block's sources, positions into local_of[]
//   k_lw_count/fill  row v lists the drawn nodes among v and its adjacency row (self edge first,
//                    then slot order) with weight P_vi / (s p_i), optionally divided by the row sum;
//                    k_lw_fill also writes indptr and the block's sizes
// A row is shared by kRowChunks wavefronts, each with a contiguous range of adjacency slots, so
// that a hub does not become a kernel's tail; counts and partial weight sums are kept per (row,
// chunk) and one scan over all of them gives every wavefront its first edge position.
//   k_lw_drawn_keys / k_lw_draw_order / k_lw_debias   (the "+debias" variants, Eq. 12) the drawn nodes in
//                    the order of the race and their debiased coefficients, three scans in one workgroup
//   k_lw_reset       masses and positions back to their idle values
#include <algorithm>
#include <type_traits>

#include "common.h"
#include "device_utils.h"
#include "radix.h"

namespace mqg {

namespace {

constexpr uint64_t kGolden = 0x9E3779B97F4A7C15ULL;
constexpr int kLayerwiseTag = 64;
constexpr int64_t kMassScanNodes = int64_t(8) << 20;   // up to here the candidates are read off the masses
constexpr int64_t kDenseNodes = int64_t(1) << 20;      // up to here every node has a key slot: no candidate list

uint64_t host_mix64(uint64_t z) {
    z ^= z >> 30;
    z *= 0xBF58476D1CE4E5B9ULL;
    z ^= z >> 27;
    z *= 0x94D049BB133111EBULL;
    z ^= z >> 31;
    return z;
}

__device__ __forceinline__ void set_bit(uint32_t *bitmap, uint32_t i) {
    uint32_t *w = bitmap + (i >> 5);
    const uint32_t bit = 1u << (i & 31);
    if (!(__hip_atomic_load(w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) & bit))
        (void)__hip_atomic_fetch_or(w, bit, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// the caller's seeds, checked: an id outside the graph is replaced by node 0 and flagged; also clears
// the histograms of the radix select
template <typename IdxT>
__global__ void __launch_bounds__(kBlock)
k_lw_seeds(const IdxT *__restrict__ seeds, int64_t n, int64_t num_nodes, IdxT *__restrict__ dst, int64_t *sizes,
           int32_t *__restrict__ flags, int32_t *__restrict__ sel_hist, int hist_len) {
    const int64_t t = int64_t(blockIdx.x) * kBlock + threadIdx.x;
    for (int64_t k = t; k < hist_len; k += int64_t(gridDim.x) * kBlock) sel_hist[k] = 0;    // for the first block's select
    if (t == 0) sizes[0] = n;
    if (t >= n) return;
    IdxT v = seeds[t];
    if (v < 0 || static_cast<int64_t>(v) >= num_nodes) {
        v = 0;
        atomicOr(flags, 1);
    }
    dst[t] = v;
}

constexpr int kRowChunks = 16;      // wavefronts that share one row

// the contiguous range of adjacency slots of chunk c of a row of d slots (multiples of 64)
__device__ __forceinline__ void chunk_range(int64_t d, int c, int64_t *begin, int64_t *end) {
    const int64_t len = ((d + kRowChunks - 1) / kRowChunks + kWave - 1) / kWave * kWave;
    *begin = len * c < d ? len * c : d;
    *end = len * (c + 1) < d ? len * (c + 1) : d;
}

template <typename PtrT, typename IdxT>
__global__ void __launch_bounds__(kBlock)
k_lw_mass(const PtrT *__restrict__ row_ptr, const IdxT *__restrict__ col_idx, const IdxT *__restrict__ dst,
          const int64_t *__restrict__ sizes, unsigned long long *__restrict__ mass, uint32_t *__restrict__ bitmap,
          int64_t *__restrict__ zero_me) {
    const int lane = lane_id();
    if (zero_me && blockIdx.x == 0 && threadIdx.x == 0) *zero_me = 0;     // the candidate count k_lw_keys adds up
    const int64_t n = sizes[0] * kRowChunks;
    const int64_t wave0 = int64_t(blockIdx.x) * kWavesPerBlock + (threadIdx.x >> 6);
    const int64_t nwaves = int64_t(gridDim.x) * kWavesPerBlock;
    for (int64_t u = wave0; u < n; u += nwaves) {
        const int64_t t = u / kRowChunks;
        const int c = static_cast<int>(u % kRowChunks);
        const int64_t v = dst ? static_cast<int64_t>(dst[t]) : t;      // no row list: every node of the graph
        const int64_t start = static_cast<int64_t>(row_ptr[v]);
        const int64_t d = static_cast<int64_t>(row_ptr[v + 1]) - start;
        const unsigned long long add = (1ull << 40) / static_cast<unsigned long long>(d + 1);
        if (c == 0 && lane == 0) {
            atomicAdd(&mass[v], add);
            if (bitmap) set_bit(bitmap, static_cast<uint32_t>(v));
        }
        int64_t jb, je;
        chunk_range(d, c, &jb, &je);
        for (int64_t j = jb + lane; j < je; j += kWave) {
            const uint32_t i = static_cast<uint32_t>(col_idx[start + j]);
            atomicAdd(&mass[i], add);
            if (bitmap) set_bit(bitmap, i);
        }
    }
}

// Bitmap -> ascending list, two launches: the set bits of every tile are counted, then every tile's
// workgroup adds up the counts of the tiles before its own and writes its ids.  A tile is
// kBlock * WPT words (WPT = 1 up to 32 M nodes, ids staged through LDS and written coalesced;
// otherwise 4, one 16-byte load per thread, ids written from the bit loop: those bitmaps are sparse).
constexpr int kMassTileNodes = kBlock * 32;          // nodes behind one tile of kBlock words

// The touched nodes from the masses themselves (bit i = mass[i] != 0), for graphs small enough that
// reading every mass costs less than marking a bit per adjacency slot in k_lw_mass; the same launch
// counts the tile (WPT = 1).  In round r thread t looks at node tile * 8192 + r * 256 + t, so the
// ballot of a wavefront is the word pair r * 8 + 2 * wave of the tile.
__global__ void __launch_bounds__(kBlock)
k_lw_mass_bits(const unsigned long long *__restrict__ mass, int64_t n, uint32_t *__restrict__ bitmap,
               int32_t *__restrict__ tile_sums) {
    __shared__ unsigned long long pairs[kBlock / 2];
    __shared__ int lds[kWavesPerBlock];
    const int tid = threadIdx.x;
    const int wave = tid >> 6;
    const int64_t base = int64_t(blockIdx.x) * kMassTileNodes + tid;
    unsigned long long v[32];
#pragma unroll
    for (int r = 0; r < 32; ++r) {
        const int64_t i = base + r * kBlock;
        v[r] = i < n ? mass[i] : 0ull;
    }
    int cnt = 0;
#pragma unroll
    for (int r = 0; r < 32; ++r) {
        const uint64_t m = ballot64(v[r] != 0);
        cnt += popc64(m);
        if (lane_id() == 0) pairs[r * kWavesPerBlock + wave] = m;
    }
    if (lane_id() == 0) lds[wave] = cnt;
    __syncthreads();
    bitmap[int64_t(blockIdx.x) * kBlock + tid] = reinterpret_cast<const uint32_t *>(pairs)[tid];
    if (tid == 0) {
        int t = 0;
#pragma unroll
        for (int k = 0; k < kWavesPerBlock; ++k) t += lds[k];
        tile_sums[blockIdx.x] = t;
    }
}

template <int WPT>
__global__ void __launch_bounds__(kBlock)
k_lw_tile_counts(const uint32_t *__restrict__ bitmap, int32_t *__restrict__ tile_sums) {
    __shared__ int lds[kWavesPerBlock];
    const int64_t w0 = (int64_t(blockIdx.x) * kBlock + threadIdx.x) * WPT;
    int c;
    if (WPT == 4) {
        const uint4 w = *reinterpret_cast<const uint4 *>(bitmap + w0);
        c = __popc(w.x) + __popc(w.y) + __popc(w.z) + __popc(w.w);
    } else {
        c = __popc(bitmap[w0]);
    }
    const int s = wave_sum(c);
    if (lane_id() == 0) lds[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        int t = 0;
#pragma unroll
        for (int k = 0; k < kWavesPerBlock; ++k) t += lds[k];
        tile_sums[blockIdx.x] = t;
    }
}

// ids of the set bits, ascending, into out[0..total); the words are cleared; total to count_a/b.
// scanned: tile_vals holds the exclusive scan of the tile counts, otherwise the counts themselves.
template <typename OutT, int WPT>
__global__ void __launch_bounds__(kBlock)
k_lw_emit(uint32_t *__restrict__ bitmap, const int32_t *__restrict__ tile_vals, int scanned, OutT *__restrict__ out,
          int32_t *__restrict__ local_of, int64_t *count_a, int64_t *count_b) {
    __shared__ int lds[kWavesPerBlock];
    __shared__ int32_t staged[WPT == 1 ? kBlock * 32 : 1];   // every id of the tile, ascending
    const int tile_base = scanned ? tile_vals[blockIdx.x] : tiles_before(tile_vals, lds);
    const int64_t w0 = (int64_t(blockIdx.x) * kBlock + threadIdx.x) * WPT;
    uint32_t words[WPT];
    if constexpr (WPT == 4) {
        const uint4 w = *reinterpret_cast<const uint4 *>(bitmap + w0);
        words[0] = w.x;
        words[1] = w.y;
        words[2] = w.z;
        words[3] = w.w;
    } else {
        words[0] = bitmap[w0];
    }
    int c = 0;
#pragma unroll
    for (int q = 0; q < WPT; ++q) c += __popc(words[q]);
    int total;
    int ex = block_excl_scan<kWavesPerBlock>(c, &total, lds);
    if (blockIdx.x == gridDim.x - 1 && threadIdx.x == 0) {
        const int64_t all = int64_t(tile_base) + total;
        if (count_a) *count_a = all;
        if (count_b) *count_b = all;
    }
    if (total == 0) return;                                // workgroup-uniform
    if constexpr (WPT == 1) {
        if (c) {
            bitmap[w0] = 0;
            const int32_t v0 = static_cast<int32_t>(w0 * 32);
            uint32_t bits = words[0];
            while (bits) {
                const int b = __ffs(bits) - 1;
                bits &= bits - 1;
                staged[ex++] = v0 + b;
            }
        }
        __syncthreads();
        for (int k = threadIdx.x; k < total; k += kBlock) {
            const int32_t v = staged[k];
            out[tile_base + k] = static_cast<OutT>(v);
            if (local_of) local_of[v] = tile_base + k;
        }
    } else {
        if (c == 0) return;
        int32_t pos = tile_base + ex;
#pragma unroll
        for (int q = 0; q < WPT; ++q) {
            uint32_t bits = words[q];
            if (!bits) continue;
            bitmap[w0 + q] = 0;
            while (bits) {
                const int b = __ffs(bits) - 1;
                bits &= bits - 1;
                const int64_t v = (w0 + q) * 32 + b;
                out[pos] = static_cast<OutT>(v);
                if (local_of) local_of[v] = pos;
                ++pos;
            }
        }
    }
}

// The race key of a candidate and the measure its probability is proportional to.  Plain: rate
// q = mass / (deg + 1).  Flat (paper Eq. 10: in proportion to the column norm, not its square): rate
// sqrt(q); the race compares ticket / sqrt(q), and squaring that keeps the order with nothing but
// multiplications and one division, each rounded once, as the CPU statement of the same steps does.
__device__ __forceinline__ double lw_race_key(double ticket, double deg1, double m, int flat) {
    return flat ? ((ticket * ticket) * deg1) / m : (ticket * deg1) / m;
}
__device__ __forceinline__ double lw_measure(double m, double deg1, int flat) {
    const double q = m / deg1;
    return flat ? sqrt(q) : q;
}

// Radix select of the s-th smallest 64-bit key pattern: kSelPasses counting passes over all keys, most
// significant digit first - the top 12 bits (sign and exponent of a double), then 13 bits; what
// is left undecided after these 25 bits is a short list (k_lw_mark, k_lw_finish).
constexpr int kSelPasses = 2;
constexpr int kSelBins = 8192;
constexpr int kSelHistLen = kSelPasses * kSelBins;
__host__ __device__ constexpr int sel_shift(int pass) { return 52 - 13 * pass; }

// Race keys of the candidates and the per-workgroup partial sums of q (a fixed launch shape, so the
// sums are the same from run to run); the keys' leading 12 bits are counted into hist[0..4096) - the
// first pass of the radix select.  Candidates: cand[0..n) if given, otherwise the nodes 0..n-1
// themselves, of which those with no mass are none (key = all ones, not counted); their number is
// added to *count_out then.  n = *n_dev if given, else n_fixed.  hist must be clear.
constexpr uint64_t kNoKey = ~uint64_t(0);
template <typename PtrT>
__global__ void __launch_bounds__(kBlock)
k_lw_keys(const PtrT *__restrict__ row_ptr, const int32_t *__restrict__ cand, const int64_t *__restrict__ n_dev, int64_t n_fixed,
          const unsigned long long *__restrict__ mass, uint64_t tag_hash, int flat, uint64_t *__restrict__ key64,
          double *__restrict__ q_part, int32_t *__restrict__ hist, int64_t *__restrict__ count_out,
          unsigned long long *__restrict__ state, int64_t layer_size, unsigned long long *__restrict__ bcount) {
    __shared__ double lds[kWavesPerBlock];
    __shared__ int cnt_lds[kWavesPerBlock];
    __shared__ int h[4096];
    if (blockIdx.x == 0 && threadIdx.x == 0) {             // the select's state before its first pass
        state[0] = 0;
        state[1] = static_cast<unsigned long long>(layer_size);
        *bcount = 0;                                       // the boundary list is empty
    }
    const int64_t n = n_dev ? *n_dev : n_fixed;
    const int64_t stride = int64_t(gridDim.x) * kBlock;
#pragma unroll
    for (int q = 0; q < 4096 / kBlock; ++q) h[q * kBlock + threadIdx.x] = 0;
    __syncthreads();
    double q = 0.0;
    int cnt = 0;
    for (int64_t c = int64_t(blockIdx.x) * kBlock + threadIdx.x; c < n; c += stride) {
        const int64_t i = cand ? cand[c] : c;
        const unsigned long long mi = mass[i];
        if (mi == 0) {
            key64[c] = kNoKey;
            continue;
        }
        const double deg1 = static_cast<double>(static_cast<int64_t>(row_ptr[i + 1]) - static_cast<int64_t>(row_ptr[i]) + 1);
        const double m = static_cast<double>(mi);
        const double ticket = static_cast<double>(exp_ticket64(mix64(mix64(tag_hash ^ static_cast<uint64_t>(i)))));
        const uint64_t key = static_cast<uint64_t>(__double_as_longlong(lw_race_key(ticket, deg1, m, flat)));
        key64[c] = key;
        atomicAdd(&h[key >> 52], 1);
        q += lw_measure(m, deg1, flat);
        ++cnt;
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) q += __shfl_xor(q, off, 64);
    cnt = wave_sum(cnt);
    if (lane_id() == 0) {
        lds[threadIdx.x >> 6] = q;
        cnt_lds[threadIdx.x >> 6] = cnt;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        q_part[blockIdx.x] = ((lds[0] + lds[1]) + lds[2]) + lds[3];
        const int total = cnt_lds[0] + cnt_lds[1] + cnt_lds[2] + cnt_lds[3];
        if (count_out && total) atomicAdd(reinterpret_cast<unsigned long long *>(count_out), static_cast<unsigned long long>(total));
    }
#pragma unroll
    for (int q4 = 0; q4 < 4096 / kBlock; ++q4) {
        const int d = q4 * kBlock + threadIdx.x;
        if (h[d]) atomicAdd(&hist[d], h[d]);
    }
}

// q_total = sum of the partial sums, in a fixed order (one workgroup; `lds` needs kBlock doubles)
__device__ __forceinline__ void lw_sum_parts(const double *__restrict__ q_part, int parts, double *__restrict__ q_total, double *lds) {
    double a = 0.0;
    for (int k = threadIdx.x; k < parts; k += kBlock) a += q_part[k];
    lds[threadIdx.x] = a;
    __syncthreads();
    for (int off = kBlock / 2; off > 0; off >>= 1) {
        if (static_cast<int>(threadIdx.x) < off) lds[threadIdx.x] += lds[threadIdx.x + off];
        __syncthreads();
    }
    if (threadIdx.x == 0) *q_total = lds[0];
}

// The state of the select before pass `pass`:
//   st[0] = the digits chosen in the passes before, most significant first, as the low bits of a word
//   st[1] = how many of the keys with that prefix are still wanted
// derived from the state before the previous pass (state[2(pass-1)], state[2(pass-1)+1]) and that
// pass's histogram: the first digit at which the running count reaches the wanted number.  Every
// thread of the workgroup calls it; st[] is valid after the next __syncthreads().  If fewer keys
// exist than are wanted no digit qualifies and st stays {0, 0}.
__device__ __forceinline__ void sel_derive(const unsigned long long *__restrict__ state, const int32_t *__restrict__ hist,
                                           int64_t layer_size, int pass, unsigned long long *st, int *lds) {
    const int tid = threadIdx.x;
    if (pass == 0) {
        if (tid == 0) {
            st[0] = 0;
            st[1] = static_cast<unsigned long long>(layer_size);
        }
        return;
    }
    if (tid == 0) {
        st[0] = 0;
        st[1] = 0;
    }
    const unsigned long long prefix = state[2 * (pass - 1)];
    const long long want = static_cast<long long>(state[2 * (pass - 1) + 1]);
    constexpr int kPer = kSelBins / kBlock;                // consecutive digits per thread
    const int4 *hp = reinterpret_cast<const int4 *>(hist + int64_t(pass - 1) * kSelBins + tid * kPer);
    int v[kPer];
    int c = 0;
#pragma unroll
    for (int q = 0; q < kPer / 4; ++q) {
        const int4 x = hp[q];
        v[4 * q] = x.x;
        v[4 * q + 1] = x.y;
        v[4 * q + 2] = x.z;
        v[4 * q + 3] = x.w;
        c += x.x + x.y + x.z + x.w;
    }
    int total;
    const int before = block_excl_scan<kWavesPerBlock>(c, &total, lds);   // its barriers order the stores to st[] above
    // exactly one digit has before < want <= before + count (if 1 <= want <= total)
    if (before < want && want <= static_cast<long long>(before) + c) {
        long long run = before;
#pragma unroll
        for (int q = 0; q < kPer; ++q) {
            if (run < want && want <= run + v[q]) {
                st[0] = (prefix << 13) | static_cast<unsigned long long>(tid * kPer + q);
                st[1] = static_cast<unsigned long long>(want - run);
            }
            run += v[q];
        }
    }
}

// Counting pass `pass` of the select: the keys that carry the prefix found so far are counted by
// their next digit, per workgroup in LDS and then into hist[pass].  Workgroup 0 stores the state.
__global__ void __launch_bounds__(kBlock)
k_lw_select(const uint64_t *__restrict__ key64, const int64_t *__restrict__ n_dev, int64_t n_fixed, int64_t layer_size,
            unsigned long long *__restrict__ state, int32_t *__restrict__ hist, int pass) {
    __shared__ int lds[kWavesPerBlock];
    __shared__ int h[kSelBins];
    __shared__ unsigned long long st[2];
    const int tid = threadIdx.x;
    sel_derive(state, hist, layer_size, pass, st, lds);
#pragma unroll
    for (int q = 0; q < kSelBins / kBlock; ++q) h[q * kBlock + tid] = 0;
    __syncthreads();
    if (blockIdx.x == 0 && tid == 0) {
        state[2 * pass] = st[0];
        state[2 * pass + 1] = st[1];
    }
    const unsigned long long prefix = st[0];
    const int shift = sel_shift(pass);
    const int64_t n = n_dev ? *n_dev : n_fixed;
    const int64_t stride = int64_t(gridDim.x) * kBlock;
    int mine = 0;
    for (int64_t c = int64_t(blockIdx.x) * kBlock + tid; c < n; c += stride) {
        const uint64_t k = key64[c];
        if (pass == 0 || (k >> (shift + 13)) == prefix) {
            atomicAdd(&h[(k >> shift) & (kSelBins - 1)], 1);
            mine = 1;
        }
    }
    if (!__syncthreads_or(mine)) return;                   // no key of this workgroup carries the prefix
#pragma unroll
    for (int q = 0; q < kSelBins / kBlock; ++q) {
        const int d = q * kBlock + tid;
        if (h[d]) atomicAdd(&hist[pass * kSelBins + d], h[d]);
    }
}

// n keys (*n_dev if given, else n_fixed), of which *n_cand are candidates (all of them without
// n_cand; with skip_no_key the keys equal to kNoKey are none).
// After the two counting passes 25 leading bits of the threshold are known (every workgroup derives
// them from the second histogram; workgroup 0 stores them and the number of keys still wanted among
// those that share them in state[4], state[5]).  Keys with smaller leading bits are marked.  Keys with
// these leading bits - a few dozen of random keys - go to the boundary list (key, position), which
// k_lw_finish settles.  Workgroup 0 also adds up the partial sums of q, if there are any.
constexpr int kSelKnownShift = 39;                        // bits below the two counted digits
__global__ void __launch_bounds__(kBlock)
k_lw_mark(const int32_t *__restrict__ cand, const uint64_t *__restrict__ key64, const int64_t *__restrict__ n_dev, int64_t n_fixed,
          const int64_t *__restrict__ n_cand, int skip_no_key, int64_t layer_size, unsigned long long *__restrict__ state,
          const int32_t *__restrict__ hist, uint32_t *__restrict__ bitmap, const double *__restrict__ q_part, int parts,
          double *__restrict__ q_total, uint64_t *__restrict__ bkey, int32_t *__restrict__ bpos,
          unsigned long long *__restrict__ bcount) {
    __shared__ double qlds[kBlock];
    __shared__ int lds[kWavesPerBlock];
    __shared__ unsigned long long st[2];
    if (q_part && blockIdx.x == 0) lw_sum_parts(q_part, parts, q_total, qlds);
    const int64_t n = n_dev ? *n_dev : n_fixed;            // keys
    const int64_t stride = int64_t(gridDim.x) * kBlock;
    if ((n_cand ? *n_cand : n) <= layer_size) {            // every candidate is drawn
        for (int64_t c = int64_t(blockIdx.x) * kBlock + threadIdx.x; c < n; c += stride)
            if (!skip_no_key || key64[c] != kNoKey) set_bit(bitmap, cand ? static_cast<uint32_t>(cand[c]) : static_cast<uint32_t>(c));
        return;
    }
    sel_derive(state, hist, layer_size, 2, st, lds);
    __syncthreads();
    const uint64_t lead = st[0];
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        state[4] = st[0];
        state[5] = st[1];
    }
    const int lane = lane_id();
    const int64_t first = int64_t(blockIdx.x) * kBlock + threadIdx.x;
    for (int64_t c0 = first - lane; c0 < n; c0 += stride) {          // whole wavefronts: the ballot below
        const int64_t c = c0 + lane;
        const uint64_t k = c < n ? key64[c] : kNoKey;
        const uint64_t kl = k >> kSelKnownShift;
        if (c < n && kl < lead) set_bit(bitmap, cand ? static_cast<uint32_t>(cand[c]) : static_cast<uint32_t>(c));
        const bool edge = c < n && kl == lead;
        const uint64_t m = ballot64(edge);
        if (m) {
            unsigned long long at = 0;
            if (lane == 0) at = atomicAdd(bcount, static_cast<unsigned long long>(popc64(m)));
            at = __shfl(at, 0, 64);
            if (edge) {
                const unsigned long long o = at + popc64(m & lanes_below(lane));
                bkey[o] = k;
                bpos[o] = static_cast<int32_t>(c);
            }
        }
    }
}

// The boundary list: m keys that share the 25 known leading bits, of which the state[5] smallest in
// (key, position) order are drawn (positions ascend with the ids).  One workgroup.  Up to
// kBoundaryRanked entries: every entry counts the entries ahead of it.  More (many equal keys):
// a radix select over the remaining 39 key bits and, among the keys equal to the threshold, over the
// 32 position bits, eight bits at a time.
constexpr int kBoundaryRanked = 1024;
__global__ void __launch_bounds__(kBlock)
k_lw_finish(const int32_t *__restrict__ cand, const int64_t *__restrict__ n_dev, int64_t n_fixed,
            const int64_t *__restrict__ n_cand, int64_t layer_size, const unsigned long long *__restrict__ state,
            const uint64_t *__restrict__ bkey, const int32_t *__restrict__ bpos, const unsigned long long *__restrict__ bcount,
            uint32_t *__restrict__ bitmap) {
    __shared__ uint64_t lk[kBoundaryRanked];
    __shared__ int32_t lp[kBoundaryRanked];
    __shared__ int h[256];
    __shared__ int lds[kWavesPerBlock];
    __shared__ long long pick[2];
    const int tid = threadIdx.x;
    const int64_t n = n_dev ? *n_dev : n_fixed;
    if ((n_cand ? *n_cand : n) <= layer_size) return;      // every candidate was drawn by k_lw_mark
    const int64_t m = static_cast<int64_t>(*bcount);
    long long want = static_cast<long long>(state[5]);
    if (m <= kBoundaryRanked) {
        for (int e = tid; e < m; e += kBlock) {
            lk[e] = bkey[e];
            lp[e] = bpos[e];
        }
        __syncthreads();
        constexpr int PER = kBoundaryRanked / kBlock;
        uint64_t mk[PER];
        int32_t mp[PER];
        int rank[PER];
#pragma unroll
        for (int q = 0; q < PER; ++q) {
            const int e = q * kBlock + tid;
            mk[q] = e < m ? lk[e] : 0;
            mp[q] = e < m ? lp[e] : 0;
            rank[q] = 0;
        }
        for (int j = 0; j < m; ++j) {
            const uint64_t ok = lk[j];
            const int32_t op = lp[j];
#pragma unroll
            for (int q = 0; q < PER; ++q) rank[q] += (ok < mk[q] || (ok == mk[q] && op < mp[q])) ? 1 : 0;
        }
#pragma unroll
        for (int q = 0; q < PER; ++q) {
            const int e = q * kBlock + tid;
            if (e < m && rank[q] < want) set_bit(bitmap, cand ? static_cast<uint32_t>(cand[mp[q]]) : static_cast<uint32_t>(mp[q]));
        }
        return;
    }
    // radix select: first the key (bits 38..0: seven bits, then four times eight), then the position
    uint64_t kp = state[4] << kSelKnownShift;              // the threshold key as far as known
    int known = kSelKnownShift;                            // its bits from here up are known
    uint32_t pp = 0;                                       // the threshold position as far as known
    int pknown = 32;
    for (int pass = 0; pass < 9; ++pass) {
        const bool on_key = pass < 5;
        const int shift = on_key ? 32 - 8 * pass : 24 - 8 * (pass - 5);
        h[tid] = 0;
        __syncthreads();
        for (int64_t e = tid; e < m; e += kBlock) {
            const uint64_t k = bkey[e];
            if (on_key) {
                if ((k >> known) == (kp >> known)) atomicAdd(&h[(k >> shift) & 255], 1);
            } else if (k == kp) {
                const uint32_t ps = static_cast<uint32_t>(bpos[e]);
                if (pknown == 32 || (ps >> pknown) == (pp >> pknown)) atomicAdd(&h[(ps >> shift) & 255], 1);
            }
        }
        __syncthreads();
        const int c = h[tid];
        int total;
        const int before = block_excl_scan<kWavesPerBlock>(c, &total, lds);
        if (before < want && want <= static_cast<long long>(before) + c) {      // exactly one digit
            pick[0] = tid;
            pick[1] = want - before;
        }
        __syncthreads();
        const uint64_t digit = static_cast<uint64_t>(pick[0]);
        want = pick[1];
        if (on_key) {
            kp |= digit << shift;
            known = shift;
        } else {
            pp |= static_cast<uint32_t>(digit) << shift;
            pknown = shift;
        }
        __syncthreads();                                   // pick[] and h[] are rewritten by the next pass
    }
    // kp, pp: the last drawn entry
    for (int64_t e = tid; e < m; e += kBlock) {
        const uint64_t k = bkey[e];
        const int32_t ps = bpos[e];
        if (k < kp || (k == kp && static_cast<uint32_t>(ps) <= pp)) set_bit(bitmap, cand ? static_cast<uint32_t>(cand[ps]) : static_cast<uint32_t>(ps));
    }
}

__global__ void __launch_bounds__(kBlock)
k_lw_zero_i32(int32_t *__restrict__ p, int64_t n) {
    const int64_t i = int64_t(blockIdx.x) * kBlock + threadIdx.x;
    if (i < n) p[i] = 0;
}

// Eq. 8 with p_i = q_i / q_total, q_i = mass_i / di: P_vi / (s p_i) = (q_total / s) * di / (mass_i sqrt(dv di))
// With debiased coefficients (paper Eq. 12) the column of the drawn node at source position li is scaled
// by beta[li] instead: P_vi * beta.
template <typename PtrT>
__device__ __forceinline__ double lw_raw_weight(const PtrT *__restrict__ row_ptr, const unsigned long long *__restrict__ mass,
                                                double scale, double dv, int64_t i, const double *__restrict__ beta, int32_t li,
                                                int flat) {
    const double di = static_cast<double>(static_cast<int64_t>(row_ptr[i + 1]) - static_cast<int64_t>(row_ptr[i]) + 1);
    if (beta) return beta[li] / sqrt(dv * di);
    if (flat) return scale / (sqrt(static_cast<double>(mass[i]) / di) * sqrt(dv * di));   // p_i = sqrt(q_i) / total
    return scale * di / (static_cast<double>(mass[i]) * sqrt(dv * di));
}

// per (row, chunk): the number of drawn nodes in the chunk's slots (chunk 0 also counts the self
// edge) and the sum of their raw weights
template <typename PtrT, typename IdxT>
__global__ void __launch_bounds__(kBlock)
k_lw_count(const PtrT *__restrict__ row_ptr, const IdxT *__restrict__ col_idx, const IdxT *__restrict__ dst,
           const int64_t *__restrict__ sizes, const int32_t *__restrict__ local_of, const unsigned long long *__restrict__ mass,
           const double *__restrict__ q_total, const double *__restrict__ beta, int flat, int32_t *__restrict__ counts,
           double *__restrict__ psum) {
    const int lane = lane_id();
    const int64_t n = sizes[0] * kRowChunks;
    const double scale = *q_total / static_cast<double>(sizes[1]);
    const int64_t wave0 = int64_t(blockIdx.x) * kWavesPerBlock + (threadIdx.x >> 6);
    const int64_t nwaves = int64_t(gridDim.x) * kWavesPerBlock;
    for (int64_t u = wave0; u < n; u += nwaves) {
        const int64_t t = u / kRowChunks;
        const int c = static_cast<int>(u % kRowChunks);
        const int64_t v = static_cast<int64_t>(dst[t]);
        const int64_t start = static_cast<int64_t>(row_ptr[v]);
        const int64_t d = static_cast<int64_t>(row_ptr[v + 1]) - start;
        const double dv = static_cast<double>(d + 1);
        int cnt = 0;
        double acc = 0.0;
        if (c == 0 && local_of[v] >= 0) {
            cnt = 1;
            if (lane == 0) acc = lw_raw_weight(row_ptr, mass, scale, dv, v, beta, local_of[v], flat);
        }
        int64_t jb, je;
        chunk_range(d, c, &jb, &je);
        for (int64_t base = jb; base < je; base += kWave) {
            const int64_t j = base + lane;
            bool in = false;
            if (j < je) {
                const int64_t i = static_cast<int64_t>(col_idx[start + j]);
                const int32_t li = local_of[i];
                in = li >= 0;
                if (in) acc += lw_raw_weight(row_ptr, mass, scale, dv, i, beta, li, flat);
            }
            cnt += popc64(ballot64(in));
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off, 64);
        if (lane == 0) {
            counts[u] = cnt;
            psum[u] = acc;
        }
    }
}

template <typename PtrT, typename IdxT>
__global__ void __launch_bounds__(kBlock)
k_lw_fill(const PtrT *__restrict__ row_ptr, const IdxT *__restrict__ col_idx, const IdxT *__restrict__ dst,
          int64_t *sizes, const int32_t *__restrict__ local_of, const unsigned long long *__restrict__ mass,
          const double *__restrict__ q_total, const double *__restrict__ beta, int flat, const int32_t *__restrict__ offs,
          const double *__restrict__ psum, int32_t *__restrict__ indptr, int32_t *__restrict__ indices,
          float *__restrict__ edge_w, int normalise, int64_t cap_nnz, const int32_t *__restrict__ seed_flags) {
    const int lane = lane_id();
    const int64_t rows = sizes[0];
    const int64_t n = rows * kRowChunks;
    const double scale = *q_total / static_cast<double>(sizes[1]);
    if (blockIdx.x == 0 && threadIdx.x == 0) {             // the end of indptr, the block's nnz and flags
        const int64_t nnz = offs[n];
        indptr[rows] = static_cast<int32_t>(nnz);
        sizes[2] = nnz < cap_nnz ? nnz : cap_nnz;
        sizes[3] = (seed_flags ? *seed_flags : 0) | (nnz > cap_nnz ? 4 : 0);
    }
    const int64_t wave0 = int64_t(blockIdx.x) * kWavesPerBlock + (threadIdx.x >> 6);
    const int64_t nwaves = int64_t(gridDim.x) * kWavesPerBlock;
    for (int64_t u = wave0; u < n; u += nwaves) {
        const int64_t t = u / kRowChunks;
        const int c = static_cast<int>(u % kRowChunks);
        if (c == 0 && lane == 0) indptr[t] = offs[u];      // first edge position of row t
        if (offs[u + 1] == offs[u]) continue;              // nothing drawn in this chunk (wavefront-uniform)
        const int64_t v = static_cast<int64_t>(dst[t]);
        const int64_t start = static_cast<int64_t>(row_ptr[v]);
        const int64_t d = static_cast<int64_t>(row_ptr[v + 1]) - start;
        const double dv = static_cast<double>(d + 1);
        double inv_sum = 1.0;
        if (normalise) {                                   // the row's sum: its chunks' partial sums in order
            double row_sum = 0.0;
            for (int k = 0; k < kRowChunks; ++k) row_sum += psum[t * kRowChunks + k];
            inv_sum = 1.0 / row_sum;
        }
        int64_t pos = offs[u];
        if (c == 0) {
            const int32_t self_pos = local_of[v];
            if (self_pos >= 0) {
                if (lane == 0 && pos < cap_nnz) {
                    indices[pos] = self_pos;
                    edge_w[pos] = static_cast<float>(lw_raw_weight(row_ptr, mass, scale, dv, v, beta, self_pos, flat) * inv_sum);
                }
                pos += 1;
            }
        }
        int64_t jb, je;
        chunk_range(d, c, &jb, &je);
        for (int64_t base = jb; base < je; base += kWave) {
            const int64_t j = base + lane;
            int64_t i = 0;
            int32_t li = -1;
            if (j < je) {
                i = static_cast<int64_t>(col_idx[start + j]);
                li = local_of[i];
            }
            const uint64_t m = ballot64(li >= 0);
            if (li >= 0) {
                const int64_t p = pos + popc64(m & lanes_below(lane));
                if (p < cap_nnz) {
                    indices[p] = li;
                    edge_w[p] = static_cast<float>(lw_raw_weight(row_ptr, mass, scale, dv, i, beta, li, flat) * inv_sum);
                }
            }
            pos += popc64(m);
        }
    }
}

// ---- debiased coefficients (paper Eq. 12) of the drawn nodes

// race key and q = mass / (deg + 1) of every drawn node, by source position
template <typename PtrT, typename IdxT>
__global__ void __launch_bounds__(kBlock)
k_lw_drawn_keys(const PtrT *__restrict__ row_ptr, const IdxT *__restrict__ src_ids, const int64_t *__restrict__ sizes,
                const unsigned long long *__restrict__ mass, uint64_t tag_hash, int flat, uint64_t *__restrict__ dkey,
                double *__restrict__ dq) {
    const int64_t ns = sizes[1];
    const int64_t pos = int64_t(blockIdx.x) * kBlock + threadIdx.x;
    if (pos >= ns) return;
    const int64_t i = static_cast<int64_t>(src_ids[pos]);
    const double deg1 = static_cast<double>(static_cast<int64_t>(row_ptr[i + 1]) - static_cast<int64_t>(row_ptr[i]) + 1);
    const double m = static_cast<double>(mass[i]);
    const double ticket = static_cast<double>(exp_ticket64(mix64(mix64(tag_hash ^ static_cast<uint64_t>(i)))));
    dkey[pos] = static_cast<uint64_t>(__double_as_longlong(lw_race_key(ticket, deg1, m, flat)));
    dq[pos] = lw_measure(m, deg1, flat);
}

// order[r] = source position of the r-th drawn node: the race order is ascending (key, id), and
// positions ascend with the ids.  Every thread counts the drawn nodes ahead of its own.
__global__ void __launch_bounds__(kBlock)
k_lw_draw_order(const uint64_t *__restrict__ dkey, const int64_t *__restrict__ sizes, int32_t *__restrict__ order) {
    const int64_t ns = sizes[1];
    const int64_t pos = int64_t(blockIdx.x) * kBlock + threadIdx.x;
    if (pos >= ns) return;
    const uint64_t k = dkey[pos];
    int rank = 0;
    for (int64_t t = 0; t < ns; ++t) {
        const uint64_t o = dkey[t];
        rank += (o < k || (o == k && t < pos)) ? 1 : 0;
    }
    order[rank] = static_cast<int32_t>(pos);
}

// Inclusive scan over the 256 threads of a workgroup with a binary operation on doubles (sum or
// product); *total gets the workgroup's result.  `lds` needs kWavesPerBlock doubles.
template <bool PRODUCT>
__device__ __forceinline__ double lw_block_scan_incl(double v, double *total, double *lds) {
    const int lane = lane_id();
    const int wave = static_cast<int>(threadIdx.x) >> 6;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const double t = __shfl_up(v, off, 64);
        if (lane >= off) v = PRODUCT ? v * t : v + t;
    }
    __syncthreads();                                       // lds may still be read from an earlier use
    if (lane == 63) lds[wave] = v;
    __syncthreads();
    double before = PRODUCT ? 1.0 : 0.0, all = PRODUCT ? 1.0 : 0.0;
#pragma unroll
    for (int k = 0; k < kWavesPerBlock; ++k) {
        const double t = lds[k];
        if (k < wave) before = PRODUCT ? before * t : before + t;
        all = PRODUCT ? all * t : all + t;
    }
    *total = all;
    return PRODUCT ? before * v : before + v;
}

// The recursion of Eq. 12 in closed form.  With a_r = n / ((n - r)(r + 1)) (r = 0 for the first draw)
// and b0_r = a_r (1 - sum of the p drawn before) / p_r the coefficient an item gets when it is
// drawn, later steps turn a coefficient b into (1 - a_u) b + a_u, so the final one is
//   beta_r = b0_r G_r + H_r,  G_r = prod_{u > r} (1 - a_u),  H_r = sum_{u > r} a_u G_u.
// One workgroup: a prefix sum over the draws for b0, then, from the last draw backwards, a prefix
// product for G and a prefix sum of a_u G_u for H, 256 draws at a time with running carries.
// Every candidate drawn: beta = 1.
__global__ void __launch_bounds__(kBlock)
k_lw_debias(const int32_t *__restrict__ order, const double *__restrict__ dq, const double *__restrict__ q_total,
            const int64_t *__restrict__ sizes, const int64_t *__restrict__ n_cand, double *__restrict__ b0,
            double *__restrict__ beta) {
    __shared__ double lds[kWavesPerBlock];
    __shared__ double incl_of[kBlock];
    const int64_t s = sizes[1];
    const int64_t n = *n_cand;
    if (s >= n) {
        for (int64_t r = threadIdx.x; r < s; r += kBlock) beta[r] = 1.0;
        return;
    }
    const double total = *q_total;
    const double nd = static_cast<double>(n);
    double drawn = 0.0;                                    // probability mass of the draws before this chunk
    for (int64_t base = 0; base < s; base += kBlock) {
        const int64_t r = base + threadIdx.x;
        const bool in = r < s;
        const double p = in ? dq[order[r]] / total : 0.0;
        double chunk;
        const double incl = lw_block_scan_incl<false>(p, &chunk, lds);
        if (in) {
            const double alpha = nd / (static_cast<double>(n - r) * static_cast<double>(r + 1));
            b0[r] = alpha * (1.0 - (drawn + (incl - p))) / p;
        }
        drawn += chunk;
    }
    __syncthreads();
    double G = 1.0, H = 0.0;                               // over the draws after this chunk
    for (int64_t top = s; top > 0; top -= kBlock) {        // thread t takes draw top - 1 - t
        const int64_t r = top - 1 - threadIdx.x;
        const bool in = r >= 0;
        const double alpha = in ? nd / (static_cast<double>(n - r) * static_cast<double>(r + 1)) : 0.0;
        const double x = 1.0 - alpha;
        double gprod, hsum;
        const double g_incl = lw_block_scan_incl<true>(x, &gprod, lds);
        incl_of[threadIdx.x] = g_incl;                     // the exclusive product is the previous thread's inclusive one
        __syncthreads();
        const double Gr = G * (threadIdx.x == 0 ? 1.0 : incl_of[threadIdx.x - 1]);
        const double term = alpha * Gr;
        const double h_incl = lw_block_scan_incl<false>(term, &hsum, lds);
        if (in) beta[order[r]] = b0[r] * Gr + (H + (h_incl - term));
        H += hsum;
        G *= gprod;
        __syncthreads();                                   // incl_of[] is rewritten by the next chunk
    }
}

template <typename IdxT>
__global__ void __launch_bounds__(kBlock)
k_lw_reset(const int32_t *__restrict__ cand, const int64_t *__restrict__ n_cand, int64_t all_nodes,
           unsigned long long *__restrict__ mass, const IdxT *__restrict__ src_ids, const int64_t *__restrict__ sizes,
           int32_t *__restrict__ local_of, int32_t *__restrict__ flags, int32_t *__restrict__ sel_hist, int hist_len) {
    if (flags && blockIdx.x == 0 && threadIdx.x == 0) *flags = 0;     // the seed check's word, for the next call
    const int64_t ns = sizes[1];
    const int64_t stride = int64_t(gridDim.x) * kBlock;
    for (int64_t k = int64_t(blockIdx.x) * kBlock + threadIdx.x; k < hist_len; k += stride) sel_hist[k] = 0;   // for the next block
    if (cand) {
        const int64_t nc = *n_cand;
        for (int64_t k = int64_t(blockIdx.x) * kBlock + threadIdx.x; k < nc; k += stride) mass[cand[k]] = 0;
    } else {
        for (int64_t k = int64_t(blockIdx.x) * kBlock + threadIdx.x; k < all_nodes; k += stride) mass[k] = 0;
    }
    for (int64_t k = int64_t(blockIdx.x) * kBlock + threadIdx.x; k < ns; k += stride) local_of[src_ids[k]] = -1;
}

__global__ void k_lw_store_i64(int64_t *p, int64_t v, int64_t *zero) {
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        *p = v;
        if (zero) *zero = 0;
    }
}


template <typename T>
bool dev_alloc(T **p, int64_t count) {
    return hipMalloc(reinterpret_cast<void **>(p), static_cast<size_t>(std::max<int64_t>(count, 1)) * sizeof(T)) == hipSuccess;
}

}  // namespace

void free_layerwise_scratch(mqg_ctx *ctx) {
    LayerwiseScratch &w = ctx->lw;
    void *ptrs[] = {w.mass, w.cand, w.key64, w.bkey, w.bpos, w.xkey, w.xpos, w.word_offs, w.scan_tiles, w.q_part, w.counters, w.q_total, w.seeds_copy, w.flags,
                    w.sel_state, w.sel_hist, w.chunk_offs, w.chunk_scan, w.chunk_sum, w.fg_mass, w.dkey, w.dq, w.order, w.beta};
    for (void *p : ptrs) (void)hipFree(p);
    w = LayerwiseScratch{};
}

// scratch of the layer-wise sampler: about 32 bytes per graph node, allocated at the first call
int ensure_layerwise_scratch(mqg_ctx *ctx, int64_t rows_cap, hipStream_t s) {
    LayerwiseScratch &w = ctx->lw;
    if (w.mass && rows_cap <= w.rows_cap) return MQG_OK;
    hipError_t e = hipStreamSynchronize(s);
    if (e != hipSuccess) return fail(ctx, MQG_ERR_HIP, std::string("mqg_sample_layerwise: ") + hipGetErrorString(e));
    free_layerwise_scratch(ctx);
    const int64_t n = std::max<int64_t>(ctx->num_nodes, 1);
    const int64_t chunks = rows_cap * kRowChunks;
    const int64_t scan_len = std::max<int64_t>(ctx->bitmap_words + 1, chunks + 1);
    bool ok = dev_alloc(&w.mass, n) && dev_alloc(&w.cand, n) && dev_alloc(&w.key64, n) && dev_alloc(&w.bkey, n) && dev_alloc(&w.bpos, n) && dev_alloc(&w.word_offs, ctx->bitmap_words + 1) &&
              dev_alloc(&w.scan_tiles, ceil_div(scan_len, kScanTile) + 2) && dev_alloc(&w.q_part, ceil_div(n, kBlock) + 1) &&
              dev_alloc(&w.counters, 4) && dev_alloc(&w.q_total, 1) && dev_alloc(&w.seeds_copy, rows_cap) && dev_alloc(&w.flags, 1) &&
              dev_alloc(&w.sel_state, 18) && dev_alloc(&w.sel_hist, kSelHistLen) && dev_alloc(&w.chunk_offs, chunks + 1) &&
              dev_alloc(&w.chunk_scan, std::min<int64_t>(chunks + 1, int64_t(kScanSelfTiles) * kScanTile)) &&
              dev_alloc(&w.chunk_sum, chunks) && dev_alloc(&w.dkey, rows_cap) && dev_alloc(&w.dq, rows_cap) &&
              dev_alloc(&w.order, rows_cap) && dev_alloc(&w.beta, rows_cap);
    if (ok) ok = hipMemset(w.mass, 0, static_cast<size_t>(n) * sizeof(unsigned long long)) == hipSuccess &&
                 hipMemset(w.flags, 0, sizeof(int32_t)) == hipSuccess && hipDeviceSynchronize() == hipSuccess;
    if (!ok) {
        free_layerwise_scratch(ctx);
        return fail(ctx, MQG_ERR_HIP, "mqg_sample_layerwise: scratch allocation failed");
    }
    w.rows_cap = rows_cap;
    return MQG_OK;
}

template <typename PtrT, typename IdxT>
static int sample_layerwise_impl(mqg_ctx *ctx, const mqg_graph *g, const void *seeds_v, int32_t num_seeds,
                                 const int32_t *layer_sizes, int32_t L, uint64_t rng_seed, int32_t normalise, bool fastgcn, bool debias, bool flat_p,
                                 mqg_block *blocks, float *const *edge_w, hipStream_t s) {
    LayerwiseScratch &w = ctx->lw;
    const int flat = flat_p ? 1 : 0;
    const PtrT *row_ptr = static_cast<const PtrT *>(g->row_ptr);
    const IdxT *col_idx = static_cast<const IdxT *>(g->col_idx);
    const int64_t n = ctx->num_nodes;
    // bitmap -> list: tiles of kBlock * wpt words, counted by the launch before (w.word_offs)
    const int wpt = ctx->bitmap_words <= (int64_t(1) << 20) ? 1 : 4;
    const int tiles = static_cast<int>(ctx->bitmap_words / (int64_t(kBlock) * wpt));
    const int tiles_scanned = tiles > kSelfPrefixTiles ? 1 : 0;
    auto count_tiles = [&]() -> int {
        if (wpt == 1) MQG_LAUNCH(ctx, "k_lw_tile_counts", s, (k_lw_tile_counts<1><<<tiles, kBlock, 0, s>>>(ctx->bitmap, w.word_offs)));
        else MQG_LAUNCH(ctx, "k_lw_tile_counts", s, (k_lw_tile_counts<4><<<tiles, kBlock, 0, s>>>(ctx->bitmap, w.word_offs)));
        return MQG_OK;
    };
    auto emit_list = [&](auto *out, int32_t *local_of, int64_t *count_a, int64_t *count_b) -> int {
        using OutT = std::remove_pointer_t<decltype(out)>;
        if (tiles_scanned) {
            int rc = device_scan(ctx, w.word_offs, tiles, w.scan_tiles, s);
            if (rc != MQG_OK) return rc;
        }
        if (wpt == 1)
            MQG_LAUNCH(ctx, "k_lw_emit", s, (k_lw_emit<OutT, 1><<<tiles, kBlock, 0, s>>>(ctx->bitmap, w.word_offs, tiles_scanned, out, local_of, count_a, count_b)));
        else
            MQG_LAUNCH(ctx, "k_lw_emit", s, (k_lw_emit<OutT, 4><<<tiles, kBlock, 0, s>>>(ctx->bitmap, w.word_offs, tiles_scanned, out, local_of, count_a, count_b)));
        return MQG_OK;
    };
    const int cand_grid = static_cast<int>(std::max<int64_t>(1, ceil_div(n, kBlock)));
    const uint64_t seed_hash = host_mix64(rng_seed + kGolden);
    // Three ways to the candidates.  FastGCN: every node, with batch-independent masses.  Graphs of up
    // to kDenseNodes nodes: every node gets a key slot and the nodes without mass hold no key - no
    // candidate list, a node's key sits at its id (on "medium" 200 k of the 233 k nodes are candidates
    // anyway).  Otherwise: the list of touched nodes, ascending.
    const int how = ctx->layerwise_candidates;
    const bool dense = !fastgcn && (how == 0 ? n <= kDenseNodes : how == 1);
    const bool keyed_by_id = fastgcn || dense;
    int64_t *n_cand = fastgcn ? w.counters + 2 : w.counters;
    const int32_t *cand = keyed_by_id ? nullptr : w.cand;
    const int64_t *n_keys_dev = keyed_by_id ? nullptr : w.counters;       // keyed by id: n keys
    const unsigned long long *mass = fastgcn ? w.fg_mass : w.mass;
    unsigned long long *bcount = reinterpret_cast<unsigned long long *>(w.counters + 3);
    if (fastgcn && !w.fg_ready) {
        // the batch-independent masses: the mass kernel over every row of the graph, once per context
        MQG_LAUNCH(ctx, "k_lw_store_i64", s, (k_lw_store_i64<<<1, 64, 0, s>>>(w.counters + 2, n, nullptr)));
        const int grid = static_cast<int>(std::min<int64_t>(std::max<int64_t>(1, ceil_div(n * kRowChunks, kWavesPerBlock)), 256 * 64));
        MQG_LAUNCH(ctx, "k_lw_mass", s,
                   (k_lw_mass<PtrT, IdxT><<<grid, kBlock, 0, s>>>(row_ptr, col_idx, nullptr, w.counters + 2, w.fg_mass, nullptr, nullptr)));
        w.fg_ready = true;
    }

    IdxT *dst0 = reinterpret_cast<IdxT *>(w.seeds_copy);
    {
        const int grid = static_cast<int>(std::max<int64_t>(1, ceil_div(num_seeds, kBlock)));
        MQG_LAUNCH(ctx, "k_lw_seeds", s,
                   (k_lw_seeds<IdxT><<<grid, kBlock, 0, s>>>(static_cast<const IdxT *>(seeds_v), num_seeds, n, dst0,
                                                             blocks[L - 1].sizes, w.flags, w.sel_hist, kSelHistLen)));
    }
    for (int l = L - 1; l >= 0; --l) {
        mqg_block &b = blocks[l];
        const IdxT *dst = l == L - 1 ? dst0 : static_cast<const IdxT *>(blocks[l + 1].src_ids);
        IdxT *src_ids = static_cast<IdxT *>(b.src_ids);
        const int64_t rows_cap = l == L - 1 ? num_seeds : std::min<int64_t>(n, layer_sizes[l + 1]);
        const uint64_t tag_hash = host_mix64(seed_hash ^ static_cast<uint64_t>(int64_t(kLayerwiseTag + l)));

        int rc = MQG_OK;
        if (!fastgcn) {
            const int mass_grid = static_cast<int>(std::min<int64_t>(std::max<int64_t>(1, ceil_div(rows_cap * kRowChunks, kWavesPerBlock)), 256 * 64));
            // list of candidates: marked slot by slot in the node bitmap, or, on graphs of up to
            // kMassScanNodes nodes, read off the masses afterwards
            const bool scan_masses = how == 0 ? n <= kMassScanNodes : how == 2;
            MQG_LAUNCH(ctx, "k_lw_mass", s,
                       (k_lw_mass<PtrT, IdxT><<<mass_grid, kBlock, 0, s>>>(row_ptr, col_idx, dst, b.sizes, w.mass,
                                                                           dense || scan_masses ? nullptr : ctx->bitmap,
                                                                           dense ? w.counters : nullptr)));
            if (!dense) {
                if (scan_masses)
                    MQG_LAUNCH(ctx, "k_lw_mass_bits", s, (k_lw_mass_bits<<<tiles, kBlock, 0, s>>>(w.mass, n, ctx->bitmap, w.word_offs)));
                else
                    rc = count_tiles();
                if (rc == MQG_OK) rc = emit_list(w.cand, nullptr, n_cand, nullptr);
                if (rc != MQG_OK) return rc;
            }
        }
        // race keys and the first digit's counts, then the other digits, then the drawn nodes
        // (few workgroups: the keys' leading digits take a handful of values, and every workgroup adds its
        // counts to the same few words - 911 workgroups spent 9 us of 15 queueing there)
        const int key_grid = static_cast<int>(std::min<int64_t>(cand_grid, n <= (int64_t(1) << 22) ? 256 : 2048));
        MQG_LAUNCH(ctx, "k_lw_keys", s,
                   (k_lw_keys<PtrT><<<key_grid, kBlock, 0, s>>>(row_ptr, cand, n_keys_dev, n, mass, tag_hash, flat, w.key64, w.q_part, w.sel_hist,
                                                                dense ? w.counters : nullptr, w.sel_state, layer_sizes[l], bcount)));
        const int sel_grid = static_cast<int>(std::min<int64_t>(cand_grid, 1024));
        for (int pass = 1; pass < kSelPasses; ++pass)
            MQG_LAUNCH(ctx, "k_lw_select", s,
                       (k_lw_select<<<sel_grid, kBlock, 0, s>>>(w.key64, n_keys_dev, n, layer_sizes[l], w.sel_state, w.sel_hist, pass)));
        MQG_LAUNCH(ctx, "k_lw_mark", s,
                   (k_lw_mark<<<sel_grid, kBlock, 0, s>>>(cand, w.key64, n_keys_dev, n, n_cand, dense ? 1 : 0, layer_sizes[l], w.sel_state,
                                                          w.sel_hist, ctx->bitmap, w.q_part, key_grid, w.q_total, w.bkey, w.bpos, bcount)));
        MQG_LAUNCH(ctx, "k_lw_finish", s,
                   (k_lw_finish<<<1, kBlock, 0, s>>>(cand, n_keys_dev, n, n_cand, layer_sizes[l], w.sel_state, w.bkey, w.bpos, bcount,
                                                     ctx->bitmap)));
        rc = count_tiles();
        if (rc == MQG_OK) rc = emit_list(src_ids, ctx->local_of, &b.sizes[1], l > 0 ? &blocks[l - 1].sizes[0] : nullptr);
        if (rc != MQG_OK) return rc;
        const double *beta = nullptr;
        if (debias) {
            const int64_t src_cap = std::min<int64_t>(n, layer_sizes[l]);
            const int sgrid = static_cast<int>(std::max<int64_t>(1, ceil_div(src_cap, kBlock)));
            MQG_LAUNCH(ctx, "k_lw_drawn_keys", s,
                       (k_lw_drawn_keys<PtrT, IdxT><<<sgrid, kBlock, 0, s>>>(row_ptr, src_ids, b.sizes, mass, tag_hash, flat, w.dkey, w.dq)));
            MQG_LAUNCH(ctx, "k_lw_draw_order", s, (k_lw_draw_order<<<sgrid, kBlock, 0, s>>>(w.dkey, b.sizes, w.order)));
            MQG_LAUNCH(ctx, "k_lw_debias", s,
                       (k_lw_debias<<<1, kBlock, 0, s>>>(w.order, w.dq, w.q_total, b.sizes, n_cand, w.chunk_sum, w.beta)));
            beta = w.beta;
        }
        // rows: per (row, chunk) counts and weight sums, one scan, then the edges
        const int64_t chunks_cap = rows_cap * kRowChunks;
        const int chunk_grid = static_cast<int>(std::min<int64_t>(std::max<int64_t>(1, ceil_div(chunks_cap, kWavesPerBlock)), 256 * 64));
        // (entries of chunk_offs past the block's rows are not cleared: an exclusive scan's values up to
        // the last row's end, the only ones read, do not depend on them)
        MQG_LAUNCH(ctx, "k_lw_count", s,
                   (k_lw_count<PtrT, IdxT><<<chunk_grid, kBlock, 0, s>>>(row_ptr, col_idx, dst, b.sizes, ctx->local_of, mass, w.q_total,
                                                                         beta, flat, w.chunk_offs, w.chunk_sum)));
        // one launch when the table is small (the scan goes to a second array), else in place
        const int32_t *offs = w.chunk_offs;
        if (chunks_cap + 1 <= int64_t(kScanSelfTiles) * kScanTile) {
            rc = device_scan_copy(ctx, w.chunk_offs, w.chunk_scan, chunks_cap + 1, s);
            offs = w.chunk_scan;
        } else {
            rc = device_scan(ctx, w.chunk_offs, chunks_cap + 1, w.scan_tiles, s);
        }
        if (rc != MQG_OK) return rc;
        MQG_LAUNCH(ctx, "k_lw_fill", s,
                   (k_lw_fill<PtrT, IdxT><<<chunk_grid, kBlock, 0, s>>>(row_ptr, col_idx, dst, b.sizes, ctx->local_of, mass, w.q_total,
                                                                        beta, flat, offs, w.chunk_sum, b.indptr, b.indices, edge_w[l],
                                                                        normalise, b.cap_nnz, l == L - 1 ? w.flags : nullptr)));
        const int reset_grid = static_cast<int>(std::min<int64_t>(cand_grid, 4096));
        MQG_LAUNCH(ctx, "k_lw_reset", s,
                   (k_lw_reset<IdxT><<<reset_grid, kBlock, 0, s>>>(cand, n_cand, dense ? n : 0, w.mass, src_ids, b.sizes, ctx->local_of,
                                                                   l == L - 1 ? w.flags : nullptr, w.sel_hist, kSelHistLen)));
    }
    return MQG_OK;
}

// the selection step on its own: bit c of out_bitmap = key c is among the k smallest (key, index) pairs
int run_select_smallest_keys(mqg_ctx *ctx, const uint64_t *keys, int64_t n, int64_t k, uint32_t *out_bitmap, hipStream_t s) {
    int rc = ensure_layerwise_scratch(ctx, 1, s);
    if (rc != MQG_OK) return rc;
    LayerwiseScratch &w = ctx->lw;
    // the boundary list may hold every key: the sampler's own list has room for one per graph node
    uint64_t *bkey = w.bkey;
    int32_t *bpos = w.bpos;
    if (n > std::max<int64_t>(ctx->num_nodes, 1)) {
        if (n > w.xcap) {
            hipError_t e = hipStreamSynchronize(s);
            if (e != hipSuccess) return fail(ctx, MQG_ERR_HIP, std::string("mqg_select_smallest_keys: ") + hipGetErrorString(e));
            (void)hipFree(w.xkey);
            (void)hipFree(w.xpos);
            w.xkey = nullptr;
            w.xpos = nullptr;
            w.xcap = 0;
            if (!dev_alloc(&w.xkey, n) || !dev_alloc(&w.xpos, n)) {
                (void)hipFree(w.xkey);
                w.xkey = nullptr;
                return fail(ctx, MQG_ERR_HIP, "mqg_select_smallest_keys: scratch allocation failed");
            }
            w.xcap = n;
        }
        bkey = w.xkey;
        bpos = w.xpos;
    }
    int64_t *n_dev = w.counters + 1;
    const int64_t words = ceil_div(n, 32);
    MQG_LAUNCH(ctx, "k_lw_store_i64", s, (k_lw_store_i64<<<1, 64, 0, s>>>(n_dev, n, w.counters + 3)));
    if (words > 0)
        MQG_LAUNCH(ctx, "k_lw_zero_i32", s,
                   (k_lw_zero_i32<<<static_cast<int>(ceil_div(words, kBlock)), kBlock, 0, s>>>(reinterpret_cast<int32_t *>(out_bitmap), words)));
    MQG_LAUNCH(ctx, "k_lw_zero_i32", s, (k_lw_zero_i32<<<kSelHistLen / kBlock, kBlock, 0, s>>>(w.sel_hist, kSelHistLen)));
    const int grid = static_cast<int>(std::min<int64_t>(std::max<int64_t>(1, ceil_div(n, kBlock)), 1024));
    for (int pass = 0; pass < kSelPasses; ++pass)
        MQG_LAUNCH(ctx, "k_lw_select", s, (k_lw_select<<<grid, kBlock, 0, s>>>(keys, n_dev, 0, k, w.sel_state, w.sel_hist, pass)));
    unsigned long long *bcount = reinterpret_cast<unsigned long long *>(w.counters + 3);
    MQG_LAUNCH(ctx, "k_lw_mark", s,
               (k_lw_mark<<<grid, kBlock, 0, s>>>(nullptr, keys, n_dev, 0, nullptr, 0, k, w.sel_state, w.sel_hist, out_bitmap, nullptr, 0, nullptr,
                                                  bkey, bpos, bcount)));
    MQG_LAUNCH(ctx, "k_lw_finish", s,
               (k_lw_finish<<<1, kBlock, 0, s>>>(nullptr, n_dev, 0, nullptr, k, w.sel_state, bkey, bpos, bcount, out_bitmap)));
    return MQG_OK;
}

int run_sample_layerwise(mqg_ctx *ctx, const mqg_graph *g, const void *seeds, int32_t num_seeds, const int32_t *layer_sizes,
                         int32_t L, uint64_t rng_seed, int32_t normalise, int32_t method, mqg_block *blocks, float *const *edge_w,
                         hipStream_t s) {
    const bool fg = (method & MQG_LAYERWISE_FASTGCN) != 0;
    const bool db = (method & MQG_LAYERWISE_DEBIAS) != 0;
    const bool fl = (method & MQG_LAYERWISE_FLAT) != 0;
    int64_t rows_cap = num_seeds;
    for (int l = 0; l < L; ++l) rows_cap = std::max<int64_t>(rows_cap, std::min<int64_t>(ctx->num_nodes, layer_sizes[l]));
    int rc = ensure_layerwise_scratch(ctx, rows_cap, s);
    if (rc != MQG_OK) return rc;
    if (fg && !ctx->lw.fg_mass) {
        const int64_t n = std::max<int64_t>(ctx->num_nodes, 1);
        if (!dev_alloc(&ctx->lw.fg_mass, n) ||
            hipMemsetAsync(ctx->lw.fg_mass, 0, static_cast<size_t>(n) * sizeof(unsigned long long), s) != hipSuccess) {
            (void)hipFree(ctx->lw.fg_mass);
            ctx->lw.fg_mass = nullptr;
            return fail(ctx, MQG_ERR_HIP, "mqg_sample_layerwise: scratch allocation failed");
        }
        ctx->lw.fg_ready = false;
    }
    const bool p64 = g->ptr_type == MQG_I64, i64 = g->idx_type == MQG_I64;
    if (p64 && i64) return sample_layerwise_impl<int64_t, int64_t>(ctx, g, seeds, num_seeds, layer_sizes, L, rng_seed, normalise, fg, db, fl, blocks, edge_w, s);
    if (p64) return sample_layerwise_impl<int64_t, int32_t>(ctx, g, seeds, num_seeds, layer_sizes, L, rng_seed, normalise, fg, db, fl, blocks, edge_w, s);
    if (i64) return sample_layerwise_impl<int32_t, int64_t>(ctx, g, seeds, num_seeds, layer_sizes, L, rng_seed, normalise, fg, db, fl, blocks, edge_w, s);
    return sample_layerwise_impl<int32_t, int32_t>(ctx, g, seeds, num_seeds, layer_sizes, L, rng_seed, normalise, fg, db, fl, blocks, edge_w, s);
}

}  // namespace mqg
