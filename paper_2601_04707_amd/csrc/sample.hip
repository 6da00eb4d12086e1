// L-hop fixed-fanout neighbour sampling into bipartite blocks (paper Sec. III-A, GraphSAGE
// paragraph; block layout after Sec. IV "Mini-Batch Transfer To GPU" and Eq. 16).
//
// Per block, outward from the seeds (five launches; the first block's row information is a launch
// of its own, every other block's rides with the block before it):
//   row info       adjacency start/degree of every destination, copy of the destinations into the
//                  block's source list, per-tile sums of min(fanout, degree), list of the hubs
//   k_sample       one wavefront per destination: smallest-k random keys, neighbours written in
//                  ascending adjacency slot at row * fanout (no offsets needed yet), first-seen
//                  nodes marked in an N-bit bitmap (destinations whose degree exceeds heavy_degree
//                  are taken by whole workgroups in the same launch, so that a hub's key
//                  evaluation is spread over four wavefronts instead of stretching the kernel's tail)
//   k_offsets_count  two independent jobs in one launch: indptr from the row tile sums (every
//                  workgroup adds up the sums of the tiles before its own; only above 8,192 tiles
//                  does one k_scan_tiles launch scan them first) and the popcount of every tile
//                  of the bitmap
//   k_bitmap_emit  popcount-rank the bitmap: new source nodes come out ascending by id, get their
//                  position recorded in local_of[], the bitmap is cleared on the way
//   k_emit_offsets  graphs of up to half a million nodes: the two launches above in one - every
//                  tile's workgroup counts the bits of the tiles before its own itself (the relabel
//                  launch clears the bitmap then)
//   k_relabel_rowinfo  indices[indptr[row] + j] = local_of[neighbour j of row], and in the same
//                  launch the row information of the next block outward (whose destinations are
//                  this block's sources); the outermost block ends with a plain k_relabel
// The hash-table dedup (an option) keeps the older order: offsets first, neighbours written compactly.
// All sizes that depend on the data stay on the device; grids are sized by worst-case bounds.
#include "common.h"
#include "device_utils.h"

namespace mqg {

namespace {

constexpr uint64_t kGolden = 0x9E3779B97F4A7C15ULL;
constexpr uint64_t kMaxKey = ~uint64_t(0);

uint64_t host_mix64(uint64_t z) {
    z ^= z >> 30;
    z *= 0xBF58476D1CE4E5B9ULL;
    z ^= z >> 27;
    z *= 0x94D049BB133111EBULL;
    z ^= z >> 31;
    return z;
}

// ------------------------------------------------------------------------------------------

// Arguments of the row-information step of one block.
template <typename PtrT, typename IdxT>
struct RowInfoArgs {
    const PtrT *row_ptr;
    const IdxT *dst;             // the block's destinations (the caller's seeds, or the previous block's sources)
    const int64_t *sizes;        // this block's sizes: [0] = number of destinations (unless n_seeds >= 0)
    IdxT *src_out;
    int fanout;
    int64_t *row_start;
    int32_t *row_deg;
    int32_t *tile_sums;
    int64_t *sizes_rw;
    int heavy_degree;
    int32_t *heavy_rows;
    int32_t *heavy_count;
    int64_t n_seeds;             // >= 0: innermost block
    int32_t *local_of;
    int64_t num_nodes;
    int32_t *seed_flags;
};

template <typename PtrT, typename IdxT>
__device__ __forceinline__ void row_info_tile(const RowInfoArgs<PtrT, IdxT> &a, int tile, int *lds) {
    // innermost block (n_seeds >= 0): the destinations are the caller's seeds; their number comes
    // from the host and their positions are entered into local_of here
    const int64_t n = a.n_seeds >= 0 ? a.n_seeds : a.sizes[0];
    const int64_t i = int64_t(tile) * kBlock + threadIdx.x;
    int cnt = 0;
    bool heavy = false;
    if (i < n) {
        IdxT v = a.dst[i];
        if (a.n_seeds >= 0) {
            // caller-supplied ids: an id outside the graph is flagged and replaced by node 0, so that
            // nothing downstream ever indexes with it; a repeated id is flagged (its rows are kept and
            // share one position in the source lists)
            if (v < 0 || static_cast<int64_t>(v) >= a.num_nodes) {
                v = 0;
                atomicOr(a.seed_flags, 1);
            }
            if (a.local_of && atomicCAS(&a.local_of[v], -1, static_cast<int32_t>(i)) != -1) atomicOr(a.seed_flags, 2);
        }
        int64_t s = static_cast<int64_t>(a.row_ptr[v]);
        int64_t d = static_cast<int64_t>(a.row_ptr[v + 1]) - s;
        a.row_start[i] = s;
        a.row_deg[i] = static_cast<int32_t>(d);
        a.src_out[i] = v;
        cnt = d < a.fanout ? static_cast<int>(d) : a.fanout;
        heavy = d > a.heavy_degree;
    }
    {   // list the hubs: one atomic per wavefront that has any
        uint64_t m = ballot64(heavy);
        if (m) {
            int base = 0;
            if (lane_id() == 0) base = atomicAdd(a.heavy_count, popc64(m));
            base = __shfl(base, 0, 64);
            if (heavy) a.heavy_rows[base + popc64(m & lanes_below(lane_id()))] = static_cast<int32_t>(i);
        }
    }
    int w = wave_sum(cnt);
    if (lane_id() == 0) lds[threadIdx.x >> 6] = w;
    __syncthreads();
    if (threadIdx.x == 0) {
        int t = 0;
#pragma unroll
        for (int k = 0; k < kWavesPerBlock; ++k) t += lds[k];
        a.tile_sums[tile] = t;
        if (tile == 0 && a.n_seeds >= 0) a.sizes_rw[0] = a.n_seeds;
    }
}

template <typename PtrT, typename IdxT>
__global__ void __launch_bounds__(kBlock)
k_row_info(RowInfoArgs<PtrT, IdxT> a) {
    __shared__ int lds[kWavesPerBlock];
    row_info_tile(a, static_cast<int>(blockIdx.x), lds);
}

// One workgroup of 1024 threads: vals[0..n) -> exclusive scan in place; totals stored.
__global__ void __launch_bounds__(1024)
k_scan_tiles(int32_t *__restrict__ vals, int64_t n, const int64_t *__restrict__ addend,
             int64_t *__restrict__ total_a, int64_t *__restrict__ total_b) {
    __shared__ int lds[16];
    int64_t carry = 0;
    for (int64_t base = 0; base < n; base += 1024) {
        int64_t i = base + threadIdx.x;
        int v = i < n ? vals[i] : 0;
        int total;
        int ex = block_excl_scan<16>(v, &total, lds);
        if (i < n) vals[i] = static_cast<int32_t>(carry + ex);
        carry += total;
    }
    if (threadIdx.x == 0) {
        int64_t t = carry + (addend ? *addend : 0);
        if (total_a) *total_a = t;
        if (total_b) *total_b = t;
    }
}

// scanned: tile_vals holds the exclusive scan of the tile sums (k_scan_tiles ran, and stored nnz);
// otherwise it holds the sums themselves, every workgroup adds up its own base and the last one
// stores nnz.
__device__ __forceinline__ void row_offsets_tile(const int32_t *__restrict__ row_deg, int fanout, int64_t *sizes,
                                                 const int32_t *__restrict__ tile_vals, int scanned,
                                                 int32_t *__restrict__ indptr, const int32_t *__restrict__ seed_flags,
                                                 int tile, int ntiles, int *lds) {
    const int64_t n = sizes[0];
    // the block's flags word: what the seed check found (innermost block), 0 otherwise
    if (tile == 0 && threadIdx.x == 0) sizes[3] = seed_flags ? *seed_flags : 0;
    const int tile_base = scanned ? tile_vals[tile] : tiles_before(tile_vals, lds, tile);
    const int64_t i = int64_t(tile) * kBlock + threadIdx.x;
    int cnt = 0;
    if (i < n) {
        int d = row_deg[i];
        cnt = d < fanout ? d : fanout;
    }
    int total;
    int ex = block_excl_scan<kWavesPerBlock>(cnt, &total, lds);
    int off = tile_base + ex;
    if (i < n) {
        indptr[i] = off;
        if (i == n - 1) indptr[n] = off + cnt;
    }
    if (n == 0 && i == 0) indptr[0] = 0;
    if (!scanned && tile == ntiles - 1 && threadIdx.x == 0) sizes[2] = tile_base + total;
}

__global__ void __launch_bounds__(kBlock)
k_row_offsets(const int32_t *__restrict__ row_deg, int fanout, int64_t *sizes,
              const int32_t *__restrict__ tile_vals, int scanned, int32_t *__restrict__ indptr,
              const int32_t *__restrict__ seed_flags) {
    __shared__ int lds[kWavesPerBlock];
    row_offsets_tile(row_deg, fanout, sizes, tile_vals, scanned, indptr, seed_flags, static_cast<int>(blockIdx.x),
                     static_cast<int>(gridDim.x), lds);
}

// ------------------------------------------------------------------------------------------
// Neighbour selection.  One wavefront owns one destination node.

struct SampleArgs {
    const int64_t *row_start;
    const int32_t *row_deg;
    const int32_t *indptr;    // null: row r's neighbours go to nbr[r * fanout ...) and are compacted by the relabel
    const int64_t *sizes;
    int32_t *nbr;
    const int32_t *local_of;
    uint32_t *bitmap;
    uint64_t layer_hash;      // mix(mix(rng_seed + golden) ^ block index), used when seed_dev is null
    const uint64_t *seed_dev; // the sampling seed in device memory (calls recorded into a HIP graph)
    int layer;                // block index, for seed_dev
    int fanout;
    int force_slow;
    int heavy_degree;         // rows longer than this are sampled by whole workgroups
};

__device__ __forceinline__ int32_t out_base_of(const SampleArgs &a, int64_t row) {
    return a.indptr ? a.indptr[row] : static_cast<int32_t>(row * a.fanout);
}

__device__ __forceinline__ uint64_t layer_hash_of(const SampleArgs &a) {
    if (!a.seed_dev) return a.layer_hash;
    return mix64(mix64(*a.seed_dev + 0x9E3779B97F4A7C15ULL) ^ static_cast<uint64_t>(a.layer));
}

template <typename IdxT>
__device__ __forceinline__ void emit_neighbour(const IdxT *__restrict__ col_idx, int64_t start, int slot,
                                               int32_t out_pos, const SampleArgs &a) {
    int32_t u = static_cast<int32_t>(col_idx[start + slot]);
    a.nbr[out_pos] = u;
    if (a.local_of && a.local_of[u] < 0) {                 // (no marking when the hash path dedups)
        uint32_t bit = 1u << (u & 31);
        uint32_t *w = a.bitmap + (u >> 5);
        (void)__hip_atomic_fetch_or(w, bit, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// key(j) = mix64(hv ^ j) for the slots j of one row, with everything that depends only on the row
// hoisted out: j < 2^31 touches only the low word of hv ^ j, so the high word after the first
// xor-shift and its share of the first multiply are per-row constants.  Written on 32-bit halves
// (funnel shifts are one v_alignbit each): 5 multiplies per key instead of 6.
struct RowKeys {
    static constexpr uint32_t kC1Lo = 0x1CE4E5B9u, kC1Hi = 0xBF58476Du;
    static constexpr uint32_t kC2Lo = 0x133111EBu, kC2Hi = 0x94D049BBu;
    uint32_t lo, hi_shl2, a_hi, c1_term;
    __device__ __forceinline__ explicit RowKeys(uint64_t hv) {
        const uint32_t hi = static_cast<uint32_t>(hv >> 32);
        lo = static_cast<uint32_t>(hv);
        hi_shl2 = hi << 2;
        a_hi = hi ^ (hi >> 30);
        c1_term = a_hi * kC1Lo;
    }
    __device__ __forceinline__ uint64_t operator()(int j) const {
        const uint32_t lo0 = lo ^ static_cast<uint32_t>(j);
        const uint32_t a_lo = lo0 ^ (hi_shl2 | (lo0 >> 30));                       // z ^= z >> 30
        const uint64_t p = static_cast<uint64_t>(a_lo) * kC1Lo;                      // z *= C1
        const uint32_t b_lo = static_cast<uint32_t>(p);
        const uint32_t b_hi = static_cast<uint32_t>(p >> 32) + a_lo * kC1Hi + c1_term;
        const uint32_t c_lo = b_lo ^ __builtin_amdgcn_alignbit(b_hi, b_lo, 27);      // z ^= z >> 27
        const uint32_t c_hi = b_hi ^ (b_hi >> 27);
        const uint64_t q = static_cast<uint64_t>(c_lo) * kC2Lo;                      // z *= C2
        const uint32_t d_lo = static_cast<uint32_t>(q);
        const uint32_t d_hi = static_cast<uint32_t>(q >> 32) + c_lo * kC2Hi + c_hi * kC2Lo;
        const uint32_t e_lo = d_lo ^ __builtin_amdgcn_alignbit(d_hi, d_lo, 31);      // z ^= z >> 31
        const uint32_t e_hi = d_hi ^ (d_hi >> 31);
        return (static_cast<uint64_t>(e_hi) << 32) | e_lo;
    }
};

// lexicographic (key, slot) order
__device__ __forceinline__ bool pair_less(uint64_t ka, int sa, uint64_t kb, int sb) {
    return ka < kb || (ka == kb && sa < sb);
}

// Candidates 0..cnt of a row in LDS (key, slot; bit 31 of the slot word = comes after every
// unmarked candidate, PRIO only).  Picks the k first in the sampling order and returns, per chunk
// of 64 candidates, the chosen lanes; slot[] gets each lane's slot words.  ORDERED: the candidates
// are stored in ascending slot order, so equal keys need no second key.
template <int NCH, bool PRIO, bool ORDERED, typename SlotT>
__device__ __forceinline__ void select_candidates(const uint64_t *ck, const SlotT *cs, int cnt, int k,
                                                  uint32_t (&slot)[NCH], uint64_t (&sel)[NCH]) {
    const int lane = lane_id();
    uint64_t key[NCH], late[NCH], cand[NCH];
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        const int ci = c * kWave + lane;
        const bool valid = ci < cnt;
        key[c] = valid ? ck[ci] : 0;
        slot[c] = valid ? static_cast<uint32_t>(cs[ci]) : 0u;
        const int left = cnt - c * kWave;
        cand[c] = left <= 0 ? 0 : low_lanes(left);
        late[c] = PRIO ? ballot64((slot[c] >> 31) != 0) : 0;
    }
    uint32_t tie[NCH];
#pragma unroll
    for (int c = 0; c < NCH; ++c) tie[c] = slot[c] & 0x7FFFFFFFu;
    wave_select_smallest<NCH, PRIO, !ORDERED>(key, late, tie, cand, k, sel);
}

// The same for candidates in ascending slot order, emitted as the row's neighbours.
template <int NCH, bool PRIO, typename IdxT, typename SlotT>
__device__ __forceinline__ void emit_selected(const uint64_t *ck, const SlotT *cs, int cnt, int k,
                                              const IdxT *__restrict__ col_idx, int64_t start, int32_t out_base,
                                              const SampleArgs &a) {
    const int lane = lane_id();
    uint32_t slot[NCH];
    uint64_t sel[NCH];
    select_candidates<NCH, PRIO, true>(ck, cs, cnt, k, slot, sel);
    int out_pos = out_base;
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        if ((sel[c] >> lane) & 1)
            emit_neighbour(col_idx, start, static_cast<int>(slot[c] & 0x7FFFFFFFu),
                           out_pos + popc64(sel[c] & lanes_below(lane)), a);
        out_pos += popc64(sel[c]);
    }
}
template <bool PRIO, typename IdxT, typename SlotT>
__device__ __forceinline__ void emit_selected_any(const uint64_t *ck, const SlotT *cs, int cnt, int k,
                                                  const IdxT *__restrict__ col_idx, int64_t start, int32_t out_base,
                                                  const SampleArgs &a) {
    if (cnt <= kWave) emit_selected<1, PRIO>(ck, cs, cnt, k, col_idx, start, out_base, a);
    else if (cnt <= 2 * kWave) emit_selected<2, PRIO>(ck, cs, cnt, k, col_idx, start, out_base, a);
    else emit_selected<kCandidates / kWave, PRIO>(ck, cs, cnt, k, col_idx, start, out_base, a);
}

// Hub rows: the candidates sit in LDS in arrival order.  The first wavefront picks the k winners,
// lists their slots in sel_slot and emits them in ascending slot order.
template <bool PRIO, typename IdxT, typename SlotT>
__device__ __forceinline__ void emit_selected_unordered(const uint64_t *ck, const SlotT *cs, int cnt, int k,
                                                        int32_t *sel_slot, const IdxT *__restrict__ col_idx,
                                                        int64_t start, int32_t out_base, const SampleArgs &a) {
    constexpr int NCH = kCandidates / kWave;
    const int lane = lane_id();
    uint32_t slot[NCH];
    uint64_t sel[NCH];
    select_candidates<NCH, PRIO, false>(ck, cs, cnt, k, slot, sel);
    int pos = 0;
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        if ((sel[c] >> lane) & 1) sel_slot[pos + popc64(sel[c] & lanes_below(lane))] = static_cast<int32_t>(slot[c] & 0x7FFFFFFFu);
        pos += popc64(sel[c]);
    }
    wave_lds_sync();
    const int my_slot = lane < k ? sel_slot[lane] : 0x7FFFFFFF;
    int rank = 0;
    for (int t = 0; t < k; ++t) {
        int other = static_cast<int>(readlane32(static_cast<uint32_t>(my_slot), t));
        rank += (other < my_slot) ? 1 : 0;
    }
    if (lane < k) emit_neighbour(col_idx, start, my_slot, out_base + rank, a);
}

// The per-row selection on caller-supplied candidates (mqg_select_row_candidates): one wavefront,
// the same code path as k_sample / k_sample_prio after their threshold pass.
template <bool PRIO, bool ORDERED>
__global__ void __launch_bounds__(kWave)
k_select_candidates(const uint64_t *__restrict__ keys, const uint32_t *__restrict__ slot_words, int cnt, int k,
                    uint32_t *__restrict__ out_mask) {
    constexpr int NCH = kCandidates / kWave;
    uint32_t slot[NCH];
    uint64_t sel[NCH];
    select_candidates<NCH, PRIO, ORDERED>(keys, slot_words, cnt, k, slot, sel);
    if (lane_id() == 0) {
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            out_mask[2 * c] = static_cast<uint32_t>(sel[c]);
            out_mask[2 * c + 1] = static_cast<uint32_t>(sel[c] >> 32);
        }
    }
}

// Unconditional selection: k rounds, each finding the smallest (key, slot) pair above the
// previous round's.  O(k*d/64) key evaluations; used when the threshold pass cannot be
// trusted (fewer than k or more than kCandidates keys under the threshold) and in tests.
template <typename IdxT>
__device__ void select_by_repeated_min(const IdxT *__restrict__ col_idx, int64_t start, int d, int k,
                                       uint64_t hv, int32_t out_base, const SampleArgs &a) {
    const int lane = lane_id();
    const RowKeys key_of(hv);
    uint64_t prev_key = 0;
    int prev_slot = -1;
    int my_slot = -1;                                // lane r keeps the r-th selected slot
    for (int r = 0; r < k; ++r) {
        uint64_t best_key = kMaxKey;
        int best_slot = 0x7FFFFFFF;
        for (int base = 0; base < d; base += kWave) {
            int j = base + lane;
            if (j < d) {
                uint64_t key = key_of(j);
                bool above = (r == 0) || pair_less(prev_key, prev_slot, key, j);
                if (above && pair_less(key, j, best_key, best_slot)) {
                    best_key = key;
                    best_slot = j;
                }
            }
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            uint64_t ok = __shfl_xor(best_key, off, 64);
            int os = __shfl_xor(best_slot, off, 64);
            if (pair_less(ok, os, best_key, best_slot)) {
                best_key = ok;
                best_slot = os;
            }
        }
        prev_key = best_key;
        prev_slot = best_slot;
        if (lane == r) my_slot = best_slot;
    }
    // order the k chosen slots ascending
    int rank = 0;
    for (int t = 0; t < k; ++t) {
        int other = static_cast<int>(readlane32(static_cast<uint32_t>(my_slot), t));
        rank += (other < my_slot) ? 1 : 0;
    }
    if (lane < k) emit_neighbour(col_idx, start, my_slot, out_base + rank, a);
}

// Hubs (degree > heavy_degree, listed by k_row_info): the four wavefronts of a workgroup share
// one row.  Candidates under the threshold are appended to one LDS list in arrival order (an LDS
// atomic per wavefront and chunk); the result does not depend on that order because the
// k winners are selected by (key, slot) and then ordered by slot.
template <typename IdxT>
__device__ void sample_hubs(const IdxT *__restrict__ col_idx, const IdxT *__restrict__ dst_ids, const SampleArgs &a,
                            const int32_t *__restrict__ heavy_rows, int nheavy, int first, int step,
                            uint64_t *ck, int32_t *cs, int32_t *sel_slot, int *cnt_s) {
    const int tid = threadIdx.x;
    const int lane = lane_id();
    const int wave = tid >> 6;
    const int k = a.fanout;
    for (int h = first; h < nheavy; h += step) {
        const int row = heavy_rows[h];
        const int64_t start = a.row_start[row];
        const int d = a.row_deg[row];
        const int32_t out_base = out_base_of(a, row);
        const uint64_t hv = mix64(layer_hash_of(a) ^ uint64_t(dst_ids[row]));
        const RowKeys key_of(hv);
        if (tid == 0) *cnt_s = 0;
        __syncthreads();
        const int expect = 2 * k + 32;
        uint64_t thr = kMaxKey;
        if (d > expect) thr = static_cast<uint64_t>((double(expect) / double(d)) * 18446744073709551616.0);
        for (int base = wave * kWave; base < d; base += kBlock) {
            int j = base + lane;
            uint64_t key = key_of(j);
            bool c = j < d && key <= thr;
            uint64_t m = ballot64(c);
            if (m) {
                int p0 = 0;
                if (lane == 0) p0 = atomicAdd(cnt_s, popc64(m));
                p0 = __shfl(p0, 0, 64);
                if (c) {
                    int p = p0 + popc64(m & lanes_below(lane));
                    if (p < kCandidates) {
                        ck[p] = key;
                        cs[p] = j;
                    }
                }
            }
        }
        __syncthreads();
        const int cnt = *cnt_s;
        if (cnt < k || cnt > kCandidates) {                // workgroup-uniform; practically never
            if (wave == 0) select_by_repeated_min(col_idx, start, d, k, hv, out_base, a);
            __syncthreads();
            continue;
        }
        if (wave == 0) emit_selected_unordered<false>(ck, cs, cnt, k, sel_slot, col_idx, start, out_base, a);
        __syncthreads();                                   // LDS is reused by the next row
    }
}

static_assert(kCandidates % kWave == 0, "candidates are selected in chunks of one per lane");

// The first hub_blocks workgroups take the hubs (they are dispatched first and run the longest);
// every other workgroup gives each of its four wavefronts one destination.
template <typename IdxT>
__global__ void __launch_bounds__(kBlock)
k_sample(const IdxT *__restrict__ col_idx, const IdxT *__restrict__ dst_ids, SampleArgs a,
         const int32_t *__restrict__ heavy_rows, const int32_t *__restrict__ heavy_count, int hub_blocks) {
    __shared__ uint64_t cand_key[kWavesPerBlock][kCandidates];
    __shared__ int32_t cand_slot[kWavesPerBlock][kCandidates];
    __shared__ int32_t sel_slot[kWave];
    __shared__ int cnt_s;
    if (static_cast<int>(blockIdx.x) < hub_blocks) {
        sample_hubs(col_idx, dst_ids, a, heavy_rows, *heavy_count, static_cast<int>(blockIdx.x), hub_blocks,
                    cand_key[0], cand_slot[0], sel_slot, &cnt_s);
        return;
    }
    const int lane = lane_id();
    const int wave = static_cast<int>(threadIdx.x) >> 6;
    const int64_t n = a.sizes[0];
    const int64_t row = (int64_t(blockIdx.x) - hub_blocks) * kWavesPerBlock + wave;
    if (row >= n) return;                                  // whole wavefront leaves together

    const int64_t start = a.row_start[row];
    const int d = a.row_deg[row];
    const int k = a.fanout;
    const int32_t out_base = out_base_of(a, row);

    if (d <= k) {                                          // the whole row, no randomness
        if (lane < d) emit_neighbour(col_idx, start, lane, out_base + lane, a);
        return;
    }
    if (d > a.heavy_degree) return;                        // a hub: sampled by the first workgroups
    const uint64_t hv = mix64(layer_hash_of(a) ^ uint64_t(dst_ids[row]));
    if (a.force_slow) {
        select_by_repeated_min(col_idx, start, d, k, hv, out_base, a);
        return;
    }
    if (d <= kWave) {
        // one key per lane
        const uint64_t key[1] = {RowKeys(hv)(lane)};
        const uint64_t late[1] = {0};
        const uint32_t tie[1] = {0};
        uint64_t cand[1] = {low_lanes(d)}, sel[1];
        wave_select_smallest<1, false, false>(key, late, tie, cand, k, sel);
        if ((sel[0] >> lane) & 1) emit_neighbour(col_idx, start, lane, out_base + popc64(sel[0] & lanes_below(lane)), a);
        return;
    }

    // d > 64: keep the slots whose key falls under a threshold expected to pass 2k+32 of them,
    // then select among those candidates only.  Candidates are stored in ascending slot order.
    uint64_t *ck = cand_key[wave];
    int32_t *cs = cand_slot[wave];
    const int expect = 2 * k + 32;
    uint64_t thr = kMaxKey;
    if (d > expect) thr = static_cast<uint64_t>((double(expect) / double(d)) * 18446744073709551616.0);
    int cnt = 0;
    const RowKeys key_of(hv);
    for (int base = 0; base < d; base += kWave) {
        int j = base + lane;
        uint64_t key = key_of(j);
        bool c = j < d && key <= thr;
        uint64_t m = ballot64(c);
        if (c) {
            int p = cnt + popc64(m & lanes_below(lane));
            if (p < kCandidates) {
                ck[p] = key;
                cs[p] = j;
            }
        }
        cnt += popc64(m);
    }
    if (cnt < k || cnt > kCandidates) {                    // wavefront-uniform
        select_by_repeated_min(col_idx, start, d, k, hv, out_base, a);
        return;
    }
    wave_lds_sync();
    emit_selected_any<false>(ck, cs, cnt, k, col_idx, start, out_base, a);
}

// ------------------------------------------------------------------------------------------
// Cache-prioritised selection (the paper's Sec. I on global neighbour sampling: neighbours that are
// in the feature cache are preferred, so that fewer distinct uncached rows enter a mini-batch).
// The k slots of a row are the first k in the order (not cached, key, slot): with c cached
// neighbours the row keeps min(k, c) of them, drawn uniformly, and fills up from the uncached ones,
// drawn uniformly.  `prio` is a bitmap over the nodes, bit set = cached.

__device__ __forceinline__ bool prio_less(bool ua, uint64_t ka, int sa, bool ub, uint64_t kb, int sb) {
    return ua != ub ? !ua : pair_less(ka, sa, kb, sb);
}

template <typename IdxT>
__device__ __forceinline__ bool is_cached(const IdxT *__restrict__ row, int j, const uint32_t *__restrict__ prio) {
    const uint32_t u = static_cast<uint32_t>(row[j]);
    return (prio[u >> 5] >> (u & 31)) & 1u;
}

// k rounds of wave-wide minimum extraction in the (not cached, key, slot) order; unconditional.
template <typename IdxT>
__device__ void select_by_repeated_min_prio(const IdxT *__restrict__ col_idx, int64_t start, int d, int k, uint64_t hv,
                                            int32_t out_base, const SampleArgs &a, const uint32_t *__restrict__ prio) {
    const int lane = lane_id();
    const RowKeys key_of(hv);
    const IdxT *row = col_idx + start;
    bool prev_unc = false;
    uint64_t prev_key = 0;
    int prev_slot = -1;
    int my_slot = -1;
    for (int r = 0; r < k; ++r) {
        bool best_unc = true;
        uint64_t best_key = kMaxKey;
        int best_slot = 0x7FFFFFFF;
        for (int base = 0; base < d; base += kWave) {
            int j = base + lane;
            if (j < d) {
                const uint64_t key = key_of(j);
                const bool unc = !is_cached(row, j, prio);
                const bool above = (r == 0) || prio_less(prev_unc, prev_key, prev_slot, unc, key, j);
                if (above && prio_less(unc, key, j, best_unc, best_key, best_slot)) {
                    best_unc = unc;
                    best_key = key;
                    best_slot = j;
                }
            }
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            const uint64_t ok = __shfl_xor(best_key, off, 64);
            const int os = __shfl_xor(best_slot, off, 64);
            const bool ou = __shfl_xor(static_cast<int>(best_unc), off, 64) != 0;
            if (prio_less(ou, ok, os, best_unc, best_key, best_slot)) {
                best_unc = ou;
                best_key = ok;
                best_slot = os;
            }
        }
        prev_unc = best_unc;
        prev_key = best_key;
        prev_slot = best_slot;
        if (lane == r) my_slot = best_slot;
    }
    int rank = 0;
    for (int t = 0; t < k; ++t) {
        int other = static_cast<int>(readlane32(static_cast<uint32_t>(my_slot), t));
        rank += (other < my_slot) ? 1 : 0;
    }
    if (lane < k) emit_neighbour(col_idx, start, my_slot, out_base + rank, a);
}

// Candidate test shared by both shapes of the prioritised kernel: which pool competes and under
// which key threshold (about 2k+32 candidates are expected to pass).
struct PrioRule {
    bool only_cached;        // at least k cached neighbours: only they compete
    uint64_t thr;
    __device__ __forceinline__ PrioRule(int d, int k, int cached) {
        only_cached = cached >= k;
        const int pool = only_cached ? cached : d - cached;
        const int expect = 2 * (only_cached ? k : k - cached) + 32;
        thr = kMaxKey;
        if (pool > expect) thr = static_cast<uint64_t>((double(expect) / double(pool)) * 18446744073709551616.0);
    }
    __device__ __forceinline__ bool operator()(bool is_cached_slot, uint64_t key) const {
        return only_cached ? (is_cached_slot && key <= thr) : (is_cached_slot || key <= thr);
    }
};

constexpr int kPrioUnroll = 4;   // chunks of 64 slots whose loads are issued together

// Hubs: the four wavefronts of a workgroup share one row, as in sample_hubs.
template <typename IdxT>
__device__ void sample_hubs_prio(const IdxT *__restrict__ col_idx, const IdxT *__restrict__ dst_ids, const SampleArgs &a,
                                 const uint32_t *__restrict__ prio, const int32_t *__restrict__ prio_count,
                                 const int32_t *__restrict__ heavy_rows, int nheavy, int first, int step,
                                 uint64_t *ck, uint32_t *cs, int32_t *sel_slot, int *cnt_s) {
    const int tid = threadIdx.x;
    const int lane = lane_id();
    const int wave = tid >> 6;
    const int k = a.fanout;
    for (int h = first; h < nheavy; h += step) {
        const int row = heavy_rows[h];
        const int64_t start = a.row_start[row];
        const int d = a.row_deg[row];
        const int32_t out_base = out_base_of(a, row);
        const IdxT node = dst_ids[row];
        const uint64_t hv = mix64(layer_hash_of(a) ^ uint64_t(node));
        const RowKeys key_of(hv);
        const IdxT *nbrs = col_idx + start;
        const PrioRule rule(d, k, prio_count[node]);
        if (tid == 0) *cnt_s = 0;
        __syncthreads();
        for (int base = 0; base < d; base += kPrioUnroll * kBlock) {
            uint32_t u[kPrioUnroll], wbits[kPrioUnroll];
#pragma unroll
            for (int q = 0; q < kPrioUnroll; ++q) {
                const int j = base + q * kBlock + tid;
                u[q] = j < d ? static_cast<uint32_t>(nbrs[j]) : 0u;
            }
#pragma unroll
            for (int q = 0; q < kPrioUnroll; ++q) wbits[q] = prio[u[q] >> 5];
#pragma unroll
            for (int q = 0; q < kPrioUnroll; ++q) {
                const int j = base + q * kBlock + tid;
                const bool cj = j < d && ((wbits[q] >> (u[q] & 31)) & 1u);
                const uint64_t key = key_of(j);
                const bool c = j < d && rule(cj, key);
                const uint64_t m = ballot64(c);
                if (m) {
                    int p0 = 0;
                    if (lane == 0) p0 = atomicAdd(cnt_s, popc64(m));
                    p0 = __shfl(p0, 0, 64);
                    if (c) {
                        const int p = p0 + popc64(m & lanes_below(lane));
                        if (p < kCandidates) {
                            ck[p] = key;
                            cs[p] = static_cast<uint32_t>(j) | (cj ? 0u : 0x80000000u);
                        }
                    }
                }
            }
        }
        __syncthreads();
        const int cnt = *cnt_s;
        if (cnt < k || cnt > kCandidates) {                // workgroup-uniform; practically never
            if (wave == 0) select_by_repeated_min_prio(col_idx, start, d, k, hv, out_base, a, prio);
            __syncthreads();
            continue;
        }
        if (wave == 0) emit_selected_unordered<true>(ck, cs, cnt, k, sel_slot, col_idx, start, out_base, a);
        __syncthreads();
    }
}

// Same launch shape as k_sample: the first hub_blocks workgroups take the hubs, every other
// workgroup gives each of its four wavefronts one destination.
template <typename IdxT>
__global__ void __launch_bounds__(kBlock)
k_sample_prio(const IdxT *__restrict__ col_idx, const IdxT *__restrict__ dst_ids, SampleArgs a,
              const uint32_t *__restrict__ prio, const int32_t *__restrict__ prio_count,
              const int32_t *__restrict__ heavy_rows, const int32_t *__restrict__ heavy_count, int hub_blocks) {
    __shared__ uint64_t cand_key[kWavesPerBlock][kCandidates];
    __shared__ uint32_t cand_slot[kWavesPerBlock][kCandidates];   // bit 31: not cached
    __shared__ int32_t sel_slot[kWave];
    __shared__ int cnt_s;
    if (static_cast<int>(blockIdx.x) < hub_blocks) {
        sample_hubs_prio(col_idx, dst_ids, a, prio, prio_count, heavy_rows, *heavy_count, static_cast<int>(blockIdx.x),
                         hub_blocks, cand_key[0], cand_slot[0], sel_slot, &cnt_s);
        return;
    }
    const int lane = lane_id();
    const int wave = static_cast<int>(threadIdx.x) >> 6;
    const int64_t n = a.sizes[0];
    const int64_t row = (int64_t(blockIdx.x) - hub_blocks) * kWavesPerBlock + wave;
    if (row >= n) return;

    const int64_t start = a.row_start[row];
    const int d = a.row_deg[row];
    const int k = a.fanout;
    const int32_t out_base = out_base_of(a, row);
    if (d <= k) {
        if (lane < d) emit_neighbour(col_idx, start, lane, out_base + lane, a);
        return;
    }
    if (d > a.heavy_degree) return;                        // a hub: sampled by the first workgroups
    const IdxT node = dst_ids[row];
    const uint64_t hv = mix64(layer_hash_of(a) ^ uint64_t(node));
    if (a.force_slow) {
        select_by_repeated_min_prio(col_idx, start, d, k, hv, out_base, a, prio);
        return;
    }
    const IdxT *nbrs = col_idx + start;
    if (d <= kWave) {
        const bool unc = lane < d ? !is_cached(nbrs, lane, prio) : true;
        const uint64_t key[1] = {RowKeys(hv)(lane)};
        const uint64_t late[1] = {ballot64(unc)};
        const uint32_t tie[1] = {0};
        uint64_t cand[1] = {low_lanes(d)}, sel[1];
        wave_select_smallest<1, true, false>(key, late, tie, cand, k, sel);
        if ((sel[0] >> lane) & 1) emit_neighbour(col_idx, start, lane, out_base + popc64(sel[0] & lanes_below(lane)), a);
        return;
    }

    // d > 64.  The number of cached neighbours of the row (tabulated when the priority was set)
    // decides the pool the threshold applies to: with at least k of them only cached slots compete;
    // otherwise all of them are taken and the uncached slots compete for the rest.
    const PrioRule rule(d, k, prio_count[node]);
    uint64_t *ck = cand_key[wave];
    uint32_t *cs = cand_slot[wave];
    int cnt = 0;
    const RowKeys key_of(hv);
    for (int base = 0; base < d; base += kPrioUnroll * kWave) {
        uint32_t u[kPrioUnroll], wbits[kPrioUnroll];
#pragma unroll
        for (int q = 0; q < kPrioUnroll; ++q) {
            const int j = base + q * kWave + lane;
            u[q] = j < d ? static_cast<uint32_t>(nbrs[j]) : 0u;
        }
#pragma unroll
        for (int q = 0; q < kPrioUnroll; ++q) wbits[q] = prio[u[q] >> 5];
#pragma unroll
        for (int q = 0; q < kPrioUnroll; ++q) {
            const int j = base + q * kWave + lane;
            const bool cj = j < d && ((wbits[q] >> (u[q] & 31)) & 1u);
            const uint64_t key = key_of(j);
            const bool c = j < d && rule(cj, key);
            const uint64_t m = ballot64(c);
            if (c) {
                const int p = cnt + popc64(m & lanes_below(lane));
                if (p < kCandidates) {
                    ck[p] = key;
                    cs[p] = static_cast<uint32_t>(j) | (cj ? 0u : 0x80000000u);
                }
            }
            cnt += popc64(m);
        }
    }
    if (cnt < k || cnt > kCandidates) {
        select_by_repeated_min_prio(col_idx, start, d, k, hv, out_base, a, prio);
        return;
    }
    wave_lds_sync();
    emit_selected_any<true>(ck, cs, cnt, k, col_idx, start, out_base, a);
}

// prio_count[v] = number of cached neighbours of node v.  A lane owns a node; rows of up to 32 slots
// are walked by their lane, longer rows by the whole wavefront, one after the other.
template <typename PtrT, typename IdxT>
__global__ void __launch_bounds__(kBlock)
k_prio_counts(const PtrT *__restrict__ row_ptr, const IdxT *__restrict__ col_idx, int64_t n,
              const uint32_t *__restrict__ prio, int32_t *__restrict__ prio_count) {
    const int lane = lane_id();
    const int64_t v = int64_t(blockIdx.x) * kBlock + threadIdx.x;
    int64_t start = 0;
    int d = 0;
    if (v < n) {
        start = static_cast<int64_t>(row_ptr[v]);
        d = static_cast<int>(static_cast<int64_t>(row_ptr[v + 1]) - start);
    }
    int c = 0;
    if (d <= 32)
        for (int j = 0; j < d; ++j) c += is_cached(col_idx + start, j, prio) ? 1 : 0;
    uint64_t big = ballot64(d > 32);
    while (big) {
        const int l = __ffsll(static_cast<long long>(big)) - 1;
        big &= big - 1;
        const int dl = static_cast<int>(readlane32(static_cast<uint32_t>(d), l));
        const int64_t sl = static_cast<int64_t>(readlane64(static_cast<uint64_t>(start), l));
        int m = 0;
        for (int base = 0; base < dl; base += kWave) {
            const int j = base + lane;
            m += popc64(ballot64(j < dl && is_cached(col_idx + sl, j, prio)));
        }
        if (lane == l) c = m;
    }
    if (v < n) prio_count[v] = c;
}

// bit v of the bitmap = node v is cached (slot_of[v] >= 0); one lane per node
__global__ void __launch_bounds__(kBlock)
k_prio_bitmap(const int32_t *__restrict__ slot_of, int64_t n, uint32_t *__restrict__ prio) {
    const int64_t v = int64_t(blockIdx.x) * kBlock + threadIdx.x;
    const uint64_t m = ballot64(v < n && slot_of[v] >= 0);
    if (lane_id() == 0) {                                  // v is a multiple of 64 here; padding words get zeros
        prio[v >> 5] = static_cast<uint32_t>(m);
        prio[(v >> 5) + 1] = static_cast<uint32_t>(m >> 32);
    }
}

// ------------------------------------------------------------------------------------------
// Bitmap -> ascending list of new source nodes.

// Two tile shapes.  Dense bitmaps (up to 32 M nodes): one word per thread, 256 words per
// workgroup, ids staged through LDS so that the source list is written coalesced.  Larger graphs:
// four words per thread (one 16-byte load), ids written straight from the bit loop - their bitmaps
// are sparse, a thread rarely has more than a bit or two.
template <int WPT>
__device__ __forceinline__ void bitmap_count_tile(const uint32_t *__restrict__ bitmap, int32_t *__restrict__ tile_sums, int tile,
                                                  int *lds) {
    const int64_t w0 = (int64_t(tile) * kBlock + threadIdx.x) * WPT;
    int c;
    if (WPT == 4) {
        uint4 w = *reinterpret_cast<const uint4 *>(bitmap + w0);
        c = __popc(w.x) + __popc(w.y) + __popc(w.z) + __popc(w.w);
    } else {
        c = __popc(bitmap[w0]);
    }
    int s = wave_sum(c);
    if (lane_id() == 0) lds[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        int t = 0;
#pragma unroll
        for (int k = 0; k < kWavesPerBlock; ++k) t += lds[k];
        tile_sums[tile] = t;
    }
}

// The first row_tiles workgroups turn the row tile sums into indptr, the others count the bits of
// one bitmap tile each: both only need what the launches before produced.
template <int WPT>
__global__ void __launch_bounds__(kBlock)
k_offsets_count(const int32_t *__restrict__ row_deg, int fanout, int64_t *sizes, const int32_t *__restrict__ row_tile_vals,
                int rows_scanned, int32_t *__restrict__ indptr, const int32_t *__restrict__ seed_flags, int row_tiles,
                const uint32_t *__restrict__ bitmap, int32_t *__restrict__ bitmap_tile_sums) {
    __shared__ int lds[kWavesPerBlock];
    const int b = static_cast<int>(blockIdx.x);
    if (b < row_tiles) row_offsets_tile(row_deg, fanout, sizes, row_tile_vals, rows_scanned, indptr, seed_flags, b, row_tiles, lds);
    else bitmap_count_tile<WPT>(bitmap, bitmap_tile_sums, b - row_tiles, lds);
}

// num_src of a block is also num_dst of the next block outward
__device__ __forceinline__ void store_num_src(int64_t *sizes, int64_t *next_num_dst, int64_t num_src) {
    sizes[1] = num_src;
    if (next_num_dst) *next_num_dst = num_src;
}

template <typename IdxT>
__global__ void __launch_bounds__(kBlock)
k_bitmap_emit4(uint32_t *__restrict__ bitmap, const int32_t *__restrict__ tile_vals, int scanned,
               int64_t *__restrict__ sizes, int64_t *__restrict__ next_num_dst, IdxT *__restrict__ src_ids,
               int32_t *__restrict__ local_of) {
    __shared__ int lds[kWavesPerBlock];
    const int tile_base = scanned ? tile_vals[blockIdx.x] : tiles_before(tile_vals, lds);
    const int64_t w0 = (int64_t(blockIdx.x) * kBlock + threadIdx.x) * 4;
    uint4 w = *reinterpret_cast<const uint4 *>(bitmap + w0);
    int c = __popc(w.x) + __popc(w.y) + __popc(w.z) + __popc(w.w);
    int total;
    int ex = block_excl_scan<kWavesPerBlock>(c, &total, lds);
    const int64_t num_dst = sizes[0];
    if (!scanned && blockIdx.x == gridDim.x - 1 && threadIdx.x == 0) store_num_src(sizes, next_num_dst, num_dst + tile_base + total);
    if (c == 0) return;
    int64_t pos = num_dst + tile_base + ex;
    uint32_t words[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        uint32_t bits = words[q];
        while (bits) {
            int b = __ffs(bits) - 1;
            bits &= bits - 1;
            int32_t v = static_cast<int32_t>((w0 + q) * 32 + b);
            src_ids[pos] = static_cast<IdxT>(v);
            local_of[v] = static_cast<int32_t>(pos);
            ++pos;
        }
    }
    *reinterpret_cast<uint4 *>(bitmap + w0) = make_uint4(0, 0, 0, 0);
}

template <typename IdxT>
__global__ void __launch_bounds__(kBlock)
k_bitmap_emit1(uint32_t *__restrict__ bitmap, const int32_t *__restrict__ tile_vals, int scanned,
               int64_t *__restrict__ sizes, int64_t *__restrict__ next_num_dst, IdxT *__restrict__ src_ids,
               int32_t *__restrict__ local_of) {
    __shared__ int lds[kWavesPerBlock];
    __shared__ int32_t staged[kBlock * 32];                // every id of the tile, ascending
    const int tile_base = scanned ? tile_vals[blockIdx.x] : tiles_before(tile_vals, lds);
    const int64_t w0 = int64_t(blockIdx.x) * kBlock + threadIdx.x;
    uint32_t bits = bitmap[w0];
    const int c = __popc(bits);
    int total;
    int ex = block_excl_scan<kWavesPerBlock>(c, &total, lds);
    const int64_t num_dst = sizes[0];
    if (!scanned && blockIdx.x == gridDim.x - 1 && threadIdx.x == 0) store_num_src(sizes, next_num_dst, num_dst + tile_base + total);
    if (total == 0) return;                                // workgroup-uniform
    if (c) {
        bitmap[w0] = 0;
        const int32_t v0 = static_cast<int32_t>(w0 * 32);
        while (bits) {
            int b = __ffs(bits) - 1;
            bits &= bits - 1;
            staged[ex++] = v0 + b;
        }
    }
    __syncthreads();
    const int64_t base = num_dst + tile_base;
    for (int k = threadIdx.x; k < total; k += kBlock) {
        const int32_t v = staged[k];
        src_ids[base + k] = static_cast<IdxT>(v);
        local_of[v] = static_cast<int32_t>(base + k);
    }
}

// Small bitmaps (at most kSelfCountTiles tiles of 256 words, i.e. graphs of up to half a million
// nodes): no counting launch.  Every tile's workgroup counts the set bits of the tiles before its own
// itself, so the words must stay as they are until every workgroup has read them: they are cleared by
// the relabel launch that follows.  The same launch turns the row tile sums into indptr (the
// workgroups past the bitmap's tiles), as k_offsets_count does on larger graphs.
constexpr int kSelfCountTiles = 64;
template <typename IdxT>
__global__ void __launch_bounds__(kBlock)
k_emit_offsets(const uint32_t *__restrict__ bitmap, int bitmap_tiles, int64_t *sizes, int64_t *__restrict__ next_num_dst,
               IdxT *__restrict__ src_ids, int32_t *__restrict__ local_of, const int32_t *__restrict__ row_deg, int fanout,
               const int32_t *__restrict__ row_tile_vals, int rows_scanned, int32_t *__restrict__ indptr,
               const int32_t *__restrict__ seed_flags, int row_tiles) {
    __shared__ int lds[kWavesPerBlock];
    __shared__ int32_t staged[kBlock * 32];                // every id of the tile, ascending
    const int tile = static_cast<int>(blockIdx.x);
    if (tile >= bitmap_tiles) {
        row_offsets_tile(row_deg, fanout, sizes, row_tile_vals, rows_scanned, indptr, seed_flags, tile - bitmap_tiles, row_tiles, lds);
        return;
    }
    int part = 0;
#pragma unroll 4
    for (int t = 0; t < tile; ++t) part += __popc(bitmap[t * kBlock + threadIdx.x]);
    part = wave_sum(part);
    if (lane_id() == 0) lds[threadIdx.x >> 6] = part;
    __syncthreads();
    int tile_base = 0;
#pragma unroll
    for (int k = 0; k < kWavesPerBlock; ++k) tile_base += lds[k];
    const int64_t w0 = int64_t(tile) * kBlock + threadIdx.x;
    uint32_t bits = bitmap[w0];
    const int c = __popc(bits);
    int total;
    int ex = block_excl_scan<kWavesPerBlock>(c, &total, lds);
    const int64_t num_dst = sizes[0];
    if (tile == bitmap_tiles - 1 && threadIdx.x == 0) store_num_src(sizes, next_num_dst, num_dst + tile_base + total);
    if (total == 0) return;                                // workgroup-uniform
    if (c) {
        const int32_t v0 = static_cast<int32_t>(w0 * 32);
        while (bits) {
            int b = __ffs(bits) - 1;
            bits &= bits - 1;
            staged[ex++] = v0 + b;
        }
    }
    __syncthreads();
    const int64_t base = num_dst + tile_base;
    for (int k = threadIdx.x; k < total; k += kBlock) {
        const int32_t v = staged[k];
        src_ids[base + k] = static_cast<IdxT>(v);
        local_of[v] = static_cast<int32_t>(base + k);
    }
}

// Neighbour j of row r sits at nbr[r * fanout + j]; its edge position is indptr[r] + j.  Workgroups
// vb of nb walk the num_dst * fanout slots.
__device__ __forceinline__ void relabel_slots(const int32_t *__restrict__ nbr, const int64_t *__restrict__ sizes,
                                              const int32_t *__restrict__ indptr, int fanout,
                                              const int32_t *__restrict__ local_of, int32_t *__restrict__ indices, int vb, int nb) {
    const uint32_t total = static_cast<uint32_t>(sizes[0] * fanout);
    const uint32_t stride = static_cast<uint32_t>(nb) * kBlock;
    for (uint64_t t64 = uint64_t(vb) * kBlock + threadIdx.x; t64 < total; t64 += stride) {
        const uint32_t t = static_cast<uint32_t>(t64);
        const uint32_t row = t / static_cast<uint32_t>(fanout);
        const int j = static_cast<int>(t - row * static_cast<uint32_t>(fanout));
        const int b = indptr[row];
        if (j < indptr[row + 1] - b) indices[b + j] = local_of[nbr[t]];
    }
}

// (clear: the frontier bitmap, when the emit launch left its words set; vb of nb workgroups)
__device__ __forceinline__ void clear_words(uint32_t *__restrict__ clear, int64_t clear_words, int vb, int nb) {
    if (!clear) return;
    for (int64_t w = int64_t(vb) * kBlock + threadIdx.x; w < clear_words; w += int64_t(nb) * kBlock) clear[w] = 0;
}

__global__ void __launch_bounds__(kBlock)
k_relabel(const int32_t *__restrict__ nbr, const int64_t *__restrict__ sizes, const int32_t *__restrict__ indptr, int fanout,
          const int32_t *__restrict__ local_of, int32_t *__restrict__ indices, uint32_t *__restrict__ clear, int64_t nclear) {
    clear_words(clear, nclear, static_cast<int>(blockIdx.x), static_cast<int>(gridDim.x));
    relabel_slots(nbr, sizes, indptr, fanout, local_of, indices, static_cast<int>(blockIdx.x), static_cast<int>(gridDim.x));
}

// The relabel of one block and, in the same launch, the row information of the next block outward
// (its destinations are this block's sources, complete since k_bitmap_emit).
template <typename PtrT, typename IdxT>
__global__ void __launch_bounds__(kBlock)
k_relabel_rowinfo(const int32_t *__restrict__ nbr, const int64_t *__restrict__ sizes, const int32_t *__restrict__ indptr,
                  int fanout, const int32_t *__restrict__ local_of, int32_t *__restrict__ indices, int relabel_blocks,
                  RowInfoArgs<PtrT, IdxT> next, uint32_t *__restrict__ clear, int64_t nclear) {
    __shared__ int lds[kWavesPerBlock];
    const int b = static_cast<int>(blockIdx.x);
    if (b < relabel_blocks) {
        clear_words(clear, nclear, b, relabel_blocks);
        relabel_slots(nbr, sizes, indptr, fanout, local_of, indices, b, relabel_blocks);
    } else {
        row_info_tile(next, b - relabel_blocks, lds);
    }
}

template <typename IdxT>
__global__ void __launch_bounds__(kBlock)
k_reset_local(const IdxT *__restrict__ src_ids, const int64_t *__restrict__ sizes, int32_t *__restrict__ local_of,
              int32_t *__restrict__ heavy_count) {
    if (blockIdx.x == 0 && threadIdx.x <= MQG_MAX_LAYERS) heavy_count[threadIdx.x] = 0;  // hub counts and seed flags of the next call
    if (!local_of) return;
    const int64_t n = sizes[1];
    const int64_t stride = int64_t(gridDim.x) * kBlock;
    for (int64_t i = int64_t(blockIdx.x) * kBlock + threadIdx.x; i < n; i += stride) {
        local_of[src_ids[i]] = -1;
    }
}

template <typename PtrT, typename IdxT>
int sample_blocks_impl(mqg_ctx *ctx, const mqg_graph *g, const void *seeds_v, int32_t num_seeds, const uint64_t *seed_dev,
                       const int32_t *fanouts, int32_t L, uint64_t rng_seed, mqg_block *blocks, hipStream_t s) {
    const PtrT *row_ptr = static_cast<const PtrT *>(g->row_ptr);
    const IdxT *col_idx = static_cast<const IdxT *>(g->col_idx);
    const IdxT *seeds = static_cast<const IdxT *>(seeds_v);
    int32_t *nbr = static_cast<int32_t *>(ctx->nbr);
    const uint64_t seed_hash = host_mix64(rng_seed + kGolden);

    const bool use_hash = ctx->dedup_hash;
    int32_t *local_of = use_hash ? nullptr : ctx->local_of;
    int64_t need_dst = num_seeds;
    const int bitmap_wpt = ctx->bitmap_words <= (int64_t(1) << 20) ? 1 : 4;     // words per thread, see k_bitmap_emit*
    const int bitmap_tiles = static_cast<int>(std::max<int64_t>(1, ctx->bitmap_words / (int64_t(kBlock) * bitmap_wpt)));
    const bool self_count = !use_hash && bitmap_wpt == 1 && bitmap_tiles <= kSelfCountTiles;    // see k_emit_offsets
    const int heavy_degree = ctx->force_slow_select ? 0x7FFFFFFF : ctx->heavy_degree;
    auto row_info_args = [&](int l, int64_t dst_count) {
        RowInfoArgs<PtrT, IdxT> r;
        r.row_ptr = row_ptr;
        r.dst = (l == L - 1) ? seeds : static_cast<const IdxT *>(blocks[l + 1].src_ids);
        r.sizes = blocks[l].sizes;
        r.src_out = static_cast<IdxT *>(blocks[l].src_ids);
        r.fanout = fanouts[l];
        r.row_start = ctx->row_start;
        r.row_deg = ctx->row_deg;
        r.tile_sums = ctx->tile_vals;
        r.sizes_rw = blocks[l].sizes;
        r.heavy_degree = heavy_degree;
        r.heavy_rows = ctx->heavy_rows;
        r.heavy_count = ctx->heavy_count + l;
        r.n_seeds = l == L - 1 ? dst_count : int64_t(-1);
        r.local_of = local_of;
        r.num_nodes = g->num_nodes;
        r.seed_flags = ctx->heavy_count + MQG_MAX_LAYERS;
        return r;
    };
    auto tiles_of = [](int64_t rows) { return static_cast<int>(std::max<int64_t>(1, ceil_div(rows, kBlock))); };
    // the innermost block's row information; every other block's is launched with the relabel before it
    MQG_LAUNCH(ctx, "k_row_info", s, (k_row_info<PtrT, IdxT><<<tiles_of(need_dst), kBlock, 0, s>>>(row_info_args(L - 1, need_dst))));
    for (int l = L - 1; l >= 0; --l) {
        mqg_block &b = blocks[l];
        const int k = fanouts[l];
        IdxT *src_ids = static_cast<IdxT *>(b.src_ids);
        const int64_t need_nnz = need_dst * k;
        const int row_tiles = tiles_of(need_dst);
        const int64_t next_dst = std::max(need_dst, std::min<int64_t>(g->num_nodes, need_dst + need_nnz));

        // few tiles: every workgroup of the consumer adds up the tile sums before its own; many: one scan launch
        const int rows_scanned = row_tiles > kSelfPrefixTiles ? 1 : 0;
        int rc = MQG_OK;
        if (rows_scanned) rc = launch_scan_tiles(ctx, ctx->tile_vals, row_tiles, nullptr, &b.sizes[2], nullptr, s, "k_scan_tiles(rows)");
        if (rc != MQG_OK) return rc;
        const int32_t *seed_flags = l == L - 1 ? ctx->heavy_count + MQG_MAX_LAYERS : nullptr;
        if (use_hash) {
            if (l == L - 1) {                              // the seeds enter the table (and repeated ones are flagged) first
                rc = hash_put_seeds(ctx, b.src_ids, g->idx_type, need_dst, b.sizes, s);   // ids as the row info checked them
                if (rc != MQG_OK) return rc;
            }
            MQG_LAUNCH(ctx, "k_row_offsets", s,
                       (k_row_offsets<<<row_tiles, kBlock, 0, s>>>(ctx->row_deg, k, b.sizes, ctx->tile_vals, rows_scanned, b.indptr, seed_flags)));
        }

        SampleArgs a;
        a.row_start = ctx->row_start;
        a.row_deg = ctx->row_deg;
        a.indptr = use_hash ? b.indptr : nullptr;
        a.sizes = b.sizes;
        a.nbr = nbr;
        a.local_of = local_of;
        a.bitmap = ctx->bitmap;
        a.layer_hash = host_mix64(seed_hash ^ uint64_t(l));
        a.seed_dev = seed_dev;
        a.layer = l;
        a.fanout = k;
        a.force_slow = ctx->force_slow_select ? 1 : 0;
        a.heavy_degree = heavy_degree;
        const int hub_blocks = static_cast<int>(std::min<int64_t>(std::max<int64_t>(1, need_dst), 2048));
        int sample_grid = hub_blocks + static_cast<int>(std::max<int64_t>(1, ceil_div(need_dst, kWavesPerBlock)));
        if (ctx->prio_enabled) {
            MQG_LAUNCH(ctx, "k_sample_prio", s,
                       (k_sample_prio<IdxT><<<sample_grid, kBlock, 0, s>>>(col_idx, src_ids, a, ctx->prio_bitmap, ctx->prio_count,
                                                                           ctx->heavy_rows, ctx->heavy_count + l, hub_blocks)));
        } else {
            MQG_LAUNCH(ctx, "k_sample", s,
                       (k_sample<IdxT><<<sample_grid, kBlock, 0, s>>>(col_idx, src_ids, a, ctx->heavy_rows, ctx->heavy_count + l, hub_blocks)));
        }

        if (use_hash) {
            rc = hash_dedup_block(ctx, nbr, need_nnz, g->num_nodes, g->idx_type, b.src_ids, b.sizes,
                                  l > 0 ? blocks[l - 1].sizes : nullptr, b.indices, s);
            if (rc != MQG_OK) return rc;
            need_dst = next_dst;
            if (l > 0) MQG_LAUNCH(ctx, "k_row_info", s, (k_row_info<PtrT, IdxT><<<tiles_of(need_dst), kBlock, 0, s>>>(row_info_args(l - 1, need_dst))));
            continue;
        }
        // num_src = num_dst + number of new nodes; it is also the next block's num_dst
        int64_t *next_num_dst = l > 0 ? &blocks[l - 1].sizes[0] : nullptr;
        if (self_count) {
            // indptr from the row tile sums and the new sources from the bitmap, one launch
            MQG_LAUNCH(ctx, "k_emit_offsets", s,
                       (k_emit_offsets<IdxT><<<bitmap_tiles + row_tiles, kBlock, 0, s>>>(ctx->bitmap, bitmap_tiles, b.sizes, next_num_dst, src_ids,
                                                                                        ctx->local_of, ctx->row_deg, k, ctx->tile_vals, rows_scanned,
                                                                                        b.indptr, seed_flags, row_tiles)));
        } else {
            // indptr from the row tile sums, and the bitmap's tile popcounts
            if (bitmap_wpt == 1) {
                MQG_LAUNCH(ctx, "k_offsets_count", s,
                           (k_offsets_count<1><<<row_tiles + bitmap_tiles, kBlock, 0, s>>>(ctx->row_deg, k, b.sizes, ctx->tile_vals, rows_scanned, b.indptr,
                                                                                          seed_flags, row_tiles, ctx->bitmap, ctx->bitmap_tile_vals)));
            } else {
                MQG_LAUNCH(ctx, "k_offsets_count", s,
                           (k_offsets_count<4><<<row_tiles + bitmap_tiles, kBlock, 0, s>>>(ctx->row_deg, k, b.sizes, ctx->tile_vals, rows_scanned, b.indptr,
                                                                                          seed_flags, row_tiles, ctx->bitmap, ctx->bitmap_tile_vals)));
            }
            const int bits_scanned = bitmap_tiles > kSelfPrefixTiles ? 1 : 0;
            if (bits_scanned) rc = launch_scan_tiles(ctx, ctx->bitmap_tile_vals, bitmap_tiles, &b.sizes[0], &b.sizes[1], next_num_dst, s, "k_scan_tiles(bitmap)");
            if (rc != MQG_OK) return rc;
            if (bitmap_wpt == 1) {
                MQG_LAUNCH(ctx, "k_bitmap_emit", s,
                           (k_bitmap_emit1<IdxT><<<bitmap_tiles, kBlock, 0, s>>>(ctx->bitmap, ctx->bitmap_tile_vals, bits_scanned, b.sizes, next_num_dst, src_ids, ctx->local_of)));
            } else {
                MQG_LAUNCH(ctx, "k_bitmap_emit", s,
                           (k_bitmap_emit4<IdxT><<<bitmap_tiles, kBlock, 0, s>>>(ctx->bitmap, ctx->bitmap_tile_vals, bits_scanned, b.sizes, next_num_dst, src_ids, ctx->local_of)));
            }
        }
        const int relabel_grid = static_cast<int>(std::min<int64_t>(std::max<int64_t>(1, ceil_div(need_nnz, kBlock)), 4096));
        need_dst = next_dst;
        if (l > 0) {
            MQG_LAUNCH(ctx, "k_relabel_rowinfo", s,
                       (k_relabel_rowinfo<PtrT, IdxT><<<relabel_grid + tiles_of(need_dst), kBlock, 0, s>>>(nbr, b.sizes, b.indptr, k, ctx->local_of, b.indices,
                                                                                                          relabel_grid, row_info_args(l - 1, need_dst),
                                                                                                          self_count ? ctx->bitmap : nullptr, ctx->bitmap_words)));
        } else {
            MQG_LAUNCH(ctx, "k_relabel", s, (k_relabel<<<relabel_grid, kBlock, 0, s>>>(nbr, b.sizes, b.indptr, k, ctx->local_of, b.indices,
                                                                                       self_count ? ctx->bitmap : nullptr, ctx->bitmap_words)));
        }
    }
    {
        int grid = static_cast<int>(std::min<int64_t>(std::max<int64_t>(1, ceil_div(need_dst, kBlock)), 4096));
        MQG_LAUNCH(ctx, "k_reset_local", s,
                   (k_reset_local<IdxT><<<grid, kBlock, 0, s>>>(static_cast<const IdxT *>(blocks[0].src_ids), blocks[0].sizes,
                                                                 local_of, ctx->heavy_count)));
    }
    if (use_hash) return hash_clear(ctx, s);
    return MQG_OK;
}

}  // namespace

int launch_scan_tiles(mqg_ctx *ctx, int32_t *vals, int64_t n, const int64_t *addend, int64_t *total_a,
                      int64_t *total_b, hipStream_t s, const char *name) {
    MQG_LAUNCH(ctx, name, s, (k_scan_tiles<<<1, 1024, 0, s>>>(vals, n, addend, total_a, total_b)));
    return MQG_OK;
}

int run_sample_blocks(mqg_ctx *ctx, const mqg_graph *g, const void *seeds, int32_t num_seeds, const int32_t *fanouts,
                      int32_t L, uint64_t rng_seed, const uint64_t *seed_dev, mqg_block *blocks, hipStream_t s) {
    const bool p64 = g->ptr_type == MQG_I64, i64 = g->idx_type == MQG_I64;
    if (p64 && i64) return sample_blocks_impl<int64_t, int64_t>(ctx, g, seeds, num_seeds, seed_dev, fanouts, L, rng_seed, blocks, s);
    if (p64 && !i64) return sample_blocks_impl<int64_t, int32_t>(ctx, g, seeds, num_seeds, seed_dev, fanouts, L, rng_seed, blocks, s);
    if (!p64 && i64) return sample_blocks_impl<int32_t, int64_t>(ctx, g, seeds, num_seeds, seed_dev, fanouts, L, rng_seed, blocks, s);
    return sample_blocks_impl<int32_t, int32_t>(ctx, g, seeds, num_seeds, seed_dev, fanouts, L, rng_seed, blocks, s);
}

int run_select_row_candidates(mqg_ctx *ctx, const uint64_t *keys, const uint32_t *slot_words, int32_t cnt, int32_t k,
                              int32_t prioritised, int32_t ordered, uint32_t *out_mask, hipStream_t s) {
    if (prioritised && ordered) MQG_LAUNCH(ctx, "k_select_candidates", s, (k_select_candidates<true, true><<<1, kWave, 0, s>>>(keys, slot_words, cnt, k, out_mask)));
    else if (prioritised) MQG_LAUNCH(ctx, "k_select_candidates", s, (k_select_candidates<true, false><<<1, kWave, 0, s>>>(keys, slot_words, cnt, k, out_mask)));
    else if (ordered) MQG_LAUNCH(ctx, "k_select_candidates", s, (k_select_candidates<false, true><<<1, kWave, 0, s>>>(keys, slot_words, cnt, k, out_mask)));
    else MQG_LAUNCH(ctx, "k_select_candidates", s, (k_select_candidates<false, false><<<1, kWave, 0, s>>>(keys, slot_words, cnt, k, out_mask)));
    return MQG_OK;
}

// the membership bitmap and the table of cached-neighbour counts
int ensure_priority_scratch(mqg_ctx *ctx) {
    if (ctx->prio_bitmap) return MQG_OK;
    bool ok = hipMalloc(reinterpret_cast<void **>(&ctx->prio_bitmap), static_cast<size_t>(ctx->bitmap_words) * sizeof(uint32_t)) == hipSuccess &&
              hipMalloc(reinterpret_cast<void **>(&ctx->prio_count), static_cast<size_t>(std::max<int64_t>(ctx->num_nodes, 1)) * sizeof(int32_t)) == hipSuccess;
    if (!ok) {
        (void)hipFree(ctx->prio_bitmap);
        (void)hipFree(ctx->prio_count);
        ctx->prio_bitmap = nullptr;
        ctx->prio_count = nullptr;
        return fail(ctx, MQG_ERR_HIP, "mqg_ctx_set_sampling_priority: allocation failed");
    }
    return MQG_OK;
}

// cache == nullptr switches the priority off; otherwise the membership bitmap is (re)built from cache->slot_of
int run_set_sampling_priority(mqg_ctx *ctx, const mqg_graph *g, const mqg_cache *cache, hipStream_t s) {
    if (!cache) {
        ctx->prio_enabled = false;
        return MQG_OK;
    }
    int rc0 = ensure_priority_scratch(ctx);
    if (rc0 != MQG_OK) return rc0;
    const int grid = static_cast<int>(ctx->bitmap_words * 32 / kBlock);
    MQG_LAUNCH(ctx, "k_prio_bitmap", s, (k_prio_bitmap<<<grid, kBlock, 0, s>>>(cache->slot_of, ctx->num_nodes, ctx->prio_bitmap)));
    const int64_t n = ctx->num_nodes;
    const int ngrid = static_cast<int>(std::max<int64_t>(1, ceil_div(n, kBlock)));
#define MQG_PRIOC(PT, IT)                                                                                        \
    MQG_LAUNCH(ctx, "k_prio_counts", s,                                                                          \
               (k_prio_counts<PT, IT><<<ngrid, kBlock, 0, s>>>(static_cast<const PT *>(g->row_ptr),               \
                                                              static_cast<const IT *>(g->col_idx), n, ctx->prio_bitmap, \
                                                              ctx->prio_count)))
    if (g->ptr_type == MQG_I64 && g->idx_type == MQG_I64) MQG_PRIOC(int64_t, int64_t);
    else if (g->ptr_type == MQG_I64) MQG_PRIOC(int64_t, int32_t);
    else if (g->idx_type == MQG_I64) MQG_PRIOC(int32_t, int64_t);
    else MQG_PRIOC(int32_t, int32_t);
#undef MQG_PRIOC
    ctx->prio_enabled = true;
    return MQG_OK;
}

}  // namespace mqg
