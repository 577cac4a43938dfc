// GPU construction of a CSF tree from coordinate lists (Sec. 2.1, "CSF representation").
//
// Steps, all on the device:
//   1. pack each coordinate tuple, permuted into level order, into one 64-bit key (outermost
//      level in the most significant bits) and check ranges; tuples that need 65 to 128 bits get a
//      second, more significant word holding the outer levels (no level straddles the two words);
//   2. stable radix sort of (key, original position) -- lexicographic order in mode_order
//      (own LSD sort, 8 bits per pass, see below);
//   3. per tile, count for every level the positions where the key prefix of that level
//      changes ("head" of a node); a duplicate coordinate is a position whose full key
//      equals its predecessor's;
//   4. scan the tile counts; the host reads the node totals and allocates the level arrays;
//   5. per tile, rank the heads (block scan) and emit idx[l], ptr[l] and the permuted values.
// The result is the canonical array layout documented in include/conststn.h.
#include <algorithm>
#include <cstring>

#include "plan.hpp"

namespace cst {

constexpr int kTileThreads = 256;
constexpr int kItems = 8;
constexpr int kTile = kTileThreads * kItems;

struct Levels {
    int order;
    int word[CONSTSTN_MAX_ORDER];           // 0: the level's field lies in the low key word, 1: in the high one
    int shift[CONSTSTN_MAX_ORDER];          // bit offset of the level's field inside its word
    uint64_t mask[CONSTSTN_MAX_ORDER];      // field mask (after shifting)
    int64_t dim[CONSTSTN_MAX_ORDER];        // extent of the mode at this level
    const int32_t *coord[CONSTSTN_MAX_ORDER];
};

struct LevelOut {
    int32_t *idx[CONSTSTN_MAX_ORDER];
    int64_t *ptr[CONSTSTN_MAX_ORDER];
};

__device__ __forceinline__ uint64_t prefix_of(uint64_t key, int shift) {
    return shift >= 64 ? 0 : (key >> shift);
}

// keys_hi = nullptr for keys of one word
__global__ void __launch_bounds__(256)
pack_keys_kernel(int64_t nnz, Levels lv, uint64_t *keys, uint64_t *keys_hi, uint32_t *payload, int *flags) {
    int64_t n = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    const int64_t stride = int64_t(gridDim.x) * blockDim.x;
    bool bad = false;
    for (; n < nnz; n += stride) {
        uint64_t key = 0, hi = 0;
        for (int l = 0; l < lv.order; ++l) {
            int32_t c = lv.coord[l][n];
            if (c < 0 || int64_t(c) >= lv.dim[l]) { bad = true; c = 0; }
            if (lv.shift[l] < 64) {
                if (lv.word[l]) hi |= uint64_t(uint32_t(c)) << lv.shift[l];
                else key |= uint64_t(uint32_t(c)) << lv.shift[l];
            }
        }
        keys[n] = key;
        if (keys_hi) keys_hi[n] = hi;
        payload[n] = uint32_t(n);
    }
    if (bad) atomicOr(&flags[0], 1);
}

// out[i] = in[index[i]]
__global__ void __launch_bounds__(256)
gather_u64_kernel(int64_t n, const uint64_t *__restrict__ in, const uint32_t *__restrict__ index, uint64_t *__restrict__ out) {
    const int64_t i = int64_t(blockIdx.x) * 256 + threadIdx.x;
    if (i < n) out[i] = in[index[i]];
}

// A two-word key (hi = 0 throughout for keys of one word).  The prefix of level l is every bit from the
// level's field upwards: inside the high word for a level stored there, the whole high word plus the
// upper part of the low word otherwise.
struct Key2 { uint64_t hi, lo; };
template <bool WIDE>
__device__ __forceinline__ Key2 load_key(const uint64_t *keys, const uint64_t *keys_hi, int64_t n) {
    return Key2{WIDE ? keys_hi[n] : 0, keys[n]};
}
template <bool WIDE>
__device__ __forceinline__ bool same_prefix(const Levels &lv, int l, Key2 a, Key2 b) {
    if (WIDE && lv.word[l]) return prefix_of(a.hi, lv.shift[l]) == prefix_of(b.hi, lv.shift[l]);
    return (!WIDE || a.hi == b.hi) && prefix_of(a.lo, lv.shift[l]) == prefix_of(b.lo, lv.shift[l]);
}

__device__ __forceinline__ unsigned wave_sum(unsigned v) {
    for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
    return v;
}

// For every level the number of node heads inside each tile; leaf-level non-heads are duplicates.
template <bool WIDE>
__global__ void __launch_bounds__(kTileThreads)
count_heads_kernel(int64_t nnz, Levels lv, const uint64_t *__restrict__ keys, const uint64_t *__restrict__ keys_hi,
                   unsigned *__restrict__ tile_counts, int64_t ntiles, int *flags) {
    __shared__ unsigned wsum[CONSTSTN_MAX_ORDER][kTileThreads / 64];
    const int64_t tile = blockIdx.x;
    const int64_t base = tile * kTile + int64_t(threadIdx.x) * kItems;
    unsigned cnt[CONSTSTN_MAX_ORDER];
    for (int l = 0; l < CONSTSTN_MAX_ORDER; ++l) cnt[l] = 0;
    Key2 prev{0, 0};
    bool have_prev = false;
    if (base > 0 && base <= nnz) { prev = load_key<WIDE>(keys, keys_hi, base - 1); have_prev = true; }
    bool dup = false;
    for (int i = 0; i < kItems; ++i) {
        const int64_t n = base + i;
        if (n >= nnz) break;
        const Key2 k = load_key<WIDE>(keys, keys_hi, n);
        for (int l = 0; l < lv.order; ++l) {
            const bool head = !have_prev || !same_prefix<WIDE>(lv, l, k, prev);
            cnt[l] += head ? 1u : 0u;
            if (l == lv.order - 1 && !head) dup = true;
        }
        prev = k;
        have_prev = true;
    }
    if (dup) atomicOr(&flags[1], 1);
    const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
    for (int l = 0; l < lv.order; ++l) {
        unsigned s = wave_sum(cnt[l]);
        if (lane == 0) wsum[l][wave] = s;
    }
    __syncthreads();
    if (threadIdx.x < lv.order) {
        unsigned s = 0;
        for (int w = 0; w < kTileThreads / 64; ++w) s += wsum[threadIdx.x][w];
        tile_counts[int64_t(threadIdx.x) * ntiles + tile] = s;
    }
}

// Exclusive scan of the tile counts of every level (one block per level); totals[l] = node count.
// The block walks its row in chunks of 4096 counts, four adjacent ones per thread, and carries the
// running total from chunk to chunk.
__global__ void __launch_bounds__(1024)
scan_tiles_kernel(const unsigned *__restrict__ tile_counts, int64_t *__restrict__ tile_offsets,
                  int64_t ntiles, int64_t *totals) {
    __shared__ int64_t wtot[16];
    const int l = blockIdx.x;
    const unsigned *in = tile_counts + int64_t(l) * ntiles;
    int64_t *out = tile_offsets + int64_t(l) * ntiles;
    const int lane = threadIdx.x % 64, wave = threadIdx.x / 64;
    int64_t carry = 0;
    for (int64_t t0 = 0; t0 < ntiles; t0 += 4096) {
        const int64_t t = t0 + int64_t(threadIdx.x) * 4;
        unsigned v[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) v[k] = t + k < ntiles ? in[t + k] : 0u;
        const int64_t mine = int64_t(v[0]) + v[1] + v[2] + v[3];
        int64_t inc = mine;
        for (int off = 1; off < 64; off <<= 1) {
            const int64_t up = __shfl_up(inc, off, 64);
            if (lane >= off) inc += up;
        }
        if (lane == 63) wtot[wave] = inc;
        __syncthreads();
        int64_t before = 0, total = 0;
#pragma unroll
        for (int w = 0; w < 16; ++w) {
            const int64_t x = wtot[w];
            before += w < wave ? x : 0;
            total += x;
        }
        int64_t run = carry + before + inc - mine;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            if (t + k < ntiles) out[t + k] = run;
            run += v[k];
        }
        carry += total;
        __syncthreads();
    }
    if (threadIdx.x == 0) totals[l] = carry;
}

// ---- stable LSD radix sort of (key, position) pairs, 8 bits per pass ------------------------
//
// A workgroup of four wavefronts owns a tile of kSortTile consecutive pairs, wavefront w the w-th
// quarter of it.  Per pass: (1) every workgroup counts the digits of its tile; (2) scan_tiles_kernel
// (one block per digit value) turns the counts into the tile's starting offset inside each digit's
// bucket, a one-wave kernel turns the bucket totals into bucket bases; (3) every workgroup re-reads
// its tile, ranks each pair among the pairs of the tile with the same digit that come before it (in
// a wavefront: 64 pairs at a time, eight ballots narrow the set of peers; across wavefronts: their
// digit counts), lays the tile out by digit in LDS and writes it from there, so that neighbouring
// threads write neighbouring addresses of a bucket.  Tiles are visited in index order inside a
// bucket and pairs in order inside a tile, so the sort is stable, which the CSF needs: equal keys
// (duplicates) must keep input order.
constexpr int kSortItems = 16;
constexpr int kSortWave = kSortItems * 64;            // pairs of one wavefront
constexpr int kSortTile = 4 * kSortWave;

__global__ void __launch_bounds__(256)
radix_count_kernel(int64_t n, const uint64_t *__restrict__ keys, int shift, unsigned *__restrict__ tile_counts,
                   int64_t ntiles) {
    __shared__ unsigned hist[256];
    const int64_t tile = blockIdx.x;
    hist[threadIdx.x] = 0;
    __syncthreads();
    const int64_t base = tile * kSortTile;
#pragma unroll 4
    for (int i = 0; i < kSortItems; ++i) {
        const int64_t e = base + int64_t(i) * 256 + threadIdx.x;
        if (e < n) atomicAdd(&hist[unsigned(keys[e] >> shift) & 255u], 1u);
    }
    __syncthreads();
    tile_counts[int64_t(threadIdx.x) * ntiles + tile] = hist[threadIdx.x];
}

__global__ void radix_bases_kernel(const int64_t *__restrict__ totals, int64_t *__restrict__ bases) {
    // one wave: exclusive scan of the 256 bucket totals
    const int lane = threadIdx.x;
    int64_t v[4], s = 0;
    for (int i = 0; i < 4; ++i) { v[i] = totals[lane * 4 + i]; s += v[i]; }
    int64_t inc = s;
    for (int off = 1; off < 64; off <<= 1) {
        const int64_t t = __shfl_up(inc, off, 64);
        if (lane >= off) inc += t;
    }
    int64_t run = inc - s;
    for (int i = 0; i < 4; ++i) { bases[lane * 4 + i] = run; run += v[i]; }
}

__global__ void __launch_bounds__(256)
radix_scatter_kernel(int64_t n, const uint64_t *__restrict__ keys_in, const uint32_t *__restrict__ pay_in,
                     uint64_t *__restrict__ keys_out, uint32_t *__restrict__ pay_out, int shift,
                     const int64_t *__restrict__ tile_offsets, const int64_t *__restrict__ bases, int64_t ntiles) {
    __shared__ uint64_t lkey[kSortTile];
    __shared__ uint32_t lpay[kSortTile];
    __shared__ unsigned run[4][256];                  // per wavefront: pairs of each digit seen so far
    __shared__ unsigned start[4][256];                // first place in the tile's layout of a wavefront's pairs of a digit
    __shared__ int64_t gbase[256];                    // address of the tile's place p holding digit d: gbase[d] + p
    __shared__ unsigned wsum[4];
    const int wv = threadIdx.x / 64, lane = threadIdx.x % 64;
    const int64_t tile = blockIdx.x;
    const int64_t base = tile * kSortTile + int64_t(wv) * kSortWave;
    for (int w = 0; w < 4; ++w) run[w][threadIdx.x] = 0;
    __syncthreads();
    const unsigned long long lt = (1ull << lane) - 1ull;
    uint64_t key[kSortItems];
    uint32_t pay[kSortItems];
    unsigned rank[kSortItems];                        // among the wavefront's earlier pairs of the same digit
    // pairs past the end sort last: all-ones keys, and they are the last pairs of the last tile
#pragma unroll
    for (int i = 0; i < kSortItems; ++i) {
        const int64_t e = base + int64_t(i) * 64 + lane;
        const bool live = e < n;
        key[i] = live ? keys_in[e] : ~uint64_t(0);
        pay[i] = live ? pay_in[e] : 0u;
    }
#pragma unroll
    for (int i = 0; i < kSortItems; ++i) {
        const unsigned digit = unsigned(key[i] >> shift) & 255u;
        unsigned long long peers = ~0ull;
#pragma unroll
        for (int b = 0; b < 8; ++b) {
            const bool bit = (digit >> b) & 1u;
            const unsigned long long m = __builtin_amdgcn_ballot_w64(bit);
            peers &= bit ? m : ~m;
        }
        const unsigned before = unsigned(__popcll(peers & lt));
        rank[i] = run[wv][digit] + before;
        __builtin_amdgcn_wave_barrier();
        if (before == 0) run[wv][digit] += unsigned(__popcll(peers));      // the lowest peer advances the digit's count
        __builtin_amdgcn_wave_barrier();
    }
    __syncthreads();
    {
        // thread d: where digit d begins in the tile's layout, and inside that where each wavefront's share begins
        const int d = threadIdx.x;
        unsigned c[4], total = 0;
        for (int w = 0; w < 4; ++w) { c[w] = run[w][d]; total += c[w]; }
        unsigned inc = total;
        for (int off = 1; off < 64; off <<= 1) {
            const unsigned up = __shfl_up(inc, off, 64);
            if (lane >= off) inc += up;
        }
        if (lane == 63) wsum[wv] = inc;
        __syncthreads();
        unsigned first = inc - total;
        for (int w = 0; w < wv; ++w) first += wsum[w];
        gbase[d] = bases[d] + tile_offsets[int64_t(d) * ntiles + tile] - int64_t(first);
        for (int w = 0; w < 4; ++w) { start[w][d] = first; first += c[w]; }
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < kSortItems; ++i) {
        const unsigned digit = unsigned(key[i] >> shift) & 255u;
        const unsigned p = start[wv][digit] + rank[i];
        lkey[p] = key[i];
        lpay[p] = pay[i];
    }
    __syncthreads();
    const int64_t rest = n - tile * kSortTile;
    const int live_pairs = rest < kSortTile ? int(rest) : kSortTile;
#pragma unroll 4
    for (int i = 0; i < kSortItems; ++i) {
        const int p = i * 256 + int(threadIdx.x);
        if (p < live_pairs) {
            const uint64_t k = lkey[p];
            const int64_t pos = gbase[unsigned(k >> shift) & 255u] + p;
            keys_out[pos] = k;
            pay_out[pos] = lpay[p];
        }
    }
}

// Sorts n (key, payload) pairs by the low `bits` bits of the key, stably; a and b are two buffers of n
// entries each, the input is in a, the result in whichever *keys_sorted / *pay_sorted name.  Waits
// for the stream before it returns (the pass tables are released then).
static size_t up256(size_t bytes) { return (bytes + 255) / 256 * 256; }

// bytes of pass tables a sort of n pairs needs (handed in by callers that keep one allocation for all their
// temporaries; every device allocation and release costs a fraction of a millisecond)
size_t radix_sort_scratch_bytes(int64_t n) {
    const size_t stiles = size_t(div_up(std::max<int64_t>(n, 1), kSortTile));
    return up256(stiles * 256 * sizeof(unsigned)) + up256(stiles * 256 * sizeof(int64_t)) + 2 * up256(256 * sizeof(int64_t));
}

conststn_status radix_sort_pairs_u64(uint64_t *keys_a, uint64_t *keys_b, uint32_t *pay_a, uint32_t *pay_b, int64_t n,
                                     int bits, hipStream_t stream, const uint64_t **keys_sorted,
                                     const uint32_t **pay_sorted, void *scratch) {
    *keys_sorted = keys_a;
    *pay_sorted = pay_a;
    if (bits <= 0 || n <= 1) return CONSTSTN_OK;
    const int64_t stiles = div_up(n, kSortTile);
    DevBuf<char> own;
    if (!scratch) {
        CST_TRY(own.alloc(radix_sort_scratch_bytes(n)));
        scratch = own.p;
    }
    struct { unsigned *p; } scounts;
    struct { int64_t *p; } soffsets, stotals, sbases;
    {
        char *at = static_cast<char *>(scratch);
        scounts.p = reinterpret_cast<unsigned *>(at);
        at += up256(size_t(stiles) * 256 * sizeof(unsigned));
        soffsets.p = reinterpret_cast<int64_t *>(at);
        at += up256(size_t(stiles) * 256 * sizeof(int64_t));
        stotals.p = reinterpret_cast<int64_t *>(at);
        at += up256(256 * sizeof(int64_t));
        sbases.p = reinterpret_cast<int64_t *>(at);
    }
    uint64_t *kin = keys_a, *kout = keys_b;
    uint32_t *pin = pay_a, *pout = pay_b;
    const dim3 sgrid{unsigned(stiles)}, sblock(256);
    for (int shift = 0; shift < bits; shift += 8) {
        radix_count_kernel<<<sgrid, sblock, 0, stream>>>(n, kin, shift, scounts.p, stiles);
        scan_tiles_kernel<<<dim3(256), dim3(1024), 0, stream>>>(scounts.p, soffsets.p, stiles, stotals.p);
        radix_bases_kernel<<<dim3(1), dim3(64), 0, stream>>>(stotals.p, sbases.p);
        radix_scatter_kernel<<<sgrid, sblock, 0, stream>>>(n, kin, pin, kout, pout, shift, soffsets.p, sbases.p, stiles);
        CST_HIP(hipGetLastError());
        std::swap(kin, kout);
        std::swap(pin, pout);
    }
    CST_HIP(hipStreamSynchronize(stream));
    *keys_sorted = kin;
    *pay_sorted = pin;
    return CONSTSTN_OK;
}

__device__ __forceinline__ unsigned block_exclusive_scan(unsigned v, unsigned *wtot /*[4]*/) {
    const int lane = threadIdx.x % 64, wave = threadIdx.x / 64;
    unsigned inc = v;
    for (int off = 1; off < 64; off <<= 1) {
        unsigned t = __shfl_up(inc, off, 64);
        if (lane >= off) inc += t;
    }
    if (lane == 63) wtot[wave] = inc;
    __syncthreads();
    unsigned add = 0;
    for (int w = 0; w < wave; ++w) add += wtot[w];
    __syncthreads();
    return add + inc - v;
}

// Rank heads and write the level arrays.  A head at level l is also a head at every deeper
// level, so its child pointer is simply its own rank one level down.  Thread t of a tile takes the
// pairs t, t + 256, ...: every read and write of a wavefront is to neighbouring addresses, the tile's
// keys go through LDS so that each pair sees the one before it, and the values (one read through
// the sorted position per pair, at random) are requested before anything else is done.  A pair's
// rank among the heads of a level is its rank in its wavefront's ballot plus the heads of the
// wavefronts and chunks of 256 before it in the tile.
template <bool WIDE>
__global__ void __launch_bounds__(kTileThreads)
emit_levels_kernel(int64_t nnz, Levels lv, const uint64_t *__restrict__ keys, const uint64_t *__restrict__ keys_hi,
                   const uint32_t *__restrict__ payload, const double *__restrict__ vals_in,
                   const int64_t *__restrict__ tile_offsets, int64_t ntiles, LevelOut out,
                   double *__restrict__ vals_out, int has_dups) {
    static_assert(CONSTSTN_MAX_ORDER * kItems * (kTileThreads / 64) == kTileThreads, "one thread per (level, chunk, wavefront)");
    constexpr int kWaves = kTileThreads / 64, kSlots = kItems * kWaves;
    __shared__ uint64_t lkey[kTile + 1];                       // [0]: the last key of the tile before
    __shared__ uint64_t lkey_hi[WIDE ? kTile + 1 : 1];
    __shared__ unsigned heads[CONSTSTN_MAX_ORDER][kSlots];     // heads of (chunk, wavefront), then those before it in the tile
    const int64_t tile = blockIdx.x, base = tile * kTile;
    const int lane = threadIdx.x % 64, wave = threadIdx.x / 64;
    Key2 k[kItems];
    double v[kItems];
#pragma unroll
    for (int i = 0; i < kItems; ++i) {
        const int m = i * kTileThreads + int(threadIdx.x);
        const int64_t n = base + m;
        k[i] = Key2{0, 0};
        v[i] = 0.0;
        if (n < nnz) {
            k[i] = load_key<WIDE>(keys, keys_hi, n);
            v[i] = vals_in[payload[n]];
        }
        lkey[1 + m] = k[i].lo;
        if (WIDE) lkey_hi[1 + m] = k[i].hi;
    }
    if (threadIdx.x == 0) {
        lkey[0] = base > 0 ? keys[base - 1] : 0;
        if (WIDE) lkey_hi[0] = base > 0 ? keys_hi[base - 1] : 0;
    }
    __syncthreads();
    unsigned headbits[kItems];                       // bit l set: head at level l
#pragma unroll
    for (int i = 0; i < kItems; ++i) {
        const int m = i * kTileThreads + int(threadIdx.x);
        const int64_t n = base + m;
        headbits[i] = 0;
        if (n < nnz) {
            const Key2 prev{WIDE ? lkey_hi[m] : 0, lkey[m]};
            for (int l = 0; l < lv.order; ++l)
                if (n == 0 || !same_prefix<WIDE>(lv, l, k[i], prev)) headbits[i] |= 1u << l;
        }
#pragma unroll
        for (int l = 0; l < CONSTSTN_MAX_ORDER; ++l) {
            const unsigned long long mask = __builtin_amdgcn_ballot_w64((headbits[i] >> l) & 1u);
            if (lane == 0) heads[l][i * kWaves + wave] = unsigned(__popcll(mask));
        }
    }
    __syncthreads();
    {
        // thread (l, slot): exclusive scan over the 32 (chunk, wavefront) slots of level l, in tile order
        const int l = int(threadIdx.x) / kSlots, slot = int(threadIdx.x) % kSlots;
        const unsigned mine = heads[l][slot];
        unsigned inc = mine;
        for (int off = 1; off < kSlots; off <<= 1) {
            const unsigned up = __shfl_up(inc, off, kSlots);
            if (slot >= off) inc += up;
        }
        heads[l][slot] = inc - mine;
    }
    __syncthreads();
    const unsigned long long lt = (1ull << lane) - 1ull;
    const int last = lv.order - 1;
#pragma unroll
    for (int i = 0; i < kItems; ++i) {
        const int64_t n = base + i * kTileThreads + int(threadIdx.x);
        int64_t pos[CONSTSTN_MAX_ORDER];
#pragma unroll
        for (int l = 0; l < CONSTSTN_MAX_ORDER; ++l) {
            const unsigned long long mask = __builtin_amdgcn_ballot_w64((headbits[i] >> l) & 1u);
            pos[l] = l < lv.order ? tile_offsets[int64_t(l) * ntiles + tile] + heads[l][i * kWaves + wave] + __popcll(mask & lt) : 0;
        }
#pragma unroll
        for (int l = 0; l < CONSTSTN_MAX_ORDER; ++l) {
            if (l < lv.order && (headbits[i] & (1u << l))) {
                const uint64_t w = (WIDE && lv.word[l]) ? k[i].hi : k[i].lo;
                out.idx[l][pos[l]] = int32_t((lv.shift[l] >= 64 ? 0 : (w >> lv.shift[l])) & lv.mask[l]);
                if (l < last) out.ptr[l][pos[l]] = pos[l + 1 < CONSTSTN_MAX_ORDER ? l + 1 : l];
                if (l == last) {
                    // leaf head: its value is the sum of the run of equal keys, in input order
                    // (the sort is stable); without duplicates the run has length one
                    double sum = v[i];
                    if (has_dups)
                        for (int64_t m = n + 1; m < nnz && keys[m] == k[i].lo && (!WIDE || keys_hi[m] == k[i].hi); ++m) sum += vals_in[payload[m]];
                    vals_out[pos[l]] = sum;
                }
            }
        }
    }
}

__global__ void close_ptrs_kernel(LevelOut out, int order, const int64_t *totals) {
    const int l = threadIdx.x;
    if (l < order - 1) out.ptr[l][totals[l]] = totals[l + 1];
}

conststn_status build_csf_device(int order, const int64_t *dims, int64_t nnz,
                                 const int32_t *const *coords, const double *vals,
                                 const int *mode_order, unsigned flags, hipStream_t stream,
                                 conststn_csf_s *csf) {
    Levels lv{};
    lv.order = order;
    int total_bits = 0;
    int bits[CONSTSTN_MAX_ORDER];
    for (int l = 0; l < order; ++l) {
        const int m = mode_order[l];
        bits[l] = ceil_log2_u64(uint64_t(dims[m]));
        total_bits += bits[l];
        lv.dim[l] = dims[m];
        lv.coord[l] = coords[m];
    }
    // The innermost levels fill the low word as far as whole fields fit, the others the high word.
    int sh = 0, lo_bits = 0, hi_bits = 0;
    bool in_hi = false;
    for (int l = order - 1; l >= 0; --l) {
        if (!in_hi && sh + bits[l] > 64) { in_hi = true; lo_bits = sh; sh = 0; }
        lv.word[l] = in_hi ? 1 : 0;
        lv.shift[l] = sh;
        lv.mask[l] = bits[l] >= 64 ? ~uint64_t(0) : ((uint64_t(1) << bits[l]) - 1);
        sh += bits[l];
    }
    if (in_hi) hi_bits = sh; else lo_bits = sh;
    const bool wide = in_hi;
    if (hi_bits > 64) {
        set_error("packed coordinate key needs %d bits in fields that do not fit two 64-bit words", total_bits);
        return CONSTSTN_EUNSUPPORTED;
    }

    csf->order = order;
    csf->nnz = nnz;
    for (int l = 0; l < order; ++l) {
        csf->dims[l] = dims[l];
        csf->mode_order[l] = mode_order[l];
    }
    CST_HIP(hipGetDevice(&csf->device));

    LevelOut lo{};
    if (nnz == 0) {
        for (int l = 0; l < order; ++l) {
            csf->nodes[l] = 0;
            CST_TRY(csf->idx[l].alloc(0));
            if (l < order - 1) {
                CST_TRY(csf->ptr[l].alloc(1));
                CST_HIP(hipMemsetAsync(csf->ptr[l].p, 0, sizeof(int64_t), stream));
            }
        }
        CST_TRY(csf->vals.alloc(0));
        CST_HIP(hipStreamSynchronize(stream));
        return CONSTSTN_OK;
    }

    // every temporary of the build in one allocation
    const int64_t ntiles = div_up(nnz, kTile);
    const size_t sort_bytes = radix_sort_scratch_bytes(nnz);
    const size_t arena_bytes = 2 * up256(size_t(nnz) * 8) + 2 * up256(size_t(nnz) * 4) + up256(2 * sizeof(int)) +
                               (wide ? 2 * up256(size_t(nnz) * 8) : 0) + sort_bytes +
                               up256(size_t(ntiles) * order * sizeof(unsigned)) + up256(size_t(ntiles) * order * sizeof(int64_t)) +
                               up256(CONSTSTN_MAX_ORDER * sizeof(int64_t));
    DevBuf<char> arena;
    CST_TRY(arena.alloc(arena_bytes));
    size_t arena_at = 0;
    auto take = [&](size_t bytes) { char *q = arena.p + arena_at; arena_at += up256(bytes); return q; };
    struct { uint64_t *p; } keys_a{reinterpret_cast<uint64_t *>(take(size_t(nnz) * 8))}, keys_b{reinterpret_cast<uint64_t *>(take(size_t(nnz) * 8))};
    struct { uint32_t *p; } pay_a{reinterpret_cast<uint32_t *>(take(size_t(nnz) * 4))}, pay_b{reinterpret_cast<uint32_t *>(take(size_t(nnz) * 4))};
    struct { int *p; } dflags{reinterpret_cast<int *>(take(2 * sizeof(int)))};
    CST_HIP(hipMemsetAsync(dflags.p, 0, 2 * sizeof(int), stream));
    struct { uint64_t *p; } lo_orig{nullptr}, hi_orig{nullptr};      // two-word keys only: the words in input order
    if (wide) {
        lo_orig.p = reinterpret_cast<uint64_t *>(take(size_t(nnz) * 8));
        hi_orig.p = reinterpret_cast<uint64_t *>(take(size_t(nnz) * 8));
    }
    void *sort_scratch = take(sort_bytes);
    {
        const int64_t blocks = std::min<int64_t>(div_up(nnz, 256), 65536);
        pack_keys_kernel<<<dim3(unsigned(blocks)), dim3(256), 0, stream>>>(nnz, lv, wide ? lo_orig.p : keys_a.p,
                                                                          wide ? hi_orig.p : nullptr, pay_a.p, dflags.p);
        CST_HIP(hipGetLastError());
    }

    const uint64_t *skeys = keys_a.p, *skeys_hi = nullptr;
    const uint32_t *spay = pay_a.p;
    if (!wide) {
        CST_TRY(radix_sort_pairs_u64(keys_a.p, keys_b.p, pay_a.p, pay_b.p, nnz, total_bits, stream, &skeys, &spay, sort_scratch));
    } else {
        // least significant word first: sort (low word, position), bring the high words into that order, sort
        // again by the high word (stable), then fetch the low words in the final order
        const unsigned gb = unsigned(div_up(nnz, 256));
        CST_HIP(hipMemcpyAsync(keys_a.p, lo_orig.p, size_t(nnz) * sizeof(uint64_t), hipMemcpyDeviceToDevice, stream));
        CST_TRY(radix_sort_pairs_u64(keys_a.p, keys_b.p, pay_a.p, pay_b.p, nnz, lo_bits, stream, &skeys, &spay, sort_scratch));
        uint64_t *k_free = skeys == keys_a.p ? keys_b.p : keys_a.p, *k_used = skeys == keys_a.p ? keys_a.p : keys_b.p;
        uint32_t *p_used = spay == pay_a.p ? pay_a.p : pay_b.p, *p_free = spay == pay_a.p ? pay_b.p : pay_a.p;
        gather_u64_kernel<<<dim3(gb), dim3(256), 0, stream>>>(nnz, hi_orig.p, p_used, k_free);
        CST_HIP(hipGetLastError());
        const uint64_t *shi = nullptr;
        CST_TRY(radix_sort_pairs_u64(k_free, k_used, p_used, p_free, nnz, hi_bits, stream, &shi, &spay, sort_scratch));
        uint64_t *lo_sorted = shi == k_free ? k_used : k_free;
        gather_u64_kernel<<<dim3(gb), dim3(256), 0, stream>>>(nnz, lo_orig.p, spay, lo_sorted);
        CST_HIP(hipGetLastError());
        skeys = lo_sorted;
        skeys_hi = shi;
    }

    struct { unsigned *p; } tile_counts{reinterpret_cast<unsigned *>(take(size_t(ntiles) * order * sizeof(unsigned)))};
    struct { int64_t *p; } tile_offsets{reinterpret_cast<int64_t *>(take(size_t(ntiles) * order * sizeof(int64_t)))},
        totals{reinterpret_cast<int64_t *>(take(CONSTSTN_MAX_ORDER * sizeof(int64_t)))};
    if (wide)
        count_heads_kernel<true><<<dim3(unsigned(ntiles)), dim3(kTileThreads), 0, stream>>>(
            nnz, lv, skeys, skeys_hi, tile_counts.p, ntiles, dflags.p);
    else
        count_heads_kernel<false><<<dim3(unsigned(ntiles)), dim3(kTileThreads), 0, stream>>>(
            nnz, lv, skeys, nullptr, tile_counts.p, ntiles, dflags.p);
    CST_HIP(hipGetLastError());
    scan_tiles_kernel<<<dim3(unsigned(order)), dim3(1024), 0, stream>>>(tile_counts.p, tile_offsets.p,
                                                                      ntiles, totals.p);
    CST_HIP(hipGetLastError());

    int hflags[2] = {0, 0};
    int64_t htotals[CONSTSTN_MAX_ORDER] = {0};
    CST_HIP(hipMemcpyAsync(hflags, dflags.p, sizeof(hflags), hipMemcpyDeviceToHost, stream));
    CST_HIP(hipMemcpyAsync(htotals, totals.p, sizeof(int64_t) * order, hipMemcpyDeviceToHost, stream));
    CST_HIP(hipStreamSynchronize(stream));
    if (hflags[0]) {
        set_error("a coordinate is negative or not below its mode extent");
        return CONSTSTN_ERANGE;
    }
    if (hflags[1] && !(flags & CONSTSTN_COALESCE_DUPS)) {
        set_error("duplicate coordinate in the input (the nonzero structure must be a set)");
        return CONSTSTN_EDUP;
    }

    for (int l = 0; l < order; ++l) {
        csf->nodes[l] = htotals[l];
        CST_TRY(csf->idx[l].alloc(size_t(htotals[l])));
        lo.idx[l] = csf->idx[l].p;
        if (l < order - 1) {
            CST_TRY(csf->ptr[l].alloc(size_t(htotals[l]) + 1));
            lo.ptr[l] = csf->ptr[l].p;
        }
    }
    CST_TRY(csf->vals.alloc(size_t(htotals[order - 1])));
    csf->nnz = htotals[order - 1];

    if (wide)
        emit_levels_kernel<true><<<dim3(unsigned(ntiles)), dim3(kTileThreads), 0, stream>>>(
            nnz, lv, skeys, skeys_hi, spay, vals, tile_offsets.p, ntiles, lo, csf->vals.p, hflags[1]);
    else
        emit_levels_kernel<false><<<dim3(unsigned(ntiles)), dim3(kTileThreads), 0, stream>>>(
            nnz, lv, skeys, nullptr, spay, vals, tile_offsets.p, ntiles, lo, csf->vals.p, hflags[1]);
    CST_HIP(hipGetLastError());
    close_ptrs_kernel<<<dim3(1), dim3(64), 0, stream>>>(lo, order, totals.p);
    CST_HIP(hipGetLastError());
    CST_HIP(hipStreamSynchronize(stream));
    return CONSTSTN_OK;
}

// ---- a second layout of a tensor that is already a CSF ------------------------------------------
//
// The level order fixes the loop order (Sec. 3.2), and a result indexed by a level other than the root
// would have to be added into from everywhere.  For the order-3 MTTKRP / TTMc of such a mode the plan
// therefore keeps a copy of the tensor with that level at the root: the coordinates are read back
// out of the level arrays (a leaf's ancestors by binary search in the pointer arrays) and sorted again.
__global__ void expand_csf3_kernel(int64_t nnz, int64_t n0, int64_t n1, const int64_t *__restrict__ ptr0,
                                   const int64_t *__restrict__ ptr1, const int32_t *__restrict__ idx0,
                                   const int32_t *__restrict__ idx1, const int32_t *__restrict__ idx2,
                                   int32_t *c0, int32_t *c1, int32_t *c2) {
    const int64_t e = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (e >= nnz) return;
    const int64_t f = parent_of(ptr1, n1, e);
    const int64_t s = parent_of(ptr0, n0, f);
    c0[e] = idx0[s];
    c1[e] = idx1[f];
    c2[e] = idx2[e];
}

conststn_status reroot_csf3(const conststn_csf_s *src, const int new_levels[3], conststn_csf_s *dst) {
    if (src->order != 3) { set_error("only order-3 tensors are re-sorted"); return CONSTSTN_EUNSUPPORTED; }
    const int64_t nnz = src->nnz;
    DevBuf<int32_t> c[3];
    for (int l = 0; l < 3; ++l) CST_TRY(c[l].alloc(size_t(nnz)));
    if (nnz > 0) {
        expand_csf3_kernel<<<dim3(unsigned(div_up(nnz, 256))), dim3(256)>>>(
            nnz, src->nodes[0], src->nodes[1], src->ptr[0].p, src->ptr[1].p, src->idx[0].p, src->idx[1].p,
            src->idx[2].p, c[0].p, c[1].p, c[2].p);
        CST_HIP(hipGetLastError());
    }
    // coordinates by tensor mode, and the new level order in tensor modes
    const int32_t *by_mode[3] = {nullptr, nullptr, nullptr};
    int mode_order[3];
    for (int l = 0; l < 3; ++l) by_mode[src->mode_order[l]] = c[l].p;
    for (int l = 0; l < 3; ++l) mode_order[l] = src->mode_order[new_levels[l]];
    CST_TRY(build_csf_device(3, src->dims, nnz, by_mode, src->vals.p, mode_order, 0, hipStream_t(0), dst));
    CST_HIP(hipDeviceSynchronize());
    return CONSTSTN_OK;
}

}  // namespace cst
