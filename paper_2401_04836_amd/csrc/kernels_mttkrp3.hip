// Fused order-3 MTTKRP over a CSF tensor (Sec. 5.2):  M[i,r] = sum_{j,k} X[i,j,k] B[j,r] C[k,r].
//
// The schedule is the two-statement tree  T[i,j,r] = X[i,j,k] C[k,r] ; M[i,r] = T[i,j,r] B[j,r]
// fused on the loops i and j, so the intermediate shrinks to one length-R vector per (i,j)
// fiber (the reduced-order dense workspace of Fig. 3b); r is a batch index.
//
// Mapping: the leaf array is cut into equal chunks (partition.hip).  A group of LPR lanes
// owns one chunk and walks it leaf by leaf; each lane keeps two rank entries of the fiber
// vector T and of the slice accumulator in registers.  At a fiber end the group folds
// T * B[j,:] into the accumulator; at a slice end it stores the row (slice wholly inside the
// chunk) or a partial row (slice shared with neighbouring chunks).  A second kernel adds the
// partial rows of shared slices in chunk order, so results are bit-reproducible.
#include "plan.hpp"

namespace cst {

struct MttkrpArgs {
    int64_t nnz, q, n_chunks, slices;
    int R;
    const int64_t *ptr0, *ptr1;
    const int32_t *idx0, *idx1, *idx2;
    const double *vals;
    const int64_t *chunk_fiber;
    const int32_t *chunk_slice;
    const int64_t *slice_leaf;
    const double *B, *C;
    double *out, *partial;
    int compact;
    const int32_t *heavy_slices;
    double *heavy_partial;
    int n_heavy;
    int accumulate;            // add to what `out` already holds (second sub-tensor of the split path)
};

template <bool VEC>
__device__ __forceinline__ void load2(const double *__restrict__ row, int r0, int R, double &x, double &y) {
    if (VEC) {
        const double2 v = *reinterpret_cast<const double2 *>(row + r0);
        x = v.x;
        y = v.y;
    } else {
        x = r0 < R ? row[r0] : 0.0;
        y = r0 + 1 < R ? row[r0 + 1] : 0.0;
    }
}

template <bool VEC>
__device__ __forceinline__ void store2(double *__restrict__ row, int r0, int R, double x, double y) {
    if (VEC) {
        *reinterpret_cast<double2 *>(row + r0) = make_double2(x, y);
    } else {
        if (r0 < R) row[r0] = x;
        if (r0 + 1 < R) row[r0 + 1] = y;
    }
}

template <int LPR, bool VEC>
__global__ void __launch_bounds__(256)
mttkrp3_kernel(MttkrpArgs a) {
    const int64_t gid = (int64_t(blockIdx.x) * 256 + threadIdx.x) / LPR;
    const int gl = threadIdx.x % LPR;
    if (gid >= a.n_chunks) return;
    const int r0 = 2 * gl;
    const int R = a.R;
    if (VEC && r0 >= R) return;
    const int64_t n0 = gid * a.q;
    const int64_t n1 = n0 + a.q < a.nnz ? n0 + a.q : a.nnz;
    int64_t f = a.chunk_fiber[gid];
    int32_t s = a.chunk_slice[gid];
    const int32_t s_first = s;
    int64_t fiber_end = a.ptr1[f + 1];
    if (fiber_end > n1) fiber_end = n1;
    int64_t slice_fend = a.ptr0[s + 1];
    int32_t j = a.idx1[f];
    double t0 = 0.0, t1 = 0.0, acc0 = 0.0, acc1 = 0.0;

    auto emit = [&](int32_t sl, double x, double y) {
        const int64_t lo = a.slice_leaf[sl], hi = a.slice_leaf[sl + 1];
        if (lo >= n0 && hi <= n1) {
            const int64_t row = a.compact ? int64_t(sl) : int64_t(a.idx0[sl]);
            store2<VEC>(a.out + row * R, r0, R, x, y);
        } else {
            const int64_t slot = 2 * gid + (sl == s_first ? 0 : 1);
            store2<VEC>(a.partial + slot * R, r0, R, x, y);
        }
    };
    auto fiber_done = [&](int64_t n) {          // n = position after the fiber's last leaf in this chunk
        double b0, b1;
        load2<VEC>(a.B + int64_t(j) * R, r0, R, b0, b1);
        acc0 = fma(b0, t0, acc0);
        acc1 = fma(b1, t1, acc1);
        t0 = 0.0;
        t1 = 0.0;
        if (n < n1) {
            ++f;
            if (f == slice_fend) {
                emit(s, acc0, acc1);
                acc0 = 0.0;
                acc1 = 0.0;
                ++s;
                slice_fend = a.ptr0[s + 1];
            }
            j = a.idx1[f];
            fiber_end = a.ptr1[f + 1];
            if (fiber_end > n1) fiber_end = n1;
        }
    };

    constexpr int U = 4;
    int64_t n = n0;
    while (n + U <= n1) {
        int32_t kk[U];
        double vv[U], c0[U], c1[U];
#pragma unroll
        for (int u = 0; u < U; ++u) { kk[u] = a.idx2[n + u]; vv[u] = a.vals[n + u]; }
#pragma unroll
        for (int u = 0; u < U; ++u) load2<VEC>(a.C + int64_t(kk[u]) * R, r0, R, c0[u], c1[u]);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            t0 = fma(vv[u], c0[u], t0);
            t1 = fma(vv[u], c1[u], t1);
            ++n;
            if (n == fiber_end) fiber_done(n);
        }
    }
    for (; n < n1;) {
        const int32_t k = a.idx2[n];
        const double v = a.vals[n];
        double c0, c1;
        load2<VEC>(a.C + int64_t(k) * R, r0, R, c0, c1);
        t0 = fma(v, c0, t0);
        t1 = fma(v, c1, t1);
        ++n;
        if (n == fiber_end) fiber_done(n);
    }
    emit(s, acc0, acc1);
}

// ---- rank-32 path ---------------------------------------------------------------------------
//
// Same chunking and the same partial-row protocol as the general kernel, specialised for
// R = 32 (a factor row is 256 B = 16 lanes x 16 B) and restructured around what limits the
// general kernel, the rate of vector-memory instructions per compute unit:
//   * the leaf stream is read 16 entries at a time, one entry per lane of the 16-lane group,
//     and handed round with DPP row broadcasts instead of one broadcast load per leaf;
//   * the stream is the plan's re-encoded copy: a leaf whose factor row is among the most
//     referenced ("hot") rows carries an LDS slot, and the row comes from LDS, where the
//     workgroup staged all hot rows once; power-law index distributions put most references
//     there.  Other rows are fetched from L2/HBM as before;
//   * end-of-fiber / end-of-slice marks travel in the stream, so the child-pointer arrays
//     are not read at all;
//   * workgroups are persistent and loop over chunks, so the staging cost is paid once.
constexpr uint32_t kHotBit = 0x80000000u, kFiberEnd = 0x40000000u, kSliceEnd = 0x20000000u,
                   kRowMask = 0x0fffffffu;

struct MttkrpR32Args {
    MttkrpArgs base;
    const uint32_t *code;
    const int32_t *hot_rows;
    int n_hot;
    int64_t fibers;
};

struct lds_pair { double x, y; };
typedef __attribute__((address_space(3))) lds_pair lds_double2;

template <int T>
__device__ __forceinline__ uint32_t row_bcast(uint32_t x) {
    return uint32_t(__builtin_amdgcn_mov_dpp(int(x), 0x150 + T, 0xf, 0xf, false));
}
template <int T>
__device__ __forceinline__ double row_bcast(double x) {
    const int lo = __builtin_amdgcn_mov_dpp(__double2loint(x), 0x150 + T, 0xf, 0xf, false);
    const int hi = __builtin_amdgcn_mov_dpp(__double2hiint(x), 0x150 + T, 0xf, 0xf, false);
    return __hiloint2double(hi, lo);
}

// Exclusive count, inside each 16-lane row, of the lanes below this one whose flag is set.
__device__ __forceinline__ int row_rank_of_flag(bool flag, int gl, int &row_total) {
    const unsigned long long m = __builtin_amdgcn_ballot_w64(flag);
    const int shift = (threadIdx.x & 48);                 // first lane of this row inside the wave
    const unsigned row = unsigned(m >> shift) & 0xffffu;
    row_total = __popc(row);
    return __popc(row & ((1u << gl) - 1u));
}

// MODE 0: hot and cold leaves mixed in one stream; MODE 1: every leaf is hot (LDS only);
// MODE 2: every leaf is cold (no LDS).  Modes 1 and 2 serve the split path, where the plan has
// separated the tensor into a hot and a cold sub-tensor: the hot pass then issues no gather to
// the vector-memory path for leaf rows and the cold pass issues only fully populated ones.
// The traversal itself, for NT threads (tid = 0 .. NT-1, whole wavefronts) that are the `part`-th of
// `parts` such teams: the teams share the chunks round-robin.  `hot` = the staged hot rows (MODE 0, 1).
template <int NT, int MODE>
__device__ __forceinline__ void mttkrp3_r32_body(const MttkrpR32Args &aa, int tid, int64_t part, int64_t parts,
                                                 const double2 *hot) {
    const MttkrpArgs &a = aa.base;
    const int gl = tid & 15;
    const lds_double2 *hot_lds = (const lds_double2 *)hot;
    const double2 *Cv = reinterpret_cast<const double2 *>(a.C);
    const double2 *Bv = reinterpret_cast<const double2 *>(a.B);
    const int64_t groups = parts * (NT / 16);
    // every lane group of a wave runs the same number of rounds so that the wave-wide ballot
    // and the row broadcasts below always execute with all rows present
    const int64_t rounds = (a.n_chunks + groups - 1) / groups;
    for (int64_t rnd = 0; rnd < rounds; ++rnd) {
        const int64_t c = rnd * groups + part * (NT / 16) + tid / 16;
        const bool live = c < a.n_chunks;
        const int64_t n0 = live ? c * a.q : 0;
        const int64_t n1 = live ? (n0 + a.q < a.nnz ? n0 + a.q : a.nnz) : 0;
        int64_t f = live ? a.chunk_fiber[c] : 0;          // first fiber not yet closed
        int32_t s = live ? a.chunk_slice[c] : 0;
        const int32_t s_first = s;
        double t0 = 0.0, t1 = 0.0, acc0 = 0.0, acc1 = 0.0;
        uint32_t last = kFiberEnd | kSliceEnd;            // marks of the last leaf consumed

        auto emit = [&]() {
            const int64_t lo = a.slice_leaf[s], hi = a.slice_leaf[s + 1];
            double2 *dst;
            if (lo >= n0 && hi <= n1) {
                const int64_t row = a.compact ? int64_t(s) : int64_t(a.idx0[s]);
                dst = reinterpret_cast<double2 *>(a.out + row * 32);
            } else {
                dst = reinterpret_cast<double2 *>(a.partial + (2 * c + (s == s_first ? 0 : 1)) * 32);
            }
            if (a.accumulate && lo >= n0 && hi <= n1) {
                const double2 old = dst[gl];
                acc0 += old.x;
                acc1 += old.y;
            }
            dst[gl] = make_double2(acc0, acc1);
            acc0 = 0.0;
            acc1 = 0.0;
        };
        // The factor row of a leaf comes from LDS (hot) or from global memory (cold).  The two
        // loads target different registers and the LDS one is unconditional (slot 0 for cold
        // leaves): a shared destination would make the global load wait for the LDS read, and
        // the LDS read goes through an explicitly LDS-qualified pointer so that the compiler
        // cannot merge the two into one flat load.
        auto fetch_hot = [&](uint32_t cd) -> double2 {
            if (MODE == 2) return make_double2(0.0, 0.0);
            const uint32_t slot = (MODE == 1 || (cd & kHotBit)) ? (cd & kRowMask) : 0u;
            const lds_double2 *src = hot_lds + (slot * 16 + gl);
            return make_double2(src->x, src->y);
        };
        auto fetch_cold = [&](uint32_t cd) -> double2 {
            double2 r = make_double2(0.0, 0.0);        // only used where the condition holds
            if (MODE == 1) return make_double2(0.0, 0.0);
            if (MODE == 2) return Cv[(cd & kRowMask) * 16u + uint32_t(gl)];
            if (!(cd & kHotBit)) r = Cv[(cd & kRowMask) * 16u + uint32_t(gl)];
            return r;
        };
        auto pick = [&](uint32_t cd, double2 h, double2 g) -> double2 {
            if (MODE == 1) return h;
            if (MODE == 2) return g;
            return (cd & kHotBit) ? h : g;
        };
        // B row of the fiber that ends at this leaf (no load when the leaf ends no fiber)
        auto fetch_b = [&](uint32_t cd, int32_t j) -> double2 {
            double2 r = make_double2(0.0, 0.0);        // only used where the condition holds
            if (cd & kFiberEnd) r = Bv[uint32_t(j) * 16u + uint32_t(gl)];
            return r;
        };
        auto consume = [&](uint32_t cd, double v, double2 cv, double2 bv) {
            t0 = fma(v, cv.x, t0);
            t1 = fma(v, cv.y, t1);
            last = cd;
            if (cd & kFiberEnd) {
                acc0 = fma(bv.x, t0, acc0);
                acc1 = fma(bv.y, t1, acc1);
                t0 = 0.0;
                t1 = 0.0;
                if (cd & kSliceEnd) { emit(); ++s; }
            }
        };

        // Software pipeline over blocks of 16 leaves.  While block b is consumed, the leaf
        // entries of block b+2 and the level-1 indices (j) of the fibers ending in block b+1
        // are already in flight, and every load a block needs is issued before the first wait,
        // so no step waits on a dependent load.
        const int64_t nblocks = (n1 - n0 + 15) / 16;
        auto load_block = [&](int64_t blk, uint32_t &cd, double &vl) {
            cd = 0;
            vl = 0.0;
            const int64_t pos = n0 + blk * 16 + gl;
            if (blk < nblocks && pos < n1) { cd = aa.code[pos]; vl = a.vals[pos]; }
        };
        // j of the fiber closed by this lane's leaf, given the first fiber open at block start
        auto load_j = [&](uint32_t cd, int64_t fbase, int &ends) -> int32_t {
            const bool is_end = (cd & kFiberEnd) != 0;
            const int rank = row_rank_of_flag(is_end, gl, ends);
            int32_t j = 0;
            if (is_end) j = a.idx1[fbase + rank];
            return j;
        };
        uint32_t code_cur, code_nxt, code_n2 = 0;
        double val_cur, val_nxt, val_n2 = 0.0;
        load_block(0, code_cur, val_cur);
        load_block(1, code_nxt, val_nxt);
        int ends_cur = 0, ends_nxt = 0;
        int32_t j_cur = load_j(code_cur, f, ends_cur), j_nxt = 0;
        for (int64_t b = 0; b < nblocks; ++b) {
            const int64_t base = n0 + b * 16;
            load_block(b + 2, code_n2, val_n2);
            j_nxt = load_j(code_nxt, f + ends_cur, ends_nxt);
            if (base + 16 <= n1) {
#define CST_GROUP(T0)                                                                         \
                {                                                                             \
                    const uint32_t c0 = row_bcast<T0 + 0>(code_cur), c1 = row_bcast<T0 + 1>(code_cur), \
                                   c2 = row_bcast<T0 + 2>(code_cur), c3 = row_bcast<T0 + 3>(code_cur); \
                    const double2 h0 = fetch_hot(c0), h1 = fetch_hot(c1), h2 = fetch_hot(c2),  \
                                  h3 = fetch_hot(c3);                                         \
                    const double2 g0 = fetch_cold(c0), g1 = fetch_cold(c1), g2 = fetch_cold(c2), \
                                  g3 = fetch_cold(c3);                                        \
                    const double2 b0 = fetch_b(c0, int32_t(row_bcast<T0 + 0>(uint32_t(j_cur)))), \
                                  b1 = fetch_b(c1, int32_t(row_bcast<T0 + 1>(uint32_t(j_cur)))), \
                                  b2 = fetch_b(c2, int32_t(row_bcast<T0 + 2>(uint32_t(j_cur)))), \
                                  b3 = fetch_b(c3, int32_t(row_bcast<T0 + 3>(uint32_t(j_cur)))); \
                    consume(c0, row_bcast<T0 + 0>(val_cur), pick(c0, h0, g0), b0);            \
                    consume(c1, row_bcast<T0 + 1>(val_cur), pick(c1, h1, g1), b1);            \
                    consume(c2, row_bcast<T0 + 2>(val_cur), pick(c2, h2, g2), b2);            \
                    consume(c3, row_bcast<T0 + 3>(val_cur), pick(c3, h3, g3), b3);            \
                }
                // Eight leaves at a time where the rows come from one place only (the hot or the cold sub-tensor):
                // what a step waits for is the B rows of the fibers that end in it (and the C rows of cold
                // leaves), a trip to L2 each time, so twice as many in flight halve the waits per block.
#define CST_GROUP8(T0)                                                                        \
                {                                                                             \
                    const uint32_t c0 = row_bcast<T0 + 0>(code_cur), c1 = row_bcast<T0 + 1>(code_cur), \
                                   c2 = row_bcast<T0 + 2>(code_cur), c3 = row_bcast<T0 + 3>(code_cur), \
                                   c4 = row_bcast<T0 + 4>(code_cur), c5 = row_bcast<T0 + 5>(code_cur), \
                                   c6 = row_bcast<T0 + 6>(code_cur), c7 = row_bcast<T0 + 7>(code_cur); \
                    const double2 b0 = fetch_b(c0, int32_t(row_bcast<T0 + 0>(uint32_t(j_cur)))), \
                                  b1 = fetch_b(c1, int32_t(row_bcast<T0 + 1>(uint32_t(j_cur)))), \
                                  b2 = fetch_b(c2, int32_t(row_bcast<T0 + 2>(uint32_t(j_cur)))), \
                                  b3 = fetch_b(c3, int32_t(row_bcast<T0 + 3>(uint32_t(j_cur)))), \
                                  b4 = fetch_b(c4, int32_t(row_bcast<T0 + 4>(uint32_t(j_cur)))), \
                                  b5 = fetch_b(c5, int32_t(row_bcast<T0 + 5>(uint32_t(j_cur)))), \
                                  b6 = fetch_b(c6, int32_t(row_bcast<T0 + 6>(uint32_t(j_cur)))), \
                                  b7 = fetch_b(c7, int32_t(row_bcast<T0 + 7>(uint32_t(j_cur)))); \
                    const double2 g0 = fetch_cold(c0), g1 = fetch_cold(c1), g2 = fetch_cold(c2), g3 = fetch_cold(c3), \
                                  g4 = fetch_cold(c4), g5 = fetch_cold(c5), g6 = fetch_cold(c6), g7 = fetch_cold(c7); \
                    const double2 h0 = fetch_hot(c0), h1 = fetch_hot(c1), h2 = fetch_hot(c2), h3 = fetch_hot(c3); \
                    consume(c0, row_bcast<T0 + 0>(val_cur), pick(c0, h0, g0), b0);            \
                    consume(c1, row_bcast<T0 + 1>(val_cur), pick(c1, h1, g1), b1);            \
                    consume(c2, row_bcast<T0 + 2>(val_cur), pick(c2, h2, g2), b2);            \
                    consume(c3, row_bcast<T0 + 3>(val_cur), pick(c3, h3, g3), b3);            \
                    const double2 h4 = fetch_hot(c4), h5 = fetch_hot(c5), h6 = fetch_hot(c6), h7 = fetch_hot(c7); \
                    consume(c4, row_bcast<T0 + 4>(val_cur), pick(c4, h4, g4), b4);            \
                    consume(c5, row_bcast<T0 + 5>(val_cur), pick(c5, h5, g5), b5);            \
                    consume(c6, row_bcast<T0 + 6>(val_cur), pick(c6, h6, g6), b6);            \
                    consume(c7, row_bcast<T0 + 7>(val_cur), pick(c7, h7, g7), b7);            \
                }
                if (MODE != 0) {
                    CST_GROUP8(0)
                    CST_GROUP8(8)
                } else {
                    CST_GROUP(0)
                    CST_GROUP(4)
                    CST_GROUP(8)
                    CST_GROUP(12)
                }
#undef CST_GROUP8
#undef CST_GROUP
            } else {
                // ragged tail of the last chunk: same steps, one leaf at a time, bounds-checked
                const int left = int(n1 - base);
#define CST_ONE(T)                                                                            \
                {                                                                             \
                    const uint32_t cd = row_bcast<T>(code_cur);                               \
                    const double v = row_bcast<T>(val_cur);                                   \
                    const int32_t jj = int32_t(row_bcast<T>(uint32_t(j_cur)));                \
                    if (T < left) consume(cd, v, pick(cd, fetch_hot(cd), fetch_cold(cd)), fetch_b(cd, jj)); \
                }
                CST_ONE(0) CST_ONE(1) CST_ONE(2) CST_ONE(3) CST_ONE(4) CST_ONE(5) CST_ONE(6) CST_ONE(7)
                CST_ONE(8) CST_ONE(9) CST_ONE(10) CST_ONE(11) CST_ONE(12) CST_ONE(13) CST_ONE(14) CST_ONE(15)
#undef CST_ONE
            }
            f += ends_cur;
            code_cur = code_nxt;
            val_cur = val_nxt;
            code_nxt = code_n2;
            val_nxt = val_n2;
            j_cur = j_nxt;
            ends_cur = ends_nxt;
        }
        if (!(last & kFiberEnd)) {                         // the chunk ends inside fiber f
            const double2 bv = Bv[int64_t(a.idx1[f]) * 16 + gl];
            acc0 = fma(bv.x, t0, acc0);
            acc1 = fma(bv.y, t1, acc1);
        }
        if (!(last & kSliceEnd)) emit();
    }
}

template <int BLOCK, int MODE>
__global__ void __launch_bounds__(BLOCK, 4)
mttkrp3_r32_kernel(MttkrpR32Args aa) {
    extern __shared__ double2 hot[];                       // n_hot rows x 16 double2
    if (MODE != 2) {
        for (int e = threadIdx.x; e < aa.n_hot * 16; e += BLOCK)
            hot[e] = reinterpret_cast<const double2 *>(aa.base.C + int64_t(aa.hot_rows[e >> 4]) * 32)[e & 15];
        __syncthreads();
    }
    mttkrp3_r32_body<BLOCK, MODE>(aa, int(threadIdx.x), int64_t(blockIdx.x), int64_t(gridDim.x), hot);
}

// Hot and cold sub-tensor in ONE launch: the first NH wavefronts of every workgroup walk chunks of the
// hot sub-tensor (rows from LDS: vector issue slots and LDS bandwidth), the other NC chunks of the cold
// one (rows from L2 / memory: the vector-memory path), so that the two passes load different units of
// a CU at the same time instead of one after the other.  The two write different buffers (the cold team
// `cold.base.out`), added afterwards: both may own the same output row.
struct MttkrpDualArgs { MttkrpR32Args hot, cold; };

template <int NH, int NC>
__global__ void __launch_bounds__(64 * (NH + NC), 4)
mttkrp3_r32_dual_kernel(MttkrpDualArgs d) {
    extern __shared__ double2 hot[];
    for (int e = threadIdx.x; e < d.hot.n_hot * 16; e += 64 * (NH + NC))
        hot[e] = reinterpret_cast<const double2 *>(d.hot.base.C + int64_t(d.hot.hot_rows[e >> 4]) * 32)[e & 15];
    __syncthreads();
    if (threadIdx.x < 64 * NH) mttkrp3_r32_body<64 * NH, 1>(d.hot, int(threadIdx.x), int64_t(blockIdx.x), int64_t(gridDim.x), hot);
    else mttkrp3_r32_body<64 * NC, 2>(d.cold, int(threadIdx.x) - 64 * NH, int64_t(blockIdx.x), int64_t(gridDim.x), hot);
}

__global__ void __launch_bounds__(256)
mttkrp3_add_kernel(double2 *__restrict__ out, const double2 *__restrict__ add, int64_t n) {
    const int64_t e = int64_t(blockIdx.x) * 256 + threadIdx.x;
    if (e < n) {
        const double2 x = out[e], y = add[e];
        out[e] = make_double2(x.x + y.x, x.y + y.y);
    }
}

// Rows of slices shared by several chunks: add the partial rows in chunk order.
// One block per slice; G lane groups stride over the chunks, then a fixed-order LDS reduction.
template <int LPR>
__device__ __forceinline__ void mttkrp3_fixup_body(const MttkrpArgs &a, int64_t s, double *red) {
    constexpr int G = 256 / LPR;
    const int64_t lo = a.slice_leaf[s], hi = a.slice_leaf[s + 1];
    const int64_t ca = lo / a.q, cb = (hi - 1) / a.q;
    if (ca == cb) return;                           // stored directly by the main kernel
    if (cb - ca >= kHeavySpan) return;              // left to the two-stage kernels below
    const int g = threadIdx.x / LPR, gl = threadIdx.x % LPR;
    const int r0 = 2 * gl, R = a.R;
    double x = 0.0, y = 0.0;
    for (int64_t c = ca + g; c <= cb; c += G) {
        const int64_t slot = 2 * c + ((c == ca && lo != ca * a.q) ? 1 : 0);
        const double *row = a.partial + slot * R;
        if (r0 < R) x += row[r0];
        if (r0 + 1 < R) y += row[r0 + 1];
    }
    red[threadIdx.x * 2] = x;
    red[threadIdx.x * 2 + 1] = y;
    __syncthreads();
    if (g == 0) {
        for (int gg = 1; gg < G; ++gg) {
            x += red[(gg * LPR + gl) * 2];
            y += red[(gg * LPR + gl) * 2 + 1];
        }
        const int64_t row = a.compact ? s : int64_t(a.idx0[s]);
        if (a.accumulate) {
            if (r0 < R) x += a.out[row * R + r0];
            if (r0 + 1 < R) y += a.out[row * R + r0 + 1];
        }
        if (r0 < R) a.out[row * R + r0] = x;
        if (r0 + 1 < R) a.out[row * R + r0 + 1] = y;
    }
}
template <int LPR>
__global__ void __launch_bounds__(256)
mttkrp3_fixup_kernel(MttkrpArgs a) {
    __shared__ double red[256 * 2];
    mttkrp3_fixup_body<LPR>(a, blockIdx.x, red);
}

// Heavy slices (shared by at least kHeavySpan chunks): stage 1 reduces kHeavySegments equal
// segments of the slice's chunk range in parallel, stage 2 adds the segment sums in order.
template <int LPR>
__device__ __forceinline__ void mttkrp3_fixup_heavy_body(const MttkrpArgs &a, int64_t h, int seg, double *red) {
    constexpr int G = 256 / LPR;
    const int64_t s = a.heavy_slices[h];
    const int64_t lo = a.slice_leaf[s], hi = a.slice_leaf[s + 1];
    const int64_t ca = lo / a.q, cb = (hi - 1) / a.q;
    const int64_t n = cb - ca + 1;
    const int64_t c0 = ca + n * seg / kHeavySegments, c1 = ca + n * (seg + 1) / kHeavySegments;
    const int g = threadIdx.x / LPR, gl = threadIdx.x % LPR;
    const int r0 = 2 * gl, R = a.R;
    double x = 0.0, y = 0.0;
    for (int64_t c = c0 + g; c < c1; c += G) {
        const int64_t slot = 2 * c + ((c == ca && lo != ca * a.q) ? 1 : 0);
        const double *row = a.partial + slot * R;
        if (r0 < R) x += row[r0];
        if (r0 + 1 < R) y += row[r0 + 1];
    }
    red[threadIdx.x * 2] = x;
    red[threadIdx.x * 2 + 1] = y;
    __syncthreads();
    if (g == 0) {
        for (int gg = 1; gg < G; ++gg) {
            x += red[(gg * LPR + gl) * 2];
            y += red[(gg * LPR + gl) * 2 + 1];
        }
        double *dst = a.heavy_partial + (h * kHeavySegments + seg) * R;
        if (r0 < R) dst[r0] = x;
        if (r0 + 1 < R) dst[r0 + 1] = y;
    }
}
template <int LPR>
__global__ void __launch_bounds__(256)
mttkrp3_fixup_heavy_kernel(MttkrpArgs a) {
    __shared__ double red[256 * 2];
    mttkrp3_fixup_heavy_body<LPR>(a, blockIdx.x, int(blockIdx.y), red);
}

__device__ __forceinline__ void mttkrp3_fixup_final_body(const MttkrpArgs &a, int64_t h) {
    const int64_t s = a.heavy_slices[h];
    const int r = threadIdx.x;
    if (r >= a.R) return;
    double x = 0.0;
    for (int seg = 0; seg < kHeavySegments; ++seg)
        x += a.heavy_partial[(h * kHeavySegments + seg) * a.R + r];
    const int64_t row = a.compact ? s : int64_t(a.idx0[s]);
    if (a.accumulate) x += a.out[row * a.R + r];
    a.out[row * a.R + r] = x;
}
__global__ void __launch_bounds__(128)
mttkrp3_fixup_final_kernel(MttkrpArgs a) {
    mttkrp3_fixup_final_body(a, blockIdx.x);
}

// The same three passes for two sub-tensors that write different outputs, in one launch each: the
// first blocks take the first sub-tensor's slices (heavy slices), the others the second's.
struct MttkrpPairArgs { MttkrpArgs first, second; };
template <int LPR>
__global__ void __launch_bounds__(256)
mttkrp3_fixup_pair_kernel(MttkrpPairArgs p) {
    __shared__ double red[256 * 2];
    if (int64_t(blockIdx.x) < p.first.slices) mttkrp3_fixup_body<LPR>(p.first, blockIdx.x, red);
    else mttkrp3_fixup_body<LPR>(p.second, int64_t(blockIdx.x) - p.first.slices, red);
}
template <int LPR>
__global__ void __launch_bounds__(256)
mttkrp3_fixup_heavy_pair_kernel(MttkrpPairArgs p) {
    __shared__ double red[256 * 2];
    if (int(blockIdx.x) < p.first.n_heavy) mttkrp3_fixup_heavy_body<LPR>(p.first, blockIdx.x, int(blockIdx.y), red);
    else mttkrp3_fixup_heavy_body<LPR>(p.second, int64_t(blockIdx.x) - p.first.n_heavy, int(blockIdx.y), red);
}
__global__ void __launch_bounds__(128)
mttkrp3_fixup_final_pair_kernel(MttkrpPairArgs p) {
    if (int(blockIdx.x) < p.first.n_heavy) mttkrp3_fixup_final_body(p.first, blockIdx.x);
    else mttkrp3_fixup_final_body(p.second, int64_t(blockIdx.x) - p.first.n_heavy);
}

template <int LPR>
static conststn_status launch_fixup_pair(const MttkrpArgs &a0, const MttkrpArgs &a1, hipStream_t stream) {
    const MttkrpPairArgs p{a0, a1};
    mttkrp3_fixup_pair_kernel<LPR><<<dim3(unsigned(a0.slices + a1.slices)), dim3(256), 0, stream>>>(p);
    CST_HIP(hipGetLastError());
    const int nh = a0.n_heavy + a1.n_heavy;
    if (nh > 0) {
        mttkrp3_fixup_heavy_pair_kernel<LPR><<<dim3(unsigned(nh), kHeavySegments), dim3(256), 0, stream>>>(p);
        CST_HIP(hipGetLastError());
        mttkrp3_fixup_final_pair_kernel<<<dim3(unsigned(nh)), dim3(128), 0, stream>>>(p);
        CST_HIP(hipGetLastError());
    }
    return CONSTSTN_OK;
}

template <int LPR>
static conststn_status launch_fixup(const MttkrpArgs &a, hipStream_t stream) {
    mttkrp3_fixup_kernel<LPR><<<dim3(unsigned(a.slices)), dim3(256), 0, stream>>>(a);
    CST_HIP(hipGetLastError());
    if (a.n_heavy > 0) {
        mttkrp3_fixup_heavy_kernel<LPR><<<dim3(unsigned(a.n_heavy), kHeavySegments), dim3(256), 0, stream>>>(a);
        CST_HIP(hipGetLastError());
        mttkrp3_fixup_final_kernel<<<dim3(unsigned(a.n_heavy)), dim3(128), 0, stream>>>(a);
        CST_HIP(hipGetLastError());
    }
    return CONSTSTN_OK;
}

template <int LPR>
static conststn_status launch_lpr(const conststn_plan_s *plan, const MttkrpArgs &a, bool vec, hipStream_t stream) {
    const int64_t groups_per_block = 256 / LPR;
    const dim3 grid(unsigned(div_up(a.n_chunks, groups_per_block))), block(256);
    {
        ProfScope prof(plan, stream);
        if (vec)
            mttkrp3_kernel<LPR, true><<<grid, block, 0, stream>>>(a);
        else
            mttkrp3_kernel<LPR, false><<<grid, block, 0, stream>>>(a);
    }
    CST_HIP(hipGetLastError());
    return launch_fixup<LPR>(a, stream);
}

// The rank-32 kernels keep the hot factor rows in LDS (256 B per row): the dynamic-LDS limit of the two
// forms that use them is raised when the plan is built.
conststn_status prepare_mttkrp3_launch(conststn_plan_s *plan) {
    if (plan->n_hot <= 0) return CONSTSTN_OK;
    const int lds = plan->n_hot * 256;
    CST_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&mttkrp3_r32_kernel<512, 0>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, lds));
    CST_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&mttkrp3_r32_kernel<512, 1>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, lds));
    const void *dual = nullptr;
    switch (plan->mttkrp_dual) {
        case 44: dual = reinterpret_cast<const void *>(&mttkrp3_r32_dual_kernel<4, 4>); break;
        case 35: dual = reinterpret_cast<const void *>(&mttkrp3_r32_dual_kernel<3, 5>); break;
        case 53: dual = reinterpret_cast<const void *>(&mttkrp3_r32_dual_kernel<5, 3>); break;
        case 88: dual = reinterpret_cast<const void *>(&mttkrp3_r32_dual_kernel<8, 8>); break;
        default: break;
    }
    if (dual) CST_HIP(hipFuncSetAttribute(dual, hipFuncAttributeMaxDynamicSharedMemorySize, lds));
    return CONSTSTN_OK;
}

conststn_status launch_mttkrp3(const conststn_plan_s *plan, const double *const *dense, double *out,
                               hipStream_t stream) {
    const conststn_csf_s *X = plan->X;
    MttkrpArgs a{};
    a.nnz = X->nnz;
    a.q = plan->chunk_q;
    a.n_chunks = plan->n_chunks;
    a.slices = X->nodes[0];
    a.R = plan->rank_of_level[1];
    a.ptr0 = X->ptr[0].p;
    a.ptr1 = X->ptr[1].p;
    a.idx0 = X->idx[0].p;
    a.idx1 = X->idx[1].p;
    a.idx2 = X->idx[2].p;
    a.vals = X->vals.p;
    a.chunk_fiber = plan->chunk_fiber.p;
    a.chunk_slice = plan->chunk_slice.p;
    a.slice_leaf = plan->slice_leaf.p;
    a.B = dense[plan->factor_of_level[1]];
    a.C = dense[plan->factor_of_level[2]];
    a.out = out;
    a.partial = plan->partial.p;
    a.compact = plan->compact ? 1 : 0;
    a.heavy_slices = plan->heavy_slices.p;
    a.heavy_partial = plan->heavy_partial.p;
    a.n_heavy = plan->n_heavy;
    if (!plan->compact && a.slices < plan->out_rows)        // rows of empty slices are zero
        CST_TRY(zero_fill(out, plan->out_rows * plan->row_elems, stream));
    if (a.nnz == 0) return CONSTSTN_OK;
    const int R = a.R;
    const bool aligned = (reinterpret_cast<uintptr_t>(a.B) % 16 == 0) && (reinterpret_cast<uintptr_t>(a.C) % 16 == 0) &&
                         (reinterpret_cast<uintptr_t>(out) % 16 == 0);
    if (R > 128) { set_error("MTTKRP rank %d above 128 is not implemented", R); return CONSTSTN_EUNSUPPORTED; }
    if (R == 32 && aligned && plan->n_hot > 0 && plan->leaf_code.p) {
        const int cus = plan->n_cus;
        const size_t lds = size_t(plan->n_hot) * 256;
        auto run = [&](const MttkrpR32Args &aa, int mode) -> conststn_status {
            const size_t l = mode == 2 ? 0 : lds;
            const int per_cu = mode == 2 ? 4 : std::max<int>(1, std::min<int>(int(160 * 1024 / std::max<size_t>(l, 1)), 4));
            const int64_t wgs = std::min<int64_t>(div_up(aa.base.n_chunks, 32), int64_t(cus) * per_cu);
            const dim3 grid(unsigned(std::max<int64_t>(wgs, 1))), block(512);
            if (mode == 0) {
                mttkrp3_r32_kernel<512, 0><<<grid, block, l, stream>>>(aa);
            } else if (mode == 1) {
                mttkrp3_r32_kernel<512, 1><<<grid, block, l, stream>>>(aa);
            } else {
                mttkrp3_r32_kernel<512, 2><<<grid, block, 0, stream>>>(aa);
            }
            CST_HIP(hipGetLastError());
            return CONSTSTN_OK;
        };
        if (plan->split) {
            // X = X_hot + X_cold: the hot sub-tensor writes the output, the cold one adds to it
            CST_TRY(zero_fill(out, plan->out_rows * plan->row_elems, stream));
            MttkrpR32Args pa[2];
            for (int part = 0; part < 2; ++part) {
                const MttkrpPart &P = plan->part[part];
                MttkrpR32Args &aa = pa[part];
                aa = MttkrpR32Args{};
                aa.base = a;
                aa.base.nnz = P.nnz;
                aa.base.q = P.chunk_q;
                aa.base.n_chunks = P.n_chunks;
                aa.base.slices = P.slices;
                aa.base.ptr0 = P.ptr0.p;
                aa.base.ptr1 = P.ptr1.p;
                aa.base.idx0 = P.row_of_slice.p;
                aa.base.idx1 = P.idx1.p;
                aa.base.idx2 = nullptr;
                aa.base.vals = P.vals.p;
                aa.base.chunk_fiber = P.chunk_fiber.p;
                aa.base.chunk_slice = P.chunk_slice.p;
                aa.base.slice_leaf = P.slice_leaf.p;
                aa.base.partial = P.partial.p;
                aa.base.compact = 0;                      // row_of_slice already maps to output rows
                aa.base.heavy_slices = P.heavy_slices.p;
                aa.base.heavy_partial = P.heavy_partial.p;
                aa.base.n_heavy = P.n_heavy;
                aa.base.accumulate = 1;                   // every writer adds to the zero-filled output
                aa.code = P.code.p;
                aa.hot_rows = plan->hot_rows.p;
                aa.n_hot = plan->n_hot;
                aa.fibers = P.fibers;
            }
            if (plan->mttkrp_dual && plan->part[0].nnz > 0 && plan->part[1].nnz > 0) {
                // one launch for both sub-tensors; the cold team writes its own buffer
                const int64_t n = plan->out_rows * plan->row_elems;
                CST_TRY(zero_fill(plan->mttkrp_out2.p, n, stream));
                pa[1].base.out = plan->mttkrp_out2.p;
                MttkrpDualArgs d{pa[0], pa[1]};
                // wavefronts per workgroup, and as many workgroups per CU as its LDS and its registers (96 per
                // lane: five wavefronts per SIMD) hold
                const int waves = plan->mttkrp_dual / 10 + plan->mttkrp_dual % 10;
                const int per_cu = std::max(1, std::min(int(160 * 1024 / lds), 20 / waves));
                const dim3 grid(unsigned(cus * per_cu)), block(unsigned(64 * waves));
                {
                    ProfScope prof(plan, stream);
                    switch (plan->mttkrp_dual) {
                        case 44: mttkrp3_r32_dual_kernel<4, 4><<<grid, block, lds, stream>>>(d); break;
                        case 35: mttkrp3_r32_dual_kernel<3, 5><<<grid, block, lds, stream>>>(d); break;
                        case 53: mttkrp3_r32_dual_kernel<5, 3><<<grid, block, lds, stream>>>(d); break;
                        default: mttkrp3_r32_dual_kernel<8, 8><<<grid, block, lds, stream>>>(d); break;
                    }
                    CST_HIP(hipGetLastError());
                }
                CST_TRY(launch_fixup_pair<16>(pa[0].base, pa[1].base, stream));      // different outputs: no order between them
                mttkrp3_add_kernel<<<dim3(unsigned(div_up(n / 2, 256))), dim3(256), 0, stream>>>(
                    reinterpret_cast<double2 *>(out), reinterpret_cast<const double2 *>(plan->mttkrp_out2.p), n / 2);
                CST_HIP(hipGetLastError());
                return CONSTSTN_OK;
            }
            {
                ProfScope prof(plan, stream);             // the two traversal kernels, back to back
                if (plan->part[0].nnz > 0) CST_TRY(run(pa[0], 1));
                if (plan->part[1].nnz > 0) CST_TRY(run(pa[1], 2));
            }
            for (int part = 0; part < 2; ++part)
                if (plan->part[part].nnz > 0) CST_TRY(launch_fixup<16>(pa[part].base, stream));
            return CONSTSTN_OK;
        }
        MttkrpR32Args aa{};
        aa.base = a;
        aa.code = plan->leaf_code.p;
        aa.hot_rows = plan->hot_rows.p;
        aa.n_hot = plan->n_hot;
        aa.fibers = X->nodes[1];
        {
            ProfScope prof(plan, stream);
            CST_TRY(run(aa, 0));
        }
        return launch_fixup<16>(a, stream);
    }
    // smallest power-of-two lane group covering ceil(R/2) lanes; 16-byte accesses when every
    // lane of the group holds two valid, aligned entries
    int lpr = 1;
    while (2 * lpr < R) lpr *= 2;
    const bool vec = aligned && (R % 2 == 0);
    switch (lpr) {
        case 1: return launch_lpr<1>(plan, a, vec, stream);
        case 2: return launch_lpr<2>(plan, a, vec, stream);
        case 4: return launch_lpr<4>(plan, a, vec, stream);
        case 8: return launch_lpr<8>(plan, a, vec, stream);
        case 16: return launch_lpr<16>(plan, a, vec, stream);
        case 32: return launch_lpr<32>(plan, a, vec, stream);
        default: return launch_lpr<64>(plan, a, vec, stream);
    }
}

}  // namespace cst
