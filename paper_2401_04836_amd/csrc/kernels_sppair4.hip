// Product of two SPARSE order-3 tensors over a shared index with a SPARSE order-4 result (Sec. 5.1,
// the four-index integrals):
//        V[i,j,m,n] = sum_K  Ea[K,i,m] * Eb[K,j,n]
// as the single statement  V[i,j,m,n] = Ea[i,K,m] * Eb[j,K,n]  with loops i,j,K,m,n: the summed index
// in the middle, the two innermost loops fill a dense m x n workspace per (i,j) (the workspace of
// Sec. 2.2's last paragraph), which is then compressed to the stored elements.  Operand layouts:
// Ea as CSF (i > K > m), Eb as CSF (j > K > n); the two may be one tensor under two names.
//
// For one (i,j) the sum over K is a dense contraction: with A = Ea[i] as a (K x m) matrix restricted
// to the m that occur under i, and B = Eb[j] likewise, V[i,j] = A^T . B over the K stored in both.
// It runs on the fp64 matrix cores (v_mfma_f64_16x16x4), the K in chunks staged densely in LDS.
//
//   symbolic (with the plan)  one workgroup per (i,j): co-iterates the two K lists (binary search),
//             and for every shared K marks, for each m of Ea[i,K,:], the n of Eb[j,K,:] in a bit
//             matrix [m of i x n of j] -- the join of Sec. 2.1.  Counts are scanned into the pointer
//             arrays of V (CSF i > j > m > n), a second run lists the m and n (ascending).
//   numeric   one workgroup per stored (i,j): the list of shared K in order, the same bit matrix
//             (it gives every stored element its place), then per chunk of shared K the two dense
//             chunk matrices (double-buffered: the next chunk is fetched during the pass over the
//             current one) and one matrix-core pass over the 16 x 16 tiles of the block, whose
//             accumulators stay in registers; stored elements are written in place.  No atomics on
//             values; the K are visited in ascending order.
#include "plan.hpp"
#include <type_traits>

namespace cst {

constexpr int kP4Waves = 16;                 // wavefronts per workgroup
constexpr int kP4Chunk = 8;                // shared K staged per pass
constexpr int kP4Tiles = 9;                // result tiles a wavefront keeps in registers

typedef double p4_v4d __attribute__((ext_vector_type(4)));
typedef double p4_v2d __attribute__((ext_vector_type(2)));

struct P4Side {                             // one operand: levels (root, K, leaf index)
    const int32_t *idx0, *idx1;
    const int64_t *ptr0, *ptr1;
    const double *vals;
    const int64_t *u_ptr;                   // per root: its distinct leaf indices (ascending) ...
    const int32_t *u_list;
    const uint16_t *slot;                   // ... and every leaf's place among them
    int64_t roots;
    // dense rows (when the plan keeps them): every level-1 node's leaves spread over its root's distinct
    // innermost indices, padded to whole tiles; row_at = first element of the node's row
    const double *dense;
    const int64_t *row_at;
};

struct P4Args {
    P4Side a, b;
    int W;                                  // 32-bit words per row of the bit matrix (n of j)
    int max_ua, max_ub, max_common;
    int mp, np;                             // row strides of the two chunk matrices (doubles)
    int nbuf;                               // chunk buffers per matrix (2; 1 on request)
};

struct P4Out {
    int32_t *idx0, *idx1, *idx2, *idx3;
    int64_t *ptr0, *ptr1, *ptr2;
    int32_t *node_a, *node_b;               // per (i,j) node: root node of Ea, of Eb
    int32_t *root_a;                        // per root of V: root node of Ea
    int64_t roots, pairs, rows, nnz;
    const int32_t *wg_pair;                 // workgroup -> (i,j) node (-1: none), see sppair4_xcd_* below
    int64_t n_wg;
    // kept from the symbolic pass when they fit: per (i,j) node the shared K (level-1 nodes of the two
    // operands, ascending K) and the bit matrix, so that the numeric pass need not find them again
    int64_t *k_ptr;                         // [pairs + 1]
    int64_t *k_a, *k_b;                     // first leaf of the K's row in Ea / Eb (first element of its dense row if dense) ...
    int32_t *k_alen, *k_blen;               // ... and its length
    int dense;                              // the operands' dense rows are kept
    uint32_t *masks;                        // [pairs x mask_stride]
    int64_t mask_stride;
};

__device__ __forceinline__ int64_t p4_find(const int32_t *a, int64_t lo, int64_t hi, int32_t key) {
    while (lo < hi) {
        const int64_t mid = (lo + hi) >> 1;
        const int32_t x = a[mid];
        if (x == key) return mid;
        if (x < key) lo = mid + 1; else hi = mid;
    }
    return -1;
}

__device__ __forceinline__ void p4_wave_sync() {
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// The K stored under both roots, in ascending order: match_a / match_b receive the level-1 nodes.
// Returns the count (the same in every thread).  `scratch` holds one int per wavefront + 1.
template <int WAVES>
__device__ int p4_shared_k(const P4Args &A, int64_t ra, int64_t rb, int32_t *match_a, int32_t *match_b, int cap,
                           int *scratch) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t a0 = A.a.ptr0[ra], a1 = A.a.ptr0[ra + 1];
    const int64_t b0 = A.b.ptr0[rb], b1 = A.b.ptr0[rb + 1];
    int total = 0;
    for (int64_t base = a0; base < a1; base += 64 * WAVES) {
        const int64_t n = base + threadIdx.x;
        int64_t at = -1;
        if (n < a1) at = p4_find(A.b.idx1, b0, b1, A.a.idx1[n]);
        const uint64_t bal = __ballot(at >= 0);
        if (lane == 0) scratch[wave] = __popcll(bal);
        __syncthreads();
        int before = 0, all = 0;
        for (int w = 0; w < WAVES; ++w) { if (w < wave) before += scratch[w]; all += scratch[w]; }
        if (at >= 0) {
            const int pos = total + before + __popcll(bal & ((uint64_t(1) << lane) - 1));
            if (pos < cap) { match_a[pos] = int32_t(n); match_b[pos] = int32_t(at); }
        }
        total += all;
        __syncthreads();
    }
    return total;
}

// Bit matrix of one (i,j): bit (m slot, n slot) set when some shared K stores both.  One wavefront
// per shared K; rows are OR-ed with LDS atomics (the result does not depend on the order).
template <int WAVES>
__device__ void p4_bit_matrix(const P4Args &A, const int32_t *match_a, const int32_t *match_b, int n_shared,
                              int n_ua, uint32_t *rowmask, uint32_t *nmask_all) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int W = A.W;
    uint32_t *nmask = nmask_all + wave * W;
    for (int x = threadIdx.x; x < n_ua * W; x += 64 * WAVES) rowmask[x] = 0;
    __syncthreads();
    for (int k = wave; k < n_shared; k += WAVES) {
        for (int w = lane; w < W; w += 64) nmask[w] = 0;
        p4_wave_sync();
        const int64_t nb = match_b[k], na = match_a[k];
        for (int64_t l = A.b.ptr1[nb] + lane; l < A.b.ptr1[nb + 1]; l += 64) {
            const uint32_t s = A.b.slot[l];
            atomicOr(&nmask[s >> 5], 1u << (s & 31));
        }
        p4_wave_sync();
        for (int64_t l = A.a.ptr1[na] + lane; l < A.a.ptr1[na + 1]; l += 64) {
            const int row = A.a.slot[l];
            for (int w = 0; w < W; ++w) {
                const uint32_t bits = nmask[w];
                if (bits) atomicOr(&rowmask[row * W + w], bits);
            }
        }
        p4_wave_sync();
    }
    __syncthreads();
}

// Per row of the bit matrix: number of set bits -> rowcnt; then (by the first wavefront) the set bits
// before each row -> rowleaf[0..n_ua] and the nonempty rows before each row -> rowrank[0..n_ua].
template <int WAVES>
__device__ void p4_row_offsets(const P4Args &A, const uint32_t *rowmask, int n_ua, int32_t *rowleaf, int32_t *rowrank) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int W = A.W;
    for (int r = threadIdx.x; r < n_ua; r += 64 * WAVES) {
        int c = 0;
        for (int w = 0; w < W; ++w) c += __popc(rowmask[r * W + w]);
        rowleaf[r] = c;
    }
    __syncthreads();
    if (wave == 0) {
        int carry_l = 0, carry_r = 0;
        for (int base = 0; base < n_ua; base += 64) {
            const int r = base + lane;
            const int c = r < n_ua ? rowleaf[r] : 0;
            const int f = c > 0 ? 1 : 0;
            int il = c, ir = f;
            for (int d = 1; d < 64; d <<= 1) {
                const int yl = __shfl_up(il, d, 64), yr = __shfl_up(ir, d, 64);
                if (lane >= d) { il += yl; ir += yr; }
            }
            if (r < n_ua) { rowleaf[r] = carry_l + il - c; rowrank[r] = carry_r + ir - f; }
            carry_l += __shfl(il, 63, 64);
            carry_r += __shfl(ir, 63, 64);
        }
        if (lane == 0) { rowleaf[n_ua] = carry_l; rowrank[n_ua] = carry_r; }
    }
    __syncthreads();
}

// LDS of the symbolic kernels: match lists, bit matrix, per-wavefront n masks, row offsets
struct P4SymLds {
    int match_a, match_b, rowmask, nmask, rowleaf, rowrank, scratch, total;
};

// mode 0: count rows and leaves of every candidate (i,j); mode 1: write them
__global__ void __launch_bounds__(64 * kP4Waves)
sppair4_symbolic_kernel(P4Args A, P4Out V, P4SymLds O, int mode, int64_t *rows, int64_t *leaves, int64_t *shared,
                        const int64_t *__restrict__ k_off, const int64_t *__restrict__ row_off, const int64_t *__restrict__ leaf_off,
                        const int64_t *__restrict__ node_of) {
    extern __shared__ unsigned char lds[];
    int32_t *match_a = reinterpret_cast<int32_t *>(lds + O.match_a), *match_b = reinterpret_cast<int32_t *>(lds + O.match_b);
    uint32_t *rowmask = reinterpret_cast<uint32_t *>(lds + O.rowmask), *nmask = reinterpret_cast<uint32_t *>(lds + O.nmask);
    int32_t *rowleaf = reinterpret_cast<int32_t *>(lds + O.rowleaf), *rowrank = reinterpret_cast<int32_t *>(lds + O.rowrank);
    int *scratch = reinterpret_cast<int *>(lds + O.scratch);
    const int64_t c = blockIdx.x;
    const int64_t ra = c / A.b.roots, rb = c - ra * A.b.roots;
    if (mode == 1 && leaves[c] == 0) return;
    const int n_ua = int(A.a.u_ptr[ra + 1] - A.a.u_ptr[ra]);
    // the lists hold max_common entries, the longest K list of any root of Ea: every shared K fits
    const int n_shared = p4_shared_k<kP4Waves>(A, ra, rb, match_a, match_b, A.max_common, scratch);
    if (n_shared == 0) {
        if (mode == 0 && threadIdx.x == 0) { rows[c] = 0; leaves[c] = 0; shared[c] = 0; }
        return;
    }
    p4_bit_matrix<kP4Waves>(A, match_a, match_b, n_shared, n_ua, rowmask, nmask);
    p4_row_offsets<kP4Waves>(A, rowmask, n_ua, rowleaf, rowrank);
    if (mode == 0) {
        if (threadIdx.x == 0) { rows[c] = rowrank[n_ua]; leaves[c] = rowleaf[n_ua]; shared[c] = rowleaf[n_ua] > 0 ? n_shared : 0; }
        return;
    }
    const int64_t node = node_of[c], r0 = row_off[c], l0 = leaf_off[c];
    if (V.k_ptr) {
        const int64_t k0 = k_off[c];
        if (threadIdx.x == 0) V.k_ptr[node] = k0;
        for (int x = threadIdx.x; x < n_shared; x += 64 * kP4Waves) {
            const int64_t a0 = A.a.ptr1[match_a[x]], b0 = A.b.ptr1[match_b[x]];
            V.k_a[k0 + x] = V.dense ? A.a.row_at[match_a[x]] : a0;
            V.k_alen[k0 + x] = int32_t(A.a.ptr1[match_a[x] + 1] - a0);
            V.k_b[k0 + x] = V.dense ? A.b.row_at[match_b[x]] : b0;
            V.k_blen[k0 + x] = int32_t(A.b.ptr1[match_b[x] + 1] - b0);
        }
        for (int x = threadIdx.x; x < n_ua * A.W; x += 64 * kP4Waves) V.masks[node * V.mask_stride + x] = rowmask[x];
    }
    if (threadIdx.x == 0) {
        V.idx1[node] = A.b.idx0[rb];
        V.ptr1[node] = r0;
        V.node_a[node] = int32_t(ra);
        V.node_b[node] = int32_t(rb);
    }
    const int64_t ua0 = A.a.u_ptr[ra], ub0 = A.b.u_ptr[rb];
    for (int r = threadIdx.x; r < n_ua; r += 64 * kP4Waves) {
        const int cnt = rowleaf[r + 1] - rowleaf[r];
        if (cnt == 0) continue;
        const int64_t row = r0 + rowrank[r];
        V.idx2[row] = A.a.u_list[ua0 + r];
        V.ptr2[row] = l0 + rowleaf[r];
        int64_t at = l0 + rowleaf[r];
        for (int w = 0; w < A.W; ++w) {
            uint32_t word = rowmask[r * A.W + w];
            while (word) {
                V.idx3[at++] = A.b.u_list[ub0 + (w << 5) + __ffs(word) - 1];
                word &= word - 1;
            }
        }
    }
}

__global__ void sppair4_flag_kernel(const int64_t *leaves, int64_t n, int64_t *flag) {
    const int64_t x = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (x < n) flag[x] = leaves[x] > 0 ? 1 : 0;
}

__global__ void sppair4_root_flag_kernel(P4Out V, int64_t *flag) {
    const int64_t n = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (n >= V.pairs) return;
    flag[n] = (n == 0 || V.node_a[n - 1] != V.node_a[n]) ? 1 : 0;
}

__global__ void sppair4_root_fill_kernel(P4Args A, P4Out V, const int64_t *__restrict__ flag,
                                         const int64_t *__restrict__ root_of) {
    const int64_t n = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (n > V.pairs) return;
    if (n == V.pairs) {
        V.ptr0[V.roots] = V.pairs;
        V.ptr1[V.pairs] = V.rows;
        V.ptr2[V.rows] = V.nnz;
        return;
    }
    if (flag[n]) {
        const int64_t r = root_of[n];
        V.idx0[r] = A.a.idx0[V.node_a[n]];
        V.ptr0[r] = n;
        V.root_a[r] = V.node_a[n];
    }
}

// ---- dense rows of an operand -----------------------------------------------------------------
__device__ __forceinline__ int64_t p4_pitch(const P4Side &T, int64_t r) { return (T.u_ptr[r + 1] - T.u_ptr[r] + 15) / 16 * 16; }

__global__ void sppair4_row_size_kernel(P4Side T, int64_t *size) {
    const int64_t r = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (r < T.roots) size[r] = (T.ptr0[r + 1] - T.ptr0[r]) * p4_pitch(T, r);
}

__global__ void sppair4_row_at_kernel(P4Side T, const int64_t *__restrict__ base, int64_t n1, int64_t *row_at) {
    const int64_t nd = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (nd >= n1) return;
    const int64_t r = parent_of(T.ptr0, T.roots, nd);
    row_at[nd] = base[r] + (nd - T.ptr0[r]) * p4_pitch(T, r);
}

// One wavefront per level-1 node: the row is put together in LDS (zeros, then the leaves at their
// places) and written out whole.  `cap` doubles of LDS per wavefront hold the longest row.
constexpr int kP4DenseWaves = 4;
__global__ void __launch_bounds__(64 * kP4DenseWaves)
sppair4_dense_kernel(P4Side T, const int64_t *__restrict__ row_at, int64_t n1, int cap, double *__restrict__ dense) {
    extern __shared__ double p4_rows[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t nd = int64_t(blockIdx.x) * kP4DenseWaves + wave;
    if (nd >= n1) return;
    double *row = p4_rows + size_t(wave) * cap;
    const int64_t r = parent_of(T.ptr0, T.roots, nd);
    const int pitch = int(p4_pitch(T, r));
    for (int x = lane; x < pitch; x += 64) row[x] = 0.0;
    p4_wave_sync();
    for (int64_t l = T.ptr1[nd] + lane; l < T.ptr1[nd + 1]; l += 64) row[T.slot[l]] = T.vals[l];
    p4_wave_sync();
    double *dst = dense + row_at[nd];
    for (int x = lane; x < pitch; x += 64) dst[x] = row[x];
}

// ---- which workgroup takes which (i,j) --------------------------------------------------------
// Workgroups are dealt to the 8 XCDs round-robin, each XCD with an L2 of its own.  In node order
// (i-major) the pairs an XCD works on at one time share a few i but hardly any j, and the dense rows of
// E[j] miss L2 on almost every pair.  Instead XCD x takes the pairs with j % 8 == x, in node order: the
// pairs of neighbouring i then meet the same few j on one XCD.
// Cost of a pair's workgroup in matrix instructions (shared K x tiles of the block), as a key that sorts
// the costliest first: the grid then starts its long workgroups first and fills the tail with short ones.
__global__ void sppair4_cost_key_kernel(P4Args A, P4Out V, uint64_t *keys, uint32_t *pair) {
    const int64_t n = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (n >= V.pairs) return;
    const int64_t ra = V.node_a[n], rb = V.node_b[n];
    const int64_t ta = (A.a.u_ptr[ra + 1] - A.a.u_ptr[ra] + 15) / 16, tb = (A.b.u_ptr[rb + 1] - A.b.u_ptr[rb] + 15) / 16;
    const int64_t shared = V.k_ptr ? V.k_ptr[n + 1] - V.k_ptr[n] : 8;
    const uint64_t cost = uint64_t(ta * tb) * uint64_t((shared + 3) / 4) + uint64_t(ta * tb);      // + write-out
    keys[n] = ~cost & 0xffffffffffull;                    // 40 bits are plenty; ascending sort = falling cost
    pair[n] = uint32_t(n);
}
__global__ void sppair4_order_fill_kernel(int64_t pairs, const uint32_t *__restrict__ sorted, int32_t *wg_pair) {
    const int64_t n = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (n < pairs) wg_pair[n] = int32_t(sorted[n]);
}

__global__ void sppair4_xcd_flag_kernel(P4Out V, int x, int64_t *flag) {
    const int64_t n = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (n < V.pairs) flag[n] = (V.idx1[n] & 7) == x ? 1 : 0;
}
__global__ void sppair4_xcd_fill_kernel(P4Out V, int x, const int64_t *__restrict__ rank, int32_t *wg_pair) {
    const int64_t n = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (n < V.pairs && (V.idx1[n] & 7) == x) wg_pair[8 * rank[n] + x] = int32_t(n);
}
__global__ void sppair4_fill_minus1_kernel(int32_t *p, int64_t n) {
    const int64_t x = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (x < n) p[x] = -1;
}

// LDS of the numeric kernel
struct P4NumLds {
    int match_a, match_b, rowmask, nmask, rowleaf, rowrank, scratch, rowpre, achunk, bchunk, total;
};

// DENSE: the rows of the chunk matrices are copied from the operands' dense rows; otherwise they are
// put together from the leaf lists.
template <bool DENSE>
__global__ void __launch_bounds__(64 * kP4Waves)
sppair4_kernel(P4Args A, P4Out V, P4NumLds O, double *__restrict__ out) {
    extern __shared__ unsigned char lds[];
    int32_t *match_a = reinterpret_cast<int32_t *>(lds + O.match_a), *match_b = reinterpret_cast<int32_t *>(lds + O.match_b);
    uint32_t *rowmask = reinterpret_cast<uint32_t *>(lds + O.rowmask), *nmask = reinterpret_cast<uint32_t *>(lds + O.nmask);
    int32_t *rowleaf = reinterpret_cast<int32_t *>(lds + O.rowleaf), *rowrank = reinterpret_cast<int32_t *>(lds + O.rowrank);
    int *scratch = reinterpret_cast<int *>(lds + O.scratch);
    double *Ac = reinterpret_cast<double *>(lds + O.achunk), *Bc = reinterpret_cast<double *>(lds + O.bchunk);
    int32_t *rowpre = reinterpret_cast<int32_t *>(lds + O.rowpre);
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave: the same in every lane
    const int side = wave & 1, krow = wave >> 1;
    const int nthreads = 64 * kP4Waves;
    const int64_t node = V.wg_pair ? int64_t(V.wg_pair[blockIdx.x]) : int64_t(blockIdx.x);
    if (node < 0) return;                                              // padding of a shorter XCD list
    const int64_t ra = V.node_a[node], rb = V.node_b[node];
    // block-wide values are moved to scalar registers, so that the tests on them cost no vector instructions
    const int n_ua = __builtin_amdgcn_readfirstlane(int(A.a.u_ptr[ra + 1] - A.a.u_ptr[ra]));
    const int n_ub = __builtin_amdgcn_readfirstlane(int(A.b.u_ptr[rb + 1] - A.b.u_ptr[rb]));
    const int64_t leaf0 = V.ptr2[V.ptr1[node]];
    int n_shared;
    const int64_t *k_first = nullptr;       // kept by the plan: leaf range of every shared K, this wavefront's operand
    const int32_t *k_len = nullptr;
    if (V.k_ptr) {
        const int64_t kp = V.k_ptr[node];
        n_shared = int(V.k_ptr[node + 1] - kp);
        k_first = (side ? V.k_b : V.k_a) + kp;
        k_len = (side ? V.k_blen : V.k_alen) + kp;
        for (int x = threadIdx.x; x < n_ua * A.W; x += nthreads) rowmask[x] = V.masks[node * V.mask_stride + x];
        __syncthreads();
    } else {
        n_shared = p4_shared_k<kP4Waves>(A, ra, rb, match_a, match_b, A.max_common, scratch);
        p4_bit_matrix<kP4Waves>(A, match_a, match_b, n_shared, n_ua, rowmask, nmask);
    }
    p4_row_offsets<kP4Waves>(A, rowmask, n_ua, rowleaf, rowrank);
    n_shared = __builtin_amdgcn_readfirstlane(n_shared);
    // position, within the pair's leaves, of the first stored element of every word of the bit matrix
    for (int r = threadIdx.x; r < n_ua; r += nthreads) {
        int at = rowleaf[r];
        for (int w = 0; w < A.W; ++w) {
            rowpre[r * A.W + w] = at;
            at += __popc(rowmask[r * A.W + w]);
        }
    }
    __syncthreads();

    const int tiles_n = (n_ub + 15) >> 4;
    const int li = lane & 15, lk = lane >> 4;
    const int mp = A.mp, np = A.np;
    // Chunks of kP4Chunk shared K, double-buffered: every wavefront owns one row of one of the two chunk
    // matrices (K number wave / 2, operand wave % 2).  During the matrix-core pass over chunk c the leaves
    // of its row of chunk c+1 and the leaf range of its row of chunk c+2 are in flight; the row of chunk
    // c+1 is laid out in the other LDS buffer after the pass.
    static_assert(2 * kP4Chunk == kP4Waves, "one chunk row per wavefront");
    const P4Side &T = side ? A.b : A.a;
    const int32_t *kn = side ? match_b : match_a;
    const int stride = side ? np : mp;
    // Tiles: the 16 wavefronts form a 4 x 4 grid; wavefront (wm, wn) takes the tiles (wm + 4x, wn + 4y),
    // x, y < 3, of a super-block of 12 x 12 tiles, so that per depth step three A and three B operands
    // feed nine matrix-core instructions and the tile origins need no division.
    static_assert(kP4Waves == 16 && kP4Tiles == 9, "4 x 4 wavefronts, 3 x 3 tiles each");
    // (the four wavefronts of one SIMD, wave % 4 equal, get four different rows and columns of the grid:
    // ragged blocks then load the SIMDs evenly)
    const int wm = wave >> 2, wn = (wave + (wave >> 2)) & 3;
    const int tiles_m = (n_ua + 15) >> 4;
    for (int mg = 0; mg < tiles_m; mg += 12)
    for (int ng = 0; ng < tiles_n; ng += 12) {
        // tiles x < nx, y < ny of this wavefront lie inside the block (counts, kept in scalar registers)
        const int nx = max(0, min(3, (tiles_m - mg - wm + 3) >> 2)), ny = max(0, min(3, (tiles_n - ng - wn + 3) >> 2));
        const int shape = __builtin_amdgcn_readfirstlane(nx > 0 && ny > 0 ? 4 * nx + ny : 0);
        const int a_off = lk * mp + 16 * (mg + wm) + li, b_off = lk * np + 16 * (ng + wn) + li;   // tile x lies 64 x further
        int sl[2];                         // leaf lists: the first 128 leaves of the row being fetched
        double vl[2];
        p4_v2d dv[2];                      // dense rows: the row being fetched (at most 256 long), 16 bytes per lane and load
        int64_t r1 = 0, r2 = 0;            // start of this wavefront's row of the next chunk / the one after (-1: none)
        int n1 = 0, n2 = 0;                // ... and their lengths (leaf lists)
        const double *D = side ? A.b.dense : A.a.dense;
        const int pitch = 16 * (side ? tiles_n : tiles_m);
        auto get_range = [&](int k0, int64_t &first, int &len) {
            first = -1;
            len = 0;
            const int k = k0 + krow;
            if (k < n_shared) {
                if (DENSE) first = k_first[k];
                else if (k_first) { first = k_first[k]; len = k_len[k]; }
                else { const int64_t nd = kn[k]; first = T.ptr1[nd]; len = int(T.ptr1[nd + 1] - first); }
            }
        };
        auto get_leaves = [&](int64_t first, int len) {
            if (DENSE) {
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const int x = 128 * h + 2 * lane;                   // rows start at multiples of 16 doubles, x is even
                    dv[h] = (first >= 0 && x < pitch) ? *reinterpret_cast<const p4_v2d *>(D + first + x) : p4_v2d{0.0, 0.0};
                }
            } else {
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const int l = 64 * h + lane;
                    sl[h] = -1;
                    vl[h] = 0.0;
                    if (l < len) { sl[h] = T.slot[first + l]; vl[h] = T.vals[first + l]; }
                }
            }
        };
        auto lay_out = [&](int buf, int64_t first, int len) {
            double *row = (side ? Bc + buf * kP4Chunk * np : Ac + buf * kP4Chunk * mp) + krow * stride;
            if (DENSE) {
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const int x = 128 * h + 2 * lane;
                    if (x < pitch) *reinterpret_cast<p4_v2d *>(row + x) = dv[h];
                }
            } else {
                for (int x = lane; x < stride; x += 64) row[x] = 0.0;
                p4_wave_sync();
#pragma unroll
                for (int h = 0; h < 2; ++h)
                    if (sl[h] >= 0) row[sl[h]] = vl[h];
                for (int l = 128 + lane; l < len; l += 64) row[T.slot[first + l]] = T.vals[first + l];    // rows beyond 128 leaves
            }
        };
        // The pass over the shared K and the write-out, compiled once per shape (CX x CY tiles) of the
        // wavefront's tile set, so that the accumulators stay in fixed registers and no tile is tested
        // inside the loop.  A wavefront without tiles still fetches and lays out its row.
        auto run = [&](auto CX, auto CY) {
            constexpr int cx = decltype(CX)::value, cy = decltype(CY)::value;
            p4_v4d acc[cx ? cx : 1][cy ? cy : 1];
#pragma unroll
            for (int x = 0; x < cx; ++x)
#pragma unroll
                for (int y = 0; y < cy; ++y) acc[x][y] = p4_v4d{0.0, 0.0, 0.0, 0.0};
            __syncthreads();                                           // the buffers of the previous super-block are no longer read
            get_range(0, r1, n1);
            get_range(kP4Chunk, r2, n2);
            get_leaves(r1, n1);
            lay_out(0, r1, n1);
            r1 = r2;
            n1 = n2;
            for (int k0 = 0, c = 0; k0 < n_shared; k0 += kP4Chunk, ++c) {
                const bool more = k0 + kP4Chunk < n_shared;
                if (more) {                                            // fetches touch no LDS: issued ahead of the barrier
                    get_leaves(r1, n1);                                // chunk c+1 (range fetched a pass ago)
                    get_range(k0 + 2 * kP4Chunk, r2, n2);              // chunk c+2
                }
                __syncthreads();                                       // chunk c laid out; chunk c-1 no longer read
                if constexpr (cx > 0 && cy > 0) {
                    const int cb = A.nbuf == 2 ? (c & 1) : 0;
                    const double *Ab = Ac + cb * kP4Chunk * mp + a_off, *Bb = Bc + cb * kP4Chunk * np + b_off;
#pragma unroll
                    for (int kk = 0; kk < kP4Chunk; kk += 4) {
                        double av[cx ? cx : 1], bv[cy ? cy : 1];
#pragma unroll
                        for (int x = 0; x < cx; ++x) av[x] = Ab[kk * mp + 64 * x];
#pragma unroll
                        for (int y = 0; y < cy; ++y) bv[y] = Bb[kk * np + 64 * y];
#pragma unroll
                        for (int x = 0; x < cx; ++x)
#pragma unroll
                            for (int y = 0; y < cy; ++y)
                                acc[x][y] = __builtin_amdgcn_mfma_f64_16x16x4f64(av[x], bv[y], acc[x][y], 0, 0, 0);
                    }
                }
                if (more) {
                    if (A.nbuf == 1) __syncthreads();                  // one buffer: every wavefront is done reading chunk c
                    lay_out(A.nbuf == 2 ? (c + 1) & 1 : 0, r1, n1);
                    r1 = r2;
                    n1 = n2;
                }
            }
            // lane holds V[i,j][m0 + lk + 4v][n0 + li]; stored elements go to their place
#pragma unroll
            for (int x = 0; x < cx; ++x)
#pragma unroll
                for (int y = 0; y < cy; ++y) {
                    const int m0 = 16 * (mg + wm + 4 * x), n = 16 * (ng + wn + 4 * y) + li;
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const int m = m0 + lk + 4 * v;
                        if (m < n_ua && n < n_ub) {
                            const int w = m * A.W + (n >> 5);
                            const uint32_t word = rowmask[w];
                            if ((word >> (n & 31)) & 1u)
                                out[leaf0 + rowpre[w] + __popc(word & ((1u << (n & 31)) - 1u))] = acc[x][y][v];
                        }
                    }
                }
        };
        using std::integral_constant;
        switch (shape) {
            case 5: run(integral_constant<int, 1>{}, integral_constant<int, 1>{}); break;
            case 6: run(integral_constant<int, 1>{}, integral_constant<int, 2>{}); break;
            case 7: run(integral_constant<int, 1>{}, integral_constant<int, 3>{}); break;
            case 9: run(integral_constant<int, 2>{}, integral_constant<int, 1>{}); break;
            case 10: run(integral_constant<int, 2>{}, integral_constant<int, 2>{}); break;
            case 11: run(integral_constant<int, 2>{}, integral_constant<int, 3>{}); break;
            case 13: run(integral_constant<int, 3>{}, integral_constant<int, 1>{}); break;
            case 14: run(integral_constant<int, 3>{}, integral_constant<int, 2>{}); break;
            case 15: run(integral_constant<int, 3>{}, integral_constant<int, 3>{}); break;
            default: run(integral_constant<int, 0>{}, integral_constant<int, 0>{}); break;
        }
    }
}

// ---- host side -------------------------------------------------------------------------------

static inline dim3 p4_grid(int64_t n, int block = 256) { return dim3(unsigned(std::max<int64_t>(1, div_up(n, block)))); }

static void p4_side(const conststn_csf_s *T, const DevBuf<int64_t> &u_ptr, const DevBuf<int32_t> &u_list,
                    const DevBuf<uint16_t> &slot, P4Side &s) {
    s.idx0 = T->idx[0].p; s.idx1 = T->idx[1].p;
    s.ptr0 = T->ptr[0].p; s.ptr1 = T->ptr[1].p;
    s.vals = T->vals.p;
    s.u_ptr = u_ptr.p; s.u_list = u_list.p; s.slot = slot.p;
    s.roots = T->nodes[0];
    s.dense = nullptr; s.row_at = nullptr;
}

static P4Args p4_args(const conststn_plan_s *plan) {
    P4Args A{};
    p4_side(plan->X, plan->p4_ua_ptr, plan->p4_ua_list, plan->p4_a_slot, A.a);
    p4_side(plan->W, plan->p4_ub_ptr, plan->p4_ub_list, plan->p4_b_slot, A.b);
    A.W = plan->p4_words;
    A.max_ua = plan->p4_max_ua;
    A.max_ub = plan->p4_max_ub;
    A.max_common = plan->p4_max_common;
    A.mp = plan->p4_mp;
    A.np = plan->p4_np;
    A.nbuf = plan->p4_nbuf;
    if (plan->p4_dense) {
        const bool same = plan->X == plan->W;                      // one tensor in both places: one set of rows
        A.a.dense = plan->p4_dense_a.p; A.a.row_at = plan->p4_row_at_a.p;
        A.b.dense = same ? plan->p4_dense_a.p : plan->p4_dense_b.p;
        A.b.row_at = same ? plan->p4_row_at_a.p : plan->p4_row_at_b.p;
    }
    return A;
}

static P4Out p4_out(const conststn_plan_s *plan) {
    conststn_csf_s *E = plan->sc_E.get();
    P4Out o{};
    o.idx0 = E->idx[0].p; o.idx1 = E->idx[1].p; o.idx2 = E->idx[2].p; o.idx3 = E->idx[3].p;
    o.ptr0 = E->ptr[0].p; o.ptr1 = E->ptr[1].p; o.ptr2 = E->ptr[2].p;
    o.node_a = plan->p4_node_a.p; o.node_b = plan->p4_node_b.p; o.root_a = plan->p4_root_a.p;
    o.roots = E->nodes[0]; o.pairs = E->nodes[1]; o.rows = E->nodes[2]; o.nnz = E->nodes[3];
    if (plan->p4_stored) {
        o.k_ptr = plan->p4_k_ptr.p; o.k_a = plan->p4_k_a.p; o.k_b = plan->p4_k_b.p;
        o.k_alen = plan->p4_k_alen.p; o.k_blen = plan->p4_k_blen.p;
        o.masks = plan->p4_masks.p;
        o.mask_stride = int64_t(plan->p4_max_ua) * plan->p4_words;
    }
    o.dense = plan->p4_dense ? 1 : 0;
    o.wg_pair = plan->p4_wg_pair.p;
    o.n_wg = plan->p4_n_wg;
    return o;
}

// Places of an operand's dense rows: per root, (its level-1 nodes) x (its distinct innermost indices,
// padded to whole tiles) doubles, roots one after the other.
static conststn_status p4_dense_places(const P4Side &T, int64_t n1, DevBuf<int64_t> &row_at, int64_t *elems) {
    DevBuf<int64_t> size, base;
    *elems = 0;
    if (T.roots == 0 || n1 == 0) return CONSTSTN_OK;
    CST_TRY(size.alloc(size_t(T.roots)));
    CST_TRY(base.alloc(size_t(T.roots)));
    sppair4_row_size_kernel<<<p4_grid(T.roots), 256>>>(T, size.p);
    CST_HIP(hipGetLastError());
    CST_TRY(exscan(size.p, base.p, T.roots, elems));
    CST_TRY(row_at.alloc(size_t(n1)));
    sppair4_row_at_kernel<<<p4_grid(n1), 256>>>(T, base.p, n1, row_at.p);
    CST_HIP(hipGetLastError());
    CST_HIP(hipDeviceSynchronize());
    return CONSTSTN_OK;
}

conststn_status build_sppair4_tables(conststn_plan_s *plan) {
    const conststn_csf_s *Ea = plan->X, *Eb = plan->W;
    const hipStream_t st = nullptr;
    int64_t max_ua = 1, max_ub = 1;
    CST_TRY(csf3_leaf_universe(Ea, plan->p4_ua_ptr, plan->p4_ua_list, plan->p4_a_slot, &max_ua, nullptr));
    CST_TRY(csf3_leaf_universe(Eb, plan->p4_ub_ptr, plan->p4_ub_list, plan->p4_b_slot, &max_ub, nullptr));
    // the longest K list of a root of Ea bounds the K two roots can share
    std::vector<int64_t> hp(size_t(Ea->nodes[0] + 1));
    CST_HIP(hipMemcpy(hp.data(), Ea->ptr[0].p, hp.size() * sizeof(int64_t), hipMemcpyDeviceToHost));
    int64_t max_k = 1;
    for (size_t r = 0; r + 1 < hp.size(); ++r) max_k = std::max(max_k, hp[r + 1] - hp[r]);
    plan->p4_max_ua = int(max_ua);
    plan->p4_max_ub = int(max_ub);
    plan->p4_words = int((max_ub + 31) / 32);
    plan->p4_max_common = int(std::min<int64_t>(max_k, int64_t(1) << 20));
    // chunk matrices: rows padded to whole tiles
    // ... and to an odd number of 16-double units: the four depth rows one matrix-core operand reads
    // then fall into alternating halves of the LDS banks instead of all into the same ones
    plan->p4_mp = int((max_ua + 15) / 16 * 16);
    plan->p4_np = int((max_ub + 15) / 16 * 16);
    if (plan->p4_mp % 32 == 0) plan->p4_mp += 16;
    if (plan->p4_np % 32 == 0) plan->p4_np += 16;
    auto up16 = [](int64_t x) { return (x + 15) / 16 * 16; };
    int64_t at = 0;
    P4NumLds L{};
    L.match_a = int(at); at = up16(at + 4 * int64_t(plan->p4_max_common));
    L.match_b = int(at); at = up16(at + 4 * int64_t(plan->p4_max_common));
    L.rowmask = int(at); at = up16(at + 4 * int64_t(plan->p4_words) * max_ua);
    L.nmask = int(at); at = up16(at + 4 * int64_t(plan->p4_words) * kP4Waves);
    L.rowleaf = int(at); at = up16(at + 4 * (max_ua + 1));
    L.rowrank = int(at); at = up16(at + 4 * (max_ua + 1));
    L.scratch = int(at); at = up16(at + 4 * (kP4Waves + 1));
    const int64_t sym_bytes = at;
    L.rowpre = int(at); at = up16(at + 4 * int64_t(plan->p4_words) * max_ua);
    // Two chunk buffers per matrix overlap the fetch of a chunk with the pass over the one before.  One
    // buffer and a second barrier per chunk (CONSTSTN_SPPAIR4_BUFFERS=1) halve the LDS, which at the
    // lattice workload lets two workgroups share a CU, but measured 5 % slower there.
    plan->p4_nbuf = plan->opt("sppair4_buffers", 2) == 1 ? 1 : 2;
    L.achunk = int(at); at = up16(at + plan->p4_nbuf * 8 * int64_t(kP4Chunk) * plan->p4_mp);
    L.bchunk = int(at); at = up16(at + plan->p4_nbuf * 8 * int64_t(kP4Chunk) * plan->p4_np);
    L.total = int(at);
    if (at > 160 * 1024) {
        set_error("the blocks of one (i,j) pair need %lld bytes of LDS (shared K up to %d, %lld x %lld distinct inner indices)",
                  (long long)at, plan->p4_max_common, (long long)max_ua, (long long)max_ub);
        return CONSTSTN_EUNSUPPORTED;
    }
    const int lay[11] = {L.match_a, L.match_b, L.rowmask, L.nmask, L.rowleaf, L.rowrank, L.scratch, L.rowpre, L.achunk, L.bchunk, L.total};
    plan->p4_layout.assign(lay, lay + 11);
    const P4SymLds S{L.match_a, L.match_b, L.rowmask, L.nmask, L.rowleaf, L.rowrank, L.scratch, int(sym_bytes)};
    CST_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(sppair4_symbolic_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, int(sym_bytes)));
    CST_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(sppair4_kernel<true>), hipFuncAttributeMaxDynamicSharedMemorySize, L.total));
    CST_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(sppair4_kernel<false>), hipFuncAttributeMaxDynamicSharedMemorySize, L.total));

    const int64_t nc = Ea->nodes[0] * Eb->nodes[0];
    if (nc > (int64_t(1) << 28)) { set_error("%lld candidate (i,j) pairs; the symbolic pass holds counters per pair", (long long)nc); return CONSTSTN_EUNSUPPORTED; }
    plan->sc_E.reset(new conststn_csf_s());
    conststn_csf_s *E = plan->sc_E.get();
    E->order = 4;
    E->dims[0] = Ea->dims[Ea->mode_order[0]]; E->dims[1] = Eb->dims[Eb->mode_order[0]];
    E->dims[2] = Ea->dims[Ea->mode_order[2]]; E->dims[3] = Eb->dims[Eb->mode_order[2]];
    for (int l = 0; l < 4; ++l) E->mode_order[l] = l;
    E->device = Ea->device;
    P4Args A = p4_args(plan);
    int64_t pairs = 0, rows = 0, nnz = 0, roots = 0, total_k = 0;
    DevBuf<int64_t> c_rows, c_leaves, c_shared, k_off, row_off, leaf_off, flag, node_of;
    if (nc > 0) {
        CST_TRY(c_rows.alloc(size_t(nc)));
        CST_TRY(c_leaves.alloc(size_t(nc)));
        CST_TRY(c_shared.alloc(size_t(nc)));
        CST_TRY(k_off.alloc(size_t(nc)));
        CST_TRY(row_off.alloc(size_t(nc)));
        CST_TRY(leaf_off.alloc(size_t(nc)));
        CST_TRY(flag.alloc(size_t(nc)));
        CST_TRY(node_of.alloc(size_t(nc)));
        P4Out none{};
        sppair4_symbolic_kernel<<<dim3(unsigned(nc)), 64 * kP4Waves, size_t(sym_bytes), st>>>(A, none, S, 0, c_rows.p, c_leaves.p, c_shared.p, nullptr,
                                                                                           nullptr, nullptr, nullptr);
        CST_HIP(hipGetLastError());
        CST_TRY(exscan(c_rows.p, row_off.p, nc, &rows));
        CST_TRY(exscan(c_leaves.p, leaf_off.p, nc, &nnz));
        sppair4_flag_kernel<<<p4_grid(nc), 256, 0, st>>>(c_leaves.p, nc, flag.p);
        CST_HIP(hipGetLastError());
        CST_TRY(exscan(flag.p, node_of.p, nc, &pairs));
        CST_TRY(exscan(c_shared.p, k_off.p, nc, &total_k));
    }
    // shared K lists and bit matrices are kept for the numeric pass when they are of modest size
    const int64_t mask_words = pairs * int64_t(plan->p4_max_ua) * plan->p4_words;
    plan->p4_stored = (mask_words * 4 + total_k * 24) <= (plan->opt("sppair4_keep_gb", 4) << 30) &&
                      plan->opt("sppair4_keep", 1) == 1;
    if (plan->p4_stored) {
        CST_TRY(plan->p4_k_ptr.alloc(size_t(pairs + 1)));
        CST_TRY(plan->p4_k_a.alloc(size_t(total_k)));
        CST_TRY(plan->p4_k_b.alloc(size_t(total_k)));
        CST_TRY(plan->p4_k_alen.alloc(size_t(total_k)));
        CST_TRY(plan->p4_k_blen.alloc(size_t(total_k)));
        CST_TRY(plan->p4_masks.alloc(size_t(mask_words)));
        CST_HIP(hipMemcpy(plan->p4_k_ptr.p + pairs, &total_k, sizeof(int64_t), hipMemcpyHostToDevice));
    }
    // Dense rows of the operands (rebuilt from the values by every execute) let the numeric pass copy the
    // rows of its chunk matrices instead of putting them together leaf by leaf; a wavefront holds a row of
    // at most 256 in registers while it is in flight.
    plan->p4_dense = false;
    if (plan->p4_stored && max_ua <= 256 && max_ub <= 256 && plan->opt("sppair4_rows", 1) == 1) {
        int64_t ea = 0, eb = 0;
        CST_TRY(p4_dense_places(A.a, Ea->nodes[1], plan->p4_row_at_a, &ea));
        if (Eb != Ea) CST_TRY(p4_dense_places(A.b, Eb->nodes[1], plan->p4_row_at_b, &eb));
        if ((ea + eb) * 8 <= (plan->opt("sppair4_rows_gb", 8) << 30)) {
            CST_TRY(plan->p4_dense_a.alloc(size_t(std::max<int64_t>(ea, 1))));
            if (Eb != Ea) CST_TRY(plan->p4_dense_b.alloc(size_t(std::max<int64_t>(eb, 1))));
            plan->p4_dense = true;
            A = p4_args(plan);
        }
    }
    CST_TRY(E->idx[1].alloc(size_t(pairs)));
    CST_TRY(E->ptr[1].alloc(size_t(pairs + 1)));
    CST_TRY(E->idx[2].alloc(size_t(rows)));
    CST_TRY(E->ptr[2].alloc(size_t(rows + 1)));
    CST_TRY(E->idx[3].alloc(size_t(nnz)));
    CST_TRY(plan->p4_node_a.alloc(size_t(pairs)));
    CST_TRY(plan->p4_node_b.alloc(size_t(pairs)));
    E->nodes[1] = pairs; E->nodes[2] = rows; E->nodes[3] = nnz;
    E->nnz = nnz;
    P4Out O = p4_out(plan);
    if (pairs > 0) {
        sppair4_symbolic_kernel<<<dim3(unsigned(nc)), 64 * kP4Waves, size_t(sym_bytes), st>>>(A, O, S, 1, c_rows.p, c_leaves.p, c_shared.p, k_off.p,
                                                                                           row_off.p, leaf_off.p, node_of.p);
        CST_HIP(hipGetLastError());
    }
    DevBuf<int64_t> rflag, root_of;
    CST_TRY(rflag.alloc(size_t(pairs)));
    CST_TRY(root_of.alloc(size_t(pairs)));
    if (pairs > 0) {
        sppair4_root_flag_kernel<<<p4_grid(pairs), 256, 0, st>>>(O, rflag.p);
        CST_HIP(hipGetLastError());
        CST_TRY(exscan(rflag.p, root_of.p, pairs, &roots));
    }
    CST_TRY(E->idx[0].alloc(size_t(roots)));
    CST_TRY(E->ptr[0].alloc(size_t(roots + 1)));
    CST_TRY(plan->p4_root_a.alloc(size_t(roots)));
    E->nodes[0] = roots;
    O = p4_out(plan);
    sppair4_root_fill_kernel<<<p4_grid(pairs + 1), 256, 0, st>>>(A, O, rflag.p, root_of.p);
    CST_HIP(hipGetLastError());
    CST_HIP(hipStreamSynchronize(st));
    // workgroup order of the numeric pass (pairs < 2^31: a pair holds at least one of the nnz < 2^31 leaves)
    plan->p4_n_wg = 0;
    if (pairs > 0 && plan->opt("sppair4_xcd", 2) == 2) {
        // costliest first (stable: equal costs stay in node order)
        DevBuf<uint64_t> ka, kb;
        DevBuf<uint32_t> pa, pb;
        CST_TRY(ka.alloc(size_t(pairs)));
        CST_TRY(kb.alloc(size_t(pairs)));
        CST_TRY(pa.alloc(size_t(pairs)));
        CST_TRY(pb.alloc(size_t(pairs)));
        sppair4_cost_key_kernel<<<p4_grid(pairs), 256, 0, st>>>(A, O, ka.p, pa.p);
        CST_HIP(hipGetLastError());
        const uint64_t *ks = nullptr;
        const uint32_t *ps = nullptr;
        CST_TRY(radix_sort_pairs_u64(ka.p, kb.p, pa.p, pb.p, pairs, 40, st, &ks, &ps));
        plan->p4_n_wg = pairs;
        CST_TRY(plan->p4_wg_pair.alloc(size_t(pairs)));
        sppair4_order_fill_kernel<<<p4_grid(pairs), 256, 0, st>>>(pairs, ps, plan->p4_wg_pair.p);
        CST_HIP(hipGetLastError());
        CST_HIP(hipStreamSynchronize(st));
    } else if (pairs > 0 && plan->opt("sppair4_xcd", 2) == 1) {
        DevBuf<int64_t> xflag, xrank;
        CST_TRY(xflag.alloc(size_t(pairs)));
        CST_TRY(xrank.alloc(size_t(pairs)));
        int64_t longest = 0;
        for (int x = 0; x < 8; ++x) {                                   // length of the longest XCD list
            int64_t cnt = 0;
            sppair4_xcd_flag_kernel<<<p4_grid(pairs), 256, 0, st>>>(O, x, xflag.p);
            CST_HIP(hipGetLastError());
            CST_TRY(exscan(xflag.p, xrank.p, pairs, &cnt));
            longest = std::max(longest, cnt);
        }
        plan->p4_n_wg = 8 * longest;
        CST_TRY(plan->p4_wg_pair.alloc(size_t(plan->p4_n_wg)));
        sppair4_fill_minus1_kernel<<<p4_grid(plan->p4_n_wg), 256, 0, st>>>(plan->p4_wg_pair.p, plan->p4_n_wg);
        CST_HIP(hipGetLastError());
        for (int x = 0; x < 8; ++x) {
            int64_t cnt = 0;
            sppair4_xcd_flag_kernel<<<p4_grid(pairs), 256, 0, st>>>(O, x, xflag.p);
            CST_HIP(hipGetLastError());
            CST_TRY(exscan(xflag.p, xrank.p, pairs, &cnt));
            sppair4_xcd_fill_kernel<<<p4_grid(pairs), 256, 0, st>>>(O, x, xrank.p, plan->p4_wg_pair.p);
            CST_HIP(hipGetLastError());
        }
        CST_HIP(hipStreamSynchronize(st));
    }
    plan->out_rows = nnz;
    plan->row_elems = 1;
    return CONSTSTN_OK;
}

conststn_status launch_sppair4(const conststn_plan_s *plan, double *out, hipStream_t stream) {
    const P4Args A = p4_args(plan);
    const P4Out O = p4_out(plan);
    if (O.pairs == 0) return CONSTSTN_OK;
    const std::vector<int> &l = plan->p4_layout;
    const P4NumLds L{l[0], l[1], l[2], l[3], l[4], l[5], l[6], l[7], l[8], l[9], l[10]};
    if (plan->p4_dense) {
        const int64_t n1a = plan->X->nodes[1], n1b = plan->W->nodes[1];
        const int cap_a = (plan->p4_max_ua + 15) / 16 * 16, cap_b = (plan->p4_max_ub + 15) / 16 * 16;
        sppair4_dense_kernel<<<p4_grid(n1a, kP4DenseWaves), 64 * kP4DenseWaves, size_t(kP4DenseWaves) * cap_a * 8, stream>>>(
            A.a, A.a.row_at, n1a, cap_a, plan->p4_dense_a.p);
        CST_HIP(hipGetLastError());
        if (plan->W != plan->X) {
            sppair4_dense_kernel<<<p4_grid(n1b, kP4DenseWaves), 64 * kP4DenseWaves, size_t(kP4DenseWaves) * cap_b * 8, stream>>>(
                A.b, A.b.row_at, n1b, cap_b, plan->p4_dense_b.p);
            CST_HIP(hipGetLastError());
        }
    }
    ProfScope prof(plan, stream);
    const unsigned n_wg = unsigned(O.wg_pair ? O.n_wg : O.pairs);
    if (plan->p4_dense) sppair4_kernel<true><<<dim3(n_wg), 64 * kP4Waves, size_t(L.total), stream>>>(A, O, L, out);
    else sppair4_kernel<false><<<dim3(n_wg), 64 * kP4Waves, size_t(L.total), stream>>>(A, O, L, out);
    CST_HIP(hipGetLastError());
    return CONSTSTN_OK;
}

}  // namespace cst
