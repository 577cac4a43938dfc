// Chain of three SPARSE tensors with a SPARSE result (Sec. 5.1):
//        E[K,i,m] = sum_{u,v} I[K,u,v] * C[u,i] * P[v,m]                  (unrestricted form)
//        E[K,i,m] = sum_{u,v} I[K,u,v] * C[u,i] * P[v,m] * L[K,i]         (restricted form)
// as the fused tree  T[K,i,v] = I[K,u,v] * C[i,u]  (loops K,i,u,v);  E[K,i,m] = T[K,i,v] * P[m,v]
// (loops K,i,m,v), fused on (K,i): the intermediate shrinks to a vector over v (Sec. 2.2), which is
// the dense workspace of Sec. 2.2's last paragraph -- here compressed to the v that occur under K.
// Operand layouts: I as CSF (K > u > v), C as CSF (i > u), P as CSF (m > v), L as CSF (K > i).
//
// The structure of E does not depend on the values, so it is found once, when the plan is made
// (symbolic pass), and every execute only fills the values (numeric pass):
//
//   symbolic  one wavefront per candidate (K,i) pair -- every pair of a K of I with an i of C,
//             or the stored pairs of L -- intersects the u lists of I[K] and C[i] (co-iteration
//             by binary search), marks the v below the matching u in a bit set, then the m that P
//             joins to those v (through a transposed copy of P) in a second bit set.  Counts are
//             scanned into the pointer arrays of E (CSF K > i > m) and a second run writes the m.
//   numeric   one workgroup per K of E.  A table v -> slot (position of v among the distinct v
//             under K) sits in LDS.  Each wavefront takes (K,i) nodes in turn: clears its
//             workspace t[slot], adds I[K,u,v]*C[i,u] row by row for the matching u (lanes over
//             v: no two lanes meet in one slot, rows in ascending u: a fixed summation order),
//             then every lane owns one stored m of E[K,i,:] and gathers
//             sum_v t[slot(v)] * P[m,v] along P's row, and stores the value in place.
//             No atomics; the result is bit-reproducible.
//   numeric, block-local form.  The sparse maps of Sec. 5.1 are local: under one K only a few
//             u, v and m occur, and the blocks  I_K [u rows of K x v slots of K],
//             C_K [(K,i) nodes x u rows of K]  and  P_K [v slots of K x m of K]  are small and
//             fairly dense.  The whole slice then is two dense products,
//             T_K = C_K . I_K  and  E_K = T_K . P_K,  of which only the stored (node, m) elements
//             are kept: a dense contraction, run on the fp64 matrix cores.  I_K, C_K and T_K live
//             in LDS; P_K depends on the lists of v and m only, so it is prepared with the plan,
//             once per run of K that share both lists, and read from memory.  The extra terms are
//             exact zeros.  Chosen by the plan when every K fits LDS; otherwise the general form.
#include "plan.hpp"

namespace cst {

constexpr int kScWaves = 4;                 // wavefronts per workgroup
constexpr uint16_t kNoSlot = 0xFFFF;

struct ScArgs {
    // I: levels (K,u,v)
    const int32_t *i_idx0, *i_idx1;
    const int64_t *i_ptr0, *i_ptr1;
    const double *i_vals;
    int64_t i_roots;
    // C: levels (i,u)
    const int32_t *c_idx0, *c_idx1;
    const int64_t *c_ptr0;
    const double *c_vals;
    int64_t c_roots;
    // P: levels (m,v), and which root node holds m
    const int32_t *p_idx1;
    const int64_t *p_ptr0;
    const double *p_vals;
    const int32_t *p_node_of_m;
    // P transposed, levels (v,m), and which of its root nodes holds v (symbolic pass only)
    const int32_t *pt_idx1;
    const int64_t *pt_ptr0;
    const int32_t *pt_node_of_v;
    // distinct v under each K node of I, ascending; slot of every leaf of I in that list
    const int64_t *nu_ptr;
    const int32_t *nu_list;
    const uint16_t *i_slot;
    int64_t n_v, n_m;
    int max_slots;
    // candidate (K,i) pairs: all of them (restricted = 0) or the leaves of L
    int64_t n_cand;
    int restricted;
    const int32_t *l_knode, *l_cnode;       // node of I / of C per leaf of L, -1 where absent
    const double *l_vals;
    // block-local form: the m that occur under each root of E, ascending
    const int64_t *mu_ptr;
    const int32_t *mu_list;
    int64_t n_u;
};

// the result's structure and, per (K,i) node, where its operands are
struct ScOut {
    int32_t *idx0, *idx1, *idx2;
    int64_t *ptr0, *ptr1;
    int32_t *knode, *cnode;                 // per level-1 node: K node of I, root node of C
    double *lval;                           // per level-1 node: value of L, or 1
    int32_t *root_knode;                    // per root: K node of I
    int64_t roots, nodes, nnz;
};

__device__ __forceinline__ void wave_sync() {
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

__device__ __forceinline__ int wave_sum(int x) {
    for (int d = 32; d >= 1; d >>= 1) x += __shfl_xor(x, d, 64);
    return x;
}

// position of `key` in the ascending list a[lo..hi), or -1
__device__ __forceinline__ int64_t find_in(const int32_t *a, int64_t lo, int64_t hi, int32_t key) {
    while (lo < hi) {
        const int64_t mid = (lo + hi) >> 1;
        const int32_t x = a[mid];
        if (x == key) return mid;
        if (x < key) lo = mid + 1; else hi = mid;
    }
    return -1;
}

__device__ __forceinline__ void decode_candidate(const ScArgs &A, int64_t c, int64_t &a, int64_t &b) {
    if (A.restricted) { a = A.l_knode[c]; b = A.l_cnode[c]; }
    else { a = c / A.c_roots; b = c - a * A.c_roots; }
}

// Bit sets of one (K node a, C root b) pair: slots of the v reached through a matching u, then
// the m joined to those v.  Returns false (sets undefined) when no u matches.
__device__ bool pair_sets(const ScArgs &A, int64_t a, int64_t b, uint32_t *smask, uint32_t *mmask, int lane) {
    const int sw = (A.max_slots + 31) >> 5, mw = int((A.n_m + 31) >> 5);
    for (int w = lane; w < sw; w += 64) smask[w] = 0;
    wave_sync();
    const int64_t n0 = A.i_ptr0[a], n1 = A.i_ptr0[a + 1];
    const int64_t c0 = A.c_ptr0[b], c1 = A.c_ptr0[b + 1];
    bool any = false;
    for (int64_t base = n0; base < n1; base += 64) {
        const int64_t n = base + lane;
        bool hit = false;
        if (n < n1) hit = find_in(A.c_idx1, c0, c1, A.i_idx1[n]) >= 0;
        uint64_t bal = __ballot(hit);
        any = any || bal != 0;
        while (bal) {
            const int bit = __ffsll((unsigned long long)bal) - 1;
            bal &= bal - 1;
            const int64_t l0 = A.i_ptr1[base + bit], l1 = A.i_ptr1[base + bit + 1];
            for (int64_t l = l0 + lane; l < l1; l += 64) {
                const uint32_t s = A.i_slot[l];
                atomicOr(&smask[s >> 5], 1u << (s & 31));
            }
        }
    }
    if (!any) return false;
    for (int w = lane; w < mw; w += 64) mmask[w] = 0;
    wave_sync();
    const int64_t nu0 = A.nu_ptr[a];
    for (int w = 0; w < sw; ++w) {
        uint32_t word = smask[w];                                   // the same word in every lane
        while (word) {
            const int s = (w << 5) + __ffs(word) - 1;
            word &= word - 1;
            const int32_t pn = A.pt_node_of_v[A.nu_list[nu0 + s]];
            if (pn < 0) continue;
            const int64_t q0 = A.pt_ptr0[pn], q1 = A.pt_ptr0[pn + 1];
            for (int64_t q = q0 + lane; q < q1; q += 64) {
                const uint32_t m = uint32_t(A.pt_idx1[q]);
                atomicOr(&mmask[m >> 5], 1u << (m & 31));
            }
        }
    }
    wave_sync();
    return true;
}

__global__ void __launch_bounds__(64 * kScWaves)
spchain3_count_kernel(ScArgs A, int64_t *count) {
    extern __shared__ uint32_t sets[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int sw = (A.max_slots + 31) >> 5, mw = int((A.n_m + 31) >> 5);
    uint32_t *smask = sets + size_t(wave) * (sw + mw), *mmask = smask + sw;
    const int64_t c = int64_t(blockIdx.x) * kScWaves + wave;
    if (c >= A.n_cand) return;
    int64_t a, b;
    decode_candidate(A, c, a, b);
    int total = 0;
    if (a >= 0 && b >= 0 && pair_sets(A, a, b, smask, mmask, lane)) {
        int n = 0;
        for (int w = lane; w < mw; w += 64) n += __popc(mmask[w]);
        total = wave_sum(n);
    }
    if (lane == 0) count[c] = total;
}

__global__ void __launch_bounds__(64 * kScWaves)
spchain3_fill_kernel(ScArgs A, ScOut E, const int64_t *__restrict__ count, const int64_t *__restrict__ leaf_off,
                     const int64_t *__restrict__ node_of) {
    extern __shared__ uint32_t sets[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int sw = (A.max_slots + 31) >> 5, mw = int((A.n_m + 31) >> 5);
    uint32_t *smask = sets + size_t(wave) * (sw + mw), *mmask = smask + sw;
    const int64_t c = int64_t(blockIdx.x) * kScWaves + wave;
    if (c >= A.n_cand || count[c] == 0) return;
    int64_t a, b;
    decode_candidate(A, c, a, b);
    pair_sets(A, a, b, smask, mmask, lane);
    const int64_t node = node_of[c];
    int64_t off = leaf_off[c];
    if (lane == 0) {
        E.idx1[node] = A.c_idx0[b];
        E.ptr1[node] = off;
        E.knode[node] = int32_t(a);
        E.cnode[node] = int32_t(b);
        E.lval[node] = A.restricted ? A.l_vals[c] : 1.0;
    }
    for (int wb = 0; wb < mw; wb += 64) {
        const int w = wb + lane;
        uint32_t word = w < mw ? mmask[w] : 0u;
        const int n = __popc(word);
        int incl = n;                                               // inclusive scan over the lanes
        for (int d = 1; d < 64; d <<= 1) {
            const int y = __shfl_up(incl, d, 64);
            if (lane >= d) incl += y;
        }
        int64_t at = off + incl - n;
        while (word) {
            E.idx2[at++] = (w << 5) + __ffs(word) - 1;
            word &= word - 1;
        }
        off += __shfl(incl, 63, 64);
    }
}

// roots of E: the K nodes that own at least one (K,i) node
__global__ void spchain3_root_flag_kernel(ScOut E, int64_t *flag) {
    const int64_t n = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (n >= E.nodes) return;
    flag[n] = (n == 0 || E.knode[n - 1] != E.knode[n]) ? 1 : 0;
}

__global__ void spchain3_root_fill_kernel(ScArgs A, ScOut E, const int64_t *__restrict__ flag,
                                          const int64_t *__restrict__ root_of) {
    const int64_t n = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (n > E.nodes) return;
    if (n == E.nodes) {
        E.ptr0[E.roots] = E.nodes;
        E.ptr1[E.nodes] = E.nnz;
        return;
    }
    if (flag[n]) {
        const int64_t r = root_of[n];
        E.idx0[r] = A.i_idx0[E.knode[n]];
        E.ptr0[r] = n;
        E.root_knode[r] = E.knode[n];
    }
}

__global__ void __launch_bounds__(64 * kScWaves)
spchain3_kernel(ScArgs A, ScOut E, double *__restrict__ out, int map_bytes) {
    extern __shared__ unsigned char lds[];
    uint16_t *map = reinterpret_cast<uint16_t *>(lds);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    double *t = reinterpret_cast<double *>(lds + map_bytes) + size_t(wave) * A.max_slots;
    const int64_t r = blockIdx.x;
    const int64_t a = E.root_knode[r];
    const int64_t nu0 = A.nu_ptr[a];
    const int ns = int(A.nu_ptr[a + 1] - nu0);
    for (int64_t x = threadIdx.x; x < (A.n_v + 1) / 2; x += blockDim.x) reinterpret_cast<uint32_t *>(map)[x] = 0xFFFFFFFFu;
    __syncthreads();
    for (int s = threadIdx.x; s < ns; s += blockDim.x) map[A.nu_list[nu0 + s]] = uint16_t(s);
    __syncthreads();
    const int64_t n0 = A.i_ptr0[a], n1 = A.i_ptr0[a + 1];
    for (int64_t node = E.ptr0[r] + wave; node < E.ptr0[r + 1]; node += kScWaves) {
        for (int s = lane; s < ns; s += 64) t[s] = 0.0;
        wave_sync();
        const int64_t b = E.cnode[node];
        const int64_t c0 = A.c_ptr0[b], c1 = A.c_ptr0[b + 1];
        // producer: t[v] += I[K,u,v] * C[i,u] over the u stored in both
        for (int64_t base = n0; base < n1; base += 64) {
            const int64_t n = base + lane;
            int64_t pos = -1;
            if (n < n1) pos = find_in(A.c_idx1, c0, c1, A.i_idx1[n]);
            const double cv = pos >= 0 ? A.c_vals[pos] : 0.0;
            uint64_t bal = __ballot(pos >= 0);
            while (bal) {
                const int bit = __ffsll((unsigned long long)bal) - 1;
                bal &= bal - 1;
                const double c = __shfl(cv, bit, 64);
                const int64_t l0 = A.i_ptr1[base + bit], l1 = A.i_ptr1[base + bit + 1];
                for (int64_t l = l0 + lane; l < l1; l += 64) {
                    const int s = A.i_slot[l];
                    t[s] = fma(A.i_vals[l], c, t[s]);
                }
                wave_sync();
            }
        }
        // consumer: E[K,i,m] = sum_v t[v] * P[m,v], one stored m per lane
        const double lv = E.lval[node];
        for (int64_t q = E.ptr1[node] + lane; q < E.ptr1[node + 1]; q += 64) {
            const int32_t pn = A.p_node_of_m[E.idx2[q]];
            double acc = 0.0;
            for (int64_t p = A.p_ptr0[pn]; p < A.p_ptr0[pn + 1]; ++p) {
                const uint16_t s = map[A.p_idx1[p]];
                if (s != kNoSlot) acc = fma(t[s], A.p_vals[p], acc);
            }
            out[q] = acc * lv;
        }
        wave_sync();
    }
}

// The m that occur anywhere under one root of E: mode 0 counts them, mode 1 lists them (ascending).
__global__ void __launch_bounds__(256)
spchain3_root_mset_kernel(ScOut E, int64_t n_m, int mode, int64_t *count, const int64_t *__restrict__ off, int32_t *list) {
    extern __shared__ uint32_t mset[];
    __shared__ int wave_tot[4];
    const int mw = int((n_m + 31) >> 5);
    const int64_t r = blockIdx.x;
    for (int w = threadIdx.x; w < mw; w += 256) mset[w] = 0;
    __syncthreads();
    const int64_t q0 = E.ptr1[E.ptr0[r]], q1 = E.ptr1[E.ptr0[r + 1]];
    for (int64_t q = q0 + threadIdx.x; q < q1; q += 256) {
        const uint32_t m = uint32_t(E.idx2[q]);
        atomicOr(&mset[m >> 5], 1u << (m & 31));
    }
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int64_t base = mode ? off[r] : 0;
    int total = 0;
    for (int wb = 0; wb < mw; wb += 256) {
        const int w = wb + threadIdx.x;
        uint32_t word = w < mw ? mset[w] : 0u;
        const int n = __popc(word);
        int incl = n;
        for (int d = 1; d < 64; d <<= 1) {
            const int y = __shfl_up(incl, d, 64);
            if (lane >= d) incl += y;
        }
        if (lane == 63) wave_tot[wave] = incl;
        __syncthreads();
        int before = 0, all = 0;
        for (int x = 0; x < 4; ++x) { if (x < wave) before += wave_tot[x]; all += wave_tot[x]; }
        if (mode) {
            int64_t at = base + before + incl - n;
            while (word) {
                list[at++] = (w << 5) + __ffs(word) - 1;
                word &= word - 1;
            }
        }
        base += all;
        total += all;
        __syncthreads();
    }
    if (!mode && threadIdx.x == 0) count[r] = total;
}

constexpr int kScLocalWaves = 8;

// LDS layout of the block-local kernel, in bytes from the start (set up by the plan)
struct ScLocalLds {
    int cd, tk, pos, lval, rowptr, c0, clen, qoff, mmap, umap, total;
    int ns_pad, rows_pad;                    // row strides of T_K and of C_K (doubles)
};

// Everything the workgroup of one K needs to know before its first load (built with the plan).
struct alignas(64) ScRoot {
    int64_t n0, mu0, e0, li0, q0;            // first: u row of I, m of K, (K,i) node, leaf of I, leaf of E
    int64_t pk;                              // where the dense block P_K starts in the plan's copy
    int32_t ns, nrows, nm, nn;               // v slots, u rows, m and (K,i) nodes of K
    int32_t nleaves;                         // leaves of I under K
    int32_t pad[3];
};

typedef double sc_v4d __attribute__((ext_vector_type(4)));
constexpr int kScAhead = 6;                  // (K,i) nodes per wavefront whose loads are issued together
constexpr int kScDepth = 10;                 // depth steps (of 4 slots) of a result tile whose P_K values sit in registers

// largest x in [0, n) with arr[x] <= key (arr ascending, arr[0] <= key)
__device__ __forceinline__ int last_not_above(const int32_t *arr, int n, int32_t key) {
    int lo = 0, hi = n;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (arr[mid] <= key) lo = mid; else hi = mid;
    }
    return lo;
}

// One workgroup per K of E.  The dense block P_K [v slots of K x m of K] is prepared with the plan
// (K that share their v and m lists share one copy) and stays in global memory; I_K [u rows x v
// slots], C_K [nodes x u rows] and T_K [nodes x v slots] live in LDS.  Three dependent trips to
// memory, a barrier after each:
//   1  the descriptor of K; meanwhile the u -> row table is cleared
//   2  what the descriptor addresses: u -> row and m -> position tables, row pointers of I[K], per
//      (K,i) node the range of C[i,:], of its leaves in E and the value of L; blocks zeroed
//   3  the stored entries: I_K one thread per leaf; per node (one wavefront each) the entries of
//      C[i,:] that meet a u row of K into C_K; the m of the node's leaves wait in registers and become
//      pos[node, m of K] = leaf of E[K,i,m] in the node once I_K is dead and its space free
//   then on the fp64 matrix cores (v_mfma_f64_16x16x4, tiles of 16 x 16, depth in steps of 4)
//   T_K = C_K . I_K into LDS, a barrier, and E_K = T_K . P_K with P_K read from memory; every element
//   that is a stored leaf goes to its place in `out`.
__global__ void __launch_bounds__(64 * kScLocalWaves, 6)
spchain3_local_kernel(ScArgs A, ScOut E, double *__restrict__ out, ScLocalLds O, const ScRoot *__restrict__ roots,
                      const double *__restrict__ pk_blocks, const int32_t *__restrict__ e_c0,
                      const int32_t *__restrict__ e_clen) {
    extern __shared__ unsigned char lds[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);    // the same in every lane: loop counters built on it stay scalar
    const int nthreads = 64 * kScLocalWaves;
    double *Ik = reinterpret_cast<double *>(lds);
    double *Cd = reinterpret_cast<double *>(lds + O.cd);
    double *Tk = reinterpret_cast<double *>(lds + O.tk);
    uint16_t *pos = reinterpret_cast<uint16_t *>(lds + O.pos);
    double *lval = reinterpret_cast<double *>(lds + O.lval);
    int32_t *rowptr = reinterpret_cast<int32_t *>(lds + O.rowptr);       // leaves of K before each u row
    int32_t *c0s = reinterpret_cast<int32_t *>(lds + O.c0);              // per node: first entry of C[i,:], its length,
    int32_t *clen = reinterpret_cast<int32_t *>(lds + O.clen);           //           leaves of E before the node
    int32_t *qoff = reinterpret_cast<int32_t *>(lds + O.qoff);
    uint16_t *mmap = reinterpret_cast<uint16_t *>(lds + O.mmap);
    uint16_t *umap = reinterpret_cast<uint16_t *>(lds + O.umap);
    const int tstride = O.ns_pad, cstride = O.rows_pad;

    // trip 1
    const ScRoot R = roots[blockIdx.x];
    for (int64_t x = threadIdx.x; x < (A.n_u + 1) / 2; x += nthreads) reinterpret_cast<uint32_t *>(umap)[x] = 0xFFFFFFFFu;
    const int ns = R.ns, nrows = R.nrows, nm = R.nm, nn = R.nn;
    __syncthreads();
    // trip 2
    for (int x = threadIdx.x; x < nrows; x += nthreads) umap[A.i_idx1[R.n0 + x]] = uint16_t(x);
    for (int x = threadIdx.x; x <= nrows; x += nthreads) rowptr[x] = int32_t(A.i_ptr1[R.n0 + x] - R.li0);
    for (int j = threadIdx.x; j < nm; j += nthreads) mmap[A.mu_list[R.mu0 + j]] = uint16_t(j);
    for (int x = threadIdx.x; x <= nn; x += nthreads) {
        qoff[x] = int32_t(E.ptr1[R.e0 + x] - R.q0);
        if (x < nn) {
            c0s[x] = e_c0[R.e0 + x];
            clen[x] = e_clen[R.e0 + x];
            lval[x] = E.lval[R.e0 + x];
        }
    }
    for (int x = threadIdx.x; x < nrows * ns; x += nthreads) Ik[x] = 0.0;
    for (int x = threadIdx.x; x < nn * cstride; x += nthreads) Cd[x] = 0.0;
    __syncthreads();
    // trip 3: every load of this wavefront's first kScAhead nodes is issued before any is used
    int cidx[kScAhead], m0[kScAhead], m1[kScAhead];
    double cval[kScAhead];
#pragma unroll
    for (int b = 0; b < kScAhead; ++b) {
        const int x = wave + b * kScLocalWaves;
        cidx[b] = -1;
        cval[b] = 0.0;
        m0[b] = m1[b] = -1;
        if (x < nn) {
            if (lane < clen[x]) { cidx[b] = A.c_idx1[int64_t(c0s[x]) + lane]; cval[b] = A.c_vals[int64_t(c0s[x]) + lane]; }
            const int64_t qa = R.q0 + qoff[x];
            const int nl = qoff[x + 1] - qoff[x];
            if (lane < nl) m0[b] = E.idx2[qa + lane];
            if (lane + 64 < nl) m1[b] = E.idx2[qa + lane + 64];
        }
    }
    for (int l = threadIdx.x; l < R.nleaves; l += nthreads) {
        const int row = last_not_above(rowptr, nrows, l);
        Ik[row * ns + A.i_slot[R.li0 + l]] = A.i_vals[R.li0 + l];
    }
#pragma unroll
    for (int b = 0; b < kScAhead; ++b) {
        const int x = wave + b * kScLocalWaves;
        if (cidx[b] >= 0) {
            const uint16_t row = umap[cidx[b]];
            if (row != kNoSlot) Cd[x * cstride + row] = cval[b];
        }
    }
    // what the registers did not cover: entries of C[i,:] beyond 64, nodes beyond the first kScAhead
    for (int x = wave; x < nn; x += kScLocalWaves) {
        const bool ahead = x < kScAhead * kScLocalWaves;
        const int64_t c0 = c0s[x];
        for (int c = (ahead ? 64 : 0) + lane; c < clen[x]; c += 64) {
            const uint16_t row = umap[A.c_idx1[c0 + c]];
            if (row != kNoSlot) Cd[x * cstride + row] = A.c_vals[c0 + c];
        }
    }
    __syncthreads();
    const int li = lane & 15, lk = lane >> 4;
    // the first tile of E_K this wavefront will compute: its part of P_K is fetched now
    const double *Pk = pk_blocks + R.pk;
    // 32-bit offsets against scalar bases: a block P_K and the leaves of one K stay far below 2^29 elements
    const char *Pkb = reinterpret_cast<const char *>(Pk);
    char *outb = reinterpret_cast<char *>(out + R.q0);
    const int tiles_m = (nm + 15) >> 4, tiles_e = ((nn + 15) >> 4) * tiles_m;
    double bpre[kScDepth];
    {
        const int j0 = (wave % tiles_m) << 4;
        const bool jb = wave < tiles_e && j0 + li < nm;
#pragma unroll
        for (int kb = 0; kb < kScDepth; ++kb) {
            const int k = 4 * kb + lk;
            bpre[kb] = (jb && k < ns) ? *reinterpret_cast<const double *>(Pkb + (uint32_t(k * nm + j0 + li) << 3)) : 0.0;
        }
    }
    // T_K = C_K . I_K
    {
        const int tiles_s = (ns + 15) >> 4, tiles = ((nn + 15) >> 4) * tiles_s;
        for (int tile = wave; tile < tiles; tile += kScLocalWaves) {
            const int x0 = (tile / tiles_s) << 4, s0 = (tile % tiles_s) << 4;
            const bool xa = x0 + li < nn, sb = s0 + li < ns;
            const double *crow = Cd + (xa ? x0 + li : 0) * cstride;
            const double *icol = Ik + (sb ? s0 + li : 0);
            sc_v4d acc = {0.0, 0.0, 0.0, 0.0};
            // Rows of C_K beyond the nodes and columns of I_K beyond the slots are read from a valid
            // place as they are: what they produce lies in rows and columns of the tile that are
            // not stored.  Only the last, partial depth step needs its operands masked.
            int k0 = 0;
            for (; k0 + 4 <= nrows; k0 += 4)
                acc = __builtin_amdgcn_mfma_f64_16x16x4f64(crow[k0 + lk], icol[(k0 + lk) * ns], acc, 0, 0, 0);
            if (k0 < nrows) {
                const int k = k0 + lk;
                const bool kk = k < nrows;
                const double av = kk ? crow[kk ? k : 0] : 0.0;
                const double bv = kk ? icol[(kk ? k : 0) * ns] : 0.0;
                acc = __builtin_amdgcn_mfma_f64_16x16x4f64(av, bv, acc, 0, 0, 0);
            }
            if (sb) {
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int x = x0 + lk + 4 * v;
                    if (x < nn) Tk[x * tstride + s0 + li] = acc[v];
                }
            }
        }
    }
    __syncthreads();
    // I_K is dead: pos[node, m of K] = leaf of E[K,i,m] within the node takes its place
    for (int x = threadIdx.x; x < (nn * nm + 1) / 2; x += nthreads) reinterpret_cast<uint32_t *>(pos)[x] = 0xFFFFFFFFu;
    __syncthreads();
#pragma unroll
    for (int b = 0; b < kScAhead; ++b) {
        const int x = wave + b * kScLocalWaves;
        if (m0[b] >= 0) pos[x * nm + mmap[m0[b]]] = uint16_t(lane);
        if (m1[b] >= 0) pos[x * nm + mmap[m1[b]]] = uint16_t(lane + 64);
    }
    for (int x = wave; x < nn; x += kScLocalWaves) {
        const bool ahead = x < kScAhead * kScLocalWaves;
        const int64_t qa = R.q0 + qoff[x];
        const int nl = qoff[x + 1] - qoff[x];
        for (int l = (ahead ? 128 : 0) + lane; l < nl; l += 64) pos[x * nm + mmap[E.idx2[qa + l]]] = uint16_t(l);
    }
    __syncthreads();
    // E_K = T_K . P_K
    for (int tile = wave; tile < tiles_e; tile += kScLocalWaves) {
        const int x0 = (tile / tiles_m) << 4, j0 = (tile % tiles_m) << 4;
        const bool xa = x0 + li < nn, jb = j0 + li < nm;
        const double *trow = Tk + (xa ? x0 + li : 0) * tstride;
        const double *pcol = Pk + (jb ? j0 + li : 0);
        // the next tile's part of P_K, fetched while this tile is computed
        double bnext[kScDepth];
        {
            const int tn = tile + kScLocalWaves;
            const int jn = (tn % tiles_m) << 4;
            const bool jnb = tn < tiles_e && jn + li < nm;
#pragma unroll
            for (int kb = 0; kb < kScDepth; ++kb) {
                const int k = 4 * kb + lk;
                bnext[kb] = (jnb && k < ns) ? *reinterpret_cast<const double *>(Pkb + (uint32_t(k * nm + jn + li) << 3)) : 0.0;
            }
        }
        sc_v4d acc = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
        for (int kb = 0; kb < kScDepth; ++kb) {
            if (4 * kb + 4 <= ns) {                                     // whole step: rows beyond the nodes are not stored
                acc = __builtin_amdgcn_mfma_f64_16x16x4f64(trow[4 * kb + lk], bpre[kb], acc, 0, 0, 0);
            } else if (4 * kb < ns) {
                const int k = 4 * kb + lk;
                const double av = k < ns ? trow[k < ns ? k : 0] : 0.0;
                acc = __builtin_amdgcn_mfma_f64_16x16x4f64(av, bpre[kb], acc, 0, 0, 0);
            }
        }
        for (int k0 = 4 * kScDepth; k0 < ns; k0 += 4) {                 // more than 4 * kScDepth slots
            const int k = k0 + lk;
            const bool kk = k < ns;
            const double av = kk ? trow[kk ? k : 0] : 0.0;
            const double bv = (jb && kk) ? pcol[int64_t(kk ? k : 0) * nm] : 0.0;
            acc = __builtin_amdgcn_mfma_f64_16x16x4f64(av, bv, acc, 0, 0, 0);
        }
        // lane holds E_K[x0 + lk + 4v][j0 + li]
        if (jb) {
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int x = x0 + lk + 4 * v;
                if (x < nn) {
                    const uint16_t at = pos[x * nm + j0 + li];
                    if (at != kNoSlot) *reinterpret_cast<double *>(outb + (uint32_t(qoff[x] + at) << 3)) = acc[v] * lval[x];
                }
            }
        }
#pragma unroll
        for (int kb = 0; kb < kScDepth; ++kb) bpre[kb] = bnext[kb];
    }
}

// per (K,i) node: the range of C[i,:]
__global__ void spchain3_row_tables_kernel(ScArgs A, ScOut E, int32_t *e_c0, int32_t *e_clen) {
    const int64_t x = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (x < E.nodes) {
        const int64_t b0 = A.c_ptr0[E.cnode[x]];
        e_c0[x] = int32_t(b0);
        e_clen[x] = int32_t(A.c_ptr0[E.cnode[x] + 1] - b0);
    }
}

// does root r list other v or other m than root r - 1?  (the same lists share one block P_K)
__global__ void spchain3_class_flag_kernel(ScArgs A, ScOut E, int64_t *flag, int64_t *elems) {
    const int64_t r = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (r >= E.roots) return;
    const int64_t a = E.root_knode[r];
    const int64_t nu0 = A.nu_ptr[a], ns = A.nu_ptr[a + 1] - nu0;
    const int64_t mu0 = A.mu_ptr[r], nm = A.mu_ptr[r + 1] - mu0;
    bool differs = r == 0;
    if (!differs) {
        const int64_t b = E.root_knode[r - 1];
        const int64_t nub = A.nu_ptr[b], mub = A.mu_ptr[r - 1];
        differs = (A.nu_ptr[b + 1] - nub) != ns || (A.mu_ptr[r] - mub) != nm;
        for (int64_t s = 0; !differs && s < ns; ++s) differs = A.nu_list[nu0 + s] != A.nu_list[nub + s];
        for (int64_t j = 0; !differs && j < nm; ++j) differs = A.mu_list[mu0 + j] != A.mu_list[mub + j];
    }
    flag[r] = differs ? 1 : 0;
    elems[r] = differs ? ns * nm : 0;
}

// P_K of every class: one workgroup per root that opens a class; one wavefront per m of K
__global__ void __launch_bounds__(256)
spchain3_pk_fill_kernel(ScArgs A, ScOut E, const int64_t *__restrict__ flag, const int64_t *__restrict__ block_off,
                        double *pk_blocks) {
    const int64_t r = blockIdx.x;
    if (!flag[r]) return;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t a = E.root_knode[r];
    const int64_t nu0 = A.nu_ptr[a], nu1 = A.nu_ptr[a + 1];
    const int64_t mu0 = A.mu_ptr[r], nm = A.mu_ptr[r + 1] - mu0;
    double *Pk = pk_blocks + block_off[r];
    for (int64_t j = wave; j < nm; j += 4) {
        const int32_t pn = A.p_node_of_m[A.mu_list[mu0 + j]];
        for (int64_t p = A.p_ptr0[pn] + lane; p < A.p_ptr0[pn + 1]; p += 64) {
            const int64_t at = find_in(A.nu_list, nu0, nu1, A.p_idx1[p]);
            if (at >= 0) Pk[(at - nu0) * nm + j] = A.p_vals[p];
        }
    }
}

// Cost of a root's workgroup in matrix instructions (T_K = C_K . I_K, then E_K = T_K . P_K), as a key that
// sorts the costliest first: the grid starts its long workgroups first and fills the tail with short ones.
__global__ void spchain3_cost_key_kernel(ScArgs A, ScOut E, uint64_t *keys, uint32_t *root) {
    const int64_t r = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (r >= E.roots) return;
    const int64_t a = E.root_knode[r];
    const int64_t ns = A.nu_ptr[a + 1] - A.nu_ptr[a], nrows = A.i_ptr0[a + 1] - A.i_ptr0[a];
    const int64_t nm = A.mu_ptr[r + 1] - A.mu_ptr[r], nn = E.ptr0[r + 1] - E.ptr0[r];
    const int64_t tn = (nn + 15) / 16, ts = (ns + 15) / 16, tm = (nm + 15) / 16;
    const uint64_t cost = uint64_t(tn * ts * ((nrows + 3) / 4) + tn * tm * ((ns + 3) / 4) + tn * tm);
    keys[r] = ~cost & 0xffffffffffull;
    root[r] = uint32_t(r);
}

// the descriptor of every root of E, written in the order the workgroups take the roots (`order`, or
// root order when it is null); flag / block_off: the root that opened r's class of equal lists and its block
__global__ void spchain3_root_desc_kernel(ScArgs A, ScOut E, const int64_t *__restrict__ flag,
                                          const int64_t *__restrict__ block_off, const uint32_t *__restrict__ order,
                                          ScRoot *roots) {
    const int64_t p = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (p >= E.roots) return;
    const int64_t r = order ? int64_t(order[p]) : p;
    const int64_t a = E.root_knode[r];
    ScRoot R{};
    R.ns = int32_t(A.nu_ptr[a + 1] - A.nu_ptr[a]);
    R.n0 = A.i_ptr0[a];
    R.nrows = int32_t(A.i_ptr0[a + 1] - R.n0);
    R.mu0 = A.mu_ptr[r];
    R.nm = int32_t(A.mu_ptr[r + 1] - R.mu0);
    R.e0 = E.ptr0[r];
    R.nn = int32_t(E.ptr0[r + 1] - R.e0);
    R.li0 = A.i_ptr1[R.n0];
    R.nleaves = int32_t(A.i_ptr1[R.n0 + R.nrows] - R.li0);
    R.q0 = E.ptr1[R.e0];
    int64_t opener = r;
    while (!flag[opener]) --opener;
    R.pk = block_off[opener];
    roots[p] = R;
}

// ---- host side -------------------------------------------------------------------------------

// index of the level-`level` ancestor of every leaf of a CSF tensor
__global__ void leaf_ancestor_index_kernel(int order, int level, int64_t nnz, const int64_t *p0, int64_t n0,
                                           const int64_t *p1, int64_t n1, const int32_t *idx, int32_t *out) {
    const int64_t l = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (l >= nnz) return;
    int64_t c = l;
    if (order == 3) {
        c = parent_of(p1, n1, c);
        if (level == 0) c = parent_of(p0, n0, c);
    } else {
        c = parent_of(p0, n0, c);
    }
    out[l] = idx[c];
}

__global__ void sc_fill_i32_kernel(int32_t *p, int64_t n, int32_t v) {
    const int64_t x = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (x < n) p[x] = v;
}

__global__ void node_of_index_kernel(const int32_t *idx0, int64_t roots, int32_t *node_of) {
    const int64_t x = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (x < roots) node_of[idx0[x]] = int32_t(x);
}

__global__ void leaf_slot_kernel(int64_t nnz, const int64_t *p0, int64_t n0, const int64_t *p1, int64_t n1,
                                 const int32_t *idx2, const int64_t *nu_ptr, const int32_t *nu_list, uint16_t *slot) {
    const int64_t l = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (l >= nnz) return;
    const int64_t a = parent_of(p0, n0, parent_of(p1, n1, l));
    const int64_t at = find_in(nu_list, nu_ptr[a], nu_ptr[a + 1], idx2[l]);
    slot[l] = uint16_t(at - nu_ptr[a]);
}

// per leaf of L: node of I holding its K, root node of C holding its i (-1 where absent)
__global__ void filter_nodes_kernel(int64_t nnz, const int64_t *lp0, int64_t ln0, const int32_t *l_idx0,
                                    const int32_t *l_idx1, const int32_t *i_idx0, int64_t i_roots,
                                    const int32_t *c_idx0, int64_t c_roots, int32_t *knode, int32_t *cnode) {
    const int64_t l = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (l >= nnz) return;
    const int32_t K = l_idx0[parent_of(lp0, ln0, l)];
    knode[l] = int32_t(find_in(i_idx0, 0, i_roots, K));
    cnode[l] = int32_t(find_in(c_idx0, 0, c_roots, l_idx1[l]));
}

__global__ void nonzero_flag_kernel(const int64_t *count, int64_t n, int64_t *flag) {
    const int64_t x = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (x < n) flag[x] = count[x] > 0 ? 1 : 0;
}

static inline dim3 grid_for(int64_t n, int block = 256) { return dim3(unsigned(std::max<int64_t>(1, div_up(n, block)))); }

static ScArgs make_args(const conststn_plan_s *plan) {
    const conststn_csf_s *I = plan->X, *C = plan->sc_C, *P = plan->sc_P, *L = plan->sc_L;
    ScArgs A{};
    A.i_idx0 = I->idx[0].p; A.i_idx1 = I->idx[1].p;
    A.i_ptr0 = I->ptr[0].p; A.i_ptr1 = I->ptr[1].p;
    A.i_vals = I->vals.p;
    A.i_roots = I->nodes[0];
    A.c_idx0 = C->idx[0].p; A.c_idx1 = C->idx[1].p; A.c_ptr0 = C->ptr[0].p; A.c_vals = C->vals.p;
    A.c_roots = C->nodes[0];
    A.p_idx1 = P->idx[1].p; A.p_ptr0 = P->ptr[0].p; A.p_vals = P->vals.p;
    A.p_node_of_m = plan->sc_p_node_of_m.p;
    A.nu_ptr = plan->sc_nu_ptr.p;
    A.nu_list = plan->sc_nu_list.p;
    A.i_slot = plan->sc_i_slot.p;
    A.n_v = I->dims[I->mode_order[2]];
    A.n_m = P->dims[P->mode_order[0]];
    A.max_slots = plan->sc_max_slots;
    A.restricted = L ? 1 : 0;
    A.n_cand = L ? L->nnz : A.i_roots * A.c_roots;
    A.l_knode = plan->sc_l_knode.p;
    A.l_cnode = plan->sc_l_cnode.p;
    A.l_vals = L ? L->vals.p : nullptr;
    A.mu_ptr = plan->sc_mu_ptr.p;
    A.mu_list = plan->sc_mu_list.p;
    A.n_u = I->dims[I->mode_order[1]];
    return A;
}

static ScOut make_out(const conststn_plan_s *plan) {
    conststn_csf_s *E = plan->sc_E.get();
    ScOut o{};
    o.idx0 = E->idx[0].p; o.idx1 = E->idx[1].p; o.idx2 = E->idx[2].p;
    o.ptr0 = E->ptr[0].p; o.ptr1 = E->ptr[1].p;
    o.knode = plan->sc_e_knode.p; o.cnode = plan->sc_e_cnode.p; o.lval = plan->sc_e_lval.p;
    o.root_knode = plan->sc_e_root_knode.p;
    o.roots = E->nodes[0]; o.nodes = E->nodes[1]; o.nnz = E->nodes[2];
    return o;
}

// Order-3 CSF tensor T (levels a > b > c): the distinct c under every root a, ascending (u_ptr over the
// root nodes, u_list), found as the level-1 nodes of T re-sorted a > c > b, and for every leaf the
// position of its c in the list of its root (16 bits).
conststn_status csf3_leaf_universe(const conststn_csf_s *T, DevBuf<int64_t> &u_ptr, DevBuf<int32_t> &u_list,
                                   DevBuf<uint16_t> &slot, int64_t *largest, std::vector<int64_t> *host_ptr) {
    const hipStream_t st = nullptr;
    if (T->order != 3) { set_error("internal: leaf universe of an order-%d tensor", T->order); return CONSTSTN_EINVAL; }
    conststn_csf_s acb;
    DevBuf<int32_t> ca, cb;
    CST_TRY(ca.alloc(size_t(T->nnz)));
    CST_TRY(cb.alloc(size_t(T->nnz)));
    if (T->nnz) {
        leaf_ancestor_index_kernel<<<grid_for(T->nnz), 256, 0, st>>>(3, 0, T->nnz, T->ptr[0].p, T->nodes[0], T->ptr[1].p,
                                                                    T->nodes[1], T->idx[0].p, ca.p);
        leaf_ancestor_index_kernel<<<grid_for(T->nnz), 256, 0, st>>>(3, 1, T->nnz, T->ptr[0].p, T->nodes[0], T->ptr[1].p,
                                                                    T->nodes[1], T->idx[1].p, cb.p);
    }
    CST_HIP(hipGetLastError());
    const int32_t *coords[3] = {ca.p, cb.p, T->idx[2].p};
    const int64_t dims3[3] = {T->dims[T->mode_order[0]], T->dims[T->mode_order[1]], T->dims[T->mode_order[2]]};
    const int mo[3] = {0, 2, 1};
    CST_TRY(build_csf_device(3, dims3, T->nnz, coords, T->vals.p, mo, 0, st, &acb));
    if (acb.nodes[0] != T->nodes[0]) { set_error("internal: re-sorted copy has %lld roots, the tensor has %lld", (long long)acb.nodes[0], (long long)T->nodes[0]); return CONSTSTN_EINVAL; }
    CST_TRY(u_ptr.alloc(size_t(acb.nodes[0] + 1)));
    CST_TRY(u_list.alloc(size_t(acb.nodes[1])));
    CST_HIP(hipMemcpy(u_ptr.p, acb.ptr[0].p, size_t(acb.nodes[0] + 1) * sizeof(int64_t), hipMemcpyDeviceToDevice));
    if (acb.nodes[1])
        CST_HIP(hipMemcpy(u_list.p, acb.idx[1].p, size_t(acb.nodes[1]) * sizeof(int32_t), hipMemcpyDeviceToDevice));
    std::vector<int64_t> h(size_t(acb.nodes[0] + 1));
    CST_HIP(hipMemcpy(h.data(), acb.ptr[0].p, h.size() * sizeof(int64_t), hipMemcpyDeviceToHost));
    int64_t mx = 1;
    for (size_t a = 0; a + 1 < h.size(); ++a) mx = std::max(mx, h[a + 1] - h[a]);
    if (mx > 65534) { set_error("one root index joins %lld distinct innermost indices; they are numbered with 16 bits", (long long)mx); return CONSTSTN_EUNSUPPORTED; }
    *largest = mx;
    if (host_ptr) host_ptr->swap(h);
    CST_TRY(slot.alloc(size_t(T->nnz)));
    if (T->nnz)
        leaf_slot_kernel<<<grid_for(T->nnz), 256, 0, st>>>(T->nnz, T->ptr[0].p, T->nodes[0], T->ptr[1].p, T->nodes[1], T->idx[2].p,
                                                          u_ptr.p, u_list.p, slot.p);
    CST_HIP(hipGetLastError());
    return CONSTSTN_OK;
}

conststn_status build_spchain3_tables(conststn_plan_s *plan) {
    const conststn_csf_s *I = plan->X, *C = plan->sc_C, *P = plan->sc_P, *L = plan->sc_L;
    const hipStream_t st = nullptr;
    const int64_t n_K = I->dims[I->mode_order[0]], n_u = I->dims[I->mode_order[1]], n_v = I->dims[I->mode_order[2]];
    const int64_t n_i = C->dims[C->mode_order[0]], n_m = P->dims[P->mode_order[0]];
    if (n_v > 70000) { set_error("the sparse-chain kernel keeps a v -> slot table of 2 bytes per v in LDS; extent %lld is beyond it", (long long)n_v); return CONSTSTN_EUNSUPPORTED; }

    // P transposed to (v > m), for the symbolic pass only
    conststn_csf_s pt;
    {
        DevBuf<int32_t> cm;
        CST_TRY(cm.alloc(size_t(P->nnz)));
        if (P->nnz)
            leaf_ancestor_index_kernel<<<grid_for(P->nnz), 256, 0, st>>>(2, 0, P->nnz, P->ptr[0].p, P->nodes[0], nullptr, 0,
                                                                        P->idx[0].p, cm.p);
        CST_HIP(hipGetLastError());
        const int32_t *coords[2] = {P->idx[1].p, cm.p};
        const int64_t dims2[2] = {n_v, n_m};
        const int mo[2] = {0, 1};
        CST_TRY(build_csf_device(2, dims2, P->nnz, coords, P->vals.p, mo, 0, st, &pt));
    }
    DevBuf<int32_t> pt_node_of_v;
    CST_TRY(pt_node_of_v.alloc(size_t(n_v)));
    CST_TRY(plan->sc_p_node_of_m.alloc(size_t(n_m)));
    sc_fill_i32_kernel<<<grid_for(n_v), 256, 0, st>>>(pt_node_of_v.p, n_v, -1);
    sc_fill_i32_kernel<<<grid_for(n_m), 256, 0, st>>>(plan->sc_p_node_of_m.p, n_m, -1);
    node_of_index_kernel<<<grid_for(pt.nodes[0]), 256, 0, st>>>(pt.idx[0].p, pt.nodes[0], pt_node_of_v.p);
    node_of_index_kernel<<<grid_for(P->nodes[0]), 256, 0, st>>>(P->idx[0].p, P->nodes[0], plan->sc_p_node_of_m.p);
    CST_HIP(hipGetLastError());

    // distinct v under every K, and the place of every leaf's v among them
    std::vector<int64_t> h_nu_ptr;
    {
        int64_t mx = 1;
        CST_TRY(csf3_leaf_universe(I, plan->sc_nu_ptr, plan->sc_nu_list, plan->sc_i_slot, &mx, &h_nu_ptr));
        plan->sc_max_slots = int(mx);
    }

    // candidates
    if (L) {
        CST_TRY(plan->sc_l_knode.alloc(size_t(L->nnz)));
        CST_TRY(plan->sc_l_cnode.alloc(size_t(L->nnz)));
        if (L->nnz)
            filter_nodes_kernel<<<grid_for(L->nnz), 256, 0, st>>>(L->nnz, L->ptr[0].p, L->nodes[0], L->idx[0].p, L->idx[1].p,
                                                                 I->idx[0].p, I->nodes[0], C->idx[0].p, C->nodes[0],
                                                                 plan->sc_l_knode.p, plan->sc_l_cnode.p);
        CST_HIP(hipGetLastError());
    }
    ScArgs A = make_args(plan);
    A.pt_idx1 = pt.idx[1].p;
    A.pt_ptr0 = pt.ptr[0].p;
    A.pt_node_of_v = pt_node_of_v.p;
    if (A.n_cand > (int64_t(1) << 30)) {
        set_error("%lld candidate (K,i) pairs; the symbolic pass holds one counter per pair -- use the restricted form "
                  "with a K -> i map", (long long)A.n_cand);
        return CONSTSTN_EUNSUPPORTED;
    }
    const size_t set_bytes = size_t(kScWaves) * (size_t((A.max_slots + 31) >> 5) + size_t((n_m + 31) >> 5)) * 4;
    if (set_bytes > 160 * 1024) { set_error("bit sets of %zu bytes per workgroup do not fit LDS (extent of m %lld)", set_bytes, (long long)n_m); return CONSTSTN_EUNSUPPORTED; }
    CST_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(spchain3_count_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, int(set_bytes)));
    CST_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(spchain3_fill_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, int(set_bytes)));

    plan->sc_E.reset(new conststn_csf_s());
    conststn_csf_s *E = plan->sc_E.get();
    E->order = 3;
    E->dims[0] = n_K; E->dims[1] = n_i; E->dims[2] = n_m;
    for (int l = 0; l < 3; ++l) E->mode_order[l] = l;
    E->device = I->device;
    int64_t nnz = 0, nodes = 0, roots = 0;
    DevBuf<int64_t> count, leaf_off, flag, node_of;
    const int64_t nc = A.n_cand;
    if (nc > 0) {
        CST_TRY(count.alloc(size_t(nc)));
        CST_TRY(leaf_off.alloc(size_t(nc)));
        CST_TRY(flag.alloc(size_t(nc)));
        CST_TRY(node_of.alloc(size_t(nc)));
        spchain3_count_kernel<<<grid_for(nc, kScWaves), 64 * kScWaves, set_bytes, st>>>(A, count.p);
        CST_HIP(hipGetLastError());
        CST_TRY(exscan(count.p, leaf_off.p, nc, &nnz));
        nonzero_flag_kernel<<<grid_for(nc), 256, 0, st>>>(count.p, nc, flag.p);
        CST_HIP(hipGetLastError());
        CST_TRY(exscan(flag.p, node_of.p, nc, &nodes));
    }
    CST_TRY(E->idx[1].alloc(size_t(nodes)));
    CST_TRY(E->ptr[1].alloc(size_t(nodes + 1)));
    CST_TRY(E->idx[2].alloc(size_t(nnz)));
    CST_TRY(plan->sc_e_knode.alloc(size_t(nodes)));
    CST_TRY(plan->sc_e_cnode.alloc(size_t(nodes)));
    CST_TRY(plan->sc_e_lval.alloc(size_t(nodes)));
    E->nodes[1] = nodes;
    E->nodes[2] = nnz;
    E->nnz = nnz;
    ScOut O = make_out(plan);
    if (nodes > 0) {
        spchain3_fill_kernel<<<grid_for(nc, kScWaves), 64 * kScWaves, set_bytes, st>>>(A, O, count.p, leaf_off.p, node_of.p);
        CST_HIP(hipGetLastError());
    }
    // roots
    DevBuf<int64_t> rflag, root_of;
    CST_TRY(rflag.alloc(size_t(nodes)));
    CST_TRY(root_of.alloc(size_t(nodes)));
    if (nodes > 0) {
        spchain3_root_flag_kernel<<<grid_for(nodes), 256, 0, st>>>(O, rflag.p);
        CST_HIP(hipGetLastError());
        CST_TRY(exscan(rflag.p, root_of.p, nodes, &roots));
    }
    CST_TRY(E->idx[0].alloc(size_t(roots)));
    CST_TRY(E->ptr[0].alloc(size_t(roots + 1)));
    CST_TRY(plan->sc_e_root_knode.alloc(size_t(roots)));
    E->nodes[0] = roots;
    O = make_out(plan);
    spchain3_root_fill_kernel<<<grid_for(nodes + 1), 256, 0, st>>>(A, O, rflag.p, root_of.p);
    CST_HIP(hipGetLastError());
    CST_HIP(hipStreamSynchronize(st));

    // numeric pass, general form: LDS = v -> slot table + one workspace per wavefront
    plan->sc_map_bytes = int(((n_v + 1) / 2 * 4 + 15) / 16 * 16);
    const size_t lds = size_t(plan->sc_map_bytes) + size_t(kScWaves) * size_t(plan->sc_max_slots) * sizeof(double);
    if (lds > 160 * 1024) {
        set_error("v -> slot table (%d bytes) and %d workspaces of %d slots do not fit LDS", plan->sc_map_bytes, kScWaves, plan->sc_max_slots);
        return CONSTSTN_EUNSUPPORTED;
    }
    plan->sc_lds_bytes = int(lds);
    CST_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(spchain3_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, int(lds)));

    // block-local form: the m under every root of E, and whether every K's dense blocks fit LDS
    plan->sc_local = false;
    CST_TRY(plan->sc_mu_ptr.alloc(size_t(roots + 1)));
    if (roots > 0 && n_m <= 65534) {
        DevBuf<int64_t> mcount;
        CST_TRY(mcount.alloc(size_t(roots)));
        const size_t mset_bytes = size_t((n_m + 31) >> 5) * 4;
        spchain3_root_mset_kernel<<<dim3(unsigned(roots)), 256, mset_bytes, st>>>(O, n_m, 0, mcount.p, nullptr, nullptr);
        CST_HIP(hipGetLastError());
        int64_t total_m = 0;
        CST_TRY(exscan(mcount.p, plan->sc_mu_ptr.p, roots, &total_m));
        CST_HIP(hipMemcpy(plan->sc_mu_ptr.p + roots, &total_m, sizeof(int64_t), hipMemcpyHostToDevice));
        CST_TRY(plan->sc_mu_list.alloc(size_t(total_m)));
        spchain3_root_mset_kernel<<<dim3(unsigned(roots)), 256, mset_bytes, st>>>(O, n_m, 1, nullptr, plan->sc_mu_ptr.p, plan->sc_mu_list.p);
        CST_HIP(hipGetLastError());
        std::vector<int64_t> h_mu(size_t(roots + 1)), h_iptr(size_t(I->nodes[0] + 1));
        std::vector<int32_t> h_rk(static_cast<size_t>(roots), 0);
        CST_HIP(hipMemcpy(h_mu.data(), plan->sc_mu_ptr.p, h_mu.size() * sizeof(int64_t), hipMemcpyDeviceToHost));
        CST_HIP(hipMemcpy(h_iptr.data(), I->ptr[0].p, h_iptr.size() * sizeof(int64_t), hipMemcpyDeviceToHost));
        CST_HIP(hipMemcpy(h_rk.data(), plan->sc_e_root_knode.p, h_rk.size() * sizeof(int32_t), hipMemcpyDeviceToHost));
        std::vector<int64_t> h_ep(size_t(roots + 1));
        CST_HIP(hipMemcpy(h_ep.data(), E->ptr[0].p, h_ep.size() * sizeof(int64_t), hipMemcpyDeviceToHost));
        int64_t ik = 1, pk = 1, rows_max = 1, nm_max = 1, nn_max = 1;
        for (int64_t r = 0; r < roots; ++r) {
            const int64_t a = h_rk[size_t(r)];
            const int64_t ns = h_nu_ptr[size_t(a + 1)] - h_nu_ptr[size_t(a)];
            const int64_t rows = h_iptr[size_t(a + 1)] - h_iptr[size_t(a)];
            const int64_t nm = h_mu[size_t(r + 1)] - h_mu[size_t(r)];
            ik = std::max(ik, rows * ns);
            pk = std::max(pk, ns * nm);
            rows_max = std::max(rows_max, rows);
            nm_max = std::max(nm_max, nm);
            nn_max = std::max(nn_max, h_ep[size_t(r + 1)] - h_ep[size_t(r)]);
        }
        auto up16 = [](int64_t x) { return (x + 15) / 16 * 16; };
        int64_t posb = 4;                                       // leaf positions, 2 bytes each
        for (int64_t r = 0; r < roots; ++r)
            posb = std::max(posb, 2 * (h_ep[size_t(r + 1)] - h_ep[size_t(r)]) * (h_mu[size_t(r + 1)] - h_mu[size_t(r)]) + 4);
        // odd row strides: the 16 rows a tile reads fall in different banks
        const int64_t ns_pad = plan->sc_max_slots | 1, rows_pad = rows_max | 1;
        int64_t at = 0;
        int64_t o_cd, o_t, o_pos, o_lval, o_rowptr, o_c0, o_clen, o_qoff, o_mmap, o_umap;
        at = up16(std::max(8 * ik, posb)); o_cd = at;           // I_K, later the leaf positions
        at = up16(at + 8 * nn_max * rows_pad); o_t = at;
        at = up16(at + 8 * nn_max * ns_pad); o_pos = 0;
        o_lval = at;
        at = up16(at + 8 * nn_max); o_rowptr = at;
        at = up16(at + 4 * (rows_max + 1)); o_c0 = at;
        at = up16(at + 4 * nn_max); o_clen = at;
        at = up16(at + 4 * nn_max); o_qoff = at;
        at = up16(at + 4 * (nn_max + 1)); o_mmap = at;
        at = up16(at + 2 * n_m); o_umap = at;
        at = up16(at + 4 * ((n_u + 1) / 2));
        const int64_t bytes = at;
        const int64_t budget = plan->opt("spchain3_local_kb", 78) * 1024;      // two workgroups per compute unit
        const bool offsets_fit = I->nnz < (int64_t(1) << 31) && C->nnz < (int64_t(1) << 31) && nnz < (int64_t(1) << 31);
        // a node holds each m of its K at most once, so nm_max also bounds the leaves of a node (16-bit positions)
        // (pk < 2^29: the kernel reaches into a block P_K with 32-bit byte offsets)
        if (rows_max <= 65534 && nm_max <= 65534 && pk < (int64_t(1) << 29) && offsets_fit && bytes <= budget && bytes <= 160 * 1024 &&
            plan->opt("spchain3_form", 1) == 1) {
            ScArgs A2 = make_args(plan);
            // the dense blocks P_K, one per run of K with the same v and m lists
            DevBuf<int64_t> cflag, celems, coff;
            CST_TRY(cflag.alloc(size_t(roots)));
            CST_TRY(celems.alloc(size_t(roots)));
            CST_TRY(coff.alloc(size_t(roots)));
            spchain3_class_flag_kernel<<<grid_for(roots), 256, 0, st>>>(A2, O, cflag.p, celems.p);
            CST_HIP(hipGetLastError());
            int64_t pk_total = 0;
            CST_TRY(exscan(celems.p, coff.p, roots, &pk_total));
            const int64_t pk_cap = plan->opt("spchain3_pk_gb", 4) << 27;       // doubles
            if (pk_total <= pk_cap) {
                CST_TRY(plan->sc_pk_blocks.alloc(size_t(pk_total)));
                CST_TRY(zero_fill(plan->sc_pk_blocks.p, pk_total, st));
                spchain3_pk_fill_kernel<<<dim3(unsigned(roots)), 256, 0, st>>>(A2, O, cflag.p, coff.p, plan->sc_pk_blocks.p);
                CST_HIP(hipGetLastError());
                CST_TRY(plan->sc_e_c0.alloc(size_t(nodes)));
                CST_TRY(plan->sc_e_clen.alloc(size_t(nodes)));
                CST_TRY(plan->sc_roots.alloc(size_t(roots) * sizeof(ScRoot)));
                spchain3_row_tables_kernel<<<grid_for(nodes), 256, 0, st>>>(A2, O, plan->sc_e_c0.p, plan->sc_e_clen.p);
                CST_HIP(hipGetLastError());
                DevBuf<uint64_t> ka, kb;
                DevBuf<uint32_t> ra, rb;
                const uint32_t *order = nullptr;
                if (plan->opt("spchain3_order", 1) == 1) {           // costliest roots first (stable)
                    CST_TRY(ka.alloc(size_t(roots)));
                    CST_TRY(kb.alloc(size_t(roots)));
                    CST_TRY(ra.alloc(size_t(roots)));
                    CST_TRY(rb.alloc(size_t(roots)));
                    spchain3_cost_key_kernel<<<grid_for(roots), 256, 0, st>>>(A2, O, ka.p, ra.p);
                    CST_HIP(hipGetLastError());
                    const uint64_t *ks = nullptr;
                    CST_TRY(radix_sort_pairs_u64(ka.p, kb.p, ra.p, rb.p, roots, 40, st, &ks, &order));
                }
                spchain3_root_desc_kernel<<<grid_for(roots), 256, 0, st>>>(A2, O, cflag.p, coff.p, order,
                                                                          reinterpret_cast<ScRoot *>(plan->sc_roots.p));
                CST_HIP(hipGetLastError());
                CST_HIP(hipStreamSynchronize(st));
                plan->sc_local = true;
                plan->sc_local_lds = int(bytes);
                plan->sc_pk_doubles = pk_total;
                const int lay[13] = {int(o_cd), int(o_t), int(o_pos), int(o_lval), int(o_rowptr), int(o_c0), int(o_clen),
                                     int(o_qoff), int(o_mmap), int(o_umap), int(bytes), int(ns_pad), int(rows_pad)};
                plan->sc_local_layout.assign(lay, lay + 13);
                CST_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(spchain3_local_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, int(bytes)));
            }
        }
    }
    CST_HIP(hipStreamSynchronize(st));
    plan->out_rows = nnz;
    plan->row_elems = 1;
    return CONSTSTN_OK;
}

conststn_status launch_spchain3(const conststn_plan_s *plan, double *out, hipStream_t stream) {
    const ScArgs A = make_args(plan);
    const ScOut O = make_out(plan);
    ProfScope prof(plan, stream);
    if (O.roots == 0) return CONSTSTN_OK;
    if (plan->sc_local)
    {
        const std::vector<int> &l = plan->sc_local_layout;
        const ScLocalLds lay{l[0], l[1], l[2], l[3], l[4], l[5], l[6], l[7], l[8], l[9], l[10], l[11], l[12]};
        spchain3_local_kernel<<<dim3(unsigned(O.roots)), 64 * kScLocalWaves, size_t(plan->sc_local_lds), stream>>>(
            A, O, out, lay, reinterpret_cast<const ScRoot *>(plan->sc_roots.p), plan->sc_pk_blocks.p, plan->sc_e_c0.p,
            plan->sc_e_clen.p);
    }
    else
        spchain3_kernel<<<dim3(unsigned(O.roots)), 64 * kScWaves, size_t(plan->sc_lds_bytes), stream>>>(A, O, out, plan->sc_map_bytes);
    CST_HIP(hipGetLastError());
    return CONSTSTN_OK;
}

}  // namespace cst
