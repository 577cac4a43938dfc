// Fused order-3 TTMc over a CSF tensor (Sec. 5.3):
//     Y[i,r2,r3] = sum_{j,k} X[i,j,k] U2[j,r2] U3[k,r3]
// as the tree  T[i,j,r3] = X[i,j,k] U3[k,r3] ; Y[i,r2,r3] = T[i,j,r3] U2[j,r2]  fused on the
// loops i and j: the intermediate is one length-R3 vector per (i,j) fiber, the consumer is
// the rank-1 update Y_i += U2[j,:]^T (x) T, i.e. per slice Y_i = U2[J_i,:]^T . T_i.
//
// General kernel (any ranks up to 64): one wavefront per work item (a leaf range inside one
// slice, see partition.hip); lane = r3, the R2 accumulators of column r3 live in registers.
// All control flow is wave-uniform, so leaf indices/values and the U2 row are fetched with
// scalar loads and the update is R2 FMAs with a scalar operand.
#include <type_traits>

#include "plan.hpp"

namespace cst {

struct Ttmc3Args {
    int64_t n_items, n_split;
    int R2, R3;
    const int64_t *ptr1;
    const int32_t *idx0, *idx1, *idx2;
    const double *vals;
    const SliceItem *items;
    const int32_t *split_slices;
    const int64_t *split_first;
    const int32_t *split_count;
    const double *U2, *U3;
    double *out, *partial;
    int compact;
};

__device__ __forceinline__ int64_t uniform64(int64_t v) {
    const int lo = __builtin_amdgcn_readfirstlane(int(v & 0xffffffffll));
    const int hi = __builtin_amdgcn_readfirstlane(int(v >> 32));
    return (int64_t(hi) << 32) | int64_t(uint32_t(lo));
}

template <int R2T>
__global__ void __launch_bounds__(256)
ttmc3_kernel(Ttmc3Args a) {
    const int lane = threadIdx.x % 64;
    const int64_t w = uniform64(int64_t(blockIdx.x) * 4 + threadIdx.x / 64);
    if (w >= a.n_items) return;
    const SliceItem it = a.items[w];
    const int32_t s = __builtin_amdgcn_readfirstlane(it.slice);
    const int64_t nb = uniform64(it.end);
    int64_t f = uniform64(it.first);
    const int64_t dest = uniform64(it.dest);
    const int R2 = a.R2, R3 = a.R3;
    const bool active = lane < R3;
    const int col = active ? lane : 0;

    double y[R2T];
#pragma unroll
    for (int r = 0; r < R2T; ++r) y[r] = 0.0;
    double t = 0.0;
    int64_t fiber_end = uniform64(a.ptr1[f + 1]);
    if (fiber_end > nb) fiber_end = nb;
    int32_t j = __builtin_amdgcn_readfirstlane(a.idx1[f]);

    for (int64_t n = uniform64(it.begin); n < nb;) {
        // leaves of the current fiber that fall inside this item
        for (; n < fiber_end; ++n) {
            const int32_t k = __builtin_amdgcn_readfirstlane(a.idx2[n]);
            const double v = a.vals[n];
            t = fma(v, a.U3[int64_t(k) * R3 + col], t);
        }
        const double *u2 = a.U2 + int64_t(j) * R2;
#pragma unroll
        for (int r = 0; r < R2T; ++r)
            if (r < R2) y[r] = fma(u2[r], t, y[r]);
        t = 0.0;
        if (n < nb) {
            ++f;
            j = __builtin_amdgcn_readfirstlane(a.idx1[f]);
            fiber_end = uniform64(a.ptr1[f + 1]);
            if (fiber_end > nb) fiber_end = nb;
        }
    }
    const int64_t RR = int64_t(R2) * R3;
    double *base = dest < 0 ? a.out + (a.compact ? int64_t(s) : int64_t(a.idx0[s])) * RR
                            : a.partial + dest * RR;
    if (active) {
#pragma unroll
        for (int r = 0; r < R2T; ++r)
            if (r < R2) base[int64_t(r) * R3 + lane] = y[r];
    }
}

// ---- MFMA kernel (ranks multiples of 16, up to 64) ------------------------------------------
//
// Per slice the consumer is a dense contraction, Y_i = U2[J_i,:]^T . T_i, with the fibers of the
// slice as the K dimension.  It runs on the fp64 matrix cores, v_mfma_f64_16x16x4: K = 4 rows per
// instruction.  The plan cuts every fiber into rows of at most kRowLeaves leaves (a long fiber
// gives several rows with the same j: U2[j,:]^T (x) (T' + T'') = the sum of the two rank-1
// updates), so the four rows of one K-step have similar lengths.
// One wavefront per (item, column part): lane = (slot, c) with slot = lane/16 the K index.
//   leaf stage   slot s walks the leaves of row g+s:  T_s[16q + c] += v * U3[k, 16q + c]
//                (each 16-lane row reads 128-B segments of the factor row)     -> B operand
//   A operand    U2[j_s, 16p + c]
//   update       acc[p][q] += A_p (16x4) . T_q (4x16)   for every 16x16 tile of the row block
// The accumulators (PN x QN tiles, 4 doubles per lane each) stay in registers for the whole item;
// a wave covers QN of the R3/16 column tiles so that registers leave room for several waves per
// SIMD (gridDim.y waves share an item).
typedef double v4f64 __attribute__((ext_vector_type(4)));

struct Ttmc3RowArgs {
    int64_t n_items;
    int R2, R3;
    const RowDesc *rows;
    const int32_t *idx0, *idx2;
    const double *vals;
    const SliceItem *items;
    const double *U2, *U3;
    double *out, *partial;
    int compact;
};

template <int PN, int QN>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(QN == 1 ? 5 : (QN == 2 ? 4 : 2), 8)))
ttmc3_mfma_kernel(Ttmc3RowArgs a) {
    const int lane = threadIdx.x % 64;
    // The wavefronts of a workgroup take the column parts of the same item(s): they gather the same
    // U2 rows, which then come from the CU's L1 for all but the first (measured against giving
    // each XCD one column part of U3: 6 % faster on the 2M x 2M x 25000 tensor, where the U2
    // rows, not U3, are the larger stream).
    const int parts = a.R3 / (16 * QN);
    // one item per workgroup (its `parts` wavefronts): items differ in length, and a slot shared
    // with a longer item would stay idle until that one is done
    const int part = threadIdx.x / 64;
    const int64_t w = uniform64(int64_t(blockIdx.x));
    if (w >= a.n_items) return;
    const SliceItem it = a.items[w];
    const int32_t s = __builtin_amdgcn_readfirstlane(it.slice);
    const int64_t ra = uniform64(it.begin), rb = uniform64(it.end), dest = uniform64(it.dest);
    const int slot = lane >> 4, c = lane & 15;
    const int R2 = a.R2, R3 = a.R3;
    // A lane's QN columns are adjacent in memory (column of tile q = col0 + q): one vector load
    // per factor row and one vector store per output row instead of QN scalar ones.  Which
    // columns form a tile is free to choose -- a tile is a set of 16 columns of the result.
    const int col0 = part * QN * 16 + QN * c;

    v4f64 acc[PN][QN];
#pragma unroll
    for (int p = 0; p < PN; ++p)
#pragma unroll
        for (int q = 0; q < QN; ++q) acc[p][q] = v4f64{0.0, 0.0, 0.0, 0.0};

    // Three-stage software pipeline over K-steps (4 rows each): while step g is computed, the
    // leaf entries and U2 segments of step g+4 and the row descriptors of step g+8 are in
    // flight, so a step waits only for its own U3 gathers.
    struct Desc { int64_t la; int cnt; int32_t j; };
    auto load_desc = [&](int64_t g) -> Desc {
        Desc d{0, 0, 0};
        if (g + slot < rb) {
            const RowDesc r = a.rows[g + slot];          // one 16-byte load
            d.la = r.leaf;
            d.cnt = r.cnt;
            d.j = r.j;
        }
        return d;
    };
    struct Feed { int32_t k; double v; int cnt; int32_t j; };
    auto load_feed = [&](const Desc &d) -> Feed {
        Feed f;
        f.k = 0;
        f.v = 0.0;
        f.cnt = d.cnt;
        f.j = d.j;
        if (c < d.cnt) { f.k = a.idx2[d.la + c]; f.v = a.vals[d.la + c]; }
        return f;
    };
    Desc d1 = load_desc(ra);
    Desc d2 = load_desc(ra + 4);
    Feed cur = load_feed(d1);
    for (int64_t g = ra; g < rb; g += 4) {
        const Feed nxt = load_feed(d2);          // step g+4 (its descriptor arrived a step ago)
        d2 = load_desc(g + 8);
        double t[QN];
#pragma unroll
        for (int q = 0; q < QN; ++q) t[q] = 0.0;
        // the (at most kRowLeaves = 16) leaves of the row were loaded one entry per lane of the
        // slot and are handed round inside the slot with lane shuffles -- a broadcast load per
        // leaf would cost the memory pipeline 16 lanes' worth each time
        const int cnt = cur.cnt;
        const int32_t myk = cur.k;
        const double myv = cur.v;
        // A operands, issued with the step's U3 gathers.  As with the columns, which 16 rows of
        // the result form tile p is free to choose: tile p takes rows PN*i + p, so a lane's PN
        // entries of the U2 row are adjacent and come with one vector load.
        double av[PN];
        {
            typedef double vp __attribute__((ext_vector_type(PN == 3 ? 4 : (PN == 1 ? 2 : PN))));
            const double *src = a.U2 + int64_t(cur.j) * R2 + PN * c;
            if (PN == 2 || PN == 4) {
                vp x = {};
                if (cnt > 0) x = *reinterpret_cast<const vp *>(src);
#pragma unroll
                for (int p = 0; p < PN; ++p) av[p] = x[p];
            } else {
#pragma unroll
                for (int p = 0; p < PN; ++p) av[p] = cnt > 0 ? src[p] : 0.0;
            }
        }
        for (int t0 = 0; t0 < cnt; t0 += 4) {
            int32_t kk[4];
            double vv[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                kk[u] = __shfl(myk, t0 + u, 16);
                vv[u] = __shfl(myv, t0 + u, 16);
            }
            typedef double vq __attribute__((ext_vector_type(QN == 1 ? 2 : QN)));
            double uu[4][QN];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const double *src = a.U3 + int64_t(kk[u]) * R3 + col0;
                if (QN == 1) {
                    uu[u][0] = t0 + u < cnt ? src[0] : 0.0;
                } else {
                    vq x = {};
                    if (t0 + u < cnt) x = *reinterpret_cast<const vq *>(src);
#pragma unroll
                    for (int q = 0; q < QN; ++q) uu[u][q] = x[q];
                }
            }
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int q = 0; q < QN; ++q) t[q] = fma(vv[u], uu[u][q], t[q]);
        }
#pragma unroll
        for (int p = 0; p < PN; ++p)
#pragma unroll
            for (int q = 0; q < QN; ++q)
                acc[p][q] = __builtin_amdgcn_mfma_f64_16x16x4f64(av[p], t[q], acc[p][q], 0, 0, 0);
        cur = nxt;
    }
    const int64_t RR = int64_t(R2) * R3;
    double *base = dest < 0 ? a.out + (a.compact ? int64_t(s) : int64_t(a.idx0[s])) * RR
                            : a.partial + dest * RR;
    // tile (p,q): accumulator register v of a lane holds row PN*(slot + 4v) + p, column col0 + q.
    // The row block is written once and never re-read by this kernel: streaming (non-temporal)
    // stores keep the gathered factor rows resident in L2 instead of the output.
#pragma unroll
    for (int p = 0; p < PN; ++p)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            double *dst = base + int64_t(PN * (slot + 4 * v) + p) * R3 + col0;
            if (QN == 1) {
                __builtin_nontemporal_store(acc[p][0][v], dst);
            } else {
                typedef double vq __attribute__((ext_vector_type(QN == 1 ? 2 : QN)));
                vq x;
#pragma unroll
                for (int q = 0; q < QN; ++q) x[q] = acc[p][q][v];
                __builtin_nontemporal_store(x, reinterpret_cast<vq *>(dst));
            }
        }
}

// ---- streaming form of the MFMA kernel ---------------------------------------------------------
//
// The kernel above gathers, multiplies and stores in one wavefront.  Vector loads and stores of a
// wavefront retire through one in-order counter, so a wavefront that has issued the 16 KB of stores
// of a row block cannot see its next gathers arrive before those stores have drained, and the slot
// stays occupied while they do: gather time and store time add up.  Here the two are separate
// wavefronts of one workgroup:
//   producers   (NP wavefronts) walk the plan's flat table of K-steps, every NP-th K-step each: leaf
//               stage on the vector units (T_s += v * U3[k,:] for the four rows of the step), the four
//               U2 rows, both written to a packet in LDS in exactly the lane layout of the matrix
//               instruction's operands.  They never store to memory, so their loads stay in flight
//               across K-steps and items (descriptors three, rows two, leaves one K-step ahead).
//   consumers   (R3/32 wavefronts, two column tiles each) take the packets in K-step order, issue the
//               matrix instructions, and at the last K-step of an item stream the row block out.  They
//               never load from memory, so nothing waits on the stores.
// Packets are double-buffered; one s_barrier per round (NP K-steps) orders the two sides.  A workgroup
// takes a batch of whole items of about equal cost (plan table wg_kstep).  Empty rows of a partial
// K-step repeat the step's last row with value 0 and a zero U2 operand, so every load is
// unconditional.  (A ring of packets with ready flags instead of the barrier, letting the producers
// run sixteen K-steps ahead, measured slower: 20.2 against 18.2 ms on the 140 M-nonzero tensor.)
struct Ttmc3StreamArgs {
    int R2, R3;
    const int32_t *wg_kstep;
    const KStepDesc *ksteps;
    const RowDesc *rows;
    const int32_t *idx2;
    const double *vals;
    const double *U2, *U3;
    double *out, *partial;
};

typedef double v2f64 __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(3))) v2f64 lds_v2f64;

template <int T>
__device__ __forceinline__ int32_t row_bcast_i32(int32_t x) {
    return __builtin_amdgcn_mov_dpp(x, 0x150 + T, 0xf, 0xf, false);
}
template <int T>
__device__ __forceinline__ double row_bcast_f64(double x) {
    const int lo = __builtin_amdgcn_mov_dpp(__double2loint(x), 0x150 + T, 0xf, 0xf, false);
    const int hi = __builtin_amdgcn_mov_dpp(__double2hiint(x), 0x150 + T, 0xf, 0xf, false);
    return __hiloint2double(hi, lo);
}

// wait for this wavefront's LDS traffic, then meet the other wavefronts of the workgroup (outstanding
// vector loads stay in flight: the barrier orders LDS only)
__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

template <int PN, int NC, int NP>
__global__ void __launch_bounds__(64 * (NP + NC))
ttmc3_stream_kernel(Ttmc3StreamArgs a) {
    constexpr int APV = (PN + 1) / 2;                 // 16-byte vectors of a lane's U2 operand
    constexpr int PKT = (APV + NC) * 64;              // 16-byte vectors per packet
    __shared__ v2f64 pkt[2][NP][PKT];
    __shared__ int64_t pkt_dest[2][NP];
    __shared__ int32_t pkt_meta[2][NP];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(int(threadIdx.x >> 6));
    const int ka = a.wg_kstep[blockIdx.x], kb = a.wg_kstep[blockIdx.x + 1];
    if (kb <= ka) return;
    const int rounds = (kb - ka + NP - 1) / NP;
    const int slot = lane >> 4, c = lane & 15;
    const int R2 = a.R2, R3 = a.R3;

    if (wave < NP) {
        // ------------------------------------------------------------------ producer
        struct Rows { int64_t leaf; int cnt; int32_t j; bool live; };
        struct Feed { int32_t k; double v; int maxcnt; v2f64 av[APV]; };
        typedef int v4i32 __attribute__((ext_vector_type(4)));
        auto kstep_of = [&](int r) -> KStepDesc {
            int g = ka + r * NP + wave;
            g = g < kb ? g : kb - 1;
            // one 16-byte load of the whole record (wave-uniform address); fetched field by field the
            // compiler moves the part only lane 0 uses under that lane's mask and then waits for it
            const v4i32 raw = *reinterpret_cast<const v4i32 *>(a.ksteps + g);
            KStepDesc d;
            d.row0 = raw[0];
            d.meta = raw[1];
            d.dest = int64_t((uint64_t(uint32_t(raw[3])) << 32) | uint32_t(raw[2]));
            return d;
        };
        auto load_rows = [&](const KStepDesc &d) -> Rows {
            const int n = d.meta & 7;
            const RowDesc r = a.rows[d.row0 + (slot < n ? slot : n - 1)];
            return Rows{r.leaf, r.cnt, r.j, slot < n};
        };
        auto load_feed = [&](const Rows &r) -> Feed {
            Feed f;
            const int ci = c < r.cnt ? c : r.cnt - 1;   // lanes beyond the row repeat its last leaf, value 0
            f.k = a.idx2[r.leaf + ci];
            const double v = a.vals[r.leaf + ci];
            const bool keep = (c < r.cnt) & r.live;     // no short circuit: a branch here draws the load under it
            f.v = keep ? v : 0.0;
            const v2f64 *src = reinterpret_cast<const v2f64 *>(a.U2 + int64_t(r.j) * R2 + PN * c);
#pragma unroll
            for (int x = 0; x < APV; ++x) {
                v2f64 u;
                if (PN % 2 == 1 && x == APV - 1) u = v2f64{a.U2[int64_t(r.j) * R2 + PN * c + PN - 1], 0.0};
                else u = src[x];
                f.av[x] = r.live ? u : v2f64{0.0, 0.0};
            }
            const int c0 = __builtin_amdgcn_readlane(r.cnt, 0), c1 = __builtin_amdgcn_readlane(r.cnt, 16),
                      c2 = __builtin_amdgcn_readlane(r.cnt, 32), c3 = __builtin_amdgcn_readlane(r.cnt, 48);
            f.maxcnt = max(max(c0, c1), max(c2, c3));
            return f;
        };
        KStepDesc d1 = kstep_of(1), d2 = kstep_of(2);
        Rows r1;
        Feed cur;
        int32_t meta_cur;
        int64_t dest_cur;
        {
            const KStepDesc d0 = kstep_of(0);
            const Rows r0 = load_rows(d0);
            r1 = load_rows(d1);
            cur = load_feed(r0);
            meta_cur = d0.meta;
            dest_cur = d0.dest;
        }
        const char *u3 = reinterpret_cast<const char *>(a.U3);
        const uint32_t row_bytes = uint32_t(R3) * 8u, lane_off = uint32_t(c) * 16u;
        for (int r = 0; r < rounds; ++r) {
            // loads of the rounds ahead, issued before this round's gathers
            const Feed nxt = load_feed(r1);
            const int32_t meta_nxt = d1.meta;
            const int64_t dest_nxt = d1.dest;
            r1 = load_rows(d2);
            d1 = d2;
            d2 = kstep_of(r + 3);

            double t[NC][2];
#pragma unroll
            for (int q = 0; q < NC; ++q) t[q][0] = t[q][1] = 0.0;
            // leaf steps t0 .. t0+N-1 of the four rows: 2N gathers in flight, then the products.  N is exact
            // (not rounded up to four): most K-steps of a power-law tensor hold rows of a single leaf, and
            // every gather instruction counts.
            auto batch = [&](auto T0, auto NN) {
                constexpr int t0 = decltype(T0)::value, N = decltype(NN)::value;
                int32_t kk[4] = {row_bcast_i32<t0>(cur.k), 0, 0, 0};
                double vv[4] = {row_bcast_f64<t0>(cur.v), 0.0, 0.0, 0.0};
                if (N > 1) { kk[1] = row_bcast_i32<t0 + 1>(cur.k); vv[1] = row_bcast_f64<t0 + 1>(cur.v); }
                if (N > 2) { kk[2] = row_bcast_i32<t0 + 2>(cur.k); vv[2] = row_bcast_f64<t0 + 2>(cur.v); }
                if (N > 3) { kk[3] = row_bcast_i32<t0 + 3>(cur.k); vv[3] = row_bcast_f64<t0 + 3>(cur.v); }
                v2f64 uu[N][NC];
#pragma unroll
                for (int u = 0; u < N; ++u)
#pragma unroll
                    for (int q = 0; q < NC; ++q)
                        uu[u][q] = *reinterpret_cast<const v2f64 *>(
                            u3 + size_t(uint32_t(kk[u]) * row_bytes + lane_off) + q * 256);
#pragma unroll
                for (int u = 0; u < N; ++u)
#pragma unroll
                    for (int q = 0; q < NC; ++q) {
                        t[q][0] = fma(vv[u], uu[u][q][0], t[q][0]);
                        t[q][1] = fma(vv[u], uu[u][q][1], t[q][1]);
                    }
            };
            auto chunk = [&](auto T0, int n) {
                using I1 = std::integral_constant<int, 1>;
                using I2 = std::integral_constant<int, 2>;
                using I3 = std::integral_constant<int, 3>;
                using I4 = std::integral_constant<int, 4>;
                if (n >= 4) batch(T0, I4{});
                else if (n == 3) batch(T0, I3{});
                else if (n == 2) batch(T0, I2{});
                else batch(T0, I1{});
            };
            const int maxcnt = cur.maxcnt;
            chunk(std::integral_constant<int, 0>{}, maxcnt);
            if (maxcnt > 4) {
                chunk(std::integral_constant<int, 4>{}, maxcnt - 4);
                if (maxcnt > 8) {
                    chunk(std::integral_constant<int, 8>{}, maxcnt - 8);
                    if (maxcnt > 12) chunk(std::integral_constant<int, 12>{}, maxcnt - 12);
                }
            }
            v2f64 *dst = &pkt[r & 1][wave][0];
#pragma unroll
            for (int x = 0; x < APV; ++x) dst[x * 64 + lane] = cur.av[x];
#pragma unroll
            for (int q = 0; q < NC; ++q) dst[(APV + q) * 64 + lane] = v2f64{t[q][0], t[q][1]};
            if (lane == 0) {
                pkt_meta[r & 1][wave] = meta_cur;
                pkt_dest[r & 1][wave] = dest_cur;
            }
            cur = nxt;
            meta_cur = meta_nxt;
            dest_cur = dest_nxt;
            lds_barrier();
        }
    } else {
        // ------------------------------------------------------------------ consumer
        const int part = wave - NP;                    // columns part*32 + 2c, +1 of the row block
        v4f64 acc[PN][2];
#pragma unroll
        for (int p = 0; p < PN; ++p) acc[p][0] = acc[p][1] = v4f64{0.0, 0.0, 0.0, 0.0};
        const int64_t RR = int64_t(R2) * R3;
        lds_barrier();                                 // round 0 has been produced
        for (int r = 0; r < rounds; ++r) {
#pragma unroll
            for (int w = 0; w < NP; ++w) {
                if (ka + r * NP + w < kb) {
                    const v2f64 *src = &pkt[r & 1][w][0];
                    v2f64 av[APV];
#pragma unroll
                    for (int x = 0; x < APV; ++x) av[x] = src[x * 64 + lane];
                    const v2f64 tv = src[(APV + part) * 64 + lane];
                    const int32_t meta = __builtin_amdgcn_readfirstlane(pkt_meta[r & 1][w]);
#pragma unroll
                    for (int p = 0; p < PN; ++p) {
                        const double ap = av[p / 2][p % 2];
                        acc[p][0] = __builtin_amdgcn_mfma_f64_16x16x4f64(ap, tv[0], acc[p][0], 0, 0, 0);
                        acc[p][1] = __builtin_amdgcn_mfma_f64_16x16x4f64(ap, tv[1], acc[p][1], 0, 0, 0);
                    }
                    if (meta & 8) {
                        const int64_t dest = uniform64(pkt_dest[r & 1][w]);
                        double *base = dest >= 0 ? a.out + dest * RR : a.partial + (~dest) * RR;
                        // tile (p,q): accumulator register v of a lane holds row PN*(slot + 4v) + p,
                        // column part*32 + 2c + q; streaming stores, the block is never read here
#pragma unroll
                        for (int p = 0; p < PN; ++p)
#pragma unroll
                            for (int v = 0; v < 4; ++v) {
                                double *o = base + int64_t(PN * (slot + 4 * v) + p) * R3 + part * 32 + 2 * c;
                                __builtin_nontemporal_store(v2f64{acc[p][0][v], acc[p][1][v]}, reinterpret_cast<v2f64 *>(o));
                            }
#pragma unroll
                        for (int p = 0; p < PN; ++p) acc[p][0] = acc[p][1] = v4f64{0.0, 0.0, 0.0, 0.0};
                    }
                }
            }
            if (r + 1 < rounds) lds_barrier();
        }
    }
}

template <int PN, int NC>
static conststn_status launch_stream_np(const conststn_plan_s *plan, const Ttmc3StreamArgs &a, hipStream_t stream) {
    ProfScope prof(plan, stream);
    const dim3 grid(unsigned(plan->n_stream_wg));
    switch (plan->stream_producers) {
        case 2: ttmc3_stream_kernel<PN, NC, 2><<<grid, dim3(64 * (2 + NC)), 0, stream>>>(a); break;
        case 3: ttmc3_stream_kernel<PN, NC, 3><<<grid, dim3(64 * (3 + NC)), 0, stream>>>(a); break;
        case 6: ttmc3_stream_kernel<PN, NC, 6><<<grid, dim3(64 * (6 + NC)), 0, stream>>>(a); break;
        case 8: ttmc3_stream_kernel<PN, NC, 8><<<grid, dim3(64 * (8 + NC)), 0, stream>>>(a); break;
        default: ttmc3_stream_kernel<PN, NC, 4><<<grid, dim3(64 * (4 + NC)), 0, stream>>>(a); break;
    }
    return CONSTSTN_OK;
}

static conststn_status launch_stream(const conststn_plan_s *plan, const Ttmc3StreamArgs &a, hipStream_t stream) {
    const int pn = a.R2 / 16;
    if (a.R3 == 64) {
        switch (pn) {
            case 1: return launch_stream_np<1, 2>(plan, a, stream);
            case 2: return launch_stream_np<2, 2>(plan, a, stream);
            case 3: return launch_stream_np<3, 2>(plan, a, stream);
            default: return launch_stream_np<4, 2>(plan, a, stream);
        }
    }
    switch (pn) {
        case 1: return launch_stream_np<1, 1>(plan, a, stream);
        case 2: return launch_stream_np<2, 1>(plan, a, stream);
        case 3: return launch_stream_np<3, 1>(plan, a, stream);
        default: return launch_stream_np<4, 1>(plan, a, stream);
    }
}

template <int PN>
static conststn_status launch_mfma_pn(const conststn_plan_s *plan, const Ttmc3RowArgs &a, hipStream_t stream) {
    const int qt = a.R3 / 16;
    ProfScope prof(plan, stream);
    const dim3 grid(unsigned(a.n_items));
    // column tiles per wavefront: two where R3 allows it (vector accesses need the alignment)
    int qn = plan->ttmc3_qn;
    while (qn > 1 && (qt % qn != 0 ||
                      (reinterpret_cast<uintptr_t>(a.U3) | reinterpret_cast<uintptr_t>(a.out) |
                       reinterpret_cast<uintptr_t>(a.partial)) % (8u * unsigned(qn)) != 0))
        qn /= 2;
    if (qn == 4)
        ttmc3_mfma_kernel<PN, 4><<<grid, dim3(64 * (qt / 4)), 0, stream>>>(a);
    else if (qn == 2)
        ttmc3_mfma_kernel<PN, 2><<<grid, dim3(64 * (qt / 2)), 0, stream>>>(a);
    else
        ttmc3_mfma_kernel<PN, 1><<<grid, dim3(64 * qt), 0, stream>>>(a);
    return CONSTSTN_OK;
}

// Row blocks of slices made of several items: add the partial blocks in item order.
__global__ void __launch_bounds__(256)
ttmc_fixup_kernel(int64_t RR, const int32_t *__restrict__ split_slices,
                  const int64_t *__restrict__ split_first, const int32_t *__restrict__ split_count,
                  const int32_t *__restrict__ idx0, int compact, const double *__restrict__ partial,
                  double *__restrict__ out) {
    const int64_t q = blockIdx.x;
    const int64_t s = split_slices[q];
    const int64_t first = split_first[q];
    const int cnt = split_count[q];
    const int64_t row = compact ? s : int64_t(idx0[s]);
    for (int64_t e = int64_t(blockIdx.y) * blockDim.x + threadIdx.x; e < RR; e += int64_t(gridDim.y) * blockDim.x) {
        double sum = 0.0;
        for (int p = 0; p < cnt; ++p) sum += partial[(first + p) * RR + e];
        out[row * RR + e] = sum;
    }
}

conststn_status launch_ttmc_fixup(const conststn_plan_s *plan, double *out, hipStream_t stream, const double *partial) {
    if (plan->n_split == 0) return CONSTSTN_OK;
    if (!partial) partial = plan->partial.p;
    const int64_t RR = plan->row_elems;
    const unsigned gy = unsigned(std::min<int64_t>(div_up(RR, 256), 64));
    ttmc_fixup_kernel<<<dim3(unsigned(plan->n_split), gy), dim3(256), 0, stream>>>(
        RR, plan->split_slices.p, plan->split_first.p, plan->split_count.p, plan->X->idx[0].p,
        plan->compact ? 1 : 0, partial, out);
    CST_HIP(hipGetLastError());
    return CONSTSTN_OK;
}

// Partial row blocks for callers that may not allocate: one array per device, linked into the code
// object, shared by every call of conststn_execute_static on that device.
static __device__ __align__(256) unsigned char scratch[CONSTSTN_STATIC_SCRATCH_BYTES];
constexpr int kMaxDevices = 64;
static double *g_scratch_of_device[kMaxDevices];      // address of `scratch` on each device, looked up once

static conststn_status static_scratch(double **p) {
    int dev = 0;
    CST_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) { set_error("device ordinal %d beyond %d", dev, kMaxDevices); return CONSTSTN_EUNSUPPORTED; }
    if (!g_scratch_of_device[dev]) {
        void *addr = nullptr;
        CST_HIP(hipGetSymbolAddress(&addr, HIP_SYMBOL(scratch)));
        g_scratch_of_device[dev] = static_cast<double *>(addr);
    }
    *p = g_scratch_of_device[dev];
    return CONSTSTN_OK;
}

static conststn_status launch_ttmc3_with(const conststn_plan_s *plan, const double *const *dense, double *out,
                                         hipStream_t stream, double *partial);

conststn_status launch_ttmc3(const conststn_plan_s *plan, const double *const *dense, double *out,
                             hipStream_t stream) {
    return launch_ttmc3_with(plan, dense, out, stream, plan->partial.p);
}

conststn_status launch_ttmc3_static(const conststn_plan_s *plan, const double *const *dense, double *out,
                                    hipStream_t stream) {
    const int64_t need = plan->n_partials * plan->row_elems * int64_t(sizeof(double));
    if (need > int64_t(CONSTSTN_STATIC_SCRATCH_BYTES)) {
        set_error("the plan needs %lld bytes of partial row blocks, the static scratch area holds %lld: use conststn_execute",
                  (long long)need, (long long)CONSTSTN_STATIC_SCRATCH_BYTES);
        return CONSTSTN_EUNSUPPORTED;
    }
    double *ptr = nullptr;
    CST_TRY(static_scratch(&ptr));
    return launch_ttmc3_with(plan, dense, out, stream, ptr);
}

static conststn_status launch_ttmc3_with(const conststn_plan_s *plan, const double *const *dense, double *out,
                                         hipStream_t stream, double *partial) {
    const conststn_csf_s *X = plan->X;
    Ttmc3Args a{};
    a.n_items = plan->n_items;
    a.n_split = plan->n_split;
    a.R2 = plan->rank_of_level[1];
    a.R3 = plan->rank_of_level[2];
    a.ptr1 = X->ptr[1].p;
    a.idx0 = X->idx[0].p;
    a.idx1 = X->idx[1].p;
    a.idx2 = X->idx[2].p;
    a.vals = X->vals.p;
    a.items = plan->items.p;
    a.U2 = dense[plan->factor_of_level[1]];
    a.U3 = dense[plan->factor_of_level[2]];
    a.out = out;
    a.partial = partial;
    a.compact = plan->compact ? 1 : 0;
    if (a.R2 > 64 || a.R3 > 64) { set_error("TTMc ranks above 64 are not implemented"); return CONSTSTN_EUNSUPPORTED; }
    if (!plan->compact && X->nodes[0] < plan->out_rows)
        CST_TRY(zero_fill(out, plan->out_rows * plan->row_elems, stream));
    if (a.n_items == 0) return CONSTSTN_OK;
    if (plan->use_rows && plan->use_stream &&
        (reinterpret_cast<uintptr_t>(a.U2) | reinterpret_cast<uintptr_t>(a.U3) | reinterpret_cast<uintptr_t>(out)) % 16 == 0 &&
        int64_t(X->dims[X->mode_order[2]]) * a.R3 * 8 < (int64_t(1) << 32)) {
        Ttmc3StreamArgs sa{};
        sa.R2 = a.R2;
        sa.R3 = a.R3;
        sa.wg_kstep = plan->wg_kstep.p;
        sa.ksteps = plan->ksteps.p;
        sa.rows = plan->rows.p;
        sa.idx2 = a.idx2;
        sa.vals = a.vals;
        sa.U2 = a.U2;
        sa.U3 = a.U3;
        sa.out = out;
        sa.partial = a.partial;
        CST_TRY(launch_stream(plan, sa, stream));
        CST_HIP(hipGetLastError());
        return launch_ttmc_fixup(plan, out, stream, partial);
    }
    if (plan->use_rows) {
        Ttmc3RowArgs ra{};
        ra.n_items = plan->n_items;
        ra.R2 = a.R2;
        ra.R3 = a.R3;
        ra.rows = plan->rows.p;
        ra.idx0 = a.idx0;
        ra.idx2 = a.idx2;
        ra.vals = a.vals;
        ra.items = a.items;
        ra.U2 = a.U2;
        ra.U3 = a.U3;
        ra.out = out;
        ra.partial = a.partial;
        ra.compact = a.compact;
        switch (a.R2 / 16) {
            case 1: CST_TRY(launch_mfma_pn<1>(plan, ra, stream)); break;
            case 2: CST_TRY(launch_mfma_pn<2>(plan, ra, stream)); break;
            case 3: CST_TRY(launch_mfma_pn<3>(plan, ra, stream)); break;
            default: CST_TRY(launch_mfma_pn<4>(plan, ra, stream)); break;
        }
        CST_HIP(hipGetLastError());
        return launch_ttmc_fixup(plan, out, stream, partial);
    }
    const dim3 grid(unsigned(div_up(a.n_items, 4))), block(256);
    {
        ProfScope prof(plan, stream);
        if (a.R2 <= 8) ttmc3_kernel<8><<<grid, block, 0, stream>>>(a);
        else if (a.R2 <= 16) ttmc3_kernel<16><<<grid, block, 0, stream>>>(a);
        else if (a.R2 <= 32) ttmc3_kernel<32><<<grid, block, 0, stream>>>(a);
        else ttmc3_kernel<64><<<grid, block, 0, stream>>>(a);
    }
    CST_HIP(hipGetLastError());
    return launch_ttmc_fixup(plan, out, stream, partial);
}

}  // namespace cst
