// Fused three-tensor network of Sec. 1:  Z[i,m] = sum_{j,k,l} U[i,j,k] V[j,l] W[k,l,m]
// evaluated as the tree (U.V).W:
//     T[i,k,l] = U[i,k,j] V[j,l]   loops i,k,j,l      (U stored i>k>j)
//     Z[i,m]   = T[i,k,l] W[k,l,m] loops i,k,l,m      (W stored k>l>m)
// fused on the loops i and k, so T shrinks to one length-L vector per (i,k) fiber of U and no
// full intermediate is formed.
//
// Baseline kernel: one workgroup per root slice i of U.  For each (i,k) fiber the threads
// build T[0..L) in LDS (thread = l, coalesced rows of V), then the wavefronts walk the (k,l)
// fibers of W below root k: lanes take the m leaves and add T[l]*W into a per-wavefront copy
// of Z_i in LDS (no atomics: leaves of one fiber have distinct m).  The copies are added in
// fixed order at the end, so results are bit-reproducible.
#include <type_traits>

#include "plan.hpp"

namespace cst {

struct Sptn3Args {
    int64_t slices;
    int64_t L, M;
    const int64_t *uptr0, *uptr1;
    const int32_t *uidx0, *uidx1, *uidx2;
    const double *uvals;
    const int64_t *wptr0, *wptr1;
    const int32_t *widx1, *widx2;
    const double *wvals;
    const int64_t *w_root_of_k;
    const double *V;
    double *out;
    int compact;
};

__global__ void __launch_bounds__(256)
sptn3_kernel(Sptn3Args a) {
    extern __shared__ double lds[];
    double *T = lds;                         // L
    double *Zw = lds + a.L;                  // 4 x M
    const int64_t s = blockIdx.x;
    const int tid = threadIdx.x, wave = tid / 64, lane = tid % 64;
    const int64_t L = a.L, M = a.M;
    for (int64_t e = tid; e < 4 * M; e += 256) Zw[e] = 0.0;
    const int64_t fa = a.uptr0[s], fb = a.uptr0[s + 1];
    for (int64_t f = fa; f < fb; ++f) {
        const int32_t k = a.uidx1[f];
        const int64_t root = a.w_root_of_k[k];
        if (root < 0) continue;                                   // W has nothing at this k
        const int64_t na = a.uptr1[f], nb = a.uptr1[f + 1];
        __syncthreads();                                          // T free for reuse
        for (int64_t l = tid; l < L; l += 256) {
            double t = 0.0;
            for (int64_t n = na; n < nb; ++n)
                t = fma(a.uvals[n], a.V[int64_t(a.uidx2[n]) * L + l], t);
            T[l] = t;
        }
        __syncthreads();
        const int64_t ga = a.wptr0[root], gb = a.wptr0[root + 1];
        double *Z = Zw + int64_t(wave) * M;
        for (int64_t g = ga + wave; g < gb; g += 4) {
            const double tl = T[a.widx1[g]];
            const int64_t ea = a.wptr1[g], eb = a.wptr1[g + 1];
            for (int64_t e = ea + lane; e < eb; e += 64) {
                const int32_t m = a.widx2[e];
                Z[m] = fma(tl, a.wvals[e], Z[m]);
            }
        }
    }
    __syncthreads();
    const int64_t row = a.compact ? s : int64_t(a.uidx0[s]);
    for (int64_t m = tid; m < M; m += 256)
        a.out[row * M + m] = ((Zw[m] + Zw[M + m]) + Zw[2 * M + m]) + Zw[3 * M + m];
}

// ---- tiled kernel: both stages on the fp64 matrix cores --------------------------------------
//
// Sixteen root slices of U are taken together (a "group"); a workgroup owns one group and one
// chunk of the k range and walks the k values present in any of its slices (a 16-way merge of
// the slices' level-1 lists).  For one k:
//   1. the j indices of the up to sixteen (i,k) fibers are merged through a bit mask in LDS into
//      their sorted union; the fibers are scattered into a dense LDS tile Uc[union rank][i]
//      (zero where a slice has no such j) -- at most kCap union rows per pass, more passes if
//      the union is longer (each pass is a unit of its own: the consumer is linear in T);
//   2. producer, per tile of 16 l values:  T^t[l, i] = sum_j V[j, l] Uc[j, i]  as 16x16x4 matrix
//      instructions, A = V[j_s, l0 + c] (row segments of 128 B from L2), B = Uc[j_s, c];
//   3. consumer: the accumulator registers of T^t are exactly the B operand layout, so
//      Z^t[m, i] += sum_l W[l, m] T^t[l, i]  follows without any data movement, A = the dense
//      16 x 16 tiles of W that the plan prepared (only tiles that hold a nonzero).
// A wavefront owns every fourth l tile and accumulates its own Z^t (all m tiles) in registers
// while it works on one k; after each k the four wavefronts add theirs, one after the other, to
// the group's Z^t in LDS, and the partial results of the k chunks are added by a fix-up kernel in
// chunk order, so results are bit-reproducible.  One wavefront per SIMD: latency is hidden by a
// software pipeline (kRing batches of four K-steps in flight) that runs across l tile boundaries;
// every load in it is unconditional (clamped addresses), and the W tiles of the current l tile
// are parked in a per-lane LDS area (indexable at run time, which registers are not).
// The zero entries of Uc and of the W tiles multiply real factor values, so V must be finite.

typedef double v4d __attribute__((ext_vector_type(4)));
typedef double v2d __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(3))) v2d lds_v2d;

constexpr int kCap = 320;             // union rows of Uc per pass (40 KB)
constexpr int kStage = 6;             // W tiles parked in LDS per l tile and wavefront
constexpr int kBatch = 4;             // K-steps per pipeline batch
constexpr int kHeld = 16;             // leaves per lane kept in registers between mask and scatter
constexpr int kRing = 3;              // batches in flight (loads issued kRing - 1 batches ahead)

struct Sptn3TileArgs {
    int64_t slices, L, M, LT;
    int MT, nwords, n_groups, n_kc;
    int64_t k_per;
    const int64_t *uptr0, *uptr1;
    const int32_t *uidx0, *uidx1, *uidx2;
    const double *uvals;
    const int64_t *w_root_of_k;
    const uint32_t *wmask, *wfirst;
    const double *wtiles;
    uint32_t zero_tile;
    const double *V;
    double *out, *partial;
    int compact, xcd_ranges;
    const int32_t *wg_order;               // workgroup -> (k chunk, group) pair, heaviest pairs first (or null)
};

__device__ inline int64_t lower_bound_i32(const int32_t *__restrict__ a, int64_t lo, int64_t hi, int64_t key) {
    while (lo < hi) {
        const int64_t mid = (lo + hi) >> 1;
        if (int64_t(a[mid]) < key) lo = mid + 1; else hi = mid;
    }
    return lo;
}

struct SpPipe {
    double Vr[kRing][kBatch], Ur[kRing][kBatch];
    int32_t Jr[kRing][kBatch];
    v2d Wr[kRing][2];
};

__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1)))
sptn3_tiled_kernel(Sptn3TileArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    double *Uc = reinterpret_cast<double *>(smem);                        // kCap x 16
    double *Wb = Uc + kCap * 16;                                          // 4 x kStage x 256
    double *Zs = Wb + 4 * kStage * 256;                                   // MT x 16 x 16: Z^t[m][i]
    int32_t *jl = reinterpret_cast<int32_t *>(Zs + a.MT * 256);           // kCap: row offset j*L
    uint32_t *mask = reinterpret_cast<uint32_t *>(jl + kCap);             // nwords
    int32_t *wpre = reinterpret_cast<int32_t *>(mask + a.nwords);         // nwords
    int32_t *scan = wpre + a.nwords;                                      // 8

    const int tid = threadIdx.x, lane = tid & 63, slot = lane >> 4, c = lane & 15;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);          // uniform, and known to be
    // Workgroups are dealt to the 8 XCDs round-robin.  Optionally each XCD gets a contiguous range
    // of (k chunk, group) pairs instead, so that the workgroups sharing one L2 walk the same k
    // values over neighbouring groups (same W tiles, largely the same rows of V).
    const int n_wg = a.n_groups * a.n_kc, per_xcd = (n_wg + 7) / 8;
    if (int(blockIdx.x) >= n_wg && !a.xcd_ranges) return;
    const int logical = a.xcd_ranges ? (int(blockIdx.x) % 8) * per_xcd + int(blockIdx.x) / 8
                                     : (a.wg_order ? a.wg_order[blockIdx.x] : int(blockIdx.x));
    if (logical >= n_wg) return;
    const int group = logical % a.n_groups, kc = logical / a.n_groups;
    const int64_t s0 = int64_t(group) * kSpGroup;
    const int64_t k_lo = int64_t(kc) * a.k_per, k_hi = k_lo + a.k_per;
    const int64_t L = a.L;
    const int L32 = int(a.L);
    const char *Vbytes = reinterpret_cast<const char *>(a.V);
    const uint32_t lane16 = uint32_t(lane) * 16u;
    const int nwords = a.nwords;
    double *Wbw = Wb + wave * (kStage * 256);
    // the same area through an LDS-typed pointer, so that reads of it stay LDS instructions
    const lds_v2d *Wpark = (const lds_v2d *)(Wbw);

    // lane c (in each of the four lane rows) holds the cursor of slice s0 + c
    int64_t cur = 0, end = 0;
    if (s0 + c < a.slices) {
        const int64_t na = a.uptr0[s0 + c], nb = a.uptr0[s0 + c + 1];
        cur = lower_bound_i32(a.uidx1, na, nb, k_lo);
        end = lower_bound_i32(a.uidx1, cur, nb, k_hi);
    }
    for (int x = tid; x < a.MT * 256; x += 256) Zs[x] = 0.0;

    const int NTw = a.LT > wave ? int((a.LT - wave + 3) >> 2) : 0;       // l tiles of this wavefront

    for (;;) {
        const int32_t kk = cur < end ? a.uidx1[cur] : INT32_MAX;
        int32_t kmin = kk;
        kmin = min(kmin, __shfl_xor(kmin, 8, 16));
        kmin = min(kmin, __shfl_xor(kmin, 4, 16));
        kmin = min(kmin, __shfl_xor(kmin, 2, 16));
        kmin = min(kmin, __shfl_xor(kmin, 1, 16));
        kmin = __builtin_amdgcn_readfirstlane(kmin);
        if (kmin == INT32_MAX) break;
        const bool has = kk == kmin;
        const int64_t f = cur;
        cur += has ? 1 : 0;
        const int64_t root = a.w_root_of_k[kmin];                         // same address in every lane
        if (root < 0) continue;                                           // W has nothing at this k
        int64_t la = 0, lb = 0;
        if (has) { la = a.uptr1[f]; lb = a.uptr1[f + 1]; }
        // this lane row scatters the fiber of slice 4*wave + slot
        const int irow = 4 * wave + slot;
        const int64_t ea = __shfl(la, irow), eb = __shfl(lb, irow);

        __syncthreads();                                                  // LDS of the previous k is free
        for (int w = tid; w < nwords; w += 256) mask[w] = 0u;
        __syncthreads();
        // the first kHeld leaves per lane stay in registers for the scatter below: all their loads
        // are in flight together instead of one memory round trip per loop iteration
        int32_t jheld[kHeld];
        double vheld[kHeld];
#pragma unroll
        for (int h = 0; h < kHeld; ++h) {
            const int64_t e = ea + c + 16 * h;
            jheld[h] = e < eb ? a.uidx2[e] : -1;
            vheld[h] = e < eb ? a.uvals[e] : 0.0;
        }
#pragma unroll
        for (int h = 0; h < kHeld; ++h)
            if (jheld[h] >= 0) atomicOr(&mask[jheld[h] >> 5], 1u << (jheld[h] & 31));
        for (int64_t e = ea + c + 16 * kHeld; e < eb; e += 16) {
            const int32_t j = a.uidx2[e];
            atomicOr(&mask[j >> 5], 1u << (j & 31));
        }
        __syncthreads();
        {   // exclusive prefix of the set-bit counts of the mask words (thread t: words 4t .. 4t+3)
            int cnt[4], mine = 0;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int w = 4 * tid + q;
                cnt[q] = w < nwords ? __popc(mask[w]) : 0;
                mine += cnt[q];
            }
            int incl = mine;
#pragma unroll
            for (int d = 1; d < 64; d <<= 1) {
                const int up = __shfl_up(incl, d);
                if (lane >= d) incl += up;
            }
            if (lane == 63) scan[wave] = incl;
            __syncthreads();
            int base = 0;
            for (int w = 0; w < wave; ++w) base += scan[w];
            int run = base + incl - mine;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int w = 4 * tid + q;
                if (w < nwords) wpre[w] = run;
                run += cnt[q];
            }
        }
        const int n_union = __builtin_amdgcn_readfirstlane(scan[0] + scan[1] + scan[2] + scan[3]);
        __syncthreads();

        // Prepare one pass: union rows [p0, p0 + np) -> Uc rows and j offsets.  The first pass takes
        // the leaves held in registers (they are dead before the matrix stages start); later passes
        // re-read the fibers.
        auto prepare = [&](int p0, int np, int npad, auto first) {
            for (int x = tid; x < npad * 16; x += 256) Uc[x] = 0.0;
            if (tid < npad - np) jl[np + tid] = 0;
            for (int w = tid; w < nwords; w += 256) {
                uint32_t m = mask[w];
                int r = wpre[w] - p0;
                while (m) {
                    const int b = __builtin_ctz(m);
                    m &= m - 1u;
                    if (r >= 0 && r < np) jl[r] = int32_t(int64_t(w * 32 + b) * L);
                    ++r;
                }
            }
            __syncthreads();
            auto place = [&](int32_t j, double v) {
                const int r = wpre[j >> 5] + __popc(mask[j >> 5] & ((1u << (j & 31)) - 1u)) - p0;
                if (r >= 0 && r < np) Uc[r * 16 + irow] = v;
            };
            if (decltype(first)::value) {
#pragma unroll
                for (int h = 0; h < kHeld; ++h)
                    if (jheld[h] >= 0) place(jheld[h], vheld[h]);
            }
            for (int64_t e = ea + c + (decltype(first)::value ? 16 * kHeld : 0); e < eb; e += 16)
                place(a.uidx2[e], a.uvals[e]);
            __syncthreads();
        };
        int p0 = 0;
        int np = min(kCap, n_union);
        int npad = (np + 4 * kBatch - 1) & ~(4 * kBatch - 1);                 // whole batches
        if (n_union > 0) prepare(0, np, npad, std::true_type{});
        while (p0 < n_union) {
            // ---- the two matrix stages over this wavefront's l tiles, 64 tiles per round ----
            v4d accZ[kSpMaxMTiles];
#pragma unroll
            for (int mt = 0; mt < kSpMaxMTiles; ++mt) accZ[mt] = v4d{0.0, 0.0, 0.0, 0.0};
            const int nBt = npad / (4 * kBatch);                          // batches per l tile
            for (int tr = 0; tr < NTw; tr += 64) {
                const int NT = min(64, NTw - tr);
                // lane t holds mask and first tile of its t-th l tile of this round
                uint32_t mreg = 0u, freg = a.zero_tile;
                if (lane < NT) {
                    const int64_t cell = root * a.LT + (wave + 4 * (tr + lane));
                    mreg = a.wmask[cell];
                    freg = mreg ? a.wfirst[cell] : a.zero_tile;
                }
                const int TB = NT * nBt;
                SpPipe P;
                v4d accT0 = v4d{0.0, 0.0, 0.0, 0.0}, accT1 = accT0;
                // stream positions: (t, q) = (l tile of the round, batch inside it)
                int t0 = 0, q0 = 0;                                       // batch being consumed
                int t2 = 0, q2 = 0;                                       // batch whose V/U/W loads are issued
                int q3 = 0;                                               // batch whose j offsets are read

                auto read_j = [&](int32_t (&J)[kBatch]) {
#pragma unroll
                    for (int ks = 0; ks < kBatch; ++ks) J[ks] = jl[q3 * (4 * kBatch) + ks * 4 + slot];
                    q3 = q3 + 1 == nBt ? 0 : q3 + 1;
                };
                auto issue = [&](const int32_t (&J)[kBatch], double (&Vv)[kBatch], double (&Uu)[kBatch], v2d (&Ww)[2]) {
                    const int tt = min(t2, NT - 1);
                    const int col = min(16 * (wave + 4 * (tr + tt)) + c, L32 - 1);
                    // 32-bit element offsets against the scalar base of V (J L < 2^29, checked by the plan):
                    // one vector instruction per address
#pragma unroll
                    for (int ks = 0; ks < kBatch; ++ks) {
                        Vv[ks] = *reinterpret_cast<const double *>(Vbytes + (uint32_t(J[ks] + col) << 3));
                        Uu[ks] = Uc[q2 * (64 * kBatch) + ks * 64 + lane];
                    }
                    const uint32_t m2 = __builtin_amdgcn_readlane(mreg, tt);
                    const uint32_t f2 = __builtin_amdgcn_readlane(freg, tt);
                    const int last = max(__popc(m2) - 1, 0);
                    const int tq = min(min(q2, kStage - 1), last);            // all scalar
                    const char *tb = reinterpret_cast<const char *>(a.wtiles + (int64_t(f2) + tq) * 256);
                    Ww[0] = *reinterpret_cast<const v2d *>(tb + lane16);
                    Ww[1] = *reinterpret_cast<const v2d *>(tb + lane16 + 1024);
                    if (q2 + 1 == nBt) { q2 = 0; ++t2; } else ++q2;
                };
                auto consume = [&](int b, const double (&Vv)[kBatch], const double (&Uu)[kBatch], const v2d (&Ww)[2]) {
                    // park the W tile that came with this batch
                    double *wp = Wbw + min(q0, kStage - 1) * 256 + lane * 2;
                    *reinterpret_cast<v2d *>(wp) = Ww[0];
                    *reinterpret_cast<v2d *>(wp + 128) = Ww[1];
                    if (b < TB) {
                        accT0 = __builtin_amdgcn_mfma_f64_16x16x4f64(Vv[0], Uu[0], accT0, 0, 0, 0);
                        accT1 = __builtin_amdgcn_mfma_f64_16x16x4f64(Vv[1], Uu[1], accT1, 0, 0, 0);
                        accT0 = __builtin_amdgcn_mfma_f64_16x16x4f64(Vv[2], Uu[2], accT0, 0, 0, 0);
                        accT1 = __builtin_amdgcn_mfma_f64_16x16x4f64(Vv[3], Uu[3], accT1, 0, 0, 0);
                        if (q0 + 1 == nBt) {
                            // consumer: Z^t += W^t . T^t for the m tiles present below this l tile
                            const v4d T = accT0 + accT1;
                            const uint32_t m0 = __builtin_amdgcn_readlane(mreg, t0);
                            const uint32_t f0 = __builtin_amdgcn_readlane(freg, t0);
                            const int have = __popc(m0);
                            int staged = min(nBt, kStage);                // tiles parked so far
                            int first_p = 0;                              // tile held by slot 0
                            for (;;) {
                                int p = 0;
#pragma unroll
                                for (int mt = 0; mt < kSpMaxMTiles; ++mt) {
                                    if ((m0 >> mt) & 1u) {
                                        if (p >= first_p && p < first_p + staged) {
                                            const lds_v2d *rp = Wpark + ((p - first_p) * 128 + lane);
                                            const v2d w0 = rp[0], w1 = rp[64];
                                            v4d z = accZ[mt];
                                            z = __builtin_amdgcn_mfma_f64_16x16x4f64(w0.x, T.x, z, 0, 0, 0);
                                            z = __builtin_amdgcn_mfma_f64_16x16x4f64(w0.y, T.y, z, 0, 0, 0);
                                            z = __builtin_amdgcn_mfma_f64_16x16x4f64(w1.x, T.z, z, 0, 0, 0);
                                            z = __builtin_amdgcn_mfma_f64_16x16x4f64(w1.y, T.w, z, 0, 0, 0);
                                            accZ[mt] = z;
                                        }
                                        ++p;
                                    }
                                }
                                first_p += staged;
                                if (first_p >= have) break;               // the usual case: one round
                                // more tiles below this l tile than were parked (rare): fetch the
                                // next ones and park them, then go round again
                                staged = min(kStage, have - first_p);
                                for (int sl = 0; sl < staged; ++sl) {
                                    const double *tp = a.wtiles + (int64_t(f0) + first_p + sl) * 256 + lane * 2;
                                    const v2d w0 = *reinterpret_cast<const v2d *>(tp);
                                    const v2d w1 = *reinterpret_cast<const v2d *>(tp + 128);
                                    double *wp = Wbw + sl * 256 + lane * 2;
                                    *reinterpret_cast<v2d *>(wp) = w0;
                                    *reinterpret_cast<v2d *>(wp + 128) = w1;
                                }
                            }
                            accT0 = v4d{0.0, 0.0, 0.0, 0.0};
                            accT1 = accT0;
                            q0 = 0;
                            ++t0;
                        } else {
                            ++q0;
                        }
                    }
                };

                if (TB > 0) {
#pragma unroll
                    for (int u = 0; u < kRing; ++u) read_j(P.Jr[u]);
#pragma unroll
                    for (int u = 0; u < kRing - 1; ++u) issue(P.Jr[u], P.Vr[u], P.Ur[u], P.Wr[u]);
                    for (int b = 0; b < TB; b += kRing) {
#pragma unroll
                        for (int u = 0; u < kRing; ++u) {
                            const int su = (u + kRing - 1) % kRing;
                            issue(P.Jr[su], P.Vr[su], P.Ur[su], P.Wr[su]);
                            read_j(P.Jr[u]);
                            consume(b + u, P.Vr[u], P.Ur[u], P.Wr[u]);
                        }
                    }
                }
            }
            // add this k's contribution to the group's Z^t, wavefront after wavefront
            for (int w = 0; w < 4; ++w) {
                if (wave == w) {
#pragma unroll
                    for (int mt = 0; mt < kSpMaxMTiles; ++mt) {
                        if (mt < a.MT) {
#pragma unroll
                            for (int v = 0; v < 4; ++v) Zs[(16 * mt + slot + 4 * v) * 16 + c] += accZ[mt][v];
                        }
                    }
                }
                __syncthreads();
            }
            p0 += kCap;
            if (p0 < n_union) {
                np = min(kCap, n_union - p0);
                npad = (np + 4 * kBatch - 1) & ~(4 * kBatch - 1);
                prepare(p0, np, npad, std::false_type{});
            }
        }
    }

    // ---- store the group's rows ----------------------------------------------------------------
    __syncthreads();
    const int64_t M = a.M;
    for (int64_t x = tid; x < 16 * M; x += 256) {
        const int64_t i = x / M, m = x - i * M;
        const int64_t s = s0 + i;
        if (s >= a.slices) break;
        const double z = Zs[m * 16 + i];
        if (a.n_kc == 1) {
            const int64_t row = a.compact ? s : int64_t(a.uidx0[s]);
            a.out[row * M + m] = z;
        } else {
            a.partial[(int64_t(kc) * a.slices + s) * M + m] = z;
        }
    }
}

// ---- tiled kernel with two wavefronts per SIMD ------------------------------------------------
// The kernel above keeps Z^t for all m tiles of its l tiles in 200 accumulator registers, which
// leaves room for one wavefront per SIMD; fp64 matrix instructions then issue at two thirds of
// the rate two wavefronts reach, and every vector instruction in between costs three times as
// much.  Here a workgroup has eight wavefronts (two per SIMD).  The producer is unchanged: in a
// *round* wavefront w computes T^t of l tile 8 r + w.  The consumer is split by m instead of by
// l: wavefront w owns the m tiles w, w + 8, w + 16, w + 24 (four accumulator tiles, kept in
// registers across all k of the workgroup), the eight T^t of a round go through LDS, and after
// a barrier every wavefront multiplies its own W tiles of all eight l tiles.  The W tiles of a
// round are fetched by the eight wavefronts in turn, one per producer batch, and parked in a pool
// of LDS slots shared by the workgroup (slot = rank of the tile among the round's tiles); what
// does not fit, or exceeds eight tiles per batch, is fetched when it is used.
constexpr int kOwnWaves = 8;
constexpr int kRingO = 2;                                             // batches in flight in this kernel
constexpr int kOwnZ = (kSpMaxMTiles + kOwnWaves - 1) / kOwnWaves;       // accumulator tiles per wavefront
constexpr int kPool = 48;                                             // W tiles parked per round

struct SpPipeO {
    double Vr[kRingO][kBatch], Ur[kRingO][kBatch];
    int32_t Jr[kRingO][kBatch];
    v2d Wr[kRingO][2];
    int Sr[kRingO];                                                    // pool slot of the W tile (-1: not parked)
};

__global__ void __launch_bounds__(64 * kOwnWaves) __attribute__((amdgpu_waves_per_eu(2, 2)))
sptn3_owned_kernel(Sptn3TileArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    double *Uc = reinterpret_cast<double *>(smem);                        // kCap x 16
    double *Pool = Uc + kCap * 16;                                        // kPool x 256
    double *Tx = Pool + kPool * 256;                                      // 8 x 256: T^t of the round's l tiles
    int32_t *jl = reinterpret_cast<int32_t *>(Tx + kOwnWaves * 256);      // kCap: row offset j*L
    uint32_t *mask = reinterpret_cast<uint32_t *>(jl + kCap);             // nwords
    int32_t *wpre = reinterpret_cast<int32_t *>(mask + a.nwords);         // nwords
    int32_t *scan = wpre + a.nwords;                                      // 8

    const int tid = threadIdx.x, lane = tid & 63, slot = lane >> 4, c = lane & 15;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n_wg = a.n_groups * a.n_kc, per_xcd = (n_wg + 7) / 8;
    if (int(blockIdx.x) >= n_wg && !a.xcd_ranges) return;
    const int logical = a.xcd_ranges ? (int(blockIdx.x) % 8) * per_xcd + int(blockIdx.x) / 8
                                     : (a.wg_order ? a.wg_order[blockIdx.x] : int(blockIdx.x));
    if (logical >= n_wg) return;
    const int group = logical % a.n_groups, kc = logical / a.n_groups;
    const int64_t s0 = int64_t(group) * kSpGroup;
    const int64_t k_lo = int64_t(kc) * a.k_per, k_hi = k_lo + a.k_per;
    const int64_t L = a.L;
    const int L32 = int(a.L);
    const int LT = int(a.LT);
    const char *Vbytes = reinterpret_cast<const char *>(a.V);
    const uint32_t lane16 = uint32_t(lane) * 16u;
    const int nwords = a.nwords;
    const lds_v2d *PoolV = (const lds_v2d *)(Pool);
    const lds_v2d *TxV = (const lds_v2d *)(Tx);
    // m tiles of this wavefront, as a mask over the 25
    uint32_t own = 0u;
#pragma unroll
    for (int x = 0; x < kOwnZ; ++x)
        if (wave + kOwnWaves * x < a.MT) own |= 1u << (wave + kOwnWaves * x);

    // lane c (in each of the four lane rows) holds the cursor of slice s0 + c
    int64_t cur = 0, end = 0;
    if (s0 + c < a.slices) {
        const int64_t na = a.uptr0[s0 + c], nb = a.uptr0[s0 + c + 1];
        cur = lower_bound_i32(a.uidx1, na, nb, k_lo);
        end = lower_bound_i32(a.uidx1, cur, nb, k_hi);
    }
    v4d accZ[kOwnZ];
#pragma unroll
    for (int x = 0; x < kOwnZ; ++x) accZ[x] = v4d{0.0, 0.0, 0.0, 0.0};
    const int rounds = (LT + kOwnWaves - 1) / kOwnWaves;

    for (;;) {
        const int32_t kk = cur < end ? a.uidx1[cur] : INT32_MAX;
        int32_t kmin = kk;
        kmin = min(kmin, __shfl_xor(kmin, 8, 16));
        kmin = min(kmin, __shfl_xor(kmin, 4, 16));
        kmin = min(kmin, __shfl_xor(kmin, 2, 16));
        kmin = min(kmin, __shfl_xor(kmin, 1, 16));
        kmin = __builtin_amdgcn_readfirstlane(kmin);
        if (kmin == INT32_MAX) break;
        const bool has = kk == kmin;
        const int64_t f = cur;
        cur += has ? 1 : 0;
        const int64_t root = a.w_root_of_k[kmin];                         // same address in every lane
        if (root < 0) continue;                                           // W has nothing at this k
        int64_t la = 0, lb = 0;
        if (has) { la = a.uptr1[f]; lb = a.uptr1[f + 1]; }
        // two lane rows per slice: slice 2*wave + slot/2, leaves of parity slot%2
        const int irow = 2 * wave + (slot >> 1), half = slot & 1;
        const int64_t ea = __shfl(la, irow), eb = __shfl(lb, irow);
        __syncthreads();                                                  // LDS of the previous k is free
        for (int w = tid; w < nwords; w += 64 * kOwnWaves) mask[w] = 0u;
        __syncthreads();
        // the first kHeldO leaves per lane stay in registers for the scatter below
        constexpr int kHeldO = kHeld / 2;
        int32_t jheld[kHeldO];
        double vheld[kHeldO];
#pragma unroll
        for (int h = 0; h < kHeldO; ++h) {
            const int64_t e = ea + c + 16 * (2 * h + half);
            jheld[h] = e < eb ? a.uidx2[e] : -1;
            vheld[h] = e < eb ? a.uvals[e] : 0.0;
        }
#pragma unroll
        for (int h = 0; h < kHeldO; ++h)
            if (jheld[h] >= 0) atomicOr(&mask[jheld[h] >> 5], 1u << (jheld[h] & 31));
        for (int64_t e = ea + c + 16 * (2 * kHeldO + half); e < eb; e += 32) {
            const int32_t j = a.uidx2[e];
            atomicOr(&mask[j >> 5], 1u << (j & 31));
        }
        __syncthreads();
        {   // exclusive prefix of the set-bit counts of the mask words (thread t: words 2t, 2t+1)
            int cnt[2], mine = 0;
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                const int w = 2 * tid + q;
                cnt[q] = w < nwords ? __popc(mask[w]) : 0;
                mine += cnt[q];
            }
            int incl = mine;
#pragma unroll
            for (int d = 1; d < 64; d <<= 1) {
                const int up = __shfl_up(incl, d);
                if (lane >= d) incl += up;
            }
            if (lane == 63) scan[wave] = incl;
            __syncthreads();
            int base = 0;
            for (int w = 0; w < wave; ++w) base += scan[w];
            int run = base + incl - mine;
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                const int w = 2 * tid + q;
                if (w < nwords) wpre[w] = run;
                run += cnt[q];
            }
        }
        int n_union = 0;
#pragma unroll
        for (int w = 0; w < kOwnWaves; ++w) n_union += scan[w];
        n_union = __builtin_amdgcn_readfirstlane(n_union);
        __syncthreads();

        auto prepare = [&](int p0, int np, int npad, auto first) {
            for (int x = tid; x < npad * 16; x += 64 * kOwnWaves) Uc[x] = 0.0;
            if (tid < npad - np) jl[np + tid] = 0;
            for (int w = tid; w < nwords; w += 64 * kOwnWaves) {
                uint32_t m = mask[w];
                int r = wpre[w] - p0;
                while (m) {
                    const int b = __builtin_ctz(m);
                    m &= m - 1u;
                    if (r >= 0 && r < np) jl[r] = int32_t(int64_t(w * 32 + b) * L);
                    ++r;
                }
            }
            __syncthreads();
            auto place = [&](int32_t j, double v) {
                const int r = wpre[j >> 5] + __popc(mask[j >> 5] & ((1u << (j & 31)) - 1u)) - p0;
                if (r >= 0 && r < np) Uc[r * 16 + irow] = v;
            };
            if (decltype(first)::value) {
#pragma unroll
                for (int h = 0; h < kHeldO; ++h)
                    if (jheld[h] >= 0) place(jheld[h], vheld[h]);
            }
            for (int64_t e = ea + c + 16 * ((decltype(first)::value ? 2 * kHeldO : 0) + half); e < eb; e += 32)
                place(a.uidx2[e], a.uvals[e]);
            __syncthreads();
        };
        int p0 = 0;
        int np = min(kCap, n_union);
        int npad = (np + 4 * kBatch - 1) & ~(4 * kBatch - 1);                 // whole batches
        if (n_union > 0) prepare(0, np, npad, std::true_type{});
        while (p0 < n_union) {
            const int nBt = npad / (4 * kBatch);                          // batches per l tile
            for (int r0 = 0; r0 < rounds; r0 += 8) {                      // 8 rounds = 64 l tiles: one mask per lane
                const int NR = min(8, rounds - r0);
                uint32_t mreg = 0u, freg = a.zero_tile;
                if (8 * r0 + lane < LT) {
                    const int64_t cell = root * a.LT + (8 * r0 + lane);
                    mreg = a.wmask[cell];
                    freg = mreg ? a.wfirst[cell] : a.zero_tile;
                }
                // tiles of the lane's round before the lane's l tile (rounds are groups of 8 lanes)
                int preg;
                {
                    const int pc = __popc(mreg);
                    int incl = pc;
#pragma unroll
                    for (int d = 1; d < 8; d <<= 1) {
                        const int up = __shfl_up(incl, d, 8);
                        if ((lane & 7) >= d) incl += up;
                    }
                    preg = incl - pc;
                }
                const int TB = NR * nBt;
                SpPipeO P;
                v4d accT0 = v4d{0.0, 0.0, 0.0, 0.0}, accT1 = accT0;
                int t0 = 0, q0 = 0;                                       // batch being consumed: (round, batch in it)
                int t2 = 0, q2 = 0;                                       // batch whose V/U/W loads are issued
                int q3 = 0;                                               // batch whose j offsets are read
                // The W tiles of round t2, in the order (l tile, m tile), are fetched by the eight wavefronts
                // in turn: tile n by wavefront n % 8 with its batch n / 8, into pool slot n.

                auto read_j = [&](int32_t (&J)[kBatch]) {
#pragma unroll
                    for (int ks = 0; ks < kBatch; ++ks) J[ks] = jl[q3 * (4 * kBatch) + ks * 4 + slot];
                    q3 = q3 + 1 == nBt ? 0 : q3 + 1;
                };
                auto issue = [&](const int32_t (&J)[kBatch], double (&Vv)[kBatch], double (&Uu)[kBatch], v2d (&Ww)[2], int &S) {
                    const int tt = min(t2, NR - 1);
                    const int col = min(16 * (8 * (r0 + tt) + wave) + c, L32 - 1);
#pragma unroll
                    for (int ks = 0; ks < kBatch; ++ks) {
                        Vv[ks] = *reinterpret_cast<const double *>(Vbytes + (uint32_t(J[ks] + col) << 3));
                        Uu[ks] = Uc[q2 * (64 * kBatch) + ks * 64 + lane];
                    }
                    // W tile n = wave + 8 q2 of round t2, found without a loop or a branch: the l tile it
                    // lies under is the last lane of the round's group whose prefix does not exceed n
                    const int n = wave + kOwnWaves * q2;
                    const uint64_t below = __ballot((lane >> 3) == tt && n >= preg);
                    const int ln = 8 * tt + __popcll(below) - 1;          // the group's first lane always counts
                    const uint32_t full = __builtin_amdgcn_readlane(mreg, ln);
                    const int base = __builtin_amdgcn_readlane(preg, ln);
                    const bool ok = t2 < NR && n < base + __popc(full) && n < kPool;
                    const uint32_t tile = ok ? __builtin_amdgcn_readlane(freg, ln) + uint32_t(n - base) : a.zero_tile;
                    S = ok ? n : -1;
                    const char *tb = reinterpret_cast<const char *>(a.wtiles + int64_t(tile) * 256);
                    Ww[0] = *reinterpret_cast<const v2d *>(tb + lane16);     // unconditional (the all-zero tile when there
                    Ww[1] = *reinterpret_cast<const v2d *>(tb + lane16 + 1024);  // is none): skipping the fetch measured slower
                    if (q2 + 1 == nBt) { q2 = 0; ++t2; } else ++q2;
                };
                auto consume = [&](int b, const double (&Vv)[kBatch], const double (&Uu)[kBatch], const v2d (&Ww)[2], int S) {
                    if (b < TB) {
                        if (S >= 0) {                                     // park the W tile that came with this batch
                            double *wp = Pool + S * 256 + lane * 2;
                            *reinterpret_cast<v2d *>(wp) = Ww[0];
                            *reinterpret_cast<v2d *>(wp + 128) = Ww[1];
                        }
                        accT0 = __builtin_amdgcn_mfma_f64_16x16x4f64(Vv[0], Uu[0], accT0, 0, 0, 0);
                        accT1 = __builtin_amdgcn_mfma_f64_16x16x4f64(Vv[1], Uu[1], accT1, 0, 0, 0);
                        accT0 = __builtin_amdgcn_mfma_f64_16x16x4f64(Vv[2], Uu[2], accT0, 0, 0, 0);
                        accT1 = __builtin_amdgcn_mfma_f64_16x16x4f64(Vv[3], Uu[3], accT1, 0, 0, 0);
                        if (q0 + 1 == nBt) {
                            // end of the round: T^t of this wavefront's l tile goes to LDS ...
                            const v4d T = accT0 + accT1;
                            double *tp = Tx + wave * 256 + lane * 2;
                            *reinterpret_cast<v2d *>(tp) = v2d{T.x, T.y};
                            *reinterpret_cast<v2d *>(tp + 128) = v2d{T.z, T.w};
                            __syncthreads();
                            // ... and every wavefront multiplies the W tiles of its m tiles with the eight T^t,
                            // even and odd l tiles into two accumulators (two independent instruction chains)
                            uint32_t fm[8], any = 0u;
                            int pre[8], seen = 0;
#pragma unroll
                            for (int t = 0; t < 8; ++t) {
                                fm[t] = __builtin_amdgcn_readlane(mreg, 8 * t0 + t);
                                pre[t] = seen;
                                seen += __popc(fm[t]);
                                any |= fm[t];
                            }
                            // Parked tiles first, in a loop without global loads (a load that may or may not
                            // have been issued makes the compiler wait for every load in flight, the
                            // pipeline's included); the tiles that were not parked follow in a loop of their own.
                            const int parked = min(kPool, kOwnWaves * nBt);      // tiles n < parked lie in the pool
                            auto multiply = [&](auto from_pool) {
#pragma unroll
                                for (int x = 0; x < kOwnZ; ++x) {
                                    const int mt = wave + kOwnWaves * x;
                                    if ((any >> mt) & 1u) {
                                        v4d z0 = accZ[x], z1 = v4d{0.0, 0.0, 0.0, 0.0};
#pragma unroll
                                        for (int t = 0; t < 8; ++t) {
                                            const int r = __popc(fm[t] & ((1u << mt) - 1u));
                                            const int n = pre[t] + r;                 // place in the round's tile sequence
                                            if (((fm[t] >> mt) & 1u) && (n < parked) == decltype(from_pool)::value) {
                                                const lds_v2d *tr = TxV + (t * 128 + lane);
                                                const v2d Ta = tr[0], Tb = tr[64];
                                                v2d w0, w1;
                                                if (decltype(from_pool)::value) {
                                                    const lds_v2d *rp = PoolV + (n * 128 + lane);
                                                    w0 = rp[0];
                                                    w1 = rp[64];
                                                } else {
                                                    const uint32_t tile = __builtin_amdgcn_readlane(freg, 8 * t0 + t) + uint32_t(r);
                                                    const char *tb = reinterpret_cast<const char *>(a.wtiles + int64_t(tile) * 256);
                                                    w0 = *reinterpret_cast<const v2d *>(tb + lane16);
                                                    w1 = *reinterpret_cast<const v2d *>(tb + lane16 + 1024);
                                                }
                                                v4d z = (t & 1) ? z1 : z0;
                                                z = __builtin_amdgcn_mfma_f64_16x16x4f64(w0.x, Ta.x, z, 0, 0, 0);
                                                z = __builtin_amdgcn_mfma_f64_16x16x4f64(w0.y, Ta.y, z, 0, 0, 0);
                                                z = __builtin_amdgcn_mfma_f64_16x16x4f64(w1.x, Tb.x, z, 0, 0, 0);
                                                z = __builtin_amdgcn_mfma_f64_16x16x4f64(w1.y, Tb.y, z, 0, 0, 0);
                                                if (t & 1) z1 = z; else z0 = z;
                                            }
                                        }
                                        accZ[x] = z0 + z1;
                                    }
                                }
                            };
                            if (any & own) {
                                multiply(std::true_type{});
                                if (seen > parked) multiply(std::false_type{});
                            }
                            __syncthreads();                              // T^t and the pool are free for the next round
                            accT0 = v4d{0.0, 0.0, 0.0, 0.0};
                            accT1 = accT0;
                            q0 = 0;
                            ++t0;
                        } else {
                            ++q0;
                        }
                    }
                };

                if (TB > 0) {
#pragma unroll
                    for (int u = 0; u < kRingO; ++u) read_j(P.Jr[u]);
#pragma unroll
                    for (int u = 0; u < kRingO - 1; ++u) issue(P.Jr[u], P.Vr[u], P.Ur[u], P.Wr[u], P.Sr[u]);
                    for (int b = 0; b < TB; b += kRingO) {
#pragma unroll
                        for (int u = 0; u < kRingO; ++u) {
                            const int su = (u + kRingO - 1) % kRingO;
                            issue(P.Jr[su], P.Vr[su], P.Ur[su], P.Wr[su], P.Sr[su]);
                            read_j(P.Jr[u]);
                            consume(b + u, P.Vr[u], P.Ur[u], P.Wr[u], P.Sr[u]);
                        }
                    }
                }
            }
            p0 += kCap;
            if (p0 < n_union) {
                np = min(kCap, n_union - p0);
                npad = (np + 4 * kBatch - 1) & ~(4 * kBatch - 1);
                prepare(p0, np, npad, std::false_type{});
            }
        }
    }

    // ---- store the group's rows: lane holds Z^t[m = 16 mt + slot + 4 v][i = c] ----------------------
    const int64_t M = a.M;
    const int64_t s = s0 + c;
    if (s < a.slices) {
        const int64_t row = a.compact ? s : int64_t(a.uidx0[s]);
        double *dst = a.n_kc == 1 ? a.out + row * M : a.partial + (int64_t(kc) * a.slices + s) * M;
#pragma unroll
        for (int x = 0; x < kOwnZ; ++x) {
            const int mt = wave + kOwnWaves * x;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int m = 16 * mt + slot + 4 * v;
                if (mt < a.MT && m < M) dst[m] = accZ[x][v];
            }
        }
    }
}

// sums the partial results of the k chunks in chunk order
__global__ void sptn3_fixup_kernel(int64_t slices, int64_t M, int n_kc, const int32_t *__restrict__ uidx0,
                                   const double *__restrict__ partial, double *out, int compact) {
    const int64_t x = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (x >= slices * M) return;
    const int64_t s = x / M, m = x - s * M;
    double z = 0.0;
    for (int kc = 0; kc < n_kc; ++kc) z += partial[(int64_t(kc) * slices + s) * M + m];
    const int64_t row = compact ? s : int64_t(uidx0[s]);
    out[row * M + m] = z;
}

static size_t sptn3_owned_lds(int nwords) {
    return size_t(kCap * 16 + kPool * 256 + kOwnWaves * 256) * 8 + size_t(kCap) * 4 + size_t(nwords) * 8 + 64;
}

bool sptn3_two_waves_fit(int nwords) { return sptn3_owned_lds(nwords) <= 160 * 1024; }

static conststn_status launch_sptn3_tiled(const conststn_plan_s *plan, const double *const *dense, double *out,
                                          hipStream_t stream) {
    const conststn_csf_s *U = plan->X, *W = plan->W;
    Sptn3TileArgs a{};
    a.slices = U->nodes[0];
    a.L = W->dims[W->mode_order[1]];
    a.M = W->dims[W->mode_order[2]];
    a.LT = (a.L + 15) / 16;
    a.MT = int((a.M + 15) / 16);
    const int64_t J = U->dims[U->mode_order[2]];
    a.nwords = int((J + 31) / 32);
    a.n_groups = int((a.slices + kSpGroup - 1) / kSpGroup);
    a.n_kc = plan->sp_kc;
    a.k_per = plan->sp_k_per;
    a.uptr0 = U->ptr[0].p;
    a.uptr1 = U->ptr[1].p;
    a.uidx0 = U->idx[0].p;
    a.uidx1 = U->idx[1].p;
    a.uidx2 = U->idx[2].p;
    a.uvals = U->vals.p;
    a.w_root_of_k = plan->w_root_of_k.p;
    a.wmask = plan->w_tile_mask.p;
    a.wfirst = plan->w_tile_first.p;
    a.wtiles = plan->w_tiles.p;
    a.zero_tile = uint32_t(plan->n_w_tiles);
    a.V = dense[0];
    a.out = out;
    a.partial = plan->partial.p;
    a.compact = plan->compact ? 1 : 0;
    a.wg_order = plan->sp_xcd_ranges ? nullptr : plan->sp_wg_order.p;
    a.xcd_ranges = plan->sp_xcd_ranges ? 1 : 0;      // measured: halves the HBM fetch, 4 % slower
    const size_t lds_bytes = size_t(kCap) * 16 * 8 + size_t(4 * kStage) * 256 * 8 + size_t(a.MT) * 256 * 8 +
                             size_t(kCap) * 4 + size_t(a.nwords) * 8 + 64;
    if (!plan->compact && a.slices < plan->out_rows)
        CST_TRY(zero_fill(out, plan->out_rows * plan->row_elems, stream));
    if (a.slices == 0) return CONSTSTN_OK;
    // two wavefronts per SIMD (m tiles owned by wavefronts) when the plan chose it, else one (l tiles owned)
    const size_t lds_owned = sptn3_owned_lds(a.nwords);
    const bool owned = plan->sp_two_waves;
    {
        ProfScope prof(plan, stream);
        const unsigned n_wg = unsigned(a.n_groups) * unsigned(a.n_kc);
        if (owned) sptn3_owned_kernel<<<dim3((n_wg + 7) / 8 * 8), dim3(64 * kOwnWaves), lds_owned, stream>>>(a);
        else sptn3_tiled_kernel<<<dim3((n_wg + 7) / 8 * 8), dim3(256), lds_bytes, stream>>>(a);
    }
    CST_HIP(hipGetLastError());
    if (a.n_kc > 1) {
        const int64_t n = a.slices * a.M;
        sptn3_fixup_kernel<<<dim3(unsigned((n + 255) / 256)), dim3(256), 0, stream>>>(
            a.slices, a.M, a.n_kc, a.uidx0, a.partial, out, a.compact);
        CST_HIP(hipGetLastError());
    }
    return CONSTSTN_OK;
}

// Both tiled kernels take up to the whole 160 KB of a CU's LDS: the limit is raised when the plan is built.
conststn_status prepare_sptn3_launch(conststn_plan_s *plan) {
    plan->sp_xcd_ranges = plan->opt("sptn3_xcd", 0) == 1;
    CST_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(sptn3_tiled_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
    CST_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(sptn3_owned_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
    return CONSTSTN_OK;
}

conststn_status launch_sptn3(const conststn_plan_s *plan, const double *const *dense, double *out,
                             hipStream_t stream) {
    if (plan->w_tiled) return launch_sptn3_tiled(plan, dense, out, stream);
    const conststn_csf_s *U = plan->X, *W = plan->W;
    Sptn3Args a{};
    a.slices = U->nodes[0];
    a.L = W->dims[W->mode_order[1]];
    a.M = W->dims[W->mode_order[2]];
    a.uptr0 = U->ptr[0].p;
    a.uptr1 = U->ptr[1].p;
    a.uidx0 = U->idx[0].p;
    a.uidx1 = U->idx[1].p;
    a.uidx2 = U->idx[2].p;
    a.uvals = U->vals.p;
    a.wptr0 = W->ptr[0].p;
    a.wptr1 = W->ptr[1].p;
    a.widx1 = W->idx[1].p;
    a.widx2 = W->idx[2].p;
    a.wvals = W->vals.p;
    a.w_root_of_k = plan->w_root_of_k.p;
    a.V = dense[0];
    a.out = out;
    a.compact = plan->compact ? 1 : 0;
    const size_t lds_bytes = size_t(a.L + 4 * a.M) * sizeof(double);
    if (lds_bytes > 64 * 1024) {
        set_error("three-tensor kernel needs %zu bytes of LDS (L=%lld, M=%lld); at most 65536 implemented",
                  lds_bytes, (long long)a.L, (long long)a.M);
        return CONSTSTN_EUNSUPPORTED;
    }
    if (!plan->compact && a.slices < plan->out_rows)
        CST_TRY(zero_fill(out, plan->out_rows * plan->row_elems, stream));
    if (a.slices == 0) return CONSTSTN_OK;
    {
        ProfScope prof(plan, stream);
        sptn3_kernel<<<dim3(unsigned(a.slices)), dim3(256), lds_bytes, stream>>>(a);
    }
    CST_HIP(hipGetLastError());
    return CONSTSTN_OK;
}

}  // namespace cst
