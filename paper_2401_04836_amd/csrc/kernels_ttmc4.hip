// Fused order-4 TTMc over a CSF tensor (order-4 form of Sec. 5.3):
//     Y[i,r1,r2,r3] = sum_{j,k,l} X[i,j,k,l] U1[j,r1] U2[k,r2] U3[l,r3]
// as the three-statement tree
//     T1[i,j,k,r3] = X U3 ;  T2[i,j,r2,r3] = T1 U2 ;  Y[i,r1,r2,r3] = T2 U1
// fused on (i,j,k) and (i,j): T1 shrinks to a length-R3 vector per (i,j,k) node and T2 to an
// R2 x R3 matrix per (i,j) fiber -- the largest intermediate is order 2 (the l = 2 solution
// of Sec. 3).
//
// General kernel, ranks up to 16: one wavefront per work item (a range of (i,j) fibers of one
// slice).  Lane = (q, r3) with q = lane/16: the four lane rows split the leaves of a node for
// T1 (then an xor-shuffle sum), and row q holds T2[r2, r3] for r2 = q, q+4, q+8, q+12 and the
// matching 16 x 4 part of Y_i in registers.
#include <type_traits>

#include "plan.hpp"

namespace cst {

struct Ttmc4Args {
    int64_t n_items;
    int R1, R2, R3;
    const int64_t *ptr1, *ptr2;
    const int32_t *idx0, *idx1, *idx2, *idx3;
    const double *vals;
    const SliceItem *items;
    const double *U1, *U2, *U3;
    double *out, *partial;
    int compact;
};

__device__ __forceinline__ int64_t uni64(int64_t v) {
    const int lo = __builtin_amdgcn_readfirstlane(int(v & 0xffffffffll));
    const int hi = __builtin_amdgcn_readfirstlane(int(v >> 32));
    return (int64_t(hi) << 32) | int64_t(uint32_t(lo));
}

__global__ void __launch_bounds__(256)
ttmc4_kernel(Ttmc4Args a) {
    const int lane = threadIdx.x % 64;
    const int64_t w = uni64(int64_t(blockIdx.x) * 4 + threadIdx.x / 64);
    if (w >= a.n_items) return;
    const SliceItem it = a.items[w];
    const int32_t s = __builtin_amdgcn_readfirstlane(it.slice);
    const int64_t fa = uni64(it.begin), fb = uni64(it.end), dest = uni64(it.dest);
    const int R1 = a.R1, R2 = a.R2, R3 = a.R3;
    const int q = lane / 16, c3 = lane % 16;
    const bool col_ok = c3 < R3;
    const int col = col_ok ? c3 : 0;

    double y[16][4];
#pragma unroll
    for (int r = 0; r < 16; ++r)
#pragma unroll
        for (int t = 0; t < 4; ++t) y[r][t] = 0.0;

    for (int64_t f = fa; f < fb; ++f) {
        const int32_t j = __builtin_amdgcn_readfirstlane(a.idx1[f]);
        const int64_t ga = uni64(a.ptr1[f]), gb = uni64(a.ptr1[f + 1]);
        double t2[4] = {0.0, 0.0, 0.0, 0.0};
        for (int64_t g = ga; g < gb; ++g) {
            const int32_t k = __builtin_amdgcn_readfirstlane(a.idx2[g]);
            const int64_t la = uni64(a.ptr2[g]), lb = uni64(a.ptr2[g + 1]);
            double t1 = 0.0;
            for (int64_t n = la; n < lb; n += 4) {
                const int64_t m = n + q;
                if (m < lb) {
                    const int32_t l = a.idx3[m];
                    t1 = fma(a.vals[m], a.U3[int64_t(l) * R3 + col], t1);
                }
            }
            t1 += __shfl_xor(t1, 16, 64);
            t1 += __shfl_xor(t1, 32, 64);
            const double *u2 = a.U2 + int64_t(k) * R2;
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int r2 = q + 4 * t;
                if (r2 < R2) t2[t] = fma(u2[r2], t1, t2[t]);
            }
        }
        const double *u1 = a.U1 + int64_t(j) * R1;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            if (r < R1) {
                const double u = u1[r];
#pragma unroll
                for (int t = 0; t < 4; ++t) y[r][t] = fma(u, t2[t], y[r][t]);
            }
        }
    }
    const int64_t RR = int64_t(R1) * R2 * R3;
    double *base = dest < 0 ? a.out + (a.compact ? int64_t(s) : int64_t(a.idx0[s])) * RR
                            : a.partial + dest * RR;
    if (col_ok) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            if (r < R1) {
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const int r2 = q + 4 * t;
                    if (r2 < R2) base[(int64_t(r) * R2 + r2) * R3 + c3] = y[r][t];
                }
            }
        }
    }
}

// ---- MFMA kernel (all three ranks equal to 16) ----------------------------------------------
//
// Both dense stages run on the fp64 matrix cores (v_mfma_f64_16x16x4, K = 4):
//   mid level   T2_f (16x16) = sum over the fiber's pieces  U2[k,:]^T . T1      K = four pieces
//   slice level Y_i (16x256) += U1[J,:]^T . T2                                  K = four fibers
// A piece is at most two leaves of one (i,j,k) node.  The plan stores the pieces of a fiber four
// at a time in "groups" (the last group of a fiber padded with empty records) and the fibers of
// a slice four at a time in "K-steps"; a long node or fiber simply gives several pieces or
// groups, which is legal by distributivity, so the kernel walks ONE flat stream of groups whatever
// the skew of the tensor.  Per group: lane (s,c) takes record s -- level-2 index, two leaf indices,
// two leaf values, 32 bytes -- builds T1_s[r3 = c] and supplies U2[k_s, r2 = c]; one
// matrix instruction adds the group to the fiber's T2 (accumulator layout: register v of lane
// (s,c) = T2[r2 = s+4v][r3 = c]).  When a group ends its fiber the tile goes to the wave-private
// LDS buffer; when it ends its K-step, slot s reads back the tile of fiber s as the B operand
// of the 16 slice-level instructions, A = U1[j_s, c].  The structure (ends a fiber / ends a
// K-step / starts a K-step, and the four j of a K-step) travels in the records, so nothing
// but the stream itself is read.  A fiber costs ceil(pieces/4) mid-level instructions and
// exactly four slice-level ones, however many pieces it has.
// Records are fetched three groups ahead and the factor rows one group ahead (register rings,
// loop unrolled four times), so a group waits for no load issued in its own iteration.
typedef double v4d __attribute__((ext_vector_type(4)));
constexpr int kT2Stride = 16 * 16 + 16;        // doubles per tile in LDS (+16: bank skew)

struct Ttmc4RowArgs {
    int64_t n_items;
    const int64_t *kstep_group;
    const PieceDesc *rec;
    const int32_t *idx0;
    const SliceItem *items;                 // ranges of K-steps inside one slice
    const double *U1, *U2, *U3;
    double *out, *partial;
    int compact;
};

// One wavefront per workgroup: items differ in length, and a wavefront slot shared with three
// others stays idle until the longest of them is done.
__global__ void __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(2, 8)))
ttmc4_mfma_kernel(Ttmc4RowArgs a) {
    __shared__ double t2buf[4 * kT2Stride];
    const int lane = threadIdx.x;
    const int slot = lane >> 4, c = lane & 15;
    double *lds = t2buf;
    // tiles of absent fibers (a slice's last K-step may hold fewer than four) are multiplied by a
    // zero A operand: whatever they hold must be finite
    for (int e = lane; e < 4 * kT2Stride; e += 64) lds[e] = 0.0;
    const int64_t w = int64_t(blockIdx.x);
    const SliceItem it = a.items[w];
    const int32_t s = __builtin_amdgcn_readfirstlane(it.slice);
    const int64_t dest = uni64(it.dest);
    const int64_t ga = uni64(a.kstep_group[it.begin]), gb = uni64(a.kstep_group[it.end]);

    v4d acc[16];
#pragma unroll
    for (int t = 0; t < 16; ++t) acc[t] = v4d{0.0, 0.0, 0.0, 0.0};
    v4d t2 = v4d{0.0, 0.0, 0.0, 0.0};
    double av = 0.0;                         // U1[j_s, c] of the current K-step
    int ft = 0;                              // fibers of the current K-step already parked in LDS

    // A group's four records are 128 bytes.  Lane (s, c) fetches dword c mod 8 of record s -- one
    // 4-byte load per lane for the whole group instead of two 16-byte ones -- and the eight
    // dwords of a record are handed round inside the 16-lane row when they are needed.
    constexpr int kRec = 4;                  // record ring (fetched kRec - 1 groups ahead)
    uint32_t raw[kRec];
    double gu2[2], gx0[2], gx1[2];           // factor-row ring (fetched one group ahead)
    const uint32_t *words = reinterpret_cast<const uint32_t *>(a.rec);
    auto load_rec = [&](int64_t g) -> uint32_t {
        return words[((g < gb ? g : gb - 1) * 4 + slot) * 8 + (c & 7)];
    };
    auto field = [&](uint32_t x, auto which) -> int32_t {
        return __builtin_amdgcn_mov_dpp(int(x), 0x150 + decltype(which)::value, 0xf, 0xf, false);
    };
    auto field64 = [&](uint32_t x, auto lo, auto hi) -> double {
        return __hiloint2double(field(x, hi), field(x, lo));
    };
    using W0 = std::integral_constant<int, 0>;
    using W1 = std::integral_constant<int, 1>;
    using W2 = std::integral_constant<int, 2>;
    using W3 = std::integral_constant<int, 3>;
    using W4 = std::integral_constant<int, 4>;
    using W5 = std::integral_constant<int, 5>;
    using W6 = std::integral_constant<int, 6>;
    using W7 = std::integral_constant<int, 7>;
    const char *U1b = reinterpret_cast<const char *>(a.U1), *U2b = reinterpret_cast<const char *>(a.U2),
               *U3b = reinterpret_cast<const char *>(a.U3);
    auto load_rows = [&](uint32_t x, double &u2, double &x0, double &x1) {
        const int32_t kf = field(x, W0{}), l0 = field(x, W1{}), l1 = field(x, W2{});
        const int32_t k = int32_t(uint32_t(kf) & kGrpIndexMask);
        // 32-bit byte offsets against the scalar bases of the factors (their extents stay below 2^25 on
        // this path): one vector instruction per address
        u2 = *reinterpret_cast<const double *>(U2b + (uint32_t(k * 16 + c) << 3));
        x0 = *reinterpret_cast<const double *>(U3b + (uint32_t(l0 * 16 + c) << 3));
        x1 = *reinterpret_cast<const double *>(U3b + (uint32_t(l1 * 16 + c) << 3));
    };
    auto consume = [&](uint32_t x, double u2, double x0, double x1) {
        const int32_t kf = field(x, W0{});
        const uint32_t flags = uint32_t(__builtin_amdgcn_readfirstlane(kf));            // same on the four records
        if (flags & kGrpStartsKstep) {
            const int32_t j = field(x, W3{});
            av = j >= 0 ? *reinterpret_cast<const double *>(U1b + (uint32_t(j * 16 + c) << 3)) : 0.0;
        }
        // empty records and absent second leaves carry value 0
        const double t1 = fma(field64(x, W6{}, W7{}), x1, field64(x, W4{}, W5{}) * x0);
        t2 = __builtin_amdgcn_mfma_f64_16x16x4f64(u2, t1, t2, 0, 0, 0);
        if (flags & kGrpEndsFiber) {
#pragma unroll
            for (int v = 0; v < 4; ++v) lds[ft * kT2Stride + (slot + 4 * v) * 16 + c] = t2[v];
            t2 = v4d{0.0, 0.0, 0.0, 0.0};
            ++ft;
            if (flags & kGrpEndsKstep) {
                // slot s supplies fiber s; fibers the K-step lacks have av = 0
                const double a_op = slot < ft ? av : 0.0;
#pragma unroll
                for (int t = 0; t < 16; ++t) {
                    const double bv = lds[slot * kT2Stride + t * 16 + c];
                    acc[t] = __builtin_amdgcn_mfma_f64_16x16x4f64(a_op, bv, acc[t], 0, 0, 0);
                }
                ft = 0;
            }
        }
    };
#pragma unroll
    for (int u = 0; u < kRec - 1; ++u) raw[u] = load_rec(ga + u);
    load_rows(raw[0], gu2[0], gx0[0], gx1[0]);
    for (int64_t g0 = ga; g0 < gb; g0 += kRec) {
#pragma unroll
        for (int u = 0; u < kRec; ++u) {
            const int64_t g = g0 + u;
            raw[(u + kRec - 1) % kRec] = load_rec(g + kRec - 1);
            load_rows(raw[(u + 1) % kRec], gu2[(u + 1) % 2], gx0[(u + 1) % 2], gx1[(u + 1) % 2]);
            if (g < gb) consume(raw[u], gu2[u % 2], gx0[u % 2], gx1[u % 2]);
        }
    }
    const int64_t RR = 4096;
    double *base = dest < 0 ? a.out + (a.compact ? int64_t(s) : int64_t(a.idx0[s])) * RR
                            : a.partial + dest * RR;
    // acc[t][v] = Y[r1 = slot + 4v][r2 = t][r3 = c]
#pragma unroll
    for (int t = 0; t < 16; ++t)
#pragma unroll
        for (int v = 0; v < 4; ++v) base[((slot + 4 * v) * 16 + t) * 16 + c] = acc[t][v];
}

conststn_status launch_ttmc4(const conststn_plan_s *plan, const double *const *dense, double *out,
                             hipStream_t stream) {
    const conststn_csf_s *X = plan->X;
    Ttmc4Args a{};
    a.n_items = plan->n_items;
    a.R1 = plan->rank_of_level[1];
    a.R2 = plan->rank_of_level[2];
    a.R3 = plan->rank_of_level[3];
    a.ptr1 = X->ptr[1].p;
    a.ptr2 = X->ptr[2].p;
    a.idx0 = X->idx[0].p;
    a.idx1 = X->idx[1].p;
    a.idx2 = X->idx[2].p;
    a.idx3 = X->idx[3].p;
    a.vals = X->vals.p;
    a.items = plan->items.p;
    a.U1 = dense[plan->factor_of_level[1]];
    a.U2 = dense[plan->factor_of_level[2]];
    a.U3 = dense[plan->factor_of_level[3]];
    a.out = out;
    a.partial = plan->partial.p;
    a.compact = plan->compact ? 1 : 0;
    if (a.R1 > 16 || a.R2 > 16 || a.R3 > 16) {
        set_error("order-4 TTMc ranks above 16 are not implemented");
        return CONSTSTN_EUNSUPPORTED;
    }
    if (!plan->compact && X->nodes[0] < plan->out_rows)
        CST_TRY(zero_fill(out, plan->out_rows * plan->row_elems, stream));
    if (a.n_items == 0) return CONSTSTN_OK;
    {
        ProfScope prof(plan, stream);
        if (plan->use_rows) {
            Ttmc4RowArgs ra{};
            ra.n_items = plan->n_items;
            ra.kstep_group = plan->kstep_group.p;
            ra.rec = plan->pieces.p;
            ra.idx0 = a.idx0;
            ra.items = a.items;
            ra.U1 = a.U1;
            ra.U2 = a.U2;
            ra.U3 = a.U3;
            ra.out = out;
            ra.partial = a.partial;
            ra.compact = a.compact;
            ttmc4_mfma_kernel<<<dim3(unsigned(a.n_items)), dim3(64), 0, stream>>>(ra);
        } else
            ttmc4_kernel<<<dim3(unsigned(div_up(a.n_items, 4))), dim3(256), 0, stream>>>(a);
    }
    CST_HIP(hipGetLastError());
    return launch_ttmc_fixup(plan, out, stream);
}

}  // namespace cst
