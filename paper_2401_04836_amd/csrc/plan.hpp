// The plan handle: a validated schedule matched to one kernel family, plus the device-side
// work tables (load-balanced partition of the CSF tree) and scratch the kernels need.
#pragma once

#include <map>
#include <memory>

#include "common.hpp"
#include "schedule.hpp"

namespace cst {

constexpr int kHeavySpan = 64;        // a slice spanning at least this many chunks is "heavy"
constexpr int kHeavySegments = 32;    // its chunk range is reduced in this many parallel segments
constexpr int kRowLeaves = 16;        // longest run of leaves one MFMA K-row sums
constexpr int kPieceLeaves = 2;       // order-4 path: leaves per piece of a level-2 node
// three-tensor network, tiled path
constexpr int kSpGroup = 16;          // root slices of U processed together (one MFMA operand side)
constexpr int kSpMaxMTiles = 25;      // m tiles whose accumulators a wavefront holds (M <= 400)
constexpr int kSpMaxJ = 32768;        // extent of the contracted mode j the LDS bit mask covers

enum Family { FAM_NONE = 0, FAM_TTMC3, FAM_TTMC4, FAM_MTTKRP3, FAM_SPTN3, FAM_GENERIC, FAM_SPCHAIN3, FAM_SPPAIR4 };

// One statement of the generic executor (generic.hip), passed to its kernel by value.
// Dense loop indices: the first n_out are the result's dense indices in storage order, the
// next n_red are summed over; strides are in elements, 0 where a tensor lacks the index.
constexpr int kGenMaxIdx = 8;
constexpr int kGenMaxUpper = 2;
constexpr int64_t kGenSegment = 256;          // children per segment of a long sum
constexpr int64_t kGenLeafSegment = 512;      // leaves per segment when the producers are inlined
constexpr int64_t kGenHeavy = 64;             // a result node with more segments than this is added up by workgroups
struct GenStmt {
    int kind;                                  // 0: one thread per result element walks the subtree below its node;
                                               // 1: one thread per (node of depth d_node, dense result element)
    int d_in, d_out;                           // CSF prefix depth of the sparse-side input / of the result (kind 1: 0 = stored dense)
    int d_f, d_node;                           // kind 1: prefix depth of the other input; depth of the nodes the threads stand on
    int atomic;                                // kind 1: several threads add to one result element
    int in_is_leaf;                            // the sparse-side input is the CSF operand itself
    int n_out, n_red;
    int scatter_rows;                          // result row = root index instead of root node number
    int64_t extent[kGenMaxIdx];
    int64_t in_stride[kGenMaxIdx], f_stride[kGenMaxIdx], out_stride[kGenMaxIdx];
    // stride of each CSF level's index in a tensor stored dense (0 where it lacks the index); kind 0 uses
    // f_level_stride only, for the summed levels
    int64_t in_level_stride[CONSTSTN_MAX_ORDER], f_level_stride[CONSTSTN_MAX_ORDER], out_level_stride[CONSTSTN_MAX_ORDER];
    int64_t in_block, f_block, out_block;      // elements per CSF node of a tensor stored by prefix
    int64_t out_threads;                       // kind 1: dense result elements per node
    int64_t out_elems;                         // elements of the result's storage
    int64_t out_nodes, roots;
    int64_t nodes[CONSTSTN_MAX_ORDER];
    const int32_t *idx[CONSTSTN_MAX_ORDER];
    const int64_t *ptr[CONSTSTN_MAX_ORDER];
    const double *in, *f;
    double *out;
    int in_operand, in_buffer, f_operand, f_buffer, out_buffer;   // resolved to pointers at launch
    // kind 0, long sums: the children of a result node cut into segments, one thread per (segment,
    // element) writes a partial sum, a second pass adds the partial sums of each node in order
    int64_t n_segs;
    const int64_t *seg;                        // [3 * n_segs] result node, first child, end child (fused: first leaf, end leaf)
    const int64_t *seg_ptr;                    // [out_nodes + 1] segments of each result node
    int64_t n_heavy;                           // result nodes with so many segments that a workgroup adds them
    const int64_t *heavy;                      // [n_heavy] their numbers
    double *heavy_sums;                        // [n_heavy x parts x out_block] sums of the workgroups that share a node
    int heavy_buffer;                          // resolved to heavy_sums at launch
    double *partial;                           // [n_segs * out_block]
    int seg_table, partial_buffer;             // resolved to pointers at launch
    // kind 1 with atomics: workgroups add into `copies` private copies of the result in turn, so that a
    // result element every node meets in (a power-law index) is not one queue; a second pass adds the copies
    int copies, copies_buffer;
    // fused pair (Fig. 3b): this statement consumes a result that the statement before it forms from X's
    // leaves and a dense factor F1, one level deeper; the consumer's thread sums the leaves below each of
    // its children itself, so that the intermediate is a scalar in a register and is never stored
    int fused;                                 // 1: producer inlined (its own entry has skip = 1)
    int fused_small;                           // 1: both factors within reach of 32-bit byte offsets formed by 24-bit multiplies
    int fused_pairs;                           // 1: the layouts allow two adjacent result elements per lane (16-byte row reads)
    int skip;                                  // 1: computed inside its consumer's kernel
    int f1_operand;                            // the producer's dense factor, resolved at launch
    const double *f1;
    int64_t f1_stride[kGenMaxIdx];             // its strides for this statement's dense result indices
    int64_t f1_level_stride;                   // and for the index of the leaf level
    // fused chain: the producer may itself have inlined its producer, and so on, kGenMaxUpper times.  Then
    // `fused_upper` levels lie between this statement's summed level and X's fibers; the factor of the
    // fiber level is fu[0], of the level above it fu[1], and `f` is the factor of the summed level.
    int fused_upper;
    int fu_operand[kGenMaxUpper];
    const double *fu[kGenMaxUpper];
    int64_t fu_stride[kGenMaxUpper][kGenMaxIdx];
    int64_t fu_level_stride[kGenMaxUpper];
    const int64_t *leaf_end[kGenMaxUpper];     // [nodes + 1] first leaf below each node of the level above the fibers, the next one up
    const int64_t *out_leaf;                   // [out_nodes + 1] the same for the result's nodes; null: one node over every leaf
};

// One unit of work of the TTMc kernels: a range of leaf positions (order 3) or of level-1
// fibers (order 4) inside ONE root slice.  dest < 0: the slice has a single item and its row
// block is stored straight to the output; otherwise dest is the slot of a partial row block.
struct SliceItem {
    int32_t slice;
    int32_t pad;
    int64_t begin, end;     // order 3: leaf range; order 4: level-1 fiber range
    int64_t first;          // order 3: level-1 fiber containing `begin`; order 4: unused
    int64_t dest;
};

// One row of the order-3 TTMc MFMA path: at most kRowLeaves consecutive leaves of one fiber.
struct alignas(16) RowDesc {
    int64_t leaf;           // first leaf
    int32_t cnt;            // number of leaves
    int32_t j;              // level-1 index of the fiber
};

// One K-step (four rows, the K of one matrix instruction) of the streaming order-3 TTMc path.
struct alignas(16) KStepDesc {
    int32_t row0;           // first row
    int32_t meta;           // bits 0-2: rows in the step (1..4); bit 3: last step of its item
    int64_t dest;           // last step only: >= 0 row block of the output, < 0: ~(partial row block)
};

// One piece of the order-4 TTMc MFMA path: at most kPieceLeaves (= 2) consecutive leaves of one
// (i,j,k) node, copied out of the CSF so that one 32-byte read brings everything the leaf stage
// needs and no second, dependent load of the leaves follows.
struct alignas(32) PieceDesc {
    int32_t k;              // level-2 index of the node | kGrp* flags
    int32_t l0, l1;         // leaf indices; l1 = l0 (with v1 = 0) when the piece has one leaf; an empty record
                            // that pads a group repeats the fiber's first node and leaf with both values 0
    int32_t pad;            // first group of a K-step, slot s: level-1 index of the K-step's fiber s (-1: none)
    double v0, v1;          // leaf values (v1 = 0 when absent)
};
static_assert(kPieceLeaves == 2, "PieceDesc holds two leaves");
// structure flags carried in PieceDesc::k (the same on the four records of a group)
constexpr uint32_t kGrpEndsFiber = 1u << 28, kGrpEndsKstep = 1u << 29, kGrpStartsKstep = 1u << 30,
                   kGrpIndexMask = (1u << 28) - 1u;

// One of the two sub-tensors of the split rank-32 MTTKRP path: the leaves whose factor row is
// "hot" (kept in LDS) or the rest.  X = X_hot + X_cold and the contraction is linear in X, so each
// part is a CSF tensor of its own (only the slices and fibers that keep a leaf) with its own
// chunk tables; the second part accumulates onto the output of the first.
struct MttkrpPart {
    int64_t slices = 0, fibers = 0, nnz = 0;
    DevBuf<int32_t> row_of_slice, idx1;
    DevBuf<int64_t> ptr0, ptr1;
    DevBuf<uint32_t> code;                 // leaf index or LDS slot, with end-of-fiber / end-of-slice marks
    DevBuf<double> vals;
    DevBuf<int64_t> slice_leaf, chunk_fiber;
    DevBuf<int32_t> chunk_slice;
    int64_t chunk_q = 0, n_chunks = 0;
    DevBuf<double> partial;
    DevBuf<int32_t> heavy_slices;
    DevBuf<double> heavy_partial;
    int n_heavy = 0;
};

}  // namespace cst

struct conststn_plan_s {
    cst::Schedule sched;
    cst::Family family = cst::FAM_NONE;
    unsigned flags = 0;
    std::string description;
    // tuning options given to conststn_plan_options ("name=value,..."): read while the plan is built,
    // never by an execute
    std::map<std::string, int64_t> options;
    int64_t opt(const char *name, int64_t dflt) const {
        const auto it = options.find(name);
        return it == options.end() ? dflt : it->second;
    }
    int n_cus = 256;                      // compute units of the device the plan was made on

    const conststn_csf_s *X = nullptr;    // the sparse operand walked by the fused loops
    // MTTKRP / TTMc of order 3 whose output index is not the root level of the caller's CSF: the plan keeps a
    // private copy of the tensor sorted with the output mode at the root (X points to it) and runs the
    // kernels written for that case
    std::unique_ptr<conststn_csf_s> rerooted_x;
    int rerooted_level = -1;              // level of the caller's CSF that indexes the output, or -1
    const conststn_csf_s *W = nullptr;    // second sparse operand (three-tensor network only)
    int n_dense = 0;
    int factor_of_level[CONSTSTN_MAX_ORDER] = {0};   // dense ordinal of the factor contracted at CSF level l
    int rank_of_level[CONSTSTN_MAX_ORDER] = {0};     // its rank extent
    int64_t out_rows = 0, row_elems = 0;
    bool compact = false;

    // --- device tables ---
    cst::DevBuf<int64_t> slice_leaf;       // [slices+1] leaf position where each root slice starts
    // MTTKRP: equal leaf-count chunks
    int64_t chunk_q = 0, n_chunks = 0;
    cst::DevBuf<int64_t> chunk_fiber;      // level-1 fiber containing the chunk's first leaf
    cst::DevBuf<int32_t> chunk_slice;      // root slice containing that fiber
    // MTTKRP rank-32 path: private re-encoding of the leaf index stream.  Each entry holds the
    // leaf index, or -- for the most frequently referenced ("hot") factor rows, which the kernel
    // keeps in LDS -- the LDS slot, plus end-of-fiber / end-of-slice marks.
    cst::DevBuf<uint32_t> leaf_code;
    cst::DevBuf<int32_t> hot_rows;         // [n_hot] leaf index held by each LDS slot
    int n_hot = 0;
    bool split = false;                    // hot and cold leaves run as two sub-tensors
    std::vector<std::unique_ptr<cst::DevBuf<double>>> gen_densified;   // generic executor: dense copies of further CSF operands
    int mttkrp_dual = 0;                   // 0: two launches; NH * 10 + NC: one launch, NH hot and NC cold wavefronts per workgroup
    cst::DevBuf<double> mttkrp_out2;       // the cold team's output in that form, added to the result afterwards
    cst::MttkrpPart part[2];
    // slices shared by very many chunks get a two-stage fix-up
    cst::DevBuf<int32_t> heavy_slices;
    cst::DevBuf<double> heavy_partial;     // [n_heavy x kHeavySegments x R]
    int n_heavy = 0;
    // TTMc: items inside slices
    int64_t n_items = 0, n_partials = 0, n_split = 0;
    cst::DevBuf<cst::SliceItem> items;
    cst::DevBuf<int32_t> split_slices;     // slices made of more than one item
    cst::DevBuf<int64_t> split_first;      // [n_split] first partial slot of that slice
    cst::DevBuf<int32_t> split_count;      // [n_split] number of partial slots
    // TTMc order-3 MFMA path: fibers cut into "rows" of at most kRowLeaves leaves (a long fiber
    // becomes several rows with the same level-1 index); items are ranges of rows
    bool use_rows = false;
    int64_t n_rows_tab = 0;
    cst::DevBuf<cst::RowDesc> rows;        // [rows] order-3 path; rows of a slice ordered from long to short
    cst::DevBuf<int32_t> row_j;            // [rows] order-4 path: level-1 index of the row's fiber
    cst::DevBuf<int64_t> slice_row;        // [slices+1] first row of each slice
    // streaming form of that path: the K-steps of all items as one flat table, and the first K-step of
    // the batch of whole items each workgroup walks
    int ttmc3_qn = 2;                      // column tiles per wavefront of the one-wavefront-per-item kernel
    bool use_stream = false;
    int stream_producers = 4;              // wavefronts of a workgroup that gather (the others multiply and store)
    int64_t n_ksteps = 0, n_stream_wg = 0;
    cst::DevBuf<cst::KStepDesc> ksteps;
    cst::DevBuf<int32_t> wg_kstep;         // [n_stream_wg + 1]
    // TTMc order-4 MFMA path: level-2 nodes cut into "pieces" of at most kPieceLeaves leaves,
    // level-1 fibers cut into rows of at most 4 pieces; rows index pieces, pieces index leaves
    int64_t n_pieces = 0;
    cst::DevBuf<cst::PieceDesc> pieces;    // [pieces] first leaf, level-2 index, leaf count
    cst::DevBuf<int64_t> kstep_group;      // [K-steps+1] first group (of four piece records) of each K-step
    cst::DevBuf<double> partial;           // partial row blocks
    // three-tensor network
    cst::DevBuf<int64_t> w_root_of_k;      // [K] root node of W holding index k, or -1
    bool w_tiled = false;                  // W also stored as dense 16 x 16 (l, m) tiles
    bool sp_two_waves = false;             // tiled kernel with two wavefronts per SIMD (m tiles owned by wavefronts)
    int64_t n_w_tiles = 0;
    cst::DevBuf<uint32_t> w_tile_mask;     // [roots x ceil(L/16)] m tiles present
    cst::DevBuf<uint32_t> w_tile_first;    // [roots x ceil(L/16)] index of the first of them
    cst::DevBuf<double> w_tiles;           // [(tiles + 1) x 256], the last one all zero
    bool sp_xcd_ranges = false;            // contiguous workgroup ranges per XCD
    cst::DevBuf<int32_t> sp_wg_order;      // [groups x k chunks] pairs by falling number of U leaves, or empty
    int sp_kc = 1;                         // chunks of the k range (one workgroup per group and chunk)
    int64_t sp_k_per = 0;                  // k values per chunk

    // generic executor: one entry per statement, intermediates held whole
    std::vector<cst::GenStmt> gen;
    std::vector<std::unique_ptr<cst::DevBuf<double>>> gen_buffers;
    std::vector<std::unique_ptr<cst::DevBuf<int64_t>>> gen_tables;   // segment tables of long sums
    std::vector<std::unique_ptr<cst::DevBuf<int64_t>>> gen_leaf_tables;   // first leaf below each node of a level, for fused statements
    bool gen_rooted = false;               // the result has one row block per root index
    bool gen_zero_out = false;             // the last statement adds into the result: cleared before every run

    // chain of three sparse tensors with a sparse result (X is the order-3 tensor)
    const conststn_csf_s *sc_C = nullptr, *sc_P = nullptr, *sc_L = nullptr;
    std::unique_ptr<conststn_csf_s> sc_E;  // structure of the result (no values): CSF K > i > m
    cst::DevBuf<int32_t> sc_p_node_of_m;   // [extent of m] root node of P holding m, or -1
    cst::DevBuf<int64_t> sc_nu_ptr;        // [K nodes + 1] into sc_nu_list
    cst::DevBuf<int32_t> sc_nu_list;       // distinct v under each K node, ascending
    cst::DevBuf<uint16_t> sc_i_slot;       // [leaves of X] position of the leaf's v in its K's list
    cst::DevBuf<int32_t> sc_l_knode, sc_l_cnode;        // per leaf of L: K node of X, root node of C (-1: absent)
    cst::DevBuf<int32_t> sc_e_knode, sc_e_cnode;        // per (K,i) node of the result: the same
    cst::DevBuf<double> sc_e_lval;         // per (K,i) node: value of L (1 without a filter)
    cst::DevBuf<int32_t> sc_e_root_knode;  // per root of the result: K node of X
    int sc_max_slots = 0, sc_map_bytes = 0, sc_lds_bytes = 0;
    cst::DevBuf<int64_t> sc_mu_ptr;        // [roots of the result + 1] into sc_mu_list
    cst::DevBuf<int32_t> sc_mu_list;       // distinct m under each root of the result, ascending
    bool sc_local = false;                 // every K's dense blocks fit LDS: block-local numeric kernel
    int sc_local_lds = 0;
    cst::DevBuf<double> sc_pk_blocks;                        // dense blocks P_K [v slots x m], one per run of K sharing both lists
    int64_t sc_pk_doubles = 0;
    cst::DevBuf<int32_t> sc_e_c0, sc_e_clen;                 // per (K,i) node: range of C[i,:]
    cst::DevBuf<unsigned char> sc_roots;                     // per root of the result: the kernel's descriptor
    std::vector<int> sc_local_layout;      // byte offsets of the kernel's LDS arrays

    // product of two sparse order-3 tensors with a sparse order-4 result (X = Ea, W = Eb; structure in sc_E)
    cst::DevBuf<int64_t> p4_ua_ptr, p4_ub_ptr;           // per root: its distinct innermost indices ...
    cst::DevBuf<int32_t> p4_ua_list, p4_ub_list;
    cst::DevBuf<uint16_t> p4_a_slot, p4_b_slot;          // ... and every leaf's place among them
    cst::DevBuf<int32_t> p4_node_a, p4_node_b, p4_root_a;   // per (i,j) node / per root of the result: root nodes of the operands
    int p4_words = 0, p4_max_ua = 0, p4_max_ub = 0, p4_max_common = 0, p4_mp = 0, p4_np = 0;
    std::vector<int> p4_layout;
    bool p4_stored = false;                              // shared-K lists and bit matrices kept from the symbolic pass
    cst::DevBuf<int64_t> p4_k_ptr;
    cst::DevBuf<int64_t> p4_k_a, p4_k_b;                 // first leaf of each shared K's row in the two operands
    cst::DevBuf<int32_t> p4_k_alen, p4_k_blen;           // and its length
    cst::DevBuf<uint32_t> p4_masks;
    cst::DevBuf<int32_t> p4_wg_pair;                     // workgroup -> (i,j) node of the numeric pass (-1: none)
    int64_t p4_n_wg = 0;
    int p4_nbuf = 2;                                     // chunk buffers per matrix in LDS
    bool p4_dense = false;                               // dense rows of the operands kept (rebuilt by every execute)
    cst::DevBuf<int64_t> p4_row_at_a, p4_row_at_b;       // per level-1 node: first element of its dense row
    cst::DevBuf<double> p4_dense_a, p4_dense_b;

    // measurement hook: event pairs around the dominant kernel of each execute
    mutable std::vector<hipEvent_t> prof_start, prof_stop;
    mutable int64_t prof_count = 0;        // executes recorded since the last read
    ~conststn_plan_s() {
        for (hipEvent_t e : prof_start) (void)hipEventDestroy(e);
        for (hipEvent_t e : prof_stop) (void)hipEventDestroy(e);
    }
};

namespace cst {

// partition.hip
conststn_status build_mttkrp3_tables(conststn_plan_s *plan);
conststn_status build_ttmc_tables(conststn_plan_s *plan);
conststn_status build_sptn3_tables(conststn_plan_s *plan);
// whether the LDS of the two-wavefront form of the tiled kernel fits a workgroup (nwords = 32-bit words of the j bit mask)
bool sptn3_two_waves_fit(int nwords);

// kernels_*.hip
conststn_status launch_mttkrp3(const conststn_plan_s *plan, const double *const *dense, double *out,
                               hipStream_t stream);
conststn_status launch_ttmc3(const conststn_plan_s *plan, const double *const *dense, double *out,
                             hipStream_t stream);
// the same with the partial row blocks in the library's static scratch array instead of the plan's buffer
conststn_status launch_ttmc3_static(const conststn_plan_s *plan, const double *const *dense, double *out,
                                    hipStream_t stream);
conststn_status launch_ttmc4(const conststn_plan_s *plan, const double *const *dense, double *out,
                             hipStream_t stream);
conststn_status launch_sptn3(const conststn_plan_s *plan, const double *const *dense, double *out,
                             hipStream_t stream);
// kernels_spchain3.hip: three sparse tensors, sparse result
conststn_status build_spchain3_tables(conststn_plan_s *plan);
conststn_status launch_spchain3(const conststn_plan_s *plan, double *out, hipStream_t stream);
// shared by the sparse x sparse kernels: distinct innermost indices under every root of an order-3 CSF
// tensor, and every leaf's place among them
conststn_status csf3_leaf_universe(const conststn_csf_s *T, DevBuf<int64_t> &u_ptr, DevBuf<int32_t> &u_list,
                                   DevBuf<uint16_t> &slot, int64_t *largest, std::vector<int64_t> *host_ptr);
// kernels_sppair4.hip: two sparse order-3 tensors, sparse order-4 result
conststn_status build_sppair4_tables(conststn_plan_s *plan);
conststn_status launch_sppair4(const conststn_plan_s *plan, double *out, hipStream_t stream);
// generic.hip: any tree over one CSF operand that the tuned families do not take
conststn_status build_generic(conststn_plan_s *plan);
conststn_status launch_generic(const conststn_plan_s *plan, const double *const *dense, double *out,
                               hipStream_t stream);
// sums the partial row blocks of slices made of several items (shared by the TTMc kernels)
conststn_status launch_ttmc_fixup(const conststn_plan_s *plan, double *out, hipStream_t stream, const double *partial = nullptr);

// csf_build.hip
// a copy of an order-3 CSF tensor with its levels in the order `new_levels` (levels of `src`)
conststn_status reroot_csf3(const conststn_csf_s *src, const int new_levels[3], conststn_csf_s *dst);
conststn_status build_csf_device(int order, const int64_t *dims, int64_t nnz,
                                 const int32_t *const *coords, const double *vals,
                                 const int *mode_order, unsigned flags, hipStream_t stream,
                                 conststn_csf_s *csf);

// stable radix sort of (64-bit key, 32-bit payload) pairs by the low `bits` key bits (csf_build.hip)
conststn_status radix_sort_pairs_u64(uint64_t *keys_a, uint64_t *keys_b, uint32_t *pay_a, uint32_t *pay_b, int64_t n,
                                     int bits, hipStream_t stream, const uint64_t **keys_sorted,
                                     const uint32_t **pay_sorted, void *scratch = nullptr);
size_t radix_sort_scratch_bytes(int64_t n);     // device bytes `scratch` must hold when it is handed in

// exclusive prefix sum of n int64 on the default stream; *total_host = sum of all inputs
conststn_status exscan(int64_t *in, int64_t *out, int64_t n, int64_t *total_host);

// parent of CSF node c one level up: the last p in [0, n) with ptr[p] <= c
__device__ __forceinline__ int64_t parent_of(const int64_t *ptr, int64_t n, int64_t c) {
    int64_t lo = 0, hi = n;                       // invariant: ptr[lo] <= c < ptr[hi]
    while (hi - lo > 1) {
        const int64_t mid = (lo + hi) >> 1;
        if (ptr[mid] <= c) lo = mid; else hi = mid;
    }
    return lo;
}

// fill `n` doubles with zero on `stream` (a kernel, so that it is safe inside graph capture)
conststn_status zero_fill(double *p, int64_t n, hipStream_t stream);

// Records the plan's event pair around the dominant kernel when the measurement hook is on.
struct ProfScope {
    const conststn_plan_s *plan;
    hipStream_t stream;
    int slot = -1;
    ProfScope(const conststn_plan_s *p, hipStream_t s) : plan(p), stream(s) {
        if (!plan->prof_start.empty()) {
            slot = int(plan->prof_count % int64_t(plan->prof_start.size()));
            (void)hipEventRecord(plan->prof_start[slot], stream);
        }
    }
    ~ProfScope() {
        if (slot >= 0) {
            (void)hipEventRecord(plan->prof_stop[slot], stream);
            plan->prof_count++;
        }
    }
};

// names conststn_plan_options accepts
// kernels with more dynamic LDS than the default limit: raised once per plan build
conststn_status prepare_mttkrp3_launch(conststn_plan_s *plan);
conststn_status prepare_sptn3_launch(conststn_plan_s *plan);

}  // namespace cst
