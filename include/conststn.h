/*
 * conststn -- fused execution of sparse tensor contraction trees on one AMD CDNA4 GPU.
 *
 * The library executes the fused loop nest that the CoNST paper (arXiv 2401.04836)
 * derives for a tree of binary contractions over a sparse tensor stored in CSF:
 * the schedule (execution order, one loop permutation per contraction, CSF mode
 * orders, fusion depth) is SUPPLIED by the caller as the plan -- the paper's
 * constraint search (Sec. 3) is not part of this library.
 *
 * Three verbs:   conststn_build_csf  ->  conststn_plan  ->  conststn_execute
 *
 * Conventions
 *   - "device pointer": memory of the current HIP device, owned by the caller
 *     unless stated otherwise.  "host pointer": ordinary process memory.
 *   - Every function returns a conststn_status; on failure a human-readable
 *     message is available from conststn_last_error() (thread local).  The
 *     library never aborts and never throws across this boundary.  After a
 *     failed conststn_execute the contents of `out` are unspecified.
 *   - All values are IEEE fp64.  Indices are int32, child pointers int64.
 *   - Handles are not thread safe; use one handle from one thread at a time.
 */
#ifndef CONSTSTN_H
#define CONSTSTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define CONSTSTN_MAX_ORDER 8

typedef enum {
    CONSTSTN_OK = 0,
    CONSTSTN_EINVAL = 1,        /* null pointer, bad order/rank/size, malformed schedule text      */
    CONSTSTN_ERANGE = 2,        /* a coordinate is negative or >= its mode extent                   */
    CONSTSTN_EDUP = 3,          /* duplicate coordinate: the nonzero structure is a set (Sec. 2.1)  */
    CONSTSTN_ESCHED = 4,        /* schedule violates a legality rule of Sec. 3.2                    */
    CONSTSTN_EUNSUPPORTED = 5,  /* legal, but no kernel family implements it                        */
    CONSTSTN_ENOMEM = 6,        /* device or host allocation failed                                 */
    CONSTSTN_EHIP = 7           /* a HIP runtime call failed                                        */
} conststn_status;

typedef struct conststn_csf_s conststn_csf_t;     /* a sparse tensor in CSF, resident on the device */
typedef struct conststn_plan_s conststn_plan_t;   /* a validated schedule bound to its kernels      */
typedef void *conststn_stream;                    /* a hipStream_t (NULL = the default stream)      */

/* flags of conststn_build_csf */
#define CONSTSTN_COALESCE_DUPS 1u   /* sum duplicate coordinates in input order instead of failing  */
/* flags of conststn_plan */
#define CONSTSTN_OUT_COMPACT 1u     /* output holds one row block per NONEMPTY root index only      */

/* ------------------------------------------------------------------------------------------
 * (1) COO -> CSF on the GPU.      [Sec. 2.1 "Sparse tensors", "CSF representation"]
 *
 * A CSF is the tree fixed by a permutation of the tensor's modes: level l holds, for every
 * distinct coordinate prefix of length l+1 (in mode_order), the index value in mode
 * mode_order[l]; leaves carry the values.  mode_order[l] = the mode at level l, outermost
 * first; it is the inverse of the paper's dp_{T,j} (position of mode j in the layout,
 * Sec. 3.2 "Ordering of tensor modes").
 *
 *   order      number of modes, 1..CONSTSTN_MAX_ORDER
 *   dims       host pointer, order extents (each 1 .. 2^31-1)
 *   nnz        number of nonzeros (>= 0; 0 gives an empty CSF)
 *   coords     host pointer to `order` DEVICE pointers; coords[m][n] = index of nonzero n in mode m
 *   vals       device pointer, nnz values (stored zeros are kept as structural nonzeros)
 *   mode_order host pointer, a permutation of 0..order-1
 *   flags      0 or CONSTSTN_COALESCE_DUPS
 *   stream     the work is enqueued on this stream and the call waits for it: on return the
 *              CSF is complete and range / duplicate errors have been reported
 *   out        receives the handle; the library owns every array inside it (the inputs are
 *              copied/permuted, never aliased) until conststn_csf_destroy
 *
 * Array layout of the result (what conststn_csf_export hands out), for level l:
 *   idx[l]  int32[nodes_l]      index value of each node, children of one parent strictly ascending
 *   ptr[l]  int64[nodes_l + 1]  children of node p are nodes ptr[l][p] .. ptr[l][p+1]-1 of level
 *                               l+1 (no ptr for the last level); ptr[l][0] = 0
 *   vals    fp64[nnz]           aligned with the last level (nodes_{order-1} = nnz)
 * No explicit root node: the root's children are all nodes of level 0.
 *
 * Errors: EINVAL, ERANGE, EDUP, EUNSUPPORTED (the packed coordinate tuple does not fit two 64-bit sort keys), ENOMEM, EHIP.
 */
conststn_status conststn_build_csf(int order, const int64_t *dims, int64_t nnz,
                                   const int32_t *const *coords, const double *vals,
                                   const int *mode_order, unsigned flags,
                                   conststn_stream stream, conststn_csf_t **out);

/* Describe a CSF: any output pointer may be NULL.  dims/mode_order receive `order` entries. */
conststn_status conststn_csf_info(const conststn_csf_t *csf, int *order, int64_t *dims,
                                  int *mode_order, int64_t *nnz);

/* Borrow the device arrays of one level (valid until destroy).  ptr is NULL for the last
 * level; vals is non-NULL only for the last level.  Any output pointer may be NULL. */
conststn_status conststn_csf_export(const conststn_csf_t *csf, int level, const int32_t **idx,
                                    const int64_t **ptr, int64_t *nodes, const double **vals);

/* Debugging aid: checks on the device every invariant of the array layout above (indices inside their
 * mode extents, ptr[l][0] = 0, every node with at least one child, ptr[l][nodes_l] = nodes_{l+1},
 * children of one parent and the roots strictly ascending).  CONSTSTN_OK, or CONSTSTN_EINVAL with the
 * violated invariants named in conststn_last_error().  Reads only inside the arrays' sizes. */
conststn_status conststn_csf_check(const conststn_csf_t *csf);

void conststn_csf_destroy(conststn_csf_t *csf);

/* ------------------------------------------------------------------------------------------
 * (2) Plan: a schedule in the paper's abstraction -- the sequence S of pairs <A, pi>
 *     (Sec. 4.2), in execution order (the ap_i of Sec. 3.2 "Ordering of assignments").
 *
 * schedule   host string, statements separated by ';', each
 *                 OUT[i,j,..] = A[..] * B[..] | loop,order,of,all,indices
 *            e.g. mode-0 TTMc of Sec. 5.3 with X stored i>j>k:
 *                 "T[i,j,s] = X[i,j,k] * U3[k,s] | i,j,k,s ; Y[i,r,s] = T[i,j,s] * U2[j,r] | i,j,r,s"
 *            A reference to a CSF operand lists its indices in LEVEL order (the paper writes
 *            A_ipq stored <d1,d2,d0> as A[p,q,i], Sec. 2.1); a dense operand's reference lists
 *            them in row-major storage order; the last statement's left side fixes the row-major
 *            layout of the output.
 * fusion     host pointer or NULL; fusion[p] = number of outermost loops statement p shares with
 *            the consumer of its result (-1 or NULL: the longest legal common prefix, which is
 *            what Algorithm 1 of Sec. 4.2 produces).  The entry of the last statement is ignored.
 *            The order of an intermediate after fusion is its order minus this depth.
 * operands   host pointer, n_operands descriptors naming every INPUT tensor of the schedule
 * flags      0 or CONSTSTN_OUT_COMPACT
 *
 * Legality rules checked (CONSTSTN_ESCHED when violated), all from Sec. 3.2:
 *   - every consumed intermediate is produced by an EARLIER statement, exactly once consumed
 *     (topological order of a tree);
 *   - each loop order is a permutation of the statement's indices; an index has one extent;
 *   - for every CSF operand, level order implies loop order ("Consistency between mode order
 *     and loop order"); not required of dense operands and of intermediates, which are dense
 *     workspaces;
 *   - the fused prefix of a producer consists of indices of its result ("Producer constraints"),
 *     equals the consumer's prefix position by position ("Consumer constraints"), and every
 *     statement between the two shares it ("Statements between producer and consumer").
 * Kernel choice.  Tuned kernels take: TTMc of order 3 (ranks up to 64) and order 4 (ranks up to
 * 16), MTTKRP of order 3 (rank up to 128), each with the sparse prefix fully fused, and the
 * three-tensor network (U.V).W fused on its two outer loops.  The chain of three sparse tensors of
 * Sec. 5.1 (every operand a CSF handle, sparse result: see conststn_plan_output_csf),
 *      "T[K,i,v] = I[K,u,v] * C[i,u] | K,i,u,v ; E[K,i,m] = T[K,i,v] * P[m,v] | K,i,m,v"
 * and its restricted form with a statement "F[K,i,v] = T[K,i,v] * L[K,i] | K,i,v" in between,
 * fused on the two outer loops, has a kernel of its own, and so has the four-index product of the
 * same section, "V[i,j,m,n] = Ea[i,K,m] * Eb[j,K,n] | i,j,K,m,n" (two CSF operands of order 3, which
 * may be one handle under two names; sparse result with levels i > j > m > n).  Every other legal tree over ONE CSF
 * operand and dense operands -- other orders and ranks, dense-only subtrees, several CSF levels
 * summed by one statement, a fully contracted result, a result indexed by CSF levels other than
 * the root (every output mode on one CSF; such a result is a dense array over the extents of all
 * its indices and is added into with fp64 atomics), any fusion choice -- runs on a generic
 * executor (one pass per statement, intermediates held whole in device memory; plan option
 * generic_max_gb bounds them, default 64).  A legal schedule outside all of
 * these gives CONSTSTN_EUNSUPPORTED with the reason.
 * The plan keeps pointers into the CSF handles: destroy the plan first.
 */
typedef enum { CONSTSTN_OPERAND_CSF = 0, CONSTSTN_OPERAND_DENSE = 1 } conststn_operand_kind;

typedef struct {
    const char *name;                    /* tensor name as written in the schedule             */
    int kind;                            /* conststn_operand_kind                               */
    const conststn_csf_t *csf;           /* CSF operands: the handle; otherwise NULL            */
    int order;                           /* dense operands: number of modes                     */
    int64_t dims[CONSTSTN_MAX_ORDER];    /* dense operands: extents in storage (row-major) order */
} conststn_operand_desc;

conststn_status conststn_plan(const char *schedule, const int *fusion, int n_operands,
                              const conststn_operand_desc *operands, unsigned flags,
                              conststn_plan_t **out);

/* conststn_plan with tuning options: `options` is a host string "name=value,name=value" (NULL or ""
 * = every default; values are non-negative integers; an unknown name, or a value outside what the
 * option takes, is CONSTSTN_EINVAL and the message names the values it takes).  The
 * options choose among kernel forms and partition sizes that compute the same result; they are read
 * while the plan is built and stored in it -- nothing is read from the environment, and an execute
 * reads no option.  Names (default): force_generic (0; 1 = the generic executor also where a tuned
 * kernel exists), generic_max_gb (64), generic_span (4096), generic_densify (1: a tree over several CSF operands runs on the generic executor, which walks the
 * largest and keeps dense copies of the others; 0 = such trees are refused), generic_fuse (1; 0 = the generic
 * executor stores every intermediate whole even where the schedule fuses), reroot (1; 0 = no private re-sorted copy of the
 * tensor for MTTKRP / TTMc of a non-root level: the generic executor takes those), mttkrp_split (1), mttkrp_dual (44 = hot and cold sub-tensor in one launch, four
 * wavefronts of a workgroup each; 35, 53, 88 likewise; 0 = two launches), mttkrp_hot (256),
 * mttkrp_chunk (0 = by tensor size), ttmc3_mfma (1), ttmc3_stream (1), ttmc3_producers (4),
 * ttmc3_batch (2048), ttmc3_itemcost (2), ttmc3_qn (2), ttmc3_split (4096), ttmc3_rowsplit (by size),
 * ttmc4_mfma (1), ttmc4_split (256), ttmc4_ksplit (by size), sptn3_tiled (1; 0 = baseline kernel, 2 = tiled kernel
 * also where W fills its 16 x 16 tiles to less than a sixteenth),
 * sptn3_waves (2), sptn3_wgs (8000), sptn3_xcd (0), spchain3_form (1; 2 = general numeric pass),
 * spchain3_local_kb (78), spchain3_pk_gb (4), sppair4_keep (1), sppair4_keep_gb (4), sppair4_rows (1),
 * spchain3_order (1 = workgroups take the roots of the result by falling cost, 0 = in root order),
 * sppair4_rows_gb (8), sppair4_buffers (2), sppair4_xcd (2 = workgroups take the pairs by falling cost,
 * 1 = by j mod 8 per XCD, 0 = in node order). */
conststn_status conststn_plan_options(const char *schedule, const int *fusion, int n_operands,
                                      const conststn_operand_desc *operands, unsigned flags,
                                      const char *options, conststn_plan_t **out);

/* Host-only: parse and check a schedule exactly as conststn_plan does, and lower it to
 * nested forall / where text (the concrete-index-notation shape of Sec. 4.1, produced by the
 * grouping recursion of Sec. 4.2), without binding kernels or touching a device.  CSF operands
 * may be described by structure only: csf = NULL, order and dims (extents in LEVEL order) set.
 * reduced_orders (host pointer or NULL) receives, per statement, the order of its result
 * after fusion.  Writes at most len-1 characters + NUL to buf (buf may be NULL). */
conststn_status conststn_schedule_check(const char *schedule, const int *fusion, int n_operands,
                                        const conststn_operand_desc *operands, char *buf,
                                        size_t len, int *reduced_orders);

/* Host-only: schedule search -- the question of Sec. 3 asked for l = 1, 2, ... until it has an answer.
 * tree        statements "OUT[..] = A[..] * B[..]" separated by ';', WITHOUT loop orders, forming
 *             a tree (every intermediate consumed once; any statement order).  At most 6
 *             statements of at most 8 indices each; every operand referenced once.
 * operands    as for conststn_schedule_check, CSF operands by structure only (csf = NULL); their
 *             extents follow the order of the reference in `tree`
 * flags       0: a reference to a CSF operand lists its MODES and the level order is chosen (the
 *             dp variables of Sec. 3.2); CONSTSTN_SEARCH_KEEP_LAYOUT: it is a level order to keep
 * max_order   stop after this l (0: no bound other than the largest intermediate)
 * buf, len    receives a schedule in the form conststn_plan takes: statements in the order found,
 *             CSF references rewritten in level order, one loop order each
 * order_found receives the smallest l for which every intermediate has order <= l after fusion
 * level_modes NULL or n_operands * CONSTSTN_MAX_ORDER ints: for operand o, entry
 *             [o * CONSTSTN_MAX_ORDER + level] = position in the tree's reference of the mode stored
 *             at that level (-1 beyond the operand's order) -- pass it, composed with the modes of
 *             the reference, as mode_order to conststn_build_csf
 * The space of Sec. 3.2 (topological orders x loop permutations; layouts follow the loops) is
 * enumerated with pruning instead of being given to a solver.  Among the schedules for the smallest
 * l found within a bounded walk the one with the fewest statements whose summed index is the
 * innermost loop, then with the smallest intermediates, is returned.  CONSTSTN_ESCHED when layouts
 * that were fixed admit no schedule up to max_order. */
#define CONSTSTN_SEARCH_KEEP_LAYOUT 1u
conststn_status conststn_schedule_search(const char *tree, int n_operands,
                                         const conststn_operand_desc *operands, unsigned flags,
                                         int max_order, char *buf, size_t len, int *order_found,
                                         int *level_modes);

/* Output shape: n_rows row blocks of row_elems fp64 each, row-major.  Without
 * CONSTSTN_OUT_COMPACT n_rows is the extent of the output's first index (rows of empty
 * slices are zero); with it n_rows is the number of nonempty root indices. */
conststn_status conststn_plan_output_size(const conststn_plan_t *plan, int64_t *n_rows,
                                          int64_t *row_elems);

/* Compact output only: device pointer to the n_rows root index values (ascending) the row
 * blocks belong to; borrowed, valid until the CSF is destroyed. */
conststn_status conststn_plan_output_rows(const conststn_plan_t *plan, const int32_t **rows,
                                          int64_t *n_rows);

/* Sparse result (Sec. 5.1: a product of sparse tensors whose result is sparse too).  The
 * structure of the result -- its structural nonzeros by the join of Sec. 2.1, independent of the
 * values -- is computed when the plan is made and is returned here as a CSF handle without
 * values (conststn_csf_export gives idx/ptr per level, vals = NULL; levels in the order of the
 * result's indices in the schedule).  conststn_plan_output_size then reports n_rows = number of
 * structural nonzeros, row_elems = 1, and conststn_execute writes one value per leaf of that
 * structure, in leaf order.  Borrowed: valid until the plan is destroyed; never pass it to
 * conststn_csf_destroy.  CONSTSTN_EINVAL when the plan's result is dense. */
conststn_status conststn_plan_output_csf(const conststn_plan_t *plan, const conststn_csf_t **structure);

/* Debugging aid: the kernels trust the tables a plan holds (an index out of range there is a memory
 * fault, not an error code).  This pass checks, on the device, that every table of an order-3 MTTKRP
 * or TTMc plan (Sec. 5.2, 5.3) stays inside the arrays it indexes: chunk tables against the pointer arrays,
 * the re-encoded leaf stream (LDS slots, factor rows, end-of-fiber / end-of-slice marks), row
 * descriptors, items, K-steps and workgroup batches of the TTMc kernels, and the tensor the kernels
 * walk (conststn_csf_check of it).  For a plan of the generic executor: the segment tables of its long
 * sums (every result node's children, or leaves, tiled in order by segments of the stated length), the
 * lists of nodes with many segments, and the first-leaf tables of fused statements against the
 * composition of the pointer arrays.  CONSTSTN_OK; CONSTSTN_EINVAL with the violations named;
 * CONSTSTN_EUNSUPPORTED for plans of other kernel families. */
conststn_status conststn_plan_check(const conststn_plan_t *plan);

/* Text description of the lowered plan (kernel family, loop tree in forall/where form,
 * order of each intermediate after fusion).  Writes at most len-1 characters + NUL. */
conststn_status conststn_plan_describe(const conststn_plan_t *plan, char *buf, size_t len);

void conststn_plan_destroy(conststn_plan_t *plan);

/* ------------------------------------------------------------------------------------------
 * (3) Execute the fused loop nest (Fig. 3b / Fig. 4 of the paper: outer fused loops walk
 *     the top CSF levels, reduced-order dense temporaries live on chip, the consumer
 *     accumulates into the output).
 *
 *   dense_factors  host pointer to device pointers, one per DENSE operand, in the order the
 *                  dense operands appear in the plan's operand list; row-major, read only
 *   out            device pointer, n_rows * row_elems fp64; fully overwritten
 *   stream         all work is enqueued here; the call does not wait for it
 *
 * Scratch memory owned by the plan is reused by every execute of that plan: two executes of
 * ONE plan must not overlap in time (different plans may).
 */
conststn_status conststn_execute(const conststn_plan_t *plan, const double *const *dense_factors,
                                 double *out, conststn_stream stream);

/* conststn_execute for callers that may not allocate device memory -- code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc -- and want no plan-owned scratch either:
 * the partial row blocks of slices cut into several work items live in a static device array of
 * CONSTSTN_STATIC_SCRATCH_BYTES that is part of the library's code object (each GPU the library runs
 * on holds its own copy until the process ends).  The call allocates and frees nothing.  Plans of
 * the order-3 TTMc kernels only (CONSTSTN_EUNSUPPORTED otherwise, and when the plan's partial row
 * blocks need more than the static area: the message names both sizes).  Arguments, output layout
 * and results are those of conststn_execute.  Every call on one GPU shares that GPU's array,
 * whatever the plan: calls that overlap in time on one GPU race (conststn_execute calls of other
 * plans do not use it).  Nothing in the array needs clearing between calls: every partial block a
 * call reads it has written before. */
#define CONSTSTN_STATIC_SCRATCH_BYTES (64u << 20)
conststn_status conststn_execute_static(const conststn_plan_t *plan, const double *const *dense_factors,
                                        double *out, conststn_stream stream);

/* Measurement hook (for benchmarks; not part of the method).  After
 * conststn_plan_profile(plan, capacity > 0) every conststn_execute of the plan brackets its
 * DOMINANT kernel (the fused traversal kernel, not the zero-fill or fix-up passes) with a pair
 * of HIP events recorded on the execute's stream; capacity pairs are kept (older ones are
 * overwritten).  conststn_plan_kernel_times waits for the recorded events and writes up to
 * max_n durations in milliseconds, oldest first, to the host array ms, and their count to n;
 * it then forgets them.  capacity = 0 switches the hook off.  The name of the bracketed kernel
 * family is given by conststn_plan_describe ("family=..."). */
conststn_status conststn_plan_profile(conststn_plan_t *plan, int capacity);
conststn_status conststn_plan_kernel_times(conststn_plan_t *plan, float *ms, int max_n, int *n);

/* Measurement hook (for benchmarks; not part of the method): what the current device delivers on
 * the ceilings the kernels are priced against, so that a benchmark can print a measured figure
 * beside the published one.  Synchronous; allocates and frees its own device buffers.
 *   CONSTSTN_PEAK_COPY      size = bytes (multiple of 16): a plain streaming copy of `size` bytes,
 *                           repeated `repeats` times; *result = GB/s counting bytes read + written
 *   CONSTSTN_PEAK_WRITE     size = bytes (multiple of 16): a plain fill; *result = GB/s written
 *   CONSTSTN_PEAK_MFMA_F64  size = rounds: every wavefront of a full-chip launch (four per SIMD)
 *                           issues 8 * size independent v_mfma_f64_16x16x4f64; *result = TFLOP/s
 *   CONSTSTN_PEAK_MFMA_CLOCK  the same loop; *result = shader clock in MHz while it runs (cycle counter
 *                           of one wavefront against the constant-rate wall clock)
 *   CONSTSTN_PEAK_VALU_CLOCK  size = rounds of a loop of dependent 32-bit adds on one wavefront per CU;
 *                           *result = shader clock in MHz of a lightly loaded chip
 * Errors: EINVAL, ENOMEM, EHIP. */
#define CONSTSTN_PEAK_COPY 0
#define CONSTSTN_PEAK_WRITE 1
#define CONSTSTN_PEAK_MFMA_F64 2
#define CONSTSTN_PEAK_MFMA_CLOCK 3
#define CONSTSTN_PEAK_VALU_CLOCK 4
conststn_status conststn_measure_peak(int what, int64_t size, int repeats, conststn_stream stream,
                                      double *result);

/* Message of the last failure on this thread ("" if none). */
const char *conststn_last_error(void);

/* Library version string. */
const char *conststn_version(void);

#ifdef __cplusplus
}
#endif
#endif /* CONSTSTN_H */
