/*
 * hgnn -- half-precision sparse aggregation kernels for GNN training on
 * AMD MI355X (CDNA4, gfx950): C ABI of libhgnn.so.
 *
 * The operations are the sparse kernels of "Optimization of GNN Training
 * Through Half-precision" (HalfGNN, HPDC'25): SpMM  Y <- A_w X  and its
 * backward  dX <- A_w^T dY  (section 2.1.2), the discretized-reduction SpMM
 * without atomic writes (section 5.2), SDDMM  dW_e <- A (.) (dY X^T)
 * (sections 2.1.2, 5.1), and the edge softmax of Eq. 1 with its backward.
 *
 * General rules
 *  - Every pointer in this header that is not marked HOST is a DEVICE pointer
 *    owned by the caller.  The library never frees or keeps caller memory: a plan
 *    remembers the sizes of the graph it was built for, and a column-blocked plan
 *    (hgnn_plan_create, col_blocks) also keeps its own re-ordered copy of the column ids
 *    and of the edge-id map of that graph.
 *  - fp16 data (hgnn_half) is IEEE binary16 stored as 16-bit words.
 *    Vertex-level tensors are row major [rows][ld] with ld >= F (section 2.1.1:
 *    |V| x |F|); edge-level tensors are edge major [nnz][H].  Head h owns the
 *    features [h*D, (h+1)*D), D = F / H.
 *  - Graph orientation: row i = destination vertex, the non-zeros of row i are
 *    its neighbourhood N(i); columns are neighbour ids.  Duplicate non-zeros
 *    are separate edges.
 *  - `stream` is a hipStream_t passed as void* (NULL = the null stream).  All
 *    compute entry points are asynchronous on that stream, never synchronize and
 *    never allocate: scratch memory comes from the plan or from a workspace argument
 *    that the caller owns (hgnn_spmm, hgnn_linear_wgrad, hgnn_gat_feature_grad).
 *    hgnn_plan_create, hgnn_plan_add_groups, hgnn_plan_add_slices, the export calls, hgnn_transpose,
 *    hgnn_coo_to_csr and hgnn_csr_validate allocate and/or synchronize (one-off set-up calls).
 *  - A plan owns scratch that the calls using it write (staging rows, per-vertex
 *    tables, per-block partial outputs): calls that use the same plan must be ordered
 *    on one stream, or otherwise not overlap in time; different plans are independent.
 *    The same holds for a workspace.  Host-side, the library keeps no mutable state
 *    except the thread-local error string and two per-device facts that are looked up once
 *    (the cache sizes, the address of the static scratch array of hgnn_spmm_static).
 *  - Arithmetic: fp16 in memory, fp32 in registers, one round-to-nearest-even
 *    conversion when a value is stored.
 *  - Errors: every call returns an hgnn_status; argument errors are detected on
 *    the host before anything is launched.  hgnn_last_error() returns a
 *    thread-local detail string for the last failing call of this thread.
 *  - Feature widths: odd F is rejected (HGNN_EINVAL): pad to the next even
 *    number as section 4.1 prescribes for half2.  The 16-byte vector path needs
 *    row pitches (ld) that are multiples of 8 halves and 16-byte aligned base
 *    pointers; F itself may be any even number up to 512 (e.g. 42 classes in rows
 *    of pitch 48): rows are read in 16-byte pieces up to the pitch, whatever the
 *    padding columns hold never reaches a result, and padding columns of outputs
 *    are not written.  With several heads of edge values (or SDDMM heads) D must
 *    be a multiple of 8.  Other shapes take a slower scalar path in hgnn_spmm /
 *    hgnn_sddmm and are HGNN_EUNSUPPORTED in hgnn_spmm_discretized.
 */
#ifndef HGNN_H
#define HGNN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef uint16_t hgnn_half; /* IEEE binary16 bit pattern */

typedef enum {
  HGNN_OK = 0,
  HGNN_EINVAL = 1,       /* bad argument (NULL, size, alignment, odd F, inconsistent graph) */
  HGNN_EUNSUPPORTED = 2, /* valid but not implemented for this shape */
  HGNN_ENOMEM = 3,       /* device or host allocation failed */
  HGNN_EHIP = 4          /* a HIP call or kernel launch failed */
} hgnn_status;

/* reduce op of SpMM.  MEAN = SUM followed by the degree norm 1/deg(i)
 * (section 5.2.2 treats "SpMM + degree-norm" as SpMM with reduce = mean). */
typedef enum { HGNN_SUM = 0, HGNN_MEAN = 1 } hgnn_reduce;

typedef enum {
  HGNN_SDDMM_DOT = 0,      /* out[k,h] = sum_d U[row k,h,d] * Vt[col k,h,d]              (section 2.1.2) */
  HGNN_SDDMM_GAT_SCORE = 1 /* out[k,h] = LeakyReLU(a_l[h].U[row k,h] + a_r[h].Vt[col k,h]) (section 3.1.2) */
} hgnn_sddmm_op;

/* A sparse matrix / graph in CSR (section 2.1.1: offset array + column ids),
 * optionally with COO row ids and an edge-id map. */
typedef struct {
  int32_t nrows;         /* |V| of the destination side */
  int32_t ncols;         /* |V| of the neighbour side */
  int64_t nnz;           /* |E|, must be < 2^31 */
  const int32_t* rowptr; /* [nrows+1] non-decreasing, rowptr[0] = 0, rowptr[nrows] = nnz */
  const int32_t* col;    /* [nnz] 0 <= col < ncols, ascending inside a row (duplicates allowed) */
  const int32_t* row;    /* [nnz] COO row id of every non-zero, or NULL (only read by hgnn_sddmm without a plan) */
  const int32_t* eid;    /* [nnz] or NULL.  Edge tensors are read at slot eid[k] for CSR position k
                            (the transposed graph refers to the original graph's edge tensors) */
} hgnn_csr;

typedef struct hgnn_plan hgnn_plan; /* opaque; device arrays owned by the library */

const char* hgnn_status_str(hgnn_status s);
const char* hgnn_last_error(void);

/* One device pass over the graph: rowptr monotone with the right end points,
 * columns in range and ascending inside a row, row ids (if given) consistent with
 * rowptr, eid (if given) in [0,nnz).  Synchronizes.  HGNN_EINVAL names the first
 * rule broken. */
hgnn_status hgnn_csr_validate(const hgnn_csr* g, void* stream);

/* CSR of A^T plus the edge-id map, for the backward SpMM dX <- A_w^T dY
 * (section 2.1.2).  Outputs (device, caller allocated): rowptr_T [ncols+1],
 * col_T [nnz] (= source rows of A), eid_T [nnz] (= CSR position in A of that
 * non-zero).  Inside a row of A^T entries keep their order in A (a stable sort
 * by column).  g->eid must be NULL.  Allocates temporary storage, synchronizes. */
hgnn_status hgnn_transpose(const hgnn_csr* g, int32_t* rowptr_T, int32_t* col_T, int32_t* eid_T, void* stream);

/* CSR from a COO edge list (section 2.1.1: COO stores one (rowID, colID) pair per non-zero, CSR the
 * offset array and the column ids row by row).  Inputs (device): row [nnz], col [nnz] in any order,
 * 0 <= row < nrows, 0 <= col < ncols; duplicate pairs are separate edges.  Outputs (device, caller
 * allocated): rowptr [nrows+1], col_out [nnz] (ascending inside a row, duplicates in list order: a stable
 * sort by (row, col)) and, unless NULL, eid [nnz] = the list position of every CSR non-zero, so that an
 * edge tensor given in list order is read through it (hgnn_csr.eid) or reordered once
 * (hgnn_edge_to_transposed with a graph that carries this map).  Allocates temporary storage,
 * synchronizes.  HGNN_EINVAL for an id out of range (the outputs are then unspecified). */
hgnn_status hgnn_coo_to_csr(int32_t nrows, int32_t ncols, int64_t nnz, const int32_t* row, const int32_t* col,
                            int32_t* rowptr, int32_t* col_out, int32_t* eid, void* stream);

/* Brings an edge tensor into the edge order of the transposed graph: t_T[k,h] = t[gt->eid[k], h]
 * (fp16 [nnz][H], not in place).  For edge values that do not change between steps (the
 * normalised weights of a GCN, section 3.1.3) this is done once; the backward SpMM then runs
 * on the transposed graph *without* its edge-id map, reading t_T as a stream instead of
 * gathering two bytes per non-zero.  Asynchronous on `stream`. */
hgnn_status hgnn_edge_to_transposed(const hgnn_csr* gt, int32_t H, const hgnn_half* t, hgnn_half* t_T, void* stream);

/* Segment plan for the discretized SpMM (section 5.2.1, observation rules 1-3):
 * the non-zeros are dealt out in storage order in segments of seg_edges edges,
 * segment k = [k*S, min(nnz,(k+1)*S)).  The plan holds, on the device: the row
 * of the first and last edge of every segment, the ascending list of "split"
 * rows (first and last edge in different segments) with the segments they
 * span, the list of rows longer than 2048 edges, the staging buffer for
 * conflicting partial sums (2 vectors of max_F halves per segment; the paper's
 * buffer is one vector per CTA, section 5.2.3) and per-vertex fp32 scratch of
 * 2*max_H floats per row/column for the factorised GAT score.
 * The graph is validated first.  A plan may be used by one stream at a time.
 * seg_edges in [1, 2048]; max_F >= 8 multiple of 8; max_H >= 1.
 *
 * col_blocks: column blocking of hgnn_spmm_discretized.  1 = none.  n in [2, 64]:
 * the columns are cut into n equal ranges, the non-zeros of every range are
 * copied into a CSR of their own (a row's share of a range is a contiguous piece
 * of the row because columns ascend inside a row) with a segment plan each; the
 * SpMM then runs range after range, so that all compute units gather from one
 * slice of X at a time, into n partial outputs [n][nrows][max_F] fp16 that one
 * more pass adds per row.  Every partial still covers at most seg_edges edges and
 * is scaled before it is rounded (section 5.2.2).  0 = automatic: blocking is
 * chosen when the feature table (ncols * max_F halves) is larger than three L2s but
 * fits three quarters of the cache behind them (sizes read from the device) and rows
 * average 128 non-zeros or more; with blocks chosen this way a call whose own table
 * (ncols * ldx halves) is below that size runs unblocked (blocks asked for by number are
 * always used).  Costs nnz * 8 bytes plus the partial outputs.  A graph that is blocked by
 * the automatic rule is also kept in twice as many blocks: hgnn_spmm_discretized takes those
 * when it has edge values to read through an edge-id map (the scattered reads of the edge
 * tensor are a second table to keep in the L2s), hgnn_sddmm (dot) always (it leaves no
 * partial rows behind); the same cost once more.
 * Edge tensors with a blocked plan: a call whose graph has no edge-id map reads them at the
 * graph's own CSR positions, whatever graph the plan was built from; a call whose graph has
 * an edge-id map reads them through the plan's blocked copy of the map, so the plan must
 * have been built from a graph with that same map (HGNN_EINVAL when it was built without
 * one).  hgnn_sddmm and hgnn_edge_rowsum use the blocks only where they match the call
 * (a plan built without a map for hgnn_sddmm, with one for hgnn_edge_rowsum over a map). */
hgnn_status hgnn_plan_create(const hgnn_csr* g, int32_t seg_edges, int32_t max_F, int32_t max_H, int32_t col_blocks,
                             hgnn_plan** out, void* stream);
int64_t hgnn_plan_num_segments(const hgnn_plan* p);
int32_t hgnn_plan_num_split_rows(const hgnn_plan* p);
int32_t hgnn_plan_seg_edges(const hgnn_plan* p);
int32_t hgnn_plan_col_blocks(const hgnn_plan* p); /* 1 when the plan is not column blocked */
int32_t hgnn_plan_col_blocks_fine(const hgnn_plan* p); /* blocks of the finer cut (= col_blocks when there is none) */
/* The cache sizes that hgnn_plan_create read from the device for its automatic column-block rule (HOST
 * outputs, each may be NULL): one L2 (per XCD) and the last-level cache behind the L2s, in bytes. */
void hgnn_plan_cache_bytes(const hgnn_plan* p, int64_t* l2_bytes, int64_t* llc_bytes);
/* Column block b of a blocked plan, copied to HOST buffers (each may be NULL):
 * *nnz_b; rowptr_b [nrows+1]; col_b, eid_b [*nnz_b] (eid_b = slot in the edge
 * tensors = g->eid[k] or k of the original non-zero k); seg_row_lo / seg_row_hi
 * [ceil(*nnz_b / seg_edges)].  Call once with NULL arrays to learn *nnz_b.  Synchronizes. */
hgnn_status hgnn_plan_block_export(const hgnn_plan* p, int32_t b, int64_t* nnz_b, int32_t* rowptr_b, int32_t* col_b,
                                   int32_t* eid_b, int32_t* seg_row_lo, int32_t* seg_row_hi);
/* Copies the plan's integer arrays to HOST buffers (each may be NULL to skip):
 * seg_row_lo / seg_row_hi [num_segments]; split_row / split_seg_lo /
 * split_seg_hi [num_split_rows].  Synchronizes. */
hgnn_status hgnn_plan_export(const hgnn_plan* p, int32_t* seg_row_lo, int32_t* seg_row_hi, int32_t* split_row,
                             int32_t* split_seg_lo, int32_t* split_seg_hi);
void hgnn_plan_destroy(hgnn_plan* p);

/* SpMM, vertex-parallel (sections 2.1.2, 4.1): for every row i
 *   Y[i,f] = s_i * sum_{k in row i} w[slot(k), f/D] * X[col[k], f],   slot(k) = eid ? eid[k] : k,
 * w == NULL means all ones (SpMMv); s_i = 1 (SUM) or 1/max(deg_i,1) (MEAN), times
 * row_scale[i] (fp32 [nrows]) when row_scale != NULL.  The scale is applied once,
 * after the whole row is reduced (post-reduction scaling).  Y is fully
 * overwritten (empty rows become 0).  X is [ncols][ldx], Y is [nrows][ldy].
 * Rows above 8 times the mean length (the threshold kept within 256..1024 non-zeros) are cut
 * into chunks of 512 non-zeros that are reduced by a wavefront each and added in chunk order;
 * their lists and fp32 partial rows live in `workspace`: device memory of at least
 * hgnn_spmm_workspace(nrows, ncols, nnz, F) bytes, 16-byte aligned, owned by the caller,
 * overwritten, not to be shared by calls that overlap in time.  The size is a bound from the
 * four numbers alone (0 when no row of such a graph can be that long).  workspace == NULL is
 * allowed: every long row is then reduced by a single wavefront (correct, slow on hubs).
 * Where the table X (ncols rows of F halves) is beyond three L2s, fits three quarters of the
 * cache behind them and rows average 128 non-zeros or more, the call walks the columns in
 * passes (ranges of about two L2 sizes of feature rows, all wavefronts in the same range at
 * the same time): a row's share of a pass is reduced into an fp32 partial row in the
 * workspace and the partials are added in pass order, scaled and rounded once -- the same
 * arithmetic, the sums in another fixed order.  hgnn_spmm_workspace counts that room in
 * (npass * nrows * F * 4 bytes and the cut positions); with ncols = 0 it returns the bound of
 * the long rows alone, and a workspace of that size is accepted too: the call then takes one
 * sweep per row. */
size_t hgnn_spmm_workspace(int32_t nrows, int32_t ncols, int64_t nnz, int32_t F);
hgnn_status hgnn_spmm(const hgnn_csr* g, const hgnn_half* edge_val, int32_t H, const hgnn_half* X, int64_t ldx,
                      hgnn_half* Y, int64_t ldy, int32_t F, hgnn_reduce op, const float* row_scale, void* workspace,
                      size_t workspace_bytes, void* stream);

/* hgnn_spmm for callers that cannot allocate and own no workspace: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, kernels and results as hgnn_spmm with a
 * workspace of hgnn_spmm_workspace(nrows, 0, nnz, F) bytes (one sweep per row, no column passes); the scratch of the long rows is a static device array of hgnn_spmm_static_limit() bytes
 * (32 MiB) inside the library, held by every device the library runs on until the process ends.  A graph
 * whose bound for the long rows, hgnn_spmm_workspace(nrows, 0, nnz, F), exceeds that limit is refused with HGNN_EUNSUPPORTED
 * before anything is launched (use hgnn_spmm with a workspace).  Allocates nothing, asynchronous on
 * `stream`.  All calls on one device share the array: calls that overlap in time on one device (two
 * streams, two threads) race; order them on one stream. */
size_t hgnn_spmm_static_limit(void);
hgnn_status hgnn_spmm_static(const hgnn_csr* g, const hgnn_half* edge_val, int32_t H, const hgnn_half* X, int64_t ldx,
                             hgnn_half* Y, int64_t ldy, int32_t F, hgnn_reduce op, const float* row_scale, void* stream);

/* Discretized-reduction SpMM, edge-parallel, no atomic writes (section 5.2):
 * same result as hgnn_spmm, but every wavefront reduces one segment of the plan,
 * each partial sum covers at most seg_edges edges and is scaled by s_i before it
 * is rounded to fp16 (discretized reduction scaling, section 5.2.2), rows inside
 * one segment are stored directly, partials of rows that cross a segment boundary
 * go to the plan's staging buffer and a follow-up kernel adds them in ascending
 * segment order and stores the row once (section 5.2.3).  Deterministic.
 * Needs F <= 512, ld % 8 == 0, 16-byte aligned X and Y, D % 8 == 0 when edge values have
 * several heads, F <= plan max_F, and the plan of this graph. */
hgnn_status hgnn_spmm_discretized(const hgnn_plan* p, const hgnn_csr* g, const hgnn_half* edge_val, int32_t H,
                                  const hgnn_half* X, int64_t ldx, hgnn_half* Y, int64_t ldy, int32_t F,
                                  hgnn_reduce op, const float* row_scale, void* stream);

/* Degree norms and the GIN epilogue fused into the discretized SpMM (sections 3.1.3,
 * 5.2.2; Eq. 2, Eq. 3 and its half-precision form):
 *   Y[i,f] = self_coef * self[i,f] + sum over the partials P of row i of fp16(P),
 *   P = agg_coef * s_i * sum_{k in batch} w[slot(k), f/D] * col_scale[col[k]] * X[col[k], f]
 * with s_i as in hgnn_spmm (reduce op and row_scale).  GCN "both" norm: row_scale =
 * deg^-1/2 of the rows, col_scale = deg^-1/2 of the columns, no edge values.  GIN:
 * self = X, self_coef = 1 + eps, agg_coef = 1 (Eq. 3) or lambda with reduce = MEAN
 * (the overflow-safe form, lambda = 0.1 in the paper).  Empty rows get the self term
 * alone.  A NULL pointer or fz == NULL drops that part (agg_coef must then be 1).
 * scaled_x is an optional workspace for the column scale: when it and col_scale are given, the call
 * first writes fp16(col_scale[j] * X[j,f]) into it (one pass over the table) and then gathers from
 * it without a per-edge factor.  A per-edge factor fetched from another table costs a third cache
 * request per non-zero beside the two of a 128-byte feature row; the workspace form costs one pass
 * over ncols x F halves and one more fp16 rounding per table element (within the tolerance of the
 * plain call).  The caller owns the workspace; it is overwritten. */
typedef struct {
  const float* col_scale; /* [ncols] fp32 or NULL */
  const hgnn_half* self;  /* [nrows][ld_self] fp16 or NULL; ld_self >= F, ld_self % 8 == 0, 16-byte aligned */
  int64_t ld_self;
  float self_coef;
  float agg_coef;
  hgnn_half* scaled_x;    /* [ncols][ld_scaled] fp16 workspace or NULL; ld_scaled >= F, % 8 == 0, 16-byte aligned */
  int64_t ld_scaled;
} hgnn_spmm_fusion;

hgnn_status hgnn_spmm_discretized_fused(const hgnn_plan* p, const hgnn_csr* g, const hgnn_half* edge_val, int32_t H,
                                        const hgnn_half* X, int64_t ldx, hgnn_half* Y, int64_t ldy, int32_t F,
                                        hgnn_reduce op, const float* row_scale, const hgnn_spmm_fusion* fz,
                                        void* stream);

/* The comparison variants of the discretized SpMM that the paper measures against its own
 * design (sections 4.2, 5.4, 6.3.2 "atomic vs. non-atomic writes", 6.3.3 vertex-parallel form); same
 * arguments, same result up to fp16 rounding order, always on the whole graph (a plan's
 * column blocks are not used).
 *  HGNN_EDGE_SEGMENTS          the library's own design, identical to hgnn_spmm_discretized.
 *  HGNN_EDGE_SEGMENTS_ATOMIC   same segment kernel, but the partials of a row that crosses a
 *      segment boundary are added to Y with packed fp16 atomic adds (rows concerned are zeroed
 *      first) instead of going through the staging buffer and the follow-up kernel; the order
 *      of those additions, hence the last bits of such rows, varies from run to run.
 *  HGNN_VERTEX_GROUPS          vertex-parallel: every row is cut into neighbour groups of at
 *      most group_edges non-zeros, a wavefront reduces one group, so no batch holds two rows;
 *      a row of several groups stages one scaled fp16 partial per group and a follow-up kernel
 *      adds them (no atomics, deterministic).  Edge values of a group that starts at an odd
 *      position are fetched as aligned pairs from one position earlier.  Needs
 *      hgnn_plan_add_groups on the plan first.
 *  HGNN_VERTEX_GROUPS_HALF2    HGNN_VERTEX_GROUPS with the paper's arithmetic (section 4.2): inside a
 *      lane's share of a neighbour group the products and the sum are packed fp16 (two features per
 *      instruction, the edge value mirrored into both halves); everything after that as above.  For
 *      measurement: the result carries fp16 accumulation error (about group_edges * 2^-11 relative
 *      to the sum of the terms' magnitudes) and a lane's partial must fit fp16. */
typedef enum {
  HGNN_EDGE_SEGMENTS = 0,
  HGNN_EDGE_SEGMENTS_ATOMIC = 1,
  HGNN_VERTEX_GROUPS = 2,
  HGNN_VERTEX_GROUPS_HALF2 = 3
} hgnn_spmm_variant;

hgnn_status hgnn_spmm_discretized_variant(const hgnn_plan* p, const hgnn_csr* g, const hgnn_half* edge_val, int32_t H,
                                          const hgnn_half* X, int64_t ldx, hgnn_half* Y, int64_t ldy, int32_t F,
                                          hgnn_reduce op, const float* row_scale, hgnn_spmm_variant variant,
                                          void* stream);

/* Builds (or rebuilds) inside plan p the neighbour groups of graph g for HGNN_VERTEX_GROUPS
 * (section 5.4): group_edges in [1, 1024] neighbours per group, groups listed in row order, a
 * staging slot of max_F halves for every group of a row that has more than one.  Device
 * allocations owned by the plan; synchronizes the stream.  Not to be called while a kernel
 * that uses the plan is in flight. */
hgnn_status hgnn_plan_add_groups(hgnn_plan* p, const hgnn_csr* g, int32_t group_edges, void* stream);
int64_t hgnn_plan_num_groups(const hgnn_plan* p);
int32_t hgnn_plan_group_edges(const hgnn_plan* p);
/* Copies the group list to host arrays of hgnn_plan_num_groups entries: group_row[j] = row of
 * group j, group_first[j] = CSR position of its first non-zero.  Synchronizes the device. */
hgnn_status hgnn_plan_groups_export(const hgnn_plan* p, const hgnn_csr* g, int32_t* group_row, int32_t* group_first);

/* Column slices for the per-edge passes whose only random access is one scalar per column (section 3.1.2: the
 * factorised GAT score adds a per-column term to every non-zero; section 2.1.2: the backward pass sums an edge
 * tensor per column): the columns are cut into equal slices of at most slice_cols columns (64 .. 16384, 0 = 16384: the
 * scalars of a slice then fill the LDS of one workgroup), the rows into chunks of about equal numbers of non-zeros, and the
 * plan stores where every row's piece of every slice begins ((slices + 1) * nrows ints) plus partial column sums
 * (8 bytes * ncols per row chunk).  hgnn_sddmm GAT_SCORE, hgnn_gat_alpha (one head) and hgnn_edge_colsum then walk
 * (slice, chunk) pairs with the slice's scalars in LDS, so that memory only sees the streams of column ids and
 * edge values.  It pays where rows are long: hgnn_plan_create(col_blocks = 0) adds the slices by itself when a
 * row's piece of a slice averages 16 non-zeros or more.  Device allocations owned by the plan; synchronizes the
 * stream; not to be called while a kernel that uses the plan is in flight. */
hgnn_status hgnn_plan_add_slices(hgnn_plan* p, const hgnn_csr* g, int32_t slice_cols, void* stream);
int32_t hgnn_plan_num_slices(const hgnn_plan* p); /* 0 = none */

/* Vector-width study (sections 5.1.2-5.1.3 and 6.3.1: half2 against half8): halves that a lane
 * moves per feature load, 8 (16 bytes, the default and the library's design), 4 or 2.  A setting
 * of the plan, read at launch time by the two kernels that exist in all three widths: the SDDMM
 * DOT over the plan (hgnn_sddmm) and the main kernel of HGNN_VERTEX_GROUPS.  A narrower width
 * uses more lanes per feature row (F <= 64 * halves, D % halves == 0, feature table below 4 GiB
 * for the SpMM; otherwise HGNN_EUNSUPPORTED).  Every other kernel ignores it.  Results are the
 * same up to the order of the fp32 additions.  Host-side state of the plan: set it while no call
 * that uses the plan is being issued from another thread. */
hgnn_status hgnn_plan_set_vector_halves(hgnn_plan* p, int32_t halves);
int32_t hgnn_plan_vector_halves(const hgnn_plan* p); /* 0 for NULL */

/* out[i, f] = fp16(scale[i] * X[i, f]) for i < n, f < F (rows of pitch ldx / ldo, both multiples of 8;
 * the last 16-byte piece of a row is written up to the pitch when F is not a multiple of 8).  The
 * cheaper way to apply a column-side degree norm (Eq. 2) on graphs with more than a few edges per
 * vertex: scale the feature table once, then run the SpMM without a per-edge factor, instead of
 * col_scale in hgnn_spmm_discretized_fused, which fetches four more bytes per non-zero. */
hgnn_status hgnn_scale_rows(int64_t n, int32_t F, const hgnn_half* X, int64_t ldx, const float* scale, hgnn_half* out,
                            int64_t ldo, void* stream);

/* ---- the dense side of a layer, on the matrix cores ----------------------------------------------
 * The linear layer's output is the dense input of the sparse kernels (section 3.1.3, Eq. 2); the input
 * width is projected to the intermediate width by a GeMM (section 6).  These calls make a whole layer
 * expressible on this library; they use v_mfma_f32_32x32x16_f16 with fp32 accumulation. */

/* Y[i, f] = fp16( sum_k X[i, k] * W[k, f] )   (trans_w = 0, W is [K][ldw >= F]) or
 *           fp16( sum_k X[i, k] * W[f, k] )   (trans_w != 0, W is [F][ldw >= K]: the product with the
 * transposed weight, which carries the gradient of Y back to X).  X is [n][ldx], Y is [n][ldy]; all
 * device pointers, caller-owned.  Needs K % 8 == 0, ldx % 8 == 0, ldy % 8 == 0 and 16-byte aligned X, Y
 * (HGNN_EUNSUPPORTED otherwise: pad with zeros); F may be any positive number.  W needs no alignment. */
hgnn_status hgnn_linear(int64_t n, int32_t K, int32_t F, const hgnn_half* X, int64_t ldx, const hgnn_half* W, int64_t ldw,
                        int32_t trans_w, hgnn_half* Y, int64_t ldy, void* stream);

/* dW[k, f] = sum_i X[i, k] * dY[i, f], fp32 [K][lddw >= F]: the gradient of the weight of hgnn_linear
 * (trans_w = 0) given the gradient dY of its output.  Partial sums of fixed row sets are written to the
 * workspace and added in a fixed order: no atomics, the same bits on every run.  workspace is device
 * memory of at least hgnn_linear_wgrad_workspace(K, F) bytes (4-byte aligned), owned by the caller and
 * overwritten; the call allocates nothing.  Needs K, F, ldx, ldy % 8 == 0, K, F <= 4096 and 16-byte
 * aligned X, dY. */
size_t hgnn_linear_wgrad_workspace(int32_t K, int32_t F);
hgnn_status hgnn_linear_wgrad(int64_t n, int32_t K, int32_t F, const hgnn_half* X, int64_t ldx, const hgnn_half* dY,
                              int64_t ldy, float* dW, int64_t lddw, void* workspace, size_t workspace_bytes, void* stream);

/* Ties hgnn_gat_backward_fused to the projection of a GAT layer whose row and column side are the same
 * table hfeat [n][ldh] (section 2.1.1: the score is a_l.h_i + a_r.h_j, so its gradient reaches the
 * features through both vectors):
 *   dh[i, h*D+d] = fp16( dV[i, h*D+d] + d_el[i,h] * a_l[h*D+d] + d_er[i,h] * a_r[h*D+d] )   [n][lddh]
 *   da_l[h*D+d]  = sum_i d_el[i,h] * hfeat[i, h*D+d],  da_r likewise with d_er            fp32 [H*D]
 * dV is [n][lddv], d_el / d_er are fp16 [n][H].  The sums over i are formed per workgroup and added in a
 * fixed order through the workspace (at least hgnn_gat_feature_grad_workspace(H, D) bytes of device
 * memory, caller-owned, overwritten).  Needs D % 8 == 0, H*D <= 512, ld % 8 == 0, 16-byte aligned
 * dV, hfeat, dh. */
size_t hgnn_gat_feature_grad_workspace(int32_t H, int32_t D);
hgnn_status hgnn_gat_feature_grad(int64_t n, int32_t H, int32_t D, const hgnn_half* dV, int64_t lddv, const hgnn_half* d_el,
                                  const hgnn_half* d_er, const hgnn_half* a_l, const hgnn_half* a_r, const hgnn_half* hfeat,
                                  int64_t ldh, hgnn_half* dh, int64_t lddh, float* da_l, float* da_r, void* workspace,
                                  size_t workspace_bytes, void* stream);

/* SDDMM over the non-zeros of g (sections 2.1.2, 5.1.3), result in out[k*H + h]:
 *   DOT:        sum_{d<D} U[i, h*D+d] * Vt[col[k], h*D+d],  i = row of k
 *   GAT_SCORE:  s = a_l[h].U[i,h,:] + a_r[h].Vt[col[k],h,:];  s > 0 ? s : neg_slope*s
 * U is [nrows][ldu], Vt is [ncols][ldv], a_l / a_r are [H*D] (GAT_SCORE only).
 * With a plan (p != NULL, the fast path) the kernels walk the plan's segments and
 * take row ids from rowptr; GAT_SCORE then projects every vertex once (fp32
 * scratch in the plan) and adds per edge.  Without a plan the row of a non-zero
 * comes from g->row when given, else from a binary search in rowptr (slow).
 * g->eid must be NULL. */
hgnn_status hgnn_sddmm(const hgnn_csr* g, const hgnn_plan* p, hgnn_sddmm_op op, int32_t H, int32_t D,
                       const hgnn_half* U, int64_t ldu, const hgnn_half* Vt, int64_t ldv, const hgnn_half* a_l,
                       const hgnn_half* a_r, float neg_slope, hgnn_half* out, void* stream);

/* One GAT aggregation in a single pass over the graph (score, edge softmax of Eq. 1 and the
 * weighted sum of section 2.1.1 fused; no |E| x H tensor is written):
 *   e_k = LeakyReLU(a_l[h].U[i,h] + a_r[h].Vt[col k,h]),  alpha = softmax over row i,
 *   out[i, h*D+d] = sum_k alpha_k * Vt[col k, h*D+d],      lse[i,h] = log sum_k exp(e_k).
 * U [nrows][ldu] is the row side, Vt [ncols][ldv] the column side (the same table for a GAT
 * layer), a_l / a_r are [H*D], out is [nrows][ldo], lse is fp32 [nrows][H] or NULL.  Empty
 * rows give out = 0, lse = 0.  Walks the plan's segments (and column blocks); partial
 * results of a row are merged by rescaling to the larger maximum, pieces that cross a segment
 * border are staged as normalised fp16 vectors plus fp32 (max, sum) and merged by a follow-up
 * kernel: no atomics, deterministic.  Needs a plan with max_H >= H and max_F >= H*D,
 * D = 8 * 2^k, H*D <= 512, ld % 8 == 0 and 16-byte aligned tensors; g without edge-id map.
 * Overwrites the plan's per-vertex scratch (as hgnn_sddmm GAT_SCORE does). */
hgnn_status hgnn_gat_forward_fused(const hgnn_csr* g, const hgnn_plan* p, int32_t H, int32_t D, const hgnn_half* U,
                                   int64_t ldu, const hgnn_half* Vt, int64_t ldv, const hgnn_half* a_l,
                                   const hgnn_half* a_r, float neg_slope, hgnn_half* out, int64_t ldo, float* lse,
                                   void* stream);

/* Backward of hgnn_gat_forward_fused without per-edge tensors.  Given the forward inputs, the
 * forward result out, its lse, and dOut (the gradient of out), with
 *   alpha_ij = exp(e_ij - lse_i),  dalpha_ij = <dOut[i,h], Vt[j,h]>,  t_i = <dOut[i,h], out[i,h]>,
 *   ds_ij = alpha_ij * (dalpha_ij - t_i) * (score_ij > 0 ? 1 : neg_slope)      (Eq. 1 differentiated)
 * it writes  dV[j, h*D+d] = sum_i alpha_ij * dOut[i, h*D+d]   (fp16 [ncols][lddv], the gradient
 * through the aggregated values), d_el[i,h] = sum_j ds_ij (fp16 [nrows][H]) and
 * d_er[j,h] = sum_i ds_ij (fp16 [ncols][H]); the gradients of the features through the scores
 * are the dense products d_el * a_l and d_er * a_r, outside this call.  Two passes: over gt with
 * plan pt (gathers dOut rows: dV and d_er) and over g with plan p (gathers Vt rows: d_el).
 * gt must be the transpose of g (hgnn_transpose; its edge-id map is not used).  Same shape
 * requirements as the forward call, for both plans.  Overwrites the per-vertex scratch of p. */
hgnn_status hgnn_gat_backward_fused(const hgnn_csr* g, const hgnn_plan* p, const hgnn_csr* gt, const hgnn_plan* pt,
                                    int32_t H, int32_t D, const hgnn_half* U, int64_t ldu, const hgnn_half* Vt,
                                    int64_t ldv, const hgnn_half* a_l, const hgnn_half* a_r, float neg_slope,
                                    const hgnn_half* out, int64_t ldo, const float* lse, const hgnn_half* dOut,
                                    int64_t lddo, hgnn_half* dV, int64_t lddv, hgnn_half* d_el, hgnn_half* d_er,
                                    void* stream);

/* hgnn_gat_forward_fused that also keeps what lets the backward pass skip its pass over g.  With
 * mu_k = 1 where the score s_k > 0 and neg_slope elsewhere (the LeakyReLU derivative),
 *   out_masked[i, h*D+d] = sum_k alpha_k * mu_k * Vt[col k, h*D+d]   (fp16 [nrows][ldom]),
 *   csum[i,h]            = sum_k alpha_k * mu_k                      (fp32 [nrows][H]);
 * then sum_k ds_ik = <dOut[i,h], out_masked[i,h]> - <dOut[i,h], out[i,h]> * csum[i,h] (Eq. 1
 * differentiated, summed over the row).  Both ride on the rows the pass gathers anyway: a second
 * accumulator per lane, no further memory traffic but the two outputs.  lse, out_masked and csum are
 * required; neg_slope >= 0; ldom % 8 == 0 and out_masked 16-byte aligned; otherwise as
 * hgnn_gat_forward_fused. */
hgnn_status hgnn_gat_forward_fused_save(const hgnn_csr* g, const hgnn_plan* p, int32_t H, int32_t D, const hgnn_half* U,
                                        int64_t ldu, const hgnn_half* Vt, int64_t ldv, const hgnn_half* a_l,
                                        const hgnn_half* a_r, float neg_slope, hgnn_half* out, int64_t ldo, float* lse,
                                        hgnn_half* out_masked, int64_t ldom, float* csum, void* stream);

/* hgnn_gat_backward_fused given out_masked and csum of hgnn_gat_forward_fused_save: d_el is formed per
 * vertex from them and only the pass over gt runs (dV and d_er).  Same outputs, same requirements; g and
 * p are still needed for sizes and the per-vertex scratch. */
hgnn_status hgnn_gat_backward_fused_saved(const hgnn_csr* g, const hgnn_plan* p, const hgnn_csr* gt, const hgnn_plan* pt,
                                          int32_t H, int32_t D, const hgnn_half* U, int64_t ldu, const hgnn_half* Vt,
                                          int64_t ldv, const hgnn_half* a_l, const hgnn_half* a_r, float neg_slope,
                                          const hgnn_half* out, int64_t ldo, const float* lse, const hgnn_half* out_masked,
                                          int64_t ldom, const float* csum, const hgnn_half* dOut, int64_t lddo,
                                          hgnn_half* dV, int64_t lddv, hgnn_half* d_el, hgnn_half* d_er, void* stream);

/* Rebuilds alpha[k,h] = exp(e_k - lse[i,h]) (fp16 [nnz][H]) from the lse of
 * hgnn_gat_forward_fused, for a backward pass that wants the attention weights as a tensor.
 * Same requirements as above. */
hgnn_status hgnn_gat_alpha(const hgnn_csr* g, const hgnn_plan* p, int32_t H, int32_t D, const hgnn_half* U, int64_t ldu,
                           const hgnn_half* Vt, int64_t ldv, const hgnn_half* a_l, const hgnn_half* a_r, float neg_slope,
                           const float* lse, hgnn_half* alpha, void* stream);

/* Edge softmax, Eq. 1, over every row (neighbourhood) and head:
 *   m_i = max_k e[k,h];  alpha[k,h] = exp(e[k,h]-m_i) / sum_k exp(e[k,h]-m_i).
 * exp and the sums are fp32 in registers (the argument is <= 0, so the value is in
 * (0,1], section 3.1.2).  e and alpha are [nnz][H]; empty rows write nothing.
 * p may be NULL (then very long rows are slower; the same when H exceeds the plan's max_H, because
 * the plan holds the partial results of its long rows' chunks for max_H heads).  With a plan the call
 * writes that scratch: order it with the other calls on the plan.  g->eid must be NULL. */
hgnn_status hgnn_edge_softmax(const hgnn_csr* g, const hgnn_plan* p, int32_t H, const hgnn_half* e, hgnn_half* alpha,
                              void* stream);

/* Backward of Eq. 1:  t_i = sum_k alpha[k,h] dalpha[k,h];  de[k,h] = alpha (dalpha - t_i).
 * With e != NULL the LeakyReLU of the GAT score is undone as well:
 *   de[k,h] *= (e[k,h] > 0 ? 1 : neg_slope). */
hgnn_status hgnn_edge_softmax_bwd(const hgnn_csr* g, const hgnn_plan* p, int32_t H, const hgnn_half* alpha,
                                  const hgnn_half* dalpha, const hgnn_half* e, float neg_slope, hgnn_half* de,
                                  void* stream);

/* Row sums of an edge tensor: out[i,h] = sum_{k in row i} t[slot(k), h], out is
 * [nrows][H] fp16.  On g it gives d(e_l); on the transposed graph (with its eid
 * map) it gives the column sums d(e_r) of the GAT score backward.  p may be NULL
 * (then very long rows are slower); when given it must be the plan of g. */
hgnn_status hgnn_edge_rowsum(const hgnn_csr* g, const hgnn_plan* p, int32_t H, const hgnn_half* t, hgnn_half* out,
                             void* stream);

/* Column sums of an edge tensor over the graph itself: out[j] = sum_{k: col[k] = j} t[k], t fp16 [nnz] (one head),
 * out fp16 [ncols]; the same values as hgnn_edge_rowsum on the transposed graph with its edge-id map (d(e_r) of the
 * GAT score backward), without a transposed graph and without a gather through that map.  Needs column slices in
 * the plan (hgnn_plan_add_slices, HGNN_EINVAL otherwise) and g without an edge-id map.  The sums are formed exactly
 * (64-bit fixed point, integer adds in LDS and per row chunk) and rounded once, so the result does not depend on the
 * order of the additions.  Writes the plan's partial sums: order it with the other calls on the plan. */
hgnn_status hgnn_edge_colsum(const hgnn_csr* g, const hgnn_plan* p, int32_t H, const hgnn_half* t, hgnn_half* out,
                             void* stream);

#ifdef __cplusplus
}
#endif
#endif /* HGNN_H */
