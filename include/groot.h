/*
 * groot.h -- C ABI of libgroot: the degree-split sparse aggregation Y = A_hat * X
 * of GROOT (arXiv 2511.18297) for AMD MI355X (gfx950).
 *
 * The library covers the GPU hot path of the paper's GNN verification flow:
 * the EDA-graph adjacency built from an And-Inverter Graph, the split of its
 * rows into a high-degree and a low-degree class, the two kernels that
 * multiply the adjacency with the node-feature matrix, and the partition of a
 * large graph into sub-graphs whose boundary edges are re-grown.
 *
 * Conventions
 *   - Every call returns a groot_status and never throws or aborts; on failure
 *     *out is left untouched and groot_last_error() describes the reason.
 *   - "host" pointers are ordinary CPU memory, "device" pointers are HIP device
 *     memory of the current device (e.g. torch.Tensor.data_ptr()).
 *   - Input arrays are copied; the caller keeps ownership of everything it
 *     passes in.  Objects returned through **out are owned by the caller and
 *     released with the matching *_free (NULL is accepted).  Pointers returned
 *     by the *_view calls are borrowed and live as long as the viewed object.
 *   - Node ids and columns are int32 (N < 2^31), row pointers are int64.
 *   - No global state except a thread-local error string, the tuning table of
 *     groot_set_tuning() (atomic integers, each read at the call its
 *     description names) and the fixed scratch array of
 *     groot_plan_lists_device_static().
 */
#ifndef GROOT_H
#define GROOT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    GROOT_OK     = 0,
    GROOT_EINVAL = 1,   /* bad argument (NULL, misaligned, out of range, not topological, ...) */
    GROOT_ENOMEM = 2,   /* host or device allocation failed */
    GROOT_EHIP   = 3,   /* a HIP runtime call or kernel launch failed */
    GROOT_ERANGE = 4    /* the graph does not fit the index types (N >= 2^31) */
} groot_status;

typedef struct groot_graph groot_graph;
typedef struct groot_plan  groot_plan;
typedef struct groot_parts groot_parts;
typedef struct groot_dev_part groot_dev_part;

/* flags of groot_graph_build */
#define GROOT_SYMMETRIC  1u   /* store both directions of every AIG edge */
#define GROOT_SELF_LOOPS 2u   /* add (v,v) for every node */
#define GROOT_NORM_MEAN  4u   /* weight 1/(stored row length); otherwise 1 */
/* flags of groot_partition_regrow */
#define GROOT_REGROW     1u   /* add boundary nodes and crossing edges (0: plain induced sub-graphs) */
/* phases of groot_spmm_execute_phases: one kernel launch each */
#define GROOT_PHASE_LD     1u
#define GROOT_PHASE_HD     2u
#define GROOT_PHASE_FINISH 4u
#define GROOT_PHASE_ALL    7u

/* ---------------------------------------------------------------------------
 * groot_graph_build -- EDA graph of an And-Inverter Graph.
 * Paper: Section "Converting Netlists into Transitional Graph" (AIG: two-input
 * AND nodes, inverted edges, primary inputs/outputs) and Section "Node Features
 * and Node Label creation" (G=(V,E), adjacency A, degree D_ii = sum_j A_ij);
 * the weights are those of GraphSAGE mean aggregation, A_hat = D^-1 A.
 *
 * n1, type, fanin0, fanin1 (host): one copy of the AIG, nodes in topological
 *   order.  type[v]: 0 = primary input, 1 = AND, 2 = primary output.  A fanin
 *   literal is 2*source + inverted; a PI holds -1,-1; a PO holds its driver
 *   literal in both slots.
 * batch: number of disjoint copies laid out block-diagonally (copy c shifts
 *   all ids by c*n1), as in the paper's batch-16 workload.
 * flags: GROOT_SYMMETRIC | GROOT_SELF_LOOPS | GROOT_NORM_MEAN in any mix.
 * Result: CSR with strictly ascending columns per row, duplicate edges merged,
 *   val = 1.0f/(float)row_length (correctly rounded) or 1, and one polarity
 *   byte per entry (bit0 the edge is inverted, bit1 the column drives the row,
 *   bit2 self-loop).
 * Errors: EINVAL for NULL arrays, n1 < 1, batch < 1, unknown flag bits, a bad
 *   type, a literal that is negative / not smaller than 2*v, a PI with fanins,
 *   a PO whose two slots differ; ERANGE if n1*batch >= 2^31; ENOMEM.
 * ------------------------------------------------------------------------- */
groot_status groot_graph_build(int64_t n1, const uint8_t *type, const int32_t *fanin0,
                               const int32_t *fanin1, int32_t batch, uint32_t flags,
                               groot_graph **out);

/* A graph from caller-supplied CSR arrays (host; copied).  Columns of a row
 * must be strictly ascending and inside [0,n).  Weights are kept as given. */
groot_status groot_graph_from_csr(int64_t n, const int64_t *rowptr, const int32_t *col,
                                  const float *val, groot_graph **out);

/* groot_graph_transpose -- the graph of A_hat^T (host; a new graph owned by the
 * caller).  The backward pass of a GNN layer multiplies by the transpose of the
 * forward aggregation (the paper motivates its kernels by training time,
 * Section "Accuracy and Accuracy Recovery of Various Multipliers"): plan and
 * execute on the transposed graph give dX = A_hat^T dY with the same kernels.
 * Entry (j,i) carries the weight of (i,j) as an explicit weight; rows list
 * their columns ascending; no polarity bytes; the copy size of a batched
 * graph is kept.  Errors: EINVAL (NULL), ENOMEM. */
groot_status groot_graph_transpose(const groot_graph *g, groot_graph **out);

/* Borrowed host pointers to the CSR; any output pointer may be NULL.  *pol is
 * set to NULL for graphs that did not come from an AIG. */
groot_status groot_graph_view(const groot_graph *g, int64_t *n, int64_t *nnz,
                              const int64_t **rowptr, const int32_t **col, const float **val,
                              const uint8_t **pol);
void groot_graph_free(groot_graph *g);

/* ---------------------------------------------------------------------------
 * groot_spmm_plan -- degree classes and row lists.
 * Paper: Section "Kernel Design - GROOT-GPU": rows are served by an HD kernel
 * or an LD kernel according to their degree; the LD side computes every row's
 * degree from the row pointer and stably sorts rows by degree (count sort).
 * One threshold: a row is high-degree iff its stored length >= degree_threshold.
 * Host only; the graph must outlive the plan.
 *   row_class[i]        1 = HD, 0 = LD
 *   hd_rows, ld_rows    ids of each class, ascending
 *   ld_rows_by_degree   LD ids by ascending degree, ties by ascending id
 *   ld_deg_offsets[d]   number of LD rows with degree < d, d = 0..threshold
 * Errors: EINVAL for NULL, degree_threshold < 1; ENOMEM.
 * ------------------------------------------------------------------------- */
groot_status groot_spmm_plan(const groot_graph *g, int32_t degree_threshold, groot_plan **out);
groot_status groot_plan_view(const groot_plan *plan, int64_t *n_hd, int64_t *n_ld,
                             const uint8_t **row_class, const int32_t **hd_rows,
                             const int32_t **ld_rows, const int32_t **ld_rows_by_degree,
                             const int64_t **ld_deg_offsets);

/* Copies the CSR and the kernel schedule of the plan to the current HIP
 * device (allocates device memory owned by the plan; synchronous).  Must be
 * called once before groot_spmm_execute; max_F (multiple of 4 in [4,512]) is
 * the widest feature matrix the plan will be executed with and sizes the
 * scratch for split high-degree rows.  Calling it again re-uploads.
 * For a graph from groot_graph_from_csr it also looks (one pass over the weights)
 * whether they are bit for bit fl(1 / row length), or all 1; then the kernels
 * recompute them from the row pointer like for a graph built from an AIG and do
 * not read the weight array (results agree with the entry-by-entry form within
 * rounding: the row sum is scaled once instead of every term).
 * Errors: EINVAL, EHIP, ENOMEM. */
groot_status groot_plan_upload(groot_plan *plan, int32_t max_F);

/* ---------------------------------------------------------------------------
 * groot_spmm_execute -- Y = A_hat * X with the HD and LD kernels.
 * Paper: Section "Kernel Design - GROOT-GPU" (HD kernel: the non-zeros of a
 * high-degree row are split statically over many wavefronts and reduced; LD
 * kernel: many short rows per wavefront, results of consecutive rows written
 * to one contiguous area).
 * X_dev, Y_dev (device): row-major [N,F] fp32, 16-byte aligned, not
 *   overlapping.  F: multiple of 4, 4 <= F <= 512.  Y is overwritten entirely;
 *   empty rows give 0.  Accumulation is fp32.
 * hip_stream: a hipStream_t (NULL = default stream).  The call only enqueues
 *   kernels: it never synchronises, allocates or clears memory, so it may be
 *   recorded into a HIP graph by stream capture and replayed.  At most one execute per plan may be in
 *   flight at a time (the plan owns the scratch for split rows).
 * Errors: EINVAL (NULL, alignment, F, plan not uploaded), EHIP (launch failed).
 * groot_spmm_execute_phases runs a subset of the kernels (bit-or of
 * GROOT_PHASE_*), for per-kernel timing.
 * ------------------------------------------------------------------------- */
groot_status groot_spmm_execute(const groot_plan *plan, const float *X_dev, float *Y_dev,
                                int32_t F, void *hip_stream);
groot_status groot_spmm_execute_phases(const groot_plan *plan, const float *X_dev, float *Y_dev,
                                       int32_t F, uint32_t phases, void *hip_stream);
/* ---------------------------------------------------------------------------
 * groot_spmm_execute_rows -- the same product restricted to the first n_rows
 * rows, each written where the caller wants it:
 *     Y[out_ids[r], :] = (A_hat X)[r, :]      r < n_rows      (out_ids NULL: Y[r, :])
 * Paper: Section "GNN and Edge Re-growth After Partition", Algorithm 1: on a
 * re-grown sub-graph only the rows of S_p are results (local ids 0..n_owned-1,
 * the boundary rows behind them are computed only to be dropped), and they
 * belong at their global positions.  With n_rows = n_owned and out_ids = the
 * first n_owned entries of the part's global_id this writes the part's result
 * straight into the full Y: no boundary rows are computed, no copy of Y_p, no
 * scatter pass.
 * out_ids_dev (device, int64[n_rows], may be NULL): distinct row numbers of Y;
 * the caller guarantees that Y has those rows and does not overlap X (neither
 * can be checked here).  Other rows of Y are not touched.  Stream, scratch
 * and error behaviour as groot_spmm_execute; n_rows outside [0, N] is EINVAL.
 * ------------------------------------------------------------------------- */
groot_status groot_spmm_execute_rows(const groot_plan *plan, const float *X_dev, float *Y_dev,
                                     int32_t F, int64_t n_rows, const int64_t *out_ids_dev,
                                     void *hip_stream);
/* ---------------------------------------------------------------------------
 * groot_plan_use_global_columns -- lets the plan of a part's sub-graph read the
 * feature matrix of the WHOLE graph in place.
 * Paper: Section "GNN and Edge Re-growth After Partition", Algorithm 1: the
 * sub-graph (S_p+, E_p+) names its nodes by local ids, and global_id maps them
 * back.  When the whole feature matrix is resident on the device anyway, there
 * is no need to copy the rows of S_p+ into a compact matrix first: this call
 * rewrites the plan's resident column indices once, col <- global_id[col], and
 * from then on X_dev of groot_spmm_execute / groot_spmm_execute_rows is the
 * whole graph's matrix ([n_global, F]); rows (and Y without out_ids) stay
 * local.  With out_ids = global_id a partitioned pass is then one
 * groot_spmm_execute_rows per part and nothing else.  (The compact form remains
 * the one to use when only one part's features fit on the device.)
 * plan: resident; global_id_dev (device, int64 [rows of the plan]): the part's
 * global_id, every entry in [0, n_global) (not checked); n_global < 2^31.
 * Enqueues one kernel on hip_stream; the plan's next execute must be ordered
 * after it (same stream, or synchronise).  Afterwards groot_sage_layer_forward
 * and groot_partition_regrow_device refuse the plan, and a second call is
 * EINVAL.  Errors: EINVAL, ERANGE (n_global >= 2^31), EHIP.
 * ------------------------------------------------------------------------- */
groot_status groot_plan_use_global_columns(groot_plan *plan, const int64_t *global_id_dev,
                                           int64_t n_global, void *hip_stream);

/* ---------------------------------------------------------------------------
 * groot_sage_layer_forward -- one GraphSAGE-mean layer with the aggregation fused in:
 *     H = act( (A_hat X) Wn + X Ws + b ),   act = ReLU if relu != 0, identity otherwise.
 * Paper: Section "GNN and Edge Re-growth After Partition" (the GraphSAGE layer takes
 * the graph with node features and aggregates them; the aggregation is the product
 * the paper's kernels compute).  The aggregated rows stay on chip and feed the dense
 * products on the matrix cores, so A_hat X is neither written nor re-read.
 * X_dev (device): row-major [N,F_in] fp32; H_dev (device): row-major [N,F_out] fp32;
 * both 16-byte aligned, not overlapping.
 * Wn_dev, Ws_dev (device): row-major [F_in,F_out] fp32 (input feature major: H = X W);
 * bias_dev: [F_out] fp32 or NULL.
 * groot_sage_layer_forward_io: F_in = 32 or 64, F_out = 16, 32 or 64 for graphs with
 * row-uniform weights (every graph built from an AIG: a classifier that narrows or
 * widens from layer to layer; pad a narrower input or a class count with zero
 * columns / zero weights up to the next supported width); graphs with explicit
 * weights: 64 -> 64 only.  groot_sage_layer_forward is the same call with
 * F_in = F_out = F (64 or 32).  fp32 in and out,
 * fp32 sums; a dense product is formed on the matrix cores from three bf16 pieces per
 * fp32 operand (six piece products, fp32 accumulation), which keeps the relative error
 * of a product below 2^-23, as an fp32 multiplication does (the pieces have the
 * exponent range of fp32; an input above 3.38e38 in magnitude rounds to infinity in
 * its first piece and gives NaN).
 * The plan must be uploaded with max_F >= F_in.  Only enqueues on hip_stream; one
 * call per plan in flight (the aggregated high-degree rows pass through a buffer of
 * the plan).  Errors: EINVAL (NULL, alignment, unsupported widths, plan not
 * uploaded), EHIP.
 * ------------------------------------------------------------------------- */
groot_status groot_sage_layer_forward(const groot_plan *plan, const float *X_dev, const float *Wn_dev,
                                      const float *Ws_dev, const float *bias_dev, int32_t relu,
                                      float *H_dev, int32_t F, void *hip_stream);
groot_status groot_sage_layer_forward_io(const groot_plan *plan, const float *X_dev, const float *Wn_dev,
                                         const float *Ws_dev, const float *bias_dev, int32_t relu,
                                         float *H_dev, int32_t F_in, int32_t F_out, void *hip_stream);

/* ---------------------------------------------------------------------------
 * groot_sage_layer_backward_data -- the fused layer's gradient with respect to
 * its input, for training (Section "GNN and Edge Re-growth After Partition":
 * the GraphSAGE model is trained on small multipliers).  With Z = (A_hat X) Wn
 * + X Ws + b the layer's pre-activation output and dZ the gradient of the loss
 * at Z (the caller has already applied the activation's derivative),
 *     dX = A_hat^T (dZ Wn^T) + dZ Ws^T = (A_hat^T dZ) Wn^T + dZ Ws^T.
 * For a graph built symmetric with mean weights (groot_graph_build's default
 * flags) A_hat^T = A D^-1, so the aggregation is the unit-weight sum of the
 * rows of dZ / deg, and the call runs the forward layer's kernel on that
 * matrix with the row's own operand scaled back by its stored length: one
 * pass over dZ, no transposed graph, no N x F intermediate.
 * dZ_over_deg_dev (device): row-major [N, F_out] fp32, row i of dZ divided by
 * the stored length of row i (do it in the kernel that applies the
 * activation's derivative, or with groot_rows_over_degree);
 * WnT_dev, WsT_dev (device): the forward layer's weights transposed, row-major
 * [F_out, F_in] fp32; dX_dev (device): row-major [N, F_in] fp32, fully
 * overwritten, not overlapping dZ_over_deg_dev.  F_out = 32 or 64 (the width
 * of dZ), F_in = 16, 32 or 64.  Accuracy, the "sage_pieces" knob, the plan's
 * side buffer (one call per plan in flight) and the stream: as for
 * groot_sage_layer_forward.  The gradients of the weights (X^T and (A_hat X)^T
 * times dZ): groot_sage_layer_backward_weights below.
 * Errors: EINVAL (NULL, alignment, widths, plan not uploaded or made on the
 * device, graph not built symmetric with mean weights, overlap), EHIP.
 *
 * groot_rows_over_degree: out[i, :] = Z[i, :] / stored length of row i (rows
 * of length 0 give 0), F a multiple of 4 in [4, 512], out_dev may be Z_dev.
 * Only enqueues.  Errors: EINVAL, EHIP.
 * ------------------------------------------------------------------------- */
groot_status groot_sage_layer_backward_data(const groot_plan *plan, const float *dZ_over_deg_dev,
                                            const float *WnT_dev, const float *WsT_dev, float *dX_dev,
                                            int32_t F_out, int32_t F_in, void *hip_stream);
groot_status groot_rows_over_degree(const groot_plan *plan, const float *Z_dev, float *out_dev, int32_t F,
                                    void *hip_stream);

/* ---------------------------------------------------------------------------
 * groot_sage_layer_backward_weights -- the fused layer's gradients with respect
 * to its two weight matrices, for training (Section "GNN and Edge Re-growth
 * After Partition").  With Z = (A_hat X) Wn + X Ws + b and dZ the gradient of
 * the loss at Z,
 *     dWn = (A_hat X)^T dZ,   dWs = X^T dZ,
 * both in one pass over X and dZ with the aggregation kept on chip (A_hat X is
 * never written to memory); fp32 accuracy per product from bf16 piece products
 * as in the forward layer ("sage_pieces"), fp32 sums over the rows that one
 * wavefront sweeps (N / 1024 of them on an MI355X), fp64 across wavefronts, in
 * a fixed order: the same bits on every run.  The bias gradient is the column
 * sum of dZ and is left to the caller.
 * X_dev (device): row-major [N, F_in] fp32, F_in = 32 or 64; dZ_dev (device):
 * row-major [N, F_out] fp32, F_out = 16, 32 or 64 (other widths: pad with zero
 * columns); dWn_dev, dWs_dev (device): row-major [F_in, F_out] fp32, fully
 * overwritten; workspace_dev (device, 16-byte aligned): at least the number of
 * bytes that groot_sage_layer_backward_weights_workspace reports for these
 * widths (2 F_in F_out floats per wavefront of the launch: 32 MiB at 64 x 64
 * on an MI355X), contents overwritten, owned by the caller.  The plan must be
 * uploaded with max_F >= F_in and have row-uniform weights.  Only enqueues on
 * hip_stream, allocates nothing; one call per plan in flight (the aggregated
 * high-degree rows pass through a buffer of the plan).  Errors: EINVAL (NULL,
 * alignment, widths, plan not uploaded, explicit weights, workspace too
 * small), EHIP.
 * ------------------------------------------------------------------------- */
groot_status groot_sage_layer_backward_weights_workspace(const groot_plan *plan, int32_t F_in, int32_t F_out,
                                                         size_t *bytes);
groot_status groot_sage_layer_backward_weights(const groot_plan *plan, const float *X_dev, const float *dZ_dev,
                                               float *dWn_dev, float *dWs_dev, int32_t F_in, int32_t F_out,
                                               void *workspace_dev, size_t workspace_bytes, void *hip_stream);
void groot_plan_free(groot_plan *plan);

/* ---------------------------------------------------------------------------
 * groot_plan_lists_device -- the lists of groot_spmm_plan computed on the GPU.
 * Paper: Section "Kernel Design - GROOT-GPU", LD kernel: every row's degree is
 * taken from the row pointer and the rows are sorted by degree with a stable
 * count sort, which is linear in the number of rows.  Here that runs on the
 * device from the plan's uploaded row pointer (per-block degree histograms, a
 * prefix over blocks, ballot ranks inside a wavefront), for graphs whose CSR
 * lives on the device and changes between runs.
 * All outputs are device pointers owned by the caller:
 *   row_class_dev          uint8  [N]     1 = HD, 0 = LD
 *   hd_rows_dev            int32  [N]     first n_hd entries written
 *   ld_rows_dev            int32  [N]     first n_ld entries written
 *   ld_rows_by_degree_dev  int32  [N]     first n_ld entries written
 *   ld_deg_offsets_dev     int64  [T+1]   T = the plan's degree threshold
 *   counts_dev             int64  [2]     {n_hd, n_ld}
 * The written entries are bit-identical to groot_plan_view's arrays.
 * Allocates and frees its own scratch (4 (T+2) bytes per 4096 rows) and
 * synchronises hip_stream before it returns.
 * Errors: EINVAL (NULL, plan not uploaded), ERANGE (threshold > 1024), ENOMEM,
 * EHIP.
 * ------------------------------------------------------------------------- */
groot_status groot_plan_lists_device(const groot_plan *plan, uint8_t *row_class_dev,
                                     int32_t *hd_rows_dev, int32_t *ld_rows_dev,
                                     int32_t *ld_rows_by_degree_dev, int64_t *ld_deg_offsets_dev,
                                     int64_t *counts_dev, void *hip_stream);

/* ---------------------------------------------------------------------------
 * groot_plan_lists_device_static -- groot_plan_lists_device for callers that
 * cannot allocate device memory or synchronise: code under HIP graph capture,
 * tight serving loops that rebuild the lists of a changing graph every step,
 * harnesses that forbid hipMalloc.  Same arguments, same kernels and bit for
 * bit the same outputs; the per-block degree table lives in a fixed 8 MiB
 * array inside the library (one copy per GPU, held until the process ends)
 * instead of allocated scratch, so the call only enqueues four kernels on
 * hip_stream: no hipMalloc, no hipFree, no synchronisation, no memset (the
 * kernels write every scratch byte they later read).
 * Limit: 256-byte-rounded 8 (T+2) + 4 (T+2) ceil(N / 4096) bytes must fit
 * 8 MiB (T = the plan's degree threshold), e.g. 134 M rows up to T = 62,
 * 16.7 M rows up to T = 509; beyond that the call fails with ERANGE and leaves
 * the outputs untouched.
 * All calls on one GPU share that array: two calls whose kernels can overlap
 * on the same GPU (different streams, or the same plan from two threads) race
 * and give wrong lists; calls on one stream are ordered and safe.
 * Errors: EINVAL (NULL, plan not uploaded), ERANGE (threshold > 1024, scratch
 * limit), EHIP.
 * ------------------------------------------------------------------------- */
groot_status groot_plan_lists_device_static(const groot_plan *plan, uint8_t *row_class_dev,
                                            int32_t *hd_rows_dev, int32_t *ld_rows_dev,
                                            int32_t *ld_rows_by_degree_dev,
                                            int64_t *ld_deg_offsets_dev, int64_t *counts_dev,
                                            void *hip_stream);

/* ---------------------------------------------------------------------------
 * groot_partition_regrow -- partition into sub-graphs with re-grown boundary.
 * Paper: Section "GNN and Edge Re-growth After Partition", Eq. (1), Eq. (2)
 * and Algorithm 1.  For every part p with node set S_p:
 *   B_p  = (union of one-hop neighbours of S_p) \ S_p          boundary nodes
 *   C_p  = edges with one end in S_p and the other in B_p      crossing edges
 *   S_p+ = S_p u B_p,   E_p+ = E[S_p] u C_p
 * E is the stored pattern of g; the neighbours of a node are the other columns
 * of its row.  Edges between two boundary nodes are not part of E_p+; a stored
 * self-loop of a boundary node is kept.  Local ids: S_p ascending, then B_p
 * ascending (global_id lists them).  Sub-graph weights: 1/(local row length)
 * for mean-normalised graphs, 1 for unit-weight graphs, the original entry's
 * weight for graphs from groot_graph_from_csr.  Rows of S_p keep their whole
 * neighbourhood, so one aggregation on the sub-graph reproduces the full-graph
 * result on them; rows of B_p are computed and dropped.
 * num_parts: P >= 1.  part_of (host, may be NULL): part of every node in
 *   [0,P); NULL selects the built-in rule, the p-th contiguous slice of every
 *   copy: min(P-1, floor((v mod n1) * P / n1)).
 * flags: GROOT_REGROW, or 0 for induced sub-graphs without boundary.
 * n_crossing counts unordered pairs {i,j}, i in S_p, j in B_p.
 * Errors: EINVAL (NULL, P < 1, P > N, part_of out of range, unknown flags);
 *   ENOMEM.
 * ------------------------------------------------------------------------- */
groot_status groot_partition_regrow(const groot_graph *g, int32_t num_parts,
                                    const int32_t *part_of, uint32_t flags, groot_parts **out);
groot_status groot_parts_view(const groot_parts *parts, int32_t p, int64_t *n_owned,
                              int64_t *n_halo, int64_t *n_crossing, const int64_t **global_id,
                              const groot_graph **sub);
int32_t groot_parts_count(const groot_parts *parts);
void groot_parts_free(groot_parts *parts);

/* ---------------------------------------------------------------------------
 * groot_partition_regrow_device -- one part of the same partition, built on
 * the device from the CSR that an uploaded plan keeps there.
 * Paper: Section "GNN and Edge Re-growth After Partition", Eq. (1), Eq. (2)
 * and Algorithm 1; definitions, local numbering, kept edges, weights and
 * n_crossing exactly as in groot_partition_regrow, and the arrays are
 * bit-identical to that call's part p.
 * plan: resident (groot_plan_upload, or a plan made by groot_dev_part_plan).
 * part_of_dev (device, int32 [N], may be NULL): part of every node; NULL
 *   selects the built-in rule of groot_partition_regrow (nodes per copy are
 *   those of the plan's graph; a plan made by groot_dev_part_plan counts as
 *   one copy).
 * p: the part to build, in [0, num_parts).
 * The result owns its device arrays (groot_dev_part_view; layout of the
 * sub-graph: rowptr int64 [n_owned + n_halo + 1], col int32 [nnz] local ids,
 * val float [nnz] or NULL when the graph's weights are row-uniform,
 * global_id int64 [n_owned + n_halo]).  Allocates device memory (4 bytes per
 * node of the whole graph as scratch, freed before it returns) and
 * synchronises hip_stream.
 * Errors: EINVAL (NULL, plan not resident, P < 1, P > N, p or a part_of entry
 *   outside [0,P), unknown flags); ENOMEM (host or device); EHIP.
 *
 * groot_dev_part_plan -- an executable plan for the part's sub-graph, built
 * from the device arrays (degree classes and counting sort as in
 * groot_plan_lists_device; the schedule of the high-degree rows is made on
 * the host from those rows' extents only).  The sub-graph's arrays MOVE into
 * the plan: afterwards groot_dev_part_view gives NULL for rowptr/col/val, the
 * part keeps its counts and global_id, and a second call gives EINVAL.  The
 * plan is resident (groot_plan_upload on it is a no-op for max_F' <= max_F and
 * EINVAL above), has no host lists (groot_plan_view gives EINVAL; use
 * groot_plan_lists_device), and is freed with groot_plan_free.
 * Errors: EINVAL, ERANGE (degree_threshold > 1024), ENOMEM, EHIP.
 *
 * groot_dev_part_download -- copies of the part's arrays in host buffers of
 * the caller (sizes as above; any pointer may be NULL = not wanted);
 * synchronises hip_stream.  EINVAL for rowptr/col/val once they have moved
 * into a plan, and for val when the sub-graph has no weight array.
 * ------------------------------------------------------------------------- */
groot_status groot_partition_regrow_device(const groot_plan *plan, int32_t num_parts,
                                           const int32_t *part_of_dev, uint32_t flags, int32_t p,
                                           void *hip_stream, groot_dev_part **out);
groot_status groot_dev_part_view(const groot_dev_part *part, int64_t *n_owned, int64_t *n_halo,
                                 int64_t *n_crossing, int64_t *nnz, const int64_t **global_id_dev,
                                 const int64_t **rowptr_dev, const int32_t **col_dev,
                                 const float **val_dev);
groot_status groot_dev_part_plan(groot_dev_part *part, int32_t degree_threshold, int32_t max_F,
                                 void *hip_stream, groot_plan **out);
groot_status groot_dev_part_download(const groot_dev_part *part, int64_t *global_id_host,
                                     int64_t *rowptr_host, int32_t *col_host, float *val_host,
                                     void *hip_stream);
void groot_dev_part_free(groot_dev_part *part);

/* Row gather / scatter for the partitioned mode (device pointers; ids int64):
 *   gather : out[i,:]     = X[ids[i],:]      i < n
 *   scatter: Y[ids[i],:]  = in[i,:]          i < n   (ids distinct)
 * F as in groot_spmm_execute.  Only enqueues on hip_stream. */
groot_status groot_rows_gather(const int64_t *ids_dev, int64_t n, const float *X_dev,
                               float *out_dev, int32_t F, void *hip_stream);
groot_status groot_rows_scatter(const int64_t *ids_dev, int64_t n, const float *in_dev,
                                float *Y_dev, int32_t F, void *hip_stream);

/* ---------------------------------------------------------------------------
 * groot_feature_placement -- where in an arena of device memory X and Y should
 * lie.  Not in the paper: a property of this machine.  The same kernels on the
 * same data take up to 10 % longer when the two feature matrices lie in
 * address ranges of the same one of two classes that alternate every 64 GiB or
 * so than when each of them straddles a boundary between the classes (the first
 * two allocations of a process are the slow case).  The class of an address is
 * not visible to a program, but it shows in the time, so this call measures:
 * it runs groot_spmm_execute (three times per try, timed with events on
 * hip_stream, which it synchronises) with X and Y at every pair of offsets in
 * the arena that are multiples of half a matrix (of a larger even number of
 * quarters once the arena holds more than 16 such offsets: at most 256 pairs
 * are tried, whatever the arena's size) and do not overlap, then at
 * the quarter-matrix neighbours of the best pair (offsets in whole 4 KB
 * units), and returns the byte offsets of the fastest pair, its time per step,
 * and the time with the two matrices back to back at the start of the arena.
 * arena_dev (device, 16-byte aligned, owned by the caller, contents are
 * overwritten): at least 2.25 matrices of max(rows, feature rows) x F fp32;
 * five matrices give the search room.  A caller that reuses its feature
 * buffers over many layers and epochs does this once.  Errors: EINVAL (NULL,
 * plan not uploaded, F, alignment, arena too small), EHIP.
 * ------------------------------------------------------------------------- */
groot_status groot_feature_placement(const groot_plan *plan, void *arena_dev, size_t arena_bytes,
                                     int32_t F, void *hip_stream, size_t *x_offset,
                                     size_t *y_offset, float *best_ms, float *first_ms);

/* What the library decided for an uploaded plan, for diagnostics and benchmarks:
 * "ld_pipelined" (0 the plain LD kernel always, 2 the pipelined one for F = 32,
 * 64 and 128), "pipe_depth" (gather slots per row of the pipelined kernel, 5 to
 * 8), "mid_rows" (low-degree rows with more entries than that, which a row-list
 * kernel computes), "csr_compressed" (1 when the pipelined kernel reads 4-byte
 * row pointers and 2-byte column codes instead of the 8- and 4-byte arrays), "hd_pieces" (launch size of the HD kernel),
 * "hd_partials" (partial-sum slots of split high-degree rows), "weight_mode"
 * (how the kernels take the weights: 0 all 1, 1 fl(1 / row length) recomputed
 * from the row pointer, 2 read from the weight array), "nnz_hd" (stored entries
 * of the high-degree rows), "csr_bytes" (bytes of the graph's device arrays
 * that one execute reads: row pointers, column indices, the weights only when
 * the kernels read them, the high-degree pieces' descriptors; "csr_bytes_ld" /
 * "csr_bytes_hd" its split over the low-degree and the high-degree kernel).
 * Errors: EINVAL (NULL, unknown name, plan not uploaded). */
groot_status groot_plan_query(const groot_plan *plan, const char *what, int64_t *value);

/* The HD kernel's launch list of an uploaded plan, in launch order, copied to
 * host arrays of `capacity` entries each (any of them may be NULL = not
 * wanted): piece c covers stored entries [begin[c], begin[c] + len[c]) of row
 * row[c]; slot[c] is its partial-sum slot, or -1 when the row has one piece.
 * Paper: Section "Kernel Design - GROOT-GPU" (static split of a high-degree
 * row's non-zeros).  For tests and diagnostics: a plan made on the device
 * (groot_dev_part_plan) carries the same list, bit for bit, as a host plan of
 * the same sub-graph.  A plan made by groot_spmm_plan answers before its
 * upload too, from the host copy of the list that the upload will send (so do
 * "hd_pieces" and "hd_partials" of groot_plan_query).  Synchronous.  Errors:
 * EINVAL (NULL plan, a device-built plan that is gone from the device,
 * capacity below "hd_pieces"), EHIP. */
groot_status groot_plan_hd_pieces(const groot_plan *plan, int64_t capacity, int64_t *begin_host,
                                  int32_t *len_host, int32_t *row_host, int32_t *slot_host);

/* Launch-shape knobs for experiments: "xcd_remap" (0/1, read by
 * groot_plan_upload), "hd_chunk" (largest piece of a high-degree row,
 * 64..4096 non-zeros, read by groot_spmm_plan), "uniform_detect" (1, default:
 * groot_plan_upload checks whether the weights of a graph from
 * groot_graph_from_csr are bit for bit fl(1 / row length), or all 1, and then
 * runs it like a graph built from an AIG, without reading the weight array; 0:
 * never), "sage_kernel" (1, default: the fused
 * layer runs as self-contained wavefronts; 0: as producer and consumer
 * wavefronts; graphs with explicit weights always take the latter),
 * "sage_split" (kernel 0 only: 1 bf16 piece products, 0 fp32 matrix
 * instructions), "sage_gap" (kernel 0 only: 0..4, the pause between its matrix
 * instructions; all three read at each call of groot_sage_layer_forward),
 * "sage_pieces" (kernel 1 only: 3, default: every fp32 operand of the layer's
 * dense products is cut into three bf16 pieces and six piece products are
 * kept, fp32 accuracy; 2: two pieces and three products, half the matrix
 * instructions, every product exact to 3 x 2^-18 of its magnitude instead of
 * 2^-23; read at each call),
 * "csr_compress" (1, default: groot_plan_upload also builds a compact copy of
 * the matrix for the pipelined LD kernel, 4-byte row pointers and 2-byte column
 * codes, when every entry of a short row lies within 16,384 rows of its own row
 * or names one of the first 32,768 high-degree rows, and the matrix has fewer
 * than 2^32 entries; 0: never),
 * "ld_pipeline" (which LD kernel is used: 1 the software-pipelined one for
 * F = 32, 64, 128; 0 the plain one; -1 (default) the pipelined one with the
 * smallest number of gather slots per row, 5 to 8, that leaves at most 2
 * low-degree rows in 100 with more entries than slots, the plain one if none
 * does; read by groot_plan_upload) and "pipe_depth" (0, default: that rule;
 * 5..8: this many slots whenever the pipelined kernel is used; read by
 * groot_plan_upload).
 * Unknown names give EINVAL.  Not needed for normal use. */
groot_status groot_set_tuning(const char *name, int64_t value);

/* Thread-local description of the last failure on this thread; never NULL. */
const char *groot_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* GROOT_H */
