/* libampsens -- per-operator loss-MSE sensitivity statistics for FP8 mixed precision,
 * hand-written for AMD MI355X (gfx950).
 *
 * What the library computes (paper: "Automatic mixed precision for optimizing gained time
 * with constrained loss mean-squared-error based on model partition to sequential
 * sub-graphs", arXiv 2505.13060):
 *
 *   For every linear operation l of a network (a linear layer with operands X_l, W_l, or a
 *   BGEMM with operands X_{0,l}, X_{1,l}; Sec. 2.2, definition of the extended input z_l)
 *   and every calibration sample r, with zdot = dg/dz evaluated at high precision:
 *
 *     A = sum_k zdot_k^2 z_k^2            the sensitivity s_l^r = ||z (.) zdot||^2 of Sec. 2.2,
 *                                         restricted to one operand;
 *     E = sum_k zdot_k^2 (z_k - ztilde_k)^2   the first-order Taylor term (ztilde)^T zdot of
 *                                         Sec. 2.2 with the actual rounding error of an FP8 cast
 *                                         in place of the uniform-noise model, components taken
 *                                         as independent as the paper does.
 *
 *   ztilde is the absmax-scaled FP8 fake quantisation of z, with one scale per tensor or,
 *   optionally, one per row (see "scale granularity" below).  The paper names the
 *   format only by its bit split, four exponent and three mantissa bits (Sec. 3.1), and does not describe
 *   the cast; this library uses the OCP 8-bit formats (E4M3: max 448, no infinities; E5M2:
 *   max 57344), round to nearest even, saturating:
 *
 *     amax  = max_k |z_k| over the whole operand buffer
 *     scale = amax / FMAX, inv = FMAX / amax   (fp32 divisions; amax == 0, or an inv that
 *                                               overflows fp32, gives scale = inv = 1)
 *     y     = fl32(z_k * inv) clamped to +-FMAX;  code = RNE_f(y);  q = decode_f(code)
 *     ztilde_k = q * scale;   z_k - ztilde_k is formed as one fused multiply-add in fp32.
 *
 *   The sums then feed the host-side selection of eq. (ip) (Sec. 2.1): one format combination
 *   per sequential sub-graph, maximising gained time under a loss-MSE budget.
 *
 * Conventions
 *   - bf16 tensors are uint16_t storage.  "device" pointers are HIP device memory, "host"
 *     pointers ordinary memory.  Inputs are never written.  The caller owns every buffer,
 *     including the workspace; the library allocates no device memory and frees nothing.
 *   - Device calls validate their arguments on the host first (no launch happens on an error),
 *     then enqueue on the caller's stream (a hipStream_t passed as void*, NULL = the null
 *     stream).  They launch kernels and nothing else: no device or pinned memory is allocated or
 *     freed, no copy engine is used, nothing waits for the GPU, and nothing of the host arguments
 *     is referenced after the call returns (the small descriptor table of a call travels to the
 *     head of the workspace as kernel arguments, at most 3840 bytes per launch; the records of
 *     an operand's samples, which differ by fixed steps, travel as one record that a kernel
 *     expands).  Such calls may be recorded into a HIP graph by stream capture.
 *   - Every device call is a set-up (host work per op, the table, the chunk map) followed by a run
 *     (kernel launches only).  Callers that repeat a call on the same buffers keep the set-up:
 *     amp_*_setup fills a caller-owned amp_plan_t, amp_run replays it (see "plans" below).
 *   - Pointers need only 2-byte alignment; 16-byte aligned buffers take the fast path
 *     (128-bit loads).  Results do not depend on the launch grid.
 *   - Every call returns amp_status_t.  After AMP_ERR_DEVICE, amp_last_device_error() gives
 *     the hipError_t of the failing runtime call (per host thread).
 *   - Non-finite inputs: amp_absmax_scale raises bit 0 of the tensor's flag word; the sums of
 *     an operand that holds NaN or Inf are unspecified.  The sensitivity kernels leave the clamp to
 *     +-FMAX to the FP8 conversion, which saturates finite values but not infinities: the scales passed
 *     to a sensitivity call must keep |z_k| * inv below 2^128 (any scale derived from an absmax of
 *     data within a factor 2^88 of these does); otherwise that operand's sums are NaN.
 */
#ifndef AMPSENS_H
#define AMPSENS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum amp_status {
    AMP_OK = 0,
    AMP_ERR_INVALID_ARG = 1,         /* null pointer, negative size, inconsistent descriptor */
    AMP_ERR_BAD_FORMAT = 2,          /* format enum out of range, or n_fmts not in [1, AMP_MAX_FORMATS] */
    AMP_ERR_WORKSPACE_TOO_SMALL = 3,
    AMP_ERR_NONFINITE_INPUT = 4,     /* reserved for callers that read the flag words back */
    AMP_ERR_DEVICE = 5,              /* a HIP runtime call failed; see amp_last_device_error() */
    AMP_ERR_INFEASIBLE = 6,          /* amp_select_subgraphs: no configuration meets the budget */
    AMP_ERR_TOO_LARGE = 7            /* more work than the 32-bit chunk index can address */
} amp_status_t;

typedef enum amp_fp8_format {
    AMP_FP8_E4M3 = 0,                /* OCP E4M3: bias 7, max 448, S.1111.111 = NaN, m_f = 3 */
    AMP_FP8_E5M2 = 1,                /* OCP E5M2: bias 15, max 57344, IEEE-like, m_f = 2 */
    AMP_FP8_FORMAT_INT_RANGE_ = 0x7FFFFFFF   /* not a format: gives the type the range of int, so that a
                                                format or-ed with a flag (AMP_SCALE_POW2), or an invalid
                                                value on its way to AMP_ERR_BAD_FORMAT, is a valid value
                                                of the type in C++ as well */
} amp_fp8_format_t;

#define AMP_MAX_FORMATS 2

/* Scale granularity.  The paper does not say at which granularity its FP8 casts are scaled (Sec. 3.1
 * only mentions that scales exist).  By default every operand buffer has one scale per candidate
 * format.  With a bit of `scale_rows` set in a descriptor, the operand is a [rows, row_len] array
 * and row i is cast with its own scale: per token for the activations X of a linear layer
 * (row_len = C), per output channel for its weight W [K, C], per row of a BGEMM operand.  The
 * scale / reciprocal arrays of that operand are then device tables [rows][n_fmts] covering all
 * samples (X: rows_total rows; W: K rows shared by the samples; BGEMM: R * rows-per-sample rows),
 * as amp_absmax_scale_rows writes them.  Fast path: row_len a multiple of 8 and 16-byte aligned
 * buffers; anything else is computed element by element. */
/* Scale rule.  Or-ed into a format passed to amp_absmax_scale / amp_absmax_scale_rows: the scale
 * is the smallest power of two s with amax / s <= FMAX_f and the reciprocal is 1 / s, both exact
 * (exponent-only scale factors), instead of amax / FMAX_f and FMAX_f / amax.  amax == 0, a
 * non-finite amax, or an s whose reciprocal is not an fp32 number give scale = inv = 1.
 * On a sensitivity call the flag, set on every format, says two things.  (1) Operands whose row
 * scales the call computes itself (AMP_ROWS_COMPUTE0 / 1 below) get them by this rule.  (2) It is a
 * promise about the operands that come with one scale per tensor: their scales are powers of two s
 * with reciprocal 1 / s and no element exceeds FMAX_f * s in magnitude, which is what the absmax
 * calls give under this rule for the data they scanned.  The pass then casts with gfx950's scaled
 * FP8 conversions (packed bf16 in, exponent-only scale), which saves about a fifth of its vector
 * instructions and gives the same codes and the same sums as the general cast, bit for bit; an element that breaks the promise is not saturated but
 * turns into the format's NaN / Inf code, and the sums of its operand are then NaN. */
#define AMP_SCALE_POW2 0x100

#define AMP_ROWS_OPERAND0 1          /* X of a linear layer / X0 of a BGEMM */
#define AMP_ROWS_OPERAND1 2          /* W of a linear layer / X1 of a BGEMM */
/* Single-read variant: the sensitivity pass itself finds each row's absmax, derives the scales with
 * the arithmetic of amp_absmax_scale_rows (the rule, amax / FMAX or power of two, is taken from the
 * formats passed to the sensitivity call, which may carry AMP_SCALE_POW2 for this purpose) and casts the
 * row with them.  The threads that reduce a row keep it in on-chip memory and stream its gradient
 * against it, so every byte of the operand is fetched once and no separate absmax pass runs over it.  The operand's scale / reciprocal tables are then OUTPUTS of the pass (same
 * [rows][n_fmts] layout), and no amax or non-finite flag is produced (a NaN or Inf in a row shows in
 * that sample's sums).  Requires rows made of whole 16-byte vectors (row length a multiple of 8,
 * 16-byte aligned buffers) of at most AMP_ROWS_COMPUTE_MAX_ROW_LEN elements; anything else is
 * AMP_ERR_INVALID_ARG (use the two-pass form).  For a
 * linear layer only the activations can be computed this way: the weight is shared by the samples and
 * small next to its R gradients, its table comes from amp_absmax_scale_rows. */
#define AMP_ROWS_COMPUTE_MAX_ROW_LEN 24576
#define AMP_ROWS_COMPUTE0 4          /* operand 0: one scale per row, computed by the pass */
#define AMP_ROWS_COMPUTE1 8          /* operand 1 of a BGEMM, likewise */
/* One scale per 1 x n block (tile scaling, e.g. n = 128): or-ed into scale_rows next to the bits above, it
 * cuts every row of the operands those bits name into blocks of n consecutive elements, each cast with
 * its own scale.  n must divide the row length (C of a linear layer, cols of a dense BGEMM operand;
 * causal operands have no blocks: AMP_ERR_INVALID_ARG), 0 < n < 2^23.  The tables are then
 * [rows * row_len / n][n_fmts], blocks of a row consecutive: exactly the tables amp_absmax_scale_rows
 * writes for the same buffer described as a dense layout with cols = n.  Fast path: n a multiple of 8. */
#define AMP_ROWS_BLOCK(n) ((int32_t)((uint32_t)(n) << 8))
#define AMP_ROWS_BLOCK_OF(scale_rows) ((int64_t)((uint32_t)(scale_rows) >> 8))

/* Shape of one sample's block of an operand.
 * causal == 0: n_elems consecutive elements (batch/rows/cols ignored).
 * causal == 1: a [batch, rows, cols] array of which entry (b, i, j) belongs to the operand
 *              iff j <= i + (cols - rows) (lower triangle, aligned bottom-right; the attention
 *              probabilities P of a causal model).  Other entries count as zero whatever they
 *              hold (they may be fetched along with neighbouring entries of the same row, but
 *              their values, NaN included, have no effect).  n_elems is ignored; the block
 *              spans batch*rows*cols elements. */
typedef struct amp_layout {
    int64_t n_elems;
    int64_t batch, rows, cols;       /* causal == 0: only cols is read, and only where rows matter (per-row
                                        scales): the block is [n_elems / cols, cols] */
    int32_t causal;
    int32_t reserved;
} amp_layout_t;

/* One operand buffer for amp_absmax_scale: n_samples consecutive blocks of `layout`. */
typedef struct amp_tensor {
    const uint16_t* data;            /* device, bf16 */
    amp_layout_t layout;
    int64_t n_samples;
} amp_tensor_t;

/* Linear layer Y = X W^T (+ bias, which is not part of z; Sec. 2.2 eq. (lin_layer)).
 * X stacks the R samples along its rows. */
typedef struct amp_linear_desc {
    const uint16_t* x;               /* device bf16 [rows_total, C] */
    const uint16_t* dx;              /* device bf16 [rows_total, C]: dg/dX */
    const uint16_t* w;               /* device bf16 [K, C], shared by all samples */
    const uint16_t* dw;              /* device bf16 [R, K, C]: dg^r/dW of each sample */
    int64_t C, K;
    int64_t tokens;                  /* rows per sample, used when sample_row_offsets == NULL */
    const int64_t* sample_row_offsets; /* HOST, R+1 non-decreasing entries, first 0: sample r owns
                                          rows [off[r], off[r+1]); NULL = equal blocks of `tokens` */
    int32_t R;
    int32_t scale_rows;              /* 0, or AMP_ROWS_OPERAND0 (one scale per token) | AMP_ROWS_OPERAND1
                                        (one per output channel) */
    const float* x_scale;            /* device [n_fmts]: scale of X per candidate format
                                        (per token: [rows_total][n_fmts]) */
    const float* x_inv;              /* device, same shape: reciprocal scale of X */
    const float* w_scale;            /* device [n_fmts] (per output channel: [K][n_fmts]) */
    const float* w_inv;              /* device, same shape */
} amp_linear_desc_t;

/* BGEMM (Sec. 2.2 eq. (bgemm_layer)); both operands carry one block per sample. */
typedef struct amp_bgemm_desc {
    const uint16_t* x0;              /* device bf16 [R] x layout0 */
    const uint16_t* dx0;             /* device bf16, same shape: dg/dX0 */
    const uint16_t* x1;              /* device bf16 [R] x layout1 */
    const uint16_t* dx1;
    amp_layout_t layout0, layout1;
    int32_t R;
    int32_t scale_rows;              /* 0, or AMP_ROWS_OPERAND0 | AMP_ROWS_OPERAND1: one scale per row of
                                        that operand; a dense layout then gives its row length in cols */
    const float* scale0;             /* device [n_fmts] (per row: [R * rows per sample][n_fmts]) */
    const float* inv0;
    const float* scale1;
    const float* inv1;
} amp_bgemm_desc_t;

/* ---- step 1: per-tensor absmax and scales ----------------------------------------------
 * For tensor t and format index f:
 *   d_amax[t]                = max |x| over the entries that belong to the tensor
 *   d_scale[t*n_fmts + f]    = amax / FMAX_f          d_inv[t*n_fmts + f] = FMAX_f / amax
 *   d_flags[t]               = bit 0 set iff a NaN or Inf was seen
 * One launch sequence covers all tensors.  Outputs are device arrays; workspace is device
 * memory of at least amp_absmax_workspace_bytes() bytes, 256-byte aligned, and must not be
 * shared with a call still in flight.  n_tensors == 0 is a no-op. */
amp_status_t amp_absmax_workspace_bytes(const amp_tensor_t* tensors, int n_tensors, size_t* bytes);
amp_status_t amp_absmax_scale(const amp_tensor_t* tensors /* host array */, int n_tensors,
                              const amp_fp8_format_t* fmts /* host */, int n_fmts,
                              float* d_amax, float* d_scale, float* d_inv, uint32_t* d_flags,
                              void* workspace, size_t workspace_bytes, void* stream);

/* The same per row (scale granularity above): tensor t is n_samples blocks of `layout`, seen as
 * rows of layout.cols entries (a causal row owns its valid prefix only).  With row_base(t) = rows
 * of the tensors before t,
 *   d_amax[row_base(t) + i], d_scale[(row_base(t) + i) * n_fmts + f], d_inv[...] as above per row,
 *   d_flags[t] = bit 0 set iff a NaN or Inf was seen anywhere in tensor t.
 * amp_absmax_rows_workspace_bytes also reports the total number of rows (n_rows, may be NULL). */
amp_status_t amp_absmax_rows_workspace_bytes(const amp_tensor_t* tensors, int n_tensors, size_t* bytes,
                                             int64_t* n_rows);
amp_status_t amp_absmax_scale_rows(const amp_tensor_t* tensors /* host array */, int n_tensors,
                                   const amp_fp8_format_t* fmts /* host */, int n_fmts,
                                   float* d_amax, float* d_scale, float* d_inv, uint32_t* d_flags,
                                   void* workspace, size_t workspace_bytes, void* stream);

/* ---- step 2 (standalone): FP8 fake quantisation ------------------------------------------
 *   d_codes[i]   = RNE_sat_f(fl32(x_i * inv_scale))      (uint8 FP8 code)
 *   d_dequant[i] = fl32(decode_f(d_codes[i]) * scale)     (optional, may be NULL)
 * d_x, d_codes, d_dequant: device, n elements each.  n == 0 is a no-op. */
amp_status_t amp_fake_quant_fp8(const uint16_t* d_x, int64_t n, float scale, float inv_scale,
                                amp_fp8_format_t fmt, uint8_t* d_codes, float* d_dequant,
                                void* stream);

/* ---- step 3: the fused sensitivity pass --------------------------------------------------
 * One pass over x and xdot of every operand of every op, for all n_fmts candidate formats at
 * once (each byte is read once whatever n_fmts is).
 * Output, fp32, device:  with base(k) = sum of R over ops before k,
 *   d_out[((base(k) + r) * n_fmts + f) * 4 + {0,1,2,3}] = (E_op0, A_op0, E_op1, A_op1)
 * for op k, sample r, format index f; operand 0 is X (linear) / X0 (BGEMM), operand 1 is W / X1.
 * A does not depend on f and is repeated.  Sample blocks of zero elements give zeros.
 * Workspace as for amp_absmax_scale, sized by the matching *_workspace_bytes call. */
amp_status_t amp_sens_linear_workspace_bytes(const amp_linear_desc_t* ops, int n_ops, int n_fmts,
                                             size_t* bytes);
amp_status_t amp_sens_linear(const amp_linear_desc_t* ops /* host array */, int n_ops,
                             const amp_fp8_format_t* fmts /* host */, int n_fmts, float* d_out,
                             void* workspace, size_t workspace_bytes, void* stream);

amp_status_t amp_sens_bgemm_workspace_bytes(const amp_bgemm_desc_t* ops, int n_ops, int n_fmts,
                                            size_t* bytes);
amp_status_t amp_sens_bgemm(const amp_bgemm_desc_t* ops /* host array */, int n_ops,
                            const amp_fp8_format_t* fmts /* host */, int n_fmts, float* d_out,
                            void* workspace, size_t workspace_bytes, void* stream);

/* Linear layers and BGEMMs of one call (a whole transformer block, or a whole model): the same sums,
 * bit for bit, as amp_sens_linear followed by amp_sens_bgemm, with one descriptor table, one set-up
 * and one finalisation for all of them, and the BGEMM operands streamed by the same launch as the
 * activations.  d_out holds the linear layers' block first ([sum of R over the linears][n_fmts][4],
 * laid out as above) and the BGEMMs' block right behind it.  Either array may be empty. */
amp_status_t amp_sens_block_workspace_bytes(const amp_linear_desc_t* linears, int n_linears,
                                            const amp_bgemm_desc_t* bgemms, int n_bgemms, int n_fmts,
                                            size_t* bytes);
amp_status_t amp_sens_block(const amp_linear_desc_t* linears /* host array */, int n_linears,
                            const amp_bgemm_desc_t* bgemms /* host array */, int n_bgemms,
                            const amp_fp8_format_t* fmts /* host */, int n_fmts, float* d_out,
                            void* workspace, size_t workspace_bytes, void* stream);

/* amp_sens_block for callers that cannot allocate (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc) and have no workspace at hand: the same pass, the same
 * sums bit for bit, with the workspace in a device array of AMP_STATIC_WORKSPACE_BYTES that is part
 * of the library's code object (every GPU the library runs on holds it until the process ends).
 * Calls whose amp_sens_block_workspace_bytes exceed it return AMP_ERR_WORKSPACE_TOO_SMALL before
 * anything is launched (16 MiB covers one Llama-7B-shaped block at S = 2048 with 16 resident
 * samples).  The call allocates and frees nothing on the device or in pinned memory and does not
 * wait for the GPU.  All calls on a GPU share that GPU's array: two calls that overlap in time on
 * one GPU (different streams, or different host threads without ordering) race; calls on one
 * stream, or ordered by events, are safe.  Nothing in the array needs clearing between calls: every
 * word a pass reads has been written earlier in the same pass. */
#define AMP_STATIC_WORKSPACE_BYTES (16u << 20)
amp_status_t amp_sens_block_static(const amp_linear_desc_t* linears /* host array */, int n_linears,
                                   const amp_bgemm_desc_t* bgemms /* host array */, int n_bgemms,
                                   const amp_fp8_format_t* fmts /* host */, int n_fmts, float* d_out,
                                   void* stream);

/* ---- step 4 (host): epilogue of Sec. 2.2 -------------------------------------------------
 * sums: HOST copy of one op's block of d_out, [R][n_fmts][4].
 *   *s_layer       = (1/R) sum_r (A_op0^r + A_op1^r)                 (eq. (sensl))
 *   d_model[f]     = s_layer * alpha_f, alpha_f = 2^(-2 m_f)/12      (noise-model loss MSE)
 *   d_measured[f]  = (1/R) sum_r (E_op0^r + E_op1^r)                 (measured first-order term)
 * d_model / d_measured: host arrays of n_fmts doubles, either may be NULL. */
amp_status_t amp_layer_loss_mse(const float* sums, int R, const amp_fp8_format_t* fmts, int n_fmts,
                                double* s_layer, double* d_model, double* d_measured);

/* The loss-MSE budget of eq. (ip) (Sec. 2.1): tau^2 E[g^2], with tau < 1 the threshold on the
 * normalised RMSE and E[g^2] the mean of the squared losses g^r of the n calibration samples
 * (host array; NaN for n < 1). */
double amp_loss_second_moment(const double* losses, int n);
double amp_mse_budget(double tau, double mean_g2);

/* alpha_f = 2^(-2 m)/12 for a float format with m mantissa bits (Sec. 2.2). */
double amp_alpha(int mantissa_bits);

/* Tables of one group V_j of L_j layers with F formats each (Sec. 2.1, matrix Q_j):
 * column p is the base-F digit string of p, layer 0 least significant;
 *   d[p] = sum_l layer_mse[l*F + digit_l(p)],   c[p] = sum_l layer_gain[l*F + digit_l(p)]
 * (last equation of Sec. 2.2; additive gain of Sec. 2.3.2).  d and c hold F^L_j doubles.
 * All host pointers.  F^L_j above 2^24 is rejected. */
amp_status_t amp_group_tables(int n_layers, int F, const double* layer_mse, const double* layer_gain,
                              double* d, double* c);

/* ---- step 5 (host): eq. (ip) of Sec. 2.1 --------------------------------------------------
 * Maximise sum_j gain[j][p_j] subject to sum_j mse[j][p_j] <= mse_budget, one p_j per group.
 * n_choices[J]; gain and mse are the concatenation of the groups' vectors (sum n_choices
 * doubles).  Exact (branch and bound).  Among optimal configurations the one with the smaller
 * total mse is returned.  All pointers host; choice[J] receives p_j; total_gain / total_mse may
 * be NULL.  AMP_ERR_INFEASIBLE when no configuration meets the budget.  Non-finite or negative
 * mse entries are AMP_ERR_INVALID_ARG. */
amp_status_t amp_select_subgraphs(int J, const int32_t* n_choices, const double* gain,
                                  const double* mse, double mse_budget, int32_t* choice,
                                  double* total_gain, double* total_mse);

/* ---- next to the path (host): partition, gain formulas, baseline strategies ------------------
 *
 * amp_partition_sequential: partition of a model's computation DAG into sequential sub-graphs
 * (Appendix B, Algorithm 2): single-entry / single-exit regions, each closed by the first vertex
 * through which every path to the sink passes; that vertex belongs to the group it closes.
 * Vertices 0..n-1, edges src -> dst (host arrays); exactly one vertex without predecessors (the
 * start vertex, never part of a group) and one without successors (the sink); the graph must be
 * acyclic.  quantizable[v] != 0 marks the linear operations (NULL = all); other vertices are dropped
 * and groups left empty disappear.  group_of[v] receives the group index in execution order, or -1.
 * Residual connections are edges like any other: leave them out to obtain the per-block groups of
 * the paper's figure for a Llama layer. */
amp_status_t amp_partition_sequential(int n_vertices, int n_edges, const int32_t* edge_src,
                                      const int32_t* edge_dst, const uint8_t* quantizable,
                                      int32_t* group_of, int32_t* n_groups);

/* Theoretical time gain of Sec. 2.3.2: N*C*K*delta_t for a linear layer, N*C*C*delta_t for a
 * BGEMM; memory gain of Sec. 2.3.3: C*K*delta_m for a linear layer, 0 for a BGEMM. */
double amp_time_gain_macs(int is_bgemm, double N, double C, double K, double delta_t);
double amp_memory_gain(int is_bgemm, double C, double K, double delta_m);

/* Baseline strategies of Sec. 3.1 under the same loss-MSE bound: walk the groups in `order`
 * (host, a permutation of 0..J-1; NULL = 0,1,2,... which is the paper's Prefix; a random
 * permutation gives its Random) and switch each group to its largest-gain choice while the total
 * MSE stays within the budget; the first group that does not fit ends the walk.  Same table layout
 * as amp_select_subgraphs; choice 0 of a group is its high-precision column. */
amp_status_t amp_select_ordered(int J, const int32_t* n_choices, const double* gain, const double* mse,
                                double mse_budget, const int32_t* order, int32_t* choice,
                                double* total_gain, double* total_mse);

/* ---- plans: set-up once, run many times -----------------------------------------------------------
 * The calibration loop of the paper's Algorithm 1 (step "sensitivity calibration") visits the same
 * operand buffers sample after sample; the set-up of a call depends on pointers and shapes only.
 * amp_*_setup does everything the one-shot call of the same name does except the pass itself, on
 * `stream`, and records what a run needs in *plan (plain data, caller-owned, may be copied; it
 * holds the workspace and output pointers given here).  amp_run enqueues the pass: it reads the
 * scales (sensitivity pass) or the operands (absmax) as they are when it executes, so an absmax
 * run followed by a sensitivity run on the same stream is one calibration step.  The workspace
 * must stay untouched between the set-up and the last run, runs of one plan must not overlap, and
 * a run must be ordered after the set-up (same stream, or an event).  A call without work gives a
 * plan whose run does nothing.  amp_sens_block_setup takes the flags below.
 * amp_plan_limit_grid caps the number of workgroups of the plan's persistent grids (0 = as many as
 * are resident), e.g. to leave compute units to a concurrent forward pass; results do not change. */
typedef struct amp_plan { uint64_t opaque[64]; } amp_plan_t;

#define AMP_PLAN_STREAM_WEIGHTS 1u   /* read W with every sample's gradient instead of once per batch of
                                        8 resident gradients (same sums, bit for bit) */
#define AMP_PLAN_INTERLEAVE(n) ((uint32_t)((n) & 0xFF) << 8)   /* tuning: chunks of one reader of a shared W
                                        that sit next to each other in the schedule (0 = default 8) */

amp_status_t amp_absmax_scale_setup(const amp_tensor_t* tensors /* host array */, int n_tensors,
                                    const amp_fp8_format_t* fmts /* host */, int n_fmts,
                                    float* d_amax, float* d_scale, float* d_inv, uint32_t* d_flags,
                                    void* workspace, size_t workspace_bytes, void* stream, amp_plan_t* plan);
amp_status_t amp_absmax_scale_rows_setup(const amp_tensor_t* tensors /* host array */, int n_tensors,
                                         const amp_fp8_format_t* fmts /* host */, int n_fmts,
                                         float* d_amax, float* d_scale, float* d_inv, uint32_t* d_flags,
                                         void* workspace, size_t workspace_bytes, void* stream,
                                         amp_plan_t* plan);
amp_status_t amp_sens_block_setup(const amp_linear_desc_t* linears /* host array */, int n_linears,
                                  const amp_bgemm_desc_t* bgemms /* host array */, int n_bgemms,
                                  const amp_fp8_format_t* fmts /* host */, int n_fmts, float* d_out,
                                  void* workspace, size_t workspace_bytes, uint32_t flags, void* stream,
                                  amp_plan_t* plan);
amp_status_t amp_plan_limit_grid(amp_plan_t* plan, int max_workgroups);
amp_status_t amp_run(const amp_plan_t* plan, void* stream);

/* ---- optional kernel timing ---------------------------------------------------------------
 * amp_profile_enable(n > 0) creates n pairs of HIP events on the current device; from then on
 * every launch of a fused sensitivity kernel records one pair on the run's stream, immediately
 * before and after the kernel, until n launches have been recorded.  A sensitivity run launches
 * the weight kernel (W read once per batch of samples) if it has whole weight chunks for it, then
 * the streaming kernel for everything else (activations, BGEMM operands, ragged ends).  Operands
 * with one scale per row have kernels of their own: a run then launches up to two weight kernels
 * (per-tensor, per-channel) and up to seven streaming kernels (one scale per tensor; long or
 * causal rows; other shapes; short power-of-two rows; three launches of the single-read pass), in that
 * order, each only if it has work.
 * amp_profile_read waits for the recorded events, writes the elapsed milliseconds of each
 * launch to ms[0..*n_launches) and, if not NULL, to pairs[] the number of element pairs the
 * launch covered and to bytes[] the operand bytes it is defined to read (4 per pair for the
 * streaming kernel; for the weight kernel 2 per pair plus W's bytes once per batch of samples)
 * (host arrays; capacity must be >= the n given to enable), and resets the count.
 * amp_profile_kinds (call it before amp_profile_read, which resets the count) tells which kernel each
 * recorded launch was: AMP_KERNEL_WEIGHTS (+1 with per-channel scales), or AMP_KERNEL_STREAM + c with
 * c = 0 one scale per tensor; 1 long or causal rows; 2 other row shapes; 3 short power-of-two rows;
 * 4, 5, 6 the single-read pass (rows held in registers; staged in up to 32 KiB; in up to 48 KiB of LDS).
 * amp_profile_enable(0) destroys the events.  Meant for benchmarks: do not enable it around a
 * stream capture, and do not call enable / read while runs are being enqueued from other threads. */
#define AMP_KERNEL_WEIGHTS 0
#define AMP_KERNEL_STREAM 16
amp_status_t amp_profile_enable(int max_launches);
amp_status_t amp_profile_kinds(int* kinds /* host */, int capacity, int* n_launches);
amp_status_t amp_profile_read(float* ms, uint64_t* pairs, uint64_t* bytes, int capacity, int* n_launches);

/* ---- misc ---------------------------------------------------------------------------------*/
const char* amp_status_string(amp_status_t status);
int amp_last_device_error(void);
int amp_version(void);               /* major*10000 + minor*100 + patch */

#ifdef __cplusplus
}
#endif
#endif /* AMPSENS_H */
