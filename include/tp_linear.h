/*
 * tp_linear.h -- C ABI of libtplinear: one rank's share of a tensor-parallel linear layer on one
 * MI355X (gfx950), forward and backward.
 *
 * What is computed (paper Section 2.2 "Model Parallelism", tensor-parallelism paragraphs; Section
 * 3.1 and Table 1 for the notation): a linear layer  Y = GeLU(X W + 1 b^T)  whose input, weight and
 * output are cut into chunks over a rank grid -- 1D (Megatron feed-forward: first weight cut by
 * columns, second by rows, every rank holding a partial output that an all-reduce would sum), 2D
 * (SUMMA on a q x q square, chunks [P/q, Q/q]), 2.5D (q x q x d cuboid, N = S^2 D) and 3D (p x p x p
 * cube, chunks [P/p^2, Q/p]).  One rank's work is an ordered loop of local block products
 *      C += A_k B_k,   k = 0 .. n_steps-1,
 * followed by bias add and erf-GeLU, and in backward  dX = sum_k dA_k W_k^T,  dW = sum_k X_k^T dA_k.
 * The blocks other ranks would broadcast or gather are already in this GPU's memory: the library
 * performs no communication.
 *
 * Conventions.  Tokens are rows.  All blocks are row-major with a leading dimension `ld` counted in
 * elements.  X:[M,H], W:[H,F] (in x out), b:[F].  bf16 inputs, fp32 accumulation, fp32 or bf16
 * outputs (bf16 by round-to-nearest-even).  Every pointer in this ABI is a DEVICE pointer unless it
 * is explicitly called a host array; host arrays are read during the call and may be freed after it.
 *
 * Ownership / errors.  The caller owns every buffer; the library never allocates, frees or
 * synchronises.  Work is enqueued on the HIP stream passed in (a hipStream_t cast to void*, NULL =
 * the default stream) and the call returns immediately.  Inputs are read-only and may alias each
 * other but not outputs.  Every failure is a return code found before anything is launched; nothing
 * is written on error.  Row counts may be any value >= 1 (ragged tails are masked); column extents
 * of every block and every `ld` must be multiples of 8 elements and every pointer, the workspace
 * included, 16-byte aligned (128-bit loads and stores), else TP_ERR_ALIGN (TP_ERR_WORKSPACE for the
 * workspace).  The library keeps no mutable state between calls apart from per-device caches of kernel
 * attributes, of the device's compute-unit count and of the address of its built-in scratch array;
 * every entry point may be called from several threads at once (tp_linear_fwd_static: see its own
 * note on calls that overlap on one GPU).
 */
#ifndef TP_LINEAR_H
#define TP_LINEAR_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define TP_MAX_STEPS 16

typedef enum {
    TP_OK = 0,
    TP_ERR_NULL = 1,       /* a required pointer is NULL */
    TP_ERR_MODE = 2,       /* unknown mode / pass / epilogue */
    TP_ERR_GRID = 3,       /* q, d or p < 1, or a rank coordinate outside the grid */
    TP_ERR_SHAPE = 4,      /* M, H, F not divisible as the mode requires; n_steps out of range */
    TP_ERR_ALIGN = 5,      /* pointer not 16-byte aligned, or ld / column extent not a multiple of 8 */
    TP_ERR_DTYPE = 6,      /* output dtype not supported for this output */
    TP_ERR_WORKSPACE = 7,  /* workspace NULL or smaller than tp_linear_workspace_size() says */
    TP_ERR_HIP = 8,        /* a HIP call (launch) reported an error */
    TP_ERR_SCRATCH = 9     /* tp_linear_fwd_static: the product needs more than the built-in scratch */
} tp_status_t;

/* Partition modes.  The 1D scheme is two modes because its two weights are cut differently. */
typedef enum {
    TP_MODE_1D_COL = 10,   /* W cut by columns: rank r owns W[:, r];  Y[:, r] = act(X W[:, r] + b[r])   */
    TP_MODE_1D_ROW = 11,   /* W cut by rows:    rank r owns W[r, :];  partial Y_r = X[:, r] W[r, :]      */
    TP_MODE_2D = 2,        /* q x q,      rank (ri, rj)                                                  */
    TP_MODE_2P5D = 25,     /* q x q x d,  rank (ri, rj, rk = depth layer)                                */
    TP_MODE_3D = 3,        /* p x p x p,  rank (ri, rj, rk)                                              */
    TP_MODE_3D_GATHERED = 33 /* p x p x p with the operands as they are after the all-gathers: one product
                              per pass on slabs [P/p, Q/p], every result a partial (see tp_block_map)   */
} tp_mode_t;

typedef enum { TP_BF16 = 0, TP_F32 = 1 } tp_dtype_t;
typedef enum { TP_EPI_NONE = 0, TP_EPI_BIAS = 1, TP_EPI_BIAS_GELU = 2 } tp_epilogue_t;
typedef enum {
    TP_PASS_FWD = 0, TP_PASS_DX = 1, TP_PASS_DW = 2,
    TP_PASS_DX_PARTIALS = 3, TP_PASS_DW_PARTIALS = 4     /* tp_partials_map / tp_linear_bwd_partials only */
} tp_pass_t;

/* 1D: p = size, ri = rank (q = d = 1).  2D: q, (ri, rj).  2.5D: q, d, (ri, rj, rk).  3D: p, (ri, rj, rk).
 * Unused sizes must be 1 and unused coordinates 0. */
typedef struct { int mode; int q, d, p; int ri, rj, rk; } tp_grid_t;
/* The FULL (unpartitioned) layer: M tokens, H input features, F output features. */
typedef struct { int64_t M, H, F; } tp_dims_t;
/* A read-only device block: bf16, row-major, ld in elements. */
typedef struct { const void* ptr; int64_t ld; } tp_cblk_t;
/* An output device block: row-major, ld in elements, dtype a tp_dtype_t.  ptr == NULL means "not wanted". */
typedef struct { void* ptr; int64_t ld; int dtype; } tp_oblk_t;
/* Launch-plan options of one call (tuning and tests; NULL = all automatic).  The same options must be
 * given to the workspace query and to the call it sizes.
 *   tile   : macro-tile of C.  0 automatic; 1 = 256x256 (four-wave stream kernel); 2 = 128x256,
 *            3 = 256x128, 4 = 128x128 (eight-wave kernel); 5 = 256x256 on the eight-wave kernel.
 *   split_k: workgroups sharing one C tile along K.  0 automatic, 1..8.
 *   group_m: height, in tile rows, of the groups of the tile order.  0 automatic, 1..64.
 *   rotate : rotate the K-tile order inside a step from C tile to C tile.  0 automatic (on for the
 *            eight-wave kernel, off for the four-wave one), 1 on, 2 off.
 *   trim   : when the tiles are a little more than a whole number of rounds of the persistent
 *            workgroups, run the last tile rows as a second, smaller launch.  0 automatic (on), 1 on, 2 off. */
typedef struct { int tile, split_k, group_m, rotate, trim; } tp_plan_opts_t;

/*
 * tp_block_map -- the partition map (host only, no GPU needed).  For rank `grid` of a layer `dims`
 * and a pass, reports how many steps the exact share has, the local product's extents and which
 * chunks take part, as (row chunk, col chunk) indices into the chunk grids below.
 *   chunk grids: X, dX: [rc x kc];  W, dW: [kc x cc];  Y, A, dA: [rc x cc];  b: [cc]
 *     1D_COL: rc=1, kc=1, cc=p      1D_ROW: rc=1, kc=p, cc=1      2D: rc=kc=cc=q
 *     2.5D: rc=q d, kc=cc=q (row chunk of rank (i,j,l) is l q + i; W and b repeat on every layer)
 *     3D:   rc=p^2, kc=cc=p (row chunk of rank (i,j,l) is i p + l)
 *   TP_PASS_FWD: C[m,n] = sum_k X[a_k] W[b_k];          out indexes Y (bias chunk = out_col)
 *   TP_PASS_DX : C[m,n] = sum_k dA[a_k] W[b_k]^T;       out indexes dX
 *   TP_PASS_DW : C[m,n] = sum_k X[a_k]^T dA[b_k];       out indexes dW
 *   3D_GATHERED (Section 2.2: the stored chunk is [P/p^2, Q/p]; gathered along one cube axis it is
 *     the slab [P/p, Q/p]): rc=kc=cc=p, one step per pass, every output a partial:
 *       FWD: X[i,l] W[l,j] -> partial of (X W)[i,j] over l      DX: dA[i,j] W[l,j]^T -> dX[i,l] over j
 *       DW : X[i,l]^T dA[i,j] -> dW[l,j] over i.   Bias and GeLU belong after the summation
 *     (tp_bias_act); row chunk l of the summed slab (i,j) is rank (i,j,l)'s block under TP_MODE_3D.
 * m, n = extents of the output block, k_per_step = contraction length of one step.
 * a_row..b_col are host arrays of TP_MAX_STEPS ints (may be NULL if not wanted); *is_partial = 1
 * when the block is an additive partial that a reduction over other ranks would complete
 * (1D partial sums; 2.5D dW over depth; 3D dW over the first cube axis).
 * Errors: TP_ERR_NULL, TP_ERR_MODE, TP_ERR_GRID, TP_ERR_SHAPE.
 */
int tp_block_map(const tp_grid_t* grid, const tp_dims_t* dims, int pass,
                 int* n_steps, int64_t* m, int64_t* n, int64_t* k_per_step,
                 int* a_row, int* a_col, int* b_row, int* b_col,
                 int* out_row, int* out_col, int* is_partial);

/* Bytes of device workspace tp_linear_fwd (pass TP_PASS_FWD), tp_linear_bwd (TP_PASS_DX and
 * TP_PASS_DW each; pass the larger, the two products run one after the other) or
 * tp_linear_bwd_partials (TP_PASS_DX_PARTIALS, TP_PASS_DW_PARTIALS) may need for this share:
 * cross-workgroup split-K partials in fp32 (never more than 8 x m x n x 4 bytes per product), and, for
 * the two backward passes, the row-slab sums of the bias gradient (at most 64 x n_fwd x 4 bytes; a
 * smaller workspace makes tp_linear_bwd fall back to the single-pass column sum).  0 on invalid
 * arguments. */
size_t tp_linear_workspace_size(const tp_grid_t* grid, const tp_dims_t* dims, int pass);
/* The same for calls made with plan options (NULL = tp_linear_workspace_size). */
size_t tp_linear_workspace_size_ex(const tp_grid_t* grid, const tp_dims_t* dims, int pass, const tp_plan_opts_t* opts);

/*
 * tp_linear_fwd -- forward share:  C = sum_{k<n_steps} X_k W_k  with the fp32 accumulator kept
 * on-chip across all steps;  A = C + b (epi >= TP_EPI_BIAS);  Y = GeLU(A) (TP_EPI_BIAS_GELU), else Y = A.
 *   x_blocks, w_blocks : host arrays [n_steps] of device blocks; X_k is [m, k], W_k is [k, n] with
 *                        m, n, k as tp_block_map reports for TP_PASS_FWD.
 *   n_steps            : 1 .. the map's step count (fewer steps = a prefix of the sum).
 *   bias               : bf16 [n] (this rank's chunk) or NULL when epi == TP_EPI_NONE.
 *   y                  : [m, n], fp32 or bf16.
 *   preact             : optional bf16 [m, n]: A rounded to bf16, saved for backward.
 *   workspace          : >= tp_linear_workspace_size(.., TP_PASS_FWD) bytes, 16-byte aligned (may be
 *                        NULL when that size is 0).
 * Defined by: Section 2.2, tensor-parallelism paragraphs (1D: first weight cut by columns, second by
 * rows, partial outputs; 2D / 2.5D / 3D: the chunk shapes) with the layer Y = W X of Section 3.1
 * written tokens-major and completed by bias and erf-GeLU.  When the map marks the output as an
 * additive partial (1D_ROW with p > 1, 3D_GATHERED) bias, GeLU and preact are refused (TP_ERR_MODE:
 * they belong after the summation, see tp_bias_act) and y must be fp32 (TP_ERR_DTYPE).
 * Errors: TP_ERR_NULL, TP_ERR_MODE, TP_ERR_GRID, TP_ERR_SHAPE, TP_ERR_ALIGN, TP_ERR_DTYPE,
 * TP_ERR_WORKSPACE, TP_ERR_HIP; nothing is launched unless every check has passed.
 */
int tp_linear_fwd(const tp_grid_t* grid, const tp_dims_t* dims, int n_steps,
                  const tp_cblk_t* x_blocks, const tp_cblk_t* w_blocks,
                  const void* bias, int epi, tp_oblk_t y, tp_oblk_t preact,
                  void* workspace, size_t workspace_bytes, void* hip_stream);
int tp_linear_fwd_ex(const tp_grid_t* grid, const tp_dims_t* dims, int n_steps,
                     const tp_cblk_t* x_blocks, const tp_cblk_t* w_blocks,
                     const void* bias, int epi, tp_oblk_t y, tp_oblk_t preact,
                     void* workspace, size_t workspace_bytes, void* hip_stream, const tp_plan_opts_t* opts);

/*
 * tp_linear_fwd_static -- tp_linear_fwd for callers that cannot allocate device memory and have no
 * workspace to hand over: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments, same checks and the same result as tp_linear_fwd with default plan
 * options, minus the workspace: the fp32 partial planes of a K-split product go to a fixed array of
 * tp_static_scratch_bytes() = 64 MiB that is part of the library's device image (each GPU the library
 * runs on holds its own copy until the process ends).  The call allocates and frees nothing; the
 * first call on a device looks the array's address up once (not capturable: make one call on the
 * device before capturing).  A product whose planes need more than the array is refused with
 * TP_ERR_SCRATCH and nothing is launched.  All calls on one GPU share the array: calls that may
 * overlap in time on one GPU (different streams, different threads) race on it and must be ordered
 * by the caller.  Nothing in the array has to start at zero: every partial the fix-up pass reads
 * was written by the product kernel of the same call.
 * Errors: those of tp_linear_fwd except TP_ERR_WORKSPACE, plus TP_ERR_SCRATCH.
 */
int tp_linear_fwd_static(const tp_grid_t* grid, const tp_dims_t* dims, int n_steps,
                         const tp_cblk_t* x_blocks, const tp_cblk_t* w_blocks,
                         const void* bias, int epi, tp_oblk_t y, tp_oblk_t preact, void* hip_stream);
/* Size in bytes of the built-in scratch array of tp_linear_fwd_static (host only, no GPU call). */
size_t tp_static_scratch_bytes(void);

/*
 * tp_linear_bwd -- backward share.  In order, each part only if its outputs are wanted:
 *   (1) own dA:  da_own_out = bf16(dy_own * GeLU'(preact_own))          [m_y, n_y] of the forward block;
 *                needs dy_own, preact_own, da_own_out.  When own_slot_dx >= 0 (own_slot_dw >= 0) the
 *                block just written is used as da_row_blocks[own_slot_dx] (da_col_blocks[own_slot_dw]),
 *                whatever those host entries hold.  db (fp32 [n_y], optional) receives its column sums.
 *   (2) dX = sum_{k<n_steps_dx} da_row_blocks[k] w_blocks_dx[k]^T        extents from TP_PASS_DX;
 *                if dgelu_preact is given (bf16, same shape as dX: the previous layer's saved
 *                pre-activation; the 1D chain) the result is multiplied by GeLU' of it in the epilogue.
 *   (3) dW = sum_{k<n_steps_dw} x_blocks_dw[k]^T da_col_blocks[k]        extents from TP_PASS_DW;
 *                fp32 output only (TP_ERR_DTYPE otherwise).
 *   For a layer without activation (1D_ROW) pass the upstream gradient blocks as the "da" blocks.
 *   workspace: >= max(tp_linear_workspace_size(DX), tp_linear_workspace_size(DW)).
 * Defined by: the gradients of the layer of tp_linear_fwd under the same partition (Section 2.2; the
 * three products of a layer, forward and two backward, are what the factor 3 of Table 1, Section 3.1,
 * counts for 2D and 2.5D), each rank accumulating its own block of dX and dW over the steps.  A dX
 * that the map marks as an additive partial (1D_COL with p > 1, 3D_GATHERED) must be fp32
 * (TP_ERR_DTYPE) and takes no dgelu_preact (TP_ERR_MODE).
 * Errors: as tp_linear_fwd.
 */
int tp_linear_bwd(const tp_grid_t* grid, const tp_dims_t* dims, int n_steps_dx, int n_steps_dw,
                  const tp_cblk_t* dy_own, const tp_cblk_t* preact_own,
                  const tp_cblk_t* da_row_blocks, const tp_cblk_t* w_blocks_dx,
                  const tp_cblk_t* x_blocks_dw, const tp_cblk_t* da_col_blocks,
                  int own_slot_dx, int own_slot_dw,
                  const tp_cblk_t* dgelu_preact,
                  tp_oblk_t dx, tp_oblk_t dw, tp_oblk_t da_own_out, void* db_f32,
                  void* workspace, size_t workspace_bytes, void* hip_stream);
int tp_linear_bwd_ex(const tp_grid_t* grid, const tp_dims_t* dims, int n_steps_dx, int n_steps_dw,
                     const tp_cblk_t* dy_own, const tp_cblk_t* preact_own,
                     const tp_cblk_t* da_row_blocks, const tp_cblk_t* w_blocks_dx,
                     const tp_cblk_t* x_blocks_dw, const tp_cblk_t* da_col_blocks,
                     int own_slot_dx, int own_slot_dw,
                     const tp_cblk_t* dgelu_preact,
                     tp_oblk_t dx, tp_oblk_t dw, tp_oblk_t da_own_out, void* db_f32,
                     void* workspace, size_t workspace_bytes, void* hip_stream, const tp_plan_opts_t* opts);

/*
 * tp_partials_map -- the partition map of the backward products in their other SUMMA form, for 2D
 * and 2.5D grids (host only).  The rank's own dA block (own_row, own_col) stays in place, one block
 * of the other operand takes part per step, and step k's product is an additive partial of the
 * block (out_row[k], out_col[k]) that another rank of the same row (dX) or column (dW) group owns.
 * This is the form whose traffic Table 1 (Section 3.1) counts for 2D and 2.5D: per product,
 * (side - 1) operand blocks in and (side - 1) partial blocks out.  Chunk grids as in tp_block_map.
 *   TP_PASS_DX_PARTIALS: P_k[m,n] = dA[own] W[other_k]^T      out indexes dX;   m, n, k = M_blk, H_blk, F_blk
 *   TP_PASS_DW_PARTIALS: P_k[m,n] = X[other_k]^T dA[own]      out indexes dW;   m, n, k = H_blk, F_blk, M_blk
 * other_row .. out_col are host arrays of TP_MAX_STEPS ints (may be NULL).
 * Errors: TP_ERR_NULL, TP_ERR_MODE (other modes or passes), TP_ERR_GRID, TP_ERR_SHAPE.
 */
int tp_partials_map(const tp_grid_t* grid, const tp_dims_t* dims, int pass,
                    int* n_steps, int64_t* m, int64_t* n, int64_t* k,
                    int* own_row, int* own_col, int* other_row, int* other_col,
                    int* out_row, int* out_col);

/*
 * tp_linear_bwd_partials -- backward share in the form tp_partials_map describes: all n_dx (n_dw)
 * products of a pass run in ONE launch whose tile grid covers every product, so a share whose
 * single product has too few tiles for the chip still fills it.
 *   da_own        : the rank's own dA block, bf16 [M_blk, F_blk].
 *   w_blocks_dx   : host array [n_dx] of W blocks [H_blk, F_blk];  dx_partials: host array [n_dx] of
 *                   fp32 outputs [M_blk, H_blk];  dx_partials[k] = da_own w_blocks_dx[k]^T.
 *   x_blocks_dw   : host array [n_dw] of X blocks [M_blk, H_blk];  dw_partials: host array [n_dw] of
 *                   fp32 outputs [H_blk, F_blk];  dw_partials[k] = x_blocks_dw[k]^T da_own.
 *   n_dx, n_dw    : 0 (skip that pass) .. the map's step count.
 *   workspace     : >= max over the passes used of tp_linear_workspace_size(.., TP_PASS_D?_PARTIALS).
 * Outputs are fp32 (they are summands of a reduction): TP_ERR_DTYPE otherwise.  The output blocks of
 * one call must not overlap each other (their byte ranges [ptr, ptr + ((rows - 1) ld + cols) 4) are
 * compared pairwise): TP_ERR_SHAPE otherwise.
 * Defined by: Section 3.1, Table 1 (2D, 2.5D rows) read with Section 2.2's chunk shapes.
 */
int tp_linear_bwd_partials(const tp_grid_t* grid, const tp_dims_t* dims, int n_dx, int n_dw,
                           const tp_cblk_t* da_own,
                           const tp_cblk_t* w_blocks_dx, const tp_oblk_t* dx_partials,
                           const tp_cblk_t* x_blocks_dw, const tp_oblk_t* dw_partials,
                           void* workspace, size_t workspace_bytes, void* hip_stream);
int tp_linear_bwd_partials_ex(const tp_grid_t* grid, const tp_dims_t* dims, int n_dx, int n_dw,
                              const tp_cblk_t* da_own,
                              const tp_cblk_t* w_blocks_dx, const tp_oblk_t* dx_partials,
                              const tp_cblk_t* x_blocks_dw, const tp_oblk_t* dw_partials,
                              void* workspace, size_t workspace_bytes, void* hip_stream, const tp_plan_opts_t* opts);

/*
 * tp_bias_act -- what follows the summation of forward partials (1D_ROW and 3D_GATHERED outputs
 * after their reduction):  A = c + bias,  y = GeLU(A) (epi TP_EPI_BIAS_GELU) or A (TP_EPI_BIAS) or c
 * (TP_EPI_NONE: a dtype conversion).  c: fp32 [rows, cols] with leading dimension ld_c; bias: bf16
 * [cols] or NULL with TP_EPI_NONE; y: fp32 or bf16; preact: optional bf16 copy of A.  cols and every
 * ld multiples of 8.  HBM-bound.
 * Defined by: Section 2.2, 1D paragraph (every device holds a partial output and an all-reduce
 * completes it) and the 3D chunk shape [P/p^2, Q/p]: what is applied to the rank's chunk once the sum
 * exists.  Errors: TP_ERR_NULL, TP_ERR_MODE, TP_ERR_SHAPE, TP_ERR_ALIGN, TP_ERR_DTYPE, TP_ERR_HIP.
 */
int tp_bias_act(const void* c, int64_t ld_c, const void* bias, int epi, tp_oblk_t y, tp_oblk_t preact,
                int64_t rows, int64_t cols, void* hip_stream);

/*
 * tp_dgelu -- the elementwise part of backward on its own:  da = bf16(dy * GeLU'(preact)),
 * all three bf16 [rows, cols] row-major with their own leading dimensions.  HBM-bound.
 * Defined by: the derivative of the erf-GeLU of tp_linear_fwd, GeLU'(a) = Phi(a) + a phi(a), applied to
 * a rank's own block of the output gradient (the chunk [P/q, Q/q], [P/(q d), Q/q] or [P/p^2, Q/p] of
 * Section 2.2).  Errors: TP_ERR_NULL, TP_ERR_SHAPE, TP_ERR_ALIGN, TP_ERR_HIP.
 */
int tp_dgelu(const void* dy, int64_t ld_dy, const void* preact, int64_t ld_pre,
             void* da, int64_t ld_da, int64_t rows, int64_t cols, void* hip_stream);

/*
 * tp_bias_grad -- db = 1^T dA: column sums of a bf16 block [rows, cols] (leading dimension ld) into
 * fp32 [cols], in a summation order fixed by (rows, cols) alone (the same bits on every call).  This is
 * what tp_linear_bwd writes to db_f32 for the block it forms itself; here for a dA block that already
 * exists (the 1D chain, where dA is the epilogue of the second layer's dX).  HBM-bound.
 *   workspace : optional device scratch of >= tp_bias_grad_workspace_size(rows, cols) bytes, 16-byte
 *               aligned: the rows are then summed in slabs by many workgroups and the slab sums added
 *               in ascending order by a second kernel.  NULL: one workgroup per 64 columns sums all
 *               rows (slow when cols is small).  The two forms add in different orders and may differ
 *               in the last bits; each is reproducible.  Too small or misaligned: TP_ERR_WORKSPACE.
 * Defined by: the bias gradient of the layer of tp_linear_fwd for one column chunk of the bias
 * (Section 2.2 chunking of the output columns).
 * Errors: TP_ERR_NULL, TP_ERR_SHAPE, TP_ERR_ALIGN, TP_ERR_WORKSPACE, TP_ERR_HIP.
 */
int tp_bias_grad(const void* da, int64_t ld_da, int64_t rows, int64_t cols, void* db_f32,
                 void* workspace, size_t workspace_bytes, void* hip_stream);
/* Bytes of workspace the slab form of tp_bias_grad wants (0: it would not split the rows).  Host only. */
size_t tp_bias_grad_workspace_size(int64_t rows, int64_t cols);

/* Human-readable name of a status code (static storage). */
const char* tp_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* TP_LINEAR_H */
