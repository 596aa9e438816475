/*
 * sparse_vdit.h - C ABI of the MI355X (gfx950) sparse 3D-attention forward of
 * Sparse-vDiT (arxiv 2506.03065).
 *
 * What the library computes.  For every batch entry b and head h of one
 * attention layer, with Q, K, V of shape [B, H, L, D]:
 *
 *     O[b,h,i,:] = sum_{j in kept_h(i)} softmax_j( Q[b,h,i,:].K[b,h,j,:] / sqrt(D) ) V[b,h,j,:]
 *
 * (Section 3, Eq. 1, restricted to the kept part of the attention map as in
 * Section 3 "Sparse Attention" and Section 4.2 "Sparse Computation
 * Pre-definition").  kept_h(i) depends on the head's mode M_0..M_4
 * (Section 4.2) and its parameters (Section 4.1.2):
 *
 *     0 dense          every key j
 *     1 skip           no key; the head's output is all zeros (Section 4.2)
 *     2 diagonal       |j - i| <= half_width
 *     3 multi-diagonal exists o in offsets: |j - i - o| <= half_width
 *     4 vertical       j in cols
 *
 * The softmax is renormalised over the kept keys.  Heads of one layer that
 * share a mode are fused into one kernel launch (Section 4.2, last paragraph).
 * The per-head mode table is an input of the forward pass.  Around it the
 * library also offers: one layer of the offline search that produces the table
 * (Section 4.2, Eq. 2-3, Algorithm 1: svd_search_layer and its parts), an FP8
 * variant of the forward pass (Appendix B: svd_attn_forward_fp8), dense borders
 * for a text prefix (Section 4.1.1: plan option text_tokens), and the
 * multi-diagonal mode in rearranged form (Section 4.1.2: head parameters
 * rearr_*, svd_rearrange_tokens).
 *
 * Conventions for every entry point
 *  - Tensors q, k, v, out are DEVICE pointers to bf16 (bfloat16) data described
 *    by one svd_tensor_desc: element strides for the B, H and L axes, the D axis
 *    is contiguous; every row start must be 16-byte aligned (base pointer and
 *    strides multiples of 8 elements).  q, k, v are read only; out is fully
 *    overwritten for every head (zeros for skipped heads).
 *  - strategy_table and pattern_params are HOST pointers; they are read during
 *    the call and not kept.  The same table applies to every batch entry.
 *  - The library never allocates or frees device memory and never synchronises
 *    the device (svd_search_layer excepted, which returns results to the host).  Plans place their index lists in a caller-provided DEVICE
 *    workspace that must stay alive and untouched while the plan is in use.
 *  - hip_stream is a hipStream_t passed as void* (NULL = the default stream).
 *    Kernels are enqueued on it and the call returns without waiting.
 *  - Every function returns an svd_status.  Arguments are validated on the host
 *    before anything is enqueued; on error nothing is launched and out is left
 *    untouched.  No exception or abort crosses this boundary.
 */
#ifndef SPARSE_VDIT_H
#define SPARSE_VDIT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t svd_status;
enum {
  SVD_OK = 0,
  SVD_ERR_NULL = 1,          /* a required pointer is NULL */
  SVD_ERR_SHAPE = 2,         /* B, H, L < 1, D not 64 or 128, bad group/list index */
  SVD_ERR_DTYPE = 3,         /* reserved: only bf16 exists */
  SVD_ERR_ALIGN = 4,         /* pointer or stride breaks the 16-byte row alignment */
  SVD_ERR_MODE = 5,          /* mode id outside 0..4 */
  SVD_ERR_PARAMS = 6,        /* negative width, no/duplicate offsets, column out of range or duplicate */
  SVD_ERR_EMPTY_PATTERN = 7, /* some query row would keep no key */
  SVD_ERR_WORKSPACE = 8,     /* workspace missing or too small */
  SVD_ERR_UNSUPPORTED = 9,   /* block shape the kernels do not implement, or a tensor beyond the size limits */
  SVD_ERR_HIP = 10,          /* a HIP call (copy, launch) failed */
  SVD_ERR_STATIC_LIMIT = 11  /* sparse_vdit_attn_forward_static: the layer does not fit the library's static buffer */
};

/* Mode ids = M_0..M_4 of Section 4.2, sparse modes in the order of Section 4.1.2. */
enum { SVD_DENSE = 0, SVD_SKIP = 1, SVD_DIAG = 2, SVD_MULTIDIAG = 3, SVD_VSTRIPE = 4 };

typedef struct {
  int32_t B, H, L, D;                     /* D in {64, 128} */
  int64_t stride_b, stride_h, stride_l;   /* in elements; the D axis has stride 1 */
} svd_tensor_desc;
/* Size limits (SVD_ERR_UNSUPPORTED beyond them): the rows of one head span less
 * than 4 GiB (L * stride_l * 2 < 2^32), L < 2^24, and a row stride below 16 MiB. */

/* Parameters of one head (pattern_params is an array of H of these).  Only the
 * fields of the head's mode are read. */
typedef struct {
  int32_t half_width;        /* w in tokens, modes 2 and 3; the band is inclusive: 2w+1 diagonals */
  int32_t n_offsets;         /* mode 3: number of band centres */
  const int32_t* offsets;    /* mode 3: band centres o (key index minus query index), any order, host */
  int32_t n_cols;            /* mode 4: number of key columns */
  const int32_t* cols;       /* mode 4: key columns in [0, L), any order, no duplicates, host */
  /* mode 3 in rearranged form (Section 4.1.2: "by rearranging tokens" the evenly
   * spaced diagonals become one diagonal band).  rearr_frames = F > 0 selects it:
   * the video block is F frames of rearr_frame_tokens = N tokens starting at token
   * rearr_first, frame f and position p at rearr_first + f*N + p; with pi the move
   * to position-major order (rearr_first + p*F + f, other tokens unmoved) the head
   * keeps (i, j) iff |pi(i) - pi(j)| <= half_width.  half_width = w*F + F - 1 keeps
   * every pair of positions at most w apart, in any two frames.  offsets are not
   * read.  The kernels walk the band in the rearranged order and reach the rows of
   * q, k, v and out through a row map; nothing is copied (the FP8 variant writes
   * its quantised keys and values in the rearranged order).  Not combined with a
   * text prefix (SVD_ERR_UNSUPPORTED); SVD_ERR_PARAMS when the video block does
   * not fit L.  F = 0: the head is a plain multi-diagonal head. */
  int32_t rearr_first, rearr_frame_tokens, rearr_frames;
} svd_head_params;

/* Plan options (a NULL pointer or zeros select the defaults).
 * block_q x block_k: block shape of the key-block lists, block_q query rows by
 * block_k keys; 0 selects the shape the kernels run for the given D.  A plan
 * compiled with another shape can be inspected but not launched.
 * dense_split: key-range chunks per query tile of the dense heads.  A work-group
 * occupies a whole compute unit, so few long dense items leave the last round
 * of work-groups partly empty; splitting the key range makes the rounds shorter
 * at the price of a merge pass over partial results kept in the workspace.
 * 0 = chosen from the shape and the device's compute-unit count, 1 = off,
 * 2..8 = forced (capped at the number of key tiles).
 * text_tokens: Section 4.1.1 describes the attention map of a sequence of text
 * and video tokens as four regions, T-T, T-V, V-T and V-V, and the sparse
 * patterns for V-V.  With text_tokens = T > 0 the first T tokens are text and
 * every head in a sparse mode (diagonal, multi-diagonal, vertical-stripe) keeps
 * the three border regions whole: key j < T for every query, every key for
 * query i < T; bands are still taken on the global token index.  T must be
 * smaller than L and a multiple of block_q and of block_k (256 for the kernels'
 * shapes), else SVD_ERR_UNSUPPORTED.  The band lists of the text query blocks
 * are then empty (their rows come from a dense launch over the group's heads),
 * the other query blocks list the text tiles first, and the column lists gain
 * columns 0..T-1.  0 = no text prefix.  sparse_vdit_attn_forward takes no
 * options and therefore no text prefix.
 * single_launch: Section 4.2 fuses the heads that share a mode into one launch;
 * with single_launch = 1 the whole layer is ONE launch: resident work-groups (one
 * of eight waves per compute unit) pull (group, head, query tile) items off eight
 * work queues, one per XCD, heaviest group first, and move on to the other
 * queues when their own is empty, so no group pays for a partly filled last
 * round.  Every item runs on the kernels' 256-row query tile (one work-group of
 * eight waves per compute unit), dense heads are not split,
 * text rows of a text prefix are items of the dense
 * kind, and nothing is forked.  The queue positions are words of the plan
 * workspace that a small fill kernel zeroes ahead of the layer kernel (no
 * memset, so the call can be captured); with vertical-stripe heads the gather
 * pre-pass of their K and V rows runs ahead of it too.  Results are
 * bit-identical to the grouped launches of a plan with dense_split = 1.
 * 3 = the single launch with a DENSE HEAD START: as many whole rounds of dense
 * items as there are (one work-group per compute unit and round, none partly
 * filled) first go through the dense kernel in a launch of its own; the rest of
 * the dense group and everything else is the layer kernel's.  Same bits.
 * 2 = grouped launches.  0 = the library's choice: form 1 for D = 128 when the
 * layer's items are long (48 key tiles per item or more, averaged over the heads
 * that compute: picking an item costs a few microseconds), grouped launches
 * otherwise - for D = 64 (there they measure 2-8 % faster than both forms), for
 * short items, whenever dense_split > 1 is forced,
 * the block shape is not the kernels' or no device is present.  1 and 3
 * need the kernels' block shape (SVD_ERR_UNSUPPORTED otherwise) and a device
 * (SVD_ERR_HIP).  The split of the dense heads is still chosen and its scratch
 * still part of the workspace: the FP8 forward pass and the per-group entry
 * points run such a plan group by group.
 * no_fork: 1 = grouped launches always run one after the other on the caller's
 * stream (see svd_attn_forward_planned); 0 = the library forks them onto its own
 * streams when that fills an otherwise idle last round. */
typedef struct { int32_t block_q, block_k, dense_split, text_tokens, single_launch, no_fork; } svd_plan_options;

typedef struct svd_plan svd_plan;

/* Block shape the kernels use for head dimension D (the default of the plan
 * options).  D must be 64 or 128. */
svd_status svd_default_blocks(int32_t D, int32_t* block_q, int32_t* block_k);

/* Bytes of device workspace a plan for this layer needs: the compiled lists plus,
 * when the dense heads are split, the scratch of their partial results.  Reads
 * the current device's compute-unit count when dense_split is 0 (no device: no
 * split); touches no device memory. */
svd_status svd_plan_workspace_bytes(const svd_tensor_desc* desc, const int32_t* strategy_table,
                                    const svd_head_params* pattern_params,
                                    const svd_plan_options* options, size_t* bytes);

/* Pattern compiler (Section 4.2: head fusion + block-level sparsity).  Groups the
 * heads by mode, builds for every distinct band pattern the CSR list of key
 * blocks per query block and for every distinct column set the padded sorted
 * column list, and copies them to device_workspace on hip_stream (the copy has
 * completed when the call returns).  With device_workspace == NULL the plan is
 * host-only: it can be inspected but svd_attn_forward_planned refuses it.
 * options may be NULL.  The plan is released with svd_plan_destroy. */
svd_status svd_plan_create(svd_plan** plan, const svd_tensor_desc* desc,
                           const int32_t* strategy_table, const svd_head_params* pattern_params,
                           const svd_plan_options* options, void* device_workspace,
                           size_t workspace_bytes, void* hip_stream);
svd_status svd_plan_destroy(svd_plan* plan);

/* Key-range chunks per dense query tile this plan launches (1 = no split; always
 * 1 for host-only plans). */
svd_status svd_plan_dense_split(const svd_plan* plan, int32_t* dense_split);

/* How svd_attn_forward_planned runs this plan (Section 4.2, fusion of heads; plan
 * option single_launch): 1 = the layer kernel alone, 3 = the
 * layer kernel after the dense head start (plan option single_launch, or the
 * library's choice), 0 = a launch per group. */
svd_status svd_plan_single_launch(const svd_plan* plan, int32_t* single_launch);

/* Inspection of a compiled plan (host copies owned by the plan, valid until
 * svd_plan_destroy).  Groups are ordered by ascending mode id. */
svd_status svd_plan_num_groups(const svd_plan* plan, int32_t* n_groups);
/* Block shape of one group's lists and launches.  block_k is the plan's; block_q
 * is the plan's too, except for a band group (modes 2, 3) of a plan created
 * without an explicit block shape: when its lists cover at least 8 % less area
 * with the kernels' small query tile (128 rows instead of 256: the listed tiles
 * hug the bands more closely, and two work-groups share a compute unit; the
 * large tile is the faster one per listed FLOP), the group is compiled and
 * launched with it - always, in a plan that runs through the layer kernel.
 * svd_plan_band_list reports the matching number of query blocks. */
svd_status svd_plan_group_blocks(const svd_plan* plan, int32_t group, int32_t* block_q, int32_t* block_k);
/* (Rearranged multi-diagonal heads form a group of their own, after the plain
 * multi-diagonal group; both report mode 3, svd_plan_group_rearranged tells them
 * apart.) */
svd_status svd_plan_group_rearranged(const svd_plan* plan, int32_t group, int32_t* rearranged);
/* heads: ascending head ids of the group; list_id[t]: which list of the group
 * head heads[t] uses (heads with the same kept region share a list; ids are
 * numbered by first appearance); n_lists is 0 for dense and skip groups. */
svd_status svd_plan_group_info(const svd_plan* plan, int32_t group, int32_t* mode, int32_t* n_heads,
                               const int32_t** heads, const int32_t** list_id, int32_t* n_lists);
/* A list of a band group (modes 2, 3).  row_ptr[n_q_blocks+1] is the CSR
 * pointer; for entry e: kv_block_idx[e] (ascending inside a query block),
 * flags[e] = 1 if the whole block_q x block_k tile is kept for every in-range
 * query row and lies inside [0, L) (no masking needed), else 0.  runs[2*r],
 * runs[2*r+1] = inclusive bounds of the r-th maximal run of kept diagonals
 * (key index minus query index) inside [-(L-1), L-1]; run_first[e] and
 * run_count[e] name the consecutive runs that have a kept element in tile e. */
svd_status svd_plan_band_list(const svd_plan* plan, int32_t group, int32_t list,
                              int32_t* n_q_blocks, const int32_t** row_ptr,
                              const int32_t** kv_block_idx, const int32_t** flags,
                              const int32_t** run_first, const int32_t** run_count,
                              int32_t* n_runs, const int32_t** runs);
/* The row map of a list of a rearranged multi-diagonal group: row_map[r] = original
 * row of position r of the rearranged order, padded with -1 to padded_len, a
 * multiple of block_k; the lists of such a group (svd_plan_band_list) are those of
 * the plain band in the rearranged order.  SVD_ERR_SHAPE for other groups. */
svd_status svd_plan_row_map(const svd_plan* plan, int32_t group, int32_t list, int32_t* padded_len,
                            const int32_t** row_map);
/* A list of a vertical-stripe group (mode 4): the sorted unique columns padded
 * with -1 to padded_len, a multiple of block_k. */
svd_status svd_plan_column_list(const svd_plan* plan, int32_t group, int32_t list,
                                int32_t* n_cols, int32_t* padded_len, const int32_t** cols);
/* Work the plan launches per forward pass, summed over batch and heads:
 * computed_tiles counts block_q x block_k tiles (dense heads: all of them,
 * vertical heads: column tiles), computed_flops = 4 * D * (tile area inside
 * [0,L) x [0,L) or the column list) and kept_pairs the element-level count. */
svd_status svd_plan_work(const svd_plan* plan, int64_t* computed_tiles, double* computed_flops,
                         double* kept_pairs);

/* The same figures for one group (all its heads, all batch entries). */
svd_status svd_plan_group_work(const svd_plan* plan, int32_t group, int64_t* computed_tiles,
                               double* computed_flops, double* kept_pairs);

/* The work of the FP8 forward pass (svd_attn_forward_fp8, the Appendix B variant): its band groups always walk
 * small-tile lists (kept in the plan beside the lists of a group that the bf16
 * kernels run on the large tile), so their tile count and listed area can differ
 * from svd_plan_group_work.  group = -1: the whole layer. */
svd_status svd_plan_group_work_fp8(const svd_plan* plan, int32_t group, int64_t* computed_tiles,
                                   double* computed_flops);

/* Forward pass of one layer with a compiled plan (Section 4.2: one fused launch
 * per mode present in the table, heaviest group first, plus a zero fill for
 * skipped heads).  The tensors must match the plan's descriptor.  The group
 * kernels are independent.  Normally they are enqueued one after the other on
 * hip_stream.  When the last round of work-groups of the heaviest group would
 * leave more than half of the compute units idle, the groups are instead forked
 * from hip_stream onto streams owned by the plan, run concurrently, and are
 * joined on hip_stream before the call returns; either way everything is
 * ordered on hip_stream for the caller.  One forward pass per plan may be in
 * flight at a time (calls with the same plan on one stream are fine; concurrent
 * calls on different streams need different plans).  The plan option no_fork
 * disables the fork.  Only kernel launches and
 * event records/waits are enqueued, so the call may be recorded into a stream
 * capture - except for a plan with a text prefix: while hip_stream is capturing,
 * such a plan is refused with SVD_ERR_UNSUPPORTED before anything is enqueued
 * (this holds for every forward entry point that takes a plan). */
svd_status svd_attn_forward_planned(const svd_plan* plan, const void* q, const void* k, const void* v,
                                    void* out, void* hip_stream);

/* The launch of a single group of the plan (Section 4.2: the fused kernel of one
 * mode).  Writes only the heads of that group.  For callers that place groups
 * on different streams or time them one by one. */
svd_status svd_attn_forward_group(const svd_plan* plan, int32_t group, const void* q, const void* k,
                                  const void* v, void* out, void* hip_stream);

/* One-shot form: compiles the table (or reuses the plan compiled by the previous
 * call with identical arguments and workspace) and launches.  workspace_bytes
 * must be at least svd_plan_workspace_bytes(...). */
svd_status sparse_vdit_attn_forward(const void* q, const void* k, const void* v,
                                    const int32_t* strategy_table,
                                    const svd_head_params* pattern_params, void* out,
                                    const svd_tensor_desc* desc, void* device_workspace,
                                    size_t workspace_bytes, void* hip_stream);

/* The one-shot form for callers that cannot allocate device memory or hand over a
 * workspace: code running under HIP stream capture, tight serving loops, harnesses
 * that forbid hipMalloc.  Same result as sparse_vdit_attn_forward, but the
 * compiled lists and the partial results of split dense heads live in a buffer of
 * SVD_STATIC_SCRATCH_BYTES (64 MiB) that is part of the library's device image
 * (as are the gathered rows of stripe heads and the layer kernel's queue positions):
 * every GPU the library runs on holds its own copy until the process ends.  The
 * call allocates no device memory and creates no streams or events; the groups of
 * the layer run one after the other on hip_stream.  A layer whose split dense
 * heads do not fit the buffer runs them unsplit; a layer whose lists alone do not
 * fit is refused with SVD_ERR_STATIC_LIMIT (nothing is enqueued).  The plan of the
 * previous call on the device is reused when table, parameters and descriptor are
 * identical; otherwise the new lists are copied into the buffer on hip_stream and
 * the call waits for that copy - which a capturing stream cannot record
 * (SVD_ERR_UNSUPPORTED), so the first call for a layer belongs before the capture.
 * All calls on one GPU share the buffer, and it keeps what the last call left in
 * it; the one thing that must start at zero, the queue positions of the layer
 * kernel, is cleared by a fill kernel in every call, and the gathered K/V rows of
 * vertical-stripe heads are rewritten by every call.  Calls that overlap in time
 * on one GPU race, whatever their streams.  No text prefix (the call takes no options). */
#define SVD_STATIC_SCRATCH_BYTES (64u << 20)
svd_status sparse_vdit_attn_forward_static(const void* q, const void* k, const void* v,
                                           const int32_t* strategy_table,
                                           const svd_head_params* pattern_params, void* out,
                                           const svd_tensor_desc* desc, void* hip_stream);

/* Eq. 1 for all H heads with the same kernel family: the dense baseline the
 * sparse layer's speed-up is measured against.  Needs no workspace. */
svd_status svd_dense_attn_forward(const void* q, const void* k, const void* v, void* out,
                                  const svd_tensor_desc* desc, void* hip_stream);

/* ---- Offline search step (Section 4.2 "Offline Sparse Diffusion Search", Eq. 2-3,
 * Algorithm 1): all five modes run on the same Q, K, V; per head and sparse mode
 * i = 1..4 the loss is L_i = MSE(O_i - O_0) + lambda * (1 - S_i) (Eq. 2; the
 * listing of Algorithm 1 prints lambda * S_i, the equation and its text are
 * followed); a head keeps mode 0 when all four losses exceed epsilon, else it
 * takes the arg-min mode, lower id on ties (Eq. 3). ---- */

/* Bytes of device scratch svd_head_mse needs for this shape.  Host only. */
svd_status svd_head_mse_workspace_bytes(const svd_tensor_desc* desc, size_t* bytes);

/* MSE(O_i - O_0) per head: mse[h] = mean over batch, tokens and channels of
 * (o - o_ref)^2.  o, o_ref: DEVICE bf16 tensors of layout desc; mse: DEVICE
 * float[H]; device_workspace: DEVICE scratch of svd_head_mse_workspace_bytes.
 * Two kernels with a fixed summation order (same bits on every run); enqueued
 * on hip_stream, no synchronisation. */
svd_status svd_head_mse(const void* o, const void* o_ref, const svd_tensor_desc* desc, float* mse,
                        void* device_workspace, size_t workspace_bytes, void* hip_stream);

/* S_i of Eq. 2 for every head of a plan: the share of the L x L attention map the
 * head's mode leaves out (0 dense, 1 skip, element-level count for the patterns:
 * this library's reading, since the block size of the paper's kernels is not
 * given and an element count does not depend on one).
 * sparsity: HOST double[H]. */
svd_status svd_plan_head_sparsity(const svd_plan* plan, double* sparsity);

/* The block-level count of the same quantity, in the wording of Section 4.2 ("the
 * ratio of actual computation blocks to the total number of blocks"): 1 minus the
 * number of block_q x block_k tiles the head's launches compute over the number
 * of tiles of the map, on the tile shape of the head's group (a tile that holds
 * one kept pair counts whole, the text rows of a text prefix count as dense
 * tiles).  It depends on the tile shape; the element-level figure above is its
 * limit for small tiles and is what svd_search_layer uses for S_i.
 * sparsity: HOST double[H]. */
svd_status svd_plan_head_block_sparsity(const svd_plan* plan, double* sparsity);

/* Eq. 2 and Eq. 3 on the host.  mse (float) and sparsity (double) are HOST arrays
 * of 4 * H values, row i - 1 = mode i; table: HOST int32[H], out; loss: HOST
 * double[4 * H], out, may be NULL. */
svd_status svd_search_select(int32_t H, const float* mse, const double* sparsity, double lambda, double epsilon,
                             int32_t* table, double* loss);

/* x^o of Algorithm 1: out[:, h] = o_modes[table[h]][:, h].  o_modes: HOST array of
 * five DEVICE tensors of layout src_desc (entries of modes the table does not use
 * may be NULL); table: HOST int32[H]; out: DEVICE tensor of layout out_desc (same
 * shape).  H <= 1024. */
svd_status svd_select_heads(const void* const* o_modes, const svd_tensor_desc* src_desc, const int32_t* table,
                            void* out, const svd_tensor_desc* out_desc, void* hip_stream);

/* One layer of the search (the loop body of Algorithm 1 between "Attention Part"
 * and "FFN Part").  params_by_mode: HOST array of five pointers, entries 2, 3, 4 =
 * the H candidate parameter sets of the diagonal, multi-diagonal and vertical
 * mode (entries 0, 1 unused).  Runs mode i on all heads for i = 0..4 with the
 * library's kernels, reduces the four MSEs, applies Eq. 2-3, writes the chosen
 * outputs to out and returns table (HOST int32[H]) and loss (HOST double[4 * H],
 * may be NULL).  q, k, v, out must be contiguous [B, H, L, D].  device_workspace:
 * svd_search_layer_workspace_bytes bytes, 256-byte aligned (five output tensors +
 * one plan + scratch).  Unlike the forward entry points this call SYNCHRONISES
 * hip_stream: the losses are needed on the host. */
svd_status svd_search_layer_workspace_bytes(const svd_tensor_desc* desc,
                                            const svd_head_params* const* params_by_mode, size_t* bytes);
svd_status svd_search_layer(const void* q, const void* k, const void* v, const svd_tensor_desc* desc,
                            const svd_head_params* const* params_by_mode, double lambda, double epsilon,
                            int32_t* table, double* loss, void* out, void* device_workspace,
                            size_t workspace_bytes, void* hip_stream);

/* ---- Token rearrangement (Section 4.1.2, multi-diagonal pattern) ----
 * Video tokens are ordered frame by frame (Section 4.1.1); the evenly spaced
 * diagonals of the multi-diagonal pattern are attention between nearby spatial
 * positions of different frames, and the paper notes that rearranging the tokens
 * turns them into one diagonal band that window attention computes.  This call
 * is that rearrangement: with F = frames frames of N = frame_tokens tokens
 * starting at token first_video_token, the token of frame f and position p moves
 * from row first + f*N + p to row first + p*F + f (inverse != 0: back); rows
 * outside the video block are copied unchanged.  A caller rearranges q, k and v,
 * runs the diagonal mode with half width w*F + F - 1 on them (every pair of
 * positions at most w apart, in any two frames) and rearranges the output back.
 * src, dst: DEVICE bf16 tensors of layout desc, distinct and not overlapping
 * (SVD_ERR_UNSUPPORTED for src == dst).  SVD_ERR_PARAMS when the video block does
 * not fit L.  One streaming kernel on hip_stream; no synchronisation, no
 * allocation. */
svd_status svd_rearrange_tokens(const void* src, void* dst, const svd_tensor_desc* desc, int32_t first_video_token,
                                int32_t frame_tokens, int32_t frames, int32_t inverse, void* hip_stream);

/* ---- FP8 variant (Appendix B, Table 4: "Sparse-vDiT + FP8") ----
 * The paper combines the sparse kernels with FP8 quantisation but gives no
 * recipe.  This library's reading: OCP E4M3 operands with fixed power-of-two
 * scales, Q8 = e4m3(q * 4 log2(e) / sqrt(D)) (product in fp32), K8 = e4m3(k / 4),
 * V8 = e4m3(v), P8 = e4m3(2^(Q8.K8 - m)) with the integer reference
 * m = ceil(row max) - 8; values beyond +-448 saturate; scores, row sums and the
 * output accumulate in fp32, the output is rounded to bf16.  Masks, modes and
 * the plan are those of the bf16 path.
 *
 * svd_attn_forward_fp8: the layer of svd_attn_forward_planned in this
 * arithmetic.  q, k, v, out: DEVICE bf16 tensors of the plan's descriptor.
 * fp8_workspace: DEVICE scratch of svd_fp8_workspace_bytes(desc) bytes, 256-byte
 * aligned, owned by the caller; the call fills it with the quantised keys and
 * values of the layer (first half K8 [B][H][Lp][D] bytes, Lp = L rounded up to a
 * multiple of 128; second half V8 [B][H][Lp/64][D][64], byte 32*h + 16*b + 4*g + r
 * of a 64-byte record = key 32*b + 8*g + 4*h + r of the group of 64; keys past
 * the head's key count are zero; a vertical-stripe head's arrays hold its listed
 * columns in list order) and reads it back; nothing is kept between calls.  All
 * launches go to hip_stream in order; the call does not synchronise and
 * allocates nothing.  Errors as for svd_attn_forward_planned, plus
 * SVD_ERR_WORKSPACE for a missing, small or misaligned fp8_workspace. */
svd_status svd_fp8_workspace_bytes(const svd_tensor_desc* desc, size_t* bytes);
svd_status svd_attn_forward_fp8(const svd_plan* plan, const void* q, const void* k, const void* v, void* out,
                                void* fp8_workspace, size_t fp8_workspace_bytes, void* hip_stream);
/* One group of the plan in the FP8 arithmetic (pre-pass of the group's heads,
 * attention, merge of a split dense launch), as svd_attn_forward_group is to
 * svd_attn_forward_planned.  SVD_ERR_SHAPE for a group index out of range. */
svd_status svd_attn_forward_fp8_group(const svd_plan* plan, int32_t group, const void* q, const void* k,
                                      const void* v, void* out, void* fp8_workspace, size_t fp8_workspace_bytes,
                                      void* hip_stream);

/* ---- Calibration probes for the benchmark's roofline (no part of the method) ----
 * The published matrix peak assumes the peak clock; under load the power limit
 * grants less.  svd_probe_mfma runs a loop of nothing but the bf16 matrix
 * instruction of the attention kernels' two products (v_mfma_f32_32x32x16_bf16,
 * eight independent accumulators per wave, each with pseudo-random operands of
 * its own, work_groups of 512 threads, two waves per SIMD) and returns the FLOPs of the launch through *flops (HOST); timing is
 * the caller's.  device_scratch: DEVICE, work_groups * 512 floats at least.
 * svd_probe_copy copies bytes (a multiple of 16) from src to dst (DEVICE, 16-byte
 * aligned, not overlapping) with one plain streaming kernel: bytes read and bytes
 * written of known size, for the HBM ceiling and for scaling hardware counters. */
svd_status svd_probe_mfma(void* device_scratch, size_t scratch_bytes, int32_t iters, int32_t work_groups,
                          double* flops, void* hip_stream);
svd_status svd_probe_copy(const void* src, void* dst, size_t bytes, void* hip_stream);

/* Static, human-readable name of a status code. */
const char* svd_status_string(svd_status status);

#ifdef __cplusplus
}
#endif
#endif /* SPARSE_VDIT_H */
