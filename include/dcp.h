/*
 * dcp.h -- C ABI of libdcp_attn.so: the per-device hot path of Dynamic Context Parallelism
 * (DCP): blockwise attention over packed variable-length sequences driven by a block table,
 * the LSE-carrying merge of partial outputs, and the backward pass, for AMD gfx950.
 *
 * General rules
 *   - Every function returns a dcp_status_t; nothing throws across this boundary.  On any
 *     error no kernel is launched and no output is touched; dcp_last_error() then returns a
 *     human-readable message (thread-local storage owned by the library).
 *   - "host" pointers are read during the call and may be freed on return.  "device" pointers
 *     are HIP device memory owned by the caller; the library never frees or keeps them.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).  Launching calls only
 *     enqueue work on it and return without synchronising, with one exception: the first launch
 *     that uses a plan (or a copy list) on a device uploads its integer arrays, which allocates
 *     device memory and waits for the stream once; dcp_plan_prepare does that ahead of time.
 *     A launch writes nothing into the plan: several streams may run one (prepared) plan at the same time on
 *     tensors and workspaces of their own.
 *   - Tensors: q, out, dout, dq are [T, Hq, D]; k, v, dk, dv are [T, Hkv, D]; D is contiguous;
 *     token and head strides are given in elements.  lse and delta are float [Hq, T] contiguous.
 *     Query head h reads KV head h / (Hq / Hkv).  T = cu_seqlens[n_seq] packed tokens.
 *
 * Block numbering (Sec. 4.1 "Block Generation" of the paper): sequence s with L_s tokens is
 * cut into ceil(L_s / block_size) data blocks, the last possibly short; blocks never straddle
 * sequences; global block id = (blocks of earlier sequences) + index inside the sequence.
 * A block-table row (q_blk, kv_blk, mask_kind) is one computation block of Sec. 4.1: the attention
 * of query block q_blk against key-value block kv_blk, whose result belongs to output block q_blk.
 * It applies to every head.  The table DEFINES the mask: a (query, key) pair is visible iff a listed
 * row covers it and the row's predicate holds; pairs not listed are not visible.
 */
#ifndef DCP_H_
#define DCP_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  DCP_OK = 0,
  DCP_ERR_INVALID_ARG = -1,    /* NULL pointer, negative size, bad stride, missing ranges ...   */
  DCP_ERR_BAD_CU_SEQLENS = -2, /* cu_seqlens[0] != 0 or not strictly increasing                 */
  DCP_ERR_BAD_TABLE = -3,      /* block id out of range, blocks of two sequences, duplicate row, */
                               /* bad mask_kind, RANGES and WINDOW rows together, inconsistent   */
                               /* output slot                                                    */
  DCP_ERR_UNSUPPORTED = -4,    /* head_dim / dtype / head ratio no kernel covers                 */
  DCP_ERR_WORKSPACE = -5,      /* workspace NULL or too small                                    */
  DCP_ERR_HIP = -6             /* a HIP runtime call failed (message holds hipGetErrorString)    */
} dcp_status_t;

/* Predicate of one table row for query i and key j of the same sequence:
 *   NONE   every pair of the tile is visible;
 *   CAUSAL visible iff position(j) <= position(i);
 *   RANGES visible iff packed index of j lies in [r[i][0], r[i][1]) or [r[i][2], r[i][3]) -- the
 *          per-token range arrays of Sec. 5 "Blockwise Attention" (no more than two ranges for a
 *          token); r is int32 [T, 4], packed-token coordinates, half open, an empty range has
 *          hi <= lo;
 *   SKIP   never (the row is ignored);
 *   WINDOW sliding window with an attention sink (the lambda-shaped mask of Sec. 2.4; sink 0 gives
 *          the plain sliding window): visible iff j <= i and (i - j < window or j is one of the
 *          first `sink` tokens of the sequence).  window and sink are two numbers for the whole
 *          plan (dcp_plan_set_window); no range array is read.  A table holds RANGES rows or
 *          WINDOW rows, not both.                                                                */
typedef enum {
  DCP_MASK_NONE = 0, DCP_MASK_CAUSAL = 1, DCP_MASK_RANGES = 2, DCP_MASK_SKIP = 3, DCP_MASK_WINDOW = 4
} dcp_mask_kind_t;

typedef enum { DCP_BF16 = 0, DCP_F32 = 1 } dcp_dtype_t;

/* Which kernel family runs.  AUTO picks MFMA when (dtype, D) is covered, else SCALAR. */
typedef enum { DCP_IMPL_AUTO = 0, DCP_IMPL_SCALAR = 1, DCP_IMPL_MFMA = 2 } dcp_impl_t;

typedef struct dcp_plan dcp_plan_t; /* opaque; created and destroyed by the library */

/* ---------------------------------------------------------------------------------------------
 * Block generation (Sec. 4.1): from per-token range arrays build the block table.  A computation
 * block is emitted for every same-sequence (q_blk, kv_blk) whose mask tile is not all zeros
 * (fully masked tiles get no computation block), classified NONE (all ones), CAUSAL (tile equals the
 * causal predicate) or RANGES, in ascending (q_blk, kv_blk) order.
 *   cu_seqlens_host  host int32[n_seq+1]
 *   attn_ranges_host host int32[T,4]
 *   table_out        host int32[capacity,3] or NULL (count only)
 *   n_entries_out    receives the number of rows the full table has
 * Returns DCP_ERR_INVALID_ARG if capacity is too small (n_entries_out is still set).  Host only. */
dcp_status_t dcp_build_block_table(const int32_t* cu_seqlens_host, int32_t n_seq, int32_t block_size,
                                   const int32_t* attn_ranges_host, int32_t* table_out,
                                   int64_t capacity, int64_t* n_entries_out);

/* The same block generation for a sliding window of `window` keys (the query included) with `sink`
 * sink tokens per sequence, without range arrays: tiles that are neither all ones nor the causal
 * predicate are tagged WINDOW.  window >= 1, sink >= 0.  Other arguments and errors as above. */
dcp_status_t dcp_build_block_table_window(const int32_t* cu_seqlens_host, int32_t n_seq, int32_t block_size,
                                          int32_t window, int32_t sink, int32_t* table_out, int64_t capacity,
                                          int64_t* n_entries_out);

/* Visible (query, key) pairs of every table row taken alone (the unit of the paper's FLOP
 * accounting for a computation block, Sec. 4.2 vertex weights).  attn_ranges_host may be NULL if
 * no row is RANGES.  pairs_out: host int64[n_entries].  Host only. */
dcp_status_t dcp_count_pairs(const int32_t* cu_seqlens_host, int32_t n_seq, int32_t block_size,
                             const int32_t* table_host, int64_t n_entries,
                             const int32_t* attn_ranges_host, int64_t* pairs_out);

/* dcp_count_pairs for tables with WINDOW rows (a RANGES row is DCP_ERR_BAD_TABLE here). */
dcp_status_t dcp_count_pairs_window(const int32_t* cu_seqlens_host, int32_t n_seq, int32_t block_size,
                                    const int32_t* table_host, int64_t n_entries, int32_t window, int32_t sink,
                                    int64_t* pairs_out);

/* Block buffers (Sec. 5 "Block buffers", and "Blockwise Attention": input and output blocks are
 * given by the buffer's start address and per-block offsets recorded with the block table, as in
 * paged attention).  After this call the tensors of every launch with this plan are block buffers:
 *   q, out, dout, dq : [n_q_slots * block_size, Hq, D];  lse (and the backward workspace) : [Hq, n_q_slots * block_size]
 *   k, v, dk, dv     : [n_kv_slots * block_size, Hkv, D]
 * and row r of block b lives at row slot[b] * block_size + r of its buffer.  attn_ranges stays
 * indexed by packed token (it is mask metadata, not a data block), and so do the ranges it holds.
 *   q_slot, kv_slot  host int32 [n_blocks], copied; -1 = the block is not in that buffer
 * Blocks with q_slot -1 get no output (their rows do not exist); rows of the buffers that no block
 * owns are never read or written by the attention kernels.  dcp_bwd_delta works on whole buffers.
 * Must be called before the plan is first used on a device (DCP_ERR_INVALID_ARG otherwise).
 * DCP_ERR_BAD_TABLE: a slot out of range, two blocks in one slot, or a block the table uses
 * (as q_blk / kv_blk of a non-SKIP row) that is absent from the buffer it is needed in. */
dcp_status_t dcp_plan_set_block_buffers(dcp_plan_t* plan, const int32_t* q_slot_host, int32_t n_q_slots,
                                        const int32_t* kv_slot_host, int32_t n_kv_slots);

/* ---------------------------------------------------------------------------------------------
 * Plan: the executor's per-iteration state (Sec. 3.2: the plan is set once per iteration and
 * shared by all layers).  Validates the table, derives block token ranges, groups rows by output
 * (forward, dQ) and by kv_blk (dK/dV), and orders work longest-first.  Host work only; device
 * copies of the integer arrays are made on the first launch that needs them and freed by
 * dcp_plan_destroy.
 *   table_host    host int32[n_entries,3] rows (q_blk, kv_blk, mask_kind)
 *   out_slot_host host int32[n_entries] or NULL.  NULL: one output per q_blk, written to the
 *                 packed `out`/`lse`.  Otherwise row e accumulates into partial slot out_slot[e]
 *                 (0 <= slot < n_slots); all rows of a slot must share one q_blk (a slot is one of
 *                 the not-yet-reduced intermediate results that Sec. 5's block buffers hold),
 *                 merged later by dcp_merge_partials.
 * n_entries == 0 is legal.  Errors: BAD_CU_SEQLENS, BAD_TABLE, INVALID_ARG. */
dcp_status_t dcp_plan_create(dcp_plan_t** plan, const int32_t* cu_seqlens_host, int32_t n_seq,
                             int32_t block_size, const int32_t* table_host, int64_t n_entries,
                             const int32_t* out_slot_host, int32_t n_slots);
dcp_status_t dcp_plan_destroy(dcp_plan_t* plan);

/* Creates now what the launching calls would otherwise create at their first use of the plan: the device copy of the
 * plan's integer arrays and the work lists of the forward, dQ and dK/dV kernels that (dtype, d, impl) selects, for
 * hq / hkv heads, on the device that is current.  This is the one place that allocates device memory (hipMalloc)
 * and waits for `stream` (the upload of the arrays); after it, dcp_block_attn_fwd, dcp_block_attn_bwd and
 * dcp_merge_partials with this plan and shape only enqueue kernels.  Without it the first of those calls does the same
 * work itself, once.  Call it after dcp_plan_set_block_buffers, if that is used.  Errors as for the launching calls.
 * A prepared plan's launches are kernel launches and nothing else (no memset or copy nodes, no events), so they may
 * be recorded into a HIP graph by stream capture and replayed. */
dcp_status_t dcp_plan_prepare(dcp_plan_t* plan, int32_t hq, int32_t hkv, int32_t d, int32_t dtype, int32_t impl,
                              void* stream);

/* Parameters of the plan's WINDOW rows: window >= 1 keys including the query, sink >= 0 tokens at the
 * start of every sequence (both at most 2^30).  Launches of a plan with WINDOW rows fail with
 * DCP_ERR_INVALID_ARG until this has been called; it may be called again between launches. */
dcp_status_t dcp_plan_set_window(dcp_plan_t* plan, int32_t window, int32_t sink);

typedef enum {
  DCP_EXPORT_BLK_START = 0, /* [n_blocks] packed token index of each block's first token        */
  DCP_EXPORT_BLK_LEN = 1,   /* [n_blocks]                                                        */
  DCP_EXPORT_BLK_SEQ = 2,   /* [n_blocks] sequence of each block                                 */
  DCP_EXPORT_FWD_PTR = 3,   /* [n_units+1] CSR over output units (q_blk, or slot when slots used)*/
  DCP_EXPORT_FWD_IDX = 4,   /* [n_kept] table row numbers, per unit ascending kv_blk, stable     */
  DCP_EXPORT_BWDQ_PTR = 5,  /* [n_blocks+1] CSR by q_blk                                         */
  DCP_EXPORT_BWDQ_IDX = 6,  /* [n_kept] per q_blk ascending kv_blk, stable                       */
  DCP_EXPORT_BWDKV_PTR = 7, /* [n_blocks+1] CSR by kv_blk                                        */
  DCP_EXPORT_BWDKV_IDX = 8, /* [n_kept] per kv_blk ascending q_blk, stable                       */
  DCP_EXPORT_SLOT_QBLK = 9, /* [n_slots] q_blk of each slot, -1 for a slot no row uses           */
  DCP_EXPORT_MERGE_PTR = 10,/* [n_blocks+1] CSR: slots of each q_blk                             */
  DCP_EXPORT_MERGE_IDX = 11 /* [n_used_slots] slot numbers, ascending per q_blk                  */
} dcp_export_t;

/* Copies one of the plan's integer arrays (int32) to host memory for bit-exact checks.
 * dst may be NULL to query the length.  n_out receives the array length. */
dcp_status_t dcp_plan_export(const dcp_plan_t* plan, dcp_export_t which, int32_t* dst_host,
                             int64_t capacity, int64_t* n_out);

/* The dK/dV work list of the bf16 MFMA kernels for `hkv` KV heads, for bit-exact host checks: rows
 * (unit = kv_blk position in the BWDKV CSR, tile = 128-key tile of that block, e0, e1 = the CSR entries
 * [e0, e1) the piece covers, pslot).  An item that would keep one workgroup busy much longer than its
 * share of the launch is cut along its table rows into parts; each part has its own pslot >= 0 (a slot
 * of fp32 partial sums in the backward workspace, which a reduce kernel adds up in slot order) and
 * unsplit items have pslot -1.  Pieces are listed in launch order (sequence by sequence when that balances as well as
 * strict longest-first, else longest first).  dst_host may be NULL to query the
 * length; n_items_out receives the number of rows (5 int32 each).  Host only. */
dcp_status_t dcp_plan_export_dkv_items(dcp_plan_t* plan, int32_t hkv, int32_t* dst_host, int64_t capacity_rows,
                                       int64_t* n_items_out);

/* How the list above is divided among the 8 XCDs of the chip, for host checks.  Workgroup ids go to the XCDs
 * round-robin, and the kernels give XCD x a fixed eighth of the work: whole KV heads when hkv is a multiple of 8.
 * Otherwise the list is dealt into n_seg = 8 / gcd(8, hkv) segments of about equal cost (sequences whole, except
 * those that are more than half a segment by themselves), the order inside a segment kept, and an XCD takes (KV head,
 * segment) pairs.  seg_out receives 9 numbers: segment s is rows [seg[s], seg[s + 1]) of dcp_plan_export_dkv_items'
 * list, entries past n_seg repeat the list length.  The forward and dQ lists are divided the same way.  Host only. */
dcp_status_t dcp_plan_export_dkv_segments(dcp_plan_t* plan, int32_t hkv, int32_t* n_seg_out, int32_t* seg_out);

/* ---------------------------------------------------------------------------------------------
 * Tensor descriptor shared by the launching calls.  Unused members are NULL / 0. */
typedef struct {
  int32_t hq, hkv, d;      /* heads and head dim; hq % hkv == 0                                  */
  int32_t dtype;           /* dcp_dtype_t of q,k,v,out,dout,dq,dk,dv and of partial outputs      */
  int32_t impl;            /* dcp_impl_t                                                         */
  float softmax_scale;     /* multiplies Q K^T; the paper's 1/sqrt(D) (Sec. 2.1) is the default  */
                           /* the caller passes explicitly                                       */
  const void* q;  int64_t q_stride_t, q_stride_h;      /* device                                 */
  const void* k;  int64_t k_stride_t, k_stride_h;
  const void* v;  int64_t v_stride_t, v_stride_h;
  const int32_t* attn_ranges; /* device int32[T,4]; required iff a kept row is RANGES            */
  /* forward outputs.  Without slots: out [T,Hq,D] (strides below), lse [Hq,T].                  */
  /* With slots: out = o_part [n_slots, block_size, Hq, D] contiguous, lse = lse_part            */
  /* [n_slots, Hq, block_size]; rows past the block's length are not written.                    */
  void* out;      int64_t o_stride_t, o_stride_h;
  float* lse;
  /* backward: out/lse above are then INPUTS holding the final (merged) O and LSE in the packed  */
  /* layout, even when the plan uses slots.                                                      */
  const void* dout; int64_t do_stride_t, do_stride_h;
  void* dq;       int64_t dq_stride_t, dq_stride_h;
  void* dk;       int64_t dk_stride_t, dk_stride_h;
  void* dv;       int64_t dv_stride_t, dv_stride_h;
} dcp_tensors_t;

/* Blockwise Attention, forward (Listing 1 line 5; Sec. 5 "Blockwise Attention"): for every listed
 * computation block S = scale * Q_i K_j^T, mask, online softmax, acc += P V_j; rows of one output
 * unit accumulate in the kernel; O = acc / l, LSE = m + ln l (natural log of the sum of exp of
 * scaled scores).  A query row that sees no key gets O = 0, LSE = -inf.  Every row of every
 * q_blk (no slots) or of every used slot is written, also when no entry lists it. */
dcp_status_t dcp_block_attn_fwd(dcp_plan_t* plan, const dcp_tensors_t* t, void* stream);

/* Blockwise Reduction (Listing 1 line 6 "RescaleAndSum"; Sec. 5 "Blockwise Reduction"):
 * LSE = ln sum_p exp(LSE_p), O = sum_p exp(LSE_p - LSE) O_p over the slots of each q_blk.
 *   o_part   device [n_slots, block_size, Hq, D] of `dtype`;  lse_part device float [n_slots, Hq, block_size]
 *   out      device [T,Hq,D] of `dtype` with the given strides; lse device float [Hq,T]
 * q blocks without any slot get O = 0, LSE = -inf. */
dcp_status_t dcp_merge_partials(dcp_plan_t* plan, const void* o_part, const float* lse_part,
                                void* out, int64_t o_stride_t, int64_t o_stride_h, float* lse,
                                int32_t hq, int32_t d, int32_t dtype, void* stream);

/* Backward preprocess: delta[h,t] = sum_d dO[t,h,d] * O[t,h,d] from the final O.  Reads t->out,
 * t->dout (hq, d, dtype, strides); writes delta device float [Hq,T]. */
dcp_status_t dcp_bwd_delta(const dcp_tensors_t* t, int64_t total_tokens, float* delta, void* stream);

/* Bytes of device workspace dcp_block_attn_bwd needs for this plan and shape: delta and the rescaled LSE, each
 * float [Hq, rows of the Q-type buffers], plus, for tables with RANGES or WINDOW rows, 32 bytes per 32-row tile of every block
 * (bounds of the rows' range arrays, which let the dK/dV kernel pass over query tiles that see none of its keys),
 * plus, for the bf16 MFMA kernels, 128 KiB per KV head for every part of a split dK/dV item (fp32 partial sums, see
 * dcp_plan_export_dkv_items).  The first call for a given hkv builds and caches the work list in the plan. */
size_t dcp_bwd_workspace_bytes(const dcp_plan_t* plan, int32_t hq, int32_t hkv, int32_t d, int32_t dtype);

/* Blockwise Attention, backward (the mirrored instruction stream of Sec. 5; gradients of blocks
 * that share a Q or KV block are reduced, Sec. 7.5): with P = exp(scale*S - LSE) on listed visible
 * pairs (recomputed, never stored), dV_j += P^T dO_i, dP = dO_i V_j^T, dS = P * (dP - delta_i),
 * dQ_i += scale dS K_j, dK_j += scale dS^T Q_i, KV-head gradients summed over the query heads of
 * the group.  Inputs q,k,v,out,lse,dout; outputs dq,dk,dv (every element written; blocks nothing
 * lists get zeros).  LSE and O are the GLOBAL ones: for a device's share of a plan the gradients
 * are that share's partial sums.  workspace: device, >= dcp_bwd_workspace_bytes, 256-byte aligned. */
dcp_status_t dcp_block_attn_bwd(dcp_plan_t* plan, const dcp_tensors_t* t, void* workspace,
                                size_t workspace_bytes, void* stream);

/* dcp_block_attn_bwd for callers that cannot allocate device memory or pass a workspace (code that runs under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc): the same kernels and results, with the
 * workspace in a fixed device array of DCP_STATIC_SCRATCH_BYTES that the library holds on every GPU it runs on.
 * The call allocates nothing and does not synchronise.  Conditions:
 *   - dcp_plan_prepare(plan, hq, hkv, d, dtype, impl, ...) has been called for this plan and shape on this device
 *     (DCP_ERR_INVALID_ARG otherwise: the call will not create the plan's device copies itself);
 *   - dcp_bwd_workspace_bytes(plan, hq, hkv, d, dtype) <= DCP_STATIC_SCRATCH_BYTES (DCP_ERR_WORKSPACE otherwise, with
 *     both figures in the message; e.g. 32 query heads x 131 072 rows need 32 MiB plus the parts of cut dK/dV items);
 *   - per-kernel timing (dcp_profile_enable) does not cover this call.
 * All calls on one GPU share that GPU's array: two calls that overlap in time on one GPU (two streams, two threads)
 * race; calls ordered on one stream do not.  Inputs, outputs and errors otherwise as dcp_block_attn_bwd. */
#define DCP_STATIC_SCRATCH_BYTES (64u << 20)
dcp_status_t dcp_block_attn_bwd_static(dcp_plan_t* plan, const dcp_tensors_t* t, void* stream);

/* Gradient reduction across blocks (Sec. 5 "Blockwise Reduction" used on gradients, Sec. 7.5):
 * dst[i] = sum_p parts[p][i], accumulated in fp32, stored as dst_dtype.
 *   parts_host_array_of_device_ptrs  host array of n_parts (1..8) device pointers, read during the
 *               call; each points to n_elems contiguous elements of parts_dtype
 *   dst         device, n_elems contiguous elements of dst_dtype, 16-byte aligned like the parts
 * DCP_ERR_INVALID_ARG: n_parts outside 1..8, a NULL or misaligned pointer, n_elems negative or
 * not a multiple of 8.  n_elems == 0 is legal (nothing is launched). */
dcp_status_t dcp_sum_partials(const void* const* parts_host_array_of_device_ptrs, int32_t n_parts,
                              int32_t parts_dtype, void* dst, int32_t dst_dtype, int64_t n_elems,
                              void* stream);

/* Blockwise Copy (Sec. 5 "Blockwise Copy": several data blocks copied inside one device's memory
 * by one fused kernel; used to manage the block buffers of Sec. 5 "Block buffers").
 * A copy list is built once per iteration, like the plan (Sec. 3.2), and replayed for every layer.
 *   entries_host  host int32 [n,3] rows (src_row, dst_row, n_rows), copied; a row is one row of a
 *                 2-D view of a buffer (e.g. one token's [heads, D] slab)
 *   src_rows, dst_rows   number of rows the source / destination buffer holds
 * DCP_ERR_BAD_TABLE: a negative field, a range that leaves its buffer, or two destination ranges
 * that overlap.  n = 0 is legal (the copy does nothing).  The list owns a small device array,
 * created on the device that is current at the first dcp_blockwise_copy and freed by destroy. */
typedef struct dcp_copy_list dcp_copy_list_t;
dcp_status_t dcp_copy_list_create(dcp_copy_list_t** list, const int32_t* entries_host, int64_t n,
                                  int64_t src_rows, int64_t dst_rows);
dcp_status_t dcp_copy_list_destroy(dcp_copy_list_t* list);
/* dst[(dst_row + r) * dst_row_stride + 0 .. row_bytes) = src[(src_row + r) * src_row_stride + ..]
 * for every entry and r < n_rows.  src, dst: device, 16-byte aligned; strides and row_bytes in
 * bytes, multiples of 16, stride >= row_bytes.  The two buffers may be the same allocation
 * (same pointer and stride) only if no destination range of the list overlaps a source range;
 * any other overlap of the two buffers is rejected (DCP_ERR_INVALID_ARG).  Asynchronous on stream. */
dcp_status_t dcp_blockwise_copy(dcp_copy_list_t* list, const void* src, int64_t src_row_stride,
                                void* dst, int64_t dst_row_stride, int64_t row_bytes, void* stream);

/* Execution plans (Sec. 5: a plan is a list of instructions that the executor carries out one after the other;
 * Sec. 4.3: the transfer of one division overlaps the computation of another).  The five instruction
 * types of Sec. 5 map to ops: Blockwise Attention (forward, backward), Blockwise Reduction (LSE merge of partial
 * outputs; plain sum of gradient partials), Blockwise Copy, Comm.Launch and Comm.Wait.  With one device a transfer is
 * a Blockwise Copy handed to a second stream: Comm.Launch starts it after everything issued before it and returns at
 * once, Comm.Wait makes the compute stream wait for it.
 * Fields used per op (others ignored):
 *   ATTN_FWD     plan, tensors                       -> dcp_block_attn_fwd
 *   ATTN_BWD     plan, tensors, workspace(+bytes)    -> dcp_block_attn_bwd
 *   MERGE        plan, o_part, lse_part, tensors.{out, o_stride_t, o_stride_h, lse, hq, d, dtype} -> dcp_merge_partials
 *   COPY         copy_list, src, src_row_stride, dst, dst_row_stride, row_bytes -> dcp_blockwise_copy
 *   SUM          parts, n_parts, parts_dtype, dst, dst_dtype, n_elems -> dcp_sum_partials
 *   COMM_LAUNCH  comm_id + the COPY fields;  COMM_WAIT  comm_id
 * The program copies the instruction array; plans, copy lists and buffers stay the caller's and must outlive it. */
typedef enum { DCP_OP_ATTN_FWD = 0, DCP_OP_ATTN_BWD = 1, DCP_OP_MERGE = 2, DCP_OP_COPY = 3, DCP_OP_SUM = 4,
               DCP_OP_COMM_LAUNCH = 5, DCP_OP_COMM_WAIT = 6 } dcp_op_t;
typedef struct {
  int32_t op, comm_id;
  dcp_plan_t* plan;
  dcp_tensors_t tensors;
  void* workspace;
  size_t workspace_bytes;
  const void* o_part;
  const float* lse_part;
  dcp_copy_list_t* copy_list;
  const void* src;
  void* dst;
  int64_t src_row_stride, dst_row_stride, row_bytes;
  const void* parts[8];
  int32_t n_parts, parts_dtype, dst_dtype;
  int64_t n_elems;
} dcp_instr_t;
typedef struct dcp_program dcp_program_t;
/* DCP_ERR_INVALID_ARG: unknown op, a missing handle, a transfer id launched twice or waited for before its launch. */
dcp_status_t dcp_program_create(dcp_program_t** program, const dcp_instr_t* instrs_host, int64_t n);
dcp_status_t dcp_program_destroy(dcp_program_t* program);
/* Issues every instruction (asynchronous).  compute_stream runs everything except the transfers, which run on
 * comm_stream (a different stream if the program has any).  On return the compute stream also waits for every
 * transfer that no Comm.Wait covered, so synchronising it is enough.  The first error stops the walk and is returned. */
dcp_status_t dcp_program_run(dcp_program_t* program, void* compute_stream, void* comm_stream);

/* Communication volume of a placement (host only; Sec. 4.1, the volume of a configuration, and Sec. 4.2, the
 * connectivity metric of the hypergraph whose hyperedges join each data block to the computation blocks that
 * consume it or contribute to it).  A table row is one computation block (all heads): it consumes Q block q_blk
 * and KV block kv_blk and contributes to O block q_blk; SKIP rows are not computation blocks.
 *   blk_dev   host int32 [n_blocks]: device of each block's tokens (their Q, KV and O live together, Sec. 4.1)
 *   comp_dev  host int32 [n_entries]: device of each computation block
 *   *_bytes_per_token: bytes one token holds in Q, in K and V together, in O (all heads)
 * Outputs (each may be NULL):
 *   pairwise      sum over computation blocks of Size(input)[Dev(input) != Dev(C)] + Size(output)[Dev(output) != Dev(C)]
 *   connectivity  sum over hyperedges of s_e (lambda_e - 1): every remote device moves the block once
 *   n_hyperedges  hyperedges with at least one computation block
 *   send, recv    host int64 [n_devices]: bytes each device sends / receives under the connectivity model (an input
 *                 block goes from its owner to each other device that computes with it; a partial output goes from
 *                 each other device that contributes to the block's owner)
 * DCP_ERR_BAD_TABLE: block or device id out of range. */
dcp_status_t dcp_comm_volume(const int32_t* cu_seqlens_host, int32_t n_seq, int32_t block_size,
                             const int32_t* table_host, int64_t n_entries, const int32_t* blk_dev,
                             const int32_t* comp_dev, int32_t n_devices, int64_t q_bytes_per_token,
                             int64_t kv_bytes_per_token, int64_t o_bytes_per_token, int64_t* pairwise,
                             int64_t* connectivity, int64_t* n_hyperedges, int64_t* send, int64_t* recv);

/* Per-kernel timing for benchmarks.  While enabled, every kernel the library launches is
 * bracketed by hipEvents recorded on the launch stream (the kernels of one backward call are timed
 * one by one).  dcp_profile_read synchronises on the recorded events, returns the summed duration
 * and the number of launches of one kernel since the last enable, and leaves the records in place;
 * dcp_profile_enable(1) clears them.  Not thread-safe; meant for a single benchmarking thread. */
typedef enum { DCP_K_FWD = 0, DCP_K_MERGE = 1, DCP_K_DELTA = 2, DCP_K_DQ = 3, DCP_K_DKV = 4, DCP_K_SUM = 5, DCP_K_COPY = 6 } dcp_kernel_id_t;
dcp_status_t dcp_profile_enable(int32_t enable);
dcp_status_t dcp_profile_read(int32_t kernel_id, double* total_ms, int64_t* launches);

/* Last error message of the calling thread ("" if none). */
const char* dcp_last_error(void);

/* Library version string and the kernel tile sizes in use, for logs. */
const char* dcp_version(void);

#ifdef __cplusplus
}
#endif
#endif /* DCP_H_ */
