/*
 * libhspmd_attn -- causal self-attention forward and backward over packed
 * variable-length sequences on ONE GPU's share of the attention heads,
 * written for AMD MI355X (gfx950).
 *
 * Where this sits in the paper (HSPMD / Hetu v2): it is the device-level work
 * behind the AttentionFwd / AttentionBwd operators of the forward and backward
 * executable subgraphs (Appendix "Implementation Details", subsection
 * "Execution").  What reaches such an operator at run time is what the
 * arguments below carry:
 *   - packed mixed-length sequences whose concrete shapes are only resolved
 *     when the inputs arrive on the device (Section 6.3 "Execution"; Appendix,
 *     "Symbolic shape extension"; Evaluations, scenario (c) "Mixed-length
 *     data")                                      -> cu_seqlens;
 *   - a shard of the hidden dimension whose size may differ between sharding
 *     subgroups (Section 4.2, HDim / HSize and its footnote: the shape of each
 *     shard can vary and is determined at runtime)
 *                                                 -> local_q_heads, local_kv_heads;
 *   - optional grouped KV heads (model table "Query Groups")
 *                                                 -> local_q_heads / local_kv_heads.
 * The paper does not write the attention formula; it is the standard causal
 * scaled-dot-product attention (Section 2.1 cites it), per sequence:
 *
 *   S_rj = scale <q_r, k_j>  (j <= r),   P = softmax_j S,   O_r = sum_j P_rj v_j,
 *   LSE_r = ln sum_{j<=r} exp(S_rj);
 *   dP_rj = <dO_r, v_j>, D_r = <dO_r, O_r>, dS = P (dP - D),
 *   dQ_r = scale sum_j dS_rj k_j,  dK_j = scale sum_{h,r} dS_rj q_r,  dV_j = sum_{h,r} P_rj dO_r
 *   (h runs over the query heads that share the KV head; query head h uses KV
 *   head h / (local_q_heads / local_kv_heads)).
 *
 * Conventions for every entry point
 *   - Device pointers are plain `void*` / `float*` to memory the CALLER owns
 *     (allocate it with anything: hipMalloc, a PyTorch tensor).  Host pointers
 *     are marked "host".
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Forward and backward only enqueue work; they never synchronise and never
 *     allocate, so they may be recorded into a HIP graph (with per-kernel timing
 *     off, see hspmd_profile_enable).  Plan creation allocates the plan's small index arrays and
 *     copies them to the device before returning; hspmd_attn_plan_update refills them without
 *     allocating.
 *   - Every call returns an hspmd_status; no exception crosses this boundary
 *     and nothing aborts.  Arguments are validated on the host before any
 *     launch.  hspmd_last_error() returns a thread-local description of the
 *     last failure on the calling thread.
 *   - Threads: every entry point may be used by several host threads at once, on plans, streams
 *     and workspaces of their own.  Launches that share a plan, or a workspace, must be ordered on the
 *     device (same stream, or an event between them): the persistent kernels draw their work items
 *     from counters that belong to the plan, and the launch that finishes leaves them at zero for the
 *     next one.  hspmd_attn_plan_update and hspmd_attn_plan_destroy need the plan to themselves.
 *   - bf16 tensors are raw 16-bit bfloat16 values.
 */
#ifndef HSPMD_ATTN_H
#define HSPMD_ATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    HSPMD_OK = 0,
    HSPMD_ERR_INVALID_ARG = 1,        /* null pointer, bad lengths, bad strides, heads not a whole number of groups */
    HSPMD_ERR_UNSUPPORTED = 2,        /* head_dim not a multiple of 8 in 8..128, unknown dtype */
    HSPMD_ERR_WORKSPACE_TOO_SMALL = 3,
    HSPMD_ERR_HIP = 4                 /* a HIP runtime call failed; see hspmd_last_error() */
} hspmd_status;

/* dtype of the gradients written by hspmd_attn_varlen_bwd */
typedef enum { HSPMD_GRAD_BF16 = 0, HSPMD_GRAD_F32 = 1 } hspmd_grad_dtype;

/* which work list of a plan (see hspmd_attn_schedule) */
typedef enum {
    HSPMD_LIST_FWD = 0,   /* items (sequence, q tile, q head): forward kernel          */
    HSPMD_LIST_DQ = 1,    /* items (sequence, q tile, q head): backward dQ pass        */
    HSPMD_LIST_DKV = 2    /* items (sequence, k tile, kv head): backward dK/dV pass    */
} hspmd_list_kind;

/* launch order of a work list */
typedef enum {
    HSPMD_ORDER_XCD_COST = 0,   /* default: chains per XCD queue, balanced by cost, expensive items first */
    HSPMD_ORDER_NATURAL = 1,    /* sequence-major, tiles ascending, heads innermost: no cost model at all    */
    HSPMD_ORDER_COST = 2        /* one global list, most expensive item first, no XCD placement             */
} hspmd_order;

/* One unit of work for one workgroup.  tile < 0 marks a padding slot that does nothing. */
typedef struct {
    int32_t token_start;  /* first packed token of the sequence (cu_seqlens[seq])      */
    int32_t seq_len;      /* L of that sequence                                          */
    int32_t tile;         /* q tile index (FWD, DQ) or k tile index (DKV) within it      */
    int32_t head;         /* local q head (FWD, DQ) or local kv head (DKV)               */
} hspmd_work_item;

/*
 * One unit of work of the block variant (one step of context-parallel attention, see
 * hspmd_attn_block_plan_create): the sequence's query chunk and key/value chunk are separate
 * token ranges and the causal mask is shifted by the difference of their positions.
 */
typedef struct {
    int32_t q_start;   /* first token of the sequence's query chunk in the packed q / o / d_o / dq tensors  */
    int32_t q_len;     /* rows in that chunk                                                               */
    int32_t k_start;   /* first token of the sequence's key/value chunk in the packed k / v / dk / dv tensors */
    int32_t k_len;     /* keys in that chunk                                                               */
    int32_t offset;    /* q_pos - k_pos: key j of the chunk is visible to row r of the chunk iff j <= r + offset */
    int32_t tile;      /* q tile index (FWD, DQ) or k tile index (DKV) within the chunk; < 0: padding slot  */
    int32_t head;      /* local q head (FWD, DQ) or local kv head (DKV)                                     */
    int32_t q_pos;     /* position of the query chunk's first row inside its sequence (the key chunk's is q_pos - offset) */
} hspmd_block_item;

/* Never NULL.  Thread-local. */
const char* hspmd_last_error(void);

/* Rows per tile of each list kind (q rows for FWD/DQ, key rows for DKV). */
int32_t hspmd_attn_tile_rows(hspmd_list_kind kind);

/*
 * Packed-sequence offsets (run-time shapes; Section 6.3, Appendix "Symbolic
 * shape extension").  Host only.
 *   lengths      host, [num_seqs], each >= 0 (zero-length sequences are legal)
 *   cu_seqlens   host, [num_seqs + 1], caller-owned, receives the exclusive prefix sum
 *   max_seqlen   host, may be NULL
 *   total_tokens host, may be NULL
 * Fails with INVALID_ARG on a null pointer, num_seqs < 0, a negative length, or a
 * running sum above INT32_MAX.
 */
hspmd_status hspmd_build_cu_seqlens(const int32_t* lengths, int32_t num_seqs, int32_t* cu_seqlens,
                                    int32_t* max_seqlen, int64_t* total_tokens);

/*
 * The cost-sorted work list, host only (no GPU needed).  This is the on-device
 * counterpart of the paper's cost-model-driven dispatch of mixed-length
 * sequences (Appendix "Scenario-specific Planning", mixed-length case): the
 * unit here is one tile of one sequence and head, its cost the number of tile
 * pairs it visits under the causal mask.
 *
 * Items are emitted in launch order: slot p is executed by workgroup p.  Slots
 * p with equal p % num_queues form one queue; a queue keeps tiles that share
 * K/V (FWD, DQ) or Q/dO (DKV) together, queues are balanced by total cost and
 * each queue runs its expensive items first.  Shorter queues are padded with
 * tile = -1 slots so that every queue has the same length.
 *
 *   cu_seqlens   host, [num_seqs + 1], cu[0] == 0, non-decreasing
 *   num_queues   >= 1 (the library uses 8, the number of XCDs of an MI355X)
 *   items        host, caller-owned, capacity entries; may be NULL when capacity == 0
 *   count        receives the number of slots the list needs; if it exceeds capacity
 *                nothing is written and INVALID_ARG is returned (call with capacity 0
 *                first to size the buffer: that call returns OK)
 */
hspmd_status hspmd_attn_schedule(hspmd_list_kind kind, const int32_t* cu_seqlens, int32_t num_seqs,
                                 int32_t local_q_heads, int32_t local_kv_heads, int32_t num_queues,
                                 hspmd_work_item* items, int64_t capacity, int64_t* count);

/* Same with an explicit launch order (the alternatives exist to measure what the default buys). */
hspmd_status hspmd_attn_schedule_ordered(hspmd_list_kind kind, hspmd_order order, const int32_t* cu_seqlens,
                                         int32_t num_seqs, int32_t local_q_heads, int32_t local_kv_heads,
                                         int32_t num_queues, hspmd_work_item* items, int64_t capacity, int64_t* count);

/*
 * Plan: the three device-resident work lists for one pack and one local head
 * configuration.  One plan serves every layer and both passes of a micro-batch.
 * Opaque, library-owned; destroy it with hspmd_attn_plan_destroy.  Creating a
 * plan needs a GPU: the lists are uploaded through a copy stream that the library owns (one per
 * device, created on first use) and the call waits for that upload only, never for `stream` or any
 * other work of the caller, so the plan of the next micro-batch can be built while the kernels of the
 * current one run.  The lists are in place when the call returns (`stream` is accepted and unused).
 *   local_q_heads   query heads held by this GPU (any positive count: an uneven share is fine)
 *   local_kv_heads  KV heads held by this GPU; local_q_heads % local_kv_heads must be 0
 *   head_dim        a multiple of 8 in 8..128 (rows move in 16-byte chunks).  The kernels are built for
 *                   tile widths 64 and 128; other sizes, such as the 104 of the paper's 32B model (model
 *                   configuration table: hidden 6656, 64 heads), run on the next width up: same results,
 *                   the matrix-core work of the padded width
 */
typedef struct hspmd_attn_plan hspmd_attn_plan;
hspmd_status hspmd_attn_plan_create(const int32_t* cu_seqlens_host, int32_t num_seqs, int32_t local_q_heads,
                                    int32_t local_kv_heads, int32_t head_dim, void* stream,
                                    hspmd_attn_plan** out);
hspmd_status hspmd_attn_plan_create_ordered(const int32_t* cu_seqlens_host, int32_t num_seqs, int32_t local_q_heads,
                                            int32_t local_kv_heads, int32_t head_dim, hspmd_order order,
                                            void* stream, hspmd_attn_plan** out);
/*
 * Refill of a plan with the next pack (same local head counts, head_dim and launch order): the work lists are rebuilt
 * on the host and uploaded into device storage the plan already owns.  The paper plans every mixed-length batch on the
 * CPU while the GPU works on the previous one (Appendix "Scenario-specific Planning", mixed-length case); this is that
 * step for the attention operator, and it is what a training loop calls once per micro-batch.
 *   A plan holds three copies ("slots") of its lists and a refill writes the one used longest ago, so launches that
 *   read the current lists may still be running.  Each forward / backward / rotary call records an event on its stream
 *   for the slot it reads; the refill waits on the host for the event of the slot it is about to overwrite (finished
 *   long ago once the ring has gone round), never for the device as a whole.  A slot that is too small is replaced
 *   by a larger one (hipFree + hipMalloc, with a quarter of headroom); packs of similar size therefore stop
 *   allocating after the first few refills.
 *   Not for concurrent use: no other thread may launch with the plan during the call.  A launch recorded into a HIP
 *   graph records no event (events cannot be waited for from inside a capture): a plan that a graph replays must not be
 *   refilled while the graph may run.  On error the plan keeps its previous pack.
 * Errors: INVALID_ARG for a NULL plan, the wrong kind of plan, bad cu_seqlens; HIP for a failed runtime call.
 */
hspmd_status hspmd_attn_plan_update(hspmd_attn_plan* plan, const int32_t* cu_seqlens_host, int32_t num_seqs);
/* hipFree of the lists' device storage: waits for the device to go idle.  NULL is accepted. */
hspmd_status hspmd_attn_plan_destroy(hspmd_attn_plan* plan);
int64_t hspmd_attn_plan_total_tokens(const hspmd_attn_plan* plan); /* -1 on NULL */
int64_t hspmd_attn_plan_num_items(const hspmd_attn_plan* plan, hspmd_list_kind kind); /* slots incl. padding */

/* Bytes of device workspace the backward needs (two fp32 [local_q_heads, T] arrays: the row statistics
 * D = rowsum(dO * O) and the logsumexp in the form the kernels consume them, plus a few constants). */
size_t hspmd_attn_bwd_workspace_bytes(const hspmd_attn_plan* plan);

/*
 * Forward (AttentionFwd).  All tensors device memory.
 *   q   bf16 [T, local_q_heads, head_dim]; token t, head h at q + t*q_token_stride + h*head_dim
 *   k,v bf16 [T, local_kv_heads, head_dim]; token stride kv_token_stride (same for k and v)
 *       Strides are in elements and let q/k/v be views into a fused QKV projection output;
 *       they must be multiples of 8 (16-byte rows) and >= heads*head_dim; base pointers 16-byte aligned.
 *   softmax_scale   <= 0 selects 1/sqrt(head_dim); a positive value must be finite and lie in [2^-60, 2^60]
 *                   (INVALID_ARG otherwise: the backward carries lse / scale in fp32)
 *   o   bf16 [T, local_q_heads, head_dim], contiguous, written
 *   lse fp32 [local_q_heads, T], natural-log logsumexp of the scaled scores, written
 * T == 0 returns OK without launching.
 */
hspmd_status hspmd_attn_varlen_fwd(const hspmd_attn_plan* plan, const void* q, const void* k, const void* v,
                                   int64_t q_token_stride, int64_t kv_token_stride, float softmax_scale,
                                   void* o, float* lse, void* stream);

/*
 * Backward (AttentionBwd): two launches on `stream` -- the dQ pass, which also computes the
 * row statistic D = rowsum(dO * O) of its rows and leaves it in the workspace; the dK/dV pass.
 * Both passes recompute P from the stored lse.  No atomics: results are run-to-run bit-identical.
 *   o, d_o  bf16 [T, local_q_heads, head_dim], contiguous
 *   lse     fp32 [local_q_heads, T] as written by the forward
 *   dq      [T, local_q_heads, head_dim]; dk, dv [T, local_kv_heads, head_dim]; contiguous,
 *           bf16 or fp32 according to grad_dtype; fully overwritten
 *   workspace  device, at least hspmd_attn_bwd_workspace_bytes(plan) bytes, 16-byte aligned
 */
hspmd_status hspmd_attn_varlen_bwd(const hspmd_attn_plan* plan, const void* q, const void* k, const void* v,
                                   const void* o, const float* lse, const void* d_o,
                                   int64_t q_token_stride, int64_t kv_token_stride, float softmax_scale,
                                   void* dq, void* dk, void* dv, hspmd_grad_dtype grad_dtype,
                                   void* workspace, size_t workspace_bytes, void* stream);

/*
 * hspmd_attn_varlen_bwd for callers that cannot allocate device memory and have no workspace to pass: code that
 * runs under HIP graph capture, tight serving / training loops, harnesses that forbid hipMalloc.  Same arguments,
 * kernels and results as hspmd_attn_varlen_bwd, without `workspace`: the row statistics that the dQ pass leaves for
 * the dK/dV pass go into a fixed device array inside the library (HSPMD_STATIC_WORKSPACE_BYTES bytes on every GPU the
 * library runs on, held until the process ends).  The call allocates and frees nothing and creates no events
 * (per-kernel timing does not apply to it).
 *   Limit: hspmd_attn_bwd_workspace_bytes(plan) <= HSPMD_STATIC_WORKSPACE_BYTES, i.e.
 *   local_q_heads * total_tokens <= 2^21 (the 65536-token, 32-head configuration just fits);
 *   larger packs get WORKSPACE_TOO_SMALL and nothing is launched.
 *   All calls on one GPU share the array: two calls that may overlap on one GPU (different streams, no event between
 *   them) race on it; calls on one stream are ordered and safe.  Nothing in it needs clearing between calls: every
 *   value the dK/dV pass reads is written by the dQ pass of the same call.
 *   The array's device address is looked up on the first call on each device; make that first call outside a graph
 *   capture.
 * Other errors as hspmd_attn_varlen_bwd.
 */
#define HSPMD_STATIC_WORKSPACE_BYTES (16u * 1024u * 1024u + 256u)
hspmd_status hspmd_attn_varlen_bwd_static_ws(const hspmd_attn_plan* plan, const void* q, const void* k, const void* v,
                                             const void* o, const float* lse, const void* d_o, int64_t q_token_stride,
                                             int64_t kv_token_stride, float softmax_scale, void* dq, void* dk, void* dv,
                                             hspmd_grad_dtype grad_dtype, void* stream);

/*
 * Rotary position embedding around the attention of a pack.  The paper's models are Llama-style with RoPE as
 * position encoding (experimental setup, model configuration table) and give no formula; this is the published
 * definition in the rotate-half pairing: with theta_i = base^(-2i/head_dim), i = 0 .. head_dim/2-1, a token at
 * position p INSIDE ITS SEQUENCE (positions restart at every sequence of the pack) has every head vector x of
 * q and k replaced by
 *     y_i = x_i cos(p theta_i) - x_{i+head_dim/2} sin(p theta_i),
 *     y_{i+head_dim/2} = x_{i+head_dim/2} cos(p theta_i) + x_i sin(p theta_i).
 * Division of the work: q and k are rotated by one elementwise kernel before the forward (hspmd_rope_qk; K and Q
 * tiles are streamed many times by the attention kernels, so rotating them at tile load would repeat the work
 * per tile); in the backward the transposed rotation of dQ and dK is applied inside the epilogues of the two
 * passes (hspmd_attn_varlen_bwd_rope), which saves a pass over the gradients.
 *
 * hspmd_rope_table: fills a device table (cos, sin) pairs, fp32 [positions, head_dim/2, 2], evaluated in fp64.
 *   table     device, hspmd_rope_table_bytes(positions, head_dim) bytes, 16-byte aligned, caller-owned
 *   base      the frequency base (10000 in Llama); must be positive
 * hspmd_rope_qk: q_out, k_out = rope(q), rope(k) (inverse != 0: the rotation by the opposite angle).
 *   q, k, q_out, k_out  bf16, layouts and stride rules as in hspmd_attn_varlen_fwd, each with its own token
 *                       stride; q_out == q and k_out == k (in place) are allowed, other overlaps are not
 *   table_positions     positions the table holds; must cover every position a token of the plan has (packed
 *                       plans: the longest sequence; block plans: the largest q_pos + chunk length and
 *                       k_pos + chunk length)
 *   Arithmetic in fp32, one rounding to bf16.  With a block plan (hspmd_attn_block_plan_create) q is the
 *   plan's query chunks and k its key chunks, each token rotated by its position inside its sequence
 *   (q_pos / k_pos of the chunk + index in the chunk): a device rotates its own chunks once, and the rotated
 *   key chunk travels around the ring.
 * hspmd_attn_varlen_bwd_rope: hspmd_attn_varlen_bwd where q and k are the ROTATED tensors the forward consumed
 *   and dq, dk are returned with respect to the unrotated ones (dv is unaffected).  Other arguments, workspace and
 *   errors as hspmd_attn_varlen_bwd.
 * hspmd_attn_block_bwd_rope: the same for hspmd_attn_block_bwd; the rotation is linear, so the accumulated dq
 *   (dq_accumulate) is the sum of the blocks' turned-back shares, and each block's dk is turned back before it
 *   travels on.
 * Errors: INVALID_ARG for NULL / misaligned pointers, bad strides, a table that is too short, the wrong kind of
 * plan; UNSUPPORTED for a head_dim outside the supported set.  Nothing is launched on error.
 */
size_t hspmd_rope_table_bytes(int32_t positions, int32_t head_dim);   /* 0 on bad arguments */
hspmd_status hspmd_rope_table(float* table, int32_t positions, int32_t head_dim, double base, void* stream);
hspmd_status hspmd_rope_qk(const hspmd_attn_plan* plan, const void* q, const void* k, int64_t q_token_stride,
                           int64_t kv_token_stride, void* q_out, void* k_out, int64_t q_out_token_stride,
                           int64_t kv_out_token_stride, const float* table, int32_t table_positions, int32_t inverse,
                           void* stream);
hspmd_status hspmd_attn_varlen_bwd_rope(const hspmd_attn_plan* plan, const void* q, const void* k, const void* v,
                                        const void* o, const float* lse, const void* d_o, int64_t q_token_stride,
                                        int64_t kv_token_stride, float softmax_scale, void* dq, void* dk, void* dv,
                                        hspmd_grad_dtype grad_dtype, const float* table, int32_t table_positions,
                                        void* workspace, size_t workspace_bytes, void* stream);
hspmd_status hspmd_attn_block_bwd_rope(const hspmd_attn_plan* plan, const void* q, const void* k, const void* v,
                                       const void* o, const float* lse, const void* d_o, int64_t q_token_stride,
                                       int64_t kv_token_stride, float softmax_scale, float* dq, int32_t dq_accumulate,
                                       float* dk, float* dv, int32_t reuse_statistics, const float* table,
                                       int32_t table_positions, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Predicted kernel time (milliseconds, MI355X) of forward and backward of a pack on this library's
 * kernels: the per-operator cost that the paper's planner needs when it dispatches mixed-length
 * sequences to pipelines by a cost model evaluated on the CPU (Appendix "Scenario-specific Planning",
 * mixed-length case).  Host only, no GPU needed; costs about as much as building the work lists.
 * Model: each pass walks its work list; an item weighs (inner steps x a step time + a fixed time per
 * item), a pass takes a launch time plus the weight of its heaviest XCD queue divided by the
 * workgroups resident per XCD, and not less than its heaviest item; backward = dQ pass + dK/dV
 * pass.  The coefficients are fitted to measured kernel times
 * (paper_2504_20490_amd/fit_cost_model.py refits them): mean error 6-9 %, up to 15-29 % on packs
 * that take only about a hundred microseconds.  Host-side plan creation is not included.
 */
hspmd_status hspmd_attn_estimate_ms(const int32_t* cu_seqlens, int32_t num_seqs, int32_t local_q_heads,
                                    int32_t local_kv_heads, int32_t head_dim, double* fwd_ms, double* bwd_ms);

/*
 * ---- Block variant: one step of context-parallel attention on one device ----
 * The paper shards long sequences over devices (context parallelism) with ring-based send-receive
 * inside attention, wrapped in its fused ParallelAttn operator (Section 2.1, data sharding; system
 * overview, footnote on ParallelAttn).  What one device computes per ring step is attention of its
 * own chunk of query rows against one chunk of keys/values (its own or a received one); the steps'
 * partial results are merged.  Positions are positions inside the whole sequence:
 *   sequence i: rows at q_pos[i] + r (r < q_len[i]), keys at k_pos[i] + j (j < k_len[i]);
 *   key j is visible to row r iff k_pos[i] + j <= q_pos[i] + r.
 * Chunks may be empty, lie wholly in the past (every key visible) or wholly in the future (nothing
 * visible: O = 0, LSE = -inf, zero gradients).  The sends and receives themselves are not part of
 * this library.
 *
 * hspmd_attn_block_schedule / hspmd_attn_block_plan_create mirror hspmd_attn_schedule /
 * hspmd_attn_plan_create:
 *   cu_q, cu_k     host, [num_seqs + 1]: packed offsets of the query chunks / key chunks
 *   q_pos, k_pos   host, [num_seqs], >= 0: position of each chunk's first row / key in its sequence
 * A plan made here works only with the hspmd_attn_block_* calls (and the other plans only with
 * hspmd_attn_varlen_*); hspmd_attn_plan_total_tokens counts its query tokens,
 * hspmd_attn_plan_total_kv_tokens its key tokens, and hspmd_attn_bwd_workspace_bytes applies as is.
 */
hspmd_status hspmd_attn_block_schedule(hspmd_list_kind kind, const int32_t* cu_q, const int32_t* cu_k,
                                       const int32_t* q_pos, const int32_t* k_pos, int32_t num_seqs,
                                       int32_t local_q_heads, int32_t local_kv_heads, int32_t num_queues,
                                       hspmd_block_item* items, int64_t capacity, int64_t* count);
hspmd_status hspmd_attn_block_plan_create(const int32_t* cu_q_host, const int32_t* cu_k_host, const int32_t* q_pos_host,
                                          const int32_t* k_pos_host, int32_t num_seqs, int32_t local_q_heads,
                                          int32_t local_kv_heads, int32_t head_dim, void* stream, hspmd_attn_plan** out);
int64_t hspmd_attn_plan_total_kv_tokens(const hspmd_attn_plan* plan);   /* -1 on NULL */
/* hspmd_attn_plan_update for a block plan: the chunks of the next ring step or the next pack. */
hspmd_status hspmd_attn_block_plan_update(hspmd_attn_plan* plan, const int32_t* cu_q_host, const int32_t* cu_k_host,
                                          const int32_t* q_pos_host, const int32_t* k_pos_host, int32_t num_seqs);

/*
 * Forward of one block.  q bf16 [Tq, Hq, d], k / v bf16 [Tk, Hkv, d] (strides as in hspmd_attn_varlen_fwd).
 *   o_partial    fp32 [Tq, Hq, d], contiguous, written: softmax over the block's visible keys only
 *   lse_partial  fp32 [Hq, Tq], written: logsumexp over the block's visible keys, -inf where none is visible
 * Partial results stay in fp32 until the last merge.
 */
hspmd_status hspmd_attn_block_fwd(const hspmd_attn_plan* plan, const void* q, const void* k, const void* v,
                                  int64_t q_token_stride, int64_t kv_token_stride, float softmax_scale,
                                  float* o_partial, float* lse_partial, void* stream);

/*
 * Merge of two partial results of the same rows over disjoint key sets:
 *   LSE = ln(exp(LSE_a) + exp(LSE_b)),  O = exp(LSE_a - LSE) O_a + exp(LSE_b - LSE) O_b;
 * a partial result with LSE = -inf is the neutral element.  All tensors device memory, O fp32
 * [total_tokens, local_q_heads, head_dim], LSE fp32 [local_q_heads, total_tokens].  o_out / lse_out may be
 * the same buffers as o_a / lse_a (in-place accumulation), not o_b / lse_b.  o_out_bf16 (may be NULL)
 * also receives the merged O rounded to bf16: pass it on the last merge to get the tensor the backward
 * and the next layer consume.
 */
hspmd_status hspmd_attn_merge(int64_t total_tokens, int32_t local_q_heads, int32_t head_dim, const float* o_a,
                              const float* lse_a, const float* o_b, const float* lse_b, float* o_out, float* lse_out,
                              void* o_out_bf16, void* stream);

/*
 * Backward of one block.  o (bf16) and lse are the MERGED results of the whole rows (all blocks), d_o
 * the gradient of that output; P is recomputed as exp(S - lse), so every block can be processed
 * independently of the others.
 *   dq   fp32 [Tq, Hq, d]: this block's share of dQ; dq_accumulate != 0 adds it to the buffer's
 *        contents (the caller zeroes or overwrites on the first block), 0 overwrites
 *   dk, dv  fp32 [Tk, Hkv, d], overwritten: gradients of this block's keys / values from this block's
 *        rows (in a ring they travel on with the chunk and are summed by the caller)
 *   reuse_statistics != 0: the D pass is skipped and `workspace` must still hold what an earlier
 *        call with the same o, lse, d_o, scale and a plan of the same query chunks left there
 *        (o and lse may then be NULL)
 * Gradients are fp32 only: partial sums are not rounded to bf16.
 */
hspmd_status hspmd_attn_block_bwd(const hspmd_attn_plan* plan, const void* q, const void* k, const void* v,
                                  const void* o, const float* lse, const void* d_o,
                                  int64_t q_token_stride, int64_t kv_token_stride, float softmax_scale,
                                  float* dq, int32_t dq_accumulate, float* dk, float* dv, int32_t reuse_statistics,
                                  void* workspace, size_t workspace_bytes, void* stream);

/*
 * Per-kernel timing for measurement (the evidence the kernels are tuned against; not part of
 * the paper's method).  While enabled, every kernel launch made by forward / backward on the
 * calling process is bracketed by a pair of HIP events recorded on the launch stream.
 * hspmd_profile_read waits for the recorded events, adds each kernel's elapsed time and launch
 * count to the caller's arrays and forgets the records.
 *   kernel index: 0 forward, 1 backward D = rowsum(dO*O) (block variant only: the packed dQ pass computes D
 *                 itself), 2 backward dQ pass, 3 backward dK/dV pass,
 *                 4 rotary embedding of q and k
 *   ms, launches  host, [HSPMD_NUM_KERNELS] each, accumulated into (the caller zeroes them)
 * The switch is process-wide: while it is on, launches from every thread are recorded (the records are guarded by a
 * lock) and a read returns all of them.  Events are created on first use and reused; enabling allocates nothing on
 * the device.
 */
#define HSPMD_NUM_KERNELS 5
hspmd_status hspmd_profile_enable(int32_t on);
hspmd_status hspmd_profile_read(double* ms, int64_t* launches);
/* The same records as per-kernel statistics: sum, number of launches, minimum and median of the launches' elapsed
 * times (all four arrays host, [HSPMD_NUM_KERNELS], overwritten; 0 for a kernel without launches). */
hspmd_status hspmd_profile_read_stats(double* sum_ms, int64_t* launches, double* min_ms, double* median_ms);
const char* hspmd_kernel_name(int32_t kernel);   /* symbol-like name, NULL if out of range */

/*
 * Measured matrix-core rate of the device the library runs on: a second denominator beside the
 * nominal bf16 peak (measurement only; not part of the paper's method).  Launches, on `stream`, a
 * kernel in which every wave of every compute unit issues `mfma_per_wave` back-to-back
 * v_mfma_f32_32x32x16_bf16 on register operands (four independent accumulators, no memory traffic),
 * times it with a pair of HIP events and returns the dense bf16 rate in TFLOP/s.  One untimed
 * launch precedes the timed one.  Synchronises the stream; scratch_out is caller-owned device
 * memory of at least hspmd_probe_scratch_bytes() bytes that receives a checksum (so that the
 * compiler keeps the products).  mfma_per_wave is rounded up to a multiple of 16; <= 0 is INVALID_ARG.
 */
size_t       hspmd_probe_scratch_bytes(void);
hspmd_status hspmd_probe_mfma_tflops(int64_t mfma_per_wave, void* scratch_out, size_t scratch_bytes,
                                     void* stream, double* tflops);
/* The same with operands that vary: four pairs of pseudo-random bf16 values in +-[0.5, 2), different in every
 * lane, used in turn.  The chip limits its power, and the clock it sustains under matrix work depends on how
 * many bits toggle: this is the rate the matrix cores deliver on data like the attention kernels' (they too
 * run about a quarter faster on all-zero inputs than on random ones). */
hspmd_status hspmd_probe_mfma_tflops_varied(int64_t mfma_per_wave, void* scratch_out, size_t scratch_bytes,
                                     void* stream, double* tflops);

/*
 * Variants of the matrix-core rate probe, all on varying operands unless named constant (measurement only; not part
 * of the paper's method).  They answer the questions the attention kernels raise about the chip they run on:
 * which MFMA shape delivers more flops inside the chip's power limit, what streaming the A operand from LDS costs,
 * and whether idle time of the matrix pipes is returned as clock (the limit is an average one, not an instantaneous one).
 * Arguments, scratch and synchronisation as hspmd_probe_mfma_tflops; one round is 16 products 32x32x16 or 32 products
 * 16x16x32 (the same flops).  INVALID_ARG for an unknown mode.
 */
typedef enum {
    HSPMD_PROBE_32X32X16_CONSTANT = 0,   /* = hspmd_probe_mfma_tflops */
    HSPMD_PROBE_32X32X16 = 1,            /* register operands, two waves per SIMD */
    HSPMD_PROBE_16X16X32 = 2,
    HSPMD_PROBE_32X32X16_LDS = 3,        /* every A fragment read from LDS (1 KB per 32x32x16 product), B in registers */
    HSPMD_PROBE_16X16X32_LDS = 4,        /* every A fragment read from LDS and used by two products */
    HSPMD_PROBE_IDLE_0 = 5,              /* one wave per SIMD, no idle time */
    HSPMD_PROBE_IDLE_256 = 6,            /* ... 256 clocks of s_sleep after every 512 clocks of products */
    HSPMD_PROBE_IDLE_512 = 7,
    HSPMD_PROBE_IDLE_1024 = 8
} hspmd_probe_mode;
hspmd_status hspmd_probe_mfma_rate(hspmd_probe_mode mode, int64_t mfma_per_wave, void* scratch_out, size_t scratch_bytes,
                                   void* stream, double* tflops);

#ifdef __cplusplus
}
#endif
#endif /* HSPMD_ATTN_H */
