/*
 * flexsp.h - C ABI of the MI355X (gfx950) library for one device's share of
 * Ulysses-style sequence parallelism with heterogeneous groups (FlexSP).
 *
 * After the sequence-to-head exchange (paper Sec. 2.1.2, Eq. 2) a device holds H/P
 * attention heads for a packed stream of complete, variable-length sequences
 * (Sec. 2.2.2, sequence packing) and evaluates attention on them (Eq. 3); the result goes
 * back through the inverse exchange (Eq. 4).  This library provides, for one GPU:
 *
 *   flexsp_pack / flexsp_unpack   the local layout permute either side of the exchange,
 *   flexsp_plan_create            the per-micro-batch tile plan (lengths are known on the
 *                                 host before the step, Sec. 5 "Disaggregating Solving
 *                                 and Training"),
 *   flexsp_attn_varlen_fwd / _bwd Eq. 3 and its gradient over the packed stream.
 *
 * Conventions
 *   - Every function returns FLEXSP_OK (0) or a negative flexsp_status; nothing throws or
 *     aborts.  Arguments are validated before anything is launched.
 *   - "device pointer" = memory of the GPU the context was created on, owned by the
 *     caller; "host pointer" = ordinary host memory, copied before the call returns.
 *   - The four hot calls (pack, unpack, fwd, bwd) are asynchronous on the caller's HIP
 *     stream, allocate nothing and never synchronise the host.
 *   - The library owns only contexts and plans.  A plan is passed to the hot calls as a
 *     NON-const pointer on purpose: it owns device memory the kernels WRITE while they run
 *     (the ticket counters of its work queues, which the last workgroup of a launch clears
 *     again, and the backward's fp32 scratch), and the host side notes which stream used it
 *     last.  So a plan may be used by one in-flight forward and one in-flight backward at a
 *     time (each has its own queue counters); launches that share a plan must be ordered on
 *     one stream or by events, and two host threads must not launch through one plan at once.
 *   - There is no CPU fallback: without a usable gfx950 device the hot calls fail.
 */
#ifndef FLEXSP_H
#define FLEXSP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum flexsp_status {
    FLEXSP_OK = 0,
    FLEXSP_INVALID_ARGUMENT = -1, /* null pointer, negative size, non-monotone cu_seqlens, ... */
    FLEXSP_UNSUPPORTED = -2,      /* head dim not in {64,128}, element size not in {1,2,4,8,16}, ... */
    FLEXSP_PLAN_MISMATCH = -3,    /* call arguments disagree with the plan they were given */
    FLEXSP_HIP_ERROR = -4,        /* a HIP runtime call failed (see flexsp_last_hip_error) */
    FLEXSP_OUT_OF_MEMORY = -5,
    FLEXSP_NO_DEVICE = -6         /* no gfx950 device / context is host-only */
} flexsp_status;

/* Element type of the gradients written by the backward call. */
typedef enum flexsp_dtype { FLEXSP_BF16 = 0, FLEXSP_F32 = 1 } flexsp_dtype;

typedef struct flexsp_ctx flexsp_ctx;   /* opaque: device id, CU / XCD counts            */
typedef struct flexsp_plan flexsp_plan; /* opaque: tile queues (device + host copy), delta */
typedef void *flexsp_stream;            /* a hipStream_t owned by the caller; NULL = default stream */

/* Static, human-readable text for a status code. */
const char *flexsp_strerror(int status);
/* The hipError_t (as int) of the most recent FLEXSP_HIP_ERROR on this thread. */
int flexsp_last_hip_error(void);
/* Library version, "major.minor". */
const char *flexsp_version(void);

/*
 * Context.  flexsp_ctx_create binds to HIP device `device` (>= 0) and fails with
 * FLEXSP_NO_DEVICE if it does not exist or is not gfx950.  device == -1 creates a
 * HOST-ONLY context: plans can be built and inspected with it (for tests of the host
 * logic), every launch through it fails with FLEXSP_NO_DEVICE.
 * Creating or destroying a device context or one of its plans, and flexsp_profile_start,
 * leave the context's device as the calling thread's current HIP device; the hot calls do
 * not touch the current device (the stream they are given must belong to the context's
 * device).  Destroy every plan before its context.
 */
int flexsp_ctx_create(flexsp_ctx **out, int device);
void flexsp_ctx_destroy(flexsp_ctx *ctx);
/* Number of compute units / XCDs the scheduler assumes (0 / 8 for a host-only context). */
int flexsp_ctx_num_cu(const flexsp_ctx *ctx);
int flexsp_ctx_num_xcd(const flexsp_ctx *ctx);

/*
 * Tile plan for one packed batch.
 *   cu_seqlens_host  host pointer, B+1 int32 prefix sums: cu[0] = 0, non-decreasing,
 *                    cu[B] = T (tokens).  Sequence b owns tokens cu[b] .. cu[b+1]-1.
 *                    Empty sequences are allowed and contribute nothing.
 *   Hq, Hkv          query / key-value heads THIS GPU holds; Hq % Hkv == 0 (query head h
 *                    reads kv head h / (Hq/Hkv)).
 *   D                head dim, 64 or 128.
 *   causal           nonzero: key j of a sequence is visible to query i iff j <= i.
 * The plan lists work items (sequence, tile, head; the longest tiles cut into parts when few
 * heads and a dominant sequence would leave compute units waiting for them, see flexsp_item),
 * longest first (the tiles of a short sequence side by side, where its longest tile would stand),
 * in one queue per XCD, for the forward kernel and for the two backward kernels,
 * and holds the fp32 scratch the kernels need (delta and the base-2 log-sum-exp [Hq, T] for the
 * backward, one 66 KiB record per part of a cut tile), so the hot calls allocate nothing.
 * Everything is copied before the call returns; the caller keeps ownership of
 * cu_seqlens_host.  On a device context the queues go to the GPU with an asynchronous copy on
 * a stream of the context's own, and the first forward / backward call that uses the plan
 * makes its stream wait for that copy (a call made under stream capture should find the copy
 * finished: create the plan, let work that follows it complete, then capture).  Device and
 * pinned memory of destroyed plans is kept by the context (up to 16 buffers) and handed to new
 * plans (a buffer whose kernels have finished is preferred; a context makes at most four, 1 GiB
 * in all, before it reuses a busy one), so a plan per micro-batch costs neither an allocation
 * nor a device-wide synchronisation after the first steps.  When every buffer is still in use
 * by kernels, THIS CALL BLOCKS THE HOST until those of the buffer released first have finished:
 * a caller that makes a plan per step runs at most four steps ahead of the GPU.  A context, and
 * the plans made from it, belong to one host thread at a time.
 * Errors: INVALID_ARGUMENT, UNSUPPORTED (D), OUT_OF_MEMORY, HIP_ERROR.
 */
int flexsp_plan_create(flexsp_ctx *ctx, const int32_t *cu_seqlens_host, int32_t B,
                       int32_t Hq, int32_t Hkv, int32_t D, int causal, flexsp_plan **out);
void flexsp_plan_destroy(flexsp_plan *plan);

/* Plan inspection (host logic; works for host-only contexts).
 * A work item is one tile of one (sequence, head): 128 query rows (forward, dQ pass) walking the key
 * tiles they can see, or 64 keys (dK/dV pass) walking the query rows that see them, for every query
 * head of the kv head's group.  When a batch has so few, so long items that the longest would outlast
 * an even share of the whole pass (few heads, a dominant sequence: the usual case for a large
 * sequence-parallel group), the plan cuts such a tile's inner loop into `nparts` consecutive ranges,
 * one work item each; every part leaves its partial result (fp32) in the plan's scratch and the part
 * that finishes last adds them up in part order and writes the tile, so results do not depend on
 * which part that is. */
typedef struct flexsp_item {
    int32_t seq_start; /* first token of the sequence in the packed stream            */
    int32_t seq_len;   /* its length                                                   */
    int32_t tile;      /* tile index inside the sequence (query tile or key tile)      */
    int32_t head;      /* query head (forward, dQ pass) or kv head (dK/dV pass)        */
    int32_t step_begin; /* the item walks steps step_begin .. step_end-1 of the tile's inner loop    */
    int32_t step_end;   /* (a step = 64 keys for a query tile; 64 query rows of one head of the group
                           for a key tile, heads one after the other); a whole tile: 0 .. its step count */
    int32_t slot;       /* nparts > 1: first partial-result record of the tile; else -1              */
    int32_t parts;      /* (part << 16) | nparts: this item is part `part` of `nparts` of its tile
                           (0 and 1 for a whole tile)                                                */
} flexsp_item;
enum { FLEXSP_PASS_FWD = 0, FLEXSP_PASS_BWD_DKV = 1, FLEXSP_PASS_BWD_DQ = 2 };
/* Number of items of a pass, or a negative status. */
int64_t flexsp_plan_num_items(const flexsp_plan *plan, int pass);
/* Copies the items of a pass in queue order (queue 0 first) into `items` (host pointer,
 * capacity >= num_items) and the num_xcd+1 queue boundaries into `queue_offsets` (host
 * pointer, may be NULL). */
int flexsp_plan_get_items(const flexsp_plan *plan, int pass, flexsp_item *items,
                          int64_t capacity, int64_t *queue_offsets);
/* Rows per tile used by a pass (query rows for FWD and BWD_DQ, key rows for BWD_DKV). */
int flexsp_plan_tile_rows(const flexsp_plan *plan, int pass);
/* Bytes of device scratch the plan holds for the backward pass. */
size_t flexsp_attn_bwd_workspace_bytes(const flexsp_plan *plan);

/*
 * Layout permute, the local half of the exchanges in Eq. 2 / Eq. 4 (Sec. 2.1.2): a device
 * holds T tokens x all H heads ("sequence-sharded", Q_s in the paper) and regroups them
 * into one contiguous slab per peer, each slab holding H/P heads ("head-sharded", Q_h):
 *
 *   pack:    dst[r, t, h, :] = src[t, r*(H/P) + h, :]      src [T, H, D] -> dst [P, T, H/P, D]
 *   unpack:  dst[t, r*(H/P) + h, :] = src[r, t, h, :]      src [P, T, H/P, D] -> dst [T, H, D]
 *
 * Tokens are split evenly over the group irrespective of sequence boundaries (Sec. 4.1.2),
 * so no cu_seqlens is involved.  src and dst are device pointers to dense row-major
 * tensors of `elem_bytes`-byte elements (1, 2, 4, 8 or 16; pure bit copy), must not
 * overlap, and need T*H*D*elem_bytes bytes each.  Requires H % P == 0.  T == 0 is a no-op.
 * 16-byte accesses are used when (H/P)*D*elem_bytes and both base addresses are multiples
 * of 16, narrower ones otherwise.
 * Errors: INVALID_ARGUMENT, UNSUPPORTED, NO_DEVICE, HIP_ERROR.
 */
int flexsp_pack(flexsp_ctx *ctx, const void *src, void *dst, int64_t T, int32_t H, int32_t D,
                int32_t P, int32_t elem_bytes, flexsp_stream stream);
int flexsp_unpack(flexsp_ctx *ctx, const void *src, void *dst, int64_t T, int32_t H, int32_t D,
                  int32_t P, int32_t elem_bytes, flexsp_stream stream);

/*
 * The same permutes for up to FLEXSP_PACK_MANY_MAX tensors in ONE launch: the q, k, v slabs on
 * the way in (Eq. 2), the dq, dk, dv slabs on the way back.  Tensor i is [T, H[i], D] (the
 * head counts may differ: grouped-query K and V have fewer heads than Q); T, D, P and
 * elem_bytes are shared.  src, dst and H are HOST arrays of n entries (read before the call
 * returns); src[i] / dst[i] are device pointers with the requirements of flexsp_pack, and no
 * two of the 2n buffers may overlap.  Falls back to one launch per tensor when a tensor does
 * not qualify for 16-byte accesses or has 2^31 or more of them.  n == 0 or T == 0 is a no-op.
 * Errors: as flexsp_pack.
 */
#define FLEXSP_PACK_MANY_MAX 4
int flexsp_pack_many(flexsp_ctx *ctx, int32_t n, const void *const *src, void *const *dst, int64_t T,
                     const int32_t *H, int32_t D, int32_t P, int32_t elem_bytes, flexsp_stream stream);
int flexsp_unpack_many(flexsp_ctx *ctx, int32_t n, const void *const *src, void *const *dst, int64_t T,
                       const int32_t *H, int32_t D, int32_t P, int32_t elem_bytes, flexsp_stream stream);

/*
 * Strided view of a [T, heads, D] bf16 tensor in device memory: element (t, h, d) lives at
 * ptr + (t*stride_token + h*stride_head + d) elements.  The last dim is contiguous, ptr and
 * both strides (in elements) must keep every row 16-byte aligned (multiples of 8 elements);
 * stride_token <= 2^24 and stride_head < 2^30, else FLEXSP_INVALID_ARGUMENT.
 * A view lets a heads subset of a larger tensor be used in place.
 */
typedef struct flexsp_tensor {
    void *ptr;
    int64_t stride_token;
    int64_t stride_head;
} flexsp_tensor;

/*
 * Forward of Eq. 3 over the packed stream, per sequence and per head:
 *   O[i,h,:] = sum_j softmax_j(scale * q[i,h,:].k[j,g,:]) v[j,g,:],  g = kv head of h,
 *   j over the keys of i's own sequence (j <= i when causal),
 *   LSE[h,i] = natural-log-sum-exp of the scaled scores of row i.
 *   q, o              views of [T, *, D] bf16; heads head_begin .. head_begin+head_count-1 are used
 *   k, v              views of [T, *, D] bf16; kv heads kv_head_begin .. +kv_head_count-1
 *   cu_seqlens_dev    the device copy of the prefix sums (B+1 int32), or NULL.  The plan already
 *                     holds every length (its work items carry each sequence's start and size),
 *                     so the plan-based calls neither read nor check this array; it is part of
 *                     the signature because the path's callers have it at hand, and
 *                     flexsp_attn_varlen_fwd_static, which has no plan, works from it alone
 *   head_count, kv_head_count must equal the plan's Hq, Hkv
 *   softmax_scale     <= 0 selects 1/sqrt(D)
 *   lse               device pointer, fp32 [head_count, T]
 * Scores and softmax statistics are fp32; P is rounded to bf16 before the PV product;
 * accumulation is fp32; O is rounded to bf16 once.  Any finite input is handled; rows whose
 * scaled scores rise more than 44 (natural units) above the maximum of the row's first keys
 * are recomputed block by block by their wavefront, which costs time, not accuracy (a launch
 * in which every row does takes about 2.4 times as long).
 * Errors: INVALID_ARGUMENT, PLAN_MISMATCH, NO_DEVICE, HIP_ERROR.
 */
int flexsp_attn_varlen_fwd(flexsp_ctx *ctx, flexsp_plan *plan, flexsp_tensor q, flexsp_tensor k,
                           flexsp_tensor v, const int32_t *cu_seqlens_dev, int32_t head_begin,
                           int32_t head_count, int32_t kv_head_begin, int32_t kv_head_count,
                           int causal, float softmax_scale, flexsp_tensor o, float *lse,
                           flexsp_stream stream);

/*
 * Backward of Eq. 3 for the loss L = sum(O * dO): writes dq [T,*,D] (query heads as in q)
 * and dk, dv [T,*,D] (kv heads as in k; summed over the query heads of each group).
 * o and lse are the forward's outputs.  Softmax is recomputed from lse (no second
 * reduction); delta = rowsum(dO * O) is formed in fp32 in the plan's scratch.
 * grad_dtype selects the element type of dq, dk and dv (their strides count elements of that
 * type): FLEXSP_BF16 rounds the fp32 accumulators to bf16 once; FLEXSP_F32 stores them as
 * they are (useful when grouped-query sums grow past the range where bf16's spacing is fine
 * enough).  Results are deterministic (no floating-point atomics).
 * Errors: INVALID_ARGUMENT, UNSUPPORTED (grad_dtype), PLAN_MISMATCH, NO_DEVICE, HIP_ERROR.
 */
int flexsp_attn_varlen_bwd(flexsp_ctx *ctx, flexsp_plan *plan, flexsp_tensor q, flexsp_tensor k,
                           flexsp_tensor v, flexsp_tensor o, flexsp_tensor dO, const float *lse,
                           const int32_t *cu_seqlens_dev, int32_t head_begin, int32_t head_count,
                           int32_t kv_head_begin, int32_t kv_head_count, int causal,
                           float softmax_scale, flexsp_tensor dq, flexsp_tensor dk,
                           flexsp_tensor dv, int32_t grad_dtype, flexsp_stream stream);

/*
 * Attention against ONE SHARD of the keys, and the merge of such partial results: the per-device
 * work of context parallelism (Sec. 2.1.3, paragraph "Context Parallelism": queries, keys and values
 * are split along the sequence, key/value chunks travel round a ring and attention is computed chunk
 * by chunk; the appendix on integrating context parallelism into FlexSP).
 *
 * flexsp_plan_create_kvshard - tile plan for B sequences whose QUERIES are rows cu_q[b] .. cu_q[b+1]-1
 *   of q / o / lse and whose shard KEYS are rows cu_k[b] .. cu_k[b+1]-1 of k / v (host pointers, B+1
 *   int32 prefix sums each; either side may be empty for a sequence).  shift_host[b] (B int32,
 *   |shift| <= 2^30) = position of sequence b's first query inside the full sequence minus position of
 *   the shard's first key: with `causal`, shard key j is visible to query row i iff j <= i + shift[b];
 *   without, every shard key is visible and shift is ignored.  The plan serves
 *   flexsp_attn_varlen_fwd_kvshard (_acc) and flexsp_attn_varlen_bwd_kvshard only (the other attention calls
 *   answer PLAN_MISMATCH); it is destroyed by flexsp_plan_destroy and inspected by flexsp_plan_num_items /
 *   _get_items, where an item's seq_start holds the sequence INDEX b (and, in FLEXSP_PASS_BWD_DKV, tile
 *   counts 64-key tiles of the SHARD).  Long query tiles are cut into parts as in flexsp_plan_create (a
 *   step = 64 shard keys); key tiles are not.  Hq <= 65 535, else UNSUPPORTED.
 *
 * flexsp_attn_varlen_fwd_kvshard - per query row, softmax over the visible shard keys only:
 *   O = sum_j P_j v_j (bf16), LSE = log sum_j exp(scale q.k_j) (fp32, natural log, [head_count, Tq]).
 *   A row that sees no key of the shard gets O = 0 and LSE = -inf.  Arguments as flexsp_attn_varlen_fwd.
 *
 * flexsp_attn_varlen_fwd_kvshard_acc - the same attention folded straight into the fp32 running result of a
 *   ring, without writing the shard's own O and LSE and without a merge pass:
 *   (o_acc, lse_acc) <- merge((o_acc, lse_acc), (O, LSE) of the rows over this shard), as flexsp_lse_merge_acc
 *   does it (below), except that the shard's O enters in fp32, unrounded.  o_acc: view of [Tq, Hq, D] FP32;
 *   lse_acc fp32 [head_count, Tq]; start a ring with lse_acc = -inf (o_acc may then hold anything).  If
 *   o_bf16.ptr is not NULL the merged rows are also written there rounded to bf16 (view of [Tq, Hq, D]).
 *   Calls on the same o_acc must be ordered (one stream).
 *
 * flexsp_attn_varlen_bwd_kvshard - the backward's share of one key shard (gradient of Eq. 3 restricted to
 *   the shard's keys), for the same plan.  `lse` ([head_count, Tq] fp32, natural log) must be each row's
 *   log-sum-exp over ALL its keys and `o` the complete output (both as left by the merges of the forward
 *   ring), so that P_ij = exp(scale q_i.k_j - lse_i) and delta_i = dO_i . o_i are those of the complete
 *   attention; then, over the visible keys j of the shard,
 *       dQ_i = scale sum_j dS_ij k_j (this shard's part),  dK_j = scale sum_i dS_ij q_i,  dV_j = sum_i P_ij dO_i,
 *       dS_ij = P_ij (dO_i.v_j - delta_i).
 *   dq is [Tq, Hq, D], dk / dv are [Tk, Hkv, D] (rows of the shard), grad_dtype as in flexsp_attn_varlen_bwd.
 *   accumulate = 0: the three outputs are overwritten (rows and keys that see nothing get zeros);
 *   accumulate = 1 (fp32 gradients only, else UNSUPPORTED): the results are ADDED to what dq / dk / dv
 *   hold, as a ring needs it (dq gathers the shards' parts; dk / dv travel with their shard and gather
 *   the devices' parts).  A row whose lse is -inf contributes nothing.  Deterministic; the plan's scratch
 *   is used as in flexsp_attn_varlen_bwd (calls on one plan must not overlap).
 *
 * flexsp_lse_merge - two partial results of the same queries over DISJOINT key sets -> the result
 *   over their union:  LSE = log(exp(lse_a) + exp(lse_b)),  O = exp(lse_a - LSE) O_a + exp(lse_b - LSE) O_b
 *   (fp32 arithmetic, O rounded to bf16 once).  o_* are views of [T, H, D] bf16 (the H heads start at each
 *   view's ptr), lse_* fp32 [H, T] contiguous; D is 64 or 128.  A part with LSE = -inf counts nothing,
 *   whatever its O holds; both -inf: O = 0, LSE = -inf.  o_out / lse_out may be the very same memory as
 *   one of the inputs (merge in place), but must not overlap them otherwise.  Merging is associative up
 *   to rounding, so shards can be folded in as they arrive.
 *
 * flexsp_lse_merge_acc - the same merge with the running result kept in fp32, for rings of many shards
 *   (folding P parts into a bf16 result rounds it P - 1 times; here only `o_bf16` is rounded, once):
 *   (o_acc, lse_acc) <- merge((o_acc, lse_acc), (o_b, lse_b)) in place.  o_acc is a view of [T, H, D] FP32
 *   (strides in fp32 elements, rows 16-byte aligned), lse_acc fp32 [H, T]; o_b a bf16 view, lse_b fp32
 *   [H, T].  Start a ring with lse_acc = -inf everywhere (o_acc may then hold anything: a part with
 *   LSE = -inf counts nothing).  If o_bf16.ptr is not NULL the merged rows are also written there rounded
 *   to bf16 (a view of [T, H, D] bf16: what flexsp_attn_varlen_bwd_kvshard takes as `o`); pass it on the
 *   last fold, or on every one.
 * Errors: INVALID_ARGUMENT, UNSUPPORTED, PLAN_MISMATCH, NO_DEVICE, OUT_OF_MEMORY, HIP_ERROR.
 */
int flexsp_plan_create_kvshard(flexsp_ctx *ctx, const int32_t *cu_q_host, const int32_t *cu_k_host,
                               const int32_t *shift_host, int32_t B, int32_t Hq, int32_t Hkv, int32_t D,
                               int causal, flexsp_plan **out);
int flexsp_attn_varlen_fwd_kvshard(flexsp_ctx *ctx, flexsp_plan *plan, flexsp_tensor q, flexsp_tensor k,
                                   flexsp_tensor v, int32_t head_begin, int32_t head_count, int32_t kv_head_begin,
                                   int32_t kv_head_count, int causal, float softmax_scale, flexsp_tensor o,
                                   float *lse, flexsp_stream stream);
int flexsp_attn_varlen_fwd_kvshard_acc(flexsp_ctx *ctx, flexsp_plan *plan, flexsp_tensor q, flexsp_tensor k,
                                       flexsp_tensor v, int32_t head_begin, int32_t head_count,
                                       int32_t kv_head_begin, int32_t kv_head_count, int causal, float softmax_scale,
                                       flexsp_tensor o_acc, float *lse_acc, flexsp_tensor o_bf16, flexsp_stream stream);
int flexsp_attn_varlen_bwd_kvshard(flexsp_ctx *ctx, flexsp_plan *plan, flexsp_tensor q, flexsp_tensor k,
                                   flexsp_tensor v, flexsp_tensor o, flexsp_tensor dO, const float *lse,
                                   int32_t head_begin, int32_t head_count, int32_t kv_head_begin,
                                   int32_t kv_head_count, int causal, float softmax_scale, flexsp_tensor dq,
                                   flexsp_tensor dk, flexsp_tensor dv, int32_t grad_dtype, int32_t accumulate,
                                   flexsp_stream stream);
int flexsp_lse_merge(flexsp_ctx *ctx, flexsp_tensor o_a, const float *lse_a, flexsp_tensor o_b, const float *lse_b,
                     flexsp_tensor o_out, float *lse_out, int64_t T, int32_t H, int32_t D, flexsp_stream stream);
int flexsp_lse_merge_acc(flexsp_ctx *ctx, flexsp_tensor o_acc, float *lse_acc, flexsp_tensor o_b, const float *lse_b,
                         flexsp_tensor o_bf16, int64_t T, int32_t H, int32_t D, flexsp_stream stream);

/*
 * The forward for callers that cannot allocate: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same result as flexsp_attn_varlen_fwd, bit for bit, but it takes
 * no plan and calls no hipMalloc, hipFree or any other allocating routine: the work queues are built
 * on the device from `cu_seqlens_dev` (device pointer, B+1 int32 prefix sums, cu[0] = 0,
 * non-decreasing, cu[B] <= T) by a small kernel launched in front of the attention kernel, into a
 * fixed array of about 2 MiB that each GPU the library runs on holds from library load until the
 * process ends (its address on the context's device is resolved by flexsp_ctx_create).
 *   B, T            sequences in the batch; tokens the q / k / v / o tensors hold (rows of lse)
 *   D               head dim, 64 or 128; the remaining arguments are those of flexsp_attn_varlen_fwd
 * Limits: T <= 524 288 and (ceil(T / 128) + B) * head_count <= 65 536, else FLEXSP_UNSUPPORTED.
 * The lengths are read on the device only, so they cannot be checked by the host: if the device
 * array is not a valid prefix-sum list inside [0, T], NOTHING is computed (o and lse keep their
 * contents).  Every call on a GPU shares that GPU's array: calls that may overlap in time on one
 * GPU (different streams, or graph replays running concurrently) race; order them.  Sequences are
 * served longest tile first like a plan's queues, but without the plan's grouping of a head's tiles
 * onto one XCD, so it is somewhat slower than the plan-based call; nothing synchronises the host.
 * Errors: INVALID_ARGUMENT, UNSUPPORTED, NO_DEVICE, HIP_ERROR.
 */
int flexsp_attn_varlen_fwd_static(flexsp_ctx *ctx, flexsp_tensor q, flexsp_tensor k, flexsp_tensor v,
                                  const int32_t *cu_seqlens_dev, int32_t B, int64_t T, int32_t head_begin,
                                  int32_t head_count, int32_t kv_head_begin, int32_t kv_head_count, int32_t D,
                                  int causal, float softmax_scale, flexsp_tensor o, float *lse,
                                  flexsp_stream stream);

/*
 * ---------------------------------------------------------------------------------------------
 * Planner pieces that are exact and need no external solver (host only, no GPU involved).
 * All lengths are token counts, 0 <= s <= 2^40; arrays are host pointers.
 *
 * flexsp_bucket_dp - adaptive sequence bucketing (Sec. 4.1.3 "Problem Solving", the bucketing
 *   objective and its dynamic programme).  Groups K sequence lengths (any order) into at most Q
 *   buckets, bucket q holding the lengths in (limit[q-1], limit[q]], such that the total
 *   deviation sum_k (limit[bucket(k)] - s_k) is minimal.
 *     limits       out, capacity Q: the buckets' upper limits, ascending (each is one of the lengths)
 *     num_buckets  out: how many limits were written (< Q when fewer distinct lengths exist)
 *     bucket_of    out, K entries, or NULL: bucket index of every input length
 *     error        out: the minimal total deviation
 *
 * flexsp_chunk_dp - memory-balanced micro-batch chunking (Appendix A, the min-max objective and
 *   its dynamic programme).  Splits the K lengths, IN THE GIVEN ORDER, into M consecutive,
 *   non-empty micro-batches so that the largest micro-batch token count is minimal (1 <= M <= K).
 *     ends         out, M entries: ends[i] = index one past the last sequence of micro-batch i
 *                  (ends[M-1] = K).  When several splits are optimal, one of them.
 *     max_tokens   out: the minimal possible largest micro-batch token count
 *
 * flexsp_min_microbatches - smallest feasible micro-batch count (Sec. 4.2, takeaway #1):
 *   ceil(batch_tokens / cluster_token_capacity); negative status for invalid arguments.
 *
 * Errors: INVALID_ARGUMENT (null pointers, negative or oversized lengths, Q <= 0, M outside
 * 1..K), UNSUPPORTED (K >= 2^31), OUT_OF_MEMORY.
 */
int flexsp_bucket_dp(const int64_t *lens, int64_t K, int32_t Q, int64_t *limits, int32_t *num_buckets,
                     int32_t *bucket_of, int64_t *error);
int flexsp_chunk_dp(const int64_t *lens, int64_t K, int32_t M, int64_t *ends, int64_t *max_tokens);
int64_t flexsp_min_microbatches(int64_t batch_tokens, int64_t cluster_token_capacity);

/*
 * Per-kernel timing for benchmarks.  Between flexsp_profile_start and flexsp_profile_stop every
 * kernel launched through `ctx` is bracketed by a pair of HIP events on the caller's stream.
 * flexsp_profile_stop waits for the recorded events (it synchronises the host), adds up the
 * elapsed time and the number of launches per kernel and turns recording off.  At most
 * `max_launches` launches are recorded (events are created by flexsp_profile_start, none in
 * the hot calls); later ones run untimed and are counted in `dropped`.
 * Errors: INVALID_ARGUMENT, NO_DEVICE, HIP_ERROR, OUT_OF_MEMORY.
 */
enum {
    FLEXSP_K_PACK = 0,
    FLEXSP_K_UNPACK = 1,
    FLEXSP_K_FWD = 2,
    FLEXSP_K_BWD_DELTA = 3, /* reserved: the row-dot preprocessing is part of the dQ kernel, never launched */
    FLEXSP_K_BWD_DKV = 4,
    FLEXSP_K_BWD_DQ = 5,
    FLEXSP_K_COUNT = 6
};
typedef struct flexsp_profile {
    double ms[FLEXSP_K_COUNT];        /* summed kernel time, milliseconds */
    int64_t launches[FLEXSP_K_COUNT]; /* launches recorded                */
    int64_t dropped;                  /* launches beyond max_launches     */
} flexsp_profile;
int flexsp_profile_start(flexsp_ctx *ctx, int32_t max_launches);
int flexsp_profile_stop(flexsp_ctx *ctx, flexsp_profile *out);

#ifdef __cplusplus
}
#endif
#endif /* FLEXSP_H */
