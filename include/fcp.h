/*
 * fcp.h -- C ABI of the MI355X block-level attention library (one FCP worker).
 *
 * The paper splits every sequence of a batch into fixed-size blocks (section
 * "Block Distributor", sharding policy), derives the (query block, KV block)
 * dependencies from the attention mask (Zig-Zag figure caption; congestion-free
 * solver figure), coalesces c consecutive KV blocks into one execution stage
 * (section "Communication Planner", bottom-up coalescer), runs a flash-style
 * attention kernel per stage and reduces the per-stage results to the final
 * output (section "Context Parallelism": attention over slices of the context is
 * associative).  This library is the part one worker executes once every KV
 * block its dependencies name is resident in its HBM.
 *
 * Conventions for every entry point
 *   - returns FCP_OK (0) or a negative fcp_status; never throws or aborts;
 *     fcp_last_error() gives the text for the calling thread's last failure.
 *   - "host" pointers are ordinary CPU memory, "device" pointers are HIP device
 *     memory of the current device.  The library allocates no device memory:
 *     tensors, tables and the workspace are caller-allocated and caller-freed.
 *   - kernels are enqueued on the given hipStream_t (passed as void*; NULL = the
 *     default stream) and the call returns without waiting, except
 *     fcp_queue_build which returns after its upload has completed.
 *   - tensor layout is packed token-major: Q, O, dO, dQ [T_q, Hq, d];
 *     K, V, dK, dV [T_kv, Hkv, d]; LSE, D [T_q, Hq]; row-major, no padding.
 *     Q/K/V/dO are bf16; partial O, LSE, dQ/dK/dV are fp32; final O is bf16 or
 *     fp32 (FCP_FLAG_O_F32).  Query head h reads KV head h * Hkv / Hq.
 */
#ifndef FCP_H_
#define FCP_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  FCP_OK = 0,
  FCP_ERR_INVALID_ARG = -1,      /* null pointer, negative size, owned block out of range ... */
  FCP_ERR_BUFFER_TOO_SMALL = -2, /* a table capacity (or the workspace) is too small; needed counts are written back */
  FCP_ERR_UNSUPPORTED = -3,      /* head_dim not in {64,128}, Hq % Hkv != 0, ... */
  FCP_ERR_HIP = -4,              /* a HIP call failed; see fcp_last_error() */
  FCP_ERR_INFEASIBLE = -5        /* the scheduling problem has no solution under the given limits */
} fcp_status;

/* Kind of a pair: which (row, column) entries of query block x KV block are attended.
 *   FULL: all of them.  DIAG: the same block on both sides under a causal mask: column <= row.
 *   PACKED_FULL / PACKED_DIAG: the same packed block on both sides (a block that holds several whole short
 *   sequences, see fcp_segment): FULL / DIAG restricted to entries whose row and column lie in the same member. */
enum { FCP_KIND_FULL = 0, FCP_KIND_DIAG = 1, FCP_KIND_PACKED_FULL = 2, FCP_KIND_PACKED_DIAG = 3 };

/* One fixed-size block of one sequence (the paper's scheduling, compute and transfer unit). */
typedef struct { int32_t seq, idx, tok_start, tok_len; } fcp_block;
/* One work item of the dependency list: query block x KV block, FULL or causal-diagonal. */
typedef struct { int32_t q_blk, kv_blk, kind, slot; } fcp_pair;
/* One execution stage of a query block: up to c consecutive pairs -> one partial (O, LSE). */
typedef struct { int32_t q_blk, pair_begin, n_pairs, row_start; } fcp_slot;
/* One member sequence of a packed block: tokens [tok_off, tok_off + tok_len) of KV block kv_blk are the whole
 * sequence seq.  The members of a block are listed in token order and tile it exactly. */
typedef struct { int32_t kv_blk, seq, tok_off, tok_len; } fcp_segment;

enum {
  FCP_FLAG_O_F32 = 1,            /* the final O is fp32 instead of bf16 (the backward then reads fp32 O) */
  FCP_FLAG_PART_BF16 = 4,        /* the partial O buffer (o_part) holds bf16 instead of fp32: half the memory and half the
                                    traffic of the partials; LSE partials stay fp32.  Set it for every call on a problem.
                                    A final O merged from bf16 partials carries bf16 rounding whatever its own dtype:
                                    meant for forward-only use (the backward's D = rowsum(dO o O) inherits it). */
  FCP_FLAG_GRAD_BF16 = 8,        /* the backward writes dq, dk, dv as bf16 instead of fp32 */
  FCP_FLAG_BWD_SPILL_DS = 16,    /* the backward keeps dS (bf16, scale folded in) of every visible 32x32 score tile in the
                                    workspace: the dK/dV kernel, which computes it anyway, writes it, and dQ = dS K is then
                                    one streaming contraction (fcp_block_attn_bwd_dq_ds) instead of a second kernel that
                                    recomputes S and dP.  Costs 2 bytes of workspace per unmasked score entry and query head
                                    (rounded up to 32x32 tiles; fcp_workspace_bytes accounts for it) and trades two of the
                                    backward's seven executed contractions for that much HBM traffic each way.  Set it
                                    before fcp_workspace_bytes / fcp_queue_build and keep it for every call on the
                                    workspace.  Shares whose dS does not fit in memory leave it unset. */
  FCP_FLAG_RUNNING_MERGE = 32,   /* fcp_block_attn_fwd_out folds the result of every slot into the running (o, lse) in place instead of
                                    writing a partial: (O, LSE) <- merge((O, LSE), slot result), the two-way form of the reduction that
                                    fcp_merge_partials does in one go.  One launch handles ONE stage: the problem may hold at most one
                                    slot per query block (fcp_stage_tables cuts a plan into such stages), launches of successive
                                    stages go to one stream, and before the first one the caller fills lse with -inf (o is then
                                    ignored).  Needs FCP_FLAG_O_F32; the partial buffers are not touched and may be NULL; no merge call
                                    follows.  The worker then holds no partials at all, at the price of reading and writing the
                                    running result once per stage. */
  FCP_FLAG_DIRECT_SINGLE = 2     /* a query block with ONE slot needs no reduction: fcp_block_attn_fwd_out writes its
                                    result straight to the final o / lse and fcp_merge_partials leaves it alone.
                                    Set it before fcp_workspace_bytes / fcp_queue_build and keep it for every call
                                    on that workspace; with it, call fcp_block_attn_fwd_out, not fcp_block_attn_fwd. */
};

/* Problem descriptor.  All table pointers are HOST pointers to tables produced by
 * fcp_plan_blocks (or built by the caller to the same rules). */
typedef struct {
  int32_t n_q_heads, n_kv_heads, head_dim, block_size;
  float   softmax_scale;         /* 0 -> 1/sqrt(head_dim) */
  int32_t flags;
  int32_t n_kv_blocks, n_q_blocks, n_pairs, n_slots, n_slot_rows;
  const fcp_block* kv_blocks;
  const fcp_block* q_blocks;
  const fcp_pair*  pairs;
  const fcp_slot*  slots;
  int32_t n_segments;            /* 0 unless the tables come from fcp_plan_blocks_packed */
  const fcp_segment* segments;   /* members of the packed blocks, by (kv_blk, tok_off); NULL when n_segments is 0 */
} fcp_problem;

/*
 * fcp_plan_blocks -- sharding policy G and the worker's dependency list (host, integer only).
 *
 * Paper: section "Block Distributor" (every sequence is cut into fixed-size blocks, more blocks
 * for longer sequences; a sequence shorter than a block is one ragged block handled by the
 * variable-length path); Zig-Zag figure caption (under a causal mask the i-th query block
 * computes with KV blocks 0..i of its sequence); bottom-up coalescer (c sub-stages per stage).
 *
 * seq_lens[n_seqs]  host; length of every sequence whose KV is resident (>= 0; 0 -> no block).
 * block_size > 0; causal 0/1; coalesce c >= 1, or 0 = all KV blocks of a query block in one slot.
 * q_owned           host; n_q_owned rows of (seq, idx_in_seq), strictly increasing; NULL = the
 *                   worker owns the query side of every block.
 * Tables (host, caller-allocated): *n_x holds the capacity on entry and the count on return.
 * A NULL table pointer makes the call a size query (counts only).  If a capacity is too small
 * the counts are still written and FCP_ERR_BUFFER_TOO_SMALL is returned.
 *   kv_blocks: all blocks by (seq, idx); tok_start = row in the K/V buffers.
 *   q_blocks : owned blocks by (seq, idx); tok_start = row in the Q buffer (owned blocks packed).
 *   pairs    : by (q_blk, kv_blk); causal -> FULL for j < i, DIAG for j == i; else FULL for all j.
 *   slots    : the r-th pair of a query block belongs to its local slot r / c; slots are numbered
 *              globally in pair order; slot rows [row_start, row_start + tok_len) of the partial
 *              buffers belong to it.  *n_slot_rows = total rows of the partial buffers.
 */
int fcp_plan_blocks(const int32_t* seq_lens, int32_t n_seqs, int32_t block_size,
                    int32_t causal, int32_t coalesce,
                    const int32_t* q_owned, int32_t n_q_owned,
                    fcp_block* kv_blocks, int32_t* n_kv_blocks,
                    fcp_block* q_blocks, int32_t* n_q_blocks,
                    fcp_pair* pairs, int32_t* n_pairs,
                    fcp_slot* slots, int32_t* n_slots,
                    int32_t* n_slot_rows);

/*
 * fcp_plan_blocks_packed -- fcp_plan_blocks in which the short sequences of a scheduling unit share ONE block.
 *
 * Paper: section "Block Distributor", sharding policy: sequences shorter than the block size are packed into as few
 * blocks as possible and computed through the kernel's variable-length path.  Here such a block is one block of the
 * tables, one slot and one chain of work items for the kernels, and the variable-length path is the mask of the
 * PACKED pair kinds: a query row sees the keys of its own member sequence only.
 *
 * unit_of_block[n]: host; the scheduling unit of every block of the unpacked table (the blocks fcp_block_costs and
 * fcp_plan_blocks list, by (seq, idx)), as written by fcp_pack_units.  A unit with two or more blocks becomes one
 * packed block; each of its blocks must be a whole sequence shorter than block_size and their lengths must sum
 * to at most block_size (FCP_ERR_INVALID_ARG otherwise).  Every other block is planned as by fcp_plan_blocks.
 * Tables, and what differs from fcp_plan_blocks:
 *   kv_blocks: in the order of the unpacked table, a packed block standing where its lowest member stood (the other
 *              members are gone): seq = that member's sequence, idx = 0, tok_len = the sum of the members.  tok_start
 *              is again the running sum, so the K / V buffers hold the tokens in THIS order: the members of a packed
 *              block next to each other, in ascending order of their unpacked block index.
 *   q_blocks : the owned blocks in the same order.  q_owned still lists unpacked (seq, idx) rows; a unit is owned as
 *              a whole or not at all (FCP_ERR_INVALID_ARG otherwise).
 *   pairs    : a packed query block has ONE pair, with itself: PACKED_DIAG if causal, else PACKED_FULL; one slot.
 *   segments : the members of every packed block, by (kv_blk, tok_off); *n_segments = capacity / count as for the
 *              other tables (a NULL segments pointer with the other four tables NULL is the size query).
 * With no multi-block unit the four tables equal those of fcp_plan_blocks and *n_segments is 0.
 */
int fcp_plan_blocks_packed(const int32_t* seq_lens, int32_t n_seqs, int32_t block_size,
                           int32_t causal, int32_t coalesce,
                           const int32_t* q_owned, int32_t n_q_owned,
                           const int32_t* unit_of_block,
                           fcp_block* kv_blocks, int32_t* n_kv_blocks,
                           fcp_block* q_blocks, int32_t* n_q_blocks,
                           fcp_pair* pairs, int32_t* n_pairs,
                           fcp_slot* slots, int32_t* n_slots,
                           int32_t* n_slot_rows,
                           fcp_segment* segments, int32_t* n_segments);

/*
 * fcp_stage_tables -- the tables of one execution stage of a plan (host, integer only).
 *
 * Paper: section "Communication Planner": a worker runs its stages one after the other (the KV blocks of a stage
 * arrive while the previous stage computes) and reduces each stage's result into what it has so far.  Stage k of a
 * plan = the k-th slot of every query block that has one.  The stage's tables describe the same blocks with only
 * those slots: pairs keep their (q_blk, kv_blk, kind) and point at the renumbered slots; a slot's row_start is its
 * query block's tok_start, so that a partial buffer of the stage has the layout of the final output
 * (n_slot_rows = all query tokens).  Together with the plan's block tables they form a valid fcp_problem.
 * pairs / slots / q_blocks: the plan's tables (host).  stage >= 0.
 * stage_pairs / stage_slots: host, caller-allocated; *n_stage_pairs / *n_stage_slots hold the capacities on entry
 * and the counts on return (NULL tables = size query; too small = FCP_ERR_BUFFER_TOO_SMALL with the counts written).
 * *n_stages = the largest number of slots any query block has (stages beyond it are empty, which is not an error).
 */
int fcp_stage_tables(const fcp_pair* pairs, int32_t n_pairs, const fcp_slot* slots, int32_t n_slots,
                     const fcp_block* q_blocks, int32_t n_q_blocks, int32_t stage,
                     fcp_pair* stage_pairs, int32_t* n_stage_pairs, fcp_slot* stage_slots, int32_t* n_stage_slots,
                     int32_t* n_stages);

/*
 * fcp_workspace_bytes -- size of the device workspace that fcp_queue_build fills for `p`.
 * Validates the descriptor (table consistency, supported shapes).
 */
int fcp_workspace_bytes(const fcp_problem* p, size_t* bytes);

/*
 * fcp_queue_build -- work-queue scheduler, host part.
 *
 * Paper analogue: the attention kernel is launched with a margin of idle units to dodge wave
 * quantisation (section "Implementation"); here the pair list is expanded into weighted work
 * items (forward: slot x query tile x query head; backward: KV tile x KV head with its list of
 * dependent query blocks for dK/dV, query block x tile x head for dQ; merge: row ranges), ordered heavy-first and spread over the chip's
 * eight XCD queues, which persistent workgroups drain through atomic counters.
 *
 * workspace: device, >= fcp_workspace_bytes, 256-byte aligned; owned by the caller, must stay
 * untouched between this call and the last fwd/merge/bwd call that uses it.  Calls using one
 * workspace must not overlap in time (they share its counters).  Synchronises `stream`.
 */
int fcp_queue_build(const fcp_problem* p, void* workspace, size_t workspace_bytes, void* stream);

/*
 * fcp_block_attn_fwd -- partial attention of every slot (flash-style, online softmax).
 *
 * Paper: section "Attention Computation" (O = Softmax(Q K^T / sqrt(D), mask) V) restricted to
 * the KV blocks of one stage; per-row log-sum-exp kept so that stages can be reduced later.
 * For slot s of query block b, rows r < tok_len(b):
 *   o_part [row_start(s) + r, h, :] = softmax over the slot's visible keys (normalised)
 *   lse_part[row_start(s) + r, h]   = ln sum exp(scale * q.k) over those keys
 * q [T_q,Hq,d], k, v [T_kv,Hkv,d]: device bf16.  o_part [n_slot_rows,Hq,d] (fp32, or bf16 with FCP_FLAG_PART_BF16), lse_part
 * [n_slot_rows,Hq]: device fp32, fully overwritten.  workspace: as built by fcp_queue_build.
 */
int fcp_block_attn_fwd(const fcp_problem* p, const void* q, const void* k, const void* v,
                       void* o_part, float* lse_part, void* workspace, void* stream);

/*
 * fcp_block_attn_fwd_out -- fcp_block_attn_fwd that also knows the final outputs.
 *
 * Paper: section "Context Parallelism": the per-stage results of a query block are reduced to
 * its final output; with a single stage the reduction is the identity.  With
 * FCP_FLAG_DIRECT_SINGLE set, the slot of a query block that has exactly one slot is written
 * to o / lse (rows tok_start .. of the query block; dtype of o per FCP_FLAG_O_F32) instead of
 * the partial buffers, whose rows for that slot are left untouched; all other slots go to
 * o_part / lse_part as in fcp_block_attn_fwd.  Without the flag it behaves exactly like
 * fcp_block_attn_fwd and ignores o / lse.  o [T_q,Hq,d], lse [T_q,Hq]: device.
 */
int fcp_block_attn_fwd_out(const fcp_problem* p, const void* q, const void* k, const void* v,
                           void* o_part, float* lse_part, void* o, float* lse,
                           void* workspace, void* stream);

/*
 * fcp_block_attn_fwd_static -- fcp_block_attn_fwd for callers that cannot allocate device memory or keep a
 * workspace (code under HIP graph capture set-up, tight serving loops, harnesses that forbid hipMalloc).
 *
 * Same result as fcp_queue_build + fcp_block_attn_fwd, bit for bit, with no workspace argument: the
 * forward's queue tables (header with the queue counters, resolved pairs, forward work items) are built
 * on the host at every call and copied into a fixed array of 2 MiB inside the library's device image,
 * which every device the library runs on holds until the process ends.  The call allocates no device
 * memory (no hipMalloc / hipFree, no allocating library routine); it waits on `stream` for its table
 * copy, then enqueues the kernel and returns.
 * Limits and errors: FCP_ERR_BUFFER_TOO_SMALL if the tables need more than 2 MiB (about 25 000 forward
 * work items: the packed 64K-token training batch fits, the 1M-token share does not);
 * FCP_ERR_INVALID_ARG with FCP_FLAG_DIRECT_SINGLE (every slot goes to the partial buffers here);
 * otherwise as fcp_block_attn_fwd.  All calls on one device share that device's array, counters
 * included: calls that overlap in time on one device race, whatever their streams.
 */
int fcp_block_attn_fwd_static(const fcp_problem* p, const void* q, const void* k, const void* v,
                              void* o_part, float* lse_part, void* stream);

/*
 * fcp_merge_partials -- reduce the partials of each query block to the final output.
 *
 * Paper: section "Context Parallelism" (intermediate results over slices are reduced to the
 * final outputs).  LSE = ln sum_p exp(LSE_p); O = sum_p exp(LSE_p - LSE) O_p; exp(-inf) = 0;
 * a row with only empty partials gets O = 0, LSE = -inf.
 * o [T_q,Hq,d]: device, bf16 (default) or fp32 (FCP_FLAG_O_F32); lse [T_q,Hq]: device fp32.
 * With FCP_FLAG_DIRECT_SINGLE, query blocks with one slot are skipped (fcp_block_attn_fwd_out wrote them).
 */
int fcp_merge_partials(const fcp_problem* p, const void* o_part, const float* lse_part,
                       void* o, float* lse, void* workspace, void* stream);

/*
 * fcp_block_attn_bwd -- gradients of the worker's share.
 *
 * Paper: section "Attention Computation" states that the backward pass is implemented alongside
 * the forward; this is the analytic gradient of the forward definition, recomputing P from the
 * final LSE: D = rowsum(dO o O); P = exp(scale q.k - LSE); dV += P^T dO; dP = dO V^T;
 * dS = P o (dP - D); dQ += scale dS K; dK += scale dS^T Q; dK/dV are summed over the query
 * heads of a KV head and hold only the owned query rows' contribution.
 * o: final O as written by fcp_merge_partials (dtype per flags); lse: final LSE; d_o bf16.
 * dq [T_q,Hq,d], dk, dv [T_kv,Hkv,d]: device fp32, or bf16 with FCP_FLAG_GRAD_BF16 (the fp32 sums are
 * rounded to nearest-even once, in the kernel that holds them: no cast pass); fully overwritten; every
 * row has exactly one writer and a fixed summation order, so results are bit-reproducible from run to run.
 */
int fcp_block_attn_bwd(const fcp_problem* p, const void* q, const void* k, const void* v,
                       const void* o, const float* lse, const void* d_o,
                       void* dq, void* dk, void* dv, void* workspace, void* stream);

/*
 * The stages of the backward as separate calls, so that a caller can time or overlap them.  fcp_block_attn_bwd
 * itself runs fcp_block_attn_bwd_dq_d (below) followed by fcp_block_attn_bwd_dkdv.
 * fcp_bwd_preprocess:      computes D = rowsum(dO o O) and leaves scale*D and log2(e)*LSE
 *                          ([Hq,T_q] fp32 each) in the workspace.
 * fcp_block_attn_bwd_dkdv: KV-stationary kernel, writes dk and dv.
 * fcp_block_attn_bwd_dq:   query-stationary kernel, writes dq.
 * The last two need fcp_bwd_preprocess (or, for fcp_block_attn_bwd_dkdv, fcp_block_attn_bwd_dq_d) to have run on
 * the same workspace (same stream, or ordered after it) with the same o / lse / d_o, and are independent of each other.
 * Arguments, layouts and errors as for fcp_block_attn_bwd.
 */
int fcp_bwd_preprocess(const fcp_problem* p, const void* o, const float* lse, const void* d_o,
                       void* workspace, void* stream);
int fcp_block_attn_bwd_dkdv(const fcp_problem* p, const void* q, const void* k, const void* v,
                            const void* d_o, void* dk, void* dv, void* workspace, void* stream);
int fcp_block_attn_bwd_dq(const fcp_problem* p, const void* q, const void* k, const void* v,
                          const void* d_o, void* dq, void* workspace, void* stream);

/*
 * fcp_block_attn_bwd_dq_d -- fcp_block_attn_bwd_dq that needs no fcp_bwd_preprocess: the kernel computes
 * D = rowsum(dO o O) for the rows of each work item itself (it holds their dO already) and leaves scale*D and
 * log2(e)*LSE in the workspace, where a later fcp_block_attn_bwd_dkdv on the same workspace finds them.
 * fcp_block_attn_bwd = this call followed by fcp_block_attn_bwd_dkdv.
 * o / lse: the forward's final outputs, as for fcp_block_attn_bwd.
 */
int fcp_block_attn_bwd_dq_d(const fcp_problem* p, const void* q, const void* k, const void* v,
                            const void* o, const float* lse, const void* d_o, void* dq,
                            void* workspace, void* stream);

/*
 * fcp_block_attn_bwd_dq_ds -- dQ from the dS that fcp_block_attn_bwd_dkdv left in the workspace (FCP_FLAG_BWD_SPILL_DS).
 *
 * dQ[i, h, :] = sum_j dS[i, j] K[j, :] over the visible keys j of row i, with dS = P o (dP - D) * scale as the dK/dV
 * kernel formed and rounded it (same backward definition as fcp_block_attn_bwd).  Needs fcp_block_attn_bwd_dkdv to
 * have run on the same workspace with the flag set (same stream, or ordered after it).  k: device bf16 [T_kv,Hkv,d];
 * dq: device [T_q,Hq,d] fp32 (bf16 with FCP_FLAG_GRAD_BF16), fully overwritten, one writer per row.
 * Errors: FCP_ERR_INVALID_ARG when the flag is not set or a pointer is NULL; otherwise as fcp_block_attn_bwd.
 * With the flag, fcp_block_attn_bwd = fcp_bwd_preprocess, fcp_block_attn_bwd_dkdv, then this call.
 */
int fcp_block_attn_bwd_dq_ds(const fcp_problem* p, const void* k, void* dq, void* workspace, void* stream);

/* Text of the calling thread's last error ("" if none).  The pointer stays valid until the
 * thread's next failing call. */
const char* fcp_last_error(void);

/* Persistent grid sizes used by the kernels on the current device (for reports). */
int fcp_device_info(int32_t* n_compute_units, int32_t* fwd_grid, int32_t* bwd_grid);

#ifdef __cplusplus
}
#endif
#endif /* FCP_H_ */
