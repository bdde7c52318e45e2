/*
 * fcp_sched.h -- C ABI of the host-side scheduling of FCP: which worker owns which block,
 * which blocks travel between workers, and in what order they travel.
 *
 * Everything here is host code on host memory (integers and IEEE doubles, no GPU, no
 * allocation that outlives a call).  The output of fcp_assign_blocks, turned into a worker's
 * list of owned blocks by fcp_worker_blocks, is the q_owned argument of fcp_plan_blocks.
 * Conventions as in fcp.h: every call returns FCP_OK or a negative fcp_status and leaves the
 * text of a failure in fcp_last_error(); tables are caller-allocated; a count argument holds
 * the capacity on entry and the count on return, a NULL table makes the call a size query,
 * and a capacity that is too small still writes the count and returns FCP_ERR_BUFFER_TOO_SMALL.
 */
#ifndef FCP_SCHED_H_
#define FCP_SCHED_H_

#include "fcp.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * fcp_block_costs -- the blocks of a batch and the two costs the assignment balances.
 *
 * Paper: appendix "Block Assignment Algorithm" (every block i has a memory usage m_i and a
 * compute amount c_i that depends on the context length of its sequence); section "Block
 * Distributor" (fixed-size blocks, the last one of a sequence ragged).
 *   mem[i]  = tokens of block i;
 *   comp[i] = unmasked score entries of the block's query rows, per head: a row at position p of
 *             a sequence of length L attends p + 1 keys under a causal mask, L keys otherwise.
 * blocks: by (seq, idx); tok_start = row in the packed token buffer of the whole batch.
 * seq_lens[n_seqs] >= 0, block_size > 0, causal 0/1.
 */
int fcp_block_costs(const int32_t* seq_lens, int32_t n_seqs, int32_t block_size, int32_t causal,
                    fcp_block* blocks, int64_t* mem, int64_t* comp, int32_t* n_blocks);

/*
 * fcp_pack_units -- scheduling units: short sequences share a unit, every other block is its own.
 *
 * Paper: section "Block Distributor", sharding policy (sequences shorter than the block size are
 * packed into as few blocks as possible and computed through the variable-length path).  The paper
 * names no packing rule; this is first-fit decreasing: the blocks of single-block sequences with
 * fewer than block_size tokens, in descending length (equal lengths: lower block index first), each
 * go into the first open unit that still has room for them, else open a new unit.  Units are
 * numbered by their lowest member block.  For fcp_plan_blocks a unit's blocks stay separate ragged
 * blocks (the unit only makes them travel and get assigned together); fcp_plan_blocks_packed takes
 * unit_of_block and turns every unit of two or more blocks into one block for the kernels.
 * blocks / mem / comp: as written by fcp_block_costs.  unit_of_block[n_blocks]: out.
 * unit_mem / unit_comp: out, summed costs, capacity *n_units on entry (n_blocks always suffices);
 * *n_units: count on return.  Feed unit_mem / unit_comp to fcp_assign_blocks; the owner of block b
 * is then owner[unit_of_block[b]].
 */
int fcp_pack_units(const fcp_block* blocks, const int64_t* mem, const int64_t* comp, int32_t n_blocks,
                   int32_t block_size, int32_t* unit_of_block, int64_t* unit_mem, int64_t* unit_comp,
                   int32_t* n_units);

/*
 * fcp_assign_blocks -- Greedy Load-Balanced Assignment (the paper's appendix algorithm of that name).
 *
 * m_hat = sum(mem) / N, c_hat = sum(comp) / N.  Blocks are taken in descending order of
 * max(mem_i / m_hat, comp_i / c_hat) (equal keys: lower block index first); each goes to the
 * worker w that minimises max(alpha (m_w + mem_i) / m_hat, beta (c_w + comp_i) / c_hat) among the
 * workers with m_w + mem_i <= mem_limit (1 + delta) (equal loads: lowest worker index).  A cost
 * whose sum is zero contributes 0 to keys and loads.  mem_limit <= 0: no limit.
 * All loads are IEEE doubles computed as written above, so the result is reproducible bit for bit.
 *
 * owner[n_blocks]: out, worker of every block.  worker_mem / worker_comp [n_workers]: out, final
 * loads; either may be NULL.  Costs must be >= 0.
 * Errors: FCP_ERR_INVALID_ARG (NULL, negative cost, n_workers <= 0, alpha/beta/delta negative or NaN);
 * FCP_ERR_INFEASIBLE when some block fits on no worker (owner[] is then unspecified).
 */
int fcp_assign_blocks(const int64_t* mem, const int64_t* comp, int32_t n_blocks, int32_t n_workers,
                      double alpha, double beta, int64_t mem_limit, double delta,
                      int32_t* owner, int64_t* worker_mem, int64_t* worker_comp);

/*
 * fcp_worker_blocks -- the (seq, idx) rows of the blocks one worker owns, in block order: the
 * q_owned table of fcp_plan_blocks.  q_owned: n rows of two int32.
 */
int fcp_worker_blocks(const fcp_block* blocks, const int32_t* owner, int32_t n_blocks, int32_t worker,
                      int32_t* q_owned, int32_t* n_q_owned);

/* One block transfer: KV block kv_blk (index into the block table) goes from worker src to
 * worker dst in sub-stage `stage` (-1 until a solver has run). */
typedef struct { int32_t src, dst, kv_blk, stage; } fcp_edge;

/*
 * fcp_comm_edges -- the data flow as a bipartite multigraph of send and receive nodes.
 *
 * Paper: section "Communication Planner", congestion-free solver (an edge S(i) -> R(j) for every
 * block that must travel from worker i to worker j) and the caption of its figure.  A query block
 * (s, i) depends on KV blocks (s, j) with j <= i under a causal mask, every j otherwise; a worker
 * pulls a remote block once however many of its query blocks need it.
 * blocks: as written by fcp_block_costs (by (seq, idx)); owner[i] in [0, n_workers).
 * edges: out, ordered by (kv_blk, dst), stage = -1.  n_edges: capacity in, count out.
 */
int fcp_comm_edges(const fcp_block* blocks, const int32_t* owner, int32_t n_blocks, int32_t n_workers,
                   int32_t causal, fcp_edge* edges, int64_t* n_edges);

/*
 * fcp_solve_matchings -- congestion-free ordering: every edge gets a sub-stage in [0, Delta) such
 * that in one sub-stage no worker sends twice and no worker receives twice, Delta being the largest
 * number of blocks any worker sends or receives.
 *
 * Paper: section "Communication Planner", Lemma 1 (a congestion-free sub-stage is a matching),
 * Lemma 2 (at least Delta sub-stages are needed) and the appendix proof that Delta suffice.  The
 * split is not unique; this routine is deterministic for a given edge order.
 * edges[n_edges]: in (src, dst in [0, n_workers), src != dst not required) / out (stage).
 * *n_substages: out, Delta (0 for no edges).
 */
int fcp_solve_matchings(fcp_edge* edges, int64_t n_edges, int32_t n_workers, int32_t* n_substages);

/*
 * fcp_coalesce_stages -- bottom-up coalescer (section "Communication Planner"): sub-stages
 * [k c, (k + 1) c) become stage k, in which a worker sends at most c and receives at most c blocks.
 * coalesce c >= 1, or 0 = one stage.  stage_of_edge[n_edges]: out.  *n_stages: out.
 */
int fcp_coalesce_stages(const fcp_edge* edges, int64_t n_edges, int32_t coalesce,
                        int32_t* stage_of_edge, int32_t* n_stages);

#ifdef __cplusplus
}
#endif
#endif /* FCP_SCHED_H_ */
