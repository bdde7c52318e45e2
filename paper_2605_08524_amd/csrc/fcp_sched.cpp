// Host-side scheduling: block costs, greedy load-balanced assignment, data-flow graph,
// congestion-free ordering, coalescer.  Integers and IEEE doubles only; no HIP calls.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <vector>

#include "fcp_internal.h"
#include "fcp_sched.h"

namespace {

using fcp::set_error;

// x / x_hat, or 0 when the cost is absent from the batch (x_hat == 0)
inline double rel(int64_t x, double x_hat) { return x_hat > 0.0 ? (double)x / x_hat : 0.0; }

}  // namespace

extern "C" int fcp_block_costs(const int32_t* seq_lens, int32_t n_seqs, int32_t block_size, int32_t causal,
                               fcp_block* blocks, int64_t* mem, int64_t* comp, int32_t* n_blocks) {
  if (n_seqs < 0 || (n_seqs > 0 && !seq_lens) || !n_blocks) { set_error("fcp_block_costs: NULL argument or negative count"); return FCP_ERR_INVALID_ARG; }
  if (block_size <= 0) { set_error("fcp_block_costs: block_size must be positive"); return FCP_ERR_INVALID_ARG; }
  int64_t count = 0, tokens = 0;
  for (int s = 0; s < n_seqs; s++) {
    if (seq_lens[s] < 0) { set_error("fcp_block_costs: seq_lens[%d] is negative", s); return FCP_ERR_INVALID_ARG; }
    count += ((int64_t)seq_lens[s] + block_size - 1) / block_size;
    tokens += seq_lens[s];
  }
  if (count > INT32_MAX || tokens > INT32_MAX) { set_error("fcp_block_costs: more than 2^31-1 blocks or tokens"); return FCP_ERR_UNSUPPORTED; }
  const int32_t cap = *n_blocks;
  *n_blocks = (int32_t)count;
  if (!blocks && !mem && !comp) return FCP_OK;           // size query
  if (cap < count) { set_error("fcp_block_costs: capacity %d < %lld blocks", cap, (long long)count); return FCP_ERR_BUFFER_TOO_SMALL; }
  int32_t b = 0, row = 0;
  for (int s = 0; s < n_seqs; s++) {
    const int64_t L = seq_lens[s];
    for (int64_t lo = 0, i = 0; lo < L; lo += block_size, i++, b++) {
      const int64_t hi = std::min<int64_t>(L, lo + block_size), len = hi - lo;
      if (blocks) blocks[b] = fcp_block{s, (int32_t)i, (int32_t)(row + lo), (int32_t)len};
      if (mem) mem[b] = len;
      // rows lo .. hi-1 attend lo+1 .. hi keys: an arithmetic series
      if (comp) comp[b] = causal ? len * (lo + hi + 1) / 2 : len * L;
    }
    row += (int32_t)L;
  }
  return FCP_OK;
}

extern "C" int fcp_pack_units(const fcp_block* blocks, const int64_t* mem, const int64_t* comp, int32_t n_blocks,
                              int32_t block_size, int32_t* unit_of_block, int64_t* unit_mem, int64_t* unit_comp,
                              int32_t* n_units) {
  if (n_blocks < 0 || block_size <= 0 || !n_units || (n_blocks > 0 && (!blocks || !mem || !comp || !unit_of_block || !unit_mem || !unit_comp))) {
    set_error("fcp_pack_units: NULL argument, negative count or block_size <= 0"); return FCP_ERR_INVALID_ARG;
  }
  // a short sequence = a sequence with one block of fewer than block_size tokens
  std::vector<int32_t> shorts;
  for (int i = 0; i < n_blocks; i++) {
    const bool alone = (i == 0 || blocks[i - 1].seq != blocks[i].seq) && (i + 1 == n_blocks || blocks[i + 1].seq != blocks[i].seq);
    if (alone && mem[i] < block_size) shorts.push_back(i);
  }
  std::stable_sort(shorts.begin(), shorts.end(), [&](int32_t a, int32_t b) { return mem[a] > mem[b]; });
  // first fit: bins in the order they were opened
  std::vector<int64_t> room;
  std::vector<int32_t> bin_of(n_blocks, -1), bin_first;
  for (int32_t i : shorts) {
    size_t b = 0;
    while (b < room.size() && room[b] < mem[i]) b++;
    if (b == room.size()) { room.push_back(block_size); bin_first.push_back(i); }
    room[b] -= mem[i];
    bin_of[i] = (int32_t)b;
    bin_first[b] = std::min(bin_first[b], i);
  }
  // number the units by their lowest member block
  std::vector<int32_t> unit_of_bin(room.size(), -1);
  int32_t n = 0;
  for (int i = 0; i < n_blocks; i++) {
    if (bin_of[i] < 0) unit_of_block[i] = n++;
    else {
      if (bin_first[bin_of[i]] == i) unit_of_bin[bin_of[i]] = n++;
      unit_of_block[i] = -1 - bin_of[i];       // resolved below, once its bin has a number
    }
  }
  const int32_t cap = *n_units;
  *n_units = n;
  if (cap < n) { set_error("fcp_pack_units: capacity %d < %d units", cap, n); return FCP_ERR_BUFFER_TOO_SMALL; }
  std::fill(unit_mem, unit_mem + n, 0);
  std::fill(unit_comp, unit_comp + n, 0);
  for (int i = 0; i < n_blocks; i++) {
    if (unit_of_block[i] < 0) unit_of_block[i] = unit_of_bin[-1 - unit_of_block[i]];
    unit_mem[unit_of_block[i]] += mem[i];
    unit_comp[unit_of_block[i]] += comp[i];
  }
  return FCP_OK;
}

extern "C" int fcp_assign_blocks(const int64_t* mem, const int64_t* comp, int32_t n_blocks, int32_t n_workers,
                                 double alpha, double beta, int64_t mem_limit, double delta,
                                 int32_t* owner, int64_t* worker_mem, int64_t* worker_comp) {
  if (n_blocks < 0 || n_workers <= 0) { set_error("fcp_assign_blocks: n_blocks < 0 or n_workers <= 0"); return FCP_ERR_INVALID_ARG; }
  if (n_blocks > 0 && (!mem || !comp || !owner)) { set_error("fcp_assign_blocks: NULL argument"); return FCP_ERR_INVALID_ARG; }
  if (!(alpha >= 0.0) || !(beta >= 0.0) || !(delta >= 0.0)) { set_error("fcp_assign_blocks: alpha, beta, delta must be >= 0"); return FCP_ERR_INVALID_ARG; }
  int64_t sum_m = 0, sum_c = 0;
  for (int i = 0; i < n_blocks; i++) {
    if (mem[i] < 0 || comp[i] < 0) { set_error("fcp_assign_blocks: block %d has a negative cost", i); return FCP_ERR_INVALID_ARG; }
    if (mem[i] > INT64_MAX - sum_m || comp[i] > INT64_MAX - sum_c) { set_error("fcp_assign_blocks: total cost overflows 63 bits"); return FCP_ERR_UNSUPPORTED; }
    sum_m += mem[i]; sum_c += comp[i];
  }
  const double m_hat = (double)sum_m / n_workers, c_hat = (double)sum_c / n_workers;
  std::vector<double> key(n_blocks);
  for (int i = 0; i < n_blocks; i++) key[i] = std::max(rel(mem[i], m_hat), rel(comp[i], c_hat));
  std::vector<int32_t> order(n_blocks);
  for (int i = 0; i < n_blocks; i++) order[i] = i;
  std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) { return key[a] > key[b]; });

  std::vector<int64_t> w_m(n_workers, 0), w_c(n_workers, 0);
  const bool limited = mem_limit > 0;
  const double cap = (double)mem_limit * (1.0 + delta);
  for (int32_t i : order) {
    int best = -1;
    double best_load = 0.0;
    for (int w = 0; w < n_workers; w++) {
      if (limited && (double)(w_m[w] + mem[i]) > cap) continue;
      const double load = std::max(alpha * rel(w_m[w] + mem[i], m_hat), beta * rel(w_c[w] + comp[i], c_hat));
      if (best < 0 || load < best_load) { best = w; best_load = load; }
    }
    if (best < 0) {
      set_error("fcp_assign_blocks: block %d (%lld tokens) fits on no worker under the memory limit", i, (long long)mem[i]);
      return FCP_ERR_INFEASIBLE;
    }
    owner[i] = best;
    w_m[best] += mem[i];
    w_c[best] += comp[i];
  }
  if (worker_mem) std::copy(w_m.begin(), w_m.end(), worker_mem);
  if (worker_comp) std::copy(w_c.begin(), w_c.end(), worker_comp);
  return FCP_OK;
}

extern "C" int fcp_worker_blocks(const fcp_block* blocks, const int32_t* owner, int32_t n_blocks, int32_t worker,
                                 int32_t* q_owned, int32_t* n_q_owned) {
  if (n_blocks < 0 || !n_q_owned || (n_blocks > 0 && (!blocks || !owner))) { set_error("fcp_worker_blocks: NULL argument or negative count"); return FCP_ERR_INVALID_ARG; }
  int32_t count = 0;
  for (int i = 0; i < n_blocks; i++) count += owner[i] == worker;
  const int32_t cap = *n_q_owned;
  *n_q_owned = count;
  if (!q_owned) return FCP_OK;
  if (cap < count) { set_error("fcp_worker_blocks: capacity %d < %d blocks", cap, count); return FCP_ERR_BUFFER_TOO_SMALL; }
  for (int i = 0, n = 0; i < n_blocks; i++)
    if (owner[i] == worker) { q_owned[2 * n] = blocks[i].seq; q_owned[2 * n + 1] = blocks[i].idx; n++; }
  return FCP_OK;
}

extern "C" int fcp_comm_edges(const fcp_block* blocks, const int32_t* owner, int32_t n_blocks, int32_t n_workers,
                              int32_t causal, fcp_edge* edges, int64_t* n_edges) {
  if (n_blocks < 0 || n_workers <= 0 || !n_edges || (n_blocks > 0 && (!blocks || !owner))) {
    set_error("fcp_comm_edges: NULL argument, negative count or n_workers <= 0"); return FCP_ERR_INVALID_ARG;
  }
  for (int i = 0; i < n_blocks; i++) {
    if (owner[i] < 0 || owner[i] >= n_workers) { set_error("fcp_comm_edges: owner[%d] = %d out of range", i, owner[i]); return FCP_ERR_INVALID_ARG; }
    const bool first = i == 0 || blocks[i].seq != blocks[i - 1].seq;
    if (first ? (blocks[i].idx != 0 || (i > 0 && blocks[i].seq < blocks[i - 1].seq)) : blocks[i].idx != blocks[i - 1].idx + 1) {
      set_error("fcp_comm_edges: blocks[%d] is out of (seq, idx) order", i); return FCP_ERR_INVALID_ARG;
    }
  }
  const int64_t cap = *n_edges;
  int64_t count = 0;
  // Per sequence, from its last block to its first: `needs` is the set of workers that own a query
  // block depending on KV block j (the blocks j .. end under a causal mask, all of them otherwise).
  std::vector<uint8_t> needs(n_workers);
  std::vector<int64_t> first_edge_of(n_blocks + 1, 0);
  // pass 1 counts per block so that edges can be written in ascending block order
  for (int pass = 0; pass < 2; pass++) {
    for (int lo = 0; lo < n_blocks;) {
      int hi = lo;
      while (hi < n_blocks && blocks[hi].seq == blocks[lo].seq) hi++;
      std::fill(needs.begin(), needs.end(), 0);
      if (!causal) for (int i = lo; i < hi; i++) needs[owner[i]] = 1;
      for (int j = hi - 1; j >= lo; j--) {
        if (causal) needs[owner[j]] = 1;
        int64_t n = 0;
        for (int w = 0; w < n_workers; w++) {
          if (!needs[w] || w == owner[j]) continue;
          if (pass == 1) edges[first_edge_of[j] + n] = fcp_edge{owner[j], w, j, -1};
          n++;
        }
        if (pass == 0) first_edge_of[j + 1] = n;
      }
      lo = hi;
    }
    if (pass == 0) {
      for (int j = 0; j < n_blocks; j++) first_edge_of[j + 1] += first_edge_of[j];
      count = first_edge_of[n_blocks];
      *n_edges = count;
      if (!edges) return FCP_OK;
      if (cap < count) { set_error("fcp_comm_edges: capacity %lld < %lld edges", (long long)cap, (long long)count); return FCP_ERR_BUFFER_TOO_SMALL; }
    }
  }
  return FCP_OK;
}

// Edge colouring of a bipartite multigraph with Delta colours by alternating paths (Koenig's
// constructive proof): for an edge (u, w) take a colour a unused at send node u and a colour b
// unused at receive node w; if a is taken at w, swap a and b along the path that starts at w with
// its a-edge.  The path alternates a-edges into send nodes and b-edges into receive nodes, so it can
// never reach u (u has no a-edge); afterwards a is free at both ends.  O(E (N + Delta)).
extern "C" int fcp_solve_matchings(fcp_edge* edges, int64_t n_edges, int32_t n_workers, int32_t* n_substages) {
  if (n_edges < 0 || n_workers <= 0 || !n_substages || (n_edges > 0 && !edges)) {
    set_error("fcp_solve_matchings: NULL argument, negative count or n_workers <= 0"); return FCP_ERR_INVALID_ARG;
  }
  std::vector<int64_t> deg_s(n_workers, 0), deg_r(n_workers, 0);
  for (int64_t e = 0; e < n_edges; e++) {
    if (edges[e].src < 0 || edges[e].src >= n_workers || edges[e].dst < 0 || edges[e].dst >= n_workers) {
      set_error("fcp_solve_matchings: edge %lld has a worker out of range", (long long)e); return FCP_ERR_INVALID_ARG;
    }
    deg_s[edges[e].src]++; deg_r[edges[e].dst]++;
  }
  int64_t delta = 0;
  for (int w = 0; w < n_workers; w++) delta = std::max(delta, std::max(deg_s[w], deg_r[w]));
  if (delta > INT32_MAX) { set_error("fcp_solve_matchings: degree overflows 31 bits"); return FCP_ERR_UNSUPPORTED; }
  *n_substages = (int32_t)delta;
  if (n_edges == 0) return FCP_OK;
  // at_s[u * delta + colour] = the edge of that colour at send node u (-1: colour unused there)
  std::vector<int64_t> at_s((size_t)n_workers * delta, -1), at_r((size_t)n_workers * delta, -1);
  std::vector<int32_t> free_s(n_workers, 0), free_r(n_workers, 0);   // below these every colour is taken
  std::vector<int64_t> path;
  for (int64_t e = 0; e < n_edges; e++) {
    const int u = edges[e].src, w = edges[e].dst;
    int64_t* su = &at_s[(size_t)u * delta];
    int64_t* rw = &at_r[(size_t)w * delta];
    int a = free_s[u];
    while (su[a] >= 0) a++;
    free_s[u] = a;
    int b = free_r[w];
    while (rw[b] >= 0) b++;
    free_r[w] = b;
    if (rw[a] >= 0) {
      // collect the a/b alternating path from w, then recolour it
      path.clear();
      int col = a;
      bool at_recv = true;
      int node = w;
      for (;;) {
        const int64_t pe = at_recv ? at_r[(size_t)node * delta + col] : at_s[(size_t)node * delta + col];
        if (pe < 0) break;
        path.push_back(pe);
        node = at_recv ? edges[pe].src : edges[pe].dst;
        at_recv = !at_recv;
        col = (col == a) ? b : a;
      }
      for (int64_t pe : path) {
        const int c = edges[pe].stage;
        at_s[(size_t)edges[pe].src * delta + c] = -1;
        at_r[(size_t)edges[pe].dst * delta + c] = -1;
      }
      for (int64_t pe : path) {
        const int c = edges[pe].stage == a ? b : a;
        edges[pe].stage = c;
        at_s[(size_t)edges[pe].src * delta + c] = pe;
        at_r[(size_t)edges[pe].dst * delta + c] = pe;
      }
      // recolouring may have freed colours below the scan positions of the nodes on the path
      for (int64_t pe : path) {
        free_s[edges[pe].src] = std::min<int32_t>(free_s[edges[pe].src], std::min(a, b));
        free_r[edges[pe].dst] = std::min<int32_t>(free_r[edges[pe].dst], std::min(a, b));
      }
    }
    edges[e].stage = a;
    su[a] = e;
    rw[a] = e;
  }
  return FCP_OK;
}

extern "C" int fcp_coalesce_stages(const fcp_edge* edges, int64_t n_edges, int32_t coalesce,
                                   int32_t* stage_of_edge, int32_t* n_stages) {
  if (n_edges < 0 || coalesce < 0 || !n_stages || (n_edges > 0 && (!edges || !stage_of_edge))) {
    set_error("fcp_coalesce_stages: NULL argument or negative count"); return FCP_ERR_INVALID_ARG;
  }
  int32_t top = -1;
  for (int64_t e = 0; e < n_edges; e++) {
    if (edges[e].stage < 0) { set_error("fcp_coalesce_stages: edge %lld has no sub-stage (run fcp_solve_matchings first)", (long long)e); return FCP_ERR_INVALID_ARG; }
    stage_of_edge[e] = coalesce > 0 ? edges[e].stage / coalesce : 0;
    top = std::max(top, stage_of_edge[e]);
  }
  *n_stages = top + 1;
  return FCP_OK;
}
