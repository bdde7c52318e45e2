// Host side of the library: block planner, descriptor validation, work-queue scheduler.
// Integer work only; the only HIP calls are the workspace upload in fcp_queue_build.
#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <numeric>
#include <utility>
#include <vector>

#include "fcp_internal.h"

namespace fcp {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}

static inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

int validate_problem(const fcp_problem* p) {
  if (!p) { set_error("problem descriptor is NULL"); return FCP_ERR_INVALID_ARG; }
  if (p->n_q_heads <= 0 || p->n_kv_heads <= 0 || p->block_size <= 0) {
    set_error("heads and block_size must be positive"); return FCP_ERR_INVALID_ARG;
  }
  if (p->head_dim != 64 && p->head_dim != 128) {
    set_error("head_dim %d unsupported (64 or 128)", p->head_dim); return FCP_ERR_UNSUPPORTED;
  }
  if (p->n_q_heads % p->n_kv_heads != 0) {
    set_error("n_q_heads %d is not a multiple of n_kv_heads %d", p->n_q_heads, p->n_kv_heads);
    return FCP_ERR_UNSUPPORTED;
  }
  if (p->n_kv_blocks < 0 || p->n_q_blocks < 0 || p->n_pairs < 0 || p->n_slots < 0 || p->n_slot_rows < 0) {
    set_error("negative table count"); return FCP_ERR_INVALID_ARG;
  }
  if ((p->n_kv_blocks && !p->kv_blocks) || (p->n_q_blocks && !p->q_blocks) || (p->n_pairs && !p->pairs) ||
      (p->n_slots && !p->slots)) {
    set_error("NULL table with a non-zero count"); return FCP_ERR_INVALID_ARG;
  }
  if (!(p->softmax_scale >= 0.0f)) { set_error("softmax_scale must be >= 0 (0 = 1/sqrt(d))"); return FCP_ERR_INVALID_ARG; }
  if (p->n_segments < 0 || (p->n_segments && !p->segments)) { set_error("segments: negative count or NULL table"); return FCP_ERR_INVALID_ARG; }
  int64_t tok = 0;
  for (int i = 0; i < p->n_kv_blocks; i++) {
    const fcp_block& b = p->kv_blocks[i];
    if (b.tok_len <= 0 || b.tok_len > p->block_size || b.tok_start != tok) {
      set_error("kv_blocks[%d]: tok_len/tok_start inconsistent (blocks must be packed in order)", i);
      return FCP_ERR_INVALID_ARG;
    }
    tok += b.tok_len;
    if (tok > INT32_MAX) { set_error("more than 2^31-1 KV tokens"); return FCP_ERR_UNSUPPORTED; }
  }
  tok = 0;
  for (int i = 0; i < p->n_q_blocks; i++) {
    const fcp_block& b = p->q_blocks[i];
    if (b.tok_len <= 0 || b.tok_len > p->block_size || b.tok_start != tok) {
      set_error("q_blocks[%d]: tok_len/tok_start inconsistent (blocks must be packed in order)", i);
      return FCP_ERR_INVALID_ARG;
    }
    tok += b.tok_len;
  }
  // members of packed blocks: by (kv_blk, tok_off), tiling their block exactly
  std::vector<char> segmented;
  if (p->n_segments) {
    segmented.assign(p->n_kv_blocks, 0);
    int32_t blk = -1, covered = 0;
    for (int i = 0; i <= p->n_segments; i++) {
      if (i == p->n_segments || p->segments[i].kv_blk != blk) {
        if (blk >= 0 && covered != p->kv_blocks[blk].tok_len) {
          set_error("segments: the members of kv block %d do not cover it", blk); return FCP_ERR_INVALID_ARG;
        }
        if (i == p->n_segments) break;
        const int32_t nb = p->segments[i].kv_blk;
        if (nb <= blk || nb >= p->n_kv_blocks) { set_error("segments[%d]: kv_blk out of range or not ascending", i); return FCP_ERR_INVALID_ARG; }
        if (p->kv_blocks[nb].tok_len > kMaxPackedBlock) { set_error("segments[%d]: a packed block holds at most %d tokens", i, kMaxPackedBlock); return FCP_ERR_UNSUPPORTED; }
        blk = nb; covered = 0; segmented[nb] = 1;
      }
      const fcp_segment& sg = p->segments[i];
      if (sg.tok_off != covered || sg.tok_len <= 0 || (int64_t)sg.tok_off + sg.tok_len > p->kv_blocks[blk].tok_len) {
        set_error("segments[%d]: members must follow each other inside their block", i); return FCP_ERR_INVALID_ARG;
      }
      covered += sg.tok_len;
    }
  }
  int prev_q = -1;
  int64_t pair_cursor = 0;
  for (int s = 0; s < p->n_slots; s++) {
    const fcp_slot& sl = p->slots[s];
    if (sl.q_blk < 0 || sl.q_blk >= p->n_q_blocks || sl.q_blk < prev_q) {
      set_error("slots[%d]: q_blk out of range or not ascending", s); return FCP_ERR_INVALID_ARG;
    }
    prev_q = sl.q_blk;
    if (sl.pair_begin != pair_cursor || sl.n_pairs < 0 || pair_cursor + sl.n_pairs > p->n_pairs) {
      set_error("slots[%d]: pair range must continue where the previous slot ended", s);
      return FCP_ERR_INVALID_ARG;
    }
    pair_cursor += sl.n_pairs;
    const int qlen = p->q_blocks[sl.q_blk].tok_len;
    if (sl.row_start < 0 || (int64_t)sl.row_start + qlen > p->n_slot_rows) {
      set_error("slots[%d]: rows outside the partial buffers", s); return FCP_ERR_INVALID_ARG;
    }
    for (int64_t i = sl.pair_begin; i < sl.pair_begin + sl.n_pairs; i++) {
      const fcp_pair& pr = p->pairs[i];
      if (pr.q_blk != sl.q_blk || pr.slot != s || pr.kv_blk < 0 || pr.kv_blk >= p->n_kv_blocks ||
          pr.kind < FCP_KIND_FULL || pr.kind > FCP_KIND_PACKED_DIAG) {
        set_error("pairs[%lld]: inconsistent with slot %d", (long long)i, s); return FCP_ERR_INVALID_ARG;
      }
      if (pr.kind != FCP_KIND_FULL) {
        const fcp_block& qb = p->q_blocks[pr.q_blk];
        const fcp_block& kb = p->kv_blocks[pr.kv_blk];
        if (qb.seq != kb.seq || qb.idx != kb.idx || qb.tok_len != kb.tok_len) {
          set_error("pairs[%lld]: a DIAG or PACKED pair must join a block with itself", (long long)i);
          return FCP_ERR_INVALID_ARG;
        }
      }
      const bool seg = !segmented.empty() && segmented[pr.kv_blk];
      if (seg != ((pr.kind & 2) != 0)) {
        set_error("pairs[%lld]: a PACKED kind needs a KV block with members, the other kinds one without", (long long)i);
        return FCP_ERR_INVALID_ARG;
      }
      if ((pr.kind & 2) && sl.n_pairs != 1) {
        set_error("pairs[%lld]: a packed query block has one pair", (long long)i); return FCP_ERR_INVALID_ARG;
      }
    }
  }
  if (pair_cursor != p->n_pairs) { set_error("slots do not cover all pairs"); return FCP_ERR_INVALID_ARG; }
  return FCP_OK;
}

int compute_layout(const fcp_problem* p, WsLayout* L) {
  std::memset(L, 0, sizeof(*L));
  L->fwd_tile_m = kFwdTileM;
  {
    // forward items pair two query heads of a KV head when the group size is even, else two row tiles
    const int G = p->n_q_heads / p->n_kv_heads;
    for (int s = 0; s < p->n_slots; s++) {
      const int64_t n_tiles = ceil_div(p->q_blocks[p->slots[s].q_blk].tok_len, L->fwd_tile_m);
      const int64_t n = (G % 2 == 0) ? n_tiles * (p->n_q_heads / 2) : ceil_div(n_tiles, 2) * p->n_q_heads;
      L->n_fwd_items += n;
      if (p->slots[s].n_pairs == 1 && (p->pairs[p->slots[s].pair_begin].kind & 2)) L->n_fwd_packed_items += n;
    }
  }
  for (int b = 0; b < p->n_kv_blocks; b++)
    L->n_bwd_items += ceil_div(p->kv_blocks[b].tok_len, kBwdTileN) * p->n_kv_heads;
  L->n_bwd_deps = p->n_pairs;
  std::vector<int32_t> slots_of(p->n_q_blocks, 0);
  for (int s = 0; s < p->n_slots; s++) slots_of[p->slots[s].q_blk]++;
  const bool direct = (p->flags & FCP_FLAG_DIRECT_SINGLE) != 0;
  {
    // Chunk of the merge: small enough for kMergeMinItems work items (the kernel walks the slots of a chunk one
    // after the other, so a few long items leave most of the chip idle), a multiple of 32 entries, at most kMergeChunk.
    int64_t entries = 0;
    for (int b = 0; b < p->n_q_blocks; b++)
      if (!(direct && slots_of[b] == 1)) entries += (int64_t)p->q_blocks[b].tok_len * p->n_q_heads;
    L->merge_chunk = (int)std::min<int64_t>(kMergeChunk, std::max<int64_t>(32, ceil_div(ceil_div(entries, kMergeMinItems), 32) * 32));
  }
  for (int b = 0; b < p->n_q_blocks; b++) {
    if (!(direct && slots_of[b] == 1))
      L->n_merge_items += ceil_div((int64_t)p->q_blocks[b].tok_len * p->n_q_heads, L->merge_chunk);
    {
      const int G = p->n_q_heads / p->n_kv_heads;
      const int64_t n_tiles = ceil_div(p->q_blocks[b].tok_len, kFwdTileM);
      L->n_dq_items += (G % 2 == 0) ? n_tiles * (p->n_q_heads / 2) : ceil_div(n_tiles, 2) * p->n_q_heads;
    }
    L->t_q += p->q_blocks[b].tok_len;
  }
  for (int b = 0; b < p->n_kv_blocks; b++) L->t_kv += p->kv_blocks[b].tok_len;
  if (L->t_q * p->n_q_heads > INT32_MAX) { set_error("more than 2^31-1 (query row, head) entries"); return FCP_ERR_UNSUPPORTED; }
  if (L->n_fwd_items > INT32_MAX || L->n_bwd_items > INT32_MAX || L->n_merge_items > INT32_MAX) {
    set_error("too many work items"); return FCP_ERR_UNSUPPORTED;
  }
  auto align = [](size_t x) { return (x + 255) & ~(size_t)255; };
  size_t off = align(sizeof(WsHeader));
  L->off_pairs = off;       off = align(off + sizeof(DevPair) * (size_t)std::max(1, p->n_pairs));
  L->off_fwd_items = off;   off = align(off + sizeof(QItem) * (size_t)std::max<int64_t>(1, L->n_fwd_items));
  L->off_q_seg = off;       off = align(off + (p->n_segments ? sizeof(uint32_t) * (size_t)L->t_q : 0));
  L->off_bwd_deps = off;    off = align(off + sizeof(BwdDep) * (size_t)std::max<int64_t>(1, L->n_bwd_deps));
  L->off_bwd_items = off;   off = align(off + sizeof(BwdItem) * (size_t)std::max<int64_t>(1, L->n_bwd_items));
  L->off_merge_items = off; off = align(off + sizeof(MergeItem) * (size_t)std::max<int64_t>(1, L->n_merge_items));
  L->off_slot_rh = off;     off = align(off + sizeof(int32_t) * (size_t)std::max(1, p->n_slots));
  L->off_dq_items = off;    off = align(off + sizeof(QItem) * (size_t)std::max<int64_t>(1, L->n_dq_items));
  L->off_kv_seg = off;      off = align(off + (p->n_segments ? sizeof(uint32_t) * (size_t)L->t_kv : 0));
  // backward scratch, head-major [Hq][T_q] fp32: D * scale, then LSE * log2(e)
  L->off_dls = off;         off = align(off + sizeof(float) * (size_t)std::max<int64_t>(1, L->t_q * p->n_q_heads));
  L->off_lse2 = off;        off = align(off + sizeof(float) * (size_t)std::max<int64_t>(1, L->t_q * p->n_q_heads));
  L->off_ds = off;
  if (p->flags & FCP_FLAG_BWD_SPILL_DS) {
    int64_t frags = kDsSinkFrags;
    for (int i = 0; i < p->n_pairs; i++)
      frags += p->n_q_heads * ds_frags_per_head(p->pairs[i].kind, p->q_blocks[p->pairs[i].q_blk].tok_len,
                                                p->kv_blocks[p->pairs[i].kv_blk].tok_len);
    frags += 1;   // the dQ kernel requests fragments in pairs: one past the last may be named (never used)
    if (frags > INT32_MAX) { set_error("FCP_FLAG_BWD_SPILL_DS: more than 2^31-1 dS fragments"); return FCP_ERR_UNSUPPORTED; }
    L->n_ds_frags = frags;
    off = align(off + (size_t)frags * kDsFragBytes);
  }
  L->total = off;
  return FCP_OK;
}

// Layouts validated by fcp_queue_build, keyed by the workspace they were built into.  A launch on that
// workspace with the same descriptor scalars reuses the layout instead of walking every table again: the
// kernels read the device copy of the tables that fcp_queue_build made, so the host tables matter to a
// launch only through their counts.  A workspace the registry does not know (or a descriptor that differs)
// takes the full validation path.
namespace {
struct LayoutKey {
  const void* workspace;
  int32_t v[11];
  bool operator==(const LayoutKey& o) const { return workspace == o.workspace && std::memcmp(v, o.v, sizeof(v)) == 0; }
};
LayoutKey make_key(const fcp_problem* p, const void* ws) {
  return LayoutKey{ws, {p->n_q_heads, p->n_kv_heads, p->head_dim, p->block_size, p->flags & (FCP_FLAG_DIRECT_SINGLE | FCP_FLAG_BWD_SPILL_DS),
                        p->n_kv_blocks, p->n_q_blocks, p->n_pairs, p->n_slots, p->n_slot_rows, p->n_segments}};
}
constexpr int kLayoutCacheSize = 32;
std::mutex g_layout_mutex;
std::pair<LayoutKey, WsLayout> g_layout_cache[kLayoutCacheSize];
int g_layout_count = 0, g_layout_next = 0;
}  // namespace

void remember_layout(const fcp_problem* p, const void* workspace, const WsLayout& L) {
  const LayoutKey key = make_key(p, workspace);
  std::lock_guard<std::mutex> lock(g_layout_mutex);
  for (int i = 0; i < g_layout_count; i++)
    if (g_layout_cache[i].first.workspace == workspace) { g_layout_cache[i] = {key, L}; return; }
  g_layout_cache[g_layout_next] = {key, L};
  g_layout_next = (g_layout_next + 1) % kLayoutCacheSize;
  g_layout_count = std::min(g_layout_count + 1, kLayoutCacheSize);
}

int layout_for(const fcp_problem* p, const void* workspace, WsLayout* L) {
  if (p && workspace && p->softmax_scale >= 0.0f) {
    const LayoutKey key = make_key(p, workspace);
    std::lock_guard<std::mutex> lock(g_layout_mutex);
    for (int i = 0; i < g_layout_count; i++)
      if (g_layout_cache[i].first == key) { *L = g_layout_cache[i].second; return FCP_OK; }
  }
  int rc = validate_problem(p);
  if (rc) return rc;
  return compute_layout(p, L);
}

namespace {

// 64-row KV tiles that a query-stationary item visits: every pair in full, a DIAG pair up to the item's last row,
// a PACKED pair the item's column range.
void count_tiles(QItem* it, const DevPair* dpairs) {
  const int row_hi = std::max(it->tile_off[0] + it->q_rows[0], it->tile_off[1] + it->q_rows[1]);
  int n = 0;
  for (int i = it->pair_begin; i < it->pair_begin + it->n_pairs; i++) {
    if (dpairs[i].kind & 2) { n += (it->col_end - it->col_begin + kQTileN - 1) / kQTileN; continue; }
    const int nc = dpairs[i].kind == FCP_KIND_DIAG ? std::min(dpairs[i].kv_len, row_hi) : dpairs[i].kv_len;
    n += (nc + kQTileN - 1) / kQTileN;
  }
  it->n_tiles = n;
}

// Column range of an item of a packed query block: from the first column any of its rows can see (rounded down
// to a tile) to one past the last.  seg = the member bounds of the block's rows (seg_word), row 0 of the block first.
void packed_columns(QItem* it, const uint32_t* seg, bool causal) {
  int lo = INT32_MAX, hi = 0;
  for (int k = 0; k < 2; k++)
    for (int r = it->tile_off[k]; r < it->tile_off[k] + it->q_rows[k]; r++) {
      lo = std::min(lo, (int)(seg[r] & 0xffff));
      hi = std::max(hi, causal ? std::min((int)(seg[r] >> 16), r + 1) : (int)(seg[r] >> 16));
    }
  it->col_begin = hi ? (lo / kQTileN) * kQTileN : 0;
  it->col_end = hi;
}

// XCD affinity: groups with the same key (sequence, KV head) become one group (items concatenated in the order the
// groups came), so that all work that streams the K / V (forward, dQ) or Q / dO (dK/dV) rows of one sequence and KV
// head runs on one XCD and finds them in that XCD's L2 (measured on the training step: forward -1.2 %, dK/dV -0.6 %,
// dQ from dS -2 %).  Only done while the largest merged group stays below three quarters of an XCD's fair share:
// a batch dominated by one sequence keeps the finer groups, which balance better.
template <class Item>
void merge_groups_by_key(std::vector<std::vector<Item>>& groups, std::vector<int64_t>& weight, const std::vector<int64_t>& key) {
  {
    std::vector<int64_t> k2, w2;
    int64_t total = 0, largest = 0;
    for (size_t i = 0; i < groups.size(); i++) {
      size_t j = 0;
      while (j < k2.size() && k2[j] != key[i]) j++;
      if (j == k2.size()) { k2.push_back(key[i]); w2.push_back(0); }
      w2[j] += weight[i];
      total += weight[i];
      largest = std::max(largest, w2[j]);
    }
    if (largest * kNumXcd * 4 > total * 3) return;
  }
  std::vector<std::vector<Item>> g2;
  std::vector<int64_t> w2, k2;
  for (size_t i = 0; i < groups.size(); i++) {
    size_t j = 0;
    while (j < k2.size() && k2[j] != key[i]) j++;
    if (j == k2.size()) { k2.push_back(key[i]); g2.emplace_back(); w2.push_back(0); }
    g2[j].insert(g2[j].end(), groups[i].begin(), groups[i].end());
    w2[j] += weight[i];
  }
  groups.swap(g2); weight.swap(w2);
}

// Longest-processing-time assignment of weighted groups to the XCD queues: groups in
// descending weight, each to the currently lightest queue.  Ties resolve to the lower index.
template <class Item>
void spread_over_xcds(std::vector<std::vector<Item>>& groups, std::vector<int64_t>& weight,
                      std::vector<Item>* out, int32_t begin[kNumXcd + 1]) {
  std::vector<int> order(groups.size());
  std::iota(order.begin(), order.end(), 0);
  std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return weight[a] > weight[b]; });
  std::vector<std::vector<int>> per_xcd(kNumXcd);
  int64_t load[kNumXcd] = {0};
  for (int g : order) {
    int best = 0;
    for (int x = 1; x < kNumXcd; x++)
      if (load[x] < load[best]) best = x;
    per_xcd[best].push_back(g);
    load[best] += weight[g];
  }
  out->clear();
  for (int x = 0; x < kNumXcd; x++) {
    begin[x] = (int32_t)out->size();
    for (int g : per_xcd[x])
      for (const Item& it : groups[g]) out->push_back(it);
  }
  begin[kNumXcd] = (int32_t)out->size();
}

// Column range [lo, hi) of the dQ item that holds each 128-row tile of a packed query block (the items pair
// neighbouring row tiles when the group size is odd, exactly as the dQ queue builder below does).
void packed_tile_columns(int tok_len, int G, const uint32_t* seg, bool causal, std::vector<int>* lo, std::vector<int>* hi) {
  const int n_tiles = (int)ceil_div(tok_len, kFwdTileM);
  lo->assign(n_tiles, 0); hi->assign(n_tiles, 0);
  auto range = [&](int t0, int t1) {      // the item of tiles t0 (and t1, or -1)
    QItem it{};
    it.tile_off[0] = t0 * kFwdTileM; it.q_rows[0] = std::min(kFwdTileM, tok_len - t0 * kFwdTileM);
    if (t1 >= 0) { it.tile_off[1] = t1 * kFwdTileM; it.q_rows[1] = std::min(kFwdTileM, tok_len - t1 * kFwdTileM); }
    packed_columns(&it, seg, causal);
    (*lo)[t0] = it.col_begin; (*hi)[t0] = it.col_end;
    if (t1 >= 0) { (*lo)[t1] = it.col_begin; (*hi)[t1] = it.col_end; }
  };
  if (G % 2 == 0) for (int t = 0; t < n_tiles; t++) range(t, -1);
  else for (int t = n_tiles - 1; t >= 0; t -= 2) range(t, t >= 1 ? t - 1 : -1);
}

}  // namespace
}  // namespace fcp

using namespace fcp;

extern "C" const char* fcp_last_error(void) { return g_err; }

extern "C" int fcp_plan_blocks(const int32_t* seq_lens, int32_t n_seqs, int32_t block_size,
                               int32_t causal, int32_t coalesce,
                               const int32_t* q_owned, int32_t n_q_owned,
                               fcp_block* kv_blocks, int32_t* n_kv_blocks,
                               fcp_block* q_blocks, int32_t* n_q_blocks,
                               fcp_pair* pairs, int32_t* n_pairs,
                               fcp_slot* slots, int32_t* n_slots,
                               int32_t* n_slot_rows) {
  if (n_seqs < 0 || (n_seqs > 0 && !seq_lens) || block_size <= 0 || coalesce < 0 || n_q_owned < 0 ||
      !n_kv_blocks || !n_q_blocks || !n_pairs || !n_slots || !n_slot_rows) {
    set_error("fcp_plan_blocks: invalid argument"); return FCP_ERR_INVALID_ARG;
  }
  // Pass 1: per-sequence block counts and offsets.
  std::vector<int64_t> first_blk(n_seqs + 1, 0), tok_off(n_seqs + 1, 0);
  for (int s = 0; s < n_seqs; s++) {
    if (seq_lens[s] < 0) { set_error("fcp_plan_blocks: seq_lens[%d] < 0", s); return FCP_ERR_INVALID_ARG; }
    first_blk[s + 1] = first_blk[s] + ceil_div(seq_lens[s], block_size);
    tok_off[s + 1] = tok_off[s] + seq_lens[s];
  }
  if (tok_off[n_seqs] > INT32_MAX || first_blk[n_seqs] > INT32_MAX) {
    set_error("fcp_plan_blocks: more than 2^31-1 tokens or blocks"); return FCP_ERR_UNSUPPORTED;
  }
  auto nblk = [&](int s) { return (int32_t)(first_blk[s + 1] - first_blk[s]); };
  auto blk_len = [&](int s, int i) { return std::min<int32_t>(block_size, seq_lens[s] - i * block_size); };
  const int64_t need_kv = first_blk[n_seqs];
  // Owned query blocks.
  const bool all_owned = (q_owned == nullptr);
  if (!all_owned) {
    for (int t = 0; t < n_q_owned; t++) {
      const int32_t s = q_owned[2 * t], i = q_owned[2 * t + 1];
      if (s < 0 || s >= n_seqs || i < 0 || i >= nblk(s)) {
        set_error("fcp_plan_blocks: q_owned[%d] = (%d, %d) out of range", t, s, i); return FCP_ERR_INVALID_ARG;
      }
      if (t > 0) {
        const int32_t ps = q_owned[2 * t - 2], pi = q_owned[2 * t - 1];
        if (ps > s || (ps == s && pi >= i)) {
          set_error("fcp_plan_blocks: q_owned must be strictly increasing in (seq, idx)");
          return FCP_ERR_INVALID_ARG;
        }
      }
    }
  }
  const int64_t need_q = all_owned ? need_kv : n_q_owned;
  // Pass 2: counts of pairs, slots, partial rows.
  int64_t need_pairs = 0, need_slots = 0, need_rows = 0;
  auto for_each_owned = [&](auto&& fn) {
    if (all_owned) {
      for (int s = 0; s < n_seqs; s++)
        for (int i = 0; i < nblk(s); i++) fn(s, i);
    } else {
      for (int t = 0; t < n_q_owned; t++) fn(q_owned[2 * t], q_owned[2 * t + 1]);
    }
  };
  for_each_owned([&](int s, int i) {
    const int64_t np = causal ? (i + 1) : nblk(s);
    const int64_t ns = coalesce == 0 ? 1 : ceil_div(np, coalesce);
    need_pairs += np;
    need_slots += ns;
    need_rows += ns * blk_len(s, i);
  });
  if (need_pairs > INT32_MAX || need_rows > INT32_MAX) {
    set_error("fcp_plan_blocks: more than 2^31-1 pairs or partial rows"); return FCP_ERR_UNSUPPORTED;
  }
  const int32_t cap_kv = *n_kv_blocks, cap_q = *n_q_blocks, cap_p = *n_pairs, cap_s = *n_slots;
  *n_kv_blocks = (int32_t)need_kv; *n_q_blocks = (int32_t)need_q; *n_pairs = (int32_t)need_pairs;
  *n_slots = (int32_t)need_slots; *n_slot_rows = (int32_t)need_rows;
  if (!kv_blocks && !q_blocks && !pairs && !slots) return FCP_OK;   // size query
  if (!kv_blocks || !q_blocks || !pairs || !slots) {
    set_error("fcp_plan_blocks: pass all four tables or none"); return FCP_ERR_INVALID_ARG;
  }
  if (cap_kv < need_kv || cap_q < need_q || cap_p < need_pairs || cap_s < need_slots) {
    set_error("fcp_plan_blocks: table capacity too small (need %lld kv, %lld q, %lld pairs, %lld slots)",
              (long long)need_kv, (long long)need_q, (long long)need_pairs, (long long)need_slots);
    return FCP_ERR_BUFFER_TOO_SMALL;
  }
  // Pass 3: fill.
  for (int s = 0; s < n_seqs; s++)
    for (int i = 0; i < nblk(s); i++)
      kv_blocks[first_blk[s] + i] = {s, i, (int32_t)(tok_off[s] + (int64_t)i * block_size), blk_len(s, i)};
  int32_t qb = 0, qtok = 0, np_out = 0, ns_out = 0, row = 0;
  for_each_owned([&](int s, int i) {
    const int32_t len = blk_len(s, i);
    q_blocks[qb] = {s, i, qtok, len};
    qtok += len;
    const int32_t np = causal ? (i + 1) : nblk(s);
    for (int32_t r = 0; r < np; r++) {
      const bool opens = (coalesce == 0) ? (r == 0) : (r % coalesce == 0);
      if (opens) {
        slots[ns_out] = {qb, np_out, 0, row};
        ns_out++;
        row += len;
      }
      const int32_t kind = (causal && r == i) ? FCP_KIND_DIAG : FCP_KIND_FULL;
      pairs[np_out] = {qb, (int32_t)(first_blk[s] + r), kind, ns_out - 1};
      slots[ns_out - 1].n_pairs++;
      np_out++;
    }
    qb++;
  });
  return FCP_OK;
}

extern "C" int fcp_plan_blocks_packed(const int32_t* seq_lens, int32_t n_seqs, int32_t block_size,
                                      int32_t causal, int32_t coalesce,
                                      const int32_t* q_owned, int32_t n_q_owned,
                                      const int32_t* unit_of_block,
                                      fcp_block* kv_blocks, int32_t* n_kv_blocks,
                                      fcp_block* q_blocks, int32_t* n_q_blocks,
                                      fcp_pair* pairs, int32_t* n_pairs,
                                      fcp_slot* slots, int32_t* n_slots,
                                      int32_t* n_slot_rows,
                                      fcp_segment* segments, int32_t* n_segments) {
  if (n_seqs < 0 || (n_seqs > 0 && !seq_lens) || block_size <= 0 || coalesce < 0 || n_q_owned < 0 ||
      !n_kv_blocks || !n_q_blocks || !n_pairs || !n_slots || !n_slot_rows || !n_segments) {
    set_error("fcp_plan_blocks_packed: invalid argument"); return FCP_ERR_INVALID_ARG;
  }
  // The unpacked table: block u of it is (u_seq[u], u_idx[u]) with u_len[u] tokens.
  std::vector<int32_t> u_seq, u_idx, u_len, first_u(n_seqs + 1, 0);
  for (int s = 0; s < n_seqs; s++) {
    if (seq_lens[s] < 0) { set_error("fcp_plan_blocks_packed: seq_lens[%d] < 0", s); return FCP_ERR_INVALID_ARG; }
    const int64_t nb = ceil_div(seq_lens[s], block_size);
    if ((int64_t)u_seq.size() + nb > INT32_MAX) { set_error("fcp_plan_blocks_packed: more than 2^31-1 blocks"); return FCP_ERR_UNSUPPORTED; }
    for (int i = 0; i < nb; i++) {
      u_seq.push_back(s); u_idx.push_back(i);
      u_len.push_back(std::min<int32_t>(block_size, seq_lens[s] - i * block_size));
    }
    first_u[s + 1] = (int32_t)u_seq.size();
  }
  const int32_t nu = (int32_t)u_seq.size();
  if (nu > 0 && !unit_of_block) { set_error("fcp_plan_blocks_packed: unit_of_block is NULL"); return FCP_ERR_INVALID_ARG; }
  // Units: size, lowest member, summed length; a multi-block unit is a packed block led by its lowest member.
  std::vector<int32_t> u_count(nu, 0), u_lead(nu, -1), u_last(nu, -1), next_member(nu, -1);
  std::vector<int64_t> u_sum(nu, 0);
  for (int u = 0; u < nu; u++) {
    const int32_t g = unit_of_block[u];
    if (g < 0 || g >= nu) { set_error("fcp_plan_blocks_packed: unit_of_block[%d] = %d out of range", u, g); return FCP_ERR_INVALID_ARG; }
    if (u_count[g]++ == 0) u_lead[g] = u; else next_member[u_last[g]] = u;
    u_last[g] = u;
    u_sum[g] += u_len[u];
  }
  for (int u = 0; u < nu; u++) {
    const int32_t g = unit_of_block[u];
    if (u_count[g] < 2) continue;
    if (u_idx[u] != 0 || first_u[u_seq[u] + 1] - first_u[u_seq[u]] != 1 || u_len[u] >= block_size) {
      set_error("fcp_plan_blocks_packed: block %d shares unit %d but is not a whole sequence shorter than a block", u, g);
      return FCP_ERR_INVALID_ARG;
    }
    if (u_sum[g] > block_size) { set_error("fcp_plan_blocks_packed: unit %d does not fit into one block", g); return FCP_ERR_INVALID_ARG; }
  }
  auto packed = [&](int u) { return u_count[unit_of_block[u]] >= 2; };
  auto leads = [&](int u) { return !packed(u) || u_lead[unit_of_block[u]] == u; };
  // Ownership per unpacked block.
  std::vector<char> own(nu, q_owned ? 0 : 1);
  if (q_owned) {
    for (int t = 0; t < n_q_owned; t++) {
      const int32_t s = q_owned[2 * t], i = q_owned[2 * t + 1];
      if (s < 0 || s >= n_seqs || i < 0 || i >= first_u[s + 1] - first_u[s]) {
        set_error("fcp_plan_blocks_packed: q_owned[%d] = (%d, %d) out of range", t, s, i); return FCP_ERR_INVALID_ARG;
      }
      if (t > 0 && (q_owned[2 * t - 2] > s || (q_owned[2 * t - 2] == s && q_owned[2 * t - 1] >= i))) {
        set_error("fcp_plan_blocks_packed: q_owned must be strictly increasing in (seq, idx)"); return FCP_ERR_INVALID_ARG;
      }
      own[first_u[s] + i] = 1;
    }
    for (int u = 0; u < nu; u++)
      if (packed(u) && own[u] != own[u_lead[unit_of_block[u]]]) {
        set_error("fcp_plan_blocks_packed: unit %d is owned in part", unit_of_block[u]); return FCP_ERR_INVALID_ARG;
      }
  }
  // Counts.
  int64_t need_kv = 0, need_q = 0, need_pairs = 0, need_slots = 0, need_rows = 0, need_seg = 0, tokens = 0;
  for (int u = 0; u < nu; u++) {
    tokens += u_len[u];
    if (packed(u)) need_seg++;
    if (!leads(u)) continue;
    need_kv++;
    if (!own[u]) continue;
    need_q++;
    const int64_t len = packed(u) ? u_sum[unit_of_block[u]] : u_len[u];
    const int64_t np = packed(u) ? 1 : (causal ? u_idx[u] + 1 : first_u[u_seq[u] + 1] - first_u[u_seq[u]]);
    const int64_t ns = coalesce == 0 ? 1 : ceil_div(np, coalesce);
    need_pairs += np; need_slots += ns; need_rows += ns * len;
  }
  if (tokens > INT32_MAX || need_pairs > INT32_MAX || need_rows > INT32_MAX) {
    set_error("fcp_plan_blocks_packed: more than 2^31-1 tokens, pairs or partial rows"); return FCP_ERR_UNSUPPORTED;
  }
  const int32_t cap_kv = *n_kv_blocks, cap_q = *n_q_blocks, cap_p = *n_pairs, cap_s = *n_slots, cap_g = *n_segments;
  *n_kv_blocks = (int32_t)need_kv; *n_q_blocks = (int32_t)need_q; *n_pairs = (int32_t)need_pairs;
  *n_slots = (int32_t)need_slots; *n_slot_rows = (int32_t)need_rows; *n_segments = (int32_t)need_seg;
  if (!kv_blocks && !q_blocks && !pairs && !slots && !segments) return FCP_OK;   // size query
  if (!kv_blocks || !q_blocks || !pairs || !slots || (need_seg > 0 && !segments)) {
    set_error("fcp_plan_blocks_packed: pass all tables or none"); return FCP_ERR_INVALID_ARG;
  }
  if (cap_kv < need_kv || cap_q < need_q || cap_p < need_pairs || cap_s < need_slots || cap_g < need_seg) {
    set_error("fcp_plan_blocks_packed: table capacity too small (need %lld kv, %lld q, %lld pairs, %lld slots, %lld segments)",
              (long long)need_kv, (long long)need_q, (long long)need_pairs, (long long)need_slots, (long long)need_seg);
    return FCP_ERR_BUFFER_TOO_SMALL;
  }
  // Fill: KV blocks and segments first (a pair needs the new index of an unpacked block), then the owned side.
  std::vector<int32_t> kv_of(nu, -1);
  int32_t nk = 0, ng = 0, tok = 0;
  for (int u = 0; u < nu; u++) {
    if (!leads(u)) continue;
    int32_t len = u_len[u];
    if (packed(u)) {
      len = 0;
      for (int m = u; m >= 0; m = next_member[m]) {     // members in ascending unpacked order; the lead is the lowest
        segments[ng++] = {nk, u_seq[m], len, u_len[m]};
        len += u_len[m];
      }
    }
    kv_of[u] = nk;
    kv_blocks[nk++] = {u_seq[u], packed(u) ? 0 : u_idx[u], tok, len};
    tok += len;
  }
  int32_t nq = 0, qtok = 0, np_out = 0, ns_out = 0, row = 0;
  for (int u = 0; u < nu; u++) {
    if (!leads(u) || !own[u]) continue;
    const fcp_block& kb = kv_blocks[kv_of[u]];
    q_blocks[nq] = {kb.seq, kb.idx, qtok, kb.tok_len};
    qtok += kb.tok_len;
    if (packed(u)) {
      slots[ns_out] = {nq, np_out, 1, row};
      pairs[np_out++] = {nq, kv_of[u], causal ? FCP_KIND_PACKED_DIAG : FCP_KIND_PACKED_FULL, ns_out};
      ns_out++;
      row += kb.tok_len;
    } else {
      const int32_t s = u_seq[u], i = u_idx[u];
      const int32_t np = causal ? (i + 1) : first_u[s + 1] - first_u[s];
      for (int32_t r = 0; r < np; r++) {
        if ((coalesce == 0) ? (r == 0) : (r % coalesce == 0)) {
          slots[ns_out++] = {nq, np_out, 0, row};
          row += kb.tok_len;
        }
        pairs[np_out++] = {nq, kv_of[first_u[s] + r], (causal && r == i) ? FCP_KIND_DIAG : FCP_KIND_FULL, ns_out - 1};
        slots[ns_out - 1].n_pairs++;
      }
    }
    nq++;
  }
  return FCP_OK;
}

extern "C" int fcp_stage_tables(const fcp_pair* pairs, int32_t n_pairs, const fcp_slot* slots, int32_t n_slots,
                                const fcp_block* q_blocks, int32_t n_q_blocks, int32_t stage,
                                fcp_pair* stage_pairs, int32_t* n_stage_pairs, fcp_slot* stage_slots, int32_t* n_stage_slots,
                                int32_t* n_stages) {
  if (n_pairs < 0 || n_slots < 0 || n_q_blocks < 0 || stage < 0 || (n_pairs && !pairs) || (n_slots && !slots) ||
      (n_q_blocks && !q_blocks) || !n_stage_pairs || !n_stage_slots || !n_stages) {
    set_error("fcp_stage_tables: invalid argument"); return FCP_ERR_INVALID_ARG;
  }
  // pass 1: the stage-th slot of every query block (slots of a block are consecutive), counts
  int64_t need_pairs = 0, need_slots = 0;
  int32_t most = 0;
  for (int s = 0, local = 0; s < n_slots; s++) {
    const fcp_slot& sl = slots[s];
    if (sl.q_blk < 0 || sl.q_blk >= n_q_blocks || sl.pair_begin < 0 || sl.n_pairs < 0 || (int64_t)sl.pair_begin + sl.n_pairs > n_pairs ||
        (s > 0 && sl.q_blk < slots[s - 1].q_blk)) {
      set_error("fcp_stage_tables: slots[%d] is inconsistent", s); return FCP_ERR_INVALID_ARG;
    }
    local = (s > 0 && slots[s - 1].q_blk == sl.q_blk) ? local + 1 : 0;
    most = std::max(most, local + 1);
    if (local == stage) { need_slots++; need_pairs += sl.n_pairs; }
  }
  const int32_t cap_p = *n_stage_pairs, cap_s = *n_stage_slots;
  *n_stage_pairs = (int32_t)need_pairs; *n_stage_slots = (int32_t)need_slots; *n_stages = most;
  if (!stage_pairs && !stage_slots) return FCP_OK;
  if (!stage_pairs || !stage_slots) { set_error("fcp_stage_tables: pass both tables or none"); return FCP_ERR_INVALID_ARG; }
  if (cap_p < need_pairs || cap_s < need_slots) {
    set_error("fcp_stage_tables: table capacity too small (need %lld pairs, %lld slots)", (long long)need_pairs, (long long)need_slots);
    return FCP_ERR_BUFFER_TOO_SMALL;
  }
  int32_t np = 0, ns = 0;
  for (int s = 0, local = 0; s < n_slots; s++) {
    const fcp_slot& sl = slots[s];
    local = (s > 0 && slots[s - 1].q_blk == sl.q_blk) ? local + 1 : 0;
    if (local != stage) continue;
    stage_slots[ns] = {sl.q_blk, np, sl.n_pairs, q_blocks[sl.q_blk].tok_start};
    for (int i = sl.pair_begin; i < sl.pair_begin + sl.n_pairs; i++)
      stage_pairs[np++] = {pairs[i].q_blk, pairs[i].kv_blk, pairs[i].kind, ns};
    ns++;
  }
  return FCP_OK;
}

extern "C" int fcp_workspace_bytes(const fcp_problem* p, size_t* bytes) {
  if (!bytes) { set_error("fcp_workspace_bytes: bytes is NULL"); return FCP_ERR_INVALID_ARG; }
  int rc = validate_problem(p);
  if (rc) return rc;
  WsLayout L;
  rc = compute_layout(p, &L);
  if (rc) return rc;
  *bytes = L.total;
  return FCP_OK;
}

// The host image of the workspace sections that the kernels read: header (zeroed counters, queue
// ranges, zero / +inf pages), resolved pairs, forward items and, unless forward_only, the backward,
// dQ and merge tables.  `host` is resized to the image (everything before the backward scratch
// region, or before the backward dependency lists when forward_only).
int fcp::build_queue_image(const fcp_problem* p, const WsLayout& L, bool forward_only, std::vector<unsigned char>* image) {
  const size_t upload = forward_only ? L.off_bwd_deps : L.off_dls;
  image->assign(upload, 0);
  std::vector<unsigned char>& host = *image;
  WsHeader* hdr = reinterpret_cast<WsHeader*>(host.data());
  for (float& x : hdr->infs) x = INFINITY;
  DevPair* dpairs = reinterpret_cast<DevPair*>(host.data() + L.off_pairs);
  {
    const bool spill = (p->flags & FCP_FLAG_BWD_SPILL_DS) != 0;
    int64_t frag = kDsSinkFrags;
    for (int i = 0; i < p->n_pairs; i++) {
      const fcp_block& kb = p->kv_blocks[p->pairs[i].kv_blk];
      dpairs[i] = {kb.tok_start, kb.tok_len, p->pairs[i].kind, spill ? (int32_t)frag : 0};
      frag += p->n_q_heads * ds_frags_per_head(p->pairs[i].kind, p->q_blocks[p->pairs[i].q_blk].tok_len, kb.tok_len);
    }
  }
  // ---- member bounds of the rows of packed blocks, per Q-buffer row and (with the backward tables) per KV-buffer row
  const uint32_t* q_seg = nullptr;
  if (p->n_segments) {
    std::vector<int32_t> seg_begin(p->n_kv_blocks + 1, 0);
    for (int i = 0; i < p->n_segments; i++) seg_begin[p->segments[i].kv_blk + 1]++;
    for (int b = 0; b < p->n_kv_blocks; b++) seg_begin[b + 1] += seg_begin[b];
    uint32_t* qs = reinterpret_cast<uint32_t*>(host.data() + L.off_q_seg);
    uint32_t* ks = forward_only ? nullptr : reinterpret_cast<uint32_t*>(host.data() + L.off_kv_seg);
    for (int i = 0; i < p->n_pairs; i++) {
      if (!(p->pairs[i].kind & 2)) continue;
      const int kb = p->pairs[i].kv_blk;
      const int32_t q0 = p->q_blocks[p->pairs[i].q_blk].tok_start;
      for (int m = seg_begin[kb]; m < seg_begin[kb + 1]; m++)
        for (int r = 0; r < p->segments[m].tok_len; r++)
          qs[q0 + p->segments[m].tok_off + r] = seg_word(p->segments[m].tok_off, p->segments[m].tok_off + p->segments[m].tok_len);
    }
    if (ks)
      for (int m = 0; m < p->n_segments; m++)
        for (int r = 0; r < p->segments[m].tok_len; r++)
          ks[p->kv_blocks[p->segments[m].kv_blk].tok_start + p->segments[m].tok_off + r] =
              seg_word(p->segments[m].tok_off, p->segments[m].tok_off + p->segments[m].tok_len);
    q_seg = qs;
  }
  const int G = p->n_q_heads / p->n_kv_heads;
  // ---- forward: one group per (slot, KV head): its items share K/V.  An item joins two sub-tiles:
  // heads (2j, 2j+1) of the group on one row tile when G is even, else row tiles (2j, 2j+1) of one head.
  {
    std::vector<std::vector<QItem>> groups, groups_p;      // _p: items of packed query blocks, queued apart
    std::vector<int64_t> weight, gkey, weight_p;
    groups.reserve((size_t)p->n_slots * p->n_kv_heads);
    std::vector<int32_t> n_slots_of(p->n_q_blocks, 0);
    for (int s = 0; s < p->n_slots; s++) n_slots_of[p->slots[s].q_blk]++;
    for (int s = 0; s < p->n_slots; s++) {
      const fcp_slot& sl = p->slots[s];
      const fcp_block& qb = p->q_blocks[sl.q_blk];
      const int n_tiles = (int)ceil_div(qb.tok_len, L.fwd_tile_m);
      std::vector<int64_t> tile_w(n_tiles, 0);
      for (int t = n_tiles - 1; t >= 0; t--) {
        const int off = t * L.fwd_tile_m;
        const int rows = std::min(L.fwd_tile_m, qb.tok_len - off);
        for (int i = sl.pair_begin; i < sl.pair_begin + sl.n_pairs; i++) {
          const int kvlen = dpairs[i].kv_len;
          const int cols = (dpairs[i].kind & 1) ? std::min(kvlen, off + rows) : kvlen;
          tile_w[t] += (int64_t)rows * cols;
        }
      }
      const int packed_kind = (sl.n_pairs == 1 && (dpairs[sl.pair_begin].kind & 2)) ? dpairs[sl.pair_begin].kind : 0;
      auto finish = [&](QItem* it) {
        if (packed_kind) packed_columns(it, q_seg + qb.tok_start, (packed_kind & 1) != 0);
        count_tiles(it, dpairs);
      };
      const int to_final = ((p->flags & FCP_FLAG_DIRECT_SINGLE) && n_slots_of[sl.q_blk] == 1) ? 1 : 0;
      auto sub = [&](QItem* it, int k, int t, int head) {
        const int off = t * L.fwd_tile_m;
        it->q_start[k] = qb.tok_start + off; it->q_rows[k] = std::min(L.fwd_tile_m, qb.tok_len - off);
        it->out_row[k] = sl.row_start + off; it->tile_off[k] = off; it->head[k] = head;
      };
      for (int g = 0; g < p->n_kv_heads; g++) {
        std::vector<QItem> items;
        int64_t w = 0;
        if (G % 2 == 0) {
          for (int t = n_tiles - 1; t >= 0; t--)         // later tiles of a DIAG pair are heavier
            for (int hh = 0; hh < G; hh += 2) {
              QItem it{};
              it.pair_begin = sl.pair_begin; it.n_pairs = sl.n_pairs; it.to_final = to_final;
              sub(&it, 0, t, g * G + hh); sub(&it, 1, t, g * G + hh + 1);
              finish(&it);
              items.push_back(it);
              w += 2 * tile_w[t];
            }
        } else {
          for (int t = n_tiles - 1; t >= 0; t -= 2)
            for (int hh = 0; hh < G; hh++) {
              QItem it{};
              it.pair_begin = sl.pair_begin; it.n_pairs = sl.n_pairs; it.to_final = to_final;
              sub(&it, 0, t, g * G + hh);
              if (t >= 1) { sub(&it, 1, t - 1, g * G + hh); w += tile_w[t - 1]; }
              else { it.q_start[1] = it.q_start[0]; it.q_rows[1] = 0; it.out_row[1] = it.out_row[0]; it.tile_off[1] = it.tile_off[0]; it.head[1] = it.head[0]; }
              finish(&it);
              items.push_back(it);
              w += tile_w[t];
            }
        }
        if (packed_kind) {
          groups_p.push_back(std::move(items));
          weight_p.push_back(w);
        } else {
          groups.push_back(std::move(items));
          weight.push_back(w);
          gkey.push_back((int64_t)qb.seq * p->n_kv_heads + g);
        }
      }
    }
    merge_groups_by_key(groups, weight, gkey);
    std::vector<QItem> flat, flat_p;
    spread_over_xcds(groups, weight, &flat, hdr->fwd_begin);
    spread_over_xcds(groups_p, weight_p, &flat_p, hdr->fwdp_begin);
    for (int x = 0; x <= kNumXcd; x++) hdr->fwdp_begin[x] += (int32_t)flat.size();      // they follow the others
    if ((int64_t)flat.size() != L.n_fwd_items - L.n_fwd_packed_items || (int64_t)flat_p.size() != L.n_fwd_packed_items) {
      set_error("internal: forward item count mismatch"); return FCP_ERR_INVALID_ARG;
    }
    flat.insert(flat.end(), flat_p.begin(), flat_p.end());
    if (!flat.empty()) std::memcpy(host.data() + L.off_fwd_items, flat.data(), flat.size() * sizeof(QItem));
  }
  if (forward_only) return FCP_OK;
  // ---- backward: dependency lists per KV block, one group per (KV block, KV head).
  {
    std::vector<int32_t> dep_count(p->n_kv_blocks + 1, 0);
    for (int i = 0; i < p->n_pairs; i++) dep_count[p->pairs[i].kv_blk + 1]++;
    for (int b = 0; b < p->n_kv_blocks; b++) dep_count[b + 1] += dep_count[b];
    std::vector<int32_t> cursor(dep_count.begin(), dep_count.end() - 1);
    BwdDep* deps = reinterpret_cast<BwdDep*>(host.data() + L.off_bwd_deps);
    for (int i = 0; i < p->n_pairs; i++) {           // pairs are visited in q order -> deps ascend in q
      const fcp_block& qb = p->q_blocks[p->pairs[i].q_blk];
      deps[cursor[p->pairs[i].kv_blk]++] = {qb.tok_start, qb.tok_len, p->pairs[i].kind, dpairs[i].ds_frag};
    }
    // The DIAG dependency goes last: the tiles of one KV block then walk the FULL dependencies in
    // lockstep (identical step sequences, same XCD), so the Q / dO stream they share stays in L2;
    // they only diverge on the diagonal block, where each tile starts at its own row.
    for (int b = 0; b < p->n_kv_blocks; b++)
      std::stable_partition(deps + dep_count[b], deps + dep_count[b + 1],
                            [](const BwdDep& d) { return !(d.kind & 1); });
    std::vector<std::vector<BwdItem>> groups;
    std::vector<int64_t> weight, gkey;
    groups.reserve((size_t)p->n_kv_blocks * p->n_kv_heads);
    for (int b = 0; b < p->n_kv_blocks; b++) {
      const fcp_block& kb = p->kv_blocks[b];
      const int n_tiles = (int)ceil_div(kb.tok_len, kBwdTileN);
      const int d0 = dep_count[b], nd = dep_count[b + 1] - dep_count[b];
      std::vector<int64_t> tile_w(n_tiles, 0);
      for (int t = 0; t < n_tiles; t++) {
        const int off = t * kBwdTileN;
        const int rows = std::min(kBwdTileN, kb.tok_len - off);
        for (int i = d0; i < d0 + nd; i++) {
          const int qrows = (deps[i].kind & 1) ? std::max(0, deps[i].q_len - off) : deps[i].q_len;
          tile_w[t] += (int64_t)rows * qrows * G;
        }
      }
      const int packed_kind = (nd == 1 && (deps[d0].kind & 2)) ? deps[d0].kind : 0;
      std::vector<int> q_end(n_tiles, 0);
      if (packed_kind) {
        // a KV tile serves the dQ items whose columns meet its own: a contiguous run of row tiles, since the members
        // follow each other; under a causal mask it starts at the tile itself
        std::vector<int> lo, hi;
        packed_tile_columns(kb.tok_len, G, q_seg + deps[d0].q_start, (packed_kind & 1) != 0, &lo, &hi);
        for (int t = 0; t < n_tiles; t++) {
          const int c0 = t * kBwdTileN, c1 = std::min(kb.tok_len, c0 + kBwdTileN);
          for (int k = 0; k < (int)lo.size(); k++)
            if (lo[k] < c1 && hi[k] > c0) q_end[t] = std::min(kb.tok_len, (k + 1) * kFwdTileM);
          tile_w[t] = (int64_t)(c1 - c0) * std::max(0, q_end[t] - ((packed_kind & 1) ? c0 : 0)) * G;
        }
      }
      for (int g = 0; g < p->n_kv_heads; g++) {
        std::vector<BwdItem> items;
        int64_t w = 0;
        for (int t = 0; t < n_tiles; t++) {            // earlier tiles of a DIAG pair are heavier
          const int off = t * kBwdTileN;
          items.push_back({kb.tok_start + off, std::min(kBwdTileN, kb.tok_len - off), off, d0, nd, g, kb.tok_len,
                           packed_kind, q_end[t], 0});
          w += tile_w[t];
        }
        groups.push_back(std::move(items));
        weight.push_back(w);
        gkey.push_back((int64_t)kb.seq * p->n_kv_heads + g);
      }
    }
    merge_groups_by_key(groups, weight, gkey);
    std::vector<BwdItem> flat;
    spread_over_xcds(groups, weight, &flat, hdr->bwd_begin);
    if ((int64_t)flat.size() != L.n_bwd_items) { set_error("internal: backward item count mismatch"); return FCP_ERR_INVALID_ARG; }
    if (!flat.empty()) std::memcpy(host.data() + L.off_bwd_items, flat.data(), flat.size() * sizeof(BwdItem));
  }
  // ---- backward dQ: query-stationary items over ALL pairs of a query block (its slots are
  // consecutive, so their pairs form one range); one group per (query block, KV head); items
  // join two sub-tiles like the forward's.
  {
    std::vector<int32_t> pb(p->n_q_blocks, 0), pn(p->n_q_blocks, 0);
    for (int s = 0; s < p->n_slots; s++) {
      const fcp_slot& sl = p->slots[s];
      if (pn[sl.q_blk] == 0) pb[sl.q_blk] = sl.pair_begin;
      pn[sl.q_blk] += sl.n_pairs;
    }
    std::vector<std::vector<QItem>> groups;
    std::vector<int64_t> weight, gkey;
    groups.reserve((size_t)p->n_q_blocks * p->n_kv_heads);
    for (int b = 0; b < p->n_q_blocks; b++) {
      const fcp_block& qb = p->q_blocks[b];
      const int n_tiles = (int)ceil_div(qb.tok_len, kFwdTileM);
      std::vector<int64_t> tile_w(n_tiles, 0);
      for (int t = 0; t < n_tiles; t++) {
        const int off = t * kFwdTileM;
        const int rows = std::min(kFwdTileM, qb.tok_len - off);
        for (int i = pb[b]; i < pb[b] + pn[b]; i++) {
          const int cols = (dpairs[i].kind & 1) ? std::min(dpairs[i].kv_len, off + rows) : dpairs[i].kv_len;
          tile_w[t] += (int64_t)rows * cols;
        }
      }
      const int packed_kind = (pn[b] == 1 && (dpairs[pb[b]].kind & 2)) ? dpairs[pb[b]].kind : 0;
      auto finish = [&](QItem* it) {
        if (packed_kind) packed_columns(it, q_seg + qb.tok_start, (packed_kind & 1) != 0);
        count_tiles(it, dpairs);
      };
      auto sub = [&](QItem* it, int k, int t, int head) {
        const int off = t * kFwdTileM;
        it->q_start[k] = qb.tok_start + off; it->q_rows[k] = std::min(kFwdTileM, qb.tok_len - off);
        it->out_row[k] = qb.tok_start + off; it->tile_off[k] = off; it->head[k] = head;
      };
      for (int g = 0; g < p->n_kv_heads; g++) {
        std::vector<QItem> items;
        int64_t w = 0;
        if (G % 2 == 0) {
          for (int t = n_tiles - 1; t >= 0; t--)
            for (int hh = 0; hh < G; hh += 2) {
              QItem it{};
              it.pair_begin = pb[b]; it.n_pairs = pn[b]; it.q_blk_len = qb.tok_len;
              sub(&it, 0, t, g * G + hh); sub(&it, 1, t, g * G + hh + 1);
              finish(&it);
              items.push_back(it);
              w += 2 * tile_w[t];
            }
        } else {
          for (int t = n_tiles - 1; t >= 0; t -= 2)
            for (int hh = 0; hh < G; hh++) {
              QItem it{};
              it.pair_begin = pb[b]; it.n_pairs = pn[b]; it.q_blk_len = qb.tok_len;
              sub(&it, 0, t, g * G + hh);
              if (t >= 1) { sub(&it, 1, t - 1, g * G + hh); w += tile_w[t - 1]; }
              else { it.q_start[1] = it.q_start[0]; it.q_rows[1] = 0; it.out_row[1] = it.out_row[0]; it.tile_off[1] = it.tile_off[0]; it.head[1] = it.head[0]; }
              finish(&it);
              items.push_back(it);
              w += tile_w[t];
            }
        }
        groups.push_back(std::move(items));
        weight.push_back(w);
        gkey.push_back((int64_t)qb.seq * p->n_kv_heads + g);
      }
    }
    merge_groups_by_key(groups, weight, gkey);
    std::vector<QItem> flat;
    spread_over_xcds(groups, weight, &flat, hdr->dq_begin);
    if ((int64_t)flat.size() != L.n_dq_items) { set_error("internal: dQ item count mismatch"); return FCP_ERR_INVALID_ARG; }
    if (!flat.empty()) std::memcpy(host.data() + L.off_dq_items, flat.data(), flat.size() * sizeof(QItem));
  }
  // ---- merge: row-head chunks per query block; slots of a query block are consecutive.
  {
    std::vector<int32_t> slot_begin(p->n_q_blocks + 1, 0);
    for (int s = 0; s < p->n_slots; s++) slot_begin[p->slots[s].q_blk + 1]++;
    for (int b = 0; b < p->n_q_blocks; b++) slot_begin[b + 1] += slot_begin[b];
    int32_t* slot_rh = reinterpret_cast<int32_t*>(host.data() + L.off_slot_rh);
    for (int s = 0; s < p->n_slots; s++) {
      const int64_t rh = (int64_t)p->slots[s].row_start * p->n_q_heads;
      if (rh > INT32_MAX) { set_error("partial buffers exceed 2^31-1 (row, head) entries"); return FCP_ERR_UNSUPPORTED; }
      slot_rh[s] = (int32_t)rh;
    }
    MergeItem* mi = reinterpret_cast<MergeItem*>(host.data() + L.off_merge_items);
    int64_t n = 0;
    for (int b = 0; b < p->n_q_blocks; b++) {
      const fcp_block& qb = p->q_blocks[b];
      if ((p->flags & FCP_FLAG_DIRECT_SINGLE) && slot_begin[b + 1] - slot_begin[b] == 1) continue;   // written by the forward
      const int64_t total = (int64_t)qb.tok_len * p->n_q_heads;
      for (int64_t off = 0; off < total; off += L.merge_chunk) {
        mi[n++] = {(int32_t)((int64_t)qb.tok_start * p->n_q_heads + off), (int32_t)std::min<int64_t>(L.merge_chunk, total - off),
                   slot_begin[b], slot_begin[b + 1] - slot_begin[b], (int32_t)off, 0, 0, 0};
      }
    }
    if (n != L.n_merge_items) { set_error("internal: merge item count mismatch"); return FCP_ERR_INVALID_ARG; }
  }
  return FCP_OK;
}

extern "C" int fcp_queue_build(const fcp_problem* p, void* workspace, size_t workspace_bytes, void* stream) {
  int rc = validate_problem(p);
  if (rc) return rc;
  WsLayout L;
  rc = compute_layout(p, &L);
  if (rc) return rc;
  if (!workspace || ((uintptr_t)workspace & 255)) {
    set_error("fcp_queue_build: workspace is NULL or not 256-byte aligned"); return FCP_ERR_INVALID_ARG;
  }
  if (workspace_bytes < L.total) {
    set_error("fcp_queue_build: workspace too small (%zu < %zu)", workspace_bytes, L.total);
    return FCP_ERR_BUFFER_TOO_SMALL;
  }
  std::vector<unsigned char> host;
  rc = build_queue_image(p, L, false, &host);
  if (rc) return rc;
  hipError_t e = hipMemcpyAsync(workspace, host.data(), host.size(), hipMemcpyHostToDevice, (hipStream_t)stream);
  if (e == hipSuccess) e = hipStreamSynchronize((hipStream_t)stream);
  if (e != hipSuccess) { set_error("fcp_queue_build: %s", hipGetErrorString(e)); return FCP_ERR_HIP; }
  remember_layout(p, workspace, L);
  return FCP_OK;
}
