// Internal layout shared by the host scheduler and the HIP kernels (not part of the ABI).
#ifndef FCP_INTERNAL_H_
#define FCP_INTERNAL_H_

#include <stddef.h>
#include <stdint.h>

#include <vector>

#include "fcp.h"

namespace fcp {

constexpr int kNumXcd = 8;          // MI355X: 8 XCDs, each with its own L2; workgroup b runs on XCD b % 8
constexpr int kFwdTileM = 128;      // query rows per query-stationary work item (4 waves x 32 rows)
constexpr int kBwdTileN = 128;      // KV rows per backward work item (4 waves x 32 rows)
constexpr int kMergeChunk = 1024;   // most (row, head) entries per merge work item (fewer when there is little to merge)
constexpr int kMergeMinItems = 2048;  // the merge aims at this many work items at least: 8 per compute unit

// Device-side records (all int32 so the host can build them as plain arrays).
// ds_frag: first 32x32 dS fragment of the pair in the spill buffer (FCP_FLAG_BWD_SPILL_DS; else 0).
struct DevPair { int32_t kv_start, kv_len, kind, ds_frag; };
// Query-stationary item of two 128-row sub-tiles that walk the same pair list and share a KV head
// (two query heads of a group, or two neighbouring row tiles of one head; q_rows[1] = 0: none).
// to_final != 0 (forward items only): the slot is the only one of its query block.
// q_blk_len (dQ items only): rows of the whole query block.
// n_tiles: 64-row KV tiles the item walks (a DIAG pair only up to the item's last query row).
// col_begin, col_end: items of a packed query block (its one pair has a PACKED kind) walk only the columns
// [col_begin, col_end) that some row of the item can see, col_begin a multiple of kQTileN; col_end = 0 otherwise.
struct QItem { int32_t q_start[2], q_rows[2], out_row[2], tile_off[2], head[2], pair_begin, n_pairs, to_final, q_blk_len, n_tiles, col_begin, col_end, pad; };
constexpr int kQTileN = 64;         // KV rows per LDS tile of the query-stationary kernels
struct BwdDep  { int32_t q_start, q_len, kind, ds_frag; };
// packed: the KV block is a packed block (its one dependency has a PACKED kind, which this field holds); the item then
// walks the query rows up to q_end only: the rows of every dQ item whose column range meets this tile's columns
// (later rows belong to other members; with the dS spill, the dQ pass reads exactly the fragments written this way).
struct BwdItem { int32_t kv_start, kv_rows, tile_off, dep_begin, n_deps, kv_head, kv_blk_len, packed, q_end, pad; };
// Member bounds of one token of a packed block, as the kernels read them per query row (q_seg) or per KV row
// (kv_seg): first token of its member in the low half, one past its last in the high half, both inside the block.
inline uint32_t seg_word(int lo, int hi) { return (uint32_t)lo | ((uint32_t)hi << 16); }
constexpr int kMaxPackedBlock = 65535;   // tokens; the halves above are 16 bits

// The dS spill buffer (FCP_FLAG_BWD_SPILL_DS) is a sequence of 2 KB fragments, one per (pair, query head,
// 32 query rows, 32 KV rows).  Fragments [0, kDsSinkFrags) take the stores of steps that have no fragment
// (pipeline fill, tiles above the diagonal); a pair's fragments follow from its ds_frag, head-major, then by
// 32-row query group; a FULL pair keeps ceil(kv_len / 32) fragments per query group, a DIAG pair only those at or
// below the diagonal (query group i keeps i + 1); the PACKED kinds keep what FULL / DIAG keep (entries between
// different members are stored as zeros).
constexpr int kDsFragBytes = 2048;
constexpr int kDsSinkFrags = 256;
inline int64_t ds_frags_per_head(int kind, int q_len, int kv_len) {
  const int64_t nq = (q_len + 31) / 32, nk = (kv_len + 31) / 32;
  return (kind & 1) ? nq * (nq + 1) / 2 : nq * nk;   // DIAG and PACKED_DIAG: at or below the diagonal
}
struct MergeItem { int32_t out_rh, n_rh, slot_begin, n_slots, rh_off, pad0, pad1, pad2; };

// Header at the start of the workspace.  Counters are zero between launches: the last
// workgroup of a persistent launch to run dry clears the ones it used.
struct WsHeader {
  int32_t fwd_counter[kNumXcd];
  int32_t bwd_counter[kNumXcd];
  int32_t dq_counter[kNumXcd];
  int32_t fwd_done, bwd_done, dq_done, pad0[5];
  int32_t fwd_begin[kNumXcd + 1];   // item range of each XCD queue
  int32_t pad1[7];
  int32_t bwd_begin[kNumXcd + 1];
  int32_t pad2[7];
  int32_t dq_begin[kNumXcd + 1];
  int32_t pad3[7];
  int32_t zeros[64];                // 256-byte zero page: source of LDS-DMA loads past a ragged end
  float infs[64];                   // +inf page: LSE of query rows past a ragged end (their P is 0)
  // Forward items of packed query blocks have queues of their own (they follow the others in the item array),
  // drained by a second launch of the kernel instance that knows their mask.
  int32_t fwdp_counter[kNumXcd];
  int32_t fwdp_begin[kNumXcd + 1];
  int32_t fwdp_done, pad4[6];
};

// Byte offsets of the workspace sections, a pure function of the problem's counts.
struct WsLayout {
  int64_t n_fwd_items, n_bwd_items, n_bwd_deps, n_merge_items, n_dq_items, t_q, t_kv;
  int64_t n_fwd_packed_items;   // those of n_fwd_items that belong to packed query blocks
  int fwd_tile_m;   // query rows per forward item, chosen per problem
  int merge_chunk;  // (row, head) entries per merge work item, chosen per problem
  int64_t n_ds_frags;   // fragments of the dS spill buffer, sinks and one fragment of slack included (0 without the flag)
  size_t off_q_seg, off_kv_seg;   // member bounds per Q-buffer row / KV-buffer row (empty without packed blocks)
  size_t off_pairs, off_fwd_items, off_bwd_deps, off_bwd_items, off_merge_items, off_slot_rh, off_dq_items, off_dls, off_lse2, off_ds, total;
};

int validate_problem(const fcp_problem* p);           // host; sets the error text
int compute_layout(const fcp_problem* p, WsLayout* L); // host
// the layout of a problem on a workspace: from the registry that fcp_queue_build fills, else validated and computed
int layout_for(const fcp_problem* p, const void* workspace, WsLayout* L);   // host
void remember_layout(const fcp_problem* p, const void* workspace, const WsLayout& L);
void set_error(const char* fmt, ...);
int build_queue_image(const fcp_problem* p, const WsLayout& L, bool forward_only, std::vector<unsigned char>* image);  // host

}  // namespace fcp
#endif
