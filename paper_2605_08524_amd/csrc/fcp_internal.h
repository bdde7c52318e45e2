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
struct DevPair { int32_t kv_start, kv_len, kind, pad; };
// Query-stationary item of two 128-row sub-tiles that walk the same pair list and share a KV head
// (two query heads of a group, or two neighbouring row tiles of one head; q_rows[1] = 0: none).
// pad[0] != 0 (forward items only): the slot is the only one of its query block.
struct QItem { int32_t q_start[2], q_rows[2], out_row[2], tile_off[2], head[2], pair_begin, n_pairs, pad[4]; };
struct BwdDep  { int32_t q_start, q_len, kind, pad; };
struct BwdItem { int32_t kv_start, kv_rows, tile_off, dep_begin, n_deps, kv_head, pad0, pad1; };
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
};

// Byte offsets of the workspace sections, a pure function of the problem's counts.
struct WsLayout {
  int64_t n_fwd_items, n_bwd_items, n_bwd_deps, n_merge_items, n_dq_items, t_q, t_kv;
  int fwd_tile_m;   // query rows per forward item, chosen per problem
  int merge_chunk;  // (row, head) entries per merge work item, chosen per problem
  size_t off_pairs, off_fwd_items, off_bwd_deps, off_bwd_items, off_merge_items, off_slot_rh, off_dq_items, off_dls, off_lse2, total;
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
