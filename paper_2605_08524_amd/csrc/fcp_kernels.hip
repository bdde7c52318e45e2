// HIP kernels for gfx950 (MI355X) and their launchers.
//
// Contractions run on v_mfma_f32_32x32x16_bf16.  Operand layouts (64 lanes, l = lane):
//   A (32 x 16): lane holds row l%32, k = 8*(l/32) .. +7          (8 bf16 = 4 VGPRs)
//   B (16 x 32): lane holds col l%32, k = 8*(l/32) .. +7
//   C/D (32 x 32 fp32, 16 VGPRs): reg r of lane l = row 8*(r/4) + 4*(l/32) + r%4, col l%32
// Because a sum over k does not care about the order of k, any k-slot assignment is valid as
// long as A and B use the same one; the kernels exploit this to feed an accumulator straight
// back as the B operand of the next contraction.
//
// ds_read_b64_tr_b16 (LDS transpose read): inside each group of 16 lanes, lane i receives, for
// e = 0..3, element (i%4) of the 8-byte row addressed by lane 4*e + i/4.  With lane s of a
// group pointing at M[r0 + s/4][c0 + 4*(s%4)], lane i ends up with M[r0 + 0..3][c0 + i]: four
// consecutive rows of one column, which is what an MFMA operand needs when the contracted index
// runs down the rows of a row-major LDS tile.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <type_traits>
#include <vector>

#include "fcp_internal.h"

namespace fcp {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

#define LDS_PTR(T, p) ((__attribute__((address_space(3))) T*)(p))

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  f32x2 f = {a, b};
  bf16x2 h = __builtin_convertvector(f, bf16x2);   // round-to-nearest-even
  return __builtin_bit_cast(uint32_t, h);
}

// Two transpose reads -> one 8-slot MFMA operand.
__device__ __forceinline__ bf16x8 lds_tr_pair(const unsigned char* lo, const unsigned char* hi) {
  s16x4 a = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, lo));
  s16x4 b = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, hi));
  typedef __attribute__((ext_vector_type(8))) short s16x8;
  s16x8 c = __builtin_shufflevector(a, b, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, c);
}

__device__ __forceinline__ float xor32(float x) { return __shfl_xor(x, 32, 64); }

// Stores one 32x32 accumulator tile as bf16 when a lane owns one output row: lane (l32, g) holds the
// 16 values of columns 8*q4 + 4*g .. +3 (q4 = 0..3) of its row, its partner (lane ^ 32, same row)
// the other four of every group of eight.  The two trade halves so that each stores 16 contiguous
// bytes (8 columns): the lower lane keeps the even groups, the upper lane the odd ones.
// dst = first of the tile's 32 columns in this lane's row.  Both lanes of a row must be active.
__device__ __forceinline__ void store_tile_bf16(uint16_t* dst, const f32x16& x, float mul, int g) {
#pragma unroll
  for (int m = 0; m < 2; m++) {
    const uint32_t e0 = pack_bf16(x[8 * m] * mul, x[8 * m + 1] * mul), e1 = pack_bf16(x[8 * m + 2] * mul, x[8 * m + 3] * mul);
    const uint32_t f0 = pack_bf16(x[8 * m + 4] * mul, x[8 * m + 5] * mul), f1 = pack_bf16(x[8 * m + 6] * mul, x[8 * m + 7] * mul);
    // swap(x, y): lanes 32-63 of x trade places with lanes 0-31 of y
    const u32x2 r = __builtin_amdgcn_permlane32_swap(e0, f0, false, false);
    const u32x2 t = __builtin_amdgcn_permlane32_swap(e1, f1, false, false);
    const u32x4 h = {r[0], t[0], r[1], t[1]};
    *reinterpret_cast<u32x4*>(dst + 16 * m + 8 * g) = h;
  }
}

// LDS accesses through 32-bit LDS addresses kept in registers: a tile buffer switch is then one
// add per address (in place) and row / tile offsets fold into the instruction's immediate field.
__device__ __forceinline__ uint32_t lds_addr(const void* p) {
  return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const unsigned char*)p;
}
__device__ __forceinline__ u32x4 lds_read16(uint32_t addr) {
  return *(const __attribute__((address_space(3))) u32x4*)(uintptr_t)addr;
}
__device__ __forceinline__ bf16x8 lds_tr_pair_at(uint32_t lo, uint32_t hi) {
  s16x4 a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(uintptr_t)lo);
  s16x4 b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(uintptr_t)hi);
  typedef __attribute__((ext_vector_type(8))) short s16x8;
  s16x8 c = __builtin_shufflevector(a, b, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, c);
}

// Byte offset of 16-byte chunk c of row r in an LDS tile.  Rows are unpadded (D*2 bytes) because
// tiles are filled by LDS-DMA loads that write 1 KB of consecutive LDS per wave instruction; the
// chunk index is XOR-swizzled with the row so that both access patterns are conflict free for
// D = 128 (rows of exactly 64 banks): row-wise ds_read_b128 (16 lanes = 16 consecutive rows, one
// chunk column) and transpose reads (32 lanes = 4 consecutive rows x 4 consecutive chunks).
template <int D>
__device__ __forceinline__ int swz(int r) {
  if constexpr (D == 128) return ((r & 3) << 2) | ((r >> 2) & 3);
  else return (r >> 1) & 7;
}
template <int D>
__device__ __forceinline__ int tile_off(int r, int c) { return r * (D * 2) + ((c ^ swz<D>(r)) << 4); }

// Asynchronous copy of a [ROWS x D] bf16 tile from global memory straight into LDS (no
// registers): each global_load_lds_dwordx4 moves 64 x 16 B into 1 KB of consecutive LDS, so lane
// i of instruction n fills physical chunk i % (D/8) of row n*(1024/(2D)) + i/(D/8) and fetches
// the logical chunk that the swizzle places there.  Rows >= valid_rows are filled from a zero
// page.  Completion: s_waitcnt vmcnt(0) by the issuing wave, then a workgroup barrier.
// The load is issued through inline assembly on purpose: the compiler then does not model it as
// a write to LDS, so it does not make every later LDS read of the *other* buffer wait for it
// (it cannot tell run-time-indexed buffers apart).  Ordering is explicit instead: dma_wait()
// and a barrier before anyone reads what was loaded.  m0 carries the wave-uniform LDS address.
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"   // m0 is clobbered on purpose; nothing else here lives in it
__device__ __forceinline__ void lds_dma16(const unsigned char* gptr, uint32_t lds_addr) {
  const uint32_t m0 = __builtin_amdgcn_readfirstlane(lds_addr);
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
               :: "v"(gptr), "s"(m0) : "memory", "m0");
}
#pragma clang diagnostic pop
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void lds_dma16_s(const unsigned char* sbase, uint32_t voff, uint32_t lds_addr) {
  const uint32_t m0 = __builtin_amdgcn_readfirstlane(lds_addr);
  const uint64_t b = reinterpret_cast<uint64_t>(sbase);       // wave-uniform by construction
  // readfirstlane returns a signed int: widen through uint32_t, or the low half sign-extends
  // into the high half of the address.
  const uint32_t b_lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)b);
  const uint32_t b_hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(b >> 32));
  const uint64_t sb = ((uint64_t)b_hi << 32) | (uint64_t)b_lo;
  // s_nop 4: a vector-memory instruction may read an SGPR only 5 wait states after a scalar or
  // v_readfirstlane write to it; the compiler's hazard pass does not look inside inline assembly,
  // and the base in %1 is typically produced right before this statement.  (Also covers m0.)
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 4\n\tglobal_load_lds_dwordx4 %0, %1"
               :: "v"(voff), "s"(sb), "s"(m0) : "memory", "m0");
}
#pragma clang diagnostic pop
// Same for 64 x 4 bytes: lane i's dword lands at lds_addr + 4*i.
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void lds_dma4(const float* gptr, uint32_t lds_addr) {
  const uint32_t m0 = __builtin_amdgcn_readfirstlane(lds_addr);
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dword %0, off"
               :: "v"(gptr), "s"(m0) : "memory", "m0");
}
#pragma clang diagnostic pop
// Byte offset, from the first row of a 1 KB load instruction, of the chunk that lane `lane` of
// wave `wave` fetches.  Instruction n*NWAVES + wave covers rows that differ from wave's first
// instruction by a multiple of 16, the period of the swizzle, so the offset is one per-lane
// constant for the whole kernel.
template <int D>
__device__ __forceinline__ uint32_t dma_lane_offset(int wave, int lane, int64_t row_stride) {
  constexpr int CPR = D / 8, RPI = 64 / CPR;
  const int r = wave * RPI + lane / CPR, pc = lane % CPR;
  return (uint32_t)((lane / CPR) * row_stride * 2 + ((pc ^ swz<D>(r)) << 4));
}
template <int D, int ROWS, int NWAVES>
__device__ __forceinline__ void tile_dma(unsigned char* lds_tile, const uint16_t* src, int64_t row_stride,
                                         int valid_rows, const unsigned char* zeros, int wave, int lane,
                                         uint32_t lane_off) {
  constexpr int CPR = D / 8, RPI = 64 / CPR, NI = ROWS / RPI;
  static_assert(NI % NWAVES == 0, "tile does not split evenly over the waves");
  const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)lds_tile;
  if (valid_rows >= ROWS) {
    // whole tile in range (wave-uniform): scalar base per instruction + the per-lane constant
#pragma unroll
    for (int n = 0; n < NI / NWAVES; n++) {
      const int inst = n * NWAVES + wave;
      lds_dma16_s(reinterpret_cast<const unsigned char*>(src + (int64_t)inst * RPI * row_stride), lane_off,
                  lds_base + inst * 1024);
    }
    return;
  }
#pragma unroll
  for (int n = 0; n < NI / NWAVES; n++) {
    const int inst = n * NWAVES + wave;
    const int r = inst * RPI + lane / CPR;
    const int pc = lane % CPR;
    const unsigned char* gp = zeros + pc * 16;
    if (r < valid_rows) gp = reinterpret_cast<const unsigned char*>(src + (int64_t)r * row_stride + ((pc ^ swz<D>(r)) << 3));
    lds_dma16(gp, lds_base + inst * 1024);
  }
}
__device__ __forceinline__ void dma_wait() { __builtin_amdgcn_s_waitcnt(0x0F70); }   // vmcnt(0)

template <int D> constexpr int tile_bytes(int rows) { return rows * D * 2; }

// Pop one item index from the eight XCD queues, own queue first, then stealing.  Returns -1
// when every queue is dry.  Every call terminates: each queue is probed at most once.
__device__ __forceinline__ int pop_item(int32_t* counter, const int32_t* begin) {
  // The XCD this workgroup actually runs on: hardware register XCC_ID (id 20), bits [3:0].
  const int home = __builtin_amdgcn_s_getreg((3 << 11) | 20) & (kNumXcd - 1);
  for (int t = 0; t < kNumXcd; t++) {
    const int q = (home + t) % kNumXcd;
    const int n = begin[q + 1] - begin[q];
    if (n <= 0) continue;
    if (__hip_atomic_load(&counter[q], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= n) continue;
    const int i = atomicAdd(&counter[q], 1);
    if (i < n) return begin[q] + i;
  }
  return -1;
}

// The last workgroup to run dry clears the counters for the next launch.
__device__ __forceinline__ void retire(int32_t* counter, int32_t* done) {
  const int prev = atomicAdd(done, 1);
  if (prev == (int)gridDim.x - 1) {
    for (int q = 0; q < kNumXcd; q++) atomicExch(&counter[q], 0);
    atomicExch(done, 0);
  }
}

// The item sequence of one persistent workgroup of a query-stationary kernel.  The index of the NEXT item is
// requested when the current one starts (one atomic add on the home queue by thread 0, not waited for) and
// published through LDS when the current one ends, so the round trip to the counter overlaps the item's work
// instead of sitting between two items.  Once the home queue runs dry the slower pop_item (which also steals
// from the other queues) takes over; every workgroup leaves the loop when all queues are dry.
struct ItemStream {
  int32_t* counter; const int32_t* begin;
  int home, home_n, home_begin, ticket;
  bool home_dry;
  __device__ __forceinline__ void init(int32_t* c, const int32_t* b) {
    counter = c; begin = b;
    home = __builtin_amdgcn_s_getreg((3 << 11) | 20) & (kNumXcd - 1);
    home_begin = b[home]; home_n = b[home + 1] - home_begin;
    home_dry = home_n <= 0; ticket = 0;
  }
  // thread 0 only: ask for the next item (returns at once; the ticket arrives while the item runs)
  __device__ __forceinline__ void request() { if (!home_dry) ticket = atomicAdd(&counter[home], 1); }
  // thread 0 only: the item the ticket stands for, or one stolen elsewhere, or -1
  __device__ __forceinline__ int resolve() {
    if (!home_dry) {
      if (ticket < home_n) return home_begin + ticket;
      home_dry = true;
    }
    return pop_item(counter, begin);
  }
};

// =====================================================================================
// Forward: partial attention.  Item = (slot, two 128-row query sub-tiles that share the slot's
// K/V stream: two query heads of one KV head, or two neighbouring row tiles of one head);
// workgroup of 8 waves, two per SIMD, 32 query rows per wave.
// The wave computes S^T = K Q^T so that a lane owns one query row (column of S^T): row
// statistics need one cross-half exchange, and the exponentiated accumulator is, as is,
// the B operand of O^T += V^T P^T.  The loop over 64-row K/V tiles is software-pipelined by
// hand: in iteration i the wave issues the MFMAs of S(i+1) and then of O += V(i)^T P(i), and
// places the exponentials of tile i, and later the maximum of tile i+1, between them, so the
// matrix pipe does not wait for the vector ALU inside a wave.  [K | V] tiles sit in a ring of
// four LDS buffers filled by LDS-DMA three tiles ahead (all 8 waves share one stream); one
// workgroup barrier per tile.  The first iteration of an item computes S of its first tile only
// and the last one only adds the last tile to O, so the pipeline fill costs no MFMAs; all
// iterations issue the same tile loads, and the ring runs on from item to item.
// =====================================================================================
constexpr int kFwdTileN = kQTileN;   // KV rows per LDS tile (the host counts an item's tiles with the same constant)
constexpr int kFwdBufs = 4;     // ring of [K | V] tile buffers
constexpr float kRescaleSlack = 8.0f;   // log2 units

struct FwdArgs {
  const uint16_t* q; const uint16_t* k; const uint16_t* v;
  void* o_part; float* lse_part; int32_t part_is_bf16;
  void* o; float* lse; int32_t o_is_f32;     // final outputs for query blocks with a single slot (or NULL)
  int32_t running;                            // fold every slot into the running (o, lse) in place (fp32 o)
  WsHeader* hdr; const DevPair* pairs; const QItem* items;
  int32_t* counter; const int32_t* begin; int32_t* done;   // the XCD queues this launch drains (header fields)
  const uint32_t* q_seg;                      // member bounds per Q-buffer row (packed blocks only)
  int32_t n_q_heads, n_kv_heads;
  float scale_log2;   // softmax scale * log2(e)
};

// Iterator over the KV tiles of an item's pairs, in pair order.  For a DIAG pair only the
// columns up to the tile's last query row are visited, for a PACKED pair the item's column range.
struct TileIter {
  const DevPair* pairs;
  int pair, pair_end, c0, ncols, row_hi;   // row_hi = tile_off + q_rows (first row past the tile)
  DevPair cur;
  bool more;
  __device__ __forceinline__ void load_pair() {
    // the pair index is wave-uniform; readfirstlane says so to the compiler, which then keeps the record (and
    // everything derived from it) in scalar registers and branches on it with scalar branches
    const DevPair p = pairs[pair];
    cur.kv_start = __builtin_amdgcn_readfirstlane(p.kv_start); cur.kv_len = __builtin_amdgcn_readfirstlane(p.kv_len);
    cur.kind = __builtin_amdgcn_readfirstlane(p.kind); cur.ds_frag = __builtin_amdgcn_readfirstlane(p.ds_frag);
    ncols = (cur.kind & 1) ? min(cur.kv_len, row_hi) : cur.kv_len;
  }
  __device__ __forceinline__ void init(const DevPair* p, const QItem& it) {
    pairs = p; pair = it.pair_begin; pair_end = it.pair_begin + it.n_pairs; c0 = 0; ncols = 0;
    row_hi = max(it.tile_off[0] + it.q_rows[0], it.tile_off[1] + it.q_rows[1]);
    cur = DevPair{0, 0, 0, 0};
    more = it.n_pairs > 0;
    if (more) load_pair();
    // a PACKED pair is the only pair of its item: the item's column range replaces the pair's, here and nowhere else
    if (it.col_end > 0) { c0 = it.col_begin; ncols = it.col_end; }
  }
  __device__ __forceinline__ void advance() {
    c0 += kFwdTileN;
    if (c0 >= ncols) {
      pair++;
      c0 = 0;
      if (pair < pair_end) load_pair(); else more = false;
    }
  }
};

// What a wave needs to know about a tile when it masks it: first column, visible length, kind of its pair.
// A tile past the end of the item has len = 0: everything is masked.
struct TileMeta { int c0, len, kind; };

// PACKED: the instance for the items of packed blocks (several short sequences in one block), which have queues of
// their own and a launch of their own; only it carries the per-row member bounds and the second mask, which cost
// the other instance 4 % when they were compiled into it.
template <int D, bool PACKED>
__global__ void __launch_bounds__(512, 2) fwd_kernel(FwdArgs a) {
  constexpr int KC = D / 16;      // k-chunks of the QK^T contraction
  constexpr int DT = D / 32;      // row tiles of O^T
  constexpr int NS1 = 2 * KC;     // MFMAs of S^T (two 32-row halves of the KV tile)
  constexpr int NS2 = 4 * DT;     // MFMAs of O^T += V^T P^T
  constexpr int PF = 4;           // an LDS operand is requested this many MFMAs before its use
  constexpr int TB = tile_bytes<D>(kFwdTileN);
  constexpr int BUF = 2 * TB;     // [K tile | V tile]
  constexpr int NB = kFwdBufs;
  constexpr int CPR = D / 8, RPI = 64 / CPR, NDMA = kFwdTileN / RPI / 8;   // LDS-DMA geometry, see issue()
  constexpr int DMA_PER_TILE = 2 * NDMA;
  __shared__ __attribute__((aligned(1024))) unsigned char lds_kv[NB][BUF];
  __shared__ uint32_t s_seg[512];   // member bounds of each lane's query row in a packed block (written and read by that lane)
  __shared__ int s_item;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform, kept in a scalar register
  const int sub = wave >> 2, wq = wave & 3;                    // sub-item, 32-row group inside it
  const int l32 = lane & 31, g = lane >> 5;
  const int group = a.n_q_heads / a.n_kv_heads;
  const int64_t q_row_stride = (int64_t)a.n_q_heads * D;     // elements
  const int64_t kv_row_stride = (int64_t)a.n_kv_heads * D;
  const unsigned char* zeros = reinterpret_cast<const unsigned char*>(a.hdr->zeros);
  // LDS-DMA of a 64-row tile: instruction n of this wave fills LDS rows r_n = (8n + wave) * RPI + lane / CPR.
  // A lane fetches chunk (pc ^ swz(r_n)) of global row min(r_n, valid - 1): rows past a ragged end
  // repeat the last valid row (finite values; those columns are masked).
  uint32_t dma_row[NDMA], dma_chunk[NDMA];
#pragma unroll
  for (int n = 0; n < NDMA; n++) {
    const int r = (8 * n + wave) * RPI + lane / CPR, pc = lane % CPR;
    dma_row[n] = (uint32_t)(r * kv_row_stride * 2);
    dma_chunk[n] = (uint32_t)((pc ^ swz<D>(r)) << 4);
  }
  // transpose-read pattern inside a 16-lane group: row tr_row, 4 columns from tr_col
  const int tr_row = (lane & 15) >> 2, tr_col = 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
  for (int i = tid * 16; i < NB * BUF; i += 512 * 16)
    *reinterpret_cast<u32x4*>(&lds_kv[0][0] + i) = u32x4{0, 0, 0, 0};
  // Ring positions, advanced by one buffer per tile and kept across items: in iteration i the
  // wave reads the K rows of tile i+1 (b_k), transposes V of tile i (b_v), and tile i+3 is requested (b_dma).
  int b_k = 0, b_v = NB - 1, b_dma = 2;
  // Per-lane LDS addresses into the current buffers (the swizzle has period 16 in the row, so
  // rows +16 / +32 are plain immediate offsets), advanced in place.
  uint32_t tr_lo[DT], tr_hi[DT], kk_off[KC];
#pragma unroll
  for (int dt = 0; dt < DT; dt++) {
    tr_lo[dt] = lds_addr(lds_kv[b_v]) + TB + tile_off<D>(4 * g + tr_row, 4 * dt + (tr_col >> 3)) + (tr_col & 4) * 2;
    tr_hi[dt] = lds_addr(lds_kv[b_v]) + TB + tile_off<D>(4 * g + tr_row + 8, 4 * dt + (tr_col >> 3)) + (tr_col & 4) * 2;
  }
#pragma unroll
  for (int kc = 0; kc < KC; kc++) kk_off[kc] = lds_addr(lds_kv[b_k]) + tile_off<D>(l32, 2 * kc + g);
  __syncthreads();

  ItemStream items;
  if (tid == 0) { items.init(a.counter, a.begin); items.request(); s_item = items.resolve(); }
  __syncthreads();
  for (;;) {
    const int item_idx = __builtin_amdgcn_readfirstlane(s_item);   // uniform: tables are read with scalar loads
    if (item_idx < 0) break;
    if (tid == 0) items.request();      // the item after this one
    const QItem it = a.items[item_idx];
    // selects, not it.q_rows[sub]: a run-time index would put the whole item into private memory
    const int q_rows = (sub ? it.q_rows[1] : it.q_rows[0]), tile_off_q = (sub ? it.tile_off[1] : it.tile_off[0]), head = (sub ? it.head[1] : it.head[0]);
    const int kvh = it.head[0] / group;
    const int my_row = wq * 32 + l32;                        // row inside the sub-tile
    const bool row_ok = my_row < q_rows;
    const int wave_row_lo = tile_off_q + wq * 32;            // rows of this wave inside the block
    const int my_limit = tile_off_q + my_row;                // last visible column of a DIAG pair for this lane
    const uint16_t* kbase = a.k + (int64_t)kvh * D;
    const uint16_t* vbase = a.v + (int64_t)kvh * D;
    // packed block: the columns this lane's row may see, parked in LDS until a tile is masked (rows past the end: none)
    if constexpr (PACKED) {
      if (it.col_end > 0) s_seg[tid] = row_ok ? a.q_seg[(sub ? it.q_start[1] : it.q_start[0]) + my_row] : 0u;
    }

    // Q^T fragments (B operand of S^T = K Q^T): lane = query row, 8 consecutive d per k-chunk.
    bf16x8 qf[KC];
    {
      const uint16_t* qp = a.q + (int64_t)((sub ? it.q_start[1] : it.q_start[0]) + my_row) * q_row_stride + (int64_t)head * D + 8 * g;
#pragma unroll
      for (int kc = 0; kc < KC; kc++) {
        u32x4 v = {0, 0, 0, 0};
        if (row_ok) v = *reinterpret_cast<const u32x4*>(qp + kc * 16);
        qf[kc] = as_bf16x8(v);
      }
    }
    f32x16 o[DT];
#pragma unroll
    for (int dt = 0; dt < DT; dt++)
#pragma unroll
      for (int r = 0; r < 16; r++) o[dt][r] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;

    // number of tiles of the item, and of iterations: tiles + 1 (pipeline fill)
    TileIter ti;                      // names the next tile to LOAD
    ti.init(a.pairs, it);
    const int n_it = 1 + it.n_tiles;

    // The load of one tile in two parts.  describe(): scalar bookkeeping with branches, run at
    // an iteration boundary.  issue(): branch-free, sits between the MFMAs.
    uint64_t d_k = 0, d_v = 0;
    uint32_t d_lim = 0;
    TileMeta d_meta = {0, 0, 0};
    auto describe = [&]() {
      d_k = reinterpret_cast<uint64_t>(zeros); d_v = d_k; d_lim = 0; d_meta = TileMeta{0, 0, 0};
      if (ti.more) {
        const int64_t row0 = (int64_t)(ti.cur.kv_start + ti.c0) * kv_row_stride;
        d_k = reinterpret_cast<uint64_t>(kbase + row0);
        d_v = reinterpret_cast<uint64_t>(vbase + row0);
        const int valid = min(kFwdTileN, ti.cur.kv_len - ti.c0);
        d_lim = (uint32_t)((valid - 1) * kv_row_stride * 2);
        d_meta = TileMeta{ti.c0, ti.cur.kv_len, ti.cur.kind};
        ti.advance();
      }
    };
    auto issue = [&]() {
      const uint32_t lbase = lds_addr(lds_kv[0]) + b_dma * BUF;
#pragma unroll
      for (int n = 0; n < NDMA; n++) {
        const uint32_t voff = min(dma_row[n], d_lim) + dma_chunk[n];
        lds_dma16_s(reinterpret_cast<const unsigned char*>(d_k), voff, lbase + (8 * n + wave) * 1024);
        lds_dma16_s(reinterpret_cast<const unsigned char*>(d_v), voff, lbase + TB + (8 * n + wave) * 1024);
      }
      b_dma = (b_dma == NB - 1) ? 0 : b_dma + 1;
    };
    // prologue: tiles 0 and 1 into the two buffers before the next one to load
    TileMeta meta[3];                 // tiles i+1, i+2, i+3 (shift register)
    b_dma = (b_dma + NB - 2) % NB;
    describe(); issue(); meta[0] = d_meta;
    describe(); issue(); meta[1] = d_meta;
    describe(); meta[2] = d_meta;     // tile 2, requested inside the first iteration
    dma_wait();
    __syncthreads();

    f32x16 s_a[2], s_b[2];            // S^T of the tile being exponentiated / being computed
#pragma unroll
    for (int rt = 0; rt < 2; rt++)
#pragma unroll
      for (int r = 0; r < 16; r++) { s_a[rt][r] = -INFINITY; s_b[rt][r] = 0.f; }

    // One iteration.  sc = scores of tile i (masked, maximum already folded into m_run);
    // sn receives S^T of tile i+1.
    // FIRST: nothing to exponentiate or to add to O yet (S^T of tile 0 only); LAST: no next tile (O += V P of the
    // last tile only).  An item thus costs one iteration's worth of MFMAs per tile and nothing for the pipeline fill.
    auto iteration = [&](auto first_t, auto last_t, f32x16 (&sc)[2], f32x16 (&sn)[2]) {
      constexpr bool FIRST = decltype(first_t)::value, LAST = decltype(last_t)::value;
      const float m_use = (m_run == -INFINITY) ? 0.f : m_run;
      u32x4 pb[4];                    // P^T of tile i as four B operands (rt, j)
      float rs = 0.f;
      float p_prev = 0.f;
      // the exponential of the NEXT element is issued before this one is consumed, so its latency
      // does not sit in a dependent chain (the wave issues in order)
      float p_ahead = 0.f;
      if constexpr (!FIRST) p_ahead = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[0][0], a.scale_log2, -m_use));
      auto expo = [&](int e) {        // element e = (rt, r) of tile i
        const int r = e & 15;
        const float p = p_ahead;
        if (e + 1 < 32) p_ahead = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[(e + 1) >> 4][(e + 1) & 15], a.scale_log2, -m_use));
        rs += p;
        if (r & 1) {
          pb[e >> 3][(e >> 1) & 3] = pack_bf16(p_prev, p);
          // keeps the vector work between the MFMAs it was written between
          asm volatile("" :: "v"(pb[e >> 3][(e >> 1) & 3]));
        } else p_prev = p;
      };
      // ---- phase 1: S^T(i+1) = K Q^T (two 32-row halves); exponentials of tile i between the MFMAs
      if constexpr (LAST) {
        issue();
#pragma unroll
        for (int e = 0; e < 24; e++) expo(e);
      } else {
        u32x4 op[PF];
#pragma unroll
        for (int u = 0; u < PF; u++) op[u] = lds_read16(kk_off[u / 2] + (u & 1) * 32 * (D * 2));
#pragma unroll
        for (int u = 0; u < NS1; u++) {
          const int kc = u / 2, rt = u & 1;
          if (kc == 0) {
#pragma unroll
            for (int r = 0; r < 16; r++) sn[rt][r] = 0.f;
          }
          sn[rt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(op[u % PF]), qf[kc], sn[rt], 0, 0, 0);
          if (u + PF < NS1) op[u % PF] = lds_read16(kk_off[(u + PF) / 2] + ((u + PF) & 1) * 32 * (D * 2));
          // 24 of the 32 elements in this phase
          if constexpr (!FIRST) {
#pragma unroll
            for (int e = u * 24 / NS1; e < (u + 1) * 24 / NS1; e++) expo(e);
          }
          if (u == NS1 / 2) issue();
          __builtin_amdgcn_sched_barrier(0);
        }
      }
      // ---- phase 2: O^T += V^T P^T; the rest of the exponentials
      if constexpr (!FIRST) {
        u32x4 op[PF];
        auto fetch = [&](int u) {
          const uint32_t rows = 16 * (u / DT) * (D * 2);
          return __builtin_bit_cast(u32x4, lds_tr_pair_at(tr_lo[u % DT] + rows, tr_hi[u % DT] + rows));
        };
#pragma unroll
        for (int u = 0; u < PF; u++) op[u] = fetch(u);
#pragma unroll
        for (int u = 0; u < NS2; u++) {
          o[u % DT] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(op[u % PF]), as_bf16x8(pb[u / DT]), o[u % DT], 0, 0, 0);
          if (u + PF < NS2) op[u % PF] = fetch(u + PF);
#pragma unroll
          for (int e = 24 + u * 8 / (NS2 / 2); e < 24 + (u + 1) * 8 / (NS2 / 2) && u < NS2 / 2; e++) expo(e);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
      l_run += rs;
      // the tile two ahead has landed once at most one tile's loads are in flight
      __builtin_amdgcn_s_waitcnt(0x0F70 | (DMA_PER_TILE & 15) | ((DMA_PER_TILE >> 4) << 14));
      __syncthreads();
      // ---- mask of tile i+1 (only tiles that touch the diagonal or a ragged end, or lie past the
      // end of the item), then its maximum
      if constexpr (!LAST) {
        const TileMeta tm = meta[0];
        // readfirstlane: the condition is wave-uniform, but the compiler does not know it and would
        // otherwise run the rare path on every tile as 64 compares and selects
        const int need_mask = __builtin_amdgcn_readfirstlane(
            (int)(tm.len == 0 || tm.c0 + kFwdTileN > tm.len || (PACKED && (tm.kind & 2)) || ((tm.kind & 1) && tm.c0 + kFwdTileN - 1 > wave_row_lo)));
        if (need_mask) {
          if (PACKED && __builtin_amdgcn_readfirstlane(tm.kind & 2)) {
            // packed block: the row sees the columns of its own member (up to itself under a causal mask)
            const uint32_t sg = s_seg[tid];
            const int first = (int)(sg & 0xffff) - tm.c0 - 4 * g;
            const int last = ((tm.kind & 1) ? min((int)(sg >> 16) - 1, my_limit) : (int)(sg >> 16) - 1) - tm.c0 - 4 * g;
#pragma unroll
            for (int rt = 0; rt < 2; rt++)
#pragma unroll
              for (int r = 0; r < 16; r++) {
                const int c = rt * 32 + 8 * (r >> 2) + (r & 3);
                if (c > last || c < first) sn[rt][r] = -INFINITY;
              }
          } else {
            // last visible column for this lane, relative to the tile's first column
            const int limit = ((tm.kind & 1) ? min(tm.len - 1, my_limit) : tm.len - 1) - tm.c0 - 4 * g;
#pragma unroll
            for (int rt = 0; rt < 2; rt++)
#pragma unroll
              for (int r = 0; r < 16; r++)
                if (rt * 32 + 8 * (r >> 2) + (r & 3) > limit) sn[rt][r] = -INFINITY;
          }
        }
      }
      if constexpr (!LAST) {
        float mx = fmaxf(sn[0][0], sn[1][0]);
#pragma unroll
        for (int r = 1; r < 16; r++) mx = fmaxf(fmaxf(mx, sn[0][r]), sn[1][r]);
        // ---- online softmax bookkeeping for tile i+1, in the log2 domain.  The reference maximum
        // m_run only moves when some row's maximum exceeds it by more than kRescaleSlack (a
        // wave-uniform decision): any reference gives the same O and LSE as long as exp2 stays in
        // range, and P <= 2^slack is harmless in bf16/fp32.  Most tiles skip the rescaling of O.
        mx = fmaxf(mx, xor32(mx)) * a.scale_log2;
        if (__builtin_amdgcn_ballot_w64(mx > m_run + kRescaleSlack) != 0) {
          const float m_new = fmaxf(m_run, mx);
          const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
          const float alpha = __builtin_amdgcn_exp2f(m_run - m_safe);   // m_run = -inf -> 0
          m_run = m_new;
          l_run *= alpha;
#pragma unroll
          for (int dt = 0; dt < DT; dt++)
#pragma unroll
            for (int r = 0; r < 16; r++) o[dt][r] *= alpha;
        }
      }
      // ---- rotate the ring
      meta[0] = meta[1]; meta[1] = meta[2];
      describe(); meta[2] = d_meta;
      {
        const int sk = (b_k == NB - 1) ? -(NB - 1) * BUF : BUF;
#pragma unroll
        for (int kc = 0; kc < KC; kc++) kk_off[kc] += sk;
        b_k = (b_k == NB - 1) ? 0 : b_k + 1;
        const int sv = (b_v == NB - 1) ? -(NB - 1) * BUF : BUF;
#pragma unroll
        for (int dt = 0; dt < DT; dt++) { tr_lo[dt] += sv; tr_hi[dt] += sv; }
        b_v = (b_v == NB - 1) ? 0 : b_v + 1;
      }
    };
    const std::true_type yes;
    const std::false_type no;
    iteration(yes, no, s_a, s_b);          // S^T of tile 0 (of nothing, masked, for an item without tiles)
    if (n_it >= 2) {
      int rem = n_it - 2;                  // iterations that do both phases; they alternate (s_b, s_a), (s_a, s_b)
      for (; rem >= 2; rem -= 2) {
        iteration(no, no, s_b, s_a);
        iteration(no, no, s_a, s_b);
      }
      if (rem) {
        iteration(no, no, s_b, s_a);       // a tail, not a branch inside the loop (which costs dozens of spills)
      } else {
#pragma unroll
        for (int rt = 0; rt < 2; rt++) s_a[rt] = s_b[rt];
      }
      iteration(no, yes, s_a, s_b);        // O += V P of the last tile
    }
    dma_wait();         // the look-ahead loads past the end of the item (zero tiles)

    // ---- epilogue: normalise, write the partial (fp32) and its LSE
    const float l_tot = l_run + xor32(l_run);
    const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;
    if (row_ok && a.running) {
      // Two-way reduction in place: the running (O, LSE) of this row and head, as the earlier stages left it, and
      // this slot's (o / l_tot, lse_s) combine with weights exp(LSE - m); a running LSE of -inf means "nothing
      // yet" (whatever O holds then is ignored).  One writer per row and launch; stages are ordered by the stream.
      const int64_t row = (int64_t)((sub ? it.q_start[1] : it.q_start[0]) + my_row);
      float* op = reinterpret_cast<float*>(a.o) + row * q_row_stride + (int64_t)head * D;
      float* lp = a.lse + row * a.n_q_heads + head;
      const float lse_s = l_tot > 0.f ? (m_run + __builtin_amdgcn_logf(l_tot)) * kLn2 : -INFINITY;
      const float lse_o = *lp;
      const float m = fmaxf(lse_o, lse_s);
      const float w_o = lse_o == -INFINITY ? 0.f : __expf(lse_o - m);
      const float w_s = lse_s == -INFINITY ? 0.f : __expf(lse_s - m);
      const float tot = w_o + w_s;
      const float c_o = tot > 0.f ? w_o / tot : 0.f, c_s = tot > 0.f ? w_s / tot * inv : 0.f;
#pragma unroll
      for (int dt = 0; dt < DT; dt++)
#pragma unroll
        for (int q4 = 0; q4 < 4; q4++) {
          f32x4* ptr = reinterpret_cast<f32x4*>(op + dt * 32 + 8 * q4 + 4 * g);
          f32x4 old = *ptr;
          if (lse_o == -INFINITY) old = f32x4{0.f, 0.f, 0.f, 0.f};
          const f32x4 cur = {o[dt][4 * q4], o[dt][4 * q4 + 1], o[dt][4 * q4 + 2], o[dt][4 * q4 + 3]};
          *ptr = old * c_o + cur * c_s;
        }
      if (g == 0) *lp = tot > 0.f ? m + __logf(tot) : -INFINITY;
    } else if (row_ok) {
      // the only slot of its query block: this is the final result, not a partial
      const bool to_final = it.to_final != 0;
      const int64_t row = to_final ? (int64_t)((sub ? it.q_start[1] : it.q_start[0]) + my_row) : (int64_t)((sub ? it.out_row[1] : it.out_row[0]) + my_row);
      const int64_t off = row * q_row_stride + (int64_t)head * D;
      if (to_final ? !a.o_is_f32 : a.part_is_bf16) {
        uint16_t* op = reinterpret_cast<uint16_t*>(to_final ? a.o : a.o_part) + off;
#pragma unroll
        for (int dt = 0; dt < DT; dt++) store_tile_bf16(op + dt * 32, o[dt], inv, g);
      } else {
        float* op = reinterpret_cast<float*>(to_final ? a.o : a.o_part) + off;
#pragma unroll
        for (int dt = 0; dt < DT; dt++)
#pragma unroll
          for (int q4 = 0; q4 < 4; q4++) {
            f32x4 w = {o[dt][4 * q4] * inv, o[dt][4 * q4 + 1] * inv, o[dt][4 * q4 + 2] * inv, o[dt][4 * q4 + 3] * inv};
            *reinterpret_cast<f32x4*>(op + dt * 32 + 8 * q4 + 4 * g) = w;
          }
      }
      if (g == 0) {
        const float lse = l_tot > 0.f ? (m_run + __builtin_amdgcn_logf(l_tot)) * kLn2 : -INFINITY;
        (to_final ? a.lse : a.lse_part)[row * a.n_q_heads + head] = lse;
      }
    }
    __syncthreads();   // every wave has read s_item
    if (tid == 0) s_item = items.resolve();
    __syncthreads();
  }
  if (tid == 0) retire(a.counter, a.done);
}

// =====================================================================================
// Merge: LSE-weighted reduction of the partials of each query block.  HBM-bound.
// One group of D/4 lanes owns one (row, head) entry: a float4 of the head vector per lane.
// =====================================================================================
struct MergeArgs {
  const void* o_part; const float* lse_part; void* o; float* lse;
  const MergeItem* items; const int32_t* slot_rh;
  int32_t o_is_f32, part_is_bf16;
};

template <int D>
__global__ void __launch_bounds__(256) merge_kernel(MergeArgs a) {
  constexpr int LPE = D / 4;            // lanes per entry
  constexpr int EPP = 256 / LPE;        // entries per pass
  constexpr int U = 4;                  // entries per thread and step (independent loads; 2, 6 and 8 measured slower)
  constexpr int STEP = EPP * U;         // entries the workgroup handles per step
  const MergeItem it = a.items[blockIdx.x];
  const int sub = threadIdx.x / LPE, ln = threadIdx.x % LPE;
  // The item is one stream of steps (chunk of STEP entries, slot), slots innermost; the loads of a step are issued two
  // steps before they are used, across chunk boundaries too, so that a query block with few partials keeps as many
  // bytes in flight as one with many.  acc and tot are kept relative to a running maximum (the online-softmax
  // recurrence) and rescaled when a larger LSE arrives.
  const int n_chunks = (it.n_rh + STEP - 1) / STEP;
  const int ns = max(it.n_slots, 1);    // a query block without any partial still gets O = 0, LSE = -inf: one empty step per chunk
  const int n_steps = n_chunks * ns;
  struct Buf { float l[U]; f32x4 x[U]; };
  auto load = [&](int t, Buf& bf) {
#pragma unroll
    for (int u = 0; u < U; u++) { bf.l[u] = -INFINITY; bf.x[u] = f32x4{0.f, 0.f, 0.f, 0.f}; }
    if (t >= n_steps || it.n_slots == 0) return;
    const int c = t / ns, s = t - c * ns;
    const int e0 = c * STEP + sub;
    const int64_t base = (int64_t)a.slot_rh[it.slot_begin + s] + it.rh_off + e0;
#pragma unroll
    for (int u = 0; u < U; u++) {
      if (e0 + u * EPP < it.n_rh) {
        bf.l[u] = a.lse_part[base + u * EPP];
        if (a.part_is_bf16) {
          const u32x2 h = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(reinterpret_cast<const uint16_t*>(a.o_part) + (base + u * EPP) * D + ln * 4));
          bf.x[u] = f32x4{__builtin_bit_cast(float, h[0] << 16), __builtin_bit_cast(float, h[0] & 0xffff0000u),
                          __builtin_bit_cast(float, h[1] << 16), __builtin_bit_cast(float, h[1] & 0xffff0000u)};
        } else {
          bf.x[u] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(reinterpret_cast<const float*>(a.o_part) + (base + u * EPP) * D + ln * 4));
        }
      }
    }
  };
  float mx[U], tot[U];
  f32x4 acc[U];
  int s_in_chunk = 0, chunk = 0;
  auto fold = [&](const Buf& bf) {
    if (s_in_chunk == 0) {
#pragma unroll
      for (int u = 0; u < U; u++) { mx[u] = -INFINITY; tot[u] = 0.f; acc[u] = f32x4{0.f, 0.f, 0.f, 0.f}; }
    }
#pragma unroll
    for (int u = 0; u < U; u++) {
      // an empty partial (LSE = -inf) carries weight 0; its payload must not leak through (0 * NaN)
      if (bf.l[u] != -INFINITY) {
        const float m_new = fmaxf(mx[u], bf.l[u]);
        const float keep = __expf(mx[u] - m_new);        // mx = -inf -> 0
        const float w = __expf(bf.l[u] - m_new);
        tot[u] = tot[u] * keep + w;
        acc[u] = acc[u] * keep + w * bf.x[u];
        mx[u] = m_new;
      }
    }
    if (++s_in_chunk == ns) {
      const int e0 = chunk * STEP + sub;
#pragma unroll
      for (int u = 0; u < U; u++) {
        if (e0 + u * EPP >= it.n_rh) continue;
        const float inv = tot[u] > 0.f ? 1.0f / tot[u] : 0.f;
        const f32x4 r = acc[u] * inv;
        const int64_t out = (int64_t)it.out_rh + e0 + u * EPP;
        if (a.o_is_f32) {
          __builtin_nontemporal_store(r, reinterpret_cast<f32x4*>(reinterpret_cast<float*>(a.o) + out * D + ln * 4));
        } else {
          u32x2 h = {pack_bf16(r[0], r[1]), pack_bf16(r[2], r[3])};
          __builtin_nontemporal_store(h, reinterpret_cast<u32x2*>(reinterpret_cast<uint16_t*>(a.o) + out * D + ln * 4));
        }
        if (ln == 0) a.lse[out] = tot[u] > 0.f ? mx[u] + __logf(tot[u]) : -INFINITY;
      }
      s_in_chunk = 0; chunk++;
    }
  };
  constexpr int NBUF = 3;               // two steps in flight + the one being folded (three in flight: no faster)
  Buf b[NBUF];
#pragma unroll
  for (int k = 0; k < NBUF - 1; k++) load(k, b[k]);
  for (int t = 0; t < n_steps; t += NBUF) {
#pragma unroll
    for (int k = 0; k < NBUF; k++) {
      if (t + k < n_steps) {
        load(t + k + NBUF - 1, b[(k + NBUF - 1) % NBUF]);
        fold(b[k]);
      }
    }
  }
}

// =====================================================================================
// Backward preprocess: D[t,h] = sum_c dO[t,h,c] * O[t,h,c].  HBM-bound.
// Emits what the two backward kernels consume, head-major [Hq][T_q] so that 32 consecutive
// query rows of one head are one 128-byte line:  dls = scale * D  and  lse2 = log2(e) * LSE,
// with +inf in place of an LSE of -inf (a row that saw no key has P = 0 and no gradient).
// One workgroup handles 16 tokens x all heads; results pass through LDS for the transposition.
// =====================================================================================
constexpr int kDeltaTok = 16;       // tokens per workgroup
constexpr int kDeltaHeads = 128;    // heads per pass through LDS

template <int D>
__global__ void __launch_bounds__(256) delta_kernel(const void* o, int o_is_f32, const uint16_t* d_o, const float* lse,
                                                    float* dls, float* lse2, int64_t t_q, int n_heads, float scale) {
  constexpr int LPE = D / 8;      // lanes per (token, head) entry, 8 elements each
  constexpr int EPP = 256 / LPE;  // entries per pass
  __shared__ float sm_d[kDeltaHeads][kDeltaTok + 1];
  __shared__ float sm_l[kDeltaHeads][kDeltaTok + 1];
  const int64_t t0 = (int64_t)blockIdx.x * kDeltaTok;
  const int n_tok = (int)min((int64_t)kDeltaTok, t_q - t0);
  const int sub = threadIdx.x / LPE, ln = threadIdx.x % LPE;
  for (int h0 = 0; h0 < n_heads; h0 += kDeltaHeads) {
    const int nh = min(kDeltaHeads, n_heads - h0);
    for (int e0 = 0; e0 < n_tok * nh; e0 += EPP) {
      const int el = e0 + sub;                 // entry inside the (token, head chunk) tile
      float acc = 0.f;
      const bool ok = el < n_tok * nh;
      const int tt = ok ? el / nh : 0, hh = ok ? el % nh : 0;
      const int64_t e = (t0 + tt) * n_heads + h0 + hh;
      if (ok) {
        const u32x4 dv = *reinterpret_cast<const u32x4*>(d_o + e * D + ln * 8);
        float ov[8];
        if (o_is_f32) {
          const f32x4 x0 = *reinterpret_cast<const f32x4*>(reinterpret_cast<const float*>(o) + e * D + ln * 8);
          const f32x4 x1 = *reinterpret_cast<const f32x4*>(reinterpret_cast<const float*>(o) + e * D + ln * 8 + 4);
          for (int i = 0; i < 4; i++) { ov[i] = x0[i]; ov[4 + i] = x1[i]; }
        } else {
          const u32x4 x = *reinterpret_cast<const u32x4*>(reinterpret_cast<const uint16_t*>(o) + e * D + ln * 8);
          for (int i = 0; i < 4; i++) {
            ov[2 * i] = __uint_as_float(x[i] << 16);
            ov[2 * i + 1] = __uint_as_float(x[i] & 0xffff0000u);
          }
        }
        for (int i = 0; i < 4; i++) {
          acc += __uint_as_float(dv[i] << 16) * ov[2 * i];
          acc += __uint_as_float(dv[i] & 0xffff0000u) * ov[2 * i + 1];
        }
      }
      for (int off = LPE / 2; off > 0; off >>= 1) acc += __shfl_xor(acc, off, 64);
      if (ok && ln == 0) {
        const float l = lse[e];
        sm_d[hh][tt] = acc * scale;
        sm_l[hh][tt] = (l == -INFINITY) ? INFINITY : l * kLog2e;
      }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < nh * kDeltaTok; i += 256) {
      const int hh = i / kDeltaTok, tt = i % kDeltaTok;
      if (tt < n_tok) {
        const int64_t dst = (int64_t)(h0 + hh) * t_q + t0 + tt;
        dls[dst] = sm_d[hh][tt];
        lse2[dst] = sm_l[hh][tt];
      }
    }
    __syncthreads();
  }
}

// =====================================================================================
// Backward, part 1 -- dK and dV.  Item = (KV tile of 128 rows, KV head); workgroup of 8 waves, two
// per SIMD: four producers and four consumers.  A step is 32 query rows of one head:
//   producer s, KV rows 32*s .. +32 of the tile:
//             A(t): S = Q K^T, dP = dO V^T      (A operands: row-wise reads of the Q / dO tiles in
//                                                LDS; B operands: the wave's K / V rows in registers)
//             B(t): P = exp2(S*c - LSE*log2e), masked on the diagonal; dS = P o (dP*scale - D*scale);
//                   P and dS go to the consumers as bf16 MFMA B operands through LDS
//   consumer c, d rows 32*c .. +32 of dK^T / dV^T for all 128 KV rows (d = 64: 32 d rows x 64 KV rows):
//             C(t): dV^T += dO^T P, dK^T += Q^T dS   (A operands: transpose reads of its d rows of the
//                   same tiles, each used for every 32-row KV group; B operands: every producer's P / dS)
// dK^T / dV^T (rows = d, cols = KV rows) stay in the consumers' accumulators across every dependent
// query block and the G query heads of the group, so each dK / dV element has exactly one writer.
// The roles are decoupled by whole steps: in one barrier interval the consumer runs C(t) while
// the producer issues the MFMAs of A(t+2) with the vector work B(t+1) interleaved between them by
// hand.  The vector ALU work of the SIMD thus sits in one wave and half of its MFMAs in the
// other, and neither wave waits for the other inside an interval.  Q / dO tiles and the per-row
// scalars sit in a ring of seven LDS buffers filled by LDS-DMA (issued by the consumers) six
// steps ahead of their C phase; a tile is in place two intervals before the producer reads it,
// so the producer requests its first LDS operands of an interval, and the consumer all its A
// operands, before the barrier that opens it.
// One workgroup barrier per step.  Steps before the first and past the last of an item run on
// +inf LSE (P = dS = 0), which keeps the instruction stream and the count of loads in flight
// identical for every step; the ring runs on from item to item.
// LDS time per step and SIMD pair: 16 row reads + 8 scalar reads + 16 hand-over reads (b128,
// 256 B/clk), 8 transpose reads (b64, 160 B/clk), the 8 KB hand-over and the 4 KB of DMA writes
// (writes: 76 B/clk), about 1.15x the 1024 cycles of the 32 MFMAs (rates measured on this chip).
// dQ is not produced here: accumulating it across KV tiles needs fp32 atomics, and the chip
// sustains only about 1.35 TB/s of them (measured), several times below what this kernel would
// emit.  dq_kernel below recomputes S and dP query-stationary instead.
// =====================================================================================
struct BwdArgs {
  const uint16_t* q; const uint16_t* k; const uint16_t* v; const uint16_t* d_o;
  const float* lse2; const float* dls;     // head-major [Hq][T_q]: LSE*log2(e) (+inf for empty rows), D*scale
  // dq_kernel<D, true, *> computes those two itself from O, LSE and dO and writes them for dkdv_kernel
  const void* o; const float* lse; int32_t o_is_f32; float* lse2_out; float* dls_out;
  void* dq; void* dk; void* dv;    // fp32, or bf16 in the GRAD_BF16 instances of the kernels
  unsigned char* ds;               // dS spill buffer (2 KB fragments), or NULL
  WsHeader* hdr; const DevPair* pairs; const BwdDep* deps; const BwdItem* items; const QItem* dq_items;
  const uint32_t* q_seg; const uint32_t* kv_seg;   // member bounds per Q-buffer row / KV-buffer row (packed blocks only)
  int64_t t_q;
  int32_t n_q_heads, n_kv_heads;
  float scale, scale_log2;
};

// Iterator over the 32-row query steps of a backward item: rows, then the G query heads of
// the group, then the dependent query blocks.  A DIAG (or PACKED_DIAG) dependency starts at the tile's own rows.
struct StepIter {
  const BwdDep* deps;
  int dep, n_deps, hh, group, q0, first_diag, q_stop;   // q_stop: first row past the rows to walk in the current dependency
  BwdDep cur;
  bool more;
  __device__ __forceinline__ int first_q0() const { return (cur.kind & 1) ? first_diag : 0; }
  // packed_q_end: of an item of a packed block (whose one dependency is walked up to that row only), else 0
  __device__ __forceinline__ void init(const BwdDep* d, int n, int group_, int tile_off, int packed_q_end) {
    deps = d; dep = 0; n_deps = n; hh = 0; group = group_; first_diag = tile_off & ~31; q0 = 0; q_stop = 0;
    cur = BwdDep{0, 0, 0, 0};
    more = n > 0;
    if (more) {
      cur = deps[0]; q0 = first_q0();
      q_stop = packed_q_end > 0 ? packed_q_end : cur.q_len;
      more = q0 < q_stop;
    }
  }
  __device__ __forceinline__ void advance() {
    q0 += 32;
    if (q0 >= q_stop) {
      hh++;
      if (hh < group) {
        q0 = first_q0();
      } else {
        hh = 0;
        dep++;
        if (dep < n_deps) { cur = deps[dep]; q0 = first_q0(); q_stop = cur.q_len; } else { more = false; }
      }
    }
  }
};

constexpr int kDkdvBufs = 7;        // ring of LDS step buffers
constexpr int kNoMask = 1 << 30;    // diagonal threshold of a step that needs no mask

template <int D, bool GRAD_BF16, bool SPILL>
__global__ void __launch_bounds__(512, 2) dkdv_kernel(BwdArgs a) {
  constexpr int KC = D / 16;
  constexpr int DT = D / 32;
  constexpr int NS = 2 * KC;                 // MFMAs per wave and step (= 4 * DT)
  constexpr int PFC = 4;                     // consumer: an LDS operand is requested this many MFMAs before its use
  constexpr int PFP = 4;                     // producer
  constexpr int TB = tile_bytes<D>(32);
  constexpr int BUF = 2 * TB;                // [Q tile | dO tile]
  constexpr int NB = kDkdvBufs;
  constexpr int CPR = D / 8, RPI = 64 / CPR, NDMA = 32 / RPI / 4;   // LDS-DMA geometry, see issue()
  constexpr int DMA_PER_STEP = 2 * NDMA + 1;                        // instructions per consumer wave and step
  __shared__ __attribute__((aligned(1024))) unsigned char lds_t[NB][BUF];
  __shared__ __attribute__((aligned(1024))) unsigned char lds_h[2][4][4096];   // [parity][KV sub-tile][operand][lane] 16 B
  __shared__ __attribute__((aligned(256))) float lds_sc[NB][64];   // [LSE*log2e x 32 | D*scale x 32]
  __shared__ int s_khi[256];        // packed block: first query row past the member of each producer lane's KV row, minus 4g
  __shared__ int s_item;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform, kept in a scalar register
  const int sub = wave & 3;
  const bool consumer = wave >= 4;
  const int l32 = lane & 31, g = lane >> 5;
  const int group = a.n_q_heads / a.n_kv_heads;
  const int64_t q_row_stride = (int64_t)a.n_q_heads * D;
  const int64_t kv_row_stride = (int64_t)a.n_kv_heads * D;
  const unsigned char* zeros = reinterpret_cast<const unsigned char*>(a.hdr->zeros);
  const float* infs = a.hdr->infs;
  const uint32_t lds_sc0 = lds_addr(lds_sc[0]);
  const uint32_t lds_h0 = lds_addr(lds_h[0][sub]) + lane * 16;

  // Zero the tile ring and the hand-over buffers, +inf / 0 into the scalars: the steps before the
  // first one of the first item then contribute nothing.
  for (int i = tid * 16; i < NB * BUF; i += 512 * 16)
    *reinterpret_cast<u32x4*>(&lds_t[0][0] + i) = u32x4{0, 0, 0, 0};
  for (int i = tid * 16; i < 2 * 4 * 4096; i += 512 * 16)
    *reinterpret_cast<u32x4*>(&lds_h[0][0][0] + i) = u32x4{0, 0, 0, 0};
  for (int i = tid; i < NB * 64; i += 512) lds_sc[0][i] = (i & 32) ? 0.f : INFINITY;
  // Ring positions, advanced by one buffer per step and kept across items.  In interval i the
  // consumer transposes tile i (b_c), the producer reads the rows of tile i+2 and the scalars of
  // step i+1 (b_p, b_s), and the consumers request tile i+6 (b_dma).  A tile is in place (landed
  // and published by a barrier) two intervals before the producer's interval, so both roles can
  // request their first LDS operands of an interval before the barrier that opens it.
  int b_c = NB - 2, b_p = 0, b_s = NB - 1, b_dma = 4, hb = 0;
  __syncthreads();

  for (;;) {
    if (tid == 0) s_item = pop_item(a.hdr->bwd_counter, a.hdr->bwd_begin);
    __syncthreads();
    const int item_idx = __builtin_amdgcn_readfirstlane(s_item);   // uniform: tables are read with scalar loads
    if (item_idx < 0) break;
    const BwdItem it = a.items[item_idx];
    const int my_kv = sub * 32 + l32;                  // KV row inside the tile
    const bool kv_ok = my_kv < it.kv_rows;
    int n_iv = 2;       // barrier intervals of the item: its steps plus two of pipeline fill, rounded up to even
    for (int d = 0; d < it.n_deps; d++) {
      const BwdDep dd = a.deps[it.dep_begin + d];
      const int first = (dd.kind & 1) ? (it.tile_off & ~31) : 0;
      const int stop = it.packed ? it.q_end : dd.q_len;
      n_iv += group * (max(0, stop - first + 31) / 32);
    }
    n_iv = (n_iv + 1) & ~1;
    StepIter si;
    si.init(a.deps + it.dep_begin, it.n_deps, group, it.tile_off, it.packed ? it.q_end : 0);

    if (consumer) {
      // =============================== consumer ===============================
      const int cw = sub;     // index among the four loading waves
      // LDS-DMA of a 32-row tile: instruction n of this wave fills LDS rows r_n = (4n + cw) * RPI + lane / CPR.
      // A lane fetches chunk (pc ^ swz(r_n)) of global row min(r_n, valid - 1): rows past a ragged end
      // repeat the last valid row (finite values; their P is 0 because their LSE is +inf).
      uint32_t dma_row[NDMA], dma_chunk[NDMA];
#pragma unroll
      for (int n = 0; n < NDMA; n++) {
        const int r = (4 * n + cw) * RPI + lane / CPR, pc = lane % CPR;
        dma_row[n] = (uint32_t)(r * q_row_stride * 2);
        dma_chunk[n] = (uint32_t)((pc ^ swz<D>(r)) << 4);
      }
      // scalars: lanes 0-31 fetch LSE*log2e of row lane, lanes 32-63 D*scale of row lane-32
      const float* sc_arr = (g ? a.dls : a.lse2) + l32;
      const float* sc_page = (g ? reinterpret_cast<const float*>(zeros) : infs) + l32;
      const int tr_row = (lane & 15) >> 2, tr_col = 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
      // This wave owns d rows 32*cdt .. +31 of dK^T / dV^T for NN of the tile's 32-row KV groups.
      constexpr int NN = DT;
      const int cdt = sub % DT, n0 = (sub / DT) * NN;
      uint32_t tr_lo1 = lds_addr(lds_t[0]) + b_c * BUF + tile_off<D>(4 * g + tr_row, 4 * cdt + (tr_col >> 3)) + (tr_col & 4) * 2;
      uint32_t tr_hi1 = lds_addr(lds_t[0]) + b_c * BUF + tile_off<D>(4 * g + tr_row + 8, 4 * cdt + (tr_col >> 3)) + (tr_col & 4) * 2;
      const uint32_t hsrc = lds_addr(lds_h[0][0]) + n0 * 4096 + lane * 16;
      f32x16 acc_k[DT], acc_v[DT];     // dK^T, dV^T: rows = d, cols = KV rows
#pragma unroll
      for (int dt = 0; dt < DT; dt++)
#pragma unroll
        for (int r = 0; r < 16; r++) { acc_k[dt][r] = 0.f; acc_v[dt][r] = 0.f; }

      // The load of one step in two parts.  describe(): scalar bookkeeping with branches, run at a
      // step boundary.  issue(): branch-free, sits between the MFMAs of the step.
      uint64_t d_q = 0, d_do = 0;          // tile sources (row q0 of the head)
      uint32_t d_lim = 0;                  // byte offset of the last valid row
      int d_valid = 0;
      int64_t d_sc = 0;                    // element offset of the step's first row in the head-major scalars
      const uint32_t row_bytes = (uint32_t)(q_row_stride * 2);
      int run_dep = -1, run_hh = -1;       // the run (dependency, head) of the step described last
      auto describe = [&]() {
        if (!si.more) {
          d_q = reinterpret_cast<uint64_t>(zeros); d_do = d_q; d_lim = 0; d_valid = 0; d_sc = 0;
          run_dep = -1;
          return;
        }
        if (si.dep == run_dep && si.hh == run_hh) {
          // the next 32 rows of the same run: advance the pointers instead of recomputing them
          d_q += 32 * (uint64_t)row_bytes; d_do += 32 * (uint64_t)row_bytes; d_sc += 32;
        } else {
          const int head = it.kv_head * group + si.hh;
          const int64_t row = (int64_t)(si.cur.q_start + si.q0);
          d_q = reinterpret_cast<uint64_t>(a.q + row * q_row_stride + (int64_t)head * D);
          d_do = reinterpret_cast<uint64_t>(a.d_o + row * q_row_stride + (int64_t)head * D);
          d_sc = (int64_t)head * a.t_q + row;
          run_dep = si.dep; run_hh = si.hh;
        }
        d_valid = min(32, si.cur.q_len - si.q0);
        d_lim = (uint32_t)(d_valid - 1) * row_bytes;
        si.advance();
      };
      auto issue = [&]() {
        const uint32_t lbase = lds_addr(lds_t[0]) + b_dma * BUF;
#pragma unroll
        for (int n = 0; n < NDMA; n++) {
          const uint32_t voff = min(dma_row[n], d_lim) + dma_chunk[n];
          lds_dma16_s(reinterpret_cast<const unsigned char*>(d_q), voff, lbase + (4 * n + cw) * 1024);
          lds_dma16_s(reinterpret_cast<const unsigned char*>(d_do), voff, lbase + TB + (4 * n + cw) * 1024);
        }
        // all four loading waves fetch the 64 scalars (same values, same place): they then have
        // the same number of loads in flight
        const float* sp = (l32 < d_valid) ? sc_arr + d_sc : sc_page;
        lds_dma4(sp, lds_sc0 + b_dma * 256);
        b_dma = (b_dma == NB - 1) ? 0 : b_dma + 1;
      };
      // prologue: tiles 0 .. 3 into the four buffers before the next one to load
      b_dma = (b_dma + NB - 4) % NB;
#pragma unroll
      for (int i = 0; i < 4; i++) { describe(); issue(); }
      describe();          // tile 4, requested inside the first interval
      dma_wait();
      __syncthreads();
      // A operands of a step: (k-chunk j of 16 query rows, w = 0: dO^T for dV, 1: Q^T for dK), index 2j + w.
      // Each serves the NN MFMAs of its KV groups; the B operands (P / dS of every group) stream from the
      // hand-over buffers, PFC MFMAs ahead.  While interval i runs, the A operands of step i+1 are fetched
      // from the next tile as soon as their registers are free.
      auto fetch_a = [&](int jw) {
        const uint32_t o = 16 * (jw >> 1) * (D * 2) + ((jw & 1) == 0 ? TB : 0);
        return __builtin_bit_cast(u32x4, lds_tr_pair_at(tr_lo1 + o, tr_hi1 + o));
      };
      auto next_tile = [&]() {
        const int st = (b_c == NB - 1) ? -(NB - 1) * BUF : BUF;
        tr_lo1 += st; tr_hi1 += st;
        b_c = (b_c == NB - 1) ? 0 : b_c + 1;
      };
      u32x4 aop[4];
#pragma unroll
      for (int jw = 0; jw < 4; jw++) aop[jw] = fetch_a(jw);
      next_tile();
      for (int iv = 0; iv < n_iv; iv++) {
        const uint32_t hb_src = hsrc + hb * (4 * 4096);
        // MFMA u = (2j + w) * NN + n reads operand (w ? 2 : 0) + j of KV group n0 + n
        auto fetch_b = [&](int u) {
          const int jw = u / NN, n = u % NN;
          return lds_read16(hb_src + n * 4096 + (((jw & 1) ? 2 : 0) + (jw >> 1)) * 1024);
        };
        u32x4 bop[PFC];
#pragma unroll
        for (int u = 0; u < PFC; u++) bop[u] = fetch_b(u);
#pragma unroll
        for (int u = 0; u < NS; u++) {
          const int jw = u / NN, n = u % NN;
          if ((jw & 1) == 0) acc_v[n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(aop[jw]), as_bf16x8(bop[u % PFC]), acc_v[n], 0, 0, 0);
          else acc_k[n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(aop[jw]), as_bf16x8(bop[u % PFC]), acc_k[n], 0, 0, 0);
          if (u + PFC < NS) bop[u % PFC] = fetch_b(u + PFC);
          if (n == NN - 1) aop[jw] = fetch_a(jw);
          if (u == NS / 2) issue();
          __builtin_amdgcn_sched_barrier(0);
        }
        next_tile();
        __builtin_amdgcn_s_waitcnt(0x0F70 | ((2 * DMA_PER_STEP) & 15) | (((2 * DMA_PER_STEP) >> 4) << 14));
        asm volatile("s_barrier" ::: "memory");
        describe();
        hb ^= 1;
      }
      b_c = (b_c == 0) ? NB - 1 : b_c - 1;     // the tile looked ahead to belongs to the next item's first interval
      dma_wait();
      // ---- epilogue: the only writer of these dK / dV elements
#pragma unroll
      for (int n = 0; n < NN; n++) {
        const int kv_r = (n0 + n) * 32 + l32;
        if (kv_r < it.kv_rows) {
          const int64_t off = (int64_t)(it.kv_start + kv_r) * kv_row_stride + (int64_t)it.kv_head * D + cdt * 32;
          if constexpr (GRAD_BF16) {
            store_tile_bf16(reinterpret_cast<uint16_t*>(a.dk) + off, acc_k[n], 1.0f, g);
            store_tile_bf16(reinterpret_cast<uint16_t*>(a.dv) + off, acc_v[n], 1.0f, g);
          } else {
#pragma unroll
            for (int q4 = 0; q4 < 4; q4++) {
              f32x4 wk = {acc_k[n][4 * q4], acc_k[n][4 * q4 + 1], acc_k[n][4 * q4 + 2], acc_k[n][4 * q4 + 3]};
              f32x4 wv = {acc_v[n][4 * q4], acc_v[n][4 * q4 + 1], acc_v[n][4 * q4 + 2], acc_v[n][4 * q4 + 3]};
              *reinterpret_cast<f32x4*>(reinterpret_cast<float*>(a.dk) + off + 8 * q4 + 4 * g) = wk;
              *reinterpret_cast<f32x4*>(reinterpret_cast<float*>(a.dv) + off + 8 * q4 + 4 * g) = wv;
            }
          }
        }
      }
    } else {
      // =============================== producer ===============================
      int kvg = it.tile_off + my_kv - 4 * g;       // masked iff kvg > q0 + 8*(r/4) + r%4 on a DIAG step
      if (it.packed) {
        // Packed block: a KV row is seen by the query rows of its own member only, [first, last + 1) inside the
        // block: kvg becomes that first row under a full mask (under a causal one it is the row itself, as
        // above), and the bound past the last row waits in LDS for the masked intervals.
        const uint32_t sg = kv_ok ? a.kv_seg[it.kv_start + my_kv] : 0u;
        if (!(it.packed & 1)) kvg = (int)(sg & 0xffff) - 4 * g;
        s_khi[tid] = (int)(sg >> 16) - 4 * g;
      }
      // SPILL: the dS this wave forms also goes to memory, one 2 KB fragment per step, for the dQ pass.  There a
      // KV row past the ragged end of the tile must carry dS = 0 (here its column of dK^T / dV^T is simply never
      // stored): such lanes get a threshold nothing passes, and a ragged tile runs every step through the masked
      // variant.  Fragment layout, shared with dq_ds_kernel: the 16 bytes that lane (KV row r = lane % 32,
      // g = lane / 32) holds for j = 0, 1 (query rows 16j + 4g + {0..3} and 16j + 8 + 4g + {0..3} of the step)
      // sit at byte 1024 j + 512 g + 16 ((r + 8 j + 4 g) % 32): every store instruction writes 1 KB of consecutive
      // memory, and the rotation makes the transposing LDS reads of the dQ pass bank-conflict free.
      if constexpr (SPILL) { if (!kv_ok) kvg = 0x7fff0000; }
      const int thr_none = (SPILL && it.kv_rows < kBwdTileN) ? kNoMask - 1 : kNoMask;
      const int nkv32 = (it.kv_blk_len + 31) >> 5, my_kv32 = (it.tile_off >> 5) + sub;
      const int sink = (int)(blockIdx.x & (kDsSinkFrags - 1));
      int frag_t = sink;         // fragment of the step that B handles in this interval
      uint32_t sp_off[2];
#pragma unroll
      for (int j = 0; j < 2; j++) sp_off[j] = 1024 * j + 512 * g + 16 * ((l32 + 8 * j + 4 * g) & 31);
      // B operands of S and dP: this pair's K and V rows; lane = KV row, 8 consecutive d per k-chunk.
      bf16x8 kf[KC], vf[KC];
      {
        const int64_t off = (int64_t)(it.kv_start + my_kv) * kv_row_stride + (int64_t)it.kv_head * D + 8 * g;
#pragma unroll
        for (int kc = 0; kc < KC; kc++) {
          u32x4 zk = {0, 0, 0, 0}, zv = {0, 0, 0, 0};
          if (kv_ok) {
            zk = *reinterpret_cast<const u32x4*>(a.k + off + kc * 16);
            zv = *reinterpret_cast<const u32x4*>(a.v + off + kc * 16);
          }
          kf[kc] = as_bf16x8(zk); vf[kc] = as_bf16x8(zv);
        }
      }
      uint32_t row_a[KC];        // row-read addresses inside the step buffer of tile i+2 (Q tile; dO is +TB)
#pragma unroll
      for (int kc = 0; kc < KC; kc++) row_a[kc] = lds_addr(lds_t[0]) + b_p * BUF + tile_off<D>(l32, 2 * kc + g);
      uint32_t sc_a = lds_sc0 + b_s * 256 + 16 * g;      // scalars of step i+1: rows 8*q4 + 4g .. +3 at +32*q4, D*scale at +128
      int thr_t = thr_none;      // diagonal threshold of the step that B handles in this interval
      f32x16 s_a, dp_a, s_b, dp_b;
#pragma unroll
      for (int r = 0; r < 16; r++) { s_a[r] = 0.f; dp_a[r] = 0.f; s_b[r] = 0.f; dp_b[r] = 0.f; }
      dma_wait();          // K / V fragments
      __syncthreads();     // the prologue's tiles are in place
      // requested before an interval starts: its first PFP row operands and its first four scalars
      u32x4 op[PFP];
#pragma unroll
      for (int k = 0; k < PFP; k++) op[k] = lds_read16(row_a[k / 2] + ((k & 1) ? TB : 0));
      f32x4 lse_n = __builtin_bit_cast(f32x4, lds_read16(sc_a)), dl_n = __builtin_bit_cast(f32x4, lds_read16(sc_a + 128));

      // One interval: MFMAs of A(i+2) into (sn, dpn); B(i+1) on (sc, dpc) between them.
      auto interval = [&](auto masked, f32x16& sc, f32x16& dpc, f32x16& sn, f32x16& dpn) {
        constexpr int MASK = decltype(masked)::value;     // 0: no mask, 1: diagonal / ragged end, 2: packed block
        const int thr_s = __builtin_amdgcn_readfirstlane(thr_t);
        int hlim = 0;                                     // packed: rows 8*(r/4) + r%4 >= hlim of the step are past the member
        if constexpr (MASK == 2) hlim = s_khi[tid] - thr_s;
        f32x4 lse_c = lse_n, dl_c = dl_n;      // scalars of rows 8*q4 + 4g .. +3, one group of four ahead
        uint32_t pk[16];           // [0..7] P pairs, [8..15] dS pairs: four B operands for the consumer
        float p_prev = 0.f, ds_prev = 0.f;
        const uint32_t hdst = lds_h0 + (hb ^ 1) * (4 * 4096);
        unsigned char* fptr = nullptr;
        if constexpr (SPILL) fptr = a.ds + (int64_t)__builtin_amdgcn_readfirstlane(frag_t) * kDsFragBytes;
        float p_ahead = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[0], a.scale_log2, -lse_c[0]));
#pragma unroll
        for (int k = 0; k < NS; k++) {
          const int kc = k / 2;
          if (k == 0) {
#pragma unroll
            for (int r = 0; r < 16; r++) { sn[r] = 0.f; dpn[r] = 0.f; }
          }
          if ((k & 1) == 0) sn = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(op[k % PFP]), kf[kc], sn, 0, 0, 0);
          else dpn = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(op[k % PFP]), vf[kc], dpn, 0, 0, 0);
          if (k == NS - PFP) {
            // the last row operand of this tile has been requested: move on to the next tile
            const int st = (b_p == NB - 1) ? -(NB - 1) * BUF : BUF;
#pragma unroll
            for (int kc2 = 0; kc2 < KC; kc2++) row_a[kc2] += st;
            b_p = (b_p == NB - 1) ? 0 : b_p + 1;
          }
          {
            const int kk = (k + PFP) % NS;
            op[k % PFP] = lds_read16(row_a[kk / 2] + ((kk & 1) ? TB : 0));
          }
          // vector work: 16 / NS score registers per slot
#pragma unroll
          for (int r = k * 16 / NS; r < (k + 1) * 16 / NS; r++) {
            if ((r & 3) == 0) {
              if (r > 0) { lse_c = lse_n; dl_c = dl_n; }
              if (r == 12) {
                // the scalars of the next interval's first four rows
                sc_a += (b_s == NB - 1) ? -(NB - 1) * 256 : 256;
                b_s = (b_s == NB - 1) ? 0 : b_s + 1;
                lse_n = __builtin_bit_cast(f32x4, lds_read16(sc_a));
                dl_n = __builtin_bit_cast(f32x4, lds_read16(sc_a + 128));
              } else {
                lse_n = __builtin_bit_cast(f32x4, lds_read16(sc_a + 32 * ((r >> 2) + 1)));
                dl_n = __builtin_bit_cast(f32x4, lds_read16(sc_a + 32 * ((r >> 2) + 1) + 128));
              }
            }
            // the exponential of the NEXT register is issued before this register is finished, so
            // its latency does not sit in a dependent chain (the wave issues in order)
            float p = p_ahead;
            if (r + 1 < 16) {
              const float lse_q = ((r + 1) & 3) ? lse_c[(r + 1) & 3] : lse_n[0];
              p_ahead = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[r + 1], a.scale_log2, -lse_q));
            }
            const float dl_r = dl_c[r & 3];
            if constexpr (MASK == 1) p = (kvg > thr_s + 8 * (r >> 2) + (r & 3)) ? 0.f : p;
            if constexpr (MASK == 2) p = (kvg > thr_s + 8 * (r >> 2) + (r & 3) || 8 * (r >> 2) + (r & 3) >= hlim) ? 0.f : p;
            const float ds = p * __builtin_fmaf(dpc[r], a.scale, -dl_r);
            if (r & 1) {
              pk[r >> 1] = pack_bf16(p_prev, p); pk[8 + (r >> 1)] = pack_bf16(ds_prev, ds);
              // keeps the vector work between the MFMAs it was written between
              asm volatile("" :: "v"(pk[r >> 1]), "v"(pk[8 + (r >> 1)]));
            } else { p_prev = p; ds_prev = ds; }
            if ((r & 7) == 7) {
              // rows 8*(r/8) .. r done: one P operand and one dS operand (k-chunk r/8)
              const int j = r >> 3;
              const u32x4 wp = {pk[4 * j], pk[4 * j + 1], pk[4 * j + 2], pk[4 * j + 3]};
              const u32x4 wd = {pk[8 + 4 * j], pk[8 + 4 * j + 1], pk[8 + 4 * j + 2], pk[8 + 4 * j + 3]};
              *(__attribute__((address_space(3))) u32x4*)(uintptr_t)(hdst + j * 1024) = wp;
              *(__attribute__((address_space(3))) u32x4*)(uintptr_t)(hdst + (2 + j) * 1024) = wd;
              if constexpr (SPILL) *reinterpret_cast<u32x4*>(fptr + sp_off[j]) = wd;
            }
          }
          __builtin_amdgcn_sched_barrier(0);
        }
        if constexpr (SPILL) {
          // the hand-over writes must have landed; the fragment stores need not (a full fence would wait for them)
          __builtin_amdgcn_s_waitcnt(0xC07F);      // lgkmcnt(0)
          asm volatile("s_barrier" ::: "memory");
        } else {
          __syncthreads();
        }
        // the step that B handles next
        thr_t = thr_none;
        if constexpr (SPILL) frag_t = sink;
        if (si.more) {
          if (si.cur.kind != FCP_KIND_FULL) thr_t = si.q0;
          if constexpr (SPILL) {
            const int q32 = si.q0 >> 5, nq32 = (si.cur.q_len + 31) >> 5;
            const int head = it.kv_head * group + si.hh;
            if (sub * 32 < it.kv_rows) {
              if (si.cur.kind & 1) {
                if (my_kv32 <= q32) frag_t = si.cur.ds_frag + head * (nq32 * (nq32 + 1) / 2) + q32 * (q32 + 1) / 2 + my_kv32;
              } else {
                frag_t = si.cur.ds_frag + (head * nq32 + q32) * nkv32 + my_kv32;
              }
            }
          }
          si.advance();
        }
        hb ^= 1;
      };
      // the first interval handles B(-1) (nothing) and A(0), the second B(0) and A(1), ...
      const std::integral_constant<int, 0> no_mask;
      const std::integral_constant<int, 1> with_mask;
      const std::integral_constant<int, 2> packed_mask;
      if (it.packed) {
        // every step masked by member; outside the item's steps thr_t names no row at all, which masks everything
        for (int iv = 0; iv < n_iv; iv += 2) {
          interval(packed_mask, s_a, dp_a, s_b, dp_b);
          interval(packed_mask, s_b, dp_b, s_a, dp_a);
        }
      } else {
        for (int iv = 0; iv < n_iv; iv += 2) {
          if (thr_t != kNoMask) interval(with_mask, s_a, dp_a, s_b, dp_b); else interval(no_mask, s_a, dp_a, s_b, dp_b);
          if (thr_t != kNoMask) interval(with_mask, s_b, dp_b, s_a, dp_a); else interval(no_mask, s_b, dp_b, s_a, dp_a);
        }
      }
    }
    __syncthreads();
  }
  if (tid == 0) retire(a.hdr->bwd_counter, &a.hdr->bwd_done);
}

// =====================================================================================
// Backward, part 2 -- dQ.  Query-stationary like the forward and with the same item shape (two
// 128-row query sub-tiles that share a KV head, here over all pairs of the query block); 8 waves
// share one double-buffered stream of [K | V] tiles; lane = query row.
//   S^T = K Q^T, dP^T = V dO^T       (A = K / V rows from LDS, B = Q / dO fragments in registers)
//   P^T = exp2(S^T*c - LSE*log2e), dS^T = P^T o (dP^T - D) * scale     (LSE, D per lane)
//   dQ^T += K^T dS^T                 (A = K by transpose reads, B = accumulator registers)
// Columns past the diagonal or past a ragged end get P = 0.  Every dQ row has one writer: plain
// stores, deterministic.
// =====================================================================================
// PACKED: the problem has packed blocks; only that instance carries the per-row member bounds (as in the forward).
// It exists without WITH_D only: on such a problem the launcher runs the stand-alone D pass first.
template <int D, bool WITH_D, bool GRAD_BF16, bool PACKED = false>
__global__ void __launch_bounds__(512, 2) dq_kernel(BwdArgs a) {
  constexpr int KC = D / 16;
  constexpr int DT = D / 32;
  constexpr int TB = tile_bytes<D>(kFwdTileN);
  __shared__ __attribute__((aligned(1024))) unsigned char lds_kv[2][2 * TB];   // [buffer][K tile | V tile]
  __shared__ uint32_t s_seg[512];   // member bounds of each lane's query row in a packed block (written and read by that lane)
  __shared__ int s_item;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform, kept in a scalar register
  const int sub = wave >> 2, wq = wave & 3;                    // sub-item, 32-row group inside it
  const int l32 = lane & 31, g = lane >> 5;
  const int group = a.n_q_heads / a.n_kv_heads;
  const int64_t q_row_stride = (int64_t)a.n_q_heads * D;
  const int64_t kv_row_stride = (int64_t)a.n_kv_heads * D;
  const unsigned char* zeros = reinterpret_cast<const unsigned char*>(a.hdr->zeros);
  const uint32_t dma_off = dma_lane_offset<D>(wave, lane, kv_row_stride);
  const int tr_row = (lane & 15) >> 2, tr_col = 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
  // absolute LDS addresses into the K tile of the CURRENT buffer (V = +TB), switched in place
  uint32_t tr_lo[DT], tr_hi[DT], row_off[KC];
#pragma unroll
  for (int dt = 0; dt < DT; dt++) {
    tr_lo[dt] = lds_addr(lds_kv[0]) + tile_off<D>(4 * g + tr_row, 4 * dt + (tr_col >> 3)) + (tr_col & 4) * 2;
    tr_hi[dt] = lds_addr(lds_kv[0]) + tile_off<D>(4 * g + tr_row + 8, 4 * dt + (tr_col >> 3)) + (tr_col & 4) * 2;
  }
#pragma unroll
  for (int kc = 0; kc < KC; kc++) row_off[kc] = lds_addr(lds_kv[0]) + tile_off<D>(l32, 2 * kc + g);
  int buf = 0;                              // buffer the addresses above point into
  auto switch_buffer = [&]() {
    const int step = buf ? -2 * TB : 2 * TB;
#pragma unroll
    for (int dt = 0; dt < DT; dt++) { tr_lo[dt] += step; tr_hi[dt] += step; }
#pragma unroll
    for (int kc = 0; kc < KC; kc++) row_off[kc] += step;
    buf ^= 1;
  };

  ItemStream items;
  if (tid == 0) { items.init(a.hdr->dq_counter, a.hdr->dq_begin); items.request(); s_item = items.resolve(); }
  __syncthreads();
  for (;;) {
    const int item_idx = __builtin_amdgcn_readfirstlane(s_item);   // uniform: tables are read with scalar loads
    if (item_idx < 0) break;
    if (tid == 0) items.request();      // the item after this one
    const QItem it = a.dq_items[item_idx];
    const int q_start = (sub ? it.q_start[1] : it.q_start[0]), q_rows = (sub ? it.q_rows[1] : it.q_rows[0]), tile_off_q = (sub ? it.tile_off[1] : it.tile_off[0]), head = (sub ? it.head[1] : it.head[0]);
    const int kvh = it.head[0] / group;
    const int my_row = wq * 32 + l32;
    const bool row_ok = my_row < q_rows;
    const int wave_row_lo = tile_off_q + wq * 32;
    const uint16_t* kbase = a.k + (int64_t)kvh * D;
    const uint16_t* vbase = a.v + (int64_t)kvh * D;
    if constexpr (PACKED) {
      if (it.col_end > 0) s_seg[tid] = row_ok ? a.q_seg[q_start + my_row] : 0u;   // packed block: visible columns of the row
    }

    bf16x8 qf[KC], dof[KC];
    float lse_l = INFINITY, dl_l = 0.f;     // rows past the end: P = exp2(-inf) = 0
    {
      const int64_t off = (int64_t)(q_start + my_row) * q_row_stride + (int64_t)head * D + 8 * g;
#pragma unroll
      for (int kc = 0; kc < KC; kc++) {
        u32x4 zq = {0, 0, 0, 0}, zd = {0, 0, 0, 0};
        if (row_ok) {
          zq = *reinterpret_cast<const u32x4*>(a.q + off + kc * 16);
          zd = *reinterpret_cast<const u32x4*>(a.d_o + off + kc * 16);
        }
        qf[kc] = as_bf16x8(zq); dof[kc] = as_bf16x8(zd);
      }
      if constexpr (WITH_D) {
        // D = rowsum(dO o O) of this lane's row: its 8 columns of every k-chunk, plus the partner lane's
        // (lane ^ 32, same row, the other 8).  The backward preprocess pass is then not needed: the two
        // per-row scalars are written here, head-major, for the dK/dV kernel that runs afterwards.
        float part = 0.f;
        if (row_ok) {
          // all loads of the row first, then the arithmetic: one round trip to memory, not one per k-chunk
          auto dot8 = [&](const u32x4 dv, const float (&ov)[8]) {
#pragma unroll
            for (int i = 0; i < 4; i++) {
              part += __uint_as_float(dv[i] << 16) * ov[2 * i];
              part += __uint_as_float(dv[i] & 0xffff0000u) * ov[2 * i + 1];
            }
          };
          if (a.o_is_f32) {
            const float* op = reinterpret_cast<const float*>(a.o) + off;
            f32x4 x[2 * KC];
#pragma unroll
            for (int kc = 0; kc < KC; kc++) {
              x[2 * kc] = *reinterpret_cast<const f32x4*>(op + kc * 16);
              x[2 * kc + 1] = *reinterpret_cast<const f32x4*>(op + kc * 16 + 4);
            }
#pragma unroll
            for (int kc = 0; kc < KC; kc++) {
              const float ov[8] = {x[2 * kc][0], x[2 * kc][1], x[2 * kc][2], x[2 * kc][3], x[2 * kc + 1][0], x[2 * kc + 1][1], x[2 * kc + 1][2], x[2 * kc + 1][3]};
              dot8(__builtin_bit_cast(u32x4, dof[kc]), ov);
            }
          } else {
            const uint16_t* op = reinterpret_cast<const uint16_t*>(a.o) + off;
            u32x4 x[KC];
#pragma unroll
            for (int kc = 0; kc < KC; kc++) x[kc] = *reinterpret_cast<const u32x4*>(op + kc * 16);
#pragma unroll
            for (int kc = 0; kc < KC; kc++) {
              float ov[8];
#pragma unroll
              for (int i = 0; i < 4; i++) { ov[2 * i] = __uint_as_float(x[kc][i] << 16); ov[2 * i + 1] = __uint_as_float(x[kc][i] & 0xffff0000u); }
              dot8(__builtin_bit_cast(u32x4, dof[kc]), ov);
            }
          }
        }
        const float d_row = part + xor32(part);
        if (row_ok) {
          const float l = a.lse[(int64_t)(q_start + my_row) * a.n_q_heads + head];
          lse_l = (l == -INFINITY) ? INFINITY : l * kLog2e;
          dl_l = d_row * a.scale;
          if (g == 0) {
            const int64_t hr = (int64_t)head * a.t_q + q_start + my_row;
            a.lse2_out[hr] = lse_l;
            a.dls_out[hr] = dl_l;
          }
        }
      } else if (row_ok) {
        const int64_t hr = (int64_t)head * a.t_q + q_start + my_row;
        lse_l = a.lse2[hr];
        dl_l = a.dls[hr];
      }
    }
    f32x16 acc[DT];
#pragma unroll
    for (int dt = 0; dt < DT; dt++)
#pragma unroll
      for (int r = 0; r < 16; r++) acc[dt][r] = 0.f;

    TileIter ti;
    ti.init(a.pairs, it);
    auto dma = [&](int b) {
      const int64_t row0 = (int64_t)(ti.cur.kv_start + ti.c0) * kv_row_stride;
      // Only the waves of sub-item 0 load: they reach every tile barrier well before the others (the SIMD
      // favours the wave that was started first), so the loads cost them nothing and relieve the slower four.
      if (sub == 0) {
        tile_dma<D, kFwdTileN, 4>(lds_kv[b], kbase + row0, kv_row_stride, ti.cur.kv_len - ti.c0, zeros, wave, lane, dma_off);
        tile_dma<D, kFwdTileN, 4>(lds_kv[b] + TB, vbase + row0, kv_row_stride, ti.cur.kv_len - ti.c0, zeros, wave, lane, dma_off);
      }
    };
    DevPair tp = ti.cur;
    int tc0 = ti.c0;       // not always 0: an item of a packed block starts at its own first column
    bool have = ti.more;
    if (have) { dma(buf); ti.advance(); }
    dma_wait();
    __syncthreads();
    while (have) {
      const DevPair np = ti.cur;
      const int nc0 = ti.c0;
      const bool nhave = ti.more;
      if (nhave) { dma(buf ^ 1); ti.advance(); }

      const bool diag = (tp.kind & 1) != 0, packed = PACKED && (tp.kind & 2) != 0;
      if (!(diag && tc0 > wave_row_lo + 31)) {      // else nothing visible for this wave
        // wave-uniform: tiles that straddle the diagonal, and tiles that hold a ragged end (their K rows past
        // the end are zero in LDS, but S = 0 there still gives P = exp2(-LSE), which overflows for a row whose
        // logits are all strongly negative; inf * 0 would then poison the whole dQ row)
        const bool need_mask = packed || (diag && tc0 + kFwdTileN - 1 > wave_row_lo) || tc0 + kFwdTileN > tp.kv_len;
        int limit = diag ? tile_off_q + my_row : tp.kv_len - 1;      // last visible column for this lane
        int first = 0;                                               // first one (a packed block: the row's own member)
        if (packed) {
          const uint32_t sg = s_seg[tid];
          first = (int)(sg & 0xffff);
          limit = min(limit, (int)(sg >> 16) - 1);
        }
        // the two 32-row halves of the KV tile one after the other: half the live accumulators
#pragma unroll
        for (int rt = 0; rt < 2; rt++) {
          f32x16 s, dp;
#pragma unroll
          for (int r = 0; r < 16; r++) { s[r] = 0.f; dp[r] = 0.f; }
          // K and V rows are requested PFQ k-chunks (2 PFQ MFMAs) before the MFMAs that use them; left to
          // the compiler each read is issued one MFMA ahead and waited for in full (depths 1 .. 4 measured: 2)
          constexpr int PFQ = 2;
          u32x4 opk[PFQ], opv[PFQ];
#pragma unroll
          for (int i = 0; i < PFQ; i++) {
            opk[i] = lds_read16(row_off[i] + rt * 32 * (D * 2));
            opv[i] = lds_read16(row_off[i] + rt * 32 * (D * 2) + TB);
          }
#pragma unroll
          for (int kc = 0; kc < KC; kc++) {
            s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(opk[kc % PFQ]), qf[kc], s, 0, 0, 0);
            dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(opv[kc % PFQ]), dof[kc], dp, 0, 0, 0);
            if (kc + PFQ < KC) {
              opk[kc % PFQ] = lds_read16(row_off[kc + PFQ] + rt * 32 * (D * 2));
              opv[kc % PFQ] = lds_read16(row_off[kc + PFQ] + rt * 32 * (D * 2) + TB);
            }
            __builtin_amdgcn_sched_barrier(0);
          }
#pragma unroll
          for (int r = 0; r < 16; r++) s[r] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[r], a.scale_log2, -lse_l));
          if (need_mask) {                    // wave-uniform: only tiles that straddle the diagonal
#pragma unroll
            for (int r = 0; r < 16; r++) {
              const int c = tc0 + rt * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
              if (c > limit || c < first) s[r] = 0.f;
            }
          }
#pragma unroll
          for (int r = 0; r < 16; r++) s[r] *= __builtin_fmaf(dp[r], a.scale, -dl_l);
#pragma unroll
          for (int j = 0; j < 2; j++) {
            u32x4 db;
#pragma unroll
            for (int i = 0; i < 4; i++) db[i] = pack_bf16(s[8 * j + 2 * i], s[8 * j + 2 * i + 1]);
            const uint32_t rows = (rt * 32 + 16 * j) * (D * 2);
#pragma unroll
            for (int dt = 0; dt < DT; dt++) {
              const bf16x8 kt = lds_tr_pair_at(tr_lo[dt] + rows, tr_hi[dt] + rows);
              acc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kt, as_bf16x8(db), acc[dt], 0, 0, 0);
            }
          }
        }
      }
      tp = np; tc0 = nc0; have = nhave;
      dma_wait();
      __syncthreads();
      switch_buffer();
    }
    if (row_ok) {
      const int64_t off = (int64_t)(q_start + my_row) * q_row_stride + (int64_t)head * D;
      if constexpr (GRAD_BF16) {
#pragma unroll
        for (int dt = 0; dt < DT; dt++) store_tile_bf16(reinterpret_cast<uint16_t*>(a.dq) + off + dt * 32, acc[dt], 1.0f, g);
      } else {
        float* op = reinterpret_cast<float*>(a.dq) + off;
#pragma unroll
        for (int dt = 0; dt < DT; dt++)
#pragma unroll
          for (int q4 = 0; q4 < 4; q4++) {
            f32x4 w = {acc[dt][4 * q4], acc[dt][4 * q4 + 1], acc[dt][4 * q4 + 2], acc[dt][4 * q4 + 3]};
            *reinterpret_cast<f32x4*>(op + dt * 32 + 8 * q4 + 4 * g) = w;
          }
      }
    }
    __syncthreads();   // every wave has read s_item
    if (tid == 0) s_item = items.resolve();
    __syncthreads();
  }
  if (tid == 0) retire(a.hdr->dq_counter, &a.hdr->dq_done);
}

// =====================================================================================
// Backward, part 2 without recomputation -- dQ from the dS fragments that dkdv_kernel<.., SPILL> left in memory.
// Same items as dq_kernel (two 128-row query sub-tiles that share a KV head, over all pairs of the query block);
// 8 waves, wave = (sub-item, 32-row query group).  Per 64-row KV tile:
//   dQ^T (d x 32 query rows) += K^T (d x 64) dS^T (64 x 32)
// A = K^T by transpose reads of the shared K tile; B = dS^T by transpose reads of the wave's own two fragments,
// which hold dS^T[kv][q] in the 8-byte pieces the producer wrote (4 consecutive query rows of one KV row) at
// rotated positions (see dkdv_kernel), so that a half-wave's 32 pieces cover the 64 banks once.  Both operands
// assign the 8 k-slots of lane half g to KV rows {4g..4g+3} and {8+4g..8+4g+3} of the 16-row chunk.
// The kernel is bound by the HBM stream of fragments (2 bytes per score entry and head against 2 d FLOPs), so the
// ring of three stages (K tile + 8 x 2 fragments each) is there to keep two stages of loads in flight, filled by
// LDS-DMA; one workgroup barrier per tile.  Nothing is masked here: dS is already zero wherever a score is masked,
// and fragments above a wave's diagonal or past a ragged end are skipped, not read.
// =====================================================================================
constexpr int kDqDsBufs = 3;

template <int D, bool GRAD_BF16>
__global__ void __launch_bounds__(512, 2) dq_ds_kernel(BwdArgs a) {
  constexpr int DT = D / 32;
  constexpr int TBK = tile_bytes<D>(kFwdTileN);
  constexpr int WDS = 2 * kDsFragBytes;               // a wave's two fragments of a tile
  constexpr int STAGE = TBK + 8 * WDS;
  constexpr int NB = kDqDsBufs;
  constexpr int CPR = D / 8, RPI = 64 / CPR, NDMA = kFwdTileN / RPI / 8;
  constexpr int DMA_PER_TILE = NDMA + WDS / 1024;
  __shared__ __attribute__((aligned(1024))) unsigned char lds_st[NB][STAGE];
  __shared__ int s_item;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int sub = wave >> 2, wq = wave & 3;
  const int l32 = lane & 31, g = lane >> 5;
  const int group = a.n_q_heads / a.n_kv_heads;
  const int64_t q_row_stride = (int64_t)a.n_q_heads * D;
  const int64_t kv_row_stride = (int64_t)a.n_kv_heads * D;
  const unsigned char* zeros = reinterpret_cast<const unsigned char*>(a.hdr->zeros);
  // K tile loads: as in the forward (rows past a ragged end repeat the last valid row: their dS is zero)
  uint32_t dma_row[NDMA], dma_chunk[NDMA];
#pragma unroll
  for (int n = 0; n < NDMA; n++) {
    const int r = (8 * n + wave) * RPI + lane / CPR, pc = lane % CPR;
    dma_row[n] = (uint32_t)(r * kv_row_stride * 2);
    dma_chunk[n] = (uint32_t)((pc ^ swz<D>(r)) << 4);
  }
  // K^T operands: transpose reads of the K tile, d rows 32 dt .. of k-chunk rows {4g..} / {8+4g..}
  const int tr_row = (lane & 15) >> 2, tr_col = 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
  uint32_t tr_lo[DT], tr_hi[DT];
#pragma unroll
  for (int dt = 0; dt < DT; dt++) {
    tr_lo[dt] = lds_addr(lds_st[0]) + tile_off<D>(4 * g + tr_row, 4 * dt + (tr_col >> 3)) + (tr_col & 4) * 2;
    tr_hi[dt] = lds_addr(lds_st[0]) + tile_off<D>(4 * g + tr_row + 8, 4 * dt + (tr_col >> 3)) + (tr_col & 4) * 2;
  }
  // dS^T operands: lane s of a 16-lane group names the piece of KV row r0 + s / 4, query columns 16 (G & 1) + 4 (s & 3) ..
  uint32_t ds_a[2][2];      // [k-chunk of the fragment][rows +0..3 / +8..11]
  {
    const int s16 = lane & 15, G = lane >> 4;
    const int j = G & 1, gg = s16 & 1, mm = (s16 >> 1) & 1;
#pragma unroll
    for (int kc = 0; kc < 2; kc++)
#pragma unroll
      for (int h = 0; h < 2; h++) {
        const int r = 16 * kc + 8 * h + 4 * g + (s16 >> 2);
        ds_a[kc][h] = lds_addr(lds_st[0]) + TBK + wave * WDS + 1024 * j + 512 * gg + 16 * ((r + 8 * j + 4 * gg) & 31) + 8 * mm;
      }
  }
  int b_c = 0, b_dma = 0;       // ring positions: stage being read, stage being filled
  auto advance_read_stage = [&]() {
    const int st = (b_c == NB - 1) ? -(NB - 1) * STAGE : STAGE;
#pragma unroll
    for (int dt = 0; dt < DT; dt++) { tr_lo[dt] += st; tr_hi[dt] += st; }
#pragma unroll
    for (int kc = 0; kc < 2; kc++) { ds_a[kc][0] += st; ds_a[kc][1] += st; }
    b_c = (b_c == NB - 1) ? 0 : b_c + 1;
  };

  ItemStream items;
  if (tid == 0) { items.init(a.hdr->dq_counter, a.hdr->dq_begin); items.request(); s_item = items.resolve(); }
  __syncthreads();
  for (;;) {
    const int item_idx = __builtin_amdgcn_readfirstlane(s_item);
    if (item_idx < 0) break;
    if (tid == 0) items.request();      // the item after this one
    const QItem it = a.dq_items[item_idx];
    const int q_start = (sub ? it.q_start[1] : it.q_start[0]), q_rows = (sub ? it.q_rows[1] : it.q_rows[0]), tile_off_q = (sub ? it.tile_off[1] : it.tile_off[0]), head = (sub ? it.head[1] : it.head[0]);
    const int kvh = it.head[0] / group;
    const int my_row = wq * 32 + l32;
    const bool row_ok = my_row < q_rows;
    const int wave_row_lo = tile_off_q + wq * 32;
    const bool wave_ok = wq * 32 < q_rows;                       // the wave has at least one valid row
    const int nq32 = (it.q_blk_len + 31) >> 5;
    const int q32 = min((tile_off_q >> 5) + wq, nq32 - 1);       // clamped: a wave past the ragged end reads valid memory and uses nothing
    const uint16_t* kbase = a.k + (int64_t)kvh * D;

    f32x16 acc[DT];
#pragma unroll
    for (int dt = 0; dt < DT; dt++)
#pragma unroll
      for (int r = 0; r < 16; r++) acc[dt][r] = 0.f;

    TileIter ti;
    ti.init(a.pairs, it);
    const int n_tiles = it.n_tiles;
    // The load of one tile: describe() = scalar bookkeeping, issue() = branch-free requests.
    uint64_t d_k = 0, d_ds = 0;
    uint32_t d_lim = 0;
    int d_vis = 0;                  // columns of the tile that this wave's rows can see (0 .. 64)
    auto describe = [&]() {
      d_k = reinterpret_cast<uint64_t>(zeros); d_lim = 0; d_vis = 0;
      d_ds = reinterpret_cast<uint64_t>(a.ds);
      if (ti.more) {
        const int64_t row0 = (int64_t)(ti.cur.kv_start + ti.c0) * kv_row_stride;
        d_k = reinterpret_cast<uint64_t>(kbase + row0);
        const int valid = min(kFwdTileN, ti.cur.kv_len - ti.c0);
        d_lim = (uint32_t)((valid - 1) * kv_row_stride * 2);
        const int f0 = ti.c0 >> 5;
        int frag;
        if (ti.cur.kind & 1) {
          frag = ti.cur.ds_frag + head * (nq32 * (nq32 + 1) / 2) + q32 * (q32 + 1) / 2 + min(f0, q32);
        } else {
          const int nkv32 = (ti.cur.kv_len + 31) >> 5;
          frag = ti.cur.ds_frag + (head * nq32 + q32) * nkv32 + min(f0, nkv32 - 1);
        }
        d_ds = reinterpret_cast<uint64_t>(a.ds + (int64_t)frag * kDsFragBytes);
        const int vis = (ti.cur.kind & 1) ? min(ti.cur.kv_len, wave_row_lo + 32) : ti.cur.kv_len;
        d_vis = wave_ok ? max(0, min(kFwdTileN, vis - ti.c0)) : 0;
        ti.advance();
      }
    };
    auto issue = [&]() {
      const uint32_t lbase = lds_addr(lds_st[0]) + b_dma * STAGE;
#pragma unroll
      for (int n = 0; n < NDMA; n++) {
        const uint32_t voff = min(dma_row[n], d_lim) + dma_chunk[n];
        lds_dma16_s(reinterpret_cast<const unsigned char*>(d_k), voff, lbase + (8 * n + wave) * 1024);
      }
#pragma unroll
      for (int n = 0; n < WDS / 1024; n++)
        lds_dma16_s(reinterpret_cast<const unsigned char*>(d_ds), (uint32_t)(1024 * n + 16 * lane), lbase + TBK + wave * WDS + 1024 * n);
      b_dma = (b_dma == NB - 1) ? 0 : b_dma + 1;
    };
    // prologue: tiles 0 and 1 of the item into the stage to be read first and the one after it
    int vis[3];
    b_dma = b_c;
    describe(); issue(); vis[0] = d_vis;
    describe(); issue(); vis[1] = d_vis;
    for (int t = 0; t < n_tiles; t++) {
      // tile t has landed once at most one tile's loads are in flight; the barrier also says that every wave
      // is done with the stage that tile t + 2 goes into
      __builtin_amdgcn_s_waitcnt(0x0F70 | (DMA_PER_TILE & 15) | ((DMA_PER_TILE >> 4) << 14));
      __syncthreads();
      describe(); issue(); vis[2] = d_vis;
      const int nv = __builtin_amdgcn_readfirstlane(vis[0]);
#pragma unroll
      for (int f = 0; f < 2; f++) {
        if (nv > 32 * f) {
#pragma unroll
          for (int kc = 0; kc < 2; kc++) {
            const bf16x8 b = lds_tr_pair_at(ds_a[kc][0] + kDsFragBytes * f, ds_a[kc][1] + kDsFragBytes * f);
            const uint32_t rows = (32 * f + 16 * kc) * (D * 2);
#pragma unroll
            for (int dt = 0; dt < DT; dt++) {
              const bf16x8 kt = lds_tr_pair_at(tr_lo[dt] + rows, tr_hi[dt] + rows);
              acc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kt, b, acc[dt], 0, 0, 0);
            }
          }
        }
      }
      vis[0] = vis[1]; vis[1] = vis[2];
      advance_read_stage();
    }
    dma_wait();          // the two look-ahead requests past the end of the item
    if (row_ok) {
      const int64_t off = (int64_t)(q_start + my_row) * q_row_stride + (int64_t)head * D;
      if constexpr (GRAD_BF16) {
#pragma unroll
        for (int dt = 0; dt < DT; dt++) store_tile_bf16(reinterpret_cast<uint16_t*>(a.dq) + off + dt * 32, acc[dt], 1.0f, g);
      } else {
        float* op = reinterpret_cast<float*>(a.dq) + off;
#pragma unroll
        for (int dt = 0; dt < DT; dt++)
#pragma unroll
          for (int q4 = 0; q4 < 4; q4++) {
            f32x4 w = {acc[dt][4 * q4], acc[dt][4 * q4 + 1], acc[dt][4 * q4 + 2], acc[dt][4 * q4 + 3]};
            *reinterpret_cast<f32x4*>(op + dt * 32 + 8 * q4 + 4 * g) = w;
          }
      }
    }
    __syncthreads();   // every wave has read s_item
    if (tid == 0) s_item = items.resolve();
    __syncthreads();
  }
  if (tid == 0) retire(a.hdr->dq_counter, &a.hdr->dq_done);
}

// =====================================================================================
// Launchers
// =====================================================================================
static int cu_count() {
  static int cached[64] = {0};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
  if (cached[dev] == 0) {
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
    cached[dev] = n;
  }
  return cached[dev];
}

static int check_launch(const char* what) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) { set_error("%s: %s", what, hipGetErrorString(e)); return FCP_ERR_HIP; }
  return FCP_OK;
}

static float resolve_scale(const fcp_problem* p) {
  return p->softmax_scale > 0.f ? p->softmax_scale : 1.0f / sqrtf((float)p->head_dim);
}

constexpr int kFwdWgPerCu = 1;   // 8 waves, two per SIMD
constexpr int kDkdvWgPerCu = 1;   // 8 waves, two per SIMD
constexpr int kDqWgPerCu = 1;   // 8 waves, two per SIMD

}  // namespace fcp

using namespace fcp;

extern "C" int fcp_device_info(int32_t* n_compute_units, int32_t* fwd_grid, int32_t* bwd_grid) {
  const int n = cu_count();
  if (n_compute_units) *n_compute_units = n;
  if (fwd_grid) *fwd_grid = n * kFwdWgPerCu;
  if (bwd_grid) *bwd_grid = n * kDkdvWgPerCu;
  return FCP_OK;
}

static int launch_fwd(const char* who, const fcp_problem* p, const void* q, const void* k, const void* v,
                      void* o_part, float* lse_part, void* o, float* lse, void* workspace, void* stream) {
  WsLayout L;
  int rc = layout_for(p, workspace, &L);
  if (rc) return rc;
  if (L.n_fwd_items == 0) return FCP_OK;
  if (!q || !k || !v || !workspace || (p->n_slot_rows && !(p->flags & FCP_FLAG_RUNNING_MERGE) && (!o_part || !lse_part))) {
    set_error("%s: NULL pointer", who); return FCP_ERR_INVALID_ARG;
  }
  const bool direct = (p->flags & FCP_FLAG_DIRECT_SINGLE) != 0;
  const bool running = (p->flags & FCP_FLAG_RUNNING_MERGE) != 0;
  if (running) {
    if (!o || !lse || !(p->flags & FCP_FLAG_O_F32)) {
      set_error("%s: FCP_FLAG_RUNNING_MERGE needs the running o (fp32: FCP_FLAG_O_F32) and lse (call fcp_block_attn_fwd_out)", who);
      return FCP_ERR_INVALID_ARG;
    }
    for (int s = 1; s < p->n_slots; s++)
      if (p->slots[s].q_blk == p->slots[s - 1].q_blk) {
        set_error("%s: FCP_FLAG_RUNNING_MERGE takes one stage per launch, but query block %d has several slots (see fcp_stage_tables)",
                  who, p->slots[s].q_blk);
        return FCP_ERR_INVALID_ARG;
      }
  }
  if (direct && (!o || !lse)) {
    set_error("%s: FCP_FLAG_DIRECT_SINGLE needs the final o and lse (call fcp_block_attn_fwd_out)", who);
    return FCP_ERR_INVALID_ARG;
  }
  unsigned char* ws = static_cast<unsigned char*>(workspace);
  FwdArgs a;
  a.q = (const uint16_t*)q; a.k = (const uint16_t*)k; a.v = (const uint16_t*)v;
  a.o_part = o_part; a.lse_part = lse_part; a.part_is_bf16 = (p->flags & FCP_FLAG_PART_BF16) ? 1 : 0;
  a.o = (direct || running) ? o : nullptr; a.lse = (direct || running) ? lse : nullptr;
  a.running = running ? 1 : 0;
  a.o_is_f32 = (p->flags & FCP_FLAG_O_F32) ? 1 : 0;
  a.hdr = reinterpret_cast<WsHeader*>(ws);
  a.pairs = reinterpret_cast<const DevPair*>(ws + L.off_pairs);
  a.items = reinterpret_cast<const QItem*>(ws + L.off_fwd_items);
  a.q_seg = reinterpret_cast<const uint32_t*>(ws + L.off_q_seg);
  a.n_q_heads = p->n_q_heads; a.n_kv_heads = p->n_kv_heads;
  a.scale_log2 = resolve_scale(p) * kLog2e;
  // two launches: the items of ordinary blocks, then (if any) those of packed blocks through the instance for them;
  // they write different rows, and the stream keeps them in order
  const int64_t n_plain = L.n_fwd_items - L.n_fwd_packed_items;
  if (n_plain > 0) {
    a.counter = a.hdr->fwd_counter; a.begin = a.hdr->fwd_begin; a.done = &a.hdr->fwd_done;
    const int grid = (int)std::min<int64_t>(n_plain, (int64_t)cu_count() * kFwdWgPerCu);
    if (p->head_dim == 128) hipLaunchKernelGGL((fwd_kernel<128, false>), dim3(grid), dim3(512), 0, (hipStream_t)stream, a);
    else hipLaunchKernelGGL((fwd_kernel<64, false>), dim3(grid), dim3(512), 0, (hipStream_t)stream, a);
  }
  if (L.n_fwd_packed_items > 0) {
    a.counter = a.hdr->fwdp_counter; a.begin = a.hdr->fwdp_begin; a.done = &a.hdr->fwdp_done;
    const int grid = (int)std::min<int64_t>(L.n_fwd_packed_items, (int64_t)cu_count() * kFwdWgPerCu);
    if (p->head_dim == 128) hipLaunchKernelGGL((fwd_kernel<128, true>), dim3(grid), dim3(512), 0, (hipStream_t)stream, a);
    else hipLaunchKernelGGL((fwd_kernel<64, true>), dim3(grid), dim3(512), 0, (hipStream_t)stream, a);
  }
  return check_launch(who);
}

extern "C" int fcp_block_attn_fwd(const fcp_problem* p, const void* q, const void* k, const void* v,
                                  void* o_part, float* lse_part, void* workspace, void* stream) {
  return launch_fwd("fcp_block_attn_fwd", p, q, k, v, o_part, lse_part, nullptr, nullptr, workspace, stream);
}

// ---- forward without any allocation: the queue tables live in a fixed device array ----
namespace fcp {
constexpr size_t kStaticScratchBytes = 2u << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
// Device address of `scratch` on each device (the array's name is a host-side stand-in, not an
// address a kernel can use; every device holds its own copy at its own address).
static void* g_scratch_ptr[64] = {nullptr};

static int static_scratch(void** ptr) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) { set_error("fcp_block_attn_fwd_static: hipGetDevice: %s", hipGetErrorString(e)); return FCP_ERR_HIP; }
  if (dev < 0 || dev >= 64) { set_error("fcp_block_attn_fwd_static: device index %d out of range", dev); return FCP_ERR_UNSUPPORTED; }
  if (!g_scratch_ptr[dev]) {
    void* sym = nullptr;
    e = hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !sym) {
      set_error("fcp_block_attn_fwd_static: hipGetSymbolAddress: %s", hipGetErrorString(e));
      return FCP_ERR_HIP;
    }
    g_scratch_ptr[dev] = sym;
  }
  *ptr = g_scratch_ptr[dev];
  return FCP_OK;
}
}  // namespace fcp

extern "C" int fcp_block_attn_fwd_static(const fcp_problem* p, const void* q, const void* k, const void* v,
                                         void* o_part, float* lse_part, void* stream) {
  int rc = validate_problem(p);
  if (rc) return rc;
  if (p->flags & FCP_FLAG_DIRECT_SINGLE) {
    set_error("fcp_block_attn_fwd_static: FCP_FLAG_DIRECT_SINGLE is not supported here (all slots go to the partial buffers)");
    return FCP_ERR_INVALID_ARG;
  }
  WsLayout L;
  rc = compute_layout(p, &L);
  if (rc) return rc;
  if (L.off_bwd_deps > kStaticScratchBytes) {
    set_error("fcp_block_attn_fwd_static: the forward's queue tables need %zu bytes, the fixed scratch array holds %zu "
              "(use fcp_queue_build + fcp_block_attn_fwd with a workspace of your own)", L.off_bwd_deps, kStaticScratchBytes);
    return FCP_ERR_BUFFER_TOO_SMALL;
  }
  if (L.n_fwd_items == 0) return FCP_OK;
  void* ws = nullptr;
  rc = static_scratch(&ws);
  if (rc) return rc;
  // The tables are rebuilt on every call (the array keeps the previous call's contents): header with
  // zeroed counters, resolved pairs, forward items.  Host memory only; one copy; the copy is waited for
  // because its source dies with this frame.
  std::vector<unsigned char> image;
  rc = build_queue_image(p, L, true, &image);
  if (rc) return rc;
  hipError_t e = hipMemcpyAsync(ws, image.data(), image.size(), hipMemcpyHostToDevice, (hipStream_t)stream);
  if (e == hipSuccess) e = hipStreamSynchronize((hipStream_t)stream);
  if (e != hipSuccess) { set_error("fcp_block_attn_fwd_static: %s", hipGetErrorString(e)); return FCP_ERR_HIP; }
  return launch_fwd("fcp_block_attn_fwd_static", p, q, k, v, o_part, lse_part, nullptr, nullptr, ws, stream);
}

extern "C" int fcp_block_attn_fwd_out(const fcp_problem* p, const void* q, const void* k, const void* v,
                                      void* o_part, float* lse_part, void* o, float* lse,
                                      void* workspace, void* stream) {
  return launch_fwd("fcp_block_attn_fwd_out", p, q, k, v, o_part, lse_part, o, lse, workspace, stream);
}

extern "C" int fcp_merge_partials(const fcp_problem* p, const void* o_part, const float* lse_part,
                                  void* o, float* lse, void* workspace, void* stream) {
  WsLayout L;
  int rc = layout_for(p, workspace, &L);
  if (rc) return rc;
  if (L.n_merge_items == 0) return FCP_OK;
  if (!o || !lse || !workspace || (p->n_slots && (!o_part || !lse_part))) { set_error("fcp_merge_partials: NULL pointer"); return FCP_ERR_INVALID_ARG; }
  unsigned char* ws = static_cast<unsigned char*>(workspace);
  MergeArgs a;
  a.o_part = o_part; a.lse_part = lse_part; a.o = o; a.lse = lse;
  a.items = reinterpret_cast<const MergeItem*>(ws + L.off_merge_items);
  a.slot_rh = reinterpret_cast<const int32_t*>(ws + L.off_slot_rh);
  a.o_is_f32 = (p->flags & FCP_FLAG_O_F32) ? 1 : 0;
  a.part_is_bf16 = (p->flags & FCP_FLAG_PART_BF16) ? 1 : 0;
  if (p->head_dim == 128) hipLaunchKernelGGL(merge_kernel<128>, dim3((unsigned)L.n_merge_items), dim3(256), 0, (hipStream_t)stream, a);
  else hipLaunchKernelGGL(merge_kernel<64>, dim3((unsigned)L.n_merge_items), dim3(256), 0, (hipStream_t)stream, a);
  return check_launch("fcp_merge_partials");
}

extern "C" int fcp_bwd_preprocess(const fcp_problem* p, const void* o, const float* lse, const void* d_o,
                                  void* workspace, void* stream) {
  WsLayout L;
  int rc = layout_for(p, workspace, &L);
  if (rc) return rc;
  if (L.t_q == 0) return FCP_OK;
  if (!o || !lse || !d_o || !workspace) { set_error("fcp_bwd_preprocess: NULL pointer"); return FCP_ERR_INVALID_ARG; }
  hipStream_t st = (hipStream_t)stream;
  unsigned char* ws = static_cast<unsigned char*>(workspace);
  float* dls = reinterpret_cast<float*>(ws + L.off_dls);
  float* lse2 = reinterpret_cast<float*>(ws + L.off_lse2);
  const int o_f32 = (p->flags & FCP_FLAG_O_F32) ? 1 : 0;
  const float scale = resolve_scale(p);
  const unsigned blocks = (unsigned)((L.t_q + kDeltaTok - 1) / kDeltaTok);
  if (p->head_dim == 128) hipLaunchKernelGGL(delta_kernel<128>, dim3(blocks), dim3(256), 0, st, o, o_f32, (const uint16_t*)d_o, lse, dls, lse2, L.t_q, p->n_q_heads, scale);
  else hipLaunchKernelGGL(delta_kernel<64>, dim3(blocks), dim3(256), 0, st, o, o_f32, (const uint16_t*)d_o, lse, dls, lse2, L.t_q, p->n_q_heads, scale);
  return check_launch("fcp_bwd_preprocess");
}

static int fill_bwd_args(const fcp_problem* p, WsLayout* L, BwdArgs* a, void* workspace) {
  int rc = layout_for(p, workspace, L);
  if (rc) return rc;
  unsigned char* ws = static_cast<unsigned char*>(workspace);
  a->hdr = reinterpret_cast<WsHeader*>(ws);
  a->dls = reinterpret_cast<const float*>(ws + L->off_dls);
  a->lse2 = reinterpret_cast<const float*>(ws + L->off_lse2);
  a->t_q = L->t_q;
  a->pairs = reinterpret_cast<const DevPair*>(ws + L->off_pairs);
  a->deps = reinterpret_cast<const BwdDep*>(ws + L->off_bwd_deps);
  a->items = reinterpret_cast<const BwdItem*>(ws + L->off_bwd_items);
  a->dq_items = reinterpret_cast<const QItem*>(ws + L->off_dq_items);
  a->q_seg = reinterpret_cast<const uint32_t*>(ws + L->off_q_seg);
  a->kv_seg = reinterpret_cast<const uint32_t*>(ws + L->off_kv_seg);
  a->n_q_heads = p->n_q_heads; a->n_kv_heads = p->n_kv_heads;
  a->scale = resolve_scale(p); a->scale_log2 = a->scale * kLog2e;
  a->dq = nullptr; a->dk = nullptr; a->dv = nullptr;
  a->o = nullptr; a->lse = nullptr; a->o_is_f32 = 0; a->lse2_out = nullptr; a->dls_out = nullptr; a->ds = nullptr;
  return FCP_OK;
}

extern "C" int fcp_block_attn_bwd_dkdv(const fcp_problem* p, const void* q, const void* k, const void* v,
                                       const void* d_o, void* dk, void* dv, void* workspace, void* stream) {
  WsLayout L;
  BwdArgs a;
  int rc = fill_bwd_args(p, &L, &a, workspace);
  if (rc) return rc;
  if (L.n_bwd_items == 0) return FCP_OK;
  if (!q || !k || !v || !d_o || !dk || !dv || !workspace) { set_error("fcp_block_attn_bwd_dkdv: NULL pointer"); return FCP_ERR_INVALID_ARG; }
  a.q = (const uint16_t*)q; a.k = (const uint16_t*)k; a.v = (const uint16_t*)v; a.d_o = (const uint16_t*)d_o;
  a.dk = dk; a.dv = dv;
  int grid = (int)std::min<int64_t>(L.n_bwd_items, (int64_t)cu_count() * kDkdvWgPerCu);
  const bool gb = (p->flags & FCP_FLAG_GRAD_BF16) != 0;
  const bool spill = (p->flags & FCP_FLAG_BWD_SPILL_DS) != 0;
  if (spill) a.ds = static_cast<unsigned char*>(workspace) + L.off_ds;
  void (*kern)(BwdArgs) =
      spill ? (p->head_dim == 128 ? (gb ? dkdv_kernel<128, true, true> : dkdv_kernel<128, false, true>)
                                  : (gb ? dkdv_kernel<64, true, true> : dkdv_kernel<64, false, true>))
            : (p->head_dim == 128 ? (gb ? dkdv_kernel<128, true, false> : dkdv_kernel<128, false, false>)
                                  : (gb ? dkdv_kernel<64, true, false> : dkdv_kernel<64, false, false>));
  hipLaunchKernelGGL(kern, dim3(grid), dim3(512), 0, (hipStream_t)stream, a);
  return check_launch("fcp_block_attn_bwd_dkdv");
}

// o / lse == NULL: the per-row scalars come from fcp_bwd_preprocess; else the kernel computes and publishes them.
static int launch_dq(const char* who, const fcp_problem* p, const void* q, const void* k, const void* v,
                     const void* o, const float* lse, const void* d_o, void* dq, void* workspace, void* stream) {
  WsLayout L;
  BwdArgs a;
  int rc = fill_bwd_args(p, &L, &a, workspace);
  if (rc) return rc;
  if (L.n_dq_items == 0) return FCP_OK;
  if (!q || !k || !v || !d_o || !dq || !workspace) { set_error("%s: NULL pointer", who); return FCP_ERR_INVALID_ARG; }
  a.q = (const uint16_t*)q; a.k = (const uint16_t*)k; a.v = (const uint16_t*)v; a.d_o = (const uint16_t*)d_o;
  a.dq = dq;
  const int grid = (int)std::min<int64_t>(L.n_dq_items, (int64_t)cu_count() * kDqWgPerCu);
  const bool gb = (p->flags & FCP_FLAG_GRAD_BF16) != 0, d128 = p->head_dim == 128, packed = p->n_segments > 0;
  if (packed) {
    // the kernel instance for packed blocks reads D and LSE from the workspace: run the D pass here if the caller has not
    if (o) {
      rc = fcp_bwd_preprocess(p, o, lse, d_o, workspace, stream);
      if (rc) return rc;
    }
    void (*kern)(BwdArgs) = d128 ? (gb ? dq_kernel<128, false, true, true> : dq_kernel<128, false, false, true>)
                                 : (gb ? dq_kernel<64, false, true, true> : dq_kernel<64, false, false, true>);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(512), 0, (hipStream_t)stream, a);
    return check_launch(who);
  }
  const bool with_d = o != nullptr;
  if (with_d) {
    unsigned char* ws = static_cast<unsigned char*>(workspace);
    a.o = o; a.lse = lse; a.o_is_f32 = (p->flags & FCP_FLAG_O_F32) ? 1 : 0;
    a.dls_out = reinterpret_cast<float*>(ws + L.off_dls);
    a.lse2_out = reinterpret_cast<float*>(ws + L.off_lse2);
  }
  void (*kern)(BwdArgs) =
      with_d ? (d128 ? (gb ? dq_kernel<128, true, true> : dq_kernel<128, true, false>) : (gb ? dq_kernel<64, true, true> : dq_kernel<64, true, false>))
             : (d128 ? (gb ? dq_kernel<128, false, true> : dq_kernel<128, false, false>) : (gb ? dq_kernel<64, false, true> : dq_kernel<64, false, false>));
  hipLaunchKernelGGL(kern, dim3(grid), dim3(512), 0, (hipStream_t)stream, a);
  return check_launch(who);
}

extern "C" int fcp_block_attn_bwd_dq(const fcp_problem* p, const void* q, const void* k, const void* v,
                                     const void* d_o, void* dq, void* workspace, void* stream) {
  return launch_dq("fcp_block_attn_bwd_dq", p, q, k, v, nullptr, nullptr, d_o, dq, workspace, stream);
}

extern "C" int fcp_block_attn_bwd_dq_d(const fcp_problem* p, const void* q, const void* k, const void* v,
                                       const void* o, const float* lse, const void* d_o, void* dq,
                                       void* workspace, void* stream) {
  if (!o || !lse) {
    int rc = validate_problem(p);
    if (rc) return rc;
    set_error("fcp_block_attn_bwd_dq_d: NULL pointer");
    return FCP_ERR_INVALID_ARG;
  }
  return launch_dq("fcp_block_attn_bwd_dq_d", p, q, k, v, o, lse, d_o, dq, workspace, stream);
}

extern "C" int fcp_block_attn_bwd_dq_ds(const fcp_problem* p, const void* k, void* dq, void* workspace, void* stream) {
  WsLayout L;
  BwdArgs a;
  int rc = fill_bwd_args(p, &L, &a, workspace);
  if (rc) return rc;
  if (!(p->flags & FCP_FLAG_BWD_SPILL_DS)) {
    set_error("fcp_block_attn_bwd_dq_ds: FCP_FLAG_BWD_SPILL_DS is not set on this problem");
    return FCP_ERR_INVALID_ARG;
  }
  if (L.n_dq_items == 0) return FCP_OK;
  if (!k || !dq || !workspace) { set_error("fcp_block_attn_bwd_dq_ds: NULL pointer"); return FCP_ERR_INVALID_ARG; }
  a.k = (const uint16_t*)k;
  a.dq = dq;
  a.ds = static_cast<unsigned char*>(workspace) + L.off_ds;
  const int grid = (int)std::min<int64_t>(L.n_dq_items, (int64_t)cu_count() * kDqWgPerCu);
  const bool gb = (p->flags & FCP_FLAG_GRAD_BF16) != 0;
  void (*kern)(BwdArgs) = p->head_dim == 128 ? (gb ? dq_ds_kernel<128, true> : dq_ds_kernel<128, false>)
                                             : (gb ? dq_ds_kernel<64, true> : dq_ds_kernel<64, false>);
  hipLaunchKernelGGL(kern, dim3(grid), dim3(512), 0, (hipStream_t)stream, a);
  return check_launch("fcp_block_attn_bwd_dq_ds");
}

extern "C" int fcp_block_attn_bwd(const fcp_problem* p, const void* q, const void* k, const void* v,
                                  const void* o, const float* lse, const void* d_o,
                                  void* dq, void* dk, void* dv, void* workspace, void* stream) {
  if (!q || !k || !v || !o || !lse || !d_o || !dq || !dk || !dv || !workspace) {
    int rc = validate_problem(p);
    if (rc) return rc;
    set_error("fcp_block_attn_bwd: NULL pointer");
    return FCP_ERR_INVALID_ARG;
  }
  if (p && (p->flags & FCP_FLAG_BWD_SPILL_DS)) {
    // D first (a pass of its own), then dK/dV, which also writes dS, then dQ from that dS
    int rc = fcp_bwd_preprocess(p, o, lse, d_o, workspace, stream);
    if (rc) return rc;
    rc = fcp_block_attn_bwd_dkdv(p, q, k, v, d_o, dk, dv, workspace, stream);
    if (rc) return rc;
    return fcp_block_attn_bwd_dq_ds(p, k, dq, workspace, stream);
  }
  // dQ first: its kernel also leaves the per-row scalars (D * scale, LSE * log2 e) that dK/dV needs
  int rc = fcp_block_attn_bwd_dq_d(p, q, k, v, o, lse, d_o, dq, workspace, stream);
  if (rc) return rc;
  return fcp_block_attn_bwd_dkdv(p, q, k, v, d_o, dk, dv, workspace, stream);
}

