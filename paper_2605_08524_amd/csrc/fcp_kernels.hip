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

// Pop one item index from the eight XCD queues, own queue first, then stealing.  Returns -1
// when every queue is dry.  Every call terminates: each queue is probed at most once.
__device__ __forceinline__ int pop_item(int32_t* counter, const int32_t* begin) {
  const int home = blockIdx.x % kNumXcd;
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

// =====================================================================================
// Forward: partial attention of one (slot, query tile, query head) item.
// The wave computes S^T = K Q^T so that a lane owns one query row (column of S^T): row
// statistics need one cross-half exchange, and the exponentiated accumulator is, as is,
// the B operand of O^T += V^T P^T.
// =====================================================================================
constexpr int kFwdTileN = 64;   // KV rows per LDS tile

template <int D>
struct FwdCfg {
  static constexpr int kKStride = D * 2 + 16;   // bytes; +16 keeps 16 rows x 16 B on distinct banks
  static constexpr int kVStride = D * 2 + 64;   // bytes; +64 keeps 4 rows x 64 B on distinct banks
  static constexpr int kKBytes = kFwdTileN * kKStride;
  static constexpr int kVBytes = kFwdTileN * kVStride;
  static constexpr int kChunksPerRow = D / 8;                       // 16-byte chunks
  static constexpr int kChunksPerThread = kFwdTileN * kChunksPerRow / 256;
  static constexpr int kRowsPerPass = 256 / kChunksPerRow;
};

struct FwdArgs {
  const uint16_t* q; const uint16_t* k; const uint16_t* v;
  float* o_part; float* lse_part;
  WsHeader* hdr; const DevPair* pairs; const FwdItem* items;
  int32_t n_q_heads, n_kv_heads;
  float scale_log2;   // softmax scale * log2(e)
};

template <int D>
__global__ void __launch_bounds__(256) fwd_kernel(FwdArgs a) {
  using C = FwdCfg<D>;
  constexpr int KC = D / 16;      // k-chunks of the QK^T contraction
  constexpr int DT = D / 32;      // row tiles of O^T
  __shared__ __attribute__((aligned(16))) unsigned char lds_k[C::kKBytes];
  __shared__ __attribute__((aligned(16))) unsigned char lds_v[C::kVBytes];
  __shared__ int s_item;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, g = lane >> 5;
  const int group = a.n_q_heads / a.n_kv_heads;
  const int64_t q_row_stride = (int64_t)a.n_q_heads * D;     // elements
  const int64_t kv_row_stride = (int64_t)a.n_kv_heads * D;
  const int ld_chunk = tid % C::kChunksPerRow, ld_row = tid / C::kChunksPerRow;
  // transpose-read address pattern inside a 16-lane group
  const int tr_row = (lane & 15) >> 2, tr_col = 16 * ((lane >> 4) & 1) + 4 * (lane & 3);

  for (;;) {
    if (tid == 0) s_item = pop_item(a.hdr->fwd_counter, a.hdr->fwd_begin);
    __syncthreads();
    const int item_idx = s_item;
    if (item_idx < 0) break;
    const FwdItem it = a.items[item_idx];
    const int kvh = it.head / group;
    const int my_row = wave * 32 + l32;                      // row inside the tile
    const bool row_ok = my_row < it.q_rows;
    const int wave_row_lo = it.tile_off + wave * 32;         // rows of this wave inside the block

    // Q^T fragments (B operand of S^T = K Q^T): lane = query row, 8 consecutive d per k-chunk.
    bf16x8 qf[KC];
    {
      const uint16_t* qp = a.q + (int64_t)(it.q_start + my_row) * q_row_stride + (int64_t)it.head * D + 8 * g;
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

    // Tile iterator over (pair, column offset).
    int pair = it.pair_begin;
    const int pair_end = it.pair_begin + it.n_pairs;
    bool more = it.n_pairs > 0;       // an empty slot yields O = 0, LSE = -inf
    DevPair cur = {0, 0, 0, 0};
    if (more) cur = a.pairs[pair];
    int c0 = 0;
    auto ncols_of = [&](const DevPair& p) {
      return p.kind == FCP_KIND_DIAG ? min(p.kv_len, it.tile_off + it.q_rows) : p.kv_len;
    };
    int ncols = ncols_of(cur);

    u32x4 pk[C::kChunksPerThread], pv[C::kChunksPerThread];
    auto issue_loads = [&](const DevPair& p, int col0) {
#pragma unroll
      for (int i = 0; i < C::kChunksPerThread; i++) {
        const int r = col0 + ld_row + i * C::kRowsPerPass;
        u32x4 zk = {0, 0, 0, 0}, zv = {0, 0, 0, 0};
        if (r < p.kv_len) {
          const int64_t off = (int64_t)(p.kv_start + r) * kv_row_stride + (int64_t)kvh * D + ld_chunk * 8;
          zk = *reinterpret_cast<const u32x4*>(a.k + off);
          zv = *reinterpret_cast<const u32x4*>(a.v + off);
        }
        pk[i] = zk; pv[i] = zv;
      }
    };
    if (more) issue_loads(cur, 0);

    while (more) {
      const DevPair tp = cur;     // the tile about to be computed
      const int tc0 = c0;
      __syncthreads();            // everyone is done reading the previous tile
#pragma unroll
      for (int i = 0; i < C::kChunksPerThread; i++) {
        const int r = ld_row + i * C::kRowsPerPass;
        *reinterpret_cast<u32x4*>(lds_k + r * C::kKStride + ld_chunk * 16) = pk[i];
        *reinterpret_cast<u32x4*>(lds_v + r * C::kVStride + ld_chunk * 16) = pv[i];
      }
      __syncthreads();
      // advance the iterator and prefetch the next tile into registers
      c0 += kFwdTileN;
      if (c0 >= ncols) {
        pair++;
        c0 = 0;
        if (pair < pair_end) { cur = a.pairs[pair]; ncols = ncols_of(cur); } else { more = false; }
      }
      if (more) issue_loads(cur, c0);

      const bool diag = tp.kind == FCP_KIND_DIAG;
      // a wave whose rows all lie above this tile's first column has nothing visible in it
      if (diag && tc0 > wave_row_lo + 31) continue;

      // ---- S^T = K Q^T  (two 32-row tiles of KV)
      f32x16 s[2];
#pragma unroll
      for (int rt = 0; rt < 2; rt++)
#pragma unroll
        for (int r = 0; r < 16; r++) s[rt][r] = 0.f;
#pragma unroll
      for (int kc = 0; kc < KC; kc++) {
#pragma unroll
        for (int rt = 0; rt < 2; rt++) {
          const u32x4 kk = *reinterpret_cast<const u32x4*>(lds_k + (rt * 32 + l32) * C::kKStride + kc * 32 + g * 16);
          s[rt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(kk), qf[kc], s[rt], 0, 0, 0);
        }
      }
      // ---- mask (only tiles that touch the diagonal or the ragged end)
      const bool need_mask = (tc0 + kFwdTileN > tp.kv_len) || (diag && tc0 + kFwdTileN - 1 > wave_row_lo);
      if (need_mask) {
        const int limit = diag ? min(tp.kv_len - 1, it.tile_off + my_row) : tp.kv_len - 1;   // last visible column
#pragma unroll
        for (int rt = 0; rt < 2; rt++)
#pragma unroll
          for (int r = 0; r < 16; r++) {
            const int col = tc0 + rt * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
            if (col > limit) s[rt][r] = -INFINITY;
          }
      }
      // ---- online softmax in the log2 domain
      float mx = s[0][0];
#pragma unroll
      for (int rt = 0; rt < 2; rt++)
#pragma unroll
        for (int r = 0; r < 16; r++) mx = fmaxf(mx, s[rt][r]);
      mx = fmaxf(mx, xor32(mx));
      const float m_new = fmaxf(m_run, mx * a.scale_log2);
      const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
      const float alpha = __builtin_amdgcn_exp2f(m_run - m_use);
      m_run = m_new;
      float rs = 0.f;
#pragma unroll
      for (int rt = 0; rt < 2; rt++)
#pragma unroll
        for (int r = 0; r < 16; r++) {
          const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s[rt][r], a.scale_log2, -m_use));
          s[rt][r] = p;
          rs += p;
        }
      l_run = l_run * alpha + rs;
#pragma unroll
      for (int dt = 0; dt < DT; dt++)
#pragma unroll
        for (int r = 0; r < 16; r++) o[dt][r] *= alpha;
      // ---- O^T += V^T P^T ; P^T's accumulator registers are its B operand
#pragma unroll
      for (int rt = 0; rt < 2; rt++) {
#pragma unroll
        for (int j = 0; j < 2; j++) {
          u32x4 pb;
          pb[0] = pack_bf16(s[rt][8 * j + 0], s[rt][8 * j + 1]);
          pb[1] = pack_bf16(s[rt][8 * j + 2], s[rt][8 * j + 3]);
          pb[2] = pack_bf16(s[rt][8 * j + 4], s[rt][8 * j + 5]);
          pb[3] = pack_bf16(s[rt][8 * j + 6], s[rt][8 * j + 7]);
          const int kv0 = rt * 32 + 16 * j + 4 * g;
          const unsigned char* base = lds_v + (kv0 + tr_row) * C::kVStride + tr_col * 2;
#pragma unroll
          for (int dt = 0; dt < DT; dt++) {
            const bf16x8 vt = lds_tr_pair(base + dt * 64, base + 8 * C::kVStride + dt * 64);
            o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vt, as_bf16x8(pb), o[dt], 0, 0, 0);
          }
        }
      }
    }

    // ---- epilogue: normalise, write the partial (fp32) and its LSE
    const float l_tot = l_run + xor32(l_run);
    const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;
    if (row_ok) {
      float* op = a.o_part + (int64_t)(it.out_row + my_row) * q_row_stride + (int64_t)it.head * D;
#pragma unroll
      for (int dt = 0; dt < DT; dt++)
#pragma unroll
        for (int q4 = 0; q4 < 4; q4++) {
          f32x4 w = {o[dt][4 * q4] * inv, o[dt][4 * q4 + 1] * inv, o[dt][4 * q4 + 2] * inv, o[dt][4 * q4 + 3] * inv};
          *reinterpret_cast<f32x4*>(op + dt * 32 + 8 * q4 + 4 * g) = w;
        }
      if (g == 0) {
        const float lse = l_tot > 0.f ? (m_run + __builtin_amdgcn_logf(l_tot)) * kLn2 : -INFINITY;
        a.lse_part[(int64_t)(it.out_row + my_row) * a.n_q_heads + it.head] = lse;
      }
    }
    __syncthreads();   // s_item is rewritten next
  }
  if (tid == 0) retire(a.hdr->fwd_counter, &a.hdr->fwd_done);
}

// =====================================================================================
// Merge: LSE-weighted reduction of the partials of each query block.  HBM-bound.
// One group of D/4 lanes owns one (row, head) entry: a float4 of the head vector per lane.
// =====================================================================================
struct MergeArgs {
  const float* o_part; const float* lse_part; void* o; float* lse;
  const MergeItem* items; const int32_t* slot_rh;
  int32_t o_is_f32;
};

template <int D>
__global__ void __launch_bounds__(256) merge_kernel(MergeArgs a) {
  constexpr int LPE = D / 4;            // lanes per entry
  constexpr int EPP = 256 / LPE;        // entries per pass
  const MergeItem it = a.items[blockIdx.x];
  const int sub = threadIdx.x / LPE, ln = threadIdx.x % LPE;
  for (int e = sub; e < it.n_rh; e += EPP) {
    const int64_t in_off = it.rh_off + e;
    float mx = -INFINITY;
    for (int s = 0; s < it.n_slots; s++)
      mx = fmaxf(mx, a.lse_part[(int64_t)a.slot_rh[it.slot_begin + s] + in_off]);
    const float m_use = (mx == -INFINITY) ? 0.f : mx;
    float tot = 0.f;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    for (int s = 0; s < it.n_slots; s++) {
      const int64_t rh = (int64_t)a.slot_rh[it.slot_begin + s] + in_off;
      const float w = __expf(a.lse_part[rh] - m_use);
      const f32x4 x = *reinterpret_cast<const f32x4*>(a.o_part + rh * D + ln * 4);
      tot += w;
      // an empty partial carries weight 0; its payload must not leak through (0 * NaN)
      if (w > 0.f) acc += w * x;
    }
    const float inv = tot > 0.f ? 1.0f / tot : 0.f;
    acc *= inv;
    const int64_t out = (int64_t)it.out_rh + e;
    if (a.o_is_f32) {
      *reinterpret_cast<f32x4*>(reinterpret_cast<float*>(a.o) + out * D + ln * 4) = acc;
    } else {
      u32x2 h = {pack_bf16(acc[0], acc[1]), pack_bf16(acc[2], acc[3])};
      *reinterpret_cast<u32x2*>(reinterpret_cast<uint16_t*>(a.o) + out * D + ln * 4) = h;
    }
    if (ln == 0) a.lse[out] = tot > 0.f ? m_use + __logf(tot) : -INFINITY;
  }
}

// =====================================================================================
// Backward preprocess: D[t,h] = sum_c dO[t,h,c] * O[t,h,c].  HBM-bound.
// =====================================================================================
template <int D>
__global__ void __launch_bounds__(256) delta_kernel(const void* o, int o_is_f32, const uint16_t* d_o,
                                                    float* delta, int64_t n_rh) {
  constexpr int LPE = D / 8;      // lanes per entry, 8 elements each
  const int64_t e = ((int64_t)blockIdx.x * 256 + threadIdx.x) / LPE;
  const int ln = threadIdx.x % LPE;
  float acc = 0.f;
  if (e < n_rh) {
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
  if (e < n_rh && ln == 0) delta[e] = acc;
}

__global__ void __launch_bounds__(256) zero_kernel(f32x4* p, int64_t n4) {
  const f32x4 z = {0.f, 0.f, 0.f, 0.f};
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += (int64_t)gridDim.x * 256) p[i] = z;
}

// =====================================================================================
// Backward: one (KV tile of 128 rows, KV head) item; each wave keeps 32 KV rows' dK^T and
// dV^T accumulators in registers across every dependent query block and the G query heads
// of the group; dQ is reduced over the tile's 128 KV rows through LDS and added atomically.
// Per 32-row query step:
//   S = Q K^T, dP = dO V^T          (A from LDS tiles, B = the wave's K / V fragments)
//   P = exp2(S*c - LSE*log2e), dS = P o (dP - D) * scale
//   dV^T += dO^T P, dK^T += Q^T dS  (A by transpose reads, B = accumulator registers)
//   dQ[:, 32-wide slice of d] = dS K (dS^T staged in LDS, K by transpose-read fragments)
// =====================================================================================
template <int D>
struct BwdCfg {
  static constexpr int kTStride = D * 2 + 16;            // Q / dO / K tile row stride in bytes
  static constexpr int kKBytes = kBwdTileN * kTStride;
  static constexpr int kQBytes = 32 * kTStride;
  static constexpr int kDsBytes = kBwdTileN * 64;        // dS^T [128 kv][32 q] bf16, swizzled
  static constexpr int kChunksPerRow = D / 8;
  static constexpr int kQChunksPerThread = 32 * kChunksPerRow / 256;   // 2 (D=128) or 1 (D=64)
  static constexpr int kRowsPerPass = 256 / kChunksPerRow;
};

struct BwdArgs {
  const uint16_t* q; const uint16_t* k; const uint16_t* v; const uint16_t* d_o;
  const float* lse; const float* delta;
  float* dq; float* dk; float* dv;
  WsHeader* hdr; const BwdDep* deps; const BwdItem* items;
  int32_t n_q_heads, n_kv_heads;
  float scale, scale_log2;
};

template <int D>
__global__ void __launch_bounds__(256) bwd_kernel(BwdArgs a) {
  using C = BwdCfg<D>;
  constexpr int KC = D / 16;
  constexpr int DT = D / 32;
  __shared__ __attribute__((aligned(16))) unsigned char lds_kt[C::kKBytes];
  __shared__ __attribute__((aligned(16))) unsigned char lds_q[C::kQBytes];
  __shared__ __attribute__((aligned(16))) unsigned char lds_do[C::kQBytes];
  __shared__ __attribute__((aligned(16))) unsigned char lds_ds[C::kDsBytes];
  __shared__ __attribute__((aligned(16))) float lds_lse[32];
  __shared__ __attribute__((aligned(16))) float lds_dl[32];
  __shared__ int s_item;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, g = lane >> 5;
  const int group = a.n_q_heads / a.n_kv_heads;
  const int64_t q_row_stride = (int64_t)a.n_q_heads * D;
  const int64_t kv_row_stride = (int64_t)a.n_kv_heads * D;
  const int ld_chunk = tid % C::kChunksPerRow, ld_row = tid / C::kChunksPerRow;
  const int tr_row = (lane & 15) >> 2, tr_col = 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
  const bool dq_wave = wave < DT;     // waves that own a 32-wide slice of d for dQ

  for (;;) {
    if (tid == 0) s_item = pop_item(a.hdr->bwd_counter, a.hdr->bwd_begin);
    __syncthreads();
    const int item_idx = s_item;
    if (item_idx < 0) break;
    const BwdItem it = a.items[item_idx];
    const int my_kv = wave * 32 + l32;                 // KV row inside the tile
    const bool kv_ok = my_kv < it.kv_rows;

    // K tile -> LDS (zero-filled past the ragged end), for the transpose-read fragments of dQ.
    for (int r = ld_row; r < kBwdTileN; r += C::kRowsPerPass) {
      u32x4 z = {0, 0, 0, 0};
      if (r < it.kv_rows)
        z = *reinterpret_cast<const u32x4*>(a.k + (int64_t)(it.kv_start + r) * kv_row_stride + (int64_t)it.kv_head * D + ld_chunk * 8);
      *reinterpret_cast<u32x4*>(lds_kt + r * C::kTStride + ld_chunk * 16) = z;
    }
    // B operands of S = Q K^T and dP = dO V^T: lane = KV row, 8 consecutive d per k-chunk.
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
    __syncthreads();
    // B operands of dQ = dS K for this wave's d slice: lane = d column, k-slot (g, i) = kv 16j + 8g + i.
    bf16x8 kb[kBwdTileN / 16];
    if (dq_wave) {
#pragma unroll
      for (int j = 0; j < kBwdTileN / 16; j++) {
        const unsigned char* base = lds_kt + (16 * j + 8 * g + tr_row) * C::kTStride + (wave * 32 + tr_col) * 2;
        kb[j] = lds_tr_pair(base, base + 4 * C::kTStride);
      }
    }
    f32x16 dkt[DT], dvt[DT];
#pragma unroll
    for (int dt = 0; dt < DT; dt++)
#pragma unroll
      for (int r = 0; r < 16; r++) { dkt[dt][r] = 0.f; dvt[dt][r] = 0.f; }

    // Step iterator over (dependency, query head of the group, 32-row query step).
    const int n_deps = it.n_deps;
    int dep = 0, hh = 0, q0 = 0;
    BwdDep cd = {0, 0, 0, 0};
    auto first_q0 = [&](const BwdDep& d) { return d.kind == FCP_KIND_DIAG ? (it.tile_off & ~31) : 0; };
    bool more = n_deps > 0;
    if (more) {
      cd = a.deps[it.dep_begin];
      q0 = first_q0(cd);
      // a DIAG dependency always has rows at or below this tile's first row (same block)
    }
    u32x4 pq[C::kQChunksPerThread], pdo[C::kQChunksPerThread];
    float p_lse = 0.f, p_dl = 0.f;
    auto issue_loads = [&](const BwdDep& d, int head, int row0) {
#pragma unroll
      for (int i = 0; i < C::kQChunksPerThread; i++) {
        const int r = row0 + ld_row + i * C::kRowsPerPass;
        u32x4 zq = {0, 0, 0, 0}, zd = {0, 0, 0, 0};
        if (r < d.q_len) {
          const int64_t off = (int64_t)(d.q_start + r) * q_row_stride + (int64_t)head * D + ld_chunk * 8;
          zq = *reinterpret_cast<const u32x4*>(a.q + off);
          zd = *reinterpret_cast<const u32x4*>(a.d_o + off);
        }
        pq[i] = zq; pdo[i] = zd;
      }
      if (tid < 32) {
        const int r = row0 + tid;
        float l = INFINITY, dl = 0.f;      // rows past the end get P = exp2(-inf) = 0
        if (r < d.q_len) {
          const int64_t rh = (int64_t)(d.q_start + r) * a.n_q_heads + head;
          l = a.lse[rh];
          if (l == -INFINITY) l = INFINITY;  // a row that saw no key has no gradient
          dl = a.delta[rh];
        }
        p_lse = l * kLog2e; p_dl = dl * a.scale;
      }
    };
    if (more) issue_loads(cd, it.kv_head * group + hh, q0);

    while (more) {
      const BwdDep td = cd;
      const int t_head = it.kv_head * group + hh;
      const int tq0 = q0;
      __syncthreads();     // previous step's readers of the Q/dO/dS tiles are done
#pragma unroll
      for (int i = 0; i < C::kQChunksPerThread; i++) {
        const int r = ld_row + i * C::kRowsPerPass;
        *reinterpret_cast<u32x4*>(lds_q + r * C::kTStride + ld_chunk * 16) = pq[i];
        *reinterpret_cast<u32x4*>(lds_do + r * C::kTStride + ld_chunk * 16) = pdo[i];
      }
      if (tid < 32) { lds_lse[tid] = p_lse; lds_dl[tid] = p_dl; }
      __syncthreads();
      // advance: rows, then heads of the group, then dependencies
      q0 += 32;
      if (q0 >= cd.q_len) {
        hh++;
        if (hh < group) {
          q0 = first_q0(cd);
        } else {
          hh = 0;
          dep++;
          if (dep < n_deps) { cd = a.deps[it.dep_begin + dep]; q0 = first_q0(cd); } else { more = false; }
        }
      }
      if (more) issue_loads(cd, it.kv_head * group + hh, q0);

      // ---- S = Q K^T and dP = dO V^T   (rows = query, cols = this wave's 32 KV rows)
      f32x16 s, dp;
#pragma unroll
      for (int r = 0; r < 16; r++) { s[r] = 0.f; dp[r] = 0.f; }
#pragma unroll
      for (int kc = 0; kc < KC; kc++) {
        const u32x4 qa = *reinterpret_cast<const u32x4*>(lds_q + l32 * C::kTStride + kc * 32 + g * 16);
        const u32x4 da = *reinterpret_cast<const u32x4*>(lds_do + l32 * C::kTStride + kc * 32 + g * 16);
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(qa), kf[kc], s, 0, 0, 0);
        dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(da), vf[kc], dp, 0, 0, 0);
      }
      // ---- P and dS (register r = query row 8*(r/4) + 4g + r%4, lane = KV row)
      const bool diag = td.kind == FCP_KIND_DIAG;
      const int kv_in_blk = it.tile_off + my_kv;
#pragma unroll
      for (int q4 = 0; q4 < 4; q4++) {
        const f32x4 lse4 = *reinterpret_cast<const f32x4*>(&lds_lse[8 * q4 + 4 * g]);
        const f32x4 dl4 = *reinterpret_cast<const f32x4*>(&lds_dl[8 * q4 + 4 * g]);
#pragma unroll
        for (int i = 0; i < 4; i++) {
          const int r = 4 * q4 + i;
          float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s[r], a.scale_log2, -lse4[i]));
          if (diag && kv_in_blk > tq0 + 8 * q4 + 4 * g + i) p = 0.f;
          s[r] = p;
          dp[r] = p * __builtin_fmaf(dp[r], a.scale, -dl4[i]);
        }
      }
      u32x4 pb[2], dsb[2];
#pragma unroll
      for (int j = 0; j < 2; j++)
#pragma unroll
        for (int i = 0; i < 4; i++) {
          pb[j][i] = pack_bf16(s[8 * j + 2 * i], s[8 * j + 2 * i + 1]);
          dsb[j][i] = pack_bf16(dp[8 * j + 2 * i], dp[8 * j + 2 * i + 1]);
        }
      // ---- stage dS^T for the dQ contraction: row = KV, 8-byte granules of 4 query rows, swizzled
      {
        unsigned char* row = lds_ds + my_kv * 64;
        const int sw = (my_kv >> 2) & 7;
#pragma unroll
        for (int q4 = 0; q4 < 4; q4++) {
          u32x2 w = {dsb[q4 >> 1][2 * (q4 & 1)], dsb[q4 >> 1][2 * (q4 & 1) + 1]};
          *reinterpret_cast<u32x2*>(row + (((2 * q4 + g) ^ sw) * 8)) = w;
        }
      }
      // ---- dV^T += dO^T P ; dK^T += Q^T dS   (k-slot (g, i) of chunk j = query 16j + 8(i/4) + 4g + i%4)
#pragma unroll
      for (int j = 0; j < 2; j++) {
        const int qr = 16 * j + 4 * g + tr_row;
        const unsigned char* bq = lds_q + qr * C::kTStride + tr_col * 2;
        const unsigned char* bd = lds_do + qr * C::kTStride + tr_col * 2;
#pragma unroll
        for (int dt = 0; dt < DT; dt++) {
          const bf16x8 dot = lds_tr_pair(bd + dt * 64, bd + 8 * C::kTStride + dt * 64);
          dvt[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dot, as_bf16x8(pb[j]), dvt[dt], 0, 0, 0);
          const bf16x8 qt = lds_tr_pair(bq + dt * 64, bq + 8 * C::kTStride + dt * 64);
          dkt[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qt, as_bf16x8(dsb[j]), dkt[dt], 0, 0, 0);
        }
      }
      __syncthreads();     // dS^T of all four waves is in LDS
      // ---- dQ[32 q][this wave's 32 d] = dS[32 q][128 kv] K[128 kv][32 d]
      if (dq_wave) {
        f32x16 dq;
#pragma unroll
        for (int r = 0; r < 16; r++) dq[r] = 0.f;
#pragma unroll
        for (int j = 0; j < kBwdTileN / 16; j++) {
          // A: lane = query row; k-slot (g, i) = kv 16j + 8g + i  -> two transpose reads of 4 KV rows
          const int kv0 = 16 * j + 8 * g + tr_row;              // row this lane addresses (first read)
          const int gran = (tr_col >> 2);                       // logical granule of 4 query rows
          const unsigned char* lo = lds_ds + kv0 * 64 + ((gran ^ ((kv0 >> 2) & 7)) * 8);
          const unsigned char* hi = lds_ds + (kv0 + 4) * 64 + ((gran ^ (((kv0 + 4) >> 2) & 7)) * 8);
          dq = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lds_tr_pair(lo, hi), kb[j], dq, 0, 0, 0);
        }
        float* dst = a.dq + (int64_t)td.q_start * q_row_stride + (int64_t)t_head * D + wave * 32 + l32;
#pragma unroll
        for (int r = 0; r < 16; r++) {
          const int qr = tq0 + 8 * (r >> 2) + 4 * g + (r & 3);
          if (qr < td.q_len) unsafeAtomicAdd(dst + (int64_t)qr * q_row_stride, dq[r]);
        }
      }
    }

    // ---- epilogue: this item is the only writer of its dK / dV rows (plain stores)
    if (kv_ok) {
      float* kp = a.dk + (int64_t)(it.kv_start + my_kv) * kv_row_stride + (int64_t)it.kv_head * D;
      float* vp = a.dv + (int64_t)(it.kv_start + my_kv) * kv_row_stride + (int64_t)it.kv_head * D;
#pragma unroll
      for (int dt = 0; dt < DT; dt++)
#pragma unroll
        for (int q4 = 0; q4 < 4; q4++) {
          const int d0 = dt * 32 + 8 * q4 + 4 * g;
          f32x4 wk = {dkt[dt][4 * q4], dkt[dt][4 * q4 + 1], dkt[dt][4 * q4 + 2], dkt[dt][4 * q4 + 3]};
          f32x4 wv = {dvt[dt][4 * q4], dvt[dt][4 * q4 + 1], dvt[dt][4 * q4 + 2], dvt[dt][4 * q4 + 3]};
          *reinterpret_cast<f32x4*>(kp + d0) = wk;
          *reinterpret_cast<f32x4*>(vp + d0) = wv;
        }
    }
    __syncthreads();
  }
  if (tid == 0) retire(a.hdr->bwd_counter, &a.hdr->bwd_done);
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

constexpr int kFwdWgPerCu = 2;
constexpr int kBwdWgPerCu = 1;

}  // namespace fcp

using namespace fcp;

extern "C" int fcp_device_info(int32_t* n_compute_units, int32_t* fwd_grid, int32_t* bwd_grid) {
  const int n = cu_count();
  if (n_compute_units) *n_compute_units = n;
  if (fwd_grid) *fwd_grid = n * kFwdWgPerCu;
  if (bwd_grid) *bwd_grid = n * kBwdWgPerCu;
  return FCP_OK;
}

extern "C" int fcp_block_attn_fwd(const fcp_problem* p, const void* q, const void* k, const void* v,
                                  float* o_part, float* lse_part, void* workspace, void* stream) {
  int rc = validate_problem(p);
  if (rc) return rc;
  WsLayout L;
  rc = compute_layout(p, &L);
  if (rc) return rc;
  if (L.n_fwd_items == 0) return FCP_OK;
  if (!q || !k || !v || !o_part || !lse_part || !workspace) { set_error("fcp_block_attn_fwd: NULL pointer"); return FCP_ERR_INVALID_ARG; }
  unsigned char* ws = static_cast<unsigned char*>(workspace);
  FwdArgs a;
  a.q = (const uint16_t*)q; a.k = (const uint16_t*)k; a.v = (const uint16_t*)v;
  a.o_part = o_part; a.lse_part = lse_part;
  a.hdr = reinterpret_cast<WsHeader*>(ws);
  a.pairs = reinterpret_cast<const DevPair*>(ws + L.off_pairs);
  a.items = reinterpret_cast<const FwdItem*>(ws + L.off_fwd_items);
  a.n_q_heads = p->n_q_heads; a.n_kv_heads = p->n_kv_heads;
  a.scale_log2 = resolve_scale(p) * kLog2e;
  const int grid = (int)std::min<int64_t>(L.n_fwd_items, (int64_t)cu_count() * kFwdWgPerCu);
  if (p->head_dim == 128) hipLaunchKernelGGL(fwd_kernel<128>, dim3(grid), dim3(256), 0, (hipStream_t)stream, a);
  else hipLaunchKernelGGL(fwd_kernel<64>, dim3(grid), dim3(256), 0, (hipStream_t)stream, a);
  return check_launch("fcp_block_attn_fwd");
}

extern "C" int fcp_merge_partials(const fcp_problem* p, const float* o_part, const float* lse_part,
                                  void* o, float* lse, void* workspace, void* stream) {
  int rc = validate_problem(p);
  if (rc) return rc;
  WsLayout L;
  rc = compute_layout(p, &L);
  if (rc) return rc;
  if (L.n_merge_items == 0) return FCP_OK;
  if (!o || !lse || !workspace || (p->n_slots && (!o_part || !lse_part))) { set_error("fcp_merge_partials: NULL pointer"); return FCP_ERR_INVALID_ARG; }
  unsigned char* ws = static_cast<unsigned char*>(workspace);
  MergeArgs a;
  a.o_part = o_part; a.lse_part = lse_part; a.o = o; a.lse = lse;
  a.items = reinterpret_cast<const MergeItem*>(ws + L.off_merge_items);
  a.slot_rh = reinterpret_cast<const int32_t*>(ws + L.off_slot_rh);
  a.o_is_f32 = (p->flags & FCP_FLAG_O_F32) ? 1 : 0;
  if (p->head_dim == 128) hipLaunchKernelGGL(merge_kernel<128>, dim3((unsigned)L.n_merge_items), dim3(256), 0, (hipStream_t)stream, a);
  else hipLaunchKernelGGL(merge_kernel<64>, dim3((unsigned)L.n_merge_items), dim3(256), 0, (hipStream_t)stream, a);
  return check_launch("fcp_merge_partials");
}

extern "C" int fcp_bwd_preprocess(const fcp_problem* p, const void* o, const void* d_o, float* dq,
                                  void* workspace, void* stream) {
  int rc = validate_problem(p);
  if (rc) return rc;
  WsLayout L;
  rc = compute_layout(p, &L);
  if (rc) return rc;
  const int64_t n_rh = L.t_q * p->n_q_heads;
  if (n_rh == 0) return FCP_OK;
  if (!o || !d_o || !dq || !workspace) { set_error("fcp_bwd_preprocess: NULL pointer"); return FCP_ERR_INVALID_ARG; }
  hipStream_t st = (hipStream_t)stream;
  float* delta = reinterpret_cast<float*>(static_cast<unsigned char*>(workspace) + L.off_delta);
  const int o_f32 = (p->flags & FCP_FLAG_O_F32) ? 1 : 0;
  const int D = p->head_dim;
  // dQ is accumulated with atomics: clear it (a fill kernel, so the call can sit in a captured graph).
  const int64_t n4 = n_rh * D / 4;
  const int zgrid = (int)std::min<int64_t>((n4 + 255) / 256, (int64_t)cu_count() * 8);
  hipLaunchKernelGGL(zero_kernel, dim3(zgrid), dim3(256), 0, st, reinterpret_cast<f32x4*>(dq), n4);
  const int64_t blocks = (n_rh * (D / 8) + 255) / 256;
  if (D == 128) hipLaunchKernelGGL(delta_kernel<128>, dim3((unsigned)blocks), dim3(256), 0, st, o, o_f32, (const uint16_t*)d_o, delta, n_rh);
  else hipLaunchKernelGGL(delta_kernel<64>, dim3((unsigned)blocks), dim3(256), 0, st, o, o_f32, (const uint16_t*)d_o, delta, n_rh);
  return check_launch("fcp_bwd_preprocess");
}

extern "C" int fcp_block_attn_bwd_main(const fcp_problem* p, const void* q, const void* k, const void* v,
                                       const float* lse, const void* d_o,
                                       float* dq, float* dk, float* dv, void* workspace, void* stream) {
  int rc = validate_problem(p);
  if (rc) return rc;
  WsLayout L;
  rc = compute_layout(p, &L);
  if (rc) return rc;
  if (L.n_bwd_items == 0) return FCP_OK;
  if (!q || !k || !v || !lse || !d_o || !dq || !dk || !dv || !workspace) { set_error("fcp_block_attn_bwd_main: NULL pointer"); return FCP_ERR_INVALID_ARG; }
  unsigned char* ws = static_cast<unsigned char*>(workspace);
  BwdArgs a;
  a.q = (const uint16_t*)q; a.k = (const uint16_t*)k; a.v = (const uint16_t*)v; a.d_o = (const uint16_t*)d_o;
  a.lse = lse; a.delta = reinterpret_cast<const float*>(ws + L.off_delta); a.dq = dq; a.dk = dk; a.dv = dv;
  a.hdr = reinterpret_cast<WsHeader*>(ws);
  a.deps = reinterpret_cast<const BwdDep*>(ws + L.off_bwd_deps);
  a.items = reinterpret_cast<const BwdItem*>(ws + L.off_bwd_items);
  a.n_q_heads = p->n_q_heads; a.n_kv_heads = p->n_kv_heads;
  a.scale = resolve_scale(p); a.scale_log2 = a.scale * kLog2e;
  const int grid = (int)std::min<int64_t>(L.n_bwd_items, (int64_t)cu_count() * kBwdWgPerCu);
  if (p->head_dim == 128) hipLaunchKernelGGL(bwd_kernel<128>, dim3(grid), dim3(256), 0, (hipStream_t)stream, a);
  else hipLaunchKernelGGL(bwd_kernel<64>, dim3(grid), dim3(256), 0, (hipStream_t)stream, a);
  return check_launch("fcp_block_attn_bwd_main");
}

extern "C" int fcp_block_attn_bwd(const fcp_problem* p, const void* q, const void* k, const void* v,
                                  const void* o, const float* lse, const void* d_o,
                                  float* dq, float* dk, float* dv, void* workspace, void* stream) {
  if (!q || !k || !v || !o || !lse || !d_o || !dq || !dk || !dv || !workspace) {
    int rc = validate_problem(p);
    if (rc) return rc;
    set_error("fcp_block_attn_bwd: NULL pointer");
    return FCP_ERR_INVALID_ARG;
  }
  int rc = fcp_bwd_preprocess(p, o, d_o, dq, workspace, stream);
  if (rc) return rc;
  return fcp_block_attn_bwd_main(p, q, k, v, lse, d_o, dq, dk, dv, workspace, stream);
}
