// Measurement aids (fcp_probe.h): synthetic kernels that show what one unit of the chip sustains.  Nothing in the
// attention path calls them; bench.py reports them so that the design choices of the attention kernels can be
// checked against numbers measured on the machine they run on.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "fcp_internal.h"
#include "fcp_probe.h"

namespace fcp {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }
__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  f32x2 f = {a, b};
  bf16x2 h = __builtin_convertvector(f, bf16x2);
  return __builtin_bit_cast(uint32_t, h);
}

// Operand fragments of chosen values: 0 = zeros, 1 = every element 0.5, 2 = pseudo-random, close to N(0,1)
// (integer hash of (thread, fragment, element), then the sum of its four bytes).
__device__ __forceinline__ void make_operands(int kind, u32x4 (&fa)[8], u32x4 (&fb)[8]) {
#pragma unroll
  for (int i = 0; i < 16; i++) {
    u32x4 f = {0, 0, 0, 0};
#pragma unroll
    for (int e = 0; e < 4; e++) {
      float v[2] = {0.f, 0.f};
#pragma unroll
      for (int half = 0; half < 2; half++) {
        if (kind == 1) v[half] = 0.5f;
        if (kind == 2) {
          uint32_t h = ((threadIdx.x * 16u + i) * 8u + 2u * e + half) * 2654435761u;
          h ^= h >> 15; h *= 2246822519u; h ^= h >> 13; h *= 3266489917u; h ^= h >> 16;
          v[half] = ((float)((h & 255u) + ((h >> 8) & 255u) + ((h >> 16) & 255u) + (h >> 24)) - 510.f) * (1.f / 147.8f);
        }
      }
      f[e] = pack_bf16(v[0], v[1]);
    }
    if (i < 8) fa[i] = f; else fb[i - 8] = f;
  }
}

// A stream of back-to-back MFMAs on register operands, two waves per SIMD on every compute unit; VALU > 0 puts
// that many independent fp32 FMAs after every MFMA (the vector work that shares the SIMD's issue slots with it).
template <int VALU>
__global__ void __launch_bounds__(512, 2) mfma_probe_kernel(int kind, int iters, float* out) {
  u32x4 fa[8], fb[8];
  make_operands(kind, fa, fb);
  f32x16 acc[4];
#pragma unroll
  for (int j = 0; j < 4; j++)
#pragma unroll
    for (int r = 0; r < 16; r++) acc[j][r] = 0.f;
  float fill[8];
#pragma unroll
  for (int i = 0; i < 8; i++) fill[i] = 0.001f * (float)(threadIdx.x + i);
  for (int it = 0; it < iters; it++) {
#pragma unroll
    for (int m = 0; m < 16; m++) {
      acc[m & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(fa[m & 7]), as_bf16x8(fb[(m * 3) & 7]), acc[m & 3], 0, 0, 0);
#pragma unroll
      for (int v = 0; v < VALU; v++) {
        fill[v & 7] = __builtin_fmaf(fill[v & 7], 0.999f, 0.001f);
        asm volatile("" : "+v"(fill[v & 7]));       // stays where it was written: between the MFMAs
      }
      if (VALU > 0) __builtin_amdgcn_sched_barrier(0);
    }
    if ((it & 63) == 63) {      // random operands make the sums a random walk: keep them bounded
#pragma unroll
      for (int j = 0; j < 4; j++)
#pragma unroll
        for (int r = 0; r < 16; r++) acc[j][r] *= 0.125f;
    }
  }
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < 4; j++)
#pragma unroll
    for (int r = 0; r < 16; r++) s += acc[j][r];
  if (VALU > 0) {         // keeps the filler work alive; the plain MFMA stream's checksum stays the sum of its products
#pragma unroll
    for (int i = 0; i < 8; i++) s += fill[i] * 1e-30f;
  }
  s += __shfl_xor(s, 32, 64);
  if ((threadIdx.x & 63) == 0) out[blockIdx.x * 8 + (threadIdx.x >> 6)] = s;
}

// Raw LDS throughput of one compute unit for the access patterns of the attention kernels: every wave issues
// iters x 16 instructions of one kind on a 16 KB region (inline assembly: the compiler can neither drop nor merge them).
// MODE 0: ds_read_b128, lane = row of a swizzled 256-byte-row tile (the K / Q / dO row operands)
//      1: ds_read_b64_tr_b16 on the same tile (the transposed operands)     2: ds_write_b128, 16 B per lane, linear
//      3: ds_write_b64, 8 B per lane, linear                                 4: LDS-DMA, global_load_lds_dwordx4 from a
//         64 KB buffer that stays in the L2 cache (what a tile load costs the LDS, not the memory)
template <int MODE>
__global__ void __launch_bounds__(512) lds_probe_kernel(const unsigned char* src, int iters, float* out) {
  __shared__ __attribute__((aligned(1024))) unsigned char lds[65536];
  for (int i = threadIdx.x * 16; i < 65536; i += blockDim.x * 16) *reinterpret_cast<u32x4*>(lds + i) = u32x4{1, 2, 3, 4};
  __syncthreads();
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int l32 = lane & 31, g = lane >> 5;
  const int tr_row = (lane & 15) >> 2, tr_col = 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
  auto swz = [](int r) { return ((r & 3) << 2) | ((r >> 2) & 3); };
  auto toff = [&](int r, int c) { return r * 256 + ((c ^ swz(r)) << 4); };
  const uint32_t base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)lds + (wave & 3) * 16384;
  uint32_t ad;
  if (MODE == 0) ad = base + toff(l32, g);
  else if (MODE == 1) ad = base + toff(4 * g + tr_row, tr_col >> 3) + (tr_col & 4) * 2;
  else if (MODE == 3) ad = base + lane * 8;
  else ad = base + lane * 16;
  u32x4 acc = {0, 0, 0, 0};
  for (int it = 0; it < iters; it++) {
#pragma unroll
    for (int j = 0; j < 16; j++) {
      if (MODE == 0) {
        u32x4 y;
        asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(y) : "v"(ad), "n"((j & 7) * 1024));
        asm volatile("s_waitcnt lgkmcnt(8)" ::: "memory");
        acc[0] ^= y[0];
      } else if (MODE == 1) {
        u32x2 y;
        asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(y) : "v"(ad), "n"((j & 7) * 1024 + (j >> 3) * 2048 % 4096));
        asm volatile("s_waitcnt lgkmcnt(8)" ::: "memory");
        acc[0] ^= y[0];
      } else if (MODE == 2) {
        asm volatile("ds_write_b128 %0, %1 offset:%2" :: "v"(ad), "v"(acc), "n"(j * 1024) : "memory");
      } else if (MODE == 3) {
        u32x2 w = {acc[0], acc[1]};
        asm volatile("ds_write_b64 %0, %1 offset:%2" :: "v"(ad), "v"(w), "n"(j * 512) : "memory");
      } else {
        // 1 KB of consecutive LDS per instruction; m0 = wave-uniform LDS address
        const uint32_t m0 = __builtin_amdgcn_readfirstlane(base + j * 1024);
        const unsigned char* gp = src + ((wave * 16 + j) & 63) * 1024 + lane * 16;
        asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" :: "v"(gp), "s"(m0) : "memory", "m0");
        if (j == 15) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
      }
    }
  }
  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
  if (acc[0] == 0x12345678u) out[0] = 1.0f;
}

// fp32 atomic adds to memory in the pattern a KV-stationary backward would use to accumulate dQ: per wave and
// iteration, 16 rows of 32 consecutive floats (one accumulator tile), rows one token apart.
__global__ void __launch_bounds__(256) atomic_probe_kernel(float* buf, long n_rows, int row_stride, int iters) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const long base_row = ((long)blockIdx.x * 977) % (n_rows - 64);
  for (int it = 0; it < iters; it++) {
    float* dst = buf + (base_row + (it * 32) % 1024) % (n_rows - 64) * row_stride + wave * 32 + (lane & 31);
#pragma unroll
    for (int r = 0; r < 16; r++) {
      const int qr = 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
      unsafeAtomicAdd(dst + (long)qr * row_stride, 1.0f);
    }
  }
}

int n_cus() {
  int dev = 0, n = 0;
  if (hipGetDevice(&dev) != hipSuccess) return 256;
  if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
  return n;
}

int launched(const char* what) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) { set_error("%s: %s", what, hipGetErrorString(e)); return FCP_ERR_HIP; }
  return FCP_OK;
}

}  // namespace
}  // namespace fcp

using namespace fcp;

extern "C" int fcp_mfma_probe(int32_t operand_kind, int32_t iters, float* out, void* stream) {
  return fcp_mfma_valu_probe(operand_kind, 0, iters, out, stream);
}

extern "C" int fcp_mfma_valu_probe(int32_t operand_kind, int32_t valu_per_mfma, int32_t iters, float* out, void* stream) {
  if (!out || iters <= 0 || operand_kind < 0 || operand_kind > 2) {
    set_error("fcp_mfma_valu_probe: out must be non-NULL, iters > 0, operand_kind in 0..2");
    return FCP_ERR_INVALID_ARG;
  }
  void (*kern)(int, int, float*) = nullptr;
  switch (valu_per_mfma) {
    case 0: kern = mfma_probe_kernel<0>; break;
    case 2: kern = mfma_probe_kernel<2>; break;
    case 4: kern = mfma_probe_kernel<4>; break;
    case 6: kern = mfma_probe_kernel<6>; break;
    case 8: kern = mfma_probe_kernel<8>; break;
    case 12: kern = mfma_probe_kernel<12>; break;
    default: set_error("fcp_mfma_valu_probe: valu_per_mfma must be 0, 2, 4, 6, 8 or 12"); return FCP_ERR_INVALID_ARG;
  }
  hipLaunchKernelGGL(kern, dim3(n_cus()), dim3(512), 0, (hipStream_t)stream, (int)operand_kind, (int)iters, out);
  return launched("fcp_mfma_valu_probe");
}

extern "C" int fcp_lds_probe(int32_t mode, int32_t n_waves, int32_t iters, const void* src, float* out, void* stream) {
  if (!out || !src || iters <= 0 || mode < 0 || mode > 4 || (n_waves != 4 && n_waves != 8)) {
    set_error("fcp_lds_probe: mode in 0..4, n_waves 4 or 8, iters > 0, src (64 KB) and out non-NULL");
    return FCP_ERR_INVALID_ARG;
  }
  void (*kern)(const unsigned char*, int, float*) =
      mode == 0 ? lds_probe_kernel<0> : mode == 1 ? lds_probe_kernel<1> : mode == 2 ? lds_probe_kernel<2>
      : mode == 3 ? lds_probe_kernel<3> : lds_probe_kernel<4>;
  hipLaunchKernelGGL(kern, dim3(n_cus()), dim3(64 * n_waves), 0, (hipStream_t)stream, (const unsigned char*)src, (int)iters, out);
  return launched("fcp_lds_probe");
}

extern "C" int fcp_atomic_probe(float* buf, int64_t n_rows, int32_t row_stride, int32_t iters, int32_t workgroups_per_cu,
                                void* stream) {
  if (!buf || n_rows < 2048 || row_stride < 256 || iters <= 0 || workgroups_per_cu <= 0 || workgroups_per_cu > 8) {
    set_error("fcp_atomic_probe: buf non-NULL, n_rows >= 2048, row_stride >= 256 floats, iters > 0, workgroups_per_cu in 1..8");
    return FCP_ERR_INVALID_ARG;
  }
  hipLaunchKernelGGL(atomic_probe_kernel, dim3(n_cus() * workgroups_per_cu), dim3(256), 0, (hipStream_t)stream, buf,
                     (long)n_rows, (int)row_stride, (int)iters);
  return launched("fcp_atomic_probe");
}
