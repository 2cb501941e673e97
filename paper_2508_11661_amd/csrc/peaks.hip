// Two micro-kernels that measure what THIS device sustains, so that the benchmark can quote a kernel's rate
// against the measured ceiling as well as against the published one:
//   k_peak_mfma   nothing but independent v_mfma_f32_32x32x16_bf16 instructions (the product the attention kernels
//                 are built on), four accumulators per wave so that the matrix pipe never waits on a result
//   k_peak_copy   a plain streaming copy, 16 bytes per lane, non-temporal
//   k_peak_read   a plain streaming read (what the score kernels do to K)
// Neither is part of the method; the benchmark times the launches with HIP events.
#include "common.hpp"

namespace samkv {
namespace {

// operand pattern: 0 small integers (a few mantissa bits set), 1 zeros, 2 pseudo-random values in [-2, 2) with full
// mantissas.  The pattern matters: the matrix unit's power grows with the number of bits that toggle, and under
// sustained load the device lowers its clock to stay inside its power limit, so the rate with realistic operands
// (2) is the ceiling a kernel that multiplies real data can be measured against.
__device__ __forceinline__ uint32_t mix32(uint32_t x) {
  x ^= x >> 16; x *= 0x7feb352dU; x ^= x >> 15; x *= 0x846ca68bU; x ^= x >> 16;
  return x;
}

__global__ __launch_bounds__(256) void k_peak_mfma(float* sink, int iters, int pattern) {
  bf16x8 a[4], b[4];
#pragma unroll
  for (int v = 0; v < 4; ++v)
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      float fa = 0.f, fb = 0.f;
      if (pattern == 0) {
        fa = (float)((threadIdx.x + e) & 3);
        fb = (float)((threadIdx.x * 3 + e) & 1);
      } else if (pattern == 2) {
        fa = ((int)(mix32(threadIdx.x * 64 + v * 8 + e + 1) & 0xFFFF) - 32768) / 16384.f;
        fb = ((int)(mix32(threadIdx.x * 64 + v * 8 + e + 7777) & 0xFFFF) - 32768) / 16384.f;
      }
      a[v][e] = (__bf16)fa;
      b[v][e] = (__bf16)fb;
    }
  f32x16 acc[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 16; ++j) acc[i][j] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int i = 0; i < 4; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[(u + i) & 3], b[u], acc[i], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 16; ++j) s += acc[i][j];
  if (s == 12345.678f) sink[0] = s;  // keeps the loop alive; practically never true
}

__global__ __launch_bounds__(256) void k_peak_copy(const u32x4* src, u32x4* dst, size_t n16) {
  const size_t stride = (size_t)gridDim.x * 256 * 4;
  for (size_t i = (size_t)blockIdx.x * 256 * 4 + threadIdx.x; i < n16; i += stride) {
    u32x4 x[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const size_t j = i + (size_t)u * 256;
      x[u] = __builtin_nontemporal_load(src + (j < n16 ? j : n16 - 1));
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const size_t j = i + (size_t)u * 256;
      if (j < n16) __builtin_nontemporal_store(x[u], dst + j);
    }
  }
}

// a plain streaming read: every 16-byte chunk loaded once, folded into one word per lane (kept alive by a
// comparison that never holds)
__global__ __launch_bounds__(256) void k_peak_read(const u32x4* src, size_t n16, uint32_t* sink) {
  const size_t stride = (size_t)gridDim.x * 256 * 8;
  uint32_t acc = 0;
  for (size_t i = (size_t)blockIdx.x * 256 * 8 + threadIdx.x; i < n16; i += stride) {
    u32x4 x[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const size_t j = i + (size_t)u * 256;
      x[u] = __builtin_nontemporal_load(src + (j < n16 ? j : n16 - 1));
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) acc ^= x[u][0] ^ x[u][1] ^ x[u][2] ^ x[u][3];
  }
  if (acc == 0x9E3779B9u) sink[0] = acc;
}

}  // namespace

hipError_t launch_peak_read(const void* src, size_t bytes, uint32_t* sink, hipStream_t s) {
  const size_t n16 = bytes / 16;
  size_t blocks = (n16 + 2047) / 2048;
  if (blocks > 256 * 32) blocks = 256 * 32;
  hipLaunchKernelGGL(k_peak_read, dim3((unsigned)blocks), dim3(256), 0, s, static_cast<const u32x4*>(src), n16, sink);
  return hipGetLastError();
}

// flop of one launch: n_blocks * 4 waves * iters * 16 instructions * 32768
hipError_t launch_peak_mfma(float* sink, int n_blocks, int iters, int pattern, hipStream_t s) {
  hipLaunchKernelGGL(k_peak_mfma, dim3(n_blocks), dim3(256), 0, s, sink, iters, pattern);
  return hipGetLastError();
}

hipError_t launch_peak_copy(const void* src, void* dst, size_t bytes, hipStream_t s) {
  const size_t n16 = bytes / 16;
  size_t blocks = (n16 + 1023) / 1024;
  if (blocks > 256 * 32) blocks = 256 * 32;
  hipLaunchKernelGGL(k_peak_copy, dim3((unsigned)blocks), dim3(256), 0, s, static_cast<const u32x4*>(src),
                     static_cast<u32x4*>(dst), n16);
  return hipGetLastError();
}

}  // namespace samkv
