// Preparation of V for the bf16 attention kernels (Sec. 3.3 attention, both entry points).
//
// The second product of the attention, O = P V, runs on the matrix cores with 16-bit operands.  Rounding the softmax
// weights P to bf16 (8-bit significand) costs 2^-9 of the spread of V per output, which an absolute bar on the
// output only survives while |V| stays of order 10.  The weights are therefore rounded to IEEE half precision
// (11-bit significand) instead, and V, whose bf16 values have 8-bit significands, is rewritten as half precision
// once per call: every KV head is scaled by a power of two that puts its largest magnitude into [2^14, 2^15), so no
// value overflows and a bf16 value down to 2^-32 of the head's maximum is still exact; the kernels undo the scale
// in their final normalisation.  Two small streaming launches:
//   k_v_absmax   largest |v| per (KV head, row chunk), as the integer bit pattern of the bf16 magnitude
//   k_v_to_f16   reduces a head's chunk maxima (every workgroup of the head does so redundantly), converts its own
//                row chunk, and workgroup 0 of the head writes the factor that undoes the scale
// Heads of at most kOneLaunchPieces 16-byte pieces (short compacted caches, where a launch costs more than the work)
// take ONE launch instead: k_v_prep_small, a few large workgroups per head, each of which finds the head's maximum
// itself (the head is read from L2 a few times over) and converts its share.
#include "common.hpp"

namespace samkv {
namespace {

constexpr int NT = 256;

__device__ __forceinline__ uint32_t block_max_u32(uint32_t x, uint32_t* lds) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) x = max(x, (uint32_t)__shfl_xor((int)x, off));
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  __syncthreads();  // a previous use of lds has been read by everyone
  if (lane == 0) lds[wave] = x;
  __syncthreads();
  return max(max(lds[0], lds[1]), max(lds[2], lds[3]));
}

// chunk c of a head covers 16-byte pieces [c * per, min(total, (c + 1) * per)) of its `total` pieces
__global__ __launch_bounds__(NT) void k_v_absmax(const u32x4* __restrict__ v, uint32_t* __restrict__ part, long long total,
                                                 long long per) {
  __shared__ uint32_t lds[4];
  const int c = blockIdx.x, g = blockIdx.y;
  const u32x4* src = v + (size_t)g * total;
  const long long begin = (long long)c * per, end = min(total, begin + per);
  uint32_t mx = 0;
  for (long long i = begin + threadIdx.x; i < end; i += NT) {
    const u32x4 w = __builtin_nontemporal_load(src + i);
#pragma unroll
    for (int e = 0; e < 4; ++e) mx = max(mx, max(w[e] & 0x7FFFu, (w[e] >> 16) & 0x7FFFu));
  }
  mx = block_max_u32(mx, lds);
  if (threadIdx.x == 0) part[(size_t)g * gridDim.x + c] = mx;
}

__global__ __launch_bounds__(NT) void k_v_to_f16(const u32x4* __restrict__ v, const uint32_t* __restrict__ part,
                                                 u32x4* __restrict__ v16, float* __restrict__ unscale, long long total,
                                                 long long per) {
  __shared__ uint32_t lds[4];
  const int c = blockIdx.x, g = blockIdx.y, n_chunks = gridDim.x;
  uint32_t mx = 0;
  for (int i = threadIdx.x; i < n_chunks; i += NT) mx = max(mx, part[(size_t)g * n_chunks + i]);
  mx = block_max_u32(mx, lds);
  // mx is the bf16 bit pattern of the head's largest magnitude: exponent field in bits 7..14.  The shift puts that
  // magnitude into [2^14, 2^15); it is kept inside +-113 so that both 2^shift and 2^-shift are normal floats.
  const int expo = (int)(mx >> 7) & 0xFF;
  int shift = expo == 0 ? 0 : 14 - (expo - 127);
  shift = max(-113, min(113, shift));
  if (c == 0 && threadIdx.x == 0) unscale[g] = __builtin_ldexpf(1.0f, -shift);
  const u32x4* src = v + (size_t)g * total;
  u32x4* dst = v16 + (size_t)g * total;
  const long long begin = (long long)c * per, end = min(total, begin + per);
  for (long long i = begin + threadIdx.x; i < end; i += NT) {
    const u32x4 w = __builtin_nontemporal_load(src + i);
    u32x4 o;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const f16x2 h = {(_Float16)__builtin_ldexpf(bf16_lo(w[e]), shift), (_Float16)__builtin_ldexpf(bf16_hi(w[e]), shift)};
      o[e] = __builtin_bit_cast(uint32_t, h);
    }
    dst[i] = o;
  }
}

// One launch for short heads: workgroup (c, g) scans ALL of head g for its largest magnitude, then converts chunk c.
constexpr int NT1 = 1024;
constexpr int kSmallChunk = 2048;   // 16-byte pieces converted per workgroup (32 KB)
__global__ __launch_bounds__(NT1) void k_v_prep_small(const u32x4* __restrict__ v, u32x4* __restrict__ v16,
                                                      float* __restrict__ unscale, int total, int per) {
  __shared__ uint32_t lds[NT1 / 64];
  const int c = blockIdx.x, g = blockIdx.y;
  const u32x4* src = v + (size_t)g * total;
  uint32_t mx = 0;
  constexpr int U = 16;  // loads in flight per thread: a head of 512 KB is two round trips
  for (int i = threadIdx.x; i < total; i += U * NT1) {
    u32x4 w[U];
#pragma unroll
    for (int u = 0; u < U; ++u) w[u] = src[min(i + u * NT1, total - 1)];
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int e = 0; e < 4; ++e) mx = max(mx, max(w[u][e] & 0x7FFFu, (w[u][e] >> 16) & 0x7FFFu));
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) mx = max(mx, (uint32_t)__shfl_xor((int)mx, off));
  if ((threadIdx.x & 63) == 0) lds[threadIdx.x >> 6] = mx;
  __syncthreads();
  mx = lds[0];
#pragma unroll
  for (int wv = 1; wv < NT1 / 64; ++wv) mx = max(mx, lds[wv]);
  const int expo = (int)(mx >> 7) & 0xFF;
  int shift = expo == 0 ? 0 : 14 - (expo - 127);
  shift = max(-113, min(113, shift));
  if (c == 0 && threadIdx.x == 0) unscale[g] = __builtin_ldexpf(1.0f, -shift);
  u32x4* dst = v16 + (size_t)g * total;
  const int begin = c * per, end = min(total, begin + per);
  // a chunk is at most kSmallChunk pieces: both loads of a thread are in flight together
  u32x4 w[kSmallChunk / NT1];
#pragma unroll
  for (int u = 0; u < kSmallChunk / NT1; ++u) w[u] = src[min(begin + (int)threadIdx.x + u * NT1, total - 1)];
#pragma unroll
  for (int u = 0; u < kSmallChunk / NT1; ++u) {
    const int i = begin + (int)threadIdx.x + u * NT1;
    u32x4 o;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const f16x2 h = {(_Float16)__builtin_ldexpf(bf16_lo(w[u][e]), shift), (_Float16)__builtin_ldexpf(bf16_hi(w[u][e]), shift)};
      o[e] = __builtin_bit_cast(uint32_t, h);
    }
    if (i < end) dst[i] = o;
  }
}

constexpr long long kOneLaunchPieces = 32768;  // 512 KB per head

}  // namespace

int v_prep_chunks(int n_kv, int m) {
  int by_rows = (m + 63) / 64;                 // at least 64 rows per chunk
  int by_grid = n_kv >= 2048 ? 1 : 2048 / n_kv;  // about 2048 workgroups per launch
  int n = by_rows < by_grid ? by_rows : by_grid;
  if (n > 1024) n = 1024;
  return n < 1 ? 1 : n;
}

hipError_t launch_v_prep(const void* v, int n_kv, int m, int d, void* v16, uint32_t* part, float* unscale, hipStream_t s) {
  const long long total = (long long)m * d * 2 / 16;  // 16-byte pieces per head
  if (total <= kOneLaunchPieces) {
    const int c1 = (int)((total + kSmallChunk - 1) / kSmallChunk);
    const int per1 = kSmallChunk;
    hipLaunchKernelGGL(k_v_prep_small, dim3(c1, n_kv), dim3(NT1), 0, s, static_cast<const u32x4*>(v),
                       static_cast<u32x4*>(v16), unscale, (int)total, per1);
    return hipGetLastError();
  }
  const int n_chunks = v_prep_chunks(n_kv, m);
  const long long per = (total + n_chunks - 1) / n_chunks;
  const dim3 grid(n_chunks, n_kv);
  hipLaunchKernelGGL(k_v_absmax, grid, dim3(NT), 0, s, static_cast<const u32x4*>(v), part, total, per);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(k_v_to_f16, grid, dim3(NT), 0, s, static_cast<const u32x4*>(v), part, static_cast<u32x4*>(v16), unscale,
                     total, per);
  return hipGetLastError();
}

}  // namespace samkv
