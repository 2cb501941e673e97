// samkv_topk_select: per (document, KV head) row of scores, the positions of the k largest scores
// (Sec. 3.2 with a fixed budget), initial/local positions forced in, output ascending by position.
//
// One workgroup per row; the whole row lives in registers (E keys per thread, thread t owns the
// contiguous positions [t*E, t*E+E) so that the output comes out in position order).
//   1. keys: float -> order-preserving uint32; forced positions get the largest key.
//   2. radix select of the k-th largest key, one bit per pass from the top: each wave counts its
//      candidates with that bit set by ballot + popcount, the counts meet in LDS (double-buffered,
//      one barrier per pass).  No atomics, so no contention on the few exponent values real scores
//      share, and a fixed number of passes whatever the distribution.
//   3. kept = key > T, plus the first `need` positions with key == T (ties to the lower position);
//      a block-wide exclusive scan of the per-thread counts gives every thread its output offset.
#include "common.hpp"

namespace samkv {
namespace {

__device__ __forceinline__ uint32_t order_key(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u << 1) == 0u) u = 0u;  // -0 and +0 are one value: ties go by position, not by sign bit
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

template <int E, int NT>
__global__ __launch_bounds__(NT) void k_select(const float* scores, IntTable cu_len, IntTable cu_k, int total_len,
                                               int m_total, int n_ctx, int n_sink, int n_local, int32_t* idx,
                                               int32_t* cu_k_dev) {
  constexpr int NW = NT / 64;
  __shared__ uint32_t cnt[2][NW];
  __shared__ uint64_t wsum[NW];
  const int i = blockIdx.x, g = blockIdx.y, t = threadIdx.x, lane = t & 63, wave = t >> 6;
  if (cu_k_dev != nullptr && i == 0 && g == 0)
    for (int n = t; n <= n_ctx; n += NT) cu_k_dev[n] = cu_k.v[n];
  const int L = cu_len.v[i + 1] - cu_len.v[i];
  const int k = cu_k.v[i + 1] - cu_k.v[i];
  const float* row = scores + (size_t)g * total_len + cu_len.v[i];
  int32_t* out = idx + (size_t)g * m_total + cu_k.v[i];

  uint32_t key[E];
  const int p0 = t * E;
  if (E % 4 == 0 && (((uintptr_t)row) & 15) == 0 && p0 + E <= L) {
#pragma unroll
    for (int e = 0; e < E; e += 4) {
      f32x4 x = *reinterpret_cast<const f32x4*>(row + p0 + e);
#pragma unroll
      for (int c = 0; c < 4; ++c) key[e + c] = order_key(x[c]);
    }
  } else {
#pragma unroll
    for (int e = 0; e < E; ++e) key[e] = (p0 + e < L) ? order_key(row[p0 + e]) : 0u;
  }
#pragma unroll
  for (int e = 0; e < E; ++e) {
    const int p = p0 + e;
    if (p < L && (p < n_sink || p >= L - n_local)) key[e] = 0xFFFFFFFFu;
  }

  // ---- k-th largest key, bit by bit ------------------------------------------------------------
  uint32_t prefix = 0;
  uint32_t kk = (uint32_t)k;
  for (int b = 31; b >= 0; --b) {
    // candidate: agrees with the decided bits above b and has bit b set (padding keys are 0: never)
    const uint32_t want = (prefix >> b) | 1u;
    uint32_t c = 0;
#pragma unroll
    for (int e = 0; e < E; ++e) c += __popcll(__ballot((key[e] >> b) == want));
    if (lane == 0) cnt[b & 1][wave] = c;
    __syncthreads();
    uint32_t tot = 0;
#pragma unroll
    for (int w = 0; w < NW; ++w) tot += cnt[b & 1][w];
    if (tot >= kk) prefix |= (1u << b); else kk -= tot;
  }
  const uint32_t T = prefix;
  const uint32_t need = kk;  // how many positions with key == T are kept

  // ---- ordered compaction ------------------------------------------------------------------------
  uint32_t n_gt = 0, n_eq = 0;
#pragma unroll
  for (int e = 0; e < E; ++e) {
    const bool ok = p0 + e < L;
    n_gt += (ok && key[e] > T) ? 1u : 0u;
    n_eq += (ok && key[e] == T) ? 1u : 0u;
  }
  // both counts can reach 65536 (a full-length row of equal keys kept whole): 32 bits each
  uint64_t packed = (uint64_t)n_gt | ((uint64_t)n_eq << 32);
  uint64_t incl = packed;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    uint64_t o = __shfl_up(incl, off);
    if (lane >= off) incl += o;
  }
  if (lane == 63) wsum[wave] = incl;
  __syncthreads();
  uint64_t base = 0;
#pragma unroll
  for (int w = 0; w < NW; ++w) base += (w < wave) ? wsum[w] : 0ull;
  const uint64_t excl = base + incl - packed;
  uint32_t gt_before = (uint32_t)excl, eq_before = (uint32_t)(excl >> 32);
#pragma unroll
  for (int e = 0; e < E; ++e) {
    if (p0 + e < L) {
      const bool is_eq = key[e] == T;
      const bool take = key[e] > T || (is_eq && eq_before < need);
      if (take) {
        const uint32_t pos = gt_before + (eq_before < need ? eq_before : need);
        out[pos] = p0 + e;
      }
      gt_before += key[e] > T ? 1u : 0u;
      eq_before += is_eq ? 1u : 0u;
    }
  }
}

template <int E, int NT>
hipError_t run(const SelectLaunch& a, const IntTable& cu_len, const IntTable& cu_k, hipStream_t s) {
  hipLaunchKernelGGL((k_select<E, NT>), dim3(a.n_ctx, a.hkv), dim3(NT), 0, s, a.scores, cu_len, cu_k, a.total_len,
                     a.m_total, a.n_ctx, a.n_sink, a.n_local, a.idx, a.cu_k_dev);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_select(const SelectLaunch& a, const IntTable& cu_len, const IntTable& cu_k, hipStream_t s) {
  // few waves per row keep the 32 barrier rounds short; many rows share a compute unit instead
  if (a.max_len <= 1024) return run<4, 256>(a, cu_len, cu_k, s);
  if (a.max_len <= 4096) return run<16, 256>(a, cu_len, cu_k, s);
  if (a.max_len <= 16384) return run<16, 1024>(a, cu_len, cu_k, s);
  return run<64, 1024>(a, cu_len, cu_k, s);
}

}  // namespace samkv
