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
#include "kernels_core.hpp"

namespace samkv {
namespace {

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
  force_keys<E>(key, p0, L, n_sink, n_local);
  select_from_keys<E, NT>(key, p0, L, k, out, cnt, wsum);
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
