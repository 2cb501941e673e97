// samkv_gather: copy the kept K and V rows of every document into one compacted cache (Sec. 3.2:
// the filtered blocks of all documents are concatenated, in document order and original position
// order).  Pure data movement, HBM-bound: 2*d*e bytes read and 2*d*e written per kept token and KV
// head, plus the 4-byte index.
//
// A row is LPR 16-byte chunks; LPR lanes copy one K row and one V row, a wave copies 64/LPR rows per
// step and runs STEPS steps with all of its loads issued before the first store.
#include "common.hpp"

namespace samkv {
namespace {

template <int ROW_BYTES>
__global__ __launch_bounds__(256) void k_gather(PtrTable kt, PtrTable vt, IntTable cu_len, IntTable cu_k, int n_ctx,
                                                int m_total, const int32_t* idx, char* k_c, char* v_c) {
  constexpr int LPR = ROW_BYTES / 16;
  constexpr int RPS = 64 / LPR;  // rows per wave step
  constexpr int STEPS = 4;
  constexpr int ROWS_PER_BLOCK = RPS * STEPS * 4;
  const int g = blockIdx.y;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int sub = lane % LPR, rg = lane / LPR;
  const int m0 = blockIdx.x * ROWS_PER_BLOCK + wave * (RPS * STEPS);

  u32x4 xk[STEPS], xv[STEPS];
#pragma unroll
  for (int s = 0; s < STEPS; ++s) {
    int m = m0 + s * RPS + rg;
    m = m < m_total ? m : m_total - 1;
    const int i = find_ctx(cu_k, n_ctx, m);
    const int L = cu_len.v[i + 1] - cu_len.v[i];
    int p = idx[(size_t)g * m_total + m];
    p = p < 0 ? 0 : (p >= L ? L - 1 : p);
    const size_t off = ((size_t)g * L + p) * ROW_BYTES + sub * 16;
    xk[s] = *reinterpret_cast<const u32x4*>(static_cast<const char*>(kt.p[i]) + off);
    xv[s] = *reinterpret_cast<const u32x4*>(static_cast<const char*>(vt.p[i]) + off);
  }
#pragma unroll
  for (int s = 0; s < STEPS; ++s) {
    const int m = m0 + s * RPS + rg;
    if (m < m_total) {
      const size_t off = ((size_t)g * m_total + m) * ROW_BYTES + sub * 16;
      __builtin_nontemporal_store(xk[s], reinterpret_cast<u32x4*>(k_c + off));
      __builtin_nontemporal_store(xv[s], reinterpret_cast<u32x4*>(v_c + off));
    }
  }
}

template <int ROW_BYTES>
hipError_t run(const GatherLaunch& a, const PtrTable& k, const PtrTable& v, const IntTable& cu_len,
               const IntTable& cu_k, hipStream_t s) {
  constexpr int ROWS_PER_BLOCK = (64 / (ROW_BYTES / 16)) * 4 * 4;
  dim3 grid((a.m_total + ROWS_PER_BLOCK - 1) / ROWS_PER_BLOCK, a.hkv);
  hipLaunchKernelGGL((k_gather<ROW_BYTES>), grid, dim3(256), 0, s, k, v, cu_len, cu_k, a.n_ctx, a.m_total, a.idx,
                     static_cast<char*>(a.k_c), static_cast<char*>(a.v_c));
  return hipGetLastError();
}

}  // namespace

hipError_t launch_gather(const GatherLaunch& a, const PtrTable& k, const PtrTable& v, const IntTable& cu_len,
                         const IntTable& cu_k, hipStream_t s) {
  switch (a.row_bytes) {
    case 128: return run<128>(a, k, v, cu_len, cu_k, s);
    case 256: return run<256>(a, k, v, cu_len, cu_k, s);
    case 512: return run<512>(a, k, v, cu_len, cu_k, s);
  }
  return hipErrorInvalidValue;
}

}  // namespace samkv
