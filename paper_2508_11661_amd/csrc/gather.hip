// samkv_gather: copy the kept K and V rows of every document into one compacted cache (Sec. 3.2:
// the filtered blocks of all documents are concatenated, in document order and original position
// order).  Pure data movement, HBM-bound: 2*d*e bytes read and 2*d*e written per kept token and KV
// head, plus the 4-byte index.
//
// A row is LPR 16-byte chunks; LPR lanes copy one K row and one V row, a wave copies 64/LPR rows per
// step and runs STEPS steps with all of its loads issued before the first store.  The grid is
// (row chunk, document, KV head), so the document's base pointers are uniform over a workgroup.
#include "common.hpp"

namespace samkv {
namespace {

template <int ROW_BYTES>
__global__ __launch_bounds__(256) void k_gather(PtrTable kt, PtrTable vt, IntTable cu_len, IntTable cu_k, int m_total,
                                                const int32_t* idx, char* k_c, char* v_c) {
  constexpr int LPR = ROW_BYTES / 16;
  constexpr int RPS = 64 / LPR;  // rows per wave step
  constexpr int STEPS = 8;
  constexpr int ROWS_PER_BLOCK = RPS * STEPS * 4;
  const int i = blockIdx.y, g = blockIdx.z;  // document and KV head are uniform over the block
  const int k_i = cu_k.v[i + 1] - cu_k.v[i];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int sub = lane % LPR, rg = lane / LPR;
  const int r0 = blockIdx.x * ROWS_PER_BLOCK + wave * (RPS * STEPS);
  if (r0 >= k_i) return;
  const int L = cu_len.v[i + 1] - cu_len.v[i];
  const char* ksrc = static_cast<const char*>(kt.p[i]) + (size_t)g * L * ROW_BYTES + sub * 16;
  const char* vsrc = static_cast<const char*>(vt.p[i]) + (size_t)g * L * ROW_BYTES + sub * 16;
  const size_t out0 = ((size_t)g * m_total + cu_k.v[i]) * ROW_BYTES + sub * 16;
  const int32_t* ip = idx + (size_t)g * m_total + cu_k.v[i];

  int p[STEPS];
#pragma unroll
  for (int s = 0; s < STEPS; ++s) {
    const int r = r0 + s * RPS + rg;
    p[s] = ip[r < k_i ? r : k_i - 1];
  }
  u32x4 xk[STEPS], xv[STEPS];
#pragma unroll
  for (int s = 0; s < STEPS; ++s) {
    const int q = p[s] < 0 ? 0 : (p[s] >= L ? L - 1 : p[s]);
    xk[s] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(ksrc + (size_t)q * ROW_BYTES));
    xv[s] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(vsrc + (size_t)q * ROW_BYTES));
  }
#pragma unroll
  for (int s = 0; s < STEPS; ++s) {
    const int r = r0 + s * RPS + rg;
    if (r < k_i) {
      __builtin_nontemporal_store(xk[s], reinterpret_cast<u32x4*>(k_c + out0 + (size_t)r * ROW_BYTES));
      __builtin_nontemporal_store(xv[s], reinterpret_cast<u32x4*>(v_c + out0 + (size_t)r * ROW_BYTES));
    }
  }
}

// Q-cache variant: one tensor, one row set per QUERY head h, indexed by the kept positions of its KV head
// h / group (the stored per-document Q cache supplies the query states of the kept tokens).
template <int ROW_BYTES>
__global__ __launch_bounds__(256) void k_gather_q(PtrTable qt, IntTable cu_len, IntTable cu_k, int m_total, int group,
                                                  const int32_t* idx, char* q_rec) {
  constexpr int LPR = ROW_BYTES / 16;
  constexpr int RPS = 64 / LPR;
  constexpr int STEPS = 8;
  constexpr int ROWS_PER_BLOCK = RPS * STEPS * 4;
  const int i = blockIdx.y, h = blockIdx.z, g = h / group;
  const int k_i = cu_k.v[i + 1] - cu_k.v[i];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int sub = lane % LPR, rg = lane / LPR;
  const int r0 = blockIdx.x * ROWS_PER_BLOCK + wave * (RPS * STEPS);
  if (r0 >= k_i) return;
  const int L = cu_len.v[i + 1] - cu_len.v[i];
  const char* src = static_cast<const char*>(qt.p[i]) + (size_t)h * L * ROW_BYTES + sub * 16;
  const size_t out0 = ((size_t)h * m_total + cu_k.v[i]) * ROW_BYTES + sub * 16;
  const int32_t* ip = idx + (size_t)g * m_total + cu_k.v[i];
  int p[STEPS];
#pragma unroll
  for (int s = 0; s < STEPS; ++s) {
    const int r = r0 + s * RPS + rg;
    p[s] = ip[r < k_i ? r : k_i - 1];
  }
  u32x4 x[STEPS];
#pragma unroll
  for (int s = 0; s < STEPS; ++s) {
    const int q = p[s] < 0 ? 0 : (p[s] >= L ? L - 1 : p[s]);
    x[s] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(src + (size_t)q * ROW_BYTES));
  }
#pragma unroll
  for (int s = 0; s < STEPS; ++s) {
    const int r = r0 + s * RPS + rg;
    if (r < k_i) __builtin_nontemporal_store(x[s], reinterpret_cast<u32x4*>(q_rec + out0 + (size_t)r * ROW_BYTES));
  }
}

// Gather by GLOBAL token positions (position in the concatenation of all documents): used after the cross-document
// block filter, where the number of tokens a document contributes differs from KV head to KV head.  One or two
// tensors per document ([heads][L_i][d] each); head h reads the positions of KV head h / group.  The document of a
// row is found by binary search in the prefix sums, staged in LDS together with the base pointers.
template <int ROW_BYTES, bool TWO>
__global__ __launch_bounds__(256) void k_gather_g(PtrTable at, PtrTable bt, IntTable cu_len, int n_ctx, int m_total,
                                                  int group, const int32_t* gidx, char* a_out, char* b_out) {
  constexpr int LPR = ROW_BYTES / 16;
  constexpr int RPS = 64 / LPR;
  constexpr int STEPS = 4;
  __shared__ int s_cu[SAMKV_MAX_CTX + 1];
  __shared__ const char* s_a[SAMKV_MAX_CTX];
  __shared__ const char* s_b[SAMKV_MAX_CTX];
  for (int n = threadIdx.x; n <= n_ctx; n += 256) s_cu[n] = cu_len.v[n];
  for (int n = threadIdx.x; n < n_ctx; n += 256) {
    s_a[n] = static_cast<const char*>(at.p[n]);
    if (TWO) s_b[n] = static_cast<const char*>(bt.p[n]);
  }
  __syncthreads();
  const int h = blockIdx.y, g = h / group;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int sub = lane % LPR, rg = lane / LPR;
  const int r0 = blockIdx.x * (RPS * STEPS * 4) + wave * (RPS * STEPS);
  if (r0 >= m_total) return;
  const int total_len = s_cu[n_ctx];
  const int32_t* ip = gidx + (size_t)g * m_total;
  const char* pa[STEPS];
  const char* pb[STEPS];
#pragma unroll
  for (int s = 0; s < STEPS; ++s) {
    const int r = r0 + s * RPS + rg;
    int gp = ip[r < m_total ? r : m_total - 1];
    gp = gp < 0 ? 0 : (gp >= total_len ? total_len - 1 : gp);
    int lo = 0, hi = n_ctx;  // document with cu_len[doc] <= gp < cu_len[doc + 1]
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (s_cu[mid] <= gp) lo = mid; else hi = mid;
    }
    const size_t L = s_cu[lo + 1] - s_cu[lo];
    const size_t off = ((size_t)h * L + (gp - s_cu[lo])) * ROW_BYTES + sub * 16;
    pa[s] = s_a[lo] + off;
    if (TWO) pb[s] = s_b[lo] + off;
  }
  u32x4 xa[STEPS], xb[STEPS];
#pragma unroll
  for (int s = 0; s < STEPS; ++s) {
    xa[s] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(pa[s]));
    if (TWO) xb[s] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(pb[s]));
  }
  const size_t out0 = (size_t)h * m_total * ROW_BYTES + sub * 16;
#pragma unroll
  for (int s = 0; s < STEPS; ++s) {
    const int r = r0 + s * RPS + rg;
    if (r < m_total) {
      __builtin_nontemporal_store(xa[s], reinterpret_cast<u32x4*>(a_out + out0 + (size_t)r * ROW_BYTES));
      if (TWO) __builtin_nontemporal_store(xb[s], reinterpret_cast<u32x4*>(b_out + out0 + (size_t)r * ROW_BYTES));
    }
  }
}

template <int ROW_BYTES>
hipError_t run_g(const PtrTable& a, const PtrTable* b, const IntTable& cu_len, int n_ctx, int heads, int group, int m_total,
                 const int32_t* gidx, void* a_out, void* b_out, hipStream_t s) {
  constexpr int ROWS_PER_BLOCK = (64 / (ROW_BYTES / 16)) * 4 * 4;
  dim3 grid((m_total + ROWS_PER_BLOCK - 1) / ROWS_PER_BLOCK, heads);
  if (b != nullptr)
    hipLaunchKernelGGL((k_gather_g<ROW_BYTES, true>), grid, dim3(256), 0, s, a, *b, cu_len, n_ctx, m_total, group, gidx,
                       static_cast<char*>(a_out), static_cast<char*>(b_out));
  else
    hipLaunchKernelGGL((k_gather_g<ROW_BYTES, false>), grid, dim3(256), 0, s, a, a, cu_len, n_ctx, m_total, group, gidx,
                       static_cast<char*>(a_out), static_cast<char*>(nullptr));
  return hipGetLastError();
}

template <int ROW_BYTES>
hipError_t run_q(const GatherLaunch& a, const PtrTable& q, const IntTable& cu_len, const IntTable& cu_k, int hq,
                 hipStream_t s) {
  constexpr int ROWS_PER_BLOCK = (64 / (ROW_BYTES / 16)) * 8 * 4;
  dim3 grid((a.max_k + ROWS_PER_BLOCK - 1) / ROWS_PER_BLOCK, a.n_ctx, hq);
  hipLaunchKernelGGL((k_gather_q<ROW_BYTES>), grid, dim3(256), 0, s, q, cu_len, cu_k, a.m_total, hq / a.hkv, a.idx,
                     static_cast<char*>(a.k_c));
  return hipGetLastError();
}

template <int ROW_BYTES>
hipError_t run(const GatherLaunch& a, const PtrTable& k, const PtrTable& v, const IntTable& cu_len,
               const IntTable& cu_k, hipStream_t s) {
  constexpr int ROWS_PER_BLOCK = (64 / (ROW_BYTES / 16)) * 8 * 4;
  dim3 grid((a.max_k + ROWS_PER_BLOCK - 1) / ROWS_PER_BLOCK, a.n_ctx, a.hkv);
  hipLaunchKernelGGL((k_gather<ROW_BYTES>), grid, dim3(256), 0, s, k, v, cu_len, cu_k, a.m_total, a.idx,
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

hipError_t launch_gather_g(int row_bytes, const PtrTable& a, const PtrTable* b, const IntTable& cu_len, int n_ctx, int heads,
                           int group, int m_total, const int32_t* gidx, void* a_out, void* b_out, hipStream_t s) {
  switch (row_bytes) {
    case 128: return run_g<128>(a, b, cu_len, n_ctx, heads, group, m_total, gidx, a_out, b_out, s);
    case 256: return run_g<256>(a, b, cu_len, n_ctx, heads, group, m_total, gidx, a_out, b_out, s);
    case 512: return run_g<512>(a, b, cu_len, n_ctx, heads, group, m_total, gidx, a_out, b_out, s);
  }
  return hipErrorInvalidValue;
}

hipError_t launch_gather_q(const GatherLaunch& a, const PtrTable& q, const IntTable& cu_len, const IntTable& cu_k,
                           int hq, hipStream_t s) {
  switch (a.row_bytes) {
    case 128: return run_q<128>(a, q, cu_len, cu_k, hq, s);
    case 256: return run_q<256>(a, q, cu_len, cu_k, hq, s);
    case 512: return run_q<512>(a, q, cu_len, cu_k, hq, s);
  }
  return hipErrorInvalidValue;
}

}  // namespace samkv
