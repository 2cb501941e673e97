// samkv_score_select: the inner products of a document's keys with its personalized query (Sec. 3.2) and the
// selection of the kept positions in ONE pass: a workgroup owns one (document, KV head) row, streams its K rows
// once, keeps the scores in LDS and selects from there.  The scores never travel to HBM and back (unless the caller
// asks for them), and the selection's barrier-bound passes of one workgroup overlap with the K streaming of its
// neighbours on the compute unit.  Both halves are the device functions the separate kernels use, so the kept
// positions are bit-identical to samkv_score followed by samkv_topk_select.
#include "common.hpp"
#include "kernels_core.hpp"

namespace samkv {
namespace {

// GATHER: the workgroup also copies the row's kept K and V rows into the compacted cache (samkv_gather's job for
// this document and KV head): the positions it has just written are read back after a workgroup-scope fence.
template <bool BF16, int D, int E, int NT, bool GATHER>
__global__ __launch_bounds__(NT) void k_score_select(PtrTable kt, PtrTable vt, IntTable cu_len, IntTable cu_k, const float* qsrc,
                                                     int heads, int group, int total_len, int m_total, int n_ctx, int n_sink,
                                                     int n_local, float* scores, int32_t* idx, int32_t* cu_k_dev, char* k_c,
                                                     char* v_c) {
  constexpr int EPL = BF16 ? 8 : 4;
  constexpr int LPR = D / EPL;
  constexpr int ROWS_PER_WAVE = (64 / LPR) * 8 * 2;
  constexpr int NW = NT / 64;
  constexpr size_t ROW_BYTES = (size_t)D * (BF16 ? 2 : 4);
  extern __shared__ float s_sc[];  // the row's scores
  __shared__ uint32_t cnt[2][NW];
  __shared__ uint64_t wsum[NW];
  const int i = blockIdx.x, g = blockIdx.y, t = threadIdx.x, lane = t & 63, wave = t >> 6;
  if (cu_k_dev != nullptr && i == 0 && g == 0)
    for (int n = t; n <= n_ctx; n += NT) cu_k_dev[n] = cu_k.v[n];
  const int L = cu_len.v[i + 1] - cu_len.v[i];
  const int k = cu_k.v[i + 1] - cu_k.v[i];
  const int sub = lane % LPR;

  float q[EPL];
  fold_query<EPL>(qsrc + ((size_t)i * heads + (size_t)g * group) * D + sub * EPL, D, group, q);
  const char* base = static_cast<const char*>(kt.p[i]) + (size_t)g * L * ROW_BYTES + sub * 16;
  for (int row0 = wave * ROWS_PER_WAVE; row0 < L; row0 += NW * ROWS_PER_WAVE)
    score_rows<BF16, D>(base, row0, L, q, [&](int row, float s) { s_sc[row] = s; });
  __syncthreads();
  if (scores != nullptr) {
    float* out = scores + (size_t)g * total_len + cu_len.v[i];
    for (int p = t; p < L; p += NT) out[p] = s_sc[p];
  }

  uint32_t key[E];
  const int p0 = t * E;
#pragma unroll
  for (int e = 0; e < E; ++e) key[e] = (p0 + e < L) ? order_key(s_sc[p0 + e]) : 0u;
  force_keys<E>(key, p0, L, n_sink, n_local);
  int32_t* ip = idx + (size_t)g * m_total + cu_k.v[i];
  select_from_keys<E, NT>(key, p0, L, k, ip, cnt, wsum);

  if (GATHER) {
    __threadfence_block();
    __syncthreads();
    // LPR lanes copy one K row and one V row; U rows per thread in flight
    constexpr int RPP = NT / LPR, U = 4;
    const int rg = t / LPR;
    const char* vsrc = static_cast<const char*>(vt.p[i]) + (size_t)g * L * ROW_BYTES + sub * 16;
    const size_t out0 = ((size_t)g * m_total + cu_k.v[i]) * ROW_BYTES + sub * 16;
    for (int r0 = rg; r0 < k; r0 += RPP * U) {
      u32x4 xk[U], xv[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int r = r0 + u * RPP;
        int pos = ip[r < k ? r : k - 1];
        pos = pos < 0 ? 0 : (pos >= L ? L - 1 : pos);
        xk[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(base + (size_t)pos * ROW_BYTES));
        xv[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(vsrc + (size_t)pos * ROW_BYTES));
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int r = r0 + u * RPP;
        if (r < k) {
          __builtin_nontemporal_store(xk[u], reinterpret_cast<u32x4*>(k_c + out0 + (size_t)r * ROW_BYTES));
          __builtin_nontemporal_store(xv[u], reinterpret_cast<u32x4*>(v_c + out0 + (size_t)r * ROW_BYTES));
        }
      }
    }
  }
}

template <bool BF16, int D, int E, int NT>
hipError_t run(const ScoreLaunch& a, const SelectLaunch& sl, const QuerySrc& q, const PtrTable& k, const IntTable& cu_len,
               const IntTable& cu_k, const GatherLaunch* ga, const PtrTable* v, hipStream_t s) {
  const size_t lds = (size_t)E * NT * sizeof(float);
  if (ga != nullptr)
    hipLaunchKernelGGL((k_score_select<BF16, D, E, NT, true>), dim3(a.n_ctx, a.hkv), dim3(NT), lds, s, k, *v, cu_len, cu_k, q.q,
                       q.heads, q.group, a.total_len, sl.m_total, a.n_ctx, sl.n_sink, sl.n_local, a.scores, sl.idx,
                       sl.cu_k_dev, static_cast<char*>(ga->k_c), static_cast<char*>(ga->v_c));
  else
    hipLaunchKernelGGL((k_score_select<BF16, D, E, NT, false>), dim3(a.n_ctx, a.hkv), dim3(NT), lds, s, k, k, cu_len, cu_k, q.q,
                       q.heads, q.group, a.total_len, sl.m_total, a.n_ctx, sl.n_sink, sl.n_local, a.scores, sl.idx,
                       sl.cu_k_dev, nullptr, nullptr);
  return hipGetLastError();
}

template <bool BF16, int D>
hipError_t run_len(const ScoreLaunch& a, const SelectLaunch& sl, const QuerySrc& q, const PtrTable& k,
                   const IntTable& cu_len, const IntTable& cu_k, const GatherLaunch* ga, const PtrTable* v, hipStream_t s) {
  // up to 4096 keys a row: 512 threads.  They halve the passes a wave makes over its share of the row's keys
  // (2.3 us less per call at 1024 keys, 4 % at 4096 keys than 256 threads); 1024 threads lose it again in the
  // selection's barriers.
  if (a.max_len <= 1024) return run<BF16, D, 2, 512>(a, sl, q, k, cu_len, cu_k, ga, v, s);
  if (a.max_len <= 4096) return run<BF16, D, 8, 512>(a, sl, q, k, cu_len, cu_k, ga, v, s);
  return run<BF16, D, 32, 256>(a, sl, q, k, cu_len, cu_k, ga, v, s);
}

}  // namespace

hipError_t launch_score_select(const ScoreLaunch& a, const SelectLaunch& sl, const PtrTable& k, const IntTable& cu_len,
                               const IntTable& cu_k, hipStream_t s, const GatherLaunch* ga, const PtrTable* v) {
  if (a.max_len > kFusedMaxLen) {  // rows too long for LDS: the separate kernels, through the caller's score buffer
    if (a.scores == nullptr) return hipErrorInvalidValue;
    hipError_t e = launch_score(a, k, cu_len, s);
    if (e == hipSuccess) e = launch_select(sl, cu_len, cu_k, s);
    if (e == hipSuccess && ga != nullptr) e = launch_gather(*ga, k, *v, cu_len, cu_k, s);
    return e;
  }
  QuerySrc q;
  hipError_t e = launch_score_prologue(a, s, &q);
  if (e != hipSuccess) return e;
  // With thousands of rows (many layers stacked as heads) the compaction is faster as its own streaming kernel
  // (0.84 against 0.91 ms at 5120 rows); below that the row's workgroup does it and a launch is saved.
  const GatherLaunch* in_kernel = (long long)a.n_ctx * a.hkv <= kFusedGatherMaxRows ? ga : nullptr;
  if (a.dtype == SAMKV_BF16)
    e = a.d == 128 ? run_len<true, 128>(a, sl, q, k, cu_len, cu_k, in_kernel, v, s)
                   : run_len<true, 64>(a, sl, q, k, cu_len, cu_k, in_kernel, v, s);
  else
    e = a.d == 128 ? run_len<false, 128>(a, sl, q, k, cu_len, cu_k, in_kernel, v, s)
                   : run_len<false, 64>(a, sl, q, k, cu_len, cu_k, in_kernel, v, s);
  if (e == hipSuccess && ga != nullptr && in_kernel == nullptr) e = launch_gather(*ga, k, *v, cu_len, cu_k, s);
  return e;
}

}  // namespace samkv
