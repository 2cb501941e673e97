// Block-level retrieval (Sec. 3.2): the cache is managed in blocks of consecutive tokens, a block is represented
// by the mean of its keys, the first and last blocks of a document are always kept, and after the per-document
// selection a second filter compares the retrieved blocks of all documents on normalised scores.
//
// Everything here is small index and score bookkeeping around the row selection kernel (select.hip), which is
// reused unchanged: once per document on the block scores, once on the normalised scores of all candidates.
#include "common.hpp"

namespace samkv {
namespace {

template <int CTRL>
__device__ __forceinline__ float dpp_mv(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, true));
}

// Block score = mean of the token scores of the block: the inner product is linear, so the score of the mean key
// is the mean of the inner products that samkv_score already wrote.  16 lanes per block, fixed summation order
// inside a lane and a DPP tree across lanes.
__global__ __launch_bounds__(256) void k_block_scores(const float* scores, IntTable cu_len, IntTable cu_blk, int total_len,
                                                      int total_blk, int block, float* bscores) {
  const int i = blockIdx.y, g = blockIdx.z;
  const int L = cu_len.v[i + 1] - cu_len.v[i];
  const int nb = cu_blk.v[i + 1] - cu_blk.v[i];
  const int b = blockIdx.x * 16 + (threadIdx.x >> 4), sub = threadIdx.x & 15;
  if (b >= nb) return;  // whole 16-lane groups leave together; the DPP steps below stay inside a group
  const float* row = scores + (size_t)g * total_len + cu_len.v[i];
  const int t0 = b * block, t1 = min(L, t0 + block);
  float acc = 0.f;
  for (int t = t0 + sub; t < t1; t += 16) acc += row[t];
  acc += dpp_mv<0xB1>(acc);   // quad_perm [1,0,3,2]
  acc += dpp_mv<0x4E>(acc);   // quad_perm [2,3,0,1]
  acc += dpp_mv<0x141>(acc);  // row_half_mirror
  acc += dpp_mv<0x140>(acc);  // row_mirror
  if (sub == 0) bscores[(size_t)g * total_blk + cu_blk.v[i] + b] = acc / (float)(t1 - t0);
}

// Kept blocks (ascending block ids, per document and KV head) -> kept token positions.  Only a document's last
// block can be short, and it is last among the kept ones, so the t-th kept block starts at token offset t * block.
__global__ __launch_bounds__(256) void k_expand_blocks(const int32_t* bidx, IntTable cu_len, IntTable cu_kb, IntTable cu_k,
                                                       int total_kb, int m_total, int n_ctx, int block, int32_t* idx,
                                                       int32_t* cu_k_dev) {
  const int i = blockIdx.y, g = blockIdx.z;
  if (cu_k_dev != nullptr && i == 0 && g == 0 && blockIdx.x == 0)
    for (int n = threadIdx.x; n <= n_ctx; n += 256) cu_k_dev[n] = cu_k.v[n];
  const int L = cu_len.v[i + 1] - cu_len.v[i];
  const int k_i = cu_k.v[i + 1] - cu_k.v[i];
  const int r = blockIdx.x * 256 + threadIdx.x;
  if (r >= k_i) return;
  const int t = r / block, e = r - t * block;
  const int b = bidx[(size_t)g * total_kb + cu_kb.v[i] + t];
  const int pos = b * block + e;
  idx[(size_t)g * m_total + cu_k.v[i] + r] = pos < L ? pos : L - 1;
}

// Second filter, step 1: per document and KV head, min-max normalise the scores of the retrieved middle blocks;
// forced blocks get +inf so that the selection over all candidates keeps them whatever their score.
__global__ __launch_bounds__(256) void k_normalize(const float* bscores, const int32_t* bidx, IntTable cu_blk, IntTable cu_kb,
                                                   int total_blk, int total_kb, int n_init, int n_local, float* cand) {
  __shared__ float s_mn[4], s_mx[4];
  const int i = blockIdx.x, g = blockIdx.y, t0 = threadIdx.x;
  const int nb = cu_blk.v[i + 1] - cu_blk.v[i];
  const int kb = cu_kb.v[i + 1] - cu_kb.v[i];
  const float* brow = bscores + (size_t)g * total_blk + cu_blk.v[i];
  const int32_t* ids = bidx + (size_t)g * total_kb + cu_kb.v[i];
  float* out = cand + (size_t)g * total_kb + cu_kb.v[i];
  float mn = INFINITY, mx = -INFINITY;
  for (int t = t0; t < kb; t += 256) {
    const int b = ids[t];
    if (b >= n_init && b < nb - n_local) {
      const float s = brow[b];
      mn = fminf(mn, s);
      mx = fmaxf(mx, s);
    }
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    mn = fminf(mn, __shfl_xor(mn, off));
    mx = fmaxf(mx, __shfl_xor(mx, off));
  }
  if ((t0 & 63) == 0) { s_mn[t0 >> 6] = mn; s_mx[t0 >> 6] = mx; }
  __syncthreads();
  mn = fminf(fminf(s_mn[0], s_mn[1]), fminf(s_mn[2], s_mn[3]));
  mx = fmaxf(fmaxf(s_mx[0], s_mx[1]), fmaxf(s_mx[2], s_mx[3]));
  const float range = mx - mn;
  for (int t = t0; t < kb; t += 256) {
    const int b = ids[t];
    const bool mid = b >= n_init && b < nb - n_local;
    out[t] = !mid ? INFINITY : (range > 0.f ? (brow[b] - mn) / range : 1.f);
  }
}

// Second filter, step 3: the kept candidates (ascending positions in the candidate row) -> for each, its first
// global token position and the offset of its tokens in the output row (exclusive scan of the block sizes).
// One workgroup per KV head.
__global__ __launch_bounds__(1024) void k_filter_offsets(const int32_t* sel, const int32_t* bidx, IntTable cu_len,
                                                         IntTable cu_kb, int n_ctx, int total_kb, int n_sel, int block,
                                                         int32_t* start, int32_t* tok_off) {
  __shared__ int s_cu_kb[SAMKV_MAX_CTX + 1], s_cu_len[SAMKV_MAX_CTX + 1];
  __shared__ int s_wave[16];
  const int g = blockIdx.x, t = threadIdx.x, lane = t & 63, wave = t >> 6;
  for (int n = t; n <= n_ctx; n += 1024) { s_cu_kb[n] = cu_kb.v[n]; s_cu_len[n] = cu_len.v[n]; }
  __syncthreads();
  const int per = (n_sel + 1023) / 1024;
  const int j0 = t * per, j1 = min(n_sel, j0 + per);
  const int32_t* srow = sel + (size_t)g * n_sel;
  const int32_t* brow = bidx + (size_t)g * total_kb;
  auto entry = [&](int j, int* first) -> int {
    const int c = srow[j];
    int lo = 0, hi = n_ctx;  // document with cu_kb[doc] <= c < cu_kb[doc + 1]
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (s_cu_kb[mid] <= c) lo = mid; else hi = mid;
    }
    const int L = s_cu_len[lo + 1] - s_cu_len[lo];
    const int b = brow[c];
    *first = s_cu_len[lo] + b * block;
    return min(block, L - b * block);
  };
  int sum = 0, first;
  for (int j = j0; j < j1; ++j) sum += entry(j, &first);
  int incl = sum;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int o = __shfl_up(incl, off);
    if (lane >= off) incl += o;
  }
  if (lane == 63) s_wave[wave] = incl;
  __syncthreads();
  int base = 0;
#pragma unroll
  for (int w = 0; w < 16; ++w) base += (w < wave) ? s_wave[w] : 0;
  int off = base + incl - sum;
  for (int j = j0; j < j1; ++j) {
    const int size = entry(j, &first);
    start[(size_t)g * n_sel + j] = first;
    tok_off[(size_t)g * n_sel + j] = off;
    off += size;
  }
}

// Second filter, step 4: one wave per kept block writes the global positions of its tokens.
__global__ __launch_bounds__(256) void k_filter_expand(const int32_t* start, const int32_t* tok_off, int n_sel, int m_total,
                                                       int32_t* gidx) {
  const int g = blockIdx.y, j = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (j >= n_sel) return;
  const int off = tok_off[(size_t)g * n_sel + j];
  const int end = j + 1 < n_sel ? tok_off[(size_t)g * n_sel + j + 1] : m_total;
  const int first = start[(size_t)g * n_sel + j];
  for (int e = lane; off + e < end; e += 64) gidx[(size_t)g * m_total + off + e] = first + e;
}

int max_span(const IntTable& cu, int n) {
  int m = 0;
  for (int i = 0; i < n; ++i) m = cu.v[i + 1] - cu.v[i] > m ? cu.v[i + 1] - cu.v[i] : m;
  return m;
}

}  // namespace

hipError_t launch_block_scores(const float* scores, const IntTable& cu_len, const IntTable& cu_blk, int n_ctx, int hkv,
                               int total_len, int block, float* bscores, hipStream_t s) {
  hipLaunchKernelGGL(k_block_scores, dim3((max_span(cu_blk, n_ctx) + 15) / 16, n_ctx, hkv), dim3(256), 0, s, scores,
                     cu_len, cu_blk, total_len, cu_blk.v[n_ctx], block, bscores);
  return hipGetLastError();
}

hipError_t launch_expand_blocks(const int32_t* bidx, const IntTable& cu_len, const IntTable& cu_kb, const IntTable& cu_k,
                                int n_ctx, int hkv, int block, int32_t* idx, int32_t* cu_k_dev, hipStream_t s) {
  const int max_k = max_span(cu_k, n_ctx);
  hipLaunchKernelGGL(k_expand_blocks, dim3(max_k > 0 ? (max_k + 255) / 256 : 1, n_ctx, hkv), dim3(256), 0, s, bidx, cu_len,
                     cu_kb, cu_k, cu_kb.v[n_ctx], cu_k.v[n_ctx], n_ctx, block, idx, cu_k_dev);
  return hipGetLastError();
}

hipError_t launch_normalize(const float* bscores, const int32_t* bidx, const IntTable& cu_blk, const IntTable& cu_kb,
                            int n_ctx, int hkv, int n_init, int n_local, float* cand, hipStream_t s) {
  hipLaunchKernelGGL(k_normalize, dim3(n_ctx, hkv), dim3(256), 0, s, bscores, bidx, cu_blk, cu_kb, cu_blk.v[n_ctx],
                     cu_kb.v[n_ctx], n_init, n_local, cand);
  return hipGetLastError();
}

hipError_t launch_filter_expand(const int32_t* sel, const int32_t* bidx, const IntTable& cu_len, const IntTable& cu_kb,
                                int n_ctx, int hkv, int n_sel, int m_total, int block, int32_t* start, int32_t* tok_off,
                                int32_t* gidx, hipStream_t s) {
  hipLaunchKernelGGL(k_filter_offsets, dim3(hkv), dim3(1024), 0, s, sel, bidx, cu_len, cu_kb, n_ctx, cu_kb.v[n_ctx], n_sel,
                     block, start, tok_off);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(k_filter_expand, dim3((n_sel + 3) / 4, hkv), dim3(256), 0, s, start, tok_off, n_sel, m_total, gidx);
  return hipGetLastError();
}

}  // namespace samkv
