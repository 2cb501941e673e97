// samkv_score: personalized query vectors (Sec. 3.1, Eq. 1) and the inner product of every cached key
// with the vector of its own document (Sec. 3.2).
//
// Four launches on one stream:
//   k_pool    mean-pools the user query's Q rows (Q_que) and every document's local Q cache (Q_loc_j).
//   k_bias    per query head: |cos(Q_que, Q_loc_j)| for every j and the weighted sum over all documents.
//   k_qtilde  Eq. 1 for the query heads of a KV group, folded into one vector per document (the mean
//             over the group is linear, so one pass over K serves all heads of the group).
//   k_score   streams K once.  HBM-bound: d*e bytes read and 4 bytes written per token and KV head.
#include "common.hpp"

namespace samkv {
namespace {

template <int CTRL>
__device__ __forceinline__ float dpp_move(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, true));
}

// Sum over aligned groups of W lanes (W in {8, 16, 32}); every lane of a group ends with the total.
// After the quad steps the mirrors pair lanes that already hold equal partial sums.
template <int W>
__device__ __forceinline__ float group_sum(float v) {
  v += dpp_move<0xB1>(v);   // quad_perm [1,0,3,2]
  v += dpp_move<0x4E>(v);   // quad_perm [2,3,0,1]
  v += dpp_move<0x141>(v);  // row_half_mirror: lane i <-> 7 - i
  if (W >= 16) v += dpp_move<0x140>(v);  // row_mirror: lane i <-> 15 - i
  if (W >= 32) v += __int_as_float(__builtin_amdgcn_ds_swizzle(__float_as_int(v), 0x401F));  // lane ^ 16
  return v;
}

template <bool BF16>
__device__ __forceinline__ void unpack16(const u32x4& x, float* f) {
  if (BF16) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      f[2 * e] = bf16_lo(x[e]);
      f[2 * e + 1] = bf16_hi(x[e]);
    }
  } else {
#pragma unroll
    for (int e = 0; e < 4; ++e) f[e] = __uint_as_float(x[e]);
  }
}

// Mean over `n_rows` rows of D channels starting at `src` (row-major, 16-byte loads); the result
// lands in dst[0..D) (shared memory).  `red` is scratch of (256 / LPR) * D floats.  Fixed order.
template <bool BF16, int D>
__device__ void pool_rows(const void* src, int n_rows, float* red, float* dst) {
  constexpr int EPL = BF16 ? 8 : 4;
  constexpr int LPR = D / EPL;
  constexpr int RPB = 256 / LPR;
  constexpr int ROW_BYTES = D * (BF16 ? 2 : 4);
  const int t = threadIdx.x, sub = t % LPR, rg = t / LPR;
  float acc[EPL];
#pragma unroll
  for (int e = 0; e < EPL; ++e) acc[e] = 0.f;
  for (int r = rg; r < n_rows; r += RPB) {
    u32x4 x = *reinterpret_cast<const u32x4*>(static_cast<const char*>(src) + (size_t)r * ROW_BYTES + sub * 16);
    float f[EPL];
    unpack16<BF16>(x, f);
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[e] += f[e];
  }
#pragma unroll
  for (int e = 0; e < EPL; ++e) red[rg * D + sub * EPL + e] = acc[e];
  __syncthreads();
  if (t < D) {
    float s = 0.f;
    for (int r = 0; r < RPB; ++r) s += red[r * D + t];
    dst[t] = s / (float)n_rows;
  }
  __syncthreads();
}

// blockIdx.y == 0 pools the user query's rows of head h (Q_que); blockIdx.y == j + 1 pools document j's
// local Q cache (Q_loc_j).  Every input row is read exactly once.
template <bool BF16, int D>
__global__ __launch_bounds__(256) void k_pool(const void* q_tok, int n_q_tok, const void* q_loc, int w_loc,
                                              int hq, float* que, float* loc) {
  constexpr int EPL = BF16 ? 8 : 4;
  constexpr int RPB = 256 / (D / EPL);
  constexpr size_t ESZ = BF16 ? 2 : 4;
  __shared__ float red[RPB * D];
  __shared__ float s_out[D];
  const int h = blockIdx.x;
  if (blockIdx.y == 0) {
    pool_rows<BF16, D>(static_cast<const char*>(q_tok) + (size_t)h * n_q_tok * D * ESZ, n_q_tok, red, s_out);
    if (threadIdx.x < D) que[h * D + threadIdx.x] = s_out[threadIdx.x];
  } else {
    const int j = blockIdx.y - 1;
    pool_rows<BF16, D>(static_cast<const char*>(q_loc) + ((size_t)j * hq + h) * w_loc * D * ESZ, w_loc, red, s_out);
    if (threadIdx.x < D) loc[((size_t)j * hq + h) * D + threadIdx.x] = s_out[threadIdx.x];
  }
}

// One block per query head h.  Step 1: w_j[h] = |cos(Q_que[h], Q_loc_j[h])| for every document j (one
// wave per j, butterfly sums).  Step 2: bias[h][c] = sum_j w_j[h] Q_loc_j[h][c]; thread (channel c,
// slice s) adds the documents j = s, s + NS, ..., and the slices meet in LDS in a fixed order.
__global__ __launch_bounds__(1024) void k_bias(const float* que, const float* loc, float* wgt, float* bias, int n_ctx,
                                               int hq, int d) {
  __shared__ float red[1024];
  __shared__ float w_s[SAMKV_MAX_CTX];
  const int h = blockIdx.x, t = threadIdx.x, lane = t & 63, wave = t >> 6;
  for (int j = wave; j < n_ctx; j += 16) {
    float dot = 0.f, na = 0.f, nb = 0.f;
    for (int c = lane; c < d; c += 64) {
      const float a = que[h * d + c], b = loc[((size_t)j * hq + h) * d + c];
      dot = fmaf(a, b, dot); na = fmaf(a, a, na); nb = fmaf(b, b, nb);
    }
    for (int off = 32; off >= 1; off >>= 1) {
      dot += __shfl_xor(dot, off);
      na += __shfl_xor(na, off);
      nb += __shfl_xor(nb, off);
    }
    if (lane == 0) {
      const float ra = sqrtf(na), rb = sqrtf(nb);
      const float w = (ra < 1e-20f || rb < 1e-20f) ? 0.f : fabsf(dot / (ra * rb));
      w_s[j] = w;
      wgt[j * hq + h] = w;
    }
  }
  __syncthreads();
  const int c = t % d, sl = t / d, ns = 1024 / d;
  float acc = 0.f;
  for (int j = sl; j < n_ctx; j += ns) acc = fmaf(w_s[j], loc[((size_t)j * hq + h) * d + c], acc);
  red[t] = acc;
  __syncthreads();
  if (t < d) {
    float b = 0.f;
    for (int s2 = 0; s2 < ns; ++s2) b += red[s2 * d + c];
    bias[h * d + c] = b;
  }
}

// Eq. 1 for the query heads of KV group g, then their mean: the bias of document i is the sum over all
// documents minus document i's own term.  One block per (document, KV head), one thread per channel.
__global__ void k_qtilde(const float* que, const float* bias, const float* loc, const float* wgt, float* qt, int n_ctx,
                         int hq, int hkv, int d, int with_bias) {
  const int i = blockIdx.x, g = blockIdx.y, c = threadIdx.x;
  const int G = hq / hkv;
  float acc = 0.f;
  for (int h = g * G; h < (g + 1) * G; ++h) {
    float v = que[h * d + c];
    if (with_bias) {
      const float others = bias[h * d + c] - wgt[i * hq + h] * loc[((size_t)i * hq + h) * d + c];
      v += others / (float)(n_ctx - 1);
    }
    acc += v;
  }
  qt[((size_t)i * hkv + g) * d + c] = acc / (float)G;
}

// One block = 4 waves; a wave loads 16 x 16 bytes per lane up front (two batches of NB rows groups),
// so about 16 KB per wave is in flight.  LPR lanes share one key row; their partial dot products are
// combined with DPP moves, and lane (row group rg, sub < NB) stores row sub * RPL + rg of the batch:
// 32 consecutive floats per wave store.
template <bool BF16, int D>
__global__ __launch_bounds__(256) void k_score(PtrTable kt, IntTable cu_len, const float* qt, float* scores, int hkv,
                                               int total_len) {
  constexpr int EPL = BF16 ? 8 : 4;
  constexpr int LPR = D / EPL;
  constexpr int RPL = 64 / LPR;
  constexpr int NB = 8;
  constexpr int ROWS_PER_WAVE = RPL * NB * 2;
  constexpr int TILE = ROWS_PER_WAVE * 4;
  constexpr size_t ROW_BYTES = (size_t)D * (BF16 ? 2 : 4);
  static_assert(LPR >= NB, "store mapping needs at least NB lanes per row");

  const int i = blockIdx.y, g = blockIdx.z;
  const int L = cu_len.v[i + 1] - cu_len.v[i];
  const int row0 = blockIdx.x * TILE + (threadIdx.x >> 6) * ROWS_PER_WAVE;
  if (row0 >= L) return;
  const int lane = threadIdx.x & 63, sub = lane % LPR, rg = lane / LPR;

  float q[EPL];
  {
    const float* qp = qt + ((size_t)i * hkv + g) * D + sub * EPL;
#pragma unroll
    for (int e = 0; e < EPL; ++e) q[e] = qp[e];
  }
  const char* base = static_cast<const char*>(kt.p[i]) + (size_t)g * L * ROW_BYTES + sub * 16;
  float* out = scores + (size_t)g * total_len + cu_len.v[i];

  u32x4 x[2][NB];
#pragma unroll
  for (int b2 = 0; b2 < 2; ++b2)
#pragma unroll
    for (int b = 0; b < NB; ++b) {
      int row = row0 + (b2 * NB + b) * RPL + rg;
      row = row < L ? row : L - 1;
      x[b2][b] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(base + (size_t)row * ROW_BYTES));
    }
#pragma unroll
  for (int b2 = 0; b2 < 2; ++b2) {
    float keep = 0.f;
#pragma unroll
    for (int b = 0; b < NB; ++b) {
      float f[EPL];
      unpack16<BF16>(x[b2][b], f);
      float s = 0.f;
#pragma unroll
      for (int e = 0; e < EPL; ++e) s = fmaf(f[e], q[e], s);
      s = group_sum<LPR>(s);
      keep = (sub % NB == b) ? s : keep;
    }
    const int row = row0 + (b2 * NB + (sub % NB)) * RPL + rg;
    if (sub < NB && row < L) out[row] = keep;
  }
}

template <bool BF16, int D>
hipError_t run(const ScoreLaunch& a, const PtrTable& k, const IntTable& cu_len, hipStream_t s) {
  const bool bias = a.q_loc != nullptr && a.n_ctx > 1;
  hipLaunchKernelGGL((k_pool<BF16, D>), dim3(a.hq, bias ? a.n_ctx + 1 : 1), dim3(256), 0, s, a.q_tok, a.n_q_tok,
                     a.q_loc, a.w_loc, a.hq, a.ws_que, a.ws_loc);
  if (bias)
    hipLaunchKernelGGL(k_bias, dim3(a.hq), dim3(1024), 0, s, a.ws_que, a.ws_loc, a.ws_w, a.ws_base, a.n_ctx, a.hq, D);
  hipLaunchKernelGGL(k_qtilde, dim3(a.n_ctx, a.hkv), dim3(D), 0, s, a.ws_que, a.ws_base, a.ws_loc, a.ws_w, a.ws_qt,
                     a.n_ctx, a.hq, a.hkv, D, bias ? 1 : 0);
  constexpr int TILE = (64 / (D / (BF16 ? 8 : 4))) * 8 * 2 * 4;
  dim3 gs((a.max_len + TILE - 1) / TILE, a.n_ctx, a.hkv);
  hipLaunchKernelGGL((k_score<BF16, D>), gs, dim3(256), 0, s, k, cu_len, a.ws_qt, a.scores, a.hkv, a.total_len);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_score(const ScoreLaunch& a, const PtrTable& k, const IntTable& cu_len, hipStream_t s) {
  if (a.dtype == SAMKV_BF16) return a.d == 128 ? run<true, 128>(a, k, cu_len, s) : run<true, 64>(a, k, cu_len, s);
  return a.d == 128 ? run<false, 128>(a, k, cu_len, s) : run<false, 64>(a, k, cu_len, s);
}

}  // namespace samkv
