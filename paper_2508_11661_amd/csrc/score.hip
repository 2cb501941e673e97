// samkv_score: personalized query vectors (Sec. 3.1, Eq. 1) and the inner product of every cached key
// with the vector of its own document (Sec. 3.2).
//
// Four launches on one stream (short inputs: k_prologue replaces the first three, see there):
//   k_pool    mean-pools the user query's Q rows (Q_que) and every document's local Q cache (Q_loc_j).
//   k_bias    per query head: |cos(Q_que, Q_loc_j)| for every j and the weighted sum over all documents.
//   k_qtilde  Eq. 1 for the query heads of a KV group, folded into one vector per document (the mean
//             over the group is linear, so one pass over K serves all heads of the group).
//   k_score   streams K once.  HBM-bound: d*e bytes read and 4 bytes written per token and KV head.
#include "common.hpp"
#include "kernels_core.hpp"

namespace samkv {
namespace {

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
// slice s) adds the documents j = s, s + NS, ..., and the slices meet in LDS in a fixed order.  Step 3: Eq. 1 per
// query head, Q^_i[h] = Q_que[h] + (bias[h] - w_i Q_loc_i[h]) / (N - 1), written over Q_loc_i[h] in place (thread
// (c, s) is the only one that still touches element c of the documents of its slice), so that `loc` leaves as
// qhat[i][h][:] like the output of k_prologue and k_score folds the heads of a KV group.
__global__ __launch_bounds__(1024) void k_bias(const float* que, float* loc, float* wgt, float* bias, int n_ctx,
                                               int hq, int d) {
  __shared__ float red[1024];
  __shared__ float w_s[SAMKV_MAX_CTX];
  __shared__ float b_s[128];
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
    b_s[c] = b;
  }
  __syncthreads();
  const float q = que[h * d + c], b = b_s[c], inv = 1.f / (float)(n_ctx - 1);
  for (int j = sl; j < n_ctx; j += ns) {
    float* p = loc + ((size_t)j * hq + h) * d + c;
    *p = q + (b - w_s[j] * *p) * inv;
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

// The three launches above in one, for short inputs (one workgroup of 16 waves per query head; the head's local
// Q caches of all documents pass through that one workgroup, so this is for inputs of up to about a megabyte per
// head, where launch latency and not bandwidth is what the three launches cost).  Writes Eq. 1 per QUERY head,
// qhat[i][h][:]; k_score folds the heads of a KV group.
//   1. wave w takes documents w, w + 16, ...: mean of the document's local rows, into LDS.
//   2. Q_que[h]: the 16 waves split the user query's rows (requested ahead of step 1); partial sums meet in LDS.
//   3. w_j = |cos(Q_que, Q_loc_j)|, bias = sum_j w_j Q_loc_j, then Q^_i = Q_que + (bias - w_i Q_loc_i) / (N - 1).
template <bool BF16, int D>
__global__ __launch_bounds__(1024) void k_prologue(const void* q_tok, int n_q_tok, const void* q_loc, int w_loc, int n_ctx,
                                                   int hq, int with_bias, float* qhat) {
  constexpr int EPL = BF16 ? 8 : 4;
  constexpr int LPR = D / EPL;   // lanes per row
  constexpr int RPW = 64 / LPR;  // rows per wave step
  constexpr size_t ROW_BYTES = (size_t)D * (BF16 ? 2 : 4);
  extern __shared__ float sm[];
  float* s_que = sm;                 // [D]
  float* s_bias = sm + D;            // [D]
  float* red = sm + 2 * D;           // [16][D]
  float* s_w = red + 16 * D;         // [n_ctx]
  float* s_loc = s_w + SAMKV_MAX_CTX;  // [n_ctx][D]
  const int h = blockIdx.x, t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int sub = lane % LPR, rgp = lane / LPR;

  // acc += rows r0, r0 + step, ... (< n_rows) of `src`, U 16-byte loads in flight per lane; the loads of the first
  // batch can be issued ahead (issue_rows) and consumed later (take_rows), with other loads in between
  auto issue_rows = [&](const char* src, int r0, int step, int n_rows, auto& x) {
    constexpr int U = sizeof(x) / sizeof(x[0]);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int r = r0 + u * step;
      x[u] = *reinterpret_cast<const u32x4*>(src + (size_t)(r < n_rows ? r : n_rows - 1) * ROW_BYTES);
    }
  };
  auto take_rows = [&](int r0, int step, int n_rows, const auto& x, float* acc) {
    constexpr int U = sizeof(x) / sizeof(x[0]);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float f[EPL];
      unpack16<BF16>(x[u], f);
      const float keep = (r0 + u * step < n_rows) ? 1.f : 0.f;
#pragma unroll
      for (int e = 0; e < EPL; ++e) acc[e] = fmaf(f[e], keep, acc[e]);
    }
  };
  auto add_rows = [&](const char* src, int first, int step, int n_rows, float* acc) {
    constexpr int U = 16;
    for (int r0 = first; r0 < n_rows; r0 += U * step) {
      u32x4 x[U];
      issue_rows(src, r0, step, n_rows, x);
      take_rows(r0, step, n_rows, x, acc);
    }
  };
  // sum over the row groups of a wave: lanes that differ in the bits above log2(LPR)
  auto fold_rows = [&](float* acc) {
#pragma unroll
    for (int off = LPR; off < 64; off <<= 1)
#pragma unroll
      for (int e = 0; e < EPL; ++e) acc[e] += __shfl_xor(acc[e], off);
  };
  // The user query's rows and the documents' local rows are independent inputs: the first batch of the former is
  // requested before the latter are pooled, so the two memory round trips overlap.
  constexpr int UQ = 2;
  const char* tok_src = static_cast<const char*>(q_tok) + (size_t)h * n_q_tok * ROW_BYTES + sub * 16;
  const int tok_first = wave * RPW + rgp, tok_step = 16 * RPW;
  u32x4 xq[UQ];
  issue_rows(tok_src, tok_first, tok_step, n_q_tok, xq);
  if (with_bias) {
    for (int j = wave; j < n_ctx; j += 16) {
      const char* src = static_cast<const char*>(q_loc) + ((size_t)j * hq + h) * w_loc * ROW_BYTES + sub * 16;
      float acc[EPL];
#pragma unroll
      for (int e = 0; e < EPL; ++e) acc[e] = 0.f;
      add_rows(src, rgp, RPW, w_loc, acc);
      fold_rows(acc);
      if (rgp == 0)
#pragma unroll
        for (int e = 0; e < EPL; ++e) s_loc[j * D + sub * EPL + e] = acc[e] / (float)w_loc;
    }
  }
  {
    float acc[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[e] = 0.f;
    take_rows(tok_first, tok_step, n_q_tok, xq, acc);
    add_rows(tok_src, tok_first + UQ * tok_step, tok_step, n_q_tok, acc);
    fold_rows(acc);
    if (rgp == 0)
#pragma unroll
      for (int e = 0; e < EPL; ++e) red[wave * D + sub * EPL + e] = acc[e];
  }
  __syncthreads();
  if (t < D) {
    float v = 0.f;
    for (int w = 0; w < 16; ++w) v += red[w * D + t];
    s_que[t] = v / (float)n_q_tok;
  }
  __syncthreads();
  if (with_bias) {
    float qv[EPL], na = 0.f;
#pragma unroll
    for (int e = 0; e < EPL; ++e) {
      qv[e] = s_que[sub * EPL + e];
      na = fmaf(qv[e], qv[e], na);
    }
    na = group_sum<LPR>(na);
    for (int j = wave; j < n_ctx; j += 16) {
      float dot = 0.f, nb = 0.f;
#pragma unroll
      for (int e = 0; e < EPL; ++e) {
        const float lv = s_loc[j * D + sub * EPL + e];
        dot = fmaf(qv[e], lv, dot);
        nb = fmaf(lv, lv, nb);
      }
      dot = group_sum<LPR>(dot);
      nb = group_sum<LPR>(nb);
      if (lane == 0) {
        const float ra = sqrtf(na), rb = sqrtf(nb);
        s_w[j] = (ra < 1e-20f || rb < 1e-20f) ? 0.f : fabsf(dot / (ra * rb));
      }
    }
    __syncthreads();
    const int c = t % D, sl = t / D;
    constexpr int NS = 1024 / D;
    float acc = 0.f;
    for (int j = sl; j < n_ctx; j += NS) acc = fmaf(s_w[j], s_loc[j * D + c], acc);
    red[sl * D + c] = acc;
    __syncthreads();
    if (t < D) {
      float b = 0.f;
      for (int s2 = 0; s2 < NS; ++s2) b += red[s2 * D + t];
      s_bias[t] = b;
    }
    __syncthreads();
  }
  for (int x = t; x < n_ctx * D; x += 1024) {
    const int i = x / D, c = x % D;
    float v = s_que[c];
    if (with_bias) v += (s_bias[c] - s_w[i] * s_loc[i * D + c]) / (float)(n_ctx - 1);
    qhat[((size_t)i * hq + h) * D + c] = v;
  }
}

// One block = 4 waves; a wave loads 16 x 16 bytes per lane up front (two batches of NB rows groups),
// so about 16 KB per wave is in flight.  LPR lanes share one key row; their partial dot products are
// combined with DPP moves, and lane (row group rg, sub < NB) stores row sub * RPL + rg of the batch:
// 32 consecutive floats per wave store.
template <bool BF16, int D>
__global__ __launch_bounds__(256) void k_score(PtrTable kt, IntTable cu_len, const float* qsrc, int heads, int group,
                                               float* scores, int total_len) {
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

  // the document's vector for this KV head: qsrc is [N][heads][D]; `group` consecutive heads are averaged
  // (1 when the fold over the KV group has already been done, G when qsrc holds Eq. 1 per query head)
  float q[EPL];
  fold_query<EPL>(qsrc + ((size_t)i * heads + (size_t)g * group) * D + sub * EPL, D, group, q);
  const char* base = static_cast<const char*>(kt.p[i]) + (size_t)g * L * ROW_BYTES + sub * 16;
  float* out = scores + (size_t)g * total_len + cu_len.v[i];
  score_rows<BF16, D>(base, row0, L, q, [&](int row, float s) { out[row] = s; });
}

// Eq. 1 for every document; tells the caller where the vectors are and how many heads k_score must average.
template <bool BF16, int D>
hipError_t run_prologue(const ScoreLaunch& a, hipStream_t s, QuerySrc* out) {
  const bool bias = a.q_loc != nullptr && a.n_ctx > 1;
  // bytes of Q rows that pass through one query head's workgroup in the one-launch prologue
  const size_t per_head = ((size_t)a.n_q_tok + (bias ? (size_t)a.n_ctx * a.w_loc : 0)) * D * (BF16 ? 2 : 4);
  if (a.n_ctx <= 64 && per_head <= (1u << 20)) {
    const size_t lds = (size_t)(2 * D + 16 * D + SAMKV_MAX_CTX + a.n_ctx * D) * sizeof(float);
    hipLaunchKernelGGL((k_prologue<BF16, D>), dim3(a.hq), dim3(1024), lds, s, a.q_tok, a.n_q_tok, a.q_loc, a.w_loc, a.n_ctx,
                       a.hq, bias ? 1 : 0, a.ws_loc);
    out->q = a.ws_loc; out->heads = a.hq; out->group = a.hq / a.hkv;
    return hipGetLastError();
  }
  hipLaunchKernelGGL((k_pool<BF16, D>), dim3(a.hq, bias ? a.n_ctx + 1 : 1), dim3(256), 0, s, a.q_tok, a.n_q_tok,
                     a.q_loc, a.w_loc, a.hq, a.ws_que, a.ws_loc);
  if (bias) {
    // two launches: the pooled local caches leave k_bias as Eq. 1 per query head, folded by the score kernel
    hipLaunchKernelGGL(k_bias, dim3(a.hq), dim3(1024), 0, s, a.ws_que, a.ws_loc, a.ws_w, a.ws_base, a.n_ctx, a.hq, D);
    out->q = a.ws_loc; out->heads = a.hq; out->group = a.hq / a.hkv;
    return hipGetLastError();
  }
  hipLaunchKernelGGL(k_qtilde, dim3(a.n_ctx, a.hkv), dim3(D), 0, s, a.ws_que, a.ws_base, a.ws_loc, a.ws_w, a.ws_qt,
                     a.n_ctx, a.hq, a.hkv, D, bias ? 1 : 0);
  out->q = a.ws_qt; out->heads = a.hkv; out->group = 1;
  return hipGetLastError();
}

template <bool BF16, int D>
hipError_t run_keys(const ScoreLaunch& a, const QuerySrc& q, const PtrTable& k, const IntTable& cu_len, hipStream_t s) {
  constexpr int TILE = (64 / (D / (BF16 ? 8 : 4))) * 8 * 2 * 4;
  dim3 gs((a.max_len + TILE - 1) / TILE, a.n_ctx, a.hkv);
  hipLaunchKernelGGL((k_score<BF16, D>), gs, dim3(256), 0, s, k, cu_len, q.q, q.heads, q.group, a.scores, a.total_len);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_score_prologue(const ScoreLaunch& a, hipStream_t s, QuerySrc* q) {
  if (a.dtype == SAMKV_BF16) return a.d == 128 ? run_prologue<true, 128>(a, s, q) : run_prologue<true, 64>(a, s, q);
  return a.d == 128 ? run_prologue<false, 128>(a, s, q) : run_prologue<false, 64>(a, s, q);
}

hipError_t launch_score(const ScoreLaunch& a, const PtrTable& k, const IntTable& cu_len, hipStream_t s) {
  QuerySrc q;
  hipError_t e = launch_score_prologue(a, s, &q);
  if (e != hipSuccess) return e;
  if (a.dtype == SAMKV_BF16) return a.d == 128 ? run_keys<true, 128>(a, q, k, cu_len, s) : run_keys<true, 64>(a, q, k, cu_len, s);
  return a.d == 128 ? run_keys<false, 128>(a, q, k, cu_len, s) : run_keys<false, 64>(a, q, k, cu_len, s);
}

}  // namespace samkv
