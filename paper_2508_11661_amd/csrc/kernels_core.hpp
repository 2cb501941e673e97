// Device functions shared by the score, select and fused score+select kernels: the arithmetic of a score and the
// selection of a row's kept positions exist once, so the fused kernel reproduces the two-call path bit for bit.
#pragma once
#include "common.hpp"

namespace samkv {

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

// The vector a KV head scores its document's keys with: the mean of `group` consecutive head vectors of D floats
// (1 when the fold over the KV group has already been done, G when src holds Eq. 1 per query head).  The lane
// takes its EPL channels.
template <int EPL>
__device__ __forceinline__ void fold_query(const float* src, int d, int group, float* q) {
#pragma unroll
  for (int e = 0; e < EPL; ++e) q[e] = 0.f;
  for (int hh = 0; hh < group; ++hh)
#pragma unroll
    for (int e = 0; e < EPL; ++e) q[e] += src[hh * d + e];
#pragma unroll
  for (int e = 0; e < EPL; ++e) q[e] /= (float)group;
}

// One wave scores RPL * NB * 2 consecutive key rows starting at row0 (rows >= L are skipped): 16 x 16 bytes per
// lane are loaded up front, LPR lanes share one key row, their partial dot products are combined with DPP moves,
// and lane (row group rg, sub < NB) emits row sub * RPL + rg of a batch.  `base` already points at the lane's
// 16-byte column of row 0.
template <bool BF16, int D, class Emit>
__device__ __forceinline__ void score_rows(const char* base, int row0, int L, const float* q, Emit emit) {
  constexpr int EPL = BF16 ? 8 : 4;
  constexpr int LPR = D / EPL;
  constexpr int RPL = 64 / LPR;
  constexpr int NB = 8;
  constexpr size_t ROW_BYTES = (size_t)D * (BF16 ? 2 : 4);
  static_assert(LPR >= NB, "store mapping needs at least NB lanes per row");
  const int lane = threadIdx.x & 63, sub = lane % LPR, rg = lane / LPR;
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
    if (sub < NB && row < L) emit(row, keep);
  }
}

__device__ __forceinline__ uint32_t order_key(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u << 1) == 0u) u = 0u;  // -0 and +0 are one value: ties go by position, not by sign bit
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Forced positions (the first n_sink and last n_local of the row) get the largest key.
template <int E>
__device__ __forceinline__ void force_keys(uint32_t (&key)[E], int p0, int L, int n_sink, int n_local) {
#pragma unroll
  for (int e = 0; e < E; ++e) {
    const int p = p0 + e;
    if (p < L && (p < n_sink || p >= L - n_local)) key[e] = 0xFFFFFFFFu;
  }
}

// The k kept positions of a row whose order keys sit in registers (thread t owns positions p0 = t * E ... + E - 1,
// keys of positions >= L are 0), written ascending to out[0..k).  cnt and wsum are LDS scratch of the workgroup.
template <int E, int NT>
__device__ __forceinline__ void select_from_keys(uint32_t (&key)[E], int p0, int L, int k, int32_t* out,
                                                 uint32_t (*cnt)[NT / 64], uint64_t* wsum) {
  constexpr int NW = NT / 64;
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  // ---- k-th largest key, bit by bit ------------------------------------------------------------
  // `bucket` = positions < L whose keys agree with the bits decided so far; kk of them are still to be kept.  Once
  // bucket == kk every one of them is kept whatever the remaining bits say, so the walk stops there (distinct keys:
  // after about log2(L) bits below the ones all keys share; rows of equal keys walk all 32).
  uint32_t prefix = 0;
  uint32_t kk = (uint32_t)k, bucket = (uint32_t)L;
  for (int b = 31; b >= 0 && bucket != kk; --b) {
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
    if (tot >= kk) {
      prefix |= (1u << b);
      bucket = tot;
    } else {
      kk -= tot;
      bucket -= tot;
    }
  }
  // T: the decided bits, zeros below.  Stopped early: every key >= T is kept; walked to the end: keys > T and the
  // first kk positions with key == T
  const uint32_t T = prefix;
  const uint32_t need = bucket == kk ? 0xFFFFFFFFu : kk;  // how many positions with key == T are kept

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

}  // namespace samkv
