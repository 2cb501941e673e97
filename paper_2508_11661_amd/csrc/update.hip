// samkv_kv_update: what happens to the compacted cache after the kept tokens were recomputed (Sec. 3.3).
//   overwrite: the recomputed K/V rows replace the old ones;
//   fusion (Eq. 4): theta = cos(new row, old row), row <- theta * new + (1 - theta) * old, taken per cached
//   token and KV head, separately for K and for V.
// One pass, HBM-bound: 2*d*e bytes read and d*e written per row.  A row is LPR 16-byte chunks; the LPR lanes
// that share a row combine their partial dot product and norms with DPP moves, then each lane blends and
// stores its own chunk.
#include "common.hpp"

namespace samkv {
namespace {

template <int CTRL>
__device__ __forceinline__ float dpp_move(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, true));
}
template <int W>
__device__ __forceinline__ float group_sum(float v) {
  v += dpp_move<0xB1>(v);
  v += dpp_move<0x4E>(v);
  v += dpp_move<0x141>(v);
  if (W >= 16) v += dpp_move<0x140>(v);
  if (W >= 32) v += __int_as_float(__builtin_amdgcn_ds_swizzle(__float_as_int(v), 0x401F));
  return v;
}

__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {  // round to nearest, ties to even
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (u >> 16) | 0x40u;  // NaN stays NaN
  return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

template <bool BF16, int D, bool FUSION>
__global__ __launch_bounds__(256) void k_kv_update(char* k_cur, char* v_cur, const char* k_new, const char* v_new,
                                                   long long n_rows) {
  constexpr int EPL = BF16 ? 8 : 4;
  constexpr int LPR = D / EPL;
  constexpr int RPW = 64 / LPR;
  constexpr int ROWS_PER_BLOCK = RPW * 4 * 4;  // 4 waves, 4 rows groups per wave
  constexpr size_t ROW_BYTES = (size_t)D * (BF16 ? 2 : 4);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, sub = lane % LPR, rg = lane / LPR;
  char* cur = blockIdx.y == 0 ? k_cur : v_cur;
  const char* fresh = blockIdx.y == 0 ? k_new : v_new;
  const long long r0 = (long long)blockIdx.x * ROWS_PER_BLOCK + wave * (RPW * 4);
  u32x4 xo[4], xn[4];
#pragma unroll
  for (int s = 0; s < 4; ++s) {
    long long row = r0 + s * RPW + rg;
    row = row < n_rows ? row : n_rows - 1;
    xn[s] = *reinterpret_cast<const u32x4*>(fresh + row * ROW_BYTES + sub * 16);
    if (FUSION) xo[s] = *reinterpret_cast<const u32x4*>(cur + row * ROW_BYTES + sub * 16);
  }
#pragma unroll
  for (int s = 0; s < 4; ++s) {
    const long long row = r0 + s * RPW + rg;
    u32x4 out = xn[s];
    if (FUSION) {
      float fo[EPL], fn[EPL];
      if (BF16) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          fo[2 * e] = bf16_lo(xo[s][e]); fo[2 * e + 1] = bf16_hi(xo[s][e]);
          fn[2 * e] = bf16_lo(xn[s][e]); fn[2 * e + 1] = bf16_hi(xn[s][e]);
        }
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) { fo[e] = __uint_as_float(xo[s][e]); fn[e] = __uint_as_float(xn[s][e]); }
      }
      float dot = 0.f, nn = 0.f, no = 0.f;
#pragma unroll
      for (int e = 0; e < EPL; ++e) {
        dot = fmaf(fn[e], fo[e], dot);
        nn = fmaf(fn[e], fn[e], nn);
        no = fmaf(fo[e], fo[e], no);
      }
      dot = group_sum<LPR>(dot);
      nn = group_sum<LPR>(nn);
      no = group_sum<LPR>(no);
      const float rn = sqrtf(nn), ro = sqrtf(no);
      const float theta = (rn < 1e-20f || ro < 1e-20f) ? 1.f : dot / (rn * ro);
      float res[EPL];
#pragma unroll
      for (int e = 0; e < EPL; ++e) res[e] = theta * fn[e] + (1.f - theta) * fo[e];
      if (BF16) {
#pragma unroll
        for (int e = 0; e < 4; ++e) out[e] = f32_to_bf16_bits(res[2 * e]) | (f32_to_bf16_bits(res[2 * e + 1]) << 16);
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) out[e] = __float_as_uint(res[e]);
      }
    }
    if (row < n_rows) *reinterpret_cast<u32x4*>(cur + row * ROW_BYTES + sub * 16) = out;
  }
}

template <bool BF16, int D>
hipError_t run(const UpdateLaunch& a, hipStream_t s) {
  constexpr int ROWS_PER_BLOCK = (64 / (D / (BF16 ? 8 : 4))) * 16;
  dim3 grid((unsigned)((a.n_rows + ROWS_PER_BLOCK - 1) / ROWS_PER_BLOCK), 2);
  if (a.fusion)
    hipLaunchKernelGGL((k_kv_update<BF16, D, true>), grid, dim3(256), 0, s, static_cast<char*>(a.k_cur),
                       static_cast<char*>(a.v_cur), static_cast<const char*>(a.k_new), static_cast<const char*>(a.v_new),
                       a.n_rows);
  else
    hipLaunchKernelGGL((k_kv_update<BF16, D, false>), grid, dim3(256), 0, s, static_cast<char*>(a.k_cur),
                       static_cast<char*>(a.v_cur), static_cast<const char*>(a.k_new), static_cast<const char*>(a.v_new),
                       a.n_rows);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_kv_update(const UpdateLaunch& a, hipStream_t s) {
  if (a.dtype == SAMKV_BF16) return a.d == 128 ? run<true, 128>(a, s) : run<true, 64>(a, s);
  return a.d == 128 ? run<false, 128>(a, s) : run<false, 64>(a, s);
}

}  // namespace samkv
