// Attention over the compacted multi-document cache (Sec. 3.3):
//   causal     - recomputation of the kept tokens: row p sees compacted positions 0..p
//   not causal - the user query's final incremental prefill over the whole compacted cache
// Both are softmax(scale * q k^T) v with float32 statistics; they differ in the mask and in how the
// rows are cut into workgroups, so one kernel template serves both.
//
// bf16 kernel (k_attn_bf16), one workgroup = NW waves (4 or 8) of 32 query rows each, 64 keys per step:
//   S^T = K Q^T   v_mfma_f32_32x32x16_bf16, A = K rows from LDS, B = the wave's 32 query rows (registers,
//                 loaded once).  Computing the transpose puts one query row in one lane column, so the
//                 softmax weights come out of the accumulator already in the B-operand layout of the
//                 next product and never travel through LDS.
//   O^T += V^T P^T  v_mfma_f32_32x32x16_f16, A = V^T read from the row-major V tile in LDS with the
//                 transposing LDS read (ds_read_b64_tr_b16), B = P^T from registers.  Both operands are IEEE
//                 half precision: the weights keep an 11-bit significand (bf16 weights would cost 2^-9 of the
//                 spread of V per output), and V arrives as the scaled half-precision copy of vprep.hip, whose
//                 power-of-two scale the final normalisation undoes.
//   K/V tiles are double-buffered in LDS; the next tile's global loads are issued before the current
//   tile's math and land in LDS after it, one barrier per tile.
// f32 kernel (k_attn_f32): plain FMA arithmetic for float32 caches, 16 rows per workgroup.
// Keys can be cut into chunks (not causal only); k_attn_merge combines the per-chunk results with
// their log-sum-exp.
#include <math.h>

#include <mutex>

#include "common.hpp"

namespace samkv {
namespace {

struct AttnArgs {
  const void* q;
  const void* k;
  const void* v;           // half-precision copy of V (bf16 kernels)
  const float* v_unscale;  // per KV head: undoes the copy's scale
  float* out;
  float* lse;
  float* part_o;
  float* part_lse;
  int rows, m, batch_per_kv, n_batch, n_split, chunk;
  int kv_groups;  // > 0: KV heads are walked in groups of 8 (one per XCD), see map_block
  float scale;
};

// Exchange between lane l and lane l ^ 32 on the vector ALU (v_permlane32_swap; with both operands equal the first
// result holds the lower half's values in both halves and the second the upper half's): no trip through LDS as a
// 64-wide shuffle would take, which matters because the row maximum sits at the head of every step's dependence chain.
__device__ __forceinline__ float max_across_halves(float v) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float sum_across_halves(float v) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// Writes a wave's 32 x D block of normalised output rows.  In the accumulator layout a lane holds 4-float pieces of
// ONE row (row = lane % 32), so a direct store instruction scatters 32-byte pieces over 32 rows; issuing the 4 D / 32
// of them takes a few microseconds, which a short workgroup feels.  The block is therefore turned through LDS (the
// wave's own `lds` area; rows of D * 4 + 16 bytes, the pad keeps the 16 lanes of a write phase on distinct banks)
// and leaves as whole rows, 1 KB per instruction.  PARTS = 1 turns the 32 rows at once (area of 32 rows), PARTS = 2
// in two passes of 16 rows (area of 16 rows).  Only this wave touches the area, and a wave's LDS operations execute
// in order, so no workgroup barrier is needed.  dst points at the wave's first row; rows >= n_valid are not written.
template <int D, int PARTS = 1>
__device__ __forceinline__ void store_rows_via_lds(const f32x16 (&o)[D / 32], float inv, float* dst, int n_valid, char* lds,
                                                   int lane) {
  constexpr int RS = D * 4 + 16, LPR = D / 4, RPI = 64 / LPR, ROWS = 32 / PARTS;
  const int rw = lane & 31, h = lane >> 5;
#pragma unroll
  for (int part = 0; part < PARTS; ++part) {
    if (PARTS == 1 || rw / ROWS == part) {
#pragma unroll
      for (int dvb = 0; dvb < D / 32; ++dvb)
#pragma unroll
        for (int j4 = 0; j4 < 4; ++j4) {
          f32x4 x;
#pragma unroll
          for (int e = 0; e < 4; ++e) x[e] = o[dvb][4 * j4 + e] * inv;
          *reinterpret_cast<f32x4*>(lds + (rw % ROWS) * RS + (dvb * 32 + 8 * j4 + 4 * h) * 4) = x;
        }
    }
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int i = 0; i < ROWS / RPI; ++i) {
      const int lrow = i * RPI + lane / LPR, row = part * ROWS + lrow;
      const f32x4 x = *reinterpret_cast<const f32x4*>(lds + lrow * RS + (lane % LPR) * 16);
      if (row < n_valid) *reinterpret_cast<f32x4*>(dst + (size_t)row * D + (lane % LPR) * 4) = x;
    }
    __builtin_amdgcn_wave_barrier();
  }
}

// (blockIdx.x, blockIdx.y) -> (KV head, batch, row tile).  Workgroups are handed out x-fastest and round-robin over
// the 8 XCDs, each with its own L2.  The batches (query heads x row blocks) that read one KV head's K/V stream
// should run on one XCD and close in time, and an XCD should not hold more streams at once than its L2 can serve.
// So KV heads are taken in groups of 8, one head per XCD: x = 8 * member + XCD slot runs over the batches of the
// group's heads, y = group * tiles + tile, and a group's row tiles (longest first when causal) are all handed out
// before the next group starts.  With 8 KV heads there is one group and this is "KV head = x % 8, all row tiles in
// longest-first order"; with many KV heads (several layers stacked as heads) an XCD still streams one head at a
// time instead of dozens.  kv_groups == 0 (head count not a multiple of 8): plain x = batch, y = tile.
// A workgroup's coordinates in the (batch, row tile, key chunk) grid of its problem: a plain launch takes them from
// the hardware, the pair launch below hands out two problems' grids from one linear index
// (x, y, z of grid_y rows): plain ints, so that nothing of it ever lives in memory.
__device__ __forceinline__ void map_block(const AttnArgs& a, bool causal, int x, int y, int grid_y, int* kvh, int* batch,
                                          int* tile) {
  int ty;
  if (a.kv_groups > 0) {
    const int tiles = grid_y / a.kv_groups;
    const int grp = y / tiles;
    ty = y - grp * tiles;
    *kvh = grp * 8 + (x & 7);
    *batch = *kvh * a.batch_per_kv + (x >> 3);
    *tile = causal ? tiles - 1 - ty : ty;
  } else {
    const int n_kv = a.n_batch / a.batch_per_kv;
    *kvh = x % n_kv;
    *batch = *kvh * a.batch_per_kv + x / n_kv;
    *tile = causal ? grid_y - 1 - y : y;
  }
}

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// ------------------------------------------------------------------------------------------ bf16
// NW waves = RG row groups (32 query rows each) x KG key groups.  With KG = 2 a step stages 128 keys and the two
// key groups of a row group each take 64 of them, so a causal row tile walks its keys in half as many sequential
// steps; the two partial results meet through LDS at the end.  That is for short problems, where the longest row
// tile's chain of steps, not the total work, sets the kernel's duration.
template <int D, int NW_, int KG_ = 1>
struct Bf16Cfg {
  static constexpr int NW = NW_, NT = 64 * NW, KG = KG_, RG = NW / KG;
  static constexpr int BQ = 32 * RG, BK = 64, BKT = BK * KG;
  static constexpr int KSTR = D * 2 + 16;  // bytes per K row in LDS (pad: 16 rows hit 64 distinct banks)
  static constexpr int VSTR = D * 2 + 64;  // bytes per V row in LDS: the 4 rows x 32 B of a transposing read fall in disjoint bank ranges
  static constexpr int TILE_BYTES = BKT * (KSTR + VSTR);
  static constexpr int LDS_BYTES = 2 * TILE_BYTES;
  static constexpr int CHUNKS = (BKT * D * 2 / 16) / NT;  // 16-byte chunks per thread per tile and tensor
  static constexpr int MERGE_BYTES = RG * 64 * (D / 32 * 16 + 2) * 4;  // one key group's state per row group

  static_assert(KG == 1 || MERGE_BYTES <= LDS_BYTES, "the merge reuses the tile buffers");
};

typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

// SPLIT: how the second product gets 16-bit operands without losing the weights' precision.  false: the weights are
// rounded to half precision and V is the scaled half-precision copy that vprep.hip makes.  true: V is read as stored
// (bf16) and every weight travels as the sum of TWO bf16 terms (p = hi + lo, 16 significant bits), which doubles the
// second product's instructions and needs no copy.  That pays where the products are not what the kernel waits for
// and the launches that prepare V would cost more: the query attention of short and mid-size caches (bound by
// latency or by HBM; 34 -> 26 us at M = 1540, 54 -> 45 us at M = 6160 as calls).  Causal problems of the same shapes
// lose more in the products than the preparation costs (+10 to +18 % at M = 2304 .. 2816) and keep the copy.
template <int D, bool CAUSAL, int NW, int KG = 1, bool SPLIT = false>
__device__ __forceinline__ void attn_bf16_body(const AttnArgs a, int bx, int by, int bz, int grid_y) {
  using C = Bf16Cfg<D, NW, KG>;
  static_assert(KG == 1 || KG == 2, "one or two key groups");
  constexpr int ND = D / 16;   // k-steps of the S^T product
  constexpr int NV = D / 32;   // 32-row blocks of O^T
  extern __shared__ __attribute__((aligned(16))) char smem[];

  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int rw = lane & 31, h = lane >> 5;
  // grid = (batch, row tile, key chunk).  Workgroups are handed out x-fastest and round-robin over the 8
  // XCDs, so (1) every batch's longest causal row tiles start first and the short ones fill the tail,
  // and (2) map_batch puts the query heads that share a K/V stream on the same XCD, next to each other,
  // where they find its tiles in that XCD's L2.
  int kvh, batch, qt;
  map_block(a, CAUSAL, bx, by, grid_y, &kvh, &batch, &qt);
  const int q0 = qt * C::BQ;
  const int split = bz;
  const int kv_begin = CAUSAL ? 0 : split * a.chunk;
  const int kv_end = CAUSAL ? min(a.m, q0 + C::BQ) : min(a.m, kv_begin + a.chunk);
  const int n_tiles = (kv_end - kv_begin + C::BKT - 1) / C::BKT;

  const int rg = wave % C::RG, kg = wave / C::RG;  // row group, key group
  const int r = q0 + rg * 32 + rw;
  const int r_c = min(r, a.rows - 1);
  const int wave_first = q0 + rg * 32, wave_last = wave_first + 31;

  bf16x8 bq[ND];
  {
    const char* qp = static_cast<const char*>(a.q) + ((size_t)batch * a.rows + r_c) * D * 2 + h * 16;
#pragma unroll
    for (int dc = 0; dc < ND; ++dc) bq[dc] = *reinterpret_cast<const bf16x8*>(qp + dc * 32);
  }
  const char* kbase = static_cast<const char*>(a.k) + (size_t)kvh * a.m * D * 2;
  const char* vbase = static_cast<const char*>(a.v) + (size_t)kvh * a.m * D * 2;

  // Tile loads: thread t fetches chunk (row t/CPR + i*RSTEP, 16-byte column t%CPR) of K and of V.  The
  // byte offsets inside a tile are per-thread constants; the tile base is uniform, so a full tile
  // costs no address arithmetic.  Only the last, ragged tile clamps its rows to the final key.
  constexpr int CPR = D / 8, RSTEP = C::NT / CPR;
  uint32_t voff[C::CHUNKS];
#pragma unroll
  for (int i = 0; i < C::CHUNKS; ++i) voff[i] = (uint32_t)((t / CPR + i * RSTEP) * (D * 2) + (t % CPR) * 16);
  u32x4 rk[C::CHUNKS], rv[C::CHUNKS];
  auto load_tile = [&](int tile) {
    const int k0 = kv_begin + tile * C::BKT;
    const char* kt = kbase + (size_t)k0 * (D * 2);
    const char* vt = vbase + (size_t)k0 * (D * 2);
    if (k0 + C::BKT <= a.m) {
#pragma unroll
      for (int i = 0; i < C::CHUNKS; ++i) {
        rk[i] = *reinterpret_cast<const u32x4*>(kt + voff[i]);
        rv[i] = *reinterpret_cast<const u32x4*>(vt + voff[i]);
      }
    } else {
#pragma unroll
      for (int i = 0; i < C::CHUNKS; ++i) {
        const int row = min(t / CPR + i * RSTEP, a.m - 1 - k0);
        const uint32_t off = (uint32_t)(row * (D * 2) + (t % CPR) * 16);
        rk[i] = *reinterpret_cast<const u32x4*>(kt + off);
        rv[i] = *reinterpret_cast<const u32x4*>(vt + off);
      }
    }
  };
  auto store_tile = [&](int buf) {
    char* sk = smem + buf * C::TILE_BYTES;
    char* sv = sk + C::BKT * C::KSTR;
#pragma unroll
    for (int i = 0; i < C::CHUNKS; ++i) {
      const int c = t + C::NT * i;
      const int row = c / (D / 8), col = c % (D / 8);
      *reinterpret_cast<u32x4*>(sk + row * C::KSTR + col * 16) = rk[i];
      *reinterpret_cast<u32x4*>(sv + row * C::VSTR + col * 16) = rv[i];
    }
  };

  f32x16 o[NV];
#pragma unroll
  for (int i = 0; i < NV; ++i)
#pragma unroll
    for (int j = 0; j < 16; ++j) o[i][j] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;
  const float c2 = a.scale * kLog2e;

  load_tile(0);
  store_tile(0);
  // Drain every outstanding load (the query fragment included) before the loop: otherwise the loop's
  // first use of the query registers has to be guarded by waits that also cover the next tile's prefetch.
  __builtin_amdgcn_s_waitcnt(0);
  __syncthreads();

  for (int tile = 0; tile < n_tiles; ++tile) {
    const int k0 = kv_begin + tile * C::BKT + kg * C::BK;  // first key of this wave's 64 in the staged tile
    const bool more = tile + 1 < n_tiles;
    if (more) load_tile(tile + 1);

    // a wave whose rows all lie past the last row (ragged last row tile) only helps with the tile traffic
    const bool active = wave_first < a.rows && (!CAUSAL || k0 <= wave_last) && (KG == 1 || k0 < kv_end);
    if (active) {
      const char* sk = smem + (tile & 1) * C::TILE_BYTES + kg * C::BK * C::KSTR;
      const char* sv = smem + (tile & 1) * C::TILE_BYTES + C::BKT * C::KSTR + kg * C::BK * C::VSTR;
      f32x16 s[2];
      {
        // all K fragments of the tile are requested before the first product, so the LDS latency is
        // paid once per tile instead of once per instruction
        bf16x8 ak[2][ND];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int dc = 0; dc < ND; ++dc)
            ak[kb][dc] = *reinterpret_cast<const bf16x8*>(sk + (kb * 32 + rw) * C::KSTR + dc * 32 + h * 16);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
          for (int j = 0; j < 16; ++j) s[kb][j] = 0.f;
#pragma unroll
          for (int dc = 0; dc < ND; ++dc)
            s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ak[kb][dc], bq[dc], s[kb], 0, 0, 0);
        }
      }
      // accumulator register j of block kb holds key k0 + kb*32 + 8*(j/4) + 4*h + (j%4) for row r
      const bool need_mask = (CAUSAL && k0 + C::BK - 1 > wave_first) || (k0 + C::BK > kv_end);
      if (need_mask) {
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int j = 0; j < 16; ++j) {
            const int key = k0 + kb * 32 + 8 * (j >> 2) + 4 * h + (j & 3);
            if (key >= kv_end || (CAUSAL && key > r)) s[kb][j] = -INFINITY;
          }
      }
      float mx = -INFINITY;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int j = 0; j < 16; ++j) mx = fmaxf(mx, s[kb][j]);
      mx = max_across_halves(mx);
      const float m_new = fmaxf(m_run, mx * c2);
      const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
      const float alpha = __builtin_amdgcn_exp2f(m_run - m_use);
      m_run = m_new;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int j = 0; j < 16; ++j) s[kb][j] = __builtin_amdgcn_exp2f(fmaf(s[kb][j], c2, -m_use));
      // Half-precision weights: their row sum is taken over the ROUNDED weights (pair . (1,1) accumulated in
      // float32), so numerator and denominator see the same weights.  Two-term bf16 weights: hi = bf16(p),
      // lo = bf16(p - hi); hi + lo is p to 2^-17, and the row sum is the plain float32 sum of p.
      f16x8 bp[2][2];
      bf16x8 bhi[2][2], blo[2][2];
      float psum = 0.f;
      const f16x2 ones = {(_Float16)1.0f, (_Float16)1.0f};
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
          for (int e = 0; e < 8; e += 2) {
            const float p0 = s[kb][8 * s2 + e], p1 = s[kb][8 * s2 + e + 1];
            if constexpr (SPLIT) {
              const bf16x2 hi = {(__bf16)p0, (__bf16)p1};
              const bf16x2 lo = {(__bf16)(p0 - (float)hi[0]), (__bf16)(p1 - (float)hi[1])};
              bhi[kb][s2][e] = hi[0];
              bhi[kb][s2][e + 1] = hi[1];
              blo[kb][s2][e] = lo[0];
              blo[kb][s2][e + 1] = lo[1];
              psum += p0 + p1;
            } else {
              f16x2 pr = {(_Float16)p0, (_Float16)p1};
              bp[kb][s2][e] = pr[0];
              bp[kb][s2][e + 1] = pr[1];
              psum = __builtin_amdgcn_fdot2(pr, ones, psum, false);
            }
          }
      l_run = fmaf(l_run, alpha, psum);
      if (__any(alpha != 1.f)) {
#pragma unroll
        for (int i = 0; i < NV; ++i)
#pragma unroll
          for (int j = 0; j < 16; ++j) o[i][j] *= alpha;
      }
      const int i16 = lane & 15, q2 = (lane >> 4) & 1;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
          const int key1 = kb * 32 + 16 * s2 + 4 * h + (i16 >> 2);
#pragma unroll
          for (int dvb = 0; dvb < NV; ++dvb) {
            const char* vp = sv + key1 * C::VSTR + (dvb * 32 + q2 * 16 + 4 * (i16 & 3)) * 2;
            const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(vp));
            const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(vp + 8 * C::VSTR));
            union { struct { s16x4 lo, hi; } s; f16x8 v; bf16x8 b; } av;
            av.s.lo = lo;
            av.s.hi = hi;
            if constexpr (SPLIT) {
              o[dvb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av.b, bhi[kb][s2], o[dvb], 0, 0, 0);
              o[dvb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av.b, blo[kb][s2], o[dvb], 0, 0, 0);
            } else {
              o[dvb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(av.v, bp[kb][s2], o[dvb], 0, 0, 0);
            }
          }
        }
    }
    if (more) store_tile((tile + 1) & 1);
    __syncthreads();
  }

  if (KG == 2) {
    // the second key group hands its running maximum, row sum and accumulator to the first through LDS
    // (element e of lane l at word e * 64 + l: conflict-free), which rescales both to the common maximum
    float* mg = reinterpret_cast<float*>(smem) + rg * (64 * (NV * 16 + 2)) + lane;
    if (kg == 1) {
#pragma unroll
      for (int i = 0; i < NV; ++i)
#pragma unroll
        for (int j = 0; j < 16; ++j) mg[(i * 16 + j) * 64] = o[i][j];
      mg[(NV * 16) * 64] = m_run;
      mg[(NV * 16 + 1) * 64] = l_run;
    }
    __syncthreads();
    if (kg == 1) return;
    const float m1 = mg[(NV * 16) * 64], l1 = mg[(NV * 16 + 1) * 64];
    const float m_new = fmaxf(m_run, m1);
    const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
    const float a0 = __builtin_amdgcn_exp2f(m_run - m_use), a1 = __builtin_amdgcn_exp2f(m1 - m_use);
#pragma unroll
    for (int i = 0; i < NV; ++i)
#pragma unroll
      for (int j = 0; j < 16; ++j) o[i][j] = o[i][j] * a0 + mg[(i * 16 + j) * 64] * a1;
    l_run = l_run * a0 + l1 * a1;
    m_run = m_new;
  }

  const float l_tot = sum_across_halves(l_run);
  float v_unscale = 1.f;
  if constexpr (!SPLIT) v_unscale = a.v_unscale[kvh];
  const float inv = v_unscale / l_tot;
  const size_t row0 = (size_t)batch * a.rows + wave_first;
  float* op0;
  float* lp0;
  if (a.n_split > 1) {
    const size_t prow = (size_t)split * a.n_batch * a.rows + row0;
    op0 = a.part_o + prow * D;
    lp0 = a.part_lse + prow;
  } else {
    op0 = a.out + row0 * D;
    lp0 = a.lse + row0;
  }
  // The wave's rows leave as whole rows through an LDS area of its own where the tile buffers have room for one per
  // storing wave (every read of the tiles lies behind the loop's last barrier; with two key groups the area is the
  // row group's merge area, which only this wave still touches); otherwise straight from the accumulator layout.
  constexpr int TURN = 32 * (D * 4 + 16);
  if constexpr (C::RG * TURN <= C::LDS_BYTES) {
    store_rows_via_lds<D>(o, inv, op0, a.rows - wave_first, smem + rg * TURN, lane);
  } else {
    if (r < a.rows) {
      float* op = op0 + (size_t)rw * D;
#pragma unroll
      for (int dvb = 0; dvb < NV; ++dvb)
#pragma unroll
        for (int j4 = 0; j4 < 4; ++j4) {
          f32x4 x;
#pragma unroll
          for (int e = 0; e < 4; ++e) x[e] = o[dvb][4 * j4 + e] * inv;
          *reinterpret_cast<f32x4*>(op + dvb * 32 + 8 * j4 + 4 * h) = x;
        }
    }
  }
  if (r < a.rows && h == 0) lp0[rw] = (m_run + __log2f(l_tot)) * kLn2;
}

template <int D, bool CAUSAL, int NW, int KG = 1, bool SPLIT = false>
__global__ __launch_bounds__(64 * NW, KG == 1 ? 2 : 1) void k_attn_bf16(AttnArgs a) {
  attn_bf16_body<D, CAUSAL, NW, KG, SPLIT>(a, blockIdx.x, blockIdx.y, blockIdx.z, gridDim.y);
}

// Both attentions of the path in ONE launch (same head dimension, same workgroup shape).  The query attention's
// workgroups come first in the linear order and each walks ALL keys for its rows (no key chunks, no partial results,
// no merge): such a workgroup lasts as long as the causal problem's longest row tile, which is handed out right
// behind it, so the query attention hides inside the causal one instead of waiting for it.  n_q_pad, the query
// workgroups rounded up to a multiple of 8, keeps the causal workgroups on the XCD slots map_block assumes.
struct PairGrid {
  int n_q, n_q_pad, q_gx, q_gy, c_gx, c_gy;
};
template <int D, int NW, int KG>
__global__ __launch_bounds__(64 * NW, KG == 1 ? 2 : 1) void k_attn_bf16_pair(AttnArgs ac, AttnArgs aq, PairGrid g) {
  const int bid = blockIdx.x;
  if (bid < g.n_q_pad) {
    if (bid >= g.n_q) return;
    attn_bf16_body<D, false, NW, KG>(aq, bid % g.q_gx, bid / g.q_gx, 0, g.q_gy);
  } else {
    const int l = bid - g.n_q_pad;
    attn_bf16_body<D, true, NW, KG>(ac, l % g.c_gx, l / g.c_gx, 0, g.c_gy);
  }
}

// ------------------------------------------------------ bf16, d = 128, asynchronous tile loads (LDS DMA)
// Eight waves x 32 rows, one workgroup per compute unit; same arithmetic and operand layouts as
// k_attn_bf16, with two changes to how a step is organised.
//
// (1) Software pipeline.  The products of the NEXT tile's scores are issued in the same straight-line
//     block as the softmax of the CURRENT tile, so the matrix pipe and the vector ALU of a SIMD work at
//     the same time without relying on a second wave being in the other phase:
//         step t:   S(t+1) = K(t+1) Q^T      (MFMA)   |   P(t) = exp2(S(t) c - m)      (VALU)
//                   O^T   += V(t)^T P(t)^T   (MFMA)
//     To keep that block free of branches a wave splits its tiles into `n_full` unmasked tiles (this
//     path) and at most one tail tile (the causal diagonal or the ragged end; plain path with masks),
//     and the running maximum is only raised when a row outgrows it by more than 2^8 ("lazy rescale"):
//     weights then stay below 256, which float32 sums and half-precision weights hold without loss, and the
//     rescale of O becomes a rare side branch ahead of the block.
// (2) Asynchronous tile loads.  K/V tiles travel from global memory straight into LDS
//     (global_load_lds_dwordx4: no staging registers, no LDS store instructions) into a ring of three K
//     slots and three V slots, two tiles ahead of their use, so a load has two full steps to land.
//
// A wave-wide DMA instruction fills 1 KB of LDS contiguously (lane i -> base + 16 i), i.e. four 256-byte
// rows with no room for padding, so the tiles are stored unpadded and XOR-swizzled instead: the 16-byte
// chunk c of row r sits at chunk position c ^ (r & 15) for K (16 consecutive rows of one fragment read
// land in 16 different bank groups) and at c ^ 4 (r & 3) for V: a transposing read takes, from each of 8 rows,
// the 64 bytes of one 4-chunk group, and LDS serves 32 lanes (4 of those rows) per cycle over its 64 banks, so the
// 4 rows have to sit in the 4 different groups.  (c ^ 2 (r & 7) spreads 16 lanes' 32-byte pieces instead; the
// counters showed every such read paying two extra cycles of bank conflicts.)  Which global chunk a lane fetches
// is free, so the swizzle costs nothing on the load side; on the read side it is folded into per-lane address
// registers.
template <bool CAUSAL>
__device__ __forceinline__ void attn_bf16_dma_body(const AttnArgs a, int bx, int by, int bz, int grid_y) {
  constexpr int D = 128, NW = 8, BQ = 32 * NW, BK = 64;
  constexpr int ND = D / 16, NV = D / 32;
  constexpr int TILE = BK * D * 2;  // 16 KB, unpadded
  constexpr int NSLOT = 3;
  constexpr float TAU = 8.f;
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  // K(j) in slot j % 3 at smem + slot * TILE; V(j) in slot j % 3 at smem + (3 + slot) * TILE

  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int rw = lane & 31, h = lane >> 5;
  int kvh, batch, qt;
  map_block(a, CAUSAL, bx, by, grid_y, &kvh, &batch, &qt);
  const int q0 = qt * BQ;
  const int split = bz;
  const int kv_begin = CAUSAL ? 0 : split * a.chunk;
  const int kv_end = CAUSAL ? min(a.m, q0 + BQ) : min(a.m, kv_begin + a.chunk);
  const int span = kv_end - kv_begin;
  const int n_tiles = (span + BK - 1) / BK;

  const int r = q0 + wave * 32 + rw;
  const int r_c = min(r, a.rows - 1);
  const int wave_first = q0 + wave * 32;
  // A wave whose rows all lie past the last row (the ragged last row tile of a problem: 4120 rows are 16 tiles and
  // 24 rows) computes nothing: no full tiles, no tail.  It still sends its share of the tile requests and meets the
  // barriers.  The last row tile is the one with the longest key range, so this is the most expensive workgroup of
  // every head, and its SIMDs are left to the waves that have rows.
  const bool has_rows = wave_first < a.rows;
  const int n_full = !has_rows ? 0
                     : CAUSAL  ? min((wave_first + 1) / BK, span / BK)
                               : min((wave_first + (1 << 24)) / BK, span / BK);
  const bool has_tail = has_rows && n_full * BK < span;

  bf16x8 bq[ND];
  {
    const char* qp = static_cast<const char*>(a.q) + ((size_t)batch * a.rows + r_c) * D * 2 + h * 16;
#pragma unroll
    for (int dc = 0; dc < ND; ++dc) bq[dc] = *reinterpret_cast<const bf16x8*>(qp + dc * 32);
  }
  const char* kbase = static_cast<const char*>(a.k) + ((size_t)kvh * a.m + kv_begin) * D * 2;
  const char* vbase = static_cast<const char*>(a.v) + ((size_t)kvh * a.m + kv_begin) * D * 2;

  // ---- DMA side: wave w, instruction i fills rows 4 (2w + i) .. + 3 of a tile; lane L lands at chunk
  //      position L & 15 of row 4 (2w + i) + (L >> 4) and therefore fetches the chunk that belongs there
  uint32_t goff_k[2], goff_v[2];
  int grow[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int row = 4 * (2 * wave + i) + (lane >> 4), pos = lane & 15;
    grow[i] = row;
    goff_k[i] = (uint32_t)(row * (D * 2) + ((pos ^ (row & 15)) * 16));
    goff_v[i] = (uint32_t)(row * (D * 2) + ((pos ^ (4 * (row & 3))) * 16));
  }
  // The DMA is issued through inline assembly on purpose: the compiler then neither orders later LDS
  // reads behind it (it would drain every outstanding load before each fragment read) nor counts it in
  // its own vmcnt bookkeeping; arrival is awaited by hand (s_waitcnt vmcnt) ahead of the barriers.
  // LDS destinations are handled as integers (LDS address of smem + byte offset, all scalar): a generic pointer
  // would drag a null check and 64-bit arithmetic into every request.  wave_rows: where this wave's rows start
  // inside a tile, as a scalar of its own; the row and mask arithmetic above keeps the per-lane `wave`.
  const uint32_t smem_at = (uint32_t)(size_t)(const __attribute__((address_space(3))) char*)smem;
  const uint32_t wave_rows = __builtin_amdgcn_readfirstlane((uint32_t)(2 * wave * 1024));
  auto dma16 = [&](const char* tile_base, uint32_t byte_off, uint32_t lds_off) {  // lds_off: byte offset into smem
    const uint32_t m0v = __builtin_amdgcn_readfirstlane(smem_at + lds_off);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(m0v), "v"(byte_off), "s"(tile_base)
                 : "memory", "m0");
  };
  auto dma_tile = [&](const char* base, int j, uint32_t slot, const uint32_t (&goff)[2], bool is_v) {
    const int k0 = j * BK;
    const char* tp = base + (size_t)k0 * (D * 2);
    if (kv_begin + k0 + BK <= a.m) {
#pragma unroll
      for (int i = 0; i < 2; ++i) dma16(tp, goff[i], slot + wave_rows + i * 1024);
    } else {
      // last tile of the cache: rows past the final key re-read that key (their scores are masked)
      const int last = a.m - 1 - kv_begin - k0;
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int row = grow[i], pos = lane & 15;
        const int src_chunk = is_v ? (pos ^ (4 * (row & 3))) : (pos ^ (row & 15));
        const uint32_t off = (uint32_t)(min(row, last) * (D * 2) + src_chunk * 16);
        dma16(tp, off, slot + wave_rows + i * 1024);
      }
    }
  };
  auto kslot = [&](int j) { return smem + (j % NSLOT) * TILE; };
  auto vslot = [&](int j) { return smem + (NSLOT + j % NSLOT) * TILE; };
  auto kslot_off = [&](int j) { return (uint32_t)((j % NSLOT) * TILE); };  // the same as byte offsets, for the requests
  auto vslot_off = [&](int j) { return (uint32_t)((NSLOT + j % NSLOT) * TILE); };

  // ---- read side: per-lane swizzled byte offsets inside a slot
  uint32_t kaddr[ND], vaddr[NV];
  {
    const int x = rw & 15;
#pragma unroll
    for (int dc = 0; dc < ND; ++dc) kaddr[dc] = (uint32_t)(rw * 256 + (((2 * dc + h) ^ x) * 16));
    const int i16 = lane & 15, q2 = (lane >> 4) & 1;
    const int vrow = 4 * h + (i16 >> 2);       // + kb*32 + s2*16 (+8): multiples of 8, do not change row & 3
    const int xv = 4 * (vrow & 3);
#pragma unroll
    for (int dvb = 0; dvb < NV; ++dvb) {
      const int c = 4 * dvb + 2 * q2 + ((i16 & 3) >> 1);
      vaddr[dvb] = (uint32_t)(vrow * 256 + ((c ^ xv) * 16) + 8 * (i16 & 1));
    }
  }

  f32x16 o[NV];
#pragma unroll
  for (int i = 0; i < NV; ++i)
#pragma unroll
    for (int j = 0; j < 16; ++j) o[i][j] = 0.f;
  float m_ref = -INFINITY, l_run = 0.f;
  const float c2 = a.scale * kLog2e;

  auto lift = [&](float mx) {
    if (__any(mx > m_ref + TAU)) {
      const float m_new = fmaxf(m_ref, mx);
      const float al = __builtin_amdgcn_exp2f(m_ref - m_new);
      l_run *= al;
#pragma unroll
      for (int i = 0; i < NV; ++i)
#pragma unroll
        for (int j = 0; j < 16; ++j) o[i][j] *= al;
      m_ref = m_new;
    }
  };
  auto row_max = [&](const f32x16 (&s)[2]) {
    float mx = -INFINITY;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int j = 0; j < 16; ++j) mx = fmaxf(mx, s[kb][j]);
    mx = max_across_halves(mx);
    return mx * c2;
  };
  auto kfrags = [&](const char* ks, int kb, bf16x8 (&ak)[ND]) {
#pragma unroll
    for (int dc = 0; dc < ND; ++dc) ak[dc] = *reinterpret_cast<const bf16x8*>(ks + kaddr[dc] + kb * 32 * 256);
  };
  // V^T fragments of key group g (16 keys) for the NV blocks of O^T: two transposing reads each
  auto vfrags = [&](const char* vs, int g, f16x8 (&av)[NV]) {
#pragma unroll
    for (int dvb = 0; dvb < NV; ++dvb) {
      const char* vp = vs + vaddr[dvb] + g * 16 * 256;
      const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(vp));
      const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(vp + 8 * 256));
      union { struct { s16x4 lo, hi; } s; f16x8 v; } u;
      u.s.lo = lo;
      u.s.hi = hi;
      av[dvb] = u.v;
    }
  };
  // LDS reads may not be moved across this point (everything else may): keeps a fragment load where it was written,
  // i.e. one group of products ahead of its use, instead of right in front of it
  constexpr int kHoldLds = 0x47F;
  auto weights_pv = [&](f32x16 (&s)[2], const char* vs, float m_use) {
    f16x8 bp[2][2];
    f16x8 va[2][NV];
    vfrags(vs, 0, va[0]);  // lands while the weights are computed
    __builtin_amdgcn_sched_barrier(kHoldLds);
    float psum = 0.f;
    const f16x2 ones = {(_Float16)1.0f, (_Float16)1.0f};
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
        for (int e = 0; e < 8; e += 2) {
          const float p0 = __builtin_amdgcn_exp2f(fmaf(s[kb][8 * s2 + e], c2, -m_use));
          const float p1 = __builtin_amdgcn_exp2f(fmaf(s[kb][8 * s2 + e + 1], c2, -m_use));
          f16x2 pr = {(_Float16)p0, (_Float16)p1};
          bp[kb][s2][e] = pr[0];
          bp[kb][s2][e + 1] = pr[1];
          psum = __builtin_amdgcn_fdot2(pr, ones, psum, false);
        }
    l_run += psum;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      if (g + 1 < 4) {
        vfrags(vs, g + 1, va[(g + 1) & 1]);
        __builtin_amdgcn_sched_barrier(kHoldLds);
      }
#pragma unroll
      for (int dvb = 0; dvb < NV; ++dvb)
        o[dvb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(va[g & 1][dvb], bp[g >> 1][g & 1], o[dvb], 0, 0, 0);
    }
  };

  // ---- prologue: K(0), V(0), K(1) must have landed; V(1), K(2) stay in flight
  dma_tile(kbase, 0, kslot_off(0), goff_k, false);
  dma_tile(vbase, 0, vslot_off(0), goff_v, true);
  if (n_tiles > 1) dma_tile(kbase, 1, kslot_off(1), goff_k, false);
  if (n_tiles > 1) dma_tile(vbase, 1, vslot_off(1), goff_v, true);
  if (n_tiles > 2) dma_tile(kbase, 2, kslot_off(2), goff_k, false);
  if (n_tiles > 2) __builtin_amdgcn_s_waitcnt(0x0F70 | 4);        // vmcnt(4): everything but V(1), K(2)
  else if (n_tiles > 1) __builtin_amdgcn_s_waitcnt(0x0F70 | 2);   // vmcnt(2): everything but V(1)
  else __builtin_amdgcn_s_waitcnt(0x0F70);                         // vmcnt(0)
  __builtin_amdgcn_s_barrier();
  f32x16 sA[2], sB[2];
  {
    bf16x8 ak0[ND], ak1[ND];
    kfrags(kslot(0), 0, ak0);
    kfrags(kslot(0), 1, ak1);
#pragma unroll
    for (int j = 0; j < 16; ++j) { sA[0][j] = 0.f; sA[1][j] = 0.f; }
#pragma unroll
    for (int dc = 0; dc < ND; ++dc) sA[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ak0[dc], bq[dc], sA[0], 0, 0, 0);
#pragma unroll
    for (int dc = 0; dc < ND; ++dc) sA[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ak1[dc], bq[dc], sA[1], 0, 0, 0);
  }
  __builtin_amdgcn_s_barrier();  // K(0) has been read by every wave before step 0 refills its slot with K(3)

  // step `tile`: S(tile) is in sc; computes S(tile + 1) into sn and adds tile's V contribution
  auto step = [&](int tile, f32x16 (&sc)[2], f32x16 (&sn)[2]) {
    const bool more_k = tile + 3 < n_tiles, more_v = tile + 2 < n_tiles;
    if (more_k) dma_tile(kbase, tile + 3, kslot_off(tile + 3), goff_k, false);
    if (more_v) dma_tile(vbase, tile + 2, vslot_off(tile + 2), goff_v, true);
    const char* k_next = kslot(tile + 1);
    const char* v_cur = vslot(tile);
    if (tile < n_full) {
      bf16x8 ak0[ND], ak1[ND];
      kfrags(k_next, 0, ak0);
      lift(row_max(sc));
      kfrags(k_next, 1, ak1);
#pragma unroll
      for (int j = 0; j < 16; ++j) { sn[0][j] = 0.f; sn[1][j] = 0.f; }
#pragma unroll
      for (int dc = 0; dc < ND; ++dc) sn[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ak0[dc], bq[dc], sn[0], 0, 0, 0);
#pragma unroll
      for (int dc = 0; dc < ND; ++dc) sn[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ak1[dc], bq[dc], sn[1], 0, 0, 0);
      weights_pv(sc, v_cur, m_ref);
    } else if (tile == n_full && has_tail) {
      const int k0 = kv_begin + tile * BK;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int j = 0; j < 16; ++j) {
          const int key = k0 + kb * 32 + 8 * (j >> 2) + 4 * h + (j & 3);
          if (key >= kv_end || (CAUSAL && key > r)) sc[kb][j] = -INFINITY;
        }
      lift(row_max(sc));
      weights_pv(sc, v_cur, m_ref == -INFINITY ? 0.f : m_ref);
    }
    // the tiles needed by the next step were requested one step ago: wait for all but this step's loads
    if (more_k) __builtin_amdgcn_s_waitcnt(0x0F70 | 4);
    else if (more_v) __builtin_amdgcn_s_waitcnt(0x0F70 | 2);
    else __builtin_amdgcn_s_waitcnt(0x0F70);
    __builtin_amdgcn_s_barrier();
  };
  for (int tile = 0; tile < n_tiles; tile += 2) {
    step(tile, sA, sB);
    if (tile + 1 < n_tiles) step(tile + 1, sB, sA);
  }

  const float l_tot = sum_across_halves(l_run);
  const float inv = a.v_unscale[kvh] / l_tot;
  const size_t row0 = (size_t)batch * a.rows + wave_first;
  float* op0;
  float* lp0;
  if (a.n_split > 1) {
    const size_t prow = (size_t)split * a.n_batch * a.rows + row0;
    op0 = a.part_o + prow * D;
    lp0 = a.part_lse + prow;
  } else {
    op0 = a.out + row0 * D;
    lp0 = a.lse + row0;
  }
  // whole rows through the wave's 12 KB share of the tile slots (free: the last step ended with every request
  // landed and a barrier), 16 rows at a time
  store_rows_via_lds<D, 2>(o, inv, op0, a.rows - wave_first, smem + wave * (2 * NSLOT * TILE / NW), lane);
  if (r < a.rows && h == 0) lp0[rw] = (m_ref + __log2f(l_tot)) * kLn2;
}

template <bool CAUSAL>
__global__ __launch_bounds__(512, 2) void k_attn_bf16_dma(AttnArgs a) {
  attn_bf16_dma_body<CAUSAL>(a, blockIdx.x, blockIdx.y, blockIdx.z, gridDim.y);
}

// the pair launch (see k_attn_bf16_pair) of the asynchronous kernel
__global__ __launch_bounds__(512, 2) void k_attn_bf16_dma_pair(AttnArgs ac, AttnArgs aq, PairGrid g) {
  const int bid = blockIdx.x;
  if (bid < g.n_q_pad) {
    if (bid >= g.n_q) return;
    attn_bf16_dma_body<false>(aq, bid % g.q_gx, bid / g.q_gx, 0, g.q_gy);
  } else {
    const int l = bid - g.n_q_pad;
    attn_bf16_dma_body<true>(ac, l % g.c_gx, l / g.c_gx, 0, g.c_gy);
  }
}

// ------------------------------------------------------------------------------------------- f32
template <int D, bool CAUSAL>
__global__ __launch_bounds__(256) void k_attn_f32(AttnArgs a) {
  constexpr int BK = 32, R = 4, RB = 16, KS = D + 1, NC = D / 64;
  __shared__ float sK[BK * KS];
  __shared__ float sV[BK * D];
  __shared__ float sQ[RB * D];
  __shared__ float sP[RB * BK];
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int kx = lane & 31, ch = lane >> 5;
  int kvh, batch, qt;
  map_block(a, CAUSAL, blockIdx.x, blockIdx.y, gridDim.y, &kvh, &batch, &qt);
  const int q0 = qt * RB;
  const int split = blockIdx.z;
  const int kv_begin = CAUSAL ? 0 : split * a.chunk;
  const int kv_end = CAUSAL ? min(a.m, q0 + RB) : min(a.m, kv_begin + a.chunk);
  const int n_tiles = (kv_end - kv_begin + BK - 1) / BK;
  const float* q = static_cast<const float*>(a.q);
  const float* kbase = static_cast<const float*>(a.k) + (size_t)kvh * a.m * D;
  const float* vbase = static_cast<const float*>(a.v) + (size_t)kvh * a.m * D;

  for (int i = t; i < RB * D; i += 256) {
    const int rc = min(q0 + i / D, a.rows - 1);
    sQ[i] = q[((size_t)batch * a.rows + rc) * D + i % D];
  }
  float m_run[R], l_run[R], o[R][NC];
#pragma unroll
  for (int rr = 0; rr < R; ++rr) {
    m_run[rr] = -INFINITY;
    l_run[rr] = 0.f;
#pragma unroll
    for (int cc = 0; cc < NC; ++cc) o[rr][cc] = 0.f;
  }

  for (int tile = 0; tile < n_tiles; ++tile) {
    const int k0 = kv_begin + tile * BK;
    __syncthreads();
    for (int i = t; i < BK * D; i += 256) {
      const int row = i / D, c = i % D;
      const size_t off = (size_t)min(k0 + row, a.m - 1) * D + c;
      sK[row * KS + c] = kbase[off];
      sV[row * D + c] = vbase[off];
    }
    __syncthreads();
    float s[R];
#pragma unroll
    for (int rr = 0; rr < R; ++rr) s[rr] = 0.f;
    for (int i = 0; i < D / 2; ++i) {
      // the two half-waves walk the channels half a bank cycle apart
      const int c = ch ? D / 2 + ((i + 32) % (D / 2)) : i;
      const float kv = sK[kx * KS + c];
#pragma unroll
      for (int rr = 0; rr < R; ++rr) s[rr] = fmaf(sQ[(wave * R + rr) * D + c], kv, s[rr]);
    }
    const int key = k0 + kx;
#pragma unroll
    for (int rr = 0; rr < R; ++rr) {
      const int row = q0 + wave * R + rr;
      float x = s[rr] + __shfl_xor(s[rr], 32);
      x = (key >= kv_end || (CAUSAL && key > row)) ? -INFINITY : x * a.scale;
      float mx = x;
#pragma unroll
      for (int off = 16; off >= 1; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
      const float m_new = fmaxf(m_run[rr], mx);
      const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
      const float p = expf(x - m_use);
      float sum = p;
#pragma unroll
      for (int off = 16; off >= 1; off >>= 1) sum += __shfl_xor(sum, off);
      const float alpha = expf(m_run[rr] - m_use);
      l_run[rr] = l_run[rr] * alpha + sum;
#pragma unroll
      for (int cc = 0; cc < NC; ++cc) o[rr][cc] *= alpha;
      m_run[rr] = m_new;
      if (ch == 0) sP[(wave * R + rr) * BK + kx] = p;
    }
    __syncthreads();
    for (int j = 0; j < BK; ++j) {
#pragma unroll
      for (int cc = 0; cc < NC; ++cc) {
        const float vv = sV[j * D + lane + 64 * cc];
#pragma unroll
        for (int rr = 0; rr < R; ++rr) o[rr][cc] = fmaf(sP[(wave * R + rr) * BK + j], vv, o[rr][cc]);
      }
    }
  }
#pragma unroll
  for (int rr = 0; rr < R; ++rr) {
    const int row = q0 + wave * R + rr;
    if (row >= a.rows) continue;
    const size_t row_id = (size_t)batch * a.rows + row;
    float* op;
    float* lp;
    if (a.n_split > 1) {
      const size_t prow = (size_t)split * a.n_batch * a.rows + row_id;
      op = a.part_o + prow * D;
      lp = a.part_lse + prow;
    } else {
      op = a.out + row_id * D;
      lp = a.lse + row_id;
    }
    const float inv = 1.f / l_run[rr];
#pragma unroll
    for (int cc = 0; cc < NC; ++cc) op[lane + 64 * cc] = o[rr][cc] * inv;
    if (lane == 0) *lp = m_run[rr] + logf(l_run[rr]);
  }
}

// out = sum_s w_s * part_o[s] with w_s = exp(lse_s - lse), lse = log sum_s exp(lse_s).  One thread per four
// channels (16-byte loads), d/4 threads per row; chunks are visited in order, so the result is deterministic.
__global__ __launch_bounds__(256) void k_attn_merge(AttnArgs a, int d) {
  const int tpr = d / 4, rpb = 256 / tpr;
  const size_t n_rows = (size_t)a.n_batch * a.rows;
  const size_t row = (size_t)blockIdx.x * rpb + threadIdx.x / tpr;
  const int c4 = threadIdx.x % tpr;
  if (row >= n_rows) return;
  float mx = -INFINITY;
  for (int s = 0; s < a.n_split; ++s) mx = fmaxf(mx, a.part_lse[(size_t)s * n_rows + row]);
  float den = 0.f;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  for (int s = 0; s < a.n_split; ++s) {
    const float w = expf(a.part_lse[(size_t)s * n_rows + row] - mx);
    const f32x4 x = *reinterpret_cast<const f32x4*>(a.part_o + ((size_t)s * n_rows + row) * d + c4 * 4);
    den += w;
#pragma unroll
    for (int e = 0; e < 4; ++e) acc[e] = fmaf(w, x[e], acc[e]);
  }
  const float inv = 1.f / den;
#pragma unroll
  for (int e = 0; e < 4; ++e) acc[e] *= inv;
  *reinterpret_cast<f32x4*>(a.out + row * d + c4 * 4) = acc;
  if (c4 == 0) a.lse[row] = mx + logf(den);
}

AttnArgs make_args(const AttnLaunch& l) {
  AttnArgs a;
  a.q = l.q; a.k = l.k; a.v = l.v; a.v_unscale = l.v_unscale; a.out = l.out; a.lse = l.lse;
  a.part_o = l.part_o; a.part_lse = l.part_lse;
  a.rows = l.rows; a.m = l.m; a.batch_per_kv = l.batch_per_kv; a.n_batch = l.n_batch;
  a.n_split = l.causal ? 1 : l.n_split;
  a.chunk = l.chunk; a.scale = l.scale;
  a.kv_groups = 0;
  return a;
}

// Grid of an attention launch over `tiles` row tiles, and the matching kv_groups of the arguments.
dim3 attn_grid(AttnArgs* a, int tiles) {
  const int n_kv = a->n_batch / a->batch_per_kv;
  if (n_kv % 8 == 0 && (long long)tiles * (n_kv / 8) <= 65535) {
    a->kv_groups = n_kv / 8;
    return dim3(8 * a->batch_per_kv, tiles * a->kv_groups, a->n_split);
  }
  a->kv_groups = 0;
  return dim3(a->n_batch, tiles, a->n_split);
}

constexpr int kDmaLdsBytes = 6 * 64 * 256;

template <int D, bool CAUSAL, int NW, int KG = 1, bool SPLIT = false>
hipError_t raise_lds_limit() {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(&k_attn_bf16<D, CAUSAL, NW, KG, SPLIT>),
                             hipFuncAttributeMaxDynamicSharedMemorySize, Bf16Cfg<D, NW, KG>::LDS_BYTES);
}
template <int D, int NW, int KG>
hipError_t raise_lds_limit_pair() {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(&k_attn_bf16_pair<D, NW, KG>),
                             hipFuncAttributeMaxDynamicSharedMemorySize, Bf16Cfg<D, NW, KG>::LDS_BYTES);
}

template <int D, bool CAUSAL, int NW, int KG = 1, bool SPLIT = false>
hipError_t run_bf16(const AttnLaunch& l, hipStream_t s) {
  using C = Bf16Cfg<D, NW, KG>;
  AttnArgs a = make_args(l);
  dim3 grid = attn_grid(&a, (l.rows + C::BQ - 1) / C::BQ);
  hipLaunchKernelGGL((k_attn_bf16<D, CAUSAL, NW, KG, SPLIT>), grid, dim3(C::NT), C::LDS_BYTES, s, a);
  return hipGetLastError();
}

template <bool CAUSAL>
hipError_t run_bf16_dma(const AttnLaunch& l, hipStream_t s) {
  AttnArgs a = make_args(l);
  dim3 grid = attn_grid(&a, (l.rows + 255) / 256);
  hipLaunchKernelGGL((k_attn_bf16_dma<CAUSAL>), grid, dim3(512), kDmaLdsBytes, s, a);
  return hipGetLastError();
}

// Which bf16 kernel serves a problem.
enum class Shape { kDma, kWaves8, kWaves8Keys2, kWaves4 };
Shape bf16_shape(const AttnLaunch& l) {
  // the asynchronous kernel serves the long problems (d = 128, enough row tiles for 8 waves)
  if (attn_bf16_waves(l.causal, l.n_batch, l.rows) == 8) return l.d == 128 ? Shape::kDma : Shape::kWaves8;
  // short causal problems (at most two workgroups per compute unit): 128 rows per workgroup as with four waves, but
  // two key groups halve the chain of steps of the longest row tile, which is what such a launch waits for
  if (l.causal && l.rows > 256 && (long long)l.n_batch * ((l.rows + 127) / 128) <= 512) return Shape::kWaves8Keys2;
  return Shape::kWaves4;
}

template <int D, bool CAUSAL>
hipError_t run_bf16_nw(const AttnLaunch& l, hipStream_t s) {
  if (attn_bf16_reads_v16(l) != (l.v_unscale != nullptr)) return hipErrorInvalidValue;  // V prepared iff the shape reads the copy
  switch (bf16_shape(l)) {
    case Shape::kDma:
      if constexpr (D == 128) return run_bf16_dma<CAUSAL>(l, s);
      return hipErrorInvalidValue;
    case Shape::kWaves8: return run_bf16<D, CAUSAL, 8>(l, s);
    case Shape::kWaves8Keys2:
      if constexpr (CAUSAL) return run_bf16<D, CAUSAL, 8, 2>(l, s);
      return hipErrorInvalidValue;
    default:
      if constexpr (CAUSAL) return run_bf16<D, true, 4>(l, s);
      return run_bf16<D, false, 4, 1, true>(l, s);  // two-term weights, V as stored
  }
}

// Pair launch: the query problem takes the causal problem's kernel shape and walks all keys in one chunk.
bool pair_grid(AttnArgs* ac, AttnArgs* aq, int bq, PairGrid* g, unsigned* total) {
  const dim3 gc = attn_grid(ac, (ac->rows + bq - 1) / bq), gq = attn_grid(aq, (aq->rows + bq - 1) / bq);
  g->c_gx = (int)gc.x; g->c_gy = (int)gc.y; g->q_gx = (int)gq.x; g->q_gy = (int)gq.y;
  const long long n_q = (long long)gq.x * gq.y, n_c = (long long)gc.x * gc.y;
  const long long n_q_pad = (n_q + 7) / 8 * 8;
  if (n_q_pad + n_c > 0x7FFFFFFFll) return false;
  g->n_q = (int)n_q; g->n_q_pad = (int)n_q_pad;
  *total = (unsigned)(n_q_pad + n_c);
  return true;
}

template <int D, int NW, int KG>
hipError_t run_pair(const AttnLaunch& c, const AttnLaunch& q, hipStream_t s) {
  using C = Bf16Cfg<D, NW, KG>;
  AttnArgs ac = make_args(c), aq = make_args(q);
  PairGrid g;
  unsigned total;
  if (!pair_grid(&ac, &aq, C::BQ, &g, &total)) return hipErrorInvalidValue;
  hipLaunchKernelGGL((k_attn_bf16_pair<D, NW, KG>), dim3(total), dim3(C::NT), C::LDS_BYTES, s, ac, aq, g);
  return hipGetLastError();
}

hipError_t run_pair_dma(const AttnLaunch& c, const AttnLaunch& q, hipStream_t s) {
  AttnArgs ac = make_args(c), aq = make_args(q);
  PairGrid g;
  unsigned total;
  if (!pair_grid(&ac, &aq, 256, &g, &total)) return hipErrorInvalidValue;
  hipLaunchKernelGGL(k_attn_bf16_dma_pair, dim3(total), dim3(512), kDmaLdsBytes, s, ac, aq, g);
  return hipGetLastError();
}

template <int D>
hipError_t run_pair_d(const AttnLaunch& c, const AttnLaunch& q, hipStream_t s) {
  switch (bf16_shape(c)) {
    case Shape::kDma:
      if constexpr (D == 128) return run_pair_dma(c, q, s);
      return hipErrorInvalidValue;
    case Shape::kWaves8: return run_pair<D, 8, 1>(c, q, s);
    case Shape::kWaves8Keys2: return run_pair<D, 8, 2>(c, q, s);
    default: return run_pair<D, 4, 1>(c, q, s);
  }
}

template <int D, bool CAUSAL>
hipError_t run_f32(const AttnLaunch& l, hipStream_t s) {
  AttnArgs a = make_args(l);
  dim3 grid = attn_grid(&a, (l.rows + 15) / 16);
  hipLaunchKernelGGL((k_attn_f32<D, CAUSAL>), grid, dim3(256), 0, s, a);
  return hipGetLastError();
}

}  // namespace

// Every bf16 attention kernel uses more dynamic LDS than the default limit allows; the limit belongs to the function
// on a device, so it is raised for ALL variants the first time any attention call runs on that device.  After that
// no attention call touches anything but the stream, whatever variant its shape selects (HIP graph capture).
hipError_t attn_prepare_device() {
  constexpr int kMaxDev = 64;
  static std::mutex mu;
  static bool done[kMaxDev] = {};
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDev) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(mu);
  if (done[dev]) return hipSuccess;
  const hipError_t all[] = {
      raise_lds_limit<128, true, 8>(),     raise_lds_limit<128, false, 8>(), raise_lds_limit<128, true, 4>(),
      raise_lds_limit<128, false, 4, 1, true>(), raise_lds_limit<128, true, 8, 2>(), raise_lds_limit<64, true, 8>(),
      raise_lds_limit<64, false, 8>(),     raise_lds_limit<64, true, 4>(),   raise_lds_limit<64, false, 4, 1, true>(),
      raise_lds_limit<64, true, 8, 2>(),
      hipFuncSetAttribute(reinterpret_cast<const void*>(&k_attn_bf16_dma<true>),
                          hipFuncAttributeMaxDynamicSharedMemorySize, kDmaLdsBytes),
      hipFuncSetAttribute(reinterpret_cast<const void*>(&k_attn_bf16_dma<false>),
                          hipFuncAttributeMaxDynamicSharedMemorySize, kDmaLdsBytes),
      raise_lds_limit_pair<128, 8, 1>(),   raise_lds_limit_pair<128, 8, 2>(), raise_lds_limit_pair<128, 4, 1>(),
      raise_lds_limit_pair<64, 8, 1>(),    raise_lds_limit_pair<64, 8, 2>(),  raise_lds_limit_pair<64, 4, 1>(),
      hipFuncSetAttribute(reinterpret_cast<const void*>(&k_attn_bf16_dma_pair),
                          hipFuncAttributeMaxDynamicSharedMemorySize, kDmaLdsBytes)};
  for (hipError_t x : all)
    if (x != hipSuccess) return x;
  done[dev] = true;
  return hipSuccess;
}

bool attn_bf16_reads_v16(const AttnLaunch& l) { return l.causal || bf16_shape(l) != Shape::kWaves4; }

hipError_t launch_attn_bf16(const AttnLaunch& l, hipStream_t s) {
  const hipError_t e = attn_prepare_device();
  if (e != hipSuccess) return e;
  if (l.d == 128) return l.causal ? run_bf16_nw<128, true>(l, s) : run_bf16_nw<128, false>(l, s);
  return l.causal ? run_bf16_nw<64, true>(l, s) : run_bf16_nw<64, false>(l, s);
}

hipError_t launch_attn_bf16_pair(const AttnLaunch& causal, const AttnLaunch& query, hipStream_t s) {
  const hipError_t e = attn_prepare_device();
  if (e != hipSuccess) return e;
  if (causal.v_unscale == nullptr || query.v != causal.v) return hipErrorInvalidValue;  // both read the prepared copy
  AttnLaunch q = query;
  q.n_split = 1;
  q.chunk = q.m;
  q.part_o = nullptr;
  q.part_lse = nullptr;
  return causal.d == 128 ? run_pair_d<128>(causal, q, s) : run_pair_d<64>(causal, q, s);
}

hipError_t launch_attn_f32(const AttnLaunch& l, hipStream_t s) {
  if (l.d == 128) return l.causal ? run_f32<128, true>(l, s) : run_f32<128, false>(l, s);
  return l.causal ? run_f32<64, true>(l, s) : run_f32<64, false>(l, s);
}

hipError_t launch_attn_merge(const AttnLaunch& l, hipStream_t s) {
  AttnArgs a = make_args(l);
  const int rpb = 256 / (l.d / 4);
  const size_t n_rows = (size_t)l.n_batch * l.rows;
  hipLaunchKernelGGL(k_attn_merge, dim3((unsigned)((n_rows + rpb - 1) / rpb)), dim3(256), 0, s, a, l.d);
  return hipGetLastError();
}

}  // namespace samkv
