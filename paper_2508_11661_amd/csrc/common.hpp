// Shared declarations of the SamKV HIP library (gfx950 only): kernel-argument tables, small device
// helpers and the host-side launch entry points that samkv_api.hip calls.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/samkv.h"

namespace samkv {

// Per-document pointers and prefix sums travel to the kernels by value in the kernel-argument
// segment (no device allocation, no host-to-device copy, nothing for a later call to race with).
struct PtrTable {
  const void* p[SAMKV_MAX_CTX];
};
struct IntTable {
  int32_t v[SAMKV_MAX_CTX + 1];
};

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

// ---- host-side launchers (one per translation unit) -------------------------------------------
struct ScoreLaunch {
  int n_ctx, hq, hkv, d, dtype, n_q_tok, w_loc, max_len, total_len;
  const void* q_tok;
  const void* q_loc;  // may be null
  float* scores;
  float* ws_que;    // [Hq][d]
  float* ws_loc;    // [N][Hq][d]
  float* ws_w;      // [N][Hq]
  float* ws_base;   // [Hq][d]  sum over all documents of |cos| * Q_loc
  float* ws_qt;     // [N][Hkv][d]
};
hipError_t launch_score(const ScoreLaunch& a, const PtrTable& k, const IntTable& cu_len, hipStream_t s);
// Where the per-document vectors of Eq. 1 are after the prologue: [N][heads][d] float32, of which `group`
// consecutive heads are averaged into the vector of one KV head.
struct QuerySrc {
  const float* q;
  int heads, group;
};
hipError_t launch_score_prologue(const ScoreLaunch& a, hipStream_t s, QuerySrc* q);

struct SelectLaunch {
  int n_ctx, hkv, max_len, total_len, m_total, n_sink, n_local;
  const float* scores;
  int32_t* idx;
  int32_t* cu_k_dev;  // may be null
};
hipError_t launch_select(const SelectLaunch& a, const IntTable& cu_len, const IntTable& cu_k, hipStream_t s);

constexpr int kFusedMaxLen = 8192;
constexpr int kFusedGatherMaxRows = 2048;  // (document, KV head) rows up to which the fused call also compacts in-kernel

hipError_t launch_block_scores(const float* scores, const IntTable& cu_len, const IntTable& cu_blk, int n_ctx, int hkv,
                               int total_len, int block, float* bscores, hipStream_t s);
hipError_t launch_expand_blocks(const int32_t* bidx, const IntTable& cu_len, const IntTable& cu_kb, const IntTable& cu_k,
                                int n_ctx, int hkv, int block, int32_t* idx, int32_t* cu_k_dev, hipStream_t s);

hipError_t launch_gather_g(int row_bytes, const PtrTable& a, const PtrTable* b, const IntTable& cu_len, int n_ctx, int heads,
                           int group, int m_total, const int32_t* gidx, void* a_out, void* b_out, hipStream_t s);
hipError_t launch_normalize(const float* bscores, const int32_t* bidx, const IntTable& cu_blk, const IntTable& cu_kb,
                            int n_ctx, int hkv, int n_init, int n_local, float* cand, hipStream_t s);
hipError_t launch_filter_expand(const int32_t* sel, const int32_t* bidx, const IntTable& cu_len, const IntTable& cu_kb,
                                int n_ctx, int hkv, int n_sel, int m_total, int block, int32_t* start, int32_t* tok_off,
                                int32_t* gidx, hipStream_t s);

hipError_t launch_peak_mfma(float* sink, int n_blocks, int iters, int pattern, hipStream_t s);
hipError_t launch_peak_copy(const void* src, void* dst, size_t bytes, hipStream_t s);
hipError_t launch_peak_read(const void* src, size_t bytes, uint32_t* sink, hipStream_t s);

struct GatherLaunch {
  int n_ctx, hkv, row_bytes, m_total, max_k;
  const int32_t* idx;
  void* k_c;
  void* v_c;
};
hipError_t launch_gather(const GatherLaunch& a, const PtrTable& k, const PtrTable& v, const IntTable& cu_len,
                         const IntTable& cu_k, hipStream_t s);
// Score and selection in one pass over K (rows of at most kFusedMaxLen tokens): a.scores may be null.  With `ga`
// and `v` the same workgroups also compact the kept K and V rows (what launch_gather does).
hipError_t launch_score_select(const ScoreLaunch& a, const SelectLaunch& sl, const PtrTable& k, const IntTable& cu_len,
                               const IntTable& cu_k, hipStream_t s, const GatherLaunch* ga = nullptr,
                               const PtrTable* v = nullptr);
// Q-cache variant: a.k_c receives [Hq][M][d]; q holds per-document [Hq][L_i][d]
hipError_t launch_gather_q(const GatherLaunch& a, const PtrTable& q, const IntTable& cu_len, const IntTable& cu_k,
                           int hq, hipStream_t s);

// Waves per workgroup of the bf16 attention kernel (each wave owns 32 query rows).  Eight waves share
// one K/V tile stream between twice as many rows; that pays once there are enough row tiles to keep
// every compute unit busy, otherwise four waves give more workgroups to spread.
#ifndef SAMKV_WAVE8_MIN_TILES
#define SAMKV_WAVE8_MIN_TILES 384  // causal: number of 256-row tiles (1.5 per compute unit) from which eight waves pay; measured
#endif
inline int attn_bf16_waves(int causal, int n_batch, int rows) {
  if (causal) return (long long)n_batch * ((rows + 255) / 256) >= SAMKV_WAVE8_MIN_TILES ? 8 : 4;
  return rows >= 512 ? 8 : 4;   // not causal: from two 256-row tiles per KV head on (measured at 256 / 512 / 1024 rows)
}

// One attention problem: `n_batch` independent row blocks, batch b reads KV head b / batch_per_kv.
// Row r of a batch attends keys [0, r] (causal) or [0, m) (not causal).
struct AttnLaunch {
  int dtype, d, causal;
  int n_batch, batch_per_kv, rows, m;
  const void* q;   // [n_batch][rows][d]
  const void* k;   // [n_batch / batch_per_kv][m][d]
  const void* v;   // bf16 kernels that read the copy (attn_bf16_reads_v16): what launch_v_prep wrote; otherwise V itself
  const float* v_unscale;  // with the copy: [n_batch / batch_per_kv] factors that undo its power-of-two scale; else null
  float* out;      // [n_batch][rows][d]
  float* lse;      // [n_batch][rows]
  float scale;
  int n_split, chunk;  // keys are cut into n_split chunks of `chunk` keys (not causal only)
  float* part_o;       // [n_split][n_batch][rows][d]   workspace when n_split > 1
  float* part_lse;     // [n_split][n_batch][rows]
};
hipError_t launch_attn_bf16(const AttnLaunch& a, hipStream_t s);
// Whether the bf16 kernel that serves this problem reads the scaled half-precision copy of V (every causal problem,
// long problems that are not causal) or V as stored (the four-wave kernel of a problem that is not causal).  A pair
// launch always reads the copy.
bool attn_bf16_reads_v16(const AttnLaunch& a);
// Both bf16 attentions of the path in one launch: `causal` and `query` share d, K and the prepared V; the query
// attention runs without key chunks whatever `query` says (its n_split, chunk and partial buffers are ignored).
hipError_t launch_attn_bf16_pair(const AttnLaunch& causal, const AttnLaunch& query, hipStream_t s);
hipError_t launch_attn_f32(const AttnLaunch& a, hipStream_t s);
hipError_t launch_attn_merge(const AttnLaunch& a, hipStream_t s);

// Half-precision copy of a bf16 V tensor [n_kv][m][d] for the attention kernels, one power-of-two scale per KV head.
// part: [n_kv][v_prep_chunks(n_kv, m)] scratch words; unscale: [n_kv] factors that undo the scale.
int v_prep_chunks(int n_kv, int m);
hipError_t launch_v_prep(const void* v, int n_kv, int m, int d, void* v16, uint32_t* part, float* unscale, hipStream_t s);

// Raises the dynamic-LDS limit of every bf16 attention kernel variant on the current device (once per device).
hipError_t attn_prepare_device();

// Cache update after recomputation: rows of `cur` (old, updated in place) against rows of `fresh` (new).
struct UpdateLaunch {
  int dtype, d, fusion;
  long long n_rows;   // per tensor (K and V each have n_rows rows of d elements)
  void* k_cur; void* v_cur;
  const void* k_new; const void* v_new;
};
hipError_t launch_kv_update(const UpdateLaunch& a, hipStream_t s);

}  // namespace samkv
