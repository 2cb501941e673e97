// C ABI of the SamKV hot path: argument checks, host-side prefix sums, workspace carving and the
// kernel launches.  Everything a call needs on the device travels in kernel arguments; the library
// allocates nothing and synchronises with nothing.
#include <math.h>
#include <string.h>

#include <mutex>

#include "common.hpp"

using namespace samkv;

// Scratch memory of samkv_score_noalloc: lives in the library's device image, one copy per GPU, for the life of the
// process.  In host code this name is only a handle for hipGetSymbolAddress; kernels receive the address it returns.
static __device__ __align__(256) unsigned char scratch[SAMKV_NOALLOC_SCRATCH_BYTES];

namespace {

constexpr size_t kAlign = 256;
size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }
// every kernel moves tensor rows with 16-byte vector accesses
bool aligned16(const void* p) { return ((uintptr_t)p % 16) == 0; }

int kept_count(int len, float ratio) {
  if (len < 1 || !(ratio > 0.f) || ratio > 1.f) return 0;
  const double x = (double)ratio * (double)len * (1.0 - 0x1p-22);
  long long k = (long long)ceil(x);
  if (k < 1) k = 1;
  if (k > len) k = len;
  return (int)k;
}

struct Shape {
  int n_ctx, hq, hkv, d, dtype, max_len, total_len;
  IntTable cu_len;
};

int check_caches(const samkv_caches* c, bool need_k, bool need_v, Shape* s) {
  if (c == nullptr || c->len == nullptr) return SAMKV_EINVAL;
  if (c->n_ctx < 1 || c->n_q_heads < 1 || c->n_kv_heads < 1 || c->n_q_heads % c->n_kv_heads != 0) return SAMKV_EINVAL;
  if (c->dtype != SAMKV_F32 && c->dtype != SAMKV_BF16) return SAMKV_EUNSUPPORTED;
  if (c->head_dim != 64 && c->head_dim != 128) return SAMKV_EUNSUPPORTED;
  if (c->n_ctx > SAMKV_MAX_CTX) return SAMKV_EUNSUPPORTED;
  if ((need_k && c->k == nullptr) || (need_v && c->v == nullptr)) return SAMKV_EINVAL;
  s->n_ctx = c->n_ctx; s->hq = c->n_q_heads; s->hkv = c->n_kv_heads; s->d = c->head_dim; s->dtype = c->dtype;
  s->max_len = 0;
  long long total = 0;
  s->cu_len.v[0] = 0;
  for (int i = 0; i < c->n_ctx; ++i) {
    if (c->len[i] < 1) return SAMKV_EINVAL;
    if (c->len[i] > SAMKV_MAX_LEN) return SAMKV_EUNSUPPORTED;
    if ((need_k && c->k[i] == nullptr) || (need_v && c->v[i] == nullptr)) return SAMKV_EINVAL;
    if ((need_k && !aligned16(c->k[i])) || (need_v && !aligned16(c->v[i]))) return SAMKV_EINVAL;
    total += c->len[i];
    if (total > 0x7FFFFFFF / 2) return SAMKV_EUNSUPPORTED;
    s->cu_len.v[i + 1] = (int32_t)total;
    if (c->len[i] > s->max_len) s->max_len = c->len[i];
  }
  s->total_len = (int)total;
  return SAMKV_OK;
}

// Kept tokens of a document whose middle segment (everything but the forced initial and local positions)
// is sparsified to the share p in [0, 1]: forced + ceil(p * middle), with the same float32 guard as above.
int kept_count_mid(int len, float p, int n_sink, int n_local) {
  if (len < 1 || !(p >= 0.f) || p > 1.f || n_sink < 0 || n_local < 0) return -1;
  const long long forced = (long long)n_sink + n_local;
  if (forced >= len) return len;
  const long long mid = len - forced;
  long long k = (long long)ceil((double)p * (double)mid * (1.0 - 0x1p-22));
  if (k < 0) k = 0;
  if (k > mid) k = mid;
  return (int)(forced + k);
}

int kept_table_mid(const samkv_caches* c, const float* p, int n_sink, int n_local, IntTable* cu_k) {
  if (p == nullptr) return SAMKV_EINVAL;
  cu_k->v[0] = 0;
  for (int i = 0; i < c->n_ctx; ++i) {
    const int k = kept_count_mid(c->len[i], p[i], n_sink, n_local);
    if (k < 0) return SAMKV_EINVAL;
    cu_k->v[i + 1] = cu_k->v[i] + k;
  }
  return cu_k->v[c->n_ctx] >= 1 ? SAMKV_OK : SAMKV_EINVAL;
}

int kept_table(const samkv_caches* c, float ratio, int n_sink, int n_local, IntTable* cu_k) {
  if (!(ratio > 0.f) || ratio > 1.f || n_sink < 0 || n_local < 0) return SAMKV_EINVAL;
  cu_k->v[0] = 0;
  for (int i = 0; i < c->n_ctx; ++i) {
    const int k = kept_count(c->len[i], ratio);
    if ((long long)n_sink + n_local > k) return SAMKV_EINVAL;
    cu_k->v[i + 1] = cu_k->v[i] + k;
  }
  return SAMKV_OK;
}

// Score workspace: Q_que [Hq][d], Q_loc [N][Hq][d], |cos| [N][Hq], bias sums [Hq][d], folded vectors
// [N][Hkv][d], all float32.
struct ScoreWs { size_t que, loc, w, base, qt, bytes; };
ScoreWs score_ws(int n_ctx, int hq, int hkv, int d) {
  ScoreWs w;
  size_t o = 0;
  w.que = o; o = align_up(o + (size_t)hq * d * 4);
  w.loc = o; o = align_up(o + (size_t)n_ctx * hq * d * 4);
  w.w = o;   o = align_up(o + (size_t)n_ctx * hq * 4);
  w.base = o; o = align_up(o + (size_t)hq * d * 4);
  w.qt = o;  o = align_up(o + (size_t)n_ctx * hkv * d * 4);
  w.bytes = o;
  return w;
}

// Not-causal attention: cut the keys into chunks when the row tiles alone cannot fill the chip.
struct SplitPlan { int n_split, chunk; size_t part_o, part_lse, bytes; };
SplitPlan plan_splits(int dtype, int n_batch, int rows, int m, int d) {
  const int bq = dtype == SAMKV_BF16 ? 32 * attn_bf16_waves(0, n_batch, rows) : 16;
  const int bk = dtype == SAMKV_BF16 ? 64 : 32;
  const long long base = (long long)((rows + bq - 1) / bq) * n_batch;
  const int key_tiles = (m + bk - 1) / bk;
  // aim at as many workgroups as are resident at once: one per compute unit for the eight-wave kernel (256 rows),
  // two for the four-wave one; a second round of workgroups only adds partial results to merge
  const int wg_target = bq == 256 ? 256 : 512;
  long long want = (wg_target + base - 1) / base;
  if (want > 64) want = 64;
  if (want < 1) want = 1;
  int tiles_per = (int)((key_tiles + want - 1) / want);
  if (tiles_per < 4) tiles_per = 4;  // a chunk shorter than a few tiles costs more in the merge than it gains
  SplitPlan p;
  p.chunk = tiles_per * bk;
  p.n_split = (m + p.chunk - 1) / p.chunk;
  p.part_o = 0;
  p.part_lse = 0;
  p.bytes = 0;
  if (p.n_split > 1) {
    const size_t n_rows = (size_t)n_batch * rows;
    p.part_o = 0;
    p.part_lse = align_up((size_t)p.n_split * n_rows * d * 4);
    p.bytes = align_up(p.part_lse + (size_t)p.n_split * n_rows * 4);
  }
  return p;
}

// bf16 attention: the half-precision copy of V [Hkv][M][d], the per-chunk maxima and the per-head unscale factors.
struct VPrepWs { size_t v16, part, unscale, bytes; };
VPrepWs vprep_ws(int dtype, int hkv, int m, int d) {
  VPrepWs w;
  w.v16 = w.part = w.unscale = w.bytes = 0;
  if (dtype != SAMKV_BF16) return w;
  w.part = align_up((size_t)hkv * m * d * 2);
  w.unscale = align_up(w.part + (size_t)hkv * v_prep_chunks(hkv, m) * 4);
  w.bytes = align_up(w.unscale + (size_t)hkv * 4);
  return w;
}

// Workspace of one attention problem: the key-chunk partials (not causal only), then the V preparation.
struct AttnWs { SplitPlan split; VPrepWs vp; size_t vp_at, bytes; };
AttnWs attn_ws(int dtype, bool causal, int hkv, int rows_per_kv, int m, int d) {
  AttnWs w;
  if (causal) {
    w.split.n_split = 1; w.split.chunk = m; w.split.part_o = w.split.part_lse = w.split.bytes = 0;
  } else {
    w.split = plan_splits(dtype, hkv, rows_per_kv, m, d);
  }
  w.vp = vprep_ws(dtype, hkv, m, d);
  w.vp_at = w.split.bytes;
  w.bytes = w.vp_at + w.vp.bytes;
  return w;
}

// Runs the V preparation of a bf16 attention call into its workspace slice and points the launch at the copy.
hipError_t prepare_v(AttnLaunch* a, const VPrepWs& vp, char* at, int hkv, hipStream_t s) {
  if (a->dtype != SAMKV_BF16 || !attn_bf16_reads_v16(*a)) return hipSuccess;
  float* unscale = reinterpret_cast<float*>(at + vp.unscale);
  const hipError_t e = launch_v_prep(a->v, hkv, a->m, a->d, at + vp.v16, reinterpret_cast<uint32_t*>(at + vp.part), unscale, s);
  a->v = at + vp.v16;
  a->v_unscale = unscale;
  return e;
}

// Workspace of samkv_query_attn_self: two result slots [2][Hq*Lq][d] + [2][Hq*Lq] (cache part, self part),
// followed by whatever the cache part itself needs for its key chunks.
struct SelfWs { size_t part_o, part_lse, inner, bytes; };
SelfWs self_ws(int hq, int hkv, int d, int n_q_tok, int m_total, int dtype) {
  SelfWs w;
  const size_t n_rows = (size_t)hq * n_q_tok;
  w.part_o = 0;
  w.part_lse = align_up(2 * n_rows * d * 4);
  w.inner = align_up(w.part_lse + 2 * n_rows * 4);
  // the two partial attentions run one after the other on the stream and share the inner region
  const size_t cache_part = attn_ws(dtype, false, hkv, (hq / hkv) * n_q_tok, m_total, d).bytes;
  const size_t self_part = attn_ws(dtype, true, hkv, 0, n_q_tok, d).bytes;
  w.bytes = w.inner + (cache_part > self_part ? cache_part : self_part);
  return w;
}

int check_attn(const void* q, const void* k, const void* v, int rows, int m, int hq, int hkv, int d, int dtype,
               float scale, const float* out, const float* lse) {
  if (q == nullptr || k == nullptr || v == nullptr || out == nullptr || lse == nullptr) return SAMKV_EINVAL;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out) || ((uintptr_t)lse % 4) != 0) return SAMKV_EINVAL;
  if (rows < 1 || m < 1 || hq < 1 || hkv < 1 || hq % hkv != 0 || !(scale > 0.f) || !isfinite(scale)) return SAMKV_EINVAL;
  if (dtype != SAMKV_F32 && dtype != SAMKV_BF16) return SAMKV_EUNSUPPORTED;
  if (d != 64 && d != 128) return SAMKV_EUNSUPPORTED;
  if ((long long)hq * rows > 0x7FFFFFFF / 256 || m > 0x7FFFFFFF / 512 || rows / 16 > 65535 || hkv > 65535)
    return SAMKV_EUNSUPPORTED;
  return SAMKV_OK;
}

int dev(hipError_t e) { return e == hipSuccess ? SAMKV_OK : SAMKV_EDEVICE; }

}  // namespace

extern "C" {

const char* samkv_strerror(int code) {
  switch (code) {
    case SAMKV_OK: return "ok";
    case SAMKV_EINVAL: return "invalid argument";
    case SAMKV_EUNSUPPORTED: return "unsupported size or dtype";
    case SAMKV_EWORKSPACE: return "workspace missing or too small";
    case SAMKV_EDEVICE: return "HIP launch failed";
  }
  return "unknown error";
}

int32_t samkv_kept_count(int32_t len, float ratio) { return kept_count(len, ratio); }

size_t samkv_workspace_bytes(int32_t n_ctx, int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                             int32_t n_q_tok, int32_t m_total) {
  if (n_ctx < 1 || n_q_heads < 1 || n_kv_heads < 1 || head_dim < 1 || n_q_tok < 1 || m_total < 1) return 0;
  const size_t a = score_ws(n_ctx, n_q_heads, n_kv_heads, head_dim).bytes;
  const int rows = (n_q_heads / n_kv_heads) * n_q_tok;
  size_t b = attn_ws(SAMKV_BF16, false, n_kv_heads, rows, m_total, head_dim).bytes;
  const size_t c = attn_ws(SAMKV_F32, false, n_kv_heads, rows, m_total, head_dim).bytes;
  if (c > b) b = c;
  const size_t r = attn_ws(SAMKV_BF16, true, n_kv_heads, 0, m_total, head_dim).bytes;
  if (r > b) b = r;
  const size_t e = self_ws(n_q_heads, n_kv_heads, head_dim, n_q_tok, m_total, SAMKV_BF16).bytes;
  const size_t f = self_ws(n_q_heads, n_kv_heads, head_dim, n_q_tok, m_total, SAMKV_F32).bytes;
  if (e > b) b = e;
  if (f > b) b = f;
  return (a > b ? a : b) + kAlign;
}

static int score_setup(const samkv_caches* caches, const void* q_tok, int32_t n_q_tok, const void* q_loc, int32_t w_loc,
                       float* scores, void* ws, size_t ws_bytes, Shape* s, ScoreLaunch* a, PtrTable* kt) {
  int rc = check_caches(caches, true, false, s);
  if (rc != SAMKV_OK) return rc;
  if (q_tok == nullptr || n_q_tok < 1 || (q_loc != nullptr && w_loc < 1)) return SAMKV_EINVAL;
  if (!aligned16(q_tok) || !aligned16(q_loc) || ((uintptr_t)scores % 4) != 0) return SAMKV_EINVAL;
  const ScoreWs w = score_ws(s->n_ctx, s->hq, s->hkv, s->d);
  if (ws == nullptr || ((uintptr_t)ws % kAlign) != 0 || ws_bytes < w.bytes) return SAMKV_EWORKSPACE;
  memset(kt, 0, sizeof(*kt));
  for (int i = 0; i < s->n_ctx; ++i) kt->p[i] = caches->k[i];
  a->n_ctx = s->n_ctx; a->hq = s->hq; a->hkv = s->hkv; a->d = s->d; a->dtype = s->dtype;
  a->n_q_tok = n_q_tok; a->w_loc = w_loc; a->max_len = s->max_len; a->total_len = s->total_len;
  a->q_tok = q_tok; a->q_loc = q_loc; a->scores = scores;
  char* base = static_cast<char*>(ws);
  a->ws_que = reinterpret_cast<float*>(base + w.que);
  a->ws_loc = reinterpret_cast<float*>(base + w.loc);
  a->ws_w = reinterpret_cast<float*>(base + w.w);
  a->ws_base = reinterpret_cast<float*>(base + w.base);
  a->ws_qt = reinterpret_cast<float*>(base + w.qt);
  return SAMKV_OK;
}

// Device address of `scratch` on the current device, looked up once per device.
static int scratch_address(void** out) {
  constexpr int kMaxDev = 64;
  static std::mutex mu;
  static void* ptr[kMaxDev] = {};
  int d = 0;
  if (hipGetDevice(&d) != hipSuccess || d < 0 || d >= kMaxDev) return SAMKV_EDEVICE;
  std::lock_guard<std::mutex> lock(mu);
  if (ptr[d] == nullptr) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) return SAMKV_EDEVICE;
    ptr[d] = p;
  }
  *out = ptr[d];
  return SAMKV_OK;
}

int samkv_score_noalloc(const samkv_caches* caches, const void* q_tok, int32_t n_q_tok, const void* q_loc, int32_t w_loc,
                        float* scores, void* stream) {
  Shape s;
  const int rc = check_caches(caches, true, false, &s);
  if (rc != SAMKV_OK) return rc;
  if (score_ws(s.n_ctx, s.hq, s.hkv, s.d).bytes > SAMKV_NOALLOC_SCRATCH_BYTES) return SAMKV_EUNSUPPORTED;
  void* ws = nullptr;
  const int rs = scratch_address(&ws);
  if (rs != SAMKV_OK) return rs;
  // every float of the scratch area that a kernel of this call reads has been written by an earlier kernel of the
  // same call, so nothing needs clearing between calls
  return samkv_score(caches, q_tok, n_q_tok, q_loc, w_loc, scores, ws, SAMKV_NOALLOC_SCRATCH_BYTES, stream);
}

int samkv_score(const samkv_caches* caches, const void* q_tok, int32_t n_q_tok, const void* q_loc, int32_t w_loc,
                float* scores, void* ws, size_t ws_bytes, void* stream) {
  Shape s;
  ScoreLaunch a;
  PtrTable kt;
  if (scores == nullptr) return SAMKV_EINVAL;
  int rc = score_setup(caches, q_tok, n_q_tok, q_loc, w_loc, scores, ws, ws_bytes, &s, &a, &kt);
  if (rc != SAMKV_OK) return rc;
  return dev(launch_score(a, kt, s.cu_len, static_cast<hipStream_t>(stream)));
}

// samkv_score_select, and with k_c/v_c the compaction as well
static int score_select_common(const samkv_caches* caches, const void* q_tok, int32_t n_q_tok, const void* q_loc,
                               int32_t w_loc, float ratio, int32_t n_sink, int32_t n_local, float* scores, int32_t* idx,
                               int32_t* cu_k_dev, int32_t* cu_k_host, bool gather, void* k_c, void* v_c, void* ws,
                               size_t ws_bytes, void* stream) {
  Shape s;
  ScoreLaunch a;
  PtrTable kt;
  if (idx == nullptr) return SAMKV_EINVAL;
  int rc = score_setup(caches, q_tok, n_q_tok, q_loc, w_loc, scores, ws, ws_bytes, &s, &a, &kt);
  if (rc != SAMKV_OK) return rc;
  if (scores == nullptr && s.max_len > kFusedMaxLen) return SAMKV_EINVAL;
  IntTable cu_k;
  rc = kept_table(caches, ratio, n_sink, n_local, &cu_k);
  if (rc != SAMKV_OK) return rc;
  PtrTable vt;
  GatherLaunch ga;
  if (gather) {
    Shape s2;
    rc = check_caches(caches, true, true, &s2);  // V is read as well
    if (rc != SAMKV_OK) return rc;
    if (k_c == nullptr || v_c == nullptr || !aligned16(k_c) || !aligned16(v_c)) return SAMKV_EINVAL;
    memset(&vt, 0, sizeof(vt));
    for (int i = 0; i < s.n_ctx; ++i) vt.p[i] = caches->v[i];
    ga.n_ctx = s.n_ctx; ga.hkv = s.hkv; ga.row_bytes = s.d * (s.dtype == SAMKV_BF16 ? 2 : 4);
    ga.m_total = cu_k.v[s.n_ctx]; ga.idx = idx; ga.k_c = k_c; ga.v_c = v_c;
    ga.max_k = 0;
    for (int i = 0; i < s.n_ctx; ++i) ga.max_k = cu_k.v[i + 1] - cu_k.v[i] > ga.max_k ? cu_k.v[i + 1] - cu_k.v[i] : ga.max_k;
  }
  if (cu_k_host != nullptr) memcpy(cu_k_host, cu_k.v, sizeof(int32_t) * (s.n_ctx + 1));
  SelectLaunch sl;
  sl.n_ctx = s.n_ctx; sl.hkv = s.hkv; sl.max_len = s.max_len; sl.total_len = s.total_len;
  sl.m_total = cu_k.v[s.n_ctx]; sl.n_sink = n_sink; sl.n_local = n_local;
  sl.scores = scores; sl.idx = idx; sl.cu_k_dev = cu_k_dev;
  return dev(launch_score_select(a, sl, kt, s.cu_len, cu_k, static_cast<hipStream_t>(stream), gather ? &ga : nullptr,
                                 gather ? &vt : nullptr));
}

int samkv_score_select(const samkv_caches* caches, const void* q_tok, int32_t n_q_tok, const void* q_loc, int32_t w_loc,
                       float ratio, int32_t n_sink, int32_t n_local, float* scores, int32_t* idx, int32_t* cu_k_dev,
                       int32_t* cu_k_host, void* ws, size_t ws_bytes, void* stream) {
  return score_select_common(caches, q_tok, n_q_tok, q_loc, w_loc, ratio, n_sink, n_local, scores, idx, cu_k_dev, cu_k_host,
                             false, nullptr, nullptr, ws, ws_bytes, stream);
}

int samkv_score_select_gather(const samkv_caches* caches, const void* q_tok, int32_t n_q_tok, const void* q_loc,
                              int32_t w_loc, float ratio, int32_t n_sink, int32_t n_local, float* scores, int32_t* idx,
                              int32_t* cu_k_dev, int32_t* cu_k_host, void* k_c, void* v_c, void* ws, size_t ws_bytes,
                              void* stream) {
  return score_select_common(caches, q_tok, n_q_tok, q_loc, w_loc, ratio, n_sink, n_local, scores, idx, cu_k_dev, cu_k_host,
                             true, k_c, v_c, ws, ws_bytes, stream);
}

static int select_common(const float* scores, const samkv_caches* caches, const Shape& s, const IntTable& cu_k,
                         int32_t n_sink, int32_t n_local, int32_t* idx, int32_t* cu_k_dev, int32_t* cu_k_host,
                         void* stream);

int32_t samkv_kept_count_mid(int32_t len, float p, int32_t n_sink, int32_t n_local) {
  const int k = kept_count_mid(len, p, n_sink, n_local);
  return k < 0 ? 0 : k;
}

int samkv_top_p(const float* s_anc, const float* s_max, const float* s_min, int32_t n_layers, int32_t n_ctx, float* p) {
  if (s_anc == nullptr || s_max == nullptr || s_min == nullptr || p == nullptr || n_layers < 1 || n_ctx < 1)
    return SAMKV_EINVAL;
  for (int i = 0; i < n_ctx; ++i) {
    double acc = 0.0;
    for (int n = 0; n < n_layers; ++n) {
      const double a = s_anc[(size_t)n * n_ctx + i], hi = s_max[(size_t)n * n_ctx + i], lo = s_min[(size_t)n * n_ctx + i];
      if (a > lo && a <= hi) acc += (hi - a) / (hi - lo);   // Eq. 2; 0 otherwise
    }
    p[i] = (float)(acc / n_layers);                          // Eq. 3
  }
  return SAMKV_OK;
}

int samkv_topk_select_v(const float* scores, const samkv_caches* caches, const float* p, int32_t n_sink,
                        int32_t n_local, int32_t* idx, int32_t* cu_k_dev, int32_t* cu_k_host, void* ws, size_t ws_bytes,
                        void* stream) {
  (void)ws; (void)ws_bytes;
  Shape s;
  int rc = check_caches(caches, false, false, &s);
  if (rc != SAMKV_OK) return rc;
  if (scores == nullptr || idx == nullptr) return SAMKV_EINVAL;
  IntTable cu_k;
  rc = kept_table_mid(caches, p, n_sink, n_local, &cu_k);
  if (rc != SAMKV_OK) return rc;
  return select_common(scores, caches, s, cu_k, n_sink, n_local, idx, cu_k_dev, cu_k_host, stream);
}

int samkv_topk_select(const float* scores, const samkv_caches* caches, float ratio, int32_t n_sink, int32_t n_local,
                      int32_t* idx, int32_t* cu_k_dev, int32_t* cu_k_host, void* ws, size_t ws_bytes, void* stream) {
  (void)ws; (void)ws_bytes;
  Shape s;
  int rc = check_caches(caches, false, false, &s);
  if (rc != SAMKV_OK) return rc;
  if (scores == nullptr || idx == nullptr) return SAMKV_EINVAL;
  IntTable cu_k;
  rc = kept_table(caches, ratio, n_sink, n_local, &cu_k);
  if (rc != SAMKV_OK) return rc;
  return select_common(scores, caches, s, cu_k, n_sink, n_local, idx, cu_k_dev, cu_k_host, stream);
}

static int select_common(const float* scores, const samkv_caches* caches, const Shape& s, const IntTable& cu_k,
                         int32_t n_sink, int32_t n_local, int32_t* idx, int32_t* cu_k_dev, int32_t* cu_k_host,
                         void* stream) {
  (void)caches;
  if (cu_k_host != nullptr) memcpy(cu_k_host, cu_k.v, sizeof(int32_t) * (s.n_ctx + 1));
  SelectLaunch a;
  a.n_ctx = s.n_ctx; a.hkv = s.hkv; a.max_len = s.max_len; a.total_len = s.total_len;
  a.m_total = cu_k.v[s.n_ctx]; a.n_sink = n_sink; a.n_local = n_local;
  a.scores = scores; a.idx = idx; a.cu_k_dev = cu_k_dev;
  return dev(launch_select(a, s.cu_len, cu_k, static_cast<hipStream_t>(stream)));
}

// ---- block-granular selection (Sec. 3.2: blocks of tokens represented by their mean key) -----------------
static int block_table(const samkv_caches* caches, const Shape& s, int block, IntTable* cu_blk) {
  if (block < 1 || block > 4096) return SAMKV_EINVAL;
  cu_blk->v[0] = 0;
  for (int i = 0; i < s.n_ctx; ++i) cu_blk->v[i + 1] = cu_blk->v[i] + (caches->len[i] + block - 1) / block;
  return SAMKV_OK;
}

// Counts of the per-document block selection, and of the cross-document filter on top of it.
struct BlockPlan {
  IntTable cu_blk, cu_kb, cu_k;  // blocks, kept blocks, kept tokens of the per-document selection (prefix sums)
  int max_nb;
  int forced_blocks, forced_tokens, cand, keep;  // filter: candidates = kept middle blocks, keep = ceil(cand / n_ctx)
  bool any_short_unforced;                       // some document's short last block is not a forced block
};

static int block_plan(const samkv_caches* caches, const Shape& s, int block, const float* p, int n_init, int n_local,
                      BlockPlan* bp) {
  if (p == nullptr || n_init < 0 || n_local < 0) return SAMKV_EINVAL;
  int rc = block_table(caches, s, block, &bp->cu_blk);
  if (rc != SAMKV_OK) return rc;
  bp->cu_kb.v[0] = 0;
  bp->cu_k.v[0] = 0;
  bp->max_nb = 0;
  bp->forced_blocks = bp->forced_tokens = bp->cand = 0;
  bp->any_short_unforced = false;
  for (int i = 0; i < s.n_ctx; ++i) {
    const int L = caches->len[i], nb = bp->cu_blk.v[i + 1] - bp->cu_blk.v[i];
    const int kb = kept_count_mid(nb, p[i], n_init, n_local);
    if (kb < 0) return SAMKV_EINVAL;
    const bool short_last = L % block != 0;
    const long long forced_ll = (long long)n_init + n_local;
    const int forced = forced_ll >= nb ? nb : (int)forced_ll;
    // a short last block must be kept by every head or by none: it is kept whenever local blocks are forced
    if (short_last && n_local == 0 && kb != 0 && kb != nb) return SAMKV_EINVAL;
    if (short_last && n_local == 0 && forced < nb) bp->any_short_unforced = true;
    const bool last_kept = kb == nb || (n_local > 0 && kb > 0);
    const int tokens = kb * block - ((last_kept && short_last) ? (block - L % block) : 0);
    bp->cu_kb.v[i + 1] = bp->cu_kb.v[i] + kb;
    bp->cu_k.v[i + 1] = bp->cu_k.v[i] + tokens;
    if (nb > bp->max_nb) bp->max_nb = nb;
    bp->forced_blocks += forced;
    bp->forced_tokens += forced == nb ? L : n_init * block + (L - (nb - n_local) * block);
    bp->cand += kb - forced;
  }
  bp->keep = (bp->cand + s.n_ctx - 1) / s.n_ctx;
  return bp->cu_k.v[s.n_ctx] >= 1 ? SAMKV_OK : SAMKV_EINVAL;
}

static hipError_t block_select_launch(const float* bscores, const Shape& s, const BlockPlan& bp, int n_init, int n_local,
                                      int32_t* bidx, hipStream_t st) {
  SelectLaunch a;
  a.n_ctx = s.n_ctx; a.hkv = s.hkv; a.max_len = bp.max_nb; a.total_len = bp.cu_blk.v[s.n_ctx];
  a.m_total = bp.cu_kb.v[s.n_ctx]; a.n_sink = n_init; a.n_local = n_local;
  a.scores = bscores; a.idx = bidx; a.cu_k_dev = nullptr;
  return launch_select(a, bp.cu_blk, bp.cu_kb, st);
}

size_t samkv_block_workspace_bytes(const samkv_caches* caches, int32_t block) {
  Shape s;
  IntTable cu_blk;
  if (check_caches(caches, false, false, &s) != SAMKV_OK || block_table(caches, s, block, &cu_blk) != SAMKV_OK) return 0;
  // kept block ids; for the filter also the candidates' normalised scores, the kept candidates, their first token
  // positions and output offsets: five arrays of at most [Hkv][sum of blocks] 4-byte entries
  return 5 * align_up((size_t)s.hkv * cu_blk.v[s.n_ctx] * 4) + kAlign;
}

int samkv_block_scores(const float* scores, const samkv_caches* caches, int32_t block, float* bscores, void* stream) {
  Shape s;
  int rc = check_caches(caches, false, false, &s);
  if (rc != SAMKV_OK) return rc;
  if (scores == nullptr || bscores == nullptr) return SAMKV_EINVAL;
  IntTable cu_blk;
  rc = block_table(caches, s, block, &cu_blk);
  if (rc != SAMKV_OK) return rc;
  return dev(launch_block_scores(scores, s.cu_len, cu_blk, s.n_ctx, s.hkv, s.total_len, block, bscores,
                                 static_cast<hipStream_t>(stream)));
}

int samkv_block_select(const float* bscores, const samkv_caches* caches, int32_t block, const float* p,
                       int32_t n_init_blocks, int32_t n_local_blocks, int32_t* idx, int32_t* cu_k_dev,
                       int32_t* cu_k_host, void* ws, size_t ws_bytes, void* stream) {
  Shape s;
  int rc = check_caches(caches, false, false, &s);
  if (rc != SAMKV_OK) return rc;
  if (bscores == nullptr || idx == nullptr) return SAMKV_EINVAL;
  BlockPlan bp;
  rc = block_plan(caches, s, block, p, n_init_blocks, n_local_blocks, &bp);
  if (rc != SAMKV_OK) return rc;
  const size_t need = align_up((size_t)s.hkv * bp.cu_blk.v[s.n_ctx] * 4);
  if (ws == nullptr || ((uintptr_t)ws % kAlign) != 0 || ws_bytes < need) return SAMKV_EWORKSPACE;
  if (cu_k_host != nullptr) memcpy(cu_k_host, bp.cu_k.v, sizeof(int32_t) * (s.n_ctx + 1));
  int32_t* bidx = static_cast<int32_t*>(ws);
  hipStream_t st = static_cast<hipStream_t>(stream);
  hipError_t e = block_select_launch(bscores, s, bp, n_init_blocks, n_local_blocks, bidx, st);
  if (e == hipSuccess)
    e = launch_expand_blocks(bidx, s.cu_len, bp.cu_kb, bp.cu_k, s.n_ctx, s.hkv, block, idx, cu_k_dev, st);
  return dev(e);
}

int32_t samkv_block_select_count(const samkv_caches* caches, int32_t block, const float* p, int32_t n_init_blocks,
                                 int32_t n_local_blocks) {
  Shape s;
  BlockPlan bp;
  if (check_caches(caches, false, false, &s) != SAMKV_OK ||
      block_plan(caches, s, block, p, n_init_blocks, n_local_blocks, &bp) != SAMKV_OK)
    return 0;
  return bp.cu_k.v[s.n_ctx];
}

int32_t samkv_block_filter_count(const samkv_caches* caches, int32_t block, const float* p, int32_t n_init_blocks,
                                 int32_t n_local_blocks) {
  Shape s;
  BlockPlan bp;
  if (check_caches(caches, false, false, &s) != SAMKV_OK ||
      block_plan(caches, s, block, p, n_init_blocks, n_local_blocks, &bp) != SAMKV_OK || bp.any_short_unforced)
    return 0;
  return bp.forced_tokens + bp.keep * block;
}

int samkv_block_select_filter(const float* bscores, const samkv_caches* caches, int32_t block, const float* p,
                              int32_t n_init_blocks, int32_t n_local_blocks, int32_t* gidx, void* ws, size_t ws_bytes,
                              void* stream) {
  Shape s;
  int rc = check_caches(caches, false, false, &s);
  if (rc != SAMKV_OK) return rc;
  if (bscores == nullptr || gidx == nullptr) return SAMKV_EINVAL;
  BlockPlan bp;
  rc = block_plan(caches, s, block, p, n_init_blocks, n_local_blocks, &bp);
  if (rc != SAMKV_OK) return rc;
  if (bp.any_short_unforced) return SAMKV_EINVAL;  // every candidate must be a full block
  const int total_kb = bp.cu_kb.v[s.n_ctx];
  if (total_kb > SAMKV_MAX_LEN) return SAMKV_EUNSUPPORTED;  // the candidates of one head form one selection row
  const int n_sel = bp.forced_blocks + bp.keep;
  const int m_total = bp.forced_tokens + bp.keep * block;
  if (n_sel < 1 || m_total < 1) return SAMKV_EINVAL;
  const size_t slab = align_up((size_t)s.hkv * bp.cu_blk.v[s.n_ctx] * 4);
  if (ws == nullptr || ((uintptr_t)ws % kAlign) != 0 || ws_bytes < 5 * slab) return SAMKV_EWORKSPACE;
  char* w = static_cast<char*>(ws);
  int32_t* bidx = reinterpret_cast<int32_t*>(w);
  float* cand = reinterpret_cast<float*>(w + slab);
  int32_t* sel = reinterpret_cast<int32_t*>(w + 2 * slab);
  int32_t* start = reinterpret_cast<int32_t*>(w + 3 * slab);
  int32_t* tok_off = reinterpret_cast<int32_t*>(w + 4 * slab);
  hipStream_t st = static_cast<hipStream_t>(stream);
  hipError_t e = block_select_launch(bscores, s, bp, n_init_blocks, n_local_blocks, bidx, st);
  if (e == hipSuccess)
    e = launch_normalize(bscores, bidx, bp.cu_blk, bp.cu_kb, s.n_ctx, s.hkv, n_init_blocks, n_local_blocks, cand, st);
  if (e == hipSuccess) {
    // all candidates of a KV head as one row; the forced ones carry +inf and are within the budget by construction
    IntTable row, kept;
    row.v[0] = 0; row.v[1] = total_kb;
    kept.v[0] = 0; kept.v[1] = n_sel;
    SelectLaunch a;
    a.n_ctx = 1; a.hkv = s.hkv; a.max_len = total_kb; a.total_len = total_kb; a.m_total = n_sel;
    a.n_sink = 0; a.n_local = 0; a.scores = cand; a.idx = sel; a.cu_k_dev = nullptr;
    e = launch_select(a, row, kept, st);
  }
  if (e == hipSuccess)
    e = launch_filter_expand(sel, bidx, s.cu_len, bp.cu_kb, s.n_ctx, s.hkv, n_sel, m_total, block, start, tok_off, gidx, st);
  return dev(e);
}

int samkv_gather_g(const samkv_caches* caches, const int32_t* gidx, int32_t m_total, void* k_c, void* v_c, void* stream) {
  Shape s;
  int rc = check_caches(caches, true, true, &s);
  if (rc != SAMKV_OK) return rc;
  if (gidx == nullptr || k_c == nullptr || v_c == nullptr || m_total < 1) return SAMKV_EINVAL;
  if (!aligned16(k_c) || !aligned16(v_c)) return SAMKV_EINVAL;
  PtrTable kt, vt;
  memset(&kt, 0, sizeof(kt));
  memset(&vt, 0, sizeof(vt));
  for (int i = 0; i < s.n_ctx; ++i) { kt.p[i] = caches->k[i]; vt.p[i] = caches->v[i]; }
  return dev(launch_gather_g(s.d * (s.dtype == SAMKV_BF16 ? 2 : 4), kt, &vt, s.cu_len, s.n_ctx, s.hkv, 1, m_total, gidx,
                             k_c, v_c, static_cast<hipStream_t>(stream)));
}

int samkv_gather_q_g(const samkv_caches* caches, const void* const* q_cache, const int32_t* gidx, int32_t m_total,
                     void* q_rec, void* stream) {
  Shape s;
  int rc = check_caches(caches, false, false, &s);
  if (rc != SAMKV_OK) return rc;
  if (q_cache == nullptr || gidx == nullptr || q_rec == nullptr || m_total < 1 || !aligned16(q_rec)) return SAMKV_EINVAL;
  PtrTable qt;
  memset(&qt, 0, sizeof(qt));
  for (int i = 0; i < s.n_ctx; ++i) {
    if (q_cache[i] == nullptr || !aligned16(q_cache[i])) return SAMKV_EINVAL;
    qt.p[i] = q_cache[i];
  }
  return dev(launch_gather_g(s.d * (s.dtype == SAMKV_BF16 ? 2 : 4), qt, nullptr, s.cu_len, s.n_ctx, s.hq, s.hq / s.hkv,
                             m_total, gidx, q_rec, nullptr, static_cast<hipStream_t>(stream)));
}

static int gather_common(const samkv_caches* caches, const Shape& s, const IntTable& cu_k, const int32_t* idx,
                         void* k_c, void* v_c, void* stream);
static int checked_cu_k(const samkv_caches* caches, const Shape& s, const int32_t* cu_k_host, IntTable* cu_k);

int samkv_gather_v(const samkv_caches* caches, const int32_t* idx, const int32_t* cu_k_host, void* k_c, void* v_c,
                   void* stream) {
  Shape s;
  int rc = check_caches(caches, true, true, &s);
  if (rc != SAMKV_OK) return rc;
  if (idx == nullptr || k_c == nullptr || v_c == nullptr || !aligned16(k_c) || !aligned16(v_c)) return SAMKV_EINVAL;
  IntTable cu_k;
  rc = checked_cu_k(caches, s, cu_k_host, &cu_k);
  if (rc != SAMKV_OK) return rc;
  return gather_common(caches, s, cu_k, idx, k_c, v_c, stream);
}

int samkv_gather(const samkv_caches* caches, const int32_t* idx, float ratio, void* k_c, void* v_c, void* stream) {
  Shape s;
  int rc = check_caches(caches, true, true, &s);
  if (rc != SAMKV_OK) return rc;
  if (idx == nullptr || k_c == nullptr || v_c == nullptr || !aligned16(k_c) || !aligned16(v_c)) return SAMKV_EINVAL;
  IntTable cu_k;
  rc = kept_table(caches, ratio, 0, 0, &cu_k);
  if (rc != SAMKV_OK) return rc;
  return gather_common(caches, s, cu_k, idx, k_c, v_c, stream);
}

static int gather_common(const samkv_caches* caches, const Shape& s, const IntTable& cu_k, const int32_t* idx,
                         void* k_c, void* v_c, void* stream) {
  PtrTable kt, vt;
  memset(&kt, 0, sizeof(kt));
  memset(&vt, 0, sizeof(vt));
  for (int i = 0; i < s.n_ctx; ++i) { kt.p[i] = caches->k[i]; vt.p[i] = caches->v[i]; }
  GatherLaunch a;
  a.n_ctx = s.n_ctx; a.hkv = s.hkv; a.row_bytes = s.d * (s.dtype == SAMKV_BF16 ? 2 : 4);
  a.m_total = cu_k.v[s.n_ctx]; a.idx = idx; a.k_c = k_c; a.v_c = v_c;
  a.max_k = 0;
  for (int i = 0; i < s.n_ctx; ++i) a.max_k = cu_k.v[i + 1] - cu_k.v[i] > a.max_k ? cu_k.v[i + 1] - cu_k.v[i] : a.max_k;
  return dev(launch_gather(a, kt, vt, s.cu_len, cu_k, static_cast<hipStream_t>(stream)));
}

static int checked_cu_k(const samkv_caches* caches, const Shape& s, const int32_t* cu_k_host, IntTable* cu_k) {
  if (cu_k_host == nullptr || cu_k_host[0] != 0) return SAMKV_EINVAL;
  for (int i = 0; i < s.n_ctx; ++i) {
    const int k = cu_k_host[i + 1] - cu_k_host[i];
    if (k < 0 || k > caches->len[i]) return SAMKV_EINVAL;
  }
  if (cu_k_host[s.n_ctx] < 1) return SAMKV_EINVAL;
  memcpy(cu_k->v, cu_k_host, sizeof(int32_t) * (s.n_ctx + 1));
  return SAMKV_OK;
}

static int gather_q_common(const samkv_caches* caches, const Shape& s, const IntTable& cu_k, const void* const* q_cache,
                           const int32_t* idx, void* q_rec, void* stream) {
  PtrTable qt;
  memset(&qt, 0, sizeof(qt));
  for (int i = 0; i < s.n_ctx; ++i) {
    if (q_cache[i] == nullptr || !aligned16(q_cache[i])) return SAMKV_EINVAL;
    qt.p[i] = q_cache[i];
  }
  GatherLaunch a;
  a.n_ctx = s.n_ctx; a.hkv = s.hkv; a.row_bytes = s.d * (s.dtype == SAMKV_BF16 ? 2 : 4);
  a.m_total = cu_k.v[s.n_ctx]; a.idx = idx; a.k_c = q_rec; a.v_c = nullptr;
  a.max_k = 0;
  for (int i = 0; i < s.n_ctx; ++i) a.max_k = cu_k.v[i + 1] - cu_k.v[i] > a.max_k ? cu_k.v[i + 1] - cu_k.v[i] : a.max_k;
  return dev(launch_gather_q(a, qt, s.cu_len, cu_k, s.hq, static_cast<hipStream_t>(stream)));
}

int samkv_gather_q(const samkv_caches* caches, const void* const* q_cache, const int32_t* idx, float ratio, void* q_rec,
                   void* stream) {
  Shape s;
  int rc = check_caches(caches, false, false, &s);
  if (rc != SAMKV_OK) return rc;
  if (q_cache == nullptr || idx == nullptr || q_rec == nullptr || !aligned16(q_rec)) return SAMKV_EINVAL;
  IntTable cu_k;
  rc = kept_table(caches, ratio, 0, 0, &cu_k);
  if (rc != SAMKV_OK) return rc;
  return gather_q_common(caches, s, cu_k, q_cache, idx, q_rec, stream);
}

int samkv_gather_q_v(const samkv_caches* caches, const void* const* q_cache, const int32_t* idx,
                     const int32_t* cu_k_host, void* q_rec, void* stream) {
  Shape s;
  int rc = check_caches(caches, false, false, &s);
  if (rc != SAMKV_OK) return rc;
  if (q_cache == nullptr || idx == nullptr || q_rec == nullptr || !aligned16(q_rec)) return SAMKV_EINVAL;
  IntTable cu_k;
  rc = checked_cu_k(caches, s, cu_k_host, &cu_k);
  if (rc != SAMKV_OK) return rc;
  return gather_q_common(caches, s, cu_k, q_cache, idx, q_rec, stream);
}

int samkv_peak_mfma_bf16(float* sink, int32_t n_blocks, int32_t iters, void* stream) {
  return samkv_peak_mfma_bf16_data(sink, n_blocks, iters, 0, stream);
}

int samkv_peak_mfma_bf16_data(float* sink, int32_t n_blocks, int32_t iters, int32_t pattern, void* stream) {
  if (sink == nullptr || n_blocks < 1 || n_blocks > (1 << 20) || iters < 1 || pattern < 0 || pattern > 2) return SAMKV_EINVAL;
  return dev(launch_peak_mfma(sink, n_blocks, iters, pattern, static_cast<hipStream_t>(stream)));
}

int samkv_peak_copy(const void* src, void* dst, size_t bytes, void* stream) {
  if (src == nullptr || dst == nullptr || bytes < 16 || bytes % 16 != 0 || ((uintptr_t)src % 16) != 0 ||
      ((uintptr_t)dst % 16) != 0)
    return SAMKV_EINVAL;
  return dev(launch_peak_copy(src, dst, bytes, static_cast<hipStream_t>(stream)));
}

int samkv_peak_read(const void* src, size_t bytes, void* sink, void* stream) {
  if (src == nullptr || sink == nullptr || bytes < 16 || bytes % 16 != 0 || ((uintptr_t)src % 16) != 0) return SAMKV_EINVAL;
  return dev(launch_peak_read(src, bytes, static_cast<uint32_t*>(sink), static_cast<hipStream_t>(stream)));
}

// The two attention problems of the path as launch descriptions (V not yet prepared).
static AttnLaunch recompute_launch(const void* q_rec, const void* k_c, const void* v_c, int m_total, int hq, int hkv, int d,
                                   int dtype, float scale, float* out, float* lse) {
  AttnLaunch a;
  memset(&a, 0, sizeof(a));
  a.dtype = dtype; a.d = d; a.causal = 1;
  a.n_batch = hq; a.batch_per_kv = hq / hkv; a.rows = m_total; a.m = m_total;
  a.q = q_rec; a.k = k_c; a.v = v_c; a.out = out; a.lse = lse; a.scale = scale;
  a.n_split = 1; a.chunk = m_total;
  return a;
}

// q_tok [Hq][Lq][d] is, per KV head, one contiguous block of G*Lq rows that all read the same K/V.
static AttnLaunch query_launch(const void* q_tok, int n_q_tok, const void* k_c, const void* v_c, int m_total, int hq, int hkv,
                               int d, int dtype, float scale, float* out, float* lse, const SplitPlan& p, void* ws) {
  AttnLaunch a;
  memset(&a, 0, sizeof(a));
  a.dtype = dtype; a.d = d; a.causal = 0;
  a.n_batch = hkv; a.batch_per_kv = 1; a.rows = (hq / hkv) * n_q_tok; a.m = m_total;
  a.q = q_tok; a.k = k_c; a.v = v_c; a.out = out; a.lse = lse; a.scale = scale;
  a.n_split = p.n_split; a.chunk = p.chunk;
  if (p.n_split > 1) {
    a.part_o = reinterpret_cast<float*>(static_cast<char*>(ws) + p.part_o);
    a.part_lse = reinterpret_cast<float*>(static_cast<char*>(ws) + p.part_lse);
  }
  return a;
}

static hipError_t run_attn(const AttnLaunch& a, hipStream_t s) {
  hipError_t e = a.dtype == SAMKV_BF16 ? launch_attn_bf16(a, s) : launch_attn_f32(a, s);
  if (e == hipSuccess && !a.causal && a.n_split > 1) e = launch_attn_merge(a, s);
  return e;
}

int samkv_recompute_attn(const void* q_rec, const void* k_c, const void* v_c, int32_t m_total, int32_t n_q_heads,
                         int32_t n_kv_heads, int32_t head_dim, int32_t dtype, float scale, float* out, float* lse,
                         void* ws, size_t ws_bytes, void* stream) {
  int rc = check_attn(q_rec, k_c, v_c, m_total, m_total, n_q_heads, n_kv_heads, head_dim, dtype, scale, out, lse);
  if (rc != SAMKV_OK) return rc;
  const AttnWs w = attn_ws(dtype, true, n_kv_heads, 0, m_total, head_dim);
  if (w.bytes > 0 && (ws == nullptr || ((uintptr_t)ws % kAlign) != 0 || ws_bytes < w.bytes)) return SAMKV_EWORKSPACE;
  AttnLaunch a = recompute_launch(q_rec, k_c, v_c, m_total, n_q_heads, n_kv_heads, head_dim, dtype, scale, out, lse);
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e = prepare_v(&a, w.vp, static_cast<char*>(ws) + w.vp_at, n_kv_heads, s);
  if (e == hipSuccess) e = run_attn(a, s);
  return dev(e);
}

int samkv_query_attn(const void* q_tok, int32_t n_q_tok, const void* k_c, const void* v_c, int32_t m_total,
                     int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim, int32_t dtype, float scale, float* out,
                     float* lse, void* ws, size_t ws_bytes, void* stream) {
  int rc = check_attn(q_tok, k_c, v_c, n_q_tok, m_total, n_q_heads, n_kv_heads, head_dim, dtype, scale, out, lse);
  if (rc != SAMKV_OK) return rc;
  const AttnWs w = attn_ws(dtype, false, n_kv_heads, (n_q_heads / n_kv_heads) * n_q_tok, m_total, head_dim);
  if (w.bytes > 0 && (ws == nullptr || ((uintptr_t)ws % kAlign) != 0 || ws_bytes < w.bytes)) return SAMKV_EWORKSPACE;
  AttnLaunch a = query_launch(q_tok, n_q_tok, k_c, v_c, m_total, n_q_heads, n_kv_heads, head_dim, dtype, scale, out, lse,
                              w.split, ws);
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e = prepare_v(&a, w.vp, static_cast<char*>(ws) + w.vp_at, n_kv_heads, s);
  if (e == hipSuccess) e = run_attn(a, s);
  return dev(e);
}

int samkv_recompute_query_attn(const void* q_rec, const void* q_tok, int32_t n_q_tok, const void* k_c, const void* v_c,
                               int32_t m_total, int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim, int32_t dtype,
                               float scale, float* rec_out, float* rec_lse, float* q_out, float* q_lse, void* ws,
                               size_t ws_bytes, void* stream) {
  int rc = check_attn(q_rec, k_c, v_c, m_total, m_total, n_q_heads, n_kv_heads, head_dim, dtype, scale, rec_out, rec_lse);
  if (rc != SAMKV_OK) return rc;
  rc = check_attn(q_tok, k_c, v_c, n_q_tok, m_total, n_q_heads, n_kv_heads, head_dim, dtype, scale, q_out, q_lse);
  if (rc != SAMKV_OK) return rc;
  // the workspace of the query attention holds the prepared V behind its key-chunk partials; the causal attention
  // needs nothing else, so one preparation serves both
  const AttnWs w = attn_ws(dtype, false, n_kv_heads, (n_q_heads / n_kv_heads) * n_q_tok, m_total, head_dim);
  if (w.bytes > 0 && (ws == nullptr || ((uintptr_t)ws % kAlign) != 0 || ws_bytes < w.bytes)) return SAMKV_EWORKSPACE;
  AttnLaunch rec = recompute_launch(q_rec, k_c, v_c, m_total, n_q_heads, n_kv_heads, head_dim, dtype, scale, rec_out, rec_lse);
  AttnLaunch qry = query_launch(q_tok, n_q_tok, k_c, v_c, m_total, n_q_heads, n_kv_heads, head_dim, dtype, scale, q_out,
                                q_lse, w.split, ws);
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e = prepare_v(&rec, w.vp, static_cast<char*>(ws) + w.vp_at, n_kv_heads, s);
  qry.v = rec.v;
  qry.v_unscale = rec.v_unscale;
  if (dtype == SAMKV_BF16) {
    if (e == hipSuccess) e = launch_attn_bf16_pair(rec, qry, s);
  } else {
    if (e == hipSuccess) e = run_attn(rec, s);
    if (e == hipSuccess) e = run_attn(qry, s);
  }
  return dev(e);
}

int samkv_query_attn_self(const void* q_tok, int32_t n_q_tok, const void* k_c, const void* v_c, int32_t m_total,
                          const void* k_self, const void* v_self, int32_t n_q_heads, int32_t n_kv_heads,
                          int32_t head_dim, int32_t dtype, float scale, float* out, float* lse, void* ws,
                          size_t ws_bytes, void* stream) {
  int rc = check_attn(q_tok, k_c, v_c, n_q_tok, m_total, n_q_heads, n_kv_heads, head_dim, dtype, scale, out, lse);
  if (rc != SAMKV_OK) return rc;
  if (k_self == nullptr || v_self == nullptr || !aligned16(k_self) || !aligned16(v_self)) return SAMKV_EINVAL;
  const SelfWs w = self_ws(n_q_heads, n_kv_heads, head_dim, n_q_tok, m_total, dtype);
  if (ws == nullptr || ((uintptr_t)ws % kAlign) != 0 || ws_bytes < w.bytes) return SAMKV_EWORKSPACE;
  char* base = static_cast<char*>(ws);
  const size_t n_rows = (size_t)n_q_heads * n_q_tok;
  float* part_o = reinterpret_cast<float*>(base + w.part_o);
  float* part_lse = reinterpret_cast<float*>(base + w.part_lse);
  // slot 0: the query over the compacted cache (no mask); slot 1: the query over its own K/V (causal)
  rc = samkv_query_attn(q_tok, n_q_tok, k_c, v_c, m_total, n_q_heads, n_kv_heads, head_dim, dtype, scale, part_o,
                        part_lse, base + w.inner, ws_bytes - w.inner, stream);
  if (rc != SAMKV_OK) return rc;
  rc = samkv_recompute_attn(q_tok, k_self, v_self, n_q_tok, n_q_heads, n_kv_heads, head_dim, dtype, scale,
                            part_o + n_rows * head_dim, part_lse + n_rows, base + w.inner, ws_bytes - w.inner, stream);
  if (rc != SAMKV_OK) return rc;
  AttnLaunch a;
  memset(&a, 0, sizeof(a));
  a.d = head_dim; a.n_batch = n_q_heads; a.batch_per_kv = n_q_heads / n_kv_heads; a.rows = n_q_tok;
  a.out = out; a.lse = lse; a.n_split = 2; a.part_o = part_o; a.part_lse = part_lse;
  return dev(launch_attn_merge(a, static_cast<hipStream_t>(stream)));
}

int samkv_kv_update(void* k_c, void* v_c, const void* k_new, const void* v_new, int32_t m_total, int32_t n_kv_heads,
                    int32_t head_dim, int32_t dtype, int32_t mode, void* stream) {
  if (k_c == nullptr || v_c == nullptr || k_new == nullptr || v_new == nullptr) return SAMKV_EINVAL;
  if (!aligned16(k_c) || !aligned16(v_c) || !aligned16(k_new) || !aligned16(v_new)) return SAMKV_EINVAL;
  if (m_total < 1 || n_kv_heads < 1 || (mode != SAMKV_OVERWRITE && mode != SAMKV_FUSION)) return SAMKV_EINVAL;
  if (dtype != SAMKV_F32 && dtype != SAMKV_BF16) return SAMKV_EUNSUPPORTED;
  if (head_dim != 64 && head_dim != 128) return SAMKV_EUNSUPPORTED;
  UpdateLaunch a;
  a.dtype = dtype; a.d = head_dim; a.fusion = mode == SAMKV_FUSION;
  a.n_rows = (long long)m_total * n_kv_heads;
  a.k_cur = k_c; a.v_cur = v_c; a.k_new = k_new; a.v_new = v_new;
  return dev(launch_kv_update(a, static_cast<hipStream_t>(stream)));
}

}  // extern "C"
