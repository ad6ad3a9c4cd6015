// Host side of libskipkv: argument validation, workspace carving, kernel sequencing, timing.
// No device work happens here and nothing is allocated on the device.
#include <algorithm>
#include <atomic>
#include <cstdlib>
#include <new>

#include "common.h"

namespace skipkv {

struct Profile {
  hipEvent_t ev[2 * SKIPKV_PROFILE_SLOTS];
  const char *name[SKIPKV_PROFILE_SLOTS];
  int32_t n;
};

namespace {

inline size_t align_up(size_t x) { return (x + 255) & ~(size_t)255; }

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int check_cache(const skipkv_cache *c, bool need_sentences) {
  if (!c) return SKIPKV_EINVAL;
  if (c->dtype != SKIPKV_F32 && c->dtype != SKIPKV_BF16) return SKIPKV_EINVAL;
  if (c->head_dim != SKIPKV_HEAD_DIM) return SKIPKV_ECAPACITY;
  if (c->n_layers < 0 || c->n_kv_heads < 0 || c->batch < 0 || c->total_tokens < 0) return SKIPKV_EINVAL;
  const bool empty = c->n_layers == 0 || c->n_kv_heads == 0 || c->batch == 0;
  if (empty) return SKIPKV_OK;
  if (!c->seq_off) return SKIPKV_EINVAL;
  if (c->total_tokens > 0) {
    if (!c->k || !c->v || !aligned16(c->k) || !aligned16(c->v)) return SKIPKV_EINVAL;
    if (c->stride_tok < c->head_dim || (c->stride_tok % 8) || (c->stride_head % 8) || (c->stride_layer % 8)) return SKIPKV_EINVAL;
    if (c->stride_head < 0 || c->stride_layer < 0) return SKIPKV_EINVAL;
  }
  if (need_sentences) {
    if (!c->sent_ptr || !c->sent_off || c->total_sentences < 0) return SKIPKV_EINVAL;
    if (c->n_q_heads <= 0 || c->n_q_heads % c->n_kv_heads) return SKIPKV_EINVAL;
  }
  return SKIPKV_OK;
}

int check_params(const skipkv_cache *c, const skipkv_params *p, RowLayout *rl) {
  if (!p) return SKIPKV_EINVAL;
  if (p->obs_window < 1 || p->protect_window < 0) return SKIPKV_EINVAL;
  if (!(p->sigma >= 0.f && p->sigma <= 1.f) || !(p->tau == p->tau)) return SKIPKV_EINVAL;
  if (p->obs_window > p->protect_window) return SKIPKV_EBUDGET;
  if (p->max_budget < 0) return SKIPKV_EINVAL;
  if (!p->budget && (p->budget_scalar < p->protect_window || p->budget_scalar > p->max_budget)) return SKIPKV_EBUDGET;
  if (p->budget && p->max_budget < p->protect_window) return SKIPKV_EBUDGET;
  const int n = c->n_kv_heads > 0 ? c->n_q_heads / c->n_kv_heads : 1;
  if (!make_row_layout(n, p->obs_window, rl)) return SKIPKV_ECAPACITY;
  if (c->dtype == SKIPKV_F32 && rl->rows > 160) return SKIPKV_ECAPACITY;  // fp32 query tile would not fit in LDS
  rl->rows = scan_two_pass_rows(*rl, c->dtype);
  return SKIPKV_OK;
}

// Carve the workspace.  `base` may be NULL to only compute the size.
Workspace carve(const skipkv_cache *c, const RowLayout &rl, void *base) {
  Workspace w{};
  const size_t B = (size_t)c->batch, LH = (size_t)c->n_layers * c->n_kv_heads;
  const size_t T = (size_t)c->total_tokens, S = (size_t)c->total_sentences;
  // two consecutive chunks of a sequence together exceed kChunkCap tokens or kChunkMaxSent sentences
  w.nc_max = (int32_t)(2 * ((T + kChunkCap - 1) / kChunkCap + (S + kChunkMaxSent - 1) / kChunkMaxSent) + B);
  w.nrb_max = (int32_t)((S + kRowBlock - 1) / kRowBlock + B);
  // two consecutive spans of a sequence together exceed kSpanCap tokens or kSpanMaxSent sentences
  const size_t spans_max = 2 * ((T + kSpanCap - 1) / kSpanCap + (S + kSpanMaxSent - 1) / kSpanMaxSent) + B;
  w.ni_max = (int32_t)std::min<size_t>(spans_max / kItemSpans + B + 1, (size_t)0x7FFFFFFF);
  w.fits = w.nc_max <= kHdrMaxChunks && spans_max / kItemSpans + B + 1 <= (size_t)kHdrMaxItems && w.nrb_max <= kHdrMaxRowBlocks;
  w.rows = rl.rows;
  size_t off = 0;
  char *p = static_cast<char *>(base);
  auto take = [&](size_t bytes) {
    void *r = p ? p + off : nullptr;
    off += align_up(bytes);
    return r;
  };
  w.hdr = static_cast<PlanHeader *>(take(sizeof(PlanHeader)));
  w.chunk_base = static_cast<int32_t *>(take(B * 4));
  w.chunk_cnt = static_cast<int32_t *>(take(B * 4));
  w.rb_base = static_cast<int32_t *>(take(B * 4));
  w.rb_cnt = static_cast<int32_t *>(take(B * 4));
  w.seq_fused = static_cast<int32_t *>(take(B * 4));
  w.item_rec = static_cast<int32_t *>(take((size_t)w.ni_max * kItemRecInts * 4));
  w.chunks = static_cast<Chunk *>(take((size_t)w.nc_max * sizeof(Chunk)));
  w.rowblocks = static_cast<RowBlock *>(take((size_t)w.nrb_max * sizeof(RowBlock)));
  w.stat_part = static_cast<float2 *>(take(LH * w.nc_max * rl.rows * sizeof(float2)));
  w.item_stat = static_cast<float2 *>(take(LH * w.ni_max * rl.rows * sizeof(float2)));
  w.row_norm = static_cast<float *>(take(LH * B * rl.rows * sizeof(float)));
  w.vhat_hi = static_cast<uint16_t *>(take(LH * S * kD * 2));
  w.vhat_lo = static_cast<uint16_t *>(take(LH * S * kD * 2));
  w.sent_imp = static_cast<float *>(take(LH * S * 4));
  w.sent_red = static_cast<float *>(take(LH * S * 4));
  w.bytes = off;
  return w;
}

// What a call with per-head ranges adds to the (virtual) cache description: explicit lengths and
// sentence counts per virtual sequence, and how to find the query rows of the real head.
struct HeadView {
  const int32_t *len = nullptr, *cnt = nullptr;
  int32_t virt_hk = 0, virt_b = 0;
  const int32_t *row_map = nullptr;  // paged cache: logical token -> slot row
  int32_t page_size = 0;             // ... and its slots per block
  int64_t map_stride = 0;            // ... and the elements per unit of the map (0: stride_tok)
  const int32_t *sent_id = nullptr, *lam_ptr = nullptr;  // shared lambda on per-head ranges: sentence numbers, CSR of the lambda array
};

struct Timer {
  Profile *p;
  hipStream_t st;
  Timer(void *prof, hipStream_t s) : p(static_cast<Profile *>(prof)), st(s) {
    if (p) p->n = 0;
  }
  template <class F>
  hipError_t run(const char *name, F &&f) {
    int slot = -1;
    if (p && p->n < SKIPKV_PROFILE_SLOTS) {
      slot = p->n++;
      p->name[slot] = name;
      (void)hipEventRecord(p->ev[2 * slot], st);
    }
    const hipError_t e = f();
    if (slot >= 0) (void)hipEventRecord(p->ev[2 * slot + 1], st);
    return e;
  }
};

int do_score(Timer &tm, const skipkv_cache *c, const skipkv_params *p, const RowLayout &rl, const void *q_obs,
             const float *tok_red, float *sent_score, float *sent_lambda, float *tok_imp, void *ws, hipStream_t st,
             const HeadView &hv = HeadView(), const float *shared_lambda = nullptr) {
  const Workspace w = carve(c, rl, ws);
  PlanArgs pa{c->seq_off, c->sent_ptr, c->sent_off, c->batch, c->n_layers * c->n_kv_heads, w, p->dev_status, hv.len, hv.cnt};
  if (tm.run("plan", [&] { return launch_plan(pa, st); }) != hipSuccess) return SKIPKV_EHIP;
  ScanArgs sa{};
  sa.k = c->k;
  sa.q = q_obs;
  sa.stride_layer = c->stride_layer;
  sa.stride_head = c->stride_head;
  sa.stride_tok = c->stride_tok;
  sa.dtype = c->dtype;
  sa.n_layers = c->n_layers;
  sa.n_kv_heads = c->n_kv_heads;
  sa.n_q_heads = c->n_q_heads;
  sa.batch = c->batch;
  sa.total_tokens = c->total_tokens;
  sa.total_sentences = c->total_sentences;
  sa.alpha = p->obs_window;
  sa.protect = p->protect_window;
  sa.seq_off = c->seq_off;
  sa.sent_ptr = c->sent_ptr;
  sa.sent_off = c->sent_off;
  sa.tok_red = tok_red;
  sa.tok_imp = tok_imp;
  sa.ws = w;
  sa.rl = rl;
  sa.row_map = hv.row_map;
  sa.page_size = hv.page_size;
  sa.map_stride = hv.map_stride ? hv.map_stride : c->stride_tok;
  const bool pages_fit_stages = hv.page_size >= 16 && (hv.page_size & (hv.page_size - 1)) == 0;
  sa.force_two_pass = (hv.row_map != nullptr && !pages_fit_stages) || (p->flags & SKIPKV_FLAG_FORCE_TWO_PASS) || !scan_fused_supported(rl, c->stride_tok * (c->dtype == SKIPKV_BF16 ? 2 : 4));
  sa.spin_limit = p->spin_limit == 0 ? 4000000 : std::max(p->spin_limit, 0);
  sa.dev_status = p->dev_status;
  sa.virt_hk = hv.virt_hk;
  sa.virt_b = hv.virt_b;
  sa.no_pool = shared_lambda != nullptr;
  if (tm.run("scan_fused", [&] { return launch_scan_fused(sa, st); }) != hipSuccess) return SKIPKV_EHIP;
  if (tm.run("scan_stats", [&] { return launch_scan_stats(sa, st); }) != hipSuccess) return SKIPKV_EHIP;
  if (tm.run("row_norm", [&] { return launch_row_norm(sa, st); }) != hipSuccess) return SKIPKV_EHIP;
  if (tm.run("scan_scores", [&] { return launch_scan_scores(sa, st); }) != hipSuccess) return SKIPKV_EHIP;
  if (shared_lambda) {  // lambda per sequence (hidden-state similarity): no Gram matrices per head
    FuseSharedArgs fa{};
    fa.n_lh = c->n_layers * c->n_kv_heads;
    fa.batch = c->batch;
    fa.total_sentences = c->total_sentences;
    fa.protect = p->protect_window;
    fa.sigma = p->sigma;
    fa.tau = p->tau;
    fa.has_red = tok_red != nullptr;
    fa.seq_off = c->seq_off;
    fa.sent_ptr = c->sent_ptr;
    fa.sent_off = c->sent_off;
    fa.sent_imp = w.sent_imp;
    fa.sent_red = w.sent_red;
    fa.shared_lambda = shared_lambda;
    fa.sent_score = sent_score;
    fa.sent_lambda = sent_lambda;
    fa.len = hv.len;
    fa.cnt = hv.cnt;
    fa.sent_id = hv.sent_id;
    fa.lam_ptr = hv.lam_ptr;
    fa.virt_b = hv.virt_b;
    fa.dev_status = p->dev_status;
    if (tm.run("fuse", [&] { return launch_fuse_shared(fa, st); }) != hipSuccess) return SKIPKV_EHIP;
    return SKIPKV_OK;
  }
  CosineArgs ca{};
  ca.n_lh = c->n_layers * c->n_kv_heads;
  ca.batch = c->batch;
  ca.total_sentences = c->total_sentences;
  ca.protect = p->protect_window;
  ca.sigma = p->sigma;
  ca.tau = p->tau;
  ca.has_red = tok_red != nullptr;
  ca.seq_off = c->seq_off;
  ca.sent_ptr = c->sent_ptr;
  ca.sent_off = c->sent_off;
  ca.ws = w;
  ca.sent_score = sent_score;
  ca.sent_lambda = sent_lambda;
  ca.len = hv.len;
  ca.cnt = hv.cnt;
  if (tm.run("redundancy", [&] { return launch_cosine(ca, st); }) != hipSuccess) return SKIPKV_EHIP;
  return SKIPKV_OK;
}

int do_select(Timer &tm, const skipkv_cache *c, const skipkv_params *p, const float *sent_score, uint8_t *sent_keep,
              int32_t *kept_idx, int32_t *new_len, int32_t *new_sent_off, int32_t *new_sent_cnt, int32_t kept_stride,
              hipStream_t st, const HeadView &hv = HeadView()) {
  SelectArgs a{};
  a.n_lh = c->n_layers * c->n_kv_heads;
  a.batch = c->batch;
  a.total_sentences = c->total_sentences;
  a.protect = p->protect_window;
  a.budget_scalar = p->budget_scalar;
  a.kept_stride = kept_stride;
  a.budget = p->budget;
  a.seq_off = c->seq_off;
  a.sent_ptr = c->sent_ptr;
  a.sent_off = c->sent_off;
  a.sent_score = sent_score;
  a.sent_keep = sent_keep;
  a.kept_idx = kept_idx;
  a.new_len = new_len;
  a.new_sent_off = new_sent_off;
  a.new_sent_cnt = new_sent_cnt;
  a.dev_status = p->dev_status;
  a.len = hv.len;
  a.cnt = hv.cnt;
  if (tm.run("select", [&] { return launch_select(a, st); }) != hipSuccess) return SKIPKV_EHIP;
  return SKIPKV_OK;
}

int do_compact(Timer &tm, const skipkv_cache *c, const int32_t *kept_idx, const int32_t *new_len, int32_t kept_stride,
               hipStream_t st, const int32_t *row_map = nullptr, const int32_t *seq_bad = nullptr,
               int32_t *src_rows = nullptr, int32_t src_stride = 0, int64_t map_stride = 0) {
  CompactArgs a{};
  a.map_stride = map_stride ? map_stride : c->stride_tok;
  a.row_map = row_map;
  a.seq_bad = seq_bad;
  a.src_rows = src_rows;
  a.src_stride = src_stride;
  a.k = c->k;
  a.v = c->v;
  a.stride_layer = c->stride_layer;
  a.stride_head = c->stride_head;
  a.stride_tok = c->stride_tok;
  a.dtype = c->dtype;
  a.n_layers = c->n_layers;
  a.n_kv_heads = c->n_kv_heads;
  a.batch = c->batch;
  a.kept_stride = kept_stride;
  a.seq_off = c->seq_off;
  a.kept_idx = kept_idx;
  a.new_len = new_len;
  if (tm.run("compact", [&] { return launch_compact(a, st); }) != hipSuccess) return SKIPKV_EHIP;
  return SKIPKV_OK;
}

bool is_empty(const skipkv_cache *c) { return c->n_layers == 0 || c->n_kv_heads == 0 || c->batch == 0; }

// Workspace of the token redundancy: per key row a scale factor and a reciprocal row sum (fp32 each) and a
// 64-bit fixed-point accumulator.
size_t tokred_per(const skipkv_cache *c) {
  return align_up((size_t)c->n_layers * c->n_kv_heads * (size_t)c->total_tokens * sizeof(float));
}
size_t tokred_bytes(const skipkv_cache *c) { return 4 * tokred_per(c); }
TokRedArgs tokred_args(const skipkv_cache *c, void *ws, float *out) {
  const size_t per = tokred_per(c);
  TokRedArgs a{};
  a.k = c->k;
  a.stride_layer = c->stride_layer;
  a.stride_head = c->stride_head;
  a.stride_tok = c->stride_tok;
  a.dtype = c->dtype;
  a.n_layers = c->n_layers;
  a.n_kv_heads = c->n_kv_heads;
  a.batch = c->batch;
  a.total_tokens = c->total_tokens;
  a.nrb_max = (c->total_tokens + kTokredRows - 1) / kTokredRows + c->batch;
  a.seq_off = c->seq_off;
  a.scale = static_cast<float *>(ws);
  a.inv_l = reinterpret_cast<float *>(static_cast<char *>(ws) + per);
  a.acc = reinterpret_cast<unsigned long long *>(static_cast<char *>(ws) + 2 * per);
  a.out = out;
  return a;
}

// Per-head ranges.  Every (layer, KV head, sequence) triple becomes a sequence of its own of a
// cache with ONE layer and ONE KV head: v = (l * H_k + h) * B + b, whose tokens start at packed
// row (l * H_k + h) * T + seq_off[b] of the (contiguous) K and V and whose offsets start at
// (l * H_k + h) * (S + B) + sent_ptr[b] of the per-head offset array.  With this numbering the
// per-sentence, per-token and per-sequence outputs keep exactly their real layout, so the same
// kernels serve; only lengths and counts become explicit and the query rows keep the real (l, b, h).
struct VirtualView {
  skipkv_cache c;
  HeadView hv;
  int32_t *seq_off, *sent_ptr;  // [LH * B + 1] each, at the head of the workspace
  size_t head_bytes;            // bytes taken from the workspace for them
};

int make_virtual(const skipkv_cache *c, const skipkv_ranges *r, void *ws, VirtualView *out, bool paged = false) {
  if (!r || !r->len || !r->sent_cnt || !r->sent_off) return SKIPKV_EINVAL;
  const int64_t LH = (int64_t)c->n_layers * c->n_kv_heads, B = c->batch;
  const int64_t T = c->total_tokens, S = c->total_sentences;
  if (LH * B >= (1ll << 31) - 1 || LH * T >= (1ll << 31) - 1 || LH * (S + B) >= (1ll << 31) - 1) return SKIPKV_ECAPACITY;
  // K and V must be one flat array of rows over (layer, head, token), unless a row map says where the rows are
  if (!paged && T > 0 && (c->stride_head != T * c->stride_tok || c->stride_layer != c->n_kv_heads * c->stride_head)) return SKIPKV_ECAPACITY;
  VirtualView v{};
  v.c = *c;
  v.c.n_layers = 1;
  v.c.n_kv_heads = 1;
  v.c.n_q_heads = c->n_q_heads / c->n_kv_heads;
  v.c.batch = (int32_t)(LH * B);
  v.c.total_tokens = (int32_t)(LH * T);
  v.c.total_sentences = (int32_t)(LH * S);
  v.c.stride_layer = 0;
  v.c.stride_head = 0;
  v.head_bytes = 2 * align_up((size_t)(LH * B + 1) * 4);
  v.seq_off = static_cast<int32_t *>(ws);
  v.sent_ptr = ws ? reinterpret_cast<int32_t *>(static_cast<char *>(ws) + v.head_bytes / 2) : nullptr;
  v.c.seq_off = v.seq_off;
  v.c.sent_ptr = v.sent_ptr;
  v.c.sent_off = r->sent_off;
  v.hv.len = r->len;
  v.hv.cnt = r->sent_cnt;
  v.hv.virt_hk = c->n_kv_heads;
  v.hv.virt_b = c->batch;
  *out = v;
  return SKIPKV_OK;
}

int check_score_args(const skipkv_cache *c, const skipkv_params *p, RowLayout *rl, const void *q_obs, float *sent_score,
                     float *sent_lambda, void *ws, size_t ws_bytes) {
  int rc = check_cache(c, true);
  if (rc) return rc;
  rc = check_params(c, p, rl);
  if (rc) return rc;
  if (is_empty(c)) return SKIPKV_OK;
  if (!q_obs || !aligned16(q_obs)) return SKIPKV_EINVAL;
  if (c->total_sentences > 0 && (!sent_score || !sent_lambda)) return SKIPKV_EINVAL;
  const Workspace w = carve(c, *rl, nullptr);
  if (!w.fits) return SKIPKV_ECAPACITY;
  if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255u) || ws_bytes < w.bytes) return SKIPKV_EWORKSPACE;
  return SKIPKV_OK;
}

int check_select_args(const skipkv_cache *c, const skipkv_params *p, RowLayout *rl, const float *sent_score,
                      int32_t *kept_idx, int32_t *new_len, int32_t *new_sent_off, int32_t *new_sent_cnt,
                      int32_t kept_stride) {
  int rc = check_cache(c, true);
  if (rc) return rc;
  rc = check_params(c, p, rl);
  if (rc) return rc;
  if (is_empty(c)) return SKIPKV_OK;
  if (!new_len || (c->total_sentences > 0 && !sent_score)) return SKIPKV_EINVAL;
  if ((new_sent_off == nullptr) != (new_sent_cnt == nullptr)) return SKIPKV_EINVAL;
  const int32_t need = p->max_budget < c->total_tokens ? p->max_budget : c->total_tokens;
  if (kept_stride < need || (need > 0 && !kept_idx)) return SKIPKV_EINVAL;
  return SKIPKV_OK;
}

}  // namespace
}  // namespace skipkv

using namespace skipkv;

extern "C" {

int skipkv_workspace_bytes(const skipkv_cache *cache, const skipkv_params *params, size_t *out_bytes) {
  if (!out_bytes) return SKIPKV_EINVAL;
  int rc = check_cache(cache, true);
  if (rc) return rc;
  RowLayout rl;
  rc = check_params(cache, params, &rl);
  if (rc) return rc;
  const Workspace w = carve(cache, rl, nullptr);
  if (!w.fits) return SKIPKV_ECAPACITY;
  *out_bytes = w.bytes;
  return SKIPKV_OK;
}

int skipkv_score(const skipkv_cache *cache, const skipkv_params *params, const void *q_obs,
                 const float *tok_redundancy, float *sent_score, float *sent_lambda, float *tok_importance,
                 void *ws, size_t ws_bytes, void *stream) {
  RowLayout rl;
  const int rc = check_score_args(cache, params, &rl, q_obs, sent_score, sent_lambda, ws, ws_bytes);
  if (rc) return rc;
  if (is_empty(cache)) return SKIPKV_OK;
  Timer tm(params->profile, static_cast<hipStream_t>(stream));
  return do_score(tm, cache, params, rl, q_obs, tok_redundancy, sent_score, sent_lambda, tok_importance, ws,
                  static_cast<hipStream_t>(stream));
}

int skipkv_select(const skipkv_cache *cache, const skipkv_params *params, const float *sent_score,
                  uint8_t *sent_keep, int32_t *kept_idx, int32_t *new_len, int32_t *new_sent_off,
                  int32_t *new_sent_cnt, int32_t kept_stride, void *stream) {
  RowLayout rl;
  const int rc = check_select_args(cache, params, &rl, sent_score, kept_idx, new_len, new_sent_off, new_sent_cnt, kept_stride);
  if (rc) return rc;
  if (is_empty(cache)) return SKIPKV_OK;
  Timer tm(params->profile, static_cast<hipStream_t>(stream));
  return do_select(tm, cache, params, sent_score, sent_keep, kept_idx, new_len, new_sent_off, new_sent_cnt, kept_stride,
                   static_cast<hipStream_t>(stream));
}

namespace {
int do_select_tokens(const skipkv_cache *c, const skipkv_params *p, const float *tok_importance, const float *tok_redundancy,
                     const float *sent_lambda, float *tok_score, uint8_t *tok_keep, int32_t *kept_idx, int32_t *new_len,
                     int32_t *new_sent_off, int32_t *new_sent_cnt, int32_t kept_stride, hipStream_t st,
                     const HeadView &hv = HeadView()) {
  TokSelectArgs a{};
  a.n_lh = c->n_layers * c->n_kv_heads;
  a.batch = c->batch;
  a.total_tokens = c->total_tokens;
  a.total_sentences = c->total_sentences;
  a.protect = p->protect_window;
  a.budget_scalar = p->budget_scalar;
  a.kept_stride = kept_stride;
  a.sigma = p->sigma;
  a.tau = p->tau;
  a.budget = p->budget;
  a.seq_off = c->seq_off;
  a.sent_ptr = c->sent_ptr;
  a.sent_off = c->sent_off;
  a.tok_imp = tok_importance;
  a.tok_red = tok_redundancy;
  a.sent_lambda = sent_lambda;
  a.tok_score = tok_score;
  a.tok_keep = tok_keep;
  a.kept_idx = kept_idx;
  a.new_len = new_len;
  a.new_sent_off = new_sent_off;
  a.new_sent_cnt = new_sent_cnt;
  a.dev_status = p->dev_status;
  a.len = hv.len;
  a.cnt = hv.cnt;
  return launch_select_tokens(a, st) == hipSuccess ? SKIPKV_OK : SKIPKV_EHIP;
}
}  // namespace

int skipkv_select_tokens(const skipkv_cache *cache, const skipkv_params *params, const float *tok_importance,
                         const float *tok_redundancy, const float *sent_lambda, float *tok_score,
                         uint8_t *tok_keep, int32_t *kept_idx, int32_t *new_len, int32_t *new_sent_off,
                         int32_t *new_sent_cnt, int32_t kept_stride, void *stream) {
  RowLayout rl;
  const int rc = check_select_args(cache, params, &rl, sent_lambda, kept_idx, new_len, new_sent_off, new_sent_cnt, kept_stride);
  if (rc) return rc;
  if (is_empty(cache)) return SKIPKV_OK;
  if (cache->total_tokens > 0 && (!tok_importance || !tok_score)) return SKIPKV_EINVAL;
  return do_select_tokens(cache, params, tok_importance, tok_redundancy, sent_lambda, tok_score, tok_keep, kept_idx, new_len,
                          new_sent_off, new_sent_cnt, kept_stride, static_cast<hipStream_t>(stream));
}

int skipkv_compact(const skipkv_cache *cache, const int32_t *kept_idx, const int32_t *new_len, int32_t kept_stride,
                   void *stream) {
  const int rc = check_cache(cache, false);
  if (rc) return rc;
  if (is_empty(cache)) return SKIPKV_OK;
  if (!new_len || kept_stride < 0 || (!kept_idx && cache->total_tokens > 0)) return SKIPKV_EINVAL;
  Timer tm(nullptr, static_cast<hipStream_t>(stream));
  return do_compact(tm, cache, kept_idx, new_len, kept_stride, static_cast<hipStream_t>(stream));
}

int skipkv_step(const skipkv_cache *cache, const skipkv_params *params, const void *q_obs,
                const float *tok_redundancy, float *sent_score, float *sent_lambda, float *tok_importance,
                uint8_t *sent_keep, int32_t *kept_idx, int32_t *new_len, int32_t *new_sent_off,
                int32_t *new_sent_cnt, int32_t kept_stride, void *ws, size_t ws_bytes, void *stream) {
  RowLayout rl;
  int rc = check_score_args(cache, params, &rl, q_obs, sent_score, sent_lambda, ws, ws_bytes);
  if (rc) return rc;
  rc = check_select_args(cache, params, &rl, sent_score, kept_idx, new_len, new_sent_off, new_sent_cnt, kept_stride);
  if (rc) return rc;
  if (is_empty(cache)) return SKIPKV_OK;
  hipStream_t st = static_cast<hipStream_t>(stream);
  Timer tm(params->profile, st);
  rc = do_score(tm, cache, params, rl, q_obs, tok_redundancy, sent_score, sent_lambda, tok_importance, ws, st);
  if (rc) return rc;
  rc = do_select(tm, cache, params, sent_score, sent_keep, kept_idx, new_len, new_sent_off, new_sent_cnt, kept_stride, st);
  if (rc) return rc;
  return do_compact(tm, cache, kept_idx, new_len, kept_stride, st);
}

// Scratch of skipkv_step_static: one array per GPU, held by the code object from the moment it is
// loaded until the process ends.  In host code this name only stands for the symbol; the
// array's address on a device comes from hipGetSymbolAddress (static_scratch below).
static __device__ __align__(256) unsigned char scratch[SKIPKV_STATIC_WS_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::atomic<void *> g_scratch_ptr[kMaxDevices];

// Address of `scratch` on the current device, looked up once per device.
int static_scratch(void **out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) return SKIPKV_EHIP;
  if (dev < 0 || dev >= kMaxDevices) return SKIPKV_ECAPACITY;
  void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!p) {
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return SKIPKV_EHIP;
    g_scratch_ptr[dev].store(p, std::memory_order_release);  // every thread finds the same address
  }
  *out = p;
  return SKIPKV_OK;
}
}  // namespace

int skipkv_step_static(const skipkv_cache *cache, const skipkv_params *params, const void *q_obs,
                       const float *tok_redundancy, float *sent_score, float *sent_lambda, float *tok_importance,
                       uint8_t *sent_keep, int32_t *kept_idx, int32_t *new_len, int32_t *new_sent_off,
                       int32_t *new_sent_cnt, int32_t kept_stride, void *stream) {
  int rc = check_cache(cache, true);
  if (rc) return rc;
  RowLayout rl;
  rc = check_params(cache, params, &rl);
  if (rc) return rc;
  const Workspace w = carve(cache, rl, nullptr);
  if (!w.fits) return SKIPKV_ECAPACITY;
  if (w.bytes > (size_t)SKIPKV_STATIC_WS_BYTES) return SKIPKV_EWORKSPACE;  // the problem needs more scratch than the array holds
  void *ws = nullptr;
  rc = static_scratch(&ws);
  if (rc) return rc;
  // From here on this is skipkv_step on the array: the plan's fill kernels reset every counter
  // and marker that must start from a known value, so what the previous call left is harmless.
  return skipkv_step(cache, params, q_obs, tok_redundancy, sent_score, sent_lambda, tok_importance, sent_keep, kept_idx,
                     new_len, new_sent_off, new_sent_cnt, kept_stride, ws, (size_t)SKIPKV_STATIC_WS_BYTES, stream);
}

namespace {
// Validation of a paged cache's description, and where the row map and the per-sequence flags sit
// behind the step's workspace.
struct PagedView {
  size_t step_bytes, map_bytes, bad_bytes, total;
  int32_t rows_per_block, src_stride;
};
int check_paging_desc(const skipkv_cache *c, const skipkv_paging *pg, int64_t *rows_per_block) {
  if (!pg) return SKIPKV_EINVAL;
  if (pg->block_size < 1 || pg->n_blocks < 1 || pg->table_stride < 0 || pg->stride_block < 0) return SKIPKV_EINVAL;
  if (!pg->block_table && c->total_tokens > 0) return SKIPKV_EINVAL;
  if (c->stride_tok <= 0 || pg->stride_block % c->stride_tok) return SKIPKV_EINVAL;
  const int64_t rpb = pg->stride_block / c->stride_tok;
  if (rpb < pg->block_size) return SKIPKV_EINVAL;  // the slots of a block must not reach into the next one
  *rows_per_block = rpb;
  return SKIPKV_OK;
}
int check_paging(const skipkv_cache *c, const skipkv_paging *pg, const skipkv_params *p, const RowLayout &rl, PagedView *v) {
  int64_t rpb = 0;
  const int rc = check_paging_desc(c, pg, &rpb);
  if (rc) return rc;
  if ((int64_t)pg->n_blocks * rpb > 0x7FFFFFFFll) return SKIPKV_ECAPACITY;  // slot rows are 32-bit
  v->rows_per_block = (int32_t)rpb;
  const Workspace w = carve(c, rl, nullptr);
  if (!w.fits) return SKIPKV_ECAPACITY;
  v->step_bytes = align_up(w.bytes);
  v->map_bytes = align_up((size_t)c->total_tokens * 4);
  v->bad_bytes = align_up((size_t)c->batch * 4);
  // slot rows of the kept tokens of every head: no head keeps more than its budget, nor more than there is
  v->src_stride = std::max(1, std::min(p->max_budget, c->total_tokens));
  v->total = v->step_bytes + v->map_bytes + v->bad_bytes +
             align_up((size_t)c->n_layers * c->n_kv_heads * c->batch * v->src_stride * 4);
  return SKIPKV_OK;
}
}  // namespace

int skipkv_paged_workspace_bytes(const skipkv_cache *cache, const skipkv_paging *paging, const skipkv_params *params,
                                 size_t *out_bytes) {
  if (!out_bytes) return SKIPKV_EINVAL;
  int rc = check_cache(cache, true);
  if (rc) return rc;
  RowLayout rl;
  rc = check_params(cache, params, &rl);
  if (rc) return rc;
  if (is_empty(cache)) {
    *out_bytes = 0;
    return SKIPKV_OK;
  }
  PagedView pv;
  rc = check_paging(cache, paging, params, rl, &pv);
  if (rc) return rc;
  *out_bytes = pv.total;
  return SKIPKV_OK;
}

namespace {
int score_paged(const skipkv_cache *cache, const skipkv_paging *paging, const skipkv_params *params, const void *q_obs,
                const float *tok_redundancy, const float *shared_lambda, bool need_lambda_out, float *sent_score,
                float *sent_lambda, float *tok_importance, void *ws, size_t ws_bytes, void *stream) {
  RowLayout rl;
  int rc = check_cache(cache, true);
  if (rc) return rc;
  rc = check_params(cache, params, &rl);
  if (rc) return rc;
  if (is_empty(cache)) return SKIPKV_OK;
  if (!q_obs || !aligned16(q_obs)) return SKIPKV_EINVAL;
  if (cache->total_sentences > 0 && (!sent_score || (need_lambda_out && !sent_lambda))) return SKIPKV_EINVAL;
  PagedView pv;
  rc = check_paging(cache, paging, params, rl, &pv);
  if (rc) return rc;
  if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255u) || ws_bytes < pv.total) return SKIPKV_EWORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  Timer tm(params->profile, st);
  int32_t *row_map = reinterpret_cast<int32_t *>(static_cast<char *>(ws) + pv.step_bytes);
  int32_t *seq_bad = reinterpret_cast<int32_t *>(static_cast<char *>(ws) + pv.step_bytes + pv.map_bytes);
  RowMapArgs ra{cache->seq_off, paging->block_table, cache->batch, paging->table_stride, paging->block_size,
                paging->n_blocks, 1, 1, cache->total_tokens, 0, 0, pv.rows_per_block, 1, row_map, seq_bad, params->dev_status};
  if (tm.run("row_map", [&] { return launch_row_map(ra, st); }) != hipSuccess) return SKIPKV_EHIP;
  HeadView hv;
  hv.row_map = row_map;
  hv.page_size = paging->block_size;
  return do_score(tm, cache, params, rl, q_obs, tok_redundancy, sent_score, sent_lambda, tok_importance, ws, st, hv, shared_lambda);
}
}  // namespace

int skipkv_score_paged(const skipkv_cache *cache, const skipkv_paging *paging, const skipkv_params *params,
                       const void *q_obs, const float *tok_redundancy, float *sent_score, float *sent_lambda,
                       float *tok_importance, void *ws, size_t ws_bytes, void *stream) {
  return score_paged(cache, paging, params, q_obs, tok_redundancy, nullptr, true, sent_score, sent_lambda, tok_importance, ws,
                     ws_bytes, stream);
}

int skipkv_score_shared_paged(const skipkv_cache *cache, const skipkv_paging *paging, const skipkv_params *params,
                              const void *q_obs, const float *tok_redundancy, const float *shared_lambda, float *sent_score,
                              float *sent_lambda, float *tok_importance, void *ws, size_t ws_bytes, void *stream) {
  if (cache && cache->total_sentences > 0 && !shared_lambda) return SKIPKV_EINVAL;
  return score_paged(cache, paging, params, q_obs, tok_redundancy, shared_lambda, false, sent_score, sent_lambda, tok_importance,
                     ws, ws_bytes, stream);
}

namespace {
// Workspace of skipkv_compact_paged: the row map, the per-sequence flags, the slot rows of the kept tokens.
struct CompactPagedView {
  size_t map_bytes, bad_bytes, total;
  int32_t rows_per_block, src_stride;
};
int check_compact_paging(const skipkv_cache *c, const skipkv_paging *pg, int32_t kept_stride, CompactPagedView *v) {
  int64_t rpb = 0;
  const int rc = check_paging_desc(c, pg, &rpb);
  if (rc) return rc;
  if ((int64_t)pg->n_blocks * rpb > 0x7FFFFFFFll) return SKIPKV_ECAPACITY;  // slot rows are 32-bit
  if (kept_stride < 0) return SKIPKV_EINVAL;
  v->rows_per_block = (int32_t)rpb;
  v->src_stride = std::max(1, kept_stride);
  v->map_bytes = align_up((size_t)c->total_tokens * 4);
  v->bad_bytes = align_up((size_t)c->batch * 4);
  v->total = v->map_bytes + v->bad_bytes + align_up((size_t)c->n_layers * c->n_kv_heads * c->batch * v->src_stride * 4);
  return SKIPKV_OK;
}
}  // namespace

int skipkv_compact_paged_workspace_bytes(const skipkv_cache *cache, const skipkv_paging *paging, int32_t kept_stride,
                                         size_t *out_bytes) {
  if (!out_bytes) return SKIPKV_EINVAL;
  const int rc = check_cache(cache, false);
  if (rc) return rc;
  if (is_empty(cache)) {
    *out_bytes = 0;
    return SKIPKV_OK;
  }
  CompactPagedView v;
  const int rc2 = check_compact_paging(cache, paging, kept_stride, &v);
  if (rc2) return rc2;
  *out_bytes = v.total;
  return SKIPKV_OK;
}

int skipkv_compact_paged(const skipkv_cache *cache, const skipkv_paging *paging, const int32_t *kept_idx,
                         const int32_t *new_len, int32_t kept_stride, int32_t *dev_status, void *ws, size_t ws_bytes,
                         void *stream) {
  int rc = check_cache(cache, false);
  if (rc) return rc;
  if (is_empty(cache)) return SKIPKV_OK;
  if (!new_len || kept_stride < 0 || (!kept_idx && cache->total_tokens > 0)) return SKIPKV_EINVAL;
  CompactPagedView v;
  rc = check_compact_paging(cache, paging, kept_stride, &v);
  if (rc) return rc;
  if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255u) || ws_bytes < v.total) return SKIPKV_EWORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  int32_t *row_map = static_cast<int32_t *>(ws);
  int32_t *seq_bad = reinterpret_cast<int32_t *>(static_cast<char *>(ws) + v.map_bytes);
  int32_t *src_rows = reinterpret_cast<int32_t *>(static_cast<char *>(ws) + v.map_bytes + v.bad_bytes);
  RowMapArgs ra{cache->seq_off, paging->block_table, cache->batch, paging->table_stride, paging->block_size,
                paging->n_blocks, 1, 1, cache->total_tokens, 0, 0, v.rows_per_block, 1, row_map, seq_bad, dev_status};
  if (launch_row_map(ra, st) != hipSuccess) return SKIPKV_EHIP;
  Timer tm(nullptr, st);
  return do_compact(tm, cache, kept_idx, new_len, kept_stride, st, row_map, seq_bad, src_rows, v.src_stride);
}

int skipkv_step_paged(const skipkv_cache *cache, const skipkv_paging *paging, const skipkv_params *params,
                      const void *q_obs, const float *tok_redundancy, float *sent_score, float *sent_lambda,
                      float *tok_importance, uint8_t *sent_keep, int32_t *kept_idx, int32_t *new_len,
                      int32_t *new_sent_off, int32_t *new_sent_cnt, int32_t kept_stride, void *ws, size_t ws_bytes,
                      void *stream) {
  RowLayout rl;
  int rc = check_cache(cache, true);
  if (rc) return rc;
  rc = check_params(cache, params, &rl);
  if (rc) return rc;
  rc = check_select_args(cache, params, &rl, sent_score, kept_idx, new_len, new_sent_off, new_sent_cnt, kept_stride);
  if (rc) return rc;
  if (is_empty(cache)) return SKIPKV_OK;
  if (!q_obs || !aligned16(q_obs)) return SKIPKV_EINVAL;
  if (cache->total_sentences > 0 && (!sent_score || !sent_lambda)) return SKIPKV_EINVAL;
  PagedView pv;
  rc = check_paging(cache, paging, params, rl, &pv);
  if (rc) return rc;
  if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255u) || ws_bytes < pv.total) return SKIPKV_EWORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  Timer tm(params->profile, st);
  int32_t *row_map = reinterpret_cast<int32_t *>(static_cast<char *>(ws) + pv.step_bytes);
  int32_t *seq_bad = reinterpret_cast<int32_t *>(static_cast<char *>(ws) + pv.step_bytes + pv.map_bytes);
  RowMapArgs ra{cache->seq_off, paging->block_table, cache->batch, paging->table_stride, paging->block_size,
                paging->n_blocks, 1, 1, cache->total_tokens, 0, 0, pv.rows_per_block, 1, row_map, seq_bad, params->dev_status};
  if (tm.run("row_map", [&] { return launch_row_map(ra, st); }) != hipSuccess) return SKIPKV_EHIP;
  HeadView hv;
  hv.row_map = row_map;
  hv.page_size = paging->block_size;
  rc = do_score(tm, cache, params, rl, q_obs, tok_redundancy, sent_score, sent_lambda, tok_importance, ws, st, hv);
  if (rc) return rc;
  rc = do_select(tm, cache, params, sent_score, sent_keep, kept_idx, new_len, new_sent_off, new_sent_cnt, kept_stride, st);
  if (rc) return rc;
  int32_t *src_rows = reinterpret_cast<int32_t *>(static_cast<char *>(ws) + pv.step_bytes + pv.map_bytes + pv.bad_bytes);
  return do_compact(tm, cache, kept_idx, new_len, kept_stride, st, row_map, seq_bad, src_rows, pv.src_stride);
}

int skipkv_ranges_workspace_bytes(const skipkv_cache *cache, const skipkv_params *params, size_t *out_bytes) {
  if (!out_bytes) return SKIPKV_EINVAL;
  int rc = check_cache(cache, true);
  if (rc) return rc;
  RowLayout rl;
  rc = check_params(cache, params, &rl);
  if (rc) return rc;
  if (is_empty(cache)) {
    *out_bytes = 0;
    return SKIPKV_OK;
  }
  skipkv_ranges dummy{reinterpret_cast<int32_t *>(16), reinterpret_cast<int32_t *>(16), reinterpret_cast<int32_t *>(16)};
  VirtualView v;
  rc = make_virtual(cache, &dummy, nullptr, &v);
  if (rc) return rc;
  const Workspace w = carve(&v.c, rl, nullptr);
  if (!w.fits) return SKIPKV_ECAPACITY;
  *out_bytes = v.head_bytes + w.bytes;
  return SKIPKV_OK;
}

int skipkv_step_ranges(const skipkv_cache *cache, const skipkv_ranges *ranges, const skipkv_params *params,
                       const void *q_obs, const float *tok_redundancy, float *sent_score, float *sent_lambda,
                       float *tok_importance, uint8_t *sent_keep, int32_t *kept_idx, int32_t *new_len,
                       int32_t *new_sent_off, int32_t *new_sent_cnt, int32_t kept_stride, void *ws, size_t ws_bytes,
                       void *stream) {
  RowLayout rl;
  int rc = check_cache(cache, true);
  if (rc) return rc;
  rc = check_params(cache, params, &rl);
  if (rc) return rc;
  rc = check_select_args(cache, params, &rl, sent_score, kept_idx, new_len, new_sent_off, new_sent_cnt, kept_stride);
  if (rc) return rc;
  if (is_empty(cache)) return SKIPKV_OK;
  if (!q_obs || !aligned16(q_obs)) return SKIPKV_EINVAL;
  if (cache->total_sentences > 0 && (!sent_score || !sent_lambda)) return SKIPKV_EINVAL;
  if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255u)) return SKIPKV_EWORKSPACE;
  VirtualView v;
  rc = make_virtual(cache, ranges, ws, &v);
  if (rc) return rc;
  const Workspace w = carve(&v.c, rl, nullptr);
  if (!w.fits) return SKIPKV_ECAPACITY;
  if (ws_bytes < v.head_bytes + w.bytes) return SKIPKV_EWORKSPACE;
  if (ranges->sent_off == new_sent_off || ranges->len == new_len || ranges->sent_cnt == new_sent_cnt) return SKIPKV_EINVAL;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (launch_virtual_layout(cache->seq_off, cache->sent_ptr, cache->batch, cache->n_layers * cache->n_kv_heads,
                            cache->total_tokens, cache->total_sentences, v.seq_off, v.sent_ptr, st) != hipSuccess)
    return SKIPKV_EHIP;
  void *ws2 = static_cast<char *>(ws) + v.head_bytes;
  Timer tm(params->profile, st);
  rc = do_score(tm, &v.c, params, rl, q_obs, tok_redundancy, sent_score, sent_lambda, tok_importance, ws2, st, v.hv);
  if (rc) return rc;
  rc = do_select(tm, &v.c, params, sent_score, sent_keep, kept_idx, new_len, new_sent_off, new_sent_cnt, kept_stride, st, v.hv);
  if (rc) return rc;
  return do_compact(tm, &v.c, kept_idx, new_len, kept_stride, st);
}

// Shared lambda (hidden-state similarity) on per-head ranges.
int skipkv_ranges_ids_select(const skipkv_cache *cache, const skipkv_ranges *ranges, int32_t protect_window,
                             const uint8_t *sent_keep, const int32_t *sent_id_in, int32_t *sent_id_out, void *stream) {
  const int rc = check_cache(cache, true);
  if (rc) return rc;
  if (is_empty(cache) || cache->total_sentences == 0) return SKIPKV_OK;
  if (!sent_keep || !sent_id_out || protect_window < 0) return SKIPKV_EINVAL;
  if (ranges && (!ranges->len || !ranges->sent_cnt || !ranges->sent_off)) return SKIPKV_EINVAL;
  RangesIdsArgs a{};
  a.n_lh = cache->n_layers * cache->n_kv_heads;
  a.batch = cache->batch;
  a.total_sentences = cache->total_sentences;
  a.protect = protect_window;
  a.seq_off = cache->seq_off;
  a.sent_ptr = cache->sent_ptr;
  a.sent_off = cache->sent_off;
  if (ranges) {
    a.len = ranges->len;
    a.old_cnt = ranges->sent_cnt;
    a.off = ranges->sent_off;
  }
  a.keep = sent_keep;
  a.id_in = sent_id_in;
  a.id_out = sent_id_out;
  return launch_ranges_ids_select(a, static_cast<hipStream_t>(stream)) == hipSuccess ? SKIPKV_OK : SKIPKV_EHIP;
}

int skipkv_ranges_ids_append(const skipkv_cache *cache, const int32_t *old_cnt, const int32_t *new_cnt, int32_t *sent_id,
                             void *stream) {
  const int rc = check_cache(cache, true);
  if (rc) return rc;
  if (is_empty(cache) || cache->total_sentences == 0) return SKIPKV_OK;
  if (!old_cnt || !new_cnt || !sent_id || old_cnt == new_cnt) return SKIPKV_EINVAL;
  RangesIdsArgs a{};
  a.n_lh = cache->n_layers * cache->n_kv_heads;
  a.batch = cache->batch;
  a.total_sentences = cache->total_sentences;
  a.seq_off = cache->seq_off;
  a.sent_ptr = cache->sent_ptr;
  a.old_cnt = old_cnt;
  a.new_cnt = new_cnt;
  a.id_out = sent_id;
  return launch_ranges_ids_append(a, static_cast<hipStream_t>(stream)) == hipSuccess ? SKIPKV_OK : SKIPKV_EHIP;
}

int skipkv_score_shared_ranges(const skipkv_cache *cache, const skipkv_ranges *ranges, const int32_t *sent_id,
                               const int32_t *lambda_ptr, const skipkv_params *params, const void *q_obs,
                               const float *tok_redundancy, const float *shared_lambda, float *sent_score,
                               float *sent_lambda, float *tok_importance, void *ws, size_t ws_bytes, void *stream) {
  RowLayout rl;
  int rc = check_cache(cache, true);
  if (rc) return rc;
  rc = check_params(cache, params, &rl);
  if (rc) return rc;
  if (is_empty(cache)) return SKIPKV_OK;
  if (!q_obs || !aligned16(q_obs)) return SKIPKV_EINVAL;
  if (cache->total_sentences > 0 && (!sent_score || !shared_lambda || !sent_id || !lambda_ptr)) return SKIPKV_EINVAL;
  if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255u)) return SKIPKV_EWORKSPACE;
  VirtualView v;
  rc = make_virtual(cache, ranges, ws, &v);
  if (rc) return rc;
  const Workspace w = carve(&v.c, rl, nullptr);
  if (!w.fits) return SKIPKV_ECAPACITY;
  if (ws_bytes < v.head_bytes + w.bytes) return SKIPKV_EWORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (launch_virtual_layout(cache->seq_off, cache->sent_ptr, cache->batch, cache->n_layers * cache->n_kv_heads,
                            cache->total_tokens, cache->total_sentences, v.seq_off, v.sent_ptr, st) != hipSuccess)
    return SKIPKV_EHIP;
  HeadView hv = v.hv;
  hv.sent_id = sent_id;
  hv.lam_ptr = lambda_ptr;
  Timer tm(params->profile, st);
  return do_score(tm, &v.c, params, rl, q_obs, tok_redundancy, sent_score, sent_lambda, tok_importance,
                  static_cast<char *>(ws) + v.head_bytes, st, hv, shared_lambda);
}

// The parts of skipkv_step_ranges, for callers that select token by token in between.
int skipkv_score_ranges(const skipkv_cache *cache, const skipkv_ranges *ranges, const skipkv_params *params,
                        const void *q_obs, const float *tok_redundancy, float *sent_score, float *sent_lambda,
                        float *tok_importance, void *ws, size_t ws_bytes, void *stream) {
  RowLayout rl;
  int rc = check_cache(cache, true);
  if (rc) return rc;
  rc = check_params(cache, params, &rl);
  if (rc) return rc;
  if (is_empty(cache)) return SKIPKV_OK;
  if (!q_obs || !aligned16(q_obs)) return SKIPKV_EINVAL;
  if (cache->total_sentences > 0 && (!sent_score || !sent_lambda)) return SKIPKV_EINVAL;
  if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255u)) return SKIPKV_EWORKSPACE;
  VirtualView v;
  rc = make_virtual(cache, ranges, ws, &v);
  if (rc) return rc;
  const Workspace w = carve(&v.c, rl, nullptr);
  if (!w.fits) return SKIPKV_ECAPACITY;
  if (ws_bytes < v.head_bytes + w.bytes) return SKIPKV_EWORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (launch_virtual_layout(cache->seq_off, cache->sent_ptr, cache->batch, cache->n_layers * cache->n_kv_heads,
                            cache->total_tokens, cache->total_sentences, v.seq_off, v.sent_ptr, st) != hipSuccess)
    return SKIPKV_EHIP;
  Timer tm(params->profile, st);
  return do_score(tm, &v.c, params, rl, q_obs, tok_redundancy, sent_score, sent_lambda, tok_importance,
                  static_cast<char *>(ws) + v.head_bytes, st, v.hv);
}

int skipkv_select_ranges(const skipkv_cache *cache, const skipkv_ranges *ranges, const skipkv_params *params,
                         const float *sent_score, uint8_t *sent_keep, int32_t *kept_idx, int32_t *new_len,
                         int32_t *new_sent_off, int32_t *new_sent_cnt, int32_t kept_stride, void *ws, size_t ws_bytes,
                         void *stream) {
  RowLayout rl;
  int rc = check_select_args(cache, params, &rl, sent_score, kept_idx, new_len, new_sent_off, new_sent_cnt, kept_stride);
  if (rc) return rc;
  if (is_empty(cache)) return SKIPKV_OK;
  if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255u)) return SKIPKV_EWORKSPACE;
  VirtualView v;
  rc = make_virtual(cache, ranges, ws, &v, true);  // K and V are not read: any strides
  if (rc) return rc;
  if (ws_bytes < v.head_bytes) return SKIPKV_EWORKSPACE;
  if (ranges->sent_off == new_sent_off || ranges->len == new_len || ranges->sent_cnt == new_sent_cnt) return SKIPKV_EINVAL;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (launch_virtual_layout(cache->seq_off, cache->sent_ptr, cache->batch, cache->n_layers * cache->n_kv_heads,
                            cache->total_tokens, cache->total_sentences, v.seq_off, v.sent_ptr, st) != hipSuccess)
    return SKIPKV_EHIP;
  Timer tm(params->profile, st);
  return do_select(tm, &v.c, params, sent_score, sent_keep, kept_idx, new_len, new_sent_off, new_sent_cnt, kept_stride, st, v.hv);
}

int skipkv_select_tokens_ranges(const skipkv_cache *cache, const skipkv_ranges *ranges, const skipkv_params *params,
                                const float *tok_importance, const float *tok_redundancy, const float *sent_lambda,
                                float *tok_score, uint8_t *tok_keep, int32_t *kept_idx, int32_t *new_len,
                                int32_t *new_sent_off, int32_t *new_sent_cnt, int32_t kept_stride, void *ws,
                                size_t ws_bytes, void *stream) {
  RowLayout rl;
  int rc = check_select_args(cache, params, &rl, sent_lambda, kept_idx, new_len, new_sent_off, new_sent_cnt, kept_stride);
  if (rc) return rc;
  if (is_empty(cache)) return SKIPKV_OK;
  if (cache->total_tokens > 0 && (!tok_importance || !tok_score)) return SKIPKV_EINVAL;
  if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255u)) return SKIPKV_EWORKSPACE;
  VirtualView v;
  rc = make_virtual(cache, ranges, ws, &v, true);  // K and V are not read: any strides
  if (rc) return rc;
  if (ws_bytes < v.head_bytes) return SKIPKV_EWORKSPACE;
  if (ranges->sent_off == new_sent_off || ranges->len == new_len || ranges->sent_cnt == new_sent_cnt) return SKIPKV_EINVAL;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (launch_virtual_layout(cache->seq_off, cache->sent_ptr, cache->batch, cache->n_layers * cache->n_kv_heads,
                            cache->total_tokens, cache->total_sentences, v.seq_off, v.sent_ptr, st) != hipSuccess)
    return SKIPKV_EHIP;
  return do_select_tokens(&v.c, params, tok_importance, tok_redundancy, sent_lambda, tok_score, tok_keep, kept_idx, new_len,
                          new_sent_off, new_sent_cnt, kept_stride, st, v.hv);
}

int skipkv_token_redundancy_ranges(const skipkv_cache *cache, const skipkv_ranges *ranges, float *tok_redundancy, void *ws,
                                   size_t ws_bytes, void *stream) {
  const int rc = check_cache(cache, false);
  if (rc) return rc;
  if (is_empty(cache) || cache->total_tokens == 0) return SKIPKV_OK;
  if (!tok_redundancy || !ranges || !ranges->len) return SKIPKV_EINVAL;
  if (!ws || !aligned16(ws) || ws_bytes < tokred_bytes(cache)) return SKIPKV_EWORKSPACE;
  TokRedArgs a = tokred_args(cache, ws, tok_redundancy);
  a.len = ranges->len;
  return launch_token_redundancy(a, static_cast<hipStream_t>(stream)) == hipSuccess ? SKIPKV_OK : SKIPKV_EHIP;
}

namespace {
// Per-head ranges on a paged cache.  The virtual cache of make_virtual has one layer and one head,
// so the (layer, head) part of an address moves into the row map: every (layer, head) gets a map
// of its own whose unit is one head row (head_dim elements), which every stride must be a
// multiple of.  Behind the virtual layout and the step's workspace sit these maps, the
// per-(head, sequence) flags and the slot rows of the kept tokens.
struct RangesPagedView {
  VirtualView v;
  size_t step_bytes, map_bytes, bad_bytes, total;
  int32_t src_stride;
  int64_t unit_layer, unit_head, unit_block, unit_tok;
};
int check_ranges_paging(const skipkv_cache *c, const skipkv_ranges *r, const skipkv_paging *pg, const skipkv_params *p,
                        const RowLayout &rl, void *ws, RangesPagedView *o) {
  int64_t rpb = 0;
  int rc = check_paging_desc(c, pg, &rpb);
  if (rc) return rc;
  const int64_t D = c->head_dim;
  if ((c->stride_tok % D) || (c->stride_head % D) || (c->stride_layer % D) || (pg->stride_block % D)) return SKIPKV_EINVAL;
  o->unit_layer = c->stride_layer / D;
  o->unit_head = c->stride_head / D;
  o->unit_block = pg->stride_block / D;
  o->unit_tok = c->stride_tok / D;
  const int64_t last_row = (int64_t)(c->n_layers - 1) * o->unit_layer + (int64_t)(c->n_kv_heads - 1) * o->unit_head +
                           (int64_t)(pg->n_blocks - 1) * o->unit_block + (int64_t)(pg->block_size - 1) * o->unit_tok;
  if (last_row > 0x7FFFFFFFll) return SKIPKV_ECAPACITY;  // slot rows are 32-bit
  rc = make_virtual(c, r, ws, &o->v, true);
  if (rc) return rc;
  const Workspace w = carve(&o->v.c, rl, nullptr);
  if (!w.fits) return SKIPKV_ECAPACITY;
  const size_t LH = (size_t)c->n_layers * c->n_kv_heads;
  o->step_bytes = align_up(w.bytes);
  o->map_bytes = align_up(LH * c->total_tokens * 4);
  o->bad_bytes = align_up(LH * c->batch * 4);
  o->src_stride = std::max(1, std::min(p->max_budget, c->total_tokens));
  o->total = o->v.head_bytes + o->step_bytes + o->map_bytes + o->bad_bytes + align_up(LH * c->batch * o->src_stride * 4);
  return SKIPKV_OK;
}
}  // namespace

int skipkv_ranges_paged_workspace_bytes(const skipkv_cache *cache, const skipkv_paging *paging,
                                        const skipkv_params *params, size_t *out_bytes) {
  if (!out_bytes) return SKIPKV_EINVAL;
  int rc = check_cache(cache, true);
  if (rc) return rc;
  RowLayout rl;
  rc = check_params(cache, params, &rl);
  if (rc) return rc;
  if (is_empty(cache)) {
    *out_bytes = 0;
    return SKIPKV_OK;
  }
  skipkv_ranges dummy{reinterpret_cast<int32_t *>(16), reinterpret_cast<int32_t *>(16), reinterpret_cast<int32_t *>(16)};
  RangesPagedView pv;
  rc = check_ranges_paging(cache, &dummy, paging, params, rl, nullptr, &pv);
  if (rc) return rc;
  *out_bytes = pv.total;
  return SKIPKV_OK;
}

namespace {
// Scoring half of the per-head step on pages; leaves the row maps, flags and the view behind for the caller.
int score_ranges_paged(const skipkv_cache *cache, const skipkv_ranges *ranges, const skipkv_paging *paging,
                       const skipkv_params *params, const RowLayout &rl, const void *q_obs, const float *tok_redundancy,
                       const float *shared_lambda, const int32_t *sent_id, const int32_t *lambda_ptr, float *sent_score,
                       float *sent_lambda, float *tok_importance, void *ws, size_t ws_bytes, hipStream_t st, Timer &tm,
                       RangesPagedView *pv, HeadView *hv_out) {
  if (!q_obs || !aligned16(q_obs)) return SKIPKV_EINVAL;
  if (cache->total_sentences > 0 && (!sent_score || (!shared_lambda && !sent_lambda))) return SKIPKV_EINVAL;
  if (shared_lambda && cache->total_sentences > 0 && (!sent_id || !lambda_ptr)) return SKIPKV_EINVAL;
  if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255u)) return SKIPKV_EWORKSPACE;
  int rc = check_ranges_paging(cache, ranges, paging, params, rl, ws, pv);
  if (rc) return rc;
  if (ws_bytes < pv->total) return SKIPKV_EWORKSPACE;
  const VirtualView &v = pv->v;
  const int32_t n_lh = cache->n_layers * cache->n_kv_heads;
  if (launch_virtual_layout(cache->seq_off, cache->sent_ptr, cache->batch, n_lh, cache->total_tokens,
                            cache->total_sentences, v.seq_off, v.sent_ptr, st) != hipSuccess)
    return SKIPKV_EHIP;
  char *ws2 = static_cast<char *>(ws) + v.head_bytes;
  int32_t *row_map = reinterpret_cast<int32_t *>(ws2 + pv->step_bytes);
  int32_t *seq_bad = reinterpret_cast<int32_t *>(ws2 + pv->step_bytes + pv->map_bytes);
  RowMapArgs ra{cache->seq_off, paging->block_table, cache->batch, paging->table_stride, paging->block_size,
                paging->n_blocks, n_lh, cache->n_kv_heads, cache->total_tokens, pv->unit_layer, pv->unit_head,
                pv->unit_block, pv->unit_tok, row_map, seq_bad, params->dev_status};
  if (tm.run("row_map", [&] { return launch_row_map(ra, st); }) != hipSuccess) return SKIPKV_EHIP;
  HeadView hv = v.hv;
  hv.row_map = row_map;
  hv.page_size = paging->block_size;
  hv.map_stride = cache->head_dim;
  hv.sent_id = shared_lambda ? sent_id : nullptr;
  hv.lam_ptr = shared_lambda ? lambda_ptr : nullptr;
  *hv_out = hv;
  return do_score(tm, &v.c, params, rl, q_obs, tok_redundancy, sent_score, sent_lambda, tok_importance, ws2, st, hv, shared_lambda);
}
}  // namespace

int skipkv_score_ranges_paged(const skipkv_cache *cache, const skipkv_ranges *ranges, const skipkv_paging *paging,
                              const int32_t *sent_id, const int32_t *lambda_ptr, const float *shared_lambda,
                              const skipkv_params *params, const void *q_obs, const float *tok_redundancy,
                              float *sent_score, float *sent_lambda, float *tok_importance, void *ws, size_t ws_bytes,
                              void *stream) {
  RowLayout rl;
  int rc = check_cache(cache, true);
  if (rc) return rc;
  rc = check_params(cache, params, &rl);
  if (rc) return rc;
  if (is_empty(cache)) return SKIPKV_OK;
  hipStream_t st = static_cast<hipStream_t>(stream);
  Timer tm(params->profile, st);
  RangesPagedView pv;
  HeadView hv;
  return score_ranges_paged(cache, ranges, paging, params, rl, q_obs, tok_redundancy, shared_lambda, sent_id, lambda_ptr,
                            sent_score, sent_lambda, tok_importance, ws, ws_bytes, st, tm, &pv, &hv);
}

int skipkv_step_ranges_paged(const skipkv_cache *cache, const skipkv_ranges *ranges, const skipkv_paging *paging,
                             const skipkv_params *params, const void *q_obs, const float *tok_redundancy,
                             float *sent_score, float *sent_lambda, float *tok_importance, uint8_t *sent_keep,
                             int32_t *kept_idx, int32_t *new_len, int32_t *new_sent_off, int32_t *new_sent_cnt,
                             int32_t kept_stride, void *ws, size_t ws_bytes, void *stream) {
  RowLayout rl;
  int rc = check_cache(cache, true);
  if (rc) return rc;
  rc = check_params(cache, params, &rl);
  if (rc) return rc;
  rc = check_select_args(cache, params, &rl, sent_score, kept_idx, new_len, new_sent_off, new_sent_cnt, kept_stride);
  if (rc) return rc;
  if (is_empty(cache)) return SKIPKV_OK;
  if (ranges && (ranges->sent_off == new_sent_off || ranges->len == new_len || ranges->sent_cnt == new_sent_cnt)) return SKIPKV_EINVAL;
  hipStream_t st = static_cast<hipStream_t>(stream);
  Timer tm(params->profile, st);
  RangesPagedView pv;
  HeadView hv;
  rc = score_ranges_paged(cache, ranges, paging, params, rl, q_obs, tok_redundancy, nullptr, nullptr, nullptr, sent_score,
                          sent_lambda, tok_importance, ws, ws_bytes, st, tm, &pv, &hv);
  if (rc) return rc;
  const VirtualView &v = pv.v;
  rc = do_select(tm, &v.c, params, sent_score, sent_keep, kept_idx, new_len, new_sent_off, new_sent_cnt, kept_stride, st, hv);
  if (rc) return rc;
  char *ws2 = static_cast<char *>(ws) + v.head_bytes;
  int32_t *seq_bad = reinterpret_cast<int32_t *>(ws2 + pv.step_bytes + pv.map_bytes);
  int32_t *src_rows = reinterpret_cast<int32_t *>(ws2 + pv.step_bytes + pv.map_bytes + pv.bad_bytes);
  return do_compact(tm, &v.c, kept_idx, new_len, kept_stride, st, hv.row_map, seq_bad, src_rows, pv.src_stride, cache->head_dim);
}

int skipkv_ranges_append(const skipkv_cache *cache, const skipkv_ranges *ranges, const int32_t *n_new,
                         const int32_t *bnd_ptr, const int32_t *bnd_off, int32_t *dev_status, void *stream) {
  const int rc = check_cache(cache, true);
  if (rc) return rc;
  if (is_empty(cache)) return SKIPKV_OK;
  if (!ranges || !ranges->len || !ranges->sent_cnt || !ranges->sent_off || !n_new || !bnd_ptr) return SKIPKV_EINVAL;
  RangesAppendArgs a{};
  a.n_lh = cache->n_layers * cache->n_kv_heads;
  a.batch = cache->batch;
  a.total_sentences = cache->total_sentences;
  a.seq_off = cache->seq_off;
  a.sent_ptr = cache->sent_ptr;
  a.len = ranges->len;
  a.cnt = ranges->sent_cnt;
  a.off = ranges->sent_off;
  a.n_new = n_new;
  a.bnd_ptr = bnd_ptr;
  a.bnd_off = bnd_off;
  a.dev_status = dev_status;
  return launch_ranges_append(a, static_cast<hipStream_t>(stream)) == hipSuccess ? SKIPKV_OK : SKIPKV_EHIP;
}

int skipkv_similarity_workspace_bytes(const skipkv_cache *cache, int32_t d_model, size_t *out_bytes) {
  if (!out_bytes || d_model <= 0 || d_model % 128) return SKIPKV_EINVAL;
  const int rc = check_cache(cache, true);
  if (rc) return rc;
  const size_t n = (size_t)cache->total_sentences * (size_t)d_model;
  *out_bytes = align_up(n * 4) + 2 * align_up(n * 2);
  return SKIPKV_OK;
}

int skipkv_sentence_similarity(const skipkv_cache *cache, const void *hidden, int32_t d_model, int32_t dtype,
                               float *shared_lambda, void *ws, size_t ws_bytes, void *stream) {
  if (d_model <= 0 || d_model % 128) return SKIPKV_EINVAL;
  if (dtype != SKIPKV_F32 && dtype != SKIPKV_BF16) return SKIPKV_EINVAL;
  const int rc = check_cache(cache, true);
  if (rc) return rc;
  if (cache->batch == 0 || cache->total_sentences == 0) return SKIPKV_OK;
  if (!hidden || !aligned16(hidden) || !shared_lambda) return SKIPKV_EINVAL;
  const size_t n = (size_t)cache->total_sentences * (size_t)d_model;
  if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255u) || ws_bytes < align_up(n * 4) + 2 * align_up(n * 2)) return SKIPKV_EWORKSPACE;
  HiddenSimArgs a{};
  a.batch = cache->batch;
  a.total_sentences = cache->total_sentences;
  a.d_model = d_model;
  a.dtype = dtype;
  a.seq_off = cache->seq_off;
  a.sent_ptr = cache->sent_ptr;
  a.sent_off = cache->sent_off;
  a.hidden = hidden;
  char *p = static_cast<char *>(ws);
  a.sum_scratch = reinterpret_cast<float *>(p);
  a.vhat_hi = reinterpret_cast<uint16_t *>(p + align_up(n * 4));
  a.vhat_lo = reinterpret_cast<uint16_t *>(p + align_up(n * 4) + align_up(n * 2));
  a.sent_lambda = shared_lambda;
  return launch_hidden_similarity(a, static_cast<hipStream_t>(stream)) == hipSuccess ? SKIPKV_OK : SKIPKV_EHIP;
}

int skipkv_score_shared(const skipkv_cache *cache, const skipkv_params *params, const void *q_obs,
                        const float *tok_redundancy, const float *shared_lambda, float *sent_score, float *sent_lambda,
                        float *tok_importance, void *ws, size_t ws_bytes, void *stream) {
  RowLayout rl;
  float dummy = 0.f;
  const int rc = check_score_args(cache, params, &rl, q_obs, sent_score, sent_lambda ? sent_lambda : &dummy, ws, ws_bytes);
  if (rc) return rc;
  if (is_empty(cache)) return SKIPKV_OK;
  if (cache->total_sentences > 0 && !shared_lambda) return SKIPKV_EINVAL;
  Timer tm(params->profile, static_cast<hipStream_t>(stream));
  return do_score(tm, cache, params, rl, q_obs, tok_redundancy, sent_score, sent_lambda, tok_importance, ws,
                  static_cast<hipStream_t>(stream), HeadView(), shared_lambda);
}

int skipkv_redundancy_workspace_bytes(const skipkv_cache *cache, size_t *out_bytes) {
  if (!out_bytes) return SKIPKV_EINVAL;
  const int rc = check_cache(cache, false);
  if (rc) return rc;
  *out_bytes = tokred_bytes(cache);
  return SKIPKV_OK;
}

int skipkv_token_redundancy(const skipkv_cache *cache, float *tok_redundancy, void *ws, size_t ws_bytes, void *stream) {
  const int rc = check_cache(cache, false);
  if (rc) return rc;
  if (is_empty(cache) || cache->total_tokens == 0) return SKIPKV_OK;
  if (!tok_redundancy) return SKIPKV_EINVAL;
  if (!ws || !aligned16(ws) || ws_bytes < tokred_bytes(cache)) return SKIPKV_EWORKSPACE;
  TokRedArgs a = tokred_args(cache, ws, tok_redundancy);
  return launch_token_redundancy(a, static_cast<hipStream_t>(stream)) == hipSuccess ? SKIPKV_OK : SKIPKV_EHIP;
}

int skipkv_redundancy_paged_workspace_bytes(const skipkv_cache *cache, const skipkv_paging *paging, size_t *out_bytes) {
  if (!out_bytes) return SKIPKV_EINVAL;
  int rc = check_cache(cache, false);
  if (rc) return rc;
  if (is_empty(cache)) {
    *out_bytes = 0;
    return SKIPKV_OK;
  }
  CompactPagedView v;
  rc = check_compact_paging(cache, paging, 0, &v);
  if (rc) return rc;
  *out_bytes = tokred_bytes(cache) + v.map_bytes + v.bad_bytes;
  return SKIPKV_OK;
}

namespace {
int token_redundancy_paged(const skipkv_cache *cache, const int32_t *len, const skipkv_paging *paging, float *tok_redundancy,
                           int32_t *dev_status, void *ws, size_t ws_bytes, void *stream);
}

int skipkv_token_redundancy_paged(const skipkv_cache *cache, const skipkv_paging *paging, float *tok_redundancy,
                                  int32_t *dev_status, void *ws, size_t ws_bytes, void *stream) {
  return token_redundancy_paged(cache, nullptr, paging, tok_redundancy, dev_status, ws, ws_bytes, stream);
}

int skipkv_token_redundancy_ranges_paged(const skipkv_cache *cache, const skipkv_ranges *ranges, const skipkv_paging *paging,
                                         float *tok_redundancy, int32_t *dev_status, void *ws, size_t ws_bytes,
                                         void *stream) {
  if (!ranges || !ranges->len) return SKIPKV_EINVAL;
  return token_redundancy_paged(cache, ranges->len, paging, tok_redundancy, dev_status, ws, ws_bytes, stream);
}

namespace {
int token_redundancy_paged(const skipkv_cache *cache, const int32_t *len, const skipkv_paging *paging, float *tok_redundancy,
                           int32_t *dev_status, void *ws, size_t ws_bytes, void *stream) {
  int rc = check_cache(cache, false);
  if (rc) return rc;
  if (is_empty(cache) || cache->total_tokens == 0) return SKIPKV_OK;
  if (!tok_redundancy) return SKIPKV_EINVAL;
  CompactPagedView v;
  rc = check_compact_paging(cache, paging, 0, &v);
  if (rc) return rc;
  const size_t red_bytes = tokred_bytes(cache);
  if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255u) || ws_bytes < red_bytes + v.map_bytes + v.bad_bytes) return SKIPKV_EWORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  int32_t *row_map = reinterpret_cast<int32_t *>(static_cast<char *>(ws) + red_bytes);
  int32_t *seq_bad = reinterpret_cast<int32_t *>(static_cast<char *>(ws) + red_bytes + v.map_bytes);
  RowMapArgs ra{cache->seq_off, paging->block_table, cache->batch, paging->table_stride, paging->block_size,
                paging->n_blocks, 1, 1, cache->total_tokens, 0, 0, v.rows_per_block, 1, row_map, seq_bad, dev_status};
  if (launch_row_map(ra, st) != hipSuccess) return SKIPKV_EHIP;
  TokRedArgs a = tokred_args(cache, ws, tok_redundancy);
  a.row_map = row_map;
  a.len = len;
  return launch_token_redundancy(a, st) == hipSuccess ? SKIPKV_OK : SKIPKV_EHIP;
}
}  // namespace

int skipkv_steer_add(void *hidden, const void *vec, const float *coef, float coef_scalar, const uint8_t *row_mask,
                     int32_t rows, int32_t d_model, int32_t dtype, void *stream) {
  if (rows < 0 || d_model < 0) return SKIPKV_EINVAL;
  if (dtype != SKIPKV_F32 && dtype != SKIPKV_BF16) return SKIPKV_EINVAL;
  if (rows == 0 || d_model == 0) return SKIPKV_OK;
  if (!hidden || !vec) return SKIPKV_EINVAL;
  if (rows > 65535) return SKIPKV_ECAPACITY;
  SteerArgs a{hidden, vec, coef, coef_scalar, row_mask, rows, d_model, dtype};
  return launch_steer(a, static_cast<hipStream_t>(stream)) == hipSuccess ? SKIPKV_OK : SKIPKV_EHIP;
}

int skipkv_steer_strength(const int32_t *n_nonexec, float alpha0, float gamma, float *coef, int32_t rows, void *stream) {
  if (rows < 0) return SKIPKV_EINVAL;
  if (rows == 0) return SKIPKV_OK;
  if (!n_nonexec || !coef) return SKIPKV_EINVAL;
  return launch_steer_strength(n_nonexec, alpha0, gamma, coef, rows, static_cast<hipStream_t>(stream)) == hipSuccess ? SKIPKV_OK : SKIPKV_EHIP;
}

int skipkv_profile_create(void **out_profile) {
  if (!out_profile) return SKIPKV_EINVAL;
  Profile *p = new (std::nothrow) Profile();
  if (!p) return SKIPKV_EINVAL;
  p->n = 0;
  for (int i = 0; i < 2 * SKIPKV_PROFILE_SLOTS; ++i) {
    if (hipEventCreate(&p->ev[i]) != hipSuccess) {
      for (int j = 0; j < i; ++j) (void)hipEventDestroy(p->ev[j]);
      delete p;
      return SKIPKV_EHIP;
    }
  }
  *out_profile = p;
  return SKIPKV_OK;
}

int skipkv_profile_read(void *profile, int32_t *n, const char **names, float *ms) {
  if (!profile || !n) return SKIPKV_EINVAL;
  Profile *p = static_cast<Profile *>(profile);
  *n = p->n;
  for (int i = 0; i < p->n; ++i) {
    if (hipEventSynchronize(p->ev[2 * i + 1]) != hipSuccess) return SKIPKV_EHIP;
    float t = 0.f;
    if (hipEventElapsedTime(&t, p->ev[2 * i], p->ev[2 * i + 1]) != hipSuccess) return SKIPKV_EHIP;
    if (names) names[i] = p->name[i];
    if (ms) ms[i] = t;
  }
  return SKIPKV_OK;
}

int skipkv_profile_destroy(void *profile) {
  if (!profile) return SKIPKV_EINVAL;
  Profile *p = static_cast<Profile *>(profile);
  for (int i = 0; i < 2 * SKIPKV_PROFILE_SLOTS; ++i) (void)hipEventDestroy(p->ev[i]);
  delete p;
  return SKIPKV_OK;
}

const char *skipkv_strerror(int status) {
  switch (status) {
    case SKIPKV_OK: return "ok";
    case SKIPKV_EINVAL: return "invalid argument (null pointer, shape, stride, alignment or dtype)";
    case SKIPKV_EBUDGET: return "budget smaller than the protected window, or observation window larger than the protected window";
    case SKIPKV_ECAPACITY: return "shape outside the limits this build supports";
    case SKIPKV_EWORKSPACE: return "workspace missing, misaligned or too small (skipkv_step_static: the problem needs more than SKIPKV_STATIC_WS_BYTES)";
    case SKIPKV_EHIP: return "HIP runtime error";
    default: return "unknown status";
  }
}

int skipkv_version(void) { return SKIPKV_VERSION; }

}  // extern "C"
