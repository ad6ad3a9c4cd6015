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
  w.head_redo = static_cast<int32_t *>(take(LH * B * 4));
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

// ---------------------------------------------------------------------------------------------------
// One call through the scoring / selection / compaction path, as the caller described it.  Every exported
// score, select and step entry point (shared or per-head ranges, contiguous or paged cache, per-head or
// shared lambda, sentence- or token-level selection) fills one of these and hands it to run_call, and every
// size query goes through resolve: nothing else validates these arguments, lays out this workspace or
// sequences these kernels.
enum : unsigned { kScore = 1u, kSelect = 2u, kSelectTokens = 4u, kCompact = 8u };

struct Call {
  unsigned stages = 0;
  const skipkv_cache *cache = nullptr;
  const skipkv_params *params = nullptr;
  bool per_head = false;                    // the entry point works on per-head ranges (`ranges` is then required)
  const skipkv_ranges *ranges = nullptr;
  bool paged = false;                       // ... on a paged cache (`paging` is then required)
  const skipkv_paging *paging = nullptr;
  // scoring
  const void *q_obs = nullptr;
  const float *tok_red = nullptr;
  bool shared = false;                      // lambda is the caller's (hidden-state similarity), not computed per head
  const float *shared_lambda = nullptr;
  const int32_t *sent_id = nullptr, *lam_ptr = nullptr;  // ... looked up by sentence number under per-head ranges
  float *sent_score = nullptr, *sent_lambda = nullptr, *tok_imp = nullptr;
  // selection (sentence level: by sent_score; token level: from tok_imp_in, tok_red and lambda_in)
  const float *tok_imp_in = nullptr, *lambda_in = nullptr;
  float *tok_score = nullptr;
  uint8_t *keep = nullptr;                  // sent_keep, or tok_keep at token level
  int32_t *kept_idx = nullptr, *new_len = nullptr, *new_sent_off = nullptr, *new_sent_cnt = nullptr;
  int32_t kept_stride = 0;
  void *ws = nullptr;
  size_t ws_bytes = 0;
  void *stream = nullptr;
};

// What resolve makes of a call: the cache as the kernels see it (the virtual one under per-head ranges) and
// where the pieces of the workspace are: [virtual layout | step | row maps | per-sequence flags | slot rows].
struct Layout {
  bool empty = false;
  RowLayout rl;
  skipkv_cache c;
  HeadView hv;
  int32_t *v_seq_off = nullptr, *v_sent_ptr = nullptr;
  size_t head_bytes = 0, step_bytes = 0, map_bytes = 0, bad_bytes = 0, src_bytes = 0, total = 0;
  int32_t src_stride = 0;
  int64_t unit_layer = 0, unit_head = 0, unit_block = 0, unit_tok = 1;  // row-map units (per-head ranges: head rows)
};

// Validation of a paged cache's description.
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

// Checks every argument of the call on the host and computes the layout.  With `sizing` only the sizes are
// wanted (no workspace, no per-call pointers are looked at).
int resolve(const Call &k, bool sizing, Layout *o) {
  const skipkv_cache *c = k.cache;
  const skipkv_params *p = k.params;
  Layout L;
  int rc = check_cache(c, true);
  if (rc) return rc;
  rc = check_params(c, p, &L.rl);
  if (rc) return rc;
  const bool selects = (k.stages & (kSelect | kSelectTokens)) != 0;
  if (selects && !sizing && !is_empty(c)) {
    const float *ranked = (k.stages & kSelect) ? k.sent_score : k.lambda_in;
    if (!k.new_len || (c->total_sentences > 0 && !ranked)) return SKIPKV_EINVAL;
    if ((k.new_sent_off == nullptr) != (k.new_sent_cnt == nullptr)) return SKIPKV_EINVAL;
    const int32_t need = p->max_budget < c->total_tokens ? p->max_budget : c->total_tokens;
    if (k.kept_stride < need || (need > 0 && !k.kept_idx)) return SKIPKV_EINVAL;
  }
  L.c = *c;
  if (is_empty(c)) {
    L.empty = true;
    if (!k.per_head && !k.paged && (k.stages & kScore)) L.total = carve(c, L.rl, nullptr).bytes;
    *o = L;
    return SKIPKV_OK;
  }
  if ((k.stages & kScore) && !sizing) {
    if (!k.q_obs || !aligned16(k.q_obs)) return SKIPKV_EINVAL;
    if (c->total_sentences > 0 && (!k.sent_score || (!k.shared && !k.sent_lambda))) return SKIPKV_EINVAL;
    if (k.shared && c->total_sentences > 0 && (!k.shared_lambda || (k.per_head && (!k.sent_id || !k.lam_ptr)))) return SKIPKV_EINVAL;
  }
  if ((k.stages & kSelectTokens) && !sizing && c->total_tokens > 0 && (!k.tok_imp_in || !k.tok_score)) return SKIPKV_EINVAL;
  if (!sizing && (k.per_head || k.paged || (k.stages & kScore)) && (!k.ws || (reinterpret_cast<uintptr_t>(k.ws) & 255u)))
    return SKIPKV_EWORKSPACE;

  int64_t rpb = 0;
  if (k.paged) {
    rc = check_paging_desc(c, k.paging, &rpb);
    if (rc) return rc;
  }
  if (k.per_head) {
    // K and V are addressed by the kernels as one flat array of rows unless they are not read at all
    // (selection only) or a row map says where the rows are
    const bool any_strides = k.paged || !(k.stages & (kScore | kCompact));
    const skipkv_ranges sizing_ranges{reinterpret_cast<int32_t *>(16), reinterpret_cast<int32_t *>(16), reinterpret_cast<int32_t *>(16)};
    VirtualView v;
    if (k.paged) {  // the (layer, head) part of an address moves into the row maps, whose unit is one head row
      const int64_t D = c->head_dim;
      if ((c->stride_tok % D) || (c->stride_head % D) || (c->stride_layer % D) || (k.paging->stride_block % D)) return SKIPKV_EINVAL;
      L.unit_layer = c->stride_layer / D;
      L.unit_head = c->stride_head / D;
      L.unit_block = k.paging->stride_block / D;
      L.unit_tok = c->stride_tok / D;
      const int64_t last_row = (int64_t)(c->n_layers - 1) * L.unit_layer + (int64_t)(c->n_kv_heads - 1) * L.unit_head +
                               (int64_t)(k.paging->n_blocks - 1) * L.unit_block + (int64_t)(k.paging->block_size - 1) * L.unit_tok;
      if (last_row > 0x7FFFFFFFll) return SKIPKV_ECAPACITY;  // slot rows are 32-bit
    }
    rc = make_virtual(c, sizing ? &sizing_ranges : k.ranges, sizing ? nullptr : k.ws, &v, any_strides);
    if (rc) return rc;
    if (selects && !sizing &&
        (k.ranges->sent_off == k.new_sent_off || k.ranges->len == k.new_len || k.ranges->sent_cnt == k.new_sent_cnt))
      return SKIPKV_EINVAL;  // outputs must not alias the input ranges
    L.c = v.c;
    L.hv = v.hv;
    L.v_seq_off = v.seq_off;
    L.v_sent_ptr = v.sent_ptr;
    L.head_bytes = v.head_bytes;
    if (k.shared) {
      L.hv.sent_id = k.sent_id;
      L.hv.lam_ptr = k.lam_ptr;
    }
  } else if (k.paged) {
    if ((int64_t)k.paging->n_blocks * rpb > 0x7FFFFFFFll) return SKIPKV_ECAPACITY;  // slot rows are 32-bit
    L.unit_block = rpb;  // the shared map counts in token rows
  }
  if (k.stages & kScore) {
    const Workspace w = carve(&L.c, L.rl, nullptr);
    if (!w.fits) return SKIPKV_ECAPACITY;
    L.step_bytes = align_up(w.bytes);
  }
  if (k.paged) {
    const size_t LH = (size_t)c->n_layers * c->n_kv_heads;
    L.map_bytes = align_up((k.per_head ? LH : 1) * (size_t)c->total_tokens * 4);
    L.bad_bytes = align_up((k.per_head ? LH : 1) * (size_t)c->batch * 4);
    // slot rows of the kept tokens of every head: no head keeps more than its budget, nor more than there is
    L.src_stride = std::max(1, std::min(p->max_budget, c->total_tokens));
    L.src_bytes = align_up(LH * c->batch * L.src_stride * 4);
    L.hv.page_size = k.paging->block_size;
    L.hv.map_stride = k.per_head ? c->head_dim : 0;
  }
  L.total = L.head_bytes + L.step_bytes + L.map_bytes + L.bad_bytes + L.src_bytes;
  if (!sizing && L.total > 0 && k.ws_bytes < L.total) return SKIPKV_EWORKSPACE;
  *o = L;
  return SKIPKV_OK;
}

int size_call(const Call &k, size_t *out_bytes) {
  if (!out_bytes) return SKIPKV_EINVAL;
  Layout L;
  const int rc = resolve(k, true, &L);
  if (rc) return rc;
  *out_bytes = L.total;
  return SKIPKV_OK;
}

int run_call(const Call &k) {
  Layout L;
  int rc = resolve(k, false, &L);
  if (rc || L.empty) return rc;
  const skipkv_cache *c = k.cache;
  const skipkv_params *p = k.params;
  hipStream_t st = static_cast<hipStream_t>(k.stream);
  Timer tm(p->profile, st);
  char *ws = static_cast<char *>(k.ws);
  const int32_t n_lh = c->n_layers * c->n_kv_heads;
  if (k.per_head &&
      launch_virtual_layout(c->seq_off, c->sent_ptr, c->batch, n_lh, c->total_tokens, c->total_sentences, L.v_seq_off,
                            L.v_sent_ptr, st) != hipSuccess)
    return SKIPKV_EHIP;
  char *step_ws = ws + L.head_bytes;
  int32_t *row_map = nullptr, *seq_bad = nullptr, *src_rows = nullptr;
  if (k.paged) {
    row_map = reinterpret_cast<int32_t *>(step_ws + L.step_bytes);
    seq_bad = reinterpret_cast<int32_t *>(step_ws + L.step_bytes + L.map_bytes);
    src_rows = reinterpret_cast<int32_t *>(step_ws + L.step_bytes + L.map_bytes + L.bad_bytes);
    const skipkv_paging *pg = k.paging;
    RowMapArgs ra{c->seq_off, pg->block_table, c->batch, pg->table_stride, pg->block_size, pg->n_blocks,
                  k.per_head ? n_lh : 1, k.per_head ? c->n_kv_heads : 1, c->total_tokens, L.unit_layer, L.unit_head,
                  L.unit_block, L.unit_tok, row_map, seq_bad, p->dev_status};
    if (tm.run("row_map", [&] { return launch_row_map(ra, st); }) != hipSuccess) return SKIPKV_EHIP;
    L.hv.row_map = row_map;
  }
  if (k.stages & kScore) {
    rc = do_score(tm, &L.c, p, L.rl, k.q_obs, k.tok_red, k.sent_score, k.sent_lambda, k.tok_imp, step_ws, st, L.hv,
                  k.shared ? k.shared_lambda : nullptr);
    if (rc) return rc;
  }
  if (k.stages & kSelect) {
    rc = do_select(tm, &L.c, p, k.sent_score, k.keep, k.kept_idx, k.new_len, k.new_sent_off, k.new_sent_cnt, k.kept_stride, st, L.hv);
    if (rc) return rc;
  }
  if (k.stages & kSelectTokens) {
    rc = do_select_tokens(&L.c, p, k.tok_imp_in, k.tok_red, k.lambda_in, k.tok_score, k.keep, k.kept_idx, k.new_len,
                          k.new_sent_off, k.new_sent_cnt, k.kept_stride, st, L.hv);
    if (rc) return rc;
  }
  if (k.stages & kCompact) {
    rc = do_compact(tm, &L.c, k.kept_idx, k.new_len, k.kept_stride, st, row_map, seq_bad, src_rows, L.src_stride,
                    k.paged && k.per_head ? c->head_dim : 0);
    if (rc) return rc;
  }
  return SKIPKV_OK;
}

}  // namespace
}  // namespace skipkv

using namespace skipkv;

extern "C" {

// ---- the path on the cache's shared ranges, contiguous cache ------------------------------------------

int skipkv_workspace_bytes(const skipkv_cache *cache, const skipkv_params *params, size_t *out_bytes) {
  Call k;
  k.stages = kScore | kSelect | kCompact;
  k.cache = cache;
  k.params = params;
  return size_call(k, out_bytes);
}

int skipkv_score(const skipkv_cache *cache, const skipkv_params *params, const void *q_obs,
                 const float *tok_redundancy, float *sent_score, float *sent_lambda, float *tok_importance,
                 void *ws, size_t ws_bytes, void *stream) {
  Call k;
  k.stages = kScore;
  k.cache = cache;
  k.params = params;
  k.q_obs = q_obs;
  k.tok_red = tok_redundancy;
  k.sent_score = sent_score;
  k.sent_lambda = sent_lambda;
  k.tok_imp = tok_importance;
  k.ws = ws;
  k.ws_bytes = ws_bytes;
  k.stream = stream;
  return run_call(k);
}

int skipkv_score_shared(const skipkv_cache *cache, const skipkv_params *params, const void *q_obs,
                        const float *tok_redundancy, const float *shared_lambda, float *sent_score, float *sent_lambda,
                        float *tok_importance, void *ws, size_t ws_bytes, void *stream) {
  Call k;
  k.stages = kScore;
  k.cache = cache;
  k.params = params;
  k.q_obs = q_obs;
  k.tok_red = tok_redundancy;
  k.shared = true;
  k.shared_lambda = shared_lambda;
  k.sent_score = sent_score;
  k.sent_lambda = sent_lambda;
  k.tok_imp = tok_importance;
  k.ws = ws;
  k.ws_bytes = ws_bytes;
  k.stream = stream;
  return run_call(k);
}

int skipkv_select(const skipkv_cache *cache, const skipkv_params *params, const float *sent_score,
                  uint8_t *sent_keep, int32_t *kept_idx, int32_t *new_len, int32_t *new_sent_off,
                  int32_t *new_sent_cnt, int32_t kept_stride, void *stream) {
  Call k;
  k.stages = kSelect;
  k.cache = cache;
  k.params = params;
  k.sent_score = const_cast<float *>(sent_score);
  k.keep = sent_keep;
  k.kept_idx = kept_idx;
  k.new_len = new_len;
  k.new_sent_off = new_sent_off;
  k.new_sent_cnt = new_sent_cnt;
  k.kept_stride = kept_stride;
  k.stream = stream;
  return run_call(k);
}

int skipkv_select_tokens(const skipkv_cache *cache, const skipkv_params *params, const float *tok_importance,
                         const float *tok_redundancy, const float *sent_lambda, float *tok_score,
                         uint8_t *tok_keep, int32_t *kept_idx, int32_t *new_len, int32_t *new_sent_off,
                         int32_t *new_sent_cnt, int32_t kept_stride, void *stream) {
  Call k;
  k.stages = kSelectTokens;
  k.cache = cache;
  k.params = params;
  k.tok_imp_in = tok_importance;
  k.tok_red = tok_redundancy;
  k.lambda_in = sent_lambda;
  k.tok_score = tok_score;
  k.keep = tok_keep;
  k.kept_idx = kept_idx;
  k.new_len = new_len;
  k.new_sent_off = new_sent_off;
  k.new_sent_cnt = new_sent_cnt;
  k.kept_stride = kept_stride;
  k.stream = stream;
  return run_call(k);
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

namespace {
// The arguments that every whole-step entry point has in common.
Call step_call(const skipkv_cache *cache, const skipkv_params *params, const void *q_obs, const float *tok_redundancy,
               float *sent_score, float *sent_lambda, float *tok_importance, uint8_t *sent_keep, int32_t *kept_idx,
               int32_t *new_len, int32_t *new_sent_off, int32_t *new_sent_cnt, int32_t kept_stride, void *ws,
               size_t ws_bytes, void *stream) {
  Call k;
  k.stages = kScore | kSelect | kCompact;
  k.cache = cache;
  k.params = params;
  k.q_obs = q_obs;
  k.tok_red = tok_redundancy;
  k.sent_score = sent_score;
  k.sent_lambda = sent_lambda;
  k.tok_imp = tok_importance;
  k.keep = sent_keep;
  k.kept_idx = kept_idx;
  k.new_len = new_len;
  k.new_sent_off = new_sent_off;
  k.new_sent_cnt = new_sent_cnt;
  k.kept_stride = kept_stride;
  k.ws = ws;
  k.ws_bytes = ws_bytes;
  k.stream = stream;
  return k;
}
}  // namespace

int skipkv_step(const skipkv_cache *cache, const skipkv_params *params, const void *q_obs,
                const float *tok_redundancy, float *sent_score, float *sent_lambda, float *tok_importance,
                uint8_t *sent_keep, int32_t *kept_idx, int32_t *new_len, int32_t *new_sent_off,
                int32_t *new_sent_cnt, int32_t kept_stride, void *ws, size_t ws_bytes, void *stream) {
  return run_call(step_call(cache, params, q_obs, tok_redundancy, sent_score, sent_lambda, tok_importance, sent_keep,
                            kept_idx, new_len, new_sent_off, new_sent_cnt, kept_stride, ws, ws_bytes, stream));
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
  size_t need = 0;
  int rc = skipkv_workspace_bytes(cache, params, &need);
  if (rc) return rc;
  if (need > (size_t)SKIPKV_STATIC_WS_BYTES) return SKIPKV_EWORKSPACE;  // the problem needs more scratch than the array holds
  void *ws = nullptr;
  rc = static_scratch(&ws);
  if (rc) return rc;
  // From here on this is skipkv_step on the array: the plan's fill kernels reset every counter
  // and marker that must start from a known value, so what the previous call left is harmless.
  return skipkv_step(cache, params, q_obs, tok_redundancy, sent_score, sent_lambda, tok_importance, sent_keep, kept_idx,
                     new_len, new_sent_off, new_sent_cnt, kept_stride, ws, (size_t)SKIPKV_STATIC_WS_BYTES, stream);
}

// ---- paged cache ------------------------------------------------------------------------------------------

int skipkv_paged_workspace_bytes(const skipkv_cache *cache, const skipkv_paging *paging, const skipkv_params *params,
                                 size_t *out_bytes) {
  Call k;
  k.stages = kScore | kSelect | kCompact;
  k.cache = cache;
  k.params = params;
  k.paged = true;
  k.paging = paging;
  return size_call(k, out_bytes);
}

int skipkv_score_paged(const skipkv_cache *cache, const skipkv_paging *paging, const skipkv_params *params,
                       const void *q_obs, const float *tok_redundancy, float *sent_score, float *sent_lambda,
                       float *tok_importance, void *ws, size_t ws_bytes, void *stream) {
  Call k = step_call(cache, params, q_obs, tok_redundancy, sent_score, sent_lambda, tok_importance, nullptr, nullptr, nullptr,
                     nullptr, nullptr, 0, ws, ws_bytes, stream);
  k.stages = kScore;
  k.paged = true;
  k.paging = paging;
  return run_call(k);
}

int skipkv_score_shared_paged(const skipkv_cache *cache, const skipkv_paging *paging, const skipkv_params *params,
                              const void *q_obs, const float *tok_redundancy, const float *shared_lambda, float *sent_score,
                              float *sent_lambda, float *tok_importance, void *ws, size_t ws_bytes, void *stream) {
  Call k = step_call(cache, params, q_obs, tok_redundancy, sent_score, sent_lambda, tok_importance, nullptr, nullptr, nullptr,
                     nullptr, nullptr, 0, ws, ws_bytes, stream);
  k.stages = kScore;
  k.paged = true;
  k.paging = paging;
  k.shared = true;
  k.shared_lambda = shared_lambda;
  return run_call(k);
}

int skipkv_step_paged(const skipkv_cache *cache, const skipkv_paging *paging, const skipkv_params *params,
                      const void *q_obs, const float *tok_redundancy, float *sent_score, float *sent_lambda,
                      float *tok_importance, uint8_t *sent_keep, int32_t *kept_idx, int32_t *new_len,
                      int32_t *new_sent_off, int32_t *new_sent_cnt, int32_t kept_stride, void *ws, size_t ws_bytes,
                      void *stream) {
  Call k = step_call(cache, params, q_obs, tok_redundancy, sent_score, sent_lambda, tok_importance, sent_keep, kept_idx,
                     new_len, new_sent_off, new_sent_cnt, kept_stride, ws, ws_bytes, stream);
  k.paged = true;
  k.paging = paging;
  return run_call(k);
}

// ---- per-head ranges --------------------------------------------------------------------------------------

int skipkv_ranges_workspace_bytes(const skipkv_cache *cache, const skipkv_params *params, size_t *out_bytes) {
  Call k;
  k.stages = kScore | kSelect | kCompact;
  k.cache = cache;
  k.params = params;
  k.per_head = true;
  return size_call(k, out_bytes);
}

int skipkv_step_ranges(const skipkv_cache *cache, const skipkv_ranges *ranges, const skipkv_params *params,
                       const void *q_obs, const float *tok_redundancy, float *sent_score, float *sent_lambda,
                       float *tok_importance, uint8_t *sent_keep, int32_t *kept_idx, int32_t *new_len,
                       int32_t *new_sent_off, int32_t *new_sent_cnt, int32_t kept_stride, void *ws, size_t ws_bytes,
                       void *stream) {
  Call k = step_call(cache, params, q_obs, tok_redundancy, sent_score, sent_lambda, tok_importance, sent_keep, kept_idx,
                     new_len, new_sent_off, new_sent_cnt, kept_stride, ws, ws_bytes, stream);
  k.per_head = true;
  k.ranges = ranges;
  return run_call(k);
}

// The parts of skipkv_step_ranges, for callers that select token by token in between.
int skipkv_score_ranges(const skipkv_cache *cache, const skipkv_ranges *ranges, const skipkv_params *params,
                        const void *q_obs, const float *tok_redundancy, float *sent_score, float *sent_lambda,
                        float *tok_importance, void *ws, size_t ws_bytes, void *stream) {
  Call k = step_call(cache, params, q_obs, tok_redundancy, sent_score, sent_lambda, tok_importance, nullptr, nullptr, nullptr,
                     nullptr, nullptr, 0, ws, ws_bytes, stream);
  k.stages = kScore;
  k.per_head = true;
  k.ranges = ranges;
  return run_call(k);
}

// Shared lambda (hidden-state similarity) on per-head ranges.
int skipkv_score_shared_ranges(const skipkv_cache *cache, const skipkv_ranges *ranges, const int32_t *sent_id,
                               const int32_t *lambda_ptr, const skipkv_params *params, const void *q_obs,
                               const float *tok_redundancy, const float *shared_lambda, float *sent_score,
                               float *sent_lambda, float *tok_importance, void *ws, size_t ws_bytes, void *stream) {
  Call k = step_call(cache, params, q_obs, tok_redundancy, sent_score, sent_lambda, tok_importance, nullptr, nullptr, nullptr,
                     nullptr, nullptr, 0, ws, ws_bytes, stream);
  k.stages = kScore;
  k.per_head = true;
  k.ranges = ranges;
  k.shared = true;
  k.shared_lambda = shared_lambda;
  k.sent_id = sent_id;
  k.lam_ptr = lambda_ptr;
  return run_call(k);
}

int skipkv_select_ranges(const skipkv_cache *cache, const skipkv_ranges *ranges, const skipkv_params *params,
                         const float *sent_score, uint8_t *sent_keep, int32_t *kept_idx, int32_t *new_len,
                         int32_t *new_sent_off, int32_t *new_sent_cnt, int32_t kept_stride, void *ws, size_t ws_bytes,
                         void *stream) {
  Call k = step_call(cache, params, nullptr, nullptr, const_cast<float *>(sent_score), nullptr, nullptr, sent_keep, kept_idx,
                     new_len, new_sent_off, new_sent_cnt, kept_stride, ws, ws_bytes, stream);
  k.stages = kSelect;
  k.per_head = true;
  k.ranges = ranges;
  return run_call(k);
}

int skipkv_select_tokens_ranges(const skipkv_cache *cache, const skipkv_ranges *ranges, const skipkv_params *params,
                                const float *tok_importance, const float *tok_redundancy, const float *sent_lambda,
                                float *tok_score, uint8_t *tok_keep, int32_t *kept_idx, int32_t *new_len,
                                int32_t *new_sent_off, int32_t *new_sent_cnt, int32_t kept_stride, void *ws,
                                size_t ws_bytes, void *stream) {
  Call k = step_call(cache, params, nullptr, tok_redundancy, nullptr, nullptr, nullptr, tok_keep, kept_idx, new_len,
                     new_sent_off, new_sent_cnt, kept_stride, ws, ws_bytes, stream);
  k.stages = kSelectTokens;
  k.per_head = true;
  k.ranges = ranges;
  k.tok_imp_in = tok_importance;
  k.lambda_in = sent_lambda;
  k.tok_score = tok_score;
  return run_call(k);
}

// ---- per-head ranges on a paged cache --------------------------------------------------------------------

int skipkv_ranges_paged_workspace_bytes(const skipkv_cache *cache, const skipkv_paging *paging,
                                        const skipkv_params *params, size_t *out_bytes) {
  Call k;
  k.stages = kScore | kSelect | kCompact;
  k.cache = cache;
  k.params = params;
  k.per_head = true;
  k.paged = true;
  k.paging = paging;
  return size_call(k, out_bytes);
}

int skipkv_score_ranges_paged(const skipkv_cache *cache, const skipkv_ranges *ranges, const skipkv_paging *paging,
                              const int32_t *sent_id, const int32_t *lambda_ptr, const float *shared_lambda,
                              const skipkv_params *params, const void *q_obs, const float *tok_redundancy,
                              float *sent_score, float *sent_lambda, float *tok_importance, void *ws, size_t ws_bytes,
                              void *stream) {
  Call k = step_call(cache, params, q_obs, tok_redundancy, sent_score, sent_lambda, tok_importance, nullptr, nullptr, nullptr,
                     nullptr, nullptr, 0, ws, ws_bytes, stream);
  k.stages = kScore;
  k.per_head = true;
  k.ranges = ranges;
  k.paged = true;
  k.paging = paging;
  k.shared = shared_lambda != nullptr;
  k.shared_lambda = shared_lambda;
  k.sent_id = sent_id;
  k.lam_ptr = lambda_ptr;
  return run_call(k);
}

int skipkv_step_ranges_paged(const skipkv_cache *cache, const skipkv_ranges *ranges, const skipkv_paging *paging,
                             const skipkv_params *params, const void *q_obs, const float *tok_redundancy,
                             float *sent_score, float *sent_lambda, float *tok_importance, uint8_t *sent_keep,
                             int32_t *kept_idx, int32_t *new_len, int32_t *new_sent_off, int32_t *new_sent_cnt,
                             int32_t kept_stride, void *ws, size_t ws_bytes, void *stream) {
  Call k = step_call(cache, params, q_obs, tok_redundancy, sent_score, sent_lambda, tok_importance, sent_keep, kept_idx,
                     new_len, new_sent_off, new_sent_cnt, kept_stride, ws, ws_bytes, stream);
  k.per_head = true;
  k.ranges = ranges;
  k.paged = true;
  k.paging = paging;
  return run_call(k);
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

// Sentence numbers of a head's surviving sentences (shared lambda on per-head ranges).
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
