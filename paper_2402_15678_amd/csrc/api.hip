// C ABI of the verification step (declared in include/minions_verify.h): argument validation,
// workspace layout and the launch sequence of one decoder forward.  Every step of the path runs
// in the kernels of this library; this file only orders them on the caller's stream.
#include "../../include/minions_verify.h"
#include "launch.h"

#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <string>
#include <vector>

using namespace mn;

// Timing taps: pairs of events around kernel-family launches, summed per family on collect.
struct Prof {
  bool on = false;
  std::vector<hipEvent_t> pool;   // created on demand, reused after every collect
  std::vector<int> kind;          // kind[i] belongs to the pair (pool[2i], pool[2i+1])
  size_t used = 0;                // events handed out since the last collect
  hipEvent_t take() {
    if (used == pool.size()) {
      hipEvent_t e;
      if (hipEventCreate(&e) != hipSuccess) return nullptr;
      pool.push_back(e);
    }
    return pool[used++];
  }
  ~Prof() { for (hipEvent_t e : pool) (void)hipEventDestroy(e); }
};

struct Tap {  // RAII bracket around one launch
  Prof* p; hipStream_t st; hipEvent_t end = nullptr;
  Tap(Prof* prof, int kind, hipStream_t s) : p(prof && prof->on ? prof : nullptr), st(s) {
    if (!p) return;
    hipEvent_t b = p->take();
    end = p->take();
    if (!b || !end) { p = nullptr; return; }
    p->kind.push_back(kind);
    (void)hipEventRecord(b, st);
  }
  ~Tap() { if (p) (void)hipEventRecord(end, st); }
};

struct mn_ctx {
  mn_model_desc d;
  Prof prof;
  const void *tok_emb, *pos_emb, *final_norm_g, *final_norm_b, *lm_head;
  std::vector<const void*> ln1_g, ln1_b, wqkv, bqkv, wo, bo, ln2_g, ln2_b, w1, b1, w2, b2;
  std::string err;
};

static std::string g_create_err;

static mn_status fail(mn_ctx* c, mn_status s, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  if (c) c->err = buf;
  else g_create_err = buf;
  return s;
}

static mn_status hip_check(mn_ctx* c, const char* where) {
  const hipError_t e = hipGetLastError();
  if (e == hipSuccess) return MN_OK;
  return fail(c, MN_EHIP, "%s: %s", where, hipGetErrorString(e));
}

extern "C" const char* mn_status_str(mn_status s) {
  switch (s) {
    case MN_OK: return "MN_OK";
    case MN_EINVAL: return "MN_EINVAL";
    case MN_ENULL: return "MN_ENULL";
    case MN_ESHAPE: return "MN_ESHAPE";
    case MN_EUNSUPPORTED: return "MN_EUNSUPPORTED";
    case MN_ECAPACITY: return "MN_ECAPACITY";
    case MN_EWORKSPACE: return "MN_EWORKSPACE";
    case MN_EHIP: return "MN_EHIP";
  }
  return "MN_?";
}

extern "C" const char* mn_last_error(const mn_ctx* ctx) { return ctx ? ctx->err.c_str() : g_create_err.c_str(); }

static bool copy_ptrs(std::vector<const void*>& dst, const void* const* src, int n, bool required) {
  dst.assign(n, nullptr);
  if (!src) return !required;
  for (int i = 0; i < n; ++i) {
    dst[i] = src[i];
    if (required && !src[i]) return false;
  }
  return true;
}

extern "C" mn_status mn_create(mn_ctx** out, const mn_model_desc* d, const mn_weights* w) {
  if (!out) return fail(nullptr, MN_ENULL, "mn_create: out is NULL");
  *out = nullptr;
  if (!d || !w) return fail(nullptr, MN_ENULL, "mn_create: desc or weights is NULL");
  if (d->arch != MN_ARCH_OPT && d->arch != MN_ARCH_LLAMA) return fail(nullptr, MN_EINVAL, "mn_create: arch %d", d->arch);
  if (d->dtype != MN_DT_F32 && d->dtype != MN_DT_BF16) return fail(nullptr, MN_EINVAL, "mn_create: dtype %d", d->dtype);
  if (d->n_layers < 0 || d->d_model <= 0 || d->n_heads <= 0 || d->n_kv_heads <= 0 || d->head_dim <= 0 || d->d_ffn <= 0 ||
      d->vocab <= 0 || d->max_pos <= 0)
    return fail(nullptr, MN_EINVAL, "mn_create: non-positive dimension");
  if (d->n_heads % d->n_kv_heads) return fail(nullptr, MN_ESHAPE, "mn_create: n_heads %% n_kv_heads != 0");
  if (d->arch == MN_ARCH_OPT && d->n_heads != d->n_kv_heads)
    return fail(nullptr, MN_ESHAPE, "mn_create: OPT-style models have n_kv_heads == n_heads");
  if (d->head_dim % 8 || 256 % d->head_dim)
    return fail(nullptr, MN_EUNSUPPORTED, "mn_create: head_dim %d (supported: 8, 16, 32, 64, 128, 256)", d->head_dim);
  if (d->d_model % 64 || d->d_model > 8192)
    return fail(nullptr, MN_EUNSUPPORTED, "mn_create: d_model %d (must be a multiple of 64, at most 8192)", d->d_model);
  if ((d->n_heads * d->head_dim) % 64 || d->d_ffn % 64)
    return fail(nullptr, MN_EUNSUPPORTED, "mn_create: n_heads*head_dim and d_ffn must be multiples of 64");
  if (d->dtype == MN_DT_BF16 && (d->d_model % 128 || (d->n_heads * d->head_dim) % 128 || d->d_ffn % 128))
    return fail(nullptr, MN_EUNSUPPORTED, "mn_create: bf16 models need d_model, n_heads*head_dim and d_ffn to be multiples of 128");
  if (!(d->norm_eps >= 0.f)) return fail(nullptr, MN_EINVAL, "mn_create: norm_eps");
  if (d->arch == MN_ARCH_LLAMA && !(d->rope_base > 0.f)) return fail(nullptr, MN_EINVAL, "mn_create: rope_base");
  if (!w->tok_emb || !w->lm_head || !w->final_norm_g) return fail(nullptr, MN_ENULL, "mn_create: tok_emb/lm_head/final_norm_g");
  const bool opt = d->arch == MN_ARCH_OPT;
  if (opt && (!w->pos_emb || !w->final_norm_b)) return fail(nullptr, MN_ENULL, "mn_create: pos_emb/final_norm_b (OPT)");
  mn_ctx* c = new mn_ctx();
  c->d = *d;
  c->tok_emb = w->tok_emb;
  c->pos_emb = opt ? w->pos_emb : nullptr;
  c->final_norm_g = w->final_norm_g;
  c->final_norm_b = opt ? w->final_norm_b : nullptr;
  c->lm_head = w->lm_head;
  const int L = d->n_layers;
  bool good = copy_ptrs(c->ln1_g, w->ln1_g, L, true) && copy_ptrs(c->wqkv, w->wqkv, L, true) &&
              copy_ptrs(c->wo, w->wo, L, true) && copy_ptrs(c->ln2_g, w->ln2_g, L, true) &&
              copy_ptrs(c->w1, w->w1, L, true) && copy_ptrs(c->w2, w->w2, L, true) &&
              copy_ptrs(c->ln1_b, w->ln1_b, L, opt) && copy_ptrs(c->ln2_b, w->ln2_b, L, opt) &&
              copy_ptrs(c->bqkv, w->bqkv, L, opt) && copy_ptrs(c->bo, w->bo, L, opt) &&
              copy_ptrs(c->b1, w->b1, L, opt) && copy_ptrs(c->b2, w->b2, L, opt);
  if (!good) {
    delete c;
    return fail(nullptr, MN_ENULL, "mn_create: a per-layer parameter pointer is NULL");
  }
  if (!opt) {  // Llama-style models carry no biases and no norm shifts
    for (auto* v : {&c->ln1_b, &c->ln2_b, &c->bqkv, &c->bo, &c->b1, &c->b2}) v->assign(L, nullptr);
  }
  *out = c;
  return MN_OK;
}

extern "C" void mn_destroy(mn_ctx* ctx) { delete ctx; }

// ---- workspace layout ---------------------------------------------------------------------------
static size_t al(size_t x) { return (x + 255) & ~(size_t)255; }

struct Layout {
  size_t row_seq, row_j, row_pos, row_tok, row_slot, seq_row0, seq_ctx, seq_ok, attn_tps, rope_cos, rope_sin;
  size_t x, h, q, attn, act, partials, logits, attn_scratch, attn_items, attn_row_splits, total;
  size_t partials_bytes, attn_scratch_bytes, attn_items_capacity;
};

static Layout make_layout(const mn_model_desc& d, int B, int M, int max_ctx) {
  Layout L{};
  const size_t es = d.dtype == MN_DT_BF16 ? 2 : 4;
  const size_t Mr = M > 0 ? M : 1;
  size_t at = 0;
  // small arrays are packed at 256 bytes; everything from 64 KB on starts at a 4 KB boundary, so that the place of
  // the activation buffers and partial sums relative to pages and memory channels does not move with the size of
  // the bookkeeping in front of them
  auto take = [&](size_t bytes) {
    if (bytes >= (64u << 10)) at = (at + 4095) & ~(size_t)4095;
    size_t o = at;
    at += al(bytes);
    return o;
  };
  L.row_seq = take(Mr * 4); L.row_j = take(Mr * 4); L.row_pos = take(Mr * 4); L.row_tok = take(Mr * 4);
  L.row_slot = take(Mr * 4);
  L.seq_row0 = take(((size_t)B + 1) * 4); L.seq_ctx = take((size_t)B * 4 + 4); L.seq_ok = take((size_t)B * 4 + 4);
  L.attn_tps = take(4);
  L.rope_cos = take(Mr * (d.head_dim / 2) * 4); L.rope_sin = take(Mr * (d.head_dim / 2) * 4);
  L.x = take(Mr * d.d_model * 4);
  L.h = take(Mr * d.d_model * es);
  L.q = take(Mr * d.n_heads * d.head_dim * es);
  L.attn = take(Mr * d.n_heads * d.head_dim * es);
  L.act = take(Mr * d.d_ffn * es);
  // Partial sums of the widest projection at the largest split it can get with M rows OR FEWER: a workspace
  // sized for max_rows must serve every step with at most that many rows, and the k-split a projection gets is
  // not monotone in the row count (it drops where the kernel family changes and where a further row block
  // starts).  The split is constant between those borders, all of which are multiples of 16, so the largest
  // need is found at the right ends: M itself and every multiple of 16 below it.
  const int nqkv = (d.n_heads + 2 * d.n_kv_heads) * d.head_dim;
  const int w1r = d.d_ffn * (d.arch == MN_ARCH_LLAMA ? 2 : 1);
  size_t pmax = 0;
  const int Ns[5] = {nqkv, d.d_model, w1r, d.d_model, d.vocab};
  const int Ks[5] = {d.d_model, d.n_heads * d.head_dim, d.d_model, d.d_ffn, d.d_model};
  for (int i = 0; i < 5; ++i) {
    for (int m2 = (int)Mr;; m2 = (m2 - 1) / 16 * 16) {
      const size_t s = (size_t)gemm_pick_split(m2, Ns[i], Ks[i], d.dtype);
      const size_t b = s * (size_t)m2 * Ns[i] * 4;
      if (b > pmax) pmax = b;
      if (m2 <= 16 || (size_t)MN_MAX_SPLIT_K * m2 * Ns[i] * 4 <= pmax) break;  // fewer rows cannot need more
    }
  }
  L.partials_bytes = pmax;
  L.partials = take(pmax);
  L.logits = take(Mr * d.vocab * 4);
  L.attn_scratch_bytes = attention_scratch_bytes(M, d.n_heads, d.head_dim, max_ctx, d.dtype);
  L.attn_scratch = take(L.attn_scratch_bytes);
  L.attn_items_capacity = attention_items_capacity(B, M, d.n_heads, d.n_kv_heads);
  L.attn_items = take(L.attn_items_capacity * 8 * 4);
  L.attn_row_splits = take(Mr * 4);
  L.total = at;
  return L;
}

extern "C" size_t mn_workspace_bytes(const mn_ctx* ctx, int B, int max_rows, int max_ctx) {
  if (!ctx || B < 0 || B > MN_MAX_BATCH || max_rows < 0 || max_ctx < 0) return 0;
  return make_layout(ctx->d, B, max_rows, max_ctx).total;
}

// ---- vote ---------------------------------------------------------------------------------------
extern "C" mn_status mn_mv_vote(mn_ctx* ctx, const int32_t* drafts, const int32_t* spec_len, const float* ssm_w, int B,
                                int n, int k_max, int mode, int32_t* voted, int32_t* voted_ssm, int32_t* dev_status,
                                void* stream) {
  if (B < 0 || B > MN_MAX_BATCH) return fail(ctx, MN_EINVAL, "mn_mv_vote: B = %d outside [0, %d]", B, MN_MAX_BATCH);
  if (n < 1 || n > MN_MAX_DRAFTS) return fail(ctx, MN_EINVAL, "mn_mv_vote: n = %d outside [1, %d]", n, MN_MAX_DRAFTS);
  if (k_max < 0) return fail(ctx, MN_EINVAL, "mn_mv_vote: k_max = %d", k_max);
  if (mode != MN_VOTE_TREE && mode != MN_VOTE_COLUMN) return fail(ctx, MN_EINVAL, "mn_mv_vote: mode = %d", mode);
  if (B == 0) return MN_OK;
  if (!spec_len || !ssm_w || !voted_ssm) return fail(ctx, MN_ENULL, "mn_mv_vote: spec_len/ssm_w/voted_ssm is NULL");
  if (k_max > 0 && (!drafts || !voted)) return fail(ctx, MN_ENULL, "mn_mv_vote: drafts/voted is NULL");
  {
    Tap t(ctx ? &ctx->prof : nullptr, MN_PROF_VOTE, (hipStream_t)stream);
    launch_vote(drafts, spec_len, ssm_w, B, n, k_max, mode, voted, voted_ssm, dev_status, (hipStream_t)stream);
  }
  return hip_check(ctx, "mn_mv_vote");
}

// ---- accept + commit ----------------------------------------------------------------------------
extern "C" mn_status mn_accept_and_commit(mn_ctx* ctx, const int32_t* voted, const int32_t* greedy,
                                          const int32_t* spec_len, int B, int k_max, mn_kv* kv, int32_t* accepted_len,
                                          int32_t* out_tokens, int32_t* n_out, int32_t* next_last_tok,
                                          int32_t* blocks_in_use, int32_t* dev_status, void* stream) {
  if (B < 0 || B > MN_MAX_BATCH) return fail(ctx, MN_EINVAL, "mn_accept_and_commit: B = %d", B);
  if (k_max < 0) return fail(ctx, MN_EINVAL, "mn_accept_and_commit: k_max = %d", k_max);
  if (B == 0) return MN_OK;
  if (!kv || !kv->ctx_lens) return fail(ctx, MN_ENULL, "mn_accept_and_commit: kv/ctx_lens is NULL");
  if (kv->block_size <= 0 || kv->max_blocks_per_seq <= 0) return fail(ctx, MN_EINVAL, "mn_accept_and_commit: block geometry");
  if (!greedy || !spec_len || !accepted_len || !out_tokens || !n_out || !next_last_tok || !blocks_in_use)
    return fail(ctx, MN_ENULL, "mn_accept_and_commit: a required pointer is NULL");
  if (k_max > 0 && !voted) return fail(ctx, MN_ENULL, "mn_accept_and_commit: voted is NULL");
  {
    Tap t(ctx ? &ctx->prof : nullptr, MN_PROF_ACCEPT, (hipStream_t)stream);
    launch_accept_commit(voted, greedy, spec_len, B, k_max, kv->ctx_lens, kv->block_size, kv->max_blocks_per_seq,
                         accepted_len, out_tokens, n_out, next_last_tok, blocks_in_use, dev_status, (hipStream_t)stream);
  }
  return hip_check(ctx, "mn_accept_and_commit");
}

// ---- speculation quality metric + SSM weight update ------------------------------------------------
extern "C" mn_status mn_acr_update(mn_ctx* ctx, const int32_t* voted_ssm, const int32_t* accepted_len,
                                   const int32_t* spec_len, const int32_t* n_out, int B, int n, double reward_threshold,
                                   double punish_threshold, float reward_factor, float punish_factor, float* ssm_w,
                                   double* acr, void* stream) {
  if (B < 0 || B > MN_MAX_BATCH) return fail(ctx, MN_EINVAL, "mn_acr_update: B = %d", B);
  if (n < 1 || n > MN_MAX_DRAFTS) return fail(ctx, MN_EINVAL, "mn_acr_update: n = %d", n);
  if (!(reward_factor > 0.f) || !(punish_factor > 0.f)) return fail(ctx, MN_EINVAL, "mn_acr_update: factors must be positive");
  if (!(punish_threshold <= reward_threshold)) return fail(ctx, MN_EINVAL, "mn_acr_update: punish_threshold above reward_threshold");
  if (!ssm_w) return fail(ctx, MN_ENULL, "mn_acr_update: ssm_w is NULL");
  if (B > 0 && (!voted_ssm || !accepted_len || !spec_len)) return fail(ctx, MN_ENULL, "mn_acr_update: a required pointer is NULL");
  {
    Tap t(ctx ? &ctx->prof : nullptr, MN_PROF_ACCEPT, (hipStream_t)stream);
    launch_acr_update(voted_ssm, accepted_len, spec_len, n_out, B, n, reward_threshold, punish_threshold, reward_factor,
                      punish_factor, ssm_w, acr, (hipStream_t)stream);
  }
  return hip_check(ctx, "mn_acr_update");
}

extern "C" mn_status mn_verify_sample(mn_ctx* ctx, const float* logits, const int32_t* voted, const float* draft_probs,
                                      const int32_t* spec_len, const int32_t* greedy, int B, int k_max, int M, int vocab,
                                      double temperature, uint64_t seed, uint64_t step, int32_t* sampled,
                                      int32_t* dev_status, void* stream) {
  if (B < 0 || B > MN_MAX_BATCH) return fail(ctx, MN_EINVAL, "mn_verify_sample: B = %d", B);
  if (k_max < 0 || k_max > 4096) return fail(ctx, MN_EINVAL, "mn_verify_sample: k_max = %d", k_max);
  if (M < 0 || (long)M > (long)B * (k_max + 1)) return fail(ctx, MN_EINVAL, "mn_verify_sample: M = %d rows for B = %d, k_max = %d", M, B, k_max);
  if (vocab < 1 || vocab > verify_sample_max_vocab()) return fail(ctx, MN_EUNSUPPORTED, "mn_verify_sample: vocab = %d", vocab);
  if (!(temperature > 0.0) || !(temperature < INFINITY)) return fail(ctx, MN_EINVAL, "mn_verify_sample: temperature must be positive and finite");
  if (step >> 56) return fail(ctx, MN_EINVAL, "mn_verify_sample: step must be below 2^56");
  if (B > 0 && (!logits || !spec_len || !greedy || !sampled)) return fail(ctx, MN_ENULL, "mn_verify_sample: a required pointer is NULL");
  if (B > 0 && k_max > 0 && (!voted || !draft_probs)) return fail(ctx, MN_ENULL, "mn_verify_sample: voted or draft_probs is NULL");
  if (B == 0) return MN_OK;
  {
    Tap t(ctx ? &ctx->prof : nullptr, MN_PROF_ACCEPT, (hipStream_t)stream);
    launch_verify_sample(logits, voted, draft_probs, spec_len, greedy, B, k_max, M, vocab, temperature, seed, step, sampled,
                         dev_status, (hipStream_t)stream);
  }
  return hip_check(ctx, "mn_verify_sample");
}

extern "C" mn_status mn_draft_sample(mn_ctx* ctx, const float* logits, int B, int vocab, double temperature, uint64_t seed,
                                     uint64_t step, int ssm, int t, int32_t* tokens, long token_stride, float* probs,
                                     long probs_stride, void* stream) {
  if (B < 0 || B > MN_MAX_BATCH) return fail(ctx, MN_EINVAL, "mn_draft_sample: B = %d", B);
  if (vocab < 1 || vocab > verify_sample_max_vocab()) return fail(ctx, MN_EUNSUPPORTED, "mn_draft_sample: vocab = %d", vocab);
  if (!(temperature > 0.0) || !(temperature < INFINITY)) return fail(ctx, MN_EINVAL, "mn_draft_sample: temperature must be positive and finite");
  if (step >> 56) return fail(ctx, MN_EINVAL, "mn_draft_sample: step must be below 2^56");
  if (ssm < 0 || ssm >= MN_MAX_DRAFTS) return fail(ctx, MN_EINVAL, "mn_draft_sample: ssm = %d", ssm);
  if (t < 0) return fail(ctx, MN_EINVAL, "mn_draft_sample: t = %d", t);
  if (token_stride < 1 || (probs && probs_stride < vocab)) return fail(ctx, MN_EINVAL, "mn_draft_sample: strides");
  if (B > 0 && (!logits || !tokens)) return fail(ctx, MN_ENULL, "mn_draft_sample: a required pointer is NULL");
  if (B == 0) return MN_OK;
  {
    Tap tp(ctx ? &ctx->prof : nullptr, MN_PROF_VOTE, (hipStream_t)stream);
    launch_draft_sample(logits, B, vocab, temperature, seed, step, ssm, t, tokens, token_stride, probs, probs_stride,
                        (hipStream_t)stream);
  }
  return hip_check(ctx, "mn_draft_sample");
}

// ---- shared checks --------------------------------------------------------------------------------
static mn_status check_kv(mn_ctx* c, const mn_kv* kv, int max_ctx, const char* who) {
  if (!kv) return fail(c, MN_ENULL, "%s: kv is NULL", who);
  if (!kv->k_layers || !kv->v_layers || !kv->block_tables || !kv->ctx_lens) return fail(c, MN_ENULL, "%s: kv member is NULL", who);
  if (kv->block_size <= 0 || kv->num_blocks <= 0 || kv->max_blocks_per_seq <= 0)
    return fail(c, MN_EINVAL, "%s: block_size/num_blocks/max_blocks_per_seq", who);
  if ((long)max_ctx > (long)kv->max_blocks_per_seq * kv->block_size)
    return fail(c, MN_ECAPACITY, "%s: max_ctx %d exceeds the block table (%d blocks of %d)", who, max_ctx,
                kv->max_blocks_per_seq, kv->block_size);
  if (max_ctx > c->d.max_pos) return fail(c, MN_ECAPACITY, "%s: max_ctx %d exceeds max_pos %d", who, max_ctx, c->d.max_pos);
  return MN_OK;
}

static mn_status count_rows(mn_ctx* c, const int32_t* h_spec_len, int B, int k_max, int* M, int* max_q, const char* who) {
  long m = 0;
  int mq = 0;
  for (int b = 0; b < B; ++b) {
    const int k = h_spec_len[b];
    if (k < 0 || k > k_max) return fail(c, MN_EINVAL, "%s: h_spec_len[%d] = %d outside [0, %d]", who, b, k, k_max);
    m += k + 1;
    if (k + 1 > mq) mq = k + 1;
  }
  if (m > (1 << 20)) return fail(c, MN_EINVAL, "%s: %ld rows", who, m);
  *M = (int)m;
  *max_q = mq;
  return MN_OK;
}

struct Ws {
  unsigned char* base;
  Layout L;
  template <typename T> T* at(size_t off) const { return reinterpret_cast<T*>(base + off); }
};

static RowInfo row_info(const Ws& w) {
  RowInfo r;
  r.row_seq = w.at<int32_t>(w.L.row_seq);
  r.row_j = w.at<int32_t>(w.L.row_j);
  r.row_pos = w.at<int32_t>(w.L.row_pos);
  r.row_tok = w.at<int32_t>(w.L.row_tok);
  r.row_slot = w.at<int32_t>(w.L.row_slot);
  r.seq_row0 = w.at<int32_t>(w.L.seq_row0);
  r.seq_ctx = w.at<int32_t>(w.L.seq_ctx);
  r.seq_ok = w.at<int32_t>(w.L.seq_ok);
  r.attn_tps = w.at<int32_t>(w.L.attn_tps);
  return r;
}

static void run_prepare(mn_ctx* c, const Ws& w, const int32_t* last_tok, const int32_t* voted, const int32_t* spec_len,
                        int B, int k_max, int M, int max_ctx, const mn_kv* kv, bool tokens, int32_t* dev_status,
                        hipStream_t st) {
  PrepArgs p{};
  p.last_tok = tokens ? last_tok : nullptr;
  p.voted = voted;
  p.spec_len = spec_len;
  p.ctx_lens = kv->ctx_lens;
  p.block_tables = kv->block_tables;
  p.B = B; p.k_max = k_max; p.M = M;
  p.vocab = tokens ? c->d.vocab : 0;
  p.max_pos = c->d.max_pos;
  p.max_ctx = max_ctx;
  p.block_size = kv->block_size; p.num_blocks = kv->num_blocks; p.max_blocks_per_seq = kv->max_blocks_per_seq;
  p.rope_half = (tokens && c->d.arch == MN_ARCH_LLAMA) ? c->d.head_dim / 2 : 0;
  p.rope_base = c->d.rope_base;
  p.row_seq = w.at<int32_t>(w.L.row_seq); p.row_j = w.at<int32_t>(w.L.row_j);
  p.row_pos = w.at<int32_t>(w.L.row_pos); p.row_tok = w.at<int32_t>(w.L.row_tok);
  p.row_slot = w.at<int32_t>(w.L.row_slot);
  p.seq_row0 = w.at<int32_t>(w.L.seq_row0); p.seq_ctx = w.at<int32_t>(w.L.seq_ctx); p.seq_ok = w.at<int32_t>(w.L.seq_ok);
  p.attn_tps = w.at<int32_t>(w.L.attn_tps);
  p.kv_heads = c->d.n_kv_heads;
  p.q_per_kv = c->d.n_heads / c->d.n_kv_heads;
  p.attn_wgs = attention_target_workgroups();
  p.attn_min_tiles = attention_min_tiles();
  p.rope_cos = w.at<float>(w.L.rope_cos); p.rope_sin = w.at<float>(w.L.rope_sin);
  p.dev_status = dev_status;
  Tap t(&c->prof, MN_PROF_PREPARE, st);
  launch_prepare(p, st);
}

// ---- verify forward -------------------------------------------------------------------------------
extern "C" mn_status mn_verify_forward(mn_ctx* c, const int32_t* last_tok, const int32_t* voted, const int32_t* spec_len,
                                       const int32_t* h_spec_len, int B, int k_max, int max_ctx, const mn_kv* kv,
                                       int32_t* greedy, float* logits, void* workspace, size_t workspace_bytes,
                                       int32_t* dev_status, void* stream) {
  const char* who = "mn_verify_forward";
  if (!c) return MN_ENULL;
  if (B < 0 || B > MN_MAX_BATCH) return fail(c, MN_EINVAL, "%s: B = %d outside [0, %d]", who, B, MN_MAX_BATCH);
  if (k_max < 0) return fail(c, MN_EINVAL, "%s: k_max = %d", who, k_max);
  if (max_ctx < 0) return fail(c, MN_EINVAL, "%s: max_ctx = %d", who, max_ctx);
  if (B == 0) return MN_OK;
  if (!last_tok || !spec_len || !h_spec_len || !greedy) return fail(c, MN_ENULL, "%s: a required pointer is NULL", who);
  if (k_max > 0 && !voted) return fail(c, MN_ENULL, "%s: voted is NULL", who);
  if (mn_status s = check_kv(c, kv, max_ctx, who)) return s;
  int M = 0, max_q = 0;
  if (mn_status s = count_rows(c, h_spec_len, B, k_max, &M, &max_q, who)) return s;
  if (max_ctx < max_q) return fail(c, MN_EINVAL, "%s: max_ctx %d smaller than the longest scored run %d", who, max_ctx, max_q);
  if (!workspace) return fail(c, MN_ENULL, "%s: workspace is NULL", who);
  if ((uintptr_t)workspace & 255) return fail(c, MN_EWORKSPACE, "%s: workspace not 256-byte aligned", who);
  const mn_model_desc& d = c->d;
  Ws w{reinterpret_cast<unsigned char*>(workspace), make_layout(d, B, M, max_ctx)};
  if (workspace_bytes < w.L.total)
    return fail(c, MN_EWORKSPACE, "%s: workspace %zu bytes, need %zu", who, workspace_bytes, w.L.total);
  for (int l = 0; l < d.n_layers; ++l)
    if (!kv->k_layers[l] || !kv->v_layers[l]) return fail(c, MN_ENULL, "%s: kv layer %d pointer is NULL", who, l);

  hipStream_t st = (hipStream_t)stream;
  run_prepare(c, w, last_tok, voted, spec_len, B, k_max, M, max_ctx, kv, true, dev_status, st);
  const RowInfo rows = row_info(w);
  const bool llama = d.arch == MN_ARCH_LLAMA;
  const int nqkv = (d.n_heads + 2 * d.n_kv_heads) * d.head_dim;
  const int w1r = d.d_ffn * (llama ? 2 : 1);
  const int hdim = d.n_heads * d.head_dim;
  float* x = w.at<float>(w.L.x);
  void* h = w.at<void>(w.L.h);
  float* part = w.at<float>(w.L.partials);

  // partial sums of the previous projection, folded into the next norm
  const float* pend = nullptr;
  int pend_n = 0;
  const float* pend_bias = nullptr;

  hipError_t lerr = hipSuccess;  // first refusal of a launcher (a kernel attribute the runtime would not set)
  auto keep = [&](hipError_t e) { if (e != hipSuccess && lerr == hipSuccess) lerr = e; };
  auto norm = [&](const float* gain, const float* shift, bool embed) {
    NormArgs n{};
    n.x = x; n.partials = pend; n.n_partials = pend_n; n.bias = pend_bias;
    n.tok_emb = embed ? c->tok_emb : nullptr;
    n.pos_emb = embed ? c->pos_emb : nullptr;
    n.row_tok = rows.row_tok; n.row_pos = rows.row_pos;
    n.gain = gain; n.shift = shift; n.eps = d.norm_eps; n.h = h; n.M = M; n.d = d.d_model; n.dtype = d.dtype;
    n.dev_status = dev_status;
    Tap t(&c->prof, MN_PROF_NORM, st);
    launch_norm(n, st);
    pend = nullptr; pend_n = 0; pend_bias = nullptr;
  };
  auto gemm = [&](const void* a, const void* wt, float* out, int N, int K, int split) {
    GemmArgs g{};
    g.a = a; g.w = wt; g.out = out; g.bias = nullptr; g.M = M; g.N = N; g.K = K; g.split_k = split; g.dtype = d.dtype;
    g.dev_status = dev_status;
    Tap t(&c->prof, MN_PROF_GEMM, st);
    keep(launch_gemm(g, st));
  };

  for (int l = 0; l < d.n_layers; ++l) {
    norm((const float*)c->ln1_g[l], (const float*)c->ln1_b[l], l == 0);
    int s = gemm_pick_split(M, nqkv, d.d_model, d.dtype);
    gemm(h, c->wqkv[l], part, nqkv, d.d_model, s);
    RopeAppendArgs r{};
    r.qkv = part; r.n_partials = s; r.bias = (const float*)c->bqkv[l];
    r.rope_cos = llama ? w.at<float>(w.L.rope_cos) : nullptr;
    r.rope_sin = llama ? w.at<float>(w.L.rope_sin) : nullptr;
    r.rows = rows;
    r.kv = KvView{kv->k_layers[l], kv->v_layers[l], kv->block_tables, kv->block_size, kv->num_blocks, kv->max_blocks_per_seq};
    r.q = w.at<void>(w.L.q);
    // (the K/V rows of the scored tokens go to the pages in the precision the step's own attention reads them
    // back in, and every later step after it: one pass over k + 1 positions multiplies exactly the numbers k + 1
    // single-position passes multiply)
    r.M = M; r.H = d.n_heads; r.Hkv = d.n_kv_heads; r.hd = d.head_dim; r.dtype = d.dtype;
    r.dev_status = dev_status;
    {
      Tap t(&c->prof, MN_PROF_ROPE_APPEND, st);
      launch_rope_append(r, st);
    }
    AttnArgs at{};
    at.q = r.q; at.out = w.at<void>(w.L.attn); at.rows = rows; at.kv = r.kv;
    at.B = B; at.M = M; at.H = d.n_heads; at.Hkv = d.n_kv_heads; at.hd = d.head_dim; at.dtype = d.dtype;
    at.max_ctx = max_ctx; at.max_q = max_q;
    at.scratch = w.at<float>(w.L.attn_scratch); at.scratch_bytes = w.L.attn_scratch_bytes;
    at.items = w.at<int32_t>(w.L.attn_items); at.items_capacity = w.L.attn_items_capacity;
    at.row_splits = w.at<int32_t>(w.L.attn_row_splits);
    if (l == 0) {  // the list of attention workgroups is the same for every layer
      Tap t(&c->prof, MN_PROF_PREPARE, st);
      launch_attention_plan(at, st);
    }
    {
      Tap t(&c->prof, MN_PROF_ATTENTION, st);
      keep(launch_attention(at, st));
    }
    s = gemm_pick_split(M, d.d_model, hdim, d.dtype);
    gemm(at.out, c->wo[l], part, d.d_model, hdim, s);
    pend = part; pend_n = s; pend_bias = (const float*)c->bo[l];
    norm((const float*)c->ln2_g[l], (const float*)c->ln2_b[l], false);
    void* act = w.at<void>(w.L.act);
    if (llama && d.dtype == MN_DT_BF16) {
      // gate||up projection with silu(gate) * up applied in the kernel's epilogue
      GemmArgs g{};
      g.a = h; g.w = c->w1[l]; g.swiglu_act = act; g.M = M; g.N = w1r; g.K = d.d_model; g.split_k = 1; g.dtype = d.dtype;
      g.dev_status = dev_status;
      Tap t(&c->prof, MN_PROF_GEMM, st);
      keep(launch_gemm(g, st));
    } else if (!llama && d.dtype == MN_DT_BF16 && gemm_pick_split(M, w1r, d.d_model, d.dtype) == 1) {
      // one split: bias + ReLU applied in the kernel's epilogue, no partial sums and no activation kernel
      GemmArgs g{};
      g.a = h; g.w = c->w1[l]; g.relu_act = act; g.bias = (const float*)c->b1[l]; g.M = M; g.N = w1r; g.K = d.d_model;
      g.split_k = 1; g.dtype = d.dtype; g.dev_status = dev_status;
      Tap t(&c->prof, MN_PROF_GEMM, st);
      keep(launch_gemm(g, st));
    } else {
      s = gemm_pick_split(M, w1r, d.d_model, d.dtype);
      gemm(h, c->w1[l], part, w1r, d.d_model, s);
      ActArgs ac{};
      ac.partials = part; ac.n_partials = s; ac.bias = (const float*)c->b1[l]; ac.act = act;
      ac.M = M; ac.F = d.d_ffn; ac.swiglu = llama ? 1 : 0; ac.dtype = d.dtype; ac.dev_status = dev_status;
      Tap t(&c->prof, MN_PROF_ACT, st);
      launch_act(ac, st);
    }
    s = gemm_pick_split(M, d.d_model, d.d_ffn, d.dtype);
    gemm(act, c->w2[l], part, d.d_model, d.d_ffn, s);
    pend = part; pend_n = s; pend_bias = (const float*)c->b2[l];
  }
  norm((const float*)c->final_norm_g, (const float*)c->final_norm_b, d.n_layers == 0);
  float* lg = logits ? logits : w.at<float>(w.L.logits);
  {
    const int s = gemm_pick_split(M, d.vocab, d.d_model, d.dtype);
    if (s == 1) {
      gemm(h, c->lm_head, lg, d.vocab, d.d_model, 1);
    } else {
      gemm(h, c->lm_head, part, d.vocab, d.d_model, s);
      Tap t(&c->prof, MN_PROF_ARGMAX, st);
      launch_reduce_partials(part, s, (size_t)M * d.vocab, lg, (size_t)M * d.vocab, st);
    }
  }
  {
    Tap t(&c->prof, MN_PROF_ARGMAX, st);
    launch_argmax_rows(lg, M, d.vocab, rows, k_max, greedy, B, st);
  }
  if (lerr != hipSuccess) return fail(c, MN_EHIP, "%s: kernel attribute: %s", who, hipGetErrorString(lerr));
  return hip_check(c, who);
}

// ---- weight packing ---------------------------------------------------------------------------------
extern "C" size_t mn_packed_weight_bytes(int N, int K) {
  if (N < 1 || K < 128 || K % 128) return 0;
  return packed_weight_elems(N, K) * 2;
}

extern "C" mn_status mn_pack_weight(const void* src, void* dst, int N, int K, int interleave_half, int32_t* dev_status,
                                    void* stream) {
  if (N < 1 || K < 128 || K % 128) return fail(nullptr, MN_ESHAPE, "mn_pack_weight: N=%d K=%d (K must be a positive multiple of 128)", N, K);
  if (interleave_half < 0 || (interleave_half > 0 && (N != 2 * interleave_half || interleave_half % 16)))
    return fail(nullptr, MN_ESHAPE, "mn_pack_weight: interleave_half=%d needs N == 2*half and half %% 16 == 0", interleave_half);
  if (!src || !dst) return fail(nullptr, MN_ENULL, "mn_pack_weight: src/dst is NULL");
  if ((uintptr_t)dst & 255) return fail(nullptr, MN_EINVAL, "mn_pack_weight: dst not 256-byte aligned");
  launch_pack_weight(src, dst, N, K, interleave_half, dev_status, (hipStream_t)stream);
  return hip_check(nullptr, "mn_pack_weight");
}

// ---- component entry points -----------------------------------------------------------------------
extern "C" mn_status mn_proj_gemm(mn_ctx* c, const void* a, const void* w, const float* bias, float* out, int M, int N,
                                  int K, int split_k, void* workspace, size_t workspace_bytes, void* stream) {
  const char* who = "mn_proj_gemm";
  if (M < 0 || N < 1 || K < 128 || K % 128) return fail(c, MN_ESHAPE, "%s: M=%d N=%d K=%d (K must be a positive multiple of 128)", who, M, N, K);
  if (split_k < 0 || split_k > MN_MAX_SPLIT_K) return fail(c, MN_EINVAL, "%s: split_k = %d", who, split_k);
  if (M == 0) return MN_OK;
  if (!a || !w || !out) return fail(c, MN_ENULL, "%s: a/w/out is NULL", who);
  int s = split_k ? split_k : gemm_pick_split(M, N, K, MN_DT_BF16);
  if (s > K / 128) s = K / 128;
  hipStream_t st = (hipStream_t)stream;
  GemmArgs g{};
  g.a = a; g.w = w; g.bias = bias; g.M = M; g.N = N; g.K = K; g.split_k = s; g.dtype = MN_DT_BF16;
  Tap t(c ? &c->prof : nullptr, MN_PROF_GEMM, st);
  hipError_t lerr = hipSuccess;
  if (s == 1) {
    g.out = out;
    lerr = launch_gemm(g, st);
  } else {
    const size_t need = (size_t)s * M * N * 4;
    if (!workspace) return fail(c, MN_ENULL, "%s: workspace is NULL (split_k = %d)", who, s);
    if ((uintptr_t)workspace & 255) return fail(c, MN_EWORKSPACE, "%s: workspace not 256-byte aligned", who);
    if (workspace_bytes < need) return fail(c, MN_EWORKSPACE, "%s: workspace %zu bytes, need %zu", who, workspace_bytes, need);
    g.out = reinterpret_cast<float*>(workspace);
    lerr = launch_gemm(g, st);
    if (lerr == hipSuccess) launch_reduce_partials(g.out, s, (size_t)M * N, out, (size_t)M * N, st);
  }
  if (lerr != hipSuccess) return fail(c, MN_EHIP, "%s: kernel attribute: %s", who, hipGetErrorString(lerr));
  return hip_check(c, who);
}

// ---- the projection without a workspace argument ---------------------------------------------------
// For callers that can neither allocate nor bring device memory of their own (code under graph capture,
// tight serving loops): the split-K partial sums live in a buffer that is part of the library's code object.
// Each GPU the library runs on holds its own copy of the array at its own address; the name below is the
// host-side stand-in for it, never a device address: the address is looked up once per device and kept.
static __device__ __align__(256) unsigned char scratch[MN_NOALLOC_SCRATCH_BYTES];

static constexpr int kMaxDevices = 64;
static void* g_scratch_ptr[kMaxDevices];   // device address of `scratch` on device i, null until looked up
static std::mutex g_scratch_mu;

// Device address of this process's scratch array on the current device (looked up on the first call there).
static mn_status scratch_on_current_device(mn_ctx* c, const char* who, void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail(c, MN_EHIP, "%s: hipGetDevice: %s", who, hipGetErrorString(e));
  if (dev < 0 || dev >= kMaxDevices) return fail(c, MN_EUNSUPPORTED, "%s: device ordinal %d (at most %d devices)", who, dev, kMaxDevices);
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) return fail(c, MN_EHIP, "%s: hipGetSymbolAddress: %s", who, hipGetErrorString(e));
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return MN_OK;
}

extern "C" mn_status mn_proj_gemm_noalloc(mn_ctx* c, const void* a, const void* w, const float* bias, float* out, int M,
                                          int N, int K, int split_k, void* stream) {
  const char* who = "mn_proj_gemm_noalloc";
  if (M < 0 || N < 1 || K < 128 || K % 128) return fail(c, MN_ESHAPE, "%s: M=%d N=%d K=%d (K must be a positive multiple of 128)", who, M, N, K);
  if (split_k < 0 || split_k > MN_MAX_SPLIT_K) return fail(c, MN_EINVAL, "%s: split_k = %d", who, split_k);
  if (M == 0) return MN_OK;
  if (!a || !w || !out) return fail(c, MN_ENULL, "%s: a/w/out is NULL", who);
  int s = split_k ? split_k : gemm_pick_split(M, N, K, MN_DT_BF16);
  if (s > K / 128) s = K / 128;
  hipStream_t st = (hipStream_t)stream;
  GemmArgs g{};
  g.a = a; g.w = w; g.bias = bias; g.M = M; g.N = N; g.K = K; g.split_k = s; g.dtype = MN_DT_BF16;
  hipError_t lerr = hipSuccess;
  if (s == 1) {
    g.out = out;   // one split writes the result itself: no scratch in use
    Tap t(c ? &c->prof : nullptr, MN_PROF_GEMM, st);
    lerr = launch_gemm(g, st);
  } else {
    const size_t need = (size_t)s * M * N * 4;
    if (need > (size_t)MN_NOALLOC_SCRATCH_BYTES)
      return fail(c, MN_ECAPACITY, "%s: %d splits of %d x %d partial sums need %zu bytes, the built-in buffer holds %zu "
                  "(pass a smaller split_k, or use mn_proj_gemm with a workspace)", who, s, M, N, need,
                  (size_t)MN_NOALLOC_SCRATCH_BYTES);
    void* buf = nullptr;
    if (mn_status rc = scratch_on_current_device(c, who, &buf)) return rc;
    // Nothing has to start at zero: the projection kernel writes every element [split][m][n] the reduction reads
    // (a split without iterations stores zeros), so what an earlier call left behind is never seen.
    g.out = reinterpret_cast<float*>(buf);
    Tap t(c ? &c->prof : nullptr, MN_PROF_GEMM, st);
    lerr = launch_gemm(g, st);
    if (lerr == hipSuccess) launch_reduce_partials(g.out, s, (size_t)M * N, out, (size_t)M * N, st);
  }
  if (lerr != hipSuccess) return fail(c, MN_EHIP, "%s: kernel attribute: %s", who, hipGetErrorString(lerr));
  return hip_check(c, who);
}

extern "C" mn_status mn_attention(mn_ctx* c, const void* q, const int32_t* spec_len, const int32_t* h_spec_len, int B,
                                  int max_ctx, const mn_kv* kv, int layer, void* out, void* workspace,
                                  size_t workspace_bytes, int32_t* dev_status, void* stream) {
  const char* who = "mn_attention";
  if (!c) return MN_ENULL;
  if (B < 0 || B > MN_MAX_BATCH) return fail(c, MN_EINVAL, "%s: B = %d", who, B);
  if (max_ctx < 0) return fail(c, MN_EINVAL, "%s: max_ctx = %d", who, max_ctx);
  if (B == 0) return MN_OK;
  if (!q || !spec_len || !h_spec_len || !out) return fail(c, MN_ENULL, "%s: a required pointer is NULL", who);
  if (mn_status s = check_kv(c, kv, max_ctx, who)) return s;
  if (layer < 0 || layer >= (c->d.n_layers > 0 ? c->d.n_layers : 1)) return fail(c, MN_EINVAL, "%s: layer %d", who, layer);
  if (!kv->k_layers[layer] || !kv->v_layers[layer]) return fail(c, MN_ENULL, "%s: kv layer pointer is NULL", who);
  int k_max = 0;
  for (int b = 0; b < B; ++b) if (h_spec_len[b] > k_max) k_max = h_spec_len[b];
  int M = 0, max_q = 0;
  if (mn_status s = count_rows(c, h_spec_len, B, k_max, &M, &max_q, who)) return s;
  if (max_ctx < max_q) return fail(c, MN_EINVAL, "%s: max_ctx %d smaller than the longest scored run %d", who, max_ctx, max_q);
  if (!workspace) return fail(c, MN_ENULL, "%s: workspace is NULL", who);
  if ((uintptr_t)workspace & 255) return fail(c, MN_EWORKSPACE, "%s: workspace not 256-byte aligned", who);
  const mn_model_desc& d = c->d;
  Ws w{reinterpret_cast<unsigned char*>(workspace), make_layout(d, B, M, max_ctx)};
  if (workspace_bytes < w.L.total) return fail(c, MN_EWORKSPACE, "%s: workspace %zu bytes, need %zu", who, workspace_bytes, w.L.total);
  hipStream_t st = (hipStream_t)stream;
  // row bookkeeping only (no tokens): positions are ctx_b + j, the rows' K/V are already cached
  run_prepare(c, w, nullptr, nullptr, spec_len, B, k_max, M, max_ctx, kv, false, dev_status, st);
  AttnArgs at{};
  at.q = q; at.out = out; at.rows = row_info(w);
  at.kv = KvView{kv->k_layers[layer], kv->v_layers[layer], kv->block_tables, kv->block_size, kv->num_blocks, kv->max_blocks_per_seq};
  at.B = B; at.M = M; at.H = d.n_heads; at.Hkv = d.n_kv_heads; at.hd = d.head_dim; at.dtype = d.dtype;
  at.max_ctx = max_ctx; at.max_q = max_q;
  at.scratch = w.at<float>(w.L.attn_scratch); at.scratch_bytes = w.L.attn_scratch_bytes;
  at.items = w.at<int32_t>(w.L.attn_items); at.items_capacity = w.L.attn_items_capacity;
  at.row_splits = w.at<int32_t>(w.L.attn_row_splits);
  launch_attention_plan(at, st);
  hipError_t lerr = hipSuccess;
  {
    Tap t(&c->prof, MN_PROF_ATTENTION, st);
    lerr = launch_attention(at, st);
  }
  if (lerr != hipSuccess) return fail(c, MN_EHIP, "%s: kernel attribute: %s", who, hipGetErrorString(lerr));
  return hip_check(c, who);
}

// ---- timing taps ------------------------------------------------------------------------------------
extern "C" mn_status mn_profile_enable(mn_ctx* c, int on) {
  if (!c) return MN_ENULL;
  c->prof.on = on != 0;
  return MN_OK;
}

extern "C" mn_status mn_profile_collect(mn_ctx* c, double* ms, int* counts) {
  if (!c) return MN_ENULL;
  if (!ms || !counts) return fail(c, MN_ENULL, "mn_profile_collect: ms/counts is NULL");
  for (int k = 0; k < MN_PROF_KINDS; ++k) { ms[k] = 0.0; counts[k] = 0; }
  Prof& p = c->prof;
  mn_status rc = MN_OK;
  for (size_t i = 0; i < p.kind.size(); ++i) {
    float t = 0.f;
    const hipError_t e = hipEventElapsedTime(&t, p.pool[2 * i], p.pool[2 * i + 1]);
    if (e != hipSuccess) { rc = fail(c, MN_EHIP, "mn_profile_collect: %s (synchronise the stream first)", hipGetErrorString(e)); break; }
    ms[p.kind[i]] += t;
    counts[p.kind[i]] += 1;
  }
  p.kind.clear();
  p.used = 0;
  return rc;
}
