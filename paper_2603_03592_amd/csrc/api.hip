// C ABI of the stage verifier: context, workspace carving, and the launch sequences of the
// block forward (recompute of f_s) and of the input-gradient backward.  No tensor arithmetic
// happens on the host; the only host-computed table is the RoPE cos/sin table built once at
// sv_create.
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <vector>

#include "common.h"

using namespace sv;

namespace {

thread_local char g_create_error[256] = "";

struct BlockStash {   // what one block's backward reads (backward mode only)
  void *x1, *qkv, *o, *gate, *up;   // gate / up: pre-activations of the dense MLP, or of the shared experts
  float* lse;
  // mixture of experts: the routing and, in expert-sorted rows, the routed experts' pre-activations and outputs
  sv::MoeRoute route;
  void *gate_p, *up_p, *yp;
};

struct Arena {
  char* base = nullptr;
  size_t off = 0;
  void* take(size_t bytes) {
    off = (off + 255) & ~size_t(255);
    void* p = base ? base + off : nullptr;
    off += bytes;
    return p;
  }
};

constexpr int64_t kScoreScratchElems = 1 << 18;   // ScorePartial records (20 MiB)
constexpr int kSwMaxDirs = 128, kSwMaxClaims = 4096;
// Heads narrower than the matrix-core attention's widths (32, 64, 128) are zero-padded to the next one: 0 = no padding
inline int attn_pad_width(int hd) { return hd < 32 ? 32 : (hd > 32 && hd < 64 ? 64 : 0); }
constexpr int kSwSlots = 33;                      // projected tensors (kSwMaxDirs rows each) the scratch holds at max_tokens

}  // namespace

struct sv_ctx {
  sv_stage_desc d;
  uint32_t flags;
  int64_t max_tokens;
  int32_t max_seq;
  int device;
  int es;            // element size of the stage dtype
  int hd, Dq, Dkv, Dqkv;
  bool moe;          // mixture-of-experts MLP
  int Fd;            // width of the dense-path MLP: ffn_hidden, or ffn_shared (possibly 0) for a mixture of experts
  void* ws;
  size_t ws_bytes;
  // forward
  void *xbuf[2], *n, *qkv, *o, *x1, *act;
  float* lse;
  // mixture of experts (expert-sorted rows, moe_padded_rows(max_tokens) of them)
  MoeRoute route;      // forward-only contexts: one routing, reused by every block
  void *xp, *actp, *yp, *dup_p;
  // heads narrower than the matrix-core attention kernels' 64 columns: zero-padded copies [T, heads * 64]
  void *qkv_pad, *o_pad, *dout_pad, *dqkv_pad;
  int pad_hd;          // width the heads are padded to for the matrix-core attention (0: none)
  int last_T = 0;      // tokens of the most recent verify call (for sv_last_routing)
  // backward
  std::vector<void*> xs;           // outputs of blocks 0..L-2 (inputs of blocks 1..L-1)
  std::vector<BlockStash> stash;
  void *dres[2], *dn, *dx1, *dgate, *dup, *dout, *dqkv;
  struct WT { void *wq, *wk, *wv, *wo, *wg, *wu, *wd, *wsg, *wsu, *wsd; };
  std::vector<WT> wT;                   // per block: the weights transposed to [in, out] (bf16 MFMA path, backward mode)
  std::vector<sv_block_weights> prepared;   // the weights sv_prepare_weights transposed (empty: none)
  // RMSNorm inside the neighbouring products (SV_FLAG_FUSE_NORM, bf16 matrix-core path): per block the [out, in] weights
  // that follow a norm with its gain folded in, the rows' 1 / rms, and the partial sums of squares that the product which
  // writes a residual stream leaves for the norm that reads it (rowsq_of: the stream they belong to)
  struct WF { void *wq, *wk, *wv, *wg, *wu; };
  std::vector<WF> wF;
  float* rstd = nullptr;
  float* rowsq = nullptr;
  int rowsq_planes = 0;   // d_model / 128
  const void* rowsq_of = nullptr;
  float* delta;
  ScorePartial* score_scratch;
  float* attn_part;    // fp32 dk | dv contributions per query head of a group (backward, bf16 matrix-core path, one long sequence)
  size_t attn_part_floats;
  float* split_ws;     // fp32 partial products of the split-k GEMMs (bf16 matrix-core path, few tokens against a long k)
  size_t split_ws_floats;
  float* sw_w1;        // [kSwMaxClaims, kSwMaxDirs] per-direction sums (SV_FLAG_SLICED_W)
  float* sw_proj;      // kSwSlots * kSwMaxDirs rows of sw_padded_len(max_tokens) floats
  size_t sw_proj_floats;
  float* rope_cs;
  char err[256];
  // optional per-operation event timing
  bool prof_on = false;
  uint64_t prof_mask = ~0ull;   // operation classes that are bracketed while prof_on (sv_profile_select)
  struct ProfRec { int op; hipEvent_t a, b; };
  std::vector<ProfRec> prof_recs;
  std::vector<hipEvent_t> prof_pool;
  sv_profile prof_acc;
};

// error text of calls that take no context (read back through sv_last_error(NULL) on the same thread)
void sv::set_global_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_create_error, sizeof(g_create_error), fmt, ap);
  va_end(ap);
}

namespace {

void set_err(sv_ctx* c, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(c ? c->err : g_create_error, 256, fmt, ap);
  va_end(ap);
}

sv_status check_desc_impl(const sv_stage_desc* d, uint32_t flags, char* msg, int msg_len) {
  auto fail = [&](sv_status s, const char* m) {
    if (msg && msg_len > 0) snprintf(msg, (size_t)msg_len, "%s", m);
    return s;
  };
  if (!d) return fail(SV_EINVAL, "descriptor is NULL");
  if (d->n_blocks < 1 || d->d_model < 1 || d->n_heads < 1 || d->n_kv_heads < 1 || d->ffn_hidden < 1)
    return fail(SV_EINVAL, "n_blocks, d_model, n_heads, n_kv_heads and ffn_hidden must be positive");
  if (d->mlp != SV_MLP_GELU && d->mlp != SV_MLP_SWIGLU) return fail(SV_EINVAL, "unknown mlp kind");
  if (d->norm != SV_NORM_LN && d->norm != SV_NORM_RMS) return fail(SV_EINVAL, "unknown norm kind");
  if (d->dtype != SV_F32 && d->dtype != SV_BF16) return fail(SV_EINVAL, "unknown dtype");
  if (!(d->norm_eps >= 0.0f)) return fail(SV_EINVAL, "norm_eps must be >= 0");
  if (d->rope && !(d->rope_theta > 0.0f)) return fail(SV_EINVAL, "rope_theta must be > 0");
  if (flags & ~(uint32_t)(SV_FLAG_BACKWARD | SV_FLAG_PLAIN_KERNELS | SV_FLAG_SLICED_W | SV_FLAG_FUSE_NORM)) return fail(SV_EINVAL, "unknown flag bits");
  if (d->d_model % d->n_heads) return fail(SV_EINVAL, "d_model must be a multiple of n_heads");
  if (d->n_heads % d->n_kv_heads) return fail(SV_EINVAL, "n_heads must be a multiple of n_kv_heads");
  const int hd = d->d_model / d->n_heads;
  if (hd != 8 && hd != 16 && hd != 32 && hd != 64 && hd != 128)
    return fail(SV_EUNSUPPORTED, "head_dim must be one of 8, 16, 32, 64, 128");
  if (d->d_model % 8 || d->ffn_hidden % 8) return fail(SV_EUNSUPPORTED, "d_model and ffn_hidden must be multiples of 8");
  if (d->n_experts < 0 || d->ffn_shared < 0) return fail(SV_EINVAL, "n_experts and ffn_shared must be >= 0");
  if (d->n_experts == 0 && (d->top_k || d->ffn_shared || d->router_score || d->router_norm))
    return fail(SV_EINVAL, "top_k, ffn_shared, router_score and router_norm must be 0 for a dense MLP");
  if (d->n_experts > 0) {
    if (d->mlp != SV_MLP_SWIGLU) return fail(SV_EUNSUPPORTED, "a mixture of experts needs the SwiGLU MLP");
    if (d->top_k < 1 || d->top_k > d->n_experts) return fail(SV_EINVAL, "top_k must be in 1..n_experts");
    if (d->router_score != SV_ROUTER_SIGMOID && d->router_score != SV_ROUTER_SOFTMAX) return fail(SV_EINVAL, "unknown router_score");
    if (d->router_norm != 0 && d->router_norm != 1) return fail(SV_EINVAL, "router_norm must be 0 or 1");
    if (d->n_experts > kMoeMaxExperts || d->top_k > kMoeMaxTopK) return fail(SV_EUNSUPPORTED, "at most 16 experts and top_k <= 8");
    if (d->ffn_shared % 8) return fail(SV_EUNSUPPORTED, "ffn_shared must be a multiple of 8");
  }
  if (msg && msg_len > 0) msg[0] = 0;
  return SV_OK;
}

// Carve (or, with a null base, just size) the workspace.
size_t carve(sv_ctx* c, char* base) {
  const sv_stage_desc& d = c->d;
  const size_t T = (size_t)c->max_tokens, es = (size_t)c->es;
  const size_t D = d.d_model, F = d.ffn_hidden, L = d.n_blocks;
  const size_t Fd = (size_t)c->Fd;                     // dense-path MLP width (the shared experts of a mixture)
  const size_t E = d.n_experts, K = d.top_k;
  const size_t Mp = c->moe ? (size_t)moe_padded_rows(c->max_tokens, d.top_k, d.n_experts) : 0;
  const size_t lse_n = (size_t)d.n_heads * T;
  const bool bwd = c->flags & SV_FLAG_BACKWARD;
  Arena a; a.base = base;
  c->rope_cs = (float*)a.take((size_t)c->max_seq * (c->hd / 2) * 2 * sizeof(float));
  c->score_scratch = (ScorePartial*)a.take(kScoreScratchElems * sizeof(ScorePartial));
  c->split_ws = nullptr; c->split_ws_floats = 0;
  if (d.dtype == SV_BF16 && !(c->flags & SV_FLAG_PLAIN_KERNELS)) {
    // up to 8 partial products of the widest product a split can serve (below 160 tiles of 128 x 128, or below 192 tiles
    // of 256 x 256 with as many runs as this holds), and no more than this context's token bound allows
    const size_t widest = std::max(std::max(D, (size_t)c->Dq), std::max(Fd, (size_t)d.ffn_hidden));
    c->split_ws_floats = std::min((size_t)8 * 160 * 128 * 128, (size_t)8 * T * widest);
    c->split_ws = (float*)a.take(c->split_ws_floats * sizeof(float));
  }
  c->attn_part = nullptr; c->attn_part_floats = 0;
  if (bwd && d.dtype == SV_BF16 && !(c->flags & SV_FLAG_PLAIN_KERNELS) && d.n_heads > d.n_kv_heads) {
    // the head split is taken below kDkvSplitWorkgroups workgroups of at most 128 keys per (batch, kv head), i.e. below
    // that many times 128 / Hkv tokens per call
    const size_t tcap = std::min(T, (size_t)kDkvSplitWorkgroups * 128 / (size_t)d.n_kv_heads);
    const size_t hd_eff = attn_pad_width(c->hd) ? (size_t)attn_pad_width(c->hd) : (size_t)c->hd;   // narrow heads run zero-padded
    c->attn_part_floats = (size_t)(d.n_heads / d.n_kv_heads) * tcap * 2 * (size_t)d.n_kv_heads * hd_eff;
    c->attn_part = (float*)a.take(c->attn_part_floats * sizeof(float));
  }
  c->sw_w1 = nullptr; c->sw_proj = nullptr; c->sw_proj_floats = 0;
  if (c->flags & SV_FLAG_SLICED_W) {
    c->sw_w1 = (float*)a.take((size_t)kSwMaxClaims * kSwMaxDirs * sizeof(float));
    c->sw_proj_floats = (size_t)kSwSlots * kSwMaxDirs * (size_t)sw_padded_len(c->max_tokens);
    c->sw_proj = (float*)a.take(c->sw_proj_floats * sizeof(float));
  }
  c->wF.clear(); c->rstd = nullptr; c->rowsq = nullptr; c->rowsq_planes = 0;
  if ((c->flags & SV_FLAG_FUSE_NORM) && d.dtype == SV_BF16 && d.norm == SV_NORM_RMS && !(c->flags & SV_FLAG_PLAIN_KERNELS)) {
    c->rstd = (float*)a.take(T * sizeof(float));
    c->rowsq_planes = (int)((D + 127) / 128);
    c->rowsq = (float*)a.take(T * c->rowsq_planes * sizeof(float));
    for (size_t l = 0; l < L; ++l) {
      sv_ctx::WF f{};
      f.wq = a.take(D * c->Dq * es); f.wk = a.take(D * c->Dkv * es); f.wv = a.take(D * c->Dkv * es);
      if (!c->moe) {                                   // a mixture's second norm also feeds its router: it stays a pass of its own
        f.wu = a.take(D * F * es);
        f.wg = d.mlp == SV_MLP_SWIGLU ? a.take(D * F * es) : nullptr;
      }
      c->wF.push_back(f);
    }
  }
  c->xbuf[0] = a.take(T * D * es);
  c->xbuf[1] = a.take(T * D * es);
  c->n = a.take(T * D * es);
  c->act = a.take(T * Fd * es);
  auto take_route = [&](MoeRoute& r) {
    const size_t n_chunks = (T * K + kMoeChunk - 1) / kMoeChunk;
    r.sel = (int32_t*)a.take(T * K * 4); r.gate = (float*)a.take(T * K * 4); r.score = (float*)a.take(T * E * 4);
    r.pos = (int32_t*)a.take(T * K * 4); r.row_token = (int32_t*)a.take(Mp * 4); r.row_gate = (float*)a.take(Mp * 4);
    r.tile_expert = (int32_t*)a.take(Mp / 256 * 4); r.meta = (int32_t*)a.take((1 + 2 * E) * 4);
    r.chunk_counts = (int32_t*)a.take(n_chunks * E * 4); r.chunk_base = (int32_t*)a.take(n_chunks * E * 4);
  };
  c->xp = c->actp = c->yp = c->dup_p = nullptr;
  if (c->moe) {
    c->xp = a.take(Mp * D * es);
    c->actp = a.take(Mp * F * es);
    if (!bwd) { take_route(c->route); c->yp = a.take(Mp * D * es); }
    else c->dup_p = a.take(Mp * F * es);
  }
  c->qkv_pad = c->o_pad = c->dout_pad = c->dqkv_pad = nullptr;
  c->pad_hd = 0;
  if (d.dtype == SV_BF16 && !(c->flags & SV_FLAG_PLAIN_KERNELS) && attn_pad_width(c->hd)) {
    c->pad_hd = attn_pad_width(c->hd);
    const size_t hq = (size_t)d.n_heads * c->pad_hd, hall = (size_t)(d.n_heads + 2 * d.n_kv_heads) * c->pad_hd;
    c->qkv_pad = a.take(T * hall * es);
    c->o_pad = a.take(T * hq * es);
    if (bwd) { c->dout_pad = a.take(T * hq * es); c->dqkv_pad = a.take(T * hall * es); }
  }
  c->xs.clear(); c->stash.clear();
  if (!bwd) {
    c->qkv = a.take(T * c->Dqkv * es);
    c->o = a.take(T * c->Dq * es);
    c->x1 = a.take(T * D * es);
    c->lse = (float*)a.take(lse_n * sizeof(float));
  } else {
    for (size_t l = 0; l + 1 < L; ++l) c->xs.push_back(a.take(T * D * es));
    for (size_t l = 0; l < L; ++l) {
      BlockStash s;
      s.x1 = a.take(T * D * es);
      s.qkv = a.take(T * c->Dqkv * es);
      s.o = a.take(T * c->Dq * es);
      s.gate = d.mlp == SV_MLP_SWIGLU ? a.take(T * Fd * es) : nullptr;
      s.up = a.take(T * Fd * es);
      s.lse = (float*)a.take(lse_n * sizeof(float));
      s.gate_p = s.up_p = s.yp = nullptr;
      if (c->moe) {
        take_route(s.route);
        s.gate_p = a.take(Mp * F * es); s.up_p = a.take(Mp * F * es); s.yp = a.take(Mp * D * es);
      }
      c->stash.push_back(s);
    }
    c->qkv = c->stash[0].qkv; c->o = c->stash[0].o; c->x1 = c->stash[0].x1; c->lse = c->stash[0].lse;
    c->dres[0] = a.take(T * D * es);
    c->dres[1] = a.take(T * D * es);
    c->dn = a.take(T * D * es);
    c->dx1 = a.take(T * D * es);
    c->dgate = a.take(T * Fd * es);
    c->dup = d.mlp == SV_MLP_SWIGLU ? a.take(T * Fd * es) : nullptr;
    c->dout = a.take(T * c->Dq * es);
    c->dqkv = a.take(T * c->Dqkv * es);
    c->delta = (float*)a.take(lse_n * sizeof(float));
    c->wT.clear();
    if (d.dtype == SV_BF16 && !(c->flags & SV_FLAG_PLAIN_KERNELS)) {
      for (size_t l = 0; l < L; ++l) {
        sv_ctx::WT t;
        t.wq = a.take(D * c->Dq * es); t.wk = a.take(D * c->Dkv * es); t.wv = a.take(D * c->Dkv * es);
        const size_t ne = c->moe ? E : 1;              // routed experts one after the other
        t.wo = a.take(D * c->Dq * es); t.wu = a.take(ne * D * F * es); t.wd = a.take(ne * D * F * es);
        t.wg = d.mlp == SV_MLP_SWIGLU ? a.take(ne * D * F * es) : nullptr;
        t.wsg = t.wsu = t.wsd = nullptr;
        if (c->moe && Fd) { t.wsg = a.take(D * Fd * es); t.wsu = a.take(D * Fd * es); t.wsd = a.take(D * Fd * es); }
        c->wT.push_back(t);
      }
    }
  }
  return a.off + 256;
}

void init_ctx_fields(sv_ctx* c, const sv_stage_desc* desc, int64_t max_tokens, int32_t max_seq, uint32_t flags) {
  c->d = *desc; c->flags = flags; c->max_tokens = max_tokens; c->max_seq = max_seq;
  c->es = desc->dtype == SV_BF16 ? 2 : 4;
  c->hd = desc->d_model / desc->n_heads;
  c->Dq = desc->n_heads * c->hd;
  c->Dkv = desc->n_kv_heads * c->hd;
  c->Dqkv = c->Dq + 2 * c->Dkv;
  c->moe = desc->n_experts > 0;
  c->Fd = c->moe ? desc->ffn_shared : desc->ffn_hidden;
  c->ws = nullptr; c->ws_bytes = 0; c->err[0] = 0;
}

#define SV_HIP(c, call)                                                        \
  do {                                                                         \
    hipError_t e_ = (call);                                                    \
    if (e_ != hipSuccess) {                                                    \
      set_err(c, "%s failed: %s", #call, hipGetErrorString(e_));               \
      return SV_EHIP;                                                          \
    }                                                                          \
  } while (0)

// Launch `call` for operation class `op`; with profiling on, bracket it with events on `st`.
#define SV_OP(c, op, flop_, st, call)                                          \
  do {                                                                         \
    hipEvent_t ea_ = nullptr, eb_ = nullptr;                                   \
    const bool prof_ = (c)->prof_on && (((c)->prof_mask >> (op)) & 1);         \
    if (prof_) {                                                               \
      ea_ = take_event(c); eb_ = take_event(c);                                \
      if (!ea_ || !eb_) { set_err(c, "hipEventCreate failed"); return SV_EHIP; } \
      SV_HIP(c, hipEventRecord(ea_, st));                                      \
    }                                                                          \
    SV_HIP(c, call);                                                           \
    if (prof_) {                                                               \
      SV_HIP(c, hipEventRecord(eb_, st));                                      \
      (c)->prof_recs.push_back(sv_ctx::ProfRec{op, ea_, eb_});                 \
      (c)->prof_acc.flop[op] += (double)(flop_);                               \
      (c)->prof_acc.launches[op] += 1;                                         \
    }                                                                          \
  } while (0)

hipEvent_t take_event(sv_ctx* c) {
  if (!c->prof_pool.empty()) { hipEvent_t e = c->prof_pool.back(); c->prof_pool.pop_back(); return e; }
  hipEvent_t e = nullptr;
  if (hipEventCreate(&e) != hipSuccess) return nullptr;
  return e;
}

inline char* at(void* p, int64_t elems, int es) { return (char*)p + elems * es; }
inline const char* at(const void* p, int64_t elems, int es) { return (const char*)p + elems * es; }

hipError_t gemm(sv_ctx* c, const GemmArgs& a, hipStream_t st) {
  if (c->d.dtype == SV_BF16 && !(c->flags & SV_FLAG_PLAIN_KERNELS) && mfma_gemm_supported(a)) {
    GemmArgs g = a;
    g.split_ws = c->split_ws; g.split_ws_floats = (int64_t)c->split_ws_floats;
    return mfma_gemm(g, st);
  }
  return plain_gemm(a, c->d.dtype, st);
}

// Heads of 8, 16 or 32 columns run on the 64-column matrix-core kernels through zero-padded copies (the products are
// unchanged by zero columns; the softmax scale stays 1/sqrt(hd)); three quarters or more of those MFMAs multiply zeros,
// which is still several times faster than the scalar kernels.
bool attn_padded(const sv_ctx* c, int S) {
  const sv_stage_desc& d = c->d;
  return c->qkv_pad != nullptr && mfma_attn_supported(S, d.n_heads, d.n_kv_heads, c->pad_hd, (int64_t)(d.n_heads + 2 * d.n_kv_heads) * c->pad_hd);
}

hipError_t attn_fwd(sv_ctx* c, const void* qkv, void* o, float* lse, int B, int S, hipStream_t st) {
  const sv_stage_desc& d = c->d;
  if (d.dtype == SV_BF16 && !(c->flags & SV_FLAG_PLAIN_KERNELS) && mfma_attn_supported(S, d.n_heads, d.n_kv_heads, c->hd, c->Dqkv))
    return mfma_attn_fwd(qkv, c->Dqkv, o, lse, B, S, d.n_heads, d.n_kv_heads, c->hd, d.causal, st);
  if (attn_padded(c, S)) {
    const int64_t T = (int64_t)B * S, ldp = (int64_t)(d.n_heads + 2 * d.n_kv_heads) * c->pad_hd, ldo = (int64_t)d.n_heads * c->pad_hd;
    hipError_t e = plain_pad_heads(qkv, c->Dqkv, c->qkv_pad, ldp, T, d.n_heads + 2 * d.n_kv_heads, c->hd, c->pad_hd, 1, st);
    if (e == hipSuccess) e = mfma_attn_fwd(c->qkv_pad, ldp, c->o_pad, lse, B, S, d.n_heads, d.n_kv_heads, c->pad_hd, d.causal, st, c->hd);
    if (e == hipSuccess) e = plain_pad_heads(c->o_pad, ldo, o, c->Dq, T, d.n_heads, c->hd, c->pad_hd, 0, st);
    return e;
  }
  return plain_attn_fwd(qkv, c->Dqkv, o, lse, B, S, d.n_heads, d.n_kv_heads, c->hd, d.causal, d.dtype, st);
}

bool attn_on_mfma(const sv_ctx* c, int S) {
  const sv_stage_desc& d = c->d;
  return d.dtype == SV_BF16 && !(c->flags & SV_FLAG_PLAIN_KERNELS) && mfma_attn_supported(S, d.n_heads, d.n_kv_heads, c->hd, c->Dqkv);
}

// the MFMA kernels also undo RoPE on dq, dk; the plain ones (and the padded form) leave that to a separate pass
hipError_t attn_bwd(sv_ctx* c, const BlockStash& k, int B, int S, hipStream_t st) {
  const sv_stage_desc& d = c->d;
  if (attn_on_mfma(c, S))
    return mfma_attn_bwd(k.qkv, c->Dqkv, k.o, c->dout, k.lse, c->delta, c->dqkv, B, S, d.n_heads, d.n_kv_heads, c->hd, d.causal,
                         d.rope ? c->rope_cs : nullptr, st, 0, c->attn_part, (int64_t)c->attn_part_floats);
  if (attn_padded(c, S) && c->dout_pad) {
    const int nh = d.n_heads + 2 * d.n_kv_heads;
    const int64_t T = (int64_t)B * S, ldp = (int64_t)nh * c->pad_hd, ldo = (int64_t)d.n_heads * c->pad_hd;
    hipError_t e = plain_pad_heads(k.qkv, c->Dqkv, c->qkv_pad, ldp, T, nh, c->hd, c->pad_hd, 1, st);
    if (e == hipSuccess) e = plain_pad_heads(k.o, c->Dq, c->o_pad, ldo, T, d.n_heads, c->hd, c->pad_hd, 1, st);
    if (e == hipSuccess) e = plain_pad_heads(c->dout, c->Dq, c->dout_pad, ldo, T, d.n_heads, c->hd, c->pad_hd, 1, st);
    if (e == hipSuccess)
      e = mfma_attn_bwd(c->qkv_pad, ldp, c->o_pad, c->dout_pad, k.lse, c->delta, c->dqkv_pad, B, S, d.n_heads, d.n_kv_heads, c->pad_hd, d.causal,
                        nullptr, st, c->hd, c->attn_part, (int64_t)c->attn_part_floats);
    if (e == hipSuccess) e = plain_pad_heads(c->dqkv_pad, ldp, c->dqkv, c->Dqkv, T, nh, c->hd, c->pad_hd, 0, st);
    return e;
  }
  return plain_attn_bwd(k.qkv, c->Dqkv, k.o, c->dout, k.lse, c->delta, c->dqkv, B, S, d.n_heads, d.n_kv_heads, c->hd, d.causal, d.dtype, st);
}

GemmArgs nt(int M, int N, int K, const void* A, int64_t lda, const void* W, void* C, int64_t ldc, int epi) {
  GemmArgs g; memset(&g, 0, sizeof(g));
  g.M = M; g.N = N; g.nseg = 1; g.seg[0] = GemmSeg{A, lda, W, (int64_t)K, K};
  g.b_is_kn = 0; g.epi = epi; g.C = C; g.ldc = ldc;
  return g;
}

// One block forward: x -> y.  keep (nullable) receives what backward needs.  Mixture-of-experts blocks write their routing
// record and the expert outputs to keep's, else to `route` / `route_yp` (which the caller picks: the context's single
// record on a forward-only context, block l's own on a backward context, so that sv_last_routing reads what ran last).
// The weights that follow the two norms of a block, with the norm's gain folded in: W'[n][k] = W[n][k] g[k].
sv_status fold_block_weights(sv_ctx* c, const sv_block_weights& w, const sv_ctx::WF& f, hipStream_t st) {
  const sv_stage_desc& d = c->d;
  const int D = d.d_model, F = d.ffn_hidden;
  SV_OP(c, SV_OP_NORM_PIECES, 0, st, fold_gain(w.wq, w.norm1_g, f.wq, c->Dq, D, st));
  SV_OP(c, SV_OP_NORM_PIECES, 0, st, fold_gain(w.wk, w.norm1_g, f.wk, c->Dkv, D, st));
  SV_OP(c, SV_OP_NORM_PIECES, 0, st, fold_gain(w.wv, w.norm1_g, f.wv, c->Dkv, D, st));
  if (f.wu) SV_OP(c, SV_OP_NORM_PIECES, 0, st, fold_gain(w.w_up, w.norm2_g, f.wu, F, D, st));
  if (f.wg) SV_OP(c, SV_OP_NORM_PIECES, 0, st, fold_gain(w.w_gate, w.norm2_g, f.wg, F, D, st));
  return SV_OK;
}

// l: the block's index (its folded weights), or -1 for weights that have none
sv_status block_forward(sv_ctx* c, int l, const sv_block_weights& w, const void* x, void* y, int B, int S, BlockStash* keep, hipStream_t st,
                        const MoeRoute* route = nullptr, void* route_yp = nullptr) {
  const sv_stage_desc& d = c->d;
  const int T = B * S, D = d.d_model, F = d.ffn_hidden, es = c->es, dt = d.dtype;
  void* qkv = keep ? keep->qkv : c->qkv;
  void* o = keep ? keep->o : c->o;
  void* x1 = keep ? keep->x1 : c->x1;
  float* lse = keep ? keep->lse : c->lse;

  // RMSNorm inside the products: the product after a norm reads the residual stream itself, against weights that carry the
  // gain, and scales its rows by their 1 / rms; that comes from the sums of squares the product which wrote the stream
  // left behind, or from one read of the stream (the stage input; streams written by the small-tile kernels).
  const bool fuse = !c->wF.empty() && l >= 0;
  sv_ctx::WF wf{};
  if (fuse) {
    wf = c->wF[l];
    const bool ready = (int)c->prepared.size() == d.n_blocks && memcmp(&c->prepared[l], &w, sizeof(w)) == 0;
    if (!ready) {
      sv_status s = fold_block_weights(c, w, wf, st);
      if (s != SV_OK) return s;
    }
  }
  auto row_rstd = [&](const void* stream) -> sv_status {
    if (c->rowsq_of == stream) SV_OP(c, SV_OP_NORM_PIECES, 0, st, rms_rstd_from_partials(c->rowsq, c->rowsq_planes, T, c->rstd, T, D, d.norm_eps, st));
    else SV_OP(c, SV_OP_NORM_PIECES, 0, st, rms_rstd(stream, c->rstd, T, D, d.norm_eps, st));
    return SV_OK;
  };
  // a product that writes a residual stream leaves the sums of squares of its rows when the kernel it runs on can
  auto leave_rowsq = [&](GemmArgs& g) {
    c->rowsq_of = nullptr;
    if (!fuse) return;
    g.rowsq = c->rowsq; g.rowsq_ld = T;                // planes of T floats
    if (dt == SV_BF16 && !(c->flags & SV_FLAG_PLAIN_KERNELS) && mfma_gemm_emits_rowsq(g)) c->rowsq_of = g.C;
    else { g.rowsq = nullptr; g.rowsq_ld = 0; }
  };

  const double Td = T, attn_flop = (d.causal ? 2.0 : 4.0) * B * d.n_heads * (double)S * S * c->hd;
  bool fused1 = false;
  if (fuse) {
    GemmArgs f = nt(T, c->Dqkv, D, x, D, wf.wq, qkv, c->Dqkv, d.rope ? EPI_ROPE : EPI_STORE);
    f.nbcol = 3; f.Bcol[0] = wf.wq; f.Bcol[1] = wf.wk; f.Bcol[2] = wf.wv; f.ncol[0] = c->Dq; f.ncol[1] = c->Dkv; f.ncol[2] = c->Dkv;
    f.rope_cs = c->rope_cs; f.rope_S = S; f.rope_hd = c->hd; f.rope_cols = c->Dq + c->Dkv;
    f.rscale = c->rstd;
    f.split_ws = c->split_ws; f.split_ws_floats = (int64_t)c->split_ws_floats;   // few tokens: runs of k slices per tile
    if (mfma_gemm_supported(f)) {                      // the one-launch q | k | v product: the large tile (whole, or over runs of k slices)
      sv_status s = row_rstd(x);
      if (s != SV_OK) return s;
      SV_OP(c, SV_OP_GEMM_QKV, 2.0 * Td * c->Dqkv * D, st, mfma_gemm(f, st));
      fused1 = true;
    }
  }
  if (!fused1) {
    SV_OP(c, SV_OP_NORM, 0, st, plain_norm_fwd(x, w.norm1_g, w.norm1_b, c->n, T, D, d.norm, d.norm_eps, dt, st));
    // one launch over the concatenated [q | k | v] columns with RoPE in the epilogue when the kernel can do it
    GemmArgs f = nt(T, c->Dqkv, D, c->n, D, w.wq, qkv, c->Dqkv, d.rope ? EPI_ROPE : EPI_STORE);
    f.nbcol = 3; f.Bcol[0] = w.wq; f.Bcol[1] = w.wk; f.Bcol[2] = w.wv; f.ncol[0] = c->Dq; f.ncol[1] = c->Dkv; f.ncol[2] = c->Dkv;
    f.rope_cs = c->rope_cs; f.rope_S = S; f.rope_hd = c->hd; f.rope_cols = c->Dq + c->Dkv;
    f.split_ws = c->split_ws; f.split_ws_floats = (int64_t)c->split_ws_floats;
    if (dt == SV_BF16 && !(c->flags & SV_FLAG_PLAIN_KERNELS) && mfma_gemm_supported(f)) {
      SV_OP(c, SV_OP_GEMM_QKV, 2.0 * Td * c->Dqkv * D, st, mfma_gemm(f, st));
    } else {
      SV_OP(c, SV_OP_GEMM_QKV, 2.0 * Td * c->Dq * D, st, gemm(c, nt(T, c->Dq, D, c->n, D, w.wq, qkv, c->Dqkv, EPI_STORE), st));
      SV_OP(c, SV_OP_GEMM_QKV, 2.0 * Td * c->Dkv * D, st, gemm(c, nt(T, c->Dkv, D, c->n, D, w.wk, at(qkv, c->Dq, es), c->Dqkv, EPI_STORE), st));
      SV_OP(c, SV_OP_GEMM_QKV, 2.0 * Td * c->Dkv * D, st, gemm(c, nt(T, c->Dkv, D, c->n, D, w.wv, at(qkv, c->Dq + c->Dkv, es), c->Dqkv, EPI_STORE), st));
      if (d.rope) SV_OP(c, SV_OP_ROPE, 0, st, plain_rope(qkv, c->Dqkv, T, S, d.n_heads, d.n_kv_heads, c->hd, c->rope_cs, 0, dt, st));
    }
  }
  SV_OP(c, SV_OP_ATTN, attn_flop, st, attn_fwd(c, qkv, o, lse, B, S, st));
  // the second norm runs inside the MLP's first product when that product can scale its rows
  GemmArgs up{};
  bool fused2 = false;
  if (fuse && !c->moe) {
    if (d.mlp == SV_MLP_SWIGLU) { up = nt(T, F, D, x1, D, wf.wg, c->act, F, EPI_SWIGLU); up.B2 = wf.wu; up.ldb2 = D; }
    else up = nt(T, F, D, x1, D, wf.wu, c->act, F, EPI_GELU);
    up.rscale = c->rstd;
    fused2 = mfma_gemm_supported(up);
  }
  {
    GemmArgs g = nt(T, D, c->Dq, o, c->Dq, w.wo, x1, D, EPI_RESID);
    g.R = x; g.ldr = D;
    if (fused2) leave_rowsq(g); else c->rowsq_of = nullptr;
    SV_OP(c, SV_OP_GEMM_O, 2.0 * Td * D * c->Dq, st, gemm(c, g, st));
  }
  if (fused2) {
    sv_status s = row_rstd(x1);
    if (s != SV_OK) return s;
    if (d.mlp == SV_MLP_SWIGLU) {
      if (keep) { up.C2 = keep->gate; up.C3 = keep->up; }
      SV_OP(c, SV_OP_GEMM_GATEUP, 4.0 * Td * F * D, st, gemm(c, up, st));
    } else {
      if (keep) up.C2 = keep->up;
      SV_OP(c, SV_OP_GEMM_GATEUP, 2.0 * Td * F * D, st, gemm(c, up, st));
    }
    GemmArgs g = nt(T, D, F, c->act, F, w.w_down, y, D, EPI_RESID);
    g.R = x1; g.ldr = D;
    if (l + 1 < d.n_blocks) leave_rowsq(g);            // for the first norm of the next block
    else c->rowsq_of = nullptr;
    SV_OP(c, SV_OP_GEMM_DOWN, 2.0 * Td * D * F, st, gemm(c, g, st));
    return SV_OK;
  }
  c->rowsq_of = nullptr;
  SV_OP(c, SV_OP_NORM, 0, st, plain_norm_fwd(x1, w.norm2_g, w.norm2_b, c->n, T, D, d.norm, d.norm_eps, dt, st));
  if (c->moe) {
    // shared experts on the dense path (their output lands in y on top of the residual), then the routed experts:
    // route, gather the token rows expert by expert, two grouped products, weighted sum back into token order
    const int E = d.n_experts, K = d.top_k, Fs = d.ffn_shared;
    const MoeRoute& r = keep ? keep->route : (route ? *route : c->route);
    void* yp = keep ? keep->yp : (route ? route_yp : c->yp);
    // every launch below dereferences these: a context that did not carve them must never get here
    if (!r.sel || !r.gate || !r.score || !r.pos || !r.row_token || !r.row_gate || !r.tile_expert || !r.meta || !r.chunk_counts ||
        !r.chunk_base || !yp || !c->xp || !c->actp) {
      set_err(c, "internal: the routing record of this block was not allocated");
      return SV_EINVAL;
    }
    const int64_t Mp = moe_padded_rows(T, K, E);
    const double rows = Td * K;
    const void* base = x1;
    if (Fs > 0) {
      GemmArgs g = nt(T, Fs, D, c->n, D, w.ws_gate, c->act, Fs, EPI_SWIGLU);
      g.B2 = w.ws_up; g.ldb2 = D;
      if (keep) { g.C2 = keep->gate; g.C3 = keep->up; }
      SV_OP(c, SV_OP_GEMM_GATEUP, 4.0 * Td * Fs * D, st, gemm(c, g, st));
      GemmArgs h = nt(T, D, Fs, c->act, Fs, w.ws_down, y, D, EPI_RESID);
      h.R = x1; h.ldr = D;
      SV_OP(c, SV_OP_GEMM_DOWN, 2.0 * Td * D * Fs, st, gemm(c, h, st));
      base = y;
    }
    SV_OP(c, SV_OP_MOE_ROUTE, 2.0 * Td * E * D, st, launch_moe_route(c->n, w.w_router, T, D, E, K, d.router_score, d.router_norm, dt, r, st));
    SV_OP(c, SV_OP_MOE_PERMUTE, 0, st, launch_moe_gather(c->n, D, Mp, E, r, 0, c->xp, dt, st));
    {
      GemmArgs g = nt((int)Mp, F, D, c->xp, D, w.w_gate, c->actp, F, EPI_SWIGLU);
      g.B2 = w.w_up; g.ldb2 = D;
      g.tile_group = r.tile_expert; g.group_stride = (int64_t)F * D; g.m_dev = r.meta;
      if (keep) { g.C2 = keep->gate_p; g.C3 = keep->up_p; }
      SV_OP(c, SV_OP_GEMM_GATEUP, 4.0 * rows * F * D, st, gemm(c, g, st));
      GemmArgs h = nt((int)Mp, D, F, c->actp, F, w.w_down, yp, D, EPI_STORE);
      h.tile_group = r.tile_expert; h.group_stride = (int64_t)D * F; h.m_dev = r.meta;
      SV_OP(c, SV_OP_GEMM_DOWN, 2.0 * rows * D * F, st, gemm(c, h, st));
    }
    SV_OP(c, SV_OP_MOE_PERMUTE, 0, st, launch_moe_combine(base, yp, T, D, K, r, y, dt, st));
    return SV_OK;
  }
  if (d.mlp == SV_MLP_SWIGLU) {
    GemmArgs g = nt(T, F, D, c->n, D, w.w_gate, c->act, F, EPI_SWIGLU);
    g.B2 = w.w_up; g.ldb2 = D;
    if (keep) { g.C2 = keep->gate; g.C3 = keep->up; }
    SV_OP(c, SV_OP_GEMM_GATEUP, 4.0 * Td * F * D, st, gemm(c, g, st));
  } else {
    GemmArgs g = nt(T, F, D, c->n, D, w.w_up, c->act, F, EPI_GELU);
    if (keep) g.C2 = keep->up;
    SV_OP(c, SV_OP_GEMM_GATEUP, 2.0 * Td * F * D, st, gemm(c, g, st));
  }
  {
    GemmArgs g = nt(T, D, F, c->act, F, w.w_down, y, D, EPI_RESID);
    g.R = x1; g.ldr = D;
    SV_OP(c, SV_OP_GEMM_DOWN, 2.0 * Td * D * F, st, gemm(c, g, st));
  }
  return SV_OK;
}

GemmArgs nn(int M, int N, void* C, int64_t ldc, int epi) {
  GemmArgs g; memset(&g, 0, sizeof(g));
  g.M = M; g.N = N; g.nseg = 0; g.b_is_kn = 1; g.epi = epi; g.C = C; g.ldc = ldc;
  return g;
}
void add_seg(GemmArgs& g, const void* A, int64_t lda, const void* W, int64_t ldw, int K) {
  g.seg[g.nseg++] = GemmSeg{A, lda, W, ldw, K};
}

// One block backward: dy = dL/dy -> dx = dL/dx, reading the block input x and its stash.
sv_status transpose_block_weights(sv_ctx* c, const sv_block_weights& w, const sv_ctx::WT& t, hipStream_t st) {
  const sv_stage_desc& d = c->d;
  const int D = d.d_model, F = d.ffn_hidden, dt = d.dtype, es = c->es;
  for (int e = 0; e < (c->moe ? d.n_experts : 1); ++e) {
    const int64_t off = (int64_t)e * D * F;
    SV_OP(c, SV_OP_BWD_WTRANSPOSE, 0, st, plain_transpose(at(w.w_down, off, es), at(t.wd, off, es), D, F, dt, st));
    SV_OP(c, SV_OP_BWD_WTRANSPOSE, 0, st, plain_transpose(at(w.w_up, off, es), at(t.wu, off, es), F, D, dt, st));
    if (d.mlp == SV_MLP_SWIGLU) SV_OP(c, SV_OP_BWD_WTRANSPOSE, 0, st, plain_transpose(at(w.w_gate, off, es), at(t.wg, off, es), F, D, dt, st));
  }
  if (c->moe && c->Fd) {
    SV_OP(c, SV_OP_BWD_WTRANSPOSE, 0, st, plain_transpose(w.ws_down, t.wsd, D, c->Fd, dt, st));
    SV_OP(c, SV_OP_BWD_WTRANSPOSE, 0, st, plain_transpose(w.ws_up, t.wsu, c->Fd, D, dt, st));
    SV_OP(c, SV_OP_BWD_WTRANSPOSE, 0, st, plain_transpose(w.ws_gate, t.wsg, c->Fd, D, dt, st));
  }
  SV_OP(c, SV_OP_BWD_WTRANSPOSE, 0, st, plain_transpose(w.wo, t.wo, D, c->Dq, dt, st));
  SV_OP(c, SV_OP_BWD_WTRANSPOSE, 0, st, plain_transpose(w.wq, t.wq, c->Dq, D, dt, st));
  SV_OP(c, SV_OP_BWD_WTRANSPOSE, 0, st, plain_transpose(w.wk, t.wk, c->Dkv, D, dt, st));
  SV_OP(c, SV_OP_BWD_WTRANSPOSE, 0, st, plain_transpose(w.wv, t.wv, c->Dkv, D, dt, st));
  return SV_OK;
}

sv_status block_backward(sv_ctx* c, int l, const sv_block_weights& w, const void* x, const BlockStash& k, const void* dy, void* dx, int B, int S,
                         hipStream_t st) {
  const sv_stage_desc& d = c->d;
  const int T = B * S, D = d.d_model, F = d.ffn_hidden, es = c->es, dt = d.dtype;
  const double Td = T, attn_flop = (d.causal ? 2.0 : 4.0) * B * d.n_heads * (double)S * S * c->hd;
  // On the bf16 matrix-core path the [out, in] weights are used transposed to [in, out], so that
  // every backward product dY * W is again an "activations times [N, K] weights" product and runs
  // on the same direct-to-LDS kernel as the forward.  The transposed copies are made here (2 x weight
  // bytes through HBM) unless sv_prepare_weights made them for exactly these weights.
  const bool wt = !c->wT.empty();
  sv_ctx::WT t{};
  if (wt) {
    t = c->wT[l];
    const bool ready = (int)c->prepared.size() == d.n_blocks && memcmp(&c->prepared[l], &w, sizeof(w)) == 0;
    if (!ready) {
      sv_status s = transpose_block_weights(c, w, t, st);
      if (s != SV_OK) return s;
    }
  }
  // product dY [T, K] * W [K, N] with W given as stored ([K, N]) or transposed ([N, K])
  auto seg = [&](GemmArgs& g, const void* A, int64_t lda, const void* W, const void* WT, int K, int N) {
    if (wt) add_seg(g, A, lda, WT, K, K); else add_seg(g, A, lda, W, N, K);
  };
  auto args = [&](int N, void* Cout, int64_t ldc, int epi) {
    GemmArgs g = nn(T, N, Cout, ldc, epi);
    g.b_is_kn = wt ? 0 : 1;
    return g;
  };
  if (c->moe) {
    const int E = d.n_experts, K = d.top_k, Fs = d.ffn_shared;
    const MoeRoute& r = k.route;
    const int64_t Mp = moe_padded_rows(T, K, E);
    const double rows = Td * K;
    auto grouped = [&](GemmArgs& g) {
      g.M = (int)Mp; g.tile_group = r.tile_expert; g.group_stride = (int64_t)D * F; g.m_dev = r.meta;
    };
    if (Fs > 0) {                                                // shared experts: the dense backward into dn
      GemmArgs g = args(Fs, c->dgate, Fs, EPI_SWIGLU_BWD);
      seg(g, dy, D, w.ws_down, t.wsd, D, Fs);
      g.C2 = c->dup; g.R = k.gate; g.R2 = k.up; g.ldr = Fs;
      SV_OP(c, SV_OP_BWD_GEMM_DA, 2.0 * Td * Fs * D, st, gemm(c, g, st));
      GemmArgs h = args(D, c->dn, D, EPI_STORE);
      seg(h, c->dgate, Fs, w.ws_gate, t.wsg, Fs, D);
      seg(h, c->dup, Fs, w.ws_up, t.wsu, Fs, D);
      SV_OP(c, SV_OP_BWD_GEMM_DN2, 4.0 * Td * Fs * D, st, gemm(c, h, st));
    }
    // routed experts: rows gate * dy in expert order, back through down / SwiGLU / gate and up, then per token the sum
    // over its experts plus the gradient that reaches n through the gate values (router)
    SV_OP(c, SV_OP_BWD_MOE, 0, st, launch_moe_gather(dy, D, Mp, E, r, 1, c->xp, dt, st));
    {
      GemmArgs g = args(F, c->actp, F, EPI_SWIGLU_BWD);
      seg(g, c->xp, D, w.w_down, t.wd, D, F);
      g.C2 = c->dup_p; g.R = k.gate_p; g.R2 = k.up_p; g.ldr = F;
      grouped(g);
      SV_OP(c, SV_OP_BWD_GEMM_DA, 2.0 * rows * F * D, st, gemm(c, g, st));
      GemmArgs h = args(D, c->xp, D, EPI_STORE);                 // overwrites the gathered rows, which are dead by now
      seg(h, c->actp, F, w.w_gate, t.wg, F, D);
      seg(h, c->dup_p, F, w.w_up, t.wu, F, D);
      grouped(h);
      SV_OP(c, SV_OP_BWD_GEMM_DN2, 4.0 * rows * F * D, st, gemm(c, h, st));
    }
    SV_OP(c, SV_OP_BWD_MOE, 2.0 * Td * (K + E) * D, st,
          launch_moe_combine_bwd(dy, k.yp, c->xp, w.w_router, T, D, E, K, d.router_score, d.router_norm, r, Fs > 0, c->dn, dt, st));
  } else if (d.mlp == SV_MLP_SWIGLU) {
    GemmArgs g = args(F, c->dgate, F, EPI_SWIGLU_BWD);           // da = dy Wd, then through silu(g)*u
    seg(g, dy, D, w.w_down, t.wd, D, F);
    g.C2 = c->dup; g.R = k.gate; g.R2 = k.up; g.ldr = F;
    SV_OP(c, SV_OP_BWD_GEMM_DA, 2.0 * Td * F * D, st, gemm(c, g, st));
    GemmArgs h = args(D, c->dn, D, EPI_STORE);                   // dn2 = dG Wg + dU Wu
    seg(h, c->dgate, F, w.w_gate, t.wg, F, D);
    seg(h, c->dup, F, w.w_up, t.wu, F, D);
    SV_OP(c, SV_OP_BWD_GEMM_DN2, 4.0 * Td * F * D, st, gemm(c, h, st));
  } else {
    GemmArgs g = args(F, c->dgate, F, EPI_GELU_BWD);
    seg(g, dy, D, w.w_down, t.wd, D, F);
    g.R = k.up; g.ldr = F;
    SV_OP(c, SV_OP_BWD_GEMM_DA, 2.0 * Td * F * D, st, gemm(c, g, st));
    GemmArgs h = args(D, c->dn, D, EPI_STORE);
    seg(h, c->dgate, F, w.w_up, t.wu, F, D);
    SV_OP(c, SV_OP_BWD_GEMM_DN2, 2.0 * Td * F * D, st, gemm(c, h, st));
  }
  SV_OP(c, SV_OP_BWD_NORM, 0, st, plain_norm_bwd_add(c->dn, k.x1, w.norm2_g, dy, c->dx1, T, D, d.norm, d.norm_eps, dt, st));
  {
    GemmArgs g = args(c->Dq, c->dout, c->Dq, EPI_STORE);         // do = dx1 Wo
    seg(g, c->dx1, D, w.wo, t.wo, D, c->Dq);
    SV_OP(c, SV_OP_BWD_GEMM_DO, 2.0 * Td * D * c->Dq, st, gemm(c, g, st));
  }
  SV_OP(c, SV_OP_BWD_ATTN, 2.5 * attn_flop, st, attn_bwd(c, k, B, S, st));
  if (d.rope && !attn_on_mfma(c, S))
    SV_OP(c, SV_OP_BWD_ROPE, 0, st, plain_rope(c->dqkv, c->Dqkv, T, S, d.n_heads, d.n_kv_heads, c->hd, c->rope_cs, 1, dt, st));
  {
    GemmArgs g = args(D, c->dn, D, EPI_STORE);                   // dn1 = dq Wq + dk Wk + dv Wv
    seg(g, c->dqkv, c->Dqkv, w.wq, t.wq, c->Dq, D);
    seg(g, at(c->dqkv, c->Dq, es), c->Dqkv, w.wk, t.wk, c->Dkv, D);
    seg(g, at(c->dqkv, c->Dq + c->Dkv, es), c->Dqkv, w.wv, t.wv, c->Dkv, D);
    SV_OP(c, SV_OP_BWD_GEMM_DN1, 2.0 * Td * D * c->Dqkv, st, gemm(c, g, st));
  }
  SV_OP(c, SV_OP_BWD_NORM, 0, st, plain_norm_bwd_add(c->dn, x, w.norm1_g, c->dx1, dx, T, D, d.norm, d.norm_eps, dt, st));
  return SV_OK;
}

sv_status check_call(sv_ctx* c, const sv_block_weights* w, const void* h_in, int B, int S, const void* claim, const float* tau,
                     int reduce, sv_result* res) {
  if (!c) return SV_EINVAL;
  if (!w || !h_in) { set_err(c, "weights and h_in must be non-NULL"); return SV_EINVAL; }
  if (B < 1 || S < 1) { set_err(c, "B and S must be positive"); return SV_EINVAL; }
  if ((int64_t)B * S > c->max_tokens || S > c->max_seq) {
    set_err(c, "B*S=%lld or S=%d exceeds the context limits (%lld tokens, seq %d)", (long long)B * S, S, (long long)c->max_tokens, c->max_seq);
    return SV_EINVAL;
  }
  if (claim && (!res || !tau)) { set_err(c, "a claim needs result_dev and tau"); return SV_EINVAL; }
  if (reduce != SV_REDUCE_GLOBAL && reduce != SV_REDUCE_MAX_TOKEN) { set_err(c, "unknown reduce"); return SV_EINVAL; }
  for (int l = 0; l < c->d.n_blocks; ++l) {
    const sv_block_weights& b = w[l];
    const bool mats = b.wq && b.wk && b.wv && b.wo && b.w_up && b.w_down && b.norm1_g && b.norm2_g;
    const bool gate = c->d.mlp == SV_MLP_SWIGLU ? b.w_gate != nullptr : true;
    const bool bias = c->d.norm == SV_NORM_LN ? (b.norm1_b && b.norm2_b) : true;
    const bool moe_ok = !c->moe || (b.w_router && (c->Fd == 0 || (b.ws_gate && b.ws_up && b.ws_down)));
    if (!mats || !gate || !bias || !moe_ok) { set_err(c, "block %d: a required weight pointer is NULL", l); return SV_EINVAL; }
  }
  return SV_OK;
}

}  // namespace

extern "C" {

sv_status sv_check_desc(const sv_stage_desc* desc, uint32_t flags, char* msg, int32_t msg_len) {
  return check_desc_impl(desc, flags, msg, msg_len);
}

int64_t sv_workspace_bytes(const sv_stage_desc* desc, int64_t max_tokens, int32_t max_seq, uint32_t flags) {
  if (check_desc_impl(desc, flags, nullptr, 0) != SV_OK || max_tokens < 1 || max_seq < 1) return -1;
  sv_ctx tmp;
  init_ctx_fields(&tmp, desc, max_tokens, max_seq, flags);
  return (int64_t)carve(&tmp, nullptr);
}

sv_status sv_create(const sv_stage_desc* desc, int64_t max_tokens, int32_t max_seq, uint32_t flags, sv_ctx** out) {
  if (!out) { set_err(nullptr, "out is NULL"); return SV_EINVAL; }
  *out = nullptr;
  char msg[200];
  sv_status s = check_desc_impl(desc, flags, msg, sizeof(msg));
  if (s != SV_OK) { set_err(nullptr, "%s", msg); return s; }
  if (max_tokens < 1 || max_seq < 1 || max_tokens > 0x7fffffffLL) { set_err(nullptr, "max_tokens / max_seq out of range"); return SV_EINVAL; }
  if (desc->n_experts > 0 && moe_padded_rows(max_tokens, desc->top_k, desc->n_experts) > 0x7fffffffLL) {
    set_err(nullptr, "max_tokens * top_k is out of range");
    return SV_EINVAL;
  }
  sv_ctx* c = new sv_ctx();
  init_ctx_fields(c, desc, max_tokens, max_seq, flags);
  c->ws_bytes = carve(c, nullptr);
  hipError_t e = hipGetDevice(&c->device);
  if (e == hipSuccess) e = hipMalloc(&c->ws, c->ws_bytes);
  if (e != hipSuccess) {
    set_err(nullptr, "workspace of %zu bytes: %s", c->ws_bytes, hipGetErrorString(e));
    delete c;
    return e == hipErrorOutOfMemory ? SV_ENOMEM : SV_EHIP;
  }
  carve(c, (char*)c->ws);
  // RoPE table in double on the host: (cos, sin) of p * theta^(-2i/hd)
  const int half = c->hd / 2;
  std::vector<float> cs((size_t)max_seq * half * 2);
  for (int p = 0; p < max_seq; ++p)
    for (int i = 0; i < half; ++i) {
      const double ang = (double)p * pow((double)desc->rope_theta, -2.0 * i / (double)c->hd);
      cs[((size_t)p * half + i) * 2] = (float)cos(ang);
      cs[((size_t)p * half + i) * 2 + 1] = (float)sin(ang);
    }
  e = hipMemcpy(c->rope_cs, cs.data(), cs.size() * sizeof(float), hipMemcpyHostToDevice);
  if (e != hipSuccess) {
    set_err(nullptr, "uploading the RoPE table: %s", hipGetErrorString(e));
    (void)hipFree(c->ws);
    delete c;
    return SV_EHIP;
  }
  *out = c;
  return SV_OK;
}

void sv_destroy(sv_ctx* c) {
  if (!c) return;
  for (auto& r : c->prof_recs) { (void)hipEventDestroy(r.a); (void)hipEventDestroy(r.b); }
  for (auto e : c->prof_pool) (void)hipEventDestroy(e);
  if (c->ws) (void)hipFree(c->ws);
  delete c;
}

sv_status sv_profile_enable(sv_ctx* c, int32_t on) {
  if (!c) return SV_EINVAL;
  if (on) {
    for (auto& r : c->prof_recs) { c->prof_pool.push_back(r.a); c->prof_pool.push_back(r.b); }
    c->prof_recs.clear();
    memset(&c->prof_acc, 0, sizeof(c->prof_acc));
  }
  c->prof_on = on != 0;
  return SV_OK;
}

sv_status sv_profile_select(sv_ctx* c, uint64_t op_mask) {
  if (!c) return SV_EINVAL;
  c->prof_mask = op_mask ? op_mask : ~0ull;
  return SV_OK;
}

sv_status sv_profile_read(sv_ctx* c, sv_profile* out) {
  if (!c || !out) return SV_EINVAL;
  for (auto& r : c->prof_recs) {
    SV_HIP(c, hipEventSynchronize(r.b));
    float ms = 0.0f;
    SV_HIP(c, hipEventElapsedTime(&ms, r.a, r.b));
    c->prof_acc.ms[r.op] += ms;
    c->prof_pool.push_back(r.a); c->prof_pool.push_back(r.b);
  }
  c->prof_recs.clear();
  *out = c->prof_acc;
  return SV_OK;
}

const char* sv_last_error(const sv_ctx* c) { return c ? c->err : g_create_error; }

sv_status sv_verify_forward(sv_ctx* c, const sv_block_weights* w, const void* h_in, int32_t B, int32_t S, const void* claimed_h,
                            uint32_t metric_mask, const float* tau, int32_t reduce, void* h_hat_out, float* token_scores_out,
                            sv_result* result_dev, void* stream) {
  sv_status s = check_call(c, w, h_in, B, S, claimed_h, tau, reduce, result_dev);
  if (s != SV_OK) return s;
  hipStream_t st = (hipStream_t)stream;
  const int L = c->d.n_blocks;
  const bool bwd = c->flags & SV_FLAG_BACKWARD;
  c->last_T = B * S;
  c->rowsq_of = nullptr;
  const void* x = h_in;
  void* y = nullptr;
  for (int l = 0; l < L; ++l) {
    if (l == L - 1) y = h_hat_out ? h_hat_out : c->xbuf[l & 1];
    else y = bwd ? c->xs[l] : c->xbuf[l & 1];
    // a backward context owns one routing record per block and none of its own
    const bool own = c->moe && bwd;
    s = block_forward(c, l, w[l], x, y, B, S, nullptr, st, own ? &c->stash[l].route : nullptr, own ? c->stash[l].yp : nullptr);
    if (s != SV_OK) return s;
    x = y;
  }
  if (claimed_h)
    SV_OP(c, SV_OP_SCORE, 0, st, launch_score(claimed_h, 0, 1, y, 0, c->d.dtype, c->d.dtype, (int64_t)B * S, c->d.d_model, metric_mask, tau, reduce,
                           token_scores_out, result_dev, c->score_scratch, kScoreScratchElems, st));
  return SV_OK;
}

sv_status sv_verify_backward(sv_ctx* c, const sv_block_weights* w, const void* h_in, const void* g_out, int32_t B, int32_t S,
                             const void* claimed_g, uint32_t metric_mask, const float* tau, int32_t reduce, void* g_hat_out,
                             void* h_hat_out, float* token_scores_out, sv_result* result_dev, void* stream) {
  sv_status s = check_call(c, w, h_in, B, S, claimed_g, tau, reduce, result_dev);
  if (s != SV_OK) return s;
  if (!(c->flags & SV_FLAG_BACKWARD)) { set_err(c, "context was created without SV_FLAG_BACKWARD"); return SV_EINVAL; }
  if (!g_out) { set_err(c, "g_out must be non-NULL"); return SV_EINVAL; }
  hipStream_t st = (hipStream_t)stream;
  const int L = c->d.n_blocks;
  c->last_T = B * S;
  c->rowsq_of = nullptr;
  const void* x = h_in;
  for (int l = 0; l < L; ++l) {
    void* y = (l == L - 1) ? (h_hat_out ? h_hat_out : c->xbuf[0]) : c->xs[l];
    s = block_forward(c, l, w[l], x, y, B, S, &c->stash[l], st);
    if (s != SV_OK) return s;
    x = y;
  }
  const void* dy = g_out;
  void* dx = nullptr;
  for (int l = L - 1; l >= 0; --l) {
    dx = (l == 0 && g_hat_out) ? g_hat_out : c->dres[l & 1];
    const void* xin = l == 0 ? h_in : c->xs[l - 1];
    s = block_backward(c, l, w[l], xin, c->stash[l], dy, dx, B, S, st);
    if (s != SV_OK) return s;
    dy = dx;
  }
  if (claimed_g)
    SV_OP(c, SV_OP_SCORE, 0, st, launch_score(claimed_g, 0, 1, dx, 0, c->d.dtype, c->d.dtype, (int64_t)B * S, c->d.d_model, metric_mask, tau, reduce,
                           token_scores_out, result_dev, c->score_scratch, kScoreScratchElems, st));
  return SV_OK;
}

sv_status sv_last_routing(sv_ctx* c, int32_t block, int32_t* experts_out, float* gates_out, void* stream) {
  if (!c) return SV_EINVAL;
  if (!c->moe) { set_err(c, "the stage has no mixture-of-experts MLP"); return SV_EINVAL; }
  if (c->last_T < 1) { set_err(c, "no verify call has run on this context"); return SV_EINVAL; }
  const bool bwd = c->flags & SV_FLAG_BACKWARD;
  if (block < 0 || block >= c->d.n_blocks || (!bwd && block != c->d.n_blocks - 1)) {
    set_err(c, "block %d: a forward-only context keeps the routing of its last block only", block);
    return SV_EINVAL;
  }
  const MoeRoute& r = bwd ? c->stash[block].route : c->route;
  const size_t n = (size_t)c->last_T * c->d.top_k;
  if (experts_out) SV_HIP(c, hipMemcpyAsync(experts_out, r.sel, n * sizeof(int32_t), hipMemcpyDeviceToDevice, (hipStream_t)stream));
  if (gates_out) SV_HIP(c, hipMemcpyAsync(gates_out, r.gate, n * sizeof(float), hipMemcpyDeviceToDevice, (hipStream_t)stream));
  return SV_OK;
}

sv_status sv_prepare_weights(sv_ctx* c, const sv_block_weights* w, void* stream) {
  if (!c) return SV_EINVAL;
  c->prepared.clear();
  if (!w) return SV_OK;                               // forget the prepared copies
  if (c->wT.empty() && c->wF.empty()) return SV_OK;   // this context keeps no copies (fp32, plain kernels, or forward only without SV_FLAG_FUSE_NORM)
  for (int l = 0; l < c->d.n_blocks; ++l) {
    const sv_block_weights& b = w[l];
    if (!(b.wq && b.wk && b.wv && b.wo && b.w_up && b.w_down && b.norm1_g && b.norm2_g) || (c->d.mlp == SV_MLP_SWIGLU && !b.w_gate) ||
        (c->moe && (!b.w_router || (c->Fd > 0 && !(b.ws_gate && b.ws_up && b.ws_down))))) {
      set_err(c, "block %d: a required weight pointer is NULL", l);
      return SV_EINVAL;
    }
    sv_status s = c->wT.empty() ? SV_OK : transpose_block_weights(c, b, c->wT[l], (hipStream_t)stream);
    if (s == SV_OK && !c->wF.empty()) s = fold_block_weights(c, b, c->wF[l], (hipStream_t)stream);
    if (s != SV_OK) return s;
  }
  c->prepared.assign(w, w + c->d.n_blocks);
  return SV_OK;
}

sv_status sv_score_and_flag(sv_ctx* c, const void* claims, int64_t claim_stride, int32_t n_claims, const void* ref, int64_t ref_stride,
                            int32_t claim_dtype, int32_t ref_dtype, int64_t T, int32_t D, uint32_t metric_mask, const float* tau,
                            int32_t reduce, float* token_scores_out, sv_result* results_dev, void* stream) {
  if (!c) return SV_EINVAL;
  if (n_claims < 0 || T < 0 || D < 1) { set_err(c, "negative size"); return SV_EINVAL; }
  if (n_claims == 0 || T == 0) return SV_OK;
  if (!claims || !ref || !results_dev || !tau) { set_err(c, "claims, ref, tau and results_dev must be non-NULL"); return SV_EINVAL; }
  if ((claim_dtype != SV_F32 && claim_dtype != SV_BF16) || (ref_dtype != SV_F32 && ref_dtype != SV_BF16)) { set_err(c, "unknown dtype"); return SV_EINVAL; }
  if (reduce != SV_REDUCE_GLOBAL && reduce != SV_REDUCE_MAX_TOKEN) { set_err(c, "unknown reduce"); return SV_EINVAL; }
  if (D % 8) { set_err(c, "D must be a multiple of 8"); return SV_EUNSUPPORTED; }
  if (T > 0x7fffffffLL || claim_stride < 0 || ref_stride < 0) { set_err(c, "T or a stride is out of range"); return SV_EINVAL; }
  if ((T + kScoreTokensPerWG - 1) / kScoreTokensPerWG > kScoreScratchElems) { set_err(c, "T too large for the score scratch"); return SV_EUNSUPPORTED; }
  SV_HIP(c, launch_score(claims, claim_stride, n_claims, ref, ref_stride, claim_dtype, ref_dtype, T, D, metric_mask, tau, reduce,
                         token_scores_out, results_dev, c->score_scratch, kScoreScratchElems, (hipStream_t)stream));
  return SV_OK;
}

sv_status sv_score_and_sum(sv_ctx* c, const void* claims, int64_t claim_stride, int32_t n_claims, const void* ref, int32_t claim_dtype,
                           int32_t ref_dtype, int64_t T, int32_t D, uint32_t metric_mask, const float* tau, int32_t reduce,
                           float* token_scores_out, sv_result* results_dev, const uint8_t* skip_host, float* sum_out, void* stream) {
  if (!c) return SV_EINVAL;
  if (n_claims < 0 || T < 0 || D < 1) { set_err(c, "negative size"); return SV_EINVAL; }
  if (n_claims == 0 || T == 0) return SV_OK;
  if (!claims || !ref || !results_dev || !tau || !sum_out) { set_err(c, "claims, ref, tau, results_dev and sum_out must be non-NULL"); return SV_EINVAL; }
  if ((claim_dtype != SV_F32 && claim_dtype != SV_BF16) || (ref_dtype != SV_F32 && ref_dtype != SV_BF16)) { set_err(c, "unknown dtype"); return SV_EINVAL; }
  if (reduce != SV_REDUCE_GLOBAL && reduce != SV_REDUCE_MAX_TOKEN) { set_err(c, "unknown reduce"); return SV_EINVAL; }
  if (T > 0x7fffffffLL || claim_stride < 0) { set_err(c, "T or the stride is out of range"); return SV_EINVAL; }
  const int64_t tiles = (T + kScoreTokensPerWG - 1) / kScoreTokensPerWG;
  if (!score_sum_supported(n_claims, 0, claim_dtype, D) || tiles * n_claims > kScoreScratchElems) {
    set_err(c, "sv_score_and_sum needs at most 32 submissions, rows of a multiple of 2 KB and n_claims * ceil(T / 16) <= %lld",
            (long long)kScoreScratchElems);
    return SV_EUNSUPPORTED;
  }
  uint32_t skip = 0;
  for (int i = 0; skip_host && i < n_claims; ++i)
    if (skip_host[i]) skip |= 1u << i;
  SV_HIP(c, launch_score(claims, claim_stride, n_claims, ref, 0, claim_dtype, ref_dtype, T, D, metric_mask, tau, reduce, token_scores_out,
                         results_dev, c->score_scratch, kScoreScratchElems, (hipStream_t)stream, skip, sum_out));
  return SV_OK;
}

sv_status sv_ema_from_sum(sv_ctx* c, float* m, const float* sum, int32_t n_summed, int64_t T, int32_t D, float beta, void* stream) {
  if (!c) return SV_EINVAL;
  if (n_summed < 0 || T < 0 || D < 1) { set_err(c, "negative size"); return SV_EINVAL; }
  if (n_summed == 0 || T == 0) return SV_OK;
  if (!m || !sum) { set_err(c, "m and sum must be non-NULL"); return SV_EINVAL; }
  if (!(beta >= 0.0f && beta < 1.0f)) { set_err(c, "beta must be in [0, 1)"); return SV_EINVAL; }
  if (D % 8) { set_err(c, "D must be a multiple of 8"); return SV_EUNSUPPORTED; }
  SV_HIP(c, launch_ema_from_sum(m, sum, n_summed, T, D, beta, (hipStream_t)stream));
  return SV_OK;
}

sv_status sv_sliced_wasserstein(sv_ctx* c, const void* claims, int64_t claim_stride, int32_t n_claims, const void* ref, int64_t ref_stride,
                                int32_t claim_dtype, int32_t ref_dtype, int64_t T, int32_t D, const void* directions, int32_t L, float tau,
                                float* sw_out, sv_result* results_dev, void* stream) {
  if (!c) return SV_EINVAL;
  if (n_claims < 0 || T < 0 || D < 1 || L < 1) { set_err(c, "negative size"); return SV_EINVAL; }
  if (!(c->flags & SV_FLAG_SLICED_W)) { set_err(c, "context was created without SV_FLAG_SLICED_W"); return SV_EINVAL; }
  if (n_claims == 0 || T == 0) return SV_OK;
  if (!claims || !ref || !directions) { set_err(c, "claims, ref and directions must be non-NULL"); return SV_EINVAL; }
  if ((claim_dtype != SV_F32 && claim_dtype != SV_BF16) || (ref_dtype != SV_F32 && ref_dtype != SV_BF16)) { set_err(c, "unknown dtype"); return SV_EINVAL; }
  if (claim_stride < 0 || ref_stride < 0) { set_err(c, "negative stride"); return SV_EINVAL; }
  if (L % 32 || L > kSwMaxDirs) { set_err(c, "n_dirs must be a multiple of 32, at most %d", kSwMaxDirs); return SV_EUNSUPPORTED; }
  if (D % 64) { set_err(c, "D must be a multiple of 64"); return SV_EUNSUPPORTED; }
  if (n_claims > kSwMaxClaims) { set_err(c, "at most %d submissions per call", kSwMaxClaims); return SV_EUNSUPPORTED; }
  if (T > c->max_tokens) { set_err(c, "T=%lld exceeds the context's max_tokens %lld", (long long)T, (long long)c->max_tokens); return SV_EUNSUPPORTED; }
  hipStream_t st = (hipStream_t)stream;
  const int64_t Tpad = sw_padded_len(T);
  const size_t slot = (size_t)L * (size_t)Tpad;                 // floats of one projected tensor
  const int64_t n_slots = (int64_t)(c->sw_proj_floats / slot);  // >= kSwSlots by construction
  const bool shared = ref_stride == 0;
  const double flop_per = 2.0 * (double)T * D * L;
  const int ces = claim_dtype == SV_BF16 ? 2 : 4, res = ref_dtype == SV_BF16 ? 2 : 4;
  // A shared reference is projected in the first group's launch, beside the submissions (alone its few token tiles
  // leave most of the chip idle), where the kernel has that dtype pair.
  const bool ref_with_first = shared && sw_project_with_ref_supported(claim_dtype, ref_dtype);
  if (shared && !ref_with_first) {
    SV_OP(c, SV_OP_SW_PROJECT, flop_per, st, launch_sw_project(ref, 0, 1, ref_dtype, directions, L, D, T, Tpad, c->sw_proj, st));
    SV_OP(c, SV_OP_SW_SORT, 0, st, launch_sw_sort(c->sw_proj, L, T, Tpad, nullptr, 0, L, nullptr, 0, st));
  }
  const int group = (int)(shared ? n_slots - 1 : n_slots / 2);
  for (int first = 0; first < n_claims; first += group) {
    const int n = n_claims - first < group ? n_claims - first : group;
    float* pref = c->sw_proj;
    float* pcl = c->sw_proj + (shared ? slot : (size_t)group * slot);
    if (!shared) {
      SV_OP(c, SV_OP_SW_PROJECT, flop_per * n, st,
            launch_sw_project(at(ref, (int64_t)first * ref_stride, res), ref_stride, n, ref_dtype, directions, L, D, T, Tpad, pref, st));
      SV_OP(c, SV_OP_SW_SORT, 0, st, launch_sw_sort(pref, n * L, T, Tpad, nullptr, 0, L, nullptr, 0, st));
    }
    if (ref_with_first && first == 0) {
      SV_OP(c, SV_OP_SW_PROJECT, flop_per * (n + 1), st,
            launch_sw_project_with_ref(claims, claim_stride, n, claim_dtype, ref, ref_dtype, directions, L, D, T, Tpad, pcl, pref, st));
      SV_OP(c, SV_OP_SW_SORT, 0, st, launch_sw_sort(pref, L, T, Tpad, nullptr, 0, L, nullptr, 0, st));
    } else {
      SV_OP(c, SV_OP_SW_PROJECT, flop_per * n, st,
            launch_sw_project(at(claims, (int64_t)first * claim_stride, ces), claim_stride, n, claim_dtype, directions, L, D, T, Tpad, pcl, st));
    }
    SV_OP(c, SV_OP_SW_SORT, 0, st, launch_sw_sort(pcl, n * L, T, Tpad, pref, shared ? 1 : 0, L, c->sw_w1, first * L, st));
  }
  SV_HIP(c, launch_sw_finalize(c->sw_w1, n_claims, L, T, tau, sw_out, results_dev, st));
  return SV_OK;
}

int64_t sv_sw_row_len(int64_t T) { return T < 0 ? 0 : sw_padded_len(T); }

sv_status sv_sw_against_projection(sv_ctx* c, const void* claims, int64_t claim_stride, int32_t n_claims, int32_t claim_dtype, int64_t T,
                                   int32_t D, const void* directions, int32_t L, const float* ref_proj, float* claim_proj_out, float tau,
                                   float* sw_out, sv_result* results_dev, void* stream) {
  if (!c) return SV_EINVAL;
  if (n_claims < 0 || T < 0 || D < 1 || L < 1) { set_err(c, "negative size"); return SV_EINVAL; }
  if (!(c->flags & SV_FLAG_SLICED_W)) { set_err(c, "context was created without SV_FLAG_SLICED_W"); return SV_EINVAL; }
  if (n_claims == 0 || T == 0) return SV_OK;
  if (!claims || !directions || !ref_proj || !claim_proj_out) { set_err(c, "claims, directions, ref_proj and claim_proj_out must be non-NULL"); return SV_EINVAL; }
  if (claim_dtype != SV_F32 && claim_dtype != SV_BF16) { set_err(c, "unknown dtype"); return SV_EINVAL; }
  if (claim_stride < 0) { set_err(c, "negative stride"); return SV_EINVAL; }
  if (L % 32 || L > kSwMaxDirs) { set_err(c, "n_dirs must be a multiple of 32, at most %d", kSwMaxDirs); return SV_EUNSUPPORTED; }
  if (D % 64) { set_err(c, "D must be a multiple of 64"); return SV_EUNSUPPORTED; }
  if (n_claims > 256) { set_err(c, "at most 256 submissions per call"); return SV_EUNSUPPORTED; }       // one launch: grid rows
  if (T > c->max_tokens) { set_err(c, "T=%lld exceeds the context's max_tokens %lld", (long long)T, (long long)c->max_tokens); return SV_EUNSUPPORTED; }
  const int64_t Tpad = sw_padded_len(T);
  if (Tpad > kSwSortChunkMax) { set_err(c, "rows longer than %lld are sorted in place: use sv_sliced_wasserstein", (long long)kSwSortChunkMax); return SV_EUNSUPPORTED; }
  hipStream_t st = (hipStream_t)stream;
  SV_HIP(c, launch_sw_copy_pad(c->sw_proj, ref_proj, L, T, Tpad, st));
  SV_OP(c, SV_OP_SW_SORT, 0, st, launch_sw_sort(c->sw_proj, L, T, Tpad, nullptr, 0, L, nullptr, 0, st));
  SV_OP(c, SV_OP_SW_PROJECT, 2.0 * (double)T * D * L * n_claims, st,
        launch_sw_project(claims, claim_stride, n_claims, claim_dtype, directions, L, D, T, Tpad, claim_proj_out, st));
  // rows of one LDS chunk: the last sort pass adds up |a - b| against the reference and leaves the projections as they are
  SV_OP(c, SV_OP_SW_SORT, 0, st, launch_sw_sort(claim_proj_out, n_claims * L, T, Tpad, c->sw_proj, 1, L, c->sw_w1, 0, st));
  SV_HIP(c, launch_sw_finalize(c->sw_w1, n_claims, L, T, tau, sw_out, results_dev, st));
  return SV_OK;
}

sv_status sv_sw_projection_ema(sv_ctx* c, float* ref_proj, const float* claim_proj, int32_t n_claims, const uint8_t* skip_host, int64_t T,
                               int32_t L, float beta, void* stream) {
  if (!c) return SV_EINVAL;
  if (n_claims < 0 || T < 0 || L < 1) { set_err(c, "negative size"); return SV_EINVAL; }
  if (n_claims == 0 || T == 0) return SV_OK;
  if (!ref_proj || !claim_proj) { set_err(c, "ref_proj and claim_proj must be non-NULL"); return SV_EINVAL; }
  if (!(beta >= 0.0f && beta < 1.0f)) { set_err(c, "beta must be in [0, 1)"); return SV_EINVAL; }
  if (n_claims > 32) { set_err(c, "at most 32 submissions"); return SV_EUNSUPPORTED; }
  uint32_t skip = 0;
  int n = 0;
  for (int i = 0; i < n_claims; ++i) {
    if (skip_host && skip_host[i]) skip |= 1u << i;
    else ++n;
  }
  if (n == 0) return SV_OK;
  SV_HIP(c, launch_sw_proj_ema(ref_proj, claim_proj, n_claims, skip, L, T, sw_padded_len(T), beta, (1.0f - beta) / (float)n, (hipStream_t)stream));
  return SV_OK;
}

sv_status sv_ema_update(sv_ctx* c, float* m, const void* claims, int64_t claim_stride, int32_t n_claims, int32_t claim_dtype,
                        const uint8_t* flags_dev, int64_t T, int32_t D, float beta, void* stream) {
  if (!c) return SV_EINVAL;
  if (n_claims < 0 || T < 0 || D < 1) { set_err(c, "negative size"); return SV_EINVAL; }
  if (n_claims == 0 || T == 0) return SV_OK;
  if (!m || !claims) { set_err(c, "m and claims must be non-NULL"); return SV_EINVAL; }
  if (claim_dtype != SV_F32 && claim_dtype != SV_BF16) { set_err(c, "unknown dtype"); return SV_EINVAL; }
  if (!(beta >= 0.0f && beta < 1.0f)) { set_err(c, "beta must be in [0, 1)"); return SV_EINVAL; }
  if (D % 8) { set_err(c, "D must be a multiple of 8"); return SV_EUNSUPPORTED; }
  if (claim_stride < 0) { set_err(c, "negative stride"); return SV_EINVAL; }
  if (n_claims > 1024) { set_err(c, "at most 1024 submissions per EMA update"); return SV_EUNSUPPORTED; }
  SV_HIP(c, launch_ema(m, claims, claim_stride, n_claims, claim_dtype, flags_dev, T, D, beta, (hipStream_t)stream));
  return SV_OK;
}

sv_status sv_replace_with_ema(sv_ctx* c, void* signals, int64_t stride, int32_t n, int32_t dtype, const uint8_t* mask_dev, const float* m,
                              int64_t T, int32_t D, void* stream) {
  if (!c) return SV_EINVAL;
  if (n < 0 || T < 0 || D < 1 || stride < 0) { set_err(c, "negative size"); return SV_EINVAL; }
  if (n == 0 || T == 0) return SV_OK;
  if (!signals || !mask_dev || !m) { set_err(c, "signals, mask_dev and m must be non-NULL"); return SV_EINVAL; }
  if (dtype != SV_F32 && dtype != SV_BF16) { set_err(c, "unknown dtype"); return SV_EINVAL; }
  if (D % 8) { set_err(c, "D must be a multiple of 8"); return SV_EUNSUPPORTED; }
  if (n > 65535) { set_err(c, "at most 65535 signals per call"); return SV_EUNSUPPORTED; }
  SV_HIP(c, launch_replace(signals, stride, n, dtype, mask_dev, m, T, D, (hipStream_t)stream));
  return SV_OK;
}

sv_status sv_gemm_bf16(const void* A, int64_t lda, const void* B, int64_t ldb, int32_t b_is_kn, void* Cout, int64_t ldc, int32_t M,
                       int32_t N, int32_t K, int32_t tile, void* stream) {
  if (!A || !B || !Cout || M < 1 || N < 1 || K < 1 || tile < 0 || tile > 4) return SV_EINVAL;
  GemmArgs g; memset(&g, 0, sizeof(g));
  g.M = M; g.N = N; g.nseg = 1; g.seg[0] = GemmSeg{A, lda, B, ldb, K};
  g.b_is_kn = b_is_kn ? 1 : 0; g.epi = EPI_STORE; g.C = Cout; g.ldc = ldc;
  if (!mfma_gemm_supported(g) || ((tile == 1 || tile == 3) && N % 256) || (tile == 4 && b_is_kn)) return SV_EUNSUPPORTED;
  return mfma_gemm(g, (hipStream_t)stream, tile) == hipSuccess ? SV_OK : SV_EHIP;
}

}  // extern "C"
