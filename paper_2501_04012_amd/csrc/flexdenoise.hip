// C ABI and host orchestration of the denoising step / cache-hit resume loop.
// The host builds the launch sequence of one step; nothing here synchronises the
// stream or reads device memory back, so a resume call enqueues all N-k steps.
#include "../../include/flexdenoise.h"
#include "common.h"

#include <cmath>
#include <cstdio>
#include <cstring>
#include <string>
#include <vector>

using namespace fc;

namespace {

thread_local std::string g_err;

int fail(int code, const std::string& msg) {
  g_err = msg;
  return code;
}
int fail_hip(hipError_t e, const char* where) {
  g_err = std::string(where) + ": " + hipGetErrorString(e);
  return FC_ERR_DEVICE;
}
#define HIP_TRY(expr)                                         \
  do {                                                        \
    hipError_t _e = (expr);                                   \
    if (_e != hipSuccess) return fail_hip(_e, #expr);         \
  } while (0)

// Optional per-kernel timing: HIP event pairs recorded on the caller's stream around
// each launch, summed per category when read.
enum ProfCat : int {
  PC_GEMM_QKV = 0, PC_GEMM_PROJ, PC_GEMM_FC1, PC_GEMM_FC2, PC_GEMM_OTHER,
  PC_ATTN_SPATIAL, PC_ATTN_TEMPORAL, PC_ATTN_CROSS, PC_ATTN_FULL,
  PC_LN_MODULATE, PC_PATCH_EMBED, PC_TIMESTEP_MOD, PC_CFG_DDIM, PC_OTHER, PC_COUNT
};
const char* const kProfNames[PC_COUNT] = {
  "gemm_qkv", "gemm_proj", "gemm_fc1", "gemm_fc2", "gemm_other",
  "attn_spatial", "attn_temporal", "attn_cross", "attn_full3d",
  "ln_modulate", "patch_embed", "timestep_modulation", "cfg_ddim", "other"};

struct Profiler {
  bool on = false;
  int only = -1;            // -1: every category, else just this one
  struct Rec { hipEvent_t a, b; int cat; };
  std::vector<Rec> recs;
  std::vector<hipEvent_t> pool;
  hipEvent_t get() {
    if (!pool.empty()) { hipEvent_t e = pool.back(); pool.pop_back(); return e; }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
  }
  void release_all() {
    for (auto& r : recs) { pool.push_back(r.a); pool.push_back(r.b); }
    recs.clear();
  }
  ~Profiler() {
    release_all();
    for (hipEvent_t e : pool) (void)hipEventDestroy(e);
  }
};

struct Linear {           // weights [out, in] in the activation dtype, bias fp32
  void* wt = nullptr;
  float* b = nullptr;
  int in = 0, out = 0;
};

struct Block {
  Linear qkv[2], proj[2];          // [0] spatial / full-3D, [1] temporal
  Linear xq, xkv, xproj;           // cross-attention (factorized mode)
  Linear fc1, fc2;
};

}  // namespace

struct fc_model {
  fc_model_config cfg;
  int device = 0;
  bool has_weights = false;
  bool bf16 = false;
  int S = 0, N = 0, Ns = 0, pd = 0, hd = 0, nmod = 0;
  size_t esz = 4;                  // bytes per activation / weight element

  unsigned char* wbuf = nullptr;   // one device allocation for all parameters and tables
  size_t wbytes = 0;
  Linear t1, t2, y, fmod, fout;
  float* p_w = nullptr;            // patch embedding stays fp32 [pd, D] (K is tiny)
  float* p_b = nullptr;
  void* mod_w = nullptr;           // [depth][nmod*D, D]
  float* mod_b = nullptr;          // [depth][nmod*D]
  float* pos_sp = nullptr;         // [S, D]
  float* pos_t = nullptr;          // [T, D]
  std::vector<Block> blocks;
  Profiler prof;
};

namespace {

// ---------------------------------------------------------------- schedule (host, double)
int schedule_check(const fc_schedule* s) {
  if (!s) return fail(FC_ERR_NULL, "schedule is NULL");
  if (!(s->eta >= 0.0f && s->eta <= 1.0f)) return fail(FC_ERR_RANGE, "eta must be in 0..1");
  if (s->eta != 0.0f && s->sampler != FC_SAMPLER_DDIM)
    return fail(FC_ERR_UNSUPPORTED, "eta belongs to the DDIM family; the Euler step draws no noise");
  if (s->train_steps < 1 || s->num_steps < 1 || s->num_steps > s->train_steps)
    return fail(FC_ERR_RANGE, "need 1 <= num_steps <= train_steps");
  if (s->sampler != FC_SAMPLER_DDIM && s->sampler != FC_SAMPLER_FLOW_EULER)
    return fail(FC_ERR_RANGE, "unknown sampler");
  if (s->sampler == FC_SAMPLER_FLOW_EULER && s->train_steps % s->num_steps != 0)
    return fail(FC_ERR_UNSUPPORTED, "the Euler sampler needs train_steps divisible by num_steps (integer timesteps)");
  return FC_OK;
}

double abar_at(const fc_schedule* s, int t) {
  double prod = 1.0;
  const double denom = s->train_steps > 1 ? (double)(s->train_steps - 1) : 1.0;
  for (int i = 0; i <= t; ++i) {
    double beta = (double)s->beta_start + ((double)s->beta_end - (double)s->beta_start) * (double)i / denom;
    prod *= 1.0 - beta;
  }
  return prod;
}

// out4: the update kernel's coefficients; *sigma_out: standard deviation of the noise the step adds (eta > 0)
int step_coefficients(const fc_schedule* s, int step, float* out4, int* t_out, float* sigma_out = nullptr) {
  int rc = schedule_check(s);
  if (rc != FC_OK) return rc;
  if (sigma_out) *sigma_out = 0.0f;
  const int N = s->num_steps;
  if (step < 1 || step > N) return fail(FC_ERR_RANGE, "step must be in 1..num_steps");
  const int stride = s->train_steps / N;
  if (s->sampler == FC_SAMPLER_FLOW_EULER) {
    // x <- x + (sigma_next - sigma) v on sigma_j = j / N, network evaluated at t = sigma * train_steps:
    // in the update kernel's form x0 = (x - c1 e) / c0, x <- c2 x0 + c3 e that is (1, 0, 1, -1/N)
    out4[0] = 1.0f; out4[1] = 0.0f; out4[2] = 1.0f;
    out4[3] = (float)((double)(N - step) / N - (double)(N - step + 1) / N);
    if (t_out) *t_out = (N - step + 1) * stride;
    return FC_OK;
  }
  const int t = (N - step) * stride;
  const double a_t = abar_at(s, t);
  const double a_p = step == N ? 1.0 : abar_at(s, (N - step - 1) * stride);
  out4[0] = (float)std::sqrt(a_t);
  out4[1] = (float)std::sqrt(1.0 - a_t);
  // eta > 0: sigma = eta sqrt((1-abar_prev)/(1-abar_t)) sqrt(1 - abar_t/abar_prev); the eps
  // direction keeps sqrt(1 - abar_prev - sigma^2)
  const double sigma = s->eta == 0.0f ? 0.0
                                      : (double)s->eta * std::sqrt((1.0 - a_p) / (1.0 - a_t)) * std::sqrt(1.0 - a_t / a_p);
  out4[2] = (float)std::sqrt(a_p);
  out4[3] = (float)std::sqrt(std::max(1.0 - a_p - sigma * sigma, 0.0));
  if (sigma_out) *sigma_out = (float)sigma;
  if (t_out) *t_out = t;
  return FC_OK;
}

// ---------------------------------------------------------------- weight blob walking
struct BlobItem { size_t off; int rows, cols; };   // matrices [rows, cols]; vectors rows = 1

size_t weight_count(const fc_model_config& c) {
  const size_t D = c.hidden, M = c.mlp_dim, te = c.t_embed_dim, dt = c.text_dim;
  const size_t pd = (size_t)c.patch * c.patch * c.channels;
  size_t n = te * D + D + D * D + D + dt * D + D + pd * D + D;
  size_t per;
  if (c.attn_mode == FC_ATTN_FACTORIZED_CROSS)
    per = D * 9 * D + 9 * D + 2 * (D * 3 * D + 3 * D + D * D + D) + (D * D + D) + (D * 2 * D + 2 * D) + (D * D + D);
  else
    per = D * (c.text_adaln ? 12 : 6) * (D + 1) + (D * 3 * D + 3 * D + D * D + D);
  per += D * M + M + M * D + D;
  n += per * c.depth;
  n += D * 2 * D + 2 * D + D * pd + pd;
  return n;
}

struct Carver {          // bump allocator over a byte range, 256-byte aligned pieces
  unsigned char* base;
  size_t off = 0;
  explicit Carver(unsigned char* b) : base(b) {}
  void* take(size_t bytes) {
    void* p = base ? base + off : nullptr;
    off += round_up(bytes, 256);
    return p;
  }
};

// Lays out (base != NULL) or sizes (base == NULL) the parameter buffer.
size_t layout_weights(fc_model* m, unsigned char* base) {
  const fc_model_config& c = m->cfg;
  const size_t D = c.hidden, M = c.mlp_dim, es = m->esz;
  Carver cv(base);
  auto lin = [&](Linear& L, int in, int out) {
    L.in = in; L.out = out;
    L.wt = cv.take((size_t)in * out * es);
    L.b = (float*)cv.take((size_t)out * 4);
  };
  lin(m->t1, c.t_embed_dim, D);
  lin(m->t2, D, D);
  lin(m->y, c.text_dim, D);
  m->p_w = (float*)cv.take((size_t)m->pd * D * 4);
  m->p_b = (float*)cv.take(D * 4);
  m->mod_w = cv.take((size_t)c.depth * m->nmod * D * D * es);
  m->mod_b = (float*)cv.take((size_t)c.depth * m->nmod * D * 4);
  m->blocks.resize(c.depth);
  for (int l = 0; l < c.depth; ++l) {
    Block& b = m->blocks[l];
    lin(b.qkv[0], D, 3 * D);
    lin(b.proj[0], D, D);
    if (c.attn_mode == FC_ATTN_FACTORIZED_CROSS) {
      lin(b.qkv[1], D, 3 * D);
      lin(b.proj[1], D, D);
      lin(b.xq, D, D);
      lin(b.xkv, D, 2 * D);
      lin(b.xproj, D, D);
    }
    lin(b.fc1, D, M);
    lin(b.fc2, M, D);
  }
  lin(m->fmod, D, 2 * D);
  lin(m->fout, D, m->pd);
  m->pos_sp = (float*)cv.take((size_t)m->S * D * 4);
  m->pos_t = (float*)cv.take((size_t)c.frames * D * 4);
  return cv.off;
}

void sincos_1d(double pos, int dim, float* out) {   // [sin(pos w_i) | cos(pos w_i)], w_i = 10000^(-i/(dim/2))
  const int half = dim / 2;
  for (int i = 0; i < half; ++i) {
    double w = std::pow(10000.0, -(double)i / (double)half);
    out[i] = (float)std::sin(pos * w);
    out[half + i] = (float)std::cos(pos * w);
  }
}

// ---------------------------------------------------------------- workspace
struct Workspace {
  float *e, *h1, *c, *mod, *fmod;          // timestep path, fp32
  void *txt, *y;                           // text in act dtype, projected text
  void *xk, *xv;                           // cross-attention K / V per block (factorized)
  float* x;                                // residual stream fp32 [B, Ns, D]
  void *u, *q, *k, *v, *hid;               // activations
  void* p[2];                              // gated branch outputs not yet added to x
  float* eps;                              // [B, T, H, W, C]
  float* knorm;                            // [B, heads, kKeyNormChunks] largest key norms (long-sequence attention)
  size_t bytes;
  int B, NT;
};

Workspace carve(const fc_model* m, int R, int use_cfg, unsigned char* base) {
  const fc_model_config& c = m->cfg;
  const size_t D = c.hidden, es = m->esz;
  Workspace w{};
  w.B = R * (use_cfg ? 2 : 1);
  w.NT = R + (use_cfg ? 1 : 0);                 // distinct texts: R prompts (+ the shared null)
  const size_t rows = (size_t)w.B * m->Ns;
  Carver cv(base);
  w.e = (float*)cv.take((size_t)c.t_embed_dim * 4);
  w.h1 = (float*)cv.take(D * 4);
  w.c = (float*)cv.take(D * 4);
  w.mod = (float*)cv.take((size_t)c.depth * m->nmod * D * 4);
  w.fmod = (float*)cv.take(2 * D * 4);
  w.txt = cv.take((size_t)w.NT * c.text_len * c.text_dim * es);
  w.y = cv.take((size_t)w.NT * c.text_len * D * es);
  if (c.attn_mode == FC_ATTN_FACTORIZED_CROSS) {
    w.xk = cv.take((size_t)c.depth * w.NT * c.text_len * D * es);
    w.xv = cv.take((size_t)c.depth * w.NT * c.text_len * D * es);
  }
  w.x = (float*)cv.take(rows * D * 4);
  w.u = cv.take(rows * D * es);
  w.q = cv.take(rows * D * es);
  w.k = cv.take(rows * D * es);
  w.v = cv.take(rows * D * es);
  w.hid = cv.take(rows * c.mlp_dim * es);
  w.p[0] = cv.take(rows * D * es);
  w.p[1] = cv.take(rows * D * es);
  w.eps = (float*)cv.take((size_t)w.B * c.frames * c.height * c.width * c.channels * 4);
  w.knorm = (float*)cv.take((size_t)w.B * c.heads * kKeyNormChunks * 4);
  w.bytes = cv.off;
  return w;
}

// ---------------------------------------------------------------- step building blocks
struct Ctx {
  fc_model* m;
  Workspace w;
  int R, use_cfg;
  hipStream_t s;
  // Gated branch outputs sit in w.p[0 .. npend), not yet added to the residual stream: the
  // next LayerNorm launch adds them to the row it holds in registers.  With one pending it
  // leaves x in memory as it is and keeps the branch pending; with two it writes the sum
  // back.  x (fp32) is thus written and read every other LayerNorm, for one more read of a
  // branch output of half its size; the additions and their order are those of adding each
  // branch as it arrives.
  mutable int npend = 0;
  // Gate the fold applies to each (NULL: the projection's epilogue has applied it already).
  // Used when the text rows have their own modulation set: the gate then depends on the row.
  mutable const float* pend_gate[2] = {nullptr, nullptr};
  int alt_rows() const { return m->cfg.text_adaln ? m->cfg.text_len : 0; }
  size_t act_bytes() const { return (size_t)w.B * m->Ns * m->cfg.hidden * m->esz; }   // one of u, q, k, v
  int alt_off() const { return 6 * m->cfg.hidden; }
};

struct ProfScope {        // records an event pair around the launches made in its lifetime
  Profiler* p = nullptr;
  hipStream_t s;
  hipEvent_t a = nullptr, b = nullptr;
  int cat;
  ProfScope(const Ctx& c, int cat_) : s(c.s), cat(cat_) {
    if (!c.m->prof.on || (c.m->prof.only >= 0 && c.m->prof.only != cat_)) return;
    p = &c.m->prof;
    a = p->get(); b = p->get();
    if (!a || !b) { p = nullptr; return; }
    (void)hipEventRecord(a, s);
  }
  ~ProfScope() {
    if (!p) return;
    (void)hipEventRecord(b, s);
    p->recs.push_back({a, b, cat});
  }
};

// scratch: a workspace buffer that is dead while this product runs (split-K partial tiles)
int linear(const Ctx& c, int cat, int mode, const void* A, const Linear& L, int M, EpiParams ep,
           void* scratch = nullptr, size_t scratch_bytes = 0) {
  ep.bias = L.b;
  ProfScope ps(c, cat);
  HIP_TRY(launch_gemm(c.m->bf16, mode, A, L.wt, M, L.out, L.in, ep, c.s, scratch, scratch_bytes));
  return FC_OK;
}

EpiParams heads_epi(const Ctx& c, void* q, void* k, void* v, int which0, int tokens) {
  EpiParams ep;
  ep.q = q; ep.k = k; ep.v = v;
  ep.which0 = which0;
  ep.D = c.m->cfg.hidden; ep.heads = c.m->cfg.heads; ep.hd = c.m->hd;
  ep.tokens = tokens;
  ep.qscale = (float)(1.4426950408889634 / std::sqrt((double)c.m->hd));
  return ep;
}

// Timestep-invariant work: text to the activation dtype, text projection, and (factorized
// mode) the cross-attention keys / values of every block.
int prepare(const Ctx& c, const float* cond, const float* null_cond) {
  const fc_model* m = c.m;
  const fc_model_config& cf = m->cfg;
  const Workspace& w = c.w;
  const size_t per_text = (size_t)cf.text_len * cf.text_dim;
  {
  ProfScope ps(c, PC_OTHER);
  HIP_TRY(launch_convert_f32(cond, w.txt, per_text * c.R, m->bf16, c.s));
  if (c.use_cfg)
    HIP_TRY(launch_convert_f32(null_cond, (unsigned char*)w.txt + per_text * c.R * m->esz, per_text, m->bf16, c.s));
  }
  EpiParams ep;
  ep.out = w.y; ep.ldo = cf.hidden;
  // few rows, long K: split along K through hid, which nothing uses before the first block's MLP
  int rc = linear(c, PC_GEMM_OTHER, EPI_STORE, w.txt, m->y, w.NT * cf.text_len, ep, w.hid,
                  (size_t)w.B * m->Ns * cf.mlp_dim * m->esz);
  if (rc != FC_OK) return rc;
  if (cf.attn_mode == FC_ATTN_FACTORIZED_CROSS) {
    for (int l = 0; l < cf.depth; ++l) {
      void* xk = (unsigned char*)w.xk + (size_t)l * w.NT * cf.text_len * cf.hidden * m->esz;
      void* xv = (unsigned char*)w.xv + (size_t)l * w.NT * cf.text_len * cf.hidden * m->esz;
      rc = linear(c, PC_GEMM_OTHER, EPI_HEADS, w.y, m->blocks[l].xkv, w.NT * cf.text_len,
                  heads_epi(c, nullptr, xk, xv, 1, cf.text_len));
      if (rc != FC_OK) return rc;
    }
  }
  return FC_OK;
}

int ln_mod(const Ctx& c, const float* shift, const float* scale) {
  const fc_model* m = c.m;
  ProfScope ps(c, PC_LN_MODULATE);
  const int np = c.npend;
  HIP_TRY(launch_ln_modulate(m->bf16, c.w.x, np > 0 ? c.w.p[0] : nullptr, np > 0 ? c.pend_gate[0] : nullptr,
                             np > 1 ? c.w.p[1] : nullptr, np > 1 ? c.pend_gate[1] : nullptr, shift, scale, c.w.u,
                             c.w.B * m->Ns, m->cfg.hidden, m->cfg.ln_eps, m->Ns, m->Ns, 0, c.alt_rows(), c.alt_off(),
                             np == 2, c.s));
  if (np == 2) c.npend = 0;
  return FC_OK;
}

// Branch output projection: y = gate * (A W + b) into the next free pending buffer (the
// LayerNorm that opened this branch has left at most one in use).
int branch_out(const Ctx& c, int cat, const void* A, const Linear& L, const float* gate) {
  if (c.npend > 1) return fail(FC_ERR_STATE, "no free buffer for a branch output");
  EpiParams ep;
  const bool by_row = c.m->cfg.text_adaln != 0;      // the fold picks the row's gate instead
  ep.out = c.w.p[c.npend]; ep.ldo = c.m->cfg.hidden; ep.gate = by_row ? nullptr : gate;
  // k is dead by now (attention is over; the MLP never used it) and is neither operand nor output here
  int rc = linear(c, cat, EPI_GATE, A, L, c.w.B * c.m->Ns, ep, c.w.k, c.act_bytes());
  if (rc != FC_OK) return rc;
  c.pend_gate[c.npend] = by_row ? gate : nullptr;
  ++c.npend;
  return FC_OK;
}

// Self-attention branch: x += gate * proj(attn(qkv(u))).  mode 0 spatial, 1 temporal, 2 all tokens.
int self_attention_branch(const Ctx& c, const Linear& qkv, const Linear& proj, const float* gate, int mode) {
  const fc_model* m = c.m;
  const fc_model_config& cf = m->cfg;
  const Workspace& w = c.w;
  const int rows = w.B * m->Ns;
  // hid is dead between the MLP of the previous block and this block's MLP
  int rc = linear(c, PC_GEMM_QKV, EPI_HEADS, w.u, qkv, rows, heads_epi(c, w.q, w.k, w.v, 0, m->Ns), w.hid,
                  (size_t)rows * cf.mlp_dim * m->esz);
  if (rc != FC_OK) return rc;
  AttnParams ap{};
  ap.q = w.q; ap.k = w.k; ap.v = w.v; ap.out = w.u;
  ap.B = w.B; ap.heads = cf.heads; ap.hd = m->hd;
  ap.q_tokens = ap.k_tokens = m->Ns;
  if (mode == 0) { ap.groups = cf.frames; ap.nq = ap.nk = m->S; ap.q_gstride = ap.k_gstride = m->S; ap.q_istride = ap.k_istride = 1; }
  else if (mode == 1) { ap.groups = m->S; ap.nq = ap.nk = cf.frames; ap.q_gstride = ap.k_gstride = 1; ap.q_istride = ap.k_istride = m->S; }
  else { ap.groups = 1; ap.nq = ap.nk = m->Ns; ap.q_gstride = ap.k_gstride = 0; ap.q_istride = ap.k_istride = 1; }
  ap.kv_split = 0; ap.kv_shared_tail = 0;
  ap.scale_log2 = 1.0f;                  // q was stored pre-scaled by the QKV epilogue
  {
    ProfScope ps(c, mode == 0 ? PC_ATTN_SPATIAL : mode == 1 ? PC_ATTN_TEMPORAL : PC_ATTN_FULL);
    if (attention_uses_key_norms(m->bf16, ap)) {
      // long sequences: the largest key norm per head bounds every score, which lets the
      // attention kernel drop its per-tile maximum
      HIP_TRY(launch_key_norm_max(w.k, w.B, cf.heads, m->Ns, m->hd, w.knorm, c.s));
      ap.key_norm_max = w.knorm;
    }
    HIP_TRY(launch_attention(m->bf16, ap, 0, c.s));
  }
  return branch_out(c, PC_GEMM_PROJ, w.u, proj, gate);
}

int cross_attention_branch(const Ctx& c, const Block& b, int layer) {
  const fc_model* m = c.m;
  const fc_model_config& cf = m->cfg;
  const Workspace& w = c.w;
  const int rows = w.B * m->Ns;
  int rc = ln_mod(c, nullptr, nullptr);
  if (rc != FC_OK) return rc;
  rc = linear(c, PC_GEMM_PROJ, EPI_HEADS, w.u, b.xq, rows, heads_epi(c, w.q, nullptr, nullptr, 0, m->Ns));
  if (rc != FC_OK) return rc;
  AttnParams ap{};
  ap.q = w.q;
  ap.k = (unsigned char*)w.xk + (size_t)layer * w.NT * cf.text_len * cf.hidden * m->esz;
  ap.v = (unsigned char*)w.xv + (size_t)layer * w.NT * cf.text_len * cf.hidden * m->esz;
  ap.out = w.u;
  ap.B = w.B; ap.heads = cf.heads; ap.hd = m->hd;
  ap.groups = 1; ap.nq = m->Ns; ap.nk = cf.text_len;
  ap.q_tokens = m->Ns; ap.q_gstride = 0; ap.q_istride = 1;
  ap.k_tokens = cf.text_len; ap.k_gstride = 0; ap.k_istride = 1;
  ap.kv_split = c.R; ap.kv_shared_tail = c.use_cfg;      // guidance rows all read the null text
  ap.scale_log2 = 1.0f;
  {
    ProfScope ps(c, PC_ATTN_CROSS);
    HIP_TRY(launch_attention(m->bf16, ap, 0, c.s));
  }
  return branch_out(c, PC_GEMM_PROJ, w.u, b.xproj, nullptr);
}

int mlp_branch(const Ctx& c, const Block& b, const float* mod) {
  const fc_model* m = c.m;
  const int D = m->cfg.hidden, rows = c.w.B * m->Ns;
  int rc = ln_mod(c, mod, mod + D);
  if (rc != FC_OK) return rc;
  EpiParams e1;
  e1.out = c.w.hid; e1.ldo = m->cfg.mlp_dim;
  rc = linear(c, PC_GEMM_FC1, EPI_GELU, c.w.u, b.fc1, rows, e1, c.w.k, c.act_bytes());   // q, k, v are dead here
  if (rc != FC_OK) return rc;
  return branch_out(c, PC_GEMM_FC2, c.w.hid, b.fc2, mod + 2 * D);
}

// One forward pass of all B rows + guidance + DDIM update of the R latents.
int run_step(const Ctx& c, float* latent, const fc_schedule* sched, int step, float* eps_out) {
  fc_model* m = c.m;
  const fc_model_config& cf = m->cfg;
  const Workspace& w = c.w;
  const int D = cf.hidden;
  float coef[4], sigma = 0.0f;
  int t = 0;
  int rc = step_coefficients(sched, step, coef, &t, &sigma);
  if (rc != FC_OK) return rc;

  // conditioning: sinusoid -> Linear -> SiLU -> Linear -> c; every adaLN layer reads SiLU(c)
  const int nm = m->nmod * D;
  {
  ProfScope ps(c, PC_TIMESTEP_MOD);
  HIP_TRY(launch_sinusoid((float)t, cf.t_embed_dim, w.e, c.s));
  HIP_TRY(launch_gemv(m->bf16, w.e, cf.t_embed_dim, m->t1.wt, m->t1.b, w.h1, D, 0, 1, 1, 0, 0, 0, c.s));
  HIP_TRY(launch_gemv(m->bf16, w.h1, D, m->t2.wt, m->t2.b, w.c, D, 0, 0, 1, 0, 0, 0, c.s));
  // the blocks' modulation vectors and the final layer's, both from SiLU(c): one launch
  if (cf.depth > 0)
    HIP_TRY(launch_gemv(m->bf16, w.c, D, m->mod_w, m->mod_b, w.mod, nm, 1, 0, cf.depth, (size_t)nm * D, nm, nm, c.s,
                        m->fmod.wt, m->fmod.b, w.fmod, 2 * D));
  else
    HIP_TRY(launch_gemv(m->bf16, w.c, D, m->fmod.wt, m->fmod.b, w.fmod, 2 * D, 1, 0, 1, 0, 0, 0, c.s));
  }

  // tokens
  const int text_rows = cf.attn_mode == FC_ATTN_FULL3D_CONCAT ? cf.text_len : 0;
  {
  ProfScope ps(c, PC_PATCH_EMBED);
  // an fp32 model keeps fp32 arithmetic: the matrix-core kernel (bf16 high/low splits) is for bf16 models only
  HIP_TRY(launch_patch_embed(latent, c.R, w.B, m->p_w, m->p_b, m->pos_sp, m->pos_t, w.x, cf.frames, cf.height,
                             cf.width, cf.channels, cf.patch, D, m->Ns, text_rows, m->bf16 ? 0 : 1, c.s));
  if (text_rows)
    HIP_TRY(launch_act_to_f32_rows(m->bf16, w.y, w.x, w.B * cf.text_len, D, cf.text_len, m->Ns, 0, c.R, c.use_cfg,
                                   c.s));
  }

  for (int l = 0; l < cf.depth; ++l) {
    const Block& b = m->blocks[l];
    const float* mod = w.mod + (size_t)l * nm;
    if (cf.attn_mode == FC_ATTN_FACTORIZED_CROSS) {
      for (int br = 0; br < 2; ++br) {
        const float* mv = mod + (size_t)br * 3 * D;
        if ((rc = ln_mod(c, mv, mv + D)) != FC_OK) return rc;
        if ((rc = self_attention_branch(c, b.qkv[br], b.proj[br], mv + 2 * D, br)) != FC_OK) return rc;
      }
      if ((rc = cross_attention_branch(c, b, l)) != FC_OK) return rc;
      if ((rc = mlp_branch(c, b, mod + 6 * D)) != FC_OK) return rc;
    } else {
      if ((rc = ln_mod(c, mod, mod + D)) != FC_OK) return rc;
      if ((rc = self_attention_branch(c, b.qkv[0], b.proj[0], mod + 2 * D, 2)) != FC_OK) return rc;
      if ((rc = mlp_branch(c, b, mod + 3 * D)) != FC_OK) return rc;
    }
  }

  // head: LN + modulate on the video rows, Linear D -> p*p*C, scatter back to latent layout
  {
  ProfScope ps(c, PC_LN_MODULATE);
  const int np = c.npend;
  HIP_TRY(launch_ln_modulate(m->bf16, w.x, np > 0 ? w.p[0] : nullptr, np > 0 ? c.pend_gate[0] : nullptr,
                             np > 1 ? w.p[1] : nullptr, np > 1 ? c.pend_gate[1] : nullptr, w.fmod, w.fmod + D, w.u,
                             w.B * m->N, D, cf.ln_eps, m->Ns, m->N, text_rows, 0, 0, 0, c.s));
  c.npend = 0;
  }
  EpiParams ep;
  ep.eps = w.eps; ep.T = cf.frames; ep.H = cf.height; ep.W = cf.width; ep.C = cf.channels; ep.p = cf.patch;
  if ((rc = linear(c, PC_GEMM_OTHER, EPI_UNPATCH, w.u, m->fout, w.B * m->N, ep, w.k, c.act_bytes())) != FC_OK) return rc;   // q, k, v are dead here

  const size_t n = (size_t)c.R * cf.frames * cf.height * cf.width * cf.channels;
  ProfScope ps(c, PC_CFG_DDIM);
  if (sigma > 0.0f)
    HIP_TRY(launch_cfg_ddim_noise(latent, w.eps, c.use_cfg ? w.eps + n : nullptr, eps_out, n / c.R, c.R,
                                  sched->guidance_scale, coef[0], coef[1], coef[2], coef[3], sigma, sched->seed, step,
                                  c.s));
  else
    HIP_TRY(launch_cfg_ddim(latent, w.eps, c.use_cfg ? w.eps + n : nullptr, eps_out, n, sched->guidance_scale,
                            coef[0], coef[1], coef[2], coef[3], c.s));
  return FC_OK;
}

int check_call(fc_model* m, const float* latent, const float* cond, const fc_schedule* sched, int R,
               void* workspace, size_t workspace_bytes, int use_cfg, Ctx* ctx, void* stream) {
  if (!m || !latent || !cond || !sched || !workspace) return fail(FC_ERR_NULL, "NULL argument");
  if (!m->has_weights) return fail(FC_ERR_STATE, "fc_model_set_weights has not been called");
  int rc = schedule_check(sched);
  if (rc != FC_OK) return rc;
  if (R < 1) return fail(FC_ERR_RANGE, "batch_requests must be >= 1");
  const long long B = (long long)R * (use_cfg ? 2 : 1);
  if (B * m->Ns > (long long)INT32_MAX / 4) return fail(FC_ERR_RANGE, "batch too large");
  // the epilogues split a row index m into (batch row, token) by multiply-shift, exact while
  // m * divisor < 2^40 with m < B * Ns and the divisor Ns (q/k/v scatter) or T * S (un-patchify)
  if (B * m->Ns * m->Ns >= (1ll << 40))
    return fail(FC_ERR_RANGE, "batch_requests * tokens^2 must stay below 2^40");
  if (((uintptr_t)workspace & 255) != 0) return fail(FC_ERR_WORKSPACE, "workspace must be 256-byte aligned");
  Workspace w = carve(m, R, use_cfg, (unsigned char*)workspace);
  if (w.bytes > workspace_bytes) return fail(FC_ERR_WORKSPACE, "workspace smaller than fc_workspace_bytes()");
  ctx->m = m; ctx->w = w; ctx->R = R; ctx->use_cfg = use_cfg; ctx->s = (hipStream_t)stream;
  return FC_OK;
}

}  // namespace

// ================================================================ C ABI
extern "C" {

int fc_model_create(const fc_model_config* cfg, fc_model** out) {
  if (!cfg || !out) return fail(FC_ERR_NULL, "NULL argument");
  *out = nullptr;
  const fc_model_config& c = *cfg;
  if (c.frames < 1 || c.height < 1 || c.width < 1 || c.channels < 1 || c.patch < 1 || c.hidden < 1 ||
      c.heads < 1 || c.mlp_dim < 1 || c.depth < 0 || c.text_len < 1 || c.text_dim < 1 || c.t_embed_dim < 2)
    return fail(FC_ERR_SHAPE, "non-positive dimension");
  if (c.height % c.patch || c.width % c.patch) return fail(FC_ERR_SHAPE, "height/width not divisible by patch");
  if (c.hidden % c.heads) return fail(FC_ERR_SHAPE, "hidden not divisible by heads");
  if (c.hidden % 4 || c.hidden > 4096 || c.t_embed_dim % 2)
    return fail(FC_ERR_SHAPE, "hidden must be a multiple of 4, at most 4096; t_embed_dim even");
  if (c.attn_mode != FC_ATTN_FACTORIZED_CROSS && c.attn_mode != FC_ATTN_FULL3D_CONCAT)
    return fail(FC_ERR_SHAPE, "unknown attn_mode");
  if (c.dtype != FC_F32 && c.dtype != FC_BF16) return fail(FC_ERR_SHAPE, "unknown dtype");
  if (c.text_adaln != 0 && c.text_adaln != 1) return fail(FC_ERR_SHAPE, "text_adaln must be 0 or 1");
  if (c.text_adaln && c.attn_mode != FC_ATTN_FULL3D_CONCAT)
    return fail(FC_ERR_SHAPE, "text_adaln needs the full-3D mode (text rows are not in the sequence otherwise)");
  const int hd = c.hidden / c.heads;
  const int ok_hd[] = {8, 16, 32, 64, 72, 96, 128};
  bool hd_ok = false;
  for (int v : ok_hd) hd_ok |= (v == hd);
  if (!hd_ok) return fail(FC_ERR_SHAPE, "head dim must be one of 8,16,32,64,72,96,128");
  if (!(c.ln_eps >= 0.0f)) return fail(FC_ERR_SHAPE, "ln_eps must be >= 0");
  int dev = 0;
  HIP_TRY(hipGetDevice(&dev));
  fc_model* m = new fc_model();
  m->cfg = c;
  m->device = dev;
  m->bf16 = c.dtype == FC_BF16;
  m->esz = m->bf16 ? 2 : 4;
  m->S = (c.height / c.patch) * (c.width / c.patch);
  m->N = c.frames * m->S;
  m->Ns = m->N + (c.attn_mode == FC_ATTN_FULL3D_CONCAT ? c.text_len : 0);
  m->pd = c.patch * c.patch * c.channels;
  m->hd = hd;
  m->nmod = c.attn_mode == FC_ATTN_FACTORIZED_CROSS ? 9 : c.text_adaln ? 12 : 6;
  *out = m;
  return FC_OK;
}

int fc_model_weight_count(const fc_model* m, size_t* out) {
  if (!m || !out) return fail(FC_ERR_NULL, "NULL argument");
  *out = weight_count(m->cfg);
  return FC_OK;
}

int fc_model_set_weights(fc_model* m, const float* blob, size_t n_floats) {
  if (!m || !blob) return fail(FC_ERR_NULL, "NULL argument");
  if (n_floats != weight_count(m->cfg)) return fail(FC_ERR_SHAPE, "weight blob has the wrong number of floats");
  const fc_model_config& c = m->cfg;
  const int D = c.hidden;
  if (m->wbuf) { (void)hipFree(m->wbuf); m->wbuf = nullptr; m->has_weights = false; }
  m->wbytes = layout_weights(m, nullptr);
  HIP_TRY(hipMalloc((void**)&m->wbuf, m->wbytes));
  layout_weights(m, m->wbuf);

  // staging buffer for one tensor at a time (largest matrix of the model)
  size_t big = (size_t)D * std::max(std::max(3 * D, c.mlp_dim), std::max(c.text_dim, m->nmod * D));
  big = std::max(big, (size_t)c.t_embed_dim * D);
  float* stage = nullptr;
  HIP_TRY(hipMalloc((void**)&stage, big * 4));
  size_t off = 0;
  int rc = FC_OK;
  auto up_matrix_t = [&](void* dst, int in, int out) -> hipError_t {   // blob [in,out] -> device [out,in] act dtype
    hipError_t e = hipMemcpy(stage, blob + off, (size_t)in * out * 4, hipMemcpyHostToDevice);
    if (e != hipSuccess) return e;
    off += (size_t)in * out;
    e = launch_transpose_convert(stage, dst, in, out, m->bf16, nullptr);
    if (e != hipSuccess) return e;
    return hipDeviceSynchronize();
  };
  auto up_f32 = [&](float* dst, size_t n) -> hipError_t {
    hipError_t e = hipMemcpy(dst, blob + off, n * 4, hipMemcpyHostToDevice);
    off += n;
    return e;
  };
  auto up_lin = [&](Linear& L) -> hipError_t {
    hipError_t e = up_matrix_t(L.wt, L.in, L.out);
    if (e != hipSuccess) return e;
    return up_f32(L.b, L.out);
  };
#define UP(expr)                                                          \
  do {                                                                    \
    hipError_t _e = (expr);                                               \
    if (_e != hipSuccess) { rc = fail_hip(_e, #expr); goto done; }        \
  } while (0)
  UP(up_lin(m->t1));
  UP(up_lin(m->t2));
  UP(up_lin(m->y));
  UP(up_f32(m->p_w, (size_t)m->pd * D));
  UP(up_f32(m->p_b, D));
  for (int l = 0; l < c.depth; ++l) {
    Block& b = m->blocks[l];
    const size_t nm = (size_t)m->nmod * D;
    UP(up_matrix_t((unsigned char*)m->mod_w + (size_t)l * nm * D * m->esz, D, (int)nm));
    UP(up_f32(m->mod_b + (size_t)l * nm, nm));
    UP(up_lin(b.qkv[0]));
    UP(up_lin(b.proj[0]));
    if (c.attn_mode == FC_ATTN_FACTORIZED_CROSS) {
      UP(up_lin(b.qkv[1]));
      UP(up_lin(b.proj[1]));
      UP(up_lin(b.xq));
      UP(up_lin(b.xkv));
      UP(up_lin(b.xproj));
    }
    UP(up_lin(b.fc1));
    UP(up_lin(b.fc2));
  }
  UP(up_lin(m->fmod));
  UP(up_lin(m->fout));
  {
    // positional tables, computed in double: spatial [S, D] = [sincos(h') | sincos(w')], temporal [T, D]
    const int gw = c.width / c.patch;
    std::vector<float> sp((size_t)m->S * D), tp((size_t)c.frames * D);
    for (int s = 0; s < m->S; ++s) {
      sincos_1d((double)(s / gw), D / 2, &sp[(size_t)s * D]);
      sincos_1d((double)(s % gw), D / 2, &sp[(size_t)s * D + D / 2]);
    }
    for (int t = 0; t < c.frames; ++t) sincos_1d((double)t, D, &tp[(size_t)t * D]);
    UP(hipMemcpy(m->pos_sp, sp.data(), sp.size() * 4, hipMemcpyHostToDevice));
    UP(hipMemcpy(m->pos_t, tp.data(), tp.size() * 4, hipMemcpyHostToDevice));
  }
  UP(hipDeviceSynchronize());
  m->has_weights = true;
done:
#undef UP
  (void)hipFree(stage);
  return rc;
}

int fc_model_destroy(fc_model* m) {
  if (!m) return FC_OK;
  if (m->wbuf) (void)hipFree(m->wbuf);
  delete m;
  return FC_OK;
}

int fc_workspace_bytes(const fc_model* m, int32_t R, int32_t use_cfg, size_t* out) {
  if (!m || !out) return fail(FC_ERR_NULL, "NULL argument");
  if (R < 1) return fail(FC_ERR_RANGE, "batch_requests must be >= 1");
  *out = carve(m, R, use_cfg != 0, nullptr).bytes;
  return FC_OK;
}

int fc_denoise_step(fc_model* m, float* latent, const float* cond, const float* null_cond, const fc_schedule* sched,
                    int32_t step, int32_t R, float* eps_out, void* workspace, size_t workspace_bytes, void* stream) {
  Ctx ctx;
  int rc = check_call(m, latent, cond, sched, R, workspace, workspace_bytes, null_cond != nullptr, &ctx, stream);
  if (rc != FC_OK) return rc;
  if (step < 1 || step > sched->num_steps) return fail(FC_ERR_RANGE, "step must be in 1..num_steps");
  if ((rc = prepare(ctx, cond, null_cond)) != FC_OK) return rc;
  return run_step(ctx, latent, sched, step, eps_out);
}

int fc_denoise_resume_ex(fc_model* m, float* latent, const float* cond, const float* null_cond,
                         const fc_schedule* sched, int32_t k, int32_t R, int32_t n_export,
                         const int32_t* export_steps, float* const* export_dst, void* workspace,
                         size_t workspace_bytes, void* stream) {
  Ctx ctx;
  int rc = check_call(m, latent, cond, sched, R, workspace, workspace_bytes, null_cond != nullptr, &ctx, stream);
  if (rc != FC_OK) return rc;
  if (k < 0 || k > sched->num_steps) return fail(FC_ERR_RANGE, "k must be in 0..num_steps");
  if (n_export < 0) return fail(FC_ERR_RANGE, "n_export is negative");
  if (n_export > 0 && (!export_steps || !export_dst)) return fail(FC_ERR_NULL, "export arrays are NULL");
  for (int e = 0; e < n_export; ++e) {
    if (export_steps[e] <= k || export_steps[e] > sched->num_steps)
      return fail(FC_ERR_RANGE, "export steps must lie in k+1..num_steps");
    if (e > 0 && export_steps[e] <= export_steps[e - 1]) return fail(FC_ERR_RANGE, "export steps must ascend");
    if (!export_dst[e]) return fail(FC_ERR_NULL, "export destination is NULL");
  }
  if (k == sched->num_steps) return FC_OK;
  if ((rc = prepare(ctx, cond, null_cond)) != FC_OK) return rc;
  const fc_model_config& cf = m->cfg;
  const size_t lat_elems = (size_t)R * cf.frames * cf.height * cf.width * cf.channels;
  int next = 0;
  for (int s = k + 1; s <= sched->num_steps; ++s) {
    if ((rc = run_step(ctx, latent, sched, s, nullptr)) != FC_OK) return rc;
    if (next < n_export && export_steps[next] == s) {
      // stream-ordered device copy: the next step reads the latent after it, nothing waits on the host
      HIP_TRY(launch_copy_f32(latent, export_dst[next], lat_elems, ctx.s));
      ++next;
    }
  }
  return FC_OK;
}

int fc_denoise_resume(fc_model* m, float* latent, const float* cond, const float* null_cond,
                      const fc_schedule* sched, int32_t k, int32_t R, void* workspace, size_t workspace_bytes,
                      void* stream) {
  return fc_denoise_resume_ex(m, latent, cond, null_cond, sched, k, R, 0, nullptr, nullptr, workspace, workspace_bytes,
                              stream);
}

int fc_schedule_coefficients(const fc_schedule* sched, int32_t step, float* out4, int32_t* t_out) {
  if (!out4) return fail(FC_ERR_NULL, "NULL argument");
  int t = 0;
  int rc = step_coefficients(sched, step, out4, &t);
  if (rc == FC_OK && t_out) *t_out = t;
  return rc;
}

const char* fc_status_string(int status) {
  switch (status) {
    case FC_OK: return "ok";
    case FC_ERR_NULL: return "null pointer";
    case FC_ERR_SHAPE: return "bad shape or configuration";
    case FC_ERR_RANGE: return "argument out of range";
    case FC_ERR_WORKSPACE: return "workspace too small or misaligned";
    case FC_ERR_DEVICE: return "HIP error";
    case FC_ERR_UNSUPPORTED: return "unsupported";
    case FC_ERR_STATE: return "weights not set";
  }
  return "unknown status";
}

const char* fc_last_error(void) { return g_err.c_str(); }

int fc_profile_enable(fc_model* m, int32_t enable) {
  if (!m) return fail(FC_ERR_NULL, "NULL argument");
  m->prof.release_all();
  m->prof.on = enable != 0;
  return FC_OK;
}

int fc_profile_select(fc_model* m, int32_t category) {
  if (!m) return fail(FC_ERR_NULL, "NULL argument");
  if (category < -1 || category >= PC_COUNT) return fail(FC_ERR_RANGE, "no such profile category");
  m->prof.only = category;
  return FC_OK;
}

int fc_profile_categories(void) { return PC_COUNT; }

const char* fc_profile_category_name(int32_t i) { return (i >= 0 && i < PC_COUNT) ? kProfNames[i] : ""; }

int fc_profile_read(fc_model* m, int32_t n, double* ms_out, int64_t* launches_out) {
  if (!m || !ms_out || !launches_out) return fail(FC_ERR_NULL, "NULL argument");
  if (n < PC_COUNT) return fail(FC_ERR_RANGE, "need room for fc_profile_categories() entries");
  for (int i = 0; i < n; ++i) { ms_out[i] = 0.0; launches_out[i] = 0; }
  for (auto& r : m->prof.recs) {
    HIP_TRY(hipEventSynchronize(r.b));
    float ms = 0.0f;
    HIP_TRY(hipEventElapsedTime(&ms, r.a, r.b));
    ms_out[r.cat] += ms;
    launches_out[r.cat] += 1;
  }
  m->prof.release_all();
  return FC_OK;
}

// ---------------------------------------------------------------- single operators
int fc_op_linear(int32_t dtype, const void* A, const void* Wt, const float* bias, const float* gate, void* out,
                 int32_t M, int32_t N, int32_t K, int32_t epilogue, void* stream) {
  if (!A || !Wt || !out) return fail(FC_ERR_NULL, "NULL argument");
  if (M < 0 || N < 0 || K < 0 || epilogue < 0 || epilogue > 2) return fail(FC_ERR_RANGE, "bad size or epilogue");
  EpiParams ep;
  ep.bias = bias; ep.out = out; ep.ldo = N; ep.gate = gate;
  const int mode = epilogue == 0 ? EPI_STORE : epilogue == 1 ? EPI_GELU : EPI_GATE;
  HIP_TRY(launch_gemm(dtype == FC_BF16, mode, A, Wt, M, N, K, ep, (hipStream_t)stream));
  return FC_OK;
}

int fc_op_linear_scratch(int32_t dtype, const void* A, const void* Wt, const float* bias, const float* gate, void* out,
                         int32_t M, int32_t N, int32_t K, int32_t epilogue, void* scratch, size_t scratch_bytes,
                         void* stream) {
  if (!A || !Wt || !out) return fail(FC_ERR_NULL, "NULL argument");
  if (M < 0 || N < 0 || K < 0 || epilogue < 0 || epilogue > 2) return fail(FC_ERR_RANGE, "bad size or epilogue");
  if (scratch && ((uintptr_t)scratch & 15) != 0) return fail(FC_ERR_RANGE, "scratch must be 16-byte aligned");
  EpiParams ep;
  ep.bias = bias; ep.out = out; ep.ldo = N; ep.gate = gate;
  const int mode = epilogue == 0 ? EPI_STORE : epilogue == 1 ? EPI_GELU : EPI_GATE;
  HIP_TRY(launch_gemm(dtype == FC_BF16, mode, A, Wt, M, N, K, ep, (hipStream_t)stream, scratch, scratch_bytes));
  return FC_OK;
}

int fc_op_attention(int32_t dtype, const void* q, const void* k, const void* v, void* out, int32_t G, int32_t nq,
                    int32_t nk, int32_t d, int32_t impl, void* stream) {
  if (!q || !k || !v || !out) return fail(FC_ERR_NULL, "NULL argument");
  if (G < 0 || nq < 0 || nk < 1 || d < 1) return fail(FC_ERR_RANGE, "bad size");
  AttnParams ap{};
  ap.q = q; ap.k = k; ap.v = v; ap.out = out;
  ap.B = G; ap.heads = 1; ap.hd = d;
  ap.groups = 1; ap.nq = nq; ap.nk = nk;
  ap.q_tokens = nq; ap.q_gstride = 0; ap.q_istride = 1;
  ap.k_tokens = nk; ap.k_gstride = 0; ap.k_istride = 1;
  if (impl < 0 || impl > 2) return fail(FC_ERR_RANGE, "impl must be 0, 1 or 2");
  // impl 2: q already carries the factor, as the QKV epilogue of a step leaves it
  ap.scale_log2 = impl == 2 ? 1.0f : (float)(1.4426950408889634 / std::sqrt((double)d));
  hipError_t e = launch_attention(dtype == FC_BF16, ap, impl == 2 ? 0 : impl, (hipStream_t)stream);
  if (e == hipErrorInvalidValue) return fail(FC_ERR_UNSUPPORTED, "head dim not supported or pointers not 16-byte aligned");
  HIP_TRY(e);
  return FC_OK;
}

int fc_op_attention_bounded(const void* q, const void* k, const void* v, void* out, int32_t G, int32_t nq, int32_t nk,
                            int32_t d, float* key_norm_scratch, void* stream) {
  if (!q || !k || !v || !out || !key_norm_scratch) return fail(FC_ERR_NULL, "NULL argument");
  if (G < 0 || G > 65535 || nq < 0 || nk < 1) return fail(FC_ERR_RANGE, "bad size");
  if (d != 64 && d != 72) return fail(FC_ERR_UNSUPPORTED, "head dim must be 64 or 72");
  AttnParams ap{};
  ap.q = q; ap.k = k; ap.v = v; ap.out = out;
  ap.B = G; ap.heads = 1; ap.hd = d;
  ap.groups = 1; ap.nq = nq; ap.nk = nk;
  ap.q_tokens = nq; ap.q_gstride = 0; ap.q_istride = 1;
  ap.k_tokens = nk; ap.k_gstride = 0; ap.k_istride = 1;
  ap.scale_log2 = 1.0f;
  if ((((uintptr_t)q | (uintptr_t)k | (uintptr_t)v | (uintptr_t)out) & 15) != 0)
    return fail(FC_ERR_UNSUPPORTED, "pointers not 16-byte aligned");
  HIP_TRY(launch_key_norm_max(k, G, 1, nk, d, key_norm_scratch, (hipStream_t)stream));
  ap.key_norm_max = key_norm_scratch;
  HIP_TRY(launch_attention(1, ap, 0, (hipStream_t)stream));
  return FC_OK;
}

int fc_op_layernorm_modulate(int32_t dtype, float* x, const void* y, const float* shift, const float* scale,
                             void* out, int32_t M, int32_t D, float eps, void* stream) {
  if (!x || !out) return fail(FC_ERR_NULL, "NULL argument");
  if ((shift == nullptr) != (scale == nullptr)) return fail(FC_ERR_NULL, "shift and scale go together");
  if (M < 0 || D < 4 || D % 4 || D > 4096) return fail(FC_ERR_RANGE, "D must be a multiple of 4 in 4..4096");
  HIP_TRY(launch_ln_modulate(dtype == FC_BF16, x, y, nullptr, nullptr, nullptr, shift, scale, out, M, D, eps, M > 0 ? M : 1, M > 0 ? M : 1, 0, 0, 0, 1,
                             (hipStream_t)stream));
  return FC_OK;
}

int fc_op_layernorm_residual2(int32_t dtype, float* x, const void* y, const float* gate, const void* y2,
                              const float* gate2, const float* shift, const float* scale, void* out, int32_t M,
                              int32_t D, float eps, int32_t write_x, void* stream) {
  if (!x || !out) return fail(FC_ERR_NULL, "NULL argument");
  if ((shift == nullptr) != (scale == nullptr)) return fail(FC_ERR_NULL, "shift and scale go together");
  if (y2 && !y) return fail(FC_ERR_NULL, "y2 is given without y");
  if ((gate && !y) || (gate2 && !y2)) return fail(FC_ERR_NULL, "a gate is given without its branch output");
  if (M < 0 || D < 4 || D % 4 || D > 4096) return fail(FC_ERR_RANGE, "D must be a multiple of 4 in 4..4096");
  HIP_TRY(launch_ln_modulate(dtype == FC_BF16, x, y, gate, y2, gate2, shift, scale, out, M, D, eps, M > 0 ? M : 1,
                             M > 0 ? M : 1, 0, 0, 0, write_x != 0, (hipStream_t)stream));
  return FC_OK;
}

int fc_op_patch_embed(const float* latent, int32_t R, int32_t B, const float* Wp, const float* bp, const float* pos_sp,
                      const float* pos_t, float* x, int32_t T, int32_t H, int32_t W, int32_t C, int32_t p, int32_t D,
                      int32_t rows_per_b, int32_t row_off, int32_t impl, void* stream) {
  if (!latent || !Wp || !bp || !pos_sp || !pos_t || !x) return fail(FC_ERR_NULL, "NULL argument");
  if (R < 1 || B < 0 || T < 1 || H < 1 || W < 1 || C < 1 || p < 1 || H % p || W % p || D < 4 || D % 4 || row_off < 0 ||
      rows_per_b < row_off + T * (H / p) * (W / p) || impl < 0 || impl > 2)
    return fail(FC_ERR_RANGE, "bad patch embedding shape");
  if (impl == 2 && !(p == 2 && C == 16 && D % 256 == 0))
    return fail(FC_ERR_UNSUPPORTED, "the matrix-core patch embedding needs p = 2, C = 16, D % 256 = 0");
  HIP_TRY(launch_patch_embed(latent, R, B, Wp, bp, pos_sp, pos_t, x, T, H, W, C, p, D, rows_per_b, row_off, impl,
                             (hipStream_t)stream));
  return FC_OK;
}

// ---------------------------------------------------------------- restoring a cached latent
int fc_cache_stitch(const float* x_obj, const float* x_bg, const uint8_t* m_obj, const uint8_t* m_bg, float* out,
                    int64_t pixels, int32_t channels, void* stream) {
  if (!x_obj || !x_bg || !m_obj || !out) return fail(FC_ERR_NULL, "NULL argument");
  if (pixels < 0 || channels < 1) return fail(FC_ERR_RANGE, "bad pixel or channel count");
  HIP_TRY(launch_stitch(x_obj, x_bg, m_obj, m_bg, out, pixels, channels, (hipStream_t)stream));
  return FC_OK;
}

int fc_cache_decompress(const float* first, const float* diff_base, int32_t n_base, float alpha, const float* extra,
                        int32_t n_extra, const int32_t* src, int32_t frames, int64_t frame_elems, float* out,
                        void* stream) {
  if (!first || !src || !out) return fail(FC_ERR_NULL, "NULL argument");
  if (n_base < 0 || n_extra < 0 || frames < 0 || frame_elems < 0) return fail(FC_ERR_RANGE, "negative size");
  if (frames > kMaxCacheFrames) return fail(FC_ERR_UNSUPPORTED, "more than 256 frames in one entry");
  if ((n_base > 0 && !diff_base) || (n_extra > 0 && !extra)) return fail(FC_ERR_NULL, "NULL frame array");
  for (int t = 0; t < frames; ++t)
    if (src[t] > n_base || src[t] < -n_extra) return fail(FC_ERR_RANGE, "source code names a frame the entry does not hold");
  HIP_TRY(launch_decompress(first, diff_base, alpha, extra, src, frames, frame_elems, out, (hipStream_t)stream));
  return FC_OK;
}

size_t fc_cache_workspace_bytes(int32_t frames) {
  const size_t gram = (size_t)(frames > 0 ? frames : 0) * (size_t)(frames > 0 ? frames : 0) * sizeof(double);
  return gram > kCacheReduceWsBytes ? gram : kCacheReduceWsBytes;
}

int fc_cache_alpha(const float* first_s, const float* keys_s, const float* diff_base, int32_t n_base,
                   int64_t frame_elems, float* alpha_out, void* workspace, size_t workspace_bytes, void* stream) {
  if (!first_s || !keys_s || !diff_base || !alpha_out || !workspace) return fail(FC_ERR_NULL, "NULL argument");
  if (n_base < 1 || frame_elems < 1) return fail(FC_ERR_RANGE, "needs at least one base frame");
  if (workspace_bytes < kCacheReduceWsBytes || ((uintptr_t)workspace & 7))
    return fail(FC_ERR_WORKSPACE, "workspace smaller than fc_cache_workspace_bytes() or misaligned");
  HIP_TRY(launch_alpha(first_s, keys_s, diff_base, n_base, frame_elems, alpha_out, (double*)workspace,
                       (hipStream_t)stream));
  return FC_OK;
}

int fc_cache_frame_similarity(const float* frames_dev, int32_t frames, int64_t frame_elems, float* sim, void* workspace,
                              size_t workspace_bytes, void* stream) {
  if (!frames_dev || !sim || !workspace) return fail(FC_ERR_NULL, "NULL argument");
  if (frames < 0 || frame_elems < 1) return fail(FC_ERR_RANGE, "bad frame count or size");
  if (frames > kMaxCacheFrames) return fail(FC_ERR_UNSUPPORTED, "more than 256 frames in one entry");
  if (workspace_bytes < fc_cache_workspace_bytes(frames) || ((uintptr_t)workspace & 7))
    return fail(FC_ERR_WORKSPACE, "workspace smaller than fc_cache_workspace_bytes() or misaligned");
  HIP_TRY(launch_frame_similarity(frames_dev, frames, frame_elems, sim, (double*)workspace, (hipStream_t)stream));
  return FC_OK;
}

int fc_cache_frame_similarity_noalloc(const float* frames_dev, int32_t frames, int64_t frame_elems, float* sim,
                                      void* stream) {
  if (!frames_dev || !sim) return fail(FC_ERR_NULL, "NULL argument");
  if (frames < 0 || frame_elems < 1) return fail(FC_ERR_RANGE, "bad frame count or size");
  if (frames > kMaxCacheFrames)
    return fail(FC_ERR_UNSUPPORTED, "more than 256 frames: the library's own scratch holds a 256 x 256 Gram matrix");
  HIP_TRY(launch_frame_similarity_static(frames_dev, frames, frame_elems, sim, (hipStream_t)stream));
  return FC_OK;
}

int fc_cache_select_key_frames(const float* sim, int32_t frames, float threshold, int32_t* map_out) {
  if (!sim || !map_out) return fail(FC_ERR_NULL, "NULL argument");
  if (frames < 0) return fail(FC_ERR_RANGE, "negative frame count");
  for (int f = 0; f < frames; ++f) map_out[f] = -1;
  // from the last frame to the first: an unassigned frame becomes a key frame and takes
  // every unassigned frame in front of it that is similar enough
  for (int f = frames - 1; f >= 0; --f) {
    if (map_out[f] >= 0) continue;
    map_out[f] = f;
    for (int g = 0; g < f; ++g)
      if (map_out[g] < 0 && sim[(size_t)f * frames + g] >= threshold) map_out[g] = f;
  }
  return FC_OK;
}

int fc_bench_pipe_rates(const void* operands, int32_t iters, int32_t mode_first, int32_t mode_second, int32_t blocks,
                        float* sink, int64_t* clocks, void* stream) {
  if (!operands || !sink || !clocks) return fail(FC_ERR_NULL, "NULL argument");
  if (iters < 1 || iters > (1 << 24) || blocks < 1 || blocks > 65536 || mode_first < 0 || mode_first > 3 ||
      mode_second < 0 || mode_second > 3)
    return fail(FC_ERR_RANGE, "iters in 1..2^24, blocks in 1..65536, modes in 0..3");
  if (((uintptr_t)operands & 15) != 0) return fail(FC_ERR_RANGE, "operands must be 16-byte aligned");
  HIP_TRY(launch_pipe_rates(operands, iters, mode_first, mode_second, blocks, sink, (long long*)clocks,
                            (hipStream_t)stream));
  return FC_OK;
}

int fc_op_cfg_ddim(float* x, const float* eps_c, const float* eps_u, float* eps_out, size_t n, float gs,
                   const float* coef4, void* stream) {
  if (!x || !eps_c || !coef4) return fail(FC_ERR_NULL, "NULL argument");
  HIP_TRY(launch_cfg_ddim(x, eps_c, eps_u, eps_out, n, gs, coef4[0], coef4[1], coef4[2], coef4[3],
                          (hipStream_t)stream));
  return FC_OK;
}

}  // extern "C"
