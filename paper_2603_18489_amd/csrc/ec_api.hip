// Host side of the C ABI declared in include/ec.h: argument validation, workspace carving, the
// per-step launch sequence (one denoising step of the appendix algorithm), result read-back.
// All arithmetic of the step runs in the kernels; the host only chooses launch shapes.
#include <chrono>
#include <cstdio>
#include <cstring>
#include <new>
#include <string>
#include <vector>

#include "ec_internal.h"

using namespace ec;

namespace {

thread_local std::string g_init_error;

const size_t kAlign = 256;
size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

// Carves (or, with base == nullptr, only measures) the workspace.
struct Carver {
  char* base;
  size_t off = 0;
  explicit Carver(void* b) : base((char*)b) {}
  template <typename T> T* take(size_t count) {
    size_t o = off;
    off = align_up(off + count * sizeof(T));
    return base ? (T*)(base + o) : nullptr;
  }
};

// Re-tiled matrices of one layer: [q | k | v] as one matrix (rotary pairs adjacent), o, gate
// and up interleaved tile by tile, down.
struct PackedLayer {
  bf16_t *wqkv, *wo, *wgu, *wd;  // fragment order, tiles grouped by the matrix' skinny block width
};

struct Buffers {
  // sequence state
  int* x; uint8_t* masked; int* hist; DevState* st; int* mb_pos; int* rows_partial; int* mb_idx;
  float* row_stats; StepOut* out; int* forced_pos; int* forced_tok; int* prompt;
  float2* rope_cs;
  char* kv;  // [L][2][T][Hkv*hd] storage type
  // activations
  float* h; void* u; float* qkv; void* q; void* attn; float* gu; void* act; void* u_lm;
  float* logits; float4* partials;
  // bf16 only: row sums of squares [2L+1][kSumSlots][sumsq_stride] (32.32 fixed point), packed matrices
  unsigned long long* sumsq; int sumsq_stride;
  float* ksplit_part;  // [kMaxKSplit][T][d] partial products of K-split residual GEMMs; between
                       // them, the key slices of the partial-step attention
  size_t ksplit_floats;
  int* attn_tickets;   // [256] arrival counters of the key slices, zero between launches
  std::vector<PackedLayer> pl; bf16_t* lm_head_p;
};

size_t esize(int dtype) { return dtype == EC_BF16 ? 2 : 4; }
// keys held per cache slab: the packed bf16 cache is padded to whole 32-key blocks
int kv_keys(int dtype, int T) { return dtype == EC_BF16 ? (T + 31) / 32 * 32 : T; }

// elements of a packed [N, K] matrix whose tiles are grouped for the GEMM with epilogue `epi`
size_t packed_elems(int epi, size_t N, size_t K) {
  const size_t nt = N / 16, g = (size_t)skinny_tiles_per_block(epi, (int)nt);
  return (nt + g - 1) / g * g * 16 * K;
}

void carve(Carver& c, const ec_model_cfg& m, const ec_decode_cfg& d, int P, Buffers& b) {
  const int T = P + d.gen_len, N = d.gen_len;
  const size_t T16 = (size_t)(T + 15) / 16 * 16, B16 = (size_t)(d.block + 15) / 16 * 16;
  const size_t es = esize(m.dtype);
  const size_t nq = (size_t)m.n_heads * m.head_dim, nkv = (size_t)m.n_kv_heads * m.head_dim;
  b.x = c.take<int>(T); b.masked = c.take<uint8_t>(T); b.hist = c.take<int>(N);
  b.st = c.take<DevState>(1); b.mb_pos = c.take<int>(d.block); b.rows_partial = c.take<int>(T);
  b.mb_idx = c.take<int>(d.block); b.row_stats = c.take<float>((size_t)d.block * 4);
  b.out = c.take<StepOut>(1); b.forced_pos = c.take<int>(EC_MAX_N);
  b.forced_tok = c.take<int>(EC_MAX_N); b.prompt = c.take<int>(P);
  b.rope_cs = c.take<float2>((size_t)T * (m.head_dim / 2));
  b.kv = c.take<char>((size_t)m.n_layers * 2 * kv_keys(m.dtype, T) * nkv * es);
  b.h = c.take<float>((size_t)T * m.d_model);
  b.u = c.take<char>(T16 * m.d_model * es);
  b.qkv = c.take<float>((size_t)T * (nq + 2 * nkv));
  b.q = c.take<char>(T16 * nq * es);
  b.attn = c.take<char>(T16 * nq * es);
  b.gu = c.take<float>((size_t)T * 2 * m.d_ffn);
  b.act = c.take<char>(T16 * m.d_ffn * es);
  b.u_lm = c.take<char>(B16 * m.d_model * es);
  b.logits = c.take<float>((size_t)d.block * m.vocab);
  b.partials = c.take<float4>((size_t)d.block * vocab_reduce_parts(m.vocab));
  b.pl.clear();
  b.lm_head_p = nullptr;
  b.sumsq = nullptr;
  b.ksplit_part = nullptr; b.ksplit_floats = 0; b.attn_tickets = nullptr;
  b.sumsq_stride = (int)T16;
  if (m.dtype == EC_BF16) {
    b.sumsq = c.take<unsigned long long>((size_t)(2 * m.n_layers + 1) * kSumSlots * T16);
    b.ksplit_floats = (size_t)kMaxKSplit * T * m.d_model;
    b.ksplit_part = c.take<float>(b.ksplit_floats);
    b.attn_tickets = c.take<int>(256);
    b.pl.resize(m.n_layers);
    for (int l = 0; l < m.n_layers; ++l) {
      PackedLayer& p = b.pl[l];
      p.wqkv = c.take<bf16_t>(packed_elems(EPI_QKV, nq + 2 * nkv, m.d_model));
      p.wo = c.take<bf16_t>(packed_elems(EPI_RESID, m.d_model, nq));
      p.wgu = c.take<bf16_t>(packed_elems(EPI_SWIGLU, 2 * m.d_ffn, m.d_model));
      p.wd = c.take<bf16_t>(packed_elems(EPI_RESID, m.d_model, m.d_ffn));
    }
    b.lm_head_p = c.take<bf16_t>(packed_elems(EPI_LOGITS, m.vocab, m.d_model));
  }
}

const char* check_config(const ec_model_cfg* m, const ec_decode_cfg* d, int P) {
  if (m->dtype != EC_F32 && m->dtype != EC_BF16) return "dtype must be EC_F32 or EC_BF16";
  if (m->n_layers < 1 || m->d_model < 1 || m->n_heads < 1 || m->n_kv_heads < 1 || m->d_ffn < 1 ||
      m->vocab < 2)
    return "model sizes must be positive";
  if (m->head_dim != 64 && m->head_dim != 128) return "head_dim must be 64 or 128";
  if (m->n_heads % m->n_kv_heads != 0) return "n_heads must be a multiple of n_kv_heads";
  if (m->mask_id < 0 || m->mask_id >= m->vocab) return "mask_id outside the vocabulary";
  if (!(m->rms_eps >= 0.f) || !(m->rope_base > 1.f) || !(m->logit_scale > 0.f))
    return "rms_eps >= 0, rope_base > 1 and logit_scale > 0 are required";
  if (m->d_model % 8 || m->d_ffn % 8) return "d_model and d_ffn must be multiples of 8";
  if (m->dtype == EC_BF16) {
    if (m->d_model % 32 || m->d_ffn % 32 || m->vocab % 16)
      return "bf16 path: d_model, d_ffn must be multiples of 32 and vocab a multiple of 16";
  }
  if (d->batch != 1) return "batch must be 1";
  if (d->gen_len < 1) return "gen_len must be positive";
  if (d->block < 1 || d->block > EC_MAX_BLOCK) return "block must be in [1, EC_MAX_BLOCK]";
  if (d->tokens_per_step < 1 || d->tokens_per_step > EC_MAX_N)
    return "tokens_per_step must be in [1, EC_MAX_N]";
  if (d->k_recent < 0) return "k_recent must be >= 0";
  if (!(d->tau == d->tau)) return "tau is NaN";
  if (P < 0) return "negative prompt length";
  if ((long)P + d->gen_len > 15000) return "context longer than 15000 positions";
  return nullptr;
}

struct ProfEvent { int cls; hipEvent_t a, b; };

}  // namespace

struct ec_ctx {
  ec_model_cfg m;
  ec_decode_cfg d;
  ec_weights w;  // device pointers; per-layer arrays copied into the vectors below
  std::vector<const void*> attn_norm, wq, wk, wv, wo, mlp_norm, w_gate, w_up, w_down;
  int P, N, T;
  hipStream_t stream;
  Buffers b;
  StepOut* host_out = nullptr;   // pinned
  int* host_stage = nullptr;     // pinned: prompt / forced lists on their way to the device
  // host mirror of the scalar state
  int steps_run = 0, next_mode = EC_FULL, has_full = 0, done = 0, n_mb = 0, n_rows_partial = 0;
  std::vector<uint8_t> masked_host;
  int64_t rows_recomputed = 0;
  int full_steps = 0, partial_steps = 0, tokens = 0;
  // profiling
  bool prof_on = false;
  std::vector<ProfEvent> prof_pool;
  size_t prof_used = 0;
  ec_profile prof{};
  std::string err;
};

namespace {

int fail(ec_ctx* c, int code, const std::string& msg) {
  if (c) c->err = msg; else g_init_error = msg;
  return code;
}

#define EC_HIP(c, call)                                                                     \
  do {                                                                                      \
    hipError_t e_ = (call);                                                                 \
    if (e_ != hipSuccess)                                                                   \
      return fail((c), EC_ERR_HIP, std::string(#call) + ": " + hipGetErrorString(e_));      \
  } while (0)

// Brackets a launch with two events when profiling is on.
struct Scope {
  ec_ctx* c; int cls; ProfEvent* ev = nullptr;
  Scope(ec_ctx* c_, int cls_) : c(c_), cls(cls_) {
    if (!c->prof_on) return;
    if (c->prof_used == c->prof_pool.size()) {
      ProfEvent e{cls, nullptr, nullptr};
      if (hipEventCreate(&e.a) != hipSuccess || hipEventCreate(&e.b) != hipSuccess) return;
      c->prof_pool.push_back(e);
    }
    ev = &c->prof_pool[c->prof_used++];
    ev->cls = cls;
    (void)hipEventRecord(ev->a, c->stream);
  }
  ~Scope() { if (ev) (void)hipEventRecord(ev->b, c->stream); }
};

void prof_collect(ec_ctx* c) {  // stream must be idle
  for (size_t i = 0; i < c->prof_used; ++i) {
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, c->prof_pool[i].a, c->prof_pool[i].b) == hipSuccess) {
      c->prof.ms[c->prof_pool[i].cls] += ms;
      c->prof.launches[c->prof_pool[i].cls] += 1;
    }
  }
  if (c->prof_used) c->prof.steps += 1;
  c->prof_used = 0;
}

char* kv_ptr(ec_ctx* c, int layer, int which) {
  size_t row = (size_t)c->m.n_kv_heads * c->m.head_dim * esize(c->m.dtype);
  return c->b.kv + ((size_t)layer * 2 + which) * kv_keys(c->m.dtype, c->T) * row;
}

int upload_and_init_state(ec_ctx* c, const int32_t* prompt_ids) {
  if (c->P > 0) {
    memcpy(c->host_stage, prompt_ids, (size_t)c->P * sizeof(int));
    EC_HIP(c, hipMemcpyAsync(c->b.prompt, c->host_stage, (size_t)c->P * sizeof(int),
                             hipMemcpyHostToDevice, c->stream));
  }
  launch_init_state(c->b.x, c->b.masked, c->b.hist, c->b.st, c->b.prompt, c->P, c->N,
                    c->m.mask_id, c->stream);
  DecideArgs a{};
  a.init_only = 1; a.forced_n = -1;
  a.x = c->b.x; a.masked = c->b.masked; a.hist = c->b.hist; a.st = c->b.st;
  a.mb_pos = c->b.mb_pos; a.rows_partial = c->b.rows_partial; a.mb_idx = c->b.mb_idx;
  a.row_stats = c->b.row_stats; a.out = c->b.out;
  a.P = c->P; a.N = c->N; a.T = c->T; a.block = c->d.block; a.k_recent = c->d.k_recent;
  a.n_tok = c->d.tokens_per_step; a.tau = c->d.tau;
  launch_decide(a, c->stream);
  EC_HIP(c, hipGetLastError());
  EC_HIP(c, hipMemcpyAsync(c->host_out, c->b.out, sizeof(StepOut), hipMemcpyDeviceToHost,
                           c->stream));
  EC_HIP(c, hipStreamSynchronize(c->stream));
  c->steps_run = 0; c->next_mode = EC_FULL; c->has_full = 0; c->done = 0;
  c->n_mb = c->host_out->next_n_mb; c->n_rows_partial = c->host_out->next_n_rows_partial;
  c->masked_host.assign(c->T, 0);
  for (int i = c->P; i < c->T; ++i) c->masked_host[i] = 1;
  c->rows_recomputed = 0; c->full_steps = c->partial_steps = c->tokens = 0;
  return EC_OK;
}

// ---- the forward pass of one step over M rows -------------------------------------------------
int forward_f32(ec_ctx* c, int mode, int M, int n_mb) {
  const ec_model_cfg& m = c->m;
  Buffers& b = c->b;
  hipStream_t s = c->stream;
  const int d = m.d_model, F = m.d_ffn, hd = m.head_dim;
  const int nq = m.n_heads * hd, nkv = m.n_kv_heads * hd, nqkv = nq + 2 * nkv;
  const int* rows = (mode == EC_FULL) ? nullptr : b.rows_partial;
  const int* lm_sel = (mode == EC_FULL) ? b.mb_pos : b.mb_idx;
  float* u = (float*)b.u; float* q = (float*)b.q; float* attn = (float*)b.attn;
  float* act = (float*)b.act; float* u_lm = (float*)b.u_lm;
  auto W = [](const void* p) { return (const float*)p; };

  { Scope p(c, EC_K_EMBED); launch_embed_f32(W(c->w.tok_emb), b.x, rows, M, d, b.h, s); }
  for (int l = 0; l < m.n_layers; ++l) {
    float* kc = (float*)kv_ptr(c, l, 0); float* vc = (float*)kv_ptr(c, l, 1);
    { Scope p(c, EC_K_NORM);
      launch_rmsnorm_f32(b.h, nullptr, M, d, W(c->attn_norm[l]), m.rms_eps, u, s); }
    { Scope p(c, EC_K_QKV);
      launch_gemm_f32(u, W(c->wq[l]), b.qkv, nqkv, M, nq, d, 0, 1.f, s);
      launch_gemm_f32(u, W(c->wk[l]), b.qkv + nq, nqkv, M, nkv, d, 0, 1.f, s);
      launch_gemm_f32(u, W(c->wv[l]), b.qkv + nq + nkv, nqkv, M, nkv, d, 0, 1.f, s); }
    { Scope p(c, EC_K_ROPE_KV);
      launch_rope_scatter_f32(b.qkv, rows, M, m.n_heads, m.n_kv_heads, hd, b.rope_cs, q, kc, vc, s); }
    { Scope p(c, EC_K_ATTN);
      launch_attention_f32(q, kc, vc, M, c->T, m.n_heads, m.n_kv_heads, hd, attn, s); }
    { Scope p(c, EC_K_OPROJ); launch_gemm_f32(attn, W(c->wo[l]), b.h, d, M, d, nq, 1, 1.f, s); }
    { Scope p(c, EC_K_NORM);
      launch_rmsnorm_f32(b.h, nullptr, M, d, W(c->mlp_norm[l]), m.rms_eps, u, s); }
    { Scope p(c, EC_K_GATEUP);
      launch_gemm_f32(u, W(c->w_gate[l]), b.gu, 2 * F, M, F, d, 0, 1.f, s);
      launch_gemm_f32(u, W(c->w_up[l]), b.gu + F, 2 * F, M, F, d, 0, 1.f, s); }
    { Scope p(c, EC_K_SWIGLU); launch_swiglu_f32(b.gu, M, F, act, s); }
    { Scope p(c, EC_K_DOWN); launch_gemm_f32(act, W(c->w_down[l]), b.h, d, M, d, F, 1, 1.f, s); }
  }
  // logits only for the block's masked rows
  { Scope p(c, EC_K_NORM);
    launch_rmsnorm_f32(b.h, lm_sel, n_mb, d, W(c->w.final_norm), m.rms_eps, u_lm, s); }
  { Scope p(c, EC_K_LMHEAD);
    launch_gemm_f32(u_lm, W(c->w.lm_head), b.logits, m.vocab, n_mb, m.vocab, d, 0, m.logit_scale, s); }
  return EC_OK;
}

// bf16: five launches per layer.  Norms, RoPE, the KV scatter, SwiGLU and the residual adds run
// in the GEMM epilogues; `u` always holds the next GEMM's operand bf16(h * gain).
int forward_bf16(ec_ctx* c, int mode, int M, int n_mb) {
  const ec_model_cfg& m = c->m;
  Buffers& b = c->b;
  hipStream_t s = c->stream;
  const int d = m.d_model, F = m.d_ffn, hd = m.head_dim, L = m.n_layers;
  const int nq = m.n_heads * hd, nkv = m.n_kv_heads * hd, nqkv = nq + 2 * nkv;
  const int Tpad = kv_keys(EC_BF16, c->T), MT = (M + 15) / 16;
  const int* rows = (mode == EC_FULL) ? nullptr : b.rows_partial;
  const int* lm_sel = (mode == EC_FULL) ? b.mb_pos : b.mb_idx;
  bf16_t* u = (bf16_t*)b.u; bf16_t* q = (bf16_t*)b.q; bf16_t* attn = (bf16_t*)b.attn;
  bf16_t* act = (bf16_t*)b.act;
  auto G = [](const void* p) { return (const bf16_t*)p; };
  auto sums = [&](int i) { return b.sumsq + (size_t)i * kSumSlots * b.sumsq_stride; };

  { Scope p(c, EC_K_EMBED);
    launch_embed_bf16(G(c->w.tok_emb), b.x, rows, M, d, G(c->attn_norm[0]), b.h, u, b.sumsq,
                      (2 * L + 1) * kSumSlots, b.sumsq_stride, s); }
  for (int l = 0; l < L; ++l) {
    bf16_t* kc = (bf16_t*)kv_ptr(c, l, 0); bf16_t* vc = (bf16_t*)kv_ptr(c, l, 1);
    { Scope p(c, EC_K_QKV);
      GemmEpi e{}; e.M = M; e.MT = MT; e.sumsq_in = sums(2 * l); e.d_in = d; e.eps = m.rms_eps; e.sum_stride = b.sumsq_stride;
      e.rows = rows; e.cs = b.rope_cs; e.Hq = m.n_heads; e.Hkv = m.n_kv_heads; e.hd = hd;
      e.Tpad = Tpad; e.q_out = q; e.kc = kc; e.vc = vc;
      e.w_grp = skinny_tiles_per_block(EPI_QKV, nqkv / 16);
      launch_gemm_bf16(EPI_QKV, u, M, b.pl[l].wqkv, nqkv, d, e, s); }
    { Scope p(c, EC_K_ATTN);
      launch_attention_mfma(q, kc, vc, M, c->T, Tpad, m.n_heads, m.n_kv_heads, hd, attn,
                            b.ksplit_part, b.ksplit_floats, b.attn_tickets, s); }
    { Scope p(c, EC_K_OPROJ);
      GemmEpi e{}; e.M = M; e.MT = MT; e.h = b.h; e.d = d; e.gain_next = G(c->mlp_norm[l]);
      e.a_next = u; e.sumsq_out = sums(2 * l + 1); e.sum_stride = b.sumsq_stride; e.partial = b.ksplit_part;
      e.max_ksplit = kMaxKSplit;
      e.w_grp = skinny_tiles_per_block(EPI_RESID, d / 16);
      launch_gemm_bf16(EPI_RESID, attn, M, b.pl[l].wo, d, nq, e, s); }
    { Scope p(c, EC_K_GATEUP);
      GemmEpi e{}; e.M = M; e.MT = MT; e.sumsq_in = sums(2 * l + 1); e.d_in = d; e.eps = m.rms_eps; e.sum_stride = b.sumsq_stride;
      e.act = act;
      e.w_grp = skinny_tiles_per_block(EPI_SWIGLU, 2 * F / 16);
      launch_gemm_bf16(EPI_SWIGLU, u, M, b.pl[l].wgu, 2 * F, d, e, s); }
    { Scope p(c, EC_K_DOWN);
      GemmEpi e{}; e.M = M; e.MT = MT; e.h = b.h; e.d = d;
      e.gain_next = G(l + 1 < L ? c->attn_norm[l + 1] : c->w.final_norm);
      e.a_next = u; e.sumsq_out = sums(2 * l + 2); e.sum_stride = b.sumsq_stride; e.partial = b.ksplit_part;
      e.max_ksplit = kMaxKSplit;
      e.w_grp = skinny_tiles_per_block(EPI_RESID, d / 16);
      launch_gemm_bf16(EPI_RESID, act, M, b.pl[l].wd, d, F, e, s); }
  }
  // logits only for the block's masked rows: the LM head gathers them from `u`
  { Scope p(c, EC_K_LMHEAD);
    GemmEpi e{}; e.M = n_mb; e.MT = (n_mb + 15) / 16; e.row_sel = lm_sel; e.sumsq_in = sums(2 * L);
    e.d_in = d; e.eps = m.rms_eps; e.sum_stride = b.sumsq_stride; e.scale = m.logit_scale; e.logits = b.logits; e.ldc = m.vocab;
    e.w_grp = skinny_tiles_per_block(EPI_LOGITS, m.vocab / 16);
    launch_gemm_bf16(EPI_LOGITS, u, M, b.lm_head_p, m.vocab, d, e, s); }
  return EC_OK;
}

int forward(ec_ctx* c, int mode, int M, int n_mb) {
  int rc = (c->m.dtype == EC_F32) ? forward_f32(c, mode, M, n_mb) : forward_bf16(c, mode, M, n_mb);
  if (rc != EC_OK) return rc;
  { Scope p(c, EC_K_VOCAB_REDUCE);
    launch_vocab_reduce(c->b.logits, n_mb, c->m.vocab, c->b.partials, c->stream); }
  EC_HIP(c, hipGetLastError());
  return EC_OK;
}

int run_step(ec_ctx* c, int mode, int forced_n, const int32_t* fpos, const int32_t* ftok,
             ec_step_result* out) {
  if (!c) return fail(nullptr, EC_ERR_ARG, "ctx is NULL");
  if (!out) return fail(c, EC_ERR_ARG, "out is NULL");
  if (mode != EC_FULL && mode != EC_PARTIAL && mode != EC_AUTO)
    return fail(c, EC_ERR_ARG, "mode must be EC_FULL, EC_PARTIAL or EC_AUTO");
  if (c->done) return fail(c, EC_ERR_STATE, "generation is finished: no masked position left");
  if (mode == EC_AUTO) mode = (c->steps_run == 0) ? EC_FULL : c->next_mode;
  if (mode == EC_PARTIAL && !c->has_full)
    return fail(c, EC_ERR_STATE, "PARTIAL step before any FULL step: the KV cache is empty");
  if (forced_n >= 0) {
    if (forced_n > EC_MAX_N) return fail(c, EC_ERR_ARG, "more than EC_MAX_N forced tokens");
    if (forced_n > 0 && (!fpos || !ftok)) return fail(c, EC_ERR_ARG, "forced lists are NULL");
    for (int i = 0; i < forced_n; ++i) {
      if (fpos[i] < c->P || fpos[i] >= c->T || !c->masked_host[fpos[i]])
        return fail(c, EC_ERR_ARG, "forced position is not a masked generation slot");
      if (ftok[i] < 0 || ftok[i] >= c->m.vocab)
        return fail(c, EC_ERR_ARG, "forced token outside the vocabulary");
      for (int j = 0; j < i; ++j)
        if (fpos[j] == fpos[i]) return fail(c, EC_ERR_ARG, "forced position listed twice");
    }
    if (forced_n > 0) {
      memcpy(c->host_stage, fpos, forced_n * sizeof(int));
      memcpy(c->host_stage + EC_MAX_N, ftok, forced_n * sizeof(int));
      EC_HIP(c, hipMemcpyAsync(c->b.forced_pos, c->host_stage, forced_n * sizeof(int),
                               hipMemcpyHostToDevice, c->stream));
      EC_HIP(c, hipMemcpyAsync(c->b.forced_tok, c->host_stage + EC_MAX_N, forced_n * sizeof(int),
                               hipMemcpyHostToDevice, c->stream));
    }
  }
  const int M = (mode == EC_FULL) ? c->T : c->n_rows_partial;
  const int n_mb = c->n_mb;
  int rc = forward(c, mode, M, n_mb);
  if (rc != EC_OK) return rc;

  DecideArgs a{};
  a.partials = c->b.partials; a.nparts = vocab_reduce_parts(c->m.vocab); a.n_mb = n_mb;
  a.mode_run = mode; a.n_rows_run = M; a.forced_n = forced_n;
  a.forced_pos = c->b.forced_pos; a.forced_tok = c->b.forced_tok; a.init_only = 0;
  a.x = c->b.x; a.masked = c->b.masked; a.hist = c->b.hist; a.st = c->b.st;
  a.mb_pos = c->b.mb_pos; a.rows_partial = c->b.rows_partial; a.mb_idx = c->b.mb_idx;
  a.row_stats = c->b.row_stats; a.out = c->b.out;
  a.P = c->P; a.N = c->N; a.T = c->T; a.block = c->d.block; a.k_recent = c->d.k_recent;
  a.n_tok = c->d.tokens_per_step; a.tau = c->d.tau;
  { Scope p(c, EC_K_DECIDE); launch_decide(a, c->stream); }
  EC_HIP(c, hipGetLastError());
  EC_HIP(c, hipMemcpyAsync(c->host_out, c->b.out, sizeof(StepOut), hipMemcpyDeviceToHost,
                           c->stream));
  EC_HIP(c, hipStreamSynchronize(c->stream));
  if (c->prof_on) prof_collect(c);

  const StepOut& o = *c->host_out;
  c->steps_run += 1;
  c->has_full |= (mode == EC_FULL);
  c->done = o.r.done;
  c->n_mb = o.next_n_mb;
  c->n_rows_partial = o.next_n_rows_partial;
  c->rows_recomputed += M;
  (mode == EC_FULL ? c->full_steps : c->partial_steps) += 1;
  if (forced_n >= 0) {
    for (int i = 0; i < forced_n; ++i) c->masked_host[fpos[i]] = 0;
    c->tokens += forced_n;
    // the flag follows the committed tokens; the device computed it, mirror it from the state
    DevState st;
    EC_HIP(c, hipMemcpy(&st, c->b.st, sizeof(st), hipMemcpyDeviceToHost));
    c->next_mode = st.skip ? EC_PARTIAL : EC_FULL;
  } else {
    for (int i = 0; i < o.r.n_unmasked; ++i) c->masked_host[o.r.positions[i]] = 0;
    c->tokens += o.r.n_unmasked;
    c->next_mode = o.r.next_mode;
  }
  *out = o.r;
  return EC_OK;
}

}  // namespace

// =============================================================================================
// C ABI
// =============================================================================================
extern "C" {

size_t ec_workspace_bytes(const ec_model_cfg* model, const ec_decode_cfg* decode,
                          const int32_t* prompt_lens) {
  if (!model || !decode || !prompt_lens) return 0;
  if (check_config(model, decode, prompt_lens[0]) != nullptr) return 0;
  Carver c(nullptr);
  Buffers b;
  carve(c, *model, *decode, prompt_lens[0], b);
  return c.off;
}

int ec_init(ec_ctx** out, const ec_model_cfg* model, const ec_weights* weights,
            const ec_decode_cfg* decode, const int32_t* prompt_ids, const int32_t* prompt_lens,
            void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!out) return fail(nullptr, EC_ERR_ARG, "out is NULL");
  *out = nullptr;
  if (!model || !weights || !decode || !prompt_lens)
    return fail(nullptr, EC_ERR_ARG, "model, weights, decode and prompt_lens must not be NULL");
  const int P = prompt_lens[0];
  if (const char* msg = check_config(model, decode, P)) return fail(nullptr, EC_ERR_CONFIG, msg);
  if (P > 0 && !prompt_ids) return fail(nullptr, EC_ERR_ARG, "prompt_ids is NULL");
  for (int i = 0; i < P; ++i)
    if (prompt_ids[i] < 0 || prompt_ids[i] >= model->vocab)
      return fail(nullptr, EC_ERR_ARG, "prompt id outside the vocabulary");
  if (!weights->tok_emb || !weights->lm_head || !weights->final_norm || !weights->attn_norm ||
      !weights->wq || !weights->wk || !weights->wv || !weights->wo || !weights->mlp_norm ||
      !weights->w_gate || !weights->w_up || !weights->w_down)
    return fail(nullptr, EC_ERR_ARG, "a weight pointer is NULL");
  for (int l = 0; l < model->n_layers; ++l)
    if (!weights->attn_norm[l] || !weights->wq[l] || !weights->wk[l] || !weights->wv[l] ||
        !weights->wo[l] || !weights->mlp_norm[l] || !weights->w_gate[l] || !weights->w_up[l] ||
        !weights->w_down[l])
      return fail(nullptr, EC_ERR_ARG, "a per-layer weight pointer is NULL");
  size_t need = ec_workspace_bytes(model, decode, prompt_lens);
  if (!workspace) return fail(nullptr, EC_ERR_WORKSPACE, "workspace is NULL");
  if (((uintptr_t)workspace) % kAlign) return fail(nullptr, EC_ERR_WORKSPACE, "workspace is not 256-byte aligned");
  if (workspace_bytes < need) {
    char buf[128];
    snprintf(buf, sizeof buf, "workspace too small: %zu bytes given, %zu needed", workspace_bytes, need);
    return fail(nullptr, EC_ERR_WORKSPACE, buf);
  }

  ec_ctx* c = new (std::nothrow) ec_ctx();
  if (!c) return fail(nullptr, EC_ERR_ARG, "out of host memory");
  c->m = *model; c->d = *decode; c->w = *weights;
  const int L = model->n_layers;
  c->attn_norm.assign(weights->attn_norm, weights->attn_norm + L);
  c->wq.assign(weights->wq, weights->wq + L); c->wk.assign(weights->wk, weights->wk + L);
  c->wv.assign(weights->wv, weights->wv + L); c->wo.assign(weights->wo, weights->wo + L);
  c->mlp_norm.assign(weights->mlp_norm, weights->mlp_norm + L);
  c->w_gate.assign(weights->w_gate, weights->w_gate + L);
  c->w_up.assign(weights->w_up, weights->w_up + L);
  c->w_down.assign(weights->w_down, weights->w_down + L);
  c->P = P; c->N = decode->gen_len; c->T = P + decode->gen_len;
  c->stream = (hipStream_t)hip_stream;
  Carver cv(workspace);
  carve(cv, c->m, c->d, P, c->b);

  auto bail = [&](int code, const std::string& msg) {
    if (c->host_out) (void)hipHostFree(c->host_out);
    if (c->host_stage) (void)hipHostFree(c->host_stage);
    delete c;
    return fail(nullptr, code, msg);
  };
  hipError_t e = hipHostMalloc((void**)&c->host_out, sizeof(StepOut), hipHostMallocDefault);
  if (e != hipSuccess) return bail(EC_ERR_HIP, std::string("hipHostMalloc: ") + hipGetErrorString(e));
  size_t stage = (size_t)(P > 2 * EC_MAX_N ? P : 2 * EC_MAX_N) * sizeof(int);
  e = hipHostMalloc((void**)&c->host_stage, stage, hipHostMallocDefault);
  if (e != hipSuccess) return bail(EC_ERR_HIP, std::string("hipHostMalloc: ") + hipGetErrorString(e));

  // one-time device set-up: RoPE table, re-tiled bf16 matrices, finite padding keys
  launch_rope_table(c->b.rope_cs, c->T, c->m.head_dim, c->m.rope_base, c->stream);
  if (c->m.dtype == EC_BF16) {
    size_t kvbytes = (size_t)L * 2 * kv_keys(EC_BF16, c->T) * c->m.n_kv_heads * c->m.head_dim * 2;
    e = hipMemsetAsync(c->b.kv, 0, kvbytes, c->stream);
    if (e == hipSuccess) e = hipMemsetAsync(c->b.attn_tickets, 0, 256 * sizeof(int), c->stream);
    if (e != hipSuccess) return bail(EC_ERR_HIP, std::string("hipMemsetAsync: ") + hipGetErrorString(e));
    const int d = c->m.d_model, F = c->m.d_ffn;
    const int nq = c->m.n_heads * c->m.head_dim, nkv = c->m.n_kv_heads * c->m.head_dim;
    const int hd = c->m.head_dim;
    auto B = [](const void* p) { return (const bf16_t*)p; };
    for (int l = 0; l < L; ++l) {
      PackedLayer& p = c->b.pl[l];
      const int gq = skinny_tiles_per_block(EPI_QKV, (nq + 2 * nkv) / 16);
      const int go = skinny_tiles_per_block(EPI_RESID, d / 16);
      const int gg = skinny_tiles_per_block(EPI_SWIGLU, 2 * F / 16);
      launch_repack_weight(B(c->wq[l]), nq, d, p.wqkv, REPACK_ROPE_HALVES, hd, gq, 0, c->stream);
      launch_repack_weight(B(c->wk[l]), nkv, d, p.wqkv, REPACK_ROPE_HALVES, hd, gq, nq, c->stream);
      launch_repack_weight(B(c->wv[l]), nkv, d, p.wqkv, REPACK_PLAIN, hd, gq, nq + nkv, c->stream);
      launch_repack_weight(B(c->wo[l]), d, nq, p.wo, REPACK_PLAIN, hd, go, 0, c->stream);
      launch_repack_weight(B(c->w_gate[l]), F, d, p.wgu, REPACK_LO8, hd, gg, 0, c->stream);
      launch_repack_weight(B(c->w_up[l]), F, d, p.wgu, REPACK_HI8, hd, gg, 0, c->stream);
      launch_repack_weight(B(c->w_down[l]), d, F, p.wd, REPACK_PLAIN, hd, go, 0, c->stream);
    }
    launch_repack_weight(B(c->w.lm_head), c->m.vocab, d, c->b.lm_head_p, REPACK_PLAIN, hd,
                         skinny_tiles_per_block(EPI_LOGITS, c->m.vocab / 16), 0, c->stream);
  }
  e = hipGetLastError();
  if (e != hipSuccess) return bail(EC_ERR_HIP, std::string("set-up kernels: ") + hipGetErrorString(e));
  int rc = upload_and_init_state(c, prompt_ids);
  if (rc != EC_OK) return bail(rc, c->err);
  *out = c;
  return EC_OK;
}

int ec_reset(ec_ctx* ctx, const int32_t* prompt_ids) {
  if (!ctx) return fail(nullptr, EC_ERR_ARG, "ctx is NULL");
  if (ctx->P > 0 && !prompt_ids) return fail(ctx, EC_ERR_ARG, "prompt_ids is NULL");
  for (int i = 0; i < ctx->P; ++i)
    if (prompt_ids[i] < 0 || prompt_ids[i] >= ctx->m.vocab)
      return fail(ctx, EC_ERR_ARG, "prompt id outside the vocabulary");
  return upload_and_init_state(ctx, prompt_ids);
}

int ec_step(ec_ctx* ctx, int mode, ec_step_result* out) {
  return run_step(ctx, mode, -1, nullptr, nullptr, out);
}

int ec_step_forced(ec_ctx* ctx, int mode, int32_t n, const int32_t* positions,
                   const int32_t* tokens, ec_step_result* out) {
  if (n < 0) return fail(ctx, EC_ERR_ARG, "n must be >= 0");
  return run_step(ctx, mode, n, positions, tokens, out);
}

int ec_generate(ec_ctx* ctx, int32_t* out_tokens, ec_gen_stats* stats) {
  if (!ctx) return fail(nullptr, EC_ERR_ARG, "ctx is NULL");
  if (!out_tokens) return fail(ctx, EC_ERR_ARG, "out_tokens is NULL");
  auto t0 = std::chrono::steady_clock::now();
  ec_step_result r;
  while (!ctx->done) {
    int rc = run_step(ctx, EC_AUTO, -1, nullptr, nullptr, &r);
    if (rc != EC_OK) return rc;
  }
  EC_HIP(ctx, hipMemcpy(out_tokens, ctx->b.x + ctx->P, (size_t)ctx->N * sizeof(int),
                        hipMemcpyDeviceToHost));
  if (stats) {
    stats->steps = ctx->steps_run; stats->full_steps = ctx->full_steps;
    stats->partial_steps = ctx->partial_steps; stats->tokens = ctx->tokens;
    stats->rows_recomputed = ctx->rows_recomputed;
    stats->ms_total = std::chrono::duration<double, std::milli>(
                          std::chrono::steady_clock::now() - t0).count();
  }
  return EC_OK;
}

int ec_profile_enable(ec_ctx* ctx, int on) {
  if (!ctx) return fail(nullptr, EC_ERR_ARG, "ctx is NULL");
  ctx->prof_on = on != 0;
  ctx->prof_used = 0;
  if (on) memset(&ctx->prof, 0, sizeof ctx->prof);
  return EC_OK;
}

int ec_profile_read(ec_ctx* ctx, ec_profile* out) {
  if (!ctx) return fail(nullptr, EC_ERR_ARG, "ctx is NULL");
  if (!out) return fail(ctx, EC_ERR_ARG, "out is NULL");
  *out = ctx->prof;
  return EC_OK;
}

int ec_debug_read(ec_ctx* ctx, int what, int layer, void* host_dst, size_t bytes) {
  if (!ctx) return fail(nullptr, EC_ERR_ARG, "ctx is NULL");
  if (!host_dst) return fail(ctx, EC_ERR_ARG, "host_dst is NULL");
  const void* src = nullptr;
  size_t avail = 0;
  const size_t kvrow = (size_t)ctx->m.n_kv_heads * ctx->m.head_dim * esize(ctx->m.dtype);
  switch (what) {
    case EC_DBG_LOGITS: src = ctx->b.logits; avail = (size_t)ctx->d.block * ctx->m.vocab * 4; break;
    case EC_DBG_KCACHE:
    case EC_DBG_VCACHE:
      if (layer < 0 || layer >= ctx->m.n_layers) return fail(ctx, EC_ERR_ARG, "layer out of range");
      src = kv_ptr(ctx, layer, what == EC_DBG_VCACHE); avail = (size_t)ctx->T * kvrow;
      if (ctx->m.dtype == EC_BF16) {
        // the packed cache is put back into [T, Hkv, hd] order in a scratch activation buffer
        launch_unpack_cache((const bf16_t*)src, what == EC_DBG_VCACHE, ctx->T,
                            kv_keys(EC_BF16, ctx->T), ctx->m.n_kv_heads, ctx->m.head_dim,
                            (bf16_t*)ctx->b.qkv, ctx->stream);
        src = ctx->b.qkv;
      }
      break;
    case EC_DBG_X: src = ctx->b.x; avail = (size_t)ctx->T * 4; break;
    case EC_DBG_MASKED: src = ctx->b.masked; avail = (size_t)ctx->T; break;
    case EC_DBG_HIST: src = ctx->b.hist; avail = (size_t)ctx->N * 4; break;
    case EC_DBG_ROWS: src = ctx->b.rows_partial; avail = (size_t)ctx->n_rows_partial * 4; break;
    case EC_DBG_ROW_STATS: src = ctx->b.row_stats; avail = (size_t)ctx->d.block * 16; break;
    default: return fail(ctx, EC_ERR_ARG, "unknown debug item");
  }
  if (bytes > avail) return fail(ctx, EC_ERR_ARG, "bytes exceeds the size of the item");
  EC_HIP(ctx, hipStreamSynchronize(ctx->stream));
  if (bytes) EC_HIP(ctx, hipMemcpy(host_dst, src, bytes, hipMemcpyDeviceToHost));
  return EC_OK;
}

void ec_destroy(ec_ctx* ctx) {
  if (!ctx) return;
  (void)hipStreamSynchronize(ctx->stream);
  for (auto& e : ctx->prof_pool) { (void)hipEventDestroy(e.a); (void)hipEventDestroy(e.b); }
  if (ctx->host_out) (void)hipHostFree(ctx->host_out);
  if (ctx->host_stage) (void)hipHostFree(ctx->host_stage);
  delete ctx;
}

const char* ec_strerror(int code) {
  switch (code) {
    case EC_OK: return "ok";
    case EC_ERR_ARG: return "invalid argument";
    case EC_ERR_CONFIG: return "unsupported configuration";
    case EC_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case EC_ERR_STATE: return "call not valid in the current state";
    case EC_ERR_HIP: return "HIP runtime error";
    default: return "unknown error code";
  }
}

const char* ec_last_error(const ec_ctx* ctx) {
  return ctx ? ctx->err.c_str() : g_init_error.c_str();
}

}  // extern "C"
