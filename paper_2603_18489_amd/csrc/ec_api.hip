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
  // EC_FP8W: the same matrices as e4m3 fragment pairs, and their row scales in packed row order
  uint8_t *qqkv = nullptr, *qo = nullptr, *qgu = nullptr, *qd = nullptr;
  float *sqkv = nullptr, *so = nullptr, *sgu = nullptr, *sd = nullptr;
};

struct Buffers {
  // sequence state, sequence after sequence: x / masked / rows_partial / prompt by positions,
  // the others with the fixed stride named in DecideArgs
  int* x; uint8_t* masked; int* hist; DevState* st; int* mb_pos; int* rows_partial; int* mb_idx;
  float* row_stats; StepOut* out; int* forced_pos; int* forced_tok; int* prompt;
  // the step's row list (bf16 path)
  SeqDesc* seqs; int4* rowinfo; int4* tileinfo; int* lm_sel;
  int4* pairs;  // (row tile, sequence) visits of the few-row sequences, [rmax/16 + B]
  float2* rope_cs;
  char* kv;  // [L][2] planes; a plane holds every sequence's [Hkv][keys][hd] slabs, storage type
  size_t kv_plane;  // elements per plane
  // activations
  float* h; void* u; float* qkv; void* q; void* attn; float* gu; void* act; void* u_lm;
  float* logits; float4* partials;
  // bf16 only: row sums of squares [2L+1][kSumSlots][sumsq_stride] (44.20 fixed point), packed matrices
  unsigned long long* sumsq; int sumsq_stride;
  float* ksplit_part;  // [kMaxKSplit][T][d] partial products of K-split residual GEMMs; between
                       // them, the key slices of the partial-step attention
  size_t ksplit_floats;
  int* attn_tickets;   // [256] arrival counters of the key slices, zero between launches
  std::vector<PackedLayer> pl; bf16_t* lm_head_p;
  uint8_t* lm_head_q = nullptr; float* lm_head_s = nullptr;  // EC_FP8W
};

// bytes of an activation / KV-cache element (EC_FP8W computes like EC_BF16)
size_t esize(int dtype) { return dtype == EC_F32 ? 4 : 2; }
bool bf16_path(int dtype) { return dtype != EC_F32; }
// keys held per cache slab: the packed bf16 cache is padded to whole 32-key blocks
int kv_keys(int dtype, int T) { return bf16_path(dtype) ? (T + 31) / 32 * 32 : T; }

// elements of a packed [N, K] matrix whose tiles are grouped for the GEMM with epilogue `epi`
size_t packed_elems(int epi, size_t N, size_t K) {
  const size_t nt = N / 16, g = (size_t)skinny_tiles_per_block(epi, (int)nt);
  return (nt + g - 1) / g * g * 16 * K;
}

// Sizes that depend on the prompt lengths.
struct Geometry {
  int B = 0;
  std::vector<int> P, T, tpad, x_off, kv_off;
  size_t xtot = 0, ptot = 0;  // positions / prompt ids over all sequences
  size_t kv_plane = 0;        // elements of one layer's K (or V) plane
  size_t rmax = 0;            // most rows a step can have, with the padding of the row list
  int tmax = 0;
};

// rows a sequence's segment of the row list takes
int seg_rows_of(int n_rows) {
  return n_rows > kSmallRows ? (n_rows + 255) / 256 * 256 : (n_rows + 15) / 16 * 16;
}

Geometry geometry(const ec_model_cfg& m, const ec_decode_cfg& d, const int32_t* prompt_lens) {
  Geometry g;
  g.B = d.batch;
  const size_t nkv = (size_t)m.n_kv_heads * m.head_dim;
  for (int b = 0; b < g.B; ++b) {
    const int P = prompt_lens[b], T = P + d.gen_len;
    g.P.push_back(P); g.T.push_back(T); g.tpad.push_back(kv_keys(m.dtype, T));
    g.x_off.push_back((int)g.xtot); g.kv_off.push_back((int)g.kv_plane);
    g.xtot += T; g.ptot += P;
    g.kv_plane += (size_t)kv_keys(m.dtype, T) * nkv;
    g.rmax += seg_rows_of(T);
    g.tmax = T > g.tmax ? T : g.tmax;
  }
  return g;
}

void carve(Carver& c, const ec_model_cfg& m, const ec_decode_cfg& d, const Geometry& g,
           Buffers& b) {
  const int N = d.gen_len, B = g.B;
  const size_t R = g.rmax, BL = (size_t)B * d.block, BL16 = (BL + 15) / 16 * 16;
  const size_t es = esize(m.dtype);
  const size_t nq = (size_t)m.n_heads * m.head_dim, nkv = (size_t)m.n_kv_heads * m.head_dim;
  b.x = c.take<int>(g.xtot); b.masked = c.take<uint8_t>(g.xtot); b.hist = c.take<int>((size_t)B * N);
  b.st = c.take<DevState>(B); b.mb_pos = c.take<int>(BL); b.rows_partial = c.take<int>(g.xtot);
  b.mb_idx = c.take<int>(BL); b.row_stats = c.take<float>(BL * 4);
  b.out = c.take<StepOut>(B); b.forced_pos = c.take<int>((size_t)B * EC_MAX_N);
  b.forced_tok = c.take<int>((size_t)B * EC_MAX_N); b.prompt = c.take<int>(g.ptot);
  b.seqs = c.take<SeqDesc>(B); b.rowinfo = c.take<int4>(R); b.tileinfo = c.take<int4>(R / 16);
  b.lm_sel = c.take<int>(BL);
  b.pairs = c.take<int4>(R / 16 + 2 * B);   // [B sequence entries][visits]
  b.rope_cs = c.take<float2>((size_t)g.tmax * (m.head_dim / 2));
  b.kv_plane = g.kv_plane;
  b.kv = c.take<char>((size_t)m.n_layers * 2 * g.kv_plane * es);
  b.h = c.take<float>(R * m.d_model);
  b.u = c.take<char>(R * m.d_model * es);
  b.qkv = c.take<float>(R * (nq + 2 * nkv));
  b.q = c.take<char>(R * nq * es);
  b.attn = c.take<char>(R * nq * es);
  b.gu = c.take<float>(m.dtype == EC_F32 ? R * 2 * m.d_ffn : 1);
  b.act = c.take<char>(R * m.d_ffn * es);
  b.u_lm = c.take<char>(BL16 * m.d_model * es);
  b.logits = c.take<float>(BL * m.vocab);
  {  // partial tuples of the vocabulary reduction: from the LM-head epilogue or from vocab_reduce
    const size_t np_fused = bf16_path(m.dtype) ? (size_t)lm_head_parts(m.vocab) : 0;
    const size_t np_plain = (size_t)vocab_reduce_parts(m.vocab);
    b.partials = c.take<float4>(BL * (np_fused > np_plain ? np_fused : np_plain));
  }
  b.pl.clear();
  b.lm_head_p = nullptr;
  b.sumsq = nullptr;
  b.ksplit_part = nullptr; b.ksplit_floats = 0; b.attn_tickets = nullptr;
  b.sumsq_stride = (int)R;
  if (bf16_path(m.dtype)) {
    b.sumsq = c.take<unsigned long long>((size_t)(2 * m.n_layers + 1) * kSumSlots * R);
    b.ksplit_floats = (size_t)kMaxKSplit * R * m.d_model;
    b.ksplit_part = c.take<float>(b.ksplit_floats);
    b.attn_tickets = c.take<int>(256);
    b.pl.resize(m.n_layers);
    for (int l = 0; l < m.n_layers; ++l) {
      PackedLayer& p = b.pl[l];
      p.wqkv = c.take<bf16_t>(packed_elems(EPI_QKV, nq + 2 * nkv, m.d_model));
      p.wo = c.take<bf16_t>(packed_elems(EPI_RESID, m.d_model, nq));
      p.wgu = c.take<bf16_t>(packed_elems(EPI_SWIGLU, 2 * m.d_ffn, m.d_model));
      p.wd = c.take<bf16_t>(packed_elems(EPI_RESID, m.d_model, m.d_ffn));
      if (m.dtype == EC_FP8W) {  // one byte per element, one scale per (padded) packed row
        p.qqkv = c.take<uint8_t>(packed_elems(EPI_QKV, nq + 2 * nkv, m.d_model));
        p.qo = c.take<uint8_t>(packed_elems(EPI_RESID, m.d_model, nq));
        p.qgu = c.take<uint8_t>(packed_elems(EPI_SWIGLU, 2 * m.d_ffn, m.d_model));
        p.qd = c.take<uint8_t>(packed_elems(EPI_RESID, m.d_model, m.d_ffn));
        p.sqkv = c.take<float>(packed_elems(EPI_QKV, nq + 2 * nkv, 1));
        p.so = c.take<float>(packed_elems(EPI_RESID, m.d_model, 1));
        p.sgu = c.take<float>(packed_elems(EPI_SWIGLU, 2 * m.d_ffn, 1));
        p.sd = c.take<float>(packed_elems(EPI_RESID, m.d_model, 1));
      }
    }
    b.lm_head_p = c.take<bf16_t>(packed_elems(EPI_LOGITS, m.vocab, m.d_model));
    if (m.dtype == EC_FP8W) {
      b.lm_head_q = c.take<uint8_t>(packed_elems(EPI_LOGITS, m.vocab, m.d_model));
      b.lm_head_s = c.take<float>(packed_elems(EPI_LOGITS, m.vocab, 1));
    }
  }
}

const char* check_config(const ec_model_cfg* m, const ec_decode_cfg* d, const int32_t* prompt_lens) {
  if (m->dtype != EC_F32 && m->dtype != EC_BF16 && m->dtype != EC_FP8W)
    return "dtype must be EC_F32, EC_BF16 or EC_FP8W";
  if (m->n_layers < 1 || m->d_model < 1 || m->n_heads < 1 || m->n_kv_heads < 1 || m->d_ffn < 1 ||
      m->vocab < 2)
    return "model sizes must be positive";
  if (m->head_dim != 64 && m->head_dim != 128) return "head_dim must be 64 or 128";
  if (m->n_heads % m->n_kv_heads != 0) return "n_heads must be a multiple of n_kv_heads";
  if (m->mask_id < 0 || m->mask_id >= m->vocab) return "mask_id outside the vocabulary";
  if (m->vocab > 163840) return "vocab larger than 163840";  // staging room of the decision kernel
  if (!(m->rms_eps >= 0.f) || !(m->rope_base > 1.f) || !(m->logit_scale > 0.f))
    return "rms_eps >= 0, rope_base > 1 and logit_scale > 0 are required";
  if (m->d_model % 8 || m->d_ffn % 8) return "d_model and d_ffn must be multiples of 8";
  if (bf16_path(m->dtype)) {
    if (m->d_model % 32 || m->d_ffn % 32 || m->vocab % 16)
      return "bf16 path: d_model, d_ffn must be multiples of 32 and vocab a multiple of 16";
  }
  if (m->dtype == EC_FP8W && (m->d_model % 64 || m->d_ffn % 64))
    return "EC_FP8W: d_model and d_ffn must be multiples of 64";
  if (d->batch < 1 || d->batch > EC_MAX_BATCH) return "batch must be in [1, EC_MAX_BATCH]";
  if (d->batch > 1 && !bf16_path(m->dtype)) return "batch > 1 needs the bfloat16 path";
  if (d->gen_len < 1) return "gen_len must be positive";
  if (d->block < 1 || d->block > EC_MAX_BLOCK) return "block must be in [1, EC_MAX_BLOCK]";
  if (d->tokens_per_step < 1 || d->tokens_per_step > EC_MAX_N)
    return "tokens_per_step must be in [1, EC_MAX_N]";
  if (d->k_recent < 0) return "k_recent must be >= 0";
  if (!(d->tau == d->tau)) return "tau is NaN";
  if (!(d->conf_threshold >= 0.f) || d->conf_threshold >= 1.f)
    return "conf_threshold must be in [0, 1)";
  if (d->gate_metric < EC_GATE_MAX_ENTROPY || d->gate_metric > EC_GATE_MAX_CONFIDENCE)
    return "unknown gate_metric";
  if (d->schedule != EC_SCHED_BLOCKS && d->schedule != EC_SCHED_SLIDING) return "unknown schedule";
  long total = 0;
  for (int b = 0; b < d->batch; ++b) {
    if (prompt_lens[b] < 0) return "negative prompt length";
    if ((long)prompt_lens[b] + d->gen_len > 15000) return "context longer than 15000 positions";
    total += (long)prompt_lens[b] + d->gen_len + 256;
  }
  if (total > 200000) return "more than 200000 positions over the batch";
  return nullptr;
}

struct ProfEvent { int cls; hipEvent_t a, b; };

}  // namespace

namespace ec {
// message of a failure that has no context to hang on (ec_init, the context-free calls)
void set_global_error(const char* msg) { g_init_error = msg; }
}

struct ec_ctx {
  ec_model_cfg m;
  ec_decode_cfg d;
  ec_weights w;  // device pointers; per-layer arrays copied into the vectors below
  std::vector<const void*> attn_norm, wq, wk, wv, wo, mlp_norm, w_gate, w_up, w_down;
  std::vector<const float*> wq_s, wk_s, wv_s, wo_s, w_gate_s, w_up_s, w_down_s;  // EC_FP8W
  Geometry g;
  int B, N;
  hipStream_t stream;
  Buffers b;
  StepOut* host_out = nullptr;   // pinned [B]: the decision kernel writes its results here
  StepOut* host_out_dev = nullptr;  // the same memory as the device addresses it
  int serial = 0;                   // number of the last decision launch (StepOut::serial)
  int* host_stage = nullptr;     // pinned: prompts / forced lists on their way to the device
  SeqDesc* host_seqs = nullptr;  // pinned [B]
  int4* host_pairs = nullptr;    // pinned [rmax/16 + B]
  // host mirror of the scalar state, per sequence
  int steps_run = 0;
  std::vector<int> next_mode, has_full, done, n_mb, n_rows_partial;
  int all_done = 0;
  std::vector<uint8_t> masked_host;  // concatenated by x_off
  int64_t rows_recomputed = 0;
  int full_steps = 0, partial_steps = 0, tokens = 0;
  // vocabulary reduction of the step in flight: fused behind the LM head (then the logits are
  // only stored on request) or a pass of its own over materialised logits
  bool keep_logits = false;   // ec_debug_keep_logits
  bool logits_stored = false; // the last step left its logits in b.logits
  bool fused_reduce = false;
  int step_nparts = 0;
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
  return c->b.kv + ((size_t)layer * 2 + which) * c->b.kv_plane * esize(c->m.dtype);
}

void fill_decide_args(ec_ctx* c, DecideArgs& a) {
  // one sequence: its descriptor travels in the kernel arguments, no table upload
  a.seqs = c->B == 1 ? nullptr : c->b.seqs;
  a.seq0 = c->host_seqs[0];
  a.partials = c->b.partials; a.nparts = c->step_nparts;
  a.forced_pos = c->b.forced_pos; a.forced_tok = c->b.forced_tok;
  a.x = c->b.x; a.masked = c->b.masked; a.hist = c->b.hist; a.st = c->b.st;
  a.mb_pos = c->b.mb_pos; a.rows_partial = c->b.rows_partial; a.mb_idx = c->b.mb_idx;
  a.row_stats = c->b.row_stats; a.out = c->host_out_dev;
  a.N = c->N; a.block = c->d.block; a.k_recent = c->d.k_recent;
  a.n_tok = c->d.tokens_per_step; a.tau = c->d.tau;
  a.conf_threshold = c->d.conf_threshold; a.gate_metric = c->d.gate_metric;
  a.schedule = c->d.schedule;
  a.vocab = c->m.vocab;
  a.serial = c->serial = (c->serial == 0x7fffffff ? 1 : c->serial + 1);
}

// Waits for the decision kernel's results.  Every taking-part sequence's block stores the
// launch's serial number behind its result (system-scope release), so the host can take the
// result as soon as the numbers show up instead of waiting for the stream to drain and the
// runtime to notice; later work is ordered behind the kernel by the stream anyway.  The poll is
// bounded: the stream is queried now and then, and once it has drained (or failed) the ordinary
// synchronisation decides.
int wait_results(ec_ctx* c, const int* taking_part) {
  const int B = c->B;
  for (unsigned spin = 1;; ++spin) {
    bool all = true;
    for (int b = 0; b < B && all; ++b)
      if (!taking_part || taking_part[b] >= 0)
        all = __atomic_load_n(&c->host_out[b].serial, __ATOMIC_ACQUIRE) == c->serial;
    if (all) return EC_OK;
    if ((spin & 0xfff) == 0 && hipStreamQuery(c->stream) != hipErrorNotReady) break;
    __builtin_ia32_pause();
  }
  EC_HIP(c, hipStreamSynchronize(c->stream));
  return EC_OK;
}

// static part of a sequence's descriptor
SeqDesc base_desc(const ec_ctx* c, int b) {
  SeqDesc sd{};
  sd.P = c->g.P[b]; sd.T = c->g.T[b]; sd.tpad = c->g.tpad[b];
  sd.x_off = c->g.x_off[b]; sd.kv_off = c->g.kv_off[b];
  sd.mode = -1; sd.forced_n = -1;
  return sd;
}

int upload_and_init_state(ec_ctx* c, const int32_t* prompt_ids) {
  const int B = c->B;
  if (c->g.ptot > 0) {
    memcpy(c->host_stage, prompt_ids, c->g.ptot * sizeof(int));
    EC_HIP(c, hipMemcpyAsync(c->b.prompt, c->host_stage, c->g.ptot * sizeof(int),
                             hipMemcpyHostToDevice, c->stream));
  }
  size_t poff = 0;
  for (int b = 0; b < B; ++b) {
    launch_init_state(c->b.x + c->g.x_off[b], c->b.masked + c->g.x_off[b],
                      c->b.hist + (size_t)b * c->N, c->b.st + b, c->b.prompt + poff, c->g.P[b],
                      c->N, c->m.mask_id, c->stream);
    poff += c->g.P[b];
    c->host_seqs[b] = base_desc(c, b);
    c->host_seqs[b].mode = EC_FULL;  // takes part in the list building below
  }
  if (B > 1)
    EC_HIP(c, hipMemcpyAsync(c->b.seqs, c->host_seqs, (size_t)B * sizeof(SeqDesc),
                             hipMemcpyHostToDevice, c->stream));
  c->logits_stored = false;
  DecideArgs a{};
  fill_decide_args(c, a);
  a.init_only = 1;
  launch_decide(a, B, c->stream);
  EC_HIP(c, hipGetLastError());
  EC_HIP(c, hipStreamSynchronize(c->stream));   // (the results sit in host_out once the kernel ended)
  c->steps_run = 0; c->all_done = 0;
  c->next_mode.assign(B, EC_FULL); c->has_full.assign(B, 0); c->done.assign(B, 0);
  c->n_mb.assign(B, 0); c->n_rows_partial.assign(B, 0);
  c->masked_host.assign(c->g.xtot, 0);
  for (int b = 0; b < B; ++b) {
    c->n_mb[b] = c->host_out[b].next_n_mb;
    c->n_rows_partial[b] = c->host_out[b].next_n_rows_partial;
    for (int i = c->g.P[b]; i < c->g.T[b]; ++i) c->masked_host[c->g.x_off[b] + i] = 1;
  }
  c->rows_recomputed = 0; c->full_steps = c->partial_steps = c->tokens = 0;
  return EC_OK;
}

// What the host worked out for one step.
struct StepPlan {
  int R = 0, n_lm = 0;                      // rows of the list (with padding), masked block rows
  bool has_small = false, has_large = false;
  int max_T_small = 1;
  int npairs = 0;                           // (row tile, sequence) visits of few-row sequences
  int nsmall = 0, max_visits = 0;           // few-row sequences; most visits of one of them
  bool single = false;                      // one sequence takes part: one_seq is its tile entry
  int4 one_seq = make_int4(0, 0, 32, 0);
  int64_t rows = 0;                         // sum of the sequences' own row counts
  int n_full = 0, n_partial = 0;            // sequences running in each mode
};

// ---- the forward pass of one step (float32: batch 1, the sequence's M rows) --------------------
int forward_f32(ec_ctx* c, int mode, int M, int n_mb) {
  const ec_model_cfg& m = c->m;
  Buffers& b = c->b;
  hipStream_t s = c->stream;
  const int d = m.d_model, F = m.d_ffn, hd = m.head_dim, T = c->g.T[0];
  const int nq = m.n_heads * hd, nkv = m.n_kv_heads * hd, nqkv = nq + 2 * nkv;
  const int* rows = (mode == EC_FULL) ? nullptr : b.rows_partial;
  const int* lm_sel = (mode == EC_FULL) ? b.mb_pos : b.mb_idx;
  float* u = (float*)b.u; float* q = (float*)b.q; float* attn = (float*)b.attn;
  float* act = (float*)b.act; float* u_lm = (float*)b.u_lm;
  auto W = [](const void* p) { return (const float*)p; };

  { Scope p(c, EC_K_EMBED); launch_embed_f32(W(c->w.tok_emb), b.x, rows, M, d, m.vocab, b.h, s); }
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
      launch_attention_f32(q, kc, vc, M, T, m.n_heads, m.n_kv_heads, hd, attn, s); }
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

// bf16: the rows of all sequences in one list; five launches per layer.  Norms, RoPE, the KV
// scatter, SwiGLU and the residual adds run in the GEMM epilogues; `u` always holds the next
// GEMM's operand bf16(h * gain).
int forward_bf16(ec_ctx* c, const StepPlan& sp) {
  const ec_model_cfg& m = c->m;
  Buffers& b = c->b;
  hipStream_t s = c->stream;
  const int d = m.d_model, F = m.d_ffn, hd = m.head_dim, L = m.n_layers;
  const int nq = m.n_heads * hd, nkv = m.n_kv_heads * hd, nqkv = nq + 2 * nkv;
  // R rows in the list; the GEMMs work on M of them: all, or with a single sequence only its own
  // rows (the tail of the last tile is padding: skipping it saves the activation reads)
  const int R = sp.R, MT = (R + 15) / 16, M = sp.single ? (int)sp.rows : R;
  bf16_t* u = (bf16_t*)b.u; bf16_t* q = (bf16_t*)b.q; bf16_t* attn = (bf16_t*)b.attn;
  bf16_t* act = (bf16_t*)b.act;
  auto G = [](const void* p) { return (const bf16_t*)p; };
  auto sums = [&](int i) { return b.sumsq + (size_t)i * kSumSlots * b.sumsq_stride; };

  { Scope p(c, EC_K_EMBED);
    StepLists sl{};
    sl.seqs = c->B == 1 ? nullptr : b.seqs; sl.seq0 = c->host_seqs[0]; sl.B = c->B; sl.R = R; sl.n_lm = sp.n_lm; sl.x = b.x;
    sl.rows_partial = b.rows_partial; sl.mb_pos = b.mb_pos; sl.mb_idx = b.mb_idx;
    sl.vocab = m.vocab;
    sl.block = c->d.block; sl.rowinfo = b.rowinfo; sl.tileinfo = b.tileinfo; sl.lm_sel = b.lm_sel;
    launch_step_prologue_bf16(sl, G(c->w.tok_emb), d, G(c->attn_norm[0]), b.h, u, b.sumsq,
                              (2 * L + 1) * kSumSlots, b.sumsq_stride, s); }
  for (int l = 0; l < L; ++l) {
    bf16_t* kc = (bf16_t*)kv_ptr(c, l, 0); bf16_t* vc = (bf16_t*)kv_ptr(c, l, 1);
    { Scope p(c, EC_K_QKV);
      GemmEpi e{}; e.M = M; e.MT = MT; e.sumsq_in = sums(2 * l); e.d_in = d; e.eps = m.rms_eps;
      e.sum_stride = b.sumsq_stride; e.rowinfo = b.rowinfo; e.cs = b.rope_cs; e.Hq = m.n_heads;
      e.Hkv = m.n_kv_heads; e.hd = hd; e.q_out = q; e.kc = kc; e.vc = vc;
      e.w_grp = skinny_tiles_per_block(EPI_QKV, nqkv / 16); e.wscale = b.pl[l].sqkv;
      launch_gemm_bf16(EPI_QKV, u, R, b.pl[l].wqkv, b.pl[l].qqkv, nqkv, d, e, s); }
    { Scope p(c, EC_K_ATTN);
      launch_attention_mfma(q, kc, vc, R, b.rowinfo, sp.single ? nullptr : b.tileinfo,
                            sp.single ? nullptr : b.pairs + c->B, sp.npairs,
                            sp.single ? nullptr : b.pairs, sp.nsmall, sp.max_visits, sp.one_seq,
                            sp.has_small, sp.has_large, sp.max_T_small, m.n_heads, m.n_kv_heads, hd,
                            attn, b.ksplit_part, b.ksplit_floats, b.attn_tickets, s); }
    { Scope p(c, EC_K_OPROJ);
      GemmEpi e{}; e.M = M; e.MT = MT; e.h = b.h; e.d = d; e.gain_next = G(c->mlp_norm[l]);
      e.a_next = u; e.sumsq_out = sums(2 * l + 1); e.sum_stride = b.sumsq_stride;
      e.partial = b.ksplit_part; e.max_ksplit = kMaxKSplit;
      e.w_grp = skinny_tiles_per_block(EPI_RESID, d / 16); e.wscale = b.pl[l].so;
      launch_gemm_bf16(EPI_RESID, attn, R, b.pl[l].wo, b.pl[l].qo, d, nq, e, s); }
    { Scope p(c, EC_K_GATEUP);
      GemmEpi e{}; e.M = M; e.MT = MT; e.sumsq_in = sums(2 * l + 1); e.d_in = d; e.eps = m.rms_eps;
      e.sum_stride = b.sumsq_stride; e.act = act;
      e.w_grp = skinny_tiles_per_block(EPI_SWIGLU, 2 * F / 16); e.wscale = b.pl[l].sgu;
      launch_gemm_bf16(EPI_SWIGLU, u, R, b.pl[l].wgu, b.pl[l].qgu, 2 * F, d, e, s); }
    { Scope p(c, EC_K_DOWN);
      GemmEpi e{}; e.M = M; e.MT = MT; e.h = b.h; e.d = d;
      e.gain_next = G(l + 1 < L ? c->attn_norm[l + 1] : c->w.final_norm);
      e.a_next = u; e.sumsq_out = sums(2 * l + 2); e.sum_stride = b.sumsq_stride;
      e.partial = b.ksplit_part; e.max_ksplit = kMaxKSplit;
      e.w_grp = skinny_tiles_per_block(EPI_RESID, d / 16); e.wscale = b.pl[l].sd;
      launch_gemm_bf16(EPI_RESID, act, R, b.pl[l].wd, b.pl[l].qd, d, F, e, s); }
  }
  // logits only for the blocks' masked rows: the LM head gathers them from `u`
  { Scope p(c, EC_K_LMHEAD);
    GemmEpi e{}; e.M = sp.n_lm; e.MT = (sp.n_lm + 15) / 16; e.row_sel = b.lm_sel;
    e.sumsq_in = sums(2 * L); e.d_in = d; e.eps = m.rms_eps; e.sum_stride = b.sumsq_stride;
    e.scale = m.logit_scale; e.logits = b.logits; e.ldc = m.vocab;
    e.w_grp = skinny_tiles_per_block(EPI_LOGITS, m.vocab / 16); e.wscale = b.lm_head_s;
    if (sp.n_lm <= kLmSkinnyRows) {
      // the epilogue reduces the vocabulary itself; the logits go to memory only on request
      e.vparts = b.partials;
      if (!c->keep_logits) e.logits = nullptr;
      c->fused_reduce = true; c->step_nparts = lm_head_parts(m.vocab);
      c->logits_stored = c->keep_logits;
      launch_gemm_bf16(EPI_LOGITS, u, R, b.lm_head_p, b.lm_head_q, m.vocab, d, e, s);
    } else {  // many sequences: gather the rows once, then one pass over the LM head
      c->fused_reduce = false; c->step_nparts = vocab_reduce_parts(m.vocab);
      c->logits_stored = true;
      launch_gather_rows_packed(u, R, b.lm_sel, sp.n_lm, d, (bf16_t*)b.u_lm, s);
      launch_gemm_bf16(EPI_LOGITS, (bf16_t*)b.u_lm, sp.n_lm, b.lm_head_p, b.lm_head_q, m.vocab, d, e, s);
    } }
  return EC_OK;
}

// One step for every unfinished sequence.  modes: one entry per sequence or a single shared one
// (modes_n == 1).  forced_n: NULL, or per sequence the number of (position, token) pairs to
// commit, the pairs concatenated in fpos / ftok.
int run_step(ec_ctx* c, const int32_t* modes, int modes_n, const int32_t* forced_n,
             const int32_t* fpos, const int32_t* ftok, ec_step_result* out) {
  if (!c) return fail(nullptr, EC_ERR_ARG, "ctx is NULL");
  if (!out) return fail(c, EC_ERR_ARG, "out is NULL");
  if (!modes) return fail(c, EC_ERR_ARG, "modes is NULL");
  if (c->all_done) return fail(c, EC_ERR_STATE, "generation is finished: no masked position left");
  const int B = c->B;
  // ---- validate, resolve the modes -------------------------------------------------------------
  std::vector<int> mode(B, -1);
  size_t foff = 0;
  for (int b = 0; b < B; ++b) {
    int mb = modes[modes_n == 1 ? 0 : b];
    if (mb != EC_FULL && mb != EC_PARTIAL && mb != EC_AUTO)
      return fail(c, EC_ERR_ARG, "mode must be EC_FULL, EC_PARTIAL or EC_AUTO");
    const int fn = forced_n ? forced_n[b] : -1;
    if (forced_n && fn < 0) return fail(c, EC_ERR_ARG, "n must be >= 0");
    if (c->done[b]) { foff += fn > 0 ? fn : 0; continue; }
    if (mb == EC_AUTO) mb = (c->steps_run == 0) ? EC_FULL : c->next_mode[b];
    if (mb == EC_PARTIAL && !c->has_full[b])
      return fail(c, EC_ERR_STATE, "PARTIAL step before any FULL step: the KV cache is empty");
    mode[b] = mb;
    if (fn >= 0) {
      if (fn > EC_MAX_N) return fail(c, EC_ERR_ARG, "more than EC_MAX_N forced tokens");
      if (fn > 0 && (!fpos || !ftok)) return fail(c, EC_ERR_ARG, "forced lists are NULL");
      for (int i = 0; i < fn; ++i) {
        const int p = fpos[foff + i];
        if (p < c->g.P[b] || p >= c->g.T[b] || !c->masked_host[c->g.x_off[b] + p])
          return fail(c, EC_ERR_ARG, "forced position is not a masked generation slot");
        if (ftok[foff + i] < 0 || ftok[foff + i] >= c->m.vocab)
          return fail(c, EC_ERR_ARG, "forced token outside the vocabulary");
        for (int j = 0; j < i; ++j)
          if (fpos[foff + j] == p) return fail(c, EC_ERR_ARG, "forced position listed twice");
      }
      foff += fn;
    }
  }
  // ---- the step's row list: many-row sequences first -------------------------------------------
  StepPlan sp;
  for (int pass = 0; pass < 2; ++pass) {
    foff = 0;
    for (int b = 0; b < B; ++b) {
      const int fn = forced_n ? forced_n[b] : -1;
      const size_t f0 = foff;
      foff += fn > 0 ? fn : 0;
      if (pass == 0) c->host_seqs[b] = base_desc(c, b);
      if (mode[b] < 0) continue;
      const int n_rows = mode[b] == EC_FULL ? c->g.T[b] : c->n_rows_partial[b];
      const bool large = n_rows > kSmallRows;
      if (large != (pass == 0)) continue;
      SeqDesc& sd = c->host_seqs[b];
      sd.mode = mode[b]; sd.n_rows = n_rows; sd.row0 = sp.R;
      sd.seg_rows = large ? seg_rows_of(n_rows) : n_rows;   // few-row sequences: back to back
      sd.n_mb = c->n_mb[b]; sd.forced_n = fn;
      if (!large) {
        // the table starts with one entry per few-row sequence (its first visit, how many),
        // the visits follow from entry B on
        const int first = sp.npairs;
        for (int mt = sd.row0 / 16; mt <= (sd.row0 + n_rows - 1) / 16; ++mt)
          c->host_pairs[B + sp.npairs++] = make_int4(mt, sd.kv_off, sd.T, sd.tpad);
        c->host_pairs[sp.nsmall++] = make_int4(first, sp.npairs - first, 0, 0);
        if (sp.npairs - first > sp.max_visits) sp.max_visits = sp.npairs - first;
      }
      sp.R += sd.seg_rows; sp.rows += n_rows;
      (large ? sp.has_large : sp.has_small) = true;
      if (!large && c->g.T[b] > sp.max_T_small) sp.max_T_small = c->g.T[b];
      (mode[b] == EC_FULL ? sp.n_full : sp.n_partial) += 1;
      if (fn > 0) {
        memcpy(c->host_stage + (size_t)b * EC_MAX_N, fpos + f0, fn * sizeof(int));
        memcpy(c->host_stage + (size_t)(B + b) * EC_MAX_N, ftok + f0, fn * sizeof(int));
      }
    }
  }
  for (int b = 0; b < B; ++b)
    if (mode[b] >= 0) {
      SeqDesc& sd = c->host_seqs[b];
      sd.lm0 = sp.n_lm;
      sp.n_lm += c->n_mb[b];
      sp.one_seq = make_int4(sd.kv_off, sd.T, sd.tpad, sd.n_rows > kSmallRows ? 1 : 0);
    }
  sp.single = sp.n_full + sp.n_partial == 1;
  sp.R = (sp.R + 15) / 16 * 16;
  if (!sp.single && sp.npairs > 0)
    EC_HIP(c, hipMemcpyAsync(c->b.pairs, c->host_pairs, (size_t)(B + sp.npairs) * sizeof(int4),
                             hipMemcpyHostToDevice, c->stream));
  if (B > 1)
    EC_HIP(c, hipMemcpyAsync(c->b.seqs, c->host_seqs, (size_t)B * sizeof(SeqDesc),
                             hipMemcpyHostToDevice, c->stream));
  if (forced_n) {
    EC_HIP(c, hipMemcpyAsync(c->b.forced_pos, c->host_stage, (size_t)B * EC_MAX_N * sizeof(int),
                             hipMemcpyHostToDevice, c->stream));
    EC_HIP(c, hipMemcpyAsync(c->b.forced_tok, c->host_stage + (size_t)B * EC_MAX_N,
                             (size_t)B * EC_MAX_N * sizeof(int), hipMemcpyHostToDevice, c->stream));
  }
  // ---- forward, vocabulary reduction, decision ---------------------------------------------------
  c->fused_reduce = false; c->step_nparts = vocab_reduce_parts(c->m.vocab); c->logits_stored = true;
  int rc = (c->m.dtype == EC_F32) ? forward_f32(c, mode[0], c->host_seqs[0].n_rows, c->n_mb[0])
                                  : forward_bf16(c, sp);
  if (rc != EC_OK) return rc;
  if (!c->fused_reduce) {
    Scope p(c, EC_K_VOCAB_REDUCE);
    launch_vocab_reduce(c->b.logits, sp.n_lm, c->m.vocab, (size_t)c->m.vocab, c->b.partials, c->stream);
  }
  EC_HIP(c, hipGetLastError());
  DecideArgs a{};
  fill_decide_args(c, a);
  { Scope p(c, EC_K_DECIDE); launch_decide(a, B, c->stream); }
  EC_HIP(c, hipGetLastError());
  // the decision kernel writes the results straight into pinned host memory
  if (c->prof_on) {
    EC_HIP(c, hipStreamSynchronize(c->stream));
    prof_collect(c);
  } else {
    int rcw = wait_results(c, mode.data());
    if (rcw != EC_OK) return rcw;
  }

  // ---- mirror the new state ------------------------------------------------------------------------
  c->steps_run += 1;
  c->rows_recomputed += sp.rows;
  c->full_steps += sp.n_full;
  c->partial_steps += sp.n_partial;
  std::vector<DevState> st;
  if (forced_n) {
    // the flags follow the committed tokens; the device computed them, mirror them from its state
    st.resize(B);
    EC_HIP(c, hipStreamSynchronize(c->stream));
    EC_HIP(c, hipMemcpy(st.data(), c->b.st, (size_t)B * sizeof(DevState), hipMemcpyDeviceToHost));
  }
  int all_done = 1;
  foff = 0;
  for (int b = 0; b < B; ++b) {
    const int fn = forced_n ? forced_n[b] : -1;
    const size_t f0 = foff;
    foff += fn > 0 ? fn : 0;
    if (mode[b] < 0) {  // finished before this step
      memset(&out[b], 0, sizeof(ec_step_result));
      out[b].done = 1;
      continue;
    }
    const StepOut& o = c->host_out[b];
    c->has_full[b] |= (mode[b] == EC_FULL);
    c->done[b] = o.r.done;
    c->n_mb[b] = o.next_n_mb;
    c->n_rows_partial[b] = o.next_n_rows_partial;
    uint8_t* mh = c->masked_host.data() + c->g.x_off[b];
    if (fn >= 0) {
      for (int i = 0; i < fn; ++i) mh[fpos[f0 + i]] = 0;
      c->tokens += fn;
      c->next_mode[b] = st[b].skip ? EC_PARTIAL : EC_FULL;
    } else {
      for (int i = 0; i < o.r.n_unmasked; ++i) mh[o.r.positions[i]] = 0;
      c->tokens += o.r.n_unmasked;
      c->next_mode[b] = o.r.next_mode;
    }
    out[b] = o.r;
    all_done &= c->done[b];
  }
  c->all_done = all_done;
  for (int b = 0; b < B; ++b)
    if (mode[b] >= 0 && c->host_out[b].nonfinite)
      return fail(c, EC_ERR_NONFINITE,
                  "a block row's logits had no finite maximum (sequence " + std::to_string(b) +
                      "): the step's results are meaningless, reset before going on");
  return EC_OK;
}

}  // namespace

// =============================================================================================
// C ABI
// =============================================================================================
// No exception may cross the C boundary: the bodies run under this guard.
template <typename Fn> static int guarded(ec_ctx* c, Fn&& fn) {
  try {
    return fn();
  } catch (const std::bad_alloc&) {
    try { fail(c, EC_ERR_HOST_MEMORY, "out of host memory"); } catch (...) {}
    return EC_ERR_HOST_MEMORY;
  } catch (...) {
    try { fail(c, EC_ERR_ARG, "unexpected exception"); } catch (...) {}
    return EC_ERR_ARG;
  }
}

extern "C" {

size_t ec_workspace_bytes(const ec_model_cfg* model, const ec_decode_cfg* decode,
                          const int32_t* prompt_lens) {
  if (!model || !decode || !prompt_lens) return 0;
  if (decode->batch < 1 || decode->batch > EC_MAX_BATCH) return 0;
  try {
    if (check_config(model, decode, prompt_lens) != nullptr) return 0;
    Carver c(nullptr);
    Buffers b;
    carve(c, *model, *decode, geometry(*model, *decode, prompt_lens), b);
    return c.off;
  } catch (...) {
    return 0;
  }
}

static int init_impl(ec_ctx** out, const ec_model_cfg* model, const ec_weights* weights,
                     const ec_decode_cfg* decode, const int32_t* prompt_ids,
                     const int32_t* prompt_lens, void* workspace, size_t workspace_bytes,
                     void* hip_stream) {
  if (!out) return fail(nullptr, EC_ERR_ARG, "out is NULL");
  *out = nullptr;
  if (!model || !weights || !decode || !prompt_lens)
    return fail(nullptr, EC_ERR_ARG, "model, weights, decode and prompt_lens must not be NULL");
  if (decode->batch < 1 || decode->batch > EC_MAX_BATCH)
    return fail(nullptr, EC_ERR_CONFIG, "batch must be in [1, EC_MAX_BATCH]");
  if (const char* msg = check_config(model, decode, prompt_lens))
    return fail(nullptr, EC_ERR_CONFIG, msg);
  Geometry g = geometry(*model, *decode, prompt_lens);
  if (g.ptot > 0 && !prompt_ids) return fail(nullptr, EC_ERR_ARG, "prompt_ids is NULL");
  for (size_t i = 0; i < g.ptot; ++i)
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
  if (model->dtype == EC_FP8W) {
    if (!weights->lm_head_scale || !weights->wq_scale || !weights->wk_scale || !weights->wv_scale ||
        !weights->wo_scale || !weights->w_gate_scale || !weights->w_up_scale || !weights->w_down_scale)
      return fail(nullptr, EC_ERR_ARG, "EC_FP8W: a scale pointer is NULL");
    for (int l = 0; l < model->n_layers; ++l)
      if (!weights->wq_scale[l] || !weights->wk_scale[l] || !weights->wv_scale[l] ||
          !weights->wo_scale[l] || !weights->w_gate_scale[l] || !weights->w_up_scale[l] ||
          !weights->w_down_scale[l])
        return fail(nullptr, EC_ERR_ARG, "EC_FP8W: a per-layer scale pointer is NULL");
  }
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
  const int L = model->n_layers, B = decode->batch;
  c->attn_norm.assign(weights->attn_norm, weights->attn_norm + L);
  c->wq.assign(weights->wq, weights->wq + L); c->wk.assign(weights->wk, weights->wk + L);
  c->wv.assign(weights->wv, weights->wv + L); c->wo.assign(weights->wo, weights->wo + L);
  c->mlp_norm.assign(weights->mlp_norm, weights->mlp_norm + L);
  c->w_gate.assign(weights->w_gate, weights->w_gate + L);
  c->w_up.assign(weights->w_up, weights->w_up + L);
  c->w_down.assign(weights->w_down, weights->w_down + L);
  if (model->dtype == EC_FP8W) {
    c->wq_s.assign(weights->wq_scale, weights->wq_scale + L);
    c->wk_s.assign(weights->wk_scale, weights->wk_scale + L);
    c->wv_s.assign(weights->wv_scale, weights->wv_scale + L);
    c->wo_s.assign(weights->wo_scale, weights->wo_scale + L);
    c->w_gate_s.assign(weights->w_gate_scale, weights->w_gate_scale + L);
    c->w_up_s.assign(weights->w_up_scale, weights->w_up_scale + L);
    c->w_down_s.assign(weights->w_down_scale, weights->w_down_scale + L);
  }
  c->g = g; c->B = B; c->N = decode->gen_len;
  c->stream = (hipStream_t)hip_stream;
  Carver cv(workspace);
  carve(cv, c->m, c->d, c->g, c->b);

  auto bail = [&](int code, const std::string& msg) {
    if (c->host_out) (void)hipHostFree(c->host_out);
    if (c->host_stage) (void)hipHostFree(c->host_stage);
    if (c->host_seqs) (void)hipHostFree(c->host_seqs);
    if (c->host_pairs) (void)hipHostFree(c->host_pairs);
    delete c;
    return fail(nullptr, code, msg);
  };
  hipError_t e = hipHostMalloc((void**)&c->host_out, (size_t)B * sizeof(StepOut), hipHostMallocCoherent);
  if (e != hipSuccess) return bail(EC_ERR_HIP, std::string("hipHostMalloc: ") + hipGetErrorString(e));
  e = hipHostGetDevicePointer((void**)&c->host_out_dev, c->host_out, 0);
  if (e != hipSuccess) return bail(EC_ERR_HIP, std::string("hipHostGetDevicePointer: ") + hipGetErrorString(e));
  memset(c->host_out, 0, (size_t)B * sizeof(StepOut));
  size_t stage = (g.ptot > (size_t)2 * B * EC_MAX_N ? g.ptot : (size_t)2 * B * EC_MAX_N) * sizeof(int);
  e = hipHostMalloc((void**)&c->host_stage, stage, hipHostMallocDefault);
  if (e != hipSuccess) return bail(EC_ERR_HIP, std::string("hipHostMalloc: ") + hipGetErrorString(e));
  e = hipHostMalloc((void**)&c->host_seqs, (size_t)B * sizeof(SeqDesc), hipHostMallocDefault);
  if (e != hipSuccess) return bail(EC_ERR_HIP, std::string("hipHostMalloc: ") + hipGetErrorString(e));
  e = hipHostMalloc((void**)&c->host_pairs, (g.rmax / 16 + 2 * B) * sizeof(int4), hipHostMallocDefault);
  if (e != hipSuccess) return bail(EC_ERR_HIP, std::string("hipHostMalloc: ") + hipGetErrorString(e));

  // one-time device set-up: RoPE table, re-tiled bf16 matrices, finite padding keys
  launch_rope_table(c->b.rope_cs, g.tmax, c->m.head_dim, c->m.rope_base, c->stream);
  if (bf16_path(c->m.dtype)) {
    size_t kvbytes = (size_t)L * 2 * c->b.kv_plane * 2;
    e = hipMemsetAsync(c->b.kv, 0, kvbytes, c->stream);
    if (e == hipSuccess) e = hipMemsetAsync(c->b.attn_tickets, 0, 256 * sizeof(int), c->stream);
    // the last tile's padding rows of q and of the attention output are never written: zeros
    const size_t qbytes = g.rmax * (size_t)c->m.n_heads * c->m.head_dim * 2;
    if (e == hipSuccess) e = hipMemsetAsync(c->b.q, 0, qbytes, c->stream);
    if (e == hipSuccess) e = hipMemsetAsync(c->b.attn, 0, qbytes, c->stream);
    if (e != hipSuccess) return bail(EC_ERR_HIP, std::string("hipMemsetAsync: ") + hipGetErrorString(e));
    const int d = c->m.d_model, F = c->m.d_ffn;
    const int nq = c->m.n_heads * c->m.head_dim, nkv = c->m.n_kv_heads * c->m.head_dim;
    const int hd = c->m.head_dim;
    auto Bp = [](const void* p) { return (const bf16_t*)p; };
    auto Qp = [](const void* p) { return (const uint8_t*)p; };
    const bool quant = c->m.dtype == EC_FP8W;
    const int glm = skinny_tiles_per_block(EPI_LOGITS, c->m.vocab / 16);
    for (int l = 0; l < L; ++l) {
      PackedLayer& p = c->b.pl[l];
      const int gq = skinny_tiles_per_block(EPI_QKV, (nq + 2 * nkv) / 16);
      const int go = skinny_tiles_per_block(EPI_RESID, d / 16);
      const int gg = skinny_tiles_per_block(EPI_SWIGLU, 2 * F / 16);
      if (!quant) {
        launch_repack_weight(Bp(c->wq[l]), nq, d, p.wqkv, REPACK_ROPE_HALVES, hd, gq, 0, c->stream);
        launch_repack_weight(Bp(c->wk[l]), nkv, d, p.wqkv, REPACK_ROPE_HALVES, hd, gq, nq, c->stream);
        launch_repack_weight(Bp(c->wv[l]), nkv, d, p.wqkv, REPACK_PLAIN, hd, gq, nq + nkv, c->stream);
        launch_repack_weight(Bp(c->wo[l]), d, nq, p.wo, REPACK_PLAIN, hd, go, 0, c->stream);
        launch_repack_weight(Bp(c->w_gate[l]), F, d, p.wgu, REPACK_LO8, hd, gg, 0, c->stream);
        launch_repack_weight(Bp(c->w_up[l]), F, d, p.wgu, REPACK_HI8, hd, gg, 0, c->stream);
        launch_repack_weight(Bp(c->w_down[l]), d, F, p.wd, REPACK_PLAIN, hd, go, 0, c->stream);
        continue;
      }
      // e4m3 codes: fragment pairs for the weight-streaming kernels, exact bf16 fragments for
      // the tiled ones, and the row scales in the packed matrices' row order
      struct Part { const void* w; const float* sc; int N, K; uint8_t* q; bf16_t* p; float* s; int mode, grp, row0; };
      const Part parts[] = {
          {c->wq[l], c->wq_s[l], nq, d, p.qqkv, p.wqkv, p.sqkv, REPACK_ROPE_HALVES, gq, 0},
          {c->wk[l], c->wk_s[l], nkv, d, p.qqkv, p.wqkv, p.sqkv, REPACK_ROPE_HALVES, gq, nq},
          {c->wv[l], c->wv_s[l], nkv, d, p.qqkv, p.wqkv, p.sqkv, REPACK_PLAIN, gq, nq + nkv},
          {c->wo[l], c->wo_s[l], d, nq, p.qo, p.wo, p.so, REPACK_PLAIN, go, 0},
          {c->w_gate[l], c->w_gate_s[l], F, d, p.qgu, p.wgu, p.sgu, REPACK_LO8, gg, 0},
          {c->w_up[l], c->w_up_s[l], F, d, p.qgu, p.wgu, p.sgu, REPACK_HI8, gg, 0},
          {c->w_down[l], c->w_down_s[l], d, F, p.qd, p.wd, p.sd, REPACK_PLAIN, go, 0}};
      for (const Part& t : parts) {
        launch_repack_weight_e4m3(Qp(t.w), t.N, t.K, t.q, t.p, t.mode, hd, t.grp, t.row0, c->stream);
        launch_repack_rows_f32(t.sc, t.N, t.s, t.mode, hd, t.row0, c->stream);
      }
    }
    if (!quant) {
      launch_repack_weight(Bp(c->w.lm_head), c->m.vocab, d, c->b.lm_head_p, REPACK_PLAIN, hd, glm, 0,
                           c->stream);
    } else {
      launch_repack_weight_e4m3(Qp(c->w.lm_head), c->m.vocab, d, c->b.lm_head_q, c->b.lm_head_p,
                                REPACK_PLAIN, hd, glm, 0, c->stream);
      launch_repack_rows_f32(c->w.lm_head_scale, c->m.vocab, c->b.lm_head_s, REPACK_PLAIN, hd, 0,
                             c->stream);
    }
  }
  e = hipGetLastError();
  if (e != hipSuccess) return bail(EC_ERR_HIP, std::string("set-up kernels: ") + hipGetErrorString(e));
  int rc = upload_and_init_state(c, prompt_ids);
  if (rc != EC_OK) return bail(rc, c->err);
  *out = c;
  return EC_OK;
}

int ec_init(ec_ctx** out, const ec_model_cfg* model, const ec_weights* weights,
            const ec_decode_cfg* decode, const int32_t* prompt_ids, const int32_t* prompt_lens,
            void* workspace, size_t workspace_bytes, void* hip_stream) {
  return guarded(nullptr, [&] {
    return init_impl(out, model, weights, decode, prompt_ids, prompt_lens, workspace,
                     workspace_bytes, hip_stream);
  });
}

int ec_reset(ec_ctx* ctx, const int32_t* prompt_ids) {
  return guarded(ctx, [&]() -> int {
    if (!ctx) return fail(nullptr, EC_ERR_ARG, "ctx is NULL");
    if (ctx->g.ptot > 0 && !prompt_ids) return fail(ctx, EC_ERR_ARG, "prompt_ids is NULL");
    for (size_t i = 0; i < ctx->g.ptot; ++i)
      if (prompt_ids[i] < 0 || prompt_ids[i] >= ctx->m.vocab)
        return fail(ctx, EC_ERR_ARG, "prompt id outside the vocabulary");
    return upload_and_init_state(ctx, prompt_ids);
  });
}

int ec_step(ec_ctx* ctx, int mode, ec_step_result* out) {
  const int32_t m = mode;
  return guarded(ctx, [&] { return run_step(ctx, &m, 1, nullptr, nullptr, nullptr, out); });
}

int ec_step_forced(ec_ctx* ctx, int mode, int32_t n, const int32_t* positions,
                   const int32_t* tokens, ec_step_result* out) {
  if (ctx && ctx->B != 1)
    return fail(ctx, EC_ERR_ARG, "ec_step_forced is for batch 1; use ec_step_forced_batch");
  if (n < 0) return fail(ctx, EC_ERR_ARG, "n must be >= 0");
  const int32_t m = mode;
  return guarded(ctx, [&] { return run_step(ctx, &m, 1, &n, positions, tokens, out); });
}

int ec_step_forced_batch(ec_ctx* ctx, const int32_t* modes, const int32_t* n,
                         const int32_t* positions, const int32_t* tokens, ec_step_result* out) {
  if (!ctx) return fail(nullptr, EC_ERR_ARG, "ctx is NULL");
  if (!n) return fail(ctx, EC_ERR_ARG, "n is NULL");
  return guarded(ctx, [&] { return run_step(ctx, modes, ctx->B, n, positions, tokens, out); });
}

int ec_generate(ec_ctx* ctx, int32_t* out_tokens, ec_gen_stats* stats) {
  if (!ctx) return fail(nullptr, EC_ERR_ARG, "ctx is NULL");
  if (!out_tokens) return fail(ctx, EC_ERR_ARG, "out_tokens is NULL");
  return guarded(ctx, [&]() -> int {
    auto t0 = std::chrono::steady_clock::now();
    std::vector<ec_step_result> r(ctx->B);
    const int32_t m = EC_AUTO;
    while (!ctx->all_done) {
      int rc = run_step(ctx, &m, 1, nullptr, nullptr, nullptr, r.data());
      if (rc != EC_OK) return rc;
    }
    for (int b = 0; b < ctx->B; ++b)
      EC_HIP(ctx, hipMemcpy(out_tokens + (size_t)b * ctx->N, ctx->b.x + ctx->g.x_off[b] + ctx->g.P[b],
                            (size_t)ctx->N * sizeof(int), hipMemcpyDeviceToHost));
    if (stats) {
      stats->steps = ctx->steps_run; stats->full_steps = ctx->full_steps;
      stats->partial_steps = ctx->partial_steps; stats->tokens = ctx->tokens;
      stats->rows_recomputed = ctx->rows_recomputed;
      stats->ms_total = std::chrono::duration<double, std::milli>(
                            std::chrono::steady_clock::now() - t0).count();
    }
    return EC_OK;
  });
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

int ec_debug_read_seq(ec_ctx* ctx, int seq, int what, int layer, void* host_dst, size_t bytes) {
  if (!ctx) return fail(nullptr, EC_ERR_ARG, "ctx is NULL");
  if (!host_dst) return fail(ctx, EC_ERR_ARG, "host_dst is NULL");
  if (seq < 0 || seq >= ctx->B) return fail(ctx, EC_ERR_ARG, "sequence index out of range");
  const void* src = nullptr;
  size_t avail = 0;
  const size_t es = esize(ctx->m.dtype);
  const size_t kvrow = (size_t)ctx->m.n_kv_heads * ctx->m.head_dim * es;
  const int T = ctx->g.T[seq], xo = ctx->g.x_off[seq], blk = ctx->d.block;
  switch (what) {
    case EC_DBG_LOGITS:
      // rows of the last step, at the place the step gave them in the logits buffer
      src = ctx->b.logits + (size_t)ctx->host_seqs[seq].lm0 * ctx->m.vocab;
      avail = (size_t)blk * ctx->m.vocab * 4;
      if (ctx->host_seqs[seq].mode < 0) avail = 0;
      if (!ctx->logits_stored)
        return fail(ctx, EC_ERR_STATE, "the last step did not store its logits: ec_debug_keep_logits");
      break;
    case EC_DBG_KCACHE:
    case EC_DBG_VCACHE:
      if (layer < 0 || layer >= ctx->m.n_layers) return fail(ctx, EC_ERR_ARG, "layer out of range");
      src = kv_ptr(ctx, layer, what == EC_DBG_VCACHE) + (size_t)ctx->g.kv_off[seq] * es;
      avail = (size_t)T * kvrow;
      if (bf16_path(ctx->m.dtype)) {
        // the packed cache is put back into [T, Hkv, hd] order in a scratch activation buffer
        launch_unpack_cache((const bf16_t*)src, what == EC_DBG_VCACHE, T, ctx->g.tpad[seq],
                            ctx->m.n_kv_heads, ctx->m.head_dim, (bf16_t*)ctx->b.qkv, ctx->stream);
        src = ctx->b.qkv;
      }
      break;
    case EC_DBG_X: src = ctx->b.x + xo; avail = (size_t)T * 4; break;
    case EC_DBG_MASKED: src = ctx->b.masked + xo; avail = (size_t)T; break;
    case EC_DBG_HIST: src = ctx->b.hist + (size_t)seq * ctx->N; avail = (size_t)ctx->N * 4; break;
    case EC_DBG_ROWS: src = ctx->b.rows_partial + xo; avail = (size_t)ctx->n_rows_partial[seq] * 4; break;
    case EC_DBG_ROW_STATS: src = ctx->b.row_stats + (size_t)seq * blk * 4; avail = (size_t)blk * 16; break;
    default: return fail(ctx, EC_ERR_ARG, "unknown debug item");
  }
  if (bytes > avail) return fail(ctx, EC_ERR_ARG, "bytes exceeds the size of the item");
  EC_HIP(ctx, hipStreamSynchronize(ctx->stream));
  if (bytes) EC_HIP(ctx, hipMemcpy(host_dst, src, bytes, hipMemcpyDeviceToHost));
  return EC_OK;
}

int ec_debug_keep_logits(ec_ctx* ctx, int on) {
  if (!ctx) return fail(nullptr, EC_ERR_ARG, "ctx is NULL");
  ctx->keep_logits = on != 0;
  return EC_OK;
}

int ec_debug_read(ec_ctx* ctx, int what, int layer, void* host_dst, size_t bytes) {
  return ec_debug_read_seq(ctx, 0, what, layer, host_dst, bytes);
}

void ec_destroy(ec_ctx* ctx) {
  if (!ctx) return;
  (void)hipStreamSynchronize(ctx->stream);
  for (auto& e : ctx->prof_pool) { (void)hipEventDestroy(e.a); (void)hipEventDestroy(e.b); }
  if (ctx->host_out) (void)hipHostFree(ctx->host_out);
  if (ctx->host_stage) (void)hipHostFree(ctx->host_stage);
  if (ctx->host_seqs) (void)hipHostFree(ctx->host_seqs);
  if (ctx->host_pairs) (void)hipHostFree(ctx->host_pairs);
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
    case EC_ERR_HOST_MEMORY: return "out of host memory";
    case EC_ERR_NONFINITE: return "logits without a finite maximum";
    default: return "unknown error code";
  }
}

const char* ec_last_error(const ec_ctx* ctx) {
  return ctx ? ctx->err.c_str() : g_init_error.c_str();
}

}  // extern "C"
