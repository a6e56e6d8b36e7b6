// Internal declarations shared by the host driver and the kernel translation units.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/ec.h"
#include "k_common.h"

namespace ec {

// Device-resident scalar state of one sequence (the algorithm's t, flag, counters, block).
struct DevState {
  int t;               // index of the NEXT step to run, starts at 1
  int t_lastfull;      // index of the last step that ran FULL (0 = none yet)
  int dt;              // Delta t_recompute, the paper's counter
  int skip;            // 1 = next EC_AUTO step is PARTIAL
  int blk;             // current block
  int done;
  int n_mb;            // |M^t| for the next step: masked rows of the current block
  int n_rows_partial;  // |M^t u R^t| for the next step
  int n_recent;        // |R^t|
  int pad[7];
};

// One sequence of the batch as a step sees it; the host rewrites the table before every step.
// A step's rows are the sequences' row sets one after the other: first the sequences with more
// than kSmallRows rows, each padded to 256 rows (so that an attention block's query tiles never
// straddle two of them), then the others back to back without padding; the list ends on a whole
// 16-row tile.
struct SeqDesc {
  int P, T, tpad;   // prompt length, positions, keys per cache slab (padded to 32)
  int x_off;        // first element of the sequence in x / masked / rows_partial
  int kv_off;       // first element of the sequence's slabs inside one layer's K (or V) plane
  int mode;         // EC_FULL / EC_PARTIAL this step, -1 = takes no part (finished)
  int n_rows;       // rows it contributes: T or |M u R|
  int row0;         // its first row in the step's row list
  int seg_rows;     // rows of its segment (with the padding of a many-row sequence)
  int n_mb, lm0;    // masked rows of its block; the first of them in the logits buffer
  int forced_n;     // teacher forcing: tokens to commit, -1 = the step's own choice
};
constexpr int kSmallRows = 96;

// What the decision kernel hands back to the host after each step.
struct StepOut {
  ec_step_result r;
  int next_n_mb;
  int next_n_rows_partial;
  int serial;   // the launch's DecideArgs::serial once everything above has been written
  int nonfinite;  // 1: some block row had no finite maximum logit (its token was forced to 0)
  int pad[4];
};

// Arguments of the decision kernel: one block per sequence.  The pointers are those of sequence
// 0; block b moves them by its SeqDesc (x_off) or by b times the per-sequence stride given in the
// comment, and takes P, T, n_mb, mode_run, n_rows_run, forced_n from its SeqDesc.
struct DecideArgs {
  const SeqDesc* seqs;     // NULL: a single sequence, described by seq0 (no table in memory)
  SeqDesc seq0;
  // this step
  const float4* partials;  // [lm0 + row][nparts] (max, argmax as float bits, sum e, sum e*(z-max))
  int nparts;
  int n_mb;
  int mode_run;
  int n_rows_run;
  int forced_n;            // -1: commit the step's own choice
  const int* forced_pos;   // device, stride EC_MAX_N
  const int* forced_tok;   // device, stride EC_MAX_N
  int init_only;           // 1: no decode, only build the lists of the first step
  // sequence state
  int* x;                  // [T] (x_off)
  uint8_t* masked;         // [T] (x_off)
  int* hist;               // [N], INT32_MIN = never decoded (stride N)
  DevState* st;            // (stride 1)
  int* mb_pos;             // [block] positions of the block's masked rows, ascending (stride block)
  int* rows_partial;       // [T] ascending positions of M u R (x_off)
  int* mb_idx;             // [block] index of each block row inside rows_partial (stride block)
  float* row_stats;        // [block][4] token, confidence, entropy, max logit (stride 4*block)
  StepOut* out;            // (stride 1) pinned host memory, written once by thread 0
  // configuration
  int P, N, T, block, k_recent, n_tok;
  float tau;
  float conf_threshold;    // 0 = fixed n_tok per step
  int gate_metric;         // EC_GATE_*
  int schedule;            // EC_SCHED_*
  int serial;              // written to StepOut::serial as the block's very last store (> 0)
  int vocab;               // a row's argmax must lie in [0, vocab)
};

// thread-local message behind ec_last_error(NULL)
void set_global_error(const char* msg);

// ---- launchers (each enqueues on `s`; shapes are validated by the caller) --------------------
// float32 path
void launch_embed_f32(const float* emb, const int* x, const int* rows, int M, int d, int vocab,
                      float* h, hipStream_t s);
// out row r = rmsnorm(h row sel[r] (or r)) * gain
void launch_rmsnorm_f32(const float* h, const int* sel, int M, int d, const float* gain, float eps,
                        float* out, hipStream_t s);
void launch_rope_table(float2* cs, int T, int hd, float base, hipStream_t s);
// caches row-major [T, Hkv*hd]
void launch_rope_scatter_f32(const float* qkv, const int* rows, int M, int Hq, int Hkv, int hd,
                             const float2* cs, float* q_out, float* kcache, float* vcache,
                             hipStream_t s);
void launch_swiglu_f32(const float* gu, int M, int F, float* act, hipStream_t s);
// C[M,N] (ldc) = scale * A[M,K] W[N,K]^T, or C += ... when accumulate.
void launch_gemm_f32(const float* A, const float* W, float* C, int ldc, int M, int N, int K,
                     int accumulate, float scale, hipStream_t s);
void launch_attention_f32(const float* q, const float* kc, const float* vc, int M, int T, int Hq,
                          int Hkv, int hd, float* out, hipStream_t s);

// bf16 path
enum { EPI_QKV = 0, EPI_RESID = 1, EPI_SWIGLU = 2, EPI_LOGITS = 3, EPI_PARTIAL = 4 };
constexpr int kMaxKSplit = 4;
// A row's sum of squares is accumulated by many blocks at once.  Atomics on one address
// serialise, so each row has kSumSlots counters (a block adds to the one its index selects) and
// the reader adds them up; integer addition keeps the total independent of the order.
constexpr int kSumSlots = 8;
enum { REPACK_PLAIN = 0, REPACK_ROPE_HALVES = 1, REPACK_LO8 = 2, REPACK_HI8 = 3 };

// What a GEMM epilogue needs (k_gemm_bf16.hip).  Row sums of squares are 44.20 fixed point.
struct GemmEpi {
  int M;                          // activation rows of this launch
  int MT;                         // m-tiles of the packed buffers written (a_next, act)
  const int* row_sel;             // nullable: activation row m is read from source row row_sel[m]
  const unsigned long long* sumsq_in;  // [kSumSlots][sum_stride], per SOURCE row: the slots add up
                                       // to the sum of squares of the normed input (44.20)
  int sum_stride;
  int w_grp;  // tiles per group of the weight matrix' layout (k_common.h)
  const float* wscale;            // nullable: per-row scales of a matrix that came as e4m3 codes,
                                  // in the packed matrix' row order; multiply the K-reduced sums
  int d_in;                       // its length
  float eps;
  float scale;                    // EPI_LOGITS
  float* logits; int ldc;         // (skinny kernel: nullable = do not store the logits)
  float4* vparts;                 // EPI_LOGITS, skinny kernel: [row][blocks] partial tuples of
                                  // the vocabulary reduction (k_vtuple.h), one per block
  float* h; int d;                // EPI_RESID: residual stream [M, d]
  float* partial; int max_ksplit; // nullable: room for [max_ksplit][M][d] fp32 partial products
  const bf16_t* gain_next;        // gain of the norm that follows
  bf16_t* a_next;                 // packed bf16(h * gain_next)
  unsigned long long* sumsq_out;  // [kSumSlots][sum_stride], accumulated with integer atomics
  bf16_t* act;                    // EPI_SWIGLU: packed activations, K = d_ffn
  const int4* rowinfo;            // EPI_QKV: per row (position or -1 for a padding row, index
                                  // into x, offset and keys per slab of its sequence's cache)
  const float2* cs;               // RoPE table [max T][hd/2]
  int Hq, Hkv, hd;
  bf16_t* q_out;                  // [M, Hq*hd] row-major
  bf16_t* kc; bf16_t* vc;         // the layer's packed caches
};

// First kernel of a step.  From the sequence table it writes the step's row list (rowinfo, one
// int4 per row as GemmEpi describes; tileinfo, one int4 per 16 rows: cache offset, positions,
// keys per slab, 1 if the sequence has more than kSmallRows rows) and lm_sel (for each masked
// row of a current block, its row in the list); then, per row, h = Emb[x], packed bf16(h * gain)
// for the first GEMM, the row's sum of squares into sumsq[0..R) and zeros into the nbuf-1
// further sum buffers (stride sumsq_stride) of the step.  Padding rows get zeros.
struct StepLists {
  const SeqDesc* seqs; int B;   // seqs == NULL: a single sequence, described by seq0
  SeqDesc seq0;
  int vocab;                    // token ids outside [0, vocab) are read as token 0
  int R, n_lm;                  // rows of the step (with padding); masked block rows
  const int* x;                 // concatenated by x_off, like rows_partial
  const int* rows_partial;
  const int* mb_pos;            // stride block
  const int* mb_idx;            // stride block
  int block;
  int4* rowinfo; int4* tileinfo; int* lm_sel;
};
void launch_step_prologue_bf16(const StepLists& L, const bf16_t* emb, int d, const bf16_t* gain,
                               float* h, bf16_t* a_out, unsigned long long* sumsq, int nbuf,
                               int sumsq_stride, hipStream_t s);
// Re-tiles W[N,K] (row-major) into fragment order inside a packed matrix whose tiles are
// grouped by `grp`.  mode picks the destination row of each source row (row0 = first destination
// row of this source matrix): plain; rotary halves (a head's tile t holds its columns 8t..8t+7
// in rows 0-7 and their rotary partners hd/2 later in rows 8-15); or rows 0-7 / 8-15 of every
// tile of a two-matrix interleave (gate / up).
void launch_repack_weight(const bf16_t* W, int N, int K, bf16_t* Wp, int mode, int hd, int grp,
                          int row0, hipStream_t s);
// Weight tiles per block the skinny GEMM uses for a matrix of total_nt tiles, which is also the
// group size its packed layout should have.
int skinny_tiles_per_block(int epi, int total_nt);
// Up to this many activation rows the LM head runs through the skinny kernel, which reduces the
// vocabulary on the fly: lm_head_parts(V) partial tuples per row.
constexpr int kLmSkinnyRows = 64;
int lm_head_parts(int V);
// dst rows 0..n (padded with zero rows to whole tiles) = src rows sel[0..n), both packed, K wide.
void launch_gather_rows_packed(const bf16_t* src, int M_src, const int* sel, int n, int K,
                               bf16_t* dst, hipStream_t s);
void launch_unpack_cache(const bf16_t* packed, int is_v, int T, int Tpad, int Hkv, int hd,
                         bf16_t* out, hipStream_t s);
// A: packed activations holding M_src rows; W: packed [N/16 tiles][K/32]; see GemmEpi.
// Wq: nullable, the same matrix as packed e4m3 codes (then e.wscale holds its row scales): the
// weight-streaming kernels (few rows) read it instead of Wp.
void launch_gemm_bf16(int epi, const bf16_t* Ap, int M_src, const bf16_t* Wp, const void* Wq,
                      int N, int K, const GemmEpi& e, hipStream_t s);
// e4m3 source: Wq receives the codes as 1 KiB fragment pairs (64 k per weight tile and step),
// Wp the same values as bf16 fragments (exact); either may be NULL.  mode / hd / grp / row0 as
// launch_repack_weight.
void launch_repack_weight_e4m3(const uint8_t* W, int N, int K, uint8_t* Wq, bf16_t* Wp, int mode,
                               int hd, int grp, int row0, hipStream_t s);
// dst[row0 + packed row of n] = src[n]: a per-row vector in the packed matrix' row order
void launch_repack_rows_f32(const float* src, int N, float* dst, int mode, int hd, int row0,
                            hipStream_t s);
// q row-major [M, Hq*hd]; packed caches of one layer; out packed bf16 (K = Hq*hd).
// part / tickets: scratch for splitting the keys over blocks when there are few query rows
// (part_floats floats; 256 counters, zero on entry and again on exit); null = never split.
// R rows (rowinfo / tileinfo as the step prologue wrote them), kc / vc: one layer's planes.
// Sequences with at most kSmallRows rows are served through `pairs`: npairs entries (row tile,
// cache offset, positions, keys per slab), one for every sequence a row tile holds rows of.
// pairs (and tileinfo) may be NULL when the step has a single sequence: then one_seq (cache
// offset, positions, keys per slab, many-rows flag) describes every tile.  has_small /
// has_large: whether any sequence of the step has at most / more than kSmallRows rows; max_T:
// most positions of any few-row sequence taking part.
void launch_attention_mfma(const bf16_t* q, const bf16_t* kc, const bf16_t* vc, int R,
                           const int4* rowinfo, const int4* tileinfo, const int4* pairs,
                           int npairs, const int4* seqtab, int nsmall, int max_visits,
                           int4 one_seq, bool has_small, bool has_large, int max_T,
                           int Hq, int Hkv, int hd, bf16_t* out, float* part, size_t part_floats,
                           int* tickets, hipStream_t s);

// decision
int vocab_reduce_parts(int V);
// logits [n_rows, V] with row stride ld -> partials [n_rows][vocab_reduce_parts(V)]
void launch_vocab_reduce(const float* logits, int n_rows, int V, size_t ld, float4* partials,
                         hipStream_t s);
// partials -> stats [n_rows] (token id as float, confidence, entropy, max logit)
void launch_row_stats(const float4* partials, int nparts, int n_rows, float4* stats, hipStream_t s);
void launch_decide(const DecideArgs& a, int B, hipStream_t s);
void launch_init_state(int* x, uint8_t* masked, int* hist, DevState* st, const int* prompt_dev,
                       int P, int N, int mask_id, hipStream_t s);

}  // namespace ec
