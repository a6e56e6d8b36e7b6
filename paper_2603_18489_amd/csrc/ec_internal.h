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

// What the decision kernel hands back to the host after each step.
struct StepOut {
  ec_step_result r;
  int next_n_mb;
  int next_n_rows_partial;
  int pad[6];
};

struct DecideArgs {
  // this step
  const float4* partials;  // [n_mb][nparts] (max, argmax as float bits, sum e, sum e*(z-max))
  int nparts;
  int n_mb;
  int mode_run;
  int n_rows_run;
  int forced_n;            // -1: commit the step's own choice
  const int* forced_pos;   // device
  const int* forced_tok;   // device
  int init_only;           // 1: no decode, only build the lists of the first step
  // sequence state
  int* x;                  // [T]
  uint8_t* masked;         // [T]
  int* hist;               // [N], INT32_MIN = never decoded
  DevState* st;
  int* mb_pos;             // [block] positions of the block's masked rows, ascending
  int* rows_partial;       // [T] ascending positions of M u R
  int* mb_idx;             // [block] index of each block row inside rows_partial
  float* row_stats;        // [block][4] token, confidence, entropy, max logit
  StepOut* out;
  // configuration
  int P, N, T, block, k_recent, n_tok;
  float tau;
};

// ---- launchers (each enqueues on `s`; shapes are validated by the caller) --------------------
void launch_embed(int dtype, const void* emb, const int* x, const int* rows, int M, int d,
                  float* h, hipStream_t s);
// out: row-major float [M,d] (dtype f32) or packed bf16 activations with MT = ceil(M/16).
// sel (nullable) gathers source rows: out row r comes from h row sel[r].
void launch_rmsnorm(int dtype, const float* h, const int* sel, int M, int d, const void* gain,
                    float eps, void* out, hipStream_t s);
void launch_rope_table(float2* cs, int T, int hd, float base, hipStream_t s);
// f32: caches are row-major [T, Hkv*hd].  bf16: packed per kv head (k_common.h), Tpad keys.
void launch_rope_scatter(int dtype, const float* qkv, const int* rows, int M, int Hq, int Hkv,
                         int hd, const float2* cs, void* q_out, void* kcache, void* vcache,
                         int Tpad, hipStream_t s);
// bf16 only: packed cache of one layer -> row-major [T, Hkv*hd] (debug read-back).
void launch_unpack_cache(const bf16_t* packed, int is_v, int T, int Tpad, int Hkv, int hd,
                         bf16_t* out, hipStream_t s);
void launch_swiglu(int dtype, const float* gu, int M, int F, void* act, hipStream_t s);
void launch_repack_weight(const bf16_t* W, int N, int K, bf16_t* Wp, hipStream_t s);

// C[M,N] (ldc) = scale * A[M,K] W[N,K]^T, or C += ... when accumulate.
void launch_gemm_f32(const float* A, const float* W, float* C, int ldc, int M, int N, int K,
                     int accumulate, float scale, hipStream_t s);
// bf16: A packed activations (M rows), up to 3 packed weight segments laid side by side along N.
struct GemmSegs {
  const bf16_t* w[3];
  int ntiles[3];  // 16-row tiles per segment
  int nseg;
};
void launch_gemm_bf16(const bf16_t* Ap, int M, const GemmSegs& segs, int K, float* C, int ldc,
                      int accumulate, float scale, hipStream_t s);

// Non-causal attention of M query rows against all T cached positions.
// q row-major [M, Hq*hd]; caches [T, Hkv*hd]; out row-major float (f32) or packed bf16.
void launch_attention(int dtype, const void* q, const void* kc, const void* vc, int M, int T,
                      int Tpad, int Hq, int Hkv, int hd, void* out, hipStream_t s);

int vocab_reduce_parts(int V);
void launch_vocab_reduce(const float* logits, int n_rows, int V, float4* partials, hipStream_t s);
void launch_decide(const DecideArgs& a, hipStream_t s);
void launch_init_state(int* x, uint8_t* masked, int* hist, DevState* st, const int* prompt_dev,
                       int P, int N, int mask_id, hipStream_t s);

}  // namespace ec
