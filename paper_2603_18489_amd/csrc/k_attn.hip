// Non-causal attention of the recomputed rows against the whole cached context
// ("TransformerBlock(Q_[M u R], K_[I], V_[I])" of the appendix algorithm): every query row
// attends all T cached positions, no mask.
//
// Generic kernel for the float32 path (row-major cache): one block per (query row, head).
// Scores for all T keys are kept in LDS, softmax statistics in fp32, then P.V with the block
// split over hd columns.  The bf16 path uses the MFMA kernel of k_attn_mfma.hip.
#include "ec_internal.h"

namespace ec {

template <typename TA, int HD, bool PACKED>
__global__ __launch_bounds__(256) void attn_generic_kernel(const TA* __restrict__ q,
                                                           const TA* __restrict__ kc,
                                                           const TA* __restrict__ vc, int M, int T,
                                                           int Hq, int Hkv, float scale,
                                                           void* __restrict__ outv, int MT) {
  extern __shared__ float smem[];
  float* scores = smem;             // [T]
  float* qs = smem + T;             // [HD]
  float* part = qs + HD;            // [256]
  __shared__ float red[4];
  const int r = blockIdx.x, a = blockIdx.y, tid = threadIdx.x;
  const int nq = Hq * HD, nkv = Hkv * HD;
  if (r >= M) {  // padding rows of the packed layout
    if constexpr (PACKED) {
      if (tid < HD) ((bf16_t*)outv)[packed_act_index(r, a * HD + tid, MT)] = 0;
    }
    return;
  }
  const int kvh = a / (Hq / Hkv);
  if (tid < HD) qs[tid] = load_f32<TA>(q + (size_t)r * nq + a * HD + tid);
  __syncthreads();
  float lmax = -INFINITY;
  for (int j = tid; j < T; j += 256) {
    const TA* kr = kc + (size_t)j * nkv + kvh * HD;
    float dot = 0.f;
#pragma unroll 8
    for (int c = 0; c < HD; ++c) dot = fmaf(qs[c], load_f32<TA>(kr + c), dot);
    dot *= scale;
    scores[j] = dot;
    lmax = fmaxf(lmax, dot);
  }
  float mx = block_max<4>(lmax, red);
  float lsum = 0.f;
  for (int j = tid; j < T; j += 256) {
    float p = expf(scores[j] - mx);
    scores[j] = p;
    lsum += p;
  }
  float denom = block_sum<4>(lsum, red);  // also orders the score writes before the reads below
  constexpr int NP = 256 / HD;            // key partitions
  const int col = tid % HD, pp = tid / HD;
  float acc = 0.f;
  for (int j = pp; j < T; j += NP)
    acc = fmaf(scores[j], load_f32<TA>(vc + (size_t)j * nkv + kvh * HD + col), acc);
  part[tid] = acc;
  __syncthreads();
  if (tid < HD) {
    float o = 0.f;
#pragma unroll
    for (int i = 0; i < NP; ++i) o += part[i * HD + tid];
    o /= denom;
    if constexpr (PACKED)
      ((bf16_t*)outv)[packed_act_index(r, a * HD + tid, MT)] = f32_to_bf16(o);
    else
      ((float*)outv)[(size_t)r * nq + a * HD + tid] = o;
  }
}

template <typename TA, bool PACKED>
static void launch_attn_t(const void* q, const void* kc, const void* vc, int M, int T, int Hq,
                          int Hkv, int hd, void* out, hipStream_t s) {
  int MT = (M + 15) / 16;
  int rows = PACKED ? MT * 16 : M;
  dim3 grid(rows, Hq);
  size_t smem = (size_t)(T + hd + 256) * sizeof(float);
  float scale = 1.0f / sqrtf((float)hd);
  if (hd == 64)
    attn_generic_kernel<TA, 64, PACKED><<<grid, 256, smem, s>>>(
        (const TA*)q, (const TA*)kc, (const TA*)vc, M, T, Hq, Hkv, scale, out, MT);
  else
    attn_generic_kernel<TA, 128, PACKED><<<grid, 256, smem, s>>>(
        (const TA*)q, (const TA*)kc, (const TA*)vc, M, T, Hq, Hkv, scale, out, MT);
}

void launch_attention_mfma(const bf16_t* q, const bf16_t* kc, const bf16_t* vc, int M, int T,
                           int Tpad, int Hq, int Hkv, int hd, bf16_t* out, hipStream_t s);

void launch_attention(int dtype, const void* q, const void* kc, const void* vc, int M, int T,
                      int Tpad, int Hq, int Hkv, int hd, void* out, hipStream_t s) {
  if (M <= 0) return;
  if (dtype == EC_F32)
    launch_attn_t<float, false>(q, kc, vc, M, T, Hq, Hkv, hd, out, s);
  else
    launch_attention_mfma((const bf16_t*)q, (const bf16_t*)kc, (const bf16_t*)vc, M, T, Tpad, Hq,
                          Hkv, hd, (bf16_t*)out, s);
}

}  // namespace ec
