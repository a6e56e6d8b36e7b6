// Non-causal attention of the recomputed rows against the whole cached context
// ("TransformerBlock(Q_[M u R], K_[I], V_[I])" of the appendix algorithm): every query row
// attends all T cached positions, no mask.
//
// Float32 path (row-major cache): one block per (query row, head).  Scores for all T keys are
// kept in LDS, softmax statistics in fp32, then P.V with the block split over hd columns.
// The bf16 path uses the MFMA kernel of k_attn_mfma.hip.
#include "ec_internal.h"

namespace ec {

template <int HD>
__global__ __launch_bounds__(256) void attn_f32_kernel(const float* __restrict__ q,
                                                       const float* __restrict__ kc,
                                                       const float* __restrict__ vc, int T, int Hq,
                                                       int Hkv, float scale,
                                                       float* __restrict__ out) {
  extern __shared__ float smem[];
  float* scores = smem;             // [T]
  float* qs = smem + T;             // [HD]
  float* part = qs + HD;            // [256]
  __shared__ float red[4];
  const int r = blockIdx.x, a = blockIdx.y, tid = threadIdx.x;
  const int nq = Hq * HD, nkv = Hkv * HD;
  const int kvh = a / (Hq / Hkv);
  if (tid < HD) qs[tid] = q[(size_t)r * nq + a * HD + tid];
  __syncthreads();
  float lmax = -INFINITY;
  for (int j = tid; j < T; j += 256) {
    const float* kr = kc + (size_t)j * nkv + kvh * HD;
    float dot = 0.f;
#pragma unroll 8
    for (int c = 0; c < HD; ++c) dot = fmaf(qs[c], kr[c], dot);
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
    acc = fmaf(scores[j], vc[(size_t)j * nkv + kvh * HD + col], acc);
  part[tid] = acc;
  __syncthreads();
  if (tid < HD) {
    float o = 0.f;
#pragma unroll
    for (int i = 0; i < NP; ++i) o += part[i * HD + tid];
    out[(size_t)r * nq + a * HD + tid] = o / denom;
  }
}

void launch_attention_f32(const float* q, const float* kc, const float* vc, int M, int T, int Hq,
                          int Hkv, int hd, float* out, hipStream_t s) {
  if (M <= 0) return;
  dim3 grid(M, Hq);
  size_t smem = (size_t)(T + hd + 256) * sizeof(float);
  float scale = 1.0f / sqrtf((float)hd);
  if (hd == 64)
    attn_f32_kernel<64><<<grid, 256, smem, s>>>(q, kc, vc, T, Hq, Hkv, scale, out);
  else
    attn_f32_kernel<128><<<grid, 256, smem, s>>>(q, kc, vc, T, Hq, Hkv, scale, out);
}

}  // namespace ec
