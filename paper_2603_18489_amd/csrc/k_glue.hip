// Small memory-bound kernels around the GEMMs: embedding gather, RMSNorm, RoPE + KV-cache
// scatter, SwiGLU, and the one-time re-tiling of bf16 matrices.
#include "ec_internal.h"

namespace ec {

// ---------------------------------------------------------------------------------------------
// Embedding gather: h[r,:] = Emb[x[pos(r)],:]   (H^{t,0} of the appendix algorithm)
// ---------------------------------------------------------------------------------------------
template <typename TW>
__global__ __launch_bounds__(256) void embed_kernel(const TW* __restrict__ emb,
                                                    const int* __restrict__ x,
                                                    const int* __restrict__ rows, int d,
                                                    float* __restrict__ h) {
  int r = blockIdx.x;
  int pos = rows ? rows[r] : r;
  const TW* src = emb + (size_t)x[pos] * d;
  float* dst = h + (size_t)r * d;
  for (int c = threadIdx.x; c < d; c += 256) dst[c] = load_f32<TW>(src + c);
}

void launch_embed(int dtype, const void* emb, const int* x, const int* rows, int M, int d,
                  float* h, hipStream_t s) {
  if (M <= 0) return;
  if (dtype == EC_F32)
    embed_kernel<float><<<M, 256, 0, s>>>((const float*)emb, x, rows, d, h);
  else
    embed_kernel<bf16_t><<<M, 256, 0, s>>>((const bf16_t*)emb, x, rows, d, h);
}

// ---------------------------------------------------------------------------------------------
// RMSNorm: u = h * rsqrt(mean(h^2) + eps) * g, statistics in fp32.
// f32: row-major output.  bf16: packed activation layout; rows M..MT*16-1 are written as zeros.
// ---------------------------------------------------------------------------------------------
template <typename TW, bool PACKED>
__global__ __launch_bounds__(256) void rmsnorm_kernel(const float* __restrict__ h,
                                                      const int* __restrict__ sel, int M, int d,
                                                      const TW* __restrict__ gain, float eps,
                                                      void* __restrict__ outv, int MT) {
  __shared__ float red[4];
  int r = blockIdx.x;
  if (r >= M) {  // padding rows of the packed layout
    if constexpr (PACKED) {
      bf16_t* out = (bf16_t*)outv;
      for (int c8 = threadIdx.x * 8; c8 < d; c8 += 256 * 8) {
        uint4 z = {0, 0, 0, 0};
        *(uint4*)(out + packed_act_index(r, c8, MT)) = z;
      }
    }
    return;
  }
  const float* src = h + (size_t)(sel ? sel[r] : r) * d;
  float ss = 0.f;
  for (int c = threadIdx.x; c < d; c += 256) {
    float v = src[c];
    ss += v * v;
  }
  ss = block_sum<4>(ss, red);
  float rstd = 1.0f / sqrtf(ss / (float)d + eps);
  if constexpr (PACKED) {
    bf16_t* out = (bf16_t*)outv;
    for (int c8 = threadIdx.x * 8; c8 < d; c8 += 256 * 8) {
      union { uint4 v; bf16_t e[8]; } pk;
#pragma unroll
      for (int i = 0; i < 8; ++i)
        pk.e[i] = f32_to_bf16(src[c8 + i] * rstd * load_f32<TW>(gain + c8 + i));
      *(uint4*)(out + packed_act_index(r, c8, MT)) = pk.v;
    }
  } else {
    float* out = (float*)outv + (size_t)r * d;
    for (int c = threadIdx.x; c < d; c += 256) out[c] = src[c] * rstd * load_f32<TW>(gain + c);
  }
}

void launch_rmsnorm(int dtype, const float* h, const int* sel, int M, int d, const void* gain,
                    float eps, void* out, hipStream_t s) {
  if (M <= 0) return;
  if (dtype == EC_F32) {
    rmsnorm_kernel<float, false><<<M, 256, 0, s>>>(h, sel, M, d, (const float*)gain, eps, out, 0);
  } else {
    int MT = (M + 15) / 16;
    rmsnorm_kernel<bf16_t, true><<<MT * 16, 256, 0, s>>>(h, sel, M, d, (const bf16_t*)gain, eps,
                                                         out, MT);
  }
}

// ---------------------------------------------------------------------------------------------
// RoPE table: cs[pos][j] = (cos, sin)(pos * base^(-2j/hd)), evaluated in double once per context.
// ---------------------------------------------------------------------------------------------
__global__ void rope_table_kernel(float2* __restrict__ cs, int T, int half, int hd, double base) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= T * half) return;
  int pos = i / half, j = i % half;
  double inv = pow(base, -2.0 * (double)j / (double)hd);
  double a = (double)pos * inv;
  cs[i] = make_float2((float)cos(a), (float)sin(a));
}

void launch_rope_table(float2* cs, int T, int hd, float base, hipStream_t s) {
  int n = T * (hd / 2);
  rope_table_kernel<<<(n + 255) / 256, 256, 0, s>>>(cs, T, hd / 2, hd, (double)base);
}

// ---------------------------------------------------------------------------------------------
// RoPE + KV scatter: from the projected row [q | k | v] (fp32) rotate q and k by the row's
// absolute position, write q to the query buffer and k, v into the layer's cache row `pos`.
// The cache holds post-RoPE keys.  One block per row; one full cache row per (row, K/V).
// ---------------------------------------------------------------------------------------------
template <typename TA, bool PACKED>
__global__ __launch_bounds__(256) void rope_scatter_kernel(const float* __restrict__ qkv,
                                                           const int* __restrict__ rows, int Hq,
                                                           int Hkv, int hd,
                                                           const float2* __restrict__ cs,
                                                           TA* __restrict__ q_out,
                                                           TA* __restrict__ kcache,
                                                           TA* __restrict__ vcache, int Tpad) {
  int r = blockIdx.x;
  int pos = rows ? rows[r] : r;
  int half = hd / 2;
  int nq = Hq * hd, nkv = Hkv * hd;
  const float* row = qkv + (size_t)r * (nq + 2 * nkv);
  const float2* csr = cs + (size_t)pos * half;
  for (int idx = threadIdx.x; idx < (Hq + Hkv) * half; idx += 256) {
    int head = idx / half, j = idx - head * half;
    float a = row[head * hd + j], b = row[head * hd + j + half];
    float2 c = csr[j];
    float ra = a * c.x - b * c.y, rb = b * c.x + a * c.y;
    if (head < Hq) {
      TA* dst = q_out + (size_t)r * nq + head * hd + j;
      store_f32<TA>(dst, ra);
      store_f32<TA>(dst + half, rb);
    } else if constexpr (PACKED) {
      TA* slab = kcache + (size_t)(head - Hq) * Tpad * hd;
      store_f32<TA>(slab + kcache_index(pos, j, hd), ra);
      store_f32<TA>(slab + kcache_index(pos, j + half, hd), rb);
    } else {
      TA* dst = kcache + (size_t)pos * nkv + (head - Hq) * hd + j;
      store_f32<TA>(dst, ra);
      store_f32<TA>(dst + half, rb);
    }
  }
  const float* vrow = row + nq + nkv;
  if constexpr (PACKED) {
    for (int c = threadIdx.x; c < nkv; c += 256) {
      int kvh = c / hd, cc = c - kvh * hd;
      store_f32<TA>(vcache + (size_t)kvh * Tpad * hd + vcache_index(pos, cc, Tpad), vrow[c]);
    }
  } else {
    TA* vdst = vcache + (size_t)pos * nkv;
    for (int c = threadIdx.x; c < nkv; c += 256) store_f32<TA>(vdst + c, vrow[c]);
  }
}

__global__ __launch_bounds__(256) void unpack_cache_kernel(const bf16_t* __restrict__ packed,
                                                           int is_v, int T, int Tpad, int Hkv,
                                                           int hd, bf16_t* __restrict__ out) {
  int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= T * Hkv * hd) return;
  int key = i / (Hkv * hd), c = i - key * (Hkv * hd), kvh = c / hd, cc = c - kvh * hd;
  const bf16_t* slab = packed + (size_t)kvh * Tpad * hd;
  out[i] = is_v ? slab[vcache_index(key, cc, Tpad)] : slab[kcache_index(key, cc, hd)];
}

void launch_unpack_cache(const bf16_t* packed, int is_v, int T, int Tpad, int Hkv, int hd,
                         bf16_t* out, hipStream_t s) {
  int n = T * Hkv * hd;
  unpack_cache_kernel<<<(n + 255) / 256, 256, 0, s>>>(packed, is_v, T, Tpad, Hkv, hd, out);
}

void launch_rope_scatter(int dtype, const float* qkv, const int* rows, int M, int Hq, int Hkv,
                         int hd, const float2* cs, void* q_out, void* kcache, void* vcache,
                         int Tpad, hipStream_t s) {
  if (M <= 0) return;
  if (dtype == EC_F32)
    rope_scatter_kernel<float, false><<<M, 256, 0, s>>>(qkv, rows, Hq, Hkv, hd, cs, (float*)q_out,
                                                        (float*)kcache, (float*)vcache, Tpad);
  else
    rope_scatter_kernel<bf16_t, true><<<M, 256, 0, s>>>(qkv, rows, Hq, Hkv, hd, cs,
                                                        (bf16_t*)q_out, (bf16_t*)kcache,
                                                        (bf16_t*)vcache, Tpad);
}

// ---------------------------------------------------------------------------------------------
// SwiGLU: act = silu(gate) * up with gu = [gate | up] (fp32, [M, 2F]).
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ float silu_f(float x) { return x / (1.0f + expf(-x)); }

template <bool PACKED>
__global__ __launch_bounds__(256) void swiglu_kernel(const float* __restrict__ gu, int M, int F,
                                                     void* __restrict__ outv, int MT) {
  int r = blockIdx.y;
  int c8 = (blockIdx.x * 256 + threadIdx.x) * 8;
  if (c8 >= F) return;
  if constexpr (PACKED) {
    bf16_t* out = (bf16_t*)outv;
    union { uint4 v; bf16_t e[8]; } pk;
    if (r < M) {
      const float* g = gu + (size_t)r * 2 * F + c8;
#pragma unroll
      for (int i = 0; i < 8; ++i) pk.e[i] = f32_to_bf16(silu_f(g[i]) * g[F + i]);
    } else {
      pk.v = make_uint4(0, 0, 0, 0);
    }
    *(uint4*)(out + packed_act_index(r, c8, MT)) = pk.v;
  } else {
    if (r >= M) return;
    const float* g = gu + (size_t)r * 2 * F + c8;
    float* out = (float*)outv + (size_t)r * F + c8;
#pragma unroll
    for (int i = 0; i < 8; ++i)
      if (c8 + i < F) out[i] = silu_f(g[i]) * g[F + i];
  }
}

void launch_swiglu(int dtype, const float* gu, int M, int F, void* act, hipStream_t s) {
  if (M <= 0) return;
  int gx = (F + 2047) / 2048;
  if (dtype == EC_F32) {
    swiglu_kernel<false><<<dim3(gx, M), 256, 0, s>>>(gu, M, F, act, 0);
  } else {
    int MT = (M + 15) / 16;
    swiglu_kernel<true><<<dim3(gx, MT * 16), 256, 0, s>>>(gu, M, F, act, MT);
  }
}

// ---------------------------------------------------------------------------------------------
// One-time re-tiling of a bf16 matrix W[N,K] into 16x32 MFMA fragments (see k_common.h).
// A pure permutation.  One thread moves 8 consecutive k (16 bytes).
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void repack_weight_kernel(const bf16_t* __restrict__ W, int N,
                                                            int K, bf16_t* __restrict__ Wp) {
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;  // over N * K/8 groups of 8
  size_t total = (size_t)N * (K / 8);
  if (i >= total) return;
  int n = (int)(i / (K / 8));
  int k = (int)(i % (K / 8)) * 8;
  uint4 v = *(const uint4*)(W + (size_t)n * K + k);
  *(uint4*)(Wp + packed_w_index(n, k, K / 32)) = v;
}

void launch_repack_weight(const bf16_t* W, int N, int K, bf16_t* Wp, hipStream_t s) {
  size_t total = (size_t)N * (K / 8);
  repack_weight_kernel<<<(unsigned)((total + 255) / 256), 256, 0, s>>>(W, N, K, Wp);
}

}  // namespace ec
