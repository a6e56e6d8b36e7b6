// Small memory-bound kernels around the GEMMs.
//  float32 path: embedding gather, RMSNorm, RoPE + KV-cache scatter, SwiGLU (row-major tensors).
//  bf16 path:    the step prologue (row list, embedding gather fused with the first norm's
//                operand), the one-time re-tiling of the matrices, and the un-tiling of a cache
//                layer for debug read-back.  Everything else of that path lives in the GEMM
//                epilogues.
#include "ec_internal.h"

namespace ec {

// ---------------------------------------------------------------------------------------------
// Embedding gather: h[r,:] = Emb[x[pos(r)],:]   (H^{t,0} of the appendix algorithm)
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void embed_f32_kernel(const float* __restrict__ emb,
                                                        const int* __restrict__ x,
                                                        const int* __restrict__ rows, int d,
                                                        int vocab, float* __restrict__ h) {
  int r = blockIdx.x;
  int pos = rows ? rows[r] : r;
  int tok = x[pos];
  if ((unsigned)tok >= (unsigned)vocab) tok = 0;  // (never index the table with a non-token)
  const float* src = emb + (size_t)tok * d;
  float* dst = h + (size_t)r * d;
  for (int c = threadIdx.x; c < d; c += 256) dst[c] = src[c];
}

void launch_embed_f32(const float* emb, const int* x, const int* rows, int M, int d, int vocab,
                      float* h, hipStream_t s) {
  if (M <= 0) return;
  embed_f32_kernel<<<M, 256, 0, s>>>(emb, x, rows, d, vocab, h);
}

// bf16: the step's first kernel, one block per row of the step's row list.  It derives the
// row's sequence and position from the sequence table (and records them for the later kernels),
// gathers the embedding, emits the first GEMM's operand bf16(h * gain) in fragment order and the
// row's sum of squares (44.20 fixed point), and clears the step's other sum buffers for the row.
__global__ __launch_bounds__(256) void step_prologue_bf16_kernel(
    StepLists L, const bf16_t* __restrict__ emb, int d, const bf16_t* __restrict__ gain,
    float* __restrict__ h, bf16_t* __restrict__ a_out, unsigned long long* __restrict__ sumsq,
    int nbuf, int sumsq_stride, int MT) {
  __shared__ float red[4];
  __shared__ int sh_xidx;
  const int r = blockIdx.x;
  if (threadIdx.x == 0) {
    int4 ri = make_int4(-1, -1, 0, 32);
    int4 ti = make_int4(0, 0, 32, 0);
    for (int b = 0; b < L.B; ++b) {
      const SeqDesc sd = L.seqs ? L.seqs[b] : L.seq0;
      if (sd.mode < 0 || r < sd.row0 || r >= sd.row0 + sd.seg_rows) continue;
      const int i = r - sd.row0;
      int pos = -1;
      if (i < sd.n_rows) pos = sd.mode == EC_FULL ? i : L.rows_partial[sd.x_off + i];
      ri = make_int4(pos, pos >= 0 ? sd.x_off + pos : -1, sd.kv_off, sd.tpad);
      ti = make_int4(sd.kv_off, sd.T, sd.tpad, sd.n_rows > kSmallRows ? 1 : 0);
    }
    L.rowinfo[r] = ri;
    if ((r & 15) == 0) L.tileinfo[r >> 4] = ti;
    sh_xidx = ri.y;
    if (r < L.n_lm) {
      for (int b = 0; b < L.B; ++b) {
        const SeqDesc sd = L.seqs ? L.seqs[b] : L.seq0;
        if (sd.mode < 0 || r < sd.lm0 || r >= sd.lm0 + sd.n_mb) continue;
        const int i = b * L.block + (r - sd.lm0);
        L.lm_sel[r] = sd.row0 + (sd.mode == EC_FULL ? L.mb_pos[i] : L.mb_idx[i]);
      }
    }
  }
  __syncthreads();
  const int xidx = sh_xidx;
  int tok = xidx >= 0 ? L.x[xidx] : 0;
  if ((unsigned)tok >= (unsigned)L.vocab) tok = 0;  // (never index the table with a non-token)
  const bf16_t* src = emb + (size_t)tok * d;
  float* dst = h + (size_t)r * d;
  float ss = 0.f;
  for (int c8 = threadIdx.x * 8; c8 < d; c8 += 256 * 8) {
    union { uint4 v; bf16_t e[8]; } in, out;
    in.v = xidx >= 0 ? *(const uint4*)(src + c8) : make_uint4(0, 0, 0, 0);
    float f[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      f[i] = bf16_to_f32(in.e[i]);
      ss += f[i] * f[i];
      out.e[i] = f32_to_bf16(f[i] * bf16_to_f32(gain[c8 + i]));
    }
    *(float4*)(dst + c8) = make_float4(f[0], f[1], f[2], f[3]);
    *(float4*)(dst + c8 + 4) = make_float4(f[4], f[5], f[6], f[7]);
    *(uint4*)(a_out + packed_act_index(r, c8, MT)) = out.v;
  }
  ss = block_sum<4>(ss, red);
  if (threadIdx.x == 0)
    sumsq[r] = sumsq_to_fixed<62>(ss);
  for (int b = 1 + threadIdx.x; b < nbuf; b += 256) sumsq[(size_t)b * sumsq_stride + r] = 0ull;
}

void launch_step_prologue_bf16(const StepLists& L, const bf16_t* emb, int d, const bf16_t* gain,
                               float* h, bf16_t* a_out, unsigned long long* sumsq, int nbuf,
                               int sumsq_stride, hipStream_t s) {
  if (L.R <= 0) return;
  step_prologue_bf16_kernel<<<L.R, 256, 0, s>>>(L, emb, d, gain, h, a_out, sumsq, nbuf,
                                                sumsq_stride, (L.R + 15) / 16);
}

// ---------------------------------------------------------------------------------------------
// RMSNorm (float32 path): u = h * rsqrt(mean(h^2) + eps) * g
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void rmsnorm_f32_kernel(const float* __restrict__ h,
                                                          const int* __restrict__ sel, int d,
                                                          const float* __restrict__ gain,
                                                          float eps, float* __restrict__ outp) {
  __shared__ float red[4];
  int r = blockIdx.x;
  const float* src = h + (size_t)(sel ? sel[r] : r) * d;
  float ss = 0.f;
  for (int c = threadIdx.x; c < d; c += 256) {
    float v = src[c];
    ss += v * v;
  }
  ss = block_sum<4>(ss, red);
  float rstd = 1.0f / sqrtf(ss / (float)d + eps);
  float* out = outp + (size_t)r * d;
  for (int c = threadIdx.x; c < d; c += 256) out[c] = src[c] * rstd * gain[c];
}

void launch_rmsnorm_f32(const float* h, const int* sel, int M, int d, const float* gain, float eps,
                        float* out, hipStream_t s) {
  if (M <= 0) return;
  rmsnorm_f32_kernel<<<M, 256, 0, s>>>(h, sel, d, gain, eps, out);
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
// RoPE + KV scatter (float32 path): from the projected row [q | k | v] rotate q and k by the
// row's absolute position, write q to the query buffer and k, v into the cache row `pos`.
// The cache holds post-RoPE keys.  One block per row; one full cache row per (row, K/V).
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void rope_scatter_f32_kernel(
    const float* __restrict__ qkv, const int* __restrict__ rows, int Hq, int Hkv, int hd,
    const float2* __restrict__ cs, float* __restrict__ q_out, float* __restrict__ kcache,
    float* __restrict__ vcache) {
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
    float* dst = head < Hq ? q_out + (size_t)r * nq + head * hd + j
                           : kcache + (size_t)pos * nkv + (head - Hq) * hd + j;
    dst[0] = ra;
    dst[half] = rb;
  }
  const float* vrow = row + nq + nkv;
  float* vdst = vcache + (size_t)pos * nkv;
  for (int c = threadIdx.x; c < nkv; c += 256) vdst[c] = vrow[c];
}

void launch_rope_scatter_f32(const float* qkv, const int* rows, int M, int Hq, int Hkv, int hd,
                             const float2* cs, float* q_out, float* kcache, float* vcache,
                             hipStream_t s) {
  if (M <= 0) return;
  rope_scatter_f32_kernel<<<M, 256, 0, s>>>(qkv, rows, Hq, Hkv, hd, cs, q_out, kcache, vcache);
}

// ---------------------------------------------------------------------------------------------
// SwiGLU (float32 path): act = silu(gate) * up with gu = [gate | up] ([M, 2F]).
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void swiglu_f32_kernel(const float* __restrict__ gu, int F,
                                                         float* __restrict__ act) {
  int r = blockIdx.y;
  int c = blockIdx.x * 256 + threadIdx.x;
  if (c >= F) return;
  float g = gu[(size_t)r * 2 * F + c], u = gu[(size_t)r * 2 * F + F + c];
  act[(size_t)r * F + c] = g / (1.0f + expf(-g)) * u;
}

void launch_swiglu_f32(const float* gu, int M, int F, float* act, hipStream_t s) {
  if (M <= 0) return;
  swiglu_f32_kernel<<<dim3((F + 255) / 256, M), 256, 0, s>>>(gu, F, act);
}

// ---------------------------------------------------------------------------------------------
// One-time re-tiling of a bf16 matrix W[N,K] into 16x32 MFMA fragments (k_common.h).  A pure
// permutation; one thread moves 8 consecutive k (16 bytes).  Destination row of source row n
// (before adding row0):
//   REPACK_PLAIN        n
//   REPACK_ROPE_HALVES  within each head of hd rows: row c < hd/2 goes to tile c/8, row c%8; its
//                       rotary partner c + hd/2 to row 8 + c%8 of the same tile
//   REPACK_LO8 / HI8    (n/8)*16 + n%8  /  (n/8)*16 + 8 + n%8  (two matrices, 8 rows each per tile)
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ int repack_row(int n, int mode, int hd);

__global__ __launch_bounds__(256) void repack_weight_kernel(const bf16_t* __restrict__ W, int N,
                                                            int K, bf16_t* __restrict__ Wp,
                                                            int mode, int hd, int grp, int row0) {
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;  // over N * K/8 groups of 8
  size_t total = (size_t)N * (K / 8);
  if (i >= total) return;
  int n = (int)(i / (K / 8));
  int k = (int)(i % (K / 8)) * 8;
  const int dn = repack_row(n, mode, hd);
  uint4 v = *(const uint4*)(W + (size_t)n * K + k);
  *(uint4*)(Wp + packed_w_index(row0 + dn, k, K / 32, grp)) = v;
}

// destination row (before row0) of source row n under a re-tiling mode
__device__ __forceinline__ int repack_row(int n, int mode, int hd) {
  if (mode == REPACK_ROPE_HALVES) {
    int head = n / hd, c = n - head * hd, half = hd >> 1;
    int cc = c < half ? c : c - half;
    return head * hd + (cc >> 3) * 16 + (c < half ? 0 : 8) + (cc & 7);
  }
  if (mode == REPACK_LO8) return (n >> 3) * 16 + (n & 7);
  if (mode == REPACK_HI8) return (n >> 3) * 16 + 8 + (n & 7);
  return n;
}

// The same re-tiling from e4m3 codes: 8 consecutive k per thread go to the fragment pairs as they
// are (8 bytes) and, widened exactly to bf16, to the bf16 fragments (16 bytes).
__global__ __launch_bounds__(256) void repack_weight_e4m3_kernel(
    const uint8_t* __restrict__ W, int N, int K, uint8_t* __restrict__ Wq, bf16_t* __restrict__ Wp,
    int mode, int hd, int grp, int row0) {
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;  // over N * K/8 groups of 8
  size_t total = (size_t)N * (K / 8);
  if (i >= total) return;
  int n = (int)(i / (K / 8));
  int k = (int)(i % (K / 8)) * 8;
  const int dn = row0 + repack_row(n, mode, hd);
  const uint2 v = *(const uint2*)(W + (size_t)n * K + k);
  if (Wq) *(uint2*)(Wq + packed_w8_index(dn, k, K / 64, grp)) = v;
  if (Wp) {
    typedef float f2 __attribute__((ext_vector_type(2)));
    const f2 a = __builtin_amdgcn_cvt_pk_f32_fp8(v.x, false), b = __builtin_amdgcn_cvt_pk_f32_fp8(v.x, true);
    const f2 c = __builtin_amdgcn_cvt_pk_f32_fp8(v.y, false), d = __builtin_amdgcn_cvt_pk_f32_fp8(v.y, true);
    uint4 o = make_uint4(pack2_bf16(a[0], a[1]), pack2_bf16(b[0], b[1]), pack2_bf16(c[0], c[1]),
                         pack2_bf16(d[0], d[1]));
    *(uint4*)(Wp + packed_w_index(dn, k, K / 32, grp)) = o;
  }
}

void launch_repack_weight_e4m3(const uint8_t* W, int N, int K, uint8_t* Wq, bf16_t* Wp, int mode,
                               int hd, int grp, int row0, hipStream_t s) {
  size_t total = (size_t)N * (K / 8);
  repack_weight_e4m3_kernel<<<(unsigned)((total + 255) / 256), 256, 0, s>>>(W, N, K, Wq, Wp, mode,
                                                                            hd, grp, row0);
}

__global__ __launch_bounds__(256) void repack_rows_f32_kernel(const float* __restrict__ src, int N,
                                                              float* __restrict__ dst, int mode,
                                                              int hd, int row0) {
  int n = blockIdx.x * 256 + threadIdx.x;
  if (n < N) dst[row0 + repack_row(n, mode, hd)] = src[n];
}

void launch_repack_rows_f32(const float* src, int N, float* dst, int mode, int hd, int row0,
                            hipStream_t s) {
  repack_rows_f32_kernel<<<(N + 255) / 256, 256, 0, s>>>(src, N, dst, mode, hd, row0);
}

void launch_repack_weight(const bf16_t* W, int N, int K, bf16_t* Wp, int mode, int hd, int grp,
                          int row0, hipStream_t s) {
  size_t total = (size_t)N * (K / 8);
  repack_weight_kernel<<<(unsigned)((total + 255) / 256), 256, 0, s>>>(W, N, K, Wp, mode, hd, grp,
                                                                       row0);
}

// Rows sel[0..n) of a packed activation buffer (MT_src m-tiles) -> rows 0..n of another one.
__global__ __launch_bounds__(256) void gather_rows_packed_kernel(const bf16_t* __restrict__ src,
                                                                 int MT_src, const int* __restrict__ sel,
                                                                 int n, int K, bf16_t* __restrict__ dst,
                                                                 int MT_dst) {
  const int r = blockIdx.x;  // destination row, < MT_dst * 16
  const int from = r < n ? sel[r] : -1;
  for (int k8 = threadIdx.x * 8; k8 < K; k8 += 256 * 8) {
    uint4 v = make_uint4(0, 0, 0, 0);
    if (from >= 0) v = *(const uint4*)(src + packed_act_index(from, k8, MT_src));
    *(uint4*)(dst + packed_act_index(r, k8, MT_dst)) = v;
  }
}

void launch_gather_rows_packed(const bf16_t* src, int M_src, const int* sel, int n, int K,
                               bf16_t* dst, hipStream_t s) {
  if (n <= 0) return;
  const int MT_dst = (n + 15) / 16;
  gather_rows_packed_kernel<<<MT_dst * 16, 256, 0, s>>>(src, (M_src + 15) / 16, sel, n, K, dst, MT_dst);
}

// packed cache of one layer -> row-major [T, Hkv*hd]
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

}  // namespace ec
