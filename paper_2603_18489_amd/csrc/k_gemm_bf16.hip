// bf16 GEMMs on MFMA: C[M,N] = scale * A[M,K] W[N,K]^T (or C += ...), fp32 accumulation.
//
// Both operands arrive re-tiled into 16x32 fragments (k_common.h), so every wave-wide operand
// load is one contiguous, fully coalesced KiB.  The weight fragment is the MFMA "A" operand
// (16 weight rows) and the activation fragment the "B" operand (16 activation rows), hence a
// lane of the 16x16 result holds 4 consecutive output features n of one activation row m.
//
//  * skinny kernel (M <= 64): weight streaming.  A block of KS waves owns NTW weight tiles and
//    splits K across its waves; each wave streams its slice of the weights exactly once from
//    HBM while the small activation fragments come from L2.  The KS partial tiles are summed
//    in LDS in a fixed order (deterministic).
//  * tiled kernel (M > 64): 128x128 block tile, K step 32, LDS double buffering, 4 waves each
//    computing 64x64 with 16 MFMA accumulators.
#include "ec_internal.h"

namespace ec {

__device__ __forceinline__ bf16x8 as_bf16x8(uint4 v) {
  union { uint4 u; bf16x8 b; } c;
  c.u = v;
  return c.b;
}

// Segment lookup: global n-tile -> pointer to the tile's first fragment (kb = 0), or nullptr
// past the end.
__device__ __forceinline__ const uint4* seg_tile_ptr(const GemmSegs& sg, int nt, int KB) {
  int base = 0;
#pragma unroll
  for (int i = 0; i < 3; ++i) {
    if (i < sg.nseg) {
      if (nt < base + sg.ntiles[i])
        return (const uint4*)sg.w[i] + (size_t)(nt - base) * KB * 64;
      base += sg.ntiles[i];
    }
  }
  return nullptr;
}

// ---------------------------------------------------------------------------------------------
// skinny: grid = ceil(total n-tiles / NTW) blocks of KS*64 threads
// ---------------------------------------------------------------------------------------------
template <int MT, int NTW, int KS>
__global__ __launch_bounds__(KS * 64) void gemm_bf16_skinny_kernel(
    const uint4* __restrict__ Ap, GemmSegs sg, int KB, float* __restrict__ C, int ldc, int M,
    int accumulate, float scale) {
  extern __shared__ float4 red[];  // [KS][NTW*MT][64]
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int nt0 = blockIdx.x * NTW;
  const int kb_lo = (int)(((long)wave * KB) / KS), kb_hi = (int)(((long)(wave + 1) * KB) / KS);

  const uint4* wp[NTW];
#pragma unroll
  for (int i = 0; i < NTW; ++i) {
    // a tile past the end streams tile 0 instead (valid memory) and is dropped at the store
    const uint4* p = seg_tile_ptr(sg, nt0 + i, KB);
    wp[i] = (p ? p : (const uint4*)sg.w[0]) + (size_t)kb_lo * 64 + lane;
  }
  const uint4* ap = Ap + (size_t)kb_lo * MT * 64 + lane;

  f32x4 acc[NTW][MT];
#pragma unroll
  for (int i = 0; i < NTW; ++i)
#pragma unroll
    for (int j = 0; j < MT; ++j) acc[i][j] = (f32x4){0.f, 0.f, 0.f, 0.f};

  const int nkb = kb_hi - kb_lo;
#pragma unroll 4
  for (int it = 0; it < nkb; ++it) {
    uint4 wf[NTW], af[MT];
#pragma unroll
    for (int i = 0; i < NTW; ++i) wf[i] = wp[i][(size_t)it * 64];
#pragma unroll
    for (int j = 0; j < MT; ++j) af[j] = ap[((size_t)it * MT + j) * 64];
#pragma unroll
    for (int i = 0; i < NTW; ++i)
#pragma unroll
      for (int j = 0; j < MT; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(wf[i]), as_bf16x8(af[j]),
                                                            acc[i][j], 0, 0, 0);
  }

  // fixed-order reduction over the KS waves
#pragma unroll
  for (int i = 0; i < NTW; ++i)
#pragma unroll
    for (int j = 0; j < MT; ++j) {
      f32x4 v = acc[i][j];
      red[(wave * NTW * MT + i * MT + j) * 64 + lane] = make_float4(v[0], v[1], v[2], v[3]);
    }
  __syncthreads();
  for (int o = threadIdx.x; o < NTW * MT * 64; o += KS * 64) {
    float4 s = red[o];
#pragma unroll
    for (int w = 1; w < KS; ++w) {
      float4 v = red[w * NTW * MT * 64 + o];
      s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
    }
    int l = o & 63, tile = o >> 6, i = tile / MT, j = tile - i * MT;
    int m = j * 16 + (l & 15);
    int nt = nt0 + i;
    if (m < M && seg_tile_ptr(sg, nt, KB) != nullptr) {
      float4* c = (float4*)(C + (size_t)m * ldc + nt * 16 + (l >> 4) * 4);
      s.x *= scale; s.y *= scale; s.z *= scale; s.w *= scale;
      if (accumulate) {
        float4 old = *c;
        s.x += old.x; s.y += old.y; s.z += old.z; s.w += old.w;
      }
      *c = s;
    }
  }
}

template <int MT, int NTW, int KS>
static void launch_skinny_t(const bf16_t* Ap, int M, const GemmSegs& sg, int total_nt, int KB,
                            float* C, int ldc, int accumulate, float scale, hipStream_t s) {
  int grid = (total_nt + NTW - 1) / NTW;
  size_t smem = (size_t)KS * NTW * MT * 64 * sizeof(float4);
  gemm_bf16_skinny_kernel<MT, NTW, KS><<<grid, KS * 64, smem, s>>>((const uint4*)Ap, sg, KB, C, ldc,
                                                                  M, accumulate, scale);
}

template <int MT>
static void launch_skinny_mt(const bf16_t* Ap, int M, const GemmSegs& sg, int total_nt, int KB,
                             float* C, int ldc, int accumulate, float scale, hipStream_t s) {
  // enough blocks to cover 256 CUs a few times over, as many weight tiles per block as that allows
  if (total_nt >= 4096)
    launch_skinny_t<MT, 4, 4>(Ap, M, sg, total_nt, KB, C, ldc, accumulate, scale, s);
  else if (total_nt >= 1024)
    launch_skinny_t<MT, 2, 8>(Ap, M, sg, total_nt, KB, C, ldc, accumulate, scale, s);
  else
    launch_skinny_t<MT, 1, 8>(Ap, M, sg, total_nt, KB, C, ldc, accumulate, scale, s);
}

// ---------------------------------------------------------------------------------------------
// tiled: grid = (ceil(n-tiles/8), ceil(m-tiles/8)), 256 threads
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void gemm_bf16_tiled_kernel(const uint4* __restrict__ Ap,
                                                              GemmSegs sg, int total_nt, int KB,
                                                              int MT, float* __restrict__ C,
                                                              int ldc, int M, int accumulate,
                                                              float scale) {
  __shared__ uint4 lds[2][16][64];  // [stage][frag: 0..7 activations, 8..15 weights][lane]
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int mt0 = blockIdx.y * 8, nt0 = blockIdx.x * 8;
  const int wm = wave >> 1, wn = wave & 1;

  // global loads of this wave: activation tiles mt0+2w, +1 and weight tiles nt0+2w, +1
  const uint4* a_src[2];
  const uint4* w_src[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    int mt = mt0 + wave * 2 + i, nt = nt0 + wave * 2 + i;
    a_src[i] = (mt < MT) ? Ap + (size_t)mt * 64 + lane : nullptr;  // + kb*MT*64 per step
    const uint4* p = seg_tile_ptr(sg, nt, KB);
    w_src[i] = p ? p + lane : nullptr;                              // + kb*64 per step
  }
  const uint4 zero = make_uint4(0, 0, 0, 0);
  uint4 a_reg[2], w_reg[2];
  auto gload = [&](int kb) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      a_reg[i] = a_src[i] ? a_src[i][(size_t)kb * MT * 64] : zero;
      w_reg[i] = w_src[i] ? w_src[i][(size_t)kb * 64] : zero;
    }
  };
  auto lstore = [&](int stage) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      lds[stage][wave * 2 + i][lane] = a_reg[i];
      lds[stage][8 + wave * 2 + i][lane] = w_reg[i];
    }
  };

  f32x4 acc[4][4];  // [n-tile][m-tile]
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = (f32x4){0.f, 0.f, 0.f, 0.f};

  gload(0);
  lstore(0);
  __syncthreads();
  for (int kb = 0; kb < KB; ++kb) {
    int cur = kb & 1;
    if (kb + 1 < KB) gload(kb + 1);
    bf16x8 af[4], wf[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) af[j] = as_bf16x8(lds[cur][wm * 4 + j][lane]);
#pragma unroll
    for (int i = 0; i < 4; ++i) wf[i] = as_bf16x8(lds[cur][8 + wn * 4 + i][lane]);
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[i], af[j], acc[i][j], 0, 0, 0);
    if (kb + 1 < KB) lstore(cur ^ 1);
    __syncthreads();
  }

#pragma unroll
  for (int i = 0; i < 4; ++i) {
    int nt = nt0 + wn * 4 + i;
    if (nt >= total_nt) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int m = (mt0 + wm * 4 + j) * 16 + (lane & 15);
      if (m >= M) continue;
      float4* c = (float4*)(C + (size_t)m * ldc + nt * 16 + (lane >> 4) * 4);
      f32x4 v = acc[i][j];
      float4 s = make_float4(v[0] * scale, v[1] * scale, v[2] * scale, v[3] * scale);
      if (accumulate) {
        float4 old = *c;
        s.x += old.x; s.y += old.y; s.z += old.z; s.w += old.w;
      }
      *c = s;
    }
  }
}

void launch_gemm_bf16(const bf16_t* Ap, int M, const GemmSegs& sg, int K, float* C, int ldc,
                      int accumulate, float scale, hipStream_t s) {
  if (M <= 0) return;
  int total_nt = 0;
  for (int i = 0; i < sg.nseg; ++i) total_nt += sg.ntiles[i];
  int KB = K / 32, MT = (M + 15) / 16;
  if (MT <= 4) {
    switch (MT) {
      case 1: launch_skinny_mt<1>(Ap, M, sg, total_nt, KB, C, ldc, accumulate, scale, s); break;
      case 2: launch_skinny_mt<2>(Ap, M, sg, total_nt, KB, C, ldc, accumulate, scale, s); break;
      case 3: launch_skinny_mt<3>(Ap, M, sg, total_nt, KB, C, ldc, accumulate, scale, s); break;
      default: launch_skinny_mt<4>(Ap, M, sg, total_nt, KB, C, ldc, accumulate, scale, s); break;
    }
  } else {
    dim3 grid((total_nt + 7) / 8, (MT + 7) / 8);
    gemm_bf16_tiled_kernel<<<grid, 256, 0, s>>>((const uint4*)Ap, sg, total_nt, KB, MT, C, ldc, M,
                                                accumulate, scale);
  }
}

}  // namespace ec
