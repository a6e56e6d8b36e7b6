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
//  * tiled kernel (M > 64): 2x2 waves, block tile chosen per shape (up to 192x192) so that the
//    grid fills the 256 CUs, K step 32, LDS double buffering with register prefetch two steps
//    ahead.
#include "ec_internal.h"

namespace ec {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ bf16x8 v4_as_bf16x8(u32x4 v) {
  union { u32x4 u; bf16x8 b; } c;
  c.u = v;
  return c.b;
}
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
// tiled: 2x2 waves, wave tile = WTM x WTN fragments of 16 rows (activations x weights), K step 32.
// Operands are double-buffered in LDS; global loads run R k-steps ahead through R register sets
// so that L2/HBM latency is covered by R iterations of MFMA work.
// grid = (ceil(n-tiles / (2*WTN)), ceil(m-tiles / (2*WTM)))
// ---------------------------------------------------------------------------------------------
#define EC_TILED_GLOAD(REGS, KBV)                                                   \
  {                                                                                 \
    int kbc_ = min((KBV), KB - 1);                                                  \
    _Pragma("unroll") for (int i = 0; i < LF; ++i) REGS[i] = src[i][(size_t)kbc_ * stride[i]]; \
  }
#define EC_TILED_LSTORE(REGS, STAGE)                                                \
  {                                                                                 \
    _Pragma("unroll") for (int i = 0; i < LF; ++i) {                                \
      if (4 * i + 3 < NF || wave + 4 * i < NF) lds[STAGE][wave + 4 * i][lane] = REGS[i]; \
    }                                                                               \
  }
#define EC_TILED_COMPUTE(STAGE)                                                     \
  {                                                                                 \
    bf16x8 af_[WTM], wf_[WTN];                                                      \
    _Pragma("unroll") for (int j = 0; j < WTM; ++j)                                 \
        af_[j] = v4_as_bf16x8(lds[STAGE][wm * WTM + j][lane]);                         \
    _Pragma("unroll") for (int i = 0; i < WTN; ++i)                                 \
        wf_[i] = v4_as_bf16x8(lds[STAGE][BMT + wn * WTN + i][lane]);                   \
    _Pragma("unroll") for (int i = 0; i < WTN; ++i)                                 \
      _Pragma("unroll") for (int j = 0; j < WTM; ++j)                               \
        acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf_[i], af_[j], acc[i][j], 0, 0, 0); \
  }

template <int WTM, int WTN>
__global__ __launch_bounds__(256) void gemm_bf16_tiled_kernel(const u32x4* __restrict__ Ap,
                                                              GemmSegs sg, int total_nt, int KB,
                                                              int MT, float* __restrict__ C,
                                                              int ldc, int M, int accumulate,
                                                              float scale) {
  constexpr int BMT = 2 * WTM, BNT = 2 * WTN, NF = BMT + BNT;  // fragments per k-step
  constexpr int LF = (NF + 3) / 4;                             // fragments loaded per wave
  __shared__ u32x4 lds[2][NF][64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int mt0 = blockIdx.y * BMT, nt0 = blockIdx.x * BNT;
  const int wm = wave >> 1, wn = wave & 1;

  // Fragment f of the block (0..BMT-1 activations, BMT.. weights) is loaded by wave f % 4.
  // A fragment outside the matrix streams fragment 0 instead (valid memory); what it produces
  // lands in rows / columns that are never stored.
  const u32x4* src[LF];
  size_t stride[LF];  // uint4 per k-step
#pragma unroll
  for (int i = 0; i < LF; ++i) {
    int f = wave + 4 * i;
    src[i] = Ap + lane;
    stride[i] = (size_t)MT * 64;
    if (f < BMT) {
      int mt = mt0 + f;
      if (mt < MT) src[i] = Ap + (size_t)mt * 64 + lane;
    } else {
      const u32x4* p = (const u32x4*)seg_tile_ptr(sg, nt0 + (f - BMT), KB);
      if (f < NF && p) { src[i] = p + lane; stride[i] = 64; }
    }
  }

  f32x4 acc[WTN][WTM];
#pragma unroll
  for (int i = 0; i < WTN; ++i)
#pragma unroll
    for (int j = 0; j < WTM; ++j) acc[i][j] = (f32x4){0.f, 0.f, 0.f, 0.f};

  // prologue: k-step 0 into LDS stage 0, k-steps 1 and 2 in flight in the two register sets
  u32x4 r0[LF], r1[LF];
  EC_TILED_GLOAD(r0, 0)
  EC_TILED_LSTORE(r0, 0)
  EC_TILED_GLOAD(r0, 1)
  EC_TILED_GLOAD(r1, 2)
  __syncthreads();
  // iteration kb: compute stage kb&1; the register set holding k-step kb+1 goes to stage
  // (kb+1)&1 and is reloaded with k-step kb+3
  for (int kb = 0; kb < KB; kb += 2) {
    EC_TILED_COMPUTE(0)
    EC_TILED_LSTORE(r0, 1)
    EC_TILED_GLOAD(r0, kb + 3)
    __syncthreads();
    if (kb + 1 < KB) {
      EC_TILED_COMPUTE(1)
      EC_TILED_LSTORE(r1, 0)
      EC_TILED_GLOAD(r1, kb + 4)
    }
    __syncthreads();
  }

#pragma unroll
  for (int i = 0; i < WTN; ++i) {
    int nt = nt0 + wn * WTN + i;
    if (nt >= total_nt) continue;
#pragma unroll
    for (int j = 0; j < WTM; ++j) {
      int m = (mt0 + wm * WTM + j) * 16 + (lane & 15);
      if (m >= M) continue;
      float4* c = (float4*)(C + (size_t)m * ldc + nt * 16 + (lane >> 4) * 4);
      f32x4 v = acc[i][j];
      float4 o = make_float4(v[0] * scale, v[1] * scale, v[2] * scale, v[3] * scale);
      if (accumulate) {
        float4 old = *c;
        o.x += old.x; o.y += old.y; o.z += old.z; o.w += old.w;
      }
      *c = o;
    }
  }
}
#undef EC_TILED_GLOAD
#undef EC_TILED_LSTORE
#undef EC_TILED_COMPUTE

template <int WTM, int WTN>
static void launch_tiled_t(const bf16_t* Ap, int M, int MT, const GemmSegs& sg, int total_nt,
                           int KB, float* C, int ldc, int accumulate, float scale, hipStream_t s) {
  dim3 grid((total_nt + 2 * WTN - 1) / (2 * WTN), (MT + 2 * WTM - 1) / (2 * WTM));
  gemm_bf16_tiled_kernel<WTM, WTN><<<grid, 256, 0, s>>>((const u32x4*)Ap, sg, total_nt, KB, MT, C,
                                                        ldc, M, accumulate, scale);
}

// Picks the block tile whose grid wastes the least of the 256 CUs: the score is the useful
// fraction of the rounds the grid needs, weighted by how well the tile shape feeds the MFMAs.
static int pick_tile(int MT, int total_nt) {
  static const int wtm[4] = {6, 6, 4, 3}, wtn[4] = {6, 4, 4, 4};
  static const float shape_eff[4] = {1.00f, 0.90f, 0.80f, 0.62f};
  int best = 0;
  float best_score = -1.f;
  for (int i = 0; i < 4; ++i) {
    long gm = (MT + 2 * wtm[i] - 1) / (2 * wtm[i]), gn = (total_nt + 2 * wtn[i] - 1) / (2 * wtn[i]);
    long blocks = gm * gn, rounds = (blocks + 255) / 256;
    float useful = (float)((double)MT * total_nt / ((double)rounds * 256 * 4 * wtm[i] * wtn[i]));
    float score = useful * shape_eff[i];
    if (score > best_score) { best_score = score; best = i; }
  }
  return best;
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
    switch (pick_tile(MT, total_nt)) {
      case 0: launch_tiled_t<6, 6>(Ap, M, MT, sg, total_nt, KB, C, ldc, accumulate, scale, s); break;
      case 1: launch_tiled_t<6, 4>(Ap, M, MT, sg, total_nt, KB, C, ldc, accumulate, scale, s); break;
      case 2: launch_tiled_t<4, 4>(Ap, M, MT, sg, total_nt, KB, C, ldc, accumulate, scale, s); break;
      default: launch_tiled_t<3, 4>(Ap, M, MT, sg, total_nt, KB, C, ldc, accumulate, scale, s); break;
    }
  }
}

}  // namespace ec
