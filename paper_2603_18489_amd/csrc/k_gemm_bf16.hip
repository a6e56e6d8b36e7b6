// bf16 GEMMs on MFMA with the layer's element-wise work fused into their epilogues.
//
// C[M,N] = A[M,K] W[N,K]^T with fp32 accumulation.  Both operands arrive re-tiled into 16x32
// fragments (k_common.h), so every wave-wide operand load is one contiguous, fully coalesced KiB.
// The weight fragment is the MFMA "A" operand (16 weight rows) and the activation fragment the
// "B" operand (16 activation rows): a lane of the 16x16 result holds 4 consecutive output
// features n of one activation row m.
//
// RMSNorm is folded in: the A operand of a GEMM that follows a norm holds bf16(h * gain), NOT
// normalised, and the row's 1/rms is applied to the fp32 accumulator in the epilogue (it is a
// per-row scalar, so it commutes with the contraction).  The sum of squares of each row of h is
// accumulated by the producing epilogue with integer (44.20 fixed-point) atomics, which are
// order-independent and therefore bit-reproducible.
//
// Epilogues (template parameter EPI):
//   EPI_QKV    x 1/rms, rotary embedding on q and k (a weight tile holds 8 columns of a head
//              and their 8 partners hd/2 further on, so a rotation pair meets in lanes l and
//              l + 32), q -> query buffer, k / v -> the packed KV cache rows of the row's position
//   EPI_RESID  h += result; writes bf16(h * next gain) as the next GEMM's operand and adds the
//              row's sum of squares
//   EPI_SWIGLU x 1/rms, silu(gate) * up (8 gate rows and their 8 up rows share a tile), -> packed
//              activations
//   EPI_LOGITS x 1/rms x logit scale -> fp32 logits; the skinny kernel also reduces its block's
//              columns to one (max, argmax, sum e, sum e (z - max)) tuple per row - the
//              vocabulary reduction of Eq. 1 fused behind the LM head - and stores the logits
//              themselves only on request
//
// Kernels:
//   skinny (M <= 96): weight streaming.  A block of KS waves owns NTW weight tiles and splits K
//     across its waves; each weight byte is read from HBM exactly once while the small
//     activation fragments come from L2.  The KS partial tiles are summed in LDS in a fixed
//     order, then the epilogue runs on the sums.
//   tiled (M > 96): block tile chosen per shape so that the grid fills the 256 CUs.  4 waves:
//     LDS double buffer fed through four register sets.  8 waves (192x128 .. 192x384): operands
//     loaded from global memory directly into a 3-stage LDS ring.
#include "ec_internal.h"
#include "k_vtuple.h"

namespace ec {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ bf16x8 v4_as_bf16x8(u32x4 v) {
  union { u32x4 u; bf16x8 b; } c;
  c.u = v;
  return c.b;
}
// 8 e4m3 codes (two dwords, lowest byte first) -> 8 bf16 values, exactly (every e4m3 value is a
// bf16 value): four v_cvt_scalef32_pk_bf16_fp8 with scale 1
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ bf16x8 e4m3x8_as_bf16x8(uint32_t a, uint32_t b) {
  union { bf16x2_t h[4]; bf16x8 v; } c;
  c.h[0] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(a, 1.0f, false);
  c.h[1] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(a, 1.0f, true);
  c.h[2] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(b, 1.0f, false);
  c.h[3] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(b, 1.0f, true);
  return c.v;
}
__device__ __forceinline__ uint32_t pack2(float a, float b) { return pack2_bf16(a, b); }
// x * sigmoid(x) with the hardware exp2 and reciprocal (about 1 ulp each; the result is rounded
// to bf16 anyway).  exp overflow gives rcp(inf) = 0, the right limit.
__device__ __forceinline__ float silu_f(float x) {
  return x * __builtin_amdgcn_rcpf(1.0f + __expf(-x));
}

__device__ __forceinline__ float rstd_from_sum(const GemmEpi& e, unsigned long long fx) {
  double ss = sumsq_from_fixed(fx);
  return 1.0f / sqrtf((float)(ss / (double)e.d_in) + e.eps);
}
__device__ __forceinline__ float rstd_of(const GemmEpi& e, int row) {
  unsigned long long fx = 0;
#pragma unroll
  for (int sl = 0; sl < kSumSlots; ++sl) fx += e.sumsq_in[(size_t)sl * e.sum_stride + row];
  return rstd_from_sum(e, fx);
}

// ---- epilogues on one lane's values -----------------------------------------------------------
// (m: activation row, < M;  vt: virtual weight tile;  q4: lane>>4, so the lane's 4 values are
// output features vt*16 + q4*4 + 0..3.)

__device__ __forceinline__ void epi_logits(const GemmEpi& e, int m, int vt, int q4, f32x4 v,
                                           float rs) {
  float s = rs * e.scale;
  float4 o = make_float4(v[0] * s, v[1] * s, v[2] * s, v[3] * s);
  *(float4*)(e.logits + (size_t)m * e.ldc + vt * 16 + q4 * 4) = o;
}

// returns the lane's contribution to the row's sum of squares
__device__ __forceinline__ float epi_resid(const GemmEpi& e, int m, int vt, int q4, f32x4 v) {
  int n = vt * 16 + q4 * 4;
  float4* hp = (float4*)(e.h + (size_t)m * e.d + n);
  float4 h = *hp;
  h.x += v[0]; h.y += v[1]; h.z += v[2]; h.w += v[3];
  *hp = h;
  const bf16_t* g = e.gain_next + n;
  u32x2 pk;
  pk[0] = pack2(h.x * bf16_to_f32(g[0]), h.y * bf16_to_f32(g[1]));
  pk[1] = pack2(h.z * bf16_to_f32(g[2]), h.w * bf16_to_f32(g[3]));
  *(u32x2*)(e.a_next + packed_act_index(m, n, e.MT)) = pk;
  return h.x * h.x + h.y * h.y + h.z * h.z + h.w * h.w;
}

// epi_resid with h and the gains already in registers (fetched at kernel start)
__device__ __forceinline__ float epi_resid_pre(const GemmEpi& e, int m, int vt, int q4, f32x4 v,
                                               float4 h, u32x2 g4) {
  int n = vt * 16 + q4 * 4;
  h.x += v[0]; h.y += v[1]; h.z += v[2]; h.w += v[3];
  *(float4*)(e.h + (size_t)m * e.d + n) = h;
  u32x2 pk;
  pk[0] = pack2(h.x * __uint_as_float(g4[0] << 16), h.y * __uint_as_float(g4[0] & 0xffff0000u));
  pk[1] = pack2(h.z * __uint_as_float(g4[1] << 16), h.w * __uint_as_float(g4[1] & 0xffff0000u));
  *(u32x2*)(e.a_next + packed_act_index(m, n, e.MT)) = pk;
  return h.x * h.x + h.y * h.y + h.z * h.z + h.w * h.w;
}

__device__ __forceinline__ void epi_add_sumsq(const GemmEpi& e, int m, bool valid, float part) {
  // the 4 lanes l, l^16, l^32, l^48 hold the same row
  part += __shfl_xor(part, 16, 64);
  part += __shfl_xor(part, 32, 64);
  if (valid && (threadIdx.x & 63) < 16) {
    unsigned long long fx = sumsq_to_fixed(part);
    const int slot = (blockIdx.x + blockIdx.y) & (kSumSlots - 1);
    // (the padding rows of the row list are all zeros: nothing to add)
    if (fx) atomicAdd((unsigned long long*)(e.sumsq_out + (size_t)slot * e.sum_stride + m), fx);
  }
}

// Tile p of the interleaved matrix holds gate rows 8p..8p+7 in its rows 0-7 and the matching up
// rows in rows 8-15: lanes with q4 < 2 hold gates, their partners 32 lanes up hold the ups.
// (Lanes l and l^32 share the activation row, so a row-validity condition around the call keeps
// both or neither.)
__device__ __forceinline__ void epi_swiglu(const GemmEpi& e, int m, int p, int q4, f32x4 v,
                                           float rs) {
  float o[4];
#pragma unroll
  for (int r = 0; r < 4; ++r) o[r] = other_half(v[r]);
  if (q4 < 2) {
    u32x2 pk;
    pk[0] = pack2(silu_f(v[0] * rs) * (o[0] * rs), silu_f(v[1] * rs) * (o[1] * rs));
    pk[1] = pack2(silu_f(v[2] * rs) * (o[2] * rs), silu_f(v[3] * rs) * (o[3] * rs));
    *(u32x2*)(e.act + packed_act_index(m, p * 8 + q4 * 4, e.MT)) = pk;
  }
}

// Tiles p and p+1 at once, so that every lane has an activation to compute: lanes with q4 < 2
// finish tile p (own gates, partners' ups), the others tile p+1 (partners' gates, own ups).
__device__ __forceinline__ void epi_swiglu2(const GemmEpi& e, int m, int p, int q4, f32x4 va,
                                            f32x4 vb, float rs) {
  const bool lo = q4 < 2;
  u32x2 pk;
  float a[4];
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    float got = other_half(lo ? vb[r] : va[r]);
    float g = lo ? va[r] : got, u = lo ? got : vb[r];
    a[r] = silu_f(g * rs) * (u * rs);
  }
  pk[0] = pack2(a[0], a[1]); pk[1] = pack2(a[2], a[3]);
  *(u32x2*)(e.act + packed_act_index(m, (lo ? p : p + 1) * 8 + (q4 & 1) * 4, e.MT)) = pk;
}

// Virtual tile vt of the [q | k | v] matrix.  In the q and k regions tile w of a head holds the
// head's columns 8w..8w+7 in rows 0-7 and their rotary partners (hd/2 columns later) in rows
// 8-15, so a lane and its partner 32 lanes away hold one rotation pair; in the v region the
// tiles are in natural order.
__device__ __forceinline__ void epi_qkv(const GemmEpi& e, int m, int vt, int q4, f32x4 v,
                                        float rs) {
  const int hd = e.hd, tph = hd >> 4;  // tiles per head
  const int nqt = e.Hq * tph, nkt = e.Hkv * tph;
  const int4 ri = e.rowinfo[m];  // position, -, cache offset, keys per slab
  const int pos = ri.x;
  if (vt < nqt + nkt) {
    float o[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) o[r] = other_half(v[r]);
    if (pos < 0) return;  // padding row (its partner lane has the same row)
    const bool is_q = vt < nqt, hi = q4 >= 2;
    const int t = is_q ? vt : vt - nqt;
    const int head = t / tph, j = (t % tph) * 8 + (q4 & 1) * 4;  // column within the half head
    const float2* cs = e.cs + (size_t)pos * (hd >> 1) + j;
    float out[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      float x = v[r] * rs, y = o[r] * rs;
      float2 c = cs[r];
      out[r] = hi ? x * c.x + y * c.y : x * c.x - y * c.y;
    }
    u32x2 pk;
    pk[0] = pack2(out[0], out[1]); pk[1] = pack2(out[2], out[3]);
    const int col = j + (hi ? hd >> 1 : 0);
    if (is_q) {
      *(u32x2*)(e.q_out + (size_t)m * (e.Hq * hd) + head * hd + col) = pk;
    } else {
      bf16_t* slab = e.kc + ri.z + (size_t)head * ri.w * hd;
      *(u32x2*)(slab + kcache_index(pos, col, hd)) = pk;
    }
  } else if (pos >= 0) {
    const int t = vt - nqt - nkt;
    const int head = t / tph, c0 = (t % tph) * 16 + q4 * 4;
    bf16_t* slab = e.vc + ri.z + (size_t)head * ri.w * hd;
#pragma unroll
    for (int r = 0; r < 4; ++r) slab[vcache_index(pos, c0 + r, ri.w)] = f32_to_bf16(v[r] * rs);
  }
}

// ---------------------------------------------------------------------------------------------
// skinny: grid = ceil(n-tiles / NTW) blocks of KS*64 threads
// ---------------------------------------------------------------------------------------------
// W8: the weights are e4m3 codes (k_common.h: packed_w8_index), one 1 KiB fragment pair covering
// 64 k per weight tile and k-step; a lane's 16 bytes are turned into two bf16 MFMA operands in
// registers (exact), so a k-step is two MFMAs per (weight tile, m-tile) on two activation
// fragments, KB counts 64-wide steps, and the per-row scales multiply the K-reduced sums.
template <int EPI, int MT, int NTW, int KS, int U, bool W8 = false>
__global__ __launch_bounds__(KS * 64) void gemm_bf16_skinny_kernel(const u32x4* __restrict__ Ap,
                                                                   const u32x4* __restrict__ Wp,
                                                                   int total_nt, int KB,
                                                                   int MT_src, GemmEpi e) {
  constexpr int AW = W8 ? 2 : 1;   // activation fragments per k-step
  extern __shared__ float4 red[];  // [KS][NTW*MT][64]
  // the wave index is made a scalar so that everything derived from it (the K slice) is
  // provably wave-uniform: MFMA ignores the EXEC mask, so it must never sit under a condition
  // the compiler could treat as divergent
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int nt0 = blockIdx.x * NTW;
  const int kb_lo = (wave * KB) / KS, kb_hi = ((wave + 1) * KB) / KS;

  // a tile past the end streams tile 0 instead (valid memory) and is dropped at the store
  const int grp = e.w_grp;
  const u32x4* wp[NTW];
#pragma unroll
  for (int i = 0; i < NTW; ++i) {
    int nt = nt0 + i < total_nt ? nt0 + i : 0;
    wp[i] = Wp + packed_w_frag(nt, kb_lo, KB, grp) * 64 + lane;
  }
  const size_t wstep = (size_t)grp * 64;  // u32x4 per k-step
  // activation rows may be gathered (LM head: only the block's masked rows)
  const u32x4* ap[MT];
#pragma unroll
  for (int j = 0; j < MT; ++j) {
    int m = j * 16 + (lane & 15);
    int row = m < e.M ? m : 0;
    if constexpr (EPI == EPI_LOGITS) row = (m < e.M && e.row_sel) ? e.row_sel[m] : row;
    ap[j] = Ap + ((size_t)kb_lo * AW * MT_src + (row >> 4)) * 64 + (lane >> 4) * 16 + (row & 15);
  }

  constexpr bool NORMED = (EPI == EPI_QKV || EPI == EPI_SWIGLU || EPI == EPI_LOGITS);
  float* rstd_s = (float*)(red + KS * NTW * MT * 64);  // [MT*16]: 1/rms of the block's rows

  f32x4 acc[NTW][MT];
#pragma unroll
  for (int i = 0; i < NTW; ++i)
#pragma unroll
    for (int j = 0; j < MT; ++j) acc[i][j] = (f32x4){0.f, 0.f, 0.f, 0.f};

  // Two register sets of U k-steps each (U is a template parameter): while one set feeds the
  // MFMAs the other set's loads are in flight, so a wave always has up to 2*U*(NTW+MT) KiB
  // outstanding.  Every load is issued unconditionally (straight-line code lets the compiler
  // count outstanding loads exactly): k-steps past the slice re-read the slice's last fragments,
  // which are still in cache, and their activation operand is replaced by zeros, so the MFMAs,
  // which ignore EXEC and must run unconditionally anyway, add nothing.
  // The weights are loaded with the non-temporal hint: every byte of them is used once, and kept
  // out of the way they leave the L2 to the activation fragments that all blocks re-read
  // (measured: the whole partial step 3.31 -> 3.11 ms).
  const int nkb = kb_hi - kb_lo;
  const int last = nkb > 0 ? nkb - 1 : 0;
  const u32x4 zero4 = {0u, 0u, 0u, 0u};
  u32x4 wa[U][NTW], aa[U][MT * AW], wb[U][NTW], ab[U][MT * AW];
#define EC_SK_LOAD(WSET, ASET, IT0)                                                        \
  _Pragma("unroll") for (int u = 0; u < U; ++u) {                                          \
    const int it_ = (IT0) + u < last ? (IT0) + u : last;                                   \
    _Pragma("unroll") for (int i = 0; i < NTW; ++i) WSET[u][i] = __builtin_nontemporal_load(&wp[i][(size_t)it_ * wstep]);  \
    _Pragma("unroll") for (int j = 0; j < MT; ++j)                                         \
      _Pragma("unroll") for (int h = 0; h < AW; ++h)                                       \
        ASET[u][j * AW + h] = ap[j][((size_t)it_ * AW + h) * MT_src * 64];                 \
  }
#define EC_SK_ZERO_TAIL(ASET, IT0)                                                         \
  _Pragma("unroll") for (int u = 0; u < U; ++u) {                                          \
    const bool in_ = (IT0) + u < nkb;                                                      \
    _Pragma("unroll") for (int j = 0; j < MT * AW; ++j) ASET[u][j] = in_ ? ASET[u][j] : zero4;  \
  }
#define EC_SK_MMA(WSET, ASET)                                                              \
  _Pragma("unroll") for (int u = 0; u < U; ++u)                                            \
    _Pragma("unroll") for (int i = 0; i < NTW; ++i) {                                      \
      if constexpr (W8) {                                                                  \
        const bf16x8 lo_ = e4m3x8_as_bf16x8(WSET[u][i][0], WSET[u][i][1]);                 \
        const bf16x8 hi_ = e4m3x8_as_bf16x8(WSET[u][i][2], WSET[u][i][3]);                 \
        _Pragma("unroll") for (int j = 0; j < MT; ++j) {                                   \
          acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(                             \
              lo_, v4_as_bf16x8(ASET[u][j * AW]), acc[i][j], 0, 0, 0);                     \
          acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(                             \
              hi_, v4_as_bf16x8(ASET[u][j * AW + AW - 1]), acc[i][j], 0, 0, 0);            \
        }                                                                                  \
      } else {                                                                             \
        _Pragma("unroll") for (int j = 0; j < MT; ++j)                                     \
          acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(                             \
              v4_as_bf16x8(WSET[u][i]), v4_as_bf16x8(ASET[u][j]), acc[i][j], 0, 0, 0);     \
      }                                                                                    \
    }
  EC_SK_LOAD(wa, aa, 0)
  // The rows' sum-of-squares counters are fetched behind the first operand loads and turned
  // into 1/rms after the main loop, so neither the loop nor the epilogue waits on them.  All
  // threads load (those without a row of their own read row 0): no branch, so the compiler
  // still counts outstanding loads exactly.
  // Epilogue operands of the thread's first output unit are fetched here too: the residual
  // stream and gains (EPI_RESID) so that the epilogue does not start with a round trip to memory.
  constexpr int UNITS = NTW * MT * 64;  // whole waves: the wave's 64 lanes share (tile, m-tile)
  float4 pre_h = make_float4(0.f, 0.f, 0.f, 0.f);
  u32x2 pre_g = {0u, 0u};
  if constexpr (EPI == EPI_RESID) {
    const int o = threadIdx.x < UNITS ? threadIdx.x : 0;
    const int l = o & 63, unit = o >> 6, iu = unit / MT, j = unit - iu * MT;
    const int m = j * 16 + (l & 15), vt = nt0 + iu;
    const int mm = m < e.M ? m : 0, n = (vt < total_nt ? vt : 0) * 16 + (l >> 4) * 4;
    pre_h = *(const float4*)(e.h + (size_t)mm * e.d + n);
    pre_g = *(const u32x2*)(e.gain_next + n);
  }
  // W8: the block's per-row weight scales, fetched here and parked in LDS behind the main loop
  float* wsc_s = rstd_s + MT * 16 + (EPI == EPI_LOGITS ? NTW * MT * 16 * 4 : 0);  // [NTW*16]
  float wsc_reg = 1.f;
  if constexpr (W8) {
    const int n_ = nt0 * 16 + (int)threadIdx.x;
    wsc_reg = e.wscale[(threadIdx.x < NTW * 16 && n_ < total_nt * 16) ? n_ : 0];
  }
  unsigned long long ssq[kSumSlots];
  if constexpr (NORMED) {
#pragma unroll
    for (int sl = 0; sl < kSumSlots; ++sl) ssq[sl] = 0;
    __builtin_amdgcn_sched_barrier(0);
    if (threadIdx.x < MT * 16) {
      int row = (int)threadIdx.x < e.M ? (int)threadIdx.x : 0;
      if constexpr (EPI == EPI_LOGITS) row = (e.row_sel && (int)threadIdx.x < e.M) ? e.row_sel[row] : row;
#pragma unroll
      for (int sl = 0; sl < kSumSlots; ++sl) ssq[sl] = e.sumsq_in[(size_t)sl * e.sum_stride + row];
    }
    __builtin_amdgcn_sched_barrier(0);
  }
  // (the scheduling barriers keep the compiler from sinking a set's loads down to their first
  // use, which would leave nothing in flight during the MFMAs)
  int it0 = 0;
  for (; it0 + 2 * U < nkb; it0 += 2 * U) {
    EC_SK_LOAD(wb, ab, it0 + U)
    __builtin_amdgcn_sched_barrier(0);
    EC_SK_MMA(wa, aa)
    __builtin_amdgcn_sched_barrier(0);
    EC_SK_LOAD(wa, aa, it0 + 2 * U)
    __builtin_amdgcn_sched_barrier(0);
    EC_SK_MMA(wb, ab)
    __builtin_amdgcn_sched_barrier(0);
  }
  // last 1 .. 2U k-steps: nothing left to prefetch; only here can a k-step lie past the slice
  EC_SK_LOAD(wb, ab, it0 + U)
  __builtin_amdgcn_sched_barrier(0);
  EC_SK_ZERO_TAIL(aa, it0)
  EC_SK_MMA(wa, aa)
  EC_SK_ZERO_TAIL(ab, it0 + U)
  EC_SK_MMA(wb, ab)
#undef EC_SK_ZERO_TAIL
#undef EC_SK_LOAD
#undef EC_SK_MMA

  // fixed-order reduction over the KS waves
#pragma unroll
  for (int i = 0; i < NTW; ++i)
#pragma unroll
    for (int j = 0; j < MT; ++j) {
      f32x4 v = acc[i][j];
      red[(wave * NTW * MT + i * MT + j) * 64 + lane] = make_float4(v[0], v[1], v[2], v[3]);
    }
  if constexpr (NORMED) {
    unsigned long long fx = 0;
#pragma unroll
    for (int sl = 0; sl < kSumSlots; ++sl) {
      // keeps the compiler from adding the counters up (and waiting for them) before the loop
      asm volatile("" : "+v"(ssq[sl]));
      fx += ssq[sl];
    }
    if (threadIdx.x < MT * 16) rstd_s[threadIdx.x] = rstd_from_sum(e, fx);
  }
  if constexpr (W8) {
    if (threadIdx.x < NTW * 16) wsc_s[threadIdx.x] = wsc_reg;
  }
  __syncthreads();

  // sum over the KS waves of the lane's 4 output features of weight tile iu (times their scales)
  auto ksum = [&](int idx, int iu, int q4) {
    float4 s = red[idx];
#pragma unroll
    for (int w = 1; w < KS; ++w) {
      float4 v = red[w * NTW * MT * 64 + idx];
      s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
    }
    if constexpr (W8) {
      const float4 c = *(const float4*)(wsc_s + iu * 16 + q4 * 4);
      s.x *= c.x; s.y *= c.y; s.z *= c.z; s.w *= c.w;
    }
    return (f32x4){s.x, s.y, s.z, s.w};
  };

  static_assert(EPI != EPI_PARTIAL, "K-split partial products are a tiled-kernel epilogue");
  if constexpr (EPI == EPI_LOGITS) {
    // Logits of the block's NTW*16 columns, and their reduction.  A row's 16 columns of one tile
    // sit in the 4 lanes l, l^16, l^32, l^48 (4 columns each): maximum and lowest index holding
    // it through two lane swaps, then sum e^(z-max) and sum e^(z-max)(z-max) relative to that
    // maximum (added pairwise, the same pairs in all four lanes, so they agree bit for bit);
    // after a barrier one thread per row merges the NTW tiles in tile order and stores the
    // block's tuple.
    float4* tup = (float4*)(rstd_s + MT * 16);  // [NTW][MT*16]
    for (int o = threadIdx.x; o < UNITS; o += KS * 64) {  // UNITS is a multiple of the block size
      const int l = o & 63, unit = o >> 6, iu = unit / MT, j = unit - iu * MT;
      const int m = j * 16 + (l & 15), q4 = l >> 4, vt = nt0 + iu;
      const f32x4 v = ksum((iu * MT + j) * 64 + l, iu, q4);
      // (rows past M recompute row 0 and tiles past the end tile 0: finite values, dropped below)
      const float sc = rstd_s[m] * e.scale;
      const float z[4] = {v[0] * sc, v[1] * sc, v[2] * sc, v[3] * sc};
      const int n = vt * 16 + q4 * 4;
      const bool live = m < e.M && vt < total_nt;
      if (live && e.logits)
        *(float4*)(e.logits + (size_t)m * e.ldc + n) = make_float4(z[0], z[1], z[2], z[3]);
      float mx = fmaxf(fmaxf(z[0], z[1]), fmaxf(z[2], z[3]));
      mx = fmaxf(mx, other_row(mx));
      mx = fmaxf(mx, other_half(mx));
      int idx = z[0] == mx ? n : z[1] == mx ? n + 1 : z[2] == mx ? n + 2 : z[3] == mx ? n + 3 : INT_MAX;
      idx = min(idx, __float_as_int(other_row(__int_as_float(idx))));
      idx = min(idx, __float_as_int(other_half(__int_as_float(idx))));
      float s4 = 0.f, t4 = 0.f;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const float d = z[r] - mx, ex = __expf(d);
        s4 += ex;
        t4 += ex * d;
      }
      s4 += other_row(s4); t4 += other_row(t4);
      s4 += other_half(s4); t4 += other_half(t4);
      if (q4 == 0)
        tup[iu * (MT * 16) + m] = vt < total_nt ? make_float4(mx, __int_as_float(idx), s4, t4)
                                                : vt_pack(vt_identity());
    }
    __syncthreads();
    if (threadIdx.x < MT * 16 && (int)threadIdx.x < e.M) {
      VTuple t = vt_unpack(tup[threadIdx.x]);
#pragma unroll
      for (int iu = 1; iu < NTW; ++iu) t = vt_merge(t, vt_unpack(tup[iu * (MT * 16) + threadIdx.x]));
      e.vparts[(size_t)threadIdx.x * gridDim.x + blockIdx.x] = vt_pack(t);
    }
    return;
  }
  for (int o = threadIdx.x; o < UNITS; o += KS * 64) {
    const int l = o & 63, unit = o >> 6, iu = unit / MT, j = unit - iu * MT;
    const int m = j * 16 + (l & 15), q4 = l >> 4;
    const bool mvalid = m < e.M;
    const int vt = nt0 + iu;
    f32x4 v = ksum((iu * MT + j) * 64 + l, iu, q4);
    if constexpr (EPI == EPI_RESID) {
      float part = 0.f;
      if (mvalid && vt < total_nt)
        part = o < KS * 64 ? epi_resid_pre(e, m, vt, q4, v, pre_h, pre_g) : epi_resid(e, m, vt, q4, v);
      epi_add_sumsq(e, m, mvalid, part);
    } else if (mvalid && vt < total_nt) {
      if constexpr (EPI == EPI_SWIGLU) epi_swiglu(e, m, vt, q4, v, rstd_s[m]);
      else epi_qkv(e, m, vt, q4, v, rstd_s[m]);
    }
  }
}

template <int EPI, int MT, int NTW, int KS, int U = 4, bool W8 = false>
static void launch_skinny_t(const bf16_t* Ap, int MT_src, const void* Wp, int total_nt, int KB,
                            const GemmEpi& e, hipStream_t s) {
  int grid = (total_nt + NTW - 1) / NTW;
  size_t smem = (size_t)KS * NTW * MT * 64 * sizeof(float4) + MT * 16 * sizeof(float);
  if (EPI == EPI_LOGITS) smem += (size_t)NTW * MT * 16 * sizeof(float4);  // per-tile row tuples
  if (W8) smem += NTW * 16 * sizeof(float);                               // weight scales
  if (smem > 48 * 1024) {
    static bool once = false;
    if (!once) {
      hipFuncSetAttribute((const void*)gemm_bf16_skinny_kernel<EPI, MT, NTW, KS, U, W8>,
                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
      once = true;
    }
  }
  gemm_bf16_skinny_kernel<EPI, MT, NTW, KS, U, W8><<<grid, KS * 64, smem, s>>>(
      (const u32x4*)Ap, (const u32x4*)Wp, total_nt, KB, MT_src, e);
}

// Tile counts per block were chosen by timing on MI355X: the kernels are bound by what the L2
// delivers (weights once + the activation fragments once per block), so more weight tiles per
// block (fewer re-reads of the activations) win as long as the grid still covers the 256 CUs.
// blocks (= partial tuples per row) of the skinny LM-head GEMM over a vocabulary of V columns
constexpr int kLmTiles = 8;  // weight tiles (of 16 vocabulary columns) per LM-head block
int lm_head_parts(int V) { return (V / 16 + kLmTiles - 1) / kLmTiles; }

int skinny_tiles_per_block(int epi, int total_nt) {
  if (epi == EPI_RESID) return 1;
  if (epi == EPI_LOGITS) return kLmTiles;
  if (total_nt >= 6 * 256) return 6;
  if (total_nt >= 3 * 256) return 3;
  return total_nt >= 2 * 256 ? 2 : 1;
}

// e4m3 weights: KB counts 64-wide k-steps; fewer steps per register set, because a step holds
// two activation fragments per m-tile
template <int EPI, int MT>
static void launch_skinny_mt_w8(const bf16_t* Ap, int MT_src, const void* Wq, int total_nt,
                                int KB, const GemmEpi& e, hipStream_t s) {
  if constexpr (EPI == EPI_LOGITS) {
    launch_skinny_t<EPI, MT, kLmTiles, 4, 1, true>(Ap, MT_src, Wq, total_nt, KB, e, s);
  } else if constexpr (EPI == EPI_RESID) {
    launch_skinny_t<EPI, MT, 1, 8, (MT > 3 ? 1 : 2), true>(Ap, MT_src, Wq, total_nt, KB, e, s);
  } else {
    constexpr int U6 = MT > 2 ? 1 : 2, U8 = MT > 3 ? 1 : 2;
    switch (skinny_tiles_per_block(EPI, total_nt)) {
      case 6: launch_skinny_t<EPI, MT, 6, 4, U6, true>(Ap, MT_src, Wq, total_nt, KB, e, s); break;
      case 3: launch_skinny_t<EPI, MT, 3, 8, U8, true>(Ap, MT_src, Wq, total_nt, KB, e, s); break;
      case 2: launch_skinny_t<EPI, MT, 2, 8, U8, true>(Ap, MT_src, Wq, total_nt, KB, e, s); break;
      default: launch_skinny_t<EPI, MT, 1, 8, U8, true>(Ap, MT_src, Wq, total_nt, KB, e, s); break;
    }
  }
}

template <int EPI, int MT>
static void launch_skinny_mt(const bf16_t* Ap, int MT_src, const bf16_t* Wp, int total_nt, int KB,
                             const GemmEpi& e, hipStream_t s) {
  if constexpr (EPI == EPI_LOGITS) {
    launch_skinny_t<EPI, MT, kLmTiles, 4, (MT > 2 ? 1 : 2)>(Ap, MT_src, Wp, total_nt, KB, e, s);
  } else if constexpr (EPI == EPI_RESID) {
    launch_skinny_t<EPI, MT, 1, 8, 2>(Ap, MT_src, Wp, total_nt, KB, e, s);
  } else {
    // (five or six m-tiles: one k-step per register set where two would not fit 256 registers)
    constexpr int U8 = MT > 4 ? 1 : 2;
    switch (skinny_tiles_per_block(EPI, total_nt)) {
      case 6: launch_skinny_t<EPI, MT, 6, 4, 2>(Ap, MT_src, Wp, total_nt, KB, e, s); break;
      case 3: launch_skinny_t<EPI, MT, 3, 8, U8>(Ap, MT_src, Wp, total_nt, KB, e, s); break;
      case 2: launch_skinny_t<EPI, MT, 2, 8, U8>(Ap, MT_src, Wp, total_nt, KB, e, s); break;
      default: launch_skinny_t<EPI, MT, 1, 8, 2>(Ap, MT_src, Wp, total_nt, KB, e, s); break;
    }
  }
}

// ---------------------------------------------------------------------------------------------
// QKV epilogue of the tiled kernels.  The rotation factors come from a table in global memory;
// a load issued between two stores cannot be moved up by the compiler (the stores might alias
// it), so one m-tile's factors are fetched while the previous m-tile is rotated and stored:
// one exposed load latency per wave instead of one per accumulator tile.  (Needs registers the
// 8-wave kernels do not have; they rotate tile by tile.)
// ---------------------------------------------------------------------------------------------
template <int WTM, int WTN>
__device__ __forceinline__ void tiled_epilogue_qkv(const GemmEpi& e, f32x4 (&acc)[WTN][WTM],
                                                   int mt_base, int nt_base, int total_nt,
                                                   int lane) {
  const int q4 = lane >> 4, hd = e.hd, tph = hd >> 4, half = hd >> 1;
  const int nqt = e.Hq * tph, nkt = e.Hkv * tph;
  const bool hi = q4 >= 2;
  // wave-uniform description of the WTN weight tiles: kind 0 = q, 1 = k, 2 = v, 3 = past the end
  int kind[WTN], head[WTN], w[WTN];
#pragma unroll
  for (int i = 0; i < WTN; ++i) {
    const int vt = nt_base + i;
    kind[i] = vt >= total_nt ? 3 : vt < nqt ? 0 : vt < nqt + nkt ? 1 : 2;
    const int t = kind[i] == 0 ? vt : kind[i] == 1 ? vt - nqt : kind[i] == 2 ? vt - nqt - nkt : 0;
    head[i] = t / tph;
    w[i] = t - head[i] * tph;
  }
  // Addresses split into a row part (per m-tile j) and a column part (per weight tile i): the
  // cache index functions are sums of a function of the key and a function of the column.
  //   q:  row m * Hq*hd            + head*hd + col
  //   K:  slab(head) + K(key)      + C(col)       (k_common.h: kcache_index)
  //   V:  slab(head) + Vk(key)     + w * Vs + (q4*4 + r) * 8,  Vs = keys/32 * 512 per hd tile
  int pos[WTM], krow[WTM], vrow[WTM], vstep[WTM], slab[WTM];
  size_t qrow[WTM];
  float rs[WTM];
  bool mvalid[WTM];
#pragma unroll
  for (int j = 0; j < WTM; ++j) {
    const int m = (mt_base + j) * 16 + (lane & 15);
    const int mm = m < e.M ? m : 0;
    const int4 ri = e.rowinfo[mm];
    mvalid[j] = m < e.M && ri.x >= 0;  // not a padding row
    pos[j] = ri.x >= 0 ? ri.x : 0;
    qrow[j] = (size_t)mm * (e.Hq * hd);
    krow[j] = ri.z + (int)kcache_index(pos[j], 0, hd);
    vrow[j] = ri.z + (int)vcache_index(pos[j], 0, ri.w);
    vstep[j] = (ri.w >> 5) * 512;
    slab[j] = ri.w * hd;  // elements per kv head
    rs[j] = rstd_of(e, mm);
  }
  const int colq = (q4 & 1) * 4 + (hi ? half : 0);  // the lane's first column within a head, tile 0
  int qcol[WTN], kcol[WTN];
#pragma unroll
  for (int i = 0; i < WTN; ++i) {
    qcol[i] = head[i] * hd + w[i] * 8 + colq;
    kcol[i] = (int)kcache_index(0, w[i] * 8 + colq, hd);
  }
  const unsigned sin_sign = hi ? 0u : 0x80000000u;  // first half: x cos - y sin; second: x cos + y sin
  float4 ca[WTN][2], cb[WTN][2];  // (cos, sin) x 4 columns for each rotary tile of one m-tile
#define EC_QKV_LOADC(C, J)                                                                   \
  _Pragma("unroll") for (int i = 0; i < WTN; ++i) if (kind[i] < 2) {                           \
    const float4* src_ = (const float4*)(e.cs + (size_t)pos[J] * half + w[i] * 8 + (q4 & 1) * 4); \
    C[i][0] = src_[0];                                                                       \
    C[i][1] = src_[1];                                                                       \
  }
#define EC_QKV_STORE(C, J)                                                                   \
  _Pragma("unroll") for (int i = 0; i < WTN; ++i) {                                            \
    const f32x4 v = acc[i][J];                                                               \
    if (kind[i] < 2) {                                                                       \
      float out_[4];                                                                         \
      const float cc_[4] = {C[i][0].x, C[i][0].z, C[i][1].x, C[i][1].z};                      \
      const float ss_[4] = {C[i][0].y, C[i][0].w, C[i][1].y, C[i][1].w};                      \
      _Pragma("unroll") for (int r = 0; r < 4; ++r) {                                          \
        const float y_ = other_half(v[r]);                                                   \
        const float s_ = __uint_as_float(__float_as_uint(ss_[r]) ^ sin_sign);                \
        out_[r] = (v[r] * cc_[r] + y_ * s_) * rs[J];                                         \
      }                                                                                      \
      u32x2 pk_;                                                                             \
      pk_[0] = pack2(out_[0], out_[1]);                                                      \
      pk_[1] = pack2(out_[2], out_[3]);                                                      \
      if (mvalid[J]) {                                                                       \
        if (kind[i] == 0)                                                                    \
          *(u32x2*)(e.q_out + qrow[J] + qcol[i]) = pk_;                                      \
        else                                                                                 \
          *(u32x2*)(e.kc + (size_t)head[i] * slab[J] + krow[J] + kcol[i]) = pk_;             \
      }                                                                                      \
    } else if (kind[i] == 2 && mvalid[J]) {                                                  \
      bf16_t* dst_ = e.vc + (size_t)head[i] * slab[J] + vrow[J] + w[i] * vstep[J] + q4 * 32; \
      _Pragma("unroll") for (int r = 0; r < 4; ++r) dst_[r * 8] = f32_to_bf16(v[r] * rs[J]);   \
    }                                                                                        \
  }
  EC_QKV_LOADC(ca, 0)
#pragma unroll
  for (int j = 0; j < WTM; j += 2) {
    if (j + 1 < WTM) { EC_QKV_LOADC(cb, j + 1) }
    EC_QKV_STORE(ca, j)
    if (j + 1 < WTM) {
      if (j + 2 < WTM) { EC_QKV_LOADC(ca, j + 2) }
      EC_QKV_STORE(cb, j + 1)
    }
  }
#undef EC_QKV_LOADC
#undef EC_QKV_STORE
}

template <int EPI, int WTM, int WTN, bool PIPE = true>
__device__ __forceinline__ void tiled_epilogue(const GemmEpi& e, f32x4 (&acc)[WTN][WTM],
                                               int mt_base, int nt_base, int total_nt, int lane,
                                               int kz) {
  if constexpr (EPI == EPI_QKV && PIPE) {
    tiled_epilogue_qkv<WTM, WTN>(e, acc, mt_base, nt_base, total_nt, lane);
    return;
  }
  const int q4 = lane >> 4;
  // every row's 1/rms first: these loads must not be strung out between the stores below
  float rsj[WTM];
  if constexpr (EPI == EPI_SWIGLU || EPI == EPI_LOGITS || EPI == EPI_QKV) {
#pragma unroll
    for (int j = 0; j < WTM; ++j) {
      const int m = (mt_base + j) * 16 + (lane & 15);
      const int mm = m < e.M ? m : 0;
      rsj[j] = rstd_of(e, (EPI == EPI_LOGITS && e.row_sel) ? e.row_sel[mm] : mm);
    }
  }
#pragma unroll
  for (int j = 0; j < WTM; ++j) {
    const int m = (mt_base + j) * 16 + (lane & 15);
    const bool mvalid = m < e.M;
    if constexpr (EPI == EPI_RESID) {
      float part = 0.f;
#pragma unroll
      for (int i = 0; i < WTN; ++i) {
        int vt = nt_base + i;
        if (mvalid && vt < total_nt) part += epi_resid(e, m, vt, q4, acc[i][j]);
      }
      epi_add_sumsq(e, m, mvalid, part);
    } else if constexpr (EPI == EPI_LOGITS) {
      if (mvalid) {
        const float rs = rsj[j];
#pragma unroll
        for (int i = 0; i < WTN; ++i) {
          int vt = nt_base + i;
          if (vt < total_nt) epi_logits(e, m, vt, q4, acc[i][j], rs);
        }
      }
    } else if constexpr (EPI == EPI_PARTIAL) {
      if (mvalid) {
#pragma unroll
        for (int i = 0; i < WTN; ++i) {
          int vt = nt_base + i;
          if (vt < total_nt) {
            f32x4 v = acc[i][j];
            *(float4*)(e.partial + ((size_t)kz * e.M + m) * e.d + vt * 16 + q4 * 4) =
                make_float4(v[0], v[1], v[2], v[3]);
          }
        }
      }
    } else {
      if (mvalid) {
        const float rs = rsj[j];
#pragma unroll
        for (int i = 0; i < WTN; ++i) {
          int vt = nt_base + i;
          if constexpr (EPI == EPI_SWIGLU && WTN % 2 == 0) {
            if (i & 1) continue;
            if (vt + 1 < total_nt) epi_swiglu2(e, m, vt, q4, acc[i][j], acc[i + 1][j], rs);
            else if (vt < total_nt) epi_swiglu(e, m, vt, q4, acc[i][j], rs);
          } else if (vt < total_nt) {
            if constexpr (EPI == EPI_SWIGLU) epi_swiglu(e, m, vt, q4, acc[i][j], rs);
            else epi_qkv(e, m, vt, q4, acc[i][j], rs);
          }
        }
      }
    }
  }
}

// Per-row weight scales (matrices that came as e4m3 codes, expanded to bf16 for these kernels):
// the lane's 4 accumulator values of weight tile i are output features (nt_base + i)*16 + q4*4 ..
template <int WTM, int WTN>
__device__ __forceinline__ void scale_acc(const GemmEpi& e, f32x4 (&acc)[WTN][WTM], int nt_base,
                                          int total_nt, int lane) {
  const int q4 = lane >> 4;
#pragma unroll
  for (int i = 0; i < WTN; ++i) {
    const int vt = nt_base + i < total_nt ? nt_base + i : 0;
    const float4 c = *(const float4*)(e.wscale + (size_t)vt * 16 + q4 * 4);
#pragma unroll
    for (int j = 0; j < WTM; ++j) {
      f32x4 a = acc[i][j];
      a[0] *= c.x; a[1] *= c.y; a[2] *= c.z; a[3] *= c.w;
      acc[i][j] = a;
    }
  }
}

// Which (n-block, m-block) a thread block works on.  Blocks go to the 8 XCDs round-robin by
// their linear index, and each XCD has its own L2: the m-blocks that share an n-block's weight
// tiles should meet in one L2.  gridDim.x a multiple of 8 gives that by itself.  Otherwise the
// linear index is first turned into "XCD-major" order (all blocks of XCD 0, then XCD 1, ...)
// and m runs fastest in that order, so an n-block's m-blocks are neighbours on one XCD.
__device__ __forceinline__ void tiled_block_xy(int& bx, int& by) {
  const int gx = gridDim.x, gy = gridDim.y, nb = gx * gy;
  bx = blockIdx.x; by = blockIdx.y;
  if ((gx & 7) != 0) {
    const int lin = blockIdx.y * gx + blockIdx.x, xcd = lin & 7;
    // blocks before this one in XCD-major order: those of the lower XCDs, then its own earlier ones
    const int j = xcd * (nb >> 3) + min(xcd, nb & 7) + (lin >> 3);
    bx = j / gy; by = j - bx * gy;
  }
}

// ---------------------------------------------------------------------------------------------
// tiled, 4 waves (2x2): wave tile = WTM x WTN fragments, K step 32.  Operands are double-buffered
// in LDS; global loads run through four register sets, four k-steps ahead.  This variant is the
// faster one for block tiles up to 192 x 192 (one wave per SIMD, nothing to overlap with).
// grid = (ceil(n-tiles / (2*WTN)), ceil(m-tiles / (2*WTM)), k splits)
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
        af_[j] = v4_as_bf16x8(lds[STAGE][wm * WTM + j][lane]);                      \
    _Pragma("unroll") for (int i = 0; i < WTN; ++i)                                 \
        wf_[i] = v4_as_bf16x8(lds[STAGE][BMT + wn * WTN + i][lane]);                \
    _Pragma("unroll") for (int i = 0; i < WTN; ++i)                                 \
      _Pragma("unroll") for (int j = 0; j < WTM; ++j)                               \
        acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf_[i], af_[j], acc[i][j], 0, 0, 0); \
  }

template <int EPI, int WTM, int WTN, bool WS>
__global__ __launch_bounds__(256) void gemm_bf16_tiled4_kernel(const u32x4* __restrict__ Ap,
                                                              const u32x4* __restrict__ Wp,
                                                              int total_nt, int KB_all, int MT,
                                                              GemmEpi e) {
  constexpr int BMT = 2 * WTM, BNT = 2 * WTN, NF = BMT + BNT;  // fragments per k-step
  constexpr int LF = (NF + 3) / 4;                             // fragments loaded per wave
  __shared__ u32x4 lds[2][NF][64];
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  int bx, by;
  tiled_block_xy(bx, by);
  const int mt0 = by * BMT, nt0 = bx * BNT;
  const int wm = wave >> 1, wn = wave & 1;
  // blockIdx.z picks one of gridDim.z contiguous K ranges (EPI_PARTIAL; otherwise gridDim.z = 1)
  const int kb_first = (int)(((long)blockIdx.z * KB_all) / gridDim.z);
  const int KB = (int)(((long)(blockIdx.z + 1) * KB_all) / gridDim.z) - kb_first;

  // Fragment f of the block (0..BMT-1 activations, BMT.. weights) is loaded by wave f % 4.
  // A fragment outside the matrix streams fragment 0 instead (valid memory); what it produces
  // lands in rows / columns that are never stored.
  const u32x4* src[LF];
  size_t stride[LF];  // u32x4 per k-step
#pragma unroll
  for (int i = 0; i < LF; ++i) {
    int f = wave + 4 * i;
    src[i] = Ap + lane;
    stride[i] = (size_t)MT * 64;
    if (f < BMT) {
      int mt = mt0 + f;
      if (mt < MT) src[i] = Ap + (size_t)mt * 64 + lane;
    } else if (f < NF) {
      int nt = nt0 + (f - BMT);
      if (nt < total_nt) {
        src[i] = Wp + packed_w_frag(nt, 0, KB_all, e.w_grp) * 64 + lane;
        stride[i] = (size_t)e.w_grp * 64;
      }
    }
    src[i] += (size_t)kb_first * stride[i];
  }

  f32x4 acc[WTN][WTM];
#pragma unroll
  for (int i = 0; i < WTN; ++i)
#pragma unroll
    for (int j = 0; j < WTM; ++j) acc[i][j] = (f32x4){0.f, 0.f, 0.f, 0.f};

  // prologue: k-step 0 into LDS stage 0, k-steps 1..4 in flight in four register sets (the L2
  // delivers by Little's law: bytes in flight / latency, so the sets are what buys bandwidth)
  u32x4 r0[LF], r1[LF], r2[LF], r3[LF];
  EC_TILED_GLOAD(r0, 0)
  EC_TILED_LSTORE(r0, 0)
  EC_TILED_GLOAD(r0, 1)
  EC_TILED_GLOAD(r1, 2)
  EC_TILED_GLOAD(r2, 3)
  EC_TILED_GLOAD(r3, 4)
  __syncthreads();
  // iteration kb: compute stage kb&1; the register set holding k-step kb+1 goes to stage
  // (kb+1)&1 and is reloaded with k-step kb+5
#define EC_TILED_STEP(REGS, KBV, STAGE)       \
  if ((KBV) < KB) {                           \
    EC_TILED_COMPUTE(STAGE)                   \
    EC_TILED_LSTORE(REGS, (STAGE) ^ 1)        \
    EC_TILED_GLOAD(REGS, (KBV) + 5)           \
  }                                           \
  __syncthreads();
  for (int kb = 0; kb < KB; kb += 4) {
    EC_TILED_STEP(r0, kb, 0)
    EC_TILED_STEP(r1, kb + 1, 1)
    EC_TILED_STEP(r2, kb + 2, 0)
    EC_TILED_STEP(r3, kb + 3, 1)
  }
#undef EC_TILED_STEP

  if constexpr (WS) scale_acc<WTM, WTN>(e, acc, nt0 + wn * WTN, total_nt, lane);
  tiled_epilogue<EPI, WTM, WTN>(e, acc, mt0 + wm * WTM, nt0 + wn * WTN, total_nt, lane, blockIdx.z);
}
#undef EC_TILED_GLOAD
#undef EC_TILED_LSTORE
#undef EC_TILED_COMPUTE

template <int EPI, int WTM, int WTN, bool WS>
static void launch_tiled4_t(const bf16_t* Ap, int MT, const bf16_t* Wp, int total_nt, int KB,
                           const GemmEpi& e, hipStream_t s, int ksplit) {
  dim3 grid((total_nt + 2 * WTN - 1) / (2 * WTN), (MT + 2 * WTM - 1) / (2 * WTM), ksplit);
  gemm_bf16_tiled4_kernel<EPI, WTM, WTN, WS><<<grid, 256, 0, s>>>((const u32x4*)Ap, (const u32x4*)Wp,
                                                                 total_nt, KB, MT, e);
}

// ---------------------------------------------------------------------------------------------
// tiled, 8 waves (WM x WN): wave tile = WTM x WTN fragments of 16 rows (activations x weights),
// K step 32.  Operand fragments go from global memory straight into LDS (global_load_lds_dwordx4:
// lane l's 16 bytes land at base + 16 l, so a 1 KiB fragment keeps its order), NSTAGE stages deep,
// no staging registers; one barrier per k-step.
// grid = (ceil(n-tiles / (WN*WTN)), ceil(m-tiles / (WM*WTM)), k splits)
// ---------------------------------------------------------------------------------------------
template <int N> __device__ __forceinline__ void wait_vmcnt() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// (With the plain store epilogue of a K split, blocks of at most 192 x 192 fit two to a CU: the
// register count is pinned to the 128 VGPRs that allows.  The fused epilogues need more.)
// PIPE: the fragments of k-step k+1 are read from LDS into a second register set while the
// MFMAs of k-step k run.  Without it every k-step is a burst of LDS reads (all waves at once,
// right after the barrier, matrix cores idle) followed by a burst of MFMAs.
template <int EPI, int WM, int WN, int WTM, int WTN, bool PIPE>
constexpr int tiled8_waves_per_eu() {
  // four-wave blocks: two to a CU (256 registers each) unless the read-ahead needs more
  return WM * WN == 4 ? (PIPE ? 1 : 2) : (EPI == EPI_PARTIAL && WTM * WTN <= 18 ? 4 : 2);
}
template <int EPI, int WM, int WN, int WTM, int WTN, int NSTAGE, bool PIPE, bool WS>
__global__ __launch_bounds__(WM * WN * 64)
__attribute__((amdgpu_waves_per_eu(tiled8_waves_per_eu<EPI, WM, WN, WTM, WTN, PIPE>(),
                                   tiled8_waves_per_eu<EPI, WM, WN, WTM, WTN, PIPE>())))
void gemm_bf16_tiled8_kernel(
    const u32x4* __restrict__ Ap, const u32x4* __restrict__ Wp, int total_nt, int KB_all, int MT,
    GemmEpi e) {
  constexpr int NW = WM * WN, BMT = WM * WTM, BNT = WN * WTN, NF = BMT + BNT;
  constexpr int LF = (NF + NW - 1) / NW;  // loads per wave and stage (all waves issue LF)
  static_assert(LF * NSTAGE <= 63, "vmcnt counts at most 63 outstanding loads");
  extern __shared__ u32x4 lds[];  // [NSTAGE][NF][64] + one dump fragment
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  int bx, by;
  tiled_block_xy(bx, by);
  const int mt0 = by * BMT, nt0 = bx * BNT;
  const int wm = wave / WN, wn = wave % WN;
  // blockIdx.z picks one of gridDim.z contiguous K ranges (EPI_PARTIAL; otherwise gridDim.z = 1)
  const int kb_first = (int)(((long)blockIdx.z * KB_all) / gridDim.z);
  const int KB = (int)(((long)(blockIdx.z + 1) * KB_all) / gridDim.z) - kb_first;

  // Fragment f of the block (0..BMT-1 activations, BMT.. weights) is loaded by wave f % NW.
  // A fragment outside the matrix streams fragment 0 instead (valid memory); what it produces
  // lands in rows / columns that are never stored.  Slots past NF go to the dump fragment, so
  // that every wave has the same number of loads in flight (the vmcnt arithmetic needs that).
  const u32x4* src[LF];
  size_t stride[LF];  // u32x4 per k-step
  int dst[LF];        // fragment slot within a stage, or -1 = dump
#pragma unroll
  for (int i = 0; i < LF; ++i) {
    int f = wave + NW * i;
    src[i] = Ap + lane;
    stride[i] = (size_t)MT * 64;
    dst[i] = f < NF ? f : -1;
    if (f < BMT) {
      int mt = mt0 + f;
      if (mt < MT) src[i] = Ap + (size_t)mt * 64 + lane;
    } else if (f < NF) {
      int nt = nt0 + (f - BMT);
      if (nt < total_nt) {
        src[i] = Wp + packed_w_frag(nt, 0, KB_all, e.w_grp) * 64 + lane;
        stride[i] = (size_t)e.w_grp * 64;
      }
    }
    src[i] += (size_t)kb_first * stride[i];
  }
  auto issue = [&](int kb) {  // k-step kb (clamped) -> stage kb % NSTAGE
    const int kbc = min(kb, KB - 1), stage = kb % NSTAGE;
#pragma unroll
    for (int i = 0; i < LF; ++i) {
      u32x4* slot = dst[i] >= 0 ? lds + ((size_t)stage * NF + dst[i]) * 64
                                : lds + (size_t)NSTAGE * NF * 64;
      __builtin_amdgcn_global_load_lds(
          (const void __attribute__((address_space(1)))*)(src[i] + (size_t)kbc * stride[i]),
          (void __attribute__((address_space(3)))*)slot, 16, 0, 0);
    }
  };

  f32x4 acc[WTN][WTM];
#pragma unroll
  for (int i = 0; i < WTN; ++i)
#pragma unroll
    for (int j = 0; j < WTM; ++j) acc[i][j] = (f32x4){0.f, 0.f, 0.f, 0.f};

  if constexpr (!PIPE) {
#pragma unroll
    for (int sgl = 0; sgl < NSTAGE - 1; ++sgl) issue(sgl);
    for (int kb = 0; kb < KB; ++kb) {
      // this wave's loads of k-step kb have landed once at most LF*(NSTAGE-2) newer ones remain
      wait_vmcnt<LF*(NSTAGE - 2)>();
      block_barrier_nofence();  // ... and so have everyone else's; the stage read last iteration is free
      issue(kb + NSTAGE - 1);
      const u32x4* st = lds + (size_t)(kb % NSTAGE) * NF * 64;
      bf16x8 af[WTM], wf[WTN];
#pragma unroll
      for (int j = 0; j < WTM; ++j) af[j] = v4_as_bf16x8(st[(wm * WTM + j) * 64 + lane]);
#pragma unroll
      for (int i = 0; i < WTN; ++i) wf[i] = v4_as_bf16x8(st[(BMT + wn * WTN + i) * 64 + lane]);
#pragma unroll
      for (int i = 0; i < WTN; ++i)
#pragma unroll
        for (int j = 0; j < WTM; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[i], af[j], acc[i][j], 0, 0, 0);
    }
  } else {
    // All NSTAGE slots are kept in flight.  Step k: this wave has finished reading slot k (its
    // fragments sit in one register set) and its loads of k-step k+1 have landed; after the
    // barrier that holds for every wave, so slot k is refilled with k-step k + NSTAGE, the
    // fragments of k+1 go to the other register set, and the MFMAs of k run over those reads.
    bf16x8 afa[WTM], wfa[WTN], afb[WTM], wfb[WTN];
#define EC_T8_READ(AF, WF, KB_)                                                              \
  {                                                                                          \
    const u32x4* st_ = lds + (size_t)((KB_) % NSTAGE) * NF * 64;                             \
    _Pragma("unroll") for (int j = 0; j < WTM; ++j)                                          \
        AF[j] = v4_as_bf16x8(st_[(wm * WTM + j) * 64 + lane]);                               \
    _Pragma("unroll") for (int i = 0; i < WTN; ++i)                                          \
        WF[i] = v4_as_bf16x8(st_[(BMT + wn * WTN + i) * 64 + lane]);                         \
  }
#define EC_T8_MMA(AF, WF)                                                                    \
  _Pragma("unroll") for (int i = 0; i < WTN; ++i)                                            \
    _Pragma("unroll") for (int j = 0; j < WTM; ++j)                                          \
      acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(WF[i], AF[j], acc[i][j], 0, 0, 0);
#define EC_T8_STEP(AF, WF, AFN, WFN, KB_)                                                    \
  {                                                                                          \
    wait_vmcnt<LF*(NSTAGE - 2)>();  /* own loads of KB_+1 have landed */                     \
    block_barrier_nofence();        /* and slot KB_ is in registers, for every wave */       \
    issue((KB_) + NSTAGE);                                                                   \
    EC_T8_READ(AFN, WFN, (KB_) + 1)                                                          \
    __builtin_amdgcn_sched_barrier(0);                                                       \
    EC_T8_MMA(AF, WF)                                                                        \
    __builtin_amdgcn_sched_barrier(0);                                                       \
  }
#pragma unroll
    for (int sgl = 0; sgl < NSTAGE; ++sgl) issue(sgl);
    wait_vmcnt<LF*(NSTAGE - 1)>();
    block_barrier_nofence();
    EC_T8_READ(afa, wfa, 0)
    for (int kb = 0; kb < KB; kb += 2) {
      EC_T8_STEP(afa, wfa, afb, wfb, kb)
      // an odd trip count runs one surplus step on a clamped (repeated) k-step: its activation
      // fragments are zeroed so that it adds nothing
      if (kb + 1 >= KB) {
#pragma unroll
        for (int j = 0; j < WTM; ++j) afb[j] = v4_as_bf16x8((u32x4){0u, 0u, 0u, 0u});
      }
      EC_T8_STEP(afb, wfb, afa, wfa, kb + 1)
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#undef EC_T8_STEP
#undef EC_T8_MMA
#undef EC_T8_READ
  }
  wait_vmcnt<0>();  // drain the clamped tail loads before the LDS goes away

  if constexpr (WS) scale_acc<WTM, WTN>(e, acc, nt0 + wn * WTN, total_nt, lane);
  // (the read-ahead QKV epilogue needs registers that only the smaller wave tiles leave free)
  tiled_epilogue<EPI, WTM, WTN, (WTM * WTN <= 18)>(e, acc, mt0 + wm * WTM, nt0 + wn * WTN, total_nt, lane,
                                                   blockIdx.z);
}

template <int EPI, bool WS, int WM, int WN, int WTM, int WTN, int NSTAGE, bool PIPE = false>
static void launch_tiled8_t(const bf16_t* Ap, int MT, const bf16_t* Wp, int total_nt, int KB,
                            const GemmEpi& e, hipStream_t s, int ksplit) {
  constexpr int NF = WM * WTM + WN * WTN;
  const size_t smem = ((size_t)NSTAGE * NF + 1) * 1024;
  auto kern = gemm_bf16_tiled8_kernel<EPI, WM, WN, WTM, WTN, NSTAGE, PIPE, WS>;
  static bool attr_set = false;
  if (!attr_set && smem > 48 * 1024) {
    (void)hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                              (int)smem);
    attr_set = true;
  }
  dim3 grid((total_nt + WN * WTN - 1) / (WN * WTN), (MT + WM * WTM - 1) / (WM * WTM), ksplit);
  kern<<<grid, WM * WN * 64, smem, s>>>((const u32x4*)Ap, (const u32x4*)Wp, total_nt, KB, MT, e);
}

// Second half of a K-split residual GEMM: h += sum over the splits (fixed order), then what
// EPI_RESID does: next operand bf16(h * gain) and the row's sum of squares.
// grid (ceil(d / 1024), M), 256 threads, 4 columns per thread.
__global__ __launch_bounds__(256) void resid_finish_kernel(GemmEpi e, int ksplit) {
  __shared__ float red[4];
  const int m = blockIdx.y, n = (blockIdx.x * 256 + threadIdx.x) * 4;
  float part = 0.f;
  if (n < e.d) {
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int z = 0; z < ksplit; ++z) {
      float4 p = *(const float4*)(e.partial + ((size_t)z * e.M + m) * e.d + n);
      v.x += p.x; v.y += p.y; v.z += p.z; v.w += p.w;
    }
    part = epi_resid(e, m, n >> 4, (n >> 2) & 3, (f32x4){v.x, v.y, v.z, v.w});
  }
  part = block_sum<4>(part, red);
  if (threadIdx.x == 0) {
    unsigned long long fx = sumsq_to_fixed<58>(part);
    if (fx) atomicAdd((unsigned long long*)(e.sumsq_out + (size_t)(blockIdx.x & (kSumSlots - 1)) * e.sum_stride + m), fx);
  }
}

// Block shapes of the tiled kernels (rows x weight rows) and what one k-step costs on MI355X
// with all 256 CUs busy (us, measured): alone on its CU, and - for the shapes small enough that
// two blocks share a CU's LDS and registers - per k-step of such a pair.
//   8 waves: 0: 192 x 384   1: 192 x 256   2: 192 x 192   3: 192 x 128
//   4 waves: 4: 192 x 192   5: 192 x 128   6: 128 x 128   7: 96 x 128
// Two waves per SIMD overlap one wave's LDS reads and barrier waits with the other's MFMAs, four
// (two 8-wave blocks) do so better still.  The wider the block the fewer operand bytes per flop
// cross L2 and LDS.  A grid that does not fill the 256 CUs in whole rounds wastes the
// remainder, so narrow outputs (N = d_model) are also split along K into partial products that
// a small second kernel sums.  Two blocks to a CU need the 128-register kernels, which only the
// plain store epilogue of a K split fits.
struct TilePick { int tile, ksplit; };
constexpr int kNumTiles = 8;
static const int kTileM[kNumTiles] = {12, 12, 12, 12, 12, 12, 8, 6};
static const int kTileN[kNumTiles] = {24, 16, 12, 8, 12, 8, 8, 8};
static const float kTileUsAlone[kNumTiles] = {0.98f, 0.71f, 0.54f, 0.46f, 0.64f, 0.55f, 0.53f, 0.41f};
static const float kTileUsPair[kNumTiles] = {0.f, 0.f, 0.90f, 0.75f, 0.f, 0.f, 0.f, 0.f};

static TilePick pick_tile(int MT, int total_nt, int KB, int max_ksplit, int M, int N) {
  TilePick best{1, 1};
  float best_t = 1e30f;
  for (int i = 0; i < kNumTiles; ++i) {
    long gm = (MT + kTileM[i] - 1) / kTileM[i], gn = (total_nt + kTileN[i] - 1) / kTileN[i];
    for (int ks = 1; ks <= max_ksplit; ++ks) {
      const long blocks = gm * gn * ks, per_cu = (blocks + 255) / 256;
      const float ksteps = (float)((KB + ks - 1) / ks);
      const long pairs = (kTileUsPair[i] > 0.f && ks > 1) ? per_cu / 2 : 0;
      const long singles = per_cu - 2 * pairs;
      float t = ksteps * (pairs * kTileUsPair[i] + singles * kTileUsAlone[i]) + 5.0f * (pairs + singles);
      if (ks > 1) t += 2.5f + (float)M * N * (ks + 4) * 4.0f / 5.0e6f;  // finish kernel
      if (t < best_t) { best_t = t; best = TilePick{i, ks}; }
    }
  }
  return best;
}

// WS: the matrix carries per-row scales (it came as e4m3 codes): a variant of its own, so that
// the kernels of plain bf16 models are compiled exactly as they were tuned
template <int EPI, bool WS>
static void launch_tiled_pick_ws(const bf16_t* Ap, int MT, const bf16_t* Wp, int total_nt, int KB,
                                 const GemmEpi& e, hipStream_t s, int tile, int ksplit) {
  switch (tile) {
    case 0: launch_tiled8_t<EPI, WS, 2, 4, 6, 6, 3>(Ap, MT, Wp, total_nt, KB, e, s, ksplit); break;
    case 1: launch_tiled8_t<EPI, WS, 2, 4, 6, 4, 3, true>(Ap, MT, Wp, total_nt, KB, e, s, ksplit); break;
    case 2: launch_tiled8_t<EPI, WS, 2, 4, 6, 3, 3>(Ap, MT, Wp, total_nt, KB, e, s, ksplit); break;
    case 3: launch_tiled8_t<EPI, WS, 2, 4, 6, 2, 3>(Ap, MT, Wp, total_nt, KB, e, s, ksplit); break;
    case 4: launch_tiled4_t<EPI, 6, 6, WS>(Ap, MT, Wp, total_nt, KB, e, s, ksplit); break;
    case 5: launch_tiled4_t<EPI, 6, 4, WS>(Ap, MT, Wp, total_nt, KB, e, s, ksplit); break;
    case 6: launch_tiled4_t<EPI, 4, 4, WS>(Ap, MT, Wp, total_nt, KB, e, s, ksplit); break;
    default: launch_tiled4_t<EPI, 3, 4, WS>(Ap, MT, Wp, total_nt, KB, e, s, ksplit); break;
  }
}

template <int EPI>
static void launch_tiled_pick(const bf16_t* Ap, int MT, const bf16_t* Wp, int total_nt, int KB,
                              const GemmEpi& e, hipStream_t s, int tile, int ksplit) {
  if (e.wscale) launch_tiled_pick_ws<EPI, true>(Ap, MT, Wp, total_nt, KB, e, s, tile, ksplit);
  else launch_tiled_pick_ws<EPI, false>(Ap, MT, Wp, total_nt, KB, e, s, tile, ksplit);
}

template <int EPI>
static void launch_epi(const bf16_t* Ap, int M_src, const bf16_t* Wp, const void* Wq, int N, int K,
                       const GemmEpi& e, hipStream_t s) {
  const int total_nt = N / 16, KB = K / 32, MT = (e.M + 15) / 16, MT_src = (M_src + 15) / 16;
  if (Wq && MT <= 6 && !(EPI == EPI_LOGITS && MT > 4)) {  // weight streaming from e4m3 codes
    switch (MT) {
      case 1: launch_skinny_mt_w8<EPI, 1>(Ap, MT_src, Wq, total_nt, K / 64, e, s); break;
      case 2: launch_skinny_mt_w8<EPI, 2>(Ap, MT_src, Wq, total_nt, K / 64, e, s); break;
      case 3: launch_skinny_mt_w8<EPI, 3>(Ap, MT_src, Wq, total_nt, K / 64, e, s); break;
      case 4: launch_skinny_mt_w8<EPI, 4>(Ap, MT_src, Wq, total_nt, K / 64, e, s); break;
      case 5: launch_skinny_mt_w8<EPI, 5>(Ap, MT_src, Wq, total_nt, K / 64, e, s); break;
      default: launch_skinny_mt_w8<EPI, 6>(Ap, MT_src, Wq, total_nt, K / 64, e, s); break;
    }
    return;
  }
  // Up to 96 rows (a block of 32 plus the paper's default budget of 64 recent tokens) the GEMMs
  // are weight-streaming: 3.7 ms a step at 64 rows, 4.5 ms at 96, against 7.8 ms through the
  // tiled kernels.
  if (MT <= 6 && !(EPI == EPI_LOGITS && MT > 4)) {  // (gathered LM-head rows: 64 at most)
    switch (MT) {
      case 1: launch_skinny_mt<EPI, 1>(Ap, MT_src, Wp, total_nt, KB, e, s); break;
      case 2: launch_skinny_mt<EPI, 2>(Ap, MT_src, Wp, total_nt, KB, e, s); break;
      case 3: launch_skinny_mt<EPI, 3>(Ap, MT_src, Wp, total_nt, KB, e, s); break;
      case 4: launch_skinny_mt<EPI, 4>(Ap, MT_src, Wp, total_nt, KB, e, s); break;
      case 5: launch_skinny_mt<EPI, 5>(Ap, MT_src, Wp, total_nt, KB, e, s); break;
      default: launch_skinny_mt<EPI, 6>(Ap, MT_src, Wp, total_nt, KB, e, s); break;
    }
  } else {
    // the tiled kernel reads its activation rows in place (no gather) and walks every m-tile of
    // the buffer; rows from e.M on are dropped in the epilogue
    const int max_ks = (EPI == EPI_RESID && e.partial) ? e.max_ksplit : 1;
    TilePick tp = pick_tile(MT_src, total_nt, KB, max_ks, e.M, N);
    if (tp.ksplit > 1) {
      launch_tiled_pick<EPI_PARTIAL>(Ap, MT_src, Wp, total_nt, KB, e, s, tp.tile, tp.ksplit);
      resid_finish_kernel<<<dim3((N + 1023) / 1024, e.M), 256, 0, s>>>(e, tp.ksplit);
    } else {
      launch_tiled_pick<EPI>(Ap, MT_src, Wp, total_nt, KB, e, s, tp.tile, 1);
    }
  }
}

void launch_gemm_bf16(int epi, const bf16_t* Ap, int M_src, const bf16_t* Wp, const void* Wq,
                      int N, int K, const GemmEpi& e, hipStream_t s) {
  if (e.M <= 0) return;
  switch (epi) {
    case EPI_QKV: launch_epi<EPI_QKV>(Ap, M_src, Wp, Wq, N, K, e, s); break;
    case EPI_RESID: launch_epi<EPI_RESID>(Ap, M_src, Wp, Wq, N, K, e, s); break;
    case EPI_SWIGLU: launch_epi<EPI_SWIGLU>(Ap, M_src, Wp, Wq, N, K, e, s); break;
    default:
      // Up to 64 rows the skinny kernel gathers the rows row_sel names out of Ap itself.  More
      // rows go through the tiled kernels, which read their rows in place: the caller hands
      // over the gathered rows then (row_sel still names the rows whose 1/rms applies).
      launch_epi<EPI_LOGITS>(Ap, M_src, Wp, Wq, N, K, e, s);
      break;
  }
}

}  // namespace ec
