// Device helpers shared by the HIP kernels: bfloat16 conversion, wave / block reductions,
// and the index maps of the two re-tiled ("packed") bf16 layouts.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ec {

typedef uint16_t bf16_t;  // raw bfloat16 bit pattern
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kWave = 64;

__device__ __forceinline__ float bf16_to_f32(bf16_t b) {
  return __uint_as_float(((uint32_t)b) << 16);
}
// round to nearest, ties to even; NaN stays NaN
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}

// two floats -> packed bf16 pair (low half = a), one v_cvt_pk_bf16_f32 on gfx950 (RNE)
typedef __bf16 bf16x2_hw __attribute__((ext_vector_type(2)));
typedef float f32x2_hw __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack2_bf16(float a, float b) {
  f32x2_hw v = {a, b};
  union { bf16x2_hw h; uint32_t u; } c;
  c.h = __builtin_convertvector(v, bf16x2_hw);
  return c.u;
}

// Block barrier without the memory fence of __syncthreads().  That fence waits for every
// outstanding global->LDS load of the wave (vmcnt(0)), which serialises a ring of such loads;
// here the caller waits for exactly the loads it needs (s_waitcnt vmcnt(N)) beforehand.  The
// wave's own LDS reads and writes are complete on return (lgkmcnt(0)).
__device__ __forceinline__ void block_barrier_nofence() {
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// value held by the lane 32 positions away (one v_permlane32_swap, no LDS traffic)
__device__ __forceinline__ float other_half(float x) {
  const unsigned u = __float_as_uint(x);
  auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);  // {[lo,lo], [hi,hi]} of u
  return __uint_as_float((threadIdx.x & 32) ? r[0] : r[1]);
}

// value held by the lane 16 positions away within its 32-lane half, lane ^ 16 (one
// v_permlane16_swap: rows of 16 lanes; with both operands x it returns {[r0,r0,r2,r2],
// [r1,r1,r3,r3]})
__device__ __forceinline__ float other_row(float x) {
  const unsigned u = __float_as_uint(x);
  auto r = __builtin_amdgcn_permlane16_swap(u, u, false, false);
  return __uint_as_float((threadIdx.x & 16) ? r[0] : r[1]);
}

template <typename T> __device__ __forceinline__ float load_f32(const T* p);
template <> __device__ __forceinline__ float load_f32<float>(const float* p) { return *p; }
template <> __device__ __forceinline__ float load_f32<bf16_t>(const bf16_t* p) { return bf16_to_f32(*p); }
template <typename T> __device__ __forceinline__ void store_f32(T* p, float v);
template <> __device__ __forceinline__ void store_f32<float>(float* p, float v) { *p = v; }
template <> __device__ __forceinline__ void store_f32<bf16_t>(bf16_t* p, float v) { *p = f32_to_bf16(v); }

// ---- packed bf16 operand layouts -------------------------------------------------------------
// A 16 x 32 bf16 fragment is stored as 64 lanes x 8 elements = 1 KiB, lane = g*16 + r holding
// row r, columns g*8 .. g*8+7: exactly what lane `lane` feeds to v_mfma_f32_16x16x32_bf16.
//
// Activations  A[M, K]:  fragment (kb, mt) at ((kb * MT + mt) * 512) elements, MT = ceil(M/16).
// Weights      W[N, K]:  fragment (nt, kb) at ((nt * KB + kb) * 512) elements, KB = K/32.
__device__ __forceinline__ size_t packed_act_index(int m, int k, int MT) {
  int kb = k >> 5, g = (k >> 3) & 3, e = k & 7, mt = m >> 4, r = m & 15;
  return ((size_t)(kb * MT + mt) * 64 + g * 16 + r) * 8 + e;
}
// Weight fragments are stored in groups of `grp` tiles: [tile / grp][kb][tile % grp], so that a
// block that owns a whole group reads grp KiB of contiguous memory per k-step.
__device__ __forceinline__ size_t packed_w_frag(int nt, int kb, int KB, int grp) {
  return ((size_t)(nt / grp) * KB + kb) * grp + (nt % grp);
}
__device__ __forceinline__ size_t packed_w_index(int n, int k, int KB, int grp) {
  int kb = k >> 5, g = (k >> 3) & 3, e = k & 7, nt = n >> 4, r = n & 15;
  return (packed_w_frag(nt, kb, KB, grp) * 64 + g * 16 + r) * 8 + e;
}

// e4m3 weights W[N, K] (one byte each): a fragment PAIR covers 16 rows x 64 k in 1 KiB; lane
// g*16 + r holds row r, its first 8 bytes k = kb2*64 + g*8 .. +7 (the MFMA operand of k-block
// 2*kb2) and its last 8 bytes k = kb2*64 + 32 + g*8 .. +7 (k-block 2*kb2 + 1).  Pairs are ordered
// like the bf16 fragments, with KB2 = K/64 steps.  Returns a byte index.
__device__ __forceinline__ size_t packed_w8_index(int n, int k, int KB2, int grp) {
  int kb2 = k >> 6, half = (k >> 5) & 1, g = (k >> 3) & 3, e = k & 7, nt = n >> 4, r = n & 15;
  return (packed_w_frag(nt, kb2, KB2, grp) * 64 + g * 16 + r) * 16 + half * 8 + e;
}

// ---- packed bf16 KV cache (one kv head = one contiguous slab of Tpad * HD elements) -----------
// K: fragments are MFMA "A" operands of S^T = K Q^T.  A 32-key block holds two 16-row tiles;
//    tile t, row i is key (i/4)*8 + t*4 + (i%4) of the block, so that after the two tiles'
//    MFMAs a lane owns 8 CONSECUTIVE keys - the order in which P feeds the P.V MFMA.
//    fragment ((kb32*2 + t) * HD/32 + hb), lane g*16+i holds hd columns hb*32 + g*8 .. +7.
// V: stored transposed; fragments are "A" operands of O^T = V^T P^T.
//    fragment (ht * Tpad/32 + kb32), lane g*16+j holds hd row ht*16+j, keys kb32*32 + g*8 .. +7.
__device__ __forceinline__ size_t kcache_index(int key, int c, int HD) {
  int kb = key >> 5, w = key & 31, i = (w >> 3) * 4 + (w & 3), t = (w >> 2) & 1;
  int hb = c >> 5, g = (c >> 3) & 3, e = c & 7;
  return (((size_t)(kb * 2 + t) * (HD >> 5) + hb) * 64 + g * 16 + i) * 8 + e;
}
__device__ __forceinline__ size_t vcache_index(int key, int c, int Tpad) {
  int kb = key >> 5, g = (key >> 3) & 3, e = key & 7, ht = c >> 4, j = c & 15;
  return (((size_t)ht * (Tpad >> 5) + kb) * 64 + g * 16 + j) * 8 + e;
}

// ---- fixed-point row sums of squares ----------------------------------------------------------
// A row's sum of squares is accumulated by many blocks with 64-bit integer atomics (integer
// addition is associative, so the total does not depend on the order).  Format 44.20: one unit
// is 2^-20 (a contribution is rounded to it: absolute error below 5e-7).  A contribution
// saturates at 2^CAP units, CAP chosen by the caller so that all contributions of a row cannot
// wrap the 64-bit total: 52 where up to 2^10 blocks add to a row (4.3e9 each), 58 for the few
// adds of the K-split finish, 62 for the prologue's single store.  Rows whose sum of squares
// exceeds about 4e12 therefore saturate (their 1/rms comes out too large) instead of wrapping.
constexpr double kSumsqUnit = 1048576.0;  // 2^20
template <int CAP = 52>
__device__ __forceinline__ unsigned long long sumsq_to_fixed(float part) {
  constexpr unsigned long long cap = 1ull << CAP;
  const double v = (double)part * kSumsqUnit + 0.5;
  return v < (double)cap ? (unsigned long long)v : cap;  // (a NaN saturates too)
}
__device__ __forceinline__ double sumsq_from_fixed(unsigned long long fx) {
  return (double)fx * (1.0 / kSumsqUnit);
}

// ---- reductions (fixed order => deterministic) -----------------------------------------------
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
// Sum over a block of NW waves; every thread gets the result.  `scratch` holds NW floats.
template <int NW> __device__ __forceinline__ float block_sum(float v, float* scratch) {
  v = wave_sum(v);
  int w = threadIdx.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) scratch[w] = v;
  __syncthreads();
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < NW; ++i) s += scratch[i];
  return s;
}
template <int NW> __device__ __forceinline__ float block_max(float v, float* scratch) {
  v = wave_max(v);
  int w = threadIdx.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) scratch[w] = v;
  __syncthreads();
  float s = scratch[0];
#pragma unroll
  for (int i = 1; i < NW; ++i) s = fmaxf(s, scratch[i]);
  return s;
}

}  // namespace ec
