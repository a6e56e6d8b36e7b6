// bf16 non-causal attention on MFMA with an online softmax, for the packed KV cache.
//
// For one kv head the "queries" are all (row, head-in-group) pairs, so grouped-query attention
// reads each K/V fragment once for all heads of the group.  Per 32-key chunk and 16-query tile:
//   S^T[keys x queries] = K . Q^T          (2 key tiles x HD/32 MFMAs, K fragments straight from
//                                            the cache, Q fragments held in registers)
//   online softmax down the key axis        (a lane owns 8 consecutive keys of one query; the
//                                            other 24 are 2 xor-shuffles away)
//   O^T[hd x queries] += V^T . P^T          (HD/16 MFMAs; the lane's 8 probabilities ARE the
//                                            B operand, V^T fragments straight from the cache)
// Nothing is staged in LDS: every operand load is a coalesced 1 KiB fragment.
//
// Two work splits:
//   SPLIT_KEYS  (few query rows, partial step): a block owns QT query tiles of one kv head and
//               its waves stride over the key chunks; the waves' partial (m, l, O) are merged in
//               LDS by a fixed binary tree.
//   !SPLIT_KEYS (many rows, full step): every wave owns QT query tiles and walks all keys.
#include "ec_internal.h"

namespace ec {

__device__ __forceinline__ bf16x8 u4_as_bf16x8(uint4 v) {
  union { uint4 u; bf16x8 b; } c;
  c.u = v;
  return c.b;
}
__device__ __forceinline__ uint32_t pack2_bf16(float a, float b) {
  return (uint32_t)f32_to_bf16(a) | ((uint32_t)f32_to_bf16(b) << 16);
}

template <int HD, int QT, bool SPLIT_KEYS>
__global__ __launch_bounds__(SPLIT_KEYS ? 512 : 256) void attn_mfma_kernel(
    const bf16_t* __restrict__ q, const uint4* __restrict__ kp, const uint4* __restrict__ vp,
    int M, int T, int Tpad, int Hq, int Hkv, float scale_log2e, bf16_t* __restrict__ out,
    int MT) {
  constexpr int HB = HD / 32, HT = HD / 16;
  extern __shared__ float4 lds[];
  // scalar wave index: no MFMA may sit under a condition the compiler could treat as divergent
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int NW = blockDim.x >> 6;
  const int kvh = blockIdx.y, G = Hq / Hkv, nQ = M * G;
  const int nchunks = (T + 31) >> 5, KB32 = Tpad >> 5;
  const int tile0 = SPLIT_KEYS ? blockIdx.x * QT : (blockIdx.x * NW + wave) * QT;
  const int qcol = lane & 15, grp = lane >> 4;
  if constexpr (!SPLIT_KEYS) {
    if (tile0 * 16 >= nQ) return;  // no block-wide barrier on this path
  }

  // ---- Q fragments (B operand): lane (query qcol, group grp) holds 8 hd columns -------------
  bf16x8 qf[QT][HB];
  int qrow[QT], qhead[QT];
#pragma unroll
  for (int t = 0; t < QT; ++t) {
    int qi = (tile0 + t) * 16 + qcol;
    bool valid = qi < nQ;
    qrow[t] = valid ? qi / G : -1;
    qhead[t] = kvh * G + (valid ? qi % G : 0);
#pragma unroll
    for (int hb = 0; hb < HB; ++hb) {
      uint4 v = make_uint4(0, 0, 0, 0);
      if (valid)
        v = *(const uint4*)(q + (size_t)qrow[t] * Hq * HD + qhead[t] * HD + hb * 32 + grp * 8);
      qf[t][hb] = u4_as_bf16x8(v);
    }
  }

  f32x4 acc[QT][HT];
  float m_run[QT], l_run[QT];
#pragma unroll
  for (int t = 0; t < QT; ++t) {
    m_run[t] = -INFINITY;
    l_run[t] = 0.f;
#pragma unroll
    for (int h = 0; h < HT; ++h) acc[t][h] = (f32x4){0.f, 0.f, 0.f, 0.f};
  }

  const uint4* kbase = kp + (size_t)kvh * KB32 * 2 * HB * 64 + lane;
  const uint4* vbase = vp + (size_t)kvh * HT * KB32 * 64 + lane;
  const int c_begin = SPLIT_KEYS ? wave : 0, c_step = SPLIT_KEYS ? NW : 1;
  for (int c = c_begin; c < nchunks; c += c_step) {
    bf16x8 kf[2][HB];
#pragma unroll
    for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
      for (int hb = 0; hb < HB; ++hb)
        kf[t2][hb] = u4_as_bf16x8(kbase[((size_t)(c * 2 + t2) * HB + hb) * 64]);
    bf16x8 vf[HT];
#pragma unroll
    for (int h = 0; h < HT; ++h) vf[h] = u4_as_bf16x8(vbase[((size_t)h * KB32 + c) * 64]);

    const int key0 = c * 32 + grp * 8;  // the lane's 8 consecutive keys
#pragma unroll
    for (int t = 0; t < QT; ++t) {
      f32x4 s[2];
#pragma unroll
      for (int t2 = 0; t2 < 2; ++t2) {
        s[t2] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int hb = 0; hb < HB; ++hb)
          s[t2] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[t2][hb], qf[t][hb], s[t2], 0, 0, 0);
      }
      float sv[8];
      float mx = -INFINITY;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        float v = s[e >> 2][e & 3] * scale_log2e;
        if (key0 + e >= T) v = -INFINITY;  // padding keys of the last chunk
        sv[e] = v;
        mx = fmaxf(mx, v);
      }
      mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      float m_new = fmaxf(m_run[t], mx);       // finite: every chunk has at least one real key
      float alpha = exp2f(m_run[t] - m_new);   // 0 on the first chunk
      float rs = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        sv[e] = exp2f(sv[e] - m_new);
        rs += sv[e];
      }
      rs += __shfl_xor(rs, 16, 64);
      rs += __shfl_xor(rs, 32, 64);
      l_run[t] = l_run[t] * alpha + rs;
      m_run[t] = m_new;
      uint4 pu = make_uint4(pack2_bf16(sv[0], sv[1]), pack2_bf16(sv[2], sv[3]),
                            pack2_bf16(sv[4], sv[5]), pack2_bf16(sv[6], sv[7]));
      bf16x8 pf = u4_as_bf16x8(pu);
#pragma unroll
      for (int h = 0; h < HT; ++h) {
        f32x4 a = acc[t][h];
        a[0] *= alpha; a[1] *= alpha; a[2] *= alpha; a[3] *= alpha;
        acc[t][h] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[h], pf, a, 0, 0, 0);
      }
    }
  }

  // ---- merge the waves' partial results (fixed binary tree over wave ids) --------------------
  if constexpr (SPLIT_KEYS) {
    constexpr int SLOT = QT * HT * 64 + QT * 32;  // float4 per slot: O tiles + (m,l) pairs
    for (int half = NW >> 1; half >= 1; half >>= 1) {
      if (wave >= half && wave < 2 * half) {
        float4* slot = lds + (size_t)(wave - half) * SLOT;
#pragma unroll
        for (int t = 0; t < QT; ++t) {
#pragma unroll
          for (int h = 0; h < HT; ++h) {
            f32x4 a = acc[t][h];
            slot[(t * HT + h) * 64 + lane] = make_float4(a[0], a[1], a[2], a[3]);
          }
          ((float2*)(slot + QT * HT * 64))[t * 64 + lane] = make_float2(m_run[t], l_run[t]);
        }
      }
      __syncthreads();
      if (wave < half) {
        const float4* slot = lds + (size_t)wave * SLOT;
#pragma unroll
        for (int t = 0; t < QT; ++t) {
          float2 ml = ((const float2*)(slot + QT * HT * 64))[t * 64 + lane];
          if (ml.y > 0.f) {  // the other wave saw at least one key
            float m_new = fmaxf(m_run[t], ml.x);
            float a_self = (l_run[t] > 0.f) ? exp2f(m_run[t] - m_new) : 0.f;
            float a_oth = exp2f(ml.x - m_new);
            l_run[t] = l_run[t] * a_self + ml.y * a_oth;
            m_run[t] = m_new;
#pragma unroll
            for (int h = 0; h < HT; ++h) {
              float4 o = slot[(t * HT + h) * 64 + lane];
              f32x4 a = acc[t][h];
              a[0] = a[0] * a_self + o.x * a_oth;
              a[1] = a[1] * a_self + o.y * a_oth;
              a[2] = a[2] * a_self + o.z * a_oth;
              a[3] = a[3] * a_self + o.w * a_oth;
              acc[t][h] = a;
            }
          }
        }
      }
      __syncthreads();
    }
    if (wave != 0) return;
  }

  // ---- normalise and store: lane holds hd rows h*16 + grp*4 .. +3 of query qcol --------------
#pragma unroll
  for (int t = 0; t < QT; ++t) {
    if (qrow[t] < 0) continue;
    float inv = 1.0f / l_run[t];
#pragma unroll
    for (int h = 0; h < HT; ++h) {
      f32x4 a = acc[t][h];
      uint2 pk = make_uint2(pack2_bf16(a[0] * inv, a[1] * inv), pack2_bf16(a[2] * inv, a[3] * inv));
      int k = qhead[t] * HD + h * 16 + grp * 4;
      *(uint2*)(out + packed_act_index(qrow[t], k, MT)) = pk;
    }
  }
}

// LDS a block may use on this device (queried once).
static size_t max_lds_per_block() {
  static size_t v = 0;
  if (v == 0) {
    int dev = 0, val = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&val, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) == hipSuccess &&
        val > 0)
      v = (size_t)val;
    else
      v = 64 * 1024;
  }
  return v;
}

template <int HD, int QT>
static void launch_split(const bf16_t* q, const uint4* kp, const uint4* vp, int M, int T, int Tpad,
                         int Hq, int Hkv, float sc, bf16_t* out, int MT, int qtiles,
                         hipStream_t s) {
  constexpr int SLOT = QT * (HD / 16) * 64 + QT * 32;
  // 8 waves stream more keys at once; 4 waves if the merge buffers of 8 do not fit in LDS
  int NW = 8;
  size_t smem = (size_t)(NW / 2) * SLOT * sizeof(float4);
  if (smem > max_lds_per_block()) {
    NW = 4;
    smem = (size_t)(NW / 2) * SLOT * sizeof(float4);
  }
  auto kern = attn_mfma_kernel<HD, QT, true>;
  static size_t attr_set = 0;
  if (smem > 48 * 1024 && attr_set < smem) {
    (void)hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                              (int)smem);
    attr_set = smem;
  }
  dim3 grid((qtiles + QT - 1) / QT, Hkv);
  kern<<<grid, NW * 64, smem, s>>>(q, kp, vp, M, T, Tpad, Hq, Hkv, sc, out, MT);
}

template <int HD>
static void launch_attn_mfma_hd(const bf16_t* q, const uint4* kp, const uint4* vp, int M, int T,
                                int Tpad, int Hq, int Hkv, bf16_t* out, hipStream_t s) {
  const int G = Hq / Hkv, nQ = M * G, qtiles = (nQ + 15) / 16, MT = (M + 15) / 16;
  const float sc = 1.4426950408889634f / sqrtf((float)HD);
  if (((qtiles + 1) / 2) * Hkv <= 128) {
    // few (query tile, kv head) pairs: split the keys over the waves of a block, at most 2 query
    // tiles per block; otherwise every wave walks all keys for its own query tiles
    if (qtiles <= 1) launch_split<HD, 1>(q, kp, vp, M, T, Tpad, Hq, Hkv, sc, out, MT, qtiles, s);
    else launch_split<HD, 2>(q, kp, vp, M, T, Tpad, Hq, Hkv, sc, out, MT, qtiles, s);
  } else {
    constexpr int QT = 2, NW = 4;
    dim3 grid((qtiles + QT * NW - 1) / (QT * NW), Hkv);
    attn_mfma_kernel<HD, QT, false><<<grid, NW * 64, 0, s>>>(q, kp, vp, M, T, Tpad, Hq, Hkv, sc,
                                                            out, MT);
  }
}

void launch_attention_mfma(const bf16_t* q, const bf16_t* kc, const bf16_t* vc, int M, int T,
                           int Tpad, int Hq, int Hkv, int hd, bf16_t* out, hipStream_t s) {
  if (M <= 0) return;
  if (hd == 64)
    launch_attn_mfma_hd<64>(q, (const uint4*)kc, (const uint4*)vc, M, T, Tpad, Hq, Hkv, out, s);
  else
    launch_attn_mfma_hd<128>(q, (const uint4*)kc, (const uint4*)vc, M, T, Tpad, Hq, Hkv, out, s);
}

}  // namespace ec
