// bf16 non-causal attention on MFMA with an online softmax, for the packed KV cache.
//
// The step's rows come as a list (sequence after sequence, each padded to whole 16-row tiles);
// a query tile is one 16-row tile of that list for one query head, tile number g * MT + mt for
// head g of the kv head's group, so the tiles of a group share the K/V fragments in cache.
// tileinfo tells the row tiles of many-row sequences which cache they attend to (offset,
// positions, padded keys); the few-row sequences come as (row tile, sequence) pairs.  Per 32-key chunk and query tile:
//   S^T[keys x queries] = K . Q^T          (2 key tiles x HD/32 MFMAs, K fragments straight from
//                                            the cache, Q fragments held in registers)
//   online softmax down the key axis        (a lane owns 8 consecutive keys of one query; the
//                                            other 24 are 2 xor-shuffles away)
//   O^T[hd x queries] += V^T . P^T          (HD/16 MFMAs; the lane's 8 probabilities ARE the
//                                            B operand, V^T fragments straight from the cache)
// Every operand load is a coalesced 1 KiB fragment in the cache's own layout.
//
// Two kernels:
//   split   (few query rows, partial step): a block owns one query tile of one kv head and its
//           waves stride over the key chunks, fragments going straight to registers; the waves'
//           partial (m, l, O) are combined through LDS in wave order.
//   shared  (many rows, full step): a block's waves own query tiles of one kv head and walk all
//           keys together, each chunk's fragments loaded once into an LDS ring.
#include "ec_internal.h"

namespace ec {

typedef uint32_t au32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ bf16x8 av4_as_bf16x8(au32x4 v) {
  union { au32x4 u; bf16x8 b; } c;
  c.u = v;
  return c.b;
}
__device__ __forceinline__ bf16x8 u4_as_bf16x8(uint4 v) {
  union { uint4 u; bf16x8 b; } c;
  c.u = v;
  return c.b;
}

// One 32-key chunk for one 16-query tile: S^T = K Q^T, online softmax down the keys, O^T += V^T P^T.
// kf / vf: the chunk's K and V^T fragments; qf: the tile's Q fragments; the lane owns query
// (lane & 15) and keys key0 .. key0+7.  mask_tail (wave-uniform): keys >= T are padding.
template <int HB, int HT>
__device__ __forceinline__ void attn_chunk_tile(const bf16x8 (&kf)[2][HB], const bf16x8 (&vf)[HT],
                                                const bf16x8 (&qf)[HB], f32x4 (&acc)[HT],
                                                float& m_run, float& l_run, float scale_log2e,
                                                int key0, int T, bool mask_tail) {
  f32x4 s2[2];
#pragma unroll
  for (int t2 = 0; t2 < 2; ++t2) {
    s2[t2] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int hb = 0; hb < HB; ++hb)
      s2[t2] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[t2][hb], qf[hb], s2[t2], 0, 0, 0);
  }
  float sv[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) sv[e] = s2[e >> 2][e & 3];
  if (mask_tail) {
#pragma unroll
    for (int e = 0; e < 8; ++e)
      if (key0 + e >= T) sv[e] = -INFINITY;
  }
  float mx = fmaxf(fmaxf(fmaxf(sv[0], sv[1]), fmaxf(sv[2], sv[3])),
                   fmaxf(fmaxf(sv[4], sv[5]), fmaxf(sv[6], sv[7])));
  // (lane swaps in the vector ALU: the cross-lane path through LDS costs four round trips here)
  mx = fmaxf(mx, other_row(mx));
  mx = fmaxf(mx, other_half(mx));
  const float m_new = fmaxf(m_run, mx * scale_log2e);  // scale > 0: max commutes with it
  float rs = 0.f;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    sv[e] = exp2f(fmaf(sv[e], scale_log2e, -m_new));
    rs += sv[e];
  }
  rs += other_row(rs);
  rs += other_half(rs);
  // the accumulators are rescaled only when some query of the wave saw a new maximum
  if (__builtin_amdgcn_ballot_w64(m_new > m_run) != 0) {
    const float alpha = exp2f(m_run - m_new);  // 0 on the first chunk, 1 where nothing changed
    l_run *= alpha;
#pragma unroll
    for (int h = 0; h < HT; ++h) {
      f32x4 a = acc[h];
      a[0] *= alpha; a[1] *= alpha; a[2] *= alpha; a[3] *= alpha;
      acc[h] = a;
    }
  }
  l_run += rs;
  m_run = m_new;
  uint4 pu = make_uint4(pack2_bf16(sv[0], sv[1]), pack2_bf16(sv[2], sv[3]),
                        pack2_bf16(sv[4], sv[5]), pack2_bf16(sv[6], sv[7]));
  const bf16x8 pf = u4_as_bf16x8(pu);
#pragma unroll
  for (int h = 0; h < HT; ++h)
    acc[h] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[h], pf, acc[h], 0, 0, 0);
}

// Few query rows (partial step): a block owns ONE 16-query tile of one kv head and its 8 waves
// stride over the 32-key chunks; each wave keeps two chunks' fragments in flight (the second is
// loaded while the first is multiplied), and the waves' partial (m, l, O) are combined through
// LDS in wave order.  grid (kv heads, query tiles): blocks of one head are Hkv apart in launch
// order, which for Hkv a multiple of 8 puts them on the same XCD, whose L2 then serves the
// head's K/V to all its query tiles.
//
// gridDim.z > 1 also splits the keys over blocks (a compute unit can only pull so many bytes per
// microsecond, and one head's K/V is too much for one): every block leaves its unnormalised
// (m, l, O) in `part`, takes a ticket, and the block that draws the last ticket of its (head,
// query tile) adds the pieces up in slice order - so the result does not depend on which block
// that is - and stores the output.  Pieces go through agent-scope atomic stores and loads, the
// ticket is an agent-scope acquire-release increment; nobody waits for anybody, so the scheme
// cannot hang.
struct AttnSplit {
  float* part;    // [pairs][gridDim.z][HT*64*4 + 64*2] floats
  int* tickets;   // [pairs], zero between launches (the last block of a pair resets its own)
};

__device__ __forceinline__ void st_agent(float* p, float a, float b) {
  union { float f[2]; unsigned long long u; } c;
  c.f[0] = a; c.f[1] = b;
  __hip_atomic_store((unsigned long long*)p, c.u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float2 ld_agent(const float* p) {
  union { float f[2]; unsigned long long u; } c;
  c.u = __hip_atomic_load((const unsigned long long*)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  return make_float2(c.f[0], c.f[1]);
}

//
// HS > 1 also splits the head dimension of the OUTPUT over HS blocks: each of them computes the
// whole score tile (it needs all of K) but multiplies only its HD/HS columns of V and stores only
// those, so nothing has to be merged across blocks.  A compute unit pulls only so many bytes
// per microsecond; with few blocks in the grid this spreads V over more of them.
template <int HD, int HS>
__global__ __launch_bounds__(512) void attn_mfma_split_kernel(
    const bf16_t* __restrict__ q, const au32x4* __restrict__ kp, const au32x4* __restrict__ vp,
    int R, const int4* __restrict__ rowinfo, const int4* __restrict__ pairs, int npairs,
    int4 one_seq, int Hq, int Hkv, float scale_log2e, bf16_t* __restrict__ out, AttnSplit sp) {
  constexpr int HB = HD / 32, HT = HD / 16 / HS, NW = 8;  // HT: hd tiles of V / the output here
  extern __shared__ float4 lds[];
  // scalar wave index: no MFMA may sit under a condition the compiler could treat as divergent
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int kvh = blockIdx.x, G = Hq / Hkv, MT = (R + 15) >> 4;
  const int by = blockIdx.y / HS, h0 = (blockIdx.y % HS) * HT;  // (visit, head of the group); first hd tile
  // The block's (row tile, sequence) pair: the few-row sequences are packed into the row list
  // without padding, so a tile can hold rows of two of them; it is then visited once for each,
  // and a visit serves only the rows of its own sequence.  pairs == NULL: a single sequence,
  // every tile is its own (one_seq).  Entry: row tile, cache offset, positions, keys per slab.
  int mt, gq;
  int4 ti;
  if (pairs) {
    const int4 pr = pairs[by % npairs];
    mt = pr.x; gq = by / npairs;
    ti = make_int4(pr.y, pr.z, pr.w, 0);
  } else {
    mt = by % MT; gq = by / MT;
    ti = one_seq;
    if (ti.w != 0) return;  // a many-row sequence: the other kernel's
  }
  const int T = ti.y, Tpad = ti.z;
  const int nchunks = (T + 31) >> 5, KB32 = Tpad >> 5;
  const int qcol = lane & 15, grp = lane >> 4;
  // this block's chunks: [c_lo, c_hi), empty if the sequence is short
  const int cpb = (nchunks + gridDim.z - 1) / gridDim.z;
  const int c_lo = min((int)blockIdx.z * cpb, nchunks);
  const int c_hi = min(c_lo + cpb, nchunks);

  // ---- Q fragments (B operand): lane (query qcol, group grp) holds 8 hd columns -------------
  const int qrow = mt * 16 + qcol, qhead = kvh * G + gq;
  const int qr = qrow < R ? qrow : 0;
  const int4 qri = rowinfo[qr];
  const bool qvalid = qrow < R && qri.x >= 0 && qri.z == ti.x;  // a row of this pair's sequence
  bf16x8 qf[HB];
#pragma unroll
  for (int hb = 0; hb < HB; ++hb) {
    // loaded regardless of validity (row qr exists), so that it does not wait for rowinfo
    au32x4 v = *(const au32x4*)(q + (size_t)qr * Hq * HD + qhead * HD + hb * 32 + grp * 8);
    qf[hb] = av4_as_bf16x8(qvalid ? v : (au32x4){0u, 0u, 0u, 0u});
  }

  f32x4 acc[HT];
  float m_run = -INFINITY, l_run = 0.f;
#pragma unroll
  for (int h = 0; h < HT; ++h) acc[h] = (f32x4){0.f, 0.f, 0.f, 0.f};

  const size_t slab = ((size_t)ti.x + (size_t)kvh * Tpad * HD) >> 3;  // in 16-byte units
  const au32x4* kbase = kp + slab + lane;
  const au32x4* vbase = vp + slab + lane;
  // the wave's chunks are c_lo + wave, + NW, ...: n_my of them.  Loads are unconditional (a
  // chunk past the end re-reads the last one, which is in cache); a chunk past the end is
  // computed with every key masked, which changes nothing once the wave has seen one real chunk.
  const int n_my = c_lo + wave < c_hi ? (c_hi - c_lo - wave + NW - 1) / NW : 0;
  bf16x8 kfa[2][HB], vfa[HT], kfb[2][HB], vfb[HT];
#define EC_AT_LOAD(KF, VF, I)                                                               \
  {                                                                                         \
    const int c_ = max(min(c_lo + wave + NW * (I), c_hi - 1), 0);                           \
    _Pragma("unroll") for (int t2 = 0; t2 < 2; ++t2)                                        \
      _Pragma("unroll") for (int hb = 0; hb < HB; ++hb)                                     \
        KF[t2][hb] = av4_as_bf16x8(kbase[((size_t)(c_ * 2 + t2) * HB + hb) * 64]);          \
    _Pragma("unroll") for (int h = 0; h < HT; ++h)                                          \
      VF[h] = av4_as_bf16x8(vbase[((size_t)(h0 + h) * KB32 + c_) * 64]);                    \
  }
#define EC_AT_COMPUTE(KF, VF, I)                                                            \
  {                                                                                         \
    const int c_ = c_lo + wave + NW * (I);                                                  \
    const bool real_ = (I) < n_my;                                                          \
    attn_chunk_tile<HB, HT>(KF, VF, qf, acc, m_run, l_run, scale_log2e, c_ * 32 + grp * 8,  \
                            real_ ? T : 0, !real_ || ((c_ == nchunks - 1) && (T & 31)));    \
  }
  EC_AT_LOAD(kfa, vfa, 0)
  // At most three chunks per wave (up to 768 keys per block): a third register set lets every
  // load be issued before the first multiplication, one trip to memory instead of two in a row.
  const int rounds = (c_hi - c_lo + NW - 1) / NW;  // block-uniform
  if (rounds <= 3) {
    bf16x8 kfc[2][HB], vfc[HT];
    EC_AT_LOAD(kfb, vfb, 1)
    EC_AT_LOAD(kfc, vfc, 2)
    __builtin_amdgcn_sched_barrier(0);
    // (n_my is wave-uniform and scalar: these are scalar branches around whole MFMA sequences)
    if (n_my > 0) EC_AT_COMPUTE(kfa, vfa, 0)
    __builtin_amdgcn_sched_barrier(0);
    if (n_my > 1) EC_AT_COMPUTE(kfb, vfb, 1)
    __builtin_amdgcn_sched_barrier(0);
    if (n_my > 2) EC_AT_COMPUTE(kfc, vfc, 2)
    __builtin_amdgcn_sched_barrier(0);
  } else
  for (int i = 0; i < n_my; i += 2) {
    EC_AT_LOAD(kfb, vfb, i + 1)
    __builtin_amdgcn_sched_barrier(0);
    EC_AT_COMPUTE(kfa, vfa, i)
    __builtin_amdgcn_sched_barrier(0);
    EC_AT_LOAD(kfa, vfa, i + 2)
    __builtin_amdgcn_sched_barrier(0);
    EC_AT_COMPUTE(kfb, vfb, i + 1)
    __builtin_amdgcn_sched_barrier(0);
  }
#undef EC_AT_LOAD
#undef EC_AT_COMPUTE

  // ---- merge the waves' partial results ------------------------------------------------------
  // Every wave parks (m, l, O) in LDS; after one barrier wave w combines the NW copies of hd tile
  // w (and w + NW, ...) in wave order, normalises and stores it.
  constexpr int SLOT = HT * 64 + 32;  // float4 per wave: O tiles + (m, l) pairs
  {
    float4* slot = lds + (size_t)wave * SLOT;
#pragma unroll
    for (int h = 0; h < HT; ++h) {
      f32x4 a = acc[h];
      slot[h * 64 + lane] = make_float4(a[0], a[1], a[2], a[3]);
    }
    ((float2*)(slot + HT * 64))[lane] = make_float2(m_run, l_run);
  }
  __syncthreads();
  float wgt[NW], m_all = -INFINITY, l_all = 0.f;
#pragma unroll
  for (int w = 0; w < NW; ++w) {
    float2 ml = ((const float2*)(lds + (size_t)w * SLOT + HT * 64))[lane];
    wgt[w] = ml.x;
    m_all = fmaxf(m_all, ml.x);
  }
#pragma unroll
  for (int w = 0; w < NW; ++w) {
    float2 ml = ((const float2*)(lds + (size_t)w * SLOT + HT * 64))[lane];
    wgt[w] = ml.y > 0.f ? exp2f(wgt[w] - m_all) : 0.f;  // a wave without keys has weight 0
    l_all += ml.y * wgt[w];
  }
  const int nz = gridDim.z;
  const int pair = blockIdx.y * gridDim.x + blockIdx.x;
  constexpr int PSLOT = HT * 256 + 128;  // floats per (pair, slice)
  float* mine = sp.part + ((size_t)pair * nz + blockIdx.z) * PSLOT;
  for (int h = wave; h < HT; h += NW) {
    float4 o = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      float4 v = lds[(size_t)w * SLOT + h * 64 + lane];
      o.x += v.x * wgt[w]; o.y += v.y * wgt[w]; o.z += v.z * wgt[w]; o.w += v.w * wgt[w];
    }
    if (nz == 1) {
      // lane holds hd rows h*16 + grp*4 .. +3 of query qcol
      const float inv = 1.0f / l_all;
      uint2 pk = make_uint2(pack2_bf16(o.x * inv, o.y * inv), pack2_bf16(o.z * inv, o.w * inv));
      if (qvalid) *(uint2*)(out + packed_act_index(qrow, qhead * HD + (h0 + h) * 16 + grp * 4, MT)) = pk;
    } else {
      st_agent(mine + (h * 64 + lane) * 4, o.x, o.y);
      st_agent(mine + (h * 64 + lane) * 4 + 2, o.z, o.w);
    }
  }
  if (nz == 1) return;
  static_assert(HS == 1 || HD % (16 * HS) == 0, "whole hd tiles per block");
  // (key slices over blocks are only launched with HS == 1: the piece layout below assumes it)

  // ---- cross-block: leave (m, l), draw a ticket, the last block of the pair finishes ---------
  // Ordering: every thread's pieces happen-before the block barrier (work-group scope); thread
  // 0's ticket increment RELEASES them at agent scope, and the finishing block's increment
  // ACQUIRES every earlier block's pieces, which its barrier then hands to its other threads.
  if (wave == 0) st_agent(mine + HT * 256 + lane * 2, m_all, l_all);
  __syncthreads();
  int* flag = (int*)lds;  // the parked copies are no longer needed
  if (threadIdx.x == 0) {
    int old = __hip_atomic_fetch_add(sp.tickets + pair, 1, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
    // (the counter returns to zero for the next launch; no other block of this launch reads it
    // any more, and a kernel boundary orders it for the next one)
    if (old == nz - 1)
      __hip_atomic_store(sp.tickets + pair, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    *flag = (old == nz - 1);
  }
  __syncthreads();
  if (*flag == 0 || !qvalid) return;
  const float* base = sp.part + (size_t)pair * nz * PSLOT;
  float m_fin = -INFINITY, l_fin = 0.f;
  for (int z = 0; z < nz; ++z) m_fin = fmaxf(m_fin, ld_agent(base + (size_t)z * PSLOT + HT * 256 + lane * 2).x);
  for (int h = wave; h < HT; h += NW) {
    float4 o = make_float4(0.f, 0.f, 0.f, 0.f);
    l_fin = 0.f;
    for (int z = 0; z < nz; ++z) {
      const float* pz = base + (size_t)z * PSLOT;
      const float2 ml = ld_agent(pz + HT * 256 + lane * 2);
      const float wz = ml.y > 0.f ? exp2f(ml.x - m_fin) : 0.f;
      const float2 a = ld_agent(pz + (h * 64 + lane) * 4), b = ld_agent(pz + (h * 64 + lane) * 4 + 2);
      l_fin += ml.y * wz;
      o.x += a.x * wz; o.y += a.y * wz; o.z += b.x * wz; o.w += b.y * wz;
    }
    const float inv = 1.0f / l_fin;
    uint2 pk = make_uint2(pack2_bf16(o.x * inv, o.y * inv), pack2_bf16(o.z * inv, o.w * inv));
    *(uint2*)(out + packed_act_index(qrow, qhead * HD + h * 16 + grp * 4, MT)) = pk;
  }
}

// ---------------------------------------------------------------------------------------------
// Many query rows (full step): a block of NW waves owns NW*QT query tiles of one kv head and
// walks all keys.  Each 32-key chunk (K and V^T fragments, 16 KiB at hd = 128) is loaded once per
// block, straight from global memory into a 3-stage LDS ring (global_load_lds_dwordx4), and read
// by all waves.  Two waves per SIMD let one wave's softmax arithmetic run under the other's
// MFMAs.
// ---------------------------------------------------------------------------------------------
template <int N> __device__ __forceinline__ void attn_wait_vmcnt() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// Chunks of the LDS ring (a deeper ring was measured: no gain, the loop is not waiting on loads).
constexpr int kAttnStages = 3;

//
// FEW: the same ring for a batch of few-row sequences.  A block then owns one (sequence, query
// head): wave w serves the sequence's w-th row-tile visit (the packed row list lets a tile hold
// rows of two sequences; a visit serves only its own sequence's rows and stores nothing else),
// waves without a visit only help with the loads.  The sequence's K/V are read once per head
// instead of once per visit, which is what bounds a batch's partial step.
template <int HD, int QT, int NW, bool FEW = false>
__global__ __launch_bounds__(NW * 64) void attn_mfma_shared_kernel(
    const bf16_t* __restrict__ q, const au32x4* __restrict__ kp, const au32x4* __restrict__ vp,
    int R, const int4* __restrict__ rowinfo, const int4* __restrict__ tileinfo, int4 one_seq,
    int Hq, int Hkv, float scale_log2e, bf16_t* __restrict__ out,
    const int4* __restrict__ pairs, const int4* __restrict__ seqtab, int nsmall) {
  static_assert(!FEW || QT == 1, "one visit per wave");
  constexpr int HB = HD / 32, HT = HD / 16, NSTAGE = kAttnStages;
  constexpr int NFRAG = 2 * HB + HT, LF = NFRAG / NW;
  static_assert(NFRAG % NW == 0, "fragments per chunk must divide over the waves");
  extern __shared__ au32x4 ring[];  // [NSTAGE][NFRAG][64]
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  // grid (kv heads, tile groups): the blocks of one head are Hkv apart in launch order, which
  // for Hkv a multiple of 8 puts them on one XCD, whose L2 then holds the head's K/V once
  const int kvh = blockIdx.x, G = Hq / Hkv, MT = (R + 15) >> 4, MTp = (MT + 15) & ~15;
  // the block's NW*QT query tiles: one head of the group, consecutive row tiles that all lie in
  // one many-row sequence (such sequences come first and are padded to 16 row tiles) or in none
  int gq, mt0;
  int4 ti;
  bool active = true;  // (wave-uniform) this wave has query rows to serve
  if constexpr (FEW) {
    gq = blockIdx.y / nsmall;
    const int4 se = seqtab[blockIdx.y - gq * nsmall];  // first visit, number of visits (<= NW)
    const int4 p0 = pairs[se.x];
    ti = make_int4(p0.y, p0.z, p0.w, 1);
    active = __builtin_amdgcn_readfirstlane(wave < se.y ? 1 : 0) != 0;
    mt0 = __builtin_amdgcn_readfirstlane(pairs[se.x + (wave < se.y ? wave : 0)].x);
  } else {
    const int t_first = blockIdx.y * NW * QT;
    gq = t_first / MTp;
    const int mt_first = t_first - gq * MTp;
    if (mt_first >= MT) return;
    ti = tileinfo ? tileinfo[mt_first] : one_seq;
    if (ti.w == 0) return;  // few-row sequences belong to the other kernels
    mt0 = mt_first + wave * QT;
  }
  const int T = ti.y, Tpad = ti.z;
  const int nchunks = (T + 31) >> 5, KB32 = Tpad >> 5;
  const int qcol = lane & 15, grp = lane >> 4;

  // fragment f of a chunk: f < 2*HB is K tile f / HB, hd block f % HB; the rest are V^T hd tiles
  const size_t slab = ((size_t)ti.x + (size_t)kvh * Tpad * HD) >> 3;  // in 16-byte units
  const au32x4* kbase = kp + slab + lane;
  const au32x4* vbase = vp + slab + lane;
  auto issue = [&](int c) {
    const int cc = min(c, nchunks - 1), stage = c % NSTAGE;
#pragma unroll
    for (int i = 0; i < LF; ++i) {
      const int f = wave + NW * i;
      const au32x4* src = f < 2 * HB ? kbase + ((size_t)(cc * 2 + f / HB) * HB + f % HB) * 64
                                     : vbase + ((size_t)(f - 2 * HB) * KB32 + cc) * 64;
      __builtin_amdgcn_global_load_lds(
          (const void __attribute__((address_space(1)))*)src,
          (void __attribute__((address_space(3)))*)(ring + ((size_t)stage * NFRAG + f) * 64), 16,
          0, FEW ? 2 : 0);  // (few-row batches read every K/V byte once: non-temporal)
    }
  };

  bf16x8 qf[QT][HB];
  int qrow[QT];
  bool qvalid[QT];
  const int qhead = kvh * G + gq;
#pragma unroll
  for (int t = 0; t < QT; ++t) {
    qrow[t] = (mt0 + t) * 16 + qcol;
    const int4 qri = rowinfo[qrow[t] < R ? qrow[t] : 0];
    qvalid[t] = qrow[t] < R && qri.x >= 0;
    if constexpr (FEW) qvalid[t] = qvalid[t] && active && qri.z == ti.x;  // a row of this sequence
#pragma unroll
    for (int hb = 0; hb < HB; ++hb) {
      uint4 v = make_uint4(0, 0, 0, 0);
      if (qvalid[t])
        v = *(const uint4*)(q + (size_t)qrow[t] * Hq * HD + qhead * HD + hb * 32 + grp * 8);
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

#pragma unroll
  for (int sg = 0; sg < NSTAGE - 1; ++sg) issue(sg);
  for (int c = 0; c < nchunks; ++c) {
    attn_wait_vmcnt<LF*(NSTAGE - 2)>();  // this wave's loads of chunk c have landed
    block_barrier_nofence();             // ... everyone's have; the stage read last is free
    issue(c + NSTAGE - 1);
    const au32x4* st = ring + (size_t)(c % NSTAGE) * NFRAG * 64 + lane;
    bf16x8 kf[2][HB], vf[HT];
#pragma unroll
    for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
      for (int hb = 0; hb < HB; ++hb) kf[t2][hb] = av4_as_bf16x8(st[(t2 * HB + hb) * 64]);
#pragma unroll
    for (int h = 0; h < HT; ++h) vf[h] = av4_as_bf16x8(st[(2 * HB + h) * 64]);

    const int key0 = c * 32 + grp * 8;
    const bool mask_tail = (c == nchunks - 1) && (T & 31);
    if (active) {  // (a scalar branch around whole MFMA sequences)
#pragma unroll
      for (int t = 0; t < QT; ++t)
        attn_chunk_tile<HB, HT>(kf, vf, qf[t], acc[t], m_run[t], l_run[t], scale_log2e, key0, T,
                                mask_tail);
    }
  }
  attn_wait_vmcnt<0>();  // drain the clamped tail loads before the LDS goes away

#pragma unroll
  for (int t = 0; t < QT; ++t) {
    if (qrow[t] >= R) continue;
    float inv = 1.0f / l_run[t];
#pragma unroll
    for (int h = 0; h < HT; ++h) {
      f32x4 a = acc[t][h];
      uint2 pk = make_uint2(pack2_bf16(a[0] * inv, a[1] * inv), pack2_bf16(a[2] * inv, a[3] * inv));
      if (!qvalid[t]) pk = make_uint2(0u, 0u);  // padding rows read as zeros downstream
      int k = qhead * HD + h * 16 + grp * 4;
      // (FEW: the other rows of the tile belong to a neighbour sequence's visit)
      if (!FEW || qvalid[t]) *(uint2*)(out + packed_act_index(qrow[t], k, MT)) = pk;
    }
  }
}

template <int HD>
static void launch_attn_mfma_hd(const bf16_t* q, const uint4* kp, const uint4* vp, int R,
                                const int4* rowinfo, const int4* tileinfo, const int4* pairs,
                                int npairs, const int4* seqtab, int nsmall, int max_visits,
                                int4 one_seq, bool has_small, bool has_large,
                                int max_T, int Hq, int Hkv, bf16_t* out, float* part,
                                size_t part_floats, int* tickets, hipStream_t s) {
  const int G = Hq / Hkv, MT = (R + 15) / 16;
  const float sc = 1.4426950408889634f / sqrtf((float)HD);
  constexpr int kRingFrag = 2 * (HD / 32) + HD / 16;
  constexpr size_t kRingBytes = (size_t)kAttnStages * kRingFrag * 1024;
  // A batch of few-row sequences whose rows spread over several row tiles each: one block per
  // (sequence, head) that reads the sequence's K/V once, provided that fills the chip.
  const bool few_shared = has_small && pairs && seqtab && nsmall > 0 && max_visits <= 8 &&
                          npairs >= 2 * nsmall && (long)nsmall * Hq >= 256;
  if (few_shared) {
    static bool few_attr_set = false;
    if (kRingBytes > 48 * 1024 && !few_attr_set) {
      (void)hipFuncSetAttribute((const void*)attn_mfma_shared_kernel<HD, 1, 8, true>,
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)kRingBytes);
      few_attr_set = true;
    }
    attn_mfma_shared_kernel<HD, 1, 8, true><<<dim3(Hkv, G * nsmall), 512, kRingBytes, s>>>(
        q, (const au32x4*)kp, (const au32x4*)vp, R, rowinfo, tileinfo, one_seq, Hq, Hkv, sc, out,
        pairs, seqtab, nsmall);
  } else if (has_small) {
    // sequences with few rows: one block per query tile, the keys split over its waves
    constexpr int SLOT = (HD / 16) * 64 + 32;
    constexpr size_t smem = 8 * SLOT * sizeof(float4);
    static bool attr_set = false;
    if (smem > 48 * 1024 && !attr_set) {
      (void)hipFuncSetAttribute((const void*)attn_mfma_split_kernel<HD, 1>,
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
      attr_set = true;
    }
    // Key slices over blocks pay only for long contexts (the pieces go through write-through
    // stores and a ticket, about 3 us): from 64 chunks on, two or more chunks per wave, and no
    // more blocks than compute units.
    const int nvis = pairs ? npairs : MT;  // (row tile, sequence) visits
    const int nchunks = (max_T + 31) / 32, blocks1 = G * nvis * Hkv;
    constexpr size_t PSLOT = (HD / 16) * 256 + 128;
    int nz = 1;
    if (nchunks >= 64 && blocks1 <= 256) {
      nz = nchunks / 16;
      if (nz > 256 / blocks1) nz = 256 / blocks1;
      if (nz > 8) nz = 8;
      if (nz < 1) nz = 1;
    }
    while (nz > 1 && (size_t)blocks1 * nz * PSLOT > part_floats) --nz;
    if (!part || !tickets) nz = 1;
    AttnSplit sp;
    sp.part = part;
    sp.tickets = tickets;
    // output columns over blocks while the grid stays within the chip's 256 compute units
    int hs = 1;
    if (nz == 1)
      while (hs < 8 && hs * 2 <= HD / 16 && blocks1 * hs * 2 <= 256) hs *= 2;
#define EC_SPLIT_LAUNCH(HS_)                                                                     \
  attn_mfma_split_kernel<HD, HS_><<<dim3(Hkv, G * nvis * HS_, nz), 512,                          \
                                    8 * ((HD / 16 / HS_) * 64 + 32) * sizeof(float4), s>>>(      \
      q, (const au32x4*)kp, (const au32x4*)vp, R, rowinfo, pairs, npairs, one_seq, Hq, Hkv, sc,  \
      out, sp)
    if (hs == 8) { if constexpr (HD >= 128) EC_SPLIT_LAUNCH(8); }
    else if (hs == 4) EC_SPLIT_LAUNCH(4);
    else if (hs == 2) EC_SPLIT_LAUNCH(2);
    else EC_SPLIT_LAUNCH(1);
#undef EC_SPLIT_LAUNCH
  }
  if (has_large) {
    // two query tiles per wave halve the LDS reads per MFMA, but only pay once the grid still
    // covers the chip's 256 compute units
    constexpr int NW = 8, NFRAG = 2 * (HD / 32) + HD / 16;
    constexpr size_t ring_bytes = (size_t)kAttnStages * NFRAG * 1024;
    static bool ring_attr_set = false;
    if (ring_bytes > 48 * 1024 && !ring_attr_set) {
      (void)hipFuncSetAttribute((const void*)attn_mfma_shared_kernel<HD, 1, NW>,
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)ring_bytes);
      (void)hipFuncSetAttribute((const void*)attn_mfma_shared_kernel<HD, 2, NW>,
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)ring_bytes);
      ring_attr_set = true;
    }
    const int tiles = G * ((MT + 15) & ~15);
    if ((tiles / (2 * NW)) * Hkv >= 256) {
      dim3 grid(Hkv, tiles / (2 * NW));
      attn_mfma_shared_kernel<HD, 2, NW><<<grid, NW * 64, ring_bytes, s>>>(
          q, (const au32x4*)kp, (const au32x4*)vp, R, rowinfo, tileinfo, one_seq, Hq, Hkv, sc,
          out, nullptr, nullptr, 0);
    } else {
      dim3 grid(Hkv, tiles / NW);
      attn_mfma_shared_kernel<HD, 1, NW><<<grid, NW * 64, ring_bytes, s>>>(
          q, (const au32x4*)kp, (const au32x4*)vp, R, rowinfo, tileinfo, one_seq, Hq, Hkv, sc,
          out, nullptr, nullptr, 0);
    }
  }
}

void launch_attention_mfma(const bf16_t* q, const bf16_t* kc, const bf16_t* vc, int R,
                           const int4* rowinfo, const int4* tileinfo, const int4* pairs,
                           int npairs, const int4* seqtab, int nsmall, int max_visits,
                           int4 one_seq, bool has_small, bool has_large, int max_T,
                           int Hq, int Hkv, int hd, bf16_t* out, float* part, size_t part_floats,
                           int* tickets, hipStream_t s) {
  if (R <= 0) return;
  if (hd == 64)
    launch_attn_mfma_hd<64>(q, (const uint4*)kc, (const uint4*)vc, R, rowinfo, tileinfo, pairs,
                            npairs, seqtab, nsmall, max_visits, one_seq,
                            has_small, has_large, max_T, Hq, Hkv, out, part, part_floats, tickets, s);
  else
    launch_attn_mfma_hd<128>(q, (const uint4*)kc, (const uint4*)vc, R, rowinfo, tileinfo, pairs,
                             npairs, seqtab, nsmall, max_visits, one_seq,
                             has_small, has_large, max_T, Hq, Hkv, out, part, part_floats, tickets,
                             s);
}

}  // namespace ec
