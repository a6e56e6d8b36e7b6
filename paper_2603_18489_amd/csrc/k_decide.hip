// The O(V) decision of EntropyCache and the bookkeeping around it:
//   vocab_reduce : per logit row, partial (max, argmax, sum e^{z-max}, sum e^{z-max}(z-max))
//                  over chunks of the vocabulary, in one pass.
//   decide       : merges the partials (confidence = 1/S, entropy H = ln S - T/S; Eq. 1), picks
//                  the tokens to unmask (decode()), records the decode history (Eq. 2), selects
//                  the recent tokens (Eq. 3, tau_R, R), sets the skip flag (E <= tau) and builds
//                  the row set M u R of the next partial step.
// Every reduction runs in a fixed order, so results are bit-reproducible.
#include <limits.h>

#include "ec_internal.h"
#include "k_vtuple.h"

namespace ec {

constexpr int VR_CHUNK = 2048;  // logits per block

int vocab_reduce_parts(int V) { return (V + VR_CHUNK - 1) / VR_CHUNK; }

__global__ __launch_bounds__(256) void vocab_reduce_kernel(const float* __restrict__ logits, int V,
                                                           size_t ld, int nparts,
                                                           float4* __restrict__ partials) {
  __shared__ VTuple wt[4];
  const int part = blockIdx.x, row = blockIdx.y, tid = threadIdx.x;
  const float* z = logits + (size_t)row * ld;
  int lo = part * VR_CHUNK, hi = min(V, lo + VR_CHUNK);
  VTuple v = vt_identity();
  for (int i = lo + tid; i < hi; i += 256) vt_push(v, z[i], i);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    VTuple other = vt_shfl_down(v, o);
    v = vt_merge(v, other);  // lane l merges lane l+o; lane 0 ends with the wave's result
  }
  if ((tid & 63) == 0) wt[tid >> 6] = v;
  __syncthreads();
  if (tid == 0) {
    VTuple r = wt[0];
    for (int w = 1; w < 4; ++w) r = vt_merge(r, wt[w]);
    partials[(size_t)row * nparts + part] = make_float4(r.m, __int_as_float(r.idx), r.s, r.t);
  }
}

void launch_vocab_reduce(const float* logits, int n_rows, int V, size_t ld, float4* partials,
                         hipStream_t s) {
  if (n_rows <= 0) return;
  int nparts = vocab_reduce_parts(V);
  vocab_reduce_kernel<<<dim3(nparts, n_rows), 256, 0, s>>>(logits, V, ld, nparts, partials);
}

// One thread per row: merges the row's partials in part order and writes
// (token id as float, confidence, entropy, max logit).
__global__ __launch_bounds__(64) void row_stats_kernel(const float4* __restrict__ partials,
                                                       int nparts, int n_rows,
                                                       float4* __restrict__ stats) {
  const int row = blockIdx.x * 64 + threadIdx.x;
  if (row >= n_rows) return;
  VTuple v = vt_identity();
  for (int p = 0; p < nparts; ++p) {
    const float4 q = partials[(size_t)row * nparts + p];
    v = vt_merge(v, VTuple{q.x, __float_as_int(q.y), q.z, q.w});
  }
  float conf, H;
  vt_finish(v, conf, H);
  stats[row] = make_float4((float)v.idx, conf, H, v.m);
}

void launch_row_stats(const float4* partials, int nparts, int n_rows, float4* stats, hipStream_t s) {
  if (n_rows <= 0) return;
  row_stats_kernel<<<(n_rows + 63) / 64, 64, 0, s>>>(partials, nparts, n_rows, stats);
}

// ---- block-wide integer helpers (kDecideThreads threads) --------------------------------------
constexpr int kDecideThreads = 1024, kDecideWaves = kDecideThreads / 64;

// Exclusive prefix of a 0/1 flag over the block; returns the prefix, *total gets the block sum.
__device__ __forceinline__ int block_excl_scan_flag(int flag, int* scratch, int* total) {
  unsigned long long ball = __ballot(flag);
  int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  int pre = __popcll(ball & ((1ull << lane) - 1ull));
  __syncthreads();
  if (lane == 0) scratch[w] = __popcll(ball);
  __syncthreads();
  int off = 0, tot = 0;
#pragma unroll
  for (int i = 0; i < kDecideWaves; ++i) {
    const int c = scratch[i];
    off += i < w ? c : 0;
    tot += c;
  }
  *total = tot;
  return off + pre;
}

// The quantity the threshold is applied to, accumulated over the newly decoded tokens: their
// maximum entropy (Eq. 1), the sum of their entropies, or their maximum confidence (the
// alternatives of the ablation on the thresholding variable).  Empty = the value that skips.
struct GateAcc { float v; int metric; };
__device__ __forceinline__ GateAcc gate_init(int metric) {
  return GateAcc{metric == EC_GATE_MAX_CONFIDENCE ? INFINITY : -INFINITY, metric};
}
__device__ __forceinline__ void gate_add(GateAcc& g, float H, float conf) {
  if (g.metric == EC_GATE_ENTROPY_SUM) g.v = (g.v == -INFINITY) ? H : g.v + H;
  else if (g.metric == EC_GATE_MAX_CONFIDENCE) g.v = (g.v == INFINITY) ? conf : fmaxf(g.v, conf);
  else g.v = fmaxf(g.v, H);
}
__device__ __forceinline__ bool gate_skips(float v, float tau, int metric) {
  return metric == EC_GATE_MAX_CONFIDENCE ? v >= tau : v <= tau;
}

// ---------------------------------------------------------------------------------------------
// decide: one block of kDecideThreads threads per sequence.  Everything the block reads from
// memory (state, history, mask set, the rows' partial tuples, the caller's forced tokens) is
// requested up front; from then on it works in LDS and registers, so the kernel's latency is two
// memory round trips plus arithmetic.
// dynamic LDS: int hist[N4] | uint8 masked[N4], N4 = N rounded up to 4
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kDecideThreads) void decide_kernel(DecideArgs a) {
  extern __shared__ int s_dyn[];
  {  // this block's sequence: move the pointers, take the per-sequence scalars
    const int b = blockIdx.x;
    const SeqDesc sd = a.seqs ? a.seqs[b] : a.seq0;
    if (sd.mode < 0) return;  // finished earlier: no rows in this step, nothing to decide
    a.partials += (size_t)sd.lm0 * a.nparts;
    a.n_mb = sd.n_mb; a.mode_run = sd.mode; a.n_rows_run = sd.n_rows; a.forced_n = sd.forced_n;
    a.forced_pos += b * EC_MAX_N; a.forced_tok += b * EC_MAX_N;
    a.x += sd.x_off; a.masked += sd.x_off; a.rows_partial += sd.x_off;
    a.hist += (size_t)b * a.N; a.st += b; a.out += b;
    a.mb_pos += b * a.block; a.mb_idx += b * a.block; a.row_stats += b * a.block * 4;
    a.P = sd.P; a.T = sd.T;
  }
  __shared__ int s_tok[EC_MAX_BLOCK], s_pos[EC_MAX_BLOCK];
  __shared__ float s_conf[EC_MAX_BLOCK], s_H[EC_MAX_BLOCK];
  __shared__ int s_badrow[EC_MAX_BLOCK];  // 1: the row's logits had no finite maximum / sums
  __shared__ int s_sel[EC_MAX_N];    // block rows of the step's own choice, most confident first
  __shared__ int s_frow[EC_MAX_N];   // block rows of the caller's positions (-1: not in the block)
  __shared__ int scratch[kDecideWaves];
  __shared__ float sh_f[2];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int P = a.P, N = a.N;
  int* s_hist = s_dyn;
  uint8_t* s_msk = (uint8_t*)(s_dyn + ((N + 3) & ~3));
  const int nblocks = (N + a.block - 1) / a.block;

  // ---- requests: state, history, mask set, block positions, forced tokens --------------------
  DevState st = *a.st;  // every thread holds a private copy; thread 0 writes it back
  for (int i = tid; i < N; i += kDecideThreads) {
    s_hist[i] = a.hist[i];
    s_msk[i] = a.masked[P + i];
  }
  int f_pos = -1, f_tok = -1;
  if (!a.init_only) {
    if (tid < a.n_mb) s_pos[tid] = a.mb_pos[tid];
    if (tid < a.forced_n) { f_pos = a.forced_pos[tid]; f_tok = a.forced_tok[tid]; }
  }
  const int t = st.t;

  if (!a.init_only) {
    // ---- merge the vocabulary partials of each block row (fixed order) ----------------------
    // Half a wave per row, 32 rows at a time: lane l of the half merges parts l, l + 32, ... in
    // that order (sixteen loads in flight), then the 32 tuples are merged pairwise down to the
    // half's first lane.
    for (int row0 = 0; row0 < a.n_mb; row0 += 2 * kDecideWaves) {
      const int row = row0 + wave * 2 + (lane >> 5), l32 = lane & 31;
      const bool live = row < a.n_mb;
      const float4* pr = a.partials + (size_t)(live ? row : 0) * a.nparts;
      // The lane's running tuple is re-based once per batch of 16 parts (to the batch's maximum
      // if that is larger), after which a part costs one fast exponential and a few FMAs.
      VTuple v = vt_identity();
      for (int p0 = l32; p0 < a.nparts; p0 += 32 * 16) {
        float4 q[16];
#pragma unroll
        for (int u = 0; u < 16; ++u)   // unconditional loads (clamped), so that all are in flight
          q[u] = pr[min(p0 + 32 * u, a.nparts - 1)];
        bool ok[16];
        float bm = -INFINITY;
#pragma unroll
        for (int u = 0; u < 16; ++u) {
          ok[u] = live && p0 + 32 * u < a.nparts && q[u].z != 0.f;   // (an empty part has S = 0)
          bm = fmaxf(bm, ok[u] ? q[u].x : -INFINITY);
        }
        if (bm > v.m) {
          if (v.s != 0.f) {
            const float d = v.m - bm, e = __expf(d);
            v.t = e * (v.t + d * v.s);
            v.s *= e;
          }
          v.m = bm;
          v.idx = INT_MAX;
        }
#pragma unroll
        for (int u = 0; u < 16; ++u) {
          const float d = ok[u] ? q[u].x - v.m : 0.f;            // <= 0
          const float e = ok[u] ? __expf(d) : 0.f;
          v.s += q[u].z * e;
          v.t += e * (q[u].w + d * q[u].z);
          const int pi = __float_as_int(q[u].y);
          if (ok[u] && d == 0.f && pi < v.idx) v.idx = pi;       // lowest index among equal maxima
        }
      }
#pragma unroll
      for (int o = 16; o > 0; o >>= 1) v = vt_merge(v, vt_shfl_down(v, o));
      if (live && l32 == 0) {
        float conf, H;
        vt_finish(v, conf, H);
        // A row of NaNs has no maximum: its index is still the sentinel, its sums are NaN.  The
        // token becomes an index into the embedding table at the next step, so it must be a
        // token; such a row counts as least confident and of infinite entropy, and is reported.
        int tok = v.idx, bad = 0;
        if ((unsigned)tok >= (unsigned)a.vocab) { tok = 0; bad = 1; }
        if (!(v.s > 0.f) || !(conf >= 0.f) || !(v.t == v.t) || !(H >= 0.f)) bad = 1;
        if (bad) { conf = 0.f; H = INFINITY; }  // (the clamp in vt_finish turns a NaN entropy into 0)
        s_badrow[row] = bad;
        s_tok[row] = tok;
        s_conf[row] = conf;
        s_H[row] = H;
        *(float4*)(a.row_stats + row * 4) = make_float4((float)tok, conf, H, v.m);
      }
    }
    __syncthreads();
    // ---- decode(): most confident rows first; ties -> lowest position (= lowest row) --------
    // A row's rank is the number of rows that go before it; the n lowest ranks are unmasked.
    int n = min(a.n_tok, a.n_mb);
    const bool is_row = tid < a.n_mb;
    const float my_conf = is_row ? s_conf[tid] : 0.f;
    if (a.conf_threshold > 0.f) {
      // confidence-based parallel decoding: every row above the threshold, the n most
      // confident ones in any case, no more than one result can report
      const int above = __syncthreads_count(is_row && my_conf > a.conf_threshold);
      n = min(min(max(n, above), EC_MAX_N), a.n_mb);
    }
    ec_step_result& R = a.out->r;
    int rank = EC_MAX_BLOCK;
    if (is_row) {
      rank = 0;
      for (int r = 0; r < a.n_mb; ++r) {
        const float c = s_conf[r];
        rank += (c > my_conf || (c == my_conf && r < tid)) ? 1 : 0;
      }
      if (rank < n) {
        s_sel[rank] = tid;
        R.positions[rank] = s_pos[tid];
        R.tokens[rank] = s_tok[tid];
        R.entropy[rank] = s_H[tid];
        R.confidence[rank] = my_conf;
      }
    }
    if (tid >= n && tid < EC_MAX_N) {
      R.positions[tid] = -1; R.tokens[tid] = -1; R.entropy[tid] = 0.f; R.confidence[tid] = 0.f;
    }
    // ---- commit: own choice, or the caller's under teacher forcing (Eq. 2) -------------------
    // (to memory, and to the LDS copies the rest of the kernel works on)
    int c_pos = -1, c_tok = 0;
    if (a.forced_n >= 0) {
      if (tid < a.forced_n) {
        int row = -1;
        for (int r = 0; r < a.n_mb; ++r)
          if (s_pos[r] == f_pos) row = r;
        s_frow[tid] = row;
        c_pos = f_pos; c_tok = f_tok;
      }
    } else if (rank < n) {
      c_pos = s_pos[tid]; c_tok = s_tok[tid];
    }
    if (c_pos >= 0) {
      a.x[c_pos] = c_tok;
      a.masked[c_pos] = 0;
      a.hist[c_pos - P] = t;
      s_msk[c_pos - P] = 0;
      s_hist[c_pos - P] = t;
    }
    __syncthreads();
    if (tid == 0) {
      // gate values, accumulated in the order of the lists (the entropy sum is order-sensitive)
      GateAcc own = gate_init(a.gate_metric);
      for (int i = 0; i < n; ++i) gate_add(own, s_H[s_sel[i]], s_conf[s_sel[i]]);
      float E = own.v;
      if (a.forced_n >= 0) {
        bool all_in_block = true;
        GateAcc fa = gate_init(a.gate_metric);
        for (int i = 0; i < a.forced_n; ++i) {
          const int row = s_frow[i];
          if (row < 0) all_in_block = false; else gate_add(fa, s_H[row], s_conf[row]);
        }
        if (all_in_block) E = fa.v;                       // nothing committed: always skips
      }
      R.n_unmasked = n;
      R.max_entropy = own.v;
      sh_f[0] = E;
      sh_f[1] = own.v;
    }
  }
  __syncthreads();   // the LDS copies of history and mask set are complete (and committed to)

  // ---- recency threshold: tau_R = max(k-th largest history value, t - dt) --------------------
  // History values are step indices in [1, t] or "never": the k-th largest is the largest v with
  // count(hist >= v) >= k, found by bisection; fewer than k decoded -> -inf.
  int t_lastfull = st.t_lastfull;
  int tauR = INT_MAX;
  if (!a.init_only) {
    if (a.mode_run == EC_FULL) t_lastfull = t;
    int kth = INT_MIN;
    if (a.k_recent > 0) {
      int lo = 1, hi = t, found = INT_MIN;
      while (lo <= hi) {  // uniform across the block
        const int mid = (lo + hi) >> 1;
        int c = 0;
        for (int base = 0; base < N; base += kDecideThreads) {  // uniform trip count
          const int i = base + tid;
          c += __syncthreads_count(i < N && s_hist[i] >= mid);
        }
        if (c >= a.k_recent) { found = mid; lo = mid + 1; } else { hi = mid - 1; }
      }
      kth = found;
    } else {
      kth = INT_MAX;  // empty selection: nothing qualifies by rank
    }
    tauR = max(kth, t_lastfull);  // t - dt == index of the last FULL step
  }

  // ---- flag for the next step, counters, block advance ---------------------------------------
  if (!a.init_only) {
    float E = sh_f[0];
    if (gate_skips(E, a.tau, a.gate_metric)) { st.skip = 1; st.dt += 1; } else { st.skip = 0; st.dt = 0; }
    st.t_lastfull = t_lastfull;
    st.t = t + 1;
  }
  const bool sliding = a.schedule == EC_SCHED_SLIDING;
  int blk = st.blk;
  if (!sliding) {
    while (blk < nblocks) {  // uniform: every thread evaluates the same counts
      const int lo = blk * a.block, hi = min(N, lo + a.block);
      const int i = lo + tid;   // block <= EC_MAX_BLOCK <= threads
      if (__syncthreads_count(i < hi && s_msk[i]) > 0) break;
      ++blk;
    }
    st.blk = blk;
    st.done = (blk >= nblocks);
  }

  // ---- row lists of the next step: M and M u R, ascending ---------------------------------------
  // M = the masked rows of the current block, or (sliding window) the first `block` masked slots
  const int blo = blk * a.block, bhi = min(N, blo + a.block);   // in generation slots
  int n_rows = 0, n_mb = 0, n_recent = 0, masked_seen = 0;
  for (int base = 0; base < N; base += kDecideThreads) {
    const int i = base + tid, pos = P + i;
    int inM = 0, inR = 0, msk = 0;
    if (i < N) {
      msk = s_msk[i] ? 1 : 0;
      inM = (!sliding && !st.done && i >= blo && i < bhi && msk) ? 1 : 0;
      const int h = s_hist[i];
      inR = (!a.init_only && h != INT_MIN && h >= tauR) ? 1 : 0;
    }
    if (sliding) {
      int tot_msk;
      int pre_msk = block_excl_scan_flag(msk, scratch, &tot_msk);
      inM = (msk && masked_seen + pre_msk < a.block) ? 1 : 0;
      masked_seen += tot_msk;
    }
    int tot_any, tot_m;
    int pre_any = block_excl_scan_flag(inM | inR, scratch, &tot_any);
    int pre_m = block_excl_scan_flag(inM, scratch, &tot_m);
    const int tot_r = __syncthreads_count(inR);
    if (inM | inR) a.rows_partial[n_rows + pre_any] = pos;
    if (inM) {
      a.mb_pos[n_mb + pre_m] = pos;
      a.mb_idx[n_mb + pre_m] = n_rows + pre_any;
    }
    n_rows += tot_any;
    n_mb += tot_m;
    n_recent += tot_r;
  }
  if (sliding) st.done = (n_mb == 0);
  if (tid == 0) {
    st.n_mb = n_mb;
    st.n_rows_partial = n_rows;
    st.n_recent = n_recent;
    *a.st = st;
    StepOut& o = *a.out;
    o.next_n_mb = n_mb;
    o.next_n_rows_partial = n_rows;
    if (!a.init_only) {
      o.r.done = st.done;
      o.r.mode_run = a.mode_run;
      o.r.next_mode = gate_skips(sh_f[1], a.tau, a.gate_metric) ? EC_PARTIAL : EC_FULL;
      o.r.n_query_rows = a.n_rows_run;
      o.r.step_index = t;
      o.r.n_block_rows = a.n_mb;
      o.r.n_recent_next = n_recent;
    }
    // The result sits in pinned host memory.  The other threads' entries were stored before the
    // barriers above; this fence orders them and the fields above before the serial number, so
    // a host that sees the number sees the whole result.
    int bad = 0;
    if (!a.init_only)
      for (int r = 0; r < a.n_mb; ++r) bad |= s_badrow[r];
    o.nonfinite = bad;
    __threadfence_system();
    __hip_atomic_store(&o.serial, a.serial, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
  }
}

void launch_decide(const DecideArgs& a, int B, hipStream_t s) {
  const size_t smem = (size_t)((a.N + 3) & ~3) * 5;   // history (int) + mask set (byte)
  static size_t attr_bytes = 48 * 1024;
  if (smem > attr_bytes) {
    (void)hipFuncSetAttribute((const void*)decide_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                              (int)smem);
    attr_bytes = smem;
  }
  decide_kernel<<<B, kDecideThreads, smem, s>>>(a);
}

// ---------------------------------------------------------------------------------------------
// init_state: x = [prompt ; mask_id ...], mask set = generation slots, history = never,
// t = 1, flag = recompute, Delta t = 0 (initialisation lines of both algorithms).
// ---------------------------------------------------------------------------------------------
__global__ void init_state_kernel(int* x, uint8_t* masked, int* hist, DevState* st,
                                  const int* prompt, int P, int N, int mask_id) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < P + N) {
    x[i] = i < P ? prompt[i] : mask_id;
    masked[i] = i < P ? 0 : 1;
    if (i >= P) hist[i - P] = INT_MIN;
  }
  if (i == 0) {
    DevState z = {};
    z.t = 1;
    *st = z;
  }
}

void launch_init_state(int* x, uint8_t* masked, int* hist, DevState* st, const int* prompt_dev,
                       int P, int N, int mask_id, hipStream_t s) {
  int n = P + N;
  init_state_kernel<<<(n + 255) / 256, 256, 0, s>>>(x, masked, hist, st, prompt_dev, P, N, mask_id);
}

}  // namespace ec
