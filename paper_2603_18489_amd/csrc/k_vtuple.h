// (max, argmax, sum e^(z-max), sum e^(z-max) (z-max)) tuples: the one-pass form of Eq. 1.
// A row's softmax statistics follow from its tuple: confidence = 1 / S, entropy = ln S - T / S.
// Tuples of disjoint parts of the vocabulary merge associatively (re-basing both to the common
// maximum), so partial reductions can be combined in any FIXED order with bit-reproducible
// results.  Shared by the decision kernels and the LM-head epilogue.
#pragma once
#include <hip/hip_runtime.h>
#include <limits.h>

namespace ec {

struct VTuple {
  float m;   // running maximum
  int idx;   // its index (lowest index among equal maxima)
  float s;   // sum exp(z - m)
  float t;   // sum exp(z - m) * (z - m)
};

__device__ __forceinline__ VTuple vt_identity() { return {-INFINITY, INT_MAX, 0.f, 0.f}; }

// Associative merge: re-base both sides to the common maximum.
__device__ __forceinline__ VTuple vt_merge(const VTuple& a, const VTuple& b) {
  if (b.s == 0.f) return a;
  if (a.s == 0.f) return b;
  VTuple r;
  bool a_wins = (a.m > b.m) || (a.m == b.m && a.idx < b.idx);
  r.m = fmaxf(a.m, b.m);
  r.idx = a_wins ? a.idx : b.idx;
  float da = a.m - r.m, db = b.m - r.m;  // <= 0
  float ea = expf(da), eb = expf(db);
  r.s = a.s * ea + b.s * eb;
  r.t = ea * (a.t + da * a.s) + eb * (b.t + db * b.s);
  return r;
}

__device__ __forceinline__ void vt_push(VTuple& v, float z, int idx) {
  if (z == -INFINITY) return;  // probability 0 contributes 0 (0 ln 0 := 0)
  if (z > v.m) {  // new maximum: re-base what was accumulated so far
    if (v.s != 0.f) {
      float d = v.m - z, e = expf(d);
      v.t = e * (v.t + d * v.s);
      v.s = v.s * e;
    }
    v.m = z;
    v.idx = idx;
    v.s += 1.f;
  } else {
    float d = z - v.m, e = expf(d);
    v.s += e;
    v.t += e * d;
  }
}

__device__ __forceinline__ VTuple vt_shfl_down(const VTuple& v, int o) {
  VTuple r;
  r.m = __shfl_down(v.m, o, 64);
  r.idx = __shfl_down(v.idx, o, 64);
  r.s = __shfl_down(v.s, o, 64);
  r.t = __shfl_down(v.t, o, 64);
  return r;
}

// xor-shuffle of a whole tuple
__device__ __forceinline__ VTuple vt_shfl_xor(const VTuple& v, int o) {
  VTuple r;
  r.m = __shfl_xor(v.m, o, 64);
  r.idx = __shfl_xor(v.idx, o, 64);
  r.s = __shfl_xor(v.s, o, 64);
  r.t = __shfl_xor(v.t, o, 64);
  return r;
}
__device__ __forceinline__ float4 vt_pack(const VTuple& v) {
  return make_float4(v.m, __int_as_float(v.idx), v.s, v.t);
}
__device__ __forceinline__ VTuple vt_unpack(const float4& q) {
  return VTuple{q.x, __float_as_int(q.y), q.z, q.w};
}
// Eq. 1 from a row's merged tuple: confidence = max probability = e^0 / S, entropy
// H = -sum p ln p = ln S - T / S (clamped at 0 against rounding).
__device__ __forceinline__ void vt_finish(const VTuple& v, float& conf, float& H) {
  conf = 1.0f / v.s;
  H = fmaxf(logf(v.s) - v.t / v.s, 0.f);
}

}  // namespace ec
