// Shared device helpers for the C2T kernels (gfx950, 64-wide wavefronts).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace c2t {

constexpr int WAVE = 64;

// Per (row, split) result of the logits pass: Z = sum_j e^(x_j - a), S = sum_j (x_j - ref) e^(x_j - a),
// both fp64, where ref is the segment's largest logit and the exponent offset a is ref (two-pass
// path) or 0 (histogram path, whose table holds e^v itself).
struct __attribute__((aligned(16))) RowPartial {
  double ref;     // largest logit of the segment (exact); -inf for an empty or all -inf segment
  double a;       // offset of the sums
  double Z;
  double S;
  int32_t n_top;  // entries of the segment's top list that are valid (<= K)
  uint32_t flags; // bit 0: NaN or +inf seen; bit 1 (informational): a bf16 segment took the two-pass path
};

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// monotone map float -> uint32 (total order of the reals; -0 and +0 map to the same key)
__device__ __forceinline__ uint32_t sortable_key(float x) {
  uint32_t u = __float_as_uint(x + 0.0f);   // -0 + 0 = +0
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float key_to_float(uint32_t k) {
  uint32_t u = (k & 0x80000000u) ? (k & 0x7fffffffu) : ~k;
  return __uint_as_float(u);
}

__device__ __forceinline__ int lane_id() {
  return __builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, WAVE));
  return v;
}
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, WAVE);
  return v;
}
__device__ __forceinline__ int wave_sum_i(int v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, WAVE);
  return v;
}
// inclusive prefix sum across the wave
__device__ __forceinline__ int wave_scan_incl(int v) {
  const int l = lane_id();
#pragma unroll
  for (int o = 1; o < WAVE; o <<= 1) {
    int t = __shfl_up(v, o, WAVE);
    if (l >= o) v += t;
  }
  return v;
}

// K-th largest (k >= 1) of the keys held by one wave, NV keys per lane (invalid keys = 0,
// the smallest key).  Radix select from the most significant bit with wave ballots; the
// result is wave-uniform.  If fewer than k keys are valid the result is 0.
template <int NV>
__device__ __forceinline__ uint32_t wave_kth_largest(const uint32_t (&key)[NV], int k) {
  uint32_t prefix = 0, care = 0;
  for (int bit = 31; bit >= 0; --bit) {
    const uint32_t want = prefix | (1u << bit);
    const uint32_t cmask = care | (1u << bit);
    int cnt = 0;
#pragma unroll
    for (int v = 0; v < NV; ++v) cnt += __popcll(__ballot((key[v] & cmask) == want));
    if (cnt >= k) prefix = want; else k -= cnt;
    care = cmask;
  }
  return prefix;
}

}  // namespace c2t
