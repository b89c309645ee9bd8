// Shared device helpers for the C2T kernels (gfx950, 64-wide wavefronts).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace c2t {

constexpr int WAVE = 64;

// Optional build (-DC2T_PHASE_TIMES): thread 0 of every workgroup of the layer kernel notes the time
// (100 MHz wall clock) at which it passes each phase boundary; c2t_phase_times_read copies the notes
// out.  In the normal build the marks expand to nothing.
constexpr int PT_WORKGROUPS = 8192, PT_SLOTS = 16;
enum PhaseMark { PT_START = 0, PT_STREAM_END, PT_HIST_COMPLETE, PT_SUMS, PT_TAU, PT_CELLS_LISTED, PT_CELLS_READ, PT_RANKED,
                 PT_PUBLISHED, PT_TICKET, PT_PRUNED, PT_PRUNE_LOADED, PT_PRUNE_FIRST, PT_PRUNE_PRESELECTED, PT_PRUNE_RANKED, PT_MERGED };
#ifdef C2T_PHASE_TIMES
__device__ unsigned long long c2t_phase_times[PT_WORKGROUPS * PT_SLOTS];
#define C2T_PT(i) do { if (threadIdx.x == 0 && blockIdx.x < c2t::PT_WORKGROUPS) c2t::c2t_phase_times[blockIdx.x * c2t::PT_SLOTS + (i)] = wall_clock64(); } while (0)
#else
#define C2T_PT(i) do { } while (0)
#endif

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

// the record of an empty segment
__device__ __forceinline__ RowPartial empty_partial() {
  RowPartial r;
  r.ref = -INFINITY; r.a = 0.0; r.Z = 0.0; r.S = 0.0; r.n_top = 0; r.flags = 0u;
  return r;
}

// Device-coherent accesses for data one workgroup writes and another reads inside the same kernel:
// they go to the coherence point, so neither side needs cache-wide write-backs or invalidations.
__device__ __forceinline__ void st_dev(uint32_t* p, uint32_t v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ void st_dev(int32_t* p, int32_t v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ void st_dev(float* p, float v) { st_dev((uint32_t*)p, __float_as_uint(v)); }
__device__ __forceinline__ void st_dev(double* p, double v) {
  __hip_atomic_store((unsigned long long*)p, (unsigned long long)__double_as_longlong(v), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ int32_t ld_dev(const int32_t* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ uint32_t ld_dev(const uint32_t* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ float ld_dev(const float* p) { return __uint_as_float(ld_dev((const uint32_t*)p)); }
__device__ __forceinline__ double ld_dev(const double* p) {
  return __longlong_as_double((long long)__hip_atomic_load((const unsigned long long*)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
}
__device__ __forceinline__ void st_dev(RowPartial* p, const RowPartial& r) {
  st_dev(&p->ref, r.ref); st_dev(&p->a, r.a); st_dev(&p->Z, r.Z); st_dev(&p->S, r.S);
  st_dev(&p->n_top, r.n_top); st_dev(&p->flags, r.flags);
}
__device__ __forceinline__ RowPartial ld_dev(const RowPartial* p) {
  RowPartial r;
  r.ref = ld_dev(&p->ref); r.a = ld_dev(&p->a); r.Z = ld_dev(&p->Z); r.S = ld_dev(&p->S);
  r.n_top = ld_dev(&p->n_top); r.flags = ld_dev(&p->flags);
  return r;
}
// every vector memory operation this wave has issued is complete
__device__ __forceinline__ void wait_vector_memory() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

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

// ---- wavefront reductions and scan on DPP (data-parallel primitives: lane permutations inside
// the VALU, no LDS round trip).  Rows are groups of 16 lanes.  The combination order is fixed, so
// floating-point results are reproducible.
#define C2T_DPP_QUAD_XOR1 0xB1      /* quad_perm [1,0,3,2] */
#define C2T_DPP_QUAD_XOR2 0x4E      /* quad_perm [2,3,0,1] */
#define C2T_DPP_ROW_HALF_MIRROR 0x141
#define C2T_DPP_ROW_MIRROR 0x140
#define C2T_DPP_ROW_BCAST15 0x142
#define C2T_DPP_ROW_BCAST31 0x143
#define C2T_DPP_ROW_SHR(n) (0x110 | (n))

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t identity, uint32_t v) {
  return (uint32_t)__builtin_amdgcn_update_dpp((int)identity, (int)v, CTRL, ROW_MASK, 0xf, false);
}
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_f32(float identity, float v) {
  return __uint_as_float(dpp_u32<CTRL, ROW_MASK>(__float_as_uint(identity), __float_as_uint(v)));
}
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ double dpp_f64(double v) {      // identity 0.0
  const uint64_t u = (uint64_t)__double_as_longlong(v);
  const uint32_t lo = dpp_u32<CTRL, ROW_MASK>(0u, (uint32_t)u), hi = dpp_u32<CTRL, ROW_MASK>(0u, (uint32_t)(u >> 32));
  return __longlong_as_double((long long)(((uint64_t)hi << 32) | lo));
}
__device__ __forceinline__ uint32_t readlane63_u32(uint32_t v) { return (uint32_t)__builtin_amdgcn_readlane((int)v, 63); }

// every lane of a row gets the row's result; then lane 63 gets the wave's (read it with readlane63)
template <typename Op>
__device__ __forceinline__ uint32_t wave_reduce_u32(uint32_t v, uint32_t ident, Op op) {
  v = op(v, dpp_u32<C2T_DPP_QUAD_XOR1, 0xf>(ident, v));
  v = op(v, dpp_u32<C2T_DPP_QUAD_XOR2, 0xf>(ident, v));
  v = op(v, dpp_u32<C2T_DPP_ROW_HALF_MIRROR, 0xf>(ident, v));
  v = op(v, dpp_u32<C2T_DPP_ROW_MIRROR, 0xf>(ident, v));
  v = op(v, dpp_u32<C2T_DPP_ROW_BCAST15, 0xa>(ident, v));
  v = op(v, dpp_u32<C2T_DPP_ROW_BCAST31, 0xc>(ident, v));
  return readlane63_u32(v);
}
__device__ __forceinline__ float wave_max(float v) {
  return __uint_as_float(wave_reduce_u32(__float_as_uint(v), __float_as_uint(-INFINITY),
                                         [](uint32_t a, uint32_t b) { return __float_as_uint(fmaxf(__uint_as_float(a), __uint_as_float(b))); }));
}
__device__ __forceinline__ int wave_sum_i(int v) {
  return (int)wave_reduce_u32((uint32_t)v, 0u, [](uint32_t a, uint32_t b) { return a + b; });
}
__device__ __forceinline__ double wave_sum(double v) {
  v = v + dpp_f64<C2T_DPP_QUAD_XOR1, 0xf>(v);
  v = v + dpp_f64<C2T_DPP_QUAD_XOR2, 0xf>(v);
  v = v + dpp_f64<C2T_DPP_ROW_HALF_MIRROR, 0xf>(v);
  v = v + dpp_f64<C2T_DPP_ROW_MIRROR, 0xf>(v);
  v = v + dpp_f64<C2T_DPP_ROW_BCAST15, 0xa>(v);
  v = v + dpp_f64<C2T_DPP_ROW_BCAST31, 0xc>(v);
  const uint64_t u = (uint64_t)__double_as_longlong(v);
  const uint32_t lo = readlane63_u32((uint32_t)u), hi = readlane63_u32((uint32_t)(u >> 32));
  return __longlong_as_double((long long)(((uint64_t)hi << 32) | lo));
}
// inclusive prefix sum across the wave (Hillis-Steele inside each row, then row carries)
__device__ __forceinline__ int wave_scan_incl(int v) {
  uint32_t u = (uint32_t)v;
  u += dpp_u32<C2T_DPP_ROW_SHR(1), 0xf>(0u, u);
  u += dpp_u32<C2T_DPP_ROW_SHR(2), 0xf>(0u, u);
  u += dpp_u32<C2T_DPP_ROW_SHR(4), 0xf>(0u, u);
  u += dpp_u32<C2T_DPP_ROW_SHR(8), 0xf>(0u, u);
  u += dpp_u32<C2T_DPP_ROW_BCAST15, 0xa>(0u, u);
  u += dpp_u32<C2T_DPP_ROW_BCAST31, 0xc>(0u, u);
  return (int)u;
}

// Partial rank of an entry with value v (its own index: self) in a list of n values in LDS: how many of the
// entries first4, first4 + 1, .. first4 + 3, first4 + step4, ... come before it in the order (value desc, then
// `ahead_at_tie(index)` among equal values).  Four values per LDS read, the reads independent of each other, where a
// read per value has every step wait out the LDS latency (a merge of 40 list entries: 1.5 us).
// vals 16-byte aligned, first4 and step4 multiples of 4; up to three floats past the n-th are read and ignored.
template <typename AheadAtTie>
__device__ __forceinline__ int count_ahead4(const float* vals, int n, int first4, int step4, float v, int self, AheadAtTie ahead_at_tie) {
  int rank = 0;
  for (int o = first4; o < n; o += step4) {
    const float4 q = *(const float4*)(vals + o);
    const float qa[4] = {q.x, q.y, q.z, q.w};
    uint32_t eq = 0;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const bool in = o + t < n;
      rank += in && qa[t] > v; eq |= (in && qa[t] == v ? 1u : 0u) << t;
    }
    if (self >= o && self < o + 4) eq &= ~(1u << (self - o));   // not the entry itself
    while (eq) {                                                // ties: rare
      const int t = __ffs(eq) - 1; eq &= eq - 1;
      rank += ahead_at_tie(o + t) ? 1 : 0;
    }
  }
  return rank;
}

// K-th largest (k >= 1) of the keys held by one wave, NV keys per lane (invalid keys = 0,
// the smallest key).  Radix select from the most significant bit with wave ballots; the
// result is wave-uniform.  If fewer than k keys are valid the result is 0.
// LOW_BIT > 0: the select stops above that bit and the result has its low bits clear: the largest
// such key that at least k keys reach (a lower bound of the k-th largest, for a fraction of the steps).
template <int NV, int LOW_BIT = 0>
__device__ __forceinline__ uint32_t wave_kth_largest(const uint32_t (&key)[NV], int k) {
  uint32_t prefix = 0, care = 0;
  for (int bit = 31; bit >= LOW_BIT; --bit) {
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
