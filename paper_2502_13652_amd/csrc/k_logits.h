// Logits pass: one read of a logits row (or of one split of it) gives the softmax
// normaliser, the entropy sums (Eq. 2, first line) and the K largest logits with their
// token ids (Sec. 4.2.2, TopK purpose 1).
//
// Layout: a row is a sequence of 16-byte chunks (8 bf16 or 4 fp32 logits).  Workgroup
// (row, split) owns a contiguous range of chunks; lane t reads chunks t, t+NT, t+2NT, ...
// of that range, so every load instruction of the workgroup covers NT*16 contiguous bytes.
//
// Softmax sums are kept relative to a per-lane power-of-two reference 2^c (c integer valued),
// raised only if a later logit would overflow; references differ between lanes and are
// reconciled exactly (ldexp) in fp64 when the lanes are combined.
//
// Top-K without data-dependent work in the streaming loop: the loop only records each
// chunk's maximum ("cell key") in an LDS map.  Afterwards tau = K-th largest of the NT
// per-lane maxima is a lower bound of the K-th largest logit; only cells whose key reaches
// tau can hold a top-K element.  Those few cells are re-read (16 bytes each) and their
// elements ranked exactly by (logit desc, id asc).
#pragma once
#include "k_common.h"

namespace c2t {

constexpr int LP_NT = 256;          // threads per workgroup
constexpr int LP_NW = LP_NT / WAVE;
constexpr int LP_CELL_CAP = 256;    // candidate cells kept per workgroup (>= 2*K)
constexpr int LP_ELEM_CAP = LP_CELL_CAP * 8;
constexpr float LP_HEADROOM = 64.0f;   // a lane's terms stay below 2^(HEADROOM+1)

template <int DT> struct LogitTraits;
template <> struct LogitTraits<1> {     // bf16
  static constexpr int EPC = 8;         // elements per 16-byte chunk
  typedef uint16_t key_t;
  static __device__ __forceinline__ void unpack(const uint4& q, float (&x)[8]) {
    x[0] = bf16_lo(q.x); x[1] = bf16_hi(q.x); x[2] = bf16_lo(q.y); x[3] = bf16_hi(q.y);
    x[4] = bf16_lo(q.z); x[5] = bf16_hi(q.z); x[6] = bf16_lo(q.w); x[7] = bf16_hi(q.w);
  }
  static __device__ __forceinline__ key_t to_key(float cm) { return (key_t)(__float_as_uint(cm) >> 16); }
  static __device__ __forceinline__ float from_key(key_t k) { return __uint_as_float((uint32_t)k << 16); }
};
template <> struct LogitTraits<0> {     // fp32
  static constexpr int EPC = 4;
  typedef float key_t;
  static __device__ __forceinline__ void unpack(const uint4& q, float (&x)[4]) {
    x[0] = __uint_as_float(q.x); x[1] = __uint_as_float(q.y);
    x[2] = __uint_as_float(q.z); x[3] = __uint_as_float(q.w);
  }
  static __device__ __forceinline__ key_t to_key(float cm) { return cm; }
  static __device__ __forceinline__ float from_key(key_t k) { return k; }
};

struct LaneAcc {
  float Z0 = 0.f, Z1 = 0.f, S0 = 0.f, S1 = 0.f;
  float c = -INFINITY;      // reference exponent (integer valued) or -inf before the first finite logit
  float negc = 0.f;
  float thr = -INFINITY;    // raise the reference when a chunk maximum exceeds this
  float M = -INFINITY;      // running maximum of the lane
};

__device__ __forceinline__ void raise_reference(LaneAcc& a, float cm) {
  const float newc = ceilf(cm * L_HI);
  const float d = fmaxf(a.c - newc, -250.0f);             // <= 0 ; -inf on first use
  const float sc = __builtin_amdgcn_ldexpf(1.0f, (int)d);  // exact power of two
  a.S0 = (a.S0 + d * a.Z0) * sc; a.Z0 *= sc;
  a.S1 = (a.S1 + d * a.Z1) * sc; a.Z1 *= sc;
  a.c = newc; a.negc = -newc;
  a.thr = (newc + LP_HEADROOM) * (1.0f / L_HI);
}

template <int DT, bool MASKED>
__device__ __forceinline__ void consume_chunk(const uint4& q, LaneAcc& a, typename LogitTraits<DT>::key_t* map,
                                              int cell, int n_valid) {
  typedef LogitTraits<DT> T;
  float x[T::EPC];
  T::unpack(q, x);
  if (MASKED) {
#pragma unroll
    for (int j = 0; j < T::EPC; ++j) if (j >= n_valid) x[j] = -INFINITY;
  }
  float cm = x[0];
#pragma unroll
  for (int j = 1; j < T::EPC; ++j) cm = fmaxf(cm, x[j]);
  if (cm > a.thr) raise_reference(a, cm);
#pragma unroll
  for (int j = 0; j < T::EPC; ++j) {
    const float y = fmaf(x[j], L_LO, fmaf(x[j], L_HI, a.negc));
    const float e = hw_exp2(y);
    const float yc = fmaxf(y, -30000.0f);       // -inf logits: 0 * finite = 0 ; NaN still reaches Z through e
    if (j & 1) { a.Z1 += e; a.S1 = fmaf(e, yc, a.S1); }
    else       { a.Z0 += e; a.S0 = fmaf(e, yc, a.S0); }
  }
  a.M = fmaxf(a.M, cm);
  map[cell] = T::to_key(cm);
}

// grid: rows_launched * nsplit workgroups.  Dynamic LDS: max(cps * sizeof(key_t), LP_ELEM_CAP*8) bytes.
template <int DT>
__global__ __launch_bounds__(LP_NT) void k_logits_pass(
    const void* __restrict__ logits, int64_t row_stride_elems, int V, int K, int F, int rows_per_seq,
    const int32_t* __restrict__ n_frontier, int nsplit, int cps /* chunks per split */,
    RowPartial* __restrict__ part, float* __restrict__ part_topv, int32_t* __restrict__ part_topi) {
  typedef LogitTraits<DT> T;
  typedef typename T::key_t key_t;
  extern __shared__ __align__(16) unsigned char dyn_lds[];
  key_t* map = (key_t*)dyn_lds;
  __shared__ double red_d[2][LP_NW];
  __shared__ float red_f[2][LP_NW];
  __shared__ uint32_t lane_keys[LP_NT];
  __shared__ int32_t cell_list[LP_CELL_CAP];
  __shared__ int32_t scan_tmp[2][LP_NW];
  __shared__ uint32_t sh_tau;
  __shared__ int32_t sh_cnt[4];

  const int tid = threadIdx.x, lane = tid & (WAVE - 1), wid = tid >> 6;
  const int split = blockIdx.x % nsplit;
  const int rl = blockIdx.x / nsplit;
  const int b = rl / rows_per_seq, f = rl % rows_per_seq;
  if (f >= n_frontier[b]) return;                       // uniform for the workgroup
  const int64_t row = (int64_t)b * F + f;
  const int esz = DT == 1 ? 2 : 4;
  const uint4* rowp = (const uint4*)((const char*)logits + row * row_stride_elems * esz);

  const int n_chunks = (V + T::EPC - 1) / T::EPC;
  const int tail_valid = V - (n_chunks - 1) * T::EPC;  // elements of the last chunk that exist
  const int c0 = split * cps;
  int c1 = min(c0 + cps, n_chunks);
  if (c1 < c0) c1 = c0;
  const int ncell = c1 - c0;
  const bool has_tail = (c1 == n_chunks) && (tail_valid != T::EPC) && ncell > 0;
  const int c1_full = has_tail ? c1 - 1 : c1;

  // ---------------- streaming loop ----------------
  LaneAcc a;
  int g = c0 + tid;
  for (; g + 3 * LP_NT < c1_full; g += 4 * LP_NT) {
    const uint4 q0 = rowp[g], q1 = rowp[g + LP_NT], q2 = rowp[g + 2 * LP_NT], q3 = rowp[g + 3 * LP_NT];
    consume_chunk<DT, false>(q0, a, map, g - c0, 0);
    consume_chunk<DT, false>(q1, a, map, g - c0 + LP_NT, 0);
    consume_chunk<DT, false>(q2, a, map, g - c0 + 2 * LP_NT, 0);
    consume_chunk<DT, false>(q3, a, map, g - c0 + 3 * LP_NT, 0);
  }
  for (; g < c1_full; g += LP_NT) {
    const uint4 q0 = rowp[g];
    consume_chunk<DT, false>(q0, a, map, g - c0, 0);
  }
  if (has_tail && ((c1 - 1 - c0) % LP_NT) == tid) {
    const uint4 q0 = rowp[c1 - 1];
    consume_chunk<DT, true>(q0, a, map, c1 - 1 - c0, tail_valid);
  }

  // ---------------- combine the lanes (fp64, exact rescaling) ----------------
  float cw = wave_max(a.c), mw = wave_max(a.M);
  if (lane == 0) { red_f[0][wid] = cw; red_f[1][wid] = mw; }
  lane_keys[tid] = (a.M == -INFINITY && ncell <= tid) ? 0u : sortable_key(a.M);
  __syncthreads();
  float cref = red_f[0][0], mseg = red_f[1][0];
#pragma unroll
  for (int w = 1; w < LP_NW; ++w) { cref = fmaxf(cref, red_f[0][w]); mseg = fmaxf(mseg, red_f[1][w]); }
  double Zd = 0.0, Sd = 0.0;
  {
    const double Zl = (double)a.Z0 + (double)a.Z1, Sl = (double)a.S0 + (double)a.S1;
    if (a.c != -INFINITY && Zl != 0.0) {
      const double dl = fmax((double)a.c - (double)cref, -2000.0);
      const double sc = ldexp(1.0, (int)dl);
      Zd = Zl * sc;
      Sd = (Sl + dl * Zl) * sc;
    } else {
      Zd = Zl; Sd = Sl;     // zero, or NaN/inf to be reported
    }
  }
  Zd = wave_sum(Zd); Sd = wave_sum(Sd);
  if (lane == 0) { red_d[0][wid] = Zd; red_d[1][wid] = Sd; }

  // ---------------- tau = K-th largest of the lane maxima (wave 0) ----------------
  if (wid == 0) {
    uint32_t keys[LP_NW];
#pragma unroll
    for (int v = 0; v < LP_NW; ++v) keys[v] = lane_keys[v * WAVE + lane];
    const uint32_t tau = wave_kth_largest<LP_NW>(keys, K);
    if (lane == 0) sh_tau = tau;
  }
  __syncthreads();
  uint32_t tau_key = sh_tau;
  float tau = tau_key ? key_to_float(tau_key) : -INFINITY;

  // ---------------- scan the cell map: which cells can hold a top-K element ----------------
  const int cpl = (ncell + LP_NT - 1) / LP_NT;          // contiguous cells per lane
  const int s0 = min(tid * cpl, ncell), s1 = min(s0 + cpl, ncell);
  int n_gt_tot, take_eq;
  for (int attempt = 0;; ++attempt) {
    int n_gt = 0, n_eq = 0;
    for (int s = s0; s < s1; ++s) {
      const float kv = T::from_key(map[s]);
      n_gt += kv > tau; n_eq += kv == tau;
    }
    const int ig = wave_scan_incl(n_gt), ie = wave_scan_incl(n_eq);
    if (lane == WAVE - 1) { scan_tmp[0][wid] = ig; scan_tmp[1][wid] = ie; }
    __syncthreads();
    int og = 0, oe = 0, tg = 0, te = 0;
#pragma unroll
    for (int w = 0; w < LP_NW; ++w) {
      if (w < wid) { og += scan_tmp[0][w]; oe += scan_tmp[1][w]; }
      tg += scan_tmp[0][w]; te += scan_tmp[1][w];
    }
    n_gt_tot = tg;
    take_eq = min(te, K);
    if (tg + take_eq <= LP_CELL_CAP) {
      int pg = og + ig - n_gt, pe = oe + ie - n_eq;      // exclusive prefixes in cell order
      for (int s = s0; s < s1; ++s) {
        const float kv = T::from_key(map[s]);
        if (kv > tau) cell_list[pg++] = s;
        else if (kv == tau) { if (pe < take_eq) cell_list[tg + pe] = s; ++pe; }
      }
      break;
    }
    // Too many cells above the bound (maxima clustered in few lanes): find the exact K-th
    // largest cell key by radix select over the whole map; then fewer than K cells exceed it.
    __syncthreads();
    uint32_t prefix = 0, care = 0;
    int k = K;
    for (int bit = 31; bit >= 0; --bit) {
      const uint32_t want = prefix | (1u << bit), cmask = care | (1u << bit);
      int cnt = 0;
      for (int s = s0; s < s1; ++s) cnt += (sortable_key(T::from_key(map[s])) & cmask) == want;
      cnt = wave_sum_i(cnt);
      if (lane == 0) scan_tmp[0][wid] = cnt;
      __syncthreads();
      int tot = 0;
#pragma unroll
      for (int w = 0; w < LP_NW; ++w) tot += scan_tmp[0][w];
      __syncthreads();
      if (tot >= k) prefix = want; else k -= tot;
      care = cmask;
    }
    tau_key = prefix;
    tau = tau_key ? key_to_float(tau_key) : -INFINITY;
  }
  __syncthreads();
  const int n_cells = n_gt_tot + take_eq;

  // ---------------- re-read the candidate cells, keep elements >= tau ----------------
  // (the element list overlays the cell map, which is no longer needed)
  float* el_v = (float*)dyn_lds;
  int32_t* el_i = (int32_t*)(dyn_lds + LP_ELEM_CAP * 4);
  if (tid == 0) sh_cnt[0] = 0;
  int my_cell = -1;
  uint4 q = make_uint4(0, 0, 0, 0);
  if (tid < n_cells) { my_cell = c0 + cell_list[tid]; q = rowp[my_cell]; }
  __syncthreads();
  if (my_cell >= 0) {
    float x[T::EPC];
    T::unpack(q, x);
#pragma unroll
    for (int j = 0; j < T::EPC; ++j) {
      const int id = my_cell * T::EPC + j;
      if (id < V && x[j] >= tau) {
        const int slot = atomicAdd(&sh_cnt[0], 1);
        el_v[slot] = x[j]; el_i[slot] = id;
      }
    }
  }
  __syncthreads();
  const int n_el = sh_cnt[0];
  const int n_top = min(n_el, K);

  // ---------------- exact ranking of the few candidates ----------------
  const int64_t po = (int64_t)rl * nsplit + split;      // partial records are indexed by launched row
  for (int e = tid; e < n_el; e += LP_NT) {
    const float v = el_v[e]; const int id = el_i[e];
    int rank = 0;
    for (int o = 0; o < n_el; ++o) {
      const float vo = el_v[o];
      rank += (vo > v) || (vo == v && el_i[o] < id);
    }
    if (rank < K) { part_topv[po * K + rank] = v; part_topi[po * K + rank] = id; }
  }
  if (tid == 0) {
    double Zt = 0.0, St = 0.0;
#pragma unroll
    for (int w = 0; w < LP_NW; ++w) { Zt += red_d[0][w]; St += red_d[1][w]; }
    RowPartial r;
    r.Z = Zt; r.S2 = St; r.c = cref; r.m = mseg; r.n_top = n_top;
    r.flags = (Zt != Zt || Zt == INFINITY || St != St) ? 1u : 0u;
    part[po] = r;
  }
}

// Plain streaming read: the practical HBM ceiling.
__global__ __launch_bounds__(256) void k_stream_read(const uint4* __restrict__ p, size_t n16, uint32_t* out) {
  uint32_t acc = 0;
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * 256;
  for (; i + 3 * stride < n16; i += 4 * stride) {
    const uint4 a = p[i], b = p[i + stride], c = p[i + 2 * stride], d = p[i + 3 * stride];
    acc += a.x ^ a.y ^ a.z ^ a.w; acc += b.x ^ b.y ^ b.z ^ b.w;
    acc += c.x ^ c.y ^ c.z ^ c.w; acc += d.x ^ d.y ^ d.z ^ d.w;
  }
  for (; i < n16; i += stride) { const uint4 a = p[i]; acc += a.x ^ a.y ^ a.z ^ a.w; }
  acc = (uint32_t)wave_sum_i((int)acc);
  if ((threadIdx.x & 63) == 0 && acc == 0x9e3779b9u) atomicAdd(out, acc);   // keeps the loads alive
}

}  // namespace c2t
