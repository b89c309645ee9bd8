// Logits pass: one read of a logits row (or of one split of it) gives the softmax
// normaliser, the entropy sums (Eq. 2, first line) and the K largest logits with their
// token ids (Sec. 4.2.2, TopK purpose 1).
//
// Layout: a row is a sequence of 16-byte chunks (8 bf16 or 4 fp32 logits).  Workgroup
// (row, split) owns a contiguous range of chunks; lane t reads chunks t, t+NT, t+2NT, ...
// of that range, so every load instruction of the workgroup covers NT*16 contiguous bytes.
//
// Why the sums are exact.  Which children survive the two prunings is decided by comparing
// classifier logits that are often only an ulp apart (siblings with tiny joint probability
// share H and d), so the features must round to the same fp32 values as an fp64 evaluation
// of the definition: fp32 exponentials are not enough.  Two paths deliver fp64-grade sums:
//  * bf16 rows (the fast path): a bf16 logit has at most 65536 values, and all logits of
//    practical rows lie in 32 binades, |x| in [2^-25, 2^7).  The streaming loop only COUNTS
//    values: one LDS atomic per element into an 8192-bin histogram (sign, 5 exponent bits,
//    7 mantissa bits; two 16-bit counters per LDS word, overflow detected through the total).
//    Afterwards Z = sum_v n_v e^v and S = sum_v n_v (v-m) e^v are formed in fp64 from small
//    tables of exponentials: exact counts, <= 8192 fp64 terms, independent of the order in which
//    the elements were read.  Logits below the window (zeros included) are counted apart:
//    e^x = 1 + x to fp64 accuracy for |x| < 2^-25.  So are masked logits, -inf or a finite
//    x <= -2^10 (the masked tokens of constrained decoding): they add exactly nothing to either
//    sum and rank after every window value.
//  * any other row (fp32 logits; bf16 rows holding a logit >= 2^7 or in (-2^10, -2^7], +inf or
//    a NaN, a value held by more than 65535 logits, or below-window or masked logits that could
//    rank among the K largest): two passes over the segment with fp64 exponentials per element.
//
// Top-K without data-dependent work in the streaming loop: the loop records the maximum of each
// cell as a "cell key" in an LDS map.  A cell is one chunk (fp32) or the four chunks a lane reads
// in four consecutive sweeps of the workgroup (bf16: chunks i, i+NT, i+2NT, i+3NT of the segment).
// Afterwards a bound tau <= K-th largest logit is known (exactly, from the histogram; or as the
// K-th largest per-lane maximum), only cells whose key reaches tau can hold a top-K element, and
// those few cells are re-read and their elements ranked exactly by (logit desc, id asc).
#pragma once
#include "k_common.h"
#include "k_tree.h"

namespace c2t {

constexpr int SEL_CELL_CAP = 256;              // size of the candidate-cell list
#ifndef C2T_TAU_LOW_BIT
#define C2T_TAU_LOW_BIT 16
#endif

// LDS the selection may use once the cell list is built: the element list ((value, id), 8 bytes
// an entry, overlaying histogram and cell map) and the number of cells a launch may keep:
// min(SEL_CELL_CAP, NT / CPC, list entries / elements per cell), which the host keeps >= 2K - 1.
struct SelectLds {
  unsigned char* list;
  int list_cap;       // entries
  int cell_cap;
};
template <int NT, int CPC, int EPC>
__device__ __forceinline__ SelectLds make_select_lds(unsigned char* base, int bytes) {
  SelectLds s;
  s.list = base; s.list_cap = bytes / 8;
  s.cell_cap = min(min(SEL_CELL_CAP, NT / CPC), s.list_cap / (CPC * EPC));
  return s;
}

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

// A logits chunk is read once per layer: a non-temporal load keeps the stream from evicting what
// the workgroups reuse (the e^v table, the classifier) from the L2.
typedef uint32_t c2t_uint4v __attribute__((ext_vector_type(4)));
// 16 bytes at descriptor base + lane offset + scalar offset, non-temporal; zeros past the descriptor's size
__device__ __forceinline__ uint4 load_stream_buffer(__amdgpu_buffer_rsrc_t rs, uint32_t lane_off, uint32_t scalar_off) {
  const c2t_uint4v v = __builtin_amdgcn_raw_buffer_load_b128(rs, lane_off, scalar_off, 2);
  return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ uint4 load_stream(const uint4* p) {
  const c2t_uint4v v = __builtin_nontemporal_load((const c2t_uint4v*)p);
  return make_uint4(v.x, v.y, v.z, v.w);
}

// Range of chunks a (row, split) workgroup owns.
struct Segment {
  int c0, c1;        // chunks [c0, c1)
  int ncell;         // c1 - c0
  int tail_chunk;    // index of the row's last, partially valid chunk if it lies in [c0,c1), else -1
  int tail_valid;    // its number of valid elements
};
template <int EPC>
__device__ __forceinline__ Segment make_segment(int V, int split, int cps) {
  Segment s;
  const int n_chunks = (V + EPC - 1) / EPC;
  s.c0 = min(split * cps, n_chunks);
  s.c1 = min(s.c0 + cps, n_chunks);
  s.ncell = s.c1 - s.c0;
  s.tail_valid = V - (n_chunks - 1) * EPC;
  s.tail_chunk = (s.c1 == n_chunks && s.tail_valid != EPC && s.ncell > 0) ? n_chunks - 1 : -1;
  return s;
}

// Cells of a segment of n chunks.  CPC = 4: sweep s of the workgroup reads chunks [s*NT, (s+1)*NT);
// cell (s/4)*NT + t holds the chunks that lane t reads in sweeps 4*(s/4) .. 4*(s/4)+3.
template <int NT, int CPC>
__host__ __device__ inline int cells_in_segment(int n) {
  if (CPC == 1) return n;
  const int full = n / (4 * NT), rem = n - full * 4 * NT;
  return full * NT + (rem < NT ? rem : NT);
}
// chunk j (0 <= j < CPC) of a cell, as an index into the segment; may lie past its end
template <int NT, int CPC>
__device__ __forceinline__ int chunk_of_cell(int cell, int j) {
  if (CPC == 1) return cell;
  const int grp = cell / NT, t = cell - grp * NT;
  return grp * 4 * NT + j * NT + t;
}

// ---------------------------------------------------------------------------------------
// Selection, shared by both paths.
// ---------------------------------------------------------------------------------------

// Cells whose key reaches tau (exceeds it, if strict) are pushed to cell_list, in any order.
// Returns how many there are; if that is more than cell_cap the list is incomplete.
template <int DT, int NT>
__device__ __forceinline__ int list_cells(const typename LogitTraits<DT>::key_t* map, int ncells, float tau, bool strict,
                                          int cell_cap, int32_t* cell_list, int32_t* sh_n) {
  typedef LogitTraits<DT> T;
  if (threadIdx.x == 0) *sh_n = 0;
  __syncthreads();
#pragma unroll 1
  for (int c = threadIdx.x; c < ncells; c += NT) {
    const float kv = T::from_key(map[c]);
    if (strict ? kv > tau : kv >= tau) {
      const int slot = atomicAdd(sh_n, 1);
      if (slot < cell_cap) cell_list[slot] = c;
    }
  }
  __syncthreads();
  return *sh_n;
}

// Re-read the listed cells (CPC chunks each, one chunk per thread) and append their elements that
// reach tau (exceed it, if strict) to the element list, which overlays the cell map: the caller has
// put a barrier after the last read of the map and after setting *sh_cnt = 0.  Ends with a barrier.
template <int DT, int NT, int CPC>
__device__ __forceinline__ void collect_cells(const uint4* __restrict__ rowp, int c0, int c1, int V, float tau, bool strict,
                                              const int32_t* cell_list, int n_cells, const SelectLds& sel, int32_t* sh_cnt) {
  typedef LogitTraits<DT> T;
  const int tid = threadIdx.x;
  float* el_v = (float*)sel.list;
  int32_t* el_i = (int32_t*)(sel.list + (size_t)sel.list_cap * 4);
  int my_chunk = -1;
  uint4 q = make_uint4(0, 0, 0, 0);
  if (tid < n_cells * CPC) {                                 // n_cells <= cell_cap <= NT / CPC
    const int ch = c0 + chunk_of_cell<NT, CPC>(cell_list[tid / CPC], tid % CPC);
    if (ch < c1) { my_chunk = ch; q = rowp[ch]; }
  }
  if (my_chunk >= 0) {
    float x[T::EPC];
    T::unpack(q, x);
#pragma unroll
    for (int j = 0; j < T::EPC; ++j) {
      const int id = my_chunk * T::EPC + j;
      if (id < V && (strict ? x[j] > tau : x[j] >= tau)) {
        const int slot = atomicAdd(sh_cnt, 1);
        if (slot < sel.list_cap) { el_v[slot] = x[j]; el_i[slot] = id; }
      }
    }
  }
  __syncthreads();
}

// Massive ties: append the `need` lowest-id elements equal to tau, found by sweeping the segment in
// id order (one chunk per thread and sweep, prefix counts across the workgroup) until enough are seen.
template <int DT, int NT>
__device__ __forceinline__ void tie_scan(const uint4* __restrict__ rowp, const Segment& sg, int V, float tau, int need,
                                         const SelectLds& sel, int32_t* sh_cnt, int32_t (*scan_tmp)[NT / WAVE]) {
  typedef LogitTraits<DT> T;
  constexpr int NW = NT / WAVE;
  const int tid = threadIdx.x, lane = tid & (WAVE - 1), wid = tid >> 6;
  float* el_v = (float*)sel.list;
  int32_t* el_i = (int32_t*)(sel.list + (size_t)sel.list_cap * 4);
  int found = 0;                                             // uniform
#pragma unroll 1
  for (int base = sg.c0; base < sg.c1 && found < need; base += NT) {
    const int g = base + tid;
    uint32_t hit = 0;
    if (g < sg.c1) {
      float x[T::EPC];
      T::unpack(rowp[g], x);
#pragma unroll
      for (int j = 0; j < T::EPC; ++j) hit |= (g * T::EPC + j < V && x[j] == tau ? 1u : 0u) << j;
    }
    const int cnt = __popc(hit);
    const int incl = wave_scan_incl(cnt);
    if (lane == WAVE - 1) scan_tmp[0][wid] = incl;
    __syncthreads();
    int before = found + incl - cnt, total = 0;
#pragma unroll
    for (int w = 0; w < NW; ++w) { if (w < wid) before += scan_tmp[0][w]; total += scan_tmp[0][w]; }
    while (hit && before < need) {
      const int j = __ffs(hit) - 1; hit &= hit - 1;
      const int slot = atomicAdd(sh_cnt, 1);
      if (slot < sel.list_cap) { el_v[slot] = tau; el_i[slot] = g * T::EPC + j; }
      ++before;
    }
    found += total;
    __syncthreads();
  }
}

// Rank the element list exactly by (logit desc, id asc) and write the best K.
template <int NT>
__device__ __forceinline__ int rank_list(int K, const SelectLds& sel, const int32_t* sh_cnt, float* topv, int32_t* topi) {
  const int tid = threadIdx.x;
  const float* el_v = (const float*)sel.list;
  const int32_t* el_i = (const int32_t*)(sel.list + (size_t)sel.list_cap * 4);
  const int n_el = min(*sh_cnt, sel.list_cap);
  if (n_el <= 64) {
    // short list (the usual case: K to 2K-1 elements): T lanes per element, each compares it with
    // every T-th entry, one value per step; the partial ranks are summed over the T lanes
    int tshift = 0;
    while (tshift < 4 && (n_el << (tshift + 1)) <= NT) ++tshift;
    const int T = 1 << tshift, e = tid >> tshift, sub = tid & (T - 1);
    const bool mine = e < n_el;
    const float v = mine ? el_v[e] : 0.f; const int id = mine ? el_i[e] : 0;
    int rank = 0;
    if (mine) {
      for (int o = sub; o < n_el; o += T) {
        const float q = el_v[o];
        if (q > v) rank += 1;
        else if (q == v && o != e) rank += el_i[o] < id;
      }
    }
    if (tshift >= 1) rank += (int)dpp_u32<C2T_DPP_QUAD_XOR1, 0xf>(0u, (uint32_t)rank);
    if (tshift >= 2) rank += (int)dpp_u32<C2T_DPP_QUAD_XOR2, 0xf>(0u, (uint32_t)rank);
    if (tshift >= 3) rank += (int)dpp_u32<C2T_DPP_ROW_HALF_MIRROR, 0xf>(0u, (uint32_t)rank);
    if (tshift >= 4) rank += (int)dpp_u32<C2T_DPP_ROW_MIRROR, 0xf>(0u, (uint32_t)rank);
    if (mine && sub == 0 && rank < K) { topv[rank] = v; topi[rank] = id; }
    return min(n_el, K);
  }
#pragma unroll 1
  for (int e = tid; e < n_el; e += NT) {
    const float v = el_v[e]; const int id = el_i[e];
    int rank = 0;
    // eight values per step (entries past n_el are masked): every dependent LDS read is slow while
    // the neighbouring workgroups fill their histograms
#pragma unroll 1
    for (int o = 0; o < n_el; o += 8) {
      const float4 qa = *(const float4*)(el_v + o), qb = *(const float4*)(el_v + o + 4);
      const float vo[8] = {qa.x, qa.y, qa.z, qa.w, qb.x, qb.y, qb.z, qb.w};
      uint32_t eq = 0;
#pragma unroll
      for (int t = 0; t < 8; ++t) {
        const bool in = o + t < n_el;
        rank += in && vo[t] > v; eq |= (in && vo[t] == v ? 1u : 0u) << t;
      }
      eq &= ~(e >= o && e < o + 8 ? 1u << (e - o) : 0u);    // not the element itself
      while (eq) { const int t = __ffs(eq) - 1; eq &= eq - 1; rank += el_i[o + t] < id; }
    }
    if (rank < K) { topv[rank] = v; topi[rank] = id; }
  }
  return min(n_el, K);
}

// Sum of Z and S over the workgroup in a fixed order (wave butterflies, then waves ascending).
// Only thread 0 needs the totals: it leaves them in out[0..1] (LDS), so no lane keeps the
// per-wave partials alive in registers.
template <int NT>
__device__ __forceinline__ void block_sum2(double Z, double S, double (*red)[NT / WAVE], double* out) {
  constexpr int NW = NT / WAVE;
  Z = wave_sum(Z); S = wave_sum(S);
  if ((threadIdx.x & (WAVE - 1)) == 0) { red[0][threadIdx.x >> 6] = Z; red[1][threadIdx.x >> 6] = S; }
  __syncthreads();
  if (threadIdx.x == 0) {
    double tz = 0.0, ts = 0.0;
#pragma unroll 1
    for (int w = 0; w < NW; ++w) { tz += red[0][w]; ts += red[1][w]; }
    out[0] = tz; out[1] = ts;
  }
}
template <int NT>
__device__ __forceinline__ float block_max(float v, float* red /*[NT/WAVE]*/) {
  constexpr int NW = NT / WAVE;
  v = wave_max(v);
  __syncthreads();
  if ((threadIdx.x & (WAVE - 1)) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  float t = red[0];
#pragma unroll
  for (int w = 1; w < NW; ++w) t = fmaxf(t, red[w]);
  return t;
}

// ---------------------------------------------------------------------------------------
// Generic path: two passes over the segment, fp64 exponentials.  Any dtype, any values.
// ---------------------------------------------------------------------------------------
// Sums of e^(x-m) and (x-m) e^(x-m) over the M largest logits of the segment (ties at the M-th
// value: any of the equal logits, they contribute the same).  The M-th largest value is found
// exactly by a radix select over the order-preserving 32-bit keys, 8 bits per pass over the segment
// (an LDS histogram of the digit among the elements that match the prefix so far); one more pass
// sums the terms above it.  out[0..1] in LDS, valid after the caller's next barrier.
template <int DT, int NT>
__device__ __forceinline__ void top_m_sums(const uint4* __restrict__ rowp, const Segment& sg, int M, float m,
                                           double (*red)[NT / WAVE], double* out) {
  typedef LogitTraits<DT> T;
  __shared__ uint32_t dig[256];
  __shared__ int32_t sh_digit, sh_above, sh_total;
  const int tid = threadIdx.x, lane = tid & (WAVE - 1);
  uint32_t prefix = 0, care = 0;
  int remaining = M;
  bool take_all = false;
#pragma unroll 1
  for (int shift = 24; shift >= 0; shift -= 8) {
    for (int i = tid; i < 256; i += NT) dig[i] = 0u;
    __syncthreads();
    for (int g = sg.c0 + tid; g < sg.c1; g += NT) {
      float x[T::EPC];
      T::unpack(rowp[g], x);
      const int nv = (g == sg.tail_chunk) ? sg.tail_valid : T::EPC;
#pragma unroll
      for (int j = 0; j < T::EPC; ++j) {
        const uint32_t key = sortable_key(x[j]);
        if (j < nv && (key & care) == prefix) atomicAdd(&dig[(key >> shift) & 255u], 1u);
      }
    }
    __syncthreads();
    if (tid < WAVE) {                                        // wave 0: lane l owns digits 255-4l .. 252-4l
      uint32_t c[4]; int tot = 0;
#pragma unroll
      for (int j = 0; j < 4; ++j) { c[j] = dig[255 - (4 * lane + j)]; tot += (int)c[j]; }
      const int incl = wave_scan_incl(tot);
      int run = incl - tot;                                  // elements with larger digits
      if (run < remaining && incl >= remaining) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          if (run < remaining && run + (int)c[j] >= remaining) { sh_digit = 255 - (4 * lane + j); sh_above = run; }
          run += (int)c[j];
        }
      }
      if (lane == WAVE - 1) sh_total = incl;
    }
    __syncthreads();
    if (sh_total < remaining) { take_all = true; break; }   // fewer matching elements than wanted: only in the first pass
    remaining -= sh_above;
    prefix |= (uint32_t)sh_digit << shift; care |= 255u << shift;
    __syncthreads();
  }
  // prefix = key of the M-th largest logit; `remaining` (>= 1) of the logits equal to it are taken
  double Z = 0.0, S = 0.0;
  const double md = (double)m;
  for (int g = sg.c0 + tid; g < sg.c1; g += NT) {
    float x[T::EPC];
    T::unpack(rowp[g], x);
    const int nv = (g == sg.tail_chunk) ? sg.tail_valid : T::EPC;
#pragma unroll
    for (int j = 0; j < T::EPC; ++j) {
      if (j < nv && x[j] > -INFINITY && (take_all || sortable_key(x[j]) > prefix)) {
        const double t = (double)x[j] - md, e = exp(t);
        Z += e;
        if (e > 0.0) S += t * e;
      }
    }
  }
  if (!take_all && tid == 0) {
    const float xt = key_to_float(prefix);
    if (xt > -INFINITY) { const double t = (double)xt - md, e = exp(t); Z += remaining * e; if (e > 0.0) S += remaining * (t * e); }
  }
  block_sum2<NT>(Z, S, red, out);
}

// A row that was split over several workgroups: the M largest logits of the ROW cannot be told from
// the splits' own sums, so the workgroup that merged the row goes over the whole row once more
// (five passes of one workgroup: a rare configuration, fp32 rows of more than 49152 logits or bf16
// rows of more than 262144, with the entropy over the M largest).  Sums relative to the row maximum.
template <int DT, int NT>
__device__ __forceinline__ void top_m_of_split_row(const uint4* __restrict__ rowp, int V, int M, RowResult& rr) {
  if (M <= 0) return;
  __shared__ double red_t[2][NT / WAVE], sum_t[2];
  const bool usable = !(rr.part.flags & 1u) && rr.part.Z > 0.0 && rr.part.ref > -INFINITY && rr.part.ref < INFINITY;
  if (usable) {
    constexpr int EPC = LogitTraits<DT>::EPC;
    const Segment whole = make_segment<EPC>(V, 0, (V + EPC - 1) / EPC);
    top_m_sums<DT, NT>(rowp, whole, M, (float)rr.part.ref, red_t, sum_t);
  }
  __syncthreads();
  if (threadIdx.x == 0) { rr.ZM = usable ? sum_t[0] : 0.0; rr.SM = usable ? sum_t[1] : 0.0; }
  __syncthreads();
}

// map_lds: one key per cell.
template <int DT, int NT, int CPC>
__device__ __noinline__ void generic_segment(const uint4* __restrict__ rowp, int V, int K, int top_m, const Segment sg,
                                unsigned char* map_lds, const SelectLds sel, RowResult* rr, uint32_t info_flags) {
  typedef LogitTraits<DT> T;
  typedef typename T::key_t key_t;
  constexpr int NW = NT / WAVE;
  static_assert(CPC == 1 || CPC == 4, "a cell is one chunk or four sweeps of a lane");
  key_t* map = (key_t*)map_lds;
  const int ncells = cells_in_segment<NT, CPC>(sg.ncell);
  __shared__ double red_d[2][NW], sum_d[2], sum_m[2];
  __shared__ float red_f[NW];
  __shared__ uint32_t lane_keys[NT];
  __shared__ int32_t cell_list[SEL_CELL_CAP];
  __shared__ int32_t scan_tmp[2][NW];
  __shared__ uint32_t sh_tau;
  __shared__ int32_t sh_cnt, sh_bad;
  const int tid = threadIdx.x, lane = tid & (WAVE - 1), wid = tid >> 6;
  if (tid == 0) sh_bad = 0;
  __syncthreads();

  // pass 1: cell keys, lane maxima, NaN / +inf
  float M = -INFINITY;
  bool bad = false, any = false;
  float cell_max = -INFINITY;
  int sweep = 0;
  for (int g = sg.c0 + tid; g < sg.c1; g += NT, ++sweep) {
    const uint4 q = rowp[g];
    float x[T::EPC];
    T::unpack(q, x);
    const int nv = (g == sg.tail_chunk) ? sg.tail_valid : T::EPC;
    float cm = -INFINITY;
#pragma unroll
    for (int j = 0; j < T::EPC; ++j) {
      if (j < nv) { bad |= !(x[j] < INFINITY); cm = fmaxf(cm, x[j]); }
    }
    M = fmaxf(M, cm);
    if (CPC == 1) map[g - sg.c0] = T::to_key(cm);
    else {
      cell_max = fmaxf(cell_max, cm);
      if ((sweep & 3) == 3 || g + NT >= sg.c1) { map[(sweep >> 2) * NT + tid] = T::to_key(cell_max); cell_max = -INFINITY; }
    }
    any = true;
  }
  lane_keys[tid] = any ? sortable_key(M) : 0u;
  if (bad) sh_bad = 1;
  const float m = block_max<NT>(M, red_f);          // barriers inside also publish map, lane_keys, sh_bad
  const bool seg_bad = sh_bad != 0;
  C2T_PT(PT_STREAM_END);                            // (the marks of the histogram path, at the corresponding steps)

  // pass 2: Z = sum e^(x-m), S = sum (x-m) e^(x-m)
  double Z = 0.0, S = 0.0;
  if (!seg_bad && m > -INFINITY) {
    const double md = (double)m;
    for (int g = sg.c0 + tid; g < sg.c1; g += NT) {
      const uint4 q = rowp[g];
      float x[T::EPC];
      T::unpack(q, x);
      const int nv = (g == sg.tail_chunk) ? sg.tail_valid : T::EPC;
#pragma unroll
      for (int j = 0; j < T::EPC; ++j) {
        if (j < nv && x[j] > -INFINITY) {
          const double t = (double)x[j] - md;
          const double e = exp(t);
          Z += e;
          if (e > 0.0) S += t * e;
        }
      }
    }
  }
  block_sum2<NT>(Z, S, red_d, sum_d);
  C2T_PT(PT_SUMS);
  if (top_m > 0) {
    __syncthreads();
    if (!seg_bad && m > -INFINITY) top_m_sums<DT, NT>(rowp, sg, top_m, m, red_d, sum_m);
    else if (tid == 0) { sum_m[0] = 0.0; sum_m[1] = 0.0; }
    __syncthreads();
  }

  // tau = K-th largest of the lane maxima, to its upper 16 bits (half the select's steps, each a
  // ballot per key; a few more elements pass): a lower bound of the K-th largest logit
  if (wid == 0) {
    uint32_t keys[NW];
#pragma unroll
    for (int v = 0; v < NW; ++v) keys[v] = lane_keys[v * WAVE + lane];
    uint32_t t = wave_kth_largest<NW, C2T_TAU_LOW_BIT>(keys, K);
    // -inf's key with its low bits cleared is no number's key; every key that reaches it is at least -inf's
    const uint32_t key_neg_inf = 0x007FFFFFu;             // = sortable_key(-INFINITY)
    if (t != 0u && t < key_neg_inf) t = key_neg_inf;
    if (lane == 0) sh_tau = t;
  }
  __syncthreads();
  C2T_PT(PT_TAU);
  uint32_t tau_key = sh_tau;
  float tau = tau_key ? key_to_float(tau_key) : -INFINITY;
  bool ties = false;
  int n_cells = list_cells<DT, NT>(map, ncells, tau, false, sel.cell_cap, cell_list, &sh_cnt);
  if (n_cells > sel.cell_cap) {
    // Too many cells reach the bound (maxima clustered in few lanes): take the exact K-th
    // largest cell key by radix select over the whole map; fewer than K cells exceed it.
    const int cpl = (ncells + NT - 1) / NT;
    const int s0 = min(tid * cpl, ncells), s1 = min(s0 + cpl, ncells);
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
      for (int w = 0; w < NW; ++w) tot += scan_tmp[0][w];
      __syncthreads();
      if (tot >= k) prefix = want; else k -= tot;
      care = cmask;
    }
    tau = prefix ? key_to_float(prefix) : -INFINITY;
    n_cells = list_cells<DT, NT>(map, ncells, tau, false, sel.cell_cap, cell_list, &sh_cnt);
    if (n_cells > sel.cell_cap) {                            // massive ties at tau: the cells above it, then a tie scan
      n_cells = list_cells<DT, NT>(map, ncells, tau, true, sel.cell_cap, cell_list, &sh_cnt);
      ties = true;
    }
  }
  if (tid == 0) sh_cnt = 0;
  __syncthreads();
  C2T_PT(PT_CELLS_LISTED);
  collect_cells<DT, NT, CPC>(rowp, sg.c0, sg.c1, V, tau, ties, cell_list, n_cells, sel, &sh_cnt);
  if (ties) tie_scan<DT, NT>(rowp, sg, V, tau, K, sel, &sh_cnt, scan_tmp);
  C2T_PT(PT_CELLS_READ);
  const int n_top = rank_list<NT>(K, sel, &sh_cnt, rr->topv, rr->topi);
  C2T_PT(PT_RANKED);
  if (tid == 0) {
    RowPartial r;
    r.ref = (double)m; r.a = (double)m; r.Z = sum_d[0]; r.S = sum_d[1]; r.n_top = seg_bad ? 0 : n_top; r.flags = (seg_bad ? 1u : 0u) | info_flags;
    rr->part = r;
    if (top_m > 0) { rr->ZM = sum_m[0]; rr->SM = sum_m[1]; }
  }
}

// Workgroups of a sequence whose frontier is empty have nothing to read; the first of them
// records the empty next frontier (Algorithm 1's loop guard) in place of the scoring step.
__device__ __forceinline__ void end_of_sequence(const TreeState& st, const ScoreParams& sp, int b, int f, int split) {
  if (f == 0 && split == 0 && threadIdx.x == 0) { st.nf[(sp.layer + 1) & 1][b] = 0; st.n_cand[b] = 0; }
}

// Which frontier slot of which sequence a workgroup (index w among the launched rows) takes.
// A launch that fits the chip in one round (at most four workgroups per CU) is placed statically:
// workgroup w runs on CU w mod n_cus (HW_ID read-outs), so a CU hosts w, w + n_cus, w + 2 n_cus, ...
// Full layers run fastest in slot-major order (consecutive workgroups = the same slot of
// consecutive sequences: 2 % faster at B = 64 and B = 256 than sequence-major).  In a thinned-out
// layer the frontiers are of very different lengths (many sequences have used their budget up,
// others are still full), and a fixed order leaves some CUs with four live rows and others with
// none: the layer then takes as long as a full one.  With `compact` the workgroup takes the w-th
// LIVE row in slot-major order instead, which it finds from the frontier sizes alone (every wave
// by itself: one load per lane and at most launched/64 ballots, no atomics, no barrier): the live
// rows are dealt round the CUs, at most one more on one CU than on another.  Workgroups past the
// live rows take the sequences without a frontier (one each, for the loop guard) or exit.
struct RowOfWorkgroup { int b, f, nf; };
// position of the n-th set bit of m (n < popcount(m)); uniform over the wave
__device__ __forceinline__ int nth_set_bit(uint64_t m, int n) {
  const int lane = lane_id();
  const int below = (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
  const uint64_t hit = __builtin_amdgcn_ballot_w64(((m >> lane) & 1ull) != 0ull && below == n);
  return (int)__builtin_ctzll(hit);
}
constexpr int COMPACT_MAX_B = 256;            // frontier sizes held by one wave: four per lane
__device__ __forceinline__ RowOfWorkgroup row_of_workgroup(const TreeState& st, const ScoreParams& sp, int w) {
  const int* nfs = st.nf[sp.layer & 1];
  RowOfWorkgroup r;
  if (sp.compact) {
    const int lane = lane_id();
    int nfv[COMPACT_MAX_B / WAVE];
#pragma unroll
    for (int k = 0; k < COMPACT_MAX_B / WAVE; ++k) { const int i = lane + k * WAVE; nfv[k] = i < sp.B ? nfs[i] : -1; }
    int run = 0, b = -1, f = 0, nf = 0;
    for (int ff = 0; ff < sp.rows_per_seq && b < 0; ++ff) {
#pragma unroll
      for (int k = 0; k < COMPACT_MAX_B / WAVE; ++k) {
        if (k * WAVE >= sp.B) break;
        const uint64_t m = __builtin_amdgcn_ballot_w64(nfv[k] > ff);
        const int c = __builtin_popcountll(m);
        if (b < 0 && w < run + c) {
          const int bl = nth_set_bit(m, w - run);
          b = k * WAVE + bl; f = ff; nf = __builtin_amdgcn_readlane(nfv[k], bl);
        }
        run += c;
      }
    }
    if (b < 0) {                                          // run = all live rows of the layer
      int d = w - run;
#pragma unroll
      for (int k = 0; k < COMPACT_MAX_B / WAVE; ++k) {
        if (k * WAVE >= sp.B) break;
        const uint64_t m = __builtin_amdgcn_ballot_w64(nfv[k] == 0);
        const int c = __builtin_popcountll(m);
        if (b < 0 && d >= 0 && d < c) { b = k * WAVE + nth_set_bit(m, d); f = 0; nf = 0; }
        d -= c;
      }
    }
    if (b < 0) { b = 0; f = 1; nf = 1; }                 // nothing left for this workgroup
    r.b = __builtin_amdgcn_readfirstlane(b); r.f = __builtin_amdgcn_readfirstlane(f); r.nf = __builtin_amdgcn_readfirstlane(nf);
    return r;
  }
  const int b_seq = w / sp.rows_per_seq, b_slot = w % sp.B;
  const int nf_seq = nfs[b_seq], nf_slot = nfs[b_slot];         // both loads issued before the choice: no dependent round trip
  const bool slot_major = 4 * st.layer_rows[sp.layer] >= 3 * sp.B * sp.rows_per_seq;
  r.b = slot_major ? b_slot : b_seq;
  r.f = slot_major ? w / sp.B : w % sp.rows_per_seq;
  r.nf = slot_major ? nf_slot : nf_seq;
  return r;
}

// grid: rows_launched * nsplit workgroups of NT threads.
// Dynamic LDS (sp.lds_bytes): the cell map (cps keys), reused for the element list of the selection
// ((2K-1) * EPC entries of 8 bytes at least) and by the tail.
template <int DT, int NT>
__global__ __launch_bounds__(NT) void k_logits_generic(
    const void* __restrict__ logits, int64_t row_stride_elems, int V, int cps, const float* __restrict__ cls,
    TreeState st, ScoreParams sp) {
  typedef LogitTraits<DT> T;
  extern __shared__ __align__(16) unsigned char dyn_lds[];
  const int nsplit = sp.nsplit, K = sp.K;
  const int split = blockIdx.x % nsplit;
  const RowOfWorkgroup rw = row_of_workgroup(st, sp, blockIdx.x / nsplit);
  const int b = rw.b, f = rw.f, rl = b * sp.rows_per_seq + f, nf = rw.nf;
  if (f >= nf) { if (nf == 0) end_of_sequence(st, sp, b, f, split); return; }   // uniform for the workgroup
  const int64_t row = (int64_t)b * sp.F + f;
  const uint4* rowp = (const uint4*)((const char*)logits + row * row_stride_elems * (DT == 1 ? 2 : 4));
  const Segment sg = make_segment<T::EPC>(V, split, cps);
  __shared__ RowResult rr;
  C2T_PT(PT_START);
  if (threadIdx.x == 0) rr.parent_P = st.fr_P[row];        // off the tail's critical path
  if (sg.ncell == 0) { if (threadIdx.x == 0) { rr.part = empty_partial(); rr.ZM = 0.0; rr.SM = 0.0; } }
  else generic_segment<DT, NT, 1>(rowp, V, K, nsplit > 1 ? 0 : sp.M, sg, dyn_lds, make_select_lds<NT, 1, T::EPC>(dyn_lds, sp.lds_bytes), &rr, 0u);   // split rows: see top_m_of_split_row
  finish_layer<NT>(st, sp, b, f, nf, split, rl, rr, dyn_lds, cls, nullptr,     // split records are indexed by launched row
                   [&](RowResult& r) { top_m_of_split_row<DT, NT>(rowp, V, sp.M, r); });
}

// ---------------------------------------------------------------------------------------
// bf16 fast path: value histogram.
// ---------------------------------------------------------------------------------------
constexpr int HP_BINS = 8192;                 // sign(1) | exponent mod 32 (5) | mantissa (7)
constexpr int HP_WORDS = HP_BINS / 2;         // LDS words: low half counts +|v|, high half counts -|v|
constexpr int HP_CPC = 4;                     // chunks per cell of the map: four sweeps of a lane
constexpr uint32_t HP_MAG_LO = 102u << 7;     // |x| >= 2^-25
constexpr uint32_t HP_MAG_SPAN = 32u << 7;    // 32 binades: |x| < 2^7
constexpr uint32_t HP_WORD_ROT = HP_MAG_LO & (HP_WORDS - 1);   // word of magnitude index i: (i + ROT) mod 4096
constexpr uint32_t HP_F16_NEG_INF2 = 0xFC00FC00u;              // identity of the packed maximum

// value-ordered rank r in [0, 8192): larger r = larger value.  r -> bf16 code.
__device__ __forceinline__ uint32_t hp_code_of_rank(int r) {
  const uint32_t s = r < 4096 ? 1u : 0u;
  const uint32_t magidx = s ? (uint32_t)(4095 - r) : (uint32_t)(r - 4096);
  return (s << 15) | (HP_MAG_LO + magidx);
}
__device__ __forceinline__ float hp_value_of_mag(uint32_t magidx, bool negative) {
  return __uint_as_float(((HP_MAG_LO + magidx) << 16) | (negative ? 0x80000000u : 0u));
}

// e^v for the window's values, factored so that the table stays in cache and a lane holds few
// factors: v = s 2^E (1 + f/128), f = 16 fh + fl, and e^v = A[s][e][fh] * prod over the set bits k
// of fl of C[s][e][k], with A = exp(s 2^E (1 + fh/8)) and C = exp(s 2^E 2^k / 128) (every argument
// exact), e = exponent index inside the window (0..31).  Layout: A+ [256] | A- [256] | C+ [32][4] |
// C- [32][4] doubles (6 KB; a table of all 8192 values is 64 KB and was re-fetched from memory by
// nearly every workgroup).  At most five correctly rounded factors and four products: within
// 1e-15 of e^v.  Filled once per context.
constexpr int HP_TAB_A = 256, HP_TAB_C = 128, HP_TAB_DOUBLES = 2 * HP_TAB_A + 2 * HP_TAB_C;
__global__ void k_init_exp_table(double* __restrict__ tab) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= HP_TAB_DOUBLES) return;
  const bool is_c = i >= 2 * HP_TAB_A;
  const int k = is_c ? i - 2 * HP_TAB_A : i, half = is_c ? HP_TAB_C : HP_TAB_A;
  const bool neg = k >= half;
  const int kk = neg ? k - half : k;
  const int e = is_c ? kk >> 2 : kk >> 3, sub = is_c ? kk & 3 : kk & 7;
  const double p2 = ldexp(1.0, (int)(HP_MAG_LO >> 7) + e - 127);                 // 2^E
  const double arg = is_c ? p2 * (double)(1 << sub) / 128.0 : p2 * (1.0 + (double)sub / 8.0);
  tab[i] = exp(neg ? -arg : arg);
}
// The lane that owns magnitude indices 8t .. 8t+7 (one exponent, fh and bit 3 of fl fixed): the
// factors of e^(+|v_j|) and e^(-|v_j|).  Ten loads, twenty registers; the sixteen products are
// formed where they are used, one bin pair at a time.
struct ExpFactors { double ap, an, cp[4], cn[4]; };
__device__ __forceinline__ ExpFactors load_exp_factors(const double* __restrict__ tab, int tid) {
  const int mag0 = 8 * tid, e = mag0 >> 7, f0 = mag0 & 127;
  ExpFactors f;
  f.ap = tab[e * 8 + (f0 >> 4)]; f.an = tab[HP_TAB_A + e * 8 + (f0 >> 4)];
  const double2* cp = (const double2*)(tab + 2 * HP_TAB_A + e * 4);
  const double2* cn = (const double2*)(tab + 2 * HP_TAB_A + HP_TAB_C + e * 4);
  const double2 p0 = cp[0], p1 = cp[1], n0 = cn[0], n1 = cn[1];
  f.cp[0] = p0.x; f.cp[1] = p0.y; f.cp[2] = p1.x; f.cp[3] = p1.y;
  f.cn[0] = n0.x; f.cn[1] = n0.y; f.cn[2] = n1.x; f.cn[3] = n1.y;
  return f;
}

typedef _Float16 c2t_half2 __attribute__((ext_vector_type(2)));
typedef unsigned short c2t_ushort2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pk_max_f16(uint32_t a, uint32_t b) {
  return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(c2t_half2, a), __builtin_bit_cast(c2t_half2, b)));
}
// The same instruction without the canonicalising copies the builtin adds in front of it (an
// instruction per operand): for the streaming loop, whose patterns are never signalling NaNs that matter.
__device__ __forceinline__ uint32_t pk_max_f16_raw(uint32_t a, uint32_t b) {
  uint32_t d;
  asm("v_pk_max_f16 %0, %1, %2" : "=v"(d) : "v"(a), "v"(b));
  return d;
}
// per 16-bit half: a * b + c (mod 2^16)
__device__ __forceinline__ uint32_t pk_mad_u16(uint32_t a, uint32_t b_sgpr, uint32_t c) {
  uint32_t d;
  asm("v_pk_mad_u16 %0, %1, %2, %3" : "=v"(d) : "v"(a), "s"(b_sgpr), "v"(c));
  return d;
}
// bits 16..27 of w: the histogram word of the upper bf16 (written out because the compiler turns the
// bit-field extract into shift, mask and a separate add of the array base: one instruction more)
__device__ __forceinline__ uint32_t bits_16_27(uint32_t w) {
  uint32_t d;
  asm("v_bfe_u32 %0, %1, 16, 12" : "=v"(d) : "v"(w));
  return d;
}
// mask ? 65536 : 1 for mask = 0 or ~0: the histogram increment of a negative / positive value
__device__ __forceinline__ uint32_t hist_increment(int32_t sign_mask, uint32_t c65536_sgpr) {
  uint32_t d;
  asm("v_bfi_b32 %0, %1, %2, 1" : "=v"(d) : "v"(sign_mask), "s"(c65536_sgpr));
  return d;
}
__device__ __forceinline__ uint32_t pk_max_u16(uint32_t a, uint32_t b) {
  return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(c2t_ushort2, a), __builtin_bit_cast(c2t_ushort2, b)));
}
__device__ __forceinline__ uint32_t pk_min_u16(uint32_t a, uint32_t b) {
  return __builtin_bit_cast(uint32_t, __builtin_elementwise_min(__builtin_bit_cast(c2t_ushort2, a), __builtin_bit_cast(c2t_ushort2, b)));
}

// What the rows' rare logits add up to, per workgroup, in LDS: the streaming loop carries none of
// it in registers (four registers through the loop, and a copy of them per chunk, before).
struct OutsideAcc {
  double s_tiny;                    // sum of the logits with |x| < 2^-25 (zeros included): e^x = 1 + x to fp64 accuracy
  int32_t n_tiny;                   // their number
  int32_t n_masked;                 // masked logits (see hp_masked: probability 0, ranked last)
  uint32_t mag_max;                 // largest |code| seen outside the fast path: NaN, inf and |x| >= 2^7 show here
  uint32_t masked_by_lane[WAVE];    // masked logits again, counted where the rest of their chunk is in the window: lane l of every
                                    // wavefront adds to word l, in the half a negative value's count goes to (folded into n_masked)
};
typedef __attribute__((address_space(3))) OutsideAcc* OutsideAccLds;

// Chunks that hold a logit outside the window, and a row's partial last chunk (n_valid < 8).  Out
// of line: typical rows never get here, and inlined at each of the streaming loop's sites this
// code costs the whole kernel registers.  If everything outside the window is masked (see
// hp_masked), those logits are counted apart and the rest of the chunk is counted as in
// hist_chunk; otherwise one element at a time.
// Returns the maximum of the valid elements as a packed pattern; where all of them are masked, a
// value below every finite logit of the window path (a cell key only has to be an upper bound).
// Masked logits: -inf and every finite x <= -2^10 (the large negative constants used in place of
// -inf).  The row's largest logit is a window value, m > -2^7, so x - m < -896 and e^(x - m) is
// exactly 0 in fp64 (which underflows to 0 below -745.2): such a logit adds nothing to Z or S, and
// it ranks after every window value.  NaN codes (above 0xff80) are not in the range.
__device__ __forceinline__ bool hp_masked(uint32_t code16) { return code16 - 0xc480u <= 0xff80u - 0xc480u; }
__device__ __noinline__ uint32_t hist_chunk_outside(uint4 q, int n_valid, uint32_t* __restrict__ hist, OutsideAcc* acc_generic) {
  constexpr uint32_t TWO2 = 0x00020002u, BIAS2 = ((0x10000u - 2u * HP_MAG_LO) & 0xffffu) * 0x00010001u;
  constexpr uint32_t LOWEST = 0x8000u | (HP_MAG_LO + HP_MAG_SPAN - 1);   // the lowest value of the window stands in for a masked logit
  const OutsideAccLds acc = (OutsideAccLds)acc_generic;
  const uint32_t w[4] = {q.x, q.y, q.z, q.w};
  if (n_valid == 8) {
    uint32_t w2[4], inf_lo[4], inf_hi[4], dm = 0u;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      inf_lo[j] = hp_masked(w[j] & 0xffffu) ? ~0u : 0u;
      inf_hi[j] = hp_masked(w[j] >> 16) ? ~0u : 0u;
      w2[j] = w[j];
      if (inf_lo[j]) w2[j] = (w2[j] & 0xffff0000u) | LOWEST;
      if (inf_hi[j]) w2[j] = (w2[j] & 0x0000ffffu) | (LOWEST << 16);
      dm = pk_max_u16(dm, pk_mad_u16(w2[j], TWO2, BIAS2));
    }
    if (!(dm & 0xE000E000u)) {
      // Every lane issues all eight atomics, as for a chunk inside the window; a masked logit's goes to the
      // lane's own word of masked_by_lane instead of the histogram (one address select per logit: no
      // branches, no ballots, and the 64 words lie in 64 different places, so masked logits pile up nowhere).
      // The stand-in value is negative, so the count lands in the word's upper half.
      typedef __attribute__((address_space(3))) uint32_t* LdsWords;
      const LdsWords own = &acc->masked_by_lane[lane_id()], hl = (LdsWords)hist;   // LDS addresses: the selects stay 32-bit, the atomics ds_add
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const LdsWords a_hi = inf_hi[j] ? own : hl + bits_16_27(w2[j]);
        const LdsWords a_lo = inf_lo[j] ? own : hl + (w2[j] & (HP_WORDS - 1));
        __hip_atomic_fetch_add(a_hi, hist_increment((int32_t)w2[j] >> 31, 0x10000u), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        __hip_atomic_fetch_add(a_lo, hist_increment(__builtin_amdgcn_sbfe((int32_t)w2[j], 15, 1), 0x10000u), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
      }
      return pk_max_f16(pk_max_f16(w2[0], w2[1]), pk_max_f16(w2[2], w2[3]));
    }
  }
  float cm = -INFINITY;
  uint32_t mag_max = 0u;
  int n_tiny = 0, n_masked = 0;
  double s_tiny = 0.0;
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const float x = (j & 1) ? bf16_hi(w[j >> 1]) : bf16_lo(w[j >> 1]);
    const uint32_t code = __float_as_uint(x) >> 16, mag = code & 0x7fffu;
    if (j < n_valid) {
      if (hp_masked(code)) n_masked += 1;
      else {
        mag_max = max(mag_max, mag);
        cm = fmaxf(cm, x);
        if (mag < HP_MAG_LO) { n_tiny += 1; s_tiny += (double)x; }
        else atomicAdd(&hist[code & (HP_WORDS - 1)], (code & 0x8000u) ? 0x10000u : 1u);
      }
    }
  }
  if (n_masked) __hip_atomic_fetch_add(&acc->n_masked, n_masked, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
  if (n_tiny) {
    __hip_atomic_fetch_add(&acc->n_tiny, n_tiny, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    __hip_atomic_fetch_add(&acc->s_tiny, s_tiny, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
  }
  if (mag_max >= HP_MAG_LO + HP_MAG_SPAN) __hip_atomic_fetch_max(&acc->mag_max, mag_max, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
  const uint32_t c16 = cm == -INFINITY ? (HP_F16_NEG_INF2 & 0xffffu) : __float_as_uint(cm) >> 16;
  return c16 | (c16 << 16);
}

// Counts the values of a whole chunk; returns the chunk maximum as a packed pattern (both halves
// <= max, one of them equal to it).
__device__ __forceinline__ uint32_t hist_chunk(const uint4& q, uint32_t& M2, uint32_t* __restrict__ hist, OutsideAcc* acc) {
  const uint32_t w[4] = {q.x, q.y, q.z, q.w};
  // Per half d = 2 |code| - 2 LO (mod 2^16), with the sign shifted out by the doubling: the value
  // lies in the window iff d < 2 SPAN = 8192, i.e. iff bits 13..15 of d are clear.
  constexpr uint32_t TWO2 = 0x00020002u, BIAS2 = ((0x10000u - 2u * HP_MAG_LO) & 0xffffu) * 0x00010001u;
  static_assert(2 * HP_MAG_SPAN == 8192 && HP_WORDS == 4096, "window test and 12-bit word index below");
  const uint32_t dm = pk_max_u16(pk_max_u16(pk_mad_u16(w[0], TWO2, BIAS2), pk_mad_u16(w[1], TWO2, BIAS2)),
                                 pk_max_u16(pk_mad_u16(w[2], TWO2, BIAS2), pk_mad_u16(w[3], TWO2, BIAS2)));
  uint32_t pat;
  // rare: a logit outside the window.  The whole wave then takes the out-of-line routine (it counts
  // in-window chunks as well): cheaper than running both paths one after the other.
  if (__builtin_amdgcn_ballot_w64((dm & 0xE000E000u) != 0u) != 0ull) {   // (a hint that this is rare made the loop 10 % slower)
    pat = hist_chunk_outside(q, 8, hist, acc);
  } else {
    // inside the window bf16 bit patterns order exactly like fp16 bit patterns
    pat = pk_max_f16_raw(pk_max_f16_raw(w[0], w[1]), pk_max_f16_raw(w[2], w[3]));
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      // +1 into the low half for a positive value, into the high half for a negative one
      atomicAdd(&hist[bits_16_27(w[j])], hist_increment((int32_t)w[j] >> 31, 0x10000u));
      atomicAdd(&hist[w[j] & (HP_WORDS - 1)], hist_increment(__builtin_amdgcn_sbfe((int32_t)w[j], 15, 1), 0x10000u));
    }
  }
  M2 = pk_max_f16_raw(M2, pat);
  return pat;
}

// The lane that holds the M-th largest logit: the sums over the logits it contributes to the top M
// (from its top value down: positive magnitudes descending, or negative ones ascending), relative to
// its top value vt.  Out of line: one lane per row gets here, and inlined its registers would be
// charged to every workgroup's epilogue.  e^v is computed here (at most WPL values) rather than
// fetched from the tables again: a load issued at this point waits behind all the logits in flight
// on the CU, several microseconds that the whole workgroup would spend at its next barrier.
template <int WPL> struct LaneCounts { uint32_t w[WPL]; };      // by value: a reference would put the counts in scratch memory
struct TopMPart { double zm, sm; };
template <int WPL>
__device__ __noinline__ TopMPart top_m_boundary_lane(int tid, LaneCounts<WPL> counts, bool positive, int above, int M, double vt) {
  const uint32_t (&cw)[WPL] = counts.w;
  double zm = 0.0, sm = 0.0;
  int run = above;
#pragma unroll 1
  for (int jj = 0; jj < WPL; ++jj) {
    const int j = positive ? WPL - 1 - jj : jj;
    const int n = positive ? (int)(cw[j] & 0xffffu) : (int)(cw[j] >> 16), take = max(0, min(n, M - run));
    run += n;
    if (take) {
      const double v = (double)hp_value_of_mag(WPL * tid + j, !positive);
      const double t = (double)take * exp(v);
      zm += t; sm += (v - vt) * t;
    }
  }
  TopMPart r; r.zm = zm; r.sm = sm;
  return r;
}

// A thread's share of the classifier's parameters on its way from global memory to LDS.
struct ClassifierStage { float4 q; float* dst; bool mine; };
__device__ __forceinline__ ClassifierStage stage_classifier(const float* __restrict__ cls, int h, float* dst) {
  ClassifierStage c;
  c.dst = dst;
  c.mine = dst != nullptr && (int)threadIdx.x * 4 < 5 * h + 1;     // the array is padded to a multiple of four floats
  c.q = make_float4(0.f, 0.f, 0.f, 0.f);
  if (c.mine) c.q = ((const float4*)cls)[threadIdx.x];
  return c;
}
__device__ __forceinline__ void store_classifier(const ClassifierStage& c) {
  if (c.mine) ((float4*)c.dst)[threadIdx.x] = c.q;
}

// A row shared by sp.coop workgroups (launches that leave most of the chip idle: a single sequence,
// a root layer).  One workgroup counts a 256 KB row at the rate of its CU's LDS atomics, 9 us; n
// workgroups on n CUs count a segment each, and their histograms, being sums, merge exactly.  Each
// hands over through memory what the epilogue needs of its segment: the 4096 count words (copies
// already folded), the keys of its cells (segments are whole groups of four sweeps, so the row's
// map is the segments' maps laid end to end) and the few numbers of OutsideAcc.  The stores are
// device-coherent and complete before the workgroup takes the row's ticket; the workgroup that takes
// the last one adds the n histograms up in its own LDS, loads the row's map, and goes on as if it
// had counted the whole row.  The sums, the K-th largest value and the selection therefore come
// out exactly as for an unshared row (the sum of the logits below the window is added up per
// segment first: a different rounding order for a term of relative size 1e-16).
// Every slot is written once and read once per launch: nothing has to be cleared between launches.
// Returns true in the workgroup that goes on.  map: the segment's keys in LDS, with room for the row's.
constexpr int COOP_BATCH = 4;                   // other segments whose counts a lane has in flight at once (eight registers each)
template <int NT>
__device__ __forceinline__ bool share_row(const ScoreParams& sp, int split, int64_t row_launched, int32_t* row_ticket,
                                          const Segment& sg, uint32_t* __restrict__ hist, uint32_t w0, uint16_t* map,
                                          OutsideAcc* sh_out, uint32_t* red_m) {
  constexpr int NW = NT / WAVE;
  constexpr uint32_t SLOT_BYTES = HP_WORDS * 4, COHERENT = 16;          // cache policy sc1: served at the device's coherence point
  const int tid = threadIdx.x, lane = tid & (WAVE - 1), wid = tid >> 6;
  const int n = sp.coop;
  const __amdgpu_buffer_rsrc_t rh = __builtin_amdgcn_make_buffer_rsrc((void*)(sp.coop_hist + row_launched * n * HP_WORDS), 0,
                                                                      n * (int)SLOT_BYTES, 0x00020000);
  const __amdgpu_buffer_rsrc_t rm = __builtin_amdgcn_make_buffer_rsrc((void*)(sp.coop_map + row_launched * sp.coop_map_stride), 0,
                                                                      sp.coop_map_stride * 2, 0x00020000);
  CoopAcc* const acc = sp.coop_acc + row_launched * n;
  {
    const uint4 t0 = *(const uint4*)(hist + w0), t1 = *(const uint4*)(hist + w0 + 4);
    const c2t_uint4v u0 = {t0.x, t0.y, t0.z, t0.w}, u1 = {t1.x, t1.y, t1.z, t1.w};
    __builtin_amdgcn_raw_buffer_store_b128(u0, rh, w0 * 4u, (uint32_t)split * SLOT_BYTES, COHERENT);
    __builtin_amdgcn_raw_buffer_store_b128(u1, rh, w0 * 4u + 16u, (uint32_t)split * SLOT_BYTES, COHERENT);
    const int ncells = cells_in_segment<NT, HP_CPC>(sg.ncell);
    const uint32_t first_key_byte = (uint32_t)sg.c0 / HP_CPC * 2u;     // sg.c0 is a multiple of HP_CPC * NT chunks
    for (int i = tid * 8; i < ncells; i += NT * 8) {                    // (a store that reaches past the row's keys is dropped by the bounds check)
      const uint4 k = *(const uint4*)(map + i);
      const c2t_uint4v kv = {k.x, k.y, k.z, k.w};
      __builtin_amdgcn_raw_buffer_store_b128(kv, rm, (uint32_t)i * 2u, first_key_byte, COHERENT);
    }
    if (wid == NW - 1 && lane == 0) {                                   // the lane that has just folded masked_by_lane into n_masked
      uint32_t m2 = HP_F16_NEG_INF2;
#pragma unroll
      for (int w = 0; w < NW; ++w) m2 = pk_max_f16(m2, red_m[w]);
      CoopAcc* a = acc + split;
      st_dev(&a->s_tiny, sh_out->s_tiny);
      st_dev(&a->n_tiny, sh_out->n_tiny); st_dev(&a->n_masked, sh_out->n_masked);
      st_dev(&a->mag_max, sh_out->mag_max); st_dev(&a->max_pattern, m2);
    }
  }
  wait_vector_memory();                                                 // this wave's stores have reached the coherence point
  __syncthreads();                                                      // ... and every wave's; the reads of LDS above are done
  if (!last_arrival(row_ticket, n)) return false;

  // Every load of the first round trip is issued before anything waits: the segments' numbers
  // (wave 0, one segment per lane), the row's keys (two loads a thread cover the largest map) and the
  // first COOP_BATCH segments' counts.
  const bool have = wid == 0 && lane < n;
  const CoopAcc* a = acc + (have ? lane : 0);
  double st = 0.0; int nt = 0, nm = 0; uint32_t mm = 0u, mp = HP_F16_NEG_INF2;
  if (have) { st = ld_dev(&a->s_tiny); nt = ld_dev(&a->n_tiny); nm = ld_dev(&a->n_masked); mm = ld_dev(&a->mag_max); mp = ld_dev(&a->max_pattern); }
  const int k0 = tid * 8, k1 = k0 + NT * 8;
  const c2t_uint4v kv0 = __builtin_amdgcn_raw_buffer_load_b128(rm, (uint32_t)k0 * 2u, 0u, COHERENT);   // zeros past the row's keys
  const c2t_uint4v kv1 = __builtin_amdgcn_raw_buffer_load_b128(rm, (uint32_t)k1 * 2u, 0u, COHERENT);
  // The other n - 1 segments' counts, from the next segment on round the row; its own are still in LDS.
  uint4 c0 = *(const uint4*)(hist + w0), c1 = *(const uint4*)(hist + w0 + 4);
  for (int j0 = 0; j0 < n - 1; j0 += COOP_BATCH) {
    c2t_uint4v v[2 * COOP_BATCH];
#pragma unroll
    for (int j = 0; j < COOP_BATCH; ++j) {
      int sl = split + 1 + j0 + j;
      sl = sl >= n ? sl - n : sl;
      const uint32_t so = (j0 + j < n - 1) ? (uint32_t)sl * SLOT_BYTES : (uint32_t)n * SLOT_BYTES;   // past the last slot: zeros from the bounds check, no traffic
      v[2 * j] = __builtin_amdgcn_raw_buffer_load_b128(rh, w0 * 4u, so, COHERENT);
      v[2 * j + 1] = __builtin_amdgcn_raw_buffer_load_b128(rh, w0 * 4u + 16u, so, COHERENT);
    }
#pragma unroll
    for (int j = 0; j < COOP_BATCH; ++j) {                              // a carry out of a 16-bit half shows in the total, like a counter overflow
      c0.x += v[2 * j].x; c0.y += v[2 * j].y; c0.z += v[2 * j].z; c0.w += v[2 * j].w;
      c1.x += v[2 * j + 1].x; c1.y += v[2 * j + 1].y; c1.z += v[2 * j + 1].z; c1.w += v[2 * j + 1].w;
    }
  }
  *(uint4*)(hist + w0) = c0; *(uint4*)(hist + w0 + 4) = c1;             // only this lane reads these words before the next barrier
  if (k0 < sp.coop_map_stride) *(uint4*)(map + k0) = make_uint4(kv0.x, kv0.y, kv0.z, kv0.w);
  if (k1 < sp.coop_map_stride) *(uint4*)(map + k1) = make_uint4(kv1.x, kv1.y, kv1.z, kv1.w);
  for (int i = k1 + NT * 8; i < sp.coop_map_stride; i += NT * 8) {      // (longer maps than the launch code allows today)
    const c2t_uint4v kv = __builtin_amdgcn_raw_buffer_load_b128(rm, (uint32_t)i * 2u, 0u, COHERENT);
    *(uint4*)(map + i) = make_uint4(kv.x, kv.y, kv.z, kv.w);
  }
  if (wid == 0) {                                                       // fixed order of the sums
    const double st_all = wave_sum(st);
    const int nt_all = wave_sum_i(nt), nm_all = wave_sum_i(nm);
    const uint32_t mm_all = wave_reduce_u32(mm, 0u, [](uint32_t x, uint32_t y) { return max(x, y); });
    const uint32_t mp_all = wave_reduce_u32(mp, HP_F16_NEG_INF2, [](uint32_t x, uint32_t y) { return pk_max_f16(x, y); });
    if (lane == 0) { sh_out->s_tiny = st_all; sh_out->n_tiny = nt_all; sh_out->n_masked = nm_all; sh_out->mag_max = mm_all; }
    if (lane < NW) red_m[lane] = mp_all;
  }
  return true;                                                          // the caller's next barrier publishes map, sh_out and red_m
}

// One (row, split) segment on the histogram path, run by a whole workgroup of NT threads.
// hist: HP_WORDS words; map_lds: one 2-byte key per cell, padded to 16 bytes; sel: see SelectLds.
// TOPM: built with the entropy over the M largest logits (a separate instantiation, so that the
// default kernel carries none of its registers).
// COOP: built with the hand-over of a shared row (see share_row); returns false in the workgroups
// that have handed their segment over and are done, true in the one that holds the row's result.
template <int NT, bool TOPM, int WPS, int REPL, bool COOP>
__device__ __forceinline__ bool hist_segment(const uint4* __restrict__ rowp, int V, int K, int M, const Segment& sg_own,
                                             const double* __restrict__ tab_e, uint32_t* __restrict__ hist,
                                             unsigned char* map_lds, const SelectLds& sel, RowResult* rr,
                                             const ClassifierStage cst, const ScoreParams& sp, int split, int64_t row_launched,
                                             int32_t* row_ticket) {
  constexpr int NW = NT / WAVE;
  constexpr int WPL = HP_WORDS / NT;                   // words per lane in the epilogue (8 at 512 threads)
  static_assert(NW <= 16 && WPL % 4 == 0, "one DPP row holds the per-wave partials; a lane reads whole 16-byte runs");
  uint16_t* map = (uint16_t*)map_lds;
  __shared__ double red_d[2][NW], sum_d[2], sum_m[2];
  __shared__ float red_v[NW];
  __shared__ uint32_t red_m[NW];
  __shared__ OutsideAcc sh_out;
  __shared__ int32_t cell_list[SEL_CELL_CAP];
  __shared__ int32_t scan_tmp[2][NW];
  __shared__ int32_t sh_cnt, sh_ncell, sh_tau_rank, sh_n_gt;

  int tid = threadIdx.x;
  const int lane = tid & (WAVE - 1), wid = tid >> 6;
  Segment sg = sg_own;                                   // what the workgroup streams; the whole row once a shared row's counts are merged

#pragma unroll
  for (int j = 0; j < WPL * REPL; ++j) hist[tid + j * NT] = 0u;
  if (tid == 0) { sh_tau_rank = -1; sh_n_gt = 0; sh_ncell = 0; sh_out.s_tiny = 0.0; sh_out.n_tiny = 0; sh_out.n_masked = 0; sh_out.mag_max = 0u; }
  if (tid < WAVE) sh_out.masked_by_lane[tid] = 0u;
  __syncthreads();

  // ---------------- streaming loop: count values, record cell maxima ----------------
  uint32_t vo_after;
  uint32_t M2 = HP_F16_NEG_INF2;                       // packed running maximum of the bf16 patterns (compared as fp16 patterns)
  {
    // DEPTH chunks per lane in flight: a workgroup that streams while its neighbours on the CU are
    // in their epilogues still covers the HBM latency.  Unrolled by DEPTH so that each buffer is
    // refilled right after it has been counted, without register copies.  Eight in the build with
    // 80 registers, which has room for them (measured: no faster than four, also for a workgroup
    // that is alone on its CU: the CU's counting rate bounds it, not the latency of its loads).
    constexpr int DEPTH = WPS == 6 ? 8 : 4;
    const int c1 = sg.tail_chunk >= 0 ? sg.c1 - 1 : sg.c1;   // whole chunks; a partial last chunk is counted below
    // The whole chunks are read through a buffer descriptor over exactly their bytes: a lane whose
    // chunk lies past the last whole one gets zeros from the bounds check instead of needing a
    // compare and a select per load, and the address is the lane's fixed offset plus a scalar one:
    // no vector instruction per load (eight before, a seventh of the loop).
    const uint64_t base = (uint64_t)(rowp + sg.c0);      // the same for every lane: told to the compiler
    const uint64_t base_u = (uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)base) |   // the builtin returns int:
                            ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(base >> 32)) << 32);   // no sign extension
    const int whole = __builtin_amdgcn_readfirstlane(max(c1 - sg.c0, 0));
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc((void*)base_u, 0, whole * 16, 0x00020000);
    const uint32_t vo = (uint32_t)tid * 16u;
    uint32_t so = 0u;
#define C2T_LOAD(k) load_stream_buffer(rs, vo, so + (uint32_t)(k) * (NT * 16u))
    // REPL copies of the histogram, a lane counting into copy (lane mod REPL): neighbouring lanes that
    // hold the same value (common: few hundred values carry most of a row) then add to different
    // words, which the LDS does not have to serialise.  The copies are folded after the loop.
    static_assert(REPL == 1 || REPL == 2 || REPL == 4 || REPL == 8, "a lane picks its copy with a mask");
    uint32_t* __restrict__ histl = hist + (REPL > 1 ? (tid & (REPL - 1)) * HP_WORDS : 0);
#define C2T_COUNT(q) hist_chunk(q, M2, histl, &sh_out)
    uint4 q[DEPTH];
#pragma unroll
    for (int k = 0; k < DEPTH; ++k) q[k] = C2T_LOAD(k);
    uint16_t* mp = map + tid;
    // Streaming waves issue ahead of the waves of co-resident workgroups that are in their
    // (latency-bound) epilogue or tail: the memory pipeline stays fed.  Measured: 3 % per full layer.
    __builtin_amdgcn_s_setprio(3);
    // groups of DEPTH sweeps in which every lane has a chunk; a cell is four sweeps
    const int n_groups = whole / (DEPTH * NT);
    for (int it = n_groups; it > 0; --it, so += (uint32_t)DEPTH * NT * 16u, mp += (DEPTH / 4) * NT) {
#pragma unroll
      for (int c = 0; c < DEPTH / 4; ++c) {
        uint32_t key = C2T_COUNT(q[4 * c]);
        q[4 * c] = C2T_LOAD(DEPTH + 4 * c);
#pragma unroll
        for (int k = 1; k < 4; ++k) {
          key = pk_max_f16_raw(key, C2T_COUNT(q[4 * c + k]));
          q[4 * c + k] = C2T_LOAD(DEPTH + 4 * c + k);
        }
        mp[c * NT] = (uint16_t)pk_max_f16_raw(key, key >> 16);
      }
    }
    vo_after = vo;
    C2T_PT(PT_STREAM_END);
    store_classifier(cst);                               // published by the barriers below
    const int g0 = sg.c0 + (int)(vo >> 4) + n_groups * (DEPTH * NT);
    __builtin_amdgcn_s_setprio(0);
    // the last, partial group: up to DEPTH chunks of this lane, the row's partial last chunk among them
    const int tail = sg.tail_chunk;
#pragma unroll
    for (int c = 0; c < DEPTH / 4; ++c) {
      const int g = g0 + 4 * c * NT;
      if (g < c1 || g == tail) {
        uint32_t key = g < c1 ? C2T_COUNT(q[4 * c]) : hist_chunk_outside(rowp[tail], sg.tail_valid, hist, &sh_out);
#pragma unroll
        for (int k = 1; k < 4; ++k) {
          if (g + k * NT < c1) key = pk_max_f16_raw(key, C2T_COUNT(q[4 * c + k]));
          else if (g + k * NT == tail) key = pk_max_f16(key, hist_chunk_outside(rowp[tail], sg.tail_valid, hist, &sh_out));
        }
        mp[c * NT] = (uint16_t)pk_max_f16(key, key >> 16);
        M2 = pk_max_f16(M2, key);                         // the partial chunk's maximum is in no other running value
      }
    }
#undef C2T_COUNT
#undef C2T_LOAD
  }
  // The thread index should not be kept in a register through the loop on top of the lane's
  // buffer offset: a spill that crosses the loop is reloaded behind all the logits in flight on the
  // CU (microseconds, for every wave).  It is formed again here: from the offset, or, where the
  // register allocation of that build comes out better, from the wave's index and the lane.
  if (TOPM && WPS == 8) tid = __builtin_amdgcn_readfirstlane(wid) * WAVE + lane_id();
  else tid = (int)(vo_after >> 4);

  // The lane owns the magnitude indices WPL*tid .. WPL*tid + WPL-1, with both signs.  The table
  // loads for their e^v are issued now so that their latency hides behind the barrier.
  static_assert(WPL == 8, "a lane's magnitudes share one exponent, one upper fraction and bit 3 of the lower");
  const bool shared_row = COOP && sp.coop > 1;          // (uniform) then the factors are loaded behind the hand-over: they would
  ExpFactors ef;                                        // only take registers from it
  if (!shared_row) ef = load_exp_factors(tab_e, tid);
  // per-wave: maximum
  {
    const uint32_t m2 = wave_reduce_u32(M2, HP_F16_NEG_INF2, [](uint32_t x, uint32_t y) { return pk_max_f16(x, y); });
    if (lane == 0) red_m[wid] = m2;
  }
  __syncthreads();                                     // histogram, cell map and wave results complete
  C2T_PT(PT_HIST_COMPLETE);
  if (wid == NW - 1) {                                  // masked logits counted by lane: folded into the one count (read after the next barrier)
    const int nm = wave_sum_i((int)(sh_out.masked_by_lane[lane] >> 16));
    if (lane == 0 && nm) sh_out.n_masked += nm;         // every other addition to it happened before the barrier above
  }

  // ---------------- Z = sum n_v e^v and S = sum n_v (v - m) e^v ----------------
  // S is accumulated against the largest value seen so far at each level (lane, wave, workgroup),
  // so every term has the same sign and nothing cancels: rows whose entropy is tiny keep their
  // relative accuracy.
  double Z = 0.0, S = 0.0, Zp = 0.0, Sp = 0.0;
  int lane_pos = 0, lane_neg = 0;
  float vtop = -INFINITY;                               // value of the lane's highest non-empty bin
  const uint32_t w0 = ((uint32_t)(WPL * tid) + HP_WORD_ROT) & (HP_WORDS - 1);   // the lane's words; WPL-aligned: no wrap inside
  if (REPL > 1) {                                       // fold the copies into the first: only this lane touches these words
#pragma unroll
    for (int j = 0; j < WPL; j += 4) {
      uint4 t = *(const uint4*)(hist + w0 + j);
#pragma unroll
      for (int r = 1; r < REPL; ++r) {
        const uint4 u = *(const uint4*)(hist + r * HP_WORDS + w0 + j);
        t.x += u.x; t.y += u.y; t.z += u.z; t.w += u.w;  // a carry out of a 16-bit half shows in the total, like a counter overflow
      }
      *(uint4*)(hist + w0 + j) = t;
    }
  }
  if (shared_row) {
    if (!share_row<NT>(sp, split, row_launched, row_ticket, sg, hist, w0, map, &sh_out, red_m)) return false;
    sg = make_segment<8>(V, 0, (V + 7) / 8);             // the epilogue below is the whole row's
    ef = load_exp_factors(tab_e, tid);
  }
  {
    // low half: count of +|v_j|, high half: count of -|v_j|.  Not kept beyond the sums: the one or
    // two lanes that need their counts again below read them from LDS again.
    uint32_t cw[WPL];
#pragma unroll
    for (int j = 0; j < WPL; j += 4) {
      const uint4 t = *(const uint4*)(hist + w0 + j);
      cw[j] = t.x; cw[j + 1] = t.y; cw[j + 2] = t.z; cw[j + 3] = t.w;
    }
#pragma unroll
    for (int j = 0; j < WPL; ++j) { lane_pos += (int)(cw[j] & 0xffffu); lane_neg += (int)(cw[j] >> 16); }
    // typical rows leave the lanes (and whole waves) of the small magnitudes empty: they skip the fp64 work
    if (lane_pos | lane_neg) {
#pragma unroll
    for (int j = WPL - 1; j >= 0; --j)                  // lowest of the negative values last
      if (cw[j] >> 16) vtop = hp_value_of_mag(WPL * tid + j, true);
#pragma unroll
    for (int j = 0; j < WPL; ++j)                       // highest of the positive values last
      if (cw[j] & 0xffffu) vtop = hp_value_of_mag(WPL * tid + j, false);
    const double vt = (double)vtop;
#pragma unroll
    for (int j = 0; j < WPL; ++j)                       // 64-register build: the halves are unpacked again below rather than
      if (WPS == 8) asm volatile("" : "+v"(cw[j]));     // kept from above in sixteen registers (which spilled the thread index)
    const bool b3 = ((WPL * tid) & 8) != 0;
    const double e0p = b3 ? ef.ap * ef.cp[3] : ef.ap, e0n = b3 ? ef.an * ef.cn[3] : ef.an;
#pragma unroll
    for (int j = 0; j < WPL; ++j) {
      const double vp = (double)hp_value_of_mag(WPL * tid + j, false);
      double ep = e0p, en = e0n;                                   // e^(+|v_j|), e^(-|v_j|)
      if (j & 4) { ep *= ef.cp[2]; en *= ef.cn[2]; }
      if (j & 2) { ep *= ef.cp[1]; en *= ef.cn[1]; }
      if (j & 1) { ep *= ef.cp[0]; en *= ef.cn[0]; }
      const double tp = (double)(cw[j] & 0xffffu) * ep;            // n * e^v (0 for an empty bin)
      const double tn = (double)(cw[j] >> 16) * en;
      if (TOPM) {                                                  // the positive values' share kept apart
        Zp += tp; Sp += (vp - vt) * tp;
        Z += tn; S += (-vp - vt) * tn;
      } else {
        Z += tp; S += (vp - vt) * tp;
        Z += tn; S += (-vp - vt) * tn;
      }
      __builtin_amdgcn_sched_barrier(0);                           // one bin pair at a time: keeps live registers low
    }
    }
  }
  // TOPM: the lane's sums over its positive and over its negative values, relative to its top value
  const double Zpos = Zp, Spos = Sp, Zneg = Z, Sneg = S;
  if (TOPM) { Z += Zp; S += Sp; }
  const float vw = wave_max(vtop);                      // -inf only if the whole wave owns empty bins
  if (lane_pos | lane_neg) S += ((double)vtop - (double)vw) * Z;
  Z = wave_sum(Z); S = wave_sum(S);
  const int incl_p = wave_scan_incl(lane_pos), incl_n = wave_scan_incl(lane_neg);
  if (lane == 0) { red_d[0][wid] = Z; red_d[1][wid] = S; red_v[wid] = vw; }
  if (lane == WAVE - 1) { scan_tmp[0][wid] = incl_p; scan_tmp[1][wid] = incl_n; }
  __syncthreads();
  C2T_PT(PT_SUMS);

  uint32_t m2 = HP_F16_NEG_INF2;
#pragma unroll
  for (int w = 0; w < NW; ++w) m2 = pk_max_f16(m2, red_m[w]);
  const uint32_t mag_hi = sh_out.mag_max;               // 0 unless a logit above the window (or a NaN) was met
  const float m = fmaxf(bf16_lo(m2), bf16_hi(m2));      // exact whenever the row stays on this path
  const int n_tiny = sh_out.n_tiny, n_ninf = sh_out.n_masked;
  int before_p = 0, before_n = 0, tot_p = 0, tot_n = 0; // counts in lower lanes / in the whole segment
#pragma unroll
  for (int w = 0; w < NW; ++w) {
    if (w < wid) { before_p += scan_tmp[0][w]; before_n += scan_tmp[1][w]; }
    tot_p += scan_tmp[0][w]; tot_n += scan_tmp[1][w];
  }
  if (wid == 0) {                                       // lanes 0..NW-1 hold one wave's sums each; fixed order
    double tz = 0.0, ts = 0.0;
    if (lane < NW && red_d[0][lane] > 0.0) {
      tz = red_d[0][lane];
      ts = red_d[1][lane] + ((double)red_v[lane] - (double)m) * tz;
    }
    tz += dpp_f64<C2T_DPP_QUAD_XOR1, 0xf>(tz); ts += dpp_f64<C2T_DPP_QUAD_XOR1, 0xf>(ts);
    tz += dpp_f64<C2T_DPP_QUAD_XOR2, 0xf>(tz); ts += dpp_f64<C2T_DPP_QUAD_XOR2, 0xf>(ts);
    tz += dpp_f64<C2T_DPP_ROW_HALF_MIRROR, 0xf>(tz); ts += dpp_f64<C2T_DPP_ROW_HALF_MIRROR, 0xf>(ts);
    tz += dpp_f64<C2T_DPP_ROW_MIRROR, 0xf>(tz); ts += dpp_f64<C2T_DPP_ROW_MIRROR, 0xf>(ts);
    if (lane == 0) {
      if (n_tiny) {                                     // e^x = 1 + x, x e^x = x for |x| < 2^-25
        const double zt = (double)n_tiny + sh_out.s_tiny;
        tz += zt; ts += sh_out.s_tiny - (double)m * zt;
      }
      sum_d[0] = tz; sum_d[1] = ts;
    }
  }
  // tau = exact K-th largest logit: first value (from the top) where the running count reaches K.
  // Descending value order: positive values from the highest lane down, then negative values from
  // lane 0 up.
  {
    const int above_p = tot_p - (before_p + incl_p);                   // positive elements in higher lanes
    if (above_p < K && above_p + lane_pos >= K) {                      // at most one lane
      int run = above_p;
#pragma unroll
      for (int j = WPL - 1; j >= 0; --j) {
        const int n = (int)(hist[w0 + j] & 0xffffu);
        if (run < K && run + n >= K) { sh_tau_rank = HP_WORDS + WPL * tid + j; sh_n_gt = run; }
        run += n;
      }
    }
    const int above_n = tot_p + before_n + incl_n - lane_neg;          // everything positive, and negatives in lower lanes
    if (above_n < K && above_n + lane_neg >= K) {
      int run = above_n;
#pragma unroll
      for (int j = 0; j < WPL; ++j) {
        const int n = (int)(hist[w0 + j] >> 16);
        if (run < K && run + n >= K) { sh_tau_rank = HP_WORDS - 1 - (WPL * tid + j); sh_n_gt = run; }
        run += n;
      }
    }
  }
  __syncthreads();
  C2T_PT(PT_TAU);
  // Leave this path (uniformly) if a logit that is not masked lies above the window (|x| >= 2^7, +inf, NaN), if a
  // 16-bit counter overflowed (the total is then off by a multiple of 65535 or 65536), if logits
  // below the window exist and the K-th largest logit is not a positive window value (then they
  // could be among the top K, which the histogram cannot rank), or if fewer than K logits lie
  // in the window while some are masked (the top K then ends with masked entries).
  const int n_elems = (sg.tail_chunk >= 0 ? (sg.ncell - 1) * 8 + sg.tail_valid : sg.ncell * 8);
  // With the entropy over the M largest logits: also if some but not all of the logits below the
  // window are among them (which ones cannot be told from the histogram).
  if (mag_hi >= HP_MAG_LO + HP_MAG_SPAN || tot_p + tot_n + n_tiny + n_ninf != n_elems || (n_tiny > 0 && sh_tau_rank < HP_WORDS) ||
      (n_ninf > 0 && sh_tau_rank < 0) ||
      (TOPM && n_tiny > 0 && tot_p < M && M < tot_p + n_tiny)) {
    __syncthreads();
    generic_segment<1, NT, HP_CPC>(rowp, V, K, M, sg, map_lds, sel, rr, 2u);
    return true;
  }
  if (TOPM) {
    // Eq. 2, second line: Z and S restricted to the M largest logits.  A lane's values, from the
    // top: its positive magnitudes descending, then its negative ones ascending; `above` of them
    // lie in other lanes.  Same reference chain as for S (lane top, wave top, m): one sign throughout.
    double zm = 0.0, sm = 0.0;
    // (logits below the window, |x| < 2^-25, rank between the positive and the negative window values)
    const int above_p = tot_p - (before_p + incl_p), above_n = tot_p + n_tiny + before_n + incl_n - lane_neg;
    const double vt = (double)vtop;
    // A lane whose positive (negative) values all rank within the first M contributes the sums it
    // already has; only the lane that holds the M-th largest logit walks its bins.
    const bool part_p = lane_pos > 0 && above_p < M && above_p + lane_pos > M;
    const bool part_n = lane_neg > 0 && above_n < M && above_n + lane_neg > M;
    if (lane_pos > 0 && above_p + lane_pos <= M) { zm += Zpos; sm += Spos; }
    if (lane_neg > 0 && above_n + lane_neg <= M) { zm += Zneg; sm += Sneg; }
    if (part_p || part_n) {
      LaneCounts<WPL> counts;
#pragma unroll
      for (int j = 0; j < WPL; ++j) counts.w[j] = hist[w0 + j];
      const TopMPart part = top_m_boundary_lane<WPL>(tid, counts, part_p, part_p ? above_p : above_n, M, vt);
      zm += part.zm; sm += part.sm;
    }
    if (lane_pos | lane_neg) sm += (vt - (double)vw) * zm;
    zm = wave_sum(zm); sm = wave_sum(sm);
    if (lane == 0) { red_d[0][wid] = zm; red_d[1][wid] = sm; }     // red_v still holds the waves' top values
    __syncthreads();
    if (wid == 0) {
      double tz = 0.0, ts = 0.0;
      if (lane < NW && red_d[0][lane] > 0.0) { tz = red_d[0][lane]; ts = red_d[1][lane] + ((double)red_v[lane] - (double)m) * tz; }
      tz += dpp_f64<C2T_DPP_QUAD_XOR1, 0xf>(tz); ts += dpp_f64<C2T_DPP_QUAD_XOR1, 0xf>(ts);
      tz += dpp_f64<C2T_DPP_QUAD_XOR2, 0xf>(tz); ts += dpp_f64<C2T_DPP_QUAD_XOR2, 0xf>(ts);
      tz += dpp_f64<C2T_DPP_ROW_HALF_MIRROR, 0xf>(tz); ts += dpp_f64<C2T_DPP_ROW_HALF_MIRROR, 0xf>(ts);
      tz += dpp_f64<C2T_DPP_ROW_MIRROR, 0xf>(tz); ts += dpp_f64<C2T_DPP_ROW_MIRROR, 0xf>(ts);
      if (lane == 0) {
        if (n_tiny > 0 && tot_p < M) {                    // then M >= tot_p + n_tiny: all of them are among the M largest
          const double zt = (double)n_tiny + sh_out.s_tiny;
          tz += zt; ts += sh_out.s_tiny - (double)m * zt;
        }
        sum_m[0] = tz; sum_m[1] = ts;
      }
    }
  }
  float tau = -INFINITY;
  int eq_limit = K;
  if (sh_tau_rank >= 0) { tau = __uint_as_float(hp_code_of_rank(sh_tau_rank) << 16); eq_limit = K - sh_n_gt; }

  // ---------------- cells that can hold a top-K element ----------------
  // Fewer than K cells exceed tau; cells equal to tau are all taken when they fit (the exact
  // ranking below keeps the lowest ids).
  const int ncells = cells_in_segment<NT, HP_CPC>(sg.ncell);
#pragma unroll 1
  for (int c8 = tid * 8; c8 < ncells; c8 += NT * 8) {    // eight keys per read (the map is padded to 16 bytes)
    const uint4 kq = *(const uint4*)(map + c8);
    const uint32_t kw[4] = {kq.x, kq.y, kq.z, kq.w};
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const float kv = (j & 1) ? bf16_hi(kw[j >> 1]) : bf16_lo(kw[j >> 1]);
      if (c8 + j < ncells && kv >= tau) {
        const int slot = atomicAdd(&sh_ncell, 1);
        if (slot < sel.cell_cap) cell_list[slot] = c8 + j;
      }
    }
  }
  if (tid == 0) sh_cnt = 0;
  __syncthreads();
  C2T_PT(PT_CELLS_LISTED);
  int n_cells = sh_ncell;
  const bool ties = n_cells > sel.cell_cap;                  // massive ties at tau: the cells above it, then a tie scan
  if (ties) {
    n_cells = list_cells<1, NT>(map, ncells, tau, true, sel.cell_cap, cell_list, &sh_ncell);
    if (tid == 0) sh_cnt = 0;
    __syncthreads();
  }
  collect_cells<1, NT, HP_CPC>(rowp, sg.c0, sg.c1, V, tau, ties, cell_list, n_cells, sel, &sh_cnt);
  if (ties) tie_scan<1, NT>(rowp, sg, V, tau, eq_limit, sel, &sh_cnt, scan_tmp);
  C2T_PT(PT_CELLS_READ);
  const int n_top = rank_list<NT>(K, sel, &sh_cnt, rr->topv, rr->topi);
  C2T_PT(PT_RANKED);
  if (tid == 0) {
    RowPartial r;
    r.ref = (double)m; r.a = 0.0; r.Z = sum_d[0]; r.S = sum_d[1]; r.n_top = n_top; r.flags = 0u;
    rr->part = r;
    if (TOPM) { rr->ZM = sum_m[0]; rr->SM = sum_m[1]; }
  }
  return true;
}

// grid: rows_launched * nsplit workgroups of NT threads.
// Dynamic LDS (sp.lds_bytes): [HP_WORDS counters | cell map, padded to 16 bytes]; the selection's
// element list and the tail reuse all of it.
// WPS: waves per SIMD the kernel is built for.  8 = four workgroups per CU on 64 registers a lane;
// 6 = three workgroups per CU on 80 registers, which needs no spills.
template <int NT, bool TOPM, int WPS, int REPL, bool COOP>
__global__ __launch_bounds__(NT, WPS) void k_logits_hist(
    const void* __restrict__ logits, int64_t row_stride_elems, int V, int cps, const double* __restrict__ tab_e,
    const float* __restrict__ cls, TreeState st, ScoreParams sp) {
  extern __shared__ __align__(16) unsigned char dyn_lds[];
  const int nsplit = (COOP && sp.coop > 1) ? sp.coop : sp.nsplit, K = sp.K;     // workgroups per row, either way
  const int split = blockIdx.x % nsplit;
  const RowOfWorkgroup rw = row_of_workgroup(st, sp, blockIdx.x / nsplit);
  const int b = rw.b, f = rw.f, rl = b * sp.rows_per_seq + f, nf = rw.nf;
  if (f >= nf) { if (nf == 0) end_of_sequence(st, sp, b, f, split); return; }   // uniform for the workgroup
  const int64_t row = (int64_t)b * sp.F + f;
  const uint4* rowp = (const uint4*)((const char*)logits + row * row_stride_elems * 2);
  const Segment sg = make_segment<8>(V, split, cps);
  __shared__ RowResult rr;
  C2T_PT(PT_START);
  if (threadIdx.x == 0) rr.parent_P = st.fr_P[row];        // off the tail's critical path
  // The classifier's parameters (5h+1 <= 1281 floats) are copied to LDS for the scoring step: the
  // loads are issued now, four floats a thread, and stored behind the streaming loop.
  const ClassifierStage cst = stage_classifier(cls, sp.h, (!TOPM && sp.w_lds_off >= 0) ? (float*)(dyn_lds + sp.w_lds_off) : nullptr);
  if (sg.ncell == 0) {                                     // (loaded again here: the copy above must not stay in registers for this)
    store_classifier(stage_classifier(cls, sp.h, cst.dst));
    if (threadIdx.x == 0) { rr.part = empty_partial(); rr.ZM = 0.0; rr.SM = 0.0; }
  }
  else if (!hist_segment<NT, TOPM, WPS, REPL, COOP>(rowp, V, K, TOPM ? sp.M : 0, sg, tab_e, (uint32_t*)dyn_lds, dyn_lds + HP_WORDS * 4 * REPL,
                        make_select_lds<NT, HP_CPC, 8>(dyn_lds, sp.lds_bytes), &rr, cst, sp, split, rl,
                        st.row_tickets + (int64_t)b * sp.F + f))
    return;                                                // a shared row's segment, handed over
  finish_layer<NT>(st, sp, b, f, nf, split, rl, rr, dyn_lds, cls, cst.dst,
                   [&](RowResult& r) { if (TOPM) top_m_of_split_row<1, NT>(rowp, V, sp.M, r); });
}

// Plain streaming read: the practical HBM ceiling.
__global__ __launch_bounds__(1024) void k_stream_read(const uint4* __restrict__ p, size_t n16, uint32_t* out) {
  uint32_t acc = 0;
  size_t i = (size_t)blockIdx.x * 1024 + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * 1024;
  for (; i + 3 * stride < n16; i += 4 * stride) {
    const uint4 a = p[i], b = p[i + stride], c = p[i + 2 * stride], d = p[i + 3 * stride];
    acc += a.x ^ a.y ^ a.z ^ a.w; acc += b.x ^ b.y ^ b.z ^ b.w;
    acc += c.x ^ c.y ^ c.z ^ c.w; acc += d.x ^ d.y ^ d.z ^ d.w;
  }
  for (; i < n16; i += stride) { const uint4 a = p[i]; acc += a.x ^ a.y ^ a.z ^ a.w; }
  acc = (uint32_t)wave_sum_i((int)acc);
  if ((threadIdx.x & 63) == 0 && acc == 0x9e3779b9u) atomicAdd(out, acc);   // keeps the loads alive
}

// The same read with the layer kernel's access pattern and nothing else: one workgroup of 512
// threads per row, lane t reads chunks t, t+512, ... of its row, four in flight, non-temporal.  What
// the memory system delivers to that pattern is the ceiling the logits pass can be held against.
__global__ __launch_bounds__(512, 8) void k_stream_read_rows(const char* __restrict__ p, int64_t row_stride_bytes, int chunks_per_row, uint32_t* out) {
  const uint4* row = (const uint4*)(p + (int64_t)blockIdx.x * row_stride_bytes);
  uint32_t acc = 0;
  int g = threadIdx.x;
  for (; g + 3 * 512 < chunks_per_row; g += 4 * 512) {
    const uint4 a = load_stream(row + g), b = load_stream(row + g + 512), c = load_stream(row + g + 1024), d = load_stream(row + g + 1536);
    acc += a.x ^ a.y ^ a.z ^ a.w; acc += b.x ^ b.y ^ b.z ^ b.w;
    acc += c.x ^ c.y ^ c.z ^ c.w; acc += d.x ^ d.y ^ d.z ^ d.w;
  }
  for (; g < chunks_per_row; g += 512) { const uint4 a = load_stream(row + g); acc += a.x ^ a.y ^ a.z ^ a.w; }
  acc = (uint32_t)wave_sum_i((int)acc);
  if ((threadIdx.x & 63) == 0 && acc == 0x9e3779b9u) atomicAdd(out, acc);   // keeps the loads alive
}

}  // namespace c2t
