// Everything after a row's sums and top-K: the tail that the logits kernels run in place
// (merge of split rows, features + classifier (Eq. 1-3) per row, the two prunings of Sec. 4.2 with
// the node budget and the tree append per sequence, handed from workgroup to workgroup by tickets),
// and the small kernels: reset, emission of the tree mask, position ids and parent links, and the
// EAGLE-2-style reranked emission (Sec. 2.2).
#pragma once
#include "k_common.h"

namespace c2t {

struct TreeState {            // device pointers into the workspace
  float* cls;                 // W1[3h] b1[h] w2[h] b2
  int32_t* n_nodes;           // [B]
  int32_t* nf[2];             // [B] frontier sizes, ping-pong: layer l reads nf[l&1], writes nf[(l+1)&1]
  int32_t* tickets;           // [B] rows of the current layer that have been scored
  int32_t* row_tickets;       // [B][F] splits of the row that have delivered their record
  uint32_t* row_info;         // [B][F] bit 0: row unusable (NaN, +inf, no finite logit); bit 1: two-pass path taken
  uint32_t* status;           // [B]
  int32_t* n_cand;            // [B]
  int32_t* layer_rows;        // [D+1]
  int32_t* fr_tok;            // [B][F]
  int32_t* fr_pslot;          // [B][F]
  int32_t* fr_node;           // [B][F]
  float* fr_P;                // [B][F]
  int32_t* fr_hidx;           // [B][F] history index of the frontier node, -1 = root (rerank contexts only)
  float* fr_s;                // [B][F] smallest classifier logit on its path, +inf for the root
  // history of every scored candidate, [B][D][F*K] (rerank contexts only, else null)
  int32_t* h_tok; int32_t* h_par; float* h_P; float* h_H; float* h_z; float* h_s;
  int32_t* h_ncand;           // [B][D] candidates scored in each layer
  int32_t* h_pos;             // [B][D*F*K] scratch of the reranking
  int32_t* t_tok;             // [B][N]
  int32_t* t_parent;
  int32_t* t_depth;
  float* t_P;
  float* t_H;
  float* t_z;
  int32_t* c_tok;             // [B][F*K]
  float* c_p;
  float* c_P;
  float* c_H;
  float* c_z;
  int32_t* c_kept;
};

__global__ void k_reset(TreeState s, int B, int F, int D) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (s.h_tok) {
    if (i < B) { s.fr_hidx[(int64_t)i * F] = -1; s.fr_s[(int64_t)i * F] = INFINITY; }
    for (int j = i; j < B * D; j += gridDim.x * blockDim.x) s.h_ncand[j] = 0;
  }
  if (i < B) {
    s.n_nodes[i] = 0; s.nf[0][i] = 1; s.nf[1][i] = 0; s.tickets[i] = 0; s.status[i] = 0; s.n_cand[i] = 0;
    s.fr_tok[(int64_t)i * F] = -1; s.fr_pslot[(int64_t)i * F] = 0;
    s.fr_node[(int64_t)i * F] = -1; s.fr_P[(int64_t)i * F] = 1.0f;
  }
  if (i <= D) s.layer_rows[i] = (i == 0) ? B : 0;
  for (int j = i; j < B * F; j += gridDim.x * blockDim.x) s.row_tickets[j] = 0;
}

// A slice of the classifier's parameters on its way to the workspace as a kernel argument.
struct ClsChunk { static constexpr int N = 240; float v[N]; };
__global__ void k_set_classifier(float* __restrict__ cls, int off, int n, ClsChunk c) {
  if ((int)threadIdx.x < n) cls[off + threadIdx.x] = c.v[threadIdx.x];
}

// Eq. 3 in fp32: fixed chain of fused multiply-adds, hidden units in ascending order.
// `w` in global memory: every lane reads the same addresses, so the loads are scalar; but each
// group of hidden units then waits for its own loads (measured: 1.2-1.4 us for 32 hidden units).
__device__ __forceinline__ float mlp_logit(const float* __restrict__ w, int h, float P, float H, float d) {
  const float* W1 = w; const float* b1 = w + 3 * h; const float* w2 = w + 4 * h;
  float z = w[5 * h];
#pragma unroll 4
  for (int j = 0; j < h; ++j) {
    float a = __fmaf_rn(W1[3 * j + 0], P, b1[j]);
    a = __fmaf_rn(W1[3 * j + 1], H, a);
    a = __fmaf_rn(W1[3 * j + 2], d, a);
    a = a > 0.0f ? a : 0.0f;
    z = __fmaf_rn(w2[j], a, z);
  }
  return z;
}
// The same chain with the parameters staged in LDS (broadcast reads, many in flight).
typedef __attribute__((address_space(3))) const float* LdsFloats;
__device__ __forceinline__ float mlp_logit_lds(LdsFloats w, int h, float P, float H, float d) {
  LdsFloats W1 = w; LdsFloats b1 = w + 3 * h; LdsFloats w2 = w + 4 * h;
  float z = w[5 * h];
  if ((h & 3) == 0) {                                        // every array starts on 16 bytes: five wide reads per four units
    typedef float float4v __attribute__((ext_vector_type(4)));
    typedef __attribute__((address_space(3))) const float4v* LdsFloat4s;
#pragma unroll 2
    for (int j = 0; j < h; j += 4) {
      const float4v wa = *(LdsFloat4s)(W1 + 3 * j), wb = *(LdsFloat4s)(W1 + 3 * j + 4), wc = *(LdsFloat4s)(W1 + 3 * j + 8);
      const float4v bb = *(LdsFloat4s)(b1 + j), vv = *(LdsFloat4s)(w2 + j);
      float a0 = __fmaf_rn(wa.x, P, bb.x); a0 = __fmaf_rn(wa.y, H, a0); a0 = __fmaf_rn(wa.z, d, a0); a0 = a0 > 0.0f ? a0 : 0.0f;
      float a1 = __fmaf_rn(wa.w, P, bb.y); a1 = __fmaf_rn(wb.x, H, a1); a1 = __fmaf_rn(wb.y, d, a1); a1 = a1 > 0.0f ? a1 : 0.0f;
      float a2 = __fmaf_rn(wb.z, P, bb.z); a2 = __fmaf_rn(wb.w, H, a2); a2 = __fmaf_rn(wc.x, d, a2); a2 = a2 > 0.0f ? a2 : 0.0f;
      float a3 = __fmaf_rn(wc.y, P, bb.w); a3 = __fmaf_rn(wc.z, H, a3); a3 = __fmaf_rn(wc.w, d, a3); a3 = a3 > 0.0f ? a3 : 0.0f;
      z = __fmaf_rn(vv.x, a0, z); z = __fmaf_rn(vv.y, a1, z); z = __fmaf_rn(vv.z, a2, z); z = __fmaf_rn(vv.w, a3, z);
    }
    return z;
  }
#pragma unroll 4
  for (int j = 0; j < h; ++j) {
    float a = __fmaf_rn(W1[3 * j + 0], P, b1[j]);
    a = __fmaf_rn(W1[3 * j + 1], H, a);
    a = __fmaf_rn(W1[3 * j + 2], d, a);
    a = a > 0.0f ? a : 0.0f;
    z = __fmaf_rn(w2[j], a, z);
  }
  return z;
}

constexpr int SP_MAX_F = 64;
constexpr int C2T_MAX_BUDGET_DEV = 1024;                  // n_out limit of the reranking
constexpr int C2T_MAX_CANDIDATES_DEV = 2048;              // F*K limit of the per-sequence step

// What a workgroup that shares a row hands over besides its counts and cell keys.
struct __attribute__((aligned(32))) CoopAcc {
  double s_tiny; int32_t n_tiny, n_masked; uint32_t mag_max, max_pattern;   // see OutsideAcc; max_pattern: packed maximum of the segment's bf16 patterns
};

struct ScoreParams {
  RowPartial* part; float* part_topv; int32_t* part_topi;    // [launched row][split] records and their top-K lists
  int nsplit, rows_per_seq, B, F, K, N, h, layer, D;
  int M;                                                     // 0: entropy over the whole row; M > 0: over the M largest logits
  int lds_bytes;                                             // dynamic LDS of the launch
  int w_lds_off;                                             // byte offset of the classifier's copy in dynamic LDS, -1: none
  int compact;                                               // 1: workgroup w takes the w-th live row (see row_of_workgroup)
  float z_beta;
  // Shared rows of the histogram path (coop > 1, then nsplit == 1): `coop` workgroups count one row's
  // segments and hand their counts over through memory; the last to arrive runs the row's epilogue.
  int coop;
  int coop_map_stride;                                       // keys per row in coop_map (a multiple of 8)
  uint32_t* coop_hist;                                       // [launched row][coop][HP_WORDS] counts of a segment
  uint16_t* coop_map;                                        // [launched row][coop_map_stride] cell keys of the whole row
  CoopAcc* coop_acc;                                         // [launched row][coop]
};

// What one workgroup of the logits pass leaves in LDS for its (row, split): the record and the
// segment's top-K list (value desc, id asc).
struct RowResult {
  RowPartial part;
  double ZM, SM;      // the sums of Z and S restricted to the M largest logits (Eq. 2, second line); M > 0 only
  float parent_P;     // joint probability of the row's frontier node, fetched when the workgroup starts
  float topv[64];
  int32_t topi[64];
};

// ---- row level, splits > 1: combine the row's split records (fp64) and top lists into `rr`.
// Run by the workgroup that delivered the row's last split; `lds`/`lds_bytes` is free scratch.
__device__ __forceinline__ void merge_row(const ScoreParams& sp, int64_t row_launched, RowResult& rr,
                                          unsigned char* lds, size_t lds_bytes) {
  const int tid = threadIdx.x, nt = blockDim.x, nsplit = sp.nsplit, K = sp.K;
  const RowPartial* rp = sp.part + row_launched * nsplit;
  const float* tv = sp.part_topv + row_launched * nsplit * K;
  const int32_t* ti = sp.part_topi + row_launched * nsplit * K;
  const int per_row = nsplit * K;
  const bool staged = (size_t)per_row * 8 <= lds_bytes;      // the lists fit the staging area in LDS
  // Everything the merge reads is requested before anything is waited for: one memory round trip instead of
  // four dependent ones (maximum, records, list lengths, entries).  A thread's first list entry (all of them
  // when the row's lists hold at most one entry a thread): requested whether valid or not, masked below.
  const bool in0 = staged && tid < per_row;
  int n_top0 = 0, i0 = -1; float v0 = 0.f;
  if (in0) { n_top0 = ld_dev(&rp[tid / K].n_top); v0 = ld_dev(tv + tid); i0 = ld_dev(ti + tid); }
  if (tid < WAVE) {                                          // wave 0: the sums, one split per lane and step
    const int lane = tid;
    float Rf = -INFINITY; uint32_t fl = 0;                   // ref holds a logit: exact as a float
    double Z = 0.0, S = 0.0;
    if (nsplit <= WAVE) {
      RowPartial pq = empty_partial();
      if (lane < nsplit) pq = ld_dev(rp + lane);
      Rf = wave_max(lane < nsplit ? (float)pq.ref : -INFINITY);
      fl = wave_reduce_u32(pq.flags, 0u, [](uint32_t x, uint32_t y) { return x | y; });
      const double R = (double)Rf;
      if (pq.Z > 0.0 && pq.ref > -INFINITY) {
        const double da = pq.a - R, dl = pq.ref - R;         // re-reference to the row maximum R; dl <= 0
        const double sc = da == 0.0 ? 1.0 : exp(da);
        Z = pq.Z * sc; S = (pq.S + dl * pq.Z) * sc;
      }
    } else {
      for (int q = lane; q < nsplit; q += WAVE) { Rf = fmaxf(Rf, (float)ld_dev(&rp[q].ref)); fl |= ld_dev(&rp[q].flags); }
      Rf = wave_max(Rf);
      fl = wave_reduce_u32(fl, 0u, [](uint32_t x, uint32_t y) { return x | y; });
      const double R = (double)Rf;
      for (int q = lane; q < nsplit; q += WAVE) {
        const RowPartial pq = ld_dev(rp + q);
        if (pq.Z > 0.0 && pq.ref > -INFINITY) {
          const double da = pq.a - R, dl = pq.ref - R;
          const double sc = da == 0.0 ? 1.0 : exp(da);
          Z += pq.Z * sc; S += (pq.S + dl * pq.Z) * sc;
        }
      }
    }
    const double R = (double)Rf;
    Z = wave_sum(Z); S = wave_sum(S);
    if (lane == 0) { rr.part.ref = R; rr.part.a = R; rr.part.Z = Z; rr.part.S = S; rr.part.flags = fl; rr.part.n_top = 0; }
  }
  // An entry's merged rank = number of entries of the row's lists ahead of it.
  float* sv = (float*)lds; int32_t* si = (int32_t*)(lds + (size_t)per_row * 4);
  __shared__ int32_t n_valid;
  if (tid == 0) n_valid = 0;
  __syncthreads();
  if (staged) {
    // an unused slot of a list: below every entry in the order (value desc, id asc), -inf entries included
    constexpr int32_t NO_ID = 0x7fffffff;
    if (in0) {
      const bool ok = tid % K < n_top0;
      sv[tid] = ok ? v0 : -INFINITY;
      si[tid] = ok ? i0 : NO_ID;
      if (ok) atomicAdd(&n_valid, 1);
    }
    for (int ent = tid + nt; ent < per_row; ent += nt) {
      const int q = ent / K, e = ent % K;
      const bool ok = e < ld_dev(&rp[q].n_top);
      sv[ent] = ok ? ld_dev(tv + ent) : -INFINITY;
      si[ent] = ok ? ld_dev(ti + ent) : NO_ID;
      if (ok) atomicAdd(&n_valid, 1);
    }
    __syncthreads();
    for (int ent = tid; ent < per_row; ent += nt) {
      const int vi = si[ent];
      if (vi == NO_ID) continue;
      const float v = sv[ent];
      const int ahead = count_ahead4(sv, per_row, 0, 4, v, ent, [&](int o) { return si[o] < vi; });
      if (ahead < K) { rr.topv[ahead] = v; rr.topi[ahead] = vi; }
    }
  } else {
    // the lists exceed the staging area (very many splits): rank from global memory
    for (int ent = tid; ent < per_row; ent += nt) {
      const int q = ent / K, e = ent % K;
      if (e >= ld_dev(&rp[q].n_top)) continue;
      atomicAdd(&n_valid, 1);
      const float v = ld_dev(tv + ent); const int vi = ld_dev(ti + ent);
      int ahead = 0;
      for (int q2 = 0; q2 < nsplit; ++q2) {
        const int n2 = ld_dev(&rp[q2].n_top);
        for (int e2 = 0; e2 < n2; ++e2) {
          const float v2 = ld_dev(tv + q2 * K + e2);
          ahead += (v2 > v) || (v2 == v && ld_dev(ti + q2 * K + e2) < vi);
        }
      }
      if (ahead < K) { rr.topv[ahead] = v; rr.topi[ahead] = vi; }
    }
  }
  __syncthreads();
  if (tid == 0) rr.part.n_top = min(n_valid, K);
  __syncthreads();
}

// ---- row level: entropy (Eq. 2), generation and joint probabilities (Eq. 1), classifier logit
// (Eq. 3) of the row's K candidates, from the complete row result in `rr`.  One lane per candidate.
// `w`: the classifier parameters in global memory, read-only for the whole kernel: every lane
// reads the same addresses, so the loads are scalar and touch neither LDS nor the vector memory path.
__device__ __forceinline__ void score_row(const TreeState& s, const ScoreParams& sp, int b, int f, const RowResult& rr,
                                          const float* __restrict__ w, const float* w_lds) {
  const int tid = threadIdx.x, K = sp.K;
  if (tid >= K) return;
  const float parP = rr.parent_P;
  const double R = rr.part.ref, Z = rr.part.Z;
  const uint32_t fl = rr.part.flags;
  const bool bad = (fl & 1u) != 0 || !(Z > 0.0) || !(R > -INFINITY) || !(R < INFINITY);
  // re-reference the sums from the offset a to the row maximum R (= ref): p_j = e^(x_j - R) / Zr,
  // H = -sum p ln p = ln Zr - Sr / Zr
  const double sc = rr.part.a == R ? 1.0 : exp(rr.part.a - R);
  const double Zr = Z * sc, Sr = rr.part.S * sc;
  // Eq. 2, second line: -sum over the M most probable tokens of p ln p, p from the full softmax:
  // (ln Zr * ZMr - SMr) / Zr with the sums restricted to those tokens
  const float H = bad ? 0.f : sp.M > 0 ? (float)((log(Zr) * (rr.ZM * sc) - rr.SM * sc) / Zr) : (float)(log(Zr) - Sr / Zr);
  float z = -INFINITY, p32 = 0.f, P32 = 0.f; int tok = -1;
  if (!bad && tid < rr.part.n_top) {
    tok = rr.topi[tid];
    p32 = (float)(exp((double)rr.topv[tid] - R) / Zr);
    P32 = parP * p32;
    z = w_lds ? mlp_logit_lds((LdsFloats)w_lds, sp.h, P32, H, (float)sp.layer) : mlp_logit(w, sp.h, P32, H, (float)sp.layer);
  }
  const int64_t o = (int64_t)b * sp.F * K + (int64_t)f * K + tid;
  st_dev(s.c_tok + o, tok); st_dev(s.c_p + o, p32); st_dev(s.c_P + o, P32); st_dev(s.c_H + o, H); st_dev(s.c_z + o, z);
  if (tid == 0) st_dev(s.row_info + (int64_t)b * sp.F + f, (uint32_t)(bad ? 1u : 0u) | (fl & 2u));
  if (s.h_tok) {                                             // keep the candidate for the reranking
    const int FK = sp.F * K;
    const int64_t hi = ((int64_t)b * sp.D + sp.layer) * FK + (int64_t)f * K + tid;
    s.h_tok[hi] = tok; s.h_par[hi] = s.fr_hidx[(int64_t)b * sp.F + f];
    s.h_P[hi] = P32; s.h_H[hi] = H; s.h_z[hi] = z;
    s.h_s[hi] = fminf(s.fr_s[(int64_t)b * sp.F + f], z);
  }
}

// ---- sequence level: both prunings of Sec. 4.2 with the node budget, tree append, next frontier.
// Run by one whole workgroup once every row of the sequence has been scored.
//
// Survivors of the first pruning are compacted into LDS lists (a 64-bit key of z and token, and the
// candidate index).  Only the n_keep best of them matter: when the list is long, a 4096-bin histogram
// over the top 12 bits of the order-preserving key of z finds the bin that holds the n_keep-th largest z,
// and the list is cut down to the survivors from that bin upwards before the exact ranking.  The ranking
// gives each survivor to T = 2^tshift lanes, which split the list between them, two keys per LDS read.
#ifndef C2T_PRUNE_PRESELECT_MIN
#define C2T_PRUNE_PRESELECT_MIN 64
#endif
#ifndef C2T_PRUNE_UNDECIDED_MAX
#define C2T_PRUNE_UNDECIDED_MAX 64
#endif
constexpr int PRUNE_HIST_WORDS = 2048;        // 4096 bins, two 16-bit counters per word
constexpr int PRUNE_PRESELECT_MIN = C2T_PRUNE_PRESELECT_MIN;   // shorter lists are ranked directly
constexpr int PRUNE_UNDECIDED_MAX = C2T_PRUNE_UNDECIDED_MAX; // the select stops once at most so many survivors share the selected digits

__host__ __device__ inline size_t score_lds_bytes(int h, int FK) {
  (void)h;
  return ((size_t)3 * ((FK + 31) & ~31) + PRUNE_HIST_WORDS) * 4;
}

template <int NT>
__device__ __forceinline__ void prune_sequence(const TreeState& s, const ScoreParams& sp, int b, int nf, unsigned char* lds) {
  constexpr int NW = NT / WAVE;
  const int F = sp.F, K = sp.K, N = sp.N, layer = sp.layer;
  const float z_beta = sp.z_beta;
  const int FK = F * K, FKp = (FK + 31) & ~31;
  // survivors: one 64-bit key each, (order-preserving key of z) << 32 | ~token, so that a greater key comes first in
  // the order (z desc, token asc); and the candidate index, which breaks the remaining ties.  Equal z is common, not
  // rare: deep in a tree P is too small to move the classifier's fp32 sum, and the K children of a row, which
  // share H and d, all get the same z.
  uint64_t* skey = (uint64_t*)lds;
  int32_t* sidx = (int32_t*)(skey + FKp);
  uint32_t* hist = (uint32_t*)(sidx + FKp);
  __shared__ int32_t n_surv, n_red, flags_or, sel_bin, sel_above, sel_count;
  __shared__ int32_t scan_w[NW];
  __shared__ int32_t new_tok[SP_MAX_F], new_pslot[SP_MAX_F], new_node[SP_MAX_F];
  __shared__ float new_P[SP_MAX_F], new_s[SP_MAX_F];
  __shared__ int32_t new_hidx[SP_MAX_F];

  const int tid = threadIdx.x, lane = tid & (WAVE - 1), wid = tid >> 6;
  // the candidates' z and tokens are requested up front for all F*K slots: one memory round trip
  constexpr int PER = C2T_MAX_CANDIDATES_DEV / NT;           // candidates per thread
  const int per = (FK + NT - 1) / NT;
  float my_z[PER]; int32_t my_tok[PER];
#pragma unroll
  for (int k = 0; k < PER; ++k) {
    const int i = tid + k * NT;
    if (k < per && i < FK) {
      const int64_t o = (int64_t)b * FK + i;
      my_z[k] = ld_dev(s.c_z + o); my_tok[k] = ld_dev(s.c_tok + o);
    }
  }
  const uint32_t info = tid < F ? ld_dev(s.row_info + (int64_t)b * F + tid) : 0u;
  const int nn = s.n_nodes[b];
  // the kept flags start at zero (all F*K slots: slots of unused rows are unspecified anyway); stored
  // now, so that they are long complete when the ranking stores the ones
  for (int i = tid; i < FK; i += NT) s.c_kept[(int64_t)b * FK + i] = 0;
  if (tid == 0) { n_surv = 0; n_red = 0; flags_or = 0; sel_bin = 0; }
  for (int i = tid; i < PRUNE_HIST_WORDS; i += NT) hist[i] = 0u;
  __syncthreads();
  if (tid < nf && info) atomicOr(&flags_or, (int)info);
  C2T_PT(PT_PRUNE_LOADED);                                   // (thread 0's own loads have arrived: info is used above)

  // ---- first pruning: z > logit(beta) ----
  const int ncand = nf * K;
#pragma unroll
  for (int k = 0; k < PER; ++k) {
    const int i = tid + k * NT;
    if (k < per && i < ncand) {
      if (my_tok[k] >= 0 && my_z[k] > z_beta) {
        const int u = atomicAdd(&n_surv, 1);
        const uint32_t zk = sortable_key(my_z[k]);
        skey[u] = ((uint64_t)zk << 32) | (uint32_t)~my_tok[k]; sidx[u] = i;
        const uint32_t bin = zk >> 20;
        atomicAdd(&hist[bin >> 1], (bin & 1u) ? 0x10000u : 1u);
      }
    }
  }
  wait_vector_memory();                                      // the zeros are written before any thread stores a one
  __syncthreads();
  C2T_PT(PT_PRUNE_FIRST);

  // ---- second pruning + budget: rank survivors by (z desc, token asc, slot asc) ----
  int ns = n_surv;
  const int n_keep = max(0, min(min(F, N - nn), ns));
  if (n_keep > 0 && ns > PRUNE_PRESELECT_MIN) {
    // Radix select on the 64-bit keys, twelve bits a level, from the top: the histogram of the level's digit over
    // the survivors that are still undecided (those whose higher digits equal the digits selected so far; at the
    // first level all of them, counted during the first pruning) gives the digit at which the running count from
    // the top reaches what is still needed; survivors below it are dropped.  Typical layers are done after one
    // level (a dozen survivors left); layers of equal z go on into the token bits instead of ranking hundreds of
    // tied survivors against each other.
    int need = n_keep, shift = 52;                           // (uniform) still to be taken from the undecided; the level's digit is key >> shift
    uint64_t prefix = 0ull;                                  // the digits selected so far: the undecided have key >> (shift + 12) == prefix
    for (;;) {
      // thread t owns words 2047-4t .. 2047-4t-3 (bins descending)
      constexpr int WPT = PRUNE_HIST_WORDS / NT;
      uint32_t w[WPT]; int c = 0;
#pragma unroll
      for (int j = 0; j < WPT; ++j) { w[j] = hist[PRUNE_HIST_WORDS - 1 - (tid * WPT + j)]; c += (int)(w[j] & 0xffffu) + (int)(w[j] >> 16); }
      const int incl = wave_scan_incl(c);
      if (lane == WAVE - 1) scan_w[wid] = incl;
      __syncthreads();
      int above = incl - c;
#pragma unroll
      for (int v = 0; v < NW; ++v) if (v < wid) above += scan_w[v];
      if (above < need && above + c >= need) {               // exactly one thread
        int run = above;
#pragma unroll
        for (int j = 0; j < WPT; ++j) {
          const int word = PRUNE_HIST_WORDS - 1 - (tid * WPT + j);
          const int hi = (int)(w[j] >> 16), lo = (int)(w[j] & 0xffffu);
          if (run < need && run + hi >= need) { sel_bin = 2 * word + 1; sel_above = run; sel_count = hi; }
          run += hi;
          if (run < need && run + lo >= need) { sel_bin = 2 * word; sel_above = run; sel_count = lo; }
          run += lo;
        }
      }
      if (tid == 0) n_red = 0;
      __syncthreads();
      // cut the list down, in place: read, barrier, write
      const uint64_t cut = (prefix << 12) | (uint64_t)(uint32_t)sel_bin;
      const int undecided = sel_count;
      need -= sel_above;
      uint64_t rk[PER]; int32_t ri[PER];
#pragma unroll
      for (int k = 0; k < PER; ++k) {
        const int u = tid + k * NT;
        rk[k] = 0ull; ri[k] = -1;
        if (u < ns) { rk[k] = skey[u]; ri[k] = sidx[u]; }
      }
      __syncthreads();
#pragma unroll
      for (int k = 0; k < PER; ++k) {
        if (ri[k] >= 0 && (rk[k] >> shift) >= cut) {
          const int u = atomicAdd(&n_red, 1);
          skey[u] = rk[k]; sidx[u] = ri[k];
        }
      }
      for (int i = tid; i < PRUNE_HIST_WORDS; i += NT) hist[i] = 0u;   // for the next level, if there is one
      __syncthreads();
      ns = n_red;
      if (undecided <= PRUNE_UNDECIDED_MAX || shift < 12) break;      // (uniform) few enough to rank; or the last whole digit done
      prefix = cut; shift -= 12;
#pragma unroll
      for (int k = 0; k < PER; ++k) {
        const int u = tid + k * NT;
        if (u < ns) {
          const uint64_t key = skey[u];
          if ((key >> (shift + 12)) == prefix) {
            const uint32_t digit = (uint32_t)(key >> shift) & 0xfffu;
            atomicAdd(&hist[digit >> 1], (digit & 1u) ? 0x10000u : 1u);
          }
        }
      }
      __syncthreads();
    }
  }
  C2T_PT(PT_PRUNE_PRESELECTED);
  if (n_keep > 0) {
    int tshift = 0;
    while (tshift < 4 && (ns << (tshift + 1)) <= NT) ++tshift;
    const int T = 1 << tshift, sub = tid & (T - 1), ustride = NT >> tshift;
#pragma unroll 1
    for (int u0 = 0; u0 < ns; u0 += ustride) {               // uniform trip count: every lane meets in the DPP sums
      const int u = u0 + (tid >> tshift);
      const bool mine = u < ns;
      const uint64_t key = mine ? skey[u] : 0ull;
      const int i = mine ? sidx[u] : 0;
      const float z = key_to_float((uint32_t)(key >> 32));
      const int tok = (int)~(uint32_t)key;
      // what an appended node needs, requested before the ranking so that the latency overlaps it
      float P = 0.f, H = 0.f, par_s = INFINITY; int par = -1;
      if (mine && sub == 0) {
        const int64_t o = (int64_t)b * FK + i;
        P = ld_dev(s.c_P + o); H = ld_dev(s.c_H + o); par = s.fr_node[(int64_t)b * F + i / K];
        if (s.h_tok) par_s = s.fr_s[(int64_t)b * F + i / K];
      }
      // rank = survivors with a greater key, and those with the same key (the same token under two parents, with
      // the same z) and a lower candidate index; the survivor's T lanes take two keys a step each
      int rank = 0;
      if (mine) {
        for (int v = sub * 2; v < ns; v += T * 2) {
          const uint4 q = *(const uint4*)(skey + v);
          const uint64_t k0 = ((uint64_t)q.y << 32) | q.x, k1 = ((uint64_t)q.w << 32) | q.z;
          const bool in1 = v + 1 < ns;
          rank += (int)(k0 > key) + (int)(in1 && k1 > key);
          if (k0 == key && v != u) rank += (int)(sidx[v] < i);
          if (in1 && k1 == key && v + 1 != u) rank += (int)(sidx[v + 1] < i);
        }
      }
      if (tshift >= 1) rank += (int)dpp_u32<C2T_DPP_QUAD_XOR1, 0xf>(0u, (uint32_t)rank);
      if (tshift >= 2) rank += (int)dpp_u32<C2T_DPP_QUAD_XOR2, 0xf>(0u, (uint32_t)rank);
      if (tshift >= 3) rank += (int)dpp_u32<C2T_DPP_ROW_HALF_MIRROR, 0xf>(0u, (uint32_t)rank);
      if (tshift >= 4) rank += (int)dpp_u32<C2T_DPP_ROW_MIRROR, 0xf>(0u, (uint32_t)rank);
      if (mine && sub == 0 && rank < n_keep) {
        const int node = nn + rank, f = i / K;
        const int64_t o = (int64_t)b * FK + i, t = (int64_t)b * N + node;
        s.c_kept[o] = 1;
        s.t_tok[t] = tok; s.t_parent[t] = par; s.t_depth[t] = layer;
        s.t_P[t] = P; s.t_H[t] = H; s.t_z[t] = z;
        new_tok[rank] = tok; new_pslot[rank] = f; new_node[rank] = node; new_P[rank] = P;
        new_hidx[rank] = layer * FK + i; new_s[rank] = fminf(par_s, z);
      }
    }
  }
  __syncthreads();
  C2T_PT(PT_PRUNE_RANKED);
  if (tid < n_keep) {
    const int64_t o = (int64_t)b * F + tid;
    s.fr_tok[o] = new_tok[tid]; s.fr_pslot[o] = new_pslot[tid];
    s.fr_node[o] = new_node[tid]; s.fr_P[o] = new_P[tid];
    if (s.h_tok) { s.fr_hidx[o] = new_hidx[tid]; s.fr_s[o] = new_s[tid]; }
  }
  if (tid == 0) {
    if (s.h_tok) s.h_ncand[(int64_t)b * sp.D + layer] = ncand;
    s.n_nodes[b] = nn + n_keep;
    s.nf[(layer + 1) & 1][b] = n_keep;
    s.n_cand[b] = ncand;
    if (flags_or) s.status[b] |= (uint32_t)flags_or;
    if (n_keep) atomicAdd(&s.layer_rows[layer + 1], n_keep);
  }
}

// Thread 0 takes a ticket once its wave's device-coherent stores are complete: true for the
// workgroup that took the last of `expected` (it resets the counter for the next layer).  Every
// store the ticket publishes is issued by wave 0 (at most 64 candidates or list entries, lanes
// 0..63), whose own wait covers them; the other waves only meet at the barrier.
__device__ __forceinline__ bool last_arrival(int32_t* ticket, int expected) {
  __shared__ int32_t sh_last;
  if (threadIdx.x < WAVE) {
    wait_vector_memory();
    if (threadIdx.x == 0) {
      if (expected == 1) sh_last = 1;                      // the only arrival (root layers, chains): no round trip to the counter
      else {
        sh_last = __hip_atomic_fetch_add(ticket, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == expected - 1;
        if (sh_last) st_dev(ticket, 0);
      }
    }
  }
  __syncthreads();
  return sh_last != 0;
}

// Tail of the logits pass for the workgroup that owned (sequence b, frontier slot f, split): `rr`
// holds its segment's result.  The workgroup that completes a row scores the row's candidates; the
// workgroup that completes a sequence's last row prunes and appends.  Both overlap with the other
// workgroups' streaming, so the whole layer is one launch.
// after_merge(rr): called by the whole workgroup that has merged a split row, before the row is scored
// (the entropy over the M largest logits of a split row is computed there, over the whole row).
template <int NT, typename AfterMerge>
__device__ __forceinline__ void finish_layer(const TreeState& s, const ScoreParams& sp, int b, int f, int nf, int split,
                                             int64_t row_launched, RowResult& rr, unsigned char* lds,
                                             const float* __restrict__ cls, const float* cls_lds, AfterMerge after_merge) {
  const int tid = threadIdx.x, K = sp.K;
  __syncthreads();                                           // rr is complete
  if (sp.nsplit > 1) {
    const int64_t po = row_launched * sp.nsplit + split;
    if (tid < rr.part.n_top) { st_dev(sp.part_topv + po * K + tid, rr.topv[tid]); st_dev(sp.part_topi + po * K + tid, rr.topi[tid]); }
    if (tid == 0) st_dev(sp.part + po, rr.part);
    if (!last_arrival(s.row_tickets + (int64_t)b * sp.F + f, sp.nsplit)) return;
    merge_row(sp, row_launched, rr, lds, (size_t)sp.lds_bytes);
    after_merge(rr);
    C2T_PT(PT_MERGED);
  }
  score_row(s, sp, b, f, rr, cls, cls_lds);
  C2T_PT(PT_PUBLISHED);
  if (!last_arrival(s.tickets + b, nf)) return;              // nf: the sequence's frontier size, known since the workgroup started
  C2T_PT(PT_TICKET);
  prune_sequence<NT>(s, sp, b, nf, lds);
  C2T_PT(PT_PRUNED);
}

struct TreeOut {
  int32_t* tokens; int32_t* parent; int32_t* position; float* conf; float* joint_prob; float* entropy;
  int32_t* n_nodes; uint8_t* mask; uint32_t* status;
};

// One workgroup per sequence: copy the node arrays, confidence = sigmoid(z), ancestor mask.
__global__ __launch_bounds__(256) void k_finalize(TreeState s, TreeOut o, int N) {
  const int b = blockIdx.x, tid = threadIdx.x, nt = blockDim.x;
  const int n = s.n_nodes[b];
  uint8_t* mk = o.mask + (int64_t)b * N * N;
  // N*N bytes zeroed with 4-byte stores where alignment allows
  const int64_t nb = (int64_t)N * N;
  if ((((uintptr_t)mk) & 3) == 0) {
    uint32_t* m4 = (uint32_t*)mk;
    for (int64_t i = tid; i < nb / 4; i += nt) m4[i] = 0;
    for (int64_t i = (nb / 4) * 4 + tid; i < nb; i += nt) mk[i] = 0;
  } else {
    for (int64_t i = tid; i < nb; i += nt) mk[i] = 0;
  }
  for (int i = tid; i < N; i += nt) {
    const int64_t t = (int64_t)b * N + i;
    if (i < n) {
      const float z = s.t_z[t];
      o.tokens[t] = s.t_tok[t]; o.parent[t] = s.t_parent[t]; o.position[t] = s.t_depth[t] + 1;
      o.conf[t] = 1.0f / (1.0f + expf(-z));
      o.joint_prob[t] = s.t_P[t]; o.entropy[t] = s.t_H[t];
    } else {
      o.tokens[t] = -1; o.parent[t] = -1; o.position[t] = 0;
      o.conf[t] = 0.f; o.joint_prob[t] = 0.f; o.entropy[t] = 0.f;
    }
  }
  if (tid == 0) { o.n_nodes[b] = n; o.status[b] = s.status[b]; }
  __syncthreads();
  for (int i = tid; i < n; i += nt) {
    int j = i, guard = 0;
    while (j >= 0 && guard++ <= N) {       // parents have smaller indices: the walk ends at -1
      mk[(int64_t)i * N + j] = 1;
      j = s.t_parent[(int64_t)b * N + j];
    }
  }
}


// EAGLE-2-style reranking (Sec. 2.2), one workgroup of RR_NT threads per sequence: the n_out best of
// every candidate scored in this draft phase under the order (s desc, history index asc), s = the
// smallest classifier logit on the candidate's path (history index = layer * F*K + slot * K + rank
// in the row, so index order is depth, then scoring order).  The n_out-th best key is found exactly by
// a radix select over the order-preserving 32-bit keys of s (12 + 12 + 8 bits, an LDS histogram per
// pass over the sequence's history); candidates above it are taken, those equal to it in index
// order; the selection (<= 1024) is then ranked by counting.  Parents precede children because s
// never increases along a path.
constexpr int RR_NT = 1024;
__global__ __launch_bounds__(RR_NT) void k_finalize_rerank(TreeState s, TreeOut o, int n_out, int D, int FK) {
  constexpr int NW = RR_NT / WAVE;
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & (WAVE - 1), wid = tid >> 6;
  const int total = D * FK;
  const int32_t* tok = s.h_tok + (int64_t)b * total; const int32_t* par = s.h_par + (int64_t)b * total;
  const float* hs = s.h_s + (int64_t)b * total;
  const int32_t* ncand = s.h_ncand + (int64_t)b * D;
  int32_t* pos = s.h_pos + (int64_t)b * total;
  __shared__ uint32_t dig[4096];
  __shared__ int32_t scan_w[NW];
  __shared__ int32_t sh_digit, sh_above, sh_n;
  __shared__ float sel_s[C2T_MAX_BUDGET_DEV];
  __shared__ int32_t sel_i[C2T_MAX_BUDGET_DEV], sel_par[C2T_MAX_BUDGET_DEV], sel_depth[C2T_MAX_BUDGET_DEV];
  // a thread owns a contiguous range of history indices, so that index order = thread order
  const int per = (total + RR_NT - 1) / RR_NT, i0 = min(tid * per, total), i1 = min(i0 + per, total);
  auto valid = [&](int i) { return (i % FK) < ncand[i / FK] && tok[i] >= 0; };
  int my_valid = 0;
  for (int i = i0; i < i1; ++i) my_valid += valid(i);
  {
    const int incl = wave_scan_incl(my_valid);
    if (lane == WAVE - 1) scan_w[wid] = incl;
    __syncthreads();
    if (tid == 0) { int t = 0; for (int w = 0; w < NW; ++w) t += scan_w[w]; sh_n = t; }
    __syncthreads();
  }
  const int n_all = sh_n, n = min(n_out, n_all);
  uint32_t prefix = 0, care = 0;
  int remaining = n;
  if (n > 0 && n < n_all) {
    const int shifts[3] = {20, 8, 0}, widths[3] = {12, 12, 8};
#pragma unroll 1
    for (int ps = 0; ps < 3; ++ps) {
      const int shift = shifts[ps]; const uint32_t dmask = (1u << widths[ps]) - 1u;
      for (int i = tid; i < 4096; i += RR_NT) dig[i] = 0u;
      __syncthreads();
      for (int i = i0; i < i1; ++i) {
        if (!valid(i)) continue;
        const uint32_t key = sortable_key(hs[i]);
        if ((key & care) == prefix) atomicAdd(&dig[(key >> shift) & dmask], 1u);
      }
      __syncthreads();
      {                                                      // thread t owns digits 4095-4t .. 4092-4t
        uint32_t c[4]; int tot = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) { c[j] = dig[4095 - (4 * tid + j)]; tot += (int)c[j]; }
        const int incl = wave_scan_incl(tot);
        if (lane == WAVE - 1) scan_w[wid] = incl;
        __syncthreads();
        int run = incl - tot;
#pragma unroll
        for (int w = 0; w < NW; ++w) if (w < wid) run += scan_w[w];
        if (run < remaining && run + tot >= remaining) {
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            if (run < remaining && run + (int)c[j] >= remaining) { sh_digit = 4095 - (4 * tid + j); sh_above = run; }
            run += (int)c[j];
          }
        }
        __syncthreads();
      }
      remaining -= sh_above;
      prefix |= (uint32_t)sh_digit << shift; care |= dmask << shift;
      __syncthreads();
    }
  }
  // take: keys above the n-th best key, and the first `remaining` equal to it in index order
  const bool take_all = n >= n_all;
  int my_gt = 0, my_eq = 0;
  for (int i = i0; i < i1; ++i) {
    if (!valid(i)) continue;
    const uint32_t key = sortable_key(hs[i]);
    my_gt += take_all || key > prefix; my_eq += !take_all && key == prefix;
  }
  int before_gt, before_eq;
  {
    const int ig = wave_scan_incl(my_gt), ie = wave_scan_incl(my_eq);
    __shared__ int32_t scan_e[NW];
    if (lane == WAVE - 1) { scan_w[wid] = ig; scan_e[wid] = ie; }
    __syncthreads();
    before_gt = ig - my_gt; before_eq = ie - my_eq;
    int tot_gt = 0;
#pragma unroll
    for (int w = 0; w < NW; ++w) { if (w < wid) { before_gt += scan_w[w]; before_eq += scan_e[w]; } tot_gt += scan_w[w]; }
    // slots: the keys above first (any order), then the ties in index order
    int sg = before_gt, se = before_eq;
    for (int i = i0; i < i1; ++i) {
      if (!valid(i)) continue;
      const uint32_t key = sortable_key(hs[i]);
      int slot = -1;
      if (take_all || key > prefix) slot = sg++;
      else if (key == prefix) { if (se < remaining) slot = tot_gt + se; ++se; }
      if (slot >= 0 && slot < n) { sel_s[slot] = hs[i]; sel_i[slot] = i; }
    }
  }
  __syncthreads();
  // rank the selection by (s desc, index asc) and emit
  for (int e = tid; e < n; e += RR_NT) {
    const float v = sel_s[e]; const int id = sel_i[e];
    int rank = 0;
    for (int q = 0; q < n; ++q) { const float vq = sel_s[q]; rank += (vq > v) || (vq == v && sel_i[q] < id); }
    pos[id] = rank;
    sel_depth[rank] = id / FK;
    const int64_t t = (int64_t)b * n_out + rank, h = (int64_t)b * total + id;
    o.tokens[t] = tok[id]; o.position[t] = id / FK + 1;
    o.conf[t] = 1.0f / (1.0f + expf(-s.h_z[h])); o.joint_prob[t] = s.h_P[h]; o.entropy[t] = s.h_H[h];
  }
  for (int e = n + tid; e < n_out; e += RR_NT) {
    const int64_t t = (int64_t)b * n_out + e;
    o.tokens[t] = -1; o.parent[t] = -1; o.position[t] = 0; o.conf[t] = 0.f; o.joint_prob[t] = 0.f; o.entropy[t] = 0.f;
  }
  uint8_t* mk = o.mask + (int64_t)b * n_out * n_out;
  {
    const int64_t nb = (int64_t)n_out * n_out;               // zeroed with 4-byte stores where alignment allows
    if ((((uintptr_t)mk) & 3) == 0) {
      for (int64_t i = tid; i < nb / 4; i += RR_NT) ((uint32_t*)mk)[i] = 0u;
      for (int64_t i = (nb / 4) * 4 + tid; i < nb; i += RR_NT) mk[i] = 0;
    } else {
      for (int64_t i = tid; i < nb; i += RR_NT) mk[i] = 0;
    }
  }
  __threadfence_block();
  __syncthreads();                                           // pos[] of every selected candidate is written
  for (int e = tid; e < n; e += RR_NT) {
    const int id = sel_i[e], rank = pos[id], pid = par[id];
    const int prank = pid < 0 ? -1 : pos[pid];
    sel_par[rank] = prank;
    o.parent[(int64_t)b * n_out + rank] = prank;
  }
  __syncthreads();
  for (int r = tid; r < n; r += RR_NT)
    for (int j = r; j >= 0; j = sel_par[j]) mk[(int64_t)r * n_out + j] = 1;
  if (tid == 0) { o.n_nodes[b] = n; o.status[b] = s.status[b]; }
}

}  // namespace c2t
