// Per-sequence kernels: merge the row partials, features + classifier (Eq. 1-3), the two
// prunings of Sec. 4.2 with the node budget, tree append; reset; emission of the tree mask,
// position ids and parent links.
#pragma once
#include "k_common.h"

namespace c2t {

struct TreeState {            // device pointers into the workspace
  float* cls;                 // W1[3h] b1[h] w2[h] b2
  int32_t* n_nodes;           // [B]
  int32_t* n_frontier;        // [B]
  uint32_t* status;           // [B]
  int32_t* n_cand;            // [B]
  int32_t* layer_rows;        // [D+1]
  int32_t* fr_tok;            // [B][F]
  int32_t* fr_pslot;          // [B][F]
  int32_t* fr_node;           // [B][F]
  float* fr_P;                // [B][F]
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
  if (i < B) {
    s.n_nodes[i] = 0; s.n_frontier[i] = 1; s.status[i] = 0; s.n_cand[i] = 0;
    s.fr_tok[(int64_t)i * F] = -1; s.fr_pslot[(int64_t)i * F] = 0;
    s.fr_node[(int64_t)i * F] = -1; s.fr_P[(int64_t)i * F] = 1.0f;
  }
  if (i <= D) s.layer_rows[i] = (i == 0) ? B : 0;
}

// Eq. 3 in fp32: fixed chain of fused multiply-adds, hidden units in ascending order.
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

constexpr int SP_MAX_F = 64;

// One workgroup per sequence.  Dynamic LDS: (5h+1) floats (padded to 4) + 5 arrays of F*K (padded to 4)
// 4-byte entries: z, token, survivor index, P, survivor z.
__global__ __launch_bounds__(1024) void k_score_prune(
    TreeState s, const RowPartial* __restrict__ part, const float* __restrict__ part_topv,
    const int32_t* __restrict__ part_topi, int nsplit, int rows_per_seq, int F, int K, int N, int h, int layer,
    float z_beta) {
  extern __shared__ __align__(16) unsigned char dyn_lds[];
  float* w = (float*)dyn_lds;
  const int FK = F * K, FKp = (FK + 3) & ~3;
  float* cz = w + ((5 * h + 1 + 3) & ~3);
  int32_t* ctok = (int32_t*)(cz + FKp);
  int32_t* surv = ctok + FKp;
  float* cP = (float*)(surv + FKp);
  float* sz = cP + FKp;                                   // z of the survivors, contiguous, 16-byte aligned
  __shared__ double rowZ[SP_MAX_F], rowC[SP_MAX_F];
  __shared__ float rowH[SP_MAX_F], parP[SP_MAX_F];
  __shared__ int32_t rowBad[SP_MAX_F], parNode[SP_MAX_F];
  __shared__ int32_t n_surv, any_bad, any_slow;

  const int b = blockIdx.x, tid = threadIdx.x, nt = blockDim.x;
  const int nf = s.n_frontier[b];
  const int nn = s.n_nodes[b];
  for (int i = tid; i < 5 * h + 1; i += nt) w[i] = s.cls[i];
  if (tid == 0) { n_surv = 0; any_bad = 0; any_slow = 0; }
  __syncthreads();

  // ---- per row: merge the splits (fp64), entropy of Eq. 2 ----
  if (tid < nf) {
    const RowPartial* rp = part + ((int64_t)b * rows_per_seq + tid) * nsplit;
    double R = -INFINITY; uint32_t fl = 0;
    for (int q = 0; q < nsplit; ++q) { R = fmax(R, rp[q].ref); fl |= rp[q].flags & 1u; if (rp[q].flags & 2u) any_slow = 1; }
    double Z = 0.0, S = 0.0;
    for (int q = 0; q < nsplit; ++q) {
      const double Zq = rp[q].Z;
      if (Zq > 0.0 && rp[q].ref > -INFINITY) {
        const double da = rp[q].a - R, dl = rp[q].ref - R;   // re-reference to the row maximum R; dl <= 0
        const double sc = da == 0.0 ? 1.0 : exp(da);
        Z += Zq * sc; S += (rp[q].S + dl * Zq) * sc;
      }
    }
    const bool bad = fl != 0 || !(Z > 0.0) || !(R > -INFINITY) || !(R < INFINITY);
    // p_j = e^(x_j - R) / Z  =>  H = -sum p ln p = ln Z - S / Z
    const double H = bad ? 0.0 : log(Z) - S / Z;
    rowZ[tid] = Z; rowC[tid] = R; rowH[tid] = (float)H; rowBad[tid] = bad;
    parP[tid] = s.fr_P[(int64_t)b * F + tid];
    parNode[tid] = s.fr_node[(int64_t)b * F + tid];
    if (bad) any_bad = 1;
  }
  __syncthreads();

  // ---- merged top-K of each row: (logit, id) into (cz, ctok) ----
  const int ncand = nf * K;
  for (int i = tid; i < ncand; i += nt) { cz[i] = 0.f; ctok[i] = -1; }
  __syncthreads();
  if (nsplit == 1) {
    for (int i = tid; i < ncand; i += nt) {
      const int f = i / K, r = i % K;
      const int64_t base = (int64_t)b * rows_per_seq + f;
      if (!rowBad[f] && r < part[base].n_top) { cz[i] = part_topv[base * K + r]; ctok[i] = part_topi[base * K + r]; }
    }
  } else {
    // An entry's merged rank = number of entries of the row's lists ahead of it.  Rows are taken
    // in groups whose lists fit the staging area (surv/cP are free until the scoring step).
    float* sv = (float*)surv; int32_t* si = (int32_t*)cP;
    const int per_row = nsplit * K;
    const int rows_per_group = max(1, FK / per_row);       // staging holds FK entries
    for (int f0 = 0; f0 < nf; f0 += rows_per_group) {
      const int nr = min(rows_per_group, nf - f0);
      if (per_row <= FK) {
        for (int ent = tid; ent < nr * per_row; ent += nt) {
          const int f = f0 + ent / per_row, q = (ent % per_row) / K, e = ent % K;
          const int64_t base = ((int64_t)b * rows_per_seq + f) * nsplit;
          const bool ok = !rowBad[f] && e < part[base + q].n_top;
          sv[ent] = ok ? part_topv[(base + q) * K + e] : 0.f;
          si[ent] = ok ? part_topi[(base + q) * K + e] : -1;
        }
        __syncthreads();
        for (int ent = tid; ent < nr * per_row; ent += nt) {
          const int vi = si[ent];
          if (vi < 0) continue;
          const float v = sv[ent];
          const int r0 = (ent / per_row) * per_row;
          int ahead = 0;
          for (int o = r0; o < r0 + per_row; ++o) {
            const int oi = si[o];
            ahead += oi >= 0 && ((sv[o] > v) || (sv[o] == v && oi < vi));
          }
          if (ahead < K) { const int f = f0 + ent / per_row; cz[f * K + ahead] = v; ctok[f * K + ahead] = vi; }
        }
        __syncthreads();
      } else {
        // one row's lists exceed the staging area (very many splits): rank from global memory
        for (int ent = tid; ent < per_row; ent += nt) {
          const int f = f0, q = ent / K, e = ent % K;
          const int64_t base = ((int64_t)b * rows_per_seq + f) * nsplit;
          if (rowBad[f] || e >= part[base + q].n_top) continue;
          const float v = part_topv[(base + q) * K + e]; const int vi = part_topi[(base + q) * K + e];
          int ahead = 0;
          for (int q2 = 0; q2 < nsplit; ++q2) {
            const int n2 = part[base + q2].n_top;
            for (int e2 = 0; e2 < n2; ++e2) {
              const float v2 = part_topv[(base + q2) * K + e2];
              ahead += (v2 > v) || (v2 == v && part_topi[(base + q2) * K + e2] < vi);
            }
          }
          if (ahead < K) { cz[f * K + ahead] = v; ctok[f * K + ahead] = vi; }
        }
      }
    }
  }
  __syncthreads();

  // ---- per candidate: p, P (Eq. 1), z (Eq. 3), first pruning ----
  for (int i = tid; i < ncand; i += nt) {
    const int f = i / K;
    float z = -INFINITY; int tok = -1;
    float p32 = 0.f, P32 = 0.f;
    {
      const float x = cz[i]; const int id = ctok[i];
      if (id >= 0) {
        p32 = (float)(exp((double)x - rowC[f]) / rowZ[f]);
        P32 = parP[f] * p32;
        z = mlp_logit(w, h, P32, rowH[f], (float)layer);
        tok = id;
      }
    }
    cz[i] = z; ctok[i] = tok; cP[i] = P32;
    const int64_t o = (int64_t)b * FK + i;
    s.c_tok[o] = tok; s.c_p[o] = p32; s.c_P[o] = P32; s.c_H[o] = rowBad[f] ? 0.f : rowH[f]; s.c_z[o] = z;
    s.c_kept[o] = 0;
    if (tok >= 0 && z > z_beta) { const int u = atomicAdd(&n_surv, 1); surv[u] = i; sz[u] = z; }
  }
  __syncthreads();

  // ---- second pruning + budget: rank survivors by (z desc, token asc, slot asc) ----
  const int ns = n_surv;
  const int n_keep = max(0, min(min(F, N - nn), ns));
  __shared__ int32_t new_tok[SP_MAX_F], new_pslot[SP_MAX_F], new_node[SP_MAX_F];
  __shared__ float new_P[SP_MAX_F];
  for (int u = tid; u < ns; u += nt) {
    const int i = surv[u];
    const float z = sz[u]; const int tok = ctok[i];
    int rank = 0;
    // survivors ahead of this one: larger z, or equal z and (token, slot) smaller
    auto tie = [&](int v) {
      const int j = surv[v];
      if (j != i) { const int tj = ctok[j]; rank += (tj < tok) || (tj == tok && j < i); }
    };
    int v = 0;
#pragma unroll 2
    for (; v + 4 <= ns; v += 4) {
      const float4 q = *(const float4*)(sz + v);
      rank += (q.x > z) + (q.y > z) + (q.z > z) + (q.w > z);
      if (q.x == z || q.y == z || q.z == z || q.w == z) {
        if (q.x == z) tie(v);
        if (q.y == z) tie(v + 1);
        if (q.z == z) tie(v + 2);
        if (q.w == z) tie(v + 3);
      }
    }
    for (; v < ns; ++v) { const float zj = sz[v]; if (zj > z) ++rank; else if (zj == z) tie(v); }
    if (rank < n_keep) {
      const int f = i / K;
      const int node = nn + rank;
      const int64_t o = (int64_t)b * FK + i, t = (int64_t)b * N + node;
      s.c_kept[o] = 1;
      s.t_tok[t] = tok; s.t_parent[t] = parNode[f]; s.t_depth[t] = layer;
      s.t_P[t] = cP[i]; s.t_H[t] = rowH[f]; s.t_z[t] = z;
      new_tok[rank] = tok; new_pslot[rank] = f; new_node[rank] = node; new_P[rank] = cP[i];
    }
  }
  __syncthreads();
  if (tid < n_keep) {
    const int64_t o = (int64_t)b * F + tid;
    s.fr_tok[o] = new_tok[tid]; s.fr_pslot[o] = new_pslot[tid];
    s.fr_node[o] = new_node[tid]; s.fr_P[o] = new_P[tid];
  }
  if (tid == 0) {
    s.n_nodes[b] = nn + n_keep;
    s.n_frontier[b] = n_keep;
    s.n_cand[b] = ncand;
    if (any_bad) s.status[b] |= 1u;
    if (any_slow) s.status[b] |= 2u;
    if (n_keep) atomicAdd(&s.layer_rows[layer + 1], n_keep);
  }
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

}  // namespace c2t
