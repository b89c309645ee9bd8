// Host side of the C ABI declared in include/c2t.h: argument checks, workspace carving,
// launch shapes.  Every step of the path runs in the kernels of k_logits.h / k_tree.h;
// nothing here touches logits or tree data on the host, allocates device memory or
// synchronises the device.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <new>
#include <vector>

#include <hip/hip_ext.h>

#include "../../include/c2t.h"
#include "k_logits.h"
#include "k_tree.h"

using namespace c2t;

static __device__ __align__(256) int32_t scratch[C2T_STATIC_RERANK_ENTRIES];   // see scratch_on_current_device

namespace {

constexpr size_t ALIGN = 256;
static_assert(C2T_MAX_BUDGET == C2T_MAX_BUDGET_DEV && C2T_MAX_CANDIDATES == C2T_MAX_CANDIDATES_DEV && C2T_MAX_FRONTIER == SP_MAX_F && C2T_MAX_TOP_K == 64,
              "limits of the C ABI and of the kernels must agree");
// Cell map of one workgroup.  bf16: four workgroups of 512 threads share the CU's 160 KB, each with the
// 16 KB histogram, its static LDS (under 8 KB) and the map (2 bytes per 4 chunks): 16 KB at most.
constexpr int HP_NT = 512;                     // workgroup size of the histogram kernel
#ifndef C2T_HP_REPL_ALONE
#define C2T_HP_REPL_ALONE 4
#endif
constexpr int HP_REPL_ALONE = C2T_HP_REPL_ALONE;   // histogram copies of a workgroup that has its CU to itself (launches of at most one workgroup per CU)
constexpr int MAX_MAP_BYTES_BF16 = 16 * 1024;
constexpr int MAX_MAP_BYTES_F32 = 48 * 1024;
constexpr int NT_F32 = 512;                    // workgroup size of the generic kernel for fp32 logits (cfg1: 28.3 / 26.7 / 31.0 us per layer with 256 / 512 / 1024)
constexpr int PARTIAL_SLOTS_MIN = 16384;       // (row, split) records the workspace always has room for
// Row splits.  A split adds an epilogue, a device-scope ticket and a merge (a few microseconds of
// dependent round trips), which costs more than it saves on the histogram path even for a single
// sequence; the two-pass fp32 path is compute-heavy (an fp64 exp per element) and gains from a few.
constexpr int TARGET_WORKGROUPS_F32 = 256;
constexpr int MAX_DEFAULT_SPLITS_F32 = 4;
// Shared rows on the histogram path (share_row): a launch of few rows, each a workgroup alone on its
// CU, spreads every row over several CUs instead; the workgroups hand their counts over before
// the epilogue, so the row still has one epilogue and no merge of lists.
#ifndef C2T_COOP_MAX_SHARE
#define C2T_COOP_MAX_SHARE 5
#endif
#ifndef C2T_COOP_MIN_GROUPS
#define C2T_COOP_MIN_GROUPS 4
#endif
constexpr int COOP_MAX_WORKGROUPS = 256;       // workgroups of such a launch: one per CU at most
constexpr int COOP_MAX_ROWS = COOP_MAX_WORKGROUPS / 2;
constexpr int COOP_MAX_SHARE = C2T_COOP_MAX_SHARE;     // workgroups per row at most
constexpr int COOP_MIN_GROUPS = C2T_COOP_MIN_GROUPS;   // shortest row that is shared, in groups of HP_CPC sweeps (32 KB)
constexpr int COOP_GROUP_CHUNKS = HP_CPC * HP_NT;      // segments are whole groups: the row's cell map is then the segments' maps end to end

inline size_t align_up(size_t x) { return (x + ALIGN - 1) / ALIGN * ALIGN; }

struct Layout {
  size_t cls, n_nodes, nf0, nf1, tickets, row_tickets, row_info, status, n_cand, layer_rows;
  size_t fr_tok, fr_pslot, fr_node, fr_P, fr_hidx, fr_s;
  size_t h_tok, h_par, h_P, h_H, h_z, h_s, h_ncand, h_pos;   // rerank contexts only
  size_t t_tok, t_parent, t_depth, t_P, t_H, t_z;
  size_t c_tok, c_p, c_P, c_H, c_z, c_kept;
  size_t part, part_topv, part_topi, tab_e;
  size_t coop_hist, coop_map, coop_acc;                      // shared rows (bf16 rows whose cell map fits one workgroup's LDS)
  int coop_map_stride;                                       // keys per row there; 0: no shared rows for this configuration
  size_t total;
  int64_t partial_slots;
};

int epc_of(const c2t_config& c) { return c.logits_dtype == C2T_BF16 ? 8 : 4; }
int keybytes_of(const c2t_config& c) { return c.logits_dtype == C2T_BF16 ? 2 : 4; }
int chunks_of(const c2t_config& c) { return (c.vocab + epc_of(c) - 1) / epc_of(c); }
// fewest splits for which one workgroup's cell map fits its LDS budget
int cpc_of(const c2t_config& c) { return c.logits_dtype == C2T_BF16 ? HP_CPC : 1; }   // chunks per map cell
int min_splits(const c2t_config& c) {
  const int max_chunks = (c.logits_dtype == C2T_BF16 ? MAX_MAP_BYTES_BF16 : MAX_MAP_BYTES_F32) / keybytes_of(c) * cpc_of(c);
  return (chunks_of(c) + max_chunks - 1) / max_chunks;
}

int check_config(const c2t_config* c) {
  if (!c) return C2T_ERR_INVALID_ARG;
  if (c->batch <= 0 || c->vocab <= 0 || c->max_frontier <= 0 || c->top_k <= 0 || c->max_depth <= 0 ||
      c->budget <= 0 || c->hidden <= 0)
    return C2T_ERR_INVALID_ARG;
  if (!(c->beta >= 0.0f && c->beta < 1.0f)) return C2T_ERR_INVALID_ARG;
  if (c->logits_dtype != C2T_F32 && c->logits_dtype != C2T_BF16) return C2T_ERR_INVALID_ARG;
  if (c->top_k > c->vocab || c->entropy_top_m < 0 || (c->rerank != 0 && c->rerank != 1)) return C2T_ERR_INVALID_ARG;
  if (c->top_k > C2T_MAX_TOP_K || c->max_frontier > C2T_MAX_FRONTIER || c->hidden > C2T_MAX_HIDDEN ||
      c->budget > C2T_MAX_BUDGET || (int64_t)c->max_frontier * c->top_k > C2T_MAX_CANDIDATES)
    return C2T_ERR_UNSUPPORTED;
  if (c->rerank && (int64_t)c->max_depth * c->max_frontier * c->top_k > C2T_MAX_HISTORY) return C2T_ERR_UNSUPPORTED;
  if ((int64_t)c->batch * c->max_frontier * min_splits(*c) > (1 << 24)) return C2T_ERR_UNSUPPORTED;
  return C2T_OK;
}

Layout make_layout(const c2t_config& c) {
  Layout L;
  size_t o = 0;
  auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes); return at; };
  const size_t B = c.batch, F = c.max_frontier, K = c.top_k, N = c.budget, h = c.hidden;
  L.cls = take((5 * h + 1) * 4);
  L.n_nodes = take(B * 4); L.nf0 = take(B * 4); L.nf1 = take(B * 4); L.tickets = take(B * 4);
  L.row_tickets = take(B * F * 4); L.row_info = take(B * F * 4); L.status = take(B * 4); L.n_cand = take(B * 4);
  L.layer_rows = take((c.max_depth + 1) * 4);
  L.fr_tok = take(B * F * 4); L.fr_pslot = take(B * F * 4); L.fr_node = take(B * F * 4); L.fr_P = take(B * F * 4);
  L.t_tok = take(B * N * 4); L.t_parent = take(B * N * 4); L.t_depth = take(B * N * 4);
  L.t_P = take(B * N * 4); L.t_H = take(B * N * 4); L.t_z = take(B * N * 4);
  L.c_tok = take(B * F * K * 4); L.c_p = take(B * F * K * 4); L.c_P = take(B * F * K * 4);
  L.c_H = take(B * F * K * 4); L.c_z = take(B * F * K * 4); L.c_kept = take(B * F * K * 4);
  L.partial_slots = std::max<int64_t>((int64_t)B * F * min_splits(c), PARTIAL_SLOTS_MIN);
  L.part = take((size_t)L.partial_slots * sizeof(RowPartial));
  L.part_topv = take((size_t)L.partial_slots * K * 4);
  L.part_topi = take((size_t)L.partial_slots * K * 4);
  L.tab_e = take((size_t)HP_TAB_DOUBLES * 8);
  L.coop_hist = L.coop_map = L.coop_acc = 0; L.coop_map_stride = 0;
  if (c.logits_dtype == C2T_BF16 && min_splits(c) == 1 && (chunks_of(c) + COOP_GROUP_CHUNKS - 1) / COOP_GROUP_CHUNKS >= COOP_MIN_GROUPS) {
    L.coop_map_stride = (cells_in_segment<HP_NT, HP_CPC>(chunks_of(c)) + 7) / 8 * 8;
    L.coop_hist = take((size_t)COOP_MAX_WORKGROUPS * HP_WORDS * 4);
    L.coop_map = take((size_t)COOP_MAX_ROWS * L.coop_map_stride * 2);
    L.coop_acc = take((size_t)COOP_MAX_WORKGROUPS * sizeof(CoopAcc));
  }
  L.fr_hidx = L.fr_s = L.h_tok = L.h_par = L.h_P = L.h_H = L.h_z = L.h_s = L.h_ncand = L.h_pos = 0;
  if (c.rerank) {
    const size_t H = B * (size_t)c.max_depth * F * K * 4;
    L.fr_hidx = take(B * F * 4); L.fr_s = take(B * F * 4);
    L.h_tok = take(H); L.h_par = take(H); L.h_P = take(H); L.h_H = take(H); L.h_z = take(H); L.h_s = take(H);
    L.h_ncand = take(B * (size_t)c.max_depth * 4); L.h_pos = take(H);
  }
  L.total = o;
  return L;
}

// Scratch of c2t_finalize_tree_reranked_static: the reranking's position array (one int per history
// entry, [B][D*F*K]) in a file-scope device array instead of the caller's workspace.  Every GPU the
// library runs on holds its own copy until the process ends.  In host code the array's name is only
// a stand-in: its device address is asked for once per device (with that device current) and kept.
constexpr int MAX_DEVICES = 64;
std::atomic<int32_t*> scratch_ptr[MAX_DEVICES];

// Device address of `scratch` on the current device; nullptr (and *err set) if it cannot be had.
int32_t* scratch_on_current_device(hipError_t* err) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess || dev < 0 || dev >= MAX_DEVICES) { if (err) *err = e != hipSuccess ? e : hipErrorInvalidDevice; return nullptr; }
  int32_t* p = scratch_ptr[dev].load(std::memory_order_acquire);
  if (p) return p;
  void* sym = nullptr;
  e = hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch));
  if (e != hipSuccess || !sym) { if (err) *err = e != hipSuccess ? e : hipErrorInvalidSymbol; return nullptr; }
  scratch_ptr[dev].store((int32_t*)sym, std::memory_order_release);   // two threads racing here store the same address
  return (int32_t*)sym;
}

}  // namespace

struct c2t_ctx {
  c2t_config cfg;
  Layout lay;
  char* ws;
  TreeState st;
  RowPartial* part;
  float* part_topv;
  int32_t* part_topi;
  double* tab_e;
  float z_beta;
  int layer;          // layers expanded since reset; -1 before the first reset
  bool have_cls, finalized;
  int ns_first, ns_other;      // row splits in use
  bool share_first, share_other;   // rows may be shared by workgroups (the default; off where the caller has set the splits itself)
  size_t lds_raised[3];        // dynamic LDS this context has asked the runtime to allow each build of its layer kernel so far
  int n_cus;                   // compute units of the device the context was created on
  // optional event timing of the logits pass
  std::vector<hipEvent_t> ev;
  int ev_used;
  int sample_every, sample_first, phase_no;   // events go to the launches of draft phases sample_first, sample_first + sample_every, ...
};

namespace {

// default number of workgroups a row is split over when `rows` rows are launched
int default_split(const c2t_config& c, const Layout& L, int64_t rows) {
  const int nmin = min_splits(c);
  if (c.logits_dtype == C2T_BF16 || c.entropy_top_m > 0) return nmin;
  const int by_size = std::max(1, chunks_of(c) / NT_F32);   // at least one full sweep of the workgroup
  const int64_t want = std::min<int64_t>((TARGET_WORKGROUPS_F32 + rows - 1) / rows, MAX_DEFAULT_SPLITS_F32);
  const int64_t cap = L.partial_slots / rows;
  const int64_t ns = std::min<int64_t>(std::min<int64_t>(want, by_size), cap);
  return (int)std::max<int64_t>(ns, nmin);
}

// Workgroups that share a row when `rows` rows are launched unsplit; 1: rows are not shared.
// Every workgroup gets at least one whole group of chunks, and there is at most one workgroup per CU.
struct Share { int n, groups_each; };
Share share_of(const c2t_config& c, const Layout& L, int n_cus, int64_t rows) {
  Share none{1, 0};
  if (L.coop_map_stride == 0 || rows > COOP_MAX_ROWS) return none;
  const int groups = (chunks_of(c) + COOP_GROUP_CHUNKS - 1) / COOP_GROUP_CHUNKS;
  const int64_t workgroups = std::min<int64_t>(n_cus, COOP_MAX_WORKGROUPS);
  const int n_max = (int)std::min<int64_t>(std::min<int64_t>(workgroups / rows, COOP_MAX_SHARE), groups);
  if (n_max < 2 || groups < COOP_MIN_GROUPS) return none;
  Share sh;
  sh.groups_each = (groups + n_max - 1) / n_max;
  sh.n = (groups + sh.groups_each - 1) / sh.groups_each;    // the last workgroup's segment starts inside the row
  return sh.n >= 2 ? sh : none;
}

// ev0/ev1: optional events attached to the dispatch itself (they take the kernel's own begin and
// end times, without the launch gap that events recorded around a launch include).
hipError_t launch_logits(c2t_ctx* x, const void* logits, int64_t stride, int rows_per_seq, int nsplit, bool may_share,
                         hipStream_t s, hipEvent_t ev0, hipEvent_t ev1) {
  const c2t_config& c = x->cfg;
  const int cpc = cpc_of(c);
  const Share share = (may_share && nsplit == 1) ? share_of(c, x->lay, x->n_cus, (int64_t)c.batch * rows_per_seq) : Share{1, 0};
  const int per_row = share.n > 1 ? share.n : nsplit;       // workgroups per row
  const int cps = share.n > 1 ? share.groups_each * COOP_GROUP_CHUNKS : (chunks_of(c) + nsplit - 1) / nsplit;
  // the cell map in LDS: the workgroup's segment; the whole row where rows are shared (the workgroup that finishes the row loads it)
  const int cells = c.logits_dtype == C2T_BF16 ? cells_in_segment<HP_NT, HP_CPC>(share.n > 1 ? chunks_of(c) : cps) : cps;
  const size_t map_lds = ((size_t)cells * keybytes_of(c) + 15) / 16 * 16;
  // element list of the selection: (2K-1) cells of cpc chunks, 8 bytes per element
  const size_t list_lds = (size_t)(2 * c.top_k - 1) * cpc * epc_of(c) * 8;
  const size_t score_lds = score_lds_bytes(c.hidden, c.max_frontier * c.top_k);
  const unsigned grid = (unsigned)((int64_t)c.batch * rows_per_seq * per_row);
  ScoreParams sp;
  sp.part = x->part; sp.part_topv = x->part_topv; sp.part_topi = x->part_topi;
  sp.nsplit = nsplit; sp.rows_per_seq = rows_per_seq; sp.B = c.batch; sp.F = c.max_frontier; sp.K = c.top_k; sp.N = c.budget;
  sp.coop = share.n; sp.coop_map_stride = x->lay.coop_map_stride;
  sp.coop_hist = (uint32_t*)(x->ws + x->lay.coop_hist); sp.coop_map = (uint16_t*)(x->ws + x->lay.coop_map);
  sp.coop_acc = (CoopAcc*)(x->ws + x->lay.coop_acc);
  // one round of workgroups (static placement), more of them than CUs, and few enough sequences:
  // deal the live rows round the CUs
  sp.compact = (rows_per_seq > 1 && (int64_t)grid > (int64_t)x->n_cus && (int64_t)grid <= 4 * (int64_t)x->n_cus &&
                c.batch <= COMPACT_MAX_B) ? 1 : 0;
  sp.h = c.hidden; sp.layer = x->layer; sp.z_beta = x->z_beta; sp.M = c.entropy_top_m; sp.D = c.max_depth;
  if (c.logits_dtype == C2T_BF16) {
    const int64_t cus = x->n_cus;
    const bool four_per_cu = (int64_t)grid > cus;
    const int repl = four_per_cu ? 1 : HP_REPL_ALONE;       // copies of the histogram in LDS
    const size_t lds_work = (std::max(std::max((size_t)HP_WORDS * 4 * repl + map_lds, list_lds), score_lds) + 15) / 16 * 16;
    sp.lds_bytes = (int)lds_work;
    sp.w_lds_off = (int)lds_work;                           // behind it: the classifier's parameters, padded to 16 bytes
    const size_t lds = lds_work + ((size_t)(5 * c.hidden + 1) * 4 + 15) / 16 * 16;
    const int topm = c.entropy_top_m > 0;
    // Two builds of the kernel.  Four workgroups per CU on 64 registers a lane, or three per CU on
    // 80 registers.  Measured on full layers of V = 128256 (us per layer, four / three per CU):
    // 256 rows 32.4 / 31.6, 512: 38.8 / 39.8, 1024: 61.0 / 73.1, 1280: 82.7 / 86.6, 1536: 95.3 / 91.6,
    // 2048: 114 / 120, 3072: 166 / 163, 4096: 209 / 215, 8192: 388 / 393.  Four per CU whenever a CU
    // gets more than one workgroup; a workgroup that is alone on its CU is 2-3 % faster on 80 registers.
    const bool coop = share.n > 1;                           // (never with four per CU: see share_of)
#define C2T_HIST_KERNEL(TOPM)                                                                                   \
  (four_per_cu ? (const void*)k_logits_hist<HP_NT, TOPM, 8, 1, false>                                            \
               : coop ? (const void*)k_logits_hist<HP_NT, TOPM, 6, HP_REPL_ALONE, true> : (const void*)k_logits_hist<HP_NT, TOPM, 6, HP_REPL_ALONE, false>)
    const void* fn = topm ? C2T_HIST_KERNEL(true) : C2T_HIST_KERNEL(false);
#undef C2T_HIST_KERNEL
    size_t& raised = x->lds_raised[four_per_cu ? 1 : coop ? 2 : 0];
    if (lds > raised) {                                     // beyond the 48 KB a kernel may use without asking
      hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
      if (e != hipSuccess) return e;
      raised = lds;
    }
#define C2T_LAUNCH_HIST(TOPM, WPS, REPL, COOP)                                                                                      \
  hipExtLaunchKernelGGL((k_logits_hist<HP_NT, TOPM, WPS, REPL, COOP>), dim3(grid), dim3(HP_NT), lds, s, ev0, ev1, 0, logits, stride, \
                        c.vocab, cps, (const double*)x->tab_e, (const float*)x->st.cls, x->st, sp)
#define C2T_LAUNCH_HIST_BUILD(TOPM)                                      \
  do {                                                                   \
    if (four_per_cu) C2T_LAUNCH_HIST(TOPM, 8, 1, false);                 \
    else if (coop) C2T_LAUNCH_HIST(TOPM, 6, HP_REPL_ALONE, true);        \
    else C2T_LAUNCH_HIST(TOPM, 6, HP_REPL_ALONE, false);                 \
  } while (0)
    if (topm) C2T_LAUNCH_HIST_BUILD(true); else C2T_LAUNCH_HIST_BUILD(false);
#undef C2T_LAUNCH_HIST_BUILD
#undef C2T_LAUNCH_HIST
  } else {
    const size_t lds = std::max(std::max(std::max(map_lds, list_lds), score_lds), (size_t)16 * 1024);
    sp.lds_bytes = (int)lds;
    sp.w_lds_off = -1;
    hipExtLaunchKernelGGL((k_logits_generic<0, NT_F32>), dim3(grid), dim3(NT_F32), lds, s, ev0, ev1, 0, logits, stride,
                          c.vocab, cps, (const float*)x->st.cls, x->st, sp);
  }
  return hipGetLastError();
}

}  // namespace

extern "C" {

int c2t_workspace_bytes(const c2t_config* cfg, size_t* out) {
  if (!out) return C2T_ERR_INVALID_ARG;
  int rc = check_config(cfg);
  if (rc) return rc;
  *out = make_layout(*cfg).total;
  return C2T_OK;
}

int c2t_create(const c2t_config* cfg, void* ws, size_t bytes, c2t_ctx** out) {
  if (!out) return C2T_ERR_INVALID_ARG;
  *out = nullptr;
  int rc = check_config(cfg);
  if (rc) return rc;
  Layout L = make_layout(*cfg);
  if (!ws || ((uintptr_t)ws % ALIGN) != 0 || bytes < L.total) return C2T_ERR_WORKSPACE;
  c2t_ctx* x = new (std::nothrow) c2t_ctx();
  if (!x) return C2T_ERR_NOMEM;
  x->cfg = *cfg; x->lay = L; x->ws = (char*)ws;
  char* w = x->ws;
  TreeState& s = x->st;
  s.cls = (float*)(w + L.cls);
  s.n_nodes = (int32_t*)(w + L.n_nodes); s.nf[0] = (int32_t*)(w + L.nf0); s.nf[1] = (int32_t*)(w + L.nf1);
  s.tickets = (int32_t*)(w + L.tickets); s.row_tickets = (int32_t*)(w + L.row_tickets);
  s.row_info = (uint32_t*)(w + L.row_info);
  s.status = (uint32_t*)(w + L.status); s.n_cand = (int32_t*)(w + L.n_cand);
  s.layer_rows = (int32_t*)(w + L.layer_rows);
  s.fr_tok = (int32_t*)(w + L.fr_tok); s.fr_pslot = (int32_t*)(w + L.fr_pslot);
  s.fr_node = (int32_t*)(w + L.fr_node); s.fr_P = (float*)(w + L.fr_P);
  s.fr_hidx = nullptr; s.fr_s = nullptr; s.h_tok = s.h_par = s.h_ncand = s.h_pos = nullptr; s.h_P = s.h_H = s.h_z = s.h_s = nullptr;
  if (cfg->rerank) {
    s.fr_hidx = (int32_t*)(w + L.fr_hidx); s.fr_s = (float*)(w + L.fr_s);
    s.h_tok = (int32_t*)(w + L.h_tok); s.h_par = (int32_t*)(w + L.h_par); s.h_P = (float*)(w + L.h_P);
    s.h_H = (float*)(w + L.h_H); s.h_z = (float*)(w + L.h_z); s.h_s = (float*)(w + L.h_s);
    s.h_ncand = (int32_t*)(w + L.h_ncand); s.h_pos = (int32_t*)(w + L.h_pos);
  }
  s.t_tok = (int32_t*)(w + L.t_tok); s.t_parent = (int32_t*)(w + L.t_parent); s.t_depth = (int32_t*)(w + L.t_depth);
  s.t_P = (float*)(w + L.t_P); s.t_H = (float*)(w + L.t_H); s.t_z = (float*)(w + L.t_z);
  s.c_tok = (int32_t*)(w + L.c_tok); s.c_p = (float*)(w + L.c_p); s.c_P = (float*)(w + L.c_P);
  s.c_H = (float*)(w + L.c_H); s.c_z = (float*)(w + L.c_z); s.c_kept = (int32_t*)(w + L.c_kept);
  x->part = (RowPartial*)(w + L.part);
  x->part_topv = (float*)(w + L.part_topv);
  x->part_topi = (int32_t*)(w + L.part_topi);
  x->tab_e = (double*)(w + L.tab_e);
  x->z_beta = cfg->beta <= 0.0f ? -INFINITY : (float)std::log((double)cfg->beta / (1.0 - (double)cfg->beta));
  x->layer = -1; x->have_cls = false; x->finalized = false; x->ev_used = 0; x->sample_every = 1; x->sample_first = 0; x->phase_no = -1;
  x->lds_raised[0] = x->lds_raised[1] = x->lds_raised[2] = 48 * 1024;
  {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
      n = 256;                                                // no device (host-only checks of the interface): MI355X's count
    x->n_cus = n;
  }
  if (cfg->rerank) (void)scratch_on_current_device(nullptr);    // set-up of the allocation-free reranking; asked again at its first call if there is no device yet
  x->ns_first = default_split(*cfg, L, cfg->batch);
  x->ns_other = default_split(*cfg, L, (int64_t)cfg->batch * cfg->max_frontier);
  x->share_first = x->share_other = true;
  *out = x;
  return C2T_OK;
}

void c2t_destroy(c2t_ctx* x) {
  if (!x) return;
  for (hipEvent_t e : x->ev) (void)hipEventDestroy(e);
  delete x;
}

int c2t_set_classifier(c2t_ctx* x, const float* W1, const float* b1, const float* w2, float b2, void* stream) {
  if (!x || !W1 || !b1 || !w2) return C2T_ERR_INVALID_ARG;
  const int h = x->cfg.hidden, total = 5 * h + 1;
  // The parameters go to the device as kernel arguments, ClsChunk::N floats a launch: the runtime
  // copies arguments when the launch is enqueued, so nothing refers to host memory afterwards.
  for (int off = 0; off < total; off += ClsChunk::N) {
    ClsChunk c;
    const int n = std::min(ClsChunk::N, total - off);
    for (int i = 0; i < n; ++i) {
      const int j = off + i;                                  // layout: W1 [3h] | b1 [h] | w2 [h] | b2
      c.v[i] = j < 3 * h ? W1[j] : j < 4 * h ? b1[j - 3 * h] : j < 5 * h ? w2[j - 4 * h] : b2;
    }
    hipLaunchKernelGGL(k_set_classifier, dim3(1), dim3(ClsChunk::N), 0, (hipStream_t)stream, x->st.cls, off, n, c);
    if (hipGetLastError() != hipSuccess) return C2T_ERR_HIP;
  }
  // table of e^v for the bf16 value histogram (device-side fp64 exp), once per context
  if (!x->have_cls && x->cfg.logits_dtype == C2T_BF16) {
    hipLaunchKernelGGL(k_init_exp_table, dim3((HP_TAB_DOUBLES + 255) / 256), dim3(256), 0, (hipStream_t)stream, x->tab_e);
    if (hipGetLastError() != hipSuccess) return C2T_ERR_HIP;
  }
  x->have_cls = true;
  return C2T_OK;
}

int c2t_reset(c2t_ctx* x, void* stream) {
  if (!x) return C2T_ERR_INVALID_ARG;
  if (!x->have_cls) return C2T_ERR_STATE;
  const int n = std::max(x->cfg.batch, x->cfg.max_depth + 1);
  hipLaunchKernelGGL(k_reset, dim3((n + 255) / 256), dim3(256), 0, (hipStream_t)stream, x->st, x->cfg.batch,
                     x->cfg.max_frontier, x->cfg.max_depth);
  if (hipGetLastError() != hipSuccess) return C2T_ERR_HIP;
  x->layer = 0; x->finalized = false; x->phase_no += 1;
  return C2T_OK;
}

int c2t_expand_layer(c2t_ctx* x, const void* logits, int64_t row_stride_elems, void* stream) {
  if (!x || !logits) return C2T_ERR_INVALID_ARG;
  const c2t_config& c = x->cfg;
  if (x->layer < 0 || x->layer >= c.max_depth || x->finalized) return C2T_ERR_STATE;
  if (row_stride_elems < c.vocab) return C2T_ERR_INVALID_ARG;
  const int esz = c.logits_dtype == C2T_BF16 ? 2 : 4;
  if (((uintptr_t)logits % 16) != 0 || (row_stride_elems * esz) % 16 != 0) return C2T_ERR_UNSUPPORTED;
  hipStream_t s = (hipStream_t)stream;
  const bool first = x->layer == 0;
  const int rows_per_seq = first ? 1 : c.max_frontier;
  const int nsplit = first ? x->ns_first : x->ns_other;
  const bool timed = !x->ev.empty() && x->ev_used + 2 <= (int)x->ev.size() && x->phase_no % x->sample_every == x->sample_first;
  hipError_t e = launch_logits(x, logits, row_stride_elems, rows_per_seq, nsplit, first ? x->share_first : x->share_other, s,
                               timed ? x->ev[x->ev_used] : nullptr, timed ? x->ev[x->ev_used + 1] : nullptr);
  if (e != hipSuccess) return C2T_ERR_HIP;
  if (timed) x->ev_used += 2;
  x->layer += 1;
  return C2T_OK;
}

int c2t_get_frontier(c2t_ctx* x, const int32_t** tokens, const int32_t** parent_slot, const int32_t** n_frontier) {
  if (!x) return C2T_ERR_INVALID_ARG;
  if (tokens) *tokens = x->st.fr_tok;
  if (parent_slot) *parent_slot = x->st.fr_pslot;
  if (n_frontier) *n_frontier = x->st.nf[(x->layer < 0 ? 0 : x->layer) & 1];
  return C2T_OK;
}

int c2t_get_candidates(c2t_ctx* x, const int32_t** n_cand, const int32_t** token, const float** p, const float** P,
                       const float** H, const float** z, const int32_t** kept) {
  if (!x) return C2T_ERR_INVALID_ARG;
  if (n_cand) *n_cand = x->st.n_cand;
  if (token) *token = x->st.c_tok;
  if (p) *p = x->st.c_p;
  if (P) *P = x->st.c_P;
  if (H) *H = x->st.c_H;
  if (z) *z = x->st.c_z;
  if (kept) *kept = x->st.c_kept;
  return C2T_OK;
}

int c2t_finalize_tree(c2t_ctx* x, const c2t_tree_out* o, void* stream) {
  if (!x || !o) return C2T_ERR_INVALID_ARG;
  if (!o->tokens || !o->parent || !o->position || !o->conf || !o->joint_prob || !o->entropy || !o->n_nodes ||
      !o->mask || !o->status)
    return C2T_ERR_INVALID_ARG;
  if (x->layer < 0) return C2T_ERR_STATE;
  TreeOut t{o->tokens, o->parent, o->position, o->conf, o->joint_prob, o->entropy, o->n_nodes, o->mask, o->status};
  hipLaunchKernelGGL(k_finalize, dim3(x->cfg.batch), dim3(256), 0, (hipStream_t)stream, x->st, t, x->cfg.budget);
  if (hipGetLastError() != hipSuccess) return C2T_ERR_HIP;
  x->finalized = true;
  return C2T_OK;
}

int c2t_finalize_tree_reranked(c2t_ctx* x, const c2t_tree_out* o, int32_t n_out, void* stream) {
  if (!x || !o) return C2T_ERR_INVALID_ARG;
  if (!o->tokens || !o->parent || !o->position || !o->conf || !o->joint_prob || !o->entropy || !o->n_nodes ||
      !o->mask || !o->status)
    return C2T_ERR_INVALID_ARG;
  if (n_out <= 0) return C2T_ERR_INVALID_ARG;
  if (n_out > C2T_MAX_BUDGET) return C2T_ERR_UNSUPPORTED;
  if (!x->cfg.rerank || x->layer < 0) return C2T_ERR_STATE;
  TreeOut t{o->tokens, o->parent, o->position, o->conf, o->joint_prob, o->entropy, o->n_nodes, o->mask, o->status};
  hipLaunchKernelGGL(k_finalize_rerank, dim3(x->cfg.batch), dim3(RR_NT), 0, (hipStream_t)stream, x->st, t, n_out,
                     x->cfg.max_depth, x->cfg.max_frontier * x->cfg.top_k);
  if (hipGetLastError() != hipSuccess) return C2T_ERR_HIP;
  x->finalized = true;
  return C2T_OK;
}

int c2t_finalize_tree_reranked_static(c2t_ctx* x, const c2t_tree_out* o, int32_t n_out, void* stream) {
  if (!x || !o) return C2T_ERR_INVALID_ARG;
  if (!o->tokens || !o->parent || !o->position || !o->conf || !o->joint_prob || !o->entropy || !o->n_nodes ||
      !o->mask || !o->status)
    return C2T_ERR_INVALID_ARG;
  if (n_out <= 0) return C2T_ERR_INVALID_ARG;
  if (n_out > C2T_MAX_BUDGET) return C2T_ERR_UNSUPPORTED;
  if (!x->cfg.rerank || x->layer < 0) return C2T_ERR_STATE;
  const int64_t entries = (int64_t)x->cfg.batch * x->cfg.max_depth * x->cfg.max_frontier * x->cfg.top_k;
  if (entries > C2T_STATIC_RERANK_ENTRIES) return C2T_ERR_UNSUPPORTED;    // the static array is that large and no larger
  hipError_t e = hipSuccess;
  int32_t* pos = scratch_on_current_device(&e);
  if (!pos) return C2T_ERR_HIP;
  TreeState st = x->st;
  st.h_pos = pos;                                             // every entry the kernel reads it has written in the same launch: nothing to clear
  TreeOut t{o->tokens, o->parent, o->position, o->conf, o->joint_prob, o->entropy, o->n_nodes, o->mask, o->status};
  hipLaunchKernelGGL(k_finalize_rerank, dim3(x->cfg.batch), dim3(RR_NT), 0, (hipStream_t)stream, st, t, n_out,
                     x->cfg.max_depth, x->cfg.max_frontier * x->cfg.top_k);
  if (hipGetLastError() != hipSuccess) return C2T_ERR_HIP;
  x->finalized = true;
  return C2T_OK;
}

int c2t_get_layer_rows(c2t_ctx* x, const int32_t** layer_rows) {
  if (!x || !layer_rows) return C2T_ERR_INVALID_ARG;
  *layer_rows = x->st.layer_rows;
  return C2T_OK;
}

int c2t_set_row_splits(c2t_ctx* x, int32_t first_layer, int32_t other_layers) {
  if (!x || first_layer < 0 || other_layers < 0) return C2T_ERR_INVALID_ARG;
  const c2t_config& c = x->cfg;
  const int nmin = min_splits(c);
  const int nmax_size = std::max(1, chunks_of(c));
  int nf = first_layer ? first_layer : default_split(c, x->lay, c.batch);
  int no = other_layers ? other_layers : default_split(c, x->lay, (int64_t)c.batch * c.max_frontier);
  if (nf < nmin || no < nmin || nf > nmax_size || no > nmax_size) return C2T_ERR_UNSUPPORTED;
  if ((int64_t)c.batch * nf > x->lay.partial_slots || (int64_t)c.batch * c.max_frontier * no > x->lay.partial_slots)
    return C2T_ERR_WORKSPACE;
  x->ns_first = nf; x->ns_other = no;
  x->share_first = first_layer == 0; x->share_other = other_layers == 0;   // a split count the caller has set is taken literally
  return C2T_OK;
}

int c2t_get_row_workgroups(const c2t_ctx* x, int32_t* first_layer, int32_t* other_layers) {
  if (!x) return C2T_ERR_INVALID_ARG;
  const c2t_config& c = x->cfg;
  auto per_row = [&](int nsplit, bool may_share, int64_t rows) {
    const Share sh = (may_share && nsplit == 1) ? share_of(c, x->lay, x->n_cus, rows) : Share{1, 0};
    return sh.n > 1 ? sh.n : nsplit;
  };
  if (first_layer) *first_layer = per_row(x->ns_first, x->share_first, c.batch);
  if (other_layers) *other_layers = per_row(x->ns_other, x->share_other, (int64_t)c.batch * c.max_frontier);
  return C2T_OK;
}

int c2t_profile_enable(c2t_ctx* x, int32_t capacity) {
  if (!x || capacity < 0) return C2T_ERR_INVALID_ARG;
  for (hipEvent_t e : x->ev) (void)hipEventDestroy(e);
  x->ev.clear(); x->ev_used = 0; x->phase_no = -1;           // the next draft phase is phase 0
  for (int i = 0; i < 2 * capacity; ++i) {
    hipEvent_t e;
    if (hipEventCreate(&e) != hipSuccess) return C2T_ERR_HIP;
    x->ev.push_back(e);
  }
  return C2T_OK;
}

int c2t_profile_sample(c2t_ctx* x, int32_t every, int32_t first) {
  if (!x || every < 1 || first < 0 || first >= every) return C2T_ERR_INVALID_ARG;
  x->sample_every = every; x->sample_first = first;
  return C2T_OK;
}

int c2t_profile_read(c2t_ctx* x, float* ms, int32_t* n) {
  if (!x || !ms || !n) return C2T_ERR_INVALID_ARG;
  const int have = x->ev_used / 2;
  const int cnt = std::min(have, (int)*n);
  for (int i = 0; i < cnt; ++i)
    if (hipEventElapsedTime(&ms[i], x->ev[2 * i], x->ev[2 * i + 1]) != hipSuccess) return C2T_ERR_HIP;
  *n = cnt;
  x->ev_used = 0;
  return C2T_OK;
}

int c2t_stream_read(const void* p, size_t bytes, uint32_t* out, void* stream) {
  if (!p || !out || bytes % 16 != 0 || ((uintptr_t)p % 16) != 0) return C2T_ERR_INVALID_ARG;
  hipLaunchKernelGGL(k_stream_read, dim3(256 * 8), dim3(1024), 0, (hipStream_t)stream, (const uint4*)p, bytes / 16, out);
  return hipGetLastError() == hipSuccess ? C2T_OK : C2T_ERR_HIP;
}

int c2t_stream_read_rows(const void* p, int32_t rows, size_t row_bytes, size_t row_stride_bytes, uint32_t* out, void* stream) {
  if (!p || !out || rows <= 0 || row_bytes == 0 || row_bytes % 16 != 0 || row_stride_bytes % 16 != 0 ||
      row_stride_bytes < row_bytes || ((uintptr_t)p % 16) != 0 || row_bytes / 16 > (size_t)INT32_MAX)
    return C2T_ERR_INVALID_ARG;
  hipLaunchKernelGGL(k_stream_read_rows, dim3((unsigned)rows), dim3(512), 0, (hipStream_t)stream, (const char*)p,
                     (int64_t)row_stride_bytes, (int)(row_bytes / 16), out);
  return hipGetLastError() == hipSuccess ? C2T_OK : C2T_ERR_HIP;
}

int c2t_phase_times_read(uint64_t* out, int32_t n_workgroups) {
#ifdef C2T_PHASE_TIMES
  if (!out || n_workgroups <= 0 || n_workgroups > PT_WORKGROUPS) return C2T_ERR_INVALID_ARG;
  if (hipMemcpyFromSymbol(out, HIP_SYMBOL(c2t::c2t_phase_times), (size_t)n_workgroups * PT_SLOTS * 8) != hipSuccess) return C2T_ERR_HIP;
  return C2T_OK;
#else
  (void)out; (void)n_workgroups;
  return C2T_ERR_UNSUPPORTED;
#endif
}

const char* c2t_strerror(int code) {
  switch (code) {
    case C2T_OK: return "ok";
    case C2T_ERR_INVALID_ARG: return "invalid argument";
    case C2T_ERR_UNSUPPORTED: return "unsupported size, alignment or option";
    case C2T_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case C2T_ERR_STATE: return "call out of order or classifier not set";
    case C2T_ERR_HIP: return "HIP runtime call failed";
    case C2T_ERR_NOMEM: return "out of host memory";
    default: return "unknown error";
  }
}

}  // extern "C"
