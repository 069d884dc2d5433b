// C ABI of libdyn: argument checks, host-side preparation of the candidate list, and the
// launch sequences.  All arithmetic of the method runs in the kernels; the only numbers
// computed here are the frequency bracket and weight of each candidate (one IEEE
// division per candidate, independent of the trace).
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <new>
#include <numeric>

#include "dyn_ticks.h"
#include "dyn_mixed.h"
#include "dyn_path.h"
#include "dyn_account.h"
#include "dyn_hier.h"

namespace {

thread_local char g_err[512] = "";

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

bool hip_ok(hipError_t e, const char* what) {
  if (e == hipSuccess) return true;
  dyn_set_error("%s: %s", what, hipGetErrorString(e));
  return false;
}

__global__ void init_word_header_kernel(WsHeader* h, uint32_t order_word) {   // header regions are 256 bytes
  h->status = 0u;
  h->kind = DYN_WS_KIND_WORD;
  h->cells = 0;
  ((uint32_t*)h)[DYN_WS_HEADER_ORDER_WORD] = order_word;   // ingestion: "not in window order" flag
  ((uint32_t*)h)[DYN_WS_HEADER_BARRIER_WORD] = 0u;
}

// Lengths of windows and ticks, capacities and grid spacings are kept inside this range so that the
// reciprocal-based division of the kernels never meets a subnormal or infinite intermediate.
constexpr double kMinScale = 1e-100, kMaxScale = 1e100;
bool in_scale(double x) { return x >= kMinScale && x <= kMaxScale; }   // false for NaN

bool strictly_increasing(const double* g, int n) {
  for (int i = 0; i < n; ++i)
    if (!isfinite(g[i])) return false;
  for (int i = 1; i < n; ++i)
    if (!(g[i] > g[i - 1])) return false;
  return true;
}

template <typename T>
hipError_t dev_alloc(T** p, size_t count) {
  return hipMalloc((void**)p, std::max<size_t>(count, 1) * sizeof(T));
}

void free_profile_device(dyn_profile* p) {
  void* ptrs[] = {p->d_tab, p->d_ml, p->d_pw0, p->d_pfspan, p->d_theta, p->d_gridpack, p->d_jstart, p->d_tstart, p->d_thr, p->d_cfg,
                  p->d_tile_rows, p->d_slo_ttft, p->d_slo_tbt, p->d_budget, p->d_path_layout, p->d_path_order,
                  p->d_path_seg, p->d_path_trans, p->d_hier_trans, p->d_lay_n, p->d_lay_tp, p->d_tp, p->d_ident};
  for (void* q : ptrs)
    if (q) (void)hipFree(q);
}

int check_device(const dyn_profile* p) {
  int dev = -1;
  if (!hip_ok(hipGetDevice(&dev), "hipGetDevice")) return DYN_E_DEVICE;
  if (dev != p->device) {
    dyn_set_error("profile lives on device %d but device %d is current", p->device, dev);
    return DYN_E_DEVICE;
  }
  return DYN_OK;
}

// Checks the candidate list and, if it differs from what the handle already holds on the
// device, rebuilds the device table: frequency bracket/weight per candidate, the tiling
// of the configuration axis and the table rows each tile stages in LDS.
int prepare_configs(dyn_profile* p, const dyn_config* cfg, int32_t K, hipStream_t s) {
  if (!cfg) { dyn_set_error("cfg is NULL"); return DYN_E_NULL; }
  if (K < 1 || K > DYN_MAX_CONFIGS) { dyn_set_error("K=%d outside [1, %d]", K, DYN_MAX_CONFIGS); return DYN_E_SHAPE; }
  for (int k = 0; k < K; ++k) {
    if (cfg[k].n_inst < 1) { dyn_set_error("cfg[%d].n_inst=%d < 1", k, cfg[k].n_inst); return DYN_E_RANGE; }
    if (cfg[k].tp_index < 0 || cfg[k].tp_index >= p->n_tp) {
      dyn_set_error("cfg[%d].tp_index=%d outside [0, %d)", k, cfg[k].tp_index, p->n_tp);
      return DYN_E_RANGE;
    }
    if (!(cfg[k].f_mhz >= p->fg.front()) || !(cfg[k].f_mhz <= p->fg.back())) {
      dyn_set_error("cfg[%d].f_mhz=%g outside the profiled range [%g, %g]", k, cfg[k].f_mhz, p->fg.front(),
                    p->fg.back());
      return DYN_E_RANGE;
    }
  }
  if ((int32_t)p->cfg_host.size() == K) {
    bool same = true;
    for (int k = 0; k < K && same; ++k)
      same = cfg[k].n_inst == p->cfg_host[k].n_inst && cfg[k].tp_index == p->cfg_host[k].tp_index &&
             cfg[k].f_mhz == p->cfg_host[k].f_mhz;
    if (same) return DYN_OK;
  }

  std::vector<DevCfg> dc(K);
  const int n_f = p->n_f;
  for (int k = 0; k < K; ++k) {
    int fi = 0;
    double u = 0.0;
    if (n_f > 1) {
      for (int q = 0; q < n_f; ++q)
        if (p->fg[q] <= cfg[k].f_mhz) fi = q;
      if (fi > n_f - 2) fi = n_f - 2;
      u = (cfg[k].f_mhz - p->fg[fi]) / (p->fg[fi + 1] - p->fg[fi]);
      if (u == 1.0) { fi += 1; u = 0.0; }  // weight 1 on the upper row is that row itself
    }
    DevCfg& d = dc[k];
    d.u = u;
    d.nd = (double)cfg[k].n_inst;
    d.n = cfg[k].n_inst;
    const int64_t gpus = (int64_t)cfg[k].n_inst * p->tp[cfg[k].tp_index];
    d.gpus = gpus > 0x7FFFFFFF ? 0x7FFFFFFF : (int32_t)gpus;
    d.row_lo = cfg[k].tp_index * n_f + fi;
    d.row_hi = u != 0.0 ? d.row_lo + 1 : d.row_lo;
    d.slot_lo = d.slot_hi = 0;
  }
  // tiling of the configuration axis: least padding, then the widest tile
  const int cand[4] = {256, 192, 128, 64};
  int order[4] = {0, 1, 2, 3};
  std::stable_sort(order, order + 4, [&](int a, int b) {
    const int wa = (K + cand[a] - 1) / cand[a] * cand[a] - K, wb = (K + cand[b] - 1) / cand[b] * cand[b] - K;
    return wa < wb;
  });
  const size_t lds_tail = dyn_space_lds_tail(p->n_rho, p->n_bucket, DYN_MAX_WIN_PER_BLOCK);
  std::vector<int32_t> rows;
  int tile = cand[order[0]], n_tile = (K + tile - 1) / tile, n_slot = 0;
  bool fits = false;
  for (int oi = 0; oi < 4 && !fits; ++oi) {
    const int t = cand[order[oi]], nt = (K + t - 1) / t;
    std::vector<std::vector<int32_t>> per_tile(nt);
    int ns = 0;
    for (int k = 0; k < K; ++k) {
      std::vector<int32_t>& v = per_tile[k / t];
      for (int32_t r : {dc[k].row_lo, dc[k].row_hi})
        if (std::find(v.begin(), v.end(), r) == v.end()) v.push_back(r);
      ns = std::max<int>(ns, (int)v.size());
    }
    if ((size_t)ns * 3 * p->n_rho * sizeof(double) + lds_tail <= DYN_LDS_BUDGET) {
      fits = true;
      tile = t; n_tile = nt; n_slot = ns;
      rows.assign((size_t)nt * ns, -1);
      for (int q = 0; q < nt; ++q)
        for (size_t i = 0; i < per_tile[q].size(); ++i) rows[(size_t)q * ns + i] = per_tile[q][i];
      for (int k = 0; k < K; ++k) {
        const std::vector<int32_t>& v = per_tile[k / t];
        dc[k].slot_lo = (int32_t)(std::find(v.begin(), v.end(), dc[k].row_lo) - v.begin());
        dc[k].slot_hi = (int32_t)(std::find(v.begin(), v.end(), dc[k].row_hi) - v.begin());
      }
    }
  }
  if (!fits) {  // rows do not fit LDS at any tile width: read the tables from global memory
    tile = cand[order[0]]; n_tile = (K + tile - 1) / tile; n_slot = 0;
    if (lds_tail > DYN_LDS_BUDGET) {
      dyn_set_error("load grid of %d points does not fit in LDS", p->n_rho);
      return DYN_E_SHAPE;
    }
  }
  // the previous table may still be read by work enqueued on this stream
  if (!hip_ok(hipStreamSynchronize(s), "hipStreamSynchronize")) return DYN_E_DEVICE;
  p->cfg_host.clear();
  if (!hip_ok(hipMemcpy(p->d_cfg, dc.data(), (size_t)K * sizeof(DevCfg), hipMemcpyHostToDevice), "copy configs"))
    return DYN_E_DEVICE;
  if (!rows.empty() &&
      !hip_ok(hipMemcpy(p->d_tile_rows, rows.data(), rows.size() * sizeof(int32_t), hipMemcpyHostToDevice),
              "copy tile rows"))
    return DYN_E_DEVICE;
  p->tile = tile; p->n_tile = n_tile; p->n_slot = n_slot;
  p->wpb = 0; p->wpb_windows = 0; p->wpb_tuned = false;
  p->any_two_rows = false;
  for (int k = 0; k < K; ++k) p->any_two_rows = p->any_two_rows || dc[k].u != 0.0;
  p->cfg_host.assign(cfg, cfg + K);
  return DYN_OK;
}

// Uploads `n` values to a device array of the handle unless the handle already holds the same values there.  A
// changed table is uploaded after waiting for the stream: work enqueued on it may still read the old one.
template <typename T>
int cache_upload(std::vector<T>& host, T* dev, const T* src, size_t n, hipStream_t s, const char* what) {
  if (host.size() == n && (n == 0 || memcmp(host.data(), src, n * sizeof(T)) == 0)) return DYN_OK;
  if (!hip_ok(hipStreamSynchronize(s), "hipStreamSynchronize")) return DYN_E_DEVICE;
  host.clear();
  if (n && !hip_ok(hipMemcpy(dev, src, n * sizeof(T), hipMemcpyHostToDevice), what)) return DYN_E_DEVICE;
  host.assign(src, src + n);
  return DYN_OK;
}

int prepare_objective(dyn_profile* p, const dyn_objective* o, hipStream_t s) {
  if (!o) { dyn_set_error("objective is NULL"); return DYN_E_NULL; }
  if (!o->slo_ttft_ms || !o->slo_tbt_ms) { dyn_set_error("SLO arrays are NULL"); return DYN_E_NULL; }
  if (o->pct_num < 1 || o->pct_den < 1 || o->pct_num > o->pct_den) {
    dyn_set_error("percentile %d/%d outside (0, 1]", o->pct_num, o->pct_den);
    return DYN_E_RANGE;
  }
  if (!isfinite(o->idle_cost_weight)) { dyn_set_error("idle_cost_weight is not finite"); return DYN_E_NOTFINITE; }
  if (o->idle_cost_weight < 0.0) { dyn_set_error("idle_cost_weight must be >= 0"); return DYN_E_RANGE; }
  const int G = p->G;
  for (int g = 0; g < G; ++g) {
    if (isnan(o->slo_ttft_ms[g]) || isnan(o->slo_tbt_ms[g])) { dyn_set_error("SLO of class %d is NaN", g); return DYN_E_NOTFINITE; }
    if (o->gpu_budget && o->gpu_budget[g] < 0) { dyn_set_error("gpu_budget[%d] < 0", g); return DYN_E_RANGE; }
  }
  std::vector<int32_t> bud(G, 0);
  if (o->gpu_budget) bud.assign(o->gpu_budget, o->gpu_budget + G);
  if (p->obj_valid && memcmp(p->slo_ttft_host.data(), o->slo_ttft_ms, G * sizeof(double)) == 0 &&
      memcmp(p->slo_tbt_host.data(), o->slo_tbt_ms, G * sizeof(double)) == 0 && bud == p->budget_host)
    return DYN_OK;
  if (!hip_ok(hipStreamSynchronize(s), "hipStreamSynchronize")) return DYN_E_DEVICE;
  p->obj_valid = false;
  if (!hip_ok(hipMemcpy(p->d_slo_ttft, o->slo_ttft_ms, G * sizeof(double), hipMemcpyHostToDevice), "copy SLOs") ||
      !hip_ok(hipMemcpy(p->d_slo_tbt, o->slo_tbt_ms, G * sizeof(double), hipMemcpyHostToDevice), "copy SLOs") ||
      !hip_ok(hipMemcpy(p->d_budget, bud.data(), G * sizeof(int32_t), hipMemcpyHostToDevice), "copy budgets"))
    return DYN_E_DEVICE;
  p->slo_ttft_host.assign(o->slo_ttft_ms, o->slo_ttft_ms + G);
  p->slo_tbt_host.assign(o->slo_tbt_ms, o->slo_tbt_ms + G);
  p->budget_host = bud;
  p->obj_valid = true;
  return DYN_OK;
}

struct IngestWs {
  size_t status, in_edge, out_edge, key_a, key_b, in_tmp, out_tmp, hist, win_off, total;
};
IngestWs ingest_ws_layout(int64_t n_req, int32_t n_model, int32_t n_in_bin, int32_t n_out_bin, int32_t n_window) {
  IngestWs w;
  size_t off = 0;
  w.status = off; off += 256;
  w.in_edge = off; off += align256((size_t)n_model * std::max(n_in_bin - 1, 1) * 4);
  w.out_edge = off; off += align256((size_t)n_model * std::max(n_out_bin - 1, 1) * 4);
  const size_t n = (size_t)std::max<int64_t>(n_req, 1);
  w.key_a = off; off += align256(n * 4);
  w.key_b = off; off += align256(n * 4);
  w.in_tmp = off; off += align256(n * 4);
  w.out_tmp = off; off += align256(n * 4);
  const size_t nb = (size_t)dyn_ingest_blocks(n_req);
  w.hist = off; off += align256(((size_t)DYN_INGEST_MAX_BINS * nb + (DYN_INGEST_MAX_BINS * nb) / 4096 + 2) * 4);
  w.win_off = off; off += align256(((size_t)std::max(n_window, 1) + 1) * sizeof(int64_t));
  w.total = off;
  return w;
}

}  // namespace

// ---- fixed workspace of dyn_eval_select_static ---------------------------------------------
// One array per GPU the library runs on, held until the process ends.  In host code the array's
// name is only a handle for hipGetSymbolAddress: kernels and copies get the address that call
// returns for the current device, never the name.
static __device__ __align__(256) unsigned char scratch[DYN_STATIC_WORKSPACE_BYTES];

namespace {
constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {};   // device address of `scratch` on each device, once resolved

// Address of the current device's copy of `scratch` (resolved once per device, with that device current).
int scratch_address(void** out) {
  int dev = -1;
  if (!hip_ok(hipGetDevice(&dev), "hipGetDevice")) return DYN_E_DEVICE;
  if (dev < 0 || dev >= kMaxDevices) { dyn_set_error("device %d: the library keeps a fixed workspace on devices 0..%d only", dev, kMaxDevices - 1); return DYN_E_DEVICE; }
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    if (!hip_ok(hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(scratch)), "hipGetSymbolAddress(scratch)")) return DYN_E_DEVICE;
    if (!ptr || ((uintptr_t)ptr & 255)) { dyn_set_error("the fixed workspace has no usable device address"); return DYN_E_DEVICE; }
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return DYN_OK;
}

// OR of the per-cell status bytes, written (not accumulated) to *status by one block.
__global__ __launch_bounds__(1024) void cell_status_word_kernel(const uint8_t* __restrict__ cstat, int64_t cells,
                                                                uint32_t* __restrict__ status) {
  __shared__ uint32_t s_or;
  if (threadIdx.x == 0) s_or = 0u;
  __syncthreads();
  uint32_t v = 0;
  for (int64_t i = threadIdx.x; i < cells; i += blockDim.x) v |= cstat[i];
  if (v) atomicOr(&s_or, v);
  __syncthreads();
  if (threadIdx.x == 0) *status = s_or;
}
}  // namespace

// ---- optional kernel timing ---------------------------------------------------------------
namespace {
struct TimerPool {
  std::vector<hipEvent_t> start, stop;
  int used = 0;
};
TimerPool g_timers[DYN_K_COUNT];
bool g_timing = false;
}  // namespace

DynTimed::DynTimed(int kernel, hipStream_t s) : kernel_(kernel), s_(s), slot_(-1) {
  if (!g_timing) return;
  TimerPool& t = g_timers[kernel];
  if (t.used >= (int)t.start.size()) return;
  slot_ = t.used++;
  (void)hipEventRecord(t.start[slot_], s_);
}
DynTimed::~DynTimed() {
  if (slot_ >= 0) (void)hipEventRecord(g_timers[kernel_].stop[slot_], s_);
}

void dyn_set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}

EvalWs dyn_eval_ws_layout(int64_t cells, int32_t K) {
  EvalWs w;
  size_t off = 0;
  const size_t c = (size_t)std::max<int64_t>(cells, 1);
  w.n_wslot = std::max(K, 1) / DYN_WAVE + 4;   // >= n_tile * tile/64 for every tile width
  w.header = off; off += 256;
  w.tin = off; off += align256(c * 8);
  w.tout = off; off += align256(c * 8);
  w.in_p99 = off; off += align256(c * 4);
  w.rec = off; off += align256(c * sizeof(CellRec));
  w.cstat = off; off += align256(c);
  w.part = off; off += align256(c * (size_t)w.n_wslot * sizeof(SelPart));
  w.total = off;
  return w;
}

TickWs dyn_tick_ws_layout(int64_t n_req, int64_t coarse_cells, int32_t n_tick, int32_t K) {
  TickWs w;
  w.fine = dyn_eval_ws_layout(coarse_cells * n_tick, 1);
  const size_t c = (size_t)std::max<int64_t>(coarse_cells, 1);
  w.n_wslot = std::max(K, 1) / DYN_WAVE + 4;
  size_t off = w.fine.part;
  w.plan = off; off += align256(c * sizeof(TickPlan));
  w.top = off; off += align256((size_t)std::max<int64_t>(n_req, 1) * sizeof(int32_t));
  w.part = off; off += align256(c * (size_t)w.n_wslot * sizeof(SelPart));
  w.counters = off; off += 256;
  w.deep_list = off; off += align256(c * sizeof(uint32_t));
  w.slow_list = off; off += align256(c * sizeof(uint32_t));
  w.list_cells = off; off += align256(c * sizeof(uint32_t));
  w.total = off;
  return w;
}

namespace {

__global__ __launch_bounds__(256) void or_cell_status_kernel(const uint8_t* __restrict__ cstat, int64_t cells,
                                                             uint32_t* __restrict__ status) {
  uint32_t v = 0;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < cells; i += (int64_t)gridDim.x * blockDim.x)
    v |= cstat[i];
  if (v) atomicOr(status, v);
}

// Windows one block of the evaluation kernel walks.  Long runs amortise the staging of the table rows in LDS, but
// the blocks a chip holds at a time then write that many more separate streams; measured on the one-day and the two
// one-week workloads the kernel is fastest when about 16K (block, window) rows are in flight at a time (8, 6 and 8
// windows; 14 to 32 cost 8 to 22 % more), and no run should leave the chip with fewer than ~8192 blocks in all.
// dyn_eval_tune replaces the rule's value by a measured one.
int32_t space_windows_per_block(dyn_profile* p, const SpaceArgs& a_in, int32_t n_window) {
  if (p->wpb > 0 && p->wpb_windows == n_window) return p->wpb;
  const int64_t cell_tiles = (int64_t)n_window * p->G * p->n_tile;
  int64_t wpb = std::max<int64_t>(1, std::min<int64_t>(DYN_MAX_WIN_PER_BLOCK, (cell_tiles + 8191) / 8192));
  SpaceArgs a = a_in;
  a.win_per_block = 8;
  const int per_cu = dyn_space_blocks_per_cu(a);
  if (per_cu > 0 && p->n_cu > 0) wpb = std::min<int64_t>(wpb, std::max<int64_t>(4, 16384 / ((int64_t)per_cu * p->n_cu)));
  p->wpb = (int32_t)wpb; p->wpb_windows = n_window; p->wpb_tuned = false;
  return p->wpb;
}

int check_selection(const dyn_selection* out) {
  if (!out->sel || !out->sel_energy_j || !out->sel_cost || !out->window_energy_j || !out->window_infeasible) {
    dyn_set_error("a selection output array is NULL");
    return DYN_E_NULL;
  }
  return DYN_OK;
}

// dyn_eval_space (sel == nullptr) and dyn_eval_select (sel != nullptr)
int eval_impl(dyn_profile* p, const dyn_trace_view* t, const dyn_config* cfg, int32_t K, const dyn_objective* o,
              const dyn_space* out, const dyn_selection* sel, void* workspace, size_t workspace_bytes,
              void* hip_stream) {
  if (!p || !t || !out || !workspace) { dyn_set_error("profile, trace, out or workspace is NULL"); return DYN_E_NULL; }
  if (!out->energy_j || !out->p99_ttft_ms || !out->p99_tbt_ms || !out->flags) { dyn_set_error("an output array is NULL"); return DYN_E_NULL; }
  int rc;
  if (sel && (rc = check_selection(sel)) != DYN_OK) return rc;
  if (t->n_req < 0 || t->n_req >= ((int64_t)1 << 31) || t->n_window < 1) { dyn_set_error("n_req or n_window out of range"); return DYN_E_SHAPE; }
  if (!t->cell_off || (t->n_req > 0 && (!t->in_tok || !t->out_tok))) { dyn_set_error("a trace array is NULL"); return DYN_E_NULL; }
  if (!in_scale(t->window_s)) { dyn_set_error("window_s must lie in [1e-100, 1e100]"); return DYN_E_RANGE; }
  const int64_t cells = (int64_t)t->n_window * p->G;
  if (cells >= ((int64_t)1 << 30)) { dyn_set_error("n_window * classes must stay below 2^30"); return DYN_E_SHAPE; }
  if ((rc = check_device(p)) != DYN_OK) return rc;
  if (K < 1 || K > DYN_MAX_CONFIGS) { dyn_set_error("K=%d outside [1, %d]", K, DYN_MAX_CONFIGS); return DYN_E_SHAPE; }
  const EvalWs w = dyn_eval_ws_layout(cells, K);
  if (((uintptr_t)workspace & 255) || workspace_bytes < w.total) {
    dyn_set_error("workspace misaligned or too small (%zu < %zu)", workspace_bytes, w.total);
    return DYN_E_WORKSPACE;
  }
  hipStream_t s = (hipStream_t)hip_stream;
  if ((rc = prepare_configs(p, cfg, K, s)) != DYN_OK) return rc;
  if ((rc = prepare_objective(p, o, s)) != DYN_OK) return rc;

  char* base = (char*)workspace;
  if (!hip_ok(dyn_launch_cell_aggregate(t->in_tok, t->out_tok, t->cell_off, t->n_req, cells, t->window_s, o->pct_num,
                                        o->pct_den, (int64_t*)(base + w.tin), (int64_t*)(base + w.tout),
                                        (int32_t*)(base + w.in_p99), (CellRec*)(base + w.rec),
                                        (uint8_t*)(base + w.cstat), (WsHeader*)(base + w.header), s),
              "cell aggregate launch"))
    return DYN_E_DEVICE;

  SpaceArgs a;
  a.tab = p->d_tab; a.ml = p->d_ml; a.gridpack = p->d_gridpack;
  a.jstart = p->d_jstart; a.n_bucket = p->n_bucket; a.bucket_scale = p->bucket_scale; a.one_step = p->one_step;
  a.G = p->G; a.n_tp_f = p->n_tp * p->n_f; a.n_rho = p->n_rho;
  a.cfg = p->d_cfg; a.K = K; a.tile = p->tile; a.n_tile = p->n_tile; a.n_slot = p->n_slot;
  a.tile_rows = p->d_tile_rows;
  a.slo_ttft = p->d_slo_ttft; a.slo_tbt = p->d_slo_tbt; a.budget = p->d_budget;
  a.rec = (const CellRec*)(base + w.rec); a.n_window = t->n_window; a.window_s = t->window_s;
  a.win_per_block = space_windows_per_block(p, a, t->n_window);
  a.energy = out->energy_j; a.p99_ttft = out->p99_ttft_ms; a.p99_tbt = out->p99_tbt_ms; a.flags = out->flags;
  a.pw0 = p->d_pw0; a.idle_w = o->idle_cost_weight;
  a.part = sel ? (SelPart*)(base + w.part) : nullptr; a.n_wslot = w.n_wslot;
  if (!hip_ok(dyn_launch_space(a, s), "space launch")) return DYN_E_DEVICE;
  if (sel) {
    FinishArgs f;
    f.part = a.part; f.n_wslot = w.n_wslot; f.n_used = p->n_tile * (p->tile / DYN_WAVE);
    f.n_window = t->n_window; f.G = p->G;
    f.sel = sel->sel; f.sel_energy = sel->sel_energy_j; f.sel_cost = sel->sel_cost;
    f.win_energy = sel->window_energy_j; f.win_inf = sel->window_infeasible;
    if (!hip_ok(dyn_launch_finish(f, s), "finish launch")) return DYN_E_DEVICE;
  }
  return DYN_OK;
}

}  // namespace

extern "C" {

const char* dyn_last_error(void) { return g_err; }

int dyn_profile_load(const dyn_profile_desc* d, void* hip_stream, dyn_profile** out) {
  if (!d || !out) { dyn_set_error("desc or out is NULL"); return DYN_E_NULL; }
  *out = nullptr;
  if (!d->tp || !d->f_mhz || !d->rho || !d->prefill_ms_per_tok || !d->tbt_ms || !d->power_w || !d->max_load_tps) {
    dyn_set_error("a profile array is NULL");
    return DYN_E_NULL;
  }
  if (d->n_class < 1 || d->n_tp < 1 || d->n_f < 1 || d->n_rho < 2) {
    dyn_set_error("profile shape G=%d n_tp=%d n_f=%d n_rho=%d is invalid", d->n_class, d->n_tp, d->n_f, d->n_rho);
    return DYN_E_SHAPE;
  }
  const size_t n_row = (size_t)d->n_class * d->n_tp * d->n_f, n_tab = n_row * d->n_rho;
  if (n_tab > ((size_t)1 << 31)) { dyn_set_error("profile tables too large"); return DYN_E_SHAPE; }
  for (int i = 0; i < d->n_tp; ++i)
    if (d->tp[i] < 1 || (i > 0 && d->tp[i] <= d->tp[i - 1])) { dyn_set_error("tp[] must be >= 1 and strictly increasing"); return DYN_E_ORDER; }
  if (!strictly_increasing(d->f_mhz, d->n_f)) { dyn_set_error("f_mhz[] must be finite and strictly increasing"); return DYN_E_ORDER; }
  if (!strictly_increasing(d->rho, d->n_rho)) { dyn_set_error("rho[] must be finite and strictly increasing"); return DYN_E_ORDER; }
  if (d->rho[0] != 0.0) { dyn_set_error("rho[0] must be 0"); return DYN_E_RANGE; }
  for (size_t i = 0; i < n_tab; ++i) {
    const double a = d->prefill_ms_per_tok[i], b = d->tbt_ms[i], c = d->power_w[i];
    if (!isfinite(a) || !isfinite(b) || !isfinite(c) || a < 0.0 || b < 0.0 || c < 0.0) {
      dyn_set_error("table entry %zu is negative or not finite", i);
      return DYN_E_NOTFINITE;
    }
  }
  for (size_t i = 0; i < n_row; ++i)
    if (!in_scale(d->max_load_tps[i])) {
      dyn_set_error("max_load_tps[%zu] must lie in [1e-100, 1e100]", i);
      return DYN_E_NOTFINITE;
    }
  if (!(d->rho[d->n_rho - 1] <= kMaxScale)) { dyn_set_error("rho[] must stay below 1e100"); return DYN_E_RANGE; }
  for (int q = 1; q < d->n_rho; ++q)
    if (!(d->rho[q] - d->rho[q - 1] >= kMinScale)) { dyn_set_error("rho[] spacing below 1e-100"); return DYN_E_RANGE; }

  dyn_profile* p = new (std::nothrow) dyn_profile();
  if (!p) { dyn_set_error("out of host memory"); return DYN_E_DEVICE; }
  p->G = d->n_class; p->n_tp = d->n_tp; p->n_f = d->n_f; p->n_rho = d->n_rho;
  p->tp.assign(d->tp, d->tp + d->n_tp);
  p->fg.assign(d->f_mhz, d->f_mhz + d->n_f);
  p->d_tab = p->d_ml = p->d_pw0 = p->d_pfspan = p->d_gridpack = nullptr;
  p->d_theta = nullptr;
  p->d_jstart = nullptr; p->d_tstart = nullptr; p->d_thr = nullptr; p->d_cfg = nullptr; p->d_tile_rows = nullptr;
  p->d_slo_ttft = p->d_slo_tbt = nullptr; p->d_budget = nullptr;
  p->d_path_layout = p->d_path_order = p->d_path_seg = p->d_lay_n = p->d_lay_tp = p->d_tp = p->d_ident = nullptr;
  p->d_path_trans = p->d_hier_trans = nullptr;
  p->obj_valid = false; p->tile = p->n_tile = p->n_slot = 0; p->any_two_rows = false;
  p->wpb = p->wpb_windows = 0; p->wpb_tuned = false; p->n_cu = 0;
  hipStream_t s = (hipStream_t)hip_stream;

  // Bucket index over the load axis: bucket b covers [b, b+1) / bucket_scale and js[b] is the
  // largest grid index i <= n_rho-2 with rho[i] <= b / bucket_scale.  The buckets are made
  // fine enough (up to 4096 of them) that no two neighbouring buckets hold more than one
  // grid point; then a bracket is at most one step away from its bucket's index.
  const double rho_max = d->rho[d->n_rho - 1];
  double min_gap = rho_max;
  for (int q = 1; q < d->n_rho; ++q) min_gap = std::min(min_gap, d->rho[q] - d->rho[q - 1]);
  const double want = 3.0 * rho_max / min_gap;            // bucket width <= a third of the narrowest interval
  p->n_bucket = (int32_t)std::min(4096.0, std::max(16.0, ceil(want)));
  p->one_step = (double)p->n_bucket >= want;
  p->bucket_scale = (double)p->n_bucket / rho_max;
  std::vector<int32_t> js(p->n_bucket + 1);     // index n_bucket is reached only by rc == rho_max
  for (int b = 0; b <= p->n_bucket; ++b) {
    const double x = (double)b / p->bucket_scale;
    int j = 0;
    for (int q = 0; q < d->n_rho - 1; ++q)
      if (d->rho[q] <= x) j = q;
    js[b] = j;
  }
  // The same buckets seen through the kernels' bucket arithmetic (monotone in x): a grid point
  // whose bucket is below that of x is below x, one whose bucket is above is above x, and
  // only a point in x's own bucket has to be compared.
  std::vector<int32_t> tstart(p->n_bucket + 1, 0);
  std::vector<double> thr(p->n_bucket + 1, INFINITY);
  p->single_point = (int)(rho_max * p->bucket_scale) <= p->n_bucket;
  for (int q = 1; q + 1 < d->n_rho && p->single_point; ++q) {
    const int b = (int)(d->rho[q] * p->bucket_scale);
    if (b < 0 || b > p->n_bucket || thr[b] != INFINITY) { p->single_point = false; break; }
    thr[b] = d->rho[q];
    for (int c = b + 1; c <= p->n_bucket; ++c) tstart[c] += 1;
  }
  std::vector<double> gridpack(2 * (size_t)d->n_rho + 3, 0.0);
  gridpack[0] = -INFINITY;
  for (int q = 0; q < d->n_rho; ++q) gridpack[1 + q] = d->rho[q];
  gridpack[d->n_rho + 1] = INFINITY;
  for (int q = 0; q + 1 < d->n_rho; ++q) gridpack[d->n_rho + 3 + q] = 1.0 / (d->rho[q + 1] - d->rho[q]);
  // one packed row per (class, TP, f): prefill | TBT | power
  std::vector<double> packed(3 * n_tab);
  for (size_t r = 0; r < n_row; ++r) {
    memcpy(&packed[(3 * r + 0) * d->n_rho], d->prefill_ms_per_tok + r * d->n_rho, (size_t)d->n_rho * 8);
    memcpy(&packed[(3 * r + 1) * d->n_rho], d->tbt_ms + r * d->n_rho, (size_t)d->n_rho * 8);
    memcpy(&packed[(3 * r + 2) * d->n_rho], d->power_w + r * d->n_rho, (size_t)d->n_rho * 8);
  }
  std::vector<double> pw0(n_row);
  for (size_t r = 0; r < n_row; ++r) pw0[r] = d->power_w[r * d->n_rho];
  std::vector<double> pfspan(2 * n_row);
  for (size_t r = 0; r < n_row; ++r) {
    const double* row = d->prefill_ms_per_tok + r * d->n_rho;
    pfspan[2 * r] = *std::min_element(row, row + d->n_rho);
    pfspan[2 * r + 1] = *std::max_element(row, row + d->n_rho);
  }
  // per class the least ratio over its rows, as a float below the quotient by 2^-21 at least (0: no bound)
  std::vector<float> theta(p->G, 0.0f);
  {
    const size_t per_class = n_row / (size_t)p->G;
    for (int g = 0; g < p->G; ++g) {
      double th = 1.0;
      for (size_t r = (size_t)g * per_class; r < (size_t)(g + 1) * per_class; ++r)
        th = (pfspan[2 * r] > 0.0 && pfspan[2 * r + 1] > 0.0) ? std::min(th, pfspan[2 * r] / pfspan[2 * r + 1]) : 0.0;
      theta[g] = (float)th * 0.999999f;
    }
  }

  void* fixed_ws = nullptr;
  (void)scratch_address(&fixed_ws);   // set-up of dyn_eval_select_static on this device; that call reports a failure itself
  bool ok = hip_ok(hipGetDevice(&p->device), "hipGetDevice") &&
            hip_ok(hipDeviceGetAttribute(&p->n_cu, hipDeviceAttributeMultiprocessorCount, p->device), "hipDeviceGetAttribute") &&
            hip_ok(dev_alloc(&p->d_tab, 3 * n_tab), "hipMalloc") && hip_ok(dev_alloc(&p->d_ml, n_row), "hipMalloc") &&
            hip_ok(dev_alloc(&p->d_pw0, n_row), "hipMalloc") && hip_ok(dev_alloc(&p->d_pfspan, 2 * n_row), "hipMalloc") &&
            hip_ok(dev_alloc(&p->d_theta, (size_t)p->G), "hipMalloc") &&
            hip_ok(dev_alloc(&p->d_gridpack, gridpack.size()), "hipMalloc") &&
            hip_ok(dev_alloc(&p->d_jstart, js.size()), "hipMalloc") &&
            hip_ok(dev_alloc(&p->d_tstart, tstart.size()), "hipMalloc") && hip_ok(dev_alloc(&p->d_thr, thr.size()), "hipMalloc") &&
            hip_ok(dev_alloc(&p->d_cfg, DYN_MAX_CONFIGS), "hipMalloc") &&
            hip_ok(dev_alloc(&p->d_tile_rows, 2 * DYN_MAX_CONFIGS + 1024), "hipMalloc") &&
            hip_ok(dev_alloc(&p->d_slo_ttft, p->G), "hipMalloc") && hip_ok(dev_alloc(&p->d_slo_tbt, p->G), "hipMalloc") &&
            hip_ok(dev_alloc(&p->d_budget, p->G), "hipMalloc") &&
            hip_ok(dev_alloc(&p->d_path_layout, DYN_MAX_CONFIGS), "hipMalloc") && hip_ok(dev_alloc(&p->d_path_order, DYN_MAX_CONFIGS), "hipMalloc") &&
            hip_ok(dev_alloc(&p->d_path_seg, DYN_MAX_LAYOUTS + 1), "hipMalloc") &&
            hip_ok(dev_alloc(&p->d_path_trans, DYN_MAX_LAYOUTS * DYN_MAX_LAYOUTS), "hipMalloc") &&
            hip_ok(dev_alloc(&p->d_hier_trans, DYN_MAX_LAYOUTS * DYN_MAX_LAYOUTS), "hipMalloc") &&
            hip_ok(dev_alloc(&p->d_lay_n, DYN_MAX_CONFIGS), "hipMalloc") && hip_ok(dev_alloc(&p->d_lay_tp, DYN_MAX_CONFIGS), "hipMalloc") &&
            hip_ok(dev_alloc(&p->d_tp, p->n_tp), "hipMalloc") && hip_ok(dev_alloc(&p->d_ident, DYN_MAX_CONFIGS + 1), "hipMalloc");
  std::vector<int32_t> ident(DYN_MAX_CONFIGS + 1);
  std::iota(ident.begin(), ident.end(), 0);
  ok = ok && hip_ok(hipMemcpyAsync(p->d_tab, packed.data(), 3 * n_tab * 8, hipMemcpyHostToDevice, s), "copy") &&
       hip_ok(hipMemcpyAsync(p->d_ml, d->max_load_tps, n_row * 8, hipMemcpyHostToDevice, s), "copy") &&
       hip_ok(hipMemcpyAsync(p->d_pw0, pw0.data(), n_row * 8, hipMemcpyHostToDevice, s), "copy") &&
       hip_ok(hipMemcpyAsync(p->d_pfspan, pfspan.data(), 2 * n_row * 8, hipMemcpyHostToDevice, s), "copy") &&
       hip_ok(hipMemcpyAsync(p->d_theta, theta.data(), (size_t)p->G * 4, hipMemcpyHostToDevice, s), "copy") &&
       hip_ok(hipMemcpyAsync(p->d_gridpack, gridpack.data(), gridpack.size() * 8, hipMemcpyHostToDevice, s), "copy") &&
       hip_ok(hipMemcpyAsync(p->d_jstart, js.data(), js.size() * 4, hipMemcpyHostToDevice, s), "copy") &&
       hip_ok(hipMemcpyAsync(p->d_tstart, tstart.data(), tstart.size() * 4, hipMemcpyHostToDevice, s), "copy") &&
       hip_ok(hipMemcpyAsync(p->d_thr, thr.data(), thr.size() * 8, hipMemcpyHostToDevice, s), "copy") &&
       hip_ok(hipMemcpyAsync(p->d_tp, p->tp.data(), p->tp.size() * 4, hipMemcpyHostToDevice, s), "copy") &&
       hip_ok(hipMemcpyAsync(p->d_ident, ident.data(), ident.size() * 4, hipMemcpyHostToDevice, s), "copy") &&
       hip_ok(hipStreamSynchronize(s), "hipStreamSynchronize");
  if (!ok) {
    free_profile_device(p);
    delete p;
    return DYN_E_DEVICE;
  }
  *out = p;
  return DYN_OK;
}

void dyn_profile_free(dyn_profile* p) {
  if (!p) return;
  free_profile_device(p);
  delete p;
}

size_t dyn_trace_ingest_workspace(int64_t n_req, int32_t n_window, int32_t n_class) {
  // edge tables are at most one int per class and axis
  if (n_req < 0 || n_class < 1 || n_window < 1) return 0;
  return ingest_ws_layout(n_req, n_class, 2, 2, n_window).total;
}

int dyn_trace_ingest(const double* t_s, const int32_t* in_tok, const int32_t* out_tok, const int32_t* model,
                     int64_t n_req, const dyn_class_edges* e, int32_t n_window, double window_s,
                     int32_t* in_sorted, int32_t* out_sorted, int64_t* cell_off, void* workspace,
                     size_t workspace_bytes, void* hip_stream) {
  if (!e || !cell_off || !workspace) { dyn_set_error("edges, cell_off or workspace is NULL"); return DYN_E_NULL; }
  if (n_req < 0 || n_req >= ((int64_t)1 << 31)) { dyn_set_error("n_req=%lld outside [0, 2^31)", (long long)n_req); return DYN_E_SHAPE; }
  if (n_req > 0 && (!t_s || !in_tok || !out_tok || !in_sorted || !out_sorted)) { dyn_set_error("a trace array is NULL"); return DYN_E_NULL; }
  if (e->n_model < 1 || e->n_in_bin < 1 || e->n_out_bin < 1 || n_window < 1) { dyn_set_error("class or window counts < 1"); return DYN_E_SHAPE; }
  if ((e->n_in_bin > 1 && !e->in_edge) || (e->n_out_bin > 1 && !e->out_edge)) { dyn_set_error("edge array is NULL"); return DYN_E_NULL; }
  if (!in_scale(window_s)) { dyn_set_error("window_s must lie in [1e-100, 1e100]"); return DYN_E_RANGE; }
  const int64_t G = (int64_t)e->n_model * e->n_in_bin * e->n_out_bin;
  const int64_t cells = G * n_window;
  if (G >= ((int64_t)1 << 30) || cells >= ((int64_t)1 << 30)) { dyn_set_error("n_window * classes must stay below 2^30"); return DYN_E_SHAPE; }
  for (int m = 0; m < e->n_model; ++m) {
    for (int i = 1; i < e->n_in_bin - 1; ++i)
      if (e->in_edge[m * (e->n_in_bin - 1) + i] <= e->in_edge[m * (e->n_in_bin - 1) + i - 1]) { dyn_set_error("in_edge of model %d not strictly increasing", m); return DYN_E_ORDER; }
    for (int i = 1; i < e->n_out_bin - 1; ++i)
      if (e->out_edge[m * (e->n_out_bin - 1) + i] <= e->out_edge[m * (e->n_out_bin - 1) + i - 1]) { dyn_set_error("out_edge of model %d not strictly increasing", m); return DYN_E_ORDER; }
  }
  if (n_req > 0 && (in_sorted == in_tok || out_sorted == out_tok || in_sorted == out_tok || out_sorted == in_tok)) {
    dyn_set_error("sorted outputs alias the inputs");
    return DYN_E_RANGE;
  }
  const IngestWs w = ingest_ws_layout(n_req, e->n_model, e->n_in_bin, e->n_out_bin, n_window);
  if (((uintptr_t)workspace & 255) || workspace_bytes < w.total) {
    dyn_set_error("workspace misaligned or too small (%zu < %zu)", workspace_bytes, w.total);
    return DYN_E_WORKSPACE;
  }
  hipStream_t s = (hipStream_t)hip_stream;
  char* base = (char*)workspace;
  IngestArgs a;
  a.t_s = t_s; a.in_tok = in_tok; a.out_tok = out_tok; a.model = model; a.n_req = n_req;
  a.n_model = e->n_model; a.n_in_bin = e->n_in_bin; a.n_out_bin = e->n_out_bin; a.n_window = n_window;
  a.window_s = window_s;
  a.d_in_edge = (const int32_t*)(base + w.in_edge); a.d_out_edge = (const int32_t*)(base + w.out_edge);
  a.in_sorted = in_sorted; a.out_sorted = out_sorted; a.cell_off = cell_off;
  a.status = (uint32_t*)(base + w.status);
  a.key_a = (uint32_t*)(base + w.key_a); a.key_b = (uint32_t*)(base + w.key_b);
  a.in_tmp = (int32_t*)(base + w.in_tmp); a.out_tmp = (int32_t*)(base + w.out_tmp);
  a.block_hist = (uint32_t*)(base + w.hist);
  a.unsorted = (uint32_t*)(base + w.status) + DYN_WS_HEADER_ORDER_WORD;
  a.force_sort = G > DYN_INGEST_MAX_BINS ? 1 : 0;   // the window route keeps one counter per class in LDS
  a.win_off = (int64_t*)(base + w.win_off);
  a.n_block = dyn_ingest_blocks(n_req);
  int bits = 0;
  while (((int64_t)1 << bits) < cells) ++bits;
  a.key_bits = bits;
  // the workspace header (status 0, order word = "general sort forced") and the edge lists, which travel in a kernel's
  // arguments: the host arrays are free on return and nothing waits for the stream
  if (!hip_ok(dyn_launch_edges(e->in_edge, (size_t)e->n_model * (e->n_in_bin - 1), e->out_edge, (size_t)e->n_model * (e->n_out_bin - 1),
                               (int32_t*)(base + w.in_edge), (int32_t*)(base + w.out_edge), (WsHeader*)a.status, a.force_sort ? 1u : 0u, s),
              "edge launch"))
    return DYN_E_DEVICE;
  if (!hip_ok(dyn_launch_ingest(a, s), "ingest launch")) return DYN_E_DEVICE;
  return DYN_OK;
}

size_t dyn_eval_space_workspace(int32_t n_window, int32_t n_class, int32_t n_config) {
  if (n_window < 1 || n_class < 1 || n_config < 1) return 0;
  return dyn_eval_ws_layout((int64_t)n_window * n_class, n_config).total;
}

int dyn_eval_space(dyn_profile* p, const dyn_trace_view* t, const dyn_config* cfg, int32_t K,
                   const dyn_objective* o, const dyn_space* out, void* workspace, size_t workspace_bytes,
                   void* hip_stream) {
  return eval_impl(p, t, cfg, K, o, out, nullptr, workspace, workspace_bytes, hip_stream);
}

int dyn_eval_select(dyn_profile* p, const dyn_trace_view* t, const dyn_config* cfg, int32_t K,
                    const dyn_objective* o, const dyn_space* out, const dyn_selection* sel, void* workspace,
                    size_t workspace_bytes, void* hip_stream) {
  if (!sel) { dyn_set_error("selection is NULL"); return DYN_E_NULL; }
  return eval_impl(p, t, cfg, K, o, out, sel, workspace, workspace_bytes, hip_stream);
}

int dyn_eval_tune(dyn_profile* p, const dyn_trace_view* t, const dyn_config* cfg, int32_t K, const dyn_objective* o,
                  const dyn_space* out, const dyn_selection* sel, void* workspace, size_t workspace_bytes,
                  void* hip_stream, int32_t* chosen) {
  if (!sel) { dyn_set_error("selection is NULL"); return DYN_E_NULL; }
  // one plain call first: it checks every argument and leaves the handle's plan in place
  int rc = eval_impl(p, t, cfg, K, o, out, sel, workspace, workspace_bytes, hip_stream);
  if (rc != DYN_OK) return rc;
  hipStream_t s = (hipStream_t)hip_stream;
  const int32_t start = p->wpb;                                  // the rule's value (or an earlier measurement)
  const int64_t cell_tiles = (int64_t)t->n_window * p->G * p->n_tile;
  const int32_t most = (int32_t)std::max<int64_t>(1, std::min<int64_t>(DYN_MAX_WIN_PER_BLOCK, (cell_tiles + 8191) / 8192));
  hipEvent_t e0 = nullptr, e1 = nullptr;
  if (!hip_ok(hipEventCreate(&e0), "hipEventCreate") || !hip_ok(hipEventCreate(&e1), "hipEventCreate")) {
    if (e0) (void)hipEventDestroy(e0);
    return DYN_E_DEVICE;
  }
  const int32_t cand[] = {1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 12, 14, 16, 20, 24, 32};
  int reps = 3;                                                  // raised after the first measurement: about 2 ms per shape
  int32_t best = start;
  float best_ms = -1.f;
  bool first = true;
  for (int32_t c : cand) {
    if (c > most) break;
    p->wpb = c; p->wpb_windows = t->n_window;
    for (int pass = 0; pass < 2 && rc == DYN_OK; ++pass) {       // a warm-up call, then `reps` timed ones
      if (pass == 1 && !hip_ok(hipEventRecord(e0, s), "hipEventRecord")) rc = DYN_E_DEVICE;
      for (int r = 0; r < (pass ? reps : 1) && rc == DYN_OK; ++r)
        rc = eval_impl(p, t, cfg, K, o, out, sel, workspace, workspace_bytes, hip_stream);
    }
    float ms = 0.f;
    if (rc == DYN_OK && (!hip_ok(hipEventRecord(e1, s), "hipEventRecord") || !hip_ok(hipEventSynchronize(e1), "hipEventSynchronize") ||
                         !hip_ok(hipEventElapsedTime(&ms, e0, e1), "hipEventElapsedTime")))
      rc = DYN_E_DEVICE;
    if (rc != DYN_OK) break;
    ms /= (float)reps;
    if (best_ms < 0.f || ms < best_ms) { best_ms = ms; best = c; }
    if (first) {
      first = false;
      reps = (int)std::max(3.0f, std::min(16.0f, 2.0f / std::max(ms, 1e-3f)));
    }
  }
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  p->wpb = rc == DYN_OK ? best : start;
  p->wpb_windows = t->n_window;
  p->wpb_tuned = rc == DYN_OK;
  if (rc != DYN_OK) return rc;
  if (chosen) *chosen = best;
  // the outputs are those of the last candidate's run; every run writes the same values
  return DYN_OK;
}

int dyn_eval_select_static(dyn_profile* p, const dyn_trace_view* t, const dyn_config* cfg, int32_t K,
                           const dyn_objective* o, const dyn_space* out, const dyn_selection* sel,
                           uint32_t* status, void* hip_stream) {
  if (!sel) { dyn_set_error("selection is NULL"); return DYN_E_NULL; }
  if (!p || !t) { dyn_set_error("profile or trace is NULL"); return DYN_E_NULL; }
  if (t->n_window < 1 || K < 1) { dyn_set_error("n_window or K < 1"); return DYN_E_SHAPE; }
  const int64_t cells = (int64_t)t->n_window * p->G;
  if (cells >= ((int64_t)1 << 30)) { dyn_set_error("n_window * classes must stay below 2^30"); return DYN_E_SHAPE; }
  const EvalWs w = dyn_eval_ws_layout(cells, K);
  if (w.total > (size_t)DYN_STATIC_WORKSPACE_BYTES) {
    dyn_set_error("%lld cells x %d configurations need %zu bytes of workspace, the fixed one holds %zu: use dyn_eval_select with a workspace of the caller",
                  (long long)cells, K, w.total, (size_t)DYN_STATIC_WORKSPACE_BYTES);
    return DYN_E_WORKSPACE;
  }
  int rc;
  if ((rc = check_device(p)) != DYN_OK) return rc;
  void* ws = nullptr;
  if ((rc = scratch_address(&ws)) != DYN_OK) return rc;
  if ((rc = eval_impl(p, t, cfg, K, o, out, sel, ws, (size_t)DYN_STATIC_WORKSPACE_BYTES, hip_stream)) != DYN_OK) return rc;
  if (status) {
    hipLaunchKernelGGL(cell_status_word_kernel, dim3(1), dim3(1024), 0, (hipStream_t)hip_stream,
                       (const uint8_t*)((const char*)ws + w.cstat), cells, status);
    if (!hip_ok(hipGetLastError(), "status launch")) return DYN_E_DEVICE;
  }
  return DYN_OK;
}

size_t dyn_eval_ticks_workspace(int64_t n_req, int32_t n_window, int32_t n_tick, int32_t n_class, int32_t n_config) {
  if (n_req < 0 || n_window < 1 || n_tick < 1 || n_tick > DYN_TICK_LIMIT || n_class < 1 || n_config < 1) return 0;
  return dyn_tick_ws_layout(n_req, (int64_t)n_window * n_class, n_tick, n_config).total;
}

int dyn_eval_select_ticks(dyn_profile* p, const dyn_trace_view* t, int32_t n_tick, const dyn_config* cfg, int32_t K,
                          const dyn_objective* o, const dyn_space* out, const dyn_selection* sel, void* workspace,
                          size_t workspace_bytes, void* hip_stream) {
  if (!p || !t || !out || !sel || !workspace) { dyn_set_error("profile, trace, space, sel or workspace is NULL"); return DYN_E_NULL; }
  if (!out->energy_j || !out->p99_ttft_ms || !out->p99_tbt_ms || !out->flags) { dyn_set_error("an output array is NULL"); return DYN_E_NULL; }
  int rc;
  if ((rc = check_selection(sel)) != DYN_OK) return rc;
  if (n_tick < 1 || n_tick > DYN_TICK_LIMIT) { dyn_set_error("n_tick=%d outside [1, %d]", n_tick, DYN_TICK_LIMIT); return DYN_E_SHAPE; }
  if (t->n_req < 0 || t->n_req >= ((int64_t)1 << 31) || t->n_window < 1) { dyn_set_error("n_req or n_window out of range"); return DYN_E_SHAPE; }
  if (t->n_window % n_tick != 0) { dyn_set_error("fine n_window=%d is not a multiple of n_tick=%d", t->n_window, n_tick); return DYN_E_SHAPE; }
  if (!t->cell_off || (t->n_req > 0 && (!t->in_tok || !t->out_tok))) { dyn_set_error("a trace array is NULL"); return DYN_E_NULL; }
  if (!in_scale(t->window_s)) { dyn_set_error("tick length must lie in [1e-100, 1e100]"); return DYN_E_RANGE; }
  const int32_t n_window = t->n_window / n_tick;
  const int64_t cells = (int64_t)n_window * p->G, fine_cells = cells * n_tick;
  if (fine_cells >= ((int64_t)1 << 30)) { dyn_set_error("n_window * n_tick * classes must stay below 2^30"); return DYN_E_SHAPE; }
  if ((rc = check_device(p)) != DYN_OK) return rc;
  if (K < 1 || K > DYN_MAX_CONFIGS) { dyn_set_error("K=%d outside [1, %d]", K, DYN_MAX_CONFIGS); return DYN_E_SHAPE; }
  const TickWs w = dyn_tick_ws_layout(t->n_req, cells, n_tick, K);
  if (((uintptr_t)workspace & 255) || workspace_bytes < w.total) {
    dyn_set_error("workspace misaligned or too small (%zu < %zu)", workspace_bytes, w.total);
    return DYN_E_WORKSPACE;
  }
  hipStream_t s = (hipStream_t)hip_stream;
  if ((rc = prepare_configs(p, cfg, K, s)) != DYN_OK) return rc;
  if ((rc = prepare_objective(p, o, s)) != DYN_OK) return rc;

  char* base = (char*)workspace;
  TickCellArgs ca;
  ca.in = t->in_tok; ca.out = t->out_tok; ca.fine_off = t->cell_off; ca.n_req = t->n_req;
  ca.n_window = n_window; ca.n_tick = n_tick; ca.G = p->G;
  ca.tick_s = t->window_s; ca.r_tick = 1.0 / t->window_s;
  ca.pct_num = o->pct_num; ca.pct_den = o->pct_den;
  ca.rec = (TickRec*)(base + w.fine.rec); ca.plan = (TickPlan*)(base + w.plan); ca.top = (int32_t*)(base + w.top);
  ca.cstat = (uint8_t*)(base + w.fine.cstat); ca.header = (WsHeader*)(base + w.fine.header);
  ca.counters = (uint32_t*)(base + w.counters); ca.deep_list = (uint32_t*)(base + w.deep_list); ca.slow_list = (uint32_t*)(base + w.slow_list);
  ca.list_cells = (uint32_t*)(base + w.list_cells); ca.theta = p->d_theta;
  ca.few_cells = cells <= 4 * (int64_t)p->n_cu ? 1 : 0;   // every cell's block is resident at once (four blocks of four waves per compute unit)
  if (!hip_ok(dyn_launch_tick_cell(ca, s), "tick cell launch")) return DYN_E_DEVICE;

  TickArgs ta;
  SpaceArgs& a = ta.s;
  a.tab = p->d_tab; a.ml = p->d_ml; a.gridpack = p->d_gridpack;
  a.jstart = p->d_jstart; a.n_bucket = p->n_bucket; a.bucket_scale = p->bucket_scale; a.one_step = p->one_step;
  a.G = p->G; a.n_tp_f = p->n_tp * p->n_f; a.n_rho = p->n_rho;
  a.cfg = p->d_cfg; a.K = K; a.tile = p->tile; a.n_tile = p->n_tile; a.n_slot = p->n_slot;
  a.tile_rows = p->d_tile_rows;
  a.slo_ttft = p->d_slo_ttft; a.slo_tbt = p->d_slo_tbt; a.budget = p->d_budget;
  a.rec = nullptr; a.n_window = n_window; a.window_s = t->window_s;
  const int64_t cell_tiles = cells * p->n_tile;
  // about 8192 blocks; beyond 16 windows a block gains nothing more from its staged rows (measured: 10 .. 20 alike)
  a.win_per_block = (int32_t)std::max<int64_t>(1, std::min<int64_t>(16, (cell_tiles + 8191) / 8192));
  a.energy = out->energy_j; a.p99_ttft = out->p99_ttft_ms; a.p99_tbt = out->p99_tbt_ms; a.flags = out->flags;
  a.pw0 = p->d_pw0; a.idle_w = o->idle_cost_weight;
  a.part = (SelPart*)(base + w.part); a.n_wslot = w.n_wslot;
  ta.n_tick = n_tick; ta.tick_s = t->window_s; ta.window_s = (double)n_tick * t->window_s;
  ta.rec = (const TickRec*)(base + w.fine.rec); ta.plan = (const TickPlan*)(base + w.plan); ta.top = (const int32_t*)(base + w.top);
  ta.in = t->in_tok;
  ta.counters = (const uint32_t*)(base + w.counters); ta.slow_list = (const uint32_t*)(base + w.slow_list);
  ta.tstart = p->d_tstart; ta.thr = p->d_thr; ta.single_point = p->single_point; ta.any_two_rows = p->any_two_rows;
  ta.pfspan = p->d_pfspan; ta.n_cu = p->n_cu;
  if (!hip_ok(dyn_launch_tick_space(ta, s), "tick space launch")) return DYN_E_DEVICE;

  FinishArgs f;
  f.part = a.part; f.n_wslot = w.n_wslot; f.n_used = p->n_tile * (p->tile / DYN_WAVE);
  f.n_window = n_window; f.G = p->G;
  f.sel = sel->sel; f.sel_energy = sel->sel_energy_j; f.sel_cost = sel->sel_cost;
  f.win_energy = sel->window_energy_j; f.win_inf = sel->window_infeasible;
  if (!hip_ok(dyn_launch_finish(f, s), "finish launch")) return DYN_E_DEVICE;
  return DYN_OK;
}

namespace {

struct MixedWs {
  EvalWs cell;       // header .. cstat (per-cell aggregates); cell.part is where type_energy starts
  size_t type_energy, type_f, ok, total;
};
struct MixedPlan {
  MixedTypes types;
  int32_t n_entry, unit, u_max;
};
// Checks the request against the profile and lays the entries out.  Returns DYN_OK or an error status.
int plan_mixed(const dyn_profile* p, const dyn_mixed_space* m, MixedPlan* out) {
  if (!m || !m->n_max) { dyn_set_error("mixed space or n_max is NULL"); return DYN_E_NULL; }
  if (m->n_share < 1 || m->n_share > DYN_MIXED_MAX_SHARES) { dyn_set_error("n_share=%d outside [1, %d]", m->n_share, DYN_MIXED_MAX_SHARES); return DYN_E_SHAPE; }
  if (p->n_tp > DYN_MIXED_MAX_TYPES || p->n_f > DYN_MIXED_FREQ_LANES) { dyn_set_error("profile has more than %d types or %d frequencies", DYN_MIXED_MAX_TYPES, DYN_MIXED_FREQ_LANES); return DYN_E_SHAPE; }
  MixedTypes& t = out->types;
  memset(&t, 0, sizeof(t));
  t.n_tp = p->n_tp;
  int32_t unit = 0;
  for (int i = 0; i < p->n_tp; ++i) {
    if (m->n_max[i] < 0 || m->n_max[i] > 255) { dyn_set_error("n_max[%d]=%d outside [0, 255]", i, m->n_max[i]); return DYN_E_RANGE; }
    t.n_max[i] = m->n_max[i];
    t.off[i + 1] = t.off[i] + m->n_max[i] * m->n_share;
    if (m->n_max[i] > 0) unit = std::gcd(unit, p->tp[i]);
  }
  if (unit == 0) { dyn_set_error("every n_max is 0"); return DYN_E_SHAPE; }
  int64_t u_max = 0;
  for (int i = 0; i < p->n_tp; ++i) {
    t.units[i] = p->tp[i] / unit;
    u_max += (int64_t)t.n_max[i] * (t.n_max[i] > 0 ? t.units[i] : 0);
  }
  out->n_entry = t.off[p->n_tp];
  out->unit = unit;
  out->u_max = (int32_t)std::min<int64_t>(u_max, 1 << 20);
  return DYN_OK;
}
MixedWs mixed_ws_layout(int64_t cells, int32_t n_entry) {
  MixedWs w;
  w.cell = dyn_eval_ws_layout(cells, 1);
  const size_t c = (size_t)std::max<int64_t>(cells, 1);
  size_t off = w.cell.part;
  w.type_energy = off; off += align256(c * (size_t)n_entry * sizeof(double));
  w.type_f = off; off += align256(c * (size_t)n_entry);
  w.ok = off; off += align256(c * sizeof(int32_t));
  w.total = off;
  return w;
}

}  // namespace

size_t dyn_mixed_workspace(const dyn_profile* p, int32_t n_window, const dyn_mixed_space* m) {
  MixedPlan mp;
  if (!p || n_window < 1 || plan_mixed(p, m, &mp) != DYN_OK) return 0;
  return mixed_ws_layout((int64_t)n_window * p->G, mp.n_entry).total;
}

int dyn_eval_select_mixed(dyn_profile* p, const dyn_trace_view* t, const dyn_mixed_space* m, const dyn_objective* o,
                          const dyn_mixed_selection* out, void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!p || !t || !m || !o || !out || !workspace) { dyn_set_error("profile, trace, space, objective, out or workspace is NULL"); return DYN_E_NULL; }
  if (!out->energy_j || !out->n_inst || !out->f_index || !out->share || !out->window_energy_j || !out->window_infeasible) {
    dyn_set_error("an output array is NULL");
    return DYN_E_NULL;
  }
  if (t->n_req < 0 || t->n_req >= ((int64_t)1 << 31) || t->n_window < 1) { dyn_set_error("n_req or n_window out of range"); return DYN_E_SHAPE; }
  if (!t->cell_off || (t->n_req > 0 && (!t->in_tok || !t->out_tok))) { dyn_set_error("a trace array is NULL"); return DYN_E_NULL; }
  if (!in_scale(t->window_s)) { dyn_set_error("window_s must lie in [1e-100, 1e100]"); return DYN_E_RANGE; }
  const int64_t cells = (int64_t)t->n_window * p->G;
  if (cells >= ((int64_t)1 << 30)) { dyn_set_error("n_window * classes must stay below 2^30"); return DYN_E_SHAPE; }
  int rc;
  if ((rc = check_device(p)) != DYN_OK) return rc;
  MixedPlan mp;
  if ((rc = plan_mixed(p, m, &mp)) != DYN_OK) return rc;
  // the dynamic programme's state must fit one block's LDS for the largest budget in use
  int32_t u_need = 0;
  for (int g = 0; g < p->G; ++g) {
    const int32_t b = o->gpu_budget ? o->gpu_budget[g] : 0;
    u_need = std::max(u_need, b > 0 ? std::min(b / mp.unit, mp.u_max) : mp.u_max);
  }
  if (dyn_mixed_combine_lds(p->n_tp, mp.n_entry, u_need, m->n_share) > DYN_LDS_BUDGET) {
    dyn_set_error("the assignment state (%d GPU units x %d shares, %d entries) does not fit in LDS: set a GPU budget or lower n_max / n_share",
                  u_need + 1, m->n_share + 1, mp.n_entry);
    return DYN_E_SHAPE;
  }
  const MixedWs w = mixed_ws_layout(cells, mp.n_entry);
  if (((uintptr_t)workspace & 255) || workspace_bytes < w.total) {
    dyn_set_error("workspace misaligned or too small (%zu < %zu)", workspace_bytes, w.total);
    return DYN_E_WORKSPACE;
  }
  hipStream_t s = (hipStream_t)hip_stream;
  if ((rc = prepare_objective(p, o, s)) != DYN_OK) return rc;

  char* base = (char*)workspace;
  if (!hip_ok(dyn_launch_cell_aggregate(t->in_tok, t->out_tok, t->cell_off, t->n_req, cells, t->window_s, o->pct_num,
                                        o->pct_den, (int64_t*)(base + w.cell.tin), (int64_t*)(base + w.cell.tout),
                                        (int32_t*)(base + w.cell.in_p99), (CellRec*)(base + w.cell.rec),
                                        (uint8_t*)(base + w.cell.cstat), (WsHeader*)(base + w.cell.header), s),
              "cell aggregate launch"))
    return DYN_E_DEVICE;

  MixedTypeArgs ta;
  ta.tab = p->d_tab; ta.ml = p->d_ml; ta.gridpack = p->d_gridpack;
  ta.jstart = p->d_jstart; ta.tstart = p->d_tstart; ta.thr = p->d_thr; ta.n_bucket = p->n_bucket; ta.bucket_scale = p->bucket_scale;
  ta.G = p->G; ta.n_tp = p->n_tp; ta.n_f = p->n_f; ta.n_rho = p->n_rho;
  ta.slo_ttft = p->d_slo_ttft; ta.slo_tbt = p->d_slo_tbt;
  ta.rec = (const CellRec*)(base + w.cell.rec); ta.n_window = t->n_window; ta.window_s = t->window_s;
  ta.win_per_block = (int32_t)std::max<int64_t>(1, std::min<int64_t>(DYN_MAX_WIN_PER_BLOCK, (cells * p->n_tp + 4095) / 4096));
  ta.n_share = m->n_share; ta.r_share = 1.0 / (double)m->n_share;
  ta.types = mp.types;
  ta.type_energy = (double*)(base + w.type_energy); ta.type_f = (int8_t*)(base + w.type_f);
  if (!hip_ok(dyn_launch_mixed_types(ta, p->single_point, s), "mixed types launch")) return DYN_E_DEVICE;

  MixedCombineArgs ca;
  ca.type_energy = ta.type_energy; ca.type_f = ta.type_f; ca.budget = p->d_budget;
  ca.G = p->G; ca.cells = cells; ca.n_share = m->n_share; ca.unit = mp.unit; ca.u_max = u_need;
  ca.types = mp.types;
  ca.energy = out->energy_j; ca.n_inst = out->n_inst; ca.f_index = out->f_index; ca.share = out->share;
  ca.ok = (int32_t*)(base + w.ok);
  if (!hip_ok(dyn_launch_mixed_combine(ca, s), "mixed combine launch")) return DYN_E_DEVICE;
  if (!hip_ok(dyn_launch_window_totals(ca.ok, out->energy_j, t->n_window, p->G, out->window_energy_j,
                                       out->window_infeasible, s),
              "window totals launch"))
    return DYN_E_DEVICE;
  return DYN_OK;
}

namespace {
struct PathWs { size_t layout, order, seg, transition, pred, kend, min_cost, min_k, exits, total; };
PathWs path_ws_layout(int32_t n_window, int32_t G, int32_t K, int32_t n_layout) {
  PathWs w;
  size_t off = 0;
  w.layout = off; off += align256((size_t)K * sizeof(int32_t));
  w.order = off; off += align256((size_t)K * sizeof(int32_t));
  w.seg = off; off += align256(((size_t)n_layout + 1) * sizeof(int32_t));
  w.transition = off; off += align256((size_t)n_layout * n_layout * sizeof(double));
  w.pred = off; off += align256((size_t)G * n_window * n_layout * sizeof(int32_t));
  w.kend = off; off += align256((size_t)G * n_window * sizeof(int32_t));
  const size_t per_layout = n_layout <= DYN_WAVE ? (size_t)G * n_window * n_layout : 0;   // the wave-per-class route only
  w.min_cost = off; off += align256(per_layout * sizeof(double));
  w.min_k = off; off += align256(per_layout * sizeof(int32_t));
  w.exits = off; off += align256((size_t)G * dyn_path_runs(n_window) * DYN_PATH_STATES * sizeof(int32_t));
  w.total = off;
  return w;
}
}  // namespace

size_t dyn_select_path_workspace(int32_t n_window, int32_t n_class, int32_t n_config, int32_t n_layout) {
  if (n_window < 1 || n_class < 1 || n_config < 1 || n_layout < 1) return 0;
  return path_ws_layout(n_window, n_class, n_config, n_layout).total;
}

int dyn_select_path(dyn_profile* p, const dyn_space* space, const dyn_config* cfg, int32_t K, const dyn_objective* o,
                    const dyn_transitions* tr, int32_t n_window, double window_s, const dyn_path_selection* out,
                    void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!p || !space || !o || !tr || !out || !workspace) { dyn_set_error("profile, space, objective, transitions, out or workspace is NULL"); return DYN_E_NULL; }
  if (!space->energy_j || !space->flags) { dyn_set_error("space->energy_j or space->flags is NULL"); return DYN_E_NULL; }
  if (!out->sel || !out->sel_energy_j || !out->path_cost || !out->window_energy_j || !out->window_infeasible) { dyn_set_error("an output array is NULL"); return DYN_E_NULL; }
  if (!tr->layout || !tr->transition_j) { dyn_set_error("layout or transition_j is NULL"); return DYN_E_NULL; }
  if (n_window < 1) { dyn_set_error("n_window < 1"); return DYN_E_SHAPE; }
  if (!in_scale(window_s)) { dyn_set_error("window_s must lie in [1e-100, 1e100]"); return DYN_E_RANGE; }
  if (!isfinite(o->idle_cost_weight)) { dyn_set_error("idle_cost_weight is not finite"); return DYN_E_NOTFINITE; }
  if (o->idle_cost_weight < 0.0) { dyn_set_error("idle_cost_weight must be >= 0"); return DYN_E_RANGE; }
  if ((int64_t)n_window * p->G >= ((int64_t)1 << 30)) { dyn_set_error("n_window * classes must stay below 2^30"); return DYN_E_SHAPE; }
  if (K < 1 || K > DYN_MAX_CONFIGS) { dyn_set_error("K=%d outside [1, %d]", K, DYN_MAX_CONFIGS); return DYN_E_SHAPE; }
  if (tr->n_layout < 1 || tr->n_layout > DYN_MAX_LAYOUTS) { dyn_set_error("n_layout=%d outside [1, %d]", tr->n_layout, DYN_MAX_LAYOUTS); return DYN_E_SHAPE; }
  if (!dyn_path_fits(K, tr->n_layout)) {
    dyn_set_error("K=%d, n_layout=%d: beyond 64 layouts the per-class state (K <= %d candidates, n_layout^2 overheads) must fit in LDS", K, tr->n_layout, DYN_PATH_MAX_CONFIGS);
    return DYN_E_SHAPE;
  }
  for (int k = 0; k < K; ++k)
    if (tr->layout[k] < 0 || tr->layout[k] >= tr->n_layout) { dyn_set_error("layout[%d]=%d outside [0, %d)", k, tr->layout[k], tr->n_layout); return DYN_E_RANGE; }
  for (int64_t i = 0; i < (int64_t)tr->n_layout * tr->n_layout; ++i) {
    if (!isfinite(tr->transition_j[i])) { dyn_set_error("transition_j[%lld] is not finite", (long long)i); return DYN_E_NOTFINITE; }
    if (tr->transition_j[i] < 0.0) { dyn_set_error("transition_j[%lld] < 0", (long long)i); return DYN_E_RANGE; }
  }
  int rc = check_device(p);
  if (rc) return rc;
  const PathWs w = path_ws_layout(n_window, p->G, K, tr->n_layout);
  if (((uintptr_t)workspace & 255) || workspace_bytes < w.total) {
    dyn_set_error("workspace misaligned or too small (%zu < %zu)", workspace_bytes, w.total);
    return DYN_E_WORKSPACE;
  }
  hipStream_t s = (hipStream_t)hip_stream;
  if ((rc = prepare_configs(p, cfg, K, s)) != DYN_OK) return rc;
  char* base = (char*)workspace;
  // candidates sorted by (layout, index): a layout's candidates are then one contiguous run
  std::vector<int32_t> order(K), seg(tr->n_layout + 1, 0);
  for (int k = 0; k < K; ++k) seg[tr->layout[k] + 1] += 1;
  for (int l = 0; l < tr->n_layout; ++l) seg[l + 1] += seg[l];
  {
    std::vector<int32_t> fill(seg.begin(), seg.end() - 1);
    for (int k = 0; k < K; ++k) order[fill[tr->layout[k]]++] = k;
  }
  // the host tables are cached in the profile handle like the candidate list: nothing is uploaded (and nothing waits)
  // while they stay the same
  if ((rc = cache_upload(p->path_layout_host, p->d_path_layout, tr->layout, (size_t)K, s, "copy layout")) != DYN_OK ||
      (rc = cache_upload(p->path_order_host, p->d_path_order, order.data(), (size_t)K, s, "copy order")) != DYN_OK ||
      (rc = cache_upload(p->path_seg_host, p->d_path_seg, seg.data(), seg.size(), s, "copy segments")) != DYN_OK ||
      (rc = cache_upload(p->path_trans_host, p->d_path_trans, tr->transition_j, (size_t)tr->n_layout * tr->n_layout, s, "copy transitions")) != DYN_OK)
    return rc;
  PathArgs a;
  a.energy = space->energy_j; a.flags = space->flags; a.cfg = p->d_cfg; a.K = K; a.pw0 = p->d_pw0;
  a.G = p->G; a.n_tp_f = p->n_tp * p->n_f; a.n_window = n_window; a.window_s = window_s; a.idle_w = o->idle_cost_weight;
  a.n_layout = tr->n_layout; a.layout = p->d_path_layout; a.transition = p->d_path_trans;
  a.order = p->d_path_order; a.seg_start = p->d_path_seg;
  a.pred = (int32_t*)(base + w.pred); a.kend = (int32_t*)(base + w.kend);
  a.min_cost = (double*)(base + w.min_cost); a.min_k = (int32_t*)(base + w.min_k); a.exits = (int32_t*)(base + w.exits);
  a.sel = out->sel; a.sel_energy = out->sel_energy_j; a.path_cost = out->path_cost;
  if (!hip_ok(dyn_launch_path(a, s), "path launch")) return DYN_E_DEVICE;
  if (!hip_ok(dyn_launch_window_totals(out->sel, out->sel_energy_j, n_window, p->G, out->window_energy_j,
                                       out->window_infeasible, s),
              "window totals launch"))
    return DYN_E_DEVICE;
  return DYN_OK;
}

size_t dyn_account_workspace(int32_t n_window) {
  if (n_window < 1) return 0;
  return 256 + 2 * align256((size_t)n_window * sizeof(double));
}

int dyn_account(dyn_profile* p, const int32_t* sel, const double* window_energy_j, const dyn_config* cfg, int32_t K,
                int32_t n_window, double window_s, const dyn_rates* r, const dyn_accounting* out, void* workspace,
                size_t workspace_bytes, void* hip_stream) {
  if (!p || !sel || !window_energy_j || !r || !out || !workspace) { dyn_set_error("profile, sel, window_energy_j, rates, out or workspace is NULL"); return DYN_E_NULL; }
  if (!r->carbon_g_per_kwh || !out->gpus || !out->gpu_cost || !out->energy_cost || !out->carbon_g || !out->totals) { dyn_set_error("an array is NULL"); return DYN_E_NULL; }
  if (n_window < 1 || r->gpus_per_server < 1) { dyn_set_error("n_window or gpus_per_server < 1"); return DYN_E_SHAPE; }
  if (!in_scale(window_s)) { dyn_set_error("window_s must lie in [1e-100, 1e100]"); return DYN_E_RANGE; }
  if (!isfinite(r->gpu_hour_price) || !isfinite(r->kwh_price)) { dyn_set_error("a price is not finite"); return DYN_E_NOTFINITE; }
  int rc = check_device(p);
  if (rc) return rc;
  const size_t per = align256((size_t)n_window * sizeof(double));
  if (((uintptr_t)workspace & 255) || workspace_bytes < 256 + 2 * per) { dyn_set_error("workspace misaligned or too small"); return DYN_E_WORKSPACE; }
  hipStream_t s = (hipStream_t)hip_stream;
  if ((rc = prepare_configs(p, cfg, K, s)) != DYN_OK) return rc;
  char* base = (char*)workspace;
  hipLaunchKernelGGL(init_word_header_kernel, dim3(1), dim3(1), 0, s, (WsHeader*)base, 0u);
  if (!hip_ok(hipGetLastError(), "launch")) return DYN_E_DEVICE;
  AccountArgs a;
  a.sel = sel; a.window_energy = window_energy_j; a.carbon = r->carbon_g_per_kwh;
  a.cfg = p->d_cfg; a.K = K; a.G = p->G; a.n_window = n_window; a.window_s = window_s;
  a.gpu_hour_price = r->gpu_hour_price; a.kwh_price = r->kwh_price; a.gpus_per_server = r->gpus_per_server;
  a.gpus = out->gpus; a.gpu_cost = out->gpu_cost; a.energy_cost = out->energy_cost; a.carbon_g = out->carbon_g; a.totals = out->totals;
  a.hours = (double*)(base + 256); a.servers = (double*)(base + 256 + per);
  a.status = &((WsHeader*)base)->status;
  if (!hip_ok(dyn_launch_account(a, s), "account launch")) return DYN_E_DEVICE;
  return DYN_OK;
}

namespace {
struct HierWs {
  EvalWs coarse;                 // header .. cstat of the window-level aggregation (first: its header is the workspace's)
  size_t fine_base; EvalWs fine; // the tick-level aggregation, offsets relative to fine_base
  size_t tp, lay_n, lay_tp, tick_energy, tick_viol, served_c, served_f, keep, fwd, lay_energy, lay_flags, sel_energy, path, total;
};
HierWs hier_ws_layout(int64_t cells, int32_t n_tick, int32_t n_tp, int32_t n_layout) {
  HierWs w;
  w.coarse = dyn_eval_ws_layout(cells, 1);
  w.fine_base = w.coarse.part;
  w.fine = dyn_eval_ws_layout(cells * n_tick, 1);
  size_t off = w.fine_base + w.fine.part;
  const size_t c = (size_t)std::max<int64_t>(cells, 1);
  w.tp = off; off += align256((size_t)n_tp * 4);
  w.lay_n = off; off += align256((size_t)n_layout * 4);
  w.lay_tp = off; off += align256((size_t)n_layout * 4);
  w.tick_energy = off; off += align256(c * n_tick * 8);
  w.tick_viol = off; off += align256(c * n_tick);
  // only used with the fragmentation rule (keep holds at most one entry per cell)
  w.served_c = off; off += align256(c * 8);
  w.served_f = off; off += align256(c * n_tick * 8);
  w.keep = off; off += align256(c * 8);
  w.fwd = off; off += align256(c * 8);
  // only used with a transition table: the layouts' space and the sequence selection's own workspace
  w.lay_energy = off; off += align256(c * n_layout * 8);
  w.lay_flags = off; off += align256(c * n_layout);
  w.sel_energy = off; off += align256(c * 8);
  w.path = off;
  w.total = off;
  return w;
}
}  // namespace

size_t dyn_hierarchy_workspace(int32_t n_window, int32_t n_tick, int32_t n_class, int32_t n_layout) {
  if (n_window < 1 || n_tick < 1 || n_class < 1 || n_layout < 1) return 0;
  return hier_ws_layout((int64_t)n_window * n_class, n_tick, 64, n_layout).total +
         path_ws_layout(n_window, n_class, n_layout, n_layout).total;
}

int dyn_hierarchy(dyn_profile* p, const dyn_trace_view* tc, const dyn_trace_view* tf, int32_t n_tick, const dyn_controllers* c,
                  const dyn_objective* o, const dyn_hierarchy_out* out, void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!p || !tc || !tf || !c || !o || !out || !workspace) { dyn_set_error("an argument is NULL"); return DYN_E_NULL; }
  if (!out->nodes || !out->layout_sel || !out->f_sel || !out->energy_j || !out->violations || !out->window_energy_j || !out->window_infeasible) { dyn_set_error("an output array is NULL"); return DYN_E_NULL; }
  if (!c->lay_n || !c->lay_tp_index) { dyn_set_error("the layout list is NULL"); return DYN_E_NULL; }
  if (n_tick < 1 || tc->n_window < 1 || tf->n_window != (int64_t)tc->n_window * n_tick || tc->n_req != tf->n_req || tc->n_req < 0 || tc->n_req >= ((int64_t)1 << 31)) {
    dyn_set_error("the tick-level trace must hold n_window * n_tick windows of the same requests");
    return DYN_E_SHAPE;
  }
  if (!tc->cell_off || !tf->cell_off || (tc->n_req > 0 && (!tc->in_tok || !tc->out_tok || !tf->in_tok || !tf->out_tok))) { dyn_set_error("a trace array is NULL"); return DYN_E_NULL; }
  if (!in_scale(tf->window_s)) { dyn_set_error("tick length must lie in [1e-100, 1e100]"); return DYN_E_RANGE; }
  if (c->epoch_windows < 1 || c->gpus_per_node < 1 || c->n_layout < 1) { dyn_set_error("epoch_windows, gpus_per_node or n_layout < 1"); return DYN_E_SHAPE; }
  if (c->n_layout > DYN_MAX_CONFIGS || (c->transition_j && c->n_layout > DYN_MAX_LAYOUTS)) { dyn_set_error("n_layout=%d: at most %d layouts, %d with a transition table", c->n_layout, DYN_MAX_CONFIGS, DYN_MAX_LAYOUTS); return DYN_E_SHAPE; }
  if (p->n_tp > 64 || p->G > 4096) { dyn_set_error("dyn_hierarchy takes profiles of up to 64 TP degrees and 4096 classes"); return DYN_E_SHAPE; }
  if (c->tp_ref_index < 0 || c->tp_ref_index >= p->n_tp || c->f_ref_index < 0 || c->f_ref_index >= p->n_f) { dyn_set_error("reference configuration outside the profile"); return DYN_E_RANGE; }
  for (int l = 0; l < c->n_layout; ++l)
    if (c->lay_n[l] < 1 || c->lay_tp_index[l] < 0 || c->lay_tp_index[l] >= p->n_tp) { dyn_set_error("layout %d is not valid", l); return DYN_E_RANGE; }
  const int64_t cells = (int64_t)tc->n_window * p->G, fine_cells = cells * n_tick;
  if (fine_cells >= ((int64_t)1 << 30)) { dyn_set_error("n_window * n_tick * classes must stay below 2^30"); return DYN_E_SHAPE; }
  int rc;
  if ((rc = check_device(p)) != DYN_OK) return rc;
  const HierWs w = hier_ws_layout(cells, n_tick, 64, c->n_layout);
  const PathWs pw = path_ws_layout(tc->n_window, p->G, c->n_layout, c->n_layout);
  if (c->transition_j) {
    if (!out->path_cost) { dyn_set_error("out->path_cost is NULL"); return DYN_E_NULL; }
    if (!dyn_path_fits(c->n_layout, c->n_layout)) {
      dyn_set_error("n_layout=%d: the sequence selection's per-class state does not fit in LDS", c->n_layout);
      return DYN_E_SHAPE;
    }
    for (int64_t i = 0; i < (int64_t)c->n_layout * c->n_layout; ++i) {
      if (!isfinite(c->transition_j[i])) { dyn_set_error("transition_j[%lld] is not finite", (long long)i); return DYN_E_NOTFINITE; }
      if (c->transition_j[i] < 0.0) { dyn_set_error("transition_j[%lld] < 0", (long long)i); return DYN_E_RANGE; }
    }
  }
  if (((uintptr_t)workspace & 255) || workspace_bytes < w.total + pw.total) { dyn_set_error("workspace misaligned or too small (%zu < %zu)", workspace_bytes, w.total + pw.total); return DYN_E_WORKSPACE; }
  hipStream_t s = (hipStream_t)hip_stream;
  if ((rc = prepare_objective(p, o, s)) != DYN_OK) return rc;
  char* base = (char*)workspace;
  char* fb = base + w.fine_base;
  char* pb = base + w.path;
  // the controllers' small tables are cached in the profile handle (uploaded again only when they change)
  if (c->transition_j &&
      (rc = cache_upload(p->hier_trans_host, p->d_hier_trans, c->transition_j, (size_t)c->n_layout * c->n_layout, s, "copy transitions")) != DYN_OK)
    return rc;
  if ((rc = cache_upload(p->lay_n_host, p->d_lay_n, c->lay_n, (size_t)c->n_layout, s, "copy layouts")) != DYN_OK ||
      (rc = cache_upload(p->lay_tp_host, p->d_lay_tp, c->lay_tp_index, (size_t)c->n_layout, s, "copy layouts")) != DYN_OK)
    return rc;
  const double window_s = (double)n_tick * tf->window_s;
  // tick level first: the window-level aggregation then (re)writes the workspace's header
  if (!hip_ok(dyn_launch_cell_aggregate(tf->in_tok, tf->out_tok, tf->cell_off, tf->n_req, fine_cells, tf->window_s, o->pct_num, o->pct_den,
                                        (int64_t*)(fb + w.fine.tin), (int64_t*)(fb + w.fine.tout), (int32_t*)(fb + w.fine.in_p99),
                                        (CellRec*)(fb + w.fine.rec), (uint8_t*)(fb + w.fine.cstat), (WsHeader*)(fb + w.fine.header), s), "cell aggregate launch") ||
      !hip_ok(dyn_launch_cell_aggregate(tc->in_tok, tc->out_tok, tc->cell_off, tc->n_req, cells, window_s, o->pct_num, o->pct_den,
                                        (int64_t*)(base + w.coarse.tin), (int64_t*)(base + w.coarse.tout), (int32_t*)(base + w.coarse.in_p99),
                                        (CellRec*)(base + w.coarse.rec), (uint8_t*)(base + w.coarse.cstat), (WsHeader*)(base + w.coarse.header), s), "cell aggregate launch"))
    return DYN_E_DEVICE;
  HierArgs a;
  a.tab = p->d_tab; a.ml = p->d_ml; a.gridpack = p->d_gridpack; a.jstart = p->d_jstart; a.tstart = p->d_tstart; a.thr = p->d_thr; a.n_bucket = p->n_bucket; a.bucket_scale = p->bucket_scale;
  a.G = p->G; a.n_tp = p->n_tp; a.n_f = p->n_f; a.n_rho = p->n_rho; a.tp = p->d_tp;
  a.slo_ttft = p->d_slo_ttft; a.slo_tbt = p->d_slo_tbt;
  a.rec_c = (const CellRec*)(base + w.coarse.rec); a.rec_f = (const CellRec*)(fb + w.fine.rec);
  a.cstat_c = (const uint8_t*)(base + w.coarse.cstat); a.cstat_f = (const uint8_t*)(fb + w.fine.cstat); a.status = &((WsHeader*)(base + w.coarse.header))->status;
  a.n_window = tc->n_window; a.n_tick = n_tick; a.tick_s = tf->window_s; a.window_s = window_s;
  a.epoch_windows = c->epoch_windows; a.n_epoch = (tc->n_window + c->epoch_windows - 1) / c->epoch_windows;
  a.tp_ref = c->tp_ref_index; a.f_ref = c->f_ref_index; a.gpus_per_node = c->gpus_per_node;
  a.n_layout = c->n_layout; a.lay_n = p->d_lay_n; a.lay_tp = p->d_lay_tp;
  a.nodes = out->nodes; a.layout_sel = out->layout_sel; a.f_sel = out->f_sel; a.energy = out->energy_j; a.violations = out->violations;
  a.win_energy = out->window_energy_j; a.win_inf = out->window_infeasible;
  a.lay_energy = c->transition_j ? (double*)(base + w.lay_energy) : nullptr;
  a.lay_flags = c->transition_j ? (uint8_t*)(base + w.lay_flags) : nullptr;
  a.tick_energy = (double*)(base + w.tick_energy); a.tick_viol = (uint8_t*)(base + w.tick_viol);
  a.served_c = a.served_f = a.keep = a.fwd = nullptr;
  if (c->spill) {
    a.served_c = (double*)(base + w.served_c); a.served_f = (double*)(base + w.served_f);
    a.keep = out->keep ? out->keep : (double*)(base + w.keep); a.fwd = (double*)(base + w.fwd);
    if (!hip_ok(dyn_launch_hier_spill(a, s), "hierarchy launch")) return DYN_E_DEVICE;
  }
  if (!hip_ok(dyn_launch_hier_shard(a, p->single_point, s), "hierarchy launch")) return DYN_E_DEVICE;
  if (c->transition_j) {        // the windows' layouts chosen together; overwrites layout_sel
    PathArgs pa;
    pa.energy = a.lay_energy; pa.flags = a.lay_flags; pa.cfg = nullptr; pa.K = c->n_layout; pa.pw0 = p->d_pw0;
    pa.G = p->G; pa.n_tp_f = p->n_tp * p->n_f; pa.n_window = tc->n_window; pa.window_s = window_s; pa.idle_w = 0.0;
    // one candidate per layout: the layout map, the sorted order and the segment starts are all the identity
    pa.n_layout = c->n_layout; pa.layout = p->d_ident; pa.transition = p->d_hier_trans;
    pa.order = p->d_ident; pa.seg_start = p->d_ident;
    pa.pred = (int32_t*)(pb + pw.pred); pa.kend = (int32_t*)(pb + pw.kend);
    pa.min_cost = (double*)(pb + pw.min_cost); pa.min_k = (int32_t*)(pb + pw.min_k); pa.exits = (int32_t*)(pb + pw.exits);
    pa.sel = out->layout_sel; pa.sel_energy = (double*)(base + w.sel_energy); pa.path_cost = out->path_cost;
    if (!hip_ok(dyn_launch_path(pa, s), "path launch")) return DYN_E_DEVICE;
  }
  if (!hip_ok(dyn_launch_hier_ticks(a, p->single_point, s), "hierarchy launch")) return DYN_E_DEVICE;
  return DYN_OK;
}

int dyn_cell_stats(const void* workspace, size_t workspace_bytes, int32_t n_window, int32_t n_class,
                   int64_t* tok_in, int64_t* tok_out, int32_t* in_p99, void* hip_stream) {
  if (!workspace) { dyn_set_error("workspace is NULL"); return DYN_E_NULL; }
  if (n_window < 1 || n_class < 1) { dyn_set_error("n_window or n_class < 1"); return DYN_E_SHAPE; }
  const int64_t cells = (int64_t)n_window * n_class;
  const EvalWs w = dyn_eval_ws_layout(cells, 1);   // the aggregates precede everything that depends on K
  if (((uintptr_t)workspace & 255) || workspace_bytes < w.total) { dyn_set_error("workspace misaligned or too small"); return DYN_E_WORKSPACE; }
  hipStream_t s = (hipStream_t)hip_stream;
  const char* base = (const char*)workspace;
  if (tok_in && !hip_ok(hipMemcpyAsync(tok_in, base + w.tin, cells * 8, hipMemcpyDeviceToDevice, s), "copy")) return DYN_E_DEVICE;
  if (tok_out && !hip_ok(hipMemcpyAsync(tok_out, base + w.tout, cells * 8, hipMemcpyDeviceToDevice, s), "copy")) return DYN_E_DEVICE;
  if (in_p99 && !hip_ok(hipMemcpyAsync(in_p99, base + w.in_p99, cells * 4, hipMemcpyDeviceToDevice, s), "copy")) return DYN_E_DEVICE;
  return DYN_OK;
}

int dyn_workspace_status(const void* workspace, void* hip_stream, uint32_t* status) {
  if (!workspace || !status) { dyn_set_error("workspace or status is NULL"); return DYN_E_NULL; }
  hipStream_t s = (hipStream_t)hip_stream;
  WsHeader h;
  if (!hip_ok(hipMemcpyAsync(&h, workspace, sizeof(h), hipMemcpyDeviceToHost, s), "copy status")) return DYN_E_DEVICE;
  if (!hip_ok(hipStreamSynchronize(s), "hipStreamSynchronize")) return DYN_E_DEVICE;
  if (h.kind == DYN_WS_KIND_CELLS) {
    // evaluation workspace: OR the per-cell status bytes into the header word, then read it
    if (h.cells < 1 || h.cells >= ((int64_t)1 << 30)) { dyn_set_error("workspace header is corrupt"); return DYN_E_WORKSPACE; }
    const EvalWs w = dyn_eval_ws_layout(h.cells, 1);
    const char* base = (const char*)workspace;
    uint32_t* word = (uint32_t*)const_cast<char*>(base + w.header);
    const int blocks = (int)std::min<int64_t>(1024, (h.cells + 255) / 256);
    hipLaunchKernelGGL(or_cell_status_kernel, dim3(blocks), dim3(256), 0, s, (const uint8_t*)(base + w.cstat), h.cells, word);
    if (!hip_ok(hipGetLastError(), "launch")) return DYN_E_DEVICE;
    if (!hip_ok(hipMemcpyAsync(&h, workspace, sizeof(h), hipMemcpyDeviceToHost, s), "copy status")) return DYN_E_DEVICE;
    if (!hip_ok(hipStreamSynchronize(s), "hipStreamSynchronize")) return DYN_E_DEVICE;
  } else if (h.kind != DYN_WS_KIND_WORD) {
    dyn_set_error("workspace holds no result yet");
    return DYN_E_WORKSPACE;
  }
  *status = h.status;
  return DYN_OK;
}

int dyn_select_config(dyn_profile* p, const dyn_space* space, const dyn_config* cfg, int32_t K,
                      const dyn_objective* o, int32_t n_window, double window_s, const dyn_selection* out,
                      void* hip_stream) {
  if (!p || !space || !o || !out) { dyn_set_error("profile, space, objective or out is NULL"); return DYN_E_NULL; }
  if (!space->energy_j || !space->flags) { dyn_set_error("space->energy_j or space->flags is NULL"); return DYN_E_NULL; }
  if (!out->sel || !out->sel_energy_j || !out->sel_cost || !out->window_energy_j || !out->window_infeasible) { dyn_set_error("an output array is NULL"); return DYN_E_NULL; }
  if (n_window < 1) { dyn_set_error("n_window < 1"); return DYN_E_SHAPE; }
  if (!in_scale(window_s)) { dyn_set_error("window_s must lie in [1e-100, 1e100]"); return DYN_E_RANGE; }
  if (!isfinite(o->idle_cost_weight)) { dyn_set_error("idle_cost_weight is not finite"); return DYN_E_NOTFINITE; }
  if (o->idle_cost_weight < 0.0) { dyn_set_error("idle_cost_weight must be >= 0"); return DYN_E_RANGE; }
  if ((int64_t)n_window * p->G >= ((int64_t)1 << 30)) { dyn_set_error("n_window * classes must stay below 2^30"); return DYN_E_SHAPE; }
  int rc = check_device(p);
  if (rc) return rc;
  hipStream_t s = (hipStream_t)hip_stream;
  if ((rc = prepare_configs(p, cfg, K, s)) != DYN_OK) return rc;
  SelectArgs a;
  a.energy = space->energy_j; a.flags = space->flags; a.cfg = p->d_cfg; a.K = K; a.pw0 = p->d_pw0;
  a.G = p->G; a.n_tp_f = p->n_tp * p->n_f; a.n_window = n_window; a.window_s = window_s;
  a.idle_w = o->idle_cost_weight;
  a.sel = out->sel; a.sel_energy = out->sel_energy_j; a.sel_cost = out->sel_cost;
  a.win_energy = out->window_energy_j; a.win_inf = out->window_infeasible;
  if (!hip_ok(dyn_launch_select(a, s), "select launch")) return DYN_E_DEVICE;
  return DYN_OK;
}

int dyn_timing_enable(int on, int32_t max_launches) {
  g_timing = false;
  for (TimerPool& t : g_timers) {
    for (hipEvent_t e : t.start) (void)hipEventDestroy(e);
    for (hipEvent_t e : t.stop) (void)hipEventDestroy(e);
    t.start.clear(); t.stop.clear(); t.used = 0;
  }
  if (!on) return DYN_OK;
  if (max_launches < 1 || max_launches > (1 << 20)) { dyn_set_error("max_launches out of range"); return DYN_E_RANGE; }
  for (TimerPool& t : g_timers) {
    t.start.resize(max_launches); t.stop.resize(max_launches);
    for (int i = 0; i < max_launches; ++i)
      if (!hip_ok(hipEventCreate(&t.start[i]), "hipEventCreate") || !hip_ok(hipEventCreate(&t.stop[i]), "hipEventCreate"))
        return DYN_E_DEVICE;
  }
  g_timing = true;
  return DYN_OK;
}

int dyn_timing_reset(void) {
  for (TimerPool& t : g_timers) t.used = 0;
  return DYN_OK;
}

int dyn_timing_read(int32_t kernel, double* total_ms, int64_t* launches) {
  if (!total_ms || !launches) { dyn_set_error("output pointer is NULL"); return DYN_E_NULL; }
  if (kernel < 0 || kernel >= DYN_K_COUNT) { dyn_set_error("unknown kernel id %d", kernel); return DYN_E_RANGE; }
  TimerPool& t = g_timers[kernel];
  double sum = 0.0;
  for (int i = 0; i < t.used; ++i) {
    if (!hip_ok(hipEventSynchronize(t.stop[i]), "hipEventSynchronize")) return DYN_E_DEVICE;
    float ms = 0.f;
    if (!hip_ok(hipEventElapsedTime(&ms, t.start[i], t.stop[i]), "hipEventElapsedTime")) return DYN_E_DEVICE;
    sum += ms;
  }
  *total_ms = sum;
  *launches = t.used;
  return DYN_OK;
}

}  // extern "C"
