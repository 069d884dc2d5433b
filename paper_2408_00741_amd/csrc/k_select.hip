// Least-cost feasible configuration per cell (Section IV-B "Scale-up/down": filter what
// violates the SLO, then take the minimum energy), one wavefront per cell striding the
// configuration axis, then the per-window totals of the objective (Eq. 1 sums over the
// pools).  cost = energy + idle_cost_weight * n * power(load 0) * window.
#include "dyn_mixed.h"

namespace {

constexpr int kWavesPerBlock = 4;
constexpr int32_t kNone = 0x7FFFFFFF;

__global__ __launch_bounds__(kWavesPerBlock* DYN_WAVE) void select_kernel(SelectArgs a) {
  const int lane = threadIdx.x & (DYN_WAVE - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / DYN_WAVE);
  const int64_t cells = (int64_t)a.n_window * a.G;
  const int64_t cell = (int64_t)blockIdx.x * kWavesPerBlock + wave;
  if (cell >= cells) return;
  const int g = (int)(cell % a.G);
  const double* e_row = a.energy + (size_t)cell * a.K;
  const uint8_t* f_row = a.flags + (size_t)cell * a.K;
  const double* pw0_row = a.pw0 + (size_t)g * a.n_tp_f;
  const bool idle = a.idle_w != 0.0;

  double best_cost = __builtin_inf(), best_e = __builtin_inf();
  int32_t best_k = kNone;
  for (int k = lane; k < a.K; k += DYN_WAVE) {
    const double e = e_row[k];
    const uint32_t fl = f_row[k];
    double cost = e;
    if (idle) {
      const DevCfg c = a.cfg[k];
      const double pw0 = (c.u != 0.0) ? (1.0 - c.u) * pw0_row[c.row_lo] + c.u * pw0_row[c.row_hi]
                                      : pw0_row[c.row_lo];
      cost = e + a.idle_w * ((c.nd * pw0) * a.window_s);
    }
    // first feasible candidate, or strictly cheaper than the best so far (k ascending per lane)
    if ((fl & DYN_F_FEASIBLE) && (best_k == kNone || cost < best_cost)) {
      best_cost = cost;
      best_e = e;
      best_k = k;
    }
  }
  // wave minimum of (cost, k): lower cost wins, equal cost -> lower index; lanes without a
  // feasible candidate carry k = kNone and lose every comparison against a real candidate
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) {
    const double oc = __shfl_xor(best_cost, d, DYN_WAVE);
    const double oe = __shfl_xor(best_e, d, DYN_WAVE);
    const int32_t ok = __shfl_xor(best_k, d, DYN_WAVE);
    const bool take = (ok != kNone) && (best_k == kNone || oc < best_cost || (oc == best_cost && ok < best_k));
    if (take) {
      best_cost = oc;
      best_e = oe;
      best_k = ok;
    }
  }
  if (lane == 0) {
    a.sel[cell] = best_k == kNone ? -1 : best_k;
    a.sel_energy[cell] = best_e;    // +inf when nothing is feasible
    a.sel_cost[cell] = best_cost;
  }
}

__global__ void window_totals_kernel(const int32_t* __restrict__ sel, const double* __restrict__ sel_energy,
                                     int32_t n_window, int32_t G, double* __restrict__ win_energy,
                                     int32_t* __restrict__ win_inf) {
  const int w = blockIdx.x * blockDim.x + threadIdx.x;
  if (w >= n_window) return;
  double e = 0.0;
  int32_t ninf = 0;
  for (int g = 0; g < G; ++g) {  // fixed order: g ascending
    const size_t c = (size_t)w * G + g;
    if (sel[c] >= 0) e += sel_energy[c]; else ++ninf;
  }
  win_energy[w] = e;
  win_inf[w] = ninf;
}

// Fused path: every cell has n_used partial records in ascending configuration order; a
// strict "<" scan keeps the lowest index among equal costs.  One block per window when the
// classes of a window fit a block: the class results go through LDS and thread 0 adds them
// in class order.
__device__ __forceinline__ void scan_partials(const SelPart* __restrict__ p, int n, double* bc, double* be, int32_t* bk) {
  double c = __builtin_inf(), e = __builtin_inf();
  int32_t k = -1;
  int i = 0;
  if (n <= 16) {                 // the usual case: every record in flight at once, compared in candidate order
    SelPart q[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      q[j].k = -1;
      if (j < n) q[j] = p[j];
    }
#pragma unroll
    for (int j = 0; j < 16; ++j)
      if (q[j].k >= 0 && (k < 0 || q[j].cost < c)) { c = q[j].cost; e = q[j].energy; k = q[j].k; }
    *bc = c; *be = e; *bk = k;
    return;
  }
  for (; i + 4 <= n; i += 4) {   // four independent loads in flight, compared in candidate order
    const SelPart q0 = p[i], q1 = p[i + 1], q2 = p[i + 2], q3 = p[i + 3];
    if (q0.k >= 0 && (k < 0 || q0.cost < c)) { c = q0.cost; e = q0.energy; k = q0.k; }
    if (q1.k >= 0 && (k < 0 || q1.cost < c)) { c = q1.cost; e = q1.energy; k = q1.k; }
    if (q2.k >= 0 && (k < 0 || q2.cost < c)) { c = q2.cost; e = q2.energy; k = q2.k; }
    if (q3.k >= 0 && (k < 0 || q3.cost < c)) { c = q3.cost; e = q3.energy; k = q3.k; }
  }
  for (; i < n; ++i) {
    const SelPart q = p[i];
    if (q.k >= 0 && (k < 0 || q.cost < c)) { c = q.cost; e = q.energy; k = q.k; }
  }
  *bc = c; *be = e; *bk = k;
}

__global__ __launch_bounds__(256) void finish_kernel(FinishArgs a) {
  extern __shared__ double s_e[];          // [G] selected energy, NaN marks "no feasible configuration"
  const int w = blockIdx.x;
  for (int g = threadIdx.x; g < a.G; g += blockDim.x) {
    const size_t cell = (size_t)w * a.G + g;
    double bc, be;
    int32_t bk;
    scan_partials(a.part + cell * (size_t)a.n_wslot, a.n_used, &bc, &be, &bk);
    a.sel[cell] = bk;
    a.sel_energy[cell] = be;
    a.sel_cost[cell] = bc;
    s_e[g] = bk >= 0 ? be : __builtin_nan("");
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    double e = 0.0;
    int32_t ninf = 0;
    int g = 0;
    for (; g + 8 <= a.G; g += 8) {         // operands first, then the additions in class order
      double v[8];
#pragma unroll
      for (int q = 0; q < 8; ++q) v[q] = s_e[g + q];
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        if (v[q] == v[q]) e += v[q]; else ++ninf;
      }
    }
    for (; g < a.G; ++g) {
      const double v = s_e[g];
      if (v == v) e += v; else ++ninf;
    }
    a.win_energy[w] = e;
    a.win_inf[w] = ninf;
  }
}

__global__ __launch_bounds__(256) void finish_cells_kernel(FinishArgs a) {   // classes beyond one block's LDS
  const int64_t cells = (int64_t)a.n_window * a.G;
  const int64_t cell = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (cell >= cells) return;
  double bc, be;
  int32_t bk;
  scan_partials(a.part + (size_t)cell * a.n_wslot, a.n_used, &bc, &be, &bk);
  a.sel[cell] = bk;
  a.sel_energy[cell] = be;
  a.sel_cost[cell] = bc;
}

}  // namespace

hipError_t dyn_launch_finish(const FinishArgs& a, hipStream_t s) {
  if (a.G <= 4096) {
    DynTimed timed(DYN_K_SELECT, s);
    hipLaunchKernelGGL(finish_kernel, dim3((unsigned)a.n_window), dim3(a.G <= 64 ? 64 : 256), (size_t)a.G * sizeof(double),
                       s, a);
    return hipGetLastError();
  }
  const int64_t cells = (int64_t)a.n_window * a.G;
  {
    DynTimed timed(DYN_K_SELECT, s);
    hipLaunchKernelGGL(finish_cells_kernel, dim3((unsigned)((cells + 255) / 256)), dim3(256), 0, s, a);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  DynTimed timed(DYN_K_TOTALS, s);
  hipLaunchKernelGGL(window_totals_kernel, dim3((unsigned)((a.n_window + 127) / 128)), dim3(128), 0, s, a.sel,
                     a.sel_energy, a.n_window, a.G, a.win_energy, a.win_inf);
  return hipGetLastError();
}

hipError_t dyn_launch_window_totals(const int32_t* sel, const double* sel_energy, int32_t n_window, int32_t G,
                                    double* win_energy, int32_t* win_inf, hipStream_t s) {
  DynTimed timed(DYN_K_TOTALS, s);
  hipLaunchKernelGGL(window_totals_kernel, dim3((unsigned)((n_window + 127) / 128)), dim3(128), 0, s, sel, sel_energy,
                     n_window, G, win_energy, win_inf);
  return hipGetLastError();
}

hipError_t dyn_launch_select(const SelectArgs& a, hipStream_t s) {
  const int64_t cells = (int64_t)a.n_window * a.G;
  const int64_t blocks = (cells + kWavesPerBlock - 1) / kWavesPerBlock;
  hipError_t e;
  {
    DynTimed timed(DYN_K_SELECT, s);
    hipLaunchKernelGGL(select_kernel, dim3((unsigned)blocks), dim3(kWavesPerBlock * DYN_WAVE), 0, s, a);
    e = hipGetLastError();
  }
  if (e != hipSuccess) return e;
  DynTimed timed(DYN_K_TOTALS, s);
  hipLaunchKernelGGL(window_totals_kernel, dim3((unsigned)((a.n_window + 127) / 128)), dim3(128), 0, s,
                     a.sel, a.sel_energy, a.n_window, a.G, a.win_energy, a.win_inf);
  return hipGetLastError();
}
