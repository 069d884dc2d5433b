// The three controllers of Section IV-B, top down, on the aggregates of a trace:
//   hier_nodes_kernel   scale-out/in: nodes = ceil(peak load of the epoch / largest profiled load of one
//                       node at the reference configuration), at least one;
//   hier_shard_kernel   shard-up/down: per (window, class) the layout (instances, TP) of least energy at
//                       the reference frequency among those that fit the nodes' GPUs and meet the SLO;
//   hier_freq_kernel    scale-up/down: per tick the frequency of least power among those that meet the
//                       SLO under the tick's load (the reference frequency, counted, if none does);
//   hier_sum_kernel     energy of a (window, class) = its ticks' energies added in time order.
// Table look-ups read global memory: the work is a few million look-ups per call.
#include "dyn_hier.h"

namespace {

struct Looked { double pf, tb, pw; bool ov; };

// Tables of class g, row (ti, f), at per-instance load `load / n`: bracket = largest i with grid[i] <= x
// clamped to n_rho-2, linear in between; values at the last point when the load is beyond it.
__device__ __forceinline__ Looked look_up(const HierArgs& a, int g, int ti, int f, double load, double n) {
  const double ml = a.ml[((size_t)g * a.n_tp + ti) * a.n_f + f];
  const double rho = load / (n * ml);
  const double* rg = a.gridpack + 1;                         // gridpack = [-inf, grid, +inf, ...]
  const double rho_max = rg[a.n_rho - 1];
  Looked r;
  r.ov = rho > rho_max;
  const double rc = r.ov ? rho_max : rho;
  int j = a.jstart[min((int)(fmax(rc, 0.0) * a.bucket_scale), a.n_bucket)];
  while (j > 0 && rg[j] > rc) --j;
  while (j < a.n_rho - 2 && rg[j + 1] <= rc) ++j;
  const double t = (rc - rg[j]) / (rg[j + 1] - rg[j]);
  const double omt = 1.0 - t;
  const double* row = a.tab + (((size_t)g * a.n_tp + ti) * a.n_f + f) * 3 * a.n_rho;
  r.pf = omt * row[j] + t * row[j + 1];
  r.tb = omt * row[a.n_rho + j] + t * row[a.n_rho + j + 1];
  r.pw = omt * row[2 * a.n_rho + j] + t * row[2 * a.n_rho + j + 1];
  return r;
}

__global__ __launch_bounds__(128) void hier_nodes_kernel(HierArgs a) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= a.n_epoch * a.G) return;
  const int e = i / a.G, g = i - e * a.G;
  double peak = 0.0;
  const int w1 = min(a.n_window, (e + 1) * a.epoch_windows);
  for (int w = e * a.epoch_windows; w < w1; ++w) {
    const double l = a.rec_c[(size_t)w * a.G + g].load;
    if (l > peak) peak = l;
  }
  const int inst = max(1, a.gpus_per_node / a.tp[a.tp_ref]);
  const double rho_max = a.gridpack[a.n_rho];
  const double ml_node = ((double)inst * a.ml[((size_t)g * a.n_tp + a.tp_ref) * a.n_f + a.f_ref]) * rho_max;
  const double q = ceil(peak / ml_node);
  a.nodes[i] = q < 1.0 ? 1 : (q > 2147483647.0 ? 2147483647 : (int32_t)q);
}

// One wave per (window, class); lanes stride the layouts; the lowest index wins equal energies.
__global__ __launch_bounds__(256) void hier_shard_kernel(HierArgs a) {
  const int lane = threadIdx.x & (DYN_WAVE - 1);
  const int64_t cell = (int64_t)blockIdx.x * (blockDim.x / DYN_WAVE) + threadIdx.x / DYN_WAVE;
  if (cell >= (int64_t)a.n_window * a.G) return;
  const int w = (int)(cell / a.G), g = (int)(cell % a.G);
  const CellRec rec = a.rec_c[cell];
  if (lane == 0 && a.cstat_c[cell]) atomicOr(a.status, (uint32_t)a.cstat_c[cell]);
  const int64_t budget = (int64_t)a.nodes[(size_t)(w / a.epoch_windows) * a.G + g] * a.gpus_per_node;
  const double slo_t = a.slo_ttft[g], slo_b = a.slo_tbt[g];
  double best_e = __builtin_inf();
  int best = 0x7FFFFFFF;
  for (int l = lane; l < a.n_layout; l += DYN_WAVE) {
    const int n = a.lay_n[l], ti = a.lay_tp[l];
    if ((int64_t)n * a.tp[ti] > budget) continue;
    const Looked r = look_up(a, g, ti, a.f_ref, rec.load, (double)n);
    if (r.ov || rec.xp99 * r.pf > slo_t || r.tb * rec.nonempty > slo_b) continue;
    const double e = ((double)n * r.pw) * a.window_s;
    if (best == 0x7FFFFFFF || e < best_e) { best_e = e; best = l; }   // l ascends per lane
  }
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) {
    const double oe = __shfl_xor(best_e, d, DYN_WAVE);
    const int ol = __shfl_xor(best, d, DYN_WAVE);
    if (ol != 0x7FFFFFFF && (best == 0x7FFFFFFF || oe < best_e || (oe == best_e && ol < best))) { best_e = oe; best = ol; }
  }
  if (lane == 0) a.layout_sel[cell] = best == 0x7FFFFFFF ? -1 : best;
}

// One thread per (window, tick, class).
__global__ __launch_bounds__(128) void hier_freq_kernel(HierArgs a) {
  const int64_t f = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t fine_cells = (int64_t)a.n_window * a.n_tick * a.G;
  if (f >= fine_cells) return;
  const int g = (int)(f % a.G);
  const int64_t wt = f / a.G;
  const int w = (int)(wt / a.n_tick);
  if (a.cstat_f[f]) atomicOr(a.status, (uint32_t)a.cstat_f[f]);
  const int l = a.layout_sel[(size_t)w * a.G + g];
  if (l < 0) {
    a.f_sel[f] = -1;
    a.tick_energy[f] = 0.0;
    a.tick_viol[f] = 0;
    return;
  }
  const CellRec rec = a.rec_f[f];
  const int n = a.lay_n[l], ti = a.lay_tp[l];
  const double slo_t = a.slo_ttft[g], slo_b = a.slo_tbt[g];
  int bf = -1;
  double bp = __builtin_inf();
  for (int fi = 0; fi < a.n_f; ++fi) {
    const Looked r = look_up(a, g, ti, fi, rec.load, (double)n);
    if (r.ov || rec.xp99 * r.pf > slo_t || r.tb * rec.nonempty > slo_b) continue;
    if (bf < 0 || r.pw < bp) { bf = fi; bp = r.pw; }
  }
  uint8_t viol = 0;
  if (bf < 0) {                                              // nothing admissible: the reference frequency, counted
    bp = look_up(a, g, ti, a.f_ref, rec.load, (double)n).pw;
    bf = a.f_ref;
    viol = 1;
  }
  a.f_sel[f] = bf;
  a.tick_energy[f] = ((double)n * bp) * a.tick_s;
  a.tick_viol[f] = viol;
}

__global__ __launch_bounds__(128) void hier_sum_kernel(HierArgs a) {
  const int64_t cell = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (cell >= (int64_t)a.n_window * a.G) return;
  const int w = (int)(cell / a.G), g = (int)(cell % a.G);
  const bool has = a.layout_sel[cell] >= 0;
  double e = 0.0;
  int32_t v = 0;
  for (int q = 0; q < a.n_tick; ++q) {                       // time order
    const size_t f = ((size_t)w * a.n_tick + q) * a.G + g;
    e += a.tick_energy[f];
    v += a.tick_viol[f];
  }
  a.energy[cell] = has ? e : __builtin_inf();
  a.violations[cell] = has ? v : 0;
  a.ok[cell] = has ? 0 : -1;
}

}  // namespace

hipError_t dyn_launch_hierarchy(const HierArgs& a, hipStream_t s) {
  const int64_t cells = (int64_t)a.n_window * a.G, fine = cells * a.n_tick;
  DynTimed timed(DYN_K_HIER, s);
  hipLaunchKernelGGL(hier_nodes_kernel, dim3((unsigned)((a.n_epoch * a.G + 127) / 128)), dim3(128), 0, s, a);
  hipLaunchKernelGGL(hier_shard_kernel, dim3((unsigned)((cells + 3) / 4)), dim3(256), 0, s, a);
  hipLaunchKernelGGL(hier_freq_kernel, dim3((unsigned)((fine + 127) / 128)), dim3(128), 0, s, a);
  hipLaunchKernelGGL(hier_sum_kernel, dim3((unsigned)((cells + 127) / 128)), dim3(128), 0, s, a);
  return hipGetLastError();
}
