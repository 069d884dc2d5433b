// The three controllers of Section IV-B, top down, on the aggregates of a trace:
//   hier_shard_kernel   scale-out/in and shard-up/down.  Per (window, class): the node count of the
//                       window's epoch = ceil(peak load of the epoch / largest profiled load of one node
//                       at the reference configuration), at least one; then the layout (instances, TP)
//                       of least energy at the reference frequency among those that fit the nodes' GPUs
//                       and meet the SLO;
//   hier_freq_kernel    scale-up/down: per tick the frequency of least power among those that meet the
//                       SLO under the tick's load (the reference frequency, counted, if none does);
//   hier_sum_kernel     energy of a (window, class) = its ticks' energies added in time order; window
//                       totals = the classes' energies added in class order.
//   hier_spill_*        (fragmentation rule only) before the others: per epoch, classes in ascending order,
//                       the node counts, the fraction of its arriving load every pool keeps and the loads the
//                       pools serve in every window and tick once the rest has been forwarded to the next class.
// The tables stay in global memory (they are a few hundred KB and live in L2; copying a class's tables
// to LDS per block was measured to cost more than the look-ups it serves).  Two things matter instead:
// threads of a block share the class, so that a wave's gathers fall into a few table rows, and the
// frequency kernel takes its look-ups four at a time, level by level (capacity -> bucket -> grid points
// and table values), so that a thread waits for three rounds of loads per four frequencies, not twelve.
#include <algorithm>

#include "dyn_hier.h"
#include "dyn_device.h"

namespace {

constexpr int kShardWaves = 4;          // (window, class) cells per block of the shard kernel, one wave each
constexpr int kFreqThreads = 256;
constexpr int kFreqChunk = 4;           // look-ups a thread of the frequency kernel has in flight
constexpr int kSpillLds = 48 * 1024;    // an epoch's window loads are staged in LDS when they fit in this
constexpr int kSpillRun = 8;            // classes whose tick loads a thread fetches ahead of the chain

struct Looked { double pf, tb, pw; bool ov; };

// The load axis (grid points, reciprocal spacings, bucket index) is the same for every class and small.  The
// frequency kernel keeps a copy in LDS, which takes six of a look-up's thirteen gathers off the vector memory
// path (37 -> 30 us for a day of ticks); the shard kernel, whose blocks live for one look-up per lane, reads it
// from global memory (with the copy its blocks start a memory round trip later: 30 us instead of 26 us).
// LDS: [padded grid and reciprocal spacings 2 n_rho + 3] [SINGLE: grid point per bucket n_bucket + 1] [bucket index, 16-bit]
struct Axis { const double* pack; const double* thr; const uint16_t* js; const int32_t* js_global; };   // js == nullptr: js_global
template <bool SINGLE>
__device__ __forceinline__ Axis global_axis(const HierArgs& a) {
  Axis x;
  x.pack = a.gridpack; x.thr = a.thr; x.js = nullptr; x.js_global = SINGLE ? a.tstart : a.jstart;
  return x;
}
template <bool SINGLE>
__device__ __forceinline__ Axis stage_axis(const HierArgs& a, double* smem) {
  double* s_pack = smem;
  double* s_thr = s_pack + 2 * a.n_rho + 3;
  uint16_t* s_js = (uint16_t*)(s_thr + (SINGLE ? a.n_bucket + 1 : 0));
  for (int i = threadIdx.x; i < 2 * a.n_rho + 3; i += blockDim.x) s_pack[i] = a.gridpack[i];
  for (int i = threadIdx.x; i <= a.n_bucket; i += blockDim.x) {
    s_js[i] = (uint16_t)(SINGLE ? a.tstart[i] : a.jstart[i]);
    if (SINGLE) s_thr[i] = a.thr[i];
  }
  __syncthreads();
  Axis x;
  x.pack = s_pack; x.thr = s_thr; x.js = s_js; x.js_global = nullptr;
  return x;
}

// Bracket of a clamped load fraction rc: largest grid index i <= n_rho-2 with grid[i] <= rc.
// SINGLE: no bucket holds more than one interior grid point; the index is then the number of interior
// points in lower buckets plus one comparison with the bucket's own point.
template <bool SINGLE>
__device__ __forceinline__ int bracket(const HierArgs& a, const Axis& x, double rc) {
  const double* grid = x.pack + 1;
  const int b = min((int)(fmax(rc, 0.0) * a.bucket_scale), a.n_bucket);
  const int j0 = x.js ? (int)x.js[b] : x.js_global[b];
  if (SINGLE) return j0 + (rc >= x.thr[b] ? 1 : 0);
  int j = j0;
  while (j > 0 && grid[j] > rc) --j;
  while (j < a.n_rho - 2 && grid[j + 1] <= rc) ++j;
  return j;
}

// Linear interpolation in table row `row` (class, TP, frequency) between grid points j and j+1.
__device__ __forceinline__ void interpolate(const HierArgs& a, const Axis& x, size_t row, int j, double rc, Looked* r) {
  const double* grid = x.pack + 1;
  const double* rinv = x.pack + a.n_rho + 3;                 // RN(1 / spacing)
  const double g0 = grid[j], g1 = grid[j + 1];
  const double t = div_by(rc - g0, g1 - g0, rinv[j]);
  const double omt = 1.0 - t;
  const double* v = a.tab + row * 3 * a.n_rho;
  r->pf = omt * v[j] + t * v[j + 1];
  r->tb = omt * v[a.n_rho + j] + t * v[a.n_rho + j + 1];
  r->pw = omt * v[2 * a.n_rho + j] + t * v[2 * a.n_rho + j + 1];
}

// Row (g, ti, f) at per-instance load `load / n`; values at the last grid point when the load is beyond it.
template <bool SINGLE>
__device__ __forceinline__ Looked look_up(const HierArgs& a, const Axis& x, int g, int ti, int f, double load, double n) {
  const size_t row = ((size_t)g * a.n_tp + ti) * a.n_f + f;
  const double rho = load / (n * a.ml[row]);
  const double rho_max = x.pack[a.n_rho];
  Looked r;
  r.ov = rho > rho_max;
  const double rc = r.ov ? rho_max : rho;
  interpolate(a, x, row, bracket<SINGLE>(a, x, rc), rc, &r);
  return r;
}

__device__ __forceinline__ double wave_max_f64(double v) {
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) v = fmax(v, __shfl_xor(v, d, DYN_WAVE));
  return v;
}

// Largest value of each row of 16 lanes, in all of the row's lanes (rotations by 1, 2, 4 and 8 lanes).
template <int CTRL>
__device__ __forceinline__ double dpp_f64(double v) {
  const uint64_t u = (uint64_t)__double_as_longlong(v);
  const uint32_t lo = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)u, CTRL, 0xF, 0xF, false);
  const uint32_t hi = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)(u >> 32), CTRL, 0xF, 0xF, false);
  return __longlong_as_double((long long)(((uint64_t)hi << 32) | lo));
}
__device__ __forceinline__ double row_max_f64(double v) {
  v = fmax(v, dpp_f64<0x121>(v));
  v = fmax(v, dpp_f64<0x122>(v));
  v = fmax(v, dpp_f64<0x124>(v));
  return fmax(v, dpp_f64<0x128>(v));
}

// One wave per (window, class); lanes stride the layouts; the lowest index wins equal energies.
template <bool SINGLE>
__global__ __launch_bounds__(kShardWaves* DYN_WAVE) void hier_shard_kernel(HierArgs a) {
  const Axis x = global_axis<SINGLE>(a);
  const int lane = threadIdx.x & (DYN_WAVE - 1);
  const int64_t cell = (int64_t)blockIdx.x * kShardWaves + threadIdx.x / DYN_WAVE;
  if (cell >= (int64_t)a.n_window * a.G) return;
  const int w = (int)(cell / a.G), g = (int)(cell % a.G);
  const CellRec rec = a.rec_c[cell];
  if (lane == 0 && a.cstat_c[cell]) atomicOr(a.status, (uint32_t)a.cstat_c[cell]);
  // scale-out/in: the epoch's peak load over the capacity of one node at the reference configuration
  const int e = w / a.epoch_windows;
  const int e0 = e * a.epoch_windows, e1 = min(a.n_window, e0 + a.epoch_windows);
  int32_t nodes;
  double load = rec.load;
  if (a.served_c) {                                          // fragmentation rule: both come from the spill kernels
    nodes = a.nodes[(size_t)e * a.G + g];
    load = a.served_c[cell];
  } else {
    double peak = 0.0;
    for (int i = e0 + lane; i < e1; i += DYN_WAVE) peak = fmax(peak, a.rec_c[(size_t)i * a.G + g].load);
    peak = wave_max_f64(peak);
    const int inst = max(1, a.gpus_per_node / a.tp[a.tp_ref]);
    const double ml_node = ((double)inst * a.ml[((size_t)g * a.n_tp + a.tp_ref) * a.n_f + a.f_ref]) * a.gridpack[a.n_rho];
    const double q = ceil(peak / ml_node);
    nodes = q < 1.0 ? 1 : (q > 2147483647.0 ? 2147483647 : (int32_t)q);
    if (w == e0 && lane == 0) a.nodes[(size_t)e * a.G + g] = nodes;
  }
  const int64_t budget = (int64_t)nodes * a.gpus_per_node;
  // shard-up/down at the reference frequency
  const double slo_t = a.slo_ttft[g], slo_b = a.slo_tbt[g];
  double best_e = __builtin_inf();
  int best = 0x7FFFFFFF;
  for (int l = lane; l < a.n_layout; l += DYN_WAVE) {
    const int n = a.lay_n[l], ti = a.lay_tp[l];
    bool ok = (int64_t)n * a.tp[ti] <= budget;
    double en = __builtin_inf();
    if (ok) {
      const Looked r = look_up<SINGLE>(a, x, g, ti, a.f_ref, load, (double)n);
      ok = !(r.ov || rec.xp99 * r.pf > slo_t || r.tb * rec.nonempty > slo_b);
      en = ((double)n * r.pw) * a.window_s;
    }
    if (a.lay_energy) {                                      // the sequence selection takes it from here
      a.lay_energy[(size_t)cell * a.n_layout + l] = en;
      a.lay_flags[(size_t)cell * a.n_layout + l] = ok ? (uint8_t)DYN_F_FEASIBLE : (uint8_t)0;
    }
    if (ok && (best == 0x7FFFFFFF || en < best_e)) { best_e = en; best = l; }   // l ascends per lane
  }
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) {
    const double oe = __shfl_xor(best_e, d, DYN_WAVE);
    const int ol = __shfl_xor(best, d, DYN_WAVE);
    if (ol != 0x7FFFFFFF && (best == 0x7FFFFFFF || oe < best_e || (oe == best_e && ol < best))) { best_e = oe; best = ol; }
  }
  if (lane == 0) a.layout_sel[cell] = best == 0x7FFFFFFF ? -1 : best;
}

// One thread per (window, tick, class).  A block stays within one class: its threads then read the same
// few table rows, and a wave's look-up touches a handful of cache lines instead of one per lane.
template <bool SINGLE>
__global__ __launch_bounds__(kFreqThreads) void hier_freq_kernel(HierArgs a) {
  extern __shared__ double s_axis[];
  const Axis x = stage_axis<SINGLE>(a, s_axis);
  const int g = blockIdx.x % a.G;
  const int64_t wt = (int64_t)(blockIdx.x / a.G) * kFreqThreads + threadIdx.x;   // window * n_tick + tick
  if (wt >= (int64_t)a.n_window * a.n_tick) return;
  const int64_t f = wt * a.G + g;
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
  const double load = a.served_f ? a.served_f[f] : rec.load;
  const int n = a.lay_n[l], ti = a.lay_tp[l];
  const double nd = (double)n;
  const double slo_t = a.slo_ttft[g], slo_b = a.slo_tbt[g];
  const double rho_max = x.pack[a.n_rho];
  const size_t row0 = ((size_t)g * a.n_tp + ti) * a.n_f;
  int bf = -1;
  double bp = __builtin_inf(), pw_ref = 0.0;
  for (int f0 = 0; f0 < a.n_f; f0 += kFreqChunk) {
    double rc[kFreqChunk];
    bool ov[kFreqChunk];
    int j[kFreqChunk];
    Looked r[kFreqChunk];
#pragma unroll
    for (int c = 0; c < kFreqChunk; ++c) {                   // level 1: capacities
      const int fi = min(f0 + c, a.n_f - 1);
      const double rho = load / (nd * a.ml[row0 + fi]);
      ov[c] = rho > rho_max;
      rc[c] = ov[c] ? rho_max : rho;
    }
#pragma unroll
    for (int c = 0; c < kFreqChunk; ++c) j[c] = bracket<SINGLE>(a, x, rc[c]);   // level 2: bucket index
#pragma unroll
    for (int c = 0; c < kFreqChunk; ++c)                     // level 3: grid points and table values
      interpolate(a, x, row0 + min(f0 + c, a.n_f - 1), j[c], rc[c], &r[c]);
#pragma unroll
    for (int c = 0; c < kFreqChunk; ++c) {                   // ascending frequency: the lowest wins equal powers
      const int fi = f0 + c;
      if (fi >= a.n_f) break;
      if (fi == a.f_ref) pw_ref = r[c].pw;
      if (ov[c] || rec.xp99 * r[c].pf > slo_t || r[c].tb * rec.nonempty > slo_b) continue;
      if (bf < 0 || r[c].pw < bp) { bf = fi; bp = r[c].pw; }
    }
  }
  uint8_t viol = 0;
  if (bf < 0) {                                              // nothing admissible: the reference frequency, counted
    bp = pw_ref;
    bf = a.f_ref;
    viol = 1;
  }
  a.f_sel[f] = bf;
  a.tick_energy[f] = (nd * bp) * a.tick_s;
  a.tick_viol[f] = viol;
}

// Fragmentation rule, window level.  One wave per epoch, lanes stride the epoch's windows, classes one after the
// other: what a class forwards arrives at the next.  STAGED (at most one window per lane and the epoch's loads fit in
// LDS): loads and node capacities are copied to LDS up front, the forwarded load stays in a register and the results
// per class are collected in LDS, so the chain over the classes waits for LDS and a short wave reduction per class,
// never for global memory.
template <bool STAGED>
__global__ __launch_bounds__(DYN_WAVE) void hier_spill_epoch_kernel(HierArgs a) {
  extern __shared__ double s_spill[];                        // STAGED: loads [windows of the epoch][G], capacity, its reciprocal, keep [G] each, nodes [G]
  const int e = blockIdx.x, lane = threadIdx.x;
  const int e0 = e * a.epoch_windows, e1 = min(a.n_window, e0 + a.epoch_windows);
  const int G = a.G;
  const int inst = max(1, a.gpus_per_node / a.tp[a.tp_ref]);
  const double rho_max = a.gridpack[a.n_rho];
  const double guard = 1.0 - 0x1p-40;
  double* s_load = s_spill;
  double* s_cap = s_spill + (size_t)min(a.epoch_windows, a.n_window) * G;
  double* s_rcap = s_cap + G;                                // RN(1 / capacity)
  double* s_keep = s_rcap + G;
  int32_t* s_nodes = (int32_t*)(s_keep + G);
  if (STAGED) {
    for (int i = lane; i < (e1 - e0) * G; i += DYN_WAVE) s_load[i] = a.rec_c[(size_t)e0 * G + i].load;
    for (int g = lane; g < G; g += DYN_WAVE) {
      s_cap[g] = ((double)inst * a.ml[((size_t)g * a.n_tp + a.tp_ref) * a.n_f + a.f_ref]) * rho_max;
      s_rcap[g] = 1.0 / s_cap[g];
    }
    __syncthreads();
  } else {
    for (int i = e0 + lane; i < e1; i += DYN_WAVE) a.fwd[i] = 0.0;
  }
  const bool mine = e0 + lane < e1;                          // STAGED: this lane's window
  double fwd = 0.0;
  for (int g = 0; g < G; ++g) {
    double arrive = 0.0, peak = 0.0, ml_node;
    if (STAGED) {
      if (mine) arrive = s_load[lane * G + g] + fwd;
      peak = row_max_f64(arrive);                            // lanes without a window hold 0
      if (e1 - e0 > 16) peak = fmax(peak, __shfl_xor(peak, 16, DYN_WAVE));
      if (e1 - e0 > 32) peak = fmax(peak, __shfl_xor(peak, 32, DYN_WAVE));
      ml_node = s_cap[g];
    } else {
      for (int i = e0 + lane; i < e1; i += DYN_WAVE) peak = fmax(peak, a.rec_c[(size_t)i * G + g].load + a.fwd[i]);
      peak = wave_max_f64(peak);
      ml_node = ((double)inst * a.ml[((size_t)g * a.n_tp + a.tp_ref) * a.n_f + a.f_ref]) * rho_max;
    }
    const double q = STAGED ? div_by(peak, ml_node, s_rcap[g]) : peak / ml_node;
    const double fl = floor(q);
    double keep = 1.0;
    int32_t nodes;
    if (g < G - 1 && fl >= 1.0 && fl < q && fl < 2147483647.0) {
      nodes = (int32_t)fl;
      keep = ((fl * ml_node) / peak) * guard;
    } else {
      const double up = ceil(q);
      nodes = up < 1.0 ? 1 : (up > 2147483647.0 ? 2147483647 : (int32_t)up);
    }
    if (STAGED) {
      if (lane == 0) { s_nodes[g] = nodes; s_keep[g] = keep; }
      if (mine) {
        const double served = keep * arrive;
        s_load[lane * G + g] = served;
        fwd = arrive - served;
      }
    } else {
      if (lane == 0) {
        a.nodes[(size_t)e * G + g] = nodes;
        a.keep[(size_t)e * G + g] = keep;
      }
      for (int i = e0 + lane; i < e1; i += DYN_WAVE) {
        const double arr = a.rec_c[(size_t)i * G + g].load + a.fwd[i];
        const double served = keep * arr;
        a.served_c[(size_t)i * G + g] = served;
        a.fwd[i] = arr - served;                             // read again by this lane only
      }
    }
  }
  if (STAGED) {
    __syncthreads();
    for (int i = lane; i < (e1 - e0) * G; i += DYN_WAVE) a.served_c[(size_t)e0 * G + i] = s_load[i];
    for (int g = lane; g < G; g += DYN_WAVE) {
      a.nodes[(size_t)e * G + g] = s_nodes[g];
      a.keep[(size_t)e * G + g] = s_keep[g];
    }
  }
}

// Fragmentation rule, tick level: one thread per tick walks the classes with the kept fractions of the tick's epoch;
// the loads of kSpillRun classes are fetched together, ahead of the chain that links them.
__global__ __launch_bounds__(DYN_WAVE) void hier_spill_tick_kernel(HierArgs a) {
  const int64_t wt = (int64_t)blockIdx.x * DYN_WAVE + threadIdx.x;
  if (wt >= (int64_t)a.n_window * a.n_tick) return;
  const int e = (int)(wt / a.n_tick) / a.epoch_windows;
  const double* keep = a.keep + (size_t)e * a.G;
  const CellRec* rec = a.rec_f + (size_t)wt * a.G;
  double* served_f = a.served_f + (size_t)wt * a.G;
  double fwd = 0.0;
  for (int g0 = 0; g0 < a.G; g0 += kSpillRun) {
    double own[kSpillRun], k[kSpillRun];
#pragma unroll
    for (int c = 0; c < kSpillRun; ++c) {
      const int g = min(g0 + c, a.G - 1);
      own[c] = rec[g].load;
      k[c] = keep[g];
    }
#pragma unroll
    for (int c = 0; c < kSpillRun; ++c) {
      if (g0 + c >= a.G) break;
      const double arr = own[c] + fwd;
      const double served = k[c] * arr;
      served_f[g0 + c] = served;
      fwd = arr - served;
    }
  }
}

// One block per window: thread g adds the ticks of (window, g) in time order; thread 0 then adds the
// classes in class order.
__global__ __launch_bounds__(64) void hier_sum_kernel(HierArgs a) {
  extern __shared__ double s_e[];                            // [G] energy, NaN marks "no layout"
  const int w = blockIdx.x;
  for (int g = threadIdx.x; g < a.G; g += blockDim.x) {
    const size_t cell = (size_t)w * a.G + g;
    const bool has = a.layout_sel[cell] >= 0;
    double e = 0.0;
    int32_t v = 0;
    for (int q = 0; q < a.n_tick; ++q) {                     // time order
      const size_t f = ((size_t)w * a.n_tick + q) * a.G + g;
      e += a.tick_energy[f];
      v += a.tick_viol[f];
    }
    a.energy[cell] = has ? e : __builtin_inf();
    a.violations[cell] = has ? v : 0;
    s_e[g] = has ? e : __builtin_nan("");
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    double e = 0.0;
    int32_t ninf = 0;
    for (int g = 0; g < a.G; ++g) {
      const double x = s_e[g];
      if (x == x) e += x; else ++ninf;
    }
    a.win_energy[w] = e;
    a.win_inf[w] = ninf;
  }
}

size_t axis_lds(const HierArgs& a, bool single) {         // at most 4097 buckets: 42 KB
  return ((size_t)2 * a.n_rho + 3 + (single ? a.n_bucket + 1 : 0)) * sizeof(double) + ((size_t)a.n_bucket + 1) * sizeof(uint16_t) + 8;
}

}  // namespace

hipError_t dyn_launch_hier_spill(const HierArgs& a, hipStream_t s) {
  const int64_t ticks = (int64_t)a.n_window * a.n_tick;
  const size_t lds = ((size_t)std::min(a.epoch_windows, a.n_window) * a.G + 3 * (size_t)a.G) * sizeof(double) + (size_t)a.G * sizeof(int32_t);
  DynTimed timed(DYN_K_HIER, s);
  if (a.epoch_windows <= DYN_WAVE && lds <= (size_t)kSpillLds)
    hipLaunchKernelGGL(hier_spill_epoch_kernel<true>, dim3((unsigned)a.n_epoch), dim3(DYN_WAVE), lds, s, a);
  else
    hipLaunchKernelGGL(hier_spill_epoch_kernel<false>, dim3((unsigned)a.n_epoch), dim3(DYN_WAVE), 0, s, a);
  hipLaunchKernelGGL(hier_spill_tick_kernel, dim3((unsigned)((ticks + DYN_WAVE - 1) / DYN_WAVE)), dim3(DYN_WAVE), 0, s, a);
  return hipGetLastError();
}

hipError_t dyn_launch_hier_shard(const HierArgs& a, bool single_point, hipStream_t s) {
  const int64_t cells = (int64_t)a.n_window * a.G;
  const unsigned shard_blocks = (unsigned)((cells + kShardWaves - 1) / kShardWaves);
  DynTimed timed(DYN_K_HIER, s);
  if (single_point) hipLaunchKernelGGL(hier_shard_kernel<true>, dim3(shard_blocks), dim3(kShardWaves * DYN_WAVE), 0, s, a);
  else hipLaunchKernelGGL(hier_shard_kernel<false>, dim3(shard_blocks), dim3(kShardWaves * DYN_WAVE), 0, s, a);
  return hipGetLastError();
}

hipError_t dyn_launch_hier_ticks(const HierArgs& a, bool single_point, hipStream_t s) {
  const int64_t ticks = (int64_t)a.n_window * a.n_tick;
  const unsigned freq_blocks = (unsigned)(((ticks + kFreqThreads - 1) / kFreqThreads) * a.G);
  DynTimed timed(DYN_K_HIER, s);
  if (single_point) hipLaunchKernelGGL(hier_freq_kernel<true>, dim3(freq_blocks), dim3(kFreqThreads), axis_lds(a, true), s, a);
  else hipLaunchKernelGGL(hier_freq_kernel<false>, dim3(freq_blocks), dim3(kFreqThreads), axis_lds(a, false), s, a);
  hipLaunchKernelGGL(hier_sum_kernel, dim3((unsigned)a.n_window), dim3(64), (size_t)a.G * sizeof(double), s, a);
  return hipGetLastError();
}
