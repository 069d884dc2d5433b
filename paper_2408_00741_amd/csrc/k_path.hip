// Selection with transition overheads between consecutive windows (Section IV-B "Accounting for
// the overheads"; Table VI lists the re-sharding overheads between layouts): per class the
// sequence of configurations with the least  sum_w cost(w, k_w) + sum_w transition[layout(k_{w-1})]
// [layout(k_w)], found window by window.  The step from one window to the next is factored
// through the layouts: the cheapest way to arrive in layout l' is the least over source
// layouts l of (least total ending in l) + transition[l][l'] - equal to the least over all
// predecessors because rounded addition is monotone.
//
// Two routes.  Up to 64 layouts (further down): a parallel pre-pass reduces every (window, class) to
// its layouts' least costs, one block per class walks the windows with a lane per layout keeping least
// totals only, and the predecessors and the trace-back are taken afterwards, in parallel over the windows.
// More layouts (next): one block per class walks the windows in time order (the recurrence is
// sequential, so the time per window is what counts).  The candidates are visited in an order sorted by layout
// (built on the host), a fixed number per thread, their costs loaded one window ahead; per
// window: (A) totals of the sequences ending in each candidate, (B) one thread per layout takes
// the least of its contiguous run of candidates, (C) the cheapest arrival in every layout of
// the next window, the source layouts split over several threads per destination and the
// partial results combined; four LDS-only barriers per window.  Predecessors are kept per (window,
// destination layout) in the workspace and traced back at the end in runs of windows staged
// through LDS.
#include <algorithm>

#include "dyn_path.h"
static_assert(DYN_PATH_MAX_CONFIGS == 256 * 8, "candidates are held in registers, a fixed number per thread");

namespace {

constexpr int kThreads = 256;
constexpr int kRun = 64;                                   // windows traced back per LDS stage
constexpr int kPerThread = 8;                              // candidates per thread: K <= kThreads * kPerThread
constexpr int kParts = 4;                                  // threads per destination layout in the arrival step

// Barrier that orders LDS traffic only: it does not wait for the global loads of the next window's
// costs (or the predecessor stores), which __syncthreads() would do at every step of the walk.
__device__ __forceinline__ void lds_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// lower total wins, then the lower candidate index
__device__ __forceinline__ bool beats(double v, int k, double bv, int bk) { return v < bv || (v == bv && k < bk); }

// LDS: [V by sorted position: K doubles] [transition, transposed [to][from]: NL*NL doubles] [M: NL doubles]
//      [B: NL doubles] [partial arrivals: kParts*NL doubles] [arg: NL ints] [partial args: kParts*NL ints]
//      [segment starts: NL+1 ints] [trace-back stage: kRun*NL ints] [selection of the run: kRun ints]
//      [layout of candidate k: K u16] [candidate at sorted position: K u16]
__global__ __launch_bounds__(kThreads) void path_kernel(PathArgs a) {
  extern __shared__ double smem[];
  const int g = blockIdx.x;
  const int K = a.K, NL = a.n_layout, NW = a.n_window, G = a.G;
  double* s_v = smem;
  double* s_t = s_v + K;
  double* s_m = s_t + (NL + 1) * NL;
  double* s_b = s_m + NL;
  double* s_pv = s_b + NL;                                 // [kParts][NL + 1]
  int32_t* s_arg = (int32_t*)(s_pv + kParts * (NL + 1));
  int32_t* s_pk = s_arg + NL;                              // [kParts][NL + 1]
  int32_t* s_seg = s_pk + kParts * (NL + 1);               // [NL + 1]
  int32_t* s_bp = s_seg + NL + 1;                          // [kRun][NL]
  int32_t* s_sel = s_bp + kRun * NL;                       // [kRun]
  uint16_t* s_lay = (uint16_t*)(s_sel + kRun);             // [K]
  uint16_t* s_ord = s_lay + K;                             // [K]
  __shared__ int s_gap;

  for (int i = threadIdx.x; i < NL * NL; i += kThreads) {  // transposed: a destination's sources are contiguous
    const int from = i / NL, to = i - from * NL;
    s_t[to * NL + from] = a.transition[i];
  }
  for (int i = threadIdx.x; i < NL; i += kThreads) s_t[NL * NL + i] = 0.0;   // destination "end of the sequence"
  for (int k = threadIdx.x; k < K; k += kThreads) { s_lay[k] = (uint16_t)a.layout[k]; s_ord[k] = (uint16_t)a.order[k]; }
  for (int l = threadIdx.x; l <= NL; l += kThreads) s_seg[l] = a.seg_start[l];
  int32_t* bp = a.pred + (size_t)g * NW * NL;              // [NW][NL]: predecessor when window w is entered in layout l
  int32_t* kend = a.kend + (size_t)g * NW;                 // [NW]: best end of a sequence at w, -1 for a window without a feasible candidate
  const double* pw0_row = a.pw0 + (size_t)g * a.n_tp_f;
  const double inf = __builtin_inf();
  __syncthreads();

  // this thread's candidates: sorted positions p = threadIdx.x + i * kThreads
  int my_k[kPerThread], my_l[kPerThread];
  double idle_k[kPerThread];                               // idle term (0 adds nothing)
#pragma unroll
  for (int i = 0; i < kPerThread; ++i) {
    const int p = threadIdx.x + i * kThreads;
    my_k[i] = p < K ? (int)s_ord[p] : -1;
    my_l[i] = p < K ? (int)s_lay[my_k[i]] : 0;
    idle_k[i] = 0.0;
    if (p < K && a.idle_w != 0.0) {
      const DevCfg cf = a.cfg[my_k[i]];
      const double pw0 = (cf.u != 0.0) ? (1.0 - cf.u) * pw0_row[cf.row_lo] + cf.u * pw0_row[cf.row_hi] : pw0_row[cf.row_lo];
      idle_k[i] = a.idle_w * ((cf.nd * pw0) * a.window_s);
    }
  }
  // cost of this thread's candidates in window w (+inf where not feasible)
  auto load_costs = [&](int w, double (&c)[kPerThread]) {
    const size_t row = ((size_t)w * G + g) * K;
#pragma unroll
    for (int i = 0; i < kPerThread; ++i) {
      c[i] = inf;
      if (my_k[i] >= 0 && w < NW) {                        // both loads are issued before either is looked at
        const uint8_t fl = a.flags[row + my_k[i]];
        const double e = a.energy[row + my_k[i]];
        c[i] = (fl & DYN_F_FEASIBLE) ? e + idle_k[i] : inf;
      }
    }
  };
  // arrival step: thread (destination ld, part) takes the source layouts ls = part, part + n_part, ...
  const int n_part = (NL + 1) * kParts <= kThreads ? kParts : ((NL + 1) * 2 <= kThreads ? 2 : 1);
  const int c_ld = threadIdx.x % (NL + 1), c_part = threadIdx.x / (NL + 1);
  const bool c_on = c_part < n_part;
  const bool keeper = threadIdx.x == NL;                   // combines the "end" destination and keeps the class's total

  double total = 0.0, prev_end = 0.0;                      // keeper only
  bool first = true, prev_gap = true;
  double cur[kPerThread], nxt[kPerThread];
  load_costs(0, cur);
  for (int w = 0; w < NW; ++w) {
    load_costs(w + 1, nxt);                                // in flight while this window is processed
    // (A) totals of the sequences that end in window w with each candidate
#pragma unroll
    for (int i = 0; i < kPerThread; ++i) {
      const int p = threadIdx.x + i * kThreads;
      if (p < K) s_v[p] = (first || !(cur[i] < inf)) ? cur[i] : s_b[my_l[i]] + cur[i];
    }
    lds_barrier();
    // (B) least total per layout, lowest candidate among equals (a layout's candidates ascend with the position)
    for (int l = threadIdx.x; l < NL; l += kThreads) {
      double bv = inf;
      int bk = 0x7FFFFFFF;
      const int p1 = s_seg[l + 1];
#pragma unroll 4
      for (int p = s_seg[l]; p < p1; ++p) {
        const double v = s_v[p];
        if (v < bv) { bv = v; bk = (int)s_ord[p]; }
      }
      s_m[l] = bv;
      s_arg[l] = bk;
    }
    lds_barrier();
    // (C) cheapest arrival in every layout of the next window and where it comes from; destination NL stands
    // for "the sequence ends here" (no transition): the window's best end
    if (c_on) {
      double bv = inf;
      int bk = 0x7FFFFFFF;
      const double* trow = s_t + c_ld * NL;                // row NL of the transposed table is all zero
#pragma unroll 4
      for (int ls = c_part; ls < NL; ls += n_part) {
        const double cand = s_m[ls] + trow[ls];            // +inf: nothing ends in ls
        const int ak = s_arg[ls];
        if (beats(cand, ak, bv, bk)) { bv = cand; bk = ak; }
      }
      s_pv[c_part * (NL + 1) + c_ld] = bv;
      s_pk[c_part * (NL + 1) + c_ld] = bk;
    }
    lds_barrier();
    if (threadIdx.x <= NL) {
      double bv = s_pv[threadIdx.x];
      int bk = s_pk[threadIdx.x];
      for (int q = 1; q < n_part; ++q) {
        const double v = s_pv[q * (NL + 1) + threadIdx.x];
        const int k = s_pk[q * (NL + 1) + threadIdx.x];
        if (beats(v, k, bv, bk)) { bv = v; bk = k; }
      }
      if (threadIdx.x < NL) {
        s_b[threadIdx.x] = bv;                             // read by (A) of the next window, after the barrier below
        if (w + 1 < NW) bp[(size_t)(w + 1) * NL + threadIdx.x] = bk;   // not read if this window turns out to have no end
      } else {                                             // the keeper of the class's total
        const bool gap_w = !(bv < inf);
        s_gap = gap_w ? 1 : 0;
        kend[w] = gap_w ? -1 : bk;
        if (gap_w && !prev_gap) total += prev_end;         // the sequence before the gap is complete
        prev_end = bv;
        prev_gap = gap_w;
      }
    }
    lds_barrier();
    const bool gap = s_gap != 0;
    first = gap;
#pragma unroll
    for (int i = 0; i < kPerThread; ++i) cur[i] = nxt[i];
  }
  if (keeper) {
    if (!prev_gap) total += prev_end;
    a.path_cost[g] = total;
  }
  // make this block's predecessor records visible to its own later loads
  __threadfence();
  __syncthreads();

  // trace back, a run of windows at a time from the end; carry = candidate chosen in the window after the run
  int carry = -1;                                          // thread 0 only: -1 = the next window starts a sequence
  for (int hi = NW; hi > 0; hi -= kRun) {
    const int lo = hi > kRun ? hi - kRun : 0;
    // predecessor records of the windows lo+1 .. hi (row i = window lo+1+i; window NW does not exist)
    const int n_row = (hi < NW ? hi : NW - 1) - lo;
    for (int i = threadIdx.x; i < n_row * NL; i += kThreads)
      s_bp[i] = __hip_atomic_load(&bp[(size_t)(lo + 1) * NL + i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    for (int i = threadIdx.x; i < hi - lo; i += kThreads)
      s_sel[i] = __hip_atomic_load(&kend[lo + i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    if (threadIdx.x == 0) {
      for (int w = hi - 1; w >= lo; --w) {
        const int ke = s_sel[w - lo];
        int k;
        if (ke < 0) k = -1;                                // no feasible candidate in this window
        else if (carry < 0) k = ke;                        // last window of a sequence: its best end
        else k = s_bp[(w - lo) * NL + s_lay[carry]];       // predecessor of the next window's choice
        s_sel[w - lo] = k;
        carry = k;
      }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < hi - lo; i += kThreads) {
      const int k = s_sel[i];
      const size_t cell = (size_t)(lo + i) * G + g;
      a.sel[cell] = k;
      a.sel_energy[cell] = k >= 0 ? a.energy[cell * K + k] : inf;
    }
    __syncthreads();
  }
}


// ---- up to 64 layouts ----------------------------------------------------------------------------
// The step through the layouts needs, per window, only the least cost of every layout and the
// candidate that has it (adding a layout's arrival total to its candidates' costs keeps their
// order: rounded addition is monotone).  Those are independent of the recurrence:
// path_min_kernel takes them for all windows at once.  The recurrence itself only needs minima:
// path_chain_kernel walks the windows with one lane per layout and keeps, per (window, layout), the
// least total of the sequences that end there.  Which source and candidate reach a minimum is not part
// of the recurrence; path_pred_kernel recomputes the same rounded sums from the stored totals for all
// windows in parallel and records the predecessors (least total, then lowest candidate), and
// the two path_trace kernels follow them back, all runs of windows at once.  What the walk costs is the instructions one window's step takes
// in the block's waves (they share the four SIMDs of one compute unit), so the step holds nothing else:
// global memory is touched a chunk of windows at a time and a source's total is a lane read.
constexpr int kChainChunk = 16;                            // windows per visit to global memory
constexpr int kChainWaves = 8;                             // measured on a day of windows and 48 layouts: 4 waves 811 us, 8 waves 740 us, 16 waves 788 us for the whole selection
constexpr int kEndMark = -2;                               // kend: a sequence ends in this window (before path_pred_kernel fills in its best end)

// thread = (cell, layout): least cost among the layout's candidates, lowest candidate among equals
__global__ __launch_bounds__(256) void path_min_kernel(PathArgs a) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int NL = a.n_layout, K = a.K;
  if (i >= (int64_t)a.n_window * a.G * NL) return;
  const int64_t cell = i / NL;
  const int l = (int)(i - cell * NL);
  const int g = (int)(cell % a.G);
  const double* pw0_row = a.pw0 + (size_t)g * a.n_tp_f;
  const size_t row = (size_t)cell * K;
  double bv = __builtin_inf();
  int bk = 0x7FFFFFFF;
  const int p1 = a.seg_start[l + 1];
  for (int p = a.seg_start[l]; p < p1; ++p) {               // candidates of a layout ascend with the position
    const int k = a.order[p];
    const uint8_t fl = a.flags[row + k];
    double c = a.energy[row + k];
    if (a.idle_w != 0.0) {
      const DevCfg cf = a.cfg[k];
      const double pw0 = (cf.u != 0.0) ? (1.0 - cf.u) * pw0_row[cf.row_lo] + cf.u * pw0_row[cf.row_hi] : pw0_row[cf.row_lo];
      c = c + a.idle_w * ((cf.nd * pw0) * a.window_s);
    }
    if ((fl & DYN_F_FEASIBLE) && c < bv) { bv = c; bk = k; }
  }
  a.min_cost[i] = bv;
  a.min_k[i] = bk;
}

__device__ __forceinline__ double readlane_f64(double v, int lane) {   // lane must be wave-uniform
  const uint64_t u = (uint64_t)__double_as_longlong(v);
  const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)u, lane);
  const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(u >> 32), lane);
  return __longlong_as_double((long long)(((uint64_t)hi << 32) | lo));
}

// One block of WAVES waves per class; lane = destination layout in every wave, and wave q owns the source
// layouts [q * LMAX/WAVES, (q + 1) * LMAX/WAVES) with its lanes' entries of those rows of the table in registers.
// Per window every wave forms the window's totals itself (all waves carry the same state), takes the least
// arrival total over its sources; the waves' partial minima meet in LDS (atomic minimum per destination)
// behind the window's only block barrier.  min_cost[window][layout] is overwritten by the least total
// of the sequences that end there (+inf: none); kend[window] = -1: no feasible candidate, kEndMark: a
// sequence ends here, 0 otherwise.
template <int LMAX, int WAVES>
__global__ __launch_bounds__(WAVES* DYN_WAVE) void path_chain_kernel(PathArgs a) {
  constexpr int SPW = LMAX / WAVES;                          // sources per wave
  __shared__ double s_c[(kChainChunk + 1) * DYN_WAVE];       // the chunk's least costs by (window, layout), one window more; totals once a window is done
  __shared__ int32_t s_ke[kChainChunk];
  __shared__ double s_best[3][DYN_WAVE];                     // least arrival total per destination: the waves' partial minima meet here (LDS atomic minimum); three buffers in turn
  const int g = blockIdx.x, lane = threadIdx.x & (DYN_WAVE - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / DYN_WAVE);
  const int NL = a.n_layout, NW = a.n_window, G = a.G;
  const double inf = __builtin_inf();
  const bool on = lane < NL;
  double t[SPW];                                             // overhead of going from this wave's source q to this lane's layout
#pragma unroll
  for (int q = 0; q < SPW; ++q) {
    const int ls = wave * SPW + q;
    t[q] = (on && ls < NL) ? a.transition[(size_t)ls * NL + lane] : inf;   // layouts beyond NL never win
  }
  int32_t* kend = a.kend + (size_t)g * NW;
  auto row = [&](int w) { return ((size_t)w * G + g) * NL + lane; };

  double total = 0.0, arrive = inf;                          // the same in every wave
  bool first = true;
  int buf = 0;
  if (wave == 0) s_best[0][lane] = inf;                      // ordered before its first use by the chunk loop's barriers
#pragma unroll 1
  for (int w0 = 0; w0 < NW; w0 += kChainChunk) {
    __syncthreads();                                         // the previous chunk's flush has read s_c / s_ke
#pragma unroll
    for (int j = 0; j < (kChainChunk + 1 + WAVES - 1) / WAVES; ++j) {
      const int i = j * WAVES + wave;                        // row of the chunk this wave loads
      if (i <= kChainChunk) s_c[i * DYN_WAVE + lane] = (on && w0 + i < NW) ? a.min_cost[row(w0 + i)] : inf;
    }
    __syncthreads();
    const int n = NW - w0 < kChainChunk ? NW - w0 : kChainChunk;
    double c_nxt = s_c[lane];
#pragma unroll 1
    for (int i = 0; i < n; ++i) {
      const double c_cur = c_nxt;
      c_nxt = s_c[(i + 1) * DYN_WAVE + lane];                // read a window ahead, before this row is overwritten
      // least total of the sequences that end in this window in this lane's layout
      const double v = (first || !(c_cur < inf)) ? c_cur : arrive + c_cur;
      const bool gap = __ballot(v < inf) == 0;               // no feasible candidate in this window
      double m[SPW];                                         // sums are never NaN here: plain minima
#pragma unroll
      for (int q = 0; q < SPW; ++q) m[q] = readlane_f64(v, wave * SPW + q) + t[q];
#pragma unroll
      for (int d = 1; d < SPW; d *= 2)
#pragma unroll
        for (int q = 0; q + d < SPW; q += 2 * d) m[q] = fmin(m[q], m[q + d]);
      __hip_atomic_fetch_min(&s_best[buf][lane], m[0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
      const int nxt = buf == 2 ? 0 : buf + 1;
      // the next window's buffer: last read two windows ago, behind the previous window's barrier for every wave
      if (wave == WAVES - 1) s_best[nxt][lane] = inf;
      lds_barrier();                                         // the window's only block barrier
      if (wave == 0) s_c[i * DYN_WAVE + lane] = v;           // every wave has taken this row's costs before the barrier
      const double bv = s_best[buf][lane];
      buf = nxt;
      // a sequence ends here if the next window has no feasible candidate (its costs are all +inf) or does not exist
      const bool ends = !gap && (w0 + i + 1 >= NW || __ballot(c_nxt < inf) == 0);
      if (ends) {                                            // wave-uniform
        double ev = v;
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) ev = fmin(ev, __shfl_xor(ev, d, DYN_WAVE));
        total += ev;                                         // the sequences' totals in time order
      }
      if (threadIdx.x == 0) s_ke[i] = gap ? -1 : (ends ? kEndMark : 0);
      arrive = bv;
      first = gap;
    }
    __syncthreads();
    for (int i = wave; i < n; i += WAVES)
      if (on) a.min_cost[row(w0 + i)] = s_c[i * DYN_WAVE + lane];
    if (threadIdx.x < n) kend[w0 + threadIdx.x] = s_ke[threadIdx.x];
  }
  if (threadIdx.x == 0) a.path_cost[g] = total;
}

// One wave per (window, class), lane = destination layout, the lane's column of the table in registers: where
// the cheapest arrival in every layout of the next window comes from (least total + overhead, then the lowest
// candidate among the sources that reach it), as (candidate << 6) | its layout, -1: none; and the best end of a
// sequence that ends in this window.  The sums are those of the walk, from the same operands.
template <int LMAX>
__global__ __launch_bounds__(256) void path_pred_kernel(PathArgs a) {
  const int lane = threadIdx.x & (DYN_WAVE - 1);
  const int NL = a.n_layout, NW = a.n_window, G = a.G;
  const double inf = __builtin_inf();
  const bool on = lane < NL;
  double t[LMAX];
#pragma unroll
  for (int l = 0; l < LMAX; ++l) t[l] = (on && l < NL) ? a.transition[(size_t)l * NL + lane] : inf;
  const int64_t cells = (int64_t)NW * G;
  const int64_t n_wave = (int64_t)gridDim.x * (blockDim.x / DYN_WAVE);
  for (int64_t cell = (int64_t)blockIdx.x * (blockDim.x / DYN_WAVE) + threadIdx.x / DYN_WAVE; cell < cells; cell += n_wave) {
    const int w = (int)(cell / G), g = (int)(cell % G);
    const double v = on ? a.min_cost[(size_t)cell * NL + lane] : inf;
    const int k = on ? a.min_k[(size_t)cell * NL + lane] : 0;
    const uint32_t pk = (v < inf) ? (((uint32_t)k << 6) | (uint32_t)lane) : 0xFFFFFFFFu;
    int32_t* kend = a.kend + (size_t)g * NW + w;
    if (*kend == kEndMark) {                                 // wave-uniform
      double ev = v;
#pragma unroll
      for (int d = 32; d >= 1; d >>= 1) ev = fmin(ev, __shfl_xor(ev, d, DYN_WAVE));
      uint32_t ep = (v == ev) ? pk : 0xFFFFFFFFu;
#pragma unroll
      for (int d = 32; d >= 1; d >>= 1) ep = min(ep, (uint32_t)__shfl_xor((int)ep, d, DYN_WAVE));
      if (lane == 0) *kend = (int32_t)ep;
    }
    if (w + 1 >= NW) continue;
    double m = inf;
    uint32_t p = 0xFFFFFFFFu;                                // all ones: nothing arrives (then m is +inf)
#pragma unroll
    for (int l = 0; l < LMAX; ++l) {
      const double arr = readlane_f64(v, l) + t[l];
      const uint32_t sp = (uint32_t)__builtin_amdgcn_readlane((int)pk, l);
      const bool better = arr < m || (arr == m && sp < p);
      m = better ? arr : m;
      p = better ? sp : p;
    }
    if (on) a.pred[((size_t)g * NW + w + 1) * NL + lane] = (int32_t)p;
  }
}

// Trace-back.  A window's choice depends on the next window's only through a small state: the layout chosen there,
// or "none" (the next window has no feasible candidate, starts a sequence, or does not exist).  Runs of
// DYN_PATH_RUN windows are therefore followed back for every possible entry state at once (one thread per state;
// path_trace_runs_kernel records the state each run is left with), a block then finds the state its run is really
// entered with by chaining those records from the last run down to its own, follows its run once more from that
// state and writes the selection (path_trace_write_kernel).  Both kernels stage a run's records in LDS.
__device__ __forceinline__ int trace_step(int ke, int state, const int32_t* s_bp, int i, int NL) {
  // record of window i of the run: -1 none, else (candidate << 6) | layout
  if (ke < 0) return -1;                                     // no feasible candidate in this window
  if (state == DYN_PATH_STATES - 1) return ke;               // last window of a sequence: its best end
  return s_bp[i * NL + state];                               // predecessor of the next window's choice
}

__device__ __forceinline__ void trace_stage(const PathArgs& a, int g, int lo, int hi, int32_t* s_bp, int32_t* s_ke) {
  const int NL = a.n_layout, NW = a.n_window;
  const int32_t* bp = a.pred + (size_t)g * NW * NL;          // [NW][NL]: where the cheapest arrival in layout l at window w comes from
  const int32_t* kend = a.kend + (size_t)g * NW;             // [NW]: -1 gap, best end where a sequence ends, 0 otherwise
  const int n_row = (hi < NW ? hi : NW - 1) - lo;            // predecessor records of the windows lo+1 .. hi
  for (int i = threadIdx.x; i < n_row * NL; i += blockDim.x) s_bp[i] = bp[(size_t)(lo + 1) * NL + i];
  for (int i = n_row * NL + threadIdx.x; i < (hi - lo) * NL; i += blockDim.x) s_bp[i] = -1;   // nothing follows the last window
  for (int i = threadIdx.x; i < hi - lo; i += blockDim.x) s_ke[i] = kend[lo + i];
  __syncthreads();
}

// grid (runs, classes), 128 threads: thread s < DYN_PATH_STATES follows the run back from entry state s.
__global__ __launch_bounds__(128) void path_trace_runs_kernel(PathArgs a) {
  __shared__ int32_t s_bp[DYN_PATH_RUN * DYN_WAVE];
  __shared__ int32_t s_ke[DYN_PATH_RUN];
  const int r = blockIdx.x, g = blockIdx.y;
  const int lo = r * DYN_PATH_RUN, hi = min(a.n_window, lo + DYN_PATH_RUN);
  trace_stage(a, g, lo, hi, s_bp, s_ke);
  int state = threadIdx.x;
  if (state >= DYN_PATH_STATES) return;
  if (state < DYN_PATH_STATES - 1 && state >= a.n_layout) state = DYN_PATH_STATES - 1;   // not a layout: never entered with
  for (int i = hi - lo - 1; i >= 0; --i) {
    const int rec = trace_step(s_ke[i], state, s_bp, i, a.n_layout);
    state = rec < 0 ? DYN_PATH_STATES - 1 : (rec & 63);
  }
  a.exits[((size_t)g * gridDim.x + r) * DYN_PATH_STATES + threadIdx.x] = state;
}

// grid (runs, classes), 64 threads.
__global__ __launch_bounds__(DYN_WAVE) void path_trace_write_kernel(PathArgs a) {
  __shared__ int32_t s_bp[DYN_PATH_RUN * DYN_WAVE];
  __shared__ int32_t s_ke[DYN_PATH_RUN];
  __shared__ int32_t s_sel[DYN_PATH_RUN];
  const int r = blockIdx.x, g = blockIdx.y, n_run = gridDim.x;
  const int G = a.G, K = a.K;
  const int lo = r * DYN_PATH_RUN, hi = min(a.n_window, lo + DYN_PATH_RUN);
  trace_stage(a, g, lo, hi, s_bp, s_ke);
  // the state this run is entered with: the later runs' records chained from the end.  The records of kHop runs
  // are fetched together (lane s holds the record for entry state s), so a hop is a lane read, not a load.
  constexpr int kHop = 16;
  int state = DYN_PATH_STATES - 1;                           // nothing follows the last window; wave-uniform
  for (int top = n_run - 1; top > r; top -= kHop) {
    int by_layout[kHop], by_none[kHop];
#pragma unroll
    for (int j = 0; j < kHop; ++j) {
      const int q = max(top - j, r + 1);                     // runs at or below r are not used
      const int32_t* row = a.exits + ((size_t)g * n_run + q) * DYN_PATH_STATES;
      by_layout[j] = row[threadIdx.x];
      by_none[j] = row[DYN_PATH_STATES - 1];
    }
#pragma unroll
    for (int j = 0; j < kHop; ++j)
      if (top - j > r)
        state = state == DYN_PATH_STATES - 1 ? by_none[j] : __builtin_amdgcn_readlane(by_layout[j], __builtin_amdgcn_readfirstlane(state));
  }
  if (threadIdx.x == 0) {
    for (int i = hi - lo - 1; i >= 0; --i) {
      const int rec = trace_step(s_ke[i], state, s_bp, i, a.n_layout);
      state = rec < 0 ? DYN_PATH_STATES - 1 : (rec & 63);
      s_sel[i] = rec < 0 ? -1 : (rec >> 6);
    }
  }
  __syncthreads();
  for (int i = threadIdx.x; i < hi - lo; i += blockDim.x) {
    const int k = s_sel[i];
    const size_t cell = (size_t)(lo + i) * G + g;
    a.sel[cell] = k;
    a.sel_energy[cell] = k >= 0 ? a.energy[cell * K + k] : __builtin_inf();
  }
}

template <int LMAX>
void launch_layout_route(const PathArgs& a, hipStream_t s) {
  const int64_t cells = (int64_t)a.n_window * a.G;
  const int64_t n = cells * a.n_layout;
  hipLaunchKernelGGL(path_min_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, a);
  hipLaunchKernelGGL((path_chain_kernel<LMAX, kChainWaves>), dim3((unsigned)a.G), dim3(kChainWaves * DYN_WAVE), 0, s, a);
  const int64_t pred_blocks = std::min<int64_t>((cells + 3) / 4, 2048);
  hipLaunchKernelGGL(path_pred_kernel<LMAX>, dim3((unsigned)pred_blocks), dim3(256), 0, s, a);
  const dim3 runs((unsigned)dyn_path_runs(a.n_window), (unsigned)a.G);
  hipLaunchKernelGGL(path_trace_runs_kernel, runs, dim3(128), 0, s, a);
  hipLaunchKernelGGL(path_trace_write_kernel, runs, dim3(DYN_WAVE), 0, s, a);
}

}  // namespace

size_t dyn_path_lds(int32_t K, int32_t n_layout) {
  return ((size_t)K + ((size_t)n_layout + 1) * n_layout + (2 + kParts) * ((size_t)n_layout + 1)) * sizeof(double) +
         ((size_t)(2 + kParts) * (n_layout + 1) + (size_t)kRun * n_layout + kRun) * sizeof(int32_t) +
         2 * (size_t)K * sizeof(uint16_t) + 16;
}

bool dyn_path_fits(int32_t K, int32_t n_layout) {
  if (K < 1 || n_layout < 1) return false;
  if (n_layout <= DYN_WAVE) return K <= (1 << 24);           // wave-per-class route: candidates are packed into 24 bits
  return K <= DYN_PATH_MAX_CONFIGS && n_layout < kThreads && dyn_path_lds(K, n_layout) <= DYN_LDS_BUDGET;
}

hipError_t dyn_launch_path(const PathArgs& a, hipStream_t s) {
  if (!dyn_path_fits(a.K, a.n_layout)) return hipErrorInvalidValue;
  DynTimed timed(DYN_K_PATH, s);
  if (a.n_layout <= DYN_WAVE) {
    if (a.n_layout <= 16) launch_layout_route<16>(a, s);
    else if (a.n_layout <= 32) launch_layout_route<32>(a, s);
    else if (a.n_layout <= 48) launch_layout_route<48>(a, s);
    else launch_layout_route<64>(a, s);
    return hipGetLastError();
  }
  hipLaunchKernelGGL(path_kernel, dim3((unsigned)a.G), dim3(kThreads), dyn_path_lds(a.K, a.n_layout), s, a);
  return hipGetLastError();
}
