// Selection with transition overheads between consecutive windows (Section IV-B "Accounting for
// the overheads"; Table VI lists the re-sharding overheads between layouts): per class the
// sequence of configurations with the least  sum_w cost(w, k_w) + sum_w transition[layout(k_{w-1})]
// [layout(k_w)], found window by window.  The step from one window to the next is factored
// through the layouts: the cheapest way to arrive in layout l' is the least over source
// layouts l of (least total ending in l) + transition[l][l'] - equal to the least over all
// predecessors because rounded addition is monotone.
//
// One block per class walks the windows in time order (the recurrence is sequential, so the
// time per window is what counts).  The candidates are visited in an order sorted by layout
// (built on the host), a fixed number per thread, their costs loaded one window ahead; per
// window: (A) totals of the sequences ending in each candidate, (B) one thread per layout takes
// the least of its contiguous run of candidates, (C) the cheapest arrival in every layout of
// the next window, the source layouts split over several threads per destination and the
// partial results combined; four LDS-only barriers per window.  Predecessors are kept per (window,
// destination layout) in the workspace and traced back at the end in runs of windows staged
// through LDS.
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

}  // namespace

size_t dyn_path_lds(int32_t K, int32_t n_layout) {
  return ((size_t)K + ((size_t)n_layout + 1) * n_layout + (2 + kParts) * ((size_t)n_layout + 1)) * sizeof(double) +
         ((size_t)(2 + kParts) * (n_layout + 1) + (size_t)kRun * n_layout + kRun) * sizeof(int32_t) +
         2 * (size_t)K * sizeof(uint16_t) + 16;
}

hipError_t dyn_launch_path(const PathArgs& a, hipStream_t s) {
  const size_t lds = dyn_path_lds(a.K, a.n_layout);
  if (lds > DYN_LDS_BUDGET || a.n_layout >= kThreads) return hipErrorInvalidValue;
  DynTimed timed(DYN_K_PATH, s);
  hipLaunchKernelGGL(path_kernel, dim3((unsigned)a.G), dim3(kThreads), lds, s, a);
  return hipGetLastError();
}
