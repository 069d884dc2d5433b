// Selection with transition overheads between consecutive windows (Section IV-B "Accounting for
// the overheads"; Table VI lists the re-sharding overheads between layouts): per class the
// sequence of configurations with the least  sum_w cost(w, k_w) + sum_w transition[layout(k_{w-1})]
// [layout(k_w)], found window by window.  The step from one window to the next is factored
// through the layouts: the cheapest way to arrive in layout l' is the least over source
// layouts l of (least total ending in l) + transition[l][l'] - equal to the least over all
// predecessors because rounded addition is monotone.
//
// Two routes.  Up to 64 layouts (further down): a parallel pre-pass reduces every (window, class) to
// its layouts' least costs, then one block per class walks the windows with a lane per layout.
// More layouts (next): one block per class walks the windows in time order (the recurrence is
// sequential, so the time per window is what counts).  The candidates are visited in an order sorted by layout
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


// ---- up to 64 layouts ----------------------------------------------------------------------------
// The step through the layouts needs, per window, only the least cost of every layout and the
// candidate that has it (adding a layout's arrival total to its candidates' costs keeps their
// order: rounded addition is monotone).  Those are independent of the recurrence:
// path_min_kernel takes them for all windows at once.  path_chain_kernel then walks the windows
// with one lane per layout.  What the walk costs is the latency of one window's dependent steps,
// so it touches global memory only a chunk of windows at a time, keeps its lanes' entries of the
// transition table in registers, and avoids data-dependent branches (a load inside a branch per
// source costs an LDS round trip each).
constexpr int kChainRun = 64;
constexpr int kChainChunk = 16;                            // windows per visit to global memory
constexpr int kChainWaves = 8;                             // measured: 2 waves 2.4 ms, 4 waves 1.7 ms, 8 waves 1.5 ms, 16 waves 2.0 ms (one day, 48 layouts)

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

// One block of kChainWaves waves per class; lane = destination layout in every wave, and wave q owns the source
// layouts [q * LMAX/kChainWaves, (q + 1) * LMAX/kChainWaves) with its lanes' entries of those rows of the table in registers.
// Per window every wave forms the window's totals itself (all waves carry the same state), publishes
// them in its own LDS strip, takes the least arrival total over its sources and, among the sources that
// reach it, the lowest candidate; the waves' partial results meet in LDS behind the window's only block
// barrier and every wave merges them (least total, then lowest candidate: the same answer as one pass over
// all sources).  Predecessor records: (candidate << 6) | its layout, -1: none.
template <int LMAX>
__global__ __launch_bounds__(kChainWaves* DYN_WAVE) void path_chain_kernel(PathArgs a) {
  constexpr int SPW = LMAX / kChainWaves;                    // sources per wave
  __shared__ int32_t s_bp[kChainRun * LMAX];
  __shared__ int32_t s_sel[kChainRun];
  __shared__ double s_c[(kChainChunk + 1) * DYN_WAVE];       // the chunk's least costs by (window, layout), one window more
  __shared__ int32_t s_k[kChainChunk * DYN_WAVE];            // and the candidates that have them
  __shared__ int32_t s_pr[kChainChunk * DYN_WAVE];           // the chunk's predecessor records
  __shared__ int32_t s_ke[kChainChunk];
  __shared__ double s_v[kChainWaves][DYN_WAVE];              // per wave: the window's totals by layout
  __shared__ uint32_t s_pk[kChainWaves][DYN_WAVE];           // per wave: (candidate << 6) | layout, all ones where nothing ends
  __shared__ double s_m[2][kChainWaves][DYN_WAVE];           // by window parity: every wave's least arrival total per destination
  __shared__ uint32_t s_p[2][kChainWaves][DYN_WAVE];         // and the packed candidate that reaches it
  const int g = blockIdx.x, lane = threadIdx.x & (DYN_WAVE - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / DYN_WAVE);
  const int NL = a.n_layout, NW = a.n_window, G = a.G, K = a.K;
  const double inf = __builtin_inf();
  const bool on = lane < NL;
  double t[SPW];                                             // overhead of going from this wave's source q to this lane's layout
#pragma unroll
  for (int q = 0; q < SPW; ++q) {
    const int ls = wave * SPW + q;
    t[q] = (on && ls < NL) ? a.transition[(size_t)ls * NL + lane] : inf;   // layouts beyond NL never win
  }
  int32_t* bp = a.pred + (size_t)g * NW * NL;                // [NW][NL]: where the cheapest arrival in layout l at window w comes from
  int32_t* kend = a.kend + (size_t)g * NW;                   // [NW]: -1 gap, best end where a sequence ends, 0 otherwise
  auto row = [&](int w) { return ((size_t)w * G + g) * NL + lane; };

  double total = 0.0, arrive = inf;                          // the same in every wave
  bool first = true;
  int par = 0;
#pragma unroll 1
  for (int w0 = 0; w0 < NW; w0 += kChainChunk) {
    // Global memory is touched a chunk of windows at a time: costs and candidates are parked in LDS, the
    // walk itself reads and writes LDS only, the chunk's predecessor records are flushed afterwards.
    __syncthreads();                                         // the previous chunk's flush has read s_pr / s_ke
#pragma unroll
    for (int j = 0; j < (kChainChunk + 1 + kChainWaves - 1) / kChainWaves; ++j) {
      const int i = j * kChainWaves + wave;                  // row of the chunk this wave loads
      if (i <= kChainChunk) {
        const bool in = on && w0 + i < NW;
        s_c[i * DYN_WAVE + lane] = in ? a.min_cost[row(w0 + i)] : inf;
        if (i < kChainChunk) s_k[i * DYN_WAVE + lane] = in ? a.min_k[row(w0 + i)] : 0x7FFFFFFF;
      }
    }
    __syncthreads();
    const int n = NW - w0 < kChainChunk ? NW - w0 : kChainChunk;
    double c_nxt = s_c[lane];
    int k_nxt = s_k[lane];
#pragma unroll 1
    for (int i = 0; i < n; ++i) {
      const double c_cur = c_nxt;
      const int k_cur = k_nxt;
      c_nxt = s_c[(i + 1) * DYN_WAVE + lane];                // read a window ahead: out of the way of this window's chain of LDS round trips
      k_nxt = s_k[(i + 1 < kChainChunk ? i + 1 : i) * DYN_WAVE + lane];
      // least total of the sequences that end in this window in this lane's layout
      const double v = (first || !(c_cur < inf)) ? c_cur : arrive + c_cur;
      const uint32_t pk = (v < inf) ? (((uint32_t)k_cur << 6) | (uint32_t)lane) : 0xFFFFFFFFu;
      const bool gap = __ballot(v < inf) == 0;               // no feasible candidate in this window
      s_v[wave][lane] = v;
      s_pk[wave][lane] = pk;
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");  // read back by this wave's other lanes only
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      // this wave's sources: least arrival total, then the lowest candidate among the sources that reach it
      double arr[SPW];
      uint32_t spk[SPW];
#pragma unroll
      for (int q = 0; q < SPW; ++q) {
        arr[q] = s_v[wave][wave * SPW + q] + t[q];
        spk[q] = s_pk[wave][wave * SPW + q];
        asm volatile("" : "+v"(spk[q]));                     // loaded here, with the totals: not inside a branch per source later
      }
      double m0 = inf, m1 = inf;                             // sums are never NaN here: plain minima
#pragma unroll
      for (int q = 0; q < SPW; q += 2) { m0 = fmin(m0, arr[q]); if (q + 1 < SPW) m1 = fmin(m1, arr[q + 1]); }
      const double m = fmin(m0, m1);
      uint32_t p0 = 0xFFFFFFFFu, p1 = 0xFFFFFFFFu;
#pragma unroll
      for (int q = 0; q < SPW; q += 2) {
        p0 = min(p0, arr[q] == m ? spk[q] : 0xFFFFFFFFu);
        if (q + 1 < SPW) p1 = min(p1, arr[q + 1] == m ? spk[q + 1] : 0xFFFFFFFFu);
      }
      s_m[par][wave][lane] = m;
      s_p[par][wave][lane] = min(p0, p1);
      lds_barrier();                                         // the window's only block barrier (partials alternate by parity)
      double pm[kChainWaves];
      uint32_t pp[kChainWaves];
#pragma unroll
      for (int q = 0; q < kChainWaves; ++q) {
        pm[q] = s_m[par][q][lane];
        pp[q] = s_p[par][q][lane];
        asm volatile("" : "+v"(pp[q]));
      }
      double bv = pm[0];
#pragma unroll
      for (int q = 1; q < kChainWaves; ++q) bv = fmin(bv, pm[q]);
      uint32_t bp_rec = 0xFFFFFFFFu;                         // all ones: nothing arrives (then bv is +inf)
#pragma unroll
      for (int q = 0; q < kChainWaves; ++q) bp_rec = min(bp_rec, pm[q] == bv ? pp[q] : 0xFFFFFFFFu);
      par ^= 1;
      // a sequence ends here if the next window has no feasible candidate (its costs are all +inf) or does not exist
      const bool ends = !gap && (w0 + i + 1 >= NW || __ballot(c_nxt < inf) == 0);
      int32_t ke = gap ? -1 : 0;
      if (ends) {                                            // wave-uniform: least total, then the lowest candidate
        double ev = v;
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) ev = fmin(ev, __shfl_xor(ev, d, DYN_WAVE));
        uint32_t ep = (v == ev) ? pk : 0xFFFFFFFFu;
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) ep = min(ep, (uint32_t)__shfl_xor((int)ep, d, DYN_WAVE));
        total += ev;                                         // the sequences' totals in time order
        ke = (int32_t)ep;
      }
      if (wave == 0) {
        s_pr[i * DYN_WAVE + lane] = (int32_t)bp_rec;         // how the next window is entered in this lane's layout; -1: not at all
        if (lane == 0) s_ke[i] = ke;
      }
      arrive = bv;
      first = gap;
    }
    __syncthreads();
    for (int i = wave; i < n; i += kChainWaves)
      if (on && w0 + i + 1 < NW) bp[(size_t)(w0 + i + 1) * NL + lane] = s_pr[i * DYN_WAVE + lane];
    if (threadIdx.x < n) kend[w0 + threadIdx.x] = s_ke[threadIdx.x];
  }
  if (threadIdx.x == 0) a.path_cost[g] = total;
  // make the predecessor records visible to this block's own later loads
  __threadfence();
  __syncthreads();

  // trace back, a run of windows at a time from the end
  constexpr int nthr = kChainWaves * DYN_WAVE;
  int carry_k = -1, carry_l = 0;                             // thread 0: -1 = the next window starts a sequence
  for (int hi = NW; hi > 0; hi -= kChainRun) {
    const int lo = hi > kChainRun ? hi - kChainRun : 0;
    const int n_row = (hi < NW ? hi : NW - 1) - lo;          // predecessor records of the windows lo+1 .. hi
    // records written by this block before the barrier above: plain loads, all in flight together
    for (int i = threadIdx.x; i < n_row * NL; i += nthr) s_bp[i] = bp[(size_t)(lo + 1) * NL + i];
    for (int i = threadIdx.x; i < hi - lo; i += nthr) s_sel[i] = kend[lo + i];
    __syncthreads();
    if (threadIdx.x == 0) {
      for (int w = hi - 1; w >= lo; --w) {
        const int ke = s_sel[w - lo];
        int rec;
        if (ke < 0) rec = -1;                                // no feasible candidate in this window
        else if (carry_k < 0) rec = ke;                      // last window of a sequence: its best end
        else rec = s_bp[(w - lo) * NL + carry_l];            // predecessor of the next window's choice
        carry_k = rec < 0 ? -1 : (rec >> 6);
        carry_l = rec < 0 ? 0 : (rec & 63);
        s_sel[w - lo] = carry_k;
      }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < hi - lo; i += nthr) {
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

bool dyn_path_fits(int32_t K, int32_t n_layout) {
  if (K < 1 || n_layout < 1) return false;
  if (n_layout <= DYN_WAVE) return K <= (1 << 24);           // wave-per-class route: candidates are packed into 24 bits
  return K <= DYN_PATH_MAX_CONFIGS && n_layout < kThreads && dyn_path_lds(K, n_layout) <= DYN_LDS_BUDGET;
}

hipError_t dyn_launch_path(const PathArgs& a, hipStream_t s) {
  if (!dyn_path_fits(a.K, a.n_layout)) return hipErrorInvalidValue;
  DynTimed timed(DYN_K_PATH, s);
  if (a.n_layout <= DYN_WAVE) {
    const int64_t n = (int64_t)a.n_window * a.G * a.n_layout;
    hipLaunchKernelGGL(path_min_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, a);
    if (a.n_layout <= 16) hipLaunchKernelGGL(path_chain_kernel<16>, dim3((unsigned)a.G), dim3(kChainWaves * DYN_WAVE), 0, s, a);
    else if (a.n_layout <= 32) hipLaunchKernelGGL(path_chain_kernel<32>, dim3((unsigned)a.G), dim3(kChainWaves * DYN_WAVE), 0, s, a);
    else if (a.n_layout <= 48) hipLaunchKernelGGL(path_chain_kernel<48>, dim3((unsigned)a.G), dim3(kChainWaves * DYN_WAVE), 0, s, a);
    else hipLaunchKernelGGL(path_chain_kernel<64>, dim3((unsigned)a.G), dim3(kChainWaves * DYN_WAVE), 0, s, a);
    return hipGetLastError();
  }
  hipLaunchKernelGGL(path_kernel, dim3((unsigned)a.G), dim3(kThreads), dyn_path_lds(a.K, a.n_layout), s, a);
  return hipGetLastError();
}
