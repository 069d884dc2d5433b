// Tick-level load inside a window: every window is split into n_tick ticks (sub-windows of
// the sorted trace), each request is served under the load of its own tick (the instance
// manager re-tunes the frequency every few seconds under the current load, Section IV-B
// "Scale-up/down").  Per (window, class) cell and candidate configuration the profile is
// looked up once per tick; the window's energy is the sum over its ticks.
//
// The per-request percentile still collapses, tick by tick: inside one tick TTFT is
// input length x a non-negative constant, so the cell's j-th largest TTFT (j = m - rank + 1)
// is among the j largest input lengths of each tick scaled by that tick's prefill time.
// `tick_top_kernel` extracts, once per fine cell and independent of the configuration, the
// DYN_TICK_TOP largest input lengths in descending order; `tick_space_kernel` merges the
// n_tick descending candidate lists per (cell, configuration) for j steps.  The TBT
// percentile is the j-th largest of the ticks' TBT values weighted by their request counts.
#include "dyn_ticks.h"

namespace {

constexpr int kWavesPerBlock = 4;

// ---- the largest input lengths of every fine cell, descending -------------------------------
// One wave per fine cell.  Only the j = m - rank + 1 largest values of a tick can matter,
// with m and rank those of the whole (window, class) cell; cells with j > DYN_TICK_TOP are
// skipped here and reported by the evaluation kernel.  The wave keeps its best 64 values
// sorted in its lanes and merges the cell row by row: a value's position is the number of
// values that beat it (kept values win ties against new ones, lower lanes against higher
// ones); new values that cannot reach the first j positions are dropped before the merge,
// and the merged order is written through a 64-word LDS buffer.
__global__ __launch_bounds__(kWavesPerBlock* DYN_WAVE) void tick_top_kernel(
    const int32_t* __restrict__ in, const int64_t* __restrict__ fine_off, int64_t n_req, int32_t n_window,
    int32_t T, int32_t G, int32_t pct_num, int32_t pct_den, int32_t* __restrict__ top) {
  __shared__ int32_t s_buf[kWavesPerBlock][DYN_WAVE];
  const int lane = threadIdx.x & (DYN_WAVE - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / DYN_WAVE);
  const int64_t fine_cells = (int64_t)n_window * T * G;
  const int64_t f = (int64_t)blockIdx.x * kWavesPerBlock + wave;
  if (f >= fine_cells) return;
  const int64_t w = f / ((int64_t)T * G);
  const int g = (int)(f % G);
  // requests of the whole (window, class) cell: lane q holds tick q's count
  int64_t cnt = 0;
  if (lane < T) {
    const int64_t cf = (w * T + lane) * G + g;
    const int64_t b = fine_off[cf], e = fine_off[cf + 1];
    cnt = (b < 0 || e < b || e > n_req) ? 0 : e - b;
  }
  int64_t m_cell = cnt;
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) m_cell += __shfl_xor(m_cell, d, DYN_WAVE);
  const int64_t rank = (pct_num * m_cell + pct_den - 1) / pct_den;
  const int64_t j64 = m_cell - rank + 1;
  if (m_cell == 0 || j64 > DYN_TICK_TOP) return;     // wave-uniform
  const int keep = __builtin_amdgcn_readfirstlane((int)j64);

  int64_t beg = fine_off[f], end = fine_off[f + 1];
  if (beg < 0 || end < beg || end > n_req) beg = end = 0;   // reported by the aggregation kernel
  const int64_t m = end - beg;
  int32_t best = -1;                                  // input lengths are >= 0
  int32_t* buf = s_buf[wave];
  for (int64_t r0 = 0; r0 < m; r0 += DYN_WAVE) {
    const int nrow = (int)(m - r0 < DYN_WAVE ? m - r0 : DYN_WAVE);
    const int32_t cand = lane < nrow ? in[beg + r0 + lane] : -1;
    const int32_t thr = __builtin_amdgcn_readlane(best, keep - 1);
    const bool mine = lane < nrow && cand > thr;      // a value <= thr has `keep` kept values ahead of it
    uint64_t mask = __ballot(mine);
    if (mask == 0) continue;
    int rb = lane;      // position of my kept value: the kept values before it + new values above it
    int rc = 0;         // position of my new value: kept values >= it + new values that beat it
    while (mask) {
      const int u = __builtin_ctzll(mask);
      mask &= mask - 1;
      const int32_t y = __builtin_amdgcn_readlane(cand, u);
      const int n_ge = __popcll(__ballot(best >= y));
      rb += (y > best) ? 1 : 0;
      rc += (y > cand || (y == cand && u < lane)) ? 1 : 0;
      if (lane == u) rc += n_ge;
    }
    // the positions are a permutation of 0 .. 63 + (new values): every slot below 64 is written once
    if (rb < DYN_WAVE) buf[rb] = best;
    if (mine && rc < DYN_WAVE) buf[rc] = cand;
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    best = buf[lane];
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
  }
  if (lane < keep) top[f * DYN_TICK_TOP + lane] = best;
}

template <int CTRL>
__device__ __forceinline__ uint32_t dpp_row_u32(uint32_t x) {
  return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, CTRL, 0xF, 0xF, false);
}
__device__ __forceinline__ uint32_t wave_min_u32(uint32_t x) {
  x = min(x, dpp_row_u32<0x121>(x));
  x = min(x, dpp_row_u32<0x122>(x));
  x = min(x, dpp_row_u32<0x124>(x));
  x = min(x, dpp_row_u32<0x128>(x));
  const uint32_t a = (uint32_t)__builtin_amdgcn_readlane((int)x, 0), b = (uint32_t)__builtin_amdgcn_readlane((int)x, 16);
  const uint32_t c = (uint32_t)__builtin_amdgcn_readlane((int)x, 32), d = (uint32_t)__builtin_amdgcn_readlane((int)x, 48);
  return min(min(a, b), min(c, d));
}
// a / b given rb = RN(1 / b): correctly rounded for normal operands and quotients.
__device__ __forceinline__ double div_by(double a, double b, double rb) {
  const double q = a * rb;
  const double e = __builtin_fma(-b, q, a);
  return __builtin_fma(e, rb, q);
}

// LDS: [table rows n_slot*3*n_rho] [padded load grid n_rho+2] [reciprocal spacings n_rho+1]
//      [per tick: CellRec] [per tick: request count] [per tick: candidate list] [bucket index (16-bit)]
template <bool LDS, int TMAX>
__global__ __launch_bounds__(DYN_MAX_TILE) void tick_space_kernel(TickArgs a) {
  extern __shared__ double smem[];
  const SpaceArgs& sa = a.s;
  const int tile = blockIdx.x % sa.n_tile;
  const int g = (blockIdx.x / sa.n_tile) % sa.G;
  const int chunk = blockIdx.x / (sa.n_tile * sa.G);
  const int n_rho = sa.n_rho, T = a.n_tick;

  double* s_tab = smem;
  double* s_rgp = smem + (LDS ? (size_t)sa.n_slot * 3 * n_rho : 0);
  double* s_rinv = s_rgp + (n_rho + 2);
  CellRec* s_rec = (CellRec*)(s_rinv + (n_rho + 1));            // [T]
  int32_t* s_cnt = (int32_t*)(s_rec + T);                       // [T] requests per tick
  int32_t* s_top = s_cnt + T;                                   // [T][DYN_TICK_TOP]
  uint16_t* s_js = (uint16_t*)(s_top + T * DYN_TICK_TOP);       // [n_bucket + 1]

  if (LDS) {
    const int per_slot = 3 * n_rho;
    for (int slot = 0; slot < sa.n_slot; ++slot) {
      const int row = sa.tile_rows[tile * sa.n_slot + slot];
      const double* src = sa.tab + ((size_t)g * sa.n_tp_f + (row < 0 ? 0 : row)) * per_slot;
      for (int i = threadIdx.x; i < per_slot; i += blockDim.x) s_tab[slot * per_slot + i] = src[i];
    }
  }
  for (int i = threadIdx.x; i < 2 * n_rho + 3; i += blockDim.x) s_rgp[i] = sa.gridpack[i];
  for (int i = threadIdx.x; i <= sa.n_bucket; i += blockDim.x) s_js[i] = (uint16_t)sa.jstart[i];
  __syncthreads();

  const int k_raw = tile * sa.tile + threadIdx.x;
  const bool live = k_raw < sa.K;          // every lane stays alive for the wave reduction
  const int k = live ? k_raw : sa.K - 1;
  const DevCfg c = sa.cfg[k];
  const bool two_rows = c.u != 0.0;
  const double omu = 1.0 - c.u;
  const double* mlrow = sa.ml + (size_t)g * sa.n_tp_f;
  const double ml = two_rows ? omu * mlrow[c.row_lo] + c.u * mlrow[c.row_hi] : mlrow[c.row_lo];
  const double den = c.nd * ml;
  const double rden = 1.0 / den;
  const double rho_max = s_rgp[n_rho];
  const double slo_ttft = sa.slo_ttft[g], slo_tbt = sa.slo_tbt[g];
  const int32_t bud = sa.budget[g];
  const uint32_t fl_budget = (bud > 0 && c.gpus > bud) ? DYN_F_BUDGET : 0u;
  const double* p0 = sa.pw0 + (size_t)g * sa.n_tp_f;
  const double pw0 = two_rows ? omu * p0[c.row_lo] + c.u * p0[c.row_hi] : p0[c.row_lo];
  const double idle_term = sa.idle_w * ((c.nd * pw0) * a.window_s);
  const int lane = threadIdx.x & (DYN_WAVE - 1);
  const int wslot = tile * (sa.tile / DYN_WAVE) + (int)(threadIdx.x / DYN_WAVE);
  const double* lo_pf = LDS ? s_tab + (size_t)c.slot_lo * 3 * n_rho : sa.tab + ((size_t)g * sa.n_tp_f + c.row_lo) * 3 * n_rho;
  const double* hi_pf = LDS ? s_tab + (size_t)c.slot_hi * 3 * n_rho : sa.tab + ((size_t)g * sa.n_tp_f + c.row_hi) * 3 * n_rho;
  const uint32_t koff = (uint32_t)k * 8u;
  const double ninf = -__builtin_inf();

  const int w0 = chunk * sa.win_per_block;
  const int w1 = min(w0 + sa.win_per_block, sa.n_window);
  for (int w = w0; w < w1; ++w) {
    const size_t cell = (size_t)w * sa.G + g;
    __syncthreads();     // the previous window's tick data has been consumed
    for (int q = threadIdx.x; q < T; q += blockDim.x) {
      const size_t f = ((size_t)w * T + q) * sa.G + g;
      s_rec[q] = sa.rec[f];
      int64_t b = a.fine_off[f], e = a.fine_off[f + 1];
      if (b < 0 || e < b || e > a.n_req) b = e = 0;
      s_cnt[q] = (int32_t)(e - b);
    }
    __syncthreads();
    int m = 0;
    for (int q = 0; q < T; ++q) m += s_cnt[q];
    const int rank = (int)(((int64_t)a.pct_num * m + a.pct_den - 1) / a.pct_den);
    const int j = m - rank + 1;                  // the percentile is the j-th largest value
    const bool deep = m > 0 && j > DYN_TICK_TOP; // beyond the extracted candidates
    if (m > 0 && !deep) {                        // block-uniform
      for (int i = threadIdx.x; i < T * DYN_TICK_TOP; i += blockDim.x) {
        const int q = i / DYN_TICK_TOP, x = i - q * DYN_TICK_TOP;
        if (x < j && x < s_cnt[q]) s_top[i] = a.top[(((size_t)w * T + q) * sa.G + g) * DYN_TICK_TOP + x];
      }
    }
    __syncthreads();

    double pf[TMAX], tb[TMAX];
    double e = 0.0;
    bool ov = false;
#pragma unroll
    for (int q = 0; q < TMAX; ++q) {
      pf[q] = 0.0;
      tb[q] = ninf;
      if (q < T) {
        const double rho = div_by(s_rec[q].load, den, rden);
        const bool o = rho > rho_max;
        ov = ov || o;
        const double rc = o ? rho_max : rho;
        int jj = s_js[(int)(fmax(rc, 0.0) * sa.bucket_scale)];
        while (jj > 0 && s_rgp[jj + 1] > rc) --jj;
        while (jj < n_rho - 2 && s_rgp[jj + 2] <= rc) ++jj;
        const double r0 = s_rgp[jj + 1], r1 = s_rgp[jj + 2];
        const double t = div_by(rc - r0, r1 - r0, s_rinv[jj + 1]);
        const double omt = 1.0 - t;
        double x_pf = omt * lo_pf[jj] + t * lo_pf[jj + 1];
        double x_tb = omt * lo_pf[n_rho + jj] + t * lo_pf[n_rho + jj + 1];
        double x_pw = omt * lo_pf[2 * n_rho + jj] + t * lo_pf[2 * n_rho + jj + 1];
        if (two_rows) {
          const double b_pf = omt * hi_pf[jj] + t * hi_pf[jj + 1];
          const double b_tb = omt * hi_pf[n_rho + jj] + t * hi_pf[n_rho + jj + 1];
          const double b_pw = omt * hi_pf[2 * n_rho + jj] + t * hi_pf[2 * n_rho + jj + 1];
          x_pf = omu * x_pf + c.u * b_pf;
          x_tb = omu * x_tb + c.u * b_tb;
          x_pw = omu * x_pw + c.u * b_pw;
        }
        pf[q] = x_pf;
        tb[q] = s_cnt[q] > 0 ? x_tb : ninf;     // a tick without requests contributes no TBT sample
        e += (c.nd * x_pw) * a.tick_s;          // ticks in time order
      }
    }

    double p_ttft = 0.0, p_tbt = 0.0;
    if (m > 0 && !deep) {
      // TBT: ticks in descending TBT order until j requests are covered (at most T picks)
      {
        uint32_t used = 0;
        int need = j;
        double val = 0.0;
        for (int it = 0; it < TMAX && need > 0; ++it) {
          double best = ninf;
          int bi = 0;
#pragma unroll
          for (int q = 0; q < TMAX; ++q) {
            const bool better = !((used >> q) & 1u) && tb[q] > best;
            best = better ? tb[q] : best;
            bi = better ? q : bi;
          }
          used |= 1u << bi;
          need -= s_cnt[bi];
          val = best;
        }
        p_tbt = val;
      }
      // TTFT: j steps of a merge of the ticks' descending candidate lists, each scaled by its
      // tick's prefill time per token (>= 0, so every scaled list is still descending)
      {
        double h[TMAX];
        int pos[TMAX];
#pragma unroll
        for (int q = 0; q < TMAX; ++q) {
          pos[q] = 0;
          h[q] = (q < T && s_cnt[q < T ? q : 0] > 0) ? (double)s_top[(q < T ? q : 0) * DYN_TICK_TOP] * pf[q] : ninf;
        }
        double val = 0.0;
        for (int step = 0; step < j; ++step) {
          double best = ninf, bpf = 0.0;
          int bi = 0, bp = 0;
#pragma unroll
          for (int q = 0; q < TMAX; ++q) {
            const bool better = h[q] > best;
            best = better ? h[q] : best;
            bi = better ? q : bi;
            bp = better ? pos[q] : bp;
            bpf = better ? pf[q] : bpf;
          }
          val = best;
          const int np = bp + 1;   // staged while np < j; the merge ends before a later entry is needed
          const bool more = np < s_cnt[bi] && np < j;
          const double nh = more ? (double)s_top[bi * DYN_TICK_TOP + np] * bpf : ninf;
#pragma unroll
          for (int q = 0; q < TMAX; ++q) {
            const bool hit = q == bi;
            pos[q] = hit ? np : pos[q];
            h[q] = hit ? nh : h[q];
          }
        }
        p_ttft = val;
      }
    }
    if (deep) p_ttft = p_tbt = __builtin_inf();   // not computed: reported through the status word

    uint32_t fl = fl_budget;
    if (ov) fl |= DYN_F_OVERLOAD;
    if (p_ttft > slo_ttft) fl |= DYN_F_TTFT;
    if (p_tbt > slo_tbt) fl |= DYN_F_TBT;
    if (!fl) fl = DYN_F_FEASIBLE;
    if (m == 0) fl |= DYN_F_EMPTY;
    if (deep && tile == 0 && threadIdx.x == 0) a.cstat[((size_t)w * T) * sa.G + g] |= DYN_WS_TICK_RANK;

    if (live) {
      const size_t row = cell * (size_t)sa.K;
      __builtin_nontemporal_store(e, (double*)((char*)(sa.energy + row) + koff));
      __builtin_nontemporal_store(p_ttft, (double*)((char*)(sa.p99_ttft + row) + koff));
      __builtin_nontemporal_store(p_tbt, (double*)((char*)(sa.p99_tbt + row) + koff));
      __builtin_nontemporal_store((uint8_t)fl, (sa.flags + row) + (uint32_t)k);
    }
    {
      // least cost among this wave's feasible configurations (costs >= +0 order like their bits)
      const bool feas = live && (fl & DYN_F_FEASIBLE);
      const double cost = e + idle_term;
      const uint64_t bits = (uint64_t)__double_as_longlong(cost);
      const uint32_t hi = feas ? (uint32_t)(bits >> 32) : 0xFFFFFFFFu;
      const uint32_t lo = feas ? (uint32_t)bits : 0xFFFFFFFFu;
      const uint32_t mh = wave_min_u32(hi);
      uint64_t win = __ballot(feas && hi == mh);
      if (__popcll(win) > 1) {
        const uint32_t mlo = wave_min_u32(hi == mh ? lo : 0xFFFFFFFFu);
        win = __ballot(feas && hi == mh && lo == mlo);
      }
      const int wl = win ? __builtin_ctzll(win) : 0;
      if (lane == wl) {
        SelPart p;
        p.cost = win ? cost : __builtin_inf();
        p.energy = win ? e : __builtin_inf();
        p.k = win ? k_raw : -1;
        p.pad = 0;
        sa.part[cell * (size_t)sa.n_wslot + wslot] = p;
      }
    }
  }
}

size_t tick_lds_tail(int32_t n_rho, int32_t n_bucket, int32_t n_tick) {
  return (size_t)(2 * n_rho + 3) * sizeof(double) +
         (size_t)n_tick * (sizeof(CellRec) + sizeof(int32_t) * (1 + DYN_TICK_TOP)) +
         ((size_t)n_bucket + 1) * sizeof(uint16_t);
}

}  // namespace

hipError_t dyn_launch_tick_top(const int32_t* in_tok, const int64_t* fine_off, int64_t n_req, int32_t n_window,
                               int32_t n_tick, int32_t G, int32_t pct_num, int32_t pct_den, int32_t* top,
                               hipStream_t s) {
  const int64_t fine_cells = (int64_t)n_window * n_tick * G;
  const int64_t blocks = (fine_cells + kWavesPerBlock - 1) / kWavesPerBlock;
  DynTimed timed(DYN_K_TICK_TOP, s);
  hipLaunchKernelGGL(tick_top_kernel, dim3((unsigned)blocks), dim3(kWavesPerBlock * DYN_WAVE), 0, s, in_tok, fine_off,
                     n_req, n_window, n_tick, G, pct_num, pct_den, top);
  return hipGetLastError();
}

hipError_t dyn_launch_tick_space(const TickArgs& a, hipStream_t s) {
  const SpaceArgs& sa = a.s;
  const int n_chunk = (sa.n_window + sa.win_per_block - 1) / sa.win_per_block;
  const size_t blocks = (size_t)n_chunk * sa.G * sa.n_tile;
  const size_t tail = tick_lds_tail(sa.n_rho, sa.n_bucket, a.n_tick);
  const size_t with_tab = (size_t)sa.n_slot * 3 * sa.n_rho * sizeof(double) + tail;
  // the candidate lists take more LDS than the evaluation kernel's cell records: when the
  // table rows no longer fit beside them they are read from global memory instead
  const bool lds = sa.n_slot > 0 && with_tab <= DYN_LDS_BUDGET;
  if (!lds && tail > DYN_LDS_BUDGET) return hipErrorInvalidValue;
  DynTimed timed(DYN_K_TICK_SPACE, s);
  if (lds) hipLaunchKernelGGL((tick_space_kernel<true, DYN_TICK_MAX>), dim3((unsigned)blocks), dim3(sa.tile), with_tab, s, a);
  else hipLaunchKernelGGL((tick_space_kernel<false, DYN_TICK_MAX>), dim3((unsigned)blocks), dim3(sa.tile), tail, s, a);
  return hipGetLastError();
}
