// Tick-level load inside a window: every window is split into n_tick ticks (sub-windows of
// the sorted trace), each request is served under the load of its own tick (the instance
// manager re-tunes the frequency every few seconds under the current load, Section IV-B
// "Scale-up/down").  Per (window, class) cell and candidate configuration the profile is
// looked up once per tick; the window's energy is the sum over its ticks.
//
// The per-request percentile still collapses, tick by tick: inside one tick TTFT is
// input length x a non-negative constant, so the cell's j-th largest TTFT (j = m - rank + 1)
// is among the j largest input lengths of each tick scaled by that tick's prefill time.
// `tick_cell_kernel` produces, once per cell and independent of the configuration, every
// tick's load and its j largest input lengths in descending order; `tick_space_kernel`
// then finds, per (cell, configuration), the j-th largest of the scaled lists.  The TBT
// percentile is the j-th largest of the ticks' TBT values weighted by their request counts.
#include "dyn_ticks.h"
#include "dyn_device.h"

namespace {

constexpr int kWavesPerBlock = 4;
constexpr int kFastDepth = 16;      // j up to here: sorted-list path of the evaluation kernel
// LDS stride of a staged table row in doubles: odd, so that lanes reading the same load bracket of
// different rows do not all fall into one bank
#define DYN_SLOT_STRIDE(n_rho) ((3 * (n_rho)) | 1)

// ---- per-tick loads and candidate lists ------------------------------------------------------
// One wave per (window, class) cell walks the cell's ticks.  Lane q holds tick q's offsets;
// the cell's request count gives j.  Per tick the wave streams the tick's requests once:
// token sum (the tick's load) and, unless the cell is empty or j exceeds DYN_TICK_TOP, the
// j largest input lengths, kept sorted (descending) in the wave's lanes.  A row of 64 new
// values is merged either by j rounds of "take the maximum of kept and new values" or, when
// few new values can still enter the first j positions, by ranking: a value's position is the
// number of values that beat it (kept values win ties against new ones, lower lanes against
// higher ones), and the merged order is written through a 64-word LDS buffer.
__global__ __launch_bounds__(kWavesPerBlock* DYN_WAVE) void tick_cell_kernel(TickCellArgs a) {
  __shared__ int32_t s_buf[kWavesPerBlock][DYN_WAVE];
  const int lane = threadIdx.x & (DYN_WAVE - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / DYN_WAVE);
  const int T = a.n_tick, G = a.G;
  const int64_t cells = (int64_t)a.n_window * G;
  const int64_t c = (int64_t)blockIdx.x * kWavesPerBlock + wave;
  if (c >= cells) return;
  const int64_t w = c / G;
  const int g = (int)(c % G);
  const int64_t f0 = (w * T) * G + g;           // fine cell of tick 0; tick q is q*G further

  int64_t beg_l = 0;
  int32_t cnt_l = 0;
  uint32_t bad_l = 0;
  if (lane < T) {
    const int64_t f = f0 + (int64_t)lane * G;
    const int64_t b = a.fine_off[f], e = a.fine_off[f + 1];
    if (b < 0 || e < b || e > a.n_req) bad_l = DYN_WS_BAD_OFFSETS;   // such a tick is treated as empty
    else { beg_l = b; cnt_l = (int32_t)(e - b); }
  }
  const int64_t m_cell = (int64_t)wave_sum_u64((uint64_t)(uint32_t)cnt_l);
  const int64_t rank = (a.pct_num * m_cell + a.pct_den - 1) / a.pct_den;
  const int64_t j64 = m_cell - rank + 1;
  const bool deep = m_cell > 0 && j64 > DYN_TICK_TOP;
  const int keep = (m_cell == 0 || deep) ? 0 : (int)j64;        // wave-uniform, 0 .. 64

  // what the evaluation kernel needs to know about the cell: j (0 = empty, DYN_TICK_TOP + 1 = not
  // evaluated) and whether some non-empty tick holds fewer than j requests or j is beyond the
  // short-list path (then the merge path takes the cell)
  const uint32_t cmin = wave_min_u32(cnt_l > 0 ? (uint32_t)cnt_l : 0xFFFFFFFFu);
  const int jc = m_cell == 0 ? 0 : (deep ? DYN_TICK_TOP + 1 : (int)j64);
  const int32_t plan = jc | ((keep > 0 && (keep > kFastDepth || cmin < (uint32_t)keep)) ? DYN_PLAN_MERGE : 0);

  double load_l = 0.0;
  uint32_t neg_mask = 0;                        // ticks holding a negative token count
  int32_t* buf = s_buf[wave];
  // (x, y) always hold the row after the one being processed: the next row of the same tick,
  // else the first row of the next tick
  int32_t x, y;
  auto fetch = [&](int64_t at, int32_t left) {   // `left` requests from `at` on, one per lane
    x = lane < left ? a.in[at + lane] : -1;
    y = lane < left ? a.out[at + lane] : 0;
  };
  fetch(readlane_i64(beg_l, 0), __builtin_amdgcn_readlane(cnt_l, 0));
  for (int q = 0; q < T; ++q) {
    const int64_t beg_q = readlane_i64(beg_l, q);
    const int32_t n_q = __builtin_amdgcn_readlane(cnt_l, q);
    int64_t beg_n = 0;
    int32_t n_n = 0;
    if (q + 1 < T) {
      beg_n = readlane_i64(beg_l, q + 1);
      n_n = __builtin_amdgcn_readlane(cnt_l, q + 1);
    }
    if (n_q == 0) fetch(beg_n, n_n);              // nothing was fetched for an empty tick
    uint64_t acc = 0;
    uint32_t orv = 0;
    int32_t best = -1;                            // input lengths are >= 0
    for (int32_t r0 = 0; r0 < n_q; r0 += DYN_WAVE) {
      const int nrow = n_q - r0 < DYN_WAVE ? n_q - r0 : DYN_WAVE;
      const bool have = lane < nrow;
      const int32_t cx = x, cy = y;
      if (r0 + DYN_WAVE < n_q) fetch(beg_q + r0 + DYN_WAVE, n_q - r0 - DYN_WAVE);
      else fetch(beg_n, n_n);
      acc += have ? (uint64_t)((int64_t)cx + (int64_t)cy) : 0;
      orv |= have ? (uint32_t)(cx | cy) : 0u;
      if (keep == 0) continue;
      const int32_t thr = __builtin_amdgcn_readlane(best, keep - 1);
      const bool mine = have && cx > thr;          // a value <= thr has `keep` kept values ahead of it
      uint64_t mask = __ballot(mine);
      if (mask == 0) continue;
      if (__popcll(mask) * 10 > keep * 16) {
        // rounds of maximum extraction over kept and new values; a taken value leaves its lane
        int32_t bv = best, cv = mine ? cx : -1, nb = -1;
        for (int i = 0; i < keep; ++i) {
          const int32_t mx = wave_max_i32(max(bv, cv));
          if (mx < 0) break;
          const uint64_t ub = __ballot(bv == mx);
          if (ub) {
            if (lane == (int)__builtin_ctzll(ub)) bv = -1;
          } else {
            const uint64_t uc = __ballot(cv == mx);
            if (lane == (int)__builtin_ctzll(uc)) cv = -1;
          }
          if (lane == i) nb = mx;
        }
        best = nb;
      } else {
        int rb = lane;      // position of my kept value: the kept values before it + new values above it
        int rc = 0;         // position of my new value: kept values >= it + new values that beat it
        while (mask) {
          const int u = __builtin_ctzll(mask);
          mask &= mask - 1;
          const int32_t v = __builtin_amdgcn_readlane(cx, u);
          const int n_ge = __popcll(__ballot(best >= v));
          rb += (v > best) ? 1 : 0;
          rc += (v > cx || (v == cx && u < lane)) ? 1 : 0;
          if (lane == u) rc += n_ge;
        }
        // the positions are a permutation of 0 .. 63 + (new values): every slot below 64 is written once
        if (rb < DYN_WAVE) buf[rb] = best;
        if (mine && rc < DYN_WAVE) buf[rc] = cx;
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        best = buf[lane];
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
      }
    }
    // the tick's token sum: 32-bit lanes when every lane's sum is small enough for it
    uint64_t tok;
    if (__ballot((acc >> 25) != 0) == 0) tok = wave_sum_u32((uint32_t)acc);
    else tok = wave_sum_u64(acc);
    if (__ballot((int32_t)orv < 0)) neg_mask |= 1u << q;
    if (lane == q) load_l = div_by((double)tok, a.tick_s, a.r_tick);
    const int n_top = keep < n_q ? keep : n_q;
    if (lane < n_top) a.top[(c * DYN_TICK_TOP + lane) * T + q] = best;   // [cell][position][tick]
  }
  if (lane < T) {
    const int64_t f = f0 + (int64_t)lane * G;
    TickRec r;
    r.load = load_l;
    r.cnt = cnt_l;
    r.plan = plan;
    a.rec[c * T + lane] = r;
    // every fine cell writes its own status byte: nothing to clear beforehand
    a.cstat[f] = (uint8_t)(bad_l | (((neg_mask >> lane) & 1u) ? DYN_WS_BAD_REQUEST : 0u) |
                           ((deep && lane == 0) ? DYN_WS_TICK_RANK : 0u));
  }
  if (c == 0 && lane == 0) {                     // single writer of the header
    a.header->status = 0u;
    a.header->kind = DYN_WS_KIND_CELLS;
    a.header->cells = cells * T;
    *a.merge_count = 0u;                       // filled by the evaluation kernel that runs next
  }
}

// ---- evaluation of the (cell, configuration) space -----------------------------------------------
// A tick's candidates (descending input lengths x its prefill time) against the sorted list
// s[0] >= ... >= s[JF-1]: once one of them cannot enter the list in any lane, the rest of
// that tick cannot either.
template <int JF>
__device__ __forceinline__ void offer_tick(double (&s)[JF], const int32_t* s_top, int T, int q, int nc, double pf) {
  for (int x = 0; x < nc; ++x) {
    double v = (double)s_top[x * T + q] * pf;
    if (__ballot(v > s[JF - 1]) == 0) break;
#pragma unroll
    for (int i = 0; i < JF; ++i) {
      const double hi = max_num(s[i], v);
      v = min_num(s[i], v);
      s[i] = hi;
    }
  }
}

// Cells whose j fits a short sorted list: the ticks are walked once, in time order, two at a
// time so that the two look-ups overlap.  The list starts with JF - j copies of +inf, so its
// last entry is the j-th largest of what was inserted.
template <int JF, bool SINGLE, bool TWO>
__device__ __forceinline__ void walk_ticks_short(const Lookup& L, int T, int j, const double* s_load, const int32_t* s_cnt,
                                                 const int32_t* s_top, double nd, double tick_s, double* e_out,
                                                 double* ttft_out, double* tbt_out, bool* ov_out) {
  double s[JF];
#pragma unroll
  for (int i = 0; i < JF; ++i) s[i] = i < JF - j ? __builtin_inf() : -__builtin_inf();
  double e = 0.0, tbmax = -__builtin_inf();
  bool ov = false;
  int q = 0;
  for (; q + 2 <= T; q += 2) {
    double pf0, tb0, pw0, pf1, tb1, pw1;
    const bool o0 = table_lookup<SINGLE, TWO>(L, s_load[q], &pf0, &tb0, &pw0);
    const bool o1 = table_lookup<SINGLE, TWO>(L, s_load[q + 1], &pf1, &tb1, &pw1);
    ov = ov | o0 | o1;
    e += (nd * pw0) * tick_s;                    // ticks in time order
    e += (nd * pw1) * tick_s;
    const int c0 = s_cnt[q], c1 = s_cnt[q + 1];
    if (c0 > 0) {                                // block-uniform
      tbmax = max_num(tbmax, tb0);
      offer_tick<JF>(s, s_top, T, q, c0 < j ? c0 : j, pf0);
    }
    if (c1 > 0) {
      tbmax = max_num(tbmax, tb1);
      offer_tick<JF>(s, s_top, T, q + 1, c1 < j ? c1 : j, pf1);
    }
  }
  if (q < T) {
    double pf0, tb0, pw0;
    ov = ov | table_lookup<SINGLE, TWO>(L, s_load[q], &pf0, &tb0, &pw0);
    e += (nd * pw0) * tick_s;
    const int c0 = s_cnt[q];
    if (c0 > 0) {
      tbmax = max_num(tbmax, tb0);
      offer_tick<JF>(s, s_top, T, q, c0 < j ? c0 : j, pf0);
    }
  }
  *e_out = e; *ttft_out = s[JF - 1]; *tbt_out = tbmax; *ov_out = ov;
}

// All other cells: every tick's tables are kept (the ticks are unrolled), then the TBT
// percentile takes ticks in descending TBT order until j requests are covered, and the TTFT
// percentile is j steps of a merge of the ticks' scaled candidate lists.
template <int TMAX, bool SINGLE, bool TWO>
__device__ __forceinline__ void walk_ticks_merge(const Lookup& L, int T, int j, const double* s_load, const int32_t* s_cnt,
                                                 const int32_t* s_top, double nd, double tick_s, double* e_out,
                                                 double* ttft_out, double* tbt_out, bool* ov_out) {
  const double ninf = -__builtin_inf();
  double pf[TMAX], tb[TMAX];
  double e = 0.0;
  bool ov = false;
  uint32_t nonempty = 0;
#pragma unroll
  for (int q = 0; q < TMAX; ++q) {
    pf[q] = 0.0;
    tb[q] = ninf;
    if (q < T) {
      double pw;
      ov = table_lookup<SINGLE, TWO>(L, s_load[q], &pf[q], &tb[q], &pw) | ov;
      e += (nd * pw) * tick_s;
      if (s_cnt[q] > 0) nonempty |= 1u << q;
    }
  }
  {
    uint32_t avail = nonempty;        // a tick without requests contributes no TBT sample
    int need = j;
    double val = 0.0;
    for (int it = 0; it < TMAX && need > 0; ++it) {
      double best = ninf;
      int bi = 0;
#pragma unroll
      for (int q = 0; q < TMAX; ++q) {
        const bool better = ((avail >> q) & 1u) && tb[q] > best;
        best = better ? tb[q] : best;
        bi = better ? q : bi;
      }
      avail &= ~(1u << bi);
      need -= s_cnt[bi];
      val = best;
    }
    *tbt_out = val;
  }
  {
    double h[TMAX];
    int pos[TMAX];
#pragma unroll
    for (int q = 0; q < TMAX; ++q) {
      pos[q] = 0;
      h[q] = ((nonempty >> q) & 1u) ? (double)s_top[q] * pf[q] : ninf;
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
      const double nh = more ? (double)s_top[np * T + bi] * bpf : ninf;
#pragma unroll
      for (int q = 0; q < TMAX; ++q) {
        const bool hit = q == bi;
        pos[q] = hit ? np : pos[q];
        h[q] = hit ? nh : h[q];
      }
    }
    *ttft_out = val;
  }
  *e_out = e; *ov_out = ov;
}

// What the cell kernel decided about one cell (block-uniform).
struct CellPlan {
  int j;           // 0 = empty cell
  bool deep, by_merge;
};
__device__ __forceinline__ CellPlan plan_cell(int32_t plan) {
  CellPlan p;
  p.j = plan & 0xFF;                            // the percentile is the j-th largest value
  p.deep = p.j > DYN_TICK_TOP;                  // beyond the extracted candidates: not evaluated
  p.by_merge = (plan & DYN_PLAN_MERGE) != 0;
  return p;
}

// Per-thread state of one configuration inside a (class, tile) block.
struct CfgState {
  Lookup L;
  double nd, slo_ttft, slo_tbt, idle_term;
  uint32_t fl_budget, koff;
  int k, k_raw, lane, wslot;
  bool live;
};

// The configuration's constants: `g` and `tile` are block-uniform; the table rows are either the
// block's LDS copy (LDS) or global memory.
template <bool LDS>
__device__ __forceinline__ void load_config(const TickArgs& a, int g, int tile, const double* s_tab, const double* s_rgp,
                                            const double* s_rinv, const double* s_thr, const uint16_t* s_js,
                                            CfgState* st) {
  const SpaceArgs& sa = a.s;
  const int n_rho = sa.n_rho;
  st->k_raw = tile * sa.tile + threadIdx.x;
  st->live = st->k_raw < sa.K;            // every lane stays alive for the wave reduction
  st->k = st->live ? st->k_raw : sa.K - 1;
  const DevCfg c = sa.cfg[st->k];
  const size_t grow = (size_t)g * sa.n_tp_f;
  const double ml_lo = sa.ml[grow + c.row_lo], ml_hi = sa.ml[grow + c.row_hi];
  const double p0_lo = sa.pw0[grow + c.row_lo], p0_hi = sa.pw0[grow + c.row_hi];
  const bool two_rows = c.u != 0.0;
  Lookup& L = st->L;
  L.u = c.u;
  L.omu = 1.0 - c.u;
  const double ml = two_rows ? L.omu * ml_lo + c.u * ml_hi : ml_lo;
  L.den = c.nd * ml;
  L.rden = 1.0 / L.den;
  L.rho_max = s_rgp[n_rho];
  L.bucket_scale = sa.bucket_scale;
  L.rgp = s_rgp; L.rinv = s_rinv; L.js = s_js; L.thr = s_thr; L.n_rho = n_rho;
  if (LDS) {      // kept apart so that the address space of the rows is known at compile time
    L.lo = s_tab + (size_t)c.slot_lo * DYN_SLOT_STRIDE(n_rho);
    L.hi = s_tab + (size_t)c.slot_hi * DYN_SLOT_STRIDE(n_rho);
  } else {
    L.lo = sa.tab + (grow + c.row_lo) * 3 * n_rho;
    L.hi = sa.tab + (grow + c.row_hi) * 3 * n_rho;
  }
  st->nd = c.nd;
  st->slo_ttft = sa.slo_ttft[g];
  st->slo_tbt = sa.slo_tbt[g];
  const int32_t bud = sa.budget[g];
  st->fl_budget = (bud > 0 && c.gpus > bud) ? DYN_F_BUDGET : 0u;
  const double pw0 = two_rows ? L.omu * p0_lo + c.u * p0_hi : p0_lo;
  st->idle_term = sa.idle_w * ((c.nd * pw0) * a.window_s);
  st->lane = threadIdx.x & (DYN_WAVE - 1);
  st->wslot = tile * (sa.tile / DYN_WAVE) + (int)(threadIdx.x / DYN_WAVE);
  st->koff = (uint32_t)st->k * 8u;
}

// One flat loop over the rows a tile needs: the loads of different rows are in flight together.
__device__ __forceinline__ void stage_rows(const SpaceArgs& sa, int g, int tile, double* s_tab) {
  const int per_slot = 3 * sa.n_rho, total = sa.n_slot * per_slot;
  const int32_t* rows = sa.tile_rows + tile * sa.n_slot;
  const double* base = sa.tab + (size_t)g * sa.n_tp_f * per_slot;
#pragma unroll 4
  for (int i = threadIdx.x; i < total; i += blockDim.x) {
    const int slot = i / per_slot;
    const int row = rows[slot];
    s_tab[slot * DYN_SLOT_STRIDE(sa.n_rho) + (i - slot * per_slot)] = base[(size_t)(row < 0 ? 0 : row) * per_slot + (i - slot * per_slot)];
  }
}
template <bool SINGLE>
__device__ __forceinline__ void stage_grid(const TickArgs& a, double* s_rgp, double* s_thr, uint16_t* s_js) {
  const SpaceArgs& sa = a.s;
  for (int i = threadIdx.x; i < 2 * sa.n_rho + 3; i += blockDim.x) s_rgp[i] = sa.gridpack[i];
  for (int i = threadIdx.x; i <= sa.n_bucket; i += blockDim.x) {
    s_js[i] = (uint16_t)(SINGLE ? a.tstart[i] : sa.jstart[i]);
    if (SINGLE) s_thr[i] = a.thr[i];
  }
}

// Flags, streaming stores of the four outputs and the wave's partial selection for one cell.
__device__ __forceinline__ void emit_cell(const SpaceArgs& sa, const CfgState& st, size_t cell, bool empty, bool ov, double e,
                                          double p_ttft, double p_tbt) {
  uint32_t fl = st.fl_budget;
  if (ov) fl |= DYN_F_OVERLOAD;
  if (p_ttft > st.slo_ttft) fl |= DYN_F_TTFT;
  if (p_tbt > st.slo_tbt) fl |= DYN_F_TBT;
  if (!fl) fl = DYN_F_FEASIBLE;
  if (empty) fl |= DYN_F_EMPTY;
  if (st.live) {
    const size_t row = cell * (size_t)sa.K;
    __builtin_nontemporal_store(e, (double*)((char*)(sa.energy + row) + st.koff));
    __builtin_nontemporal_store(p_ttft, (double*)((char*)(sa.p99_ttft + row) + st.koff));
    __builtin_nontemporal_store(p_tbt, (double*)((char*)(sa.p99_tbt + row) + st.koff));
    __builtin_nontemporal_store((uint8_t)fl, (sa.flags + row) + (uint32_t)st.k);
  }
  // least cost among this wave's feasible configurations (costs >= +0 order like their bits)
  const bool feas = st.live && (fl & DYN_F_FEASIBLE);
  const double cost = e + st.idle_term;
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
  if (st.lane == wl) {
    SelPart p;
    p.cost = win ? cost : __builtin_inf();
    p.energy = win ? e : __builtin_inf();
    p.k = win ? st.k_raw : -1;
    p.pad = 0;
    sa.part[cell * (size_t)sa.n_wslot + st.wslot] = p;
  }
}

// Empty cells, cells beyond DYN_TICK_TOP (not evaluated) and cells with j <= kFastDepth whose
// non-empty ticks all hold at least j requests (the TBT percentile is then the largest tick
// TBT).  A block walks a run of windows of one (class, tile); the other cells are put on a
// list for tick_merge_kernel.  The next cell's candidate lists are kept in flight (NPRE
// registers per thread) while the current one is evaluated.
// LDS: [table rows n_slot*3*n_rho] [padded load grid n_rho+2] [reciprocal spacings n_rho+1]
//      [SINGLE: grid point per bucket, n_bucket+1]
//      [per window of the block, per tick: load] [the same: request count] [per window: plan]
//      [two buffers of candidate lists, [position][tick]] [bucket index (16-bit)]
template <bool LDS, bool SINGLE, bool TWO>
__global__ __launch_bounds__(DYN_MAX_TILE) __attribute__((amdgpu_waves_per_eu(4, 4))) void tick_space_kernel(TickArgs a) {
  constexpr int NPRE = kFastDepth * DYN_TICK_MAX / DYN_WAVE;   // blocks have at least 64 threads
  extern __shared__ double smem[];
  const SpaceArgs& sa = a.s;
  const int tile = blockIdx.x % sa.n_tile;
  const int g = (blockIdx.x / sa.n_tile) % sa.G;
  const int chunk = blockIdx.x / (sa.n_tile * sa.G);
  const int n_rho = sa.n_rho, T = a.n_tick;
  const int w0 = chunk * sa.win_per_block;
  const int w1 = min(w0 + sa.win_per_block, sa.n_window);

  double* s_tab = smem;
  double* s_rgp = smem + (LDS ? (size_t)sa.n_slot * DYN_SLOT_STRIDE(n_rho) : 0);
  double* s_rinv = s_rgp + (n_rho + 2);
  double* s_thr = s_rinv + (n_rho + 1);                         // [n_bucket + 1] when SINGLE
  double* s_load = s_thr + (SINGLE ? sa.n_bucket + 1 : 0);      // [win_per_block][T]
  int32_t* s_cnt = (int32_t*)(s_load + sa.win_per_block * T);   // [win_per_block][T] requests per tick
  int32_t* s_plan = s_cnt + sa.win_per_block * T;               // [win_per_block]
  int32_t* s_top = s_plan + sa.win_per_block;                   // [2][DYN_TICK_TOP][T]
  uint16_t* s_js = (uint16_t*)(s_top + 2 * T * DYN_TICK_TOP);   // [n_bucket + 1]

  if (LDS) stage_rows(sa, g, tile, s_tab);
  stage_grid<SINGLE>(a, s_rgp, s_thr, s_js);
  for (int i = threadIdx.x; i < (w1 - w0) * T; i += blockDim.x) {   // the ticks of this block's cells
    const int dw = i / T, q = i - dw * T;
    const TickRec r = a.rec[((size_t)(w0 + dw) * sa.G + g) * T + q];
    s_load[i] = r.load;
    s_cnt[i] = r.cnt;
    if (q == 0) s_plan[dw] = r.plan;
  }
  __syncthreads();
  CfgState st;
  load_config<LDS>(a, g, tile, s_tab, s_rgp, s_rinv, s_thr, s_js, &st);

  // candidate lists of a cell: the first j * T words of its block of DYN_TICK_TOP * T
  int32_t pre[NPRE];
  auto prefetch = [&](int w) {
    if (w >= w1) return;
    const CellPlan p = plan_cell(s_plan[w - w0]);
    if (p.by_merge || p.j == 0 || p.deep) return;
    const int32_t* src = a.top + ((size_t)w * sa.G + g) * DYN_TICK_TOP * T;
    const int n = p.j * T;                     // at most kFastDepth * DYN_TICK_MAX
#pragma unroll
    for (int r = 0; r < NPRE; ++r) {
      const int i = threadIdx.x + r * blockDim.x;
      if (i < n) pre[r] = src[i];
    }
  };
  prefetch(w0);
  int buf = 0;
  for (int w = w0; w < w1; ++w) {
    const size_t cell = (size_t)w * sa.G + g;
    const int32_t* cnt_w = s_cnt + (w - w0) * T;
    const double* load_w = s_load + (w - w0) * T;
    const CellPlan pl = plan_cell(s_plan[w - w0]);
    const int j = pl.j;
    const bool deep = pl.deep, empty = j == 0;
    if (pl.by_merge) {                           // block-uniform: the other kernel takes this cell
      if (tile == 0 && threadIdx.x == 0) a.merge_list[atomicAdd(a.merge_count, 1u)] = (uint32_t)cell;
      prefetch(w + 1);
      continue;
    }
    // two buffers: the lists of the cell before this one may still be read by slower waves
    int32_t* top_w = s_top + buf * (T * DYN_TICK_TOP);
    buf ^= 1;
    if (!empty && !deep) {
      const int n = j * T;
#pragma unroll
      for (int r = 0; r < NPRE; ++r) {
        const int i = threadIdx.x + r * blockDim.x;
        if (i < n) top_w[i] = pre[r];
      }
    }
    __syncthreads();
    prefetch(w + 1);

    double e, p_ttft, p_tbt;
    bool ov;
    const int jl = deep ? 0 : j;               // no candidates are read for empty or unevaluated cells
    if (jl <= 4) walk_ticks_short<4, SINGLE, TWO>(st.L, T, jl, load_w, cnt_w, top_w, st.nd, a.tick_s, &e, &p_ttft, &p_tbt, &ov);
    else if (jl <= 8) walk_ticks_short<8, SINGLE, TWO>(st.L, T, jl, load_w, cnt_w, top_w, st.nd, a.tick_s, &e, &p_ttft, &p_tbt, &ov);
    else walk_ticks_short<kFastDepth, SINGLE, TWO>(st.L, T, jl, load_w, cnt_w, top_w, st.nd, a.tick_s, &e, &p_ttft, &p_tbt, &ov);
    if (empty) p_ttft = p_tbt = 0.0;
    if (deep) p_ttft = p_tbt = __builtin_inf();   // reported through the status word
    emit_cell(sa, st, cell, empty, ov, e, p_ttft, p_tbt);
  }
}

// The cells the kernel above listed, one (cell, tile) item at a time, items dealt round-robin
// to a fixed grid so that runs of heavy cells spread over the chip.  The table rows and the
// configuration are reloaded only when the item's (class, tile) differs from the previous one.
// LDS: [table rows] [load grid] [reciprocal spacings] [SINGLE: grid point per bucket]
//      [per tick: load] [per tick: request count] [candidate lists [position][tick]] [bucket index]
template <bool LDS, bool SINGLE, bool TWO>
__global__ __launch_bounds__(DYN_MAX_TILE) void tick_merge_kernel(TickArgs a) {
  extern __shared__ double smem[];
  const SpaceArgs& sa = a.s;
  const int n_rho = sa.n_rho, T = a.n_tick;
  double* s_tab = smem;
  double* s_rgp = smem + (LDS ? (size_t)sa.n_slot * DYN_SLOT_STRIDE(n_rho) : 0);
  double* s_rinv = s_rgp + (n_rho + 2);
  double* s_thr = s_rinv + (n_rho + 1);
  double* s_load = s_thr + (SINGLE ? sa.n_bucket + 1 : 0);      // [T]
  int32_t* s_cnt = (int32_t*)(s_load + T);                      // [T]
  int32_t* s_top = s_cnt + T;                                   // [DYN_TICK_TOP][T]
  uint16_t* s_js = (uint16_t*)(s_top + T * DYN_TICK_TOP);       // [n_bucket + 1]

  const uint32_t n_item = *a.merge_count * (uint32_t)sa.n_tile;  // complete: written by the previous kernel
  if (blockIdx.x >= n_item) return;                              // block-uniform
  stage_grid<SINGLE>(a, s_rgp, s_thr, s_js);
  CfgState st;
  int cur_g = -1, cur_tile = -1;
  for (uint32_t item = blockIdx.x; item < n_item; item += gridDim.x) {
    const size_t cell = a.merge_list[item / sa.n_tile];
    const int tile = (int)(item % sa.n_tile);
    const int g = (int)(cell % sa.G);
    __syncthreads();                           // the previous item's LDS data has been consumed
    const bool fresh = g != cur_g || tile != cur_tile;
    if (LDS && fresh) stage_rows(sa, g, tile, s_tab);
    int j = 0;
    {
      const TickRec* rec = a.rec + cell * T;
      j = rec[0].plan & 0xFF;                  // 1 .. DYN_TICK_TOP for a listed cell
      for (int q = threadIdx.x; q < T; q += blockDim.x) {
        const TickRec r = rec[q];
        s_load[q] = r.load;
        s_cnt[q] = r.cnt;
      }
      const int32_t* src = a.top + cell * DYN_TICK_TOP * T;
      for (int i = threadIdx.x; i < j * T; i += blockDim.x) s_top[i] = src[i];
    }
    __syncthreads();
    if (fresh) {
      load_config<LDS>(a, g, tile, s_tab, s_rgp, s_rinv, s_thr, s_js, &st);
      cur_g = g;
      cur_tile = tile;
    }
    double e, p_ttft, p_tbt;
    bool ov;
    // the ticks are unrolled: take the smallest instance that holds them (block-uniform)
    if (T <= 4) walk_ticks_merge<4, SINGLE, TWO>(st.L, T, j, s_load, s_cnt, s_top, st.nd, a.tick_s, &e, &p_ttft, &p_tbt, &ov);
    else if (T <= 8) walk_ticks_merge<8, SINGLE, TWO>(st.L, T, j, s_load, s_cnt, s_top, st.nd, a.tick_s, &e, &p_ttft, &p_tbt, &ov);
    else if (T <= 12) walk_ticks_merge<12, SINGLE, TWO>(st.L, T, j, s_load, s_cnt, s_top, st.nd, a.tick_s, &e, &p_ttft, &p_tbt, &ov);
    else walk_ticks_merge<DYN_TICK_MAX, SINGLE, TWO>(st.L, T, j, s_load, s_cnt, s_top, st.nd, a.tick_s, &e, &p_ttft, &p_tbt, &ov);
    emit_cell(sa, st, cell, false, ov, e, p_ttft, p_tbt);
  }
}

size_t tick_lds_tail(int32_t n_rho, int32_t n_bucket, int32_t n_tick, int32_t win_per_block, bool single) {
  return (size_t)(2 * n_rho + 3) * sizeof(double) + (single ? ((size_t)n_bucket + 1) * sizeof(double) : 0) +
         (size_t)win_per_block * (n_tick * (sizeof(double) + sizeof(int32_t)) + sizeof(int32_t)) +
         (size_t)2 * n_tick * DYN_TICK_TOP * sizeof(int32_t) + ((size_t)n_bucket + 1) * sizeof(uint16_t) + 8;
}

constexpr int kMergeBlocks = 1024;

template <bool LDS, bool SINGLE, bool TWO>
void launch_both(const TickArgs& a, dim3 grid, dim3 block, size_t lds, hipStream_t s) {
  {
    DynTimed timed(DYN_K_TICK_SPACE, s);
    hipLaunchKernelGGL((tick_space_kernel<LDS, SINGLE, TWO>), grid, block, lds, s, a);
  }
  // the merge kernel's LDS needs are within the first kernel's (one window, one list buffer)
  DynTimed timed(DYN_K_TICK_MERGE, s);
  hipLaunchKernelGGL((tick_merge_kernel<LDS, SINGLE, TWO>), dim3(kMergeBlocks), block, lds, s, a);
}
template <bool LDS, bool SINGLE>
void launch_rows(const TickArgs& a, dim3 grid, dim3 block, size_t lds, hipStream_t s) {
  if (a.any_two_rows) launch_both<LDS, SINGLE, true>(a, grid, block, lds, s);
  else launch_both<LDS, SINGLE, false>(a, grid, block, lds, s);
}

}  // namespace

hipError_t dyn_launch_tick_cell(const TickCellArgs& a, hipStream_t s) {
  const int64_t cells = (int64_t)a.n_window * a.G;
  const int64_t blocks = (cells + kWavesPerBlock - 1) / kWavesPerBlock;
  DynTimed timed(DYN_K_TICK_TOP, s);
  hipLaunchKernelGGL(tick_cell_kernel, dim3((unsigned)blocks), dim3(kWavesPerBlock * DYN_WAVE), 0, s, a);
  return hipGetLastError();
}

hipError_t dyn_launch_tick_space(const TickArgs& a, hipStream_t s) {
  const SpaceArgs& sa = a.s;
  const int n_chunk = (sa.n_window + sa.win_per_block - 1) / sa.win_per_block;
  const dim3 grid((unsigned)((size_t)n_chunk * sa.G * sa.n_tile)), block(sa.tile);
  const size_t tab = (size_t)sa.n_slot * DYN_SLOT_STRIDE(sa.n_rho) * sizeof(double);
  // Preferences when LDS is short: keep the table rows in LDS first, the per-bucket grid
  // points second (without them the bracket is searched; without the rows the tables are
  // read from global memory).
  bool single = a.single_point;
  size_t tail = tick_lds_tail(sa.n_rho, sa.n_bucket, a.n_tick, sa.win_per_block, single);
  if (single && tail + tab > DYN_LDS_BUDGET) {
    single = false;
    tail = tick_lds_tail(sa.n_rho, sa.n_bucket, a.n_tick, sa.win_per_block, false);
  }
  const bool lds = sa.n_slot > 0 && tab + tail <= DYN_LDS_BUDGET;
  if (!lds && tail > DYN_LDS_BUDGET) return hipErrorInvalidValue;
  const size_t bytes = (lds ? tab : 0) + tail;
  if (lds) {
    if (single) launch_rows<true, true>(a, grid, block, bytes, s);
    else launch_rows<true, false>(a, grid, block, bytes, s);
  } else {
    if (single) launch_rows<false, true>(a, grid, block, bytes, s);
    else launch_rows<false, false>(a, grid, block, bytes, s);
  }
  return hipGetLastError();
}
