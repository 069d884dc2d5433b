// Evaluation of the search space: one thread per candidate configuration, looping over a
// run of windows of one request class.  Everything that depends only on (class,
// configuration) is hoisted out of the window loop; the table rows the block's
// configurations touch are staged in LDS once per block.  Per (cell, configuration) the
// kernel follows the profile-lookup definition of Section IV-A literally: per-instance
// load on the table axis, bracket, linear interpolation along load on the bracketing
// frequency rows and then along frequency, P99 TTFT = P99 input length x prefill
// ms/token, energy = instances x power x window, feasibility per Eq. 1.
// Output rows are written with the configuration index fastest: 8-byte stores, 512
// contiguous bytes per wave and array.
//
// The two divisions per entry (load / capacity, position inside the load bracket) have
// divisors that do not depend on the window: their correctly rounded reciprocals are
// computed once (per thread, per grid interval) and each quotient is then formed from the
// reciprocal with two residual steps (div_by), which returns the correctly rounded a/b.
//
// With the fused selection, each wave also reduces the least cost among its feasible
// configurations (Section IV-B "Scale-up/down") and one lane writes a partial record.
#include "dyn_device.h"

namespace {

// LDS: [table rows n_slot*3*n_rho] [padded load grid n_rho+2] [padded reciprocal spacings n_rho+1]
//      [cell records win_per_block] [bucket index n_bucket+1 (16-bit)]
template <bool LDS, bool SEL, bool ONE_STEP>
__global__ __launch_bounds__(DYN_MAX_TILE) void space_kernel(SpaceArgs a) {
  extern __shared__ double smem[];
  // block -> (window chunk, class, tile); tile fastest
  const int tile = blockIdx.x % a.n_tile;
  const int g = (blockIdx.x / a.n_tile) % a.G;
  const int chunk = blockIdx.x / (a.n_tile * a.G);
  const int n_rho = a.n_rho;

  double* s_tab = smem;                                              // [n_slot][3][n_rho]
  double* s_rgp = smem + (LDS ? (size_t)a.n_slot * 3 * n_rho : 0);   // s_rgp[i+1] = rho[i]; -inf, +inf pads
  double* s_rinv = s_rgp + (n_rho + 2);                              // s_rinv[i+1] = 1/(rho[i+1]-rho[i]); 0 pads
  CellRec* s_rec = (CellRec*)(s_rinv + (n_rho + 1));                 // [win_per_block]
  uint16_t* s_js = (uint16_t*)(s_rec + a.win_per_block);             // [n_bucket + 1]

  const int w0 = chunk * a.win_per_block;
  const int w1 = min(w0 + a.win_per_block, a.n_window);
  if (LDS) {
    const int per_slot = 3 * n_rho;
    for (int slot = 0; slot < a.n_slot; ++slot) {
      const int row = a.tile_rows[tile * a.n_slot + slot];       // wave-uniform; -1 = unused slot
      const double* src = a.tab + ((size_t)g * a.n_tp_f + (row < 0 ? 0 : row)) * per_slot;
      for (int i = threadIdx.x; i < per_slot; i += blockDim.x) s_tab[slot * per_slot + i] = src[i];
    }
  }
  for (int i = threadIdx.x; i < 2 * n_rho + 3; i += blockDim.x) s_rgp[i] = a.gridpack[i];
  for (int i = threadIdx.x; i <= a.n_bucket; i += blockDim.x) s_js[i] = (uint16_t)a.jstart[i];
  // the cells of this block's run of windows (load, P99 input length)
  for (int i = threadIdx.x; i < w1 - w0; i += blockDim.x) s_rec[i] = a.rec[(size_t)(w0 + i) * a.G + g];
  __syncthreads();

  const int k_raw = tile * a.tile + threadIdx.x;
  // with the fused selection every lane of a wave stays alive (the wave reduction needs full
  // waves); lanes past the last configuration compute on configuration K-1 and store nothing
  const bool live = k_raw < a.K;
  if (!SEL && !live) return;
  const int k = live ? k_raw : a.K - 1;

  const DevCfg c = a.cfg[k];
  const bool two_rows = c.u != 0.0;
  const double omu = 1.0 - c.u;
  const double* mlrow = a.ml + (size_t)g * a.n_tp_f;
  const double ml = two_rows ? omu * mlrow[c.row_lo] + c.u * mlrow[c.row_hi] : mlrow[c.row_lo];
  const double den = c.nd * ml;
  const double rden = 1.0 / den;
  const double rho_max = s_rgp[n_rho];
  const double slo_ttft = a.slo_ttft[g], slo_tbt = a.slo_tbt[g];
  const int32_t bud = a.budget[g];
  const uint32_t fl_budget = (bud > 0 && c.gpus > bud) ? DYN_F_BUDGET : 0u;
  double idle_term = 0.0;
  if (SEL) {
    const double* p0 = a.pw0 + (size_t)g * a.n_tp_f;
    const double pw0 = two_rows ? omu * p0[c.row_lo] + c.u * p0[c.row_hi] : p0[c.row_lo];
    idle_term = a.idle_w * ((c.nd * pw0) * a.window_s);
  }
  const int lane = threadIdx.x & (DYN_WAVE - 1);
  const int wslot = tile * (a.tile / DYN_WAVE) + (int)(threadIdx.x / DYN_WAVE);

  const double *lo_pf, *lo_tb, *lo_pw, *hi_pf, *hi_tb, *hi_pw;
  if (LDS) {
    lo_pf = s_tab + (size_t)c.slot_lo * 3 * n_rho; lo_tb = lo_pf + n_rho; lo_pw = lo_tb + n_rho;
    hi_pf = s_tab + (size_t)c.slot_hi * 3 * n_rho; hi_tb = hi_pf + n_rho; hi_pw = hi_tb + n_rho;
  } else {
    lo_pf = a.tab + ((size_t)g * a.n_tp_f + c.row_lo) * 3 * n_rho; lo_tb = lo_pf + n_rho; lo_pw = lo_tb + n_rho;
    hi_pf = a.tab + ((size_t)g * a.n_tp_f + c.row_hi) * 3 * n_rho; hi_tb = hi_pf + n_rho; hi_pw = hi_tb + n_rho;
  }
  const uint32_t koff = (uint32_t)k * 8u;   // byte offset of this lane inside an output row

  for (int w = w0; w < w1; ++w) {
    const size_t cell = (size_t)w * a.G + g;
    const CellRec rec = s_rec[w - w0];

    const double rho = div_by(rec.load, den, rden);
    const bool ov = rho > rho_max;
    const double rc = ov ? rho_max : rho;
    // bracket: largest j with rho[j] <= rc, at most n_rho-2; start from the bucket index
    // (rc <= rho_max keeps the bucket at or below n_bucket; a negative load maps to bucket 0)
    const int b = (int)(fmax(rc, 0.0) * a.bucket_scale);
    int j = s_js[b];                                   // <= n_rho-2 by construction
    double r0, r1, ri;
    if (ONE_STEP) {
      // the grid is coarse against the buckets: the bracket is j-1, j or j+1
      const double g0 = s_rgp[j + 1], g1 = s_rgp[j + 2];
      const bool down = g0 > rc && j > 0;
      const bool up = !down && g1 <= rc && j < n_rho - 2;
      j += up ? 1 : (down ? -1 : 0);
      r0 = s_rgp[j + 1]; r1 = s_rgp[j + 2]; ri = s_rinv[j + 1];
    } else {
      while (j > 0 && s_rgp[j + 1] > rc) --j;
      while (j < n_rho - 2 && s_rgp[j + 2] <= rc) ++j;
      r0 = s_rgp[j + 1]; r1 = s_rgp[j + 2]; ri = s_rinv[j + 1];
    }
    const double t = div_by(rc - r0, r1 - r0, ri);
    const double omt = 1.0 - t;

    double pf = omt * lo_pf[j] + t * lo_pf[j + 1];
    double tb = omt * lo_tb[j] + t * lo_tb[j + 1];
    double pw = omt * lo_pw[j] + t * lo_pw[j + 1];
    if (two_rows) {
      const double pf_b = omt * hi_pf[j] + t * hi_pf[j + 1];
      const double tb_b = omt * hi_tb[j] + t * hi_tb[j + 1];
      const double pw_b = omt * hi_pw[j] + t * hi_pw[j + 1];
      pf = omu * pf + c.u * pf_b;
      tb = omu * tb + c.u * tb_b;
      pw = omu * pw + c.u * pw_b;
    }
    const double p_ttft = rec.xp99 * pf;        // an empty cell has xp99 == 0
    const double p_tbt = tb * rec.nonempty;     // exact: times 1.0, or 0.0 for an empty cell
    const double e = (c.nd * pw) * a.window_s;

    uint32_t fl = fl_budget;
    if (ov) fl |= DYN_F_OVERLOAD;
    if (p_ttft > slo_ttft) fl |= DYN_F_TTFT;
    if (p_tbt > slo_tbt) fl |= DYN_F_TBT;
    if (!fl) fl = DYN_F_FEASIBLE;
    if (rec.nonempty == 0.0) fl |= DYN_F_EMPTY;

    if (live) {
      const size_t row = cell * (size_t)a.K;      // wave-uniform row start + 32-bit lane offset
      // streaming stores: the space is written once and is far larger than the caches
      __builtin_nontemporal_store(e, (double*)((char*)(a.energy + row) + koff));
      __builtin_nontemporal_store(p_ttft, (double*)((char*)(a.p99_ttft + row) + koff));
      __builtin_nontemporal_store(p_tbt, (double*)((char*)(a.p99_tbt + row) + koff));
      __builtin_nontemporal_store((uint8_t)fl, (a.flags + row) + (uint32_t)k);
    }
    if (SEL) {
      // Least cost among this wave's feasible configurations; costs are >= +0, so their bit
      // patterns order like unsigned integers: minimum of the high words, then of the low
      // words among the lanes that hold it.  The lowest lane (= lowest index) wins ties.
      const bool feas = live && (fl & DYN_F_FEASIBLE);
      const double cost = e + idle_term;
      const uint64_t bits = (uint64_t)__double_as_longlong(cost);
      const uint32_t hi = feas ? (uint32_t)(bits >> 32) : 0xFFFFFFFFu;
      const uint32_t lo = feas ? (uint32_t)bits : 0xFFFFFFFFu;
      const uint32_t mh = wave_min_u32(hi);
      uint64_t win = __ballot(feas && hi == mh);
      if (__popcll(win) > 1) {                     // wave-uniform: several lanes share the high word
        const uint32_t mlo = wave_min_u32(hi == mh ? lo : 0xFFFFFFFFu);
        win = __ballot(feas && hi == mh && lo == mlo);
      }
      const int wl = win ? __builtin_ctzll(win) : 0;     // wave-uniform
      if (lane == wl) {
        SelPart p;
        p.cost = win ? cost : __builtin_inf();
        p.energy = win ? e : __builtin_inf();
        p.k = win ? k_raw : -1;
        p.pad = 0;
        a.part[cell * (size_t)a.n_wslot + wslot] = p;
      }
    }
  }
}

template <bool LDS, bool SEL>
void launch_one_step(const SpaceArgs& a, dim3 grid, dim3 block, size_t lds, hipStream_t s) {
  if (a.one_step) hipLaunchKernelGGL((space_kernel<LDS, SEL, true>), grid, block, lds, s, a);
  else hipLaunchKernelGGL((space_kernel<LDS, SEL, false>), grid, block, lds, s, a);
}

}  // namespace

size_t dyn_space_lds_tail(int32_t n_rho, int32_t n_bucket, int32_t win_per_block) {
  return (size_t)(2 * n_rho + 3) * sizeof(double) + (size_t)win_per_block * sizeof(CellRec) +
         ((size_t)n_bucket + 1) * sizeof(uint16_t);
}

// Blocks of the evaluation kernel that one compute unit holds at a time for this shape (0 if the query fails).
int dyn_space_blocks_per_cu(const SpaceArgs& a) {
  const size_t lds_tab = (size_t)a.n_slot * 3 * a.n_rho * sizeof(double);
  const size_t lds = (a.n_slot > 0 ? lds_tab : 0) + dyn_space_lds_tail(a.n_rho, a.n_bucket, a.win_per_block);
  int n = 0;
  hipError_t e;
  if (a.n_slot > 0) {
    if (a.one_step) e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, space_kernel<true, true, true>, a.tile, lds);
    else e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, space_kernel<true, true, false>, a.tile, lds);
  } else {
    if (a.one_step) e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, space_kernel<false, true, true>, a.tile, lds);
    else e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, space_kernel<false, true, false>, a.tile, lds);
  }
  if (e != hipSuccess) { (void)hipGetLastError(); return 0; }
  return n;
}

hipError_t dyn_launch_space(const SpaceArgs& a, hipStream_t s) {
  const int n_chunk = (a.n_window + a.win_per_block - 1) / a.win_per_block;
  const size_t blocks = (size_t)n_chunk * a.G * a.n_tile;
  const size_t lds_tab = (size_t)a.n_slot * 3 * a.n_rho * sizeof(double);
  DynTimed timed(DYN_K_SPACE, s);
  const size_t lds = (a.n_slot > 0 ? lds_tab : 0) + dyn_space_lds_tail(a.n_rho, a.n_bucket, a.win_per_block);  // host keeps this <= 64 KB
  const dim3 grid((unsigned)blocks), block(a.tile);
  if (a.n_slot > 0) {
    if (a.part) launch_one_step<true, true>(a, grid, block, lds, s);
    else launch_one_step<true, false>(a, grid, block, lds, s);
  } else {
    if (a.part) launch_one_step<false, true>(a, grid, block, lds, s);
    else launch_one_step<false, false>(a, grid, block, lds, s);
  }
  return hipGetLastError();
}
