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
#include "dyn_internal.h"

namespace {

template <int CTRL>
__device__ __forceinline__ double dpp_mov_f64(double x) {
  const uint64_t b = (uint64_t)__double_as_longlong(x);
  const int lo = __builtin_amdgcn_update_dpp(0, (int)(uint32_t)b, CTRL, 0xF, 0xF, false);
  const int hi = __builtin_amdgcn_update_dpp(0, (int)(uint32_t)(b >> 32), CTRL, 0xF, 0xF, false);
  return __longlong_as_double((long long)(((uint64_t)(uint32_t)hi << 32) | (uint32_t)lo));
}
__device__ __forceinline__ double readlane_f64(double x, int lane) {
  const uint64_t b = (uint64_t)__double_as_longlong(x);
  const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)b, lane);
  const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(b >> 32), lane);
  return __longlong_as_double((long long)(((uint64_t)hi << 32) | lo));
}
__device__ __forceinline__ double min_no_nan(double a, double b) { return b < a ? b : a; }
// Minimum over the 64 lanes of a fully active wave (no NaNs): rotations inside each row of
// 16 lanes, then the four row minima are combined as scalars.
__device__ __forceinline__ double wave_min_f64(double x) {
  x = min_no_nan(x, dpp_mov_f64<0x121>(x));
  x = min_no_nan(x, dpp_mov_f64<0x122>(x));
  x = min_no_nan(x, dpp_mov_f64<0x124>(x));
  x = min_no_nan(x, dpp_mov_f64<0x128>(x));
  return min_no_nan(min_no_nan(readlane_f64(x, 0), readlane_f64(x, 16)),
                    min_no_nan(readlane_f64(x, 32), readlane_f64(x, 48)));
}

template <bool LDS, bool SEL>
__global__ __launch_bounds__(DYN_MAX_TILE) void space_kernel(SpaceArgs a) {
  extern __shared__ double smem[];
  // block -> (window chunk, class, tile); tile fastest
  const int tile = blockIdx.x % a.n_tile;
  const int g = (blockIdx.x / a.n_tile) % a.G;
  const int chunk = blockIdx.x / (a.n_tile * a.G);
  const int n_rho = a.n_rho;

  double* s_tab = smem;                                   // [n_slot][3][n_rho]
  double* s_rg = smem + (LDS ? (size_t)a.n_slot * 3 * n_rho : 0);   // [n_rho]
  int32_t* s_js = (int32_t*)(s_rg + n_rho);               // [n_bucket + 1]

  if (LDS) {
    const int per_slot = 3 * n_rho;
    for (int i = threadIdx.x; i < a.n_slot * per_slot; i += blockDim.x) {
      const int slot = i / per_slot, rem = i - slot * per_slot;
      const int q = rem / n_rho, j = rem - q * n_rho;
      const int row = a.tile_rows[tile * a.n_slot + slot];
      double v = 0.0;
      if (row >= 0) {
        const double* src = q == 0 ? a.pf : (q == 1 ? a.tb : a.pw);
        v = src[((size_t)g * a.n_tp_f + row) * n_rho + j];
      }
      s_tab[i] = v;
    }
  }
  for (int i = threadIdx.x; i < n_rho; i += blockDim.x) s_rg[i] = a.rg[i];
  for (int i = threadIdx.x; i <= a.n_bucket; i += blockDim.x) s_js[i] = a.jstart[i];
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
  const double rho_max = s_rg[n_rho - 1];
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
    const size_t ol = ((size_t)g * a.n_tp_f + c.row_lo) * n_rho, oh = ((size_t)g * a.n_tp_f + c.row_hi) * n_rho;
    lo_pf = a.pf + ol; lo_tb = a.tb + ol; lo_pw = a.pw + ol;
    hi_pf = a.pf + oh; hi_tb = a.tb + oh; hi_pw = a.pw + oh;
  }

  const int w0 = chunk * a.win_per_block;
  const int w1 = min(w0 + a.win_per_block, a.n_window);
  for (int w = w0; w < w1; ++w) {
    const size_t cell = (size_t)w * a.G + g;
    const CellRec rec = a.rec[cell];
    const bool empty = rec.xp99 < 0.0;

    const double rho = rec.load / den;
    const bool ov = rho > rho_max;
    const double rc = ov ? rho_max : rho;
    // bracket: largest j with rg[j] <= rc, at most n_rho-2; start from the bucket index
    int b = (int)(rc * a.bucket_scale);
    b = b < 0 ? 0 : (b > a.n_bucket ? a.n_bucket : b);
    int j = s_js[b];
    while (j > 0 && s_rg[j] > rc) --j;
    while (j < n_rho - 2 && s_rg[j + 1] <= rc) ++j;
    if (j > n_rho - 2) j = n_rho - 2;
    const double r0 = s_rg[j], r1 = s_rg[j + 1];
    const double t = (rc - r0) / (r1 - r0);
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
    const double p_ttft = empty ? 0.0 : rec.xp99 * pf;
    const double p_tbt = empty ? 0.0 : tb;
    const double e = (c.nd * pw) * a.window_s;

    uint32_t fl = fl_budget;
    if (ov) fl |= DYN_F_OVERLOAD;
    if (p_ttft > slo_ttft) fl |= DYN_F_TTFT;
    if (p_tbt > slo_tbt) fl |= DYN_F_TBT;
    if (!fl) fl = DYN_F_FEASIBLE;
    if (empty) fl |= DYN_F_EMPTY;

    if (live) {
      const size_t o = cell * (size_t)a.K + k;
      a.energy[o] = e;
      a.p99_ttft[o] = p_ttft;
      a.p99_tbt[o] = p_tbt;
      a.flags[o] = (uint8_t)fl;
    }
    if (SEL) {
      // least cost among this wave's feasible configurations; the lowest lane (= lowest
      // index) wins ties.  A feasible configuration whose cost is +inf still wins over none.
      const bool feas = live && (fl & DYN_F_FEASIBLE);
      const double cost = e + idle_term;
      const double mn = wave_min_f64(feas ? cost : __builtin_inf());
      const uint64_t win = __ballot(feas && cost == mn);
      const int wl = win ? __builtin_ctzll(win) : 0;        // wave-uniform
      const double e_win = readlane_f64(e, wl);
      if (lane == 0) {
        SelPart p;
        p.cost = __builtin_inf(); p.energy = __builtin_inf(); p.k = -1; p.pad = 0;
        if (win) {
          p.cost = mn;
          p.energy = e_win;
          p.k = k_raw + wl;          // lane 0 holds the wave's first configuration
        }
        a.part[cell * (size_t)a.n_wslot + wslot] = p;
      }
    }
  }
}

}  // namespace

hipError_t dyn_launch_space(const SpaceArgs& a, hipStream_t s) {
  const int n_chunk = (a.n_window + a.win_per_block - 1) / a.win_per_block;
  const size_t blocks = (size_t)n_chunk * a.G * a.n_tile;
  const size_t tail = (size_t)a.n_rho * sizeof(double) + ((size_t)a.n_bucket + 1) * sizeof(int32_t);
  const size_t lds_tab = (size_t)a.n_slot * 3 * a.n_rho * sizeof(double);
  DynTimed timed(DYN_K_SPACE, s);
  const size_t lds = (a.n_slot > 0 ? lds_tab : 0) + tail;   // the host keeps this within 64 KB
  const dim3 grid((unsigned)blocks), block(a.tile);
  if (a.n_slot > 0) {
    if (a.part) hipLaunchKernelGGL((space_kernel<true, true>), grid, block, lds, s, a);
    else hipLaunchKernelGGL((space_kernel<true, false>), grid, block, lds, s, a);
  } else {
    if (a.part) hipLaunchKernelGGL((space_kernel<false, true>), grid, block, lds, s, a);
    else hipLaunchKernelGGL((space_kernel<false, false>), grid, block, lds, s, a);
  }
  return hipGetLastError();
}
