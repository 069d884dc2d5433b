// Pools that mix instance types (Eq. 1 in full): per (window, class) cell the number of
// instances of every tensor parallelism, their frequency and the part of the load each type
// takes, so that the energy is least within the GPU budget and the SLO.
//
// The load is split in n_share equal shares; type i takes a_i of them and its n_i instances
// share that part equally.  The frequency of a type does not depend on the other types, so
// the search has two steps:
//   mixed_type_*_kernel   E_i(n, a) = least energy of n instances of type i carrying a shares
//                         over the frequencies that meet the SLO (Section IV-B "Scale-up/down":
//                         filter, then least energy), for every (cell, i, n, a);
//   mixed_combine_kernel  per cell a dynamic programme over the types, state = (GPUs used,
//                         shares assigned): D_{i+1}[u + n tp_i][s + a] = min(D_i[u][s] + E_i(n, a)).
// Rounded addition is monotone, so the minimum over the partial sums of a prefix followed by
// one more addition is the minimum over the extended sums: the programme returns exactly the
// least of the sums 0 + E_0 + E_1 + ... taken in type order, which is how the total is defined.
#include <algorithm>

#include "dyn_mixed.h"
#include "dyn_device.h"

namespace {

// Minimum over each row of 16 lanes, left in every lane of the row.
__device__ __forceinline__ uint32_t row_min_u32(uint32_t x) {
  x = min(x, (uint32_t)dpp_mov<0x121>((int)x));
  x = min(x, (uint32_t)dpp_mov<0x122>((int)x));
  x = min(x, (uint32_t)dpp_mov<0x124>((int)x));
  x = min(x, (uint32_t)dpp_mov<0x128>((int)x));
  return x;
}

// Block = (run of windows, class, type).  A thread is (entry, frequency): 16 entries of 16
// frequency lanes per pass over the type's entries.  The type's table rows (all frequencies)
// sit in LDS.
// LDS: [rows n_f*3*n_rho] [padded load grid n_rho+2] [reciprocal spacings n_rho+1]
//      [SINGLE: grid point per bucket n_bucket+1] [cell records win_per_block] [bucket index (16-bit)]
template <bool SINGLE>
__global__ __launch_bounds__(256) void mixed_type_kernel(MixedTypeArgs a) {
  extern __shared__ double smem[];
  const int n_rho = a.n_rho, n_f = a.n_f, S = a.n_share;
  const int i = blockIdx.x % a.n_tp;
  const int g = (blockIdx.x / a.n_tp) % a.G;
  const int chunk = blockIdx.x / (a.n_tp * a.G);
  const int n_ent = a.types.n_max[i] * S;          // entries of this type
  if (n_ent == 0) return;                          // block-uniform
  const int w0 = chunk * a.win_per_block;
  const int w1 = min(w0 + a.win_per_block, a.n_window);
  const int n_entry = a.types.off[a.n_tp];

  // rows one double apart from a multiple of the bank width: the 16 frequency lanes of an entry read
  // the same load bracket of 16 different rows, which would otherwise fall into one LDS bank
  const int row_stride = (3 * n_rho) | 1;
  double* s_tab = smem;                                        // [n_f][row_stride]: prefill, TBT, power
  double* s_rgp = s_tab + (size_t)n_f * row_stride;
  double* s_rinv = s_rgp + (n_rho + 2);
  double* s_thr = s_rinv + (n_rho + 1);
  CellRec* s_rec = (CellRec*)(s_thr + (SINGLE ? a.n_bucket + 1 : 0));
  uint16_t* s_js = (uint16_t*)(s_rec + a.win_per_block);

  {
    const double* src = a.tab + ((size_t)g * a.n_tp + i) * n_f * 3 * n_rho;   // the type's rows are contiguous
    for (int q = threadIdx.x; q < n_f * 3 * n_rho; q += blockDim.x) {
      const int r = q / (3 * n_rho);
      s_tab[r * row_stride + (q - r * 3 * n_rho)] = src[q];
    }
  }
  for (int q = threadIdx.x; q < 2 * n_rho + 3; q += blockDim.x) s_rgp[q] = a.gridpack[q];
  for (int q = threadIdx.x; q <= a.n_bucket; q += blockDim.x) {
    s_js[q] = (uint16_t)(SINGLE ? a.tstart[q] : a.jstart[q]);
    if (SINGLE) s_thr[q] = a.thr[q];
  }
  for (int q = threadIdx.x; q < w1 - w0; q += blockDim.x) s_rec[q] = a.rec[(size_t)(w0 + q) * a.G + g];
  __syncthreads();

  const int f = threadIdx.x & (DYN_MIXED_FREQ_LANES - 1);
  const int row = threadIdx.x / DYN_MIXED_FREQ_LANES;         // 0 .. 15
  const bool f_ok = f < n_f;
  const int fc = f_ok ? f : 0;
  const double ml = a.ml[((size_t)g * a.n_tp + i) * n_f + fc];
  const double slo_ttft = a.slo_ttft[g], slo_tbt = a.slo_tbt[g];
  Lookup L;
  L.u = 0.0; L.omu = 1.0;
  L.rho_max = s_rgp[n_rho];
  L.bucket_scale = a.bucket_scale;
  L.rgp = s_rgp; L.rinv = s_rinv; L.js = s_js; L.thr = s_thr; L.n_rho = n_rho;
  L.lo = s_tab + (size_t)fc * row_stride;
  L.hi = L.lo;
  const double sd = (double)S;

  for (int e0 = 0; e0 < n_ent; e0 += 256 / DYN_MIXED_FREQ_LANES) {
    const int e = e0 + row;
    const bool e_ok = e < n_ent;
    const int ec = e_ok ? e : 0;
    const int n = ec / S + 1, sh = ec % S + 1;
    const double nd = (double)n, ad = (double)sh;
    L.den = nd * ml;
    L.rden = 1.0 / L.den;
    for (int w = w0; w < w1; ++w) {
      const CellRec rec = s_rec[w - w0];
      const double ls = div_by(rec.load * ad, sd, a.r_share);      // the part of the load this type takes
      double pf, tb, pw;
      const bool ov = table_lookup<SINGLE, false>(L, ls, &pf, &tb, &pw);
      const double en = (nd * pw) * a.window_s;
      const double p_ttft = rec.xp99 * pf;
      const double p_tbt = tb * rec.nonempty;
      const bool ok = f_ok && !ov && !(p_ttft > slo_ttft) && !(p_tbt > slo_tbt);
      // least energy of the row's admissible lanes (energies are >= +0: their bits order as integers),
      // lowest frequency among equals; +inf when no lane is admissible
      const uint64_t bits = ok ? (uint64_t)__double_as_longlong(en) : 0x7FF0000000000000ull;
      const uint32_t hi = (uint32_t)(bits >> 32), lo = (uint32_t)bits;
      const uint32_t mh = row_min_u32(hi);
      const uint32_t mlw = row_min_u32(hi == mh ? lo : 0xFFFFFFFFu);
      const uint32_t fsel = row_min_u32((ok && hi == mh && lo == mlw) ? (uint32_t)f : 0xFFu);
      if (f == 0 && e_ok) {
        const size_t o = ((size_t)w * a.G + g) * n_entry + a.types.off[i] + e;
        a.type_energy[o] = __longlong_as_double((long long)(((uint64_t)mh << 32) | mlw));
        a.type_f[o] = fsel == 0xFFu ? (int8_t)-1 : (int8_t)fsel;
      }
    }
  }
}

// The same per-type energies with the frequencies walked by the thread: a thread is (entry, window), takes its
// share of the window's load once and keeps the least admissible energy over the frequencies in ascending order
// (strictly less replaces: the lowest frequency among equals), so nothing crosses lanes and every lane stores.
// The capacities n x max load and their reciprocals, which the other kernel forms per lane and pass, come from an
// LDS table [n_max][n_f] built once per block.  Chosen when that table fits beside the rows.
// LDS: as above, then [capacity n_max*n_f] [its reciprocal n_max*n_f]
template <bool SINGLE>
__global__ __launch_bounds__(256) void mixed_type_walk_kernel(MixedTypeArgs a) {
  extern __shared__ double smem[];
  const int n_rho = a.n_rho, n_f = a.n_f, S = a.n_share;
  const int i = blockIdx.x % a.n_tp;
  const int g = (blockIdx.x / a.n_tp) % a.G;
  const int chunk = blockIdx.x / (a.n_tp * a.G);
  const int n_max = a.types.n_max[i];
  const int n_ent = n_max * S;                     // entries of this type
  if (n_ent == 0) return;                          // block-uniform
  const int w0 = chunk * a.win_per_block;
  const int w1 = min(w0 + a.win_per_block, a.n_window);
  const int n_entry = a.types.off[a.n_tp];

  const int row_stride = (3 * n_rho) | 1;          // see mixed_type_kernel
  double* s_tab = smem;
  double* s_rgp = s_tab + (size_t)n_f * row_stride;
  double* s_rinv = s_rgp + (n_rho + 2);
  double* s_thr = s_rinv + (n_rho + 1);
  CellRec* s_rec = (CellRec*)(s_thr + (SINGLE ? a.n_bucket + 1 : 0));
  double* s_den = (double*)(s_rec + a.win_per_block);            // [n_max][n_f]
  double* s_rden = s_den + (size_t)n_max * n_f;
  uint16_t* s_js = (uint16_t*)(s_rden + (size_t)n_max * n_f);

  {
    const double* src = a.tab + ((size_t)g * a.n_tp + i) * n_f * 3 * n_rho;   // the type's rows are contiguous
    for (int q = threadIdx.x; q < n_f * 3 * n_rho; q += blockDim.x) {
      const int r = q / (3 * n_rho);
      s_tab[r * row_stride + (q - r * 3 * n_rho)] = src[q];
    }
  }
  for (int q = threadIdx.x; q < 2 * n_rho + 3; q += blockDim.x) s_rgp[q] = a.gridpack[q];
  for (int q = threadIdx.x; q <= a.n_bucket; q += blockDim.x) {
    s_js[q] = (uint16_t)(SINGLE ? a.tstart[q] : a.jstart[q]);
    if (SINGLE) s_thr[q] = a.thr[q];
  }
  for (int q = threadIdx.x; q < w1 - w0; q += blockDim.x) s_rec[q] = a.rec[(size_t)(w0 + q) * a.G + g];
  for (int q = threadIdx.x; q < n_max * n_f; q += blockDim.x) {
    const int n = q / n_f + 1, f = q - (n - 1) * n_f;
    const double den = (double)n * a.ml[((size_t)g * a.n_tp + i) * n_f + f];
    s_den[q] = den;
    s_rden[q] = 1.0 / den;
  }
  __syncthreads();

  const double slo_ttft = a.slo_ttft[g], slo_tbt = a.slo_tbt[g];
  Lookup L;
  L.u = 0.0; L.omu = 1.0;
  L.rho_max = s_rgp[n_rho];
  L.bucket_scale = a.bucket_scale;
  L.rgp = s_rgp; L.rinv = s_rinv; L.js = s_js; L.thr = s_thr; L.n_rho = n_rho;
  const double sd = (double)S;
  const int64_t n_pair = (int64_t)n_ent * (w1 - w0);              // (window, entry), entry fastest
  for (int64_t idx = threadIdx.x; idx < n_pair; idx += blockDim.x) {
    const int dw = (int)(idx / n_ent), e = (int)(idx - (int64_t)dw * n_ent);
    const int n = e / S + 1, sh = e - (n - 1) * S + 1;
    const double nd = (double)n, ad = (double)sh;
    const CellRec rec = s_rec[dw];
    const double ls = div_by(rec.load * ad, sd, a.r_share);      // the part of the load this type takes
    const double* den = s_den + (size_t)(n - 1) * n_f;
    const double* rden = s_rden + (size_t)(n - 1) * n_f;
    double best = __builtin_inf();
    int bf = -1;
    for (int f = 0; f < n_f; ++f) {                              // ascending: the lowest frequency wins equal energies
      L.den = den[f];
      L.rden = rden[f];
      L.lo = s_tab + (size_t)f * row_stride;
      L.hi = L.lo;
      double pf, tb, pw;
      const bool ov = table_lookup<SINGLE, false>(L, ls, &pf, &tb, &pw);
      const double en = (nd * pw) * a.window_s;
      const bool ok = !ov && !(rec.xp99 * pf > slo_ttft) && !(tb * rec.nonempty > slo_tbt);
      if (ok && en < best) { best = en; bf = f; }
    }
    const size_t o = ((size_t)(w0 + dw) * a.G + g) * n_entry + a.types.off[i] + e;
    a.type_energy[o] = best;
    a.type_f[o] = (int8_t)bf;
  }
}

// One wave per cell.  LDS: [E_i(n, a) of the cell, n_entry] [D of the previous type] [D of this type]
// [choice per type and state (16-bit: n << 8 | a)], states = (units of GPUs 0..U) x (shares 0..S).
// SMAX >= n_share bounds the unrolled loop over the shares given to a type: the loads of one
// (state, n) are issued together and the running minimum is the only dependence.
template <int SMAX>
__global__ __launch_bounds__(DYN_WAVE) void mixed_combine_kernel(MixedCombineArgs a) {
  extern __shared__ double smem[];
  const int64_t cell = blockIdx.x;
  const int g = (int)(cell % a.G);
  const int S = a.n_share, n_tp = a.types.n_tp, n_entry = a.types.off[n_tp];
  const int32_t bud = a.budget[g];
  const int U = bud > 0 ? min(bud / a.unit, a.u_max) : a.u_max;
  const int S1 = S + 1;
  const int n_state_max = (a.u_max + 1) * S1;
  const int n_state = (U + 1) * S1;
  double* s_c = smem;                                  // [n_entry]
  double* s_d0 = s_c + n_entry;                        // [n_state_max]
  double* s_d1 = s_d0 + n_state_max;
  uint16_t* s_ch = (uint16_t*)(s_d1 + n_state_max);    // [n_tp][n_state_max]
  const double inf = __builtin_inf();

  for (int q = threadIdx.x; q < n_entry; q += DYN_WAVE) s_c[q] = a.type_energy[cell * n_entry + q];
  for (int q = threadIdx.x; q < n_state; q += DYN_WAVE) s_d0[q] = q == 0 ? 0.0 : inf;   // nothing used: 0 J
  double* prev = s_d0;
  double* next = s_d1;
  for (int i = 0; i < n_tp; ++i) {
    __syncthreads();
    const int units = a.types.units[i], n_max = a.types.n_max[i];
    const double* ci = s_c + a.types.off[i];
    uint16_t* ch = s_ch + (size_t)i * n_state_max;
    for (int st = threadIdx.x; st < n_state; st += DYN_WAVE) {
      const int u = st / S1, sh = st - u * S1;
      double best = prev[st];                          // the type stays unused
      uint32_t bc = 0;
      for (int n = 1; n <= n_max && n * units <= u; ++n) {
        const double* pr = prev + (u - n * units) * S1 + sh;   // pr[-x]: x shares given to this type
        const double* cn = ci + (n - 1) * S;
#pragma unroll
        for (int x = 1; x <= SMAX; ++x) {
          if (x <= sh) {
            const double cand = pr[-x] + cn[x - 1];    // +inf marks what cannot be done
            if (cand < best) { best = cand; bc = ((uint32_t)n << 8) | (uint32_t)x; }
          }
        }
      }
      next[st] = best;
      ch[st] = (uint16_t)bc;
    }
    double* t = prev; prev = next; next = t;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    double best = inf;
    int bu = -1;
    for (int u = 0; u <= U; ++u) {
      const double v = prev[u * S1 + S];
      if (v < best) { best = v; bu = u; }
    }
    a.energy[cell] = best;
    a.ok[cell] = bu >= 0 ? 0 : -1;
    int st = bu >= 0 ? bu * S1 + S : 0;
    for (int i = n_tp - 1; i >= 0; --i) {
      const uint32_t bc = bu >= 0 ? s_ch[(size_t)i * n_state_max + st] : 0u;
      const int n = (int)(bc >> 8), x = (int)(bc & 0xFFu);
      a.n_inst[cell * n_tp + i] = n;
      a.share[cell * n_tp + i] = x;
      a.f_index[cell * n_tp + i] = n > 0 ? (int32_t)a.type_f[cell * n_entry + a.types.off[i] + (n - 1) * S + (x - 1)] : -1;
      st -= n * a.types.units[i] * S1 + x;
    }
  }
}

size_t type_lds(const MixedTypeArgs& a, bool single) {
  return ((size_t)a.n_f * ((3 * a.n_rho) | 1) + 2 * a.n_rho + 3 + (single ? a.n_bucket + 1 : 0)) * sizeof(double) +
         (size_t)a.win_per_block * sizeof(CellRec) + ((size_t)a.n_bucket + 1) * sizeof(uint16_t) + 8;
}
size_t type_walk_lds(const MixedTypeArgs& a, bool single) {   // plus the capacities of the type with most instances
  int n_max = 0;
  for (int i = 0; i < a.n_tp; ++i) n_max = std::max(n_max, a.types.n_max[i]);
  return type_lds(a, single) + (size_t)2 * n_max * a.n_f * sizeof(double);
}

}  // namespace

size_t dyn_mixed_combine_lds(int32_t n_tp, int32_t n_entry, int32_t u_max, int32_t n_share) {
  const size_t n_state = (size_t)(u_max + 1) * (n_share + 1);
  return ((size_t)n_entry + 2 * n_state) * sizeof(double) + (size_t)n_tp * n_state * sizeof(uint16_t) + 8;
}

hipError_t dyn_launch_mixed_types(const MixedTypeArgs& a, bool single_point, hipStream_t s) {
  const int n_chunk = (a.n_window + a.win_per_block - 1) / a.win_per_block;
  const dim3 grid((unsigned)((size_t)n_chunk * a.G * a.n_tp)), block(256);
  bool single = single_point;
  if (single && type_lds(a, true) > DYN_LDS_BUDGET) single = false;
  const size_t lds = type_lds(a, single);
  if (lds > DYN_LDS_BUDGET) return hipErrorInvalidValue;
  DynTimed timed(DYN_K_MIXED_TYPES, s);
  const size_t lds_walk = type_walk_lds(a, single);
  if (lds_walk <= DYN_LDS_BUDGET) {
    if (single) hipLaunchKernelGGL(mixed_type_walk_kernel<true>, grid, block, lds_walk, s, a);
    else hipLaunchKernelGGL(mixed_type_walk_kernel<false>, grid, block, lds_walk, s, a);
    return hipGetLastError();
  }
  if (single) hipLaunchKernelGGL(mixed_type_kernel<true>, grid, block, lds, s, a);
  else hipLaunchKernelGGL(mixed_type_kernel<false>, grid, block, lds, s, a);
  return hipGetLastError();
}

hipError_t dyn_launch_mixed_combine(const MixedCombineArgs& a, hipStream_t s) {
  const size_t lds = dyn_mixed_combine_lds(a.types.n_tp, a.types.off[a.types.n_tp], a.u_max, a.n_share);
  if (lds > DYN_LDS_BUDGET) return hipErrorInvalidValue;
  DynTimed timed(DYN_K_MIXED_COMBINE, s);
  const dim3 grid((unsigned)a.cells), block(DYN_WAVE);
  if (a.n_share <= 4) hipLaunchKernelGGL(mixed_combine_kernel<4>, grid, block, lds, s, a);
  else if (a.n_share <= 8) hipLaunchKernelGGL(mixed_combine_kernel<8>, grid, block, lds, s, a);
  else hipLaunchKernelGGL(mixed_combine_kernel<DYN_MIXED_MAX_SHARES>, grid, block, lds, s, a);
  return hipGetLastError();
}
