// CPU oracle for the batched evaluation of DynamoLLM's reconfiguration search space.
//
// TEST INFRASTRUCTURE.  Plain, slow, single-threaded, fp64.  It exists to define the
// expected result; only the test-suite, the smoke check and the CPU-baseline leg of the
// benchmark may build, load or call it.  It shares no code with the HIP library and
// neither includes the other.
//
// What it computes, for every (time window, request class) cell and every candidate
// configuration (instances n, tensor-parallel degree TP, GPU frequency f):
//   * the class's load in the window, in tokens per second (Section III-A, "Request
//     loads": system load is measured in tokens per second);
//   * the per-instance share of that load, every instance of a pool receiving the same
//     amount of work (Section IV-A, the fair-share assumption stated before Eq. 1);
//   * TTFT, TBT and power read from the profile, a function of (load, request class,
//     TP, frequency) that is known at a few load levels up to the maximum throughput
//     and taken piecewise-linearly in between (Section IV-A "Generating LLM profiles";
//     Section IV-E names one-dimensional linear interpolation);
//   * for every request of the cell its predicted TTFT (prefill time grows with the
//     number of input tokens, Section II), its TBT and its share of the energy, then
//     the P99 of TTFT and of TBT over the cell (Section III-A "Service SLO");
//   * feasibility: Performance <= SLO and instances x TP <= GPU budget (Eq. 1,
//     constraints 3 and 1), plus "the load does not exceed the profiled range";
//   * the objective N x Energy(load per instance) (Eq. 1) and, per cell, the feasible
//     configuration of least cost (Section IV-B "Scale-up/down": first drop what
//     violates the SLO, then take the least energy).
//
// Every request is evaluated under every configuration and the percentile is taken from
// the per-request values themselves; nothing is blocked, fused or reordered.
//
// Readings where the paper is silent (each also listed in the design notes):
//   load = (input + output tokens of the cell) / window length;
//   load axis of the tables = per-instance load / max_load_tps(class, TP, f);
//   a load beyond the last profiled point makes the configuration infeasible, values
//     are reported at the last point;
//   bracket of x on a grid = largest i with grid[i] <= x, clamped to len-2;
//   bilinear order: along load on the two bracketing frequency rows, then along f;
//   percentile = nearest rank, rank = ceil(num*m/den) in integer arithmetic;
//   empty cell: load 0, percentiles 0, SLOs hold, energy = idle energy;
//   energy in joules = n * power * window length;
//   cost = energy + idle_cost_weight * n * power(load 0) * window length;
//   ties in the argmin go to the lowest configuration index; no feasible one -> -1.
//
// Build: g++ -O2 -std=c++17 -ffp-contract=off -shared -fPIC (see build_oracle.py).

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <limits>
#include <numeric>
#include <vector>

namespace {

enum : int {
  ORC_OK = 0, ORC_E_NULL = -1, ORC_E_SHAPE = -2, ORC_E_RANGE = -3, ORC_E_NOTFINITE = -4,
  ORC_E_ORDER = -5, ORC_E_SELFCHECK = -8
};

// largest i with grid[i] <= x, clamped to [0, len-2]  (len >= 2)
int bracket(const double* grid, int len, double x) {
  int i = 0;
  for (int q = 0; q < len; ++q)
    if (grid[q] <= x) i = q;
  if (i > len - 2) i = len - 2;
  return i;
}

bool increasing(const double* g, int n) {
  for (int i = 0; i < n; ++i)
    if (!std::isfinite(g[i])) return false;
  for (int i = 1; i < n; ++i)
    if (!(g[i] > g[i - 1])) return false;
  return true;
}

}  // namespace

extern "C" {

// Section III-A, Table IV: requests are classified by input and output length; a value
// equal to a threshold belongs to the upper bin ("< 256" is Short, 256 is Medium).
// Windows are the controllers' epochs (Section IV-B): w = floor(t / window_s).
// Output: requests reordered by cell = w*G + class (order of arrival kept inside a
// cell) and the start offset of every cell.
int dynoracle_ingest(const double* t_s, const int32_t* in_tok, const int32_t* out_tok,
                     const int32_t* model, int64_t n_req, int32_t n_model, int32_t n_in_bin,
                     int32_t n_out_bin, const int32_t* in_edge, const int32_t* out_edge,
                     int32_t n_window, double window_s, int32_t* in_sorted,
                     int32_t* out_sorted, int64_t* cell_off) {
  if (!t_s || !in_tok || !out_tok || !in_sorted || !out_sorted || !cell_off) return ORC_E_NULL;
  if (n_req < 0 || n_model < 1 || n_in_bin < 1 || n_out_bin < 1 || n_window < 1) return ORC_E_SHAPE;
  if (!(window_s > 0.0)) return ORC_E_RANGE;
  const int64_t G = (int64_t)n_model * n_in_bin * n_out_bin;
  const int64_t cells = (int64_t)n_window * G;
  std::vector<int64_t> cell(n_req);
  for (int64_t r = 0; r < n_req; ++r) {
    const double wq = std::floor(t_s[r] / window_s);
    if (!(wq >= 0.0) || !(wq < (double)n_window)) return ORC_E_RANGE;
    const int64_t w = (int64_t)wq;
    const int32_t mdl = model ? model[r] : 0;
    if (mdl < 0 || mdl >= n_model) return ORC_E_RANGE;
    int bi = 0, bo = 0;
    for (int e = 0; e < n_in_bin - 1; ++e)
      if (in_tok[r] >= in_edge[(int64_t)mdl * (n_in_bin - 1) + e]) ++bi;
    for (int e = 0; e < n_out_bin - 1; ++e)
      if (out_tok[r] >= out_edge[(int64_t)mdl * (n_out_bin - 1) + e]) ++bo;
    const int64_t g = ((int64_t)mdl * n_in_bin + bi) * n_out_bin + bo;
    cell[r] = w * G + g;
  }
  std::vector<int64_t> order(n_req);
  std::iota(order.begin(), order.end(), (int64_t)0);
  std::stable_sort(order.begin(), order.end(),
                   [&](int64_t a, int64_t b) { return cell[a] < cell[b]; });
  for (int64_t c = 0; c <= cells; ++c) cell_off[c] = 0;
  for (int64_t r = 0; r < n_req; ++r) cell_off[cell[r] + 1] += 1;
  for (int64_t c = 0; c < cells; ++c) cell_off[c + 1] += cell_off[c];
  for (int64_t i = 0; i < n_req; ++i) {
    in_sorted[i] = in_tok[order[i]];
    out_sorted[i] = out_tok[order[i]];
  }
  return ORC_OK;
}

// Evaluates the cells listed in cell_ids (all cells 0..n_sel-1 when cell_ids is null)
// under all K configurations.  Outputs are indexed by position in that list:
// energy_j, p99_ttft_ms, p99_tbt_ms, cost [n_sel][K] (k fastest), flags [n_sel][K],
// m, tin, tout, in_p99, sel, sel_energy_j, sel_cost [n_sel].  Any output may be null.
// flags: bit0 feasible, bit1 load beyond the profiled range, bit2 TTFT > SLO,
// bit3 TBT > SLO, bit4 GPU budget exceeded, bit5 empty cell.
// full_sort != 0 sorts the per-request latencies completely; otherwise the element of
// the same rank is found with std::nth_element (same value by definition).
int dynoracle_eval(int32_t G, int32_t n_tp, const int32_t* tp, int32_t n_f, const double* fg,
                   int32_t n_rho, const double* rg, const double* PF, const double* TB,
                   const double* PW, const double* ML,
                   int64_t n_req, int32_t n_window, double window_s, const int32_t* in_tok,
                   const int32_t* out_tok, const int64_t* cell_off,
                   int32_t K, const int32_t* cfg_n, const int32_t* cfg_tp_index,
                   const double* cfg_f,
                   const double* slo_ttft, const double* slo_tbt, int32_t pct_num,
                   int32_t pct_den, const int32_t* gpu_budget, double idle_cost_weight,
                   int64_t n_sel, const int64_t* cell_ids, int32_t full_sort,
                   double* energy_j, double* p99_ttft_ms, double* p99_tbt_ms, uint8_t* flags,
                   double* cost_out, int64_t* m_out, int64_t* tin_out, int64_t* tout_out,
                   int32_t* in_p99_out, int32_t* sel_out, double* sel_energy_j,
                   double* sel_cost) {
  if (!tp || !fg || !rg || !PF || !TB || !PW || !ML || !cell_off || !cfg_n || !cfg_tp_index ||
      !cfg_f || !slo_ttft || !slo_tbt)
    return ORC_E_NULL;
  if (n_req > 0 && (!in_tok || !out_tok)) return ORC_E_NULL;
  if (G < 1 || n_tp < 1 || n_f < 1 || n_rho < 2 || K < 1 || n_window < 1 || n_sel < 0)
    return ORC_E_SHAPE;
  if (!(window_s > 0.0) || pct_num < 1 || pct_den < 1 || pct_num > pct_den) return ORC_E_RANGE;
  if (!increasing(fg, n_f) || !increasing(rg, n_rho)) return ORC_E_ORDER;
  if (rg[0] != 0.0) return ORC_E_RANGE;
  const int64_t n_tab = (int64_t)G * n_tp * n_f * n_rho;
  for (int64_t i = 0; i < n_tab; ++i)
    if (!std::isfinite(PF[i]) || !std::isfinite(TB[i]) || !std::isfinite(PW[i]) || PF[i] < 0.0 ||
        TB[i] < 0.0 || PW[i] < 0.0)
      return ORC_E_NOTFINITE;
  for (int64_t i = 0; i < (int64_t)G * n_tp * n_f; ++i)
    if (!std::isfinite(ML[i]) || !(ML[i] > 0.0)) return ORC_E_NOTFINITE;
  for (int k = 0; k < K; ++k) {
    if (cfg_n[k] < 1 || cfg_tp_index[k] < 0 || cfg_tp_index[k] >= n_tp) return ORC_E_RANGE;
    if (!(cfg_f[k] >= fg[0]) || !(cfg_f[k] <= fg[n_f - 1])) return ORC_E_RANGE;
  }
  const int64_t cells = (int64_t)n_window * G;
  const double INF = std::numeric_limits<double>::infinity();

  // frequency bracket and weight of every configuration (independent of the cell)
  std::vector<int> fi(K);
  std::vector<double> u(K);
  for (int k = 0; k < K; ++k) {
    if (n_f == 1) { fi[k] = 0; u[k] = 0.0; continue; }
    fi[k] = bracket(fg, n_f, cfg_f[k]);
    u[k] = (cfg_f[k] - fg[fi[k]]) / (fg[fi[k] + 1] - fg[fi[k]]);
  }
  auto tab = [&](const double* X, int g, int ti, int f, int j) -> double {
    return X[(((int64_t)g * n_tp + ti) * n_f + f) * n_rho + j];
  };

  std::vector<double> lat, e_cost(K), e_energy(K);
  std::vector<uint8_t> e_flags(K);
  for (int64_t s = 0; s < n_sel; ++s) {
    const int64_t c = cell_ids ? cell_ids[s] : s;
    if (c < 0 || c >= cells) return ORC_E_RANGE;
    const int g = (int)(c % G);
    const int64_t beg = cell_off[c], end = cell_off[c + 1];
    if (beg < 0 || end < beg || end > n_req) return ORC_E_ORDER;
    const int64_t m = end - beg;

    // load of the class in this window: tokens per second
    int64_t tin = 0, tout = 0;
    for (int64_t r = beg; r < end; ++r) { tin += in_tok[r]; tout += out_tok[r]; }
    const double L = (double)(tin + tout) / window_s;
    const int64_t rank = (m > 0) ? ((int64_t)pct_num * m + pct_den - 1) / pct_den : 0;

    // the cell's P99 input length (an intermediate the tests compare bit for bit)
    int32_t in_p99 = 0;
    if (m > 0) {
      std::vector<int32_t> tmp(in_tok + beg, in_tok + end);
      std::sort(tmp.begin(), tmp.end());
      in_p99 = tmp[rank - 1];
    }
    if (m_out) m_out[s] = m;
    if (tin_out) tin_out[s] = tin;
    if (tout_out) tout_out[s] = tout;
    if (in_p99_out) in_p99_out[s] = in_p99;

    for (int k = 0; k < K; ++k) {
      const int ti = cfg_tp_index[k], f0 = fi[k];
      const double uk = u[k], nk = (double)cfg_n[k];
      // capacity of one instance at (TP, f), then the per-instance load on the table axis
      const double* mlrow = ML + ((int64_t)g * n_tp + ti) * n_f;
      const double ml = (n_f == 1) ? mlrow[0] : (1.0 - uk) * mlrow[f0] + uk * mlrow[f0 + 1];
      const double rho = L / (nk * ml);
      const bool ov = rho > rg[n_rho - 1];
      const double rc = ov ? rg[n_rho - 1] : rho;
      const int j = bracket(rg, n_rho, rc);
      const double t = (rc - rg[j]) / (rg[j + 1] - rg[j]);
      double val[3];
      const double* X[3] = {PF, TB, PW};
      for (int q = 0; q < 3; ++q) {
        const double a = (1.0 - t) * tab(X[q], g, ti, f0, j) + t * tab(X[q], g, ti, f0, j + 1);
        if (n_f == 1) { val[q] = a; continue; }
        const double b =
            (1.0 - t) * tab(X[q], g, ti, f0 + 1, j) + t * tab(X[q], g, ti, f0 + 1, j + 1);
        val[q] = (1.0 - uk) * a + uk * b;
      }
      const double pf = val[0], tb = val[1], pw = val[2];
      const double pw0 = (n_f == 1) ? tab(PW, g, ti, 0, 0)
                                    : (1.0 - uk) * tab(PW, g, ti, f0, 0) + uk * tab(PW, g, ti, f0 + 1, 0);
      const double E = (nk * pw) * window_s;

      double p_ttft = 0.0, p_tbt = 0.0;
      if (m > 0) {
        // every request under this configuration: TTFT grows with its input length,
        // TBT is the profile's per-token latency, energy is shared by token count
        lat.resize((size_t)m);
        double esum = 0.0;
        const double tok = (double)(tin + tout);
        for (int64_t r = 0; r < m; ++r) {
          lat[(size_t)r] = (double)in_tok[beg + r] * pf;
          esum += E * ((double)((int64_t)in_tok[beg + r] + out_tok[beg + r]) / tok);
        }
        if (std::fabs(esum - E) > 1e-9 * std::fabs(E)) return ORC_E_SELFCHECK;
        if (full_sort) {
          std::sort(lat.begin(), lat.end());
        } else {
          std::nth_element(lat.begin(), lat.begin() + (rank - 1), lat.end());
        }
        p_ttft = lat[(size_t)(rank - 1)];
        p_tbt = tb;  // all m per-request TBTs equal tb, so does their percentile
      }
      const double cost = E + idle_cost_weight * ((nk * pw0) * window_s);

      uint8_t fl = 0;
      if (ov) fl |= 2;
      if (p_ttft > slo_ttft[g]) fl |= 4;
      if (p_tbt > slo_tbt[g]) fl |= 8;
      if (gpu_budget && gpu_budget[g] > 0 && (int64_t)cfg_n[k] * tp[ti] > gpu_budget[g]) fl |= 16;
      if (m == 0) fl |= 32;
      if (!(fl & (2 | 4 | 8 | 16))) fl |= 1;

      e_energy[k] = E; e_cost[k] = cost; e_flags[k] = fl;
      const int64_t o = s * K + k;
      if (energy_j) energy_j[o] = E;
      if (p99_ttft_ms) p99_ttft_ms[o] = p_ttft;
      if (p99_tbt_ms) p99_tbt_ms[o] = p_tbt;
      if (flags) flags[o] = fl;
      if (cost_out) cost_out[o] = cost;
    }

    int best = -1;
    for (int k = 0; k < K; ++k)
      if ((e_flags[k] & 1) && (best < 0 || e_cost[k] < e_cost[best])) best = k;
    if (sel_out) sel_out[s] = best;
    if (sel_energy_j) sel_energy_j[s] = best < 0 ? INF : e_energy[best];
    if (sel_cost) sel_cost[s] = best < 0 ? INF : e_cost[best];
  }
  return ORC_OK;
}

// Tick-level load inside a window (the instance manager re-tunes the frequency every few
// seconds under the current load, Section IV-B "Scale-up/down"; the paper's large-scale
// results come from a discrete-time simulator, Section V): every window is split into
// n_tick ticks of tick_s seconds, each request is served under the load of its own tick.
// Reading: the trace is sorted by fine cell = (w*n_tick + tick)*G + class (ticks are
// sub-windows: tick index = floor(t / tick_s)); per tick the class's load is its tokens /
// tick_s and the profile lookup is the one of dynoracle_eval; a request's TTFT is its
// input length x the prefill ms/token of its tick, its TBT the TBT of its tick; the
// window's energy is the sum over ticks (in tick order) of n x power(tick) x tick_s; the
// overload flag is raised if any tick exceeds the profiled load range; the idle-cost term
// uses the window length n_tick x tick_s.  With n_tick == 1 every output equals
// dynoracle_eval's.  Outputs are indexed by coarse cell w*G + class (all of them).
int dynoracle_eval_ticks(int32_t G, int32_t n_tp, const int32_t* tp, int32_t n_f, const double* fg,
                         int32_t n_rho, const double* rg, const double* PF, const double* TB,
                         const double* PW, const double* ML,
                         int64_t n_req, int32_t n_window, int32_t n_tick, double tick_s,
                         const int32_t* in_tok, const int32_t* out_tok, const int64_t* fine_off,
                         int32_t K, const int32_t* cfg_n, const int32_t* cfg_tp_index, const double* cfg_f,
                         const double* slo_ttft, const double* slo_tbt, int32_t pct_num, int32_t pct_den,
                         const int32_t* gpu_budget, double idle_cost_weight,
                         double* energy_j, double* p99_ttft_ms, double* p99_tbt_ms, uint8_t* flags,
                         double* cost_out, int64_t* m_out, int32_t* sel_out, double* sel_energy_j,
                         double* sel_cost) {
  if (!tp || !fg || !rg || !PF || !TB || !PW || !ML || !fine_off || !cfg_n || !cfg_tp_index || !cfg_f ||
      !slo_ttft || !slo_tbt)
    return ORC_E_NULL;
  if (n_req > 0 && (!in_tok || !out_tok)) return ORC_E_NULL;
  if (G < 1 || n_tp < 1 || n_f < 1 || n_rho < 2 || K < 1 || n_window < 1 || n_tick < 1) return ORC_E_SHAPE;
  if (!(tick_s > 0.0) || pct_num < 1 || pct_den < 1 || pct_num > pct_den) return ORC_E_RANGE;
  if (!increasing(fg, n_f) || !increasing(rg, n_rho)) return ORC_E_ORDER;
  if (rg[0] != 0.0) return ORC_E_RANGE;
  for (int k = 0; k < K; ++k) {
    if (cfg_n[k] < 1 || cfg_tp_index[k] < 0 || cfg_tp_index[k] >= n_tp) return ORC_E_RANGE;
    if (!(cfg_f[k] >= fg[0]) || !(cfg_f[k] <= fg[n_f - 1])) return ORC_E_RANGE;
  }
  const double INF = std::numeric_limits<double>::infinity();
  const double window_s = (double)n_tick * tick_s;
  std::vector<int> fi(K);
  std::vector<double> u(K);
  for (int k = 0; k < K; ++k) {
    if (n_f == 1) { fi[k] = 0; u[k] = 0.0; continue; }
    fi[k] = bracket(fg, n_f, cfg_f[k]);
    u[k] = (cfg_f[k] - fg[fi[k]]) / (fg[fi[k] + 1] - fg[fi[k]]);
  }
  auto tab = [&](const double* X, int g, int ti, int f, int j) -> double {
    return X[(((int64_t)g * n_tp + ti) * n_f + f) * n_rho + j];
  };
  std::vector<double> ttft, tbt, e_cost(K), e_energy(K);
  std::vector<uint8_t> e_flags(K);
  for (int w = 0; w < n_window; ++w) {
    for (int g = 0; g < G; ++g) {
      const int64_t c = (int64_t)w * G + g;
      int64_t m = 0;
      for (int q = 0; q < n_tick; ++q) {
        const int64_t f = ((int64_t)w * n_tick + q) * G + g;
        if (fine_off[f] < 0 || fine_off[f + 1] < fine_off[f] || fine_off[f + 1] > n_req) return ORC_E_ORDER;
        m += fine_off[f + 1] - fine_off[f];
      }
      const int64_t rank = (m > 0) ? ((int64_t)pct_num * m + pct_den - 1) / pct_den : 0;
      if (m_out) m_out[c] = m;
      for (int k = 0; k < K; ++k) {
        const int ti = cfg_tp_index[k], f0 = fi[k];
        const double uk = u[k], nk = (double)cfg_n[k];
        const double* mlrow = ML + ((int64_t)g * n_tp + ti) * n_f;
        const double ml = (n_f == 1) ? mlrow[0] : (1.0 - uk) * mlrow[f0] + uk * mlrow[f0 + 1];
        ttft.clear();
        tbt.clear();
        double E = 0.0;
        bool any_ov = false;
        for (int q = 0; q < n_tick; ++q) {
          const int64_t f = ((int64_t)w * n_tick + q) * G + g;
          const int64_t beg = fine_off[f], end = fine_off[f + 1];
          int64_t tok = 0;
          for (int64_t r = beg; r < end; ++r) tok += (int64_t)in_tok[r] + out_tok[r];
          const double L = (double)tok / tick_s;
          const double rho = L / (nk * ml);
          const bool ov = rho > rg[n_rho - 1];
          any_ov = any_ov || ov;
          const double rc = ov ? rg[n_rho - 1] : rho;
          const int j = bracket(rg, n_rho, rc);
          const double t = (rc - rg[j]) / (rg[j + 1] - rg[j]);
          double val[3];
          const double* X[3] = {PF, TB, PW};
          for (int x = 0; x < 3; ++x) {
            const double a = (1.0 - t) * tab(X[x], g, ti, f0, j) + t * tab(X[x], g, ti, f0, j + 1);
            if (n_f == 1) { val[x] = a; continue; }
            const double b = (1.0 - t) * tab(X[x], g, ti, f0 + 1, j) + t * tab(X[x], g, ti, f0 + 1, j + 1);
            val[x] = (1.0 - uk) * a + uk * b;
          }
          for (int64_t r = beg; r < end; ++r) {   // every request of the tick under this configuration
            ttft.push_back((double)in_tok[r] * val[0]);
            tbt.push_back(val[1]);
          }
          E += (nk * val[2]) * tick_s;
        }
        double p_ttft = 0.0, p_tbt = 0.0;
        if (m > 0) {
          std::sort(ttft.begin(), ttft.end());
          std::sort(tbt.begin(), tbt.end());
          p_ttft = ttft[(size_t)(rank - 1)];
          p_tbt = tbt[(size_t)(rank - 1)];
        }
        const double pw0 = (n_f == 1) ? tab(PW, g, ti, 0, 0)
                                      : (1.0 - uk) * tab(PW, g, ti, f0, 0) + uk * tab(PW, g, ti, f0 + 1, 0);
        const double cost = E + idle_cost_weight * ((nk * pw0) * window_s);
        uint8_t fl = 0;
        if (any_ov) fl |= 2;
        if (p_ttft > slo_ttft[g]) fl |= 4;
        if (p_tbt > slo_tbt[g]) fl |= 8;
        if (gpu_budget && gpu_budget[g] > 0 && (int64_t)cfg_n[k] * tp[ti] > gpu_budget[g]) fl |= 16;
        if (m == 0) fl |= 32;
        if (!(fl & (2 | 4 | 8 | 16))) fl |= 1;
        e_energy[k] = E; e_cost[k] = cost; e_flags[k] = fl;
        const int64_t o = c * K + k;
        if (energy_j) energy_j[o] = E;
        if (p99_ttft_ms) p99_ttft_ms[o] = p_ttft;
        if (p99_tbt_ms) p99_tbt_ms[o] = p_tbt;
        if (flags) flags[o] = fl;
        if (cost_out) cost_out[o] = cost;
      }
      int best = -1;
      for (int k = 0; k < K; ++k)
        if ((e_flags[k] & 1) && (best < 0 || e_cost[k] < e_cost[best])) best = k;
      if (sel_out) sel_out[c] = best;
      if (sel_energy_j) sel_energy_j[c] = best < 0 ? INF : e_energy[best];
      if (sel_cost) sel_cost[c] = best < 0 ? INF : e_cost[best];
    }
  }
  return ORC_OK;
}

// Pools that mix instance types (Eq. 1 in full): per (window, class) cell choose how many
// instances of every tensor parallelism run (N^TP), at which frequency (f^TP) and which part
// of the load each type takes (L^TP), so that the total energy is least while the GPUs used
// stay within the budget, the assigned loads add up to the pool's load and every type that is
// used meets the SLO under its load.
// Readings: the load is split in n_share equal shares, type i takes a_i of them (a_i >= 1
// exactly when the type is used, sum a_i = n_share) and its n_i instances share that part
// equally (fair share, as for Eq. 1): per-instance load = (L * a_i / n_share) / n_i; the
// frequencies are the profiled ones; every type serves requests of the whole cell, so the
// percentiles of a type are taken over all requests of the cell under that type's tables;
// total energy = 0 + E_0 + E_1 + ... over the used types in type order, E_i = n_i x power x
// window; the budget of a class (0 = none) bounds sum n_i x tp_i.
// The frequency of a type is chosen as the instance manager does it (Section IV-B
// "Scale-up/down"): drop the frequencies that violate the SLO or leave the profiled load
// range, then take the least energy (lowest frequency index on ties); this is independent
// of the other types, so the search enumerates (n_i, a_i) for every type and adds the
// types' least energies.  Options of a type are visited as "unused", then n ascending, a
// ascending, types nested in index order; the first assignment of least energy is kept and
// n_optimal counts the assignments that reach it.
// type_energy (may be null): [cells][sum_i n_max_i * n_share] the per-type least energies,
// entry (i, n, a) at offset(i) + (n-1)*n_share + (a-1), +inf if no frequency is admissible;
// type_f the chosen frequency index (-1 if none).
int dynoracle_mixed(int32_t G, int32_t n_tp, const int32_t* tp, int32_t n_f, const double* fg,
                    int32_t n_rho, const double* rg, const double* PF, const double* TB,
                    const double* PW, const double* ML,
                    int64_t n_req, int32_t n_window, double window_s, const int32_t* in_tok,
                    const int32_t* out_tok, const int64_t* cell_off,
                    int32_t n_share, const int32_t* n_max,
                    const double* slo_ttft, const double* slo_tbt, int32_t pct_num, int32_t pct_den,
                    const int32_t* gpu_budget,
                    double* energy_j, int32_t* n_inst, int32_t* f_index, int32_t* share,
                    int64_t* n_optimal, double* type_energy, int32_t* type_f) {
  if (!tp || !fg || !rg || !PF || !TB || !PW || !ML || !cell_off || !n_max || !slo_ttft || !slo_tbt ||
      !energy_j || !n_inst || !f_index || !share)
    return ORC_E_NULL;
  if (n_req > 0 && (!in_tok || !out_tok)) return ORC_E_NULL;
  if (G < 1 || n_tp < 1 || n_f < 1 || n_rho < 2 || n_window < 1 || n_share < 1) return ORC_E_SHAPE;
  if (!(window_s > 0.0) || pct_num < 1 || pct_den < 1 || pct_num > pct_den) return ORC_E_RANGE;
  if (!increasing(fg, n_f) || !increasing(rg, n_rho) || rg[0] != 0.0) return ORC_E_ORDER;
  int64_t n_entry = 0;
  std::vector<int64_t> off(n_tp);
  for (int i = 0; i < n_tp; ++i) {
    if (n_max[i] < 0 || tp[i] < 1) return ORC_E_RANGE;
    off[i] = n_entry;
    n_entry += (int64_t)n_max[i] * n_share;
  }
  const int64_t cells = (int64_t)n_window * G;
  const double INF = std::numeric_limits<double>::infinity();
  auto tab = [&](const double* X, int g, int ti, int f, int j) -> double {
    return X[(((int64_t)g * n_tp + ti) * n_f + f) * n_rho + j];
  };
  std::vector<double> lat, C((size_t)n_entry);
  std::vector<int32_t> F((size_t)n_entry);
  std::vector<int32_t> cur_n(n_tp), cur_a(n_tp), best_n(n_tp), best_a(n_tp);
  for (int64_t c = 0; c < cells; ++c) {
    const int g = (int)(c % G);
    const int64_t beg = cell_off[c], end = cell_off[c + 1];
    if (beg < 0 || end < beg || end > n_req) return ORC_E_ORDER;
    const int64_t m = end - beg;
    int64_t tin = 0, tout = 0;
    for (int64_t r = beg; r < end; ++r) { tin += in_tok[r]; tout += out_tok[r]; }
    const double L = (double)(tin + tout) / window_s;
    const int64_t rank = (m > 0) ? ((int64_t)pct_num * m + pct_den - 1) / pct_den : 0;

    // least energy of every (type, instances, shares) over the admissible frequencies
    for (int i = 0; i < n_tp; ++i)
      for (int n = 1; n <= n_max[i]; ++n)
        for (int a = 1; a <= n_share; ++a) {
          double best = INF;
          int32_t bf = -1;
          const double Ls = (L * (double)a) / (double)n_share;
          for (int f = 0; f < n_f; ++f) {
            const double ml = ML[((int64_t)g * n_tp + i) * n_f + f];
            const double rho = Ls / ((double)n * ml);
            const bool ov = rho > rg[n_rho - 1];
            const double rc = ov ? rg[n_rho - 1] : rho;
            const int j = bracket(rg, n_rho, rc);
            const double t = (rc - rg[j]) / (rg[j + 1] - rg[j]);
            const double pf = (1.0 - t) * tab(PF, g, i, f, j) + t * tab(PF, g, i, f, j + 1);
            const double tb = (1.0 - t) * tab(TB, g, i, f, j) + t * tab(TB, g, i, f, j + 1);
            const double pw = (1.0 - t) * tab(PW, g, i, f, j) + t * tab(PW, g, i, f, j + 1);
            const double E = ((double)n * pw) * window_s;
            double p_ttft = 0.0, p_tbt = 0.0;
            if (m > 0) {
              lat.resize((size_t)m);
              for (int64_t r = 0; r < m; ++r) lat[(size_t)r] = (double)in_tok[beg + r] * pf;
              std::nth_element(lat.begin(), lat.begin() + (rank - 1), lat.end());
              p_ttft = lat[(size_t)(rank - 1)];
              p_tbt = tb;
            }
            const bool ok = !ov && !(p_ttft > slo_ttft[g]) && !(p_tbt > slo_tbt[g]);
            if (ok && (bf < 0 || E < best)) { best = E; bf = f; }
          }
          const int64_t e = off[i] + (int64_t)(n - 1) * n_share + (a - 1);
          C[(size_t)e] = best;
          F[(size_t)e] = bf;
          if (type_energy) type_energy[c * n_entry + e] = best;
          if (type_f) type_f[c * n_entry + e] = bf;
        }

    // every assignment of instances and shares to the types
    double best_e = INF;
    int64_t n_best = 0;
    const int64_t budget = (gpu_budget && gpu_budget[g] > 0) ? gpu_budget[g] : -1;
    // iterative nested loops over the types: position i holds option index o_i in
    // [0, n_max_i * n_share]: 0 = unused, else n = (o-1)/n_share + 1, a = (o-1)%n_share + 1
    std::vector<int64_t> opt(n_tp, 0);
    while (true) {
      int64_t a_sum = 0, gpus = 0;
      bool fin = true;
      double E = 0.0;
      for (int i = 0; i < n_tp; ++i) {
        if (opt[i] == 0) { cur_n[i] = 0; cur_a[i] = 0; continue; }
        cur_n[i] = (int32_t)((opt[i] - 1) / n_share + 1);
        cur_a[i] = (int32_t)((opt[i] - 1) % n_share + 1);
        a_sum += cur_a[i];
        gpus += (int64_t)cur_n[i] * tp[i];
        const double ci = C[(size_t)(off[i] + opt[i] - 1)];
        if (!(ci < INF)) fin = false;
        E += ci;
      }
      if (fin && a_sum == n_share && (budget < 0 || gpus <= budget)) {
        if (E < best_e) { best_e = E; n_best = 1; best_n = cur_n; best_a = cur_a; }
        else if (E == best_e) ++n_best;
      }
      // next assignment: the last type varies fastest
      int i = n_tp - 1;
      while (i >= 0) {
        if (opt[i] < (int64_t)n_max[i] * n_share) { ++opt[i]; break; }
        opt[i] = 0;
        --i;
      }
      if (i < 0) break;
    }
    energy_j[c] = best_e;
    if (n_optimal) n_optimal[c] = n_best;
    for (int i = 0; i < n_tp; ++i) {
      const bool used = n_best > 0 && best_n[i] > 0;
      n_inst[c * n_tp + i] = used ? best_n[i] : 0;
      share[c * n_tp + i] = used ? best_a[i] : 0;
      f_index[c * n_tp + i] = used ? F[(size_t)(off[i] + (int64_t)(best_n[i] - 1) * n_share + (best_a[i] - 1))] : -1;
    }
  }
  return ORC_OK;
}

// Selection that accounts for the cost of changing the configuration between consecutive
// windows (Section IV-B "Accounting for the overheads": the transition overheads are kept in
// an Overhead Table and weighed against the energy a new configuration saves; Table VI lists
// the re-sharding overheads between the layouts of a server).
// Reading: per class, the configurations k_w of the windows w = 0 .. NW-1 are chosen together
// so that  sum_w cost(w, k_w) + sum_{w >= 1} transition[layout(k_{w-1})][layout(k_w)]  is
// least, cost(w, k) as in the per-window selection (energy + idle term) and only feasible
// configurations allowed.  The total of a sequence is accumulated in time order,
// V = cost(0, k_0); V = (V + transition) + cost(w, k_w).  A window without any feasible
// configuration gets -1; the sequence ends before it and a new one starts after it without a
// transition; the class's total adds the sequences' totals in time order starting from 0.
// The minimum over all sequences is found window by window (rounded addition is monotone, so
// extending the cheapest way to reach k' is the cheapest extension): for every k the least
// of V_prev[k'] + transition over all k' (lowest k' on ties), then + cost; at the end of a
// sequence the least V (lowest k) and the chain of predecessors.
// space_cost [cells][K]: cost(w, k); feasible [cells][K]: != 0 where allowed.
int dynoracle_select_path(int32_t n_window, int32_t G, int32_t K, const double* space_cost,
                          const uint8_t* feasible, int32_t n_layout, const int32_t* layout,
                          const double* transition, int32_t* sel, double* path_cost) {
  if (!space_cost || !feasible || !layout || !transition || !sel || !path_cost) return ORC_E_NULL;
  if (n_window < 1 || G < 1 || K < 1 || n_layout < 1) return ORC_E_SHAPE;
  for (int k = 0; k < K; ++k)
    if (layout[k] < 0 || layout[k] >= n_layout) return ORC_E_RANGE;
  for (int64_t i = 0; i < (int64_t)n_layout * n_layout; ++i)
    if (!std::isfinite(transition[i]) || transition[i] < 0.0) return ORC_E_NOTFINITE;
  const double INF = std::numeric_limits<double>::infinity();
  std::vector<double> V(K), Vn(K);
  std::vector<int32_t> pred((size_t)n_window * K);
  for (int g = 0; g < G; ++g) {
    double total = 0.0;
    int w = 0;
    while (w < n_window) {
      // skip windows without a feasible configuration
      auto any = [&](int ww) {
        for (int k = 0; k < K; ++k)
          if (feasible[((int64_t)ww * G + g) * K + k]) return true;
        return false;
      };
      if (!any(w)) { sel[(int64_t)w * G + g] = -1; ++w; continue; }
      const int w_beg = w;
      for (int k = 0; k < K; ++k) {
        const int64_t o = ((int64_t)w * G + g) * K + k;
        V[k] = feasible[o] ? space_cost[o] : INF;
      }
      int w_end = w + 1;
      for (; w_end < n_window && any(w_end); ++w_end) {
        for (int k = 0; k < K; ++k) {
          const int64_t o = ((int64_t)w_end * G + g) * K + k;
          double best = INF;
          int32_t bp = -1;
          for (int kp = 0; kp < K; ++kp) {
            const double c = V[kp] + transition[(int64_t)layout[kp] * n_layout + layout[k]];
            if (c < best) { best = c; bp = kp; }
          }
          pred[(size_t)w_end * K + k] = bp;
          Vn[k] = feasible[o] ? best + space_cost[o] : INF;
        }
        V.swap(Vn);
      }
      // end of the sequence [w_beg, w_end): least total, then its chain of predecessors
      int kb = -1;
      for (int k = 0; k < K; ++k)
        if (V[k] < INF && (kb < 0 || V[k] < V[kb])) kb = k;
      total += V[kb];
      for (int ww = w_end - 1; ww >= w_beg; --ww) {
        sel[(int64_t)ww * G + g] = kb;
        if (ww > w_beg) kb = pred[(size_t)ww * K + kb];
      }
      w = w_end;
    }
    path_cost[g] = total;
  }
  return ORC_OK;
}

// Cost and carbon of a selection (Section VI "Cost and Carbon Emission": the user's cost follows
// the number of GPU servers over time and the energy bill; operational CO2 is the energy of each
// interval times the grid's carbon intensity at that time).
// Per window: GPUs in use = sum over the classes with a selection of n_inst x tp; servers =
// ceil(GPUs / gpus_per_server); GPU-hours = ((double) GPUs x window_s) / 3600; GPU cost =
// GPU-hours x gpu_hour_price; kWh = window energy / 3.6e6; energy cost = kWh x kwh_price;
// carbon = kWh x carbon intensity of the window (g/kWh).  Totals are summed in window order
// from 0: {GPU-hours, GPU cost, energy cost, carbon in g, servers summed over the windows}.
int dynoracle_account(int32_t n_window, int32_t G, int32_t K, const int32_t* cfg_n, const int32_t* cfg_tp_index,
                      const int32_t* tp, const int32_t* sel, const double* window_energy_j, double window_s,
                      double gpu_hour_price, double kwh_price, const double* carbon_g_per_kwh, int32_t gpus_per_server,
                      int64_t* gpus, double* gpu_cost, double* energy_cost, double* carbon_g, double* totals) {
  if (!cfg_n || !cfg_tp_index || !tp || !sel || !window_energy_j || !carbon_g_per_kwh || !gpus || !gpu_cost ||
      !energy_cost || !carbon_g || !totals)
    return ORC_E_NULL;
  if (n_window < 1 || G < 1 || K < 1 || gpus_per_server < 1) return ORC_E_SHAPE;
  double t_hours = 0.0, t_gpu = 0.0, t_energy = 0.0, t_carbon = 0.0, t_servers = 0.0;
  for (int w = 0; w < n_window; ++w) {
    int64_t used = 0;
    for (int g = 0; g < G; ++g) {
      const int32_t k = sel[(int64_t)w * G + g];
      if (k >= K) return ORC_E_RANGE;
      if (k >= 0) used += (int64_t)cfg_n[k] * tp[cfg_tp_index[k]];
    }
    const double hours = ((double)used * window_s) / 3600.0;
    const double kwh = window_energy_j[w] / 3.6e6;
    gpus[w] = used;
    gpu_cost[w] = hours * gpu_hour_price;
    energy_cost[w] = kwh * kwh_price;
    carbon_g[w] = kwh * carbon_g_per_kwh[w];
    t_hours += hours; t_gpu += gpu_cost[w]; t_energy += energy_cost[w]; t_carbon += carbon_g[w];
    t_servers += (double)((used + gpus_per_server - 1) / gpus_per_server);
  }
  totals[0] = t_hours; totals[1] = t_gpu; totals[2] = t_energy; totals[3] = t_carbon; totals[4] = t_servers;
  return ORC_OK;
}

// The three controllers of Section IV-B on a trace, top down.
//   Scale-out/in (every epoch of `epoch_windows` windows): nodes = ceil(PL / ML) per class, PL =
//     the peak of the class's load over the epoch's windows, ML = the largest profiled load of
//     one node at the reference configuration (tp_ref, f_ref: "TP8 at 1980 MHz"): instances per
//     node (gpus_per_node / tp) x max_load_tps x last load-grid point.
//   Shard-up/down (every window): among the layouts (n_inst, tp_index) of the list with
//     n_inst x tp <= nodes x gpus_per_node, evaluated at f_ref under the window's load, the one of
//     least energy that meets the SLO (percentiles over the window's requests); -1 if none.
//   Scale-up/down (every tick of the window): for that layout, among the profiled frequencies,
//     drop those that violate the SLO under the tick's load (percentiles over the tick's
//     requests) or leave the profiled load range, then take the least power (lowest frequency
//     on ties); if none is left the tick runs at f_ref and is counted as a violation.
//   Energy of a (window, class) = sum over its ticks in time order of (n x power) x tick_s.
//   With a transition table (Section IV-B "Accounting for the overheads", Table VI): the shard
//     controller weighs the energy a layout saves against the overhead of getting there.  Per
//     class the layouts of all windows are then chosen together, as dynoracle_select_path does
//     with cost = the layout's energy at f_ref over the window, feasible = fits the nodes' GPUs
//     and meets the SLO, one candidate per layout; path_cost[g] = that class's total.  Without a
//     table (NULL) every window takes its own least-energy layout and path_cost is not written.
//   With spill != 0 (Section IV-B "Handling fragmentation"): a pool whose peak does not fill its
//     last node gets that node less, and the load the remaining nodes cannot carry goes to the
//     pool of the next class; only the last class rounds up.  Per epoch, classes in ascending
//     order: arriving load of a window A = own load + what the class below forwards; PL = peak
//     of A; q = PL / ML.  If the class is not the last and 1 <= floor(q) < q: nodes = floor(q)
//     and the pool keeps the fraction keep = ((floor(q) x ML) / PL) x (1 - 2^-40) of what
//     arrives (the factor keeps the peak window inside the profiled range whatever the rounding
//     of the later divisions); otherwise nodes = ceil(q), at least one, and keep = 1.  Served
//     load S = keep x A in every window and tick of the epoch; forwarded = A - S.  The shard
//     and frequency controllers see S; the percentiles stay those of the pool's own requests
//     (forwarded requests are smaller than the pool's own).
// Readings: the load predictor is exact (the epoch's true peak); at least one node per class;
// a window whose class has no admissible layout has energy +inf and no frequencies (-1).
// coarse_off / fine_off: offsets of the trace sorted by window*G + class and by
// (window*n_tick + tick)*G + class; both index the same requests (in_c/out_c, in_f/out_f).
int dynoracle_hierarchy(int32_t G, int32_t n_tp, const int32_t* tp, int32_t n_f, const double* fg,
                        int32_t n_rho, const double* rg, const double* PF, const double* TB,
                        const double* PW, const double* ML,
                        int64_t n_req, int32_t n_window, int32_t n_tick, double tick_s,
                        const int32_t* in_c, const int32_t* out_c, const int64_t* coarse_off,
                        const int32_t* in_f, const int32_t* out_f, const int64_t* fine_off,
                        int32_t epoch_windows, int32_t tp_ref, int32_t f_ref, int32_t gpus_per_node,
                        int32_t n_layout, const int32_t* lay_n, const int32_t* lay_tp,
                        const double* slo_ttft, const double* slo_tbt, int32_t pct_num, int32_t pct_den,
                        const double* transition, int32_t spill, int32_t* nodes, int32_t* layout_sel,
                        int32_t* f_sel, double* energy_j, int32_t* violations, double* path_cost,
                        double* keep, double* served) {
  if (!tp || !fg || !rg || !PF || !TB || !PW || !ML || !coarse_off || !fine_off || !lay_n || !lay_tp ||
      !slo_ttft || !slo_tbt || !nodes || !layout_sel || !f_sel || !energy_j || !violations)
    return ORC_E_NULL;
  if (transition && !path_cost) return ORC_E_NULL;
  if (n_req > 0 && (!in_c || !out_c || !in_f || !out_f)) return ORC_E_NULL;
  if (G < 1 || n_tp < 1 || n_f < 1 || n_rho < 2 || n_window < 1 || n_tick < 1 || epoch_windows < 1 ||
      n_layout < 1 || gpus_per_node < 1)
    return ORC_E_SHAPE;
  if (tp_ref < 0 || tp_ref >= n_tp || f_ref < 0 || f_ref >= n_f || !(tick_s > 0.0)) return ORC_E_RANGE;
  for (int l = 0; l < n_layout; ++l)
    if (lay_n[l] < 1 || lay_tp[l] < 0 || lay_tp[l] >= n_tp) return ORC_E_RANGE;
  const double INF = std::numeric_limits<double>::infinity();
  const double window_s = (double)n_tick * tick_s;
  const int n_epoch = (n_window + epoch_windows - 1) / epoch_windows;
  auto tab = [&](const double* X, int g, int ti, int f, int j) -> double {
    return X[(((int64_t)g * n_tp + ti) * n_f + f) * n_rho + j];
  };
  // profile at (class, tp, f) for a per-instance load fraction: returns overload
  auto look = [&](int g, int ti, int f, double load, double n, double* pf, double* tb, double* pw) -> bool {
    const double ml = ML[((int64_t)g * n_tp + ti) * n_f + f];
    const double rho = load / (n * ml);
    const bool ov = rho > rg[n_rho - 1];
    const double rc = ov ? rg[n_rho - 1] : rho;
    const int j = bracket(rg, n_rho, rc);
    const double t = (rc - rg[j]) / (rg[j + 1] - rg[j]);
    *pf = (1.0 - t) * tab(PF, g, ti, f, j) + t * tab(PF, g, ti, f, j + 1);
    *tb = (1.0 - t) * tab(TB, g, ti, f, j) + t * tab(TB, g, ti, f, j + 1);
    *pw = (1.0 - t) * tab(PW, g, ti, f, j) + t * tab(PW, g, ti, f, j + 1);
    return ov;
  };
  // nearest-rank percentile of in_r * pf over a run of requests (0 for an empty run)
  std::vector<double> lat;
  auto p_ttft = [&](const int32_t* in, int64_t beg, int64_t end, double pf) -> double {
    const int64_t m = end - beg;
    if (m <= 0) return 0.0;
    const int64_t rank = ((int64_t)pct_num * m + pct_den - 1) / pct_den;
    lat.resize((size_t)m);
    for (int64_t r = 0; r < m; ++r) lat[(size_t)r] = (double)in[beg + r] * pf;
    std::nth_element(lat.begin(), lat.begin() + (rank - 1), lat.end());
    return lat[(size_t)(rank - 1)];
  };
  auto load_of = [&](const int32_t* in, const int32_t* out, int64_t beg, int64_t end, double secs) -> double {
    int64_t tok = 0;
    for (int64_t r = beg; r < end; ++r) tok += (int64_t)in[r] + out[r];
    return (double)tok / secs;
  };

  // scale-out/in; served loads of every window and tick (equal to the own loads without spill)
  const int64_t cells = (int64_t)n_window * G;
  const int64_t fcells = cells * n_tick;
  std::vector<double> S_c((size_t)cells), S_f((size_t)fcells), kept((size_t)n_epoch * G, 1.0);
  const double guard = 1.0 - std::ldexp(1.0, -40);
  for (int e = 0; e < n_epoch; ++e) {
    const int w0 = e * epoch_windows, w1 = std::min(n_window, (e + 1) * epoch_windows);
    std::vector<double> fwd((size_t)(w1 - w0), 0.0), A((size_t)(w1 - w0));
    for (int g = 0; g < G; ++g) {
      double peak = 0.0;
      for (int w = w0; w < w1; ++w) {
        const int64_t c = (int64_t)w * G + g;
        A[(size_t)(w - w0)] = load_of(in_c, out_c, coarse_off[c], coarse_off[c + 1], window_s) + fwd[(size_t)(w - w0)];
        if (A[(size_t)(w - w0)] > peak) peak = A[(size_t)(w - w0)];
      }
      const int inst = std::max(1, gpus_per_node / tp[tp_ref]);
      const double ml_node = ((double)inst * ML[((int64_t)g * n_tp + tp_ref) * n_f + f_ref]) * rg[n_rho - 1];
      const double q = peak / ml_node;
      const double fl = std::floor(q);
      double k = 1.0;
      if (spill && g < G - 1 && fl >= 1.0 && fl < q && fl < 2147483647.0) {
        nodes[(int64_t)e * G + g] = (int32_t)fl;
        k = ((fl * ml_node) / peak) * guard;
      } else {
        const double up = std::ceil(q);
        nodes[(int64_t)e * G + g] = up < 1.0 ? 1 : (up > 2147483647.0 ? 2147483647 : (int32_t)up);
      }
      kept[(size_t)e * G + g] = k;
      for (int w = w0; w < w1; ++w) {
        const double s = k * A[(size_t)(w - w0)];
        S_c[(size_t)((int64_t)w * G + g)] = s;
        fwd[(size_t)(w - w0)] = A[(size_t)(w - w0)] - s;
      }
    }
  }
  for (int64_t t = 0; t < (int64_t)n_window * n_tick; ++t) {
    const int e = (int)(t / n_tick) / epoch_windows;
    double fwd = 0.0;
    for (int g = 0; g < G; ++g) {
      const int64_t f = t * G + g;
      const double a = load_of(in_f, out_f, fine_off[f], fine_off[f + 1], tick_s) + fwd;
      S_f[(size_t)f] = kept[(size_t)e * G + g] * a;
      fwd = a - S_f[(size_t)f];
    }
  }
  if (keep) std::copy(kept.begin(), kept.end(), keep);
  if (served) std::copy(S_c.begin(), S_c.end(), served);

  // shard-up/down: energy and admissibility of every layout at the reference frequency
  std::vector<double> lay_e((size_t)cells * n_layout, INF);
  std::vector<uint8_t> lay_ok((size_t)cells * n_layout, 0);
  for (int w = 0; w < n_window; ++w)
    for (int g = 0; g < G; ++g) {
      const int64_t c = (int64_t)w * G + g;
      const int64_t beg = coarse_off[c], end = coarse_off[c + 1];
      const int64_t m = end - beg;
      const double L = S_c[(size_t)c];
      const int64_t budget = (int64_t)nodes[(int64_t)(w / epoch_windows) * G + g] * gpus_per_node;
      int best = -1;
      double best_e = INF;
      for (int l = 0; l < n_layout; ++l) {
        if ((int64_t)lay_n[l] * tp[lay_tp[l]] > budget) continue;
        double pf, tb, pw;
        const bool ov = look(g, lay_tp[l], f_ref, L, (double)lay_n[l], &pf, &tb, &pw);
        const double tt = p_ttft(in_c, beg, end, pf);
        const double bt = m > 0 ? tb : 0.0;
        if (ov || tt > slo_ttft[g] || bt > slo_tbt[g]) continue;
        const double E = ((double)lay_n[l] * pw) * window_s;
        lay_e[(size_t)c * n_layout + l] = E;
        lay_ok[(size_t)c * n_layout + l] = 1;
        if (best < 0 || E < best_e) { best = l; best_e = E; }
      }
      layout_sel[c] = best;
    }
  if (transition) {                         // the windows' layouts chosen together, one candidate per layout
    std::vector<int32_t> ident(n_layout);
    for (int l = 0; l < n_layout; ++l) ident[l] = l;
    const int rc = dynoracle_select_path(n_window, G, n_layout, lay_e.data(), lay_ok.data(), n_layout, ident.data(),
                                         transition, layout_sel, path_cost);
    if (rc != ORC_OK) return rc;
  }

  for (int w = 0; w < n_window; ++w)
    for (int g = 0; g < G; ++g) {
      const int64_t c = (int64_t)w * G + g;
      const int best = layout_sel[c];
      double E = 0.0;
      int32_t viol = 0;
      for (int q = 0; q < n_tick; ++q) {
        const int64_t f = ((int64_t)w * n_tick + q) * G + g;
        if (best < 0) { f_sel[f] = -1; continue; }
        const int64_t fb = fine_off[f], fe = fine_off[f + 1];
        const double Lt = S_f[(size_t)f];
        int bf = -1;
        double bp = INF;
        for (int fi = 0; fi < n_f; ++fi) {
          double pf, tb, pw;
          const bool ov = look(g, lay_tp[best], fi, Lt, (double)lay_n[best], &pf, &tb, &pw);
          const double tt = p_ttft(in_f, fb, fe, pf);
          const double bt = fe > fb ? tb : 0.0;
          if (ov || tt > slo_ttft[g] || bt > slo_tbt[g]) continue;
          if (bf < 0 || pw < bp) { bf = fi; bp = pw; }
        }
        if (bf < 0) {                       // nothing admissible: highest-performance frequency, counted
          double pf, tb;
          look(g, lay_tp[best], f_ref, Lt, (double)lay_n[best], &pf, &tb, &bp);
          bf = f_ref;
          ++viol;
        }
        f_sel[f] = bf;
        E += ((double)lay_n[best] * bp) * tick_s;
      }
      energy_j[c] = best < 0 ? INF : E;
      violations[c] = viol;
    }
  return ORC_OK;
}

// Objective summed over the pools of a window (Eq. 1 sums over instance types; here one
// pool per class), classes added in index order; cells without a feasible configuration
// are counted, not added.
int dynoracle_window_totals(int32_t n_window, int32_t G, const int32_t* sel,
                            const double* sel_energy_j, double* window_energy_j,
                            int32_t* window_infeasible) {
  if (!sel || !sel_energy_j || !window_energy_j || !window_infeasible) return ORC_E_NULL;
  for (int w = 0; w < n_window; ++w) {
    double e = 0.0;
    int32_t ninf = 0;
    for (int g = 0; g < G; ++g) {
      const int64_t c = (int64_t)w * G + g;
      if (sel[c] >= 0) e += sel_energy_j[c]; else ++ninf;
    }
    window_energy_j[w] = e;
    window_infeasible[w] = ninf;
  }
  return ORC_OK;
}

// Least-cost feasible column of one row (used to check the selector against the energy
// tables the paper prints): lowest index on exact ties, -1 when nothing is feasible.
int dynoracle_select_row(int32_t K, const double* cost, const uint8_t* feasible) {
  int best = -1;
  for (int k = 0; k < K; ++k)
    if (feasible[k] && (best < 0 || cost[k] < cost[best])) best = k;
  return best;
}

}  // extern "C"
