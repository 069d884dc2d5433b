// Cost and carbon of a selection (Section VI "Cost and Carbon Emission"): per window the GPUs in
// use by the selected configurations, their price, the energy bill and the operational CO2 at the
// window's carbon intensity; totals in window order.
#include "dyn_account.h"

namespace {

// One thread per window.  GPUs = sum over the classes with a selection of n_inst x tp.
__global__ __launch_bounds__(128) void account_kernel(AccountArgs a) {
  const int w = blockIdx.x * blockDim.x + threadIdx.x;
  if (w >= a.n_window) return;
  int64_t used = 0;
  uint32_t bad = 0;
  for (int g = 0; g < a.G; ++g) {
    const int32_t k = a.sel[(size_t)w * a.G + g];
    if (k >= a.K) bad = 1;                                 // not a candidate of the list: counted as no selection
    else if (k >= 0) used += a.cfg[k].gpus;
  }
  const double hours = ((double)used * a.window_s) / 3600.0;
  const double kwh = a.window_energy[w] / 3.6e6;
  a.gpus[w] = used;
  a.gpu_cost[w] = hours * a.gpu_hour_price;
  a.energy_cost[w] = kwh * a.kwh_price;
  a.carbon_g[w] = kwh * a.carbon[w];
  a.hours[w] = hours;
  a.servers[w] = (double)((used + a.gpus_per_server - 1) / a.gpus_per_server);
  if (bad) atomicOr(a.status, DYN_WS_BAD_REQUEST);
}

// Totals in window order from 0 (one lane per total: five independent sequential sums).
__global__ __launch_bounds__(64) void account_totals_kernel(AccountArgs a) {
  const double* src[5] = {a.hours, a.gpu_cost, a.energy_cost, a.carbon_g, a.servers};
  if (threadIdx.x < 5) {
    const double* x = src[threadIdx.x];
    double t = 0.0;
    for (int w = 0; w < a.n_window; ++w) t += x[w];
    a.totals[threadIdx.x] = t;
  }
}

}  // namespace

hipError_t dyn_launch_account(const AccountArgs& a, hipStream_t s) {
  DynTimed timed(DYN_K_TOTALS, s);
  hipLaunchKernelGGL(account_kernel, dim3((unsigned)((a.n_window + 127) / 128)), dim3(128), 0, s, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(account_totals_kernel, dim3(1), dim3(64), 0, s, a);
  return hipGetLastError();
}
