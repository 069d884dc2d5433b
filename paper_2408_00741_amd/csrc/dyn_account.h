// Internal declarations of the cost and carbon accounting (not part of the ABI).
#ifndef DYN_ACCOUNT_H_
#define DYN_ACCOUNT_H_

#include "dyn_internal.h"

struct AccountArgs {
  const int32_t* sel; const double* window_energy; const double* carbon;   // DEVICE [cells], [n_window], [n_window]
  const DevCfg* cfg; int32_t K, G, n_window; double window_s;
  double gpu_hour_price, kwh_price; int32_t gpus_per_server;
  int64_t* gpus; double* gpu_cost; double* energy_cost; double* carbon_g; double* totals;
  double* hours; double* servers;   // workspace [n_window] each
  uint32_t* status;                 // workspace word, zeroed by the caller of the kernels
};
hipError_t dyn_launch_account(const AccountArgs& a, hipStream_t s);

#endif  // DYN_ACCOUNT_H_
