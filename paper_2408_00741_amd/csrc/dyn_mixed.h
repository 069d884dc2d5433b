// Internal declarations of the mixed-pool search (not part of the ABI).
#ifndef DYN_MIXED_H_
#define DYN_MIXED_H_

#include "dyn_internal.h"

#define DYN_MIXED_FREQ_LANES 16   // one row of 16 lanes per (type, instances, shares) entry: lane = frequency

struct MixedTypes {               // by value in the kernel arguments
  int32_t n_tp;
  int32_t n_max[DYN_MIXED_MAX_TYPES];     // instances considered per type
  int32_t units[DYN_MIXED_MAX_TYPES];     // GPUs of one instance in units of the types' common divisor
  int32_t off[DYN_MIXED_MAX_TYPES + 1];   // first entry of each type: entry (i, n, a) = off[i] + (n-1)*n_share + (a-1)
};

struct MixedTypeArgs {            // per-type least energies over the admissible frequencies
  const double* tab; const double* ml; const double* gridpack;
  const int32_t* jstart; const int32_t* tstart; const double* thr; int32_t n_bucket; double bucket_scale;
  int32_t G, n_tp, n_f, n_rho;
  const double* slo_ttft; const double* slo_tbt;
  const CellRec* rec; int32_t n_window; int32_t win_per_block; double window_s;
  int32_t n_share; double r_share;        // r_share = RN(1 / n_share)
  MixedTypes types;
  double* type_energy;                    // [cells][n_entry]
  int8_t* type_f;                         // [cells][n_entry]
};
hipError_t dyn_launch_mixed_types(const MixedTypeArgs& a, bool single_point, hipStream_t s);

struct MixedCombineArgs {         // least total energy over the assignments of instances and shares
  const double* type_energy; const int8_t* type_f;
  const int32_t* budget;                  // [G] GPUs, 0 = none
  int32_t G; int64_t cells; int32_t n_share; int32_t unit;   // unit = common divisor of the types' GPU counts
  int32_t u_max;                          // most units any assignment can use
  MixedTypes types;
  double* energy; int32_t* n_inst; int32_t* f_index; int32_t* share; int32_t* ok;
};
hipError_t dyn_launch_mixed_combine(const MixedCombineArgs& a, hipStream_t s);
size_t dyn_mixed_combine_lds(int32_t n_tp, int32_t n_entry, int32_t u_max, int32_t n_share);

hipError_t dyn_launch_window_totals(const int32_t* sel, const double* sel_energy, int32_t n_window, int32_t G,
                                    double* win_energy, int32_t* win_inf, hipStream_t s);

#endif  // DYN_MIXED_H_
