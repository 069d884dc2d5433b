// Internal declarations of the controller hierarchy (not part of the ABI).
#ifndef DYN_HIER_H_
#define DYN_HIER_H_

#include "dyn_internal.h"

struct HierArgs {
  // profile
  const double* tab; const double* ml; const double* gridpack; const int32_t* jstart; const int32_t* tstart; const double* thr;
  int32_t n_bucket; double bucket_scale;
  int32_t G, n_tp, n_f, n_rho;
  const int32_t* tp;            // DEVICE [n_tp] GPUs per instance
  const double* slo_ttft; const double* slo_tbt;
  // trace aggregates
  const CellRec* rec_c;         // [n_window * G] window level
  const CellRec* rec_f;         // [n_window * n_tick * G] tick level
  const uint8_t* cstat_c;       // status bytes of the window-level aggregation
  const uint8_t* cstat_f;       // status bytes of the tick-level aggregation
  uint32_t* status;             // status word of the workspace header
  int32_t n_window, n_tick; double tick_s, window_s;
  // controllers
  int32_t epoch_windows, n_epoch, tp_ref, f_ref, gpus_per_node;
  int32_t n_layout; const int32_t* lay_n; const int32_t* lay_tp;   // DEVICE [n_layout]
  // outputs and scratch
  int32_t* nodes; int32_t* layout_sel; int32_t* f_sel; double* energy; int32_t* violations;
  double* win_energy; int32_t* win_inf;   // [n_window] totals over the classes
  double* lay_energy;           // workspace [cells][n_layout] or NULL: every layout's energy at the reference frequency
  uint8_t* lay_flags;           // workspace [cells][n_layout]: DYN_F_FEASIBLE where the layout fits and meets the SLO
  double* tick_energy;          // workspace [fine cells]
  uint8_t* tick_viol;           // workspace [fine cells]
  // fragmentation rule (all NULL without it): loads the pools serve after forwarding, kept fractions
  double* served_c;             // workspace [cells]
  double* served_f;             // workspace [fine cells]
  double* keep;                 // [n_epoch][G]
  double* fwd;                  // workspace [n_window]: load forwarded to the class in hand
};
// fragmentation rule: node counts, kept fractions and served loads of every window and tick (before the shard level)
hipError_t dyn_launch_hier_spill(const HierArgs& a, hipStream_t s);
// window level: node counts, per-window layouts and (lay_energy != NULL) every layout's energy and admissibility
hipError_t dyn_launch_hier_shard(const HierArgs& a, bool single_point, hipStream_t s);
// tick level: frequencies under layout_sel, energies, window totals
hipError_t dyn_launch_hier_ticks(const HierArgs& a, bool single_point, hipStream_t s);

#endif  // DYN_HIER_H_
