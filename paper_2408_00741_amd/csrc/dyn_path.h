// Internal declarations of the selection with transition overheads (not part of the ABI).
#ifndef DYN_PATH_H_
#define DYN_PATH_H_

#include "dyn_internal.h"

#define DYN_PATH_MAX_CONFIGS 2048   // candidates the path kernel holds (8 per thread of a 256-thread block)
#define DYN_PATH_RUN 64             // windows the trace-back follows per block
#define DYN_PATH_STATES 65          // what a run can be entered with: a layout of the window after it, or (64) none
inline int32_t dyn_path_runs(int32_t n_window) { return (n_window + DYN_PATH_RUN - 1) / DYN_PATH_RUN; }

struct PathArgs {
  const double* energy; const uint8_t* flags;   // evaluated space [cells][K]
  const DevCfg* cfg; int32_t K;
  const double* pw0; int32_t G, n_tp_f; int32_t n_window; double window_s; double idle_w;
  int32_t n_layout;
  const int32_t* layout;        // DEVICE [K]
  const int32_t* order;         // DEVICE [K] candidates sorted by (layout, index)
  const int32_t* seg_start;     // DEVICE [n_layout + 1] first sorted position of every layout
  const double* transition;     // DEVICE [n_layout][n_layout] (from, to)
  int32_t* pred;                // workspace [G][n_window][n_layout]
  int32_t* kend;                // workspace [G][n_window]
  double* min_cost;             // workspace [cells][n_layout] (n_layout <= 64): least cost of a layout's candidates, then least total of the sequences ending there
  int32_t* min_k;               // workspace [cells][n_layout]: the candidate that has it
  int32_t* exits;               // workspace [G][runs][DYN_PATH_STATES] (n_layout <= 64): state a run of windows is left with, by the state it is entered with
  int32_t* sel; double* sel_energy; double* path_cost;
};
hipError_t dyn_launch_path(const PathArgs& a, hipStream_t s);
size_t dyn_path_lds(int32_t K, int32_t n_layout);
bool dyn_path_fits(int32_t K, int32_t n_layout);   // what dyn_launch_path can take

#endif  // DYN_PATH_H_
