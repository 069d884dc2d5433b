// Internal declarations of the tick-level evaluation (not part of the ABI).
#ifndef DYN_TICKS_H_
#define DYN_TICKS_H_

#include "dyn_internal.h"

#define DYN_TICK_MAX 16   // ticks per window the kernels are unrolled for
#define DYN_TICK_TOP 64   // largest input lengths kept per fine cell (one wavefront's worth)
static_assert(DYN_TICK_MAX == DYN_TICK_LIMIT && DYN_TICK_TOP == DYN_TICK_DEPTH && DYN_TICK_TOP == DYN_WAVE,
              "the ABI's limits are the kernels' limits");

struct TickArgs {
  SpaceArgs s;             // n_window = coarse windows, rec = per-fine-cell records, part = coarse partials
  int32_t n_tick;
  double tick_s;
  double window_s;         // (double) n_tick * tick_s
  const int64_t* fine_off; // [n_window * n_tick * G + 1]
  int64_t n_req;
  const int32_t* top;      // [fine cells][DYN_TICK_TOP]
  uint8_t* cstat;          // per-fine-cell status bytes
  int32_t pct_num, pct_den;
};

// Workspace: the per-cell part of the evaluation workspace for the fine cells, then the
// candidate lists, then the partial selection records of the coarse cells.
struct TickWs {
  EvalWs fine;      // header .. cstat are used; fine.part is where `top` starts
  size_t top, part, total;
  int32_t n_wslot;
};
TickWs dyn_tick_ws_layout(int64_t coarse_cells, int32_t n_tick, int32_t K);

hipError_t dyn_launch_tick_top(const int32_t* in_tok, const int64_t* fine_off, int64_t n_req, int32_t n_window,
                               int32_t n_tick, int32_t G, int32_t pct_num, int32_t pct_den, int32_t* top,
                               hipStream_t s);
hipError_t dyn_launch_tick_space(const TickArgs& a, hipStream_t s);

#endif  // DYN_TICKS_H_
