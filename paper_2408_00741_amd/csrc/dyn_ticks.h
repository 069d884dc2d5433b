// Internal declarations of the tick-level evaluation (not part of the ABI).
#ifndef DYN_TICKS_H_
#define DYN_TICKS_H_

#include "dyn_internal.h"

#define DYN_TICK_MAX 16   // ticks per window the kernels are unrolled for
#define DYN_TICK_TOP 64   // largest input lengths kept per fine cell (one wavefront's worth)
static_assert(DYN_TICK_MAX == DYN_TICK_LIMIT && DYN_TICK_TOP == DYN_TICK_DEPTH && DYN_TICK_TOP == DYN_WAVE,
              "the ABI's limits are the kernels' limits");

struct TickRec {   // what the evaluation kernel needs from one tick of a cell (16 bytes)
  double load;     // (input + output tokens of the tick) / tick_s
  int32_t cnt;     // requests in the tick
  int32_t plan;    // of the whole cell: j in the low byte (0 = empty, DYN_TICK_TOP + 1 = not evaluated), DYN_PLAN_MERGE
};
#define DYN_PLAN_MERGE 0x100

struct TickCellArgs {
  const int32_t* in; const int32_t* out;
  const int64_t* fine_off;   // [n_window * n_tick * G + 1]
  int64_t n_req;
  int32_t n_window, n_tick, G;
  double tick_s, r_tick;     // r_tick = RN(1 / tick_s)
  int64_t pct_num, pct_den;
  TickRec* rec;              // [cells][n_tick]
  int32_t* top;              // [cells][DYN_TICK_TOP][n_tick]; positions below min(j, cnt) are written
  uint8_t* cstat;            // [fine cells] status bytes
  WsHeader* header;
  uint32_t* merge_count;     // zeroed here
};

struct TickArgs {
  SpaceArgs s;             // n_window = coarse windows, part = coarse partials; s.rec and s.window_s are not used
  int32_t n_tick;
  double tick_s;
  double window_s;         // (double) n_tick * tick_s
  const TickRec* rec;      // [cells][n_tick]
  const int32_t* top;      // [cells][DYN_TICK_TOP][n_tick]
  const int32_t* tstart; const double* thr; bool single_point;   // threshold form of the bucket index
  bool any_two_rows;
  uint32_t* merge_count;   // number of cells on merge_list
  uint32_t* merge_list;    // [cells] cells left to tick_merge_kernel
};

// Workspace: the per-cell part of the evaluation workspace for the fine cells, then the
// candidate lists, then the partial selection records of the coarse cells.
struct TickWs {
  EvalWs fine;      // header, rec (as TickRec) and cstat are used; fine.part is where `top` starts
  size_t top, part, merge_count, merge_list, total;
  int32_t n_wslot;
};
TickWs dyn_tick_ws_layout(int64_t coarse_cells, int32_t n_tick, int32_t K);

hipError_t dyn_launch_tick_cell(const TickCellArgs& a, hipStream_t s);
hipError_t dyn_launch_tick_space(const TickArgs& a, hipStream_t s);

#endif  // DYN_TICKS_H_
