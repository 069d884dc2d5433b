// Internal declarations of the tick-level evaluation (not part of the ABI).
#ifndef DYN_TICKS_H_
#define DYN_TICKS_H_

#include "dyn_internal.h"

#define DYN_TICK_MAX 64     // ticks per window: a wave's lane holds a tick in the cell kernel
#define DYN_TICK_FAST 16    // percentile depth j up to which the evaluation kernel keeps a sorted list in registers
#define DYN_TICK_WAVE 64    // depth up to which one wave of the cell kernel extracts the per-tick lists
static_assert(DYN_TICK_MAX == DYN_TICK_LIMIT && DYN_TICK_MAX == DYN_WAVE && DYN_TICK_WAVE == DYN_WAVE,
              "the ABI's limits are the kernels' limits");

struct TickRec {   // one tick of a (window, class) cell (16 bytes)
  double load;     // (input + output tokens of the tick) / tick_s
  uint32_t off;    // first request of the tick in the sorted trace = start of the tick's list in `top` (DYN_TP_TIGHT cells: see there)
  int32_t cnt;     // requests in the tick
};

// What the cell kernel decides about a (window, class) cell.  The cell's percentile is its j-th largest
// per-request value, j = m - rank + 1.
struct TickPlan {
  int32_t j;       // 0 = empty cell
  int32_t xj;      // j-th largest input length of the whole cell
  uint32_t flags;  // DYN_TP_*
  uint32_t place;  // DYN_TP_TIGHT: rank of the percentile among the ticks that hold requests of length xj (bit 31: from below)
};
#define DYN_TP_DENSE 1u   // every non-empty tick holds at least j requests: the TBT percentile is the largest tick TBT
#define DYN_TP_SMALL 2u   // the four non-empty ticks of largest TBT hold at least j requests, whichever they are
#define DYN_TP_DEEP 4u    // j > DYN_TICK_WAVE: lists and xj come from the deep-cell kernel
#define DYN_TP_RAW 8u     // j > DYN_TICK_DEPTH: the lists are whole ticks, sorted
#define DYN_TICK_PIECES 0x80000000u   // in TickRec.off of a tick of such a cell that is too long to sort in LDS: its list is sorted in pieces of DYN_TICK_DEPTH (offsets stay below 2^31)
#define DYN_TP_GENERAL 16u  // left to the general kernel: j beyond the walk's register list, or a TBT percentile that needs all ticks
#define DYN_TP_TIGHT 32u   // settled by the ticks' requests of length xj (TickRec.off then holds their number, not a list offset)

struct TickCellArgs {
  const int32_t* in; const int32_t* out;
  const int64_t* fine_off;   // [n_window * n_tick * G + 1]
  int64_t n_req;
  int32_t n_window, n_tick, G;
  double tick_s, r_tick;     // r_tick = RN(1 / tick_s)
  int64_t pct_num, pct_den;
  TickRec* rec;              // [cells][n_tick]
  TickPlan* plan;            // [cells]
  int32_t* top;              // [n_req]: per tick its min(j, cnt) largest input lengths, descending, at rec.off
  uint8_t* cstat;            // [fine cells] status bytes
  WsHeader* header;
  uint32_t* counters;        // [0] cells on deep_list, [1] cells on slow_list, [2] cells on list_cells, [3] cells walked with lists; zeroed before the cell kernels
  uint32_t* deep_list;       // [cells]
  uint32_t* slow_list;       // [cells] cells left to the general kernel
  uint32_t* list_cells;      // [cells] cells that need per-tick lists
  const float* theta;        // [G] per class: least (smallest / largest prefill time of a table row), rounded down
  int32_t few_cells;         // so few cells that a block per cell leaves no compute unit short of work
};

struct TickArgs {
  SpaceArgs s;             // n_window = coarse windows, part = coarse partials; s.rec and s.window_s are not used
  int32_t n_tick;
  double tick_s;
  double window_s;         // (double) n_tick * tick_s
  const TickRec* rec;      // [cells][n_tick]
  const TickPlan* plan;    // [cells]
  const int32_t* top;      // [n_req]
  const int32_t* in;       // [n_req] input lengths of the trace sorted by tick (DYN_TP_RAW cells)
  const int32_t* tstart; const double* thr; bool single_point;   // threshold form of the bucket index
  bool any_two_rows;
  int32_t n_cu;               // compute units of the device (0: unknown)
  const double* pfspan;       // [G][n_tp_f][2] smallest and largest prefill time of every table row
  const uint32_t* counters;   // [1]: number of cells on slow_list, [3]: number of cells walked with lists
  const uint32_t* slow_list;  // [cells] cells left to the general kernel
};

// Workspace: the per-cell part of the evaluation workspace for the fine cells, then the plans, the
// per-tick lists, the partial selection records of the coarse cells and the two work lists.
struct TickWs {
  EvalWs fine;      // header, rec (as TickRec) and cstat are used; fine.part is where `plan` starts
  size_t plan, top, part, counters, deep_list, slow_list, list_cells, total;
  int32_t n_wslot;
};
TickWs dyn_tick_ws_layout(int64_t n_req, int64_t coarse_cells, int32_t n_tick, int32_t K);

hipError_t dyn_launch_tick_cell(const TickCellArgs& a, hipStream_t s);
hipError_t dyn_launch_tick_space(const TickArgs& a, hipStream_t s);

#endif  // DYN_TICKS_H_
