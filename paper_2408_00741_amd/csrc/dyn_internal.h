// Internal declarations shared by the HIP sources of libdyn (not part of the ABI).
#ifndef DYN_INTERNAL_H_
#define DYN_INTERNAL_H_

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <vector>

#include "dyn.h"

#define DYN_WAVE 64

// ---- device-side views ------------------------------------------------------------------
// One candidate configuration, prepared on the host.  (ti, row_lo, row_hi) address table
// rows; row = ti * n_f + fi.  u is the weight of row_hi; when u == 0 only row_lo is read.
struct DevCfg {
  double u;       // frequency weight in [0, 1)
  double nd;      // (double) n_inst
  int32_t n;      // n_inst
  int32_t gpus;   // n_inst * tp (saturated to INT32_MAX)
  int32_t row_lo; // ti * n_f + fi
  int32_t row_hi; // ti * n_f + fi + 1 (== row_lo when u == 0)
  int32_t slot_lo, slot_hi;  // LDS slots of the two rows inside the configuration's tile
};

struct CellRec {  // what the space kernel needs from a cell (32 bytes)
  double load;      // (tin + tout) / window_s
  double xp99;      // (double) in_p99; 0 for an empty cell
  double nonempty;  // 1.0, or 0.0 for an empty cell (exact multiplier for the cell's percentiles)
  double pad;
};

#define DYN_MAX_CONFIGS 65536     // capacity of a profile handle's configuration table
#define DYN_MAX_TILE 256          // configurations per tile of the space kernel
#define DYN_LDS_BUDGET (64 * 1024)
#define DYN_MAX_WIN_PER_BLOCK 32  // windows one block of the space kernel walks

// ---- host-side profile handle -----------------------------------------------------------
// Besides the tables it owns the device copies of the last candidate list and objective
// it was used with ("plan"), so that repeated evaluations upload nothing.
struct dyn_profile {
  int32_t G, n_tp, n_f, n_rho;
  std::vector<int32_t> tp;   // host copies used to validate candidate configurations
  std::vector<double> fg;
  int device;
  // device copy of the tables, one packed row per (class, TP, f):
  // [G][n_tp*n_f][3][n_rho] with the three tables (prefill, TBT, power) side by side
  double* d_tab;
  double* d_ml;   // [G][n_tp][n_f]
  double* d_pw0;  // [G][n_tp][n_f]  power at load 0 (first column of d_pw)
  double* d_pfspan;  // [G][n_tp][n_f][2]  smallest and largest prefill time of the row over the load axis
  float* d_theta;    // [G]  least ratio smallest / largest prefill time over the class's rows, rounded down
  // load grid for the kernels: [-inf, rho[0..n_rho-1], +inf] followed by
  // [0, 1/(rho[1]-rho[0]), ..., 1/(rho[n_rho-1]-rho[n_rho-2]), 0]
  double* d_gridpack;   // [2*n_rho + 3]
  bool one_step;        // every bracket is at most one step away from its bucket's index
  // bucket index over the load axis: bucket b covers [b, b+1) / bucket_scale and jstart[b]
  // is the largest grid index i with rg[i] <= b / bucket_scale
  int32_t* d_jstart;  // [n_bucket + 1]
  int32_t n_bucket;
  double bucket_scale;
  // the same buckets by what the kernels' own bucket arithmetic b(x) = (int)(x * bucket_scale)
  // returns: tstart[b] = number of interior grid points (1 .. n_rho-2) whose bucket is below b,
  // thr[b] = the interior grid point whose bucket is b (+inf if none).  When no bucket holds
  // two of them (single_point), the bracket of x is tstart[b(x)] + (x >= thr[b(x)]).
  int32_t* d_tstart;  // [n_bucket + 1]
  double* d_thr;      // [n_bucket + 1]
  bool single_point;
  // plan: candidate list
  std::vector<dyn_config> cfg_host;   // what d_cfg currently holds
  DevCfg* d_cfg;                      // [DYN_MAX_CONFIGS]
  int32_t* d_tile_rows;               // [2*DYN_MAX_CONFIGS + 1024]
  int32_t tile, n_tile, n_slot;       // n_slot == 0: table rows are read from global memory
  bool any_two_rows;                  // some candidate's frequency lies between two profiled ones
  // windows one block of the evaluation kernel walks: the rule's value for this list, or what dyn_eval_tune measured
  // (both for the number of windows they were made for)
  int32_t wpb, wpb_windows;
  bool wpb_tuned;
  int32_t n_cu;                       // compute units of the device
  // plan: objective
  std::vector<double> slo_ttft_host, slo_tbt_host;
  std::vector<int32_t> budget_host;
  bool obj_valid;
  double* d_slo_ttft;  // [G]
  double* d_slo_tbt;   // [G]
  int32_t* d_budget;   // [G]
  // plan: the small host tables of dyn_select_path and dyn_hierarchy, cached like the candidate list (a table that
  // equals the handle's copy is not uploaded again)
  std::vector<int32_t> path_layout_host, path_order_host, path_seg_host, lay_n_host, lay_tp_host;
  std::vector<double> path_trans_host, hier_trans_host;
  int32_t* d_path_layout;  // [DYN_MAX_CONFIGS]
  int32_t* d_path_order;   // [DYN_MAX_CONFIGS]
  int32_t* d_path_seg;     // [DYN_MAX_LAYOUTS + 1]
  double* d_path_trans;    // [DYN_MAX_LAYOUTS^2]
  double* d_hier_trans;    // [DYN_MAX_LAYOUTS^2]
  int32_t* d_lay_n;        // [DYN_MAX_CONFIGS]
  int32_t* d_lay_tp;       // [DYN_MAX_CONFIGS]
  int32_t* d_tp;           // [n_tp]
  int32_t* d_ident;        // [DYN_MAX_CONFIGS + 1] 0, 1, 2, ...
};
#define DYN_MAX_LAYOUTS 255   // layouts a transition table can hold

// Per-(cell, wave of configurations) partial result of the fused selection.
struct SelPart {
  double cost;     // least cost among the wave's feasible configurations, +inf if none
  double energy;   // energy of that configuration
  int32_t k;       // its index, -1 if none
  int32_t pad;
};

// Header at the start of every workspace.
struct WsHeader {
  uint32_t status;   // DYN_WS_* bits (final for an ingest workspace)
  uint32_t kind;     // 1: `status` is final; 2: per-cell status bytes still have to be OR-ed in
  int64_t cells;     // kind 2: number of per-cell status bytes
};
#define DYN_WS_HEADER_ORDER_WORD 8   // 32-bit word of a 256-byte header region used by the ingestion kernels
#define DYN_WS_HEADER_BARRIER_WORD 9 // arrival counter of the general sort's grid-wide barriers (zeroed with the header)
#define DYN_WS_KIND_WORD 1u
#define DYN_WS_KIND_CELLS 2u

// Layout of the evaluation workspace (offsets in bytes, all multiples of 256).
struct EvalWs {
  size_t header, tin, tout, in_p99, rec, cstat, part, total;
  int32_t n_wslot;   // partial records per cell
};
EvalWs dyn_eval_ws_layout(int64_t cells, int32_t K);

// ---- kernel launchers (each returns a hipError_t from the launch) ------------------------
hipError_t dyn_launch_cell_aggregate(const int32_t* in_tok, const int32_t* out_tok,
                                     const int64_t* cell_off, int64_t n_req, int64_t cells,
                                     double window_s, int32_t pct_num, int32_t pct_den,
                                     int64_t* tin, int64_t* tout, int32_t* in_p99, CellRec* rec,
                                     uint8_t* cstat, WsHeader* header, hipStream_t s);

struct SpaceArgs {
  const double* tab; const double* ml; const double* gridpack;
  const int32_t* jstart; int32_t n_bucket; double bucket_scale; bool one_step;
  int32_t G, n_tp_f /* n_tp*n_f */, n_rho;
  const DevCfg* cfg; int32_t K;
  int32_t tile, n_tile, n_slot;       // configurations per tile, tiles, LDS slots per tile
  const int32_t* tile_rows;           // [n_tile][n_slot] table rows staged by each tile (-1 = unused)
  const double* slo_ttft; const double* slo_tbt; const int32_t* budget;
  const CellRec* rec; int32_t n_window; int32_t win_per_block; double window_s;
  double* energy; double* p99_ttft; double* p99_tbt; uint8_t* flags;
  // fused selection (part != nullptr): per-wave partial argmin of cost = energy + idle term
  const double* pw0; double idle_w; SelPart* part; int32_t n_wslot;
};
hipError_t dyn_launch_space(const SpaceArgs& a, hipStream_t s);
int dyn_space_blocks_per_cu(const SpaceArgs& a);   // resident blocks of the evaluation kernel per compute unit (0: unknown)
size_t dyn_space_lds_tail(int32_t n_rho, int32_t n_bucket, int32_t win_per_block);   // LDS bytes besides the table rows

struct FinishArgs {   // reduces the partial records of every cell, then the window totals
  const SelPart* part; int32_t n_wslot; int32_t n_used; int32_t n_window, G;
  int32_t* sel; double* sel_energy; double* sel_cost; double* win_energy; int32_t* win_inf;
};
hipError_t dyn_launch_finish(const FinishArgs& a, hipStream_t s);

struct SelectArgs {
  const double* energy; const uint8_t* flags; const DevCfg* cfg; int32_t K;
  const double* pw0; int32_t G, n_tp_f; int32_t n_window; double window_s; double idle_w;
  int32_t* sel; double* sel_energy; double* sel_cost; double* win_energy; int32_t* win_inf;
};
hipError_t dyn_launch_select(const SelectArgs& a, hipStream_t s);

struct IngestArgs {
  const double* t_s; const int32_t* in_tok; const int32_t* out_tok; const int32_t* model;
  int64_t n_req; int32_t n_model, n_in_bin, n_out_bin, n_window; double window_s;
  const int32_t* d_in_edge; const int32_t* d_out_edge;   // device copies inside the workspace
  int32_t* in_sorted; int32_t* out_sorted; int64_t* cell_off;
  uint32_t* status; uint32_t* key_a; uint32_t* key_b; int32_t* in_tmp; int32_t* out_tmp;
  uint32_t* block_hist; int64_t n_block; int32_t key_bits;
  uint32_t* unsorted;      // word in the workspace header: 0 while every request's window is >= the one before
  int32_t force_sort;      // != 0: take the general sort whatever the order (the word then starts at 1)
  int64_t* win_off;        // workspace [n_window + 1]
};
hipError_t dyn_launch_ingest(const IngestArgs& a, hipStream_t s);
#define DYN_EDGE_PACK 960   // class edges that travel in one kernel's arguments
hipError_t dyn_launch_edges(const int32_t* in_edge, size_t n_in, const int32_t* out_edge, size_t n_out, int32_t* d_in,
                            int32_t* d_out, WsHeader* header, uint32_t order_word, hipStream_t s);
int64_t dyn_ingest_blocks(int64_t n_req);
#define DYN_INGEST_MAX_BINS 1024

void dyn_set_error(const char* fmt, ...);

// Optional event bracket around one kernel launch (see dyn_timing_enable).
struct DynTimed {
  DynTimed(int kernel, hipStream_t s);
  ~DynTimed();
  int kernel_;
  hipStream_t s_;
  int slot_;
};

#endif  // DYN_INTERNAL_H_
