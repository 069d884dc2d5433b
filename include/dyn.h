/*
 * dyn.h - C ABI of the batched evaluator of DynamoLLM's reconfiguration search space
 *         (arXiv 2408.00741) for AMD MI355X (gfx950).
 *
 * The paper's energy manager chooses, per pool of one request class, the number of
 * instances, the tensor-parallel degree and the GPU frequency that minimise energy under
 * P99 TTFT/TBT SLOs, using profiled energy/latency tables interpolated over load
 * (Section IV-A, Eq. 1; Section IV-B "Scale-up/down").  This library evaluates that whole
 * search space at once: for every (time window, request class) cell and every candidate
 * configuration it computes the predicted P99 TTFT, P99 TBT, energy and SLO feasibility,
 * and then the least-cost feasible configuration per cell.
 *
 * Conventions shared by every entry point
 *   - Return value: DYN_OK (0) or a negative dyn_status.  Nothing throws or aborts.
 *     dyn_last_error() gives a message for the last failure on the calling thread.
 *   - "HOST" pointers are read during the call and may be freed on return.
 *     "DEVICE" pointers are memory of the current HIP device owned by the caller; the
 *     library never frees them.  Only dyn_profile_load allocates device memory (released by
 *     dyn_profile_free).
 *   - Work is enqueued on `hip_stream` (a hipStream_t passed as void*; NULL = the default
 *     stream) and the call returns after enqueueing; no entry point waits for the device
 *     except dyn_profile_load and dyn_workspace_status, and any call whose candidate list,
 *     objective or small host tables (layouts, transition table, controller lists) differ
 *     from the copies the profile handle keeps: those are uploaded after waiting for the
 *     stream.  The status covers argument checks and launch errors.  Conditions that depend on device data (an offset array that is
 *     not monotone, a timestamp outside the windows) cannot be seen by the host: the
 *     kernels bound-check them, skip the offending item and raise a bit in the status
 *     word at the start of the workspace, which dyn_workspace_status reads back.
 *   - Cells are numbered cell = w * G + g with w the window and g the class,
 *     g = (model * n_in_bin + in_bin) * n_out_bin + out_bin.
 *   - All floating point is IEEE binary64 without contraction.  Window and tick lengths,
 *     max_load_tps and the spacings of the load grid must lie in [1e-100, 1e100]
 *     (DYN_E_RANGE / DYN_E_NOTFINITE otherwise): inside that range every division of the
 *     method is reproduced exactly by the kernels' reciprocal-based form.
 */
#ifndef DYN_H_
#define DYN_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  DYN_OK = 0,
  DYN_E_NULL = -1,      /* a required pointer is NULL                                   */
  DYN_E_SHAPE = -2,     /* a count or dimension is out of range or inconsistent         */
  DYN_E_RANGE = -3,     /* a value is outside its allowed range                         */
  DYN_E_NOTFINITE = -4, /* a table entry is NaN, infinite or negative                   */
  DYN_E_ORDER = -5,     /* a grid or edge list is not strictly increasing               */
  DYN_E_WORKSPACE = -6, /* workspace missing, misaligned (256 B) or too small           */
  DYN_E_DEVICE = -7     /* a HIP call failed                                            */
} dyn_status;

/* Message of the last error on this thread; static storage, never freed by the caller. */
const char* dyn_last_error(void);

/* ------------------------------------------------------------------ profile tables -----
 * Section IV-A, "Generating LLM profiles": the profile is a function of (load, request
 * class, tensor parallelism, GPU frequency) giving expected energy and TTFT/TBT; it is
 * measured at a few load levels up to the maximum throughput and taken linearly in
 * between (Section IV-E: one-dimensional linear interpolation).
 * Tables are row-major [n_class][n_tp][n_f][n_rho]; the load axis `rho` is the
 * per-instance load divided by max_load_tps (tokens/s one instance sustains at that
 * class, TP and frequency).  All HOST pointers; the library keeps device copies.       */
typedef struct {
  int32_t n_class;                  /* G >= 1, all models' classes                        */
  int32_t n_tp;                     /* >= 1                                               */
  const int32_t* tp;                /* [n_tp] GPUs per instance, >= 1, strictly increasing */
  int32_t n_f;                      /* >= 1                                               */
  const double* f_mhz;              /* [n_f] profiled frequencies, strictly increasing    */
  int32_t n_rho;                    /* >= 2                                               */
  const double* rho;                /* [n_rho] load grid, strictly increasing, rho[0]==0  */
  const double* prefill_ms_per_tok; /* [G][n_tp][n_f][n_rho] finite, >= 0                  */
  const double* tbt_ms;             /* [G][n_tp][n_f][n_rho] finite, >= 0                  */
  const double* power_w;            /* [G][n_tp][n_f][n_rho] watts of one whole instance   */
  const double* max_load_tps;       /* [G][n_tp][n_f] within [1e-100, 1e100]               */
} dyn_profile_desc;

/* Opaque; owns the device copies of the tables and of the candidate list and objective it
 * was last used with, so that repeated calls with the same candidates upload nothing.
 * A handle must not be used by two host threads at once, and a call that changes the
 * candidate list or the SLOs first waits for `hip_stream`; work still in flight on
 * another stream must not be using the same handle at that moment.  Calls with the same
 * candidates and objective may be in flight on several streams at once when each has its
 * own outputs and workspace (one call's aggregation then overlaps another's stores).
 * Limits: at most 65536 candidate configurations.                                      */
typedef struct dyn_profile dyn_profile;

/* Validates the tables (DYN_E_NULL/SHAPE/ORDER/RANGE/NOTFINITE), copies them to the
 * current device on `hip_stream` and waits for the copy.  *out receives the handle. */
int dyn_profile_load(const dyn_profile_desc* desc, void* hip_stream, dyn_profile** out);
void dyn_profile_free(dyn_profile* p); /* NULL is allowed */

/* ---------------------------------------------------------------- trace ingestion -----
 * Section III: a trace record is (arrival timestamp, input tokens, output tokens).
 * Section III-A, Table IV: requests are classified by input and output length; a length
 * equal to a threshold belongs to the upper bin.  Windows are the controllers' epochs
 * (Section IV-B): w = floor(t_s / window_s) in binary64.                               */
typedef struct {
  int32_t n_model, n_in_bin, n_out_bin; /* G = n_model * n_in_bin * n_out_bin            */
  const int32_t* in_edge;  /* HOST [n_model][n_in_bin-1], strictly increasing per model  */
  const int32_t* out_edge; /* HOST [n_model][n_out_bin-1]; bin = #{edges e : x >= e}     */
} dyn_class_edges;

size_t dyn_trace_ingest_workspace(int64_t n_req, int32_t n_window, int32_t n_class);

/* Reorders a raw trace by cell, keeping arrival order inside a cell (a stable sort), and
 * writes the start offset of every cell.
 *   t_s, in_tok, out_tok, model : DEVICE [n_req]; model may be NULL (all model 0); time
 *                                 order is not required.
 *   in_sorted, out_sorted       : DEVICE [n_req] outputs; must not alias the inputs.
 *   cell_off                    : DEVICE [n_window*G + 1] output, cell_off[last] = n_req.
 *   workspace                   : DEVICE, 256-byte aligned, >= dyn_trace_ingest_workspace.
 * A trace already in window order is moved window by window, any other by a general stable
 * sort; the route is picked on the device (the call does not wait for it), both give the same
 * bytes.  The edge lists travel in kernel arguments, so the HOST arrays are free on return.
 * A request whose timestamp falls outside [0, n_window*window_s) or whose model index is
 * outside [0, n_model) raises DYN_WS_BAD_REQUEST in the workspace status and is filed
 * under the nearest valid window / model 0, so that offsets stay consistent.  The general
 * sort runs as one kernel whose blocks wait for each other between its phases; the wait is
 * bounded: should other work hold the device for seconds, every block leaves, the outputs
 * are not valid and DYN_WS_SORT_ABANDONED is raised.
 * Limits: n_window * G < 2^30.                                                         */
int dyn_trace_ingest(const double* t_s, const int32_t* in_tok, const int32_t* out_tok,
                     const int32_t* model, int64_t n_req, const dyn_class_edges* edges,
                     int32_t n_window, double window_s, int32_t* in_sorted, int32_t* out_sorted,
                     int64_t* cell_off, void* workspace, size_t workspace_bytes,
                     void* hip_stream);

/* The cell-sorted trace the evaluator reads.  All DEVICE pointers, caller-owned. */
typedef struct {
  int64_t n_req;
  int32_t n_window;
  double window_s;        /* seconds, within [1e-100, 1e100]                            */
  const int32_t* in_tok;  /* [n_req] sorted by cell                                     */
  const int32_t* out_tok; /* [n_req]                                                    */
  const int64_t* cell_off; /* [n_window*G + 1] non-decreasing, [0]==0, last == n_req    */
} dyn_trace_view;

/* ------------------------------------------------- candidates, SLOs and objective -----
 * Section IV-A: the knobs are the number of instances, their tensor parallelism and
 * their frequency; all instances of a pool share the load equally.                     */
typedef struct {
  int32_t n_inst;   /* >= 1                                                             */
  int32_t tp_index; /* index into dyn_profile_desc.tp                                   */
  double f_mhz;     /* within [f_mhz[0], f_mhz[n_f-1]] of the profile, else DYN_E_RANGE */
} dyn_config;

/* Eq. 1: minimise sum N x Energy subject to GPUs <= budget and Performance <= SLO;
 * Section III-A: the SLO statistic is the P99 latency.                                 */
typedef struct {
  const double* slo_ttft_ms; /* HOST [G]                                                */
  const double* slo_tbt_ms;  /* HOST [G]                                                */
  int32_t pct_num, pct_den;  /* percentile = pct_num/pct_den in (0, 1]; 99, 100         */
  const int32_t* gpu_budget; /* HOST [G] or NULL; 0 = unlimited; needs n_inst*tp <= it  */
  double idle_cost_weight;   /* cost = energy + weight * n_inst * power(load 0) * window */
} dyn_objective;

/* The evaluated space.  DEVICE pointers, caller-owned, each [n_window*G][K], k fastest. */
typedef struct {
  double* energy_j;    /* n_inst * power * window_s                                     */
  double* p99_ttft_ms; /* nearest-rank percentile of per-request TTFT; 0 for an empty cell */
  double* p99_tbt_ms;
  uint8_t* flags;
} dyn_space;
#define DYN_F_FEASIBLE 1u /* none of the four violations below                          */
#define DYN_F_OVERLOAD 2u /* per-instance load beyond the last profiled point           */
#define DYN_F_TTFT 4u     /* p99_ttft_ms > slo_ttft_ms[g]                               */
#define DYN_F_TBT 8u      /* p99_tbt_ms  > slo_tbt_ms[g]                                */
#define DYN_F_BUDGET 16u  /* n_inst * tp > gpu_budget[g] > 0                            */
#define DYN_F_EMPTY 32u   /* the cell holds no request                                  */

/* Status bits kept in the first 4 bytes of a workspace. */
#define DYN_WS_BAD_OFFSETS 1u /* cell_off not monotone / outside [0, n_req]: cell treated as empty */
#define DYN_WS_BAD_REQUEST 2u /* ingest: timestamp or model index out of range          */
#define DYN_WS_TICK_RANK 4u   /* not raised any more (tick evaluation once left cells deeper than DYN_TICK_DEPTH out) */
#define DYN_WS_SORT_ABANDONED 8u /* ingest: the general sort stopped waiting for its own blocks after seconds
                                  * (the device was held by other work); the sorted outputs are not valid  */

/* Bytes of workspace dyn_eval_space needs (a multiple of 256). */
size_t dyn_eval_space_workspace(int32_t n_window, int32_t n_class, int32_t n_config);

/* Evaluates every (cell, configuration) pair.
 * Per cell: load L = (sum of input + output tokens) / window_s (Section III-A: load in
 * tokens per second); per configuration: rho = L / (n_inst * max_load_tps) (fair share,
 * Section IV-A); prefill ms/token, TBT and power from the tables at (f_mhz, min(rho,
 * rho_max)), interpolated along rho on the two bracketing frequency rows and then along
 * f; per-request TTFT = input tokens * prefill ms/token, per-request TBT = the table's
 * TBT; the P99 of both over the cell (nearest rank, rank = ceil(pct_num*m/pct_den));
 * energy; and the feasibility flags (Eq. 1 constraints 1 and 3).
 * Arguments: `cfg` HOST [K]; `out` arrays DEVICE; workspace DEVICE, 256-byte aligned, at
 * least dyn_eval_space_workspace bytes; it keeps the per-cell aggregates that
 * dyn_cell_stats returns.  Errors: see dyn_status; nothing is launched on error.        */
int dyn_eval_space(dyn_profile* profile, const dyn_trace_view* trace, const dyn_config* cfg,
                   int32_t K, const dyn_objective* objective, const dyn_space* out,
                   void* workspace, size_t workspace_bytes, void* hip_stream);

/* Per-cell aggregates of the last dyn_eval_space on `workspace` (exact integers):
 * tok_in, tok_out = token sums, in_p99 = input length of nearest rank (0 if empty).
 * Outputs DEVICE [n_window*G]; any may be NULL.  Enqueues device-to-device copies.      */
int dyn_cell_stats(const void* workspace, size_t workspace_bytes, int32_t n_window,
                   int32_t n_class, int64_t* tok_in, int64_t* tok_out, int32_t* in_p99,
                   void* hip_stream);

/* Reads the workspace status word (DYN_WS_* bits) after waiting for `hip_stream`. */
int dyn_workspace_status(const void* workspace, void* hip_stream, uint32_t* status);

/* Per-cell selection and per-window totals.  DEVICE pointers, caller-owned. */
typedef struct {
  int32_t* sel;               /* [cells] index of the chosen configuration, -1 if none  */
  double* sel_energy_j;       /* [cells] its energy, +inf if none                       */
  double* sel_cost;           /* [cells] its cost,   +inf if none                       */
  double* window_energy_j;    /* [n_window] sum of sel_energy_j over classes with a choice, g ascending */
  int32_t* window_infeasible; /* [n_window] number of classes with sel == -1            */
} dyn_selection;

/* Section IV-B "Scale-up/down": drop what violates the SLO, then take the least energy.
 * Reads space->energy_j and space->flags; cost = energy + idle_cost_weight * n_inst *
 * power(load 0 at that TP and f) * window_s; the lowest index wins exact ties.
 * `cfg` HOST [K].  space->p99_* are not read and may be NULL.                          */
int dyn_select_config(dyn_profile* profile, const dyn_space* space, const dyn_config* cfg,
                      int32_t K, const dyn_objective* objective, int32_t n_window,
                      double window_s, const dyn_selection* out, void* hip_stream);

/* dyn_eval_space and dyn_select_config in one pass: the selection is reduced inside the
 * evaluation kernel (per wave of configurations) and finished by a small kernel, so the
 * evaluated space is written once and not read back.  Outputs are identical to calling
 * the two entry points one after the other with the same arguments.  `space` and `sel`
 * DEVICE arrays as documented above; same workspace as dyn_eval_space.                  */
int dyn_eval_select(dyn_profile* profile, const dyn_trace_view* trace, const dyn_config* cfg,
                    int32_t K, const dyn_objective* objective, const dyn_space* space,
                    const dyn_selection* sel, void* workspace, size_t workspace_bytes,
                    void* hip_stream);

/* Measurement aid, optional: times dyn_eval_select on the caller's own buffers for several shapes of
 * the evaluation kernel's blocks (how many windows one block walks: more amortise the staging of
 * the table rows, fewer keep the streams the chip writes at a time closer together) and keeps the
 * fastest in the profile handle, for this candidate list and this number of windows, until the
 * list changes.  Without it a rule picks the shape.  The shape does not change any result: every
 * run writes the same values, and `space` / `sel` hold them on return.  Arguments as for
 * dyn_eval_select; `chosen` (HOST, may be NULL) receives the windows per block.  Waits for the
 * stream between the runs (a few dozen evaluations in all).                               */
int dyn_eval_tune(dyn_profile* profile, const dyn_trace_view* trace, const dyn_config* cfg, int32_t K,
                  const dyn_objective* objective, const dyn_space* space, const dyn_selection* sel,
                  void* workspace, size_t workspace_bytes, void* hip_stream, int32_t* chosen);

/* dyn_eval_select for callers that cannot allocate device memory: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same computation and outputs as
 * dyn_eval_select, but the workspace is a fixed array of DYN_STATIC_WORKSPACE_BYTES that the
 * library keeps on every GPU it runs on until the process ends; the call allocates and frees
 * nothing.  n_window * G cells with K configurations must satisfy
 * dyn_eval_space_workspace(n_window, G, K) <= DYN_STATIC_WORKSPACE_BYTES (the one-day workload
 * of 36000 cells x 576 configurations needs 13.1 MB), else DYN_E_WORKSPACE and nothing is launched.
 * `status` (DEVICE, one word, may be NULL) receives the DYN_WS_* bits of this call.
 * All calls on one GPU share the array: calls that overlap in time on one GPU (two streams, two
 * host threads) race; every call rewrites all of it that it reads, so nothing has to be cleared
 * between calls.  As with dyn_eval_select, a candidate list or objective that differs from the one
 * the profile handle holds is uploaded first, which waits for the stream: make the first call
 * with a new list outside a graph capture.                                                */
#define DYN_STATIC_WORKSPACE_BYTES (16u << 20)
int dyn_eval_select_static(dyn_profile* profile, const dyn_trace_view* trace, const dyn_config* cfg,
                           int32_t K, const dyn_objective* objective, const dyn_space* space,
                           const dyn_selection* sel, uint32_t* status, void* hip_stream);

/* ----------------------------------------------------------- tick-level load in a window --
 * Section IV-B "Scale-up/down": inside a window the instance manager follows the load at
 * a finer grain (every few seconds) than the window the configuration is chosen for.  Here
 * every window is split into n_tick ticks of tick_s seconds; each request is served under
 * the load of its own tick: per tick the load is that tick's tokens / tick_s and the
 * tables are looked up at it; per-request TTFT = input tokens * the tick's prefill
 * ms/token, per-request TBT = the tick's TBT; the percentiles are taken over all requests
 * of the (window, class) cell; energy = sum over the ticks, in time order, of
 * (n_inst * power) * tick_s; a configuration is overloaded when it is in any tick; the
 * idle term of the cost uses the window length (double) n_tick * tick_s.  With
 * n_tick == 1 every output equals dyn_eval_select's.
 *
 * `fine` is the trace sorted by tick: the result of dyn_trace_ingest with
 * n_window * n_tick windows of tick_s seconds (fine->n_window = n_window * n_tick,
 * fine->window_s = tick_s; tick q of window w is fine window w * n_tick + q).
 * `space` and `sel` are indexed by the coarse cell w * G + g: [n_window*G][K], [n_window*G]
 * and [n_window].  1 <= n_tick <= DYN_TICK_LIMIT, else DYN_E_SHAPE.
 * The percentile of a cell with m requests is its j-th largest value, j = m - rank + 1; any
 * j is evaluated (DYN_TICK_DEPTH is the depth up to which a tick's list is cut down to its
 * j largest input lengths; beyond it whole ticks are sorted, long ones in pieces).
 * Workspace: dyn_eval_ticks_workspace bytes (it depends on the number of requests: the
 * per-tick candidate lists take 4 bytes per request), DEVICE, 256-byte aligned.          */
#define DYN_TICK_LIMIT 64
#define DYN_TICK_DEPTH 8192
size_t dyn_eval_ticks_workspace(int64_t n_req, int32_t n_window, int32_t n_tick, int32_t n_class, int32_t n_config);
int dyn_eval_select_ticks(dyn_profile* profile, const dyn_trace_view* fine, int32_t n_tick,
                          const dyn_config* cfg, int32_t K, const dyn_objective* objective,
                          const dyn_space* space, const dyn_selection* sel, void* workspace,
                          size_t workspace_bytes, void* hip_stream);

/* ------------------------------------------------- pools that mix instance types (Eq. 1) --
 * Eq. 1 in full: per (window, class) cell choose the number of instances of every tensor
 * parallelism (N^TP), their frequency (f^TP) and the part of the load each type takes
 * (L^TP) so that the total energy is least, the GPUs used stay within the class's budget,
 * the parts add up to the load and every used type meets the SLO under its part.
 * The load is split in n_share equal shares; type i takes a_i >= 1 of them exactly when it
 * is used (sum a_i = n_share) and its n_i instances share that part equally: per-instance
 * load = (L * a_i / n_share) / n_i.  Frequencies are the profiled ones.  Per type the
 * frequency is chosen as in Section IV-B "Scale-up/down" (drop what violates the SLO or
 * leaves the profiled load range, then least energy, lowest frequency on ties); the
 * percentiles of a type are taken over all requests of the cell under that type's tables.
 * Total energy = 0 + E_0 + E_1 + ... over the used types in type order,
 * E_i = n_i * power * window_s.  objective->gpu_budget[g] > 0 bounds sum n_i * tp_i;
 * objective->idle_cost_weight is not used.
 * Limits: n_share <= DYN_MIXED_MAX_SHARES, profile n_tp <= DYN_MIXED_MAX_TYPES and
 * n_f <= 16, n_max[i] in [0, 255]; the per-cell state (GPU units x shares) must fit in LDS,
 * else DYN_E_SHAPE.  Outputs DEVICE, caller-owned: where several assignments reach the least
 * energy any one of them is returned.                                                    */
#define DYN_MIXED_MAX_TYPES 8
#define DYN_MIXED_MAX_SHARES 16
typedef struct {
  int32_t n_share;        /* S: equal shares the pool's load is split into                */
  const int32_t* n_max;   /* HOST [n_tp] most instances of each type considered (0 = type not used) */
} dyn_mixed_space;
typedef struct {
  double* energy_j;           /* [cells] least total energy, +inf if no assignment is feasible */
  int32_t* n_inst;            /* [cells][n_tp] instances of each type (0 = type unused)   */
  int32_t* f_index;           /* [cells][n_tp] index into the profile's f_mhz, -1 if unused */
  int32_t* share;             /* [cells][n_tp] shares given to each type (sum = n_share)  */
  double* window_energy_j;    /* [n_window] sum over the classes with an assignment, g ascending */
  int32_t* window_infeasible; /* [n_window] classes without one                           */
} dyn_mixed_selection;
size_t dyn_mixed_workspace(const dyn_profile* profile, int32_t n_window, const dyn_mixed_space* space);
int dyn_eval_select_mixed(dyn_profile* profile, const dyn_trace_view* trace, const dyn_mixed_space* space,
                          const dyn_objective* objective, const dyn_mixed_selection* out,
                          void* workspace, size_t workspace_bytes, void* hip_stream);

/* ------------------------------------- selection with transition overheads across windows --
 * Section IV-B "Accounting for the overheads": the cost of changing the configuration is
 * weighed against the energy the new one saves (Table VI: re-sharding overheads between the
 * layouts of a server).  Per class the configurations of all windows are chosen together so
 * that  sum_w cost(w, k_w) + sum_{w>=1} transition_j[layout[k_{w-1}]][layout[k_w]]  is least;
 * cost and feasibility as in dyn_select_config (reads space->energy_j and space->flags).
 * The total of a sequence is accumulated in time order: V = cost(0, k_0);
 * V = (V + transition) + cost(w, k_w).  A window without a feasible configuration gets -1,
 * ends the sequence before it and the next window starts a new one without a transition;
 * path_cost[g] adds the sequences' totals in time order from 0.  Where several sequences
 * reach the least total any one of them is returned.
 * `layout` HOST [K] in [0, n_layout); `transition_j` HOST [n_layout][n_layout], row = from,
 * finite and >= 0.  Limits: up to 64 layouts any K the profile handle takes; beyond that
 * n_layout <= 255, K <= 2048 and the per-class state (K totals, the transition table) must
 * fit in LDS: (K + n_layout^2) * 8 bytes + small <= 64 KB, else DYN_E_SHAPE.
 * `layout` and `transition_j` are kept in the profile handle like the candidate list: a call
 * with the same tables as the one before uploads nothing and does not wait for the stream.
 * Workspace DEVICE, 256-byte aligned, dyn_select_path_workspace bytes.                    */
typedef struct {
  int32_t n_layout;
  const int32_t* layout;
  const double* transition_j;
} dyn_transitions;
typedef struct {
  int32_t* sel;               /* [cells] chosen configuration, -1 where the window has none */
  double* sel_energy_j;       /* [cells] its energy, +inf where sel == -1                  */
  double* path_cost;          /* [G] total cost of the class's sequences incl. transitions */
  double* window_energy_j;    /* [n_window] as in dyn_selection                            */
  int32_t* window_infeasible; /* [n_window]                                                */
} dyn_path_selection;
size_t dyn_select_path_workspace(int32_t n_window, int32_t n_class, int32_t n_config, int32_t n_layout);
int dyn_select_path(dyn_profile* profile, const dyn_space* space, const dyn_config* cfg, int32_t K,
                    const dyn_objective* objective, const dyn_transitions* transitions,
                    int32_t n_window, double window_s, const dyn_path_selection* out,
                    void* workspace, size_t workspace_bytes, void* hip_stream);

/* ---------------------------------------------------------- cost and carbon of a selection --
 * Section VI "Cost and Carbon Emission": the user's cost follows the GPU servers in use over
 * time and the energy bill; operational CO2 is each interval's energy times the grid's
 * carbon intensity at that time.  Per window: GPUs = sum over the classes with a selection
 * (sel >= 0) of n_inst * tp; GPU-hours = ((double) GPUs * window_s) / 3600; GPU cost =
 * GPU-hours * gpu_hour_price; kWh = window_energy_j / 3.6e6; energy cost = kWh * kwh_price;
 * carbon = kWh * carbon_g_per_kwh[w]; servers = ceil(GPUs / gpus_per_server).
 * totals[5] = {GPU-hours, GPU cost, energy cost, carbon in g, servers summed over the
 * windows}, each added in window order from 0.
 * `sel` DEVICE [n_window*G] and `window_energy_j` DEVICE [n_window] as a selection entry point
 * returns them; `carbon_g_per_kwh` DEVICE [n_window]; outputs DEVICE; `cfg` HOST [K] (the
 * candidate list the selection indexes).  Workspace DEVICE, 256-byte aligned,
 * dyn_account_workspace bytes; its status word reports sel values >= K (DYN_WS_BAD_REQUEST),
 * which count as no selection.                                                           */
typedef struct {
  double gpu_hour_price;       /* currency per GPU-hour                                   */
  double kwh_price;            /* currency per kWh                                        */
  const double* carbon_g_per_kwh; /* DEVICE [n_window]                                    */
  int32_t gpus_per_server;     /* >= 1                                                    */
} dyn_rates;
typedef struct {
  int64_t* gpus;       /* [n_window] */
  double* gpu_cost;    /* [n_window] */
  double* energy_cost; /* [n_window] */
  double* carbon_g;    /* [n_window] */
  double* totals;      /* [5]        */
} dyn_accounting;
size_t dyn_account_workspace(int32_t n_window);
int dyn_account(dyn_profile* profile, const int32_t* sel, const double* window_energy_j,
                const dyn_config* cfg, int32_t K, int32_t n_window, double window_s,
                const dyn_rates* rates, const dyn_accounting* out, void* workspace,
                size_t workspace_bytes, void* hip_stream);

/* --------------------------------------------------------- the hierarchy of controllers --
 * Section IV-B "Hierarchical Control": instead of one global search, three controllers set
 * one knob each, top down, each assuming the ones below run at the highest performance.
 *   Scale-out/in, every epoch of `epoch_windows` windows: nodes = ceil(PL / ML) per class,
 *     PL = the peak of the class's load over the epoch's windows (the load predictor is taken
 *     to be exact), ML = the largest profiled load of one node at the reference
 *     configuration (tp_ref_index, f_ref_index; the paper's TP8 at 1980 MHz):
 *     (gpus_per_node / tp) instances * max_load_tps * last load-grid point; at least 1 node.
 *   Shard-up/down, every window: among the layouts (lay_n[l] instances of TP lay_tp_index[l])
 *     with n * tp <= nodes * gpus_per_node, evaluated at f_ref under the window's load with
 *     the percentiles over the window's requests, the one of least energy that meets the
 *     SLO (lowest l on ties); -1 and energy +inf if none.
 *   Scale-up/down, every tick: for that layout, among the profiled frequencies, drop those
 *     that violate the SLO under the tick's load (percentiles over the tick's requests) or
 *     leave the profiled load range, then take the least power (lowest frequency on ties);
 *     if none is left the tick runs at f_ref and counts as a violation.
 *   Energy of a (window, class) = sum over its ticks in time order of (n * power) * tick_s.
 *   With controllers->transition_j (Section IV-B "Accounting for the overheads", Table VI;
 *     HOST [n_layout][n_layout] joules, from -> to, finite and >= 0): the shard controller
 *     chooses the layouts of all windows of a class together, as dyn_select_path does with one
 *     candidate per layout, cost = the layout's energy at f_ref over the window and feasible =
 *     fits the nodes' GPUs and meets the SLO; out->path_cost[g] (DEVICE [G], required then) =
 *     that class's total of energies and overheads.  Where several sequences reach the least
 *     total any one of them is returned.  Limits as for dyn_select_path with K = n_layout.
 *     NULL: every window takes its own least-energy layout and path_cost is not written.
 *   With controllers->spill != 0 (Section IV-B "Handling fragmentation"): a pool whose peak does
 *     not fill its last node gets that node less and the load its other nodes cannot carry is
 *     forwarded to the pool of the next class (classes are taken to be ordered by request
 *     size); only the last class rounds up.  Per epoch, classes ascending: arriving load of a
 *     window A = own load + what the class below forwards, PL = peak of A, q = PL / ML.  If the
 *     class is not the last and 1 <= floor(q) < q: nodes = floor(q) and the pool serves the
 *     fraction keep = ((floor(q) * ML) / PL) * (1 - 2^-40) of what arrives (the last factor
 *     keeps the peak window inside the profiled load range whatever the later roundings);
 *     otherwise nodes = ceil(q), at least 1, and keep = 1.  Served load S = keep * A in every
 *     window and every tick of the epoch, forwarded load = A - S.  The shard and frequency
 *     controllers see S; percentiles stay those of the pool's own requests.  out->keep
 *     (DEVICE [n_epoch][G], may be NULL) receives the fractions; it is not written without spill.
 * `coarse` is the trace sorted by window (n_window windows of n_tick * tick_s seconds), `fine`
 * the same requests sorted by tick (n_window * n_tick windows of tick_s seconds), both as
 * dyn_trace_ingest returns them.  lay_n / lay_tp_index HOST [n_layout].  Outputs DEVICE.
 * objective->gpu_budget and idle_cost_weight are not used.  Profiles of more than 64 TP
 * degrees or 4096 classes are refused (DYN_E_SHAPE), as are more than 65536 layouts (255 with
 * a transition table).  The layout list and the table are kept in the profile handle: a call
 * with the same ones as the call before uploads nothing and does not wait for the stream.  */
typedef struct {
  int32_t epoch_windows;
  int32_t tp_ref_index, f_ref_index;
  int32_t gpus_per_node;
  int32_t n_layout;
  int32_t spill;              /* != 0: the fragmentation rule */
  const int32_t* lay_n;
  const int32_t* lay_tp_index;
  const double* transition_j; /* HOST [n_layout][n_layout] or NULL */
} dyn_controllers;
typedef struct {
  int32_t* nodes;             /* [n_epoch][G], n_epoch = ceil(n_window / epoch_windows)    */
  int32_t* layout_sel;        /* [n_window*G] index into the layout list, -1 if none       */
  int32_t* f_sel;             /* [n_window*n_tick][G] index into the profile's f_mhz, -1   */
  double* energy_j;           /* [n_window*G], +inf where layout_sel == -1                 */
  int32_t* violations;        /* [n_window*G] ticks that had to run at f_ref               */
  double* window_energy_j;    /* [n_window] */
  int32_t* window_infeasible; /* [n_window] */
  double* path_cost;          /* [G], only with transition_j; may be NULL without */
  double* keep;               /* [n_epoch][G], only with spill; may be NULL                */
} dyn_hierarchy_out;
size_t dyn_hierarchy_workspace(int32_t n_window, int32_t n_tick, int32_t n_class, int32_t n_layout);
int dyn_hierarchy(dyn_profile* profile, const dyn_trace_view* coarse, const dyn_trace_view* fine,
                  int32_t n_tick, const dyn_controllers* controllers, const dyn_objective* objective,
                  const dyn_hierarchy_out* out, void* workspace, size_t workspace_bytes,
                  void* hip_stream);

/* ------------------------------------------------------------- kernel timing (optional) --
 * Measurement aid, not part of the method: when enabled, the library brackets each of its
 * kernels with a pair of HIP events recorded on the stream the kernel is launched on, so
 * that a caller can obtain per-kernel durations of its own timed region without a
 * profiler.  Off by default (no events are recorded).                                   */
#define DYN_K_CELL 0    /* per-cell aggregation + rank selection                        */
#define DYN_K_SPACE 1   /* evaluation of the (cell, configuration) space                */
#define DYN_K_SELECT 2  /* per-cell least-cost feasible configuration (or its fused finish) */
#define DYN_K_TOTALS 3  /* per-window totals                                            */
#define DYN_K_TICK_TOP 4   /* tick evaluation: per-tick loads, ranks among the ties or candidate lists (all the per-cell kernels) */
#define DYN_K_TICK_SPACE 5 /* tick evaluation of the (cell, configuration) space: the two walks over the ticks */
#define DYN_K_TICK_MERGE 6 /* the same for the (cell, tile) items the walk cannot settle    */
#define DYN_K_MIXED_TYPES 7   /* mixed pools: per-type least energies                      */
#define DYN_K_MIXED_COMBINE 8 /* mixed pools: assignment of instances and shares          */
#define DYN_K_PATH 9          /* selection with transition overheads                     */
#define DYN_K_HIER 10         /* the four kernels of the controller hierarchy            */
#define DYN_K_COUNT 11
/* on != 0: create the event pool (up to `max_launches` launches per kernel are recorded,
 * later ones are not) and start recording; on == 0: stop and destroy the pool.         */
int dyn_timing_enable(int on, int32_t max_launches);
/* Forget what was recorded so far (the pool is kept). */
int dyn_timing_reset(void);
/* Waits for the recorded events of `kernel` and returns their summed duration and count. */
int dyn_timing_read(int32_t kernel, double* total_ms, int64_t* launches);

#ifdef __cplusplus
}
#endif
#endif /* DYN_H_ */
