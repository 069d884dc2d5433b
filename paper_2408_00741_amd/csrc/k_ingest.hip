// Trace ingestion: every request gets the key of its cell (window from the timestamp,
// class from the input/output length bins of Table IV's convention), then a stable
// least-significant-digit radix sort by key moves (input tokens, output tokens) into cell
// order, and the cell offsets are read off the sorted keys.
//
// A trace that is already in window order (a request log is in time order) does not need the
// general sort: the key kernel notices it (a flag word in the workspace header stays 0; it also
// writes where every window starts), and one block per window then counts its requests by class
// and moves them, stably, to their cells (window_sort_kernel).  Any other trace takes the radix
// sort.  The host does not read the flag: both routes are enqueued and the kernels of the route
// not taken return at their first instruction.  The general sort is one launch of a grid the device
// holds at once, with grid-wide barriers between the phases, so the route not taken costs one empty
// launch; where the device does not tell what it holds it is the separate kernels below.
//
// One radix pass = per-block digit histogram -> exclusive scan of the (digit, block)
// counters -> stable scatter.  Inside a block every wave owns a contiguous run of rows of
// 64 requests and walks them in order; the position of a request among the requests of
// its row with the same digit comes from wave ballots, so arrival order is preserved.
#include <string.h>

#include <algorithm>
#include <atomic>

#include "dyn_internal.h"
#include "dyn_device.h"

namespace {

constexpr int kWaves = 4;
constexpr int kRows = 32;                              // rows of 64 requests per wave
constexpr int kTile = kWaves * kRows * DYN_WAVE;       // 8192 requests per block
constexpr int kScanChunk = 4096;                       // counters per block of the scan kernels

constexpr int kKeyRows = 4;                            // requests per thread of the key kernel (rows of 256)

// Window of a timestamp: floor(t / window_s), the quotient formed from RN(1 / window_s) by div_by (correctly rounded
// for timestamps whose quotient is a normal number; a handful of multiply-adds instead of a division).  Quotients that are
// not finite, and tiny ones (below 2^-900, where a residual could underflow), take the IEEE division; clamped, out-of-range flagged.
__device__ __forceinline__ double window_of(double t, double window_s, double r_window, int32_t n_window, uint32_t* bad) {
  double q = div_by(t, window_s, r_window);
  if (!(fabs(q) >= 0x1p-900 && fabs(q) <= 0x1p900)) q = t / window_s;   // also NaN: a residual step on an infinite product
  double wq = floor(q);
  if (!(wq >= 0.0)) { *bad = DYN_WS_BAD_REQUEST; wq = 0.0; }                      // negative or NaN
  if (!(wq < (double)n_window)) { *bad = DYN_WS_BAD_REQUEST; wq = (double)(n_window - 1); }
  return wq;
}

// A block takes kKeyRows rows of 256 consecutive requests (all loads of a thread in flight together); the class
// edges sit in LDS when they fit (lds_edges != 0).
__global__ __launch_bounds__(256) void key_kernel(IngestArgs a, double r_window, int lds_edges) {
  extern __shared__ int32_t s_edge[];                  // [n_model][n_in_bin - 1] then [n_model][n_out_bin - 1]
  const int n_ie = a.n_in_bin - 1, n_oe = a.n_out_bin - 1;
  const int32_t* in_edge = a.d_in_edge;
  const int32_t* out_edge = a.d_out_edge;
  if (lds_edges) {
    for (int q = threadIdx.x; q < a.n_model * n_ie; q += blockDim.x) s_edge[q] = a.d_in_edge[q];
    for (int q = threadIdx.x; q < a.n_model * n_oe; q += blockDim.x) s_edge[a.n_model * n_ie + q] = a.d_out_edge[q];
    __syncthreads();
    in_edge = s_edge;
    out_edge = s_edge + a.n_model * n_ie;
  }
  const int lane = threadIdx.x & (DYN_WAVE - 1);
  const int64_t base = (int64_t)blockIdx.x * (kKeyRows * 256) + threadIdx.x;
  double t[kKeyRows], tp[kKeyRows];
  int32_t x[kKeyRows], y[kKeyRows], md[kKeyRows];
#pragma unroll
  for (int r = 0; r < kKeyRows; ++r) {
    const int64_t i = base + r * 256;
    const bool in = i < a.n_req;
    t[r] = in ? a.t_s[i] : 0.0;
    tp[r] = (in && lane == 0 && i > 0) ? a.t_s[i - 1] : 0.0;   // the request before a wave's first
    x[r] = in ? a.in_tok[i] : 0;
    y[r] = in ? a.out_tok[i] : 0;
    md[r] = (in && a.model) ? a.model[i] : 0;
  }
  const int64_t G = (int64_t)a.n_model * a.n_in_bin * a.n_out_bin;
  uint32_t bad = 0;
  bool dis = false;
#pragma unroll
  for (int r = 0; r < kKeyRows; ++r) {
    const int64_t i = base + r * 256;
    const bool in = i < a.n_req;                       // the lanes that are in are a prefix of the wave: lane - 1 is among them
    uint32_t bad_r = 0;
    const double wq = window_of(t[r], a.window_s, r_window, a.n_window, &bad_r);
    int32_t mdl = md[r];
    if (mdl < 0 || mdl >= a.n_model) { bad_r = DYN_WS_BAD_REQUEST; mdl = 0; }
    const int32_t* ie = in_edge + (size_t)mdl * n_ie;
    const int32_t* oe = out_edge + (size_t)mdl * n_oe;
    int bi = 0, bo = 0;
    for (int e = 0; e < n_ie; ++e) bi += (x[r] >= ie[e]) ? 1 : 0;
    for (int e = 0; e < n_oe; ++e) bo += (y[r] >= oe[e]) ? 1 : 0;
    const int64_t g = ((int64_t)mdl * a.n_in_bin + bi) * a.n_out_bin + bo;
    // Window order: compare with the request before (the neighbouring lane; the first lane of a wave recomputes it).
    // Where the window changes the boundaries are written: in a trace in window order win_off[w] = number of
    // requests in windows before w (the values are not used otherwise).
    double wp = __shfl_up(wq, 1, DYN_WAVE);
    if (lane == 0) {
      uint32_t ignore = 0;
      wp = window_of(tp[r], a.window_s, r_window, a.n_window, &ignore);
    }
    if (i == 0) wp = -1.0;
    // The boundaries only matter to the window route: a wave that sees a request out of order, or finds the flag
    // raised already, writes none (on a shuffled trace every request would otherwise fill hundreds of them).
    const bool back = in && wp > wq;
    const bool fill = __ballot(back) == 0 && __hip_atomic_load(a.unsorted, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0u;
    if (in) {
      a.key_a[i] = (uint32_t)((int64_t)wq * G + g);
      bad |= bad_r;
      dis = dis || back;
      if (fill) {
        for (int64_t w = (int64_t)wp + 1; w <= (int64_t)wq; ++w) a.win_off[w] = i;
        if (i == a.n_req - 1)
          for (int64_t w = (int64_t)wq + 1; w <= a.n_window; ++w) a.win_off[w] = a.n_req;
      }
    }
  }
  if (bad) atomicOr(a.status, bad);
  const uint64_t any = __ballot(dis);
  if (any && lane == __builtin_ctzll(any) && __hip_atomic_load(a.unsorted, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0u)
    atomicOr(a.unsorted, 1u);
}

// The route is chosen on the device: every kernel of the two routes is launched and the kernels of the route that
// is not taken return at once.  `order` is the flag word the key kernel leaves: 0 = every request's window is at
// or after the window of the request before it (the trace is moved window by window), else the general sort runs.
__device__ __forceinline__ bool sort_route(const uint32_t* order) { return *order != 0u; }

// Class edges from the kernel's arguments into the workspace (a few hundred values at most per launch): the host
// arrays are free when the call returns and nothing waits for the stream.  The first launch also writes the
// workspace header: status 0, the order word (1 when the general sort is forced).
struct EdgePack { int32_t v[DYN_EDGE_PACK]; };
__global__ void edge_store_kernel(EdgePack p, int n_a, int32_t* __restrict__ dst_a, int n_b, int32_t* __restrict__ dst_b,
                                  WsHeader* header, uint32_t order_word) {
  for (int i = threadIdx.x; i < n_a; i += blockDim.x) dst_a[i] = p.v[i];
  for (int i = threadIdx.x; i < n_b; i += blockDim.x) dst_b[i] = p.v[n_a + i];
  if (header && threadIdx.x == 0) {
    header->status = 0u;
    header->kind = DYN_WS_KIND_WORD;
    header->cells = 0;
    ((uint32_t*)header)[DYN_WS_HEADER_ORDER_WORD] = order_word;
    ((uint32_t*)header)[DYN_WS_HEADER_BARRIER_WORD] = 0u;
  }
}

// digit counts of one tile -> block_hist[digit * n_block + tile]; `cnt` is DYN_INGEST_MAX_BINS words of LDS
__device__ __forceinline__ void hist_tile(int64_t tile, const uint32_t* keys, int64_t n, int shift, int bits,
                                          uint32_t* block_hist, int64_t n_block, uint32_t* cnt) {
  const int nbins = 1 << bits;
  const uint32_t mask = (uint32_t)nbins - 1u;
  for (int b = threadIdx.x; b < nbins; b += blockDim.x) cnt[b] = 0;
  __syncthreads();
  const int64_t base = tile * kTile;
  for (int r = 0; r < kTile / (kWaves * DYN_WAVE); ++r) {
    const int64_t idx = base + (int64_t)r * (kWaves * DYN_WAVE) + threadIdx.x;
    if (idx < n) atomicAdd(&cnt[(keys[idx] >> shift) & mask], 1u);
  }
  __syncthreads();
  for (int b = threadIdx.x; b < nbins; b += blockDim.x) block_hist[(size_t)b * n_block + tile] = cnt[b];
}

__global__ __launch_bounds__(kWaves* DYN_WAVE) void hist_kernel(const uint32_t* __restrict__ keys, int64_t n,
                                                                int shift, int bits, uint32_t* __restrict__ block_hist,
                                                                int64_t n_block, const uint32_t* __restrict__ order) {
  if (!sort_route(order)) return;
  __shared__ uint32_t cnt[DYN_INGEST_MAX_BINS];
  hist_tile(blockIdx.x, keys, n, shift, bits, block_hist, n_block, cnt);
}

// ---- exclusive scan of `count` uint32 counters in three small kernels --------------------
__device__ __forceinline__ uint32_t block_exclusive_scan_256(uint32_t v, uint32_t* total, uint32_t* s_wave) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  uint32_t incl = v;
#pragma unroll
  for (int d = 1; d < DYN_WAVE; d <<= 1) {
    const uint32_t up = __shfl_up(incl, d, DYN_WAVE);
    if (lane >= d) incl += up;
  }
  if (lane == 63) s_wave[wave] = incl;
  __syncthreads();
  uint32_t off = 0, tot = 0;
  for (int w = 0; w < 4; ++w) {
    if (w < wave) off += s_wave[w];
    tot += s_wave[w];
  }
  __syncthreads();
  *total = tot;
  return off + incl - v;
}

__device__ __forceinline__ void scan_reduce_chunk(int64_t chunk, const uint32_t* x, int64_t count, uint32_t* partial, uint32_t* s_wave) {
  const int64_t base = chunk * kScanChunk;
  uint32_t v = 0;
  for (int q = 0; q < kScanChunk / 256; ++q) {
    const int64_t i = base + q * 256 + threadIdx.x;
    if (i < count) v += x[i];
  }
  uint32_t tot;
  block_exclusive_scan_256(v, &tot, s_wave);
  if (threadIdx.x == 0) partial[chunk] = tot;
}

__device__ __forceinline__ void scan_partials_all(uint32_t* partial, int64_t n_partial, uint32_t* s_wave) {
  uint32_t carry = 0;
  for (int64_t base = 0; base < n_partial; base += 256) {
    const int64_t i = base + threadIdx.x;
    const uint32_t v = i < n_partial ? partial[i] : 0u;
    uint32_t tot;
    const uint32_t ex = block_exclusive_scan_256(v, &tot, s_wave);
    if (i < n_partial) partial[i] = carry + ex;
    carry += tot;
  }
}

__device__ __forceinline__ void scan_apply_chunk(int64_t chunk, uint32_t* x, int64_t count, const uint32_t* partial, uint32_t* s_wave) {
  // thread t owns 16 consecutive counters of the chunk
  constexpr int per = kScanChunk / 256;
  const int64_t base = chunk * kScanChunk + (int64_t)threadIdx.x * per;
  uint32_t v[per], sum = 0;
#pragma unroll
  for (int q = 0; q < per; ++q) {
    v[q] = (base + q < count) ? x[base + q] : 0u;
    sum += v[q];
  }
  uint32_t tot;
  uint32_t run = partial[chunk] + block_exclusive_scan_256(sum, &tot, s_wave);
#pragma unroll
  for (int q = 0; q < per; ++q) {
    if (base + q < count) x[base + q] = run;
    run += v[q];
  }
}

__global__ __launch_bounds__(256) void scan_reduce_kernel(const uint32_t* __restrict__ x, int64_t count,
                                                          uint32_t* __restrict__ partial, const uint32_t* __restrict__ order) {
  if (!sort_route(order)) return;
  __shared__ uint32_t s_wave[4];
  scan_reduce_chunk(blockIdx.x, x, count, partial, s_wave);
}

__global__ __launch_bounds__(256) void scan_partials_kernel(uint32_t* __restrict__ partial, int64_t n_partial, const uint32_t* __restrict__ order) {
  if (!sort_route(order)) return;
  __shared__ uint32_t s_wave[4];
  scan_partials_all(partial, n_partial, s_wave);
}

__global__ __launch_bounds__(256) void scan_apply_kernel(uint32_t* __restrict__ x, int64_t count,
                                                         const uint32_t* __restrict__ partial, const uint32_t* __restrict__ order) {
  if (!sort_route(order)) return;
  __shared__ uint32_t s_wave[4];
  scan_apply_chunk(blockIdx.x, x, count, partial, s_wave);
}

// ---- stable scatter of one radix pass -----------------------------------------------------
__device__ __forceinline__ void scatter_tile(int64_t tile, const uint32_t* keys_in, const int32_t* in_in, const int32_t* out_in,
                                             uint32_t* keys_out, int32_t* in_out, int32_t* out_out, int64_t n, int shift, int bits,
                                             const uint32_t* scanned, int64_t n_block, uint32_t (*wcnt)[DYN_INGEST_MAX_BINS]) {
  const int nbins = 1 << bits;
  const uint32_t mask = (uint32_t)nbins - 1u;
  const int lane = threadIdx.x & (DYN_WAVE - 1);
  const int wave = threadIdx.x / DYN_WAVE;
  for (int b = threadIdx.x; b < kWaves * DYN_INGEST_MAX_BINS; b += blockDim.x) (&wcnt[0][0])[b] = 0;
  __syncthreads();

  // phase 1: digit counts of each wave's run of rows
  const int64_t wbase = tile * kTile + (int64_t)wave * (kRows * DYN_WAVE);
  uint32_t key[kRows];
  int32_t vin[kRows], vout[kRows];                       // the payload, loaded with the keys: not one row at a time later
#pragma unroll
  for (int r = 0; r < kRows; ++r) {
    const int64_t idx = wbase + r * DYN_WAVE + lane;
    key[r] = idx < n ? keys_in[idx] : 0u;
    vin[r] = idx < n ? in_in[idx] : 0;
    vout[r] = idx < n ? out_in[idx] : 0;
    if (idx < n) atomicAdd(&wcnt[wave][(key[r] >> shift) & mask], 1u);
  }
  __syncthreads();
  // phase 2: per digit, the first output position of each wave's requests
  for (int d = threadIdx.x; d < nbins; d += blockDim.x) {
    uint32_t run = scanned[(size_t)d * n_block + tile];
    for (int w = 0; w < kWaves; ++w) {
      const uint32_t c = wcnt[w][d];
      wcnt[w][d] = run;
      run += c;
    }
  }
  __syncthreads();
  // phase 3: rows in order; inside a row, rank among the lanes with the same digit
  uint32_t* my = wcnt[wave];
#pragma unroll
  for (int r = 0; r < kRows; ++r) {
    const int64_t idx = wbase + r * DYN_WAVE + lane;
    const bool valid = idx < n;
    if (__ballot(valid) == 0) break;                     // wave-uniform: nothing left in this run
    const uint32_t d = (key[r] >> shift) & mask;
    uint64_t peers = __ballot(valid);
    for (int b = 0; b < bits; ++b) {
      const bool bit = (d >> b) & 1u;
      const uint64_t bal = __ballot(bit);
      peers &= bit ? bal : ~bal;
    }
    const int before = __popcll(peers & ((1ull << lane) - 1ull));
    const int group = __popcll(peers);
    uint32_t pos = 0;
    if (valid) pos = my[d] + (uint32_t)before;
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    if (valid && before == group - 1) my[d] += (uint32_t)group;   // one lane per digit advances it
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    if (valid) {
      if (keys_out) keys_out[pos] = key[r];
      in_out[pos] = vin[r];
      out_out[pos] = vout[r];
    }
  }
}

__global__ __launch_bounds__(kWaves* DYN_WAVE) void scatter_kernel(
    const uint32_t* __restrict__ keys_in, const int32_t* __restrict__ in_in, const int32_t* __restrict__ out_in,
    uint32_t* __restrict__ keys_out, int32_t* __restrict__ in_out, int32_t* __restrict__ out_out, int64_t n,
    int shift, int bits, const uint32_t* __restrict__ scanned, int64_t n_block, const uint32_t* __restrict__ order) {
  if (!sort_route(order)) return;
  __shared__ uint32_t wcnt[kWaves][DYN_INGEST_MAX_BINS];
  scatter_tile(blockIdx.x, keys_in, in_in, out_in, keys_out, in_out, out_out, n, shift, bits, scanned, n_block, wcnt);
}

// cell_off[c] = number of requests with key < c, read off the sorted keys
__device__ __forceinline__ void offsets_at(int64_t i, const uint32_t* keys, int64_t n, int64_t cells, int64_t* cell_off) {
  if (i > n) return;
  const int64_t prev = i == 0 ? -1 : (int64_t)keys[i - 1];
  int64_t cur = i == n ? cells : (int64_t)keys[i];
  if (cur > cells) cur = cells;
  for (int64_t c = prev + 1; c <= cur; ++c) cell_off[c] = i;
}

__global__ __launch_bounds__(256) void offsets_kernel(const uint32_t* __restrict__ keys, int64_t n, int64_t cells,
                                                      int64_t* __restrict__ cell_off, const uint32_t* __restrict__ order) {
  if (!sort_route(order)) return;
  offsets_at((int64_t)blockIdx.x * blockDim.x + threadIdx.x, keys, n, cells, cell_off);
}

// The whole general sort in one launch: a grid that the device holds at once walks the tiles of every phase, with a
// grid-wide barrier between the phases.  A trace in window order costs this one launch that returns at its first
// instruction (eleven gated launches otherwise).  The barrier: an arrival counter in the workspace header, zeroed with
// the header; barrier number k is passed when the counter reaches k * blocks.  The grid is a fraction of what the
// device holds at once (occupancy query), so every block is running when the first one waits; if other work keeps
// part of the device for seconds the wait is given up (every block leaves, DYN_WS_SORT_ABANDONED is raised).
// A barrier costs a write-back of the block's cache level per block, which is why the grid is kept small.
struct RadixArgs {
  const uint32_t* order;
  uint32_t* barrier; uint32_t* status;
  uint32_t* key_a; uint32_t* key_b;
  const int32_t* in_tok; const int32_t* out_tok;
  int32_t* in_sorted; int32_t* out_sorted; int32_t* in_tmp; int32_t* out_tmp;
  uint32_t* block_hist; int64_t n_block;
  int64_t n, cells; int64_t* cell_off;
  int32_t passes, bits;
};

constexpr int kRadixGridShare = 4;               // the grid is this fraction of what the device holds at once
constexpr uint32_t kBarrierSpins = 1u << 22;     // x about a microsecond per look: seconds

// false: given up (block-uniform).  All writes of the block before the call are visible to every block after it.
// The waiting thread looks at the counter with relaxed loads (acquiring loads would invalidate caches all over the
// device for as long as anyone waits) and acquires once at the end.
__device__ __forceinline__ bool grid_barrier(uint32_t* counter, uint32_t target, uint32_t* s_flag) {
  __syncthreads();                                // the block's stores have been issued and acknowledged
  if (threadIdx.x == 0) {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
    __hip_atomic_fetch_add(counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    uint32_t spins = 0;
    bool ok = true;
    while (__hip_atomic_load(counter, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target) {
      if (++spins > kBarrierSpins) { ok = false; break; }
      __builtin_amdgcn_s_sleep(20);
    }
    *s_flag = ok ? 1u : 0u;
  }
  __syncthreads();
  const bool ok = *s_flag != 0u;
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");   // later reads see the other blocks' writes
  return ok;
}

__global__ __launch_bounds__(kWaves* DYN_WAVE) __attribute__((amdgpu_waves_per_eu(4, 4))) void radix_route_kernel(RadixArgs a) {
  if (!sort_route(a.order)) return;              // the same word for every block: all leave, or none
  __shared__ uint32_t wcnt[kWaves][DYN_INGEST_MAX_BINS];
  __shared__ uint32_t s_wave[4];
  __shared__ uint32_t s_flag;
  uint32_t passed = 0;                           // barriers behind this block
  auto sync = [&]() {
    ++passed;
    return grid_barrier(a.barrier, passed * gridDim.x, &s_flag);
  };
  auto give_up = [&]() {
    if (threadIdx.x == 0) atomicOr(a.status, DYN_WS_SORT_ABANDONED);
  };
  const uint32_t* k_src = a.key_a;
  uint32_t* k_dst = a.key_b;
  const int32_t *i_src = a.in_tok, *o_src = a.out_tok;
  const uint32_t* sorted_keys = a.key_a;
  uint32_t* partial = a.block_hist + (size_t)DYN_INGEST_MAX_BINS * a.n_block;
  for (int p = 0; p < a.passes; ++p) {
    const bool to_final = ((a.passes - 1 - p) % 2) == 0;   // ping-pong so that the last pass lands in the caller's arrays
    int32_t* i_dst = to_final ? a.in_sorted : a.in_tmp;
    int32_t* o_dst = to_final ? a.out_sorted : a.out_tmp;
    const int shift = p * a.bits;
    const int64_t count = (int64_t)(1 << a.bits) * a.n_block;
    const int64_t n_part = (count + kScanChunk - 1) / kScanChunk;
    for (int64_t t = blockIdx.x; t < a.n_block; t += gridDim.x) {
      hist_tile(t, k_src, a.n, shift, a.bits, a.block_hist, a.n_block, wcnt[0]);
      __syncthreads();
    }
    if (!sync()) { give_up(); return; }
    for (int64_t c = blockIdx.x; c < n_part; c += gridDim.x) scan_reduce_chunk(c, a.block_hist, count, partial, s_wave);
    if (!sync()) { give_up(); return; }
    if (blockIdx.x == 0) scan_partials_all(partial, n_part, s_wave);
    if (!sync()) { give_up(); return; }
    for (int64_t c = blockIdx.x; c < n_part; c += gridDim.x) scan_apply_chunk(c, a.block_hist, count, partial, s_wave);
    if (!sync()) { give_up(); return; }
    for (int64_t t = blockIdx.x; t < a.n_block; t += gridDim.x) {
      scatter_tile(t, k_src, i_src, o_src, k_dst, i_dst, o_dst, a.n, shift, a.bits, a.block_hist, a.n_block, wcnt);
      __syncthreads();
    }
    if (!sync()) { give_up(); return; }
    sorted_keys = k_dst;
    i_src = i_dst;
    o_src = o_dst;
    uint32_t* old_src = const_cast<uint32_t*>(k_src);
    k_src = k_dst;
    k_dst = old_src;
  }
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i <= a.n; i += (int64_t)gridDim.x * blockDim.x)
    offsets_at(i, sorted_keys, a.n, a.cells, a.cell_off);
}

// ---- a trace in window order ----------------------------------------------------------------
// win_off[w] = number of requests in windows before w, read off the keys (window = key / G)
__global__ __launch_bounds__(256) void window_offsets_kernel(const uint32_t* __restrict__ keys, int64_t n, uint32_t G,
                                                             int32_t n_window, int64_t* __restrict__ win_off) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i > n) return;
  const int64_t prev = i == 0 ? -1 : (int64_t)(keys[i - 1] / G);
  int64_t cur = i == n ? n_window : (int64_t)(keys[i] / G);
  if (cur > n_window) cur = n_window;
  for (int64_t w = prev + 1; w <= cur; ++w) win_off[w] = i;
}

// One block per window: class totals of the window, their exclusive prefix (the window's cell offsets),
// then a stable move tile by tile: every wave owns a contiguous run of rows of a tile and walks them in
// order, a request's position = start of its class + requests of the class in earlier tiles and earlier
// waves' runs + its rank among the lanes of its row with the same class (wave ballots).
__global__ __launch_bounds__(kWaves* DYN_WAVE) void window_sort_kernel(
    const uint32_t* __restrict__ keys, const int32_t* __restrict__ in_in, const int32_t* __restrict__ out_in,
    int32_t* __restrict__ in_out, int32_t* __restrict__ out_out, const int64_t* __restrict__ win_off, int32_t G,
    int32_t n_window, int64_t n, int64_t* __restrict__ cell_off, const uint32_t* __restrict__ order) {
  if (sort_route(order)) return;
  __shared__ uint32_t wcnt[kWaves][DYN_INGEST_MAX_BINS];
  __shared__ uint32_t run[DYN_INGEST_MAX_BINS];          // next output position of every class, relative to the window's start
  const int w = blockIdx.x;
  const int lane = threadIdx.x & (DYN_WAVE - 1), wave = threadIdx.x / DYN_WAVE;
  const int64_t beg = win_off[w], end = win_off[w + 1];
  const uint32_t key0 = (uint32_t)w * (uint32_t)G;
  int bits = 0;
  while ((1 << bits) < G) ++bits;
  for (int d = threadIdx.x; d < G; d += blockDim.x) run[d] = 0;
  __syncthreads();
  {                                                      // class totals of the window, four loads per thread in flight
    int64_t i = beg + threadIdx.x;
    for (; i + 3 * (int64_t)blockDim.x < end; i += 4 * (int64_t)blockDim.x) {
      const uint32_t k0 = keys[i], k1 = keys[i + blockDim.x], k2 = keys[i + 2 * blockDim.x], k3 = keys[i + 3 * blockDim.x];
      atomicAdd(&run[k0 - key0], 1u); atomicAdd(&run[k1 - key0], 1u); atomicAdd(&run[k2 - key0], 1u); atomicAdd(&run[k3 - key0], 1u);
    }
    for (; i < end; i += blockDim.x) atomicAdd(&run[keys[i] - key0], 1u);
  }
  __syncthreads();
  if (threadIdx.x == 0) {                                // exclusive prefix over the classes
    uint32_t acc = 0;
    for (int d = 0; d < G; ++d) {
      const uint32_t c = run[d];
      run[d] = acc;
      acc += c;
    }
  }
  __syncthreads();
  for (int d = threadIdx.x; d < G; d += blockDim.x) cell_off[(int64_t)w * G + d] = beg + run[d];
  if (w == n_window - 1 && threadIdx.x == 0) cell_off[(int64_t)n_window * G] = n;

  for (int64_t tile = beg; tile < end; tile += kTile) {
    for (int b = threadIdx.x; b < kWaves * G; b += blockDim.x) wcnt[b / G][b % G] = 0;
    __syncthreads();
    // phase 1: class counts of each wave's run of rows
    const int64_t wbase = tile + (int64_t)wave * (kRows * DYN_WAVE);
    uint32_t cls[kRows];
    int32_t vin[kRows], vout[kRows];                     // the payload, loaded with the keys: not one row at a time later
#pragma unroll
    for (int r = 0; r < kRows; ++r) {
      const int64_t idx = wbase + r * DYN_WAVE + lane;
      cls[r] = idx < end ? keys[idx] - key0 : 0u;
      vin[r] = idx < end ? in_in[idx] : 0;
      vout[r] = idx < end ? out_in[idx] : 0;
      if (idx < end) atomicAdd(&wcnt[wave][cls[r]], 1u);
    }
    __syncthreads();
    // phase 2: per class, the first output position of each wave's requests
    for (int d = threadIdx.x; d < G; d += blockDim.x) {
      uint32_t pos = run[d];
      for (int q = 0; q < kWaves; ++q) {
        const uint32_t c = wcnt[q][d];
        wcnt[q][d] = pos;
        pos += c;
      }
      run[d] = pos;
    }
    __syncthreads();
    // phase 3: rows in order; inside a row, rank among the lanes with the same class
    uint32_t* my = wcnt[wave];
#pragma unroll
    for (int r = 0; r < kRows; ++r) {
      const int64_t idx = wbase + r * DYN_WAVE + lane;
      const bool valid = idx < end;
      if (__ballot(valid) == 0) break;                   // wave-uniform: nothing left in this run
      const uint32_t d = cls[r];
      uint64_t peers = __ballot(valid);
      for (int b = 0; b < bits; ++b) {
        const bool bit = (d >> b) & 1u;
        const uint64_t bal = __ballot(bit);
        peers &= bit ? bal : ~bal;
      }
      const int before = __popcll(peers & ((1ull << lane) - 1ull));
      const int group = __popcll(peers);
      uint32_t pos = 0;
      if (valid) pos = my[d] + (uint32_t)before;
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
      __builtin_amdgcn_wave_barrier();
      if (valid && before == group - 1) my[d] += (uint32_t)group;   // one lane per class advances it
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
      __builtin_amdgcn_wave_barrier();
      if (valid) {
        in_out[beg + pos] = vin[r];
        out_out[beg + pos] = vout[r];
      }
    }
    __syncthreads();
  }
}

}  // namespace

int64_t dyn_ingest_blocks(int64_t n_req) { return n_req > 0 ? (n_req + kTile - 1) / kTile : 1; }

hipError_t dyn_launch_edges(const int32_t* in_edge, size_t n_in, const int32_t* out_edge, size_t n_out, int32_t* d_in,
                            int32_t* d_out, WsHeader* header, uint32_t order_word, hipStream_t s) {
  EdgePack p;
  if (n_in + n_out <= DYN_EDGE_PACK) {          // the usual case: header and both lists in one launch
    if (n_in) memcpy(p.v, in_edge, n_in * sizeof(int32_t));
    if (n_out) memcpy(p.v + n_in, out_edge, n_out * sizeof(int32_t));
    hipLaunchKernelGGL(edge_store_kernel, dim3(1), dim3(256), 0, s, p, (int)n_in, d_in, (int)n_out, d_out, header, order_word);
    return hipGetLastError();
  }
  hipLaunchKernelGGL(edge_store_kernel, dim3(1), dim3(64), 0, s, p, 0, d_in, 0, d_out, header, order_word);
  const struct { const int32_t* src; size_t n; int32_t* dst; } parts[2] = {{in_edge, n_in, d_in}, {out_edge, n_out, d_out}};
  for (const auto& part : parts)
    for (size_t at = 0; at < part.n; at += DYN_EDGE_PACK) {
      const int n = (int)std::min<size_t>(DYN_EDGE_PACK, part.n - at);
      memcpy(p.v, part.src + at, (size_t)n * sizeof(int32_t));
      hipLaunchKernelGGL(edge_store_kernel, dim3(1), dim3(256), 0, s, p, n, part.dst + at, 0, part.dst, (WsHeader*)nullptr, 0u);
    }
  return hipGetLastError();
}

hipError_t dyn_launch_ingest(const IngestArgs& a, hipStream_t s) {
  const int64_t n = a.n_req;
  const int32_t G = a.n_model * a.n_in_bin * a.n_out_bin;
  const int64_t cells = (int64_t)a.n_window * G;
  hipError_t e;
  // Keys, and whether the trace is in window order already: the key kernel ORs into the flag word, which the header
  // kernel before it set to 0, or to 1 when the general sort is forced (more classes than the window route counts).
  if (n > 0) {
    const size_t edge_bytes = (size_t)a.n_model * ((a.n_in_bin - 1) + (a.n_out_bin - 1)) * sizeof(int32_t);
    const int lds_edges = edge_bytes <= 32 * 1024 ? 1 : 0;
    hipLaunchKernelGGL(key_kernel, dim3((unsigned)((n + kKeyRows * 256 - 1) / (kKeyRows * 256))), dim3(256), lds_edges ? edge_bytes : 0, s, a,
                       1.0 / a.window_s, lds_edges);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  } else {
    hipLaunchKernelGGL(window_offsets_kernel, dim3(1), dim3(256), 0, s, a.key_a, n, (uint32_t)G, a.n_window, a.win_off);
  }
  if (!a.force_sort) {        // in window order: one block per window moves its requests to their cells
    hipLaunchKernelGGL(window_sort_kernel, dim3((unsigned)a.n_window), dim3(kWaves * DYN_WAVE), 0, s, a.key_a, a.in_tok,
                       a.out_tok, a.in_sorted, a.out_sorted, a.win_off, G, a.n_window, n, a.cell_off, a.unsorted);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    if (n == 0) return hipSuccess;   // nothing to sort: the flag word stays 0
  }
  const int passes = a.key_bits <= 0 ? 1 : (a.key_bits + 9) / 10;
  const int bits = a.key_bits <= 0 ? 1 : (a.key_bits + passes - 1) / passes;
  {
    // one launch of a resident grid when the device tells what it holds; else the launches below
    // what the device holds at once, asked once per device (0: not asked yet, -1: unknown: the separate kernels below)
    static std::atomic<int> resident[64];
    int dev = 0;
    int fit = 0;
    if (hipGetDevice(&dev) == hipSuccess && dev >= 0 && dev < 64) {
      fit = resident[dev].load(std::memory_order_relaxed);
      if (fit == 0) {
        int n_cu = 0, per_cu = 0;
        fit = -1;
        if (hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess &&
            hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, radix_route_kernel, kWaves * DYN_WAVE, 0) == hipSuccess && per_cu > 0)
          fit = std::max(1, per_cu * n_cu / kRadixGridShare);
        (void)hipGetLastError();
        resident[dev].store(fit, std::memory_order_relaxed);
      }
    }
    if (fit > 0) {
      RadixArgs r;
      r.order = a.unsorted; r.barrier = a.unsorted + (DYN_WS_HEADER_BARRIER_WORD - DYN_WS_HEADER_ORDER_WORD); r.status = a.status;
      r.key_a = a.key_a; r.key_b = a.key_b; r.in_tok = a.in_tok; r.out_tok = a.out_tok;
      r.in_sorted = a.in_sorted; r.out_sorted = a.out_sorted; r.in_tmp = a.in_tmp; r.out_tmp = a.out_tmp;
      r.block_hist = a.block_hist; r.n_block = a.n_block; r.n = n; r.cells = cells; r.cell_off = a.cell_off;
      r.passes = passes; r.bits = bits;
      const int64_t useful = std::max<int64_t>(a.n_block, 1);
      const unsigned blocks = (unsigned)std::min<int64_t>((int64_t)fit, useful);
      hipLaunchKernelGGL(radix_route_kernel, dim3(blocks), dim3(kWaves * DYN_WAVE), 0, s, r);
      return hipGetLastError();
    }
  }
  // ping-pong so that the last pass lands in the caller's arrays
  const uint32_t* k_src = a.key_a;
  uint32_t* k_dst = a.key_b;
  const int32_t *i_src = a.in_tok, *o_src = a.out_tok;
  const uint32_t* sorted_keys = a.key_a;
  for (int p = 0; p < passes; ++p) {
    const bool to_final = ((passes - 1 - p) % 2) == 0;
    int32_t* i_dst = to_final ? a.in_sorted : a.in_tmp;
    int32_t* o_dst = to_final ? a.out_sorted : a.out_tmp;
    const int shift = p * bits;
    const int64_t count = (int64_t)(1 << bits) * a.n_block;
    const int64_t n_part = (count + kScanChunk - 1) / kScanChunk;
    uint32_t* partial = a.block_hist + (size_t)DYN_INGEST_MAX_BINS * a.n_block;
    hipLaunchKernelGGL(hist_kernel, dim3((unsigned)a.n_block), dim3(kWaves * DYN_WAVE), 0, s, k_src, n, shift,
                       bits, a.block_hist, a.n_block, a.unsorted);
    hipLaunchKernelGGL(scan_reduce_kernel, dim3((unsigned)n_part), dim3(256), 0, s, a.block_hist, count, partial, a.unsorted);
    hipLaunchKernelGGL(scan_partials_kernel, dim3(1), dim3(256), 0, s, partial, n_part, a.unsorted);
    hipLaunchKernelGGL(scan_apply_kernel, dim3((unsigned)n_part), dim3(256), 0, s, a.block_hist, count, partial, a.unsorted);
    hipLaunchKernelGGL(scatter_kernel, dim3((unsigned)a.n_block), dim3(kWaves * DYN_WAVE), 0, s, k_src, i_src,
                       o_src, k_dst, i_dst, o_dst, n, shift, bits, a.block_hist, a.n_block, a.unsorted);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    sorted_keys = k_dst;
    i_src = i_dst;
    o_src = o_dst;
    uint32_t* old_src = const_cast<uint32_t*>(k_src);   // both key buffers live in the workspace
    k_src = k_dst;
    k_dst = old_src;
  }
  hipLaunchKernelGGL(offsets_kernel, dim3((unsigned)((n + 1 + 255) / 256)), dim3(256), 0, s, sorted_keys, n, cells,
                     a.cell_off, a.unsorted);
  return hipGetLastError();
}
