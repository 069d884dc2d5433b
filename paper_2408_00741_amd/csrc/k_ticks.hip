// Tick-level load inside a window: every window is split into n_tick ticks (sub-windows of
// the sorted trace), each request is served under the load of its own tick (the instance
// manager re-tunes the frequency every few seconds under the current load, Section IV-B
// "Scale-up/down").  Per (window, class) cell and candidate configuration the profile is
// looked up once per tick; the window's energy is the sum over its ticks.
//
// The per-request percentile still collapses, tick by tick: inside one tick TTFT is
// input length x a non-negative constant, so the cell's j-th largest TTFT (j = m - rank + 1)
// is among the j largest input lengths of each tick scaled by that tick's prefill time.
// The request stream is read once, independent of the configurations:
//   tick_cell_kernel   per cell every tick's load, its min(j, count) largest input lengths in
//                      descending order (j <= 64: kept sorted in a wave's lanes) and the cell's
//                      j-th largest input length x_j; what the later kernels do with the cell;
//   tick_deep_kernel   the same lists and x_j for the cells with j > 64 (a block per cell:
//                      bitonic sort of a tick in LDS); beyond j = 8192 the lists are whole ticks, and a
//                      tick of more than 8192 requests is then sorted in pieces of 8192 (marked: the
//                      general kernel searches every piece);
//   tick_space_kernel  the cells with j <= 16: per (cell, configuration) a walk over the ticks, energy in time
//                      order, the TBT percentile (largest tick TBT when every non-empty tick holds j
//                      requests, else from the four largest tick TBTs), the TTFT percentile through a
//                      sorted register list of the scaled candidates;
//   tick_general_kernel every other cell, (cell, tile) by (cell, tile): the ticks' prefill times (TBTs)
//                      kept in an LDS strip, the TBT percentile by taking ticks in descending TBT
//                      order, the TTFT percentile from the bracket [x_j * least, x_j * largest prefill
//                      time of the ticks]: a single value, or settled by ranking the ticks that hold
//                      lengths equal to x_j, or bisected on the ticks' sorted lists.
#include <algorithm>
#include <type_traits>

#include "dyn_ticks.h"
#include "dyn_device.h"

namespace {

constexpr int kWavesPerBlock = 4;
constexpr int kFastDepth = DYN_TICK_FAST;
constexpr int kDeepCap = DYN_TICK_DEPTH;     // largest j, and the largest tick the deep-cell kernel sorts in one go
constexpr int kDeepBlocks = 512;
constexpr int kGeneralBlocks = 1024;          // grid of the general kernel when the device cannot be asked what fits
constexpr int kListCap = 2048;               // list entries of one cell the general kernel stages in LDS
constexpr int kStripBytes = 32 * 1024;       // per-tick values of a block's configurations in the general kernel
static_assert(kDeepCap == 8192, "the deep-cell kernel's LDS buffer");
// LDS stride of a staged table row in doubles: odd, so that lanes reading the same load bracket of
// different rows do not all fall into one bank
#define DYN_SLOT_STRIDE(n_rho) ((3 * (n_rho)) | 1)

__global__ void tick_init_kernel(uint32_t* counters) {
  counters[0] = 0u;
  counters[1] = 0u;
  counters[2] = 0u;
  counters[3] = 0u;
}

// How the TBT percentile of a cell can be found (lane q holds tick q's request count, 0 beyond the ticks): from the
// largest tick TBT when every non-empty tick holds j requests (DENSE); from the four largest tick TBTs when any four
// non-empty ticks hold j between them: the four smallest counts do, or there are no more than four (SMALL).
__device__ __forceinline__ uint32_t tbt_route(int32_t cnt_l, int64_t j64, int lane) {
  uint32_t flags = 0;
  uint32_t cpos = cnt_l > 0 ? (uint32_t)cnt_l : 0xFFFFFFFFu;
  if ((int64_t)wave_min_u32(cpos) >= j64) flags |= DYN_TP_DENSE;
  int64_t s4 = 0;
  bool all_in = false;
  for (int r = 0; r < 4; ++r) {
    const uint32_t mn = wave_min_u32(cpos);
    if (mn == 0xFFFFFFFFu) { all_in = true; break; }
    s4 += mn;
    const uint64_t who = __ballot(cpos == mn);
    if (lane == (int)__builtin_ctzll(who)) cpos = 0xFFFFFFFFu;
  }
  if (all_in || s4 >= j64) flags |= DYN_TP_SMALL;
  return flags;
}

// ---- cells settled by their ties at x_j ----------------------------------------------------------
// With theta_g = the least ratio (smallest / largest prefill time of a table row) over the rows of class g, every
// configuration of the class has per-tick prefill times within a factor theta_g of each other.  If theta_g * (x_j + 1) > x_j
// (flat prefill tables: always), a request longer than x_j has a larger TTFT than any request of length x_j, whatever
// their ticks, and a shorter one a smaller TTFT: the cell's j-th largest TTFT belongs to a request of length x_j, and
// it is x_j times the prefill time that ranks (j - number of longer requests) from the top among the ticks, each tick
// counted as often as it holds requests of length x_j.  All the evaluation needs of such a cell is x_j, that rank and
// the per-tick counts.  A wave takes a cell whose ticks fit its registers (rows of 64 requests, the same number of
// rows for every tick, two 16-bit lengths to a register), finds x_j by the bit-wise search of the window-level
// aggregation and counts.  The evaluation keeps four ticks: the rank must be within their reach from the top or from
// the bottom (tight_place), else the cell is ranked over all ticks by the general kernel, like a cell whose TBT
// percentile needs all ticks.  Cells it cannot take (the bound does not hold, ticks too uneven for the registers,
// token counts of 2^16 or more) are listed for the kernel that builds per-tick lists.
struct TightCell {
  uint32_t tok_l;     // lane q: token sum of tick q
  uint32_t eq_l;      // lane q: requests of length x_j in tick q
  uint32_t xj, place; // place: the rank among the ticks, from the top, or from the bottom with DYN_TIGHT_FROM_BELOW set
  uint32_t need;      // the rank from the top
  bool walk;          // the rank is within reach of the walk's four ticks from one end
};
#define DYN_TIGHT_FROM_BELOW 0x80000000u

// The up to four smallest positive per-tick counts of a wave (e_l: lane q holds tick q's count, 0 elsewhere), ascending,
// 0xFFFFFFFF where there are fewer; returns the number of positive counts.  Wave-uniform results.
__device__ __forceinline__ int smallest_four(uint32_t e_l, int lane, uint32_t (&m4)[4]) {
  const int npos = __popcll(__ballot(e_l > 0u));
  uint32_t cur = e_l > 0u ? e_l : 0xFFFFFFFFu;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    m4[i] = wave_min_u32(cur);
    const uint64_t at = __ballot(cur == m4[i] && cur != 0xFFFFFFFFu);
    if (at != 0 && lane == __builtin_ctzll(at)) cur = 0xFFFFFFFFu;   // one lane leaves per round
  }
  return npos;
}

// Where the walk finds the rank `need` (1 .. n_eq) among the ticks weighted by their counts of lengths equal to x_j,
// with its list of four ticks: from the top if the four ticks of largest prefill time are sure to weigh `need`
// together (need <= 4, or at most four ticks have such lengths, or the four smallest positive counts add up to it),
// else from the bottom by the same test on n_eq - need + 1, else not at all (returns false; `place` = need).
__device__ __forceinline__ bool tight_place(int need, int n_eq, int npos, uint32_t s4, uint32_t* place) {
  const int below = n_eq - need + 1;
  *place = (uint32_t)need;
  if (need <= 4 || npos <= 4 || (uint32_t)need <= s4) return true;
  if (below <= 4 || (uint32_t)below <= s4) {
    *place = (uint32_t)below | DYN_TIGHT_FROM_BELOW;
    return true;
  }
  return false;
}

template <int P>   // P registers = 2P rows
__device__ __forceinline__ bool tight_cell(const int32_t* __restrict__ in, const int32_t* __restrict__ out, int64_t beg_l,
                                           int32_t cnt_l, int T, int rpt, int m, int rank, float theta, int lane,
                                           TightCell* res) {
  uint32_t v[P];
  uint32_t orv = 0, lmax = 0, lmax2 = 0, tok_acc = 0, tok_l = 0;
  constexpr int CH = P < 4 ? P : 4;      // registers per round: up to 8 + 8 loads in flight
  int q = 0, r = 0;                      // tick and row of the slot being filled (wave-uniform)
#pragma unroll
  for (int p0 = 0; p0 < P; p0 += CH) {
    uint32_t a[2 * CH], b[2 * CH];
    int qs[2 * CH], rs[2 * CH];
#pragma unroll
    for (int u = 0; u < 2 * CH; ++u) {
      qs[u] = q; rs[u] = r;
      // lane reads without a branch around them: beyond the last tick the lane index is clamped and the count zeroed
      const int qc = q < DYN_WAVE - 1 ? q : DYN_WAVE - 1;
      const int64_t beg_q = readlane_i64(beg_l, qc);
      const int cnt_q = __builtin_amdgcn_readlane(cnt_l, qc);
      const int left = (q < T ? cnt_q : 0) - r * DYN_WAVE;
      const bool ok = lane < left;
      // the padding of a slot without a request goes into its half of the register now; the length is ORed in below
      // (a lane without a request loads 0), so no mask has to live across the loads
      if (u % 2 == 0) v[p0 + u / 2] = ok ? 0u : 0xFFFFu;
      else v[p0 + u / 2] |= ok ? 0u : 0xFFFF0000u;
      const int64_t row_q = beg_q + (int64_t)(r * DYN_WAVE);   // one scalar offset for both arrays
      a[u] = ok ? (uint32_t)in[row_q + lane] : 0u;
      b[u] = ok ? (uint32_t)out[row_q + lane] : 0u;
      if (++r == rpt) { r = 0; ++q; }
    }
#pragma unroll
    for (int u = 0; u < 2 * CH; ++u) {
      tok_acc += a[u] + b[u];
      orv |= a[u] | b[u];
      if (u % 2 == 0) lmax = max(lmax, a[u]); else lmax2 = max(lmax2, a[u]);
      if (rs[u] == rpt - 1) {            // the tick's last row: its token sum goes to lane q (below 2^30 when the cell qualifies)
        const uint32_t tok = wave_sum_u32(tok_acc);
        if (lane == qs[u]) tok_l = tok;
        tok_acc = 0;
      }
    }
#pragma unroll
    for (int u = 0; u < CH; ++u) {
      v[p0 + u] |= (a[2 * u] & 0xFFFFu) | (a[2 * u + 1] << 16);   // lengths of 2^16 and more: the cell is given up below
    }
    // keep the rounds apart: with all loads hoisted to the top 4P loaded values would be live at once
    if (CH == 4)
      asm volatile("" : "+v"(tok_acc), "+v"(tok_l), "+v"(orv), "+v"(lmax), "+v"(lmax2), "+v"(v[p0]), "+v"(v[p0 + 1]),
                   "+v"(v[p0 + 2]), "+v"(v[p0 + 3])::"memory");
  }
  orv = wave_or_u32(orv);
  if (orv >= (1u << 16)) return false;   // wave-uniform
  const uint32_t top = wave_max_u32(max(lmax, lmax2));
  if (top == 0xFFFFu) return false;      // the padding value itself; the search's candidates (up to top + 1) must fit 16 bits
  uint32_t xj = top;
  const int j = m - rank + 1;
  if (rank != m) {
    uint32_t lo = 0;
    if (j <= 2 * DYN_WAVE) {
      const int nb = 32 - __builtin_clz(top | 1u);
      for (int b = nb - 1; b >= 0; --b) {   // largest c with #{the 128 half-lane maxima >= c} >= j (all elements of the cell)
        const uint32_t cand = lo | (1u << b);
        if (__popcll(__ballot(lmax >= cand)) + __popcll(__ballot(lmax2 >= cand)) >= j) lo = cand;
      }
    }
    uint32_t d = 0;
    const int nb = 32 - __builtin_clz((top - lo) | 1u);
    for (int b = nb - 1; b >= 0; --b) {
      const uint32_t cand = lo + (d | (1u << b));
      const uint16_t cand_lo = (uint16_t)cand;   // low half by a 16-bit compare; high half: hi < cand exactly when the
      const uint32_t cand_hi = cand << 16;       // whole register < cand << 16
      int below = 0;
#pragma unroll
      for (int i = 0; i < P; ++i)
        below += __popcll(__ballot((uint16_t)v[i] < cand_lo)) + __popcll(__ballot(v[i] < cand_hi));
      if (below < rank) d |= 1u << b;
    }
    xj = lo + d;
  }
  // the bound: theta * (x_j + 1) > x_j, with theta below the true ratio by 2^-21 at least (so that no rounding of the
  // scaled lengths can turn the order around)
  if (!((double)theta * ((double)xj + 1.0) > (double)xj)) return false;
  // longer requests, and per tick the requests of length x_j.  The padding (0xFFFF in every slot beyond a tick's
  // requests) counts as longer: it is taken off afterwards.
  int n_gt = -(2 * P * DYN_WAVE - m), n_eq = 0, eq_acc = 0;
  uint32_t eq_l = 0;
  q = 0; r = 0;
  const uint32_t xj_hi = xj << 16;
#pragma unroll
  for (int i = 0; i < P; ++i) {
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      // low half by 16-bit compares; high half on the whole register (hi > x_j exactly when v >= (x_j + 1) << 16)
      n_gt += h ? __popcll(__ballot(v[i] >= xj_hi + 0x10000u)) : __popcll(__ballot((uint16_t)v[i] > (uint16_t)xj));
      eq_acc += h ? __popcll(__ballot((v[i] >> 16) == xj)) : __popcll(__ballot((uint16_t)v[i] == (uint16_t)xj));
      if (++r == rpt) {
        if (lane == q) eq_l = (uint32_t)eq_acc;
        n_eq += eq_acc;
        eq_acc = 0;
        r = 0; ++q;
      }
    }
  }
  const int need = j - n_gt;             // 1 .. n_eq
  uint32_t place = (uint32_t)need;       // out of the list's reach from both ends: for the general kernel, from the top
  res->walk = true;
  if (need > 4 && n_eq - need + 1 > 4) {
    uint32_t m4[4];
    const int npos = smallest_four(eq_l, lane, m4);
    const uint32_t s4 = npos >= 4 ? m4[0] + m4[1] + m4[2] + m4[3] : 0u;   // counts stay below 2^24
    res->walk = tight_place(need, n_eq, npos, s4, &place);
  } else if (need > 4) {
    place = (uint32_t)(n_eq - need + 1) | DYN_TIGHT_FROM_BELOW;
  }
  res->need = (uint32_t)need;
  res->tok_l = tok_l;
  res->eq_l = eq_l;
  res->xj = xj;
  res->place = place;
  return true;
}

__global__ __launch_bounds__(kWavesPerBlock* DYN_WAVE) __attribute__((amdgpu_waves_per_eu(6, 8))) void tick_tight_kernel(TickCellArgs a) {
  const int lane = threadIdx.x & (DYN_WAVE - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / DYN_WAVE);
  const int T = a.n_tick, G = a.G;
  const int64_t cells = (int64_t)a.n_window * G;
  const int64_t c = (int64_t)blockIdx.x * kWavesPerBlock + wave;
  if (c >= cells) return;
  if (c == 0 && lane == 0) {                     // single writer of the header
    a.header->status = 0u;
    a.header->kind = DYN_WS_KIND_CELLS;
    a.header->cells = cells * T;
  }
  const int64_t w = c / G;
  const int g = (int)(c % G);
  const int64_t f0 = (w * T) * G + g;           // fine cell of tick 0; tick q is q*G further
  int64_t beg_l = 0;
  int32_t cnt_l = 0;
  uint32_t bad_l = 0;
  if (lane < T) {
    const int64_t f = f0 + (int64_t)lane * G;
    const int64_t b = a.fine_off[f], e = a.fine_off[f + 1];
    if (b < 0 || e < b || e > a.n_req) bad_l = DYN_WS_BAD_OFFSETS;   // such a tick is treated as empty
    else { beg_l = b; cnt_l = (int32_t)(e - b); }
  }
  const int64_t m_cell = (int64_t)wave_sum_u64((uint64_t)(uint32_t)cnt_l);
  const int64_t rank = (a.pct_num * m_cell + a.pct_den - 1) / a.pct_den;
  const int64_t j64 = m_cell > 0 ? m_cell - rank + 1 : 0;
  TightCell tc;
  tc.tok_l = 0; tc.eq_l = 0; tc.xj = 0; tc.place = 0; tc.need = 0; tc.walk = true;
  uint32_t flags = 0;
  bool done = m_cell == 0;                       // an empty cell: loads 0, nothing else
  if (!done) {
    flags = tbt_route(cnt_l, j64, lane);
    const int rpt = ((int)wave_max_u32((uint32_t)cnt_l) + DYN_WAVE - 1) / DYN_WAVE;   // rows per tick
    const int rows = T * rpt;
    // with few cells on the whole device a cell of many rows is quicker with a block's four waves: it goes on the list
    if (rows <= 128 && !(a.few_cells && rows > 8)) {
      const float theta = a.theta[g];
      const int m = (int)m_cell, rk = (int)rank;
      if (rows <= 4) done = tight_cell<2>(a.in, a.out, beg_l, cnt_l, T, rpt, m, rk, theta, lane, &tc);
      else if (rows <= 8) done = tight_cell<4>(a.in, a.out, beg_l, cnt_l, T, rpt, m, rk, theta, lane, &tc);
      else if (rows <= 16) done = tight_cell<8>(a.in, a.out, beg_l, cnt_l, T, rpt, m, rk, theta, lane, &tc);
      else if (rows <= 32) done = tight_cell<16>(a.in, a.out, beg_l, cnt_l, T, rpt, m, rk, theta, lane, &tc);
      else if (rows <= 64) done = tight_cell<32>(a.in, a.out, beg_l, cnt_l, T, rpt, m, rk, theta, lane, &tc);
      else done = tight_cell<64>(a.in, a.out, beg_l, cnt_l, T, rpt, m, rk, theta, lane, &tc);
      if (done) {
        flags |= DYN_TP_TIGHT;
        // the walk keeps four ticks and finds the TBT percentile from the largest tick TBT or the four largest
        if (!tc.walk || !(flags & (DYN_TP_DENSE | DYN_TP_SMALL))) {
          flags |= DYN_TP_GENERAL;
          tc.place = tc.need;
        }
      }
    }
  }
  if (!done) {                                   // the kernel that builds per-tick lists writes everything about this cell
    if (lane == 0) a.list_cells[atomicAdd(&a.counters[2], 1u)] = (uint32_t)c;
    return;
  }
  if (lane < T) {
    TickRec r;
    r.load = div_by((double)tc.tok_l, a.tick_s, a.r_tick);
    r.off = tc.eq_l;                             // no list: the tick's requests of length x_j
    r.cnt = cnt_l;
    a.rec[c * T + lane] = r;
    a.cstat[f0 + (int64_t)lane * G] = (uint8_t)bad_l;   // every fine cell writes its own status byte
  }
  if (lane == 0) {
    TickPlan p;
    p.j = (int32_t)j64;
    p.xj = (int32_t)tc.xj;
    p.flags = flags;
    p.place = tc.place;
    a.plan[c] = p;
    if (flags & DYN_TP_GENERAL) a.slow_list[atomicAdd(&a.counters[1], 1u)] = (uint32_t)c;
  }
}

// The same for the listed cells whose ticks do not fit one wave's registers: a block per cell, wave w takes the ticks
// w, w + 4, ...; x_j by the bit-wise search with the waves' counts added up through LDS (one barrier per bit).  A cell
// it settles is taken off the list (its entry becomes DYN_LIST_DONE).
#define DYN_LIST_DONE 0xFFFFFFFFu
constexpr int kTightBlocks = 1024;

template <int P>   // P registers = 2P rows per wave
__device__ __forceinline__ bool tight_cell_block(const int32_t* __restrict__ in, const int32_t* __restrict__ out,
                                                 int64_t beg_l, int32_t cnt_l, int T, int rpt, int m, int rank, float theta,
                                                 int lane, int wave, uint32_t* s_x /* [2][kWavesPerBlock] */,
                                                 uint32_t* s_m /* [4 * kWavesPerBlock] */, TightCell* res) {
  uint32_t v[P];
  uint32_t orv = 0, vmax = 0, tok_acc = 0, tok_l = 0;
  constexpr int CH = 4;
  int q = wave, r = 0;                   // tick and row of the slot being filled (wave-uniform)
#pragma unroll
  for (int p0 = 0; p0 < P; p0 += CH) {
    uint32_t a[2 * CH], b[2 * CH];
    int qs[2 * CH], rs[2 * CH];
#pragma unroll
    for (int u = 0; u < 2 * CH; ++u) {
      qs[u] = q; rs[u] = r;
      // lane reads without a branch around them: beyond the last tick the lane index is clamped and the count zeroed
      const int qc = q < DYN_WAVE - 1 ? q : DYN_WAVE - 1;
      const int64_t beg_q = readlane_i64(beg_l, qc);
      const int cnt_q = __builtin_amdgcn_readlane(cnt_l, qc);
      const int left = (q < T ? cnt_q : 0) - r * DYN_WAVE;
      const bool ok = lane < left;
      // the padding of a slot without a request goes into its half of the register now; the length is ORed in below
      // (a lane without a request loads 0), so no mask has to live across the loads
      if (u % 2 == 0) v[p0 + u / 2] = ok ? 0u : 0xFFFFu;
      else v[p0 + u / 2] |= ok ? 0u : 0xFFFF0000u;
      const int64_t row_q = beg_q + (int64_t)(r * DYN_WAVE);   // one scalar offset for both arrays
      a[u] = ok ? (uint32_t)in[row_q + lane] : 0u;
      b[u] = ok ? (uint32_t)out[row_q + lane] : 0u;
      if (++r == rpt) { r = 0; q += kWavesPerBlock; }
    }
#pragma unroll
    for (int u = 0; u < 2 * CH; ++u) {
      tok_acc += a[u] + b[u];
      orv |= a[u] | b[u];
      vmax = max(vmax, a[u]);
      if (rs[u] == rpt - 1) {
        const uint32_t tok = wave_sum_u32(tok_acc);
        if (lane == qs[u]) tok_l = tok;
        tok_acc = 0;
      }
    }
#pragma unroll
    for (int u = 0; u < CH; ++u) {
      v[p0 + u] |= (a[2 * u] & 0xFFFFu) | (a[2 * u + 1] << 16);   // lengths of 2^16 and more: the cell is given up below
    }
    asm volatile("" : "+v"(tok_acc), "+v"(tok_l), "+v"(orv), "+v"(vmax), "+v"(v[p0]), "+v"(v[p0 + 1]), "+v"(v[p0 + 2]),
                 "+v"(v[p0 + 3])::"memory");
  }
  // sums over the block: every wave writes its word, a barrier, every wave reads all four (two buffers in turn)
  int turn = 0;
  auto block_or = [&](uint32_t x) {
    if (lane == 0) s_x[turn * kWavesPerBlock + wave] = x;
    __syncthreads();
    uint32_t all = 0;
    for (int w = 0; w < kWavesPerBlock; ++w) all |= s_x[turn * kWavesPerBlock + w];
    turn ^= 1;
    return all;
  };
  auto block_max = [&](uint32_t x) {
    if (lane == 0) s_x[turn * kWavesPerBlock + wave] = x;
    __syncthreads();
    uint32_t all = 0;
    for (int w = 0; w < kWavesPerBlock; ++w) all = max(all, s_x[turn * kWavesPerBlock + w]);
    turn ^= 1;
    return all;
  };
  auto block_sum = [&](uint32_t x) {
    if (lane == 0) s_x[turn * kWavesPerBlock + wave] = x;
    __syncthreads();
    uint32_t all = 0;
    for (int w = 0; w < kWavesPerBlock; ++w) all += s_x[turn * kWavesPerBlock + w];
    turn ^= 1;
    return all;
  };
  const uint32_t all_or = block_or(wave_or_u32(orv));
  const uint32_t top = block_max(wave_max_u32(vmax));
  if (all_or >= (1u << 16) || top == 0xFFFFu) return false;   // block-uniform; 0xFFFF is the padding value
  uint32_t xj = top;
  const int j = m - rank + 1;
  if (rank != m) {
    uint32_t d = 0;
    const int nb = 32 - __builtin_clz(top | 1u);
    for (int b = nb - 1; b >= 0; --b) {
      const uint32_t cand = d | (1u << b);
      const uint16_t cand_lo = (uint16_t)cand;
      const uint32_t cand_hi = cand << 16;
      int below = 0;
#pragma unroll
      for (int i = 0; i < P; ++i)
        below += __popcll(__ballot((uint16_t)v[i] < cand_lo)) + __popcll(__ballot(v[i] < cand_hi));
      if ((int)block_sum((uint32_t)below) < rank) d |= 1u << b;
    }
    xj = d;
  }
  if (!((double)theta * ((double)xj + 1.0) > (double)xj)) return false;
  int n_gt = 0, n_eq = 0, eq_acc = 0;      // the padding (0xFFFF) counts as longer: taken off after the block's sum
  uint32_t eq_l = 0;
  q = wave; r = 0;
  const uint32_t xj_hi = xj << 16;
#pragma unroll
  for (int i = 0; i < P; ++i) {
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      n_gt += h ? __popcll(__ballot(v[i] >= xj_hi + 0x10000u)) : __popcll(__ballot((uint16_t)v[i] > (uint16_t)xj));
      eq_acc += h ? __popcll(__ballot((v[i] >> 16) == xj)) : __popcll(__ballot((uint16_t)v[i] == (uint16_t)xj));
      if (++r == rpt) {
        if (lane == q) eq_l = (uint32_t)eq_acc;
        n_eq += eq_acc;
        eq_acc = 0;
        r = 0; q += kWavesPerBlock;
      }
    }
  }
  n_gt = (int)block_sum((uint32_t)n_gt) - (2 * P * DYN_WAVE * kWavesPerBlock - m);
  n_eq = (int)block_sum((uint32_t)n_eq);
  const int need = j - n_gt;
  uint32_t place = (uint32_t)need;
  res->walk = true;
  if (need > 4 && n_eq - need + 1 > 4) {   // block-uniform
    // every wave's four smallest positive counts meet in LDS; the four smallest of the sixteen are the block's
    uint32_t m4[4];
    const int npos_w = smallest_four(eq_l, lane, m4);
    const int npos = (int)block_sum((uint32_t)npos_w);
    if (lane < 4) s_m[wave * 4 + lane] = lane == 0 ? m4[0] : lane == 1 ? m4[1] : lane == 2 ? m4[2] : m4[3];
    __syncthreads();
    uint32_t best[4] = {0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu};
    for (int i = 0; i < 4 * kWavesPerBlock; ++i) {
      uint32_t x = s_m[i];
#pragma unroll
      for (int k = 0; k < 4; ++k) {        // insertion into the ascending four
        const uint32_t lo = min(best[k], x);
        x = max(best[k], x);
        best[k] = lo;
      }
    }
    __syncthreads();                       // s_m is free again
    const uint32_t s4 = npos >= 4 ? best[0] + best[1] + best[2] + best[3] : 0u;
    res->walk = tight_place(need, n_eq, npos, s4, &place);
  } else if (need > 4) {
    place = (uint32_t)(n_eq - need + 1) | DYN_TIGHT_FROM_BELOW;
  }
  res->need = (uint32_t)need;
  res->tok_l = tok_l;                    // lanes q with q % 4 == wave
  res->eq_l = eq_l;
  res->xj = xj;
  res->place = place;
  return true;
}

__global__ __launch_bounds__(kWavesPerBlock* DYN_WAVE) void tick_tight_block_kernel(TickCellArgs a) {
  __shared__ uint32_t s_x[2 * kWavesPerBlock];
  __shared__ uint32_t s_m[4 * kWavesPerBlock];
  const int lane = threadIdx.x & (DYN_WAVE - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / DYN_WAVE);
  const int T = a.n_tick, G = a.G;
  const uint32_t n_item = a.counters[2];         // complete: written by the kernel before this one
  for (uint32_t item = blockIdx.x; item < n_item; item += gridDim.x) {
    const int64_t c = a.list_cells[item];
    const int64_t w = c / G;
    const int g = (int)(c % G);
    const int64_t f0 = (w * T) * G + g;
    int64_t beg_l = 0;
    int32_t cnt_l = 0;
    uint32_t bad_l = 0;
    if (lane < T) {
      const int64_t f = f0 + (int64_t)lane * G;
      const int64_t b = a.fine_off[f], e = a.fine_off[f + 1];
      if (b < 0 || e < b || e > a.n_req) bad_l = DYN_WS_BAD_OFFSETS;
      else { beg_l = b; cnt_l = (int32_t)(e - b); }
    }
    const int64_t m_cell = (int64_t)wave_sum_u64((uint64_t)(uint32_t)cnt_l);
    const int64_t rank = (a.pct_num * m_cell + a.pct_den - 1) / a.pct_den;
    const int64_t j64 = m_cell > 0 ? m_cell - rank + 1 : 0;
    const int rpt = ((int)wave_max_u32((uint32_t)cnt_l) + DYN_WAVE - 1) / DYN_WAVE;
    const int rows = ((T + kWavesPerBlock - 1) / kWavesPerBlock) * rpt;   // rows of the wave with most ticks
    TightCell tc;
    tc.tok_l = 0; tc.eq_l = 0; tc.xj = 0; tc.place = 0; tc.need = 0; tc.walk = true;
    bool done = false;                           // block-uniform from here on
    if (m_cell > 0 && m_cell < (1 << 24) && rows <= 128) {
      const float theta = a.theta[g];
      const int m = (int)m_cell, rk = (int)rank;
      if (rows <= 32) done = tight_cell_block<16>(a.in, a.out, beg_l, cnt_l, T, rpt, m, rk, theta, lane, wave, s_x, s_m, &tc);
      else if (rows <= 64) done = tight_cell_block<32>(a.in, a.out, beg_l, cnt_l, T, rpt, m, rk, theta, lane, wave, s_x, s_m, &tc);
      else done = tight_cell_block<64>(a.in, a.out, beg_l, cnt_l, T, rpt, m, rk, theta, lane, wave, s_x, s_m, &tc);
    }
    __syncthreads();                             // s_x is reused by the next item
    if (!done) continue;
    uint32_t flags = tbt_route(cnt_l, j64, lane) | DYN_TP_TIGHT;
    if (!tc.walk || !(flags & (DYN_TP_DENSE | DYN_TP_SMALL))) {
      flags |= DYN_TP_GENERAL;
      tc.place = tc.need;
    }
    if (lane < T && (lane % kWavesPerBlock) == wave) {   // the wave that walked the tick
      TickRec r;
      r.load = div_by((double)tc.tok_l, a.tick_s, a.r_tick);
      r.off = tc.eq_l;
      r.cnt = cnt_l;
      a.rec[c * T + lane] = r;
      a.cstat[f0 + (int64_t)lane * G] = (uint8_t)bad_l;
    }
    if (threadIdx.x == 0) {
      TickPlan p;
      p.j = (int32_t)j64;
      p.xj = (int32_t)tc.xj;
      p.flags = flags;
      p.place = tc.place;
      a.plan[c] = p;
      if (flags & DYN_TP_GENERAL) a.slow_list[atomicAdd(&a.counters[1], 1u)] = (uint32_t)c;
      a.list_cells[item] = DYN_LIST_DONE;
    }
  }
}

// ---- per-tick loads and candidate lists ------------------------------------------------------
// One wave per (window, class) cell walks the cell's ticks.  Lane q holds tick q's offsets;
// the cell's request count gives j.  Per tick the wave streams the tick's requests once:
// token sum (the tick's load) and, for 0 < j <= 64, the j largest input lengths, kept sorted
// (descending) in the wave's lanes.  A row of 64 new values is merged either by j rounds of
// "take the maximum of kept and new values" or, when few new values can still enter the
// first j positions, by ranking: a value's position is the number of values that beat it
// (kept values win ties against new ones, lower lanes against higher ones), and the merged
// order is written through a 64-word LDS buffer.  A second list, merged with every finished
// tick's list, holds the j largest lengths of the whole cell: its last entry is x_j.
__global__ __launch_bounds__(kWavesPerBlock* DYN_WAVE) void tick_cell_kernel(TickCellArgs a) {
  __shared__ int32_t s_buf[kWavesPerBlock][DYN_WAVE];
  const int lane = threadIdx.x & (DYN_WAVE - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / DYN_WAVE);
  const int T = a.n_tick, G = a.G;
  const int64_t item = (int64_t)blockIdx.x * kWavesPerBlock + wave;
  if (item >= (int64_t)a.counters[2]) return;   // complete: written by the kernel before this one
  if (a.list_cells[item] == DYN_LIST_DONE) return;   // settled by the kernel before this one
  const int64_t c = a.list_cells[item];
  const int64_t w = c / G;
  const int g = (int)(c % G);
  const int64_t f0 = (w * T) * G + g;           // fine cell of tick 0; tick q is q*G further

  int64_t beg_l = 0;
  int32_t cnt_l = 0;
  uint32_t bad_l = 0;
  if (lane < T) {
    const int64_t f = f0 + (int64_t)lane * G;
    const int64_t b = a.fine_off[f], e = a.fine_off[f + 1];
    if (b < 0 || e < b || e > a.n_req) bad_l = DYN_WS_BAD_OFFSETS;   // such a tick is treated as empty
    else { beg_l = b; cnt_l = (int32_t)(e - b); }
  }
  const int64_t m_cell = (int64_t)wave_sum_u64((uint64_t)(uint32_t)cnt_l);
  const int64_t rank = (a.pct_num * m_cell + a.pct_den - 1) / a.pct_den;
  const int64_t j64 = m_cell > 0 ? m_cell - rank + 1 : 0;
  const bool raw = j64 > DYN_TICK_DEPTH;         // deeper than a cut-down list: whole ticks are sorted, or scanned unsorted
  const bool deep = !raw && j64 > DYN_TICK_WAVE;
  const int keep = (raw || deep) ? 0 : (int)j64;                // wave-uniform, 0 .. 64

  // How the TBT percentile can be found: from the largest tick TBT when every non-empty tick holds
  // j requests; from the four largest tick TBTs when any four non-empty ticks hold j between them
  // (the four smallest counts do, or there are no more than four).
  uint32_t flags = raw ? DYN_TP_RAW : (deep ? DYN_TP_DEEP : 0u);
  if (m_cell > 0) {
    flags |= tbt_route(cnt_l, j64, lane);
    // the walk kernel keeps a register list of 16 candidates beside the largest tick TBT, of 8 beside the four largest
    const bool walk = ((flags & DYN_TP_DENSE) && j64 <= kFastDepth) || ((flags & DYN_TP_SMALL) && j64 <= kFastDepth / 2);
    if (raw || !walk) flags |= DYN_TP_GENERAL;
  }

  int32_t* buf = s_buf[wave];
  // Merges the values `cx` of the lanes with `mine` set into the descending list `best` (one entry per lane,
  // -1 = none); the first `keep` positions of the result are exact.
  auto merge = [&](int32_t best, int32_t cx, bool mine) -> int32_t {
    uint64_t mask = __ballot(mine);
    if (mask == 0) return best;
    if (__popcll(mask) * 10 > keep * 16) {
      // rounds of maximum extraction over kept and new values; a taken value leaves its lane
      int32_t bv = best, cv = mine ? cx : -1, nb = -1;
      for (int i = 0; i < keep; ++i) {
        const int32_t mx = wave_max_i32(max(bv, cv));
        if (mx < 0) break;
        const uint64_t ub = __ballot(bv == mx);
        if (ub) {
          if (lane == (int)__builtin_ctzll(ub)) bv = -1;
        } else {
          const uint64_t uc = __ballot(cv == mx);
          if (lane == (int)__builtin_ctzll(uc)) cv = -1;
        }
        if (lane == i) nb = mx;
      }
      return nb;
    }
    int rb = lane;      // position of my kept value: the kept values before it + new values above it
    int rc = 0;         // position of my new value: kept values >= it + new values that beat it
    while (mask) {
      const int u = __builtin_ctzll(mask);
      mask &= mask - 1;
      const int32_t v = __builtin_amdgcn_readlane(cx, u);
      const int n_ge = __popcll(__ballot(best >= v));
      rb += (v > best) ? 1 : 0;
      rc += (v > cx || (v == cx && u < lane)) ? 1 : 0;
      if (lane == u) rc += n_ge;
    }
    // the positions are a permutation of 0 .. 63 + (new values): every slot below 64 is written once
    if (rb < DYN_WAVE) buf[rb] = best;
    if (mine && rc < DYN_WAVE) buf[rc] = cx;
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    const int32_t merged = buf[lane];
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    return merged;
  };

  double load_l = 0.0;
  uint32_t neg_mask_lo = 0, neg_mask_hi = 0;    // ticks holding a negative token count
  int32_t gbest = -1;                           // the j largest input lengths of the cell so far
  bool g_empty = true;
  // (x, y) always hold the row after the one being processed: the next row of the same tick,
  // else the first row of the next tick
  int32_t x, y;
  auto fetch = [&](int64_t at, int32_t left) {   // `left` requests from `at` on, one per lane
    x = lane < left ? a.in[at + lane] : -1;
    y = lane < left ? a.out[at + lane] : 0;
  };
  fetch(readlane_i64(beg_l, 0), __builtin_amdgcn_readlane(cnt_l, 0));
  for (int q = 0; q < T; ++q) {
    const int64_t beg_q = readlane_i64(beg_l, q);
    const int32_t n_q = __builtin_amdgcn_readlane(cnt_l, q);
    int64_t beg_n = 0;
    int32_t n_n = 0;
    if (q + 1 < T) {
      beg_n = readlane_i64(beg_l, q + 1);
      n_n = __builtin_amdgcn_readlane(cnt_l, q + 1);
    }
    if (n_q == 0) fetch(beg_n, n_n);              // nothing was fetched for an empty tick
    uint64_t acc = 0;
    uint32_t orv = 0;
    int32_t best = -1;                            // input lengths are >= 0
    for (int32_t r0 = 0; r0 < n_q; r0 += DYN_WAVE) {
      const int nrow = n_q - r0 < DYN_WAVE ? n_q - r0 : DYN_WAVE;
      const bool have = lane < nrow;
      const int32_t cx = x, cy = y;
      if (r0 + DYN_WAVE < n_q) fetch(beg_q + r0 + DYN_WAVE, n_q - r0 - DYN_WAVE);
      else fetch(beg_n, n_n);
      acc += have ? (uint64_t)((int64_t)cx + (int64_t)cy) : 0;
      orv |= have ? (uint32_t)(cx | cy) : 0u;
      if (keep == 0) continue;
      const int32_t thr = __builtin_amdgcn_readlane(best, keep - 1);
      best = merge(best, cx, have && cx > thr);    // a value <= thr has `keep` kept values ahead of it
    }
    // the tick's token sum: 32-bit lanes when every lane's sum is small enough for it
    uint64_t tok;
    if (__ballot((acc >> 25) != 0) == 0) tok = wave_sum_u32((uint32_t)acc);
    else tok = wave_sum_u64(acc);
    if (__ballot((int32_t)orv < 0)) {
      if (q < 32) neg_mask_lo |= 1u << q; else neg_mask_hi |= 1u << (q - 32);
    }
    if (lane == q) load_l = div_by((double)tok, a.tick_s, a.r_tick);
    const int n_top = keep < n_q ? keep : n_q;
    if (lane < n_top) a.top[beg_q + lane] = best;           // the tick's list sits where its requests start
    if (n_top > 0) {                             // towards x_j: the walk prunes its lists with it, the general kernel brackets with it
      const int32_t mine_v = lane < n_top ? best : -1;
      if (g_empty) {
        gbest = mine_v;
        g_empty = false;
      } else {
        const int32_t thr = __builtin_amdgcn_readlane(gbest, keep - 1);
        gbest = merge(gbest, mine_v, mine_v > thr);
      }
    }
  }
  if (lane < T) {
    const int64_t f = f0 + (int64_t)lane * G;
    TickRec r;
    r.load = load_l;
    r.off = (uint32_t)beg_l;                     // n_req < 2^31
    r.cnt = cnt_l;
    a.rec[c * T + lane] = r;
    const uint32_t neg = lane < 32 ? (neg_mask_lo >> lane) & 1u : (neg_mask_hi >> (lane - 32)) & 1u;
    // every fine cell writes its own status byte: nothing to clear beforehand
    a.cstat[f] = (uint8_t)(bad_l | (neg ? DYN_WS_BAD_REQUEST : 0u));
  }
  const int32_t xj = keep > 0 ? __builtin_amdgcn_readlane(gbest, keep - 1) : 0;
  if (lane == 0) {
    TickPlan p;
    p.j = (int32_t)j64;                          // below 2^31 like the number of requests
    p.xj = xj < 0 ? 0 : xj;
    p.flags = flags;
    p.place = 0;
    a.plan[c] = p;
    if (deep || raw) a.deep_list[atomicAdd(&a.counters[0], 1u)] = (uint32_t)c;   // x_j and the sorted ticks come from there
    if (flags & DYN_TP_GENERAL) a.slow_list[atomicAdd(&a.counters[1], 1u)] = (uint32_t)c;
    else if (j64 > 0) atomicAdd(&a.counters[3], 1u);   // a cell the walk takes with its lists
  }
}

// ---- cells whose percentile lies more than 64 deep ------------------------------------------------
// A block per listed cell.  x_j by a most-significant-bit-first search on the value, every step a
// count over the cell's requests; then every tick's min(j, count) largest input lengths in descending
// order: a tick of up to 8192 requests is sorted whole in LDS (bitonic), a larger one is first cut
// down to its j largest (threshold by the same bit search, the values above it gathered, the rest of
// the j places filled with the threshold itself).
__global__ __launch_bounds__(256) void tick_deep_kernel(TickCellArgs a) {
  __shared__ int32_t s_val[kDeepCap];
  __shared__ uint32_t s_part[4];
  __shared__ uint32_t s_fill;
  const int tid = threadIdx.x, lane = tid & (DYN_WAVE - 1), wave = tid / DYN_WAVE;
  const int T = a.n_tick;
  const uint32_t n_deep = a.counters[0];         // complete: written by the kernel before this one
  auto block_sum = [&](uint32_t v) -> uint32_t {
    const uint32_t ws = wave_sum_u32(v);
    __syncthreads();
    if (lane == 0) s_part[wave] = ws;
    __syncthreads();
    return s_part[0] + s_part[1] + s_part[2] + s_part[3];
  };
  auto block_max = [&](int32_t v) -> int32_t {
    const int32_t wm = wave_max_i32(v);
    __syncthreads();
    if (lane == 0) s_part[wave] = (uint32_t)wm;
    __syncthreads();
    return max(max((int32_t)s_part[0], (int32_t)s_part[1]), max((int32_t)s_part[2], (int32_t)s_part[3]));
  };
  // j-th largest value of the ticks q0 .. q1-1 of the cell (at least j values, all bits above `bits` clear)
  auto jth_largest = [&](const TickRec* rec, int q0, int q1, int bits, int32_t j) -> int32_t {
    int32_t v = 0;
    for (int b = bits - 1; b >= 0; --b) {
      const int32_t cand = v | (int32_t)(1u << b);
      uint32_t n = 0;
      for (int q = q0; q < q1; ++q) {
        const TickRec r = rec[q];
        const int32_t* src = a.in + r.off;
        for (int i = tid; i < r.cnt; i += 256) n += src[i] >= cand ? 1u : 0u;
      }
      if (block_sum(n) >= (uint32_t)j) v = cand;
    }
    return v;
  };
  for (uint32_t it = blockIdx.x; it < n_deep; it += gridDim.x) {
    const int64_t c = a.deep_list[it];
    const int32_t j = a.plan[c].j;               // beyond 64; beyond 8192 for DYN_TP_RAW cells
    const TickRec* rec = a.rec + c * T;
    int32_t mx = 0;
    for (int q = 0; q < T; ++q) {
      const TickRec r = rec[q];
      const int32_t* src = a.in + r.off;
      for (int i = tid; i < r.cnt; i += 256) mx = max(mx, src[i]);
    }
    mx = block_max(mx);
    const int bits = 32 - __builtin_clz((uint32_t)mx | 1u);   // mx >= 0: at most 31
    const int32_t xj = jth_largest(rec, 0, T, bits, j);
    if (tid == 0) a.plan[c].xj = xj;
    // sorts s_val[0 .. n_sort) descending (bitonic, padded to a power of two) and writes its first n_out entries to dst
    auto sort_and_store = [&](int n_sort, int n_out, int32_t* dst) {
      int n2 = 2;
      while (n2 < n_sort) n2 <<= 1;              // at most 8192
      for (int i = n_sort + tid; i < n2; i += 256) s_val[i] = (int32_t)0x80000000;
      __syncthreads();
      for (int k = 2; k <= n2; k <<= 1)
        for (int d = k >> 1; d > 0; d >>= 1) {
          for (int i = tid; i < n2; i += 256) {
            const int o = i ^ d;
            if (o > i) {
              const int32_t u = s_val[i], v = s_val[o];
              const bool down = (i & k) == 0;    // descending runs first: the whole array ends descending
              if (down ? u < v : u > v) { s_val[i] = v; s_val[o] = u; }
            }
          }
          __syncthreads();
        }
      for (int i = tid; i < n_out; i += 256) dst[i] = s_val[i];
      __syncthreads();                           // s_val is reused
    };
    for (int q = 0; q < T; ++q) {
      const TickRec r = rec[q];
      if (r.cnt == 0) continue;                  // block-uniform
      const int32_t* src = a.in + r.off;
      int32_t* dst = a.top + r.off;
      if (r.cnt <= kDeepCap) {
        for (int i = tid; i < r.cnt; i += 256) s_val[i] = src[i];
        sort_and_store(r.cnt, r.cnt < j ? r.cnt : j, dst);
      } else if (j > kDeepCap) {                 // block-uniform: neither the tick nor its j largest fit: sorted piece by piece
        for (int base = 0; base < r.cnt; base += kDeepCap) {
          const int n = r.cnt - base < kDeepCap ? r.cnt - base : kDeepCap;
          for (int i = tid; i < n; i += 256) s_val[i] = src[base + i];
          sort_and_store(n, n, dst + base);
        }
        if (tid == 0) a.rec[c * T + q].off = r.off | DYN_TICK_PIECES;
      } else {                                   // more than 8192 requests, of which the j <= 8192 largest are wanted
        const int32_t thr = jth_largest(rec, q, q + 1, bits, j);
        if (tid == 0) s_fill = 0u;
        __syncthreads();
        for (int i = tid; i < r.cnt; i += 256) {
          const int32_t v = src[i];
          if (v > thr) {                         // fewer than j of them
            const uint32_t at = atomicAdd(&s_fill, 1u);
            if (at < (uint32_t)kDeepCap) s_val[at] = v;
          }
        }
        __syncthreads();
        const int got = (int)min(s_fill, (uint32_t)j);
        for (int i = got + tid; i < j; i += 256) s_val[i] = thr;
        sort_and_store(j, j, dst);
      }
    }
  }
}

// ---- evaluation of the (cell, configuration) space -----------------------------------------------
// A tick's candidates (descending input lengths x its prefill time) against the sorted list
// s[0] >= ... >= s[JF-1]: once one of them cannot enter the list in any lane, the rest of
// that tick cannot either.
// Lengths below `xmin` (block-uniform) cannot reach the cell's percentile under any configuration of the block.
template <int JF>
__device__ __forceinline__ void offer_tick(double (&s)[JF], const int32_t* s_top, int T, int q, int nc, int xmin, double pf) {
  for (int x = 0; x < nc; ++x) {
    const int len = __builtin_amdgcn_readfirstlane(s_top[x * T + q]);
    if (len < xmin) break;
    double v = (double)len * pf;
    if (__ballot(v > s[JF - 1]) == 0) break;
#pragma unroll
    for (int i = 0; i < JF; ++i) {
      const double hi = max_num(s[i], v);
      v = min_num(s[i], v);
      s[i] = hi;
    }
  }
}

// Power of the configuration at load 0: what table_lookup returns for it (bracket 0, weight 0 on the second load point).
template <bool TWO>
__device__ __forceinline__ double idle_power(const Lookup& L) {
  const double a = L.lo[2 * L.n_rho];
  return TWO ? L.omu * a + L.u * L.hi[2 * L.n_rho] : a;
}

// The four largest tick TBTs with their request counts (descending; ties keep the earlier tick first).
struct TbtTop {
  double tb[4];
  int32_t cnt[4];
  __device__ __forceinline__ void clear() {
#pragma unroll
    for (int i = 0; i < 4; ++i) { tb[i] = -__builtin_inf(); cnt[i] = 0; }
  }
  __device__ __forceinline__ void offer(double v, int32_t c) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const bool gt = v > tb[i];
      const double tv = tb[i];
      const int32_t tc = cnt[i];
      tb[i] = gt ? v : tv;
      cnt[i] = gt ? c : tc;
      v = gt ? tv : v;
      c = gt ? tc : c;
    }
  }
  __device__ __forceinline__ double jth(int32_t j) const {    // the kept ticks hold at least j requests
    double r = tb[3];
    int32_t cum = 0;
    bool found = false;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      cum += cnt[i];
      const bool hit = !found && cum >= j;
      r = hit ? tb[i] : r;
      found = found || hit;
    }
    return r;
  }
};

struct WalkOut {
  double e, ttft, tbt;
  bool ov;
};

// One walk over the ticks of a cell, in time order, two look-ups in flight (PAIR; one at a time leaves registers for
// a fifth wave per SIMD in the kernel without lists, which gains more than the second look-up in flight).  The cell's j <= JF largest scaled
// candidates go through a sorted list that starts with JF - j copies of +inf, so that its last entry is the j-th
// largest of what was inserted (j == 0: nothing is inserted).  SPARSE: the TBT percentile from the four largest
// tick TBTs, else the largest tick TBT.
// TIGHT: the TTFT percentile is x_j times the prefill time of rank `place` (bit 31: from below) among the ticks, each
// counted as often as it holds requests of length x_j (`s_top`: that number per tick; `xmin` carries x_j): the four
// largest (smallest) prefill times are kept with their counts.
template <int JF, bool SPARSE, bool SINGLE, bool TWO, bool TIGHT = false, bool PAIR = true>
__device__ __forceinline__ WalkOut walk_ticks(const Lookup& L, int T, int j, const double* s_load, const int32_t* s_cnt,
                                              const int32_t* s_top, int xmin, double nd, double tick_s, uint32_t place = 0) {
  double s[JF];
  int wt[TIGHT ? JF : 1];
  const double sign = (place & DYN_TIGHT_FROM_BELOW) ? -1.0 : 1.0;
#pragma unroll
  for (int i = 0; i < JF; ++i) s[i] = (!TIGHT && i < JF - j) ? __builtin_inf() : -__builtin_inf();
  if (TIGHT) {
#pragma unroll
    for (int i = 0; i < JF; ++i) wt[i] = 0;
  }
  double e = 0.0, tbmax = -__builtin_inf();
  TbtTop tt;
  if (SPARSE) tt.clear();
  bool ov = false;
  auto one = [&](int q, int c0, double pf0, double tb0) {
    if (c0 > 0 && j > 0) {                       // block-uniform
      if (SPARSE) tt.offer(tb0, c0); else tbmax = max_num(tbmax, tb0);
      if (TIGHT) {
        const int eq = __builtin_amdgcn_readfirstlane(s_top[q]);
        double key = pf0 * sign;
        if (eq > 0 && __ballot(key > s[JF - 1]) != 0) {
          int w_in = eq;
#pragma unroll
          for (int i = 0; i < JF; ++i) {
            const bool gt = key > s[i];
            const double tk = s[i];
            const int tw = wt[i];
            s[i] = gt ? key : tk;
            wt[i] = gt ? w_in : tw;
            key = gt ? tk : key;
            w_in = gt ? tw : w_in;
          }
        }
      } else {
        offer_tick<JF>(s, s_top, T, q, c0 < j ? c0 : j, xmin, pf0);
      }
    }
  };
  // a tick without requests has load 0: the tables at their first load point, no look-up
  const double e_idle = (nd * idle_power<TWO>(L)) * tick_s;
  int q = 0;
  for (; q + 2 <= T; q += 2) {
    const int c0 = s_cnt[q], c1 = s_cnt[q + 1];                 // block-uniform
    if (PAIR && c0 > 0 && c1 > 0) {
      double pf0, tb0, pw0, pf1, tb1, pw1;
      const bool o0 = table_lookup<SINGLE, TWO>(L, s_load[q], &pf0, &tb0, &pw0);
      const bool o1 = table_lookup<SINGLE, TWO>(L, s_load[q + 1], &pf1, &tb1, &pw1);
      ov = ov | o0 | o1;
      e += (nd * pw0) * tick_s;                  // ticks in time order
      e += (nd * pw1) * tick_s;
      one(q, c0, pf0, tb0);
      one(q + 1, c1, pf1, tb1);
    } else {
#pragma unroll
      for (int d = 0; d < 2; ++d) {
        const int cd = d ? c1 : c0;
        if (cd > 0) {
          double pf0, tb0, pw0;
          ov = ov | table_lookup<SINGLE, TWO>(L, s_load[q + d], &pf0, &tb0, &pw0);
          e += (nd * pw0) * tick_s;
          one(q + d, cd, pf0, tb0);
        } else {
          e += e_idle;
        }
      }
    }
  }
  if (q < T) {
    const int c0 = s_cnt[q];
    if (c0 > 0) {
      double pf0, tb0, pw0;
      ov = ov | table_lookup<SINGLE, TWO>(L, s_load[q], &pf0, &tb0, &pw0);
      e += (nd * pw0) * tick_s;
      one(q, c0, pf0, tb0);
    } else {
      e += e_idle;
    }
  }
  WalkOut r;
  r.e = e; r.ov = ov; r.ttft = s[JF - 1];
  if (TIGHT) {
    const int want = (int)(place & ~DYN_TIGHT_FROM_BELOW);
    double pick = s[JF - 1];
    int cum = 0;
    bool found = false;
#pragma unroll
    for (int i = 0; i < JF; ++i) {
      cum += wt[i];
      const bool hit = !found && cum >= want;
      pick = hit ? s[i] : pick;
      found = found || hit;
    }
    r.ttft = (double)xmin * (pick * sign);
  }
  r.tbt = SPARSE ? tt.jth(j) : tbmax;
  return r;
}

// Per-thread state of one configuration inside a (class, tile) block.
struct CfgState {
  Lookup L;
  double nd, slo_ttft, slo_tbt, idle_term;
  uint32_t fl_budget, koff;
  int k, k_raw, lane, wslot;
  bool live;
};

// The constants of configuration k_raw (>= K: a copy of the last one that stores nothing): `g` is
// block-uniform; the table rows are either the block's LDS copy (LDS) or global memory.
template <bool LDS>
__device__ __forceinline__ void load_config(const TickArgs& a, int g, int k_raw, const double* s_tab, const double* s_rgp,
                                            const double* s_rinv, const double* s_thr, const uint16_t* s_js,
                                            CfgState* st) {
  const SpaceArgs& sa = a.s;
  const int n_rho = sa.n_rho;
  st->k_raw = k_raw;
  st->live = st->k_raw < sa.K;            // every lane stays alive for the wave reduction
  st->k = st->live ? st->k_raw : sa.K - 1;
  const DevCfg c = sa.cfg[st->k];
  const size_t grow = (size_t)g * sa.n_tp_f;
  const double ml_lo = sa.ml[grow + c.row_lo], ml_hi = sa.ml[grow + c.row_hi];
  const double p0_lo = sa.pw0[grow + c.row_lo], p0_hi = sa.pw0[grow + c.row_hi];
  const bool two_rows = c.u != 0.0;
  Lookup& L = st->L;
  L.u = c.u;
  L.omu = 1.0 - c.u;
  const double ml = two_rows ? L.omu * ml_lo + c.u * ml_hi : ml_lo;
  L.den = c.nd * ml;
  L.rden = 1.0 / L.den;
  L.rho_max = s_rgp[n_rho];
  L.bucket_scale = sa.bucket_scale;
  L.rgp = s_rgp; L.rinv = s_rinv; L.js = s_js; L.thr = s_thr; L.n_rho = n_rho;
  if (LDS) {      // kept apart so that the address space of the rows is known at compile time
    L.lo = s_tab + (size_t)c.slot_lo * DYN_SLOT_STRIDE(n_rho);
    L.hi = s_tab + (size_t)c.slot_hi * DYN_SLOT_STRIDE(n_rho);
  } else {
    L.lo = sa.tab + (grow + c.row_lo) * 3 * n_rho;
    L.hi = sa.tab + (grow + c.row_hi) * 3 * n_rho;
  }
  st->nd = c.nd;
  st->slo_ttft = sa.slo_ttft[g];
  st->slo_tbt = sa.slo_tbt[g];
  const int32_t bud = sa.budget[g];
  st->fl_budget = (bud > 0 && c.gpus > bud) ? DYN_F_BUDGET : 0u;
  const double pw0 = two_rows ? L.omu * p0_lo + c.u * p0_hi : p0_lo;
  st->idle_term = sa.idle_w * ((c.nd * pw0) * a.window_s);
  st->lane = threadIdx.x & (DYN_WAVE - 1);
  st->wslot = st->k_raw / DYN_WAVE;       // tiles are multiples of 64 configurations wide
  st->koff = (uint32_t)st->k * 8u;
}

// One flat loop over the rows a tile needs: the loads of different rows are in flight together.
__device__ __forceinline__ void stage_rows(const SpaceArgs& sa, int g, int tile, double* s_tab) {
  const int per_slot = 3 * sa.n_rho, total = sa.n_slot * per_slot;
  const int32_t* rows = sa.tile_rows + tile * sa.n_slot;
  const double* base = sa.tab + (size_t)g * sa.n_tp_f * per_slot;
#pragma unroll 4
  for (int i = threadIdx.x; i < total; i += blockDim.x) {
    const int slot = i / per_slot;
    const int row = rows[slot];
    s_tab[slot * DYN_SLOT_STRIDE(sa.n_rho) + (i - slot * per_slot)] = base[(size_t)(row < 0 ? 0 : row) * per_slot + (i - slot * per_slot)];
  }
}
template <bool SINGLE>
__device__ __forceinline__ void stage_grid(const TickArgs& a, double* s_rgp, double* s_thr, uint16_t* s_js) {
  const SpaceArgs& sa = a.s;
  for (int i = threadIdx.x; i < 2 * sa.n_rho + 3; i += blockDim.x) s_rgp[i] = sa.gridpack[i];
  for (int i = threadIdx.x; i <= sa.n_bucket; i += blockDim.x) {
    s_js[i] = (uint16_t)(SINGLE ? a.tstart[i] : sa.jstart[i]);
    if (SINGLE) s_thr[i] = a.thr[i];
  }
}

// Flags, streaming stores of the four outputs and the wave's partial selection for one cell.
__device__ __forceinline__ void emit_cell(const SpaceArgs& sa, const CfgState& st, size_t cell, bool empty, bool ov, double e,
                                          double p_ttft, double p_tbt) {
  uint32_t fl = st.fl_budget;
  if (ov) fl |= DYN_F_OVERLOAD;
  if (p_ttft > st.slo_ttft) fl |= DYN_F_TTFT;
  if (p_tbt > st.slo_tbt) fl |= DYN_F_TBT;
  if (!fl) fl = DYN_F_FEASIBLE;
  if (empty) fl |= DYN_F_EMPTY;
  if (st.live) {
    const size_t row = cell * (size_t)sa.K;
    __builtin_nontemporal_store(e, (double*)((char*)(sa.energy + row) + st.koff));
    __builtin_nontemporal_store(p_ttft, (double*)((char*)(sa.p99_ttft + row) + st.koff));
    __builtin_nontemporal_store(p_tbt, (double*)((char*)(sa.p99_tbt + row) + st.koff));
    __builtin_nontemporal_store((uint8_t)fl, (sa.flags + row) + (uint32_t)st.k);
  }
  // least cost among this wave's feasible configurations (costs >= +0 order like their bits)
  const bool feas = st.live && (fl & DYN_F_FEASIBLE);
  const double cost = e + st.idle_term;
  const uint64_t bits = (uint64_t)__double_as_longlong(cost);
  const uint32_t hi = feas ? (uint32_t)(bits >> 32) : 0xFFFFFFFFu;
  const uint32_t lo = feas ? (uint32_t)bits : 0xFFFFFFFFu;
  const uint32_t mh = wave_min_u32(hi);
  uint64_t win = __ballot(feas && hi == mh);
  if (__popcll(win) > 1) {
    const uint32_t mlo = wave_min_u32(hi == mh ? lo : 0xFFFFFFFFu);
    win = __ballot(feas && hi == mh && lo == mlo);
  }
  const int wl = win ? __builtin_ctzll(win) : 0;
  if (st.lane == wl) {
    SelPart p;
    p.cost = win ? cost : __builtin_inf();
    p.energy = win ? e : __builtin_inf();
    p.k = win ? st.k_raw : -1;
    p.pad = 0;
    sa.part[cell * (size_t)sa.n_wslot + st.wslot] = p;
  }
}

// A block walks a run of windows of one (class, tile): the empty cells, the cells that are not evaluated and
// the cells the cell kernel left to this kernel (the others are the general kernel's).  The next cell's
// candidate lists are kept in flight (NPRE registers per thread) while the current one is evaluated.
// LDS: [table rows n_slot*3*n_rho] [padded load grid n_rho+2] [reciprocal spacings n_rho+1]
//      [SINGLE: grid point per bucket, n_bucket+1]
//      [per window of the block, per tick: load] [the same: request count] [the same: list offset]
//      [per window: plan] [two buffers of candidate lists, [position][tick]] [bucket index (16-bit)]
template <int TB, bool LDS, bool SINGLE, bool TWO>
__global__ __launch_bounds__(DYN_MAX_TILE) __attribute__((amdgpu_waves_per_eu(4, 4))) void tick_space_kernel(TickArgs a) {
  constexpr int NPRE = kFastDepth * TB / DYN_WAVE;   // blocks have at least 64 threads; n_tick <= TB
  extern __shared__ double smem[];
  const SpaceArgs& sa = a.s;
  const int tile = blockIdx.x % sa.n_tile;
  const int g = (blockIdx.x / sa.n_tile) % sa.G;
  const int chunk = blockIdx.x / (sa.n_tile * sa.G);
  const int n_rho = sa.n_rho, T = a.n_tick;
  const int w0 = chunk * sa.win_per_block;
  const int w1 = min(w0 + sa.win_per_block, sa.n_window);

  double* s_tab = smem;
  double* s_rgp = smem + (LDS ? (size_t)sa.n_slot * DYN_SLOT_STRIDE(n_rho) : 0);
  double* s_rinv = s_rgp + (n_rho + 2);
  double* s_thr = s_rinv + (n_rho + 1);                         // [n_bucket + 1] when SINGLE
  uint32_t* s_ratio = (uint32_t*)(s_thr + (SINGLE ? sa.n_bucket + 1 : 0));   // [4] per wave (two doubles' room)
  double* s_load = (double*)s_ratio + 2;                        // [win_per_block][T]
  TickPlan* s_plan = (TickPlan*)(s_load + sa.win_per_block * T);   // [win_per_block]
  int32_t* s_cnt = (int32_t*)(s_plan + sa.win_per_block);       // [win_per_block][T] requests per tick
  uint32_t* s_off = (uint32_t*)(s_cnt + sa.win_per_block * T);  // [win_per_block][T] start of the tick's list
  int32_t* s_top = (int32_t*)(s_off + sa.win_per_block * T);    // [2][kFastDepth][T]
  uint16_t* s_js = (uint16_t*)(s_top + 2 * T * kFastDepth);     // [n_bucket + 1]

  // a block without a cell that is walked with lists has nothing to stage; most traces have no such cell at all
  if (a.counters[3] == 0u) return;
  bool any = false;
  for (int w = w0; w < w1; ++w) {
    const TickPlan p = a.plan[(size_t)w * sa.G + g];
    any = any || (p.j > 0 && !(p.flags & (DYN_TP_GENERAL | DYN_TP_TIGHT)));
  }
  if (!any) return;                                             // block-uniform

  if (LDS) stage_rows(sa, g, tile, s_tab);
  stage_grid<SINGLE>(a, s_rgp, s_thr, s_js);
  for (int i = threadIdx.x; i < (w1 - w0) * T; i += blockDim.x) {   // the ticks of this block's cells
    const int dw = i / T, q = i - dw * T;
    const TickRec r = a.rec[((size_t)(w0 + dw) * sa.G + g) * T + q];
    s_load[i] = r.load;
    s_cnt[i] = r.cnt;
    s_off[i] = r.off;
  }
  for (int i = threadIdx.x; i < w1 - w0; i += blockDim.x) s_plan[i] = a.plan[(size_t)(w0 + i) * sa.G + g];
  {
    // How far apart a configuration's per-tick prefill times can lie: theta = least / largest entry of its table
    // row(s), as a float rounded down; the block uses the smallest theta of its configurations.
    const int k_mine = min(tile * sa.tile + (int)threadIdx.x, sa.K - 1);
    const DevCfg c = sa.cfg[k_mine];
    const double* span = a.pfspan + 2 * ((size_t)g * sa.n_tp_f);
    double mn = span[2 * c.row_lo], mx = span[2 * c.row_lo + 1];
    if (c.u != 0.0) {
      mn = min_num(mn, span[2 * c.row_hi]);
      mx = max_num(mx, span[2 * c.row_hi + 1]);
    }
    const float th = (mx > 0.0 && mn > 0.0) ? (float)(mn / mx) * 0.999999f : 0.0f;   // below mn / mx by 2^-21 at least
    const uint32_t bits = wave_min_u32(__float_as_uint(th));                          // floats >= 0 order like their bits
    if ((threadIdx.x & (DYN_WAVE - 1)) == 0) s_ratio[threadIdx.x / DYN_WAVE] = bits;
  }
  __syncthreads();
  CfgState st;
  load_config<LDS>(a, g, tile * sa.tile + (int)threadIdx.x, s_tab, s_rgp, s_rinv, s_thr, s_js, &st);
  uint32_t ratio_bits = s_ratio[0];
  for (int i = 1; i < (int)blockDim.x / DYN_WAVE; ++i) ratio_bits = min(ratio_bits, s_ratio[i]);
  const double theta = (double)__uint_as_float(ratio_bits);

  // the cells this kernel walks with candidates: their lists are staged [position][tick]
  auto listed = [&](const TickPlan& p) { return p.j > 0 && !(p.flags & (DYN_TP_GENERAL | DYN_TP_TIGHT)); };
  int32_t pre[NPRE];
  auto prefetch = [&](int w) {
    if (w >= w1) return;
    const TickPlan p = s_plan[w - w0];
    if (!listed(p)) return;
    const int n = p.j * T;                     // at most kFastDepth * TB
    const int32_t* cnt_w = s_cnt + (w - w0) * T;
    const uint32_t* off_w = s_off + (w - w0) * T;
#pragma unroll
    for (int r = 0; r < NPRE; ++r) {
      const int i = threadIdx.x + r * blockDim.x;
      if (i < n) {
        const int pos = i / T, q = i - pos * T;
        pre[r] = pos < cnt_w[q] ? a.top[(size_t)off_w[q] + pos] : 0;   // a tick's list has min(j, count) entries
      }
    }
  };
  prefetch(w0);
  int buf = 0;
  for (int w = w0; w < w1; ++w) {
    const size_t cell = (size_t)w * sa.G + g;
    const int32_t* cnt_w = s_cnt + (w - w0) * T;
    const double* load_w = s_load + (w - w0) * T;
    const TickPlan pl = s_plan[w - w0];
    if (!listed(pl)) {                           // block-uniform: another kernel's cell
      prefetch(w + 1);
      continue;
    }
    const int j = pl.j;
    // two buffers: the lists of the cell before this one may still be read by slower waves
    int32_t* top_w = s_top + buf * (T * kFastDepth);
    {
      buf ^= 1;
      const int n = j * T;
#pragma unroll
      for (int r = 0; r < NPRE; ++r) {
        const int i = threadIdx.x + r * blockDim.x;
        if (i < n) top_w[i] = pre[r];
      }
      __syncthreads();
    }
    prefetch(w + 1);

    // Pruning: a request of length a < x_j * theta has, under every configuration of the block, TTFT = a * pf <
    // x_j * (least pf of that configuration) <= the TTFT of each of the j requests of length >= x_j: it lies below the
    // percentile, which is the j-th largest of what is left all the same.  With flat prefill tables what is left are
    // the cell's j largest lengths, whichever ticks hold them.
    const int xmin = (int)((double)pl.xj * theta);
    WalkOut o;
    if (pl.flags & DYN_TP_DENSE) {
      if (j <= 4) o = walk_ticks<4, false, SINGLE, TWO>(st.L, T, j, load_w, cnt_w, top_w, xmin, st.nd, a.tick_s);
      else if (j <= 8) o = walk_ticks<8, false, SINGLE, TWO>(st.L, T, j, load_w, cnt_w, top_w, xmin, st.nd, a.tick_s);
      else o = walk_ticks<kFastDepth, false, SINGLE, TWO>(st.L, T, j, load_w, cnt_w, top_w, xmin, st.nd, a.tick_s);
    } else {
      if (j <= 4) o = walk_ticks<4, true, SINGLE, TWO>(st.L, T, j, load_w, cnt_w, top_w, xmin, st.nd, a.tick_s);
      else o = walk_ticks<kFastDepth / 2, true, SINGLE, TWO>(st.L, T, j, load_w, cnt_w, top_w, xmin, st.nd, a.tick_s);
    }
    emit_cell(sa, st, cell, false, o.ov, o.e, o.ttft, o.tbt);
  }
}

// The same block mapping for the cells that need no lists: empty cells, cells that are not evaluated, and the cells
// settled by their ticks' requests of length x_j (DYN_TP_TIGHT).  Nothing is staged per cell and the block has no
// barrier after its set-up.
// LDS: [table rows] [padded load grid] [reciprocal spacings] [SINGLE: grid point per bucket]
//      [per window of the block, per tick: load] [per window: plan] [per window and tick: request count, requests of length x_j]
//      [bucket index (16-bit)]
template <bool LDS, bool SINGLE, bool TWO>
__global__ __launch_bounds__(DYN_MAX_TILE) __attribute__((amdgpu_waves_per_eu(5, 5))) void tick_tight_walk_kernel(TickArgs a) {
  extern __shared__ double smem[];
  const SpaceArgs& sa = a.s;
  const int tile = blockIdx.x % sa.n_tile;
  const int g = (blockIdx.x / sa.n_tile) % sa.G;
  const int chunk = blockIdx.x / (sa.n_tile * sa.G);
  const int n_rho = sa.n_rho, T = a.n_tick;
  const int w0 = chunk * sa.win_per_block;
  const int w1 = min(w0 + sa.win_per_block, sa.n_window);

  double* s_tab = smem;
  double* s_rgp = smem + (LDS ? (size_t)sa.n_slot * DYN_SLOT_STRIDE(n_rho) : 0);
  double* s_rinv = s_rgp + (n_rho + 2);
  double* s_thr = s_rinv + (n_rho + 1);                         // [n_bucket + 1] when SINGLE
  double* s_load = s_thr + (SINGLE ? sa.n_bucket + 1 : 0);      // [win_per_block][T]
  TickPlan* s_plan = (TickPlan*)(s_load + sa.win_per_block * T);   // [win_per_block]
  int32_t* s_cnt = (int32_t*)(s_plan + sa.win_per_block);       // [win_per_block][T] requests per tick
  int32_t* s_eq = s_cnt + sa.win_per_block * T;                 // [win_per_block][T] requests of length x_j per tick
  uint16_t* s_js = (uint16_t*)(s_eq + sa.win_per_block * T);    // [n_bucket + 1]

  auto mine = [](const TickPlan& p) {
    return p.j == 0 || ((p.flags & DYN_TP_TIGHT) && !(p.flags & DYN_TP_GENERAL));
  };
  bool any = false;
  for (int w = w0; w < w1; ++w) any = any || mine(a.plan[(size_t)w * sa.G + g]);
  if (!any) return;                                             // block-uniform

  if (LDS) stage_rows(sa, g, tile, s_tab);
  stage_grid<SINGLE>(a, s_rgp, s_thr, s_js);
  for (int i = threadIdx.x; i < (w1 - w0) * T; i += blockDim.x) {   // the ticks of this block's cells
    const int dw = i / T, q = i - dw * T;
    const TickRec r = a.rec[((size_t)(w0 + dw) * sa.G + g) * T + q];
    s_load[i] = r.load;
    s_cnt[i] = r.cnt;
    s_eq[i] = (int32_t)r.off;
  }
  for (int i = threadIdx.x; i < w1 - w0; i += blockDim.x) s_plan[i] = a.plan[(size_t)(w0 + i) * sa.G + g];
  __syncthreads();
  CfgState st;
  load_config<LDS>(a, g, tile * sa.tile + (int)threadIdx.x, s_tab, s_rgp, s_rinv, s_thr, s_js, &st);
  for (int w = w0; w < w1; ++w) {
    const TickPlan pl = s_plan[w - w0];
    if (!mine(pl)) continue;                     // block-uniform
    const size_t cell = (size_t)w * sa.G + g;
    const int32_t* cnt_w = s_cnt + (w - w0) * T;
    const double* load_w = s_load + (w - w0) * T;
    const int32_t* eq_w = s_eq + (w - w0) * T;
    const int j = pl.j;
    const bool empty = j == 0;
    WalkOut o;
    if (empty) {
      o = walk_ticks<4, false, SINGLE, TWO, false, false>(st.L, T, 0, load_w, cnt_w, eq_w, 0, st.nd, a.tick_s);
      o.ttft = o.tbt = 0.0;
    } else if (pl.flags & DYN_TP_DENSE) {
      o = walk_ticks<4, false, SINGLE, TWO, true, false>(st.L, T, j, load_w, cnt_w, eq_w, pl.xj, st.nd, a.tick_s, pl.place);
    } else {
      o = walk_ticks<4, true, SINGLE, TWO, true, false>(st.L, T, j, load_w, cnt_w, eq_w, pl.xj, st.nd, a.tick_s, pl.place);
    }
    emit_cell(sa, st, cell, empty, o.ov, o.e, o.ttft, o.tbt);
  }
}

// Weighted order statistic over the ticks: the largest value v among those of the ticks with weight > 0 such that the
// ticks with a value >= v weigh at least `need` together (ticks are taken in descending order of value, equal
// values together).  strip[q * NT + tid] is this thread's value of tick q.
__device__ __forceinline__ double weighted_from_top(const double* strip, const int32_t* weight, int T, int NT, int need, int tid) {
  double prev = __builtin_inf(), val = 0.0;
  while (need > 0) {
    double best = -__builtin_inf();
    int c = 0;
    for (int q = 0; q < T; ++q) {
      const int wq = weight[q];
      if (wq == 0) continue;
      const double v = strip[q * NT + tid];
      const bool lt = v < prev;
      const bool gt = lt && v > best;
      const bool eq = lt && v == best;
      c = gt ? wq : (eq ? c + wq : c);
      best = gt ? v : best;
    }
    if (c == 0) break;                       // cannot happen while the weights add up to at least `need`
    need -= c;
    prev = best;
    val = best;
  }
  return val;
}

// The cells the cell kernel left to this kernel, (cell, tile) by (cell, tile), the items dealt round-robin to a
// fixed grid so that runs of heavy cells spread over the chip.  A block of NT threads takes the tile's
// configurations NT at a time.  One strip in LDS holds a value per (tick, configuration).  Cells whose
// non-empty ticks all hold j requests: one pass over the ticks (energy, largest TBT = the TBT percentile,
// prefill times into the strip).  Other cells: a first pass with the TBTs in the strip, the TBT percentile
// by taking ticks in descending TBT order until j requests are covered, then the look-ups again for the
// prefill times.  The TTFT percentile lies in the bracket [x_j * least, x_j * largest prefill time].  If
// its ends differ but the prefill times are so close that (x_j + 1) * least > x_j * largest, the scaled
// lengths above x_j lie above the bracket and those below it below: the percentile is x_j times the
// prefill time that ranks (j - number of lengths above x_j) among the ticks weighted by their number of
// lengths equal to x_j.  Otherwise the bracket is bisected: a probe value v is ranked in every tick's list
// (binary search on the scaled entries), and either at least j scaled entries are >= v, then the least
// of them is a new lower end, or fewer, then the largest one below v is a new upper end.  Both ends are
// values of the lists from then on, so the search ends with the percentile itself.
// LDS: [load grid] [reciprocal spacings] [SINGLE: grid point per bucket] [strip NT x n_tick]
//      [per tick: load] [per tick: count] [per tick: entries listed] [per tick: entries equal to x_j]
//      [per tick: start of its list, then two words] [the cell's lists when they fit] [bucket index]
template <bool SINGLE, bool TWO>
__global__ __launch_bounds__(DYN_MAX_TILE) void tick_general_kernel(TickArgs a) {
  extern __shared__ double smem[];
  const SpaceArgs& sa = a.s;
  const int n_rho = sa.n_rho, T = a.n_tick;
  const int tid = threadIdx.x, NT = blockDim.x;
  // The table rows stay in global memory (they are read through the caches): consecutive items of a block belong to
  // different classes, and staging a class's rows per item cost more than the look-ups of the item.
  double* s_rgp = smem;
  double* s_rinv = s_rgp + (n_rho + 2);
  double* s_thr = s_rinv + (n_rho + 1);
  double* s_strip = s_thr + (SINGLE ? sa.n_bucket + 1 : 0);     // [T][NT]
  double* s_load = s_strip + (size_t)T * NT;                    // [T]
  int32_t* s_cnt = (int32_t*)(s_load + T);                      // [T]
  int32_t* s_len = s_cnt + T;                                   // [T] min(j, count)
  int32_t* s_neq = s_len + T;                                   // [T] listed lengths equal to x_j
  uint32_t* s_lbase = (uint32_t*)(s_neq + T);                   // [T] start of the tick's list; [T]: entries staged in LDS + 1, or 0; [T+1]: lengths above x_j
  uint32_t* s_goff = s_lbase + T + 2;                           // [T] start of the tick's list in global memory
  int32_t* s_lists = (int32_t*)(s_goff + T);                    // [kListCap]
  uint16_t* s_js = (uint16_t*)(s_lists + kListCap);             // [n_bucket + 1]

  const uint64_t n_item = (uint64_t)a.counters[1] * (uint64_t)sa.n_tile;   // complete: written by the cell kernel
  if (blockIdx.x >= n_item) return;                              // block-uniform
  stage_grid<SINGLE>(a, s_rgp, s_thr, s_js);
  for (uint64_t item = blockIdx.x; item < n_item; item += gridDim.x) {
    const size_t cell = a.slow_list[item / (uint64_t)sa.n_tile];
    const int tile = (int)(item % (uint64_t)sa.n_tile);
    const int g = (int)(cell % sa.G);
    __syncthreads();                           // the previous item's LDS data has been consumed
    const TickPlan pl = a.plan[cell];
    const int j = pl.j;
    const bool dense = (pl.flags & DYN_TP_DENSE) != 0;
    const bool tight = (pl.flags & DYN_TP_TIGHT) != 0;   // no lists: per tick the number of requests of length x_j, and the rank among them
    const bool raw = (pl.flags & DYN_TP_RAW) != 0;       // the lists are whole ticks; a tick marked DYN_TICK_PIECES is sorted in pieces of DYN_TICK_DEPTH
    const TickRec* rec = a.rec + cell * T;
    if (tid < DYN_WAVE) {                      // the first wave, a tick per lane: where each tick's list is read from
      TickRec r;
      r.load = 0.0; r.off = 0u; r.cnt = 0;
      if (tid < T) r = rec[tid];
      const bool pieces = raw && (r.off & DYN_TICK_PIECES) != 0u;
      const uint32_t off = raw ? (r.off & ~DYN_TICK_PIECES) : r.off;
      const int len = (tid < T && !tight) ? (raw ? r.cnt : min(r.cnt, j)) : 0;
      int incl = len;                          // inclusive prefix over the ticks
#pragma unroll
      for (int d = 1; d < DYN_WAVE; d <<= 1) {
        const int up = __shfl_up(incl, d, DYN_WAVE);
        if (tid >= d) incl += up;
      }
      const uint32_t total = (uint32_t)__builtin_amdgcn_readlane(incl, DYN_WAVE - 1);
      const bool fits = !raw && total <= (uint32_t)kListCap;
      if (tid < T) {
        s_load[tid] = r.load;
        s_cnt[tid] = r.cnt;
        s_len[tid] = pieces ? -len : len;        // negative: a long tick whose list is sorted piece by piece
        s_goff[tid] = off;
        s_lbase[tid] = fits ? (uint32_t)(incl - len) : off;
        if (tight) s_neq[tid] = (int32_t)r.off;
      }
      if (tid == 0) {
        s_lbase[T] = fits ? total + 1u : 0u;   // 0: the lists stay in global memory
        s_lbase[T + 1] = 0u;
      }
    }
    __syncthreads();
    const bool staged = s_lbase[T] != 0u;
    if (staged) {                              // one flat copy: the loads of all ticks are in flight together
      const int total = (int)s_lbase[T] - 1;
#pragma unroll 4
      for (int i = tid; i < total; i += NT) {
        int l = 0, h = T - 1;                  // the tick whose list holds entry i: the last q with s_lbase[q] <= i
        while (l < h) {
          const int mid = (l + h + 1) >> 1;
          if ((int)s_lbase[mid] <= i) l = mid; else h = mid - 1;
        }
        s_lists[i] = a.top[(size_t)s_goff[l] + (uint32_t)(i - (int)s_lbase[l])];
      }
      __syncthreads();
    }
    const int32_t* lists = staged ? s_lists : a.top;
    if (tid < T && !tight && s_len[tid] < 0) s_neq[tid] = 0;
    if (tid < T && !tight && s_len[tid] >= 0) {        // per tick: listed lengths above x_j and equal to it (the list is descending)
      const int len = s_len[tid];
      const int32_t* lq = lists + s_lbase[tid];
      int l = 0, h = len;                      // first entry <= x_j
      while (l < h) {
        const int mid = (l + h) >> 1;
        if (lq[mid] > pl.xj) l = mid + 1; else h = mid;
      }
      const int n_gt = l;
      h = len;                                 // first entry < x_j
      while (l < h) {
        const int mid = (l + h) >> 1;
        if (lq[mid] >= pl.xj) l = mid + 1; else h = mid;
      }
      s_neq[tid] = l - n_gt;
      if (n_gt) atomicAdd(&s_lbase[T + 1], (uint32_t)n_gt);
    }
    if (raw) {                                 // block-uniform: the same two counts of the ticks sorted in pieces, by the whole block (from the trace)
      __syncthreads();
      for (int q = 0; q < T; ++q) {
        const int len = -s_len[q];
        if (len <= 0) continue;
        const int32_t* lq = a.in + s_lbase[q];
        uint32_t n_gt = 0;
        int32_t n_eq = 0;
        for (int i = tid; i < len; i += NT) {
          const int32_t x = lq[i];
          n_gt += x > pl.xj ? 1u : 0u;
          n_eq += x == pl.xj ? 1 : 0;
        }
        if (n_gt) atomicAdd(&s_lbase[T + 1], n_gt);
        if (n_eq) atomicAdd(&s_neq[q], n_eq);
      }
    }
    __syncthreads();
    const double xj = (double)pl.xj;
    const int need_eq = tight ? (int)pl.place : j - (int)s_lbase[T + 1];   // >= 1: fewer than j lengths lie above the j-th largest

    for (int sub = 0; sub < sa.tile; sub += NT) {
      const bool in_tile = sub + (tid & ~(DYN_WAVE - 1)) < sa.tile;   // wave-uniform: a wave past the tile's end stores nothing
      CfgState st;
      load_config<false>(a, g, tile * sa.tile + (in_tile ? sub + tid : 0), nullptr, s_rgp, s_rinv, s_thr, s_js, &st);
      double e = 0.0, pf_min = __builtin_inf(), pf_max = -__builtin_inf(), tb_max = -__builtin_inf();
      bool ov = false;
      const double e_idle = (st.nd * idle_power<TWO>(st.L)) * a.tick_s;
      for (int q = 0; q < T; ++q) {            // energy in time order; the strip takes the prefill times, or first the TBTs
        if (s_cnt[q] == 0) {                   // block-uniform: load 0, and nothing of this tick enters a percentile
          e += e_idle;
          continue;
        }
        double pf, tb, pw;
        ov = table_lookup<SINGLE, TWO>(st.L, s_load[q], &pf, &tb, &pw) | ov;
        e += (st.nd * pw) * a.tick_s;
        s_strip[q * NT + tid] = dense ? pf : tb;
        pf_min = min_num(pf_min, pf);
        pf_max = max_num(pf_max, pf);
        tb_max = max_num(tb_max, tb);
      }
      double p_tbt = tb_max;
      if (!dense) {                            // block-uniform
        p_tbt = weighted_from_top(s_strip, s_cnt, T, NT, j, tid);
        for (int q = 0; q < T; ++q) {
          if (s_cnt[q] == 0) continue;
          double pf, tb, pw;
          table_lookup<SINGLE, TWO>(st.L, s_load[q], &pf, &tb, &pw);
          s_strip[q * NT + tid] = pf;
        }
      }
      // TTFT percentile
      double lo = xj * pf_min, hi = xj * pf_max;
      bool open = lo != hi;
      if (tight || (open && xj * pf_max < (xj + 0.5) * pf_min)) {
        // only lengths equal to x_j scale into the bracket: rank the ticks' prefill times by those
        lo = hi = xj * weighted_from_top(s_strip, s_neq, T, NT, need_eq, tid);
        open = false;
      }
      while (open) {
        double v = lo + (hi - lo) * 0.5;
        if (!(v > lo)) v = hi;
        int n_ge = 0;
        double a_min = __builtin_inf(), b_max = -__builtin_inf();
        for (int q = 0; q < T; ++q) {
          int len = s_len[q];
          if (len == 0) continue;
          const double pf = s_strip[q * NT + tid];
          const int32_t* lq = lists + s_lbase[q];
          if (len < 0) {                       // block-uniform: a long tick, sorted piece by piece
            len = -len;
            for (int base = 0; base < len; base += DYN_TICK_DEPTH) {
              const int n = len - base < DYN_TICK_DEPTH ? len - base : DYN_TICK_DEPTH;
              const int32_t* lp = lq + base;
              int l = 0, h = n;                // entries [0, l) of the piece are >= v scaled, entries [h, n) are below
              while (l < h) {
                const int mid = (l + h) >> 1;
                const bool ge = (double)lp[mid] * pf >= v;
                l = ge ? mid + 1 : l;
                h = ge ? h : mid;
              }
              n_ge += l;
              if (l > 0) a_min = min_num(a_min, (double)lp[l - 1] * pf);
              if (l < n) b_max = max_num(b_max, (double)lp[l] * pf);
            }
            continue;
          }
          int l = 0, h = len;                  // entries [0, l) are >= v scaled, entries [h, len) are below
          while (l < h) {
            const int mid = (l + h) >> 1;
            const bool ge = (double)lq[mid] * pf >= v;
            l = ge ? mid + 1 : l;
            h = ge ? h : mid;
          }
          n_ge += l;
          if (l > 0) a_min = min_num(a_min, (double)lq[l - 1] * pf);
          if (l < len) b_max = max_num(b_max, (double)lq[l] * pf);
        }
        if (n_ge >= j) lo = a_min; else hi = b_max;
        open = lo < hi;                        // also ends a search that lost its bracket (never with consistent lists)
      }
      if (in_tile) emit_cell(sa, st, cell, false, ov, e, lo, p_tbt);
      __syncthreads();                         // the strip is rewritten by the next group of configurations
    }
  }
}

size_t tick_lds_tail(int32_t n_rho, int32_t n_bucket, int32_t n_tick, int32_t win_per_block, bool single) {
  return (size_t)(2 * n_rho + 3) * sizeof(double) + (single ? ((size_t)n_bucket + 1) * sizeof(double) : 0) +
         2 * sizeof(double) + (size_t)win_per_block * (n_tick * (sizeof(double) + 2 * sizeof(int32_t)) + sizeof(TickPlan)) +
         (size_t)2 * n_tick * kFastDepth * sizeof(int32_t) + ((size_t)n_bucket + 1) * sizeof(uint16_t) + 8;
}
size_t tight_lds_tail(int32_t n_rho, int32_t n_bucket, int32_t n_tick, int32_t win_per_block, bool single) {
  return (size_t)(2 * n_rho + 3) * sizeof(double) + (single ? ((size_t)n_bucket + 1) * sizeof(double) : 0) +
         (size_t)win_per_block * (n_tick * (sizeof(double) + 2 * sizeof(int32_t)) + sizeof(TickPlan)) +
         ((size_t)n_bucket + 1) * sizeof(uint16_t) + 8;
}
size_t general_lds_tail(int32_t n_rho, int32_t n_bucket, int32_t n_tick, int nt, bool single) {
  return (size_t)(2 * n_rho + 3) * sizeof(double) + (single ? ((size_t)n_bucket + 1) * sizeof(double) : 0) +
         (size_t)n_tick * nt * sizeof(double) + (size_t)n_tick * (sizeof(double) + 5 * sizeof(int32_t)) +
         2 * sizeof(uint32_t) + (size_t)kListCap * sizeof(int32_t) + ((size_t)n_bucket + 1) * sizeof(uint16_t) + 8;
}
// Threads of a block of the general kernel: the tile's width, less where the strip (one double per tick and
// thread) would pass 32 KB.
int general_threads(const TickArgs& a) {
  const int cap = a.n_tick <= 16 ? 256 : (a.n_tick <= 32 ? 128 : 64);
  return a.s.tile < cap ? a.s.tile : cap;
}
static_assert(256 * 16 * sizeof(double) <= kStripBytes && 128 * 32 * sizeof(double) <= kStripBytes &&
                  64 * DYN_TICK_MAX * sizeof(double) <= kStripBytes,
              "the strip of the general kernel");

template <bool LDS, bool SINGLE, bool TWO>
void launch_tight_walk(const TickArgs& a, dim3 grid, dim3 block, size_t lds, hipStream_t s) {
  hipLaunchKernelGGL((tick_tight_walk_kernel<LDS, SINGLE, TWO>), grid, block, lds, s, a);
}
template <bool LDS, bool SINGLE, bool TWO>
void launch_space(const TickArgs& a, dim3 grid, dim3 block, size_t lds, hipStream_t s) {
  if (a.n_tick <= 16) hipLaunchKernelGGL((tick_space_kernel<16, LDS, SINGLE, TWO>), grid, block, lds, s, a);
  else hipLaunchKernelGGL((tick_space_kernel<DYN_TICK_MAX, LDS, SINGLE, TWO>), grid, block, lds, s, a);
}
template <bool SINGLE, bool TWO>
void launch_general(const TickArgs& a, size_t lds, hipStream_t s) {
  DynTimed timed(DYN_K_TICK_MERGE, s);
  // The items are dealt round-robin to the grid: as many blocks as the device holds at once, so that none starts late.
  const int nt = general_threads(a);
  int per_cu = 0, blocks = kGeneralBlocks;
  if (a.n_cu > 0 && hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, tick_general_kernel<SINGLE, TWO>, nt, lds) == hipSuccess &&
      per_cu > 0)
    blocks = per_cu * a.n_cu;
  hipLaunchKernelGGL((tick_general_kernel<SINGLE, TWO>), dim3(blocks), dim3(nt), lds, s, a);
}

template <typename F>
void dispatch(bool lds, bool single, bool two, F&& f) {
  if (lds) {
    if (single) { if (two) f(std::true_type(), std::true_type(), std::true_type()); else f(std::true_type(), std::true_type(), std::false_type()); }
    else { if (two) f(std::true_type(), std::false_type(), std::true_type()); else f(std::true_type(), std::false_type(), std::false_type()); }
  } else {
    if (single) { if (two) f(std::false_type(), std::true_type(), std::true_type()); else f(std::false_type(), std::true_type(), std::false_type()); }
    else { if (two) f(std::false_type(), std::false_type(), std::true_type()); else f(std::false_type(), std::false_type(), std::false_type()); }
  }
}

}  // namespace

hipError_t dyn_launch_tick_cell(const TickCellArgs& a, hipStream_t s) {
  const int64_t cells = (int64_t)a.n_window * a.G;
  const int64_t blocks = (cells + kWavesPerBlock - 1) / kWavesPerBlock;
  DynTimed timed(DYN_K_TICK_TOP, s);
  hipLaunchKernelGGL(tick_init_kernel, dim3(1), dim3(1), 0, s, a.counters);
  hipLaunchKernelGGL(tick_tight_kernel, dim3((unsigned)blocks), dim3(kWavesPerBlock * DYN_WAVE), 0, s, a);
  hipLaunchKernelGGL(tick_tight_block_kernel, dim3(kTightBlocks), dim3(kWavesPerBlock * DYN_WAVE), 0, s, a);
  hipLaunchKernelGGL(tick_cell_kernel, dim3((unsigned)blocks), dim3(kWavesPerBlock * DYN_WAVE), 0, s, a);
  hipLaunchKernelGGL(tick_deep_kernel, dim3(kDeepBlocks), dim3(256), 0, s, a);
  return hipGetLastError();
}

// Windows a block of the evaluation kernel walks: as for the window-level kernel, less where the per-tick
// records of that many windows would not fit beside the table rows.
int32_t dyn_tick_win_per_block(const TickArgs& a, int32_t wanted) {
  const SpaceArgs& sa = a.s;
  const size_t tab = (size_t)sa.n_slot * DYN_SLOT_STRIDE(sa.n_rho) * sizeof(double);
  int32_t wpb = wanted;
  while (wpb > 1 && tab + tick_lds_tail(sa.n_rho, sa.n_bucket, a.n_tick, wpb, a.single_point) > DYN_LDS_BUDGET) wpb /= 2;
  return wpb;
}

hipError_t dyn_launch_tick_space(const TickArgs& a_in, hipStream_t s) {
  TickArgs a = a_in;
  SpaceArgs& sa = a.s;
  sa.win_per_block = dyn_tick_win_per_block(a, sa.win_per_block);
  const int n_chunk = (sa.n_window + sa.win_per_block - 1) / sa.win_per_block;
  const dim3 grid((unsigned)((size_t)n_chunk * sa.G * sa.n_tile)), block(sa.tile);
  const size_t tab = (size_t)sa.n_slot * DYN_SLOT_STRIDE(sa.n_rho) * sizeof(double);
  // Preferences when LDS is short: keep the table rows in LDS first, the per-bucket grid
  // points second (without them the bracket is searched; without the rows the tables are
  // read from global memory).
  {
    DynTimed timed(DYN_K_TICK_SPACE, s);         // both walks
    {
    bool single = a.single_point;
    size_t tail = tight_lds_tail(sa.n_rho, sa.n_bucket, a.n_tick, sa.win_per_block, single);
    if (single && tail + tab > DYN_LDS_BUDGET) {
      single = false;
      tail = tight_lds_tail(sa.n_rho, sa.n_bucket, a.n_tick, sa.win_per_block, false);
    }
    const bool lds = sa.n_slot > 0 && tab + tail <= DYN_LDS_BUDGET;
    if (!lds && tail > DYN_LDS_BUDGET) return hipErrorInvalidValue;
    const size_t bytes = (lds ? tab : 0) + tail;
    dispatch(lds, single, a.any_two_rows, [&](auto L, auto S, auto W) {
      launch_tight_walk<decltype(L)::value, decltype(S)::value, decltype(W)::value>(a, grid, block, bytes, s);
    });
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  {
    bool single = a.single_point;
    size_t tail = tick_lds_tail(sa.n_rho, sa.n_bucket, a.n_tick, sa.win_per_block, single);
    if (single && tail + tab > DYN_LDS_BUDGET) {
      single = false;
      tail = tick_lds_tail(sa.n_rho, sa.n_bucket, a.n_tick, sa.win_per_block, false);
    }
    const bool lds = sa.n_slot > 0 && tab + tail <= DYN_LDS_BUDGET;
    if (!lds && tail > DYN_LDS_BUDGET) return hipErrorInvalidValue;
    const size_t bytes = (lds ? tab : 0) + tail;
    dispatch(lds, single, a.any_two_rows, [&](auto L, auto S, auto W) {
      launch_space<decltype(L)::value, decltype(S)::value, decltype(W)::value>(a, grid, block, bytes, s);
    });
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  }
  {
    const int nt = general_threads(a);
    bool single = a.single_point;
    size_t tail = general_lds_tail(sa.n_rho, sa.n_bucket, a.n_tick, nt, single);
    if (single && tail > DYN_LDS_BUDGET) {
      single = false;
      tail = general_lds_tail(sa.n_rho, sa.n_bucket, a.n_tick, nt, false);
    }
    if (tail > DYN_LDS_BUDGET) return hipErrorInvalidValue;
    dispatch(false, single, a.any_two_rows, [&](auto, auto S, auto W) {
      launch_general<decltype(S)::value, decltype(W)::value>(a, tail, s);
    });
  }
  return hipGetLastError();
}
