// Per-cell aggregation and rank selection: one wavefront per (window, class) cell streams
// the cell's requests once and produces the exact token sums (the class's load in the
// window, Section III-A "Request loads") and the input length of nearest rank
// ceil(pct*m) (the request whose TTFT is the cell's P99 under every configuration, since
// per-request TTFT = input tokens x a non-negative per-(cell, configuration) factor and
// IEEE multiplication by a non-negative constant is monotone).
//
// Cells of up to 2048 requests are held in registers (32 values per lane at most) and the
// selection is a most-significant-bit-first search on the value: for every bit one
// compare per register row and a scalar population count of the wave mask, no LDS and no
// cross-lane traffic.  The search interval is first narrowed to [lo, max], where lo is the
// j-th largest of the 64 per-lane maxima (j = m - rank + 1; those maxima are elements of
// the cell, so the j-th largest element cannot be below it): for a high percentile only a
// few bits are left.  Larger cells are streamed from global memory by the whole block,
// once for the sums and once per 10-bit digit, through an LDS histogram (radix select).
#include "dyn_device.h"

namespace {

constexpr int kWavesPerBlock = 4;
constexpr int kHistBits = 10;
constexpr int kHistBins = 1 << kHistBits;
constexpr int kRegRowsMax = 32;  // register path handles m <= 64 * kRegRowsMax

struct CellOut {
  int64_t tin, tout;
  uint32_t p99;
  uint32_t orv;
};

// Exact token sums of a register-sized cell the slow way (16-bit halves keep every partial
// sum inside 32 bits: at most 32 values per lane, 2048 per wave); only needed when a token
// count of 2^20 or more makes plain 32-bit sums unsafe.
__device__ __forceinline__ void cell_sums_wide(const int32_t* __restrict__ in, const int32_t* __restrict__ out,
                                               int64_t beg, int m, int lane, int64_t* tin, int64_t* tout) {
  int lo_in = 0, hi_in = 0, lo_out = 0, hi_out = 0;
#pragma unroll 1
  for (int idx = lane; idx < m; idx += DYN_WAVE) {
    const int a = in[beg + idx];
    const int b = out[beg + idx];
    lo_in += a & 0xFFFF;
    hi_in += a >> 16;
    lo_out += b & 0xFFFF;
    hi_out += b >> 16;
  }
  *tin = ((int64_t)wave_sum_i32(hi_in) << 16) + (int64_t)wave_sum_i32(lo_in);
  *tout = ((int64_t)wave_sum_i32(hi_out) << 16) + (int64_t)wave_sum_i32(lo_out);
}

// Reduction of a register-resident cell of m <= 64*R requests: v[i] = input tokens of request
// i*64 + lane (0xFFFFFFFF beyond m); s_in / s_out / or_all / lmax = the lane's sums, OR and
// largest input over its requests.
template <int R>
__device__ __forceinline__ CellOut cell_reduce(const uint32_t (&v)[R], uint32_t s_in, uint32_t s_out, uint32_t or_all,
                                               uint32_t lmax, const int32_t* __restrict__ in,
                                               const int32_t* __restrict__ out, int64_t beg, int m, int rank, int lane) {
  CellOut r;
  r.orv = wave_or_u32(or_all);
  // at most 2048 values: if all are below 2^20 the 32-bit sums are exact (else redone below)
  r.tin = (int64_t)(uint32_t)wave_sum_i32((int)s_in);
  r.tout = (int64_t)(uint32_t)wave_sum_i32((int)s_out);
  // Answer = largest a with #{v < a} < rank.  It lies in [lo, top]: top = largest element,
  // lo = 0, or for cells of several rows the j-th largest per-lane maximum, j = m - rank + 1.
  const uint32_t top = wave_max_u32(lmax);
  if (rank == m) {                          // the nearest rank of a small cell is its last: the maximum
    r.p99 = top;
  } else {
    uint32_t lo = 0;
    if (R >= 4) {
      const int j = m - rank + 1;
      if (j <= DYN_WAVE) {
        const int nb = 32 - __builtin_clz(top | 1u);
        for (int b = nb - 1; b >= 0; --b) {   // largest c with #{lane maxima >= c} >= j
          const uint32_t cand = lo | (1u << b);
          if (__popcll(__ballot(lmax >= cand)) >= j) lo = cand;
        }
      }
    }
    uint32_t d = 0;
    const int nb = 32 - __builtin_clz((top - lo) | 1u);
    for (int b = nb - 1; b >= 0; --b) {
      const uint32_t cand = lo + (d | (1u << b));
      int below = 0;
#pragma unroll
      for (int i = 0; i < R; ++i) below += __popcll(__ballot(v[i] < cand));
      if (below < rank) d |= 1u << b;
    }
    r.p99 = lo + d;
  }
  if (r.orv >= (1u << 20)) cell_sums_wide(in, out, beg, m, lane, &r.tin, &r.tout);
  return r;
}

// Register-resident cell: m <= 64*R requests.
template <int R>
__device__ __forceinline__ CellOut cell_in_registers(const int32_t* __restrict__ in,
                                                     const int32_t* __restrict__ out, int64_t beg,
                                                     int m, int rank, int lane) {
  uint32_t v[R];
  uint32_t s_in = 0, s_out = 0, or_all = 0, lmax = 0;
#pragma unroll
  for (int i = 0; i < R; ++i) {
    const int idx = i * DYN_WAVE + lane;
    const bool ok = idx < m;
    const uint32_t a = ok ? (uint32_t)in[beg + idx] : 0u;
    const uint32_t b = ok ? (uint32_t)out[beg + idx] : 0u;
    v[i] = ok ? a : 0xFFFFFFFFu;  // padding is never below a candidate value
    or_all |= a | b;
    lmax = max(lmax, a);
    s_in += a;
    s_out += b;
  }
  return cell_reduce<R>(v, s_in, s_out, or_all, lmax, in, out, beg, m, rank, lane);
}

// Any register-sized cell (0 < mi <= 64 * kRegRowsMax) by one wave.
__device__ __forceinline__ CellOut cell_by_wave(const int32_t* __restrict__ in, const int32_t* __restrict__ out,
                                                int64_t beg, int mi, int rk, int lane) {
  if (mi <= 64 * 1) return cell_in_registers<1>(in, out, beg, mi, rk, lane);
  if (mi <= 64 * 2) return cell_in_registers<2>(in, out, beg, mi, rk, lane);
  if (mi <= 64 * 3) return cell_in_registers<3>(in, out, beg, mi, rk, lane);
  if (mi <= 64 * 4) return cell_in_registers<4>(in, out, beg, mi, rk, lane);
  if (mi <= 64 * 6) return cell_in_registers<6>(in, out, beg, mi, rk, lane);
  if (mi <= 64 * 8) return cell_in_registers<8>(in, out, beg, mi, rk, lane);
  if (mi <= 64 * 12) return cell_in_registers<12>(in, out, beg, mi, rk, lane);
  if (mi <= 64 * 16) return cell_in_registers<16>(in, out, beg, mi, rk, lane);
  if (mi <= 64 * 24) return cell_in_registers<24>(in, out, beg, mi, rk, lane);
  return cell_in_registers<32>(in, out, beg, mi, rk, lane);
}

// The threads of a group wait for each other: the whole block at a barrier; a single wave runs in lockstep and its LDS
// operations complete in program order, so only the compiler has to be kept from moving them across this point.
template <int WAVES>
__device__ __forceinline__ void group_sync() {
  if (WAVES == 1) {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
  } else {
    __syncthreads();
  }
}

// Large cell, by a group of WAVES waves (the whole block, or one wave on its own): the group streams the cell from
// global memory once for the sums and once per 10-bit digit of the selection (radix select through one LDS histogram).
// Every thread returns the same result.  `hist` (kHistBins counters) and `xch` (16 words) are LDS scratch of the
// group; the caller guarantees nobody else uses them.
template <int U, int WAVES>   // U independent loads per array in flight
__device__ __forceinline__ CellOut cell_by_group(const int32_t* __restrict__ in, const int32_t* __restrict__ out, int64_t beg,
                                 int64_t m, int64_t rank, uint32_t* hist, int64_t* xch) {
  static_assert(WAVES == 1 || WAVES == kWavesPerBlock, "one wave or the block");
  const int lane = threadIdx.x & (DYN_WAVE - 1);
  const int tid = WAVES == 1 ? lane : (int)threadIdx.x, wave = tid / DYN_WAVE;
  constexpr int nthr = WAVES * DYN_WAVE;
  int64_t sin = 0, sout = 0;
  uint32_t orv = 0;
  for (int64_t i0 = 0; i0 < m; i0 += U * nthr) {
    int a[U], b[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t i = i0 + u * nthr + tid;
      a[u] = i < m ? in[beg + i] : 0;
      b[u] = i < m ? out[beg + i] : 0;
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      sin += a[u];
      sout += b[u];
      orv |= (uint32_t)(a[u] | b[u]);
    }
  }
  sin = wave_sum_i64(sin);
  sout = wave_sum_i64(sout);
  orv = wave_or_u32(orv);
  group_sync<WAVES>();
  if (lane == 0) { xch[wave * 3 + 0] = sin; xch[wave * 3 + 1] = sout; xch[wave * 3 + 2] = (int64_t)orv; }
  group_sync<WAVES>();
  CellOut r;
  r.tin = r.tout = 0;
  r.orv = 0;
  for (int w = 0; w < WAVES; ++w) {
    r.tin += xch[w * 3 + 0];
    r.tout += xch[w * 3 + 1];
    r.orv |= (uint32_t)xch[w * 3 + 2];
  }

  int hi_bit = 32 - __builtin_clz(r.orv | 1u);  // bits >= hi_bit of the answer are `prefix`
  uint32_t prefix = 0;
  int64_t need = rank;
  while (hi_bit > 0) {
    const int w = hi_bit < kHistBits ? hi_bit : kHistBits;
    const int shift = hi_bit - w;
    const uint32_t dmask = (1u << w) - 1u;
    group_sync<WAVES>();
    for (int b = tid; b < kHistBins; b += nthr) hist[b] = 0;
    group_sync<WAVES>();
    for (int64_t i0 = 0; i0 < m; i0 += U * nthr) {
      uint32_t a[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int64_t i = i0 + u * nthr + tid;
        a[u] = i < m ? (uint32_t)in[beg + i] : 0u;
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int64_t i = i0 + u * nthr + tid;
        const bool match = i < m && (hi_bit >= 32 ? true : ((a[u] >> hi_bit) == prefix));
        if (match) atomicAdd(&hist[(a[u] >> shift) & dmask], 1u);
      }
    }
    group_sync<WAVES>();
    if (wave == 0) {
      // lane l owns bins [16 l, 16 l + 16); find the bin where the running count reaches `need`
      constexpr int per = kHistBins / DYN_WAVE;
      uint32_t cnt[per];
      int64_t mine = 0;
#pragma unroll
      for (int q = 0; q < per; ++q) {
        cnt[q] = hist[lane * per + q];
        mine += cnt[q];
      }
      int64_t incl = mine;  // inclusive scan over lanes
#pragma unroll
      for (int d = 1; d < DYN_WAVE; d <<= 1) {
        const int64_t up = __shfl_up(incl, d, DYN_WAVE);
        if (lane >= d) incl += up;
      }
      const uint64_t reach = __ballot(incl >= need);
      const int owner = reach ? __builtin_ctzll(reach) : DYN_WAVE - 1;  // reach != 0: need <= matches
      int64_t run = incl - mine;
      bool found = false;
      uint32_t digit = (uint32_t)(lane * per + per - 1);
      int64_t below = 0;
#pragma unroll
      for (int q = 0; q < per; ++q) {
        const bool hit = !found && (run + cnt[q] >= need || q == per - 1);
        if (hit) {
          digit = (uint32_t)(lane * per + q);
          below = run;
          found = true;
        }
        run += cnt[q];
      }
      if (lane == owner) { xch[12] = (int64_t)digit; xch[13] = below; }
    }
    group_sync<WAVES>();
    const uint32_t digit = (uint32_t)xch[12];
    need -= xch[13];
    prefix = (prefix << w) | digit;
    hi_bit = shift;
  }
  group_sync<WAVES>();
  r.p99 = prefix;
  return r;
}

// Register-resident cell of 2048 < m <= 128*P requests by one wave: two 16-bit input lengths to a register (request
// i*64 + lane in half i%2 of register i/2; 0xFFFF beyond m).  Same sums and the same search as above.  Returns false,
// and nothing else, when a token count of 2^16 or more (a negative one included) rules the packing out: the caller
// streams the cell instead.
constexpr int kPackedRowsMax = 128;  // the packed path handles m <= 64 * kPackedRowsMax
template <int P>
__device__ __forceinline__ bool cell_in_registers_packed(const int32_t* __restrict__ in, const int32_t* __restrict__ out,
                                                         int m, int rank, int lane, CellOut* res) {
  uint32_t v[P];
  uint32_t s_in = 0, s_out = 0, orv = 0, lmax = 0, lmax2 = 0;   // lmax / lmax2: largest input of the even / odd rows
  constexpr int CH = 4;                  // registers per round: 8 + 8 loads in flight
  static_assert(P % CH == 0, "whole rounds");
#pragma unroll
  for (int p0 = 0; p0 < P; p0 += CH) {
    uint32_t a[2 * CH], b[2 * CH];
#pragma unroll
    for (int u = 0; u < 2 * CH; ++u) {
      const int idx = (2 * p0 + u) * DYN_WAVE + lane;
      a[u] = idx < m ? (uint32_t)in[idx] : 0u;
      b[u] = idx < m ? (uint32_t)out[idx] : 0u;
    }
#pragma unroll
    for (int u = 0; u < 2 * CH; ++u) {
      s_in += a[u];
      s_out += b[u];
      orv |= a[u] | b[u];
      if (u % 2 == 0) lmax = max(lmax, a[u]);
      else lmax2 = max(lmax2, a[u]);
    }
#pragma unroll
    for (int u = 0; u < CH; ++u) {
      const int idx = (2 * (p0 + u)) * DYN_WAVE + lane;
      const uint32_t x0 = idx < m ? a[2 * u] & 0xFFFFu : 0xFFFFu;
      const uint32_t x1 = idx + DYN_WAVE < m ? a[2 * u + 1] & 0xFFFFu : 0xFFFFu;
      v[p0 + u] = x0 | (x1 << 16);
    }
    // keep the rounds apart (the next round's loads after this round's arithmetic): with all loads hoisted to the
    // top, or the arithmetic sunk to the end, 4P loaded values would be live at once
    asm volatile("" : "+v"(s_in), "+v"(s_out), "+v"(orv), "+v"(lmax), "+v"(lmax2), "+v"(v[p0]), "+v"(v[p0 + 1]),
                 "+v"(v[p0 + 2]), "+v"(v[p0 + 3])::"memory");
  }
  orv = wave_or_u32(orv);
  if (orv >= (1u << 16)) return false;   // uniform over the wave
  // all values below 2^16: a lane's sum stays below 2^23, the wave's below 2^29
  res->orv = orv;
  res->tin = (int64_t)wave_sum_u32(s_in);
  res->tout = (int64_t)wave_sum_u32(s_out);
  const uint32_t top = wave_max_u32(max(lmax, lmax2));
  if (top == 0xFFFFu) return false;      // the padding value; and the search's candidates (up to top + 1) must fit 16 bits
  if (rank == m) {
    res->p99 = top;
    return true;
  }
  uint32_t lo = 0;
  const int j = m - rank + 1;
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
    // low half by a 16-bit compare; high half: hi < cand exactly when the whole register < cand << 16 (no unpacking,
    // which the compiler would otherwise hoist out of this loop into 2P registers)
    const uint16_t cand_lo = (uint16_t)cand;
    const uint32_t cand_hi = cand << 16;
    int below = 0;
#pragma unroll
    for (int i = 0; i < P; ++i)
      below += __popcll(__ballot((uint16_t)v[i] < cand_lo)) + __popcll(__ballot(v[i] < cand_hi));
    if (below < rank) d |= 1u << b;
  }
  res->p99 = lo + d;
  return true;
}

__device__ __forceinline__ bool cell_by_wave_packed(const int32_t* __restrict__ in, const int32_t* __restrict__ out,
                                                    int mi, int rk, int lane, CellOut* res) {
  if (mi <= 128 * 24) return cell_in_registers_packed<24>(in, out, mi, rk, lane, res);
  if (mi <= 128 * 32) return cell_in_registers_packed<32>(in, out, mi, rk, lane, res);
  if (mi <= 128 * 48) return cell_in_registers_packed<48>(in, out, mi, rk, lane, res);
  return cell_in_registers_packed<64>(in, out, mi, rk, lane, res);
}

__device__ __forceinline__ void write_cell(int64_t c, const CellOut& r, int64_t m, uint32_t bad, double window_s,
                                           double r_window,
                                           int64_t cells, int64_t* __restrict__ tin, int64_t* __restrict__ tout,
                                           int32_t* __restrict__ in_p99, CellRec* __restrict__ rec,
                                           uint8_t* __restrict__ cstat, WsHeader* __restrict__ header) {
  tin[c] = r.tin;
  tout[c] = r.tout;
  in_p99[c] = (int32_t)r.p99;
  CellRec cr;
  cr.load = div_by((double)(r.tin + r.tout), window_s, r_window);   // tokens / window_s, r_window = RN(1 / window_s)
  cr.xp99 = (double)(int32_t)r.p99;
  cr.nonempty = m > 0 ? 1.0 : 0.0;
  cr.pad = 0.0;
  rec[c] = cr;
  cstat[c] = (uint8_t)bad;       // every cell writes its own byte: nothing to clear beforehand
  if (c == 0) {                  // single writer of the header
    header->status = 0u;
    header->kind = DYN_WS_KIND_CELLS;
    header->cells = cells;
  }
}

// Four consecutive cells per block, one wave each; cells beyond the register tiers are then
// taken one after the other by the whole block.
__global__ __launch_bounds__(kWavesPerBlock* DYN_WAVE) __attribute__((amdgpu_waves_per_eu(6, 8))) void cell_aggregate_kernel(
    const int32_t* __restrict__ in, const int32_t* __restrict__ out,
    const int64_t* __restrict__ cell_off, int64_t n_req, int64_t cells, double window_s, double r_window,
    int32_t pct_num, int32_t pct_den, int64_t* __restrict__ tin, int64_t* __restrict__ tout,
    int32_t* __restrict__ in_p99, CellRec* __restrict__ rec, uint8_t* __restrict__ cstat,
    WsHeader* __restrict__ header) {
  __shared__ uint32_t s_hist[kWavesPerBlock][kHistBins];
  __shared__ int64_t s_xch[kWavesPerBlock][16];
  const int lane = threadIdx.x & (DYN_WAVE - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / DYN_WAVE);
  const int64_t c0 = (int64_t)blockIdx.x * kWavesPerBlock;
  // lane q of every wave holds offset q of the block's cells (kWavesPerBlock + 1 of them)
  const int nc = (int)(cells - c0 < kWavesPerBlock ? cells - c0 : kWavesPerBlock);
  const int64_t myoff = lane <= nc ? cell_off[c0 + lane] : 0;
  const int64_t nxoff = __shfl_down(myoff, 1, DYN_WAVE);
  const bool sound = lane < nc && myoff >= 0 && nxoff >= myoff && nxoff <= n_req;
  // cells of this block left to the whole block, and cells beyond the plain register tiers that a wave takes with
  // packed registers (both uniform over the block)
  const uint32_t big_mask = (uint32_t)__ballot(sound && nxoff - myoff > DYN_WAVE * kPackedRowsMax);
  const uint32_t packed_mask = (uint32_t)__ballot(sound && nxoff - myoff > DYN_WAVE * kRegRowsMax &&
                                                  nxoff - myoff <= DYN_WAVE * kPackedRowsMax);
  if (wave < nc && !((big_mask >> wave) & 1u)) {
    const int64_t c = c0 + wave;
    int64_t beg = readlane_i64(myoff, wave), end = readlane_i64(nxoff, wave);
    // the status lives in a scalar register while the cell is reduced (a vector register would be spilled)
    uint32_t bad = __builtin_amdgcn_readfirstlane((beg < 0 || end < beg || end > n_req) ? DYN_WS_BAD_OFFSETS : 0u);
    asm volatile("" : "+s"(bad));
    if (bad) beg = end = 0;   // never read outside the trace
    const int mi = (int)(end - beg);
    CellOut r;
    r.tin = r.tout = 0;
    r.p99 = 0;
    r.orv = 0;
    if (mi > 0) {
      const int rk = (int)(((int64_t)pct_num * mi + pct_den - 1) / pct_den);
      if ((packed_mask >> wave) & 1u) {
        // values the packing cannot hold: the wave streams its cell on its own (its own histogram; no other wave waits)
        if (!cell_by_wave_packed(in + beg, out + beg, mi, rk, lane, &r))
          r = cell_by_group<8, 1>(in, out, beg, mi, rk, s_hist[wave], s_xch[wave]);
      } else {
        r = cell_by_wave(in, out, beg, mi, rk, lane);
      }
      asm volatile("" : "+s"(bad));
      if (r.orv >> 31) bad |= DYN_WS_BAD_REQUEST;  // a negative token count
    }
    if (lane == 0) write_cell(c, r, mi, bad, window_s, r_window, cells, tin, tout, in_p99, rec, cstat, header);
  }
  if (big_mask == 0) return;   // uniform over the block
  for (int q = 0; q < kWavesPerBlock; ++q) {
    if (!((big_mask >> q) & 1u)) continue;
    const int64_t beg = cell_off[c0 + q];          // read again (the mask vouches for them): nothing is kept in
    const int64_t m = cell_off[c0 + q + 1] - beg;  // registers across the waves' own cells
    const int64_t rank = ((int64_t)pct_num * m + pct_den - 1) / pct_den;
    const CellOut r = cell_by_group<8, kWavesPerBlock>(in, out, beg, m, rank, s_hist[0], s_xch[0]);
    const uint32_t bad = (r.orv >> 31) ? DYN_WS_BAD_REQUEST : 0u;
    if (threadIdx.x == 0) write_cell(c0 + q, r, m, bad, window_s, r_window, cells, tin, tout, in_p99, rec, cstat, header);
  }
}

// Traces cut into many small cells (a tick-level view: a few dozen requests per cell).  A wave
// per cell spends its life waiting for two dependent loads and its 64 lanes reduce a handful
// of values.  Here a wave takes kTinyCells consecutive cells.  Their requests are one contiguous
// run of the trace: if it has at most kTinyCap requests the wave copies it to LDS (coalesced,
// all loads in flight at once) and kTinyLanes lanes per cell walk the cell's requests, each
// keeping sums, the OR and the two largest inputs; a quad exchange combines them.  That
// settles every cell whose nearest rank is its largest or second-largest input (any cell of
// fewer than 200 requests at the 99th percentile); the others, cells with token counts of
// 2^20 or more, and groups whose run does not fit are taken one cell at a time by the wave
// (cells beyond 64 * kRegRowsMax requests by the whole block, after a block barrier).
constexpr int kTinyCells = 16;
constexpr int kTinyLanes = DYN_WAVE / kTinyCells;
constexpr int kTinyCap = 1024;
static_assert(kTinyLanes == 4, "the quad exchange below combines four lanes");

__global__ __launch_bounds__(kWavesPerBlock* DYN_WAVE) __attribute__((amdgpu_waves_per_eu(4, 4))) void cell_aggregate_tiny_kernel(
    const int32_t* __restrict__ in, const int32_t* __restrict__ out,
    const int64_t* __restrict__ cell_off, int64_t n_req, int64_t cells, double window_s, double r_window,
    int32_t pct_num, int32_t pct_den, int64_t* __restrict__ tin, int64_t* __restrict__ tout,
    int32_t* __restrict__ in_p99, CellRec* __restrict__ rec, uint8_t* __restrict__ cstat,
    WsHeader* __restrict__ header) {
  __shared__ uint2 s_run[kWavesPerBlock][kTinyCap];
  __shared__ int64_t s_off[kWavesPerBlock][kTinyCells + 1];
  __shared__ uint32_t s_big[kWavesPerBlock];
  __shared__ uint32_t s_hist[kHistBins];
  __shared__ int64_t s_xch[16];
  const int lane = threadIdx.x & (DYN_WAVE - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / DYN_WAVE);
  const int64_t c0 = ((int64_t)blockIdx.x * kWavesPerBlock + wave) * kTinyCells;
  const int nq = cells - c0 < kTinyCells ? (int)(cells - c0 > 0 ? cells - c0 : 0) : kTinyCells;   // cells of this wave
  const int64_t myoff = (nq > 0 && lane <= nq) ? cell_off[c0 + lane] : 0;
  const int64_t nxoff = __shfl_down(myoff, 1, DYN_WAVE);
  const bool good = lane < nq && myoff >= 0 && nxoff >= myoff && nxoff <= n_req;   // never read outside the trace
  const int64_t len = good ? nxoff - myoff : 0;
  const uint32_t good_mask = (uint32_t)__ballot(good);
  const uint32_t big_mask = (uint32_t)__ballot(len > DYN_WAVE * kRegRowsMax);
  const int len32 = (int)(len > 0x7FFFFFFF ? 0x7FFFFFFF : len);
  if (lane <= kTinyCells) s_off[wave][lane] = myoff;
  if (lane == 0) s_big[wave] = big_mask;

  const int u = lane / kTinyLanes, sub = lane % kTinyLanes;   // this lane's cell of the wave, and its share of it
  CellOut mine;                                  // lane kTinyLanes * u keeps the result of cell u
  mine.tin = mine.tout = 0;
  mine.p99 = 0;
  mine.orv = 0;
  int my_m = 0;
  uint32_t my_bad = 0;
  if (nq > 0) {
    const uint32_t grp = (1u << nq) - 1u;
    const int64_t sb = readlane_i64(myoff, 0), se = readlane_i64(myoff, nq);
    if ((good_mask & grp) == grp && se - sb <= kTinyCap) {
      // every offset of the group is in order: 0 <= sb <= each cell's bounds <= se <= n_req
      const int span = (int)(se - sb);
      uint2* run = s_run[wave];
#pragma unroll 4
      for (int pos = lane; pos < span; pos += DYN_WAVE) run[pos] = make_uint2((uint32_t)in[sb + pos], (uint32_t)out[sb + pos]);
      // the run is read back by other lanes of this wave only
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      const int64_t ob = __shfl(myoff, u, DYN_WAVE), oe = __shfl(myoff, u + 1, DYN_WAVE);
      const int m = u < nq ? (int)(oe - ob) : 0;
      const int rb = u < nq ? (int)(ob - sb) : 0;
      uint32_t s_in = 0, s_out = 0, orv = 0, t1 = 0, t2 = 0;   // t1 >= t2: the two largest inputs so far
      for (int i = rb + sub; i < rb + m; i += kTinyLanes) {
        const uint2 v = run[i];
        s_in += v.x;
        s_out += v.y;
        orv |= v.x | v.y;
        t2 = max(t2, min(t1, v.x));
        t1 = max(t1, v.x);
      }
#pragma unroll
      for (int step = 0; step < 2; ++step) {     // lanes sub ^ 1, then sub ^ 2
        const uint32_t o_in = step ? (uint32_t)dpp_mov<0x4E>((int)s_in) : (uint32_t)dpp_mov<0xB1>((int)s_in);
        const uint32_t o_out = step ? (uint32_t)dpp_mov<0x4E>((int)s_out) : (uint32_t)dpp_mov<0xB1>((int)s_out);
        const uint32_t o_or = step ? (uint32_t)dpp_mov<0x4E>((int)orv) : (uint32_t)dpp_mov<0xB1>((int)orv);
        const uint32_t o1 = step ? (uint32_t)dpp_mov<0x4E>((int)t1) : (uint32_t)dpp_mov<0xB1>((int)t1);
        const uint32_t o2 = step ? (uint32_t)dpp_mov<0x4E>((int)t2) : (uint32_t)dpp_mov<0xB1>((int)t2);
        s_in += o_in;
        s_out += o_out;
        orv |= o_or;
        t2 = max(max(t2, o2), min(t1, o1));
        t1 = max(t1, o1);
      }
      // nearest rank ceil(pct * m) counted from the top: j = 1 is the largest input
      const int rk = m > 0 ? (int)(((int64_t)pct_num * m + pct_den - 1) / pct_den) : 0;
      const int j = m - rk + 1;
      // at most 1024 values: 32-bit sums are exact if all are below 2^20
      const bool again = m > 0 && (orv >= (1u << 20) || j > 2);
      mine.tin = (int64_t)s_in;
      mine.tout = (int64_t)s_out;
      mine.p99 = j == 1 ? t1 : t2;
      mine.orv = orv;
      my_m = m;
      uint64_t todo = __ballot(sub == 0 && again);
      while (todo) {                             // uniform over the wave
        const int l = __builtin_ctzll(todo);
        todo &= todo - 1;
        const int q = l / kTinyLanes;
        const int64_t beg = readlane_i64(myoff, q);
        const int mi = __builtin_amdgcn_readlane(len32, q);
        const int rk1 = (int)(((int64_t)pct_num * mi + pct_den - 1) / pct_den);
        const CellOut r = cell_by_wave(in, out, beg, mi, rk1, lane);
        if (lane == l) mine = r;
      }
      if (mine.orv >> 31) my_bad = DYN_WS_BAD_REQUEST;   // a negative token count
    } else {
#pragma unroll 1
      for (int q = 0; q < nq; ++q) {
        if ((big_mask >> q) & 1u) continue;      // uniform over the wave
        CellOut r;
        r.tin = r.tout = 0;
        r.p99 = 0;
        r.orv = 0;
        uint32_t bad = 0;
        int mi = 0;
        if (!((good_mask >> q) & 1u)) {
          bad = DYN_WS_BAD_OFFSETS;
        } else {
          const int64_t beg = readlane_i64(myoff, q);
          mi = __builtin_amdgcn_readlane(len32, q);
          if (mi > 0) {
            const int rk = (int)(((int64_t)pct_num * mi + pct_den - 1) / pct_den);
            r = cell_by_wave(in, out, beg, mi, rk, lane);
            if (r.orv >> 31) bad |= DYN_WS_BAD_REQUEST;
          }
        }
        if (lane == q * kTinyLanes) { mine = r; my_m = mi; my_bad = bad; }
      }
    }
  }
  if (sub == 0 && u < nq && !((big_mask >> u) & 1u))
    write_cell(c0 + u, mine, my_m, my_bad, window_s, r_window, cells, tin, tout, in_p99, rec, cstat, header);
  __syncthreads();             // every wave of the block arrives here: s_off and s_big are complete
  if ((s_big[0] | s_big[1] | s_big[2] | s_big[3]) == 0) return;   // uniform over the block
  static_assert(kWavesPerBlock == 4, "the line above names the block's four waves");
  for (int w = 0; w < kWavesPerBlock; ++w)
    for (int q = 0; q < kTinyCells; ++q) {
      if (!((s_big[w] >> q) & 1u)) continue;
      const int64_t beg = s_off[w][q];
      const int64_t m = s_off[w][q + 1] - beg;
      const int64_t rank = ((int64_t)pct_num * m + pct_den - 1) / pct_den;
      const CellOut r = cell_by_group<2, kWavesPerBlock>(in, out, beg, m, rank, s_hist, s_xch);
      const uint32_t bad = (r.orv >> 31) ? DYN_WS_BAD_REQUEST : 0u;
      const int64_t c = ((int64_t)blockIdx.x * kWavesPerBlock + w) * kTinyCells + q;
      if (threadIdx.x == 0) write_cell(c, r, m, bad, window_s, r_window, cells, tin, tout, in_p99, rec, cstat, header);
    }
}

}  // namespace

hipError_t dyn_launch_cell_aggregate(const int32_t* in_tok, const int32_t* out_tok,
                                     const int64_t* cell_off, int64_t n_req, int64_t cells,
                                     double window_s, int32_t pct_num, int32_t pct_den,
                                     int64_t* tin, int64_t* tout, int32_t* in_p99, CellRec* rec,
                                     uint8_t* cstat, WsHeader* header, hipStream_t s) {
  DynTimed timed(DYN_K_CELL, s);
  if (n_req / 48 <= cells) {                     // a few dozen requests per cell on average
    const int64_t per = kWavesPerBlock * kTinyCells;
    hipLaunchKernelGGL(cell_aggregate_tiny_kernel, dim3((unsigned)((cells + per - 1) / per)),
                       dim3(kWavesPerBlock * DYN_WAVE), 0, s, in_tok, out_tok, cell_off, n_req, cells, window_s,
                       1.0 / window_s, pct_num, pct_den, tin, tout, in_p99, rec, cstat, header);
    return hipGetLastError();
  }
  const int64_t blocks = (cells + kWavesPerBlock - 1) / kWavesPerBlock;
  hipLaunchKernelGGL(cell_aggregate_kernel, dim3((unsigned)blocks), dim3(kWavesPerBlock * DYN_WAVE),
                     0, s, in_tok, out_tok, cell_off, n_req, cells, window_s, 1.0 / window_s, pct_num, pct_den, tin,
                     tout, in_p99, rec, cstat, header);
  return hipGetLastError();
}
