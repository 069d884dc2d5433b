// Device-side helpers shared by the HIP sources that look the profile up per thread
// (wave reductions, exact division by a fixed divisor, the table look-up itself).
#ifndef DYN_DEVICE_H_
#define DYN_DEVICE_H_

#include "dyn_internal.h"

namespace {

template <int CTRL>
__device__ __forceinline__ int dpp_mov(int v) {
  return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xF, 0xF, false);
}
// Reductions over the 64 lanes of a fully active wave (wave-uniform result): rotations by
// 1, 2, 4, 8 inside each row of 16 lanes leave the row's result in every lane of the row, the
// four row results are then read from lanes 0, 16, 32, 48 and combined as scalars.
__device__ __forceinline__ int wave_sum_i32(int v) {
  v += dpp_mov<0x121>(v);  // row_ror:1
  v += dpp_mov<0x122>(v);  // row_ror:2
  v += dpp_mov<0x124>(v);  // row_ror:4
  v += dpp_mov<0x128>(v);  // row_ror:8
  return __builtin_amdgcn_readlane(v, 0) + __builtin_amdgcn_readlane(v, 16) +
         __builtin_amdgcn_readlane(v, 32) + __builtin_amdgcn_readlane(v, 48);
}
__device__ __forceinline__ uint32_t wave_sum_u32(uint32_t x) { return (uint32_t)wave_sum_i32((int)x); }
__device__ __forceinline__ uint32_t wave_or_u32(uint32_t x) {
  int v = (int)x;
  v |= dpp_mov<0x121>(v);
  v |= dpp_mov<0x122>(v);
  v |= dpp_mov<0x124>(v);
  v |= dpp_mov<0x128>(v);
  return (uint32_t)(__builtin_amdgcn_readlane(v, 0) | __builtin_amdgcn_readlane(v, 16) |
                    __builtin_amdgcn_readlane(v, 32) | __builtin_amdgcn_readlane(v, 48));
}
__device__ __forceinline__ int wave_max_i32(int v) {
  v = max(v, dpp_mov<0x121>(v));
  v = max(v, dpp_mov<0x122>(v));
  v = max(v, dpp_mov<0x124>(v));
  v = max(v, dpp_mov<0x128>(v));
  return max(max(__builtin_amdgcn_readlane(v, 0), __builtin_amdgcn_readlane(v, 16)),
             max(__builtin_amdgcn_readlane(v, 32), __builtin_amdgcn_readlane(v, 48)));
}
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t x) {
  x = max(x, (uint32_t)dpp_mov<0x121>((int)x));
  x = max(x, (uint32_t)dpp_mov<0x122>((int)x));
  x = max(x, (uint32_t)dpp_mov<0x124>((int)x));
  x = max(x, (uint32_t)dpp_mov<0x128>((int)x));
  const uint32_t a = (uint32_t)__builtin_amdgcn_readlane((int)x, 0), b = (uint32_t)__builtin_amdgcn_readlane((int)x, 16);
  const uint32_t c = (uint32_t)__builtin_amdgcn_readlane((int)x, 32), d = (uint32_t)__builtin_amdgcn_readlane((int)x, 48);
  return max(max(a, b), max(c, d));
}
__device__ __forceinline__ uint32_t wave_min_u32(uint32_t x) {
  x = min(x, (uint32_t)dpp_mov<0x121>((int)x));
  x = min(x, (uint32_t)dpp_mov<0x122>((int)x));
  x = min(x, (uint32_t)dpp_mov<0x124>((int)x));
  x = min(x, (uint32_t)dpp_mov<0x128>((int)x));
  const uint32_t a = (uint32_t)__builtin_amdgcn_readlane((int)x, 0), b = (uint32_t)__builtin_amdgcn_readlane((int)x, 16);
  const uint32_t c = (uint32_t)__builtin_amdgcn_readlane((int)x, 32), d = (uint32_t)__builtin_amdgcn_readlane((int)x, 48);
  return min(min(a, b), min(c, d));
}
__device__ __forceinline__ uint64_t wave_sum_u64(uint64_t x) {
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) x += __shfl_xor(x, d, DYN_WAVE);
  return __builtin_amdgcn_readfirstlane((uint32_t)x) |
         ((uint64_t)__builtin_amdgcn_readfirstlane((uint32_t)(x >> 32)) << 32);
}
__device__ __forceinline__ int64_t wave_sum_i64(int64_t v) {   // every lane ends with the total
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, DYN_WAVE);
  return v;
}
__device__ __forceinline__ int64_t readlane_i64(int64_t x, int lane) {   // lane must be wave-uniform
  const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)x, lane);
  const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)((uint64_t)x >> 32), lane);
  return (int64_t)(((uint64_t)hi << 32) | lo);
}
// a / b, correctly rounded, given rb = RN(1 / b): the one division routine of the library.
// q0 = RN(a * rb) is within 3/2 ulp of a / b; one residual step (the residual a - b*q0 is exact
// in a fused multiply-add) brings q1 within 1/2 ulp + a relative 2^-52 of it, i.e. q1 is a
// faithful rounding; for a faithful q1 and a correctly rounded reciprocal a second residual
// step returns RN(a / b) (Markstein's theorem on the final step of a Newton-Raphson division).
// Holds while nothing under- or overflows: the host keeps window lengths, capacities and grid
// spacings within [1e-100, 1e100], which leaves every operand, residual and quotient normal
// (a == 0 gives 0 exactly).
__device__ __forceinline__ double div_by(double a, double b, double rb) {
  const double q0 = a * rb;
  const double e0 = __builtin_fma(-b, q0, a);
  const double q1 = __builtin_fma(e0, rb, q0);
  const double e1 = __builtin_fma(-b, q1, a);
  return __builtin_fma(e1, rb, q1);
}

struct Lookup {          // per-thread constants of the table look-up
  double den, rden, rho_max, bucket_scale, omu, u;
  const double *lo, *hi;         // the configuration's two table rows: [3][n_rho] prefill, TBT, power
  const double *rgp, *rinv;      // padded load grid and reciprocal spacings
  const uint16_t* js;            // bucket index
  const double* thr;             // SINGLE: the grid point inside each bucket
  int n_rho;
};

// Plain v_max_f64 / v_min_f64 of two values known not to be NaN (no quieting of the operands).
__device__ __forceinline__ double max_num(double a, double b) {
  double r;
  asm("v_max_f64 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
  return r;
}
__device__ __forceinline__ double min_num(double a, double b) {
  double r;
  asm("v_min_f64 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
  return r;
}

// Tables at (f, min(rho, rho_max)) for load `load` (>= 0): the window-level kernel's arithmetic.
// SINGLE: every bucket of the load axis holds at most one interior grid point, so the bracket
// is the bucket's start index plus one comparison; otherwise the bracket is searched from the
// bucket's index.  TWO: both frequency rows are combined (weight 0 on the upper row leaves
// the lower row's value unchanged, so lanes with a profiled frequency may run it too).
template <bool SINGLE, bool TWO>
__device__ __forceinline__ bool table_lookup(const Lookup& L, double load, double* pf, double* tb, double* pw) {
  const double rho = div_by(load, L.den, L.rden);
  const bool ov = rho > L.rho_max;
  const double rc = ov ? L.rho_max : rho;
  int jj;
  if (SINGLE) {
    const int b = (int)(rc * L.bucket_scale);
    jj = (int)L.js[b] + (rc >= L.thr[b] ? 1 : 0);
  } else {
    jj = L.js[(int)(fmax(rc, 0.0) * L.bucket_scale)];
    while (jj > 0 && L.rgp[jj + 1] > rc) --jj;
    while (jj < L.n_rho - 2 && L.rgp[jj + 2] <= rc) ++jj;
  }
  const double r0 = L.rgp[jj + 1], r1 = L.rgp[jj + 2];
  const double t = div_by(rc - r0, r1 - r0, L.rinv[jj + 1]);
  const double omt = 1.0 - t;
  const int n_rho = L.n_rho;
  double x_pf = omt * L.lo[jj] + t * L.lo[jj + 1];
  double x_tb = omt * L.lo[n_rho + jj] + t * L.lo[n_rho + jj + 1];
  double x_pw = omt * L.lo[2 * n_rho + jj] + t * L.lo[2 * n_rho + jj + 1];
  if (TWO) {
    const double b_pf = omt * L.hi[jj] + t * L.hi[jj + 1];
    const double b_tb = omt * L.hi[n_rho + jj] + t * L.hi[n_rho + jj + 1];
    const double b_pw = omt * L.hi[2 * n_rho + jj] + t * L.hi[2 * n_rho + jj + 1];
    x_pf = L.omu * x_pf + L.u * b_pf;
    x_tb = L.omu * x_tb + L.u * b_tb;
    x_pw = L.omu * x_pw + L.u * b_pw;
  }
  *pf = x_pf; *tb = x_tb; *pw = x_pw;
  return ov;
}

}  // namespace

#endif  // DYN_DEVICE_H_
