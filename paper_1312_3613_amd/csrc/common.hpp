// Shared pieces of the HIP library: error plumbing, device random streams,
// Gamma draws, wave-level helpers.  gfx950 (CDNA4, wave64) only.
#pragma once

#include <hip/hip_runtime.h>

#include <cfloat>
#include <cmath>
#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <string>

#include "../../include/augur.h"

namespace augur {

// ------------------------------------------------------------------ host errors
void set_error(const char* fmt, ...);

#define AUGUR_HIP_TRY(expr)                                                              \
  do {                                                                                   \
    hipError_t e_ = (expr);                                                              \
    if (e_ != hipSuccess) {                                                              \
      ::augur::set_error("%s failed: %s (%s:%d)", #expr, hipGetErrorString(e_), __FILE__, \
                         __LINE__);                                                      \
      (void)hipGetLastError(); /* or the runtime hands it to the next caller */ \
      return AUGUR_ERR_HIP;                                                              \
    }                                                                                    \
  } while (0)

#define AUGUR_REQUIRE(cond, ...)            \
  do {                                      \
    if (!(cond)) {                          \
      ::augur::set_error(__VA_ARGS__);      \
      return AUGUR_ERR_INVALID_ARG;         \
    }                                       \
  } while (0)

// Restores the caller's current device when it goes out of scope.
struct DeviceGuard {
  int prev = -1;
  bool ok = false;
  explicit DeviceGuard(int dev) {
    if (hipGetDevice(&prev) != hipSuccess) prev = -1;
    ok = hipSetDevice(dev) == hipSuccess;
  }
  ~DeviceGuard() {
    if (prev >= 0) (void)hipSetDevice(prev);
  }
};

// ------------------------------------------------------------ random streams
enum : uint32_t {
  kStreamInitZ = 0, kStreamZ = 1, kStreamTheta = 2, kStreamPhi = 3, kStreamGmmPi = 4,
  kStreamGmmMu = 5, kStreamGmmVar = 6, kStreamMhProposal = 7, kStreamMhAccept = 8
};

struct U4 { uint32_t x, y, z, w; };

// Philox4x32 with ten rounds (Salmon, Moraes, Dror, Shaw; SC'11).  Each round
// needs two full 32x32->64 products.
__device__ __forceinline__ U4 philox10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                       uint32_t k0, uint32_t k1) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint64_t p0 = (uint64_t)0xD2511F53u * (uint64_t)c0;
    const uint64_t p1 = (uint64_t)0xCD9E8D57u * (uint64_t)c2;
    c0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
    c1 = (uint32_t)p1;
    c2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
    c3 = (uint32_t)p0;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  return U4{c0, c1, c2, c3};
}

// Block of (seed, variable index, sweep, stream, attempt).
__device__ __forceinline__ U4 random_block(uint64_t seed, uint64_t index, uint32_t sweep,
                                           uint32_t stream, uint32_t attempt) {
  return philox10((uint32_t)index, (uint32_t)(index >> 32), sweep, (stream << 24) | attempt,
                  (uint32_t)seed, (uint32_t)(seed >> 32));
}

__device__ __forceinline__ uint32_t word_of(const U4& b, uint32_t i) {
  return i == 0 ? b.x : i == 1 ? b.y : i == 2 ? b.z : b.w;
}

// 23 random bits -> odd multiple of 2^-24 in (0,1): exact in fp32.
__device__ __forceinline__ float u24(uint32_t r) {
  return (float)(2u * (r >> 9) + 1u) * 0x1p-24f;
}
// floor(u24(r) * K) in integers.
__device__ __forceinline__ int u24_times(uint32_t r, int K) {
  return (int)(((uint64_t)(2u * (r >> 9) + 1u) * (uint64_t)K) >> 24);
}
// 32 random bits -> (r + 1/2) 2^-32 in (0,1): exact in fp64.
__device__ __forceinline__ double u32d(uint32_t r) { return ((double)r + 0.5) * 0x1p-32; }

// Natural logarithm of a positive, finite, normal double (every argument on the
// draw paths is one: uniforms in [2^-33, 1), cubes of positive numbers, shape
// constants).  x = m 2^e with m in [sqrt(1/2), sqrt(2)); with s = (m-1)/(m+1),
// ln m = 2 atanh(s) = 2 s (1 + s^2/3 + s^4/5 + ...); |s| < 0.1716, so the series
// is cut after s^22 (next term below 2^-60 relative).  About 1 ulp; a third of
// the instructions of the general-purpose library routine, which dominated the
// Gamma kernels.
// 2/23, 2/21, ..., 2/3: coefficients of 2 atanh(s) / s - 2 in powers of s^2, highest first.
__constant__ double kLogSeries[11] = {2.0 / 23.0, 2.0 / 21.0, 2.0 / 19.0, 2.0 / 17.0,
                                            2.0 / 15.0, 2.0 / 13.0, 2.0 / 11.0, 2.0 / 9.0,
                                            2.0 / 7.0,  2.0 / 5.0,  2.0 / 3.0};
__device__ __forceinline__ double log_pos(double x) {
  const long long bits = __double_as_longlong(x);
  int e = (int)(bits >> 52) - 1023;
  double m = __longlong_as_double((bits & 0x000FFFFFFFFFFFFFLL) | 0x3FF0000000000000LL);  // [1, 2)
  const bool big = m > 1.4142135623730951;
  m = big ? 0.5 * m : m;
  e += big ? 1 : 0;
  const double f = m - 1.0;  // exact
  const double den = 2.0 + f;
  double r = __builtin_amdgcn_rcp(den);
  r = fma(fma(-den, r, 1.0), r, r);
  r = fma(fma(-den, r, 1.0), r, r);
  double s = f * r;
  s = fma(fma(-den, s, f), r, s);  // s = f / den, correctly rounded or next to it
  const double z = s * s;
  // Horner steps take their coefficients from scalar registers (a table in constant memory,
  // loaded once per wave) instead of materialising each 64-bit literal in vector registers on
  // every use: a tenth of the instructions of a Gamma attempt were such moves.
  double p = kLogSeries[0];
#pragma unroll
  for (int i = 1; i < 11; ++i) p = fma(p, z, kLogSeries[i]);
  const double lm = fma(s * z, p, 2.0 * s);
  const double de = (double)e;
  // ln 2 split so that e * hi is exact for |e| < 2^11
  return fma(de, 0x1.62e42fee00000p-1, fma(de, 0x1.a39ef35793c76p-33, lm));
}

// cos(pi y) for y in [0, 2] (the Box-Muller angle is a whole turn times a uniform, so no wider
// range reduction is needed).  y = k/2 + r with k = 0..4 and |r| <= 1/4, r exact;
// cos(pi y) is +-cos(pi r) or +-sin(pi r) by quadrant; both are Taylor polynomials in r^2
// (terms to r^15 and r^16: next term below 2^-54 of the first).  Within 2 ulp; a third of the
// instructions of the general-purpose cospi, which was a seventh of a Gamma attempt.
// (-1)^n pi^(2n+1)/(2n+1)!, n = 7..0, and (-1)^n pi^(2n)/(2n)!, n = 8..0.
__constant__ double kSinPiSeries[8] = {-0x1.6fadb9f155744p-16, 0x1.e8f434d018d63p-12,
                                       -0x1.e3074fde8871fp-8,  0x1.50783487ee782p-4,
                                       -0x1.32d2cce62bd86p-1,  0x1.466bc6775aae2p+1,
                                       -0x1.4abbce625be53p+2,  0x1.921fb54442d18p+1};
__constant__ double kCosPiSeries[9] = {0x1.20c62c2f2d7f5p-18, -0x1.b6e24f44b128fp-14,
                                       0x1.f9d38a3763cc3p-10, -0x1.a6d1f2a204a8cp-6,
                                       0x1.e1f506891babbp-3,  -0x1.55d3c7e3cbffap+0,
                                       0x1.03c1f081b5ac4p+2,  -0x1.3bd3cc9be45dep+2,
                                       1.0};
__device__ __forceinline__ double cospi_0_2(double y) {
  const double k = rint(2.0 * y);
  const double r = fma(-0.5, k, y);
  const int q = (int)k;
  const double z = r * r;
  double ps = kSinPiSeries[0], pc = kCosPiSeries[0];
#pragma unroll
  for (int i = 1; i < 8; ++i) ps = fma(ps, z, kSinPiSeries[i]);
#pragma unroll
  for (int i = 1; i < 9; ++i) pc = fma(pc, z, kCosPiSeries[i]);
  const double v = (q & 1) ? r * ps : pc;
  return ((q + 1) & 2) ? -v : v;  // quadrants 1 and 2 are negated: -sin, -cos
}

// The same logarithm with a table in LDS, for the kernels that take millions of them: x = m 2^e,
// m in [1, 2); i = round(128 (m - 1)) in 0..128 picks c_i = 1 + i/128; the table holds 1/c_i
// (rounded) and -ln of that stored value (minus ln 2 from i = 53 on, where c_i > sqrt 2 and e is
// raised by one instead, so that x just below a power of two meets no cancellation).  Then
// r = m / c_i - 1 is one exact fma, |r| <= 2^-8, and ln(1 + r) needs the series to r^6 only.
// The ends of the table are exact (1/c = 1 and 1/2, ln = 0), so arguments next to 1 keep their
// relative accuracy.  Within 6e-16 relative; 22 instructions against 37.
constexpr int kLogTableSize = 129;
constexpr int kLogTableFold = 53;  // first i with c_i > sqrt(2)
inline void fill_log_table(double2* t) {  // host
  for (int i = 0; i < kLogTableSize; ++i) {
    const double inv = 1.0 / (1.0 + (double)i / 128.0);
    long double l = -logl((long double)inv);
    if (i >= kLogTableFold) l -= logl(2.0L);
    if (i == 0 || i == kLogTableSize - 1) l = 0.0L;
    t[i] = make_double2(inv, (double)l);
  }
}
__device__ __forceinline__ double log_tab(double x, const double2* __restrict__ lt) {
  const uint32_t hi = (uint32_t)__double2hiint(x), lo = (uint32_t)__double2loint(x);
  const uint32_t idx = (((hi >> 12) & 0xFFu) + 1u) >> 1;
  const double m = __hiloint2double((int)((hi & 0x000FFFFFu) | 0x3FF00000u), (int)lo);
  const double2 t = lt[idx];
  const int e = (int)(hi >> 20) - 1023 + (idx >= (uint32_t)kLogTableFold ? 1 : 0);
  const double r = fma(m, t.x, -1.0);
  double p = fma(r, -1.0 / 6.0, 0.2);
  p = fma(p, r, -0.25);
  p = fma(p, r, 1.0 / 3.0);
  p = fma(p, r, -0.5);
  const double lnr = fma(p, r * r, r);
  const double de = (double)e;
  return fma(de, 0x1.62e42fee00000p-1, fma(de, 0x1.a39ef35793c76p-33, t.y + lnr));
}
// exp(x) for x <= 0 (and anything up to a few hundred) with a table in LDS: x = n ln2/128 + r,
// n = round(x 128/ln2), |r| <= ln2/256; exp(x) = 2^(n >> 7) T[n & 127] exp(r) with T[j] = 2^(j/128)
// and exp(r) - 1 by its series to r^5.  Arguments below -750 (also -inf) give 0.  Within
// 3e-16 relative; 18 instructions against 42 of the general routine.
constexpr int kExpTableSize = 128;
inline void fill_exp_table(double* t) {  // host
  for (int j = 0; j < kExpTableSize; ++j) t[j] = (double)powl(2.0L, (long double)j / 128.0L);
}
__device__ __forceinline__ double exp_tab(double x, const double* __restrict__ et) {
  x = fmax(x, -750.0);
  const double nf = rint(x * 0x1.71547652b82fep+7);  // 128 / ln 2
  const int n = (int)nf;
  double r = fma(nf, -0x1.62e42fef80000p-8, x);      // ln2/128, 35 bits: nf * hi is exact
  r = fma(nf, -0x1.1cf79ac000000p-43, r);
  const double T = et[n & (kExpTableSize - 1)];
  double p = fma(r, 1.0 / 120.0, 1.0 / 24.0);
  p = fma(p, r, 1.0 / 6.0);
  p = fma(p, r, 0.5);
  p = fma(p, r * r, r);
  return ldexp(fma(T, p, T), n >> 7);
}

// One logarithm, by the table if the caller has one in LDS.
__device__ __forceinline__ double log_of(double x, const double2* __restrict__ lt) {
  return lt != nullptr ? log_tab(x, lt) : log_pos(x);
}

// Square root of a positive normal double well inside the exponent range (the Box-Muller radicand
// -2 ln u lies in (0, 45]): reciprocal square root estimate, one coupled Newton step for the root
// and half its reciprocal, one correction of the root by its residual.  Within 1 ulp; a third of
// the instructions of the general routine, which guards ranges that cannot occur here.
__device__ __forceinline__ double sqrt_pos(double a) {
  const double y = __builtin_amdgcn_rsq(a);
  double s = a * y;
  double h = 0.5 * y;
  const double r = fma(-h, s, 0.5);
  s = fma(s, r, s);
  h = fma(h, r, h);
  const double d = fma(-s, s, a);
  return fma(d, h, s);
}
__device__ __forceinline__ double normal_from(const U4& b, const double2* __restrict__ lt) {
  return sqrt_pos(-2.0 * log_of(u32d(b.x), lt)) * cospi_0_2(2.0 * u32d(b.y));
}
__device__ __forceinline__ double normal_from(const U4& b) {
  return sqrt_pos(-2.0 * log_pos(u32d(b.x))) * cospi_0_2(2.0 * u32d(b.y));
}

constexpr int kGammaAttemptCap = 64;

// Gamma(a,1) draws in the log domain by Marsaglia & Tsang's squeeze-rejection
// method (2000), fp64: d = a' - 1/3, c = 1/sqrt(9 d), v = (1 + c x)^3 with x
// normal; accept if U < 1 - 0.0331 x^4 or ln U < x^2/2 + d (1 - v + ln v); the
// draw is d v.  a < 1 draws for a' = a + 1 and multiplies by U'^(1/a).  Attempt
// j of a variable reads Philox block j (x from words 0 and 1, U from 2, U' from
// 3).  Split into per-variable constants and a single attempt so that callers
// can let every lane retry on its own variable instead of waiting for the
// slowest lane of the wave.
struct GammaShape {
  double d, c, ln_d, inv_a;  // a < 1 exactly when inv_a > 1
};
__device__ __forceinline__ GammaShape gamma_shape(double a) {
  GammaShape g;
  g.d = (a < 1.0 ? a + 1.0 : a) - 1.0 / 3.0;
  g.c = 1.0 / sqrt(9.0 * g.d);
  g.ln_d = log(g.d);
  g.inv_a = 1.0 / a;
  return g;
}
// Shapes a0 + n for small integer counts n are read from a table built once
// per handle (the per-variable constants cost a square root, a division and a
// logarithm otherwise); larger counts are computed on the spot.
constexpr int kShapeTable = 1024;
constexpr int kShapeLds = 32;  // entries that the theta and phi kernels copy into LDS
__device__ __forceinline__ GammaShape gamma_shape_count(const GammaShape* __restrict__ table,
                                                        double a0, int n) {
  if (n < kShapeTable) return table[n];
  return gamma_shape(a0 + (double)n);
}
// One attempt; on acceptance writes ln(draw) and returns true.
__device__ __forceinline__ bool gamma_attempt(const GammaShape& g, const U4& b, double& lg,
                                              const double2* __restrict__ lt = nullptr) {
  const double x = normal_from(b, lt);
  const double t = 1.0 + g.c * x;
  const double v = t * t * t;
  const double U = u32d(b.z);
  const double x2 = x * x;
  const double lv = log_of(fabs(v), lt);  // only used when t > 0 (then v is a positive normal)
  bool accept = U < 1.0 - 0.0331 * x2 * x2;
  if (!accept) {
    // ln U < rhs.  A wave reaches this test on most attempts (any lane failing the squeeze
    // brings all 64 here), so the fp64 logarithm is kept for the cases a single-precision one
    // cannot decide: that one is good to 1e-6 + 2e-6 |ln U|, and a difference beyond four
    // times that has the sign of the exact difference.
    const double rhs = 0.5 * x2 + g.d * (1.0 - v + lv);
    const float lf = __logf((float)U);
    const float gap = lf - (float)rhs;
    const float margin = 4e-6f + 8e-6f * fabsf(lf);
    accept = gap < -margin;
    if (__builtin_expect(fabsf(gap) <= margin, 0)) accept = log_pos(U) < rhs;
  }
  accept = accept && t > 0.0;
  lg = g.ln_d + lv;
  if (g.inv_a > 1.0) lg += log_of(u32d(b.w), lt) * g.inv_a;
  return accept;
}
// Loop form: attempts until accepted.  `capped` is raised if the cap is reached.
__device__ __forceinline__ double gamma_log_draw(double a, uint64_t seed, uint64_t index,
                                                 uint32_t sweep, uint32_t stream, bool& capped) {
  const GammaShape g = gamma_shape(a);
  for (uint32_t j = 0; j < (uint32_t)kGammaAttemptCap; ++j) {
    double lg;
    if (gamma_attempt(g, random_block(seed, index, sweep, stream, j), lg)) return lg;
  }
  capped = true;
  return g.ln_d;
}

// The sweep index of a launch: a value (eager launches), or a value plus a counter in device
// memory (launches recorded in a HIP graph, which replays the same arguments every time: the
// counter is advanced by a kernel at the end of each recorded sweep).
struct SweepRef {
  uint32_t base;
  const uint32_t* dev;
  __device__ __forceinline__ uint32_t get() const { return base + (dev != nullptr ? *dev : 0u); }
};
__global__ void sweep_counter_add_kernel(uint32_t* counter, uint32_t add);   // *counter += add
__global__ void sweep_counter_set_kernel(uint32_t* counter, uint32_t value); // *counter = value

// --------------------------------------------------------------- wave helpers
// Orders LDS traffic between lanes of one wave (no cross-wave barrier).
__device__ __forceinline__ void wave_lds_fence() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <typename T>
__device__ __forceinline__ T wave_allreduce_sum(T v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
template <typename T>
__device__ __forceinline__ T wave_allreduce_max(T v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const T other = __shfl_xor(v, o, 64);
    v = other > v ? other : v;
  }
  return v;
}

// Deterministic grid-wide fp64 sum: every block writes one partial (sum of its
// threads in a fixed tree order); the host adds the partials in index order.
__device__ __forceinline__ void block_partial_sum(double v, double* partials, double* smem) {
  v = wave_allreduce_sum(v);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (lane == 0) smem[wave] = v;
  __syncthreads();
  if (threadIdx.x == 0) {
    double s = 0.0;
    const int nw = (blockDim.x + 63) >> 6;
    for (int i = 0; i < nw; ++i) s += smem[i];
    partials[blockIdx.x] = s;
  }
  __syncthreads();
}

inline int64_t round_up(int64_t x, int64_t m) { return (x + m - 1) / m * m; }

}  // namespace augur
