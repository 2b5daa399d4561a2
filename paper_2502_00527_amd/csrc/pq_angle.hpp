// Angle bin of the uniform t-bit grid over [-pi, pi) (paper Section 3.2 with a uniform grid):
// the code is floor((atan2(y, x) + pi) * 2^t / (2 pi)) evaluated as in exact arithmetic, without
// an arc tangent.  Plain C++ (host and device) so that the rule can also be checked on the CPU.
//
// The grid is cut into eight octants that start on an axis or a diagonal.  The octant follows
// from sign and magnitude comparisons, which are exact, so a point exactly on an octant boundary
// lands in the octant that STARTS there (bins are half-open arcs; these are the only directions
// where a float pair can sit exactly on a bin edge, because the other edges have irrational
// slopes).  Inside an octant the 2^t / 8 bins are separated by the slopes tan(k D), D = 2 pi / 2^t:
// the bin is a count of float64 comparisons against mx * tan(k D) (mn, mx = the smaller / larger
// of |x|, |y|), whose rounding moves an edge by ~1e-16 rad.  In odd octants the angle runs against
// the ratio mn / mx, so the count is taken from the other side.
// Conventions: x = y = 0 -> bin 2^(t-1) (theta = 0); y = +0, x < 0 (theta = +pi) -> last bin;
// y = -0, x < 0 (theta = -pi) -> bin 0.
#pragma once

#include <math.h>
#include <stdint.h>

#ifndef PQ_HD
#define PQ_HD
#endif

namespace pq {

// tan_edge[k] = tan(k * 2 pi / 2^t) for 1 <= k < 2^t / 8 (unused entries are ignored)
template <int TB>
PQ_HD inline uint32_t angle_bin(float x, float y, const double* tan_edge) {
  constexpr int NB = 1 << TB;
  constexpr int S = NB >= 8 ? NB / 8 : 1;           // bins per octant
  // Everything about the octant is integer arithmetic on the IEEE bit patterns (finite inputs):
  // magnitudes compare like unsigned integers, and 0/1 flags are combined without branches.
  uint32_t bx, by;
  __builtin_memcpy(&bx, &x, 4);
  __builtin_memcpy(&by, &y, 4);
  const uint32_t ax = bx & 0x7fffffffu, ay = by & 0x7fffffffu;
  const uint32_t xnz = (ax + 0x7fffffffu) >> 31, ynz = (ay + 0x7fffffffu) >> 31;   // 1 if non-zero
  const uint32_t xn = (bx >> 31) & xnz;                      // x < 0
  const uint32_t yn = (by >> 31) & (ynz | xn);               // y < 0, or y = -0 with x < 0 (theta = -pi)
  const uint32_t lt = (ay - ax) >> 31, gt = (ax - ay) >> 31; // |y| < |x|, |y| > |x|
  // octant:
  //   lower half plane (yn): x < 0 -> 0 | 1 (the diagonal starts 1); x = 0 -> 2; x > 0 -> 2 | 3
  //   upper half plane     : x > 0 -> 4 | 5;                         x = 0 -> 6; x < 0 -> 6 | 7
  const uint32_t same = 1u ^ xn ^ yn;
  const uint32_t within_nz = same * (1u - lt) + (1u ^ same) * (3u - gt);
  const uint32_t within = xnz * within_nz + (1u ^ xnz) * 2u;
  const uint32_t o = (1u ^ yn) * 4u + within;
  uint32_t code;
  if (TB == 2) {
    code = o >> 1;                                  // bins are quadrants
  } else {
    uint32_t sub = 0;
    if (S > 1) {
      const uint32_t mnb = ax < ay ? ax : ay, mxb = ax < ay ? ay : ax;
      float mnf, mxf;
      __builtin_memcpy(&mnf, &mnb, 4);
      __builtin_memcpy(&mxf, &mxb, 4);
      const double mn = mnf, mx = mxf;
      const uint32_t odd = o & 1u;
      for (int k = 1; k < S; ++k) {
        const double edge = mx * tan_edge[k];
        const uint32_t past_odd = mn <= edge, past_even = edge <= mn;
        sub += odd * past_odd + (1u ^ odd) * past_even;
      }
    }
    code = o * S + sub;
  }
  const uint32_t origin = 1u ^ (xnz | ynz);
  return origin * (NB / 2) + (1u ^ origin) * code;
}

// The same bin for a pair strictly inside an octant (x != 0, y != 0, |x| != |y|; `interior` says
// whether that holds -- if not, the result is meaningless and angle_bin decides).  There the
// octant is a table look-up on (x < 0, y < 0, |y| > |x|): entry = first bin of the octant, plus
// S - 1 in odd octants, where the angle runs against the ratio mn / mx and the count of passed
// edges is subtracted; since the count is below S, both cases are one XOR with the entry.  (A
// float64 product that equals mn exactly is counted as passed in both directions; angle_bin
// counts it as passed towards the upper bin.  Edges have irrational slopes, so this is a
// statement about rounding noise, not about points on an edge.)
namespace detail {
constexpr uint32_t octant_of(int idx) {          // idx = (x < 0) + 2 (y < 0) + 4 (|y| > |x|)
  constexpr uint32_t o[8] = {4, 7, 3, 0, 5, 6, 2, 1};
  return o[idx];
}
template <int TB>
constexpr uint32_t octant_entries(int gt) {      // 4 entries of 8 bits, for idx = 4 gt .. 4 gt + 3
  constexpr int NB = 1 << TB;
  constexpr int S = NB >= 8 ? NB / 8 : 1;
  uint32_t w = 0;
  for (int i = 0; i < 4; ++i) {
    const uint32_t o = octant_of(4 * gt + i);
    const uint32_t e = TB == 2 ? (o >> 1) : o * S + (o & 1u) * (S - 1);
    w |= e << (8 * i);
  }
  return w;
}
}  // namespace detail

template <int TB>
PQ_HD inline uint32_t angle_bin_interior(float x, float y, const double* tan_edge, bool& interior) {
  constexpr int NB = 1 << TB;
  constexpr int S = NB >= 8 ? NB / 8 : 1;
  constexpr uint32_t lo = detail::octant_entries<TB>(0), hi = detail::octant_entries<TB>(1);
  uint32_t bx, by;
  __builtin_memcpy(&bx, &x, 4);
  __builtin_memcpy(&by, &y, 4);
  const float ax = __builtin_fabsf(x), ay = __builtin_fabsf(y);
  const float mnf = ax < ay ? ax : ay, mxf = ax < ay ? ay : ax;
  interior = mnf != 0.f && mnf != mxf;
  const uint32_t shift = ((bx >> 28) & 8u) | ((by >> 27) & 16u);      // 8 * ((x < 0) + 2 (y < 0))
  uint32_t code = ((ay > ax ? hi : lo) >> shift) & 0xffu;
  if (S > 1) {
    const double mn = mnf, mx = mxf;
    uint32_t passed = 0;
    for (int k = 1; k < S; ++k) passed += mx * tan_edge[k] <= mn;
    code ^= passed;
  }
  return code;
}

// v rounded to the nearest fp16 value, ties to even, returned as a double (|v| < 65504).  One
// rounding, straight from float64: the quantum is 2^(e - 10) for |v| in [2^e, 2^(e+1)), and 2^-24
// below the smallest normal fp16.  Used for the 16-bit parameters of the grouped angle quantizer,
// whose statistics are float64.
PQ_HD inline double round_to_half(double v) {
  uint64_t b;
  __builtin_memcpy(&b, &v, 8);
  int e = static_cast<int>((b >> 52) & 0x7ffu) - 1023;
  if (e < -14) e = -14;
  const uint64_t qb = static_cast<uint64_t>(e - 10 + 1023) << 52, ib = static_cast<uint64_t>(10 - e + 1023) << 52;
  double q, iq;
  __builtin_memcpy(&q, &qb, 8);
  __builtin_memcpy(&iq, &ib, 8);
  return rint(v * iq) * q;         // both scalings are exact (powers of two)
}

}  // namespace pq
