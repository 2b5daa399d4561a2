// CPU build of the library's angle-bin rule (csrc/pq_angle.hpp) for tests: fills codes[i] for
// n pairs; t_bits in 2..5.  Returns 0, or -1 for an unsupported t_bits.
#include <math.h>
#include <stdint.h>

#include "pq_angle.hpp"

extern "C" int angle_bins_host(const float* x, const float* y, int64_t n, int t_bits, int32_t* codes) {
  double tan_edge[4] = {0, 0, 0, 0};
  const int nb = 1 << t_bits;
  for (int k = 1; k < nb / 8 && k < 4; ++k) tan_edge[k] = tan(k * (2.0 * M_PI / nb));
  for (int64_t i = 0; i < n; ++i) {
    switch (t_bits) {
      case 2: codes[i] = (int32_t)pq::angle_bin<2>(x[i], y[i], tan_edge); break;
      case 3: codes[i] = (int32_t)pq::angle_bin<3>(x[i], y[i], tan_edge); break;
      case 4: codes[i] = (int32_t)pq::angle_bin<4>(x[i], y[i], tan_edge); break;
      case 5: codes[i] = (int32_t)pq::angle_bin<5>(x[i], y[i], tan_edge); break;
      default: return -1;
    }
  }
  return 0;
}

// The rule for pairs strictly inside an octant: codes[i] where it applies, -1 where the pair sits
// on an axis, a diagonal or the origin (the library then uses angle_bin).
extern "C" int angle_bins_interior_host(const float* x, const float* y, int64_t n, int t_bits, int32_t* codes) {
  double tan_edge[4] = {0, 0, 0, 0};
  const int nb = 1 << t_bits;
  for (int k = 1; k < nb / 8 && k < 4; ++k) tan_edge[k] = tan(k * (2.0 * M_PI / nb));
  for (int64_t i = 0; i < n; ++i) {
    bool interior = false;
    uint32_t c;
    switch (t_bits) {
      case 2: c = pq::angle_bin_interior<2>(x[i], y[i], tan_edge, interior); break;
      case 3: c = pq::angle_bin_interior<3>(x[i], y[i], tan_edge, interior); break;
      case 4: c = pq::angle_bin_interior<4>(x[i], y[i], tan_edge, interior); break;
      case 5: c = pq::angle_bin_interior<5>(x[i], y[i], tan_edge, interior); break;
      default: return -1;
    }
    codes[i] = interior ? (int32_t)c : -1;
  }
  return 0;
}

// The library's float64 -> fp16-grid rounding (parameters of the grouped angle quantizer).
extern "C" void round_to_half_host(const double* v, int64_t n, double* out) {
  for (int64_t i = 0; i < n; ++i) out[i] = pq::round_to_half(v[i]);
}
