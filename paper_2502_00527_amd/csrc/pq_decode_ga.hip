// Attention and score-only kernels for the grouped angle quantizer (Section 3.2 as printed:
// per-group angle min / scale, table rebuilt per group), instantiated here so that they compile
// beside the uniform-grid kernels.
#include "pq_decode_kernels.hpp"

namespace pq {
namespace {

template <int G, int RB, int TB>
hipError_t launch_ga(const DecodeArgs& a, pq_dtype qdt, dim3 grid, hipStream_t st) {
  const bool sc = a.scores != nullptr;
  if (qdt == PQ_F16) {
    if (sc) hipLaunchKernelGGL((pq_decode_partials_kernel<G, RB, TB, __half, true, 16, true>), grid, dim3(kThreads), 0, st, a);
    else    hipLaunchKernelGGL((pq_decode_partials_kernel<G, RB, TB, __half, false, 16, true>), grid, dim3(kThreads), 0, st, a);
  } else {
    if (sc) hipLaunchKernelGGL((pq_decode_partials_kernel<G, RB, TB, float, true, 16, true>), grid, dim3(kThreads), 0, st, a);
    else    hipLaunchKernelGGL((pq_decode_partials_kernel<G, RB, TB, float, false, 16, true>), grid, dim3(kThreads), 0, st, a);
  }
  return hipGetLastError();
}

template <int RB, int TB>
hipError_t launch_ga_g(int G, const DecodeArgs& a, pq_dtype qdt, dim3 grid, hipStream_t st) {
  switch (G) {
    case 1: return launch_ga<1, RB, TB>(a, qdt, grid, st);
    case 2: return launch_ga<2, RB, TB>(a, qdt, grid, st);
    case 4: return launch_ga<4, RB, TB>(a, qdt, grid, st);
    default: return hipErrorInvalidValue;
  }
}

template <int G, int RB, int TB>
hipError_t launch_sc(const DecodeArgs& a, pq_dtype qdt, dim3 grid, hipStream_t st) {
  if (qdt == PQ_F16) hipLaunchKernelGGL((pq_score_keys_kernel<G, RB, TB, __half, true>), grid, dim3(kThreads), 0, st, a);
  else               hipLaunchKernelGGL((pq_score_keys_kernel<G, RB, TB, float, true>), grid, dim3(kThreads), 0, st, a);
  return hipGetLastError();
}

template <int RB, int TB>
hipError_t launch_sc_g(int G, const DecodeArgs& a, pq_dtype qdt, dim3 grid, hipStream_t st) {
  switch (G) {
    case 1: return launch_sc<1, RB, TB>(a, qdt, grid, st);
    case 2: return launch_sc<2, RB, TB>(a, qdt, grid, st);
    case 4: return launch_sc<4, RB, TB>(a, qdt, grid, st);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace

hipError_t launch_partials_ga(int rt, int G, const DecodeArgs& a, pq_dtype qdt, dim3 grid, hipStream_t st) {
  switch (rt) {
    case 44: return launch_ga_g<4, 4>(G, a, qdt, grid, st);
    case 33: return launch_ga_g<3, 3>(G, a, qdt, grid, st);
    default: return hipErrorInvalidValue;
  }
}

hipError_t launch_scores_ga(int rt, int G, const DecodeArgs& a, pq_dtype qdt, dim3 grid, hipStream_t st) {
  switch (rt) {
    case 44: return launch_sc_g<4, 4>(G, a, qdt, grid, st);
    case 33: return launch_sc_g<3, 3>(G, a, qdt, grid, st);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace pq
