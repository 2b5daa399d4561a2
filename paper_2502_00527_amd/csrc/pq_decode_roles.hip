// Instantiations of the role-specialised attention kernel (fp16 values, uniform angle grid): the
// kernels that share a launch out evenly and merge inside.  pq_decode_roles_grid.hip compiles this
// file a second time for the one-work-group-per-chunk kernels.
#include "pq_decode_roles.hpp"

#ifndef PQ_ROLES_BALANCED
#define PQ_ROLES_BALANCED true
#define PQ_ROLES_LAUNCH launch_attention_roles
#endif

namespace pq {
namespace {

template <int G, int RB, int TB, typename QT, bool SCORES>
void launch_mode(const DecodeArgs& a, const dim3 grid, hipStream_t st) {
  hipLaunchKernelGGL((pq_decode_roles_kernel<G, RB, TB, QT, SCORES, PQ_ROLES_BALANCED>), grid, dim3(kRoleThreads), 0, st, a);
}

template <int G, int RB, int TB>
void launch_one(const DecodeArgs& a, pq_dtype qdt, int n_wg, hipStream_t st) {
  const dim3 grid(n_wg);
  const bool sc = a.scores != nullptr;
  if (qdt == PQ_F16) {
    if (sc) launch_mode<G, RB, TB, __half, true>(a, grid, st);
    else    launch_mode<G, RB, TB, __half, false>(a, grid, st);
  } else {
    if (sc) launch_mode<G, RB, TB, float, true>(a, grid, st);
    else    launch_mode<G, RB, TB, float, false>(a, grid, st);
  }
}

template <int RB, int TB>
bool launch_g(int G, const DecodeArgs& a, pq_dtype qdt, int grid, hipStream_t st) {
  switch (G) {
    case 1: launch_one<1, RB, TB>(a, qdt, grid, st); return true;
    case 2: launch_one<2, RB, TB>(a, qdt, grid, st); return true;
    case 4: launch_one<4, RB, TB>(a, qdt, grid, st); return true;
    default: return false;
  }
}

}  // namespace

hipError_t PQ_ROLES_LAUNCH(int rt, int G, const DecodeArgs& a, pq_dtype qdt, int grid, hipStream_t st) {
  bool ok = false;
  switch (rt) {
    case 44: ok = launch_g<4, 4>(G, a, qdt, grid, st); break;
    case 33: ok = launch_g<3, 3>(G, a, qdt, grid, st); break;
    case 53: ok = launch_g<5, 3>(G, a, qdt, grid, st); break;
    case 35: ok = launch_g<3, 5>(G, a, qdt, grid, st); break;
    case 42: ok = launch_g<4, 2>(G, a, qdt, grid, st); break;
    case 24: ok = launch_g<2, 4>(G, a, qdt, grid, st); break;
    default: break;
  }
  if (!ok) return hipErrorInvalidValue;
  return hipGetLastError();
}

}  // namespace pq

