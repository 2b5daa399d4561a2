// Instantiations of the role-specialised attention kernel (uniform angle grid): the kernels that
// share a launch out evenly and merge inside.  pq_decode_roles_grid.hip compiles this file a
// second time for the one-work-group-per-chunk kernels.
#include "pq_decode_roles.hpp"

#ifndef PQ_ROLES_BALANCED
#define PQ_ROLES_BALANCED true
#define PQ_ROLES_LAUNCH launch_attention_roles
#endif

namespace pq {
namespace {

template <int G, int RB, int TB, int VB>
void launch_one(const DecodeArgs& a, int n_wg, hipStream_t st) {
  hipLaunchKernelGGL((pq_decode_roles_kernel<G, RB, TB, VB, PQ_ROLES_BALANCED>), dim3(n_wg), dim3(kRoleThreads), 0, st, a);
}
template <int RB, int TB, int VB>
bool launch_g(int G, const DecodeArgs& a, int n_wg, hipStream_t st) {
  switch (G) {
    case 1: launch_one<1, RB, TB, VB>(a, n_wg, st); return true;
    case 2: launch_one<2, RB, TB, VB>(a, n_wg, st); return true;
    case 4: launch_one<4, RB, TB, VB>(a, n_wg, st); return true;
    case 8:
      if constexpr (VB == 16) {
        launch_one<8, RB, TB, VB>(a, n_wg, st);
        return true;
      }
      return false;
    default: return false;
  }
}

template <int RB, int TB>
bool launch_v(int v_bits, int G, const DecodeArgs& a, int n_wg, hipStream_t st) {
  switch (v_bits) {
    case 16: return launch_g<RB, TB, 16>(G, a, n_wg, st);
    case 4: return launch_g<RB, TB, 4>(G, a, n_wg, st);
    case 2: return launch_g<RB, TB, 2>(G, a, n_wg, st);
    default: return false;
  }
}

}  // namespace

bool PQ_ROLES_LAUNCH(int rt, int G, int v_bits, const DecodeArgs& a, int n_wg, hipStream_t st) {
  switch (rt) {
    case 44: return launch_v<4, 4>(v_bits, G, a, n_wg, st);
    case 33: return launch_v<3, 3>(v_bits, G, a, n_wg, st);
    case 53: return launch_v<5, 3>(v_bits, G, a, n_wg, st);
    case 35: return launch_v<3, 5>(v_bits, G, a, n_wg, st);
    case 42: return launch_v<4, 2>(v_bits, G, a, n_wg, st);
    case 24: return launch_v<2, 4>(v_bits, G, a, n_wg, st);
    default: return false;
  }
}

}  // namespace pq
