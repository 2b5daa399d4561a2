// Instantiations of the attention kernel for token-wise quantized values (paper Section 2 and
// Section 6.3, "+ value quantization") together with the grouped angle quantizer of Section 3.2:
// 4-bit and 2-bit values, (r, t) = (4, 4) and (3, 3).
#include "pq_decode_kernels.hpp"

namespace pq {
namespace {

template <int G, int RB, int TB, int VB>
void launch_one(const DecodeArgs& a, pq_dtype qdt, dim3 grid, hipStream_t st) {
  const bool sc = a.scores != nullptr;
  if (qdt == PQ_F16) {
    if (sc) hipLaunchKernelGGL((pq_decode_partials_kernel<G, RB, TB, __half, true, VB, true>), grid, dim3(kThreads), 0, st, a);
    else    hipLaunchKernelGGL((pq_decode_partials_kernel<G, RB, TB, __half, false, VB, true>), grid, dim3(kThreads), 0, st, a);
  } else {
    if (sc) hipLaunchKernelGGL((pq_decode_partials_kernel<G, RB, TB, float, true, VB, true>), grid, dim3(kThreads), 0, st, a);
    else    hipLaunchKernelGGL((pq_decode_partials_kernel<G, RB, TB, float, false, VB, true>), grid, dim3(kThreads), 0, st, a);
  }
}

template <int RB, int TB, int VB>
bool launch_g(int G, const DecodeArgs& a, pq_dtype qdt, dim3 grid, hipStream_t st) {
  switch (G) {
    case 1: launch_one<1, RB, TB, VB>(a, qdt, grid, st); return true;
    case 2: launch_one<2, RB, TB, VB>(a, qdt, grid, st); return true;
    case 4: launch_one<4, RB, TB, VB>(a, qdt, grid, st); return true;
    default: return false;
  }
}

}  // namespace

hipError_t launch_partials_ga_vq(int rt, int G, int v_bits, const DecodeArgs& a, pq_dtype qdt, dim3 grid,
                              hipStream_t st) {
  bool ok = false;
  if (rt == 44 && v_bits == 4) ok = launch_g<4, 4, 4>(G, a, qdt, grid, st);
  else if (rt == 44 && v_bits == 2) ok = launch_g<4, 4, 2>(G, a, qdt, grid, st);
  else if (rt == 33 && v_bits == 4) ok = launch_g<3, 3, 4>(G, a, qdt, grid, st);
  else if (rt == 33 && v_bits == 2) ok = launch_g<3, 3, 2>(G, a, qdt, grid, st);
  if (!ok) return hipErrorInvalidValue;
  return hipGetLastError();
}

}  // namespace pq
