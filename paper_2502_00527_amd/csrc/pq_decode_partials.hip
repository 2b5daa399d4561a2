// Instantiations of the attention kernel whose wavefronts alternate between a score and a value
// phase (pq_decode_partials_kernel), uniform angle grid: fp16 and quantized values, all bit
// allocations.  pq_decode_partials_ga.hip compiles this file a second time for the grouped angle
// quantizer of Section 3.2 (per-group angle min / scale, table rebuilt per group).
#include "pq_decode_kernels.hpp"

#ifndef PQ_PARTIALS_GA
#define PQ_PARTIALS_GA false
#define PQ_PARTIALS_LAUNCH launch_attention_partials
#endif

namespace pq {
namespace {

template <int RB, int TB, int VB>
bool launch_g(int G, const DecodeArgs& a, dim3 grid, hipStream_t st) {
  const dim3 block(kThreads);
  switch (G) {
    case 1: hipLaunchKernelGGL((pq_decode_partials_kernel<1, RB, TB, VB, PQ_PARTIALS_GA>), grid, block, 0, st, a); return true;
    case 2: hipLaunchKernelGGL((pq_decode_partials_kernel<2, RB, TB, VB, PQ_PARTIALS_GA>), grid, block, 0, st, a); return true;
    case 4: hipLaunchKernelGGL((pq_decode_partials_kernel<4, RB, TB, VB, PQ_PARTIALS_GA>), grid, block, 0, st, a); return true;
    default: return false;
  }
}

template <int RB, int TB>
bool launch_v(int v_bits, int G, const DecodeArgs& a, dim3 grid, hipStream_t st) {
  switch (v_bits) {
    case 16: return launch_g<RB, TB, 16>(G, a, grid, st);
    case 4: return launch_g<RB, TB, 4>(G, a, grid, st);
    case 2: return launch_g<RB, TB, 2>(G, a, grid, st);
    default: return false;
  }
}

}  // namespace

bool PQ_PARTIALS_LAUNCH(int rt, int G, int v_bits, const DecodeArgs& a, dim3 grid, hipStream_t st) {
  switch (rt) {
    case 44: return launch_v<4, 4>(v_bits, G, a, grid, st);
    case 33: return launch_v<3, 3>(v_bits, G, a, grid, st);
    case 53: return launch_v<5, 3>(v_bits, G, a, grid, st);
    case 35: return launch_v<3, 5>(v_bits, G, a, grid, st);
    case 42: return launch_v<4, 2>(v_bits, G, a, grid, st);
    case 24: return launch_v<2, 4>(v_bits, G, a, grid, st);
    default: return false;
  }
}

}  // namespace pq
