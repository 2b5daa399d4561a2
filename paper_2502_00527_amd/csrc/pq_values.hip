// Token-wise value quantization (paper Section 2, the formula for Q(V_n[j]); used by the paper in
// Section 6.3 "+ value quantization" and the dagger rows of its throughput table):
//   code = Clamp(round((v - z) / s), 0, 2^b - 1),  z = min of the token's d values, s = (max - min) / (2^b - 1),
// round-half-to-even, s and z stored as fp16 and used as stored, fp32 arithmetic with IEEE
// division; a constant row (s == 0) gets code 0.  Dequantized value: code * s + z.
//
// One work-group quantizes one page (128 tokens) of one KV head: thread = (dim slice tid % 16 of
// 8 dims, token tid / 16), 8 passes of 16 tokens; the row minimum / maximum are folded over the 16
// lanes of a token with shuffles.
#pragma clang fp contract(off)

#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>
#include <math.h>

#include "pq_internal.hpp"

namespace pq {
namespace {

struct ValueArgs {
  const __half* values;
  const int32_t* page_ids;
  uint8_t* vq;
  uint32_t* vparams;
  int64_t token_stride;
  int64_t head_stride;
  int64_t n_tokens;
  int64_t n_pool_pages;
  int32_t n_kv_heads;
};

template <int VB>
__global__ __launch_bounds__(256) void pq_encode_values_kernel(const ValueArgs a) {
  constexpr int T = 16 / VB;                     // tokens per 16-byte unit
  constexpr float kLevels = static_cast<float>((1 << VB) - 1);
  const int grp = blockIdx.x, kvh = blockIdx.y;
  const int64_t page = a.page_ids[grp];
  if (page < 0 || page >= a.n_pool_pages) return;
  const int64_t tok0 = static_cast<int64_t>(grp) * kGroup;
  const int nv = static_cast<int>(min<int64_t>(kGroup, a.n_tokens - tok0));
  const int64_t ph = page * a.n_kv_heads + kvh;
  const int sl = threadIdx.x & 15, tl = threadIdx.x >> 4;
  const __half* base = a.values + kvh * a.head_stride + sl * 8;
  uint8_t* const dst = a.vq + ph * (kGroup * kHeadDim * VB / 8);
#pragma unroll 2
  for (int it = 0; it < 8; ++it) {
    const int tok = it * 16 + tl;
    const bool valid = tok < nv;
    float v[8];
    if (valid) {
      const uint4 r = *reinterpret_cast<const uint4*>(base + (tok0 + tok) * a.token_stride);
      const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const __half2 h = *reinterpret_cast<const __half2*>(&w[e]);
        v[2 * e] = __low2float(h);
        v[2 * e + 1] = __high2float(h);
      }
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] = 0.f;
    }
    float mn = v[0], mx = v[0];
#pragma unroll
    for (int e = 1; e < 8; ++e) { mn = fminf(mn, v[e]); mx = fmaxf(mx, v[e]); }
#pragma unroll
    for (int m = 1; m < 16; m <<= 1) {
      mn = fminf(mn, __shfl_xor(mn, m));
      mx = fmaxf(mx, __shfl_xor(mx, m));
    }
    const __half sh = __float2half_rn((mx - mn) / kLevels), zh = __float2half_rn(mn);
    const float sf = __half2float(sh), zf = __half2float(zh);
    uint32_t field = 0;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      float q = rintf((v[e] - zf) / sf);                      // round half to even, IEEE division
      q = fminf(fmaxf(q, 0.f), kLevels);
      q = sf != 0.f ? q : 0.f;
      field |= static_cast<uint32_t>(q) << (VB * e);
    }
    if (!valid) field = 0;
    // A unit's 32-bit words hold two consecutive tokens each, the even one in the low half:
    // 4-bit codes word 2 * pair + (dims 0-3 | dims 4-7), 2-bit codes word pair (all 8 dims).
    uint8_t* unit = dst + ((tok / T) * 16 + sl) * 16;
    const int pair = (tok % T) >> 1, half = tok & 1;
    if constexpr (VB == 4) {
      *reinterpret_cast<uint16_t*>(unit + (2 * pair) * 4 + half * 2) = static_cast<uint16_t>(field);
      *reinterpret_cast<uint16_t*>(unit + (2 * pair + 1) * 4 + half * 2) = static_cast<uint16_t>(field >> 16);
    } else {
      *reinterpret_cast<uint16_t*>(unit + pair * 4 + half * 2) = static_cast<uint16_t>(field);
    }
    if (sl == 0)
      a.vparams[ph * kGroup + tok] =
          valid ? (static_cast<uint32_t>(__half_as_ushort(sh)) | (static_cast<uint32_t>(__half_as_ushort(zh)) << 16)) : 0u;
  }
}

bool value_bits_ok(int v_bits) { return v_bits == 4 || v_bits == 2; }

}  // namespace
}  // namespace pq

using namespace pq;

extern "C" size_t pq_vq_bytes_per_page(const pq_layout* l, int32_t v_bits) {
  if (!layout_supported(l) || !value_bits_ok(v_bits)) return 0;
  return static_cast<size_t>(l->n_kv_heads) * kGroup * kHeadDim * v_bits / 8;
}

extern "C" size_t pq_vq_params_bytes_per_page(const pq_layout* l) {
  if (!layout_supported(l)) return 0;
  return static_cast<size_t>(l->n_kv_heads) * kGroup * 4;
}

extern "C" int pq_encode_values(const pq_layout* layout, int32_t v_bits, const void* values, int64_t token_stride,
                                int64_t head_stride, int64_t n_tokens, const int32_t* page_ids, void* vq_pool,
                                void* vq_params_pool, int64_t n_pool_pages, void* hip_stream) {
  if (!layout) return PQ_ERR_INVALID_ARG;
  if (!layout_supported(layout) || !value_bits_ok(v_bits)) return PQ_ERR_UNSUPPORTED;
  if (n_tokens < 0 || n_pool_pages <= 0) return PQ_ERR_INVALID_ARG;
  if (n_tokens == 0) return PQ_OK;
  if (!values || !page_ids || !vq_pool || !vq_params_pool) return PQ_ERR_INVALID_ARG;
  if ((reinterpret_cast<uintptr_t>(values) & 15u) || token_stride % 8 || head_stride % 8 || token_stride < kHeadDim ||
      head_stride < 0 || (reinterpret_cast<uintptr_t>(vq_pool) & 15u) || (reinterpret_cast<uintptr_t>(vq_params_pool) & 3u))
    return PQ_ERR_INVALID_ARG;
  const int64_t n_groups = (n_tokens + kGroup - 1) / kGroup;
  if (n_groups > 0x7fffffff || layout->n_kv_heads > 65535) return PQ_ERR_UNSUPPORTED;
  ValueArgs a;
  a.values = static_cast<const __half*>(values);
  a.page_ids = page_ids;
  a.vq = static_cast<uint8_t*>(vq_pool);
  a.vparams = static_cast<uint32_t*>(vq_params_pool);
  a.token_stride = token_stride;
  a.head_stride = head_stride;
  a.n_tokens = n_tokens;
  a.n_pool_pages = n_pool_pages;
  a.n_kv_heads = layout->n_kv_heads;
  const dim3 grid(static_cast<uint32_t>(n_groups), layout->n_kv_heads);
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  if (v_bits == 4) hipLaunchKernelGGL(pq_encode_values_kernel<4>, grid, dim3(256), 0, st, a);
  else hipLaunchKernelGGL(pq_encode_values_kernel<2>, grid, dim3(256), 0, st, a);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return record_hip_error(e);
  return PQ_OK;
}
