// Prefill-time encoder of the polar-quantized key cache (gfx950).
//
// Per pair (x, y) = (K[j], K[j + d/2]) (Section 3.2; pairing of footnote 2 in
// Section 3.1):   rho = sqrt(x^2 + y^2),  theta = atan2(y, x),
//   angle code  a = floor((theta + pi) 2^t / 2 pi)    uniform grid over [-pi, pi)
//   radius code c = Clamp(floor((rho - z) / s), 0, 2^r - 1)
// with z = min, s = (max - min) / 2^r of rho over the tokens of the group,
// both rounded to fp16 and used as rounded.  Codes are integer decisions, so
// the arithmetic that leads to them is pinned:
//   * rho, (rho - z) / s: IEEE fp32, one rounding per operation, no fused
//     multiply-add (this file is compiled with floating-point contraction off).
//   * the angle bin is decided by exact sign/magnitude comparisons (octant)
//     and float64 slope comparisons against the bin edges inside the octant,
//     so it equals the floor of the real-number quotient; a point exactly on
//     an edge (only possible on an axis or a diagonal) belongs to the upper
//     bin, theta = +pi is clamped into the last bin, and x = y = 0 goes to
//     bin 2^(t-1).
// With the grouped angle quantizer (Section 3.2 as printed) the angle is instead
//   theta = atan2(y, x) in float64,  a = Clamp(floor((theta - z_t) / s_t), 0, 2^t - 1)
// with z_t = min, s_t = (max - min) / 2^t of theta over the group, rounded once from
// float64 to fp16 and used as rounded (a = 0 when s_t == 0); the page's parameter block
// then holds the 64 radius entries followed by the 64 angle entries.
//
// One work-group encodes one page (128 tokens) of one KV head: thread =
// (pair octet o = tid % 8, token slot tid / 8), four tokens per thread.
#pragma clang fp contract(off)

#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>
#include <math.h>

#define PQ_HD __host__ __device__
#include "pq_angle.hpp"
#include "pq_internal.hpp"

namespace pq {
namespace {

constexpr int kEncThreads = 256;
constexpr int kItems = 4;   // tokens per thread

struct EncodeArgs {
  const void* keys;
  const int32_t* page_ids;
  uint8_t* codes;
  uint32_t* params;
  int64_t token_stride;
  int64_t head_stride;
  int64_t n_tokens;
  int64_t n_pool_pages;
  int32_t n_kv_heads;
  double tan_edge[kMaxAngleBins / 8];    // tan(k * 2 pi / 2^t) for the edges inside an octant
};

__device__ __forceinline__ void load8(const __half* p, float (&v)[8]) {
  const uint4 r = *reinterpret_cast<const uint4*>(p);
  const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const __half2 h = *reinterpret_cast<const __half2*>(&w[e]);
    v[2 * e] = __low2float(h);
    v[2 * e + 1] = __high2float(h);
  }
}
__device__ __forceinline__ void load8(const float* p, float (&v)[8]) {
  const float4 a = reinterpret_cast<const float4*>(p)[0], b = reinterpret_cast<const float4*>(p)[1];
  v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
  v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}

// Correctly rounded fp32 square root.  For fp32 inputs this is the compiler's sequence (it also
// covers denormal and infinite arguments).  A sum of two squares of fp16 values is either 0 or at
// least 2^-48 and at most 2^33, so the hardware approximation (1 ulp) only needs the final
// rounding fix: step to the neighbour whose exact residual has the right sign.
template <typename KT>
__device__ __forceinline__ float sqrt_rn(float s) {
  if constexpr (sizeof(KT) == 4) {
    return sqrtf(s);
  } else {
    const float r = __builtin_amdgcn_sqrtf(s);
    const float dn = __uint_as_float(__float_as_uint(r) - 1u), up = __uint_as_float(__float_as_uint(r) + 1u);
    const float e_dn = __builtin_fmaf(-dn, r, s), e_up = __builtin_fmaf(-up, r, s);
    float out = e_dn <= 0.f ? dn : r;
    out = e_up > 0.f ? up : out;
    return s == 0.f ? 0.f : out;
  }
}
// min / max of non-negative floats through their bit patterns (no NaN canonicalisation needed)
__device__ __forceinline__ float min_nonneg(float p, float q) {
  return __uint_as_float(min(__float_as_uint(p), __float_as_uint(q)));
}
__device__ __forceinline__ float max_nonneg(float p, float q) {
  return __uint_as_float(max(__float_as_uint(p), __float_as_uint(q)));
}

// Encodes one group (page) of one KV head with the 256 threads of the calling work-group.
// `keys` points at the head's d elements of the group's first token; rows are token_stride
// elements apart; nv <= 128 tokens are valid.  codes_ph / params_ph are the (page, head) slices
// of the pools.  Contains a work-group barrier: all threads must call it.
// LDS of encode_group: per-wavefront minima / maxima of the radii (and of the angles).
template <bool GA>
struct EncodeShared {
  float mn[kEncThreads / 64][kPairs];
  float mx[kEncThreads / 64][kPairs];
  double tmn[GA ? kEncThreads / 64 : 1][GA ? kPairs : 1];
  double tmx[GA ? kEncThreads / 64 : 1][GA ? kPairs : 1];
};

__device__ __forceinline__ uint32_t pack_half2(float lo, float hi) {
  return static_cast<uint32_t>(__half_as_ushort(__float2half_rn(lo))) |
         (static_cast<uint32_t>(__half_as_ushort(__float2half_rn(hi))) << 16);
}

template <int RB, int TB, typename KT, bool GA>
__device__ __forceinline__ void encode_group(const KT* keys, int64_t token_stride, int nv, uint8_t* codes_ph,
                                             uint32_t* params_ph, const double* tan_edge, EncodeShared<GA>& sh) {
  float(*s_mn)[kPairs] = sh.mn;
  float(*s_mx)[kPairs] = sh.mx;
  constexpr int W = RB + TB;
  constexpr int UB = 2 * W;
  const int tid = threadIdx.x;
  const int o = tid & 7;          // pairs 8o .. 8o+7
  const int slot = tid >> 3;      // tokens slot, slot+32, slot+64, slot+96
  const int wave = tid >> 6;

  float rho[kItems][8];
  uint32_t ang[kItems][2];        // 8 angle codes, one byte each
  double th[GA ? kItems : 1][8];  // grouped angle quantizer: theta of every pair
  float mn[8], mx[8];
  double tmn[8], tmx[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) { mn[e] = INFINITY; mx[e] = 0.f; tmn[e] = 4.0; tmx[e] = -4.0; }

  const KT* base = keys + o * 8;
#pragma unroll
  for (int it = 0; it < kItems; ++it) {
    const int tok = slot + 32 * it;
    ang[it][0] = ang[it][1] = 0u;
    if (tok < nv) {
      float x[8], y[8];
      const KT* p = base + tok * token_stride;
      load8(p, x);
      load8(p + kPairs, y);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float xx = x[e] * x[e];
        const float yy = y[e] * y[e];
        const float r = sqrt_rn<KT>(xx + yy);
        rho[it][e] = r;
        mn[e] = min_nonneg(mn[e], r);
        mx[e] = max_nonneg(mx[e], r);
        if constexpr (GA) {
          const double t = atan2(static_cast<double>(y[e]), static_cast<double>(x[e]));
          th[it][e] = t;
          tmn[e] = fmin(tmn[e], t);
          tmx[e] = fmax(tmx[e], t);
        } else {
          // the short rule; the full one only when some lane's pair sits on an axis, a diagonal or
          // the origin (a few per cent of the wavefront steps with fp16 keys)
          bool interior;
          uint32_t bin = angle_bin_interior<TB>(x[e], y[e], tan_edge, interior);
          if (__builtin_amdgcn_ballot_w64(!interior) != 0) bin = interior ? bin : angle_bin<TB>(x[e], y[e], tan_edge);
          ang[it][e >> 2] |= bin << (8 * (e & 3));
        }
      }
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) rho[it][e] = 0.f;
    }
  }

  // group statistics: over the 8 token slots of this wavefront, then over the 4 wavefronts
#pragma unroll
  for (int e = 0; e < 8; ++e) {
#pragma unroll
    for (int m = 8; m < 64; m <<= 1) {
      mn[e] = min_nonneg(mn[e], __shfl_xor(mn[e], m));
      mx[e] = max_nonneg(mx[e], __shfl_xor(mx[e], m));
      if constexpr (GA) {
        tmn[e] = fmin(tmn[e], __shfl_xor(tmn[e], m));
        tmx[e] = fmax(tmx[e], __shfl_xor(tmx[e], m));
      }
    }
  }
  if ((tid & 63) < 8) {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      s_mn[wave][o * 8 + e] = mn[e];
      s_mx[wave][o * 8 + e] = mx[e];
      if constexpr (GA) {
        sh.tmn[wave][o * 8 + e] = tmn[e];
        sh.tmx[wave][o * 8 + e] = tmx[e];
      }
    }
  }
  __syncthreads();

  float sf[8], zf[8];
  uint32_t packed_params[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    float lo = s_mn[0][o * 8 + e], hi = s_mx[0][o * 8 + e];
#pragma unroll
    for (int w = 1; w < kEncThreads / 64; ++w) {
      lo = min_nonneg(lo, s_mn[w][o * 8 + e]);
      hi = max_nonneg(hi, s_mx[w][o * 8 + e]);
    }
    const float s32 = (hi - lo) * (1.0f / static_cast<float>(1 << RB));   // exact scaling by 2^-r
    const __half sh = __float2half_rn(s32), zh = __float2half_rn(lo);      // stored in 16 bits (Appendix B.1)
    sf[e] = __half2float(sh);
    zf[e] = __half2float(zh);
    packed_params[e] = static_cast<uint32_t>(__half_as_ushort(sh)) |
                       (static_cast<uint32_t>(__half_as_ushort(zh)) << 16);
  }
  if (slot == 0) {
    uint4* dst = reinterpret_cast<uint4*>(params_ph + o * 8);
    dst[0] = make_uint4(packed_params[0], packed_params[1], packed_params[2], packed_params[3]);
    dst[1] = make_uint4(packed_params[4], packed_params[5], packed_params[6], packed_params[7]);
  }
  // grouped angle quantizer: (s_t, z_t) of this thread's 8 pairs, as stored
  double ts[8], tz[8];
  if constexpr (GA) {
    uint32_t packed_t[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      double lo = sh.tmn[0][o * 8 + e], hi = sh.tmx[0][o * 8 + e];
#pragma unroll
      for (int w = 1; w < kEncThreads / 64; ++w) {
        lo = fmin(lo, sh.tmn[w][o * 8 + e]);
        hi = fmax(hi, sh.tmx[w][o * 8 + e]);
      }
      ts[e] = round_to_half((hi - lo) * (1.0 / static_cast<double>(1 << TB)));   // exact scaling by 2^-t
      tz[e] = round_to_half(lo);
      packed_t[e] = pack_half2(static_cast<float>(ts[e]), static_cast<float>(tz[e]));   // exact conversions
    }
    if (slot == 0) {
      uint4* dst = reinterpret_cast<uint4*>(params_ph + kPairs + o * 8);
      dst[0] = make_uint4(packed_t[0], packed_t[1], packed_t[2], packed_t[3]);
      dst[1] = make_uint4(packed_t[4], packed_t[5], packed_t[6], packed_t[7]);
    }
  }

  // radius codes, symbols, and the bit string of this thread's 8 pairs (8*W bits)
  uint8_t* const cbase = codes_ph + (o >> 1) * kGroup * UB;
#pragma unroll
  for (int it = 0; it < kItems; ++it) {
    const int tok = slot + 32 * it;
    uint64_t bits = 0;
    if (tok < nv) {
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        float qf = floorf((rho[it][e] - zf[e]) / sf[e]);    // IEEE division
        qf = fminf(fmaxf(qf, 0.f), static_cast<float>((1 << RB) - 1));
        qf = sf[e] != 0.f ? qf : 0.f;                       // constant group: code 0 (also drops the NaN of 0/0)
        uint32_t ac;
        if constexpr (GA) {
          double u = floor((th[it][e] - tz[e]) / ts[e]);     // IEEE division
          u = fmin(fmax(u, 0.0), static_cast<double>((1 << TB) - 1));
          ac = ts[e] != 0.0 ? static_cast<uint32_t>(u) : 0u;  // constant group: code 0
        } else {
          ac = (ang[it][e >> 2] >> (8 * (e & 3))) & 0xffu;
        }
        const uint64_t sym = (static_cast<uint64_t>(ac) << RB) | static_cast<uint32_t>(qf);
        bits |= sym << (e * W);
      }
    }
    // the even lane of each (o, o^1) pair stores the whole 16-pair unit
    const uint32_t lo32 = static_cast<uint32_t>(bits), hi32 = static_cast<uint32_t>(bits >> 32);
    const uint32_t plo = __shfl_xor(lo32, 1), phi = __shfl_xor(hi32, 1);
    if ((o & 1) == 0) {
      uint8_t* dst = cbase + tok * UB;
      if constexpr (W == 8) {
        *reinterpret_cast<uint4*>(dst) = make_uint4(lo32, hi32, plo, phi);
      } else {
        static_assert(W == 6, "unit width");
        uint32_t* d32 = reinterpret_cast<uint32_t*>(dst);
        d32[0] = lo32;
        d32[1] = (hi32 & 0xffffu) | (plo << 16);
        d32[2] = (plo >> 16) | (phi << 16);
      }
    }
  }
}

template <int RB, int TB, typename KT, bool GA>
__global__ __launch_bounds__(kEncThreads) void pq_encode_kernel(const EncodeArgs a) {
  __shared__ EncodeShared<GA> stats;
  const int grp = blockIdx.x, kvh = blockIdx.y;
  const int64_t page = a.page_ids[grp];
  if (page < 0 || page >= a.n_pool_pages) return;
  const int64_t tok0 = static_cast<int64_t>(grp) * kGroup;
  const int nv = static_cast<int>(min<int64_t>(kGroup, a.n_tokens - tok0));
  const int64_t ph = page * a.n_kv_heads + kvh;
  encode_group<RB, TB, KT, GA>(static_cast<const KT*>(a.keys) + tok0 * a.token_stride + kvh * a.head_stride,
                               a.token_stride, nv, a.codes + ph * (kBlocks * kGroup * 2 * (RB + TB)),
                               a.params + ph * (kPairs * (GA ? 2 : 1)), a.tan_edge, stats);
}

// Appends one decode step's key per sequence to the fp16 residual buffer and, when that fills a
// group of 128 tokens, encodes the group into its page (the residual mechanism the paper's
// Appendix B.1 refers to: recent keys stay un-quantized until a full group exists).
struct AppendArgs {
  const void* new_keys;        // [seq][kv_head][d]
  __half* residual;            // [seq][kv_head][g][d]
  const int32_t* seq_lens;     // lengths BEFORE the append
  const int32_t* block_table;
  uint8_t* codes;
  uint32_t* params;
  int64_t n_pool_pages;
  int32_t n_kv_heads;
  int32_t max_pages_per_seq;
  double tan_edge[kMaxAngleBins / 8];
};

template <int RB, int TB, typename KT, bool GA>
__global__ __launch_bounds__(kEncThreads) void pq_append_kernel(const AppendArgs a) {
  __shared__ EncodeShared<GA> stats;
  const int kvh = blockIdx.x, seq = blockIdx.y, tid = threadIdx.x;
  const int L = a.seq_lens[seq];
  if (L < 0) return;
  const int slot = L % kGroup, grp = L / kGroup;
  const int64_t sh = static_cast<int64_t>(seq) * a.n_kv_heads + kvh;
  __half* const res = a.residual + sh * (kGroup * kHeadDim);
  if (tid < kHeadDim / 8) {
    float v[8];
    load8(static_cast<const KT*>(a.new_keys) + sh * kHeadDim + tid * 8, v);
    uint32_t w[4];
#pragma unroll
    for (int e = 0; e < 4; ++e)
      w[e] = static_cast<uint32_t>(__half_as_ushort(__float2half_rn(v[2 * e]))) |
             (static_cast<uint32_t>(__half_as_ushort(__float2half_rn(v[2 * e + 1]))) << 16);
    *reinterpret_cast<uint4*>(res + slot * kHeadDim + tid * 8) = make_uint4(w[0], w[1], w[2], w[3]);
  }
  if (slot != kGroup - 1) return;                 // the group is not complete yet (uniform)
  if (grp >= a.max_pages_per_seq) return;
  const int64_t page = a.block_table[static_cast<int64_t>(seq) * a.max_pages_per_seq + grp];
  if (page < 0 || page >= a.n_pool_pages) return;
  __syncthreads();                                // the new row is visible to the whole work-group
  const int64_t ph = page * a.n_kv_heads + kvh;
  encode_group<RB, TB, __half, GA>(res, kHeadDim, kGroup, a.codes + ph * (kBlocks * kGroup * 2 * (RB + TB)),
                                   a.params + ph * (kPairs * (GA ? 2 : 1)), a.tan_edge, stats);
}

template <int RB, int TB, bool GA = false>
hipError_t launch_encode(const EncodeArgs& a, pq_dtype dt, dim3 grid, hipStream_t st) {
  if (dt == PQ_F16) hipLaunchKernelGGL((pq_encode_kernel<RB, TB, __half, GA>), grid, dim3(kEncThreads), 0, st, a);
  else              hipLaunchKernelGGL((pq_encode_kernel<RB, TB, float, GA>), grid, dim3(kEncThreads), 0, st, a);
  return hipGetLastError();
}

}  // namespace
}  // namespace pq

using namespace pq;

extern "C" int pq_encode_keys(const pq_layout* layout, const void* keys, pq_dtype key_dtype,
                              int64_t token_stride, int64_t head_stride, int64_t n_tokens,
                              const int32_t* page_ids, void* codes_pool, void* params_pool,
                              int64_t n_pool_pages, void* hip_stream) {
  if (!layout) return PQ_ERR_INVALID_ARG;
  if (!layout_supported(layout)) return PQ_ERR_UNSUPPORTED;
  if (n_tokens < 0 || n_pool_pages <= 0) return PQ_ERR_INVALID_ARG;
  if (key_dtype != PQ_F16 && key_dtype != PQ_F32) return PQ_ERR_INVALID_ARG;
  if (n_tokens == 0) return PQ_OK;
  if (!keys || !page_ids || !codes_pool || !params_pool) return PQ_ERR_INVALID_ARG;
  // 128-bit loads: rows of a head must start on 16-byte boundaries
  const int64_t vec = key_dtype == PQ_F16 ? 8 : 4;
  if ((reinterpret_cast<uintptr_t>(keys) & 15u) || token_stride % vec || head_stride % vec ||
      token_stride < kHeadDim || head_stride < 0)
    return PQ_ERR_INVALID_ARG;
  if ((reinterpret_cast<uintptr_t>(codes_pool) & 15u) || (reinterpret_cast<uintptr_t>(params_pool) & 15u))
    return PQ_ERR_INVALID_ARG;
  const int64_t n_groups = (n_tokens + kGroup - 1) / kGroup;
  if (n_groups > 0x7fffffff || layout->n_kv_heads > 65535) return PQ_ERR_UNSUPPORTED;

  EncodeArgs a;
  a.keys = keys;
  a.page_ids = page_ids;
  a.codes = static_cast<uint8_t*>(codes_pool);
  a.params = static_cast<uint32_t*>(params_pool);
  a.token_stride = token_stride;
  a.head_stride = head_stride;
  a.n_tokens = n_tokens;
  a.n_pool_pages = n_pool_pages;
  a.n_kv_heads = layout->n_kv_heads;
  const int nb = 1 << layout->t_bits;
  for (int k = 0; k < kMaxAngleBins / 8; ++k)
    a.tan_edge[k] = (k >= 1 && k < nb / 8) ? tan(k * (2.0 * M_PI / nb)) : 0.0;

  const dim3 grid(static_cast<uint32_t>(n_groups), layout->n_kv_heads);
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  hipError_t e = hipSuccess;
  switch (layout->r_bits * 10 + layout->t_bits + (layout->angle_quantizer == PQ_ANGLE_GROUPED ? 100 : 0)) {
    case 144: e = launch_encode<4, 4, true>(a, key_dtype, grid, st); break;
    case 133: e = launch_encode<3, 3, true>(a, key_dtype, grid, st); break;
    case 153: e = launch_encode<5, 3, true>(a, key_dtype, grid, st); break;
    case 135: e = launch_encode<3, 5, true>(a, key_dtype, grid, st); break;
    case 142: e = launch_encode<4, 2, true>(a, key_dtype, grid, st); break;
    case 124: e = launch_encode<2, 4, true>(a, key_dtype, grid, st); break;
    case 44: e = launch_encode<4, 4>(a, key_dtype, grid, st); break;
    case 33: e = launch_encode<3, 3>(a, key_dtype, grid, st); break;
    case 53: e = launch_encode<5, 3>(a, key_dtype, grid, st); break;
    case 35: e = launch_encode<3, 5>(a, key_dtype, grid, st); break;
    case 42: e = launch_encode<4, 2>(a, key_dtype, grid, st); break;
    case 24: e = launch_encode<2, 4>(a, key_dtype, grid, st); break;
    default: return PQ_ERR_UNSUPPORTED;
  }
  if (e != hipSuccess) return record_hip_error(e);
  return PQ_OK;
}

namespace pq {
namespace {
template <int RB, int TB, bool GA = false>
hipError_t launch_append(const AppendArgs& a, pq_dtype dt, dim3 grid, hipStream_t st) {
  if (dt == PQ_F16) hipLaunchKernelGGL((pq_append_kernel<RB, TB, __half, GA>), grid, dim3(kEncThreads), 0, st, a);
  else              hipLaunchKernelGGL((pq_append_kernel<RB, TB, float, GA>), grid, dim3(kEncThreads), 0, st, a);
  return hipGetLastError();
}
}  // namespace
}  // namespace pq

extern "C" int pq_append_keys(const pq_layout* layout, const void* new_keys, pq_dtype key_dtype, int32_t n_seqs,
                              void* residual, const int32_t* seq_lens, const int32_t* block_table,
                              int32_t max_pages_per_seq, void* codes_pool, void* params_pool,
                              int64_t n_pool_pages, void* hip_stream) {
  if (!layout) return PQ_ERR_INVALID_ARG;
  if (!layout_supported(layout)) return PQ_ERR_UNSUPPORTED;
  if (n_seqs < 0 || n_pool_pages <= 0 || max_pages_per_seq <= 0) return PQ_ERR_INVALID_ARG;
  if (key_dtype != PQ_F16 && key_dtype != PQ_F32) return PQ_ERR_INVALID_ARG;
  if (n_seqs == 0) return PQ_OK;
  if (!new_keys || !residual || !seq_lens || !block_table || !codes_pool || !params_pool) return PQ_ERR_INVALID_ARG;
  if ((reinterpret_cast<uintptr_t>(new_keys) & 15u) || (reinterpret_cast<uintptr_t>(residual) & 15u) ||
      (reinterpret_cast<uintptr_t>(codes_pool) & 15u) || (reinterpret_cast<uintptr_t>(params_pool) & 15u))
    return PQ_ERR_INVALID_ARG;
  if (n_seqs > 65535) return PQ_ERR_UNSUPPORTED;
  AppendArgs a;
  a.new_keys = new_keys;
  a.residual = static_cast<__half*>(residual);
  a.seq_lens = seq_lens;
  a.block_table = block_table;
  a.codes = static_cast<uint8_t*>(codes_pool);
  a.params = static_cast<uint32_t*>(params_pool);
  a.n_pool_pages = n_pool_pages;
  a.n_kv_heads = layout->n_kv_heads;
  a.max_pages_per_seq = max_pages_per_seq;
  const int nb = 1 << layout->t_bits;
  for (int k = 0; k < kMaxAngleBins / 8; ++k)
    a.tan_edge[k] = (k >= 1 && k < nb / 8) ? tan(k * (2.0 * M_PI / nb)) : 0.0;
  const dim3 grid(layout->n_kv_heads, n_seqs);
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  hipError_t e = hipSuccess;
  switch (layout->r_bits * 10 + layout->t_bits + (layout->angle_quantizer == PQ_ANGLE_GROUPED ? 100 : 0)) {
    case 144: e = launch_append<4, 4, true>(a, key_dtype, grid, st); break;
    case 133: e = launch_append<3, 3, true>(a, key_dtype, grid, st); break;
    case 153: e = launch_append<5, 3, true>(a, key_dtype, grid, st); break;
    case 135: e = launch_append<3, 5, true>(a, key_dtype, grid, st); break;
    case 142: e = launch_append<4, 2, true>(a, key_dtype, grid, st); break;
    case 124: e = launch_append<2, 4, true>(a, key_dtype, grid, st); break;
    case 44: e = launch_append<4, 4>(a, key_dtype, grid, st); break;
    case 33: e = launch_append<3, 3>(a, key_dtype, grid, st); break;
    case 53: e = launch_append<5, 3>(a, key_dtype, grid, st); break;
    case 35: e = launch_append<3, 5>(a, key_dtype, grid, st); break;
    case 42: e = launch_append<4, 2>(a, key_dtype, grid, st); break;
    case 24: e = launch_append<2, 4>(a, key_dtype, grid, st); break;
    default: return PQ_ERR_UNSUPPORTED;
  }
  if (e != hipSuccess) return record_hip_error(e);
  return PQ_OK;
}
