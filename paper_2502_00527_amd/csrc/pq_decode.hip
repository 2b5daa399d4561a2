// Host entry points of the decode path (pq_decode_*, pq_score_keys) and the chunk merge kernel.
// The attention and score-only kernel templates live in pq_decode_kernels.hpp.
#include <mutex>

#include "pq_decode_kernels.hpp"
#include "pq_decode_roles.hpp"

// Which attention kernel serves fp16 values with the uniform angle grid: the role-specialised
// one (1) or the one whose wavefronts alternate between a score and a value phase (0).
#ifndef PQ_USE_ROLES
#define PQ_USE_ROLES 1
#endif

// Scratch of pq_decode_attention_static: the chunk partials live here instead of in a
// caller-supplied workspace.  One copy per GPU, at its own address on each.
static __device__ __align__(256) unsigned char scratch[PQ_STATIC_SCRATCH_BYTES];

namespace pq {

namespace {

// out[seq][head][:] = sum_c 2^(m_c - M) acc_c / sum_c 2^(m_c - M) l_c over the chunks the
// sequence really has.  One work-group of 256 threads per (head, seq).  The maximum M is found
// with one (m, l) pair per thread and a shuffle / LDS reduction; then thread = (chunk slice
// tid / 32, dims 4 * (tid % 32) ..+3) and the eight slices take chunks c = slice, slice + 8, ...
// with independent 128-bit loads before they are folded through LDS.
constexpr int kMergeThreads = 256;
constexpr int kMergeSlices = kMergeThreads / 32;

__global__ __launch_bounds__(kMergeThreads) void pq_decode_merge_kernel(
    const float* __restrict__ ws_acc, const float* __restrict__ ws_ml,
    const int32_t* __restrict__ seq_lens, float* __restrict__ out, int32_t n_q_heads,
    int32_t max_seq_len, int32_t pages_per_chunk, int32_t n_chunks) {
  __shared__ float4 part_o[kMergeSlices][32];
  __shared__ float part_l[kMergeSlices];
  __shared__ float wave_max[kMergeThreads / 64];
  const int head = blockIdx.x, seq = blockIdx.y, tid = threadIdx.x;
  const int slice = tid >> 5, quad = tid & 31;
  const int L = min(seq_lens[seq], max_seq_len);
  const int64_t oh = static_cast<int64_t>(seq) * n_q_heads + head;
  if (L <= 0) {
    if (tid < kHeadDim) out[oh * kHeadDim + tid] = 0.f;
    return;
  }
  const int n_pages = (L + kGroup - 1) / kGroup;
  const int nc = (n_pages + pages_per_chunk - 1) / pages_per_chunk;
  const float2* ml = reinterpret_cast<const float2*>(ws_ml) + oh * n_chunks;
  const float4* ac = reinterpret_cast<const float4*>(ws_acc + oh * n_chunks * kHeadDim) + quad;

  float m = kNegInf;
  for (int c = tid; c < nc; c += kMergeThreads) m = fmaxf(m, ml[c].x);
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) m = fmaxf(m, __shfl_xor(m, d));
  if ((tid & 63) == 0) wave_max[tid >> 6] = m;
  __syncthreads();
  const float M = fmaxf(fmaxf(wave_max[0], wave_max[1]), fmaxf(wave_max[2], wave_max[3]));

  float4 o = make_float4(0.f, 0.f, 0.f, 0.f);
  float l = 0.f;
  if (M > kNegInf) {
#pragma unroll 4
    for (int c = slice; c < nc; c += kMergeSlices) {
      const float2 mlc = ml[c];
      const float4 v = ac[static_cast<int64_t>(c) * (kHeadDim / 4)];
      const float w = __builtin_amdgcn_exp2f(mlc.x - M);
      o.x = fmaf(w, v.x, o.x);
      o.y = fmaf(w, v.y, o.y);
      o.z = fmaf(w, v.z, o.z);
      o.w = fmaf(w, v.w, o.w);
      l = fmaf(w, mlc.y, l);
    }
  }
  part_o[slice][quad] = o;
  if (quad == 0) part_l[slice] = l;
  __syncthreads();
  if (slice == 0) {
    float lt = 0.f;
    float4 r = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
    for (int s2 = 0; s2 < kMergeSlices; ++s2) {
      const float4 t = part_o[s2][quad];
      r.x += t.x; r.y += t.y; r.z += t.z; r.w += t.w;
      lt += part_l[s2];
    }
    const float inv = lt > 0.f ? 1.f / lt : 0.f;
    reinterpret_cast<float4*>(out + oh * kHeadDim)[quad] = make_float4(r.x * inv, r.y * inv, r.z * inv, r.w * inv);
  }
}

// order[rank] = index of the sequence with `rank` longer ones before it (ties: lower index first).
// One work-group; every thread ranks the sequences t, t + 1024, ... against all lengths in LDS.
constexpr int kOrderMax = 2048;
__global__ __launch_bounds__(1024) void pq_order_kernel(const int32_t* __restrict__ seq_lens, int32_t n_seqs,
                                                        int32_t* __restrict__ order) {
  __shared__ int32_t len_s[kOrderMax];
  for (int i = threadIdx.x; i < n_seqs; i += blockDim.x) {
    if (n_seqs > kOrderMax) order[i] = i;
    else len_s[i] = seq_lens[i];
  }
  if (n_seqs > kOrderMax) return;
  __syncthreads();
  for (int i = threadIdx.x; i < n_seqs; i += blockDim.x) {
    const int32_t mine = len_s[i];
    int rank = 0;
    for (int j = 0; j < n_seqs; ++j) {
      const int32_t other = len_s[j];
      rank += (other > mine) || (other == mine && j < i);
    }
    order[rank] = i;
  }
}

template <int RB, int TB>
hipError_t launch_scores(int G, const DecodeArgs& a, pq_dtype qdt, dim3 grid, hipStream_t st) {
#define PQ_LAUNCH_SCORES(GG)                                                                            \
  if (qdt == PQ_F16) hipLaunchKernelGGL((pq_score_keys_kernel<GG, RB, TB, __half>), grid, dim3(kThreads), 0, st, a); \
  else hipLaunchKernelGGL((pq_score_keys_kernel<GG, RB, TB, float>), grid, dim3(kThreads), 0, st, a)
  switch (G) {
    case 1: PQ_LAUNCH_SCORES(1); break;
    case 2: PQ_LAUNCH_SCORES(2); break;
    default: PQ_LAUNCH_SCORES(4); break;
  }
#undef PQ_LAUNCH_SCORES
  return hipGetLastError();
}

struct Workspace {
  float* acc;
  float* ml;
  size_t bytes;
};

Workspace carve_workspace(void* base, int32_t n_seqs, int32_t n_q_heads, int32_t n_chunks) {
  const size_t slots = static_cast<size_t>(n_seqs) * n_q_heads * n_chunks;
  const size_t acc_bytes = (slots * kHeadDim * sizeof(float) + 255) & ~static_cast<size_t>(255);
  const size_t ml_bytes = (slots * 2 * sizeof(float) + 255) & ~static_cast<size_t>(255);
  Workspace w;
  w.acc = static_cast<float*>(base);
  w.ml = reinterpret_cast<float*>(static_cast<uint8_t*>(base) + acc_bytes);
  w.bytes = acc_bytes + ml_bytes;
  return w;
}

template <int G, int RB, int TB>
hipError_t launch_partials(const DecodeArgs& a, pq_dtype qdt, dim3 grid, hipStream_t st) {
  const bool sc = a.scores != nullptr;
  if (qdt == PQ_F16) {
    if (sc) hipLaunchKernelGGL((pq_decode_partials_kernel<G, RB, TB, __half, true, 16>), grid, dim3(kThreads), 0, st, a);
    else    hipLaunchKernelGGL((pq_decode_partials_kernel<G, RB, TB, __half, false, 16>), grid, dim3(kThreads), 0, st, a);
  } else {
    if (sc) hipLaunchKernelGGL((pq_decode_partials_kernel<G, RB, TB, float, true, 16>), grid, dim3(kThreads), 0, st, a);
    else    hipLaunchKernelGGL((pq_decode_partials_kernel<G, RB, TB, float, false, 16>), grid, dim3(kThreads), 0, st, a);
  }
  return hipGetLastError();
}

template <int RB, int TB>
hipError_t launch_partials_g(int G, const DecodeArgs& a, pq_dtype qdt, dim3 grid, hipStream_t st) {
  switch (G) {
    case 1: return launch_partials<1, RB, TB>(a, qdt, grid, st);
    case 2: return launch_partials<2, RB, TB>(a, qdt, grid, st);
    default: return launch_partials<4, RB, TB>(a, qdt, grid, st);
  }
}

// cos / sin of the centre of every angle bin of the uniform grid over [-pi, pi) (Section 3.2
// mid-point reconstruction), evaluated in float64 on the host.
void fill_angle_tables(DecodeArgs& a, int t_bits) {
  const int nb = 1 << t_bits;
  for (int s = 0; s < kMaxAngleBins; ++s) {
    const double th = -M_PI + (s + 0.5) * (2.0 * M_PI / nb);
    a.cos_tab[s] = s < nb ? static_cast<float>(cos(th)) : 0.f;
    a.sin_tab[s] = s < nb ? static_cast<float>(sin(th)) : 0.f;
  }
}

// Which attention kernel a launch gets.  The role-specialised kernel serves fp16 values with the
// uniform angle grid when the launch has at least 256 work-groups; launches of a few work-groups
// stay with the kernel whose four wavefronts share a chunk's pages four ways (measured: 9
// against 12 us for one head over 4096 tokens).
enum class AttentionKernel { kPartials, kRoles };
AttentionKernel choose_attention_kernel(const pq_layout* l, int32_t v_bits, int64_t n_groups) {
  if (PQ_USE_ROLES && l->angle_quantizer == PQ_ANGLE_UNIFORM && v_bits == 16 && n_groups >= 256)
    return AttentionKernel::kRoles;
  return AttentionKernel::kPartials;
}

// Device address of `scratch` on the current device (in host code the array's name is only a
// handle for the lookup, not an address a kernel can use).  Resolved once per device.
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

int static_scratch(void** ptr_out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return record_hip_error(e);
  if (dev < 0 || dev >= kMaxDevices) return PQ_ERR_UNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return record_hip_error(e);
    if (!p || (reinterpret_cast<uintptr_t>(p) & 255u)) return PQ_ERR_WORKSPACE;
    g_scratch_ptr[dev] = p;
  }
  *ptr_out = g_scratch_ptr[dev];
  return PQ_OK;
}

int check_decode_shape(const pq_layout* l, int32_t n_seqs, int32_t n_q_heads, int32_t max_seq_len) {
  if (!l || n_seqs <= 0 || n_q_heads <= 0 || max_seq_len <= 0) return PQ_ERR_INVALID_ARG;
  if (l->n_kv_heads <= 0 || n_q_heads % l->n_kv_heads != 0) return PQ_ERR_INVALID_ARG;
  if (!layout_supported(l)) return PQ_ERR_UNSUPPORTED;
  const int G = n_q_heads / l->n_kv_heads;
  if (G > 16) return PQ_ERR_UNSUPPORTED;   // groups are processed 4, 2 or 1 query heads per pass
  if (n_seqs > 65535 || n_q_heads > 65535) return PQ_ERR_UNSUPPORTED;   // grid.y, merge grid.x
  if (plan_chunks(n_seqs, l->n_kv_heads, max_seq_len).n_chunks > 65535) return PQ_ERR_UNSUPPORTED;   // grid.z
  return PQ_OK;
}

}  // namespace

}  // namespace pq

using namespace pq;

extern "C" size_t pq_decode_workspace_bytes(const pq_layout* layout, int32_t n_seqs, int32_t n_q_heads,
                                            int32_t max_seq_len) {
  if (check_decode_shape(layout, n_seqs, n_q_heads, max_seq_len) != PQ_OK) return 0;
  const ChunkPlan plan = plan_chunks(n_seqs, layout->n_kv_heads, max_seq_len);
  return carve_workspace(nullptr, n_seqs, n_q_heads, plan.n_chunks).bytes;
}

extern "C" int pq_decode_partials(const pq_layout* layout, const void* q, pq_dtype q_dtype, int32_t n_seqs,
                                  int32_t n_q_heads, const void* codes_pool, const void* params_pool,
                                  const void* v_pool, int32_t v_bits, const void* v_params_pool,
                                  int64_t n_pool_pages, const int32_t* block_table,
                                  int32_t max_pages_per_seq, const int32_t* seq_lens, int32_t max_seq_len,
                                  float sm_scale, float* scores, int64_t scores_stride,
                                  const void* residual_keys, const int32_t* seq_order, void* workspace,
                                  size_t workspace_bytes, void* hip_stream) {
  const int st = check_decode_shape(layout, n_seqs, n_q_heads, max_seq_len);
  if (st != PQ_OK) return st;
  if (!q || !codes_pool || !params_pool || !v_pool || !block_table || !seq_lens) return PQ_ERR_INVALID_ARG;
  if (q_dtype != PQ_F16 && q_dtype != PQ_F32) return PQ_ERR_INVALID_ARG;
  if (n_pool_pages <= 0 || max_pages_per_seq <= 0) return PQ_ERR_INVALID_ARG;
  const int64_t need_pages = (static_cast<int64_t>(max_seq_len) + kGroup - 1) / kGroup;
  if (need_pages > max_pages_per_seq) return PQ_ERR_INVALID_ARG;
  if (scores && scores_stride < max_seq_len) return PQ_ERR_INVALID_ARG;
  if (!isfinite(sm_scale)) return PQ_ERR_INVALID_ARG;
  if (reinterpret_cast<uintptr_t>(residual_keys) & 15u) return PQ_ERR_INVALID_ARG;
  if (v_bits != 16 && v_bits != 4 && v_bits != 2) return PQ_ERR_UNSUPPORTED;
  if (v_bits != 16 && !v_params_pool) return PQ_ERR_INVALID_ARG;

  const ChunkPlan plan = plan_chunks(n_seqs, layout->n_kv_heads, max_seq_len);
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u)) return PQ_ERR_WORKSPACE;
  const Workspace ws = carve_workspace(workspace, n_seqs, n_q_heads, plan.n_chunks);
  if (workspace_bytes < ws.bytes) return PQ_ERR_WORKSPACE;

  DecodeArgs a;
  a.q = q;
  a.codes = static_cast<const uint8_t*>(codes_pool);
  a.params = static_cast<const uint32_t*>(params_pool);
  a.values = static_cast<const __half*>(v_pool);
  a.residual = static_cast<const __half*>(residual_keys);
  a.v_params = static_cast<const uint32_t*>(v_params_pool);
  a.block_table = block_table;
  a.seq_lens = seq_lens;
  a.seq_order = seq_order;
  a.n_seqs = n_seqs;
  a.scores = scores;
  a.ws_acc = ws.acc;
  a.ws_ml = ws.ml;
  a.scores_stride = scores_stride;
  a.n_pool_pages = n_pool_pages;
  a.n_kv_heads = layout->n_kv_heads;
  a.n_q_heads = n_q_heads;
  a.max_pages_per_seq = max_pages_per_seq;
  a.max_seq_len = max_seq_len;
  a.pages_per_chunk = plan.pages_per_chunk;
  a.n_chunks = plan.n_chunks;
  a.scale_log2 = static_cast<float>(static_cast<double>(sm_scale) * 1.4426950408889634074);
  fill_angle_tables(a, layout->t_bits);

  const dim3 grid(layout->n_kv_heads, n_seqs, plan.n_chunks);
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const int group_total = n_q_heads / layout->n_kv_heads;
  hipError_t e = hipSuccess;
  const int rt = layout->r_bits * 10 + layout->t_bits;
  // A kernel instance serves 4, 2 or 1 query heads of a KV head; larger or odd groups take
  // several passes over the cache (6 = 4 + 2, 8 = 4 + 4, ...).
  a.group_total = group_total;
  for (int head0 = 0; head0 < group_total && e == hipSuccess;) {
    const int left = group_total - head0;
    const int G = left >= 4 ? 4 : (left >= 2 ? 2 : 1);
    a.head0 = head0;
    if (layout->angle_quantizer == PQ_ANGLE_GROUPED) {
      e = v_bits == 16 ? launch_partials_ga(rt, G, a, q_dtype, grid, stream)
                       : launch_partials_ga_vq(rt, G, v_bits, a, q_dtype, grid, stream);
      if (e == hipErrorInvalidValue) return PQ_ERR_UNSUPPORTED;
    } else if (v_bits != 16) {
      e = launch_partials_vq(rt, G, v_bits, a, q_dtype, grid, stream);
      if (e == hipErrorInvalidValue) return PQ_ERR_UNSUPPORTED;   // quantized values: (r,t) = (4,4), (3,3) only
    } else if (choose_attention_kernel(layout, v_bits, static_cast<int64_t>(grid.x) * grid.y * grid.z) ==
               AttentionKernel::kRoles) {
      e = launch_partials_roles(rt, G, a, q_dtype, grid, stream);
      if (e == hipErrorInvalidValue) return PQ_ERR_UNSUPPORTED;
    } else {
      switch (rt) {
        case 44: e = launch_partials_g<4, 4>(G, a, q_dtype, grid, stream); break;
        case 33: e = launch_partials_g<3, 3>(G, a, q_dtype, grid, stream); break;
        case 53: e = launch_partials_g<5, 3>(G, a, q_dtype, grid, stream); break;
        case 35: e = launch_partials_g<3, 5>(G, a, q_dtype, grid, stream); break;
        case 42: e = launch_partials_g<4, 2>(G, a, q_dtype, grid, stream); break;
        case 24: e = launch_partials_g<2, 4>(G, a, q_dtype, grid, stream); break;
        default: return PQ_ERR_UNSUPPORTED;
      }
    }
    head0 += G;
  }
  if (e != hipSuccess) return record_hip_error(e);
  return PQ_OK;
}

extern "C" const char* pq_decode_kernel_name(const pq_layout* layout, int32_t n_seqs, int32_t n_q_heads,
                                             int32_t max_seq_len, int32_t v_bits) {
  if (check_decode_shape(layout, n_seqs, n_q_heads, max_seq_len) != PQ_OK) return "";
  const ChunkPlan plan = plan_chunks(n_seqs, layout->n_kv_heads, max_seq_len);
  const int64_t n_groups = static_cast<int64_t>(layout->n_kv_heads) * n_seqs * plan.n_chunks;
  return choose_attention_kernel(layout, v_bits, n_groups) == AttentionKernel::kRoles
             ? "pq_decode_roles_kernel" : "pq_decode_partials_kernel";
}

extern "C" int pq_order_sequences(const int32_t* seq_lens, int32_t n_seqs, int32_t* order_out, void* hip_stream) {
  if (n_seqs < 0) return PQ_ERR_INVALID_ARG;
  if (n_seqs == 0) return PQ_OK;
  if (!seq_lens || !order_out) return PQ_ERR_INVALID_ARG;
  hipLaunchKernelGGL(pq_order_kernel, dim3(1), dim3(1024), 0, static_cast<hipStream_t>(hip_stream), seq_lens,
                     n_seqs, order_out);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return record_hip_error(e);
  return PQ_OK;
}

extern "C" int pq_decode_merge(const pq_layout* layout, int32_t n_seqs, int32_t n_q_heads,
                               const int32_t* seq_lens, int32_t max_seq_len, float* out,
                               const void* workspace, size_t workspace_bytes, void* hip_stream) {
  const int st = check_decode_shape(layout, n_seqs, n_q_heads, max_seq_len);
  if (st != PQ_OK) return st;
  if (!seq_lens || !out) return PQ_ERR_INVALID_ARG;
  const ChunkPlan plan = plan_chunks(n_seqs, layout->n_kv_heads, max_seq_len);
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u)) return PQ_ERR_WORKSPACE;
  const Workspace ws = carve_workspace(const_cast<void*>(workspace), n_seqs, n_q_heads, plan.n_chunks);
  if (workspace_bytes < ws.bytes) return PQ_ERR_WORKSPACE;
  hipLaunchKernelGGL(pq_decode_merge_kernel, dim3(n_q_heads, n_seqs), dim3(kMergeThreads), 0,
                     static_cast<hipStream_t>(hip_stream), ws.acc, ws.ml, seq_lens, out, n_q_heads,
                     max_seq_len, plan.pages_per_chunk, plan.n_chunks);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return record_hip_error(e);
  return PQ_OK;
}

extern "C" int pq_decode_attention(const pq_layout* layout, const void* q, pq_dtype q_dtype, int32_t n_seqs,
                                   int32_t n_q_heads, const void* codes_pool, const void* params_pool,
                                   const void* v_pool, int32_t v_bits, const void* v_params_pool,
                                   int64_t n_pool_pages, const int32_t* block_table,
                                   int32_t max_pages_per_seq, const int32_t* seq_lens, int32_t max_seq_len,
                                   float sm_scale, float* out, float* scores, int64_t scores_stride,
                                   const void* residual_keys, const int32_t* seq_order, void* workspace,
                                   size_t workspace_bytes, void* hip_stream) {
  if (!out) return PQ_ERR_INVALID_ARG;
  const int st = pq_decode_partials(layout, q, q_dtype, n_seqs, n_q_heads, codes_pool, params_pool, v_pool,
                                    v_bits, v_params_pool, n_pool_pages, block_table, max_pages_per_seq, seq_lens, max_seq_len,
                                    sm_scale, scores, scores_stride, residual_keys, seq_order, workspace,
                                    workspace_bytes, hip_stream);
  if (st != PQ_OK) return st;
  return pq_decode_merge(layout, n_seqs, n_q_heads, seq_lens, max_seq_len, out, workspace, workspace_bytes,
                         hip_stream);
}

extern "C" int pq_decode_attention_static(const pq_layout* layout, const void* q, pq_dtype q_dtype, int32_t n_seqs,
                                          int32_t n_q_heads, const void* codes_pool, const void* params_pool,
                                          const void* v_pool, int32_t v_bits, const void* v_params_pool,
                                          int64_t n_pool_pages, const int32_t* block_table,
                                          int32_t max_pages_per_seq, const int32_t* seq_lens, int32_t max_seq_len,
                                          float sm_scale, float* out, float* scores, int64_t scores_stride,
                                          const void* residual_keys, const int32_t* seq_order, void* hip_stream) {
  const int st = check_decode_shape(layout, n_seqs, n_q_heads, max_seq_len);
  if (st != PQ_OK) return st;
  const size_t need = pq_decode_workspace_bytes(layout, n_seqs, n_q_heads, max_seq_len);
  if (need == 0 || need > static_cast<size_t>(PQ_STATIC_SCRATCH_BYTES)) return PQ_ERR_STATIC_LIMIT;
  void* ws = nullptr;
  const int sp = static_scratch(&ws);
  if (sp != PQ_OK) return sp;
  return pq_decode_attention(layout, q, q_dtype, n_seqs, n_q_heads, codes_pool, params_pool, v_pool, v_bits,
                             v_params_pool, n_pool_pages, block_table, max_pages_per_seq, seq_lens, max_seq_len,
                             sm_scale, out, scores, scores_stride, residual_keys, seq_order, ws, need, hip_stream);
}

extern "C" int pq_score_keys(const pq_layout* layout, const void* q, pq_dtype q_dtype, int32_t n_seqs,
                             int32_t n_q_heads, const void* codes_pool, const void* params_pool,
                             int64_t n_pool_pages, const int32_t* block_table, int32_t max_pages_per_seq,
                             const int32_t* seq_lens, int32_t max_seq_len, float* scores,
                             int64_t scores_stride, const void* residual_keys, void* hip_stream) {
  const int st = check_decode_shape(layout, n_seqs, n_q_heads, max_seq_len);
  if (st != PQ_OK) return st;
  if (!q || !codes_pool || !params_pool || !block_table || !seq_lens || !scores) return PQ_ERR_INVALID_ARG;
  if (q_dtype != PQ_F16 && q_dtype != PQ_F32) return PQ_ERR_INVALID_ARG;
  if (n_pool_pages <= 0 || max_pages_per_seq <= 0 || scores_stride < max_seq_len) return PQ_ERR_INVALID_ARG;
  const int64_t need_pages = (static_cast<int64_t>(max_seq_len) + kGroup - 1) / kGroup;
  if (need_pages > max_pages_per_seq) return PQ_ERR_INVALID_ARG;
  if (reinterpret_cast<uintptr_t>(residual_keys) & 15u) return PQ_ERR_INVALID_ARG;
  const ChunkPlan plan = plan_chunks(n_seqs, layout->n_kv_heads, max_seq_len);
  DecodeArgs a = {};
  a.q = q;
  a.residual = static_cast<const __half*>(residual_keys);
  a.codes = static_cast<const uint8_t*>(codes_pool);
  a.params = static_cast<const uint32_t*>(params_pool);
  a.block_table = block_table;
  a.seq_lens = seq_lens;
  a.n_seqs = n_seqs;
  a.scores = scores;
  a.scores_stride = scores_stride;
  a.n_pool_pages = n_pool_pages;
  a.n_kv_heads = layout->n_kv_heads;
  a.n_q_heads = n_q_heads;
  a.max_pages_per_seq = max_pages_per_seq;
  a.max_seq_len = max_seq_len;
  a.pages_per_chunk = plan.pages_per_chunk;
  a.n_chunks = plan.n_chunks;
  fill_angle_tables(a, layout->t_bits);
  const dim3 grid(layout->n_kv_heads, n_seqs, plan.n_chunks);
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const int group_total = n_q_heads / layout->n_kv_heads;
  hipError_t e = hipSuccess;
  a.group_total = group_total;
  for (int head0 = 0; head0 < group_total && e == hipSuccess;) {
    const int left = group_total - head0;
    const int G = left >= 4 ? 4 : (left >= 2 ? 2 : 1);
    a.head0 = head0;
    if (layout->angle_quantizer == PQ_ANGLE_GROUPED) {
      e = launch_scores_ga(layout->r_bits * 10 + layout->t_bits, G, a, q_dtype, grid, stream);
      if (e == hipErrorInvalidValue) return PQ_ERR_UNSUPPORTED;
      head0 += G;
      continue;
    }
    switch (layout->r_bits * 10 + layout->t_bits) {
      case 44: e = launch_scores<4, 4>(G, a, q_dtype, grid, stream); break;
      case 33: e = launch_scores<3, 3>(G, a, q_dtype, grid, stream); break;
      case 53: e = launch_scores<5, 3>(G, a, q_dtype, grid, stream); break;
      case 35: e = launch_scores<3, 5>(G, a, q_dtype, grid, stream); break;
      case 42: e = launch_scores<4, 2>(G, a, q_dtype, grid, stream); break;
      case 24: e = launch_scores<2, 4>(G, a, q_dtype, grid, stream); break;
      default: return PQ_ERR_UNSUPPORTED;
    }
    head0 += G;
  }
  if (e != hipSuccess) return record_hip_error(e);
  return PQ_OK;
}
