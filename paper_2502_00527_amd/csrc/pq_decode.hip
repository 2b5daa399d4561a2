// Host entry points of the decode path (pq_decode_*, pq_score_keys) and the chunk merge kernel.
// The attention and score-only kernel templates live in pq_decode_kernels.hpp.
#include <algorithm>
#include <mutex>

#include "pq_decode_kernels.hpp"
#include "pq_decode_roles.hpp"

// Scratch of pq_decode_attention_static: partials and arrival words live here instead of in a
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

// Score-only kernels: uniform angle grid -> lanes are tokens (pq_score_tokens_kernel); grouped
// quantizer -> the attention kernels' lane layout with a table per page (pq_score_keys_kernel).
template <int G, int RB, int TB, bool GA>
void launch_scores_one(const DecodeArgs& a, dim3 grid, hipStream_t st) {
  if constexpr (GA) hipLaunchKernelGGL((pq_score_keys_kernel<G, RB, TB, true>), grid, dim3(kThreads), 0, st, a);
  else hipLaunchKernelGGL((pq_score_tokens_kernel<G, RB, TB>), grid, dim3(kThreads), 0, st, a);
}
template <int RB, int TB, bool GA>
bool launch_scores_g(int G, const DecodeArgs& a, dim3 grid, hipStream_t st) {
  switch (G) {
    case 1: launch_scores_one<1, RB, TB, GA>(a, grid, st); return true;
    case 2: launch_scores_one<2, RB, TB, GA>(a, grid, st); return true;
    case 4: launch_scores_one<4, RB, TB, GA>(a, grid, st); return true;
    default: return false;
  }
}
template <bool GA>
bool launch_scores_rt(int rt, int G, const DecodeArgs& a, dim3 grid, hipStream_t st) {
  switch (rt) {
    case 44: return launch_scores_g<4, 4, GA>(G, a, grid, st);
    case 33: return launch_scores_g<3, 3, GA>(G, a, grid, st);
    case 53: return launch_scores_g<5, 3, GA>(G, a, grid, st);
    case 35: return launch_scores_g<3, 5, GA>(G, a, grid, st);
    case 42: return launch_scores_g<4, 2, GA>(G, a, grid, st);
    case 24: return launch_scores_g<2, 4, GA>(G, a, grid, st);
    default: return false;
  }
}
bool launch_scores(int rt, bool grouped, int G, const DecodeArgs& a, dim3 grid, hipStream_t st) {
  return grouped ? launch_scores_rt<true>(rt, G, a, grid, st) : launch_scores_rt<false>(rt, G, a, grid, st);
}

// Which attention kernel a launch gets.  The role-specialised kernel, whose work-groups share
// the launch's pages out evenly and merge in the kernel, serves fp16 values with the uniform
// angle grid when there is work for at least 256 work-groups; smaller launches stay with the
// kernel whose four wavefronts share a chunk's pages four ways (measured: 9 against 12 us for one
// head over 4096 tokens).
enum class AttentionKernel { kPartials, kRoles };
constexpr int kComputeUnits = 256;           // MI355X

#ifndef PQ_BALANCED_MIN_PAGES
#define PQ_BALANCED_MIN_PAGES 4
#endif
#ifndef PQ_BALANCED_GROUPS
#define PQ_BALANCED_GROUPS (kComputeUnits * role_groups_per_cu(4))
#endif
constexpr int kBalancedMinPages = PQ_BALANCED_MIN_PAGES;   // smallest share of a work-group: two pages per wavefront pair
#ifndef PQ_BALANCED_UNIT_COST
#define PQ_BALANCED_UNIT_COST 2
#endif
constexpr int kBalancedUnitCost = PQ_BALANCED_UNIT_COST;   // pages' worth of time to start on a (sequence, KV head)
#ifndef PQ_BALANCED_XCD_SKEW
#define PQ_BALANCED_XCD_SKEW 30
#endif
constexpr int kBalancedXcdSkewPermille = PQ_BALANCED_XCD_SKEW;   // even-numbered work-groups (even XCDs) take 3 % more, odd ones 3 % less
constexpr int kBalancedMaxSeqs = 4096;       // every work-group scans all sequence lengths

// Work-groups of a balanced launch: all that are resident at once (3 per compute unit), fewer if
// the shape cannot have kBalancedMinPages pages for each.
int balanced_groups(const pq_layout* l, int32_t n_seqs, int32_t max_seq_len, int per_cu = role_groups_per_cu(4)) {
  const int64_t max_pages = (static_cast<int64_t>(max_seq_len) + kGroup - 1) / kGroup;
  const int64_t bound = static_cast<int64_t>(n_seqs) * l->n_kv_heads * max_pages;   // pages x KV heads, at most
  const int64_t resident = std::min<int64_t>(PQ_BALANCED_GROUPS, static_cast<int64_t>(kComputeUnits) * per_cu);
  return static_cast<int>(std::min<int64_t>(resident, (bound + kBalancedMinPages - 1) / kBalancedMinPages));
}

AttentionKernel choose_attention_kernel(const pq_layout* l, int32_t v_bits, int32_t n_seqs, int32_t n_q_heads,
                                        int32_t max_seq_len) {
  const int64_t max_pages = (static_cast<int64_t>(max_seq_len) + kGroup - 1) / kGroup;
  const int64_t bound = static_cast<int64_t>(n_seqs) * l->n_kv_heads * (max_pages + kBalancedUnitCost);
  // Quantized values make the launch arithmetic-bound, and with 4 query heads per KV head the
  // value wavefront's unpacking and dot products are the longer side of every step of the
  // specialised kernel: wavefronts that all score and aggregate use the four SIMDs evenly
  // (measured at the GQA shape, 4-bit values: 147 against 166 us; with 2 heads per KV head the
  // specialised kernel wins, 127 against 147 us).
  const bool roles_fit = v_bits == 16 || n_q_heads / l->n_kv_heads <= 2;
  if (l->angle_quantizer == PQ_ANGLE_UNIFORM && roles_fit && n_seqs <= kBalancedMaxSeqs &&
      bound < (int64_t{1} << 31) && balanced_groups(l, n_seqs, max_seq_len) >= 256)
    return AttentionKernel::kRoles;
  return AttentionKernel::kPartials;
}

// The caller's workspace holds either the chunk partials of a grid launch ([seq][q head][chunk])
// or, for a balanced launch, one partial per segment slot ([slot][head of the group], slots =
// work-groups + units) and the units' arrival words.  Its size covers both.
struct Workspace {
  float* acc;
  float* ml;
  uint64_t* arrivals;
  size_t bytes;
};

size_t round256(size_t n) { return (n + 255) & ~static_cast<size_t>(255); }

Workspace carve_workspace(void* base, const pq_layout* l, int32_t n_seqs, int32_t n_q_heads, int32_t max_seq_len) {
  const ChunkPlan plan = plan_chunks(n_seqs, l->n_kv_heads, max_seq_len);
  const size_t units = static_cast<size_t>(n_seqs) * l->n_kv_heads;
  const size_t grid_slots = static_cast<size_t>(n_seqs) * n_q_heads * plan.n_chunks;
  const size_t balanced_slots = (static_cast<size_t>(balanced_groups(l, n_seqs, max_seq_len)) + units) * (n_q_heads / l->n_kv_heads);
  const size_t slots = std::max(grid_slots, balanced_slots);
  const size_t acc_bytes = round256(slots * kHeadDim * sizeof(float));
  const size_t ml_bytes = round256(slots * 2 * sizeof(float));
  Workspace w;
  w.acc = static_cast<float*>(base);
  w.ml = reinterpret_cast<float*>(static_cast<uint8_t*>(base) + acc_bytes);
  w.arrivals = reinterpret_cast<uint64_t*>(static_cast<uint8_t*>(base) + acc_bytes + ml_bytes);
  const size_t words = units + static_cast<size_t>(balanced_groups(l, n_seqs, max_seq_len)) + units;   // per unit, per segment slot
  w.bytes = acc_bytes + ml_bytes + round256(words * sizeof(uint64_t));
  return w;
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
  return carve_workspace(nullptr, layout, n_seqs, n_q_heads, max_seq_len).bytes;
}

namespace pq {
namespace {

// Chunks of the score-only kernels: equal chunks of whole rounds of the 4 wavefronts, enough of
// them for `groups_per_cu` resident work-groups on each compute unit (4 with the token-lane
// kernel, 2 with the grouped quantizer's), at least 4 pages each.
ChunkPlan plan_score_chunks(int32_t n_seqs, int32_t n_kv_heads, int32_t max_seq_len, int groups_per_cu) {
  const int64_t max_pages = (static_cast<int64_t>(max_seq_len) + kGroup - 1) / kGroup;
  const int64_t units = static_cast<int64_t>(n_seqs) * n_kv_heads;
  const int64_t want = int64_t{256} * groups_per_cu;
  const int64_t per_unit = std::max<int64_t>(1, (want + units - 1) / units);            // chunks per (sequence, KV head)
  int64_t ppc = std::max<int64_t>(4, (max_pages + per_unit - 1) / per_unit);
  ppc = (ppc + 3) & ~int64_t{3};
  ChunkPlan p;
  p.pages_per_chunk = static_cast<int32_t>(std::min<int64_t>(ppc, 256));                 // a wavefront keeps 64 page ids
  p.n_chunks = static_cast<int32_t>((max_pages + p.pages_per_chunk - 1) / p.pages_per_chunk);
  return p;
}

// Whether pq_decode_attention shares this launch out evenly and merges inside the attention kernel
// (true), or launches one work-group per chunk and the merge kernel after it.
bool merges_in_kernel(const pq_layout* l, int32_t v_bits, int32_t n_seqs, int32_t n_q_heads, int32_t max_seq_len) {
  if (choose_attention_kernel(l, v_bits, n_seqs, n_q_heads, max_seq_len) != AttentionKernel::kRoles) return false;
  return static_cast<int64_t>(n_seqs) * l->n_kv_heads * kArriveFan >= balanced_groups(l, n_seqs, max_seq_len);
}

// Everything the decode entry points have in common: argument checks, kernel arguments, and the
// launches.  `out` null = only the first stage of the two-stage (grid) path, the chunk partials.
int decode_launch(const pq_layout* layout, const void* q, pq_dtype q_dtype, int32_t n_seqs, int32_t n_q_heads,
                  const void* codes_pool, const void* params_pool, const void* v_pool, int32_t v_bits,
                  const void* v_params_pool, int64_t n_pool_pages, const int32_t* block_table,
                  int32_t max_pages_per_seq, const int32_t* seq_lens, int32_t max_seq_len, float sm_scale,
                  float* out, float* scores, int64_t scores_stride, const void* residual_keys,
                  void* workspace, size_t workspace_bytes, void* hip_stream) {
  const int st = check_decode_shape(layout, n_seqs, n_q_heads, max_seq_len);
  if (st != PQ_OK) return st;
  if (!q || !codes_pool || !params_pool || !v_pool || !block_table || !seq_lens) return PQ_ERR_INVALID_ARG;
  if (q_dtype != PQ_F16 && q_dtype != PQ_F32) return PQ_ERR_INVALID_ARG;
  if (n_pool_pages <= 0 || max_pages_per_seq <= 0) return PQ_ERR_INVALID_ARG;
  const int64_t need_pages = (static_cast<int64_t>(max_seq_len) + kGroup - 1) / kGroup;
  if (need_pages > max_pages_per_seq) return PQ_ERR_INVALID_ARG;
  if (scores && scores_stride < max_seq_len) return PQ_ERR_INVALID_ARG;
  if (!isfinite(sm_scale)) return PQ_ERR_INVALID_ARG;
  if (v_bits != 16 && v_bits != 4 && v_bits != 2) return PQ_ERR_UNSUPPORTED;
  if (v_bits != 16 && !v_params_pool) return PQ_ERR_INVALID_ARG;
  // every pool is read with 128-bit loads
  if ((reinterpret_cast<uintptr_t>(codes_pool) | reinterpret_cast<uintptr_t>(params_pool) |
       reinterpret_cast<uintptr_t>(v_pool) | reinterpret_cast<uintptr_t>(residual_keys)) & 15u)
    return PQ_ERR_INVALID_ARG;
  if ((reinterpret_cast<uintptr_t>(v_params_pool) | reinterpret_cast<uintptr_t>(block_table) |
       reinterpret_cast<uintptr_t>(seq_lens)) & 3u)
    return PQ_ERR_INVALID_ARG;
  const int rt = layout->r_bits * 10 + layout->t_bits;
  const bool grouped = layout->angle_quantizer == PQ_ANGLE_GROUPED;

  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u)) return PQ_ERR_WORKSPACE;
  const Workspace ws = carve_workspace(workspace, layout, n_seqs, n_q_heads, max_seq_len);
  if (workspace_bytes < ws.bytes) return PQ_ERR_WORKSPACE;
  const ChunkPlan plan = plan_chunks(n_seqs, layout->n_kv_heads, max_seq_len);

  DecodeArgs a = {};
  a.q = q;
  a.codes = static_cast<const uint8_t*>(codes_pool);
  a.params = static_cast<const uint32_t*>(params_pool);
  a.values = static_cast<const __half*>(v_pool);
  a.residual = static_cast<const __half*>(residual_keys);
  a.v_params = static_cast<const uint32_t*>(v_params_pool);
  a.block_table = block_table;
  a.seq_lens = seq_lens;
  a.n_seqs = n_seqs;
  a.scores = scores;
  a.ws_acc = ws.acc;
  a.ws_ml = ws.ml;
  a.out = out;
  a.arrivals = ws.arrivals;
  a.min_pages = kBalancedMinPages;
  a.unit_cost = kBalancedUnitCost;
  a.xcd_skew_permille = kBalancedXcdSkewPermille;
  a.scores_stride = scores_stride;
  a.n_pool_pages = n_pool_pages;
  a.n_kv_heads = layout->n_kv_heads;
  a.n_q_heads = n_q_heads;
  a.max_pages_per_seq = max_pages_per_seq;
  a.max_seq_len = max_seq_len;
  a.pages_per_chunk = plan.pages_per_chunk;
  a.n_chunks = plan.n_chunks;
  a.q_is_f32 = q_dtype == PQ_F32 ? 1 : 0;
  a.scale_log2 = static_cast<float>(static_cast<double>(sm_scale) * 1.4426950408889634074);
  fill_angle_tables(a, layout->t_bits);

  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const int group_total = n_q_heads / layout->n_kv_heads;
  a.group_total = group_total;
  // The role-specialised kernel shares a launch out evenly and merges in the kernel, except when
  // the units are few and each would be shared by more work-groups than one arrival word takes
  // well (one long sequence), or when only the partials are asked for: then one work-group per
  // chunk, and the merge kernel.
  const bool roles = choose_attention_kernel(layout, v_bits, n_seqs, n_q_heads, max_seq_len) == AttentionKernel::kRoles;
  const int n_balanced = balanced_groups(layout, n_seqs, max_seq_len);
  const bool balanced = out != nullptr && merges_in_kernel(layout, v_bits, n_seqs, n_q_heads, max_seq_len);
  a.grid_mode = balanced ? 0 : 1;
  const dim3 grid(layout->n_kv_heads, n_seqs, plan.n_chunks);
  hipError_t e = hipSuccess;
  // A kernel instance serves 8, 4, 2 or 1 query heads of a KV head; other groups take several
  // passes over the cache (6 = 4 + 2, 12 = 8 + 4, ...).
  for (int head0 = 0; head0 < group_total && e == hipSuccess;) {
    const int left = group_total - head0;
    // 8 heads at a time where there is a kernel for it: the role-specialised one, fp16 values
    const int G = (left >= 8 && roles && v_bits == 16) ? 8 : (left >= 4 ? 4 : (left >= 2 ? 2 : 1));
    a.head0 = head0;
    bool found;
    if (roles) {
      found = a.grid_mode ? launch_attention_roles_grid(rt, G, v_bits, a, static_cast<int>(grid.x * grid.y * grid.z), stream)
                          : launch_attention_roles(rt, G, v_bits, a, std::min(n_balanced, balanced_groups(layout, n_seqs, max_seq_len, role_groups_per_cu(G))), stream);
    } else {
      found = grouped ? launch_attention_partials_ga(rt, G, v_bits, a, grid, stream)
                      : launch_attention_partials(rt, G, v_bits, a, grid, stream);
    }
    if (!found) return PQ_ERR_UNSUPPORTED;   // not reached: layout_supported() admits what is built
    e = hipGetLastError();
    head0 += G;
  }
  if (e != hipSuccess) return record_hip_error(e);
  if (out != nullptr && a.grid_mode) {
    hipLaunchKernelGGL(pq_decode_merge_kernel, dim3(n_q_heads, n_seqs), dim3(kMergeThreads), 0, stream, ws.acc,
                       ws.ml, seq_lens, out, n_q_heads, max_seq_len, plan.pages_per_chunk, plan.n_chunks);
    e = hipGetLastError();
    if (e != hipSuccess) return record_hip_error(e);
  }
  return PQ_OK;
}

}  // namespace
}  // namespace pq

extern "C" int pq_decode_partials(const pq_layout* layout, const void* q, pq_dtype q_dtype, int32_t n_seqs,
                                  int32_t n_q_heads, const void* codes_pool, const void* params_pool,
                                  const void* v_pool, int32_t v_bits, const void* v_params_pool,
                                  int64_t n_pool_pages, const int32_t* block_table,
                                  int32_t max_pages_per_seq, const int32_t* seq_lens, int32_t max_seq_len,
                                  float sm_scale, float* scores, int64_t scores_stride,
                                  const void* residual_keys, void* workspace,
                                  size_t workspace_bytes, void* hip_stream) {
  return decode_launch(layout, q, q_dtype, n_seqs, n_q_heads, codes_pool, params_pool, v_pool, v_bits, v_params_pool,
                       n_pool_pages, block_table, max_pages_per_seq, seq_lens, max_seq_len, sm_scale, nullptr, scores,
                       scores_stride, residual_keys, workspace, workspace_bytes, hip_stream);
}

extern "C" const char* pq_decode_kernel_name(const pq_layout* layout, int32_t n_seqs, int32_t n_q_heads,
                                             int32_t max_seq_len, int32_t v_bits) {
  if (check_decode_shape(layout, n_seqs, n_q_heads, max_seq_len) != PQ_OK) return "";
  return choose_attention_kernel(layout, v_bits, n_seqs, n_q_heads, max_seq_len) == AttentionKernel::kRoles
             ? "pq_decode_roles_kernel" : "pq_decode_partials_kernel";
}

extern "C" int pq_decode_merges_in_kernel(const pq_layout* layout, int32_t n_seqs, int32_t n_q_heads,
                                          int32_t max_seq_len, int32_t v_bits) {
  const int st = check_decode_shape(layout, n_seqs, n_q_heads, max_seq_len);
  if (st != PQ_OK) return st;
  return merges_in_kernel(layout, v_bits, n_seqs, n_q_heads, max_seq_len) ? 1 : 0;
}

extern "C" int pq_decode_merge(const pq_layout* layout, int32_t n_seqs, int32_t n_q_heads,
                               const int32_t* seq_lens, int32_t max_seq_len, float* out,
                               const void* workspace, size_t workspace_bytes, void* hip_stream) {
  const int st = check_decode_shape(layout, n_seqs, n_q_heads, max_seq_len);
  if (st != PQ_OK) return st;
  if (!seq_lens || !out) return PQ_ERR_INVALID_ARG;
  const ChunkPlan plan = plan_chunks(n_seqs, layout->n_kv_heads, max_seq_len);
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u)) return PQ_ERR_WORKSPACE;
  const Workspace ws = carve_workspace(const_cast<void*>(workspace), layout, n_seqs, n_q_heads, max_seq_len);
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
                                   const void* residual_keys, void* workspace,
                                   size_t workspace_bytes, void* hip_stream) {
  if (!out || (reinterpret_cast<uintptr_t>(out) & 15u)) return PQ_ERR_INVALID_ARG;
  return decode_launch(layout, q, q_dtype, n_seqs, n_q_heads, codes_pool, params_pool, v_pool, v_bits, v_params_pool,
                       n_pool_pages, block_table, max_pages_per_seq, seq_lens, max_seq_len, sm_scale, out, scores,
                       scores_stride, residual_keys, workspace, workspace_bytes, hip_stream);
}

extern "C" int pq_decode_attention_static(const pq_layout* layout, const void* q, pq_dtype q_dtype, int32_t n_seqs,
                                          int32_t n_q_heads, const void* codes_pool, const void* params_pool,
                                          const void* v_pool, int32_t v_bits, const void* v_params_pool,
                                          int64_t n_pool_pages, const int32_t* block_table,
                                          int32_t max_pages_per_seq, const int32_t* seq_lens, int32_t max_seq_len,
                                          float sm_scale, float* out, float* scores, int64_t scores_stride,
                                          const void* residual_keys, void* hip_stream) {
  const int st = check_decode_shape(layout, n_seqs, n_q_heads, max_seq_len);
  if (st != PQ_OK) return st;
  const size_t need = pq_decode_workspace_bytes(layout, n_seqs, n_q_heads, max_seq_len);
  if (need == 0 || need > static_cast<size_t>(PQ_STATIC_SCRATCH_BYTES)) return PQ_ERR_STATIC_LIMIT;
  void* ws = nullptr;
  const int sp = static_scratch(&ws);
  if (sp != PQ_OK) return sp;
  return pq_decode_attention(layout, q, q_dtype, n_seqs, n_q_heads, codes_pool, params_pool, v_pool, v_bits,
                             v_params_pool, n_pool_pages, block_table, max_pages_per_seq, seq_lens, max_seq_len,
                             sm_scale, out, scores, scores_stride, residual_keys, ws, need, hip_stream);
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
  // the pools are read with 128-bit loads
  if ((reinterpret_cast<uintptr_t>(codes_pool) | reinterpret_cast<uintptr_t>(params_pool) |
       reinterpret_cast<uintptr_t>(residual_keys)) & 15u)
    return PQ_ERR_INVALID_ARG;
  if ((reinterpret_cast<uintptr_t>(block_table) | reinterpret_cast<uintptr_t>(seq_lens) | reinterpret_cast<uintptr_t>(scores)) & 3u)
    return PQ_ERR_INVALID_ARG;
  if (scores_stride >= (int64_t{1} << 28)) return PQ_ERR_UNSUPPORTED;   // 4 score rows are addressed with 32-bit byte offsets
  const bool grouped = layout->angle_quantizer == PQ_ANGLE_GROUPED;
#ifndef PQ_SCORE_GROUPS_PER_CU
#define PQ_SCORE_GROUPS_PER_CU 4
#endif
  const ChunkPlan plan = plan_score_chunks(n_seqs, layout->n_kv_heads, max_seq_len, grouped ? 2 : PQ_SCORE_GROUPS_PER_CU);
  if (plan.n_chunks > 65535) return PQ_ERR_UNSUPPORTED;   // grid.z
  DecodeArgs a = {};
  a.q = q;
  a.q_is_f32 = q_dtype == PQ_F32 ? 1 : 0;
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
    if (!launch_scores(layout->r_bits * 10 + layout->t_bits, grouped, G, a, grid, stream))
      return PQ_ERR_UNSUPPORTED;           // not reached: layout_supported() admits what is built
    e = hipGetLastError();
    head0 += G;
  }
  if (e != hipSuccess) return record_hip_error(e);
  return PQ_OK;
}
