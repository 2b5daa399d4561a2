// Decode attention over the polar-quantized key cache (gfx950).
//
// What is computed (paper Section 3.3 and Appendix A): for every query head a
// table T[j][a] = q_x[j] cos(theta~_a) + q_y[j] sin(theta~_a) over the 2^t angle
// states is built once; the score of a cached token is
//     sum_j rho~_j * T[j][a_j],   rho~_j = (c_j + 1/2) s_j + z_j   (Section 3.2),
// i.e. the dequantize-then-dot product with the multiplications by the query
// pulled out of the token loop.  Softmax and the fp16 value aggregation that
// consume the scores are fused behind it (standard attention, Section 2).
//
// Mapping to the machine.  One work-group = 4 wavefronts = one (sequence, KV
// head, chunk of pages); the table of all query heads that share the KV head
// lives in LDS with the heads interleaved (one 16-byte entry serves 4 heads).
// Each wavefront owns whole pages (= quantization groups), so a page's radius
// parameters are loaded once into registers and no work-group barrier is
// needed inside the loop:
//   score  : lane = (pair block q = lane / 16, token tk = lane % 16).  One
//            128-bit (96-bit for w = 6) load brings the 16 symbols of pairs
//            16q .. 16q+15; the 16 lanes of a row read 16 consecutive units.
//            The four rows' partial sums are folded with v_permlane32_swap /
//            v_permlane16_swap so that row h ends up holding head h's score.
//   softmax: online, per page, in the log2 domain (running max m, sum l).
//   values : lane = (token slot lane / 16, dims 8*(lane % 16) ..+7); 128-bit
//            loads of fp16 rows, probabilities broadcast from LDS.
// A last step folds the four wavefronts' (m, l, acc) into one partial per
// (sequence, query head, chunk); pq_decode_merge_kernel combines the chunks.
// No MFMA: the hot loop is a gather-accumulate.
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>
#include <math.h>

#include <type_traits>

#include "pq_internal.hpp"

namespace pq {

namespace {

constexpr int kWaves = 4;
constexpr int kThreads = kWaves * 64;
constexpr float kNegInf = -INFINITY;

struct DecodeArgs {
  const void* q;
  const uint8_t* codes;
  const uint32_t* params;   // {fp16 s, fp16 z} per pair, viewed as one dword
  const __half* values;
  const __half* residual;   // [seq][kv_head][g][d] un-quantized keys of the last, incomplete group (or null)
  const int32_t* block_table;
  const int32_t* seq_lens;
  float* scores;
  float* ws_acc;            // [seq][q_head][chunk][128]
  float* ws_ml;             // [seq][q_head][chunk][2] = (m in log2 units, l)
  int64_t scores_stride;
  int64_t n_pool_pages;
  int32_t n_kv_heads;
  int32_t n_q_heads;
  int32_t max_pages_per_seq;
  int32_t max_seq_len;
  int32_t pages_per_chunk;
  int32_t n_chunks;
  float scale_log2;         // sm_scale * log2(e)
  float cos_tab[kMaxAngleBins];
  float sin_tab[kMaxAngleBins];
};

__device__ __forceinline__ uint32_t f2u(float x) { return __float_as_uint(x); }
__device__ __forceinline__ float u2f(uint32_t x) { return __uint_as_float(x); }

// lanes < 32 get a[l] + a[l+32]; lanes >= 32 get b[l-32] + b[l]
__device__ __forceinline__ float tsum32(float a, float b) {
  auto r = __builtin_amdgcn_permlane32_swap(f2u(a), f2u(b), false, false);
  return u2f(r[0]) + u2f(r[1]);
}
// even 16-lane rows get a[row] + a[row+1]; odd rows get b[row-1] + b[row]
__device__ __forceinline__ float tsum16(float a, float b) {
  auto r = __builtin_amdgcn_permlane16_swap(f2u(a), f2u(b), false, false);
  return u2f(r[0]) + u2f(r[1]);
}
__device__ __forceinline__ float sum_rows(float x) {   // sum over the 4 rows, result in all rows
  x = tsum32(x, x);
  return tsum16(x, x);
}
__device__ __forceinline__ float row_max(float x) {    // over the 16 lanes of a row
  x = fmaxf(x, __shfl_xor(x, 8));
  x = fmaxf(x, __shfl_xor(x, 4));
  x = fmaxf(x, __shfl_xor(x, 2));
  return fmaxf(x, __shfl_xor(x, 1));
}
__device__ __forceinline__ float row_sum(float x) {
  x += __shfl_xor(x, 8);
  x += __shfl_xor(x, 4);
  x += __shfl_xor(x, 2);
  return x + __shfl_xor(x, 1);
}
// Sum of the four 16-lane rows' partial scores: with 4 query heads row h ends with head h's
// score (transposing fold), with 2 heads rows 0-1 / 2-3, with 1 head every row.
template <int G>
__device__ __forceinline__ float fold_rows(const float (&part)[G]) {
  if constexpr (G == 4) {
    return tsum16(tsum32(part[0], part[2]), tsum32(part[1], part[3]));
  } else if constexpr (G == 2) {
    const float b = tsum32(part[0], part[1]);
    return tsum16(b, b);
  } else {
    return sum_rows(part[0]);
  }
}

// LDS written by some lanes of this wavefront is about to be read by others.
__device__ __forceinline__ void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Tuning constants of the attention kernel (measured on MI355X): 4 quads of 4 value rows in
// flight per wavefront (8 or 32 rows change nothing), and a register budget of 2 wavefronts
// per SIMD -- 3 or 4 only fit with spills and run 1.5-2x slower.
#ifndef PQ_RING_SETS
#define PQ_RING_SETS 4
#endif
#ifndef PQ_WAVES_PER_EU
#define PQ_WAVES_PER_EU 2
#endif
#define PQ_KERNEL_ATTR \
  __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(PQ_WAVES_PER_EU, PQ_WAVES_PER_EU)))

// ---- streaming loads --------------------------------------------------------
// Codes, parameters and values are read through buffer descriptors that cover
// exactly one page of one KV head: the lane offset stays in one VGPR, the
// position inside the page is a scalar/immediate offset, and a read past the
// descriptor's size returns zeros instead of faulting (value rows beyond the
// sequence end are masked that way).  Everything streamed is read once, so the
// loads are non-temporal.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x3 __attribute__((ext_vector_type(3)));
constexpr int kAuxStream = 2;     // gfx950 cache-policy bit "nt"
constexpr int kAuxCached = 0;

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, uint32_t bytes) {
  // raw buffer, 32-bit data format, no swizzle
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, static_cast<int>(bytes), 0x00020000);
}
template <int AUX>
__device__ __forceinline__ uint4 buf_load16(__amdgpu_buffer_rsrc_t r, uint32_t voff, uint32_t soff) {
  const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(r, voff, soff, AUX);
  return make_uint4(v.x, v.y, v.z, v.w);
}

template <int NW>
struct Unit {
  uint32_t d[NW];
};

template <int W>
__device__ __forceinline__ Unit<W / 2> load_unit(__amdgpu_buffer_rsrc_t r, uint32_t voff, uint32_t soff) {
  Unit<W / 2> u;
  if constexpr (W == 8) {
    const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(r, voff, soff, kAuxStream);
    u.d[0] = v.x; u.d[1] = v.y; u.d[2] = v.z; u.d[3] = v.w;
  } else {
    static_assert(W == 6, "unit width");
    const u32x3 v = __builtin_amdgcn_raw_buffer_load_b96(r, voff, soff, kAuxStream);
    u.d[0] = v.x; u.d[1] = v.y; u.d[2] = v.z;
  }
  return u;
}

template <int W, int K>
__device__ __forceinline__ uint32_t symbol(const Unit<W / 2>& u) {
  constexpr int bit = K * W, wi = bit >> 5, sh = bit & 31;
  uint32_t v = u.d[wi] >> sh;
  if constexpr (sh + W > 32) v |= u.d[wi + 1] << (32 - sh);
  return v & ((1u << W) - 1u);
}

template <int G>
struct Heads {
  float v[G];
};

// LDS is addressed by 32-bit byte addresses (address space 3) so that the table
// gather is a ds_read with an immediate offset.
#define PQ_LDS __attribute__((address_space(3)))
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t lds_addr(const void* p) {
  return static_cast<uint32_t>(reinterpret_cast<uintptr_t>((const PQ_LDS uint8_t*)p));
}

template <int G>
__device__ __forceinline__ Heads<G> lut_read(uint32_t addr) {
  Heads<G> t;
  if constexpr (G == 4) {
    const f32x4 f = *(const PQ_LDS f32x4*)static_cast<uintptr_t>(addr);
    t.v[0] = f.x; t.v[1] = f.y; t.v[2] = f.z; t.v[3] = f.w;
  } else if constexpr (G == 2) {
    const f32x2 f = *(const PQ_LDS f32x2*)static_cast<uintptr_t>(addr);
    t.v[0] = f.x; t.v[1] = f.y;
  } else {
    t.v[0] = *(const PQ_LDS float*)static_cast<uintptr_t>(addr);
  }
  return t;
}

// Byte B of `x` as a float / added to `base`: one instruction each on gfx9
// (v_cvt_f32_ubyteB, and v_add_u32 with a sub-dword operand select).
template <int B>
__device__ __forceinline__ float byte_to_float(uint32_t x) {
  float f;
  if constexpr (B == 0) asm("v_cvt_f32_ubyte0 %0, %1" : "=v"(f) : "v"(x));
  else if constexpr (B == 1) asm("v_cvt_f32_ubyte1 %0, %1" : "=v"(f) : "v"(x));
  else if constexpr (B == 2) asm("v_cvt_f32_ubyte2 %0, %1" : "=v"(f) : "v"(x));
  else asm("v_cvt_f32_ubyte3 %0, %1" : "=v"(f) : "v"(x));
  return f;
}
template <int B>
__device__ __forceinline__ uint32_t add_byte(uint32_t x, uint32_t base) {
  uint32_t r;
  if constexpr (B == 0)
    asm("v_add_u32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:BYTE_0 src1_sel:DWORD" : "=v"(r) : "v"(x), "v"(base));
  else if constexpr (B == 1)
    asm("v_add_u32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:BYTE_1 src1_sel:DWORD" : "=v"(r) : "v"(x), "v"(base));
  else if constexpr (B == 2)
    asm("v_add_u32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:BYTE_2 src1_sel:DWORD" : "=v"(r) : "v"(x), "v"(base));
  else
    asm("v_add_u32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:BYTE_3 src1_sel:DWORD" : "=v"(r) : "v"(x), "v"(base));
  return r;
}

// One pair step: part[h] += rho~ * T[h][pair K of this lane's block][angle code].
// `lut_row0` is the LDS byte address of the lane's block (pair 16*row); radius
// parameters are (s, z + s/2) so that rho~ = c * s + zz.
template <int G, int RB, int TB, int K>
__device__ __forceinline__ void score_steps(const Unit<(RB + TB) / 2>& u, uint32_t lut_row0,
                                            const float (&sf)[16], const float (&zz)[16],
                                            float (&part)[G]) {
  if constexpr (K < 16) {
    constexpr int W = RB + TB;
    constexpr int ROW = 16 << TB;
    float c;
    uint32_t addr;
    if constexpr (RB == 4 && TB == 4) {
      // byte K of the unit is (a << 4) | c: mask once per dword, then one op per field
      const uint32_t d = u.d[K >> 2];
      const uint32_t rad = d & 0x0f0f0f0fu, ang = d & 0xf0f0f0f0u;   // CSE'd across the dword's 4 pairs
      c = byte_to_float<K & 3>(rad);
      addr = add_byte<K & 3>(ang, lut_row0);                        // (a << 4) is the entry's byte offset
    } else {
      // generic widths: bit-field extract per field (after an alignbit if the symbol straddles
      // two dwords), then v_lshl_add for the table address -- written as instructions because
      // the compiler otherwise re-associates them into a longer shift/mask/add chain
      constexpr int bit = K * W, wi = bit >> 5, sh = bit & 31;
      uint32_t src = u.d[wi];
      int off = sh;
      if constexpr (sh + W > 32) {
        src = __builtin_amdgcn_alignbit(u.d[wi + 1], u.d[wi], sh);
        off = 0;
      }
      uint32_t cq, aq;
      asm("v_bfe_u32 %0, %1, %2, %3" : "=v"(cq) : "v"(src), "n"(off), "n"(RB));
      asm("v_bfe_u32 %0, %1, %2, %3" : "=v"(aq) : "v"(src), "n"(off + RB), "n"(TB));
      asm("v_lshl_add_u32 %0, %1, 4, %2" : "=v"(addr) : "v"(aq), "v"(lut_row0));
      c = byte_to_float<0>(cq);
    }
    const float rho = fmaf(c, sf[K], zz[K]);
    const Heads<G> t = lut_read<G>(addr + K * ROW);
#pragma unroll
    for (int h = 0; h < G; ++h) part[h] = fmaf(rho, t.v[h], part[h]);
    score_steps<G, RB, TB, K + 1>(u, lut_row0, sf, zz, part);
  }
}

// Residual keys (the un-quantized tail of a sequence): part[h] += sum over this lane's 32 dims
// (pairs 16*row .. 16*row+15, i.e. dims 16*row.. and 64+16*row..) of k[dim] * q_h[dim].
// kx / ky are the 16 fp16 x- and y-coordinates of the lane's pairs; `qs_row` is the LDS byte
// address of q[dim = 16*row][heads], 16 bytes per dim.
template <int G>
__device__ __forceinline__ void dense_steps(const uint4 (&kx)[2], const uint4 (&ky)[2], uint32_t qs_row,
                                            float (&part)[G]) {
#pragma unroll
  for (int half = 0; half < 2; ++half) {
    const uint4(&kk)[2] = half == 0 ? kx : ky;
#pragma unroll
    for (int v = 0; v < 2; ++v) {
      const uint32_t w4[4] = {kk[v].x, kk[v].y, kk[v].z, kk[v].w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const __half2 hv = *reinterpret_cast<const __half2*>(&w4[e]);
        const float k0 = __low2float(hv), k1 = __high2float(hv);
        const int dim = half * kPairs + v * 8 + 2 * e;            // relative to 16 * row
        const Heads<G> q0 = lut_read<G>(qs_row + dim * 16);
        const Heads<G> q1 = lut_read<G>(qs_row + (dim + 1) * 16);
#pragma unroll
        for (int h = 0; h < G; ++h) part[h] = fmaf(k1, q1.v[h], fmaf(k0, q0.v[h], part[h]));
      }
    }
  }
}

// acc[h][0..7] += p_h[token] * V[token][this lane's 8 dims] for the 4 value rows in `vv`
// (tokens 4 * (it0 + i) + row); pw is prob[token][G] in LDS.
template <int G>
__device__ __forceinline__ void consume_values(const uint4 (&vv)[4], int it0, uint32_t pw, int row,
                                               float (&acc)[G][8]) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int tok = (it0 + i) * 4 + row;
    const Heads<G> p = lut_read<G>(pw + tok * (G * 4));
    const uint32_t w4[4] = {vv[i].x, vv[i].y, vv[i].z, vv[i].w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const __half2 hv = *reinterpret_cast<const __half2*>(&w4[e]);
      const float v0 = __low2float(hv), v1 = __high2float(hv);
#pragma unroll
      for (int h = 0; h < G; ++h) {
        acc[h][2 * e] = fmaf(p.v[h], v0, acc[h][2 * e]);
        acc[h][2 * e + 1] = fmaf(p.v[h], v1, acc[h][2 * e + 1]);
      }
    }
  }
}

template <int G, int RB, int TB, typename QT, bool SCORES>
__global__ PQ_KERNEL_ATTR void pq_decode_partials_kernel(const DecodeArgs a) {
  constexpr int W = RB + TB;
  constexpr int UB = 2 * W;              // bytes per unit
  constexpr int NA = 1 << TB;            // angle states
  constexpr int ROW = NA * 16;           // table bytes per pair

  __shared__ __attribute__((aligned(16))) uint8_t lut[kPairs * ROW];
  __shared__ __attribute__((aligned(16))) float prob[kWaves][kGroup * G];
  __shared__ __attribute__((aligned(16))) float alpha_s[kWaves][4];
  __shared__ __attribute__((aligned(16))) float red_acc[kWaves][G][kHeadDim];
  __shared__ float red_ml[kWaves][G][2];
  __shared__ __attribute__((aligned(16))) float q_lds[kHeadDim][4];   // q[dim][head] for residual keys
  __shared__ float res_sc[kGroup * G];                                // raw scores of the residual group

  // Chunk-major launch order: the KV heads of one page are neighbours in memory and run
  // together; every sequence's first chunks run first, and the chunks that only long sequences
  // have (with the empty work-groups of the short ones) come last, which balances ragged batches.
  const int kvh = blockIdx.x, seq = blockIdx.y, chunk = blockIdx.z;
  const int L = min(a.seq_lens[seq], a.max_seq_len);
  if (L <= 0) return;
  const int n_pages = (L + kGroup - 1) / kGroup;
  const int page0 = chunk * a.pages_per_chunk;
  if (page0 >= n_pages) return;
  const int npg = min(a.pages_per_chunk, n_pages - page0);

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);


  const int row = lane >> 4;             // score phase: pair block; value phase: token slot
  const int col = lane & 15;             // score phase: token in the pass; value phase: dim slice
  const int my_head = (G == 4) ? row : (G == 2 ? (row >> 1) : 0);
  const bool owner = (G == 4) || (G == 2 && (row & 1) == 0) || (G == 1 && row == 0);

  float m_run = kNegInf, l_run = 0.f;
  float acc[G][8];
#pragma unroll
  for (int h = 0; h < G; ++h)
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[h][e] = 0.f;

  const uint32_t lut_row0 = lds_addr(lut) + row * (kPairsPerUnit * ROW);
  const uint32_t pw_addr = lds_addr(prob[wave]);
  const uint32_t voff_codes = (row * kGroup + col) * UB;          // unit of (block row, token col) of pass 0
  const uint32_t voff_params = row * (kPairsPerUnit * 4);
  const uint32_t voff_values = row * (kHeadDim * 2) + col * 16;   // token slot row, dims 8*col..

  // This wavefront's pages are chunk pages wave, wave + 4, ...; lane k remembers the pool page
  // of the k-th of them (-1 if the block table entry is out of range: such a page is masked).
  const int n_w = npg > wave ? (npg - wave + kWaves - 1) / kWaves : 0;
  int pid_lane = -1;
  if (lane < n_w) {
    const int64_t pid = a.block_table[static_cast<int64_t>(seq) * a.max_pages_per_seq + page0 + wave + kWaves * lane];
    if (pid >= 0 && pid < a.n_pool_pages) pid_lane = static_cast<int>(pid);
  }
  constexpr uint32_t kCodesBytes = kBlocks * kGroup * UB;          // codes of one (page, kv head)
  // With a residual buffer the last, incomplete group of the sequence is kept as fp16 keys.
  const int res_page = (a.residual != nullptr && (L % kGroup) != 0) ? L / kGroup : -1;
  // Buffer descriptors of the wavefront's k-th page; a masked page gets empty descriptors
  // (every read returns zero) and zero valid tokens.
  auto page_setup = [&](int k, __amdgpu_buffer_rsrc_t& rc, __amdgpu_buffer_rsrc_t& rp,
                        __amdgpu_buffer_rsrc_t& rv, int& nv) {
    const int pid = __builtin_amdgcn_readlane(pid_lane, k);
    const bool ok = pid >= 0;
    const int64_t ph = ok ? static_cast<int64_t>(pid) * a.n_kv_heads + kvh : 0;
    nv = ok ? min(kGroup, L - (page0 + wave + kWaves * k) * kGroup) : 0;
    const bool packed = ok && (page0 + wave + kWaves * k) != res_page;   // the residual group has no codes yet
    rc = make_rsrc(a.codes + ph * kCodesBytes, packed ? kCodesBytes : 0u);
    rp = make_rsrc(a.params + ph * kPairs, packed ? kPairs * 4u : 0u);
    rv = make_rsrc(a.values + ph * (kGroup * kHeadDim), static_cast<uint32_t>(nv) * (kHeadDim * 2));
  };

  // ---- loop over the wavefront's pages ---------------------------------------------------
  // Per page: score its 128 tokens (8 passes), online softmax, then aggregate its 32 x 4 value
  // rows.  Loads run ahead of their use:
  //   * value rows ride in a ring of 4 x 4 register quads; a quad is refilled, as soon as it has
  //     been consumed, with the row 16 further on -- the last 16 refills of a page fetch the
  //     first 16 rows of the NEXT page, which then arrive during that page's score phase;
  //   * codes and parameters of the next page are loaded at the start of the value phase, into
  //     registers the score phase has just released.
  // When there is no next page those loads go to an empty descriptor: they return zeros
  // without touching memory, so the loop body has no branches.
  const __amdgpu_buffer_rsrc_t rs_empty = make_rsrc(a.values, 0u);
  __amdgpu_buffer_rsrc_t rc_cur = rs_empty, rp_cur = rs_empty, rv_cur = rs_empty;
  __amdgpu_buffer_rsrc_t rc_nxt = rs_empty, rp_nxt = rs_empty, rv_nxt = rs_empty;
  int nv_cur = 0, nv_nxt = 0;
  uint4 praw[4];
  Unit<W / 2> cu[8];
  constexpr int kRingSets = PQ_RING_SETS;                          // register quads of 4 value rows in flight
  uint4 ring[kRingSets][4];
  if (n_w > 0) {
    page_setup(0, rc_cur, rp_cur, rv_cur, nv_cur);
#pragma unroll
    for (int i = 0; i < 4; ++i) praw[i] = buf_load16<kAuxCached>(rp_cur, voff_params, i * 16);
#pragma unroll
    for (int i = 0; i < 8; ++i) cu[i] = load_unit<W>(rc_cur, voff_codes, i * 16 * UB);
#pragma unroll
    for (int k = 0; k < kRingSets; ++k)
#pragma unroll
      for (int r = 0; r < 4; ++r) ring[k][r] = buf_load16<kAuxStream>(rv_cur, voff_values, (4 * k + r) * 1024);
  }

  // ---- table of the G query heads that share this KV head (Section 3.3) ----
  // (built while the first page's loads, issued above, are in flight)
  {
    const QT* qb = static_cast<const QT*>(a.q) + (static_cast<int64_t>(seq) * a.n_q_heads + kvh * G) * kHeadDim;
    float* lf = reinterpret_cast<float*>(lut);
    for (int idx = tid; idx < kPairs * NA; idx += kThreads) {
      const int j = idx >> TB, s = idx & (NA - 1);
      const float cs = a.cos_tab[s], sn = a.sin_tab[s];
#pragma unroll
      for (int h = 0; h < G; ++h) {
        const float qx = static_cast<float>(qb[h * kHeadDim + j]);
        const float qy = static_cast<float>(qb[h * kHeadDim + j + kPairs]);
        lf[idx * 4 + h] = fmaf(qx, cs, qy * sn);
      }
    }
    if (tid < kHeadDim) {
#pragma unroll
      for (int h = 0; h < G; ++h) q_lds[tid][h] = static_cast<float>(qb[h * kHeadDim + tid]);
    }
  }
  __syncthreads();

  // ---- residual group (at most one per sequence): scored here, before the page loop, by the
  // wavefront that owns its page -- plain dot products with the fp16 keys in the same lane
  // layout (each lane takes the 32 dims of its 16 pairs) and with the same fold; key rows past
  // the sequence end read as zero.  The loop below picks the scores up from LDS.
  if (res_page >= page0 + wave && res_page < page0 + npg && ((res_page - page0 - wave) & (kWaves - 1)) == 0) {
    const int nv_res = L - res_page * kGroup;
    const __amdgpu_buffer_rsrc_t rs_res = make_rsrc(
        a.residual + (static_cast<int64_t>(seq) * a.n_kv_heads + kvh) * (kGroup * kHeadDim),
        static_cast<uint32_t>(nv_res) * (kHeadDim * 2));
    const uint32_t voff_res = col * (kHeadDim * 2) + row * 32;
    const uint32_t qs_row = lds_addr(q_lds) + row * (16 * 16);
#pragma unroll 1
    for (int s = 0; s < 8; ++s) {
      uint4 kx[2], ky[2];
      const uint32_t soff = s * 16 * kHeadDim * 2;
      kx[0] = buf_load16<kAuxCached>(rs_res, voff_res, soff);
      kx[1] = buf_load16<kAuxCached>(rs_res, voff_res + 16, soff);
      ky[0] = buf_load16<kAuxCached>(rs_res, voff_res + kPairs * 2, soff);
      ky[1] = buf_load16<kAuxCached>(rs_res, voff_res + kPairs * 2 + 16, soff);
      float part[G];
#pragma unroll
      for (int h = 0; h < G; ++h) part[h] = 0.f;
      dense_steps<G>(kx, ky, qs_row, part);
      const float v = fold_rows<G>(part);
      if (owner) res_sc[(s * 16 + col) * G + my_head] = v;
    }
    wave_lds_sync();
  }

  for (int i = 0; i < n_w; ++i) {
    const int pi = page0 + wave + kWaves * i;                      // chunk-relative page of iteration i
    if (i + 1 < n_w) {
      page_setup(i + 1, rc_nxt, rp_nxt, rv_nxt, nv_nxt);
    } else {
      rc_nxt = rp_nxt = rv_nxt = rs_empty;
      nv_nxt = 0;
    }

    // radius parameters of this lane's 16 pairs: rho~ = c * s + (z + s/2)
    float sf[16], zz[16];
#pragma unroll
    for (int v4 = 0; v4 < 4; ++v4) {
      const uint32_t w4[4] = {praw[v4].x, praw[v4].y, praw[v4].z, praw[v4].w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const __half2 sz = *reinterpret_cast<const __half2*>(&w4[e]);
        const float s = __low2float(sz), z = __high2float(sz);
        sf[v4 * 4 + e] = s;
        zz[v4 * 4 + e] = fmaf(0.5f, s, z);
      }
    }

    // ---- scores of the page's 128 tokens: 8 passes of 16 tokens ----
    float sc[8];
    if (pi != res_page) {
#pragma unroll
      for (int s = 0; s < 8; ++s) {
        float part[G];
#pragma unroll
        for (int h = 0; h < G; ++h) part[h] = 0.f;
        score_steps<G, RB, TB, 0>(cu[s], lut_row0, sf, zz, part);
        sc[s] = fold_rows<G>(part);
      }
    } else {
      // residual group: its scores were computed before the loop (plain dot products)
#pragma unroll
      for (int s = 0; s < 8; ++s)
        sc[s] = *(const PQ_LDS float*)static_cast<uintptr_t>(lds_addr(res_sc) + ((s * 16 + col) * G + my_head) * 4);
    }

    // ---- online softmax over the page (log2 domain) ----
    float pm = kNegInf;
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      const int tok = t * 16 + col;
      if constexpr (SCORES) {
        if (owner && tok < nv_cur)
          a.scores[(static_cast<int64_t>(seq) * a.n_q_heads + kvh * G + my_head) * a.scores_stride +
                   static_cast<int64_t>(pi) * kGroup + tok] = sc[t];
      }
      sc[t] = (tok < nv_cur) ? sc[t] * a.scale_log2 : kNegInf;
      pm = fmaxf(pm, sc[t]);
    }
    pm = row_max(pm);
    const float m_new = fmaxf(m_run, pm);
    const bool dead = !(m_new > kNegInf);                          // nothing valid seen so far
    const float alpha = dead ? 1.f : __builtin_amdgcn_exp2f(m_run - m_new);   // 0 on the first page
    float psum = 0.f;
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      const float p = dead ? 0.f : __builtin_amdgcn_exp2f(sc[t] - m_new);
      psum += p;
      if (owner) *(PQ_LDS float*)static_cast<uintptr_t>(pw_addr + ((t * 16 + col) * G + my_head) * 4) = p;
    }
    l_run = fmaf(l_run, alpha, psum);
    m_run = m_new;
    if (owner && col == 0) alpha_s[wave][my_head] = alpha;
    wave_lds_sync();

    // ---- next page's parameters and codes, into the registers the score phase released ----
#pragma unroll
    for (int v4 = 0; v4 < 4; ++v4) praw[v4] = buf_load16<kAuxCached>(rp_nxt, voff_params, v4 * 16);
#pragma unroll
    for (int s = 0; s < 8; ++s) cu[s] = load_unit<W>(rc_nxt, voff_codes, s * 16 * UB);

    // ---- values: acc[h][:] = acc[h][:] * alpha_h + sum_n p_h[n] V[n][:] ----
    {
      const f32x4 al4 = *(const PQ_LDS f32x4*)static_cast<uintptr_t>(lds_addr(alpha_s[wave]));
      const float al[4] = {al4.x, al4.y, al4.z, al4.w};
#pragma unroll
      for (int h = 0; h < G; ++h)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[h][e] *= al[h];
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      consume_values<G>(ring[k % kRingSets], 4 * k, pw_addr, row, acc);
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        constexpr int kAhead = 4 * kRingSets;                      // rows between a refill and its use
        const int nrow = 4 * k + r + kAhead;                       // compile-time after unrolling
        if (nrow < 32) ring[k % kRingSets][r] = buf_load16<kAuxStream>(rv_cur, voff_values, nrow * 1024);
        else           ring[k % kRingSets][r] = buf_load16<kAuxStream>(rv_nxt, voff_values, (nrow - 32) * 1024);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    wave_lds_sync();   // the next page overwrites prob[] / alpha_s[]
    rc_cur = rc_nxt; rp_cur = rp_nxt; rv_cur = rv_nxt; nv_cur = nv_nxt;
  }

  // ---- fold the four wavefronts into one partial per query head ----
  {
    const float l_tot = row_sum(l_run);
    if (owner && col == 0) {
      red_ml[wave][my_head][0] = m_run;
      red_ml[wave][my_head][1] = l_tot;
    }
#pragma unroll
    for (int h = 0; h < G; ++h) {
      float t[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) t[e] = sum_rows(acc[h][e]);
      if (row == 0) {
        float4* dst = reinterpret_cast<float4*>(&red_acc[wave][h][col * 8]);
        dst[0] = make_float4(t[0], t[1], t[2], t[3]);
        dst[1] = make_float4(t[4], t[5], t[6], t[7]);
      }
    }
  }
  __syncthreads();
  for (int idx = tid; idx < G * kHeadDim; idx += kThreads) {
    const int h = idx >> 7, dim = idx & (kHeadDim - 1);
    float M = kNegInf;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) M = fmaxf(M, red_ml[w][h][0]);
    float o = 0.f, l = 0.f;
    if (M > kNegInf) {
#pragma unroll
      for (int w = 0; w < kWaves; ++w) {
        const float wgt = __builtin_amdgcn_exp2f(red_ml[w][h][0] - M);
        o = fmaf(wgt, red_acc[w][h][dim], o);
        l = fmaf(wgt, red_ml[w][h][1], l);
      }
    }
    const int64_t slot = (static_cast<int64_t>(seq) * a.n_q_heads + kvh * G + h) * a.n_chunks + chunk;
    a.ws_acc[slot * kHeadDim + dim] = o;
    if (dim == 0) {
      a.ws_ml[slot * 2] = M;
      a.ws_ml[slot * 2 + 1] = l;
    }
  }
}

// out[seq][head][:] = sum_c 2^(m_c - M) acc_c / sum_c 2^(m_c - M) l_c over the chunks the
// sequence really has.  One work-group of 128 threads per (head, seq): thread = (chunk slice
// tid / 32, dims 4 * (tid % 32) ..+3); the four slices take chunks c = slice, slice + 4, ...
// with independent 128-bit loads and are folded through LDS.
__global__ __launch_bounds__(kHeadDim) void pq_decode_merge_kernel(
    const float* __restrict__ ws_acc, const float* __restrict__ ws_ml,
    const int32_t* __restrict__ seq_lens, float* __restrict__ out, int32_t n_q_heads,
    int32_t max_seq_len, int32_t pages_per_chunk, int32_t n_chunks) {
  __shared__ float4 part_o[4][32];
  __shared__ float part_l[4];
  const int head = blockIdx.x, seq = blockIdx.y, tid = threadIdx.x;
  const int slice = tid >> 5, quad = tid & 31;
  const int L = min(seq_lens[seq], max_seq_len);
  const int64_t oh = static_cast<int64_t>(seq) * n_q_heads + head;
  if (L <= 0) {
    out[oh * kHeadDim + tid] = 0.f;
    return;
  }
  const int n_pages = (L + kGroup - 1) / kGroup;
  const int nc = (n_pages + pages_per_chunk - 1) / pages_per_chunk;
  const float2* ml = reinterpret_cast<const float2*>(ws_ml) + oh * n_chunks;
  const float4* ac = reinterpret_cast<const float4*>(ws_acc + oh * n_chunks * kHeadDim) + quad;
  float M = kNegInf;
#pragma unroll 4
  for (int c = 0; c < nc; ++c) M = fmaxf(M, ml[c].x);
  float4 o = make_float4(0.f, 0.f, 0.f, 0.f);
  float l = 0.f;
  if (M > kNegInf) {
#pragma unroll 4
    for (int c = slice; c < nc; c += 4) {
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
    const float lt = part_l[0] + part_l[1] + part_l[2] + part_l[3];
    float4 r = part_o[0][quad];
#pragma unroll
    for (int s2 = 1; s2 < 4; ++s2) {
      const float4 t = part_o[s2][quad];
      r.x += t.x; r.y += t.y; r.z += t.z; r.w += t.w;
    }
    const float inv = lt > 0.f ? 1.f / lt : 0.f;
    reinterpret_cast<float4*>(out + oh * kHeadDim)[quad] = make_float4(r.x * inv, r.y * inv, r.z * inv, r.w * inv);
  }
}

// ---- query-key scores only (the kernel the paper times in Section 5.2) ------------------
// Same table, same page walk and same pair steps as the attention kernel, without softmax and
// values: every wavefront scores its pages and stores the raw q . k~ of valid tokens.
template <int G, int RB, int TB, typename QT>
__global__ __launch_bounds__(kThreads) void pq_score_keys_kernel(const DecodeArgs a) {
  constexpr int W = RB + TB;
  constexpr int UB = 2 * W;
  constexpr int NA = 1 << TB;
  constexpr int ROW = NA * 16;
  __shared__ __attribute__((aligned(16))) uint8_t lut[kPairs * ROW];

  const int kvh = blockIdx.x, seq = blockIdx.y, chunk = blockIdx.z;
  const int L = min(a.seq_lens[seq], a.max_seq_len);
  if (L <= 0) return;
  const int n_pages = (L + kGroup - 1) / kGroup;
  const int page0 = chunk * a.pages_per_chunk;
  if (page0 >= n_pages) return;
  const int npg = min(a.pages_per_chunk, n_pages - page0);
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int row = lane >> 4, col = lane & 15;
  const int my_head = (G == 4) ? row : (G == 2 ? (row >> 1) : 0);
  const bool owner = (G == 4) || (G == 2 && (row & 1) == 0) || (G == 1 && row == 0);
  const uint32_t lut_row0 = lds_addr(lut) + row * (kPairsPerUnit * ROW);
  const uint32_t voff_codes = (row * kGroup + col) * UB;
  const uint32_t voff_params = row * (kPairsPerUnit * 4);
  constexpr uint32_t kCodesBytes = kBlocks * kGroup * UB;

  const int n_w = npg > wave ? (npg - wave + kWaves - 1) / kWaves : 0;
  int pid_lane = -1;
  if (lane < n_w) {
    const int64_t pid = a.block_table[static_cast<int64_t>(seq) * a.max_pages_per_seq + page0 + wave + kWaves * lane];
    if (pid >= 0 && pid < a.n_pool_pages) pid_lane = static_cast<int>(pid);
  }
  auto page_setup = [&](int k, __amdgpu_buffer_rsrc_t& rc, __amdgpu_buffer_rsrc_t& rp, int& nv) {
    const int pid = __builtin_amdgcn_readlane(pid_lane, k);
    const bool ok = pid >= 0;
    const int64_t ph = ok ? static_cast<int64_t>(pid) * a.n_kv_heads + kvh : 0;
    nv = ok ? min(kGroup, L - (page0 + wave + kWaves * k) * kGroup) : 0;
    rc = make_rsrc(a.codes + ph * kCodesBytes, ok ? kCodesBytes : 0u);
    rp = make_rsrc(a.params + ph * kPairs, ok ? kPairs * 4u : 0u);
  };
  const __amdgpu_buffer_rsrc_t rs_empty = make_rsrc(a.codes, 0u);
  __amdgpu_buffer_rsrc_t rc_cur = rs_empty, rp_cur = rs_empty, rc_nxt = rs_empty, rp_nxt = rs_empty;
  int nv_cur = 0, nv_nxt = 0;
  uint4 praw[4];
  Unit<W / 2> cu[8];
  if (n_w > 0) {
    page_setup(0, rc_cur, rp_cur, nv_cur);
#pragma unroll
    for (int i = 0; i < 4; ++i) praw[i] = buf_load16<kAuxCached>(rp_cur, voff_params, i * 16);
#pragma unroll
    for (int i = 0; i < 8; ++i) cu[i] = load_unit<W>(rc_cur, voff_codes, i * 16 * UB);
  }
  {
    const QT* qb = static_cast<const QT*>(a.q) + (static_cast<int64_t>(seq) * a.n_q_heads + kvh * G) * kHeadDim;
    float* lf = reinterpret_cast<float*>(lut);
    for (int idx = tid; idx < kPairs * NA; idx += kThreads) {
      const int j = idx >> TB, s = idx & (NA - 1);
      const float cs = a.cos_tab[s], sn = a.sin_tab[s];
#pragma unroll
      for (int h = 0; h < G; ++h) {
        const float qx = static_cast<float>(qb[h * kHeadDim + j]);
        const float qy = static_cast<float>(qb[h * kHeadDim + j + kPairs]);
        lf[idx * 4 + h] = fmaf(qx, cs, qy * sn);
      }
    }
  }
  __syncthreads();

  float* const out_row = a.scores + (static_cast<int64_t>(seq) * a.n_q_heads + kvh * G + my_head) * a.scores_stride;
  for (int i = 0; i < n_w; ++i) {
    const int pi = page0 + wave + kWaves * i;
    if (i + 1 < n_w) {
      page_setup(i + 1, rc_nxt, rp_nxt, nv_nxt);
    } else {
      rc_nxt = rp_nxt = rs_empty;
      nv_nxt = 0;
    }
    float sf[16], zz[16];
#pragma unroll
    for (int v4 = 0; v4 < 4; ++v4) {
      const uint32_t w4[4] = {praw[v4].x, praw[v4].y, praw[v4].z, praw[v4].w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const __half2 sz = *reinterpret_cast<const __half2*>(&w4[e]);
        const float s = __low2float(sz), z = __high2float(sz);
        sf[v4 * 4 + e] = s;
        zz[v4 * 4 + e] = fmaf(0.5f, s, z);
      }
    }
#pragma unroll
    for (int v4 = 0; v4 < 4; ++v4) praw[v4] = buf_load16<kAuxCached>(rp_nxt, voff_params, v4 * 16);
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      float part[G];
#pragma unroll
      for (int h = 0; h < G; ++h) part[h] = 0.f;
      score_steps<G, RB, TB, 0>(cu[s], lut_row0, sf, zz, part);
      cu[s] = load_unit<W>(rc_nxt, voff_codes, s * 16 * UB);       // next page's pass s
      float sc;
      if constexpr (G == 4) {
        sc = tsum16(tsum32(part[0], part[2]), tsum32(part[1], part[3]));
      } else if constexpr (G == 2) {
        const float b = tsum32(part[0], part[1]);
        sc = tsum16(b, b);
      } else {
        sc = sum_rows(part[0]);
      }
      const int tok = s * 16 + col;
      if (owner && tok < nv_cur) out_row[static_cast<int64_t>(pi) * kGroup + tok] = sc;
    }
    rc_cur = rc_nxt; rp_cur = rp_nxt; nv_cur = nv_nxt;
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
    if (sc) hipLaunchKernelGGL((pq_decode_partials_kernel<G, RB, TB, __half, true>), grid, dim3(kThreads), 0, st, a);
    else    hipLaunchKernelGGL((pq_decode_partials_kernel<G, RB, TB, __half, false>), grid, dim3(kThreads), 0, st, a);
  } else {
    if (sc) hipLaunchKernelGGL((pq_decode_partials_kernel<G, RB, TB, float, true>), grid, dim3(kThreads), 0, st, a);
    else    hipLaunchKernelGGL((pq_decode_partials_kernel<G, RB, TB, float, false>), grid, dim3(kThreads), 0, st, a);
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

int check_decode_shape(const pq_layout* l, int32_t n_seqs, int32_t n_q_heads, int32_t max_seq_len) {
  if (!l || n_seqs <= 0 || n_q_heads <= 0 || max_seq_len <= 0) return PQ_ERR_INVALID_ARG;
  if (l->n_kv_heads <= 0 || n_q_heads % l->n_kv_heads != 0) return PQ_ERR_INVALID_ARG;
  if (!layout_supported(l)) return PQ_ERR_UNSUPPORTED;
  const int G = n_q_heads / l->n_kv_heads;
  if (G != 1 && G != 2 && G != 4) return PQ_ERR_UNSUPPORTED;
  if (n_seqs > 65535 || n_q_heads > 65535) return PQ_ERR_UNSUPPORTED;   // grid.y, merge grid.x
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
                                  const void* v_pool, int64_t n_pool_pages, const int32_t* block_table,
                                  int32_t max_pages_per_seq, const int32_t* seq_lens, int32_t max_seq_len,
                                  float sm_scale, float* scores, int64_t scores_stride,
                                  const void* residual_keys, void* workspace, size_t workspace_bytes,
                                  void* hip_stream) {
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
  a.block_table = block_table;
  a.seq_lens = seq_lens;
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
  const int G = n_q_heads / layout->n_kv_heads;
  hipError_t e = hipSuccess;
  const int rt = layout->r_bits * 10 + layout->t_bits;
  switch (rt) {
    case 44: e = launch_partials_g<4, 4>(G, a, q_dtype, grid, stream); break;
    case 33: e = launch_partials_g<3, 3>(G, a, q_dtype, grid, stream); break;
    case 53: e = launch_partials_g<5, 3>(G, a, q_dtype, grid, stream); break;
    case 35: e = launch_partials_g<3, 5>(G, a, q_dtype, grid, stream); break;
    case 42: e = launch_partials_g<4, 2>(G, a, q_dtype, grid, stream); break;
    case 24: e = launch_partials_g<2, 4>(G, a, q_dtype, grid, stream); break;
    default: return PQ_ERR_UNSUPPORTED;
  }
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
  hipLaunchKernelGGL(pq_decode_merge_kernel, dim3(n_q_heads, n_seqs), dim3(kHeadDim), 0,
                     static_cast<hipStream_t>(hip_stream), ws.acc, ws.ml, seq_lens, out, n_q_heads,
                     max_seq_len, plan.pages_per_chunk, plan.n_chunks);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return record_hip_error(e);
  return PQ_OK;
}

extern "C" int pq_decode_attention(const pq_layout* layout, const void* q, pq_dtype q_dtype, int32_t n_seqs,
                                   int32_t n_q_heads, const void* codes_pool, const void* params_pool,
                                   const void* v_pool, int64_t n_pool_pages, const int32_t* block_table,
                                   int32_t max_pages_per_seq, const int32_t* seq_lens, int32_t max_seq_len,
                                   float sm_scale, float* out, float* scores, int64_t scores_stride,
                                   const void* residual_keys, void* workspace, size_t workspace_bytes,
                                   void* hip_stream) {
  if (!out) return PQ_ERR_INVALID_ARG;
  const int st = pq_decode_partials(layout, q, q_dtype, n_seqs, n_q_heads, codes_pool, params_pool, v_pool,
                                    n_pool_pages, block_table, max_pages_per_seq, seq_lens, max_seq_len,
                                    sm_scale, scores, scores_stride, residual_keys, workspace, workspace_bytes,
                                    hip_stream);
  if (st != PQ_OK) return st;
  return pq_decode_merge(layout, n_seqs, n_q_heads, seq_lens, max_seq_len, out, workspace, workspace_bytes,
                         hip_stream);
}

extern "C" int pq_score_keys(const pq_layout* layout, const void* q, pq_dtype q_dtype, int32_t n_seqs,
                             int32_t n_q_heads, const void* codes_pool, const void* params_pool,
                             int64_t n_pool_pages, const int32_t* block_table, int32_t max_pages_per_seq,
                             const int32_t* seq_lens, int32_t max_seq_len, float* scores,
                             int64_t scores_stride, void* hip_stream) {
  const int st = check_decode_shape(layout, n_seqs, n_q_heads, max_seq_len);
  if (st != PQ_OK) return st;
  if (!q || !codes_pool || !params_pool || !block_table || !seq_lens || !scores) return PQ_ERR_INVALID_ARG;
  if (q_dtype != PQ_F16 && q_dtype != PQ_F32) return PQ_ERR_INVALID_ARG;
  if (n_pool_pages <= 0 || max_pages_per_seq <= 0 || scores_stride < max_seq_len) return PQ_ERR_INVALID_ARG;
  const int64_t need_pages = (static_cast<int64_t>(max_seq_len) + kGroup - 1) / kGroup;
  if (need_pages > max_pages_per_seq) return PQ_ERR_INVALID_ARG;
  const ChunkPlan plan = plan_chunks(n_seqs, layout->n_kv_heads, max_seq_len);
  DecodeArgs a = {};
  a.q = q;
  a.codes = static_cast<const uint8_t*>(codes_pool);
  a.params = static_cast<const uint32_t*>(params_pool);
  a.block_table = block_table;
  a.seq_lens = seq_lens;
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
  const int G = n_q_heads / layout->n_kv_heads;
  hipError_t e = hipSuccess;
  switch (layout->r_bits * 10 + layout->t_bits) {
    case 44: e = launch_scores<4, 4>(G, a, q_dtype, grid, stream); break;
    case 33: e = launch_scores<3, 3>(G, a, q_dtype, grid, stream); break;
    case 53: e = launch_scores<5, 3>(G, a, q_dtype, grid, stream); break;
    case 35: e = launch_scores<3, 5>(G, a, q_dtype, grid, stream); break;
    case 42: e = launch_scores<4, 2>(G, a, q_dtype, grid, stream); break;
    case 24: e = launch_scores<2, 4>(G, a, q_dtype, grid, stream); break;
    default: return PQ_ERR_UNSUPPORTED;
  }
  if (e != hipSuccess) return record_hip_error(e);
  return PQ_OK;
}
