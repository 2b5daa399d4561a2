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
// This header holds what the decode kernels share (streaming loads, table builds, pair steps,
// value steps, residual keys) and two of the kernels: pq_decode_partials_kernel, whose
// wavefronts alternate between a score and a value phase, and the score-only kernels.  The
// attention kernel that serves large launches, with wavefronts specialised by role, is in
// pq_decode_roles.hpp; how a launch is shared out and merged inside the kernel is in
// pq_decode_sched.hpp.
//
// Mapping to the machine in the attention kernels.  A work-group is 4 wavefronts; the table of
// all query heads that share the KV head lives in LDS with the heads interleaved (one 16-byte
// entry serves 4 heads).  Pages (= quantization groups) are owned by one wavefront, so a page's
// radius parameters are loaded once into registers:
//   score  : lane = (pair block q = lane / 16, token tk = lane % 16).  One
//            128-bit (96-bit for w = 6) load brings the 16 symbols of pairs
//            16q .. 16q+15; the 16 lanes of a row read 16 consecutive units.
//            The four rows' partial sums are folded with v_permlane32_swap /
//            v_permlane16_swap so that row h ends up holding head h's score.
//   softmax: online, per page, in the log2 domain (running max m, sum l).
//   values : lane = (token slot lane / 16, dims 8*(lane % 16) ..+7); 128-bit
//            loads of fp16 rows, probabilities broadcast from LDS.
// In pq_decode_partials_kernel a last step folds the four wavefronts' (m, l, acc) into one
// partial per (sequence, query head, chunk); pq_decode_merge_kernel combines the chunks.
// (The score-only kernel of the uniform grid maps lanes to tokens instead: see PageWalk.)
// No MFMA: the hot loop is a gather-accumulate.
//
// Grouped angle quantizer (Section 3.2 as printed; template flag GA): the angle levels of a
// group are theta~_a = (a + 1/2) s_t + z_t with the group's own (s_t, z_t), so every wavefront
// keeps a table of its own in LDS and rebuilds it from the page's angle parameters before it
// scores the page (the appendix listing builds the same table from "tscale" and "tmn").
#pragma once
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>
#include <math.h>

#include <type_traits>

#include "pq_internal.hpp"

namespace pq {


constexpr int kWaves = 4;
constexpr int kThreads = kWaves * 64;
constexpr float kNegInf = -INFINITY;

struct DecodeArgs {
  const void* q;
  const uint8_t* codes;
  const uint32_t* params;   // {fp16 s, fp16 z} per pair, viewed as one dword
  const __half* values;     // fp16 value pool, or the quantized value pool when the kernel's VB is 4 or 2
  const uint32_t* v_params; // quantized values: {fp16 scale, fp16 zero} per (page, kv head, token)
  const __half* residual;   // [seq][kv_head][g][d] un-quantized keys of the last, incomplete group (or null)
  const int32_t* block_table;
  const int32_t* seq_lens;
  int32_t n_seqs;
  float* scores;
  float* ws_acc;            // [seq][q_head][chunk][128]; balanced launches: [slot][head of the group][128]
  float* ws_ml;             // [seq][q_head][chunk][2] = (m in log2 units, l); balanced: [slot][head of the group][2]
  // launches whose work-groups share the pages out evenly and merge in the kernel (pq_decode_sched.hpp)
  float* out;               // [seq][q_head][128]
  uint64_t* arrivals;       // one arrival word per (sequence, KV head), then one per segment slot
  int32_t min_pages;        // smallest share of a work-group, in pages
  int32_t unit_cost;        // what starting on a (sequence, KV head) costs a work-group, in pages
  int32_t xcd_skew_permille;  // how much more than the average share an even-numbered work-group takes
  int32_t q_is_f32;         // the query is fp32 (else fp16)
  int32_t grid_mode;        // role-specialised kernel: one work-group per (KV head, sequence, chunk) instead
  int64_t scores_stride;
  int64_t n_pool_pages;
  int32_t n_kv_heads;
  int32_t n_q_heads;
  int32_t group_total;      // query heads per KV head (any value); one launch covers G of them ...
  int32_t head0;            // ... starting at this head of the group
  int32_t max_pages_per_seq;
  int32_t max_seq_len;
  int32_t pages_per_chunk;
  int32_t n_chunks;
  float scale_log2;         // sm_scale * log2(e)
  float cos_tab[kMaxAngleBins];
  float sin_tab[kMaxAngleBins];
};

// Launchers of the instantiation units (rt = 10 r + t).  They return false, and launch nothing,
// if there is no kernel for the combination; launch errors are left to hipGetLastError().
// pq_decode_partials.hip / pq_decode_partials_ga.hip: the attention kernel whose wavefronts
// alternate between a score and a value phase, uniform angle grid / grouped angle quantizer.
bool launch_attention_partials(int rt, int G, int v_bits, const DecodeArgs& a, dim3 grid, hipStream_t st);
bool launch_attention_partials_ga(int rt, int G, int v_bits, const DecodeArgs& a, dim3 grid, hipStream_t st);

namespace {

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
// Maximum / sum over all 64 lanes, result in every lane: inside a row of 16 by DPP (lane ^ 1,
// lane ^ 2, mirror within 8, mirror within 16), across the rows by the two lane-swap instructions.
template <int CTRL>
__device__ __forceinline__ float dpp_of(float x) {
  return u2f(static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(f2u(x)), CTRL, 0xf, 0xf, true)));
}
__device__ __forceinline__ float wave_max(float x) {
  x = fmaxf(x, dpp_of<0xB1>(x));      // quad_perm(1,0,3,2)
  x = fmaxf(x, dpp_of<0x4E>(x));      // quad_perm(2,3,0,1)
  x = fmaxf(x, dpp_of<0x141>(x));     // row_half_mirror
  x = fmaxf(x, dpp_of<0x140>(x));     // row_mirror
  auto r = __builtin_amdgcn_permlane16_swap(f2u(x), f2u(x), false, false);
  x = fmaxf(u2f(r[0]), u2f(r[1]));
  auto q = __builtin_amdgcn_permlane32_swap(f2u(x), f2u(x), false, false);
  return fmaxf(u2f(q[0]), u2f(q[1]));
}
__device__ __forceinline__ float wave_sum_f(float x) {
  x += dpp_of<0xB1>(x);
  x += dpp_of<0x4E>(x);
  x += dpp_of<0x141>(x);
  x += dpp_of<0x140>(x);
  return sum_rows(x);
}

// Sum of the four 16-lane rows' partial scores: with 4 query heads row h ends with head h's
// score (transposing fold), with 2 heads rows 0-1 / 2-3, with 1 head every row; with 8 heads row h
// ends with the scores of heads h and h + 4 (two transposing folds).
template <int G>
struct Folded {
  float v[G == 8 ? 2 : 1];
};
template <int G>
__device__ __forceinline__ Folded<G> fold_rows(const float (&part)[G]) {
  Folded<G> f;
  if constexpr (G == 8) {
    f.v[0] = tsum16(tsum32(part[0], part[2]), tsum32(part[1], part[3]));
    f.v[1] = tsum16(tsum32(part[4], part[6]), tsum32(part[5], part[7]));
  } else if constexpr (G == 4) {
    f.v[0] = tsum16(tsum32(part[0], part[2]), tsum32(part[1], part[3]));
  } else if constexpr (G == 2) {
    const float b = tsum32(part[0], part[1]);
    f.v[0] = tsum16(b, b);
  } else {
    f.v[0] = sum_rows(part[0]);
  }
  return f;
}

// LDS written by some lanes of this wavefront is about to be read by others.
__device__ __forceinline__ void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Tuning constants of the attention kernel (measured on MI355X): 4 quads of 4 value rows in
// flight per wavefront (8 rows in flight measure the same, 4 rows 4 % slower; the number of
// quads must divide the 8 quads of a page), and a register budget of 2 wavefronts per SIMD --
// with 4 query heads a third wavefront only fits with spills and runs 10-30 % slower.
#ifndef PQ_RING_SETS
#define PQ_RING_SETS 4
#endif
// Quantized values: units in flight per wavefront.  With 4 instead of 8 a third wavefront per SIMD
// fits without spills; measured, that is 5 % slower than two wavefronts with a whole page in flight.
#ifndef PQ_VQ_RING
#define PQ_VQ_RING 8
#endif
#define PQ_KERNEL_ATTR __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(2, 2)))

// ---- streaming loads --------------------------------------------------------
// Codes, parameters and values are read through buffer descriptors that cover
// exactly one page of one KV head: the lane offset stays in one VGPR, the
// position inside the page is a scalar/immediate offset, and a read past the
// descriptor's size returns zeros instead of faulting (value rows beyond the
// sequence end are masked that way).  Everything streamed is read once, so the
// loads are non-temporal.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x3 __attribute__((ext_vector_type(3)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
constexpr int kAuxStream = 2;     // gfx950 cache-policy bit "nt"
constexpr int kAuxCached = 0;
constexpr int kAuxDevice = 16;    // gfx950 cache-policy bit "sc1": performed past the per-XCD L2s, coherent device-wide

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, uint32_t bytes) {
  // raw buffer, 32-bit data format, no swizzle
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, static_cast<int>(bytes), 0x00020000);
}
template <int AUX>
__device__ __forceinline__ uint4 buf_load16(__amdgpu_buffer_rsrc_t r, uint32_t voff, uint32_t soff) {
  const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(r, voff, soff, AUX);
  return make_uint4(v.x, v.y, v.z, v.w);
}

template <int AUX>
__device__ __forceinline__ uint32_t buf_load4(__amdgpu_buffer_rsrc_t r, uint32_t voff, uint32_t soff) {
  return __builtin_amdgcn_raw_buffer_load_b32(r, voff, soff, AUX);
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

// The G heads' values of one 16-byte entry; 8 heads are kept as two tables of 4-head entries, the
// second one HALF bytes after the first, so that an entry's offset is the same in both.
template <int G, int HALF = 0>
__device__ __forceinline__ Heads<G> lut_read(uint32_t addr) {
  Heads<G> t;
  if constexpr (G == 8) {
    static_assert(HALF > 0, "distance of the second table");
    const f32x4 f = *(const PQ_LDS f32x4*)static_cast<uintptr_t>(addr);
    const f32x4 g = *(const PQ_LDS f32x4*)static_cast<uintptr_t>(addr + HALF);
    t.v[0] = f.x; t.v[1] = f.y; t.v[2] = f.z; t.v[3] = f.w;
    t.v[4] = g.x; t.v[5] = g.y; t.v[6] = g.z; t.v[7] = g.w;
  } else if constexpr (G == 4) {
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

// Fields of pair K of a unit: the radius code as a float, and `base` plus the byte offset of the
// angle code's 16-byte table entry.
template <int RB, int TB, int K>
__device__ __forceinline__ void pair_fields(const Unit<(RB + TB) / 2>& u, uint32_t base, float& c, uint32_t& addr) {
  constexpr int W = RB + TB;
  if constexpr (RB == 4 && TB == 4) {
    // byte K of the unit is (a << 4) | c: mask once per dword, then one op per field
    const uint32_t d = u.d[K >> 2];
    const uint32_t rad = d & 0x0f0f0f0fu, ang = d & 0xf0f0f0f0u;   // CSE'd across the dword's 4 pairs
    c = byte_to_float<K & 3>(rad);
    addr = add_byte<K & 3>(ang, base);                            // (a << 4) is the entry's byte offset
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
    asm("v_lshl_add_u32 %0, %1, 4, %2" : "=v"(addr) : "v"(aq), "v"(base));
    c = byte_to_float<0>(cq);
  }
}

// One pair step: part[h] += rho~ * T[h][pair K of this lane's block][angle code].
// `lut_row0` is the LDS byte address of the lane's block (pair 16*row); radius
// parameters are (s, z + s/2) so that rho~ = c * s + zz.
template <int G, int RB, int TB, int K>
__device__ __forceinline__ void score_steps(const Unit<(RB + TB) / 2>& u, uint32_t lut_row0,
                                            const float (&sf)[16], const float (&zz)[16],
                                            float (&part)[G]) {
  if constexpr (K < 16) {
    constexpr int ROW = 16 << TB;
    float c;
    uint32_t addr;
    pair_fields<RB, TB, K>(u, lut_row0, c, addr);
    const float rho = fmaf(c, sf[K], zz[K]);
    const Heads<G> t = lut_read<G, kPairs * ROW>(addr + K * ROW);
#pragma unroll
    for (int h = 0; h < G; ++h) part[h] = fmaf(rho, t.v[h], part[h]);
    score_steps<G, RB, TB, K + 1>(u, lut_row0, sf, zz, part);
  }
}

// The same step where every lane of the wavefront works on the same pair (lane = token): the
// pair's radius parameters are the same for all lanes and stay in a scalar register as the
// stored {fp16 s, fp16 z} word; v_fma_mix_f32 reads the halves directly (one scalar register per
// instruction is what the hardware allows, and both halves are in one).
__device__ __forceinline__ float midpoint_offset(uint32_t sz) {     // z + s / 2
  float r;
  asm("v_fma_mix_f32 %0, %1, 0.5, %1 op_sel:[0,0,1] op_sel_hi:[1,0,1]" : "=v"(r) : "s"(sz));
  return r;
}
__device__ __forceinline__ float radius_from_code(float c, uint32_t sz, float zz) {   // c * s + zz
  float r;
  asm("v_fma_mix_f32 %0, %1, %2, %3 op_sel_hi:[0,1,0]" : "=v"(r) : "v"(c), "s"(sz), "v"(zz));
  return r;
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
        const Heads<G> q0 = lut_read<G, kHeadDim * 16>(qs_row + dim * 16);
        const Heads<G> q1 = lut_read<G, kHeadDim * 16>(qs_row + (dim + 1) * 16);
#pragma unroll
        for (int h = 0; h < G; ++h) part[h] = fmaf(k1, q1.v[h], fmaf(k0, q0.v[h], part[h]));
      }
    }
  }
}

// acc[h][0..7] += p_h[token] * V[token][this lane's 8 dims] for the 4 value rows in `vv`:
// the (it0 + i)-th 1 KB load of the page in its rotated order, i.e. tokens
// 4 * ((it0 + i + rot) % 32) + row; pw_row is the LDS address of prob[token = row][G].
template <int G>
__device__ __forceinline__ void consume_values(const uint4 (&vv)[4], int it0, uint32_t pw_row, int rot,
                                               float (&acc)[G][8]) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const Heads<G> p = lut_read<G>(pw_row + static_cast<uint32_t>((it0 + i + rot) & 31) * (4 * G * 4));
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

// ---- quantized values (token-wise b-bit codes, paper Section 2) ----------------------------
// acc[h][k] += sum over the unit's tokens of (p_h[token] * s_token) * code[token][dim k]: the
// token's scale is folded into its probability, the zero-points are summed separately (sum_n p_n
// z_n is the same for every dim).  A unit's 32-bit words hold two consecutive tokens each, the
// even one in the low half, and the probabilities come as fp16 pairs of the same two tokens, so
// that one v_dot2_f32_f16 does both tokens of a dim with an fp32 accumulator.  A code needs no
// conversion: masked in place it IS an fp16 number -- a denormal, code * 2^-24 when it sits in
// bits 0.. of its half, code * 2^(-24 + shift) further up -- so a pair of codes costs one AND
// (plus one shift per word for the fields beyond the mantissa), and each accumulator is scaled
// back by its power of two once, at the end (vq_unscale).
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float dot2(uint32_t p_pair, uint32_t code_pair, float acc) {
  f16x2 a, b;
  __builtin_memcpy(&a, &p_pair, 4);
  __builtin_memcpy(&b, &code_pair, 4);
  return __builtin_amdgcn_fdot2(a, b, acc, false);
}

template <int G>
struct Pairs {
  uint32_t v[G];
};
template <int G>
__device__ __forceinline__ Pairs<G> pairs_read(uint32_t addr) {
  const Heads<G> f = lut_read<G>(addr);
  Pairs<G> p;
#pragma unroll
  for (int h = 0; h < G; ++h) p.v[h] = f2u(f.v[h]);
  return p;
}

// The lane's value with that of its neighbour lane (lane ^ 1), as an fp16 pair (this lane's in
// the low half), round to nearest: called by the lanes that hold the probabilities of tokens
// n (even lanes) and n + 1; the even lanes store the result.
__device__ __forceinline__ uint32_t pack_with_neighbour(float x) {
  const float other = u2f(static_cast<uint32_t>(
      __builtin_amdgcn_update_dpp(0, static_cast<int>(f2u(x)), 0xB1 /* quad_perm(1,0,3,2) */, 0xf, 0xf, true)));
  const __half2 h = __floats2half2_rn(x, other);
  return *reinterpret_cast<const uint32_t*>(&h);
}

// The same with the lane four further on in its row of 16 (lane + 4): called where the lanes col
// and col + 4 hold the probabilities of tokens n and n + 4; the lanes with (col & 4) == 0 store.
__device__ __forceinline__ uint32_t pack_with_lane4(float x) {
  const float other = u2f(static_cast<uint32_t>(
      __builtin_amdgcn_update_dpp(0, static_cast<int>(f2u(x)), 0x104 /* row_shl:4 */, 0xf, 0xf, true)));
  const __half2 h = __floats2half2_rn(x, other);
  return *reinterpret_cast<const uint32_t*>(&h);
}

// fp16 values with 8 query heads: acc[h][0..7] += p_h[token] * V[token][this lane's 8 dims] for the
// 4 value rows in `vv`, the (it0 + i)-th 1 KB loads of the page in its rotated order (rot even),
// i.e. tokens 4 * ((it0 + i + rot) % 32) + row.  Rows i = 0, 1 and i = 2, 3 are token pairs
// (n, n + 4): their values are interleaved dim by dim (v_perm_b32) into fp16 pairs and meet the
// probability pairs [pair 4 * (load / 2) + row][8 heads] at `prob` in one v_dot2_f32_f16 per
// head and dim -- half the instructions of one multiply-add per token.
__device__ __forceinline__ void consume_values_pairs(const uint4 (&vv)[4], int it0, uint32_t prob, int rot, int row,
                                                     float (&acc)[8][8]) {
#pragma unroll
  for (int i = 0; i < 4; i += 2) {
    const uint32_t load = static_cast<uint32_t>((it0 + i + rot) & 31);
    const uint32_t pa = prob + ((4u * (load >> 1) + static_cast<uint32_t>(row)) * 8u) * 4u;
    const Pairs<4> p0 = pairs_read<4>(pa), p1 = pairs_read<4>(pa + 16);
    const uint32_t wa[4] = {vv[i].x, vv[i].y, vv[i].z, vv[i].w};
    const uint32_t wb[4] = {vv[i + 1].x, vv[i + 1].y, vv[i + 1].z, vv[i + 1].w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const uint32_t lo = __builtin_amdgcn_perm(wb[e], wa[e], 0x05040100u);   // dim 2e of tokens n, n + 4
      const uint32_t hi = __builtin_amdgcn_perm(wb[e], wa[e], 0x07060302u);   // dim 2e + 1
#pragma unroll
      for (int h = 0; h < 4; ++h) {
        acc[h][2 * e] = dot2(p0.v[h], lo, acc[h][2 * e]);
        acc[h][2 * e + 1] = dot2(p0.v[h], hi, acc[h][2 * e + 1]);
        acc[h + 4][2 * e] = dot2(p1.v[h], lo, acc[h + 4][2 * e]);
        acc[h + 4][2 * e + 1] = dot2(p1.v[h], hi, acc[h + 4][2 * e + 1]);
      }
    }
  }
}

// Power of two an accumulator of dim k (of the lane's 8) is multiplied with at the end: undoes
// the position of the dim's field above bit 0 of its half, and the 2^-24 of fp16 denormals.
template <int VB>
__device__ __forceinline__ constexpr float vq_unscale(int k) {
  // 4 bits: fields of dims 0-3 (or 4-7) at bits 0, 4, 8, 12 of a half; 8 and 12 are read after a shift by 8
  // 2 bits: fields of dims 0-7 at bits 0, 2, ..., 14; 10, 12, 14 are read after a shift by 10
  const int shift = VB == 4 ? ((k & 1) ? 4 : 0) : (k < 5 ? 2 * k : 2 * (k - 5));
  return static_cast<float>(1 << (24 - shift));
}

// One unit: `pp` is the LDS address of the fp16 probability pairs [token pair][G] of the unit's
// first token pair.
template <int G, int VB>
__device__ __forceinline__ void consume_quantized(const uint4& u, uint32_t pp, float (&acc)[G][8]) {
  const uint32_t w4[4] = {u.x, u.y, u.z, u.w};
  if constexpr (VB == 4) {
#pragma unroll
    for (int tp = 0; tp < 2; ++tp) {
      const Pairs<G> p = pairs_read<G>(pp + tp * (G * 4));
#pragma unroll
      for (int dh = 0; dh < 2; ++dh) {
        const uint32_t d = w4[2 * tp + dh], e = d >> 8;
        const uint32_t f[4] = {d & 0x000f000fu, d & 0x00f000f0u, e & 0x000f000fu, e & 0x00f000f0u};
#pragma unroll
        for (int k = 0; k < 4; ++k)
#pragma unroll
          for (int h = 0; h < G; ++h) acc[h][4 * dh + k] = dot2(p.v[h], f[k], acc[h][4 * dh + k]);
      }
    }
  } else {
    static_assert(VB == 2, "value bits");
#pragma unroll
    for (int tp = 0; tp < 4; ++tp) {
      const Pairs<G> p = pairs_read<G>(pp + tp * (G * 4));
      const uint32_t d = w4[tp], e = d >> 10;
      const uint32_t f[8] = {d & 0x00030003u, d & 0x000c000cu, d & 0x00300030u, d & 0x00c000c0u, d & 0x03000300u,
                             e & 0x00030003u, e & 0x000c000cu, e & 0x00300030u};
#pragma unroll
      for (int k = 0; k < 8; ++k)
#pragma unroll
        for (int h = 0; h < G; ++h) acc[h][k] = dot2(p.v[h], f[k], acc[h][k]);
    }
  }
}

// ---- pieces shared by the attention kernels and the score-only kernel -------------------

// q[dim][head] as fp32 in LDS (heads beyond G zero), and the grid's (cos, sin) pairs: first step of
// the table build; also read by the residual-key dot products and by the per-group table builds
// of the grouped angle quantizer.  In two halves, so that a kernel can put other loads between
// the fetch and its use; a work-group barrier must follow the store before LDS is read.
template <int G>
struct QueryRegs {
  float q[G];
  float2 cs;
};
template <int G, typename QT>
__device__ __forceinline__ QueryRegs<G> fetch_query(const QT* qb, const DecodeArgs& a, int tid) {
  QueryRegs<G> r = {};
  if (tid < kHeadDim) {
#pragma unroll
    for (int h = 0; h < G; ++h) r.q[h] = static_cast<float>(qb[h * kHeadDim + tid]);
  } else if (tid < kHeadDim + kMaxAngleBins) {
    r.cs = make_float2(a.cos_tab[tid - kHeadDim], a.sin_tab[tid - kHeadDim]);
  }
  return r;
}
template <int G>
__device__ __forceinline__ void store_query_lds(float (*q_lds)[4], float2* trig, const QueryRegs<G>& r, int tid) {
  if (tid < kHeadDim) {
    // heads 4-7 (G = 8) make a second [dim][4] table behind the first
#pragma unroll
    for (int h = 0; h < (G == 8 ? 8 : 4); ++h) q_lds[(h >> 2) * kHeadDim + tid][h & 3] = h < G ? r.q[h < G ? h : 0] : 0.f;
  } else if (tid < kHeadDim + kMaxAngleBins) {
    trig[tid - kHeadDim] = r.cs;
  }
}
// The G query heads from element `q_at` of a.q on; the query's type (fp16 / fp32) is a run-time
// property of the call.
template <int G>
__device__ __forceinline__ QueryRegs<G> fetch_query(const DecodeArgs& a, int64_t q_at, int tid) {
  return a.q_is_f32 ? fetch_query<G, float>(static_cast<const float*>(a.q) + q_at, a, tid)
                    : fetch_query<G, __half>(static_cast<const __half*>(a.q) + q_at, a, tid);
}
template <int G>
__device__ __forceinline__ void load_query_lds(float (*q_lds)[4], float2* trig, const DecodeArgs& a, int64_t q_at,
                                               int tid) {
  store_query_lds<G>(q_lds, trig, fetch_query<G>(a, q_at, tid), tid);
}

// Table of the uniform angle grid (Section 3.3): T[j][a][h] = q_x[h][j] cos(theta~_a) + q_y[h][j]
// sin(theta~_a), 16 bytes per (pair, state) entry whatever G is, from the q and (cos, sin) that
// load_query_lds left in LDS; written by all `n_threads` threads of the work-group.
template <int TB>
__device__ __forceinline__ void build_uniform_table(uint8_t* lut, const float (*q_lds)[4], const float2* trig, int tid,
                                                    int n_threads) {
  constexpr int NA = 1 << TB;
  const uint32_t lut_a = lds_addr(lut), q_a = lds_addr(q_lds), t_a = lds_addr(trig);
  for (int idx = tid; idx < kPairs * NA; idx += n_threads) {
    const int j = idx >> TB, s = idx & (NA - 1);
    const f32x2 cs = *(const PQ_LDS f32x2*)static_cast<uintptr_t>(t_a + s * 8);
    const f32x4 qx = *(const PQ_LDS f32x4*)static_cast<uintptr_t>(q_a + j * 16);
    const f32x4 qy = *(const PQ_LDS f32x4*)static_cast<uintptr_t>(q_a + (j + kPairs) * 16);
    f32x4 t;
    t.x = fmaf(qx.x, cs.x, qy.x * cs.y);
    t.y = fmaf(qx.y, cs.x, qy.y * cs.y);
    t.z = fmaf(qx.z, cs.x, qy.z * cs.y);
    t.w = fmaf(qx.w, cs.x, qy.w * cs.y);
    *(PQ_LDS f32x4*)static_cast<uintptr_t>(lut_a + idx * 16) = t;
  }
}

// Radius parameters of this lane's 16 pairs from the four 128-bit words {fp16 s, fp16 z} x 4:
// rho~ = c * sf + zz with zz = z + s / 2 (mid-point reconstruction, Section 3.2).
__device__ __forceinline__ void unpack_radius_params(const uint4 (&praw)[4], float (&sf)[16], float (&zz)[16]) {
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
}

// Raw scores of a residual group (the un-quantized fp16 keys of a sequence's last, incomplete
// group): plain dot products in the score-phase lane layout (lane = (pair block row, token col),
// each lane takes the 32 dims of its 16 pairs), folded like the table-lookup partial sums.  Key
// rows past `nv_res` read as zero.  `emit(pass, score)` is called once per pass of 16 tokens with
// the score(s) of token 16 * pass + col for the lane's head(s) (valid in the lanes that own a head).
template <int G, typename Emit>
__device__ __forceinline__ void residual_scores(const __half* res_rows, int nv_res, uint32_t q_lds_addr, int row,
                                                int col, Emit emit) {
  const __amdgpu_buffer_rsrc_t rs_res = make_rsrc(res_rows, static_cast<uint32_t>(nv_res) * (kHeadDim * 2));
  const uint32_t voff_res = col * (kHeadDim * 2) + row * 32;
  const uint32_t qs_row = q_lds_addr + row * (16 * 16);
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
    emit(s, fold_rows<G>(part));   // a Folded<G>
  }
}

// Grouped angle quantizer: this wavefront's table T[j][a][h] = q_x[h][j] cos(theta~) + q_y[h][j]
// sin(theta~), theta~ = (a + 1/2) s_t[j] + z_t[j] (Section 3.2 reconstruction, Section 3.3 table),
// for the page whose angle parameters {fp16 s_t, fp16 z_t} of pair `lane` are in `tpar`.
// Entry e = 64 * it + lane = (pair e >> t, state e & (2^t - 1)): consecutive lanes write
// consecutive 16-byte entries.  q_addr is the LDS byte address of q[dim][4 heads].
template <int TB>
__device__ __forceinline__ void build_group_table(uint32_t lut_w, uint32_t tpar, uint32_t q_addr, int lane) {
  constexpr int NA = 1 << TB;
  const float level = static_cast<float>(lane & (NA - 1)) + 0.5f;
#ifndef PQ_BUILD_UNROLL
#define PQ_BUILD_UNROLL 4          // fully unrolled, the attention kernel spills registers
#endif
#pragma unroll PQ_BUILD_UNROLL
  for (int it = 0; it < NA; ++it) {
    const int j = it * (64 >> TB) + (lane >> TB);
    const uint32_t p = static_cast<uint32_t>(__shfl(static_cast<int>(tpar), j));
    const __half2 sz = *reinterpret_cast<const __half2*>(&p);
    const float rev = fmaf(level, __low2float(sz), __high2float(sz)) * 0.15915494309189535f;   // turns
    const float cs = __builtin_amdgcn_cosf(rev), sn = __builtin_amdgcn_sinf(rev);
    const f32x4 qx = *(const PQ_LDS f32x4*)static_cast<uintptr_t>(q_addr + j * 16);
    const f32x4 qy = *(const PQ_LDS f32x4*)static_cast<uintptr_t>(q_addr + (j + kPairs) * 16);
    f32x4 t;
    t.x = fmaf(qx.x, cs, qy.x * sn);
    t.y = fmaf(qx.y, cs, qy.y * sn);
    t.z = fmaf(qx.z, cs, qy.z * sn);
    t.w = fmaf(qx.w, cs, qy.w * sn);
    *(PQ_LDS f32x4*)static_cast<uintptr_t>(lut_w + (it * 64 + lane) * 16) = t;
  }
}

// ---- score phase with lanes as tokens (uniform angle grid) ---------------------------------
// Used by the score-only kernel and the role-specialised attention kernel.  (In the attention
// kernel below, whose wavefronts alternate between scoring and aggregating, it measured the same
// as the lane layout that kernel has -- 158 against 157 us with 4-bit values at the GQA shape --
// and was not taken over.)  The lanes of a wavefront are 64 consecutive TOKENS of
// a page and walk the 64 pairs together, block of 16 pairs by block, both halves of the page per
// block.  Because all lanes read the same pair's table row (16 bytes per angle state, at most
// 512 bytes: every LDS bank at most once, equal states broadcast), the gather is free of bank
// conflicts whatever the codes are; the pair's radius parameters are wavefront-uniform and come
// through scalar loads, one block (64 bytes) at a time, each block replaced by the next page's
// as soon as it has been used.  Per pair and token: the field extraction, one conversion, one
// multiply-add for the radius, G for the heads.
typedef uint32_t u32x16 __attribute__((ext_vector_type(16)));
#define PQ_CONST __attribute__((address_space(4)))
struct BlockParams {
  uint32_t sz[16];     // {fp16 s, fp16 z} of the block's 16 pairs
};
// `page_params` is wavefront-uniform and points to valid memory
__device__ __forceinline__ BlockParams load_block_params(const uint32_t* page_params, int block) {
  const u32x16 v = *reinterpret_cast<const PQ_CONST u32x16*>(reinterpret_cast<uintptr_t>(page_params + block * kPairsPerUnit));
  BlockParams p;
#pragma unroll
  for (int i = 0; i < 16; ++i) p.sz[i] = v[i];
  return p;
}

// A page's 128 steps of a lane -- step S: pair block kBlockOrder[S / 32], half of the page
// (S / 16) % 2, pair S % 16 of the block -- with the table reads kScorePipe steps ahead of their
// use.  Written out step by step, each step closed for the instruction scheduler: under this
// kernel's register budget the compiler otherwise issues one read, waits for it, and so on.  As
// a block's last step goes by, its parameters are replaced by the next page's; as a unit's last
// read is issued, the unit is replaced by the next page's.
// The sum over the 64 pairs is associated exactly as in the attention kernels, where the four
// 16-lane rows each sum one block and fold_rows adds (block 0 + block 2) + (block 1 + block 3):
// a score from here equals, bit for bit, the one the attention kernels compute.
template <int G, int RB, int TB, int kScorePipe = 4>
struct PageWalk {
  static constexpr int W = RB + TB;
  static constexpr int UB = 2 * W;
  static constexpr int ROW = 16 << TB;
  static constexpr int kRing = kScorePipe + 1;   // reads in flight, plus the one in use
  Unit<W / 2> cu[2 * kBlocks];                   // unit (half, block) at [half * kBlocks + block]
  BlockParams par[kBlocks];
  float zz[16];
  float c[kRing];
  Heads<G> t[kRing];
  float cur[2][G], sum02[2][G], sum13[2][G];     // per half of the page: the running block, and the pairs of blocks
  float score[2][G];
  uint32_t lut_base, voff_codes;

  static constexpr uint32_t unit_at(int half, int b) { return static_cast<uint32_t>((b * kGroup + half * 64) * UB); }
  static constexpr int block_of(int S) { return ((S / 32) >> 1) | (((S / 32) & 1) << 1); }   // 0, 2, 1, 3

  template <int S>
  __device__ __forceinline__ void issue(__amdgpu_buffer_rsrc_t rc_nxt) {
    if constexpr (S < 128) {
      constexpr int b = block_of(S), half = (S / 16) % 2, K = S % 16;
      uint32_t addr;
      pair_fields<RB, TB, K>(cu[half * kBlocks + b], lut_base, c[S % kRing], addr);
      t[S % kRing] = lut_read<G, kPairs * ROW>(addr + (b * kPairsPerUnit + K) * ROW);
      if constexpr (K == 15) cu[half * kBlocks + b] = load_unit<W>(rc_nxt, voff_codes, unit_at(half, b));
    }
  }
  template <int S>
  __device__ __forceinline__ void steps(__amdgpu_buffer_rsrc_t rc_nxt, const uint32_t* pp_nxt) {
    if constexpr (S < 128) {
      constexpr int j = S / 32, b = block_of(S), half = (S / 16) % 2, K = S % 16;
      if constexpr (S % 32 == 0) {
#pragma unroll
        for (int k = 0; k < 16; ++k) zz[k] = midpoint_offset(par[b].sz[k]);
      }
      issue<S + kScorePipe>(rc_nxt);
      const float rho = radius_from_code(c[S % kRing], par[b].sz[K], zz[K]);
#pragma unroll
      for (int h = 0; h < G; ++h) cur[half][h] = fmaf(rho, t[S % kRing].v[h], K == 0 ? 0.f : cur[half][h]);
      if constexpr (K == 15) {
#pragma unroll
        for (int h = 0; h < G; ++h) {
          if constexpr (j == 0) sum02[half][h] = cur[half][h];
          else if constexpr (j == 1) sum02[half][h] += cur[half][h];
          else if constexpr (j == 2) sum13[half][h] = cur[half][h];
          else score[half][h] = sum02[half][h] + (sum13[half][h] + cur[half][h]);
        }
      }
      if constexpr (S % 32 == 31) par[b] = load_block_params(pp_nxt, b);
      __builtin_amdgcn_sched_barrier(0);
      steps<S + 1>(rc_nxt, pp_nxt);
    }
  }
  // scores of the page in cu / par (left in `score`); cu / par then hold the next page
  __device__ __forceinline__ void run(__amdgpu_buffer_rsrc_t rc_nxt, const uint32_t* pp_nxt) {
    issue<0>(rc_nxt);
    issue<1>(rc_nxt);
    if constexpr (kScorePipe > 2) issue<2>(rc_nxt);
    if constexpr (kScorePipe > 3) issue<3>(rc_nxt);
    if constexpr (kScorePipe > 4) issue<4>(rc_nxt);
    if constexpr (kScorePipe > 5) issue<5>(rc_nxt);
    static_assert(kScorePipe >= 2 && kScorePipe <= 6, "reads in flight");
    steps<0>(rc_nxt, pp_nxt);
    // The scores exist here, whatever the caller's control flow does with them: left to itself
    // the compiler moves a head's 64 multiply-adds behind a later condition under which the score
    // is used, away from their table reads, whose results then wait in (spilled) registers.
#pragma unroll
    for (int half = 0; half < 2; ++half)
#pragma unroll
      for (int h = 0; h < G; ++h) asm volatile("" : "+v"(score[half][h]));
  }
};

// Online softmax (log2 domain) of a score wavefront whose lanes are tokens: the lane holds the raw
// scores of tokens `lane` and 64 + `lane` of a page for all G heads (PageWalk::score), so a head's
// maximum is a wavefront-wide reduction and its running maximum and rescaling factor are
// uniform; the denominators stay per-lane partial sums until the end.  A page's probabilities go
// to LDS at `pw` in the layout the value steps read:
//   fp16 values, G <= 4 : fp32 [token][G]
//   fp16 values, G == 8 : fp16 pairs of tokens (n, n + 4), [pair = 8 (n / 16) + n % 4 + 4 ((n % 16) / 8)][8]
//   quantized values    : fp16 pairs of tokens (2m, 2m + 1) with the token's scale folded in, [m][G]
// and the heads' rescaling factors to `alpha_out[0 .. G)`.
template <int G, int VB>
struct LaneSoftmax {
  static constexpr bool kQuantV = VB != 16;
  static constexpr bool kPairs16 = kQuantV || G == 8;       // probabilities leave as fp16 pairs
  float m_run[G], l_run[G], z_run[kQuantV ? G : 1];

  __device__ __forceinline__ void reset() {
#pragma unroll
    for (int h = 0; h < G; ++h) {
      m_run[h] = kNegInf;
      l_run[h] = 0.f;
      if constexpr (kQuantV) z_run[h] = 0.f;
    }
  }
  // score[half][h]: raw scores; nv: valid tokens of the page; vpar[half]: {fp16 scale, fp16 zero} of
  // the lane's tokens (quantized values).  `is_residual`: the page is the residual group, whose
  // scores [token][G] are taken from LDS at `res_sc` instead.  `out_rows`: where to store raw scores
  // (row of head 0 at the page's first token, rows `stride` apart), or null.
  __device__ __forceinline__ void page(const float (&score)[2][G], int nv, float scale_log2, const uint32_t (&vpar)[2],
                                       bool is_residual, uint32_t res_sc, float* out_rows, int64_t stride, uint32_t pw,
                                       float* alpha_out, int lane) {
    const int col = lane & 15;
    float al[G];
    uint32_t packed[kPairs16 ? 2 : 1][G];
    float pf[kPairs16 ? 1 : 2][G];
#pragma unroll
    for (int h = 0; h < G; ++h) {
      float sc[2];
#pragma unroll
      for (int half = 0; half < 2; ++half) {
        const int tok = half * 64 + lane;
        sc[half] = score[half][h];
        if (is_residual) sc[half] = *(const PQ_LDS float*)static_cast<uintptr_t>(res_sc + (tok * G + h) * 4);
        if (out_rows != nullptr) {
          if (tok < nv) out_rows[h * stride + tok] = sc[half];
        }
        sc[half] = (tok < nv) ? sc[half] * scale_log2 : kNegInf;
      }
      const float pm = wave_max(fmaxf(sc[0], sc[1]));
      const float m_new = fmaxf(m_run[h], pm);
      const bool dead = !(m_new > kNegInf);                          // nothing valid seen so far
      const float alpha = dead ? 1.f : __builtin_amdgcn_exp2f(m_run[h] - m_new);   // 0 on the first page
      float psum = 0.f, zsum = 0.f;
#pragma unroll
      for (int half = 0; half < 2; ++half) {
        const float pr = dead ? 0.f : __builtin_amdgcn_exp2f(sc[half] - m_new);
        psum += pr;
        if constexpr (kQuantV) {
          // V~ = code * s + z (Section 2): fold s into the probability, collect p * z
          const __half2 sz = *reinterpret_cast<const __half2*>(&vpar[half]);
          zsum = fmaf(pr, __high2float(sz), zsum);
          packed[half][h] = pack_with_neighbour(pr * __low2float(sz));
        } else if constexpr (G == 8) {
          packed[half][h] = pack_with_lane4(pr);
        } else {
          pf[half][h] = pr;
        }
      }
      if constexpr (kQuantV) z_run[h] = fmaf(z_run[h], alpha, zsum);
      l_run[h] = fmaf(l_run[h], alpha, psum);
      m_run[h] = m_new;
      al[h] = alpha;
    }
    // the lane's probabilities, all heads of a token (pair) side by side
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      const int tok = half * 64 + lane;
      if constexpr (kQuantV) {
        if ((lane & 1) == 0) {
#pragma unroll
          for (int h = 0; h < G; ++h) *(PQ_LDS uint32_t*)static_cast<uintptr_t>(pw + ((tok >> 1) * G + h) * 4) = packed[half][h];
        }
      } else if constexpr (G == 8) {
        if ((col & 4) == 0) {
          const int pidx = (tok >> 4) * 8 + (col & 3) + ((col >> 3) << 2);
#pragma unroll
          for (int h = 0; h < G; ++h) *(PQ_LDS uint32_t*)static_cast<uintptr_t>(pw + (pidx * G + h) * 4) = packed[half][h];
        }
      } else {
#pragma unroll
        for (int h = 0; h < G; ++h) *(PQ_LDS float*)static_cast<uintptr_t>(pw + (tok * G + h) * 4) = pf[half][h];
      }
    }
    if (lane == 0) {
#pragma unroll
      for (int h = 0; h < G; ++h) alpha_out[h] = al[h];
    }
  }
  // (m, l, sum of p * zero-point) of head h over everything this wavefront has seen, to ml[h][0..2]
  __device__ __forceinline__ void finish(float (*ml)[3], int lane) {
#pragma unroll
    for (int h = 0; h < G; ++h) {
      const float l_tot = wave_sum_f(l_run[h]);
      const float z_tot = kQuantV ? wave_sum_f(z_run[kQuantV ? h : 0]) : 0.f;
      if (lane == 0) {
        ml[h][0] = m_run[h];
        ml[h][1] = l_tot;
        ml[h][2] = z_tot;
      }
    }
  }
};

template <int G, int RB, int TB, int VB, bool GA>
__global__ PQ_KERNEL_ATTR void pq_decode_partials_kernel(const DecodeArgs a) {
  constexpr int W = RB + TB;
  constexpr int UB = 2 * W;              // bytes per unit
  constexpr int NA = 1 << TB;            // angle states
  constexpr int ROW = NA * 16;           // table bytes per pair

  // one table per work-group, or (GA) one per wavefront; with GA the wavefront's table space is
  // reused for its accumulators in the final fold, which keeps two work-groups per compute unit
  constexpr int kLutBytes = kPairs * ROW;
  __shared__ __attribute__((aligned(16))) uint8_t lut[(GA ? kWaves : 1) * kLutBytes];
  __shared__ __attribute__((aligned(16))) float prob[kWaves][kGroup * G];
  __shared__ __attribute__((aligned(16))) float alpha_s[kWaves][4];
  __shared__ __attribute__((aligned(16))) float red_own[GA ? 4 : kWaves * G * kHeadDim];
  static_assert(!GA || kLutBytes >= G * kHeadDim * 4, "table space too small for the accumulators");
  __shared__ float red_ml[kWaves][G][3];                              // m, l, sum of p * zero-point
  __shared__ __attribute__((aligned(16))) float q_lds[kHeadDim][4];   // q[dim][head]: table build, residual keys
  __shared__ float2 trig[kMaxAngleBins];                              // (cos, sin) of the uniform grid's bin centres
  __shared__ float res_sc[kGroup * G];                                // raw scores of the residual group

  // Chunk-major launch order: the KV heads of one page are neighbours in memory and run
  // together; every sequence's first chunks run first, and the chunks that only long sequences
  // have (with the empty work-groups of the short ones) come last, which balances ragged batches.
  const int kvh = blockIdx.x, chunk = blockIdx.z;
  const int seq = blockIdx.y;
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

  float m_run = kNegInf, l_run = 0.f, z_run = 0.f;
  float acc[G][8];
#pragma unroll
  for (int h = 0; h < G; ++h)
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[h][e] = 0.f;

  const uint32_t lut_w = lds_addr(lut) + (GA ? wave * kLutBytes : 0);
  const uint32_t lut_row0 = lut_w + row * (kPairsPerUnit * ROW);
  auto red_acc = [&](int w) -> float* {   // [G][kHeadDim] accumulators of wavefront w in the final fold
    return GA ? reinterpret_cast<float*>(lut + w * kLutBytes) : red_own + w * (G * kHeadDim);
  };
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
  constexpr bool kQuantV = VB != 16;
  constexpr int kParamSets = GA ? 2 : 1;   // radius parameters (+ angle parameters) per pair
  constexpr int kVLoads = kQuantV ? kGroup * kHeadDim * VB / 8 / 1024 : 32;   // 1 KB wave-loads per page
  constexpr int kTokPerLoad = kGroup / kVLoads;                              // 16 (4 bit), 32 (2 bit)
  // The 32 one-KB value loads of a page are issued in an order rotated by a page-dependent
  // amount: pages and heads are a power-of-two number of bytes apart, and waves that walk them
  // in the same order keep hitting the same memory channels together (measured with a bare
  // streaming kernel: 6.6 TB/s in lock-step order, 7.0 TB/s rotated).
  auto page_setup = [&](int k, __amdgpu_buffer_rsrc_t& rc, __amdgpu_buffer_rsrc_t& rp,
                        __amdgpu_buffer_rsrc_t& rv, __amdgpu_buffer_rsrc_t& rvp, int& nv, int& rot) {
    const int pid = __builtin_amdgcn_readlane(pid_lane, k);
    const bool ok = pid >= 0;
    rot = ok ? (pid * 13 + kvh * 5) & 31 : 0;
    const int64_t ph = ok ? static_cast<int64_t>(pid) * a.n_kv_heads + kvh : 0;
    nv = ok ? min(kGroup, L - (page0 + wave + kWaves * k) * kGroup) : 0;
    const bool packed = ok && (page0 + wave + kWaves * k) != res_page;   // the residual group has no codes yet
    rc = make_rsrc(a.codes + ph * kCodesBytes, packed ? kCodesBytes : 0u);
    rp = make_rsrc(a.params + ph * (kPairs * kParamSets), packed ? kPairs * 4u * kParamSets : 0u);
    if constexpr (kQuantV) {
      // whole units are read; codes of slots past the sequence end are finite by construction
      // and meet a zero probability.  Their parameters could be anything: bounded by nv.
      rv = make_rsrc(reinterpret_cast<const uint8_t*>(a.values) + ph * (kGroup * kHeadDim * VB / 8),
                     nv > 0 ? kGroup * kHeadDim * VB / 8 : 0u);
      rvp = make_rsrc(a.v_params + ph * kGroup, static_cast<uint32_t>(nv) * 4u);
    } else {
      rv = make_rsrc(a.values + ph * (kGroup * kHeadDim), static_cast<uint32_t>(nv) * (kHeadDim * 2));
      rvp = rv;
    }
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
  __amdgpu_buffer_rsrc_t rc_cur = rs_empty, rp_cur = rs_empty, rv_cur = rs_empty, rvp_cur = rs_empty;
  __amdgpu_buffer_rsrc_t rc_nxt = rs_empty, rp_nxt = rs_empty, rv_nxt = rs_empty, rvp_nxt = rs_empty;
  int nv_cur = 0, nv_nxt = 0, rot_cur = 0, rot_nxt = 0;
  uint4 praw[4];
  uint32_t tpar = 0;                                               // GA: angle parameters of pair `lane`
  Unit<W / 2> cu[8];
  constexpr int kRingSets = PQ_RING_SETS;                          // register quads of 4 value rows in flight
  uint4 ring[kRingSets][4];                                        // fp16 values
  // quantized values: kVRing of the page's kVLoads units in flight; unit k sits in vq[k % kVRing]
  // and is replaced, once consumed, by unit k + kVRing (of the next page beyond the last unit)
  constexpr int kVRing = kVLoads < PQ_VQ_RING ? kVLoads : PQ_VQ_RING;
  uint4 vq[kQuantV ? kVRing : 1];
  uint32_t vpar[8];                                                // quantized values: (scale, zero) of tokens 16 t + col
  const uint32_t voff_vq = lane * 16;                              // lane (row, col): token block row, dim slice col
  const uint32_t voff_vpar = col * 4;
  if (n_w > 0) {
    page_setup(0, rc_cur, rp_cur, rv_cur, rvp_cur, nv_cur, rot_cur);
#pragma unroll
    for (int i = 0; i < 4; ++i) praw[i] = buf_load16<kAuxCached>(rp_cur, voff_params, i * 16);
    if constexpr (GA) tpar = buf_load4<kAuxCached>(rp_cur, lane * 4, kPairs * 4);
#pragma unroll
    for (int i = 0; i < 8; ++i) cu[i] = load_unit<W>(rc_cur, voff_codes, i * 16 * UB);
    if constexpr (kQuantV) {
#pragma unroll
      for (int t = 0; t < 8; ++t) vpar[t] = buf_load4<kAuxCached>(rvp_cur, voff_vpar, t * 64);
#pragma unroll
      for (int k = 0; k < kVRing; ++k) vq[k] = buf_load16<kAuxStream>(rv_cur, voff_vq, k * 1024);
    } else {
#pragma unroll
      for (int k = 0; k < kRingSets; ++k)
#pragma unroll
        for (int r = 0; r < 4; ++r)
          ring[k][r] = buf_load16<kAuxStream>(rv_cur, voff_values, static_cast<uint32_t>((4 * k + r + rot_cur) & 31) * 1024u);
    }
  }

  // ---- table of the G query heads that share this KV head (Section 3.3) ----
  // (built while the first page's loads, issued above, are in flight)
  {
    load_query_lds<G>(q_lds, trig, a, (static_cast<int64_t>(seq) * a.n_q_heads + kvh * a.group_total + a.head0) * kHeadDim, tid);
    if constexpr (!GA) {
      __syncthreads();
      build_uniform_table<TB>(lut, q_lds, trig, tid, kThreads);
    }
  }
  __syncthreads();

  // ---- residual group (at most one per sequence): scored here, before the page loop, by the
  // wavefront that owns its page -- plain dot products with the fp16 keys in the same lane
  // layout (each lane takes the 32 dims of its 16 pairs) and with the same fold; key rows past
  // the sequence end read as zero.  The loop below picks the scores up from LDS.
  if (res_page >= page0 + wave && res_page < page0 + npg && ((res_page - page0 - wave) & (kWaves - 1)) == 0) {
    residual_scores<G>(a.residual + (static_cast<int64_t>(seq) * a.n_kv_heads + kvh) * (kGroup * kHeadDim),
                       L - res_page * kGroup, lds_addr(q_lds), row, col, [&](int s, Folded<G> v) {
                         if (owner) res_sc[(s * 16 + col) * G + my_head] = v.v[0];
                       });
    wave_lds_sync();
  }

  // Two work-groups share a compute unit, and the SIMD favours the older wavefront among equal
  // priorities: the two take the higher priority in turns, page by page (see rotate_priority in
  // pq_decode_roles.hpp for the same effect there).
  const unsigned launch_index = blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z);
  const bool shares_cu = gridDim.x * gridDim.y * gridDim.z > 256u;
  const int turn0 = static_cast<int>((launch_index / 256u) & 1u);
  for (int i = 0; i < n_w; ++i) {
    if (shares_cu) {
      if ((turn0 + i) & 1) __builtin_amdgcn_s_setprio(1);
      else __builtin_amdgcn_s_setprio(0);
    }
    const int pi = page0 + wave + kWaves * i;                      // chunk-relative page of iteration i
    if (i + 1 < n_w) {
      page_setup(i + 1, rc_nxt, rp_nxt, rv_nxt, rvp_nxt, nv_nxt, rot_nxt);
    } else {
      rc_nxt = rp_nxt = rv_nxt = rvp_nxt = rs_empty;
      nv_nxt = 0;
      rot_nxt = 0;
    }

    if constexpr (GA) {
      // this page's table (the previous page's was released by the barrier that ended its value phase)
      build_group_table<TB>(lut_w, tpar, lds_addr(q_lds), lane);
      wave_lds_sync();
    }

    // radius parameters of this lane's 16 pairs: rho~ = c * s + (z + s/2)
    float sf[16], zz[16];
    unpack_radius_params(praw, sf, zz);

    // ---- scores of the page's 128 tokens: 8 passes of 16 tokens ----
    float sc[8];
    if (pi != res_page) {
#pragma unroll
      for (int s = 0; s < 8; ++s) {
        float part[G];
#pragma unroll
        for (int h = 0; h < G; ++h) part[h] = 0.f;
        score_steps<G, RB, TB, 0>(cu[s], lut_row0, sf, zz, part);
        sc[s] = fold_rows<G>(part).v[0];
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
      if (a.scores != nullptr) {
        if (owner && tok < nv_cur)
          a.scores[(static_cast<int64_t>(seq) * a.n_q_heads + kvh * a.group_total + a.head0 + my_head) * a.scores_stride +
                   static_cast<int64_t>(pi) * kGroup + tok] = sc[t];
      }
      sc[t] = (tok < nv_cur) ? sc[t] * a.scale_log2 : kNegInf;
      pm = fmaxf(pm, sc[t]);
    }
    pm = row_max(pm);
    const float m_new = fmaxf(m_run, pm);
    const bool dead = !(m_new > kNegInf);                          // nothing valid seen so far
    const float alpha = dead ? 1.f : __builtin_amdgcn_exp2f(m_run - m_new);   // 0 on the first page
    float psum = 0.f, zsum = 0.f;
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      const float p = dead ? 0.f : __builtin_amdgcn_exp2f(sc[t] - m_new);
      psum += p;
      if constexpr (kQuantV) {
        // V~ = code * s + z (Section 2): fold s into the probability, collect p * z; the
        // probabilities of tokens 2m, 2m + 1 (neighbour lanes) go to LDS as one fp16 pair
        const __half2 sz = *reinterpret_cast<const __half2*>(&vpar[t]);
        zsum = fmaf(p, __high2float(sz), zsum);
        const uint32_t pr = pack_with_neighbour(p * __low2float(sz));
        if (owner && (col & 1) == 0)
          *(PQ_LDS uint32_t*)static_cast<uintptr_t>(pw_addr + ((t * 8 + (col >> 1)) * G + my_head) * 4) = pr;
      } else {
        if (owner) *(PQ_LDS float*)static_cast<uintptr_t>(pw_addr + ((t * 16 + col) * G + my_head) * 4) = p;
      }
    }
    if constexpr (kQuantV) z_run = fmaf(z_run, alpha, zsum);
    l_run = fmaf(l_run, alpha, psum);
    m_run = m_new;
    if (owner && col == 0) alpha_s[wave][my_head] = alpha;
    wave_lds_sync();

    // ---- next page's parameters and codes, into the registers the score phase released ----
#pragma unroll
    for (int v4 = 0; v4 < 4; ++v4) praw[v4] = buf_load16<kAuxCached>(rp_nxt, voff_params, v4 * 16);
    if constexpr (GA) tpar = buf_load4<kAuxCached>(rp_nxt, lane * 4, kPairs * 4);
#pragma unroll
    for (int s = 0; s < 8; ++s) cu[s] = load_unit<W>(rc_nxt, voff_codes, s * 16 * UB);
    if constexpr (kQuantV) {
#pragma unroll
      for (int t = 0; t < 8; ++t) vpar[t] = buf_load4<kAuxCached>(rvp_nxt, voff_vpar, t * 64);
    }

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
    if constexpr (kQuantV) {
      // unit k of the page = tokens kTokPerLoad * k + (16 / VB) * row ..; refilled with the next page's unit k
#pragma unroll
      for (int k = 0; k < kVLoads; ++k) {
        consume_quantized<G, VB>(vq[k % kVRing], pw_addr + ((kTokPerLoad * k + (16 / VB) * row) >> 1) * (G * 4), acc);
        if (k + kVRing < kVLoads) vq[k % kVRing] = buf_load16<kAuxStream>(rv_cur, voff_vq, (k + kVRing) * 1024);
        else vq[k % kVRing] = buf_load16<kAuxStream>(rv_nxt, voff_vq, (k + kVRing - kVLoads) * 1024);
        __builtin_amdgcn_sched_barrier(0);
      }
    } else {
  #pragma unroll
      for (int k = 0; k < 8; ++k) {
        consume_values<G>(ring[k % kRingSets], 4 * k, pw_addr + row * (G * 4), rot_cur, acc);
  #pragma unroll
        for (int r = 0; r < 4; ++r) {
          constexpr int kAhead = 4 * kRingSets;                      // rows between a refill and its use
          const int nrow = 4 * k + r + kAhead;                       // compile-time after unrolling
          if (nrow < 32)
            ring[k % kRingSets][r] = buf_load16<kAuxStream>(rv_cur, voff_values, static_cast<uint32_t>((nrow + rot_cur) & 31) * 1024u);
          else
            ring[k % kRingSets][r] = buf_load16<kAuxStream>(rv_nxt, voff_values, static_cast<uint32_t>((nrow - 32 + rot_nxt) & 31) * 1024u);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    wave_lds_sync();   // the next page overwrites prob[] / alpha_s[]
    rc_cur = rc_nxt; rp_cur = rp_nxt; rv_cur = rv_nxt; rvp_cur = rvp_nxt; nv_cur = nv_nxt; rot_cur = rot_nxt;
  }

  // ---- fold the four wavefronts into one partial per query head ----
  {
    const float l_tot = row_sum(l_run);
    const float z_tot = kQuantV ? row_sum(z_run) : 0.f;
    if (owner && col == 0) red_ml[wave][my_head][2] = z_tot;
    if (owner && col == 0) {
      red_ml[wave][my_head][0] = m_run;
      red_ml[wave][my_head][1] = l_tot;
    }
#pragma unroll
    for (int h = 0; h < G; ++h) {
      float t[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        t[e] = sum_rows(acc[h][e]);
        if constexpr (kQuantV) t[e] *= vq_unscale<VB>(e);
      }
      if (row == 0) {
        float4* dst = reinterpret_cast<float4*>(red_acc(wave) + h * kHeadDim + col * 8);
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
        o = fmaf(wgt, red_acc(w)[h * kHeadDim + dim] + red_ml[w][h][2], o);
        l = fmaf(wgt, red_ml[w][h][1], l);
      }
    }
    const int64_t slot = (static_cast<int64_t>(seq) * a.n_q_heads + kvh * a.group_total + a.head0 + h) * a.n_chunks + chunk;
    a.ws_acc[slot * kHeadDim + dim] = o;
    if (dim == 0) {
      a.ws_ml[slot * 2] = M;
      a.ws_ml[slot * 2 + 1] = l;
    }
  }
}

// ---- query-key scores only, grouped angle quantizer --------------------------------------
// Same tables, same page walk and same pair steps as the attention kernel, without softmax and
// values: every wavefront scores its pages and stores the raw q . k~ of valid tokens.  (The
// uniform grid is served by pq_score_tokens_kernel below; GA = false is not instantiated.)
template <int G, int RB, int TB, bool GA>
__global__ __launch_bounds__(kThreads) void pq_score_keys_kernel(const DecodeArgs a) {
  static_assert(GA, "the uniform grid is served by pq_score_tokens_kernel");
  constexpr int W = RB + TB;
  constexpr int UB = 2 * W;
  constexpr int NA = 1 << TB;
  constexpr int ROW = NA * 16;
  constexpr int kLutBytes = kPairs * ROW;
  constexpr int kParamSets = GA ? 2 : 1;
  __shared__ __attribute__((aligned(16))) uint8_t lut[(GA ? kWaves : 1) * kLutBytes];   // GA: one table per wavefront
  __shared__ __attribute__((aligned(16))) float q_lds[kHeadDim][4];   // q[dim][head]: table builds, residual keys
  __shared__ float2 trig[kMaxAngleBins];                              // (cos, sin) of the uniform grid's bin centres

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
  const uint32_t lut_w = lds_addr(lut) + (GA ? wave * kLutBytes : 0);
  const uint32_t lut_row0 = lut_w + row * (kPairsPerUnit * ROW);
  const uint32_t voff_codes = (row * kGroup + col) * UB;
  const uint32_t voff_params = row * (kPairsPerUnit * 4);
  constexpr uint32_t kCodesBytes = kBlocks * kGroup * UB;

  const int res_page = (a.residual != nullptr && (L % kGroup) != 0) ? L / kGroup : -1;
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
    const bool packed = ok && (page0 + wave + kWaves * k) != res_page;   // the residual group has no codes yet
    rc = make_rsrc(a.codes + ph * kCodesBytes, packed ? kCodesBytes : 0u);
    rp = make_rsrc(a.params + ph * (kPairs * kParamSets), packed ? kPairs * 4u * kParamSets : 0u);
  };
  const __amdgpu_buffer_rsrc_t rs_empty = make_rsrc(a.codes, 0u);
  __amdgpu_buffer_rsrc_t rc_cur = rs_empty, rp_cur = rs_empty, rc_nxt = rs_empty, rp_nxt = rs_empty;
  int nv_cur = 0, nv_nxt = 0;
  uint4 praw[4];
  uint32_t tpar = 0;
  Unit<W / 2> cu[8];
  if (n_w > 0) {
    page_setup(0, rc_cur, rp_cur, nv_cur);
#pragma unroll
    for (int i = 0; i < 4; ++i) praw[i] = buf_load16<kAuxCached>(rp_cur, voff_params, i * 16);
    if constexpr (GA) tpar = buf_load4<kAuxCached>(rp_cur, lane * 4, kPairs * 4);
#pragma unroll
    for (int i = 0; i < 8; ++i) cu[i] = load_unit<W>(rc_cur, voff_codes, i * 16 * UB);
  }
  {
    load_query_lds<G>(q_lds, trig, a, (static_cast<int64_t>(seq) * a.n_q_heads + kvh * a.group_total + a.head0) * kHeadDim, tid);
    if constexpr (!GA) {
      __syncthreads();
      build_uniform_table<TB>(lut, q_lds, trig, tid, kThreads);
    }
  }
  __syncthreads();

  float* const out_row = a.scores + (static_cast<int64_t>(seq) * a.n_q_heads + kvh * a.group_total + a.head0 + my_head) * a.scores_stride;

  // With a residual buffer the last, incomplete group of the sequence is fp16 keys: plain dot
  // products, by the wavefront that owns the group's page (same lane layout and fold as below).
  if (res_page >= page0 + wave && res_page < page0 + npg && ((res_page - page0 - wave) & (kWaves - 1)) == 0) {
    const int nv_res = L - res_page * kGroup;
    residual_scores<G>(a.residual + (static_cast<int64_t>(seq) * a.n_kv_heads + kvh) * (kGroup * kHeadDim), nv_res,
                       lds_addr(q_lds), row, col, [&](int s, Folded<G> v) {
                         const int tok = s * 16 + col;
                         if (owner && tok < nv_res) out_row[static_cast<int64_t>(res_page) * kGroup + tok] = v.v[0];
                       });
  }

  for (int i = 0; i < n_w; ++i) {
    const int pi = page0 + wave + kWaves * i;
    if (i + 1 < n_w) {
      page_setup(i + 1, rc_nxt, rp_nxt, nv_nxt);
    } else {
      rc_nxt = rp_nxt = rs_empty;
      nv_nxt = 0;
    }
    if constexpr (GA) {
      wave_lds_sync();                                             // the previous page's table is no longer read
      build_group_table<TB>(lut_w, tpar, lds_addr(q_lds), lane);
      wave_lds_sync();
    }
    float sf[16], zz[16];
    unpack_radius_params(praw, sf, zz);
#pragma unroll
    for (int v4 = 0; v4 < 4; ++v4) praw[v4] = buf_load16<kAuxCached>(rp_nxt, voff_params, v4 * 16);
    if constexpr (GA) tpar = buf_load4<kAuxCached>(rp_nxt, lane * 4, kPairs * 4);
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      float part[G];
#pragma unroll
      for (int h = 0; h < G; ++h) part[h] = 0.f;
      score_steps<G, RB, TB, 0>(cu[s], lut_row0, sf, zz, part);
      cu[s] = load_unit<W>(rc_nxt, voff_codes, s * 16 * UB);       // next page's pass s
      const float sc = fold_rows<G>(part).v[0];
      const int tok = s * 16 + col;
      if (owner && tok < nv_cur && pi != res_page) out_row[static_cast<int64_t>(pi) * kGroup + tok] = sc;
    }
    rc_cur = rc_nxt; rp_cur = rp_nxt; nv_cur = nv_nxt;
  }
}

// ---- query-key scores only (the kernel the paper times in Section 5.2) ------------------
// Uniform angle grid: the token-lane walk (PageWalk) and nothing else -- every wavefront scores
// its pages, and a head's scores of 64 tokens leave as whole cache lines.
#ifndef PQ_SCORE_WAVES
#define PQ_SCORE_WAVES 4
#endif
template <int G, int RB, int TB>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(PQ_SCORE_WAVES, PQ_SCORE_WAVES)))
void pq_score_tokens_kernel(const DecodeArgs a) {
  constexpr int W = RB + TB;
  constexpr int UB = 2 * W;
  constexpr int NA = 1 << TB;
  constexpr int ROW = NA * 16;
  __shared__ __attribute__((aligned(16))) uint8_t lut[kPairs * ROW];
  __shared__ __attribute__((aligned(16))) float q_lds[kHeadDim][4];   // q[dim][head]: table build, residual keys
  __shared__ float2 trig[kMaxAngleBins];

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
  const uint32_t voff_codes = lane * UB;
  constexpr uint32_t kCodesBytes = kBlocks * kGroup * UB;

  const int res_page = (a.residual != nullptr && (L % kGroup) != 0) ? L / kGroup : -1;
  const int n_w = npg > wave ? (npg - wave + kWaves - 1) / kWaves : 0;   // pages of this wavefront: wave, wave + 4, ...
  int pid_lane = -1;
  if (lane < n_w) {
    const int64_t pid = a.block_table[static_cast<int64_t>(seq) * a.max_pages_per_seq + page0 + wave + kWaves * lane];
    if (pid >= 0 && pid < a.n_pool_pages) pid_lane = static_cast<int>(pid);
  }
  // codes descriptor, parameter address and valid tokens of the wavefront's k-th page; a masked
  // page or the residual group reads nothing (empty descriptor; parameters of pool page 0, unused)
  auto page_setup = [&](int k, __amdgpu_buffer_rsrc_t& rc, const uint32_t*& pp, int& nv) {
    const int pid = k < n_w ? __builtin_amdgcn_readlane(pid_lane, k) : -1;
    const bool ok = pid >= 0;
    const int64_t ph = (ok ? static_cast<int64_t>(pid) : 0) * a.n_kv_heads + kvh;
    nv = ok ? min(kGroup, L - (page0 + wave + kWaves * k) * kGroup) : 0;
    const bool packed = ok && (page0 + wave + kWaves * k) != res_page;
    rc = make_rsrc(a.codes + ph * kCodesBytes, packed ? kCodesBytes : 0u);
    pp = a.params + ph * kPairs;
  };
  __amdgpu_buffer_rsrc_t rc_cur, rc_nxt;
  const uint32_t* pp_cur;
  const uint32_t* pp_nxt;
  int nv_cur, nv_nxt;
  page_setup(0, rc_cur, pp_cur, nv_cur);
  PageWalk<G, RB, TB> w;
  w.voff_codes = voff_codes;
#pragma unroll
  for (int b = 0; b < kBlocks; ++b) w.par[b] = load_block_params(pp_cur, b);
#pragma unroll
  for (int b = 0; b < kBlocks; ++b)
#pragma unroll
    for (int half = 0; half < 2; ++half) w.cu[half * kBlocks + b] = load_unit<W>(rc_cur, voff_codes, w.unit_at(half, b));

  load_query_lds<G>(q_lds, trig, a, (static_cast<int64_t>(seq) * a.n_q_heads + kvh * a.group_total + a.head0) * kHeadDim, tid);
  __syncthreads();
  build_uniform_table<TB>(lut, q_lds, trig, tid, kThreads);
  __syncthreads();

  float* const out_rows = a.scores + (static_cast<int64_t>(seq) * a.n_q_heads + kvh * a.group_total + a.head0) * a.scores_stride;

  // the G heads' rows of scores through one descriptor (the host keeps 4 rows under 4 GiB): a
  // lane's offset is its token, the head's row the scalar offset
  const uint32_t row_bytes = static_cast<uint32_t>(a.scores_stride) * 4u;
  const __amdgpu_buffer_rsrc_t rs_out = make_rsrc(out_rows, static_cast<uint32_t>(G - 1) * row_bytes + static_cast<uint32_t>(L) * 4u);
  w.lut_base = lds_addr(lut);
  for (int i = 0; i < n_w; ++i) {
    const int pi = page0 + wave + kWaves * i;
    page_setup(i + 1, rc_nxt, pp_nxt, nv_nxt);
    w.run(rc_nxt, pp_nxt);
    // Unconditional stores (a conditional one would let the compiler move the page's arithmetic
    // behind the condition, away from its table reads): what must not be stored -- tokens past the
    // sequence end, a page without scores of its own -- gets an offset outside the descriptor.
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      const bool valid = pi != res_page && half * 64 + lane < nv_cur;
      const uint32_t vo = valid ? (static_cast<uint32_t>(pi) * kGroup + half * 64 + lane) * 4u : 0xffffffffu;
#pragma unroll
      for (int h = 0; h < G; ++h) __builtin_amdgcn_raw_buffer_store_b32(f2u(w.score[half][h]), rs_out, vo, h * row_bytes, kAuxStream);
    }
    rc_cur = rc_nxt; pp_cur = pp_nxt; nv_cur = nv_nxt;
  }

  // Last (the page loop's registers are free by now): with a residual buffer the last, incomplete
  // group of the sequence is fp16 keys: plain dot products, by the wavefront that owns the
  // group's page, in the lane layout of the attention kernels (lane = (pair block row, token
  // col), folded over the rows).
  if (res_page >= page0 + wave && res_page < page0 + npg && ((res_page - page0 - wave) & (kWaves - 1)) == 0) {
    const int row = lane >> 4, col = lane & 15;
    const int my_head = (G == 4) ? row : (G == 2 ? (row >> 1) : 0);
    const bool owner = (G == 4) || (G == 2 && (row & 1) == 0) || (G == 1 && row == 0);
    const int nv_res = L - res_page * kGroup;
    residual_scores<G>(a.residual + (static_cast<int64_t>(seq) * a.n_kv_heads + kvh) * (kGroup * kHeadDim), nv_res,
                       lds_addr(q_lds), row, col, [&](int s, Folded<G> v) {
                         const int tok = s * 16 + col;
                         if (owner && tok < nv_res)
                           out_rows[my_head * a.scores_stride + static_cast<int64_t>(res_page) * kGroup + tok] = v.v[0];
                       });
  }
}

}  // namespace
}  // namespace pq
