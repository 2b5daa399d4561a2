// Attention kernel with wavefronts specialised by role (fp16 values, uniform angle grid).
//
// Same work-group = one (sequence, KV head, chunk of pages), same table, layouts, score steps,
// value steps and partial results as pq_decode_partials_kernel (pq_decode_kernels.hpp); what
// differs is who does what.  The four wavefronts form two pairs; a pair takes every second page
// of the chunk.  In a pair the SCORE wavefront (0 or 1) streams the codes, runs the table-lookup
// product and the online softmax and leaves the page's probabilities and rescaling factor in
// LDS; the VALUE wavefront (2 or 3) streams the value rows and aggregates them with the
// probabilities of the page the score wavefront finished one step earlier.  One work-group
// barrier per step hands a probability buffer over (two buffers per pair).  Each role keeps only
// its own state in registers (codes, parameters and softmax state on one side; accumulators and
// the ring of value rows on the other), so three wavefronts fit a SIMD, and because wavefront w
// of a work-group runs on SIMD w, two SIMDs of a compute unit do arithmetic-heavy scoring while
// the other two keep the memory system busy -- instead of every wavefront alternating between a
// phase that waits for memory and one that does not touch it.
//
// Every wavefront of the work-group executes the same number of barriers: the step count is
// computed from the chunk's page count alone.
#pragma once
#include "pq_decode_kernels.hpp"

namespace pq {

hipError_t launch_partials_roles(int rt, int G, const DecodeArgs& a, pq_dtype qdt, dim3 grid, hipStream_t st);

namespace {

#ifndef PQ_ROLES_NP
#define PQ_ROLES_NP 2
#endif
constexpr int kPairsOfWaves = PQ_ROLES_NP;         // (score, value) wavefront pairs per work-group
constexpr int kRoleThreads = kPairsOfWaves * 128;

template <int G, int RB, int TB, typename QT, bool SCORES>
__global__ __launch_bounds__(kRoleThreads) __attribute__((amdgpu_waves_per_eu(3, 3)))
void pq_decode_roles_kernel(const DecodeArgs a) {
  constexpr int W = RB + TB;
  constexpr int UB = 2 * W;
  constexpr int NA = 1 << TB;
  constexpr int ROW = NA * 16;
  constexpr int kRing = 4;                                           // quads of 4 value rows in flight

  __shared__ __attribute__((aligned(16))) uint8_t lut[kPairs * ROW];
  __shared__ __attribute__((aligned(16))) float prob[kPairsOfWaves][2][kGroup * G];
  __shared__ __attribute__((aligned(16))) float alpha_s[kPairsOfWaves][2][4];
  __shared__ __attribute__((aligned(16))) float red_acc[kPairsOfWaves][G][kHeadDim];
  __shared__ float red_ml[kPairsOfWaves][G][2];
  __shared__ __attribute__((aligned(16))) float q_lds[kHeadDim][4];
  __shared__ float res_sc[kGroup * G];

  const int kvh = blockIdx.x, chunk = blockIdx.z;
  const int seq = a.seq_order ? a.seq_order[blockIdx.y] : static_cast<int>(blockIdx.y);
  if (seq < 0 || seq >= a.n_seqs) return;
  const int L = min(a.seq_lens[seq], a.max_seq_len);
  if (L <= 0) return;
  const int n_pages = (L + kGroup - 1) / kGroup;
  const int page0 = chunk * a.pages_per_chunk;
  if (page0 >= n_pages) return;
  const int npg = min(a.pages_per_chunk, n_pages - page0);

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int pair = wave % kPairsOfWaves;   // which share of the chunk's pages
  const bool scorer = wave < kPairsOfWaves;   // role of this wavefront
  const int row = lane >> 4, col = lane & 15;
  const int my_head = (G == 4) ? row : (G == 2 ? (row >> 1) : 0);
  const bool owner = (G == 4) || (G == 2 && (row & 1) == 0) || (G == 1 && row == 0);

  // pages of this pair: chunk pages pair, pair + 2, ...; the step count is the same for both pairs
  const int n_p = npg > pair ? (npg - pair + kPairsOfWaves - 1) / kPairsOfWaves : 0;
  const int n_steps = (npg + kPairsOfWaves - 1) / kPairsOfWaves + 1;   // pair 0's page count, plus one step of skew
  int pid_lane = -1;
  if (lane < n_p) {
    const int64_t pid = a.block_table[static_cast<int64_t>(seq) * a.max_pages_per_seq + page0 + pair + kPairsOfWaves * lane];
    if (pid >= 0 && pid < a.n_pool_pages) pid_lane = static_cast<int>(pid);
  }
  constexpr uint32_t kCodesBytes = kBlocks * kGroup * UB;
  const int res_page = (a.residual != nullptr && (L % kGroup) != 0) ? L / kGroup : -1;
  const __amdgpu_buffer_rsrc_t rs_empty = make_rsrc(a.values, 0u);

  // ---- table of the query heads, q for residual keys (all wavefronts) ----
  {
    const QT* qb = static_cast<const QT*>(a.q) + (static_cast<int64_t>(seq) * a.n_q_heads + kvh * a.group_total + a.head0) * kHeadDim;
    float* lf = reinterpret_cast<float*>(lut);
    for (int idx = tid; idx < kPairs * NA; idx += kRoleThreads) {
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
      for (int h = 0; h < 4; ++h) q_lds[tid][h] = h < G ? static_cast<float>(qb[h * kHeadDim + tid]) : 0.f;
    }
  }
  __syncthreads();

  if (scorer) {
    // =========================== SCORE wavefront ===========================
    const uint32_t lut_row0 = lds_addr(lut) + row * (kPairsPerUnit * ROW);
    const uint32_t voff_codes = (row * kGroup + col) * UB;
    const uint32_t voff_params = row * (kPairsPerUnit * 4);
    float m_run = kNegInf, l_run = 0.f;

    auto page_setup = [&](int k, __amdgpu_buffer_rsrc_t& rc, __amdgpu_buffer_rsrc_t& rp, int& nv) {
      const int pid = __builtin_amdgcn_readlane(pid_lane, k & 63);
      const bool ok = pid >= 0 && k < n_p;
      const int64_t ph = ok ? static_cast<int64_t>(pid) * a.n_kv_heads + kvh : 0;
      nv = ok ? min(kGroup, L - (page0 + pair + kPairsOfWaves * k) * kGroup) : 0;
      const bool packed = ok && (page0 + pair + kPairsOfWaves * k) != res_page;
      rc = make_rsrc(a.codes + ph * kCodesBytes, packed ? kCodesBytes : 0u);
      rp = make_rsrc(a.params + ph * kPairs, packed ? kPairs * 4u : 0u);
    };

    // residual group (plain dot products), if this pair owns its page
    if (res_page >= page0 + pair && res_page < page0 + npg && ((res_page - page0 - pair) % kPairsOfWaves) == 0) {
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

    __amdgpu_buffer_rsrc_t rc_cur, rp_cur, rc_nxt, rp_nxt;
    int nv_cur, nv_nxt;
    page_setup(0, rc_cur, rp_cur, nv_cur);
    uint4 praw[4];
    Unit<W / 2> cu[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) praw[i] = buf_load16<kAuxCached>(rp_cur, voff_params, i * 16);
#pragma unroll
    for (int i = 0; i < 8; ++i) cu[i] = load_unit<W>(rc_cur, voff_codes, i * 16 * UB);

    for (int t = 0; t < n_steps; ++t) {
      if (t < n_p) {
        const int pi = page0 + pair + kPairsOfWaves * t;
        page_setup(t + 1, rc_nxt, rp_nxt, nv_nxt);
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
        float sc[8];
#pragma unroll
        for (int s = 0; s < 8; ++s) {
          float part[G];
#pragma unroll
          for (int h = 0; h < G; ++h) part[h] = 0.f;
          score_steps<G, RB, TB, 0>(cu[s], lut_row0, sf, zz, part);
          cu[s] = load_unit<W>(rc_nxt, voff_codes, s * 16 * UB);       // the pair's next page, same pass
          sc[s] = fold_rows<G>(part);
        }
        if (pi == res_page) {
#pragma unroll
          for (int s = 0; s < 8; ++s)
            sc[s] = *(const PQ_LDS float*)static_cast<uintptr_t>(lds_addr(res_sc) + ((s * 16 + col) * G + my_head) * 4);
        }
        // online softmax (log2 domain); probabilities and rescaling factor go to buffer t % 2
        float pm = kNegInf;
#pragma unroll
        for (int k = 0; k < 8; ++k) {
          const int tok = k * 16 + col;
          if constexpr (SCORES) {
            if (owner && tok < nv_cur)
              a.scores[(static_cast<int64_t>(seq) * a.n_q_heads + kvh * a.group_total + a.head0 + my_head) * a.scores_stride +
                       static_cast<int64_t>(pi) * kGroup + tok] = sc[k];
          }
          sc[k] = (tok < nv_cur) ? sc[k] * a.scale_log2 : kNegInf;
          pm = fmaxf(pm, sc[k]);
        }
        pm = row_max(pm);
        const float m_new = fmaxf(m_run, pm);
        const bool dead = !(m_new > kNegInf);
        const float alpha = dead ? 1.f : __builtin_amdgcn_exp2f(m_run - m_new);
        const uint32_t pw = lds_addr(prob[pair][t & 1]);
        float psum = 0.f;
#pragma unroll
        for (int k = 0; k < 8; ++k) {
          const float p = dead ? 0.f : __builtin_amdgcn_exp2f(sc[k] - m_new);
          psum += p;
          if (owner) *(PQ_LDS float*)static_cast<uintptr_t>(pw + ((k * 16 + col) * G + my_head) * 4) = p;
        }
        l_run = fmaf(l_run, alpha, psum);
        m_run = m_new;
        if (owner && col == 0) alpha_s[pair][t & 1][my_head] = alpha;
        rc_cur = rc_nxt; rp_cur = rp_nxt; nv_cur = nv_nxt;
      }
      __syncthreads();                                               // hand buffer t % 2 to the value wavefront
    }
    const float l_tot = row_sum(l_run);
    if (owner && col == 0) {
      red_ml[pair][my_head][0] = m_run;
      red_ml[pair][my_head][1] = l_tot;
    }
  } else {
    // =========================== VALUE wavefront ===========================
    const uint32_t voff_values = row * (kHeadDim * 2) + col * 16;
    float acc[G][8];
#pragma unroll
    for (int h = 0; h < G; ++h)
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[h][e] = 0.f;

    auto page_setup = [&](int k, __amdgpu_buffer_rsrc_t& rv, int& rot) {
      const int pid = __builtin_amdgcn_readlane(pid_lane, k & 63);
      const bool ok = pid >= 0 && k < n_p;
      const int64_t ph = ok ? static_cast<int64_t>(pid) * a.n_kv_heads + kvh : 0;
      const int nv = ok ? min(kGroup, L - (page0 + pair + kPairsOfWaves * k) * kGroup) : 0;
      rot = ok ? (pid * 13 + kvh * 5) & 31 : 0;
      rv = make_rsrc(a.values + ph * (kGroup * kHeadDim), static_cast<uint32_t>(nv) * (kHeadDim * 2));
    };
    __amdgpu_buffer_rsrc_t rv_cur, rv_nxt;
    int rot_cur, rot_nxt;
    page_setup(0, rv_cur, rot_cur);
    uint4 ring[kRing][4];
#pragma unroll
    for (int k = 0; k < kRing; ++k)
#pragma unroll
      for (int r = 0; r < 4; ++r)
        ring[k][r] = buf_load16<kAuxStream>(rv_cur, voff_values, static_cast<uint32_t>((4 * k + r + rot_cur) & 31) * 1024u);

    for (int t = 0; t < n_steps; ++t) {
      const int j = t - 1;                                           // the page the score wavefront finished last step
      if (j >= 0 && j < n_p) {
        page_setup(j + 1, rv_nxt, rot_nxt);
        {
          const f32x4 al4 = *(const PQ_LDS f32x4*)static_cast<uintptr_t>(lds_addr(alpha_s[pair][j & 1]));
          const float al[4] = {al4.x, al4.y, al4.z, al4.w};
#pragma unroll
          for (int h = 0; h < G; ++h)
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[h][e] *= al[h];
        }
        const uint32_t pw_row = lds_addr(prob[pair][j & 1]) + row * (G * 4);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int k = 0; k < 8; ++k) {
          consume_values<G>(ring[k % kRing], 4 * k, pw_row, rot_cur, acc);
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            constexpr int kAhead = 4 * kRing;
            const int nrow = 4 * k + r + kAhead;
            if (nrow < 32)
              ring[k % kRing][r] = buf_load16<kAuxStream>(rv_cur, voff_values, static_cast<uint32_t>((nrow + rot_cur) & 31) * 1024u);
            else
              ring[k % kRing][r] = buf_load16<kAuxStream>(rv_nxt, voff_values, static_cast<uint32_t>((nrow - 32 + rot_nxt) & 31) * 1024u);
          }
          __builtin_amdgcn_sched_barrier(0);
        }
        rv_cur = rv_nxt;
        rot_cur = rot_nxt;
      }
      __syncthreads();                                               // buffer (t - 1) % 2 is free again
    }
#pragma unroll
    for (int h = 0; h < G; ++h) {
      float tt[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) tt[e] = sum_rows(acc[h][e]);
      if (row == 0) {
        float4* dst = reinterpret_cast<float4*>(&red_acc[pair][h][col * 8]);
        dst[0] = make_float4(tt[0], tt[1], tt[2], tt[3]);
        dst[1] = make_float4(tt[4], tt[5], tt[6], tt[7]);
      }
    }
  }
  __syncthreads();

  // ---- fold the two pairs into one partial per query head ----
  for (int idx = tid; idx < G * kHeadDim; idx += kRoleThreads) {
    const int h = idx >> 7, dim = idx & (kHeadDim - 1);
    float M = red_ml[0][h][0];
#pragma unroll
    for (int w = 1; w < kPairsOfWaves; ++w) M = fmaxf(M, red_ml[w][h][0]);
    float o = 0.f, l = 0.f;
    if (M > kNegInf) {
#pragma unroll
      for (int w = 0; w < kPairsOfWaves; ++w) {
        const float wgt = __builtin_amdgcn_exp2f(red_ml[w][h][0] - M);
        o = fmaf(wgt, red_acc[w][h][dim], o);
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

}  // namespace
}  // namespace pq
