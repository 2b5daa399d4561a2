// Attention kernel with wavefronts specialised by role (uniform angle grid).
//
// A work-group takes an equal share of the launch's pages (pq_decode_sched.hpp) and works through
// it segment by segment; a segment is a run of pages of one (sequence, KV head).  The four
// wavefronts form two pairs; a pair takes every second page of the segment.  In a pair the SCORE
// wavefront (0 or 1) streams the codes, runs the table-lookup product and the online softmax
// and leaves the page's probabilities and rescaling factor in LDS; the VALUE wavefront (2 or 3)
// streams the value rows and aggregates them with the probabilities of the page the score
// wavefront finished one step earlier.  One work-group barrier per step hands a probability
// buffer over (two buffers per pair).  Each role keeps only its own state in registers, so three
// wavefronts fit a SIMD, and arithmetic-heavy scoring and memory-heavy aggregation overlap
// instead of every wavefront alternating between a phase that waits for memory and one that
// does not touch it.
//
// The score wavefront's lanes are 64 consecutive tokens of the page (PageWalk in
// pq_decode_kernels.hpp, the score-only kernel's walk): all lanes look up the same pair, so the
// table reads have no bank conflicts and the pair's radius parameters sit in scalar registers; a
// lane ends a page with the scores of tokens lane and 64 + lane for all G heads, and a head's
// softmax statistics are wavefront-wide reductions.  The value wavefront's lanes are (token slot,
// 8 dims) as in pq_decode_partials_kernel, whose value steps it shares.
//
// Every wavefront of the work-group executes the same number of barriers: segment list and step
// count are computed from wavefront-uniform values that all four wavefronts derive alike.
#pragma once
#include "pq_decode_sched.hpp"

namespace pq {

// n_wg work-groups; the first shares the launch out evenly and merges in the kernel, the second
// expects n_wg = KV heads x sequences x chunks and leaves the chunks' partials in the workspace.
// Both return false if there is no kernel for ((r, t) = rt / 10, rt % 10; G; v_bits) -- nothing is
// launched then -- and leave launch errors to hipGetLastError().
bool launch_attention_roles(int rt, int G, int v_bits, const DecodeArgs& a, int n_wg, hipStream_t st);
bool launch_attention_roles_grid(int rt, int G, int v_bits, const DecodeArgs& a, int n_wg, hipStream_t st);


namespace {

constexpr int kPairsOfWaves = 2;                   // (score, value) wavefront pairs per work-group
constexpr int kRoleThreads = kPairsOfWaves * 128;
// Resident work-groups per compute unit = wavefronts per SIMD: 3 (168 registers each).
constexpr int role_groups_per_cu(int) { return 3; }

// Pool pages of the pages a wavefront pair handles in a segment (segment pages pair, pair + 2,
// ...): lane k holds the id of the (base + k)-th of them, -1 for a block-table entry outside the
// pool (such a page is masked).  Ids are asked for in increasing order; the window moves on by 64
// when the end is reached.
struct PageIds {
  const int32_t* table;   // block-table row of the sequence, at the segment's first page of this pair
  int64_t n_pool_pages;
  int n_p;                // pages of the pair in this segment
  int base;
  int ids;
  __device__ __forceinline__ void fill(int lane) {
    ids = -1;
    const int k = base + lane;
    if (k < n_p) {
      const int64_t pid = table[kPairsOfWaves * k];
      if (pid >= 0 && pid < n_pool_pages) ids = static_cast<int>(pid);
    }
  }
  __device__ __forceinline__ void start(const int32_t* t, int64_t pool, int n, int lane) {
    table = t;
    n_pool_pages = pool;
    n_p = n;
    base = 0;
    fill(lane);
  }
  // id of the pair's k-th page, -1 if masked or past the pair's last page
  __device__ __forceinline__ int get(int k, int lane) {
    if (k >= n_p) return -1;
    if (k - base >= 64) {
      base += 64;
      fill(lane);
    }
    return __builtin_amdgcn_readlane(ids, k - base);
  }
};

// Issue priority of this wavefront for one step.  The work-groups resident on a compute unit
// started one after the other, and among wavefronts of equal priority the SIMD favours the
// oldest: left alone, the first-started work-group of a compute unit finishes its (equal) share
// 15-18 % earlier than the last-started one, and the launch waits for the slowest.  Rotating the
// priorities from step to step, with the period of the number of work-groups that share the
// compute unit (3 in balanced launches; 1-3 in grid launches, by their size), gives each of them
// the same turn.
__device__ __forceinline__ void rotate_priority(int turn, int period) {
  const int p = period == 3 ? turn % 3 : (period == 2 ? (turn & 1) : 0);
  switch (p) {
    case 0: __builtin_amdgcn_s_setprio(0); break;
    case 1: __builtin_amdgcn_s_setprio(1); break;
    default: __builtin_amdgcn_s_setprio(2); break;
  }
}

// BAL: the launch is shared out evenly and merged in the kernel (pq_decode_sched.hpp); otherwise
// one work-group per (KV head, sequence, chunk) and pq_decode_merge_kernel afterwards.  Two
// kernels rather than a run-time switch: the second one carries none of the first one's code.
// VB: 16 = fp16 values, 4 / 2 = token-wise quantized values (the score wavefront then folds the
// token's scale into its probability, sums the zero-point term and hands fp16 probability pairs
// over; the value wavefront streams the page's units).  The query's type and whether raw scores
// are stored are run-time switches (a.q_is_f32, a.scores): both touch a few instructions per
// page and are not worth kernels of their own.
template <int G, int RB, int TB, int VB, bool BAL>
__global__ __launch_bounds__(kRoleThreads) __attribute__((amdgpu_waves_per_eu(role_groups_per_cu(G), role_groups_per_cu(G))))
void pq_decode_roles_kernel(const DecodeArgs a) {
  constexpr int W = RB + TB;
  constexpr int UB = 2 * W;
  constexpr int NA = 1 << TB;
  constexpr int ROW = NA * 16;
  constexpr int kRing = G == 8 ? 2 : 4;                  // quads of 4 value rows in flight (8 heads: registers for the accumulators)
  constexpr bool kQuantV = VB != 16;
  // 8 query heads: two tables of 4-head entries; a lane of the score wavefront owns heads row and
  // row + 4; probabilities go over as fp16 pairs (tokens n, n + 4) and the value wavefront uses
  // the two-term dot product, which keeps its arithmetic at the level of 4 heads
  constexpr int NH = G == 8 ? 2 : 1;
  constexpr bool kPairP = kQuantV || G == 8;
  static_assert(!(kQuantV && G == 8), "quantized values are served 4 heads at a time");
  constexpr int kVLoads = kQuantV ? kGroup * kHeadDim * VB / 8 / 1024 : 32;   // 1 KB wavefront loads per page of values
  constexpr int kTokPerLoad = kGroup / kVLoads;

  __shared__ __attribute__((aligned(16))) uint8_t lut[NH * kPairs * ROW];
  // probabilities of a page: fp32 [token][G], or fp16 pairs [token pair][G] (quantized values, 8 heads)
  __shared__ __attribute__((aligned(16))) float prob[kPairsOfWaves][2][(kPairP ? kGroup / 2 : kGroup) * G];
  __shared__ __attribute__((aligned(16))) float alpha_s[kPairsOfWaves][2][G == 8 ? 8 : 4];
  // With 8 heads the tables' memory (idle once the last page is scored, rebuilt for the next
  // segment behind a barrier) also serves the end of the segment: the wavefronts' accumulators,
  // then the combination of partials -- a third work-group per compute unit fits that way.
  constexpr int kRedBytes = kPairsOfWaves * G * kHeadDim * 4;
  constexpr bool kLendLut = G == 8 && NH * kPairs * ROW >= kRedBytes + finish_lds_floats(kRoleThreads) * 4;
  __shared__ __attribute__((aligned(16))) float red_own[kLendLut ? 4 : kPairsOfWaves * G * kHeadDim];
  float (*const red_acc)[G][kHeadDim] = reinterpret_cast<float (*)[G][kHeadDim]>(kLendLut ? reinterpret_cast<float*>(lut) : red_own);
  __shared__ float red_ml[kPairsOfWaves][G][3];                       // m, l, sum of p * zero-point
  __shared__ __attribute__((aligned(16))) float q_lds[NH * kHeadDim][4];
  __shared__ float2 trig[kMaxAngleBins];
  __shared__ float res_sc[kGroup * G];

  const int wave = __builtin_amdgcn_readfirstlane(static_cast<int>(threadIdx.x) >> 6);
  const int pair = wave % kPairsOfWaves;      // which share of a segment's pages
  const bool scorer = wave < kPairsOfWaves;   // role of this wavefront
  constexpr uint32_t kCodesBytes = kBlocks * kGroup * UB;
  // start order on a compute unit (work-groups go round the 256 compute units) and how many share one
  const int period = BAL ? 3 : min(3, static_cast<int>((gridDim.x + 255u) / 256u));
  const int tier = BAL ? static_cast<int>(blockIdx.x * 3u / gridDim.x)
                       : static_cast<int>((blockIdx.x / 256u) % static_cast<unsigned>(period));
  WorkSpan span;
  Segment seg;
  bool more;
  if constexpr (BAL) {
    span_begin<G>(a, static_cast<int>(threadIdx.x) & 63, wave == 0, span);
    more = next_segment(a, span, seg);
  } else {
    more = grid_segment(a, seg);
  }
  while (more) {
    // Everything derived from the thread index is derived anew for each segment: what the
    // compiler would otherwise compute once and keep in registers through all segments (table
    // constants of the build loop, addresses of the epilogue) costs more registers than the hot
    // loops leave free.
    int tid = threadIdx.x;
    asm volatile("" : "+v"(tid));
    const int lane = tid & 63;
    const int row = lane >> 4, col = lane & 15;
    const int my_head = (G >= 4) ? row : (G == 2 ? (row >> 1) : 0);   // with 8 heads also my_head + 4
    const bool owner = (G >= 4) || (G == 2 && (row & 1) == 0) || (G == 1 && row == 0);
    const int seq = seg.seq, kvh = seg.kvh, page0 = seg.page0, npg = seg.npg, L = seg.L;
    // pages of this pair: segment pages pair, pair + 2, ...; the step count is the same for both pairs
    const int n_p = npg > pair ? (npg - pair + kPairsOfWaves - 1) / kPairsOfWaves : 0;
    const int n_steps = (npg + kPairsOfWaves - 1) / kPairsOfWaves + 1;   // pair 0's page count, plus one step of skew
    const int res_page = (a.residual != nullptr && (L % kGroup) != 0) ? L / kGroup : -1;
    // the query is fetched first and the page ids next; both are under way together
    const QueryRegs<G> q_regs = fetch_query<G>(a, (static_cast<int64_t>(seq) * a.n_q_heads + kvh * a.group_total + a.head0) * kHeadDim, tid);
    PageIds pids;
    pids.start(a.block_table + static_cast<int64_t>(seq) * a.max_pages_per_seq + page0 + pair, a.n_pool_pages, n_p, lane);

    if (scorer) {
      // ================ SCORE wavefront: lanes = tokens (PageWalk) ================
      // The lanes are 64 consecutive tokens of a page and walk the pairs together: table reads
      // without bank conflicts, radius parameters in scalar registers.  A lane ends a page with
      // the scores of tokens lane and 64 + lane for all G heads; the softmax statistics of a
      // head are wavefront-wide reductions and therefore uniform.  Probabilities go to LDS in
      // the same layouts as below, so the value wavefront does not know the difference.
      constexpr int kPipe = G == 8 ? 3 : 4;                          // table reads in flight (8 heads: two reads per step)
      PageWalk<G, RB, TB, kPipe> w;
      w.voff_codes = lane * UB;
      w.lut_base = lds_addr(lut);
      LaneSoftmax<G, VB> sm;
      sm.reset();
      auto page_setup = [&](int k, __amdgpu_buffer_rsrc_t& rc, const uint32_t*& pp, __amdgpu_buffer_rsrc_t& rvp, int& nv) {
        const int pid = pids.get(k, lane);
        const bool ok = pid >= 0;
        const int64_t ph = (ok ? static_cast<int64_t>(pid) : 0) * a.n_kv_heads + kvh;
        nv = ok ? min(kGroup, L - (page0 + pair + kPairsOfWaves * k) * kGroup) : 0;
        const bool packed = ok && (page0 + pair + kPairsOfWaves * k) != res_page;
        rc = make_rsrc(a.codes + ph * kCodesBytes, packed ? kCodesBytes : 0u);
        pp = a.params + ph * kPairs;                     // valid memory also for a masked page (pool page 0, unused)
        if constexpr (kQuantV) rvp = make_rsrc(a.v_params + ph * kGroup, static_cast<uint32_t>(nv) * 4u);
        else rvp = rc;
      };
      __amdgpu_buffer_rsrc_t rc_cur, rvp_cur, rc_nxt, rvp_nxt;
      const uint32_t* pp_cur;
      const uint32_t* pp_nxt;
      int nv_cur, nv_nxt;
      page_setup(0, rc_cur, pp_cur, rvp_cur, nv_cur);
      uint32_t vpar[2];                                              // quantized values: (scale, zero) of tokens lane, 64 + lane
#pragma unroll
      for (int b = 0; b < kBlocks; ++b) w.par[b] = load_block_params(pp_cur, b);
      if constexpr (kQuantV) {
#pragma unroll
        for (int half = 0; half < 2; ++half) vpar[half] = buf_load4<kAuxCached>(rvp_cur, lane * 4, half * 256);
      }
#pragma unroll
      for (int b = 0; b < kBlocks; ++b)
#pragma unroll
        for (int half = 0; half < 2; ++half) w.cu[half * kBlocks + b] = load_unit<W>(rc_cur, w.voff_codes, w.unit_at(half, b));

      store_query_lds<G>(q_lds, trig, q_regs, tid);
      __syncthreads();
#pragma unroll
      for (int i = 0; i < NH; ++i) build_uniform_table<TB>(lut + i * (kPairs * ROW), q_lds + i * kHeadDim, trig, tid, kRoleThreads);
      __syncthreads();

      // residual group (plain dot products, in the lane layout of the other score path), if this pair owns its page
      if (res_page >= page0 + pair && res_page < page0 + npg && ((res_page - page0 - pair) % kPairsOfWaves) == 0) {
        residual_scores<G>(a.residual + (static_cast<int64_t>(seq) * a.n_kv_heads + kvh) * (kGroup * kHeadDim),
                           L - res_page * kGroup, lds_addr(q_lds), row, col, [&](int s, Folded<G> v) {
#pragma unroll
                             for (int i = 0; i < NH; ++i)
                               if (owner) res_sc[(s * 16 + col) * G + my_head + 4 * i] = v.v[i];
                           });
        wave_lds_sync();
      }

      for (int t = 0; t < n_steps; ++t) {
        rotate_priority(tier + t, period);
        if (t < n_p) {
          const int pi = page0 + pair + kPairsOfWaves * t;
          page_setup(t + 1, rc_nxt, pp_nxt, rvp_nxt, nv_nxt);
          w.run(rc_nxt, pp_nxt);
          float* const out_rows = a.scores == nullptr ? nullptr
              : a.scores + (static_cast<int64_t>(seq) * a.n_q_heads + kvh * a.group_total + a.head0) * a.scores_stride +
                    static_cast<int64_t>(pi) * kGroup;
          sm.page(w.score, nv_cur, a.scale_log2, vpar, pi == res_page, lds_addr(res_sc), out_rows, a.scores_stride,
                  lds_addr(prob[pair][t & 1]), alpha_s[pair][t & 1], lane);
          if constexpr (kQuantV) {
#pragma unroll
            for (int half = 0; half < 2; ++half) vpar[half] = buf_load4<kAuxCached>(rvp_nxt, lane * 4, half * 256);
          }
          rc_cur = rc_nxt; pp_cur = pp_nxt; rvp_cur = rvp_nxt; nv_cur = nv_nxt;
        }
        __syncthreads();                                               // hand buffer t % 2 to the value wavefront
      }
      sm.finish(red_ml[pair], lane);
    } else {
      // =========================== VALUE wavefront ===========================
      const uint32_t voff_values = kQuantV ? lane * 16 : row * (kHeadDim * 2) + col * 16;
      float acc[G][8];
#pragma unroll
      for (int h = 0; h < G; ++h)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[h][e] = 0.f;

      auto page_setup = [&](int k, __amdgpu_buffer_rsrc_t& rv, int& rot) {
        const int pid = pids.get(k, lane);
        const bool ok = pid >= 0;
        const int64_t ph = ok ? static_cast<int64_t>(pid) * a.n_kv_heads + kvh : 0;
        const int nv = ok ? min(kGroup, L - (page0 + pair + kPairsOfWaves * k) * kGroup) : 0;
        rot = ok ? (pid * 13 + kvh * 5) & (G == 8 ? 30 : 31) : 0;   // even with 8 heads: loads 2m, 2m + 1 stay a token pair
        if constexpr (kQuantV) {
          // whole units are read; codes of slots past the sequence end are zero bytes and meet a
          // zero probability
          rv = make_rsrc(reinterpret_cast<const uint8_t*>(a.values) + ph * (kGroup * kHeadDim * VB / 8),
                         nv > 0 ? kGroup * kHeadDim * VB / 8 : 0u);
        } else {
          rv = make_rsrc(a.values + ph * (kGroup * kHeadDim), static_cast<uint32_t>(nv) * (kHeadDim * 2));
        }
      };
      __amdgpu_buffer_rsrc_t rv_cur, rv_nxt;
      int rot_cur, rot_nxt;
      page_setup(0, rv_cur, rot_cur);
      uint4 ring[kQuantV ? 1 : kRing][4];                            // fp16 values: rows in flight
      uint4 vq[kQuantV ? kVLoads : 1];                               // quantized values: the page's units
      if constexpr (kQuantV) {
#pragma unroll
        for (int k = 0; k < kVLoads; ++k) vq[k] = buf_load16<kAuxStream>(rv_cur, voff_values, k * 1024);
      } else {
#pragma unroll
        for (int k = 0; k < kRing; ++k)
#pragma unroll
          for (int r = 0; r < 4; ++r)
            ring[k][r] = buf_load16<kAuxStream>(rv_cur, voff_values, static_cast<uint32_t>((4 * k + r + rot_cur) & 31) * 1024u);
      }

      store_query_lds<G>(q_lds, trig, q_regs, tid);
      __syncthreads();
#pragma unroll
      for (int i = 0; i < NH; ++i) build_uniform_table<TB>(lut + i * (kPairs * ROW), q_lds + i * kHeadDim, trig, tid, kRoleThreads);
      __syncthreads();

      for (int t = 0; t < n_steps; ++t) {
        rotate_priority(tier + t, period);
        const int j = t - 1;                                           // the page the score wavefront finished last step
        if (j >= 0 && j < n_p) {
          page_setup(j + 1, rv_nxt, rot_nxt);
          {
            const Heads<(G == 8 ? 8 : 4)> al = lut_read<(G == 8 ? 8 : 4), 16>(lds_addr(alpha_s[pair][j & 1]));
#pragma unroll
            for (int h = 0; h < G; ++h)
#pragma unroll
              for (int e = 0; e < 8; ++e) acc[h][e] *= al.v[h];
          }
          // all loads in flight have arrived before the page is taken up: the wavefront then issues its
          // refills in a burst, row after row of one page (measured 2 % faster than waking up for every row)
          asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
          __builtin_amdgcn_sched_barrier(0);
          if constexpr (kQuantV) {
            // unit k of the page = tokens kTokPerLoad * k + (16 / VB) * row ..; refilled with the next page's unit k
            const uint32_t pp = lds_addr(prob[pair][j & 1]) + (((16 / VB) * row) >> 1) * (G * 4);
#pragma unroll
            for (int k = 0; k < kVLoads; ++k) {
              consume_quantized<G, VB>(vq[k], pp + ((kTokPerLoad * k) >> 1) * (G * 4), acc);
              vq[k] = buf_load16<kAuxStream>(rv_nxt, voff_values, k * 1024);
              __builtin_amdgcn_sched_barrier(0);
            }
          } else {
            const uint32_t pw_row = lds_addr(prob[pair][j & 1]) + row * (G * 4);
#pragma unroll
            for (int k = 0; k < 8; ++k) {
              if constexpr (G == 8) consume_values_pairs(ring[k % kRing], 4 * k, lds_addr(prob[pair][j & 1]), rot_cur, row, acc);
              else consume_values<G>(ring[k % kRing], 4 * k, pw_row, rot_cur, acc);
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
        for (int e = 0; e < 8; ++e) {
          tt[e] = sum_rows(acc[h][e]);
          if constexpr (kQuantV) tt[e] *= vq_unscale<VB>(e);
        }
        if (row == 0) {
          float4* dst = reinterpret_cast<float4*>(&red_acc[pair][h][col * 8]);
          dst[0] = make_float4(tt[0], tt[1], tt[2], tt[3]);
          dst[1] = make_float4(tt[4], tt[5], tt[6], tt[7]);
        }
      }
    }
    __syncthreads();

    // ---- the two pairs' results become the segment's partial; finish (or merge) the unit ----
    finish_segment<G, kRoleThreads, BAL, kLendLut>(a, seg, tid, [&](int h, int quad, float& M, float& l) {
      M = fmaxf(red_ml[0][h][0], red_ml[1][h][0]);
      f32x4 o = {0.f, 0.f, 0.f, 0.f};
      l = 0.f;
      if (M > kNegInf) {
#pragma unroll
        for (int w = 0; w < kPairsOfWaves; ++w) {
          const float wgt = __builtin_amdgcn_exp2f(red_ml[w][h][0] - M);
          const f32x4 v = *reinterpret_cast<const f32x4*>(&red_acc[w][h][quad * 4]);
          const float zp = red_ml[w][h][2];                              // zero-point term: the same for every dim
          o.x = fmaf(wgt, v.x + zp, o.x);
          o.y = fmaf(wgt, v.y + zp, o.y);
          o.z = fmaf(wgt, v.z + zp, o.z);
          o.w = fmaf(wgt, v.w + zp, o.w);
          l = fmaf(wgt, red_ml[w][h][1], l);
        }
      }
      return o;
    }, kLendLut ? reinterpret_cast<float*>(lut + kRedBytes) : nullptr);
    if constexpr (BAL) more = next_segment(a, span, seg);
    else more = false;
  }
}

}  // namespace
}  // namespace pq
