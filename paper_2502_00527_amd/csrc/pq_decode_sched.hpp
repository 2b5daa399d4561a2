// How a decode launch is shared out among its work-groups, and how the pieces of one
// (sequence, KV head) are put together again -- all inside the attention kernel.
//
// Work is counted in pages.  A "unit" is one (sequence, KV head); the units are laid end to end
// in the order (sequence, KV head, page), and work-group b of the launch takes positions
// [b * per, (b + 1) * per) of that line, per = ceil(total pages / work-groups): every work-group
// streams the same number of pages whatever the mix of sequence lengths, nothing is left for a
// second round, and no work-group is launched for pages that do not exist.  A work-group's
// share may end inside a unit and go on into the next ones, so it handles a few "segments", each
// a run of consecutive pages of one unit, one after the other.
//
// A unit that lies in one work-group's share is finished there.  Otherwise every segment leaves
// its softmax partial (running maximum, denominator, un-normalised output) in a workspace slot and
// registers at the unit's arrival word; whoever registers last reads all slots of the unit, in
// slot order (so the result does not depend on who that was), and writes the output row.  Nobody
// waits for anybody: a work-group that is not last simply goes on.
//
// The arrival word needs no initialisation by the caller: it holds (mark, count), and a word
// without the mark -- memory the library has not used as an arrival word before -- is first made
// (mark, 0).  The last arriver puts the count back to zero, so a word that carries the mark
// always starts a launch at zero.
#pragma once
#include "pq_decode_kernels.hpp"

namespace pq {
namespace {

struct Segment {
  int seq, kvh;        // the unit
  int page0, npg;      // pages [page0, page0 + npg) of the sequence
  int L;               // the sequence's length (clamped to max_seq_len)
  int first_wg;        // the unit's pages are shared by work-groups first_wg .. first_wg + n_segs - 1
  int n_segs;
};

struct WorkSpan {
  int f, f1;           // next position of the line to hand out, end of this work-group's share
  int per;             // positions per work-group, on average
  int per_even;        // positions of an even-numbered work-group (the odd one after it takes 2 per - per_even)
  int seq, kvh, pos;   // where position f lies: unit and position inside it (overhead positions first)
  int n_pages;         // pages of sequence `seq`
  int L;
};

// A value every lane holds alike, moved to a scalar register (the compiler keeps the results of
// shuffles and integer divisions in vector registers otherwise, one per lane for nothing).
__device__ __forceinline__ int uni(int x) { return __builtin_amdgcn_readfirstlane(x); }

__device__ __forceinline__ int clamped_len(const DecodeArgs& a, int s) {
  return min(a.seq_lens[s], a.max_seq_len);
}
__device__ __forceinline__ int pages_of_len(int L) { return L > 0 ? (L + kGroup - 1) / kGroup : 0; }

__device__ __forceinline__ int wave_sum(int x) {
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) x += __shfl_xor(x, d);
  return x;
}
__device__ __forceinline__ int wave_inclusive_scan(int x, int lane) {
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const int y = __shfl_up(x, d);
    if (lane >= d) x += y;
  }
  return x;
}

// The share of work-group blockIdx.x.  Every wavefront calls this and gets the same answer (all
// values are wavefront-uniform).  The wavefront called with `zero_duty` also writes the all-zero
// output rows of the empty sequences s with s % gridDim.x == blockIdx.x (G query heads from
// a.head0 on, of every KV head): those sequences have no pages and nobody else visits them.
//
// On the line a unit takes a.unit_cost positions more than it has pages, in front of its pages:
// starting on a unit (table build, pipeline fill, an extra partial to merge) costs a work-group
// about as much as streaming that many pages, and a share that crosses into another unit pays it
// a second time -- counted this way, shares are equal in time rather than in pages.
template <int G>
__device__ __forceinline__ void span_begin(const DecodeArgs& a, int lane, bool zero_duty, WorkSpan& w) {
  const int n_wg = static_cast<int>(gridDim.x), wg = static_cast<int>(blockIdx.x);
  const int c = a.unit_cost;
  int mine = 0;
  for (int base = 0; base < a.n_seqs; base += 64) {
    const int s = base + lane;
    const int p = s < a.n_seqs ? pages_of_len(clamped_len(a, s)) : -1;
    mine += p > 0 ? p + c : 0;
    if (zero_duty) {
      uint64_t empty = __ballot(p == 0 && (s % n_wg) == wg);
      while (empty) {
        const int e = base + __builtin_ctzll(empty);
        empty &= empty - 1;
        for (int r = 0; r < a.n_kv_heads * G; ++r) {
          const int64_t head = static_cast<int64_t>(e) * a.n_q_heads + (r / G) * a.group_total + a.head0 + (r % G);
          a.out[head * kHeadDim + lane] = 0.f;
          a.out[head * kHeadDim + 64 + lane] = 0.f;
        }
      }
    }
  }
  const int total = uni(wave_sum(mine)) * a.n_kv_heads;
  w.per = uni(max(a.min_pages + c, (total + n_wg - 1) / n_wg));
  // Work-groups go round the XCDs in launch order, and with the memory system saturated the
  // odd-numbered XCDs of an MI355X stream 7-10 % slower than the even-numbered ones (measured
  // with time stamps per work-group, on every machine tried): of each pair of consecutive
  // work-groups the even one takes the larger part, so that the two finish together.
  int skew = (n_wg & 1) == 0 ? (w.per * a.xcd_skew_permille + 500) / 1000 : 0;
  skew = max(0, min(skew, w.per - (a.min_pages + c)));
  w.per_even = uni(w.per + skew);
  const int64_t f0 = static_cast<int64_t>(wg >> 1) * (2 * w.per) + ((wg & 1) ? w.per_even : 0);
  w.f1 = uni(static_cast<int>(min<int64_t>(total, f0 + ((wg & 1) ? 2 * w.per - w.per_even : w.per_even))));
  w.f = uni(static_cast<int>(min<int64_t>(total, f0)));
  w.seq = w.kvh = w.pos = w.n_pages = w.L = 0;
  if (w.f >= w.f1) return;
  // the sequence that position f lies in: positions before it (all KV heads) <= f < positions up to and with it
  int carry = 0;
  for (int base = 0; base < a.n_seqs; base += 64) {
    const int s = base + lane;
    const int L = s < a.n_seqs ? clamped_len(a, s) : 0;
    const int p = pages_of_len(L);
    const int len = p > 0 ? p + c : 0;
    const int incl = wave_inclusive_scan(len, lane);
    const int before = (carry + incl - len) * a.n_kv_heads;
    const uint64_t hit = __ballot(p > 0 && before <= w.f && w.f < before + len * a.n_kv_heads);
    if (hit) {
      const int src = __builtin_ctzll(hit);
      w.seq = uni(base + src);
      w.L = uni(__shfl(L, src));
      w.n_pages = uni(__shfl(p, src));
      const int rel = uni(w.f - __shfl(before, src));
      w.kvh = uni(rel / (w.n_pages + c));
      w.pos = rel - w.kvh * (w.n_pages + c);
      return;
    }
    carry += uni(__shfl(incl, 63));
  }
  w.f1 = w.f;   // not reached: position f < total always lies in some sequence
}

// The work-group whose share holds position x of the line.
__device__ __forceinline__ int share_of(const WorkSpan& w, int x) {
  const int two = 2 * w.per;
  const int pair = x / two;
  return 2 * pair + (x - pair * two >= w.per_even ? 1 : 0);
}

// Next segment of the share; false when the share is used up.
__device__ __forceinline__ bool next_segment(const DecodeArgs& a, WorkSpan& w, Segment& seg) {
  const int c = a.unit_cost;
  while (w.f < w.f1) {
    if (w.pos < c) {                       // overhead positions of the unit: nothing to do for them
      const int skip = min(c - w.pos, w.f1 - w.f);
      w.f += skip;
      w.pos += skip;
      if (w.f >= w.f1) return false;
    }
    seg.seq = w.seq;
    seg.kvh = w.kvh;
    seg.page0 = w.pos - c;
    seg.L = w.L;
    seg.npg = min(w.n_pages - seg.page0, w.f1 - w.f);
    const int first_page_at = w.f - seg.page0;     // position of the unit's page 0
    seg.first_wg = uni(share_of(w, first_page_at));
    seg.n_segs = uni(share_of(w, first_page_at + w.n_pages - 1)) - seg.first_wg + 1;
    w.f += seg.npg;
    w.pos += seg.npg;
    if (w.pos == c + w.n_pages && w.f < w.f1) {
      w.pos = 0;
      if (++w.kvh == a.n_kv_heads) {
        w.kvh = 0;
        do {   // f < f1 <= total: a later sequence with pages exists
          ++w.seq;
          w.L = w.seq < a.n_seqs ? uni(clamped_len(a, w.seq)) : 0;
          w.n_pages = pages_of_len(w.L);
        } while (w.n_pages == 0 && w.seq < a.n_seqs);
        if (w.seq >= a.n_seqs) w.f1 = w.f;
      }
    }
    return true;
  }
  return false;
}

// The other way to share a launch out, for launches of few units (one long sequence): one
// work-group per (KV head, sequence, chunk of a.pages_per_chunk pages), chunk-major, more
// work-groups than are resident at once so that the hardware hands them out as others finish.
// There a unit is shared by ~100 work-groups that all finish together, and combining them in the
// kernel is a chain of dependent round trips everybody waits out; the chunks' partials go to the
// workspace instead and pq_decode_merge_kernel follows.  seg.first_wg carries the chunk index.
__device__ __forceinline__ bool grid_segment(const DecodeArgs& a, Segment& seg) {
  const int id = static_cast<int>(blockIdx.x);
  seg.kvh = id % a.n_kv_heads;
  seg.seq = (id / a.n_kv_heads) % a.n_seqs;
  const int chunk = id / (a.n_kv_heads * a.n_seqs);
  seg.L = uni(clamped_len(a, seg.seq));
  const int n_pages = pages_of_len(seg.L);
  seg.page0 = chunk * a.pages_per_chunk;
  seg.npg = min(a.pages_per_chunk, n_pages - seg.page0);
  seg.first_wg = chunk;
  seg.n_segs = 0;
  return seg.npg > 0;
}

// All memory operations this wavefront has issued are complete (for device-coherent stores:
// performed at memory, where every other work-group's device-coherent loads will find them).
__device__ __forceinline__ void stores_done() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// Registers one arrival at a word; true for the arrival that completes `n`.  One atomic add in
// the normal case.  If the value it returns does not carry the mark, the word was never an
// arrival word (fresh memory, or memory that held partials of a launch of another shape): it is
// replaced by (mark, 0) -- one compare-and-swap wins, whatever the other arrivals have added to
// the old value meanwhile -- and every arrival that saw the unmarked word registers again.
constexpr uint64_t kArrivalMark = 0x7ff5c0dea11dull << 16;   // 48 bits above the 16-bit count
__device__ __forceinline__ bool arrive(uint64_t* word, int n) {
  unsigned long long* p = reinterpret_cast<unsigned long long*>(word);
  unsigned long long before = atomicAdd(p, 1ull);
  if ((before & ~0xffffull) != kArrivalMark) {
    unsigned long long cur = before + 1ull;
    while ((cur & ~0xffffull) != kArrivalMark) {
      const unsigned long long prev = atomicCAS(p, cur, kArrivalMark);
      if (prev == cur) break;
      cur = prev;
    }
    before = atomicAdd(p, 1ull);
  }
  return static_cast<int>(before & 0xffffull) + 1 == n;
}

// Puts a word's count back to zero (the last arriver, when nobody else will touch the word again).
__device__ __forceinline__ void reset_arrivals(uint64_t* word) {
  __hip_atomic_store(reinterpret_cast<unsigned long long*>(word), kArrivalMark, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

constexpr int kArriveFan = 16;

// Combines `count` partials, `stride` slots apart from slot `first` on, of the G query heads this
// launch serves: afterwards the threads of slice 0 of each head (thread = (head, slice, 4 dims))
// hold the un-normalised output r, the maximum M and the denominator lt.  All NT threads call it;
// part_o[NT], part_l[NT], wave_max[NT / 64] are LDS.  Loads are device-coherent (see finish_segment).
template <int G, int NT>
__device__ __forceinline__ void combine_partials(const DecodeArgs& a, int64_t first, int stride, int count, int tid,
                                                 f32x4* part_o, float* part_l, float* wave_max, f32x4& r, float& M,
                                                 float& lt) {
  constexpr int TPH = NT / G;            // threads per query head
  constexpr int kSlices = TPH / 32;      // each takes every kSlices-th partial; 32 threads x 4 dims per slice
  const int h = tid / TPH, j = tid % TPH, slice = j >> 5, quad = j & 31;
  const uint32_t slot_ml = a.group_total * 8, slot_acc = a.group_total * (kHeadDim * 4);   // bytes from slot to slot
  const uint32_t span_slots = static_cast<uint32_t>((count - 1) * stride + 1);
  const __amdgpu_buffer_rsrc_t r_acc = make_rsrc(a.ws_acc + (first * a.group_total + a.head0) * kHeadDim, span_slots * slot_acc);
  const __amdgpu_buffer_rsrc_t r_ml = make_rsrc(a.ws_ml + (first * a.group_total + a.head0) * 2, span_slots * slot_ml);
  float m = kNegInf;
  for (int k = j; k < count; k += TPH)
    m = fmaxf(m, u2f(__builtin_amdgcn_raw_buffer_load_b32(r_ml, k * stride * slot_ml + h * 8, 0, kAuxDevice)));
  // maximum over the head's TPH threads: within the wavefront by shuffles, beyond it through LDS
#pragma unroll
  for (int d = (TPH < 64 ? TPH : 64) / 2; d >= 1; d >>= 1) m = fmaxf(m, __shfl_xor(m, d));
  if ((tid & 63) == 0) wave_max[tid >> 6] = m;
  __syncthreads();
  M = m;
  if constexpr (TPH > 64) {
    M = kNegInf;
#pragma unroll
    for (int w = 0; w < TPH / 64; ++w) M = fmaxf(M, wave_max[h * (TPH / 64) + w]);
  }
  f32x4 o = {0.f, 0.f, 0.f, 0.f};
  float l = 0.f;
  if (M > kNegInf) {
#pragma unroll 8
    for (int k = slice; k < count; k += kSlices) {
      const u32x2 ml = __builtin_amdgcn_raw_buffer_load_b64(r_ml, k * stride * slot_ml + h * 8, 0, kAuxDevice);
      const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(r_acc, k * stride * slot_acc + h * (kHeadDim * 4) + quad * 16, 0, kAuxDevice);
      const float wgt = __builtin_amdgcn_exp2f(u2f(ml.x) - M);
      o.x = fmaf(wgt, u2f(v.x), o.x);
      o.y = fmaf(wgt, u2f(v.y), o.y);
      o.z = fmaf(wgt, u2f(v.z), o.z);
      o.w = fmaf(wgt, u2f(v.w), o.w);
      l = fmaf(wgt, u2f(ml.y), l);
    }
  }
  part_o[tid] = o;
  part_l[tid] = l;
  __syncthreads();
  r = f32x4{0.f, 0.f, 0.f, 0.f};
  lt = 0.f;
  if (slice == 0) {
#pragma unroll
    for (int s2 = 0; s2 < kSlices; ++s2) {
      const f32x4 t = part_o[h * TPH + s2 * 32 + quad];
      r.x += t.x; r.y += t.y; r.z += t.z; r.w += t.w;
      lt += part_l[h * TPH + s2 * 32 + quad];
    }
  }
}

// End of a segment.  `partial(h, quad, M, l)` returns the segment's un-normalised output for
// query head h (of the G this launch serves) and dimensions 4 quad .. 4 quad + 3, and sets the
// head's running maximum M (log2 units) and denominator l.  All NT threads of the work-group call
// this.  Writes a.out directly when the unit has one segment, else as described at the top.
//
// Partials travel between work-groups that may sit on different XCDs, each with an L2 of its own.
// They are written and read with device-coherent accesses (cache policy sc1: performed past the
// L2s) and ordered by waiting for the stores before the arrival is registered -- not by fences,
// which write back and invalidate whole caches (measured: with fences in every work-group the
// launch takes twice as long).
template <int G, int NT, bool OWN_LDS, typename Partial>
__device__ __forceinline__ void finish_balanced(const DecodeArgs& a, const Segment& seg, int tid, Partial partial,
                                                float* lent);

// LDS the combination of partials needs (floats): NT 4-float accumulators, NT denominators, one
// maximum per wavefront.  A kernel may lend memory that is idle at the end of a segment
// (`lent`, 16-byte aligned); otherwise the function has arrays of its own.
constexpr int finish_lds_floats(int NT) { return NT * 4 + NT + NT / 64; }

template <int G, int NT, bool BAL, bool LENT = false, typename Partial>
__device__ __forceinline__ void finish_segment(const DecodeArgs& a, const Segment& seg, int tid, Partial partial,
                                               float* lent = nullptr) {
  static_assert(NT == 256 && (G == 1 || G == 2 || G == 4 || G == 8), "thread mapping of the merge");
  if constexpr (!BAL) {
    // one work-group per (sequence, KV head, chunk): the partial goes to the chunk's slot and
    // pq_decode_merge_kernel, launched next, combines the chunks
    if (tid < G * 32) {
      const int h = tid >> 5, quad = tid & 31;
      float M, l;
      const f32x4 o = partial(h, quad, M, l);
      const int64_t sh = (static_cast<int64_t>(seg.seq) * a.n_q_heads + seg.kvh * a.group_total + a.head0 + h) * a.n_chunks + seg.first_wg;
      reinterpret_cast<float4*>(a.ws_acc + sh * kHeadDim)[quad] = make_float4(o.x, o.y, o.z, o.w);
      if (quad == 0) {
        a.ws_ml[sh * 2] = M;
        a.ws_ml[sh * 2 + 1] = l;
      }
    }
    return;
  } else {
    finish_balanced<G, NT, !LENT>(a, seg, tid, partial, lent);
  }
}

template <int G, int NT, bool OWN_LDS, typename Partial>
__device__ __forceinline__ void finish_balanced(const DecodeArgs& a, const Segment& seg, int tid, Partial partial,
                                                float* lent) {
  constexpr int TPH = NT / G;            // threads per query head in the merge
  constexpr int kSlices = TPH / 32;      // each takes every kSlices-th segment; 32 threads x 4 dims per slice
  __shared__ __attribute__((aligned(16))) float own[OWN_LDS ? finish_lds_floats(NT) : 4];
  float* const mem = OWN_LDS ? own : lent;
  f32x4* const part_o = reinterpret_cast<f32x4*>(mem);
  float* const part_l = mem + NT * 4;
  float* const wave_max = mem + NT * 5;
  __shared__ int stage;                  // after an arrival: 0 not last, 1 last at the unit's word, 2 last of a block

  const int unit = seg.seq * a.n_kv_heads + seg.kvh;
  float* const out_rows = a.out + (static_cast<int64_t>(seg.seq) * a.n_q_heads + seg.kvh * a.group_total + a.head0) * kHeadDim;
  if (seg.n_segs == 1) {
    if (tid < G * 32) {
      float M, l;
      const f32x4 o = partial(tid >> 5, tid & 31, M, l);
      const float inv = l > 0.f ? 1.f / l : 0.f;
      reinterpret_cast<float4*>(out_rows)[tid] = make_float4(o.x * inv, o.y * inv, o.z * inv, o.w * inv);
    }
    return;
  }
  // slot of (work-group b, unit u) = b + u: distinct for all segments of a launch, below
  // gridDim.x + number of units; a unit's segments have consecutive slots
  const int64_t slot = static_cast<int64_t>(blockIdx.x) + unit;
  if (tid < G * 32) {
    const int h = tid >> 5, quad = tid & 31;
    float M, l;
    const f32x4 o = partial(h, quad, M, l);
    const __amdgpu_buffer_rsrc_t r_acc = make_rsrc(a.ws_acc + (slot * a.group_total + a.head0) * kHeadDim, G * kHeadDim * 4);
    __builtin_amdgcn_raw_buffer_store_b128(u32x4{f2u(o.x), f2u(o.y), f2u(o.z), f2u(o.w)}, r_acc, tid * 16, 0, kAuxDevice);
    if (quad == 0) {
      const __amdgpu_buffer_rsrc_t r_ml = make_rsrc(a.ws_ml + (slot * a.group_total + a.head0) * 2, G * 8);
      __builtin_amdgcn_raw_buffer_store_b64(u32x2{f2u(M), f2u(l)}, r_ml, h * 8, 0, kAuxDevice);
    }
  }
  stores_done();                        // the partial has reached memory before the arrival is registered
  __syncthreads();

  // Arrivals at one word are taken one after the other by the memory system, and whoever combines
  // n partials waits for n loads in a row.  A unit shared by more than kArriveFan work-groups
  // (one long sequence: ~100) is therefore handled in blocks of kArriveFan segments: each block
  // has an arrival word of its own (the word of its first slot), its last arriver combines the
  // block into one partial (left in the block's first slot) and goes on to the unit's word, where
  // the last block to arrive combines the blocks.  Always in slot order: the result does not
  // depend on who arrived when.
  const int n = seg.n_segs;
  const int64_t slot0 = static_cast<int64_t>(seg.first_wg) + unit;
  uint64_t* const root = a.arrivals + unit;
  const bool two_levels = n > kArriveFan;
  const int n_blocks = (n + kArriveFan - 1) / kArriveFan;
  const int blk = (static_cast<int>(blockIdx.x) - seg.first_wg) / kArriveFan;
  const int in_blk = min(kArriveFan, n - blk * kArriveFan);
  uint64_t* const leaf = a.arrivals + static_cast<int64_t>(a.n_seqs) * a.n_kv_heads + slot0 + blk * kArriveFan;
  if (tid == 0) {
    if (two_levels) stage = arrive(leaf, in_blk) ? 2 : 0;
    else stage = arrive(root, n) ? 1 : 0;
  }
  __syncthreads();
  if (stage == 0) return;

  const int h = tid / TPH, slice = (tid % TPH) >> 5, quad = tid & 31;
  f32x4 r;
  float M, lt;
  auto combine = [&](int64_t first, int stride, int count) {
    combine_partials<G, NT>(a, first, stride, count, tid, part_o, part_l, wave_max, r, M, lt);
  };

  if (stage == 2) {
    // last of its block: the block's partials become one, in the block's first slot
    const int64_t first = slot0 + blk * kArriveFan;
    combine(first, 1, in_blk);
    if (slice == 0) {
      const __amdgpu_buffer_rsrc_t r_acc = make_rsrc(a.ws_acc + (first * a.group_total + a.head0) * kHeadDim, G * kHeadDim * 4);
      __builtin_amdgcn_raw_buffer_store_b128(u32x4{f2u(r.x), f2u(r.y), f2u(r.z), f2u(r.w)}, r_acc, (h * 32 + quad) * 16, 0, kAuxDevice);
      if (quad == 0) {
        const __amdgpu_buffer_rsrc_t r_ml = make_rsrc(a.ws_ml + (first * a.group_total + a.head0) * 2, G * 8);
        __builtin_amdgcn_raw_buffer_store_b64(u32x2{f2u(M), f2u(lt)}, r_ml, h * 8, 0, kAuxDevice);
      }
    }
    stores_done();
    __syncthreads();
    if (tid == 0) {
      reset_arrivals(leaf);
      stage = arrive(root, n_blocks) ? 1 : 0;
    }
    __syncthreads();
    if (stage == 0) return;
  }

  // last to arrive at the unit's word: combine segments (or blocks) and write the output row
  if (two_levels) combine(slot0, kArriveFan, n_blocks);
  else combine(slot0, 1, n);
  if (slice == 0) {
    const float inv = lt > 0.f ? 1.f / lt : 0.f;
    reinterpret_cast<float4*>(out_rows)[h * 32 + quad] = make_float4(r.x * inv, r.y * inv, r.z * inv, r.w * inv);
  }
  if (tid == 0) reset_arrivals(root);
}

}  // namespace
}  // namespace pq
