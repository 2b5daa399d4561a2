// Internal declarations shared by the host-side entry points of libpolarquant.
// Nothing here is part of the public ABI (that is include/polarquant.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "polarquant.h"

namespace pq {

constexpr int kHeadDim = 128;          // d
constexpr int kPairs = kHeadDim / 2;   // P: pair j = dims (j, j + 64)
constexpr int kGroup = 128;            // g: tokens per page / quantization group
constexpr int kPairsPerUnit = 16;      // one packed unit = 16 pairs of one token
constexpr int kBlocks = kPairs / kPairsPerUnit;
constexpr int kMaxAngleBins = 32;      // t <= 5

// Remembers the hipError_t of a failed call for pq_last_hip_error().
int record_hip_error(hipError_t e);

// True when this build has kernels for the layout.
bool layout_supported(const pq_layout* l);

// How the context of a sequence is cut into chunks of pages; one work-group
// handles one (sequence, KV head, chunk).  Pure function of the launch shape so
// that the workspace size and both decode stages agree.
struct ChunkPlan {
  int32_t pages_per_chunk;
  int32_t n_chunks;   // per sequence, for max_seq_len
};
ChunkPlan plan_chunks(int32_t n_seqs, int32_t n_kv_heads, int32_t max_seq_len);

}  // namespace pq
