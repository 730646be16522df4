// Shared by the vote selection's sources: the streaming score + per-head top-k scan on the vector ALU
// (vote_scan.hip) and its callers (vote.hip).
#pragma once

#include "common.hpp"

namespace reattn {

constexpr int kVoteThreads = 1024;
constexpr int kVoteWaves = kVoteThreads / 64;
// Paged caches: a slice of at most 16,384 rows spans at most 257 pages of 64 tokens or more (+ the spare entry);
// a multiple of 16 bytes, so that the dynamic LDS behind it keeps its 16-byte alignment (128-bit LDS accesses).
constexpr int kVotePages = 16384 / 64 + 4;
static_assert(kVotePages * sizeof(int32_t) % 16 == 0, "keeps the staging tiles 16-byte aligned");

struct HeadScanArgs {
  const void* k; const void* q;
  uint64_t* part;          // [rows = n_query * Hq][n_wg][KT] composites, best first
  int64_t ksh, kst, n_mid, first_tok;
  int Hq, Hkv, G, rows_per_block, n_wg;
  const int32_t* pt; int page_lg;   // paged cache (PAGED kernels): the page of every 2^page_lg tokens
};

// Every storage type and head dimension, any group size up to 16 (groups wider than one pass holds are scanned
// in several passes over the keys).  kt: list length, a power of two <= 8.  grid: (workgroups per row, rows).
hipError_t launch_head_scan_valu(const Plan& pl, const HeadScanArgs& a, int kt, dim3 grid, hipStream_t st);

#ifdef __HIPCC__
// (score desc, index asc) as one unsigned 64-bit maximum; 0 is "nothing".
__device__ __forceinline__ uint64_t composite(float score, uint32_t pos) {
  return ((uint64_t)score_key(score) << 32) | (uint64_t)(0xffffffffu - pos);
}
__device__ __forceinline__ uint64_t wave_max_u64(uint64_t v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const uint32_t lo = __shfl_xor((uint32_t)v, o, 64), hi = __shfl_xor((uint32_t)(v >> 32), o, 64);
    const uint64_t w = ((uint64_t)hi << 32) | lo;
    v = w > v ? w : v;
  }
  return v;
}
#endif

}  // namespace reattn
