// Selection of a decode step over a long middle without a score array (paper Eq. 2 for one query row per KV
// head; appendix decoding phase, `idx_recall = topk(score, ...)`).  A million-token row would cost 4 bytes
// written and read back per key just to find the few thousand largest; instead
//
//   sample   every f_step-th key of the middle is scored first (about 8K..16K keys per row, ~1 % of the scan);
//            the rho-th largest sampled score, rho six binomial standard deviations above the expected rank of
//            the row's k-th score among the samples, is a lower bound of that k-th score (a filter, never the
//            answer).  The same launch fills the rotary table of the attention that follows.
//   scan     (score_scan.hip, filter mode) streams the keys once; every workgroup parks its slice's scores in
//            LDS, finds the bound from the row's samples, and leaves only the (score, position) pairs at or
//            above it, in position order, in its own segment: about 1.6 times k pairs per row instead of n_mid scores.
//   pick     one workgroup per row numbers the segments' pairs through (position order), holds their keys in
//            LDS, finds the exact k-th largest (score descending, index ascending) by radix select on the
//            offsets from the smallest candidate key, and writes the winners' absolute indices in ascending
//            order (ranks from wave ballots).  A row whose bound missed (fewer than k pairs: probability
//            ~1e-9 per row on exchangeable keys) or whose pairs exceed the LDS (degenerate rows: runs of
//            equal scores) recomputes its scores with the scan's arithmetic and selects exactly over all of
//            them: slow (one workgroup streams the row), same result.  (Measured: the redo has to be inlined
//            and hinted cold; as a called function its stack cost every launch 7 us, and as a launch of its
//            own behind the pick 4.5 us for finding its list empty.)
#include "common.hpp"
#include "select.hpp"

namespace reattn {
namespace {

struct SampleArgs {
  const void* k; const void* q; float* samp;
  int64_t samp_stride, ksh, kst, first_tok, step;
  uint32_t n_samp;
  int Hq, Hkv, G;
  const int32_t* pt; int page_lg;
  int n_sblocks;                 // workgroups along x that score samples; the ones behind them fill the rotary table
  float2* rope; int S, half, D; double log2_theta; int64_t n_rope;
  uint32_t* redo_count;          // cleared here, counted up by the pick
};

template <typename T, int D>
__global__ __launch_bounds__(256) void sample_score_kernel(SampleArgs a) {
  constexpr int EPL = Store<T>::kPerLoad, LPR = D / EPL, RPL = 64 / LPR, U = 8;
  constexpr int SPB = 4 * U * RPL;                          // sampled keys per workgroup
  if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0 && a.redo_count) *a.redo_count = 0u;
  if ((int)blockIdx.x >= a.n_sblocks) {
    if (blockIdx.y) return;
    const int64_t i = (int64_t)((int)blockIdx.x - a.n_sblocks) * 256 + threadIdx.x;
    if (a.rope && i < a.n_rope) a.rope[i] = rope_table_entry(i, a.S, a.half, a.D, a.log2_theta);
    return;
  }
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int sub = lane % LPR, grp = lane / LPR;
  const int row_id = blockIdx.y;                             // query * Hkv + kv head
  const int h = row_id % a.Hkv, qi = row_id / a.Hkv;
  const char* kbase = (const char*)a.k + (int64_t)h * a.ksh * (int64_t)sizeof(T) + sub * 16;
  const int64_t row_bytes = a.kst * (int64_t)sizeof(T);
  const uint32_t j0 = (uint32_t)blockIdx.x * SPB + (uint32_t)wave * (U * RPL);
  u32x4 d[U];                                                // the key rows first: the query's loads ride along
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const uint32_t j = j0 + u * RPL + grp;
    const int64_t tok = a.first_tok + (int64_t)(j < a.n_samp ? j : a.n_samp - 1) * a.step;   // clamped: result dropped
    const int64_t row = a.pt ? paged_row(a.pt, a.page_lg, tok) : tok;
    d[u] = *(const u32x4*)(kbase + row * row_bytes);
  }
  float qv[EPL];
  group_query<T, D>(a.q, qi, h, a.Hq, a.G, sub, qv);
  float* out = a.samp + (int64_t)row_id * a.samp_stride;
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const float s = row_dot<T, D>(d[u], qv);
    const uint32_t j = j0 + u * RPL + grp;
    if (sub == 0 && j < a.n_samp) out[j] = s;
  }
}

constexpr int kPickThreads = 1024;

struct PickArgs {
  const uint2* cand; const uint32_t* segcnt;                 // [rows][nb][rpb], [rows][nb]
  int nb, rpb, k_eff;
  int64_t n_mid; int32_t index_base;
  int32_t* idx;                                              // [rows][k_eff]
  uint32_t* redo;                                            // [0] rows that took the exact redo
  // the exact redo recomputes the row's scores: over the row's own segments, which it no longer needs
  const void* q; const void* k;
  int64_t ksh, kst, first_tok;
  const int32_t* pt; int page_lg;
  int Hq, Hkv, G;
};

// Exact selection over ALL scores of score row `row_id`, recomputed by this workgroup into sc[n_mid].
template <typename T, int D>
__device__ __forceinline__ void exact_row(const PickArgs& a, int row_id, float* sc, uint32_t* bins, uint32_t* sh) {
  constexpr int EPL = Store<T>::kPerLoad, LPR = D / EPL, RPL = 64 / LPR;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int sub = lane % LPR, grp = lane / LPR;
  const int h = row_id % a.Hkv, qi = row_id / a.Hkv;
  float qv[EPL];
  group_query<T, D>(a.q, qi, h, a.Hq, a.G, sub, qv);
  const char* kb = (const char*)a.k + ((int64_t)h * a.ksh + (a.pt ? 0 : a.first_tok) * a.kst) * (int64_t)sizeof(T) + sub * 16;
  const int64_t row_bytes = a.kst * (int64_t)sizeof(T);
  for (int64_t j0 = (int64_t)wave * RPL; j0 < a.n_mid; j0 += (int64_t)(kPickThreads / 64) * RPL) {
    const int64_t j = j0 + grp;
    const int64_t jc = j < a.n_mid ? j : a.n_mid - 1;
    const int64_t krow = a.pt ? paged_row(a.pt, a.page_lg, a.first_tok + jc) : jc;
    const u32x4 d = *(const u32x4*)(kb + krow * row_bytes);
    const float s = row_dot<T, D>(d, qv);
    if (sub == 0 && j < a.n_mid) sc[j] = s;
  }
  __threadfence_block();
  __syncthreads();
  int shift = 0; uint64_t prefix = 0;
  if ((int64_t)a.k_eff < a.n_mid)
    radix_kth<kPickThreads>([&](uint32_t j) -> uint64_t {
                              return ((uint64_t)score_key(sc[j]) << 32) | (uint64_t)(0xffffffffu - j);
                            }, (uint32_t)a.n_mid, (uint32_t)a.k_eff, 64, bins, sh, shift, prefix);
  int32_t* out = a.idx + (int64_t)row_id * a.k_eff;
  uint32_t done = 0;
  for (int64_t j0 = 0; j0 < a.n_mid; j0 += kPickThreads) {
    const int64_t j = j0 + threadIdx.x;
    uint32_t take = 0;
    if (j < a.n_mid) {
      const uint64_t v = ((uint64_t)score_key(sc[j]) << 32) | (uint64_t)(0xffffffffu - (uint32_t)j);
      take = (shift >= 64 ? 0ull : (v >> shift)) >= prefix ? 1u : 0u;
    }
    uint32_t total;
    const uint32_t at = done + block_scan_incl<kPickThreads>(take, sh, total) - take;
    if (take && at < (uint32_t)a.k_eff) out[at] = a.index_base + (int32_t)j;
    done += total;
  }
}

template <typename T, int D>
__global__ __launch_bounds__(kPickThreads) void decode_pick_kernel(PickArgs a) {
  extern __shared__ uint32_t pick_lds[];
  uint32_t* pfx = pick_lds;                                  // [nb + 1] pairs in front of every segment
  uint32_t* keys = pick_lds + ((a.nb + 1 + 3) & ~3);         // [n] ordered score keys of the row's pairs, in position order
  __shared__ uint32_t bins[kBinsPad];
  __shared__ uint32_t sh[40];
  __shared__ uint16_t gseg[kPickMax / 64];                   // segment of the group's first pair
  const int row_id = blockIdx.x;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t seg0 = (int64_t)row_id * a.nb;
  uint32_t n;
  {
    const uint32_t c = (int)threadIdx.x < a.nb ? a.segcnt[seg0 + threadIdx.x] : 0u;
    const uint32_t incl = block_scan_incl<kPickThreads>(c, sh, n);
    if ((int)threadIdx.x < a.nb) pfx[threadIdx.x] = incl - c;
    if (threadIdx.x == 0) pfx[a.nb] = n;
    __syncthreads();
  }
  const uint32_t k = (uint32_t)a.k_eff;
  if (__builtin_expect(n < k || n > (uint32_t)kPickMax, 0)) {   // workgroup-uniform: bound missed, or too many pairs
    if (threadIdx.x == 0) atomicAdd(a.redo, 1u);
    exact_row<T, D>(a, row_id, (float*)(a.cand + seg0 * a.rpb), bins, sh);
    return;
  }
  // The pairs are numbered through in position order and cut into one run per wave (a multiple of 64 pairs):
  // pair w * run + 64 u + lane is slot u of that lane of wave w; its key goes into LDS, its position stays in
  // a register.  The segment of a pair is found from a table that names, for every group of 64 consecutive
  // pairs, the segment of the group's first pair (filled by the thread that owns that segment), plus a short
  // walk forward.  Sixteen pairs per thread at a time, their loads issued together (indices clamped, not
  // predicated), so a batch costs one trip to memory.
  if ((int)threadIdx.x < a.nb) {
    const uint32_t first = pfx[threadIdx.x], end = pfx[threadIdx.x + 1];
    for (uint32_t g = (first + 63) >> 6; (g << 6) < end; ++g) gseg[g] = (uint16_t)threadIdx.x;
  }
  __syncthreads();
  constexpr int kWaves = kPickThreads / 64;
  constexpr int kSlots = kPickMax / kPickThreads, kBatch = 16;
  static_assert(kSlots % kBatch == 0, "whole batches");
  const uint32_t run = ((n + kWaves - 1) / kWaves + 63) / 64 * 64;     // <= 64 * kSlots
  const uint32_t mine0 = (uint32_t)wave * run + lane;
  uint32_t pos[kSlots];
  uint32_t kmin = 0xffffffffu, kmax = 0u;
#pragma unroll
  for (int b0 = 0; b0 < kSlots; b0 += kBatch) {
    if ((uint32_t)b0 * 64 < run) {                           // workgroup-uniform
      const uint2* src[kBatch];
#pragma unroll
      for (int u = 0; u < kBatch; ++u) {
        const uint32_t i = mine0 + (uint32_t)(b0 + u) * 64;
        const uint32_t ic = i < n ? i : n - 1;
        int sg = gseg[ic >> 6];
        while (pfx[sg + 1] <= ic) ++sg;                      // ends: pfx[nb] = n > ic
        src[u] = a.cand + (seg0 + sg) * a.rpb + (ic - pfx[sg]);
      }
      uint2 c[kBatch];
#pragma unroll
      for (int u = 0; u < kBatch; ++u) c[u] = *src[u];
#pragma unroll
      for (int u = 0; u < kBatch; ++u) {
        const uint32_t i = mine0 + (uint32_t)(b0 + u) * 64;
        pos[b0 + u] = c[u].y;
        if (i < n && (uint32_t)(b0 + u) * 64 < run) {
          const uint32_t key = score_key(__uint_as_float(c[u].x));
          keys[i] = key;
          kmin = min(kmin, key); kmax = max(kmax, key);
        }
      }
    } else {
#pragma unroll
      for (int u = 0; u < kBatch; ++u) pos[b0 + u] = 0u;
    }
  }
  block_minmax<kPickThreads>(kmin, kmax, sh);                // its barriers also publish the keys
  const int nbits = 32 - __clz((int)(kmax - kmin));          // significant bits of the offsets (0 when all keys are equal)

  // Winners: in the offset part d = key - kmin, d >> dsh >= dpref; once a tie on d = dpref had to be broken,
  // d > dpref, or d == dpref and the pair's number i (position order: lower first) satisfies ~i >> psh >= ppref.
  const bool all = k == n;
  bool tie = false;
  uint32_t dpref = 0, ppref = 0;
  int dsh = nbits, psh = 32;
  if (!all) {
    uint32_t remaining = k;
    bool done = false;
    auto pass = [&](bool on_pos, int sft, int w) {
      for (int b = threadIdx.x; b < kBinsPad; b += kPickThreads) bins[b] = 0;
      __syncthreads();
      const int up = sft + w;                                // up == 32 only on a first pass: no prefix yet
      for (uint32_t i = threadIdx.x; i < n; i += kPickThreads) {
        const uint32_t d = keys[i] - kmin;
        const uint32_t v = on_pos ? ~i : d;
        const bool in = (up >= 32 || (v >> up) == (on_pos ? ppref : dpref)) && (!on_pos || d == dpref);
        if (in) atomicAdd(&bins[bslot((int)((v >> sft) & ((1u << w) - 1u)))], 1u);
      }
      __syncthreads();
      uint32_t d, ab;
      kth_bin<kPickThreads>(bins, remaining, sh, d, ab);
      const uint32_t in_bin = bins[bslot((int)d)];
      remaining -= ab;
      if (on_pos) ppref = (ppref << w) | d; else dpref = (dpref << w) | d;
      __syncthreads();
      done = in_bin == remaining;                            // everything that shares this prefix is selected
    };
    while (dsh > 0 && !done) {
      const int w = dsh < 11 ? dsh : 11;
      dsh -= w;
      pass(false, dsh, w);
    }
    if (!done) {                                             // dpref is the k-th entry's d: the tie ends on the position
      tie = true;
      while (psh > 0 && !done) {
        const int w = psh < 11 ? psh : 11;
        psh -= w;
        pass(true, psh, w);
      }
    }
  }
  auto wins = [&](uint32_t i) -> bool {
    if (i >= n) return false;
    if (all) return true;
    const uint32_t d = keys[i] - kmin;
    return tie ? (d > dpref || (d == dpref && (~i >> psh) >= ppref)) : (dsh >= 32 || (d >> dsh) >= dpref);
  };
  // ranks: pairs are numbered in position order, so a winner's place in the ascending index list is the
  // number of winners in front of it: the totals of the waves before its own, the ballots of its wave's
  // earlier slots, and the lanes below it in its own slot's ballot
  uint32_t won = 0, total = 0;
#pragma unroll 4
  for (int u = 0; u < kSlots; ++u) {
    const bool live = (uint32_t)u * 64 < run;                // wave-uniform
    const bool win = live && wins(mine0 + (uint32_t)u * 64);
    const uint64_t b = __ballot(win);
    won |= win ? 1u << u : 0u;
    total += (uint32_t)__popcll(b);
  }
  if (lane == 0) sh[wave] = total;
  __syncthreads();
  uint32_t at0 = 0;
#pragma unroll
  for (int w = 0; w < kWaves; ++w) at0 += w < wave ? sh[w] : 0u;
  int32_t* out = a.idx + (int64_t)row_id * a.k_eff;
  const uint64_t below = (1ull << lane) - 1ull;
#pragma unroll
  for (int u = 0; u < kSlots; ++u) {
    if ((uint32_t)u * 64 < run) {                            // wave-uniform
      const bool win = (won >> u) & 1u;
      const uint64_t b = __ballot(win);
      const uint32_t at = at0 + (uint32_t)__popcll(b & below);
      if (win && at < k) out[at] = a.index_base + (int32_t)pos[u];
      at0 += (uint32_t)__popcll(b);
    }
  }
}

template <typename T, int D>
hipError_t sample_td(const SampleArgs& a0, int rows, hipStream_t st) {
  constexpr int EPL = Store<T>::kPerLoad, RPL = 64 / (D / EPL);
  constexpr int SPB = 4 * 8 * RPL;
  SampleArgs a = a0;
  a.n_sblocks = (int)((a.n_samp + SPB - 1) / SPB);
  const int extra = (int)((a.n_rope + 255) / 256);
  hipLaunchKernelGGL((sample_score_kernel<T, D>), dim3(a.n_sblocks + extra, rows), dim3(256), 0, st, a);
  return hipGetLastError();
}

template <typename T, int D>
hipError_t pick_td(const PickArgs& a, int rows, hipStream_t st) {
  const size_t lds = ((size_t)((a.nb + 1 + 3) & ~3) + kPickMax) * 4;     // segment prefix + the pairs' keys
  auto kern = decode_pick_kernel<T, D>;
  hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, dim3(rows), dim3(kPickThreads), lds, st, a);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_decode_sample(const Plan& pl, const void* q, const void* k_cache, float* samp, float2* rope,
                                uint32_t* redo_count, hipStream_t st) {
  if (!pl.filter) return hipErrorInvalidValue;
  SampleArgs a;
  a.redo_count = redo_count;
  a.k = k_cache; a.q = q; a.samp = samp; a.samp_stride = pl.f_samp_stride;
  a.ksh = pl.ksh; a.kst = pl.kst; a.first_tok = pl.s_eff; a.step = pl.f_step; a.n_samp = pl.f_nsamp;
  a.Hq = pl.Hq; a.Hkv = pl.Hkv; a.G = pl.G; a.pt = pl.pt; a.page_lg = pl.page_lg; a.n_sblocks = 0;
  a.rope = rope; a.S = pl.S; a.half = pl.D / 2; a.D = pl.D; a.log2_theta = log2((double)pl.theta);
  a.n_rope = rope ? (int64_t)(rope_rows_hi(pl.S) + kRopeLo) * (pl.D / 2) : 0;
  const int rows = pl.Hkv;                                  // one query row: the filter path is a decode step's
  if (pl.dtype == kF32) return pl.D == 64 ? sample_td<float, 64>(a, rows, st) : sample_td<float, 128>(a, rows, st);
  if (pl.dtype == kF16) return pl.D == 64 ? sample_td<f16bits, 64>(a, rows, st) : sample_td<f16bits, 128>(a, rows, st);
  return pl.D == 64 ? sample_td<uint16_t, 64>(a, rows, st) : sample_td<uint16_t, 128>(a, rows, st);
}

hipError_t launch_decode_pick(const Plan& pl, const void* q, const void* k_cache, const uint2* cand,
                              const uint32_t* segcnt, int32_t* idx, uint32_t* redo_count, hipStream_t st) {
  if (!pl.filter || pl.f_nb > kPickSlices) return hipErrorInvalidValue;
  PickArgs a;
  a.cand = cand; a.segcnt = segcnt; a.nb = pl.f_nb; a.rpb = pl.f_rpb; a.k_eff = pl.k_eff;
  a.n_mid = pl.n_mid; a.index_base = (int32_t)pl.s_eff; a.idx = idx; a.redo = redo_count;
  a.q = q; a.k = k_cache; a.ksh = pl.ksh; a.kst = pl.kst; a.first_tok = pl.s_eff;
  a.pt = pl.pt; a.page_lg = pl.page_lg; a.Hq = pl.Hq; a.Hkv = pl.Hkv; a.G = pl.G;
  const int rows = pl.Hkv;
  if (pl.dtype == kF32) return pl.D == 64 ? pick_td<float, 64>(a, rows, st) : pick_td<float, 128>(a, rows, st);
  if (pl.dtype == kF16) return pl.D == 64 ? pick_td<f16bits, 64>(a, rows, st) : pick_td<f16bits, 128>(a, rows, st);
  return pl.D == 64 ? pick_td<uint16_t, 64>(a, rows, st) : pick_td<uint16_t, 128>(a, rows, st);
}

}  // namespace reattn
