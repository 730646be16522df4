// Stage 1, second half: exact top-k over each row of middle scores (paper Eq. 2,
// `Indices = top-k(q K_middle^T)`), returned as absolute cache positions in
// ascending order so that the selected entries keep their relative order
// (paper, "Training-Free Integration").  Order: higher score first, ties by lower
// index; the result is deterministic.
//
// A row holds up to millions of fp32 scores and k is a few thousand, so the work
// is a radix select on the order-preserving uint32 image of the scores:
//   hist    (optional; the decode scan produces it on the fly) 4096-bin histogram
//           of the top 12 key bits, built in LDS per workgroup;
//   pivot   (a device function run by every select/refine workgroup, 16 KiB of L2
//           reads) finds the bin that holds the k-th largest key;
//   select  ONE pass over the scores: entries in higher bins are final and go
//           straight into a per-row bitmap via wave ballots (no atomics); entries
//           in the pivot bin (typically < 1 % of the row) go to per-chunk segments
//           of a candidate array;
//   refine  one workgroup per row resolves the remaining 20 key bits and the index
//           tie-break among the candidates with LDS histograms (11-bit digits over
//           the 52-bit composite (key_low, ~index)) and marks the winners;
//   emit    ordered compaction of the bitmap: per-chunk counts + popcount scan give
//           every set bit its rank, i.e. its place in the ascending index list.
#include "common.hpp"

namespace reattn {
namespace {

// ---- hist: first radix digit of every score of a row ----------------------
__global__ __launch_bounds__(256) void topk_hist_kernel(const float* __restrict__ scores,
                                                        int64_t n_mid, uint32_t* hist) {
  __shared__ uint32_t lh[kHistBins];
  for (int b = threadIdx.x; b < kHistBins; b += 256) lh[b] = 0;
  __syncthreads();
  const int row = blockIdx.y;
  const float* sc = scores + (int64_t)row * n_mid;
  const int64_t p0 = (int64_t)blockIdx.x * kChunk;
#pragma unroll 8
  for (int i = 0; i < kChunk / 256; ++i) {
    const int64_t pos = p0 + i * 256 + threadIdx.x;
    if (pos < n_mid) atomicAdd(&lh[score_key(sc[pos]) >> kKeyShift], 1u);
  }
  __syncthreads();
  uint32_t* gh = hist + (int64_t)row * kHistBins;
  for (int b = threadIdx.x; b < kHistBins; b += 256) {
    const uint32_t c = lh[b];
    if (c) atomicAdd(&gh[b], c);
  }
}

// ---- select: one pass over the scores --------------------------------------
// A workgroup owns kChunk consecutive positions; each wave 2048 of them, 64 per
// iteration.  Lane `it` keeps the two ballots of iteration `it` (final entries,
// pivot-bin entries), so after the loop the wave holds its slice of the bitmap in
// registers.  Candidates go to the chunk's own segment of the candidate array and the
// chunk's count is a plain store: no global atomics (returning atomics on one address
// serialise at ~135 ns each on this chip, which made a shared list the bottleneck).
__global__ __launch_bounds__(256) void topk_select_kernel(
    const float* __restrict__ scores, int64_t n_mid, const uint32_t* __restrict__ hist, uint32_t k,
    uint32_t* ncand, int32_t* cand, uint32_t* bitmap, int64_t nwords, uint32_t* cnt, int nchunks) {
  __shared__ uint32_t w_take[4], w_cand[4], sh[40];
  const int row = blockIdx.y, c = blockIdx.x;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const float* sc = scores + (int64_t)row * n_mid;
  const int64_t wbase = (int64_t)c * kChunk + wave * (kChunk / 4);
  // all 32 loads of this lane go out before anything waits on them
  float v[32];
#pragma unroll
  for (int j = 0; j < 32; ++j) {
    const int64_t pos = wbase + j * 64 + lane;
    v[j] = sc[pos < n_mid ? pos : n_mid - 1];      // clamped, not predicated: a predicated load waits for the one before it
  }
  uint32_t pbin, above;
  find_kth_bin<256, kHistBins>(hist + (int64_t)row * kHistBins, k, sh, pbin, above);
  uint64_t take_mask = 0, cand_mask = 0;
#pragma unroll
  for (int j = 0; j < 32; ++j) {
    const int64_t pos = wbase + j * 64 + lane;
    const bool valid = pos < n_mid;
    const uint32_t bin = score_key(v[j]) >> kKeyShift;
    const uint64_t mt = __ballot(valid && bin > pbin);
    const uint64_t mc = __ballot(valid && bin == pbin);
    if (lane == j) { take_mask = mt; cand_mask = mc; }
  }
  // lanes 0..31 hold the masks of iterations 0..31 (lanes 32..63 hold zeros)
  const uint32_t n_take = (uint32_t)__popcll(take_mask);
  const uint32_t n_cand = (uint32_t)__popcll(cand_mask);
  uint32_t tsum = n_take, cincl = n_cand;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) tsum += __shfl_xor(tsum, o, 64);
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const uint32_t y = __shfl_up(cincl, o, 64);
    if (lane >= o) cincl += y;
  }
  if (lane < 32) ((uint64_t*)(bitmap + (int64_t)row * nwords))[(wbase >> 6) + lane] = take_mask;
  if (lane == 63) { w_take[wave] = tsum; w_cand[wave] = cincl; }
  __syncthreads();
  if (threadIdx.x == 0) {
    cnt[(int64_t)row * nchunks + c] = w_take[0] + w_take[1] + w_take[2] + w_take[3];
    ncand[(int64_t)row * nchunks + c] = w_cand[0] + w_cand[1] + w_cand[2] + w_cand[3];
  }
  if (cand_mask) {
    uint32_t at = cincl - n_cand;
    for (int w = 0; w < wave; ++w) at += w_cand[w];
    int32_t* my_cand = cand + ((int64_t)row * nchunks + c) * kChunk;
    const int32_t first = (int32_t)(wbase + lane * 64);
    uint64_t m = cand_mask;
    while (m) {
      const int b = __ffsll((unsigned long long)m) - 1;
      m &= m - 1;
      my_cand[at++] = first + b;
    }
  }
}

// ---- refine: exact choice inside the pivot bin ------------------------------
__device__ __forceinline__ uint64_t composite(const float* sc, int32_t pos) {
  const uint64_t low = score_key(sc[pos]) & ((1u << kKeyShift) - 1u);
  return (low << 32) | (uint64_t)(0xffffffffu - (uint32_t)pos);   // lower index = larger value
}

constexpr int kRefineCache = 12288;   // candidates whose composite keys are kept in LDS (96 KiB)
constexpr int kRefinePfx = 4096;      // chunks whose candidate offsets are kept in LDS
constexpr size_t kRefineLds = 2048 * 4 + kRefinePfx * 4 + (size_t)kRefineCache * 8;

__global__ __launch_bounds__(1024) void topk_refine_kernel(
    const float* __restrict__ scores, int64_t n_mid, uint32_t* __restrict__ hist, uint32_t k,
    const uint32_t* __restrict__ ncand, const int32_t* __restrict__ cand, uint32_t* gpfx,
    uint32_t* bitmap, int64_t nwords, uint32_t* cnt, int nchunks) {
  extern __shared__ uint64_t refine_lds[];
  uint64_t* cached = refine_lds;                              // [kRefineCache]
  uint32_t* bins = (uint32_t*)(refine_lds + kRefineCache);    // [2048]
  uint32_t* lpfx = bins + 2048;                               // [kRefinePfx]
  __shared__ uint32_t sh[40];
  const int row = blockIdx.x;
  const float* sc = scores + (int64_t)row * n_mid;
  const int32_t* my_cand = cand + (int64_t)row * nchunks * kChunk;
  const uint32_t* my_n = ncand + (int64_t)row * nchunks;
  uint32_t pbin, above;
  find_kth_bin<1024, kHistBins>(hist + (int64_t)row * kHistBins, k, sh, pbin, above);
  const uint32_t need = k - above;               // entries of the pivot bin that are selected
  // the row's histogram has had its last reader: left zeroed for the next selection over this workspace
  static_assert(kHistBins == 4 * 1024, "four bins per thread");
  *(uint4*)(hist + (int64_t)row * kHistBins + 4 * threadIdx.x) = uint4{0u, 0u, 0u, 0u};

  // flatten the per-chunk candidate segments: exclusive prefix of their counts
  uint32_t* pfx = nchunks <= kRefinePfx ? lpfx : gpfx + (int64_t)row * nchunks;
  uint32_t n = 0;
  for (int c0 = 0; c0 < nchunks; c0 += 1024) {
    const int c = c0 + threadIdx.x;
    const uint32_t x = c < nchunks ? my_n[c] : 0u;
    uint32_t tot;
    const uint32_t incl = block_scan_incl<1024>(x, sh, tot);
    if (c < nchunks) pfx[c] = n + incl - x;
    n += tot;
  }
  __threadfence_block();
  __syncthreads();
  auto position = [&](uint32_t f) -> int32_t {   // f-th candidate of the row
    int lo = 0, hi = nchunks - 1;                // largest chunk with pfx[chunk] <= f
    while (lo < hi) {
      const int mid = (lo + hi + 1) >> 1;
      if (pfx[mid] <= f) lo = mid; else hi = mid - 1;
    }
    return my_cand[(int64_t)lo * kChunk + (f - pfx[lo])];
  };
  for (uint32_t i = threadIdx.x; i < n && i < kRefineCache; i += 1024)
    cached[i] = composite(sc, position(i));
  __syncthreads();
  auto comp = [&](uint32_t i) -> uint64_t {
    return i < kRefineCache ? cached[i] : composite(sc, position(i));
  };

  int shift = 0;
  uint64_t prefix = 0;                           // select comp >> shift >= prefix
  if (need < n) {
    shift = kKeyShift + 32;
    uint32_t remaining = need;
    while (shift > 0) {
      const int w = shift < 11 ? shift : 11;
      shift -= w;
      for (int b = threadIdx.x; b < 2048; b += 1024) bins[b] = 0;
      __syncthreads();
      for (uint32_t i = threadIdx.x; i < n; i += 1024) {
        const uint64_t cv = comp(i);
        if ((cv >> (shift + w)) == prefix)
          atomicAdd(&bins[(uint32_t)(cv >> shift) & ((1u << w) - 1u)], 1u);
      }
      __syncthreads();
      uint32_t d, ab;
      find_kth_bin<1024, 2048>(bins, remaining, sh, d, ab);
      const uint32_t in_bin = bins[d];
      remaining -= ab;
      prefix = (prefix << w) | d;
      __syncthreads();
      if (in_bin == remaining) break;            // every entry sharing this prefix is selected
    }
  }
  // mark the winners; per-chunk counts go through LDS (this workgroup owns the row)
  uint32_t* bm = bitmap + (int64_t)row * nwords;
  uint32_t* ct = cnt + (int64_t)row * nchunks;
  for (int c0 = 0; c0 < nchunks; c0 += 2048) {
    const int nc = nchunks - c0 < 2048 ? nchunks - c0 : 2048;
    for (int b = threadIdx.x; b < nc; b += 1024) bins[b] = 0;
    __syncthreads();
    for (uint32_t i = threadIdx.x; i < n; i += 1024) {
      const uint64_t cv = comp(i);
      const int32_t pos = (int32_t)(0xffffffffu - (uint32_t)cv);
      const int ch = pos / kChunk - c0;
      if (ch >= 0 && ch < nc && (cv >> shift) >= prefix) {
        atomicOr(&bm[pos >> 5], 1u << (pos & 31));
        atomicAdd(&bins[ch], 1u);
      }
    }
    __syncthreads();
    for (int b = threadIdx.x; b < nc; b += 1024)
      if (bins[b]) ct[c0 + b] += bins[b];
    __syncthreads();
  }
}

// ---- emit: ordered compaction of the bitmap ---------------------------------
__global__ __launch_bounds__(256) void topk_emit_kernel(
    const uint32_t* __restrict__ bitmap, int64_t nwords, const uint32_t* __restrict__ cnt,
    int nchunks, int32_t index_base, int32_t* idx, int k_eff) {
  __shared__ uint32_t sh[8];
  const int row = blockIdx.y, c = blockIdx.x;
  uint32_t before = 0;
  for (int i = threadIdx.x; i < c; i += 256) before += cnt[(int64_t)row * nchunks + i];
  uint32_t chunk_base;
  block_scan_incl<256>(before, sh, chunk_base);   // only the total is used
  uint32_t w = bitmap[(int64_t)row * nwords + (int64_t)c * kChunkWords + threadIdx.x];
  const uint32_t p = (uint32_t)__popc(w);
  uint32_t chunk_total;
  uint32_t at = chunk_base + block_scan_incl<256>(p, sh, chunk_total) - p;
  int32_t* out = idx + (int64_t)row * k_eff;
  const int32_t first = index_base + c * kChunk + (int)threadIdx.x * 32;
  while (w) {
    const int b = __ffs((int)w) - 1;
    w &= w - 1;
    if (at < (uint32_t)k_eff) out[at] = first + b;
    ++at;
  }
}

// ---- one workgroup per row: select + refine + emit without leaving the CU ----------------
// For rows of up to kRowMax scores (contexts up to ~64K tokens) the three kernels above are
// mostly launch gaps and dependent trips to memory (past that size one CU cannot pull a row
// fast enough and the chip-wide select pass wins): a whole row's bitmap (8 KiB) and its
// pivot-bin candidates fit one workgroup's LDS, so one workgroup reads the row once (entries
// above the pivot bin go to the LDS bitmap through wave ballots, entries in it to an LDS list
// of composites), resolves the pivot bin with the same 11-bit radix passes, and ranks the
// bitmap into the ascending index list, which leaves in 16-byte rows.  Rows whose pivot bin
// holds more than kRowCand entries (degenerate score distributions) keep what fits in LDS and
// re-read the rest from the scores on every pass: slower, same result.
constexpr int kRowCand = 8192;                    // pivot-bin entries cached in LDS (64 KiB)
constexpr int kRowThreads = 1024;
constexpr size_t kRowLds = (size_t)kRowMax / 8 + (size_t)kRowCand * 8 + 2048 * 4;

__global__ __launch_bounds__(kRowThreads) void topk_row_kernel(
    const float* __restrict__ scores, int64_t n_mid, uint32_t* __restrict__ hist, uint32_t k,
    int32_t index_base, int32_t* idx, int k_eff) {
  extern __shared__ uint64_t row_lds[];
  uint64_t* cand = row_lds;                                   // [kRowCand] composites; later the ranked indices
  uint32_t* bitmap = (uint32_t*)(row_lds + kRowCand);         // [kRowMax / 32]
  uint32_t* bins = bitmap + kRowMax / 32;                     // [2048]
  __shared__ uint32_t sh[40];
  __shared__ uint32_t s_ncand;
  const int row = blockIdx.x;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const float* sc = scores + (int64_t)row * n_mid;
  const int n = (int)n_mid;
  const int nwords = (n + 31) / 32;
  const int nwords_pad = (nwords + kRowThreads - 1) / kRowThreads * kRowThreads;
  if (threadIdx.x == 0) s_ncand = 0;
  uint32_t pbin, above;
  find_kth_bin<kRowThreads, kHistBins>(hist + (int64_t)row * kHistBins, k, sh, pbin, above);
  const uint32_t need = k - above;                            // entries of the pivot bin that are selected
  // the row's histogram has had its only reader: left zeroed for the next selection over this workspace
  static_assert(kHistBins == 4 * kRowThreads, "four bins per thread");
  *(uint4*)(hist + (int64_t)row * kHistBins + 4 * threadIdx.x) = uint4{0u, 0u, 0u, 0u};
  for (int w = nwords + threadIdx.x; w < nwords_pad; w += kRowThreads) bitmap[w] = 0;   // words past the row

  // one pass over the row: a wave takes 64 consecutive positions per load, 16 loads in flight
  constexpr int U = 16;
  for (int base = wave * 64 * U; base < n; base += (kRowThreads / 64) * 64 * U) {
    float v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int pos = base + u * 64 + lane;
      v[u] = sc[pos < n ? pos : n - 1];                          // clamped, not predicated: the loads go out together
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int p0 = base + u * 64;
      if (p0 >= n) break;                                      // wave-uniform
      const int pos = p0 + lane;
      const uint32_t key = score_key(v[u]);
      const uint32_t bin = key >> kKeyShift;
      const bool valid = pos < n;
      const uint64_t take = __ballot(valid && bin > pbin);
      const bool is_cand = valid && bin == pbin;
      const uint64_t cm = __ballot(is_cand);
      if (lane == 0) ((uint64_t*)bitmap)[p0 >> 6] = take;
      if (cm) {
        uint32_t at = 0;
        if (lane == 0) at = atomicAdd(&s_ncand, (uint32_t)__popcll(cm));
        at = __shfl((int)at, 0, 64) + (uint32_t)__popcll(cm & ((1ull << lane) - 1ull));
        if (is_cand && at < (uint32_t)kRowCand)
          cand[at] = ((uint64_t)(key & ((1u << kKeyShift) - 1u)) << 32) | (uint64_t)(0xffffffffu - (uint32_t)pos);
      }
    }
  }
  __syncthreads();
  const uint32_t ncand = s_ncand;
  const uint32_t ncached = ncand < (uint32_t)kRowCand ? ncand : (uint32_t)kRowCand;
  const bool spill = ncand > (uint32_t)kRowCand;              // workgroup-uniform
  // every pivot-bin entry once: the cached ones from LDS; on a spill, all of them from the scores
  auto for_each_cand = [&](auto&& f) {
    if (!spill) {
      for (uint32_t i = threadIdx.x; i < ncached; i += kRowThreads) f(cand[i]);
    } else {
      for (int pos = threadIdx.x; pos < n; pos += kRowThreads) {
        const uint32_t key = score_key(sc[pos]);
        if ((key >> kKeyShift) == pbin)
          f(((uint64_t)(key & ((1u << kKeyShift) - 1u)) << 32) | (uint64_t)(0xffffffffu - (uint32_t)pos));
      }
    }
  };
  int shift = 0;
  uint64_t prefix = 0;                                        // winners: composite >> shift >= prefix
  if (need < ncand) {
    shift = kKeyShift + 32;
    uint32_t remaining = need;
    while (shift > 0) {
      const int w = shift < 11 ? shift : 11;
      shift -= w;
      for (int b = threadIdx.x; b < 2048; b += kRowThreads) bins[b] = 0;
      __syncthreads();
      for_each_cand([&](uint64_t cv) {
        if ((cv >> (shift + w)) == prefix) atomicAdd(&bins[(uint32_t)(cv >> shift) & ((1u << w) - 1u)], 1u);
      });
      __syncthreads();
      uint32_t d, ab;
      find_kth_bin<kRowThreads, 2048>(bins, remaining, sh, d, ab);
      const uint32_t in_bin = bins[d];
      remaining -= ab;
      prefix = (prefix << w) | d;
      __syncthreads();
      if (in_bin == remaining) break;                          // every entry sharing this prefix is selected
    }
  }
  if (need > 0)
    for_each_cand([&](uint64_t cv) {
      if ((cv >> shift) >= prefix) {
        const uint32_t pos = 0xffffffffu - (uint32_t)cv;
        atomicOr(&bitmap[pos >> 5], 1u << (pos & 31));
      }
    });
  __syncthreads();
  // ordered compaction: thread t owns words [t*wpt, (t+1)*wpt), wpt <= 2
  const int wpt = nwords_pad / kRowThreads;
  uint32_t word[kRowMax / 32 / kRowThreads];
  uint32_t mine = 0;
#pragma unroll
  for (int w = 0; w < kRowMax / 32 / kRowThreads; ++w) {
    word[w] = w < wpt ? bitmap[threadIdx.x * wpt + w] : 0u;
    mine += __popc(word[w]);
  }
  uint32_t total;
  uint32_t at = block_scan_incl<kRowThreads>(mine, sh, total) - mine;
  int32_t* out = idx + (int64_t)row * k_eff;
  const bool staged = (size_t)k_eff * 4 <= (size_t)kRowCand * 8;   // the candidate list is spent: it stages the indices
  int32_t* dst = staged ? (int32_t*)cand : out;
#pragma unroll
  for (int w = 0; w < kRowMax / 32 / kRowThreads; ++w) {
    uint32_t bits = word[w];
    const int32_t first = index_base + (threadIdx.x * wpt + w) * 32;
    while (bits) {
      const int b = __ffs((int)bits) - 1;
      bits &= bits - 1;
      if (at < (uint32_t)k_eff) dst[at] = first + b;
      ++at;
    }
  }
  if (staged) {
    __syncthreads();
    if ((k_eff & 3) == 0 && ((uintptr_t)idx & 15) == 0) {
      for (int j = threadIdx.x; j < k_eff / 4; j += kRowThreads) ((int4*)out)[j] = ((const int4*)dst)[j];
    } else {
      for (int j = threadIdx.x; j < k_eff; j += kRowThreads) out[j] = dst[j];
    }
  }
}

}  // namespace

hipError_t launch_topk(const Plan& pl, int rows, const float* scores, bool hist_ready,
                       uint32_t* hist, uint32_t* pfx, uint32_t* ncand, int32_t* cand,
                       uint32_t* bitmap, uint32_t* cnt, int32_t* idx, hipStream_t st) {
  if (pl.k_eff <= 0 || rows <= 0) return hipSuccess;
  {
    hipError_t e = hipFuncSetAttribute((const void*)topk_refine_kernel,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)kRefineLds);
    if (e != hipSuccess) return e;
  }
  const dim3 per_chunk((unsigned)pl.nchunks, (unsigned)rows);
  const uint32_t k = (uint32_t)pl.k_eff;
  if (!hist_ready)
    hipLaunchKernelGGL(topk_hist_kernel, per_chunk, dim3(256), 0, st, scores, pl.n_mid, hist);
  if (pl.n_mid <= kRowMax) {                        // short rows: one workgroup does the whole row
    hipError_t e = hipFuncSetAttribute((const void*)topk_row_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)kRowLds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(topk_row_kernel, dim3(rows), dim3(kRowThreads), kRowLds, st, scores, pl.n_mid, hist, k,
                       (int32_t)pl.s_eff, idx, pl.k_eff);
    return hipGetLastError();
  }
  hipLaunchKernelGGL(topk_select_kernel, per_chunk, dim3(256), 0, st, scores, pl.n_mid, hist, k,
                     ncand, cand, bitmap, pl.nwords, cnt, pl.nchunks);
  hipLaunchKernelGGL(topk_refine_kernel, dim3(rows), dim3(1024), kRefineLds, st, scores, pl.n_mid,
                     hist, k, ncand, cand, pfx, bitmap, pl.nwords, cnt, pl.nchunks);
  hipLaunchKernelGGL(topk_emit_kernel, per_chunk, dim3(256), 0, st, bitmap, pl.nwords, cnt,
                     pl.nchunks, (int32_t)pl.s_eff, idx, pl.k_eff);
  return hipGetLastError();
}

}  // namespace reattn
