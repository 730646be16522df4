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
    v[j] = pos < n_mid ? sc[pos] : 0.f;
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
    const float* __restrict__ scores, int64_t n_mid, const uint32_t* __restrict__ hist, uint32_t k,
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
  hipLaunchKernelGGL(topk_select_kernel, per_chunk, dim3(256), 0, st, scores, pl.n_mid, hist, k,
                     ncand, cand, bitmap, pl.nwords, cnt, pl.nchunks);
  hipLaunchKernelGGL(topk_refine_kernel, dim3(rows), dim3(1024), kRefineLds, st, scores, pl.n_mid,
                     hist, k, ncand, cand, pfx, bitmap, pl.nwords, cnt, pl.nchunks);
  hipLaunchKernelGGL(topk_emit_kernel, per_chunk, dim3(256), 0, st, bitmap, pl.nwords, cnt,
                     pl.nchunks, (int32_t)pl.s_eff, idx, pl.k_eff);
  return hipGetLastError();
}

}  // namespace reattn
