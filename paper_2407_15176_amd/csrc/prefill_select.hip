// Per-query top-k for a prefill chunk (paper Eq. 2 applied to each query row of the
// chunk; appendix prefilling phase, `idx_recall = topk(score, ...)`) without ever
// holding the M x N_mid score matrix:
//
//   sample_threshold  per (query, KV head): the rho-th largest of the scores of a
//                     strided sample of the keys.  rho sits six binomial standard
//                     deviations above the expected rank of the true k-th score, so
//                     the value is a lower bound of it except with probability ~1e-9
//                     per row; it is only a filter, never the answer.
//   (score_gemm.hip)  the fused MFMA contraction appends every (score, key) pair at
//                     or above that bound to the row's candidate segment.
//   cand_topk         one workgroup per row: exact k-th largest composite
//                     (score desc, key asc) among the ~1.5 k candidates by radix
//                     select with LDS histograms, winners marked in an LDS bitmap over
//                     the middle, popcount scan -> ascending absolute indices.  Rows
//                     whose candidate count is below k (bound too high) or above the
//                     segment capacity go to a redo list.
//   row_exact         the redo path: one workgroup recomputes the row's scores with
//                     the streaming kernel's arithmetic and selects exactly, whatever
//                     the distribution (all-equal scores, adversarial data).
#include "common.hpp"

namespace reattn {
namespace {

template <int NT>
__device__ __forceinline__ uint32_t bscan_incl(uint32_t v, uint32_t* wsum, uint32_t& total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  uint32_t x = v;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const uint32_t y = __shfl_up(x, o, 64);
    if (lane >= o) x += y;
  }
  if (lane == 63) wsum[wave] = x;
  __syncthreads();
  uint32_t base = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < NT / 64; ++w) {
    const uint32_t s = wsum[w];
    base += (w < wave) ? s : 0u;
    tot += s;
  }
  __syncthreads();
  total = tot;
  return x + base;
}

// bins[0..2048): largest-first search for the bin holding the k-th entry (1 <= k <= total).
template <int NT>
__device__ __forceinline__ void kth_bin(const uint32_t* bins, uint32_t k, uint32_t* sh,
                                        uint32_t& bin, uint32_t& above) {
  constexpr int BPT = 2048 / NT;
  uint32_t loc[BPT], sum = 0;
#pragma unroll
  for (int i = 0; i < BPT; ++i) { loc[i] = bins[threadIdx.x * BPT + i]; sum += loc[i]; }
  uint32_t total;
  const uint32_t incl = bscan_incl<NT>(sum, sh, total);
  const uint32_t higher = total - incl;
  if (higher < k && k <= higher + sum) {
    uint32_t acc = higher;
#pragma unroll
    for (int i = BPT - 1; i >= 0; --i) {
      if (acc < k && k <= acc + loc[i]) { sh[32] = threadIdx.x * BPT + i; sh[33] = acc; }
      acc += loc[i];
    }
  }
  __syncthreads();
  bin = sh[32]; above = sh[33];
  __syncthreads();
}

// k-th largest of n 64-bit values produced by get(i), all distinct or not: returns the
// (shift, prefix) pair such that "value >> shift >= prefix" selects exactly the k largest when
// values are distinct (and every value tied with the k-th otherwise).  `bits` = width of the values.
template <int NT, typename Get>
__device__ __forceinline__ void radix_kth(Get get, uint32_t n, uint32_t k, int bits, uint32_t* bins,
                                          uint32_t* sh, int& shift_out, uint64_t& prefix_out) {
  int shift = bits;
  uint64_t prefix = 0;
  uint32_t remaining = k;
  while (shift > 0) {
    const int w = shift < 11 ? shift : 11;
    shift -= w;
    for (int b = threadIdx.x; b < 2048; b += NT) bins[b] = 0;
    __syncthreads();
    for (uint32_t i = threadIdx.x; i < n; i += NT) {
      const uint64_t v = get(i);
      if ((shift + w >= 64 ? 0ull : (v >> (shift + w))) == prefix)
        atomicAdd(&bins[(uint32_t)(v >> shift) & ((1u << w) - 1u)], 1u);
    }
    __syncthreads();
    uint32_t d, ab;
    kth_bin<NT>(bins, remaining, sh, d, ab);
    const uint32_t in_bin = bins[d];
    remaining -= ab;
    prefix = (prefix << w) | d;
    __syncthreads();
    if (in_bin == remaining) break;
  }
  shift_out = shift; prefix_out = prefix;
}

// ---- sample_threshold -------------------------------------------------------
// samp[(i*Hkv + h) * n_s + j]: sampled scores; thr[h*M + i] = rho-th largest (or -inf if rho > n_s).
__global__ __launch_bounds__(256) void sample_threshold_kernel(const float* __restrict__ samp,
                                                               int64_t n_s, uint32_t rho, int M,
                                                               int Hkv, float* thr) {
  __shared__ uint32_t bins[2048];
  __shared__ uint32_t sh[40];
  const int i = blockIdx.x, h = blockIdx.y;
  const float* row = samp + ((int64_t)i * Hkv + h) * n_s;
  float out = -__builtin_inff();
  if (rho <= n_s) {
    int shift; uint64_t prefix;
    radix_kth<256>([&](uint32_t j) -> uint64_t { return score_key(row[j]); }, (uint32_t)n_s, rho, 32,
                   bins, sh, shift, prefix);
    // smallest key with (key >> shift) == prefix is a lower bound of the rho-th largest
    const uint32_t key = (uint32_t)(prefix << shift);
    const uint32_t u = (key & 0x80000000u) ? (key & 0x7fffffffu) : ~key;
    out = __uint_as_float(u);
  }
  if (threadIdx.x == 0) thr[(int64_t)h * M + i] = out;
}

// ---- cand_topk ---------------------------------------------------------------
struct CandArgs {
  const uint2* cand; const uint32_t* ccount; uint32_t cap;
  int M, Hkv, k_eff; int64_t n_mid; int32_t index_base;
  int32_t* idx;              // [M][Hkv][k_eff]
  uint32_t* redo;            // redo[0] = count, redo[1..] = rows (h*M + i)
};

__device__ __forceinline__ uint64_t cand_composite(uint2 c) {
  return ((uint64_t)score_key(__uint_as_float(c.x)) << 32) | (uint64_t)(0xffffffffu - c.y);
}

__global__ __launch_bounds__(256) void cand_topk_kernel(CandArgs a) {
  extern __shared__ uint32_t bitmap[];            // ceil(n_mid / 32) words, rounded up to 256
  __shared__ uint32_t bins[2048];
  __shared__ uint32_t sh[40];
  const int i = blockIdx.x, h = blockIdx.y;
  const int64_t row = (int64_t)h * a.M + i;
  const uint32_t n_all = a.ccount[row];
  if (n_all < (uint32_t)a.k_eff || n_all > a.cap) {
    if (threadIdx.x == 0) {
      const uint32_t at = atomicAdd(&a.redo[0], 1u);
      a.redo[1 + at] = (uint32_t)row;
    }
    return;
  }
  const uint2* seg = a.cand + row * a.cap;
  const uint32_t n = n_all;
  int shift = 0; uint64_t prefix = 0;
  if ((uint32_t)a.k_eff < n)
    radix_kth<256>([&](uint32_t j) -> uint64_t { return cand_composite(seg[j]); }, n,
                   (uint32_t)a.k_eff, 64, bins, sh, shift, prefix);
  const int nwords = (int)((a.n_mid + 31) / 32);
  const int nwords_pad = (nwords + 255) / 256 * 256;
  for (int w = threadIdx.x; w < nwords_pad; w += 256) bitmap[w] = 0;
  __syncthreads();
  for (uint32_t j = threadIdx.x; j < n; j += 256) {
    const uint2 c = seg[j];
    if ((shift >= 64 ? 0ull : (cand_composite(c) >> shift)) >= prefix)
      atomicOr(&bitmap[c.y >> 5], 1u << (c.y & 31));
  }
  __syncthreads();
  // ordered compaction: thread t owns words [t*wpt, (t+1)*wpt)
  const int wpt = nwords_pad / 256;
  uint32_t mine = 0;
  for (int w = 0; w < wpt; ++w) mine += __popc(bitmap[threadIdx.x * wpt + w]);
  uint32_t total;
  uint32_t at = bscan_incl<256>(mine, sh, total) - mine;
  int32_t* out = a.idx + ((int64_t)i * a.Hkv + h) * a.k_eff;
  for (int w = 0; w < wpt; ++w) {
    uint32_t bits = bitmap[threadIdx.x * wpt + w];
    const int32_t first = a.index_base + (threadIdx.x * wpt + w) * 32;
    while (bits) {
      const int b = __ffs((int)bits) - 1;
      bits &= bits - 1;
      if (at < (uint32_t)a.k_eff) out[at] = first + b;
      ++at;
    }
  }
}

// ---- row_exact (redo path) ----------------------------------------------------
struct ExactArgs {
  const uint16_t* q; const uint16_t* k;
  int64_t ksh, kst, first_tok, n_mid;
  int M, Hq, Hkv, G, k_eff; int32_t index_base;
  const uint32_t* redo;
  float* scratch;            // [gridDim.x][n_mid] scores
  int32_t* idx;
};

__global__ __launch_bounds__(1024) void row_exact_kernel(ExactArgs a) {
  __shared__ uint32_t bins[2048];
  __shared__ uint32_t sh[40];
  const uint32_t n_redo = a.redo[0];
  float* sc = a.scratch + (int64_t)blockIdx.x * a.n_mid;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int sub = lane & 15, grp = lane >> 4;
  for (uint32_t e = blockIdx.x; e < n_redo; e += gridDim.x) {
    const uint32_t row = a.redo[1 + e];
    const int h = (int)(row / a.M), i = (int)(row % a.M);
    // scores with the streaming kernel's arithmetic: fp32 group sum, 16 lanes per 256-byte key row
    float qv[8];
#pragma unroll
    for (int c = 0; c < 8; ++c) qv[c] = 0.f;
    for (int g = 0; g < a.G; ++g) {
      const uint16_t* qr = a.q + ((int64_t)i * a.Hq + (int64_t)h * a.G + g) * 128 + sub * 8;
#pragma unroll
      for (int c = 0; c < 8; ++c) qv[c] += __uint_as_float(((uint32_t)qr[c]) << 16);
    }
    const uint16_t* kb = a.k + (int64_t)h * a.ksh + a.first_tok * a.kst + sub * 8;
    for (int64_t j0 = (int64_t)wave * 4; j0 < a.n_mid; j0 += 64) {
      int64_t j = j0 + grp;
      const int64_t jc = j < a.n_mid ? j : a.n_mid - 1;
      const u32x4 d = *(const u32x4*)(kb + jc * a.kst);
      float s = 0.f;
      s = fmaf(bf16_lo(d.x), qv[0], s); s = fmaf(bf16_hi(d.x), qv[1], s);
      s = fmaf(bf16_lo(d.y), qv[2], s); s = fmaf(bf16_hi(d.y), qv[3], s);
      s = fmaf(bf16_lo(d.z), qv[4], s); s = fmaf(bf16_hi(d.z), qv[5], s);
      s = fmaf(bf16_lo(d.w), qv[6], s); s = fmaf(bf16_hi(d.w), qv[7], s);
      s = group_sum<16>(s);
      if (sub == 0 && j < a.n_mid) sc[j] = s;
    }
    __threadfence_block();
    __syncthreads();
    // exact k-th largest composite (score desc, index asc) over the whole row
    int shift = 0; uint64_t prefix = 0;
    if ((int64_t)a.k_eff < a.n_mid)
      radix_kth<1024>([&](uint32_t j) -> uint64_t {
                        return ((uint64_t)score_key(sc[j]) << 32) | (uint64_t)(0xffffffffu - j);
                      }, (uint32_t)a.n_mid, (uint32_t)a.k_eff, 64, bins, sh, shift, prefix);
    // ordered emit
    int32_t* out = a.idx + ((int64_t)i * a.Hkv + h) * a.k_eff;
    uint32_t done = 0;
    for (int64_t j0 = 0; j0 < a.n_mid; j0 += 1024) {
      const int64_t j = j0 + threadIdx.x;
      uint32_t take = 0;
      if (j < a.n_mid) {
        const uint64_t v = ((uint64_t)score_key(sc[j]) << 32) | (uint64_t)(0xffffffffu - (uint32_t)j);
        take = (shift >= 64 ? 0ull : (v >> shift)) >= prefix ? 1u : 0u;
      }
      uint32_t total;
      const uint32_t at = done + bscan_incl<1024>(take, sh, total) - take;
      if (take && at < (uint32_t)a.k_eff) out[at] = a.index_base + (int32_t)j;
      done += total;
    }
    __syncthreads();
  }
}

}  // namespace

// Sampling plan shared by the host side: stride, sample size, rank and segment capacity.
void prefill_sampling(const Plan& pl, int64_t* stride, int64_t* n_s, uint32_t* rho, uint32_t* cap) {
  int64_t st = pl.n_mid / 8192;
  if (st < 1) st = 1;
  const int64_t ns = (pl.n_mid + st - 1) / st;
  const double p = (double)pl.k_eff / (double)pl.n_mid;
  const double mu = (double)ns * p;
  double r = mu + 6.0 * sqrt(mu * (1.0 - p) + 1.0) + 2.0;
  if (st == 1) r = (double)pl.k_eff;                     // the "sample" is every key: exact rank
  if (r > (double)ns) r = (double)ns + 1.0;               // take everything
  const double expect = r * (double)st;
  double c = expect * (1.0 + 6.0 / sqrt(r)) + 64.0;
  if (c > (double)pl.n_mid) c = (double)pl.n_mid;
  if (c < (double)pl.k_eff) c = (double)pl.k_eff;
  *stride = st; *n_s = ns; *rho = (uint32_t)r; *cap = (uint32_t)c;
}

hipError_t launch_sample_threshold(const Plan& pl, int n_query, const float* samp, int64_t n_s,
                                   uint32_t rho, float* thr, hipStream_t st) {
  hipLaunchKernelGGL(sample_threshold_kernel, dim3(n_query, pl.Hkv), dim3(256), 0, st, samp, n_s, rho,
                     n_query, pl.Hkv, thr);
  return hipGetLastError();
}

size_t cand_topk_lds(const Plan& pl) {
  const size_t nwords = (size_t)((pl.n_mid + 31) / 32);
  return (nwords + 255) / 256 * 256 * 4;
}

hipError_t launch_cand_topk(const Plan& pl, int n_query, const uint2* cand, const uint32_t* ccount,
                            uint32_t cap, int32_t* idx, uint32_t* redo, hipStream_t st) {
  CandArgs a;
  a.cand = cand; a.ccount = ccount; a.cap = cap; a.M = n_query; a.Hkv = pl.Hkv; a.k_eff = pl.k_eff;
  a.n_mid = pl.n_mid; a.index_base = (int32_t)pl.s_eff; a.idx = idx; a.redo = redo;
  const size_t lds = cand_topk_lds(pl);
  // set on every launch: the attribute belongs to the current device, and nothing is remembered between calls
  hipError_t e = hipFuncSetAttribute((const void*)cand_topk_kernel,
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(cand_topk_kernel, dim3(n_query, pl.Hkv), dim3(256), lds, st, a);
  return hipGetLastError();
}

hipError_t launch_row_exact(const Plan& pl, int n_query, const void* q, const void* k_cache,
                            const uint32_t* redo, float* scratch, int n_slots, int32_t* idx,
                            hipStream_t st) {
  ExactArgs a;
  a.q = (const uint16_t*)q; a.k = (const uint16_t*)k_cache;
  a.ksh = pl.ksh; a.kst = pl.kst; a.first_tok = pl.s_eff; a.n_mid = pl.n_mid;
  a.M = n_query; a.Hq = pl.Hq; a.Hkv = pl.Hkv; a.G = pl.G; a.k_eff = pl.k_eff;
  a.index_base = (int32_t)pl.s_eff; a.redo = redo; a.scratch = scratch; a.idx = idx;
  hipLaunchKernelGGL(row_exact_kernel, dim3(n_slots), dim3(1024), 0, st, a);
  return hipGetLastError();
}

}  // namespace reattn
