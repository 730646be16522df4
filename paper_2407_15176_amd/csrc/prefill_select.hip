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
#include "select.hpp"

namespace reattn {
namespace {

// ---- sample_threshold -------------------------------------------------------
// samp[(i*Hkv + h) * row_stride + j], j < n_s: sampled scores; thr[h*M + i] = a lower bound of the rho-th
// largest, at most 2^-22 of the row's key range below it (or -inf if rho > n_s).  The row is read once
// into registers (n_s <= 256 * R); the radix select walks the significant bits of the offsets from the
// row's smallest ordered key, 11 at a time, and stops after two passes: the bits left undecided only
// lower the bound, by less than any two distinct scores of the distribution differ.
template <int R>
__global__ __launch_bounds__(256) void sample_threshold_kernel(const float* __restrict__ samp, int64_t n_s,
                                                               int64_t row_stride, uint32_t rho, int M,
                                                               int Hkv, float* thr) {
  __shared__ uint32_t bins[kBinsPad];
  __shared__ uint32_t sh[40];
  const int i = blockIdx.x, h = blockIdx.y;
  const float* row = samp + ((int64_t)i * Hkv + h) * row_stride;
  if (rho > n_s) {
    if (threadIdx.x == 0) thr[(int64_t)h * M + i] = -__builtin_inff();
    return;
  }
  const uint32_t n = (uint32_t)n_s;
  uint32_t key[R];
  uint32_t kmin = 0xffffffffu, kmax = 0u;
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const uint32_t j = (uint32_t)r * 256u + threadIdx.x;
    key[r] = __float_as_uint(row[j < n ? j : n - 1]);        // clamped, not predicated: all loads go out before the first wait
  }
#pragma unroll
  for (int r = 0; r < R; ++r) {
    key[r] = score_key(__uint_as_float(key[r]));
    if ((uint32_t)r * 256u + threadIdx.x < n) { kmin = min(kmin, key[r]); kmax = max(kmax, key[r]); }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    kmin = min(kmin, (uint32_t)__shfl_xor((int)kmin, o, 64));
    kmax = max(kmax, (uint32_t)__shfl_xor((int)kmax, o, 64));
  }
  if ((threadIdx.x & 63) == 0) { sh[34 + (threadIdx.x >> 6)] = kmin; sh[30 + (threadIdx.x >> 6)] = kmax; }
  __syncthreads();
  kmin = min(min(sh[34], sh[35]), min(sh[36], sh[37]));
  kmax = max(max(sh[30], sh[31]), max(sh[32], sh[33]));
  __syncthreads();
  // The rho-th largest of a few thousand samples lies in the top few percent, so the select is run on a
  // window below the maximum: keys down to an eighth of the largest score (three exponent steps; the
  // ordered key of a positive float is its bit pattern with the sign set).  Over the whole row the first
  // digits are sign and exponent, which put thousands of samples into a handful of bins: LDS atomics on
  // one address serialise, and that was most of this kernel's time.  A row whose window holds fewer than
  // rho samples (outliers far above the bulk) falls back to the whole range.
  uint32_t cut = kmin;
  if (kmax >= 0x80000000u + (4u << 23)) {
    const uint32_t c = kmax - (3u << 23);
    uint32_t in = 0;
#pragma unroll
    for (int r = 0; r < R; ++r) in += ((uint32_t)r * 256u + threadIdx.x < n && key[r] >= c) ? 1u : 0u;
    uint32_t total;
    block_scan_incl<256>(in, sh, total);
    if (total >= rho) cut = c;                                 // workgroup-uniform
  }
  int dsh = 32 - __clz((int)(kmax - cut));
  uint32_t dpref = 0, remaining = rho;
  for (int p = 0; p < 2 && dsh > 0; ++p) {
    const int w = dsh < 11 ? dsh : 11;
    dsh -= w;
    for (int b = threadIdx.x; b < kBinsPad; b += 256) bins[b] = 0;
    __syncthreads();
    const int up = dsh + w;
#pragma unroll
    for (int r = 0; r < R; ++r) {
      if ((uint32_t)r * 256u + threadIdx.x < n && key[r] >= cut) {
        const uint32_t d = key[r] - cut;
        if (up >= 32 || (d >> up) == dpref) atomicAdd(&bins[bslot((int)((d >> dsh) & ((1u << w) - 1u)))], 1u);
      }
    }
    __syncthreads();
    uint32_t d, ab;
    kth_bin<256>(bins, remaining, sh, d, ab);
    remaining -= ab;
    dpref = (dpref << w) | d;
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    // smallest key that shares the decided prefix: a lower bound of the rho-th largest
    const uint32_t k = cut + (dsh >= 32 ? 0u : (dpref << dsh));
    const uint32_t u = (k & 0x80000000u) ? (k & 0x7fffffffu) : ~k;
    thr[(int64_t)h * M + i] = __uint_as_float(u);
  }
}

// ---- cand_topk ---------------------------------------------------------------
struct CandArgs {
  const uint2* cand; const uint32_t* ccount; uint32_t cap;   // row r: n_split parts of cap entries, counts ccount[r * n_split + z]
  int n_split;
  int M, Hkv, k_eff; int64_t n_mid; int32_t index_base;
  int32_t* idx;              // [M][Hkv][k_eff]
  uint32_t* redo;            // redo[0] = count, redo[1..] = rows (h*M + i)
};

__device__ __forceinline__ uint64_t cand_composite(uint2 c) {
  return ((uint64_t)score_key(__uint_as_float(c.x)) << 32) | (uint64_t)(0xffffffffu - c.y);
}

__global__ __launch_bounds__(256) void cand_topk_kernel(CandArgs a) {
  extern __shared__ uint32_t bitmap[];            // ceil(n_mid / 32) words, rounded up to 256
  __shared__ uint32_t bins[kBinsPad];
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
  uint32_t at = block_scan_incl<256>(mine, sh, total) - mine;
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

// The same selection with the row's candidates held in registers (segments of up to 256 * R entries):
// the segment is read once instead of once per radix pass, and its loads are issued before anything
// waits (not even for the row's count: slots past it are read and ignored).  Every candidate passed the
// row's threshold, so the ordered score keys span a narrow range above the smallest one; the radix
// select runs on the 32-bit offsets d from that smallest key, whose significant bits alone are walked
// (typically two passes of 11 bits settle the k-th entry), and only a tie on d goes on to the key
// index (lower first, as everywhere).  Winners are marked in an LDS bitmap over the middle; every
// thread then takes its 32 consecutive bitmap words into registers, ranks them with one block scan and
// writes the indices, in order, into LDS (over the spent bitmap), from where they leave in 16-byte
// rows: written straight from the ranking loop, every lane of a store would touch its own cache line.
constexpr int kRankWords = 32;                   // bitmap words a thread can rank out of registers

template <int R>
__global__ __launch_bounds__(256, 3) void cand_topk_reg_kernel(CandArgs a) {
  extern __shared__ uint32_t bitmap[];            // wslot(nwords_pad) words; later the ranked indices
  __shared__ uint32_t bins[kBinsPad];
  __shared__ uint32_t sh[40];
  const int i = blockIdx.x, h = blockIdx.y;
  const int64_t row = (int64_t)h * a.M + i;
  static_assert(R % 2 == 0, "candidates are loaded in pairs");
  // The row's candidates sit in n_split parts (one per key split of the filter), part z holding cnt[z] of
  // them.  Two candidates per 16-byte load (parts start 16-byte aligned: the capacity is even); the parts'
  // pairs are numbered through, pair j of the row goes to register slots 2j', 2j'+1 of thread j % 256.  Only
  // the row's own entries are fetched: pairs past them repeat the last one (clamped, not predicated: all
  // loads go out before the first wait).  valid: bit r set when register slot r holds a candidate.
  __shared__ uint32_t s_first[9], s_cnt[8];                  // first pair of each part; its count
  if (threadIdx.x == 0) {
    const uint32_t* cnt = a.ccount + row * a.n_split;
    uint32_t pairs = 0, total = 0, over = 0;
    for (int z = 0; z < a.n_split; ++z) {
      const uint32_t c = cnt[z];
      over |= c > a.cap ? 1u : 0u;
      s_first[z] = pairs; s_cnt[z] = c;
      pairs += (c + 1) >> 1; total += c;
    }
    s_first[8] = pairs;
    sh[0] = total; sh[1] = over;
  }
  __syncthreads();
  const uint32_t n = sh[0], n_pair = s_first[8];
  if (sh[1] || n < (uint32_t)a.k_eff || n_pair > 256u * (R / 2) || n == 0) {
    if (threadIdx.x == 0 && (sh[1] || n < (uint32_t)a.k_eff || n_pair > 256u * (R / 2))) {
      const uint32_t at = atomicAdd(&a.redo[0], 1u);
      a.redo[1 + at] = (uint32_t)row;
    }
    return;
  }
  const uint4* seg = (const uint4*)(a.cand + row * a.n_split * a.cap);
  const uint32_t part_pairs = a.cap >> 1;
  uint32_t key[R], pos[R];
  uint64_t valid = 0;
  uint32_t pfirst[8], pcnt[8];                               // the parts' first pairs and counts, in registers
#pragma unroll
  for (int z = 0; z < 8; ++z) {
    pfirst[z] = z < a.n_split ? s_first[z] : 0xffffffffu;    // no pair reaches a part that is not there
    pcnt[z] = z < a.n_split ? s_cnt[z] : 0u;
  }
#pragma unroll
  for (int r2 = 0; r2 < R / 2; ++r2) {
    const uint32_t j = (uint32_t)r2 * 256u + threadIdx.x;
    const uint32_t jc = j < n_pair ? j : n_pair - 1;
    uint32_t first = 0, cnt = pcnt[0], part = 0;
    if (a.n_split > 1) {                                     // the last part that starts at or before pair jc
#pragma unroll
      for (int z = 1; z < 8; ++z) {
        const bool at = jc >= pfirst[z];
        first = at ? pfirst[z] : first; cnt = at ? pcnt[z] : cnt; part = at ? (uint32_t)z : part;
      }
    }
    const uint32_t local = jc - first;
    const uint4 c = seg[part * part_pairs + local];
    key[2 * r2] = c.x; pos[2 * r2] = c.y; key[2 * r2 + 1] = c.z; pos[2 * r2 + 1] = c.w;
    if (j < n_pair) {
      if (2 * local < cnt) valid |= 1ull << (2 * r2);
      if (2 * local + 1 < cnt) valid |= 1ull << (2 * r2 + 1);
    }
  }
  auto live = [&](int r) -> bool { return (valid >> r) & 1ull; };
  __syncthreads();                                           // sh is reused below
  const int nwords = (int)((a.n_mid + 31) / 32);
  const int nwords_pad = (nwords + 255) / 256 * 256;
  const int nslots = wslot(nwords_pad);
  for (int w = threadIdx.x; w < nslots; w += 256) bitmap[w] = 0;     // while the loads are in flight
  uint32_t kmin = 0xffffffffu, kmax = 0u;
#pragma unroll
  for (int r = 0; r < R; ++r) {
    key[r] = score_key(__uint_as_float(key[r]));
    if (live(r)) { kmin = min(kmin, key[r]); kmax = max(kmax, key[r]); }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    kmin = min(kmin, (uint32_t)__shfl_xor((int)kmin, o, 64));
    kmax = max(kmax, (uint32_t)__shfl_xor((int)kmax, o, 64));
  }
  if ((threadIdx.x & 63) == 0) { sh[34 + (threadIdx.x >> 6)] = kmin; sh[30 + (threadIdx.x >> 6)] = kmax; }
  __syncthreads();
  kmin = min(min(sh[34], sh[35]), min(sh[36], sh[37]));
  kmax = max(max(sh[30], sh[31]), max(sh[32], sh[33]));
  __syncthreads();
  const int nbits = 32 - __clz((int)(kmax - kmin));          // significant bits of the offsets (0 when all keys are equal)
#pragma unroll
  for (int r = 0; r < R; ++r) { key[r] -= kmin; pos[r] = ~pos[r]; }   // d, and the index as a descending key

  // Winners: in the offset part, d >> dsh >= dpref; once a tie on d = dpref had to be broken,
  // d > dpref, or d == dpref and ~index >> psh >= ppref.
  bool all = (uint32_t)a.k_eff == n, tie = false;
  uint32_t dpref = 0, ppref = 0;
  int dsh = nbits, psh = 32;
  if (!all) {
    uint32_t remaining = (uint32_t)a.k_eff;
    bool done = false;
    auto pass = [&](bool on_index, int sft, int w) {
      for (int b = threadIdx.x; b < kBinsPad; b += 256) bins[b] = 0;
      __syncthreads();
      const int up = sft + w;                                // up == 32 only on a first pass: no prefix yet
#pragma unroll
      for (int r = 0; r < R; ++r) {
        if (live(r)) {
          const uint32_t v = on_index ? pos[r] : key[r];
          const bool in = (up >= 32 || (v >> up) == (on_index ? ppref : dpref)) && (!on_index || key[r] == dpref);
          if (in) atomicAdd(&bins[bslot((int)((v >> sft) & ((1u << w) - 1u)))], 1u);
        }
      }
      __syncthreads();
      uint32_t d, ab;
      kth_bin<256>(bins, remaining, sh, d, ab);
      const uint32_t in_bin = bins[bslot((int)d)];
      remaining -= ab;
      if (on_index) ppref = (ppref << w) | d; else dpref = (dpref << w) | d;
      __syncthreads();
      done = in_bin == remaining;                            // everything that shares this prefix is selected
    };
    while (dsh > 0 && !done) {
      const int w = dsh < 11 ? dsh : 11;
      dsh -= w;
      pass(false, dsh, w);
    }
    if (!done) {                                             // dpref is the k-th entry's d: the tie ends on the index
      tie = true;
      while (psh > 0 && !done) {
        const int w = psh < 11 ? psh : 11;
        psh -= w;
        pass(true, psh, w);
      }
    }
  }
#pragma unroll
  for (int r = 0; r < R; ++r) {
    if (live(r)) {
      const bool win = all || (tie ? (key[r] > dpref || (key[r] == dpref && (pos[r] >> psh) >= ppref))
                                   : (dsh >= 32 || (key[r] >> dsh) >= dpref));
      const uint32_t p = ~pos[r];
      if (win) atomicOr(&bitmap[wslot((int)(p >> 5))], 1u << (p & 31));
    }
  }
  __syncthreads();
  // ordered compaction: thread t owns words [t*wpt, (t+1)*wpt)
  const int wpt = nwords_pad / 256;
  int32_t* out = a.idx + ((int64_t)i * a.Hkv + h) * a.k_eff;
  uint32_t total;
  if (wpt <= kRankWords) {
    uint32_t word[kRankWords];
    uint32_t mine = 0;
#pragma unroll
    for (int w = 0; w < kRankWords; ++w) {
      word[w] = w < wpt ? bitmap[wslot(threadIdx.x * wpt + w)] : 0u;
      mine += __popc(word[w]);
    }
    uint32_t at = block_scan_incl<256>(mine, sh, total) - mine;   // its barriers also end every read of the bitmap
    int32_t* ranked = (int32_t*)bitmap;                      // [k_eff]
#pragma unroll
    for (int w = 0; w < kRankWords; ++w) {
      uint32_t bits = word[w];
      const int32_t first = a.index_base + (threadIdx.x * wpt + w) * 32;
      while (bits) {
        const int b = __ffs((int)bits) - 1;
        bits &= bits - 1;
        if (at < (uint32_t)a.k_eff) ranked[at] = first + b;
        ++at;
      }
    }
    __syncthreads();
    if ((a.k_eff & 3) == 0 && ((uintptr_t)a.idx & 15) == 0) {
      for (int j = threadIdx.x; j < a.k_eff / 4; j += 256) ((int4*)out)[j] = ((const int4*)ranked)[j];
    } else {
      for (int j = threadIdx.x; j < a.k_eff; j += 256) out[j] = ranked[j];
    }
  } else {                                                   // a long middle: ranked from LDS, written directly
    uint32_t mine = 0;
    for (int w = 0; w < wpt; ++w) mine += __popc(bitmap[wslot(threadIdx.x * wpt + w)]);
    uint32_t at = block_scan_incl<256>(mine, sh, total) - mine;
    for (int w = 0; w < wpt; ++w) {
      uint32_t bits = bitmap[wslot(threadIdx.x * wpt + w)];
      const int32_t first = a.index_base + (threadIdx.x * wpt + w) * 32;
      while (bits) {
        const int b = __ffs((int)bits) - 1;
        bits &= bits - 1;
        if (at < (uint32_t)a.k_eff) out[at] = first + b;
        ++at;
      }
    }
  }
}

// ---- row_exact (redo path) ----------------------------------------------------
struct ExactArgs {
  const uint16_t* q; const uint16_t* k;
  int64_t ksh, kst, first_tok, n_mid;
  const int32_t* pt; int page_lg;   // paged cache (nullptr: none)
  int M, Hq, Hkv, G, k_eff; int32_t index_base;
  const uint32_t* redo;
  float* scratch;            // [gridDim.x][n_mid] scores
  int32_t* idx;
};

template <bool F16>
__global__ __launch_bounds__(1024) void row_exact_kernel(ExactArgs a) {
  __shared__ uint32_t bins[kBinsPad];
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
      for (int c = 0; c < 8; ++c) qv[c] += Mm<F16>::widen(qr[c]);
    }
    const uint16_t* kb = a.k + (int64_t)h * a.ksh + (a.pt ? 0 : a.first_tok) * a.kst + sub * 8;
    for (int64_t j0 = (int64_t)wave * 4; j0 < a.n_mid; j0 += 64) {
      int64_t j = j0 + grp;
      const int64_t jc = j < a.n_mid ? j : a.n_mid - 1;
      const int64_t krow = a.pt ? paged_row(a.pt, a.page_lg, a.first_tok + jc) : jc;
      const u32x4 d = *(const u32x4*)(kb + krow * a.kst);
      float s = 0.f;
      const uint32_t dw[4] = {d.x, d.y, d.z, d.w};
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        s = fmaf(F16 ? f16_lo(dw[c]) : bf16_lo(dw[c]), qv[2 * c], s);
        s = fmaf(F16 ? f16_hi(dw[c]) : bf16_hi(dw[c]), qv[2 * c + 1], s);
      }
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
      const uint32_t at = done + block_scan_incl<1024>(take, sh, total) - take;
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
  *stride = st; *n_s = ns; *rho = (uint32_t)r; *cap = ((uint32_t)c + 1u) & ~1u;   // even: 16-byte segment starts
}

void prefill_filter_splits(const Plan& pl, uint32_t cap, int* n_split, uint32_t* cap_split) {
  const int64_t wgs = (int64_t)pl.Hkv * ((pl.M + 127) / 128);       // workgroups of the filter without a key split
  const int64_t n_tiles = (pl.n_mid + 127) / 128;
  int64_t z = 1;
  if (wgs < 256 && cap <= 256u * 40u) {                  // the register kernel reads the parts; its limit is 8
    z = (256 + wgs - 1) / wgs;
    if (z > 8) z = 8;
    if (z > n_tiles) z = n_tiles;
    if (z < 1) z = 1;
    const int64_t per = (n_tiles + z - 1) / z;           // tiles per split; the last split may be shorter
    z = (n_tiles + per - 1) / per;
  }
  // candidates are not spread evenly over the keys: a part takes three times its even share (a row that
  // overflows one goes to the exact redo)
  uint64_t c = cap;
  if (z > 3) c = ((uint64_t)3 * cap + z - 1) / z;
  *n_split = (int)z;
  *cap_split = ((uint32_t)c + 1u) & ~1u;
}

hipError_t launch_sample_threshold(const Plan& pl, int n_query, const float* samp, int64_t n_s,
                                   int64_t row_stride, uint32_t rho, float* thr, hipStream_t st) {
  // the sample of prefill_sampling() is shorter than 2 * 8192 keys
  if (n_s > 256 * 64) return hipErrorInvalidValue;
  if (n_s <= 256 * 36)
    hipLaunchKernelGGL(sample_threshold_kernel<36>, dim3(n_query, pl.Hkv), dim3(256), 0, st, samp, n_s,
                       row_stride, rho, n_query, pl.Hkv, thr);
  else
    hipLaunchKernelGGL(sample_threshold_kernel<64>, dim3(n_query, pl.Hkv), dim3(256), 0, st, samp, n_s,
                       row_stride, rho, n_query, pl.Hkv, thr);
  return hipGetLastError();
}

size_t cand_topk_lds(const Plan& pl) {                     // selection bitmap over the middle + the ranked indices
  const size_t nwords = (size_t)((pl.n_mid + 31) / 32);
  const size_t padded = (nwords + 255) / 256 * 256;
  const size_t bitmap = (padded + padded / 32 + 4) * 4;
  const size_t ranked = (size_t)pl.k_eff * 4;                // written over the bitmap once it is in registers
  return bitmap > ranked ? bitmap : ranked;
}

hipError_t launch_cand_topk(const Plan& pl, int n_query, const uint2* cand, const uint32_t* ccount,
                            uint32_t cap, int n_split, int32_t* idx, uint32_t* redo, hipStream_t st) {
  CandArgs a;
  a.cand = cand; a.ccount = ccount; a.cap = cap; a.n_split = n_split < 1 ? 1 : n_split;
  a.M = n_query; a.Hkv = pl.Hkv; a.k_eff = pl.k_eff;
  a.n_mid = pl.n_mid; a.index_base = (int32_t)pl.s_eff; a.idx = idx; a.redo = redo;
  const size_t lds = cand_topk_lds(pl);
  // set on every launch: the attribute belongs to the current device, and nothing is remembered between calls
  constexpr int kRegs = 40;                               // segments of up to 10,240 candidates stay in registers
  if (a.n_split > 1 && (a.n_split > 8 || cap > 256u * kRegs)) return hipErrorInvalidValue;   // splits are read by the register kernel only
  auto kern = cap <= 256u * kRegs ? cand_topk_reg_kernel<kRegs> : cand_topk_kernel;
  hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, dim3(n_query, pl.Hkv), dim3(256), lds, st, a);
  return hipGetLastError();
}

hipError_t launch_row_exact(const Plan& pl, int n_query, const void* q, const void* k_cache,
                            const uint32_t* redo, float* scratch, int n_slots, int32_t* idx,
                            hipStream_t st) {
  ExactArgs a;
  a.q = (const uint16_t*)q; a.k = (const uint16_t*)k_cache;
  a.ksh = pl.ksh; a.kst = pl.kst; a.first_tok = pl.s_eff; a.n_mid = pl.n_mid; a.pt = pl.pt; a.page_lg = pl.page_lg;
  a.M = n_query; a.Hq = pl.Hq; a.Hkv = pl.Hkv; a.G = pl.G; a.k_eff = pl.k_eff;
  a.index_base = (int32_t)pl.s_eff; a.redo = redo; a.scratch = scratch; a.idx = idx;
  if (pl.dtype == kF16) hipLaunchKernelGGL(row_exact_kernel<true>, dim3(n_slots), dim3(1024), 0, st, a);
  else hipLaunchKernelGGL(row_exact_kernel<false>, dim3(n_slots), dim3(1024), 0, st, a);
  return hipGetLastError();
}

}  // namespace reattn
