// Device helpers shared by the selection kernels (paper Eq. 2, `Indices = top-k(q K_middle^T)`):
// radix selection with LDS histograms, the lower bound of a row's k-th score taken from a strided
// sample of its scores, and the storage-type widening of the streaming kernels.
#pragma once

#include "common.hpp"

namespace reattn {
#ifdef __HIPCC__

// ---- stored elements -> fp32, one 16-byte load at a time -------------------------------------
template <typename T> struct Store;
template <> struct Store<float> {
  static constexpr int kPerLoad = 4;
  static __device__ __forceinline__ void widen(const u32x4& d, float* x) {
    x[0] = __uint_as_float(d.x); x[1] = __uint_as_float(d.y);
    x[2] = __uint_as_float(d.z); x[3] = __uint_as_float(d.w);
  }
  static __device__ __forceinline__ float one(const void* p, int64_t i) { return ((const float*)p)[i]; }
};
template <> struct Store<uint16_t> {   // bf16 bit patterns
  static constexpr int kPerLoad = 8;
  static __device__ __forceinline__ void widen(const u32x4& d, float* x) {
    x[0] = bf16_lo(d.x); x[1] = bf16_hi(d.x); x[2] = bf16_lo(d.y); x[3] = bf16_hi(d.y);
    x[4] = bf16_lo(d.z); x[5] = bf16_hi(d.z); x[6] = bf16_lo(d.w); x[7] = bf16_hi(d.w);
  }
  static __device__ __forceinline__ float one(const void* p, int64_t i) {
    return __uint_as_float(((uint32_t)((const uint16_t*)p)[i]) << 16);
  }
};
template <> struct Store<f16bits> {    // IEEE half bit patterns
  static constexpr int kPerLoad = 8;
  static __device__ __forceinline__ void widen(const u32x4& d, float* x) {
    x[0] = f16_lo(d.x); x[1] = f16_hi(d.x); x[2] = f16_lo(d.y); x[3] = f16_hi(d.y);
    x[4] = f16_lo(d.z); x[5] = f16_hi(d.z); x[6] = f16_lo(d.w); x[7] = f16_hi(d.w);
  }
  static __device__ __forceinline__ float one(const void* p, int64_t i) { return f16_one(((const uint16_t*)p)[i]); }
};

// The group's query rows summed in fp32 (sum_g (q_g . k) = (sum_g q_g) . k): the EPL channels
// [sub * EPL, sub * EPL + EPL) of score row (qi, h).
template <typename T, int D>
__device__ __forceinline__ void group_query(const void* q, int qi, int h, int Hq, int G, int sub, float* qv) {
  constexpr int EPL = Store<T>::kPerLoad;
#pragma unroll
  for (int e = 0; e < EPL; ++e) qv[e] = 0.f;
  for (int g = 0; g < G; ++g) {
    const int64_t qoff = ((int64_t)qi * Hq + (int64_t)h * G + g) * D + sub * EPL;
#pragma unroll
    for (int e = 0; e < EPL; ++e) qv[e] += Store<T>::one(q, qoff + e);
  }
}

// One key row's share of the dot product held by this lane, summed over the D / EPL lanes of the row.
template <typename T, int D>
__device__ __forceinline__ float row_dot(const u32x4& d, const float* qv) {
  constexpr int EPL = Store<T>::kPerLoad;
  float x[EPL];
  Store<T>::widen(d, x);
  float s = 0.f;
#pragma unroll
  for (int e = 0; e < EPL; ++e) s = fmaf(x[e], qv[e], s);
  return group_sum<D / EPL>(s);
}

// Max aggregation (REATTN_AGG_MAX): the score of a key is the largest of its G per-head dot products, so the
// heads cannot be summed first.  The group's query rows sit in LDS as fp32, qs[g * D + c].
template <typename T, int D>
__device__ __forceinline__ void group_rows_to_lds(const void* q, int qi, int h, int Hq, int G, float* qs, int n_threads) {
  const int64_t q0 = ((int64_t)qi * Hq + (int64_t)h * G) * D;
  for (int i = threadIdx.x; i < G * D; i += n_threads) qs[i] = Store<T>::one(q, q0 + i);
}
template <typename T, int D>
__device__ __forceinline__ float row_dot_max(const u32x4& d, const float* qs, int G, int sub) {
  constexpr int EPL = Store<T>::kPerLoad;
  float x[EPL];
  Store<T>::widen(d, x);
  float best = 0.f;
  for (int g = 0; g < G; ++g) {
    const float* qg = qs + g * D + sub * EPL;
    float s = 0.f;
#pragma unroll
    for (int e = 0; e < EPL; ++e) s = fmaf(x[e], qg[e], s);
    s = group_sum<D / EPL>(s);
    best = g == 0 ? s : fmaxf(best, s);
  }
  return best;
}

// The same out of registers for groups of up to four heads (the usual GQA groups): qr[g][e], rows past G unused.
template <typename T, int D>
__device__ __forceinline__ void group_rows_to_regs(const void* q, int qi, int h, int Hq, int G, int sub, float (*qr)[Store<T>::kPerLoad]) {
  constexpr int EPL = Store<T>::kPerLoad;
#pragma unroll
  for (int g = 0; g < 4; ++g) {
    const int gg = g < G ? g : G - 1;
    const int64_t qoff = ((int64_t)qi * Hq + (int64_t)h * G + gg) * D + sub * EPL;
#pragma unroll
    for (int e = 0; e < EPL; ++e) qr[g][e] = Store<T>::one(q, qoff + e);
  }
}
template <typename T, int D>
__device__ __forceinline__ float row_dot_max4(const u32x4& d, const float (*qr)[Store<T>::kPerLoad]) {
  constexpr int EPL = Store<T>::kPerLoad;
  float x[EPL];
  Store<T>::widen(d, x);
  float best = 0.f;
#pragma unroll
  for (int g = 0; g < 4; ++g) {                      // rows past G repeat the last head: the maximum does not change
    float s = 0.f;
#pragma unroll
    for (int e = 0; e < EPL; ++e) s = fmaf(x[e], qr[g][e], s);
    s = group_sum<D / EPL>(s);
    best = g == 0 ? s : fmaxf(best, s);
  }
  return best;
}

// ---- LDS histograms of 2048 bins -----------------------------------------------------------------
// A thread that owns consecutive bins (or 32 consecutive bitmap words) would meet the other owners in
// every bank it touches (64 banks of 4 bytes): one pad word per 8 bins / per 32 words makes the owners'
// strides odd.
constexpr int kBins = 2048, kBinsPad = kBins + kBins / 8;
__device__ __forceinline__ int bslot(int b) { return b + (b >> 3); }
__device__ __forceinline__ int wslot(int w) { return w + (w >> 5); }

// bins[bslot(0..2048)): largest-first search for the bin holding the k-th entry (1 <= k <= total).
// sh: 40 words of LDS scratch.
template <int NT>
__device__ __forceinline__ void kth_bin(const uint32_t* bins, uint32_t k, uint32_t* sh,
                                        uint32_t& bin, uint32_t& above) {
  constexpr int BPT = kBins / NT;
  static_assert(BPT >= 1 && BPT * NT == kBins, "bins per thread");
  uint32_t loc[BPT], sum = 0;
#pragma unroll
  for (int i = 0; i < BPT; ++i) { loc[i] = bins[bslot(threadIdx.x * BPT + i)]; sum += loc[i]; }
  uint32_t total;
  const uint32_t incl = block_scan_incl<NT>(sum, sh, total);
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
    for (int b = threadIdx.x; b < kBinsPad; b += NT) bins[b] = 0;
    __syncthreads();
    for (uint32_t i = threadIdx.x; i < n; i += NT) {
      const uint64_t v = get(i);
      if ((shift + w >= 64 ? 0ull : (v >> (shift + w))) == prefix)
        atomicAdd(&bins[bslot((int)((uint32_t)(v >> shift) & ((1u << w) - 1u)))], 1u);
    }
    __syncthreads();
    uint32_t d, ab;
    kth_bin<NT>(bins, remaining, sh, d, ab);
    const uint32_t in_bin = bins[bslot((int)d)];
    remaining -= ab;
    prefix = (prefix << w) | d;
    __syncthreads();
    if (in_bin == remaining) break;
  }
  shift_out = shift; prefix_out = prefix;
}

// min and max of one value per thread over the NT threads of the workgroup (sh: 40 words, NT <= 1024).
template <int NT>
__device__ __forceinline__ void block_minmax(uint32_t& lo, uint32_t& hi, uint32_t* sh) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    lo = min(lo, (uint32_t)__shfl_xor((int)lo, o, 64));
    hi = max(hi, (uint32_t)__shfl_xor((int)hi, o, 64));
  }
  constexpr int NW = NT / 64;
  static_assert(NW <= 16, "at most 16 waves");
  if ((threadIdx.x & 63) == 0) { sh[threadIdx.x >> 6] = lo; sh[16 + (threadIdx.x >> 6)] = hi; }
  __syncthreads();
#pragma unroll
  for (int w = 0; w < NW; ++w) { lo = min(lo, sh[w]); hi = max(hi, sh[16 + w]); }
  __syncthreads();
}

// Lower bound of the rho-th largest of n ordered score keys held R per thread (slot r of thread t is entry
// r * NT + t; entries past n are ignored), as an ordered key; at most 2^-22 of the keys' range below the
// rho-th largest itself.  rho > n returns 0 (every key passes).  The select walks the significant bits of
// the offsets from a cut three exponent steps below the largest key, 11 at a time, and stops after two
// passes: the bits left undecided only lower the bound.  Over the whole range the first digits would be sign
// and exponent, which put thousands of entries into a handful of bins (LDS atomics on one address
// serialise); a row whose window holds fewer than rho entries falls back to the whole range.
template <int NT, int R>
__device__ __forceinline__ uint32_t kth_lower_bound_key(const uint32_t* key, uint32_t n, uint32_t rho,
                                                        uint32_t* bins, uint32_t* sh) {
  if (rho > n) return 0u;
  uint32_t kmin = 0xffffffffu, kmax = 0u;
#pragma unroll
  for (int r = 0; r < R; ++r)
    if ((uint32_t)r * NT + threadIdx.x < n) { kmin = min(kmin, key[r]); kmax = max(kmax, key[r]); }
  block_minmax<NT>(kmin, kmax, sh);
  uint32_t cut = kmin;
  if (kmax >= 0x80000000u + (4u << 23)) {
    const uint32_t c = kmax - (3u << 23);
    uint32_t in = 0;
#pragma unroll
    for (int r = 0; r < R; ++r) in += ((uint32_t)r * NT + threadIdx.x < n && key[r] >= c) ? 1u : 0u;
    uint32_t total;
    block_scan_incl<NT>(in, sh, total);
    if (total >= rho) cut = c;                                 // workgroup-uniform
  }
  int dsh = 32 - __clz((int)(kmax - cut));
  uint32_t dpref = 0, remaining = rho;
  for (int p = 0; p < 2 && dsh > 0; ++p) {
    const int w = dsh < 11 ? dsh : 11;
    dsh -= w;
    for (int b = threadIdx.x; b < kBinsPad; b += NT) bins[b] = 0;
    __syncthreads();
    const int up = dsh + w;
#pragma unroll
    for (int r = 0; r < R; ++r) {
      if ((uint32_t)r * NT + threadIdx.x < n && key[r] >= cut) {
        const uint32_t d = key[r] - cut;
        if (up >= 32 || (d >> up) == dpref) atomicAdd(&bins[bslot((int)((d >> dsh) & ((1u << w) - 1u)))], 1u);
      }
    }
    __syncthreads();
    uint32_t d, ab;
    kth_bin<NT>(bins, remaining, sh, d, ab);
    remaining -= ab;
    dpref = (dpref << w) | d;
    __syncthreads();
  }
  // smallest key that shares the decided prefix
  return cut + (dsh >= 32 ? 0u : (dpref << dsh));
}

// ordered key -> the float it stands for
__device__ __forceinline__ float key_score(uint32_t k) {
  return __uint_as_float((k & 0x80000000u) ? (k & 0x7fffffffu) : ~k);
}

#endif  // __HIPCC__
}  // namespace reattn
