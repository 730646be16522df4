// Sequential positional embedding after selection (paper Eq. 3, "PE", and the
// remark that the cached keys carry no positional information): slot r of the
// concatenation [global, select, local] is rotary-encoded at position r.
// Pairing (c, c + D/2), angle r * theta^(-2c/D), as in the LLaMA family.
//
//   prep         clears the top-k histograms and fills the two-level
//                (cos, sin) table used by the attention kernel: rows [0, n_hi) hold
//                the angles of positions 128*a, rows [n_hi, n_hi+128) those of
//                positions b < 128; position r = 128a + b is their complex product.
//                Angles are formed in fp64 so that the fp32 entries are correctly
//                rounded even at position 131071, where an fp32 product r*w is off
//                by ~1e-2 rad; the table has (S/128 + 128) rows instead of S.
//   gather_rope  materialised form of the concatenation: K rows rotated into an
//                fp32 buffer, V rows copied.
#include "common.hpp"
#include <type_traits>

namespace reattn {
namespace {

__global__ __launch_bounds__(256) void prep_kernel(uint32_t* hist, int64_t n_hist, AppendArgs ap,
                                                   float2* rope, int S, int half, int D,
                                                   double log2_theta) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n_hist) { hist[i] = 0u; return; }
  if (i < n_hist + ap.n_vec) { append_piece(ap, i - n_hist); return; }
  const int64_t j = i - n_hist - ap.n_vec;
  if (rope && j < (int64_t)(rope_rows_hi(S) + kRopeLo) * half) rope[j] = rope_table_entry(j, S, half, D, log2_theta);
}

__global__ void fill_u32_kernel(uint32_t* p, int64_t n, uint32_t v) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

struct GatherArgs {
  const void* k; const void* v; const int32_t* idx; float* k_sel; void* v_sel;
  int64_t ksh, kst, vsh, vst, N;
  int Hkv, M, S, s_eff, k_eff, l_eff;
  const int32_t* pt; int page_lg;                  // paged cache, or nullptr
  double omega[64];                                // w_c = theta^(-2c/D), formed on the host in fp64
};

// E consecutive stored elements -> fp32, and the raw copy of them (vector accesses of E * sizeof(T) bytes).
template <typename T, int E> struct Piece;
template <int E> struct Piece<float, E> {
  typedef typename std::conditional<E == 4, u32x4, u32x2>::type raw;
  static __device__ __forceinline__ void widen(const raw& d, float* x) {
#pragma unroll
    for (int e = 0; e < E; ++e) x[e] = __uint_as_float(d[e]);
  }
};
template <int E> struct Piece<uint16_t, E> {
  typedef typename std::conditional<E == 4, u32x2, uint32_t>::type raw;
  static __device__ __forceinline__ uint32_t word(const u32x2& d, int i) { return d[i]; }
  static __device__ __forceinline__ uint32_t word(const uint32_t& d, int) { return d; }
  static __device__ __forceinline__ void widen(const raw& d, float* x) {
#pragma unroll
    for (int e = 0; e < E; e += 2) { x[e] = bf16_lo(word(d, e / 2)); x[e + 1] = bf16_hi(word(d, e / 2)); }
  }
};
template <int E> struct Piece<f16bits, E> {
  typedef typename std::conditional<E == 4, u32x2, uint32_t>::type raw;
  static __device__ __forceinline__ void widen(const raw& d, float* x) {
#pragma unroll
    for (int e = 0; e < E; e += 2) {
      x[e] = f16_lo(Piece<uint16_t, E>::word(d, e / 2)); x[e + 1] = f16_hi(Piece<uint16_t, E>::word(d, e / 2));
    }
  }
};

// One 16-lane group per (query, KV head, slot).  Lane `sub` owns channels [sub*E, sub*E+E) and their partners
// D/2 higher, so a rotation never leaves the lane, and every access is one vector of the lane's E elements.
// The kernel is a gather: 2 * D * b bytes read and D * (4 + b) written per slot.  The angle r * w_c is formed
// and reduced to [-pi, pi] in fp64 (exact to ~1e-11 rad at any position), its sine and cosine taken in fp32:
// a full fp64 sincos per element made the kernel compute-bound at four times its memory time.
template <typename T, int D>
__global__ __launch_bounds__(256) void gather_rope_kernel(GatherArgs a) {
  constexpr int E = D / 32;                       // channels per lane per half
  typedef Piece<T, E> P;
  typedef typename P::raw Raw;
  typedef typename Piece<float, E>::raw FRaw;
  const int sub = threadIdx.x & 15;
  const int64_t slot_id = (int64_t)blockIdx.x * 16 + (threadIdx.x >> 4);
  const int64_t total = (int64_t)a.M * a.Hkv * a.S;
  if (slot_id >= total) return;
  const int r = (int)(slot_id % a.S);
  const int h = (int)((slot_id / a.S) % a.Hkv);
  const int qi = (int)(slot_id / ((int64_t)a.S * a.Hkv));
  const int visible = a.S - (a.M - 1 - qi);       // causal cut inside the local part
  float* ko = a.k_sel + slot_id * D;
  T* vo = (T*)a.v_sel + slot_id * D;
  const int c0 = sub * E;
  if (r >= visible) {
    FRaw zf; Raw zv;
    memset(&zf, 0, sizeof zf); memset(&zv, 0, sizeof zv);
    *(FRaw*)(ko + c0) = zf; *(FRaw*)(ko + D / 2 + c0) = zf;
    *(Raw*)(vo + c0) = zv; *(Raw*)(vo + D / 2 + c0) = zv;
    return;
  }
  int64_t tok;
  if (r < a.s_eff) tok = r;
  else if (r < a.s_eff + a.k_eff) tok = a.idx[((int64_t)qi * a.Hkv + h) * a.k_eff + (r - a.s_eff)];
  else tok = a.N - a.l_eff + (r - a.s_eff - a.k_eff);
  if (a.pt) tok = paged_row(a.pt, a.page_lg, tok);
  const T* kr = (const T*)a.k + (int64_t)h * a.ksh + tok * a.kst;
  const T* vr = (const T*)a.v + (int64_t)h * a.vsh + tok * a.vst;
  const Raw klo = *(const Raw*)(kr + c0), khi = *(const Raw*)(kr + D / 2 + c0);
  const Raw vlo = *(const Raw*)(vr + c0), vhi = *(const Raw*)(vr + D / 2 + c0);
  float lo[E], hi[E];
  P::widen(klo, lo); P::widen(khi, hi);
  FRaw olo, ohi;
#pragma unroll
  for (int e = 0; e < E; ++e) {
    const double turns = (double)r * a.omega[c0 + e] * 0.15915494309189535;     // angle / (2 pi)
    const float ang = (float)((turns - rint(turns)) * 6.283185307179586);
    float sn, cs;
    sincosf(ang, &sn, &cs);
    olo[e] = __float_as_uint(lo[e] * cs - hi[e] * sn);
    ohi[e] = __float_as_uint(hi[e] * cs + lo[e] * sn);
  }
  *(FRaw*)(ko + c0) = olo; *(FRaw*)(ko + D / 2 + c0) = ohi;
  *(Raw*)(vo + c0) = vlo; *(Raw*)(vo + D / 2 + c0) = vhi;
}

__global__ __launch_bounds__(256) void cache_append_kernel(AppendArgs a) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < a.n_vec) append_piece(a, i);
}

}  // namespace

namespace {
__global__ __launch_bounds__(256) void translate_rows_kernel(const int32_t* idx, int32_t* rows, int64_t n,
                                                             const int32_t* pt, int page_lg) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) rows[i] = (int32_t)paged_row(pt, page_lg, idx[i]);
}
}  // namespace

hipError_t launch_translate_rows(const Plan& pl, const int32_t* idx, int32_t* rows, int64_t n, hipStream_t st) {
  if (n <= 0 || !pl.pt) return hipSuccess;
  hipLaunchKernelGGL(translate_rows_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, idx, rows, n, pl.pt,
                     pl.page_lg);
  return hipGetLastError();
}

hipError_t launch_cache_append(const Plan& pl, int64_t first_tok, int n_tok, const void* k_new, const void* v_new,
                               void* k_cache, void* v_cache, hipStream_t st) {
  if (n_tok <= 0) return hipSuccess;
  const AppendJob j{k_new, v_new, k_cache, v_cache, first_tok, n_tok};
  const AppendArgs a = append_args(pl, &j);
  hipLaunchKernelGGL(cache_append_kernel, dim3((unsigned)((a.n_vec + 255) / 256)), dim3(256), 0, st, a);
  return hipGetLastError();
}

hipError_t launch_prep(const Plan& pl, int rows, uint32_t* hist, float2* rope, hipStream_t st,
                       const AppendJob* append) {
  if (!hist) rows = 0;
  const AppendArgs ap = append_args(pl, append);
  const int64_t n_hist = (int64_t)rows * kHistBins;
  const int64_t n_rope = rope ? (int64_t)(rope_rows_hi(pl.S) + kRopeLo) * (pl.D / 2) : 0;
  const int64_t n = n_hist + ap.n_vec + n_rope;
  if (n == 0) return hipSuccess;
  hipLaunchKernelGGL(prep_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st,
                     hist, n_hist, ap, rope, pl.S, pl.D / 2, pl.D, log2((double)pl.theta));
  return hipGetLastError();
}

hipError_t launch_fill_u32(uint32_t* p, int64_t n, uint32_t v, hipStream_t st) {
  if (n <= 0) return hipSuccess;
  hipLaunchKernelGGL(fill_u32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, p, n, v);
  return hipGetLastError();
}

hipError_t launch_gather_rope(const Plan& pl, const void* k_cache, const void* v_cache,
                              const int32_t* idx, float* k_sel, void* v_sel, hipStream_t st) {
  GatherArgs a;
  a.k = k_cache; a.v = v_cache; a.idx = idx; a.k_sel = k_sel; a.v_sel = v_sel;
  a.ksh = pl.ksh; a.kst = pl.kst; a.vsh = pl.vsh; a.vst = pl.vst; a.N = pl.N;
  a.Hkv = pl.Hkv; a.M = pl.M; a.S = pl.S;
  a.s_eff = (int)pl.s_eff; a.k_eff = pl.k_eff; a.l_eff = (int)pl.l_eff; a.pt = pl.pt; a.page_lg = pl.page_lg;
  for (int c = 0; c < pl.D / 2; ++c) a.omega[c] = exp2(-2.0 * (double)c / (double)pl.D * log2((double)pl.theta));
  const int64_t total = (int64_t)pl.M * pl.Hkv * pl.S;
  if (total == 0) return hipSuccess;
  const dim3 grid((unsigned)((total + 15) / 16));
  if (pl.dtype == kF32) {
    if (pl.D == 64) hipLaunchKernelGGL((gather_rope_kernel<float, 64>), grid, dim3(256), 0, st, a);
    else            hipLaunchKernelGGL((gather_rope_kernel<float, 128>), grid, dim3(256), 0, st, a);
  } else if (pl.dtype == kF16) {
    if (pl.D == 64) hipLaunchKernelGGL((gather_rope_kernel<f16bits, 64>), grid, dim3(256), 0, st, a);
    else            hipLaunchKernelGGL((gather_rope_kernel<f16bits, 128>), grid, dim3(256), 0, st, a);
  } else {
    if (pl.D == 64) hipLaunchKernelGGL((gather_rope_kernel<uint16_t, 64>), grid, dim3(256), 0, st, a);
    else            hipLaunchKernelGGL((gather_rope_kernel<uint16_t, 128>), grid, dim3(256), 0, st, a);
  }
  return hipGetLastError();
}

}  // namespace reattn
