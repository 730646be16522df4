// Stage 2 for a chunk of query rows that share ONE selection (the vote selection: paper,
// Method, "Full-Context Cache Selection", last paragraph, then Eq. 3): every query row attends
// over the same [global, select, local] entries at the same re-assigned positions 0..S-1 and
// differs only in its causal cut inside the local part.  So the concatenation is formed once
//
//   pack_shared   slot r -> cache row, key rotary-encoded at position r in fp32 and split into
//                 two halves hi + lo of the storage format (a rotated bf16 key is not a bf16
//                 number; the split keeps ~16 mantissa bits for bf16, ~22 for IEEE half), value
//                 rows transposed per tile of 32 slots so that the slot index is the contiguous
//                 one (the contraction index of P.V);
//   qprep_shared  query rows rotary-encoded at their own slot, pre-scaled by
//                 softmax_scale * log2(e), split hi + lo;
//
// and the attention itself is a flash-attention kernel on the matrix cores
// (v_mfma_f32_32x32x16_bf16): a workgroup of 4 waves owns 128 (query row, head) pairs of one
// KV head and walks the shared slots in tiles of 32 staged through LDS.  Scores are formed
// transposed, S^T = K Q^T (keys are the A operand), so a lane holds ONE (query, head) column
// and 16 slots of it: the running maximum and sum of the online softmax are per-lane scalars
// and cost one shuffle per tile.  The key rows of a tile enter the A operand in the order
// 0-3, 8-11, 4-7, 12-15 (per 16): the 16 scores a lane holds are then the slots
// 8*(lane/32) + 0..7 and 16 + 8*(lane/32) + 0..7 of the tile, which is exactly the B operand
// layout of the following O^T += V^T P^T, so the weights go from the first contraction into
// the second without leaving their registers.  Weights are split hi + lo as well.
// Per tile of 32 slots and 32 columns: 24 MFMAs for the scores (hi.hi + lo.hi + hi.lo over 8
// k-steps) and 16 for the output.  The scores of tile t + 1 are issued before the weights of tile t are
// formed (three tile buffers): measured 2 % (1.50 -> 1.475 ms at 4,096 rows, 0.296 -> 0.290 at 512); the kernel
// stays bound by the issue of its LDS operand reads (24 KB per wave and tile against 40 matrix instructions).
#include "common.hpp"

namespace reattn {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x8 __attribute__((ext_vector_type(8)));

constexpr int kSlots = 32;                      // slots per tile
constexpr int kKPitch = 528;                    // bytes per staged key slot: 256 hi + 256 lo + 16 pad
constexpr int kVPitch = 80;                     // bytes per staged value channel: 32 slots + 16 pad
constexpr int kKTile = kSlots * kKPitch;        // 16,896
constexpr int kVTile = 128 * kVPitch;           // 10,240
constexpr int kBuf = kKTile + kVTile;
constexpr float kNoMax = -1.0e30f;               // running maximum before any visible slot
constexpr float kMasked = -2.0e30f;              // score of a hidden slot: 2^(kMasked - max) is 0 even against kNoMax

__device__ __forceinline__ u32x4 pack8(const uint16_t* h) {
  u32x4 w;
  w.x = (uint32_t)h[0] | ((uint32_t)h[1] << 16); w.y = (uint32_t)h[2] | ((uint32_t)h[3] << 16);
  w.z = (uint32_t)h[4] | ((uint32_t)h[5] << 16); w.w = (uint32_t)h[6] | ((uint32_t)h[7] << 16);
  return w;
}
__device__ __forceinline__ uint16_t half_of(const u32x4& w, int e) {    // e-th 16-bit element
  const uint32_t d = e < 2 ? w.x : e < 4 ? w.y : e < 6 ? w.z : w.w;
  return (uint16_t)((e & 1) ? d >> 16 : d & 0xffffu);
}

struct SharedArgs {
  const uint16_t* q; const uint16_t* k; const uint16_t* v;
  const int32_t* sel; const int32_t* n_sel;     // shared ascending selection and its length (device)
  const float2* rope; int rope_n_hi;            // two-level (cos, sin) table
  uint16_t* kp;       // [Hkv][s_pad][2][128]  rotated keys, hi then lo
  uint16_t* vp;       // [Hkv][s_pad / 32][128][32]  values, slot-contiguous per tile
  uint16_t* qp;       // [M][Hq][2][128]  rotated, scaled queries, hi then lo
  float* out;         // [M][Hq][128]
  int64_t ksh, kst, vsh, vst, N;
  const int32_t* pt; int page_lg;               // paged cache (nullptr: none)
  int Hq, Hkv, G, M, s_eff, l_eff, s_pad;
  float scale_log2e;
};

__device__ __forceinline__ float2 rope_cs(const SharedArgs& a, int r, int c) {
  const float2 x = a.rope[(int64_t)(r / kRopeLo) * 64 + c];
  const float2 y = a.rope[(int64_t)(a.rope_n_hi + r % kRopeLo) * 64 + c];
  return make_float2(x.x * y.x - x.y * y.y, x.y * y.x + x.x * y.y);
}

// One workgroup per (tile of 32 slots, KV head).
template <bool F16>
__global__ __launch_bounds__(256) void pack_shared_kernel(SharedArgs a) {
  typedef Mm<F16> F;
  __shared__ uint16_t vt[kSlots][128 + 8];
  const int tile = blockIdx.x, h = blockIdx.y, tid = threadIdx.x;
  const int n_sel = *a.n_sel;
  const int s_total = a.s_eff + n_sel + a.l_eff;
  const int j = tid >> 3, c0 = (tid & 7) * 8;              // slot of the tile, first of 8 channels (and c0 + 64)
  const int r = tile * kSlots + j;
  u32x4 klo = {0u, 0u, 0u, 0u}, khi = klo, vlo = klo, vhi = klo;
  if (r < s_total) {
    int64_t tok;
    if (r < a.s_eff) tok = r;
    else if (r < a.s_eff + n_sel) tok = a.sel[r - a.s_eff];
    else tok = a.N - a.l_eff + (r - a.s_eff - n_sel);
    if (a.pt) tok = paged_row(a.pt, a.page_lg, tok);
    const uint16_t* kr = a.k + (int64_t)h * a.ksh + tok * a.kst;
    const uint16_t* vr = a.v + (int64_t)h * a.vsh + tok * a.vst;
    klo = *(const u32x4*)(kr + c0); khi = *(const u32x4*)(kr + 64 + c0);
    vlo = *(const u32x4*)(vr + c0); vhi = *(const u32x4*)(vr + 64 + c0);
  }
  // rotate the pairs (c, c + 64) at position r, split hi + lo
  uint16_t o_hi_a[8], o_hi_b[8], o_lo_a[8], o_lo_b[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const float2 cs = rope_cs(a, r < s_total ? r : 0, c0 + e);
    const float x = F::widen(half_of(klo, e)), y = F::widen(half_of(khi, e));
    const float ra = x * cs.x - y * cs.y, rb = y * cs.x + x * cs.y;
    o_hi_a[e] = F::narrow(ra); o_lo_a[e] = F::narrow(ra - F::widen(o_hi_a[e]));
    o_hi_b[e] = F::narrow(rb); o_lo_b[e] = F::narrow(rb - F::widen(o_hi_b[e]));
  }
  uint16_t* ko = a.kp + (((int64_t)h * a.s_pad + r) * 2) * 128;
  *(u32x4*)(ko + c0) = pack8(o_hi_a);
  *(u32x4*)(ko + 64 + c0) = pack8(o_hi_b);
  *(u32x4*)(ko + 128 + c0) = pack8(o_lo_a);
  *(u32x4*)(ko + 192 + c0) = pack8(o_lo_b);
  // values: through LDS into [channel][slot]
  *(u32x4*)&vt[j][c0] = vlo;
  *(u32x4*)&vt[j][64 + c0] = vhi;
  __syncthreads();
  const int d = tid >> 1, s0 = (tid & 1) * 16;
  uint16_t col[16];
#pragma unroll
  for (int s = 0; s < 16; ++s) col[s] = vt[s0 + s][d];
  uint16_t* vo = a.vp + (((int64_t)h * (a.s_pad / kSlots) + tile) * 128 + d) * kSlots + s0;
  *(u32x4*)vo = pack8(col);
  *(u32x4*)(vo + 8) = pack8(col + 8);
}

// One thread per channel pair of one (query row, head).
template <bool F16>
__global__ __launch_bounds__(64) void qprep_shared_kernel(SharedArgs a) {
  typedef Mm<F16> F;
  const int i = blockIdx.x, hq = blockIdx.y, c = threadIdx.x;
  const int p = a.s_eff + *a.n_sel + (a.l_eff - a.M + i);   // the slot of the query's own key
  const uint16_t* qr = a.q + ((int64_t)i * a.Hq + hq) * 128;
  const float2 cs = rope_cs(a, p, c);
  const float x = F::widen(qr[c]), y = F::widen(qr[c + 64]);
  const float ra = (x * cs.x - y * cs.y) * a.scale_log2e, rb = (y * cs.x + x * cs.y) * a.scale_log2e;
  uint16_t* o = a.qp + (((int64_t)i * a.Hq + hq) * 2) * 128;
  const uint16_t ha = F::narrow(ra), hb = F::narrow(rb);
  o[c] = ha; o[c + 64] = hb;
  o[128 + c] = F::narrow(ra - F::widen(ha));
  o[192 + c] = F::narrow(rb - F::widen(hb));
}


// grid: (row tiles of one KV head, Hkv); longest scopes first.
// With few query rows the slots are also split over blockIdx.z (flash-decoding): a workgroup then
// writes its unnormalised (max, sum, output) triple per column and attend_combine merges them.
template <bool F16>
__global__ __launch_bounds__(256) void attend_shared_kernel(SharedArgs a, int q_per_wg, int n_row_tiles, int nsplit,
                                                            float* part) {
  typedef typename Mm<F16>::op8 op8;
  constexpr int NT = 256, KP = 1024 / NT, VP = 512 / NT;   // threads, 16-byte pieces per thread of a key / value tile
  extern __shared__ __attribute__((aligned(16))) unsigned char as_lds[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int ln = lane & 31, lh = lane >> 5;
  const int h = blockIdx.y;
  const int rt = n_row_tiles - 1 - (int)blockIdx.x;
  const int n_sel = *a.n_sel;
  const int base_scope = a.s_eff + n_sel + (a.l_eff - a.M) + 1;          // scope of query row 0
  // this lane's column: (query row, head)
  const int lr = wave * 32 + ln;
  const int qi = rt * q_per_wg + lr / a.G, g = lr % a.G;
  const bool live = lr / a.G < q_per_wg && qi < a.M;
  const int scope = live ? base_scope + qi : 1;                          // slots [0, scope) are visible
  int q_last = rt * q_per_wg + q_per_wg - 1;
  if (q_last > a.M - 1) q_last = a.M - 1;
  const int n_tiles_all = (base_scope + q_last + kSlots - 1) / kSlots;   // the workgroup's longest scope
  const int per_split = (n_tiles_all + nsplit - 1) / nsplit;
  const int t_first = (int)blockIdx.z * per_split;
  const int t_end = t_first + per_split < n_tiles_all ? t_first + per_split : n_tiles_all;

  op8 qh[8], ql[8];
  {
    const uint16_t* qr = a.qp + (((int64_t)(live ? qi : 0) * a.Hq + (int64_t)h * a.G + (live ? g : 0)) * 2) * 128 + lh * 8;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      qh[ks] = *(const op8*)(qr + ks * 16);
      ql[ks] = *(const op8*)(qr + 128 + ks * 16);
    }
  }
  f32x16 o[4];
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int i = 0; i < 16; ++i) o[db][i] = 0.f;
  float m_run = kNoMax, l_run = 0.f;

  // staging: a key tile is 32 x 512 contiguous bytes (1024 pieces of 16), a value tile 128 x 64 (512 pieces)
  const unsigned char* kg = (const unsigned char*)(a.kp + ((int64_t)h * a.s_pad) * 256);
  const unsigned char* vg = (const unsigned char*)(a.vp + ((int64_t)h * (a.s_pad / kSlots)) * 128 * kSlots);
  u32x4 sk[KP], sv[VP];
  auto load_tile = [&](int t) {
#pragma unroll
    for (int j = 0; j < KP; ++j) sk[j] = *(const u32x4*)(kg + (int64_t)t * (kSlots * 512) + (tid + NT * j) * 16);
#pragma unroll
    for (int j = 0; j < VP; ++j) sv[j] = *(const u32x4*)(vg + (int64_t)t * (128 * 64) + (tid + NT * j) * 16);
  };
  auto stash_tile = [&](int buf) {
    unsigned char* kb = as_lds + buf * kBuf;
    unsigned char* vb = kb + kKTile;
#pragma unroll
    for (int j = 0; j < KP; ++j) { const int p = tid + NT * j; *(u32x4*)(kb + (p >> 5) * kKPitch + (p & 31) * 16) = sk[j]; }
#pragma unroll
    for (int j = 0; j < VP; ++j) { const int p = tid + NT * j; *(u32x4*)(vb + (p >> 2) * kVPitch + (p & 3) * 16) = sv[j]; }
  };
  // Three tile buffers (tile t in buffer t mod 3): the scores of tile t + 1 are already in the matrix pipe while
  // the weights of tile t are formed on the vector ALUs, so its keys have to be in LDS a step early; tile t + 2
  // is written during step t from registers that were loaded during step t - 1.
  const int n_t = t_end - t_first;
  if (n_t > 0) { load_tile(t_first); stash_tile(0); }
  if (n_t > 1) { load_tile(t_first + 1); stash_tile(1); }
  if (n_t > 2) load_tile(t_first + 2);
  __syncthreads();

  // A row m of the score contraction takes slot pi(m): 4-blocks 1 and 2 of every 16 swapped
  const int pim = (ln & ~12) | ((ln & 4) << 1) | ((ln & 8) >> 1);
  // S^T = K Q^T: hi.hi + lo.hi + hi.lo
  auto scores_of = [&](int buf) -> f32x16 {
    const unsigned char* arow = as_lds + buf * kBuf + pim * kKPitch + lh * 16;
    f32x16 s;
#pragma unroll
    for (int i = 0; i < 16; ++i) s[i] = 0.f;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      const op8 kh = *(const op8*)(arow + ks * 32);
      const op8 kl = *(const op8*)(arow + 256 + ks * 32);
      s = Mm<F16>::mfma32(kh, qh[ks], s);
      s = Mm<F16>::mfma32(kl, qh[ks], s);
      s = Mm<F16>::mfma32(kh, ql[ks], s);
    }
    return s;
  };
  f32x16 s, s_next;
#pragma unroll
  for (int i = 0; i < 16; ++i) { s[i] = 0.f; s_next[i] = 0.f; }
  if (n_t > 0) s = scores_of(0);
  int buf = 0;
  for (int t = t_first; t < t_end; ++t) {
    const int buf1 = buf == 2 ? 0 : buf + 1, buf2 = buf1 == 2 ? 0 : buf1 + 1;
    if (t + 2 < t_end) stash_tile(buf2);                     // its last readers finished two steps ago
    if (t + 3 < t_end) load_tile(t + 3);
    if (t + 1 < t_end) s_next = scores_of(buf1);             // issued ahead of the vector work on tile t
    asm volatile("" : "+v"(s_next));
    const unsigned char* vb = as_lds + buf * kBuf + kKTile;
    // s[i] is slot 32t + 16(i/8) + 8(lane/32) + i%8 of this lane's column; slots past the causal cut are hidden
    const int slot0 = t * kSlots + lh * 8;
#pragma unroll
    for (int i = 0; i < 16; ++i) s[i] = slot0 + 16 * (i >> 3) + (i & 7) >= scope ? kMasked : s[i];
    float mx = s[0];
#pragma unroll
    for (int i = 1; i < 16; ++i) mx = fmaxf(mx, s[i]);
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float m_new = fmaxf(m_run, mx);
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
    m_run = m_new;
    // weights p = 2^(s - m) and their split into two bf16 halves (hardware conversions)
    f32x8 pv[2];
    float psum = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const float p = __builtin_amdgcn_exp2f(s[i] - m_new);
      psum += p;
      pv[i >> 3][i & 7] = p;
    }
    op8 ph[2], pl[2];
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) {
      ph[kk] = __builtin_convertvector(pv[kk], op8);
      pl[kk] = __builtin_convertvector(pv[kk] - __builtin_convertvector(ph[kk], f32x8), op8);
    }
    l_run = l_run * alpha + psum;
    if (__any(alpha != 1.0f)) {
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[db][i] *= alpha;
    }
    // O^T += V^T P^T: A = values [channel][slot], B = this lane's weights (two k-steps of 16 slots)
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) {
      const op8 bh = ph[kk], bl = pl[kk];
#pragma unroll
      for (int db = 0; db < 4; ++db) {
        const op8 va = *(const op8*)(vb + (db * 32 + ln) * kVPitch + kk * 32 + lh * 16);
        o[db] = Mm<F16>::mfma32(va, bh, o[db]);
        o[db] = Mm<F16>::mfma32(va, bl, o[db]);
      }
    }
    s = s_next;
    buf = buf1;
    __syncthreads();
  }

  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  if (live) {
    const int64_t row = (int64_t)qi * a.Hq + (int64_t)h * a.G + g;
    const float inv = nsplit == 1 ? 1.0f / l_tot : 1.0f;
    float* orow = nsplit == 1 ? a.out + row * 128 : part + (row * nsplit + blockIdx.z) * 130 + 2;
    if (nsplit > 1 && lh == 0) { orow[-2] = m_run; orow[-1] = l_tot; }
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        // o[db][4j .. 4j+3] are channels 32 db + 8 j + 4 (lane/32) + 0..3
        float* dst = orow + db * 32 + j * 8 + lh * 4;
        if (nsplit == 1) {
          *(float4*)dst = make_float4(o[db][4 * j] * inv, o[db][4 * j + 1] * inv, o[db][4 * j + 2] * inv, o[db][4 * j + 3] * inv);
        } else {                                           // rows of 130 floats: 8-byte aligned only
          *(float2*)dst = make_float2(o[db][4 * j], o[db][4 * j + 1]);
          *(float2*)(dst + 2) = make_float2(o[db][4 * j + 2], o[db][4 * j + 3]);
        }
      }
  }
}

}  // namespace

bool attend_shared_applies(const Plan& pl) { return pl.dtype != kF32 && pl.D == 128 && pl.M > 1 && pl.G <= 16; }

int attend_shared_spad(const Plan& pl) { return (pl.S + kSlots - 1) / kSlots * kSlots; }

// Splits of the slot axis: with few query rows the row tiles alone leave most of the chip idle.
int attend_shared_splits(const Plan& pl) {
  const int64_t wgs = (int64_t)((pl.M + 128 / pl.G - 1) / (128 / pl.G)) * pl.Hkv;
  int64_t n = 512 / (wgs > 0 ? wgs : 1);
  const int64_t tiles = (pl.S + kSlots - 1) / kSlots;
  if (n > tiles / 8) n = tiles / 8;                     // at least 8 tiles per split
  return (int)(n < 1 ? 1 : n > 8 ? 8 : n);
}

// bytes of the packed keys, packed values, prepared queries and split partials
void attend_shared_layout(const Plan& pl, size_t* kp, size_t* vp, size_t* qp, size_t* part) {
  const size_t sp = (size_t)attend_shared_spad(pl);
  *kp = (size_t)pl.Hkv * sp * 512;
  *vp = (size_t)pl.Hkv * sp * 256;
  *qp = (size_t)pl.M * pl.Hq * 512;
  const int ns = attend_shared_splits(pl);
  *part = ns > 1 ? (size_t)pl.M * pl.Hq * ns * 130 * 4 : 0;
}

// pl.S is the largest scope (s_eff + cap + l_eff); `rope` must cover it.
hipError_t launch_attend_shared(const Plan& pl, const void* q, const void* k_cache, const void* v_cache,
                                const int32_t* sel, const int32_t* n_sel, const float2* rope, void* kp,
                                void* vp, void* qp, float* part, float* out, hipStream_t st) {
  SharedArgs a;
  a.q = (const uint16_t*)q; a.k = (const uint16_t*)k_cache; a.v = (const uint16_t*)v_cache;
  a.sel = sel; a.n_sel = n_sel; a.rope = rope; a.rope_n_hi = rope_rows_hi(pl.S);
  a.kp = (uint16_t*)kp; a.vp = (uint16_t*)vp; a.qp = (uint16_t*)qp; a.out = out;
  a.ksh = pl.ksh; a.kst = pl.kst; a.vsh = pl.vsh; a.vst = pl.vst; a.N = pl.N; a.pt = pl.pt; a.page_lg = pl.page_lg;
  a.Hq = pl.Hq; a.Hkv = pl.Hkv; a.G = pl.G; a.M = pl.M;
  a.s_eff = (int)pl.s_eff; a.l_eff = (int)pl.l_eff; a.s_pad = attend_shared_spad(pl);
  a.scale_log2e = pl.scale * 1.4426950408889634f;
  const dim3 pgrid((unsigned)(a.s_pad / kSlots), (unsigned)pl.Hkv), qgrid((unsigned)pl.M, (unsigned)pl.Hq);
  const int q_per_wg = 128 / pl.G;
  const int n_row_tiles = (pl.M + q_per_wg - 1) / q_per_wg;
  const int nsplit = attend_shared_splits(pl);
  const dim3 agrid((unsigned)n_row_tiles, (unsigned)pl.Hkv, (unsigned)nsplit);
  auto run = [&](auto pack, auto qprep, auto att) -> hipError_t {
    hipLaunchKernelGGL(pack, pgrid, dim3(256), 0, st, a);
    hipLaunchKernelGGL(qprep, qgrid, dim3(64), 0, st, a);
    hipError_t e = hipFuncSetAttribute((const void*)att, hipFuncAttributeMaxDynamicSharedMemorySize, 3 * kBuf);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(att, agrid, dim3(256), 3 * kBuf, st, a, q_per_wg, n_row_tiles, nsplit, part);
    return hipGetLastError();
  };
  hipError_t e = pl.dtype == kF16 ? run(pack_shared_kernel<true>, qprep_shared_kernel<true>, attend_shared_kernel<true>)
                                  : run(pack_shared_kernel<false>, qprep_shared_kernel<false>, attend_shared_kernel<false>);
  if (e != hipSuccess || nsplit == 1) return e;
  return launch_attend_combine(128, pl.M * pl.Hq, nsplit, part, out, st);
}

}  // namespace reattn
