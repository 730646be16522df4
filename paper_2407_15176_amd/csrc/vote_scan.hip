// Vote selection, first step (paper, Method, "Full-Context Cache Selection", last paragraph): the fused
// score + top-k of every (query row, query head) on the vector ALU, for the shapes the matrix-core scan
// does not take (fp32 storage; 16-bit storage with D = 64).  The key cache is streamed once per query row
// with 16-byte non-temporal loads, D / (elements per load) adjacent lanes cover one key row, dot products
// finish with DPP row reductions, and every lane keeps running top-k lists in registers for the heads and
// loads it owns, so no score ever leaves the chip.  Lists are merged inside the wave, then over the waves;
// each workgroup writes k (score, index) composites per (query row, head).
#include "common.hpp"
#include "select.hpp"
#include "vote_scan.hpp"

namespace reattn {
namespace {

// KT: list length kept per head (>= vote_k); GH: lists a lane keeps (one per head it owns).
// A row's LPR lanes all hold the reduced dot product; lane `sub` keeps the result of load u = sub % U for the
// heads g with g % NPAR == sub / U (NPAR = LPR / U), so the U loads x GH * NPAR heads of a wave iteration are
// spread over the row's lanes.  The launch covers heads [g0, g0 + gcount) of every group, gcount <= GH * NPAR.
template <typename T, int D, int KT, int GH, bool PAGED>
__global__ __launch_bounds__(kVoteThreads) void head_topk_scan_kernel(HeadScanArgs a, int g0, int gcount) {
  __shared__ int32_t s_pages[PAGED ? kVotePages : 1];
  constexpr int EPL = Store<T>::kPerLoad, LPR = D / EPL, RPL = 64 / LPR;
  constexpr int U = LPR >= 16 ? 8 : LPR / 2, NPAR = LPR / U, RW = U * RPL;
  static_assert(LPR == 8 || LPR == 16 || LPR == 32, "a key row spans 8, 16 or 32 lanes");
  constexpr int GMAX = NPAR * GH;
  __shared__ uint64_t wave_best[kVoteWaves][GMAX][KT];

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int sub = lane % LPR, grp = lane / LPR;
  const int row_id = blockIdx.y;                       // query * Hkv + kv head
  const int h = row_id % a.Hkv, qi = row_id / a.Hkv;

  float qv[GMAX][EPL];
#pragma unroll
  for (int g = 0; g < GMAX; ++g) {
    const int gg = g0 + (g < gcount ? g : gcount - 1);
    const int64_t qoff = ((int64_t)qi * a.Hq + (int64_t)h * a.G + gg) * D + sub * EPL;
#pragma unroll
    for (int e = 0; e < EPL; ++e) qv[g][e] = Store<T>::one(a.q, qoff + e);
  }
  const int my_u = sub % U, my_par = sub / U;
  float bv[GH][KT]; uint32_t bi[GH][KT];
#pragma unroll
  for (int x = 0; x < GH; ++x)
#pragma unroll
    for (int t = 0; t < KT; ++t) { bv[x][t] = -__builtin_inff(); bi[x][t] = 0xffffffffu; }

  const int64_t blk_row0 = (int64_t)blockIdx.x * a.rows_per_block;
  const int64_t left = a.n_mid - blk_row0;
  const int nrows = left < a.rows_per_block ? (int)left : a.rows_per_block;
  const int64_t row_bytes = a.kst * (int64_t)sizeof(T);
  const int64_t tok0 = a.first_tok + blk_row0;
  const char* kbase = (const char*)a.k +
      ((int64_t)h * a.ksh + (PAGED ? 0 : tok0) * a.kst) * (int64_t)sizeof(T) + sub * 16;
  if (PAGED) slice_pages_fill(s_pages, a.pt, a.page_lg, tok0, nrows, kVoteThreads);
  static_assert(RW <= 64, "a wave's tile lies in at most two pages");

  for (int t = wave * RW; t < nrows; t += kVoteWaves * RW) {
    u32x4 d[U];
    TilePages tp;
    if (PAGED) tp = tile_pages(s_pages, a.page_lg, tok0, tok0 + t);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      int r = t + u * RPL + grp;
      r = r < nrows ? r : nrows - 1;                   // tail rows re-read the last row; result dropped
      const int64_t row = PAGED ? tp.row(r - t) : r;
      d[u] = __builtin_nontemporal_load((const u32x4*)(kbase + row * row_bytes));
    }
    float mine[GH];
#pragma unroll
    for (int x = 0; x < GH; ++x) mine[x] = -__builtin_inff();
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float xk[EPL];
      Store<T>::widen(d[u], xk);
#pragma unroll
      for (int g = 0; g < GMAX; ++g) {
        float s = 0.f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) s = fmaf(xk[e], qv[g][e], s);
        s = group_sum<LPR>(s);
        const bool keep = (my_u == u) && (my_par == g % NPAR);
        mine[g / NPAR] = keep ? s : mine[g / NPAR];
      }
    }
    const int r = t + my_u * RPL + grp;
    if (r < nrows) {
      const uint32_t pos = (uint32_t)(blk_row0 + r);
#pragma unroll
      for (int x = 0; x < GH; ++x) {
        // rows arrive in ascending position per lane: a later equal score never displaces
        if (NPAR * x + my_par < gcount && mine[x] > bv[x][KT - 1]) {
          bv[x][KT - 1] = mine[x]; bi[x][KT - 1] = pos;
#pragma unroll
          for (int tt = KT - 1; tt > 0; --tt) {
            if (bv[x][tt] > bv[x][tt - 1]) {
              const float fv = bv[x][tt]; bv[x][tt] = bv[x][tt - 1]; bv[x][tt - 1] = fv;
              const uint32_t iv = bi[x][tt]; bi[x][tt] = bi[x][tt - 1]; bi[x][tt - 1] = iv;
            }
          }
        }
      }
    }
  }

  // wave merge: for each head, KT rounds of arg-max over the lanes' list heads
#pragma unroll
  for (int g = 0; g < GMAX; ++g) {
    const int x = g / NPAR;
    const bool owner = my_par == g % NPAR;
#pragma unroll
    for (int round = 0; round < KT; ++round) {
      const uint64_t c = (owner && bi[x][0] != 0xffffffffu) ? composite(bv[x][0], bi[x][0]) : 0ull;
      const uint64_t best = wave_max_u64(c);
      if (owner && c == best && best != 0ull) {          // pop: composites are unique (distinct positions)
#pragma unroll
        for (int tt = 0; tt + 1 < KT; ++tt) { bv[x][tt] = bv[x][tt + 1]; bi[x][tt] = bi[x][tt + 1]; }
        bv[x][KT - 1] = -__builtin_inff(); bi[x][KT - 1] = 0xffffffffu;
      }
      if (lane == 0) wave_best[wave][g][round] = best;
    }
  }
  __syncthreads();
  // workgroup merge: wave g takes head g0 + g; its lanes hold the 16 waves' KT entries (two per lane at most)
  if (wave < gcount) {
    const int g = wave;
    uint64_t c0 = 0ull, c1 = 0ull;
    if (lane < kVoteWaves * KT) c0 = wave_best[lane / KT][g][lane % KT];
    if (lane + 64 < kVoteWaves * KT) c1 = wave_best[(lane + 64) / KT][g][(lane + 64) % KT];
    uint64_t* out = a.part + (((int64_t)qi * a.Hq + (int64_t)h * a.G + g0 + g) * a.n_wg + blockIdx.x) * KT;
#pragma unroll
    for (int round = 0; round < KT; ++round) {
      const uint64_t best = wave_max_u64(c0 > c1 ? c0 : c1);
      if (c0 == best) c0 = 0ull;
      if (c1 == best) c1 = 0ull;
      if (lane == 0) out[round] = best;
    }
  }
}

template <typename T, int D, int KT, int GH>
void scan_launch_paged(const HeadScanArgs& a, int g0, int gcount, dim3 grid, hipStream_t st) {
  if (a.pt) hipLaunchKernelGGL((head_topk_scan_kernel<T, D, KT, GH, true>), grid, dim3(kVoteThreads), 0, st, a, g0, gcount);
  else      hipLaunchKernelGGL((head_topk_scan_kernel<T, D, KT, GH, false>), grid, dim3(kVoteThreads), 0, st, a, g0, gcount);
}

// Heads per pass: as many as four lists per lane hold.
template <typename T, int D, int KT>
hipError_t scan_launch_gh(const HeadScanArgs& a, dim3 grid, hipStream_t st) {
  constexpr int EPL = Store<T>::kPerLoad, LPR = D / EPL, U = LPR >= 16 ? 8 : LPR / 2, NPAR = LPR / U;
  constexpr int kPass = 4 * NPAR;
  for (int g0 = 0; g0 < a.G; g0 += kPass) {
    const int gcount = a.G - g0 < kPass ? a.G - g0 : kPass;
    switch ((gcount + NPAR - 1) / NPAR) {
      case 1: scan_launch_paged<T, D, KT, 1>(a, g0, gcount, grid, st); break;
      case 2: scan_launch_paged<T, D, KT, 2>(a, g0, gcount, grid, st); break;
      case 3: scan_launch_paged<T, D, KT, 3>(a, g0, gcount, grid, st); break;
      default: scan_launch_paged<T, D, KT, 4>(a, g0, gcount, grid, st); break;
    }
  }
  return hipGetLastError();
}

template <typename T, int D>
hipError_t scan_launch_kt(const HeadScanArgs& a, int kt, dim3 grid, hipStream_t st) {
  switch (kt) {
    case 1: return scan_launch_gh<T, D, 1>(a, grid, st);
    case 2: return scan_launch_gh<T, D, 2>(a, grid, st);
    case 4: return scan_launch_gh<T, D, 4>(a, grid, st);
    default: return scan_launch_gh<T, D, 8>(a, grid, st);
  }
}

}  // namespace

hipError_t launch_head_scan_valu(const Plan& pl, const HeadScanArgs& a, int kt, dim3 grid, hipStream_t st) {
  if (pl.dtype == kF32) return pl.D == 64 ? scan_launch_kt<float, 64>(a, kt, grid, st) : scan_launch_kt<float, 128>(a, kt, grid, st);
  if (pl.dtype == kF16) return pl.D == 64 ? scan_launch_kt<f16bits, 64>(a, kt, grid, st) : scan_launch_kt<f16bits, 128>(a, kt, grid, st);
  return pl.D == 64 ? scan_launch_kt<uint16_t, 64>(a, kt, grid, st) : scan_launch_kt<uint16_t, 128>(a, kt, grid, st);
}

}  // namespace reattn
