// Vote selection (paper, Method, "Full-Context Cache Selection", last paragraph; Setup:
// k = 4, k' = 127, span 32): every (query row, query head) votes for its own top-k middle
// tokens by raw position-agnostic score, the k' most voted tokens are kept together with
// their m neighbouring entries, overlaps deduplicated; one shared set per layer.
//
//   head_topk_scan   the fused score + top-k of the paper: the key cache is streamed once
//                    (same load shape as the group-sum scan: 16-byte non-temporal loads,
//                    DPP row reductions) and every lane keeps a running top-k per head in
//                    registers, so no score ever leaves the chip; lists are merged by wave
//                    arg-max rounds and each workgroup writes k (score, index) composites
//                    per head;
//   head_topk_merge  one wave per (query, head): the best k of the workgroups' partial lists,
//                    ascending absolute indices;
//   vote_scatter     one fp32 atomic add of 1.0 per vote into a dense array over the middle
//                    (exact up to 2^24 votes per token);
//   (topk.hip)       the k' most voted tokens = top-k of that array, ties by lower index;
//   span_union       sorted centres -> clipped spans -> union by prefix maximum / prefix sum
//                    -> ascending index list and its length (a device scalar: the scope of
//                    the following attention is data dependent).
#include "common.hpp"

namespace reattn {
namespace {

template <typename T> struct Elem;
template <> struct Elem<float> {
  static constexpr int kPerLoad = 4;
  static __device__ __forceinline__ void widen(const u32x4& d, float* x) {
    x[0] = __uint_as_float(d.x); x[1] = __uint_as_float(d.y);
    x[2] = __uint_as_float(d.z); x[3] = __uint_as_float(d.w);
  }
  static __device__ __forceinline__ float one(const void* p, int64_t i) { return ((const float*)p)[i]; }
};
template <> struct Elem<uint16_t> {   // bf16 bit patterns
  static constexpr int kPerLoad = 8;
  static __device__ __forceinline__ void widen(const u32x4& d, float* x) {
    x[0] = bf16_lo(d.x); x[1] = bf16_hi(d.x); x[2] = bf16_lo(d.y); x[3] = bf16_hi(d.y);
    x[4] = bf16_lo(d.z); x[5] = bf16_hi(d.z); x[6] = bf16_lo(d.w); x[7] = bf16_hi(d.w);
  }
  static __device__ __forceinline__ float one(const void* p, int64_t i) {
    return __uint_as_float(((uint32_t)((const uint16_t*)p)[i]) << 16);
  }
};

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

constexpr int kVoteThreads = 1024;
constexpr int kVoteWaves = kVoteThreads / 64;

struct HeadScanArgs {
  const void* k; const void* q;
  uint64_t* part;          // [rows = n_query * Hq][n_wg][KT] composites, best first
  int64_t ksh, kst, n_mid, first_tok;
  int Hq, Hkv, G, rows_per_block, n_wg;
};

// KT: list length kept per head (>= vote_k); GH: heads a lane keeps lists for (ceil(G / 2)).
template <typename T, int D, int KT, int GH>
__global__ __launch_bounds__(kVoteThreads) void head_topk_scan_kernel(HeadScanArgs a) {
  constexpr int EPL = Elem<T>::kPerLoad, LPR = D / EPL, RPL = 64 / LPR, U = 8, RW = U * RPL;
  static_assert(LPR == 16, "a key row spans 16 lanes (D = 128 bf16 or D = 64 fp32)");
  constexpr int GMAX = 2 * GH;
  __shared__ uint64_t wave_best[kVoteWaves][GMAX][KT];

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int sub = lane % LPR, grp = lane / LPR;
  const int row_id = blockIdx.y;                       // query * Hkv + kv head
  const int h = row_id % a.Hkv, qi = row_id / a.Hkv;

  float qv[GMAX][EPL];
#pragma unroll
  for (int g = 0; g < GMAX; ++g) {
    const int gg = g < a.G ? g : a.G - 1;
    const int64_t qoff = ((int64_t)qi * a.Hq + (int64_t)h * a.G + gg) * D + sub * EPL;
#pragma unroll
    for (int e = 0; e < EPL; ++e) qv[g][e] = Elem<T>::one(a.q, qoff + e);
  }
  // lane `sub` keeps the result of load u = sub % 8 for the heads of parity sub / 8
  const int my_u = sub & 7, my_par = sub >> 3;
  float bv[GH][KT]; uint32_t bi[GH][KT];
#pragma unroll
  for (int x = 0; x < GH; ++x)
#pragma unroll
    for (int t = 0; t < KT; ++t) { bv[x][t] = -__builtin_inff(); bi[x][t] = 0xffffffffu; }

  const int64_t blk_row0 = (int64_t)blockIdx.x * a.rows_per_block;
  const int64_t left = a.n_mid - blk_row0;
  const int nrows = left < a.rows_per_block ? (int)left : a.rows_per_block;
  const int64_t row_bytes = a.kst * (int64_t)sizeof(T);
  const char* kbase = (const char*)a.k +
      ((int64_t)h * a.ksh + (a.first_tok + blk_row0) * a.kst) * (int64_t)sizeof(T) + sub * 16;

  for (int t = wave * RW; t < nrows; t += kVoteWaves * RW) {
    u32x4 d[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      int r = t + u * RPL + grp;
      r = r < nrows ? r : nrows - 1;                   // tail rows re-read the last row; result dropped
      d[u] = __builtin_nontemporal_load((const u32x4*)(kbase + (int64_t)r * row_bytes));
    }
    float mine[GH];
#pragma unroll
    for (int x = 0; x < GH; ++x) mine[x] = -__builtin_inff();
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float xk[EPL];
      Elem<T>::widen(d[u], xk);
#pragma unroll
      for (int g = 0; g < GMAX; ++g) {
        float s = 0.f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) s = fmaf(xk[e], qv[g][e], s);
        s = group_sum<LPR>(s);
        const bool keep = (my_u == u) && (my_par == (g & 1));
        mine[g >> 1] = keep ? s : mine[g >> 1];
      }
    }
    const int r = t + my_u * RPL + grp;
    if (r < nrows) {
      const uint32_t pos = (uint32_t)(blk_row0 + r);
#pragma unroll
      for (int x = 0; x < GH; ++x) {
        // rows arrive in ascending position per lane: a later equal score never displaces
        if (2 * x + my_par < a.G && mine[x] > bv[x][KT - 1]) {
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
    const int x = g >> 1;
    const bool owner = my_par == (g & 1);
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
  // workgroup merge: wave g takes head g; its lanes hold the 16 waves' KT entries (two per lane at most)
  if (wave < a.G) {
    const int g = wave;
    uint64_t c0 = 0ull, c1 = 0ull;
    if (lane < kVoteWaves * KT) c0 = wave_best[lane / KT][g][lane % KT];
    if (lane + 64 < kVoteWaves * KT) c1 = wave_best[(lane + 64) / KT][g][(lane + 64) % KT];
    uint64_t* out = a.part + (((int64_t)qi * a.Hq + (int64_t)h * a.G + g) * a.n_wg + blockIdx.x) * KT;
#pragma unroll
    for (int round = 0; round < KT; ++round) {
      const uint64_t best = wave_max_u64(c0 > c1 ? c0 : c1);
      if (c0 == best) c0 = 0ull;
      if (c1 == best) c1 = 0ull;
      if (lane == 0) out[round] = best;
    }
  }
}

// One wave per (query, head): best vote_k of n_wg * KT composites -> ascending absolute indices.
__global__ __launch_bounds__(64) void head_topk_merge_kernel(const uint64_t* __restrict__ part, int n_cand,
                                                             int vote_k, int32_t index_base,
                                                             int32_t* head_topk) {
  const int lane = threadIdx.x;
  const uint64_t* p = part + (int64_t)blockIdx.x * n_cand;
  uint32_t mine = 0xffffffffu;                         // lane t < vote_k ends up with the t-th best position
  uint64_t taken_below = ~0ull;                        // composites are distinct: walk down strictly
  for (int round = 0; round < vote_k; ++round) {
    uint64_t c = 0ull;
    for (int i = lane; i < n_cand; i += 64) {
      const uint64_t v = p[i];
      if (v < taken_below && v > c) c = v;
    }
    const uint64_t best = wave_max_u64(c);
    taken_below = best;
    if (lane == round) mine = best ? 0xffffffffu - (uint32_t)best : 0xffffffffu;
  }
  // ascending order: rank of each kept position among the kept ones
  int rank = 0;
  for (int t = 0; t < vote_k; ++t) {
    const uint32_t o = __shfl(mine, t, 64);
    rank += (o < mine) ? 1 : 0;
  }
  if (lane < vote_k) head_topk[(int64_t)blockIdx.x * vote_k + rank] = index_base + (int32_t)mine;
}

__global__ __launch_bounds__(256) void vote_scatter_kernel(const int32_t* __restrict__ head_topk, int64_t n_votes,
                                                           int32_t index_base, float* votes) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n_votes) atomicAdd(&votes[head_topk[i] - index_base], 1.0f);
}

// centres: kc ascending absolute indices (the top-kc of the vote array; some may have no vote).
__global__ __launch_bounds__(1024) void span_union_kernel(const int32_t* __restrict__ centres, int kc,
                                                          const float* __restrict__ votes, int32_t s_eff,
                                                          int64_t n_mid, int span, int32_t* sel,
                                                          int32_t* n_sel) {
  __shared__ int32_t sh_a[1024], sh_b[1024];
  const int i = threadIdx.x;
  int32_t lo = 0, hi = 0;                              // relative to the middle; empty when no vote
  if (i < kc) {
    const int32_t c = centres[i] - s_eff;
    if (votes[c] > 0.f) {
      lo = c - span / 2; hi = lo + span;
      lo = lo < 0 ? 0 : lo;
      hi = hi > (int32_t)n_mid ? (int32_t)n_mid : hi;
    }
  }
  // exclusive prefix maximum of hi (centres ascend, so spans overlap only with predecessors)
  sh_a[i] = hi;
  __syncthreads();
  for (int o = 1; o < 1024; o <<= 1) {
    const int32_t v = i >= o ? sh_a[i - o] : 0;
    __syncthreads();
    sh_a[i] = sh_a[i] > v ? sh_a[i] : v;
    __syncthreads();
  }
  const int32_t before = i > 0 ? sh_a[i - 1] : 0;
  const int32_t start = lo > before ? lo : before;
  const int32_t len = hi > start ? hi - start : 0;
  sh_b[i] = len;
  __syncthreads();
  for (int o = 1; o < 1024; o <<= 1) {
    const int32_t v = i >= o ? sh_b[i - o] : 0;
    __syncthreads();
    sh_b[i] += v;
    __syncthreads();
  }
  const int32_t at = sh_b[i] - len;
  for (int32_t t = 0; t < len; ++t) sel[at + t] = s_eff + start + t;
  if (i == 1023) *n_sel = sh_b[1023];
}

template <typename T, int D, int KT>
hipError_t scan_launch_gh(const HeadScanArgs& a, dim3 grid, hipStream_t st) {
  const int gh = (a.G + 1) / 2;
  switch (gh) {
    case 1: hipLaunchKernelGGL((head_topk_scan_kernel<T, D, KT, 1>), grid, dim3(kVoteThreads), 0, st, a); break;
    case 2: hipLaunchKernelGGL((head_topk_scan_kernel<T, D, KT, 2>), grid, dim3(kVoteThreads), 0, st, a); break;
    case 3: hipLaunchKernelGGL((head_topk_scan_kernel<T, D, KT, 3>), grid, dim3(kVoteThreads), 0, st, a); break;
    default: hipLaunchKernelGGL((head_topk_scan_kernel<T, D, KT, 4>), grid, dim3(kVoteThreads), 0, st, a); break;
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

int scan_rows_per_block(int64_t n_mid, int64_t score_rows);

int vote_list_len(int vote_k) { return vote_k <= 1 ? 1 : vote_k <= 2 ? 2 : vote_k <= 4 ? 4 : 8; }

// The streaming path handles 16-lane key rows (bf16 D = 128, fp32 D = 64) and groups of up to 8 heads.
bool vote_scan_applies(const Plan& pl) {
  return pl.G <= 8 && ((pl.dtype == 1 && pl.D == 128) || (pl.dtype == 0 && pl.D == 64));
}

int vote_scan_workgroups(const Plan& pl, int n_query) {
  const int rpb = scan_rows_per_block(pl.n_mid, (int64_t)pl.Hkv * n_query);
  return (int)((pl.n_mid + rpb - 1) / rpb);
}

size_t vote_part_bytes(const Plan& pl, int n_query, int vote_k) {
  return (size_t)n_query * pl.Hq * vote_scan_workgroups(pl, n_query) * vote_list_len(vote_k) * sizeof(uint64_t);
}

// head_topk[i][hq][vote_k] for queries [0, n_query): ascending absolute indices.
hipError_t launch_head_topk_scan(const Plan& pl, const void* q, int n_query, const void* k_cache,
                                 int vote_k, uint64_t* part, int32_t* head_topk, hipStream_t st) {
  if (pl.n_mid <= 0 || n_query <= 0 || vote_k <= 0) return hipSuccess;
  HeadScanArgs a;
  a.k = k_cache; a.q = q; a.part = part;
  a.ksh = pl.ksh; a.kst = pl.kst; a.n_mid = pl.n_mid; a.first_tok = pl.s_eff;
  a.Hq = pl.Hq; a.Hkv = pl.Hkv; a.G = pl.G;
  a.rows_per_block = scan_rows_per_block(pl.n_mid, (int64_t)pl.Hkv * n_query);
  a.n_wg = (int)((pl.n_mid + a.rows_per_block - 1) / a.rows_per_block);
  const int kt = vote_list_len(vote_k);
  const dim3 grid((unsigned)a.n_wg, (unsigned)(pl.Hkv * n_query));
  hipError_t e = pl.dtype == 0 ? scan_launch_kt<float, 64>(a, kt, grid, st)
                               : scan_launch_kt<uint16_t, 128>(a, kt, grid, st);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(head_topk_merge_kernel, dim3((unsigned)(n_query * pl.Hq)), dim3(64), 0, st, part,
                     a.n_wg * kt, vote_k, (int32_t)pl.s_eff, head_topk);
  return hipGetLastError();
}

hipError_t launch_vote_scatter(const Plan& pl, const int32_t* head_topk, int64_t n_votes, float* votes,
                               hipStream_t st) {
  if (n_votes <= 0) return hipSuccess;
  hipLaunchKernelGGL(vote_scatter_kernel, dim3((unsigned)((n_votes + 255) / 256)), dim3(256), 0, st,
                     head_topk, n_votes, (int32_t)pl.s_eff, votes);
  return hipGetLastError();
}

hipError_t launch_span_union(const Plan& pl, const int32_t* centres, int kc, const float* votes, int span,
                             int32_t* sel, int32_t* n_sel, hipStream_t st) {
  hipLaunchKernelGGL(span_union_kernel, dim3(1), dim3(1024), 0, st, centres, kc, votes, (int32_t)pl.s_eff,
                     pl.n_mid, span, sel, n_sel);
  return hipGetLastError();
}

}  // namespace reattn
