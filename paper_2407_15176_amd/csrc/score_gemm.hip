// Stage 1 for a prefill chunk: the scores of M queries against the whole middle
// of the key cache are one dense contraction per KV head (paper Eq. 2 applied to
// every query of the chunk; appendix prefilling phase, `score = query @ key[...]^T`),
// so it runs on the matrix cores: v_mfma_f32_32x32x16_bf16, fp32 accumulation.
//
// Group aggregation first: sum_g (q_g . k) = (sum_g q_g) . k.  The group sum qbar is
// formed in fp32 and split into two bf16 operands hi + lo (|qbar - hi - lo| <= 2^-17
// |qbar|), so each key block meets two MFMAs per k-step instead of G: half the
// matrix work of scoring the heads one by one, at fp32-level accuracy (a single bf16
// rounding of qbar would eat half of the 1e-3 tie band of the selection).
//
// Tiling: a workgroup of NQW x 4 waves owns NQW x 64 queries of one KV head and walks
// key tiles of 128 rows.  Keys are the A operand (row = key), queries the B operand
// (column = query): a lane then holds ONE query column per 32x32 block, so a per-query
// threshold test needs one register.  Wave (kw, qw) takes key block kw (32 keys) and
// the two query blocks of half qw; its 2 x 16 query operands (hi, lo for 8 k-steps,
// 128 VGPRs) stay in registers for the whole kernel, the key tile is staged through
// LDS (272-byte row pitch: conflict-free 16-byte reads) with register double-buffering
// of the next tile.  NQW = 2 (512 threads, 128 queries) is what every launch uses: it
// halves the L2->LDS key traffic, and measured 1.9x faster than two independent
// 256-thread workgroups per CU in the fused-filter mode.
//
// Fused filter (prefill selection): instead of writing the M x N_mid scores (33.8 GB at
// M = 4096, N_mid = 258044) each score is compared with a per-(query, KV head) lower
// bound on the k-th largest score, estimated beforehand from a strided sample of the
// keys; the few percent that pass are appended as (score, key) pairs to the row's
// candidate segment.  A workgroup owns its query rows for ALL keys, so the per-row
// counters live in LDS and no global atomics are needed.
#include "common.hpp"

namespace reattn {
int gemm_m_pad(int n_query);
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kTileKeys = 128;
constexpr int kPitch = 272;                     // bytes per staged key row (256 + 16 pad)

__device__ __forceinline__ uint16_t bf16_rne(float x) {
  uint32_t u = __float_as_uint(x);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

// qs[h][i][0][:] = hi, qs[h][i][1][:] = lo of qbar[i][h][:] = sum_g q[i][hG+g][:]; rows i >= M are zero.
__global__ __launch_bounds__(128) void qsplit_kernel(const uint16_t* __restrict__ q, int M, int m_pad,
                                                     int Hq, int Hkv, int G, uint16_t* qs) {
  const int i = blockIdx.x, h = blockIdx.y, c = threadIdx.x;          // D == 128
  float s = 0.f;
  if (i < M)
    for (int g = 0; g < G; ++g)
      s += __uint_as_float(((uint32_t)q[((int64_t)i * Hq + (int64_t)h * G + g) * 128 + c]) << 16);
  const uint16_t hi = bf16_rne(s);
  const uint16_t lo = bf16_rne(s - __uint_as_float((uint32_t)hi << 16));
  uint16_t* o = qs + (((int64_t)h * m_pad + i) * 2) * 128;
  o[c] = hi;
  o[128 + c] = lo;
}

struct GemmArgs {
  const uint16_t* k;        // key cache (bf16 bits)
  const uint16_t* qs;       // split queries [Hkv][m_pad][2][128]
  int64_t ksh, kst;         // key strides in elements
  int64_t first_tok;        // cache row of key 0
  int64_t key_step;         // key j is cache row first_tok + j * key_step (1, or the sampling stride)
  int64_t n_keys;           // keys to score
  int M, m_pad, Hkv;
  int tiles_per_block;      // key tiles one workgroup walks (STORE mode splits the keys over blockIdx.x)
  // STORE: scores[(i * Hkv + h) * score_stride + key]
  float* scores; int64_t score_stride;
  // FILTER: per-row threshold, candidate segments and counts (row = h * M + i)
  const float* thr; uint2* cand; uint32_t* ccount; uint32_t cap;
};

enum { kStore = 0, kFilter = 1, kDiscard = 2 };

template <int MODE, int NQW>
__global__ __launch_bounds__(256 * NQW) void score_gemm_kernel(GemmArgs a) {
  constexpr int kTileQ = 64 * NQW, kGemmThreads = 256 * NQW;
  extern __shared__ __attribute__((aligned(16))) unsigned char gemm_lds[];   // two staged key tiles
  unsigned char (*lds)[kTileKeys * kPitch] = (unsigned char (*)[kTileKeys * kPitch])gemm_lds;
  __shared__ uint32_t lcount[kTileQ];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int kw = wave & 3, qw = wave >> 2;
  const int ln = lane & 31, lh = lane >> 5;
  const int h = blockIdx.z;
  const int q0 = blockIdx.y * kTileQ;
  const int64_t tile0 = (int64_t)blockIdx.x * a.tiles_per_block;
  const int64_t n_tiles_all = (a.n_keys + kTileKeys - 1) / kTileKeys;
  int64_t n_tiles = n_tiles_all - tile0;
  if (n_tiles > a.tiles_per_block) n_tiles = a.tiles_per_block;
  if (MODE == kFilter) {
    if (tid < kTileQ) lcount[tid] = 0;
  }

  // query operands of this wave: 2 blocks x 8 k-steps x (hi, lo), 8 bf16 each
  bf16x8 bhi[2][8], blo[2][8];
#pragma unroll
  for (int qb = 0; qb < 2; ++qb) {
    const int qi = q0 + (qw * 2 + qb) * 32 + ln;
    const uint16_t* row = a.qs + (((int64_t)h * a.m_pad + qi) * 2) * 128 + lh * 8;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      bhi[qb][ks] = *(const bf16x8*)(row + ks * 16);
      blo[qb][ks] = *(const bf16x8*)(row + 128 + ks * 16);
    }
  }
  float thr[2] = {0.f, 0.f};
  if (MODE == kFilter) {
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      const int qi = q0 + (qw * 2 + qb) * 32 + ln;
      thr[qb] = qi < a.M ? a.thr[(int64_t)h * a.M + qi] : __builtin_inff();
    }
  }

  // staging: thread t moves NS x 16 bytes of the 128 x 256-byte key tile: rows t/16 + RS*j, column t%16
  constexpr int NS = 2048 / kGemmThreads, RS = kGemmThreads / 16;
  const int srow = tid >> 4, scol = tid & 15;
  const uint16_t* kbase = a.k + (int64_t)h * a.ksh;
  u32x4 stg[NS];
  auto load_tile = [&](int64_t tile) {
#pragma unroll
    for (int j = 0; j < NS; ++j) {
      int64_t key = tile * kTileKeys + srow + RS * j;
      if (key >= a.n_keys) key = a.n_keys - 1;
      stg[j] = *(const u32x4*)(kbase + (a.first_tok + key * a.key_step) * a.kst + scol * 8);
    }
  };
  auto stash_tile = [&](int buf) {
#pragma unroll
    for (int j = 0; j < NS; ++j)
      *(u32x4*)(&lds[buf][(srow + RS * j) * kPitch + scol * 16]) = stg[j];
  };

  if (n_tiles > 0) { load_tile(tile0); stash_tile(0); }
  __syncthreads();

  for (int64_t t = 0; t < n_tiles; ++t) {
    const int buf = (int)(t & 1);
    if (t + 1 < n_tiles) load_tile(tile0 + t + 1);

    f32x16 acc[2];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[qb][i] = 0.f;
    const unsigned char* arow = &lds[buf][(kw * 32 + ln) * kPitch + lh * 16];
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      const bf16x8 av = *(const bf16x8*)(arow + ks * 32);
#pragma unroll
      for (int qb = 0; qb < 2; ++qb) {
        acc[qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, bhi[qb][ks], acc[qb], 0, 0, 0);
        acc[qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, blo[qb][ks], acc[qb], 0, 0, 0);
      }
    }

    // C layout of a 32x32 block: acc[i] is row (i/4)*8 + (lane/32)*4 + i%4 (key), column lane%32 (query)
    const int64_t key_blk = (tile0 + t) * kTileKeys + kw * 32 + lh * 4;
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      const int qi = q0 + (qw * 2 + qb) * 32 + ln;
      if (MODE == kStore) {
        if (qi < a.M) {
          float* orow = a.scores + ((int64_t)qi * a.Hkv + h) * a.score_stride;
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const int64_t key = key_blk + (i >> 2) * 8 + (i & 3);
            if (key < a.n_keys) orow[key] = acc[qb][i];
          }
        }
      } else if (MODE == kFilter) {
        // one LDS atomic per lane reserves room for all of its hits in this block
        uint32_t mask = 0;
#pragma unroll
        for (int i = 0; i < 16; ++i) mask |= (acc[qb][i] >= thr[qb] ? 1u : 0u) << i;
        if (key_blk + 27 >= a.n_keys) {             // only the ragged last tile can hold invalid keys
#pragma unroll
          for (int i = 0; i < 16; ++i)
            if (key_blk + (i >> 2) * 8 + (i & 3) >= a.n_keys) mask &= ~(1u << i);
        }
        if (mask) {
          const int ql = (qw * 2 + qb) * 32 + ln;
          uint32_t pos = atomicAdd(&lcount[ql], (uint32_t)__popc(mask));
          uint2* seg = a.cand + ((int64_t)h * a.M + qi) * a.cap;
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            if (mask & (1u << i)) {
              if (pos < a.cap)
                seg[pos] = make_uint2(__float_as_uint(acc[qb][i]),
                                      (uint32_t)(key_blk + (i >> 2) * 8 + (i & 3)));
              ++pos;
            }
          }
        }
      } else {
        float s = 0.f;
#pragma unroll
        for (int i = 0; i < 16; ++i) s += acc[qb][i];
        if (s == 1.2345e30f) a.scores[0] = s;    // keeps the MFMAs alive in the timing-only mode
      }
    }

    if (t + 1 < n_tiles) stash_tile(buf ^ 1);
    __syncthreads();
  }

  if (MODE == kFilter) {
    if (tid < kTileQ && q0 + tid < a.M) a.ccount[(int64_t)h * a.M + q0 + tid] = lcount[tid];
  }
}

constexpr size_t kGemmLds = 2 * (size_t)kTileKeys * kPitch;

template <int MODE, int NQW>
hipError_t gemm_launch(const GemmArgs& a, dim3 grid, hipStream_t st) {
  static bool attr_done = false;
  auto kern = score_gemm_kernel<MODE, NQW>;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)kGemmLds);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  hipLaunchKernelGGL(kern, grid, dim3(256 * NQW), kGemmLds, st, a);
  return hipGetLastError();
}

GemmArgs base_args(const Plan& pl, int n_query, const void* k_cache, const void* q_split) {
  GemmArgs a;
  a.k = (const uint16_t*)k_cache; a.qs = (const uint16_t*)q_split;
  a.ksh = pl.ksh; a.kst = pl.kst; a.first_tok = pl.s_eff; a.n_keys = pl.n_mid; a.key_step = 1;
  a.M = n_query; a.m_pad = gemm_m_pad(n_query); a.Hkv = pl.Hkv;
  a.tiles_per_block = 0;
  a.scores = nullptr; a.score_stride = 0;
  a.thr = nullptr; a.cand = nullptr; a.ccount = nullptr; a.cap = 0;
  return a;
}

}  // namespace

int gemm_m_pad(int n_query) { return (n_query + 127) / 128 * 128; }

size_t score_gemm_qsplit_bytes(const Plan& pl) {
  return (size_t)pl.Hkv * gemm_m_pad(pl.M) * 2 * 128 * 2;
}

hipError_t launch_qsplit(const Plan& pl, const void* q, int q_first, int n_query, void* q_split,
                         hipStream_t st) {
  const int m_pad = gemm_m_pad(n_query);
  const uint16_t* qp = (const uint16_t*)q + (int64_t)q_first * pl.Hq * pl.D;
  hipLaunchKernelGGL(qsplit_kernel, dim3(m_pad, pl.Hkv), dim3(128), 0, st, qp, n_query, m_pad, pl.Hq,
                     pl.Hkv, pl.G, (uint16_t*)q_split);
  return hipGetLastError();
}

// Scores of keys first_tok + j * key_step, j < n_keys, written to scores[(i*Hkv + h) * score_stride + j].
hipError_t launch_score_gemm_store(const Plan& pl, int n_query, const void* k_cache,
                                   const void* q_split, int64_t key_step, int64_t n_keys,
                                   float* scores, int64_t score_stride, hipStream_t st) {
  if (n_query <= 0 || n_keys <= 0) return hipSuccess;
  GemmArgs a = base_args(pl, n_query, k_cache, q_split);
  a.key_step = key_step; a.n_keys = n_keys; a.scores = scores; a.score_stride = score_stride;
  const int64_t n_tiles = (n_keys + kTileKeys - 1) / kTileKeys;
  const int64_t qtiles = (int64_t)(a.m_pad / 128) * pl.Hkv;
  int64_t split = (1024 + qtiles - 1) / qtiles;          // enough workgroups to fill the chip
  if (split > n_tiles) split = n_tiles;
  a.tiles_per_block = (int)((n_tiles + split - 1) / split);
  const dim3 grid((unsigned)((n_tiles + a.tiles_per_block - 1) / a.tiles_per_block),
                  (unsigned)(a.m_pad / 128), (unsigned)pl.Hkv);
  return gemm_launch<kStore, 2>(a, grid, st);
}

// Fused filter over all n_mid keys: candidates with score >= thr[h*M + i] go to cand[(h*M + i) * cap ...],
// ccount[h*M + i] receives the number of hits (which may exceed cap: the excess is dropped).
hipError_t launch_score_gemm_filter(const Plan& pl, int n_query, const void* k_cache,
                                    const void* q_split, const float* thr, uint2* cand,
                                    uint32_t* ccount, uint32_t cap, hipStream_t st) {
  if (n_query <= 0 || pl.n_mid <= 0) return hipSuccess;
  GemmArgs a = base_args(pl, n_query, k_cache, q_split);
  a.thr = thr; a.cand = cand; a.ccount = ccount; a.cap = cap;
  const int64_t n_tiles = (pl.n_mid + kTileKeys - 1) / kTileKeys;
  a.tiles_per_block = (int)n_tiles;
  const dim3 grid(1u, (unsigned)(a.m_pad / 128), (unsigned)pl.Hkv);
  return gemm_launch<kFilter, 2>(a, grid, st);
}

// Timing aid: the contraction alone (scores are neither written nor filtered).
hipError_t launch_score_gemm_discard(const Plan& pl, int n_query, const void* k_cache,
                                     const void* q_split, float* sink, hipStream_t st) {
  if (n_query <= 0 || pl.n_mid <= 0) return hipSuccess;
  GemmArgs a = base_args(pl, n_query, k_cache, q_split);
  a.scores = sink;
  const int64_t n_tiles = (pl.n_mid + kTileKeys - 1) / kTileKeys;
  a.tiles_per_block = (int)((n_tiles + 3) / 4);
  const dim3 grid(4u, (unsigned)(a.m_pad / 128), (unsigned)pl.Hkv);
  return gemm_launch<kDiscard, 2>(a, grid, st);
}

hipError_t launch_score_gemm(const Plan& pl, const void* q, int q_first, int n_query,
                             const void* k_cache, float* scores, void* q_split, hipStream_t st) {
  if (n_query <= 0 || pl.n_mid <= 0) return hipSuccess;
  hipError_t e = launch_qsplit(pl, q, q_first, n_query, q_split, st);
  if (e != hipSuccess) return e;
  return launch_score_gemm_store(pl, n_query, k_cache, q_split, 1, pl.n_mid, scores, pl.n_mid, st);
}

}  // namespace reattn
