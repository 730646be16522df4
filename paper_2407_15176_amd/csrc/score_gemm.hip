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
// Tiling: a workgroup of 8 waves (512 threads) owns 128 queries of one KV head and walks
// key tiles of 128 rows.  Keys are the A operand (row = key), queries the B operand
// (column = query): a lane then holds ONE query column per 32x32 block, so a per-query
// threshold test needs one register.  Wave (kw, qw) takes key block kw (32 keys) and
// the two query blocks of half qw; its 2 x 16 query operands (hi, lo for 8 k-steps,
// 128 VGPRs) stay in registers for the whole kernel, the key tile is staged through
// LDS (272-byte row pitch: conflict-free 16-byte reads), two buffers, the next tile
// travelling through registers.  128 queries per workgroup halves the L2->LDS key
// traffic of a 64-query one.  blockIdx.x is the KV head, so that with 8 heads each of
// the 8 XCDs streams one head's keys through its own L2 (HBM sees the keys once).
//
// Fused filter (prefill selection): instead of writing the M x N_mid scores (33.8 GB at
// M = 4096, N_mid = 258044) each score is compared with a per-(query, KV head) lower
// bound on the k-th largest score, estimated beforehand from a strided sample of the
// keys; the few percent that pass are appended as (score, key) pairs to the row's
// candidate segment.  A workgroup owns its query rows for ALL keys, so the per-row
// counters live in LDS and no global atomics are needed.  A finished tile's 32 x 64 scores
// are tested in the accumulator registers (score >= bound as the sign bit of their
// difference, shifted into a per-lane hit word: two vector instructions per score, no
// condition registers) and parked in a wave-private LDS stage, from which the few hits are
// fetched by index and appended during the NEXT tile's MFMAs: between its two halves or
// after them, depending on the wave's query half, so that the two waves sharing a SIMD
// are not both away from the matrix pipe.
//
// Measured on MI355X (random bf16 operands): the matrix pipe itself sustains 1790
// TFLOP/s from registers and 1680 with one LDS operand read per four MFMAs (all-zero
// operands reach 2480: the clock is power-limited under real data), the bare loop of
// this kernel 1400, the fused filter about 900 executed = 1800 algorithmic (testing the scores
// out of the stage, in the shadow of the next tile's first MFMAs, cost more in LDS
// traffic than it hid).
#include "common.hpp"

namespace reattn {
int gemm_m_pad(int n_query);
namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kTileKeys = 128;
constexpr int kPitch = 272;                     // bytes per staged key row (256 + 16 pad)

// qs[h][i][0][:] = hi, qs[h][i][1][:] = lo of qbar[i][h][:] = sum_g q[i][hG+g][:]; rows i >= M are zero.
// F16: IEEE half storage and operands (hi + lo then carry ~22 mantissa bits), else bf16.
template <bool F16>
__global__ __launch_bounds__(128) void qsplit_kernel(const uint16_t* __restrict__ q, int M, int m_pad,
                                                     int Hq, int Hkv, int G, uint16_t* qs) {
  const int i = blockIdx.x, h = blockIdx.y, c = threadIdx.x;          // D == 128
  float s = 0.f;
  if (i < M)
    for (int g = 0; g < G; ++g)
      s += Mm<F16>::widen(q[((int64_t)i * Hq + (int64_t)h * G + g) * 128 + c]);
  const uint16_t hi = Mm<F16>::narrow(s);
  const uint16_t lo = Mm<F16>::narrow(s - Mm<F16>::widen(hi));
  uint16_t* o = qs + (((int64_t)h * m_pad + i) * 2) * 128;
  o[c] = hi;
  o[128 + c] = lo;
}

struct GemmArgs {
  const uint16_t* k;        // key cache (bf16 or IEEE half bits)
  bool f16;                 // IEEE half storage
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
  const float* thr; uint2* cand; uint32_t* ccount; uint32_t cap;   // cap: of one key split's part of a row's segment
  const int32_t* pt; int page_lg;   // paged cache (nullptr: none): token -> row of the head's pool slice
  int n_split;              // FILTER: key splits (blockIdx.z); split z of row r owns segment part and count r * n_split + z
};

enum { kStore = 0, kFilter = 1, kDiscard = 2 };

constexpr int kGemmThreads = 512;               // 8 waves: 4 key blocks x 2 query halves
constexpr int kTileQ = 128;                     // queries per workgroup
constexpr int kTileBytes = kTileKeys * kPitch;  // one staged key tile
constexpr int kStageBytes = 32 * 64 * 4;        // one wave's 32 x 64 scores of a tile (filter mode)
constexpr int kStageNS = 2048 / kGemmThreads;   // 16-byte pieces of a key tile per thread

template <int MODE, bool F16>
__global__ __launch_bounds__(kGemmThreads) void score_gemm_kernel(GemmArgs a) {
  typedef typename Mm<F16>::op8 bf16x8;                     // the operand vector of the storage format
  extern __shared__ __attribute__((aligned(16))) unsigned char gemm_lds[];
  unsigned char* tiles = gemm_lds;                          // two staged key tiles
  __shared__ uint32_t lcount[kTileQ];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int kw = wave & 3, qw = wave >> 2;
  const int ln = lane & 31, lh = lane >> 5;
  // blockIdx.x is the KV head: consecutive workgroup ids go to different XCDs, so with 8 heads
  // every XCD streams the keys of one head through its own L2
  const int h = blockIdx.x;
  const int q0 = blockIdx.y * kTileQ;
  const int64_t tile0 = (int64_t)blockIdx.z * a.tiles_per_block;
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
  uint2* seg[2] = {nullptr, nullptr};
  if (MODE == kFilter) {
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      const int qi = q0 + (qw * 2 + qb) * 32 + ln;
      thr[qb] = qi < a.M ? a.thr[(int64_t)h * a.M + qi] : __builtin_inff();
      seg[qb] = a.cand + (((int64_t)h * a.M + qi) * a.n_split + blockIdx.z) * a.cap;
    }
  }
  // filter mode: this wave's 32 x 64 scores of the previous tile, as 8 rows of 64 float4:
  // row qb*4 + j holds acc[qb][4j .. 4j+3] of every lane
  float4* stage = (float4*)(gemm_lds + 2 * kTileBytes + wave * kStageBytes);

  // staging: thread t moves kStageNS x 16 bytes of the 128 x 256-byte key tile:
  // rows t/16 + 32*j, column t%16.  Tile t + 2 is requested at the start of step t, right after
  // tile t + 1 has been moved from the same registers to LDS, so a load has a whole step to
  // arrive.  The wait sits at the start of a step, before anything else is requested, because
  // the hardware counts loads and stores in one queue and the number of candidate stores a
  // step issues is not known at compile time: a wait placed after them would also wait for
  // the loads just issued.
  constexpr int RS = kGemmThreads / 16;
  const int srow = tid >> 4, scol = tid & 15;
  const int64_t row_bytes = a.key_step * a.kst * 2;          // distance of consecutive scored keys
  const char* kbase = (const char*)(a.k + (int64_t)h * a.ksh + a.first_tok * a.kst) + scol * 16;
  const char* next = kbase + (tile0 * kTileKeys + srow) * row_bytes;   // this thread's piece of the next tile to request
  u32x4 stg[kStageNS];
  auto load_tile = [&](int64_t tile, u32x4* s) {
    if (a.pt) {                                              // paged cache: every row through the page table
      const char* hbase = (const char*)(a.k + (int64_t)h * a.ksh) + scol * 16;
#pragma unroll
      for (int j = 0; j < kStageNS; ++j) {
        int64_t key = tile * kTileKeys + srow + RS * j;
        if (key >= a.n_keys) key = a.n_keys - 1;
        s[j] = *(const u32x4*)(hbase + paged_row(a.pt, a.page_lg, a.first_tok + key * a.key_step) * a.kst * 2);
      }
    } else if ((tile + 1) * kTileKeys <= a.n_keys) {         // wave-uniform: every tile but a ragged last one
#pragma unroll
      for (int j = 0; j < kStageNS; ++j) s[j] = *(const u32x4*)(next + (int64_t)(RS * j) * row_bytes);
    } else {
#pragma unroll
      for (int j = 0; j < kStageNS; ++j) {
        int64_t key = tile * kTileKeys + srow + RS * j;
        if (key >= a.n_keys) key = a.n_keys - 1;             // rows past the end repeat the last key; their scores are dropped
        s[j] = *(const u32x4*)(kbase + key * row_bytes);
      }
    }
    next += (int64_t)kTileKeys * row_bytes;
  };
  auto stash_tile = [&](int buf, const u32x4* s) {
#pragma unroll
    for (int j = 0; j < kStageNS; ++j)
      *(u32x4*)(tiles + buf * kTileBytes + (srow + RS * j) * kPitch + scol * 16) = s[j];
  };

  // C layout of a 32x32 block: acc[i] is row (i/4)*8 + (lane/32)*4 + i%4 (key), column lane%32 (query).
  // Filter epilogue of a finished tile whose scores sit in `stage` and whose per-lane hit mask
  // (bit qb*16 + i for acc[qb][i]) was formed in the shadow of the next tile's MFMAs.
  auto append_hits = [&](int64_t tile, uint32_t mask) {
    const int64_t key_blk = tile * kTileKeys + kw * 32 + lh * 4;
    if (key_blk + 27 >= a.n_keys) {                 // only the ragged last tile can hold invalid keys
#pragma unroll
      for (int i = 0; i < 16; ++i)
        if (key_blk + (i >> 2) * 8 + (i & 3) >= a.n_keys) mask &= ~(0x10001u << i);
    }
    // one LDS atomic per (lane, query block) reserves room for all of its hits
    uint32_t pos[2];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      const uint32_t c = (uint32_t)__popc((mask >> (qb * 16)) & 0xffffu);
      pos[qb] = c ? atomicAdd(&lcount[(qw * 2 + qb) * 32 + ln], c) : 0u;
    }
    // a lane has 0.8 hits on average: four are fetched from the stage together (one LDS round
    // trip instead of four in a row), the loop is for the rare lane with more
    constexpr int kBatch = 4;
    while (mask) {
      int b[kBatch]; float sc[kBatch]; bool on[kBatch];
#pragma unroll
      for (int u = 0; u < kBatch; ++u) {
        on[u] = mask != 0;
        b[u] = on[u] ? __ffs((int)mask) - 1 : 0;
        mask &= mask - 1;                            // 0 stays 0
        sc[u] = ((const float*)stage)[((b[u] >> 2) * 64 + lane) * 4 + (b[u] & 3)];
      }
#pragma unroll
      for (int u = 0; u < kBatch; ++u) {
        if (on[u]) {
          const int qb = b[u] >> 4, i = b[u] & 15;
          const uint32_t at = qb ? pos[1]++ : pos[0]++;
          if (at < a.cap)
            (qb ? seg[1] : seg[0])[at] =
                make_uint2(__float_as_uint(sc[u]), (uint32_t)(key_blk + (i >> 2) * 8 + (i & 3)));
        }
      }
    }
  };
  // score >= thr <=> the sign bit of (score - thr) is clear (the difference of equal finite values is +0);
  // v_alignbit shifts that bit into a running word, so after the 32 scores of a lane, in the order
  // n = qb*16 + i, score n sits at bit 31 - n, inverted.
  auto hits_of = [](uint32_t word) -> uint32_t { return __brev(~word); };   // bit qb*16 + i for acc[qb][i]
  if (n_tiles > 0) {
    load_tile(tile0, stg);
    stash_tile(0, stg);
    if (n_tiles > 1) load_tile(tile0 + 1, stg);
  }
  __syncthreads();

  // One tile: MFMAs of tile t out of LDS buffer `buf`.  In filter mode the threshold tests of
  // tile t - 1 run between the first 16 of them (the matrix pipe and the vector ALUs work side
  // by side), and its hits are appended either between the two halves (waves of query half 1)
  // or after the second (query half 0): the two waves that share a SIMD are then never both
  // away from the matrix pipe.
  uint32_t pending = 0;                           // hit mask of the previous tile (bit qb*16 + i for acc[qb][i])
  auto step = [&](int64_t t, int buf) {
    if (t + 1 < n_tiles) stash_tile(buf ^ 1, stg);
    if (t + 2 < n_tiles) load_tile(tile0 + t + 2, stg);
    f32x16 acc[2];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[qb][i] = 0.f;
    const unsigned char* arow = tiles + buf * kTileBytes + (kw * 32 + ln) * kPitch + lh * 16;
    auto mfma_step = [&](int ks) {
      const bf16x8 av = *(const bf16x8*)(arow + ks * 32);
      acc[0] = Mm<F16>::mfma32(av, bhi[0][ks], acc[0]);
      acc[1] = Mm<F16>::mfma32(av, bhi[1][ks], acc[1]);
      acc[0] = Mm<F16>::mfma32(av, blo[0][ks], acc[0]);
      acc[1] = Mm<F16>::mfma32(av, blo[1][ks], acc[1]);
    };
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) mfma_step(ks);
    if (MODE == kFilter) {
      if (qw == 1) append_hits(tile0 + t - 1, pending);
    }
#pragma unroll
    for (int ks = 4; ks < 8; ++ks) mfma_step(ks);
    const int64_t key_blk = (tile0 + t) * kTileKeys + kw * 32 + lh * 4;
    if (MODE == kFilter) {
      if (qw == 0) append_hits(tile0 + t - 1, pending);
      // this tile's scores against the thresholds, out of the accumulators
      uint32_t word = 0;
#pragma unroll
      for (int qb = 0; qb < 2; ++qb)
#pragma unroll
        for (int i = 0; i < 16; ++i) word = __builtin_amdgcn_alignbit(word, __float_as_uint(acc[qb][i] - thr[qb]), 31);
      pending = hits_of(word);
#pragma unroll
      for (int qb = 0; qb < 2; ++qb)
#pragma unroll
        for (int j = 0; j < 4; ++j)
          stage[(qb * 4 + j) * 64 + lane] =
              make_float4(acc[qb][4 * j], acc[qb][4 * j + 1], acc[qb][4 * j + 2], acc[qb][4 * j + 3]);
    } else if (MODE == kStore) {
#pragma unroll
      for (int qb = 0; qb < 2; ++qb) {
        const int qi = q0 + (qw * 2 + qb) * 32 + ln;
        if (qi < a.M) {
          float* orow = a.scores + ((int64_t)qi * a.Hkv + h) * a.score_stride;
          // a lane holds four consecutive keys per group: one 16-byte store where the row layout allows it
          const bool vec = (a.score_stride & 3) == 0 && ((uintptr_t)a.scores & 15) == 0;
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const int64_t key = key_blk + j * 8;
            if (vec && key + 3 < a.n_keys) {
              *(float4*)(orow + key) = make_float4(acc[qb][4 * j], acc[qb][4 * j + 1], acc[qb][4 * j + 2], acc[qb][4 * j + 3]);
            } else {
#pragma unroll
              for (int c = 0; c < 4; ++c)
                if (key + c < a.n_keys) orow[key + c] = acc[qb][4 * j + c];
            }
          }
        }
      }
    } else {
      float s = 0.f;
#pragma unroll
      for (int qb = 0; qb < 2; ++qb)
#pragma unroll
        for (int i = 0; i < 16; ++i) s += acc[qb][i];
      if (s == 1.2345e30f) a.scores[0] = s;        // keeps the MFMAs alive in the timing-only mode
    }
    __syncthreads();
  };

  for (int64_t t = 0; t < n_tiles; t += 2) {
    step(t, 0);
    if (t + 1 < n_tiles) step(t + 1, 1);
  }

  if (MODE == kFilter) {
    if (n_tiles > 0) append_hits(tile0 + n_tiles - 1, pending);   // the last tile has no successor to hide behind
    __syncthreads();
    if (tid < kTileQ && q0 + tid < a.M) a.ccount[((int64_t)h * a.M + q0 + tid) * a.n_split + blockIdx.z] = lcount[tid];
  }
}

template <int MODE, bool F16>
hipError_t gemm_launch_t(const GemmArgs& a, dim3 grid, hipStream_t st) {
  constexpr size_t lds = 2 * (size_t)kTileBytes + (MODE == kFilter ? 8 * (size_t)kStageBytes : 0);
  auto kern = score_gemm_kernel<MODE, F16>;
  hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, grid, dim3(kGemmThreads), lds, st, a);
  return hipGetLastError();
}
template <int MODE>
hipError_t gemm_launch(const GemmArgs& a, dim3 grid, hipStream_t st) {
  return a.f16 ? gemm_launch_t<MODE, true>(a, grid, st) : gemm_launch_t<MODE, false>(a, grid, st);
}

GemmArgs base_args(const Plan& pl, int n_query, const void* k_cache, const void* q_split) {
  GemmArgs a;
  a.k = (const uint16_t*)k_cache; a.qs = (const uint16_t*)q_split;
  a.ksh = pl.ksh; a.kst = pl.kst; a.first_tok = pl.s_eff; a.n_keys = pl.n_mid; a.key_step = 1;
  a.M = n_query; a.m_pad = gemm_m_pad(n_query); a.Hkv = pl.Hkv; a.f16 = pl.dtype == kF16;
  a.pt = pl.pt; a.page_lg = pl.page_lg;
  a.tiles_per_block = 0;
  a.scores = nullptr; a.score_stride = 0;
  a.thr = nullptr; a.cand = nullptr; a.ccount = nullptr; a.cap = 0; a.n_split = 1;
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
  if (pl.dtype == kF16)
    hipLaunchKernelGGL(qsplit_kernel<true>, dim3(m_pad, pl.Hkv), dim3(128), 0, st, qp, n_query, m_pad, pl.Hq,
                       pl.Hkv, pl.G, (uint16_t*)q_split);
  else
    hipLaunchKernelGGL(qsplit_kernel<false>, dim3(m_pad, pl.Hkv), dim3(128), 0, st, qp, n_query, m_pad, pl.Hq,
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
  const dim3 grid((unsigned)pl.Hkv, (unsigned)(a.m_pad / 128),
                  (unsigned)((n_tiles + a.tiles_per_block - 1) / a.tiles_per_block));
  return gemm_launch<kStore>(a, grid, st);
}

// Fused filter over all n_mid keys, the keys cut into n_split equal runs of tiles (blockIdx.z): candidates of
// row r = h*M + i with score >= thr[r] found by split z go to cand[(r * n_split + z) * cap ...], and
// ccount[r * n_split + z] receives their number (which may exceed cap: the excess is dropped).
hipError_t launch_score_gemm_filter(const Plan& pl, int n_query, const void* k_cache,
                                    const void* q_split, const float* thr, uint2* cand,
                                    uint32_t* ccount, uint32_t cap, int n_split, hipStream_t st) {
  if (n_query <= 0 || pl.n_mid <= 0) return hipSuccess;
  GemmArgs a = base_args(pl, n_query, k_cache, q_split);
  a.thr = thr; a.cand = cand; a.ccount = ccount; a.cap = cap; a.n_split = n_split < 1 ? 1 : n_split;
  const int64_t n_tiles = (pl.n_mid + kTileKeys - 1) / kTileKeys;
  a.tiles_per_block = (int)((n_tiles + a.n_split - 1) / a.n_split);
  const dim3 grid((unsigned)pl.Hkv, (unsigned)(a.m_pad / 128), (unsigned)a.n_split);
  return gemm_launch<kFilter>(a, grid, st);
}

// Timing aid: the contraction alone (scores are neither written nor filtered).
hipError_t launch_score_gemm_discard(const Plan& pl, int n_query, const void* k_cache,
                                     const void* q_split, float* sink, hipStream_t st) {
  if (n_query <= 0 || pl.n_mid <= 0) return hipSuccess;
  GemmArgs a = base_args(pl, n_query, k_cache, q_split);
  a.scores = sink;
  const int64_t n_tiles = (pl.n_mid + kTileKeys - 1) / kTileKeys;
  a.tiles_per_block = (int)((n_tiles + 3) / 4);
  const dim3 grid((unsigned)pl.Hkv, (unsigned)(a.m_pad / 128), 4u);
  return gemm_launch<kDiscard>(a, grid, st);
}

hipError_t launch_score_gemm(const Plan& pl, const void* q, int q_first, int n_query,
                             const void* k_cache, float* scores, void* q_split, hipStream_t st) {
  if (n_query <= 0 || pl.n_mid <= 0) return hipSuccess;
  hipError_t e = launch_qsplit(pl, q, q_first, n_query, q_split, st);
  if (e != hipSuccess) return e;
  return launch_score_gemm_store(pl, n_query, k_cache, q_split, 1, pl.n_mid, scores, pl.n_mid, st);
}

}  // namespace reattn
