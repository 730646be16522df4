// Stage 2 for a prefill chunk: softmax attention of every chunk query over its own
// [global, select_i, local up to token i] (paper Eq. 3, second line, applied per query
// row; appendix prefilling phase, `rope_attention`), bf16 storage, D = 128.
//
// One wave owns one (query, KV head) pair and walks its scope in blocks of 16 slots.
// Per block:
//   * lane (n, j) = (lane % 16, lane / 16) fetches 64 bytes of the key row of slot n
//     (channels 32*ks + 8*j + [0, 8) for ks = 0..3, so both members of every rotary pair
//     (c, c + 64) sit in the same lane) and rotates them at position r = 16*b + n; the
//     (cos, sin) of r is the product of a row of a per-block table (angle 16*b*w) and
//     lane-constant values (angle n*w);
//   * the logits of the (up to four) query heads of the group are one 16x16x32 bf16 MFMA
//     chain: the A operand holds the rotary-encoded, pre-scaled queries as rows
//     (2g, 2g+1) = (hi, lo) halves of a two-term bf16 split, the B operand the rotated key
//     split the same way (two MFMAs per k-step), so the products carry ~16 mantissa bits
//     and the logit of head g is the sum of two accumulator rows of the same lane;
//   * online softmax per head in fp32 (row maxima by DPP, running sums kept per lane);
//   * P.V is a second MFMA chain (16x16x16 bf16) whose contraction index is the slot: the A
//     operand holds the weights as rows (2g, 2g+1) = (hi, lo) bf16 halves, handed from the
//     slot-per-lane to the row-per-lane layout through 256 bytes of wave-private LDS; the B
//     operand needs, per lane, four consecutive slots of ONE channel, so lane (n, j) loads
//     the channel pairs (32u + 2n, 32u + 2n + 1), u < 4, of slots 4j .. 4j+3 as dwords and
//     regroups the 16-bit halves; the accumulators are 8 tiles x 4 registers.
// Nothing is shared between waves: no barriers, no split of a row across workgroups.
#include "common.hpp"

namespace reattn {
namespace {

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));

constexpr int kBlk = 16;                     // slots per block
constexpr float kNegBig = -1.0e30f;

struct PfArgs {
  const uint16_t* q; const uint16_t* k; const uint16_t* v;
  const int32_t* idx; const float2* rope; float* out;
  int64_t ksh, kst, vsh, vst, N;
  const int32_t* pt; int page_lg;            // paged cache (nullptr: none): token -> row of the head's pool slice
  int idx_is_rows;                           // idx already holds pool rows (paged: looked up once per chunk)
  int Hq, Hkv, G, M, S, s_eff, k_eff, l_eff, nsub;
  int nb;                                    // rows of the per-block table: ceil(S / 16)
  float scale_log2e;
};

// rope[row][f], f < 64: rows [0, nb) hold (cos, sin) of 16*row*w_f, rows [nb, nb + 16) those of
// (row - nb)*w_f, w_f = theta^(-f/64).  Angles in fp64, entries correctly rounded.
__global__ __launch_bounds__(256) void rope16_kernel(float2* rope, int nb, double log2_theta) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= (nb + kBlk) * 64) return;
  const int row = i >> 6, f = i & 63;
  const int r = row < nb ? row * kBlk : row - nb;
  const double w = exp2(-(double)f / 64.0 * log2_theta);
  double sn, cs;
  sincos((double)r * w, &sn, &cs);
  rope[i] = make_float2((float)cs, (float)sn);
}

// The two 16-bit storage / operand formats: F16 = false is bf16, true IEEE half.
typedef _Float16 f16x2v __attribute__((ext_vector_type(2)));
typedef _Float16 f16x4v __attribute__((ext_vector_type(4)));
template <bool F16> struct Fmt;
template <> struct Fmt<false> {
  static __device__ __forceinline__ uint32_t pack(float a, float b) {   // round to nearest even
    const f32x2 v = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
  }
  static __device__ __forceinline__ float lo(uint32_t w) { return bf16_lo(w); }
  static __device__ __forceinline__ float hi(uint32_t w) { return bf16_hi(w); }
  static __device__ __forceinline__ f32x4 mfma_pv(u32x2 a, u32x2 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(s16x4, a), __builtin_bit_cast(s16x4, b), c, 0, 0, 0);
  }
};
template <> struct Fmt<true> {
  static __device__ __forceinline__ uint32_t pack(float a, float b) {   // round to nearest even
    const f32x2 v = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, f16x2v));
  }
  static __device__ __forceinline__ float lo(uint32_t w) { return f16_lo(w); }
  static __device__ __forceinline__ float hi(uint32_t w) { return f16_hi(w); }
  static __device__ __forceinline__ f32x4 mfma_pv(u32x2 a, u32x2 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x16f16(__builtin_bit_cast(f16x4v, a), __builtin_bit_cast(f16x4v, b), c, 0, 0, 0);
  }
};
__device__ __forceinline__ float2 cmul(float2 a, float2 b) {
  return make_float2(a.x * b.x - a.y * b.y, a.x * b.y + a.y * b.x);
}
__device__ __forceinline__ float row_max16(float v) {     // max over the 16 lanes of a DPP row, in every lane
  v = fmaxf(v, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xB1, 0xf, 0xf, true)));
  v = fmaxf(v, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x4E, 0xf, 0xf, true)));
  v = fmaxf(v, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x141, 0xf, 0xf, true)));
  v = fmaxf(v, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x140, 0xf, 0xf, true)));
  return v;
}

// Two fp32 rows x[0..8) (channels c..c+7) and y[0..8) (channels c+64..) rotated by cs[0..8),
// each result split into bf16 hi + lo; out: {lo-half hi, lo-half lo, hi-half hi, hi-half lo} operands.
template <bool F16>
__device__ __forceinline__ void rotate_split(const u32x4& klo, const u32x4& khi, const float2* cs,
                                             float mul, u32x4& a_hi, u32x4& a_lo, u32x4& b_hi,
                                             u32x4& b_lo) {
  const uint32_t wl[4] = {klo.x, klo.y, klo.z, klo.w}, wh[4] = {khi.x, khi.y, khi.z, khi.w};
  uint32_t ah[4], al[4], bh[4], bl[4];
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    const float x0 = Fmt<F16>::lo(wl[p]), x1 = Fmt<F16>::hi(wl[p]), y0 = Fmt<F16>::lo(wh[p]), y1 = Fmt<F16>::hi(wh[p]);
    const float2 c0 = cs[2 * p], c1 = cs[2 * p + 1];
    const float r0 = (x0 * c0.x - y0 * c0.y) * mul, r1 = (x1 * c1.x - y1 * c1.y) * mul;   // channels c
    const float s0 = (y0 * c0.x + x0 * c0.y) * mul, s1 = (y1 * c1.x + x1 * c1.y) * mul;   // channels c + 64
    ah[p] = Fmt<F16>::pack(r0, r1);
    al[p] = Fmt<F16>::pack(r0 - Fmt<F16>::lo(ah[p]), r1 - Fmt<F16>::hi(ah[p]));
    bh[p] = Fmt<F16>::pack(s0, s1);
    bl[p] = Fmt<F16>::pack(s0 - Fmt<F16>::lo(bh[p]), s1 - Fmt<F16>::hi(bh[p]));
  }
  a_hi = u32x4{ah[0], ah[1], ah[2], ah[3]}; a_lo = u32x4{al[0], al[1], al[2], al[3]};
  b_hi = u32x4{bh[0], bh[1], bh[2], bh[3]}; b_lo = u32x4{bl[0], bl[1], bl[2], bl[3]};
}

template <bool F16>
__device__ __forceinline__ typename Mm<F16>::op8 as_op8(const u32x4& v) { return __builtin_bit_cast(typename Mm<F16>::op8, v); }

// (cos, sin) of position 16*b + n for the 16 frequencies of lane (n, j): per-block row times the
// lane's own factors (tl: 8 x float4 = two factors each, as kept in LDS by the attention kernel).
template <typename LaneFactors>
__device__ __forceinline__ void block_factors(const float2* t_hi_row, LaneFactors tl, float2 (*cs)[8]) {
#pragma unroll
  for (int x = 0; x < 8; ++x) {
    const float4 t = tl(x);
    const int e = 2 * (x & 3), ks2 = x >> 2;
    cs[ks2][e] = cmul(t_hi_row[32 * ks2 + e], make_float2(t.x, t.y));
    cs[ks2][e + 1] = cmul(t_hi_row[32 * ks2 + e + 1], make_float2(t.z, t.w));
  }
}

// B operands of the logit MFMAs from a raw key row: ops[4*ks2 + {0,1,2,3}] = {hi, lo} halves of the
// rotated channels 32*ks2 + 8j + e, then of the channels 64 higher.
template <bool F16>
__device__ __forceinline__ void key_operands(const u32x4* kr, const float2 (*cs)[8], u32x4* ops) {
#pragma unroll
  for (int ks2 = 0; ks2 < 2; ++ks2)
    rotate_split<F16>(kr[ks2], kr[ks2 + 2], cs[ks2], 1.0f, ops[4 * ks2], ops[4 * ks2 + 1], ops[4 * ks2 + 2],
                      ops[4 * ks2 + 3]);
}

// The local window's slots s + k + t hold the same key at the same position for every query of
// the chunk, so their MFMA operands are formed once: pre[h][lb][x][lane], block b = b0 + lb.
template <bool F16>
__global__ __launch_bounds__(64) void local_keys_kernel(PfArgs a, int b0, u32x4* pre) {
  const int lane = threadIdx.x, n = lane & 15, j = lane >> 4;
  const int lb = blockIdx.x, h = blockIdx.y, b = b0 + lb;
  const int r = b * kBlk + n;
  const float2* t_hi = a.rope;
  const float2* t_lo = a.rope + (int64_t)a.nb * 64;
  const int fo = 8 * j;
  u32x4 ops[8];
  if (r < a.S) {
    float4 tl[8];
#pragma unroll
    for (int x = 0; x < 8; ++x) {
      const float2 t0 = t_lo[n * 64 + 32 * (x >> 2) + fo + 2 * (x & 3)];
      const float2 t1 = t_lo[n * 64 + 32 * (x >> 2) + fo + 2 * (x & 3) + 1];
      tl[x] = make_float4(t0.x, t0.y, t1.x, t1.y);
    }
    float2 cs[2][8];
    block_factors(t_hi + (int64_t)b * 64 + fo, [&](int x) { return tl[x]; }, cs);
    int64_t tok = a.N - a.l_eff + (r - a.s_eff - a.k_eff);
    if (a.pt) tok = paged_row(a.pt, a.page_lg, tok);
    const uint16_t* row = a.k + (int64_t)h * a.ksh + tok * a.kst + fo;
    u32x4 kr[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) kr[ks] = *(const u32x4*)(row + 32 * ks);
    key_operands<F16>(kr, cs, ops);
  } else {
#pragma unroll
    for (int x = 0; x < 8; ++x) ops[x] = u32x4{0u, 0u, 0u, 0u};
  }
  u32x4* o = pre + (((int64_t)h * gridDim.x + lb) * 8) * 64 + lane;
#pragma unroll
  for (int x = 0; x < 8; ++x) o[x * 64] = ops[x];
}

constexpr int kFacBlocks = 4;                              // blocks per round of shared rotary factors
constexpr size_t kFacLds = 2 * (size_t)kFacBlocks * 8 * 64 * sizeof(float4);

// PAGED: cache rows are found through the page table (selected slots come translated in idx).
template <int GT, bool F16, bool PAGED = false>
__global__ __launch_bounds__(256, 2) void attend_prefill_kernel(PfArgs a, int b_local0, int n_lb,
                                                                const u32x4* __restrict__ pre) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n = lane & 15, j = lane >> 4;
  const int qi = a.M - 1 - (blockIdx.x * 4 + wave);        // longest scopes are dispatched first
  const int h = blockIdx.y / a.nsub, g0 = (blockIdx.y % a.nsub) * GT;
  const int visible = a.S - (a.M - 1 - qi);                // slots this query sees; its own key is the last
  const int nblk = (visible + kBlk - 1) / kBlk;
  const int32_t* my_idx = a.idx + ((int64_t)qi * a.Hkv + h) * a.k_eff;
  const float2* t_hi = a.rope;
  const float2* t_lo = a.rope + (int64_t)a.nb * 64;
  const int fo = 8 * j;                                    // this lane's frequencies: fo + 32*ks2 + e

  // (cos, sin) of n*w for this lane's 16 frequencies: the same for all four waves, kept in LDS
  // as 8 rows of 64 float4 (two factors each) so that a lane reads its own 16 bytes per row
  __shared__ float4 tl_lds[8][64];
  if (wave == 0) {
#pragma unroll
    for (int x = 0; x < 8; ++x) {
      const float2 t0 = t_lo[n * 64 + 32 * (x >> 2) + fo + 2 * (x & 3)];
      const float2 t1 = t_lo[n * 64 + 32 * (x >> 2) + fo + 2 * (x & 3) + 1];
      tl_lds[x][lane] = make_float4(t0.x, t0.y, t1.x, t1.y);
    }
  }
  __syncthreads();

  // The rotary factors of a block of slots are the same for every query, so the four waves form them for
  // kFacBlocks blocks at a time, one block each, into LDS (two buffers: one barrier per round), and every wave
  // reads the factors of its current block from there: a quarter of the complex products and table loads.
  // The number of rounds is the workgroup's (wave 0 has the longest scope); a wave past the last query only
  // produces and waits.
  extern __shared__ __attribute__((aligned(16))) unsigned char pf_lds[];
  float4 (*fac)[kFacBlocks][8][64] = (float4 (*)[kFacBlocks][8][64])pf_lds;      // [2][kFacBlocks][8][64]
  const int vis0 = a.S - blockIdx.x * 4;                   // slots the workgroup's first wave sees
  const int nblk0 = (vis0 + kBlk - 1) / kBlk;
  const int n_round = ((nblk0 < b_local0 ? nblk0 : b_local0) + kFacBlocks - 1) / kFacBlocks;
  auto produce = [&](int round) {
    const int b = round * kFacBlocks + wave;
    if (round < n_round && b < a.nb) {
      float2 cs[2][8];
      block_factors(t_hi + (int64_t)b * 64 + fo, [&](int x) { return tl_lds[x][lane]; }, cs);
#pragma unroll
      for (int x = 0; x < 8; ++x) {
        const float2 c0 = cs[x >> 2][2 * (x & 3)], c1 = cs[x >> 2][2 * (x & 3) + 1];
        fac[round & 1][wave][x][lane] = make_float4(c0.x, c0.y, c1.x, c1.y);
      }
    }
  };
  produce(0);
  __syncthreads();
  if (qi < 0) {                                            // wave-uniform: as many barriers as the other waves pass
    for (int round = 0; round < n_round; ++round) {
      produce(round + 1);
      __syncthreads();
    }
    return;
  }

  // A operand: row m = lane % 16 -> head m / 2, half m % 2 (hi, lo) of the query rotated at the
  // slot of its own key and scaled by softmax_scale * log2(e); rows past the group are zero.
  typename Mm<F16>::op8 aop[4];
  {
    const int g = n >> 1, part = n & 1;
    const bool row_ok = g < GT && g0 + g < a.G;
    const int gg = row_ok ? g0 + g : 0;
    const uint16_t* qr = a.q + ((int64_t)qi * a.Hq + (int64_t)h * a.G + gg) * 128 + fo;
    const int pq = visible - 1;
    const float mul = row_ok ? a.scale_log2e : 0.f;
#pragma unroll
    for (int ks2 = 0; ks2 < 2; ++ks2) {
      float2 cs[8];
#pragma unroll
      for (int e = 0; e < 8; ++e)
        cs[e] = cmul(t_hi[(int64_t)(pq >> 4) * 64 + 32 * ks2 + fo + e], t_lo[(pq & 15) * 64 + 32 * ks2 + fo + e]);
      const u32x4 lo = *(const u32x4*)(qr + 32 * ks2), hi = *(const u32x4*)(qr + 64 + 32 * ks2);
      u32x4 ah, al, bh, bl;
      rotate_split<F16>(lo, hi, cs, mul, ah, al, bh, bl);
      aop[ks2] = as_op8<F16>(part ? al : ah);
      aop[ks2 + 2] = as_op8<F16>(part ? bl : bh);
    }
  }

  // weights of the current block, [head][slot], private to this wave
  __shared__ float p_lds[4][4][kBlk];
  float (*pw)[kBlk] = p_lds[wave];

  float m_run[GT], l_run[GT];
  f32x4 acc[8];                                            // tile t = 2u + parity: channels 32u + 2n + parity
#pragma unroll
  for (int g = 0; g < GT; ++g) { m_run[g] = kNegBig; l_run[g] = 0.f; }
#pragma unroll
  for (int t = 0; t < 8; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};

  auto slot_token = [&](int r) -> int {                    // cache row of slot r (clamped into the scope)
    const int rc = r < visible ? r : visible - 1;
    int tok;
    if (rc < a.s_eff) tok = rc;
    else if (rc < a.s_eff + a.k_eff) {
      tok = my_idx[rc - a.s_eff];
      if (PAGED && a.idx_is_rows) return tok;
    } else tok = (int)(a.N - a.l_eff) + (rc - a.s_eff - a.k_eff);
    return PAGED ? (int)paged_row(a.pt, a.page_lg, tok) : tok;   // a paged cache: the row of the head's pool slice
  };
  const uint16_t* kh = a.k + (int64_t)h * a.ksh + fo;
  const uint16_t* vh = a.v + (int64_t)h * a.vsh + 2 * n;
  auto load_key = [&](int tok, u32x4* kr) {
    const uint16_t* row = kh + (int64_t)tok * a.kst;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) kr[ks] = *(const u32x4*)(row + 32 * ks);
  };
  auto load_values = [&](const int* ts, uint32_t (*vw)[4]) {   // slots 4j .. 4j+3: channel pairs (32u + 2n, +1)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint16_t* row = vh + (int64_t)ts[i] * a.vst;
#pragma unroll
      for (int u = 0; u < 4; ++u) vw[i][u] = *(const uint32_t*)(row + 32 * u);
    }
  };
  const int pg = n >> 1, ppart = n & 1;                    // A-operand row of this lane in the P.V product

  // logits of one block from its 8 key operands
  auto logits = [&](const u32x4* ops) -> f32x4 {
    f32x4 c = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ks2 = 0; ks2 < 2; ++ks2) {
      c = Mm<F16>::mfma16(aop[ks2], as_op8<F16>(ops[4 * ks2]), c);
      c = Mm<F16>::mfma16(aop[ks2], as_op8<F16>(ops[4 * ks2 + 1]), c);
      c = Mm<F16>::mfma16(aop[ks2 + 2], as_op8<F16>(ops[4 * ks2 + 2]), c);
      c = Mm<F16>::mfma16(aop[ks2 + 2], as_op8<F16>(ops[4 * ks2 + 3]), c);
    }
    return c;
  };
  // online softmax of the block's logits and P.V
  auto finish_block = [&](int b, const f32x4& c, const uint32_t (*vw)[4]) {
    // lane (n, j) holds rows 4j .. 4j+3 of column n: heads 2j (rows 4j, 4j+1) and 2j+1
    const float s_even = c[0] + c[1], s_odd = c[2] + c[3];
    const bool valid = b * kBlk + n < visible;
    float sg[GT];
    bool grew = false;
#pragma unroll
    for (int g = 0; g < GT; ++g) {
      const float s = __shfl((g & 1) ? s_odd : s_even, n + 16 * (g >> 1), 64);
      sg[g] = valid ? s : kNegBig;
      grew = grew || (sg[g] > m_run[g]);
    }
    if (__any(grew)) {                                     // a new maximum: rare after the first blocks
      float corr[4] = {1.f, 1.f, 1.f, 1.f};
#pragma unroll
      for (int g = 0; g < GT; ++g) {
        const float m_new = fmaxf(m_run[g], row_max16(sg[g]));
        corr[g] = __builtin_amdgcn_exp2f(m_run[g] - m_new);
        l_run[g] *= corr[g];
        m_run[g] = m_new;
      }
      // accumulator rows 4j, 4j+1 belong to head 2j, rows 4j+2, 4j+3 to head 2j+1
      const float ce = j == 0 ? corr[0] : (j == 1 ? corr[2] : 1.f);
      const float co = j == 0 ? corr[1] : (j == 1 ? corr[3] : 1.f);
#pragma unroll
      for (int t = 0; t < 8; ++t) { acc[t][0] *= ce; acc[t][1] *= ce; acc[t][2] *= co; acc[t][3] *= co; }
    }
    float p[GT];
#pragma unroll
    for (int g = 0; g < GT; ++g) {
      p[g] = __builtin_amdgcn_exp2f(sg[g] - m_run[g]);      // invalid slots: 2^(-1e30) = 0
      l_run[g] += p[g];
    }
    // weights: slot-per-lane -> row-per-lane through LDS, then (hi, lo) bf16 halves by row parity
    if (j == 0) {
#pragma unroll
      for (int g = 0; g < GT; ++g) pw[g][n] = p[g];
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    float4 pr = make_float4(0.f, 0.f, 0.f, 0.f);
    if (pg < GT) pr = *(const float4*)&pw[pg][4 * j];
    uint32_t pa0 = Fmt<F16>::pack(pr.x, pr.y), pa1 = Fmt<F16>::pack(pr.z, pr.w);
    if (ppart) {
      const uint32_t l0 = Fmt<F16>::pack(pr.x - Fmt<F16>::lo(pa0), pr.y - Fmt<F16>::hi(pa0));
      const uint32_t l1 = Fmt<F16>::pack(pr.z - Fmt<F16>::lo(pa1), pr.w - Fmt<F16>::hi(pa1));
      pa0 = l0; pa1 = l1;
    }
    __builtin_amdgcn_wave_barrier();                        // the stage is rewritten by the next block
    const u32x2 pop = u32x2{pa0, pa1};
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      // even channel 32u + 2n: low halves of the four slots; odd channel: high halves
      const uint32_t e0 = __builtin_amdgcn_perm(vw[1][u], vw[0][u], 0x05040100u);
      const uint32_t e1 = __builtin_amdgcn_perm(vw[3][u], vw[2][u], 0x05040100u);
      const uint32_t o0 = __builtin_amdgcn_perm(vw[1][u], vw[0][u], 0x07060302u);
      const uint32_t o1 = __builtin_amdgcn_perm(vw[3][u], vw[2][u], 0x07060302u);
      acc[2 * u] = Fmt<F16>::mfma_pv(pop, u32x2{e0, e1}, acc[2 * u]);
      acc[2 * u + 1] = Fmt<F16>::mfma_pv(pop, u32x2{o0, o1}, acc[2 * u + 1]);
    }
  };

  // ---- phase 1: blocks with sink or selected slots: gather, rotate, split -----------------
  const int b_gen = nblk < b_local0 ? nblk : b_local0;
  {
    int tok = slot_token(n);
    u32x4 kr[4];
    if (b_gen > 0) load_key(tok, kr);
    int tok_next = slot_token(kBlk + n);
    for (int round = 0; round < n_round; ++round) {
      produce(round + 1);
      const int b_end = (round + 1) * kFacBlocks < b_gen ? (round + 1) * kFacBlocks : b_gen;
      for (int b = round * kFacBlocks; b < b_end; ++b) {
        uint32_t vw[4][4];
        int ts[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) ts[i] = __shfl(tok, 4 * j + i, 64);
        load_values(ts, vw);
        float2 cs[2][8];
#pragma unroll
        for (int x = 0; x < 8; ++x) {
          const float4 f = fac[round & 1][b - round * kFacBlocks][x][lane];
          cs[x >> 2][2 * (x & 3)] = make_float2(f.x, f.y);
          cs[x >> 2][2 * (x & 3) + 1] = make_float2(f.z, f.w);
        }
        u32x4 ops[8];
        key_operands<F16>(kr, cs, ops);
        // the key registers are free: request the next block's rows
        tok = tok_next;
        if (b + 1 < b_gen) load_key(tok, kr);
        tok_next = slot_token((b + 2) * kBlk + n);
        const f32x4 c = logits(ops);
        finish_block(b, c, vw);
      }
      __syncthreads();                                      // the other buffer is complete; this one may be rewritten
    }
  }
  // ---- phase 2: blocks of the local window: operands formed once for the whole chunk -------
  if (nblk > b_local0) {
    const u32x4* pp = pre + ((int64_t)h * n_lb * 8) * 64 + lane;
    const int tok0 = (int)(a.N - a.l_eff) - a.s_eff - a.k_eff;   // token of slot r is tok0 + r
    u32x4 ops[8];
#pragma unroll
    for (int x = 0; x < 8; ++x) ops[x] = pp[x * 64];
    auto local_rows = [&](int b, int* ts) {                 // cache rows of this lane's four slots of block b
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int r = b * kBlk + 4 * j + i;
        ts[i] = tok0 + (r < visible ? r : visible - 1);
        if (PAGED) ts[i] = (int)paged_row(a.pt, a.page_lg, ts[i]);
      }
    };
    int ts_next[4];
    if (PAGED) local_rows(b_local0, ts_next);
    for (int b = b_local0; b < nblk; ++b) {
      uint32_t vw[4][4];
      int ts[4];
      if (PAGED) {                                          // the next block's page entries are on their way
#pragma unroll
        for (int i = 0; i < 4; ++i) ts[i] = ts_next[i];
        if (b + 1 < nblk) local_rows(b + 1, ts_next);
      } else {
        local_rows(b, ts);
      }
      load_values(ts, vw);
      const f32x4 c = logits(ops);
      if (b + 1 < nblk) {                                   // the operand registers are free again
        const u32x4* nx = pp + (int64_t)(b + 1 - b_local0) * 8 * 64;
#pragma unroll
        for (int x = 0; x < 8; ++x) ops[x] = nx[x * 64];
      }
      finish_block(b, c, vw);
    }
  }

  // out[g][c] = (row 2g + row 2g+1) / l: lane (n, j) holds heads 2j, 2j+1 at channels 32u + 2n + parity
  float l_tot[GT];
#pragma unroll
  for (int g = 0; g < GT; ++g) l_tot[g] = group_sum<16>(l_run[g]);   // every 16-lane row holds the same partials per n
  if (j < 2) {
#pragma unroll
    for (int gg = 0; gg < 2; ++gg) {
      const int g = 2 * j + gg;
      if (g < GT && g0 + g < a.G) {
        float lt = l_tot[0];
#pragma unroll
        for (int x = 1; x < GT; ++x) lt = (g == x) ? l_tot[x] : lt;
        const float inv = 1.0f / lt;
        float* o = a.out + ((int64_t)qi * a.Hq + (int64_t)h * a.G + g0 + g) * 128 + 2 * n;
#pragma unroll
        for (int u = 0; u < 4; ++u)
          *(float2*)(o + 32 * u) = make_float2((acc[2 * u][2 * gg] + acc[2 * u][2 * gg + 1]) * inv,
                                               (acc[2 * u + 1][2 * gg] + acc[2 * u + 1][2 * gg + 1]) * inv);
      }
    }
  }
}

}  // namespace

namespace {
inline int pf_blocks(const Plan& pl) { return (pl.S + kBlk - 1) / kBlk; }
inline int pf_local0(const Plan& pl) { return (int)((pl.s_eff + pl.k_eff + kBlk - 1) / kBlk); }
}  // namespace

// Scratch of the chunk attention: rotary tables, then the local window's key operands.
size_t attend_prefill_table_bytes(const Plan& pl) {
  const size_t table = (size_t)(pf_blocks(pl) + kBlk) * 64 * sizeof(float2);
  const int n_lb = pf_blocks(pl) - pf_local0(pl);
  const size_t pre = n_lb > 0 ? (size_t)pl.Hkv * n_lb * 8 * 64 * 16 : 0;
  return (table + 255) / 256 * 256 + pre;
}

bool attend_prefill_applies(const Plan& pl) {
  return pl.M > 1 && (pl.dtype == kBF16 || pl.dtype == kF16) && pl.D == 128;
}

// out[i][hq] for all M queries; `table` is scratch of attend_prefill_table_bytes().
hipError_t launch_attend_prefill(const Plan& pl, const void* q, const void* k_cache,
                                 const void* v_cache, const int32_t* idx, float2* table, float* out,
                                 hipStream_t st, bool idx_is_rows) {
  PfArgs a;
  a.q = (const uint16_t*)q; a.k = (const uint16_t*)k_cache; a.v = (const uint16_t*)v_cache;
  a.idx = idx; a.rope = table; a.out = out;
  a.ksh = pl.ksh; a.kst = pl.kst; a.vsh = pl.vsh; a.vst = pl.vst; a.N = pl.N; a.pt = pl.pt; a.page_lg = pl.page_lg;
  a.idx_is_rows = idx_is_rows ? 1 : 0;
  a.Hq = pl.Hq; a.Hkv = pl.Hkv; a.G = pl.G; a.M = pl.M; a.S = pl.S;
  a.s_eff = (int)pl.s_eff; a.k_eff = pl.k_eff; a.l_eff = (int)pl.l_eff;
  a.nb = pf_blocks(pl);
  a.scale_log2e = pl.scale * 1.4426950408889634f;
  const int gt = pl.G < 4 ? pl.G : 4;
  a.nsub = (pl.G + gt - 1) / gt;
  const int n_tab = (a.nb + kBlk) * 64;
  hipLaunchKernelGGL(rope16_kernel, dim3((n_tab + 255) / 256), dim3(256), 0, st, table, a.nb,
                     log2((double)pl.theta));
  const int b_local0 = pf_local0(pl);
  const int n_lb = a.nb - b_local0 > 0 ? a.nb - b_local0 : 0;
  const size_t table_bytes = ((size_t)n_tab * sizeof(float2) + 255) / 256 * 256;
  u32x4* pre = (u32x4*)((char*)table + table_bytes);
  const bool f16 = pl.dtype == kF16;
  if (n_lb > 0) {
    if (f16) hipLaunchKernelGGL(local_keys_kernel<true>, dim3((unsigned)n_lb, (unsigned)pl.Hkv), dim3(64), 0, st, a, b_local0, pre);
    else     hipLaunchKernelGGL(local_keys_kernel<false>, dim3((unsigned)n_lb, (unsigned)pl.Hkv), dim3(64), 0, st, a, b_local0, pre);
  }
  const dim3 grid((unsigned)((pl.M + 3) / 4), (unsigned)(pl.Hkv * a.nsub));
#define REATTN_PF_LAUNCH_P(GT_, F16_, PAGED_)                                                                       \
  do {                                                                                                              \
    auto kern = attend_prefill_kernel<GT_, F16_, PAGED_>;                                                           \
    const hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kFacLds); \
    if (e != hipSuccess) return e;                                                                                  \
    hipLaunchKernelGGL(kern, grid, dim3(256), kFacLds, st, a, b_local0, n_lb, pre);                                 \
  } while (0)
#define REATTN_PF_LAUNCH(GT_)                                                                                       \
  do {                                                                                                              \
    if (a.pt) { if (f16) REATTN_PF_LAUNCH_P(GT_, true, true); else REATTN_PF_LAUNCH_P(GT_, false, true); }          \
    else      { if (f16) REATTN_PF_LAUNCH_P(GT_, true, false); else REATTN_PF_LAUNCH_P(GT_, false, false); }        \
  } while (0)
  switch (gt) {
    case 1: REATTN_PF_LAUNCH(1); break;
    case 2: REATTN_PF_LAUNCH(2); break;
    case 3: REATTN_PF_LAUNCH(3); break;
    default: REATTN_PF_LAUNCH(4); break;
  }
#undef REATTN_PF_LAUNCH
#undef REATTN_PF_LAUNCH_P
  return hipGetLastError();
}

}  // namespace reattn
