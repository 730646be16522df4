// Internal definitions shared by the HIP sources of libreattn (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

namespace reattn {

// ---- launch plan: clamped partition (Eq. 1) + workspace layout --------------
constexpr int kHistBits = 12;                 // first radix digit: top 12 bits of the ordered key
constexpr int kHistBins = 1 << kHistBits;     // 4096 bins, 16 KiB of LDS per workgroup
constexpr int kKeyShift = 32 - kHistBits;     // remaining 20 key bits are resolved among candidates
constexpr int kChunk = 8192;                  // middle positions per select/emit workgroup (256 x 32 bits)
constexpr int kChunkWords = kChunk / 32;
constexpr int kExactSlots = 64;               // workgroups (and score scratch rows) of the prefill redo path
constexpr int kRopeLo = 128;                  // positions covered by the low rotary table
constexpr int kRowMax = 65536;                // scores per row the one-workgroup top-k takes
constexpr int kPickMax = 32768;               // candidate pairs the one-workgroup pick of the filter path holds in registers
constexpr int kPickSlices = 1024;             // scan slices per row it can number through
constexpr int kFilterSampMax = 18 * 1024;     // sampled scores per row the scan's bound search holds in registers
__host__ __device__ inline int rope_rows_hi(int S) { return (S + kRopeLo - 1) / kRopeLo; }

// storage dtype codes as in reattn_dtype
constexpr int kF32 = 0, kBF16 = 1, kF16 = 2;
constexpr int kAggSum = 0, kAggMax = 1;       // reattn_agg
inline int64_t elem_bytes(int dtype) { return dtype == kF32 ? 4 : 2; }

struct Plan {
  int Hq, Hkv, D, G, dtype, M;
  int agg;                        // reattn_agg: how the G heads of a group become one score
  int64_t N, s_eff, l_eff, n_mid;
  int k_eff, S;
  int64_t ksh, kst, vsh, vst;     // strides in elements
  const int32_t* pt;              // page table of a paged cache (device), or nullptr
  int page_lg;                    // log2 of the page size
  float theta, scale;
  // top-k geometry for one row of n_mid scores
  int nchunks;                    // ceil(n_mid / kChunk)
  int64_t nwords;                 // bitmap words per row (nchunks * kChunkWords)
  // attention geometry
  int gt, nsub;                   // heads per attention workgroup, workgroups per KV head
  int split_len, nsplit;          // slots per attention workgroup, workgroups along S
  // query tile of the prefill path and workspace offsets (bytes)
  int m_tile;
  size_t off_scores, off_hist, off_pfx, off_ncand, off_cand, off_bitmap, off_cnt,
         off_idx, off_rope, off_rope16, off_part, off_qsplit,
         off_samp, off_thr, off_pcand, off_pcount, off_redo, off_exact, total;
  bool fused_prefill;             // M > 1 on the MFMA path with sampled thresholds
  // decode step over a long middle: no score array, the scan keeps only the pairs above a sampled bound
  bool filter;
  int f_rpb, f_nb;                // rows per scan slice, slices per score row (fixed by the plan, not by the device)
  int64_t f_step, f_samp_stride;  // every f_step-th key of the middle is sampled; floats between two rows' samples
  uint32_t f_nsamp, f_rho;        // samples per row; rank of the sampled score that serves as the bound
  size_t off_fsamp, off_fcnt, off_fcand;   // laid over the score / candidate / bitmap blocks of the other selection
};

// ---- host-side launchers (one per .hip file) -------------------------------
hipError_t launch_fill_u32(uint32_t* p, int64_t n, uint32_t v, hipStream_t st);
// rows of a token-major [n_tok][Hkv][D] block on their way into a head-major cache, in 16-byte pieces
struct AppendJob {
  const void* k_new; const void* v_new; void* k_cache; void* v_cache;
  int64_t first_tok; int n_tok;
};
// clears `rows` first-digit histograms, fills the rotary table and copies the appended rows (each part optional):
// the small jobs that precede a layer's scan share one launch
hipError_t launch_prep(const Plan& pl, int rows, uint32_t* hist, float2* rope, hipStream_t st,
                       const AppendJob* append = nullptr);
hipError_t launch_cache_append(const Plan& pl, int64_t first_tok, int n_tok, const void* k_new, const void* v_new,
                               void* k_cache, void* v_cache, hipStream_t st);
// append: rows of new tokens past the middle, copied into the caches by the same launch
hipError_t launch_score_scan(const Plan& pl, const void* q, int n_query, const void* k_cache,
                             float* scores, uint32_t* hist, hipStream_t st, const AppendJob* append = nullptr);
void prefill_sampling(const Plan& pl, int64_t* stride, int64_t* n_s, uint32_t* rho, uint32_t* cap);
// Filter path of a decode step (plan.filter): sampled scores (+ the rotary table), the scan that keeps the pairs
// at or above the sampled bound, the exact pick out of them (one workgroup per score row; a row whose bound
// missed or whose pairs do not fit recomputes its scores and selects exactly, slowly).
int scan_rows_per_block_for(int64_t n_mid, int64_t score_rows, int max_rows, int n_cu);
hipError_t launch_decode_sample(const Plan& pl, const void* q, const void* k_cache, float* samp, float2* rope,
                                uint32_t* redo_count, hipStream_t st);
hipError_t launch_score_scan_filter(const Plan& pl, const void* q, const void* k_cache, const float* samp,
                                    uint2* cand, uint32_t* segcnt, hipStream_t st, const AppendJob* append = nullptr);
hipError_t launch_decode_pick(const Plan& pl, const void* q, const void* k_cache, const uint2* cand,
                              const uint32_t* segcnt, int32_t* idx, uint32_t* redo_count, hipStream_t st);
// Key splits of the fused filter (few query tiles would leave most of the chip idle) and the capacity of one
// split's part of a row's candidate segment.
void prefill_filter_splits(const Plan& pl, uint32_t cap, int* n_split, uint32_t* cap_split);
size_t cand_topk_lds(const Plan& pl);
hipError_t launch_sample_threshold(const Plan& pl, int n_query, const float* samp, int64_t n_s,
                                   int64_t row_stride, uint32_t rho, float* thr, hipStream_t st);
hipError_t launch_cand_topk(const Plan& pl, int n_query, const uint2* cand, const uint32_t* ccount,
                            uint32_t cap, int n_split, int32_t* idx, uint32_t* redo, hipStream_t st);
hipError_t launch_row_exact(const Plan& pl, int n_query, const void* q, const void* k_cache,
                            const uint32_t* redo, float* scratch, int n_slots, int32_t* idx,
                            hipStream_t st);
hipError_t launch_read_probe(const void* buf, size_t bytes, hipStream_t st);
size_t score_gemm_qsplit_bytes(const Plan& pl);
hipError_t launch_qsplit(const Plan& pl, const void* q, int q_first, int n_query, void* q_split,
                         hipStream_t st);
hipError_t launch_score_gemm_store(const Plan& pl, int n_query, const void* k_cache,
                                   const void* q_split, int64_t key_step, int64_t n_keys,
                                   float* scores, int64_t score_stride, hipStream_t st);
hipError_t launch_score_gemm_filter(const Plan& pl, int n_query, const void* k_cache,
                                    const void* q_split, const float* thr, uint2* cand,
                                    uint32_t* ccount, uint32_t cap, int n_split, hipStream_t st);
hipError_t launch_score_gemm_discard(const Plan& pl, int n_query, const void* k_cache,
                                     const void* q_split, float* sink, hipStream_t st);
hipError_t launch_score_gemm(const Plan& pl, const void* q, int q_first, int n_query,
                             const void* k_cache, float* scores, void* q_split, hipStream_t st);
// The kernel that reads a row's histogram last (one workgroup per row) leaves it zeroed: the next
// selection over the same workspace needs no clearing launch.
hipError_t launch_topk(const Plan& pl, int rows, const float* scores, bool hist_ready,
                       uint32_t* hist, uint32_t* pfx, uint32_t* ncand, int32_t* cand,
                       uint32_t* bitmap, uint32_t* cnt, int32_t* idx, hipStream_t st);
hipError_t launch_gather_rope(const Plan& pl, const void* k_cache, const void* v_cache,
                              const int32_t* idx, float* k_sel, void* v_sel, hipStream_t st);
hipError_t launch_attend(const Plan& pl, bool fused, const void* q, int q_first, int n_query,
                         const void* k_src, const void* v_src, const int32_t* idx,
                         const float2* rope, float* part, float* out, hipStream_t st,
                         const int32_t* k_dyn = nullptr, int64_t idx_stride = -1, int seq_heads = 0);
// vote selection (vote.hip)
int vote_list_len(int vote_k);
bool vote_scan_applies(const Plan& pl);
int vote_queries_per_launch(const Plan& pl, int vote_k);
int vote_gemm_splits(const Plan& pl, int n_query, int list_len);
hipError_t launch_vote_gemm(const Plan& pl, const void* q, int n_query, const void* k_cache, int list_len,
                            uint64_t* part, hipStream_t st);
size_t vote_part_bytes(const Plan& pl, int n_query, int vote_k);
hipError_t launch_head_topk_scan(const Plan& pl, const void* q, int n_query, const void* k_cache,
                                 int vote_k, uint64_t* part, int32_t* head_topk, hipStream_t st);
void vote_merge_layout(const Plan& pl, int64_t n_votes, size_t* counts_bytes, size_t* seg_bytes,
                       size_t* comp_bytes);
hipError_t launch_vote_merge(const Plan& pl, const int32_t* lists, int64_t n_rows, int kk, int kc, int span,
                             uint32_t* counts, int32_t* seg, uint64_t* comp, int32_t* sel, int32_t* n_sel,
                             hipStream_t st, int n_seq = 1, int64_t sel_stride = 0);
// a decode step's selection in two launches: the fused score + per-head top-k scan, then one workgroup per
// sequence that closes the per-head lists, counts the votes, expands the spans and copies the appended rows
bool vote_decode_applies(const Plan& pl, int kk, int kc, int n_seq);
hipError_t launch_vote_decode_scan(const Plan& pl, const void* q, const void* k_cache, int kk, uint64_t* part,
                                   int* n_cand, hipStream_t st);
hipError_t launch_vote_decode_merge(const Plan& pl, const uint64_t* part, int n_cand, int kk, int kc, int span,
                                    int32_t* sel, int32_t* n_sel, hipStream_t st, int n_seq, int64_t sel_stride,
                                    const AppendJob* append);

bool attend_shared_applies(const Plan& pl);
void attend_shared_layout(const Plan& pl, size_t* kp, size_t* vp, size_t* qp, size_t* part);
hipError_t launch_attend_shared(const Plan& pl, const void* q, const void* k_cache, const void* v_cache,
                                const int32_t* sel, const int32_t* n_sel, const float2* rope, void* kp,
                                void* vp, void* qp, float* part, float* out, hipStream_t st);
// merges split partials [(rows)][nsplit][D + 2] = (max, sum, unnormalised output) into out [rows][D]
hipError_t launch_attend_combine(int D, int64_t rows, int nsplit, const float* part, float* out, hipStream_t st);
size_t attend_prefill_table_bytes(const Plan& pl);
bool attend_prefill_applies(const Plan& pl);
hipError_t launch_attend_prefill(const Plan& pl, const void* q, const void* k_cache,
                                 const void* v_cache, const int32_t* idx, float2* table, float* out,
                                 hipStream_t st, bool idx_is_rows = false);
// rows[i] = pool row of token idx[i] (paged caches; rows may be idx itself)
hipError_t launch_translate_rows(const Plan& pl, const int32_t* idx, int32_t* rows, int64_t n, hipStream_t st);

// ---- device helpers ---------------------------------------------------------
#ifdef __HIPCC__

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// Storage tags of the 16-bit formats: bf16 travels as uint16_t, IEEE half as f16bits.
struct f16bits { uint16_t v; };
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float f16_lo(uint32_t w) { return (float)__builtin_bit_cast(f16x2, w)[0]; }
__device__ __forceinline__ float f16_hi(uint32_t w) { return (float)__builtin_bit_cast(f16x2, w)[1]; }
__device__ __forceinline__ float f16_one(uint16_t h) { return (float)__builtin_bit_cast(_Float16, h); }

// The two 16-bit matrix-core operand formats behind one interface: F16 = false is bf16, true IEEE half.
typedef __bf16 mm_bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 mm_f16x8 __attribute__((ext_vector_type(8)));
typedef float mm_f32x4 __attribute__((ext_vector_type(4)));
typedef float mm_f32x8 __attribute__((ext_vector_type(8)));
typedef float mm_f32x16 __attribute__((ext_vector_type(16)));
template <bool F16> struct Mm;
template <> struct Mm<false> {
  typedef mm_bf16x8 op8;
  static __device__ __forceinline__ mm_f32x16 mfma32(op8 a, op8 b, mm_f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
  }
  static __device__ __forceinline__ mm_f32x4 mfma16(op8 a, op8 b, mm_f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
  }
  static __device__ __forceinline__ float widen(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }
  static __device__ __forceinline__ uint16_t narrow(float x) {           // round to nearest even
    uint32_t u = __float_as_uint(x);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
  }
};
template <> struct Mm<true> {
  typedef mm_f16x8 op8;
  static __device__ __forceinline__ mm_f32x16 mfma32(op8 a, op8 b, mm_f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
  }
  static __device__ __forceinline__ mm_f32x4 mfma16(op8 a, op8 b, mm_f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
  }
  static __device__ __forceinline__ float widen(uint16_t h) { return f16_one(h); }
  static __device__ __forceinline__ uint16_t narrow(float x) { return __builtin_bit_cast(uint16_t, (_Float16)x); }
};

// Paged cache: token t of the sequence -> row of every head's slice of the pool.
__device__ __forceinline__ int64_t paged_row(const int32_t* pt, int lg, int64_t tok) {
  return ((int64_t)pt[tok >> lg] << lg) | (tok & (((int64_t)1 << lg) - 1));
}

// Paged cache, streaming kernels: a workgroup keeps the first pool rows of the pages its slice of tokens spans
// in LDS (one spare entry behind the last), and a wave's tile of at most 64 consecutive tokens lies in at most
// two of them (pages hold 64 tokens or more): the two bases are read once per tile into scalars and a lane
// picks one by comparing its offset in the first page against the page size.
__device__ __forceinline__ void slice_pages_fill(int32_t* pages, const int32_t* pt, int lg, int64_t tok0, int nrows,
                                                 int n_threads) {
  const int64_t pg0 = tok0 >> lg;
  const int n_pg = nrows > 0 ? (int)(((tok0 + nrows - 1) >> lg) - pg0) + 1 : 0;
  for (int i = threadIdx.x; i <= n_pg; i += n_threads) pages[i] = i < n_pg ? pt[pg0 + i] << lg : 0;
  __syncthreads();
}
struct TilePages {
  int32_t first, second_less_page, in0, page;
  // pool row of token (tile's first token + c)
  __device__ __forceinline__ int32_t row(int c) const {
    const int32_t in = in0 + c;
    return (in < page ? first : second_less_page) + in;
  }
};
// tok = the tile's first token (wave-uniform), tok0 = the slice's first token
__device__ __forceinline__ TilePages tile_pages(const int32_t* pages, int lg, int64_t tok0, int64_t tok) {
  const int i = __builtin_amdgcn_readfirstlane((int)((tok >> lg) - (tok0 >> lg)));
  TilePages t;
  t.page = 1 << lg;
  t.first = __builtin_amdgcn_readfirstlane(pages[i]);
  t.second_less_page = __builtin_amdgcn_readfirstlane(pages[i + 1]) - t.page;
  t.in0 = __builtin_amdgcn_readfirstlane((int)(tok & (t.page - 1)));
  return t;
}

// Rows of a token-major [n_tok][Hkv][D] block on their way into a head-major cache, as kernels see them.
struct AppendArgs {
  const u32x4* k_new; const u32x4* v_new; char* k_cache; char* v_cache;
  int64_t first_tok, n_vec, ksh_b, kst_b, vsh_b, vst_b;    // n_vec 16-byte pieces (0: nothing to append)
  int Hkv, vec_per_row;
  const int32_t* pt; int page_lg;                          // paged cache, or nullptr
};
// piece i of the block: row i / vec_per_row = t * Hkv + h
__device__ __forceinline__ void append_piece(const AppendArgs& a, int64_t i) {
  const int piece = (int)(i % a.vec_per_row);
  const int64_t row = i / a.vec_per_row;
  const int h = (int)(row % a.Hkv);
  const int64_t t = row / a.Hkv;
  const int64_t r = a.pt ? paged_row(a.pt, a.page_lg, a.first_tok + t) : a.first_tok + t;
  *(u32x4*)(a.k_cache + h * a.ksh_b + r * a.kst_b + piece * 16) = a.k_new[i];
  *(u32x4*)(a.v_cache + h * a.vsh_b + r * a.vst_b + piece * 16) = a.v_new[i];
}
inline AppendArgs append_args(const Plan& pl, const AppendJob* j) {
  AppendArgs a;
  const int64_t eb = elem_bytes(pl.dtype);
  a.k_new = nullptr; a.v_new = nullptr; a.k_cache = nullptr; a.v_cache = nullptr;
  a.first_tok = 0; a.n_vec = 0; a.pt = pl.pt; a.page_lg = pl.page_lg;
  a.Hkv = pl.Hkv; a.vec_per_row = (int)(pl.D * eb / 16);
  a.ksh_b = pl.ksh * eb; a.kst_b = pl.kst * eb; a.vsh_b = pl.vsh * eb; a.vst_b = pl.vst * eb;
  if (j && j->n_tok > 0) {
    a.k_new = (const u32x4*)j->k_new; a.v_new = (const u32x4*)j->v_new;
    a.k_cache = (char*)j->k_cache; a.v_cache = (char*)j->v_cache;
    a.first_tok = j->first_tok; a.n_vec = (int64_t)j->n_tok * pl.Hkv * a.vec_per_row;
  }
  return a;
}

// Entry j of the two-level rotary table: rows [0, n_hi) hold the angles of positions 128 a, rows
// [n_hi, n_hi + 128) those of positions b < 128; half = D / 2 entries per row.  Angles in fp64.
__device__ __forceinline__ float2 rope_table_entry(int64_t j, int S, int half, int D, double log2_theta) {
  const int n_hi = rope_rows_hi(S);
  const int row = (int)(j / half), c = (int)(j % half);
  const int r = row < n_hi ? row * kRopeLo : row - n_hi;
  const double w = exp2(-2.0 * (double)c / (double)D * log2_theta);
  // whole turns taken off in fp64 first (exact to ~1e-11 rad at position 131,071): the library routine then
  // stays on its small-argument path
  const double turns = (double)r * w * 0.15915494309189535;
  double sn, cs;
  sincos((turns - rint(turns)) * 6.283185307179586, &sn, &cs);
  return make_float2((float)cs, (float)sn);
}

// Order-preserving image of an fp32 score: larger float <=> larger key.  -0 maps to +0's key.
__device__ __forceinline__ uint32_t score_key(float x) {
  uint32_t u = __float_as_uint(x);
  if (u == 0x80000000u) u = 0u;
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Sum over a group of 2^k adjacent lanes with DPP row operations (no LDS traffic).
template <int CTRL>
__device__ __forceinline__ float dpp_add(float v) {
  int moved = __builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true);
  return v + __int_as_float(moved);
}
// quad_perm [1,0,3,2] = 0xB1, quad_perm [2,3,0,1] = 0x4E, row_half_mirror = 0x141, row_mirror = 0x140
template <int LANES>
__device__ __forceinline__ float group_sum(float v) {
  static_assert(LANES == 4 || LANES == 8 || LANES == 16 || LANES == 32, "group size");
  v = dpp_add<0xB1>(v);
  v = dpp_add<0x4E>(v);
  if (LANES >= 8) v = dpp_add<0x141>(v);
  if (LANES >= 16) v = dpp_add<0x140>(v);
  if (LANES >= 32) v += __shfl_xor(v, 16, 64);
  return v;
}

// Inclusive prefix sum over the NT threads of a workgroup; `total` gets the grand sum.
template <int NT>
__device__ __forceinline__ uint32_t block_scan_incl(uint32_t v, uint32_t* wsum, uint32_t& total) {
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

// bins[0..NB) counts, higher bin = larger key.  Finds the bin d with
// count(bins > d) < k <= count(bins >= d) and `above` = count(bins > d).  1 <= k <= total.
template <int NT, int NB, typename BinPtr>
__device__ __forceinline__ void find_kth_bin(BinPtr bins, uint32_t k, uint32_t* sh,
                                             uint32_t& bin, uint32_t& above) {
  constexpr int BPT = NB / NT;
  static_assert(BPT >= 1 && BPT * NT == NB, "bins per thread");
  uint32_t loc[BPT], sum = 0;
#pragma unroll
  for (int i = 0; i < BPT; ++i) { loc[i] = bins[threadIdx.x * BPT + i]; sum += loc[i]; }
  uint32_t total;
  const uint32_t incl = block_scan_incl<NT>(sum, sh, total);
  const uint32_t higher = total - incl;          // entries owned by threads above this one
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

#endif  // __HIPCC__
}  // namespace reattn
