// C ABI of libreattn: argument validation, launch planning, workspace layout.
// Everything here runs on the host and returns before the enqueued kernels finish.
#include "../../include/reattn.h"
#include "common.hpp"

#include <cmath>
#include <cstring>
#include <mutex>

using namespace reattn;

namespace {

constexpr size_t kAlign = 256;
inline size_t up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }
inline bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

// Decides whether a decode step takes the filter path (no score array) and fixes its geometry: the sampling
// step and rank, the scan's slices.  Everything follows from the params alone (the scan is cut for the 256
// compute units of the part this library is built for), so the workspace layout never depends on a device.
static_assert(kAggSum == REATTN_AGG_SUM && kAggMax == REATTN_AGG_MAX && kF32 == REATTN_F32 && kBF16 == REATTN_BF16 && kF16 == REATTN_F16,
              "the kernels' constants are the header's");

bool filter_plan(Plan* pl, int route) {
  pl->filter = false;
  if (pl->M != 1 || pl->n_mid <= kRowMax || pl->k_eff <= 0 || route == REATTN_ROUTE_SCORES) return false;
  if (pl->agg != REATTN_AGG_SUM) return false;        // the sampling and the exact redo score group sums
  // Measured on MI355X: the route costs a sampling launch, ~5 us at the head of every scan workgroup and a
  // one-workgroup pick (~37 us in all) against ~40 us for histogram + select + refine + emit over the written
  // scores; it wins once the scores no longer fit one round of workgroups (their bursts then fall into the
  // next round's reads) and is level at a million tokens of 8 KV heads; below that the written scores win.
  if (route != REATTN_ROUTE_FILTER && pl->n_mid * (int64_t)pl->Hkv < ((int64_t)1 << 22)) return false;
  const int64_t target = pl->n_mid > ((int64_t)1 << 21) ? 16384 : 8192;   // longer rows: a tighter bound, or the pairs outgrow the pick
  int64_t step = pl->n_mid / target;
  if (step < 1) step = 1;
  const int64_t ns = (pl->n_mid + step - 1) / step;
  const double p = (double)pl->k_eff / (double)pl->n_mid;
  const double mu = (double)ns * p;                     // sampled scores expected above the row's k-th score
  const double r = mu + 6.0 * std::sqrt(mu * (1.0 - p) + 1.0) + 2.0;
  if (r >= (double)ns) return false;                    // nearly everything is selected: nothing to filter
  const double expect = r * (double)step;               // pairs at or above the bound, and six deviations on top
  const double most = expect * (1.0 + 6.0 / std::sqrt(r)) + 64.0;
  if (most > (double)kPickMax || ns > kFilterSampMax) return false;
  const int rpb = scan_rows_per_block_for(pl->n_mid, pl->Hkv, 16384, 512);   // two workgroups of 512 threads per CU, 32 rows per thread
  const int64_t nb = (pl->n_mid + rpb - 1) / rpb;
  if (nb > kPickSlices) return false;
  pl->filter = true;
  pl->f_rpb = rpb; pl->f_nb = (int)nb; pl->f_step = step;
  pl->f_nsamp = (uint32_t)ns; pl->f_rho = (uint32_t)r; pl->f_samp_stride = (ns + 3) / 4 * 4;
  return true;
}

int make_plan(const reattn_params* p, Plan* out) {
  if (!p) return REATTN_ERR_NULL;
  Plan pl;
  std::memset(&pl, 0, sizeof pl);
  if (p->n_q_heads < 1 || p->n_kv_heads < 1 || p->n_q_heads % p->n_kv_heads) return REATTN_ERR_SHAPE;
  if (p->n_q_heads / p->n_kv_heads > 16) return REATTN_ERR_SHAPE;
  if (p->head_dim != 64 && p->head_dim != 128) return REATTN_ERR_SHAPE;
  if (p->dtype != REATTN_F32 && p->dtype != REATTN_BF16 && p->dtype != REATTN_F16) return REATTN_ERR_DTYPE;
  if (p->agg != REATTN_AGG_SUM && p->agg != REATTN_AGG_MAX) return REATTN_ERR_DTYPE;
  if (p->n_ctx < 1 || p->n_ctx > 0x7fffffffLL) return REATTN_ERR_RANGE;
  if (p->n_query < 1 || p->n_query > p->n_ctx || p->n_query > 65535) return REATTN_ERR_RANGE;
  if (p->n_sink < 0 || p->n_local < 1 || p->top_k < 0) return REATTN_ERR_RANGE;
  if (!(p->rope_theta > 1.0f) || !std::isfinite(p->rope_theta)) return REATTN_ERR_RANGE;
  if (!(p->softmax_scale >= 0.0f) || !std::isfinite(p->softmax_scale)) return REATTN_ERR_RANGE;
  if (p->max_position < 0) return REATTN_ERR_RANGE;
  if (p->route != REATTN_ROUTE_AUTO && p->route != REATTN_ROUTE_FILTER && p->route != REATTN_ROUTE_SCORES) return REATTN_ERR_RANGE;

  pl.Hq = p->n_q_heads; pl.Hkv = p->n_kv_heads; pl.D = p->head_dim; pl.G = pl.Hq / pl.Hkv;
  pl.dtype = p->dtype; pl.M = p->n_query; pl.N = p->n_ctx; pl.agg = p->agg;
  pl.s_eff = p->n_sink < pl.N ? p->n_sink : pl.N;
  pl.l_eff = p->n_local < pl.N - pl.s_eff ? p->n_local : pl.N - pl.s_eff;
  pl.n_mid = pl.N - pl.s_eff - pl.l_eff;
  pl.k_eff = (int)(p->top_k < pl.n_mid ? p->top_k : pl.n_mid);
  const int64_t S = pl.s_eff + pl.k_eff + pl.l_eff;
  // a chunk lies inside the local window; with an empty middle the kept entries are simply all
  // N tokens in order, so any M <= N is causal attention (the first prefill chunk of l_global + l_local)
  if (pl.M > pl.l_eff && pl.n_mid > 0) return REATTN_ERR_RANGE;
  if (p->max_position > 0 && S > p->max_position) return REATTN_ERR_WINDOW;
  pl.S = (int)S;

  const int64_t eb = elem_bytes(pl.dtype);
  const bool kdef = p->k_stride_head == 0 && p->k_stride_tok == 0;
  const bool vdef = p->v_stride_head == 0 && p->v_stride_tok == 0;
  pl.kst = kdef ? pl.D : p->k_stride_tok;  pl.ksh = kdef ? pl.N * pl.D : p->k_stride_head;
  pl.vst = vdef ? pl.D : p->v_stride_tok;  pl.vsh = vdef ? pl.N * pl.D : p->v_stride_head;
  if (pl.kst < pl.D || pl.vst < pl.D || pl.ksh < 0 || pl.vsh < 0) return REATTN_ERR_SHAPE;
  if (pl.Hkv > 1 && (pl.ksh < pl.D || pl.vsh < pl.D)) return REATTN_ERR_SHAPE;   // heads must not alias
  if ((pl.kst * eb) % 16 || (pl.ksh * eb) % 16 || (pl.vst * eb) % 16 || (pl.vsh * eb) % 16)
    return REATTN_ERR_ALIGN;
  pl.pt = nullptr; pl.page_lg = 0;
  if (p->page_table || p->page_size) {                 // paged cache: pools [Hkv][P * page_size][D]
    if (!p->page_table) return REATTN_ERR_NULL;
    if (p->page_size < 64 || (p->page_size & (p->page_size - 1))) return REATTN_ERR_RANGE;
    if (kdef || vdef) return REATTN_ERR_SHAPE;         // the pool's extent is not the sequence's: strides must be given
    if (pl.ksh / pl.D > 0x7fffffffLL || pl.vsh / pl.D > 0x7fffffffLL) return REATTN_ERR_RANGE;   // pool rows are int32
    pl.pt = p->page_table;
    while ((1 << pl.page_lg) < p->page_size) ++pl.page_lg;
  }

  pl.theta = p->rope_theta;
  pl.scale = p->softmax_scale > 0.f ? p->softmax_scale : 1.0f / std::sqrt((float)pl.D);

  pl.nchunks = (int)((pl.n_mid + kChunk - 1) / kChunk);
  pl.nwords = (int64_t)pl.nchunks * kChunkWords;

  pl.nsub = (pl.G + 3) / 4;
  pl.gt = (pl.G + pl.nsub - 1) / pl.nsub;
  {
    // slots per workgroup: 256 (16 per 16-lane group) unless that leaves CUs idle
    const int64_t units = (int64_t)pl.Hkv * pl.nsub * pl.M;
    int64_t want = (768 + units - 1) / units;             // workgroups along S: three per CU keep the row gathers in flight
    if (want < 1) want = 1;
    int64_t len = (S + want - 1) / want;
    len = (len + 63) / 64 * 64;
    if (len < 64) len = 64;
    if (units >= 256 && len < S) len = (S + 63) / 64 * 64; // plenty of (query, head) units: no split
    pl.split_len = (int)len;
    pl.nsplit = (int)((S + len - 1) / len);
  }

  // query tile of the prefill path: per-tile scratch stays near 4 GiB
  const size_t per_query = (size_t)pl.Hkv * ((size_t)pl.n_mid * 4 + (size_t)pl.nchunks * kChunk * 4 +
                                             (size_t)kHistBins * 4 + (size_t)pl.nwords * 4 +
                                             (size_t)pl.nchunks * 12 + 64);
  int64_t mt = (int64_t)(((size_t)2 << 30) / (per_query ? per_query : 1));
  if (mt < 1) mt = 1;
  if (mt > pl.M) mt = pl.M;
  if (mt * pl.Hkv > 65535) mt = 65535 / pl.Hkv;
  if (mt < 1) return REATTN_ERR_SHAPE;
  pl.m_tile = (int)mt;

  const size_t rows = (size_t)pl.m_tile * pl.Hkv;
  // What a warm workspace keeps from one decode step to the next (reattn_params.ws_warm) comes first, at
  // offsets that do not move as the context grows: the histograms (left zeroed by their last reader) and the
  // rotary table.
  size_t off = 0;
  pl.off_hist = off;   off += up(rows * kHistBins * 4);
  pl.off_rope = off;   off += up((size_t)(rope_rows_hi(pl.S) + kRopeLo) * (pl.D / 2) * sizeof(float2));
  const size_t front = off;
  pl.off_scores = off; off += up(rows * (size_t)pl.n_mid * 4);
  pl.off_pfx = off;    off += up(rows * (size_t)pl.nchunks * 4);
  pl.off_ncand = off;  off += up(rows * (size_t)pl.nchunks * 4);
  pl.off_cand = off;   off += up(rows * (size_t)pl.nchunks * kChunk * 4);
  pl.off_bitmap = off; off += up(rows * (size_t)pl.nwords * 4);
  pl.off_cnt = off;    off += up(rows * (size_t)pl.nchunks * 4);
  if (filter_plan(&pl, p->route)) {                              // the same bytes, laid out for the filter path
    size_t f = front;
    pl.off_fsamp = f;  f += up((size_t)pl.Hkv * (size_t)pl.f_samp_stride * 4);
    pl.off_fcnt = f;   f += up((size_t)pl.Hkv * (size_t)pl.f_nb * 4 + 4 + (size_t)pl.Hkv * 4);   // + the redo list
    pl.off_fcand = f;  f += up((size_t)pl.Hkv * (size_t)pl.f_nb * (size_t)pl.f_rpb * 8);
    if (f > off) off = f;
  }
  pl.off_idx = off;    off += up((size_t)pl.M * pl.Hkv * (size_t)pl.k_eff * 4);
  pl.off_rope16 = off; off += up(attend_prefill_applies(pl) ? attend_prefill_table_bytes(pl) : 0);
  pl.off_part = off;   off += up((size_t)pl.M * pl.Hq * (size_t)pl.nsplit * (pl.D + 2) * 4);
  pl.off_qsplit = off; off += up(pl.M > 1 ? score_gemm_qsplit_bytes(pl) : 0);
  // fused prefill selection: MFMA scores filtered against sampled thresholds
  pl.fused_prefill = pl.M > 1 && (pl.dtype == REATTN_BF16 || pl.dtype == REATTN_F16) && pl.D == 128 && pl.k_eff > 0 &&
                     pl.agg == REATTN_AGG_SUM &&
                     cand_topk_lds(pl) <= (size_t)128 * 1024;
  if (pl.fused_prefill) {
    int64_t stride, n_s; uint32_t rho, cap;
    prefill_sampling(pl, &stride, &n_s, &rho, &cap);
    int nz; uint32_t cap_z;
    prefill_filter_splits(pl, cap, &nz, &cap_z);
    const size_t prow = (size_t)pl.M * pl.Hkv;
    pl.off_samp = off;   off += up(prow * (size_t)((n_s + 3) / 4 * 4) * 4);   // rows padded to 16 bytes
    pl.off_thr = off;    off += up(prow * 4);
    pl.off_pcand = off;  off += up(prow * (size_t)nz * cap_z * 8);
    pl.off_pcount = off; off += up(prow * (size_t)nz * 4);
    pl.off_redo = off;   off += up((prow + 1) * 4);
    pl.off_exact = off;  off += up((size_t)kExactSlots * (size_t)pl.n_mid * 4);
  }
  pl.total = off ? off : kAlign;
  *out = pl;
  return REATTN_OK;
}

struct Ws {
  float* scores; uint32_t* hist; uint32_t* pfx; uint32_t* ncand; int32_t* cand;
  uint32_t* bitmap; uint32_t* cnt; int32_t* idx; float2* rope; float* part; void* qsplit;
  float* fsamp; uint32_t* fcnt; uint32_t* fredo; uint2* fcand;     // filter path (same bytes as scores .. cnt)
};

int bind_ws(const Plan& pl, void* ws, size_t ws_bytes, Ws* w) {
  if (!ws || ws_bytes < pl.total) return REATTN_ERR_WORKSPACE;
  if ((uintptr_t)ws % kAlign) return REATTN_ERR_ALIGN;
  char* b = (char*)ws;
  w->scores = (float*)(b + pl.off_scores);   w->hist = (uint32_t*)(b + pl.off_hist);
  w->pfx = (uint32_t*)(b + pl.off_pfx);     w->ncand = (uint32_t*)(b + pl.off_ncand);
  w->cand = (int32_t*)(b + pl.off_cand);     w->bitmap = (uint32_t*)(b + pl.off_bitmap);
  w->cnt = (uint32_t*)(b + pl.off_cnt);      w->idx = (int32_t*)(b + pl.off_idx);
  w->rope = (float2*)(b + pl.off_rope);      w->part = (float*)(b + pl.off_part);
  w->qsplit = b + pl.off_qsplit;
  w->fsamp = (float*)(b + pl.off_fsamp);     w->fcnt = (uint32_t*)(b + pl.off_fcnt);
  w->fredo = w->fcnt + (size_t)pl.Hkv * (pl.filter ? pl.f_nb : 0);
  w->fcand = (uint2*)(b + pl.off_fcand);
  return REATTN_OK;
}

// M > 1 on 16-bit storage / D = 128 takes the MFMA kernel; everything else streams per query.
// (the matrix-core contraction scores the group SUM, (sum_g q_g) . k: max aggregation streams too)
inline bool use_mfma(const Plan& pl) {
  return pl.M > 1 && (pl.dtype == REATTN_BF16 || pl.dtype == REATTN_F16) && pl.D == 128 && pl.agg == REATTN_AGG_SUM;
}

inline int hip_rc(hipError_t e) { return e == hipSuccess ? REATTN_OK : REATTN_ERR_HIP; }

// Stage 2 over the cache: chunks on bf16 / D = 128 take the MFMA kernel (one wave per query
// and KV head), everything else the flash-decoding kernel with its split-S combine.
int attend_cache(const Plan& pl, const Ws& w, char* ws, const void* q, const void* k_cache,
                 const void* v_cache, const int32_t* idx, float* out, hipStream_t st) {
  if (attend_prefill_applies(pl)) {                        // an empty middle (M > l) is the same walk: every slot is its own token
    bool rows = false;
    if (pl.pt && pl.k_eff > 0) {
      // paged cache: the selected tokens' pool rows are looked up once, into the workspace's index block
      // (in place when the indices already live there: then nobody else reads them)
      const int rc = hip_rc(launch_translate_rows(pl, idx, w.idx, (int64_t)pl.M * pl.Hkv * pl.k_eff, st));
      if (rc) return rc;
      idx = w.idx; rows = true;
    }
    return hip_rc(launch_attend_prefill(pl, q, k_cache, v_cache, idx, (float2*)(ws + pl.off_rope16),
                                        out, st, rows));
  }
  return hip_rc(launch_attend(pl, true, q, 0, pl.M, k_cache, v_cache, idx, w.rope, w.part, out, st));
}

// score -> top-k for the queries [q0, q0 + nq), then the caller attends.
// `ev`, when given, holds REATTN_N_STAGES + 1 events recorded at the stage boundaries.
inline void mark(hipEvent_t* ev, int i, hipStream_t st) { if (ev) (void)hipEventRecord(ev[i], st); }

// hist_clean: the previous selection over this workspace left the histograms of these rows zeroed.
int select_tile(const Plan& pl, const Ws& w, const void* q, int q0, int nq, const void* k_cache,
                int32_t* idx_all, bool rope_too, hipEvent_t* ev, hipStream_t st, const AppendJob* append = nullptr,
                bool hist_clean = false) {
  const int rows = nq * pl.Hkv;
  const size_t eb = (size_t)elem_bytes(pl.dtype);
  const char* qt = (const char*)q + (size_t)q0 * pl.Hq * pl.D * eb;
  if (pl.filter) {                                     // a decode step over a long middle: sample -> filtering scan -> pick
    const bool with_scan = append && append->first_tok >= pl.s_eff + pl.n_mid;
    int rc = REATTN_OK;
    if (append && !with_scan)                          // rows inside the middle must be in place before anything reads it
      rc = hip_rc(launch_cache_append(pl, append->first_tok, append->n_tok, append->k_new, append->v_new,
                                      append->k_cache, append->v_cache, st));
    if (!rc) rc = hip_rc(launch_decode_sample(pl, qt, k_cache, w.fsamp, rope_too ? w.rope : nullptr, w.fredo, st));
    mark(ev, 1, st);
    if (!rc) rc = hip_rc(launch_score_scan_filter(pl, qt, k_cache, w.fsamp, w.fcand, w.fcnt, st, with_scan ? append : nullptr));
    mark(ev, 2, st);
    if (!rc) rc = hip_rc(launch_decode_pick(pl, qt, k_cache, w.fcand, w.fcnt, idx_all, w.fredo, st));
    mark(ev, 3, st);
    return rc;
  }
  // new rows past the middle ride with the scan (which never reads them); otherwise with the clearing launch
  const bool with_scan = append && pl.k_eff > 0 && append->first_tok >= pl.s_eff + pl.n_mid;
  const int clear_rows = pl.k_eff > 0 && !hist_clean ? rows : 0;
  int rc = REATTN_OK;
  if (clear_rows || rope_too || (append && !with_scan))
    rc = hip_rc(launch_prep(pl, clear_rows, w.hist, rope_too ? w.rope : nullptr, st, with_scan ? nullptr : append));
  mark(ev, 1, st);
  if (rc || pl.k_eff == 0) { mark(ev, 2, st); mark(ev, 3, st); return rc; }
  rc = hip_rc(launch_score_scan(pl, qt, nq, k_cache, w.scores, w.hist, st, with_scan ? append : nullptr));
  mark(ev, 2, st);
  if (rc) return rc;
  rc = hip_rc(launch_topk(pl, rows, w.scores, true, w.hist, w.pfx, w.ncand, w.cand, w.bitmap,
                          w.cnt, idx_all + (size_t)q0 * pl.Hkv * pl.k_eff, st));
  mark(ev, 3, st);
  return rc;
}

// Prefill selection on the matrix cores: sample -> thresholds -> fused filter -> exact per-row
// top-k over the candidates -> redo of the (rare) rows whose threshold missed.
int fused_prefill_select(const Plan& pl, const Ws& w, char* ws, const void* q, const void* k_cache,
                         int32_t* idx, hipEvent_t* ev, hipStream_t st) {
  int64_t stride, n_s; uint32_t rho, cap;
  prefill_sampling(pl, &stride, &n_s, &rho, &cap);
  int nz; uint32_t cap_z;
  prefill_filter_splits(pl, cap, &nz, &cap_z);
  float* samp = (float*)(ws + pl.off_samp);
  float* thr = (float*)(ws + pl.off_thr);
  uint2* cand = (uint2*)(ws + pl.off_pcand);
  uint32_t* ccount = (uint32_t*)(ws + pl.off_pcount);
  uint32_t* redo = (uint32_t*)(ws + pl.off_redo);
  float* exact = (float*)(ws + pl.off_exact);
  // the histogram-clear of prep doubles as the clear of the redo counter (one word)
  int rc = hip_rc(launch_prep(pl, 0, nullptr, w.rope, st));
  if (!rc) rc = hip_rc(launch_fill_u32(redo, 1, 0u, st));
  if (!rc) rc = hip_rc(launch_qsplit(pl, q, 0, pl.M, w.qsplit, st));
  const int64_t samp_stride = (n_s + 3) / 4 * 4;         // 16-byte rows: the sampled scores leave in float4 stores
  if (!rc) rc = hip_rc(launch_score_gemm_store(pl, pl.M, k_cache, w.qsplit, stride, n_s, samp, samp_stride, st));
  if (!rc) rc = hip_rc(launch_sample_threshold(pl, pl.M, samp, n_s, samp_stride, rho, thr, st));
  mark(ev, 1, st);
  if (!rc) rc = hip_rc(launch_score_gemm_filter(pl, pl.M, k_cache, w.qsplit, thr, cand, ccount, cap_z, nz, st));
  mark(ev, 2, st);
  if (!rc) rc = hip_rc(launch_cand_topk(pl, pl.M, cand, ccount, cap_z, nz, idx, redo, st));
  if (!rc) rc = hip_rc(launch_row_exact(pl, pl.M, q, k_cache, redo, exact, kExactSlots, idx, st));
  mark(ev, 3, st);
  return rc;
}

int run_layer(const reattn_params* p, bool decode_only, const void* q, const void* k_cache,
              const void* v_cache, int32_t* idx_out, float* out, void* ws, size_t ws_bytes,
              void* stream, hipEvent_t* ev = nullptr, bool rope_ready = false, const AppendJob* append = nullptr,
              bool hist_clean = false) {
  Plan pl;
  int rc = make_plan(p, &pl);
  if (rc) return rc;
  if (decode_only && pl.M != 1) return REATTN_ERR_RANGE;
  if (!q || !k_cache || !v_cache || !out) return REATTN_ERR_NULL;
  if (!aligned16(q) || !aligned16(k_cache) || !aligned16(v_cache) || !aligned16(out))
    return REATTN_ERR_ALIGN;
  Ws w;
  rc = bind_ws(pl, ws, ws_bytes, &w);
  if (rc) return rc;
  hipStream_t st = (hipStream_t)stream;
  int32_t* idx = idx_out ? idx_out : w.idx;
  mark(ev, 0, st);
  if (pl.fused_prefill) {
    if (append) {                                      // not the decode shape: the rows go in with a launch of their own
      rc = hip_rc(launch_cache_append(pl, append->first_tok, append->n_tok, append->k_new, append->v_new,
                                      append->k_cache, append->v_cache, st));
      if (rc) return rc;
    }
    rc = fused_prefill_select(pl, w, (char*)ws, q, k_cache, idx, ev, st);
    if (rc) return rc;
    rc = attend_cache(pl, w, (char*)ws, q, k_cache, v_cache, idx, out, st);
    mark(ev, 4, st);
    return rc;
  }
  for (int q0 = 0; q0 < pl.M; q0 += pl.m_tile) {
    const int nq = pl.M - q0 < pl.m_tile ? pl.M - q0 : pl.m_tile;
    rc = select_tile(pl, w, q, q0, nq, k_cache, idx, q0 == 0 && !rope_ready, ev, st, q0 == 0 ? append : nullptr,
                     hist_clean && q0 == 0);
    if (rc) return rc;
  }
  rc = attend_cache(pl, w, (char*)ws, q, k_cache, v_cache, idx, out, st);
  mark(ev, 4, st);
  return rc;
}

}  // namespace

extern "C" {

int reattn_version(void) { return 100; }
size_t reattn_params_bytes(void) { return sizeof(reattn_params); }
size_t reattn_vote_bytes(void) { return sizeof(reattn_vote); }

const char* reattn_status_string(int s) {
  switch (s) {
    case REATTN_OK: return "ok";
    case REATTN_ERR_NULL: return "a required pointer is NULL";
    case REATTN_ERR_SHAPE: return "unsupported head counts, head_dim or strides";
    case REATTN_ERR_DTYPE: return "unknown storage dtype or aggregation";
    case REATTN_ERR_RANGE: return "n_ctx, n_query, n_sink, n_local, top_k or rope parameters out of range";
    case REATTN_ERR_WINDOW: return "attention scope exceeds max_position";
    case REATTN_ERR_WORKSPACE: return "workspace missing or too small";
    case REATTN_ERR_ALIGN: return "pointer or stride not 16-byte aligned (workspace: 256)";
    case REATTN_ERR_HIP: return "HIP launch failed";
    case REATTN_ERR_STATIC_LIMIT: return "problem needs more scratch than the no-allocation entry point holds";
    default: return "unknown status";
  }
}

int reattn_validate(const reattn_params* p) {
  Plan pl;
  return make_plan(p, &pl);
}

int reattn_scope(const reattn_params* p, int64_t* n_sink_eff, int64_t* n_local_eff,
                 int64_t* n_mid, int64_t* k_eff, int64_t* scope) {
  Plan pl;
  const int rc = make_plan(p, &pl);
  if (rc) return rc;
  if (n_sink_eff) *n_sink_eff = pl.s_eff;
  if (n_local_eff) *n_local_eff = pl.l_eff;
  if (n_mid) *n_mid = pl.n_mid;
  if (k_eff) *k_eff = pl.k_eff;
  if (scope) *scope = pl.S;
  return REATTN_OK;
}

size_t reattn_workspace_bytes(const reattn_params* p) {
  Plan pl;
  return make_plan(p, &pl) == REATTN_OK ? pl.total : 0;
}

int reattn_score(const reattn_params* p, const void* q, const void* k_cache, float* scores,
                 void* ws, size_t ws_bytes, void* stream) {
  Plan pl;
  int rc = make_plan(p, &pl);
  if (rc) return rc;
  if (!q || !k_cache || (!scores && pl.n_mid > 0)) return REATTN_ERR_NULL;
  if (!aligned16(q) || !aligned16(k_cache)) return REATTN_ERR_ALIGN;
  hipStream_t st = (hipStream_t)stream;
  if (use_mfma(pl)) {                       // dense contraction on the matrix cores
    Ws w;
    rc = bind_ws(pl, ws, ws_bytes, &w);
    if (rc) return rc;
    return hip_rc(launch_score_gemm(pl, q, 0, pl.M, k_cache, scores, w.qsplit, st));
  }
  const int per = 65535 / pl.Hkv;
  const size_t eb = (size_t)elem_bytes(pl.dtype);
  for (int q0 = 0; q0 < pl.M && !rc; q0 += per) {
    const int nq = pl.M - q0 < per ? pl.M - q0 : per;
    rc = hip_rc(launch_score_scan(pl, (const char*)q + (size_t)q0 * pl.Hq * pl.D * eb, nq, k_cache,
                                  scores + (size_t)q0 * pl.Hkv * pl.n_mid, nullptr, st));
  }
  return rc;
}

int reattn_topk(const reattn_params* p, const float* scores, int32_t* idx, void* ws,
                size_t ws_bytes, void* stream) {
  Plan pl;
  int rc = make_plan(p, &pl);
  if (rc) return rc;
  if (pl.k_eff == 0) return REATTN_OK;
  if (!scores || !idx) return REATTN_ERR_NULL;
  Ws w;
  rc = bind_ws(pl, ws, ws_bytes, &w);
  if (rc) return rc;
  hipStream_t st = (hipStream_t)stream;
  for (int q0 = 0; q0 < pl.M; q0 += pl.m_tile) {
    const int nq = pl.M - q0 < pl.m_tile ? pl.M - q0 : pl.m_tile;
    const int rows = nq * pl.Hkv;
    rc = hip_rc(launch_prep(pl, rows, w.hist, nullptr, st));
    if (rc) return rc;
    rc = hip_rc(launch_topk(pl, rows, scores + (size_t)q0 * pl.Hkv * pl.n_mid, false, w.hist,
                            w.pfx, w.ncand, w.cand, w.bitmap, w.cnt,
                            idx + (size_t)q0 * pl.Hkv * pl.k_eff, st));
    if (rc) return rc;
  }
  return REATTN_OK;
}

int reattn_gather_rope(const reattn_params* p, const void* k_cache, const void* v_cache,
                       const int32_t* idx, float* k_sel, void* v_sel, void* stream) {
  Plan pl;
  int rc = make_plan(p, &pl);
  if (rc) return rc;
  if (!k_cache || !v_cache || !k_sel || !v_sel || (!idx && pl.k_eff > 0)) return REATTN_ERR_NULL;
  if (!aligned16(k_cache) || !aligned16(v_cache) || !aligned16(k_sel) || !aligned16(v_sel))
    return REATTN_ERR_ALIGN;
  return hip_rc(launch_gather_rope(pl, k_cache, v_cache, idx, k_sel, v_sel, (hipStream_t)stream));
}

int reattn_attend(const reattn_params* p, const void* q, const float* k_sel, const void* v_sel,
                  float* out, void* ws, size_t ws_bytes, void* stream) {
  Plan pl;
  int rc = make_plan(p, &pl);
  if (rc) return rc;
  if (!q || !k_sel || !v_sel || !out) return REATTN_ERR_NULL;
  if (!aligned16(q) || !aligned16(k_sel) || !aligned16(v_sel) || !aligned16(out))
    return REATTN_ERR_ALIGN;
  Ws w;
  rc = bind_ws(pl, ws, ws_bytes, &w);
  if (rc) return rc;
  hipStream_t st = (hipStream_t)stream;
  rc = hip_rc(launch_prep(pl, 0, nullptr, w.rope, st));
  if (rc) return rc;
  return hip_rc(launch_attend(pl, false, q, 0, pl.M, k_sel, v_sel, nullptr, w.rope, w.part, out, st));
}

int reattn_decode_step(const reattn_params* p, const void* q, const void* k_cache,
                       const void* v_cache, int32_t* idx_out, float* out, void* ws,
                       size_t ws_bytes, void* stream) {
  const bool warm = p && p->ws_warm != 0;
  return run_layer(p, true, q, k_cache, v_cache, idx_out, out, ws, ws_bytes, stream, nullptr, warm, nullptr, warm);
}

// ---- the decode step for callers that cannot allocate ----------------------------------------
// The step's scratch lives in the library's own device image instead of a caller's buffer.  The
// array's name is only a host-side stand-in: its device address is asked for once per device
// (every GPU holds its own copy at its own address) and that pointer is what the kernels get.
}  // extern "C"

static __device__ __align__(256) unsigned char scratch[REATTN_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_lock;
void* g_scratch_ptr[kMaxDevices];

// Device address of `scratch` on the current device; nullptr (and *err) when the runtime refuses.
void* static_scratch(hipError_t* err) {
  int dev = 0;
  *err = hipGetDevice(&dev);
  if (*err != hipSuccess) return nullptr;
  if (dev < 0 || dev >= kMaxDevices) { *err = hipErrorInvalidDevice; return nullptr; }
  std::lock_guard<std::mutex> hold(g_scratch_lock);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    *err = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (*err != hipSuccess || !ptr) { if (*err == hipSuccess) *err = hipErrorInvalidSymbol; return nullptr; }
    g_scratch_ptr[dev] = ptr;
  }
  return g_scratch_ptr[dev];
}
}  // namespace

extern "C" {

size_t reattn_static_scratch_bytes(void) { return (size_t)REATTN_STATIC_SCRATCH_BYTES; }

int reattn_decode_step_static(const reattn_params* p, const void* q, const void* k_cache,
                              const void* v_cache, int32_t* idx_out, float* out, void* stream) {
  Plan pl;
  const int rc = make_plan(p, &pl);
  if (rc) return rc;
  if (pl.M != 1) return REATTN_ERR_RANGE;
  if (pl.total > (size_t)REATTN_STATIC_SCRATCH_BYTES) return REATTN_ERR_STATIC_LIMIT;   // decided on the host, before any launch
  hipError_t e;
  void* ws = static_scratch(&e);
  if (!ws) return REATTN_ERR_HIP;
  // every kernel of the step starts from what the step itself wrote or cleared (the first launch zeroes
  // the histograms), so what the previous call left in the array does not matter -- unless the caller
  // vouches for it (ws_warm: the previous step through this entry point on this GPU had the same shape)
  const bool warm = p->ws_warm != 0;
  return run_layer(p, true, q, k_cache, v_cache, idx_out, out, ws, (size_t)REATTN_STATIC_SCRATCH_BYTES, stream,
                   nullptr, warm, nullptr, warm);
}

int reattn_prefill_chunk(const reattn_params* p, const void* q, const void* k_cache,
                         const void* v_cache, int32_t* idx_out, float* out, void* ws,
                         size_t ws_bytes, void* stream) {
  return run_layer(p, false, q, k_cache, v_cache, idx_out, out, ws, ws_bytes, stream);
}

// ---- vote selection ----------------------------------------------------------------------
namespace {
struct VotePlan {
  Plan pl;                 // base plan with k_eff = cap (largest selection)
  int kk, kc, span;        // votes per list, centres, span (all clamped)
  int n_seq;               // sequences folded into the head axis
  size_t off_rope, off_apart, off_part, off_lists, off_counts, off_seg, off_comp, off_sel, off_nsel, off_kp, off_vp,
         off_qp, off_spart, total;
};

int make_vote_plan(const reattn_params* p, const reattn_vote* v, VotePlan* out) {
  if (!p || !v) return REATTN_ERR_NULL;
  if (v->vote_k < 1 || v->vote_k > 8 || v->n_centres < 1 || v->n_centres > 1024 || v->span < 1)
    return REATTN_ERR_RANGE;
  reattn_params pp = *p;
  const int64_t want = (int64_t)v->n_centres * v->span;
  pp.top_k = want > 0x7fffffffLL ? 0x7fffffff : (int32_t)want;       // make_plan clamps to N_mid: cap
  VotePlan vp;
  int rc = make_plan(&pp, &vp.pl);
  if (rc) return rc;
  const Plan& pl = vp.pl;
  vp.kk = (int)(v->vote_k < pl.n_mid ? v->vote_k : pl.n_mid);
  vp.kc = (int)(v->n_centres < pl.n_mid ? v->n_centres : pl.n_mid);
  {
    // a span longer than twice the middle covers it wherever its centre lies
    const int64_t widest = 2 * pl.n_mid + 2;
    vp.span = (int)(v->span < widest ? v->span : (widest < 0x7fffffffLL ? widest : 0x7fffffffLL));
  }
  if (pl.n_mid > 0 && !vote_scan_applies(pl)) return REATTN_ERR_SHAPE;
  vp.n_seq = v->n_seq > 1 ? v->n_seq : 1;
  if (v->n_seq < 0) return REATTN_ERR_RANGE;
  if (vp.n_seq > 1) {
    if (pl.M != 1) return REATTN_ERR_RANGE;            // a folded batch is a decode step
    if (pl.Hq % vp.n_seq || pl.Hkv % vp.n_seq) return REATTN_ERR_SHAPE;
    if ((int64_t)(pl.Hq / vp.n_seq) * vp.kk > 1024) return REATTN_ERR_SHAPE;
  }
  const int per = pl.n_mid > 0 ? vote_queries_per_launch(pl, vp.kk > 0 ? vp.kk : 1) : 1;
  // own layout: of the group-sum path's scratch only the rotary table and (for the flash-decoding
  // kernel) the split-S partials are needed here
  size_t off = 0;
  vp.off_rope = off;    off += up((size_t)(rope_rows_hi(pl.S) + kRopeLo) * (pl.D / 2) * sizeof(float2));
  vp.off_apart = off;   off += up(attend_shared_applies(pl) ? 0 : (size_t)pl.M * pl.Hq * (size_t)pl.nsplit * (pl.D + 2) * 4);
  size_t part_bytes = 0;                               // the last launch may take fewer query rows
  if (pl.n_mid > 0) {
    part_bytes = vote_part_bytes(pl, per, vp.kk > 0 ? vp.kk : 1);
    const size_t tail = pl.M % per ? vote_part_bytes(pl, pl.M % per, vp.kk > 0 ? vp.kk : 1) : 0;
    if (tail > part_bytes) part_bytes = tail;
  }
  vp.off_part = off;    off += up(part_bytes);
  vp.off_lists = off;   off += up((size_t)pl.M * pl.Hq * (vp.kk > 0 ? vp.kk : 1) * 4);
  size_t cb, sb, mb;
  vote_merge_layout(pl, (int64_t)pl.M * pl.Hq * vp.kk, &cb, &sb, &mb);
  vp.off_counts = off;  off += up(cb);
  vp.off_seg = off;     off += up(sb);
  vp.off_comp = off;    off += up(mb);
  vp.off_sel = off;     off += up((size_t)vp.n_seq * (pl.k_eff > 0 ? pl.k_eff : 1) * 4);
  vp.off_nsel = off;    off += up((size_t)vp.n_seq * 4);
  size_t kpb = 0, vpb = 0, qpb = 0, spb = 0;
  if (attend_shared_applies(pl)) attend_shared_layout(pl, &kpb, &vpb, &qpb, &spb);
  vp.off_kp = off;      off += up(kpb);
  vp.off_vp = off;      off += up(vpb);
  vp.off_qp = off;      off += up(qpb);
  vp.off_spart = off;   off += up(spb);
  vp.total = off;
  *out = vp;
  return REATTN_OK;
}

int vote_topk_impl(const VotePlan& vp, const void* q, const void* k_cache, int32_t* head_topk,
                   char* ws, hipStream_t st) {
  const Plan& pl = vp.pl;
  if (vp.kk == 0) return REATTN_OK;
  const int per = vote_queries_per_launch(pl, vp.kk);
  const size_t eb = (size_t)elem_bytes(pl.dtype);
  int rc = REATTN_OK;
  for (int q0 = 0; q0 < pl.M && !rc; q0 += per) {
    const int nq = pl.M - q0 < per ? pl.M - q0 : per;
    rc = hip_rc(launch_head_topk_scan(pl, (const char*)q + (size_t)q0 * pl.Hq * pl.D * eb, nq, k_cache,
                                      vp.kk, (uint64_t*)(ws + vp.off_part),
                                      head_topk + (size_t)q0 * pl.Hq * vp.kk, st));
  }
  return rc;
}

int vote_merge_impl(const VotePlan& vp, const int32_t* head_topk, int32_t* sel, int32_t* n_sel,
                    char* ws, hipStream_t st) {
  const Plan& pl = vp.pl;
  if (vp.kk == 0 || vp.kc == 0)                        // empty middle: nothing can be selected
    return hip_rc(launch_fill_u32((uint32_t*)n_sel, vp.n_seq, 0u, st));
  return hip_rc(launch_vote_merge(pl, head_topk, (int64_t)pl.M * pl.Hq, vp.kk, vp.kc, vp.span,
                                  (uint32_t*)(ws + vp.off_counts), (int32_t*)(ws + vp.off_seg),
                                  (uint64_t*)(ws + vp.off_comp), sel, n_sel, st, vp.n_seq,
                                  pl.k_eff > 0 ? pl.k_eff : 1));
}
}  // namespace

extern "C" size_t reattn_vote_workspace_bytes(const reattn_params* p, const reattn_vote* v) {
  VotePlan vp;
  return make_vote_plan(p, v, &vp) == REATTN_OK ? vp.total : 0;
}

extern "C" int reattn_vote_topk(const reattn_params* p, const reattn_vote* v, const void* q,
                                const void* k_cache, int32_t* head_topk, void* ws, size_t ws_bytes,
                                void* stream) {
  VotePlan vp;
  int rc = make_vote_plan(p, v, &vp);
  if (rc) return rc;
  if (vp.kk == 0) return REATTN_OK;
  if (!q || !k_cache || !head_topk) return REATTN_ERR_NULL;
  if (!aligned16(q) || !aligned16(k_cache)) return REATTN_ERR_ALIGN;
  if (!ws || ws_bytes < vp.total) return REATTN_ERR_WORKSPACE;
  if ((uintptr_t)ws % kAlign) return REATTN_ERR_ALIGN;
  return vote_topk_impl(vp, q, k_cache, head_topk, (char*)ws, (hipStream_t)stream);
}

extern "C" int reattn_vote_merge(const reattn_params* p, const reattn_vote* v, const int32_t* head_topk,
                                 int32_t* sel, int32_t* n_sel, void* ws, size_t ws_bytes, void* stream) {
  VotePlan vp;
  int rc = make_vote_plan(p, v, &vp);
  if (rc) return rc;
  if (!n_sel || (vp.kk > 0 && (!head_topk || !sel))) return REATTN_ERR_NULL;
  if (!ws || ws_bytes < vp.total) return REATTN_ERR_WORKSPACE;
  if ((uintptr_t)ws % kAlign) return REATTN_ERR_ALIGN;
  return vote_merge_impl(vp, head_topk, sel, n_sel, (char*)ws, (hipStream_t)stream);
}

static int vote_layer_impl(const reattn_params* p, const reattn_vote* v, const void* q, const void* k_cache,
                           const void* v_cache, int32_t* sel_out, int32_t* n_sel_out, float* out, void* ws,
                           size_t ws_bytes, void* stream, hipEvent_t* ev, bool rope_ready = false,
                           const AppendJob* append = nullptr) {
  VotePlan vp;
  int rc = make_vote_plan(p, v, &vp);
  if (rc) return rc;
  if (!q || !k_cache || !v_cache || !out) return REATTN_ERR_NULL;
  if (!aligned16(q) || !aligned16(k_cache) || !aligned16(v_cache) || !aligned16(out)) return REATTN_ERR_ALIGN;
  if (!ws || ws_bytes < vp.total) return REATTN_ERR_WORKSPACE;
  if ((uintptr_t)ws % kAlign) return REATTN_ERR_ALIGN;
  const Plan& pl = vp.pl;
  char* b = (char*)ws;
  hipStream_t st = (hipStream_t)stream;
  int32_t* lists = (int32_t*)(b + vp.off_lists);
  int32_t* sel = sel_out ? sel_out : (int32_t*)(b + vp.off_sel);
  int32_t* n_sel = n_sel_out ? n_sel_out : (int32_t*)(b + vp.off_nsel);
  mark(ev, 0, st);
  if (vote_decode_applies(pl, vp.kk, vp.kc, vp.n_seq)) {
    // a decode step: the scan, then one workgroup per sequence for lists + votes + spans (+ the appended rows)
    int n_cand = 0;
    rc = hip_rc(launch_vote_decode_scan(pl, q, k_cache, vp.kk, (uint64_t*)(b + vp.off_part), &n_cand, st));
    mark(ev, 1, st);
    if (!rc) rc = hip_rc(launch_vote_decode_merge(pl, (const uint64_t*)(b + vp.off_part), n_cand, vp.kk, vp.kc, vp.span,
                                                  sel, n_sel, st, vp.n_seq, pl.k_eff > 0 ? pl.k_eff : 1, append));
  } else {
    if (append) rc = hip_rc(launch_cache_append(pl, append->first_tok, append->n_tok, append->k_new, append->v_new,
                                                append->k_cache, append->v_cache, st));
    if (!rc) rc = vote_topk_impl(vp, q, k_cache, lists, b, st);
    mark(ev, 1, st);
    if (!rc) rc = vote_merge_impl(vp, lists, sel, n_sel, b, st);
  }
  mark(ev, 2, st);
  if (rc) return rc;
  float2* rope = (float2*)(b + vp.off_rope);
  if (!rope_ready) rc = hip_rc(launch_prep(pl, 0, nullptr, rope, st));
  if (rc) return rc;
  // one shared index row for every (query, KV head); its length is read on the device
  if (attend_shared_applies(pl))       // a chunk on bf16 / D = 128: packed once, flash attention on the matrix cores
    rc = hip_rc(launch_attend_shared(pl, q, k_cache, v_cache, sel, n_sel, rope, b + vp.off_kp, b + vp.off_vp,
                                     b + vp.off_qp, (float*)(b + vp.off_spart), out, st));
  else
    rc = hip_rc(launch_attend(pl, true, q, 0, pl.M, k_cache, v_cache, sel, rope, (float*)(b + vp.off_apart), out,
                              st, n_sel, vp.n_seq > 1 ? (pl.k_eff > 0 ? pl.k_eff : 1) : 0,
                              vp.n_seq > 1 ? pl.Hkv / vp.n_seq : 0));
  mark(ev, 3, st);
  return rc;
}

extern "C" int reattn_vote_layer(const reattn_params* p, const reattn_vote* v, const void* q,
                                 const void* k_cache, const void* v_cache, int32_t* sel_out,
                                 int32_t* n_sel_out, float* out, void* ws, size_t ws_bytes, void* stream) {
  // a decode step on a warm workspace: the rotary table (first in the vote layout too) is already there
  const bool warm = p && p->ws_warm != 0 && p->n_query == 1;
  return vote_layer_impl(p, v, q, k_cache, v_cache, sel_out, n_sel_out, out, ws, ws_bytes, stream, nullptr, warm);
}

extern "C" int reattn_vote_layer_timed(const reattn_params* p, const reattn_vote* v, const void* q,
                                       const void* k_cache, const void* v_cache, int32_t* sel_out,
                                       int32_t* n_sel_out, float* out, void* ws, size_t ws_bytes,
                                       void* stream, float* stage_ms) {
  if (!stage_ms) return REATTN_ERR_NULL;
  constexpr int kStages = REATTN_N_VOTE_STAGES;
  hipEvent_t ev[kStages + 1];
  int made = 0;
  for (; made <= kStages; ++made)
    if (hipEventCreate(&ev[made]) != hipSuccess) break;
  int rc = made == kStages + 1 ? REATTN_OK : REATTN_ERR_HIP;
  const bool warm = p && p->ws_warm != 0 && p->n_query == 1;
  if (!rc) rc = vote_layer_impl(p, v, q, k_cache, v_cache, sel_out, n_sel_out, out, ws, ws_bytes, stream, ev, warm);
  if (!rc) {
    if (hipEventSynchronize(ev[kStages]) != hipSuccess) rc = REATTN_ERR_HIP;
    for (int i = 0; i < kStages && !rc; ++i)
      if (hipEventElapsedTime(&stage_ms[i], ev[i], ev[i + 1]) != hipSuccess) rc = REATTN_ERR_HIP;
  }
  for (int i = 0; i < made; ++i) (void)hipEventDestroy(ev[i]);
  return rc;
}

// ---- streaming prefill of one layer ---------------------------------------------------------
namespace {
// Explicit strides of the cache described by p (whose n_ctx is the final length L).
void cache_strides(const reattn_params* p, int64_t* ksh, int64_t* kst, int64_t* vsh, int64_t* vst) {
  const bool kdef = p->k_stride_head == 0 && p->k_stride_tok == 0;
  const bool vdef = p->v_stride_head == 0 && p->v_stride_tok == 0;
  *kst = kdef ? p->head_dim : p->k_stride_tok;  *ksh = kdef ? p->n_ctx * p->head_dim : p->k_stride_head;
  *vst = vdef ? p->head_dim : p->v_stride_tok;  *vsh = vdef ? p->n_ctx * p->head_dim : p->v_stride_head;
}

// Chunk c of the prefilling phase: tokens [*s, *e).  Returns false past the last chunk.
bool sequence_chunk(const reattn_params* p, int32_t chunk, int64_t c, int64_t* s, int64_t* e) {
  const int64_t L = p->n_ctx;
  int64_t first = (int64_t)p->n_sink + p->n_local;
  if (first > L) first = L;
  if (c == 0) { *s = 0; *e = first; return true; }
  *s = first + (c - 1) * (int64_t)chunk;
  if (*s >= L) return false;
  *e = *s + chunk < L ? *s + chunk : L;
  return true;
}

// p as seen by the chunk [s, e): the cache holds e tokens, the chunk's rows are the queries.
reattn_params chunk_params(const reattn_params* p, int64_t s, int64_t e) {
  reattn_params pp = *p;
  cache_strides(p, &pp.k_stride_head, &pp.k_stride_tok, &pp.v_stride_head, &pp.v_stride_tok);
  pp.n_ctx = e;
  pp.n_query = (int32_t)(e - s);
  return pp;
}

int sequence_check(const reattn_params* p, int32_t chunk) {
  if (!p) return REATTN_ERR_NULL;
  if (chunk < 1 || chunk > 65535) return REATTN_ERR_RANGE;
  if ((int64_t)p->n_sink + p->n_local > 65535) return REATTN_ERR_RANGE;   // the first chunk is one launch
  return REATTN_OK;
}
}  // namespace

extern "C" int reattn_prefill_sequence_chunk_bounds(const reattn_params* p, int32_t chunk, int64_t c, int64_t* first,
                                                    int64_t* end) {
  const int rc = sequence_check(p, chunk);
  if (rc) return rc;
  if (p->n_ctx < 1 || c < 0) return REATTN_ERR_RANGE;
  int64_t s, e;
  if (!sequence_chunk(p, chunk, c, &s, &e)) return REATTN_ERR_RANGE;
  if (first) *first = s;
  if (end) *end = e;
  return REATTN_OK;
}

extern "C" int64_t reattn_prefill_sequence_chunks(const reattn_params* p, int32_t chunk) {
  if (sequence_check(p, chunk) || p->n_ctx < 1) return 0;
  int64_t c = 0, s, e;
  while (sequence_chunk(p, chunk, c, &s, &e)) ++c;
  return c;
}

extern "C" size_t reattn_prefill_sequence_workspace_bytes(const reattn_params* p, const reattn_vote* v,
                                                          int32_t chunk) {
  if (sequence_check(p, chunk)) return 0;
  size_t need = 0;
  int64_t s, e;
  for (int64_t c = 0; sequence_chunk(p, chunk, c, &s, &e); ++c) {
    const reattn_params pp = chunk_params(p, s, e);
    size_t t;
    if (v) {
      VotePlan vp;
      if (make_vote_plan(&pp, v, &vp)) return 0;
      t = vp.total;
    } else {
      Plan pl;
      if (make_plan(&pp, &pl)) return 0;
      t = pl.total;
    }
    if (t > need) need = t;
  }
  return need;
}

extern "C" int reattn_cache_append(const reattn_params* p, int64_t first_tok, int32_t n_tok, const void* k_new,
                                   const void* v_new, void* k_cache, void* v_cache, void* stream) {
  if (!p) return REATTN_ERR_NULL;
  reattn_params pp = *p;
  pp.n_query = 1;                                      // not used here
  Plan pl;
  const int rc = make_plan(&pp, &pl);
  if (rc) return rc;
  if (first_tok < 0 || n_tok < 0 || first_tok + n_tok > pl.N) return REATTN_ERR_RANGE;
  if (n_tok == 0) return REATTN_OK;
  if (!k_new || !v_new || !k_cache || !v_cache) return REATTN_ERR_NULL;
  if (!aligned16(k_new) || !aligned16(v_new) || !aligned16(k_cache) || !aligned16(v_cache)) return REATTN_ERR_ALIGN;
  return hip_rc(launch_cache_append(pl, first_tok, n_tok, k_new, v_new, k_cache, v_cache, (hipStream_t)stream));
}

extern "C" int reattn_prefill_sequence(const reattn_params* p, const reattn_vote* v, int32_t chunk, const void* q,
                                       const void* k_new, const void* v_new, void* k_cache, void* v_cache,
                                       float* out, int32_t* idx_out, int32_t* sel_out, int32_t* n_sel_out,
                                       void* ws, size_t ws_bytes, void* stream) {
  int rc = sequence_check(p, chunk);
  if (rc) return rc;
  {                                                    // the sequence as a whole: shapes, strides, L
    reattn_params p1 = *p;
    p1.n_query = 1;
    Plan pl;
    rc = make_plan(&p1, &pl);
    if (rc && rc != REATTN_ERR_WINDOW) return rc;      // the window is checked chunk by chunk
  }
  if (!q || !k_new || !v_new || !k_cache || !v_cache || !out) return REATTN_ERR_NULL;
  if (!aligned16(q) || !aligned16(k_new) || !aligned16(v_new) || !aligned16(k_cache) || !aligned16(v_cache) ||
      !aligned16(out))
    return REATTN_ERR_ALIGN;
  const size_t need = reattn_prefill_sequence_workspace_bytes(p, v, chunk);
  if (need == 0) {                                     // some chunk is invalid: report which rule it breaks
    int64_t s, e;
    for (int64_t c = 0; sequence_chunk(p, chunk, c, &s, &e); ++c) {
      const reattn_params pp = chunk_params(p, s, e);
      VotePlan vp; Plan pl;
      const int r = v ? make_vote_plan(&pp, v, &vp) : make_plan(&pp, &pl);
      if (r) return r;
    }
    return REATTN_ERR_RANGE;
  }
  if (!ws || ws_bytes < need) return REATTN_ERR_WORKSPACE;
  if ((uintptr_t)ws % kAlign) return REATTN_ERR_ALIGN;
  const size_t eb = (size_t)elem_bytes(p->dtype);
  const size_t qrow = (size_t)p->n_q_heads * p->head_dim, krow = (size_t)p->n_kv_heads * p->head_dim;
  // the largest selection of any chunk is the last one's: it strides sel_out
  int64_t sel_stride = 0;
  if (v) {
    reattn_params pl_last = *p;
    pl_last.n_query = 1; pl_last.max_position = 0;     // only the clamped cap is wanted here
    VotePlan vp;
    if (make_vote_plan(&pl_last, v, &vp)) return REATTN_ERR_RANGE;
    sel_stride = vp.pl.k_eff > 0 ? vp.pl.k_eff : 1;
  }
  int64_t s, e, idx_at = 0;
  for (int64_t c = 0; sequence_chunk(p, chunk, c, &s, &e); ++c) {
    const reattn_params pp = chunk_params(p, s, e);
    Plan pl;
    rc = make_plan(&pp, &pl);
    if (rc) return rc;
    rc = hip_rc(launch_cache_append(pl, s, (int)(e - s), (const char*)k_new + (size_t)s * krow * eb,
                                    (const char*)v_new + (size_t)s * krow * eb, k_cache, v_cache,
                                    (hipStream_t)stream));
    if (rc) return rc;
    const char* qc = (const char*)q + (size_t)s * qrow * eb;
    float* oc = out + (size_t)s * qrow;
    if (v) {
      rc = vote_layer_impl(&pp, v, qc, k_cache, v_cache, sel_out ? sel_out + c * sel_stride : nullptr,
                           n_sel_out ? n_sel_out + c : nullptr, oc, ws, ws_bytes, stream, nullptr);
    } else {
      rc = run_layer(&pp, false, qc, k_cache, v_cache, idx_out ? idx_out + idx_at : nullptr, oc, ws, ws_bytes,
                     stream);
      idx_at += (int64_t)pl.M * pl.Hkv * pl.k_eff;
    }
    if (rc) return rc;
  }
  return REATTN_OK;
}

// ---- one decode token through all layers ----------------------------------------------------
extern "C" int reattn_decode_token(const reattn_params* p, const reattn_vote* v, int32_t n_layers,
                                   const void* const* q, const void* const* k_new, const void* const* v_new,
                                   void* const* k_cache, void* const* v_cache, float* const* out,
                                   void* ws, size_t ws_bytes, void* stream) {
  if (!p) return REATTN_ERR_NULL;
  if (n_layers < 1) return REATTN_ERR_RANGE;
  if (!q || !k_new || !v_new || !k_cache || !v_cache || !out) return REATTN_ERR_NULL;
  reattn_params pp = *p;
  pp.n_query = 1;
  Plan pl;
  int rc = make_plan(&pp, &pl);
  if (rc) return rc;
  if (v) {
    VotePlan vp;
    rc = make_vote_plan(&pp, v, &vp);
    if (rc) return rc;
    if (!ws || ws_bytes < vp.total) return REATTN_ERR_WORKSPACE;
  } else if (!ws || ws_bytes < pl.total) {
    return REATTN_ERR_WORKSPACE;
  }
  for (int l = 0; l < n_layers; ++l) {                  // every pointer is checked before anything is launched
    if (!q[l] || !k_new[l] || !v_new[l] || !k_cache[l] || !v_cache[l] || !out[l]) return REATTN_ERR_NULL;
    if (!aligned16(q[l]) || !aligned16(k_new[l]) || !aligned16(v_new[l]) || !aligned16(k_cache[l]) ||
        !aligned16(v_cache[l]) || !aligned16(out[l]))
      return REATTN_ERR_ALIGN;
  }
  for (int l = 0; l < n_layers && !rc; ++l) {
    // the rotary table depends on the scope's upper bound alone: the first layer's serves them all
    // the token's rows ride along with one of the layer's small launches
    const AppendJob job{k_new[l], v_new[l], k_cache[l], v_cache[l], pl.N - 1, 1};
    rc = v ? vote_layer_impl(&pp, v, q[l], k_cache[l], v_cache[l], nullptr, nullptr, out[l], ws, ws_bytes, stream, nullptr, l > 0, &job)
           : run_layer(&pp, true, q[l], k_cache[l], v_cache[l], nullptr, out[l], ws, ws_bytes, stream, nullptr, l > 0, &job,
                       l > 0);                        // layer l - 1's top-k left the histograms zeroed
  }
  return rc;
}

static int layer_timed(const reattn_params* p, bool decode_only, const void* q, const void* k_cache,
                       const void* v_cache, int32_t* idx_out, float* out, void* ws,
                       size_t ws_bytes, void* stream, float* stage_ms) {
  if (!stage_ms) return REATTN_ERR_NULL;
  hipEvent_t ev[REATTN_N_STAGES + 1];
  int made = 0;
  for (; made <= REATTN_N_STAGES; ++made)
    if (hipEventCreate(&ev[made]) != hipSuccess) break;
  int rc = made == REATTN_N_STAGES + 1 ? REATTN_OK : REATTN_ERR_HIP;
  const bool warm = decode_only && p && p->ws_warm != 0;
  if (!rc) rc = run_layer(p, decode_only, q, k_cache, v_cache, idx_out, out, ws, ws_bytes, stream, ev, warm, nullptr, warm);
  if (!rc) {
    if (hipEventSynchronize(ev[REATTN_N_STAGES]) != hipSuccess) rc = REATTN_ERR_HIP;
    for (int i = 0; i < REATTN_N_STAGES && !rc; ++i)
      if (hipEventElapsedTime(&stage_ms[i], ev[i], ev[i + 1]) != hipSuccess) rc = REATTN_ERR_HIP;
  }
  for (int i = 0; i < made; ++i) (void)hipEventDestroy(ev[i]);
  return rc;
}

int reattn_decode_step_timed(const reattn_params* p, const void* q, const void* k_cache,
                             const void* v_cache, int32_t* idx_out, float* out, void* ws,
                             size_t ws_bytes, void* stream, float* stage_ms) {
  return layer_timed(p, true, q, k_cache, v_cache, idx_out, out, ws, ws_bytes, stream, stage_ms);
}

int reattn_prefill_chunk_timed(const reattn_params* p, const void* q, const void* k_cache,
                               const void* v_cache, int32_t* idx_out, float* out, void* ws,
                               size_t ws_bytes, void* stream, float* stage_ms) {
  Plan pl;
  const int rc = make_plan(p, &pl);
  if (rc) return rc;
  if (!pl.fused_prefill) return REATTN_ERR_SHAPE;   // stage boundaries are defined for the MFMA path
  return layer_timed(p, false, q, k_cache, v_cache, idx_out, out, ws, ws_bytes, stream, stage_ms);
}

int reattn_redo_list_offset(const reattn_params* p, size_t* offset) {
  Plan pl;
  const int rc = make_plan(p, &pl);
  if (rc) return rc;
  if (!offset) return REATTN_ERR_NULL;
  if (pl.fused_prefill) { *offset = pl.off_redo; return REATTN_OK; }
  if (pl.filter) { *offset = pl.off_fcnt + (size_t)pl.Hkv * pl.f_nb * 4; return REATTN_OK; }
  return REATTN_ERR_SHAPE;
}

int reattn_probe_read_bandwidth(const void* buf, size_t bytes, int iters, void* stream,
                                float* gb_per_s) {
  if (!buf || !gb_per_s) return REATTN_ERR_NULL;
  if (!aligned16(buf)) return REATTN_ERR_ALIGN;
  if (bytes < 16 || iters < 1) return REATTN_ERR_RANGE;
  hipStream_t st = (hipStream_t)stream;
  hipEvent_t a, b;
  if (hipEventCreate(&a) != hipSuccess) return REATTN_ERR_HIP;
  if (hipEventCreate(&b) != hipSuccess) { (void)hipEventDestroy(a); return REATTN_ERR_HIP; }
  int rc = hip_rc(launch_read_probe(buf, bytes, st));              // warm-up
  if (!rc) rc = hip_rc(hipEventRecord(a, st));
  for (int i = 0; i < iters && !rc; ++i) rc = hip_rc(launch_read_probe(buf, bytes, st));
  if (!rc) rc = hip_rc(hipEventRecord(b, st));
  if (!rc) rc = hip_rc(hipEventSynchronize(b));
  float ms = 0.f;
  if (!rc) rc = hip_rc(hipEventElapsedTime(&ms, a, b));
  if (!rc) *gb_per_s = ms > 0.f ? (float)((double)(bytes / 16 * 16) * iters / (ms * 1e-3) / 1e9) : 0.f;
  (void)hipEventDestroy(a); (void)hipEventDestroy(b);
  return rc;
}

}  // extern "C"
