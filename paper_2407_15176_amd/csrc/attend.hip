// Stage 2: ordinary softmax attention over [global, select, local] (paper Eq. 3,
// second line; appendix `rope_attention`).  The scope S is a few thousand slots
// and a decode step has one query per head, so this is a flash-decoding kernel:
// S is split across workgroups, every workgroup keeps an online softmax per query
// head of one GQA group, partial (max, sum, weighted V) triples are merged with a
// log-sum-exp combine.  All arithmetic is fp32 on the vector ALUs (0.2 GFLOP per
// step: the cost is the 2*S*Hkv*D*bytes of gathered rows, not the math).
//
// Fused form (used by decode_step / prefill_chunk): the concatenation is never
// materialised.  Slot r is resolved to a cache row on the fly (sink: r, selected:
// idx[r - s], local: N - l + ...), the K row is rotary-encoded in registers at
// position r from a (cos, sin) table, the V row is consumed directly.
// Materialised form (reattn_attend): reads the fp32 rotated k_sel / v_sel buffers.
//
// Sixteen lanes own one slot at a time: lane `sub` holds channels [sub*E, sub*E+E)
// and the partner channels D/2 higher, so the rotary pairing (c, c + D/2) stays
// inside a lane and dot products finish with DPP row reductions.
#include "common.hpp"

namespace reattn {
namespace {

constexpr int kGroupsPerBlock = 16;   // 256 threads / 16 lanes
constexpr float kNegBig = -1.0e30f;

struct AttendArgs {
  const void* q; const void* k; const void* v;
  const int32_t* idx; const float2* rope;
  const int32_t* k_dyn;      // device scalar: number of selected entries, or nullptr for the static k_eff
  int64_t idx_stride;        // elements between the index rows of consecutive (query, KV head) pairs; 0 = one shared row
  int seq_heads;             // > 0: KV heads [b * seq_heads, (b + 1) * seq_heads) share index row b and length k_dyn[b]
  const int32_t* pt; int page_lg;   // paged cache (fused form): token -> row of the head's pool slice
  float* part; float* out;
  int64_t ksh, kst, vsh, vst, N;
  int Hq, Hkv, G, M, S, s_eff, k_eff, l_eff;
  int q_first, split_len, nsplit, nsub;
  float scale_log2e;
};

template <typename T, int E> struct Half;          // E consecutive channels of one row -> fp32
template <> struct Half<float, 4> {
  static __device__ __forceinline__ void load(const void* p, float* x) {
    const u32x4 d = *(const u32x4*)p;
    x[0] = __uint_as_float(d.x); x[1] = __uint_as_float(d.y);
    x[2] = __uint_as_float(d.z); x[3] = __uint_as_float(d.w);
  }
};
template <> struct Half<float, 2> {
  static __device__ __forceinline__ void load(const void* p, float* x) {
    const u32x2 d = *(const u32x2*)p;
    x[0] = __uint_as_float(d.x); x[1] = __uint_as_float(d.y);
  }
};
template <> struct Half<uint16_t, 4> {
  static __device__ __forceinline__ void load(const void* p, float* x) {
    const u32x2 d = *(const u32x2*)p;
    x[0] = bf16_lo(d.x); x[1] = bf16_hi(d.x); x[2] = bf16_lo(d.y); x[3] = bf16_hi(d.y);
  }
};
template <> struct Half<uint16_t, 2> {
  static __device__ __forceinline__ void load(const void* p, float* x) {
    const uint32_t d = *(const uint32_t*)p;
    x[0] = bf16_lo(d); x[1] = bf16_hi(d);
  }
};

template <> struct Half<f16bits, 4> {
  static __device__ __forceinline__ void load(const void* p, float* x) {
    const u32x2 d = *(const u32x2*)p;
    x[0] = f16_lo(d.x); x[1] = f16_hi(d.x); x[2] = f16_lo(d.y); x[3] = f16_hi(d.y);
  }
};
template <> struct Half<f16bits, 2> {
  static __device__ __forceinline__ void load(const void* p, float* x) {
    const uint32_t d = *(const uint32_t*)p;
    x[0] = f16_lo(d); x[1] = f16_hi(d);
  }
};

// 2^x for x <= 0 as the bare instruction: results below the smallest normal number come out as 0, which a
// softmax weight may (the library call wraps the instruction in a range test and a rescale, 4 instructions more,
// and this kernel is bound by its vector instruction count once there are enough heads to fill the chip).
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// T: storage type of q / V (and of K when FUSED).  GT: query heads per workgroup.
template <typename T, int D, int GT, bool FUSED>
__global__ __launch_bounds__(256) void attend_kernel(AttendArgs a) {
  constexpr int E = D / 32;
  constexpr int UNR = 2;                      // slots per 16-lane group in flight.  Measured at a million tokens (attention + combine by HIP events): 2: 27.6 us, 4: 28.6, 8: 33.4, 1: 30.7; reading the rotary table only every fourth turn: no gain
  typedef typename std::conditional<FUSED, T, float>::type KT;

  __shared__ float s_m[kGroupsPerBlock][GT];
  __shared__ float s_l[kGroupsPerBlock][GT];
  __shared__ float s_acc[kGroupsPerBlock][GT][D];

  const int sub = threadIdx.x & 15, gi = threadIdx.x >> 4;
  const int split = blockIdx.x;
  const int h = blockIdx.y / a.nsub, g0 = (blockIdx.y % a.nsub) * GT;
  const int qn = blockIdx.z, qi = a.q_first + qn;
  // a.S / a.k_eff are the largest scope the launch was shaped for (table layout, split geometry);
  // the scope actually attended to may be shorter when the selection length is data dependent
  const int seq = a.seq_heads > 0 ? h / a.seq_heads : 0;
  const int k_eff = (FUSED && a.k_dyn) ? a.k_dyn[seq] : a.k_eff;
  const int S = a.s_eff + k_eff + a.l_eff;
  const int visible = S - (a.M - 1 - qi);           // slots this query may see; its own key is the last
  const int c0 = sub * E;

  // (cos, sin) of position r for this lane's E channel pairs: product of the two table levels
  const int n_hi = rope_rows_hi(a.S);
  auto rope_at = [&](int r, float2* cs) {
    const float2* hi = a.rope + (int64_t)(r / kRopeLo) * (D / 2) + c0;
    const float2* lo = a.rope + (int64_t)(n_hi + r % kRopeLo) * (D / 2) + c0;
#pragma unroll
    for (int e = 0; e < E; ++e) {
      const float2 x = hi[e], y = lo[e];
      cs[e] = make_float2(x.x * y.x - x.y * y.y, x.y * y.x + x.x * y.y);
    }
  };

  // query rows of this group, rotary-encoded at the slot of the query's own key
  float qlo[GT][E], qhi[GT][E];
  {
    float2 rp[E];
    rope_at(visible - 1, rp);
#pragma unroll
    for (int g = 0; g < GT; ++g) {
      const int gg = (g0 + g < a.G) ? g0 + g : a.G - 1;
      const T* qr = (const T*)a.q + ((int64_t)qi * a.Hq + (int64_t)h * a.G + gg) * D;
      float lo[E], hi[E];
      Half<T, E>::load(qr + c0, lo);
      Half<T, E>::load(qr + D / 2 + c0, hi);
#pragma unroll
      for (int e = 0; e < E; ++e) {
        const float2 cs = rp[e];
        qlo[g][e] = (lo[e] * cs.x - hi[e] * cs.y) * a.scale_log2e;
        qhi[g][e] = (hi[e] * cs.x + lo[e] * cs.y) * a.scale_log2e;
      }
    }
  }

  int tok_cache = 0;
  float m[GT], l[GT], alo[GT][E], ahi[GT][E];
#pragma unroll
  for (int g = 0; g < GT; ++g) {
    m[g] = kNegBig; l[g] = 0.f;
#pragma unroll
    for (int e = 0; e < E; ++e) { alo[g][e] = 0.f; ahi[g][e] = 0.f; }
  }

  const int r0 = split * a.split_len;
  const int r_end = (r0 + a.split_len < visible) ? r0 + a.split_len : visible;
  const int64_t row_kv = (int64_t)qi * a.Hkv + h;
  const int32_t* my_idx = FUSED ? a.idx + (a.seq_heads > 0 ? (int64_t)seq : row_kv) * a.idx_stride : nullptr;

  // slot -> cache row: lane `sub` resolves the group's slot number `sub` of every batch of
  // 16 slots up front, so the index load is off the critical path of the row loads
  auto resolve = [&](int r) -> int {
    const int r2 = r < r_end ? r : r_end - 1;
    int tok;
    if (r2 < a.s_eff) tok = r2;
    else if (r2 < a.s_eff + k_eff) tok = my_idx[r2 - a.s_eff];
    else tok = (int)(a.N - a.l_eff) + (r2 - a.s_eff - k_eff);
    return (FUSED && a.pt) ? (int)paged_row(a.pt, a.page_lg, tok) : tok;
  };

  // Rotary factors of the group's slots: slot r + 16 * UNR follows from slot r by one complex multiplication
  // with a fixed step, and only every kReseed-th turn reads the table again (rounding does not pile up, and the
  // low table level, 64 KB at D = 128, does not fit the first-level cache: read per slot it doubled the bytes
  // a slot pulls out of L2).
  constexpr int kReseed = 8;
  float2 cs_run[UNR][E], cs_step[E];
  if (FUSED) {
    const int stride = kGroupsPerBlock * UNR;
    rope_at(stride < a.S ? stride : a.S - 1, cs_step);     // a scope shorter than one turn never steps
  }

  for (int base = r0, turn = 0; base < r_end; base += kGroupsPerBlock * UNR, ++turn) {
    float klo[UNR][E], khi[UNR][E], vlo[UNR][E], vhi[UNR][E];
    bool valid[UNR];
    int rr[UNR];
    int64_t tok[UNR];
    int tok_lane = 0;
    if (FUSED) {
      // 16 slots of this group per pass of 16 lanes: pass index = (base - r0) / (16 * 16)
      if (((base - r0) / (kGroupsPerBlock * UNR)) % (16 / UNR) == 0) {
        tok_cache = resolve(base + sub * kGroupsPerBlock + gi);
      }
      tok_lane = tok_cache;
    }
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      const int r = base + u * kGroupsPerBlock + gi;
      valid[u] = r < r_end;
      rr[u] = valid[u] ? r : r_end - 1;
      if (FUSED) {
        const int which = (((base - r0) / (kGroupsPerBlock * UNR)) % (16 / UNR)) * UNR + u;
        tok[u] = __shfl(tok_lane, which, 16);
      }
    }
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      const KT* kr; const T* vr;
      if (FUSED) {
        kr = (const KT*)a.k + (int64_t)h * a.ksh + tok[u] * a.kst;
        vr = (const T*)a.v + (int64_t)h * a.vsh + tok[u] * a.vst;
      } else {
        kr = (const KT*)a.k + (row_kv * a.S + rr[u]) * D;
        vr = (const T*)a.v + (row_kv * a.S + rr[u]) * D;
      }
      Half<KT, E>::load(kr + c0, klo[u]);
      Half<KT, E>::load(kr + D / 2 + c0, khi[u]);
      Half<T, E>::load(vr + c0, vlo[u]);
      Half<T, E>::load(vr + D / 2 + c0, vhi[u]);
    }
    if (FUSED) {
#pragma unroll
      for (int u = 0; u < UNR; ++u) {
        if (turn % kReseed == 0) {
          rope_at(rr[u], cs_run[u]);
        } else {
#pragma unroll
          for (int e = 0; e < E; ++e) {
            const float2 x = cs_run[u][e], y = cs_step[e];
            cs_run[u][e] = make_float2(x.x * y.x - x.y * y.y, x.y * y.x + x.x * y.y);
          }
        }
#pragma unroll
        for (int e = 0; e < E; ++e) {
          const float2 cs = cs_run[u][e];
          const float lo = klo[u][e], hi = khi[u][e];
          klo[u][e] = lo * cs.x - hi * cs.y;
          khi[u][e] = hi * cs.x + lo * cs.y;
        }
      }
    }
#pragma unroll
    for (int g = 0; g < GT; ++g) {
      float s[UNR];
      float mx = m[g];
#pragma unroll
      for (int u = 0; u < UNR; ++u) {
        float d = 0.f;
#pragma unroll
        for (int e = 0; e < E; ++e) d = fmaf(klo[u][e], qlo[g][e], fmaf(khi[u][e], qhi[g][e], d));
        d = group_sum<16>(d);
        s[u] = valid[u] ? d : kNegBig;
        mx = fmaxf(mx, s[u]);
      }
      float lsum = l[g];
      if (__any(mx > m[g])) {                      // a running maximum moves O(log n) times in n slots: mostly skipped
        const float corr = fast_exp2(m[g] - mx);
        m[g] = mx;
        lsum *= corr;
#pragma unroll
        for (int e = 0; e < E; ++e) { alo[g][e] *= corr; ahi[g][e] *= corr; }
      }
#pragma unroll
      for (int u = 0; u < UNR; ++u) {
        const float p = valid[u] ? fast_exp2(s[u] - mx) : 0.f;
        lsum += p;
#pragma unroll
        for (int e = 0; e < E; ++e) {
          alo[g][e] = fmaf(p, vlo[u][e], alo[g][e]);
          ahi[g][e] = fmaf(p, vhi[u][e], ahi[g][e]);
        }
      }
      l[g] = lsum;
    }
  }

  // merge the 16 slot-groups of this workgroup
#pragma unroll
  for (int g = 0; g < GT; ++g) {
    if (sub == 0) { s_m[gi][g] = m[g]; s_l[gi][g] = l[g]; }
#pragma unroll
    for (int e = 0; e < E; ++e) {
      s_acc[gi][g][c0 + e] = alo[g][e];
      s_acc[gi][g][D / 2 + c0 + e] = ahi[g][e];
    }
  }
  __syncthreads();
  for (int o = threadIdx.x; o < GT * D; o += 256) {
    const int g = o / D, c = o % D;
    if (g0 + g >= a.G) continue;
    float mx = kNegBig;
#pragma unroll
    for (int j = 0; j < kGroupsPerBlock; ++j) mx = fmaxf(mx, s_m[j][g]);
    float lsum = 0.f, acc = 0.f;
#pragma unroll
    for (int j = 0; j < kGroupsPerBlock; ++j) {
      const float w = exp2f(s_m[j][g] - mx);
      lsum = fmaf(s_l[j][g], w, lsum);
      acc = fmaf(s_acc[j][g][c], w, acc);
    }
    float* pp = a.part + (((int64_t)qn * a.Hq + (int64_t)h * a.G + g0 + g) * a.nsplit + split) * (D + 2);
    if (c == 0) { pp[0] = mx; pp[1] = lsum; }
    pp[2 + c] = acc;
  }
}

// out[q][hq][c] = sum_s A_s[c] 2^(m_s - m) / sum_s l_s 2^(m_s - m)
// One workgroup per (query, head); NG thread groups of D lanes each take every NG-th split.
template <int D, int NG>
__global__ __launch_bounds__(D * NG) void attend_combine_kernel(const float* __restrict__ part,
                                                                int nsplit, float* out) {
  __shared__ float s_m[NG], s_l[NG][D], s_a[NG][D];
  const int c = threadIdx.x % D, grp = threadIdx.x / D;
  const int64_t qh = blockIdx.x;
  const float* pp = part + qh * nsplit * (D + 2);
  // one pass, the running maximum carried along: every load is independent of the arithmetic,
  // so the partials arrive in one round trip
  float mx = kNegBig, lsum = 0.f, acc = 0.f;
#pragma unroll 4
  for (int s = grp; s < nsplit; s += NG) {
    const float* ps = pp + (int64_t)s * (D + 2);
    const float ms = ps[0], ls = ps[1], as = ps[2 + c];
    const float nm = fmaxf(mx, ms);
    const float w_old = exp2f(mx - nm), w = exp2f(ms - nm);
    lsum = fmaf(ls, w, lsum * w_old);
    acc = fmaf(as, w, acc * w_old);
    mx = nm;
  }
  if (c == 0) s_m[grp] = mx;
  s_l[grp][c] = lsum; s_a[grp][c] = acc;
  __syncthreads();
  if (grp == 0) {
    float gm = kNegBig;
#pragma unroll
    for (int g = 0; g < NG; ++g) gm = fmaxf(gm, s_m[g]);
    float L = 0.f, A = 0.f;
#pragma unroll
    for (int g = 0; g < NG; ++g) {
      const float w = exp2f(s_m[g] - gm);
      L = fmaf(s_l[g][c], w, L);
      A = fmaf(s_a[g][c], w, A);
    }
    out[qh * D + c] = A / L;
  }
}

template <typename T, int D, bool FUSED>
void launch_gt(const AttendArgs& a, int gt, dim3 grid, hipStream_t st) {
  switch (gt) {
    case 1: hipLaunchKernelGGL((attend_kernel<T, D, 1, FUSED>), grid, dim3(256), 0, st, a); break;
    case 2: hipLaunchKernelGGL((attend_kernel<T, D, 2, FUSED>), grid, dim3(256), 0, st, a); break;
    case 3: hipLaunchKernelGGL((attend_kernel<T, D, 3, FUSED>), grid, dim3(256), 0, st, a); break;
    default: hipLaunchKernelGGL((attend_kernel<T, D, 4, FUSED>), grid, dim3(256), 0, st, a); break;
  }
}

template <bool FUSED>
void launch_td(const Plan& pl, const AttendArgs& a, dim3 grid, hipStream_t st) {
  if (pl.dtype == kF32) {
    if (pl.D == 64) launch_gt<float, 64, FUSED>(a, pl.gt, grid, st);
    else            launch_gt<float, 128, FUSED>(a, pl.gt, grid, st);
  } else if (pl.dtype == kF16) {
    if (pl.D == 64) launch_gt<f16bits, 64, FUSED>(a, pl.gt, grid, st);
    else            launch_gt<f16bits, 128, FUSED>(a, pl.gt, grid, st);
  } else {
    if (pl.D == 64) launch_gt<uint16_t, 64, FUSED>(a, pl.gt, grid, st);
    else            launch_gt<uint16_t, 128, FUSED>(a, pl.gt, grid, st);
  }
}

}  // namespace

hipError_t launch_attend(const Plan& pl, bool fused, const void* q, int q_first, int n_query,
                         const void* k_src, const void* v_src, const int32_t* idx,
                         const float2* rope, float* part, float* out, hipStream_t st,
                         const int32_t* k_dyn, int64_t idx_stride, int seq_heads) {
  if (n_query <= 0) return hipSuccess;
  AttendArgs a;
  a.q = q; a.k = k_src; a.v = v_src; a.idx = idx; a.rope = rope; a.part = part; a.out = out;
  a.k_dyn = k_dyn; a.idx_stride = idx_stride < 0 ? pl.k_eff : idx_stride; a.seq_heads = seq_heads;
  a.pt = fused ? pl.pt : nullptr; a.page_lg = pl.page_lg;
  a.ksh = pl.ksh; a.kst = pl.kst; a.vsh = pl.vsh; a.vst = pl.vst; a.N = pl.N;
  a.Hq = pl.Hq; a.Hkv = pl.Hkv; a.G = pl.G; a.M = pl.M; a.S = pl.S;
  a.s_eff = (int)pl.s_eff; a.k_eff = pl.k_eff; a.l_eff = (int)pl.l_eff;
  a.q_first = q_first; a.split_len = pl.split_len; a.nsplit = pl.nsplit; a.nsub = pl.nsub;
  a.scale_log2e = pl.scale * 1.4426950408889634f;
  const dim3 grid((unsigned)pl.nsplit, (unsigned)(pl.Hkv * pl.nsub), (unsigned)n_query);
  if (fused) launch_td<true>(pl, a, grid, st); else launch_td<false>(pl, a, grid, st);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  return launch_attend_combine(pl.D, (int64_t)n_query * pl.Hq, pl.nsplit, part,
                               out + (int64_t)q_first * pl.Hq * pl.D, st);
}

hipError_t launch_attend_combine(int D, int64_t rows, int nsplit, const float* part, float* o, hipStream_t st) {
  const dim3 cgrid((unsigned)rows);
  if (nsplit > 4) {
    if (D == 64) hipLaunchKernelGGL((attend_combine_kernel<64, 16>), cgrid, dim3(1024), 0, st, part, nsplit, o);
    else         hipLaunchKernelGGL((attend_combine_kernel<128, 8>), cgrid, dim3(1024), 0, st, part, nsplit, o);
  } else {
    if (D == 64) hipLaunchKernelGGL((attend_combine_kernel<64, 1>), cgrid, dim3(64), 0, st, part, nsplit, o);
    else         hipLaunchKernelGGL((attend_combine_kernel<128, 1>), cgrid, dim3(128), 0, st, part, nsplit, o);
  }
  return hipGetLastError();
}

}  // namespace reattn
