// Score kernel: one work-group per (utterance, beam slot) hypothesis g.
//   1. candidate pre-selection: the K ids with the largest attention log-prob, ties to the
//      smaller id, output in ascending id order.  Fast path: a pivot L that is provably not
//      above the K-th largest value (every wave contributes the ceil(K/#waves)-th largest of
//      its lanes' chunk maxima), then an exact ranking of the few values >= L.  Rows with so
//      many values >= L that the short list overflows (heavy ties) take a radix select.
//   2. window [s, e] from g's time indices (the two equations after Eq. (5));
//   3. prefix score of every extension g.c: log-sum over t in [s, e] of
//      f_t + log p^c(z_t = c), f_t = blank variable of g at t-1 if c repeats g's last label,
//      else phi_{t-1}(g)  (Eq. (3) / Eq. (5)); frames run along lanes (16 or 64 lanes per
//      candidate, float4 per lane), all of a lane's column loads are issued before the first
//      is consumed, streaming log-sum-exp with one exp per term;
//   4. eos score phi_T(g), joint scores (Eq. (1)), the eos-run test, and the group's
//      best-first list of at most Wb candidates for the per-utterance selection.
#pragma once
#include "common.h"

#define PIVOT_CAP 512

struct ScoreSmem {
  // byte offsets into dynamic LDS, computed on the host
  int32_t off_att;    // float[V]           attention row (restricted mode)
  int32_t off_work;   // union: uint32 hist[RADIX_BINS] | { uint32 key[PIVOT_CAP]; int32 idx[PIVOT_CAP] }
  int32_t off_f;      // float F[wp_max], Fb[wp_max]
  int32_t off_small;  // double J[Ks]; int32 cand_id[Ks]; float inc[Ks], att[Ks]  (Ks = K if K <= BLOCK else 0)
  int32_t wp_max;     // floats available per F array
};

__device__ __forceinline__ int f2ord(float v) {
  int i = __float_as_int(v);
  return i >= 0 ? i : i ^ 0x7fffffff;
}

// ---- candidate selection -----------------------------------------------------------------
// Pivot path.  Returns false (uniformly) if more than PIVOT_CAP values reach the pivot.
template <int BLOCK>
__device__ __forceinline__ bool select_pivot(const float* s_att, int V, int K, int blank_id, int eos_id,
                                             uint32_t* s_key, int32_t* s_idx, uint32_t* s_scan,
                                             uint32_t* s_w, int32_t* out_lds, int32_t* out_g) {
  constexpr int NW = BLOCK / 64;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int chunk = ((V + BLOCK - 1) / BLOCK) | 1;          // odd stride: conflict-free LDS reads
  const int i0 = min(V, tid * chunk), i1 = min(V, i0 + chunk);
  uint32_t lmax = 0;
  for (int i = i0; i < i1; ++i) lmax = max(lmax, att_key(s_att[i], i, blank_id, eos_id));
  // r-th largest chunk maximum of this wave, by bisection on the key bits
  const int r = (K + NW - 1) / NW;
  uint32_t thr = 0;
#pragma unroll 1
  for (int bit = 31; bit >= 0; --bit) {
    const uint32_t trial = thr | (1u << bit);
    if (__popcll(__ballot(lmax >= trial)) >= r) thr = trial;
  }
  if (lane == 0) s_w[w] = thr;
  __syncthreads();
  uint32_t L = s_w[0];
#pragma unroll
  for (int i = 1; i < NW; ++i) L = min(L, s_w[i]);
  // at least NW * r >= K values are >= L; collect them in ascending id order
  uint32_t cnt = 0;
  for (int i = i0; i < i1; ++i) cnt += att_key(s_att[i], i, blank_id, eos_id) >= L;
  uint32_t total;
  uint32_t pos = block_excl_scan_u32<BLOCK>(cnt, s_scan, &total);
  if (total > PIVOT_CAP) return false;
  for (int i = i0; i < i1; ++i) {
    const uint32_t k = att_key(s_att[i], i, blank_id, eos_id);
    if (k >= L) { s_key[pos] = k; s_idx[pos] = i; ++pos; }
  }
  __syncthreads();
  const int n = (int)total;
  // exact rank by (key desc, id asc) = (key desc, list position asc); entries tid and tid + BLOCK
  uint32_t flags = 0;
#pragma unroll
  for (int j = 0; j < PIVOT_CAP / BLOCK; ++j) {
    const int e = tid + j * BLOCK;
    if (e < n) {
      const uint32_t me = s_key[e];
      int rank = 0;
      for (int o = 0; o < n; ++o) {
        const uint32_t v = s_key[o];
        rank += (v > me) || (v == me && o < e);
      }
      if (rank < K) flags |= 1u << (16 * j);
    }
  }
  uint32_t tot2;
  const uint32_t ex = block_excl_scan_u32<BLOCK>(flags, s_scan, &tot2);
  const uint32_t first_half = tot2 & 0xffffu;
#pragma unroll
  for (int j = 0; j < PIVOT_CAP / BLOCK; ++j) {
    if (flags & (1u << (16 * j))) {
      const uint32_t o = j == 0 ? (ex & 0xffffu) : first_half + (ex >> 16);
      const int id = s_idx[tid + j * BLOCK];
      if (o < (uint32_t)K) {
        if (out_lds) out_lds[o] = id;
        out_g[o] = id;
      }
    }
  }
  return true;
}

// Radix select on the order-preserving keys (12 + 12 + 8 bits), ordered compaction.
template <int BLOCK>
__device__ __noinline__ void select_radix(const float* s_att, int V, int K, int blank_id, int eos_id,
                                          uint32_t* s_hist, uint32_t* s_scan, uint32_t* s_sel,
                                          int32_t* out_lds, int32_t* out_g) {
  const int tid = threadIdx.x;
  uint32_t prefix = 0, pmask = 0, krem = (uint32_t)K;
#pragma unroll 1
  for (int pass = 0; pass < 3; ++pass) {
    const int shift = pass == 0 ? 20 : (pass == 1 ? 8 : 0);
    const int bits = pass == 2 ? 8 : 12;
    const uint32_t bmask = (1u << bits) - 1u;
    const int nb = 1 << bits;
    __syncthreads();
    for (int i = tid; i < nb; i += BLOCK) s_hist[i] = 0;
    __syncthreads();
    for (int i = tid; i < V; i += BLOCK) {
      uint32_t k = att_key(s_att[i], i, blank_id, eos_id);
      if ((k & pmask) == prefix) atomicAdd(&s_hist[(k >> shift) & bmask], 1u);
    }
    __syncthreads();
    // find the bin in which the count of larger-or-equal keys reaches krem
    const int per = nb / BLOCK > 0 ? nb / BLOCK : 1;
    uint32_t local = 0;
    const int b_lo = tid * per;
    if (b_lo < nb)
      for (int b = 0; b < per; ++b) local += s_hist[b_lo + b];
    uint32_t total;
    uint32_t excl = block_excl_scan_u32<BLOCK>(local, s_scan, &total);
    uint32_t above = total - excl - local;                   // keys in bins owned by higher threads
    if (b_lo < nb && above < krem && above + local >= krem) {
      uint32_t run = above;
      for (int b = per - 1; b >= 0; --b) {
        uint32_t h = s_hist[b_lo + b];
        if (run + h >= krem) { s_sel[0] = (uint32_t)(b_lo + b); s_sel[1] = krem - run; break; }
        run += h;
      }
    }
    __syncthreads();
    prefix |= s_sel[0] << shift;
    pmask |= bmask << shift;
    krem = s_sel[1];
  }
  // prefix = key of the K-th best; krem = how many of the keys equal to it are taken
  // (those with the smallest ids).  Ordered compaction, contiguous id chunk per thread.
  const int chunk = (V + BLOCK - 1) / BLOCK;
  const int i0 = min(V, tid * chunk), i1 = min(V, i0 + chunk);
  uint32_t gt = 0, eq = 0;
  for (int i = i0; i < i1; ++i) {
    uint32_t k = att_key(s_att[i], i, blank_id, eos_id);
    gt += (k > prefix); eq += (k == prefix);
  }
  uint32_t total;
  uint32_t ex = block_excl_scan_u32<BLOCK>((gt << 16) | eq, s_scan, &total);
  uint32_t gt_before = ex >> 16, eq_before = ex & 0xffffu;
  uint32_t pos = gt_before + min(eq_before, krem);
  for (int i = i0; i < i1; ++i) {
    uint32_t k = att_key(s_att[i], i, blank_id, eos_id);
    bool take = (k > prefix) || (k == prefix && eq_before < krem);
    if (k == prefix) ++eq_before;
    if (take && pos < (uint32_t)K) {
      if (out_lds) out_lds[pos] = i;
      out_g[pos] = i;
      ++pos;
    }
  }
}

// ---- streaming log-sum-exp pieces -----------------------------------------------------------
struct Lse { float m, s; };

__device__ __forceinline__ void lse_add4(Lse& a, const float4 x, const float4 f) {
  const float v0 = f.x + x.x, v1 = f.y + x.y, v2 = f.z + x.z, v3 = f.w + x.w;
  const float mn = fmaxf(a.m, fmaxf(fmaxf(v0, v1), fmaxf(v2, v3)));
  a.s = a.s * __expf(a.m - mn) + (__expf(v0 - mn) + __expf(v1 - mn)) + (__expf(v2 - mn) + __expf(v3 - mn));
  a.m = mn;
}

template <int LPC>
__device__ __forceinline__ float lse_finish(Lse a) {
  float M = a.m;
#pragma unroll
  for (int o = LPC / 2; o > 0; o >>= 1) M = fmaxf(M, __shfl_xor(M, o));
  float s = a.s * __expf(a.m - M);
#pragma unroll
  for (int o = LPC / 2; o > 0; o >>= 1) s += __shfl_xor(s, o);
  return (M < LOG0_CLASS) ? LOG0F : M + __logf(s);
}

// log-sum-exp over float4 groups [0, n4) of one column (used by the eos-run rule)
template <int LPC>
__device__ __forceinline__ float chain_lse(const float4* __restrict__ col, const float4* __restrict__ f4,
                                           int n4, int q) {
  Lse a; a.m = LOG0F; a.s = 0.0f;
  for (int i = q; i < n4; i += LPC) lse_add4(a, col[i], f4[i]);
  return lse_finish<LPC>(a);
}

template <int BLOCK, int LPC, int CB, int IT>
__global__ __launch_bounds__(BLOCK) void k_score(Params p, ScoreSmem sm, const float* __restrict__ att,
                                                 int l, int cur) {
  extern __shared__ __align__(16) unsigned char smem[];
  __shared__ uint32_t s_scan[BLOCK / 64 + 1];
  __shared__ uint32_t s_w[BLOCK / 64];
  __shared__ uint32_t s_sel[2];
  __shared__ int s_e2[MAX_EOS_RUN];
  __shared__ int s_nvalid;

  const int tid = threadIdx.x;
  const int grp = blockIdx.x;
  const int u = grp / p.Wb;
  const int K = p.K, V = p.V;
  const bool smallk = (K <= BLOCK);

  if (p.finished[u] || !p.h_live[cur][grp]) {
    if (tid == 0) {
      p.grp_n[grp] = 0; p.win_s[grp] = 0; p.win_e[grp] = -1; p.stopped[grp] = 0;
      p.ctc_eos[grp] = LOG0D; p.joint_eos[grp] = LOG0D; p.grp_cells[grp] = 0;
    }
    return;
  }

  float* s_att = (float*)(smem + sm.off_att);
  uint32_t* s_work = (uint32_t*)(smem + sm.off_work);
  float* s_F = (float*)(smem + sm.off_f);
  float* s_Fb = s_F + sm.wp_max;
  const int Ks = smallk ? K : 0;
  double* s_J = (double*)(smem + sm.off_small);
  int32_t* s_cid = smallk ? (int32_t*)(s_J + Ks) : nullptr;
  float* s_inc = (float*)(smem + sm.off_small) + 3 * Ks;    // after J (2 words each) and cand_id
  float* s_av = s_inc + Ks;

  const float* arow = att + (size_t)grp * V;
  int32_t* g_cid = p.cand_id + (size_t)grp * K;

  // ---------------- window (needs only g's record) ----------------------------------------
  const int T = p.lens[u];
  const int tau = p.h_tau[cur][grp], tau_end = p.h_tau_end[cur][grp];
  const int rs = p.h_rs[cur][grp], re = p.h_re[cur][grp], last = p.h_last[cur][grp];
  const double off = p.h_off[cur][grp], acum = p.h_att[cur][grp];
  int s = l > 1 ? l : 1, e = T;
  if (p.win_m1 >= 0) s = max(s, tau - p.win_m1);
  if (p.win_m2 >= 0) e = min(e, tau_end + p.win_m2);
  const int W = e >= s ? e - s + 1 : 0;
  const int t0 = s & ~3;                                   // column loads start on a 16-byte boundary
  const int n4 = W > 0 ? ((e - t0) >> 2) + 1 : 0;
  const int Wp = n4 * 4;
  const float* gn = p.gn[cur] + (size_t)grp * p.Tp;
  const float* gb = p.gb[cur] + (size_t)grp * p.Tp;

  // ---------------- stage the attention row and the f terms (loads overlap) ---------------
  if (p.restricted)
    for (int i = tid; i < V; i += BLOCK) s_att[i] = arow[i];
  for (int i = tid; i < Wp; i += BLOCK) {
    const int t = t0 + i;
    float f = LOG0F, fb = LOG0F;
    if (t >= s && t <= e) {
      const int pr = t - 1;
      if (pr >= rs && pr <= re) { const float n = gn[pr]; fb = gb[pr]; f = lae(n, fb); }
    }
    s_F[i] = f; s_Fb[i] = fb;
  }
  const int R = p.eos_run;
  const bool e2 = (p.end_flags & 4) && R > 0 && T >= R && W > 0 && e == T && re == T &&
                  max(s, rs) <= T - R + 1;
  if (e2 && tid < R) s_e2[tid] = f2ord(LOG0F) - 1;
  __syncthreads();

  // ---------------- 1. candidates -----------------------------------------------------------
  if (p.restricted) {
    const bool ok = select_pivot<BLOCK>(s_att, V, K, p.blank_id, p.eos_id, s_work, (int32_t*)(s_work + PIVOT_CAP),
                                        s_scan, s_w, s_cid, g_cid);
    if (!ok) select_radix<BLOCK>(s_att, V, K, p.blank_id, p.eos_id, s_work, s_scan, s_sel, s_cid, g_cid);
  } else {
    const int lo_ex = min(p.blank_id, p.eos_id), hi_ex = max(p.blank_id, p.eos_id);
    for (int i = tid; i < K; i += BLOCK) {
      const int id = full_v_id(i, lo_ex, hi_ex);
      if (smallk) s_cid[i] = id;
      g_cid[i] = id;
    }
  }
  __syncthreads();                                         // candidate ids visible to the whole block

  // ---------------- 3. prefix scores ----------------------------------------------------
  constexpr int NSG = BLOCK / LPC;
  const int sg = tid / LPC, q = tid % LPC;
  const float* xu = p.xT + (size_t)u * V * p.Tp;
  const double lam = p.lambda, jbase = (1.0 - lam) * acum + p.beta * (double)l;
  float* g_inc = p.cand_inc + (size_t)grp * K;
  float* g_catt = p.cand_att + (size_t)grp * K;
  double* g_ctc = p.cand_ctc + (size_t)grp * K;
  double* g_joint = p.cand_joint + (size_t)grp * K;
  for (int c0 = sg; c0 < K; c0 += NSG * CB) {
    float4 x[CB][IT];
    int ids[CB];
#pragma unroll
    for (int b = 0; b < CB; ++b) {
      const int c = c0 + b * NSG;
      ids[b] = (c < K) ? (smallk ? s_cid[c] : g_cid[c]) : -1;
      const float4* col = (const float4*)(xu + (size_t)(ids[b] < 0 ? 0 : ids[b]) * p.Tp + t0);
#pragma unroll
      for (int it = 0; it < IT; ++it) {
        const int i = q + it * LPC;
        x[b][it] = (ids[b] >= 0 && i < n4) ? col[i] : make_float4(0.f, 0.f, 0.f, 0.f);
      }
    }
#pragma unroll
    for (int b = 0; b < CB; ++b) {
      const int c = c0 + b * NSG;
      if (ids[b] < 0) continue;                            // uniform over the LPC lanes of a chain
      const int id = ids[b];
      const float4* col = (const float4*)(xu + (size_t)id * p.Tp + t0);
      const float4* f4 = (const float4*)((id == last) ? s_Fb : s_F);
      Lse a; a.m = LOG0F; a.s = 0.0f;
#pragma unroll
      for (int it = 0; it < IT; ++it) {
        const int i = q + it * LPC;
        if (i < n4) lse_add4(a, x[b][it], f4[i]);
      }
      for (int i = q + IT * LPC; i < n4; i += LPC) lse_add4(a, col[i], f4[i]);
      const float inc = (W > 0) ? lse_finish<LPC>(a) : LOG0F;
      if (q == 0) {
        const float av = p.restricted ? s_att[id] : arow[id];
        const bool valid = inc > LOG0_CLASS;
        const double ctc = valid ? off + (double)inc : LOG0D;
        const double J = valid ? lam * ctc + (1.0 - lam) * (double)av + jbase : LOG0D;
        g_inc[c] = inc; g_catt[c] = av; g_ctc[c] = ctc; g_joint[c] = J;
        if (smallk) { s_J[c] = (valid && J == J) ? J : LOG0D; s_inc[c] = inc; s_av[c] = av; }
      }
      if (e2) {
        // running prefix score up to frame T-R: same sum with the last R frames cut off
        // (the cut is not float4-aligned: the last partial float4 is added term by term)
        const int t_cut = T - R;                           // last frame included
        float pre = LOG0F;
        if (t_cut >= s) {
          const int full4 = (t_cut + 1 - t0) >> 2;         // float4 groups entirely <= t_cut
          pre = chain_lse<LPC>(col, f4, full4, q);
          const float* colf = (const float*)col; const float* ff = (const float*)f4;
          for (int i = full4 * 4; t0 + i <= t_cut; ++i) pre = lae(pre, ff[i] + colf[i]);
        }
        if (q == 0) p.cand_pre[(size_t)grp * K + c] = pre;
      }
    }
  }

  // ---------------- 4. eos, eos-run rule, group list -------------------------------------
  if (tid == 0) {
    float ce = LOG0F;
    if (rs <= T && re >= T) ce = canon0(lae(gn[T], gb[T]));
    const bool v = ce > LOG0_CLASS;
    const double ctc = v ? off + (double)ce : LOG0D;
    p.ctc_eos[grp] = ctc;
    p.joint_eos[grp] = v ? lam * ctc + (1.0 - lam) * (double)arow[p.eos_id] + jbase : LOG0D;
    p.win_s[grp] = s; p.win_e[grp] = e;
    p.grp_cells[grp] = (long long)K * (long long)W;
  }
  int fire = 0;
  if (e2) {
    __syncthreads();                                       // cand_pre written by this block
    for (int c = tid; c < K; c += BLOCK) {
      const int id = smallk ? s_cid[c] : g_cid[c];
      const float* colf = xu + (size_t)id * p.Tp;
      const float* ff = (id == last) ? s_Fb : s_F;
      float acc = p.cand_pre[(size_t)grp * K + c];
      for (int k = 0; k < R; ++k) {
        const int t = T - R + 1 + k;
        acc = lae(acc, ff[t - t0] + colf[t]);
        atomicMax(&s_e2[k], f2ord(canon0(acc)));
      }
    }
    __syncthreads();
    if (tid == 0) {
      fire = 1;
      for (int k = 0; k < R; ++k) {
        const int t = T - R + 1 + k;
        const float Et = canon0(lae(gn[t], gb[t]));
        const int Xo = s_e2[k];
        // E_t > X_t with log0 on the left never true, log0 on the right always true
        const bool gt = (Et > LOG0_CLASS) && (Xo < f2ord(LOG0_CLASS) || f2ord(Et) > Xo);
        if (!gt) fire = 0;
      }
      p.stopped[grp] = fire;
      s_e2[0] = fire;
    }
    __syncthreads();
    fire = s_e2[0];
  } else if (tid == 0) {
    p.stopped[grp] = 0;
  }

  if (smallk) {
    // rank by (joint desc, candidate index asc); candidate index order is token order
    if (tid == 0) s_nvalid = 0;
    __syncthreads();                                       // s_J complete
    if (tid < K && !fire) {
      const double me = s_J[tid];
      if (me > (double)LOG0_CLASS) {
        int rank = 0;
        for (int c = 0; c < K; ++c) {
          const double o = s_J[c];
          rank += (o > me) || (o == me && c < tid);
        }
        if (rank < p.Wb) {
          const size_t o = (size_t)grp * p.Wb + rank;
          p.grp_J[o] = me; p.grp_ci[o] = tid; p.grp_tok[o] = s_cid[tid];
          p.grp_inc[o] = s_inc[tid]; p.grp_att[o] = s_av[tid];
        }
        atomicAdd(&s_nvalid, 1);
      }
    }
    __syncthreads();
    if (tid == 0) p.grp_n[grp] = fire ? 0 : min(s_nvalid, p.Wb);
  }
}

// Group list for large candidate sets (K > block size): Wb rounds of a block-wide argmax
// over the joint scores in global memory.  One work-group per (utterance, beam slot).
template <int BLOCK>
__global__ __launch_bounds__(BLOCK) void k_group_top(Params p, int cur) {
  __shared__ double s_v[BLOCK / 64];
  __shared__ int s_i[BLOCK / 64];
  __shared__ int s_pick[MAX_BEAM];
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int grp = blockIdx.x, u = grp / p.Wb, K = p.K;
  if (p.finished[u] || !p.h_live[cur][grp]) return;      // k_score already wrote grp_n = 0
  if (p.stopped[grp]) { if (tid == 0) p.grp_n[grp] = 0; return; }
  const double* J = p.cand_joint + (size_t)grp * K;
  int n = 0;
  for (int r = 0; r < p.Wb; ++r) {
    double bv = LOG0D; int bi = 0x7fffffff;
    for (int c = tid; c < K; c += BLOCK) {
      double v = J[c];
      if (!(v > (double)LOG0_CLASS)) continue;
      bool taken = false;
      for (int k = 0; k < r; ++k) taken |= (s_pick[k] == c);
      if (taken) continue;
      if (v > bv || (v == bv && c < bi)) { bv = v; bi = c; }
    }
    for (int o = 32; o > 0; o >>= 1) {
      double ov = __shfl_xor(bv, o); int oi = __shfl_xor(bi, o);
      if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
    }
    if (lane == 0) { s_v[w] = bv; s_i[w] = bi; }
    __syncthreads();
    if (tid == 0) {
      for (int k = 1; k < BLOCK / 64; ++k)
        if (s_v[k] > bv || (s_v[k] == bv && s_i[k] < bi)) { bv = s_v[k]; bi = s_i[k]; }
      s_pick[r] = (bi == 0x7fffffff) ? -1 : bi;
      if (bi != 0x7fffffff) {
        const size_t o = (size_t)grp * p.Wb + r;
        p.grp_J[o] = bv; p.grp_ci[o] = bi; p.grp_tok[o] = p.cand_id[(size_t)grp * K + bi];
        p.grp_inc[o] = p.cand_inc[(size_t)grp * K + bi]; p.grp_att[o] = p.cand_att[(size_t)grp * K + bi];
      }
    }
    __syncthreads();
    if (s_pick[r] < 0) break;
    ++n;
  }
  if (tid == 0) p.grp_n[grp] = n;
}
