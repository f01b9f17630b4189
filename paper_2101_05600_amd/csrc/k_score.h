// Score kernel: one work-group per (utterance, beam slot) hypothesis g.
//   1. candidate pre-selection: the K ids with the largest attention log-prob (radix select
//      on order-preserving keys, ties to the smaller id, output in ascending id order);
//   2. window [s, e] from g's time indices (the two equations after Eq. (5));
//   3. prefix score of every extension g.c: log-sum over t in [s, e] of
//      f_t + log p^c(z_t = c), f_t = blank variable of g at t-1 if c repeats g's last label,
//      else phi_{t-1}(g)  (Eq. (3) / Eq. (5)); frames run along lanes, 16 or 64 lanes per
//      candidate, streaming log-sum-exp with one exp per term;
//   4. eos score phi_T(g), joint scores (Eq. (1)), the eos-run test, and the group's
//      best-first list of at most Wb candidates for the per-utterance selection.
#pragma once
#include "common.h"

struct ScoreSmem {
  // byte offsets into dynamic LDS, computed on the host
  int32_t off_att;    // float[V]           attention row (restricted mode)
  int32_t off_work;   // union: uint32 hist[RADIX_BINS] | float F[Wp], Fb[Wp]
  int32_t off_small;  // int32 cand_id[Ks], double J[Ks]  (Ks = K if K <= BLOCK else 0)
  int32_t wp_max;     // floats available per F array
};

__device__ __forceinline__ int f2ord(float v) {
  int i = __float_as_int(v);
  return i >= 0 ? i : i ^ 0x7fffffff;
}

// log-sum-exp over the candidate column `col` (aligned to the window's 4-frame boundary)
// plus the staged f terms, float4 index range [0, n4); LPC lanes cooperate.
template <int LPC>
__device__ __forceinline__ float chain_lse(const float4* __restrict__ col, const float4* __restrict__ f4,
                                           int n4, int q) {
  float m = LOG0F, s = 0.0f;
  for (int i = q; i < n4; i += LPC) {
    float4 x = col[i];
    float4 f = f4[i];
    float v0 = f.x + x.x, v1 = f.y + x.y, v2 = f.z + x.z, v3 = f.w + x.w;
    float mx = fmaxf(fmaxf(v0, v1), fmaxf(v2, v3));
    float mn = fmaxf(m, mx);
    s = s * __expf(m - mn) + (__expf(v0 - mn) + __expf(v1 - mn)) + (__expf(v2 - mn) + __expf(v3 - mn));
    m = mn;
  }
  float M = m;
#pragma unroll
  for (int o = LPC / 2; o > 0; o >>= 1) M = fmaxf(M, __shfl_xor(M, o));
  s *= __expf(m - M);
#pragma unroll
  for (int o = LPC / 2; o > 0; o >>= 1) s += __shfl_xor(s, o);
  return (M < LOG0_CLASS) ? LOG0F : M + __logf(s);
}

template <int BLOCK, int LPC>
__global__ __launch_bounds__(BLOCK) void k_score(Params p, ScoreSmem sm, const float* __restrict__ att,
                                                 int l, int cur) {
  extern __shared__ __align__(16) unsigned char smem[];
  __shared__ uint32_t s_scan[BLOCK / 64 + 1];
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
  uint32_t* s_hist = (uint32_t*)(smem + sm.off_work);
  float* s_F = (float*)(smem + sm.off_work);
  int32_t* s_cid = (int32_t*)(smem + sm.off_small);
  double* s_J = (double*)(smem + sm.off_small + (((size_t)(smallk ? K : 0) * 4 + 7) & ~(size_t)7));

  const float* arow = att + (size_t)grp * V;
  const int lo_ex = min(p.blank_id, p.eos_id), hi_ex = max(p.blank_id, p.eos_id);
  int32_t* g_cid = p.cand_id + (size_t)grp * K;

  // ---------------- 1. candidates -------------------------------------------------------
  if (p.restricted) {
    for (int i = tid; i < V; i += BLOCK) s_att[i] = arow[i];
    uint32_t prefix = 0, pmask = 0, krem = (uint32_t)K;
#pragma unroll 1
    for (int pass = 0; pass < 3; ++pass) {
      const int shift = pass == 0 ? 20 : (pass == 1 ? 8 : 0);
      const int bits = pass == 2 ? 8 : 12;
      const uint32_t bmask = (1u << bits) - 1u;
      const int nb = 1 << bits;
      for (int i = tid; i < nb; i += BLOCK) s_hist[i] = 0;
      __syncthreads();                 // also orders the s_att writes before the first pass
      for (int i = tid; i < V; i += BLOCK) {
        uint32_t k = att_key(s_att[i], i, p.blank_id, p.eos_id);
        if ((k & pmask) == prefix) atomicAdd(&s_hist[(k >> shift) & bmask], 1u);
      }
      __syncthreads();
      // find the bin in which the count of larger-or-equal keys reaches krem
      const int per = nb / BLOCK > 0 ? nb / BLOCK : 1;        // bins per thread (nb >= BLOCK or fewer threads used)
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
    const int i0 = tid * chunk, i1 = min(V, i0 + chunk);
    uint32_t gt = 0, eq = 0;
    for (int i = i0; i < i1; ++i) {
      uint32_t k = att_key(s_att[i], i, p.blank_id, p.eos_id);
      gt += (k > prefix); eq += (k == prefix);
    }
    uint32_t total;
    uint32_t ex = block_excl_scan_u32<BLOCK>((gt << 16) | eq, s_scan, &total);
    uint32_t gt_before = ex >> 16, eq_before = ex & 0xffffu;
    uint32_t pos = gt_before + min(eq_before, krem);
    for (int i = i0; i < i1; ++i) {
      uint32_t k = att_key(s_att[i], i, p.blank_id, p.eos_id);
      bool take = (k > prefix) || (k == prefix && eq_before < krem);
      if (k == prefix) ++eq_before;
      if (take && pos < (uint32_t)K) {
        if (smallk) s_cid[pos] = i;
        g_cid[pos] = i;
        ++pos;
      }
    }
  } else {
    for (int i = tid; i < K; i += BLOCK) {
      int id = full_v_id(i, lo_ex, hi_ex);
      if (smallk) s_cid[i] = id;
      g_cid[i] = id;
    }
  }

  // ---------------- 2. window -----------------------------------------------------------
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
  float* s_Fb = s_F + sm.wp_max;
  const float* gn = p.gn[cur] + (size_t)grp * p.Tp;
  const float* gb = p.gb[cur] + (size_t)grp * p.Tp;
  __syncthreads();                                         // radix histogram is dead, candidates are visible
  for (int i = tid; i < Wp; i += BLOCK) {
    int t = t0 + i;
    float f = LOG0F, fb = LOG0F;
    if (t >= s && t <= e) {
      int pr = t - 1;
      if (pr >= rs && pr <= re) { float n = gn[pr]; fb = gb[pr]; f = lae(n, fb); }
    }
    s_F[i] = f; s_Fb[i] = fb;
  }
  // eos-run eligibility (uniform over the block)
  const int R = p.eos_run;
  const bool e2 = (p.end_flags & 4) && R > 0 && T >= R && W > 0 && e == T && re == T &&
                  max(s, rs) <= T - R + 1;
  if (e2 && tid < R) s_e2[tid] = f2ord(LOG0F) - 1;
  __syncthreads();

  // ---------------- 3. prefix scores ----------------------------------------------------
  constexpr int NSG = BLOCK / LPC;
  const int sg = tid / LPC, q = tid % LPC;
  const float* xu = p.xT + (size_t)u * V * p.Tp;
  const double lam = p.lambda, jbase = (1.0 - lam) * acum + p.beta * (double)l;
  float* g_inc = p.cand_inc + (size_t)grp * K;
  float* g_catt = p.cand_att + (size_t)grp * K;
  double* g_ctc = p.cand_ctc + (size_t)grp * K;
  double* g_joint = p.cand_joint + (size_t)grp * K;
  const int n4_pre = e2 ? ((T - R - t0) >> 2) + 1 : 0;      // covers frames <= T-R (masked below)
  for (int c = sg; c < K; c += NSG) {
    const int id = smallk ? s_cid[c] : g_cid[c];
    const float4* col = (const float4*)(xu + (size_t)id * p.Tp + t0);
    const float4* f4 = (const float4*)((id == last) ? s_Fb : s_F);
    float inc = (W > 0) ? chain_lse<LPC>(col, f4, n4, q) : LOG0F;
    if (q == 0) {
      float a = p.restricted ? s_att[id] : arow[id];
      bool valid = inc > LOG0_CLASS;
      double ctc = valid ? off + (double)inc : LOG0D;
      double J = valid ? lam * ctc + (1.0 - lam) * (double)a + jbase : LOG0D;
      g_inc[c] = inc; g_catt[c] = a; g_ctc[c] = ctc; g_joint[c] = J;
      if (smallk) s_J[c] = (valid && J == J) ? J : LOG0D;
    }
    if (e2) {
      // running prefix score up to frame T-R: same sum with the last R frames cut off
      // (the cut is not float4-aligned: redo the tail of the last float4 by hand)
      const int t_cut = T - R;                             // last frame included
      float pre = LOG0F;
      if (t_cut >= s) {
        int full4 = (t_cut + 1 - t0) >> 2;                 // float4 groups entirely <= t_cut
        pre = chain_lse<LPC>(col, f4, full4, q);
        const float* colf = (const float*)col; const float* ff = (const float*)f4;
        for (int i = full4 * 4; t0 + i <= t_cut; ++i) pre = lae(pre, ff[i] + colf[i]);
      }
      if (q == 0) p.cand_pre[(size_t)grp * K + c] = pre;
    }
  }
  (void)n4_pre;

  // ---------------- 4. eos, eos-run rule, group list -------------------------------------
  if (tid == 0) {
    float ce = LOG0F;
    if (rs <= T && re >= T) ce = canon0(lae(gn[T], gb[T]));
    bool v = ce > LOG0_CLASS;
    double ctc = v ? off + (double)ce : LOG0D;
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
        int t = T - R + 1 + k;
        acc = lae(acc, ff[t - t0] + colf[t]);
        atomicMax(&s_e2[k], f2ord(canon0(acc)));
      }
    }
    __syncthreads();
    if (tid == 0) {
      fire = 1;
      for (int k = 0; k < R; ++k) {
        int t = T - R + 1 + k;
        float Et = canon0(lae(gn[t], gb[t]));
        int Xo = s_e2[k];
        // E_t > X_t with log0 on the left never true, log0 on the right always true
        bool gt = (Et > LOG0_CLASS) && (Xo < f2ord(LOG0_CLASS) || f2ord(Et) > Xo);
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
    __syncthreads();
    // rank by (joint desc, candidate index asc); candidate index order is token order
    if (tid == 0) s_nvalid = 0;
    __syncthreads();
    if (tid < K && !fire) {
      double me = s_J[tid];
      if (me > (double)LOG0_CLASS) {
        int rank = 0;
        for (int c = 0; c < K; ++c) {
          double o = s_J[c];
          rank += (o > me) || (o == me && c < tid);
        }
        if (rank < p.Wb) p.grp_idx[(size_t)grp * p.Wb + rank] = tid;
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
      if (bi != 0x7fffffff) p.grp_idx[(size_t)grp * p.Wb + r] = bi;
    }
    __syncthreads();
    if (s_pick[r] < 0) break;
    ++n;
  }
  if (tid == 0) p.grp_n[grp] = n;
}
