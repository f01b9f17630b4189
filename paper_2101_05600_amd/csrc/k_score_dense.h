// Score kernel for unrestricted candidate sets (every id but blank and eos is scored: the
// paper's Eq. (3) as it stands, no pre-selection).  With V - 2 candidates per hypothesis the
// posteriors of an utterance would be read once per beam slot; here one work-group serves ALL
// beam slots of its utterance: the f terms of every slot's window sit in LDS, a wave loads a
// candidate's column once into registers and runs it against each slot's f terms in turn.
// Column traffic falls by the beam width and the kernel is bound by the ALUs (one exp per term).
//   grid: U * nch work-groups, each taking a contiguous chunk of the candidate list;
//   the candidate that repeats a slot's last label (blank variable only, third alignment
//   rule of Sec. 2.1) is left out of the main loop and done by chunk 0 in a small pass of its own;
//   eos scores, windows and work counters: chunk 0, thread j for slot j.
// Not handled here (the host then launches k_score): top-K candidates, the eos-run rule, raw
// decoder scores, the batch-wide window, f terms that do not fit LDS.
// The groups' best-first lists are built by k_group_top afterwards.
#pragma once
#include "common.h"
#include "k_score.h"

template <int BLOCK, int NIT>
__global__ __launch_bounds__(BLOCK) void k_score_dense(Params p, const float* __restrict__ att, int l, int cur,
                                                        int nch) {
  extern __shared__ __align__(16) unsigned char smem[];
  float* s_F = (float*)smem;                                  // [Wb][Tp]
  __shared__ int q_live[MAX_BEAM], q_last[MAX_BEAM], q_s[MAX_BEAM], q_e[MAX_BEAM], q_rs[MAX_BEAM], q_re[MAX_BEAM],
      q_ref[MAX_BEAM];
  __shared__ double q_offr[MAX_BEAM], q_jbase[MAX_BEAM];
  __shared__ float q_mref[MAX_BEAM];
  __shared__ int q_some[MAX_BEAM];
  __shared__ int s_lo, s_hi;
  constexpr int NW = BLOCK / 64;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int Wb = p.Wb, K = p.K, V = p.V, Tp = p.Tp;
  const int u = blockIdx.x / nch, chunk = blockIdx.x - u * nch;
  const size_t h0 = (size_t)u * Wb;

  if (blockIdx.x == 0 && tid == 0) {
    // the count of finished utterances (as of the previous step) for the host's non-blocking look
    *(volatile int32_t*)p.host_finished = *p.n_finished;
    __threadfence_system();
  }
  const int T = p.lens[u];
  const bool fin = p.finished[u] != 0;
  const double* Bu = p.Bcum + (size_t)u * Tp;
  // ---- the Wb records; windows (the two equations after Eq. (5); unrestricted: s = l, e = T) ----
  if (tid == 0) { s_lo = 0x7fffffff; s_hi = -1; }
  __syncthreads();
  if (tid < Wb) {
    const size_t h = h0 + tid;
    const HypRec r = p.rec[cur][h];
    const int live = !fin && r.live != 0;
    const int tau = r.tau, tau_end = r.tau_end;
    int s = l > 1 ? l : 1, e = T;
    if (p.win_m1 >= 0) s = max(s, tau - p.win_m1);
    if (p.win_m2 >= 0) e = min(e, tau_end + p.win_m2);
    // (a slot that never held a hypothesis has a record nobody wrote: nothing of it may steer an access)
    const int ref = live ? checked(p, r.ref, 0, T, ERR_TIME_INDEX) : 0;
    q_live[tid] = live; q_last[tid] = r.last; q_s[tid] = s; q_e[tid] = e;
    q_rs[tid] = r.rs; q_re[tid] = r.re; q_ref[tid] = ref;
    q_offr[tid] = r.off + Bu[ref];
    q_jbase[tid] = (1.0 - p.lambda) * r.att + p.beta * (double)l;
    if (live && e >= s) { atomicMin(&s_lo, s); atomicMax(&s_hi, e); }
    if (chunk == 0 && !live) {
      p.grp_n[h] = 0; p.win_s[h] = 0; p.win_e[h] = -1; p.stopped[h] = 0;
      p.ctc_eos[h] = LOG0D; p.joint_eos[h] = LOG0D; p.grp_cells[h] = 0;
    }
  }
  __syncthreads();
  if (fin) return;
  const int smin = s_lo, emax = s_hi;
  const bool any = emax >= smin;
  const int t0 = any ? (smin & ~3) : 0;
  const int n4 = any ? ((emax - t0) >> 2) + 1 : 0;            // float4 per column window; n4 * 4 <= Tp
  const int Wp = n4 * 4;

  // ---- f terms of every live slot over [t0, t0 + Wp): log0 outside the slot's own window ----
  for (int j = 0; j < Wb; ++j) {
    if (!q_live[j]) continue;
    const float* gn = p.gn[cur] + (h0 + j) * Tp;
    const float* gb = p.gb[cur] + (h0 + j) * Tp;
    const int s = q_s[j], e = q_e[j], rs = q_rs[j], re = q_re[j];
    const double Bref = Bu[q_ref[j]];
    for (int i = tid; i < Wp; i += BLOCK) {
      const int t = t0 + i, pr = t - 1;
      float f = LOG0F;
      if (t >= s && t <= e && pr >= rs && pr <= re)
        f = canon0(lae(gn[pr], gb[pr]) + (float)(Bu[pr] - Bref));
      s_F[(size_t)j * Tp + i] = f;
    }
  }
  // ---- eos scores, windows, work counters (chunk 0, thread j) ----
  if (chunk == 0 && tid < Wb && q_live[tid]) {
    const int j = tid;
    const size_t h = h0 + j;
    const float* gn = p.gn[cur] + h * Tp;
    const float* gb = p.gb[cur] + h * Tp;
    const bool has = q_rs[j] <= T && q_re[j] >= T;
    const float ce = has ? canon0(lae(gn[T], gb[T])) : LOG0F;
    const bool v = ce > LOG0_CLASS;
    const double ctc = v ? q_offr[j] + (Bu[T] - Bu[q_ref[j]]) + (double)ce : LOG0D;
    p.ctc_eos[h] = ctc;
    p.joint_eos[h] = v ? p.lambda * ctc + (1.0 - p.lambda) * (double)att[h * V + p.eos_id] + q_jbase[j] : LOG0D;
    p.win_s[h] = q_s[j]; p.win_e[h] = q_e[j]; p.stopped[h] = 0;
    const int W = q_e[j] >= q_s[j] ? q_e[j] - q_s[j] + 1 : 0;
    p.grp_cells[h] = (long long)K * (long long)W;
  }
  __syncthreads();
  // ---- per slot: the largest f term M_j; the terms are then held as (f - M_j) * log2(e), so that
  // a product term is 2^(x * log2(e) + held) <= 1: one fused multiply-add, one exp2, one add per
  // term, no running maximum.  (A sum that underflows -- every term more than ~85 nats below
  // M_j -- is redone the careful way, see below.)
  constexpr float L2E = 1.4426950408889634f, LN2 = 0.6931471805599453f;
  for (int j = w; j < Wb; j += NW) {
    if (!q_live[j]) continue;
    float* Fj = s_F + (size_t)j * Tp;
    float m = LOG0F;
    for (int i = lane; i < Wp; i += 64) m = fmaxf(m, Fj[i]);
    m = row16_max(m);
    m = fmaxf(fmaxf(lane_f(m, 0), lane_f(m, 16)), fmaxf(lane_f(m, 32), lane_f(m, 48)));
    const bool some = m > LOG0_CLASS;                       // else: no term at all, every increment is log0
    for (int i = lane; i < Wp; i += 64) Fj[i] = (Fj[i] - m) * L2E;
    if (lane == 0) { q_mref[j] = m; q_some[j] = some ? 1 : 0; }
  }
  __syncthreads();

  // ---- main loop: one candidate per wave at a time, against every slot ----
  const float* xu = p.xT + (size_t)u * V * Tp;
  const int lo_ex = min(p.blank_id, p.eos_id), hi_ex = max(p.blank_id, p.eos_id);
  const int per = (K + nch - 1) / nch;
  const int c_lo = chunk * per, c_hi = min(K, c_lo + per);
  const double lam = p.lambda;
  for (int c = c_lo + w; c < c_hi; c += NW) {
    const int id = full_v_id(c, lo_ex, hi_ex);
    const float4* col = (const float4*)(xu + (size_t)id * Tp + t0);
    float4 x[NIT];
#pragma unroll
    for (int it = 0; it < NIT; ++it) x[it] = col[min(lane + it * 64, max(n4 - 1, 0))];   // all in flight
    float mine = LOG0F;
    for (int j = 0; j < Wb; ++j) {
      if (!q_live[j]) continue;                             // uniform
      float inc = LOG0F;
      if (q_some[j]) {
        const float4* F4 = (const float4*)(s_F + (size_t)j * Tp);
        const float mref = q_mref[j];
        float s0 = 0.0f, s1 = 0.0f;
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
          const int i = lane + it * 64;
          if (i < n4) {
            const float4 f = F4[i];
            s0 += __builtin_amdgcn_exp2f(fmaf(x[it].x, L2E, f.x)) + __builtin_amdgcn_exp2f(fmaf(x[it].y, L2E, f.y));
            s1 += __builtin_amdgcn_exp2f(fmaf(x[it].z, L2E, f.z)) + __builtin_amdgcn_exp2f(fmaf(x[it].w, L2E, f.w));
          }
        }
        float sum = row16_sum(s0 + s1);
        sum = (lane_f(sum, 0) + lane_f(sum, 16)) + (lane_f(sum, 32) + lane_f(sum, 48));
        if (sum > 1.0e-30f) {
          inc = mref + __logf(sum);
        } else {
          // every term far below M_j (or none finite): streaming log-sum-exp on the natural-log terms
          Lse a; a.m = LOG0F; a.s = 0.0f;
#pragma unroll
          for (int it = 0; it < NIT; ++it) {
            const int i = lane + it * 64;
            if (i < n4) {
              const float4 f2 = F4[i];
              float4 f;
              f.x = canon0(fmaf(f2.x, LN2, mref)); f.y = canon0(fmaf(f2.y, LN2, mref));
              f.z = canon0(fmaf(f2.z, LN2, mref)); f.w = canon0(fmaf(f2.w, LN2, mref));
              lse_add4(a, x[it], f);
            }
          }
          inc = lse_finish<64>(a);
        }
      }
      mine = (lane == j) ? inc : mine;
    }
    if (lane < Wb && q_live[lane] && id != q_last[lane]) {
      const int j = lane;
      const size_t o = (h0 + j) * (size_t)K + c;
      const float av = att[(h0 + j) * V + id];
      const bool valid = mine > LOG0_CLASS;
      const double ctc = valid ? q_offr[j] + (double)mine : LOG0D;
      const double J = valid ? lam * ctc + (1.0 - lam) * (double)av + q_jbase[j] : LOG0D;
      p.cand_id[o] = id; p.cand_inc[o] = valid ? mine : LOG0F; p.cand_att[o] = av;
      p.cand_ctc[o] = ctc; p.cand_joint[o] = J;
    }
  }

  // ---- the candidate that repeats slot j's last label: blank variable only (chunk 0, wave per slot) ----
  if (chunk == 0) {
    for (int j = w; j < Wb; j += NW) {
      const int id = q_last[j];
      if (!q_live[j] || id < 0 || id == p.blank_id || id == p.eos_id) continue;
      const int c = id - (id > lo_ex ? 1 : 0) - (id > hi_ex ? 1 : 0);     // its place in the candidate list
      const float* gb = p.gb[cur] + (h0 + j) * Tp;
      const float* colf = xu + (size_t)id * Tp;
      const int s = q_s[j], e = q_e[j], rs = q_rs[j], re = q_re[j];
      const double Bref = Bu[q_ref[j]];
      Lse a; a.m = LOG0F; a.s = 0.0f;
      for (int t = s + lane; t <= e; t += 64) {
        const int pr = t - 1;
        if (pr < rs || pr > re) continue;
        const float v = canon0(gb[pr] + (float)(Bu[pr] - Bref)) + colf[t];
        const float mn = fmaxf(a.m, v);
        a.s = a.s * __expf(a.m - mn) + __expf(v - mn);
        a.m = mn;
      }
      const float inc = lse_finish<64>(a);
      if (lane == 0) {
        const size_t o = (h0 + j) * (size_t)K + c;
        const float av = att[(h0 + j) * V + id];
        const bool valid = inc > LOG0_CLASS;
        const double ctc = valid ? q_offr[j] + (double)inc : LOG0D;
        const double J = valid ? lam * ctc + (1.0 - lam) * (double)av + q_jbase[j] : LOG0D;
        p.cand_id[o] = id; p.cand_inc[o] = valid ? inc : LOG0F; p.cand_att[o] = av;
        p.cand_ctc[o] = ctc; p.cand_joint[o] = J;
      }
    }
  }
}
