// Select kernel: one work-group per utterance.  Algorithm 2 from TopB on:
//   - merge the groups' best-first lists into the utterance's new beam (TopB / GatherB),
//     total order (joint desc, parent slot asc, token asc);
//   - the "p > best_score" test that moves g.<eos> into the ended set, forced ending at the
//     step cap, the eos-run stops;
//   - ENDDETECT: Eq. (4), then Algorithm 3's tau count;
//   - forward variables of the new hypotheses over their parent's window (one wave each,
//     the recurrence evaluated as two wave-level scans of affine maps in the (logaddexp, +)
//     semiring), their time indices tau / tau~ (first argmax from the parent's tau on);
//   - back-pointer record and the step's outputs.
#pragma once
#include "common.h"

struct Aff { float a, b; };   // v -> (v + a) (+) b   in the log semiring

__device__ __forceinline__ Aff aff_then(Aff first, Aff second) {
  Aff r; r.a = first.a + second.a; r.b = lae(first.b + second.a, second.b); return r;
}

__device__ __forceinline__ Aff wave_scan_aff(Aff v, int lane) {
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    Aff left; left.a = __shfl_up(v.a, o); left.b = __shfl_up(v.b, o);
    if (lane >= o) v = aff_then(left, v);
  }
  return v;
}

template <int BLOCK>
__global__ __launch_bounds__(BLOCK) void k_select(Params p, int l, int cur) {
  constexpr int NW = BLOCK / 64;
  constexpr int MAXE = MAX_BEAM * MAX_BEAM;
  __shared__ double s_J[MAXE];
  __shared__ int s_par[MAXE], s_ci[MAXE];
  __shared__ int s_base[MAX_BEAM + 1];
  __shared__ int s_sel[MAX_BEAM];          // entry index of the new beam's slot n
  __shared__ int s_nnew, s_fin;

  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int u = blockIdx.x, Wb = p.Wb, K = p.K;
  if (p.finished[u]) return;               // outputs of a finished utterance were settled when it finished
  const int nxt = cur ^ 1;
  const size_t h0 = (size_t)u * Wb;
  const int T = p.lens[u];

  // ---- gather the groups' lists ----------------------------------------------------------
  if (tid == 0) {
    int acc = 0;
    for (int j = 0; j < Wb; ++j) { s_base[j] = acc; acc += p.grp_n[h0 + j]; }
    s_base[Wb] = acc;
  }
  if (tid < MAX_BEAM) s_sel[tid] = -1;
  __syncthreads();
  const int ne = s_base[Wb];
  for (int i = tid; i < Wb * Wb; i += BLOCK) {
    int j = i / Wb, r = i % Wb;
    if (r < p.grp_n[h0 + j]) {
      int ci = p.grp_idx[(h0 + j) * Wb + r];
      int e = s_base[j] + r;
      s_J[e] = p.cand_joint[(h0 + j) * K + ci];
      s_par[e] = j; s_ci[e] = ci;
    }
  }
  __syncthreads();
  // ---- rank (entries of one parent are already in token order among equals) --------------
  for (int e = tid; e < ne; e += BLOCK) {
    double me = s_J[e]; int mp = s_par[e], mc = s_ci[e];
    int rank = 0;
    for (int o = 0; o < ne; ++o) {
      double v = s_J[o];
      rank += (v > me) || (v == me && (s_par[o] < mp || (s_par[o] == mp && s_ci[o] < mc)));
    }
    if (rank < Wb) s_sel[rank] = e;
  }
  __syncthreads();

  // ---- ended set, end detection (one thread) ---------------------------------------------
  if (tid == 0) {
    const int n_new = min(ne, Wb);
    const bool has_best = ne > 0;
    const double best = has_best ? s_J[s_sel[0]] : LOG0D;
    const bool forced = (l >= p.lmax[u]);
    UttState st = p.utt[u];
    long long cells = 0, ngroups = 0;
    for (int j = 0; j < Wb; ++j) {
      const size_t h = h0 + j;
      int added = 0, stp = 0;
      if (p.h_live[cur][h]) {
        cells += p.grp_cells[h];
        ++ngroups;
        stp = p.stopped[h];
        const double je = p.joint_eos[h];
        const bool je_ok = je > (double)LOG0_CLASS;
        added = forced || stp || (je_ok && (!has_best || je > best));
        if (added) {
          if (st.n_ended == 0 || je > st.best_score) { st.best_score = je; st.best_step = l; st.best_slot = j; }
          ++st.n_ended;
          const int ri = l % p.end_m;
          if (st.ring_tag[ri] != l) { st.ring_tag[ri] = l; st.ring_score[ri] = je; }
          else if (je > st.ring_score[ri]) st.ring_score[ri] = je;
          if (p.h_tau[cur][h] == T) ++st.cnt_tau_T;
        }
      }
      p.out_eos_added[h] = (uint8_t)added;
      p.out_stopped[h] = (uint8_t)stp;
    }
    bool fin = forced || n_new == 0;
    if (!fin && st.n_ended > 0) {
      if (p.end_flags & 1) {                       // Eq. (4)
        int count = 0;
        for (int m = 0; m < p.end_m; ++m) {
          const int tag = l - m;
          if (tag < 1) continue;
          const int ri = tag % p.end_m;
          if (st.ring_tag[ri] == tag && st.ring_score[ri] - st.best_score < (double)p.end_d) ++count;
        }
        if (count == p.end_m) fin = true;
      }
      if (!fin && (p.end_flags & 2) && st.cnt_tau_T > p.end_c) fin = true;   // Algorithm 3
    }
    if (fin) {
      st.finished_step = l;
      p.finished[u] = 1;
      atomicAdd(p.n_finished, 1);
    }
    p.utt[u] = st;
    p.cells[u] += (unsigned long long)cells;
    p.groups[u] += (unsigned long long)ngroups;
    s_nnew = n_new; s_fin = fin ? 1 : 0;
  }
  __syncthreads();
  const int n_new = s_nnew;
  const bool fin = s_fin != 0;

  // ---- new beam: records, outputs, back-pointers ------------------------------------------
  const size_t trie_l = ((size_t)l * p.U + u) * Wb;
  for (int n = tid; n < Wb; n += BLOCK) {
    const size_t h = h0 + n;
    if (n < n_new) {
      const int e = s_sel[n], par = s_par[e], ci = s_ci[e];
      const size_t hp = h0 + par, cidx = hp * K + ci;
      const int tok = p.cand_id[cidx];
      p.out_parent[h] = par; p.out_token[h] = tok; p.out_score[h] = (float)s_J[e];
      p.out_live[h] = fin ? 0 : 1;
      p.trie_parent[trie_l + n] = par; p.trie_token[trie_l + n] = tok;
      p.h_live[nxt][h] = fin ? 0 : 1;
      p.h_last[nxt][h] = tok;
      p.h_rs[nxt][h] = p.win_s[hp]; p.h_re[nxt][h] = p.win_e[hp];
      p.h_off[nxt][h] = p.cand_ctc[cidx];
      p.h_att[nxt][h] = p.h_att[cur][hp] + (double)p.cand_att[cidx];
      p.h_joint[nxt][h] = s_J[e];
    } else {
      p.out_parent[h] = -1; p.out_token[h] = -1; p.out_score[h] = LOG0F; p.out_live[h] = 0;
      p.out_tau[h] = 0; p.out_tau_end[h] = 0;
      p.trie_parent[trie_l + n] = -1; p.trie_token[trie_l + n] = -1; p.trie_tau[trie_l + n] = 0;
      p.h_live[nxt][h] = 0;
    }
  }

  // ---- forward variables of the new hypotheses --------------------------------------------
  const float* xu = p.xT + (size_t)u * p.V * p.Tp;
  const float* x0 = xu + (size_t)p.blank_id * p.Tp;
  for (int n = w; n < n_new && !fin; n += NW) {
    const int e = s_sel[n], par = s_par[e], ci = s_ci[e];
    const size_t hp = h0 + par, cidx = hp * K + ci;
    const int tok = p.cand_id[cidx];
    const float inc = p.cand_inc[cidx];
    const int s = p.win_s[hp], en = p.win_e[hp];
    const int rs = p.h_rs[cur][hp], re = p.h_re[cur][hp];
    const int ptau = p.h_tau[cur][hp], ptau_end = p.h_tau_end[cur][hp];
    const bool rep = (tok == p.h_last[cur][hp]);
    const float* pgn = p.gn[cur] + hp * p.Tp;
    const float* pgb = p.gb[cur] + hp * p.Tp;
    float* cgn = p.gn[nxt] + (h0 + n) * p.Tp;
    float* cgb = p.gb[nxt] + (h0 + n) * p.Tp;
    const float* xc = xu + (size_t)tok * p.Tp;
    const int lo = max(s, ptau);
    float carry_n = LOG0F, carry_b = LOG0F;
    float best_n = LOG0F, best_b = LOG0F;
    int arg_n = ptau, arg_b = ptau_end;
    for (int base = s; base <= en; base += 64) {
      const int t = base + lane;
      const bool valid = t <= en;
      Aff an, ab;
      float xb = 0.0f;
      if (valid) {
        const int pr = t - 1;
        float f = LOG0F;
        if (pr >= rs && pr <= re) { float fb = pgb[pr]; f = rep ? fb : lae(pgn[pr], fb); }
        const float x = xc[t];
        xb = x0[t];
        an.a = x; an.b = f + x;                  // n_t = (n_{t-1} (+) f_t) + x_t(c)
      } else { an.a = 0.0f; an.b = LOG0F; }
      an = wave_scan_aff(an, lane);
      const float nt = lae(an.a + carry_n, an.b);
      float nprev = __shfl_up(nt, 1);
      if (lane == 0) nprev = carry_n;
      if (valid) { ab.a = xb; ab.b = nprev + xb; }   // b_t = (n_{t-1} (+) b_{t-1}) + x_t(blank)
      else { ab.a = 0.0f; ab.b = LOG0F; }
      ab = wave_scan_aff(ab, lane);
      const float bt = lae(ab.a + carry_b, ab.b);
      carry_n = __shfl(nt, 63); carry_b = __shfl(bt, 63);
      // re-base on the child's own prefix score and store
      const float rn = (nt < LOG0_CLASS) ? LOG0F : nt - inc;
      const float rb = (bt < LOG0_CLASS) ? LOG0F : bt - inc;
      if (valid) { cgn[t] = rn; cgb[t] = rb; }
      // first argmax over t >= lo
      float vn = (valid && t >= lo) ? rn : LOG0F, vb = (valid && t >= lo) ? rb : LOG0F;
      int tn = t, tb = t;
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) {
        float ov = __shfl_xor(vn, o); int ot = __shfl_xor(tn, o);
        if (ov > vn || (ov == vn && ot < tn)) { vn = ov; tn = ot; }
        ov = __shfl_xor(vb, o); ot = __shfl_xor(tb, o);
        if (ov > vb || (ov == vb && ot < tb)) { vb = ov; tb = ot; }
      }
      if (vn > LOG0_CLASS && vn > best_n) { best_n = vn; arg_n = tn; }
      if (vb > LOG0_CLASS && vb > best_b) { best_b = vb; arg_b = tb; }
    }
    if (lane == 0) {
      p.h_tau[nxt][h0 + n] = arg_n; p.h_tau_end[nxt][h0 + n] = arg_b;
      p.out_tau[h0 + n] = arg_n; p.out_tau_end[h0 + n] = arg_b;
      p.trie_tau[trie_l + n] = arg_n;
    }
  }
}
