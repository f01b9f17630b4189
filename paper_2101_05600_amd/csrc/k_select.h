// Select kernels (k_select: one work-group per utterance; k_select_split, further down: one per
// new beam slot).  Algorithm 2 from TopB on:
//   - merge the groups' best-first lists into the utterance's new beam (TopB / GatherB),
//     total order (joint desc, parent slot asc, token asc);
//   - the "p > best_score" test that moves g.<eos> into the ended set, forced ending at the
//     step cap, the eos-run stops;
//   - ENDDETECT: Eq. (4), then Algorithm 3's tau count;
//   - forward variables of the new hypotheses over their parent's window (one wave each,
//     the recurrence evaluated as two wave-level scans of affine maps in the (logaddexp, +)
//     semiring), their time indices tau / tau~ (first argmax from the parent's tau on);
//   - back-pointer record and the step's outputs.
// Everything the decisions need is fetched in one round of independent loads at the top
// (old slots' records and the group lists); the only dependent second round is the
// survivors' state and posterior columns.
#pragma once
#include "common.h"

struct Aff { float a, b; };   // v -> (v + a) (+) b   in the log semiring

__device__ __forceinline__ Aff aff_then(Aff first, Aff second) {
  Aff r; r.a = first.a + second.a; r.b = lae(first.b + second.a, second.b); return r;
}

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ Aff aff_stage(Aff v) {
  Aff left;                                 // lanes without a source get the identity map
  left.a = dpp_f<CTRL, ROW_MASK>(0.0f, v.a);
  left.b = dpp_f<CTRL, ROW_MASK>(LOG0F, v.b);
  return aff_then(left, v);
}

// inclusive scan of affine maps over the wave: lane t ends with map_0 then ... then map_t
__device__ __forceinline__ Aff wave_scan_aff(Aff v) {
  v = aff_stage<0x111, 0xf>(v);
  v = aff_stage<0x112, 0xf>(v);
  v = aff_stage<0x114, 0xf>(v);
  v = aff_stage<0x118, 0xf>(v);
  v = aff_stage<0x142, 0xa>(v);
  v = aff_stage<0x143, 0xc>(v);
  return v;
}

struct ArgMax { float v; int t; };
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ ArgMax argmax_stage(ArgMax x) {
  const float ov = dpp_f<CTRL, ROW_MASK>(-3.0e38f, x.v);
  const int ot = dpp_i<CTRL, ROW_MASK>(0x7fffffff, x.t);
  if (ov > x.v || (ov == x.v && ot < x.t)) { x.v = ov; x.t = ot; }
  return x;
}
// largest value, earliest frame among equals; result valid in lane 63
__device__ __forceinline__ ArgMax wave_argmax(ArgMax x) {
  x = argmax_stage<0x111, 0xf>(x);
  x = argmax_stage<0x112, 0xf>(x);
  x = argmax_stage<0x114, 0xf>(x);
  x = argmax_stage<0x118, 0xf>(x);
  x = argmax_stage<0x142, 0xa>(x);
  x = argmax_stage<0x143, 0xc>(x);
  x.v = lane_f(x.v, 63); x.t = __builtin_amdgcn_readlane(x.t, 63);
  return x;
}

// Forward variables of one new hypothesis (parent slot `par` extended by `tok`) over the
// parent's window, by one wave: two scans of affine maps in the (logaddexp, +) semiring (each lane
// owns a few consecutive frames, composes their maps, the wave scans the composed maps, and the
// lane then replays its own frames).
// The recurrence runs on the stored form of the variables (per-frame reference B_t taken out,
// see Params::Bcum): with x'_t(c) = x_t(c) - max(x_t(blank), floor) and d_t = x_t(blank) -
// max(x_t(blank), floor) (zero unless the floor cut),
//   n_t = (n_{t-1} (+) f_t) + x'_t(c),     b_t = (n_{t-1} (+) b_{t-1}) + d_t,
// so that staying in blank costs nothing and values do not drift with t.  The child's state is
// re-based by delta = inc + (B_r - B_r'), r the parent's reference frame and r' = the parent's
// tau the child's: its values are then near zero around its own tau.  Writes the new state into
// slot n of the other buffer and returns delta and tau / tau~ (first argmax of the true variables,
// stored + B_t, from the parent's tau on; the parent's values if nothing is finite).
struct SurvivorIn {
  int par, tok, s, en, rs, re, ptau, ptau_end, plast, pref;
  float inc;
  int T;            // frames of the utterance (bounds of every time index)
};
// FPL consecutive frames per lane, 64 * FPL frames per pass.
template <int FPL>
__device__ __forceinline__ void wave_survivor_fpl(const Params& p, int u, int n, int cur, const SurvivorIn& in,
                                                  int& arg_n, int& arg_b, float& delta_out, double& bref_out) {
  const int lane = threadIdx.x & 63;
  const size_t h0 = (size_t)u * p.Wb;
  const size_t hp = h0 + checked(p, in.par, 0, p.Wb - 1, ERR_LIST_ENTRY);
  const float* xu = p.xT + (size_t)u * p.V * p.Tp;
  const float* x0 = xu + (size_t)p.blank_id * p.Tp;
  const float* xc = xu + (size_t)checked(p, in.tok, 0, p.V - 1, ERR_TOKEN) * p.Tp;
  const double* Bu = p.Bcum + (size_t)u * p.Tp;
  const float* pgn = p.gn[cur] + hp * p.Tp;
  const float* pgb = p.gb[cur] + hp * p.Tp;
  float* cgn = p.gn[cur ^ 1] + (h0 + n) * p.Tp;
  float* cgb = p.gb[cur ^ 1] + (h0 + n) * p.Tp;
  const int T = in.T;
  const int s = checked(p, in.s, 1, T, ERR_WINDOW), en = checked(p, in.en, s, T, ERR_WINDOW), rs = in.rs, re = in.re;
  const double Bnew = Bu[checked(p, in.ptau, 0, T, ERR_TIME_INDEX)];   // the child's reference frame is the parent's tau
  const float delta = in.inc + (float)(Bu[checked(p, in.pref, 0, T, ERR_TIME_INDEX)] - Bnew);
  delta_out = delta;
  bref_out = Bnew;
  const bool rep = (in.tok == in.plast);
  const int lo = max(s, in.ptau);
  float carry_n = LOG0F, carry_b = LOG0F;
  float best_n = LOG0F, best_b = LOG0F;
  arg_n = in.ptau; arg_b = in.ptau_end;
  for (int base = s; base <= en; base += 64 * FPL) {
    int t[FPL]; bool v[FPL]; float bt[FPL];
    Aff mn[FPL];                                         // n_t = (n_{t-1} (+) f_t) + x'_t(c)
    float d[FPL];
#pragma unroll
    for (int k = 0; k < FPL; ++k) {
      t[k] = base + FPL * lane + k;
      v[k] = t[k] <= en;
      const int tc = min(t[k], en);                      // clamped: loads are unconditional
      const float gn = pgn[max(tc - 1, 0)], gb = pgb[max(tc - 1, 0)];
      const float x0v = x0[tc];
      const float x = xc[tc] - fmaxf(x0v, BLANK_FLOOR);
      d[k] = x0v - fmaxf(x0v, BLANK_FLOOR);
      bt[k] = (float)(Bu[tc] - Bnew);
      float f = LOG0F;
      if (t[k] - 1 >= rs && t[k] - 1 <= re) f = rep ? gb : lae(gn, gb);
      mn[k].a = v[k] ? x : 0.0f; mn[k].b = v[k] ? f + x : LOG0F;
    }
    Aff C = mn[0];
#pragma unroll
    for (int k = 1; k < FPL; ++k) C = aff_then(C, mn[k]);
    Aff P = wave_scan_aff(C);
    Aff E;                                               // maps of all earlier lanes
    E.a = dpp_f<0x138, 0xf>(0.0f, P.a); E.b = dpp_f<0x138, 0xf>(LOG0F, P.b);
    const float n_in = lae(E.a + carry_n, E.b);
    float nv[FPL];
    nv[0] = lae(n_in + mn[0].a, mn[0].b);
#pragma unroll
    for (int k = 1; k < FPL; ++k) nv[k] = lae(nv[k - 1] + mn[k].a, mn[k].b);
    Aff mb[FPL];                                         // b_t = (n_{t-1} (+) b_{t-1}) + d_t
#pragma unroll
    for (int k = 0; k < FPL; ++k) {
      const float nprev = k == 0 ? n_in : nv[k - 1];
      mb[k].a = v[k] ? d[k] : 0.0f; mb[k].b = v[k] ? nprev + d[k] : LOG0F;
    }
    C = mb[0];
#pragma unroll
    for (int k = 1; k < FPL; ++k) C = aff_then(C, mb[k]);
    P = wave_scan_aff(C);
    E.a = dpp_f<0x138, 0xf>(0.0f, P.a); E.b = dpp_f<0x138, 0xf>(LOG0F, P.b);
    const float b_in = lae(E.a + carry_b, E.b);
    float bv[FPL];
    bv[0] = lae(b_in + mb[0].a, mb[0].b);
#pragma unroll
    for (int k = 1; k < FPL; ++k) bv[k] = lae(bv[k - 1] + mb[k].a, mb[k].b);
    carry_n = lane_f(nv[FPL - 1], 63); carry_b = lane_f(bv[FPL - 1], 63);
    // re-base, store, and the lane's own first argmax over t >= lo of the true variables
    // (stored + B_t; B relative to the child's reference)
    ArgMax xn, xb;
    xn.v = LOG0F; xn.t = t[0]; xb.v = LOG0F; xb.t = t[0];
#pragma unroll
    for (int k = 0; k < FPL; ++k) {
      const float rn = (nv[k] < LOG0_CLASS) ? LOG0F : nv[k] - delta;
      const float rb = (bv[k] < LOG0_CLASS) ? LOG0F : bv[k] - delta;
      if (v[k]) { cgn[t[k]] = rn; cgb[t[k]] = rb; }
      const bool ok = v[k] && t[k] >= lo;
      const float cn = (ok && rn > LOG0_CLASS) ? rn + bt[k] : LOG0F;
      const float cb = (ok && rb > LOG0_CLASS) ? rb + bt[k] : LOG0F;
      if (cn > xn.v) { xn.v = cn; xn.t = t[k]; }           // (strict: the earlier frame keeps a tie)
      if (cb > xb.v) { xb.v = cb; xb.t = t[k]; }
    }
    xn = wave_argmax(xn); xb = wave_argmax(xb);
    if (xn.v > LOG0_CLASS && xn.v > best_n) { best_n = xn.v; arg_n = xn.t; }
    if (xb.v > LOG0_CLASS && xb.v > best_b) { best_b = xb.v; arg_b = xb.t; }
  }
}

// windows of up to 128 frames: two frames per lane, one pass; up to 256: four per lane (a pass costs
// about 1.4 times as much and covers twice as many frames); longer ones: eight per lane.
// FPLMAX = 2: the kernel carries the two-frames form only (wider windows take several passes of it).  The
// host asks for that when the window margins keep windows within 128 frames but for rare exceptions: the
// forms with more frames per lane are what sets the kernel's register count (97 against 58).
template <int FPLMAX>
__device__ __forceinline__ void wave_survivor(const Params& p, int u, int n, int cur, const SurvivorIn& in,
                                              int& arg_n, int& arg_b, float& delta_out, double& bref_out) {
  const int W = in.en - in.s + 1;
  if (FPLMAX == 2 || W <= 128) wave_survivor_fpl<2>(p, u, n, cur, in, arg_n, arg_b, delta_out, bref_out);
  else if (W <= 256) wave_survivor_fpl<4>(p, u, n, cur, in, arg_n, arg_b, delta_out, bref_out);
  else wave_survivor_fpl<8>(p, u, n, cur, in, arg_n, arg_b, delta_out, bref_out);
}

// How many of the keys s_k2[0 .. 2 * quads) (four per quad, zero padding at the end) exceed `me`,
// counting every L-th quad from `part` on.  Sixteen keys are fetched before the first is compared, so
// that the LDS round trips overlap.
__device__ __forceinline__ int count_greater(const ulonglong2* s_k2, unsigned long long me, int part, int L,
                                             int quads) {
  int n = 0, q4 = part;
  for (; q4 + 3 * L < quads; q4 += 4 * L) {
    ulonglong2 v[8];
#pragma unroll
    for (int k = 0; k < 4; ++k) { v[2 * k] = s_k2[2 * (q4 + k * L)]; v[2 * k + 1] = s_k2[2 * (q4 + k * L) + 1]; }
#pragma unroll
    for (int k = 0; k < 8; ++k) n += (int)(v[k].x > me) + (int)(v[k].y > me);
  }
  for (; q4 < quads; q4 += L) {
    const ulonglong2 v = s_k2[2 * q4], v2 = s_k2[2 * q4 + 1];
    n += (int)(v.x > me) + (int)(v.y > me) + (int)(v2.x > me) + (int)(v2.y > me);
  }
  return n;
}

// The lists are sorted, so few of their Wb * Wb entries can reach the new beam.  A lower bound on the
// Wb-th largest key: the smallest of the first R entries of every non-empty list, R such that those
// are at least Wb entries (if the lists are too short for that: no bound).  Entries below the bound
// cannot rank among the first Wb; the others are packed into s_ck (keys) / s_cidx (their entry
// numbers), followed by zero keys, and only they are ranked against each other: a key carries its
// entry number, so the rank among them is the rank among all.  s_ck must hold zeros on entry,
// s_cnt[0..1] zeros and *s_min all ones; both barriers are inside.  Returns how many were packed.
template <int BLOCK>
__device__ __forceinline__ int pack_contenders(const unsigned long long* s_key, int NE, int Wb, const int* o_n,
                                               unsigned long long* s_ck, int* s_cidx, int* s_cnt,
                                               unsigned long long* s_min) {
  const int tid = threadIdx.x;
  int nl = 0;
#pragma unroll 8
  for (int j = 0; j < Wb; ++j) nl += (o_n[j] > 0);
  const int R = nl > 0 ? (Wb + nl - 1) / nl : 0;
  for (int i = tid; i < NE; i += BLOCK) {
    const int j = i / Wb, r = i - j * Wb;
    if (r < R && r < o_n[j]) { atomicMin(s_min, s_key[i]); atomicAdd(&s_cnt[0], 1); }
  }
  lds_barrier();
  const unsigned long long bound = s_cnt[0] >= Wb ? *s_min : 0ull;
  for (int i = tid; i < NE; i += BLOCK) {
    const unsigned long long k = s_key[i];
    if (k > 1023ull && k >= bound) {
      const int pos = atomicAdd(&s_cnt[1], 1);
      s_ck[pos] = k; s_cidx[pos] = i;
    }
  }
  lds_barrier();
  return s_cnt[1];
}

// Ended set and ENDDETECT of one utterance, by one wave (lane j = old slot j).  `mine`: slot j
// held a live hypothesis; je / stp / tau_j / cells_j: its eos joint score, eos-run stop, tau and
// prefix-score terms of this step.  st_* / ring_*: the utterance's state as loaded by lane 0
// (scalars) and lanes m < M (ring entries).  Writes the state back, the two per-old-slot
// outputs and the work counters; returns whether the utterance finishes at this step.
__device__ __forceinline__ bool wave_ended_set(const Params& p, int u, int l, int T, int lmax_u, bool has_best,
                                               double best, int n_new, bool mine, double je_in, int stp_in,
                                               int tau_j, long long cells_j, double st_best, int st_n,
                                               int st_cnt, double ring_sc, int ring_tag) {
  const int lane = threadIdx.x & 63, Wb = p.Wb;
  const size_t h0 = (size_t)u * Wb;
  UttState* us = p.utt + u;
  const bool forced = (l >= lmax_u);
  const double je = mine ? je_in : LOG0D;
  const int stp = mine ? stp_in : 0;
  const bool je_ok = je > (double)LOG0_CLASS;
  const bool added = mine && (forced || stp || (je_ok && (!has_best || je > best)));
  long long cells = mine ? cells_j : 0;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) cells += __shfl_xor(cells, o);
  const int ngroups = __popcll(__ballot(mine));
  const int n_add = __popcll(__ballot(added));
  const int n_tauT = __popcll(__ballot(added && tau_j == T));
  // best newly ended entry: largest score, lowest slot among equals (the one added first)
  double bje = added ? je : -1.0e300; int bj = added ? lane : 0x7fffffff;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const double ov = __shfl_xor(bje, o); const int oj = __shfl_xor(bj, o);
    if (ov > bje || (ov == bje && oj < bj)) { bje = ov; bj = oj; }
  }
  if (lane < Wb) { p.out_eos_added[h0 + lane] = (uint8_t)added; p.out_stopped[h0 + lane] = (uint8_t)stp; }
  const int n_before = __shfl(st_n, 0);
  const int n_ended = n_before + n_add;
  const int cnt = __shfl(st_cnt, 0) + n_tauT;
  double ybest = __shfl(st_best, 0);
  const bool new_best = n_add > 0 && (n_before == 0 || bje > ybest);
  if (new_best) ybest = bje;
  // ring of the best ended score per length (slot = length % M)
  const int M = p.end_m;
  const bool ring_upd = (lane == (l % M)) && n_add > 0;
  if (ring_upd) { ring_tag = l; ring_sc = bje; }
  bool fin = forced || n_new == 0;
  if (!fin && n_ended > 0) {
    if (p.end_flags & 1) {                       // Eq. (4)
      const bool counts = lane < M && ring_tag >= 1 && ring_tag > l - M && ring_tag <= l &&
                          (ring_sc - ybest < (double)p.end_d);
      if (__popcll(__ballot(counts)) == M) fin = true;
    }
    if (!fin && (p.end_flags & 2) && cnt > p.end_c) fin = true;   // Algorithm 3
  }
  if (ring_upd) { us->ring_tag[lane] = ring_tag; us->ring_score[lane] = ring_sc; }
  if (lane == 0) {
    us->n_ended = n_ended; us->cnt_tau_T = cnt;
    if (new_best) { us->best_score = ybest; us->best_step = l; us->best_slot = bj; }
    if (fin) {
      us->finished_step = l;
      p.finished[u] = 1;
      atomicAdd(p.n_finished, 1);
    }
    p.cells[u] += (unsigned long long)cells;
    p.groups[u] += (unsigned long long)ngroups;
  }
  return fin;
}

// Dynamic LDS: 16 * ((Wb * Wb + 9) & ~1) + 32 * Wb * Wb bytes (the list entries and the packed contenders).
template <int BLOCK, int FPLMAX>
__global__ __launch_bounds__(BLOCK) void k_select(Params p, int l, int cur) {
  constexpr int NW = BLOCK / 64;
  extern __shared__ __align__(16) unsigned char sel_smem[];
  const int NE_ = p.Wb * p.Wb;
  const int NK_ = (NE_ + 9) & ~1;                                     // NE + 8 keys, an even count: both key arrays on 16-byte boundaries
  unsigned long long* s_key = (unsigned long long*)sel_smem;          // [NE + 8]
  unsigned long long* s_ck = s_key + NK_;                             // [NE + 8] keys of the entries that can reach the new beam
  double* s_J = (double*)(s_ck + NK_);                                // [NE]
  int* s_par = (int*)(s_J + NE_);                                     // [NE] each
  int* s_ci = s_par + NE_;
  int* s_tok = s_ci + NE_;
  int* s_cidx = s_tok + NE_;
  float* s_inc = (float*)(s_cidx + NE_);
  float* s_att = s_inc + NE_;
  __shared__ int s_sel[MAX_BEAM];          // entry index of the new beam's slot n
  __shared__ int s_cnt[2];
  __shared__ unsigned long long s_min;
  // old slots' records
  __shared__ int o_live[MAX_BEAM], o_n[MAX_BEAM], o_stp[MAX_BEAM], o_tau[MAX_BEAM], o_tau_end[MAX_BEAM];
  __shared__ int o_rs[MAX_BEAM], o_re[MAX_BEAM], o_last[MAX_BEAM], o_ws[MAX_BEAM], o_we[MAX_BEAM], o_ref[MAX_BEAM];
  __shared__ long long o_cells[MAX_BEAM];
  __shared__ double o_je[MAX_BEAM], o_hatt[MAX_BEAM], o_off[MAX_BEAM];
  __shared__ int s_fin;
  __shared__ int s_ntau[MAX_BEAM], s_ntau_end[MAX_BEAM];   // time indices of the new hypotheses
  __shared__ float s_delta[MAX_BEAM];                      // by how much each new hypothesis was re-based
  __shared__ double s_bref[MAX_BEAM];                      // B at each new hypothesis's reference frame

  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int u = blockIdx.x, Wb = p.Wb;
  if (p.finished[u]) return;               // outputs of a finished utterance were settled when it finished
  const int nxt = cur ^ 1;
  const size_t h0 = (size_t)u * Wb;
  TRACE_POINT(p, u, 8);

  // ---- first round of loads: everything that depends on nothing --------------------------------
  if (tid < Wb) {
    const size_t h = h0 + tid;
    const HypRec r = p.rec[cur][h];
    o_live[tid] = r.live; o_n[tid] = p.grp_n[h]; o_stp[tid] = p.stopped[h];
    o_tau[tid] = r.tau; o_tau_end[tid] = r.tau_end;
    o_rs[tid] = r.rs; o_re[tid] = r.re; o_last[tid] = r.last;
    o_ws[tid] = p.win_s[h]; o_we[tid] = p.win_e[h]; o_ref[tid] = r.ref;
    o_cells[tid] = p.grp_cells[h];
    o_je[tid] = p.joint_eos[h]; o_hatt[tid] = r.att; o_off[tid] = r.off;
  }
  const int T = p.lens[u];
  const int lmax_u = p.lmax[u];
  // utterance state, wave 0: lane 0 the scalars, lanes m < M the ring entries
  UttState* us = p.utt + u;
  double st_best = LOG0D, ring_sc = LOG0D;
  int st_n = 0, st_cnt = 0, ring_tag = -1;
  if (w == 0) {
    if (lane == 0) { st_best = us->best_score; st_n = us->n_ended; st_cnt = us->cnt_tau_T; }
    if (lane < p.end_m) { ring_sc = us->ring_score[lane]; ring_tag = us->ring_tag[lane]; }
  }
  // group lists: entry i = j * Wb + r of this utterance (group j's r-th best; Wb * Wb <= 1024 entries),
  // each with a 64-bit sort key: the score as an order-preserving integer whose 10 lowest mantissa
  // bits are replaced by the entry's position (earlier position = larger key).  One integer comparison
  // then gives a strict total order: joint score descending and, among scores equal to within 2^-42
  // relative (far inside the tolerance to which scores are meaningful), parent slot, then token,
  // ascending.  Entries past a list's length and the padding get keys below every score.
  const int NE = Wb * Wb;
  for (int i = tid; i < NE + 8; i += BLOCK) {
    unsigned long long key = 0ull;
    if (i < NE) {
      const int j = i / Wb, r = i - j * Wb;
      const size_t o = h0 * Wb + i;
      const int nj = p.grp_n[h0 + j];
      const double Jv = p.grp_J[o];
      s_par[i] = j; s_ci[i] = p.grp_ci[o]; s_tok[i] = p.grp_tok[o];
      s_inc[i] = p.grp_inc[o]; s_att[i] = p.grp_att[o];
      s_J[i] = Jv;
      const unsigned long long bb = (unsigned long long)__double_as_longlong(Jv);
      const unsigned long long k = (bb >> 63) ? ~bb : (bb | 0x8000000000000000ull);
      key = r < nj ? ((k & ~1023ull) | (unsigned long long)(1023 - i)) : (unsigned long long)(1023 - i) >> 1;
    }
    s_key[i] = key;
    s_ck[i] = 0ull;
  }
  if (tid < MAX_BEAM) s_sel[tid] = -1;
  if (tid < 2) s_cnt[tid] = 0;
  if (tid == 2) s_min = ~0ull;
  lds_barrier();
  TRACE_POINT(p, u, 9);
  int ne = 0;
#pragma unroll 8
  for (int j = 0; j < Wb; ++j) ne += o_n[j];
  // ---- rank the contenders: L lanes per entry, each comparing against every L-th quad of keys ----
  {
    const int NC = pack_contenders<BLOCK>(s_key, NE, Wb, o_n, s_ck, s_cidx, s_cnt, &s_min);
    const int L = NC <= BLOCK / 8 ? 8 : (NC <= BLOCK / 4 ? 4 : (NC <= BLOCK / 2 ? 2 : 1));
    const int part = tid & (L - 1);
    const int quads = (NC + 3) >> 2;                       // (zeros follow the packed keys)
    const ulonglong2* s_k2 = (const ulonglong2*)s_ck;
    for (int e0 = 0; e0 < NC; e0 += BLOCK / L) {
      const int e = e0 + tid / L;
      const unsigned long long me = s_ck[min(e, NC)];
      int rank = count_greater(s_k2, me, part, L, quads);
      if (L >= 2) rank += dpp_i<0xB1, 0xf>(0, rank);       // quad_perm [1,0,3,2]
      if (L >= 4) rank += dpp_i<0x4E, 0xf>(0, rank);       // quad_perm [2,3,0,1]
      if (L == 8) rank += dpp_i<0x104, 0xf>(0, rank);      // row_shl:4: the first lane of the eight gets the other quad's sum
      if (part == 0 && e < NC && rank < Wb) s_sel[rank] = s_cidx[e];
    }
  }
  lds_barrier();

  TRACE_POINT(p, u, 10);
  // ---- ended set, end detection: wave 0, lane j = old slot j ---------------------------------
  const int n_new = min(ne, Wb);
  if (w == 0) {
    const bool has_best = ne > 0;
    const double best = has_best ? s_J[checked(p, s_sel[0], 0, NE - 1, ERR_LIST_ENTRY)] : LOG0D;
    const int j = lane < Wb ? lane : 0;
    const bool mine = lane < Wb && o_live[j];
    const bool fin = wave_ended_set(p, u, l, T, lmax_u, has_best, best, n_new, mine, o_je[j], o_stp[j], o_tau[j],
                                    o_cells[j], st_best, st_n, st_cnt, ring_sc, ring_tag);
    if (lane == 0) s_fin = fin ? 1 : 0;
  }
  TRACE_POINT(p, u, 11);

  TRACE_POINT(p, u, 12);
  // ---- forward variables of the new hypotheses --------------------------------------------
  // (wave 0 is busy with the ended set above; the other waves take the survivors at once.  A
  // finished utterance's new state is computed too but never used: its slots are marked dead.)
  const size_t trie_l = ((size_t)l * p.U + u) * Wb;
  for (int n = w - 1; n >= 0 && n < n_new; n += NW - 1) {
    const int e = checked(p, s_sel[n], 0, NE - 1, ERR_LIST_ENTRY), par = s_par[e];
    SurvivorIn in;
    in.par = par; in.tok = s_tok[e]; in.inc = s_inc[e]; in.T = T;
    in.s = o_ws[par]; in.en = o_we[par]; in.rs = o_rs[par]; in.re = o_re[par];
    in.ptau = o_tau[par]; in.ptau_end = o_tau_end[par]; in.plast = o_last[par]; in.pref = o_ref[par];
    int arg_n, arg_b;
    float delta;
    double bref;
    wave_survivor<FPLMAX>(p, u, n, cur, in, arg_n, arg_b, delta, bref);
    if (lane == 0) {
      p.out_tau[h0 + n] = arg_n; p.out_tau_end[h0 + n] = arg_b;
      p.trie_tau[trie_l + n] = arg_n;
      s_ntau[n] = arg_n; s_ntau_end[n] = arg_b; s_delta[n] = delta; s_bref[n] = bref;
    }
  }
  lds_barrier();                       // (the survivors' state stores stay in flight)
  const bool fin = s_fin != 0;
  // ---- new beam: records, outputs, back-pointers ------------------------------------------
  for (int n = tid; n < Wb; n += BLOCK) {
    const size_t h = h0 + n;
    if (n < n_new) {
      const int e = checked(p, s_sel[n], 0, NE - 1, ERR_LIST_ENTRY), par = s_par[e], tok = s_tok[e];
      p.out_parent[h] = par; p.out_token[h] = tok; p.out_score[h] = (float)s_J[e];
      p.out_live[h] = fin ? 0 : 1;
      p.trie_parent[trie_l + n] = par; p.trie_token[trie_l + n] = tok;
      HypRec r;
      r.live = fin ? 0 : 1; r.last = tok; r.rs = o_ws[par]; r.re = o_we[par];
      r.tau = s_ntau[n]; r.tau_end = s_ntau_end[n]; r.ref = o_tau[par]; r.pad = 0;
      r.off = o_off[par] + (double)s_delta[n];
      r.att = o_hatt[par] + (double)s_att[e];
      r.joint = s_J[e];
      r.bref = s_bref[n];
      p.rec[nxt][h] = r;
      if (p.win_union && !fin) {                 // this hypothesis's share of the next step's window
        atomicMin(&p.union_win[2 * ((l + 1) & 1)], s_ntau[n]);
        atomicMax(&p.union_win[2 * ((l + 1) & 1) + 1], min(s_ntau_end[n] + p.win_m2, T));
      }
    } else {
      p.out_parent[h] = -1; p.out_token[h] = -1; p.out_score[h] = LOG0F; p.out_live[h] = 0;
      p.out_tau[h] = 0; p.out_tau_end[h] = 0;
      p.trie_parent[trie_l + n] = -1; p.trie_token[trie_l + n] = -1; p.trie_tau[trie_l + n] = 0;
      p.rec[nxt][h].live = 0;
    }
  }

  TRACE_POINT(p, u, 13);
}

// Split form of the select kernel: one work-group per (utterance, new beam slot n), used
// whenever no state is shared across utterances (per-hypothesis windows).  Every work-group of
// an utterance ranks the utterance's Wb * Wb list entries itself (the lists are small, the
// ranking is cheaper than a second launch), wave 0 then evaluates the forward variables of
// new hypothesis n and writes its record; in the work-group of slot 0, wave 1 meanwhile
// updates the ended set, runs ENDDETECT and writes what belongs to the utterance as a whole
// (finished flag, live flags of all slots, the per-old-slot outputs, work counters).  The
// survivors of one utterance so run on Wb compute units instead of sharing one.
// Within a launch the work-groups of an utterance only read what the others do not write:
// the utterance state is read by slot 0's work-group alone, and "finished before this step"
// is taken from the step number at which the utterance finished (0 or the current step both
// mean no).
// Dynamic LDS: 28 * Wb * Wb + 64 bytes (the list entries).
// The arguments in front of the parameter block are what the first round of loads needs (p.rec[cur], p.utt,
// p.grp_n and the list arrays, p.Wb): plain leading arguments reach the wave in registers when it starts
// (kernel-argument preload), so that those loads do not wait for a load of the argument block first.
template <int BLOCK, int FPLMAX>
__global__ __launch_bounds__(BLOCK) void k_select_split(const HypRec* __restrict__ rec_now, UttState* __restrict__ utt,
                                                        const int32_t* __restrict__ grp_n, const double* __restrict__ grp_J,
                                                        const int32_t* __restrict__ grp_tok, const float* __restrict__ grp_inc,
                                                        const float* __restrict__ grp_att, int Wb, int l, Params p, int cur) {
  static_assert(BLOCK >= 128, "wave 0 and wave 1 have different jobs");
  extern __shared__ __align__(16) unsigned char split_smem[];
  const int NE = Wb * Wb;
  unsigned long long* s_key = (unsigned long long*)split_smem;        // [NE + 8]
  double* s_J = (double*)(s_key + NE + 8);                            // [NE]
  int* s_tok = (int*)(s_J + NE);                                      // [NE]
  float* s_inc = (float*)(s_tok + NE);                                // [NE]
  float* s_att = s_inc + NE;                                          // [NE]
  __shared__ int o_live[MAX_BEAM], o_n[MAX_BEAM], o_stp[MAX_BEAM], o_tau[MAX_BEAM], o_tau_end[MAX_BEAM];
  __shared__ int o_rs[MAX_BEAM], o_re[MAX_BEAM], o_last[MAX_BEAM], o_ws[MAX_BEAM], o_we[MAX_BEAM], o_ref[MAX_BEAM];
  __shared__ long long o_cells[MAX_BEAM];
  __shared__ double o_je[MAX_BEAM], o_hatt[MAX_BEAM], o_off[MAX_BEAM];
  __shared__ int s_pick[2];                // entry ranked n, entry ranked 0

  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int u = blockIdx.x / Wb, n = blockIdx.x - u * Wb;
  UttState* us = utt + u;
  const int fs = us->finished_step;        // (tested after the first round of loads is on its way)
  const int nxt = cur ^ 1;
  const size_t h0 = (size_t)u * Wb;
  const bool lead = (n == 0);
  if (lead) TRACE_POINT(p, u, 8);

  // ---- first round of loads: everything that depends on nothing --------------------------------
  if (tid < Wb) {
    const size_t h = h0 + tid;
    const HypRec r = rec_now[h];
    o_live[tid] = r.live; o_n[tid] = grp_n[h]; o_stp[tid] = p.stopped[h];
    o_tau[tid] = r.tau; o_tau_end[tid] = r.tau_end;
    o_rs[tid] = r.rs; o_re[tid] = r.re; o_last[tid] = r.last;
    o_ws[tid] = p.win_s[h]; o_we[tid] = p.win_e[h]; o_ref[tid] = r.ref;
    o_cells[tid] = p.grp_cells[h];
    o_je[tid] = p.joint_eos[h]; o_hatt[tid] = r.att; o_off[tid] = r.off;
  }
  const int T = p.lens[u];
  const int lmax_u = p.lmax[u];
  double st_best = LOG0D, ring_sc = LOG0D;
  int st_n = 0, st_cnt = 0, ring_tag = -1;
  if (lead && w == 1) {
    if (lane == 0) { st_best = us->best_score; st_n = us->n_ended; st_cnt = us->cnt_tau_T; }
    if (lane < p.end_m) { ring_sc = us->ring_score[lane]; ring_tag = us->ring_tag[lane]; }
  }
  // list entries i = j * Wb + r (group j's r-th best), each with a 64-bit sort key: the score as
  // an order-preserving integer whose 10 lowest mantissa bits are replaced by the entry's
  // position (earlier position = larger key).  One integer comparison then gives a strict total
  // order: joint score descending, and among scores equal to within 2^-42 relative (far inside
  // the tolerance to which scores are meaningful) parent slot, then token, ascending.  Entries
  // past a list's length and the padding get keys below every score.
  for (int i = tid; i < NE + 8; i += BLOCK) {
    unsigned long long key = 0ull;
    if (i < NE) {
      const int j = i / Wb, r = i - j * Wb;
      const size_t o = h0 * Wb + i;
      const int nj = grp_n[h0 + j];
      const double Jv = grp_J[o];
      s_tok[i] = grp_tok[o]; s_inc[i] = grp_inc[o]; s_att[i] = grp_att[o];
      s_J[i] = Jv;
      const unsigned long long b = (unsigned long long)__double_as_longlong(Jv);
      const unsigned long long k = (b >> 63) ? ~b : (b | 0x8000000000000000ull);
      key = r < nj ? ((k & ~1023ull) | (unsigned long long)(1023 - i)) : (unsigned long long)(1023 - i) >> 1;
    }
    s_key[i] = key;
  }
  if (tid < 2) s_pick[tid] = -1;
  if (fs != 0 && fs < l) return;           // outputs of a finished utterance were settled when it finished
  lds_barrier();
  if (lead) TRACE_POINT(p, u, 9);

  // ---- rank (total order: joint desc, parent slot asc, token asc = position asc) -------------
  // L lanes per entry, each comparing against every L-th pair of the list
  int ne = 0;
#pragma unroll 8
  for (int j = 0; j < Wb; ++j) ne += o_n[j];
  const int n_new = min(ne, Wb);
  // (all entries against all: packing the contenders first, as the per-utterance kernel does, costs two
  // barriers more than it saves at these sizes -- measured)
  {
    const int L = NE <= 64 ? 4 : (NE <= 128 ? 2 : 1);
    const int part = tid & (L - 1);
    const int quads = (NE + 3) >> 2;                       // (the padding holds zeros)
    const ulonglong2* s_k2 = (const ulonglong2*)s_key;
    for (int e0 = 0; e0 < NE; e0 += BLOCK / L) {
      const int e = e0 + tid / L;
      const unsigned long long me = s_key[min(e, NE)];
      int rank = count_greater(s_k2, me, part, L, quads);
      if (L >= 2) rank += dpp_i<0xB1, 0xf>(0, rank);       // quad_perm [1,0,3,2]
      if (L == 4) rank += dpp_i<0x4E, 0xf>(0, rank);       // quad_perm [2,3,0,1]
      if (part == 0 && e < NE && me > 1023ull) {
        if (rank == n) s_pick[0] = e;
        if (rank == 0) s_pick[1] = e;
      }
    }
  }
  lds_barrier();
  if (lead) TRACE_POINT(p, u, 10);

  const size_t trie_l = ((size_t)l * p.U + u) * Wb;
  if (w == 0) {
    // ---- new hypothesis n: forward variables, record, outputs, back-pointer -----------------
    const size_t h = h0 + n;
    if (n < n_new) {
      const int e = checked(p, s_pick[0], 0, NE - 1, ERR_LIST_ENTRY), par = e / Wb;
      SurvivorIn in;
      in.par = par; in.tok = s_tok[e]; in.inc = s_inc[e]; in.T = T;
      in.s = o_ws[par]; in.en = o_we[par]; in.rs = o_rs[par]; in.re = o_re[par];
      in.ptau = o_tau[par]; in.ptau_end = o_tau_end[par]; in.plast = o_last[par]; in.pref = o_ref[par];
      int arg_n, arg_b;
      float delta;
      double bref;
      wave_survivor<FPLMAX>(p, u, n, cur, in, arg_n, arg_b, delta, bref);
      if (lane == 0) {
        p.out_tau[h] = arg_n; p.out_tau_end[h] = arg_b;
        p.trie_tau[trie_l + n] = arg_n;
        p.out_parent[h] = par; p.out_token[h] = in.tok; p.out_score[h] = (float)s_J[e];
        p.trie_parent[trie_l + n] = par; p.trie_token[trie_l + n] = in.tok;
        // (the record's live flag belongs to the utterance's lead work-group, see below)
        HypRec* r = p.rec[nxt] + h;
        r->last = in.tok; r->rs = in.s; r->re = in.en; r->tau = arg_n; r->tau_end = arg_b; r->ref = in.ptau;
        r->off = o_off[par] + (double)delta;
        r->att = o_hatt[par] + (double)s_att[e];
        r->joint = s_J[e];
        r->bref = bref;
      }
    } else if (lane == 0) {
      p.out_parent[h] = -1; p.out_token[h] = -1; p.out_score[h] = LOG0F;
      p.out_tau[h] = 0; p.out_tau_end[h] = 0;
      p.trie_parent[trie_l + n] = -1; p.trie_token[trie_l + n] = -1; p.trie_tau[trie_l + n] = 0;
    }
  } else if (lead && w == 1) {
    // ---- the utterance as a whole: ended set, end detection, live flags ----------------------
    const bool has_best = ne > 0;
    const double best = has_best ? s_J[checked(p, s_pick[1], 0, NE - 1, ERR_LIST_ENTRY)] : LOG0D;
    const int j = lane < Wb ? lane : 0;
    const bool mine = lane < Wb && o_live[j];
    const bool fin = wave_ended_set(p, u, l, T, lmax_u, has_best, best, n_new, mine, o_je[j], o_stp[j], o_tau[j],
                                    o_cells[j], st_best, st_n, st_cnt, ring_sc, ring_tag);
    if (lane < Wb) {
      const int lv = (lane < n_new && !fin) ? 1 : 0;
      p.out_live[h0 + lane] = (uint8_t)lv;
      p.rec[nxt][h0 + lane].live = lv;
    }
  }
  if (lead) TRACE_POINT(p, u, 13);
}
