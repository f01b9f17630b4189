// Score kernel: one work-group per (utterance, beam slot) hypothesis g.
//   1. candidate pre-selection: the K ids with the largest attention log-prob, ties to the
//      smaller id.  The row never goes through LDS: every lane keeps its float4 loads in
//      registers.  Fast path: a
//      pivot L that is provably not above
//      the K-th largest value (every wave contributes the ceil(K/#waves)-th largest of its
//      lanes' maxima, found by bisection on the upper key bits), then an exact ranking of the
//      few values >= L.  Rows that do not fit the registers, or with so many values >= L that
//      the short list overflows (heavy ties), take a radix select that re-reads the row.
//   2. window [s, e] from g's time indices (the two equations after Eq. (5));
//   3. prefix score of every extension g.c: log-sum over t in [s, e] of
//      f_t + log p^c(z_t = c), f_t = blank variable of g at t-1 if c repeats g's last label,
//      else phi_{t-1}(g)  (Eq. (3) / Eq. (5)); frames run along lanes (16 or 64 lanes per
//      candidate, float4 per lane), all of a lane's column loads are issued before the first
//      is consumed, streaming log-sum-exp with one exp per term;
//   4. eos score phi_T(g), joint scores (Eq. (1)), the eos-run test, and the group's
//      best-first list of at most Wb candidates for the per-utterance selection.
// The candidate list of a group is in no particular (but reproducible) order; wherever
// equal scores must be ordered the token id decides.
#pragma once
#include "common.h"

#define PIVOT_CAP 512     // entries of the short list (all waves together)
#define PIVOT_NV4 6       // float4 loads per lane held in registers (rows of up to 6144 ids)
#define RADIX_BITS 10

struct ScoreSmem {
  // byte offsets into dynamic LDS, computed on the host
  int32_t off_work;   // union: uint32 hist[1 << RADIX_BITS] | short list of the pivot selection
  int32_t off_f;      // float F[wp_max], Fb[wp_max]
  int32_t off_small;  // per-candidate arrays of the group (K <= block size), see k_score
  int32_t wp_max;     // floats available per F array
};

__device__ __forceinline__ float key_to_att(uint32_t k) {
  return __uint_as_float((k & 0x80000000u) ? (k & 0x7fffffffu) : ~k);
}

// ---- candidate selection -----------------------------------------------------------------
// Pivot path on the lane's register-resident row values (v[k] = ids 4 * (tid + k * BLOCK) ..+3;
// excluded ids and ids past the row's end hold -inf).  Comparisons run on the floats
// themselves; only each lane's maximum and the few collected values are turned into
// order-preserving keys.  Short-list entries are 64-bit: key in the upper word, ~id in the
// lower, so that one integer comparison orders by (value descending, id ascending).
// Returns false (uniformly) if the short list would overflow or, with NaNs in the row, would
// hold fewer than K values.  Writes the K ids (and their attention values) best first.
// s_ent: PIVOT_CAP + 4 entries; s_w: 2 * (BLOCK / 64) words.
template <int BLOCK>
__device__ __forceinline__ bool select_pivot(const float4 (&v)[PIVOT_NV4], int K, int blank_id, int eos_id,
                                             unsigned long long* s_ent, uint32_t* s_w, bool use_lds,
                                             int32_t* out_lds, float* out_att_lds, int32_t* out_g,
                                             unsigned long long* tr) {
  constexpr int NW = BLOCK / 64;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const float ninf = -__builtin_huge_valf();
  float fmx = ninf;
#pragma unroll
  for (int k = 0; k < PIVOT_NV4; ++k)
    fmx = fmaxf(fmx, fmaxf(fmaxf(v[k].x, v[k].y), fmaxf(v[k].z, v[k].w)));
  const uint32_t lmax = att_key(fmx, -1, -2, -2);
  TRACE_MARK_AT(tr, 6);
  // r-th largest lane maximum of this wave, by bisection on the upper 16 key bits (sign,
  // exponent, 7 mantissa bits): stopping early only lowers the pivot, which stays valid
  const int r = (K + NW - 1) / NW;
  uint32_t thr = 0;
#pragma unroll 4
  for (int bit = 31; bit >= 16; --bit) {
    const uint32_t trial = thr | (1u << bit);
    if (__popcll(__ballot(lmax >= trial)) >= r) thr = trial;
  }
  TRACE_MARK_AT(tr, 7);
  if (lane == 0) s_w[w] = thr;
  lds_barrier();
  uint32_t Lk = s_w[0];
#pragma unroll
  for (int i = 1; i < NW; ++i) Lk = min(Lk, s_w[i]);
  // at least NW * r >= K values are >= L (as a float: -inf if no wave had r finite maxima)
  const float L = Lk <= att_key(ninf, -1, -2, -2) ? ninf : key_to_att(Lk);
  // hits are rare (about 1.4 K of the whole row).  Every lane notes its own in a bit mask (bit
  // 4k+j = component j of v[k]); a wave scan of the counts and the waves' totals give each lane the
  // place of its first hit in the short list
  uint32_t mask = 0;
#pragma unroll
  for (int k = 0; k < PIVOT_NV4; ++k)
    mask |= ((uint32_t)(v[k].x >= L) << (4 * k)) | ((uint32_t)(v[k].y >= L) << (4 * k + 1)) |
            ((uint32_t)(v[k].z >= L) << (4 * k + 2)) | ((uint32_t)(v[k].w >= L) << (4 * k + 3));
  const int cnt = __popc(mask);
  const int inc = (int)wave_incl_scan_u32((uint32_t)cnt, lane);
  if (lane == 63) s_w[NW + w] = (uint32_t)inc;
  lds_barrier();
  int base = 0, total = 0;
#pragma unroll
  for (int i = 0; i < NW; ++i) { const int c = (int)s_w[NW + i]; base += i < w ? c : 0; total += c; }
  if (total > PIVOT_CAP || total < K) return false;
  TRACE_MARK_AT(tr, 14);
  const bool linf = (L == ninf);                           // then excluded ids (held as -inf) are hits too
  int pos = base + inc - cnt;
  // per float4 slot, one hit per trip (most lanes have none, hardly any more than one)
#pragma unroll
  for (int k = 0; k < PIVOT_NV4; ++k) {
    uint32_t m4 = (mask >> (4 * k)) & 15u;
    while (m4 != 0u) {
      const int j = __ffs((int)m4) - 1;
      m4 &= m4 - 1u;
      const float val = j == 0 ? v[k].x : (j == 1 ? v[k].y : (j == 2 ? v[k].z : v[k].w));
      const int id = 4 * (tid + k * BLOCK) + j;
      const uint32_t u = __float_as_uint(val);
      uint32_t key = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
      if (linf && (id == blank_id || id == eos_id)) key = 0u;   // below a genuine -inf
      s_ent[pos++] = ((unsigned long long)key << 32) | (uint32_t)~id;
    }
  }
  const int n = total;
  const int n4 = (n + 3) >> 2;
  if (tid < 4 && n + tid < 4 * n4) s_ent[n + tid] = 0ull;    // pad to a multiple of four
  lds_barrier();
  TRACE_MARK_AT(tr, 15);
  // exact rank: four lanes per entry, each comparing against a quarter of the list (two entries
  // per read), partial ranks summed inside the quad; the rank is the output slot
  const int part = tid & 3;
  const ulonglong2* s_ent2 = (const ulonglong2*)s_ent;
  for (int e = tid >> 2; e < ((n + BLOCK / 4 - 1) / (BLOCK / 4)) * (BLOCK / 4); e += BLOCK / 4) {
    const unsigned long long me = e < n ? s_ent[e] : ~0ull;
    int rank = 0;
    for (int o4 = part; o4 < n4; o4 += 4) {
      const ulonglong2 a = s_ent2[2 * o4], b = s_ent2[2 * o4 + 1];
      rank += (int)(a.x > me) + (int)(a.y > me) + (int)(b.x > me) + (int)(b.y > me);
    }
    rank += dpp_i<0xB1, 0xf>(0, rank);                     // quad_perm [1,0,3,2]
    rank += dpp_i<0x4E, 0xf>(0, rank);                     // quad_perm [2,3,0,1]
    if (part == 0 && e < n && rank < K) {
      const int mid = (int)~(uint32_t)me;
      // (small K: the ids stay in LDS; the global copy is written with the scores at the end, so that
      // no store is pending when the candidates' columns are fetched)
      if (use_lds) { out_lds[rank] = mid; out_att_lds[rank] = key_to_att((uint32_t)(me >> 32)); }
      else out_g[rank] = mid;
    }
  }
  return true;
}

// Radix select on the order-preserving keys (10 + 10 + 10 + 2 bits) straight from the row in
// global memory, then an ordered compaction (ascending ids).
template <int BLOCK>
__device__ __forceinline__ void select_radix(const float* __restrict__ arow, int V, int K, int blank_id, int eos_id,
                                          uint32_t* s_hist, uint32_t* s_scan, uint32_t* s_sel,
                                          bool use_lds, int32_t* out_lds, float* out_att_lds, int32_t* out_g) {
  const int tid = threadIdx.x;
  uint32_t prefix = 0, pmask = 0, krem = (uint32_t)K;
#pragma unroll 1
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = pass == 0 ? 22 : (pass == 1 ? 12 : (pass == 2 ? 2 : 0));
    const int bits = pass == 3 ? 2 : RADIX_BITS;
    const uint32_t bmask = (1u << bits) - 1u;
    const int nb = 1 << bits;
    __syncthreads();
    for (int i = tid; i < nb; i += BLOCK) s_hist[i] = 0;
    __syncthreads();
    for (int i = tid; i < V; i += BLOCK) {
      uint32_t k = att_key(arow[i], i, blank_id, eos_id);
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
  // (those with the smallest ids).  Ordered compaction, contiguous id chunk per thread; the
  // two counts are scanned separately (either can be as large as the row).
  const int chunk = (V + BLOCK - 1) / BLOCK;
  const int i0 = min(V, tid * chunk), i1 = min(V, i0 + chunk);
  uint32_t gt = 0, eq = 0;
  for (int i = i0; i < i1; ++i) {
    uint32_t k = att_key(arow[i], i, blank_id, eos_id);
    gt += (k > prefix); eq += (k == prefix);
  }
  uint32_t total;
  const uint32_t gt_before = block_excl_scan_u32<BLOCK>(gt, s_scan, &total);
  uint32_t eq_before = block_excl_scan_u32<BLOCK>(eq, s_scan, &total);
  uint32_t pos = gt_before + min(eq_before, krem);
  for (int i = i0; i < i1; ++i) {
    const float a = arow[i];
    uint32_t k = att_key(a, i, blank_id, eos_id);
    bool take = (k > prefix) || (k == prefix && eq_before < krem);
    if (k == prefix) ++eq_before;
    if (take && pos < (uint32_t)K) {
      if (use_lds) { out_lds[pos] = i; out_att_lds[pos] = a; }
      else out_g[pos] = i;
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
  static_assert(LPC == 16 || LPC == 64, "a candidate's lanes are one DPP row or one wave");
  float M = row16_max(a.m);
  if (LPC == 64) M = fmaxf(fmaxf(lane_f(M, 0), lane_f(M, 16)), fmaxf(lane_f(M, 32), lane_f(M, 48)));
  float s = row16_sum(a.s * __expf(a.m - M));
  if (LPC == 64) s = (lane_f(s, 0) + lane_f(s, 16)) + (lane_f(s, 32) + lane_f(s, 48));
  return (M < LOG0_CLASS) ? LOG0F : M + fast_logf(s);    // (s >= 1: the largest term contributes 1)
}

// Block-wide maximum / sum (logits mode: log-sum-exp of a whole attention row).  The per-lane
// partials are floats; partial sums are added in fp64.
template <int BLOCK>
__device__ __forceinline__ float block_max_f(float m, float* s_red /*[BLOCK / 64]*/) {
  constexpr int NW = BLOCK / 64;
  m = row16_max(m);
  m = fmaxf(fmaxf(lane_f(m, 0), lane_f(m, 16)), fmaxf(lane_f(m, 32), lane_f(m, 48)));
  lds_barrier();
  if ((threadIdx.x & 63) == 0) s_red[threadIdx.x >> 6] = m;
  lds_barrier();
  float M = s_red[0];
#pragma unroll
  for (int i = 1; i < NW; ++i) M = fmaxf(M, s_red[i]);
  return M;
}
template <int BLOCK>
__device__ __forceinline__ double block_sum_d(float sum, double* s_d /*[BLOCK / 64]*/) {
  constexpr int NW = BLOCK / 64;
  sum = row16_sum(sum);
  const double ws = ((double)lane_f(sum, 0) + (double)lane_f(sum, 16)) +
                    ((double)lane_f(sum, 32) + (double)lane_f(sum, 48));
  lds_barrier();
  if ((threadIdx.x & 63) == 0) s_d[threadIdx.x >> 6] = ws;
  lds_barrier();
  double tot = 0.0;
#pragma unroll
  for (int i = 0; i < NW; ++i) tot += s_d[i];
  return tot;
}

// Order-preserving 64-bit image of a joint score with the token in its 16 lowest mantissa bits:
// one integer comparison then orders by (score descending, token ascending); scores equal to
// within 2^-36 relative count as equal.  0 = not a competitor.  Needs token ids below 65536.
__device__ __forceinline__ unsigned long long joint_key(double J, int tok, bool valid) {
  if (!valid) return 0ull;
  const unsigned long long b = (unsigned long long)__double_as_longlong(J);
  const unsigned long long k = (b >> 63) ? ~b : (b | 0x8000000000000000ull);
  return (k & ~0xFFFFull) | (unsigned long long)(0xFFFF - tok);
}

// Grid: (Wb, U).  flags bit 0: the attention rows start on 16-byte boundaries.
// The arguments in front of the parameter block are what the first loads of a work-group need (the records
// of the current buffer = p.rec[cur], p.uinfo, p.finished as words, the attention rows, p.Wb, p.V): as plain
// leading arguments they are handed to the wave in registers when it starts (kernel-argument preload),
// so that the record's load does not have to wait for a load of the argument block first.
// BIGK: more candidates per hypothesis than one wave ranks (K > 64, or ids beyond 65535).  Only that form of the
// kernel carries the paths for it: candidate arrays in global memory when K exceeds the work-group, the exact
// ranking by the whole work-group, the eos-run rule's work-group-wide path (a second sum beside the first in
// the column pass, the test across all waves).  They cost registers that the common form does without (69
// against 77-89, i.e. seven work-groups per compute unit against five or six).
template <int BLOCK, int LPC, int CB, int IT, bool BIGK>
__global__ __launch_bounds__(BLOCK, (CB * IT > 8 ? 4 : 5)) void k_score(const HypRec* __restrict__ rec_now,
                                                 const UttInfo* __restrict__ uinfo, const uint32_t* __restrict__ fin_words,
                                                 const float* __restrict__ att, int Wb, int V, int flags, int l,
                                                 Params p, ScoreSmem sm, int cur) {
  extern __shared__ __align__(16) unsigned char smem[];
  __shared__ uint32_t s_scan[BLOCK / 64 + 1];
  __shared__ uint32_t s_w[2 * (BLOCK / 64)];
  __shared__ uint32_t s_sel[2];
  __shared__ float s_e2w[(BLOCK / 64) * MAX_EOS_RUN + 1];
  __shared__ int s_nvalid;
  __shared__ __align__(8) float s_red[4 * (BLOCK / 64)];   // BLOCK/64 floats, then BLOCK/64 doubles
  __shared__ double s_eos[2];                              // eos scores, computed early, written at the end
  __shared__ float s_e2f[2 * MAX_EOS_RUN];                 // eos-run rule: f terms of the last R frames (both kinds)

  const int tid = threadIdx.x;
  const int u = blockIdx.y;
  const int grp = u * Wb + blockIdx.x;
  // first round of loads, g's record and the utterance's constants: one 64-byte line and one 16-byte entry
  // through the scalar path (uniform addresses, nothing in this kernel writes them)
  const HypRec rec = rec_now[grp];
  const UttInfo ui = uinfo[u];
  // (the utterance's finished byte is fetched as part of its aligned word: a uniform word load
  // can take the scalar path, a byte load cannot)
  const uint32_t fin_word = fin_words[u >> 2];
  TRACE_DECL;
  const int K = p.K;
  const bool smallk = !BIGK || (K <= BLOCK);

  // ---------------- the attention row -----------------------------------------------------------
  // As soon as the record says that the slot holds a hypothesis its row is fetched, all loads in
  // flight together (a dead slot fetches nothing).
  const float* arow = att + (size_t)grp * V;
  const bool in_regs = p.restricted && (V & 3) == 0 && (V >> 2) <= PIVOT_NV4 * BLOCK && (flags & 1);
  float4 arow_r[PIVOT_NV4];
  const int dead = (int)((fin_word >> (8 * (u & 3))) & 0xffu) | (rec.live == 0);
  if (in_regs && !dead) {
    const float4* a4 = (const float4*)arow;
    const int nv4 = V >> 2;
#pragma unroll
    for (int k = 0; k < PIVOT_NV4; ++k) arow_r[k] = a4[min(tid + k * BLOCK, nv4 - 1)];
  }
  const int T = ui.T;
  const int tau = rec.tau, tau_end = rec.tau_end;
  const int rs = rec.rs, re = rec.re, last = rec.last;
  const double off = rec.off, acum = rec.att;
  // publish the count of finished utterances (as of the previous step) where the host can
  // read it without synchronising: one writer, plain store to device-mapped pinned memory
  if (grp == 0 && tid == 0) {
    *(volatile int32_t*)p.host_finished = *p.n_finished;
    __threadfence_system();
    // batch-union window: clear the slot the select kernel of this step will fill for the next one
    p.union_win[2 * ((l + 1) & 1)] = 0x7fffffff;
    p.union_win[2 * ((l + 1) & 1) + 1] = -1;
  }
  if (dead) {
    if (tid == 0) {
      p.grp_n[grp] = 0; p.win_s[grp] = 0; p.win_e[grp] = -1; p.stopped[grp] = 0;
      p.ctc_eos[grp] = LOG0D; p.joint_eos[grp] = LOG0D; p.grp_cells[grp] = 0;
    }
    return;
  }

  TRACE_MARK(0);
  uint32_t* s_work = (uint32_t*)(smem + sm.off_work);
  float* s_F = (float*)(smem + sm.off_f);
  float* s_Fb = s_F + sm.wp_max;
  // per-candidate arrays of the group (K <= BLOCK): sort key and joint score (8 bytes each), then
  // id, prefix-score increment, attention value, eos-run scratch (4 bytes each)
  const int Ks = smallk ? K : 0;
  unsigned long long* s_key = (unsigned long long*)(smem + sm.off_small);
  double* s_J = (double*)(s_key + Ks);                     // joint score as computed (NaN kept)
  int32_t* s_cid = (int32_t*)(s_J + Ks);                   // only touched when smallk
  float* s_inc = (float*)(s_cid + Ks);
  float* s_av = s_inc + Ks;
  float* s_pre = s_av + Ks;                                // eos-run rule: prefix score without the last R frames
  int32_t* g_cid = p.cand_id + (size_t)grp * K;

  // logits mode: the row holds unnormalised scores; log_softmax is folded in here (the order of
  // the ids is the same, only the values the scores use are shifted by the row's log-sum-exp)
  float row_lse = 0.0f;
  if (p.att_logits) {
    float* s_redf = s_red;
    double* s_redd = (double*)(s_red + 2 * (BLOCK / 64));
    float m = -3.0e38f, sum = 0.0f;
    if (in_regs) {
      const int nv4 = V >> 2;
#pragma unroll
      for (int k = 0; k < PIVOT_NV4; ++k)
        if (tid + k * BLOCK < nv4)
          m = fmaxf(m, fmaxf(fmaxf(arow_r[k].x, arow_r[k].y), fmaxf(arow_r[k].z, arow_r[k].w)));
      const float M = block_max_f<BLOCK>(m, s_redf);
#pragma unroll
      for (int k = 0; k < PIVOT_NV4; ++k)
        if (tid + k * BLOCK < nv4)
          sum += (__expf(arow_r[k].x - M) + __expf(arow_r[k].y - M)) + (__expf(arow_r[k].z - M) + __expf(arow_r[k].w - M));
      row_lse = (float)((double)M + log(block_sum_d<BLOCK>(sum, s_redd)));
    } else {
      for (int i = tid; i < V; i += BLOCK) m = fmaxf(m, arow[i]);
      const float M = block_max_f<BLOCK>(m, s_redf);
      for (int i = tid; i < V; i += BLOCK) sum += __expf(arow[i] - M);
      row_lse = (float)((double)M + log(block_sum_d<BLOCK>(sum, s_redd)));
    }
  }

  // ---------------- window (needs only g's record) ----------------------------------------
  int s = l > 1 ? l : 1, e = T;
  if (p.win_union) {            // s^l = min_ij s_ij, e^l = max_ij e_ij (last two equations of Sec. 3.2.3)
    if (p.win_m1 >= 0) s = max(s, p.union_win[2 * (l & 1)] - p.win_m1);
    if (p.win_m2 >= 0) e = min(e, p.union_win[2 * (l & 1) + 1]);
  } else {
    if (p.win_m1 >= 0) s = max(s, tau - p.win_m1);
    if (p.win_m2 >= 0) e = min(e, tau_end + p.win_m2);
  }
  s = checked(p, s, 1, T + 1, ERR_WINDOW);                 // (an empty window is e < s; its loads stay inside the row)
  e = checked(p, e, -1, T, ERR_WINDOW);
  const int W = e >= s ? e - s + 1 : 0;
  const int t0 = s & ~3;                                   // column loads start on a 16-byte boundary
  const int n4 = W > 0 ? ((e - t0) >> 2) + 1 : 0;
  const int Wp = n4 * 4;
  const float* gn = p.gn[cur] + (size_t)grp * p.Tp;
  const float* gb = p.gb[cur] + (size_t)grp * p.Tp;
  // Stored forward variables have the per-frame reference B_t taken out (see Params::Bcum); all
  // increments of this step are relative to off'(g) + B_r, r = g's reference frame
  const double* Bu = p.Bcum + (size_t)u * p.Tp;
  const double Bref = rec.bref;
  const double offr = off + Bref;
  const double BT = ui.BT - Bref;                          // B_T - B_r

  // eos inputs (thread 0), fetched now so that nothing waits for them later
  float eos_n = LOG0F, eos_b = LOG0F, eos_a = 0.0f;
  if (tid == 0) {
    if (rs <= T && re >= T) { eos_n = gn[T]; eos_b = gb[T]; }
    eos_a = arow[p.eos_id];               // (logits mode: shifted by the row's log-sum-exp below)
  }

  TRACE_MARK(1);
  // ---------------- stage the f terms of the window in LDS ---------------------------------
  // gamma_{t-1}(g) - off' - B_r = stored_{t-1} + (B_{t-1} - B_r); far from r the second part is
  // large and coarse in fp32, and the term is then negligible by that same factor
  auto f_terms = [&](int t, float& f, float& fb) {
    f = LOG0F; fb = LOG0F;
    if (t >= s && t <= e) {
      const int pr = t - 1;
      if (pr >= rs && pr <= re) {
        const float bt = (float)(Bu[pr] - Bref);
        const float n = gn[pr]; fb = gb[pr]; f = canon0(lae(n, fb) + bt); fb = canon0(fb + bt);
      }
    }
  };
  const int R = p.eos_run;
  const bool e2 = (p.end_flags & 4) && R > 0 && T >= R && W > 0 && e == T && re == T &&
                  max(s, rs) <= T - R + 1;
  const bool wave_rank = !BIGK || (smallk && K <= 64 && V <= 65536);  // the group's list is ranked by one wave on 64-bit keys
  // eos-run rule with few candidates: the f terms of the last R frames are kept apart (and left out of the
  // window's arrays), so that the sums below stop at frame T - R; the first wave completes them at the end
  const bool e2w = e2 && wave_rank;
  const bool e2g = BIGK && e2 && !wave_rank;               // the rule by the whole work-group (many candidates)
  for (int i = tid; i < Wp; i += BLOCK) {
    float f, fb;
    f_terms(t0 + i, f, fb);
    const int k = t0 + i - (T - R + 1);
    if (e2w && k >= 0 && k < R) { s_e2f[k] = f; s_e2f[MAX_EOS_RUN + k] = fb; f = LOG0F; fb = LOG0F; }
    s_F[i] = f; s_Fb[i] = fb;
  }
  const double lam = p.lambda, jbase = (1.0 - lam) * acum + p.beta * (double)l;
  // eos-run rule: E_t = phi_t(g) of frame t = T-R+1+tid, fetched now so that the test at the end does not wait for it
  float e2_Et = LOG0F;
  if (e2 && tid < R) {
    const int t = T - R + 1 + tid;
    e2_Et = canon0(lae(gn[t], gb[t]) + (float)(Bu[t] - Bref));
  }
  if (tid == 0) {
    // eos: phi_T(g) = off' + B_T + stored
    const float ce = (rs <= T && re >= T) ? canon0(lae(eos_n, eos_b)) : LOG0F;
    const bool v = ce > LOG0_CLASS;
    const double ctc = v ? offr + BT + (double)ce : LOG0D;
    s_eos[0] = ctc;
    s_eos[1] = v ? lam * ctc + (1.0 - lam) * (double)(eos_a - row_lse) + jbase : LOG0D;
  }
  TRACE_MARK(2);

  // ---------------- 1. candidates -----------------------------------------------------------
  if (p.restricted) {
    bool ok = false;
    if (in_regs) {
      // ids past the row's end, blank and eos never compete: hold them as -inf
      const int nv4 = V >> 2;
      const float ninf = -__builtin_huge_valf();
#pragma unroll
      for (int k = 0; k < PIVOT_NV4; ++k) {
        const int i4 = tid + k * BLOCK;
        if (i4 >= nv4) arow_r[k] = make_float4(ninf, ninf, ninf, ninf);
        if (i4 == (p.blank_id >> 2) || i4 == (p.eos_id >> 2)) {
          const int jb = i4 == (p.blank_id >> 2) ? (p.blank_id & 3) : -1;
          const int je = i4 == (p.eos_id >> 2) ? (p.eos_id & 3) : -1;
          if (jb == 0 || je == 0) arow_r[k].x = ninf;
          if (jb == 1 || je == 1) arow_r[k].y = ninf;
          if (jb == 2 || je == 2) arow_r[k].z = ninf;
          if (jb == 3 || je == 3) arow_r[k].w = ninf;
        }
      }
      ok = select_pivot<BLOCK>(arow_r, K, p.blank_id, p.eos_id, (unsigned long long*)s_work,
                               s_w, smallk, s_cid, s_av, g_cid, TRACE_ARG);
    }
    if (!ok) select_radix<BLOCK>(arow, V, K, p.blank_id, p.eos_id, s_work, s_scan, s_sel, smallk, s_cid, s_av, g_cid);
  } else {
    const int lo_ex = min(p.blank_id, p.eos_id), hi_ex = max(p.blank_id, p.eos_id);
    for (int i = tid; i < K; i += BLOCK) {
      const int id = full_v_id(i, lo_ex, hi_ex);
      if (smallk) { s_cid[i] = id; s_av[i] = arow[id]; }
      else g_cid[i] = id;
    }
  }
  // candidates and f terms visible to the whole block (large K: the ids are read back from global memory)
  if (smallk) lds_barrier(); else __syncthreads();
  TRACE_MARK(3);

  // ---------------- 3. prefix scores ----------------------------------------------------
  constexpr int NSG = BLOCK / LPC;
  const int sg = tid / LPC, q = tid % LPC;
  const float* xu = p.xT + (size_t)u * V * p.Tp;
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
      ids[b] = (c < K) ? checked(p, smallk ? s_cid[c] : g_cid[c], 0, V - 1, ERR_CAND_ID) : -1;
      const float4* col = (const float4*)(xu + (size_t)(ids[b] < 0 ? 0 : ids[b]) * p.Tp + t0);
#pragma unroll
      for (int it = 0; it < IT; ++it)                        // unconditional (clamped) loads: all in flight together
        x[b][it] = col[min(q + it * LPC, max(n4 - 1, 0))];
    }
#pragma unroll
    for (int b = 0; b < CB; ++b) {
      const int c = c0 + b * NSG;
      if (ids[b] < 0) continue;                            // uniform over the LPC lanes of a chain
      const int id = ids[b];
      const float4* col = (const float4*)(xu + (size_t)id * p.Tp + t0);
      const float4* f4 = (const float4*)(s_F + ((id == last) ? sm.wp_max : 0));   // Fb follows F
      float inc = LOG0F, pre = LOG0F;
      {
        Lse a; a.m = LOG0F; a.s = 0.0f;
        if (!e2g) {
#pragma unroll
          for (int it = 0; it < IT; ++it) {
            const int i = q + it * LPC;
            if (i < n4) lse_add4(a, x[b][it], f4[i]);
          }
          for (int i = q + IT * LPC; i < n4; i += LPC) lse_add4(a, col[i], f4[i]);
        } else {
          // the sum in two parts: frames up to T - R (needed on its own below) and the last R frames,
          // which only the few lanes at the window's end hold
          Lse aq; aq.m = LOG0F; aq.s = 0.0f;
          const int tc = T - R;
          auto split = [&](const float4 xv, const float4 fv, int tb) {
            float4 fc;
            fc.x = tb <= tc ? fv.x : LOG0F; fc.y = tb + 1 <= tc ? fv.y : LOG0F;
            fc.z = tb + 2 <= tc ? fv.z : LOG0F; fc.w = tb + 3 <= tc ? fv.w : LOG0F;
            lse_add4(a, xv, fc);
            if (tb + 3 > tc) {
              fc.x = tb > tc ? fv.x : LOG0F; fc.y = tb + 1 > tc ? fv.y : LOG0F;
              fc.z = tb + 2 > tc ? fv.z : LOG0F; fc.w = tb + 3 > tc ? fv.w : LOG0F;
              lse_add4(aq, xv, fc);
            }
          };
#pragma unroll
          for (int it = 0; it < IT; ++it) {
            const int i = q + it * LPC;
            if (i < n4) split(x[b][it], f4[i], t0 + 4 * i);
          }
          for (int i = q + IT * LPC; i < n4; i += LPC) split(col[i], f4[i], t0 + 4 * i);
          pre = lse_finish<LPC>(a);
          const float mn = fmaxf(a.m, aq.m);                // whole window: both parts
          a.s = a.s * __expf(a.m - mn) + aq.s * __expf(aq.m - mn);
          a.m = mn;
        }
        inc = (W > 0) ? lse_finish<LPC>(a) : LOG0F;
      }
      if (q == 0 && wave_rank) {
        // (joint scores and sort keys: one lane per candidate at the end, not one pass per chain here)
        s_inc[c] = inc;                                    // (eos-run rule armed: the sum up to frame T - R so far)
      } else if (q == 0) {
        const float av = (smallk ? s_av[c] : arow[id]) - row_lse;
        const bool valid = inc > LOG0_CLASS;
        const double ctc = valid ? offr + (double)inc : LOG0D;
        const double J = valid ? lam * ctc + (1.0 - lam) * (double)av + jbase : LOG0D;
        // small K: scores stay in LDS for the ranking below; per-candidate arrays in global memory
        // (read back by ctcbs_peek only) are written from there at the very end, so that no store
        // is pending while columns are still being fetched
        if (smallk) {
          s_J[c] = J; s_inc[c] = inc; s_av[c] = av;
          s_key[c] = joint_key(J, id & 0xFFFF, valid && J == J);
          if (e2) s_pre[c] = pre;
        } else {
          g_inc[c] = inc; g_catt[c] = av; g_ctc[c] = ctc; g_joint[c] = J;
          if (e2) p.cand_pre[(size_t)grp * K + c] = pre;
        }
      }
    }
  }

  TRACE_MARK(4);
  // ---------------- 4. eos-run rule, group list, outputs -----------------------------------
  // (few candidates: the first wave runs this test alone, further down, without a barrier)
  int fire = 0;
  if (e2g) {
    // Frame T is one of the R frames and there X_T is simply the best full prefix score of the
    // extensions, which is already known: most eligible hypotheses fail this test and skip the rest.
    if (smallk) lds_barrier(); else __syncthreads();       // s_inc / g_inc of all candidates written
    float xt = -3.0e38f;
    for (int c = tid; c < K; c += BLOCK) xt = fmaxf(xt, canon0(smallk ? s_inc[c] : g_inc[c]));
    xt = row16_max(xt);
    xt = fmaxf(fmaxf(lane_f(xt, 0), lane_f(xt, 16)), fmaxf(lane_f(xt, 32), lane_f(xt, 48)));
    if ((tid & 63) == 0) s_e2w[tid >> 6] = xt;
    if (tid == 0) s_e2w[BLOCK / 64] = (rs <= T && re >= T) ? canon0(lae(eos_n, eos_b) + (float)BT) : LOG0F;
    lds_barrier();
    float XT = s_e2w[0];
#pragma unroll
    for (int w2 = 1; w2 < BLOCK / 64; ++w2) XT = fmaxf(XT, s_e2w[w2]);
    const float ET = s_e2w[BLOCK / 64];
    const bool maybe = (ET > LOG0_CLASS) && (XT < LOG0_CLASS || ET > XT);
    lds_barrier();                                         // s_e2w is reused below
    if (maybe) {
    // the last R frames, sixteen at a time: every lane carries the
    // running prefix score of its candidates from chunk to chunk through the pre array (each entry
    // is only ever touched by one lane from here on) and keeps, per frame, the best score it has seen
    constexpr int E2C = 16;
    for (int k0 = 0; k0 < R; k0 += E2C) {
      float xmax[E2C];
#pragma unroll
      for (int k = 0; k < E2C; ++k) xmax[k] = -3.0e38f;
      for (int c = tid; c < K; c += BLOCK) {
        const int id = smallk ? s_cid[c] : g_cid[c];
        const float* colf = xu + (size_t)id * p.Tp;
        const float* ff = s_F + ((id == last) ? sm.wp_max : 0);
        float xv[E2C];
#pragma unroll
        for (int k = 0; k < E2C; ++k) xv[k] = colf[min(T - R + 1 + k0 + k, T)];   // all loads in flight
        float acc = smallk ? s_pre[c] : p.cand_pre[(size_t)grp * K + c];
#pragma unroll
        for (int k = 0; k < E2C; ++k) {
          if (k0 + k < R) {
            acc = lae(acc, ff[T - R + 1 + k0 + k - t0] + xv[k]);
            xmax[k] = fmaxf(xmax[k], canon0(acc));
          }
        }
        if (smallk) s_pre[c] = acc; else p.cand_pre[(size_t)grp * K + c] = acc;
      }
#pragma unroll
      for (int k = 0; k < E2C; ++k) {                      // max over the wave, one slot per wave and frame
        if (k0 + k < R) {
          float v = row16_max(xmax[k]);
          v = fmaxf(fmaxf(lane_f(v, 0), lane_f(v, 16)), fmaxf(lane_f(v, 32), lane_f(v, 48)));
          if ((tid & 63) == 0) s_e2w[(tid >> 6) * MAX_EOS_RUN + k0 + k] = v;
        }
      }
    }
    if (tid == 0) s_nvalid = 1;                            // reused as the "all frames passed" flag
    lds_barrier();
    if (tid < R) {
      const float Et = e2_Et;
      float X = s_e2w[tid];
#pragma unroll
      for (int w2 = 1; w2 < BLOCK / 64; ++w2) X = fmaxf(X, s_e2w[w2 * MAX_EOS_RUN + tid]);
      // E_t > X_t with log0 on the left never true, log0 on the right always true
      const bool gt = (Et > LOG0_CLASS) && (X < LOG0_CLASS || Et > X);
      if (!gt) s_nvalid = 0;                               // every writer stores the same value
    }
    lds_barrier();
    fire = s_nvalid;
    }                                                      // maybe
    lds_barrier();                                         // s_nvalid is reset below
  }
  auto group_outputs = [&]() {
    p.stopped[grp] = fire;
    p.ctc_eos[grp] = s_eos[0]; p.joint_eos[grp] = s_eos[1];
    p.win_s[grp] = s; p.win_e[grp] = e;
    p.grp_cells[grp] = (long long)K * (long long)W;
  };
  if (!wave_rank && tid == 0) group_outputs();

  if (smallk) {
    if (wave_rank) {
      // one lane of the first wave per candidate from here on
      constexpr int E2W = 16;                              // eos-run rule: frames per round of loads
      constexpr bool E2_EARLY = (CB * IT <= 6);            // (the forms with more column loads in flight have no registers to spare)
      float xv0[E2_EARLY ? E2W : 1];
      if (E2_EARLY && e2 && tid < 64) {                    // the candidate's posteriors of the last R frames: on
        const float* colf = xu + (size_t)s_cid[tid < K ? tid : 0] * p.Tp;   // their way while the other waves finish
#pragma unroll
        for (int k = 0; k < E2W; ++k) xv0[k] = colf[min(T - R + 1 + k, T)];
      }
      lds_barrier();                                       // prefix scores complete; the other waves are done
      if (tid >= 64) return;
      if (e2) {
        // eos-run rule by one wave.  The sums so far stop at frame T - R; walking through the last R frames
        // completes them and gives, on the way, X_t = best running prefix score of the extensions at frame
        // t, to be held against E_t (in lane t - (T-R+1) since the start of the kernel).
        const bool has = tid < K;
        auto wave_max = [](float v) {
          v = row16_max(v);
          return fmaxf(fmaxf(lane_f(v, 0), lane_f(v, 16)), fmaxf(lane_f(v, 32), lane_f(v, 48)));
        };
        const int e2id = s_cid[has ? tid : 0];
        const float* colf = xu + (size_t)e2id * p.Tp;
        const float* ff = s_e2f + ((e2id == last) ? MAX_EOS_RUN : 0);
        float acc = has ? s_inc[tid] : LOG0F;
        fire = 1;
        for (int k0 = 0; k0 < R; k0 += E2W) {
          float xv[E2W];
          if (E2_EARLY && k0 == 0) {
#pragma unroll
            for (int k = 0; k < E2W; ++k) xv[k] = xv0[E2_EARLY ? k : 0];
          } else {
#pragma unroll
            for (int k = 0; k < E2W; ++k) xv[k] = colf[min(T - R + 1 + k0 + k, T)];   // all loads in flight
          }
#pragma unroll
          for (int k = 0; k < E2W; ++k) {
            if (k0 + k < R) {                              // (uniform)
              acc = lae(acc, ff[k0 + k] + xv[k]);
              const float X = wave_max(has ? canon0(acc) : -3.0e38f);
              const float Et = k0 == 0 ? lane_f(e2_Et, k) : lane_f(e2_Et, k + E2W);
              // E_t > X_t with log0 on the left never true, log0 on the right always true
              if (!((Et > LOG0_CLASS) && (X < LOG0_CLASS || Et > X))) fire = 0;
            }
          }
        }
        if (has) s_inc[tid] = canon0(acc);                 // the whole window's sum
        wave_lds_fence();
      }
      if (tid == 0) group_outputs();
      // rank by (joint desc, token asc) on 64-bit keys
      unsigned long long me = 0ull;
      if (tid < K) {                                       // joint score (Eq. (1)) and sort key of candidate `tid`
        const float inc = s_inc[tid], av = s_av[tid] - row_lse;
        const bool valid = inc > LOG0_CLASS;
        const double ctc = valid ? offr + (double)inc : LOG0D;
        const double J = valid ? lam * ctc + (1.0 - lam) * (double)av + jbase : LOG0D;
        me = joint_key(J, s_cid[tid] & 0xFFFF, valid && J == J);
        s_J[tid] = J; s_av[tid] = av; s_key[tid] = me;
      }
      wave_lds_fence();                                    // keys: written by their lanes, read by all below
      int rank = 0;
      const ulonglong2* k2 = (const ulonglong2*)s_key;
      int c = 0;
      for (; c + 8 <= K; c += 8) {                         // four reads in flight at a time
        const ulonglong2 o0 = k2[c >> 1], o1 = k2[(c >> 1) + 1], o2 = k2[(c >> 1) + 2], o3 = k2[(c >> 1) + 3];
        rank += ((int)(o0.x > me) + (int)(o0.y > me)) + ((int)(o1.x > me) + (int)(o1.y > me)) +
                ((int)(o2.x > me) + (int)(o2.y > me)) + ((int)(o3.x > me) + (int)(o3.y > me));
      }
      for (; c + 1 < K; c += 2) {
        const ulonglong2 o = k2[c >> 1];
        rank += (int)(o.x > me) + (int)(o.y > me);
      }
      if (K & 1) rank += (int)(s_key[K - 1] > me);
      const int nv = __popcll(__ballot(me != 0ull));
      if (!fire && me != 0ull && rank < p.Wb) {
        const size_t o = (size_t)grp * p.Wb + rank;
        p.grp_J[o] = s_J[tid]; p.grp_ci[o] = tid; p.grp_tok[o] = s_cid[tid];
        p.grp_inc[o] = s_inc[tid]; p.grp_att[o] = s_av[tid];
      }
      if (tid == 0) p.grp_n[grp] = fire ? 0 : min(nv, p.Wb);
    } else {
      // rank by (joint desc, token asc), exact comparison: four lanes per candidate
      if (tid == 0) s_nvalid = 0;
      lds_barrier();                                       // scores complete
      if (!fire) {
        const int part = tid & 3;
        for (int e0 = 0; e0 < K; e0 += BLOCK / 4) {
          const int ee = e0 + (tid >> 2);
          const bool mv = ee < K && s_key[ee] != 0ull;
          const double me = mv ? s_J[ee] : LOG0D;
          const int mtok = ee < K ? s_cid[ee] : 0x7fffffff;
          int rank = 0;
          for (int c = part; c < K; c += 4) {
            const double o = s_key[c] != 0ull ? s_J[c] : LOG0D;
            rank += (o > me) || (o == me && s_cid[c] < mtok);
          }
          rank += dpp_i<0xB1, 0xf>(0, rank);               // quad_perm [1,0,3,2]
          rank += dpp_i<0x4E, 0xf>(0, rank);               // quad_perm [2,3,0,1]
          if (part == 0 && mv) {
            if (rank < p.Wb) {
              const size_t o = (size_t)grp * p.Wb + rank;
              p.grp_J[o] = me; p.grp_ci[o] = ee; p.grp_tok[o] = s_cid[ee];
              p.grp_inc[o] = s_inc[ee]; p.grp_att[o] = s_av[ee];
            }
            atomicAdd(&s_nvalid, 1);
          }
        }
      }
      lds_barrier();
      if (tid == 0) p.grp_n[grp] = fire ? 0 : min(s_nvalid, p.Wb);
    }
    if (p.keep_cand) {
      for (int c = tid; c < K; c += BLOCK) {
        const float inc = s_inc[c];
        g_cid[c] = s_cid[c]; g_inc[c] = inc; g_catt[c] = s_av[c];
        g_ctc[c] = inc > LOG0_CLASS ? offr + (double)inc : LOG0D;
        g_joint[c] = s_J[c];
      }
    }
  }
  TRACE_MARK(5);
  TRACE_FLUSH(p, grp);
}
// Group list for large candidate sets (K > block size): Wb rounds of a block-wide argmax
// over the joint scores in global memory.  One work-group per (utterance, beam slot).
template <int BLOCK>
__global__ __launch_bounds__(BLOCK) void k_group_top(Params p, int cur) {
  __shared__ double s_v[BLOCK / 64];
  __shared__ int s_i[BLOCK / 64], s_t[BLOCK / 64];
  __shared__ int s_pick[MAX_BEAM];
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int grp = blockIdx.x, u = grp / p.Wb, K = p.K;
  if (p.finished[u] || !p.rec[cur][grp].live) return;      // k_score already wrote grp_n = 0
  if (p.stopped[grp]) { if (tid == 0) p.grp_n[grp] = 0; return; }
  const double* J = p.cand_joint + (size_t)grp * K;
  const int32_t* ids = p.cand_id + (size_t)grp * K;       // equal scores: smaller token id first
  int n = 0;
  for (int r = 0; r < p.Wb; ++r) {
    double bv = LOG0D; int bi = 0x7fffffff, bt = 0x7fffffff;
    for (int c = tid; c < K; c += BLOCK) {
      double v = J[c];
      if (!(v > (double)LOG0_CLASS)) continue;
      bool taken = false;
      for (int k = 0; k < r; ++k) taken |= (s_pick[k] == c);
      if (taken) continue;
      const int tk = ids[c];
      if (v > bv || (v == bv && tk < bt)) { bv = v; bi = c; bt = tk; }
    }
    for (int o = 32; o > 0; o >>= 1) {
      double ov = __shfl_xor(bv, o); int oi = __shfl_xor(bi, o); int ot = __shfl_xor(bt, o);
      if (ov > bv || (ov == bv && ot < bt)) { bv = ov; bi = oi; bt = ot; }
    }
    if (lane == 0) { s_v[w] = bv; s_i[w] = bi; s_t[w] = bt; }
    __syncthreads();
    if (tid == 0) {
      for (int k = 1; k < BLOCK / 64; ++k)
        if (s_v[k] > bv || (s_v[k] == bv && s_t[k] < bt)) { bv = s_v[k]; bi = s_i[k]; bt = s_t[k]; }
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

// The same list for candidate sets of up to BLOCK * EPT ids, from registers: every thread loads
// its share of the joint scores once, as 64-bit keys (order-preserving image of the score whose
// 13 lowest mantissa bits carry 8191 - candidate index: larger score first, then the smaller
// index = the smaller token id; scores equal to within 2^-39 relative count as equal); each of
// the Wb rounds is then a block-wide maximum of keys and the owner retires the winner.
template <int BLOCK, int EPT>
__global__ __launch_bounds__(BLOCK) void k_group_top_regs(Params p, int cur) {
  constexpr int NW = BLOCK / 64;
  __shared__ unsigned long long s_k[2][NW];
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int grp = blockIdx.x, u = grp / p.Wb, K = p.K;
  if (p.finished[u] || !p.rec[cur][grp].live) return;      // the score kernel already wrote grp_n = 0
  if (p.stopped[grp]) { if (tid == 0) p.grp_n[grp] = 0; return; }
  const double* J = p.cand_joint + (size_t)grp * K;
  unsigned long long key[EPT];
#pragma unroll
  for (int k = 0; k < EPT; ++k) {
    const int c = tid + k * BLOCK;
    const double v = c < K ? J[c] : LOG0D;
    unsigned long long kk = 0ull;                           // not a competitor
    if (v > (double)LOG0_CLASS) {                           // (false for NaN)
      const unsigned long long b = (unsigned long long)__double_as_longlong(v);
      kk = (((b >> 63) ? ~b : (b | 0x8000000000000000ull)) & ~0x1FFFull) | (unsigned long long)(0x1FFF - c);
    }
    key[k] = kk;
  }
  int n = 0;
  for (int r = 0; r < p.Wb; ++r) {
    unsigned long long best = key[0];
#pragma unroll
    for (int k = 1; k < EPT; ++k) best = key[k] > best ? key[k] : best;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      const unsigned long long ob = __shfl_xor(best, o);
      best = ob > best ? ob : best;
    }
    if (lane == 0) s_k[r & 1][w] = best;
    lds_barrier();                                          // (two buffers: one barrier per round is enough)
    best = s_k[r & 1][0];
#pragma unroll
    for (int i = 1; i < NW; ++i) best = s_k[r & 1][i] > best ? s_k[r & 1][i] : best;
    if (best == 0ull) break;                                // uniform: no finite candidate left
    const int c = 0x1FFF - (int)(best & 0x1FFFull);
#pragma unroll
    for (int k = 0; k < EPT; ++k)
      if (key[k] == best) key[k] = 0ull;                    // only its owner holds this key
    if (tid == 0) {
      const size_t o = (size_t)grp * p.Wb + r, g = (size_t)grp * K + c;
      p.grp_J[o] = J[c]; p.grp_ci[o] = c; p.grp_tok[o] = p.cand_id[g];
      p.grp_inc[o] = p.cand_inc[g]; p.grp_att[o] = p.cand_att[g];
    }
    ++n;
  }
  if (tid == 0) p.grp_n[grp] = n;
}
