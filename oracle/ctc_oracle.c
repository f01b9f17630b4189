/*
 * CPU oracle for the batched joint CTC/attention beam-search step.
 *
 * TEST INFRASTRUCTURE ONLY.  Plain, slow, fp64, one utterance at a time; it
 * shares no code with the GPU library and must never be called from the
 * product path.  Only tests, the smoke check and the benchmark's CPU-baseline
 * leg use it.
 *
 * What each part follows (paper = arXiv 2101.05600):
 *   - CTC alignment rules and the prefix probability: Sec. 2.1, the four rules
 *     for z_t and Eq. (3) ("Eq. ctc").  The paper prints only phi_t and the sum;
 *     the two forward variables used here (paths ending in the last label /
 *     ending in blank) are derived from those rules.
 *   - Joint score: Eq. (1); attention score accumulation: Eq. (2).
 *   - Search loop, eos column split-off, TopB/GatherB, the "p > best_score"
 *     test, final argmax: Algorithm 2 (Algorithm 1 is its one-utterance form).
 *   - Baseline end detection: Eq. (4), M = 3, D_end = e^-10 (log domain: -10).
 *   - Time indices tau / tau~ of the last label: the two argmax equations of
 *     Sec. 3.2.2; tau-count end detection: Algorithm 3, C = 2.  A hypothesis keeps the tau
 *     found when each of its labels was appended (the per-label time stamps of Fig. 2(a));
 *     the tau recorded with an ended hypothesis g.<eos> is tau(g), that of g's last label.
 *   - Time-restricted prefix score and the window [s, e]: Eq. (5) and the two
 *     equations for s and e after it.
 *   Parts that are not in the paper but in this build's brief (top-K attention
 *   candidates, length bonus, the eos-run stop rule "E2") are marked [brief].
 *
 * Pins: brute-force alignment enumeration, prefix-sum invariant, textbook CTC
 * forward lattice / library CTC loss, closed forms (tests/test_oracle_pins.py).
 * The eos-run rule E2, the forced ending at the length cap and the length
 * bonus have no outside definition: for them parity is pinned only by
 * constructed cases ("parity unpinned" beyond those).
 *
 * Conventions: frames t = 1..T, x[(t-1)*V + k] = log p^c(z_t = k); a hypothesis
 * g is its label list without the start symbol; step l extends length l-1
 * hypotheses.  log0 is -inf inside and reported as ORC_LOG0 at the interface.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORC_LOG0 (-1.0e30)
#define ORC_END_BASELINE 1
#define ORC_END_TAU_COUNT 2
#define ORC_END_EOS_RUN 4

typedef struct {
  int32_t vocab, beam, blank_id, eos_id;
  int32_t cand_k;          /* 0 or >= V-2: every id except blank and eos [brief]          */
  int32_t win_m1, win_m2;  /* M1, M2 of the window equations; < 0: unrestricted           */
  int32_t max_len_abs;     /* 0: none                                                       */
  int32_t end_flags, end_m, end_c, eos_run;
  int32_t win_union;       /* 1: one window for the whole batch (last two equations of Sec. 3.2.3) */
  int32_t pad_;
  double ctc_weight, length_bonus, max_len_ratio, end_d;
} orc_cfg;

typedef struct {
  int32_t live;
  int32_t len;             /* number of labels                                              */
  int32_t* labels;         /* [cap]                                                         */
  int32_t* taus;           /* [cap] taus[i] = tau found when labels[i] was appended         */
  double *gn, *gb;         /* [T+1] forward variables, -inf outside [rs, re]                */
  int32_t rs, re;          /* stored range                                                  */
  int32_t tau, tau_end;
  double att, ctc, joint;  /* cumulative attention log-prob, log psi(g), joint score        */
} orc_hyp;

typedef struct {
  int32_t parent, token;
  double joint, ctc, att;  /* of the extended hypothesis                                    */
} orc_cand;

typedef struct {
  int32_t len, tau, slot, step;
  double score;
  int32_t* labels;         /* without eos                                                   */
  int32_t* taus;           /* time stamp of each label                                      */
} orc_ended;

typedef struct orc_utt {
  orc_cfg cfg;
  int32_t T, V, lmax, step, finished, cap;
  const float* x;          /* borrowed, [T][V]                                              */
  orc_hyp *cur, *nxt;      /* [beam]                                                        */
  /* results of the last orc_score */
  int32_t n_cand_per, *win_s, *win_e, *cand_id;   /* [beam], [beam], [beam][K]              */
  double *cand_ctc, *cand_att, *cand_joint;       /* [beam][K]                              */
  double *ctc_eos, *joint_eos;                    /* [beam]                                 */
  int32_t *e2_eligible, *e2_fire;                 /* [beam]                                 */
  double *e2_margin;                              /* [beam] min_t (E_t - X_t)               */
  orc_cand* sorted; int32_t n_sorted;             /* finite candidates, best first          */
  double best;
  /* ended hypotheses */
  orc_ended* ended; int32_t n_ended, cap_ended;
  double cells;            /* sum over live groups of K * (e - s + 1)                       */
  /* children of the last commit */
  double *child_max_n, *child_max_b;              /* [beam] max of gn / gb over the tau range */
  int32_t *child_lo;                              /* [beam] lower end of the tau range      */
  double e1_margin;        /* distance of the deciding comparison from its threshold        */
  int32_t union_tau_min, union_e_max;   /* batch-wide values, set by the caller before each score   */
} orc_utt;

static double lae(double a, double b) {
  if (a == -INFINITY) return b;
  if (b == -INFINITY) return a;
  double m = a > b ? a : b;
  return m + log1p(exp(-fabs(a - b)));
}

static double Xv(const orc_utt* u, int t, int k) { return (double)u->x[(size_t)(t - 1) * u->V + k]; }

static double GN(const orc_hyp* h, int t) { return (t < h->rs || t > h->re) ? -INFINITY : h->gn[t]; }
static double GB(const orc_hyp* h, int t) { return (t < h->rs || t > h->re) ? -INFINITY : h->gb[t]; }

/* f_t of Eq. (3)/(5): forward mass of g at t-1 that may be followed by label c at t. */
static double f_term(const orc_hyp* g, int t, int c) {
  int last = g->len > 0 ? g->labels[g->len - 1] : -1;
  if (c == last) return GB(g, t - 1);           /* a repeated label needs a blank in between */
  return lae(GN(g, t - 1), GB(g, t - 1));
}

static void hyp_alloc(orc_hyp* h, int T, int cap) {
  memset(h, 0, sizeof *h);
  h->labels = (int32_t*)calloc((size_t)cap + 1, sizeof(int32_t));
  h->taus = (int32_t*)calloc((size_t)cap + 1, sizeof(int32_t));
  h->gn = (double*)malloc(sizeof(double) * (size_t)(T + 1));
  h->gb = (double*)malloc(sizeof(double) * (size_t)(T + 1));
}
static void hyp_free(orc_hyp* h) { free(h->labels); free(h->taus); free(h->gn); free(h->gb); }

int orc_lmax(const orc_cfg* c, int T) {
  int l = T;                                    /* Algorithm 2 never runs past |h| steps     */
  if (c->max_len_ratio > 0.0) { int r = (int)floor(c->max_len_ratio * T); if (r < l) l = r; }
  if (c->max_len_abs > 0 && c->max_len_abs < l) l = c->max_len_abs;
  if (l < 1) l = 1;
  return l;
}

int orc_n_cand(const orc_cfg* c) {
  int all = c->vocab - 2;
  return (c->cand_k <= 0 || c->cand_k >= all) ? all : c->cand_k;
}

orc_utt* orc_create(const float* x, int T, int V, const orc_cfg* cfg) {
  if (!x || !cfg || T < 1 || V < 3 || cfg->vocab != V || cfg->beam < 1) return NULL;
  if (cfg->blank_id < 0 || cfg->blank_id >= V || cfg->eos_id < 0 || cfg->eos_id >= V ||
      cfg->blank_id == cfg->eos_id) return NULL;
  orc_utt* u = (orc_utt*)calloc(1, sizeof *u);
  u->cfg = *cfg; u->T = T; u->V = V; u->x = x;
  u->lmax = orc_lmax(cfg, T);
  u->cap = u->lmax + 1;
  int B = cfg->beam, K = orc_n_cand(cfg);
  u->n_cand_per = K;
  u->cur = (orc_hyp*)calloc((size_t)B, sizeof(orc_hyp));
  u->nxt = (orc_hyp*)calloc((size_t)B, sizeof(orc_hyp));
  for (int j = 0; j < B; ++j) { hyp_alloc(&u->cur[j], T, u->cap); hyp_alloc(&u->nxt[j], T, u->cap); }
  u->win_s = (int32_t*)calloc((size_t)B, sizeof(int32_t));
  u->win_e = (int32_t*)calloc((size_t)B, sizeof(int32_t));
  u->cand_id = (int32_t*)calloc((size_t)B * K, sizeof(int32_t));
  u->cand_ctc = (double*)calloc((size_t)B * K, sizeof(double));
  u->cand_att = (double*)calloc((size_t)B * K, sizeof(double));
  u->cand_joint = (double*)calloc((size_t)B * K, sizeof(double));
  u->ctc_eos = (double*)calloc((size_t)B, sizeof(double));
  u->joint_eos = (double*)calloc((size_t)B, sizeof(double));
  u->e2_eligible = (int32_t*)calloc((size_t)B, sizeof(int32_t));
  u->e2_fire = (int32_t*)calloc((size_t)B, sizeof(int32_t));
  u->e2_margin = (double*)calloc((size_t)B, sizeof(double));
  u->sorted = (orc_cand*)calloc((size_t)B * K, sizeof(orc_cand));
  u->child_max_n = (double*)calloc((size_t)B, sizeof(double));
  u->child_max_b = (double*)calloc((size_t)B, sizeof(double));
  u->child_lo = (int32_t*)calloc((size_t)B, sizeof(int32_t));
  /* empty prefix: z_0 = blank (first alignment rule), so only the blank variable is alive */
  orc_hyp* h = &u->cur[0];
  h->live = 1; h->len = 0; h->rs = 0; h->re = T; h->tau = 0; h->tau_end = 0;
  h->att = 0.0; h->ctc = 0.0; h->joint = 0.0;
  h->gb[0] = 0.0; h->gn[0] = -INFINITY;
  for (int t = 1; t <= T; ++t) { h->gb[t] = h->gb[t - 1] + Xv(u, t, cfg->blank_id); h->gn[t] = -INFINITY; }
  u->step = 0; u->finished = 0;
  return u;
}

void orc_destroy(orc_utt* u) {
  if (!u) return;
  for (int j = 0; j < u->cfg.beam; ++j) { hyp_free(&u->cur[j]); hyp_free(&u->nxt[j]); }
  free(u->cur); free(u->nxt); free(u->win_s); free(u->win_e); free(u->cand_id);
  free(u->cand_ctc); free(u->cand_att); free(u->cand_joint); free(u->ctc_eos); free(u->joint_eos);
  free(u->e2_eligible); free(u->e2_fire); free(u->e2_margin); free(u->sorted);
  free(u->child_max_n); free(u->child_max_b); free(u->child_lo);
  for (int i = 0; i < u->n_ended; ++i) { free(u->ended[i].labels); free(u->ended[i].taus); }
  free(u->ended);
  free(u);
}

/* [brief] the K ids with the largest attention log-prob, blank and eos excluded,
 * equal values resolved towards the smaller id; returned in ascending id order. */
static void select_candidates(const orc_utt* u, const float* att_row, int K, int32_t* out) {
  int V = u->V, n = 0;
  int32_t* best = (int32_t*)malloc(sizeof(int32_t) * (size_t)K);   /* sorted: best first */
  for (int k = 0; k < V; ++k) {
    if (k == u->cfg.blank_id || k == u->cfg.eos_id) continue;
    float a = att_row[k];
    if (n == K && !(a > att_row[best[K - 1]])) continue;            /* later id must be strictly better */
    int pos = n < K ? n : K - 1;
    while (pos > 0 && a > att_row[best[pos - 1]]) { best[pos] = best[pos - 1]; --pos; }
    best[pos] = k;
    if (n < K) ++n;
  }
  /* ascending id */
  for (int i = 1; i < n; ++i) {
    int32_t v = best[i]; int j = i;
    while (j > 0 && best[j - 1] > v) { best[j] = best[j - 1]; --j; }
    best[j] = v;
  }
  memcpy(out, best, sizeof(int32_t) * (size_t)n);
  free(best);
}

static int cand_cmp(const void* pa, const void* pb) {
  const orc_cand* a = (const orc_cand*)pa; const orc_cand* b = (const orc_cand*)pb;
  if (a->joint > b->joint) return -1;
  if (a->joint < b->joint) return 1;
  if (a->parent != b->parent) return a->parent < b->parent ? -1 : 1;
  if (a->token != b->token) return a->token < b->token ? -1 : 1;
  return 0;
}

/*
 * Score phase of step l = step+1: candidates, window, prefix scores, eos scores,
 * joint scores, the eos-run test, and the sorted list of finite candidates.
 * att: [beam][V] attention log-probs of this step (rows of dead slots unread).
 */
int orc_score(orc_utt* u, const float* att) {
  if (!u || !att || u->finished) return -1;
  const orc_cfg* c = &u->cfg;
  int B = c->beam, K = u->n_cand_per, V = u->V, T = u->T, l = u->step + 1;
  double lam = c->ctc_weight;
  u->n_sorted = 0; u->best = -INFINITY;
  for (int j = 0; j < B; ++j) {
    orc_hyp* g = &u->cur[j];
    u->e2_eligible[j] = 0; u->e2_fire[j] = 0; u->e2_margin[j] = INFINITY;
    u->win_s[j] = 0; u->win_e[j] = -1;
    if (!g->live) continue;
    const float* a = att + (size_t)j * V;
    int32_t* ids = u->cand_id + (size_t)j * K;
    select_candidates(u, a, K, ids);
    /* window: Sec. 3.2.3, the equations for s and e; unrestricted = Eq. (3) limits */
    int s, e;
    if (c->win_union) {
      /* s^l = min_ij s_ij, e^l = max_ij e_ij over the whole batch; an utterance has no frames beyond T */
      if (c->win_m1 >= 0) { s = u->union_tau_min - c->win_m1; if (s < l) s = l; if (s < 1) s = 1; } else s = l;
      if (c->win_m2 >= 0) { e = u->union_e_max; if (e > T) e = T; } else e = T;
    } else {
      if (c->win_m1 >= 0) { s = g->tau - c->win_m1; if (s < l) s = l; if (s < 1) s = 1; } else s = l;
      if (c->win_m2 >= 0) { e = g->tau_end + c->win_m2; if (e > T) e = T; } else e = T;
    }
    u->win_s[j] = s; u->win_e[j] = e;
    if (e >= s) u->cells += (double)K * (double)(e - s + 1);
    for (int i = 0; i < K; ++i) {
      int k = ids[i];
      double psi = -INFINITY;
      for (int t = s; t <= e; ++t) psi = lae(psi, f_term(g, t, k) + Xv(u, t, k));   /* Eq. (3)/(5) */
      u->cand_ctc[(size_t)j * K + i] = psi;                                          /* absolute log psi(g.c) */
      u->cand_att[(size_t)j * K + i] = g->att + (double)a[k];                       /* Eq. (2) */
      u->cand_joint[(size_t)j * K + i] =
          lam * psi + (1.0 - lam) * (g->att + (double)a[k]) + c->length_bonus * l; /* Eq. (1) */
    }
    /* eos: the whole output is g  <=>  all T frames consumed by g */
    u->ctc_eos[j] = (g->rs <= T && g->re >= T) ? lae(g->gn[T], g->gb[T]) : -INFINITY;
    u->joint_eos[j] = (u->ctc_eos[j] == -INFINITY) ? -INFINITY
        : lam * u->ctc_eos[j] + (1.0 - lam) * (g->att + (double)a[c->eos_id]) + c->length_bonus * l;
    /* [brief] E2: phi_t(g) beats every extension's running prefix score on each of the last R frames */
    int R = c->eos_run;
    if ((c->end_flags & ORC_END_EOS_RUN) && R > 0 && T >= R && e == T && g->re == T) {
      int t0 = T - R + 1;
      int lo = s > g->rs ? s : g->rs;
      if (lo <= t0) {
        u->e2_eligible[j] = 1;
        double margin = INFINITY;
        for (int t = t0; t <= T; ++t) {
          double Xt = -INFINITY;
          for (int i = 0; i < K; ++i) {
            int k = ids[i];
            double run = -INFINITY;
            for (int q = s; q <= t; ++q) run = lae(run, f_term(g, q, k) + Xv(u, q, k));
            if (run > Xt) Xt = run;
          }
          double Et = lae(GN(g, t), GB(g, t));
          double d = (Et == -INFINITY) ? -INFINITY : (Xt == -INFINITY ? INFINITY : Et - Xt);
          if (d < margin) margin = d;
        }
        u->e2_margin[j] = margin;
        u->e2_fire[j] = margin > 0.0;
      }
    }
  }
  return 0;
}

/* Sorted list of finite candidates of the slots not stopped by E2, and best. */
static void build_sorted(orc_utt* u, const int32_t* stopped) {
  int B = u->cfg.beam, K = u->n_cand_per;
  u->n_sorted = 0; u->best = -INFINITY;
  for (int j = 0; j < B; ++j) {
    if (!u->cur[j].live || stopped[j]) continue;
    for (int i = 0; i < K; ++i) {
      double J = u->cand_joint[(size_t)j * K + i];
      if (J == -INFINITY || isnan(J)) continue;
      orc_cand* o = &u->sorted[u->n_sorted++];
      o->parent = j; o->token = u->cand_id[(size_t)j * K + i];
      o->joint = J; o->ctc = u->cand_ctc[(size_t)j * K + i]; o->att = u->cand_att[(size_t)j * K + i];
      if (J > u->best) u->best = J;
    }
  }
  qsort(u->sorted, (size_t)u->n_sorted, sizeof(orc_cand), cand_cmp);
}

/* Rank the candidates given the stop flags (NULL: the oracle's own E2 outcome). */
int orc_rank(orc_utt* u, const int32_t* stopped) {
  if (!u) return -1;
  build_sorted(u, stopped ? stopped : u->e2_fire);
  return u->n_sorted;
}

static void add_ended(orc_utt* u, const orc_hyp* g, int slot, double score, int l) {
  if (u->n_ended == u->cap_ended) {
    u->cap_ended = u->cap_ended ? 2 * u->cap_ended : 16;
    u->ended = (orc_ended*)realloc(u->ended, sizeof(orc_ended) * (size_t)u->cap_ended);
  }
  orc_ended* e = &u->ended[u->n_ended++];
  e->len = l; e->tau = g->tau; e->slot = slot; e->step = l; e->score = score;
  e->labels = (int32_t*)malloc(sizeof(int32_t) * (size_t)(g->len + 1));
  memcpy(e->labels, g->labels, sizeof(int32_t) * (size_t)g->len);
  e->taus = (int32_t*)malloc(sizeof(int32_t) * (size_t)(g->len + 1));
  memcpy(e->taus, g->taus, sizeof(int32_t) * (size_t)g->len);
}

/* Algorithm 3 on a plain list of ended hypotheses (length, tau, score): Eq. (4) first,
 * then the count of ended hypotheses whose tau sits on T.  *margin receives the distance of
 * the closest Eq. (4) comparison from its threshold. */
int orc_end_detect(const orc_cfg* c, int T, int l, int n, const int32_t* len, const int32_t* tau,
                   const double* score, double* margin) {
  if (margin) *margin = INFINITY;
  if (n == 0) return 0;
  double best = -INFINITY;
  for (int i = 0; i < n; ++i) if (score[i] > best) best = score[i];
  if (c->end_flags & ORC_END_BASELINE) {
    int count = 0;
    for (int m = 0; m < c->end_m; ++m) {
      double bl = -INFINITY; int have = 0;
      for (int i = 0; i < n; ++i)
        if (len[i] == l - m) { have = 1; if (score[i] > bl) bl = score[i]; }
      if (!have) continue;                       /* a length with no ended hypothesis does not count */
      double d = fabs(bl - best - c->end_d);
      if (margin && d < *margin) *margin = d;
      if (bl - best < c->end_d) ++count;
    }
    if (count == c->end_m) return 1;
  }
  if (c->end_flags & ORC_END_TAU_COUNT) {
    int cnt = 0;
    for (int i = 0; i < n; ++i) if (tau[i] == T) ++cnt;
    if (cnt > c->end_c) return 1;
  }
  return 0;
}

static int end_detect(orc_utt* u, int l) {
  int n = u->n_ended;
  int32_t* len = (int32_t*)malloc(sizeof(int32_t) * (size_t)(n + 1));
  int32_t* tau = (int32_t*)malloc(sizeof(int32_t) * (size_t)(n + 1));
  double* sc = (double*)malloc(sizeof(double) * (size_t)(n + 1));
  for (int i = 0; i < n; ++i) { len[i] = u->ended[i].len; tau[i] = u->ended[i].tau; sc[i] = u->ended[i].score; }
  int r = orc_end_detect(&u->cfg, u->T, l, n, len, tau, sc, &u->e1_margin);
  free(len); free(tau); free(sc);
  return r;
}

/*
 * Commit phase.  sel_parent/sel_token: the n_sel new hypotheses in beam order;
 * eos_add[j], stopped[j]: decisions per old slot.  Passing NULL pointers makes
 * the oracle take its own decisions (free-running mode).  Returns 1 if the
 * utterance finished at this step, 0 if not, < 0 on error.
 */
int orc_commit(orc_utt* u, int n_sel, const int32_t* sel_parent, const int32_t* sel_token,
               const int32_t* eos_add, const int32_t* stopped) {
  if (!u || u->finished) return -1;
  const orc_cfg* c = &u->cfg;
  int B = c->beam, K = u->n_cand_per, T = u->T, l = u->step + 1;
  const int32_t* stp = stopped ? stopped : u->e2_fire;
  build_sorted(u, stp);
  int own_sel = (sel_parent == NULL);
  if (own_sel) n_sel = u->n_sorted < B ? u->n_sorted : B;
  if (n_sel > B) return -2;
  int forced = (l == u->lmax);
  /* ended hypotheses: Algorithm 2's "p > best_score" test, in slot order */
  for (int j = 0; j < B; ++j) {
    orc_hyp* g = &u->cur[j];
    if (!g->live) continue;
    int add;
    if (eos_add) add = eos_add[j];
    else add = forced || stp[j] || (u->joint_eos[j] > u->best);
    if (add) add_ended(u, g, j, u->joint_eos[j], l);
  }
  /* new beam with its forward variables: state recursion over the parent's window */
  for (int n = 0; n < B; ++n) u->nxt[n].live = 0;
  for (int n = 0; n < n_sel; ++n) {
    int p = own_sel ? u->sorted[n].parent : sel_parent[n];
    int k = own_sel ? u->sorted[n].token : sel_token[n];
    if (p < 0 || p >= B || !u->cur[p].live) return -3;
    orc_hyp* g = &u->cur[p]; orc_hyp* h = &u->nxt[n];
    int idx = -1;
    for (int i = 0; i < K; ++i) if (u->cand_id[(size_t)p * K + i] == k) { idx = i; break; }
    if (idx < 0) return -4;                       /* not one of the parent's candidates */
    int s = u->win_s[p], e = u->win_e[p];
    h->live = 1; h->len = g->len + 1;
    memcpy(h->labels, g->labels, sizeof(int32_t) * (size_t)g->len);
    h->labels[g->len] = k;
    h->att = u->cand_att[(size_t)p * K + idx];
    h->ctc = u->cand_ctc[(size_t)p * K + idx];
    h->joint = u->cand_joint[(size_t)p * K + idx];
    h->rs = s; h->re = e;
    for (int t = 0; t <= T; ++t) { h->gn[t] = -INFINITY; h->gb[t] = -INFINITY; }
    double np = -INFINITY, bp = -INFINITY;
    for (int t = s; t <= e; ++t) {
      double ft = f_term(g, t, k);
      double nn = lae(np, ft) + Xv(u, t, k);
      double bb = lae(np, bp) + Xv(u, t, c->blank_id);
      h->gn[t] = nn; h->gb[t] = bb; np = nn; bp = bb;
    }
    /* tau, tau~: first argmax of the two forward variables from the parent's tau on */
    int lo = s > g->tau ? s : g->tau;
    h->tau = g->tau; h->tau_end = g->tau_end;
    double mn = -INFINITY, mb = -INFINITY;
    for (int t = lo; t <= e; ++t) {
      if (h->gn[t] > mn) { mn = h->gn[t]; h->tau = t; }
      if (h->gb[t] > mb) { mb = h->gb[t]; h->tau_end = t; }
    }
    memcpy(h->taus, g->taus, sizeof(int32_t) * (size_t)g->len);
    h->taus[g->len] = h->tau;                    /* time stamp of the label just appended */
    u->child_max_n[n] = mn; u->child_max_b[n] = mb; u->child_lo[n] = lo;
  }
  orc_hyp* tmp = u->cur; u->cur = u->nxt; u->nxt = tmp;
  u->step = l;
  int fin = forced || n_sel == 0 || end_detect(u, l);
  u->finished = fin;
  return fin;
}

/* Batch-union window: this utterance's share (min tau, max of min(tau~ + M2, T)) over its live
 * hypotheses; returns 0 if it has none (finished or empty beam). */
int orc_union_contrib(const orc_utt* u, int32_t* tau_min, int32_t* e_max) {
  int any = 0;
  if (u->finished) return 0;
  for (int j = 0; j < u->cfg.beam; ++j) {
    const orc_hyp* g = &u->cur[j];
    if (!g->live) continue;
    int e = g->tau_end + u->cfg.win_m2; if (e > u->T) e = u->T;
    if (!any || g->tau < *tau_min) *tau_min = g->tau;
    if (!any || e > *e_max) *e_max = e;
    any = 1;
  }
  return any;
}
void orc_set_union(orc_utt* u, int32_t tau_min, int32_t e_max) { u->union_tau_min = tau_min; u->union_e_max = e_max; }

/* Adopt externally validated values for the new beam's time indices / the finished flag. */
void orc_override(orc_utt* u, const int32_t* tau, const int32_t* tau_end, int finished) {
  for (int j = 0; j < u->cfg.beam; ++j) {
    if (!u->cur[j].live) continue;
    if (tau && tau[j] >= 0) { u->cur[j].tau = tau[j]; if (u->cur[j].len > 0) u->cur[j].taus[u->cur[j].len - 1] = tau[j]; }
    if (tau_end && tau_end[j] >= 0) u->cur[j].tau_end = tau_end[j];
  }
  if (finished >= 0) u->finished = finished;
}

/* One free-running step: score, own decisions, commit. */
int orc_step_auto(orc_utt* u, const float* att) {
  int r = orc_score(u, att);
  if (r < 0) return r;
  return orc_commit(u, 0, NULL, NULL, NULL, NULL);
}

/* Final result: argmax over the ended set, earliest added wins ties (Algorithm 2, last line).
 * If nothing ended, the best live hypothesis is returned and *fallback = 1. */
int orc_result_frames(const orc_utt* u, int32_t* labels, int32_t* frames, int cap, double* score, int32_t* fallback);
int orc_result(const orc_utt* u, int32_t* labels, int cap, double* score, int32_t* fallback) {
  return orc_result_frames(u, labels, NULL, cap, score, fallback);
}
/* The same with the time stamp of every label (frames may be NULL). */
int orc_result_frames(const orc_utt* u, int32_t* labels, int32_t* frames, int cap, double* score, int32_t* fallback) {
  int best = -1;
  for (int i = 0; i < u->n_ended; ++i)
    if (best < 0 || u->ended[i].score > u->ended[best].score) best = i;
  if (best >= 0) {
    int n = u->ended[best].len - 1;
    if (n > cap) return -1;
    memcpy(labels, u->ended[best].labels, sizeof(int32_t) * (size_t)n);
    if (frames) memcpy(frames, u->ended[best].taus, sizeof(int32_t) * (size_t)n);
    *score = u->ended[best].score; if (fallback) *fallback = 0;
    return n;
  }
  if (fallback) *fallback = 1;
  for (int j = 0; j < u->cfg.beam; ++j)
    if (u->cur[j].live) {
      if (u->cur[j].len > cap) return -1;
      memcpy(labels, u->cur[j].labels, sizeof(int32_t) * (size_t)u->cur[j].len);
      if (frames) memcpy(frames, u->cur[j].taus, sizeof(int32_t) * (size_t)u->cur[j].len);
      *score = u->cur[j].joint;
      return u->cur[j].len;
    }
  *score = -INFINITY;
  return 0;
}

/* ---- accessors for the Python side ---------------------------------------------------- */
int orc_step_index(const orc_utt* u) { return u->step; }
int orc_finished(const orc_utt* u) { return u->finished; }
int orc_T(const orc_utt* u) { return u->T; }
int orc_lmax_of(const orc_utt* u) { return u->lmax; }
int orc_k(const orc_utt* u) { return u->n_cand_per; }
double orc_cells(const orc_utt* u) { return u->cells; }
double orc_best(const orc_utt* u) { return u->best; }
double orc_e1_margin(const orc_utt* u) { return u->e1_margin; }
int orc_n_sorted(const orc_utt* u) { return u->n_sorted; }
const orc_cand* orc_sorted(const orc_utt* u) { return u->sorted; }
const int32_t* orc_win_s(const orc_utt* u) { return u->win_s; }
const int32_t* orc_win_e(const orc_utt* u) { return u->win_e; }
const int32_t* orc_cand_id(const orc_utt* u) { return u->cand_id; }
const double* orc_cand_ctc(const orc_utt* u) { return u->cand_ctc; }
const double* orc_cand_att(const orc_utt* u) { return u->cand_att; }
const double* orc_cand_joint(const orc_utt* u) { return u->cand_joint; }
const double* orc_ctc_eos(const orc_utt* u) { return u->ctc_eos; }
const double* orc_joint_eos(const orc_utt* u) { return u->joint_eos; }
const int32_t* orc_e2_eligible(const orc_utt* u) { return u->e2_eligible; }
const int32_t* orc_e2_fire(const orc_utt* u) { return u->e2_fire; }
const double* orc_e2_margin(const orc_utt* u) { return u->e2_margin; }
const double* orc_child_max_n(const orc_utt* u) { return u->child_max_n; }
const double* orc_child_max_b(const orc_utt* u) { return u->child_max_b; }
const int32_t* orc_child_lo(const orc_utt* u) { return u->child_lo; }
int orc_n_ended(const orc_utt* u) { return u->n_ended; }
void orc_ended_get(const orc_utt* u, int i, int32_t* len, int32_t* tau, int32_t* slot, double* score) {
  *len = u->ended[i].len; *tau = u->ended[i].tau; *slot = u->ended[i].slot; *score = u->ended[i].score;
}
const int32_t* orc_ended_labels(const orc_utt* u, int i) { return u->ended[i].labels; }
const int32_t* orc_ended_taus(const orc_utt* u, int i) { return u->ended[i].taus; }
/* hypothesis j of the current beam */
void orc_hyp_get(const orc_utt* u, int j, int32_t* live, int32_t* len, int32_t* tau, int32_t* tau_end,
                 int32_t* rs, int32_t* re, double* att, double* ctc, double* joint) {
  const orc_hyp* h = &u->cur[j];
  *live = h->live; *len = h->len; *tau = h->tau; *tau_end = h->tau_end; *rs = h->rs; *re = h->re;
  *att = h->att; *ctc = h->ctc; *joint = h->joint;
}
const int32_t* orc_hyp_labels(const orc_utt* u, int j) { return u->cur[j].labels; }
const int32_t* orc_hyp_taus(const orc_utt* u, int j) { return u->cur[j].taus; }
const double* orc_hyp_gn(const orc_utt* u, int j) { return u->cur[j].gn; }
const double* orc_hyp_gb(const orc_utt* u, int j) { return u->cur[j].gb; }

/*
 * Stand-alone definitions used by the pins: log psi(g) (Eq. (3), unrestricted) and
 * log phi_T(g) for a given label sequence, by extending the empty prefix label by label.
 */
int orc_prefix_and_full(const float* x, int T, int V, int blank_id, const int32_t* labels, int n,
                        double* log_psi, double* log_phi_T) {
  orc_cfg c; memset(&c, 0, sizeof c);
  c.vocab = V; c.beam = 1; c.blank_id = blank_id;
  c.eos_id = -1;                                   /* no id is special here */
  orc_utt u; memset(&u, 0, sizeof u); u.cfg = c; u.T = T; u.V = V; u.x = x;
  orc_hyp a, b; hyp_alloc(&a, T, n + 1); hyp_alloc(&b, T, n + 1);
  orc_hyp *g = &a, *h = &b;
  g->len = 0; g->rs = 0; g->re = T; g->gb[0] = 0.0; g->gn[0] = -INFINITY;
  for (int t = 1; t <= T; ++t) { g->gb[t] = g->gb[t - 1] + Xv(&u, t, blank_id); g->gn[t] = -INFINITY; }
  double psi = 0.0;
  for (int i = 0; i < n; ++i) {
    int k = labels[i], l = i + 1;
    psi = -INFINITY;
    for (int t = l; t <= T; ++t) psi = lae(psi, f_term(g, t, k) + Xv(&u, t, k));
    h->len = g->len + 1; memcpy(h->labels, g->labels, sizeof(int32_t) * (size_t)g->len);
    h->labels[g->len] = k; h->rs = l; h->re = T;
    for (int t = 0; t <= T; ++t) { h->gn[t] = -INFINITY; h->gb[t] = -INFINITY; }
    double np = -INFINITY, bp = -INFINITY;
    for (int t = l; t <= T; ++t) {
      double ft = f_term(g, t, k);
      double nn = lae(np, ft) + Xv(&u, t, k);
      double bb = lae(np, bp) + Xv(&u, t, blank_id);
      h->gn[t] = nn; h->gb[t] = bb; np = nn; bp = bb;
    }
    orc_hyp* t2 = g; g = h; h = t2;
  }
  *log_psi = psi;
  *log_phi_T = (g->rs <= T && g->re >= T) ? lae(g->gn[T], g->gb[T]) : -INFINITY;
  hyp_free(&a); hyp_free(&b);
  return 0;
}

void orc_set_threads(int n) {
#ifdef _OPENMP
  omp_set_num_threads(n > 0 ? n : 1);
#else
  (void)n;
#endif
}

/* Parallel-for over utterances of one free-running step (CPU-baseline timing only). */
void orc_batch_step_auto(orc_utt** utts, int n, const float* att /*[n][beam][V]*/, int32_t* fin) {
#pragma omp parallel for schedule(dynamic)
  for (int i = 0; i < n; ++i) {
    orc_utt* u = utts[i];
    if (u->finished) { fin[i] = 1; continue; }
    fin[i] = orc_step_auto(u, att + (size_t)i * u->cfg.beam * u->V);
  }
}
