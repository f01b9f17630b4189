// Host side of the ctcbs C ABI (see include/ctcbs.h): argument checks, device memory,
// kernel launches.  Every step of the decoding path runs in the kernels of k_*.h.
#include "../../include/ctcbs.h"

#include <hip/hip_runtime.h>
#include <math.h>
#include <map>
#include <mutex>
#include <new>
#include <stdlib.h>
#include <string.h>
#include <vector>

#include "common.h"
#include "k_finalize.h"
#include "k_ingest.h"
#include "k_score.h"
#include "k_score_dense.h"
#include "k_select.h"

static thread_local int g_last_hip = 0;

#define HIPCHK(expr)                                   \
  do {                                                 \
    hipError_t _e = (expr);                            \
    if (_e != hipSuccess) { g_last_hip = (int)_e; return CTCBS_EHIP; } \
  } while (0)

struct ctcbs {
  ctcbs_config_t cfg;
  Params p;
  Params p_step;       // the parameter block of the last step enqueued
  ScoreSmem sm;
  hipStream_t stream;
  int device;          // the device the handle lives on (current at creation)
  std::vector<void*> allocs;
  std::vector<int32_t> lens, lmax;
  int32_t step;        // steps enqueued
  int32_t cur;         // buffer holding the current beam
  int32_t l_cap;       // largest step cap over the batch
  int32_t l_cap_alloc; // step cap of an utterance of t_max frames: what the buffers are sized for
  int32_t *d_lens, *d_lmax;
  int32_t union_init[4];
  int32_t known_finished;
  size_t score_smem_bytes;
  int score_block, score_lpc, select_block;
  bool select_fpl2;            // the select kernels' form with the two-frames-per-lane recurrence only
  bool score_wide;
  int dense_nit, dense_nch;   // all-candidates score kernel: float4 per lane and column (0: not used), chunks per utterance
  size_t dense_smem_bytes;
  // result staging
  int32_t *d_tokens, *d_frames, *d_ntok, *d_flags;
  float* d_score;
  int32_t res_cap;
  // non-blocking progress: pinned, device-mapped word the score kernel refreshes every step, and
  // two events that keep the host at most two poll intervals ahead of the device
  int32_t* h_flag;
  hipEvent_t throttle[2];
  bool throttle_made, throttle_armed[2];
  int32_t throttle_k;
  // optional per-kernel timing
  bool profiling;
  std::vector<hipEvent_t> events;   // 3 per recorded step: before score, after score, after select
  size_t ev_used;
};

template <typename T>
static int dev_alloc(ctcbs* h, T** out, size_t n) {
  void* ptr = nullptr;
  size_t bytes = n * sizeof(T);
  if (bytes == 0) bytes = sizeof(T);
  hipError_t e = hipMalloc(&ptr, bytes);
  if (e != hipSuccess) { g_last_hip = (int)e; (void)hipGetLastError(); return CTCBS_ENOMEM; }
  h->allocs.push_back(ptr);
  *out = (T*)ptr;
  return CTCBS_OK;
}

static void free_all(ctcbs* h) {
  for (void* q : h->allocs) (void)hipFree(q);
  h->allocs.clear();
  if (h->h_flag) { (void)hipHostFree(h->h_flag); h->h_flag = nullptr; }
  if (h->throttle_made) {
    (void)hipEventDestroy(h->throttle[0]); (void)hipEventDestroy(h->throttle[1]);
    h->throttle_made = false;
  }
}

static int step_cap(const ctcbs_config_t* c, int T) {
  int l = T;
  if (c->max_len_ratio > 0.0f) { int r = (int)floor((double)c->max_len_ratio * (double)T); if (r < l) l = r; }
  if (c->max_len_abs > 0 && c->max_len_abs < l) l = c->max_len_abs;
  if (l < 1) l = 1;
  return l;
}

extern "C" const char* ctcbs_strerror(int code) {
  switch (code) {
    case CTCBS_OK: return "ok";
    case CTCBS_DONE: return "all utterances finished";
    case CTCBS_EINVAL: return "invalid argument or unsupported size";
    case CTCBS_ENOMEM: return "out of memory";
    case CTCBS_EHIP: return "HIP runtime error";
    case CTCBS_ESTATE: return "call not valid in this state";
    case CTCBS_ECAP: return "output capacity too small";
    default: return "unknown ctcbs error code";
  }
}

extern "C" int ctcbs_last_hip_error(void) { return g_last_hip; }

static int validate(const ctcbs_config_t* c) {
  if (c->n_utt < 1 || c->t_max < 1 || c->t_max > 6140 || c->vocab < 3) return CTCBS_EINVAL;
  if (c->beam < 1 || c->beam > MAX_BEAM) return CTCBS_EINVAL;
  if (c->blank_id < 0 || c->blank_id >= c->vocab || c->eos_id < 0 || c->eos_id >= c->vocab ||
      c->blank_id == c->eos_id) return CTCBS_EINVAL;
  if (c->cand_k < 0) return CTCBS_EINVAL;
  bool restricted = c->cand_k > 0 && c->cand_k < c->vocab - 2;
  if (!(c->ctc_weight >= 0.0f && c->ctc_weight <= 1.0f)) return CTCBS_EINVAL;
  if (c->length_bonus != c->length_bonus || c->max_len_ratio != c->max_len_ratio || c->max_len_ratio < 0.0f)
    return CTCBS_EINVAL;
  if (c->max_len_abs < 0) return CTCBS_EINVAL;
  if (c->end_flags & ~7) return CTCBS_EINVAL;
  if ((c->end_flags & CTCBS_END_BASELINE) && (c->end_m < 1 || c->end_m > MAX_END_M)) return CTCBS_EINVAL;
  if ((c->end_flags & CTCBS_END_TAU_COUNT) && c->end_c < 0) return CTCBS_EINVAL;
  if ((c->end_flags & CTCBS_END_EOS_RUN) && (c->eos_run < 1 || c->eos_run > MAX_EOS_RUN)) return CTCBS_EINVAL;
  if (c->poll_every < 0) return CTCBS_EINVAL;
  if (c->att_is_logits != 0 && c->att_is_logits != 1) return CTCBS_EINVAL;
  if (c->win_union != 0 && c->win_union != 1) return CTCBS_EINVAL;
  if (c->keep_candidates != 0 && c->keep_candidates != 1) return CTCBS_EINVAL;
  if ((long long)c->n_utt * c->beam > (1ll << 24)) return CTCBS_EINVAL;
  return CTCBS_OK;
}

// Per-batch part of the initialisation: lengths, step caps, transposed posteriors, empty beams.
static int ingest(ctcbs* h, const float* d_ctc_logp, const int32_t* h_lens) {
  const ctcbs_config_t& c = h->cfg;
  Params& p = h->p;
  const int U = c.n_utt;
  std::vector<int32_t> lens(h_lens, h_lens + U), lmax(U);
  int l_cap = 1, n_empty = 0;
  for (int u = 0; u < U; ++u) {
    if (lens[u] < 0 || lens[u] > c.t_max) return CTCBS_EINVAL;
    if (lens[u] == 0) { lmax[u] = 1; ++n_empty; continue; }   // an unused slot of the batch
    lmax[u] = step_cap(&c, lens[u]);
    if (lmax[u] > l_cap) l_cap = lmax[u];
  }
  hipStream_t st = h->stream;
  HIPCHK(hipStreamSynchronize(st));              // the staging vectors below are reused
  h->lens.swap(lens); h->lmax.swap(lmax); h->l_cap = l_cap;
  const size_t UW = (size_t)U * p.Wb;
  HIPCHK(hipMemcpyAsync(h->d_lens, h->lens.data(), sizeof(int32_t) * U, hipMemcpyHostToDevice, st));
  HIPCHK(hipMemcpyAsync(h->d_lmax, h->lmax.data(), sizeof(int32_t) * U, hipMemcpyHostToDevice, st));
  {
    // step 1: every hypothesis is empty, tau = tau~ = 0
    int e_max = 0;
    for (int u = 0; u < U; ++u) { int e = c.win_m2 < h->lens[u] ? c.win_m2 : h->lens[u]; if (e > e_max) e_max = e; }
    h->union_init[0] = 0x7fffffff; h->union_init[1] = -1; h->union_init[2] = 0; h->union_init[3] = e_max;
    HIPCHK(hipMemcpyAsync(p.union_win, h->union_init, sizeof(h->union_init), hipMemcpyHostToDevice, st));
  }
  HIPCHK(hipMemsetAsync(p.grp_n, 0, sizeof(int32_t) * UW, st));
  HIPCHK(hipMemsetAsync(p.stopped, 0, sizeof(int32_t) * UW, st));
  HIPCHK(hipMemsetAsync(p.err, 0, sizeof(int32_t), st));
  {
    const int nvt = (p.V + 255) / 256, ntt = (c.t_max + 5 + 31) / 32;   // stored indices 0 .. t_max + 4
    const int n_tiles = nvt * ntt, per_xcd = (n_tiles + 7) / 8;
    const dim3 tg(8 * per_xcd, U);
    if (p.V % 4 == 0 && ((uintptr_t)d_ctc_logp & 15) == 0)
      hipLaunchKernelGGL(k_transpose<true>, tg, dim3(256), 0, st, p, d_ctc_logp, nvt, n_tiles, per_xcd);
    else
      hipLaunchKernelGGL(k_transpose<false>, tg, dim3(256), 0, st, p, d_ctc_logp, nvt, n_tiles, per_xcd);
  }
  HIPCHK(hipGetLastError());
  hipLaunchKernelGGL(k_init_state, dim3(U), dim3(64), 0, st, p, n_empty);
  HIPCHK(hipGetLastError());
  h->step = 0; h->cur = 0; h->known_finished = n_empty;
  h->profiling = false; h->ev_used = 0;
  h->throttle_k = 0; h->throttle_armed[0] = h->throttle_armed[1] = false;
  *h->h_flag = n_empty;
  HIPCHK(hipStreamSynchronize(st));
  return CTCBS_OK;
}

static int create_impl(ctcbs* h, const float* d_ctc_logp, const int32_t* h_lens) {
  const ctcbs_config_t& c = h->cfg;
  Params& p = h->p;
  memset(&p, 0, sizeof p);
  const int U = c.n_utt, V = c.vocab, Wb = c.beam;
  const bool restricted = c.cand_k > 0 && c.cand_k < V - 2;
  const int K = restricted ? c.cand_k : V - 2;
  p.U = U; p.V = V; p.Wb = Wb; p.K = K;
  p.Tp = ((c.t_max + 5 + 31) / 32) * 32;        // frames 0..t_max plus slack for aligned float4 reads; rows of whole 128-byte lines
  p.t_max = c.t_max; p.blank_id = c.blank_id; p.eos_id = c.eos_id; p.restricted = restricted ? 1 : 0;
  p.win_m1 = c.win_m1; p.win_m2 = c.win_m2; p.end_flags = c.end_flags;
  p.end_m = (c.end_m >= 1 && c.end_m <= MAX_END_M) ? c.end_m : 1;
  p.end_c = c.end_c; p.eos_run = c.eos_run; p.end_d = c.end_d;
  p.lambda = (double)c.ctc_weight; p.beta = (double)c.length_bonus;
  p.att_logits = c.att_is_logits ? 1 : 0;
  p.win_union = c.win_union ? 1 : 0;
  // large candidate sets go through the per-candidate arrays in global memory whatever the caller asked for
  p.keep_cand = (c.keep_candidates || K > 256 || !restricted) ? 1 : 0;

  // capacity for any batch of lengths <= t_max (the step cap grows with the length)
  h->l_cap_alloc = step_cap(&c, c.t_max);
  h->l_cap = h->l_cap_alloc;
  p.l_cap = h->l_cap_alloc;

  const size_t UW = (size_t)U * Wb;
  int rc;
  int32_t*& d_lens = h->d_lens; int32_t*& d_lmax = h->d_lmax;
#define A(ptr, n) if ((rc = dev_alloc(h, &(ptr), (n))) != CTCBS_OK) return rc
  A(p.xT, (size_t)U * V * p.Tp);
  A(p.Bcum, (size_t)U * p.Tp);
  A(d_lens, (size_t)U); A(d_lmax, (size_t)U);
  p.lens = d_lens; p.lmax = d_lmax;
  for (int b = 0; b < 2; ++b) {
    A(p.gn[b], UW * p.Tp); A(p.gb[b], UW * p.Tp);
    A(p.rec[b], UW);
  }
  A(p.uinfo, (size_t)U);
  A(p.win_s, UW); A(p.win_e, UW);
  {
    const size_t nc = p.keep_cand ? UW * K : 1;            // (not kept: never touched)
    A(p.cand_id, nc); A(p.cand_inc, nc); A(p.cand_att, nc); A(p.cand_pre, nc);
    A(p.cand_ctc, nc); A(p.cand_joint, nc);
  }
  A(p.grp_n, UW); A(p.grp_J, UW * Wb); A(p.grp_ci, UW * Wb); A(p.grp_tok, UW * Wb);
  A(p.grp_inc, UW * Wb); A(p.grp_att, UW * Wb);
  A(p.ctc_eos, UW); A(p.joint_eos, UW); A(p.stopped, UW); A(p.grp_cells, UW);
  A(p.utt, (size_t)U); A(p.finished, (size_t)((U + 3) & ~3));   /* read as whole words by the score kernel */ A(p.cells, (size_t)U); A(p.groups, (size_t)U);
  A(p.n_finished, (size_t)1); A(p.union_win, (size_t)4); A(p.err, (size_t)1);
  const size_t trie_n = (size_t)(h->l_cap_alloc + 1) * UW;
  A(p.trie_parent, trie_n); A(p.trie_token, trie_n); A(p.trie_tau, trie_n);
  A(p.out_parent, UW); A(p.out_token, UW); A(p.out_score, UW); A(p.out_live, UW);
  A(p.out_tau, UW); A(p.out_tau_end, UW); A(p.out_eos_added, UW); A(p.out_stopped, UW);
#ifdef CTCBS_TRACE
  A(p.trace, UW * 16);
#endif
  h->res_cap = h->l_cap_alloc;
  A(h->d_tokens, (size_t)U * h->res_cap); A(h->d_frames, (size_t)U * h->res_cap);
  A(h->d_ntok, (size_t)U); A(h->d_flags, (size_t)U); A(h->d_score, (size_t)U);
#undef A

  {
    void* hp = nullptr;
    hipError_t e = hipHostMalloc(&hp, 64, hipHostMallocMapped);
    if (e != hipSuccess) { g_last_hip = (int)e; (void)hipGetLastError(); return CTCBS_ENOMEM; }
    h->h_flag = (int32_t*)hp;
    *h->h_flag = 0;
    void* dp = nullptr;
    HIPCHK(hipHostGetDevicePointer(&dp, hp, 0));
    p.host_finished = (int32_t*)dp;
    HIPCHK(hipEventCreateWithFlags(&h->throttle[0], hipEventDisableTiming));
    HIPCHK(hipEventCreateWithFlags(&h->throttle[1], hipEventDisableTiming));
    h->throttle_made = true;
  }
  // launch shapes of the per-step kernels
  h->score_block = 256;
  const bool windowed = c.win_m1 >= 0 && c.win_m2 >= 0 && (c.win_m1 + c.win_m2) <= 448;
  // whole-utterance windows of utterances of up to ~500 frames are faster in the 16-lane form too (twice
  // the candidates per round; measured: T <= 250 20.0 -> 15.3 us, T <= 500 21.1 -> 18.8 us, T in 500..800
  // 25.1 -> 26.9 us, T in 1000..1500 34.2 -> 43.5 us: beyond 512 frames the 64-lane form stays)
  const bool short_whole = !windowed && p.Tp <= 512;
  h->score_lpc = (windowed || short_whole) ? 16 : 64;
  // windows beyond 128 frames (16 lanes x 2 float4): four float4 per lane in flight, two candidates at a time
  h->score_wide = short_whole || (windowed && (c.win_m1 + c.win_m2 + 1 + 3) > 128);
  ScoreSmem& sm = h->sm;
  size_t off = 0;
  sm.off_work = (int32_t)off;
  off += restricted ? (size_t)PIVOT_CAP * 12 : 0;       // short list (key, id, flag); also holds the radix histogram
  sm.off_f = (int32_t)off;
  off += (size_t)2 * p.Tp * 4;                   // Tp is a multiple of 4: both arrays 16-byte aligned
  sm.off_small = (int32_t)off;
  if (K <= h->score_block) off += (size_t)K * 32 + 8;
  sm.wp_max = p.Tp;
  h->score_smem_bytes = off;
  // all-candidates kernel: needs the f terms of all beam slots in LDS and a column window in registers
  h->dense_nit = 0; h->dense_nch = 1; h->dense_smem_bytes = (size_t)Wb * p.Tp * 4;
  if (!restricted && !(c.end_flags & CTCBS_END_EOS_RUN) && !c.att_is_logits && !c.win_union &&
      h->dense_smem_bytes <= 150 * 1024 && p.Tp <= 2048) {
    h->dense_nit = p.Tp <= 256 ? 1 : (p.Tp <= 512 ? 2 : (p.Tp <= 1024 ? 4 : (p.Tp <= 1536 ? 6 : 8)));
    // enough work-groups to cover the chip, but at least a few dozen candidates each
    int nch = (256 + U - 1) / U;
    const int most = K / 32 > 1 ? K / 32 : 1;
    h->dense_nch = nch < 1 ? 1 : (nch > most ? most : nch);
  }
  if (off > 160 * 1024) return CTCBS_EINVAL;
  // per-hypothesis windows whose margins keep them within 128 frames (but for a hypothesis whose two time
  // indices lie far apart): the select kernels then carry the two-frames-per-lane recurrence only
  h->select_fpl2 = windowed && !c.win_union && (c.win_m1 + c.win_m2 + 1 + 3) <= 128;
  int nw = Wb < 16 ? Wb : 16;
  h->select_block = 64 * (nw <= 4 ? 4 : (nw <= 8 ? 8 : 16));
  // One wave for the ended set plus one per new hypothesis is the shape that finishes an utterance soonest.
  // From two utterances per compute unit on, what counts is how many utterances are resident: at beam
  // 9..12, eight waves (survivors in two rounds) then beat sixteen (measured at beam 10: 14.9 against 18.1 us
  // at 512 utterances, 37.9 against 55.0 at 2048; at 256 utterances 12.8 against 11.4)
  if (h->select_block == 1024 && Wb <= 12 && U >= 512) h->select_block = 512;

  return ingest(h, d_ctc_logp, h_lens);
}

extern "C" int ctcbs_create(const ctcbs_config_t* cfg, const float* d_ctc_logp, const int32_t* h_lens,
                            ctcbs_t** out) {
  if (out) *out = nullptr;
  if (!cfg || !d_ctc_logp || !h_lens || !out) return CTCBS_EINVAL;
  int rc = validate(cfg);
  if (rc != CTCBS_OK) return rc;
  ctcbs* h = new (std::nothrow) ctcbs();
  if (!h) return CTCBS_ENOMEM;
  h->h_flag = nullptr; h->throttle_made = false;
  h->cfg = *cfg;
  h->stream = (hipStream_t)cfg->stream;
  if (hipGetDevice(&h->device) != hipSuccess) { g_last_hip = (int)hipGetLastError(); delete h; return CTCBS_EHIP; }
  rc = create_impl(h, d_ctc_logp, h_lens);
  if (rc != CTCBS_OK) { free_all(h); delete h; return rc; }
  *out = h;
  return CTCBS_OK;
}

// Kernels that want more than 64 KB of dynamic LDS need the attribute raised first.  It belongs to
// the kernel, not to a handle: it is only ever raised (handles of different sizes, on different
// threads, share it), and only when a launch needs more than what is already allowed.
static hipError_t allow_lds(const void* kernel, size_t bytes) {
  if (bytes <= 64 * 1024) return hipSuccess;
  static std::mutex mu;
  static std::map<const void*, size_t> allowed;
  std::lock_guard<std::mutex> lock(mu);
  try {
    size_t& have = allowed[kernel];
    if (bytes <= have) return hipSuccess;
    hipError_t e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e == hipSuccess) have = bytes;
    return e;
  } catch (...) {                                          // (the map could not grow)
    return hipErrorOutOfMemory;
  }
}

template <int BLOCK, int LPC, int CB, int IT, bool BIGK>
static hipError_t launch_score_as(ctcbs* h, const Params& p, const float* att, int l) {
  hipError_t ea = allow_lds((const void*)k_score<BLOCK, LPC, CB, IT, BIGK>, h->score_smem_bytes);
  if (ea != hipSuccess) return ea;
  // attention rows that do not start on 16-byte boundaries cannot be loaded as float4: the candidate
  // selection then reads them element by element (slower, equivalent)
  const int flags = (((uintptr_t)att & 15) == 0 && p.V % 4 == 0) ? 1 : 0;
  hipLaunchKernelGGL((k_score<BLOCK, LPC, CB, IT, BIGK>), dim3(p.Wb, p.U), dim3(BLOCK), h->score_smem_bytes,
                     h->stream, (const HypRec*)p.rec[h->cur], (const UttInfo*)p.uinfo, (const uint32_t*)p.finished,
                     att, (int)p.Wb, (int)p.V, flags, l, p, h->sm, h->cur);
  return hipGetLastError();
}

// the kernel's form with the paths for many candidates only where they can be taken (see k_score)
template <int BLOCK, int LPC, int CB, int IT>
static hipError_t launch_score(ctcbs* h, const Params& p, const float* att, int l) {
  const bool one_wave_ranks = p.K <= BLOCK && p.K <= 64 && p.V <= 65536;
  if (!one_wave_ranks) return launch_score_as<BLOCK, LPC, CB, IT, true>(h, p, att, l);
  return launch_score_as<BLOCK, LPC, CB, IT, false>(h, p, att, l);
}

template <int NIT>
static hipError_t launch_dense(ctcbs* h, const Params& p, const float* att, int l) {
  hipError_t ea = allow_lds((const void*)k_score_dense<1024, NIT>, h->dense_smem_bytes);
  if (ea != hipSuccess) return ea;
  hipLaunchKernelGGL((k_score_dense<1024, NIT>), dim3(p.U * h->dense_nch), dim3(1024), h->dense_smem_bytes,
                     h->stream, p, att, l, h->cur, h->dense_nch);
  return hipGetLastError();
}

// One step with the kernels working on `p`: the handle's own parameter block, or a copy of it whose
// per-step scratch arrays lie elsewhere (ctcbs_step_static).
static int step_impl(ctcbs_t* h, const Params& p, const float* d_att_logp, ctcbs_step_out_t* out) {
  if (!h || !d_att_logp) return CTCBS_EINVAL;
  if (h->known_finished >= p.U || h->step >= h->l_cap) return CTCBS_DONE;
  const int l = h->step + 1;
  hipEvent_t* ev = nullptr;
  if (h->profiling && h->ev_used + 3 <= h->events.size()) {
    ev = &h->events[h->ev_used];
    h->ev_used += 3;
    HIPCHK(hipEventRecord(ev[0], h->stream));
  }
  // 16 lanes x 2 float4 per candidate cover windows of up to 128 frames without a second trip to
  // memory, 16 lanes x 4 float4 wider windows and whole utterances of up to 512 frames; whole-utterance
  // windows beyond that use whole waves, 4 float4 (1024 frames) in flight (see create_impl)
  hipError_t e;
  switch (h->dense_nit) {                 // every id a candidate: one work-group serves all beam slots
    case 1: e = launch_dense<1>(h, p, d_att_logp, l); break;
    case 2: e = launch_dense<2>(h, p, d_att_logp, l); break;
    case 4: e = launch_dense<4>(h, p, d_att_logp, l); break;
    case 6: e = launch_dense<6>(h, p, d_att_logp, l); break;
    case 8: e = launch_dense<8>(h, p, d_att_logp, l); break;
    default:
      e = (h->score_lpc == 16) ? (h->score_wide ? launch_score<256, 16, 2, 4>(h, p, d_att_logp, l)
                                                : launch_score<256, 16, 3, 2>(h, p, d_att_logp, l))
                               : launch_score<256, 64, 2, 4>(h, p, d_att_logp, l);
  }
  HIPCHK(e);
  if (ev) HIPCHK(hipEventRecord(ev[1], h->stream));       // (the list builder below counts as selection)
  if (h->dense_nit || p.K > h->score_block) {
    if (p.K <= 1024 * 8)
      hipLaunchKernelGGL((k_group_top_regs<1024, 8>), dim3(p.U * p.Wb), dim3(1024), 0, h->stream, p, h->cur);
    else
      hipLaunchKernelGGL((k_group_top<256>), dim3(p.U * p.Wb), dim3(256), 0, h->stream, p, h->cur);
    HIPCHK(hipGetLastError());
  }
  // Small batches leave most compute units idle in the one-work-group-per-utterance form: there the
  // split form (one work-group per new beam slot, each ranking the utterance's lists itself) is
  // faster (measured: U=64 and U=128 at beam 10).  Large batches fill the chip either way and the
  // Wb-fold repeated ranking only costs (U=256 at beam 20: three times slower).  The batch-union
  // window needs the utterance's hypotheses in one place.
  const bool split = !p.win_union && p.U * p.Wb <= 2048;
  const size_t split_lds = (size_t)28 * p.Wb * p.Wb + 64;
  if (split) {
    if (h->select_fpl2)
      hipLaunchKernelGGL((k_select_split<256, 2>), dim3(p.U * p.Wb), dim3(256), split_lds, h->stream,
                         (const HypRec*)p.rec[h->cur], p.utt, (const int32_t*)p.grp_n, (const double*)p.grp_J,
                         (const int32_t*)p.grp_tok, (const float*)p.grp_inc, (const float*)p.grp_att, (int)p.Wb, l, p, h->cur);
    else
      hipLaunchKernelGGL((k_select_split<256, 8>), dim3(p.U * p.Wb), dim3(256), split_lds, h->stream,
                         (const HypRec*)p.rec[h->cur], p.utt, (const int32_t*)p.grp_n, (const double*)p.grp_J,
                         (const int32_t*)p.grp_tok, (const float*)p.grp_inc, (const float*)p.grp_att, (int)p.Wb, l, p, h->cur);
  } else {
    const int NE = p.Wb * p.Wb;
    const size_t sel_lds = (size_t)16 * ((NE + 9) & ~1) + (size_t)32 * NE;
#define CTCBS_SELECT(BS, F) hipLaunchKernelGGL((k_select<BS, F>), dim3(p.U), dim3(BS), sel_lds, h->stream, p, l, h->cur)
    switch (h->select_block) {
      case 256: if (h->select_fpl2) CTCBS_SELECT(256, 2); else CTCBS_SELECT(256, 8); break;
      case 512: if (h->select_fpl2) CTCBS_SELECT(512, 2); else CTCBS_SELECT(512, 8); break;
      default: if (h->select_fpl2) CTCBS_SELECT(1024, 2); else CTCBS_SELECT(1024, 8); break;
    }
#undef CTCBS_SELECT
  }
  HIPCHK(hipGetLastError());
  if (ev) HIPCHK(hipEventRecord(ev[2], h->stream));
  h->step = l;
  h->cur ^= 1;
  h->p_step = p;                           // where this step's intermediate arrays lie (ctcbs_peek)
  int polled = -1;
  if (h->cfg.poll_every > 0 && (l % h->cfg.poll_every) == 0) {
    // wait (normally not at all) for the interval before the last one, then look at the count the
    // device has published; the device keeps at least one interval of queued work meanwhile
    const int k = h->throttle_k++;
    if (h->throttle_armed[(k + 1) & 1]) HIPCHK(hipEventSynchronize(h->throttle[(k + 1) & 1]));
    HIPCHK(hipEventRecord(h->throttle[k & 1], h->stream));
    h->throttle_armed[k & 1] = true;
    polled = *(volatile int32_t*)h->h_flag;
    h->known_finished = polled;
  }
  if (out) {
    out->step = l; out->n_finished = polled;
    out->d_parent = p.out_parent; out->d_token = p.out_token; out->d_score = p.out_score;
    out->d_live = p.out_live; out->d_finished = p.finished; out->d_tau = p.out_tau;
    out->d_tau_end = p.out_tau_end; out->d_eos_added = p.out_eos_added; out->d_stopped = p.out_stopped;
  }
  return CTCBS_OK;
}

extern "C" int ctcbs_step(ctcbs_t* h, const float* d_att_logp, ctcbs_step_out_t* out) {
  if (!h || !d_att_logp) return CTCBS_EINVAL;
  return step_impl(h, h->p, d_att_logp, out);
}

// ---- the step for callers that cannot allocate --------------------------------------------------
// Same kernels, same results; the arrays that carry a step's intermediate values from the score kernel
// to the select kernel (windows, eos scores, the groups' best-first lists, stop flags, work counts) lie
// in a fixed array in the library's own image instead of memory the handle allocated.  Every GPU holds
// its own copy of that array at its own address, so its address is asked for once per device.
#define CTCBS_STATIC_SCRATCH_BYTES (4u << 20)
#define CTCBS_MAX_DEVICES 64
static __device__ __align__(256) unsigned char scratch[CTCBS_STATIC_SCRATCH_BYTES];
static std::mutex g_scratch_mu;
static unsigned char* g_scratch_ptr[CTCBS_MAX_DEVICES];     // device address of `scratch` on each device (0: not asked yet)

// bytes of the per-step scratch arrays of a handle, each array on a 256-byte boundary
static size_t static_scratch_need(const Params& p) {
  const size_t UW = (size_t)p.U * p.Wb, L = UW * p.Wb;
  auto r = [](size_t n) { return (n + 255) & ~(size_t)255; };
  return r(UW * 4) * 4 /* win_s, win_e, grp_n, stopped */ + r(UW * 8) * 3 /* ctc_eos, joint_eos, grp_cells */ +
         r(L * 8) /* grp_J */ + r(L * 4) * 4 /* grp_ci, grp_tok, grp_inc, grp_att */;
}

__global__ void k_clear_words(int32_t* a, int32_t* b, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) { a[i] = 0; b[i] = 0; }
}

extern "C" int ctcbs_step_static(ctcbs_t* h, const float* d_att_logp, ctcbs_step_out_t* out) {
  if (!h || !d_att_logp) return CTCBS_EINVAL;
  // candidate sets that go through arrays in global memory (more than 256 candidates per hypothesis, or
  // every id a candidate) would need those arrays here too: not offered
  if (h->dense_nit || h->p.K > h->score_block) return CTCBS_EINVAL;
  if (static_scratch_need(h->p) > CTCBS_STATIC_SCRATCH_BYTES) return CTCBS_EINVAL;
  int dev = -1;
  HIPCHK(hipGetDevice(&dev));
  if (dev != h->device || dev < 0 || dev >= CTCBS_MAX_DEVICES) return CTCBS_ESTATE;   // the handle's device must be current
  unsigned char* base = nullptr;
  {
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
      void* ptr = nullptr;
      HIPCHK(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
      g_scratch_ptr[dev] = (unsigned char*)ptr;
    }
    base = g_scratch_ptr[dev];
  }
  if (!base) return CTCBS_EHIP;
  if (h->known_finished >= h->p.U || h->step >= h->l_cap) return CTCBS_DONE;
  Params p = h->p;
  const size_t UW = (size_t)p.U * p.Wb, L = UW * p.Wb;
  size_t off = 0;
  auto take = [&](size_t bytes) { unsigned char* q = base + off; off += (bytes + 255) & ~(size_t)255; return q; };
  p.win_s = (int32_t*)take(UW * 4); p.win_e = (int32_t*)take(UW * 4);
  p.grp_n = (int32_t*)take(UW * 4); p.stopped = (int32_t*)take(UW * 4);
  p.ctc_eos = (double*)take(UW * 8); p.joint_eos = (double*)take(UW * 8); p.grp_cells = (long long*)take(UW * 8);
  p.grp_J = (double*)take(L * 8);
  p.grp_ci = (int32_t*)take(L * 4); p.grp_tok = (int32_t*)take(L * 4);
  p.grp_inc = (float*)take(L * 4); p.grp_att = (float*)take(L * 4);
  // the array keeps what the last call on this GPU (of any handle) left: list lengths and stop flags start
  // from zero (a fill kernel, not a memset node: the call may be under graph capture)
  hipLaunchKernelGGL(k_clear_words, dim3((unsigned)((UW + 255) / 256)), dim3(256), 0, h->stream, p.grp_n, p.stopped, (int)UW);
  HIPCHK(hipGetLastError());
  return step_impl(h, p, d_att_logp, out);
}

extern "C" int ctcbs_reset(ctcbs_t* h, const float* d_ctc_logp, const int32_t* h_lens) {
  if (!h || !d_ctc_logp || !h_lens) return CTCBS_EINVAL;
  return ingest(h, d_ctc_logp, h_lens);
}

extern "C" int ctcbs_poll(ctcbs_t* h, int32_t* n_finished) {
  if (!h) return CTCBS_EINVAL;
  int32_t v = 0;
  HIPCHK(hipMemcpyAsync(&v, h->p.n_finished, sizeof v, hipMemcpyDeviceToHost, h->stream));
  HIPCHK(hipStreamSynchronize(h->stream));
  h->known_finished = v;
  if (n_finished) *n_finished = v;
  return CTCBS_OK;
}

extern "C" int ctcbs_finalize(ctcbs_t* h, int32_t* h_tokens, int32_t cap, int32_t* h_ntok, float* h_score,
                              int32_t* h_frames, int32_t* h_flags) {
  if (!h || !h_tokens || !h_ntok || !h_score || cap < 0) return CTCBS_EINVAL;
  const int U = h->p.U, rc_cap = h->res_cap;
  const size_t fin_lds = (size_t)(h->l_cap_alloc + 1) * h->p.Wb + (size_t)h->l_cap_alloc + 1;
  const int use_lds = fin_lds <= 60 * 1024;
  hipLaunchKernelGGL((k_finalize<256>), dim3(U), dim3(256), use_lds ? fin_lds : 0, h->stream, h->p, h->cur,
                     h->step, rc_cap, use_lds, h->d_tokens, h->d_frames, h->d_ntok, h->d_score, h->d_flags);
  HIPCHK(hipGetLastError());
  std::vector<int32_t> tok((size_t)U * rc_cap), frm((size_t)U * rc_cap), nt(U), fl(U);
  HIPCHK(hipMemcpyAsync(tok.data(), h->d_tokens, tok.size() * 4, hipMemcpyDeviceToHost, h->stream));
  HIPCHK(hipMemcpyAsync(frm.data(), h->d_frames, frm.size() * 4, hipMemcpyDeviceToHost, h->stream));
  HIPCHK(hipMemcpyAsync(nt.data(), h->d_ntok, (size_t)U * 4, hipMemcpyDeviceToHost, h->stream));
  HIPCHK(hipMemcpyAsync(fl.data(), h->d_flags, (size_t)U * 4, hipMemcpyDeviceToHost, h->stream));
  HIPCHK(hipMemcpyAsync(h_score, h->d_score, (size_t)U * 4, hipMemcpyDeviceToHost, h->stream));
  int32_t err = 0;
  HIPCHK(hipMemcpyAsync(&err, h->p.err, sizeof err, hipMemcpyDeviceToHost, h->stream));
  HIPCHK(hipStreamSynchronize(h->stream));
  if (err != 0) return CTCBS_ESTATE;     // a kernel's consistency check failed during this decode: no result
  for (int u = 0; u < U; ++u) {
    if (nt[u] < 0 || nt[u] > cap) return CTCBS_ECAP;
    h_ntok[u] = nt[u];
    for (int k = 0; k < nt[u]; ++k) {
      h_tokens[(size_t)u * cap + k] = tok[(size_t)u * rc_cap + k];
      if (h_frames) h_frames[(size_t)u * cap + k] = frm[(size_t)u * rc_cap + k];
    }
    if (h_flags) h_flags[u] = fl[u];
  }
  return CTCBS_OK;
}

extern "C" int ctcbs_stats(ctcbs_t* h, uint64_t* cells, uint64_t* groups, int32_t* steps) {
  if (!h) return CTCBS_EINVAL;
  std::vector<unsigned long long> c(h->p.U), g(h->p.U);
  HIPCHK(hipMemcpyAsync(c.data(), h->p.cells, c.size() * 8, hipMemcpyDeviceToHost, h->stream));
  HIPCHK(hipMemcpyAsync(g.data(), h->p.groups, g.size() * 8, hipMemcpyDeviceToHost, h->stream));
  HIPCHK(hipStreamSynchronize(h->stream));
  unsigned long long tot = 0, gt = 0;
  for (auto v : c) tot += v;
  for (auto v : g) gt += v;
  if (cells) *cells = tot;
  if (groups) *groups = gt;
  if (steps) *steps = h->step;
  return CTCBS_OK;
}

extern "C" int ctcbs_profile(ctcbs_t* h, int32_t enable) {
  if (!h) return CTCBS_EINVAL;
  if (enable && h->events.empty()) {
    h->events.resize((size_t)3 * (h->l_cap_alloc + 1));
    for (size_t i = 0; i < h->events.size(); ++i) {
      hipError_t e = hipEventCreate(&h->events[i]);
      if (e != hipSuccess) {
        for (size_t k = 0; k < i; ++k) (void)hipEventDestroy(h->events[k]);
        h->events.clear();
        g_last_hip = (int)e;
        return CTCBS_EHIP;
      }
    }
  }
  h->profiling = enable != 0;
  h->ev_used = 0;
  return CTCBS_OK;
}

extern "C" int ctcbs_profile_read(ctcbs_t* h, double* score_ms, double* select_ms, int32_t* n_steps) {
  if (!h) return CTCBS_EINVAL;
  HIPCHK(hipStreamSynchronize(h->stream));
  double a = 0.0, b = 0.0;
  for (size_t i = 0; i + 3 <= h->ev_used; i += 3) {
    float ms = 0.0f;
    HIPCHK(hipEventElapsedTime(&ms, h->events[i], h->events[i + 1])); a += ms;
    HIPCHK(hipEventElapsedTime(&ms, h->events[i + 1], h->events[i + 2])); b += ms;
  }
  if (score_ms) *score_ms = a;
  if (select_ms) *select_ms = b;
  if (n_steps) *n_steps = (int32_t)(h->ev_used / 3);
  return CTCBS_OK;
}

extern "C" int ctcbs_peek(ctcbs_t* h, int32_t what, void* h_dst, size_t bytes, size_t* need) {
  if (!h) return CTCBS_EINVAL;
  const Params& p = h->step > 0 ? h->p_step : h->p;
  const size_t UW = (size_t)p.U * p.Wb;
  const void* src = nullptr; size_t sz = 0;
  int32_t k = p.K;
  if (!p.keep_cand && (what == CTCBS_PEEK_CAND_ID || what == CTCBS_PEEK_CAND_CTC || what == CTCBS_PEEK_CAND_JOINT))
    return CTCBS_ESTATE;                                   // created without keep_candidates
  switch (what) {
    case CTCBS_PEEK_CAND_ID: src = p.cand_id; sz = UW * p.K * 4; break;
    case CTCBS_PEEK_CAND_CTC: src = p.cand_ctc; sz = UW * p.K * 8; break;
    case CTCBS_PEEK_CAND_JOINT: src = p.cand_joint; sz = UW * p.K * 8; break;
    case CTCBS_PEEK_WIN_S: src = p.win_s; sz = UW * 4; break;
    case CTCBS_PEEK_WIN_E: src = p.win_e; sz = UW * 4; break;
    case CTCBS_PEEK_CTC_EOS: src = p.ctc_eos; sz = UW * 8; break;
    case CTCBS_PEEK_JOINT_EOS: src = p.joint_eos; sz = UW * 8; break;
    case CTCBS_PEEK_N_CAND:
      if (need) *need = 4;
      if (h_dst && bytes >= 4) memcpy(h_dst, &k, 4);
      return CTCBS_OK;
    default: return CTCBS_EINVAL;
  }
  if (need) *need = sz;
  if (h_dst && bytes) {
    HIPCHK(hipMemcpyAsync(h_dst, src, bytes < sz ? bytes : sz, hipMemcpyDeviceToHost, h->stream));
    HIPCHK(hipStreamSynchronize(h->stream));
  }
  return CTCBS_OK;
}

#ifdef CTCBS_TRACE
extern "C" int ctcbs_trace_read(ctcbs_t* h, unsigned long long* dst) {
  HIPCHK(hipMemcpyAsync(dst, h->p.trace, (size_t)h->p.U * h->p.Wb * 16 * 8, hipMemcpyDeviceToHost, h->stream));
  HIPCHK(hipStreamSynchronize(h->stream));
  return CTCBS_OK;
}
#endif

#include "sched.h"

extern "C" void ctcbs_destroy(ctcbs_t* h) {
  if (!h) return;
  (void)hipStreamSynchronize(h->stream);
  for (hipEvent_t e : h->events) (void)hipEventDestroy(e);
  free_all(h);
  delete h;
}
