/*
 * ctcbs -- batched joint CTC/attention beam-search step on one MI355X (gfx950).
 *
 * C ABI of the decoding hot path of arXiv 2101.05600 ("Fast offline Transformer-based
 * end-to-end ASR for real-world applications"): Algorithm 2 (multiple-utterance batched
 * beam search) with Eq. (1)-(3) as its scoring function, the time-restricted prefix score
 * of Eq. (5), and the end-of-speech detection of Eq. (4) / Algorithm 3.  The acoustic
 * encoder and the attention decoder are outside: their outputs (CTC log-posteriors once
 * per batch, attention log-probabilities once per step) are inputs.
 *
 * Symbols: U utterances, Wb beam width, V output ids (blank and eos included), T_i frames
 * of utterance i, l the 1-based decoding step.  All scores are natural-log probabilities;
 * "log0" is reported as any value below -1e29 (canonically -1e30).
 *
 * Pointers named d_* are DEVICE pointers, h_* are HOST pointers.  The library never takes
 * ownership of a caller's buffer.  Every call returns 0 on success, a negative CTCBS_E*
 * code on failure (nothing is thrown, nothing aborts) and ctcbs_step may return the
 * positive CTCBS_DONE.  All device work is enqueued on the stream given at creation; the
 * only host synchronisations are inside ctcbs_create (end), ctcbs_finalize,
 * ctcbs_poll/ctcbs_peek/ctcbs_stats/ctcbs_profile_read; the optional periodic look of
 * ctcbs_step only waits for work enqueued two intervals earlier.
 * A handle is not thread-safe.
 */
#ifndef CTCBS_H
#define CTCBS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ctcbs ctcbs_t; /* opaque, owned by the library */

enum {
  CTCBS_OK = 0,
  CTCBS_DONE = 1,     /* every utterance of the batch has finished                       */
  CTCBS_EINVAL = -1,  /* bad argument or unsupported size (see limits below)             */
  CTCBS_ENOMEM = -2,  /* device or host allocation failed                                */
  CTCBS_EHIP = -3,    /* a HIP runtime call failed; ctcbs_last_hip_error() has the code  */
  CTCBS_ESTATE = -4,  /* call not valid in the handle's state, or (ctcbs_finalize) a kernel's
                         own consistency check failed during the decode: no result          */
  CTCBS_ECAP = -5     /* caller's output capacity too small                              */
};

/* end_flags bits */
enum {
  CTCBS_END_BASELINE = 1,  /* Eq. (4): the last M lengths' best ended hypotheses all lie more
                              than |D_end| below the best ended hypothesis                 */
  CTCBS_END_TAU_COUNT = 2, /* Algorithm 3: more than C ended hypotheses whose start-time
                              index tau equals T_i                                         */
  CTCBS_END_EOS_RUN = 4    /* not in the paper: stop a hypothesis g when, on each of the last
                              eos_run frames t, phi_t(g) exceeds the running prefix score of
                              every candidate extension; applies only if those frames lie in
                              both g's stored range and the current window                 */
};

/*
 * Search configuration (Algorithm 2's inputs plus the constants of Sec. 3.2).
 * Limits: 1 <= beam <= 32; 3 <= vocab; 1 <= t_max <= 6140; end_m <= 8; eos_run <= 32.
 * (With 0 < cand_k < vocab-2 the fast candidate selection needs vocab to be a multiple of 4
 * and at most 6144; other vocabularies take a slower, equivalent path.)
 */
typedef struct {
  int32_t n_utt;        /* U                                                               */
  int32_t t_max;        /* frame pitch of d_ctc_logp (>= every T_i)                        */
  int32_t vocab;        /* V                                                               */
  int32_t beam;         /* Wb, the paper's B                                               */
  int32_t blank_id;     /* CTC blank                                                       */
  int32_t eos_id;       /* <eos>; also the start symbol of Algorithm 2                     */
  int32_t cand_k;       /* CTC-score only the cand_k ids with the largest attention
                           log-prob (blank and eos never count; equal values: smaller id);
                           0 or >= V-2: score all V-2 ids                                  */
  int32_t win_m1;       /* M1 of s = max(tau - M1, l, 1);        < 0: s = l                */
  int32_t win_m2;       /* M2 of e = min(tau~ + M2, T_i);        < 0: e = T_i              */
  float ctc_weight;     /* lambda of Eq. (1)                                               */
  float length_bonus;   /* added once per label (eos included) to the joint score          */
  float max_len_ratio;  /* step cap: min(T_i, floor(ratio*T_i) if ratio > 0,               */
  int32_t max_len_abs;  /*           max_len_abs if > 0), at least 1.  At the cap every
                           live hypothesis is ended and the utterance finishes.            */
  int32_t end_flags;    /* CTCBS_END_* bits                                                */
  int32_t end_m;        /* M of Eq. (4) (paper: 3)                                         */
  float end_d;          /* log-domain D_end of Eq. (4) (paper: -10)                        */
  int32_t end_c;        /* C of Algorithm 3 (paper: 2)                                     */
  int32_t eos_run;      /* frames of the CTCBS_END_EOS_RUN rule (10)                       */
  int32_t poll_every;   /* > 0: every that many steps ctcbs_step looks, without draining the
                           stream, at the count of finished utterances the device has
                           published (it may lag by up to two such intervals) and keeps the
                           host from running further ahead than that; 0: never             */
  int32_t win_union;    /* 0: every hypothesis has its own window (the two equations for s_ij, e_ij);
                           1: one window for the whole batch, s^l = min_ij s_ij, e^l = max_ij
                           e_ij (last two equations of Sec. 3.2.3), cut at each T_i          */
  int32_t att_is_logits; /* 0: ctcbs_step takes log-probabilities p^a; 1: it takes the decoder's
                           unnormalised output scores and applies log_softmax over the V ids of
                           each row itself (folded into the candidate pass; Eq. (2)'s p^a)  */
  int32_t keep_candidates; /* 1: every step also leaves each hypothesis's candidate ids and their
                           prefix / joint scores in device memory for ctcbs_peek (checking and
                           inspection; costs a few per cent of the step's memory traffic);
                           0: they stay on chip and ctcbs_peek of them returns CTCBS_ESTATE.
                           Step outputs and results are the same either way.               */
  void* stream;         /* hipStream_t; NULL = the null stream                             */
} ctcbs_config_t;

/*
 * Views of one step's results.  Device arrays are owned by the library and stay valid
 * (stream-ordered) until the next ctcbs_step or ctcbs_destroy on the handle.
 */
typedef struct {
  int32_t step;             /* l of the step just enqueued                                 */
  int32_t n_finished;       /* finished utterances as last published by the device if this
                               call looked (see poll_every; a lower bound), else -1          */
  const int32_t* d_parent;  /* [U][Wb] old beam slot each new hypothesis extends (GatherB)  */
  const int32_t* d_token;   /* [U][Wb] label appended                                      */
  const float* d_score;     /* [U][Wb] joint score, Eq. (1) (+ length bonus)               */
  const uint8_t* d_live;    /* [U][Wb] 1 = slot holds a hypothesis                         */
  const uint8_t* d_finished;/* [U]     1 = utterance finished at or before this step       */
  const int32_t* d_tau;     /* [U][Wb] start-time index tau of the new hypothesis          */
  const int32_t* d_tau_end; /* [U][Wb] end-time index tau~                                 */
  const uint8_t* d_eos_added; /* [U][Wb] by OLD slot: g.<eos> entered the ended set        */
  const uint8_t* d_stopped;   /* [U][Wb] by OLD slot: stopped by the eos-run rule          */
} ctcbs_step_out_t;

/*
 * Algorithm 2, initialisation: take the batch's CTC log-posteriors
 * d_ctc_logp[u][t][k] = log p^c(z_{t+1} = k | h_u), t < h_lens[u] (device, fp32, row pitch
 * vocab, utterance pitch t_max*vocab; frames at and beyond h_lens[u] are never read), and
 * set every utterance's beam to the single empty hypothesis.  The posteriors are copied
 * (token-major) before the call returns, so the caller may release d_ctc_logp afterwards.
 * 0 <= h_lens[u] <= t_max; a length of 0 marks an unused slot of the batch (a last batch that
 * is not full): it is finished from the start, holds no hypothesis (its d_live flags are 0),
 * none of its rows is read, and ctcbs_finalize reports it with no tokens, score -1e30 and
 * flag 1.  On failure *out is NULL.
 */
int ctcbs_create(const ctcbs_config_t* cfg, const float* d_ctc_logp, const int32_t* h_lens,
                 ctcbs_t** out);

/*
 * Algorithm 2's initialisation again, on an existing handle, for the next batch: same
 * configuration and number of utterances, new posteriors and lengths (each <= t_max).  All
 * device memory is reused, so an offline run allocates once.  Results of the previous batch
 * are gone afterwards.  Synchronises the stream.
 */
int ctcbs_reset(ctcbs_t* h, const float* d_ctc_logp, const int32_t* h_lens);

/*
 * One iteration of Algorithm 2's loop (Score_Fn with Eq. (1)-(3)/(5), eos split-off, TopB,
 * GatherB, the "p > best_score" test, ENDDETECT) for all utterances.
 * d_att_logp[u][j][k] = log p^a(y^l = k | hypothesis in beam slot j of utterance u) (device,
 * fp32, [U][Wb][V], the whole buffer valid device memory); rows of dead slots and finished
 * utterances may be fetched but their contents are never looked at (garbage and NaN are fine).
 * At the first step only slot 0 of each utterance is live.  The buffer must stay valid until
 * the step's work has run on the stream.  Rows that start on 16-byte boundaries (d_att_logp
 * 16-byte aligned and V a multiple of 4) take the fast candidate selection; any other
 * alignment is accepted and takes a slower, equivalent path.  `out` may be NULL.
 * Returns CTCBS_DONE (and enqueues nothing) once the handle knows that all utterances are
 * finished: after a look or ctcbs_poll saw it, or when the step index passes every
 * utterance's cap.  Steps enqueued after the last utterance finished do nothing.
 */
int ctcbs_step(ctcbs_t* h, const float* d_att_logp, ctcbs_step_out_t* out);

/*
 * ctcbs_step for callers that cannot allocate device memory and want a step whose working set
 * beyond the handle's state lies at a fixed place: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same arguments, same kernels, same outputs and return
 * codes as ctcbs_step, bit for bit; the two may be mixed freely on one handle.  The arrays that
 * carry a step's intermediate values from the score kernel to the select kernel (windows, eos
 * scores, the groups' best-first lists, stop flags, work counts) lie in a fixed 4 MiB array inside
 * the library's image (one copy per GPU, held until the process ends) instead of the handle's own
 * memory.  The call allocates nothing, on the host or on the device, and enqueues no memset.
 * Limits: the device the handle was created on must be current (else CTCBS_ESTATE); at most 256
 * candidates per hypothesis and not every id a candidate, and
 * 40*U*Wb + 24*U*Wb*Wb bytes (each array rounded up to 256) within the 4 MiB (else CTCBS_EINVAL:
 * e.g. U = 256 at beam 20 fits, U = 2048 at beam 10 does not).
 * Every call on a GPU uses that GPU's one array, whatever the handle: steps of different handles
 * (or streams) that overlap in time on one GPU race on it.  Callers that keep several batches in
 * flight use ctcbs_step.  ctcbs_peek of windows and eos scores reads the arrays of the handle's
 * last step, wherever they lie; with this call they hold what the GPU's last call left there.
 */
int ctcbs_step_static(ctcbs_t* h, const float* d_att_logp, ctcbs_step_out_t* out);

/* Synchronise and read how many utterances have finished (Algorithm 2's loop exit test). */
int ctcbs_poll(ctcbs_t* h, int32_t* n_finished);

/*
 * Algorithm 2, last line: per utterance the best hypothesis of its ended set (ties: the
 * one added first).  h_tokens[u*cap ..] receives its labels without the start symbol and
 * without <eos>, h_ntok[u] their count, h_score[u] its joint score; h_frames (optional,
 * may be NULL, same layout as h_tokens) receives each label's start-time index tau.
 * h_flags (optional) gets bit 0 set if the ended set was empty and the best live hypothesis
 * was returned instead.  May be called at any time; synchronises the stream.
 */
int ctcbs_finalize(ctcbs_t* h, int32_t* h_tokens, int32_t cap, int32_t* h_ntok, float* h_score,
                   int32_t* h_frames, int32_t* h_flags);

/*
 * Work counters: *cells = sum over steps and live (utterance, beam) groups of
 * K * (e - s + 1), the number of (utt, beam, candidate, frame) prefix-score terms the
 * method defines (Eq. (3)/(5) summands); *groups = live (utterance, beam) groups summed over
 * steps; *steps = steps enqueued so far.  Any pointer may be NULL.  Synchronises.
 */
int ctcbs_stats(ctcbs_t* h, uint64_t* cells, uint64_t* groups, int32_t* steps);

/*
 * Measurement aid.  After ctcbs_profile(h, 1) every ctcbs_step brackets its score kernel
 * and its select kernel with HIP events on the handle's stream; ctcbs_profile_read
 * synchronises and returns the summed durations (milliseconds) of the steps recorded since
 * profiling was enabled, and their count.
 */
int ctcbs_profile(ctcbs_t* h, int32_t enable);
int ctcbs_profile_read(ctcbs_t* h, double* score_ms, double* select_ms, int32_t* n_steps);

/*
 * Inspection of internal arrays of the last step (tests and debugging; synchronises).
 * Copies min(bytes, size of the array) bytes to the host buffer and returns the array's
 * full size in *need (may be NULL).
 */
enum {
  CTCBS_PEEK_CAND_ID = 1,    /* int32  [U][Wb][K] candidate ids (no particular order)       */
  CTCBS_PEEK_CAND_CTC = 2,   /* double [U][Wb][K] log psi(g.c), Eq. (3)/(5)                 */
  CTCBS_PEEK_CAND_JOINT = 3, /* double [U][Wb][K] joint score of g.c                        */
  CTCBS_PEEK_WIN_S = 4,      /* int32  [U][Wb] window start s                               */
  CTCBS_PEEK_WIN_E = 5,      /* int32  [U][Wb] window end e (e < s: empty)                  */
  CTCBS_PEEK_CTC_EOS = 6,    /* double [U][Wb] log phi_T(g)                                 */
  CTCBS_PEEK_JOINT_EOS = 7,  /* double [U][Wb] joint score of g.<eos>                       */
  CTCBS_PEEK_N_CAND = 8      /* int32  [1] K, candidates per group                          */
};
int ctcbs_peek(ctcbs_t* h, int32_t what, void* h_dst, size_t bytes, size_t* need);

/*
 * ---- Offline scheduling around the path (host side; none of these touches a kernel) ----
 *
 * Hard segmentation by length (Sec. 3.3, second method; Sec. 4.4): cut a recording of
 * n_frames frames into the fewest pieces no longer than max_len, with lengths as uniform as
 * possible, the last piece included (they differ by at most one frame, longer ones first).
 * Every piece is also >= min_len whenever n_frames allows it (always once n_frames >=
 * min_len * max_len / (max_len - min_len)); a shorter recording still gets uniform pieces.
 * h_len[0..*n_seg) receives the lengths in order.  CTCBS_ECAP (with *n_seg set) if cap is
 * too small or h_len is NULL.
 */
int ctcbs_hard_segments(int64_t n_frames, int32_t min_len, int32_t max_len, int32_t* h_len,
                        int32_t cap, int32_t* n_seg);

/*
 * Segments from voice-activity pieces (Sec. 4.4, first method; the detector itself is outside):
 * consecutive pieces (lengths h_piece_len[0..n_pieces), in time order) are merged until a
 * segment is at least min_len long; a segment longer than max_len is split again, uniformly,
 * into the fewest parts that fit; what is left at the end stays a segment of its own.
 * Output as for ctcbs_hard_segments.
 */
int ctcbs_merge_pieces(const int32_t* h_piece_len, int32_t n_pieces, int32_t min_len, int32_t max_len,
                       int32_t* h_len, int32_t cap, int32_t* n_seg);

/*
 * Length-sorted batching (Sec. 4.2: segments are ordered by length so that a batch holds
 * segments of similar length).  h_order[0..n) receives the segment indices longest first
 * (equal lengths in input order); batch b is h_order[h_begin[b] .. h_begin[b+1]): at most
 * max_utt segments and, if max_padded_frames > 0, at most that many frames after padding every
 * segment of the batch to its longest (= first) one.  h_begin needs cap_batches + 1 entries;
 * with h_begin NULL or too small the call only counts (*n_batches) and returns CTCBS_ECAP.
 */
int ctcbs_plan_batches(const int32_t* h_len, int32_t n, int32_t max_utt, int64_t max_padded_frames,
                       int32_t* h_order, int32_t* h_begin, int32_t cap_batches, int32_t* n_batches);

/*
 * Where the attention rows of a step come from: called before every ctcbs_step of batch
 * `index` with the 1-based step about to run and the previous step's views (NULL before the
 * first), it must set *d_att to the [U][Wb][V] device rows for that step -- typically after
 * enqueuing the decoder on the batch's stream -- and return 0, or a negative code to abort.
 * With more than one thread in ctcbs_run_many it is called concurrently for different batches.
 */
typedef int (*ctcbs_att_fn)(void* user, int32_t index, int32_t step, const ctcbs_step_out_t* prev,
                            const float** d_att);

/*
 * Decode n batches at once: handle hs[i] (created on a stream of its own for the kernels of
 * different batches to overlap) is stepped until it reports CTCBS_DONE; n_threads host threads
 * (the caller's included) share the batches, each stepping its own round-robin.  One batch of
 * 64 utterances leaves most of the chip idle through its dependent phases; a few batches in
 * flight fill it.  Results are read with ctcbs_finalize afterwards.  Returns the first error.
 */
int ctcbs_run_many(ctcbs_t* const* hs, int32_t n, ctcbs_att_fn fn, void* user, int32_t n_threads);

/* A ready-made ctcbs_att_fn that replays recorded inputs: user = ctcbs_replay_t[n], entry i
 * listing the device rows of batch i step by step (steps past n_steps get the last rows). */
typedef struct {
  const float* const* d_att;  /* [n_steps] device pointers, each [U][Wb][V]                    */
  int32_t n_steps;
} ctcbs_replay_t;
int ctcbs_att_replay(void* user, int32_t index, int32_t step, const ctcbs_step_out_t* prev,
                     const float** d_att);

/*
 * Decode a queue of n_jobs batches on n_slots handles (n_slots batches in flight).  Whenever a
 * handle is free the next job is taken: job_fn(user, job, slot, h, CTCBS_JOB_LOAD) must make
 * h ready for it (ctcbs_reset with that batch's posteriors); the batch is then stepped, with
 * att_fn called with index = job, until it reports CTCBS_DONE, and
 * job_fn(..., CTCBS_JOB_DONE) collects its result (ctcbs_finalize).  n_threads host threads
 * (the caller's included) share the slots; the callbacks run on those threads, concurrently
 * for different slots.  All handles must accept every job (same configuration, t_max and
 * n_utt large enough).  Returns the first error (callbacks return 0 or a negative code).
 */
enum { CTCBS_JOB_LOAD = 0, CTCBS_JOB_DONE = 1 };
typedef int (*ctcbs_job_fn)(void* user, int32_t job, int32_t slot, ctcbs_t* h, int32_t phase);
int ctcbs_run_queue(ctcbs_t* const* hs, int32_t n_slots, int32_t n_jobs, ctcbs_job_fn job_fn,
                    ctcbs_att_fn att_fn, void* user, int32_t n_threads);

void ctcbs_destroy(ctcbs_t* h);

const char* ctcbs_strerror(int code);
int ctcbs_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* CTCBS_H */
