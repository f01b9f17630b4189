// Shared device-side definitions of the ctcbs kernels (gfx950, wave64).
//
// Numeric form.  Every hypothesis g keeps its two CTC forward variables (paths ending in
// its last label / ending in blank; their log-sum is the paper's phi_t(g) of Eq. (3)) as
// fp32 values in a STORED form: gamma_t(g) = stored_t + B_t + off'(g), with B_t the
// utterance's cumulative blank log-posterior (fp64, Params::Bcum) and off'(g) an fp64 offset
// per hypothesis (HypRec::off).  Staying in blank leaves the stored value unchanged, so stored
// values are O(1) near the frames that matter however long the utterance is and however
// negative the cumulative score has become; the parts that grow (B_t, off') and the cumulative
// CTC, attention and joint scores are fp64, one add per hypothesis and step.
// log0 is the finite sentinel -1e30 (anything below -1e29 is treated as log0).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#define CTCBS_WAVE 64
#define LOG0F (-1.0e30f)
#define LOG0_CLASS (-1.0e29f)
#define LOG0D (-1.0e30)
// Blank log-posteriors enter the per-frame reference B_t (see Params::Bcum) floored at this value, so
// that B_t stays finite even if a frame gives blank probability zero.
#define BLANK_FLOOR (-1.0e4f)
#define MAX_BEAM 32
#define MAX_END_M 8
#define MAX_EOS_RUN 32

// Phase time stamps for kernel tuning; compiled in only with -DCTCBS_TRACE (never in the
// shipped library).  TRACE_POINT stores at once (cheap to place, but the store is then waited
// for by the next wait on the memory counter); TRACE_MARK keeps the stamp in registers and
// TRACE_FLUSH stores them all at the end of the kernel, which leaves the timing undisturbed.
#ifdef CTCBS_TRACE
#define TRACE_POINT(p, blk, i) do { if ((p).trace && threadIdx.x == 0) (p).trace[(size_t)(blk) * 16 + (i)] = wall_clock64(); } while (0)
#define TRACE_DECL unsigned long long tr_[16] = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0}
#define TRACE_MARK(i) do { tr_[i] = wall_clock64(); } while (0)
#define TRACE_MARK_AT(ptr, i) do { (ptr)[i] = wall_clock64(); } while (0)
#define TRACE_ARG tr_
#define TRACE_FLUSH(p, blk) do { if ((p).trace && threadIdx.x == 0) { _Pragma("unroll") for (int i_ = 0; i_ < 16; ++i_) if (tr_[i_]) (p).trace[(size_t)(blk) * 16 + i_] = tr_[i_]; } } while (0)
#else
#define TRACE_POINT(p, blk, i) do { } while (0)
#define TRACE_DECL do { } while (0)
#define TRACE_MARK(i) do { } while (0)
#define TRACE_MARK_AT(ptr, i) do { } while (0)
#define TRACE_ARG nullptr
#define TRACE_FLUSH(p, blk) do { } while (0)
#endif

struct UttState {            // per utterance, touched by one thread of the select kernel
  double best_score;         // best joint score in the ended set
  double ring_score[MAX_END_M];  // best ended score per length, lengths l, l-1, ... (ring by l % M)
  double fb_score;
  int32_t ring_tag[MAX_END_M];
  int32_t n_ended, best_step, best_slot, cnt_tau_T;
  int32_t finished_step;     // 0 while running
  int32_t pad;
};

// One hypothesis of the current beam: a 64-byte line, so that a work-group fetches the whole
// record of its hypothesis with one uniform (scalar-path) load.
struct __align__(64) HypRec {
  int32_t live;              // slot holds a hypothesis
  int32_t last;              // its last label (-1: the empty hypothesis)
  int32_t rs, re;            // stored range of its forward variables (log0 outside)
  int32_t tau, tau_end;      // first argmax of the label / blank variable (the two argmax equations of Sec. 3.2.2)
  int32_t ref;               // reference frame r: prefix-score increments are relative to off' + B_r
  int32_t pad;
  double off;                // off'(g): log psi(g) = off'(g) + B_r(g) up to the rounding of the re-basing
  double att;                // cumulative attention log-prob, Eq. (2)
  double joint;              // joint score of the hypothesis, Eq. (1)
  double bref;               // B_r (copied from Bcum so that no load depends on `ref`)
};

struct UttInfo {             // per utterance, constant over a decode
  int32_t T, lmax;           // frames, step cap
  double BT;                 // B_T
};

struct Params {
  // sizes and configuration
  int32_t U, V, Wb, K, Tp, t_max, blank_id, eos_id;
  int32_t restricted;        // 1: top-K attention candidates; 0: every id but blank/eos
  int32_t att_logits;        // 1: the step input holds unnormalised logits (log_softmax folded in)
  int32_t win_union;         // 1: one window for the whole batch (min start / max end over all hypotheses)
  int32_t win_m1, win_m2, end_flags, end_m, end_c, eos_run, l_cap;
  float end_d;
  double lambda, beta;
  // posteriors, token-major: xT[(u*V + k)*Tp + t] = log p^c(z_t = k), t = 1..T_u; 0 elsewhere
  float* xT;
  const int32_t* lens;       // [U]
  const int32_t* lmax;       // [U] step cap per utterance
  // Cumulative blank log-posterior per utterance, fp64: Bcum[u*Tp + t] = sum_{v<=t} max(x_v(blank),
  // BLANK_FLOOR), Bcum[u*Tp] = 0.  Forward variables are stored with B_t taken out: for a hypothesis
  // g with offset off'(g), gamma_t(g) = stored_t + B_t + off'(g).  On the path that stays in blank the
  // stored value does not change from frame to frame, so stored values stay within tens of nats of
  // zero however long the utterance is, and the large part (B_t) is carried in fp64.
  double* Bcum;
  UttInfo* uinfo;            // [U]
  // hypothesis state, two buffers (index b): forward variables [b][U][Wb][Tp] (stored form) and
  // per-hypothesis records [b][U][Wb]
  float* gn[2];
  float* gb[2];
  HypRec* rec[2];
  int32_t keep_cand;         // 1: the per-candidate arrays below are filled every step (ctcbs_peek; large K needs them)
  // per-step scratch between the score and the select kernel
  int32_t* win_s;            // [U][Wb]
  int32_t* win_e;
  int32_t* cand_id;          // [U][Wb][K]
  float* cand_inc;           // [U][Wb][K] log psi(g.c) - off(g)
  float* cand_att;           // [U][Wb][K] this step's attention log-prob of c
  float* cand_pre;           // [U][Wb][K] scratch of the eos-run rule
  double* cand_ctc;          // [U][Wb][K] log psi(g.c)
  double* cand_joint;        // [U][Wb][K]
  int32_t* grp_n;            // [U][Wb] entries of the group's sorted list
  // the group's best-first list, [U][Wb][Wb]: joint score, candidate index, token,
  // prefix-score increment, this step's attention log-prob
  double* grp_J;
  int32_t* grp_ci;
  int32_t* grp_tok;
  float* grp_inc;
  float* grp_att;
  double* ctc_eos;           // [U][Wb]
  double* joint_eos;         // [U][Wb]
  int32_t* stopped;          // [U][Wb] eos-run rule fired
  long long* grp_cells;      // [U][Wb]
  // utterance state
  UttState* utt;             // [U]
  uint8_t* finished;         // [U]
  unsigned long long* cells; // [U] prefix-score terms so far
  unsigned long long* groups;// [U] live (utterance, beam) groups so far
  int32_t* n_finished;       // [1]
  int32_t* err;              // [1] bits set by the kernels' own consistency checks (0: none failed)
  int32_t* union_win;        // [2][2] per step parity: (min tau, max of min(tau~ + M2, T)) over live hypotheses
  int32_t* host_finished;    // [1] host-resident copy (device-mapped pinned memory), one step behind
  // back-pointer trie, level l holds the hypotheses of length l: [l_cap+1][U][Wb]
  int32_t* trie_parent;
  int32_t* trie_token;
  int32_t* trie_tau;
  // step outputs
  int32_t* out_parent;
  int32_t* out_token;
  float* out_score;
  uint8_t* out_live;
  int32_t* out_tau;
  int32_t* out_tau_end;
  uint8_t* out_eos_added;
  uint8_t* out_stopped;
  unsigned long long* trace; // [max(U*Wb, U)][16] per-block phase time stamps (tuning builds only)
};

// natural logarithm of a normal positive number: the hardware's log2 times ln 2 (about 1.5 ulp; the
// library's logf spends a dozen instructions more on denormal arguments and the last half ulp)
__device__ __forceinline__ float fast_logf(float x) { return __builtin_amdgcn_logf(x) * 0.69314718055994531f; }

__device__ __forceinline__ float lae(float a, float b) {
  // log(e^a + e^b); with both operands at the log0 sentinel the result stays in the log0 class
  float m = fmaxf(a, b);
  float d = -fabsf(a - b);
  return m + fast_logf(1.0f + __expf(d));
}

// Work-group barrier for data exchanged through LDS only.  __syncthreads() also waits for the
// wave's outstanding global loads and stores (they share one counter with nothing to tell them
// apart); here they stay in flight: prefetched rows and columns keep arriving, and stores of
// results nobody in this work-group reads back are not waited for.  Never use it to publish
// global memory to other waves of the block.
__device__ __forceinline__ void lds_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// Between LDS stores of some lanes of a wave and LDS loads of the same addresses by other lanes of that
// wave.  The hardware needs nothing here (a wave's LDS instructions execute in order, all lanes of an
// instruction together); the call keeps the compiler from moving LDS accesses across this point and gives
// a CPU build of the kernels, where lanes are threads, its synchronisation point.
__device__ __forceinline__ void wave_lds_fence() { __builtin_amdgcn_wave_barrier(); }

// Consistency checks on indices that come from device data (candidate ids, list entries, time
// indices): a value outside its range is clamped into it, so that no access leaves its array, and
// the step's error bit is set; ctcbs_finalize then reports CTCBS_ESTATE instead of a result.
enum { ERR_CAND_ID = 1, ERR_WINDOW = 2, ERR_LIST_ENTRY = 4, ERR_TOKEN = 8, ERR_TIME_INDEX = 16, ERR_BACKTRACK = 32 };
__device__ __forceinline__ int checked(const Params& p, int v, int lo, int hi, int bit) {
  if (v < lo || v > hi) { atomicOr(p.err, bit); v = v < lo ? lo : hi; }
  return v;
}

__device__ __forceinline__ float canon0(float v) { return v < LOG0_CLASS ? LOG0F : v; }

// ---- wave64 data movement through DPP (no LDS round trip) -----------------------------------
// row_shr:n = 0x110+n and row_ror:n = 0x120+n act inside each row of 16 lanes; row_bcast:15
// (0x142) / row_bcast:31 (0x143) copy the last lane of a row / of the lower half-wave into
// the following row(s); wave_shr:1 = 0x138.  Lanes without a source keep `old`.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ int dpp_i(int old, int src) {
  return __builtin_amdgcn_update_dpp(old, src, CTRL, ROW_MASK, 0xf, false);
}
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_f(float old, float src) {
  return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(old), __float_as_int(src), CTRL, ROW_MASK,
                                                    0xf, false));
}

// all-reduce inside each row of 16 lanes (commutative op through rotations)
// (a rotation gives every lane a source, so there is no old value to keep: the move can then be folded
// into the instruction that consumes it)
template <int CTRL>
__device__ __forceinline__ float rot_f(float src) {
  return __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(src), CTRL, 0xf, 0xf, true));
}
__device__ __forceinline__ float row16_max(float v) {
  v = fmaxf(v, rot_f<0x128>(v));
  v = fmaxf(v, rot_f<0x124>(v));
  v = fmaxf(v, rot_f<0x122>(v));
  v = fmaxf(v, rot_f<0x121>(v));
  return v;
}
__device__ __forceinline__ float row16_sum(float v) {
  v += rot_f<0x128>(v);
  v += rot_f<0x124>(v);
  v += rot_f<0x122>(v);
  v += rot_f<0x121>(v);
  return v;
}
__device__ __forceinline__ float lane_f(float v, int lane) {
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), lane));
}
// inclusive prefix sum over the 64 lanes
__device__ __forceinline__ uint32_t wave_incl_scan_u32(uint32_t x, int /*lane*/) {
  int v = (int)x;
  v += dpp_i<0x111, 0xf>(0, v);
  v += dpp_i<0x112, 0xf>(0, v);
  v += dpp_i<0x114, 0xf>(0, v);
  v += dpp_i<0x118, 0xf>(0, v);
  v += dpp_i<0x142, 0xa>(0, v);
  v += dpp_i<0x143, 0xc>(0, v);
  return (uint32_t)v;
}

// Exclusive prefix sum of one uint32 per thread over the block; *total = block sum.
// scratch: one uint32 per wave (+1).  Contains two barriers.
template <int BLOCK>
__device__ __forceinline__ uint32_t block_excl_scan_u32(uint32_t v, uint32_t* scratch, uint32_t* total) {
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  constexpr int NW = BLOCK / 64;
  uint32_t inc = wave_incl_scan_u32(v, lane);
  __syncthreads();                    // scratch may still be read from a previous use
  if (lane == 63) scratch[w] = inc;
  __syncthreads();
  uint32_t base = 0, tot = 0;
#pragma unroll
  for (int i = 0; i < NW; ++i) {
    uint32_t s = scratch[i];
    if (i < w) base += s;
    tot += s;
  }
  *total = tot;
  return base + inc - v;
}

// Order-preserving map of an attention log-prob to uint32 (larger value -> larger key).
// Excluded ids get key 0, NaN gets key 1: both sort below every number, -inf included.
__device__ __forceinline__ uint32_t att_key(float v, int id, int blank_id, int eos_id) {
  if (id == blank_id || id == eos_id) return 0u;
  if (v != v) return 1u;
  uint32_t u = __float_as_uint(v);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// k-th candidate id when every id except blank and eos is a candidate (ascending ids).
__device__ __forceinline__ int full_v_id(int i, int lo_ex, int hi_ex) {
  int id = i;
  if (id >= lo_ex) ++id;
  if (id >= hi_ex) ++id;
  return id;
}
