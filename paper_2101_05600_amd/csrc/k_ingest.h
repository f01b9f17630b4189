// Batch ingest: Algorithm 2's initialisation on the device.
#pragma once
#include "common.h"

// CTC log-posteriors [U][t_max][V] (frame-major, as an encoder emits them) -> token-major
// xT[u][k][t], t = 1..T_u, so that one candidate's frames are contiguous.  64x64 tiles
// through LDS; frames at and beyond T_u are never read.  Index 0 and the four entries after
// T_u are set to zero: aligned float4 loads of a window may touch them (their terms are
// masked through the f array, which needs finite values there).
__global__ __launch_bounds__(256) void k_transpose(Params p, const float* __restrict__ x) {
  __shared__ float tile[64][65];
  const int u = blockIdx.z;
  const int T = p.lens[u];
  const int t0 = blockIdx.y * 64, v0 = blockIdx.x * 64;
  if (t0 >= T + 4) return;
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  const float* src = x + (size_t)u * p.t_max * p.V;
#pragma unroll 4
  for (int i = 0; i < 16; ++i) {
    int tt = t0 + ty * 16 + i, vv = v0 + tx;
    tile[ty * 16 + i][tx] = (tt < T && vv < p.V) ? fmaxf(src[(size_t)tt * p.V + vv], LOG0F) : 0.0f;
  }
  __syncthreads();
  float* dst = p.xT + (size_t)u * p.V * p.Tp;
#pragma unroll 4
  for (int i = 0; i < 16; ++i) {
    int vv = v0 + ty * 16 + i, tt = t0 + tx;
    if (vv < p.V) {
      if (tt < T) dst[(size_t)vv * p.Tp + tt + 1] = tile[tx][ty * 16 + i];
      else if (tt < T + 4) dst[(size_t)vv * p.Tp + tt + 1] = 0.0f;
      if (tt == 0) dst[(size_t)vv * p.Tp] = 0.0f;
    }
  }
}

// Per-frame reference and empty-prefix state.  z_0 = blank (first alignment rule of Sec. 2.1), so
// the blank variable of the empty hypothesis at frame t is the running sum of the blank
// log-posteriors and the label variable is log0.  That running sum (fp64, each term floored at
// BLANK_FLOOR) is also the reference B_t every stored forward variable is taken relative to: the
// empty hypothesis's stored blank variable is therefore 0 at every frame (minus whatever the
// floor cut off: log0 from the first frame on whose blank probability is zero).
// One wave per utterance.
__global__ __launch_bounds__(64) void k_init_state(Params p) {
  const int u = blockIdx.x, lane = threadIdx.x;
  const int T = p.lens[u];
  const size_t hyp0 = (size_t)u * p.Wb;
  float* gn = p.gn[0] + hyp0 * p.Tp;
  float* gb = p.gb[0] + hyp0 * p.Tp;
  double* Bu = p.Bcum + (size_t)u * p.Tp;
  const float* xb = p.xT + ((size_t)u * p.V + p.blank_id) * p.Tp;
  double carry = 0.0, carry_cut = 0.0;
  if (lane == 0) { gn[0] = LOG0F; gb[0] = 0.0f; Bu[0] = 0.0; }
  for (int base = 1; base <= T; base += 64) {
    int t = base + lane;
    const float x0 = (t <= T) ? xb[t] : 0.0f;
    double v = (double)fmaxf(x0, BLANK_FLOOR);           // floored term of B_t
    double c = (double)x0 - v;                            // what the floor cut off (0 or negative)
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      double n = __shfl_up(v, o), nc = __shfl_up(c, o);
      if (lane >= o) { v += n; c += nc; }
    }
    v += carry; c += carry_cut;
    if (t <= T) { Bu[t] = v; gb[t] = fmaxf((float)c, LOG0F); gn[t] = LOG0F; }
    carry = __shfl(v, 63); carry_cut = __shfl(c, 63);
  }
  for (int t = T + 1 + lane; t < p.Tp; t += 64) Bu[t] = carry;   // (never weighted: keeps reads defined)
  for (int j = lane; j < p.Wb; j += 64) {
    size_t h = hyp0 + j;
    p.h_live[0][h] = (j == 0); p.h_last[0][h] = -1;
    p.h_rs[0][h] = 0; p.h_re[0][h] = T; p.h_tau[0][h] = 0; p.h_tau_end[0][h] = 0; p.h_ref[0][h] = 0;
    p.h_off[0][h] = 0.0; p.h_att[0][h] = 0.0; p.h_joint[0][h] = 0.0;
    p.h_live[1][h] = 0;
    p.out_live[h] = (j == 0); p.out_parent[h] = 0; p.out_token[h] = -1; p.out_score[h] = 0.0f;
    p.out_tau[h] = 0; p.out_tau_end[h] = 0; p.out_eos_added[h] = 0; p.out_stopped[h] = 0;
    p.trie_parent[h] = 0; p.trie_token[h] = -1; p.trie_tau[h] = 0;   // level 0: the empty hypothesis
  }
  if (lane == 0) {
    UttState s;
    s.best_score = LOG0D; s.fb_score = LOG0D;
    for (int i = 0; i < MAX_END_M; ++i) { s.ring_score[i] = LOG0D; s.ring_tag[i] = -1; }
    s.n_ended = 0; s.best_step = 0; s.best_slot = 0; s.cnt_tau_T = 0; s.finished_step = 0; s.pad = 0;
    p.utt[u] = s;
    p.finished[u] = 0;
    p.cells[u] = 0ull;
    p.groups[u] = 0ull;
    if (u == 0) *p.n_finished = 0;
  }
}
