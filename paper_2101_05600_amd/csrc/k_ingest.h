// Batch ingest: Algorithm 2's initialisation on the device.
#pragma once
#include "common.h"

// CTC log-posteriors [U][t_max][V] (frame-major, as an encoder emits them) -> token-major
// xT[u][k][t], t = 1..T_u, so that one candidate's frames are contiguous.  A work-group moves a
// tile of 256 tokens x 32 stored frames through LDS: 1 KB contiguous per frame on the way in
// (float4 per lane when rows are 16-byte aligned: VEC), whole aligned 128-byte lines per token on
// the way out (rows of xT start on line boundaries, and the tile is cut in STORED frame indices,
// which are one more than the 0-based input frame).  Frames at and beyond T_u are never read.
// Index 0 and the entries after T_u up to the end of their tile (at least four) are set to zero:
// aligned float4 loads of a window may touch them (their terms are masked through the f array,
// which needs finite values there).  Work-groups go round-robin over the eight XCDs; tiles are
// numbered so that each XCD walks through one contiguous eighth of the utterance's tiles, token
// tiles of a 32-frame band one after the other: the lines two neighbouring tiles share are then
// fetched into one L2 instead of two, and each XCD streams through its own region of memory.
// Which eighth an XCD takes rotates with the utterance, so that short utterances (whose last
// eighths are empty) do not leave the same XCDs idle.
template <bool VEC>
__global__ __launch_bounds__(256) void k_transpose(Params p, const float* __restrict__ x, int nvt, int n_tiles,
                                                   int per_xcd) {
  __shared__ __attribute__((aligned(16))) float tile[32][260];
  const int u = blockIdx.y;
  const int T = p.lens[u];
  const int g = (((int)blockIdx.x - u) & 7) * per_xcd + (blockIdx.x >> 3);
  if (g >= n_tiles) return;
  const int jt = g / nvt, vt = g - jt * nvt;
  const int d0 = jt * 32;                                // first stored frame index of the tile
  if (d0 > T + 4) return;
  const int v0 = vt * 256;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const float* src = x + (size_t)u * p.t_max * p.V;
  float4 r[8];
  const int v = v0 + 4 * lane;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int tt = d0 - 1 + w * 8 + i;                   // 0-based input frame of stored index tt + 1
    r[i] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    if (tt >= 0 && tt < T) {
      const float* row = src + (size_t)tt * p.V + v;
      if (VEC) {
        if (v < p.V) r[i] = *(const float4*)row;         // V is a multiple of 4 here
      } else {
        if (v + 0 < p.V) r[i].x = row[0];
        if (v + 1 < p.V) r[i].y = row[1];
        if (v + 2 < p.V) r[i].z = row[2];
        if (v + 3 < p.V) r[i].w = row[3];
      }
    }
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    float4 c;
    c.x = fmaxf(r[i].x, LOG0F); c.y = fmaxf(r[i].y, LOG0F); c.z = fmaxf(r[i].z, LOG0F); c.w = fmaxf(r[i].w, LOG0F);
    const int t = w * 8 + i;
    *(float4*)&tile[t][(4 * lane) ^ (((t >> 3) & 3) << 2)] = c;   // (swizzle: see the reads below)
  }
  __syncthreads();
  float* dst = p.xT + (size_t)u * p.V * p.Tp;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int q = i * 256 + threadIdx.x;
    const int vl = q >> 3, t4 = (q & 7) * 4;             // eight lanes cover one token's 32 frames
    // a wave reads 8 tokens x 8 groups of 4 frames; with rows of 260 floats, frames 8 apart would
    // share banks, so each band of 8 rows keeps its float4 columns in a different order: the lanes
    // of a wave (of a half wave too) fall on distinct banks
    const int vs = vl ^ ((t4 >> 3) << 2);
    const int d = d0 + t4;
    if (v0 + vl < p.V && d < p.Tp) {                     // Tp is a multiple of 4
      float4 o;
      o.x = (d + 0 >= 1 && d + 0 <= T) ? tile[t4 + 0][vs] : 0.0f;
      o.y = (d + 1 <= T) ? tile[t4 + 1][vs] : 0.0f;
      o.z = (d + 2 <= T) ? tile[t4 + 2][vs] : 0.0f;
      o.w = (d + 3 <= T) ? tile[t4 + 3][vs] : 0.0f;
      *(float4*)(dst + (size_t)(v0 + vl) * p.Tp + d) = o;
    }
  }
}

// Per-frame reference and empty-prefix state.  z_0 = blank (first alignment rule of Sec. 2.1), so
// the blank variable of the empty hypothesis at frame t is the running sum of the blank
// log-posteriors and the label variable is log0.  That running sum (fp64, each term floored at
// BLANK_FLOOR) is also the reference B_t every stored forward variable is taken relative to: the
// empty hypothesis's stored blank variable is therefore 0 at every frame (minus whatever the
// floor cut off: log0 from the first frame on whose blank probability is zero).
// One wave per utterance.  An utterance of no frames is an unused slot of the batch: it counts as
// finished from the start (n_empty of them, counted by the host), holds no hypothesis and takes
// part in nothing.
__global__ __launch_bounds__(64) void k_init_state(Params p, int n_empty) {
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
    HypRec r;
    r.live = (j == 0 && T > 0); r.last = -1; r.rs = 0; r.re = T; r.tau = 0; r.tau_end = 0; r.ref = 0; r.pad = 0;
    r.off = 0.0; r.att = 0.0; r.joint = 0.0; r.bref = 0.0;
    p.rec[0][h] = r;
    // the other buffer: dead until the first selection fills it, but never left holding what the
    // allocation happened to contain (a kernel may load a dead slot's record before it looks at its flag)
    r.live = 0;
    p.rec[1][h] = r;
    p.out_live[h] = (j == 0 && T > 0); p.out_parent[h] = 0; p.out_token[h] = -1; p.out_score[h] = 0.0f;
    p.out_tau[h] = 0; p.out_tau_end[h] = 0; p.out_eos_added[h] = 0; p.out_stopped[h] = 0;
    p.trie_parent[h] = 0; p.trie_token[h] = -1; p.trie_tau[h] = 0;   // level 0: the empty hypothesis
  }
  if (lane == 0) {
    UttInfo ui;
    ui.T = T; ui.lmax = p.lmax[u]; ui.BT = carry;          // (B_T: the running sum after the last frame; 0 for T = 0)
    p.uinfo[u] = ui;
    UttState s;
    s.best_score = LOG0D; s.fb_score = LOG0D;
    for (int i = 0; i < MAX_END_M; ++i) { s.ring_score[i] = LOG0D; s.ring_tag[i] = -1; }
    s.n_ended = 0; s.best_step = 0; s.best_slot = 0; s.cnt_tau_T = 0; s.finished_step = T > 0 ? 0 : -1; s.pad = 0;
    p.utt[u] = s;
    p.finished[u] = T > 0 ? 0 : 1;
    p.cells[u] = 0ull;
    p.groups[u] = 0ull;
    if (u == 0) *p.n_finished = n_empty;
  }
}
