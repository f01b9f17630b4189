// Result extraction: Algorithm 2's last line.  One work-group per utterance: the best ended
// hypothesis (or, if nothing has ended yet, the best live hypothesis) is traced back through
// the back-pointer trie.  The utterance's parent pointers are first staged in LDS (one byte
// each, loaded by all threads at once) so that the serial walk never waits on global memory;
// the labels and their start-time indices are then gathered by all threads in parallel.
#pragma once
#include "common.h"

template <int BLOCK>
__global__ __launch_bounds__(BLOCK) void k_finalize(Params p, int cur, int steps_done, int cap, int use_lds,
                                                    int32_t* tokens, int32_t* frames, int32_t* ntok,
                                                    float* score, int32_t* flags) {
  extern __shared__ unsigned char fsm[];
  __shared__ int s_level, s_slot0;
  const int u = blockIdx.x, tid = threadIdx.x, Wb = p.Wb;
  if (tid == 0) {
    const UttState st = p.utt[u];
    int level, slot, flag = 0;
    double sc;
    if (st.n_ended > 0) {
      level = checked(p, st.best_step - 1, 0, steps_done, ERR_BACKTRACK); slot = st.best_slot; sc = st.best_score;
    } else {
      flag = 1;
      // beam of the last step this utterance took part in; slot 0 is its best hypothesis
      const size_t h = (size_t)u * Wb;
      if (!st.finished_step && p.rec[cur][h].live) { level = steps_done; slot = 0; sc = p.rec[cur][h].joint; }
      else { level = 0; slot = 0; sc = LOG0D; }
    }
    flags[u] = flag;
    score[u] = (float)sc;
    ntok[u] = level > cap ? -level : level;             // negative: capacity error, reported by the host
    s_level = level > cap ? 0 : level; s_slot0 = slot;
  }
  __syncthreads();
  const int level = s_level;
  if (level == 0) return;
  if (use_lds) {
    unsigned char* s_par = fsm;                          // [level + 1][Wb]
    unsigned char* s_path = fsm + (size_t)(p.l_cap + 1) * Wb;   // slot on the path at each level
    for (int i = tid; i < level * Wb; i += BLOCK) {
      const int k = 1 + i / Wb, j = i % Wb;
      s_par[k * Wb + j] = (unsigned char)p.trie_parent[((size_t)k * p.U + u) * Wb + j];
    }
    __syncthreads();
    if (tid == 0) {
      int slot = s_slot0;
      for (int k = level; k >= 1; --k) {
        if (slot >= Wb) { atomicOr(p.err, ERR_BACKTRACK); slot = 0; }   // (a dead slot on the path: -1 read back as 255)
        s_path[k] = (unsigned char)slot; slot = s_par[k * Wb + slot];
      }
    }
    __syncthreads();
    for (int k = 1 + tid; k <= level; k += BLOCK) {
      const size_t idx = ((size_t)k * p.U + u) * Wb + s_path[k];
      tokens[(size_t)u * cap + k - 1] = p.trie_token[idx];
      frames[(size_t)u * cap + k - 1] = p.trie_tau[idx];
    }
  } else if (tid == 0) {
    int slot = s_slot0;
    for (int k = level; k >= 1; --k) {
      slot = checked(p, slot, 0, Wb - 1, ERR_BACKTRACK);
      const size_t idx = ((size_t)k * p.U + u) * Wb + slot;
      tokens[(size_t)u * cap + k - 1] = p.trie_token[idx];
      frames[(size_t)u * cap + k - 1] = p.trie_tau[idx];
      slot = p.trie_parent[idx];
    }
  }
}
