// Result extraction: Algorithm 2's last line.  One thread per utterance walks the
// back-pointer trie from the best ended hypothesis (or, if nothing has ended yet, from the
// best live hypothesis) and writes its labels and their start-time indices.
#pragma once
#include "common.h"

__global__ void k_finalize(Params p, int cur, int steps_done, int cap, int32_t* tokens, int32_t* frames,
                           int32_t* ntok, float* score, int32_t* flags) {
  const int u = blockIdx.x * blockDim.x + threadIdx.x;
  if (u >= p.U) return;
  const UttState st = p.utt[u];
  int level, slot, flag = 0;
  double sc;
  if (st.n_ended > 0) {
    level = st.best_step - 1; slot = st.best_slot; sc = st.best_score;
  } else {
    flag = 1;
    // beam of the last step this utterance took part in; slot 0 is its best hypothesis
    const size_t h = (size_t)u * p.Wb;
    if (!st.finished_step && p.h_live[cur][h]) { level = steps_done; slot = 0; sc = p.h_joint[cur][h]; }
    else { level = 0; slot = 0; sc = LOG0D; }
  }
  flags[u] = flag;
  score[u] = (float)sc;
  if (level > cap) { ntok[u] = -level; return; }      // capacity error, reported by the host
  ntok[u] = level;
  for (int k = level; k >= 1; --k) {
    const size_t idx = ((size_t)k * p.U + u) * p.Wb + slot;
    tokens[(size_t)u * cap + k - 1] = p.trie_token[idx];
    frames[(size_t)u * cap + k - 1] = p.trie_tau[idx];
    slot = p.trie_parent[idx];
  }
}
