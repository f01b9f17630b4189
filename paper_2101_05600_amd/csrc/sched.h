// Offline scheduling around the decoding path: the host-side half of the paper's throughput
// recipe.  Long recordings are cut into segments (hard segmentation by length, or merged
// voice-activity pieces; Sec. 3.3 and Sec. 4.4), the segments are sorted by length so that a
// batch holds segments of similar length (Sec. 4.2), and several batches are decoded at once,
// each on its own handle and stream, driven by a few host threads.
// Host code only; included by ctcbs.hip (it needs the handle's fields).
#pragma once
#include <algorithm>
#include <atomic>
#include <thread>

extern "C" int ctcbs_hard_segments(int64_t n_frames, int32_t min_len, int32_t max_len, int32_t* h_len,
                                   int32_t cap, int32_t* n_seg) {
  if (n_frames < 0 || min_len < 1 || max_len < min_len || !n_seg) return CTCBS_EINVAL;
  if (n_frames == 0) { *n_seg = 0; return CTCBS_OK; }
  // fewest pieces that respect max_len; their lengths then differ by at most one frame
  const int64_t n = (n_frames + max_len - 1) / max_len;
  if (n > 0x7fffffff) return CTCBS_EINVAL;
  *n_seg = (int32_t)n;
  if (n > cap || !h_len) return CTCBS_ECAP;
  const int64_t base = n_frames / n, extra = n_frames % n;   // the first `extra` pieces get one more frame
  for (int64_t i = 0; i < n; ++i) h_len[i] = (int32_t)(base + (i < extra ? 1 : 0));
  return CTCBS_OK;
}

extern "C" int ctcbs_merge_pieces(const int32_t* h_piece_len, int32_t n_pieces, int32_t min_len, int32_t max_len,
                                  int32_t* h_len, int32_t cap, int32_t* n_seg) {
  if (n_pieces < 0 || (n_pieces > 0 && !h_piece_len) || min_len < 1 || max_len < min_len || !n_seg)
    return CTCBS_EINVAL;
  int64_t count = 0;
  bool fits = true;
  auto emit = [&](int64_t len) {
    // a segment longer than max_len is split again, uniformly, into the fewest parts that fit
    const int64_t parts = (len + max_len - 1) / max_len;
    const int64_t base = len / parts, extra = len % parts;
    for (int64_t i = 0; i < parts; ++i) {
      if (h_len && count < cap) h_len[count] = (int32_t)(base + (i < extra ? 1 : 0)); else fits = false;
      ++count;
    }
  };
  int64_t acc = 0;
  for (int32_t i = 0; i < n_pieces; ++i) {
    if (h_piece_len[i] < 0) return CTCBS_EINVAL;
    acc += h_piece_len[i];
    if (acc >= min_len) { emit(acc); acc = 0; }       // consecutive pieces merged until min_len is reached
  }
  if (acc > 0) emit(acc);                              // what is left at the end stays a (short) segment
  if (count > 0x7fffffff) return CTCBS_EINVAL;
  *n_seg = (int32_t)count;
  return fits ? CTCBS_OK : CTCBS_ECAP;
}

extern "C" int ctcbs_plan_batches(const int32_t* h_len, int32_t n, int32_t max_utt, int64_t max_padded_frames,
                                  int32_t* h_order, int32_t* h_begin, int32_t cap_batches, int32_t* n_batches) {
  if (n < 0 || (n > 0 && (!h_len || !h_order)) || max_utt < 1 || !n_batches) return CTCBS_EINVAL;
  for (int32_t i = 0; i < n; ++i) {
    if (h_len[i] < 1) return CTCBS_EINVAL;
    if (max_padded_frames > 0 && h_len[i] > max_padded_frames) return CTCBS_EINVAL;   // fits no batch
    h_order[i] = i;
  }
  // longest first, equal lengths in input order
  std::stable_sort(h_order, h_order + n, [&](int32_t a, int32_t b) { return h_len[a] > h_len[b]; });
  int32_t nb = 0;
  bool fits = true;
  int32_t i = 0;
  while (i < n) {
    // the first segment of a batch is its longest: the batch is padded to that length
    const int64_t t_max = h_len[h_order[i]];
    int64_t take = max_utt;
    if (max_padded_frames > 0) take = std::min<int64_t>(take, max_padded_frames / t_max);
    take = std::min<int64_t>(take, n - i);
    if (h_begin && nb < cap_batches) h_begin[nb] = i; else fits = false;
    ++nb;
    i += (int32_t)take;
  }
  if (h_begin && nb <= cap_batches) h_begin[nb] = n; else fits = false;   // h_begin holds cap_batches + 1 entries
  *n_batches = nb;
  return fits ? CTCBS_OK : CTCBS_ECAP;
}

extern "C" int ctcbs_att_replay(void* user, int32_t index, int32_t step, const ctcbs_step_out_t* /*prev*/,
                                const float** d_att) {
  if (!user || !d_att || index < 0 || step < 1) return CTCBS_EINVAL;
  const ctcbs_replay_t& r = ((const ctcbs_replay_t*)user)[index];
  if (!r.d_att || r.n_steps < 1) return CTCBS_EINVAL;
  *d_att = r.d_att[std::min(step, r.n_steps) - 1];   // past the recording: the last rows again (such steps do nothing)
  return *d_att ? CTCBS_OK : CTCBS_EINVAL;
}

extern "C" int ctcbs_run_many(ctcbs_t* const* hs, int32_t n, ctcbs_att_fn fn, void* user, int32_t n_threads) {
  if (n < 0 || (n > 0 && !hs) || !fn || n_threads < 1) return CTCBS_EINVAL;
  for (int32_t i = 0; i < n; ++i)
    if (!hs[i]) return CTCBS_EINVAL;
  if (n == 0) return CTCBS_OK;
  n_threads = std::min(n_threads, n);
  std::atomic<int> first_error{CTCBS_OK};
  auto worker = [&](int32_t t) {
   try {
    // this thread's handles, stepped round-robin so that their kernels interleave on the device
    std::vector<int32_t> mine;
    for (int32_t i = t; i < n; i += n_threads) mine.push_back(i);
    std::vector<ctcbs_step_out_t> outs(mine.size());
    std::vector<char> started(mine.size(), 0), live(mine.size(), 1);
    if (hipSetDevice(hs[mine[0]]->device) != hipSuccess) { int ok = CTCBS_OK; first_error.compare_exchange_strong(ok, CTCBS_EHIP); return; }
    size_t n_live = mine.size();
    while (n_live > 0 && first_error.load(std::memory_order_relaxed) == CTCBS_OK) {
      for (size_t k = 0; k < mine.size(); ++k) {
        if (!live[k]) continue;
        ctcbs_t* h = hs[mine[k]];
        int rc = CTCBS_OK;
        if (h->known_finished >= h->p.U || h->step >= h->l_cap) rc = CTCBS_DONE;
        const float* att = nullptr;
        if (rc == CTCBS_OK) rc = fn(user, mine[k], h->step + 1, started[k] ? &outs[k] : nullptr, &att);
        if (rc == CTCBS_OK) rc = ctcbs_step(h, att, &outs[k]);
        if (rc == CTCBS_OK) { started[k] = 1; continue; }
        live[k] = 0; --n_live;
        if (rc != CTCBS_DONE) { int ok = CTCBS_OK; first_error.compare_exchange_strong(ok, rc); break; }
      }
    }
   } catch (...) {                                       // allocation failure inside the thread
    int ok = CTCBS_OK; first_error.compare_exchange_strong(ok, CTCBS_ENOMEM);
   }
  };
  std::vector<std::thread> pool;
  int32_t started_threads = 1;
  try {
    for (int32_t t = 1; t < n_threads; ++t) { pool.emplace_back(worker, t); ++started_threads; }
  } catch (...) {
    // not every thread could be started: the error flag stops those that were, nothing else runs
    int ok = CTCBS_OK; first_error.compare_exchange_strong(ok, CTCBS_ENOMEM);
  }
  if (started_threads == n_threads) worker(0);
  for (auto& th : pool) th.join();
  return first_error.load();
}

extern "C" int ctcbs_run_queue(ctcbs_t* const* hs, int32_t n_slots, int32_t n_jobs, ctcbs_job_fn job_fn,
                               ctcbs_att_fn att_fn, void* user, int32_t n_threads) {
  if (n_slots < 1 || !hs || n_jobs < 0 || !job_fn || !att_fn || n_threads < 1) return CTCBS_EINVAL;
  for (int32_t i = 0; i < n_slots; ++i)
    if (!hs[i]) return CTCBS_EINVAL;
  if (n_jobs == 0) return CTCBS_OK;
  n_threads = std::min(n_threads, n_slots);
  std::atomic<int> first_error{CTCBS_OK};
  std::atomic<int32_t> next_job{0};
  auto fail = [&](int rc) { int ok = CTCBS_OK; first_error.compare_exchange_strong(ok, rc); };
  auto worker = [&](int32_t t) {
   try {
    std::vector<int32_t> slots;
    for (int32_t i = t; i < n_slots; i += n_threads) slots.push_back(i);
    std::vector<int32_t> job(slots.size(), -1);          // -1: the slot is idle
    std::vector<ctcbs_step_out_t> outs(slots.size());
    std::vector<char> started(slots.size(), 0);
    if (hipSetDevice(hs[slots[0]]->device) != hipSuccess) { fail(CTCBS_EHIP); return; }
    bool more = true;                                     // jobs may be left in the queue
    size_t busy = 0;
    while ((more || busy > 0) && first_error.load(std::memory_order_relaxed) == CTCBS_OK) {
      for (size_t k = 0; k < slots.size(); ++k) {
        ctcbs_t* h = hs[slots[k]];
        if (job[k] < 0) {
          if (!more) continue;
          const int32_t j = next_job.fetch_add(1);
          if (j >= n_jobs) { more = false; continue; }
          const int rc = job_fn(user, j, slots[k], h, CTCBS_JOB_LOAD);
          if (rc != CTCBS_OK) { fail(rc < 0 ? rc : CTCBS_EINVAL); return; }
          job[k] = j; started[k] = 0; ++busy;
        }
        int rc = CTCBS_OK;
        if (h->known_finished >= h->p.U || h->step >= h->l_cap) rc = CTCBS_DONE;
        const float* att = nullptr;
        if (rc == CTCBS_OK) rc = att_fn(user, job[k], h->step + 1, started[k] ? &outs[k] : nullptr, &att);
        if (rc == CTCBS_OK) rc = ctcbs_step(h, att, &outs[k]);
        if (rc == CTCBS_OK) { started[k] = 1; continue; }
        if (rc != CTCBS_DONE) { fail(rc); return; }
        rc = job_fn(user, job[k], slots[k], h, CTCBS_JOB_DONE);
        if (rc != CTCBS_OK) { fail(rc < 0 ? rc : CTCBS_EINVAL); return; }
        job[k] = -1; --busy;
      }
    }
   } catch (...) {
    fail(CTCBS_ENOMEM);
   }
  };
  std::vector<std::thread> pool;
  int32_t started_threads = 1;
  try {
    for (int32_t t = 1; t < n_threads; ++t) { pool.emplace_back(worker, t); ++started_threads; }
  } catch (...) {
    fail(CTCBS_ENOMEM);
  }
  if (started_threads == n_threads) worker(0);
  for (auto& th : pool) th.join();
  return first_error.load();
}
