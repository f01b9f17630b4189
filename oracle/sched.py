"""Plain definitions of the offline scheduling helpers (test infrastructure, like the rest of
oracle/: only tests may import this).  Written from the paper's description, one step at a time:

* hard segmentation (Sec. 3.3, second method; Sec. 4.4): lengths between a minimum and a maximum,
  as uniform as possible, the last segment included;
* segments from voice-activity pieces (Sec. 4.4, first method): consecutive pieces merged until
  the minimum length is reached, over-long segments split again uniformly;
* length-sorted batching (Sec. 4.2).
"""


def hard_segments(n_frames, min_len, max_len):
    if n_frames == 0:
        return []
    n = 1
    while n * max_len < n_frames:          # fewest pieces that can respect max_len
        n += 1
    lens = [n_frames // n] * n
    for i in range(n_frames - sum(lens)):  # spread the remainder one frame at a time
        lens[i] += 1
    return lens


def merge_pieces(pieces, min_len, max_len):
    out, acc = [], 0
    for p in list(pieces) + [None]:
        if p is not None:
            acc += p
        if acc and (p is None or acc >= min_len):
            out.extend(hard_segments(acc, 1, max_len))
            acc = 0
    return out


def plan_batches(lens, max_utt, max_padded_frames=0):
    order = sorted(range(len(lens)), key=lambda i: (-lens[i], i))
    begin, i = [], 0
    while i < len(order):
        begin.append(i)
        take = 1                            # grow the batch while both limits hold
        while (i + take < len(order) and take + 1 <= max_utt and
               (max_padded_frames <= 0 or (take + 1) * lens[order[i]] <= max_padded_frames)):
            take += 1
        i += take
    begin.append(len(order))
    return order, begin
