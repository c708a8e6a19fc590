"""Host-only simulator of the four-block KV cache sizes (Sec. 3.3 "Tailored Streaming Design").

TEST INFRASTRUCTURE ONLY.  Tracks (Size_init, Size_sep, Size_past_w, Size_local_w) token by
token: the Initial Cache fills first (capacity a), then the window; when the runtime usage
Size_run reaches c the Past Window (the oldest n-w window entries) is compressed: its separators
are appended to the Separator Cache (capacity s, oldest dropped on overflow), its other entries
are discarded, and the window keeps its newest w entries.
"""
from __future__ import annotations

from typing import Dict

import numpy as np


def simulate(is_sep: np.ndarray, a: int, s: int, w: int, c: int) -> Dict[str, np.ndarray]:
    """Feed a stream of tokens (is_sep[m] flags) and record the sizes after each token.

    Returns arrays of length len(is_sep):
      size_run_pre[m]  runtime usage right after token m was appended, before any compression;
      size_run[m]      runtime usage after the compression step (if it fired at m);
      n[m]             number of contiguous neighbouring tokens kept after token m (post step);
      size_sep[m], compressed[m] (bool).
    """
    assert a + s + w < c, "the paper requires a + s + w < c"
    init = 0
    sep = 0
    window = []  # separator flags of the window entries, oldest first
    M = len(is_sep)
    size_run_pre = np.zeros(M, dtype=np.int64)
    size_run = np.zeros(M, dtype=np.int64)
    n_hist = np.zeros(M, dtype=np.int64)
    sep_hist = np.zeros(M, dtype=np.int64)
    fired = np.zeros(M, dtype=bool)
    for m in range(M):
        if init < a:
            init += 1
        else:
            window.append(bool(is_sep[m]))
        run = init + sep + len(window)
        size_run_pre[m] = run
        if run == c:
            past = window[: len(window) - w]
            window = window[len(window) - w:]
            sep = min(s, sep + sum(past))
            fired[m] = True
        size_run[m] = init + sep + len(window)
        n_hist[m] = len(window)
        sep_hist[m] = sep
    return {"size_run_pre": size_run_pre, "size_run": size_run, "n": n_hist,
            "size_sep": sep_hist, "compressed": fired}
