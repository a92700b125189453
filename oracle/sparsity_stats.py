"""CPU oracle for the sparsity statistics of activation masks: TEST INFRASTRUCTURE.

Only the tests, the smoke check and the benchmark's cpu_baseline leg may import this file.
It shares no code with the HIP library.

What it computes, from the per-token activation masks (bit i of a token's mask is set iff
the token activates expert i, i.e. A^0_i > 0 in Eq. 3):

* ``cls_sweep``    CLS_L for L = 1 .. L_max (Sec. 2.1): the share of experts that no token of
  a window of L consecutive tokens activates, averaged over the windows; CLS_1 is TLS.  Two
  families of windows are evaluated, each straight from its definition:
    - disjoint: a sequence is cut into floor(seq_len / L) windows [j*L, (j+1)*L); a tail
      shorter than L is left out;
    - sliding: every start s with s + L <= seq_len gives the window [s, s + L).
  This is the quantity plotted against the chunk length in Fig. 1(a).
* ``reuse_ratio``  expert selection stability (Sec. 4.1.2 and Table 4): with S_i the set of
  experts token i activates, the mean over neighbouring pairs of |S_i & S_{i+1}| / |S_i|.

Readings where the paper is silent:
  - windows and pairs never cross a sequence boundary (the token stream is n_tok / seq_len
    sequences of seq_len tokens each);
  - a pair whose first token activates no expert has no ratio (0 / 0) and is left out of
    both the sum and the number of pairs averaged over;
  - all pairs of all sequences are pooled into one mean (equal to the mean of the
    per-sequence means whenever no pair is left out, the sequences having equal lengths);
  - a length with no window (L > seq_len) and a stream with no valid pair report 0.

Everything but the two final divisions is integer arithmetic.
"""

from __future__ import annotations

import numpy as np


def _bitsets(token_mask: np.ndarray, E: int):
    """One Python integer per token holding its expert set (bits at or above E dropped)."""
    m = np.ascontiguousarray(token_mask, dtype=np.uint64)
    keep = (1 << E) - 1
    out = []
    for row in m:
        v = 0
        for w, word in enumerate(row):
            v |= int(word) << (64 * w)
        out.append(v & keep)
    return out


def _popcount(v: int) -> int:
    return bin(v).count("1")


def cls_sweep(token_mask: np.ndarray, E: int, seq_len: int, L_max: int):
    """Returns (inactive, windows, cls), each [2][L_max]; row 0 disjoint windows, row 1 sliding.

    inactive[m][L-1] = sum over the windows of (E - number of experts active in the window),
    windows[m][L-1]  = number of windows, cls = inactive / (windows * E) in fp64.
    """
    sets = _bitsets(token_mask, E)
    n_tok = len(sets)
    assert seq_len >= 1 and n_tok % seq_len == 0 and L_max >= 1
    inactive = np.zeros((2, L_max), dtype=np.int64)
    windows = np.zeros((2, L_max), dtype=np.int64)
    for base in range(0, n_tok, seq_len):
        seq = sets[base:base + seq_len]
        for L in range(1, L_max + 1):
            disjoint = [j * L for j in range(seq_len // L)]
            sliding = [s for s in range(seq_len) if s + L <= seq_len]
            for mode, starts in ((0, disjoint), (1, sliding)):
                for s in starts:
                    union = 0
                    for t in range(s, s + L):
                        union |= seq[t]
                    inactive[mode, L - 1] += E - _popcount(union)
                    windows[mode, L - 1] += 1
    cls = np.zeros((2, L_max), dtype=np.float64)
    nz = windows > 0
    cls[nz] = inactive[nz].astype(np.float64) / (windows[nz].astype(np.float64) * float(E))
    return inactive, windows, cls


def reuse_ratio(token_mask: np.ndarray, E: int, seq_len: int):
    """Returns (num, cnt, ratio): num[c] = sum of |S_i & S_{i+1}| over the pairs with |S_i| = c,
    cnt[c] = number of such pairs (both int64 [E + 1], entry 0 stays 0), and ratio = the mean of
    |S_i & S_{i+1}| / |S_i| over the pairs with a non-empty S_i (fp64)."""
    sets = _bitsets(token_mask, E)
    n_tok = len(sets)
    assert seq_len >= 1 and n_tok % seq_len == 0
    num = np.zeros(E + 1, dtype=np.int64)
    cnt = np.zeros(E + 1, dtype=np.int64)
    total, pairs = 0.0, 0
    for base in range(0, n_tok, seq_len):
        for i in range(base, base + seq_len - 1):
            card = _popcount(sets[i])
            if card == 0:
                continue
            inter = _popcount(sets[i] & sets[i + 1])
            num[card] += inter
            cnt[card] += 1
            total += inter / card
            pairs += 1
    return num, cnt, (total / pairs if pairs else 0.0)
