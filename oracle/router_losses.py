"""CPU oracle for the forward values of the CLS-aware training objectives: TEST INFRASTRUCTURE.

Only the tests, the smoke check and the benchmark's cpu_baseline leg may import this file.
It shares no code with the HIP library.

Both losses are functions of the router pre-activations A^0 = W_router^T x (Eq. 3) of a token
stream cut into sequences of ``seq_len`` tokens, evaluated here in fp64 on the fp32 values:

* ``activation_locality_loss`` (Eq. 4): with A^0_s the pre-activations shifted left by one token
  along the sequence, L_al = BCE[ sigmoid(alpha * A^0), sigmoid(alpha * A^0_s) ]: the binary
  cross entropy -[q ln p + (1 - q) ln(1 - p)] with input p = sigmoid(alpha * A^0[t, i]) and
  target q = sigmoid(alpha * A^0[t + 1, i]), averaged over every (token, expert) pair that has
  a successor token.
* ``chunk_sparsification_loss`` (Eq. 5): p_ik = Norm(A^1(x_k))_i with A^1 = ReLU(A^0);
  P^i_act = 1 - exp(sum_{k=1..L} ln(1 - p_ik)); L_cs = (1 / N_e) sum_i P^i_act.

Readings where the paper is silent:
  - the last token of a sequence has no successor and contributes no term to L_al; the mean is
    over (seq_len - 1) * N_e terms per sequence, all sequences pooled (0 when seq_len = 1);
  - ln p and ln(1 - p) are taken as the exact log-sigmoids -softplus(-z) and -softplus(z) of
    z = alpha * A^0 (no clamping of the logarithms), so the loss stays finite and exact for
    sharp alpha where p itself rounds to 0 or 1;
  - Norm is the L1 normalisation over the expert dimension (the text requires
    sum_i p_ik = 1); a token with no active expert has p_ik = 0 for every i;
  - chunks are the disjoint windows [j*L, (j+1)*L) of each sequence (a shorter tail is left
    out) and L_cs is averaged over all chunks (0 when there is none);
  - p_ik = 1 gives ln 0 = -inf and P^i_act = 1, the limit.
"""

from __future__ import annotations

import numpy as np
from scipy.special import expit


def _as_sequences(a0: np.ndarray, seq_len: int) -> np.ndarray:
    a = np.asarray(a0, dtype=np.float32).astype(np.float64)
    n_tok, E = a.shape
    assert seq_len >= 1 and n_tok % seq_len == 0
    return a.reshape(n_tok // seq_len, seq_len, E)


def activation_locality_loss(a0: np.ndarray, seq_len: int, alpha: float) -> float:
    a = _as_sequences(a0, seq_len)
    if seq_len < 2 or a.size == 0:
        return 0.0
    alpha = float(np.float32(alpha))
    z = alpha * a[:, :-1, :]          # token t
    zs = alpha * a[:, 1:, :]          # token t + 1 (the left-shifted sequence)
    q = expit(zs)
    one_minus_q = expit(-zs)
    log_p = -np.logaddexp(0.0, -z)            # ln sigmoid(z)
    log_one_minus_p = -np.logaddexp(0.0, z)   # ln (1 - sigmoid(z))
    bce = -(q * log_p + one_minus_q * log_one_minus_p)
    return float(bce.mean())


def chunk_sparsification_loss(a0: np.ndarray, seq_len: int, L: int) -> float:
    a = _as_sequences(a0, seq_len)
    n_seq, _, E = a.shape
    n_win = seq_len // L
    if n_win == 0 or n_seq == 0:
        return 0.0
    a1 = np.maximum(a, 0.0)
    norm = a1.sum(axis=2, keepdims=True)
    p = np.divide(a1, norm, out=np.zeros_like(a1), where=norm > 0)
    p = p[:, :n_win * L, :].reshape(n_seq, n_win, L, E)
    with np.errstate(divide="ignore"):
        log_idle = np.log1p(-p).sum(axis=2)       # ln prod_k (1 - p_ik)
    p_act = 1.0 - np.exp(log_idle)                # [n_seq][n_win][E]
    return float(p_act.mean(axis=2).mean())
