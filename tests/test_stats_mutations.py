"""The pins of the statistics, objective and offload oracles really pin: one plausible mistake
at a time is planted in a copy of an oracle's source (in memory, on the CPU; the committed file
is never touched), and the pin suite of that oracle must notice."""

import importlib.util
import os
import types

import pytest

import test_losses_pins
import test_offload_pins
import test_stats_pins

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

# oracle file, the name the pins module binds it to, the pins module
TARGETS = {
    "stats": ("oracle/sparsity_stats.py", "ss", test_stats_pins),
    "losses": ("oracle/router_losses.py", "rl", test_losses_pins),
    "offload": ("oracle/offload_sim.py", "osim", test_offload_pins),
}

MUTATIONS = {
    # CLS_L sweep
    "cls_union_is_intersection": ("stats", "union |= seq[t]", "union = seq[t] if t == s else union & seq[t]"),
    "cls_counts_active_not_inactive": ("stats", "inactive[mode, L - 1] += E - _popcount(union)",
                                       "inactive[mode, L - 1] += _popcount(union)"),
    "cls_disjoint_windows_overlap": ("stats", "disjoint = [j * L for j in range(seq_len // L)]",
                                     "disjoint = [j for j in range(seq_len // L)]"),
    "cls_sliding_off_by_one": ("stats", "sliding = [s for s in range(seq_len) if s + L <= seq_len]",
                               "sliding = [s for s in range(seq_len) if s + L < seq_len]"),
    "cls_windows_cross_sequences": ("stats", "for base in range(0, n_tok, seq_len):\n        seq = sets[base:base + seq_len]\n        for L in range(1, L_max + 1):",
                                    "seq_len = n_tok\n    for base in range(0, n_tok, seq_len):\n        seq = sets[base:base + seq_len]\n        for L in range(1, L_max + 1):"),
    "cls_divides_by_windows_only": ("stats", "(windows[nz].astype(np.float64) * float(E))", "(windows[nz].astype(np.float64))"),
    "cls_keeps_bits_above_E": ("stats", "out.append(v & keep)", "out.append(v)"),
    # reuse ratio
    "reuse_divides_by_next_set": ("stats", "card = _popcount(sets[i])\n            if card == 0:",
                                  "card = _popcount(sets[i + 1])\n            if card == 0:"),
    "reuse_union_instead_of_intersection": ("stats", "inter = _popcount(sets[i] & sets[i + 1])", "inter = _popcount(sets[i] | sets[i + 1])"),
    "reuse_pairs_cross_sequences": ("stats", "for i in range(base, base + seq_len - 1):", "for i in range(base, min(base + seq_len, n_tok - 1)):"),
    "reuse_empty_sets_count_as_zero": ("stats", "if card == 0:\n                continue", "if card == 0:\n                pairs += 1\n                continue"),
    # Eq. 4
    "al_target_and_input_swapped": ("losses", "bce = -(q * log_p + one_minus_q * log_one_minus_p)",
                                    "bce = -(expit(z) * (-np.logaddexp(0.0, -zs)) + expit(-z) * (-np.logaddexp(0.0, zs)))"),
    "al_alpha_dropped": ("losses", "z = alpha * a[:, :-1, :]", "z = a[:, :-1, :]"),
    "al_shift_right_instead_of_left": ("losses", "zs = alpha * a[:, 1:, :]          # token t + 1 (the left-shifted sequence)",
                                       "zs = alpha * np.concatenate([a[:, :1, :], a[:, :-2, :]], axis=1) if a.shape[1] > 2 else alpha * a[:, :1, :]"),
    "al_missing_second_term": ("losses", "bce = -(q * log_p + one_minus_q * log_one_minus_p)", "bce = -(q * log_p)"),
    "al_pairs_cross_sequences": ("losses", "    a = _as_sequences(a0, seq_len)\n    if seq_len < 2 or a.size == 0:\n        return 0.0\n    alpha",
                                 "    a = _as_sequences(a0, seq_len)\n    if seq_len < 2 or a.size == 0:\n        return 0.0\n    a = a.reshape(1, -1, a.shape[2])\n    alpha"),
    # Eq. 5
    "cs_softmax_instead_of_l1": ("losses", "p = np.divide(a1, norm, out=np.zeros_like(a1), where=norm > 0)",
                                 "p = np.exp(a1) / np.exp(a1).sum(axis=2, keepdims=True)"),
    "cs_norm_over_tokens": ("losses", "norm = a1.sum(axis=2, keepdims=True)", "norm = a1.sum(axis=1, keepdims=True) + 0 * a1.sum(axis=2, keepdims=True)"),
    "cs_relu_dropped": ("losses", "a1 = np.maximum(a, 0.0)", "a1 = np.abs(a)"),
    "cs_probability_of_all_tokens": ("losses", "p_act = 1.0 - np.exp(log_idle)", "p_act = np.exp(np.log(np.maximum(p, 1e-300)).sum(axis=2))"),
    "cs_sum_not_mean_over_experts": ("losses", "return float(p_act.mean(axis=2).mean())", "return float(p_act.sum(axis=2).mean())"),
    "cs_sliding_chunks": ("losses", "    n_win = seq_len // L\n", "    n_win = seq_len // L\n    a = np.roll(a, 1, axis=1)\n"),
    # offload
    "lru_is_fifo": ("offload", "                cache.move_to_end(e)\n", ""),
    "lru_evicts_most_recent": ("offload", "cache.popitem(last=False)", "cache.popitem(last=True)"),
    "lru_capacity_off_by_one": ("offload", "if len(cache) >= capacity:", "if len(cache) > capacity:"),
    "lru_hits_count_as_loads": ("offload", "            if e in cache:\n                cache.move_to_end(e)\n                continue",
                                "            if e in cache:\n                cache.move_to_end(e)\n                loads[c] += 1\n                continue"),
}


def load_mutated(which, old, new):
    path, _, _ = TARGETS[which]
    src = open(os.path.join(ROOT, path)).read()
    if old is not None:
        assert src.count(old) == 1, "the mutation must apply exactly once: %r" % old
        src = src.replace(old, new)
    mod = types.ModuleType("mutated_" + which)
    mod.__file__ = path
    exec(compile(src, path, "exec"), mod.__dict__)
    return mod


def run_pins(pins_mod):
    """Runs every test function of a pins module that needs no library or GPU; returns the failures."""
    failed = []
    for name, fn in sorted(vars(pins_mod).items()):
        if not name.startswith("test_") or "library" in name or not callable(fn):
            continue
        cases = [()]
        for mark in getattr(fn, "pytestmark", []):
            if mark.name == "parametrize":
                names = [n.strip() for n in mark.args[0].split(",")]
                cases = [v if len(names) > 1 else (v,) for v in mark.args[1]]
        for args in cases:
            try:
                fn(*args)
            except Exception as exc:   # noqa: BLE001 - any failure counts as "noticed"
                failed.append((name, args, type(exc).__name__))
    return failed


@pytest.mark.parametrize("which", sorted(TARGETS))
def test_unmodified_copy_passes(which, monkeypatch):
    _, attr, pins_mod = TARGETS[which]
    monkeypatch.setattr(pins_mod, attr, load_mutated(which, None, None))
    assert run_pins(pins_mod) == []


@pytest.mark.parametrize("name", sorted(MUTATIONS))
def test_planted_mistake_is_caught(name, monkeypatch):
    which, old, new = MUTATIONS[name]
    _, attr, pins_mod = TARGETS[which]
    monkeypatch.setattr(pins_mod, attr, load_mutated(which, old, new))
    failed = run_pins(pins_mod)
    assert failed, "no pin noticed the planted mistake %r" % name
