"""The pins must notice plausible mistakes.  Each case plants one mistake in the
numpy oracle (on the CPU, by patching one of its functions) and checks that at
least one pin of test_oracle_pins fails."""
import inspect

import numpy as np
import pytest

from oracle import decode_attention as np_oracle

import test_oracle_pins as pins

PIN_FUNCS = [f for name, f in inspect.getmembers(pins, inspect.isfunction)
             if name.startswith("test_") and list(inspect.signature(f).parameters) == ["impl"]]


def run_pins():
    """Names of the pins that fail with the (patched) numpy oracle."""
    failed = []
    for f in PIN_FUNCS:
        try:
            f(np_oracle)
        except AssertionError:
            failed.append(f.__name__)
        except Exception:            # shape errors etc. also count as noticed
            failed.append(f.__name__)
    return failed


def test_unpatched_oracle_passes_every_pin():
    assert len(PIN_FUNCS) >= 15
    assert run_pins() == []


ORIG_ATTEND = np_oracle.attend_one
ORIG_GATHER = np_oracle.gather_rows
ORIG_APPEND = np_oracle.kv_append
ORIG_DECODE = np_oracle.decode


def drop_scale(q, K, V, scale):
    return ORIG_ATTEND(q, K, V, 1.0)


def flip_sign(q, K, V, scale):
    return ORIG_ATTEND(q, K, V, -scale)


def swap_k_v(q, K, V, scale):
    return ORIG_ATTEND(q, V, K, scale)


def drop_last_row(q, K, V, scale):
    if len(K) > 1:
        return ORIG_ATTEND(q, K[:-1], V[:-1], scale)
    return ORIG_ATTEND(q, K, V, scale)


def unnormalised(q, K, V, scale):
    out, lse, w = ORIG_ATTEND(q, K, V, scale)
    return out * np.exp(lse - (scale * (np.asarray(K, float) @ np.asarray(q, float))).max()), lse, w


def lse_without_max(q, K, V, scale):
    out, lse, w = ORIG_ATTEND(q, K, V, scale)
    s = np.float64(np.float32(scale)) * (np.asarray(K, float) @ np.asarray(q, float))
    return out, lse - s.max(), w


def hard_max(q, K, V, scale):
    out, lse, w = ORIG_ATTEND(q, K, V, scale)
    return np.asarray(V, float)[int(np.argmax(w))], lse, w


def reversed_query(q, K, V, scale):
    return ORIG_ATTEND(np.asarray(q)[::-1], K, V, scale)


def gather_one_too_far(cache, b, hk, L, page_table=None):
    return ORIG_GATHER(cache, b, hk, L, page_table)[::-1][: max(L - 1, 1)]


def gather_swapped_page_index(cache, b, hk, L, page_table=None):
    if page_table is None:
        return ORIG_GATHER(cache, b, hk, L, page_table)
    ps = cache.shape[2]
    return np.stack([cache[int(page_table[b, (t % ps) % page_table.shape[1]]), hk, (t // ps) % ps]
                     for t in range(L)])


def gather_wrong_head(cache, b, hk, L, page_table=None):
    return ORIG_GATHER(cache, b, (hk + 1) % cache.shape[1], L, page_table)


def append_one_slot_late(k_cache, v_cache, k_new, v_new, seq_lens, page_table=None):
    return ORIG_APPEND(k_cache, v_cache, k_new, v_new, np.asarray(seq_lens) + 1, page_table)


def append_swaps_k_v(k_cache, v_cache, k_new, v_new, seq_lens, page_table=None):
    return ORIG_APPEND(k_cache, v_cache, v_new, k_new, seq_lens, page_table)


def decode_interleaved_groups(q, k_cache, v_cache, seq_lens, scale, page_table=None):
    """Head h read from KV head h % Hkv instead of h // G."""
    B, Hq, D = q.shape
    Hkv = k_cache.shape[1]
    G = Hq // Hkv
    perm = np.array([(h % Hkv) * G + h // Hkv for h in range(Hq)])
    out, lse = ORIG_DECODE(q[:, np.argsort(perm)], k_cache, v_cache, seq_lens, scale, page_table)
    return out[:, perm], lse[:, perm]


MUTANTS = [
    ("attend_one", drop_scale), ("attend_one", flip_sign), ("attend_one", swap_k_v),
    ("attend_one", drop_last_row), ("attend_one", unnormalised), ("attend_one", lse_without_max),
    ("attend_one", hard_max), ("attend_one", reversed_query),
    ("gather_rows", gather_one_too_far), ("gather_rows", gather_swapped_page_index),
    ("gather_rows", gather_wrong_head),
    ("kv_append", append_one_slot_late), ("kv_append", append_swaps_k_v),
    ("decode", decode_interleaved_groups),
]


@pytest.mark.parametrize("target,mutant", MUTANTS, ids=[m.__name__ for _, m in MUTANTS])
def test_planted_mistake_is_caught(monkeypatch, target, mutant):
    monkeypatch.setattr(np_oracle, target, mutant)
    assert run_pins(), "no pin noticed the mistake '%s'" % mutant.__name__
