"""Pins of the carried-match oracle (stateful lookup of Alg. 4's decoding loop), none of which call it to
produce their own expected value: an independent longest-suffix scan on a fixed memory, a worked example
with a growing memory computed by hand, and the invariants of the recursion."""
import numpy as np

from oracle import carried_match_len_oracle, draft_oracle, draft_step_oracle


def _longest_suffix_plain(T, ctx):
    """Longest suffix of ctx that occurs in T, by trying every length and every start position."""
    T, ctx = list(T), list(ctx)
    for L in range(min(len(ctx), len(T)), 0, -1):
        pat = ctx[len(ctx) - L:]
        for i in range(len(T) - L + 1):
            if T[i:i + L] == pat:
                return L
    return 0


def test_fixed_memory_any_chunking_gives_the_longest_suffix():
    rng = np.random.default_rng(5)
    for trial in range(30):
        vocab = int(rng.integers(3, 9))
        T = rng.integers(0, vocab, int(rng.integers(5, 60))).astype(np.int32)
        ctx = []
        for _ in range(int(rng.integers(1, 6))):             # context: copies of memory spans and noise
            if rng.random() < 0.7:
                p = int(rng.integers(0, len(T))); ctx += list(T[p:p + int(rng.integers(1, 12))])
            else:
                ctx += [int(x) for x in rng.integers(0, vocab + 1, int(rng.integers(1, 4)))]
        ctx = np.asarray(ctx, np.int32)
        L, done = 0, 0
        while done < len(ctx):                               # feed in pieces of random size (0 allowed)
            n = int(rng.integers(0, 5))
            n = min(n, len(ctx) - done)
            done += n
            L_new = carried_match_len_oracle(T, ctx[:done], L, n)
            assert L_new <= L + n
            L = L_new
            assert L == _longest_suffix_plain(T, ctx[:done]), (trial, done)


def test_growing_memory_worked_example():
    sep = 9
    T1 = np.array([1, 2, 3, sep], np.int32)
    # tokens 5, 2, 3 against T1: "5" does not occur (0); "2" occurs (1); "2 3" occurs (2)
    assert carried_match_len_oracle(T1, [5], 0, 1) == 0
    assert carried_match_len_oracle(T1, [5, 2], 0, 1) == 1
    assert carried_match_len_oracle(T1, [5, 2, 3], 1, 1) == 2
    assert carried_match_len_oracle(T1, [5, 2, 3], 0, 3) == 2
    # the memory grows by "5 2 3 4 7 8 <sep>"; the next token is 4.  Carried: "2 3" + "4" = "2 3 4" occurs -> 3.
    # A fresh search over the whole context would find "5 2 3 4" (4): the carried match is not that.
    T2 = np.array([1, 2, 3, sep, 5, 2, 3, 4, 7, 8, sep], np.int32)
    ctx = [5, 2, 3, 4]
    assert carried_match_len_oracle(T2, ctx, 2, 1) == 3
    assert _longest_suffix_plain(T2, ctx) == 4
    # proposal: "2 3 4" ends at index 7 of T2, followed by 7 8 and then the separator
    L, d, nd, ml, me = draft_step_oracle(T2, ctx, 2, 1, 4, sep)
    assert (L, nd, ml, me) == (3, 2, 3, 7) and list(d) == [7, 8, -1, -1]
    # a mismatching token cuts the match from the left: "... 4" then 2 -> only "2" is left (occurs), length 1
    assert carried_match_len_oracle(T2, ctx + [2], 3, 1) == 1
    # and a token that occurs nowhere resets it
    assert carried_match_len_oracle(T2, ctx + [6], 3, 1) == 0
    L, d, nd, ml, me = draft_step_oracle(T2, ctx + [6], 3, 1, 4, sep)
    assert (L, nd, ml, me) == (0, 0, 0, -1) and list(d) == [-1] * 4


def test_step_proposal_equals_window_proposal_of_the_carried_length():
    rng = np.random.default_rng(11)
    sep = 50
    T = np.concatenate([rng.integers(0, 6, 80), [sep], rng.integers(0, 6, 60), [sep]]).astype(np.int32)
    ctx = list(T[10:25]) + [3, 1] + list(T[90:110])
    L = 0
    for n in range(1, len(ctx) + 1):
        L2, d, nd, ml, me = draft_step_oracle(T, ctx[:n], L, 1, 5, sep)
        assert L2 <= L + 1
        assert L2 == _longest_suffix_plain(T, ctx[:n])
        od, ond, oml, ome = draft_oracle(T, np.asarray(ctx[n - L2:n], np.int32), 5, sep, 1) if L2 else (np.full(5, -1), 0, 0, -1)
        assert (nd, ml, me) == (ond, oml, ome) and list(d) == list(od)
        L = L2
