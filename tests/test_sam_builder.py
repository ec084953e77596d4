"""Asynchronous automaton construction: submit returns at once, the child thread builds, the automaton
is handed out only when nothing of the request is waiting, and it equals a synchronous build."""
import time

import numpy as np
import pytest

import paper_2512_18337_amd as A
from paper_2512_18337_amd import workloads as W


def _same(a, b):
    fa, fb = A.sam_flatten([a]), A.sam_flatten([b])
    return all(np.array_equal(getattr(fa, n), getattr(fb, n))
               for n in ("len", "link", "row_ptr", "edge_tok", "edge_dst", "lastpos", "corpus", "state_rec"))


def test_prompt_then_streamed_tokens_equal_a_synchronous_build():
    cfg = W.scaled(W.baseline_config(1), sam_session_len=131072)        # a 128k-token prompt
    T = W.token_memory(cfg, 0)
    b = A.SamBuilder()
    t0 = time.perf_counter()
    b.submit(7, T[:120000], cfg.sep)
    t_submit = time.perf_counter() - t0
    sam, pending = b.poll(7)                          # almost surely still building: no drafts yet
    assert sam is None or pending == 0
    for i in range(120000, len(T), 9):                # generated tokens arrive a few at a time
        b.submit(7, T[i:i + 9], cfg.sep)
    b.wait(7)
    t_all = time.perf_counter() - t0
    sam, pending = b.poll(7)
    assert sam is not None and pending == 0
    assert _same(sam, A.sam_build(T, cfg.sep))
    # the caller's cost is a copy of the tokens; the build itself (paper: about a second for 128k tokens
    # on its host) runs beside it
    assert t_submit < 0.05 and t_submit < t_all
    print(f"submit of 120k tokens returned in {t_submit * 1e3:.2f} ms; automaton of {len(T)} tokens ready after "
          f"{t_all * 1e3:.0f} ms ({len(T) / t_all / 1e6:.2f} M tokens/s in the background)")
    b.close()


def test_interleaved_requests_errors_and_release():
    rng = np.random.default_rng(3)
    b = A.SamBuilder()
    texts = {r: rng.integers(0, 50, 3000).astype(np.int32) for r in (1, 2, 3)}
    for lo in range(0, 3000, 500):
        for r in (1, 2, 3):
            b.submit(r, texts[r][lo:lo + 500], 99)
    for r in (1, 2, 3):
        b.wait(r)
        sam, pending = b.poll(r)
        assert pending == 0 and _same(sam, A.sam_build(texts[r], 99))
    with pytest.raises(A.AgentSamError):
        b.poll(42)                                    # never submitted
    b.submit(4, [1, 2, -5, 3], 99)                    # a negative token id surfaces at wait / poll
    with pytest.raises(A.AgentSamError):
        b.wait(4)
    with pytest.raises(A.AgentSamError):
        b.poll(4)
    b.release(2)
    with pytest.raises(A.AgentSamError):
        b.poll(2)
    b.submit(2, [5, 6, 7], 99)                        # the id can be used again once released
    b.wait(2)
    assert A.sam_flat_sizes(b.poll(2)[0])[2] == 3
    b.submit(1, np.zeros(200000, np.int32), 99)       # destroy with work still queued must not hang
    b.close()


def test_maintained_copy_fed_by_the_builder():
    """The builder's automaton is an ordinary one: flatten, stream more tokens, export the delta."""
    b = A.SamBuilder()
    b.submit(1, [1, 2, 3], 9)
    b.wait(1)
    sam, _ = b.poll(1)
    A.sam_flatten([sam])
    b.submit(1, [4, 5], 9)
    b.wait(1)
    sam, _ = b.poll(1)
    n_rec, n_lp, n_ov, n_ov_new, n_tok, flat_states = A.sam_delta_sizes(sam)
    assert n_tok == 2 and flat_states == 4 and n_ov > 0 and n_ov_new == n_ov
    b.close()


def test_flatten_again_on_the_child_thread():
    """A grown automaton is flattened again through the queue: ordered after the appends submitted before it,
    into the caller's arrays, with the same result as a flatten on the calling thread; too-small arrays are
    reported and leave the automaton usable."""
    rng = np.random.default_rng(3)
    T = rng.integers(0, 50, 5000).astype(np.int32)
    b = A.SamBuilder()
    b.submit(1, T[:3000], 99)
    b.wait(1)
    sam, _ = b.poll(1)
    A.sam_flatten([sam])
    assert b.flatten_result(1) == -2                          # none yet
    b.submit(1, T[3000:], 99)                                 # the flatten below must see these tokens
    ns_cap, ne_cap, nt_cap = 2 * 5000 + 2, 3 * 5000, 5000
    fill = lambda n: np.full(n, -1, np.int32)
    out = A.FlatSam(fill(ns_cap), fill(ns_cap), np.zeros(ns_cap + 1, np.int32), fill(ne_cap), fill(ne_cap), fill(ns_cap),
                    fill(nt_cap), fill(4 * ns_cap), np.zeros(1, np.int32), np.zeros(1, np.int32), np.zeros(1, np.int32))
    b.flatten(1, out)
    assert b.poll(1)[0] is None or b.flatten_result(1) == 0   # not available while the flatten is pending
    b.wait(1)
    assert b.flatten_result(1) == 0
    sam, pending = b.poll(1)
    assert sam is not None and pending == 0
    ns, ne, nt = A.sam_flat_sizes(sam)
    assert nt == 5000
    assert A.sam_delta_sizes(sam) == (0, 0, 0, 0, 0, ns)      # the flatten has reset the log
    ref = A.sam_flatten([A.sam_build(T, 99)])
    for name in ("len", "link", "lastpos", "corpus"):
        assert np.array_equal(getattr(out, name)[:getattr(ref, name).shape[0]], getattr(ref, name)), name
    assert np.array_equal(out.row_ptr[:ns + 1], ref.row_ptr) and np.array_equal(out.edge_tok[:ne], ref.edge_tok)
    assert np.array_equal(out.edge_dst[:ne], ref.edge_dst) and np.array_equal(out.state_rec[:4 * ns], ref.state_rec)
    small = A.FlatSam(fill(10), fill(10), np.zeros(11, np.int32), fill(10), fill(10), fill(10), fill(10), fill(40),
                      np.zeros(1, np.int32), np.zeros(1, np.int32), np.zeros(1, np.int32))
    b.flatten(1, small)
    b.wait(1)
    assert b.flatten_result(1) == -4                          # does not fit; nothing was written past the arrays
    assert b.poll(1)[0] is not None
    with pytest.raises(A.AgentSamError):
        b.flatten(77, out)                                    # unknown request
    b.close()
