"""The decoding loop of Alg. 4 closed on the device: stateful lookup -> (a stand-in model's logits) -> accept ->
the committed tokens feed the next lookup without leaving the device.  Whatever the drafts are, the committed
text equals what greedy decoding of the same model emits (Sec. 5.4.1: the speculation is lossless), and on a
memory that contains most of that text several tokens are committed per step."""
import numpy as np
import pytest
import torch

import paper_2512_18337_amd as A
from paper_2512_18337_amd import workloads as W
from _util import to_np

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def test_speculative_loop_commits_exactly_the_greedy_text():
    cfg = W.scaled(W.baseline_config(2), B=12, sam_sessions=4, sam_session_len=1500, vocab=300, m=32, k=6)
    rng = np.random.default_rng(2024)
    T = [int(x) for x in W.token_memory(cfg)]
    flat = A.sam_flatten([A.sam_build(np.asarray(T, np.int32), cfg.sep)])
    fd = flat.to(DEV)
    B, k, R, V, n_out = cfg.B, cfg.k, cfg.k + 1, cfg.vocab, 70
    # what the "model" will say: text that mostly follows spans of the memory, with its own words in between
    truth = []
    for b in range(B):
        g = []
        while len(g) < 8 * n_out + R:     # (fast sessions run on while the slowest catches up)
            if rng.random() < 0.8:
                p = int(rng.integers(0, len(T) - 40))
                g += [t for t in T[p:p + int(rng.integers(5, 30))] if t != cfg.sep]
            else:
                g += [int(x) for x in rng.integers(0, V, int(rng.integers(1, 4)))]
        truth.append(g)
    root = torch.full((B,), int(flat.roots[0]), dtype=torch.int32, device=DEV)
    cend = torch.full((B,), int(flat.corpus_end[0]), dtype=torch.int32, device=DEV)
    cur_state = torch.full((B,), -1, dtype=torch.int32, device=DEV)
    cur_len = torch.zeros((B,), dtype=torch.int32, device=DEV)
    committed = [[truth[b][0]] for b in range(B)]             # the prompt: one token
    new_tok = torch.as_tensor(np.array([[truth[b][0]] + [0] * k for b in range(B)], np.int32), device=DEV)
    n_new = torch.ones((B,), dtype=torch.int32, device=DEV)
    steps = 0
    while min(len(c) for c in committed) < n_out:
        steps += 1
        d, nd, _, _ = A.sam_draft_step(fd, root, cend, new_tok, n_new, cur_state, cur_len, k, cfg.sep)
        dh = to_np(d)
        # the stand-in model: row i answers with the token that follows committed + drafts[:i] in its own text as
        # long as those drafts are its own text, with anything else afterwards
        logits = rng.standard_normal((B, R, V)).astype(np.float32)
        for b in range(B):
            pos, ok = len(committed[b]), True
            for i in range(R):
                ok = ok and (i == 0 or int(dh[b, i - 1]) == truth[b][pos + i - 1])
                logits[b, i, truth[b][pos + i] if ok else int(rng.integers(0, V))] = 9.0
        a, toks, _ = A.spec_accept(torch.as_tensor(logits, device=DEV), d, nd)
        new_tok, n_new = toks, a + 1                          # the next lookup consumes them, all on the device
        ah, th = to_np(a), to_np(toks)
        for b in range(B):
            got = [int(x) for x in th[b, :ah[b] + 1]]
            pos = len(committed[b])
            assert got == truth[b][pos:pos + len(got)], (steps, b)     # exactly the greedy text
            assert (th[b, ah[b] + 1:] == -1).all()
            committed[b] += got
    total = sum(len(c) - 1 for c in committed)
    assert total / (steps * B) > 1.5                          # the memory earns more than one token per step
