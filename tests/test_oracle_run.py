"""Pins of the oracle's multi-step greedy run (CPU only).

The run is the decode step of Eq. 3 applied repeatedly, each step extending the caches by one
entry (Eq. 4).  What fixes the expected values here: greedy generation by brute force (a causal
forward over prompt + everything generated so far, recomputed from scratch for every new token,
with the library-pinned forward of test_oracle_pins), and counting arguments for the page bookkeeping.
"""
import numpy as np
import pytest

from helpers import MiniShape, random_weights
from test_oracle_pins import PT, _pool_for, _prefill_into_pool


def _greedy_by_brute_force(orc, cfg, params, prompt, n_steps):
    toks = list(prompt)
    out = []
    for _ in range(n_steps):
        logits = orc.full_forward(cfg, params, toks, round_kv=True)
        nxt = int(np.argmax(logits[-1]))
        out.append(nxt)
        toks.append(nxt)
    return out


@pytest.mark.parametrize("L", [3, 14, 30])
def test_run_equals_brute_force_greedy_generation(orc, L):
    """One request: prompt KV in pages, then 20 steps that cross one or two page boundaries with
    pages taken from a free list; the generated tokens must be those of from-scratch greedy decoding."""
    shape = MiniShape()
    rng = np.random.default_rng(900 + L)
    w = random_weights(shape, rng)
    cfg, params = orc.make_cfg(shape), orc.params_from_arrays(w)
    n_steps = 20
    prompt = rng.integers(0, shape.vocab, size=L + 1)
    n_pages = 12
    perm = rng.permutation(n_pages).astype(np.int32)
    have = L // PT + 1                       # pages that hold slots 0..L
    max_pages = (L + n_steps) // PT + 2
    table = np.full((1, max_pages), -1, np.int32)
    table[0, :have] = perm[:have]
    free = perm[have:]
    base, pool = _prefill_into_pool(orc, shape, cfg, params, prompt[:L], n_pages, table[0], rng)
    res = orc.decode_run(cfg, params, pool, prompt[L:L + 1], table, [L], [0], free, 0, n_steps)
    want = _greedy_by_brute_force(orc, cfg, params, prompt, n_steps)
    assert res["tokens"][:, 0].tolist() == want
    assert res["status"] == 0 and int(res["seq_lens"][0]) == L + n_steps
    crossed = (L + n_steps) // PT - L // PT
    assert res["free_head"] == crossed
    assert res["page_tables"][0, have:have + crossed].tolist() == free[:crossed].tolist()
    assert (res["page_tables"][0, have + crossed:] == -1).all()


def test_page_bookkeeping_by_counting(orc):
    """Several requests, 40 steps: every request ends n_steps longer; the number of pages taken is the
    number of multiples of 16 in (L_i, L_i + n_steps]; they are the first entries of the free list, each
    used once, and within a step lower request indices are served first."""
    shape = MiniShape(n_layers=1)
    rng = np.random.default_rng(77)
    w = random_weights(shape, rng)
    cfg, params = orc.make_cfg(shape), orc.params_from_arrays(w)
    lens = np.array([0, 15, 16, 31, 7, 47], np.int32)
    n_steps = 40
    B = len(lens)
    have = lens // PT + 1
    n_pages = int(have.sum()) + 30
    perm = rng.permutation(n_pages).astype(np.int32)
    max_pages = int((lens + n_steps).max()) // PT + 1
    tables = np.full((B, max_pages), -1, np.int32)
    o = 0
    for i in range(B):
        tables[i, :have[i]] = perm[o:o + have[i]]
        o += int(have[i])
    free = perm[o:]
    base, pool = _pool_for(orc, shape, n_pages, rng)
    toks = rng.integers(0, shape.vocab, size=B)
    res = orc.decode_run(cfg, params, pool, toks, tables, lens, np.zeros(B, np.int32), free, 0, n_steps)
    assert res["status"] == 0
    assert (res["seq_lens"] == lens + n_steps).all()
    taken_per_req = (lens + n_steps) // PT - lens // PT
    assert res["free_head"] == int(taken_per_req.sum())
    new_pages = [res["page_tables"][i, have[i]:have[i] + taken_per_req[i]].tolist() for i in range(B)]
    flat = sorted(p for lst in new_pages for p in lst)
    assert flat == sorted(free[:res["free_head"]].tolist()) and len(set(flat)) == len(flat)
    # order: replay the counting argument step by step
    head, expect = 0, [[] for _ in range(B)]
    cur = lens.copy()
    for _ in range(n_steps):
        for i in range(B):
            cur[i] += 1
            if cur[i] % PT == 0:
                expect[i].append(int(free[head]))
                head += 1
    assert new_pages == expect
    # the original entries are untouched
    for i in range(B):
        assert (res["page_tables"][i, :have[i]] == tables[i, :have[i]]).all()


def test_requests_freeze_when_pages_run_out_or_the_table_is_full(orc):
    shape = MiniShape(n_layers=1)
    rng = np.random.default_rng(5)
    w = random_weights(shape, rng)
    cfg, params = orc.make_cfg(shape), orc.params_from_arrays(w)
    lens = np.array([14, 14, 3], np.int32)
    n_pages = 8
    perm = rng.permutation(n_pages).astype(np.int32)
    tables = np.full((3, 2), -1, np.int32)
    tables[:, 0] = perm[:3]
    free = perm[3:4]                          # one page for two requests that both need one at step 2
    base, pool = _pool_for(orc, shape, n_pages, rng)
    toks = rng.integers(0, shape.vocab, size=3)
    res = orc.decode_run(cfg, params, pool, toks, tables, lens, np.zeros(3, np.int32), free, 0, 20)
    # request 0 gets the page and runs until its 2-page table is full (length 31 is the last slot);
    # request 1 freezes at length 15; request 2 crosses no page until length 16, then freezes too
    assert res["status"] == 3
    assert res["seq_lens"].tolist() == [31, 15, 15]
    assert res["page_tables"][0, 1] == free[0] and res["page_tables"][1, 1] == -1 and res["page_tables"][2, 1] == -1
    assert res["free_head"] == 1


def test_teacher_forcing_feeds_given_tokens_and_records_the_argmax(orc):
    shape = MiniShape(n_layers=1)
    rng = np.random.default_rng(6)
    w = random_weights(shape, rng)
    cfg, params = orc.make_cfg(shape), orc.params_from_arrays(w)
    lens = np.array([2, 9], np.int32)
    n_pages = 6
    tables = np.array([[0, -1], [1, -1]], np.int32)
    free = np.array([2, 3, 4, 5], np.int32)
    forced = rng.integers(0, shape.vocab, size=(5, 2)).astype(np.int32)
    toks = rng.integers(0, shape.vocab, size=2)
    base, pool = _pool_for(orc, shape, n_pages, rng)
    base2 = base.copy()
    pool2 = orc.make_pool(base2, n_pages, PT, orc.default_strides(shape, n_pages, PT))
    res = orc.decode_run(cfg, params, pool, toks, tables, lens, [0, 0], free, 0, 5, forced_tokens=forced)
    # the same thing, step by step by hand
    cur_t, cur_l = toks.astype(np.int32), lens.copy()
    for s in range(5):
        r = orc.decode_step(cfg, params, pool2, cur_t, tables, cur_l, [0, 0])
        assert (res["tokens"][s] == r["next"]).all()
        cur_t, cur_l = forced[s], cur_l + 1
    assert np.array_equal(base, base2)
