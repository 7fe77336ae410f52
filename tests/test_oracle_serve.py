"""Pins of the oracle's continuous-batching loop (CPU only).

What a request generates is fixed by Eq. 3 alone: greedy decoding of its own prompt, whatever rows it
shares a batch with and whenever it is admitted; brute force (a cache-free forward per new token) gives the
expected tokens.  The bookkeeping (who sits in which row when, which pages go where) is fixed by counting
arguments worked out by hand below."""
import numpy as np
import pytest

from helpers import MiniShape, random_weights
from test_oracle_pins import PT, _pool_for


def _setup(orc, lens, budgets, n_pages, seed, table_cols, models=None):
    """Requests with random prompts, prefilled by the oracle's causal forward into pages dealt from a
    shuffled permutation; page perm[0] is the idle page; the rest not handed out is the free ring."""
    shape = MiniShape()
    rng = np.random.default_rng(seed)
    w = random_weights(shape, rng)
    cfg, params = orc.make_cfg(shape), orc.params_from_arrays(w)
    base, pool = _pool_for(orc, shape, n_pages, rng)
    st = orc.default_strides(shape, n_pages, PT)
    perm = rng.permutation(n_pages).astype(np.int32)
    idle, o = int(perm[0]), 1
    waiting, prompts = [], []
    for r, (L, b) in enumerate(zip(lens, budgets)):
        prompt = rng.integers(0, shape.vocab, size=L + 1)
        have = L // PT + 1
        row = np.full(table_cols, -1, np.int32)
        row[:have] = perm[o:o + have]
        o += have
        if L:
            _, K, V = orc.full_forward(cfg, params, prompt[:L], round_kv=True, want_kv=True)
            orc.kv_ingest(base, st, orc.bf16_bits(K), orc.bf16_bits(V), 0, row, PT)
        waiting.append({"req": 100 + r, "token": int(prompt[L]), "table": row, "len": L,
                        "model": 0 if models is None else models[r], "budget": b})
        prompts.append(prompt)
    return shape, cfg, params, base, pool, waiting, prompts, [int(p) for p in perm[o:]], idle


def _greedy(orc, cfg, params, prompt, n, eos=-1):
    toks, out = list(prompt), []
    for _ in range(n):
        nxt = int(np.argmax(orc.full_forward(cfg, params, toks, round_kv=True)[-1]))
        out.append(nxt)
        toks.append(nxt)
        if nxt == eos:
            break
    return out


def _per_request(res):
    got = {}
    for s in range(res["tokens"].shape[0]):
        for i in range(res["tokens"].shape[1]):
            if res["reqs"][s, i] >= 0:
                got.setdefault(int(res["reqs"][s, i]), []).append(int(res["tokens"][s, i]))
    return got


@pytest.mark.parametrize("slots", [1, 2, 5])
def test_every_request_gets_its_own_greedy_continuation(orc, slots):
    lens, budgets = [3, 14, 30, 0, 17], [6, 3, 20, 5, 1]
    shape, cfg, params, base, pool, waiting, prompts, ring, idle = _setup(orc, lens, budgets, 40, 700 + slots, 4)
    res = orc.serve_run(cfg, params, pool, slots, 4, 40, waiting, ring, idle)
    got = _per_request(res)
    for r, w in enumerate(waiting):
        assert got[w["req"]] == _greedy(orc, cfg, params, prompts[r], budgets[r]), f"request {r}"
    assert res["retired"] == 5 and res["admitted"] == 5 and res["generated"] == sum(budgets) and res["status"] == 0
    assert all(q == -1 for q in res["req"])
    # every page is back: the ring holds each non-idle page once, the rows hold only the idle page
    assert sorted(res["ring"]) == sorted(set(range(40)) - {idle})
    assert (res["tables"][:, 0] == idle).all() and (res["tables"][:, 1:] == -1).all()


def test_schedule_by_hand(orc):
    """Two rows, budgets 3, 1, 2, 2 and no end token: rows after each step work out by hand to
       step 0: [a b]  b done -> c enters row 1
       step 1: [a c]
       step 2: [a c]  both done -> d enters row 0, row 1 stays idle
       step 3: [d -]
       step 4: [d -]  done."""
    lens, budgets = [2, 5, 1, 9], [3, 1, 2, 2]
    shape, cfg, params, base, pool, waiting, prompts, ring, idle = _setup(orc, lens, budgets, 12, 710, 2)
    res = orc.serve_run(cfg, params, pool, 2, 2, 6, waiting, ring, idle)
    a, b, c, d = 100, 101, 102, 103
    assert res["reqs"].tolist() == [[a, b], [a, c], [a, c], [d, -1], [d, -1], [-1, -1]]
    assert (res["tokens"][res["reqs"] < 0] == -1).all() and res["steps"] == 6


def test_pages_return_in_table_order_and_are_reused_first_in_first_out(orc):
    """One row.  Request x (length 15, 2 tokens) crosses into a second page, taking ring[0]; when it retires
    its two pages go to the ring's tail in column order; request y then needs one page at its second step and
    takes what is now the head, ring[1]."""
    lens, budgets = [15, 15], [2, 2]
    shape, cfg, params, base, pool, waiting, prompts, ring, idle = _setup(orc, lens, budgets, 7, 720, 2)
    x_page, y_page = int(waiting[0]["table"][0]), int(waiting[1]["table"][0])
    assert len(ring) == 4
    mid = orc.serve_run(cfg, params, pool, 1, 2, 1, waiting, ring, idle)
    assert mid["tables"][0].tolist() == [x_page, ring[0]] and mid["ring"] == ring[1:] and mid["len"] == [16]
    res = orc.serve_run(cfg, params, pool, 1, 2, 2, waiting, ring, idle, state=mid)
    assert res["reqs"][:, 0].tolist() == [100, 101]
    assert res["tables"][0].tolist() == [y_page, ring[1]] and res["ring"] == ring[2:] + [x_page, ring[0]]
    # and the split call equals one call of three steps
    shape, cfg, params, base2, pool2, waiting2, _, ring2, idle2 = _setup(orc, lens, budgets, 7, 720, 2)
    one = orc.serve_run(cfg, params, pool2, 1, 2, 3, waiting2, ring2, idle2)
    assert np.array_equal(one["tokens"], np.concatenate([mid["tokens"], res["tokens"]])) and one["ring"] == res["ring"]
    assert np.array_equal(base, base2)


def test_admission_waits_for_pages_and_keeps_the_order(orc):
    """Three rows but only two free pages.  p (length 10, 30 tokens: positions up to 39, three pages, holds
    one) reserves both free pages.  q (length 3, 20 tokens: needs one more page) does not fit, and r behind it
    (length 2, 3 tokens: needs none) must wait too.  They enter when p retires after step 29 and its three pages
    are back; idle rows are filled in row order, so q takes row 0 and r row 1, and row 2 is never used."""
    lens, budgets = [10, 3, 2], [30, 20, 3]
    shape, cfg, params, base, pool, waiting, prompts, ring, idle = _setup(orc, lens, budgets, 6, 730, 3)
    assert len(ring) == 2
    res = orc.serve_run(cfg, params, pool, 3, 3, 51, waiting, ring, idle)
    reqs = res["reqs"]
    assert (reqs[:30, 0] == 100).all() and (reqs[:30, 1:] == -1).all()
    assert (reqs[30:50, 0] == 101).all() and (reqs[30:33, 1] == 102).all() and (reqs[33:, 1] == -1).all()
    assert (reqs[:, 2] == -1).all() and (reqs[50] == -1).all()
    got = _per_request(res)
    for r in range(3):
        assert got[100 + r] == _greedy(orc, cfg, params, prompts[r], budgets[r])
    assert res["status"] == 0 and len(res["ring"]) == 5


def test_end_token_retires_early_and_frees_the_reservation(orc):
    lens, budgets = [14, 4], [12, 3]
    shape, cfg, params, base, pool, waiting, prompts, ring, idle = _setup(orc, lens, budgets, 4, 740, 2)
    assert len(ring) == 1
    full = _greedy(orc, cfg, params, prompts[0], 12)
    eos = full[2]
    stop = full.index(eos)                     # first time it appears (may be before the third token)
    res = orc.serve_run(cfg, params, pool, 2, 2, 8, waiting, ring, idle, eos_id=eos)
    got = _per_request(res)
    assert got[100] == full[:stop + 1]
    # request 1 was admitted together with request 0 (it needs no further page), and is cut short only if it
    # generates the end token itself
    want1 = _greedy(orc, cfg, params, prompts[1], 3, eos=eos)
    assert got[101] == want1
    assert res["retired"] == 2 and sorted(res["ring"]) == sorted(set(range(4)) - {idle})


def test_budget_is_cut_to_the_table(orc):
    lens, budgets = [20], [100]
    shape, cfg, params, base, pool, waiting, prompts, ring, idle = _setup(orc, lens, budgets, 6, 750, 2)
    res = orc.serve_run(cfg, params, pool, 1, 2, 20, waiting, ring, idle)
    got = _per_request(res)
    assert len(got[100]) == 12 and got[100] == _greedy(orc, cfg, params, prompts[0], 12)   # positions 20..31
    assert res["status"] == 2 and res["retired"] == 1


def test_bookkeeping_alone_gives_the_same_schedule(orc):
    """Without an end token the schedule and the page accounting do not depend on the tokens: the loop with the
    model switched off (fed any tokens) must reproduce who sat where, the tables, the ring and every write."""
    lens, budgets = [3, 14, 30, 0, 17, 15], [6, 3, 20, 5, 1, 9]
    shape, cfg, params, base, pool, waiting, prompts, ring, idle = _setup(orc, lens, budgets, 14, 760, 4)
    full = orc.serve_run(cfg, params, pool, 2, 4, 30, waiting, ring, idle)
    fake = np.full((30, 2), 5, np.int32)
    book = orc.serve_run(None, None, None, 2, 4, 30, waiting, ring, idle, forced_tokens=fake, bookkeeping_only=True)
    assert np.array_equal(book["reqs"], full["reqs"]) and book["ring"] == full["ring"] and book["writes"] == full["writes"]
    assert np.array_equal(book["tables"], full["tables"]) and book["retired"] == full["retired"] == 6
    assert (book["tokens"][book["reqs"] >= 0] == 5).all()
