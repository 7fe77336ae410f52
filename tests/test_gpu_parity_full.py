"""GPU parity at the benchmark sizes, in the launch configuration bench.py times: the full
8B-shaped step (batch 64 and 256, bf16 and QSUN) is run on the GPU and a sample of its
requests is recomputed by the CPU oracle from exactly the bytes the GPU consumed.  The 14B-shaped
configurations have a module of their own (test_gpu_parity_14b.py: their pools need the memory these
fixtures hold)."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from paper_2603_02599_amd import binding as sun  # noqa: E402
from paper_2603_02599_amd import workloads as wl  # noqa: E402


@pytest.fixture(scope="module")
def H():
    import gpu_harness
    assert torch.cuda.is_available(), "these tests need the MI355X"
    sun.lib()
    return gpu_harness


@pytest.fixture(scope="module")
def dense8b(H):
    H.say("building 8B-shaped bf16 weights")
    sw = H.SharedWeights(wl.LLAMA_8B, "bf16", wl.SEED_BASE + 100)
    yield sw
    del sw
    torch.cuda.empty_cache()


@pytest.fixture(scope="module")
def quant8b(H):
    H.say("building 8B-shaped 4-bit weights (affine RTN, group 128)")
    sw = H.SharedWeights(wl.LLAMA_8B, "bf16", wl.SEED_BASE + 100, quant_mode="asym")
    for k in sun.QUANT_KEYS:           # dense projection sources are not needed any more
        sw.w[k] = None
    torch.cuda.empty_cache()
    yield sw
    del sw
    torch.cuda.empty_cache()


def _sample_rows(work, k, must=()):
    order = np.argsort(work.seq_lens, kind="stable")
    picks = {int(order[0]), int(order[-1])} | {int(r) for r in must}
    rng = np.random.default_rng(work.seed)
    while len(picks) < k:
        picks.add(int(rng.integers(0, work.batch)))
    return sorted(picks)


def _sampled_parity(H, work, shared, k, must=()):
    case = H.GpuCase(work, shared=shared)
    rows = _sample_rows(work, k, must)
    quant = shared.quant is not None
    H.say(f"{work.name} B={work.batch} quant={quant}: oracle on rows {rows} "
          f"(lengths {[int(work.seq_lens[r]) for r in rows]})")
    extracted = case.extract_pool(rows)
    used = extracted[3]
    case.step(flags=sun.SUN_VALIDATE)
    after = case.pool_pages_now(used)
    ref = H.oracle_step_next_to_gpu_cache(case, rows, extracted, after, quant=quant)
    got_logits = case.logits.cpu().numpy()[rows]
    got_next = case.next.cpu().numpy()[rows]
    rep = H.logits_report(got_logits, ref["logits"])
    H.say(f"   logits {rep}")
    H.check_logits(got_logits, ref["logits"], "bf16")
    near = H.check_next_tokens(got_next, ref["logits"], 2e-2)
    H.say(f"   near-tie rows {near}; appended K/V entries {ref['peer']}")
    # every request's argmax equals the argmax of the GPU's own logits (lowest index on ties)
    all_logits = case.logits
    assert torch.equal(case.next.long(), all_logits.argmax(dim=1))
    return case, rep


def test_cfg2_batch64_bf16_sampled(H, dense8b):
    _sampled_parity(H, wl.make_workload("cfg2"), dense8b, 8)


def test_cfg3_batch256_bf16_sampled(H, dense8b):
    work = wl.make_workload("cfg3")
    assert work.seq_lens.max() >= 8192
    _sampled_parity(H, work, dense8b, 8)


def test_cfg4_qsun_batch64_sampled(H, quant8b):
    _sampled_parity(H, wl.make_workload("cfg2"), quant8b, 8)


def test_cfg4_qsun_batch256_sampled(H, quant8b):
    _sampled_parity(H, wl.make_workload("cfg3"), quant8b, 4)


def test_cfg2_batch64_run_of_three_steps_sampled(H, dense8b):
    """sun_decode_run at the benchmark size: 3 steps of cfg2 with requests placed so that several cross a
    page boundary.  Page bookkeeping for all 64 requests is checked against a host replay of the counting
    argument; the oracle replays 6 sampled requests fed with the GPU's tokens."""
    n_steps = 3
    work = wl.make_workload("cfg2")
    work.seq_lens = (work.seq_lens - work.seq_lens % 16 + np.arange(work.batch) % 16).astype(np.int32)  # all residues mod 16
    rng = np.random.default_rng(work.seed + 9)
    work.page_tables, work.n_pages = wl.deal_page_tables(work.seq_lens, rng)
    B = work.batch
    cols = (int(work.seq_lens.max()) + n_steps) // 16 + 1
    wide = np.full((B, cols), -1, np.int32)
    wide[:, :work.max_pages] = work.page_tables
    referenced = np.zeros(work.n_pages, bool)
    referenced[work.page_tables[work.page_tables >= 0]] = True
    free = np.flatnonzero(~referenced).astype(np.int32)
    # host replay: which request takes which free page at which step
    expect, head, cur = wide.copy(), 0, work.seq_lens.copy()
    for _ in range(n_steps):
        for i in range(B):
            cur[i] += 1
            if cur[i] % 16 == 0:
                expect[i, cur[i] // 16] = free[head]
                head += 1
    assert head >= 8, "the test should exercise page allocation"
    work.page_tables = expect                      # the oracle sees the pages as already provided
    case = H.GpuCase(work, shared=dense8b)
    rows = sorted(set(_sample_rows(work, 4)) | {int(np.flatnonzero(work.seq_lens % 16 == 15)[0]),
                                                 int(np.flatnonzero(work.seq_lens % 16 == 14)[0])})
    H.say(f"cfg2 run of {n_steps} steps: oracle on rows {rows} (lengths {[int(work.seq_lens[r]) for r in rows]})")
    before_host, opool, tabs, used = case.extract_pool(rows)
    host = before_host  # the oracle pool aliases this array and mutates it
    before = before_host.copy()
    d_tab = torch.from_numpy(wide).cuda()
    d_tok, d_len = case.tokens.clone(), case.lens.clone()
    d_free = torch.from_numpy(free).cuda()
    d_head = torch.zeros(1, dtype=torch.int32, device="cuda")
    d_status = torch.zeros(1, dtype=torch.int32, device="cuda")
    d_out = torch.empty((n_steps, B), dtype=torch.int32, device="cuda")
    ws = torch.empty(sun.sun_workspace_bytes(case.cfg, B, cols), dtype=torch.uint8, device="cuda")
    sun.sun_decode_run(case.pool, case.weights, n_steps, d_tok, d_tab, d_len, case.ids, d_free, d_head, d_status,
                       d_out, case.logits, ws, flags=sun.SUN_VALIDATE)
    torch.cuda.synchronize()
    assert np.array_equal(d_tab.cpu().numpy(), expect) and int(d_head.cpu()[0]) == head and int(d_status.cpu()[0]) == 0
    assert np.array_equal(d_len.cpu().numpy(), work.seq_lens + n_steps)
    got = d_out.cpu().numpy()
    # the cache: nothing but the appended slots of the three steps has changed ...
    st = H.layout_strides(case.lay)
    st["k_layer"] = st["v_layer"] = len(used) * int(case.lay.k_page)
    mask = np.zeros(before.size, dtype=bool)
    for s in range(n_steps):
        mask |= H.appended_mask(work.shape, st, before.size, tabs, work.seq_lens[rows] + s)
    after = case.pool_pages_now(used)
    assert np.array_equal(after[~mask], before[~mask]), "GPU wrote outside the appended slots"
    # ... and every step, replayed by the oracle from the cache the GPU holds and fed the GPU's token
    fed = [work.tokens[rows]] + [got[s][rows] for s in range(n_steps - 1)]
    logits, cnt = H.replay_steps_on_gpu_cache(case, used, after, tabs, work.seq_lens[rows], fed, work.model_ids[rows])
    near = []
    for s in range(n_steps):
        near += [(s, rows[i]) for i in H.check_next_tokens(got[s][rows], logits[s], 2e-2)]
    last = case.logits.cpu().numpy()[rows]
    H.say(f"   last-step logits {H.logits_report(last, logits[-1])}")
    H.check_logits(last, logits[-1], "bf16")
    H.say(f"   near-ties {near}; pages taken {head}; appended K/V entries {cnt}")


def test_cfg2_batch64_continuous_batching_sampled(H, dense8b):
    """sun_decode_serve at the benchmark size: 64 rows of the 8B shape fed from 160 waiting requests with
    cfg2's lengths and short output budgets, 8 iterations, so that rows retire and are refilled inside the call.
    The schedule, tables, ring and counters of all rows are compared exactly with the oracle's bookkeeping (its
    loop without the model: with no end token the schedule does not depend on the tokens); the oracle's model
    then replays four requests (one that retires early, one admitted in mid-call, the shortest and the longest
    still running at the end), fed with the GPU's tokens."""
    slots, n_wait, n_steps = 64, 160, 8
    base = wl.make_workload("cfg2")
    rng = np.random.default_rng(base.seed + 21)
    lens = rng.integers(512, 4097, size=n_wait).astype(np.int32)
    lens[:8] = lens[:8] - lens[:8] % 16 + 12 + np.arange(8) % 4          # some cross a page boundary during the call
    budgets = rng.integers(2, 7, size=n_wait).astype(np.int32)
    budgets[3] = 40                                                        # one request runs through the whole call
    cols = (int(lens.max()) + 41) // 16 + 1
    have = lens // 16 + 1
    ring_n = 96
    n_pages = 1 + int(have.sum()) + ring_n
    perm = rng.permutation(n_pages).astype(np.int32)
    idle, o = int(perm[0]), 1
    tables = np.full((n_wait, cols), -1, np.int32)
    for r in range(n_wait):
        tables[r, :have[r]] = perm[o:o + have[r]]
        o += int(have[r])
    ring = [int(p) for p in perm[o:]]
    waiting = {"req": np.arange(n_wait, dtype=np.int32), "token": rng.integers(0, base.shape.vocab, size=n_wait).astype(np.int32),
               "tables": tables, "lens": lens, "model": rng.integers(0, 4, size=n_wait).astype(np.int32), "budget": budgets}
    owait = [{"req": r, "token": int(waiting["token"][r]), "table": tables[r], "len": int(lens[r]),
              "model": int(waiting["model"][r]), "budget": int(budgets[r])} for r in range(n_wait)]
    # the schedule, from the oracle's bookkeeping alone (any tokens: there is no end token)
    fake = np.zeros((n_steps, slots), np.int32)
    book = H.orc.serve_run(None, None, None, slots, cols, n_steps, owait, ring, idle, forced_tokens=fake, bookkeeping_only=True)
    assert book["retired"] > 60 and book["admitted"] > 120 and book["status"] == 0
    last = book["reqs"][-1]
    running = [int(q) for q in last if q >= 0]
    first_step = {q: min(w[0] for w in book["writes"] if w[2] == q) for q in set(w[2] for w in book["writes"])}
    early = next(q for q in range(slots) if budgets[q] <= 3)
    mid = next(q for q in running if first_step[q] >= 2)
    picks = sorted({early, mid, min(running, key=lambda q: lens[q]), max(running, key=lambda q: lens[q]), 3})
    # tables of the picked requests as they stand after the call (pages taken during it included)
    ptab = tables[picks].copy()
    for (s, row, q, page, slot) in book["writes"]:
        if q in picks:
            ptab[picks.index(q), (int(lens[q]) + (s - first_step[q])) // 16] = page
    work = base
    work.page_tables, work.n_pages = np.full((slots, cols), -1, np.int32), n_pages
    case = H.GpuCase(work, shared=dense8b)
    case.work.page_tables = ptab                      # for the pool extraction below only
    before_host, opool, tabs, used = case.extract_pool(list(range(len(picks))))
    before = before_host.copy()
    H.say(f"cfg2 serve: {book['admitted']} admitted, {book['retired']} retired in {n_steps} steps; oracle model on requests "
          f"{picks} (lengths {[int(lens[q]) for q in picks]}, budgets {[int(budgets[q]) for q in picks]})")
    state = sun.ServeTensors(slots, cols, waiting, ring, n_pages, idle)
    ws = torch.empty(sun.sun_serve_workspace_bytes(case.cfg, slots, cols), dtype=torch.uint8, device="cuda")
    toks = torch.empty((n_steps, slots), dtype=torch.int32, device="cuda")
    reqs = torch.empty((n_steps, slots), dtype=torch.int32, device="cuda")
    sun.sun_decode_serve(case.pool, case.weights, n_steps, state, toks, reqs, case.logits, ws,
                         flags=sun.SUN_VALIDATE | sun.SUN_SERVE_RESET)
    torch.cuda.synchronize()
    got_t, got_r = toks.cpu().numpy(), reqs.cpu().numpy()
    # bookkeeping of all rows: exact (the replay is fed the GPU's tokens, which it records and feeds back)
    book = H.orc.serve_run(None, None, None, slots, cols, n_steps, owait, ring, idle, forced_tokens=got_t, bookkeeping_only=True)
    assert np.array_equal(got_r, book["reqs"]) and (got_t[got_r < 0] == -1).all()
    assert np.array_equal(state.page_tables.cpu().numpy(), book["tables"])
    assert state.seq_lens.cpu().tolist() == book["len"] and state.slot_left.cpu().tolist() == book["left"]
    assert state.slot_req.cpu().tolist() == book["req"] and state.token_ids.cpu().tolist() == book["token"]
    cnt = state.counters.cpu().tolist()
    rg = state.ring.cpu().numpy()
    assert [int(rg[i % n_pages]) for i in range(cnt[1], cnt[2])] == book["ring"]
    assert [cnt[0], cnt[3], cnt[4], cnt[5], cnt[6], cnt[7]] == [book["whead"], 0, book["retired"], book["admitted"],
                                                                book["generated"], n_steps]
    # the model, for the picked requests: each one's own steps, each replayed by the oracle from the cache the
    # GPU holds and fed the token the GPU was fed
    glogits = case.logits.cpu().numpy()
    st = H.layout_strides(case.lay)
    st["k_layer"] = st["v_layer"] = len(used) * int(case.lay.k_page)
    after = case.pool_pages_now(used)
    mask = np.zeros(before.size, dtype=bool)
    near, cnt = [], {}
    for j, q in enumerate(picks):
        where = [(s, int(np.flatnonzero(got_r[s] == q)[0])) for s in range(n_steps) if (got_r[s] == q).any()]
        fed = [waiting["token"][q:q + 1]] + [got_t[s, row:row + 1] for s, row in where[:-1]]
        logits, c = H.replay_steps_on_gpu_cache(case, used, after, tabs[j:j + 1], lens[q:q + 1], fed, waiting["model"][q:q + 1])
        cnt = {k2: cnt.get(k2, 0) + v for k2, v in c.items()}
        for n, (s, row) in enumerate(where):
            near += [(s, q) for _ in H.check_next_tokens(got_t[s, row:row + 1], logits[n], 2e-2)]
            mask |= H.appended_mask(work.shape, st, before.size, tabs[j:j + 1], lens[q:q + 1] + n)
        if where[-1][0] == n_steps - 1:
            H.check_logits(glogits[where[-1][1]][None], logits[-1], "bf16")
    assert np.array_equal(after[~mask], before[~mask]), "GPU wrote outside the appended slots of the picked requests"
    H.say(f"   near-ties {near}; appended K/V entries of the picked requests {cnt}")


def test_prefill_8b_shape(H, dense8b):
    """sun_prefill at the 8B shape: a 48-token prompt through all 32 layers.  Every position's entries depend on
    the bf16-rounded entries of the positions before it, so against the oracle's cache-free forward the
    legitimate one-ulp roundings feed forward through 48 positions and 32 layers (measured that way: 40 % of the
    entries an ulp apart, logits 0.02 apart); the small shapes are compared with that forward
    (test_gpu_prefill.py).  Here every prompt position is compared on its own, as the causal forward defines it:
    position r is the decode step of token r over positions 0..r (Eq. 2 row by row), which the oracle computes
    from the cache the GPU left, next to the GPU's entry for position r (decode_step_peer).  All 48 positions
    go through the oracle as one batch of 48 rows over the one page table."""
    shape, T = wl.LLAMA_8B, 48
    work = wl.make_workload("cfg2", batch=1, n_models=1, seed=wl.SEED_BASE + 31)
    work.seq_lens = np.array([T], np.int32)
    rng = np.random.default_rng(work.seed)
    work.page_tables, work.n_pages = wl.deal_page_tables(work.seq_lens, rng)
    case = H.GpuCase(work, shared=dense8b)
    toks = rng.integers(0, shape.vocab, size=T).astype(np.int32)
    before_host, _, tabs, used = case.extract_pool([0])
    before = before_host.copy()
    H.say(f"prefill 8B shape, {T} tokens")
    d_tok = torch.from_numpy(toks).cuda()
    table = case.tables[0].contiguous()
    ws = torch.empty(sun.sun_prefill_workspace_bytes(case.cfg, T, table.numel()), dtype=torch.uint8, device="cuda")
    logits = torch.empty(shape.vocab, dtype=torch.float32, device="cuda")
    nxt = torch.empty(1, dtype=torch.int32, device="cuda")
    sun.sun_prefill(case.pool, case.weights, d_tok, table, 0, 0, logits, nxt, ws, flags=sun.SUN_VALIDATE)
    torch.cuda.synchronize()
    after = case.pool_pages_now(used)
    st = H.layout_strides(case.lay)
    st["k_layer"] = st["v_layer"] = len(used) * int(case.lay.k_page)
    probe = np.zeros(before.size, np.uint16)
    ones = np.ones((shape.n_layers, T, shape.n_kv_heads, shape.head_dim), np.uint16)
    H.orc.kv_ingest(probe, st, ones, ones, 0, tabs[0])
    written = probe != 0
    assert np.array_equal(after[~written], before[~written]), "the prefill wrote outside the prompt's slots"
    host = after.copy()
    pool, peer = H.orc.make_pool(host, len(used), 16, st), H.orc.make_pool(after, len(used), 16, st)
    tol_abs, tol_rel, max_off = H.kv_bound("bf16", False)
    res = H.orc.decode_step_peer(H.orc.make_cfg(shape), case.oracle_params(), pool, peer, toks, np.repeat(tabs[:1], T, axis=0),
                                 np.arange(T, dtype=np.int32), np.zeros(T, np.int32), tol_abs, tol_rel)
    cnt = res["peer"]
    H.say(f"   cache entries {cnt}")
    assert cnt["rejected"] == 0 and np.array_equal(host, after) and sum(cnt.values()) == int(written.sum())
    assert cnt["neighbour"] + cnt["by_value"] <= max_off * sum(cnt.values())
    got = logits.cpu().numpy()
    H.say(f"   first-token logits {H.logits_report(got[None], res['logits'][-1][None])}")
    H.check_logits(got[None], res["logits"][-1][None], "bf16")
    H.check_next_tokens(np.array([int(nxt.cpu()[0])]), res["logits"][-1][None], 2e-2)
