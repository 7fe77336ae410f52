"""GPU parity of sun_decode_serve (continuous batching on the device) against the oracle's loop, through
the C ABI.  The GPU runs freely; the oracle replays the same iterations fed with the GPU's tokens, so one
legitimate near-tie cannot cascade.  Compared: which request sat in which row at every step (exact), every
token against the oracle's logits of that row and step, the rows, the queue head, the page ring and the
counters at the end, and every cache entry written."""
import numpy as np
import pytest
import torch

from paper_2603_02599_amd import binding as sun, workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def H():
    import gpu_harness
    assert torch.cuda.is_available(), "these tests need the MI355X"
    sun.lib()
    return gpu_harness


class _Setup:
    def __init__(self, H, shape, dtype, slots, lens, budgets, ring_n, cols, seed, quant=None, n_models=3, extra=None):
        """extra: {request: column} gives that request one more page of its own at a column past its prompt's."""
        rng = np.random.default_rng(seed)
        lens, budgets = np.asarray(lens, np.int32), np.asarray(budgets, np.int32)
        have = lens // 16 + 1
        extra = extra or {}
        n_pages = 1 + int(have.sum()) + len(extra) + ring_n
        perm = rng.permutation(n_pages).astype(np.int32)
        self.idle, o = int(perm[0]), 1
        tables = np.full((len(lens), cols), -1, np.int32)
        for r in range(len(lens)):
            tables[r, :have[r]] = perm[o:o + have[r]]
            o += int(have[r])
            if r in extra:
                assert extra[r] >= have[r]
                tables[r, extra[r]] = perm[o]
                o += 1
        self.ring = [int(p) for p in perm[o:]]
        work = wl.make_workload("cfg1", shape=shape, dtype=dtype, batch=slots, n_models=n_models, seed=seed)
        work.page_tables, work.n_pages = np.full((slots, cols), -1, np.int32), n_pages
        self.case = H.GpuCase(work, quant_mode=quant)
        self.waiting = {"req": 500 + np.arange(len(lens), dtype=np.int32),
                        "token": rng.integers(0, shape.vocab, size=len(lens)).astype(np.int32),
                        "tables": tables, "lens": lens, "model": rng.integers(0, n_models, size=len(lens)).astype(np.int32),
                        "budget": budgets}
        self.shape, self.dtype, self.slots, self.cols, self.n_pages, self.quant = shape, dtype, slots, cols, n_pages, quant
        self.before = H.to_np(self.case.pool_mem).copy()

    def oracle_waiting(self):
        w = self.waiting
        return [{"req": int(w["req"][r]), "token": int(w["token"][r]), "table": w["tables"][r], "len": int(w["lens"][r]),
                 "model": int(w["model"][r]), "budget": int(w["budget"][r])} for r in range(len(w["req"]))]


def _serve_and_compare(H, S, steps_per_call, eos=-1):
    case, slots, cols = S.case, S.slots, S.cols
    case.pool_mem.copy_(torch.from_numpy(S.before.view(np.int16)).cuda().view(torch.bfloat16))
    state = sun.ServeTensors(slots, cols, S.waiting, S.ring, S.n_pages, S.idle, eos_id=eos)
    ws = torch.empty(sun.sun_serve_workspace_bytes(case.cfg, slots, cols), dtype=torch.uint8, device="cuda")
    total = sum(steps_per_call)
    toks = torch.full((total, slots), -7, dtype=torch.int32, device="cuda")
    reqs = torch.full((total, slots), -7, dtype=torch.int32, device="cuda")
    done = 0
    for k, n in enumerate(steps_per_call):
        sun.sun_decode_serve(case.pool, case.weights, n, state, toks[done:done + n], reqs[done:done + n], case.logits, ws,
                             flags=sun.SUN_VALIDATE | (sun.SUN_SERVE_RESET if k == 0 else 0))
        done += n
    torch.cuda.synchronize()
    got_t, got_r = toks.cpu().numpy(), reqs.cpu().numpy()
    # the oracle, on its own copy of the pool, fed with the GPU's tokens
    host = S.before.copy()
    opool = H.orc.make_pool(host, S.n_pages, 16, H.layout_strides(case.lay))
    ref = H.orc.serve_run(H.orc.make_cfg(S.shape), case.oracle_params(), opool, slots, cols, total, S.oracle_waiting(),
                          S.ring, S.idle, eos_id=eos, forced_tokens=got_t, keep_logits=True,
                          **({"mode": 1} if S.quant else {}))
    assert np.array_equal(got_r, ref["reqs"]), "a different request sat in some row at some step"
    assert (got_t[got_r < 0] == -1).all()
    tol = 1e-4 if S.dtype == "f32" else 2e-2
    near = []
    for s in range(total):
        rows = np.nonzero(got_r[s] >= 0)[0]
        if len(rows):
            near += [(s, int(rows[i])) for i in H.check_next_tokens(got_t[s][rows], ref["logits"][s][rows], tol)]
    last_rows = np.nonzero(got_r[-1] >= 0)[0]
    if len(last_rows):
        H.check_logits(case.logits.cpu().numpy()[last_rows], ref["logits"][-1][last_rows], S.dtype)
    # rows, queue, ring, counters
    assert state.slot_req.cpu().tolist() == ref["req"] and state.slot_left.cpu().tolist() == ref["left"]
    assert state.seq_lens.cpu().tolist() == ref["len"] and state.token_ids.cpu().tolist() == ref["token"]
    assert state.model_ids.cpu().tolist() == ref["model"]
    assert np.array_equal(state.page_tables.cpu().numpy(), ref["tables"])
    cnt = state.counters.cpu().tolist()
    ring = state.ring.cpu().numpy()
    assert [int(ring[i % S.n_pages]) for i in range(cnt[1], cnt[2])] == ref["ring"]
    assert [cnt[0], cnt[3], cnt[4], cnt[5], cnt[6], cnt[7]] == [ref["whead"], ref["status"], ref["retired"],
                                                                ref["admitted"], ref["generated"], ref["steps"]]
    # cache: what the oracle's requests wrote, nothing else (the idle page belongs to the idle rows)
    after = H.to_np(case.pool_mem).copy()
    st = H.layout_strides(case.lay)
    probe = np.zeros(after.size, np.uint16)       # the idle page's elements, by the oracle's addressing
    ones = np.ones((S.shape.n_layers, 16, S.shape.n_kv_heads, S.shape.head_dim), np.uint16)
    H.orc.kv_ingest(probe, st, ones, ones, 0, np.array([S.idle], np.int32))
    idle_elems = probe != 0
    after[idle_elems] = S.before[idle_elems]
    mask = np.zeros(after.size, bool)             # the slots Eq. 4 says were appended to, over all steps
    one = np.ones((S.shape.n_layers, 1, S.shape.n_kv_heads, S.shape.head_dim), np.uint16)
    for page, slot in {(w[3], w[4]) for w in ref["writes"]}:
        probe[:] = 0
        H.orc.kv_ingest(probe, st, one, one, slot, np.array([page], np.int32))
        mask |= probe != 0
    assert not (mask & idle_elems).any()
    off, n_written = H.check_appended_kv(after, host, S.before, mask, S.dtype, abs_tol=2e-5, quant=S.quant is not None)
    H.say(f"   serve {S.dtype} quant={S.quant} eos={eos}: {cnt[6]} tokens, {cnt[5]} admitted, {cnt[4]} retired, status "
          f"{cnt[3]}; near-ties {near}; K/V off by one ulp: {off} of {n_written}")
    return got_t, got_r, ref


def test_serve_fp32_with_scarce_pages_in_one_call_and_in_two(H):
    H.say("serve: fp32 tiny, 4 rows, 9 requests, few free pages")
    S = _Setup(H, wl.TINY, "f32", 4, [0, 15, 16, 31, 62, 250, 5, 40, 17], [5, 20, 3, 18, 1, 30, 7, 2, 12], 3, 18, 500)
    t1, r1, ref = _serve_and_compare(H, S, [45])
    assert ref["retired"] == 9 and ref["status"] == 0 and sorted(ref["ring"]) == sorted(set(range(S.n_pages)) - {S.idle})
    # admission really waited for pages at some point: some step has an idle row while requests are waiting
    first_admit = {int(q): int(np.nonzero((r1 == q).any(axis=1))[0][0]) for q in S.waiting["req"]}
    assert any((r1[s] < 0).any() and any(first_admit[int(q)] > s for q in S.waiting["req"]) for s in range(45))
    t2, r2, _ = _serve_and_compare(H, S, [20, 25])
    assert np.array_equal(r1, r2) and np.array_equal(t1, t2)


def test_serve_end_token(H):
    H.say("serve: end token retires a request early")
    S = _Setup(H, wl.TINY, "f32", 3, [10, 3, 33, 8], [12, 9, 10, 6], 6, 6, 510)
    t0, r0, _ = _serve_and_compare(H, S, [14])
    eos = int(t0[2][0])                     # the third token of the request in row 0
    t1, r1, ref = _serve_and_compare(H, S, [14], eos=eos)
    n0 = int((r1 == r0[0][0]).sum())
    assert n0 <= 3 and ref["retired"] >= 1 and not np.array_equal(r0, r1)


@pytest.mark.parametrize("quant", [None, "asym"])
def test_serve_bf16_small(H, quant):
    H.say(f"serve: bf16 small128 quant={quant}, 6 rows, 14 requests")
    lens = [3, 14, 100, 255, 300, 17, 47, 511, 9, 128, 64, 1, 200, 33]
    budgets = [6, 18, 4, 9, 20, 2, 16, 5, 11, 3, 17, 8, 1, 10]
    S = _Setup(H, wl.SMALL128, "bf16", 6, lens, budgets, 5, 34, 520, quant=quant)
    _, _, ref = _serve_and_compare(H, S, [30])
    assert ref["retired"] >= 12 and ref["status"] == 0


def test_serve_validation(H):
    S = _Setup(H, wl.TINY, "f32", 2, [5, 20], [3, 3], 4, 4, 530)
    case = S.case
    ws = torch.empty(sun.sun_serve_workspace_bytes(case.cfg, 2, 4), dtype=torch.uint8, device="cuda")
    out = torch.empty((2, 2), dtype=torch.int32, device="cuda")

    def call(**kw):
        ring = kw.pop("ring", S.ring)
        idle = kw.pop("idle", S.idle)
        waiting = dict(S.waiting, **kw)
        st = sun.ServeTensors(2, 4, waiting, ring, S.n_pages, idle)
        sun.sun_decode_serve(case.pool, case.weights, 2, st, out, out.clone(), None, ws,
                             flags=sun.SUN_VALIDATE | sun.SUN_SERVE_RESET)

    for kw, status in (({"ring": S.ring[:-1] + [S.ring[0]]}, 5), ({"ring": S.ring[:-1] + [int(S.waiting["tables"][0, 0])]}, 5),
                       ({"idle": S.ring[0]}, 5), ({"idle": S.n_pages}, 5),
                       ({"token": np.array([1, S.shape.vocab], np.int32)}, 9), ({"model": np.array([0, 9], np.int32)}, 7),
                       ({"lens": np.array([5, 64], np.int32)}, 6), ({"budget": np.array([0, 3], np.int32)}, 6),
                       ({"lens": np.array([5, 40], np.int32)}, 5)):
        with pytest.raises(sun.SunError) as e:
            call(**kw)
        assert e.value.status == status, (kw, e.value.status)
    call()
    torch.cuda.synchronize()


def test_serve_many_rows(H):
    """More rows than one 64-row projection tile and more waiting requests than rows: 130 rows, 300 short
    requests, so that dozens of rows retire and refill in every iteration."""
    H.say("serve: fp32 tiny, 130 rows, 300 requests")
    rng = np.random.default_rng(540)
    lens = rng.integers(0, 90, size=300)
    budgets = rng.integers(1, 7, size=300)
    S = _Setup(H, wl.TINY, "f32", 130, lens, budgets, 40, 8, 541)
    _, r, ref = _serve_and_compare(H, S, [7, 6])
    assert ref["admitted"] == 300 and ref["retired"] > 250 and ref["status"] == 0
    assert (r[0] >= 0).all() and (r[-1] < 0).any()


def test_serve_wide_tables(H):
    """Page tables of 140 columns (the bookkeeping walks a row 64 columns at a time): prompts that end in the
    first, second and third stretch of 64 columns, and two requests that bring a page of their own far past
    their prompt (columns 70 and 137), which counts as held and goes back to the ring in column order."""
    H.say("serve: fp32 tiny, 3 rows, 8 requests, 140-column tables")
    lens = [2100, 1023, 1024, 30, 1500, 2047, 700, 2200]
    budgets = [10, 20, 5, 30, 17, 3, 12, 25]
    S = _Setup(H, wl.TINY, "f32", 3, lens, budgets, 4, 140, 550, extra={3: 137, 6: 70})
    _, _, ref = _serve_and_compare(H, S, [30, 40])
    assert ref["retired"] == 8 and ref["status"] == 0
    assert sorted(ref["ring"]) == sorted(set(range(S.n_pages)) - {S.idle})


def test_serve_without_retirement_equals_the_run(H):
    """With as many rows as requests and budgets longer than the call, continuous batching has nothing to retire
    or admit after the start, and must do exactly what sun_decode_run does for the same requests: same tokens,
    same pages taken in the same order, same cache bits."""
    H.say("serve == run when nobody retires")
    lens = [3, 15, 16, 31, 62, 250, 5, 40]
    S = _Setup(H, wl.SMALL128, "bf16", len(lens), lens, [20] * len(lens), 24, 18, 550)
    case, n_steps, B = S.case, 14, len(lens)
    state = sun.ServeTensors(B, S.cols, S.waiting, S.ring, S.n_pages, S.idle)
    ws = torch.empty(sun.sun_serve_workspace_bytes(case.cfg, B, S.cols), dtype=torch.uint8, device="cuda")
    toks = torch.empty((n_steps, B), dtype=torch.int32, device="cuda")
    reqs = torch.empty((n_steps, B), dtype=torch.int32, device="cuda")
    sun.sun_decode_serve(case.pool, case.weights, n_steps, state, toks, reqs, case.logits, ws,
                         flags=sun.SUN_VALIDATE | sun.SUN_SERVE_RESET)
    torch.cuda.synchronize()
    pool_serve, logits_serve = case.pool_mem.clone(), case.logits.clone()
    assert (reqs.cpu().numpy() == S.waiting["req"][None, :]).all()
    # the same requests through sun_decode_run on a fresh copy of the pool
    case.pool_mem.copy_(torch.from_numpy(S.before.view(np.int16)).cuda().view(torch.bfloat16))
    d_tok = torch.from_numpy(S.waiting["token"]).cuda()
    d_tab = torch.from_numpy(S.waiting["tables"]).cuda()
    d_len = torch.from_numpy(S.waiting["lens"]).cuda()
    d_ids = torch.from_numpy(S.waiting["model"]).cuda()
    d_free = torch.tensor(S.ring, dtype=torch.int32, device="cuda")
    d_head = torch.zeros(1, dtype=torch.int32, device="cuda")
    d_status = torch.zeros(1, dtype=torch.int32, device="cuda")
    out = torch.empty((n_steps, B), dtype=torch.int32, device="cuda")
    sun.sun_decode_run(case.pool, case.weights, n_steps, d_tok, d_tab, d_len, d_ids, d_free, d_head, d_status, out,
                       case.logits, ws, flags=sun.SUN_VALIDATE)
    torch.cuda.synchronize()
    assert torch.equal(out, toks) and torch.equal(case.logits, logits_serve)
    assert torch.equal(d_tab, state.page_tables) and torch.equal(d_len, state.seq_lens)
    assert int(d_head.cpu()[0]) == int(state.counters.cpu()[1]) and int(d_status.cpu()[0]) == 0
    assert torch.equal(case.pool_mem, pool_serve)
