"""GPU parity of the multi-step run (sun_decode_run) against the oracle's run, through the C ABI.

The GPU decodes freely for n steps.  The oracle then replays the same steps fed with the GPU's tokens
(teacher forcing), so one legitimate near-tie cannot make every later step look wrong: at every step the
GPU's token must be the oracle's argmax, or the runner-up of a documented near-tie.  Page tables, lengths,
free-list head, status and every cache entry written during the run are compared as well."""
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


def _run_case(H, shape, dtype, lens, n_steps, quant=None, spare_pages=24, n_free_cap=None, max_pages=None, seed=40):
    rng = np.random.default_rng(seed)
    lens = np.asarray(lens, np.int32)
    B = len(lens)
    work = wl.make_workload("cfg1", shape=shape, dtype=dtype, batch=B, seed=seed)
    work.seq_lens = lens
    need = (lens.astype(np.int64) + 1 + 15) // 16
    n_pages = int(need.sum()) + spare_pages
    perm = rng.permutation(n_pages).astype(np.int32)
    mp = max_pages if max_pages is not None else int((lens + n_steps).max()) // 16 + 1
    tables = np.full((B, mp), -1, np.int32)
    o = 0
    for i in range(B):
        tables[i, :need[i]] = perm[o:o + need[i]]
        o += int(need[i])
    free = perm[o:] if n_free_cap is None else perm[o:o + n_free_cap]
    work.page_tables, work.n_pages = tables, n_pages
    case = H.GpuCase(work, quant_mode=quant)
    lay = case.lay
    before = H.to_np(case.pool_mem).copy()
    host = before.copy()
    opool = H.orc.make_pool(host, int(lay.n_pages), 16, H.layout_strides(lay))
    d_free = torch.from_numpy(free.copy()).cuda()
    d_head = torch.zeros(1, dtype=torch.int32, device="cuda")
    d_status = torch.full((1,), 77, dtype=torch.int32, device="cuda")
    d_out = torch.empty((n_steps, B), dtype=torch.int32, device="cuda")
    d_tok, d_tab, d_len = case.tokens.clone(), case.tables.clone(), case.lens.clone()
    sun.sun_decode_run(case.pool, case.weights, n_steps, d_tok, d_tab, d_len, case.ids, d_free, d_head, d_status,
                       d_out, case.logits, case.ws, flags=sun.SUN_VALIDATE)
    torch.cuda.synchronize()
    got = d_out.cpu().numpy()
    ref = H.orc.decode_run(H.orc.make_cfg(shape), case.oracle_params(), opool, work.tokens, tables, lens,
                           work.model_ids, free, 0, n_steps, forced_tokens=got, keep_logits=True)
    tol = 1e-4 if dtype == "f32" else 2e-2
    near = []
    for s in range(n_steps):
        near += [(s, i) for i in H.check_next_tokens(got[s], ref["logits"][s], tol)]
    H.check_logits(case.logits.cpu().numpy(), ref["logits"][-1], dtype)
    assert np.array_equal(d_tab.cpu().numpy(), ref["page_tables"])
    assert np.array_equal(d_len.cpu().numpy(), ref["seq_lens"])
    assert int(d_head.cpu()[0]) == ref["free_head"] and int(d_status.cpu()[0]) == ref["status"]
    assert np.array_equal(d_tok.cpu().numpy(), got[-1])
    # cache: everything written during the run, nothing else
    after = H.to_np(case.pool_mem)
    st = H.layout_strides(lay)
    mask = np.zeros(after.size, dtype=bool)
    cur = lens.copy()
    final_tabs = ref["page_tables"]
    for s in range(n_steps):
        mask |= H.appended_mask(shape, st, after.size, final_tabs, cur)
        # a frozen request keeps its length; recompute lengths the way the run does
        for i in range(B):
            nl = cur[i] + 1
            if nl // 16 < mp and final_tabs[i, nl // 16] >= 0 and nl <= ref["seq_lens"][i]:
                cur[i] = nl
    off, total = H.check_appended_kv(after, host, before, mask, dtype, quant=quant is not None)
    H.say(f"   run {dtype} quant={quant} steps={n_steps}: near-ties {near}; K/V off by one ulp: {off} of {total}; "
          f"pages taken {ref['free_head']}; status {ref['status']}")
    return ref, got


def test_run_fp32_tiny_crosses_pages_and_chunks(H):
    H.say("run: fp32 tiny, 24 steps")
    ref, got = _run_case(H, wl.TINY, "f32", [0, 15, 16, 31, 62, 250, 505, 40], 24)
    assert ref["status"] == 0 and ref["free_head"] > 8


@pytest.mark.parametrize("quant", [None, "asym"])
def test_run_bf16_small(H, quant):
    H.say(f"run: bf16 small128 quant={quant}, 20 steps")
    ref, got = _run_case(H, wl.SMALL128, "bf16", [3, 14, 100, 255, 300, 17, 47, 511, 9, 128], 20, quant=quant, seed=41)
    assert ref["status"] == 0


def test_run_freezes_requests_without_pages_or_table_room(H):
    H.say("run: free list too short, table too narrow")
    ref, got = _run_case(H, wl.TINY, "f32", [14, 14, 3, 30], 20, n_free_cap=1, max_pages=2, seed=42)
    assert ref["status"] == 3
    assert ref["seq_lens"].tolist() == [31, 15, 15, 31]


def test_run_of_one_step_equals_the_step(H):
    H.say("run: one step == sun_decode_step")
    work = wl.make_workload("cfg1", seed=43)
    case = H.GpuCase(work)
    before = case.pool_mem.clone()
    case.step()
    nxt_step, logits_step, pool_step = case.next.clone(), case.logits.clone(), case.pool_mem.clone()
    case.pool_mem.copy_(before)
    free = torch.zeros(0, dtype=torch.int32, device="cuda")
    head = torch.zeros(1, dtype=torch.int32, device="cuda")
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    out = torch.empty((1, work.batch), dtype=torch.int32, device="cuda")
    tok, tab, ln = case.tokens.clone(), case.tables.clone(), case.lens.clone()
    logits = torch.empty_like(case.logits)
    sun.sun_decode_run(case.pool, case.weights, 1, tok, tab, ln, case.ids, None, head, status, out, logits, case.ws)
    torch.cuda.synchronize()
    assert torch.equal(out[0], nxt_step) and torch.equal(logits, logits_step) and torch.equal(case.pool_mem, pool_step)
    assert torch.equal(tok, nxt_step)
