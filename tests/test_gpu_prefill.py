"""GPU parity of sun_prefill (the prefill module of Eq. 2) against the oracle's causal forward, through the
C ABI.  The oracle side is the definition: a forward over the whole prompt with no cache (pinned on the CPU
against a library implementation of the same architecture); the GPU side runs the prompt through the decode
step's kernels in blocks of rows.  The cache it leaves in the pool, the first-token logits, and the decode
steps that follow must all agree with the oracle.

Cache entries in fp32: as for one step, an entry may differ from the oracle's bf16 rounding by one bf16 ulp.
Unlike in one step over a given cache, the entries of the deeper layers here depend on entries the same
call wrote: where one of those is an ulp apart (relative 2^-8), an attention score moves by about
|q_j| ulp(k_j) / sqrt(d) ~ 1e-4 and the activations after it by up to ~1e-5, far above fp32 rounding.  So
an entry near zero, where a bf16 ulp is smaller than that, is held to 2e-5 absolute instead (a fifth of the
1e-4 bar on the fp32 logits, which are checked as well)."""
PREFILL_ABS_TOL = 2e-5
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


def _one_request_case(H, shape, dtype, T, seed, n_models=2, extra=1):
    """A pool with one request whose table covers T + extra positions, pages shuffled."""
    work = wl.make_workload("cfg1", shape=shape, dtype=dtype, batch=1, n_models=n_models, seed=seed)
    work.seq_lens = np.array([T + extra - 1], np.int32)
    rng = np.random.default_rng(seed + 1)
    work.page_tables, work.n_pages = wl.deal_page_tables(work.seq_lens, rng)
    return H.GpuCase(work), rng


def _written_mask(H, st, n_elems, n_layers, n_kv, d, table, first, n):
    """Elements of the pool that hold positions first .. first+n-1 of the request (the oracle's addressing)."""
    probe = np.zeros(n_elems, np.uint16)
    ones = np.ones((n_layers, n, n_kv, d), np.uint16)
    H.orc.kv_ingest(probe, st, ones, ones, first, table)
    return probe != 0


def _prefill(case, toks, first, model_id, weights=None, row=0, flags=sun.SUN_VALIDATE):
    d_tok = torch.from_numpy(np.ascontiguousarray(toks, np.int32)).cuda()
    table = case.tables[row].contiguous()
    ws = torch.empty(sun.sun_prefill_workspace_bytes(case.cfg, len(toks), table.numel()), dtype=torch.uint8, device="cuda")
    logits = torch.empty(case.work.shape.vocab, dtype=torch.float32, device="cuda")
    nxt = torch.full((1,), -1, dtype=torch.int32, device="cuda")
    sun.sun_prefill(case.pool, case.weights if weights is None else weights, d_tok, table, first, model_id, logits, nxt,
                    ws, flags=flags)
    torch.cuda.synchronize()
    return logits.cpu().numpy(), int(nxt.cpu()[0])


@pytest.mark.parametrize("shape,dtype,T,cuts", [
    (wl.TINY, "f32", 1, None), (wl.TINY, "f32", 37, None), (wl.TINY, "f32", 300, None), (wl.TINY, "f32", 70, [16, 17, 60]),
    (wl.SMALL128, "bf16", 300, None), (wl.SMALL128, "bf16", 90, [1, 64]), (wl.TINY_QWEN, "bf16", 40, None),
    (wl.SMALL_LLAMA31, "f32", 45, None)],
    ids=["f32-1", "f32-37", "f32-300-two-blocks", "f32-70-in-pieces", "bf16-300", "bf16-90-in-pieces", "bf16-head-norm",
         "f32-scaled-rotary"])
def test_prefill_equals_the_causal_forward(H, shape, dtype, T, cuts):
    H.say(f"prefill {shape.name} {dtype} T={T} cuts={cuts}")
    case, rng = _one_request_case(H, shape, dtype, T, seed=300 + T)
    toks = rng.integers(0, shape.vocab, size=T + 1).astype(np.int32)
    before = H.to_np(case.pool_mem).copy()
    st = H.layout_strides(case.lay)
    table = case.work.page_tables[0]
    # the oracle: forward over the prompt, cache entries rounded to the pool's bf16
    ocfg, params = H.orc.make_cfg(shape), case.oracle_params()
    logits, K, V = H.orc.full_forward(ocfg, params, toks, round_kv=True, want_kv=True)
    expect = before.copy()
    H.orc.kv_ingest(expect, st, H.orc.bf16_bits(K[:, :T]), H.orc.bf16_bits(V[:, :T]), 0, table)
    # the GPU: in one call, or in pieces that continue each other
    bounds = [0] + (cuts or []) + [T]
    for a, b in zip(bounds[:-1], bounds[1:]):
        got_logits, got_next = _prefill(case, toks[a:b], a, 1)
    H.check_logits(got_logits[None], logits[T - 1][None], dtype)
    H.check_next_tokens(np.array([got_next]), logits[T - 1][None], 1e-4 if dtype == "f32" else 2e-2)
    after = H.to_np(case.pool_mem).copy()
    mask = _written_mask(H, st, after.size, shape.n_layers, shape.n_kv_heads, shape.head_dim, table, 0, T)
    off, total = H.check_appended_kv(after, expect, before, mask, dtype, abs_tol=PREFILL_ABS_TOL, max_off_frac=0.6)
    assert sun.sun_kv_pool_model_tokens(case.pool, 1) == T and sun.sun_kv_pool_model_tokens(case.pool, 0) == 0
    # Eq. 1 == Eq. 2 + Eq. 3 on the GPU alone: a decode step on top of the prefilled cache
    case.tokens[0] = int(toks[T])
    case.lens[0] = T
    case.step(flags=sun.SUN_VALIDATE)
    H.check_logits(case.logits.cpu().numpy(), logits[T][None], dtype)
    H.say(f"   cache entries off by one ulp or more: {off} of {total}")


def test_shared_decode_over_caches_prefilled_on_the_gpu_by_different_models(H):
    """The method in miniature, all on the GPU (Section 3.2.1): three task-specific prefill modules (perturbed
    copies of the base weights, standing in for prefill-only tuning) fill the caches of five requests, then
    the one frozen base decode module generates for all of them in one batch, once in bf16 and once with its
    weights in 4 bits (Eq. 8; the prefill side stays in full precision).  The oracle does the same with its
    causal forward and its multi-step run."""
    shape, dtype = wl.TINY_Q, "bf16"
    lens = np.array([5, 16, 33, 70, 129], np.int32)
    ids = np.array([0, 1, 2, 1, 0], np.int32)
    n_steps = 6
    for quant in (None, "asym"):
        H.say(f"gpu prefill by 3 perturbed models -> shared decode, quant={quant}")
        rng = np.random.default_rng(310)
        work = wl.make_workload("cfg1", shape=shape, dtype=dtype, batch=len(lens), n_models=3, seed=311)
        work.seq_lens, work.model_ids = lens + n_steps, ids       # tables wide enough for the generated tokens
        work.page_tables, work.n_pages = wl.deal_page_tables(work.seq_lens, rng)
        case = H.GpuCase(work, quant_mode=quant)
        gen = torch.Generator(device="cuda").manual_seed(312)
        prefill_w, prefill_h, prefill_p = [], [], []
        for m in range(3):      # theta_p^(m) = theta + delta_m on every matrix; the decode module stays theta
            wm = {k: ([t + 0.02 * t.float().std() * torch.randn(t.shape, device="cuda", generator=gen).to(t.dtype)
                       if t.ndim == 2 else t for t in v] if isinstance(v, list)
                      else (v + 0.02 * v.float().std() * torch.randn(v.shape, device="cuda", generator=gen).to(v.dtype)
                            if isinstance(v, torch.Tensor) and v.ndim == 2 else v))
                  for k, v in case.w.items()}
            prefill_w.append(wm)
            prefill_h.append(sun.sun_weights_create(case.cfg, wm))
            prefill_p.append(H.orc.params_from_arrays(H.weights_to_np(wm)))
        torch.cuda.synchronize()
        before = H.to_np(case.pool_mem).copy()
        host = before.copy()
        st = H.layout_strides(case.lay)
        ocfg = H.orc.make_cfg(shape)
        first_gpu, first_orc, mask = [], [], np.zeros(before.size, bool)
        for i, L in enumerate(lens):
            prompt = rng.integers(0, shape.vocab, size=int(L)).astype(np.int32)
            lg, nx = _prefill(case, prompt, 0, int(ids[i]), weights=prefill_h[ids[i]], row=i)
            ologits, K, V = H.orc.full_forward(ocfg, prefill_p[ids[i]], prompt, round_kv=True, want_kv=True)
            H.orc.kv_ingest(host, st, H.orc.bf16_bits(K), H.orc.bf16_bits(V), 0, work.page_tables[i])
            H.check_logits(lg[None], ologits[-1][None], dtype)
            H.check_next_tokens(np.array([nx]), ologits[-1][None], 2e-2)
            first_gpu.append(nx)
            first_orc.append(int(np.argmax(ologits[-1])))
            mask |= _written_mask(H, st, before.size, shape.n_layers, shape.n_kv_heads, shape.head_dim,
                                  work.page_tables[i], 0, int(L))
        after_prefill = H.to_np(case.pool_mem).copy()
        H.check_appended_kv(after_prefill, host, before, mask, dtype, abs_tol=PREFILL_ABS_TOL, max_off_frac=0.6)
        assert [sun.sun_kv_pool_model_tokens(case.pool, m) for m in range(3)] == [5 + 129, 16 + 70, 33]
        # shared decode: the oracle continues from ITS OWN prefilled pool, fed with the GPU's tokens
        B = len(lens)
        d_tok = torch.tensor(first_gpu, dtype=torch.int32, device="cuda")
        d_tab, d_len = case.tables.clone(), torch.from_numpy(lens.copy()).cuda()
        d_free = torch.zeros(1, dtype=torch.int32, device="cuda")
        d_head = torch.zeros(1, dtype=torch.int32, device="cuda")
        d_status = torch.zeros(1, dtype=torch.int32, device="cuda")
        d_out = torch.empty((n_steps, B), dtype=torch.int32, device="cuda")
        sun.sun_decode_run(case.pool, case.weights, n_steps, d_tok, d_tab, d_len, case.ids, d_free[:0], d_head,
                           d_status, d_out, case.logits, case.ws, flags=sun.SUN_VALIDATE)
        torch.cuda.synchronize()
        got = d_out.cpu().numpy()
        opool = H.orc.make_pool(host, int(case.lay.n_pages), 16, st)
        ref = H.orc.decode_run(ocfg, case.oracle_params(), opool, np.array(first_gpu, np.int32), work.page_tables, lens,
                               ids, np.zeros(0, np.int32), 0, n_steps, forced_tokens=got, keep_logits=True,
                               **({"mode": 1} if quant else {}))
        near = []
        for s in range(n_steps):
            near += [(s, i) for i in H.check_next_tokens(got[s], ref["logits"][s], 2e-2)]
        H.check_logits(case.logits.cpu().numpy(), ref["logits"][-1], dtype)
        assert int(d_status.cpu()[0]) == 0 and ref["status"] == 0
        H.say(f"   first tokens gpu {first_gpu} oracle {first_orc}; near-ties in the run {near}")


def test_prefill_rejects_what_it_cannot_run(H):
    case, rng = _one_request_case(H, wl.TINY_Q, "bf16", 20, seed=320)
    toks = rng.integers(0, wl.TINY_Q.vocab, size=20).astype(np.int32)
    with pytest.raises(sun.SunError) as e:
        _prefill(case, toks, 0, 7)
    assert e.value.status == 7
    with pytest.raises(sun.SunError) as e:
        _prefill(case, toks, 400, 0)
    assert e.value.status == 6
    bad = toks.copy()
    bad[3] = wl.TINY_Q.vocab
    with pytest.raises(sun.SunError) as e:
        _prefill(case, bad, 0, 0)
    assert e.value.status == 9
    qcase = H.GpuCase(case.work, quant_mode="asym")
    with pytest.raises(sun.SunError) as e:
        _prefill(qcase, toks, 0, 0)
    assert e.value.status == 2
