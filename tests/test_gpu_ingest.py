"""GPU parity of sun_kv_pool_ingest against the oracle's ingest: a byte-exact scatter, so the whole pool
must be identical bit for bit, through the C ABI."""
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


@pytest.mark.parametrize("shape", [wl.TINY_Q, wl.SMALL128], ids=["d64", "d128"])
def test_ingest_is_bit_exact_and_touches_nothing_else(H, shape):
    H.say(f"ingest {shape.name}")
    rng = np.random.default_rng(60)
    lens = [1, 15, 16, 17, 40, 300, 129]
    need = [(n + 15) // 16 for n in lens]
    n_pages = sum(need) + 9
    cfg = sun.make_cfg(shape, "bf16")
    mem = torch.empty(sun.sun_kv_pool_bytes(cfg, n_pages) // 2, dtype=torch.bfloat16, device="cuda")
    wl.fill_kv_pool(mem, 61)
    pool = sun.sun_kv_pool_create(cfg, mem, 16, 3)
    lay = pool.layout()
    host = H.to_np(mem).copy()
    before = host.copy()
    st = H.layout_strides(lay)
    perm = rng.permutation(n_pages).astype(np.int32)
    o, written = 0, 0
    expect_tokens = [0, 0, 0]
    for i, n in enumerate(lens):
        row = np.full(max(need) + 1, -1, np.int32)
        row[:need[i]] = perm[o:o + need[i]]
        o += need[i]
        k = torch.randn((shape.n_layers, n, shape.n_kv_heads, shape.head_dim), device="cuda").to(torch.bfloat16)
        v = torch.randn_like(k)
        d_row = torch.from_numpy(row).cuda()
        model = i % 3
        cuts = [0, n] if i % 2 == 0 or n < 3 else [0, n // 3, n]      # every other request arrives in two chunks
        for a, b in zip(cuts[:-1], cuts[1:]):
            sun.sun_kv_pool_ingest(pool, model, k[:, a:b].contiguous(), v[:, a:b].contiguous(), a, d_row,
                                   flags=sun.SUN_VALIDATE)
            H.orc.kv_ingest(host, st, H.to_np(k[:, a:b].contiguous()), H.to_np(v[:, a:b].contiguous()), a, row)
        expect_tokens[model] += n
        written += 2 * k.numel()
    torch.cuda.synchronize()
    got = H.to_np(mem)
    assert np.array_equal(got, host), f"{int((got != host).sum())} pool elements differ"
    assert int((got != before).sum()) <= written
    assert [sun.sun_kv_pool_model_tokens(pool, m) for m in range(3)] == expect_tokens
    # error paths
    row = torch.tensor([0, n_pages, -1], dtype=torch.int32, device="cuda")
    k = torch.zeros((shape.n_layers, 20, shape.n_kv_heads, shape.head_dim), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(sun.SunError) as e:
        sun.sun_kv_pool_ingest(pool, 0, k, k, 0, row, flags=sun.SUN_VALIDATE)
    assert e.value.status == 5
    with pytest.raises(sun.SunError) as e:
        sun.sun_kv_pool_ingest(pool, 0, k, k, 40, row)
    assert e.value.status == 6
    with pytest.raises(sun.SunError) as e:
        sun.sun_kv_pool_ingest(pool, 3, k, k, 0, row)
    assert e.value.status == 7
    # without validation a page id outside the pool skips that page and nothing else is written
    snap = mem.clone()
    sun.sun_kv_pool_ingest(pool, 0, k, k, 16, row)       # positions 16..35: page entry 1 (out of range) and 2 (-1)
    torch.cuda.synchronize()
    assert torch.equal(mem, snap)


def test_decode_step_consumes_an_ingested_prompt(H):
    """Prompt cache computed by the oracle's causal forward (standing in for a prefill module with the same
    parameters, Eq. 2), ingested on the GPU, then one GPU decode step: logits must equal the oracle's forward
    over prompt + token (the Eq. 1 == Eq. 2 + Eq. 3 identity, now across the two implementations)."""
    H.say("ingest + step == full forward")
    shape = wl.TINY
    work = wl.make_workload("cfg1", batch=1, n_models=1, seed=62)
    L = 37
    work.seq_lens = np.array([L], np.int32)
    rng = np.random.default_rng(63)
    work.page_tables, work.n_pages = wl.deal_page_tables(work.seq_lens, rng)
    case = H.GpuCase(work)
    params = case.oracle_params()
    ocfg = H.orc.make_cfg(shape)
    toks = rng.integers(0, shape.vocab, size=L + 1).astype(np.int32)
    logits, K, V = H.orc.full_forward(ocfg, params, toks, round_kv=True, want_kv=True)
    kb = torch.from_numpy(H.orc.bf16_bits(K[:, :L]).view(np.int16)).cuda().view(torch.bfloat16)
    vb = torch.from_numpy(H.orc.bf16_bits(V[:, :L]).view(np.int16)).cuda().view(torch.bfloat16)
    sun.sun_kv_pool_ingest(case.pool, 0, kb.contiguous(), vb.contiguous(), 0, case.tables[0].contiguous(),
                           flags=sun.SUN_VALIDATE)
    case.tokens[0] = int(toks[L])
    case.step()
    got = case.logits.cpu().numpy()[0]
    assert np.abs(got - logits[L]).max() <= 1e-4, f"max abs {np.abs(got - logits[L]).max():.3e}"
    assert int(case.next.cpu()[0]) == int(np.argmax(logits[L]))


def test_shared_decode_over_caches_from_different_prefill_models(H):
    """A miniature of the method (Section 3.2.1): three task-specific prefill models (perturbed copies of the
    base weights, standing in for prefill-only tuning) compute the prompt caches of five requests on the CPU
    (Eq. 2, the oracle's causal forward); the GPU ingests them into one pool and decodes all requests in one
    batch with the single frozen decode module (Eq. 3).  Logits, tokens and appended cache entries must match
    the oracle's decode step over the same pool."""
    H.say("prefill by 3 perturbed models -> ingest -> shared decode")
    shape = wl.TINY
    lens = np.array([5, 16, 33, 70, 129], np.int32)
    work = wl.make_workload("cfg1", batch=len(lens), n_models=3, seed=64)
    work.seq_lens = lens
    rng = np.random.default_rng(65)
    work.page_tables, work.n_pages = wl.deal_page_tables(lens, rng)
    work.model_ids = np.array([0, 1, 2, 1, 0], np.int32)
    case = H.GpuCase(work)
    base_w = H.weights_to_np(case.w)
    ocfg = H.orc.make_cfg(shape)
    prefill_params = []
    for m in range(3):          # theta_p^(m) = theta + delta_m on every matrix (the decode module stays theta)
        wm = {k: ([a + 0.01 * rng.standard_normal(a.shape).astype(np.float32) if a.ndim == 2 else a for a in v]
                  if isinstance(v, list) else (v + 0.01 * rng.standard_normal(v.shape).astype(np.float32) if v.ndim == 2 else v))
              for k, v in base_w.items()}
        prefill_params.append((wm, H.orc.params_from_arrays(wm)))
    for i, L in enumerate(lens):
        prompt = rng.integers(0, shape.vocab, size=int(L)).astype(np.int32)
        _, K, V = H.orc.full_forward(ocfg, prefill_params[work.model_ids[i]][1], prompt, round_kv=True, want_kv=True)
        kb = torch.from_numpy(H.orc.bf16_bits(K).view(np.int16)).cuda().view(torch.bfloat16).contiguous()
        vb = torch.from_numpy(H.orc.bf16_bits(V).view(np.int16)).cuda().view(torch.bfloat16).contiguous()
        sun.sun_kv_pool_ingest(case.pool, int(work.model_ids[i]), kb, vb, 0, case.tables[i].contiguous(),
                               flags=sun.SUN_VALIDATE)
    torch.cuda.synchronize()
    assert [sun.sun_kv_pool_model_tokens(case.pool, m) for m in range(3)] == [5 + 129, 16 + 70, 33]
    rows = list(range(len(lens)))
    before_host, _, tabs, used = case.extract_pool(rows)
    ref = H.run_oracle(case, rows)                     # the oracle decodes from the pool the GPU ingested
    case.step(flags=sun.SUN_VALIDATE)
    got = case.logits.cpu().numpy()
    assert np.abs(got - ref["logits"]).max() <= 1e-4
    assert np.array_equal(case.next.cpu().numpy(), ref["next"])
    st = H.layout_strides(case.lay)
    st["k_layer"] = st["v_layer"] = len(used) * int(case.lay.k_page)
    mask = H.appended_mask(shape, st, before_host.size, tabs, lens)
    H.check_appended_kv(case.pool_pages_now(used), ref["pool_after"], before_host, mask, "f32")
    # and the caches really differ by source model: the same prompt prefilled by two models gives different K
    p = rng.integers(0, shape.vocab, size=8).astype(np.int32)
    _, K0, _ = H.orc.full_forward(ocfg, prefill_params[0][1], p, round_kv=True, want_kv=True)
    _, K1, _ = H.orc.full_forward(ocfg, prefill_params[1][1], p, round_kv=True, want_kv=True)
    assert np.abs(K0 - K1).max() > 1e-3


def test_read_probe_reads_every_block_once(H):
    """The measurement kernel behind bench.py --hbm-read-probe: whatever the order of the blocks, every 16-byte
    unit is read exactly once.  Each thread folds fixed components of its units into one word, so the fold of
    all threads' words equals the fold of those components over the whole buffer, in address order and in any
    shuffled order."""
    H.say("hbm read probe")
    n_blocks, block = 777, 4096
    g = torch.Generator(device=H.DEV).manual_seed(5)
    src = torch.randint(-2 ** 31, 2 ** 31 - 1, (n_blocks * block // 4,), dtype=torch.int32, device=H.DEV, generator=g)
    a = src.cpu().numpy().view(np.uint32).reshape(n_blocks, block // 16, 4)
    comp = {0: (0, 3), 1: (1, 2), 2: (0, 2), 3: (1, 3)}      # which dwords of a unit are folded, by the unit's quarter of the block
    want = np.uint32(0)
    for quarter, (c0, c1) in comp.items():
        part = a[:, quarter * 64:(quarter + 1) * 64]
        want ^= np.bitwise_xor.reduce(part[..., c0].ravel()) ^ np.bitwise_xor.reduce(part[..., c1].ravel())
    perm = torch.randperm(n_blocks, device=H.DEV, generator=g).to(torch.int32)
    for order, wgs, streaming in ((None, 64, False), (perm, 64, False), (perm, 300, True), (None, 64, True)):
        sink = torch.full((wgs * 256,), 12345, dtype=torch.int32, device=H.DEV)
        sun.sun_hbm_read_probe(src, block, order, wgs, sink, streaming_loads=streaming)
        torch.cuda.synchronize()
        got = np.bitwise_xor.reduce(sink.cpu().numpy().view(np.uint32))
        assert got == want, f"fold {got:#x} != {want:#x} (order {'shuffled' if order is not None else 'address'}, {wgs} workgroups)"
