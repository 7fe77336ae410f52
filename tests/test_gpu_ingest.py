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
