"""GPU parity at the benchmark sizes, in the launch configuration bench.py times: the full
8B-shaped step (batch 64 and 256, bf16 and QSUN) is run on the GPU and a sample of its
requests is recomputed by the CPU oracle from exactly the bytes the GPU consumed."""
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


def _sample_rows(work, k):
    order = np.argsort(work.seq_lens, kind="stable")
    picks = {int(order[0]), int(order[-1])}
    rng = np.random.default_rng(work.seed)
    while len(picks) < k:
        picks.add(int(rng.integers(0, work.batch)))
    return sorted(picks)


def _sampled_parity(H, work, shared, k):
    case = H.GpuCase(work, shared=shared)
    rows = _sample_rows(work, k)
    H.say(f"{work.name} B={work.batch} quant={shared.quant is not None}: oracle on rows {rows} "
          f"(lengths {[int(work.seq_lens[r]) for r in rows]})")
    before_host, _, tabs, used = case.extract_pool(rows)
    ref = H.run_oracle(case, rows)
    case.step(flags=sun.SUN_VALIDATE)
    got_logits = case.logits.cpu().numpy()[rows]
    got_next = case.next.cpu().numpy()[rows]
    rep = H.logits_report(got_logits, ref["logits"])
    H.say(f"   logits {rep}")
    H.check_logits(got_logits, ref["logits"], "bf16")
    near = H.check_next_tokens(got_next, ref["logits"], 2e-2)
    st = H.layout_strides(case.lay)
    st["k_layer"] = st["v_layer"] = len(used) * int(case.lay.k_page)
    mask = H.appended_mask(work.shape, st, before_host.size, tabs, work.seq_lens[rows])
    off, total = H.check_appended_kv(case.pool_pages_now(used), ref["pool_after"], before_host, mask, "bf16")
    H.say(f"   near-tie rows {near}; appended K/V off by >=1 bf16 ulp: {off} of {total}")
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


def test_cfg5_14b_shape_sampled(H):
    """14B shape (48 layers, 40 q / 8 kv heads, vocab 152064): the first 16 requests of the cfg5
    draw (lengths up to 32768, ~50 GB of KV) in a pool without aliasing, dense and 4-bit; the
    oracle recomputes 3 of them including the longest."""
    work = wl.make_workload("cfg5", batch=16)
    for quant in (None, "asym"):
        H.say(f"building 14B-shaped weights quant={quant}")
        sw = H.SharedWeights(wl.QWEN_14B, "bf16", wl.SEED_BASE + 105, quant_mode=quant)
        if quant:
            for k in sun.QUANT_KEYS:
                sw.w[k] = None
            torch.cuda.empty_cache()
        case, rep = _sampled_parity(H, work, sw, 3)
        del case, sw
        torch.cuda.empty_cache()
