"""The attention entry point that allocates nothing (sun_paged_attention_static) against the one that takes a
workspace (sun_paged_attention): same kernels over scratch inside the library, so the outputs must agree to the
attention bar (max-abs 2e-5 for the fp32 kernel, 2e-4 for the matrix-core kernel) and are in fact expected to
be bit-identical.  Two calls in a row on the same GPU, the second with a smaller input, so that whatever the
first left in the shared scratch is there when the second runs.  Collected last on purpose."""
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


def _case(H, shape, dtype, lens, seed):
    work = wl.make_workload("cfg1", shape=shape, dtype=dtype, batch=len(lens), seed=seed)
    rng = np.random.default_rng(seed)
    work.seq_lens = np.array(lens, np.int32) - 1
    work.page_tables, work.n_pages = wl.deal_page_tables(work.seq_lens, rng)
    case = H.GpuCase(work)
    B, QD = len(lens), shape.n_q_heads * shape.head_dim
    q = torch.randn((B, QD), device=H.DEV, generator=torch.Generator(device=H.DEV).manual_seed(seed)) * 2.0
    n = torch.tensor(lens, dtype=torch.int32, device=H.DEV)
    return case, q, n


@pytest.mark.parametrize("shape,dtype", [(wl.SMALL128, "bf16"), (wl.TINY, "f32")], ids=["bf16", "f32"])
def test_attention_without_allocation_matches_the_workspace_entry_point(H, shape, dtype):
    tol = 2e-5 if dtype == "f32" else 2e-4
    big = [1000, 513, 511, 257, 256, 255, 64, 33, 17, 16, 2, 1, 777, 300, 129, 4000]
    small = [40, 1, 290, 16, 5]
    assert sun.sun_paged_attention_static_limit() == 16 << 20
    for lens, seed in ((big, 401), (small, 402)):       # the second call is smaller and finds the first one's leftovers
        case, q, n = _case(H, shape, dtype, lens, seed)
        need = sun.sun_paged_attention_static_bytes(case.cfg, len(lens), case.work.max_pages)
        assert 0 < need <= sun.sun_paged_attention_static_limit()
        layer = shape.n_layers - 1
        for host in (np.array(lens, np.int32), None):
            want, got = torch.empty_like(q), torch.full_like(q, float("nan"))
            sun.sun_paged_attention(case.pool, layer, q, case.tables, n, want, case.ws, n_tokens_host=host)
            sun.sun_paged_attention_static(case.pool, layer, q, case.tables, n, got, n_tokens_host=host)
            torch.cuda.synchronize()
            diff = float((got - want).abs().max())
            H.say(f"no-alloc attention {shape.name} {dtype}, {len(lens)} requests, host lengths "
                  f"{'given' if host is not None else 'absent'}: scratch {need} B, max abs diff {diff:.3e}, "
                  f"bit-identical {torch.equal(got, want)}")
            assert torch.isfinite(got).all() and diff <= tol
            assert torch.equal(got, want)


def test_attention_without_allocation_rejects_what_does_not_fit(H):
    case, q, n = _case(H, wl.SMALL128, "bf16", [5, 9], 403)
    # a table wide enough that the scratch for its longest possible request passes the library's 16 MiB
    wide = 1 << 16
    assert sun.sun_paged_attention_static_bytes(case.cfg, 64, wide) > sun.sun_paged_attention_static_limit()
    tables = torch.full((64, wide), -1, dtype=torch.int32, device=H.DEV)
    tables[:, 0] = 0
    qq = torch.zeros((64, q.shape[1]), device=H.DEV)
    nn = torch.ones(64, dtype=torch.int32, device=H.DEV)
    out = torch.full_like(qq, 7.0)
    with pytest.raises(sun.SunError) as e:
        sun.sun_paged_attention_static(case.pool, 0, qq, tables, nn, out)
    assert e.value.status == 4 and "scratch" in str(e.value)
    torch.cuda.synchronize()
    assert (out == 7.0).all()          # nothing was enqueued
