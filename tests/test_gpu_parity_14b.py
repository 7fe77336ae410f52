"""GPU parity on the 14B-shaped configuration at the sizes bench.py times (Section 4.1 backbones; traffic of
Appendix A.2: 128 requests Zipf(1.2) over 16 source models, contexts U[2048,32768], a pool of about 200 GB):

cfg5b  the first 52 requests of the draw in a 200 GB pool without aliasing;
cfg5a  all 128 requests over a 206 GB pool of 65 600 pages (more than 2^31 elements per layer, so every
       page address needs 64 bits) whose history pages are shared read-only between requests; the
       projections run their 128-row tiles and the SwiGLU epilogue at the 14B widths.

Each with dense and with 4-bit weights.  The oracle recomputes sampled requests, the longest among them, from
exactly the bytes the GPU consumed: logits, next tokens and the appended cache entries."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from paper_2603_02599_amd import binding as sun  # noqa: E402
from paper_2603_02599_amd import workloads as wl  # noqa: E402
from test_gpu_parity_full import _sampled_parity  # noqa: E402


@pytest.fixture(scope="module")
def H():
    import gpu_harness
    assert torch.cuda.is_available(), "these tests need the MI355X"
    sun.lib()
    return gpu_harness


@pytest.fixture(scope="module", params=[None, "asym"], ids=["bf16", "qsun"])
def weights14b(H, request):
    quant = request.param
    H.say(f"building 14B-shaped weights quant={quant}")
    sw = H.SharedWeights(wl.QWEN_14B, "bf16", wl.SEED_BASE + 105, quant_mode=quant)
    sw.oracle_params()                 # the oracle's host mirror first ...
    for k in sun.QUANT_KEYS:           # ... then the projection sources can leave the device: the library has packed them
        sw.w[k] = None
    torch.cuda.empty_cache()
    yield sw
    del sw
    torch.cuda.empty_cache()


def test_cfg5b_52_requests_200gb_pool_sampled(H, weights14b):
    work = wl.make_workload("cfg5b")
    assert work.batch == 52 and not work.aliased and abs(work.n_pages * 16 * work.shape.kv_bytes_per_token() - 200e9) < 4e6
    case, rep = _sampled_parity(H, work, weights14b, 4)
    del case
    torch.cuda.empty_cache()


def test_cfg5a_128_requests_aliased_history_sampled(H, weights14b):
    work = wl.make_workload("cfg5a")
    lay_elems_per_layer = work.n_pages * 2 * work.shape.kv_dim * 16
    assert work.batch == 128 and work.aliased and lay_elems_per_layer > 2 ** 31
    # Relabel two pages so that the pool's last page (past element 2^31 of every layer) is the page the
    # longest request writes this step, and the page before it is part of that request's history.
    r = int(np.argmax(work.seq_lens))
    need = int(wl.pages_needed(work.seq_lens[r:r + 1])[0])
    tabs = work.page_tables
    for col, target in ((need - 1, work.n_pages - 1), (0, work.n_pages - 2)):
        old = int(tabs[r, col])
        a, b = tabs == old, tabs == target
        tabs[a], tabs[b] = target, old
    assert tabs[r, need - 1] == work.n_pages - 1 and (work.n_pages - 2) * 2 * work.shape.kv_dim * 16 > 2 ** 31
    tails = np.array([tabs[i, int(wl.pages_needed(work.seq_lens[i:i + 1])[0]) - 1] for i in range(work.batch)])
    assert len(set(tails.tolist())) == work.batch
    case, rep = _sampled_parity(H, work, weights14b, 4, must=[r])
    del case
    torch.cuda.empty_cache()
