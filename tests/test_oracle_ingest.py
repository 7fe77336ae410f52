"""Pins of the oracle's KV ingest (CPU only): a byte-exact scatter of a contiguous cache into pages.
(The prefill + decode == full forward identities of test_oracle_pins also run through it.)"""
import numpy as np
import torch
import torch.nn.functional as F

from helpers import MiniShape
from test_oracle_pins import PT


def _transposed_v_strides(shape, n_pages):
    """A layout unlike the plain one: layer-major, K [head][token][dim], V [head][dim][token] in a
    separate region (the layout the GPU pool reports)."""
    d, hkv = shape.head_dim, shape.n_kv_heads
    blk = PT * d
    page = hkv * blk
    k_region = shape.n_layers * n_pages * page
    return dict(k_off=0, k_layer=n_pages * page, k_page=page, k_head=blk, k_token=d, k_dim=1,
                v_off=k_region, v_layer=n_pages * page, v_page=page, v_head=blk, v_token=1, v_dim=PT)


def test_ingested_cache_reads_back_as_library_attention(orc):
    """Cache of 41 tokens scattered over shuffled pages in the transposed-V layout; the oracle's paged
    attention over it must equal torch's scaled_dot_product_attention on the contiguous source."""
    shape = MiniShape(n_layers=2, n_q_heads=4, n_kv_heads=2, head_dim=8)
    rng = np.random.default_rng(3)
    n_pages, n = 7, 41
    st = _transposed_v_strides(shape, n_pages)
    total = 2 * shape.n_layers * n_pages * shape.n_kv_heads * PT * shape.head_dim
    base = orc.bf16_bits(rng.normal(size=total))
    before = base.copy()
    pool = orc.make_pool(base, n_pages, PT, st)
    K = orc.bf16_bits(rng.normal(size=(shape.n_layers, n, shape.n_kv_heads, shape.head_dim)))
    V = orc.bf16_bits(rng.normal(size=K.shape))
    table = rng.permutation(n_pages)[:3].astype(np.int32)
    orc.kv_ingest(base, st, K, V, 0, table, PT)
    assert int((base != before).sum()) <= 2 * K.size          # nothing but the cache entries can have changed
    cfg = orc.make_cfg(shape)
    G = shape.n_q_heads // shape.n_kv_heads
    for layer in range(shape.n_layers):
        q = rng.normal(size=shape.n_q_heads * shape.head_dim)
        a, _ = orc.attention_paged(cfg, pool, layer, table, q, n)
        Kf = torch.from_numpy(orc.bf16_values(K[layer])).permute(1, 0, 2).repeat_interleave(G, dim=0)  # [Hq, n, d]
        Vf = torch.from_numpy(orc.bf16_values(V[layer])).permute(1, 0, 2).repeat_interleave(G, dim=0)
        want = F.scaled_dot_product_attention(torch.from_numpy(q.reshape(shape.n_q_heads, 1, -1))[None], Kf[None],
                                              Vf[None])[0, :, 0].numpy().ravel()
        assert np.abs(a - want).max() < 1e-12


def test_chunked_ingest_equals_one_ingest_and_touches_only_its_slots(orc):
    shape = MiniShape(n_layers=1, n_q_heads=2, n_kv_heads=2, head_dim=8)
    rng = np.random.default_rng(4)
    n_pages, n = 6, 37
    st = _transposed_v_strides(shape, n_pages)
    total = 2 * shape.n_layers * n_pages * shape.n_kv_heads * PT * shape.head_dim
    K = orc.bf16_bits(rng.normal(size=(1, n, 2, 8)))
    V = orc.bf16_bits(rng.normal(size=K.shape))
    table = np.array([4, 0, 5, -1], np.int32)
    one = np.zeros(total, np.uint16)
    orc.kv_ingest(one, st, K, V, 0, table, PT)
    two = np.zeros(total, np.uint16)
    orc.kv_ingest(two, st, K[:, :19], V[:, :19], 0, table, PT)
    orc.kv_ingest(two, st, K[:, 19:], V[:, 19:], 19, table, PT)
    assert np.array_equal(one, two)
    # exactly n * Hkv * d elements of K and of V were written (source values are nonzero with probability 1)
    assert int((one != 0).sum()) == 2 * K.size - int((K == 0).sum()) - int((V == 0).sum())
    # pages 1, 2, 3 are not in the table and stay zero
    page = shape.n_kv_heads * PT * shape.head_dim
    for p in (1, 2, 3):
        assert not one[p * page:(p + 1) * page].any() and not one[st["v_off"] + p * page: st["v_off"] + (p + 1) * page].any()
