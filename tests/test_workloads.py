"""Closed-form checks of the synthetic workload generator (CPU only)."""
import numpy as np

from paper_2603_02599_amd import workloads as wl


def test_zipf_split_matches_the_formula():
    # Appendix A.2: P(i) = i^-a / sum_j j^-a; a = 0 is uniform
    assert np.allclose(wl.zipf_probs(4, 0.0), 0.25)
    p = wl.zipf_probs(4, 1.5)
    den = 1 + 2 ** -1.5 + 3 ** -1.5 + 4 ** -1.5
    assert np.allclose(p, [1 / den, 2 ** -1.5 / den, 3 ** -1.5 / den, 4 ** -1.5 / den])
    assert np.allclose(np.round(p, 3), [0.598, 0.212, 0.115, 0.075])
    assert abs(wl.zipf_probs(16, 1.2).sum() - 1) < 1e-12


def test_page_tables_are_a_partial_permutation():
    rng = np.random.default_rng(0)
    L = wl.draw_lengths(40, "uniform", rng, 16, 128)
    tables, n_pages = wl.deal_page_tables(L, rng)
    need = wl.pages_needed(L)
    used = tables[tables >= 0]
    assert len(used) == need.sum() == len(np.unique(used))
    assert used.max() < n_pages and n_pages >= need.sum()
    for i in range(40):
        assert np.all(tables[i, :need[i]] >= 0) and np.all(tables[i, need[i]:] == -1)
    # boundary: L % 16 == 0 needs a fresh page for the slot written this step
    assert list(wl.pages_needed(np.array([0, 15, 16, 31, 32]))) == [1, 1, 2, 2, 3]


def test_capped_pool_keeps_tail_pages_unique():
    rng = np.random.default_rng(1)
    L = wl.draw_lengths(32, "uniform", rng, 200, 400)
    tables, n_pages = wl.deal_page_tables(L, rng, n_pages=100)
    need = wl.pages_needed(L)
    tails = [tables[i, need[i] - 1] for i in range(32)]
    assert len(set(tails)) == 32 and n_pages == 100
    hist = np.concatenate([tables[i, :need[i] - 1] for i in range(32)])
    assert not set(hist.tolist()) & set(tails)


def test_configs_have_the_stated_structure():
    w1 = wl.make_workload("cfg1")
    assert w1.batch == 8 and set(w1.model_ids.tolist()) == {0, 1, 2}
    assert w1.seq_lens.min() >= 16 and w1.seq_lens.max() <= 128 and w1.shape.ffn == 688
    w2 = wl.make_workload("cfg2")
    assert w2.batch == 64 and np.bincount(w2.model_ids).tolist() == [16] * 4
    assert w2.seq_lens.min() >= 512 and w2.seq_lens.max() <= 4096
    w3 = wl.make_workload("cfg3")
    assert w3.batch == 256 and w3.seq_lens.min() >= 64 and w3.seq_lens.max() <= 16384
    assert w3.seq_lens.max() >= 8192 and np.median(w3.seq_lens) < 2048
    assert np.bincount(w3.model_ids, minlength=8)[0] > np.bincount(w3.model_ids, minlength=8)[-1]
    again = wl.make_workload("cfg3")
    assert np.array_equal(again.page_tables, w3.page_tables) and np.array_equal(again.tokens, w3.tokens)


def test_weights_are_seeded_and_shaped():
    w = wl.make_weights(wl.TINY, "f32", "cpu", 7)
    w2 = wl.make_weights(wl.TINY, "f32", "cpu", 7)
    assert all((a == b).all() for a, b in zip(w["wg"], w2["wg"]))
    assert w["wg"][0].shape == (688, 256) and w["wd"][1].shape == (256, 688) and w["wlm"].shape == (1024, 256)
    assert abs(float(w["wlm"].std()) - 0.02) < 2e-3
    # gains are spread around 1 (a dropped or swapped gain must show), each vector its own draw
    for g in w["g1"] + w["g2"] + [w["gf"]]:
        assert abs(float(g.mean()) - 1.0) < 0.03 and 0.07 < float(g.std()) < 0.13
    assert not (w["g1"][0] == w["g2"][0]).all() and not (w["g1"][0] == w["g1"][1]).all()


def test_cfg5_forms_fit_one_gpu():
    a, b = wl.make_workload("cfg5a"), wl.make_workload("cfg5b")
    full = wl.make_workload("cfg5", n_pages=10 ** 6)
    kv_tok = a.shape.kv_bytes_per_token()
    assert a.batch == 128 and a.aliased and a.n_pages == wl.CFG5A_PAGES and np.array_equal(a.seq_lens, full.seq_lens)
    assert a.n_pages * 2 * a.shape.kv_dim * 16 > 2 ** 31              # elements of one layer of the pool
    need = wl.pages_needed(a.seq_lens)
    tails = [int(a.page_tables[i, need[i] - 1]) for i in range(a.batch)]
    hist = np.concatenate([a.page_tables[i, :need[i] - 1] for i in range(a.batch)])
    assert len(set(tails)) == a.batch and not np.isin(tails, hist).any() and hist.min() >= 0 and hist.max() < a.n_pages
    assert b.batch == 52 and not b.aliased and np.array_equal(b.seq_lens, full.seq_lens[:52])
    assert b.n_pages * 16 * kv_tok <= wl.CFG5B_POOL_BYTES < (b.n_pages + 1) * 16 * kv_tok
    assert int(wl.pages_needed(full.seq_lens[:53]).sum()) > b.n_pages >= int(need[:52].sum())
