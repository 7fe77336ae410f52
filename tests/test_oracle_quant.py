"""Pins of the oracle's 4-bit group quantiser and of the QSUN decode step (CPU only).

QSUN replaces the decoder's projection weights by W_hat = (Q - Z) * S with 4-bit
codes in groups of 128 along the input dimension; lm_head stays unquantised
(Section 3.3, Eq. 8; Appendix A.1 "Quantization Configurations").
"""
import numpy as np
import pytest

from helpers import MiniShape, random_weights


def _grid_matrix(rng, rows, cols, group, full_range=True):
    ng = cols // group
    Q0 = rng.integers(0, 16, size=(rows, cols)).astype(np.int32)
    if full_range:  # every group spans codes 0..15 so that min/max recover the scale
        for r in range(rows):
            for g in range(ng):
                Q0[r, g * group] = 0
                Q0[r, g * group + 1] = 15
    Z0 = rng.integers(0, 16, size=(rows, ng)).astype(np.float32)
    S0 = rng.uniform(0.001, 0.05, size=(rows, ng)).astype(np.float16)
    W = (Q0.astype(np.float32) - np.repeat(Z0, group, axis=1)) * np.repeat(S0.astype(np.float32), group, axis=1)
    return Q0, Z0, S0, W.astype(np.float32)


def _unpack(q):
    out = np.empty((q.shape[0], q.shape[1] * 2), dtype=np.int32)
    out[:, 0::2] = q & 15
    out[:, 1::2] = q >> 4
    return out


def test_grid_matrix_roundtrips_exactly(orc):
    """A matrix already on a 4-bit grid is reproduced code for code and bit for bit."""
    rng = np.random.default_rng(21)
    Q0, Z0, S0, W = _grid_matrix(rng, 6, 512, 128)
    q, s, z = orc.quantize_w4(W, 128, "asym")
    assert np.array_equal(_unpack(q), Q0)
    assert np.array_equal(s.view(np.float16), S0)
    assert np.array_equal(z.view(np.float16).astype(np.float32), Z0)
    assert np.array_equal(orc.dequantize_w4(q, s, z, 512, 128), W)


def test_nibble_packing_is_the_identity_for_all_codes(orc):
    """Low nibble = even column, high nibble = odd column, all 16 codes at both places."""
    W = np.zeros((2, 128), dtype=np.float32)
    W[0, :16] = np.arange(16)            # codes 0..15 at columns 0..15 (even and odd)
    W[0, 16:32] = np.arange(16)[::-1]
    W[1, :] = np.tile(np.arange(16), 8)[::-1]
    q, s, z = orc.quantize_w4(W, 128, "asym")
    assert np.all(s.view(np.float16) == 1.0) and np.all(z.view(np.float16) == 0.0)
    codes = _unpack(q)
    assert np.array_equal(codes, W.astype(np.int32))
    assert q[0, 0] == (0 | (1 << 4)) and q[0, 7] == (14 | (15 << 4))


@pytest.mark.parametrize("mode", ["asym", "sym"])
def test_rounding_error_is_at_most_half_a_step(orc, mode):
    rng = np.random.default_rng(22)
    W = rng.normal(0, 0.02, size=(16, 1024)).astype(np.float32)
    q, s, z = orc.quantize_w4(W, 128, mode)
    What = orc.dequantize_w4(q, s, z, 1024, 128)
    S = np.repeat(s.view(np.float16).astype(np.float64), 128, axis=1)
    Z = np.repeat(z.view(np.float16).astype(np.float64), 128, axis=1)
    codes = _unpack(q)
    ideal = W.astype(np.float64) / S + Z
    inside = (ideal >= 0) & (ideal <= 15)
    err = np.abs(W.astype(np.float64) - What.astype(np.float64))
    assert np.all(err[inside] <= S[inside] * (0.5 + 1e-6))
    assert inside.mean() > 0.9
    assert np.all((codes >= 0) & (codes <= 15))
    if mode == "sym":
        assert np.all(Z == 8) and codes.min() >= 1
        amax = np.abs(W).reshape(16, 8, 128).max(axis=2)
        assert np.array_equal(s.view(np.float16), (amax / np.float32(7.0)).astype(np.float16))
    else:
        mn, mx = W.reshape(16, 8, 128).min(axis=2), W.reshape(16, 8, 128).max(axis=2)
        assert np.array_equal(s.view(np.float16), ((mx - mn) / np.float32(15.0)).astype(np.float16))
        assert codes.min() == 0 and codes.max() == 15


def test_round_half_to_even_and_clamping(orc):
    W = np.zeros((1, 128), dtype=np.float32)
    W[0, 0], W[0, 1] = 0.0, 15.0                 # S = 1, Z = 0
    W[0, 2:8] = [0.5, 1.5, 2.5, 3.5, 6.5, 7.5]
    q, s, z = orc.quantize_w4(W, 128, "asym")
    assert list(_unpack(q)[0, 2:8]) == [0, 2, 2, 4, 6, 8]
    Wz = np.zeros((1, 128), dtype=np.float32)    # all-zero group: scale falls back to 1
    q, s, z = orc.quantize_w4(Wz, 128, "asym")
    assert s.view(np.float16)[0, 0] == 1.0 and np.all(_unpack(q) == 0)
    q, s, z = orc.quantize_w4(Wz, 128, "sym")
    assert s.view(np.float16)[0, 0] == 1.0 and np.all(_unpack(q) == 8)


def test_short_last_group(orc):
    rng = np.random.default_rng(23)
    W = rng.normal(0, 0.02, size=(3, 176)).astype(np.float32)   # 128 + 48
    q, s, z = orc.quantize_w4(W, 128, "asym")
    assert s.shape == (3, 2)
    What = orc.dequantize_w4(q, s, z, 176, 128)
    q2, s2, z2 = orc.quantize_w4(np.ascontiguousarray(W[:, 128:]), 128, "asym")
    assert np.array_equal(What[:, 128:], orc.dequantize_w4(q2, s2, z2, 48, 128))


def test_quantised_linear_is_an_integer_matmul_when_scale_is_one(orc):
    """With S = 1, Z = 0 and integer activations the QSUN projection is an exact integer matmul."""
    rng = np.random.default_rng(24)
    codes = rng.integers(0, 16, size=(9, 256))
    codes[:, 0], codes[:, 1], codes[:, 128], codes[:, 129] = 0, 15, 0, 15
    q, s, z = orc.quantize_w4(codes.astype(np.float32), 128, "asym")
    X = rng.integers(-20, 21, size=(4, 256)).astype(np.float64)
    Y = orc.linear(orc.w4_mat(q, s, z, 256, 128), X)
    assert np.array_equal(Y, (X.astype(np.int64) @ codes.T.astype(np.int64)).astype(np.float64))


def test_qsun_step_equals_dense_step_on_dequantised_weights(orc):
    """D_q(theta_d) is D with W replaced by W_hat; embedding, gains and lm_head untouched."""
    shape = MiniShape(hidden=128, n_q_heads=4, n_kv_heads=2, head_dim=32, ffn=256, vocab=96)
    rng = np.random.default_rng(25)
    w = random_weights(shape, rng, dtype=np.float32, std=0.05)
    quant, wd = {}, dict(w)
    for k in orc.QUANT_KEYS:
        quant[k] = [orc.quantize_w4(m, 128, "asym") for m in w[k]]
        wd[k] = [orc.dequantize_w4(*quant[k][l], w[k][l].shape[1], 128) for l in range(shape.n_layers)]
    cfg = orc.make_cfg(shape)
    pq, pd = orc.params_from_arrays(w, quant), orc.params_from_arrays(wd)
    n_pages = 6
    n = orc.pool_elems(shape, n_pages)
    import torch
    base = torch.randn(n, generator=torch.Generator().manual_seed(1)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16).copy()
    tables = np.array([[4, 1, 3], [0, 5, -1]], np.int32)
    lens, toks, ids = np.array([40, 17], np.int32), np.array([3, 77], np.int32), np.array([0, 1], np.int32)
    b1 = base.copy()
    r_q = orc.decode_step(cfg, pq, orc.make_pool(b1, n_pages, 16, orc.default_strides(shape, n_pages)), toks, tables, lens, ids)
    b2 = base.copy()
    r_d = orc.decode_step(cfg, pd, orc.make_pool(b2, n_pages, 16, orc.default_strides(shape, n_pages)), toks, tables, lens, ids)
    assert np.array_equal(r_q["logits"], r_d["logits"]) and np.array_equal(b1, b2)
    # and it differs from the unquantised step (the quantiser did something)
    b3 = base.copy()
    r_f = orc.decode_step(cfg, orc.params_from_arrays(w), orc.make_pool(b3, n_pages, 16, orc.default_strides(shape, n_pages)), toks, tables, lens, ids)
    gap = np.abs(r_f["logits"] - r_q["logits"]).max()
    assert 0 < gap < 1.0


def test_zero_point_is_a_plain_integer_code(orc):
    """Z holds an integer in [0,15]; a group whose minimum is 0 stores +0 (bit pattern 0), not -0."""
    W = np.zeros((2, 128), dtype=np.float32)
    W[1, :] = np.linspace(0, 1, 128)
    q, s, z = orc.quantize_w4(W, 128, "asym")
    assert z[0, 0] == 0 and z[1, 0] == 0
