"""Pins of the oracle's causal forward against an independent implementation of the backbone family the
paper uses (Section 4.1: LLaMA-3.1 / Qwen3 class decoders): the Hugging Face transformers model classes,
built from a tiny random configuration on the CPU in float64 and loaded with the same weights.  This fixes the
reading of the block (pre-norm, RMSNorm with eps inside the root, GQA head mapping, half-split rotary
pairing, SwiGLU, untied head) by a library the oracle shares no code with.  transformers evaluates the rotary
angle in float32, the oracle in float64 (rounding cos/sin to float32): agreement is to ~1e-5 relative, not to
the last bit."""
import numpy as np
import pytest
import torch

from helpers import MiniShape, random_weights

transformers = pytest.importorskip("transformers")


def _load(model, shape, w):
    sd = {"model.embed_tokens.weight": w["embed"], "model.norm.weight": w["gf"], "lm_head.weight": w["wlm"]}
    names = {"g1": "input_layernorm", "g2": "post_attention_layernorm", "wq": "self_attn.q_proj", "wk": "self_attn.k_proj",
             "wv": "self_attn.v_proj", "wo": "self_attn.o_proj", "wg": "mlp.gate_proj", "wu": "mlp.up_proj", "wd": "mlp.down_proj"}
    if "qn" in w:
        names.update({"qn": "self_attn.q_norm", "kn": "self_attn.k_norm"})
    for l in range(shape.n_layers):
        for k, n in names.items():
            sd[f"model.layers.{l}.{n}.weight"] = w[k][l]
        if "bq" in w:
            for k, n in (("bq", "q_proj"), ("bk", "k_proj"), ("bv", "v_proj")):
                sd[f"model.layers.{l}.self_attn.{n}.bias"] = w[k][l]
    missing, unexpected = model.load_state_dict({k: torch.from_numpy(np.asarray(v, dtype=np.float64)) for k, v in sd.items()},
                                                strict=False)
    assert not unexpected and all("rotary" in m or "inv_freq" in m for m in missing), (missing, unexpected)


@pytest.mark.parametrize("shape", [MiniShape(), MiniShape(n_layers=3, n_q_heads=6, n_kv_heads=2, head_dim=16, hidden=96, ffn=80)])
def test_full_forward_equals_transformers_llama(orc, shape):
    rng = np.random.default_rng(31)
    w = random_weights(shape, rng)
    cfg = transformers.LlamaConfig(
        vocab_size=shape.vocab, hidden_size=shape.hidden, intermediate_size=shape.ffn, num_hidden_layers=shape.n_layers,
        num_attention_heads=shape.n_q_heads, num_key_value_heads=shape.n_kv_heads, head_dim=shape.head_dim,
        rms_norm_eps=shape.rms_eps, rope_theta=shape.rope_base, max_position_embeddings=512, attention_bias=False,
        mlp_bias=False, tie_word_embeddings=False, attn_implementation="eager")
    model = transformers.LlamaForCausalLM(cfg).double().eval()
    _load(model, shape, w)
    toks = rng.integers(0, shape.vocab, size=37)
    with torch.no_grad():
        want = model(torch.from_numpy(toks)[None]).logits[0].numpy()
    got = orc.full_forward(orc.make_cfg(shape), orc.params_from_arrays(w), toks)
    assert want.std() > 0.1
    # float32 rotary angles on the library side: ~1e-5 relative; any structural mistake is of order 1
    assert np.abs(got - want).max() < 3e-4 * max(1.0, want.std()), np.abs(got - want).max()


def test_head_norm_variant_equals_transformers_qwen3(orc):
    """Backbone option of the Qwen3 class: RMSNorm over head_dim on every q and k head before the rotation."""
    shape = MiniShape(n_layers=2, n_q_heads=4, n_kv_heads=2, head_dim=16, hidden=48, ffn=64, qk_norm=True)
    rng = np.random.default_rng(32)
    w = random_weights(shape, rng)
    cfg = transformers.Qwen3Config(
        vocab_size=shape.vocab, hidden_size=shape.hidden, intermediate_size=shape.ffn, num_hidden_layers=shape.n_layers,
        num_attention_heads=shape.n_q_heads, num_key_value_heads=shape.n_kv_heads, head_dim=shape.head_dim,
        rms_norm_eps=shape.rms_eps, rope_theta=shape.rope_base, max_position_embeddings=512, attention_bias=False,
        tie_word_embeddings=False, use_sliding_window=False, attn_implementation="eager")
    model = transformers.Qwen3ForCausalLM(cfg).double().eval()
    _load(model, shape, w)
    toks = rng.integers(0, shape.vocab, size=29)
    with torch.no_grad():
        want = model(torch.from_numpy(toks)[None]).logits[0].numpy()
    got = orc.full_forward(orc.make_cfg(shape), orc.params_from_arrays(w), toks)
    assert np.abs(got - want).max() < 3e-4 * max(1.0, want.std()), np.abs(got - want).max()
    # the option matters: without the head norm the result is a different function
    plain = orc.full_forward(orc.make_cfg(MiniShape(**{**shape.__dict__, "qk_norm": False})), orc.params_from_arrays(w), toks)
    assert np.abs(plain - want).max() > 1e-2
    # and the paged decode step agrees with the forward under the option (the Eq. 1 = Eq. 2 + Eq. 3 identity)
    from test_oracle_pins import _prefill_into_pool, PT
    L = 20
    table = rng.permutation(6)[:3].astype(np.int32)
    ocfg, params = orc.make_cfg(shape), orc.params_from_arrays(w)
    base, pool = _prefill_into_pool(orc, shape, ocfg, params, toks[:L], 6, table, rng)
    ref = orc.full_forward(ocfg, params, toks[:L + 1], round_kv=True)
    r = orc.decode_step(ocfg, params, pool, toks[L:L + 1], table[None], [L], [0])
    assert np.abs(r["logits"][0] - ref[L]).max() < 1e-10


def test_scaled_rotary_frequencies_equal_transformers_llama3_rule(orc):
    """LLaMA-3.1 parameters (base 500000, head_dim 128, factor 8, low 1, high 4, original length 8192): the
    oracle's per-pair frequencies against the library's initialisation routine."""
    from transformers.modeling_rope_utils import ROPE_INIT_FUNCTIONS
    scaling = {"rope_type": "llama3", "factor": 8.0, "low_freq_factor": 1.0, "high_freq_factor": 4.0,
               "original_max_position_embeddings": 8192}
    try:
        cfg = transformers.LlamaConfig(hidden_size=4096, num_attention_heads=32, head_dim=128, rope_theta=500000.0,
                                       max_position_embeddings=131072, rope_scaling=dict(scaling))
    except TypeError:
        pytest.skip("this transformers version builds the rotary configuration differently")
    inv_freq, _ = ROPE_INIT_FUNCTIONS["llama3"](cfg, "cpu")
    shape = MiniShape(head_dim=128, rope_base=500000.0, rope_scaling=(8.0, 1.0, 4.0, 8192))
    ocfg = orc.make_cfg(shape)
    got = np.array([orc.rope_freq(ocfg, j) for j in range(64)])
    want = inv_freq.double().numpy()
    assert np.abs(got / want - 1).max() < 1e-6          # the library computes in float32
    plain = np.array([orc.rope_freq(orc.make_cfg(MiniShape(head_dim=128, rope_base=500000.0)), j) for j in range(64)])
    assert np.allclose(got[:20], plain[:20], rtol=1e-12) and np.allclose(got[-10:], plain[-10:] / 8.0, rtol=1e-12)
    assert (np.diff(got) < 0).all()


def test_scaled_rotary_variant_equals_transformers_llama(orc):
    shape = MiniShape(n_layers=2, n_q_heads=4, n_kv_heads=2, head_dim=32, hidden=128, ffn=96,
                      rope_scaling=(8.0, 1.0, 4.0, 64))
    rng = np.random.default_rng(33)
    w = random_weights(shape, rng, std=0.15)
    cfg = transformers.LlamaConfig(
        vocab_size=shape.vocab, hidden_size=shape.hidden, intermediate_size=shape.ffn, num_hidden_layers=shape.n_layers,
        num_attention_heads=shape.n_q_heads, num_key_value_heads=shape.n_kv_heads, head_dim=shape.head_dim,
        rms_norm_eps=shape.rms_eps, rope_theta=shape.rope_base, max_position_embeddings=512, attention_bias=False,
        mlp_bias=False, tie_word_embeddings=False, attn_implementation="eager",
        rope_scaling={"rope_type": "llama3", "factor": 8.0, "low_freq_factor": 1.0, "high_freq_factor": 4.0,
                      "original_max_position_embeddings": 64})
    model = transformers.LlamaForCausalLM(cfg).double().eval()
    _load(model, shape, w)
    toks = rng.integers(0, shape.vocab, size=150)       # long enough for the slowed pairs to matter
    with torch.no_grad():
        want = model(torch.from_numpy(toks)[None]).logits[0].numpy()
    got = orc.full_forward(orc.make_cfg(shape), orc.params_from_arrays(w), toks)
    assert np.abs(got - want).max() < 3e-4 * max(1.0, want.std()), np.abs(got - want).max()
    plain = orc.full_forward(orc.make_cfg(MiniShape(**{**shape.__dict__, "rope_scaling": None})), orc.params_from_arrays(w), toks)
    assert np.abs(plain - want).max() > 1e-3


def test_qkv_bias_variant_equals_transformers_qwen2(orc):
    """Backbone option of the Qwen2 class: bias vectors on the q, k and v projections (added before the rotation;
    the output projection has none)."""
    shape = MiniShape(n_layers=2, n_q_heads=4, n_kv_heads=2, head_dim=16, hidden=64, ffn=48, qkv_bias=True)
    rng = np.random.default_rng(35)
    w = random_weights(shape, rng)
    cfg = transformers.Qwen2Config(
        vocab_size=shape.vocab, hidden_size=shape.hidden, intermediate_size=shape.ffn, num_hidden_layers=shape.n_layers,
        num_attention_heads=shape.n_q_heads, num_key_value_heads=shape.n_kv_heads, rms_norm_eps=shape.rms_eps,
        rope_theta=shape.rope_base, max_position_embeddings=512, tie_word_embeddings=False, use_sliding_window=False,
        attn_implementation="eager")
    model = transformers.Qwen2ForCausalLM(cfg).double().eval()
    assert model.model.layers[0].self_attn.q_proj.bias is not None and model.model.layers[0].self_attn.o_proj.bias is None
    _load(model, shape, w)
    toks = rng.integers(0, shape.vocab, size=31)
    with torch.no_grad():
        want = model(torch.from_numpy(toks)[None]).logits[0].numpy()
    ocfg, params = orc.make_cfg(shape), orc.params_from_arrays(w)
    got = orc.full_forward(ocfg, params, toks)
    assert np.abs(got - want).max() < 3e-4 * max(1.0, want.std()), np.abs(got - want).max()
    # the option matters, and each of the three vectors does
    off = orc.full_forward(orc.make_cfg(MiniShape(**{**shape.__dict__, "qkv_bias": False})), params, toks)
    assert np.abs(off - want).max() > 1e-2
    for k in ("bq", "bk", "bv"):
        w2 = dict(w)
        w2[k] = [np.zeros_like(b) for b in w[k]]
        assert np.abs(orc.full_forward(ocfg, orc.params_from_arrays(w2), toks) - want).max() > 1e-3, k
    # and the paged decode step agrees with the forward under the option (the Eq. 1 = Eq. 2 + Eq. 3 identity)
    from test_oracle_pins import _prefill_into_pool
    L = 20
    table = rng.permutation(6)[:3].astype(np.int32)
    base, pool = _prefill_into_pool(orc, shape, ocfg, params, toks[:L], 6, table, rng)
    ref = orc.full_forward(ocfg, params, toks[:L + 1], round_kv=True)
    r = orc.decode_step(ocfg, params, pool, toks[L:L + 1], table[None], [L], [0])
    assert np.abs(r["logits"][0] - ref[L]).max() < 1e-10
