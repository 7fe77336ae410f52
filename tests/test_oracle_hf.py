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
    for l in range(shape.n_layers):
        for k, n in names.items():
            sd[f"model.layers.{l}.{n}.weight"] = w[k][l]
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
