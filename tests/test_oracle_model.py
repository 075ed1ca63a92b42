"""Oracle target model against an independent library implementation of the Llama
architecture (Hugging Face `LlamaForCausalLM`, float64, CPU) and against the paper's
parameter count."""
import os

import numpy as np
import pytest
import torch

from synth import get_config, make_weights, make_prompt
from oracle.model import Weights, target_full, target_rows, head, causal_allowed, empty_kv, specialist_index
from oracle.greedy import greedy_decode

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _hf_model(cfg, W):
    from transformers import LlamaConfig, LlamaForCausalLM
    hc = LlamaConfig(hidden_size=cfg.d_model, intermediate_size=cfg.d_ffn,
                     num_hidden_layers=cfg.n_layers, num_attention_heads=cfg.n_q_heads,
                     num_key_value_heads=cfg.n_kv_heads, head_dim=cfg.head_dim, vocab_size=cfg.vocab,
                     rms_norm_eps=cfg.rms_eps, rope_theta=cfg.rope_theta, max_position_embeddings=1024,
                     attention_bias=False, mlp_bias=False, tie_word_embeddings=False,
                     attn_implementation="eager")
    m = LlamaForCausalLM(hc).double().eval()
    sd = {"model.embed_tokens.weight": W("embed"), "lm_head.weight": W("lm_head"),
          "model.norm.weight": W("final_norm")}
    names = {"attn_norm": "input_layernorm", "wq": "self_attn.q_proj", "wk": "self_attn.k_proj",
             "wv": "self_attn.v_proj", "wo": "self_attn.o_proj", "mlp_norm": "post_attention_layernorm",
             "w_gate": "mlp.gate_proj", "w_up": "mlp.up_proj", "w_down": "mlp.down_proj"}
    for l in range(cfg.n_layers):
        for mine, theirs in names.items():
            sd[f"model.layers.{l}.{theirs}.weight"] = W(f"layer{l}.{mine}")
    missing = m.load_state_dict({k: torch.from_numpy(np.ascontiguousarray(v)) for k, v in sd.items()}, strict=False)
    assert not [k for k in missing.missing_keys if "rotary" not in k], missing
    return m


@pytest.mark.parametrize("name", ["c0_tiny_f32", "t_tiny_f32_6x1"])
def test_target_matches_hf_llama(name):
    cfg = get_config(name)                      # second shape: grouped KV heads, jittered norm gains
    W = Weights(cfg, make_weights(cfg))
    m = _hf_model(cfg, W)
    prompt = make_prompt(cfg, n=40)
    feats, logits = target_full(W, cfg, prompt)
    with torch.no_grad():
        out = m(torch.from_numpy(prompt.astype(np.int64))[None], output_hidden_states=True)
    # HF evaluates the rotary angles in float32 whatever the model dtype, hence 1e-6 and not 1e-12
    assert np.abs(logits - out.logits[0].numpy()).max() < 2e-6
    # the feature is the last hidden state BEFORE the final norm; HF's last entry is after it
    normed = m.model.norm(torch.from_numpy(feats)).detach().numpy()
    assert np.abs(normed - out.hidden_states[-1][0].numpy()).max() < 2e-6


def test_greedy_matches_hf_generate():
    cfg = get_config("c0_tiny_f32")
    W = Weights(cfg, make_weights(cfg))
    m = _hf_model(cfg, W)
    prompt = make_prompt(cfg, n=24)
    mine = greedy_decode(W, cfg, prompt, 8)
    with torch.no_grad():
        ids = m.generate(torch.from_numpy(prompt.astype(np.int64))[None], max_new_tokens=8,
                         do_sample=False, use_cache=False, eos_token_id=None, pad_token_id=0)
    assert mine == ids[0].tolist()


def test_rows_with_context_equal_full_pass():
    """Splitting a causal pass into context + new rows changes nothing (cache semantics)."""
    cfg = get_config("t_tiny_f32_6x1")
    W = Weights(cfg, make_weights(cfg))
    toks = make_prompt(cfg, n=30)
    f_full, logits_full = target_full(W, cfg, toks)
    f0, kv = target_rows(W, cfg, toks[:19], np.arange(19), empty_kv(cfg), causal_allowed(0, 19))
    f1, _ = target_rows(W, cfg, toks[19:], np.arange(19, 30), kv, causal_allowed(19, 11))
    assert np.allclose(np.concatenate([f0, f1]), f_full, rtol=1e-10, atol=1e-12)
    assert np.allclose(head(W, cfg, f1), logits_full[19:], rtol=1e-10, atol=1e-12)


def test_layer_parameter_count_of_the_paper():
    for line in open(os.path.join(GOLD, "param_count.txt")):
        if line.startswith("#") or not line.strip():
            continue
        d, hq, hkv, dh, f, millions = (int(x) for x in line.split())
        cfg = get_config("c1_llama3_8b_3x2")
        assert (cfg.d_model, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.d_ffn) == (d, hq, hkv, dh, f)
        from synth import tensor_specs
        n = sum(int(np.prod(s)) for nm, s, kind in tensor_specs(cfg)
                if nm.startswith("spec0.") and kind == "w" and not nm.endswith("fc_w"))
        assert n == 218_103_808 and round(n / 1e6) == millions


def test_specialist_assignment_of_the_paper():
    for line in open(os.path.join(GOLD, "specialist_assignment.txt")):
        if line.startswith("#") or not line.strip():
            continue
        p = line.split()
        if p[0] == "layers":
            n, depth, layers = int(p[1]), int(p[2]), int(p[3])
            used = {specialist_index(i, n, 99) for i in range(depth)}
            assert len(used) == layers == -(-depth // n)
        else:
            n, pos, spec = (int(x) for x in p)
            assert specialist_index(pos, n, 99) + 1 == spec
    # depth beyond S*n stays with the last specialist (reading; unpinned by the paper)
    assert [specialist_index(i, 2, 3) for i in range(8)] == [0, 0, 1, 1, 2, 2, 2, 2]
