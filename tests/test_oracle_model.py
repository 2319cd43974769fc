"""Pins for the oracle's backbone pieces against closed forms, brute force and an independent library (no GPU)."""
import math

import pytest
import torch

import tidar_inputs as TI
from oracle import tidar_oracle as O


def test_rmsnorm_closed_forms():
    x = torch.tensor([[3.0, 4.0, 0.0, 0.0]], dtype=torch.float64)          # mean square = 25/4
    y = O.rmsnorm(x, torch.ones(4, dtype=torch.float64), 0.0)
    assert torch.allclose(y, x / 2.5)
    y2 = O.rmsnorm(7.0 * x, torch.full((4,), 2.0, dtype=torch.float64), 0.0)
    assert torch.allclose(y2, 2.0 * y)                                         # scale invariant, gain linear
    r = torch.randn(5, 64, dtype=torch.float64)
    out = O.rmsnorm(r, torch.ones(64, dtype=torch.float64), 0.0)
    assert torch.allclose((out * out).mean(-1), torch.ones(5, dtype=torch.float64))
    # eps enters under the square root, added to the mean square
    z = O.rmsnorm(torch.zeros(1, 4, dtype=torch.float64) + 1e-3, torch.ones(4, dtype=torch.float64), 1e-6)
    assert torch.allclose(z, torch.full((1, 4), 1e-3 / math.sqrt(1e-6 + 1e-6), dtype=torch.float64))


def test_silu_values():
    x = torch.tensor([0.0, 1.0, -1.0, 20.0], dtype=torch.float64)
    want = torch.tensor([0.0, 1.0 / (1.0 + math.exp(-1.0)), -1.0 / (1.0 + math.e), 20.0 / (1.0 + math.exp(-20.0))],
                        dtype=torch.float64)
    assert torch.allclose(O.silu(x), want, atol=1e-15)


def test_rope_properties():
    torch.manual_seed(0)
    hd = 8
    x = torch.randn(1, 1, hd, dtype=torch.float64)
    # position 0 is the identity; the rotation keeps norms
    assert torch.allclose(O.rope(x, torch.tensor([0]), 10000.0), x)
    y = O.rope(x, torch.tensor([5]), 10000.0)
    assert torch.allclose(y.norm(), x.norm())
    # the pair (i, i + hd/2) rotates by pos * base^(-2i/hd): explicit 2x2 rotation for pair 1
    ang = 5 * 10000.0 ** (-2.0 * 1 / hd)
    a, b = x[0, 0, 1], x[0, 0, 1 + hd // 2]
    assert torch.allclose(y[0, 0, 1], a * math.cos(ang) - b * math.sin(ang))
    assert torch.allclose(y[0, 0, 1 + hd // 2], b * math.cos(ang) + a * math.sin(ang))
    # scores depend on the position difference only
    q = torch.randn(1, 1, hd, dtype=torch.float64)
    kk = torch.randn(1, 1, hd, dtype=torch.float64)
    s1 = (O.rope(q, torch.tensor([9]), 10000.0) * O.rope(kk, torch.tensor([4]), 10000.0)).sum()
    s2 = (O.rope(q, torch.tensor([105]), 10000.0) * O.rope(kk, torch.tensor([100]), 10000.0)).sum()
    assert torch.allclose(s1, s2)


def _attention_loops(q, keys, vals, mask):
    """Brute force, one scalar at a time."""
    R, n_q, hd = q.shape
    n_kv = keys.shape[1]
    out = torch.zeros_like(q)
    for r in range(R):
        for h in range(n_q):
            g = h // (n_q // n_kv)
            cols = [t for t in range(keys.shape[0]) if mask[r, t]]
            sc = [sum(float(q[r, h, d]) * float(keys[t, g, d]) for d in range(hd)) / math.sqrt(hd) for t in cols]
            m = max(sc)
            e = [math.exp(s - m) for s in sc]
            z = sum(e)
            for d in range(hd):
                out[r, h, d] = sum(e[n] / z * float(vals[t, g, d]) for n, t in enumerate(cols))
    return out


@pytest.mark.parametrize("k,L,n_q,n_kv", [(1, 0, 2, 2), (2, 1, 4, 2), (3, 5, 4, 1), (4, 17, 2, 2), (2, 33, 4, 4)])
def test_hybrid_mask_attention_equals_brute_force(k, L, n_q, n_kv):
    torch.manual_seed(k * 100 + L)
    R, hd = O.q_len(k), 4
    q = torch.randn(R, n_q, hd, dtype=torch.float64)
    keys = torch.randn(L + R, n_kv, hd, dtype=torch.float64)
    vals = torch.randn(L + R, n_kv, hd, dtype=torch.float64)
    mask = O.decode_mask(k, L)
    got = O.attention_dense(q, keys, vals, mask)
    assert torch.allclose(got, _attention_loops(q, keys, vals, mask), atol=1e-12)


def test_attention_matches_library_sdpa():
    torch.manual_seed(3)
    k, L, n_q, n_kv, hd = 4, 9, 4, 2, 16
    R = O.q_len(k)
    q = torch.randn(R, n_q, hd, dtype=torch.float64)
    keys = torch.randn(L + R, n_kv, hd, dtype=torch.float64)
    vals = torch.randn(L + R, n_kv, hd, dtype=torch.float64)
    mask = O.decode_mask(k, L)
    got = O.attention_dense(q, keys, vals, mask)
    kk = keys.repeat_interleave(n_q // n_kv, dim=1)
    vv = vals.repeat_interleave(n_q // n_kv, dim=1)
    ref = torch.nn.functional.scaled_dot_product_attention(
        q.permute(1, 0, 2)[None], kk.permute(1, 0, 2)[None], vv.permute(1, 0, 2)[None], attn_mask=mask[None, None])
    assert torch.allclose(got, ref[0].permute(1, 0, 2), atol=1e-12)


@pytest.mark.parametrize("shape", [TI.TINY, TI.SMALL_GQA.with_layers(1)])
def test_causal_forward_matches_independent_transformer(shape):
    """The backbone F with a causal mask equals a library Llama-style decoder holding the same weights."""
    transformers = pytest.importorskip("transformers")
    from transformers import LlamaConfig, LlamaForCausalLM
    w = TI.make_weights(shape, seed=11)
    cfg = LlamaConfig(vocab_size=shape.vocab, hidden_size=shape.d_model, intermediate_size=shape.d_ff,
                      num_hidden_layers=shape.n_layers, num_attention_heads=shape.n_q_heads,
                      num_key_value_heads=shape.n_kv_heads, head_dim=shape.head_dim, hidden_act="silu",
                      max_position_embeddings=512, rms_norm_eps=shape.rms_eps, rope_theta=shape.rope_base,
                      attention_bias=False, mlp_bias=False, tie_word_embeddings=False,
                      attn_implementation="eager")
    ref = LlamaForCausalLM(cfg).double().eval()
    sd = {"model.embed_tokens.weight": w["embed"], "lm_head.weight": w["lm_head"], "model.norm.weight": w["final_norm"]}
    names = {"attn_norm": "input_layernorm.weight", "wq": "self_attn.q_proj.weight", "wk": "self_attn.k_proj.weight",
             "wv": "self_attn.v_proj.weight", "wo": "self_attn.o_proj.weight",
             "ffn_norm": "post_attention_layernorm.weight", "w_gate": "mlp.gate_proj.weight",
             "w_up": "mlp.up_proj.weight", "w_down": "mlp.down_proj.weight"}
    for l, lw in enumerate(w["layers"]):
        for kname, hname in names.items():
            sd[f"model.layers.{l}.{hname}"] = lw[kname]
    missing, unexpected = ref.load_state_dict({k: v.double() for k, v in sd.items()}, strict=False)
    assert not [m for m in missing if "rotary" not in m] and not unexpected
    prompt = TI.make_prompt(shape, 23, seed=5)[0]
    with torch.no_grad():
        want = ref(input_ids=prompt.long()[None]).logits[0]                     # [P, V]
    model = O.OracleModel(shape, w)
    st = model.new_state(64)
    got, _, _ = model.forward(prompt.long(), torch.arange(23), O.causal_mask(23, 0), st)
    # the library builds its cos/sin tables in fp32, so agreement stops near 1e-7; a wrong pairing, sign,
    # scale or norm placement shows up at 1e-2 and above
    assert torch.allclose(got, want, atol=1e-6), float((got - want).abs().max())


def test_rounded_softmax_numerators_do_not_depend_on_power_of_two_reference():
    """Reading K: bf16 rounding of 2^(s - ref) is the same for every integral ref (pure exponent shift)."""
    torch.manual_seed(5)
    s2 = torch.randn(7, 300, dtype=torch.float64) * 4.0
    ref = torch.ceil(s2.max(dim=-1, keepdim=True).values)
    e1 = O.round_bf16(torch.exp2(s2 - ref))
    e2 = O.round_bf16(torch.exp2(s2 - (ref + 5.0)))
    assert torch.equal(e1, e2 * 32.0)
    assert float(e1.max()) <= 1.0 and float(e1.max()) > 0.5


def test_rounded_attention_stays_within_bf16_resolution_of_exact():
    torch.manual_seed(6)
    k, L, n_q, n_kv, hd = 4, 50, 4, 2, 16
    R = O.q_len(k)
    q = torch.randn(R, n_q, hd, dtype=torch.float64)
    keys = torch.randn(L + R, n_kv, hd, dtype=torch.float64)
    vals = torch.randn(L + R, n_kv, hd, dtype=torch.float64)
    mask = O.decode_mask(k, L)
    exact = O.attention_dense(q, keys, vals, mask)
    rounded = O.attention_dense(q, keys, vals, mask, round_p=True)
    err = float((exact - rounded).abs().max())
    assert 0.0 < err < 2.0 ** -8
