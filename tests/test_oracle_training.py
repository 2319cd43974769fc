"""Pins for the oracle's training-layout forward, its objective and AR-mode scoring (no GPU).

Section 3.1 (doubled sequence, objective), Figure 3 left caption (training mask), Section 4.2.2 (likelihood in AR
mode).  Each pin is something other than the oracle's own formula: a hand-written worked mask, a closed-form
count, a library decoder fed the same mask, the already-pinned prefill and causal forwards, closed-form losses.
"""
import math
import os

import pytest
import torch

import tidar_inputs as TI
from oracle import tidar_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _read_matrix(name):
    rows = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            rows.append([int(v) for v in line.split()])
    return torch.tensor(rows, dtype=torch.bool)


def test_training_mask_worked_example():
    assert torch.equal(O.training_mask(6, 3), _read_matrix("training_mask_s6_b3.txt"))


@pytest.mark.parametrize("S,bl", [(1, 1), (6, 3), (7, 3), (16, 16), (33, 4), (40, 16), (5, 8)])
def test_training_mask_counts_and_structure(S, bl):
    M = O.training_mask(S, bl)
    lens = [min(bl, S - j * bl) for j in range((S + bl - 1) // bl)]
    want = S * (S + 1) // 2 + sum(n * (j * bl + n) for j, n in enumerate(lens))
    assert int(M.sum()) == want
    assert not M[:S, S:].any()                                   # text never sees a mask
    assert torch.equal(M[S:, S:], M[S:, S:].T)                   # mask-to-mask part is symmetric (bidirectional)
    assert M.diagonal().all()
    # with block length 1 a mask sees exactly the text in front of it plus itself
    M1 = O.training_mask(S, 1)
    for i in range(S):
        assert int(M1[S + i].sum()) == i + 1
    pos = O.training_positions(S)
    assert torch.equal(pos[:S], pos[S:]) and torch.equal(pos[:S], torch.arange(S))


def _library_llama(shape, w):
    pytest.importorskip("transformers")
    from transformers import LlamaConfig, LlamaForCausalLM
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
    return ref


@pytest.mark.parametrize("shape", [TI.TINY, TI.SMALL_GQA.with_layers(1)])
def test_score_equals_library_causal_lm_loss(shape):
    """AR-mode likelihood: the mean of -score is the causal-LM loss a library decoder reports for the same text."""
    w = TI.make_weights(shape, seed=21, std=0.08)             # larger weights: the distribution is far from uniform
    ref = _library_llama(shape, w)
    text = TI.make_prompt(shape, 19, seed=8)[0].long()
    with torch.no_grad():
        out = ref(input_ids=text[None], labels=text[None])
    lp = O.OracleModel(shape, w).score(text.tolist())
    assert lp.shape == (18,)
    assert abs(float(-lp.mean()) - float(out.loss)) < 1e-6
    # and token by token against the library's logits
    want = torch.log_softmax(out.logits[0, :-1], dim=-1)[torch.arange(18), text[1:]]
    assert torch.allclose(lp, want, atol=1e-6)
    assert float((lp - lp.mean()).abs().max()) > 1e-2         # not a degenerate (uniform) case


@pytest.mark.parametrize("S,bl", [(12, 4), (11, 4)])
def test_training_forward_equals_library_decoder_with_the_same_mask(S, bl):
    """The whole doubled-sequence forward against a library decoder given the worked mask as a 4-D additive mask."""
    shape = TI.SMALL_GQA.with_layers(2)
    w = TI.make_weights(shape, seed=22, std=0.08)
    ref = _library_llama(shape, w)
    text = TI.make_prompt(shape, S, seed=9)[0].long()
    rows = torch.cat([text, torch.full((S,), shape.mask_token_id)])
    # the additive mask is built here from the rule in words, not from the oracle's function
    add = torch.full((2 * S, 2 * S), float("-inf"), dtype=torch.float64)
    for r in range(2 * S):
        for c in range(2 * S):
            if r < S:
                ok = c <= r
            else:
                blk = (r - S) // bl
                ok = (c < S and c < blk * bl) or (c >= S and (c - S) // bl == blk)
            if ok:
                add[r, c] = 0.0
    pos = torch.cat([torch.arange(S), torch.arange(S)])
    with torch.no_grad():
        want = ref(input_ids=rows[None], attention_mask=add[None, None], position_ids=pos[None]).logits[0]
    model = O.OracleModel(shape, w)
    ar, diff, logits = model.training_forward(text.tolist(), bl)
    assert torch.allclose(logits, want, atol=1e-6), float((logits - want).abs().max())
    lp = torch.log_softmax(want, dim=-1)
    assert torch.allclose(ar, lp[torch.arange(S - 1), text[1:]], atol=1e-6)
    assert torch.allclose(diff, lp[S + torch.arange(S), text], atol=1e-6)


@pytest.mark.parametrize("S,bl", [(13, 4), (8, 8), (9, 2)])
def test_training_sections_reduce_to_the_decode_time_forwards(S, bl):
    """Causal section == plain causal forward (masks never leak into it); block j of the mask section == the
    prefill forward over the text in front of it plus one block of masks (what decoding drafts from)."""
    shape = TI.TINY
    w = TI.make_weights(shape, seed=23, std=0.05)
    model = O.OracleModel(shape, w)
    text = TI.make_prompt(shape, S, seed=10)[0].long().tolist()
    ar, diff, logits = model.training_forward(text, bl)
    st = model.new_state(S)
    causal, _, _ = model.forward(torch.tensor(text), torch.arange(S), O.causal_mask(S, 0), st)
    assert torch.allclose(logits[:S], causal, atol=1e-12)
    assert torch.allclose(ar, model.score(text), atol=1e-12)
    for j in range(1, (S + bl - 1) // bl):
        n = min(bl, S - j * bl)
        st = model.new_state(S)
        _, pl = model.prefill(st, text[: j * bl], n)           # rows: last prompt row, then the n mask rows
        assert torch.allclose(logits[S + j * bl: S + j * bl + n], pl[1:], atol=1e-12)
    # the mask token's own embedding must not matter to the causal section
    w2 = TI.make_weights(shape, seed=23, std=0.05)
    w2["embed"][shape.mask_token_id] += 1.0
    _, _, logits2 = O.OracleModel(shape, w2).training_forward(text, bl)
    assert torch.equal(logits2[:S], logits[:S])
    assert not torch.allclose(logits2[S:], logits[S:])


def test_objective_closed_forms():
    # a model whose logits are all equal assigns 1/V to every token: both losses are ln V for every alpha
    shape = TI.TINY
    w = TI.make_weights(shape, seed=24)
    w["lm_head"] = torch.zeros_like(w["lm_head"])
    model = O.OracleModel(shape, w)
    text = TI.make_prompt(shape, 10, seed=11)[0].long().tolist()
    ar, diff, _ = model.training_forward(text, 4)
    for alpha in (0.0, 0.3, 1.0):
        assert abs(O.tidar_loss(ar, diff, alpha) - math.log(shape.vocab)) < 1e-12
    # weighting: alpha = 0 is the mask-section mean alone, alpha = 1 the plain average of the two means
    a = torch.tensor([-1.0, -2.0, -3.0], dtype=torch.float64)
    d = torch.tensor([-4.0, -6.0, -8.0, -100.0], dtype=torch.float64)      # the last position takes no part
    assert O.tidar_loss(a, d, 0.0) == pytest.approx(6.0)
    assert O.tidar_loss(a, d, 1.0) == pytest.approx((2.0 + 6.0) / 2.0)
    assert O.tidar_loss(a, d, 0.5) == pytest.approx((0.5 * 2.0 + 6.0) / 1.5)
