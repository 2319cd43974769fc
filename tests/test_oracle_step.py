"""Pins for the oracle's decode step against the plain definition it must reach: causal AR decoding (no GPU)."""
import numpy as np
import pytest
import torch

import tidar_inputs as TI
from oracle import tidar_oracle as O

SHAPE = TI.TINY


@pytest.fixture(scope="module")
def model():
    return O.OracleModel(SHAPE, TI.make_weights(SHAPE, seed=1))


@pytest.fixture(scope="module")
def prompt():
    return [int(t) for t in TI.make_prompt(SHAPE, 64, seed=2)[0]]


def test_causal_logits_ignore_mask_tokens(model, prompt):
    """Check 2: logits at the causal rows do not depend on what sits in the mask slots, and equal a plain
    causal forward over prefix + c_1..c_i."""
    k = 4
    st = model.new_state(128)
    model.causal_prefill(st, prompt)
    drafts = [int(t) for t in TI.make_drafts(SHAPE, k, seed=3)[0]]
    L = st.L
    toks = torch.tensor(drafts + [SHAPE.mask_token_id] * (k * k))
    a, _, _ = model.forward(toks, O.decode_positions(k, L), O.decode_mask(k, L), st)
    toks2 = toks.clone()
    toks2[k:] = torch.randint(0, SHAPE.vocab, (k * k,), generator=torch.Generator().manual_seed(9))
    b, _, _ = model.forward(toks2, O.decode_positions(k, L), O.decode_mask(k, L), st)
    assert torch.equal(a[:k], b[:k])
    assert not torch.equal(a[k:], b[k:])
    c, _, _ = model.forward(torch.tensor(drafts), torch.arange(L, L + k), O.causal_mask(k, L), st)
    assert torch.allclose(a[:k], c, atol=1e-12)


@pytest.mark.parametrize("k", [1, 2, 4, 8])
def test_greedy_tidar_equals_ar_decode_for_any_drafts(model, prompt, k):
    """Check 3: token for token, whatever the untrusted draft slots hold."""
    n = 24
    want = model.ar_decode(prompt, n)
    got_natural, acc = model.tidar_decode(prompt, n, k)
    assert got_natural == want
    assert all(1 <= a <= k for a in acc)
    rng = np.random.default_rng(k)
    junk = lambda step, d, L: [d[0]] + [int(x) for x in rng.integers(0, SHAPE.vocab, len(d) - 1)]
    got_junk, _ = model.tidar_decode(prompt, n, k, draft_override=junk)
    assert got_junk == want


def test_forced_drafts_acceptance_lengths(model, prompt):
    """Check 4: drafts equal to the next AR tokens are all accepted; correct up to j then wrong gives a = j."""
    k, n = 4, 24
    P = len(prompt)
    want = model.ar_decode(prompt, n + 2 * k)

    def perfect(step, d, L):
        return want[L - P: L - P + k]

    out, acc = model.tidar_decode(prompt, n, k, draft_override=perfect)
    assert out == want[:n]
    assert acc == [k] * (n // k)
    for j in range(1, k + 1):
        def upto(step, d, L, j=j):
            good = want[L - P: L - P + k]
            return good[:j] + [(t + 1) % (SHAPE.vocab - 1) for t in good[j:]]
        out, acc = model.tidar_decode(prompt, n, k, draft_override=upto)
        assert out == want[:n]
        assert all(a == j for a in acc), (j, acc)
        assert sum(acc) >= n


def test_cache_after_steps_is_exact_causal_cache(model, prompt):
    k, n = 4, 13
    st = model.new_state(128)
    drafts, _ = model.prefill(st, prompt, k)
    out = []
    while len(out) < n:
        a, accepted, drafts, _ = model.tidar_step(st, drafts)
        out.extend(accepted)
    ref = model.new_state(128)
    model.causal_prefill(ref, prompt + out)
    assert st.L == ref.L == len(prompt) + len(out)
    for l in range(SHAPE.n_layers):
        assert torch.allclose(st.k[l][:st.L], ref.k[l][:ref.L], atol=1e-12)
        assert torch.allclose(st.v[l][:st.L], ref.v[l][:ref.L], atol=1e-12)


def test_next_drafts_are_the_selected_blocks_predictions(model, prompt):
    """next[1] is the AR token at the new frontier; next[2..k] equal the argmax of a separately computed
    forward over [text ; k masks] with the prefill-style mask."""
    k = 4
    st = model.new_state(128)
    drafts, _ = model.prefill(st, prompt, k)
    text = list(prompt)
    for _ in range(3):
        a, accepted, nxt, _ = model.tidar_step(st, drafts)
        text += accepted
        fresh = model.new_state(128)
        first, _ = model.prefill(fresh, text, k)
        assert first == nxt
        drafts = nxt


def test_prefill_first_token_is_causal_prediction(model, prompt):
    st = model.new_state(128)
    first, _ = model.prefill(st, prompt, 4)
    assert first[0] == model.ar_decode(prompt, 1)[0]


def test_sampled_tidar_equals_sampled_ar(model, prompt):
    mode = O.Mode(sample=True, temperature=1.0, seed=1234)
    want = model.ar_decode(prompt, 20, mode)
    got, _ = model.tidar_decode(prompt, 20, 4, mode)
    assert got == want
    assert want != model.ar_decode(prompt, 20)                 # it really samples
    other = model.ar_decode(prompt, 20, O.Mode(sample=True, temperature=1.0, seed=99))
    assert other != want


def test_sampling_temperature_to_zero_is_greedy(model, prompt):
    cold = O.Mode(sample=True, temperature=1e-6, seed=5)
    assert model.ar_decode(prompt, 8, cold) == model.ar_decode(prompt, 8)


def test_gumbel_max_frequencies_follow_softmax():
    """Chi-square of position-keyed Gumbel-max draws against the softmax probabilities."""
    V, n = 8, 20000
    logits = np.array([0.0, 1.0, -1.0, 0.5, 2.0, -0.5, 0.3, 1.5])
    p = np.exp(logits) / np.exp(logits).sum()
    counts = np.zeros(V)
    for pos in range(n):
        counts[int(np.argmax(logits + O.gumbel_noise(77, 0, pos, V)))] += 1
    chi2 = float(((counts - n * p) ** 2 / (n * p)).sum())
    assert chi2 < 24.3                                           # 0.999 quantile of chi-square with 7 dof
    u = (O.hash_u24(77, 0, 0, 4096).astype(np.float64) + 0.5) / (1 << 24)
    assert 0.0 < u.min() and u.max() < 1.0 and abs(u.mean() - 0.5) < 0.02


def test_hash_is_keyed_by_every_field():
    base = O.hash_u24(1, 0, 10, 16)
    assert not np.array_equal(base, O.hash_u24(2, 0, 10, 16))
    assert not np.array_equal(base, O.hash_u24(1, 1, 10, 16))
    assert not np.array_equal(base, O.hash_u24(1, 0, 11, 16))
    assert len(set(base.tolist())) > 12
    assert np.array_equal(base, O.hash_u24(1, 0, 10, 32)[:16])  # entry v does not depend on the vocabulary size


def test_beta_one_is_default_and_mix_changes_only_verification(model, prompt):
    k = 4
    st1, st2 = model.new_state(128), model.new_state(128)
    d1, _ = model.prefill(st1, prompt, k)
    d2, _ = model.prefill(st2, prompt, k)
    a1, _, n1, lg1 = model.tidar_step(st1, d1, O.Mode(beta=1.0))
    a2, _, n2, lg2 = model.tidar_step(st2, d2, O.Mode(beta=0.5))
    assert torch.equal(lg1, lg2)
    i = a2
    mixed = 0.5 * lg2[O.row_of_c(i)] + 0.5 * lg2[O.row_of_blk(k, i, 1)]
    assert n2[0] == int(torch.argmax(mixed))


def test_bf16_faithful_mode_stays_close_to_exact(prompt):
    w = TI.make_weights(SHAPE, seed=1, dtype=torch.bfloat16)
    exact = O.OracleModel(SHAPE, w)
    faithful = O.OracleModel(SHAPE, w, bf16_faithful=True)
    s1, s2 = exact.new_state(128), faithful.new_state(128)
    _, l1 = exact.prefill(s1, prompt, 4)
    _, l2 = faithful.prefill(s2, prompt, 4)
    err = float((l1 - l2).abs().max())
    assert 0.0 < err < 2e-2


def _mixed_verification_by_separate_forwards(model, text, drafts, beta):
    """What Section 4.3.3 asks of a step, built without the step: for every i, ONE prefill-style forward over
    [text + c_1..c_i ; k masks] gives the causal logits of c_i (last text row) and the logits of the first mask
    slot, both predicting the token after c_i; the verifier's token is the argmax of their beta-mix.  Returns
    (acceptance length, the verifier's token at the first unverified position, all k verifier tokens)."""
    k = len(drafts)
    y = []
    for i in range(1, k + 1):
        fresh = model.new_state(len(text) + 2 * k + 2)
        _, lg = model.prefill(fresh, list(text) + list(drafts[:i]), k)      # rows: last text row, mask slots 1..k
        y.append(int(torch.argmax(beta * lg[0] + (1.0 - beta) * lg[1])))
    a = 1
    while a < k and drafts[a] == y[a - 1]:
        a += 1
    return a, y[a - 1], y


@pytest.fixture(scope="module")
def sharp_model():
    """Weights ten times wider than the default recipe: with N(0, 0.02) the mask rows of this untrained tiny model all
    choose the same token, so that no pairing of rows could be told from another; at 0.2 every slot of every block
    has its own prediction."""
    return O.OracleModel(SHAPE, TI.make_weights(SHAPE, seed=1, std=0.2))


@pytest.mark.parametrize("beta", [0.0, 0.3, 1.0])
def test_beta_mix_pairs_each_causal_row_with_the_first_slot_of_its_own_block(sharp_model, prompt, beta, monkeypatch):
    """Pin of Mode.beta that does not reuse the step's own mix line or row helpers: the step's acceptance length
    and first next-draft must equal those of a verifier assembled from separate prefill-style forwards (one per
    draft count), for drafts built to be accepted up to a chosen length.  beta = 0 is verification by the
    diffusion logits alone, beta = 1 the default.  A planted wrong pairing (another slot, another block) in the
    oracle must fail the same comparison."""
    model = sharp_model
    k = 4
    st = model.new_state(160)
    drafts, _ = model.prefill(st, prompt, k)
    text = list(prompt)
    mode = O.Mode(beta=beta)
    differs_from_default = False
    for step in range(4):
        # drafts the mixed verifier accepts up to length `want_a`: take its own tokens, then a wrong one
        want_a = 1 + step % k
        c = [drafts[0]]
        for i in range(1, k):
            _, _, y = _mixed_verification_by_separate_forwards(model, text, c + [0] * (k - len(c)), beta)
            c.append(y[i - 1] if i < want_a else (y[i - 1] + 1) % (SHAPE.vocab - 1))
        a_ref, nxt0_ref, y_ref = _mixed_verification_by_separate_forwards(model, text, c, beta)
        assert a_ref == want_a
        _, _, y_default = _mixed_verification_by_separate_forwards(model, text, c, 1.0)
        differs_from_default |= y_ref != y_default
        probe = O.State([t.clone() for t in st.k], [t.clone() for t in st.v], st.L, st.seq_id)
        a, accepted, nxt, _ = model.tidar_step(st, c, mode)
        assert (a, nxt[0]) == (a_ref, nxt0_ref), (step, a, a_ref)
        assert accepted == c[:a]
        if beta != 1.0 and step == 3:
            # the same comparison must catch a wrong pairing planted in the oracle
            # (planted in the mix line alone: mask and positions of the planted runs are the real ones, computed
            # before the helper is replaced; a helper replaced everywhere would only relabel the blocks)
            real = O.row_of_blk
            real_mask, real_pos = O.decode_mask(k, probe.L), O.decode_positions(k, probe.L)
            monkeypatch.setattr(O, "decode_mask", lambda kk, LL: real_mask)
            monkeypatch.setattr(O, "decode_positions", lambda kk, LL: real_pos)
            for wrong in (lambda kk, j, s: real(kk, j, s + 1 if s == 1 else s),            # second slot
                          lambda kk, j, s: real(kk, j % kk + 1 if s == 1 else j, s),        # next block
                          lambda kk, j, s: real(kk, (j - 2) % kk + 1 if s == 1 else j, s)):  # previous block
                p2 = O.State([t.clone() for t in probe.k], [t.clone() for t in probe.v], probe.L, probe.seq_id)
                monkeypatch.setattr(O, "row_of_blk", wrong)
                a_bad, _, nxt_bad, _ = model.tidar_step(p2, c, mode)
                monkeypatch.setattr(O, "row_of_blk", real)
                assert (a_bad, nxt_bad[0]) != (a_ref, nxt0_ref)
            monkeypatch.undo()
        text += accepted
        drafts = nxt
    if beta != 1.0:
        assert differs_from_default          # the mix really changed at least one verifier token


def test_beta_one_equals_the_default_step(model, prompt):
    k = 4
    s1, s2 = model.new_state(128), model.new_state(128)
    d1, _ = model.prefill(s1, prompt, k)
    d2, _ = model.prefill(s2, prompt, k)
    for _ in range(3):
        r1 = model.tidar_step(s1, d1)
        r2 = model.tidar_step(s2, d2, O.Mode(beta=1.0))
        assert r1[:3] == r2[:3] and torch.equal(r1[3], r2[3])
        d1, d2 = r1[2], r2[2]
