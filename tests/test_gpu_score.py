"""GPU parity of AR-mode scoring and of the training-layout forward (Section 4.2.2, Section 3.1) through the C ABI."""
import pytest
import torch

import tidar_inputs as TI
from oracle import tidar_oracle as O

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def T():
    import paper_2511_08923_amd as T
    assert torch.cuda.is_available()
    return T


def _oracle_scores(model, text, bl):
    if bl == 0:
        return model.score(text), None
    ar, diff, _ = model.training_forward(text, bl)
    return ar, diff


# passes: one pass; several passes with a ragged tail; a chunk that is not a multiple of the block (rounded down to
# 6); a block longer than the text; block length 1; a one-token and a two-token text
@pytest.mark.parametrize("S,bl,chunk", [(37, 4, None), (200, 4, 64), (50, 3, 7), (9, 16, None), (23, 1, 8),
                                        (1, 4, None), (2, 4, None), (64, 16, 16), (150, 0, 64), (31, 0, None)])
def test_tiny_fp32_scores_match_oracle(T, S, bl, chunk):
    sh = TI.TINY
    w = TI.make_weights(sh, seed=1, std=0.05)
    eng = T.Engine(sh, w, dtype=T.TIDAR_F32, max_k=16, max_batch=1, max_seq_len=256, prefill_chunk=chunk)
    model = O.OracleModel(sh, w)
    text = TI.make_prompt(sh, S, seed=70 + S)
    tl = [int(t) for t in text[0]]
    print(f"score fp32 S={S} bl={bl} chunk={chunk}", flush=True)
    ar, diff, loss = eng.score(text, block_len=bl, alpha=0.7)
    torch.cuda.synchronize()
    if S >= 2:
        ar_o, diff_o = _oracle_scores(model, tl, bl)
        assert float((ar[0, : S - 1].cpu().double() - ar_o).abs().max()) < 3e-4
        assert float(ar[0, S - 1]) == 0.0
        if bl:
            assert float((diff[0].cpu().double() - diff_o).abs().max()) < 3e-4
            want = O.tidar_loss(ar_o, diff_o, 0.7)
        else:
            want = float(-ar_o.mean())
        assert abs(float(loss[0]) - want) < 3e-4
    else:
        assert float(ar[0, 0]) == 0.0 and float(loss[0]) == 0.0
        if bl:                                               # a lone mask row that sees only itself
            _, diff_o, _ = model.training_forward(tl, bl)
            assert float((diff[0].cpu().double() - diff_o).abs().max()) < 3e-4
    # the cache now holds the text's causal K/V
    st = model.new_state(S)
    _, nk, nv = model.forward(torch.tensor(tl), torch.arange(S), O.causal_mask(S, 0), st)
    for l in range(sh.n_layers):
        kk, vv = eng.read_cache(l, 0, S)
        assert float((kk.cpu().double() - nk[l]).abs().max()) < 1e-4
        assert float((vv.cpu().double() - nv[l]).abs().max()) < 1e-4
    eng.close()


def test_tiny_fp32_batch_of_ragged_texts(T):
    sh = TI.TINY
    w = TI.make_weights(sh, seed=1, std=0.05)
    eng = T.Engine(sh, w, dtype=T.TIDAR_F32, max_k=8, max_batch=3, max_seq_len=128, prefill_chunk=32)
    model = O.OracleModel(sh, w)
    text = TI.make_prompt(sh, 90, seed=77, batch=3)
    lens = [90, 5, 41]
    ar, diff, loss = eng.score(text, block_len=8, alpha=1.0, length=lens)
    torch.cuda.synchronize()
    for b, n in enumerate(lens):
        ar_o, diff_o, _ = model.training_forward([int(t) for t in text[b, :n]], 8)
        assert float((ar[b, : n - 1].cpu().double() - ar_o).abs().max()) < 3e-4
        assert float((diff[b, :n].cpu().double() - diff_o).abs().max()) < 3e-4
        assert abs(float(loss[b]) - O.tidar_loss(ar_o, diff_o, 1.0)) < 3e-4
        assert float(ar[b, n:].abs().max() if n < 90 else 0.0) == 0.0       # untouched beyond the text
    eng.close()


def test_score_argument_errors(T):
    sh = TI.TINY
    w = TI.make_weights(sh, seed=1)
    eng = T.Engine(sh, w, dtype=T.TIDAR_F32, max_k=8, max_batch=1, max_seq_len=64)
    text = TI.make_prompt(sh, 32, seed=3).to("cuda")
    ar = torch.zeros(1, 32, device="cuda")
    diff = torch.zeros(1, 32, device="cuda")
    for args, status in [
        (dict(block_len=4, diff=None), 1),          # mask section asked for, nowhere to put it
        (dict(block_len=0, diff=diff), 1),
        (dict(block_len=17, diff=diff), 1),
        (dict(block_len=4, diff=diff, alpha=1.5), 1),
        (dict(block_len=4, diff=diff, lens=[0]), 1),
        (dict(block_len=4, diff=diff, lens=[33]), 1),
        (dict(block_len=4, diff=diff, ws=torch.empty(1024, dtype=torch.uint8, device="cuda")), 2),
    ]:
        with pytest.raises(T.TidarError) as e:
            T.tidar_score(eng.ctx, eng.w, eng.kv, 1, text, args.get("lens", [32]), args["block_len"],
                          args.get("alpha", 1.0), ar, args["diff"], None, args.get("ws", eng.ws))
        assert e.value.status == status
    big = TI.make_prompt(sh, 80, seed=3).to("cuda")          # longer than the page table allows (64)
    with pytest.raises(T.TidarError) as e:
        T.tidar_score(eng.ctx, eng.w, eng.kv, 1, big, [80], 0, 1.0, torch.zeros(1, 80, device="cuda"), None, None,
                      eng.ws)
    assert e.value.status == 3
    eng.close()


SCORE_TOL = 4e-2        # a logit within 2e-2 of the oracle's and a log-sum-exp within 2e-2


@pytest.mark.parametrize("S,bl,chunk", [(300, 16, None), (700, 8, 256), (333, 5, 100), (1100, 0, 1024)])
def test_small_bf16_scores_match_oracle(T, S, bl, chunk):
    """bf16 MFMA path: one pass of 600 rows; three passes of 512 rows and a ragged one; blocks of 5 that straddle
    the 16-key tiles with a short last block; causal-only scoring in a pass of 1024 rows and one of 76."""
    sh = TI.SMALL_GQA
    w = TI.make_weights(sh, seed=3, dtype=torch.bfloat16, std=0.05)
    eng = T.Engine(sh, w, dtype=T.TIDAR_BF16, max_k=16, max_batch=1, max_seq_len=1280, prefill_chunk=chunk)
    model = O.OracleModel(sh, w, bf16_faithful=True)
    text = TI.make_prompt(sh, S, seed=80 + S)
    tl = [int(t) for t in text[0]]
    print(f"score bf16 S={S} bl={bl} chunk={chunk}", flush=True)
    ar, diff, loss = eng.score(text, block_len=bl, alpha=1.0)
    torch.cuda.synchronize()
    ar_o, diff_o = _oracle_scores(model, tl, bl)
    e1 = float((ar[0, : S - 1].cpu().double() - ar_o).abs().max())
    print(f"  causal section max err {e1:.2e}", flush=True)
    assert e1 < SCORE_TOL
    if bl:
        e2 = float((diff[0].cpu().double() - diff_o).abs().max())
        print(f"  mask section max err {e2:.2e}", flush=True)
        assert e2 < SCORE_TOL
        want = O.tidar_loss(ar_o, diff_o, 1.0)
    else:
        want = float(-ar_o.mean())
    assert abs(float(loss[0]) - want) < 5e-3                   # a mean: the per-token errors average out
    assert float(ar_o.std()) > 0.05                            # the scores are not a constant
    eng.close()
