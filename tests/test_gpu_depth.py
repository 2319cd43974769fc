"""The paper's two model sizes at FULL depth (Section 4.1 Setup: 1.5B- and 8B-class backbones): 28 and 36 layers,
block length 16, through the C ABI.

Two kinds of check per size:
  * against the oracle, teacher-forced: prefill and decode steps started from the oracle's state (1.5B shape), decode
    steps on a synthetic cache of 4096 tokens (8B shape), all logits and every step output;
  * on the device alone, the plain definition the method must reach (Section 3.2: the causal rows are an
    autoregressive model, accepted tokens are exactly what one-token decoding would have produced): the one-token
    step generates a continuation, then TiDAR steps are fed drafts taken from it that are right up to a planned
    length and wrong after it; every step must accept exactly the planned length and propose the continuation's
    next token.

Tolerance at depth.  With N(0, 0.02) weights the logits have standard deviation 0.78 (1.5B shape) and 1.28 (8B
shape); every bf16 rounding point turns an fp32-level difference into one-ulp flips, and after 28 or 36 layers two
correct implementations are a few bf16 ulps of the residual stream apart: the oracle with fp32 accumulation differs
from the same oracle with fp64 accumulation (identical rounding points) by max 0.08 / rms 0.011 (1.5B shape) and
max 0.15 / rms 0.024 (8B shape).  The stated 2e-2 cannot hold there for any implementation; these tests measure
that floor in the run and allow 1.5x of it (max and rms), which the device meets with the same margin the two
oracles have between themselves.
"""
import numpy as np
import pytest
import torch

import tidar_inputs as TI
from oracle import tidar_oracle as O
from gpu_util import StepParity, load_oracle_state_into_engine, mismatch_rows, step_outputs_match_within_margin

pytestmark = pytest.mark.gpu
K = 16


@pytest.fixture(scope="module")
def T():
    import paper_2511_08923_amd as T
    assert torch.cuda.is_available()
    return T


class Depth:
    """One full-depth model: the same bf16 bytes on the device (packed by the engine) and on the host (oracle)."""

    def __init__(self, T, shape, seed, max_seq_len):
        self.shape = shape
        w = TI.make_weights(shape, seed=seed, dtype=torch.bfloat16, device="cuda")
        self.w_cpu = TI.weights_to(w, device="cpu")
        self.eng = T.Engine(shape, w, dtype=T.TIDAR_BF16, max_k=K, max_batch=1, max_seq_len=max_seq_len,
                            free_source=True)
        del w
        torch.cuda.empty_cache()

    def oracle(self, dtype):
        return O.OracleModel(self.shape, self.w_cpu, dtype=dtype, bf16_faithful=True)

    def close(self):
        self.eng.close()


@pytest.fixture(scope="module")
def m15(T):
    d = Depth(T, TI.SHAPE_1P5B, seed=3, max_seq_len=512 + 512 + 4 * K)
    yield d
    d.close()


@pytest.fixture(scope="module")
def m8(T):
    d = Depth(T, TI.SHAPE_8B, seed=4, max_seq_len=4096 + 1024 + 4 * K)
    yield d
    d.close()


def copy_state(st, dtype=None):
    cv = (lambda t: t.clone()) if dtype is None else (lambda t: t.to(dtype))
    return O.State([cv(t) for t in st.k], [cv(t) for t in st.v], st.L, st.seq_id)


def dev_out(eng, a, acc, nxt):
    return int(a[0]), acc[0].tolist(), nxt[0].tolist(), int(eng.prefix_len[0])


def measured_floor(model64, model32, st, drafts, mode=O.Mode()):
    """Distance between the two oracles on one step from the same state (neither state is advanced)."""
    lg64 = model64.tidar_step(copy_state(st), drafts, mode)[3]
    lg32 = model32.tidar_step(copy_state(st, torch.float32), drafts, mode)[3].double()
    d = (lg32 - lg64).abs()
    return float(d.max()), float(d.pow(2).mean().sqrt())


# ----------------------------------------------------------------------------- 1.5B shape, 28 layers (config 3)
def test_1p5b_full_depth_prefill_and_16_steps_vs_oracle(T, m15, progress):
    """Oracle prefill of a 512-token prompt and 16 teacher-forced decode steps at 28 layers."""
    eng, sh = m15.eng, m15.shape
    model = m15.oracle(torch.float64)
    P = 512
    prompt = TI.make_prompt(sh, P, seed=33)
    st = model.new_state(P + 17 * K)
    d_o, lg_o = model.prefill(st, [int(t) for t in prompt[0]], K)
    progress(f"  1.5b-shape/28L: oracle prefill done")
    floor_max, floor_rms = measured_floor(model, m15.oracle(torch.float32), st, d_o)
    tol, rms_tol = max(2e-2, 1.5 * floor_max), max(5e-3, 1.5 * floor_rms)
    first, lg = eng.prefill(prompt, K, want_logits=True)
    torch.cuda.synchronize()
    err = float((lg[0].cpu().double() - lg_o).abs().max())
    rows, bad = mismatch_rows(lg[0].cpu().argmax(-1), lg_o, err)
    progress(f"  1.5b-shape/28L prefill: max logit err {err:.3e} (floor {floor_max:.3e}), near-tie rows {len(rows)}")
    assert err < tol and bad == 0 and int(eng.prefix_len[0]) == P
    for i in range(K):
        if (0 if i == 0 else 1 + i) not in rows:
            assert int(first[0, i]) == d_o[i]
    par = StepParity("1.5b-shape 28 layers")
    for step in range(16):
        load_oracle_state_into_engine(eng, st)
        L = st.L
        drafts = list(d_o)
        if step % 4 == 1:                  # now and then: drafts the oracle accepts up to length 3 (a causal row's
            for i in range(1, 3):          # choice depends on the drafts before it, hence one forward per draft)
                plg = model.tidar_step(copy_state(st), drafts)[3]
                drafts[i] = int(plg[i - 1].argmax())
        a_o, acc_o, nxt_o, lg_o = model.tidar_step(st, drafts)
        a, acc, nxt, lg = eng.step(torch.tensor([drafts], dtype=torch.int32, device="cuda"), K, hint=L,
                                   want_logits=True)
        torch.cuda.synchronize()
        err, rms, rows = par.check(K, lg[0].cpu(), dev_out(eng, a, acc, nxt), lg_o, (a_o, acc_o, nxt_o, st.L), tol,
                                   rms_tol=rms_tol)
        progress(f"  1.5b-shape/28L step {step}: a={a_o} max err {err:.3e} rms {rms:.3e} near-tie rows {len(rows)}")
        d_o = nxt_o
    progress(f"  1.5b-shape/28L: floor max {floor_max:.3e} rms {floor_rms:.3e}; exactness asserted on "
             f"{par.exact} of {par.steps} steps; near-tie rows {par.near_ties}")
    par.report(min_exact=4)


def device_stream_check(T, eng, sh, P, n_tokens, mode, omode, margin_tol, progress, name):
    """Check 3 on the device alone at full depth.  Returns (steps, flips).

    The wide-GEMM step and the one-token step group their sums differently, so at 28-36 layers with random-init
    weights (decision margins of 0.15-0.2 on average against a bf16 noise of 0.01-0.02 rms per logit) a few percent
    of all token decisions are near ties that the two read differently.  Such a decision is excused only below twice
    the noise bound of the depth, every one is counted, and their share of all decisions is bounded."""
    prompt = TI.make_prompt(sh, P, seed=5)
    first, _ = eng.prefill(prompt, K, mode)
    torch.cuda.synchronize()
    # the reference continuation by one-token steps, with the decision margin of every token
    stream = [int(first[0, 0])]
    margins = [float("inf")]
    tok = first[:, 0].contiguous()
    hint = P + n_tokens + 2 * K
    for i in range(n_tokens + K):
        tok, lg = eng.ar_step(tok, hint=hint, mode=mode, want_logits=True)
        sc = lg[0]
        if omode.sample:
            g = torch.from_numpy(O.gumbel_noise(omode.seed, 0, P + i + 1, sh.vocab)).to(sc.device, torch.float32)
            sc = sc / omode.temperature + g
        top = sc.topk(2).values
        margins.append(float(top[0] - top[1]))
        stream.append(int(tok[0]))
        if i % 256 == 255:
            progress(f"  {name}: one-token reference at {i + 1} tokens")
    # TiDAR steps over the same cache positions: drafts from the reference, right up to a planned length
    rng = np.random.default_rng(12)
    pos, steps, flips, worst, decisions = 0, 0, 0, 0.0, 0
    while pos < n_tokens:
        want = int(rng.integers(1, K + 1))
        good = stream[pos:pos + K]
        drafts = good[:want] + [(t + 1) % (sh.vocab - 1) for t in good[want:]]
        eng.prefix_len[:1].fill_(P + pos)
        a, acc, nxt, _ = eng.step(torch.tensor([drafts], dtype=torch.int32, device="cuda"), K, hint=hint, mode=mode)
        a = int(a[0])
        ok = a == want and int(nxt[0, 0]) == stream[pos + want]
        if not ok:
            # the wide-GEMM step and the one-token step group their sums differently: they may disagree on a token
            # only where the reference's own decision margin is within the bf16 noise of this depth
            at = pos + min(a, want)
            assert a <= want, (name, pos, a, want)
            assert margins[at] < 2 * margin_tol, (name, pos, a, want, margins[at])
            flips += 1
            worst = max(worst, margins[at])
        else:
            assert acc[0, :a].tolist() == good[:a]
        pos += want
        steps += 1
        decisions += min(a, want) + 1
        if steps % 64 == 0:
            progress(f"  {name}: {steps} TiDAR steps, {pos} tokens, {flips} near-tie flips")
    progress(f"  {name}: {steps} TiDAR steps over {pos} tokens against the one-token stream: {decisions - flips} of "
             f"{decisions} token decisions identical, {flips} near ties (largest excused margin {worst:.3e}, allowed "
             f"below {2 * margin_tol:.3e})")
    assert flips <= max(2, int(0.08 * decisions)), (name, flips, decisions)
    return steps, flips


def test_1p5b_full_depth_tidar_stream_equals_one_token_stream_on_device(T, m15, progress):
    device_stream_check(T, m15.eng, m15.shape, 512, 512, T.make_mode(), O.Mode(), 0.06, progress, "1.5b-shape/28L greedy")


# ----------------------------------------------------------------------------- 8B shape, 36 layers (config 4)
def test_8b_full_depth_steps_vs_oracle_greedy_and_sampled(T, m8, progress):
    """36 layers, a synthetic cache of 4096 tokens (a 4096-token oracle prefill at this size costs minutes; the
    prefill is compared at depth on the 1.5B shape), two teacher-forced steps: all 272 x 151936 logits against the
    fp64 oracle, greedy outputs and temperature-1 sampled outputs (same logits, two verifications)."""
    eng, sh = m8.eng, m8.shape
    L = 4096
    model = m8.oracle(torch.float64)
    progress("  8b-shape/36L: fp64 oracle built")
    st = model.new_state(L + 3 * K)
    for l in range(sh.n_layers):
        st.k[l][:L] = TI.make_normal((L, sh.n_kv_heads, sh.head_dim), 500 + l, torch.bfloat16).double()
        st.v[l][:L] = TI.make_normal((L, sh.n_kv_heads, sh.head_dim), 600 + l, torch.bfloat16).double()
    st.L = L
    load_oracle_state_into_engine(eng, st)
    drafts = [int(t) for t in TI.make_drafts(sh, K, seed=9)[0]]
    m32 = m8.oracle(torch.float32)
    floor_max, floor_rms = measured_floor(model, m32, st, drafts)
    del m32
    progress(f"  8b-shape/36L: oracle fp32 vs fp64 on this step: max {floor_max:.3e} rms {floor_rms:.3e}")
    tol, rms_tol = max(2e-2, 1.5 * floor_max), max(5e-3, 1.5 * floor_rms)
    smode, gsmode = O.Mode(sample=True, temperature=1.0, seed=77), T.make_mode(sample=True, temperature=1.0, seed=77)
    par, par_s = StepParity("8b-shape 36 layers greedy"), StepParity("8b-shape 36 layers sampled")
    for step in range(2):
        pre = copy_state(st)
        a_s, acc_s, nxt_s, _ = model.tidar_step(copy_state(st), drafts, smode)
        a_o, acc_o, nxt_o, lg_o = model.tidar_step(st, drafts)
        progress(f"  8b-shape/36L: oracle step {step} done (a = {a_o}, sampled a = {a_s})")
        dd = torch.tensor([drafts], dtype=torch.int32, device="cuda")
        a, acc, nxt, lg = eng.step(dd, K, hint=L + 2 * K, want_logits=True)
        torch.cuda.synchronize()
        lg_dev = lg[0].cpu()
        del lg
        err, rms, rows = par.check(K, lg_dev, dev_out(eng, a, acc, nxt), lg_o, (a_o, acc_o, nxt_o, st.L), tol,
                                   rms_tol=rms_tol)
        progress(f"  8b-shape/36L step {step}: max err {err:.3e} rms {rms:.3e} near-tie rows {len(rows)}")
        # the sampled verification of the same step (fused path, no logits): surfaced tokens against the oracle's
        # perturbed scores
        eng.prefix_len[:1].fill_(pre.L)
        a2, acc2, nxt2, _ = eng.step(dd, K, hint=L + 2 * K, mode=gsmode)
        torch.cuda.synchronize()
        def scores(r):
            sc = lg_o[r]
            return sc + torch.from_numpy(O.gumbel_noise(77, 0, pre.L + r + 1, sh.vocab)) if r < K else sc

        par_s.steps += 1
        par_s.exact += step_outputs_match_within_margin(K, drafts, dev_out(eng, a2, acc2, nxt2),
                                                        (a_s, acc_s, nxt_s, pre.L + a_s), scores, err)
        eng.prefix_len[:1].fill_(st.L)
        drafts = list(nxt_o)               # next step: from the oracle's state and its next drafts
        load_oracle_state_into_engine(eng, st)
    progress(f"  8b-shape/36L: greedy exactness asserted on {par.exact} of {par.steps} steps, sampled outputs exactly "
             f"equal on {par_s.exact} of {par_s.steps}")
    par.report(min_exact=0)


def test_8b_full_depth_tidar_stream_equals_one_token_stream_on_device_greedy(T, m8, progress):
    device_stream_check(T, m8.eng, m8.shape, 4096, 1024, T.make_mode(), O.Mode(), 0.12, progress, "8b-shape/36L greedy")


def test_8b_full_depth_tidar_stream_equals_one_token_stream_on_device_sampled(T, m8, progress):
    device_stream_check(T, m8.eng, m8.shape, 4096, 1024, T.make_mode(sample=True, temperature=1.0, seed=321),
                        O.Mode(sample=True, temperature=1.0, seed=321), 0.12, progress, "8b-shape/36L T=1")


def test_8b_full_depth_two_sequences_of_8192_tokens_vs_oracle(T, progress):
    """The sweep's shape at full depth (config 5: 8192-token contexts, several sequences per step): two sequences
    with caches of 8192 and 8000 tokens, k = 16, i.e. 544 rows per step - the many-row GEMM class (256 x 256
    workgroup tiles, three row passes) and a batched attention launch at the real model dimensions - against the
    fp32 oracle run for each sequence alone.  Tolerance: the 36-layer floor of this file's header."""
    sh = TI.SHAPE_8B
    lens = [8192, 8000]
    w = TI.make_weights(sh, seed=4, dtype=torch.bfloat16, device="cuda")
    w_cpu = TI.weights_to(w, device="cpu")
    eng = T.Engine(sh, w, dtype=T.TIDAR_BF16, max_k=K, max_batch=2, max_seq_len=8192 + 4 * K, free_source=True)
    del w
    torch.cuda.empty_cache()
    model = O.OracleModel(sh, w_cpu, dtype=torch.float32, bf16_faithful=True)
    del w_cpu
    progress("  8b-shape/36L x2: fp32 oracle built")
    drafts = [[int(t) for t in TI.make_drafts(sh, K, seed=19 + b)[0]] for b in range(2)]
    want = []
    for b, L in enumerate(lens):
        st = model.new_state(L + 2 * K, seq_id=b)
        for l in range(sh.n_layers):
            st.k[l][:L] = TI.make_normal((L, sh.n_kv_heads, sh.head_dim), 700 + 40 * b + l, torch.bfloat16).float()
            st.v[l][:L] = TI.make_normal((L, sh.n_kv_heads, sh.head_dim), 800 + 40 * b + l, torch.bfloat16).float()
        st.L = L
        load_oracle_state_into_engine(eng, st, seq=b)
        want.append(model.tidar_step(st, drafts[b]) + (st.L,))
        progress(f"  8b-shape/36L x2: oracle step of sequence {b} done (a = {want[-1][0]})")
        del st
    a, acc, nxt, lg = eng.step(torch.tensor(drafts, dtype=torch.int32, device="cuda"), K, hint=max(lens),
                               want_logits=True)
    torch.cuda.synchronize()
    par = StepParity("8b-shape 36 layers, 2 sequences")
    for b in range(2):
        a_o, acc_o, nxt_o, lg_o, L_new = want[b]
        got = (int(a[b]), acc[b].tolist(), nxt[b].tolist(), int(eng.prefix_len[b]))
        err, rms, rows = par.check(K, lg[b].cpu(), got, lg_o.double(), (a_o, acc_o, nxt_o, L_new), 1.5 * 0.15,
                                   rms_tol=1.5 * 0.024)
        progress(f"  8b-shape/36L x2 sequence {b}: max err {err:.3e} rms {rms:.3e} near-tie rows {len(rows)}")
    par.report(min_exact=0)
    eng.close()
