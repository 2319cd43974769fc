"""Helpers shared by the GPU parity tests: set-up and comparison only, none of the method's arithmetic."""
import torch

import tidar_inputs as TI


def near_tie_mismatches(got_tokens, oracle_logits, tol):
    """Compare chosen tokens row by row with the oracle's argmax.  If every device logit is within `tol` of
    the oracle's, the device can only prefer another token when the oracle's margin between its top token and
    that token is below 2*tol; callers pass the *measured* maximum logit error as `tol`, so a mismatch on any
    wider margin is a real error.  Returns (n_mismatch, n_unexcused)."""
    rows, bad = mismatch_rows(got_tokens, oracle_logits, tol)
    return len(rows), bad


def mismatch_rows(got_tokens, oracle_logits, tol):
    """Rows whose device token differs from the oracle's argmax, and how many of them the near-tie rule does not
    excuse (oracle margin between the two candidates >= 2 * tol)."""
    want = oracle_logits.argmax(dim=-1)
    rows, n_bad = [], 0
    for r in range(oracle_logits.shape[0]):
        g, w = int(got_tokens[r]), int(want[r])
        if g != w:
            rows.append(r)
            if float(oracle_logits[r, w] - oracle_logits[r, g]) >= 2 * tol:
                n_bad += 1
    return rows, n_bad


def rows_that_decide_the_step(k, a_oracle):
    """Rows of the step (order c_0..c_{k-1}, blk_0[0..k), ..., as tidar.h lays out logits_out) whose chosen tokens
    the step's outputs depend on when the oracle accepts a_oracle tokens: causal rows 0..a-1 (they fix the
    acceptance length and the first next draft) and slots 1..k-1 of mask block a-1 (the other next drafts)."""
    return set(range(a_oracle)) | {k + (a_oracle - 1) * k + s for s in range(1, k)}


class StepParity:
    """Bookkeeping of one bf16 parity test: how many steps had token/acceptance exactness asserted, how many rows
    were near ties, the largest logit distances seen.  `check` applies the near-tie rule to one step:
      * every device logit within `tol` of the oracle's (the caller's tolerance), rms within tol / 4;
      * a device argmax may differ from the oracle's only where the oracle's margin between the two tokens is below
        twice the measured maximum error; the number of such rows is bounded;
      * unless one of those rows is a row the step's outputs depend on (rows_that_decide_the_step), acceptance
        length, accepted tokens, next drafts and the new prefix length must equal the oracle's exactly."""

    def __init__(self, name, max_near_tie_frac=0.125):
        self.name, self.frac = name, max_near_tie_frac
        self.steps = self.exact = self.near_ties = 0
        self.max_err = self.max_err_unrounded = 0.0

    def check(self, k, dev_logits, dev_out, oracle_logits, oracle_out, tol, rms_tol=None, unrounded_logits=None):
        a, acc, nxt, prefix = dev_out                 # python ints / lists
        a_o, acc_o, nxt_o, prefix_o = oracle_out
        lg = dev_logits.double()
        err = float((lg - oracle_logits).abs().max())
        rms = float((lg - oracle_logits).pow(2).mean().sqrt())
        assert err < tol, (self.name, err, tol)
        assert rms < (rms_tol if rms_tol is not None else tol / 4), (self.name, rms)
        rows, bad = mismatch_rows(lg.argmax(-1), oracle_logits, err)
        assert bad == 0, (self.name, rows, err)
        R = oracle_logits.shape[0]
        assert len(rows) <= max(2, int(self.frac * R)), (self.name, len(rows), R)
        self.steps += 1
        self.near_ties += len(rows)
        self.max_err = max(self.max_err, err)
        if unrounded_logits is not None:
            self.max_err_unrounded = max(self.max_err_unrounded, float((lg - unrounded_logits).abs().max()))
        if not (set(rows) & rows_that_decide_the_step(k, a_o)):
            assert a == a_o, (self.name, a, a_o)
            assert acc[:a_o] == acc_o and nxt == nxt_o and prefix == prefix_o, (self.name, acc, acc_o, nxt, nxt_o)
            self.exact += 1
        return err, rms, rows

    def report(self, min_exact=1):
        print(f"  [{self.name}] steps {self.steps}, exactness asserted on {self.exact}, near-tie rows {self.near_ties}, "
              f"max |logit - oracle(bf16 points)| {self.max_err:.3e}, max |logit - oracle(fp64, unrounded)| "
              f"{self.max_err_unrounded:.3e}", flush=True)
        assert self.exact >= min_exact, (self.name, self.exact, self.steps)


def step_outputs_match_within_margin(k, drafts, dev_out, oracle_out, scores, tol):
    """The step's outputs against the oracle's when the device's logits are not available (the fused vocabulary
    reduction writes none).  `scores(row)` gives the oracle's decision scores of a row (its logits; for the causal
    rows under sampling or a beta mix, the perturbed or mixed values).  Every device token that surfaces in the
    outputs must be the oracle's, or lose to it by less than 2 * tol in the oracle's own scores (near tie).
    Returns True when everything is exactly equal."""
    a, acc, nxt, prefix = dev_out
    a_o, acc_o, nxt_o, prefix_o = oracle_out

    def excused(row, tok_dev, tok_or):
        sc = scores(row)
        return float(sc[tok_or] - sc[tok_dev]) < 2 * tol

    assert 1 <= a <= k
    if a != a_o:
        row = min(a, a_o) - 1              # the causal row the two sides read differently
        if a < a_o:                        # the oracle's row chose drafts[a]; the device's chose nxt[0]
            assert excused(row, nxt[0], drafts[a]), ("acceptance", a, a_o)
        else:                              # the oracle's row chose nxt_o[0]; the device's chose drafts[a_o]
            assert excused(row, drafts[a_o], nxt_o[0]), ("acceptance", a, a_o)
        assert acc[:a] == list(drafts[:a])
        return False
    assert acc[:a] == acc_o and prefix == prefix_o
    exact = True
    rows = [a - 1] + [k + (a - 1) * k + s for s in range(1, k)]
    for i, row in enumerate(rows):
        if nxt[i] != nxt_o[i]:
            assert excused(row, nxt[i], nxt_o[i]), ("next draft", i, nxt[i], nxt_o[i])
            exact = False
    return exact


def load_oracle_state_into_engine(eng, st, seq=0):
    """Teacher forcing: copy the oracle's cache (first L positions) into the engine's pages, set prefix_len."""
    for l in range(eng.shape.n_layers):
        eng.write_cache(l, seq, st.k[l][:st.L], st.v[l][:st.L])
    eng.prefix_len[seq] = st.L
    torch.cuda.synchronize()
