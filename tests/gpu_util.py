"""Helpers shared by the GPU parity tests: set-up and comparison only, none of the method's arithmetic."""
import torch

import tidar_inputs as TI


def near_tie_mismatches(got_tokens, oracle_logits, tol):
    """Compare chosen tokens row by row with the oracle's argmax.  If every device logit is within `tol` of
    the oracle's, the device can only prefer another token when the oracle's margin between its top token and
    that token is below 2*tol; callers pass the *measured* maximum logit error as `tol`, so a mismatch on any
    wider margin is a real error.  Returns (n_mismatch, n_unexcused)."""
    want = oracle_logits.argmax(dim=-1)
    n_mis = n_bad = 0
    for r in range(oracle_logits.shape[0]):
        g, w = int(got_tokens[r]), int(want[r])
        if g != w:
            n_mis += 1
            if float(oracle_logits[r, w] - oracle_logits[r, g]) >= 2 * tol:
                n_bad += 1
    return n_mis, n_bad


def load_oracle_state_into_engine(eng, st, seq=0):
    """Teacher forcing: copy the oracle's cache (first L positions) into the engine's pages, set prefix_len."""
    for l in range(eng.shape.n_layers):
        eng.write_cache(l, seq, st.k[l][:st.L], st.v[l][:st.L])
    eng.prefix_len[seq] = st.L
    torch.cuda.synchronize()
