"""CPU oracle for the TiDAR single-forward decode step.  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import
this module; the product path never does, and this module never imports the
HIP path.  Everything here is plain PyTorch CPU tensor code (fp64 by default),
written to be checked against the paper by eye: dense attention with an
explicitly materialised boolean mask, no tiling, no fusion, no caching tricks.

What the paper fixes, and where:
  * the three-section step (cached prefix; tokens drafted last step, encoded
    causally; mask tokens pre-drafting the next step, bidirectional within a
    block) ......................... Section 1 and Section 3.2, Figure 2 caption
  * the step's query length k*(1+k) ............. Section 3.3, footnote on q_len
  * verification by exact match against the token taken from the causal
    (autoregressive) logits, accept the longest matching prefix ... Section 3.2
    and Section 4.3.3 (the argmax-then-compare sentence)
  * no label shift for mask rows, label shift for causal rows; the causal row
    of draft j and the first slot of block j predict the same position
    ............................................... Section 3.1 and Section 4.3.3
  * exact KV cache: K/V of causally encoded tokens are stored, rejected ones
    evicted, nothing is ever recomputed ........................... Section 3.3
  * prefill: prompt causal plus one bidirectional block of masks .. Section 3.2
    and Appendix B
  * the training-time layout: the text followed by as many mask tokens, the
    text attended causally, every block of masks bidirectionally together with
    the text before the block; causal labels shifted by one, mask labels in
    place; the two cross-entropy sums and their weighting
    ....................... Section 3.1 (objective), Figure 3 (left) caption
  * likelihood of a text = the causal section alone, as for any AR model
    ............................................................ Section 4.2.2

Readings taken where the paper is silent (figures are not available):
  A. the first causal token c_1 is already final (it is the token sampled from
     the causal logits in the previous step); c_2..c_k are drafts; acceptance
     length a is in [1, k] and block j is the pre-draft for outcome a == j.
  B. position ids: pos(c_i) = L+i-1, pos(blk_j[s]) = L+j+s-1 (1-based i, j, s).
  C. "rejection sampling" is the exact-match test; sampling uses Gumbel-max
     noise keyed by the predicted absolute position, so that one-token AR
     decoding and TiDAR decoding consume the same noise.
  D. drafts are the argmax of the diffusion logits in both modes.
  E. beta = 1 (verify with the causal logits) unless a mix is requested.
  F. argmax ties go to the lowest token id.
  J. RMSNorm eps 1e-6, RoPE pairs dimension i with i + head_dim/2, no biases.
  N. the objective's two sums are printed with the same index range
     i = 1..S-1: the causal sum pairs x_i with its successor (S-1 targets,
     x_2..x_S); the mask sum is read literally as the tokens x_1..x_{S-1}
     (the last position is left out, both sums have S-1 terms).  The per-token
     log-probabilities are returned for all S mask positions, so another
     reading is one slice away.
  K. bf16-faithful mode rounds to bf16 at: normalised activations entering a
     GEMM, Q and K after RoPE, V, softmax numerators, attention output, the
     SwiGLU product; weights are bf16 values; the residual stream and all
     accumulation stay wide.  The softmax numerator is rounded as
     2^(s*log2(e) - ceil(max_row s*log2(e))): measured against a power-of-two
     reference the rounded mantissa does not depend on which reference an
     implementation happens to use, so any tiling order rounds the same way;
     the denominator sums the rounded numerators.

Parity status: every function below is pinned by tests/test_oracle_*.py
(worked-example mask, closed-form counts, brute-force loops, an independent
library transformer, AR-equivalence, cache equality; the beta-mix of
Section 4.3.3 against a verifier assembled from separate prefill-style
forwards, one per draft count, which never touches the step's row helpers).  The *values* of the
diffusion-row logits have no pin beyond those structural ones: no trained
weights exist here, so for them the status is "parity unpinned".
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np
import torch

# --------------------------------------------------------------------------
# Row layout, mask and positions of one decode step (Section 3.2, Section 3.3)
# --------------------------------------------------------------------------


def q_len(k: int) -> int:
    """Rows the step sends through the model: k causal + k blocks of k masks (Section 3.3 footnote)."""
    return k * (1 + k)


def row_of_c(i: int) -> int:
    """0-based row of causal token c_i, i in 1..k."""
    return i - 1


def row_of_blk(k: int, j: int, s: int) -> int:
    """0-based row of slot s of mask block j, both in 1..k."""
    return k + (j - 1) * k + (s - 1)


def decode_mask(k: int, L: int) -> torch.Tensor:
    """Boolean [R, L+R] attend-matrix of one decode step (Figure 2 / Figure 3 captions, Section 3.2).

    Columns 0..L-1 are the cached prefix, columns L.. are the step's own rows
    in the order c_1..c_k, blk_1[1..k], ..., blk_k[1..k].
    """
    R = q_len(k)
    M = torch.zeros(R, L + R, dtype=torch.bool)
    M[:, :L] = True                                     # every row sees the whole prefix
    for i in range(1, k + 1):                           # clean tokens: causal
        for ip in range(1, i + 1):
            M[row_of_c(i), L + row_of_c(ip)] = True
    for j in range(1, k + 1):                           # block j: pre-draft for "j accepted"
        for s in range(1, k + 1):
            r = row_of_blk(k, j, s)
            for ip in range(1, j + 1):                  # the drafts it is conditioned on
                M[r, L + row_of_c(ip)] = True
            for sp in range(1, k + 1):                  # bidirectional inside its own block
                M[r, L + row_of_blk(k, j, sp)] = True
    return M


def decode_positions(k: int, L: int) -> torch.Tensor:
    """Position id of every row (reading B): a mask sits where the token it predicts will sit."""
    pos = torch.zeros(q_len(k), dtype=torch.int64)
    for i in range(1, k + 1):
        pos[row_of_c(i)] = L + i - 1
    for j in range(1, k + 1):
        for s in range(1, k + 1):
            pos[row_of_blk(k, j, s)] = L + j + s - 1
    return pos


def prefill_mask(P: int, k: int) -> torch.Tensor:
    """Boolean [P+k, P+k]: prompt causal, one block of k masks that sees the prompt and itself (Appendix B)."""
    M = torch.zeros(P + k, P + k, dtype=torch.bool)
    for t in range(P):
        M[t, : t + 1] = True
    M[P:, :P] = True
    M[P:, P:] = True
    return M


def prefill_positions(P: int, k: int) -> torch.Tensor:
    return torch.arange(P + k, dtype=torch.int64)


def causal_mask(n_new: int, L: int) -> torch.Tensor:
    """Plain causal attend-matrix for n_new rows appended after L cached tokens."""
    M = torch.zeros(n_new, L + n_new, dtype=torch.bool)
    for t in range(n_new):
        M[t, : L + t + 1] = True
    return M


# --------------------------------------------------------------------------
# Training-time layout (Section 3.1, Figure 3 left caption): rows and columns
# are the S text tokens followed by S mask tokens; mask i stands in for token i
# and belongs to block i // bl (the last block is short when bl does not
# divide S).
# --------------------------------------------------------------------------


def training_mask(S: int, bl: int) -> torch.Tensor:
    """Boolean [2S, 2S] attend-matrix of the doubled training sequence."""
    M = torch.zeros(2 * S, 2 * S, dtype=torch.bool)
    for t in range(S):                                  # text: causal, never sees a mask
        M[t, : t + 1] = True
    for i in range(S):
        j = i // bl
        M[S + i, : j * bl] = True                       # the text before its block
        for ip in range(j * bl, min((j + 1) * bl, S)):  # its own block, both directions
            M[S + i, S + ip] = True
    return M


def training_positions(S: int) -> torch.Tensor:
    """A mask keeps the position of the token it stands in for (labels are not shifted, Section 3.1)."""
    return torch.cat([torch.arange(S, dtype=torch.int64), torch.arange(S, dtype=torch.int64)])


def tidar_loss(ar_logprob: torch.Tensor, diff_logprob: torch.Tensor, alpha: float) -> float:
    """Section 3.1 objective from per-token log-probabilities (reading N).

    ar_logprob [S-1]: log p(x_{i+1} | x_{<=i}) from the causal section; diff_logprob [S]: log p(x_i | text
    before its block, masks) from the mask section.  Both sums have S-1 terms and are divided by S-1; the
    causal one is weighted by alpha, the total by 1/(1+alpha).
    """
    S = diff_logprob.shape[0]
    assert ar_logprob.shape[0] == S - 1 and S >= 2
    l_ar = -float(ar_logprob.sum()) / (S - 1)
    l_diff = -float(diff_logprob[: S - 1].sum()) / (S - 1)
    return (alpha * l_ar + l_diff) / (1.0 + alpha)


# --------------------------------------------------------------------------
# The backbone F (a standard pre-norm decoder, Section 4.1 "Setup")
# --------------------------------------------------------------------------


def round_bf16(x: torch.Tensor) -> torch.Tensor:
    return x.to(torch.bfloat16).to(x.dtype)


def rmsnorm(x: torch.Tensor, gain: torch.Tensor, eps: float) -> torch.Tensor:
    ms = (x * x).mean(dim=-1, keepdim=True)
    return x * torch.rsqrt(ms + eps) * gain


def rope(x: torch.Tensor, positions: torch.Tensor, base: float) -> torch.Tensor:
    """Rotary embedding on [rows, heads, head_dim]; dimension i rotates with i + head_dim/2."""
    hd = x.shape[-1]
    half = hd // 2
    inv_freq = base ** (-torch.arange(half, dtype=torch.float64) * 2.0 / hd)
    ang = positions.to(torch.float64)[:, None] * inv_freq[None, :]            # [rows, half]
    cos = torch.cos(ang).to(x.dtype)[:, None, :]
    sin = torch.sin(ang).to(x.dtype)[:, None, :]
    x1, x2 = x[..., :half], x[..., half:]
    return torch.cat([x1 * cos - x2 * sin, x2 * cos + x1 * sin], dim=-1)


def silu(x: torch.Tensor) -> torch.Tensor:
    return x / (1.0 + torch.exp(-x))


def attention_dense(q: torch.Tensor, keys: torch.Tensor, vals: torch.Tensor, mask: torch.Tensor,
                    round_p: bool = False) -> torch.Tensor:
    """softmax(q k^T / sqrt(hd) + M) v with M materialised from ``mask``.

    q [R, n_q, hd]; keys, vals [T, n_kv, hd]; mask bool [R, T]; query head h
    reads kv head h // (n_q // n_kv).  Returns [R, n_q, hd].
    """
    R, n_q, hd = q.shape
    n_kv = keys.shape[1]
    group = n_q // n_kv
    scale = 1.0 / math.sqrt(hd)
    out = torch.empty_like(q)
    neg_inf = torch.tensor(float("-inf"), dtype=q.dtype)
    for h in range(n_q):
        g = h // group
        s = (q[:, h, :] @ keys[:, g, :].T) * scale                             # [R, T]
        s = torch.where(mask, s, neg_inf)
        if round_p:                                                             # reading K
            s2 = s * math.log2(math.e)
            e = round_bf16(torch.exp2(s2 - torch.ceil(s2.max(dim=-1, keepdim=True).values)))
        else:
            e = torch.exp(s - s.max(dim=-1, keepdim=True).values)
        p = e / e.sum(dim=-1, keepdim=True)
        out[:, h, :] = p @ vals[:, g, :]
    return out


@dataclass
class Mode:
    sample: bool = False
    temperature: float = 1.0
    seed: int = 0
    beta: float = 1.0       # weight of the causal logits in verification (Section 4.3.3)


@dataclass
class State:
    """Exact KV cache of one sequence: K (post-RoPE) and V of the first L tokens, per layer."""
    k: List[torch.Tensor]
    v: List[torch.Tensor]
    L: int = 0
    seq_id: int = 0


class OracleModel:
    def __init__(self, shape, weights: Dict[str, object], dtype: torch.dtype = torch.float64,
                 bf16_faithful: bool = False):
        self.shape = shape
        self.dtype = dtype
        self.faithful = bf16_faithful

        def cv(t):
            return None if t is None else t.detach().to("cpu").to(dtype)

        self.w = {k: cv(v) for k, v in weights.items() if k != "layers"}
        self.w["layers"] = [{k: cv(v) for k, v in lw.items()} for lw in weights["layers"]]
        if self.w["lm_head"] is None:
            self.w["lm_head"] = self.w["embed"]         # tied embeddings

    def _rb(self, x: torch.Tensor) -> torch.Tensor:
        return round_bf16(x) if self.faithful else x

    def new_state(self, capacity: int, seq_id: int = 0) -> State:
        sh = self.shape
        mk = lambda: torch.zeros(capacity, sh.n_kv_heads, sh.head_dim, dtype=self.dtype)
        return State([mk() for _ in range(sh.n_layers)], [mk() for _ in range(sh.n_layers)], 0, seq_id)

    # ---- one forward over new rows against a cached prefix ----
    def forward(self, tokens: torch.Tensor, positions: torch.Tensor, mask: torch.Tensor,
                state: State, logits_rows: Optional[Sequence[int]] = None
                ) -> Tuple[torch.Tensor, List[torch.Tensor], List[torch.Tensor]]:
        """Returns (logits [rows, V], new K per layer [R, n_kv, hd], new V per layer)."""
        sh, w, L = self.shape, self.w, state.L
        R = tokens.shape[0]
        assert mask.shape == (R, L + R)
        x = w["embed"][tokens.long()]                                           # [R, d]
        new_k, new_v = [], []
        for l, lw in enumerate(w["layers"]):
            n1 = self._rb(rmsnorm(x, lw["attn_norm"], sh.rms_eps))
            q = (n1 @ lw["wq"].T).view(R, sh.n_q_heads, sh.head_dim)
            k = (n1 @ lw["wk"].T).view(R, sh.n_kv_heads, sh.head_dim)
            v = (n1 @ lw["wv"].T).view(R, sh.n_kv_heads, sh.head_dim)
            q = self._rb(rope(q, positions, sh.rope_base))
            k = self._rb(rope(k, positions, sh.rope_base))
            v = self._rb(v)
            new_k.append(k)
            new_v.append(v)
            keys = torch.cat([state.k[l][:L], k], dim=0)
            vals = torch.cat([state.v[l][:L], v], dim=0)
            o = self._rb(attention_dense(q, keys, vals, mask, round_p=self.faithful))
            h = x + o.reshape(R, sh.q_dim) @ lw["wo"].T
            n2 = self._rb(rmsnorm(h, lw["ffn_norm"], sh.rms_eps))
            f = self._rb(silu(n2 @ lw["w_gate"].T) * (n2 @ lw["w_up"].T))
            x = h + f @ lw["w_down"].T
        if logits_rows is not None:
            x = x[list(logits_rows)]
        xn = self._rb(rmsnorm(x, w["final_norm"], sh.rms_eps))
        logits = xn @ w["lm_head"].T
        return logits, new_k, new_v

    def _commit(self, state: State, new_k, new_v, rows: Sequence[int]) -> None:
        """Append K/V of the given new rows (in order) to the cache; L grows by len(rows)."""
        n = len(rows)
        for l in range(self.shape.n_layers):
            state.k[l][state.L: state.L + n] = new_k[l][list(rows)]
            state.v[l][state.L: state.L + n] = new_v[l][list(rows)]
        state.L += n

    # ---- choosing a token from a row of logits ----
    def choose(self, logits_row: torch.Tensor, pos_pred: int, mode: Mode, seq_id: int) -> int:
        if not mode.sample:
            return int(torch.argmax(logits_row))                                # first maximum = lowest id
        g = torch.from_numpy(gumbel_noise(mode.seed, seq_id, pos_pred, logits_row.shape[0])).to(logits_row.dtype)
        return int(torch.argmax(logits_row / mode.temperature + g))

    # ---- prefill (Section 3.2 first paragraph of the procedure, Appendix B) ----
    def prefill(self, state: State, prompt: Sequence[int], k: int, mode: Mode = Mode()
                ) -> Tuple[List[int], torch.Tensor]:
        assert state.L == 0
        P = len(prompt)
        sh = self.shape
        tokens = torch.tensor(list(prompt) + [sh.mask_token_id] * k, dtype=torch.int64)
        logits, nk, nv = self.forward(tokens, prefill_positions(P, k), prefill_mask(P, k), state,
                                      logits_rows=range(P - 1, P + k))
        self._commit(state, nk, nv, range(P))
        first = [self.choose(logits[0], P, mode, state.seq_id)]                 # causal logit of last prompt row
        for s in range(2, k + 1):                                               # mask slot s predicts position P+s-1
            first.append(int(torch.argmax(logits[s])))
        return first, logits

    # ---- the decode step ----
    def tidar_step(self, state: State, drafts: Sequence[int], mode: Mode = Mode()
                   ) -> Tuple[int, List[int], List[int], torch.Tensor]:
        """One TiDAR step.  Returns (a, accepted tokens, next drafts, logits [R, V])."""
        k, L, sh = len(drafts), state.L, self.shape
        c = list(drafts)
        tokens = torch.tensor(c + [sh.mask_token_id] * (k * k), dtype=torch.int64)
        # 1. one forward with the hybrid mask
        logits, nk, nv = self.forward(tokens, decode_positions(k, L), decode_mask(k, L), state)
        # 2. token from the causal logits at every draft row (label shift: row c_i judges position L+i)
        y_ar = []
        for i in range(1, k + 1):
            row = logits[row_of_c(i)]
            if mode.beta != 1.0:                                                # Section 4.3.3 mix
                row = mode.beta * row + (1.0 - mode.beta) * logits[row_of_blk(k, i, 1)]
            y_ar.append(self.choose(row, L + i, mode, state.seq_id))
        # 3. accept the longest matching prefix; c_1 is final by construction
        a = 1
        while a < k and c[a] == y_ar[a - 1]:
            a += 1
        # 4. commit K/V of c_1..c_a only
        self._commit(state, nk, nv, [row_of_c(i) for i in range(1, a + 1)])
        # 5. next drafts: the AR token at the first unverified position, then block a's slots 2..k
        nxt = [y_ar[a - 1]]
        for s in range(2, k + 1):
            nxt.append(int(torch.argmax(logits[row_of_blk(k, a, s)])))
        return a, c[:a], nxt, logits

    # ---- the plain definition: one-token causal decoding ----
    def ar_step(self, state: State, token: int, mode: Mode = Mode()) -> Tuple[int, torch.Tensor]:
        L = state.L
        logits, nk, nv = self.forward(torch.tensor([token], dtype=torch.int64),
                                      torch.tensor([L], dtype=torch.int64), causal_mask(1, L), state)
        self._commit(state, nk, nv, [0])
        return self.choose(logits[0], L + 1, mode, state.seq_id), logits

    def causal_prefill(self, state: State, prompt: Sequence[int], mode: Mode = Mode()) -> Tuple[int, torch.Tensor]:
        """Plain causal forward over a prompt; returns the first generated token and the last row's logits."""
        assert state.L == 0
        P = len(prompt)
        logits, nk, nv = self.forward(torch.tensor(list(prompt), dtype=torch.int64),
                                      torch.arange(P, dtype=torch.int64), causal_mask(P, 0), state,
                                      logits_rows=[P - 1])
        self._commit(state, nk, nv, range(P))
        return self.choose(logits[0], P, mode, state.seq_id), logits

    def ar_decode(self, prompt: Sequence[int], n_tokens: int, mode: Mode = Mode(), seq_id: int = 0) -> List[int]:
        state = self.new_state(len(prompt) + n_tokens + 1, seq_id)
        tok, _ = self.causal_prefill(state, prompt, mode)
        out = [tok]
        while len(out) < n_tokens:
            tok, _ = self.ar_step(state, tok, mode)
            out.append(tok)
        return out

    # ---- likelihood of a text in AR mode (Section 4.2.2) ----
    def score(self, tokens: Sequence[int]) -> torch.Tensor:
        """log p(x_{i+1} | x_0..x_i) for i = 0..S-2 under the pure causal mask: [S-1]."""
        S = len(tokens)
        state = self.new_state(S)
        t = torch.tensor(list(tokens), dtype=torch.int64)
        logits, _, _ = self.forward(t, torch.arange(S, dtype=torch.int64), causal_mask(S, 0), state)
        lp = torch.log_softmax(logits, dim=-1)
        return lp[torch.arange(S - 1), t[1:]]

    # ---- one forward over the doubled training sequence (Section 3.1) ----
    def training_forward(self, tokens: Sequence[int], bl: int) -> Tuple[torch.Tensor, torch.Tensor, torch.Tensor]:
        """Returns (causal log-probs [S-1], label shifted; mask log-probs [S], labels in place; logits [2S, V])."""
        S = len(tokens)
        state = self.new_state(1)
        t = torch.tensor(list(tokens), dtype=torch.int64)
        rows = torch.cat([t, torch.full((S,), self.shape.mask_token_id, dtype=torch.int64)])
        logits, _, _ = self.forward(rows, training_positions(S), training_mask(S, bl), state)
        lp = torch.log_softmax(logits, dim=-1)
        ar = lp[torch.arange(S - 1), t[1:]]
        diff = lp[S + torch.arange(S), t]
        return ar, diff, logits

    def tidar_decode(self, prompt: Sequence[int], n_tokens: int, k: int, mode: Mode = Mode(), seq_id: int = 0,
                     draft_override=None) -> Tuple[List[int], List[int]]:
        """Prefill then steps until n_tokens are out.  ``draft_override(step, drafts)`` may replace
        drafts[1:] (slot 0 must stay) to force acceptance patterns.  Returns (tokens, acceptance lengths)."""
        state = self.new_state(len(prompt) + n_tokens + k + 1, seq_id)
        drafts, _ = self.prefill(state, prompt, k, mode)
        out: List[int] = []
        acc: List[int] = []
        step = 0
        while len(out) < n_tokens:
            if draft_override is not None:
                drafts = [drafts[0]] + list(draft_override(step, drafts, state.L))[1:]
            a, accepted, drafts, _ = self.tidar_step(state, drafts, mode)
            out.extend(accepted)
            acc.append(a)
            step += 1
        return out[:n_tokens], acc


# --------------------------------------------------------------------------
# Position-keyed Gumbel noise (reading C).  A counter-based generator: the same
# integer recipe is implemented on the device side, nothing is shared.
# --------------------------------------------------------------------------

_M64 = (1 << 64) - 1


def hash_u24(seed: int, seq_id: int, pos: int, vocab: int) -> np.ndarray:
    """24 random bits per vocabulary entry, keyed by (seed, sequence, predicted absolute position, token id)."""
    key = (seed ^ ((0x9E3779B97F4A7C15 * (pos + 1)) & _M64) ^ ((0xC2B2AE3D27D4EB4F * (seq_id + 1)) & _M64)) & _M64
    with np.errstate(over="ignore"):
        v = np.arange(1, vocab + 1, dtype=np.uint64)
        z = np.uint64(key) + v * np.uint64(0xD6E8FEB86659FD93)
        z ^= z >> np.uint64(30)
        z *= np.uint64(0xBF58476D1CE4E5B9)
        z ^= z >> np.uint64(27)
        z *= np.uint64(0x94D049BB133111EB)
        z ^= z >> np.uint64(31)
    return (z >> np.uint64(40)).astype(np.uint32)


def gumbel_noise(seed: int, seq_id: int, pos: int, vocab: int) -> np.ndarray:
    """G = -ln(-ln u), u = (bits + 0.5) / 2^24 in (0, 1)."""
    u = (hash_u24(seed, seq_id, pos, vocab).astype(np.float64) + 0.5) / float(1 << 24)
    return -np.log(-np.log(u))
