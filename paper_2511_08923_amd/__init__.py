"""Thin Python binding of libtidar.so (the gfx950 TiDAR decode-step library).

Argument marshalling only: every step of the path runs in the library's HIP
kernels.  PyTorch is used for device memory and streams, nothing else.  The
module-level functions carry the names of the C entry points in
include/tidar.h; `Engine` bundles the device buffers a decode loop needs
(packed weights, paged KV cache, workspace) and forwards to them.

Importing this package without a built library raises: there is no fallback.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional, Sequence

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libtidar.so")

TIDAR_F32, TIDAR_BF16 = 0, 1
PAGE = 16
STATUS = {0: "TIDAR_OK", 1: "TIDAR_EINVAL", 2: "TIDAR_ENOMEM", 3: "TIDAR_ECAPACITY", 4: "TIDAR_EDEVICE",
          5: "TIDAR_ESTATE"}

EXPORTS = ["tidar_create", "tidar_destroy", "tidar_strerror", "tidar_packed_weight_bytes", "tidar_pack_weight",
           "tidar_workspace_bytes", "tidar_prefill", "tidar_step", "tidar_ar_step", "tidar_hybrid_attention",
           "tidar_gemm_workspace_bytes", "tidar_gemm", "tidar_profile_enable", "tidar_profile_read",
           "tidar_profile_reset", "tidar_select_block_len", "tidar_set_prefill_chunk", "tidar_score_workspace_bytes",
           "tidar_score", "tidar_gemm_static"]
STATIC_SCRATCH_BYTES = 32 << 20


class TidarError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {STATUS.get(status, status)} ({_lib.tidar_strerror(status).decode()})")


class tidar_config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_q_heads", "n_kv_heads", "head_dim", "d_ff", "vocab",
                                         "tied_embeddings", "dtype", "page_size", "max_k", "max_batch",
                                         "mask_token_id")] + [("rope_base", C.c_float), ("rms_eps", C.c_float)]


class tidar_weights(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("lm_head", C.c_void_p), ("final_norm", C.c_void_p),
                ("attn_norm", C.POINTER(C.c_void_p)), ("wqkv", C.POINTER(C.c_void_p)), ("wo", C.POINTER(C.c_void_p)),
                ("ffn_norm", C.POINTER(C.c_void_p)), ("w_gate_up", C.POINTER(C.c_void_p)),
                ("w_down", C.POINTER(C.c_void_p))]


class tidar_kv_cache(C.Structure):
    _fields_ = [("k_pages", C.c_void_p), ("v_pages", C.c_void_p), ("page_table", C.c_void_p),
                ("pages_per_seq", C.c_int32), ("n_pages", C.c_int32)]


class tidar_mode(C.Structure):
    _fields_ = [("sample", C.c_int32), ("temperature", C.c_float), ("seed", C.c_uint64), ("beta", C.c_float)]


def _load() -> C.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()')")
    lib = C.CDLL(LIB_PATH)
    vp, i32, sz = C.c_void_p, C.c_int32, C.c_size_t
    lib.tidar_create.argtypes = [C.POINTER(tidar_config), C.POINTER(vp)]
    lib.tidar_create.restype = i32
    lib.tidar_destroy.argtypes = [vp]
    lib.tidar_destroy.restype = None
    lib.tidar_strerror.argtypes = [i32]
    lib.tidar_strerror.restype = C.c_char_p
    lib.tidar_packed_weight_bytes.argtypes = [i32, i32, i32]
    lib.tidar_packed_weight_bytes.restype = sz
    lib.tidar_pack_weight.argtypes = [i32, vp, i32, i32, vp, i32, i32, i32, vp]
    lib.tidar_pack_weight.restype = i32
    lib.tidar_workspace_bytes.argtypes = [vp, i32, i32, i32, C.POINTER(sz)]
    lib.tidar_workspace_bytes.restype = i32
    lib.tidar_prefill.argtypes = [vp, C.POINTER(tidar_weights), C.POINTER(tidar_kv_cache), i32, vp, i32,
                                  C.POINTER(i32), i32, C.POINTER(tidar_mode), vp, vp, vp, vp, sz, vp]
    lib.tidar_prefill.restype = i32
    lib.tidar_step.argtypes = [vp, C.POINTER(tidar_weights), C.POINTER(tidar_kv_cache), i32, vp, vp, i32,
                               C.POINTER(tidar_mode), vp, vp, vp, vp, i32, vp, sz, vp]
    lib.tidar_step.restype = i32
    lib.tidar_ar_step.argtypes = [vp, C.POINTER(tidar_weights), C.POINTER(tidar_kv_cache), i32, vp, vp,
                                  C.POINTER(tidar_mode), vp, vp, i32, vp, sz, vp]
    lib.tidar_ar_step.restype = i32
    lib.tidar_hybrid_attention.argtypes = [vp, C.POINTER(tidar_kv_cache), i32, i32, vp, vp, vp, vp, i32, i32, i32, i32,
                                           vp, i32, vp, sz, vp]
    lib.tidar_hybrid_attention.restype = i32
    lib.tidar_gemm_workspace_bytes.argtypes = [i32, i32, i32, i32]
    lib.tidar_gemm_workspace_bytes.restype = sz
    lib.tidar_gemm.argtypes = [vp, vp, vp, vp, i32, i32, i32, vp, sz, vp]
    lib.tidar_gemm.restype = i32
    lib.tidar_gemm_static.argtypes = [vp, vp, vp, vp, i32, i32, i32, vp]
    lib.tidar_gemm_static.restype = i32
    lib.tidar_profile_enable.argtypes = [vp, i32]
    lib.tidar_profile_enable.restype = i32
    lib.tidar_profile_read.argtypes = [vp, C.POINTER(C.c_char_p), C.POINTER(C.c_double), C.POINTER(C.c_int64), i32]
    lib.tidar_profile_read.restype = i32
    lib.tidar_profile_reset.argtypes = [vp]
    lib.tidar_profile_reset.restype = i32
    lib.tidar_select_block_len.argtypes = [vp, i32, i32, i32]
    lib.tidar_select_block_len.restype = i32
    lib.tidar_set_prefill_chunk.argtypes = [vp, i32]
    lib.tidar_set_prefill_chunk.restype = i32
    lib.tidar_score_workspace_bytes.argtypes = [vp, i32, i32, C.POINTER(sz)]
    lib.tidar_score_workspace_bytes.restype = i32
    lib.tidar_score.argtypes = [vp, C.POINTER(tidar_weights), C.POINTER(tidar_kv_cache), i32, vp, i32, C.POINTER(i32),
                                i32, C.c_float, vp, vp, vp, vp, sz, vp]
    lib.tidar_score.restype = i32
    return lib


_lib = _load()


def _check(status: int, where: str) -> None:
    if status != 0:
        raise TidarError(status, where)


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


# ---------------------------------------------------------------- functions named after the C entry points
def tidar_create(cfg: tidar_config) -> C.c_void_p:
    h = C.c_void_p()
    _check(_lib.tidar_create(C.byref(cfg), C.byref(h)), "tidar_create")
    return h


def tidar_destroy(ctx) -> None:
    _lib.tidar_destroy(ctx)


def tidar_strerror(status: int) -> str:
    return _lib.tidar_strerror(status).decode()


def tidar_packed_weight_bytes(dtype: int, rows: int, cols: int) -> int:
    return int(_lib.tidar_packed_weight_bytes(dtype, rows, cols))


def tidar_pack_weight(dtype: int, src: torch.Tensor, dst: torch.Tensor, dst_rows: int, tile_offset: int = 0,
                      tile_stride: int = 1) -> None:
    rows, cols = src.shape
    _check(_lib.tidar_pack_weight(dtype, src.data_ptr(), rows, cols, dst.data_ptr(), dst_rows, tile_offset,
                                  tile_stride, _stream()), "tidar_pack_weight")


def tidar_workspace_bytes(ctx, batch: int, k: int, max_prefix_len: int) -> int:
    n = C.c_size_t()
    _check(_lib.tidar_workspace_bytes(ctx, batch, k, max_prefix_len, C.byref(n)), "tidar_workspace_bytes")
    return int(n.value)


def tidar_prefill(ctx, w: tidar_weights, kv: tidar_kv_cache, batch: int, prompt: torch.Tensor, prompt_len: Sequence[int],
                  k: int, mode: tidar_mode, prefix_len: torch.Tensor, first_drafts: torch.Tensor,
                  logits_out: Optional[torch.Tensor], ws: torch.Tensor) -> None:
    plen = (C.c_int32 * batch)(*[int(x) for x in prompt_len])
    _check(_lib.tidar_prefill(ctx, C.byref(w), C.byref(kv), batch, prompt.data_ptr(), prompt.shape[1], plen, k,
                              C.byref(mode), prefix_len.data_ptr(), first_drafts.data_ptr(), _ptr(logits_out),
                              ws.data_ptr(), ws.numel() * ws.element_size(), _stream()), "tidar_prefill")


def tidar_step(ctx, w: tidar_weights, kv: tidar_kv_cache, batch: int, prefix_len: torch.Tensor, drafts: torch.Tensor,
               k: int, mode: tidar_mode, accepted_len: torch.Tensor, accepted_tokens: torch.Tensor,
               next_drafts: torch.Tensor, logits_out: Optional[torch.Tensor], max_prefix_len_hint: int,
               ws: torch.Tensor) -> None:
    _check(_lib.tidar_step(ctx, C.byref(w), C.byref(kv), batch, prefix_len.data_ptr(), drafts.data_ptr(), k,
                           C.byref(mode), accepted_len.data_ptr(), accepted_tokens.data_ptr(), next_drafts.data_ptr(),
                           _ptr(logits_out), max_prefix_len_hint, ws.data_ptr(), ws.numel() * ws.element_size(),
                           _stream()), "tidar_step")


def tidar_ar_step(ctx, w: tidar_weights, kv: tidar_kv_cache, batch: int, prefix_len: torch.Tensor,
                  token_in: torch.Tensor, mode: tidar_mode, token_out: torch.Tensor,
                  logits_out: Optional[torch.Tensor], max_prefix_len_hint: int, ws: torch.Tensor) -> None:
    _check(_lib.tidar_ar_step(ctx, C.byref(w), C.byref(kv), batch, prefix_len.data_ptr(), token_in.data_ptr(),
                              C.byref(mode), token_out.data_ptr(), _ptr(logits_out), max_prefix_len_hint,
                              ws.data_ptr(), ws.numel() * ws.element_size(), _stream()), "tidar_ar_step")


def tidar_hybrid_attention(ctx, kv: tidar_kv_cache, layer: int, batch: int, prefix_len: torch.Tensor, q: torch.Tensor,
                           k_new: torch.Tensor, v_new: torch.Tensor, n_causal: int, n_blocks: int, block_len: int,
                           cond0: int, out: torch.Tensor, max_prefix_len_hint: int, ws: torch.Tensor) -> None:
    _check(_lib.tidar_hybrid_attention(ctx, C.byref(kv), layer, batch, prefix_len.data_ptr(), q.data_ptr(),
                                       k_new.data_ptr(), v_new.data_ptr(), n_causal, n_blocks, block_len, cond0,
                                       out.data_ptr(), max_prefix_len_hint, ws.data_ptr(),
                                       ws.numel() * ws.element_size(), _stream()), "tidar_hybrid_attention")


def tidar_gemm_workspace_bytes(dtype: int, M: int, N: int, K: int) -> int:
    return int(_lib.tidar_gemm_workspace_bytes(dtype, M, N, K))


def tidar_gemm(ctx, a: torch.Tensor, w_packed: torch.Tensor, out: torch.Tensor, M: int, N: int, K: int,
               ws: torch.Tensor) -> None:
    _check(_lib.tidar_gemm(ctx, a.data_ptr(), w_packed.data_ptr(), out.data_ptr(), M, N, K, ws.data_ptr(),
                           ws.numel() * ws.element_size(), _stream()), "tidar_gemm")


def tidar_gemm_static(ctx, a: torch.Tensor, w_packed: torch.Tensor, out: torch.Tensor, M: int, N: int, K: int) -> None:
    _check(_lib.tidar_gemm_static(ctx, a.data_ptr(), w_packed.data_ptr(), out.data_ptr(), M, N, K, _stream()),
           "tidar_gemm_static")


def tidar_profile_enable(ctx, on: bool) -> None:
    _check(_lib.tidar_profile_enable(ctx, 1 if on else 0), "tidar_profile_enable")


def tidar_set_prefill_chunk(ctx, rows: int) -> None:
    _check(_lib.tidar_set_prefill_chunk(ctx, rows), "tidar_set_prefill_chunk")


def tidar_select_block_len(ctx, batch: int, k_cap: int = 0, row_budget: int = 0) -> int:
    return int(_lib.tidar_select_block_len(ctx, batch, k_cap, row_budget))


def tidar_score_workspace_bytes(ctx, max_len: int, block_len: int) -> int:
    n = C.c_size_t()
    _check(_lib.tidar_score_workspace_bytes(ctx, max_len, block_len, C.byref(n)), "tidar_score_workspace_bytes")
    return int(n.value)


def tidar_score(ctx, w: tidar_weights, kv: tidar_kv_cache, batch: int, tokens: torch.Tensor, length: Sequence[int],
                block_len: int, alpha: float, ar_logprob: torch.Tensor, diff_logprob: Optional[torch.Tensor],
                loss: Optional[torch.Tensor], ws: torch.Tensor) -> None:
    lens = (C.c_int32 * batch)(*[int(x) for x in length])
    _check(_lib.tidar_score(ctx, C.byref(w), C.byref(kv), batch, tokens.data_ptr(), tokens.shape[1], lens, block_len,
                            alpha, ar_logprob.data_ptr(), _ptr(diff_logprob), _ptr(loss), ws.data_ptr(),
                            ws.numel() * ws.element_size(), _stream()), "tidar_score")


def tidar_profile_reset(ctx) -> None:
    _check(_lib.tidar_profile_reset(ctx), "tidar_profile_reset")


def tidar_profile_read(ctx) -> Dict[str, Dict[str, float]]:
    cap = 32
    names = (C.c_char_p * cap)()
    ms = (C.c_double * cap)()
    cnt = (C.c_int64 * cap)()
    n = _lib.tidar_profile_read(ctx, names, ms, cnt, cap)
    return {names[i].decode(): {"ms": ms[i], "launches": int(cnt[i])} for i in range(min(n, cap))}


def make_config(shape, dtype: int, max_k: int = 16, max_batch: int = 1) -> tidar_config:
    """Fill a tidar_config from a tidar_inputs.ModelShape-like object."""
    return tidar_config(shape.n_layers, shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.d_ff,
                        shape.vocab, 1 if shape.tied_embeddings else 0, dtype, PAGE, max_k, max_batch,
                        shape.mask_token_id, shape.rope_base, shape.rms_eps)


def make_mode(sample: bool = False, temperature: float = 1.0, seed: int = 0, beta: float = 1.0) -> tidar_mode:
    return tidar_mode(1 if sample else 0, temperature, seed, beta)


# ---------------------------------------------------------------- device-buffer bundle
class Engine:
    """Owns the device buffers of one model instance and forwards to the C entry points."""

    def __init__(self, shape, weights: Dict[str, object], dtype: int = TIDAR_BF16, max_k: int = 16,
                 max_batch: int = 1, max_seq_len: int = 1024, n_pages: Optional[int] = None,
                 page_table: Optional[torch.Tensor] = None, device: str = "cuda:0", free_source: bool = False,
                 prefill_chunk: Optional[int] = None):
        if not torch.cuda.is_available():
            raise RuntimeError("the TiDAR HIP path needs a GPU; there is no CPU fallback")
        self.shape, self.dtype, self.device = shape, dtype, torch.device(device)
        self.tdtype = torch.bfloat16 if dtype == TIDAR_BF16 else torch.float32
        self.max_k, self.max_batch, self.max_seq_len = max_k, max_batch, max_seq_len
        self.cfg = make_config(shape, dtype, max_k, max_batch)
        self.ctx = tidar_create(self.cfg)
        if prefill_chunk is not None:
            tidar_set_prefill_chunk(self.ctx, prefill_chunk)
        self._keep: List[torch.Tensor] = []
        self._pack_weights(weights, free_source)
        self.pages_per_seq = (max_seq_len + PAGE - 1) // PAGE
        self.n_pages = n_pages if n_pages is not None else self.pages_per_seq * max_batch
        kv_shape = (shape.n_layers, self.n_pages, shape.n_kv_heads, PAGE * shape.head_dim)
        self.k_pages = torch.zeros(kv_shape, dtype=self.tdtype, device=self.device)
        self.v_pages = torch.zeros(kv_shape, dtype=self.tdtype, device=self.device)
        if page_table is None:
            page_table = torch.arange(max_batch * self.pages_per_seq, dtype=torch.int32).view(max_batch, -1)
        self.page_table = page_table.to(self.device, torch.int32).contiguous()
        assert self.page_table.shape == (max_batch, self.pages_per_seq)
        self.kv = tidar_kv_cache(self.k_pages.data_ptr(), self.v_pages.data_ptr(), self.page_table.data_ptr(),
                                 self.pages_per_seq, self.n_pages)
        self.ws_bytes = tidar_workspace_bytes(self.ctx, max_batch, max_k, max_seq_len)
        self.ws = torch.empty(self.ws_bytes, dtype=torch.uint8, device=self.device)
        self.prefix_len = torch.zeros(max_batch, dtype=torch.int32, device=self.device)

    def close(self) -> None:
        if self.ctx is not None:
            tidar_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- weights: plain [out, in] matrices in, library layout out
    def _dev(self, t: torch.Tensor) -> torch.Tensor:
        return t.to(self.device, self.tdtype).contiguous()

    def _packed(self, parts, total_rows: int, cols: int, free_source: bool) -> torch.Tensor:
        n = tidar_packed_weight_bytes(self.dtype, total_rows, cols)
        dst = torch.empty(n // (2 if self.dtype == TIDAR_BF16 else 4), dtype=self.tdtype, device=self.device)
        for src, off, stride in parts:
            s = self._dev(src)
            tidar_pack_weight(self.dtype, s, dst, total_rows, off, stride)
            torch.cuda.current_stream().synchronize()
            del s
        return dst

    def _pack_weights(self, w: Dict[str, object], free_source: bool) -> None:
        sh = self.shape
        self.embed = self._dev(w["embed"])
        head_src = w["lm_head"] if w["lm_head"] is not None else w["embed"]
        self.lm_head = self._packed([(head_src, 0, 1)], sh.vocab, sh.d_model, free_source)
        self.final_norm = self._dev(w["final_norm"])
        self.layers = []
        qt, kt = sh.q_dim // 16, sh.kv_dim // 16
        for lw in w["layers"]:
            self.layers.append({
                "attn_norm": self._dev(lw["attn_norm"]),
                "wqkv": self._packed([(lw["wq"], 0, 1), (lw["wk"], qt, 1), (lw["wv"], qt + kt, 1)],
                                     sh.q_dim + 2 * sh.kv_dim, sh.d_model, free_source),
                "wo": self._packed([(lw["wo"], 0, 1)], sh.d_model, sh.q_dim, free_source),
                "ffn_norm": self._dev(lw["ffn_norm"]),
                "w_gate_up": self._packed([(lw["w_gate"], 0, 2), (lw["w_up"], 1, 2)], 2 * sh.d_ff, sh.d_model,
                                          free_source),
                "w_down": self._packed([(lw["w_down"], 0, 1)], sh.d_model, sh.d_ff, free_source),
            })
            if free_source:
                lw.clear()
        n = sh.n_layers
        arr = lambda key: (C.c_void_p * n)(*[l[key].data_ptr() for l in self.layers])
        self._arrays = {key: arr(key) for key in ("attn_norm", "wqkv", "wo", "ffn_norm", "w_gate_up", "w_down")}
        cast = lambda a: C.cast(a, C.POINTER(C.c_void_p))
        self.w = tidar_weights(self.embed.data_ptr(), self.lm_head.data_ptr(), self.final_norm.data_ptr(),
                               cast(self._arrays["attn_norm"]), cast(self._arrays["wqkv"]), cast(self._arrays["wo"]),
                               cast(self._arrays["ffn_norm"]), cast(self._arrays["w_gate_up"]),
                               cast(self._arrays["w_down"]))

    def weight_bytes_per_step(self) -> int:
        """Bytes of weights one forward streams (every projection once; the embedding table is gathered)."""
        n = self.lm_head.numel() * self.lm_head.element_size()
        for l in self.layers:
            for key in ("wqkv", "wo", "w_gate_up", "w_down"):
                n += l[key].numel() * l[key].element_size()
        return n

    # -- calls
    def prefill(self, prompt: torch.Tensor, k: int, mode: Optional[tidar_mode] = None,
                want_logits: bool = False, prompt_len: Optional[List[int]] = None):
        """prompt: [batch, max_len] token ids; prompt_len: per-sequence lengths (default: all max_len)."""
        mode = mode or make_mode()
        batch, P = prompt.shape
        prompt_d = prompt.to(self.device, torch.int32).contiguous()
        first = torch.empty(batch, k, dtype=torch.int32, device=self.device)
        logits = (torch.empty(batch, 1 + k, self.shape.vocab, dtype=torch.float32, device=self.device)
                  if want_logits else None)
        tidar_prefill(self.ctx, self.w, self.kv, batch, prompt_d, list(prompt_len) if prompt_len else [P] * batch, k,
                      mode, self.prefix_len, first, logits, self.ws)
        return first, logits

    def step(self, drafts: torch.Tensor, k: int, hint: int, mode: Optional[tidar_mode] = None,
             want_logits: bool = False, out=None):
        mode = mode or make_mode()
        batch = drafts.shape[0]
        if out is None:
            out = (torch.empty(batch, dtype=torch.int32, device=self.device),
                   torch.empty(batch, k, dtype=torch.int32, device=self.device),
                   torch.empty(batch, k, dtype=torch.int32, device=self.device))
        a, acc, nxt = out
        logits = (torch.empty(batch, k * (k + 1), self.shape.vocab, dtype=torch.float32, device=self.device)
                  if want_logits else None)
        tidar_step(self.ctx, self.w, self.kv, batch, self.prefix_len, drafts, k, mode, a, acc, nxt, logits, hint,
                   self.ws)
        return a, acc, nxt, logits

    def ar_step(self, token_in: torch.Tensor, hint: int, mode: Optional[tidar_mode] = None,
                want_logits: bool = False, out: Optional[torch.Tensor] = None):
        mode = mode or make_mode()
        batch = token_in.shape[0]
        if out is None:
            out = torch.empty(batch, dtype=torch.int32, device=self.device)
        logits = (torch.empty(batch, self.shape.vocab, dtype=torch.float32, device=self.device)
                  if want_logits else None)
        tidar_ar_step(self.ctx, self.w, self.kv, batch, self.prefix_len, token_in, mode, out, logits, hint, self.ws)
        return out, logits

    def score(self, tokens: torch.Tensor, block_len: int = 0, alpha: float = 1.0,
              length: Optional[List[int]] = None):
        """tokens: [batch, max_len].  Returns (ar_logprob, diff_logprob or None, loss), device tensors."""
        batch, S = tokens.shape
        tok_d = tokens.to(self.device, torch.int32).contiguous()
        lens = list(length) if length else [S] * batch
        need = tidar_score_workspace_bytes(self.ctx, max(lens), block_len)
        ws = self.ws if need <= self.ws_bytes else torch.empty(need, dtype=torch.uint8, device=self.device)
        ar = torch.zeros(batch, S, dtype=torch.float32, device=self.device)
        diff = torch.zeros(batch, S, dtype=torch.float32, device=self.device) if block_len > 0 else None
        loss = torch.zeros(batch, dtype=torch.float32, device=self.device)
        tidar_score(self.ctx, self.w, self.kv, batch, tok_d, lens, block_len, alpha, ar, diff, loss, ws)
        return ar, diff, loss

    # -- cache views for tests: gather K ([L, n_kv, hd]) and V of one sequence and layer out of the pages
    def read_cache(self, layer: int, seq: int, length: int):
        sh = self.shape
        pos = torch.arange(length, device=self.device)
        pages = self.page_table[seq, (pos // PAGE).long()].long()
        slot = (pos % PAGE).long()
        kp = self.k_pages[layer].view(self.n_pages, sh.n_kv_heads, PAGE, sh.head_dim)
        vp = self.v_pages[layer].view(self.n_pages, sh.n_kv_heads, sh.head_dim, PAGE)
        return kp[pages, :, slot, :], vp[pages, :, :, slot]

    def write_cache(self, layer: int, seq: int, k: torch.Tensor, v: torch.Tensor) -> None:
        """Place K, V ([L, n_kv, hd]) of one sequence at positions 0..L-1 (test/benchmark set-up)."""
        sh = self.shape
        length = k.shape[0]
        pos = torch.arange(length, device=self.device)
        pages = self.page_table[seq, (pos // PAGE).long()].long()
        slot = (pos % PAGE).long()
        kp = self.k_pages[layer].view(self.n_pages, sh.n_kv_heads, PAGE, sh.head_dim)
        vp = self.v_pages[layer].view(self.n_pages, sh.n_kv_heads, sh.head_dim, PAGE)
        kp[pages, :, slot, :] = k.to(self.device, self.tdtype)
        vp[pages, :, :, slot] = v.to(self.device, self.tdtype)
