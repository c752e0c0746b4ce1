"""fp64 reference of the decoder-only transformer and vanilla greedy decoding.

TEST INFRASTRUCTURE (see the package docstring): plain PyTorch CPU ops in
float64, no blocking, no fusion, no reordering.

What it follows.  The paper names its models (Vicuna / LLaMA-2, Sec. 5.1 and
the appendix table "Model configurations") without restating the block; the
block below is that family's: pre-norm RMSNorm, rotary position embedding on
q and k, causal multi-head (or grouped-query) attention, SwiGLU MLP, untied
embedding and LM head.  The early-exit "norm head" is an RMSNorm followed by a
linear layer of the LM head's shape (Sec. 3.1).  The target of the whole
method is vanilla greedy autoregressive decoding of the full model: every
token is the argmax of the full model's logits given all preceding tokens
(Sec. 1; Fig. 2 "auto-regressive decoding"), which self-speculative decoding
reproduces exactly (Sec. 5.1, "Evaluation Metrics").

Readings where the paper is silent: eps inside the square root, gains applied
after normalisation, RoPE pairs element i with i+hd/2 and uses angle
pos * base^(-2i/hd), softmax scale 1/sqrt(hd), argmax ties go to the lowest
index, weights enter at their stored (fp32 or bf16) values widened exactly,
activations and the KV cache stay in fp64.
"""
from __future__ import annotations

import math
from typing import List, Optional, Sequence, Tuple

import torch

F64 = torch.float64


def widen(t: torch.Tensor) -> torch.Tensor:
    return t.to(F64)


# ----------------------------------------------------------------------------
# Elementary pieces
# ----------------------------------------------------------------------------
def rmsnorm(x: torch.Tensor, g: torch.Tensor, eps: float) -> torch.Tensor:
    """x / sqrt(mean(x^2) + eps) * g over the last axis."""
    ms = (x * x).mean(dim=-1, keepdim=True)
    return x / torch.sqrt(ms + eps) * g


def rope(v: torch.Tensor, pos: torch.Tensor, base: float) -> torch.Tensor:
    """Rotate v[..., T, n, hd] (or [T, n, hd]) by position.

    Pair (i, i + hd/2) turns by the angle pos * base^(-2i/hd).
    pos: int64 tensor [T].
    """
    hd = v.shape[-1]
    half = hd // 2
    i = torch.arange(half, dtype=F64)
    theta = torch.pow(torch.tensor(base, dtype=F64), -2.0 * i / hd)      # [half]
    ang = pos.to(F64)[:, None] * theta[None, :]                          # [T, half]
    c = torch.cos(ang)[:, None, :]                                       # [T, 1, half]
    s = torch.sin(ang)[:, None, :]
    lo, hi = v[..., :half], v[..., half:]
    return torch.cat([lo * c - hi * s, hi * c + lo * s], dim=-1)


def softmax_fp64(s: torch.Tensor) -> torch.Tensor:
    e = torch.exp(s - s.max(dim=-1, keepdim=True).values)
    return e / e.sum(dim=-1, keepdim=True)


def attend_one(q: torch.Tensor, K: torch.Tensor, V: torch.Tensor) -> torch.Tensor:
    """One query position over all cached positions.

    q [n_h, hd]; K, V [P, n_kv, hd] (P = positions 0..p).  Query head h reads
    KV head h // (n_h / n_kv).  Returns [n_h, hd].
    """
    n_h, hd = q.shape
    n_kv = K.shape[1]
    group = n_h // n_kv
    out = torch.empty(n_h, hd, dtype=F64)
    for h in range(n_h):
        kh = h // group
        s = (K[:, kh, :] @ q[h]) / math.sqrt(hd)          # [P]
        w = softmax_fp64(s)
        out[h] = w @ V[:, kh, :]
    return out


def attend_causal(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor) -> torch.Tensor:
    """All positions at once: q [T,n_h,hd], k, v [T,n_kv,hd] -> [T,n_h,hd].

    Position t sees positions 0..t only (scores above the diagonal are -inf
    before the softmax).
    """
    T, n_h, hd = q.shape
    group = n_h // k.shape[1]
    future = torch.triu(torch.ones(T, T, dtype=torch.bool), diagonal=1)
    out = torch.empty(T, n_h, hd, dtype=F64)
    for h in range(n_h):
        kh = h // group
        s = (q[:, h, :] @ k[:, kh, :].T) / math.sqrt(hd)      # [T(query), T(key)]
        s = s.masked_fill(future, float("-inf"))
        out[:, h, :] = softmax_fp64(s) @ v[:, kh, :]
    return out


def silu(z: torch.Tensor) -> torch.Tensor:
    return z / (1.0 + torch.exp(-z))


# ----------------------------------------------------------------------------
# Model
# ----------------------------------------------------------------------------
class Decoder:
    """The model as a set of fp64-evaluated functions over stored weights.

    `shape` is any object with n_layers, exit_layer, d_model, n_heads,
    n_kv_heads, head_dim, d_ffn, vocab, rope_base, rms_eps.  `weights` is the
    dict of tensors in the boundary layout: wqkv rows = q heads, k heads,
    v heads; wgu rows = gate then up.
    """

    def __init__(self, shape, weights: dict):
        self.s = shape
        self.w = weights
        self.nq = shape.n_heads * shape.head_dim
        self.nkv = shape.n_kv_heads * shape.head_dim

    # -- per-layer weight views (widened on use) ------------------------------
    def _wq(self, l): return widen(self.w["wqkv"][l][: self.nq])
    def _wk(self, l): return widen(self.w["wqkv"][l][self.nq: self.nq + self.nkv])
    def _wv(self, l): return widen(self.w["wqkv"][l][self.nq + self.nkv:])
    def _wg(self, l): return widen(self.w["wgu"][l][: self.s.d_ffn])
    def _wu(self, l): return widen(self.w["wgu"][l][self.s.d_ffn:])

    def embed(self, tokens: Sequence[int]) -> torch.Tensor:
        idx = torch.as_tensor(list(tokens), dtype=torch.int64)
        return widen(self.w["embed"][idx])

    def qkv(self, l: int, x: torch.Tensor, pos: torch.Tensor):
        """x [T, d] at positions pos [T] -> rotated q [T,n_h,hd], rotated k and v [T,n_kv,hd]."""
        s = self.s
        xn = rmsnorm(x, widen(self.w["attn_norm"][l]), s.rms_eps)
        T = x.shape[0]
        q = (xn @ self._wq(l).T).view(T, s.n_heads, s.head_dim)
        k = (xn @ self._wk(l).T).view(T, s.n_kv_heads, s.head_dim)
        v = (xn @ self._wv(l).T).view(T, s.n_kv_heads, s.head_dim)
        return rope(q, pos, s.rope_base), rope(k, pos, s.rope_base), v

    def after_attention(self, l: int, x: torch.Tensor, a: torch.Tensor) -> torch.Tensor:
        """Residual add of the attention output, then the SwiGLU MLP with its residual."""
        s = self.s
        x = x + a.reshape(x.shape[0], self.nq) @ widen(self.w["wo"][l]).T
        xn = rmsnorm(x, widen(self.w["mlp_norm"][l]), s.rms_eps)
        m = silu(xn @ self._wg(l).T) * (xn @ self._wu(l).T)
        return x + m @ widen(self.w["wdown"][l]).T

    def head_logits(self, x: torch.Tensor, which: str = "lm") -> torch.Tensor:
        """which = "lm": W_lm rmsnorm(x; g_final); "exit": the early-exit norm head."""
        g, W = ("final_norm", "lm_head") if which == "lm" else ("exit_norm", "exit_head")
        return rmsnorm(x, widen(self.w[g]), self.s.rms_eps) @ widen(self.w[W]).T

    # -- whole-sequence causal forward: the model's plain definition ----------
    def layer_full(self, l: int, x: torch.Tensor) -> torch.Tensor:
        T = x.shape[0]
        pos = torch.arange(T, dtype=torch.int64)
        q, k, v = self.qkv(l, x, pos)
        return self.after_attention(l, x, attend_causal(q, k, v))

    def hidden_full(self, tokens: Sequence[int], n_layers: Optional[int] = None) -> torch.Tensor:
        """Residual stream after the first n_layers layers, all positions: [T, d]."""
        x = self.embed(tokens)
        for l in range(self.s.n_layers if n_layers is None else n_layers):
            x = self.layer_full(l, x)
        return x

    def logits_full(self, tokens: Sequence[int]) -> torch.Tensor:
        """Full-model logits at every position: [T, V]."""
        return self.head_logits(self.hidden_full(tokens), "lm")

    @property
    def has_exit_block(self) -> bool:
        """The early-exit head is a transformer layer (entry n_layers of the per-layer lists) followed
        by the norm head (Sec. 5.4, "Impact of exit head") rather than the norm head alone."""
        return bool(getattr(self.s, "exit_block", False))

    def exit_logits_full(self, tokens: Sequence[int]) -> torch.Tensor:
        """Early-exit head logits (after exit_layer layers) at every position."""
        h = self.hidden_full(tokens, self.s.exit_layer)
        if self.has_exit_block:
            h = self.layer_full(self.s.n_layers, h)
        return self.head_logits(h, "exit")


def argmax_lowest(logits: torch.Tensor) -> int:
    """Index of the maximum; among equal maxima the lowest index."""
    m = logits.max()
    return int(torch.nonzero(logits == m)[0, 0])


def top2_margin(logits: torch.Tensor) -> Tuple[float, float]:
    """(top1 - top2, max |logit|) of one logits vector."""
    v = torch.topk(logits, 2).values
    return float(v[0] - v[1]), float(logits.abs().max())


def greedy_decode_no_cache(dec: Decoder, prompt: Sequence[int], n_new: int) -> List[int]:
    """The definition, literally: re-run the whole prefix for every new token."""
    seq = list(prompt)
    for _ in range(n_new):
        seq.append(argmax_lowest(dec.logits_full(seq)[-1]))
    return seq[len(prompt):]


# ----------------------------------------------------------------------------
# Incremental form (KV cache): same arithmetic, one position at a time.
# ----------------------------------------------------------------------------
class KVState:
    """Per-layer key/value rows with per-layer lengths (so a stage can roll back)."""

    def __init__(self, shape, max_seq: int):
        n = shape.n_layers + (1 if getattr(shape, "exit_block", False) else 0)   # the early-exit block keeps rows too
        self.K = torch.zeros(n, max_seq, shape.n_kv_heads, shape.head_dim, dtype=F64)
        self.V = torch.zeros_like(self.K)
        self.len = [0] * n

    def truncate(self, layers: range, new_len: int) -> None:
        for l in layers:
            assert new_len <= self.len[l]
            self.len[l] = new_len


def run_layers(dec: Decoder, kv: KVState, x: torch.Tensor, pos: int, layers: range) -> torch.Tensor:
    """Push one token's residual x [d] at position pos through `layers`, appending its K/V.

    Each layer must hold exactly positions 0..pos-1 beforehand: the new row is
    an append, never an overwrite of a live row.
    """
    x = x[None, :]
    p = torch.tensor([pos], dtype=torch.int64)
    for l in layers:
        assert kv.len[l] == pos, f"layer {l} holds {kv.len[l]} rows, appending position {pos}"
        q, k, v = dec.qkv(l, x, p)
        kv.K[l, pos], kv.V[l, pos] = k[0], v[0]
        kv.len[l] = pos + 1
        a = attend_one(q[0], kv.K[l, : pos + 1], kv.V[l, : pos + 1])
        x = dec.after_attention(l, x, a[None])
    return x[0]


def exit_logits(dec: Decoder, kv: KVState, h: torch.Tensor, pos: int) -> torch.Tensor:
    """Early-exit head on the layer-E hidden state h of the token at position pos.  With an exit block
    the state first goes through that layer, which appends its own K/V row at pos; the block's output
    feeds the head only, never the later layers."""
    if dec.has_exit_block:
        h = run_layers(dec, kv, h, pos, range(dec.s.n_layers, dec.s.n_layers + 1))
    return dec.head_logits(h, "exit")


def draft_layers_of(dec: Decoder) -> List[int]:
    """Layers whose KV rows a drafted token writes: 1..E, and the exit block."""
    return list(range(dec.s.exit_layer)) + ([dec.s.n_layers] if dec.has_exit_block else [])


class GreedyTrace:
    """Tokens plus, per generated token, the top-2 margin and max |logit| behind it."""

    def __init__(self):
        self.tokens: List[int] = []
        self.margin: List[float] = []
        self.absmax: List[float] = []
        self.logits: List[torch.Tensor] = []


def greedy_decode(dec: Decoder, prompt: Sequence[int], n_new: int, keep_logits: bool = False,
                  forced: Optional[Sequence[int]] = None) -> GreedyTrace:
    """Vanilla greedy autoregressive decoding with a KV cache.

    Returns n_new tokens (the first one follows the prompt).  With `forced`,
    the continuation is teacher-forced: token k fed back is forced[k] instead
    of the oracle's own argmax, while the trace still records the oracle's
    argmax and margins at every position.
    """
    L = range(dec.s.n_layers)
    kv = KVState(dec.s, len(prompt) + n_new)
    tr = GreedyTrace()
    seq = list(prompt)
    x = None
    for pos in range(len(prompt) + n_new - 1):
        x = run_layers(dec, kv, dec.embed([seq[pos]])[0], pos, L)
        if pos >= len(prompt) - 1:
            lg = dec.head_logits(x, "lm")
            tok = argmax_lowest(lg)
            m, a = top2_margin(lg)
            tr.tokens.append(tok); tr.margin.append(m); tr.absmax.append(a)
            if keep_logits:
                tr.logits.append(lg)
            k = len(tr.tokens) - 1
            seq.append(tok if forced is None else int(forced[k]))
    return tr
