"""Early-exit speculative decoding, draft-then-verify, on the CPU.  TEST INFRASTRUCTURE.

What it follows (Sec. 3.1).  The first E layers plus the early-exit head are the draft model.  A
round drafts gamma tokens one after the other, then the full model verifies them in one pass; since
the draft pass has already produced the layer-E hidden states and the KV rows of layers 1..E, the
verification only runs layers E+1..N, over all drafted positions at once (causal among them).  The
longest prefix of drafts that equals the full model's tokens is accepted and one more token, the
full model's own, is committed behind it (the correction after a mismatch, or the token after the
last draft when all were accepted).  Eq. (4) gives the expected accepted length, Eq. (5) the gain
with a cost of gamma E + N layer reads per round.

One round from a committed token y_t at position t (KV rows of all layers valid below t):

  draft      : x_0 = y_t;  for j = 0..gamma-1:  h_j = layers 1..E on x_j at t+j,  x_{j+1} = exit head(h_j)
  last hidden: h_gamma = layers 1..E on x_gamma at t+gamma          (needed for the token after the last draft)
  verify     : for j = 0..gamma: v_j = LM head(layers E+1..N on h_j at t+j)   -- one batched pass
  accept     : n = number of leading j < gamma with x_{j+1} == v_j;  commit v_0..v_n  (n + 1 tokens)
  roll back  : KV rows at positions above t+n, in every layer, belong to rejected drafts: dropped.

The verify pass is written position by position here; with causal attention that is the definition
of the batched pass.  The committed stream is the vanilla greedy stream; the tests hold the
simulator to that.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Sequence

import torch

from .decoder_fp64 import Decoder, KVState, argmax_lowest, exit_logits, run_layers
from .ppsd_schedule import prefill


@dataclass
class EESDStats:
    committed: int = 0
    rounds: int = 0
    drafts_compared: int = 0     # drafts that met their verifier token (up to and including the first mismatch)
    accepted: int = 0
    rejected: int = 0            # rounds that ended at a mismatch
    layer_reads: int = 0         # layers whose weights a round streams: (gamma + 1) E + (N - E) = gamma E + N

    @property
    def acceptance(self) -> float:
        return self.accepted / self.drafts_compared if self.drafts_compared else 0.0


@dataclass
class EESDSession:
    dec: Decoder
    kv: KVState
    t: int
    last_token: int
    gamma: int
    compared: List[int] = field(default_factory=list)   # per committed token: the draft it was checked against, -1 if none
    stats: EESDStats = field(default_factory=EESDStats)


def eesd_prefill(dec: Decoder, prompt: Sequence[int], max_seq: int, gamma: int) -> EESDSession:
    base = prefill(dec, prompt, max_seq)
    return EESDSession(dec=dec, kv=base.kv, t=base.t, last_token=base.last_token, gamma=gamma)


def eesd_round(ss: EESDSession, out: List[int], limit: int) -> None:
    """One draft-then-verify round; commits at most `limit` tokens (what lies beyond is discarded)."""
    dec, kv, s, g = ss.dec, ss.kv, ss.dec.s, ss.gamma
    draft_layers, verify_layers = range(0, s.exit_layer), range(s.exit_layer, s.n_layers)
    t = ss.t
    x: List[int] = [ss.last_token]
    h: List[torch.Tensor] = []
    for j in range(g):
        h.append(run_layers(dec, kv, dec.embed([x[j]])[0], t + j, draft_layers))
        x.append(argmax_lowest(exit_logits(dec, kv, h[j], t + j)))
    h.append(run_layers(dec, kv, dec.embed([x[g]])[0], t + g, draft_layers))
    if dec.has_exit_block:            # the block's row at t+gamma: later drafts attend to it if all are accepted
        exit_logits(dec, kv, h[g], t + g)
    v = [argmax_lowest(dec.head_logits(run_layers(dec, kv, h[j], t + j, verify_layers), "lm")) for j in range(g + 1)]
    n = 0
    while n < g and x[n + 1] == v[n]:
        n += 1
    st = ss.stats
    st.rounds += 1
    st.layer_reads += (g + 1) * len(draft_layers) + len(verify_layers)
    st.drafts_compared += min(g, n + 1)
    st.accepted += n
    st.rejected += 1 if n < g else 0
    k = min(n + 1, limit)
    for i in range(k):
        out.append(v[i])
        ss.compared.append(x[i + 1] if i < g else -1)
    st.committed += k
    ss.t = t + k
    ss.last_token = v[k - 1]
    kv.truncate(range(len(kv.len)), ss.t)


def eesd_decode(ss: EESDSession, n_tokens: int) -> List[int]:
    out: List[int] = []
    while len(out) < n_tokens:
        eesd_round(ss, out, n_tokens - len(out))
    return out
