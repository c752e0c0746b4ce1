"""Two-stage verify-while-draft decoding on the CPU.  TEST INFRASTRUCTURE.

What it follows.  The first E layers plus the early-exit head are the draft
model; the whole model is the verifier, and the verifier reuses the draft
pass's activations and KV cache so only layers E+1..N run again (Sec. 3.1).
The stages form a pipeline in which the draft stage keeps proposing while the
later stage carries the previous token to the LM head (Sec. 4.1, 4.2).  The
last stage's token is compared with the draft made for the same position; on
a mismatch generation restarts at the position after the checked token
(Alg. 1: receive check token, compare with own draft, reset the index).

Collapsed to two stages (draft = layers 1..E + exit head, verify = layers
E+1..N + LM head) there is at most one speculative token in flight.  One
step is:

  FULL state (h_t^E and draft d_{t+1} in hand):
    draft stage : d_{t+1} at position t+1 through layers 1..E -> h_{t+1}^E, d_{t+2}
    verify stage: h_t^E at position t through layers E+1..N  -> v_{t+1}
    commit      : emit v_{t+1} (always the full model's greedy token);
                  equal to d_{t+1}: stay FULL at t+1;
                  different: drop the KV row the draft stage wrote at t+1,
                  discard h_{t+1}^E and d_{t+2}, go EMPTY with v_{t+1} as the
                  next draft-stage input.
  EMPTY state (after prefill or a rejection; last committed token y_t):
    draft stage : y_t at position t through layers 1..E -> h_t^E, d_{t+1}
    verify stage: idle (the pipeline refills); no token is emitted.

The committed stream is the vanilla greedy stream whatever the exit head
produces; the tests hold this simulator to that.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Sequence

import torch

from .decoder_fp64 import Decoder, KVState, argmax_lowest, run_layers


@dataclass
class PPSDStats:
    committed: int = 0
    drafts_compared: int = 0
    accepted: int = 0
    rejected: int = 0
    steps_overlapped: int = 0
    steps_draft_only: int = 0
    kv_rollbacks: int = 0

    @property
    def acceptance(self) -> float:
        return self.accepted / self.drafts_compared if self.drafts_compared else 0.0


@dataclass
class PPSDSession:
    """State carried between steps (mirrors what the GPU library keeps on the device)."""
    dec: Decoder
    kv: KVState
    t: int = -1                     # position of the last committed token
    last_token: int = -1            # y_t
    full: bool = False
    h_exit: torch.Tensor = None     # h_t^E when full
    draft: int = -1                 # d_{t+1} when full
    stats: PPSDStats = field(default_factory=PPSDStats)


def prefill(dec: Decoder, prompt: Sequence[int], max_seq: int) -> PPSDSession:
    """Run the full model over the prompt and commit generated token #0.

    Afterwards every layer holds KV rows for positions 0..P-1, token #0 sits at
    position P and the pipeline is EMPTY.
    """
    s = dec.s
    kv = KVState(s, max_seq)
    x = None
    for pos, tok in enumerate(prompt):
        x = run_layers(dec, kv, dec.embed([tok])[0], pos, range(s.n_layers))
    tok0 = argmax_lowest(dec.head_logits(x, "lm"))
    return PPSDSession(dec=dec, kv=kv, t=len(prompt), last_token=tok0, full=False)


def step(ss: PPSDSession, out: List[int]) -> None:
    """One pipeline step; appends to `out` iff a token is committed."""
    dec, kv, s = ss.dec, ss.kv, ss.dec.s
    draft_layers, verify_layers = range(0, s.exit_layer), range(s.exit_layer, s.n_layers)
    if not ss.full:
        h = run_layers(dec, kv, dec.embed([ss.last_token])[0], ss.t, draft_layers)
        ss.h_exit, ss.draft = h, argmax_lowest(dec.head_logits(h, "exit"))
        ss.full = True
        ss.stats.steps_draft_only += 1
        return
    # draft stage on the speculative token, verify stage on the committed one
    h_next = run_layers(dec, kv, dec.embed([ss.draft])[0], ss.t + 1, draft_layers)
    d_next = argmax_lowest(dec.head_logits(h_next, "exit"))
    x = run_layers(dec, kv, ss.h_exit, ss.t, verify_layers)
    v = argmax_lowest(dec.head_logits(x, "lm"))
    st = ss.stats
    st.steps_overlapped += 1
    st.drafts_compared += 1
    st.committed += 1
    out.append(v)
    if v == ss.draft:
        st.accepted += 1
        ss.h_exit, ss.draft = h_next, d_next
    else:
        st.rejected += 1
        st.kv_rollbacks += 1
        kv.truncate(draft_layers, ss.t + 1)
        ss.full = False
    ss.t += 1
    ss.last_token = v


def decode(ss: PPSDSession, n_tokens: int) -> List[int]:
    """Commit exactly n_tokens further tokens (resumable: state stays in ss)."""
    out: List[int] = []
    while len(out) < n_tokens:
        step(ss, out)
    return out
