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
from typing import List, Optional, Sequence

import torch

from .decoder_fp64 import Decoder, KVState, argmax_lowest, draft_layers_of, exit_logits, run_layers


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
    x_prompt: torch.Tensor = None   # the full model's hidden state behind the last prompt position
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
        if dec.has_exit_block:        # the block attends over its own rows of every earlier position
            h = run_layers(dec, kv, dec.embed([tok])[0], pos, range(s.exit_layer))
            exit_logits(dec, kv, h, pos)
            x = run_layers(dec, kv, h, pos, range(s.exit_layer, s.n_layers))
        else:
            x = run_layers(dec, kv, dec.embed([tok])[0], pos, range(s.n_layers))
    tok0 = argmax_lowest(dec.head_logits(x, "lm"))
    return PPSDSession(dec=dec, kv=kv, t=len(prompt), last_token=tok0, full=False, x_prompt=x)


def step(ss: PPSDSession, out: List[int]) -> None:
    """One pipeline step; appends to `out` iff a token is committed."""
    dec, kv, s = ss.dec, ss.kv, ss.dec.s
    draft_layers, verify_layers = range(0, s.exit_layer), range(s.exit_layer, s.n_layers)
    if not ss.full:
        h = run_layers(dec, kv, dec.embed([ss.last_token])[0], ss.t, draft_layers)
        ss.h_exit, ss.draft = h, argmax_lowest(exit_logits(dec, kv, h, ss.t))
        ss.full = True
        ss.stats.steps_draft_only += 1
        return
    # draft stage on the speculative token, verify stage on the committed one
    h_next = run_layers(dec, kv, dec.embed([ss.draft])[0], ss.t + 1, draft_layers)
    d_next = argmax_lowest(exit_logits(dec, kv, h_next, ss.t + 1))
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
        kv.truncate(draft_layers_of(dec), ss.t + 1)
        ss.full = False
    ss.t += 1
    ss.last_token = v


def decode(ss: PPSDSession, n_tokens: int) -> List[int]:
    """Commit exactly n_tokens further tokens (resumable: state stays in ss)."""
    out: List[int] = []
    while len(out) < n_tokens:
        step(ss, out)
    return out


# ----------------------------------------------------------------------------
# The full ceil(N/E)-stage schedule (Sec. 4.1, 4.2, Alg. 1)
# ----------------------------------------------------------------------------
# The N layers are cut into S = ceil(N/E) stages of E layers (the last one takes what remains);
# stage 0 also holds the early-exit head and keeps drafting one token per tick from its own
# previous draft, every later stage carries the token it received one tick earlier one stage
# further, and the last stage's LM head yields the model's true next token.  That token is
# compared with the draft made for the same position (the check token of Alg. 1); on a mismatch
# every token in flight was computed from a wrong draft: all of them, and the KV rows they wrote in
# every stage, are dropped and stage 0 restarts from the verified token at the position after it
# (Alg. 1's index reset).  An accepted token therefore costs one tick and a rejected one S ticks,
# which is Eq. (7).


@dataclass
class PipelineStats:
    committed: int = 0
    drafts_compared: int = 0
    accepted: int = 0
    rejected: int = 0
    ticks: int = 0
    stage_runs: int = 0            # stage executions, summed over stages and ticks
    flushed_tokens: int = 0        # in-flight speculative tokens dropped by rejections

    @property
    def acceptance(self) -> float:
        return self.accepted / self.drafts_compared if self.drafts_compared else 0.0


def stage_ranges(n_layers: int, exit_layer: int, later_stage_layers: Optional[int] = None) -> List[range]:
    """Layers of each pipeline stage: E per stage, the remainder forms a last, shorter stage (Sec. 4.1).

    The first stage is always the draft model, layers 1..E, because the early-exit head reads the state
    behind layer E.  later_stage_layers = w cuts the N - E layers behind it into stages of w layers instead
    of E (the last takes what remains): a partition the paper does not use (its stages are one GPU each and
    must be equal), but the schedule of Alg. 1 is defined for any partition whose first stage ends at the
    exit layer; w = N - E is the two-stage schedule.
    """
    w = exit_layer if later_stage_layers is None else later_stage_layers
    assert w >= 1
    return [range(0, exit_layer)] + [range(lo, min(lo + w, n_layers)) for lo in range(exit_layer, n_layers, w)]


@dataclass
class PipelineSession:
    dec: Decoder
    kv: KVState
    t: int                                   # position of the last committed token
    last_token: int
    stages: List[range] = None
    valid: List[bool] = None                 # valid[k]: stage k has an input for the coming tick
    pos: List[int] = None                    # position that input belongs to
    hidden: List[torch.Tensor] = None        # hidden[k]: input of stage k (k >= 1)
    tok0: int = -1                           # token stage 0 will embed
    token_at: dict = field(default_factory=dict)   # position -> token stage 0 used there
    compared: List[int] = field(default_factory=list)   # per committed token: the draft it was checked against
    stats: PipelineStats = field(default_factory=PipelineStats)


def pipeline_prefill(dec: Decoder, prompt: Sequence[int], max_seq: int,
                     later_stage_layers: Optional[int] = None) -> PipelineSession:
    base = prefill(dec, prompt, max_seq)
    stages = stage_ranges(dec.s.n_layers, dec.s.exit_layer, later_stage_layers)
    S = len(stages)
    ss = PipelineSession(dec=dec, kv=base.kv, t=base.t, last_token=base.last_token, stages=stages)
    ss.valid = [True] + [False] * (S - 1)
    ss.pos = [base.t] + [0] * (S - 1)
    ss.hidden = [None] * S
    ss.tok0 = base.last_token
    return ss


def pipeline_tick(ss: PipelineSession, out: List[int]) -> None:
    dec, kv = ss.dec, ss.kv
    S = len(ss.stages)
    st = ss.stats
    st.ticks += 1
    produced = [None] * S            # produced[k]: hidden state leaving stage k this tick
    draft_next = None
    # all stages work on different tokens within a tick; their order does not matter
    for k in range(S):
        if not ss.valid[k]:
            continue
        st.stage_runs += 1
        x_in = dec.embed([ss.tok0])[0] if k == 0 else ss.hidden[k]
        if k == 0:
            ss.token_at[ss.pos[0]] = ss.tok0
        # a stage re-running a position after a flush overwrites the dropped row
        for l in list(ss.stages[k]) + ([dec.s.n_layers] if k == 0 and dec.has_exit_block else []):
            if kv.len[l] > ss.pos[k]:
                kv.len[l] = ss.pos[k]
        produced[k] = run_layers(dec, kv, x_in, ss.pos[k], ss.stages[k])
        if k == 0:
            draft_next = argmax_lowest(exit_logits(dec, kv, produced[0], ss.pos[0]))
    flush = False
    if ss.valid[S - 1]:
        v = argmax_lowest(dec.head_logits(produced[S - 1], "lm"))
        p = ss.pos[S - 1] + 1                      # the position v belongs to
        st.committed += 1
        out.append(v)
        ss.t, ss.last_token = p, v
        if p in ss.token_at:                       # a draft for that position is in flight: check token
            st.drafts_compared += 1
            ss.compared.append(ss.token_at[p])
            if ss.token_at[p] == v:
                st.accepted += 1
            else:
                st.rejected += 1
                flush = True
        elif S > 1:
            raise AssertionError("a committed token without a draft can only happen with a single stage")
    if flush or S == 1:
        if flush:
            st.flushed_tokens += sum(1 for q in ss.token_at if q >= ss.t)   # the rejected draft and all after it
        ss.token_at = {}
        ss.valid = [True] + [False] * (S - 1)
        ss.pos = [ss.t] + [0] * (S - 1)
        ss.tok0 = ss.last_token
        return
    # no flush: every token moves one stage on, stage 0 continues from its own draft
    for k in range(S - 1, 0, -1):
        ss.valid[k] = ss.valid[k - 1]
        ss.pos[k] = ss.pos[k - 1]
        ss.hidden[k] = produced[k - 1]
    ss.pos[0] += 1
    ss.tok0 = draft_next
    ss.token_at = {q: tk for q, tk in ss.token_at.items() if q > ss.t}


def pipeline_decode(ss: PipelineSession, n_tokens: int) -> List[int]:
    out: List[int] = []
    while len(out) < n_tokens:
        pipeline_tick(ss, out)
    return out
