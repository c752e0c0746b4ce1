"""Stochastic verification (Sec. 3.1, Eq. 1-2) on the CPU, fp64.  TEST INFRASTRUCTURE.

The draft token is SAMPLED from the early-exit head's distribution p (Eq. 1); the full model's
distribution q for the same position decides: the draft is accepted with probability
min(1, q(d) / p(d)) (Eq. 2), otherwise one token from the target model takes its place.  The paper
states the acceptance rule and that a rejected draft is replaced by "one additional token from the
target model"; the distribution of that token is the one of the speculative-sampling papers it
cites for the rule, normalise(max(0, q - p)), which is what makes the committed token exactly
q-distributed.  (Reading; listed with the others in the design document.)

Random numbers are a pure function of (seed, position, purpose), so the outcome does not depend on
how the work is scheduled: the splitmix64 output function applied to a key built from the three.
Both this module and the GPU library implement that generator from its published definition.

Sampling is by inverse CDF in index order: token = the first k with  sum_{i<=k} w_i > u * sum_i w_i.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Sequence, Tuple

import torch

from .decoder_fp64 import Decoder, KVState, draft_layers_of, exit_logits, run_layers
from .ppsd_schedule import PPSDStats, prefill

_M = (1 << 64) - 1
DRAFT, ACCEPT, RESAMPLE, VANILLA = 0, 1, 2, 3      # purposes (independent streams of random numbers)
_POS_MUL, _PURPOSE_MUL = 0xD1342543DE82EF95, 0xA0761D6478BD642F   # odd multipliers that spread the key bits


def splitmix64(x: int) -> int:
    """Output of the splitmix64 generator whose state before the step is x."""
    z = (x + 0x9E3779B97F4A7C15) & _M
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _M
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _M
    return z ^ (z >> 31)


def uniform(seed: int, pos: int, purpose: int) -> float:
    """u in [0, 1), a multiple of 2^-24 (exact in fp32), for one (seed, position, purpose)."""
    key = (seed ^ ((pos * _POS_MUL) & _M) ^ ((purpose * _PURPOSE_MUL) & _M)) & _M
    return (splitmix64(key) >> 40) * 2.0 ** -24


def softmax_t(logits: torch.Tensor, temperature: float) -> torch.Tensor:
    z = (logits.to(torch.float64) - logits.max().to(torch.float64)) / temperature
    w = torch.exp(z)
    return w / w.sum()


def sample(weights: torch.Tensor, u: float) -> int:
    """Inverse CDF in index order over non-negative weights (not necessarily normalised)."""
    cdf = torch.cumsum(weights.to(torch.float64), 0)
    thr = u * float(cdf[-1])
    k = int(torch.searchsorted(cdf, torch.tensor(thr, dtype=torch.float64), right=True))
    nz = torch.nonzero(weights > 0)
    return min(k, int(nz[-1, 0]))          # u*total == total cannot happen (u < 1); guards rounding only


def spec_verify(p: torch.Tensor, q: torch.Tensor, d: int, u_accept: float, u_resample: float) -> Tuple[int, bool]:
    """Eq. (2) for one draft d ~ p against the target distribution q."""
    if u_accept * float(p[d]) <= float(q[d]):
        return d, True
    r = torch.clamp(q - p, min=0.0)
    if float(r.sum()) == 0.0:              # p == q: unreachable in exact arithmetic (the draft would be accepted)
        r = q
    return sample(r, u_resample), False


@dataclass
class StochasticSession:
    dec: Decoder
    kv: KVState
    temperature: float
    seed: int
    t: int
    last_token: int
    full: bool = False
    h_exit: torch.Tensor = None
    draft: int = -1
    p_draft: torch.Tensor = None            # the distribution the in-flight draft was sampled from
    compared: List[int] = field(default_factory=list)
    stats: PPSDStats = field(default_factory=PPSDStats)


def stochastic_prefill(dec: Decoder, prompt: Sequence[int], max_seq: int, temperature: float,
                       seed: int) -> StochasticSession:
    """Prompt through the full model; token #0 is sampled from the full model's distribution."""
    base = prefill(dec, prompt, max_seq)     # runs the layers; its greedy token #0 is replaced below
    q = softmax_t(dec.head_logits(base.x_prompt, "lm"), temperature)
    tok0 = sample(q, uniform(seed, len(prompt), VANILLA))
    return StochasticSession(dec=dec, kv=base.kv, temperature=temperature, seed=seed, t=base.t, last_token=tok0)


def stochastic_step(ss: StochasticSession, out: List[int]) -> None:
    """One two-stage verify-while-draft step with sampled drafts and Eq. (2) verification."""
    dec, kv, s, T = ss.dec, ss.kv, ss.dec.s, ss.temperature
    draft_layers, verify_layers = range(0, s.exit_layer), range(s.exit_layer, s.n_layers)
    if not ss.full:
        h = run_layers(dec, kv, dec.embed([ss.last_token])[0], ss.t, draft_layers)
        ss.h_exit = h
        ss.p_draft = softmax_t(exit_logits(dec, kv, h, ss.t), T)
        ss.draft = sample(ss.p_draft, uniform(ss.seed, ss.t + 1, DRAFT))
        ss.full = True
        ss.stats.steps_draft_only += 1
        return
    pos = ss.t + 1                                    # the position being decided
    h_next = run_layers(dec, kv, dec.embed([ss.draft])[0], pos, draft_layers)
    p_next = softmax_t(exit_logits(dec, kv, h_next, pos), T)
    d_next = sample(p_next, uniform(ss.seed, pos + 1, DRAFT))
    x = run_layers(dec, kv, ss.h_exit, ss.t, verify_layers)
    q = softmax_t(dec.head_logits(x, "lm"), T)
    tok, ok = spec_verify(ss.p_draft, q, ss.draft, uniform(ss.seed, pos, ACCEPT), uniform(ss.seed, pos, RESAMPLE))
    st = ss.stats
    st.steps_overlapped += 1; st.drafts_compared += 1; st.committed += 1
    out.append(tok)
    ss.compared.append(ss.draft)
    if ok:
        st.accepted += 1
        ss.h_exit, ss.draft, ss.p_draft = h_next, d_next, p_next
    else:
        st.rejected += 1; st.kv_rollbacks += 1
        kv.truncate(draft_layers_of(dec), pos)
        ss.full = False
    ss.t = pos
    ss.last_token = tok


def stochastic_decode(ss: StochasticSession, n_tokens: int) -> List[int]:
    out: List[int] = []
    while len(out) < n_tokens:
        stochastic_step(ss, out)
    return out


def vanilla_sample_decode(dec: Decoder, prompt: Sequence[int], n_new: int, temperature: float, seed: int) -> List[int]:
    """Plain autoregressive sampling from the full model: token at position p uses uniform(seed, p, VANILLA)."""
    s = dec.s
    kv = KVState(s, len(prompt) + n_new)
    seq = list(prompt)
    out: List[int] = []
    for pos in range(len(prompt) + n_new - 1):
        x = run_layers(dec, kv, dec.embed([seq[pos]])[0], pos, range(s.n_layers))
        if pos >= len(prompt) - 1:
            tok = sample(softmax_t(dec.head_logits(x, "lm"), temperature), uniform(seed, pos + 1, VANILLA))
            out.append(tok); seq.append(tok)
    return out


# ----------------------------------------------------------------------------
# Stochastic verification in the full ceil(N/E)-stage schedule (Sec. 4.1-4.2, Alg. 1 with sampling)
# ----------------------------------------------------------------------------
# Stage 0 samples one draft per tick from the early-exit head's distribution and keeps that
# distribution until the draft's check token arrives S-1 ticks later; the last stage's
# distribution q decides by Eq. (2); a rejected draft is replaced by a token from
# normalise(max(0, q - p)) and everything in flight is flushed.  Because the uniforms are keyed by
# position and purpose, and every draft that reaches verification was made from accepted tokens
# only, the committed stream is the one the two-stage schedule commits with the same seed.
from .ppsd_schedule import PipelineSession, PipelineStats, pipeline_prefill, stage_ranges   # noqa: E402


@dataclass
class StochasticPipelineSession:
    base: PipelineSession
    temperature: float
    seed: int
    p_at: dict = field(default_factory=dict)        # position -> distribution its draft was sampled from


def stochastic_pipeline_prefill(dec: Decoder, prompt: Sequence[int], max_seq: int, temperature: float,
                                seed: int) -> StochasticPipelineSession:
    base = pipeline_prefill(dec, prompt, max_seq)
    two = prefill(dec, prompt, max_seq)
    q = softmax_t(dec.head_logits(two.x_prompt, "lm"), temperature)
    tok0 = sample(q, uniform(seed, len(prompt), VANILLA))
    base.last_token = tok0
    base.tok0 = tok0
    return StochasticPipelineSession(base=base, temperature=temperature, seed=seed)


def stochastic_pipeline_tick(sp: StochasticPipelineSession, out: List[int]) -> None:
    ss, T, seed = sp.base, sp.temperature, sp.seed
    dec, kv = ss.dec, ss.kv
    S = len(ss.stages)
    st = ss.stats
    st.ticks += 1
    produced = [None] * S
    draft_next = None
    for k in range(S):
        if not ss.valid[k]:
            continue
        st.stage_runs += 1
        x_in = dec.embed([ss.tok0])[0] if k == 0 else ss.hidden[k]
        if k == 0:
            ss.token_at[ss.pos[0]] = ss.tok0
        for l in list(ss.stages[k]) + ([dec.s.n_layers] if k == 0 and dec.has_exit_block else []):
            if kv.len[l] > ss.pos[k]:
                kv.len[l] = ss.pos[k]
        produced[k] = run_layers(dec, kv, x_in, ss.pos[k], ss.stages[k])
        if k == 0:
            p_new = softmax_t(exit_logits(dec, kv, produced[0], ss.pos[0]), T)
            sp.p_at[ss.pos[0] + 1] = p_new
            draft_next = sample(p_new, uniform(seed, ss.pos[0] + 1, DRAFT))
    flush = False
    if ss.valid[S - 1]:
        q = softmax_t(dec.head_logits(produced[S - 1], "lm"), T)
        p = ss.pos[S - 1] + 1
        d = ss.token_at[p]
        tok, ok = spec_verify(sp.p_at[p], q, d, uniform(seed, p, ACCEPT), uniform(seed, p, RESAMPLE))
        st.committed += 1; st.drafts_compared += 1
        out.append(tok)
        ss.compared.append(d)
        ss.t, ss.last_token = p, tok
        if ok:
            st.accepted += 1
        else:
            st.rejected += 1
            flush = True
    if flush:
        st.flushed_tokens += sum(1 for x in ss.token_at if x >= ss.t)
        ss.token_at = {}
        sp.p_at = {}
        ss.valid = [True] + [False] * (S - 1)
        ss.pos = [ss.t] + [0] * (S - 1)
        ss.tok0 = ss.last_token
        return
    for k in range(S - 1, 0, -1):
        ss.valid[k] = ss.valid[k - 1]
        ss.pos[k] = ss.pos[k - 1]
        ss.hidden[k] = produced[k - 1]
    ss.pos[0] += 1
    ss.tok0 = draft_next
    ss.token_at = {x: tk for x, tk in ss.token_at.items() if x > ss.t}
    sp.p_at = {x: pv for x, pv in sp.p_at.items() if x > ss.t}


def stochastic_pipeline_decode(sp: StochasticPipelineSession, n_tokens: int) -> List[int]:
    out: List[int] = []
    while len(out) < n_tokens:
        stochastic_pipeline_tick(sp, out)
    return out


# ----------------------------------------------------------------------------
# Stochastic verification in draft-then-verify rounds: Eq. (1)-(2) as stated, gamma drafts per round
# ----------------------------------------------------------------------------
# Each of the gamma drafts is sampled from the early-exit head's distribution given the drafts
# before it (Eq. 1); the full model's distributions for the same positions come from one batched
# pass; the drafts are checked in order by Eq. (2), the first rejected one is replaced by a token
# from normalise(max(0, q - p)) and the rest discarded; if all are accepted one more token is
# sampled from the full model's distribution for the next position (Sec. 3.1).
from .eesd_schedule import EESDSession, eesd_prefill   # noqa: E402


def stochastic_eesd_prefill(dec: Decoder, prompt: Sequence[int], max_seq: int, gamma: int, temperature: float,
                            seed: int) -> EESDSession:
    ss = eesd_prefill(dec, prompt, max_seq, gamma)
    two = prefill(dec, prompt, max_seq)
    q = softmax_t(dec.head_logits(two.x_prompt, "lm"), temperature)
    ss.last_token = sample(q, uniform(seed, len(prompt), VANILLA))
    return ss


def stochastic_eesd_round(ss: EESDSession, out: List[int], limit: int, temperature: float, seed: int) -> None:
    dec, kv, s, g, T = ss.dec, ss.kv, ss.dec.s, ss.gamma, temperature
    draft_layers, verify_layers = range(0, s.exit_layer), range(s.exit_layer, s.n_layers)
    t = ss.t
    x: List[int] = [ss.last_token]
    h: List[torch.Tensor] = []
    p: List[torch.Tensor] = []
    for j in range(g):
        h.append(run_layers(dec, kv, dec.embed([x[j]])[0], t + j, draft_layers))
        p.append(softmax_t(exit_logits(dec, kv, h[j], t + j), T))
        x.append(sample(p[j], uniform(seed, t + j + 1, DRAFT)))
    h.append(run_layers(dec, kv, dec.embed([x[g]])[0], t + g, draft_layers))
    if dec.has_exit_block:
        exit_logits(dec, kv, h[g], t + g)
    q = [softmax_t(dec.head_logits(run_layers(dec, kv, h[j], t + j, verify_layers), "lm"), T) for j in range(g + 1)]
    toks: List[int] = []
    n = 0
    while n < g:
        pos = t + n + 1
        tok, ok = spec_verify(p[n], q[n], x[n + 1], uniform(seed, pos, ACCEPT), uniform(seed, pos, RESAMPLE))
        toks.append(tok)
        if not ok:
            break
        n += 1
    if n == g:                                  # every draft accepted: the full model's own token follows
        toks.append(sample(q[g], uniform(seed, t + g + 1, VANILLA)))
    st = ss.stats
    st.rounds += 1
    st.layer_reads += (g + 1) * len(draft_layers) + len(verify_layers)
    st.drafts_compared += min(g, n + 1)
    st.accepted += n
    st.rejected += 1 if n < g else 0
    k = min(n + 1, limit)
    for i in range(k):
        out.append(toks[i])
        ss.compared.append(x[i + 1] if i < g else -1)
    st.committed += k
    ss.t = t + k
    ss.last_token = toks[k - 1]
    kv.truncate(range(len(kv.len)), ss.t)


def stochastic_eesd_decode(ss: EESDSession, n_tokens: int, temperature: float, seed: int) -> List[int]:
    out: List[int] = []
    while len(out) < n_tokens:
        stochastic_eesd_round(ss, out, n_tokens - len(out), temperature, seed)
    return out
