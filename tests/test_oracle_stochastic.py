"""Pins for stochastic verification (Sec. 3.1, Eq. 1-2): the generator, inverse-CDF sampling, and that the
committed token is distributed exactly as the full model's distribution whatever the draft distribution."""
import itertools

import torch

import synth_inputs as S
from oracle import decoder_fp64 as O
from oracle import ppsd_schedule as P
from oracle import stochastic as ST


def test_splitmix64_published_outputs():
    """First two outputs of splitmix64 seeded with 0 (the reference implementation's test values)."""
    assert ST.splitmix64(0) == 0xE220A8397B1DCDAF
    assert ST.splitmix64(0x9E3779B97F4A7C15) == 0x6E789E6AA1B965F4


def test_uniform_is_a_24_bit_fraction_and_spreads():
    us = [ST.uniform(7, p, k) for p in range(4000) for k in range(4)]
    assert all(0.0 <= u < 1.0 and (u * 2 ** 24) == int(u * 2 ** 24) for u in us)
    assert len(set(us)) > 0.999 * len(us)
    t = torch.tensor(us, dtype=torch.float64)
    assert abs(float(t.mean()) - 0.5) < 0.01 and abs(float(t.var()) - 1 / 12) < 0.005
    # sixteen equal bins: chi-square with 15 degrees of freedom, far below any sane rejection level
    counts = torch.histc(t, bins=16, min=0.0, max=1.0)
    chi2 = float(((counts - len(us) / 16) ** 2 / (len(us) / 16)).sum())
    assert chi2 < 45.0
    # streams are independent of each other: purposes and neighbouring positions do not repeat
    assert ST.uniform(7, 5, 0) != ST.uniform(7, 5, 1) != ST.uniform(7, 6, 0) != ST.uniform(8, 5, 0)


def test_inverse_cdf_gives_each_index_its_own_interval():
    w = torch.tensor([0.0, 0.2, 0.0, 0.5, 0.3, 0.0], dtype=torch.float64) * 7.0      # unnormalised, with zeros
    edges = [0.0, 0.2, 0.7, 1.0]
    owners = [1, 3, 4]
    for lo, hi, k in zip(edges[:-1], edges[1:], owners):
        for u in (lo + 1e-9, (lo + hi) / 2, hi - 1e-9):
            assert ST.sample(w, u) == k
    assert ST.sample(w, 0.0) == 1                      # u = 0 belongs to the first index with weight
    n = 20000
    freq = torch.zeros(6, dtype=torch.float64)
    for i in range(n):
        freq[ST.sample(w, (i + 0.5) / n)] += 1
    assert torch.allclose(freq / n, w / w.sum(), atol=1.0 / n + 1e-12)


def _output_distribution(p, q, n=160):
    """P(committed token = k) for a draft d ~ p verified against q, integrating the two uniforms on a grid."""
    V = p.numel()
    out = torch.zeros(V, dtype=torch.float64)
    grid = [(i + 0.5) / n for i in range(n)]
    for d in range(V):
        if float(p[d]) == 0.0:
            continue
        acc = torch.zeros(V, dtype=torch.float64)
        for ua in grid:
            tok, ok = ST.spec_verify(p, q, d, ua, 0.5)
            if ok:
                acc[tok] += 1.0
            else:                                     # integrate the resample uniform only where it is used
                for ur in grid[:: max(1, n // 40)]:
                    acc[ST.spec_verify(p, q, d, ua, ur)[0]] += 1.0 / len(grid[:: max(1, n // 40)])
        out += float(p[d]) * acc / n
    return out


def test_committed_token_is_distributed_as_the_target_whatever_the_draft_distribution():
    g = torch.Generator().manual_seed(3)
    for _ in range(4):
        p = torch.softmax(2.0 * torch.randn(6, generator=g, dtype=torch.float64), 0)
        q = torch.softmax(2.0 * torch.randn(6, generator=g, dtype=torch.float64), 0)
        got = _output_distribution(p, q)
        assert torch.allclose(got, q, atol=0.02), (got, q)
    # a draft distribution with holes and a peaked target
    p = torch.tensor([0.5, 0.5, 0.0, 0.0], dtype=torch.float64)
    q = torch.tensor([0.1, 0.0, 0.6, 0.3], dtype=torch.float64)
    assert torch.allclose(_output_distribution(p, q), q, atol=0.02)


def test_degenerate_cases_of_the_acceptance_rule():
    p = torch.tensor([0.25, 0.25, 0.5], dtype=torch.float64)
    for d, ua in itertools.product(range(3), (0.0, 0.5, 0.999999)):
        assert ST.spec_verify(p, p, d, ua, 0.3) == (d, True)             # identical distributions: always accepted
    q = torch.tensor([0.0, 0.0, 1.0], dtype=torch.float64)
    assert ST.spec_verify(p, q, 0, 0.0, 0.3) == (0, True)                # u = 0 accepts even a hopeless draft: u p <= q
    assert ST.spec_verify(p, q, 0, 1e-9, 0.3) == (2, False)              # q(d) = 0: rejected, replaced from q - p
    assert ST.spec_verify(p, q, 2, 0.999999, 0.3) == (2, True)           # q(d) > p(d): accepted for every u
    # acceptance probability is q(d) / p(d) where that is below one
    q2 = torch.tensor([0.1, 0.4, 0.5], dtype=torch.float64)
    n = 4000
    acc = sum(ST.spec_verify(p, q2, 0, (i + 0.5) / n, 0.3)[1] for i in range(n)) / n
    assert abs(acc - 0.1 / 0.25) < 2.0 / n


def test_low_temperature_reproduces_the_greedy_schedule(tiny_shape):
    w = tiny_shape.replace(decode_len=16)
    W = S.make_weights(w)
    dec = O.Decoder(w, W)
    prompt = S.make_prompt(w)
    g = P.prefill(dec, prompt, 64)
    gt = [g.last_token] + P.decode(g, 16)
    s = ST.stochastic_prefill(dec, prompt, 64, 1e-4, seed=11)
    st = [s.last_token] + ST.stochastic_decode(s, 16)
    assert st == gt and s.stats == g.stats
    assert ST.vanilla_sample_decode(dec, prompt, 17, 1e-4, seed=11) == gt


def test_stochastic_schedule_bookkeeping_and_rollback(tiny_shape):
    w = tiny_shape.replace(decode_len=40, exit_head="independent")
    W = S.make_weights(w)
    dec = O.Decoder(w, W)
    prompt = S.make_prompt(w)
    s = ST.stochastic_prefill(dec, prompt, 80, 1.0, seed=5)
    toks = ST.stochastic_decode(s, 40)
    st = s.stats
    assert st.committed == 40 == st.accepted + st.rejected and 0 < st.accepted < 40
    assert st.steps_draft_only == 1 + st.rejected - (0 if s.full else 1)
    # accepted <=> the committed token is the draft it was compared with
    assert sum(1 for d, t in zip(s.compared, toks) if d == t) == st.accepted
    # the KV cache holds exactly the committed positions (+ the in-flight draft's rows in layers 1..E)
    assert s.kv.len[w.n_layers - 1] == s.t
    assert s.kv.len[0] == s.t + (1 if s.full else 0)
    # the same seed gives the same stream, another seed another one
    s2 = ST.stochastic_prefill(dec, prompt, 80, 1.0, seed=5)
    assert ST.stochastic_decode(s2, 40) == toks
    s3 = ST.stochastic_prefill(dec, prompt, 80, 1.0, seed=6)
    assert ST.stochastic_decode(s3, 40) != toks


def test_pipeline_schedule_commits_the_two_stage_stream_under_sampling(tiny_shape):
    """Uniforms are keyed by position and purpose and every verified draft was made from accepted tokens,
    so the number of stages cannot change the committed stream, the compared drafts or the outcomes."""
    for E, n_layers in ((1, 3), (2, 5), (1, 4)):
        w = tiny_shape.replace(exit_layer=E, n_layers=n_layers, decode_len=30, exit_head="blend", exit_beta=1.0)
        W = S.make_weights(w)
        W["lm_head"], W["exit_head"] = W["lm_head"] * 30.0, W["exit_head"] * 30.0
        dec = O.Decoder(w, W)
        prompt = S.make_prompt(w)
        a = ST.stochastic_prefill(dec, prompt, 80, 0.9, seed=21)
        ta = [a.last_token] + ST.stochastic_decode(a, 30)
        b = ST.stochastic_pipeline_prefill(dec, prompt, 80, 0.9, seed=21)
        tb = [b.base.last_token] + ST.stochastic_pipeline_decode(b, 30)
        assert ta == tb and a.compared == b.base.compared
        assert (a.stats.accepted, a.stats.rejected) == (b.base.stats.accepted, b.base.stats.rejected)
        assert 0 < a.stats.accepted < 30
        n_stages = -(-n_layers // E)
        assert b.base.stats.flushed_tokens == (n_stages - 1) * b.base.stats.rejected


def test_sampled_rounds_reduce_to_the_greedy_rounds_at_low_temperature(tiny_shape):
    from oracle import eesd_schedule as EE
    w = tiny_shape.replace(decode_len=20)
    W = S.make_weights(w)
    dec = O.Decoder(w, W)
    prompt = S.make_prompt(w)
    for gamma in (1, 3):
        g = EE.eesd_prefill(dec, prompt, 64, gamma)
        gt = [g.last_token] + EE.eesd_decode(g, 20)
        s = ST.stochastic_eesd_prefill(dec, prompt, 64, gamma, 1e-4, seed=4)
        st = [s.last_token] + ST.stochastic_eesd_decode(s, 20, 1e-4, seed=4)
        assert st == gt and s.stats == g.stats and s.compared == g.compared


def test_sampled_rounds_follow_the_position_keyed_decisions(tiny_shape):
    """Up to the first round in which every draft is accepted (whose extra token is a plain sample), the
    stream is the one the two-stage schedule commits with the same seed: same distributions, same uniforms."""
    w = tiny_shape.replace(decode_len=30, exit_head="blend", exit_beta=1.0)
    W = S.make_weights(w)
    W["lm_head"], W["exit_head"] = W["lm_head"] * 30.0, W["exit_head"] * 30.0
    dec = O.Decoder(w, W)
    prompt = S.make_prompt(w)
    a = ST.stochastic_prefill(dec, prompt, 80, 0.9, seed=21)
    ta = [a.last_token] + ST.stochastic_decode(a, 30)
    for gamma in (2, 4):
        e = ST.stochastic_eesd_prefill(dec, prompt, 80, gamma, 0.9, seed=21)
        te = [e.last_token] + ST.stochastic_eesd_decode(e, 30, 0.9, seed=21)
        first_bonus = next((i for i, c in enumerate(e.compared) if c == -1), len(e.compared))
        assert te[: first_bonus + 1] == ta[: first_bonus + 1]
        assert e.compared[:first_bonus] == a.compared[:first_bonus]
        st = e.stats
        assert st.committed == 30 and st.rejected > 0 and st.accepted > 0
        assert e.kv.len == [e.t] * w.n_layers
