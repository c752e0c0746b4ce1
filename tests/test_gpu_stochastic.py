"""GPU parity of stochastic verification (Sec. 3.1, Eq. 1-2) against the CPU simulator, and a
distribution-level check that committed tokens follow the full model's distribution."""
import math

import pytest
import torch

import synth_inputs as S
from oracle import decoder_fp64 as O
from oracle import stochastic as ST
from tests.parity_util import to_device

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def P():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU (torch.cuda.is_available() is False)")
    import paper_2509_19368_amd as pkg
    pkg.load_library()
    return pkg


SHAPES = [
    S.WORKLOADS["C1"].replace(decode_len=48),
    S.Workload("s3", n_layers=3, exit_layer=1, d_model=192, n_heads=4, n_kv_heads=2, head_dim=64, d_ffn=328,
               vocab=1003, dtype="fp32", damp=0.2, seed=11, prompt_len=9, decode_len=40),
    S.Workload("s5", n_layers=5, exit_layer=2, d_model=128, n_heads=2, n_kv_heads=1, head_dim=64, d_ffn=264,
               vocab=515, dtype="fp32", damp=0.3, seed=23, prompt_len=4, decode_len=40, exit_block=True,
               exit_block_damp=0.3),
]


def _run(P, w, Wg, prompt, n, mode, T, seed, **kw):
    ss = P.Session(w, Wg, max_seq=len(prompt) + n + 2, mode=mode, debug_logits=n + 1, temperature=T, sample_seed=seed, **kw)
    toks = [ss.ppsd_prefill(prompt)] + ss.ppsd_decode(n)
    out = dict(tokens=toks, logits=ss.read_logits(0, n + 1), drafts=ss.read_drafts(0, n + 1), stats=ss.ppsd_stats())
    ss.close()
    return out


def _consistent(dec, prompt, r, T, seed, delta):
    """Teacher-forced protocol for sampled streams: with the GPU's own committed prefix, every decision
    the GPU took must be a valid decision for the oracle's fp64 distributions up to a shift delta of the
    uniform (delta bounds the error of the cumulative probabilities).  Returns how many decisions needed
    the slack."""
    toks, drafts = r["tokens"], r["drafts"]
    seq = list(prompt) + toks
    P0 = len(prompt)
    lm = dec.logits_full(seq[:-1])
    ex = dec.exit_logits_full(seq[:-1])
    loose = 0

    def inside(w, k, u, d_):
        cdf = torch.cumsum(w / w.sum(), 0)
        lo = float(cdf[k - 1]) if k > 0 else 0.0
        hi = float(cdf[k])
        assert lo - d_ <= u < hi + d_, (k, u, lo, hi)
        return not (lo <= u < hi)

    q0 = ST.softmax_t(lm[P0 - 1], T)
    loose += inside(q0, toks[0], ST.uniform(seed, P0, ST.VANILLA), delta)
    for k in range(1, len(toks)):
        pos = P0 + k
        q = ST.softmax_t(lm[pos - 1], T)
        p = ST.softmax_t(ex[pos - 1], T)
        d, tok = drafts[k], toks[k]
        loose += inside(p, d, ST.uniform(seed, pos, ST.DRAFT), delta)
        ua = ST.uniform(seed, pos, ST.ACCEPT)
        if tok == d:
            assert ua * float(p[d]) <= float(q[d]) + delta
        else:
            assert ua * float(p[d]) >= float(q[d]) - delta
            rres = torch.clamp(q - p, min=0.0)
            loose += inside(rres, tok, ST.uniform(seed, pos, ST.RESAMPLE), delta / float(rres.sum()))
    return loose


@pytest.mark.parametrize("T", [1.0, 0.6])
@pytest.mark.parametrize("w", SHAPES, ids=[w.name for w in SHAPES])
def test_sampled_streams_equal_the_simulator(P, w, T):
    W = S.make_weights(w)
    # N(0, 0.02) heads give almost flat distributions (every draft accepted); 20x makes p and q peaked and distinct
    W["lm_head"], W["exit_head"] = W["lm_head"] * 20.0, W["exit_head"] * 20.0
    prompt = S.make_prompt(w)
    n = w.decode_len
    dec = O.Decoder(w, W)
    Wg = to_device(W, "cuda")
    seed = 1234
    ss = ST.stochastic_prefill(dec, prompt, len(prompt) + n + 2, T, seed)
    want = [ss.last_token] + ST.stochastic_decode(ss, n)
    runs = [_run(P, w, Wg, prompt, n, m, T, seed, use_graph=g) for m, g in
            ((P.MODE_SERIAL, True), (P.MODE_OVERLAP, True), (P.MODE_OVERLAP, False))]
    for r in runs:
        assert r["tokens"] == runs[0]["tokens"] and r["drafts"] == runs[0]["drafts"]
        assert _consistent(dec, prompt, r, T, seed, 2e-5) <= 1
    r = runs[1]
    # fp32 against fp64: the streams coincide unless a uniform falls within ~1e-6 of a boundary
    assert r["tokens"] == want and r["drafts"] == [-1] + ss.compared
    st = r["stats"]
    assert (st["accepted"], st["rejected"], st["steps_draft_only"], st["kv_rollbacks"]) == \
           (ss.stats.accepted, ss.stats.rejected, ss.stats.steps_draft_only, ss.stats.kv_rollbacks)
    assert 0 < st["accepted"] < n
    # the full pipeline schedule draws the same numbers at the same positions: same stream, drafts, outcomes
    S_ = -(-w.n_layers // w.exit_layer)
    sp = ST.stochastic_pipeline_prefill(dec, prompt, len(prompt) + n + S_ + 2, T, seed)
    pwant = [sp.base.last_token] + ST.stochastic_pipeline_decode(sp, n)
    assert pwant == want
    pr = P.Session(w, Wg, max_seq=len(prompt) + 1 + n + S_, mode=P.MODE_PIPELINE, temperature=T, sample_seed=seed)
    ptoks = [pr.ppsd_prefill(prompt)] + pr.ppsd_decode(n)
    pst, pdr = pr.ppsd_stats(), pr.read_drafts(0, n + 1)
    pr.close()
    assert ptoks == want and pdr == [-1] + sp.base.compared
    assert (pst["accepted"], pst["rejected"], pst["pipeline_ticks"], pst["stage_runs"], pst["flushed_tokens"]) == \
           (sp.base.stats.accepted, sp.base.stats.rejected, sp.base.stats.ticks, sp.base.stats.stage_runs,
            sp.base.stats.flushed_tokens)
    v = _run(P, w, Wg, prompt, n, P.MODE_VANILLA, T, seed)
    assert v["tokens"] == ST.vanilla_sample_decode(dec, prompt, n + 1, T, seed)
    assert _run(P, w, Wg, prompt, n, P.MODE_OVERLAP, T, seed + 1)["tokens"] != r["tokens"]


def test_low_temperature_is_the_greedy_path(P):
    w = S.WORKLOADS["C1"]
    Wg = to_device(S.make_weights(w), "cuda")
    prompt = S.make_prompt(w)
    g = _run(P, w, Wg, prompt, 48, P.MODE_OVERLAP, 0.0, 0)
    s = _run(P, w, Wg, prompt, 48, P.MODE_OVERLAP, 1e-4, 99)
    assert g["tokens"] == s["tokens"] and g["drafts"] == s["drafts"]
    assert torch.equal(g["logits"], s["logits"])


def test_bf16_stream_is_consistent_with_the_oracle_distributions(P):
    w = S.Workload("sb", n_layers=4, exit_layer=2, d_model=256, n_heads=4, n_kv_heads=1, head_dim=128, d_ffn=712,
                   vocab=777, dtype="bf16", damp=0.2, seed=12, prompt_len=21, decode_len=40)
    W = S.make_weights(w)
    prompt = S.make_prompt(w)
    r = _run(P, w, to_device(W, "cuda"), prompt, 40, P.MODE_OVERLAP, 0.8, 77, kv_page_tokens=8)
    # bf16 storage of the KV cache moves logits by up to 2e-2 of their scale: cumulative probabilities by a few percent
    loose = _consistent(O.Decoder(w, W), prompt, r, 0.8, 77, 0.05)
    assert loose <= 8 and 0 < r["stats"]["accepted"] < 40


def test_committed_tokens_follow_the_target_distribution(P):
    """800 seeds on a 24-word model: the first decoded token, given the most frequent token #0, must be
    distributed as the full model's q for that prefix (chi-square), and the acceptance rate must be
    sum_i min(p_i, q_i)."""
    w = S.Workload("dist", n_layers=2, exit_layer=1, d_model=64, n_heads=1, n_kv_heads=1, head_dim=64, d_ffn=128,
                   vocab=24, dtype="fp32", damp=0.6, seed=3, prompt_len=5, decode_len=1, exit_head="blend", exit_beta=1.0)
    W = S.make_weights(w)
    W["lm_head"] = W["lm_head"] * 40.0          # peaked enough that a few words carry the mass
    W["exit_head"] = W["exit_head"] * 40.0
    prompt = S.make_prompt(w)
    dec = O.Decoder(w, W)
    Wg = to_device(W, "cuda")
    T = 1.0
    groups = {}
    for seed in range(800):
        ss = P.Session(w, Wg, max_seq=16, mode=P.MODE_SERIAL, temperature=T, sample_seed=seed)
        t0 = ss.ppsd_prefill(prompt)
        t1 = ss.ppsd_decode(1)[0]
        acc = ss.ppsd_stats()["accepted"]
        ss.close()
        groups.setdefault(t0, []).append((t1, acc))
    t0, obs = max(groups.items(), key=lambda kv: len(kv[1]))
    n = len(obs)
    assert n >= 150
    seq = list(prompt) + [t0]
    q = ST.softmax_t(dec.logits_full(seq)[-1], T)
    p = ST.softmax_t(dec.exit_logits_full(seq)[-1], T)
    counts = torch.zeros(w.vocab, dtype=torch.float64)
    for t1, _ in obs:
        counts[t1] += 1
    big = [i for i in range(w.vocab) if n * float(q[i]) >= 5.0]
    assert len(big) >= 3
    chi2 = sum((float(counts[i]) - n * float(q[i])) ** 2 / (n * float(q[i])) for i in big)
    rest_e = n * (1.0 - sum(float(q[i]) for i in big))
    rest_o = n - sum(float(counts[i]) for i in big)
    dof = len(big) - 1
    if rest_e >= 5.0:
        chi2 += (rest_o - rest_e) ** 2 / rest_e
        dof += 1
    assert chi2 < dof + 4.0 * math.sqrt(2.0 * dof) + 6.0, (chi2, dof)
    alpha = float(torch.minimum(p, q).sum())
    got = sum(a for _, a in obs) / n
    assert abs(got - alpha) < 4.0 * math.sqrt(alpha * (1 - alpha) / n) + 0.01, (got, alpha)
    assert 0.15 < alpha < 0.95


@pytest.mark.parametrize("gamma", [1, 3, 4])
def test_sampled_draft_then_verify_rounds_equal_the_simulator(P, gamma):
    """Eq. (1)-(2) as stated: gamma sampled drafts per round, checked in order against one batched pass."""
    for w in SHAPES:
        W = S.make_weights(w)
        W["lm_head"], W["exit_head"] = W["lm_head"] * 20.0, W["exit_head"] * 20.0
        prompt = S.make_prompt(w)
        n = w.decode_len
        dec = O.Decoder(w, W)
        T, seed = 0.8, 4321
        es = ST.stochastic_eesd_prefill(dec, prompt, len(prompt) + n + gamma + 2, gamma, T, seed)
        want = [es.last_token] + ST.stochastic_eesd_decode(es, n, T, seed)
        ss = P.Session(w, to_device(W, "cuda"), max_seq=len(prompt) + 1 + n + gamma, mode=P.MODE_EESD, eesd_gamma=gamma,
                       temperature=T, sample_seed=seed)
        toks = [ss.ppsd_prefill(prompt)] + ss.ppsd_decode(n)
        st, drafts = ss.ppsd_stats(), ss.read_drafts(0, n + 1)
        ss.close()
        assert toks == want and drafts == [-1] + es.compared
        assert (st["eesd_rounds"], st["accepted"], st["rejected"], st["drafts_compared"]) == \
               (es.stats.rounds, es.stats.accepted, es.stats.rejected, es.stats.drafts_compared)
        assert st["accepted"] > 0 and st["rejected"] > 0
