"""GPU parity of the full ceil(N/E)-stage schedule (Sec. 4.1-4.2, Alg. 1) against the CPU simulator.

Tokens, compared drafts and every counter must equal the oracle's on fp32 shapes; on any shape the
schedule must commit bit for bit what the library's own vanilla mode commits.
"""
import pytest
import torch

import synth_inputs as S
from oracle import decoder_fp64 as O
from oracle import ppsd_schedule as SCH
from tests.parity_util import REL_TOL_BF16, REL_TOL_FP32, check_against_teacher_forced_oracle, to_device

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def P():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU (torch.cuda.is_available() is False)")
    import paper_2509_19368_amd as pkg
    pkg.load_library()
    return pkg


# fp32 shapes with 2..6 stages, a shorter last stage among them, acceptance between 0.4 and 0.8
PIPE = [
    S.Workload("p7e2", n_layers=7, exit_layer=2, d_model=128, n_heads=2, n_kv_heads=2, head_dim=64, d_ffn=264,
               vocab=515, dtype="fp32", damp=0.08, seed=21, prompt_len=6, decode_len=48),
    S.Workload("p6e1", n_layers=6, exit_layer=1, d_model=192, n_heads=4, n_kv_heads=2, head_dim=64, d_ffn=328,
               vocab=1003, dtype="fp32", damp=0.05, seed=22, prompt_len=11, decode_len=48),
    S.Workload("p5e2", n_layers=5, exit_layer=2, d_model=256, n_heads=2, n_kv_heads=1, head_dim=128, d_ffn=512,
               vocab=640, dtype="fp32", damp=0.07, seed=23, prompt_len=3, decode_len=48),
    S.WORKLOADS["C1"],                                # 4 layers, E = 1: four stages
    S.WORKLOADS["C1"].replace(name="C1_E3", exit_layer=3),   # two stages of 3 and 1 layers
]


def _n_stages(w, later=0):
    return 1 + -(-(w.n_layers - w.exit_layer) // (later or w.exit_layer))


def _run(P, w, Wg, prompt, calls, mode, **kw):
    n = sum(calls)
    max_seq = kw.pop("max_seq", len(prompt) + 1 + n + _n_stages(w) - 1)
    ss = P.Session(w, Wg, max_seq=max_seq, mode=mode, debug_logits=n + 1, **kw)
    toks = [ss.ppsd_prefill(prompt)]
    stats_after = []
    for c in calls:
        toks += ss.ppsd_decode(c)
        stats_after.append(ss.ppsd_stats())
    out = dict(tokens=toks, logits=ss.read_logits(0, n + 1), drafts=ss.read_drafts(0, n + 1), stats=stats_after)
    ss.close()
    return out


def _oracle(w, W, prompt, calls, later=None):
    dec = O.Decoder(w, W)
    ss = SCH.pipeline_prefill(dec, prompt, len(prompt) + sum(calls) + 2 * _n_stages(w) + 2, later)
    toks = [ss.last_token]
    snaps = []
    for c in calls:
        toks += SCH.pipeline_decode(ss, c)
        st = ss.stats
        snaps.append(dict(committed=st.committed, drafts_compared=st.drafts_compared, accepted=st.accepted,
                          rejected=st.rejected, pipeline_ticks=st.ticks, stage_runs=st.stage_runs,
                          flushed_tokens=st.flushed_tokens))
    return dec, toks, list(ss.compared), snaps


@pytest.mark.parametrize("w", PIPE, ids=[w.name for w in PIPE])
def test_pipeline_schedule_equals_the_simulator(P, w):
    W = S.make_weights(w)
    prompt = S.make_prompt(w)
    calls = [w.decode_len]
    dec, toks, compared, snaps = _oracle(w, W, prompt, calls)
    assert 0 < snaps[-1]["rejected"] < snaps[-1]["committed"], "the case must exercise both outcomes"
    r = _run(P, w, to_device(W, "cuda"), prompt, calls, P.MODE_PIPELINE)
    assert r["tokens"] == toks
    assert r["drafts"] == [-1] + compared
    for k, v in snaps[-1].items():
        assert r["stats"][-1][k] == v, k
    assert r["stats"][-1]["kv_rollbacks"] == snaps[-1]["rejected"]
    # lossless: the stream is the vanilla greedy stream, logits to fp32 rounding of the fp64 oracle
    tr = O.greedy_decode(dec, prompt, w.decode_len + 1, keep_logits=True)
    assert r["tokens"] == tr.tokens
    ref = torch.stack(tr.logits)
    err = ((r["logits"].double() - ref).abs().max(dim=1).values / ref.abs().max(dim=1).values).max().item()
    assert err <= REL_TOL_FP32
    # Eq. (7): one tick per token, S-1 more per rejection (the last token's outcome costs nothing
    # yet), S-1 ticks to fill the pipeline after prefill
    S_ = _n_stages(w)
    n = w.decode_len
    rej_before_last = sum(1 for k in range(1, n) if r["drafts"][k] != r["tokens"][k])
    assert r["stats"][-1]["pipeline_ticks"] == (S_ - 1) + n + (S_ - 1) * rej_before_last


@pytest.mark.parametrize("later", [3, 2, 5, 1])
def test_pipeline_with_later_stages_of_another_size_equals_the_simulator(P, later):
    """pipeline_stage_layers: the layers behind the draft stage cut into stages of `later` layers (7 layers, exit
    layer 2: S = 3, 4, 2, 6).  Tokens, compared drafts and every counter equal the simulator's for that partition,
    logits bitwise equal to vanilla mode, ticks = Eq. (7)'s cost model with the partition's S."""
    w = S.Workload("pl7", n_layers=7, exit_layer=2, d_model=128, n_heads=2, n_kv_heads=2, head_dim=64, d_ffn=264,
                   vocab=515, dtype="fp32", damp=0.25, seed=61, prompt_len=7, decode_len=30)
    W = S.make_weights(w)
    prompt = S.make_prompt(w)
    calls = [11, 19]
    n = sum(calls)
    S_ = _n_stages(w, later)
    dec, want, compared, snaps = _oracle(w, W, prompt, calls, later)
    Wg = to_device(W, "cuda")
    max_seq = len(prompt) + 1 + n + S_ - 1
    g = _run(P, w, Wg, prompt, calls, P.MODE_PIPELINE, max_seq=max_seq, pipeline_stage_layers=later)
    v = _run(P, w, Wg, prompt, calls, P.MODE_VANILLA, max_seq=max_seq)
    assert g["tokens"] == want == v["tokens"] and torch.equal(g["logits"], v["logits"])
    assert g["drafts"][1:] == compared
    for got, ref in zip(g["stats"], snaps):
        for k, val in ref.items():
            assert got[k] == val, (k, got[k], val)
    rej_before_last = sum(1 for k in range(1, n) if g["drafts"][k] != g["tokens"][k])
    assert g["stats"][-1]["pipeline_ticks"] == (S_ - 1) + n + (S_ - 1) * rej_before_last
    with pytest.raises(P.PpsdError):       # capacity: S - 1 speculative positions beyond the last committed token
        _run(P, w, Wg, prompt, calls, P.MODE_PIPELINE, max_seq=max_seq - 1, pipeline_stage_layers=later)


def test_pipeline_is_resumable_and_graph_replay_equals_direct_launch(P):
    w = PIPE[0]
    W = S.make_weights(w)
    prompt = S.make_prompt(w)
    calls = [1, 7, 2, 20, 18]
    dec, toks, compared, snaps = _oracle(w, W, prompt, calls)
    Wg = to_device(W, "cuda")
    a = _run(P, w, Wg, prompt, calls, P.MODE_PIPELINE, use_graph=True)
    b = _run(P, w, Wg, prompt, calls, P.MODE_PIPELINE, use_graph=False)
    c = _run(P, w, Wg, prompt, [sum(calls)], P.MODE_PIPELINE, use_graph=True, pipeline_streams=2)
    for ns in (3, 4):      # the stages of a tick spread over more streams: same arithmetic, same result
        e = _run(P, w, Wg, prompt, [sum(calls)], P.MODE_PIPELINE, pipeline_streams=ns)
        assert e["tokens"] == toks and torch.equal(e["logits"], a["logits"])
    for r in (a, b):
        assert r["tokens"] == toks and r["drafts"] == [-1] + compared
        for got, want in zip(r["stats"], snaps):       # the counters agree at every call boundary
            for k, v in want.items():
                assert got[k] == v, k
    assert torch.equal(a["logits"], b["logits"]) and torch.equal(a["logits"], c["logits"])
    assert c["tokens"] == toks


def test_two_stage_pipeline_commits_what_the_overlap_mode_commits(P):
    for w in (PIPE[4], S.WORKLOADS["C1"].replace(name="C1_E2", exit_layer=2)):
        assert _n_stages(w) == 2
        Wg = to_device(S.make_weights(w), "cuda")
        prompt = S.make_prompt(w)
        a = _run(P, w, Wg, prompt, [w.decode_len], P.MODE_PIPELINE)
        b = _run(P, w, Wg, prompt, [w.decode_len], P.MODE_OVERLAP)
        assert a["tokens"] == b["tokens"] and a["drafts"] == b["drafts"]
        assert torch.equal(a["logits"], b["logits"])
        for k in ("committed", "drafts_compared", "accepted", "rejected", "kv_rollbacks", "steps_overlapped",
                  "steps_draft_only"):
            assert a["stats"][-1][k] == b["stats"][-1][k], k
        assert a["stats"][-1]["pipeline_ticks"] == b["stats"][-1]["steps_overlapped"] + b["stats"][-1]["steps_draft_only"]


def test_pipeline_bf16_ragged_shapes_against_vanilla_and_teacher_forced_oracle(P):
    shapes = [
        S.Workload("r16e1", n_layers=4, exit_layer=1, d_model=256, n_heads=4, n_kv_heads=1, head_dim=128, d_ffn=712,
                   vocab=777, dtype="bf16", damp=0.1, seed=12, prompt_len=21, decode_len=40),
        S.Workload("m16e1", n_layers=3, exit_layer=1, d_model=128, n_heads=2, n_kv_heads=2, head_dim=64, d_ffn=264,
                   vocab=515, dtype="bf16", damp=0.1, seed=13, prompt_len=5, decode_len=30),
    ]
    for w in shapes:
        W = S.make_weights(w)
        prompt = S.make_prompt(w)
        Wg = to_device(W, "cuda")
        a = _run(P, w, Wg, prompt, [w.decode_len], P.MODE_PIPELINE, kv_page_tokens=8)
        v = _run(P, w, Wg, prompt, [w.decode_len], P.MODE_VANILLA, kv_page_tokens=8)
        assert a["tokens"] == v["tokens"] and torch.equal(a["logits"], v["logits"])
        check_against_teacher_forced_oracle(O.Decoder(w, W), prompt, a["tokens"], a["logits"], REL_TOL_BF16)
        st = a["stats"][-1]
        assert st["committed"] == w.decode_len == st["drafts_compared"] == st["accepted"] + st["rejected"]
        assert st["flushed_tokens"] == (_n_stages(w) - 1) * st["rejected"]


def test_pipeline_capacity_and_configuration_errors(P):
    w = PIPE[0]
    Wg = to_device(S.make_weights(w), "cuda")
    prompt = S.make_prompt(w)
    S_ = _n_stages(w)
    n = 12
    # prompt + token #0 + n tokens + the S-1 positions stage 0 runs ahead: fits exactly
    fits = len(prompt) + 1 + n + S_ - 1
    ok = _run(P, w, Wg, prompt, [n], P.MODE_PIPELINE, max_seq=fits)
    assert len(ok["tokens"]) == n + 1
    ss = P.Session(w, Wg, max_seq=fits - 1, mode=P.MODE_PIPELINE)
    ss.ppsd_prefill(prompt)
    with pytest.raises(P.PpsdError) as e:
        ss.ppsd_decode(n)
    assert e.value.code == -3
    assert len(ss.ppsd_decode(n - 1)) == n - 1           # the context stays usable
    ss.close()
    with pytest.raises(P.PpsdError):
        P.Session(w, Wg, max_seq=64, mode=P.MODE_PIPELINE, engine=P.ENGINE_PERSISTENT)
    with pytest.raises(P.PpsdError):
        P.Session(w, Wg, max_seq=64, mode=P.MODE_PIPELINE, time_kernels=True)


def test_pipeline_full_size_7b_is_bitwise_the_vanilla_stream(P):
    """C2 (7B bf16) with E = 8: four stages.  Same kernels on the same committed prefix as vanilla
    decoding, so tokens and logits must be identical; the counters must obey Eq. (7)."""
    w = S.WORKLOADS["C2"]
    n = 48
    Wg = S.make_weights(w, device="cuda")
    prompt = S.make_prompt(w)
    a = _run(P, w, Wg, prompt, [n], P.MODE_PIPELINE)
    v = _run(P, w, Wg, prompt, [n], P.MODE_VANILLA)
    assert a["tokens"] == v["tokens"]
    assert torch.equal(a["logits"], v["logits"])
    st = a["stats"][-1]
    S_ = _n_stages(w)
    assert S_ == 4
    rej_before_last = sum(1 for k in range(1, n) if a["drafts"][k] != a["tokens"][k])
    assert st["pipeline_ticks"] == (S_ - 1) + n + (S_ - 1) * rej_before_last
    assert st["flushed_tokens"] == (S_ - 1) * st["rejected"]
    assert 0 < st["rejected"] < n


@pytest.mark.parametrize("name,prompt_len,n", [("C4", 48, 10), ("C5", 600, 8)], ids=["13B", "8B_GQA_long_context"])
def test_big_shapes_pipeline_and_rounds_against_vanilla(P, name, prompt_len, n):
    """13B and 8B-GQA shapes (two attention splits on the latter): the S-stage schedule must commit vanilla
    mode's stream bit for bit; draft-then-verify rounds (column slabs in the down-projection) stay within
    2e-3 of vanilla mode's logits on the common prefix."""
    w = S.WORKLOADS[name].replace(prompt_len=prompt_len, decode_len=n)
    Wg = S.make_weights(w, device="cuda")
    prompt = S.make_prompt(w)
    v = _run(P, w, Wg, prompt, [n], P.MODE_VANILLA, max_seq=prompt_len + n + 8)
    a = _run(P, w, Wg, prompt, [n], P.MODE_PIPELINE, max_seq=prompt_len + n + 8)
    assert a["tokens"] == v["tokens"] and torch.equal(a["logits"], v["logits"])
    st = a["stats"][-1]
    assert st["committed"] == n and st["flushed_tokens"] == (_n_stages(w) - 1) * st["rejected"]
    e = _run(P, w, Wg, prompt, [n], P.MODE_EESD, max_seq=prompt_len + n + 8, eesd_gamma=3)
    same = 0
    while same <= n and e["tokens"][same] == v["tokens"][same]:
        same += 1
    assert same >= 2
    scale = v["logits"].abs().max(dim=1).values
    assert ((e["logits"][:same] - v["logits"][:same]).abs().max(dim=1).values / scale[:same]).max().item() < 2e-3
    assert e["stats"][-1]["committed"] == n
