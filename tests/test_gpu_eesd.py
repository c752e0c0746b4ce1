"""GPU parity of draft-then-verify rounds (Sec. 3.1, Eq. 4-5; batched verify pass) against the CPU simulator."""
import pytest
import torch

import synth_inputs as S
from oracle import decoder_fp64 as O
from oracle import eesd_schedule as EE
from tests.parity_util import REL_TOL_BF16, REL_TOL_FP32, check_against_teacher_forced_oracle, to_device

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def P():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU (torch.cuda.is_available() is False)")
    import paper_2509_19368_amd as pkg
    pkg.load_library()
    return pkg


SHAPES = [
    S.WORKLOADS["C1"],
    S.Workload("e7", n_layers=7, exit_layer=2, d_model=128, n_heads=2, n_kv_heads=2, head_dim=64, d_ffn=264,
               vocab=515, dtype="fp32", damp=0.08, seed=21, prompt_len=6, decode_len=40),
    S.Workload("e3", n_layers=3, exit_layer=1, d_model=192, n_heads=4, n_kv_heads=2, head_dim=64, d_ffn=328,
               vocab=1003, dtype="fp32", damp=0.1, seed=11, prompt_len=9, decode_len=40),
    S.Workload("e5", n_layers=5, exit_layer=3, d_model=256, n_heads=2, n_kv_heads=1, head_dim=128, d_ffn=512,
               vocab=640, dtype="fp32", damp=0.25, seed=23, prompt_len=1, decode_len=40),
]


def _run(P, w, Wg, prompt, calls, mode, gamma=0, **kw):
    n = sum(calls)
    max_seq = kw.pop("max_seq", len(prompt) + 1 + n + max(gamma, 1))
    ss = P.Session(w, Wg, max_seq=max_seq, mode=mode, debug_logits=n + 1, eesd_gamma=gamma, **kw)
    toks = [ss.ppsd_prefill(prompt)]
    stats = []
    for c in calls:
        toks += ss.ppsd_decode(c)
        stats.append(ss.ppsd_stats())
    out = dict(tokens=toks, logits=ss.read_logits(0, n + 1), drafts=ss.read_drafts(0, n + 1), stats=stats)
    ss.close()
    return out


def _oracle(w, W, prompt, calls, gamma):
    dec = O.Decoder(w, W)
    ss = EE.eesd_prefill(dec, prompt, len(prompt) + sum(calls) + gamma + 2, gamma)
    toks = [ss.last_token]
    snaps = []
    for c in calls:
        toks += EE.eesd_decode(ss, c)
        st = ss.stats
        snaps.append(dict(committed=st.committed, eesd_rounds=st.rounds, drafts_compared=st.drafts_compared,
                          accepted=st.accepted, rejected=st.rejected, kv_rollbacks=st.rejected))
    return dec, toks, list(ss.compared), snaps


@pytest.mark.parametrize("gamma", [1, 2, 3, 4])
@pytest.mark.parametrize("w", SHAPES, ids=[w.name for w in SHAPES])
def test_rounds_equal_the_simulator(P, w, gamma):
    W = S.make_weights(w)
    prompt = S.make_prompt(w)
    calls = [w.decode_len]
    dec, toks, compared, snaps = _oracle(w, W, prompt, calls, gamma)
    Wg = to_device(W, "cuda")
    r = _run(P, w, Wg, prompt, calls, P.MODE_EESD, gamma)
    assert r["tokens"] == toks
    assert r["drafts"] == [-1] + compared
    for k, v in snaps[-1].items():
        assert r["stats"][-1][k] == v, k
    # the batched pass does, per token, what the single-token kernels do: same logits as vanilla mode
    v = _run(P, w, Wg, prompt, calls, P.MODE_VANILLA)
    assert v["tokens"] == r["tokens"] and torch.equal(v["logits"], r["logits"])
    tr = O.greedy_decode(dec, prompt, w.decode_len + 1, keep_logits=True)
    assert tr.tokens == toks
    ref = torch.stack(tr.logits)
    err = ((r["logits"].double() - ref).abs().max(dim=1).values / ref.abs().max(dim=1).values).max().item()
    assert err <= REL_TOL_FP32


def test_both_outcomes_are_exercised():
    for w in SHAPES:
        W = S.make_weights(w)
        _, _, _, snaps = _oracle(w, W, S.make_prompt(w), [w.decode_len], 3)
        assert 0 < snaps[-1]["rejected"] and snaps[-1]["accepted"] > 0, w.name


def test_resumed_calls_cut_rounds_and_graph_replay_equals_direct_launch(P):
    w = SHAPES[1]
    W = S.make_weights(w)
    prompt = S.make_prompt(w)
    calls = [1, 2, 5, 7, 3, 22]
    dec, toks, compared, snaps = _oracle(w, W, prompt, calls, 3)
    Wg = to_device(W, "cuda")
    a = _run(P, w, Wg, prompt, calls, P.MODE_EESD, 3, use_graph=True)
    b = _run(P, w, Wg, prompt, calls, P.MODE_EESD, 3, use_graph=False)
    for r in (a, b):
        assert r["tokens"] == toks and r["drafts"] == [-1] + compared
        for got, want in zip(r["stats"], snaps):
            for k, v in want.items():
                assert got[k] == v, k
    assert torch.equal(a["logits"], b["logits"])
    assert toks == O.greedy_decode(dec, prompt, sum(calls) + 1).tokens


def test_all_accept_and_never_accept_limits(P):
    w = S.WORKLOADS["C1"].replace(damp=0.0, decode_len=33)
    W = S.make_weights(w)
    prompt = S.make_prompt(w)
    Wg = to_device(W, "cuda")
    r = _run(P, w, Wg, prompt, [33], P.MODE_EESD, 3)
    st = r["stats"][-1]
    # nine rounds of three accepted drafts; the last one is cut after its first token
    assert st["rejected"] == 0 and st["eesd_rounds"] == 9 and st["accepted"] == 27 == st["drafts_compared"]
    W2 = dict(W)
    W2["exit_head"] = -W["lm_head"]
    r2 = _run(P, w, to_device(W2, "cuda"), prompt, [20], P.MODE_EESD, 3)
    st = r2["stats"][-1]
    assert st["accepted"] == 0 and st["eesd_rounds"] == 20 == st["rejected"] == st["drafts_compared"]
    assert r2["tokens"] == r["tokens"][:21]


def test_column_slabs_of_the_down_projection(P):
    """d_ffn so large that four staged input vectors exceed a slab: the down-projection of the batched
    pass walks column slabs inside one launch, keeping each row's sums in registers, so per token the
    products are still added in the single-token kernel's order: logits bitwise equal to vanilla mode.
    d_ffn 4360 (two slabs, ragged last column block) and 9000 (three)."""
    for dtype, tol, f in (("fp32", REL_TOL_FP32, 4360), ("bf16", REL_TOL_BF16, 4360), ("bf16", REL_TOL_BF16, 9000)):
        w = S.Workload("slab", n_layers=3, exit_layer=1, d_model=128, n_heads=2, n_kv_heads=1, head_dim=64, d_ffn=f,
                       vocab=331, dtype=dtype, damp=0.1, seed=41, prompt_len=4, decode_len=24)
        W = S.make_weights(w)
        prompt = S.make_prompt(w)
        Wg = to_device(W, "cuda")
        r = _run(P, w, Wg, prompt, [w.decode_len], P.MODE_EESD, 3)
        check_against_teacher_forced_oracle(O.Decoder(w, W), prompt, r["tokens"], r["logits"], tol)
        assert r["stats"][-1]["committed"] == w.decode_len
        v = _run(P, w, Wg, prompt, [w.decode_len], P.MODE_VANILLA)
        assert v["tokens"] == r["tokens"] and torch.equal(v["logits"], r["logits"])


def test_bf16_ragged_gqa_shapes(P):
    shapes = [
        S.Workload("r16", n_layers=4, exit_layer=2, d_model=256, n_heads=4, n_kv_heads=1, head_dim=128, d_ffn=712,
                   vocab=777, dtype="bf16", damp=0.1, seed=12, prompt_len=21, decode_len=40),
        S.Workload("m16", n_layers=3, exit_layer=2, d_model=128, n_heads=2, n_kv_heads=2, head_dim=64, d_ffn=264,
                   vocab=515, dtype="bf16", damp=0.1, seed=13, prompt_len=5, decode_len=30),
    ]
    for w in shapes:
        W = S.make_weights(w)
        prompt = S.make_prompt(w)
        Wg = to_device(W, "cuda")
        for gamma in (2, 4):
            a = _run(P, w, Wg, prompt, [w.decode_len], P.MODE_EESD, gamma, kv_page_tokens=8)
            v = _run(P, w, Wg, prompt, [w.decode_len], P.MODE_VANILLA, kv_page_tokens=8)
            assert a["tokens"] == v["tokens"] and torch.equal(a["logits"], v["logits"])
            check_against_teacher_forced_oracle(O.Decoder(w, W), prompt, a["tokens"], a["logits"], REL_TOL_BF16)


def test_long_context_with_attention_splits(P):
    w = S.Workload("ctx", n_layers=2, exit_layer=1, d_model=128, n_heads=4, n_kv_heads=1, head_dim=64, d_ffn=256,
                   vocab=300, dtype="fp32", damp=0.1, seed=21, prompt_len=333, decode_len=24)
    W = S.make_weights(w)
    prompt = S.make_prompt(w)
    dec, toks, compared, snaps = _oracle(w, W, prompt, [24], 3)
    r = _run(P, w, to_device(W, "cuda"), prompt, [24], P.MODE_EESD, 3, max_seq=700, tune_attn_split=64,
             page_table=S.page_permutation(5, (700 + 15) // 16))
    assert r["tokens"] == toks and r["drafts"] == [-1] + compared


def test_capacity_and_configuration_errors(P):
    w = SHAPES[1]
    Wg = to_device(S.make_weights(w), "cuda")
    prompt = S.make_prompt(w)
    n, gamma = 10, 3
    fits = len(prompt) + 1 + n + gamma
    ok = _run(P, w, Wg, prompt, [n], P.MODE_EESD, gamma, max_seq=fits)
    assert len(ok["tokens"]) == n + 1
    ss = P.Session(w, Wg, max_seq=fits - 1, mode=P.MODE_EESD, eesd_gamma=gamma)
    ss.ppsd_prefill(prompt)
    with pytest.raises(P.PpsdError) as e:
        ss.ppsd_decode(n)
    assert e.value.code == -3
    ss.close()
    with pytest.raises(P.PpsdError):
        P.Session(w, Wg, max_seq=64, mode=P.MODE_EESD, eesd_gamma=5)
    with pytest.raises(P.PpsdError):
        P.Session(w, Wg, max_seq=64, mode=P.MODE_EESD, engine=P.ENGINE_PERSISTENT)


def test_full_size_7b_rounds_under_the_teacher_forced_protocol(P):
    """C2 (7B bf16, E = 8), three drafts per round; the down-projection runs in three column slabs, so the
    logits differ from vanilla mode's by rounding order and are held to the oracle instead."""
    w = S.WORKLOADS["C2"]
    n = 40
    Wg = S.make_weights(w, device="cuda")
    prompt = S.make_prompt(w)
    r = _run(P, w, Wg, prompt, [n], P.MODE_EESD, 3)
    v = _run(P, w, Wg, prompt, [n], P.MODE_VANILLA)
    st = r["stats"][-1]
    assert st["committed"] == n and st["eesd_rounds"] < n and st["accepted"] > 0
    scale = v["logits"].abs().max(dim=1).values
    same = 0
    while same <= n and r["tokens"][same] == v["tokens"][same]:
        same += 1
    assert same >= 2
    assert ((r["logits"][:same] - v["logits"][:same]).abs().max(dim=1).values / scale[:same]).max().item() < 2e-3
    W = {k: ([t.cpu() for t in x] if isinstance(x, list) else x.cpu()) for k, x in Wg.items()}
    del Wg
    torch.cuda.empty_cache()
    worst, loose = check_against_teacher_forced_oracle(O.Decoder(w, W), prompt, r["tokens"], r["logits"], REL_TOL_BF16)
    print(f"C2 draft-then-verify: max relative logit error {worst:.3e}; {loose} positions inside the margin; "
          f"{st['eesd_rounds']} rounds, accepted {st['accepted']}")
