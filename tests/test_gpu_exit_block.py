"""GPU parity with the transformer-layer early-exit head (Sec. 5.4, "Impact of exit head") in every schedule."""
import pytest
import torch

import synth_inputs as S
from oracle import decoder_fp64 as O
from oracle import eesd_schedule as EE
from oracle import ppsd_schedule as SCH
from tests.parity_util import REL_TOL_BF16, check_against_teacher_forced_oracle, to_device

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def P():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU (torch.cuda.is_available() is False)")
    import paper_2509_19368_amd as pkg
    pkg.load_library()
    return pkg


SHAPES = [
    S.WORKLOADS["C1"].replace(name="C1xb", exit_block=True, exit_block_damp=0.5, damp=0.3),
    S.Workload("x7", n_layers=7, exit_layer=2, d_model=128, n_heads=2, n_kv_heads=2, head_dim=64, d_ffn=264,
               vocab=515, dtype="fp32", damp=0.15, seed=21, prompt_len=6, decode_len=40, exit_block=True,
               exit_block_damp=0.5),
    S.Workload("x5", n_layers=5, exit_layer=3, d_model=256, n_heads=2, n_kv_heads=1, head_dim=128, d_ffn=512,
               vocab=640, dtype="fp32", damp=0.25, seed=23, prompt_len=3, decode_len=40, exit_block=True,
               exit_block_damp=0.25),
]


def _run(P, w, Wg, prompt, n, mode, **kw):
    S_ = -(-w.n_layers // w.exit_layer)
    ss = P.Session(w, Wg, max_seq=len(prompt) + 1 + n + max(S_, 4), mode=mode, debug_logits=n + 1, **kw)
    toks = [ss.ppsd_prefill(prompt)] + ss.ppsd_decode(n)
    out = dict(tokens=toks, logits=ss.read_logits(0, n + 1), drafts=ss.read_drafts(0, n + 1), stats=ss.ppsd_stats())
    ss.close()
    return out


@pytest.mark.parametrize("w", SHAPES, ids=[w.name for w in SHAPES])
def test_every_schedule_equals_its_simulator_with_the_block(P, w):
    W = S.make_weights(w)
    prompt = S.make_prompt(w)
    n = w.decode_len
    dec = O.Decoder(w, W)
    Wg = to_device(W, "cuda")
    gold = O.greedy_decode(dec, prompt, n + 1).tokens
    # two-stage schedule
    ss = SCH.prefill(dec, prompt, len(prompt) + n + 2)
    toks = [ss.last_token] + SCH.decode(ss, n)
    assert toks == gold
    for mode in (P.MODE_SERIAL, P.MODE_OVERLAP):
        r = _run(P, w, Wg, prompt, n, mode)
        assert r["tokens"] == gold
        st = r["stats"]
        assert (st["accepted"], st["rejected"], st["steps_draft_only"]) == \
               (ss.stats.accepted, ss.stats.rejected, ss.stats.steps_draft_only)
        ex = dec.exit_logits_full((list(prompt) + gold)[:-1])
        for k in range(1, n + 1):
            assert r["drafts"][k] == O.argmax_lowest(ex[len(prompt) + k - 1])
    assert 0 < ss.stats.rejected < n, "the case must exercise both outcomes"
    # full pipeline schedule
    ps = SCH.pipeline_prefill(dec, prompt, len(prompt) + n + 20)
    ptoks = [ps.last_token] + SCH.pipeline_decode(ps, n)
    r = _run(P, w, Wg, prompt, n, P.MODE_PIPELINE)
    assert r["tokens"] == ptoks == gold and r["drafts"] == [-1] + ps.compared
    assert (r["stats"]["pipeline_ticks"], r["stats"]["stage_runs"], r["stats"]["rejected"]) == \
           (ps.stats.ticks, ps.stats.stage_runs, ps.stats.rejected)
    # draft-then-verify rounds
    es = EE.eesd_prefill(dec, prompt, len(prompt) + n + 8, 3)
    etoks = [es.last_token] + EE.eesd_decode(es, n)
    r = _run(P, w, Wg, prompt, n, P.MODE_EESD, eesd_gamma=3)
    assert r["tokens"] == etoks == gold and r["drafts"] == [-1] + es.compared
    assert (r["stats"]["eesd_rounds"], r["stats"]["accepted"], r["stats"]["rejected"]) == \
           (es.stats.rounds, es.stats.accepted, es.stats.rejected)


def test_identity_block_drafts_what_the_norm_head_drafts(P):
    w0 = S.WORKLOADS["C1"]
    w1 = w0.replace(exit_block=True, exit_block_damp=0.0)
    prompt = S.make_prompt(w0)
    a = _run(P, w0, to_device(S.make_weights(w0), "cuda"), prompt, 48, P.MODE_OVERLAP)
    b = _run(P, w1, to_device(S.make_weights(w1), "cuda"), prompt, 48, P.MODE_OVERLAP)
    assert a["tokens"] == b["tokens"] and a["drafts"] == b["drafts"] and torch.equal(a["logits"], b["logits"])


def test_block_with_matrix_core_prefill_and_bf16(P):
    """bf16, head_dim 128: the prompt goes through the MFMA prefill, which must also append the block's
    K/V rows; the looped prefill is the cross-check, the oracle the reference."""
    w = S.Workload("xpf", n_layers=3, exit_layer=1, d_model=256, n_heads=2, n_kv_heads=1, head_dim=128, d_ffn=704,
                   vocab=777, dtype="bf16", damp=0.2, seed=31, prompt_len=200, decode_len=24, exit_block=True,
                   exit_block_damp=0.5)
    W = S.make_weights(w)
    prompt = S.make_prompt(w)
    dec = O.Decoder(w, W)
    Wg = to_device(W, "cuda")
    a = _run(P, w, Wg, prompt, 24, P.MODE_OVERLAP, prefill_loop=False)
    b = _run(P, w, Wg, prompt, 24, P.MODE_OVERLAP, prefill_loop=True)
    for r in (a, b):
        check_against_teacher_forced_oracle(dec, prompt, r["tokens"], r["logits"], REL_TOL_BF16)
        assert r["stats"]["accepted"] > 0
    # the drafts are made by the block on rows both prefill paths wrote: where the streams agree the
    # drafts must agree as well, up to a near-tie in the exit head
    same = 0
    while same <= 24 and a["tokens"][same] == b["tokens"][same]:
        same += 1
    agree = sum(1 for k in range(1, same) if a["drafts"][k] == b["drafts"][k])
    assert same >= 8 and agree >= (same - 1) - 2
    # and they are the block's drafts: the oracle's whole-sequence forward through the block, teacher-forced
    ex = dec.exit_logits_full((list(prompt) + a["tokens"])[:-1])
    hits = 0
    for k in range(1, 25):
        top = torch.topk(ex[len(prompt) + k - 1], 2).indices.tolist()
        hits += a["drafts"][k] in top
    assert hits >= 23
