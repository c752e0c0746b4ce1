"""ppsd_decode_static_scratch (per-step scratch in the library's static device array, no allocation in the
call) against ppsd_decode through the C ABI: same tokens, logits, drafts and counters, bit for bit."""
import pytest
import torch

import synth_inputs as S
from oracle import decoder_fp64 as O

pytestmark = pytest.mark.gpu

BIG = S.Workload("za", n_layers=4, exit_layer=1, d_model=256, n_heads=4, n_kv_heads=4, head_dim=64, d_ffn=688,
                 vocab=2048, dtype="fp32", damp=0.1, seed=41, prompt_len=16, decode_len=40)
GQA = S.Workload("zb", n_layers=4, exit_layer=2, d_model=256, n_heads=4, n_kv_heads=1, head_dim=128, d_ffn=712,
                 vocab=777, dtype="bf16", damp=0.2, seed=42, prompt_len=21, decode_len=24)
SMALLER = S.Workload("zc", n_layers=3, exit_layer=2, d_model=128, n_heads=2, n_kv_heads=2, head_dim=64, d_ffn=264,
                     vocab=515, dtype="fp32", damp=0.3, seed=43, prompt_len=5, decode_len=12)
COUNTERS = ("committed", "drafts_compared", "accepted", "rejected", "steps_overlapped", "steps_draft_only",
            "kv_rollbacks", "pipeline_ticks", "stage_runs", "flushed_tokens", "eesd_rounds")


@pytest.fixture(scope="module")
def P():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU (torch.cuda.is_available() is False)")
    import paper_2509_19368_amd as pkg
    pkg.load_library()
    return pkg


def _weights(w):
    W = S.make_weights(w)
    return W, {k: ([t.cuda() for t in v] if isinstance(v, list) else v.cuda()) for k, v in W.items()}


def _run(P, w, Wg, calls, mode, static, **kw):
    """calls: list of (n_tokens, use_static); `static` overrides every entry when not None."""
    n = sum(c[0] for c in calls)
    ss = P.Session(w, Wg, max_seq=w.prompt_len + n + 8, mode=mode, debug_logits=n + 1, **kw)
    toks = [ss.ppsd_prefill(S.make_prompt(w))]
    for k, use_static in calls:
        use = use_static if static is None else static
        toks += ss.ppsd_decode_static_scratch(k) if use else ss.ppsd_decode(k)
    out = dict(tokens=toks, logits=ss.read_logits(0, n + 1), drafts=ss.read_drafts(0, n + 1), stats=ss.ppsd_stats())
    ss.close()
    return out


def _same(a, b):
    assert a["tokens"] == b["tokens"]
    assert a["drafts"] == b["drafts"]
    assert torch.equal(a["logits"], b["logits"])
    for k in COUNTERS:
        assert a["stats"][k] == b["stats"][k], k


def test_two_calls_in_a_row_the_second_smaller_equal_ppsd_decode(P):
    """Call 1: the larger model, 40 tokens.  Call 2, right behind it on the same device array: a smaller
    model and fewer tokens (the array still holds call 1's partials and candidates).  Both must equal
    ppsd_decode's result bit for bit, and the fp32 streams the oracle's."""
    for mode in (P.MODE_OVERLAP, P.MODE_PIPELINE, P.MODE_EESD, P.MODE_VANILLA):
        kw = dict(eesd_gamma=3) if mode == P.MODE_EESD else {}
        for w in (BIG, SMALLER):
            W, Wg = _weights(w)
            got = _run(P, w, Wg, [(w.decode_len, True)], mode, None, **kw)
            want = _run(P, w, Wg, [(w.decode_len, False)], mode, None, **kw)
            _same(got, want)
            ref = O.greedy_decode(O.Decoder(w, W), S.make_prompt(w), w.decode_len + 1).tokens
            assert got["tokens"] == ref, (mode, w.name)


def test_split_attention_and_bf16_gqa(P):
    """Several attention splits (partials and arrival counters live in the static array), bf16 storage, four
    query heads per KV head; the second call reuses the array with fewer splits in play."""
    W, Wg = _weights(GQA)
    for mode in (P.MODE_OVERLAP, P.MODE_EESD):
        for split in (64, 0):
            kw = dict(tune_attn_split=split, kv_page_tokens=8)
            if mode == P.MODE_EESD:
                kw["eesd_gamma"] = 2
            _same(_run(P, GQA, Wg, [(GQA.decode_len, True)], mode, None, **kw),
                  _run(P, GQA, Wg, [(GQA.decode_len, False)], mode, None, **kw))


def test_resumed_and_alternating_calls_on_one_context(P):
    W, Wg = _weights(BIG)
    for mode in (P.MODE_OVERLAP, P.MODE_PIPELINE):
        want = _run(P, BIG, Wg, [(27, False)], mode, None)
        _same(_run(P, BIG, Wg, [(20, True), (7, True)], mode, None), want)
        _same(_run(P, BIG, Wg, [(5, False), (13, True), (9, False)], mode, None), want)
        _same(_run(P, BIG, Wg, [(27, True)], mode, None, use_graph=False), want)


def test_sizes_beyond_the_static_region_and_unsupported_engines_are_rejected(P):
    wide = S.Workload("zw", n_layers=2, exit_layer=1, d_model=256, n_heads=64, n_kv_heads=64, head_dim=128, d_ffn=512,
                      vocab=300, dtype="bf16", damp=0.2, seed=44, prompt_len=3, decode_len=4)
    _, Wg = _weights(wide)
    ss = P.Session(wide, Wg, max_seq=16, mode=P.MODE_EESD)
    t0 = ss.ppsd_prefill(S.make_prompt(wide))
    with pytest.raises(P.PpsdError) as e:
        ss.ppsd_decode_static_scratch(4)
    assert e.value.code == -3 and "static region" in str(e.value)
    rest = ss.ppsd_decode(4)                      # the context is still usable through the workspace path
    ss.close()
    sv = P.Session(wide, Wg, max_seq=16, mode=P.MODE_VANILLA)
    assert [sv.ppsd_prefill(S.make_prompt(wide))] + sv.ppsd_decode_static_scratch(4) == [t0] + rest
    sv.close()
    _, Wb = _weights(BIG)
    sp = P.Session(BIG, Wb, max_seq=40, mode=P.MODE_OVERLAP, engine=P.ENGINE_PERSISTENT)
    sp.ppsd_prefill(S.make_prompt(BIG))
    with pytest.raises(P.PpsdError) as e:
        sp.ppsd_decode_static_scratch(4)
    assert e.value.code == -1
    with pytest.raises(P.PpsdError) as e:
        BIGs = P.Session(BIG, Wb, max_seq=40, mode=P.MODE_OVERLAP)
        BIGs.ppsd_decode_static_scratch(4)       # before prefill
    assert e.value.code == -2
    sp.close()
