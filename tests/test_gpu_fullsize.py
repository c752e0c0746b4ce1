"""GPU parity at the sizes the large workloads really run: widths, context lengths, attention split counts and
prefill chunking as bench.py times them, with only the depth (and, for the 8B shape, the vocabulary) cut so
that the fp64 oracle finishes a whole-sequence pass in about a minute.

Output of the method must equal autoregressive decoding of the full model (Sec. 5.1, "Evaluation Metrics");
the granularity cases follow Sec. 5.4 (pipeline granularity: exit layer 4, 8, 16 of 32)."""
import pytest
import torch

import synth_inputs as S
from oracle import decoder_fp64 as O
from tests.parity_util import REL_TOL_BF16, REL_TOL_FP32, check_against_teacher_forced_oracle

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def P():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU (torch.cuda.is_available() is False)")
    import paper_2509_19368_amd as pkg
    pkg.load_library()
    return pkg


def _session_run(P, w, Wg, prompt, n, mode, max_seq, **kw):
    ss = P.Session(w, Wg, max_seq=max_seq, mode=mode, debug_logits=n + 1, **kw)
    info = ss.launch_info()
    toks = [ss.ppsd_prefill(prompt)] + ss.ppsd_decode(n)
    out = dict(tokens=toks, logits=ss.read_logits(0, n + 1), drafts=ss.read_drafts(0, n + 1), stats=ss.ppsd_stats(),
               info=info)
    ss.close()
    return out


def _to_cpu(Wg):
    return {k: ([t.cpu() for t in v] if isinstance(v, list) else v.cpu()) for k, v in Wg.items()}


def _common_prefix(a, b):
    k = 0
    while k < len(a) and k < len(b) and a[k] == b[k]:
        k += 1
    return k


# Workload C5's widths (Llama-3-8B: d 4096, 32 query / 8 KV heads x 128, FFN 14336, rotary base 5e5) and its
# context (prompt 8192, capacity as bench.py sets it), two layers, vocabulary 4096.
C5W = S.WORKLOADS["C5"].replace(name="C5w", n_layers=2, exit_layer=1, vocab=4096, damp=0.3, decode_len=8)
C5_MAX_SEQ = 8192 + 1 + 512 + 4          # bench.py: prompt + token #0 + decode length + speculative positions


def test_c5_widths_at_8192_positions_bf16(P):
    """The long-context path as timed: k_attn<bf16, 128, 4> over 8.2k positions in 32 splits (one per compute unit
    and KV head), the MFMA prefill in two chunks of 4096 positions (k_pf_flash<4> over a second chunk that attends
    to the first through the KV pages).  Teacher-forced bf16 protocol against the fp64 oracle's whole-sequence
    pass; the two-stage schedule bitwise equal to vanilla mode; the looped prefill (decode kernels over all 8192
    positions) within 2e-3 of the MFMA prefill on the common prefix."""
    w, n = C5W, C5W.decode_len
    Wg = S.make_weights(w, device="cuda")
    prompt = S.make_prompt(w)
    a = _session_run(P, w, Wg, prompt, n, P.MODE_OVERLAP, C5_MAX_SEQ)
    assert a["info"]["attn_splits"] == a["info"]["compute_units"] // w.n_kv_heads >= 16
    assert a["info"]["prefill_matrix_core"] == 1 and a["info"]["prefill_chunk"] == 4096
    v = _session_run(P, w, Wg, prompt, n, P.MODE_VANILLA, C5_MAX_SEQ)
    assert v["tokens"] == a["tokens"] and torch.equal(v["logits"], a["logits"])
    lp = _session_run(P, w, Wg, prompt, n, P.MODE_VANILLA, C5_MAX_SEQ, prefill_loop=True)
    same = _common_prefix(lp["tokens"], v["tokens"])
    assert same >= 1
    scale = v["logits"].abs().max(dim=1).values
    assert ((lp["logits"] - v["logits"]).abs().max(dim=1).values / scale)[:same].max().item() < 2e-3
    dec = O.Decoder(w, _to_cpu(Wg))
    del Wg
    torch.cuda.empty_cache()
    worst, loose = check_against_teacher_forced_oracle(dec, prompt, a["tokens"], a["logits"], REL_TOL_BF16)
    print(f"C5 widths, 8192-token prompt, bf16: max relative logit error {worst:.3e}; {loose} of {n + 1} positions inside "
          f"the margin; {a['info']['attn_splits']} attention splits; looped and MFMA prefill agree on {same} tokens")
    if same <= n:      # the looped-prefill stream left the other at a near-tie: it must pass the protocol on its own
        check_against_teacher_forced_oracle(dec, prompt, lp["tokens"], lp["logits"], REL_TOL_BF16)


def test_c5_widths_at_8192_positions_fp32_storage(P):
    """Same widths and context with fp32 weights and KV cache (k_attn<float, 128, 4>, 32 splits, looped prefill):
    the kernels' arithmetic without bf16 storage rounding.  Exact oracle stream, logits within 2e-5."""
    w, n = C5W.replace(name="C5w32", dtype="fp32"), 6
    Wg = S.make_weights(w, device="cuda")
    prompt = S.make_prompt(w)
    a = _session_run(P, w, Wg, prompt, n, P.MODE_OVERLAP, C5_MAX_SEQ)
    assert a["info"]["attn_splits"] == a["info"]["compute_units"] // w.n_kv_heads and a["info"]["prefill_matrix_core"] == 0
    dec = O.Decoder(w, _to_cpu(Wg))
    del Wg
    torch.cuda.empty_cache()
    ref = dec.logits_full(list(prompt) + a["tokens"][:-1])[len(prompt) - 1:]
    assert a["tokens"] == [O.argmax_lowest(r) for r in ref]
    err = ((a["logits"].double() - ref).abs().max(dim=1).values / ref.abs().max(dim=1).values).max().item()
    print(f"C5 widths, 8192-token prompt, fp32 storage: max relative logit error {err:.3e}")
    assert err <= REL_TOL_FP32


# Workload C4's widths (Llama-2-13B: d 5120, 40 heads x 128, FFN 13824, vocabulary 32000) and its prompt of 512.
C4W = S.WORKLOADS["C4"].replace(name="C4w", n_layers=2, exit_layer=1, damp=0.3, decode_len=8)
C4_MAX_SEQ = 512 + 1 + 512 + 4


def test_c4_widths_with_the_512_token_prompt(P):
    """The 13B widths with the workload's own prompt length: the MFMA prefill's 256 x 256 tiles at d_model 5120 over
    512 positions (one chunk), decode attention with two splits (capacity 1029).  bf16: teacher-forced protocol,
    two-stage bitwise equal to vanilla; fp32 storage: exact oracle stream, logits within 2e-5."""
    n = C4W.decode_len
    for w in (C4W, C4W.replace(name="C4w32", dtype="fp32")):
        Wg = S.make_weights(w, device="cuda")
        prompt = S.make_prompt(w)
        a = _session_run(P, w, Wg, prompt, n, P.MODE_OVERLAP, C4_MAX_SEQ)
        v = _session_run(P, w, Wg, prompt, n, P.MODE_VANILLA, C4_MAX_SEQ)
        assert v["tokens"] == a["tokens"] and torch.equal(v["logits"], a["logits"])
        assert a["info"]["prefill_matrix_core"] == (1 if w.dtype == "bf16" else 0) and a["info"]["attn_splits"] >= 2
        if w.dtype == "bf16":
            # the down projection walks its 13824 input columns in two slabs here (640 workgroups would not be resident
            # with the whole vector staged); a draft stage throttled to 10 % and 1 % of its workgroups gives every wave
            # several rows per round and several rounds: same bits
            for share in (10, 1):
                t = _session_run(P, w, Wg, prompt, n, P.MODE_OVERLAP, C4_MAX_SEQ, tune_draft_share=share)
                assert t["tokens"] == v["tokens"] and torch.equal(t["logits"], v["logits"]), share
            del t
            dec = O.Decoder(w, _to_cpu(Wg))
            del Wg
            torch.cuda.empty_cache()
            worst, loose = check_against_teacher_forced_oracle(dec, prompt, a["tokens"], a["logits"], REL_TOL_BF16)
            print(f"C4 widths, prompt 512, bf16: max relative logit error {worst:.3e}; {loose} positions inside the margin")
        else:
            dec = O.Decoder(w, _to_cpu(Wg))
            del Wg
            torch.cuda.empty_cache()
            ref = dec.logits_full(list(prompt) + a["tokens"][:-1])[len(prompt) - 1:]
            assert a["tokens"] == [O.argmax_lowest(r) for r in ref]
            err = ((a["logits"].double() - ref).abs().max(dim=1).values / ref.abs().max(dim=1).values).max().item()
            print(f"C4 widths, prompt 512, fp32 storage: max relative logit error {err:.3e}")
            assert err <= REL_TOL_FP32


@pytest.mark.parametrize("cell", ["C3_E4_a70", "C3_E16_a70"])
def test_c3_grid_cells_full_size_pipeline_and_two_stage_equal_vanilla(P, cell):
    """The 7B shape at the other two granularities of the exit-layer grid (E = 4: eight stages, E = 16: two), full
    depth, the grid's prompt of 256: the S-stage and the two-stage schedule must commit vanilla mode's tokens and
    logits bit for bit, the tick count must be Eq. (7)'s (one tick per accepted token, S per rejected one), and
    vanilla mode must pass the oracle protocol at this prompt length."""
    w = {c.name: c for c in S.c3_grid()}[cell]
    n = 40
    S_ = -(-w.n_layers // w.exit_layer)
    max_seq = w.prompt_len + 1 + w.decode_len + max(1, S_ - 1)
    Wg = S.make_weights(w, device="cuda")
    prompt = S.make_prompt(w)
    v = _session_run(P, w, Wg, prompt, n, P.MODE_VANILLA, max_seq)
    p = _session_run(P, w, Wg, prompt, n, P.MODE_PIPELINE, max_seq)
    o = _session_run(P, w, Wg, prompt, n, P.MODE_OVERLAP, max_seq)
    for r in (p, o):
        assert r["tokens"] == v["tokens"] and torch.equal(r["logits"], v["logits"])
    st = p["stats"]
    assert p["info"]["pipeline_stages"] == S_ and p["info"]["streams"] == min(S_, 4)
    rej_before_last = sum(1 for k in range(1, n) if p["drafts"][k] != p["tokens"][k])
    assert st["pipeline_ticks"] == (S_ - 1) + n + (S_ - 1) * rej_before_last
    assert st["flushed_tokens"] == (S_ - 1) * st["rejected"] and st["committed"] == n
    assert st["accepted"] == o["stats"]["accepted"] and p["drafts"] == o["drafts"]     # same drafts meet the same tokens
    assert 0 < st["rejected"] < n
    if cell == "C3_E4_a70":          # one oracle pass for the shape at prompt 256 (vanilla does not depend on E)
        dec = O.Decoder(w, _to_cpu(Wg))
        del Wg
        torch.cuda.empty_cache()
        k = 12
        worst, loose = check_against_teacher_forced_oracle(dec, prompt, v["tokens"][:k + 1], v["logits"][:k + 1], REL_TOL_BF16)
        print(f"{cell}: max relative logit error {worst:.3e} over {k + 1} positions; rejected {st['rejected']} of {n}")
