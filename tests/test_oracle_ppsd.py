"""Pins for the verify-while-draft schedule: losslessness and acceptance accounting."""
import torch

import synth_inputs as S
from oracle import decoder_fp64 as O
from oracle import ppsd_schedule as P


def _run(w, W=None, n=None, prompt=None):
    W = S.make_weights(w) if W is None else W
    dec = O.Decoder(w, W)
    prompt = S.make_prompt(w) if prompt is None else prompt
    n = w.decode_len if n is None else n
    ss = P.prefill(dec, prompt, len(prompt) + n + 2)
    toks = [ss.last_token] + P.decode(ss, n)
    return dec, prompt, toks, ss


def test_lossless_for_any_exit_layer_and_head(tiny_shape):
    for E in (1, 2):
        for head in ("tied", "independent"):
            w = tiny_shape.replace(exit_layer=E, exit_head=head)
            dec, prompt, toks, ss = _run(w)
            assert toks == O.greedy_decode_no_cache(dec, prompt, w.decode_len + 1)
            st = ss.stats
            assert st.committed == w.decode_len == st.accepted + st.rejected == st.drafts_compared
            assert st.steps_overlapped == st.committed and st.kv_rollbacks == st.rejected
            assert st.steps_draft_only == 1 + st.rejected - (0 if ss.full else 1)


def test_lossless_with_adversarial_exit_head(tiny_shape):
    """An exit head that can only ever draft token 0 or 1 (all rows zero except row 0)."""
    w = tiny_shape
    W = S.make_weights(w)
    W["exit_head"].zero_(); W["exit_head"][0] = 1.0
    dec, prompt, toks, ss = _run(w, W)
    want = O.greedy_decode(dec, prompt, w.decode_len + 1).tokens
    assert toks == want
    st = ss.stats
    assert st.accepted + st.rejected == w.decode_len
    assert st.accepted <= sum(1 for t in want[1:] if t in (0, 1))
    assert st.rejected >= 1


def test_damp_zero_with_tied_head_accepts_everything(tiny_shape):
    w = tiny_shape.replace(damp=0.0, exit_head="tied")
    dec, prompt, toks, ss = _run(w)
    st = ss.stats
    assert st.rejected == 0 and st.accepted == w.decode_len
    assert st.steps_draft_only == 1 and st.steps_overlapped == w.decode_len and st.kv_rollbacks == 0
    assert st.acceptance == 1.0
    assert toks == O.greedy_decode(dec, prompt, w.decode_len + 1).tokens


def test_always_missing_head_refills_every_token(tiny_shape):
    """Exit head = negated LM head drafts the LEAST likely token: never accepted."""
    w = tiny_shape
    W = S.make_weights(w.replace(damp=0.0))
    W["exit_head"] = -W["lm_head"]
    dec, prompt, toks, ss = _run(w, W)
    st = ss.stats
    assert st.accepted == 0 and st.rejected == w.decode_len == st.kv_rollbacks
    assert st.steps_draft_only == w.decode_len and not ss.full
    assert toks == O.greedy_decode(dec, prompt, w.decode_len + 1).tokens


def test_decode_is_resumable(tiny_shape):
    w = tiny_shape
    dec = O.Decoder(w, S.make_weights(w))
    prompt = S.make_prompt(w)
    a = P.prefill(dec, prompt, 40)
    one = P.decode(a, 12)
    b = P.prefill(dec, prompt, 40)
    two = P.decode(b, 5) + P.decode(b, 7)
    assert one == two and a.stats == b.stats


def test_acceptance_counts_match_gold_prefix_definition(tiny_shape):
    """alpha = share of positions where the exit head's greedy token, computed on the TRUE prefix,
    equals the full model's greedy token (draft length 1, Sec. 3.1) -- except that a draft made
    from a rejected draft is never compared."""
    w = tiny_shape.replace(exit_layer=2, damp=0.15)
    dec, prompt, toks, ss = _run(w)
    seq = list(prompt) + toks
    ex = dec.exit_logits_full(seq[:-1])
    agree = [O.argmax_lowest(ex[len(prompt) + k]) == toks[k + 1] for k in range(w.decode_len)]
    assert ss.stats.accepted == sum(agree)
    assert 0 < ss.stats.accepted < w.decode_len      # the case exercises both branches


def test_rollback_is_needed_for_losslessness(tiny_shape):
    """Planted mistake: without dropping the rejected draft's KV row the append check trips."""
    w = tiny_shape
    W = S.make_weights(w.replace(damp=0.0)); W["exit_head"] = -W["lm_head"]
    dec = O.Decoder(w, W)
    ss = P.prefill(dec, S.make_prompt(w), 40)
    real_truncate = ss.kv.truncate
    ss.kv.truncate = lambda layers, n: None
    try:
        P.decode(ss, 3)
        raised = False
    except AssertionError:
        raised = True
    assert raised
