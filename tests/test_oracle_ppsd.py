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


# ------------------------------------------------------------------ full ceil(N/E)-stage schedule
def _pipeline(w, W=None, n=None, later=None):
    W = S.make_weights(w) if W is None else W
    dec = O.Decoder(w, W)
    prompt = S.make_prompt(w)
    n = w.decode_len if n is None else n
    ss = P.pipeline_prefill(dec, prompt, len(prompt) + n + 8, later)
    committed = []
    reject_at = []
    while len(committed) < n:
        before = ss.stats.rejected
        P.pipeline_tick(ss, committed)
        if ss.stats.rejected > before:
            reject_at.append(len(committed) - 1)
    return dec, prompt, [ss_first(dec, prompt)] + committed, ss, reject_at


def ss_first(dec, prompt):
    return O.argmax_lowest(dec.logits_full(list(prompt))[-1])


def test_stage_partition_follows_the_paper():
    assert [list(r) for r in P.stage_ranges(8, 3)] == [[0, 1, 2], [3, 4, 5], [6, 7]]     # remainder = own stage
    assert len(P.stage_ranges(32, 8)) == 4 and len(P.stage_ranges(32, 12)) == 3
    assert [len(r) for r in P.stage_ranges(40, 10)] == [10, 10, 10, 10]


def test_later_stages_of_another_size_keep_the_draft_stage_at_the_exit_layer():
    assert [list(r) for r in P.stage_ranges(8, 2, 3)] == [[0, 1], [2, 3, 4], [5, 6, 7]]
    assert [len(r) for r in P.stage_ranges(32, 8, 12)] == [8, 12, 12]
    assert [len(r) for r in P.stage_ranges(32, 8, 24)] == [8, 24]                    # the two-stage schedule
    assert [len(r) for r in P.stage_ranges(40, 10, 16)] == [10, 16, 14]              # the last takes what remains
    assert [list(r) for r in P.stage_ranges(8, 3, 3)] == [list(r) for r in P.stage_ranges(8, 3)]
    for n, e, w in ((32, 8, 12), (7, 2, 4), (9, 1, 3)):
        flat = [l for r in P.stage_ranges(n, e, w) for l in r]
        assert flat == list(range(n))                                                # every layer once, in order


def test_unequal_partitions_are_lossless_and_cost_one_tick_per_stage_on_a_rejection(tiny_shape):
    """Any partition whose first stage is the draft model commits the full model's greedy stream; the drafts
    that meet their check token and the acceptances are those of every other schedule (they depend on the exit
    head and the gold prefix only); ticks follow Eq. (7)'s cost model with S = the partition's stage count."""
    base = tiny_shape.replace(n_layers=7, decode_len=22, damp=0.2)
    for E, later in ((2, 3), (2, 5), (1, 2), (3, 2), (1, 6)):
        w = base.replace(exit_layer=E)
        dec, prompt, toks, ss, reject_at = _pipeline(w, later=later)
        Sg = len(P.stage_ranges(w.n_layers, E, later))
        assert Sg == 1 + -(-(w.n_layers - E) // later)
        assert toks == O.greedy_decode_no_cache(dec, prompt, w.decode_len + 1), (E, later)
        paid = sum(1 for k in reject_at if k < w.decode_len - 1)
        assert ss.stats.ticks == (Sg - 1) + w.decode_len + (Sg - 1) * paid
        assert ss.stats.flushed_tokens == (Sg - 1) * ss.stats.rejected
        _, _, toks_e, se, _ = _pipeline(w)                       # the paper's partition: E layers per stage
        assert toks_e == toks and se.compared == ss.compared
        assert (se.stats.accepted, se.stats.rejected) == (ss.stats.accepted, ss.stats.rejected)
    # later stage = everything behind the exit layer: the two-stage schedule, step for step
    w = base.replace(exit_layer=3)
    dec = O.Decoder(w, S.make_weights(w))
    prompt = S.make_prompt(w)
    a = P.prefill(dec, prompt, 60)
    ta = P.decode(a, 22)
    b = P.pipeline_prefill(dec, prompt, 60, w.n_layers - 3)
    assert P.pipeline_decode(b, 22) == ta
    assert b.stats.ticks == a.stats.steps_overlapped + a.stats.steps_draft_only


def test_pipeline_schedule_is_lossless_for_every_granularity(tiny_shape):
    base = tiny_shape.replace(n_layers=5, decode_len=18)
    for E in (1, 2, 3, 4):
        for head in ("tied", "independent"):
            w = base.replace(exit_layer=E, exit_head=head)
            dec, prompt, toks, ss, _ = _pipeline(w)
            assert toks == O.greedy_decode_no_cache(dec, prompt, w.decode_len + 1), (E, head)
            st = ss.stats
            assert st.committed == w.decode_len == st.accepted + st.rejected == st.drafts_compared


def test_pipeline_tick_count_is_eq7s_cost_model(tiny_shape):
    """An accepted token costs one tick, a rejected one ceil(N/E) ticks (Eq. (7)); the first token after
    prefill pays the pipeline fill, and the refill of a rejection is paid before the NEXT commit."""
    base = tiny_shape.replace(n_layers=6, decode_len=24, damp=0.2)
    for E in (1, 2, 3, 4):
        w = base.replace(exit_layer=E)
        Sg = -(-w.n_layers // E)
        _, _, _, ss, reject_at = _pipeline(w)
        n = w.decode_len
        paid = sum(1 for k in reject_at if k < n - 1)
        assert ss.stats.ticks == (Sg - 1) + n + (Sg - 1) * paid
        # in the long run: ticks per token -> alpha + (1 - alpha) S, i.e. Eq. (7)'s denominator / E
    w = base.replace(exit_layer=2, damp=0.0)          # every draft right: N/E tokens per N/E ticks
    _, _, _, ss, reject_at = _pipeline(w)
    assert not reject_at and ss.stats.ticks == 2 + w.decode_len
    from oracle import speedup_model as M
    assert (w.n_layers / 2) * w.decode_len / (ss.stats.ticks - 2) == M.ppsd_gain(1.0, 2, w.n_layers)


def test_pipeline_with_two_stages_equals_the_two_stage_schedule(tiny_shape):
    w = tiny_shape.replace(n_layers=4, exit_layer=2, decode_len=20)
    dec = O.Decoder(w, S.make_weights(w))
    prompt = S.make_prompt(w)
    a = P.prefill(dec, prompt, 40)
    ta = P.decode(a, 20)
    b = P.pipeline_prefill(dec, prompt, 40)
    tb = P.pipeline_decode(b, 20)
    assert ta == tb
    assert (a.stats.accepted, a.stats.rejected) == (b.stats.accepted, b.stats.rejected)
    assert b.stats.ticks == a.stats.steps_overlapped + a.stats.steps_draft_only


def test_pipeline_acceptance_equals_the_gold_prefix_rate(tiny_shape):
    """Chained drafts do not change what is compared: a draft reaches its check only if every
    draft before it was right, so it was computed on the true prefix (Sec. 5.3, acceptance at gamma = 1)."""
    w = tiny_shape.replace(n_layers=6, exit_layer=2, decode_len=24, damp=0.15)
    dec, prompt, toks, ss, _ = _pipeline(w)
    ex = dec.exit_logits_full((list(prompt) + toks)[:-1])
    agree = [O.argmax_lowest(ex[len(prompt) + k]) == toks[k + 1] for k in range(w.decode_len)]
    assert ss.stats.accepted == sum(agree) and 0 < sum(agree) < w.decode_len
    assert ss.stats.flushed_tokens >= ss.stats.rejected


def test_pipeline_always_missing_head_degenerates_to_autoregressive_speed(tiny_shape):
    w = tiny_shape.replace(n_layers=6, exit_layer=2, decode_len=10)
    W = S.make_weights(w.replace(damp=0.0)); W["exit_head"] = -W["lm_head"]
    dec, prompt, toks, ss, _ = _pipeline(w, W)
    assert ss.stats.accepted == 0 and toks == O.greedy_decode(dec, prompt, 11).tokens
    assert ss.stats.ticks == 3 * 10                   # S ticks per token: Eq. (7) at alpha = 0 gives 1
