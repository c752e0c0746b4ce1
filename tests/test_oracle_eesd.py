"""Pins for the draft-then-verify simulator (Sec. 3.1, Eq. 4-5): losslessness, accept accounting from
gold-prefix quantities, the per-round cost gamma E + N, the all-accept and never-accept limits."""
import math

import pytest

import synth_inputs as S
from oracle import decoder_fp64 as O
from oracle import eesd_schedule as EE
from oracle import speedup_model as M


def _run(w, gamma, W=None, n=None, calls=None):
    W = S.make_weights(w) if W is None else W
    dec = O.Decoder(w, W)
    prompt = S.make_prompt(w)
    n = w.decode_len if n is None else n
    ss = EE.eesd_prefill(dec, prompt, len(prompt) + n + gamma + 2, gamma)
    toks = [ss.last_token]
    for c in (calls or [n]):
        toks += EE.eesd_decode(ss, c)
    return dec, prompt, toks, ss


@pytest.mark.parametrize("gamma", [1, 2, 3, 4])
def test_lossless_for_any_draft_length_exit_layer_and_head(tiny_shape, gamma):
    for E in (1, 2):
        for head in ("tied", "independent"):
            w = tiny_shape.replace(exit_layer=E, exit_head=head, decode_len=14)
            dec, prompt, toks, ss = _run(w, gamma)
            assert toks == O.greedy_decode_no_cache(dec, prompt, w.decode_len + 1)
            assert ss.stats.committed == w.decode_len


def test_round_outcomes_follow_from_gold_prefix_quantities():
    """A round's accepted length is the number of leading positions (at most gamma) where the exit
    head's greedy token on the TRUE prefix equals the true next token: every draft before the first
    mismatch was computed from true tokens only.  Rebuilds rounds, compared drafts and counters from
    whole-sequence forwards (no KV cache, no simulator state)."""
    w = S.Workload("e", n_layers=4, exit_layer=2, d_model=48, n_heads=4, n_kv_heads=2, head_dim=12, d_ffn=80,
                   vocab=96, dtype="fp32", damp=0.25, seed=5, prompt_len=7, decode_len=40)
    for gamma in (1, 3, 4):
        dec, prompt, toks, ss = _run(w, gamma)
        seq = list(prompt) + toks
        ex = dec.exit_logits_full(seq[:-1])
        draft_at = lambda p: O.argmax_lowest(ex[p - 1])       # exit head's token for position p given seq[:p]
        P0 = len(prompt)
        t, rounds, acc, rej, cmp_, committed, compared = P0, 0, 0, 0, 0, 0, []
        while committed < w.decode_len:
            n = 0
            while n < gamma and t + n + 1 < len(seq) and draft_at(t + n + 1) == seq[t + n + 1]:
                n += 1
            # a run cut short by the end of the sequence is a truncated round: the simulator compared
            # further, so only rounds that end inside the sequence are rebuilt exactly
            k = min(n + 1, w.decode_len - committed)
            if t + n + 1 >= len(seq):
                break
            rounds += 1; acc += n; rej += 1 if n < gamma else 0; cmp_ += min(gamma, n + 1)
            compared += [draft_at(t + i + 1) if i < gamma else -1 for i in range(k)]
            committed += k; t += k
        st = ss.stats
        assert ss.compared[:len(compared)] == compared
        if committed == w.decode_len:                            # every round rebuilt
            assert (st.rounds, st.accepted, st.rejected, st.drafts_compared) == (rounds, acc, rej, cmp_)
        assert 0 < st.rejected and st.accepted > 0, "the case must exercise both outcomes"


def test_cost_per_round_is_gamma_E_plus_N(tiny_shape):
    for gamma in (1, 2, 4):
        for E in (1, 2):
            w = tiny_shape.replace(exit_layer=E)
            _, _, _, ss = _run(w, gamma)
            assert ss.stats.layer_reads == ss.stats.rounds * (gamma * E + w.n_layers)


def test_all_accept_limit_commits_gamma_plus_one_per_round(tiny_shape):
    w = tiny_shape.replace(damp=0.0, exit_head="tied", decode_len=13)
    for gamma in (1, 2, 3):
        dec, prompt, toks, ss = _run(w, gamma)
        st = ss.stats
        assert st.rejected == 0 and st.rounds == math.ceil(w.decode_len / (gamma + 1))
        assert toks == O.greedy_decode(dec, prompt, w.decode_len + 1).tokens
        # Eq. (5) at a = 1: (gamma + 1) N / (gamma E + N) tokens per full-model cost, up to the cut last round
        full_rounds = w.decode_len // (gamma + 1)
        gain = (gamma + 1) * full_rounds * w.n_layers / (full_rounds * (gamma * w.exit_layer + w.n_layers))
        assert abs(gain - M.eesd_gain(1.0, gamma, w.exit_layer, w.n_layers)) < 1e-12
        # every gamma+1-th committed token is the full model's own (no draft compared)
        assert [c == -1 for c in ss.compared[: full_rounds * (gamma + 1)]] == \
               [(i % (gamma + 1)) == gamma for i in range(full_rounds * (gamma + 1))]


def test_never_accept_limit_commits_one_per_round(tiny_shape):
    w = tiny_shape
    W = S.make_weights(w.replace(damp=0.0))
    W["exit_head"] = -W["lm_head"]                     # drafts the least likely token
    for gamma in (1, 3):
        dec, prompt, toks, ss = _run(w, gamma, W)
        st = ss.stats
        assert st.accepted == 0 and st.rounds == w.decode_len == st.rejected == st.drafts_compared
        assert toks == O.greedy_decode(dec, prompt, w.decode_len + 1).tokens


def test_gamma_one_commits_what_the_two_stage_schedule_commits(tiny_shape):
    """With one draft per round the compared drafts are the same tokens the verify-while-draft
    schedule compares on accepted runs: both equal the exit head's token on the true prefix."""
    from oracle import ppsd_schedule as P
    w = tiny_shape.replace(decode_len=16)
    W = S.make_weights(w)
    dec, prompt, toks, ss = _run(w, 1, W)
    ps = P.prefill(dec, prompt, len(prompt) + w.decode_len + 2)
    ptoks = [ps.last_token] + P.decode(ps, w.decode_len)
    assert toks == ptoks


def test_resumed_decode_truncates_a_round_and_stays_lossless(tiny_shape):
    w = tiny_shape.replace(damp=0.05, decode_len=15)
    W = S.make_weights(w)
    dec, prompt, toks, ss = _run(w, 3, W, calls=[1, 2, 5, 7])
    assert toks == O.greedy_decode(dec, prompt, w.decode_len + 1).tokens
    assert ss.stats.committed == w.decode_len
    assert ss.kv.len == [ss.t] * w.n_layers          # nothing speculative is left in the cache


def test_a_planted_missing_rollback_is_caught(tiny_shape):
    """Leaving the rejected drafts' KV rows in place trips the append-only check of the next round."""
    w = tiny_shape
    W = S.make_weights(w)
    W["exit_head"] = -W["lm_head"]                     # every round ends at a mismatch and leaves rows behind
    dec = O.Decoder(w, W)
    prompt = S.make_prompt(w)
    ss = EE.eesd_prefill(dec, prompt, 64, 2)
    real = ss.kv.truncate
    ss.kv.truncate = lambda layers, n: None
    out = []
    EE.eesd_round(ss, out, 10)
    with pytest.raises(AssertionError):
        for _ in range(4):
            EE.eesd_round(ss, out, 10)
    ss.kv.truncate = real
