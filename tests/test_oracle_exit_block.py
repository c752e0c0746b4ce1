"""Pins for the transformer-layer early-exit head (Sec. 5.4, "Impact of exit head"): one more layer of
the model's own structure in front of the norm head, used by the draft only."""
import pytest
import torch

import synth_inputs as S
from oracle import decoder_fp64 as O
from oracle import eesd_schedule as EE
from oracle import ppsd_schedule as P


def _two_stage(w, W, n):
    dec = O.Decoder(w, W)
    prompt = S.make_prompt(w)
    ss = P.prefill(dec, prompt, len(prompt) + n + 2)
    return dec, prompt, [ss.last_token] + P.decode(ss, n), ss


def _pipeline(w, W, n):
    dec = O.Decoder(w, W)
    prompt = S.make_prompt(w)
    ss = P.pipeline_prefill(dec, prompt, len(prompt) + n + 8)
    return dec, prompt, [ss.last_token] + P.pipeline_decode(ss, n), ss


def _eesd(w, W, n, gamma=3):
    dec = O.Decoder(w, W)
    prompt = S.make_prompt(w)
    ss = EE.eesd_prefill(dec, prompt, len(prompt) + n + gamma + 2, gamma)
    return dec, prompt, [ss.last_token] + EE.eesd_decode(ss, n), ss


def test_a_block_with_zero_output_projections_is_the_plain_norm_head(tiny_shape):
    """W_o = W_down = 0 in the block leaves the hidden state unchanged, so every schedule must draft,
    accept and count exactly as without the block."""
    w0 = tiny_shape.replace(decode_len=16)
    w1 = w0.replace(exit_block=True, exit_block_damp=0.0)
    W0, W1 = S.make_weights(w0), S.make_weights(w1)
    assert len(W1["wqkv"]) == w0.n_layers + 1 and float(W1["wo"][-1].abs().max()) == 0.0
    for run in (_two_stage, _pipeline, _eesd):
        _, _, t0, s0 = run(w0, W0, 16)
        _, _, t1, s1 = run(w1, W1, 16)
        assert t0 == t1 and s0.stats == s1.stats
        if hasattr(s0, "compared"):
            assert s0.compared == s1.compared


@pytest.mark.parametrize("E", [1, 2])
def test_lossless_with_a_real_block(tiny_shape, E):
    w = tiny_shape.replace(exit_layer=E, exit_block=True, exit_block_damp=1.0, decode_len=14)
    W = S.make_weights(w)
    for run in (_two_stage, _pipeline, _eesd):
        dec, prompt, toks, ss = run(w, W, 14)
        assert toks == O.greedy_decode_no_cache(dec, prompt, 15)
        # the block kept exactly one row per position its schedule has not rolled back
        assert ss.kv.len[w.n_layers] == ss.kv.len[0]


def test_compared_drafts_equal_the_whole_sequence_forward_through_the_block():
    """Drafts compared by the two-stage schedule are made on the true prefix: they must equal the argmax
    of embed -> layers 1..E -> block -> norm head evaluated over the whole sequence at once (no KV cache)."""
    w = S.Workload("xb", n_layers=4, exit_layer=2, d_model=48, n_heads=4, n_kv_heads=2, head_dim=12, d_ffn=80,
                   vocab=96, dtype="fp32", damp=0.25, seed=5, prompt_len=7, decode_len=30, exit_block=True,
                   exit_block_damp=0.5)
    W = S.make_weights(w)
    dec, prompt, toks, ss = _pipeline(w.replace(exit_layer=2), W, 30)      # two stages
    seq = list(prompt) + toks
    ex = dec.exit_logits_full(seq[:-1])
    want = [O.argmax_lowest(ex[len(prompt) + k - 1]) for k in range(1, len(toks))]
    assert ss.compared == want
    assert 0 < ss.stats.rejected < ss.stats.committed
    # and the block matters: without it other drafts are made
    w0 = w.replace(exit_block=False)
    W0 = {k: (v[: w.n_layers] if isinstance(v, list) else v) for k, v in W.items()}
    _, _, toks0, ss0 = _pipeline(w0, W0, 30)
    assert toks0 == toks and ss0.compared != ss.compared


def test_block_rows_follow_the_draft_layers_through_rollbacks(tiny_shape):
    w = tiny_shape.replace(exit_block=True, exit_block_damp=1.0, exit_head="independent")
    W = S.make_weights(w)
    dec = O.Decoder(w, W)
    prompt = S.make_prompt(w)
    ss = P.prefill(dec, prompt, 64)
    assert ss.kv.len[w.n_layers] == len(prompt) == ss.kv.len[0]
    out = []
    for _ in range(20):
        P.step(ss, out)
        assert ss.kv.len[w.n_layers] == ss.kv.len[0]
    assert ss.stats.rejected > 0
