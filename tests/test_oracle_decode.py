"""Pins for the whole-model oracle: brute force, textbook reductions, a library-built block."""
import math

import torch
import torch.nn.functional as F

import synth_inputs as S
from oracle import decoder_fp64 as O

F64 = torch.float64


def _library_logits(w, W, tokens):
    """The same model assembled from torch.nn.functional routines (fp64), independently written."""
    d, hd, n_h, n_kv = w.d_model, w.head_dim, w.n_heads, w.n_kv_heads
    T = len(tokens)
    x = F.embedding(torch.tensor(tokens), W["embed"].double())
    pos = torch.arange(T, dtype=F64)
    theta = w.rope_base ** (-torch.arange(0, hd, 2, dtype=F64) / hd)
    rot = torch.polar(torch.ones(T, hd // 2, dtype=F64), pos[:, None] * theta)[:, None, :]

    def rotate(v):
        z = torch.complex(v[..., : hd // 2], v[..., hd // 2:]) * rot
        return torch.cat([z.real, z.imag], -1)

    for l in range(w.n_layers):
        xn = F.rms_norm(x, (d,), W["attn_norm"][l].double(), w.rms_eps)
        qkv = F.linear(xn, W["wqkv"][l].double())
        q, k, v = qkv.split([n_h * hd, n_kv * hd, n_kv * hd], dim=-1)
        q, k, v = rotate(q.view(T, n_h, hd)), rotate(k.view(T, n_kv, hd)), v.view(T, n_kv, hd)
        k, v = k.repeat_interleave(n_h // n_kv, 1), v.repeat_interleave(n_h // n_kv, 1)
        a = F.scaled_dot_product_attention(q.transpose(0, 1), k.transpose(0, 1), v.transpose(0, 1), is_causal=True)
        x = x + F.linear(a.transpose(0, 1).reshape(T, n_h * hd), W["wo"][l].double())
        xn = F.rms_norm(x, (d,), W["mlp_norm"][l].double(), w.rms_eps)
        g, u = F.linear(xn, W["wgu"][l].double()).chunk(2, dim=-1)
        x = x + F.linear(F.silu(g) * u, W["wdown"][l].double())
    return F.linear(F.rms_norm(x, (d,), W["final_norm"].double(), w.rms_eps), W["lm_head"].double())


def test_full_forward_equals_library_assembly(tiny_shape):
    W = S.make_weights(tiny_shape)
    # non-trivial gains so a dropped gain shows
    for l in range(tiny_shape.n_layers):
        W["attn_norm"][l] = 1.0 + 0.1 * S.bell_tensor(1, 900 + l, tiny_shape.d_model, 1.0)
        W["mlp_norm"][l] = 1.0 + 0.1 * S.bell_tensor(1, 950 + l, tiny_shape.d_model, 1.0)
    W["final_norm"] = 1.0 + 0.1 * S.bell_tensor(1, 999, tiny_shape.d_model, 1.0)
    toks = S.make_prompt(tiny_shape, 9)
    got = O.Decoder(tiny_shape, W).logits_full(toks)
    want = _library_logits(tiny_shape, W, toks)
    assert torch.allclose(got, want, rtol=0, atol=1e-12 * want.abs().max().item() + 1e-15)


def test_c1_shape_equals_library_assembly():
    w = S.WORKLOADS["C1"]
    W = S.make_weights(w)
    toks = S.make_prompt(w, 6)
    got = O.Decoder(w, W).logits_full(toks)
    want = _library_logits(w, W, toks)
    assert (got - want).abs().max().item() < 1e-10 * want.abs().max().item()


def test_kv_cache_decode_equals_no_cache_brute_force(tiny_shape):
    for variant in (tiny_shape, tiny_shape.replace(n_kv_heads=4, seed=11), tiny_shape.replace(n_kv_heads=1, damp=1.0)):
        dec = O.Decoder(variant, S.make_weights(variant))
        prompt = S.make_prompt(variant)
        brute = O.greedy_decode_no_cache(dec, prompt, variant.decode_len)
        tr = O.greedy_decode(dec, prompt, variant.decode_len, keep_logits=True)
        assert tr.tokens == brute
        # logits of the cached path agree with the full re-forward at every generated position
        full = dec.logits_full(list(prompt) + brute[:-1])
        for k, lg in enumerate(tr.logits):
            assert torch.allclose(lg, full[len(prompt) - 1 + k], atol=1e-13)
        assert all(m >= 0 for m in tr.margin)


def test_teacher_forced_trace_records_own_argmax(tiny_shape):
    dec = O.Decoder(tiny_shape, S.make_weights(tiny_shape))
    prompt = S.make_prompt(tiny_shape)
    free = O.greedy_decode(dec, prompt, 6)
    forced = list(free.tokens)
    forced[2] = (forced[2] + 1) % tiny_shape.vocab                 # push the prefix off the greedy path
    tf = O.greedy_decode(dec, prompt, 6, forced=forced)
    assert tf.tokens[:3] == free.tokens[:3]                        # identical until the forced deviation is consumed
    want3 = O.argmax_lowest(dec.logits_full(list(prompt) + forced[:3])[-1])
    assert tf.tokens[3] == want3


def test_single_layer_zero_projections_is_a_token_map():
    """L = 1 with W_o = W_down = 0: logits = W_lm rms(Emb[tok]); the stream is a fixed map."""
    w = S.Workload("map", n_layers=1, exit_layer=1, d_model=16, n_heads=2, n_kv_heads=2, head_dim=8,
                   d_ffn=24, vocab=40, dtype="fp32", seed=3)
    W = S.make_weights(w)
    W["wo"][0].zero_(); W["wdown"][0].zero_()
    dec = O.Decoder(w, W)
    emb, lm = W["embed"].double(), W["lm_head"].double()
    nxt = [int(torch.argmax(lm @ (e / torch.sqrt((e * e).mean() + w.rms_eps)))) for e in emb]
    prompt = [5, 17, 2]
    got = O.greedy_decode(dec, prompt, 8).tokens
    want, t = [], prompt[-1]
    for _ in range(8):
        t = nxt[t]; want.append(t)
    assert got == want


def test_bf16_weights_enter_at_stored_value():
    w = S.Workload("b", n_layers=1, exit_layer=1, d_model=16, n_heads=2, n_kv_heads=1, head_dim=8,
                   d_ffn=24, vocab=32, dtype="bf16", seed=4)
    W = S.make_weights(w)
    assert W["lm_head"].dtype == torch.bfloat16
    Wf = {k: ([t.float() for t in v] if isinstance(v, list) else v.float()) for k, v in W.items()}
    toks = [1, 2, 3, 4]
    assert torch.equal(O.Decoder(w, W).logits_full(toks), O.Decoder(w, Wf).logits_full(toks))


def test_exit_logits_use_first_E_layers_only(tiny_shape):
    w = tiny_shape.replace(exit_layer=2)
    W = S.make_weights(w)
    dec = O.Decoder(w, W)
    toks = S.make_prompt(w, 7)
    base = dec.exit_logits_full(toks)
    W["wdown"][2].mul_(3.0)                                        # layer 3 is past the exit
    assert torch.equal(dec.exit_logits_full(toks), base)
    W["wdown"][1].mul_(3.0)                                        # layer 2 is inside the draft model
    assert not torch.equal(dec.exit_logits_full(toks), base)
    # tied exit head on a model whose later layers are switched off equals the LM head
    w0 = tiny_shape.replace(damp=0.0)
    dec0 = O.Decoder(w0, S.make_weights(w0))
    assert torch.allclose(dec0.exit_logits_full(toks), dec0.logits_full(toks), atol=1e-15)


def test_c1_stream_matches_stored_oracle_output():
    """Regression pin: the stored C1 stream was written by tests/golden/make_c1_stream.py."""
    import os
    rows = [ln.split() for ln in open(os.path.join(os.path.dirname(__file__), "golden", "c1_greedy_stream.txt"))
            if not ln.startswith("#")]
    w = S.WORKLOADS["C1"]
    tr = O.greedy_decode(O.Decoder(w, S.make_weights(w)), S.make_prompt(w), len(rows))
    assert tr.tokens == [int(r[1]) for r in rows]
    assert all(abs(m - float(r[2])) < 1e-9 for m, r in zip(tr.margin, rows))
    assert len(set(tr.tokens)) >= 8          # the random model does not collapse into a short cycle
