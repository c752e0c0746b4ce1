"""Pins for the oracle's elementary functions: closed forms, invariants, library routines.

Each check is chosen so that a plausible slip (dropped eps, wrong sign in the
rotation, transposed operand, wrong KV-head mapping, missing 1/sqrt(hd), sum
instead of mean) fails at least one assertion.
"""
import math

import pytest
import torch
import torch.nn.functional as F

from oracle import decoder_fp64 as O

F64 = torch.float64
torch.manual_seed(0)


# ------------------------------------------------------------------ RMSNorm
def test_rmsnorm_constant_vector_closed_form():
    c, eps, d = 3.0, 1e-5, 16
    g = torch.linspace(0.5, 2.0, d, dtype=F64)
    y = O.rmsnorm(torch.full((d,), c, dtype=F64), g, eps)
    assert torch.allclose(y, c / math.sqrt(c * c + eps) * g, rtol=0, atol=1e-15)


def test_rmsnorm_hand_example_and_eps_matters():
    # x = (3, 4): mean square 12.5
    y = O.rmsnorm(torch.tensor([3.0, 4.0], dtype=F64), torch.tensor([1.0, 2.0], dtype=F64), 0.5)
    r = math.sqrt(13.0)
    assert torch.allclose(y, torch.tensor([3 / r, 8 / r], dtype=F64), atol=1e-15)
    # eps sits inside the root: a tiny input is NOT blown up to unit RMS
    t = O.rmsnorm(torch.tensor([1e-4, 0.0], dtype=F64), torch.ones(2, dtype=F64), 1e-5)
    assert abs(t[0].item() - 1e-4 / math.sqrt(0.5e-8 + 1e-5)) < 1e-12


def test_rmsnorm_scale_invariance_and_library():
    x = torch.randn(5, 64, dtype=F64)
    g = torch.randn(64, dtype=F64)
    a, b = O.rmsnorm(x, g, 0.0), O.rmsnorm(7.5 * x, g, 0.0)
    assert torch.allclose(a, b, atol=1e-12)
    assert torch.allclose(O.rmsnorm(x, g, 1e-5), F.rms_norm(x, (64,), weight=g, eps=1e-5), atol=1e-13)


# ------------------------------------------------------------------ RoPE
def test_rope_position_zero_is_identity_and_norm_preserved():
    v = torch.randn(3, 2, 16, dtype=F64)
    assert torch.equal(O.rope(v, torch.zeros(3, dtype=torch.int64), 10000.0), v)
    r = O.rope(v, torch.tensor([1, 77, 4000]), 10000.0)
    assert torch.allclose(r.norm(dim=-1), v.norm(dim=-1), atol=1e-12)


def test_rope_two_dim_is_plain_rotation():
    # hd = 2: one pair, theta_0 = 1, angle = pos
    v = torch.tensor([[[1.0, 0.0]], [[0.0, 1.0]]], dtype=F64)
    r = O.rope(v, torch.tensor([2, 2]), 10000.0)
    assert torch.allclose(r[0, 0], torch.tensor([math.cos(2), math.sin(2)], dtype=F64), atol=1e-15)
    assert torch.allclose(r[1, 0], torch.tensor([-math.sin(2), math.cos(2)], dtype=F64), atol=1e-15)


def test_rope_frequencies_and_pairing():
    hd, base, p = 8, 500000.0, 3
    v = torch.zeros(1, 1, hd, dtype=F64)
    v[0, 0, 2] = 1.0                                  # element i=2 pairs with i + hd/2 = 6
    r = O.rope(v, torch.tensor([p]), base)
    ang = p * base ** (-2 * 2 / hd)
    want = torch.zeros(hd, dtype=F64)
    want[2], want[6] = math.cos(ang), math.sin(ang)
    assert torch.allclose(r[0, 0], want, atol=1e-15)


def test_rope_inner_product_depends_on_offset_only():
    q, k = torch.randn(1, 1, 32, dtype=F64), torch.randn(1, 1, 32, dtype=F64)
    def ip(pq, pk):
        return (O.rope(q, torch.tensor([pq]), 1e4) * O.rope(k, torch.tensor([pk]), 1e4)).sum().item()
    assert abs(ip(10, 3) - ip(510, 503)) < 1e-10
    assert abs(ip(10, 3) - ip(3, 10)) > 1e-6          # direction matters


def test_rope_equals_complex_multiplication():
    hd, base = 64, 10000.0
    v = torch.randn(4, 3, hd, dtype=F64)
    pos = torch.tensor([0, 5, 1234, 8700])
    z = torch.complex(v[..., : hd // 2], v[..., hd // 2:])
    theta = base ** (-torch.arange(0, hd, 2, dtype=F64) / hd)
    rot = torch.polar(torch.ones(4, hd // 2, dtype=F64), pos.to(F64)[:, None] * theta)[:, None, :]
    want = z * rot
    got = O.rope(v, pos, base)
    assert torch.allclose(got, torch.cat([want.real, want.imag], -1), atol=1e-12)


# ------------------------------------------------------------------ attention
def test_attention_single_key_returns_value():
    q = torch.randn(4, 8, dtype=F64)
    K, V = torch.randn(1, 2, 8, dtype=F64), torch.randn(1, 2, 8, dtype=F64)
    a = O.attend_one(q, K, V)
    assert torch.equal(a[0], V[0, 0]) and torch.equal(a[1], V[0, 0])
    assert torch.equal(a[2], V[0, 1]) and torch.equal(a[3], V[0, 1])       # head h -> kv head h // 2


def test_attention_equal_keys_average_values():
    q = torch.randn(2, 8, dtype=F64)
    K = torch.randn(1, 2, 8, dtype=F64).expand(6, 2, 8).contiguous()
    V = torch.randn(6, 2, 8, dtype=F64)
    assert torch.allclose(O.attend_one(q, K, V), V.mean(0), atol=1e-14)


def test_attention_two_keys_hand_softmax():
    hd = 4
    q = torch.tensor([[2.0, 0.0, 0.0, 0.0]], dtype=F64)
    K = torch.tensor([[[1.0, 0, 0, 0]], [[3.0, 0, 0, 0]]], dtype=F64)
    V = torch.tensor([[[1.0, 0, 0, 0]], [[0.0, 1, 0, 0]]], dtype=F64)
    s0, s1 = 2.0 / math.sqrt(hd), 6.0 / math.sqrt(hd)
    w1 = 1.0 / (1.0 + math.exp(s0 - s1))
    a = O.attend_one(q, K, V)[0]
    assert torch.allclose(a, torch.tensor([1 - w1, w1, 0, 0], dtype=F64), atol=1e-15)


def test_attention_permutation_invariance_and_shift_stability():
    q = torch.randn(4, 16, dtype=F64)
    K, V = torch.randn(9, 4, 16, dtype=F64), torch.randn(9, 4, 16, dtype=F64)
    perm = torch.randperm(9)
    assert torch.allclose(O.attend_one(q, K, V), O.attend_one(q, K[perm], V[perm]), atol=1e-13)
    big = O.attend_one(1000.0 * q, K, V)               # max-subtraction keeps it finite
    assert torch.isfinite(big).all()


def test_gqa_equals_mha_with_duplicated_kv():
    q = torch.randn(4, 8, dtype=F64)
    K, V = torch.randn(7, 2, 8, dtype=F64), torch.randn(7, 2, 8, dtype=F64)
    Kd, Vd = K.repeat_interleave(2, dim=1), V.repeat_interleave(2, dim=1)
    assert torch.allclose(O.attend_one(q, K, V), O.attend_one(q, Kd, Vd), atol=1e-14)


def test_causal_attention_equals_library_and_per_position_form():
    T, n_h, n_kv, hd = 11, 4, 2, 16
    q, k, v = (torch.randn(T, n, hd, dtype=F64) for n in (n_h, n_kv, n_kv))
    got = O.attend_causal(q, k, v)
    lib = F.scaled_dot_product_attention(q.transpose(0, 1), k.repeat_interleave(2, 1).transpose(0, 1),
                                         v.repeat_interleave(2, 1).transpose(0, 1), is_causal=True)
    assert torch.allclose(got, lib.transpose(0, 1), atol=1e-12)
    for t in (0, 4, T - 1):
        assert torch.allclose(got[t], O.attend_one(q[t], k[: t + 1], v[: t + 1]), atol=1e-13)
    # no leak from the future: changing a later key leaves earlier outputs alone
    k2 = k.clone(); k2[7] += 1.0
    assert torch.equal(O.attend_causal(q, k2, v)[:7], got[:7])


# ------------------------------------------------------------------ SwiGLU / heads / argmax
def test_silu_values():
    z = torch.tensor([0.0, 1.0, -1.0, 30.0], dtype=F64)
    want = torch.tensor([0.0, 1 / (1 + math.exp(-1)), -1 / (1 + math.exp(1)), 30 / (1 + math.exp(-30))], dtype=F64)
    assert torch.allclose(O.silu(z), want, atol=1e-15)
    assert torch.allclose(O.silu(z), F.silu(z), atol=1e-15)


def test_argmax_ties_take_lowest_index():
    assert O.argmax_lowest(torch.tensor([1.0, 5.0, 5.0, 2.0, 5.0], dtype=F64)) == 1
    assert O.argmax_lowest(torch.tensor([-3.0, -3.0], dtype=F64)) == 0
    m, a = O.top2_margin(torch.tensor([1.0, -7.0, 4.0], dtype=F64))
    assert m == 3.0 and a == 7.0


class _Shape:
    n_layers, exit_layer, d_model, n_heads, n_kv_heads, head_dim, d_ffn, vocab = 1, 1, 4, 2, 1, 2, 3, 5
    rope_base, rms_eps = 10000.0, 1e-5


def _hand_weights():
    s = _Shape
    eye = torch.eye(4, dtype=F64)
    W = {"embed": torch.arange(20, dtype=F64).view(5, 4) / 10, "final_norm": torch.ones(4, dtype=F64),
         "lm_head": torch.randn(5, 4, dtype=F64), "exit_norm": torch.full((4,), 2.0, dtype=F64),
         "exit_head": torch.randn(5, 4, dtype=F64), "attn_norm": [torch.ones(4, dtype=F64)],
         "mlp_norm": [torch.ones(4, dtype=F64)],
         "wqkv": [torch.cat([eye, eye[:2], eye[2:]])],         # q = xn, k = xn[:2], v = xn[2:]
         "wo": [torch.zeros(4, 4, dtype=F64)], "wgu": [torch.randn(6, 4, dtype=F64)],
         "wdown": [torch.zeros(4, 3, dtype=F64)]}
    return s, W


def test_block_with_hand_computable_weights():
    s, W = _hand_weights()
    dec = O.Decoder(s, W)
    x = torch.tensor([[1.0, 2.0, 3.0, 4.0]], dtype=F64)
    q, k, v = dec.qkv(0, x, torch.tensor([0]))
    xn = x / math.sqrt(7.5 + 1e-5)
    assert torch.allclose(q.view(1, 4), xn, atol=1e-15)
    assert torch.allclose(k.view(1, 2), xn[:, :2], atol=1e-15) and torch.allclose(v.view(1, 2), xn[:, 2:], atol=1e-15)
    # o_proj picks attention element 3 into channel 0; down is zero -> only that residual add
    W["wo"][0][0, 3] = 2.0
    a = torch.tensor([[[0.5, 0.25], [0.125, 4.0]]], dtype=F64)           # [T=1, n_h=2, hd=2], flat index 3 = 4.0
    y = dec.after_attention(0, x, a)
    assert torch.allclose(y, x + torch.tensor([[8.0, 0, 0, 0]], dtype=F64), atol=1e-15)
    # MLP: one nonzero down column -> silu(gate_1) * up_1 lands in channel 2
    W["wo"][0].zero_(); W["wdown"][0][2, 1] = 1.0
    y = dec.after_attention(0, x, a)
    g, u = W["wgu"][0][1] @ xn[0], W["wgu"][0][3 + 1] @ xn[0]
    assert torch.allclose(y[0, 2], x[0, 2] + g / (1 + torch.exp(-g)) * u, atol=1e-14)
    assert torch.equal(y[0, [0, 1, 3]], x[0, [0, 1, 3]])


def test_heads_use_their_own_norm_and_matrix():
    s, W = _hand_weights()
    dec = O.Decoder(s, W)
    x = torch.randn(4, dtype=F64)
    xn = x / torch.sqrt((x * x).mean() + 1e-5)
    assert torch.allclose(dec.head_logits(x, "lm"), W["lm_head"] @ xn, atol=1e-14)
    assert torch.allclose(dec.head_logits(x, "exit"), W["exit_head"] @ (2.0 * xn), atol=1e-14)
