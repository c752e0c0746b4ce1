"""The seeded input generator: bit-exactness of the tensor form and the recipe."""
import torch

import synth_inputs as S


def test_tensor_hash_equals_bigint_definition():
    for seed, tag, start in [(2509, 16, 0), (7, 3, 123456789), (1, 1, (1 << 33) + 5)]:
        ref = [S.bell_int_py(seed, tag, start + i) for i in range(257)]
        got = S._bell_int(seed, tag, start, 257, "cpu").tolist()
        assert ref == got


def test_chunking_does_not_change_values():
    a = S.bell_tensor(5, 9, (1 << 20) + 77, 0.02)
    b = torch.cat([(S._bell_int(5, 9, s, n, "cpu").to(torch.float32) *
                    torch.tensor(0.02 / S._IH_STD, dtype=torch.float64).float().item())
                   for s, n in [(0, 1000), (1000, (1 << 20) + 77 - 1000)]])
    assert torch.equal(a, b)


def test_moments_match_recipe():
    x = S.bell_tensor(2509, 42, 1 << 21, S.WEIGHT_STD).double()
    assert abs(x.mean().item()) < 1e-4
    assert abs(x.std().item() - 0.02) < 2e-4
    assert x.abs().max().item() < 0.02 * 4.95


def test_streams_are_distinct_and_reproducible():
    a = S.bell_tensor(1, 1, 4096, 1.0)
    assert torch.equal(a, S.bell_tensor(1, 1, 4096, 1.0))
    assert not torch.equal(a, S.bell_tensor(1, 2, 4096, 1.0))
    assert not torch.equal(a, S.bell_tensor(2, 1, 4096, 1.0))
    assert abs(torch.corrcoef(torch.stack([a, S.bell_tensor(1, 2, 4096, 1.0)]))[0, 1].item()) < 0.06


def test_weight_layout_damp_and_exit_head(tiny_shape):
    w = tiny_shape
    W = S.make_weights(w)
    assert W["wqkv"][0].shape == ((w.n_heads + 2 * w.n_kv_heads) * w.head_dim, w.d_model)
    assert W["wgu"][0].shape == (2 * w.d_ffn, w.d_model)
    assert W["wo"][0].shape == (w.d_model, w.n_heads * w.head_dim)
    assert W["wdown"][0].shape == (w.d_model, w.d_ffn)
    assert torch.equal(W["exit_head"], W["lm_head"]) and W["exit_head"].data_ptr() != W["lm_head"].data_ptr()
    full = S.make_weights(w.replace(damp=1.0))
    # layers past the exit are scaled, layers up to it are not
    assert torch.equal(W["wo"][0], full["wo"][0])
    ratio = (W["wo"][1].double().norm() / full["wo"][1].double().norm()).item()
    assert abs(ratio - w.damp) < 1e-6
    assert torch.equal(W["wqkv"][2], full["wqkv"][2])
    ind = S.make_weights(w.replace(exit_head="independent"))
    assert not torch.equal(ind["exit_head"], ind["lm_head"])


def test_bf16_weights_round_once():
    w = S.WORKLOADS["C2"].replace(n_layers=1, exit_layer=1, vocab=128, d_model=64, d_ffn=96,
                                  n_heads=2, n_kv_heads=2, head_dim=32)
    W = S.make_weights(w)
    assert W["wqkv"][0].dtype == torch.bfloat16
    ref = S.bell_tensor(w.seed, S._layer_tag(0, 0), W["wqkv"][0].numel(), 0.02).to(torch.bfloat16)
    assert torch.equal(W["wqkv"][0].flatten(), ref)


def test_prompt_and_permutation():
    p = S.make_prompt(S.WORKLOADS["C1"])
    assert len(p) == 16 and all(0 <= t < 2048 for t in p)
    perm = S.page_permutation(3, 50)
    assert sorted(perm) == list(range(50)) and perm != list(range(50))
