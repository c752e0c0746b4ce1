"""Seeded synthetic inputs: model shapes, weights and prompts.

This module serves both the CPU oracle and the GPU path.  It holds none of the
decoding method's arithmetic: only a counter-based integer hash, a bounded
bell-shaped variate built from integer sums, and the table of workload shapes.

Every value is a pure function of (seed, tensor tag, element index), computed
with wrapping 64-bit integer arithmetic plus ONE fp32 multiply, so the same
call yields bit-identical tensors on the CPU and on a GPU and a 7B-parameter
model can be produced in chunks without any sequential generator state.

Weights follow the recipe of the workload list: zero-mean, standard deviation
0.02, all norm gains 1.0, no biases.  The bell-shaped variate is an
Irwin-Hall sum of eight 16-bit uniforms (bounded at about 4.9 sigma), which
stands in for N(0, 1).
"""
from __future__ import annotations

import dataclasses
from dataclasses import dataclass
from typing import Dict, List, Optional

import torch

_MASK64 = (1 << 64) - 1
_GOLDEN = 0x9E3779B97F4A7C15
_MUL1 = 0xBF58476D1CE4E5B9
_MUL2 = 0x94D049BB133111EB
_TAGMUL = 0xD6E8FEB86659FD93
_SEEDMUL = 0xA0761D6478BD642F

# Irwin-Hall(8) over 16-bit fields: mean 8*65535/2, variance 8*(65536^2-1)/12.
_IH_MEAN = 4 * 65535
_IH_STD = (8.0 * (65536.0 ** 2 - 1.0) / 12.0) ** 0.5
WEIGHT_STD = 0.02


def _s64(v: int) -> int:
    """Two's-complement view of an unsigned 64-bit constant as a Python int."""
    v &= _MASK64
    return v - (1 << 64) if v >= (1 << 63) else v


# ----------------------------------------------------------------------------
# Pure-Python definition of the generator (arbitrary-precision ints).  The
# tensor version below must agree with it bit for bit; a test checks that.
# ----------------------------------------------------------------------------
def mix64_py(z: int) -> int:
    z &= _MASK64
    z ^= z >> 30
    z = (z * _MUL1) & _MASK64
    z ^= z >> 27
    z = (z * _MUL2) & _MASK64
    z ^= z >> 31
    return z


def stream_base(seed: int, tag: int) -> int:
    return (seed * _SEEDMUL + tag * _TAGMUL + _GOLDEN) & _MASK64


def hash_pair_py(seed: int, tag: int, idx: int):
    z1 = mix64_py((stream_base(seed, tag) + idx * _GOLDEN) & _MASK64)
    z2 = mix64_py((z1 + _GOLDEN) & _MASK64)
    return z1, z2


def bell_int_py(seed: int, tag: int, idx: int) -> int:
    """Centered integer Irwin-Hall(8) sum for one element."""
    z1, z2 = hash_pair_py(seed, tag, idx)
    s = 0
    for z in (z1, z2):
        for k in range(4):
            s += (z >> (16 * k)) & 0xFFFF
    return s - _IH_MEAN


# ----------------------------------------------------------------------------
# Tensor version (torch int64, wrapping), usable on any device.
# ----------------------------------------------------------------------------
_M2 = 0x0000FFFF0000FFFF


def _mix64_(z: torch.Tensor, t: torch.Tensor) -> torch.Tensor:
    """In-place mix64 of an int64 tensor; t is scratch of the same shape.

    `>>` on int64 is an arithmetic shift, so the sign fill is masked off.
    """
    torch.bitwise_right_shift(z, 30, out=t); t &= (1 << 34) - 1; z ^= t
    z *= _s64(_MUL1)
    torch.bitwise_right_shift(z, 27, out=t); t &= (1 << 37) - 1; z ^= t
    z *= _s64(_MUL2)
    torch.bitwise_right_shift(z, 31, out=t); t &= (1 << 33) - 1; z ^= t
    return z


def _field_sum_(z: torch.Tensor, t: torch.Tensor) -> torch.Tensor:
    """In-place sum of the four 16-bit fields of each int64 (two folding adds)."""
    torch.bitwise_right_shift(z, 16, out=t); t &= _M2; z &= _M2; z += t
    torch.bitwise_right_shift(z, 32, out=t); z &= 0xFFFFFFFF; z += t
    return z


def _bell_int(seed: int, tag: int, start: int, n: int, device) -> torch.Tensor:
    z1 = torch.arange(start, start + n, dtype=torch.int64, device=device)
    z1 *= _s64(_GOLDEN)
    z1 += _s64(stream_base(seed, tag))
    t = torch.empty_like(z1)
    _mix64_(z1, t)
    z2 = z1 + _s64(_GOLDEN)
    _mix64_(z2, t)
    _field_sum_(z1, t)
    _field_sum_(z2, t)
    z1 += z2
    z1 -= _IH_MEAN
    return z1


_CHUNK = 1 << 20


def bell_tensor(seed: int, tag: int, numel: int, scale: float, device="cpu",
                dtype=torch.float32) -> torch.Tensor:
    """`numel` values of scale * IrwinHall8 / its std, rounded once to `dtype`.

    The integer sum is exact in fp32 (|s| < 2^19); the only rounding before the
    final cast is one fp32 multiply by the fp32 constant scale/std.
    """
    out = torch.empty(numel, dtype=dtype, device=device)
    c = torch.tensor(scale / _IH_STD, dtype=torch.float64).to(torch.float32).item()
    for start in range(0, numel, _CHUNK):
        n = min(_CHUNK, numel - start)
        s = _bell_int(seed, tag, start, n, device)
        out[start:start + n] = (s.to(torch.float32) * c).to(dtype)
    return out


def uniform_ints(seed: int, tag: int, n: int, modulus: int) -> List[int]:
    """n integers in [0, modulus): hash mod modulus (prompts, page shuffles)."""
    return [hash_pair_py(seed, tag, i)[0] % modulus for i in range(n)]


# ----------------------------------------------------------------------------
# Workload shapes
# ----------------------------------------------------------------------------
@dataclass(frozen=True)
class Workload:
    """One synthetic decode workload.

    damp multiplies W_o and W_down of layers exit_layer+1..n_layers (before the
    single rounding to the storage dtype); it controls how often the early-exit
    draft equals the full model's token.  exit_head: "tied" stores separate
    copies of the LM head and final-norm gain as the exit head; "independent"
    draws the exit head from its own stream; "blend" = LM head + exit_beta *
    independent noise.  exit_block: the early-exit head is one more transformer
    layer of the model's own structure followed by the norm head (the head the
    paper's main results use, Sec. 5.4 "Impact of exit head"); its tensors are
    appended to the per-layer lists as entry n_layers, its W_o and W_down scaled
    by exit_block_damp (0 makes the block the identity, i.e. the plain norm head).
    """
    name: str
    n_layers: int
    exit_layer: int
    d_model: int
    n_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    dtype: str                  # "fp32" | "bf16": storage type of weights and KV cache
    rope_base: float = 10000.0
    rms_eps: float = 1e-5
    damp: float = 1.0
    exit_head: str = "tied"
    exit_beta: float = 0.0
    exit_block: bool = False
    exit_block_damp: float = 1.0
    seed: int = 2509
    prompt_len: int = 16
    decode_len: int = 64
    acceptance_target: float = 0.0   # the acceptance rate the workload list asks for (damp was chosen for it); 0 = none stated

    def replace(self, **kw) -> "Workload":
        return dataclasses.replace(self, **kw)

    @property
    def torch_dtype(self):
        return torch.float32 if self.dtype == "fp32" else torch.bfloat16

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "fp32" else 2

    @property
    def qkv_rows(self) -> int:
        return (self.n_heads + 2 * self.n_kv_heads) * self.head_dim

    def layer_weight_bytes(self) -> int:
        d, f = self.d_model, self.d_ffn
        n = self.qkv_rows * d + d * self.n_heads * self.head_dim + 2 * f * d + d * f
        return n * self.elem_bytes

    def head_weight_bytes(self) -> int:
        return self.vocab * self.d_model * self.elem_bytes

    @property
    def kv_layers(self) -> int:
        """Layers that keep a KV cache: the model's, plus the early-exit block if there is one."""
        return self.n_layers + (1 if self.exit_block else 0)

    def kv_bytes_per_position(self, n_layers: Optional[int] = None) -> int:
        L = self.n_layers if n_layers is None else n_layers
        return 2 * L * self.n_kv_heads * self.head_dim * self.elem_bytes


WORKLOADS: Dict[str, Workload] = {
    # Tiny Llama-style decoder, fp32.
    "C1": Workload("C1", n_layers=4, exit_layer=1, d_model=256, n_heads=4, n_kv_heads=4,
                   head_dim=64, d_ffn=688, vocab=2048, dtype="fp32", damp=0.1,
                   prompt_len=16, decode_len=64),
    # Llama-2-7B shape, bf16.
    "C2": Workload("C2", n_layers=32, exit_layer=8, d_model=4096, n_heads=32, n_kv_heads=32,
                   head_dim=128, d_ffn=11008, vocab=32000, dtype="bf16", damp=0.04,       # measured alpha 0.836
                   prompt_len=128, decode_len=256, acceptance_target=0.8),
    # Llama-2-13B shape, bf16.
    "C4": Workload("C4", n_layers=40, exit_layer=10, d_model=5120, n_heads=40, n_kv_heads=40,
                   head_dim=128, d_ffn=13824, vocab=32000, dtype="bf16", damp=0.0548,     # measured alpha 0.805
                   prompt_len=512, decode_len=512, acceptance_target=0.8),
    # Llama-3-8B shape (GQA), bf16, long context.
    "C5": Workload("C5", n_layers=32, exit_layer=8, d_model=4096, n_heads=32, n_kv_heads=8,
                   head_dim=128, d_ffn=14336, vocab=128256, dtype="bf16", rope_base=500000.0,
                   damp=0.0548, prompt_len=8192, decode_len=512,
                   acceptance_target=0.77),   # the workload list states none for this one: what this damp measures (0.768 at prompt 8192)
}


def c3_grid() -> List[Workload]:
    """The 7B exit-layer x acceptance grid: one Workload per (E, damp) cell."""
    cells = []
    for E in (4, 8, 16):
        for target, damp in C3_DAMP[E].items():
            cells.append(WORKLOADS["C2"].replace(name=f"C3_E{E}_a{int(target * 100)}", exit_layer=E,
                                                 damp=damp, prompt_len=256, decode_len=256, acceptance_target=target))
    return cells


# damp per (exit layer, acceptance target), found by bisection on the GPU path over the cell's 256
# decoded tokens and frozen; measured acceptance in the comment (the relation is noisy: one chaotic
# 256-token stream per value).
C3_DAMP = {
    4: {0.5: 0.1064, 0.7: 0.0548, 0.9: 0.0146},     # 0.539, 0.684, 0.898
    8: {0.5: 0.1481, 0.7: 0.0830, 0.9: 0.0203},     # 0.500, 0.688, 0.910
    16: {0.5: 0.2872, 0.7: 0.1481, 0.9: 0.0548},    # 0.539, 0.730, 0.895
}

# Tensor tags: 16 tags per layer, global tensors at 1..15.
_TAG_EMBED, _TAG_LM, _TAG_EXIT, _TAG_PROMPT, _TAG_PAGES = 1, 2, 3, 4, 5
_TAG_WQKV, _TAG_WO, _TAG_WGU, _TAG_WDOWN = 0, 1, 2, 3


def _layer_tag(layer: int, which: int) -> int:
    return 16 * (layer + 1) + which


def make_weights(w: Workload, device="cpu") -> dict:
    """All tensors of the model, in the layout the C-ABI boundary takes.

    embed [V,d]; per layer: attn_norm [d] (fp32), wqkv [(n_h+2n_kv)*hd, d] with
    rows ordered q heads, k heads, v heads; wo [d, n_h*hd]; mlp_norm [d] (fp32);
    wgu [2f, d] with rows ordered gate then up; wdown [d, f]; final_norm [d],
    lm_head [V,d]; exit_norm [d], exit_head [V,d].  With exit_block the per-layer
    lists have one more entry, the early-exit block.  Matrices are row-major
    [out_features, in_features] in the storage dtype; gains are fp32.
    """
    dt = w.torch_dtype
    d, f, V = w.d_model, w.d_ffn, w.vocab
    nq = w.n_heads * w.head_dim

    def mat(tag, rows, cols, scale=WEIGHT_STD):
        return bell_tensor(w.seed, tag, rows * cols, scale, device, dt).view(rows, cols)

    ones = lambda: torch.ones(d, dtype=torch.float32, device=device)
    out = {"embed": mat(_TAG_EMBED, V, d), "final_norm": ones(), "lm_head": mat(_TAG_LM, V, d),
           "attn_norm": [], "wqkv": [], "wo": [], "mlp_norm": [], "wgu": [], "wdown": []}
    for l in range(w.kv_layers):
        s = WEIGHT_STD * (w.damp if l >= w.exit_layer else 1.0)
        if l == w.n_layers:                      # the early-exit block
            s = WEIGHT_STD * w.exit_block_damp
        out["attn_norm"].append(ones())
        out["wqkv"].append(mat(_layer_tag(l, _TAG_WQKV), w.qkv_rows, d))
        out["wo"].append(mat(_layer_tag(l, _TAG_WO), d, nq, s))
        out["mlp_norm"].append(ones())
        out["wgu"].append(mat(_layer_tag(l, _TAG_WGU), 2 * f, d))
        out["wdown"].append(mat(_layer_tag(l, _TAG_WDOWN), d, f, s))
    out["exit_norm"] = ones()
    if w.exit_head == "tied":
        out["exit_head"] = out["lm_head"].clone()
    elif w.exit_head == "independent":
        out["exit_head"] = mat(_TAG_EXIT, V, d)
    elif w.exit_head == "blend":
        noise = bell_tensor(w.seed, _TAG_EXIT, V * d, WEIGHT_STD * w.exit_beta, device,
                            torch.float32).view(V, d)
        out["exit_head"] = (out["lm_head"].to(torch.float32) + noise).to(dt)
    else:
        raise ValueError(f"unknown exit_head {w.exit_head!r}")
    return out


def make_prompt(w: Workload, n: Optional[int] = None) -> List[int]:
    """Uniform-random token ids in [0, vocab)."""
    return uniform_ints(w.seed, _TAG_PROMPT, w.prompt_len if n is None else n, w.vocab)


def page_permutation(seed: int, n_pages: int) -> List[int]:
    """A seeded permutation of range(n_pages) (Fisher-Yates on hashed draws)."""
    perm = list(range(n_pages))
    draws = [hash_pair_py(seed, _TAG_PAGES, i)[1] for i in range(n_pages)]
    for i in range(n_pages - 1, 0, -1):
        j = draws[i] % (i + 1)
        perm[i], perm[j] = perm[j], perm[i]
    return perm
