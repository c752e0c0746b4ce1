"""What the compiler made of the hot kernels in the LIBRARY's translation unit (no GPU needed: hipcc
cross-compiles the device code to assembly).

The same kernel template can come out differently in the library and in a standalone benchmark: the
slab-walking down-projection of the batched verify pass once read its staged inputs from LDS with
pairs of 4-byte reads in the library build only, which cost it 40 % of its speed while the benchmark
build showed nothing.  These checks look at the library build itself."""
import collections
import os
import re
import subprocess
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def kernels():
    """name -> (instruction counts, metadata lines) for every kernel of ppsd_api.hip's device code."""
    from paper_2509_19368_amd.build import HIPCC_FLAGS, SOURCES
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = [f for f in HIPCC_FLAGS if f not in ("-shared", "-fPIC")]
    src = [s for s in SOURCES if s.endswith("ppsd_api.hip")]
    assert len(src) == 1
    out = {}
    with tempfile.TemporaryDirectory() as tmp:
        asm = os.path.join(tmp, "api.s")
        res = subprocess.run([hipcc, *flags, "--cuda-device-only", "-S", "-o", asm, src[0]], capture_output=True, text=True)
        assert res.returncode == 0, res.stderr[-2000:]
        name, counts = None, None
        for line in open(asm):
            m = re.match(r"^(_Z\w+):", line)
            if m:
                name, counts = m.group(1), collections.Counter()
                continue
            if name is None:
                continue
            tok = line.split(";")[0].split()
            if tok and re.match(r"^(ds_|global_|flat_|scratch_|buffer_|v_mfma)", tok[0]):
                counts[tok[0]] += 1
            m = re.match(r"\s*\.amdhsa_(private_segment_fixed_size|next_free_vgpr)\s+(\d+)", line)
            if m:
                counts["meta_" + m.group(1)] = int(m.group(2))
            if line.strip().startswith(".end_amdhsa_kernel"):
                out[name] = counts
                name = None
    return out


def _pick(kernels, fragment):
    hit = {k: v for k, v in kernels.items() if fragment in k}
    assert hit, fragment
    return hit


def test_no_hot_kernel_spills_or_uses_flat_addressing(kernels):
    for frag in ("k_qkvI", "k_proj_residI", "k_gate_upI", "k_headI", "k_attnI", "k_qkv_bI", "k_gate_up_bI", "k_head_bI",
                 "k_proj_resid_bI", "k_proj_resid_bsI", "k_attn_bI", "k_pf_gemmI", "k_pf_flashI"):
        for name, c in _pick(kernels, frag).items():
            assert c["meta_private_segment_fixed_size"] == 0, (name, "scratch memory in a hot kernel")
            assert not any(k.startswith("scratch_") for k in c), name
            assert not any(k.startswith("flat_load") or k.startswith("flat_store") for k in c), (name, "flat memory access")


def test_staged_inputs_are_read_with_16_byte_lds_instructions(kernels):
    """Weight-streaming kernels read the staged input vectors as whole float4.  The few narrower LDS
    reads allowed here belong to the reductions across waves (norm, argmax)."""
    # (kernel, narrow reads allowed, paired narrow writes allowed): the batched norm stage stores its B sums
    # of squares per wave with paired writes, the head kernels also their per-wave argmax candidates
    for frag, narrow_ok, pair_writes_ok in (("k_qkvI", 0, 0), ("k_proj_residI", 0, 0), ("k_gate_upI", 0, 0), ("k_headI", 8, 2),
                                            ("k_qkv_bI", 0, 3), ("k_gate_up_bI", 0, 3), ("k_proj_resid_bI", 0, 0),
                                            ("k_proj_resid_bsI", 0, 0), ("k_head_bI", 16, 8)):
        for name, c in _pick(kernels, frag).items():
            assert c["ds_read_b128"] >= 4, (name, dict(c))
            narrow = c["ds_read2_b32"] + c["ds_read2_b64"] + c["ds_read_b32"] + c["ds_read_b64"]
            assert narrow <= narrow_ok, (name, dict(c))
            assert c["ds_write2_b32"] + c["ds_write2_b64"] <= pair_writes_ok, (name, dict(c))


def test_weights_are_fetched_16_bytes_per_lane(kernels):
    for frag in ("k_qkvI", "k_proj_residI", "k_gate_upI", "k_headI", "k_qkv_bI", "k_gate_up_bI", "k_head_bI", "k_proj_resid_bI",
                 "k_proj_resid_bsI"):
        for name, c in _pick(kernels, frag).items():
            assert c["global_load_dwordx4"] >= 8, (name, dict(c))


def test_prefill_kernels_run_on_the_matrix_cores_from_16_byte_lds_reads(kernels):
    for frag in ("k_pf_gemmI", "k_pf_flashI"):
        for name, c in _pick(kernels, frag).items():
            assert c["v_mfma_f32_32x32x16_bf16"] >= 16, (name, dict(c))
            assert c["ds_read_b128"] >= 32, (name, dict(c))
            assert c["ds_read2_b32"] + c["ds_read2_b64"] + c["ds_read_b32"] == 0, (name, dict(c))


def test_register_budgets_keep_the_intended_number_of_workgroups_resident(kernels):
    """A CU holds 512 VGPRs per SIMD lane: a 512-thread workgroup puts two waves on every SIMD, so three
    resident workgroups need at most 84 registers per wave, two need at most 128, one at most 256."""
    budgets = (("k_qkvI", 84), ("k_proj_residI", 84), ("k_gate_upI", 84), ("k_headI", 84),      # three per CU
               ("k_qkv_bI", 128), ("k_gate_up_bI", 128), ("k_head_bI", 128), ("k_proj_resid_bI", 128),
               ("k_proj_resid_bsI", 128), ("k_attnI", 128), ("k_attn_bI", 128),                  # two per CU
               ("k_pf_gemmI", 256), ("k_pf_flashI", 256))
    for frag, limit in budgets:
        for name, c in _pick(kernels, frag).items():
            # five staged vectors leave room for one workgroup per CU only (LDS), whatever the registers
            lim = 256 if ("_bI" in frag or "_bsI" in frag) and "Li5E" in name and "k_attn" not in frag else limit
            # the variants with two trips in flight per wave (second template argument 2) are launched two per CU
            if frag in ("k_qkvI", "k_proj_residI", "k_gate_upI", "k_headI") and re.search(r"I[tf]Li2EE", name):
                lim = 128
            assert 0 < c["meta_next_free_vgpr"] <= lim, (name, c["meta_next_free_vgpr"], lim)
