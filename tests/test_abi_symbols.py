"""The C-ABI library loads without a GPU and exports every symbol include/ppsd.h declares."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    src = open(os.path.join(ROOT, "include", "ppsd.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(ppsd_[a-z_]+)\s*\(", src)))


def test_header_declares_the_four_boundary_calls():
    names = _declared_functions()
    for n in ("ppsd_load_weights", "ppsd_prefill", "ppsd_decode", "ppsd_stats"):
        assert n in names


def test_library_exports_every_declared_symbol():
    from paper_2509_19368_amd.build import LIB_PATH, build_library, is_stale
    if is_stale():
        build_library()
    lib = ctypes.CDLL(LIB_PATH)
    for n in _declared_functions():
        assert hasattr(lib, n), n


def test_config_validation_runs_on_the_host():
    import paper_2509_19368_amd as P
    import synth_inputs as S
    from paper_2509_19368_amd.binding import make_config
    cfg = make_config(S.WORKLOADS["C2"], 400, P.MODE_OVERLAP)
    n = P.ppsd_workspace_bytes(cfg)
    kv = 32 * 25 * 32 * 2 * 16 * 128 * 2          # layers * pages * kv heads * (K,V) * slots * hd * bytes
    # besides the KV pool: the prompt-chunk buffers of the matrix-core prefill (a chunk of 512 positions
    # at max_seq 400: fp32 residual, queries and attention output; bf16 high + low parts of one
    # projection input and of the SwiGLU output), its split-K partial sums (a few K ranges x 512 x 12288
    # floats for the QKV projection: under 96 MiB whatever the split), 4.3 MiB of attention split partials
    # (4 stream sets x 32 heads x 64 splits x 130 floats) and under 2 MiB of activations and tables
    pf = 4 * 512 * 3 * 4096 + 2 * 2 * 512 * (4096 + 11008)
    assert kv + pf < n < kv + pf + (104 << 20)
    cfg.mode = P.MODE_PIPELINE
    assert P.ppsd_workspace_bytes(cfg) == n           # the schedule does not change the layout
    cfg.exit_layer = 1                                # 32 stages: more than the schedule supports
    try:
        P.ppsd_workspace_bytes(cfg)
        assert False
    except P.PpsdError as e:
        assert "pipeline stages" in str(e)
    cfg.mode = P.MODE_OVERLAP
    cfg.exit_layer = 32
    try:
        P.ppsd_workspace_bytes(cfg)
        assert False
    except P.PpsdError as e:
        assert "exit_layer" in str(e)


def test_prefill_chunk_and_tile_settings_size_the_workspace_on_the_host():
    """prefill_chunk sizes the chunk buffers (residual, queries, attention output in fp32; the bf16 high + low
    parts), so a smaller chunk needs a smaller workspace; invalid settings are refused before any GPU call."""
    import paper_2509_19368_amd as P
    import synth_inputs as S
    from paper_2509_19368_amd.binding import make_config
    w = S.WORKLOADS["C5"]
    big = P.ppsd_workspace_bytes(make_config(w, 8192 + 600, P.MODE_VANILLA))                       # chunk 4096
    small = P.ppsd_workspace_bytes(make_config(w, 8192 + 600, P.MODE_VANILLA, prefill_chunk=512))
    looped = P.ppsd_workspace_bytes(make_config(w, 8192 + 600, P.MODE_VANILLA, prefill_loop=True))
    assert looped < small < big
    per_position = 4 * 3 * 4096 + 2 * 2 * (4096 + 14336)     # the buffers that scale with the chunk, bytes per position
    assert big - small >= (4096 - 512) * per_position
    for kw in (dict(prefill_chunk=100), dict(prefill_chunk=8192), dict(prefill_chunk=-128), dict(tune_prefill_tile=3)):
        try:
            P.ppsd_workspace_bytes(make_config(w, 9000, P.MODE_VANILLA, **kw))
            assert False, kw
        except P.PpsdError as e:
            assert "prefill" in str(e)
