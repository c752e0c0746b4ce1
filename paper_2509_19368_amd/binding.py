"""ctypes binding of include/ppsd.h: argument marshalling only.

torch provides device memory and the two HIP streams; every step of the decode
path runs inside libppsd.so.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

import torch

from .build import LIB_PATH

MODE_VANILLA, MODE_SERIAL, MODE_OVERLAP, MODE_PIPELINE, MODE_EESD = 0, 1, 2, 3, 4
ENGINE_STREAMS, ENGINE_PERSISTENT = 0, 1
KERNEL_KINDS = ("qkv", "attention", "o_proj", "gate_up", "down", "head", "commit")


class PpsdError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"ppsd error {code}: {msg}")
        self.code = code


class ppsd_config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "exit_layer", "d_model", "n_heads", "n_kv_heads", "head_dim",
                                          "d_ffn", "vocab", "dtype", "max_seq", "kv_page_tokens", "mode")] + \
               [("rope_base", C.c_float), ("rms_eps", C.c_float), ("debug_logits", C.c_int32),
                ("use_graph", C.c_int32), ("time_kernels", C.c_int32), ("engine", C.c_int32),
                ("prefill_loop", C.c_int32), ("pipeline_streams", C.c_int32), ("tune_wgs_per_cu", C.c_int32),
                ("tune_attn_split", C.c_int32), ("eesd_gamma", C.c_int32), ("exit_block", C.c_int32), ("temperature", C.c_float),
                ("sample_seed", C.c_uint32), ("prefill_chunk", C.c_int32), ("tune_prefill_tile", C.c_int32),
                ("tune_draft_share", C.c_int32), ("pipeline_stage_layers", C.c_int32)]


class ppsd_buffers(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("embed", "final_norm", "lm_head", "exit_norm", "exit_head")] + \
               [(n, C.POINTER(C.c_void_p)) for n in ("attn_norm", "wqkv", "wo", "mlp_norm", "wgu", "wdown")] + \
               [("workspace", C.c_void_p), ("workspace_bytes", C.c_size_t), ("stream_draft", C.c_void_p),
                ("stream_verify", C.c_void_p), ("kv_page_table", C.POINTER(C.c_int32))]


class ppsd_stats_t(C.Structure):
    _fields_ = [(n, C.c_int64) for n in ("committed", "drafts_compared", "accepted", "rejected", "steps_overlapped",
                                          "steps_draft_only", "kv_rollbacks", "steps_launched")] + \
               [("device_ms", C.c_double)] + \
               [(n, C.c_int64) for n in ("pipeline_ticks", "stage_runs", "flushed_tokens", "eesd_rounds")]


class ppsd_kernel_times_t(C.Structure):
    _fields_ = [("total_us", C.c_double * 7), ("launches", C.c_int64 * 7), ("event_overhead_us", C.c_double)]


class ppsd_launch_info_t(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("compute_units", "attn_splits", "prefill_matrix_core", "prefill_chunk", "grid_qkv",
                                          "grid_proj", "grid_gate_up", "grid_head", "draft_share_of_256", "streams",
                                          "pipeline_stages", "eesd_gamma")]


_lib = None


def library_path() -> str:
    return LIB_PATH


def load_library():
    """Loads libppsd.so (built in-tree by paper_2509_19368_amd.build) or raises."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2509_19368_amd.build` "
                          "(there is no CPU fallback)")
    lib = C.CDLL(LIB_PATH)
    vp, i32 = C.c_void_p, C.c_int32
    lib.ppsd_workspace_bytes.restype, lib.ppsd_workspace_bytes.argtypes = C.c_size_t, [C.POINTER(ppsd_config)]
    lib.ppsd_load_weights.restype = i32
    lib.ppsd_load_weights.argtypes = [C.POINTER(ppsd_config), C.POINTER(ppsd_buffers), C.POINTER(vp)]
    lib.ppsd_prefill.restype, lib.ppsd_prefill.argtypes = i32, [vp, C.POINTER(i32), i32, C.POINTER(i32)]
    lib.ppsd_decode.restype, lib.ppsd_decode.argtypes = i32, [vp, i32, C.POINTER(i32), C.POINTER(i32)]
    lib.ppsd_decode_static_scratch.restype = i32
    lib.ppsd_decode_static_scratch.argtypes = [vp, i32, C.POINTER(i32), C.POINTER(i32)]
    lib.ppsd_stats.restype, lib.ppsd_stats.argtypes = i32, [vp, C.POINTER(ppsd_stats_t)]
    lib.ppsd_read_logits.restype, lib.ppsd_read_logits.argtypes = i32, [vp, i32, i32, C.POINTER(C.c_float)]
    lib.ppsd_read_drafts.restype, lib.ppsd_read_drafts.argtypes = i32, [vp, i32, i32, C.POINTER(i32)]
    lib.ppsd_kernel_times.restype, lib.ppsd_kernel_times.argtypes = i32, [vp, C.POINTER(ppsd_kernel_times_t)]
    lib.ppsd_launch_info.restype, lib.ppsd_launch_info.argtypes = i32, [vp, C.POINTER(ppsd_launch_info_t)]
    lib.ppsd_trace_request.restype, lib.ppsd_trace_request.argtypes = i32, [vp, i32, i32]
    lib.ppsd_trace_read.restype, lib.ppsd_trace_read.argtypes = i32, [vp, i32, C.POINTER(C.c_uint64)]
    lib.ppsd_hbm_read_probe.restype = i32
    lib.ppsd_hbm_read_probe.argtypes = [vp, C.c_size_t, vp, i32, C.POINTER(C.c_float)]
    lib.ppsd_free.restype, lib.ppsd_free.argtypes = None, [vp]
    lib.ppsd_last_error.restype, lib.ppsd_last_error.argtypes = C.c_char_p, []
    _lib = lib
    return lib


def _check(rc: int):
    if rc != 0:
        raise PpsdError(rc, load_library().ppsd_last_error().decode())


def make_config(shape, max_seq: int, mode: int, kv_page_tokens: int = 16, debug_logits: int = 0,
                use_graph: bool = True, time_kernels: bool = False, engine: int = ENGINE_STREAMS,
                prefill_loop: bool = False, pipeline_streams: int = 0, tune_wgs_per_cu: int = 0,
                tune_attn_split: int = 0, eesd_gamma: int = 0, temperature: float = 0.0,
                sample_seed: int = 0, prefill_chunk: int = 0, tune_prefill_tile: int = 0,
                tune_draft_share: int = 0, pipeline_stage_layers: int = 0) -> ppsd_config:
    cfg = ppsd_config()
    for n in ("n_layers", "exit_layer", "d_model", "n_heads", "n_kv_heads", "head_dim", "d_ffn", "vocab"):
        setattr(cfg, n, int(getattr(shape, n)))
    cfg.dtype = 0 if shape.dtype == "fp32" else 1
    cfg.max_seq, cfg.kv_page_tokens, cfg.mode = int(max_seq), int(kv_page_tokens), int(mode)
    cfg.rope_base, cfg.rms_eps = float(shape.rope_base), float(shape.rms_eps)
    cfg.debug_logits, cfg.use_graph, cfg.time_kernels = int(debug_logits), int(use_graph), int(time_kernels)
    cfg.engine = int(engine)
    cfg.prefill_loop = int(prefill_loop)
    cfg.pipeline_streams = int(pipeline_streams)
    cfg.tune_wgs_per_cu = int(tune_wgs_per_cu)
    cfg.tune_attn_split = int(tune_attn_split)
    cfg.eesd_gamma = int(eesd_gamma)
    cfg.temperature, cfg.sample_seed = float(temperature), int(sample_seed)
    cfg.exit_block = int(bool(getattr(shape, "exit_block", False)))
    cfg.prefill_chunk = int(prefill_chunk)
    cfg.tune_prefill_tile = int(tune_prefill_tile)
    cfg.tune_draft_share = int(tune_draft_share)
    cfg.pipeline_stage_layers = int(pipeline_stage_layers)
    return cfg


def ppsd_workspace_bytes(cfg: ppsd_config) -> int:
    n = load_library().ppsd_workspace_bytes(C.byref(cfg))
    if n == 0:
        raise PpsdError(-1, load_library().ppsd_last_error().decode())
    return n


def hbm_read_probe(buf: torch.Tensor, iters: int = 20, stream: Optional[torch.cuda.Stream] = None) -> float:
    """Average ms per launch of the library's streaming-read kernel over `buf`."""
    stream = stream or torch.cuda.Stream()
    ms = C.c_float()
    _check(load_library().ppsd_hbm_read_probe(buf.data_ptr(), buf.numel() * buf.element_size(), stream.cuda_stream,
                                              iters, C.byref(ms)))
    return ms.value


class Session:
    """ppsd_load_weights / ppsd_prefill / ppsd_decode / ppsd_stats on device-resident weights.

    `weights` is the dict of CUDA tensors in the boundary layout (see include/ppsd.h); the
    session keeps them, the workspace tensor and the streams alive.
    """

    def __init__(self, shape, weights: dict, max_seq: int, mode: int = MODE_OVERLAP, kv_page_tokens: int = 16,
                 debug_logits: int = 0, use_graph: bool = True, time_kernels: bool = False,
                 page_table: Optional[Sequence[int]] = None, engine: int = ENGINE_STREAMS,
                 prefill_loop: bool = False, pipeline_streams: int = 0, tune_wgs_per_cu: int = 0,
                 tune_attn_split: int = 0, eesd_gamma: int = 0, temperature: float = 0.0, sample_seed: int = 0,
                 prefill_chunk: int = 0, tune_prefill_tile: int = 0, tune_draft_share: int = 0,
                 pipeline_stage_layers: int = 0):
        self.lib = load_library()
        self.shape = shape
        self.weights = weights
        self.cfg = make_config(shape, max_seq, mode, kv_page_tokens, debug_logits, use_graph, time_kernels, engine,
                               prefill_loop, pipeline_streams, tune_wgs_per_cu, tune_attn_split, eesd_gamma, temperature,
                               sample_seed, prefill_chunk, tune_prefill_tile, tune_draft_share, pipeline_stage_layers)
        nbytes = ppsd_workspace_bytes(self.cfg)
        dev = weights["embed"].device
        if dev.type != "cuda":
            raise PpsdError(-1, "weights must live on the GPU")
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=dev)
        self.stream_draft = torch.cuda.Stream(device=dev)
        self.stream_verify = torch.cuda.Stream(device=dev)
        want = torch.float32 if shape.dtype == "fp32" else torch.bfloat16

        def ptr(t: torch.Tensor, dt) -> int:
            if t.dtype != dt or not t.is_contiguous() or t.device != dev:
                raise PpsdError(-1, f"tensor has dtype {t.dtype}/contiguous {t.is_contiguous()}, need {dt}")
            return t.data_ptr()

        b = ppsd_buffers()
        b.embed, b.lm_head, b.exit_head = (ptr(weights[k], want) for k in ("embed", "lm_head", "exit_head"))
        b.final_norm, b.exit_norm = ptr(weights["final_norm"], torch.float32), ptr(weights["exit_norm"], torch.float32)
        self._arrays = {}
        for name, dt in (("attn_norm", torch.float32), ("wqkv", want), ("wo", want), ("mlp_norm", torch.float32),
                         ("wgu", want), ("wdown", want)):
            n_entries = shape.n_layers + self.cfg.exit_block
            if len(weights[name]) != n_entries:
                raise PpsdError(-1, f"{name} has {len(weights[name])} entries, the configuration needs {n_entries}")
            arr = (C.c_void_p * n_entries)(*[ptr(t, dt) for t in weights[name]])
            self._arrays[name] = arr
            setattr(b, name, C.cast(arr, C.POINTER(C.c_void_p)))
        b.workspace, b.workspace_bytes = self.workspace.data_ptr(), nbytes
        b.stream_draft, b.stream_verify = self.stream_draft.cuda_stream, self.stream_verify.cuda_stream
        if page_table is not None:
            self._pt = (C.c_int32 * len(page_table))(*page_table)
            b.kv_page_table = C.cast(self._pt, C.POINTER(C.c_int32))
        torch.cuda.synchronize(dev)            # weights may still be in flight on torch's stream
        self._ctx = C.c_void_p()
        _check(self.lib.ppsd_load_weights(C.byref(self.cfg), C.byref(b), C.byref(self._ctx)))

    # -- the four calls of the boundary -------------------------------------------------------
    def ppsd_prefill(self, prompt: Sequence[int]) -> int:
        arr = (C.c_int32 * len(prompt))(*prompt)
        first = C.c_int32()
        _check(self.lib.ppsd_prefill(self._ctx, arr, len(prompt), C.byref(first)))
        return first.value

    def ppsd_decode(self, n_tokens: int) -> List[int]:
        out = (C.c_int32 * max(n_tokens, 1))()
        n = C.c_int32()
        _check(self.lib.ppsd_decode(self._ctx, n_tokens, out, C.byref(n)))
        return list(out[: n.value])

    def ppsd_decode_static_scratch(self, n_tokens: int) -> List[int]:
        out = (C.c_int32 * max(n_tokens, 1))()
        n = C.c_int32()
        _check(self.lib.ppsd_decode_static_scratch(self._ctx, n_tokens, out, C.byref(n)))
        return list(out[: n.value])

    def ppsd_stats(self) -> dict:
        st = ppsd_stats_t()
        _check(self.lib.ppsd_stats(self._ctx, C.byref(st)))
        return {n: getattr(st, n) for n, _ in ppsd_stats_t._fields_}

    # -- parity / profiling helpers ------------------------------------------------------------
    def read_logits(self, first: int, count: int) -> torch.Tensor:
        out = torch.empty(count, self.shape.vocab, dtype=torch.float32)
        _check(self.lib.ppsd_read_logits(self._ctx, first, count, C.cast(out.data_ptr(), C.POINTER(C.c_float))))
        return out

    def read_drafts(self, first: int, count: int) -> List[int]:
        out = (C.c_int32 * max(count, 1))()
        _check(self.lib.ppsd_read_drafts(self._ctx, first, count, out))
        return list(out[:count])

    def launch_info(self) -> dict:
        li = ppsd_launch_info_t()
        _check(self.lib.ppsd_launch_info(self._ctx, C.byref(li)))
        return {n: getattr(li, n) for n, _ in ppsd_launch_info_t._fields_}

    def kernel_times(self) -> dict:
        kt = ppsd_kernel_times_t()
        _check(self.lib.ppsd_kernel_times(self._ctx, C.byref(kt)))
        out = {k: {"total_us": kt.total_us[i], "launches": kt.launches[i]} for i, k in enumerate(KERNEL_KINDS)}
        out["event_overhead_us"] = kt.event_overhead_us
        return out

    def trace_request(self, step: int, workgroup: int = 0):
        _check(self.lib.ppsd_trace_request(self._ctx, step, workgroup))

    def trace_read(self, n_phases: int) -> List[List[int]]:
        out = (C.c_uint64 * (4 * n_phases))()
        _check(self.lib.ppsd_trace_read(self._ctx, n_phases, out))
        return [list(out[4 * p: 4 * p + 4]) for p in range(n_phases)]

    def close(self):
        if getattr(self, "_ctx", None) and self._ctx.value:
            self.lib.ppsd_free(self._ctx)
            self._ctx = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
