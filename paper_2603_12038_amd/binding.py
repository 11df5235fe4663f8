"""ctypes binding of libsfi.so: argument marshalling only; every step of the path runs in the HIP kernels.

Functions carry the names of the C entry points declared in include/sfi.h.  Tensors are torch
tensors on the GPU (torch is used for device memory and streams only); their ``data_ptr()`` goes
straight to the library.  There is no fallback: if the library is not built, loading fails.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Tuple

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libsfi.so")

SFI_N_STAGES = 8
STAGE_NAMES = ("attn", "merge", "score", "cand", "count", "write", "attn_gather_mixed", "reorg")


class SfiError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {sfi_strerror(code)} ({code})")


class SfiConfig(C.Structure):
    _fields_ = [
        ("batch", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
        ("max_ctx", C.c_int32), ("max_budget", C.c_int32), ("n_sink", C.c_int32), ("recent", C.c_int32),
        ("scale", C.c_float), ("selector_mode", C.c_int32),
        ("k_stride_b", C.c_int64), ("k_stride_h", C.c_int64), ("k_stride_t", C.c_int64),
        ("v_stride_b", C.c_int64), ("v_stride_h", C.c_int64), ("v_stride_t", C.c_int64),
        ("gamma", C.c_float), ("beta", C.c_float), ("p", C.c_float), ("eta", C.c_float),
        ("lambda_clip", C.c_float), ("alpha_soft", C.c_float), ("alpha_cross", C.c_float), ("temp", C.c_float),
        ("eps", C.c_float), ("nms_radius", C.c_int32), ("alpha", C.c_float),
        ("page_size", C.c_int32), ("k_stride_page", C.c_int64), ("v_stride_page", C.c_int64),
        ("out_bf16", C.c_int32),
    ]


_lib: Optional[C.CDLL] = None

EXPORTS = ("sfi_workspace_bytes", "sfi_create", "sfi_set_block_table", "sfi_destroy", "sfi_strerror", "sfi_slow_step", "sfi_slow_attn",
           "sfi_slow_select", "sfi_evidence_add", "sfi_evidence_add_causal", "sfi_evidence_select", "sfi_dense_attn",
           "sfi_fast_step", "sfi_fast_step_static", "sfi_fast_step_floor", "sfi_dense_attn_floor", "sfi_reorg", "sfi_fast_step_compact", "sfi_mixed_step", "sfi_mixed_step_compact", "sfi_step_begin", "sfi_mixed_step_desc", "sfi_trigger", "sfi_advance", "sfi_set_profiling", "sfi_stage_times",
           "sfi_set_tuning", "sfi_set_dense_k_layout", "sfi_set_mixed_plan", "sfi_plan_splits", "sfi_device_status", "sfi_query_splits")


def load_library() -> C.CDLL:
    """Load the in-tree libsfi.so; raises if it has not been built (no fallback path exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(f"{LIB_PATH} is not built: run `python -c 'import __graft_entry__ as g; g.build()'`")
    lib = C.CDLL(LIB_PATH)
    vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
    lib.sfi_workspace_bytes.restype = C.c_size_t
    lib.sfi_workspace_bytes.argtypes = [C.POINTER(SfiConfig)]
    lib.sfi_create.restype = C.c_int
    lib.sfi_create.argtypes = [C.POINTER(SfiConfig), vp, C.c_size_t, C.POINTER(vp)]
    lib.sfi_set_block_table.restype = C.c_int
    lib.sfi_set_block_table.argtypes = [vp, vp, i32, i32]
    lib.sfi_destroy.restype = C.c_int
    lib.sfi_destroy.argtypes = [vp]
    lib.sfi_strerror.restype = C.c_char_p
    lib.sfi_strerror.argtypes = [C.c_int]
    lib.sfi_slow_step.restype = C.c_int
    lib.sfi_slow_step.argtypes = [vp, vp, vp, vp, vp, i32, i32, vp, vp, vp, vp]
    lib.sfi_slow_attn.restype = C.c_int
    lib.sfi_slow_attn.argtypes = [vp, vp, vp, vp, vp, i32, vp, vp]
    lib.sfi_slow_select.restype = C.c_int
    lib.sfi_slow_select.argtypes = [vp, vp, i32, i32, vp, vp, vp]
    lib.sfi_evidence_add.restype = C.c_int
    lib.sfi_evidence_add.argtypes = [vp, vp, vp, vp, vp, i32, vp, i32, vp]
    lib.sfi_evidence_add_causal.restype = C.c_int
    lib.sfi_evidence_add_causal.argtypes = [vp, vp, vp, vp, vp, vp, i32, vp, i32, vp]
    lib.sfi_evidence_select.restype = C.c_int
    lib.sfi_evidence_select.argtypes = [vp, i32, vp, i32, i32, vp, vp, vp]
    lib.sfi_dense_attn.restype = C.c_int
    lib.sfi_dense_attn.argtypes = [vp, vp, vp, vp, vp, i32, vp, vp]
    lib.sfi_fast_step.restype = C.c_int
    lib.sfi_fast_step.argtypes = [vp, vp, vp, vp, vp, vp, i32, vp, vp, vp, vp]
    lib.sfi_fast_step_static.restype = C.c_int
    lib.sfi_fast_step_static.argtypes = [C.POINTER(SfiConfig), vp, vp, vp, vp, vp, i32, vp, vp, vp, vp]
    lib.sfi_dense_attn_floor.restype = C.c_int
    lib.sfi_dense_attn_floor.argtypes = [vp, vp, vp, vp, i32, i32, vp]
    lib.sfi_fast_step_floor.restype = C.c_int
    lib.sfi_fast_step_floor.argtypes = [vp, vp, vp, vp, vp, vp, i32, vp, vp, vp, i32, vp]
    lib.sfi_reorg.restype = C.c_int
    lib.sfi_reorg.argtypes = [vp, vp, vp, vp, vp, i32, vp, vp, vp, vp, i64, i64, i32, vp]
    lib.sfi_fast_step_compact.restype = C.c_int
    lib.sfi_fast_step_compact.argtypes = [vp, vp, vp, vp, i64, i64, i32, vp, i32, vp, vp, vp, vp, vp, vp]
    lib.sfi_mixed_step.restype = C.c_int
    lib.sfi_mixed_step.argtypes = [vp, vp, vp, vp, vp, vp, vp, i32, i32, vp, vp, vp, vp]
    lib.sfi_mixed_step_compact.restype = C.c_int
    lib.sfi_mixed_step_compact.argtypes = [vp, vp, vp, vp, vp, vp, vp, i32, i32, vp, vp, vp, vp, vp, i64, i64, i32, vp]
    lib.sfi_step_begin.restype = C.c_int
    lib.sfi_step_begin.argtypes = [vp, vp, vp, vp, i32, i32, i32, vp]
    lib.sfi_mixed_step_desc.restype = C.c_int
    lib.sfi_mixed_step_desc.argtypes = [vp, vp, vp, vp, vp, i32, i32, vp, vp, vp, vp]
    lib.sfi_trigger.restype = C.c_int
    lib.sfi_trigger.argtypes = [vp, vp, vp, i32, i32, vp, vp, vp]
    lib.sfi_advance.restype = C.c_int
    lib.sfi_advance.argtypes = [vp, vp, vp, vp]
    lib.sfi_set_profiling.restype = C.c_int
    lib.sfi_set_profiling.argtypes = [vp, C.c_int]
    lib.sfi_stage_times.restype = C.c_int
    lib.sfi_stage_times.argtypes = [vp, C.POINTER(C.c_float), C.POINTER(C.c_int32)]
    lib.sfi_set_tuning.restype = C.c_int
    lib.sfi_set_tuning.argtypes = [vp, i32, i32, i32]
    lib.sfi_set_dense_k_layout.restype = C.c_int
    lib.sfi_set_dense_k_layout.argtypes = [vp, i32]
    lib.sfi_set_mixed_plan.restype = C.c_int
    lib.sfi_set_mixed_plan.argtypes = [vp, i32]
    lib.sfi_plan_splits.restype = C.c_int
    lib.sfi_plan_splits.argtypes = [vp, i32, i32, C.POINTER(i32), C.POINTER(i32)]
    lib.sfi_device_status.restype = C.c_int
    lib.sfi_device_status.argtypes = [vp, C.POINTER(i32), i32, vp]
    lib.sfi_query_splits.restype = C.c_int
    lib.sfi_query_splits.argtypes = [vp, C.POINTER(i32), C.POINTER(i32)]
    _lib = lib
    return lib


def _ptr(t) -> Optional[int]:
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


def _check(rc: int, where: str) -> None:
    if rc != 0:
        raise SfiError(rc, where)


def sfi_strerror(code: int) -> str:
    return load_library().sfi_strerror(code).decode()


def sfi_workspace_bytes(cfg: SfiConfig) -> int:
    return int(load_library().sfi_workspace_bytes(C.byref(cfg)))


def sfi_create(cfg: SfiConfig, workspace, workspace_bytes: int) -> int:
    """Returns the opaque context handle (an integer address); raises SfiError on a bad configuration."""
    h = C.c_void_p()
    _check(load_library().sfi_create(C.byref(cfg), _ptr(workspace), workspace_bytes, C.byref(h)), "sfi_create")
    return h.value


def sfi_set_block_table(ctx, block_table, n_blocks: int) -> None:
    """block_table: int32 device tensor [B, pages per sequence] (or None to detach)."""
    stride = 0 if block_table is None else block_table.stride(0)
    _check(load_library().sfi_set_block_table(ctx, _ptr(block_table), stride, n_blocks), "sfi_set_block_table")


def sfi_destroy(ctx: int) -> None:
    _check(load_library().sfi_destroy(ctx), "sfi_destroy")


def sfi_slow_step(ctx, q, K, V, ctx_len, max_len, budget, out, sel_idx, n_sel, stream=None) -> None:
    _check(load_library().sfi_slow_step(ctx, _ptr(q), _ptr(K), _ptr(V), _ptr(ctx_len), max_len, budget, _ptr(out),
                                        _ptr(sel_idx), _ptr(n_sel), _stream(stream)), "sfi_slow_step")


def sfi_slow_attn(ctx, q, K, V, ctx_len, max_len, out, stream=None) -> None:
    _check(load_library().sfi_slow_attn(ctx, _ptr(q), _ptr(K), _ptr(V), _ptr(ctx_len), max_len, _ptr(out),
                                        _stream(stream)), "sfi_slow_attn")


def sfi_slow_select(ctx, ctx_len, max_len, budget, sel_idx, n_sel, stream=None) -> None:
    _check(load_library().sfi_slow_select(ctx, _ptr(ctx_len), max_len, budget, _ptr(sel_idx), _ptr(n_sel),
                                          _stream(stream)), "sfi_slow_select")


def sfi_evidence_add(ctx, q, K, V, ctx_len, max_len, out, first: bool, stream=None) -> None:
    _check(load_library().sfi_evidence_add(ctx, _ptr(q), _ptr(K), _ptr(V), _ptr(ctx_len), max_len, _ptr(out),
                                           1 if first else 0, _stream(stream)), "sfi_evidence_add")


def sfi_evidence_add_causal(ctx, q, K, V, ctx_len, q_len, max_len, out, first: bool, stream=None) -> None:
    _check(load_library().sfi_evidence_add_causal(ctx, _ptr(q), _ptr(K), _ptr(V), _ptr(ctx_len), _ptr(q_len), max_len,
                                                  _ptr(out), 1 if first else 0, _stream(stream)), "sfi_evidence_add_causal")


def sfi_evidence_select(ctx, n_added: int, ctx_len, max_len, budget, sel_idx, n_sel, stream=None) -> None:
    _check(load_library().sfi_evidence_select(ctx, n_added, _ptr(ctx_len), max_len, budget, _ptr(sel_idx), _ptr(n_sel),
                                              _stream(stream)), "sfi_evidence_select")


def sfi_dense_attn(ctx, q, K, V, ctx_len, max_len, out, stream=None) -> None:
    _check(load_library().sfi_dense_attn(ctx, _ptr(q), _ptr(K), _ptr(V), _ptr(ctx_len), max_len, _ptr(out),
                                         _stream(stream)), "sfi_dense_attn")


def sfi_fast_step(ctx, q, K, V, sel_idx, n_sel, sel_stride, recent_start, ctx_len, out, stream=None) -> None:
    _check(load_library().sfi_fast_step(ctx, _ptr(q), _ptr(K), _ptr(V), _ptr(sel_idx), _ptr(n_sel), sel_stride,
                                        _ptr(recent_start), _ptr(ctx_len), _ptr(out), _stream(stream)),
           "sfi_fast_step")


def sfi_fast_step_static(cfg: SfiConfig, q, K, V, sel_idx, n_sel, sel_stride, recent_start, ctx_len, out, stream=None) -> None:
    """The fast step on the library's static scratch: no context, no workspace (cfg is the host-side SfiConfig)."""
    _check(load_library().sfi_fast_step_static(C.byref(cfg), _ptr(q), _ptr(K), _ptr(V), _ptr(sel_idx), _ptr(n_sel),
                                               sel_stride, _ptr(recent_start), _ptr(ctx_len), _ptr(out),
                                               _stream(stream)), "sfi_fast_step_static")


def sfi_dense_attn_floor(ctx, K, V, ctx_len, max_len, variant: int, stream=None) -> None:
    """Memory skeleton of the dense launch (measurement aid): variant 0 = the kernel's K layout, 1 = whole-line K loads;
    + 16 * u: every wave also sleeps u x 64 cycles after each half of each tile; + 2048 (4096): a fifth wave per workgroup
    stores what the slow step would expose while the four read (all to the same 2 KB)."""
    _check(load_library().sfi_dense_attn_floor(ctx, _ptr(K), _ptr(V), _ptr(ctx_len), max_len, variant, _stream(stream)),
           "sfi_dense_attn_floor")


def sfi_fast_step_floor(ctx, q, K, V, sel_idx, n_sel, sel_stride, recent_start, ctx_len, out, variant: int, stream=None) -> None:
    """Memory skeleton of the fast step (measurement aid): variant bit 0 = with the record hand-over, bit 1 = all of a
    wave's rows requested at once into LDS, bits 2-3 = 1: scalars and indices only, 2: the bare launch."""
    _check(load_library().sfi_fast_step_floor(ctx, _ptr(q), _ptr(K), _ptr(V), _ptr(sel_idx), _ptr(n_sel), sel_stride,
                                              _ptr(recent_start), _ptr(ctx_len), _ptr(out), variant, _stream(stream)),
           "sfi_fast_step_floor")


def sfi_reorg(ctx, K, V, sel_idx, n_sel, sel_stride, ctx_len, is_slow, Kc, Vc, stream=None) -> None:
    """Kc / Vc: bf16 tensors [B, Hkv, c_rows, 128] with contiguous rows; strides are taken from them."""
    assert Kc.stride() == Vc.stride() and Kc.stride(3) == 1 and Kc.stride(2) == Kc.shape[3]
    _check(load_library().sfi_reorg(ctx, _ptr(K), _ptr(V), _ptr(sel_idx), _ptr(n_sel), sel_stride, _ptr(ctx_len),
                                    _ptr(is_slow), _ptr(Kc), _ptr(Vc), Kc.stride(0), Kc.stride(1), Kc.shape[2],
                                    _stream(stream)), "sfi_reorg")


def sfi_fast_step_compact(ctx, q, Kc, Vc, n_sel, sel_stride, K, V, recent_start, ctx_len, out, stream=None) -> None:
    assert Kc.stride() == Vc.stride() and Kc.stride(3) == 1 and Kc.stride(2) == Kc.shape[3]
    _check(load_library().sfi_fast_step_compact(ctx, _ptr(q), _ptr(Kc), _ptr(Vc), Kc.stride(0), Kc.stride(1),
                                                Kc.shape[2], _ptr(n_sel), sel_stride, _ptr(K), _ptr(V),
                                                _ptr(recent_start), _ptr(ctx_len), _ptr(out), _stream(stream)),
           "sfi_fast_step_compact")


def sfi_mixed_step(ctx, q, K, V, is_slow, ctx_len, recent_start, max_len, budget, out, sel_idx, n_sel,
                   stream=None) -> None:
    _check(load_library().sfi_mixed_step(ctx, _ptr(q), _ptr(K), _ptr(V), _ptr(is_slow), _ptr(ctx_len),
                                         _ptr(recent_start), max_len, budget, _ptr(out), _ptr(sel_idx),
                                         _ptr(n_sel), _stream(stream)), "sfi_mixed_step")


def sfi_mixed_step_compact(ctx, q, K, V, is_slow, ctx_len, recent_start, max_len, budget, out, sel_idx, n_sel, Kc, Vc,
                           stream=None) -> None:
    assert Kc.stride() == Vc.stride() and Kc.stride(3) == 1 and Kc.stride(2) == Kc.shape[3]
    _check(load_library().sfi_mixed_step_compact(ctx, _ptr(q), _ptr(K), _ptr(V), _ptr(is_slow), _ptr(ctx_len),
                                                 _ptr(recent_start), max_len, budget, _ptr(out), _ptr(sel_idx),
                                                 _ptr(n_sel), _ptr(Kc), _ptr(Vc), Kc.stride(0), Kc.stride(1), Kc.shape[2],
                                                 _stream(stream)), "sfi_mixed_step_compact")


def sfi_step_begin(ctx, desc, last_token, trigger_bitmap, vocab_size, t_max, advance: bool, stream=None) -> None:
    """desc: int32 device tensor [B, 4] = (ctx_len, recent_start, is_slow, since_slow) per sequence."""
    _check(load_library().sfi_step_begin(ctx, _ptr(desc), _ptr(last_token), _ptr(trigger_bitmap), vocab_size, t_max,
                                         1 if advance else 0, _stream(stream)), "sfi_step_begin")


def sfi_mixed_step_desc(ctx, q, K, V, desc, max_len, budget, out, sel_idx, n_sel, stream=None) -> None:
    _check(load_library().sfi_mixed_step_desc(ctx, _ptr(q), _ptr(K), _ptr(V), _ptr(desc), max_len, budget, _ptr(out),
                                              _ptr(sel_idx), _ptr(n_sel), _stream(stream)), "sfi_mixed_step_desc")


def sfi_trigger(ctx, last_token, trigger_bitmap, vocab_size, t_max, since_slow, is_slow, stream=None) -> None:
    _check(load_library().sfi_trigger(ctx, _ptr(last_token), _ptr(trigger_bitmap), vocab_size, t_max, _ptr(since_slow),
                                      _ptr(is_slow), _stream(stream)), "sfi_trigger")


def sfi_advance(ctx, ctx_len, recent_start, stream=None) -> None:
    _check(load_library().sfi_advance(ctx, _ptr(ctx_len), _ptr(recent_start), _stream(stream)), "sfi_advance")


def sfi_set_profiling(ctx, max_calls: int) -> None:
    _check(load_library().sfi_set_profiling(ctx, int(max_calls)), "sfi_set_profiling")


def sfi_stage_times(ctx):
    """(sum of elapsed ms per stage, launches per stage) over the calls recorded since profiling was switched on."""
    ms = (C.c_float * SFI_N_STAGES)()
    cnt = (C.c_int32 * SFI_N_STAGES)()
    _check(load_library().sfi_stage_times(ctx, ms, cnt), "sfi_stage_times")
    return [float(x) for x in ms], [int(x) for x in cnt]


def sfi_set_tuning(ctx, dense_target_wgs: int = 0, fast_tiles_per_wave: int = 0, fast_merge: int = 0) -> None:
    _check(load_library().sfi_set_tuning(ctx, dense_target_wgs, fast_tiles_per_wave, fast_merge), "sfi_set_tuning")


def sfi_set_mixed_plan(ctx, on: bool) -> None:
    _check(load_library().sfi_set_mixed_plan(ctx, int(on)), "sfi_set_mixed_plan")


def sfi_set_dense_k_layout(ctx, whole_lines: bool) -> None:
    _check(load_library().sfi_set_dense_k_layout(ctx, 1 if whole_lines else 0), "sfi_set_dense_k_layout")


def sfi_plan_splits(ctx, max_len: int, sel_stride: int) -> Tuple[int, int]:
    d, f = C.c_int32(), C.c_int32()
    _check(load_library().sfi_plan_splits(ctx, max_len, sel_stride, C.byref(d), C.byref(f)), "sfi_plan_splits")
    return d.value, f.value


GUARD_CTX_LEN, GUARD_N_SEL, GUARD_SEL_IDX, GUARD_BLOCK = 1, 2, 4, 8


def sfi_device_status(ctx, clear: bool = True, stream=None) -> int:
    """SFI_GUARD_* bits of device-side inputs the kernels had to clamp (blocks until `stream` is done)."""
    flags = C.c_int32()
    _check(load_library().sfi_device_status(ctx, C.byref(flags), 1 if clear else 0, _stream(stream)),
           "sfi_device_status")
    return flags.value


def sfi_query_splits(ctx) -> Tuple[int, int]:
    d, f = C.c_int32(), C.c_int32()
    _check(load_library().sfi_query_splits(ctx, C.byref(d), C.byref(f)), "sfi_query_splits")
    return d.value, f.value


class SfiContext:
    """Owns the workspace tensor and the context handle for one (shape, K/V layout)."""

    def __init__(self, B, Hq, Hkv, max_ctx, max_budget, n_sink, recent, K, V, scale: float = 0.0, device="cuda",
                 selector: Optional[dict] = None, alpha: float = 0.0, page_size: int = 0, page_layout: str = "thd",
                 out_bf16: bool = False):
        """selector: None for mode 0, or the mode-1 hyper-parameters as a dict with the keys gamma, beta, p,
        eta, lambda_clip, alpha_soft, alpha_cross, temp, eps, nms_radius (all required: the paper fixes none
        of the prior's)."""
        import torch

        assert K.dtype == torch.bfloat16 and V.dtype == torch.bfloat16 and K.dim() == 4 and K.stride(3) == 1
        cfg = SfiConfig()
        cfg.page_size = page_size
        cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim = B, Hq, Hkv, K.shape[3]
        cfg.max_ctx, cfg.max_budget, cfg.n_sink, cfg.recent = max_ctx, max_budget, n_sink, recent
        cfg.scale, cfg.selector_mode = scale, 0 if selector is None else 1
        cfg.alpha = alpha
        cfg.out_bf16 = 1 if out_bf16 else 0
        if selector is not None:
            for k in ("gamma", "beta", "p", "eta", "lambda_clip", "alpha_soft", "alpha_cross", "temp", "eps"):
                setattr(cfg, k, float(selector[k]))
            cfg.nms_radius = int(selector["nms_radius"])
        if page_size:
            # K, V: block pools, [n_blocks, page_size, Hkv, d] ("thd") or [n_blocks, Hkv, page_size, d] ("htd")
            t, hd = (1, 2) if page_layout == "thd" else (2, 1)
            assert K.shape[t] == page_size and K.shape[hd] == Hkv and V.shape == K.shape
            cfg.k_stride_b, cfg.k_stride_h, cfg.k_stride_t, cfg.k_stride_page = 0, K.stride(hd), K.stride(t), K.stride(0)
            cfg.v_stride_b, cfg.v_stride_h, cfg.v_stride_t, cfg.v_stride_page = 0, V.stride(hd), V.stride(t), V.stride(0)
        else:
            cfg.k_stride_b, cfg.k_stride_h, cfg.k_stride_t = K.stride(0), K.stride(1), K.stride(2)
            cfg.v_stride_b, cfg.v_stride_h, cfg.v_stride_t = V.stride(0), V.stride(1), V.stride(2)
        self.cfg = cfg
        nbytes = sfi_workspace_bytes(cfg)
        if nbytes == 0:
            raise SfiError(-1, "sfi_workspace_bytes")
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=device)
        self.handle = sfi_create(cfg, self.workspace, nbytes)

    def close(self):
        if self.handle:
            sfi_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
