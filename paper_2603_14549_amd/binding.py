"""ctypes binding of libasap.so: same names and arguments as include/asap.h.

Argument marshalling only -- every step of the pruning stage runs in the library's HIP
kernels.  torch tensors are used for device memory (data_ptr, strides) and for the current
HIP stream; nothing here computes.  There is no CPU fallback: if the library is missing,
load() raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import torch

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "lib", "libasap.so")

ASAP_OK, ASAP_EINVAL, ASAP_EUNSUPPORTED, ASAP_EWORKSPACE, ASAP_EHIP = 0, 1, 2, 3, 4
ASAP_F32, ASAP_BF16 = 0, 1
ASAP_MASK_OFF, ASAP_MASK_KEYBIAS = 0, 1
ASAP_ROUTE_ABSORB, ASAP_ROUTE_PAPER = 0, 1
ASAP_ROWS_ALL, ASAP_ROWS_LAST = 0, 1
ASAP_STREAMS_ONE, ASAP_STREAMS_AUTO, ASAP_STREAMS_TWO = 0, 1, 2

EXPORTS = ["asap_create", "asap_destroy", "asap_last_error", "asap_check_params", "asap_workspace_bytes",
           "asap_score", "asap_score_static", "asap_score_from_hidden", "asap_front_end_workspace_bytes", "asap_select", "asap_merge", "asap_positions", "asap_compact_kv",
           "asap_compact_kv_from_kept", "asap_compact_kv_paged", "asap_stage",
           "asap_timing_enable",
           "asap_timing_collect", "asap_theoretical_flops", "asap_flops_ratio", "asap_attention",
           "asap_attention_workspace_bytes"]

_DTYPE_CODE = {"f32": ASAP_F32, "bf16": ASAP_BF16, torch.float32: ASAP_F32, torch.bfloat16: ASAP_BF16}
_TORCH_DTYPE = {ASAP_F32: torch.float32, ASAP_BF16: torch.bfloat16}


class asap_params(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("H", ctypes.c_int32), ("Hkv", ctypes.c_int32), ("d", ctypes.c_int32),
                ("D", ctypes.c_int32), ("P", ctypes.c_int32), ("V", ctypes.c_int32), ("Tmax", ctypes.c_int32),
                ("k", ctypes.c_int32),
                ("qk_dtype", ctypes.c_int), ("h_dtype", ctypes.c_int), ("kv_dtype", ctypes.c_int),
                ("lambda_max", ctypes.c_float), ("eps", ctypes.c_float), ("sim_threshold", ctypes.c_float),
                ("merge_weight", ctypes.c_float),
                ("mask_mode", ctypes.c_int), ("route", ctypes.c_int), ("score_rows", ctypes.c_int)]


class asap_stage_io(ctypes.Structure):
    """Arguments of asap_stage (field for field the struct of include/asap.h)."""
    _vp, _i64x3 = ctypes.c_void_p, ctypes.c_int64 * 3
    _fields_ = [("q_vis", _vp), ("q_vis_stride", _i64x3), ("q_txt", _vp), ("q_txt_stride", _i64x3),
                ("k_vis", _vp), ("k_vis_stride", _i64x3), ("text_len", _vp), ("lse_extra", _vp),
                ("s_raw", _vp), ("s_hat", _vp), ("score", _vp),
                ("kept_idx", _vp), ("pruned_idx", _vp),
                ("hidden", _vp), ("hidden_stride", ctypes.c_int64 * 2),
                ("out_hidden", _vp), ("pos_out", _vp), ("new_len", _vp),
                ("assign", _vp), ("best_sim", _vp), ("wsum", _vp), ("final_idx", _vp),
                ("n_layers", ctypes.c_int32),
                ("k_src", ctypes.POINTER(_vp)), ("v_src", ctypes.POINTER(_vp)),
                ("k_dst", ctypes.POINTER(_vp)), ("v_dst", ctypes.POINTER(_vp)),
                ("workspace", _vp), ("workspace_bytes", ctypes.c_size_t)]


class AsapError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"asap status {status}: {message}")
        self.status = status


_lib = None


def lib_path() -> str:
    return _LIB_PATH


def load() -> ctypes.CDLL:
    """Loads libasap.so (built by paper_2603_14549_amd.build); raises if it is not there."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise FileNotFoundError(
            f"{_LIB_PATH} not found: build it with `python -m paper_2603_14549_amd.build` "
            "(there is no fallback path)")
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i32p, f32p, i64p = ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.POINTER(ctypes.c_int64)
    pp = ctypes.POINTER(asap_params)
    lib.asap_create.argtypes = [ctypes.POINTER(vp), ctypes.c_int]
    lib.asap_create.restype = ctypes.c_int
    lib.asap_destroy.argtypes = [vp]
    lib.asap_destroy.restype = None
    lib.asap_last_error.argtypes = [vp]
    lib.asap_last_error.restype = ctypes.c_char_p
    lib.asap_check_params.argtypes = [pp, ctypes.c_char_p, ctypes.c_size_t]
    lib.asap_check_params.restype = ctypes.c_int
    lib.asap_workspace_bytes.argtypes = [pp]
    lib.asap_workspace_bytes.restype = ctypes.c_size_t
    lib.asap_score.argtypes = [vp, pp, vp, i64p, vp, i64p, vp, i64p, i32p, f32p, f32p, f32p, f32p, vp,
                               ctypes.c_size_t, vp]
    lib.asap_score.restype = ctypes.c_int
    lib.asap_score_static.argtypes = [vp, pp, vp, i64p, vp, i64p, vp, i64p, i32p, f32p, f32p, f32p, f32p, vp]
    lib.asap_score_static.restype = ctypes.c_int
    lib.asap_front_end_workspace_bytes.argtypes = [pp]
    lib.asap_front_end_workspace_bytes.restype = ctypes.c_size_t
    lib.asap_score_from_hidden.argtypes = [vp, pp, vp, i64p, vp, ctypes.c_double, i32p, vp, i64p, vp, i64p, i32p, f32p,
                                           f32p, f32p, f32p, vp, ctypes.c_size_t, vp]
    lib.asap_score_from_hidden.restype = ctypes.c_int
    lib.asap_select.argtypes = [vp, pp, f32p, i32p, i32p, vp, ctypes.c_size_t, vp]
    lib.asap_select.restype = ctypes.c_int
    lib.asap_merge.argtypes = [vp, pp, vp, i64p, f32p, f32p, i32p, i32p, i32p, vp, i32p, i32p, i32p, f32p, f32p, i32p,
                               vp, ctypes.c_size_t, vp]
    lib.asap_merge.restype = ctypes.c_int
    lib.asap_positions.argtypes = [vp, pp, i32p, i32p, i32p, i32p, vp]
    lib.asap_positions.restype = ctypes.c_int
    lib.asap_compact_kv.argtypes = [vp, pp, ctypes.c_int32, ctypes.POINTER(vp), ctypes.POINTER(vp),
                                    ctypes.POINTER(vp), ctypes.POINTER(vp), i32p, i32p, vp]
    lib.asap_compact_kv.restype = ctypes.c_int
    lib.asap_compact_kv_from_kept.argtypes = [vp, pp, ctypes.c_int32, ctypes.POINTER(vp), ctypes.POINTER(vp),
                                              ctypes.POINTER(vp), ctypes.POINTER(vp), i32p, i32p, vp]
    lib.asap_compact_kv_from_kept.restype = ctypes.c_int
    lib.asap_stage.argtypes = [vp, pp, ctypes.POINTER(asap_stage_io), ctypes.c_int32, vp]
    lib.asap_stage.restype = ctypes.c_int
    lib.asap_compact_kv_paged.argtypes = [vp, pp, ctypes.c_int32, ctypes.POINTER(vp), ctypes.POINTER(vp),
                                          ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.c_int32, i32p,
                                          ctypes.c_int32, i32p, ctypes.c_int32, i32p, i32p, vp]
    lib.asap_compact_kv_paged.restype = ctypes.c_int
    lib.asap_attention_workspace_bytes.argtypes = [pp]
    lib.asap_attention_workspace_bytes.restype = ctypes.c_size_t
    lib.asap_attention.argtypes = [vp, pp, vp, i64p, vp, i64p, vp, i64p, f32p, vp, vp, ctypes.c_size_t, vp]
    lib.asap_attention.restype = ctypes.c_int
    lib.asap_theoretical_flops.argtypes = [i32p, i32p, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                           ctypes.POINTER(ctypes.c_double)]
    lib.asap_theoretical_flops.restype = ctypes.c_int
    lib.asap_flops_ratio.argtypes = [i32p, i32p, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                     ctypes.POINTER(ctypes.c_double)]
    lib.asap_flops_ratio.restype = ctypes.c_int
    lib.asap_timing_enable.argtypes = [vp, ctypes.c_int32]
    lib.asap_timing_enable.restype = ctypes.c_int
    lib.asap_timing_collect.argtypes = [vp, ctypes.c_char_p, ctypes.c_size_t, ctypes.POINTER(ctypes.c_double),
                                        ctypes.POINTER(ctypes.c_int32), ctypes.c_int32]
    lib.asap_timing_collect.restype = ctypes.c_int32
    _lib = lib
    return lib


def make_params(B, H, Hkv, d, D, P, V, Tmax, k, qk_dtype, h_dtype, kv_dtype, lambda_max=1.0, eps=1e-6,
                sim_threshold=float("-inf"), merge_weight=1.0, mask_mode=ASAP_MASK_KEYBIAS,
                route=ASAP_ROUTE_ABSORB, score_rows=ASAP_ROWS_ALL) -> asap_params:
    return asap_params(B, H, Hkv, d, D, P, V, Tmax, k, _DTYPE_CODE[qk_dtype], _DTYPE_CODE[h_dtype],
                       _DTYPE_CODE[kv_dtype], lambda_max, eps, sim_threshold, merge_weight, mask_mode, route,
                       score_rows)


def params_from_config(cfg, **overrides) -> asap_params:
    """asap_params for a synth.StageConfig."""
    return make_params(cfg.B, cfg.H, cfg.Hkv, cfg.d, cfg.D, cfg.P, cfg.V, cfg.Tmax, cfg.k, cfg.qk_dtype,
                       cfg.h_dtype, cfg.kv_dtype, **overrides)


def asap_check_params(p: asap_params):
    buf = ctypes.create_string_buffer(256)
    st = load().asap_check_params(ctypes.byref(p), buf, 256)
    return st, buf.value.decode()


def asap_workspace_bytes(p: asap_params) -> int:
    return int(load().asap_workspace_bytes(ctypes.byref(p)))


def asap_front_end_workspace_bytes(p: asap_params) -> int:
    return int(load().asap_front_end_workspace_bytes(ctypes.byref(p)))


def asap_attention_workspace_bytes(p: asap_params) -> int:
    return int(load().asap_attention_workspace_bytes(ctypes.byref(p)))


def _i32_array(values):
    return (ctypes.c_int32 * len(values))(*[int(v) for v in values])


def asap_theoretical_flops(layers, tokens, d: int, m: int) -> float:
    """Eq. 7 through the library (host arithmetic)."""
    out = ctypes.c_double()
    st = load().asap_theoretical_flops(_i32_array(layers), _i32_array(tokens), len(layers), d, m, ctypes.byref(out))
    if st != ASAP_OK:
        raise AsapError(st, "asap_theoretical_flops: invalid arguments")
    return out.value


def asap_flops_ratio(layers, tokens, v0: int, d: int, m: int) -> float:
    """Eq. 8 through the library (host arithmetic)."""
    out = ctypes.c_double()
    st = load().asap_flops_ratio(_i32_array(layers), _i32_array(tokens), len(layers), v0, d, m, ctypes.byref(out))
    if st != ASAP_OK:
        raise AsapError(st, "asap_flops_ratio: invalid arguments")
    return out.value


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _strides(t: torch.Tensor, n: int):
    assert t.stride(-1) == 1, "last dimension must be contiguous"
    return (ctypes.c_int64 * n)(*[t.stride(i) for i in range(n)])


def _stream(stream) -> ctypes.c_void_p:
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


class Context:
    """asap_ctx for one device."""

    def __init__(self, device: int = 0):
        self._lib = load()
        self._h = ctypes.c_void_p()
        st = self._lib.asap_create(ctypes.byref(self._h), device)
        if st != ASAP_OK:
            raise AsapError(st, f"asap_create(device={device}) failed")
        self.device = device

    def close(self):
        if self._h:
            self._lib.asap_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def last_error(self) -> str:
        return self._lib.asap_last_error(self._h).decode()

    def _check(self, st: int):
        if st != ASAP_OK:
            raise AsapError(st, self.last_error())

    def asap_timing_enable(self, max_launches: int):
        self._check(self._lib.asap_timing_enable(self._h, max_launches))

    def asap_timing_collect(self) -> dict:
        """{kernel name: (total milliseconds, launches)} since the last collect."""
        names = ctypes.create_string_buffer(4096)
        ms = (ctypes.c_double * 64)()
        cnt = (ctypes.c_int32 * 64)()
        n = self._lib.asap_timing_collect(self._h, names, 4096, ms, cnt, 64)
        if n < 0:
            raise AsapError(ASAP_EHIP, "asap_timing_collect failed")
        keys = names.value.decode().split("\n")[:n]
        return {k: (ms[i], cnt[i]) for i, k in enumerate(keys)}

    # ---- the four calls, arguments as in asap.h -------------------------------------------
    def asap_score(self, p, q_vis, q_txt, k_vis, text_len, lse_extra, s_raw, s_hat, score, workspace,
                   stream=None):
        self._check(self._lib.asap_score(
            self._h, ctypes.byref(p), _ptr(q_vis), _strides(q_vis, 3), _ptr(q_txt), _strides(q_txt, 3),
            _ptr(k_vis), _strides(k_vis, 3), _ptr(text_len), _ptr(lse_extra), _ptr(s_raw), _ptr(s_hat),
            _ptr(score), _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream)))

    def asap_score_static(self, p, q_vis, q_txt, k_vis, text_len, lse_extra, s_raw, s_hat, score, stream=None):
        self._check(self._lib.asap_score_static(
            self._h, ctypes.byref(p), _ptr(q_vis), _strides(q_vis, 3), _ptr(q_txt), _strides(q_txt, 3),
            _ptr(k_vis), _strides(k_vis, 3), _ptr(text_len), _ptr(lse_extra), _ptr(s_raw), _ptr(s_hat),
            _ptr(score), _stream(stream)))

    def asap_score_from_hidden(self, p, hidden, w_q, rope_theta, vis_positions, q_txt, k_vis, text_len, lse_extra,
                               s_raw, s_hat, score, workspace, stream=None):
        self._check(self._lib.asap_score_from_hidden(
            self._h, ctypes.byref(p), _ptr(hidden), _strides(hidden, 2), _ptr(w_q), float(rope_theta),
            _ptr(vis_positions), _ptr(q_txt), _strides(q_txt, 3), _ptr(k_vis), _strides(k_vis, 3), _ptr(text_len),
            _ptr(lse_extra), _ptr(s_raw), _ptr(s_hat), _ptr(score), _ptr(workspace),
            workspace.numel() * workspace.element_size(), _stream(stream)))

    def asap_select(self, p, score, kept_idx, pruned_idx, workspace, stream=None):
        self._check(self._lib.asap_select(
            self._h, ctypes.byref(p), _ptr(score), _ptr(kept_idx), _ptr(pruned_idx), _ptr(workspace),
            workspace.numel() * workspace.element_size(), _stream(stream)))

    def asap_merge(self, p, hidden, s_raw, s_hat, text_len, kept_idx, pruned_idx, out_hidden, pos_out, new_len,
                   assign, best_sim, wsum, final_idx, workspace, stream=None):
        self._check(self._lib.asap_merge(
            self._h, ctypes.byref(p), _ptr(hidden), _strides(hidden, 2), _ptr(s_raw), _ptr(s_hat), _ptr(text_len),
            _ptr(kept_idx), _ptr(pruned_idx), _ptr(out_hidden), _ptr(pos_out), _ptr(new_len), _ptr(assign),
            _ptr(best_sim), _ptr(wsum), _ptr(final_idx), _ptr(workspace),
            workspace.numel() * workspace.element_size(), _stream(stream)))

    def asap_attention(self, p, q, k, v, s_hat, out, workspace, stream=None):
        self._check(self._lib.asap_attention(
            self._h, ctypes.byref(p), _ptr(q), _strides(q, 3), _ptr(k), _strides(k, 3), _ptr(v), _strides(v, 3),
            _ptr(s_hat), _ptr(out), _ptr(workspace), workspace.numel() * workspace.element_size(),
            _stream(stream)))

    def asap_positions(self, p, kept_idx, text_len, pos_out, new_len, stream=None):
        self._check(self._lib.asap_positions(
            self._h, ctypes.byref(p), _ptr(kept_idx), _ptr(text_len), _ptr(pos_out), _ptr(new_len),
            _stream(stream)))

    def asap_compact_kv(self, p, k_src: Sequence[torch.Tensor], v_src, k_dst, v_dst, pos_out, new_len,
                        stream=None):
        n = len(k_src)
        arr = lambda ts: (ctypes.c_void_p * n)(*[t.data_ptr() for t in ts])
        self._check(self._lib.asap_compact_kv(
            self._h, ctypes.byref(p), n, arr(k_src), arr(v_src), arr(k_dst), arr(v_dst), _ptr(pos_out),
            _ptr(new_len), _stream(stream)))

    def asap_compact_kv_from_kept(self, p, k_src, v_src, k_dst, v_dst, final_idx, text_len, stream=None):
        n = len(k_src)
        arr = lambda ts: (ctypes.c_void_p * n)(*[t.data_ptr() for t in ts])
        self._check(self._lib.asap_compact_kv_from_kept(
            self._h, ctypes.byref(p), n, arr(k_src), arr(v_src), arr(k_dst), arr(v_dst), _ptr(final_idx),
            _ptr(text_len), _stream(stream)))

    def asap_stage(self, p, io: asap_stage_io, two_streams: int = ASAP_STREAMS_AUTO, stream=None):
        self._check(self._lib.asap_stage(self._h, ctypes.byref(p), ctypes.byref(io), int(two_streams),
                                         _stream(stream)))

    def asap_compact_kv_paged(self, p, k_src_pool: Sequence[torch.Tensor], v_src_pool, k_dst_pool, v_dst_pool,
                              page_size: int, src_table, dst_table, pos_out, new_len, stream=None):
        """Pools [n_pages,Hkv,page_size,d] per layer; src_table / dst_table [B, pages per sequence] int32."""
        n = len(k_src_pool)
        arr = lambda ts: (ctypes.c_void_p * n)(*[t.data_ptr() for t in ts])
        self._check(self._lib.asap_compact_kv_paged(
            self._h, ctypes.byref(p), n, arr(k_src_pool), arr(v_src_pool), arr(k_dst_pool), arr(v_dst_pool),
            int(page_size), _ptr(src_table), int(src_table.stride(0)), _ptr(dst_table), int(dst_table.stride(0)),
            _ptr(pos_out), _ptr(new_len), _stream(stream)))
