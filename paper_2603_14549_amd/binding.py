"""ctypes binding of libasap.so: same names and arguments as include/asap.h.

Argument marshalling only -- every step of the pruning stage runs in the library's HIP
kernels.  torch tensors are used for device memory (data_ptr, strides) and for the current
HIP stream; nothing here computes.  There is no CPU fallback: if the library is missing,
load() raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence

import torch

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "lib", "libasap.so")

ASAP_OK, ASAP_EINVAL, ASAP_EUNSUPPORTED, ASAP_EWORKSPACE, ASAP_EHIP = 0, 1, 2, 3, 4
ASAP_F32, ASAP_BF16 = 0, 1
ASAP_MASK_OFF, ASAP_MASK_KEYBIAS = 0, 1
ASAP_ROUTE_ABSORB, ASAP_ROUTE_PAPER = 0, 1

EXPORTS = ["asap_create", "asap_destroy", "asap_last_error", "asap_check_params", "asap_workspace_bytes",
           "asap_score", "asap_select", "asap_merge", "asap_positions", "asap_compact_kv",
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
                ("mask_mode", ctypes.c_int), ("route", ctypes.c_int)]


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
                route=ASAP_ROUTE_ABSORB) -> asap_params:
    return asap_params(B, H, Hkv, d, D, P, V, Tmax, k, _DTYPE_CODE[qk_dtype], _DTYPE_CODE[h_dtype],
                       _DTYPE_CODE[kv_dtype], lambda_max, eps, sim_threshold, merge_weight, mask_mode, route)


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

    def asap_stage(self, p, io: asap_stage_io, two_streams: bool = True, stream=None):
        self._check(self._lib.asap_stage(self._h, ctypes.byref(p), ctypes.byref(io), 1 if two_streams else 0,
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


class StageBuffers:
    """Device buffers of one pruning stage (outputs + workspace), allocated once with torch."""

    def __init__(self, p: asap_params, n_layers: int, device="cuda:0"):
        B, V, k, D = p.B, p.V, p.k, p.D
        Nout = p.P + p.k + p.Tmax
        f32, i32 = torch.float32, torch.int32
        dev = device
        self.s_raw = torch.empty(B, V, dtype=f32, device=dev)
        self.s_hat = torch.empty(B, V, dtype=f32, device=dev)
        self.score = torch.empty(B, V, dtype=f32, device=dev)
        self.kept_idx = torch.empty(B, k, dtype=i32, device=dev)
        self.pruned_idx = torch.empty(B, max(V - k, 1), dtype=i32, device=dev)
        self.out_hidden = torch.zeros(B, Nout, D, dtype=_TORCH_DTYPE[p.h_dtype], device=dev)
        self.pos_out = torch.empty(B, Nout, dtype=i32, device=dev)
        self.new_len = torch.empty(B, dtype=i32, device=dev)
        # the same two, written by asap_positions right after the selection (read by the K/V
        # compaction while the merge still runs)
        self.pos_early = torch.empty(B, Nout, dtype=i32, device=dev)
        self.new_len_early = torch.empty(B, dtype=i32, device=dev)
        self.assign = torch.empty(B, max(V - k, 1), dtype=i32, device=dev)      # paper route: [B,k] at the start
        self.best_sim = torch.empty(B, max(V - k, 1), dtype=f32, device=dev)
        self.wsum = torch.empty(B, k, dtype=f32, device=dev)
        self.final_idx = torch.empty(B, k, dtype=i32, device=dev)
        kvd = _TORCH_DTYPE[p.kv_dtype]
        self.k_dst = [torch.zeros(B, p.Hkv, Nout, p.d, dtype=kvd, device=dev) for _ in range(n_layers)]
        self.v_dst = [torch.zeros(B, p.Hkv, Nout, p.d, dtype=kvd, device=dev) for _ in range(n_layers)]
        self.workspace = torch.empty(max(asap_workspace_bytes(p), 256), dtype=torch.uint8, device=dev)


def stage_io(p: asap_params, q: torch.Tensor, k: torch.Tensor, hidden: torch.Tensor, text_len: torch.Tensor,
             k_cache: List[torch.Tensor], v_cache: List[torch.Tensor], buf: "StageBuffers",
             lse_extra: Optional[torch.Tensor] = None) -> asap_stage_io:
    """asap_stage_io for one batch: pointers and strides only.  The returned struct refers to the
    tensors' memory (and owns the four arrays of K/V layer pointers): keep the tensors alive."""
    P, V = p.P, p.V
    q_vis, q_txt, k_vis = q[:, :, P:P + V], q[:, :, P + V:], k[:, :, P:P + V]
    io = asap_stage_io()
    addr = lambda t: None if t is None else t.data_ptr()
    io.q_vis, io.q_vis_stride = addr(q_vis), _strides(q_vis, 3)
    io.q_txt, io.q_txt_stride = addr(q_txt), _strides(q_txt, 3)
    io.k_vis, io.k_vis_stride = addr(k_vis), _strides(k_vis, 3)
    io.text_len, io.lse_extra = addr(text_len), addr(lse_extra)
    io.s_raw, io.s_hat, io.score = addr(buf.s_raw), addr(buf.s_hat), addr(buf.score)
    io.kept_idx, io.pruned_idx = addr(buf.kept_idx), addr(buf.pruned_idx)
    io.hidden, io.hidden_stride = addr(hidden), _strides(hidden, 2)
    io.out_hidden, io.pos_out, io.new_len = addr(buf.out_hidden), addr(buf.pos_out), addr(buf.new_len)
    io.assign, io.best_sim, io.wsum, io.final_idx = addr(buf.assign), addr(buf.best_sim), addr(buf.wsum), \
        addr(buf.final_idx)
    n = len(k_cache)
    io.n_layers = n
    if n:
        arr = lambda ts: (ctypes.c_void_p * n)(*[t.data_ptr() for t in ts])
        io._keep = [arr(k_cache), arr(v_cache), arr(buf.k_dst), arr(buf.v_dst)]
        cast = lambda a: ctypes.cast(a, ctypes.POINTER(ctypes.c_void_p))
        io.k_src, io.v_src, io.k_dst, io.v_dst = (cast(a) for a in io._keep)
    io.workspace, io.workspace_bytes = addr(buf.workspace), buf.workspace.numel()
    return io


class PagedKV:
    """K/V caches of the layers in front of the pruning layer as pools of pages [n_pages,Hkv,page_size,d]
    with block tables [B, pages per sequence]; built on the device from contiguous caches [B,Hkv,N,d]
    with a seeded random placement of the pages.  Source and destination pages share one pool per
    cache, as they would in a serving engine that frees the source pages afterwards."""

    def __init__(self, p: asap_params, k_cache: List[torch.Tensor], v_cache: List[torch.Tensor], page_size: int,
                 seed: int = 0):
        N, Nout, ps = p.P + p.V + p.Tmax, p.P + p.k + p.Tmax, int(page_size)
        sp, dp = -(-N // ps), -(-Nout // ps)
        self.page_size, self.n_pages = ps, p.B * (sp + dp)
        g = torch.Generator().manual_seed(seed)
        perm = torch.randperm(self.n_pages, generator=g).to(torch.int32)
        self.src_table = perm[:p.B * sp].reshape(p.B, sp).contiguous().cuda()
        self.dst_table = perm[p.B * sp:].reshape(p.B, dp).contiguous().cuda()

        def pool_of(cache):
            padded = torch.zeros(p.B, p.Hkv, sp * ps, p.d, dtype=cache.dtype, device=cache.device)
            padded[:, :, :N] = cache
            pages = padded.view(p.B, p.Hkv, sp, ps, p.d).permute(0, 2, 1, 3, 4).reshape(p.B * sp, p.Hkv, ps, p.d)
            pool = torch.zeros(self.n_pages, p.Hkv, ps, p.d, dtype=cache.dtype, device=cache.device)
            pool[self.src_table.flatten().long()] = pages
            return pool
        self.k_pool = [pool_of(c) for c in k_cache]
        self.v_pool = [pool_of(c) for c in v_cache]

    def compact(self, ctx: "Context", p: asap_params, pos_out, new_len, stream=None):
        ctx.asap_compact_kv_paged(p, self.k_pool, self.v_pool, self.k_pool, self.v_pool, self.page_size,
                                  self.src_table, self.dst_table, pos_out, new_len, stream)


def run_stage(ctx: Context, p: asap_params, q: torch.Tensor, k: torch.Tensor, hidden: torch.Tensor,
              text_len: torch.Tensor, k_cache: List[torch.Tensor], v_cache: List[torch.Tensor],
              buf: StageBuffers, lse_extra: Optional[torch.Tensor] = None, stream=None,
              side_stream=None, paged: Optional[PagedKV] = None) -> StageBuffers:
    """The calls of one stage.  q [B,H,N,d], k [B,Hkv,N,d], hidden [B,N,D]; the visual / text blocks
    are passed to the library as strided views.  With a side stream the K/V compaction, which needs
    only the kept set, runs there next to the similarity and merge kernels of the main stream (one
    hand-over between the streams after the selection -- each costs the main stream about 6 us, so
    the rows that depend on nothing are not started earlier on their own); the main stream waits for
    the side stream at the end.  Contiguous caches are compacted by the call that takes the kept
    list directly; paged caches (`paged`; k_cache / v_cache are then ignored) need asap_positions."""
    P, V = p.P, p.V
    q_vis, q_txt, k_vis = q[:, :, P:P + V], q[:, :, P + V:], k[:, :, P:P + V]
    main = torch.cuda.current_stream() if stream is None else stream
    has_kv = bool(k_cache) or paged is not None
    kv = (k_cache, v_cache, buf.k_dst, buf.v_dst)

    def hand_over(src, dst):
        ev = torch.cuda.Event()
        ev.record(src)
        dst.wait_event(ev)

    ctx.asap_score(p, q_vis, q_txt, k_vis, text_len, lse_extra, buf.s_raw, buf.s_hat, buf.score,
                   buf.workspace, main)
    ctx.asap_select(p, buf.score, buf.kept_idx, buf.pruned_idx, buf.workspace, main)
    # with ASAP_ROUTE_ABSORB the kept set is final before the merge
    early = has_kv and side_stream is not None and p.route == ASAP_ROUTE_ABSORB
    if early:
        if paged is not None:
            ctx.asap_positions(p, buf.kept_idx, text_len, buf.pos_early, buf.new_len_early, main)
        hand_over(main, side_stream)
        if paged is not None:
            paged.compact(ctx, p, buf.pos_early, buf.new_len_early, side_stream)
        else:
            ctx.asap_compact_kv_from_kept(p, *kv, buf.kept_idx, text_len, side_stream)
    ctx.asap_merge(p, hidden, buf.s_raw, buf.s_hat, text_len, buf.kept_idx, buf.pruned_idx, buf.out_hidden, buf.pos_out,
                   buf.new_len, buf.assign, buf.best_sim, buf.wsum, buf.final_idx, buf.workspace, main)
    if early:
        hand_over(side_stream, main)
    elif has_kv:
        if paged is not None:
            paged.compact(ctx, p, buf.pos_out, buf.new_len, main)
        else:
            ctx.asap_compact_kv(p, *kv, buf.pos_out, buf.new_len, main)
    return buf


def to_device(arr, dtype: str, device="cuda:0") -> torch.Tensor:
    """Host array as stored by synth.quantise (float32, or uint16 bf16 bit patterns) -> device tensor."""
    import numpy as np
    if dtype == "bf16":
        return torch.from_numpy(arr.view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(arr).to(device)


class DeviceStage:
    """One batch from synth.make_inputs uploaded to the GPU, with output buffers.  run() is one
    asap_stage call (overlap=True: two streams inside the library); with call_by_call=True, or with
    paged caches, it is the sequence of single calls of run_stage, where the second stream is torch's."""

    def __init__(self, inp: dict, ctx: Optional[Context] = None, lse_extra=None, overlap: bool = True,
                 page_size: Optional[int] = None, call_by_call: bool = False, **param_overrides):
        import numpy as np
        cfg = inp["cfg"]
        self.cfg = cfg
        self.ctx = ctx or Context(0)
        self.p = params_from_config(cfg, **param_overrides)
        self.q = to_device(inp["q"], cfg.qk_dtype)
        self.k = to_device(inp["k"], cfg.qk_dtype)
        self.hidden = to_device(inp["hidden"], cfg.h_dtype)
        self.text_len = torch.from_numpy(inp["text_len"].astype(np.int32)).cuda()
        self.k_cache = [to_device(a, cfg.kv_dtype) for a in inp.get("k_cache", [])]
        self.v_cache = [to_device(a, cfg.kv_dtype) for a in inp.get("v_cache", [])]
        self.lse_extra = None if lse_extra is None else torch.from_numpy(lse_extra.astype(np.float32)).cuda()
        self.paged = None
        if page_size and self.k_cache:
            # the caches become pools of pages; the contiguous copies and destinations are not kept
            self.paged = PagedKV(self.p, self.k_cache, self.v_cache, page_size, seed=cfg.seed)
            self.k_cache, self.v_cache = [], []
        self.buf = StageBuffers(self.p, len(self.k_cache))
        has_kv = bool(self.k_cache) or self.paged is not None
        self.call_by_call = call_by_call or self.paged is not None
        # whether the K/V compaction runs beside the similarity and merge kernels
        self.two_streams = overlap and has_kv and self.p.route == ASAP_ROUTE_ABSORB
        # torch's default-priority second stream, for the call-by-call path only
        self.side_stream = torch.cuda.Stream() if (self.call_by_call and overlap and has_kv) else None
        self.io = None if self.call_by_call else stage_io(self.p, self.q, self.k, self.hidden, self.text_len,
                                                          self.k_cache, self.v_cache, self.buf, self.lse_extra)

    def run_async(self) -> StageBuffers:
        if self.call_by_call:
            return run_stage(self.ctx, self.p, self.q, self.k, self.hidden, self.text_len, self.k_cache,
                             self.v_cache, self.buf, self.lse_extra, side_stream=self.side_stream, paged=self.paged)
        self.ctx.asap_stage(self.p, self.io, self.two_streams)
        return self.buf

    def run(self) -> StageBuffers:
        self.run_async()
        torch.cuda.synchronize()
        return self.buf
