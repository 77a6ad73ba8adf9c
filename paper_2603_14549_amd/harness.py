"""Device-side plumbing around the binding for the tests, bench.py and the smoke check: torch
tensors for the inputs of a synthetic batch and for every output buffer, the asap_stage_io struct
that points at them, and the two ways of running a stage (one asap_stage call, or the single calls
with torch's streams).  Nothing of the method is computed here -- that is all in the library."""
from __future__ import annotations

import ctypes
from typing import List, Optional

import torch

from .binding import (ASAP_ROUTE_ABSORB, ASAP_ROWS_LAST, ASAP_STREAMS_AUTO, ASAP_STREAMS_ONE, ASAP_STREAMS_TWO, Context, _TORCH_DTYPE, _strides, asap_params, asap_stage_io,
                      asap_workspace_bytes, params_from_config)


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
    asap_stage call (overlap=True: two streams inside the library whatever the sizes, "auto": the library
    chooses, False: one stream); with call_by_call=True, or with
    paged caches, it is the sequence of single calls of run_stage, where the second stream is torch's.
    last_token=True ranks the visual tokens by the last valid text token's row alone
    (score_rows = ASAP_ROWS_LAST in the params; the library picks the row from text_len)."""

    def __init__(self, inp: dict, ctx: Optional[Context] = None, lse_extra=None, overlap=True,
                 page_size: Optional[int] = None, call_by_call: bool = False, last_token: bool = False,
                 hidden_row_pad: int = 0, **param_overrides):
        import numpy as np
        cfg = inp["cfg"]
        self.cfg = cfg
        self.ctx = ctx or Context(0)
        if last_token:
            param_overrides = dict(param_overrides, score_rows=ASAP_ROWS_LAST)
        self.p = params_from_config(cfg, **param_overrides)
        self.q = to_device(inp["q"], cfg.qk_dtype)
        self.k = to_device(inp["k"], cfg.qk_dtype)
        self.hidden = to_device(inp["hidden"], cfg.h_dtype)
        if hidden_row_pad:       # rows of the hidden states hidden_row_pad elements further apart (a strided view)
            store = torch.zeros(cfg.B, self.hidden.shape[1], cfg.D + hidden_row_pad, dtype=self.hidden.dtype,
                                device=self.hidden.device)
            store[:, :, :cfg.D] = self.hidden
            self.hidden = store[:, :, :cfg.D]
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
        self.two_streams = bool(overlap) and has_kv and self.p.route == ASAP_ROUTE_ABSORB
        self.stream_mode = (ASAP_STREAMS_ONE if not self.two_streams else
                            ASAP_STREAMS_AUTO if overlap == "auto" else ASAP_STREAMS_TWO)
        # torch's default-priority second stream, for the call-by-call path only
        self.side_stream = torch.cuda.Stream() if (self.call_by_call and overlap and has_kv) else None
        self.io = None if self.call_by_call else stage_io(self.p, self.q, self.k, self.hidden, self.text_len,
                                                          self.k_cache, self.v_cache, self.buf, self.lse_extra)

    def run_async(self) -> StageBuffers:
        if self.call_by_call:
            return run_stage(self.ctx, self.p, self.q, self.k, self.hidden, self.text_len, self.k_cache,
                             self.v_cache, self.buf, self.lse_extra, side_stream=self.side_stream, paged=self.paged)
        self.ctx.asap_stage(self.p, self.io, self.stream_mode)
        return self.buf

    def run(self) -> StageBuffers:
        self.run_async()
        torch.cuda.synchronize()
        return self.buf
