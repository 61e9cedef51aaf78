"""Sequencing of the hot path over the C-ABI calls: buffers and call order only, no arithmetic.

After prefill:  vlc_score -> vlc_sparsity (finalise) -> vlc_allocate -> vlc_topk_compact.
Fused route for the scores: vlc_window_attn (attention of the window rows + row statistics) ->
vlc_score_from_stats (column sweep only).
Every decode step: vlc_decode_attn over a layer range of the compressed cache.
"""
from __future__ import annotations

from typing import Optional, Tuple

import torch

from . import binding as V


def k_min_tokens(m: int) -> int:
    """Token form of the lower clip 0.01 of the layer budget (Alg. 1)."""
    return max(1, -(-m // 100))


class VLCachePath:
    """Holds the output buffers of the compression stages and the compressed cache of one batch."""

    def __init__(self, shape: V.vlc_shape, alpha: Tuple[int, int] = (1, 10), p: float = 0.01,
                 T_max: int = 128, n_recent: int = 0, device: str = "cuda", want_idx: bool = False,
                 recent_frac: Optional[Tuple[int, int]] = None, lens: Optional[torch.Tensor] = None,
                 kv_fp8: bool = False, options: Optional[V.vlc_cache_options] = None):
        s = shape
        self.lens = lens                      # the [B, 2] tensor behind shape.lens (ragged batches), kept alive here
        self.shape, self.alpha, self.p, self.T_max, self.n_recent = s, alpha, float(p), int(T_max), int(n_recent)
        self.recent_frac = recent_frac        # (num, den): recent window = floor(k_l * num / den) per layer
        dev = torch.device(device)
        f32, i32 = torch.float32, torch.int32
        self.scores = torch.empty((s.B, s.L, s.Hkv, s.m), dtype=f32, device=dev)
        self.row_max = torch.empty((s.B, s.L, s.Hq, s.tau), dtype=f32, device=dev)
        self.row_sum = torch.empty_like(self.row_max)
        self.nnz = torch.empty((s.B, s.L, s.Hq), dtype=torch.int64, device=dev)   # uint64 counts, < 2^63
        self.gamma = torch.empty((s.B, s.L, s.Hq), dtype=f32, device=dev)
        self.k = torch.empty((s.B, s.L), dtype=i32, device=dev)
        self.beta = torch.empty((s.B, s.L), dtype=f32, device=dev)
        self.workspace = torch.empty(V.vlc_workspace_bytes(s), dtype=torch.uint8, device=dev)
        self.idx_out = torch.full((s.B, s.L, s.Hkv, s.m), -1, dtype=i32, device=dev) if want_idx else None
        b_tot = (alpha[0] * s.L * s.m) // alpha[1]
        self.sum_k_max = min(s.L * s.m, b_tot + s.L * k_min_tokens(s.m))
        if options is not None:
            options.kv_fp8 = int(bool(kv_fp8)) or options.kv_fp8
            self.cache = V.vlc_cache_create_opt(s, self.T_max, self.sum_k_max, options, device)
        else:
            self.cache = (V.vlc_cache_create_fp8 if kv_fp8 else V.vlc_cache_create)(s, self.T_max, self.sum_k_max, device)

    # -- after prefill ---------------------------------------------------------------------
    def score(self, q_win, k, sm_scale) -> None:
        V.vlc_score(self.shape, q_win, k, sm_scale, self.p, self.scores, self.row_max, self.row_sum, self.nnz,
                    self.workspace)

    def window_attn(self, q_win, k, v, sm_scale, out: Optional[torch.Tensor] = None) -> torch.Tensor:
        """Attention of the window rows that also fills row_max / row_sum: with it the scores come from
        score_from_stats and the row-statistics sweep of score() is not run."""
        if out is None:
            out = torch.empty_like(q_win)
        if getattr(self, "win_workspace", None) is None:
            self.win_workspace = torch.empty(V.vlc_window_attn_workspace_bytes(self.shape), dtype=torch.uint8,
                                             device=q_win.device)
        V.vlc_window_attn(self.shape, q_win, k, v, sm_scale, out, self.row_max, self.row_sum, self.win_workspace)
        return out

    def score_from_stats(self, q_win, k, sm_scale) -> None:
        V.vlc_score_from_stats(self.shape, q_win, k, sm_scale, self.p, self.row_max, self.row_sum, self.scores, self.nnz)

    def sparsity(self) -> None:
        V.vlc_sparsity(self.shape, None, None, None, None, self.p, self.nnz, self.gamma, None)

    def allocate(self) -> None:
        V.vlc_allocate(self.shape, self.nnz, self.alpha[0], self.alpha[1], self.k, self.beta)

    def topk_compact(self, k_full, v_full, k: Optional[torch.Tensor] = None) -> None:
        kk = self.k if k is None else k
        if self.recent_frac is not None:
            V.vlc_topk_compact_recent_frac(self.cache, self.scores, kk, self.recent_frac[0], self.recent_frac[1],
                                           k_full, v_full, self.idx_out)
        else:
            V.vlc_topk_compact(self.cache, self.scores, kk, self.n_recent, k_full, v_full, self.idx_out)

    def compress(self, q_win, k, v, sm_scale) -> None:
        self.score(q_win, k, sm_scale)
        self.sparsity()
        self.allocate()
        self.topk_compact(k, v)

    # -- every decode step -----------------------------------------------------------------
    def decode(self, layer_begin, layer_end, q, k_new, v_new, sm_scale, out) -> None:
        V.vlc_decode_attn(self.cache, layer_begin, layer_end, q, k_new, v_new, sm_scale, out)

    def decode_steps(self, layer_begin, layer_end, n_steps, q, k_new, v_new, sm_scale, out) -> None:
        V.vlc_decode_attn_steps(self.cache, layer_begin, layer_end, n_steps, q, k_new, v_new, sm_scale, out)

    def status(self) -> None:
        V.vlc_cache_status(self.cache)

    # -- diagnostic (Def. 3.1) ----------------------------------------------------------------
    def hit_rate(self, q_next, k, sm_scale):
        """CacheHitRate of the cache against the first decode query q_next [B, L, Hq, d]:
        returns (hits [B,L,Hkv] int32, rate [B,L,Hkv] float32, scores_star [B,L,Hkv,m])."""
        s = self.shape
        if not hasattr(self, "_star"):
            lens1 = None
            if self.lens is not None:             # same prompt lengths, a one-row window for every request
                lens1 = self.lens.clone()
                lens1[:, 1] = 1
            one = V.make_shape(s.B, s.L, s.Hq, s.Hkv, s.d, s.m, 1, "f32" if s.dtype == V.VLC_F32 else "bf16", lens=lens1,
                               flags=s.flags)
            dev = self.scores.device
            self._star = dict(
                shape=one, lens=lens1, scores=torch.empty_like(self.scores),
                row_max=torch.empty((s.B, s.L, s.Hq, 1), dtype=torch.float32, device=dev),
                row_sum=torch.empty((s.B, s.L, s.Hq, 1), dtype=torch.float32, device=dev),
                workspace=torch.empty(V.vlc_workspace_bytes(one), dtype=torch.uint8, device=dev),
                hits=torch.empty((s.B, s.L, s.Hkv), dtype=torch.int32, device=dev),
                rate=torch.empty((s.B, s.L, s.Hkv), dtype=torch.float32, device=dev))
        t = self._star
        V.vlc_score(t["shape"], q_next, k, sm_scale, self.p, t["scores"], t["row_max"], t["row_sum"], None, t["workspace"])
        V.vlc_cache_hit_rate(self.cache, t["scores"], t["hits"], t["rate"])
        return t["hits"], t["rate"], t["scores"]


def cache_layer_view(cache: V.Cache, b: int, l: int, appended: int = 0):
    """(Kc, Vc, idx) of request b, layer l as tensors [Hkv, n, d] / [Hkv, n] aliasing the arena,
    n = kept + appended.  Pure address arithmetic over the layout the library reports.  For an FP8
    cache Kc and Vc are pairs (codes uint8 [Hkv, n, d], scales float32 [Hkv, n])."""
    s, lay, arena = cache.shape, cache.layout, cache.arena
    BL = s.B * s.L
    slot_off = arena[lay.slot_off_off: lay.slot_off_off + 8 * BL].view(torch.int64)
    kept = arena[lay.kept_off: lay.kept_off + 4 * BL].view(torch.int32)
    so, kk = int(slot_off[b * s.L + l]), int(kept[b * s.L + l])
    cap, n = kk + cache.T_max, kk + appended
    ib = lay.idx_off + so * s.Hkv * 4
    idx = arena[ib: ib + s.Hkv * cap * 4].view(torch.int32).view(s.Hkv, cap)[:, :n]
    if lay.kv_fp8:
        slab = s.Hkv * cap * s.d
        kb = lay.kv_off + so * 2 * s.Hkv * s.d
        kcodes = arena[kb: kb + slab].view(s.Hkv, cap, s.d)[:, :n]
        vcodes = arena[kb + slab: kb + 2 * slab].view(s.Hkv, cap, s.d)[:, :n]
        sb = lay.scale_off + so * 2 * s.Hkv * 4
        ksc = arena[sb: sb + s.Hkv * cap * 4].view(torch.float32).view(s.Hkv, cap)[:, :n]
        vsc = arena[sb + s.Hkv * cap * 4: sb + 2 * s.Hkv * cap * 4].view(torch.float32).view(s.Hkv, cap)[:, :n]
        return (kcodes, ksc), (vcodes, vsc), idx
    dt = torch.float32 if s.dtype == V.VLC_F32 else torch.bfloat16
    es = 4 if s.dtype == V.VLC_F32 else 2
    slab = s.Hkv * cap * s.d * es
    kb = lay.kv_off + so * 2 * s.Hkv * s.d * es
    kc = arena[kb: kb + slab].view(dt).view(s.Hkv, cap, s.d)[:, :n]
    vc = arena[kb + slab: kb + 2 * slab].view(dt).view(s.Hkv, cap, s.d)[:, :n]
    return kc, vc, idx
