"""Seeded synthetic workloads for the VL-Cache hot path.

This module only *draws inputs*: it contains none of the method's arithmetic
(no softmax, no thresholding, no selection).  Both the CPU oracle's tests and
the HIP path's tests / benchmark take their inputs from here, so that both
sides see the same bits.

The shapes stand in for the prompts the paper evaluates on (image tiles of a
few hundred to a few thousand visual tokens followed by a short text question,
Sec. 5 and Sec. 5.2 of the paper): only token counts and the position of the
post-vision text window are taken from there, never any dataset item.

Every tensor is drawn in fp32 from a generator keyed by
(SEED, config, tensor id, request b, layer l, step) and rounded ONCE to the
config's storage dtype (round-to-nearest-even for bf16).  Arrays returned to
callers are fp32 numpy arrays that hold exactly those rounded values, so they
convert to bf16 (device side) and to fp64 (oracle side) without further
rounding.
"""
from __future__ import annotations

import dataclasses
from concurrent.futures import ThreadPoolExecutor
from typing import Dict, List, Tuple

import numpy as np

SEED = 241023317

# tensor ids used in the generator key
_T_Q, _T_K, _T_V, _T_SINK, _T_TEMP, _T_FRAME, _T_DQ, _T_DK, _T_DV = range(9)


@dataclasses.dataclass(frozen=True)
class Config:
    """One synthetic workload.  Notation follows the paper: m prompt tokens,
    tau post-vision window rows, L layers, alpha whole-model budget."""
    cid: int
    name: str
    B: int
    L: int
    Hq: int
    Hkv: int
    d: int
    dtype: str                      # "f32" or "bf16"
    m: int
    tau: int
    lead_text: int                  # text tokens before the visual span
    n_visual: int                   # visual tokens (one contiguous span)
    sinks: int                      # scaled "sink" keys per (b, l, kv head)
    alphas: Tuple[Tuple[int, int], ...]  # budgets as rationals (num, den)
    steps: int                      # decode steps
    frame_len: int = 0              # >0: keys carry per-frame structure

    @property
    def g(self) -> int:
        return self.Hq // self.Hkv

    @property
    def visual_span(self) -> Tuple[int, int]:
        return self.lead_text, self.lead_text + self.n_visual

    def layout(self) -> str:
        tail = self.m - self.lead_text - self.n_visual
        return (f"[{self.lead_text} text | {self.n_visual} visual | {tail} text, "
                f"last {self.tau} = post-vision window]")


CONFIGS: List[Config] = [
    Config(0, "tiny-f32", 1, 2, 4, 2, 64, "f32", 512, 32, 32, 448, 8, ((1, 10),), 8),
    Config(1, "7b-m2944", 1, 32, 32, 8, 128, "bf16", 2944, 32, 32, 2880, 16, ((1, 10),), 100),
    Config(2, "7b-b4-m10368", 4, 32, 32, 8, 128, "bf16", 10368, 64, 64, 10240, 16, ((1, 10),), 100),
    Config(3, "34b-b4-m10368", 4, 60, 56, 8, 128, "bf16", 10368, 64, 64, 10240, 16, ((1, 10),), 100),
    Config(4, "7b-video-m32768", 1, 32, 32, 8, 128, "bf16", 32768, 64, 64, 32640, 32,
           ((1, 100), (1, 20), (1, 10), (1, 5)), 100, frame_len=510),
]


def custom_config(**kw) -> Config:
    """A free-form config (for small parity cases with ragged tails)."""
    base = dict(cid=99, name="custom", B=1, L=2, Hq=4, Hkv=2, d=64, dtype="f32", m=128,
                tau=8, lead_text=8, n_visual=100, sinks=4, alphas=((1, 10),), steps=4,
                frame_len=0)
    base.update(kw)
    return Config(**base)


def _gen(cfg: Config, tensor: int, b: int = 0, l: int = 0, step: int = 0) -> np.random.Generator:
    ss = np.random.SeedSequence([SEED, cfg.cid, cfg.m, cfg.tau, tensor, b, l, step])
    return np.random.Generator(np.random.SFC64(ss))


def round_to_dtype(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round an fp32 array to the storage dtype, return fp32 holding those values."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "f32":
        return x
    if dtype != "bf16":
        raise ValueError(dtype)
    u = x.view(np.uint32)
    bias = u >> np.uint32(16)
    bias &= np.uint32(1)
    bias += np.uint32(0x7FFF)
    u += bias                      # round to nearest, ties to even (no NaN/Inf in these draws)
    u &= np.uint32(0xFFFF0000)
    return x


def temperatures(cfg: Config) -> np.ndarray:
    """Per-layer softmax temperature T_l ~ U(0.5, 2) (so that sparsity differs by layer)."""
    return _gen(cfg, _T_TEMP).uniform(0.5, 2.0, size=cfg.L)


def sm_scale(cfg: Config) -> np.ndarray:
    """Per-layer logit scale 1/(T_l * sqrt(d)) as fp32 (the value both sides use)."""
    return (1.0 / (temperatures(cfg) * np.sqrt(float(cfg.d)))).astype(np.float32)


def sink_positions(cfg: Config, b: int, l: int) -> np.ndarray:
    """[Hkv, sinks] distinct positions inside the visual span, per kv head."""
    g = _gen(cfg, _T_SINK, b, l)
    lo, hi = cfg.visual_span
    return np.stack([np.sort(g.choice(hi - lo, size=cfg.sinks, replace=False)) + lo
                     for _ in range(cfg.Hkv)])


def layer_inputs(cfg: Config, b: int, l: int, want_v: bool = True) -> Dict[str, np.ndarray]:
    """Prefill tensors of one (request, layer): q_win [Hq,tau,d], k, v [Hkv,m,d] (fp32 values
    already rounded to cfg.dtype)."""
    q = _gen(cfg, _T_Q, b, l).standard_normal((cfg.Hq, cfg.tau, cfg.d), dtype=np.float32)
    k = _gen(cfg, _T_K, b, l).standard_normal((cfg.Hkv, cfg.m, cfg.d), dtype=np.float32)
    if cfg.frame_len:
        lo, hi = cfg.visual_span
        n_frames = (hi - lo) // cfg.frame_len
        mu = _gen(cfg, _T_FRAME, b, l).standard_normal((cfg.Hkv, n_frames, cfg.d), dtype=np.float32)
        vis = k[:, lo:lo + n_frames * cfg.frame_len].reshape(cfg.Hkv, n_frames, cfg.frame_len, cfg.d)
        vis += mu[:, :, None, :]
    pos = sink_positions(cfg, b, l)
    for h in range(cfg.Hkv):
        k[h, pos[h]] *= np.float32(4.0)
    out = {"q_win": round_to_dtype(q, cfg.dtype), "k": round_to_dtype(k, cfg.dtype)}
    if want_v:
        v = _gen(cfg, _T_V, b, l).standard_normal((cfg.Hkv, cfg.m, cfg.d), dtype=np.float32)
        out["v"] = round_to_dtype(v, cfg.dtype)
    return out


def decode_inputs(cfg: Config, step: int, l: int) -> Dict[str, np.ndarray]:
    """Fresh decode-step tensors of one layer: q [B,Hq,d], k_new, v_new [B,Hkv,d]."""
    q = _gen(cfg, _T_DQ, 0, l, step).standard_normal((cfg.B, cfg.Hq, cfg.d), dtype=np.float32)
    k = _gen(cfg, _T_DK, 0, l, step).standard_normal((cfg.B, cfg.Hkv, cfg.d), dtype=np.float32)
    v = _gen(cfg, _T_DV, 0, l, step).standard_normal((cfg.B, cfg.Hkv, cfg.d), dtype=np.float32)
    return {"q": round_to_dtype(q, cfg.dtype), "k_new": round_to_dtype(k, cfg.dtype),
            "v_new": round_to_dtype(v, cfg.dtype)}


def decode_step_inputs(cfg: Config, step: int) -> Dict[str, np.ndarray]:
    """All layers of one decode step: q [L,B,Hq,d], k_new, v_new [L,B,Hkv,d]."""
    per = [decode_inputs(cfg, step, l) for l in range(cfg.L)]
    return {k: np.stack([p[k] for p in per]) for k in ("q", "k_new", "v_new")}


def budget_total(cfg: Config, alpha: Tuple[int, int]) -> int:
    """Whole-model token budget of one request, floor(alpha * L * m)."""
    return (alpha[0] * cfg.L * cfg.m) // alpha[1]


def for_each_layer(cfg: Config, fn, want_v: bool = True, workers: int = 8) -> None:
    """Call fn(b, l, tensors) for every (request, layer); slices are drawn on a thread pool
    (the generators release the GIL) but fn runs in the calling thread, in order."""
    items = [(b, l) for b in range(cfg.B) for l in range(cfg.L)]
    with ThreadPoolExecutor(max_workers=workers) as ex:
        window = 2 * workers
        futs = {}
        nxt = 0
        for i, (b, l) in enumerate(items):
            while nxt < len(items) and nxt < i + window:
                bb, ll = items[nxt]
                futs[nxt] = ex.submit(layer_inputs, cfg, bb, ll, want_v)
                nxt += 1
            fn(b, l, futs.pop(i).result())
