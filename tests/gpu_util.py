"""Helpers of the GPU parity tests: upload a seeded workload, run the HIP path through the
binding, compare with the oracle under the stated tolerances."""
from __future__ import annotations

import numpy as np
import torch

import workloads as W
from oracle import vlcache_oracle as O


def torch_dtype(cfg):
    return torch.float32 if cfg.dtype == "f32" else torch.bfloat16


def make_shape(cfg):
    import paper_2410_23317_amd as V
    return V.make_shape(cfg.B, cfg.L, cfg.Hq, cfg.Hkv, cfg.d, cfg.m, cfg.tau, cfg.dtype)


def upload(cfg, want_v=True, workers=8):
    """q_win [B,L,Hq,tau,d], k, v [B,L,Hkv,m,d] in the storage dtype on the GPU, sm_scale [L] fp32."""
    dt = torch_dtype(cfg)
    dev = torch.device("cuda")
    out = {"q_win": torch.empty((cfg.B, cfg.L, cfg.Hq, cfg.tau, cfg.d), dtype=dt, device=dev),
           "k": torch.empty((cfg.B, cfg.L, cfg.Hkv, cfg.m, cfg.d), dtype=dt, device=dev)}
    if want_v:
        out["v"] = torch.empty_like(out["k"])

    def put(b, l, t):
        for name in out:
            out[name][b, l].copy_(torch.from_numpy(t[name]).to(dt))

    W.for_each_layer(cfg, put, want_v=want_v, workers=workers)
    out["sm_scale"] = torch.from_numpy(W.sm_scale(cfg)).to(dev)
    return out


def decode_upload(cfg, step):
    t = W.decode_step_inputs(cfg, step)
    dt = torch_dtype(cfg)
    return {k: torch.from_numpy(v).to(dt).cuda() for k, v in t.items()}, t


def assert_close(got, want, atol, rtol, what):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    err = np.abs(got - want)
    lim = atol + rtol * np.abs(want)
    bad = err > lim
    if bad.any():
        i = np.unravel_index(np.argmax(err - lim), err.shape)
        raise AssertionError(f"{what}: {int(bad.sum())} of {bad.size} outside atol={atol} rtol={rtol}; "
                             f"worst at {i}: got {got[i]!r} want {want[i]!r}")


def check_topk(idx_gpu, psi_oracle, k, what, rel=1e-5, n_recent=0):
    """Index sets equal, except swaps among tokens whose oracle score is within rel of the k-th."""
    idx_gpu = np.asarray(idx_gpu).astype(np.int64)
    assert idx_gpu.shape == (k,), f"{what}: {idx_gpu.shape} kept, {k} expected"
    assert np.all(np.diff(idx_gpu) > 0), f"{what}: kept positions not strictly ascending"
    assert idx_gpu.min() >= 0 and idx_gpu.max() < len(psi_oracle)
    want = O.topk(psi_oracle, k, n_recent)
    if np.array_equal(idx_gpu, want):
        return 0
    r = min(n_recent, k)
    kth = np.sort(psi_oracle[: len(psi_oracle) - r])[::-1][k - r - 1]
    diff = np.setxor1d(idx_gpu, want)
    off = np.abs(psi_oracle[diff] - kth)
    assert np.all(off <= rel * abs(kth)), (f"{what}: {len(diff)} positions differ from the oracle's set and "
                                           f"are not within {rel} of the k-th score (worst {off.max() / abs(kth):.3e})")
    return len(diff)


def check_nnz(nnz_gpu, q_win, k, scale, p, what, rel=1e-5):
    """Counts equal, or differing by no more than the number of decisions the oracle itself marks
    borderline: |s - M - ln p| < rel * max(1, |s|)."""
    nnz_o, _, margin, _ = O.sparsity(q_win, k, scale, p, want_margin=True)
    nnz_gpu = np.asarray(nnz_gpu).astype(np.int64)
    if np.array_equal(nnz_gpu, nnz_o):
        return nnz_o, 0
    s = O.logits(q_win, k, scale)
    border = (margin < rel * np.maximum(1.0, np.abs(s))).sum(axis=(1, 2))
    d = np.abs(nnz_gpu - nnz_o)
    assert np.all(d <= border), f"{what}: counts differ by {d.tolist()} with only {border.tolist()} borderline entries"
    return nnz_o, int(d.sum())
