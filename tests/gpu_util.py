"""Helpers of the GPU parity tests: upload a seeded workload, run the HIP path through the
binding, compare with the oracle under the stated tolerances."""
from __future__ import annotations

import numpy as np
import pytest
import torch

import workloads as W
from oracle import vlcache_oracle as O


def torch_dtype(cfg):
    return torch.float32 if cfg.dtype == "f32" else torch.bfloat16


def make_shape(cfg, flags=0):
    import paper_2410_23317_amd as V
    return V.make_shape(cfg.B, cfg.L, cfg.Hq, cfg.Hkv, cfg.d, cfg.m, cfg.tau, cfg.dtype, flags=flags)


def upload(cfg, want_v=True, workers=16):
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


SCORE_TOL = dict(atol=1e-7, rtol=5e-5)


def out_tol(cfg):
    return dict(atol=2e-2, rtol=1e-2) if cfg.dtype == "bf16" else dict(atol=1e-4, rtol=1e-4)


def run_and_check(cfg, alpha, n_steps, n_recent=0, layers_to_check=None, requests_to_check=None, per_layer_decode=False,
                  dev=None, recent_frac=None, options=None, steps_entry_point=False, T_max=None):
    """Whole path on the GPU; oracle on every (or the listed) request/layer.  options: fields of
    vlc_cache_options; steps_entry_point: all decode steps enqueued by one vlc_decode_attn_steps call
    (how bench.py runs them) instead of one vlc_decode_attn call per step."""
    import paper_2410_23317_amd as V
    from paper_2410_23317_amd.pipeline import VLCachePath, cache_layer_view

    print(f"[case] cfg={cfg.name} cid={cfg.cid} m={cfg.m} tau={cfg.tau} d={cfg.d} g={cfg.g} alpha={alpha} "
          f"steps={n_steps} n_recent={n_recent} recent_frac={recent_frac}", flush=True)
    shape = make_shape(cfg)
    if dev is None:
        dev = upload(cfg)
    path = VLCachePath(shape, alpha=alpha, p=0.01, T_max=max(n_steps, 1) if T_max is None else T_max, n_recent=n_recent,
                       want_idx=True, recent_frac=recent_frac, options=None if options is None else V.make_options(**options))
    path.compress(dev["q_win"], dev["k"], dev["v"], dev["sm_scale"])
    path.status()
    torch.cuda.synchronize()
    scales = W.sm_scale(cfg)
    full = layers_to_check is None and requests_to_check is None
    reqs = range(cfg.B) if requests_to_check is None else requests_to_check
    lays = range(cfg.L) if layers_to_check is None else layers_to_check

    scores = path.scores.cpu().numpy()
    nnz = path.nnz.cpu().numpy()
    kk = path.k.cpu().numpy()
    # properties that hold at any size
    np.testing.assert_allclose(scores.sum(-1), cfg.g * cfg.tau, rtol=1e-4)
    lo = O.k_min(cfg.m)
    assert np.all(kk >= lo) and np.all(kk <= cfg.m)
    b_tot = W.budget_total(cfg, alpha)
    for b in range(cfg.B):
        k_o, beta_o = O.allocate(nnz[b], cfg.m, alpha[0], alpha[1])
        assert np.array_equal(kk[b], k_o), f"budgets of request {b} differ from Alg. 1 on the GPU's own counts"
        np.testing.assert_allclose(path.beta[b].cpu().numpy(), beta_o, rtol=1e-6)
        share = nnz[b].sum(1) * b_tot / nnz[b].sum()
        quota_ok = (share >= lo).all() and (share <= cfg.m - 1).all()      # no clip binds (Alg. 1 does not renormalise)
        if quota_ok:
            assert int(kk[b].sum()) == b_tot

    caches = {}
    flips = swaps = 0
    for b in reqs:
        nnz_oracle = []
        for l in lays:
            t = W.layer_inputs(cfg, b, l)
            psi, _, M, Z = O.score(t["q_win"], t["k"], scales[l])
            what = f"{cfg.name} b={b} l={l}"
            assert_close(scores[b, l], psi, what=what + " scores", **SCORE_TOL)
            assert_close(path.row_max[b, l].cpu().numpy(), M, atol=2e-5, rtol=2e-6, what=what + " row_max")
            assert_close(path.row_sum[b, l].cpu().numpy(), Z, atol=0, rtol=5e-5, what=what + " row_sum")
            n_o, d = check_nnz(nnz[b, l], t["q_win"], t["k"], scales[l], 0.01, what + " nnz")
            flips += d
            nnz_oracle.append(n_o)
            np.testing.assert_allclose(path.gamma[b, l].cpu().numpy(), 1 - nnz[b, l] / O.region_size(cfg.m, cfg.tau),
                                       rtol=1e-6, atol=1e-7)
            kc, vc, idx = cache_layer_view(path.cache, b, l)
            kc, vc, idx = kc.float().cpu().numpy(), vc.float().cpu().numpy(), idx.cpu().numpy()
            for h in range(cfg.Hkv):
                nr = n_recent if recent_frac is None else O.recent_count(int(kk[b, l]), *recent_frac)
                swaps += check_topk(idx[h], psi[h], int(kk[b, l]), what + f" hkv={h} topk", n_recent=nr)
                assert np.array_equal(path.idx_out[b, l, h, : kk[b, l]].cpu().numpy(), idx[h])
                assert np.array_equal(kc[h], t["k"][h][idx[h]]), what + " gathered K rows"
                assert np.array_equal(vc[h], t["v"][h][idx[h]]), what + " gathered V rows"
            caches[(b, l)] = ([kc[h] for h in range(cfg.Hkv)], [vc[h] for h in range(cfg.Hkv)])
        if full:
            k_e2e, _ = O.allocate(np.stack(nnz_oracle), cfg.m, alpha[0], alpha[1])
            if not np.array_equal(k_e2e, kk[b]):
                assert flips > 0, "budgets differ from the oracle's although every count matches"
                pytest.fail(f"request {b}: budgets differ from the oracle's end to end because of {flips} "
                            f"borderline threshold decisions: {kk[b].tolist()} vs {k_e2e.tolist()}")
    print(f"[compress ok] borderline count flips={flips} topk swaps={swaps}", flush=True)

    # decode steps: the GPU appends into its cache, the oracle into its own lists
    dt = torch_dtype(cfg)
    out = torch.empty((cfg.L, cfg.B, cfg.Hq, cfg.d), dtype=dt, device="cuda")
    if steps_entry_point and n_steps:
        # every step's inputs go to the GPU first (the host keeps only the layers it will check), then ONE call
        # enqueues all steps, as the benchmark does
        stack = {"q": torch.empty((n_steps, cfg.L, cfg.B, cfg.Hq, cfg.d), dtype=dt, device="cuda"),
                 "k_new": torch.empty((n_steps, cfg.L, cfg.B, cfg.Hkv, cfg.d), dtype=dt, device="cuda")}
        stack["v_new"] = torch.empty_like(stack["k_new"])
        hosts = []
        for t in range(n_steps):
            d = W.decode_step_inputs(cfg, t)
            for n in stack:
                stack[n][t].copy_(torch.from_numpy(d[n]).to(dt))
            hosts.append({n: {l: d[n][l] for l in lays} for n in d})
        out_all = torch.empty((n_steps, cfg.L, cfg.B, cfg.Hq, cfg.d), dtype=dt, device="cuda")
        path.decode_steps(0, cfg.L, n_steps, stack["q"], stack["k_new"], stack["v_new"], dev["sm_scale"], out_all)
        torch.cuda.synchronize()
    for step in range(n_steps):
        if steps_entry_point:
            d_host = hosts[step]
            got = {l: out_all[step, l].float().cpu().numpy() for l in lays}
        else:
            d_dev, d_host = decode_upload(cfg, step)
            if per_layer_decode:
                for l in range(cfg.L):
                    path.decode(l, l + 1, d_dev["q"][l], d_dev["k_new"][l], d_dev["v_new"][l], dev["sm_scale"], out[l])
            else:
                path.decode(0, cfg.L, d_dev["q"], d_dev["k_new"], d_dev["v_new"], dev["sm_scale"], out)
            torch.cuda.synchronize()
            got = out.float().cpu().numpy()
        for (b, l), (kc, vc) in caches.items():
            for h in range(cfg.Hkv):
                kc[h] = np.concatenate([kc[h], d_host["k_new"][l][b, h][None]], 0)
                vc[h] = np.concatenate([vc[h], d_host["v_new"][l][b, h][None]], 0)
            want = O.decode_attn(d_host["q"][l][b], kc, vc, scales[l])
            assert_close(got[l][b], want, what=f"{cfg.name} decode step {step} b={b} l={l}", **out_tol(cfg))
    path.status()
    # the cache now holds the appended rows too
    if n_steps:
        (b, l), (kc, vc) = next(iter(caches.items()))
        gk, gv, gi = cache_layer_view(path.cache, b, l, appended=n_steps)
        assert np.array_equal(gk.float().cpu().numpy()[0], kc[0])
        assert np.array_equal(gv.float().cpu().numpy()[0], vc[0])
        assert gi[0, -1].item() == cfg.m + n_steps - 1
        lay = path.cache.layout
        count = path.cache.arena[lay.appended_off: lay.appended_off + 4 * cfg.L].view(torch.int32)
        assert count.tolist() == [n_steps] * cfg.L, "the device-side append counts"
    print("[decode ok]", flush=True)
    return path




def check_window_attn(cfg, dev, requests_to_check, layers_to_check):
    """vlc_window_attn + vlc_score_from_stats on an uploaded workload: the oracle on the listed
    (request, layer) pairs, the score-mass property everywhere."""
    import paper_2410_23317_amd as V
    print(f"[case] window attention cfg={cfg.name} m={cfg.m} tau={cfg.tau} g={cfg.g}", flush=True)
    shape = make_shape(cfg)
    ws = torch.empty(V.vlc_window_attn_workspace_bytes(shape), dtype=torch.uint8, device="cuda")
    out = torch.empty_like(dev["q_win"])
    row_max = torch.empty((cfg.B, cfg.L, cfg.Hq, cfg.tau), dtype=torch.float32, device="cuda")
    row_sum = torch.empty_like(row_max)
    scores = torch.empty((cfg.B, cfg.L, cfg.Hkv, cfg.m), dtype=torch.float32, device="cuda")
    nnz = torch.empty((cfg.B, cfg.L, cfg.Hq), dtype=torch.int64, device="cuda")
    V.vlc_window_attn(shape, dev["q_win"], dev["k"], dev["v"], dev["sm_scale"], out, row_max, row_sum, ws)
    V.vlc_score_from_stats(shape, dev["q_win"], dev["k"], dev["sm_scale"], 0.01, row_max, row_sum, scores, nnz)
    torch.cuda.synchronize()
    assert torch.isfinite(out.float()).all()
    np.testing.assert_allclose(scores.sum(-1).cpu().numpy(), cfg.g * cfg.tau, rtol=1e-4)
    scales = W.sm_scale(cfg)
    for b in requests_to_check:
        for l in layers_to_check:
            t = W.layer_inputs(cfg, b, l)
            what = f"{cfg.name} b={b} l={l} window attention"
            o_ref, M, Z = O.window_attention(t["q_win"], t["k"], t["v"], scales[l])
            otol = dict(atol=2e-2, rtol=1e-2) if cfg.dtype == "bf16" else dict(atol=1e-4, rtol=1e-4)
            assert_close(out[b, l].float().cpu().numpy(), o_ref, what=what + " out", **otol)
            assert_close(row_max[b, l].cpu().numpy(), M, atol=2e-5, rtol=2e-6, what=what + " row_max")
            assert_close(row_sum[b, l].cpu().numpy(), Z, atol=0, rtol=5e-5, what=what + " row_sum")
            psi, _ = O.score_from_stats(t["q_win"], t["k"], scales[l], M, Z)
            assert_close(scores[b, l].cpu().numpy(), psi, what=what + " scores", **SCORE_TOL)
            check_nnz(nnz[b, l].cpu().numpy(), t["q_win"], t["k"], scales[l], 0.01, what + " nnz")
