"""Ragged batches: requests of different prompt and window length in one call, given as the optional
per-request array of the shape.  Every request is checked against the oracle run on that request alone;
the padding of the batch tensors is filled with NaN, so any read beyond a request's own lengths shows."""
import numpy as np
import pytest
import torch

import workloads as W
from oracle import vlcache_oracle as O

pytestmark = pytest.mark.gpu

from gpu_util import SCORE_TOL, assert_close, check_nnz, check_topk, out_tol, torch_dtype


def _requests(dtype, d, Hq, Hkv, L, lens, cid0):
    out = []
    for i, (m, tau) in enumerate(lens):
        lead = max(0, min(8, m - tau - 1))
        nvis = max(0, m - tau - lead - 4)
        out.append(W.custom_config(cid=cid0 + i, name=f"ragged{cid0 + i}", dtype=dtype, d=d, Hq=Hq, Hkv=Hkv, L=L, B=1, m=m,
                                   tau=tau, lead_text=lead, n_visual=nvis, sinks=min(3, nvis), alphas=((1, 5),)))
    return out


@pytest.mark.parametrize("dtype,d,Hq,Hkv,L,lens", [
    ("bf16", 128, 8, 2, 3, [(900, 40), (333, 7), (1200, 64), (64, 64)]),       # matrix-core sweeps, 8-wave blocks
    ("bf16", 128, 4, 1, 2, [(257, 1), (700, 33)]),                             # window rows padded to 64 per head
    ("f32", 64, 4, 2, 2, [(300, 20), (123, 9), (511, 31)]),                    # plain-ALU sweeps
])
def test_ragged_batch_matches_the_oracle_request_by_request(dtype, d, Hq, Hkv, L, lens):
    _ragged_case(dtype, d, Hq, Hkv, L, lens)


def test_ragged_batch_with_the_layout_in_a_kernel_of_its_own():
    """The same comparison with the cache layout forced out of the selection kernel (the form large batches take)."""
    _ragged_case("bf16", 128, 8, 2, 3, [(900, 40), (333, 7), (1200, 64), (64, 64)], options=dict(select_fold=1))


def _ragged_case(dtype, d, Hq, Hkv, L, lens, options=None):
    import paper_2410_23317_amd as V
    from paper_2410_23317_amd.pipeline import VLCachePath, cache_layer_view
    cfgs = _requests(dtype, d, Hq, Hkv, L, lens, cid0=300)
    B, m_max, tau_max = len(lens), max(m for m, _ in lens), max(t for _, t in lens)
    dt = torch_dtype(cfgs[0])
    q_win = torch.full((B, L, Hq, tau_max, d), float("nan"), dtype=dt, device="cuda")
    k = torch.full((B, L, Hkv, m_max, d), float("nan"), dtype=dt, device="cuda")
    v = torch.full((B, L, Hkv, m_max, d), float("nan"), dtype=dt, device="cuda")
    host = {}
    for b, cfg in enumerate(cfgs):
        for l in range(L):
            t = W.layer_inputs(cfg, 0, l)
            host[(b, l)] = t
            q_win[b, l, :, : cfg.tau].copy_(torch.from_numpy(t["q_win"]).to(dt))
            k[b, l, :, : cfg.m].copy_(torch.from_numpy(t["k"]).to(dt))
            v[b, l, :, : cfg.m].copy_(torch.from_numpy(t["v"]).to(dt))
    scales = W.sm_scale(cfgs[0])                                   # one per-layer scale array for the whole call
    sm = torch.from_numpy(scales).cuda()
    lens_t = torch.tensor(lens, dtype=torch.int32, device="cuda")
    shape = V.make_shape(B, L, Hq, Hkv, d, m_max, tau_max, dtype, lens=lens_t)
    alpha, T = (1, 5), 3
    path = VLCachePath(shape, alpha=alpha, p=0.01, T_max=T, want_idx=True, lens=lens_t,
                       options=None if options is None else V.make_options(**options))
    path.row_max.fill_(123.0)
    path.compress(q_win, k, v, sm)
    path.status()
    torch.cuda.synchronize()
    scores, nnz, kk = path.scores.cpu().numpy(), path.nnz.cpu().numpy(), path.k.cpu().numpy()
    assert np.isfinite(scores).all()
    caches, flips = {}, 0
    for b, cfg in enumerate(cfgs):
        assert np.all(scores[b, :, :, cfg.m:] == 0), "keys beyond the request's prompt must score zero"
        assert torch.all(path.row_max[b, :, :, cfg.tau:] == 123.0), "window rows beyond the request's are left untouched"
        k_o, beta_o = O.allocate(nnz[b], cfg.m, *alpha)            # budgets from the request's own m: bit-exact on the GPU's counts
        assert np.array_equal(kk[b], k_o), (b, kk[b], k_o)
        np.testing.assert_allclose(path.beta[b].cpu().numpy(), beta_o, rtol=1e-6)
        for l in range(L):
            t = host[(b, l)]
            psi, _, M, Z = O.score(t["q_win"], t["k"], scales[l])
            what = f"ragged b={b} l={l}"
            assert_close(scores[b, l, :, : cfg.m], psi, what=what + " scores", **SCORE_TOL)
            assert_close(path.row_max[b, l, :, : cfg.tau].cpu().numpy(), M, atol=2e-5, rtol=2e-6, what=what + " row_max")
            assert_close(path.row_sum[b, l, :, : cfg.tau].cpu().numpy(), Z, atol=0, rtol=5e-5, what=what + " row_sum")
            _, dflip = check_nnz(nnz[b, l], t["q_win"], t["k"], scales[l], 0.01, what + " nnz")
            flips += dflip
            np.testing.assert_allclose(path.gamma[b, l].cpu().numpy(), 1 - nnz[b, l] / O.region_size(cfg.m, cfg.tau),
                                       rtol=1e-6, atol=1e-7)
            kc, vc, idx = cache_layer_view(path.cache, b, l)
            kc, vc, idx = kc.float().cpu().numpy(), vc.float().cpu().numpy(), idx.cpu().numpy()
            for h in range(Hkv):
                check_topk(idx[h], psi[h], int(kk[b, l]), what + f" hkv={h} topk")
                assert idx[h].max() < cfg.m
                assert np.array_equal(kc[h], t["k"][h][idx[h]]) and np.array_equal(vc[h], t["v"][h][idx[h]])
            caches[(b, l)] = ([kc[h] for h in range(Hkv)], [vc[h] for h in range(Hkv)])
    # decode steps over the ragged cache
    out = torch.empty((L, B, Hq, d), dtype=dt, device="cuda")
    for step in range(T):
        dec = [W.decode_step_inputs(cfg, step) for cfg in cfgs]                 # each [L, 1, H, d]
        stack = {n: np.concatenate([x[n] for x in dec], axis=1) for n in ("q", "k_new", "v_new")}
        dev = {n: torch.from_numpy(a).to(dt).cuda() for n, a in stack.items()}
        path.decode(0, L, dev["q"], dev["k_new"], dev["v_new"], sm, out)
        torch.cuda.synchronize()
        got = out.float().cpu().numpy()
        for b in range(B):
            for l in range(L):
                kc, vc = caches[(b, l)]
                kc = [np.concatenate([kc[h], stack["k_new"][l, b, h][None]]) for h in range(Hkv)]
                vc = [np.concatenate([vc[h], stack["v_new"][l, b, h][None]]) for h in range(Hkv)]
                caches[(b, l)] = (kc, vc)
                want = O.decode_attn(stack["q"][l, b], kc, vc, scales[l])
                assert_close(got[l, b], want, what=f"ragged decode step={step} b={b} l={l}", **out_tol(cfgs[0]))
    # the diagnostic sees the request's own prompt only
    q_next = torch.from_numpy(np.concatenate([W.decode_step_inputs(cfg, 0)["q"] for cfg in cfgs], axis=1)).to(dt).cuda()
    hits, rate, star = path.hit_rate(q_next.permute(1, 0, 2, 3).contiguous(), k, sm)
    torch.cuda.synchronize()
    star, hits = star.cpu().numpy(), hits.cpu().numpy()
    for b, cfg in enumerate(cfgs):
        assert np.all(star[b, :, :, cfg.m:] == 0)
        for l in range(L):
            _, _, idx = cache_layer_view(path.cache, b, l, appended=0)
            for h in range(Hkv):
                want, _ = O.cache_hit_rate(star[b, l, h, : cfg.m].astype(np.float64), idx[h].cpu().numpy()[: kk[b, l]], int(kk[b, l]))
                assert hits[b, l, h] == want


def test_invalid_request_lengths_are_reported_by_the_cache():
    import paper_2410_23317_amd as V
    B, L, m, tau, d = 2, 1, 200, 8, 64
    lens = torch.tensor([[150, 8], [300, 4]], dtype=torch.int32, device="cuda")        # m_b = 300 exceeds m
    shape = V.make_shape(B, L, 2, 2, d, m, tau, "f32", lens=lens)
    cache = V.vlc_cache_create(shape, 2, 40)
    K = torch.zeros((B, L, 2, m, d), device="cuda")
    scores = torch.rand((B, L, 2, m), device="cuda")
    kk = torch.full((B, L), 10, dtype=torch.int32, device="cuda")
    V.vlc_topk_compact(cache, scores, kk, 0, K, K, None)
    with pytest.raises(V.VlcError) as e:
        V.vlc_cache_status(cache)
    assert e.value.status == V.VLC_ERR_INVALID_ARG and "request 1" in str(e.value)
