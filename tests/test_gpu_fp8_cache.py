"""The compressed cache stored as per-row scaled FP8 E4M3: the stored codes and scales are bit-exact
against the oracle's quantiser (the same fp32 divisions and round-to-nearest-even), and decode
attention over the dequantised rows, with quantise-on-append, stays within the decode tolerance."""
import numpy as np
import pytest
import torch

import workloads as W
from oracle import vlcache_oracle as O

pytestmark = pytest.mark.gpu

from gpu_util import assert_close, decode_upload, make_shape, out_tol, upload


@pytest.mark.parametrize("kw", [
    dict(cid=400, d=128, Hq=8, Hkv=2, m=900, tau=24, lead_text=8, n_visual=860, L=3, B=2, sinks=4),
    dict(cid=401, d=64, Hq=6, Hkv=2, m=333, tau=7, lead_text=5, n_visual=300, L=2, B=1, sinks=2),
    dict(cid=402, d=128, Hq=7, Hkv=1, m=1500, tau=33, lead_text=10, n_visual=1400, L=2, B=1, sinks=8),   # rows of several units
])
def test_fp8_cache_codes_are_exact_and_decode_matches_the_oracle(kw):
    import paper_2410_23317_amd as V
    from paper_2410_23317_amd.pipeline import VLCachePath, cache_layer_view
    cfg = W.custom_config(name=f"fp8-{kw['cid']}", dtype="bf16", alphas=((1, 4),), steps=4, **kw)
    dev = upload(cfg)
    T = 4
    ref = VLCachePath(make_shape(cfg), alpha=(1, 4), T_max=T, want_idx=True)                 # native cache: same selection
    ref.compress(dev["q_win"], dev["k"], dev["v"], dev["sm_scale"])
    path = VLCachePath(make_shape(cfg), alpha=(1, 4), T_max=T, want_idx=True, kv_fp8=True)
    path.compress(dev["q_win"], dev["k"], dev["v"], dev["sm_scale"])
    path.status()
    torch.cuda.synchronize()
    assert torch.equal(path.idx_out, ref.idx_out) and torch.equal(path.k, ref.k)
    assert path.cache.arena.numel() < 0.62 * ref.cache.arena.numel() or cfg.m < 400       # K/V bytes halve, scales add 3 %
    scales = W.sm_scale(cfg)
    cache = O.CompressedCache(cfg.B, cfg.L, cfg.Hkv, fp8=True)
    kk = path.k.cpu().numpy()
    for b in range(cfg.B):
        for l in range(cfg.L):
            t = W.layer_inputs(cfg, b, l)
            (kcod, ksc), (vcod, vsc), idx = cache_layer_view(path.cache, b, l)
            idx = idx.cpu().numpy()
            for h in range(cfg.Hkv):
                wk, wks = O.quantize_e4m3_rows(t["k"][h][idx[h]])
                wv, wvs = O.quantize_e4m3_rows(t["v"][h][idx[h]])
                assert np.array_equal(kcod[h].cpu().numpy(), wk) and np.array_equal(vcod[h].cpu().numpy(), wv), (b, l, h)
                assert np.array_equal(ksc[h].cpu().numpy(), wks) and np.array_equal(vsc[h].cpu().numpy(), wvs), (b, l, h)
            psi = np.zeros((cfg.Hkv, cfg.m))
            for h in range(cfg.Hkv):
                psi[h, idx[h]] = 1.0                                                    # the oracle keeps exactly the GPU's set
            cache.fill_layer(b, l, psi, int(kk[b, l]), t["k"], t["v"])
            for h in range(cfg.Hkv):
                assert np.array_equal(cache.idx[b][l][h], idx[h])
    out = torch.empty((cfg.L, cfg.B, cfg.Hq, cfg.d), dtype=torch.bfloat16, device="cuda")
    for step in range(T):
        d_dev, d_host = decode_upload(cfg, step)
        path.decode(0, cfg.L, d_dev["q"], d_dev["k_new"], d_dev["v_new"], dev["sm_scale"], out)
        torch.cuda.synchronize()
        got = out.float().cpu().numpy()
        for l in range(cfg.L):
            want = cache.decode_layer(l, d_host["q"][l], d_host["k_new"][l], d_host["v_new"][l], scales[l])
            assert_close(got[l], want, what=f"fp8 decode step={step} l={l}", **out_tol(cfg))
    # the appended rows were quantised the same way
    for b in range(cfg.B):
        for l in range(cfg.L):
            (kcod, ksc), (vcod, vsc), idx = cache_layer_view(path.cache, b, l, appended=T)
            for step in range(T):
                d = W.decode_step_inputs(cfg, step)
                for h in range(cfg.Hkv):
                    wk, wks = O.quantize_e4m3_rows(d["k_new"][l, b, h][None])
                    wv, wvs = O.quantize_e4m3_rows(d["v_new"][l, b, h][None])
                    r = int(kk[b, l]) + step
                    assert np.array_equal(kcod[h, r].cpu().numpy(), wk[0]) and ksc[h, r].item() == wks[0]
                    assert np.array_equal(vcod[h, r].cpu().numpy(), wv[0]) and vsc[h, r].item() == wvs[0]
                    assert int(idx[h, r]) == cfg.m + step


def test_fp8_cache_needs_bf16_storage():
    import paper_2410_23317_amd as V
    shape = V.make_shape(1, 1, 2, 2, 64, 100, 4, "f32")
    with pytest.raises(V.VlcError) as e:
        V.vlc_cache_create_fp8(shape, 2, 20)
    assert e.value.status in (V.VLC_ERR_DTYPE, V.VLC_ERR_INVALID_ARG)


def test_fp8_cache_with_a_ragged_batch_and_a_recent_window():
    """The options compose: per-request lengths, a recent window that is a tenth of each layer's budget,
    FP8 storage.  Kept positions against the oracle's TopK on the GPU's own scores, stored rows
    against the oracle's quantiser."""
    import paper_2410_23317_amd as V
    from paper_2410_23317_amd.pipeline import VLCachePath, cache_layer_view
    lens = [(700, 30), (260, 12)]
    cfgs = [W.custom_config(cid=410 + i, name=f"combo{i}", dtype="bf16", d=128, Hq=8, Hkv=2, L=2, B=1, m=m, tau=t,
                            lead_text=6, n_visual=m - t - 12, sinks=3, alphas=((1, 5),)) for i, (m, t) in enumerate(lens)]
    B, L, Hq, Hkv, d, m_max, tau_max = 2, 2, 8, 2, 128, 700, 30
    dt = torch.bfloat16
    q_win = torch.full((B, L, Hq, tau_max, d), float("nan"), dtype=dt, device="cuda")
    k = torch.full((B, L, Hkv, m_max, d), float("nan"), dtype=dt, device="cuda")
    v = torch.full_like(k, float("nan"))
    host = {}
    for b, cfg in enumerate(cfgs):
        for l in range(L):
            t = host[(b, l)] = W.layer_inputs(cfg, 0, l)
            q_win[b, l, :, : cfg.tau].copy_(torch.from_numpy(t["q_win"]).to(dt))
            k[b, l, :, : cfg.m].copy_(torch.from_numpy(t["k"]).to(dt))
            v[b, l, :, : cfg.m].copy_(torch.from_numpy(t["v"]).to(dt))
    sm = torch.from_numpy(W.sm_scale(cfgs[0])).cuda()
    lens_t = torch.tensor(lens, dtype=torch.int32, device="cuda")
    shape = V.make_shape(B, L, Hq, Hkv, d, m_max, tau_max, "bf16", lens=lens_t)
    path = VLCachePath(shape, alpha=(1, 5), T_max=2, want_idx=True, recent_frac=(1, 10), lens=lens_t, kv_fp8=True)
    path.compress(q_win, k, v, sm)
    path.status()
    torch.cuda.synchronize()
    scores, kk = path.scores.cpu().numpy(), path.k.cpu().numpy()
    for b, cfg in enumerate(cfgs):
        for l in range(L):
            (kcod, ksc), (vcod, vsc), idx = cache_layer_view(path.cache, b, l)
            idx = idx.cpu().numpy()
            k_l = int(kk[b, l])
            for h in range(Hkv):
                want = O.topk(scores[b, l, h, : cfg.m].astype(np.float64), k_l, O.recent_count(k_l, 1, 10))
                assert np.array_equal(idx[h], want), (b, l, h)
                wk, wks = O.quantize_e4m3_rows(host[(b, l)]["k"][h][idx[h]])
                assert np.array_equal(kcod[h].cpu().numpy(), wk) and np.array_equal(ksc[h].cpu().numpy(), wks)
    out = torch.empty((L, B, Hq, d), dtype=dt, device="cuda")
    q = torch.randn((L, B, Hq, d), device="cuda").to(dt)
    kn = torch.randn((L, B, Hkv, d), device="cuda").to(dt)
    path.decode(0, L, q, kn, kn, sm, out)
    torch.cuda.synchronize()
    assert torch.isfinite(out.float()).all()
