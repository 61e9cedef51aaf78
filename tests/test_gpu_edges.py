"""Edge cases of the HIP path against the oracle: allocation clips, TopK ties and extremes, the
recent window, device-side error flags, the standalone sparsity sweep, full-budget decode,
decode without append, determinism, and the alternative code paths (plain-ALU scoring sweeps,
multi-unit decode merges)."""
import os

import numpy as np
import pytest
import torch

import workloads as W
from oracle import vlcache_oracle as O

pytestmark = pytest.mark.gpu


def _V():
    import paper_2410_23317_amd as V
    return V


def test_allocate_bit_exact_on_random_counts_including_clips():
    V = _V()
    r = np.random.default_rng(3)
    cases = [(1, 2, 4, 512, 32, (1, 10)), (3, 32, 32, 2944, 32, (1, 10)), (2, 60, 56, 10368, 64, (1, 10)),
             (1, 32, 32, 32768, 64, (1, 100)), (2, 7, 8, 300, 8, (1, 1)), (1, 1, 8, 64, 8, (1, 2)),
             (2, 33, 16, 5000, 16, (3, 100))]
    for B, L, Hq, m, tau, alpha in cases:
        shape = V.make_shape(B, L, Hq, Hq, 128, m, tau, "bf16")
        D = O.region_size(m, tau)
        for spread in (1, 3, 6):
            hi = np.maximum(tau + 1, D // 10 ** r.integers(0, spread, size=(B, L, 1)))
            nnz = r.integers(tau, hi, size=(B, L, Hq))
            if spread == 6:
                nnz[0, 0] = 0 if L > 1 else nnz[0, 0]
            t = torch.from_numpy(nnz.astype(np.int64)).cuda()
            k = torch.empty((B, L), dtype=torch.int32, device="cuda")
            beta = torch.empty((B, L), dtype=torch.float32, device="cuda")
            V.vlc_allocate(shape, t, alpha[0], alpha[1], k, beta)
            for b in range(B):
                want, bw = O.allocate(nnz[b], m, *alpha)
                assert np.array_equal(k[b].cpu().numpy(), want), (B, L, Hq, m, alpha, spread)
                np.testing.assert_allclose(beta[b].cpu().numpy(), bw, rtol=1e-6)
    # all-zero counts: equal split
    shape = V.make_shape(1, 4, 2, 2, 128, 1000, 8, "bf16")
    k = torch.empty((1, 4), dtype=torch.int32, device="cuda")
    V.vlc_allocate(shape, torch.zeros((1, 4, 2), dtype=torch.int64, device="cuda"), 1, 10, k, None)
    assert k.cpu().numpy().tolist() == [O.allocate(np.zeros((4, 2), dtype=np.int64), 1000, 1, 10)[0].tolist()]


def _topk_case(V, scores, kk, n_recent, m, Hkv=2, L=1, B=1, T_max=2, d=64, options=None):
    """Run vlc_topk_compact alone on given scores [B,L,Hkv,m] and budgets [B,L]; returns (path-like cache, idx_out, K, Vv)."""
    from paper_2410_23317_amd.pipeline import cache_layer_view
    shape = V.make_shape(B, L, Hkv, Hkv, d, m, 1, "f32")
    cache = V.vlc_cache_create_opt(shape, T_max, min(L * m, int(max(kk.sum(1).max(), L))),
                                   V.make_options(**(options or {})))
    g = torch.Generator(device="cpu").manual_seed(1)
    K = torch.randn((B, L, Hkv, m, d), generator=g).cuda()
    Vv = torch.randn((B, L, Hkv, m, d), generator=g).cuda()
    idx_out = torch.full((B, L, Hkv, m), -1, dtype=torch.int32, device="cuda")
    V.vlc_topk_compact(cache, torch.from_numpy(scores.astype(np.float32)).cuda(),
                       torch.from_numpy(kk.astype(np.int32)).cuda(), n_recent, K, Vv, idx_out)
    torch.cuda.synchronize()
    return cache, idx_out, K, Vv, cache_layer_view


def test_topk_ties_extremes_and_recent_window():
    V = _V()
    r = np.random.default_rng(5)
    m = 1000
    for trial, (k, n_recent) in enumerate([(1, 0), (m, 0), (137, 0), (500, 0), (64, 16), (10, 10), (5, 9), (999, 0)]):
        scores = np.round(r.random((1, 1, 2, m)), 2) if trial % 2 == 0 else r.standard_normal((1, 1, 2, m))
        scores = scores.astype(np.float32)
        cache, idx_out, K, Vv, view = _topk_case(V, scores, np.array([[k]]), n_recent, m)
        V.vlc_cache_status(cache)
        kc, vc, idx = view(cache, 0, 0)
        for h in range(2):
            want = O.topk(scores[0, 0, h].astype(np.float64), k, n_recent)      # exact: ties to the lower position
            assert np.array_equal(idx[h].cpu().numpy(), want), (k, n_recent, h)
            assert np.array_equal(idx_out[0, 0, h, :k].cpu().numpy(), want)
            assert torch.equal(kc[h], K[0, 0, h][torch.from_numpy(want).cuda()])
            assert torch.equal(vc[h], Vv[0, 0, h][torch.from_numpy(want).cuda()])
    # all scores equal: the first k positions; negative and zero scores order correctly
    scores = np.zeros((1, 1, 2, m), dtype=np.float32)
    scores[0, 0, 1] = -np.arange(m)
    cache, idx_out, *_ , view = _topk_case(V, scores, np.array([[7]]), 0, m)
    _, _, idx = view(cache, 0, 0)
    assert idx[0].cpu().numpy().tolist() == list(range(7)) and idx[1].cpu().numpy().tolist() == list(range(7))


@pytest.mark.parametrize("fold", [1, 2])
def test_layout_as_its_own_kernel_or_inside_the_selection(fold):
    """Small batches build the cache layout in one extra block of the selection kernel, large ones in a kernel of
    its own.  Both forms, forced by the cache option on the same batch (unequal budgets, one of them invalid): kept
    positions against the oracle's TopK, gathered rows, the error report, and the decode work list via a decode
    call whose result must not depend on the form."""
    V = _V()
    r = np.random.default_rng(11)
    m, B, L, Hkv = 700, 2, 3, 2
    scores = r.standard_normal((B, L, Hkv, m)).astype(np.float32)
    kk = np.array([[40, 700, 1], [333, 0, 90]])
    cache, idx_out, K, Vv, view = _topk_case(V, scores, kk, 0, m, Hkv=Hkv, L=L, B=B, options=dict(select_fold=fold))
    with pytest.raises(V.VlcError) as e:
        V.vlc_cache_status(cache)
    assert e.value.status == V.VLC_ERR_INVALID_ARG and "k[1][1]" in str(e.value)
    for b in range(B):
        for l in range(L):
            if kk[b, l] == 0:
                continue
            kc, vc, idx = view(cache, b, l)
            for h in range(Hkv):
                want = O.topk(scores[b, l, h].astype(np.float64), int(kk[b, l]), 0)
                assert np.array_equal(idx[h].cpu().numpy(), want), (b, l, h)
                assert np.array_equal(idx_out[b, l, h, : kk[b, l]].cpu().numpy(), want)
                assert torch.equal(kc[h], K[b, l, h][torch.from_numpy(want).cuda()])
                assert torch.equal(vc[h], Vv[b, l, h][torch.from_numpy(want).cuda()])
    # one decode step over all layers: plain attention over the kept rows (fp64 on the host)
    g = torch.Generator(device="cpu").manual_seed(3)
    q = torch.randn((L, B, Hkv, 64), generator=g).cuda()
    out = torch.full((L, B, Hkv, 64), 7.0, device="cuda")
    V.vlc_decode_attn(cache, 0, L, q, None, None, None, out)
    torch.cuda.synchronize()
    for b in range(B):
        for l in range(L):
            if kk[b, l] == 0:
                assert torch.all(out[l, b] == 0)
                continue
            kept = [O.topk(scores[b, l, h].astype(np.float64), int(kk[b, l]), 0) for h in range(Hkv)]
            ref = O.decode_attn(q[l, b].cpu().numpy(), [K[b, l, h].cpu().numpy()[kept[h]] for h in range(Hkv)],
                                [Vv[b, l, h].cpu().numpy()[kept[h]] for h in range(Hkv)], 1.0 / np.sqrt(64))
            np.testing.assert_allclose(out[l, b].cpu().numpy(), ref, rtol=2e-4, atol=2e-5)


def test_recent_fraction_extremes():
    """Fraction 0 keeps nothing unconditionally, fraction 1 keeps exactly the last k positions."""
    V = _V()
    from paper_2410_23317_amd.pipeline import cache_layer_view
    m, d = 500, 64
    r = np.random.default_rng(11)
    scores = r.random((1, 2, 2, m)).astype(np.float32)
    kk = np.array([[37, 120]])
    shape = V.make_shape(1, 2, 2, 2, d, m, 1, "f32")
    K = torch.randn((1, 2, 2, m, d)).cuda()
    for num, den in ((0, 1), (1, 1), (1, 3)):
        cache = V.vlc_cache_create(shape, 2, int(kk.sum()))
        V.vlc_topk_compact_recent_frac(cache, torch.from_numpy(scores).cuda(), torch.from_numpy(kk.astype(np.int32)).cuda(),
                                       num, den, K, K, None)
        V.vlc_cache_status(cache)
        for l in range(2):
            _, _, idx = cache_layer_view(cache, 0, l)
            c = O.recent_count(int(kk[0, l]), num, den)
            for h in range(2):
                want = O.topk(scores[0, l, h].astype(np.float64), int(kk[0, l]), c)
                assert np.array_equal(idx[h].cpu().numpy(), want), (num, den, l, h)
                if (num, den) == (1, 1):
                    assert want.tolist() == list(range(m - int(kk[0, l]), m))


@pytest.mark.parametrize("m", [4096, 4097, 12288, 12289, 32768, 32769, 40001])
def test_topk_row_lengths_around_the_register_resident_limits(m):
    """The selection keeps a row's keys in registers up to 32768 positions (8, 24 or 64 per lane)
    and streams longer rows; each variant, with heavy ties and a ragged tail, against the oracle."""
    V = _V()
    r = np.random.default_rng(m)
    scores = np.empty((1, 1, 2, m), dtype=np.float32)
    scores[0, 0, 0] = np.round(r.random(m), 3)                     # ~1000 distinct values: many ties at the cut
    scores[0, 0, 1] = r.standard_normal(m) * 1e-3
    for k, n_recent in [(m // 10, 0), (m - 1, 0), (257, 31)]:
        cache, idx_out, K, Vv, view = _topk_case(V, scores, np.array([[k]]), n_recent, m, d=64)
        V.vlc_cache_status(cache)
        kc, vc, idx = view(cache, 0, 0)
        for h in range(2):
            want = O.topk(scores[0, 0, h].astype(np.float64), k, n_recent)
            assert np.array_equal(idx[h].cpu().numpy(), want), (m, k, n_recent, h)
            assert torch.equal(kc[h], K[0, 0, h][torch.from_numpy(want).cuda()])


def test_device_side_errors_are_sticky_and_harmless():
    V = _V()
    m = 300
    scores = np.random.default_rng(0).random((2, 3, 2, m)).astype(np.float32)
    # a budget outside [1, m]
    kk = np.array([[10, 0, 12], [5, 6, 7]])
    cache, *_ = _topk_case(V, scores, np.maximum(kk, 1) * 0 + kk, 0, m, L=3, B=2)
    with pytest.raises(V.VlcError) as e:
        V.vlc_cache_status(cache)
    assert e.value.status == V.VLC_ERR_INVALID_ARG and "k[0][1]" in str(e.value)
    # budgets that do not fit the arena of a request
    shape = V.make_shape(2, 3, 2, 2, 64, m, 1, "f32")
    cache = V.vlc_cache_create(shape, 2, 30)
    K = torch.zeros((2, 3, 2, m, 64), device="cuda")
    big = torch.tensor([[10, 10, 10], [10, 15, 10]], dtype=torch.int32, device="cuda")
    V.vlc_topk_compact(cache, torch.from_numpy(scores).cuda(), big, 0, K, K, None)
    with pytest.raises(V.VlcError) as e:
        V.vlc_cache_status(cache)
    assert e.value.status == V.VLC_ERR_CAPACITY and "request 1" in str(e.value)
    # the rejected request decodes to zeros, the other one normally; a later good call clears the flag
    q = torch.randn((3, 2, 2, 64), device="cuda")
    out = torch.full((3, 2, 2, 64), 7.0, device="cuda")
    V.vlc_decode_attn(cache, 0, 3, q, None, None, None, out)
    torch.cuda.synchronize()
    assert torch.all(out[:, 1] == 0) and torch.all(out[:, 0] == 0)      # V is all zeros here
    ok = torch.full((2, 3), 10, dtype=torch.int32, device="cuda")
    V.vlc_topk_compact(cache, torch.from_numpy(scores).cuda(), ok, 0, K, K, None)
    V.vlc_cache_status(cache)
    # more appends than reserved: host-side error, nothing enqueued
    kn = torch.zeros((3, 2, 2, 64), device="cuda")
    V.vlc_decode_attn(cache, 0, 3, q, kn, kn, None, out)
    V.vlc_decode_attn(cache, 0, 3, q, kn, kn, None, out)
    with pytest.raises(V.VlcError) as e:
        V.vlc_decode_attn(cache, 0, 3, q, kn, kn, None, out)
    assert e.value.status == V.VLC_ERR_CAPACITY
    # layers with different append counts cannot share a call
    V.vlc_topk_compact(cache, torch.from_numpy(scores).cuda(), ok, 0, K, K, None)
    V.vlc_decode_attn(cache, 0, 1, q[:1], kn[:1], kn[:1], None, out[:1])
    with pytest.raises(V.VlcError) as e:
        V.vlc_decode_attn(cache, 0, 3, q, kn, kn, None, out)
    assert e.value.status == V.VLC_ERR_INVALID_ARG
    V.vlc_cache_status(cache)


def _small_cfg(**kw):
    base = dict(cid=80, name="edge", dtype="bf16", d=128, Hq=8, Hkv=2, m=777, tau=32, lead_text=9, n_visual=700,
                L=3, B=2, sinks=6, alphas=((1, 5),))
    base.update(kw)
    return W.custom_config(**base)


def test_standalone_sparsity_sweep_matches_the_fused_counts():
    V = _V()
    from gpu_util import make_shape, upload
    from paper_2410_23317_amd.pipeline import VLCachePath
    for cfg in (_small_cfg(), _small_cfg(cid=81, dtype="f32", d=64, m=300, n_visual=250, tau=9)):
        dev = upload(cfg, want_v=False)
        path = VLCachePath(make_shape(cfg), alpha=(1, 5), T_max=1)
        path.score(dev["q_win"], dev["k"], dev["sm_scale"])
        fused = path.nnz.clone()
        for rm in (path.row_max, None):
            nnz = torch.full_like(fused, -1)
            gamma = torch.empty_like(path.gamma)
            V.vlc_sparsity(path.shape, dev["q_win"], dev["k"], dev["sm_scale"], rm, 0.01, nnz, gamma, path.workspace)
            torch.cuda.synchronize()
            if rm is None:
                assert torch.equal(nnz, fused)          # same kernels, same exponent-domain row max
            else:
                assert (nnz - fused).abs().sum().item() <= 4     # row max round-trips through the natural-log domain
            D = O.region_size(cfg.m, cfg.tau)
            np.testing.assert_allclose(gamma.cpu().numpy(), 1 - nnz.cpu().numpy() / D, rtol=1e-6, atol=1e-7)
        # a different threshold gives different, monotone counts
        nnz2 = torch.empty_like(fused)
        V.vlc_sparsity(path.shape, dev["q_win"], dev["k"], dev["sm_scale"], path.row_max, 0.1, nnz2, None, path.workspace)
        assert torch.all(nnz2 <= fused) and torch.any(nnz2 < fused)


def test_plain_alu_scoring_path_agrees_with_the_matrix_core_path():
    V = _V()
    from gpu_util import make_shape, upload
    from paper_2410_23317_amd.pipeline import VLCachePath
    cfg = _small_cfg(cid=82, m=1500, n_visual=1400, tau=50, Hq=14, Hkv=2)        # g = 7, tau not a multiple of 32
    dev = upload(cfg, want_v=False)
    res = {}
    for mode, flags in (("mfma", 0), ("simple", V.VLC_SHAPE_SCORE_PLAIN_ALU)):
        path = VLCachePath(make_shape(cfg, flags=flags), alpha=(1, 5), T_max=1)
        path.score(dev["q_win"], dev["k"], dev["sm_scale"])
        torch.cuda.synchronize()
        res[mode] = (path.scores.cpu().numpy(), path.row_max.cpu().numpy(), path.row_sum.cpu().numpy(), path.nnz.cpu().numpy())
    assert not np.array_equal(res["mfma"][0], res["simple"][0]), "the flag did not change the kernels that ran"
    np.testing.assert_allclose(res["mfma"][0], res["simple"][0], rtol=5e-5, atol=1e-7)
    np.testing.assert_allclose(res["mfma"][1], res["simple"][1], rtol=2e-6, atol=2e-5)
    np.testing.assert_allclose(res["mfma"][2], res["simple"][2], rtol=5e-5)
    assert np.abs(res["mfma"][3] - res["simple"][3]).sum() <= 8
    # and both match the oracle on one layer
    t = W.layer_inputs(cfg, 1, 2, want_v=False)
    psi, _, M, Z = O.score(t["q_win"], t["k"], W.sm_scale(cfg)[2])
    np.testing.assert_allclose(res["mfma"][0][1, 2], psi, rtol=5e-5, atol=1e-7)


def test_full_budget_decode_equals_uncompressed_attention():
    V = _V()
    from gpu_util import assert_close, make_shape, upload
    from paper_2410_23317_amd.pipeline import VLCachePath, cache_layer_view
    cfg = _small_cfg(cid=83, m=401, n_visual=360, L=2, B=1)
    dev = upload(cfg)
    path = VLCachePath(make_shape(cfg), alpha=(1, 1), T_max=3)
    path.score(dev["q_win"], dev["k"], dev["sm_scale"])
    full = torch.full((cfg.B, cfg.L), cfg.m, dtype=torch.int32, device="cuda")
    path.topk_compact(dev["k"], dev["v"], k=full)
    path.status()
    kc, vc, idx = cache_layer_view(path.cache, 0, 1)
    assert torch.equal(idx[0].cpu(), torch.arange(cfg.m, dtype=torch.int32)) and torch.equal(kc, dev["k"][0, 1])
    scales = W.sm_scale(cfg)
    out = torch.empty((cfg.L, cfg.B, cfg.Hq, cfg.d), dtype=torch.bfloat16, device="cuda")
    d = W.decode_step_inputs(cfg, 0)
    dd = {n: torch.from_numpy(x).to(torch.bfloat16).cuda() for n, x in d.items()}
    # without append: attention over exactly the prompt's keys
    path.decode(0, cfg.L, dd["q"], None, None, dev["sm_scale"], out)
    for l in range(cfg.L):
        t = W.layer_inputs(cfg, 0, l)
        want = O.decode_attn(d["q"][l, 0], list(t["k"]), list(t["v"]), scales[l])
        assert_close(out[l, 0].float().cpu().numpy(), want, atol=2e-2, rtol=1e-2, what=f"no-append full-budget l={l}")
    # with append: the new token is attended too
    path.decode(0, cfg.L, dd["q"], dd["k_new"], dd["v_new"], dev["sm_scale"], out)
    for l in range(cfg.L):
        t = W.layer_inputs(cfg, 0, l)
        Kf = [np.concatenate([t["k"][h], d["k_new"][l, 0, h][None]]) for h in range(cfg.Hkv)]
        Vf = [np.concatenate([t["v"][h], d["v_new"][l, 0, h][None]]) for h in range(cfg.Hkv)]
        want = O.decode_attn(d["q"][l, 0], Kf, Vf, scales[l])
        assert_close(out[l, 0].float().cpu().numpy(), want, atol=2e-2, rtol=1e-2, what=f"append full-budget l={l}")


def test_compression_is_deterministic_and_steps_entry_point_matches_single_steps():
    V = _V()
    from gpu_util import make_shape, upload
    from paper_2410_23317_amd.pipeline import VLCachePath
    cfg = _small_cfg(cid=84)
    dev = upload(cfg)
    T = 4
    steps = [W.decode_step_inputs(cfg, t) for t in range(T)]
    stack = {n: torch.from_numpy(np.stack([s[n] for s in steps])).to(torch.bfloat16).cuda() for n in ("q", "k_new", "v_new")}
    outs = []
    for rep in range(2):
        path = VLCachePath(make_shape(cfg), alpha=(1, 5), T_max=T, want_idx=True)
        path.compress(dev["q_win"], dev["k"], dev["v"], dev["sm_scale"])
        out = torch.empty((T, cfg.L, cfg.B, cfg.Hq, cfg.d), dtype=torch.bfloat16, device="cuda")
        if rep == 0:
            path.decode_steps(0, cfg.L, T, stack["q"], stack["k_new"], stack["v_new"], dev["sm_scale"], out)
        else:
            for t in range(T):
                path.decode(0, cfg.L, stack["q"][t], stack["k_new"][t], stack["v_new"][t], dev["sm_scale"], out[t])
        path.status()
        outs.append((path.scores.clone(), path.nnz.clone(), path.k.clone(), path.idx_out.clone(), out))
    for a, b in zip(*outs):
        assert torch.equal(a, b)


def test_whole_path_replays_from_a_hip_graph():
    """Callers may record the path into a HIP graph (nothing in it allocates, synchronises or uses a
    memset node): every replay, with eager work and synchronisations in between, equals the eager run."""
    V = _V()
    from gpu_util import make_shape, upload
    from paper_2410_23317_amd.pipeline import VLCachePath
    cfg = _small_cfg(cid=86, m=1500, n_visual=1400)                 # rows of several 256-slot units: merges replay too
    dev = upload(cfg)
    T = 3
    steps = [W.decode_step_inputs(cfg, t) for t in range(T)]
    stack = {n: torch.from_numpy(np.stack([s[n] for s in steps])).to(torch.bfloat16).cuda() for n in ("q", "k_new", "v_new")}

    def run(path, out):
        path.compress(dev["q_win"], dev["k"], dev["v"], dev["sm_scale"])
        for t in range(T):
            path.decode(0, cfg.L, stack["q"][t], stack["k_new"][t], stack["v_new"][t], dev["sm_scale"], out[t])

    eager = VLCachePath(make_shape(cfg), alpha=(1, 2), T_max=T, want_idx=True)
    out_e = torch.empty((T, cfg.L, cfg.B, cfg.Hq, cfg.d), dtype=torch.bfloat16, device="cuda")
    run(eager, out_e)
    eager.status()
    path = VLCachePath(make_shape(cfg), alpha=(1, 2), T_max=T, want_idx=True)
    out_g = torch.zeros_like(out_e)
    run(path, out_g)                                                # warm-up outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run(path, out_g)
    for rep in range(3):
        out_g.zero_()
        path.scores.zero_(); path.k.zero_(); path.idx_out.fill_(-1)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        path.status()
        assert torch.equal(path.scores, eager.scores) and torch.equal(path.k, eager.k), rep
        assert torch.equal(path.idx_out, eager.idx_out) and torch.equal(path.nnz, eager.nnz), rep
        assert torch.equal(out_g, out_e), rep


@pytest.mark.parametrize("opt", [
    dict(unit_slots=128), dict(unit_slots=128, decode_merge=2), dict(unit_slots=256),
    dict(unit_slots=128, decode_order=2), dict(unit_slots=256, decode_order=2, decode_merge=2),
    dict(unit_slots=512, decode_order=2), dict(unit_slots=512, decode_zigzag=1),
    dict(unit_slots=256, decode_zigzag=2, decode_order=2), dict(unit_slots=512, tail_unit_slots=128, decode_order=2),
    dict(unit_slots=1024, tail_unit_slots=256, decode_order=2, decode_merge=2), dict(unit_slots=512, tail_unit_slots=128, decode_order=1),
], ids=lambda o: "-".join(f"{k}{v}" for k, v in o.items()))
@pytest.mark.parametrize("per_layer", [False, True], ids=["all-layers", "per-layer"])
def test_decode_merges_across_units(opt, per_layer):
    """Rows longer than one block-unit: partial results merged in-kernel (device-scope counter) or by the
    second kernel, with the work list walked layer-major or by size class, uniform or mixed unit sizes, tiles and
    whole units walked forwards and backwards on alternate steps or always forwards, all against the oracle.
    Launches per layer take the layer list, whose unit size follows the same option here."""
    from gpu_util import run_and_check
    cfg = _small_cfg(cid=85, m=1300, n_visual=1200, L=2, B=2, alphas=((1, 2),), Hq=14, Hkv=2)
    opt = dict(opt, layer_unit_slots=min(512, opt.get("tail_unit_slots", opt["unit_slots"])))
    run_and_check(cfg, (1, 2), 3, options=opt, per_layer_decode=per_layer)


def _direct_cache(V, cfg, kk, T_max, options):
    """A cache filled by vlc_topk_compact with GIVEN budgets kk [B, L] (scores are the workload's own); returns
    the path-like pieces and, per (b, l), the lists of kept K and V rows: the rows at the positions the cache holds,
    after those positions have been checked against the oracle's ranking (equal sets, except swaps among scores
    within 1e-5 of the k-th, which fp32 and fp64 scores may order differently)."""
    from gpu_util import make_shape, upload, check_topk
    from paper_2410_23317_amd.pipeline import VLCachePath, cache_layer_view
    dev = upload(cfg)
    path = VLCachePath(make_shape(cfg), alpha=(1, 2), T_max=T_max, options=V.make_options(**options))
    path.score(dev["q_win"], dev["k"], dev["sm_scale"])
    path.topk_compact(dev["k"], dev["v"], k=torch.from_numpy(kk.astype(np.int32)).cuda())
    path.status()
    scales = W.sm_scale(cfg)
    caches = {}
    swaps = 0
    for b in range(cfg.B):
        for l in range(cfg.L):
            t = W.layer_inputs(cfg, b, l)
            psi = O.score(t["q_win"], t["k"], scales[l])[0]
            idx = cache_layer_view(path.cache, b, l)[2].cpu().numpy()
            for h in range(cfg.Hkv):
                swaps += check_topk(idx[h], psi[h], int(kk[b, l]), f"b={b} l={l} hkv={h} topk")
            caches[(b, l)] = ([t["k"][h][idx[h]] for h in range(cfg.Hkv)], [t["v"][h][idx[h]] for h in range(cfg.Hkv)])
    print(f"[direct cache] topk swaps within the tie tolerance: {swaps}", flush=True)
    return path, dev, caches, scales


def _oracle_step(cfg, caches, scales, d_host, got, step, what):
    from gpu_util import assert_close, out_tol
    for (b, l), (kc, vc) in caches.items():
        for h in range(cfg.Hkv):
            kc[h] = np.concatenate([kc[h], d_host["k_new"][l, b, h][None]], 0)
            vc[h] = np.concatenate([vc[h], d_host["v_new"][l, b, h][None]], 0)
        want = O.decode_attn(d_host["q"][l, b], kc, vc, scales[l])
        assert_close(got[l, b], want, what=f"{what} step {step} b={b} l={l}", **out_tol(cfg))


@pytest.mark.parametrize("unit", [128, 256, 512, 2048])
@pytest.mark.parametrize("merge", [1, 2])
@pytest.mark.parametrize("order", [1, 2])
def test_rows_that_grow_across_a_unit_boundary_during_decode(unit, merge, order):
    """Budgets of unit - 2 (and 2 * unit - 2, and a short row) with 6 appended tokens: on the third step a unit
    that only held append reserve becomes live, the row goes from one unit to two (from two to three) and its
    result from a direct store to a merge of partials.  Every step against the oracle, launches over all layers
    and per layer, both merge forms, both orders of the work list."""
    V = _V()
    m = 1200 if unit <= 512 else 4400           # the arena holds m / 2 slots per layer (alpha = 1/2)
    cfg = _small_cfg(cid=88, m=m, n_visual=m - 100, L=3, B=2, Hq=8, Hkv=2)
    kk = np.array([[unit - 2, 2 * unit - 2, 40], [unit - 2, 7, 2 * unit - 2]])
    T = 6
    for per_layer in (False, True):
        opts = dict(unit_slots=unit, layer_unit_slots=unit, decode_merge=merge, decode_order=order)
        path, dev, caches, scales = _direct_cache(V, cfg, kk, T, opts)
        assert path.cache.layout.unit_slots == unit and path.cache.layout.layer_unit_slots == unit
        out = torch.empty((cfg.L, cfg.B, cfg.Hq, cfg.d), dtype=torch.bfloat16, device="cuda")
        crossed = False
        for step in range(T):
            d_host = W.decode_step_inputs(cfg, step)
            dd = {n: torch.from_numpy(x).to(torch.bfloat16).cuda() for n, x in d_host.items()}
            if per_layer:
                for l in range(cfg.L):
                    path.decode(l, l + 1, dd["q"][l], dd["k_new"][l], dd["v_new"][l], dev["sm_scale"], out[l])
            else:
                path.decode(0, cfg.L, dd["q"], dd["k_new"], dd["v_new"], dev["sm_scale"], out)
            torch.cuda.synchronize()
            _oracle_step(cfg, caches, scales, d_host, out.float().cpu().numpy(), step, f"unit={unit} per_layer={per_layer}")
            crossed |= (unit - 2 + step + 1) > unit
        assert crossed
        path.status()


@pytest.mark.parametrize("B,L,m", [(6, 5, 800), (40, 13, 800), (128, 16, 400)], ids=["30-entries", "520-entries", "2048-entries"])
def test_size_class_walk_with_budgets_of_every_length(B, L, m):
    """The size-class work list puts the partly filled units longest first (a sort of the (request, layer) entries
    on the device, up to the 2048 entries a cache may have).  Budgets from 1 slot to several units, many of them equal
    (ties in the sort), rows that end exactly on a unit boundary and rows that grow over one during the steps:
    every step against the oracle, launches over all layers."""
    V = _V()
    cfg = _small_cfg(cid=92, m=m, n_visual=m - 40, L=L, B=B, Hq=4, Hkv=2, d=64, tau=16)    # alpha 1/2: m / 2 slots a layer
    rng = np.random.default_rng(92 + B)
    sizes = np.array([1, 2, 63, 126, 127, 128, 129, 200, 254, 256, 257, 300, 383, 384, 400])
    kk = rng.choice(sizes[sizes <= m // 2], size=(B, L))
    T = 4
    path, dev, caches, scales = _direct_cache(V, cfg, kk, T, dict(unit_slots=128, decode_order=2))
    out = torch.empty((cfg.L, cfg.B, cfg.Hq, cfg.d), dtype=torch.bfloat16, device="cuda")
    for step in range(T):
        d_host = W.decode_step_inputs(cfg, step)
        dd = {n: torch.from_numpy(x).to(torch.bfloat16).cuda() for n, x in d_host.items()}
        path.decode(0, cfg.L, dd["q"], dd["k_new"], dd["v_new"], dev["sm_scale"], out)
        torch.cuda.synchronize()
        _oracle_step(cfg, caches, scales, d_host, out.float().cpu().numpy(), step, f"B={B} L={L}")
    path.status()


_WORK_ITEM = np.dtype([("row", "<i4"), ("key0", "<i4"), ("kept", "<i4"), ("unit", "<i4"), ("kbase", "<i8"), ("idx_base", "<i8"),
                       ("b", "<i4"), ("l", "<i4"), ("canon", "<i4"), ("ucap", "<i4"), ("hkv", "<i4"), ("layer_units", "<i4"),
                       ("pad", "<i4", (2,))])


def _read_list(path, i, L):
    """Work list i of a cache as the layout struct describes it: (records, layer index int32[L+2])."""
    lay = path.cache.layout
    index = path.cache.arena[lay.list_index_off[i]: lay.list_index_off[i] + 4 * (L + 2)].view(torch.int32).cpu().numpy()
    n = int(index[L])
    raw = path.cache.arena[lay.list_items_off[i]: lay.list_items_off[i] + 64 * n].cpu().numpy()
    return np.frombuffer(raw.tobytes(), dtype=_WORK_ITEM), index


@pytest.mark.parametrize("unit,tail", [(128, 128), (256, 128), (512, 128)])
def test_work_lists_hold_every_unit_once_and_the_size_classes_in_order(unit, tail):
    """The lists the decode and gather kernels walk, read back from the arena: every block-unit of every row exactly
    once in each list; the all-layer list by size class, i.e. first the whole units, then the other units that hold
    kept slots with the (request, layer) entries in the order of their slots beyond whole units, longest first and
    ties in (layer, request) order, then the units that only hold append reserve; the per-layer list in (layer,
    request, kv head, unit) order with its layer index."""
    assert _WORK_ITEM.itemsize == 64
    V = _V()
    B, L, Hkv, T = 5, 7, 2, 40
    cfg = _small_cfg(cid=93, m=1600, n_visual=1500, L=L, B=B, Hq=4, Hkv=Hkv, d=64, tau=16)
    rng = np.random.default_rng(93)
    kk = rng.choice(np.array([1, 50, 127, 128, 129, 255, 256, 300, 384, 511, 512, 513, 640, 700, 767, 768]), size=(B, L))
    path, dev, caches, scales = _direct_cache(V, cfg, kk, T, dict(unit_slots=unit, tail_unit_slots=tail, layer_unit_slots=128,
                                                                   decode_order=2))
    lay = path.cache.layout
    assert list(lay.list_by_size) == [0, 1, 0]

    def units_of(k, ub, us):                   # (first slot, slots of the unit) of every unit of a row with k kept slots
        big, rem = k // ub, k % ub
        small = -(-(rem + T) // us)
        return [(u * ub, ub) for u in range(big)] + [(big * ub + u * us, us) for u in range(small)]

    for i, (ub, us) in enumerate([(128, 128), (unit, tail), (256, 256)]):
        items, index = _read_list(path, i, L)
        want = {}
        for l in range(L):                                        # the order the position field counts in
            for b in range(B):
                for h in range(Hkv):
                    for u, (k0, cap) in enumerate(units_of(int(kk[b, l]), ub, us)):
                        want[((b * L + l) * Hkv + h, u)] = (len(want), k0, cap, b, l, h)
        assert len(items) == len(want), i
        got = {(int(r["row"]), int(r["unit"])): r for r in items}
        assert len(got) == len(items), f"list {i}: a unit is listed twice"
        for key, (canon, k0, cap, b, l, h) in want.items():
            r = got[key]
            assert (r["canon"], r["key0"], r["ucap"], r["b"], r["l"], r["hkv"], r["kept"]) == (canon, k0, cap, b, l, h, kk[b, l]), (i, key)
        firsts = [want[((0 * L + l) * Hkv + 0, 0)][0] for l in range(L)]
        assert index[:L].tolist() == firsts and index[L] == len(want), i
        if not lay.list_by_size[i]:
            assert items["canon"].tolist() == list(range(len(items))), i
            continue
        # size classes: whole units | units with kept slots, entries by slots beyond whole units, longest first | reserve
        whole = items["ucap"] == ub if ub != us else (items["key0"] + ub <= items["kept"])
        whole &= items["key0"] + items["ucap"] <= items["kept"] - items["kept"] % ub
        live = ~whole & (items["key0"] < items["kept"])
        cls = np.where(whole, 0, np.where(live, 1, 2))
        assert np.all(np.diff(cls) >= 0), "size classes out of order"
        assert int(whole.sum()) == int(index[L + 1])
        mid = items[cls == 1]
        fill = mid["kept"] % ub
        entry = mid["l"] * B + mid["b"]                           # ties keep the (layer, request) order
        order = list(zip((-fill).tolist(), entry.tolist()))
        assert order == sorted(order), "partly filled units are not longest first"
    path.status()


@pytest.mark.parametrize("fp8", [False, True], ids=["bf16-cache", "fp8-cache"])
def test_launches_over_layer_ranges_that_are_neither_one_layer_nor_all(fp8):
    """A decode step issued as launches over parts of the layer stack: [0,2) + [2,4) on even steps, [0,1) + [1,4) on
    odd ones.  A launch then starts inside the layer-ordered work list and counts its layers' units on two levels;
    every layer still receives one append per step.  Every step against the oracle, with rows that cross a unit
    boundary on the way."""
    V = _V()
    cfg = _small_cfg(cid=91, m=1500, n_visual=1400, L=4, B=2, Hq=8, Hkv=2)
    kk = np.array([[126, 300, 17, 254], [510, 1, 127, 700]])
    T = 6
    path, dev, caches, scales = _direct_cache(V, cfg, kk, T, dict(kv_fp8=int(fp8)))
    if fp8:
        for key, (kc, vc) in caches.items():
            caches[key] = ([O.dequantize_e4m3_rows(*O.quantize_e4m3_rows(x)) for x in kc],
                           [O.dequantize_e4m3_rows(*O.quantize_e4m3_rows(x)) for x in vc])
    out = torch.empty((cfg.L, cfg.B, cfg.Hq, cfg.d), dtype=torch.bfloat16, device="cuda")
    for step in range(T):
        d_host = W.decode_step_inputs(cfg, step)
        dd = {n: torch.from_numpy(x).to(torch.bfloat16).cuda() for n, x in d_host.items()}
        for a, b in (((0, 2), (2, 4)) if step % 2 == 0 else ((0, 1), (1, 4))):
            path.decode(a, b, dd["q"][a:b], dd["k_new"][a:b], dd["v_new"][a:b], dev["sm_scale"], out[a:b])
        torch.cuda.synchronize()
        if fp8:
            d_host = dict(d_host, k_new=O.dequantize_e4m3_rows(*O.quantize_e4m3_rows(d_host["k_new"])),
                          v_new=O.dequantize_e4m3_rows(*O.quantize_e4m3_rows(d_host["v_new"])))
        _oracle_step(cfg, caches, scales, d_host, out.float().cpu().numpy(), step, f"layer ranges fp8={fp8}")
    path.status()
    lay = path.cache.layout
    appended = path.cache.arena[lay.appended_off: lay.appended_off + 4 * cfg.L].view(torch.int32).cpu()
    assert appended.tolist() == [T] * cfg.L, "every layer counted its appends on the device"


@pytest.mark.parametrize("fp8", [False, True], ids=["bf16-cache", "fp8-cache"])
def test_growth_across_a_1024_slot_unit_with_seven_heads_per_kv_head(fp8):
    """The unit size the library picks when a KV head serves more than four query heads (1024 slots), on the
    matrix-core logits path (g = 7) and on the FP8 cache: rows of 1022 and 2046 kept slots grow across the unit
    boundary during 6 steps; launches over all layers and per layer (512-slot units there), every step against the
    oracle."""
    V = _V()
    cfg = _small_cfg(cid=90, m=3300, n_visual=3200, L=2, B=2, Hq=14, Hkv=2)
    kk = np.array([[1022, 2046], [33, 1022]])
    T = 6
    for per_layer in (False, True):
        opts = dict(unit_slots=1024, layer_unit_slots=512, kv_fp8=int(fp8))
        path, dev, caches, scales = _direct_cache(V, cfg, kk, T, opts)
        assert path.cache.layout.unit_slots == 1024 and path.cache.layout.layer_unit_slots == 512
        if fp8:                                                  # the oracle attends over what the FP8 cache holds
            for key, (kc, vc) in caches.items():
                caches[key] = ([O.dequantize_e4m3_rows(*O.quantize_e4m3_rows(x)) for x in kc], [O.dequantize_e4m3_rows(*O.quantize_e4m3_rows(x)) for x in vc])
        out = torch.empty((cfg.L, cfg.B, cfg.Hq, cfg.d), dtype=torch.bfloat16, device="cuda")
        for step in range(T):
            d_host = W.decode_step_inputs(cfg, step)
            dd = {n: torch.from_numpy(x).to(torch.bfloat16).cuda() for n, x in d_host.items()}
            if per_layer:
                for l in range(cfg.L):
                    path.decode(l, l + 1, dd["q"][l], dd["k_new"][l], dd["v_new"][l], dev["sm_scale"], out[l])
            else:
                path.decode(0, cfg.L, dd["q"], dd["k_new"], dd["v_new"], dev["sm_scale"], out)
            torch.cuda.synchronize()
            if fp8:
                d_host = dict(d_host, k_new=O.dequantize_e4m3_rows(*O.quantize_e4m3_rows(d_host["k_new"])),
                              v_new=O.dequantize_e4m3_rows(*O.quantize_e4m3_rows(d_host["v_new"])))
            _oracle_step(cfg, caches, scales, d_host, out.float().cpu().numpy(), step, f"unit=1024 g=7 fp8={fp8} per_layer={per_layer}")
        path.status()


@pytest.mark.parametrize("per_layer", [False, True], ids=["all-layers", "per-layer"])
@pytest.mark.parametrize("fp8", [False, True], ids=["bf16-cache", "fp8-cache"])
def test_one_decode_step_replays_from_a_hip_graph(per_layer, fp8):
    """The append count lives on the device: a HIP graph that holds ONE decode step (one call over all layers, or
    one call per layer) is replayed T times, with the new q / k_new / v_new written into the same buffers before
    each replay and eager work in between, and matches the oracle at every step.  One replay more than slots
    were reserved attends without appending and raises the sticky capacity status."""
    V = _V()
    cfg = _small_cfg(cid=89, m=1400, n_visual=1300, L=3, B=2, Hq=8, Hkv=2)
    kk = np.array([[254, 600, 30], [127, 1, 511]])           # rows that cross 128- and 256-slot boundaries while replaying
    T = 7
    path, dev, caches, scales = _direct_cache(V, cfg, kk, T, dict(kv_fp8=int(fp8)))
    if fp8:
        for key, (kc, vc) in caches.items():
            caches[key] = ([O.dequantize_e4m3_rows(*O.quantize_e4m3_rows(x)) for x in kc],
                           [O.dequantize_e4m3_rows(*O.quantize_e4m3_rows(x)) for x in vc])
    bf = torch.bfloat16
    q = torch.zeros((cfg.L, cfg.B, cfg.Hq, cfg.d), dtype=bf, device="cuda")
    kn = torch.zeros((cfg.L, cfg.B, cfg.Hkv, cfg.d), dtype=bf, device="cuda")
    vn = torch.zeros_like(kn)
    out = torch.zeros_like(q)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        if per_layer:
            for l in range(cfg.L):
                path.decode(l, l + 1, q[l], kn[l], vn[l], dev["sm_scale"], out[l])
        else:
            path.decode(0, cfg.L, q, kn, vn, dev["sm_scale"], out)
    lay = path.cache.layout
    count = path.cache.arena[lay.appended_off: lay.appended_off + 4 * cfg.L].view(torch.int32)
    assert count.tolist() == [0] * cfg.L, "capturing a step must not run it"
    for step in range(T):
        d_host = W.decode_step_inputs(cfg, step)
        q.copy_(torch.from_numpy(d_host["q"]).to(bf)); kn.copy_(torch.from_numpy(d_host["k_new"]).to(bf))
        vn.copy_(torch.from_numpy(d_host["v_new"]).to(bf))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert count.tolist() == [step + 1] * cfg.L
        if fp8:
            d_host = dict(d_host, k_new=O.dequantize_e4m3_rows(*O.quantize_e4m3_rows(d_host["k_new"])),
                          v_new=O.dequantize_e4m3_rows(*O.quantize_e4m3_rows(d_host["v_new"])))
        _oracle_step(cfg, caches, scales, d_host, out.float().cpu().numpy(), step, f"replay per_layer={per_layer}")
    path.status()
    # one step too many: nothing is appended, nothing is counted, the result is the attention over the full cache
    before = out.clone()
    q.copy_(torch.from_numpy(W.decode_step_inputs(cfg, T - 1)["q"]).to(bf))
    graph.replay()
    torch.cuda.synchronize()
    assert count.tolist() == [T] * cfg.L
    with pytest.raises(V.VlcError) as e:
        path.status()
    assert e.value.status == V.VLC_ERR_CAPACITY and "reserved" in str(e.value)
    for (b, l), (kc, vc) in caches.items():
        want = O.decode_attn(W.decode_step_inputs(cfg, T - 1)["q"][l, b], kc, vc, scales[l])
        from gpu_util import assert_close, out_tol
        assert_close(out[l, b].float().cpu().numpy(), want, what=f"over-capacity replay b={b} l={l}", **out_tol(cfg))
    del before


@pytest.mark.parametrize("attr,mutant", [("causal_valid", "_strict_mask"), ("logits", "_logits_interleaved_heads"),
                                         ("score", "_score_mean_over_rows"), ("decode_attn", "_decode_without_scale"),
                                         ("k_min", "_k_min_floor")])
def test_the_parity_harness_notices_a_wrong_oracle(monkeypatch, attr, mutant):
    """The comparison of the whole path is itself checked: with one mistake planted in the oracle (on the CPU) the
    same harness that passes above must report a difference."""
    import test_oracle_mutants as Mu
    from gpu_util import run_and_check
    from oracle import vlcache_oracle as O
    cfg = _small_cfg(cid=87, L=3, alphas=((1, 100),))       # m = 777 and alpha = 1 %: the lower clip (8 tokens) binds
    run_and_check(cfg, (1, 100), 2)
    monkeypatch.setattr(O, attr, getattr(Mu, mutant))
    with pytest.raises((AssertionError, ValueError)):
        run_and_check(cfg, (1, 100), 2)
