"""Window attention with row statistics (vlc_window_attn) and the column sweep from given statistics
(vlc_score_from_stats) against the oracle: outputs, row max / sum, and the scores and counts that the
second call derives from them.  Shapes cover 4- and 8-wave blocks, windows that need several launches,
key ranges with one and with several splits, prompts shorter than a chunk, and ragged batches whose
padding is NaN."""
import numpy as np
import pytest
import torch

import workloads as W
from oracle import vlcache_oracle as O

pytestmark = pytest.mark.gpu

from gpu_util import SCORE_TOL, assert_close, check_nnz, torch_dtype

OUT_TOL = dict(atol=2e-2, rtol=1e-2)      # bf16 storage, fp32 accumulation, bf16 probabilities in the P.V product


def _cfg(cid, B, L, Hq, Hkv, m, tau, dtype="bf16", d=128):
    lead = max(0, min(8, m - tau - 1))
    nvis = max(0, m - tau - lead - 4)
    return W.custom_config(cid=cid, name=f"winattn{cid}", dtype=dtype, d=d, Hq=Hq, Hkv=Hkv, L=L, B=B, m=m, tau=tau,
                           lead_text=lead, n_visual=nvis, sinks=min(3, nvis), alphas=((1, 5),))


def _run(V, shape, q_win, k, v, sm, p=0.01):
    B, L, Hq, Hkv, tau, m, d = shape.B, shape.L, shape.Hq, shape.Hkv, shape.tau, shape.m, shape.d
    ws = torch.empty(V.vlc_window_attn_workspace_bytes(shape), dtype=torch.uint8, device="cuda")
    out = torch.full((B, L, Hq, tau, d), 7.0, dtype=torch.bfloat16, device="cuda")
    row_max = torch.full((B, L, Hq, tau), 123.0, dtype=torch.float32, device="cuda")
    row_sum = torch.full((B, L, Hq, tau), 123.0, dtype=torch.float32, device="cuda")
    V.vlc_window_attn(shape, q_win, k, v, sm, out, row_max, row_sum, ws)
    scores = torch.full((B, L, Hkv, m), float("nan"), dtype=torch.float32, device="cuda")
    nnz = torch.full((B, L, Hq), 99, dtype=torch.int64, device="cuda")
    V.vlc_score_from_stats(shape, q_win, k, sm, p, row_max, row_sum, scores, nnz)
    torch.cuda.synchronize()
    return out, row_max, row_sum, scores, nnz


@pytest.mark.parametrize("cid,B,L,Hq,Hkv,m,tau", [
    (400, 1, 2, 4, 2, 300, 32),       # 4-wave blocks, three key splits merged
    (401, 2, 1, 8, 2, 1000, 40),      # window padded to 64 rows per head, 8-wave blocks
    (402, 1, 2, 7, 1, 700, 64),       # g = 7: 14 row blocks, two launches over K and V
    (403, 1, 1, 2, 2, 90, 90),        # window = whole prompt, shorter than one chunk
    (404, 1, 1, 4, 4, 129, 1),        # one window row, a chunk with one key
    (405, 2, 32, 8, 8, 200, 16),      # 512 KV groups: a single split, written without a merge
    (406, 2, 32, 16, 8, 301, 160),    # single split and 10 row blocks: two launches, each writing its rows directly
])
def test_window_attn_and_scores_from_its_statistics_match_the_oracle(cid, B, L, Hq, Hkv, m, tau):
    import paper_2410_23317_amd as V
    cfg = _cfg(cid, B, L, Hq, Hkv, m, tau)
    dt = torch_dtype(cfg)
    q_win = torch.empty((B, L, Hq, tau, 128), dtype=dt, device="cuda")
    k = torch.empty((B, L, Hkv, m, 128), dtype=dt, device="cuda")
    v = torch.empty_like(k)
    host = {}
    for b in range(B):
        for l in range(L):
            t = W.layer_inputs(cfg, b, l)
            host[(b, l)] = t
            q_win[b, l].copy_(torch.from_numpy(t["q_win"]).to(dt))
            k[b, l].copy_(torch.from_numpy(t["k"]).to(dt))
            v[b, l].copy_(torch.from_numpy(t["v"]).to(dt))
    scales = W.sm_scale(cfg)
    sm = torch.from_numpy(scales).cuda()
    shape = V.make_shape(B, L, Hq, Hkv, 128, m, tau, "bf16")
    out, row_max, row_sum, scores, nnz = _run(V, shape, q_win, k, v, sm)
    # the scoring call's own statistics and scores, for the same inputs
    ws2 = torch.empty(V.vlc_workspace_bytes(shape), dtype=torch.uint8, device="cuda")
    s2, M2, Z2 = torch.empty_like(scores), torch.empty_like(row_max), torch.empty_like(row_sum)
    n2 = torch.empty_like(nnz)
    V.vlc_score(shape, q_win, k, sm, 0.01, s2, M2, Z2, n2, ws2)
    torch.cuda.synchronize()
    layers = range(L) if L <= 4 else (0, L // 2, L - 1)
    for b in range(B):
        for l in layers:
            t = host[(b, l)]
            what = f"cid={cid} b={b} l={l}"
            o_ref, M, Z = O.window_attention(t["q_win"], t["k"], t["v"], scales[l])
            assert_close(out[b, l].float().cpu().numpy(), o_ref, what=what + " out", **OUT_TOL)
            assert_close(row_max[b, l].cpu().numpy(), M, atol=2e-5, rtol=2e-6, what=what + " row_max")
            assert_close(row_sum[b, l].cpu().numpy(), Z, atol=0, rtol=5e-5, what=what + " row_sum")
            psi, _ = O.score_from_stats(t["q_win"], t["k"], scales[l], M, Z)
            assert_close(scores[b, l].cpu().numpy(), psi, what=what + " scores", **SCORE_TOL)
            check_nnz(nnz[b, l].cpu().numpy(), t["q_win"], t["k"], scales[l], 0.01, what + " nnz")
    # both routes to the scores agree to fp32 rounding of the statistics
    assert_close(scores.cpu().numpy(), s2.cpu().numpy(), atol=1e-7, rtol=1e-4, what=f"cid={cid} scores vs vlc_score")
    assert_close(row_max.cpu().numpy(), M2.cpu().numpy(), atol=2e-5, rtol=2e-6, what=f"cid={cid} row_max vs vlc_score")
    assert_close(row_sum.cpu().numpy(), Z2.cpu().numpy(), atol=0, rtol=5e-5, what=f"cid={cid} row_sum vs vlc_score")


def test_window_attn_ragged_batch_reads_nothing_beyond_each_request():
    import paper_2410_23317_amd as V
    lens = [(900, 40), (333, 7), (1200, 64), (64, 64)]
    Hq, Hkv, L, d = 8, 2, 2, 128
    cfgs = [_cfg(420 + i, 1, L, Hq, Hkv, m, tau) for i, (m, tau) in enumerate(lens)]
    B, m_max, tau_max = len(lens), 1200, 64
    dt = torch.bfloat16
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
    scales = W.sm_scale(cfgs[0])
    sm = torch.from_numpy(scales).cuda()
    lens_t = torch.tensor(lens, dtype=torch.int32, device="cuda")
    shape = V.make_shape(B, L, Hq, Hkv, d, m_max, tau_max, "bf16", lens=lens_t)
    out, row_max, row_sum, scores, nnz = _run(V, shape, q_win, k, v, sm)
    assert torch.isfinite(scores).all()
    for b, cfg in enumerate(cfgs):
        assert torch.all(out[b, :, :, cfg.tau:] == 7.0), "window rows beyond the request's are left untouched"
        assert torch.all(row_max[b, :, :, cfg.tau:] == 123.0)
        assert torch.all(scores[b, :, :, cfg.m:] == 0)
        for l in range(L):
            t = host[(b, l)]
            what = f"ragged b={b} l={l}"
            o_ref, M, Z = O.window_attention(t["q_win"], t["k"], t["v"], scales[l])
            assert_close(out[b, l, :, : cfg.tau].float().cpu().numpy(), o_ref, what=what + " out", **OUT_TOL)
            assert_close(row_max[b, l, :, : cfg.tau].cpu().numpy(), M, atol=2e-5, rtol=2e-6, what=what + " row_max")
            assert_close(row_sum[b, l, :, : cfg.tau].cpu().numpy(), Z, atol=0, rtol=5e-5, what=what + " row_sum")
            psi, _ = O.score_from_stats(t["q_win"], t["k"], scales[l], M, Z)
            assert_close(scores[b, l, :, : cfg.m].cpu().numpy(), psi, what=what + " scores", **SCORE_TOL)
            check_nnz(nnz[b, l].cpu().numpy(), t["q_win"], t["k"], scales[l], 0.01, what + " nnz")


def test_score_from_stats_takes_the_statistics_as_given_fp32_storage():
    """Plain-ALU sweeps (fp32 storage, d = 64): statistics computed on the host by the oracle, handed in."""
    import paper_2410_23317_amd as V
    cfg = _cfg(430, 1, 2, 4, 2, 300, 20, dtype="f32", d=64)
    q_win = torch.empty((1, 2, 4, 20, 64), dtype=torch.float32, device="cuda")
    k = torch.empty((1, 2, 2, 300, 64), dtype=torch.float32, device="cuda")
    scales = W.sm_scale(cfg)
    Ms, Zs, host = [], [], []
    for l in range(2):
        t = W.layer_inputs(cfg, 0, l)
        host.append(t)
        q_win[0, l].copy_(torch.from_numpy(t["q_win"]))
        k[0, l].copy_(torch.from_numpy(t["k"]))
        _, _, M, Z = O.score(t["q_win"], t["k"], scales[l])
        Ms.append(M); Zs.append(2.0 * Z)                    # a doubled sum must halve the scores
    row_max = torch.from_numpy(np.stack(Ms)[None].astype(np.float32)).cuda()
    row_sum = torch.from_numpy(np.stack(Zs)[None].astype(np.float32)).cuda()
    shape = V.make_shape(1, 2, 4, 2, 64, 300, 20, "f32")
    scores = torch.empty((1, 2, 2, 300), dtype=torch.float32, device="cuda")
    nnz = torch.full((1, 2, 4), 5, dtype=torch.int64, device="cuda")
    V.vlc_score_from_stats(shape, q_win, k, torch.from_numpy(scales).cuda(), 0.01, row_max, row_sum, scores, nnz)
    torch.cuda.synchronize()
    for l in range(2):
        psi, _ = O.score_from_stats(host[l]["q_win"], host[l]["k"], scales[l], Ms[l], Zs[l])
        assert_close(scores[0, l].cpu().numpy(), psi, what=f"l={l} scores", **SCORE_TOL)
        check_nnz(nnz[0, l].cpu().numpy(), host[l]["q_win"], host[l]["k"], scales[l], 0.01, f"l={l} nnz")
    assert V.vlc_window_attn_workspace_bytes(shape) == 0     # this shape takes the generic attention kernel


F32_OUT_TOL = dict(atol=1e-4, rtol=1e-4)     # fp32 storage: fp32 probabilities, fp32 accumulation


@pytest.mark.parametrize("cid,dtype,d,B,L,Hq,Hkv,m,tau,plain", [
    (440, "f32", 64, 2, 2, 4, 2, 300, 20, False),      # the tiny fp32 shape class (config 0)
    (441, "f32", 128, 1, 2, 8, 2, 200, 33, False),     # fp32 storage, d = 128; a row count that is not a multiple of 4
    (442, "bf16", 64, 1, 2, 6, 2, 257, 16, False),     # bf16 storage, d = 64: 2-byte elements per lane
    (443, "bf16", 128, 1, 2, 8, 2, 500, 40, True),     # the matrix-core shape sent to the generic kernel by the flag
    (444, "f32", 64, 1, 1, 2, 2, 64, 64, False),       # window = whole prompt: one tile, row 0 sees one key
    (445, "f32", 64, 1, 1, 1, 1, 65, 1, False),        # one window row, a second tile with one key
])
def test_generic_window_attn_matches_the_oracle_and_feeds_the_column_sweep(cid, dtype, d, B, L, Hq, Hkv, m, tau, plain):
    """The attention kernel for shapes outside the matrix-core path (fp32 storage, d = 64) and its statistics as
    inputs of vlc_score_from_stats: outputs, M, Z, scores and counts against the oracle; for the flagged bf16 shape
    also against the matrix-core kernel on the same inputs."""
    import paper_2410_23317_amd as V
    cfg = _cfg(cid, B, L, Hq, Hkv, m, tau, dtype=dtype, d=d)
    dt = torch_dtype(cfg)
    q_win = torch.empty((B, L, Hq, tau, d), dtype=dt, device="cuda")
    k = torch.empty((B, L, Hkv, m, d), dtype=dt, device="cuda")
    v = torch.empty_like(k)
    host = {}
    for b in range(B):
        for l in range(L):
            t = W.layer_inputs(cfg, b, l)
            host[(b, l)] = t
            q_win[b, l].copy_(torch.from_numpy(t["q_win"]).to(dt))
            k[b, l].copy_(torch.from_numpy(t["k"]).to(dt))
            v[b, l].copy_(torch.from_numpy(t["v"]).to(dt))
    scales = W.sm_scale(cfg)
    sm = torch.from_numpy(scales).cuda()
    shape = V.make_shape(B, L, Hq, Hkv, d, m, tau, dtype, flags=V.VLC_SHAPE_SCORE_PLAIN_ALU if plain else 0)
    assert V.vlc_window_attn_workspace_bytes(shape) == 0
    out = torch.full((B, L, Hq, tau, d), 7.0, dtype=dt, device="cuda")
    row_max = torch.full((B, L, Hq, tau), 123.0, dtype=torch.float32, device="cuda")
    row_sum = torch.full((B, L, Hq, tau), 123.0, dtype=torch.float32, device="cuda")
    V.vlc_window_attn(shape, q_win, k, v, sm, out, row_max, row_sum, None)
    scores = torch.full((B, L, Hkv, m), float("nan"), dtype=torch.float32, device="cuda")
    nnz = torch.full((B, L, Hq), 99, dtype=torch.int64, device="cuda")
    V.vlc_score_from_stats(shape, q_win, k, sm, 0.01, row_max, row_sum, scores, nnz)
    torch.cuda.synchronize()
    tol = OUT_TOL if dtype == "bf16" else F32_OUT_TOL
    for (b, l), t in host.items():
        what = f"cid={cid} b={b} l={l}"
        o_ref, M, Z = O.window_attention(t["q_win"], t["k"], t["v"], scales[l])
        assert_close(out[b, l].float().cpu().numpy(), o_ref, what=what + " out", **tol)
        assert_close(row_max[b, l].cpu().numpy(), M, atol=2e-5, rtol=2e-6, what=what + " row_max")
        assert_close(row_sum[b, l].cpu().numpy(), Z, atol=0, rtol=5e-5, what=what + " row_sum")
        psi, _ = O.score_from_stats(t["q_win"], t["k"], scales[l], M, Z)
        assert_close(scores[b, l].cpu().numpy(), psi, what=what + " scores", **SCORE_TOL)
        check_nnz(nnz[b, l].cpu().numpy(), t["q_win"], t["k"], scales[l], 0.01, what + " nnz")
    if plain:
        mshape = V.make_shape(B, L, Hq, Hkv, d, m, tau, dtype)
        out2, M2, Z2, _, _ = _run(V, mshape, q_win, k, v, sm)
        assert_close(out.float().cpu().numpy(), out2.float().cpu().numpy(), what="generic vs matrix-core out", **OUT_TOL)
        assert_close(row_max.cpu().numpy(), M2.cpu().numpy(), atol=2e-5, rtol=2e-6, what="generic vs matrix-core row_max")
        assert_close(row_sum.cpu().numpy(), Z2.cpu().numpy(), atol=0, rtol=5e-5, what="generic vs matrix-core row_sum")


def test_generic_window_attn_ragged_batch_fp32():
    """Per-request (m_b, tau_b) with NaN in all padding: the generic kernel reads nothing beyond a request's own rows
    and leaves the window rows beyond tau_b untouched."""
    import paper_2410_23317_amd as V
    lens = [(300, 20), (77, 5), (64, 33)]
    Hq, Hkv, L, d = 4, 2, 2, 64
    cfgs = [_cfg(450 + i, 1, L, Hq, Hkv, m, tau, dtype="f32", d=d) for i, (m, tau) in enumerate(lens)]
    B, m_max, tau_max = len(lens), 300, 33
    q_win = torch.full((B, L, Hq, tau_max, d), float("nan"), dtype=torch.float32, device="cuda")
    k = torch.full((B, L, Hkv, m_max, d), float("nan"), dtype=torch.float32, device="cuda")
    v = torch.full((B, L, Hkv, m_max, d), float("nan"), dtype=torch.float32, device="cuda")
    host = {}
    for b, cfg in enumerate(cfgs):
        for l in range(L):
            t = W.layer_inputs(cfg, 0, l)
            host[(b, l)] = t
            q_win[b, l, :, : cfg.tau].copy_(torch.from_numpy(t["q_win"]))
            k[b, l, :, : cfg.m].copy_(torch.from_numpy(t["k"]))
            v[b, l, :, : cfg.m].copy_(torch.from_numpy(t["v"]))
    scales = W.sm_scale(cfgs[0])
    sm = torch.from_numpy(scales).cuda()
    lens_t = torch.tensor(lens, dtype=torch.int32, device="cuda")
    shape = V.make_shape(B, L, Hq, Hkv, d, m_max, tau_max, "f32", lens=lens_t)
    out = torch.full((B, L, Hq, tau_max, d), 7.0, dtype=torch.float32, device="cuda")
    row_max = torch.full((B, L, Hq, tau_max), 123.0, dtype=torch.float32, device="cuda")
    row_sum = torch.full((B, L, Hq, tau_max), 123.0, dtype=torch.float32, device="cuda")
    V.vlc_window_attn(shape, q_win, k, v, sm, out, row_max, row_sum, None)
    torch.cuda.synchronize()
    for b, cfg in enumerate(cfgs):
        assert torch.all(out[b, :, :, cfg.tau:] == 7.0), "window rows beyond the request's are left untouched"
        assert torch.all(row_max[b, :, :, cfg.tau:] == 123.0)
        for l in range(L):
            t = host[(b, l)]
            what = f"ragged fp32 b={b} l={l}"
            o_ref, M, Z = O.window_attention(t["q_win"], t["k"], t["v"], scales[l])
            assert_close(out[b, l, :, : cfg.tau].cpu().numpy(), o_ref, what=what + " out", **F32_OUT_TOL)
            assert_close(row_max[b, l, :, : cfg.tau].cpu().numpy(), M, atol=2e-5, rtol=2e-6, what=what + " row_max")
            assert_close(row_sum[b, l, :, : cfg.tau].cpu().numpy(), Z, atol=0, rtol=5e-5, what=what + " row_sum")


def test_the_output_tolerance_notices_a_wrong_oracle():
    """The comparison itself is checked on one case: an oracle with a planted mistake (values shifted by one
    key, or the window placed one position early) must fall outside the tolerance the tests above use."""
    import paper_2410_23317_amd as V
    cfg = _cfg(440, 1, 1, 4, 2, 500, 32)
    dt = torch.bfloat16
    t = W.layer_inputs(cfg, 0, 0)
    q_win = torch.from_numpy(t["q_win"]).to(dt).cuda()[None, None].contiguous()
    k = torch.from_numpy(t["k"]).to(dt).cuda()[None, None].contiguous()
    v = torch.from_numpy(t["v"]).to(dt).cuda()[None, None].contiguous()
    scales = W.sm_scale(cfg)
    shape = V.make_shape(1, 1, 4, 2, 128, 500, 32, "bf16")
    out, row_max, row_sum, scores, nnz = _run(V, shape, q_win, k, v, torch.from_numpy(scales).cuda())
    got = out[0, 0].float().cpu().numpy()
    good, M, Z = O.window_attention(t["q_win"], t["k"], t["v"], scales[0])
    assert_close(got, good, what="as is", **OUT_TOL)
    shifted, _, _ = O.window_attention(t["q_win"], t["k"], np.roll(t["v"], 1, axis=1), scales[0])
    with pytest.raises(AssertionError):
        assert_close(got, shifted, what="values shifted by one key", **OUT_TOL)
    _, _, Z_e = O.window_attention(t["q_win"], t["k"][:, :-1], t["v"][:, :-1], scales[0])   # every row sees one key fewer
    assert_close(row_sum[0, 0].cpu().numpy(), Z, atol=0, rtol=5e-5, what="as is")
    with pytest.raises(AssertionError):
        assert_close(row_sum[0, 0].cpu().numpy(), Z_e, atol=0, rtol=5e-5, what="window one position early")
