"""vlc_score_static, the entry point that allocates nothing (its partial row statistics live in an array built
into the library): called through the C-ABI twice in a row, the second time on a smaller input, and compared
with vlc_score element by element.  Both run the same kernels on the same inputs, so the results must be
bit-identical; the oracle is applied to one layer as well, to the scoring tolerances."""
import ctypes as C

import numpy as np
import pytest
import torch

import workloads as W
from oracle import vlcache_oracle as O

pytestmark = pytest.mark.gpu


def _run_both(V, cfg):
    from gpu_util import make_shape, upload
    dev = upload(cfg, want_v=False)
    s = make_shape(cfg)
    f32 = torch.float32
    out = {}
    for which in ("workspace", "static"):
        scores = torch.full((cfg.B, cfg.L, cfg.Hkv, cfg.m), -1.0, dtype=f32, device="cuda")
        row_max = torch.full((cfg.B, cfg.L, cfg.Hq, cfg.tau), -1.0, dtype=f32, device="cuda")
        row_sum = torch.full_like(row_max, -1.0)
        nnz = torch.full((cfg.B, cfg.L, cfg.Hq), -1, dtype=torch.int64, device="cuda")
        stream = torch.cuda.current_stream().cuda_stream
        if which == "workspace":
            ws = torch.empty(V.vlc_workspace_bytes(s), dtype=torch.uint8, device="cuda")
            st = V.lib.vlc_score(C.byref(s), dev["q_win"].data_ptr(), dev["k"].data_ptr(), dev["sm_scale"].data_ptr(),
                                 0.01, scores.data_ptr(), row_max.data_ptr(), row_sum.data_ptr(), nnz.data_ptr(),
                                 ws.data_ptr(), ws.numel(), stream)
        else:
            st = V.lib.vlc_score_static(C.byref(s), dev["q_win"].data_ptr(), dev["k"].data_ptr(), dev["sm_scale"].data_ptr(),
                                        0.01, scores.data_ptr(), row_max.data_ptr(), row_sum.data_ptr(), nnz.data_ptr(),
                                        stream)
        assert st == V.VLC_OK, V.vlc_last_error_string()
        torch.cuda.synchronize()
        out[which] = (scores, row_max, row_sum, nnz)
    return out


def test_static_scratch_entry_point_matches_vlc_score_on_two_calls_in_a_row():
    import paper_2410_23317_amd as V
    from gpu_util import SCORE_TOL, assert_close, check_nnz
    assert V.vlc_score_static_max_workspace() == 16 << 20
    # first a batch whose partial statistics span several key splits and row blocks, then a smaller one
    # (fewer groups, shorter rows, fp32 storage: the other pair of kernels) that reuses the same array
    big = W.custom_config(cid=300, name="static-big", dtype="bf16", d=128, Hq=8, Hkv=2, m=1500, tau=40, lead_text=20,
                          n_visual=1400, L=3, B=2, sinks=6, alphas=((1, 5),))
    small = W.custom_config(cid=301, name="static-small", dtype="f32", d=64, Hq=4, Hkv=2, m=333, tau=7, lead_text=5,
                            n_visual=300, L=2, B=1, sinks=3, alphas=((1, 5),))
    for cfg in (big, small):
        print(f"[case] vlc_score_static cfg={cfg.name} m={cfg.m} tau={cfg.tau} dtype={cfg.dtype}", flush=True)
        res = _run_both(V, cfg)
        for a, b, name in zip(res["workspace"], res["static"], ("scores", "row_max", "row_sum", "nnz")):
            assert torch.equal(a, b), f"{cfg.name}: {name} differs between vlc_score and vlc_score_static"
        scores, row_max, row_sum, nnz = (t.cpu().numpy() for t in res["static"])
        b, l = cfg.B - 1, cfg.L - 1
        t = W.layer_inputs(cfg, b, l, want_v=False)
        scale = W.sm_scale(cfg)[l]
        psi, _, M, Z = O.score(t["q_win"], t["k"], scale)
        assert_close(scores[b, l], psi, what=f"{cfg.name} scores", **SCORE_TOL)
        assert_close(row_max[b, l], M, atol=2e-5, rtol=2e-6, what=f"{cfg.name} row_max")
        assert_close(row_sum[b, l], Z, atol=0, rtol=5e-5, what=f"{cfg.name} row_sum")
        check_nnz(nnz[b, l], t["q_win"], t["k"], scale, 0.01, f"{cfg.name} nnz")


def test_static_scratch_entry_point_rejects_shapes_beyond_its_array():
    import paper_2410_23317_amd as V
    # 4096 window rows per head: the partial statistics alone exceed 16 MiB; rejected on the host, nothing is enqueued
    s = V.make_shape(4, 64, 64, 8, 128, 16384, 4096, "bf16")
    assert V.vlc_workspace_bytes(s) > (16 << 20)
    st = V.lib.vlc_score_static(C.byref(s), 1, 1, None, 0.01, 1, 1, 1, None, None)
    assert st == V.VLC_ERR_CAPACITY and "built-in scratch" in V.vlc_last_error_string()
