"""The stated workloads at full size, in the launch configuration bench.py times.  The oracle is
run on sampled (request, layer) pairs; properties that hold at any size (score mass, budget sum,
Alg. 1 on the GPU's own counts, ascending unique kept positions) are checked everywhere."""
import gc

import pytest
import torch

import workloads as W

pytestmark = pytest.mark.gpu


def _run(cid, alphas, reqs, lays, steps=2, window_attn=False):
    from gpu_util import check_window_attn, run_and_check, upload
    cfg = W.CONFIGS[cid]
    dev = upload(cfg)
    try:
        if window_attn:
            check_window_attn(cfg, dev, reqs[:1], lays[-1:])
        for alpha in alphas:
            path = run_and_check(cfg, alpha, steps, layers_to_check=lays, requests_to_check=reqs, dev=dev)
            del path
            gc.collect()
            torch.cuda.empty_cache()
    finally:
        del dev
        gc.collect()
        torch.cuda.empty_cache()


def test_cfg2_7b_multi_image_batch():
    _run(2, [(1, 10)], reqs=[0, 3], lays=[0, 17], window_attn=True)


def test_cfg3_34b_class_shape():
    _run(3, [(1, 10)], reqs=[1], lays=[2, 59], window_attn=True)


def test_cfg4_long_context_budget_sweep():
    _run(4, [(1, 100), (1, 10), (1, 5)], reqs=[0], lays=[5])
