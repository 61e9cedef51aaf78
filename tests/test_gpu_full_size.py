"""The stated workloads at full size, in the launch configuration bench.py times: compression, then all 100
decode steps enqueued by one vlc_decode_attn_steps call over all layers (T_max = 100, so rows grow into the
units reserved for appends while the run lasts).  The oracle is run on sampled (request, layer) pairs, at every
one of the 100 steps; for the 7B shape with one request on every layer.  Properties that hold at any size
(score mass, budget sum, Alg. 1 on the GPU's own counts, ascending unique kept positions) are checked everywhere."""
import gc

import numpy as np
import pytest
import torch

import workloads as W
from oracle import vlcache_oracle as O

pytestmark = pytest.mark.gpu


def _live_units(kk, steps, ub, us):
    """Units of a row that hold slots after `steps` appends (whole units of ub slots, then units of us slots)."""
    nbig = kk // ub
    return nbig + -(-(kk + steps - nbig * ub) // us)


def _run(cid, alphas, reqs, lays, steps=100, window_attn=False):
    from gpu_util import check_window_attn, run_and_check, upload
    cfg = W.CONFIGS[cid]
    dev = upload(cfg)
    try:
        if window_attn:
            check_window_attn(cfg, dev, reqs[:1], lays[-1:])
        for alpha in alphas:
            path = run_and_check(cfg, alpha, steps, layers_to_check=lays, requests_to_check=reqs, dev=dev,
                                 steps_entry_point=True)
            del path
            gc.collect()
            torch.cuda.empty_cache()
    finally:
        del dev
        gc.collect()
        torch.cuda.empty_cache()


def test_cfg1_all_100_decode_steps_on_every_layer():
    """The headline workload exactly as the benchmark runs it; the oracle on every layer and every step.  The run
    must contain what it is meant to cover: rows that grow across a unit boundary (a unit that only held append
    reserve goes live and the row's result turns from a direct store into a merge of partials), and a layer whose
    budget is the lower clip."""
    from gpu_util import run_and_check
    cfg = W.CONFIGS[1]
    path = run_and_check(cfg, (1, 10), cfg.steps, steps_entry_point=True)
    kk = path.k[0].cpu().numpy().astype(np.int64)
    lay = path.cache.layout
    grew = [int(l) for l in range(cfg.L) if _live_units(kk[l], cfg.steps, lay.unit_slots, lay.tail_unit_slots) >
            _live_units(kk[l], 0, lay.unit_slots, lay.tail_unit_slots)]
    single_to_multi = [l for l in grew if _live_units(kk[l], 0, lay.unit_slots, lay.tail_unit_slots) == 1]
    print(f"[cfg1] units {lay.unit_slots}/{lay.tail_unit_slots}: layers whose rows grew into a new unit {grew}, "
          f"from one unit to two {single_to_multi}; clipped layers {np.flatnonzero(kk == O.k_min(cfg.m)).tolist()}", flush=True)
    assert grew and single_to_multi, "no row crossed a unit boundary during the 100 steps"
    assert (kk == O.k_min(cfg.m)).any(), "no layer sits at the lower clip"


def test_cfg1_all_100_decode_steps_one_launch_per_layer():
    """The same 100 steps issued the way a model issues them, one launch per layer and step (the fine work list);
    the oracle on a boundary-crossing layer, a clipped one and the largest one."""
    from gpu_util import run_and_check
    cfg = W.CONFIGS[1]
    run_and_check(cfg, (1, 10), cfg.steps, per_layer_decode=True, layers_to_check=[3, 4, 15, 16])


def test_cfg2_7b_multi_image_batch():
    _run(2, [(1, 10)], reqs=[0, 3], lays=[0, 17], window_attn=True)


def test_cfg3_34b_class_shape():
    _run(3, [(1, 10)], reqs=[1], lays=[2, 59], window_attn=True)


def test_cfg4_long_context_budget_sweep():
    _run(4, [(1, 100), (1, 20), (1, 10), (1, 5)], reqs=[0], lays=[5])
