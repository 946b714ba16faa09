"""The recall/speedup sweep runs on the HIP path only; these checks pin what must hold by
construction: with every word in the top-frequent list the LSH step IS the full-vocabulary step
(recall 1), and a hit threshold above the number of bands leaves exactly V_T."""
import dataclasses

import numpy as np
import pytest

import workloads

pytestmark = pytest.mark.gpu


def test_sweep_limits_on_the_tiny_shape():
    from paper_1806_00588_amd import sweep
    cfg = workloads.CONFIGS["tiny"]
    sw = sweep.Sweeper(cfg)
    everything = sw.measure(B=4, T=cfg.V, t=1, steps=5)
    assert everything["recall_at_B"] == 1.0 and everything["top1"] == 1.0
    assert everything["mean_candidates"] == cfg.V
    top_only = sw.measure(B=4, T=50, t=cfg.W + 1, steps=5)
    assert top_only["mean_candidates"] == 50.0
    lsh = sw.measure(B=4, T=50, t=1, steps=5, S=2)
    assert 50 <= lsh["mean_candidates"] <= cfg.V and 0.0 <= lsh["recall_at_B"] <= 1.0
    assert lsh["recall_at_B"] >= top_only["recall_at_B"]            # V_T is a subset of V_LSH
    assert lsh["lsh_us"] > 0 and lsh["full_us"] > 0
    assert sweep.default_settings(dataclasses.replace(cfg, W=32))[4][2] == 2   # t sweep needs bands
