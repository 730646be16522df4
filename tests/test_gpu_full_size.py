"""GPU parity at the full sizes of the benchmark configurations, in the launch
configuration bench.py times.  The oracle evaluates the whole decode step (its cost is
seconds on the host cores); config 4 (prefill) samples query rows."""
import numpy as np
import pytest
import torch

from paper_2407_15176_amd import binding as B
from paper_2407_15176_amd import workloads as wl
from tests import parity as P

pytestmark = pytest.mark.gpu


def _decode_full(cfg):
    w = wl.CONFIGS[cfg]
    t = wl.generate(w, "cuda")
    out, idx = P.run_layer(w, t)
    r = P.check_layer(w, t, out, idx)
    print(f"\n{w.name}: {r}", flush=True)
    idx_h = idx.cpu().numpy()[0]
    needles = set(t["needles"].tolist())
    assert len(needles) == w.n_needles
    for h in range(w.n_kv_heads):
        assert needles <= set(idx_h[h].tolist())          # every planted needle is retrieved
    return r


def test_config2_decode_128k():
    _decode_full(2)


def test_config3_decode_1m():
    _decode_full(3)


@pytest.mark.timeout(600)
def test_config5_decode_4m_three_query_heads_per_group():
    r = _decode_full(5)
    assert r["max_abs_err"] <= 2e-2
