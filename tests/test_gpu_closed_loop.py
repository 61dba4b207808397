"""The scheduler loop closed through the GPU layer: counts accumulated by prism_moe_layer feed
the native placement pipeline, whose masks go back into the layer.  Checks the identities that
tie the two together (Eq. 2 = the layer's remote count) and that the plan raises the local
compute ratio over the uniform split on skewed, server-specific popularity."""
import numpy as np
import pytest

from paper_2508_12851_amd.closed_loop import run_closed_loop, uniform_placement

pytestmark = pytest.mark.gpu


def test_uniform_placement_is_a_partition():
    p = uniform_placement(4, 3, 10)
    assert np.all(p.sum(axis=0) == 1) and p.sum() == 30


@pytest.mark.parametrize("config,kw", [
    ("cfg5_dsv2lite_migration", dict(T=512, H=128, F=128)),
    ("cfg2_mixtral_prefill", dict(T=512, H=128, F=192)),
    ("cfg3_mixtral_decode", dict(T=48, H=256, F=192)),
])
def test_closed_loop(config, kw):
    r = run_closed_loop(config, n_servers=4, n_layers=3, mem_fraction=0.5, **kw)
    print(r)
    assert r["plan_ok"]
    # the layer's remote list is Eq. 2 on that window's counts, for either placement
    assert r["window2_remote_uniform"] == r["window2_eq2_uniform"]
    assert r["window2_remote_planned"] == r["window2_eq2_planned"]
    assert r["window1_remote_uniform"] == r["window1_proxy_cost_uniform"]
    # planning on window 1 pays off on window 2's fresh tokens
    assert r["window1_proxy_cost_planned"] < r["window1_proxy_cost_uniform"]
    assert r["local_ratio_planned"] > r["local_ratio_uniform"]
    assert r["migration_flips"] > 0 and r["migration_seconds"] > 0
