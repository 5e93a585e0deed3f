"""Seeded random cases through the work mappings of the hop (implicit lists, per-XCD lists,
the LDS pass on row clusters and on hubs) against the oracle: graph kind and size, column
count (around every vector, strip, group and pass width), storage type, operator, hop
count, segment length, read order, plane layout and padded leading dimensions are drawn
together, so that combinations no hand-written case lists still get run."""
import numpy as np
import pytest

import gp_synth
import paper_2207_12000_amd as gp
from test_gpu_parity import community_workload, parity_case

pytestmark = pytest.mark.gpu

OPTIONS = ("segment_edges", "lds_pass", "hub_pass", "plane_strips", "cache_schedule", "split_records")
D_F32 = [4, 5, 6, 7, 8, 9, 12, 15, 16, 17, 31, 32, 33, 63, 64, 65, 100, 127, 128, 129, 255, 256, 257, 511, 602, 1000, 1024, 1028]
D_BF16 = [4, 6, 8, 10, 12, 16, 20, 36, 64, 100, 128, 132, 256, 260, 1024, 2048, 2052]


@pytest.fixture(scope="module", autouse=True)
def _need_gpu(gpu_or_skip):
    yield


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_random_cases_match_the_oracle(seed):
    rng = np.random.default_rng(seed)
    lds_launches = 0
    try:
        for it in range(24):
            hubs = bool(rng.integers(0, 2))
            dtype = [gp.GP_F32, gp.GP_BF16][int(rng.integers(0, 2))]
            d = int(rng.choice(D_F32 if dtype == gp.GP_F32 else D_BF16))
            agg = int(rng.choice([gp.GP_AGG_SUM, gp.GP_AGG_MEAN, gp.GP_AGG_SYM]))
            K = int(rng.integers(1, 4))
            shrink = 4 if d >= 500 else 1
            if hubs:
                w = gp_synth.make_workload(int(rng.choice([2, 3])), scale=float(rng.choice([0.02, 0.05, 0.1])) / shrink, d=d)
            else:
                n_comm, comm = int(rng.integers(2, 7)), max(64, int(rng.choice([300, 1000, 3000, 6000])) // shrink)
                w = community_workload(n_comm, comm, int(n_comm * comm * rng.integers(3, 30)), d, 1000 * seed + it)
            chosen = {"segment_edges": int(rng.choice([0, 0, 8, 16, 64])), "lds_pass": int(rng.choice([0, 1, 3])),
                      "hub_pass": 1 if hubs else 0, "plane_strips": int(rng.choice([0, 1, 2, 4, 8])),
                      "cache_schedule": 0 if hubs else int(rng.choice([0, 1])), "split_records": 0 if hubs else int(rng.choice([0, 1]))}
            ld_pad = int(rng.choice([0, 0, 4, 8]))
            for k, v in chosen.items():
                gp.gp_set_option(k, v)
            gp.gp_profile_enable(True)
            try:
                parity_case(w, K=K, dtype=dtype, agg=agg, ld_pad=ld_pad, budget=max(20_000, w.m // 3))
            except AssertionError as e:
                raise AssertionError(f"case {it}: {'hubs' if hubs else 'clusters'} n {w.n} m {w.m} d {d} dtype {dtype} agg {agg} "
                                     f"K {K} ld_pad {ld_pad} {chosen}: {e}") from e
            finally:
                lds_launches += gp.gp_profile_read("gp_hop_cluster_lds")[0]
                gp.gp_profile_enable(False)
    finally:
        for k in OPTIONS:
            gp.gp_set_option(k, 0)
    assert lds_launches > 0, "none of the cases took the LDS pass"
