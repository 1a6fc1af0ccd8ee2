"""The entry point that allocates nothing (estimator_run_static_dev: fixed scratch inside the library)
against estimator_run_dev, through the C ABI: two calls in a row on one handle, the second with a
smaller input, every result bit for bit; then an input the fixed scratch cannot hold."""
import numpy as np
import pytest

from paper_1812_01776_amd import estimator as binding
from paper_1812_01776_amd import workloads

pytestmark = pytest.mark.gpu


def _both(est, w, torch, dev):
    cfg = binding.pack_configs(w.cfg_hw, w.cfg_batch, w.cfg_replicas)
    arr_t = torch.from_numpy(w.arrival_us.view(np.int32)).to(dev)
    msk_t = torch.from_numpy(w.visit_mask.view(np.int32)).to(dev)
    cfg_t = torch.from_numpy(cfg.view(np.uint8).reshape(-1)).to(dev)
    C = w.n_configs
    p99 = torch.full((C,), -1, dtype=torch.int32, device=dev)
    miss = torch.full((C,), -1, dtype=torch.int32, device=dev)
    cost = torch.full((C,), -1, dtype=torch.int64, device=dev)
    torch.cuda.synchronize()
    est.run_static_dev(arr_t, msk_t, cfg_t, C, w.slo_us, p99, miss, cost)
    ref = est.run_dev(arr_t, msk_t, cfg_t, C, w.slo_us)
    torch.cuda.synchronize()
    assert torch.equal(p99, ref["p99_us"])
    assert torch.equal(miss, ref["miss_count"])
    assert torch.equal(cost, ref["cost_uusd_hr"])
    return p99.cpu().numpy()


def test_static_scratch_entry_point_matches_run_dev():
    import torch
    dev = torch.device("cuda:0")
    big = workloads.w3().subset(cfg_index=np.arange(0, 8192, 16), n_queries=20000)   # a join, 512 candidates
    small = workloads.w3().subset(cfg_index=np.arange(5, 8192, 128), n_queries=3000)  # smaller, other candidates
    est = binding.Estimator(big.parents, big.lat_us, big.cost_uusd_hr)
    a = _both(est, big, torch, dev)
    b = _both(est, small, torch, dev)
    assert a.shape == (512,) and b.shape == (64,) and (a > 0).all() and (b > 0).all()
    # degenerate sizes: no candidates, no queries
    cfg = binding.pack_configs(small.cfg_hw, small.cfg_batch, small.cfg_replicas)
    cfg_t = torch.from_numpy(cfg.view(np.uint8).reshape(-1)).to(dev)
    e_arr = torch.zeros(1, dtype=torch.int32, device=dev)[:0]
    p99 = torch.full((64,), -1, dtype=torch.int32, device=dev); miss = p99.clone(); cost = torch.zeros(64, dtype=torch.int64, device=dev)
    est.run_static_dev(e_arr, e_arr, cfg_t, 64, small.slo_us, p99, miss, cost)
    torch.cuda.synchronize()
    assert (p99 == 0).all() and (miss == 0).all()
    # beyond the fixed scratch: a clear error, outputs untouched
    n_huge = 9_000_000  # the per-query tables alone (8 B keys + accept masks) exceed the 64 MiB
    huge = workloads.Workload("huge", small.parents, small.lat_us, small.cost_uusd_hr, (np.arange(n_huge, dtype=np.uint32) * 100),
                              np.full(n_huge, 31, np.uint32), small.cfg_hw[:2], small.cfg_batch[:2], small.cfg_replicas[:2], small.slo_us)
    est2 = binding.Estimator(huge.parents, huge.lat_us, huge.cost_uusd_hr)
    assert n_huge * 8 > binding.EST_STATIC_SCRATCH_BYTES
    cfg2 = binding.pack_configs(huge.cfg_hw, huge.cfg_batch, huge.cfg_replicas)
    arr_t = torch.from_numpy(huge.arrival_us.view(np.int32)).to(dev)
    msk_t = torch.from_numpy(huge.visit_mask.view(np.int32)).to(dev)
    c2_t = torch.from_numpy(cfg2.view(np.uint8).reshape(-1)).to(dev)
    p2 = torch.full((2,), -7, dtype=torch.int32, device=dev); m2 = p2.clone(); k2 = torch.full((2,), -7, dtype=torch.int64, device=dev)
    with pytest.raises(binding.EstimatorError) as ei:
        est2.run_static_dev(arr_t, msk_t, c2_t, 2, huge.slo_us, p2, m2, k2)
    assert ei.value.code == binding.EST_ENOMEM
    torch.cuda.synchronize()
    assert (p2 == -7).all() and (k2 == -7).all()
    est.close(); est2.close()
