"""hmi_layer_forward_static, the entry point for callers that cannot allocate: its routing arrays live in a
static device array of the library.  Through the C ABI, against hmi_layer_forward on the same pool and inputs
(same kernels: bit-identical rows) and against the oracle, on two calls in a row, the second with a smaller batch."""
import numpy as np
import pytest
import torch

import synth
from tests.oracle_side import compare, oracle_forward

pytestmark = pytest.mark.gpu


def adapter_workload(n_requests, seq_max, seed):
    return synth.Workload(name="adapter_static", block=synth.BLOCK_ADAPTER, dtype="bf16", d_model=768, d_ff=64,
                          n_heads=0, n_layers=1, n_tenants=12, n_requests=n_requests, seq_min=1, seq_max=seq_max,
                          popularity="zipf", zipf_s=1.0, ln_eps=0.0, hbm_slots=12, host_tier=False, seed=seed)


def test_static_routing_arrays_two_calls_second_smaller(hmi):
    from paper_2504_17449_amd import harness
    big, small = adapter_workload(40, 300, 21), adapter_workload(7, 90, 21)
    pool = harness.create_pool(big, max_requests=300, max_tokens=40000)
    try:
        harness.load_tenants(pool, big)
        for wl, batch in ((big, 0), (small, 1)):
            ids, lens, x = harness.batch_to_device(wl, batch)
            print(f"static call: R={len(ids)} N={int(lens.sum())}", flush=True)
            y_static = torch.full_like(x, 3.0)
            y_pool = torch.full_like(x, 5.0)
            assert hmi.hmi_layer_forward_static(pool.h, 0, x.data_ptr(), y_static.data_ptr(), ids, lens) == hmi.HMI_OK, \
                hmi.hmi_last_error(pool.h)
            assert hmi.hmi_layer_forward(pool.h, 0, x.data_ptr(), y_pool.data_ptr(), ids, lens) == hmi.HMI_OK
            torch.cuda.synchronize()
            a, b = y_static.view(torch.int16).cpu().numpy(), y_pool.view(torch.int16).cpu().numpy()
            assert np.array_equal(a, b), int((a != b).sum())
            y_ref = oracle_forward(wl, ids, lens, batch=batch)
            max_abs, rel, ok = compare(harness.device_to_f64(y_static), y_ref, np.arange(len(y_ref)), "bf16")
            print(f"  max_abs={max_abs:.3e} rel_fro={rel:.3e}", flush=True)
            assert ok, (max_abs, rel)
        # limits and errors: nothing is enqueued, y stays as it was
        x = torch.zeros(300, 768, dtype=torch.bfloat16, device="cuda")
        y = torch.full_like(x, 7.0)
        call = lambda ids, lens: hmi.hmi_layer_forward_static(pool.h, 0, x.data_ptr(), y.data_ptr(), ids, lens)
        assert call([], []) == hmi.HMI_OK
        assert call([0] * 257, [1] * 257) == hmi.HMI_ERR_SHAPE          # more requests than the static arrays hold
        assert call([0, 1], [20000, 20000]) == hmi.HMI_ERR_SHAPE        # more tokens than the static arrays hold
        assert call([0, 12], [4, 4]) == hmi.HMI_ERR_TENANT
        assert call([0, 1], [4, 0]) == hmi.HMI_ERR_SHAPE
        assert hmi.hmi_layer_forward_static(pool.h, 1, x.data_ptr(), y.data_ptr(), [0], [4]) == hmi.HMI_ERR_ARG
        assert hmi.hmi_layer_forward_static(pool.h, 0, x.data_ptr(), x.data_ptr(), [0], [4]) == hmi.HMI_ERR_ARG
        torch.cuda.synchronize()
        assert bool((y == 7.0).all())
    finally:
        pool.close()
    # a pool of another kind is refused
    ffn = synth.Workload(name="ffn_static", block=synth.BLOCK_FFN, dtype="bf16", d_model=128, d_ff=256, n_heads=0,
                         n_layers=1, n_tenants=2, n_requests=2, seq_min=4, seq_max=4, popularity="uniform", zipf_s=0.0,
                         ln_eps=1e-5, hbm_slots=2, host_tier=False, seed=1)
    pool = harness.create_pool(ffn, max_requests=2, max_tokens=8)
    try:
        harness.load_tenants(pool, ffn)
        x = torch.zeros(8, 128, dtype=torch.bfloat16, device="cuda")
        y = torch.empty_like(x)
        assert hmi.hmi_layer_forward_static(pool.h, 0, x.data_ptr(), y.data_ptr(), [0, 1], [4, 4]) == hmi.HMI_ERR_ARG
    finally:
        pool.close()
