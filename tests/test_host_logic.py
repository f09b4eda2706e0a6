"""Host-side pieces that need no GPU: where bench.py's roofline.traffic comes from, the workload table against the
configurations the target names, tenants that share a weight set."""
import os
import re
import sys

import numpy as np

import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_roofline_traffic_is_read_from_the_committed_counter_summary():
    sys.path.insert(0, ROOT)
    import bench
    traffic, src = bench.measured_traffic("bert_ffn")
    assert src == os.path.join("profiles", "gemm_bf16_p256_bert_ffn.md")
    text = open(os.path.join(ROOT, src)).read()
    # the figure is the mean of the two launches' rows of that file's traffic table (total MB column)
    rows = re.findall(r"^\| FFN[12] \|.*?\| (\d+) \| \d+ \(", text, flags=re.M)
    assert len(rows) == 2
    assert abs(traffic / 1e6 - (int(rows[0]) + int(rows[1])) / 2) < 1.0
    assert bench.measured_traffic("no_such_workload") == (None, None)


def test_workload_table_matches_the_named_configurations():
    w = synth.WORKLOADS
    t = w["tiny_fp32"]
    assert (t.dtype, t.n_tenants, t.d_model, t.d_ff, t.n_requests, t.seq_min, t.seq_max) == ("f32", 4, 64, 256, 8, 16, 16)
    b = w["bert_ffn"]
    assert (b.dtype, b.n_tenants, b.d_model, b.d_ff, b.n_requests, b.seq_min, b.seq_max, b.popularity) == \
           ("bf16", 64, 768, 3072, 256, 128, 128, "uniform")
    e = w["hbert_enc2"]
    assert (e.n_tenants, e.n_layers, e.n_heads, e.n_requests, e.seq_max, e.popularity) == (1000, 2, 12, 512, 128, "zipf")
    g = w["hgpt_dec"]
    assert (g.n_tenants, g.d_model, g.d_ff, g.n_heads, g.n_requests, g.seq_min, g.seq_max) == (2000, 1024, 4096, 16, 256, 32, 512)
    k = w["hbert_10k"]
    assert (k.n_tenants, k.hbm_slots, k.host_tier, k.n_requests, k.seq_min, k.seq_max) == (10000, 2000, True, 1024, 16, 256)


def test_tenants_that_share_a_weight_set_get_the_same_tensors_and_others_do_not():
    wl = synth.WORKLOADS["hbert_10k"].scaled(n_images=500) if hasattr(synth.WORKLOADS["hbert_10k"], "scaled") else None
    assert wl is not None
    assert synth.image_of(wl, 1234) == 1234 % 500 and synth.image_of(wl, 77) == 77
    small = wl.scaled(d_model=64, d_ff=128, n_heads=1)
    a = synth.tenant_storage(small, 1234, 0)
    b = synth.tenant_storage(small, 1234 % 500, 0)
    c = synth.tenant_storage(small, 1235, 0)
    assert all(np.array_equal(x, y) for x, y in zip(a, b))
    assert not all(np.array_equal(x, y) for x, y in zip(a, c))
