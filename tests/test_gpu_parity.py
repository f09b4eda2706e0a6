"""GPU parity: the HIP path (through the C ABI) against the fp64 oracle on the same seeded
inputs.  Routing must be bit-exact; floats within max-abs 2e-2 / relative Frobenius 1e-2
(bf16) or 1e-4 (fp32)."""
import numpy as np
import pytest
import torch

import synth
from oracle import hmi_oracle as O
from tests.oracle_side import compare, oracle_forward, rows_of

pytestmark = pytest.mark.gpu


def check_route(pool, ids, lens):
    want = O.route(ids, lens)
    got = pool.route()
    R = len(ids)
    assert got["n_segments"] == len(want["seg_tenant"])
    np.testing.assert_array_equal(got["perm"][:R], want["perm"])
    np.testing.assert_array_equal(got["seg_tenant"], want["seg_tenant"])
    np.testing.assert_array_equal(got["seg_req_off"], want["seg_req_off"])
    np.testing.assert_array_equal(got["seg_tok_off"], want["seg_tok_off"])


def run_case(hmi, wl, sample=None, batch=0, tenants="touched", slack=0):
    """Create the pool, load tenants, run all layers, compare ``sample`` requests (default all).
    slack: the pool is created for that many more requests and 100 x that many more tokens than the batch has."""
    from paper_2504_17449_amd import harness
    ids, lens, x = harness.batch_to_device(wl, batch)
    print(f"case {wl.name} R={len(ids)} N={int(lens.sum())} d={wl.d_model} f={wl.d_ff} "
          f"dtype={wl.dtype} block={wl.block}", flush=True)
    pool = harness.create_pool(wl, max_requests=len(ids) + slack, max_tokens=int(lens.sum()) + 100 * slack)
    try:
        harness.load_tenants(pool, wl, sorted(set(ids.tolist())) if tenants == "touched" else None)
        cur = torch.empty_like(x)
        if wl.n_layers == 1:
            pool.forward(0, x, cur, ids, lens)
        else:
            pool.stack_forward(0, wl.n_layers, x, cur, ids, lens)
        torch.cuda.synchronize()
        check_route(pool, ids, lens)
        y_gpu = harness.device_to_f64(cur)
        if wl.n_layers > 1:
            # the same stack with its result handed out as fp32: rounded once to the storage type it is y, bit for bit
            y32 = torch.empty(x.shape, dtype=torch.float32, device=x.device)
            pool.stack_forward_f32(0, wl.n_layers, x, y32, ids, lens)
            torch.cuda.synchronize()
            assert torch.equal(y32.to(cur.dtype).view(torch.int16 if wl.dtype == "bf16" else torch.int32),
                               cur.view(torch.int16 if wl.dtype == "bf16" else torch.int32))
    finally:
        pool.close()
    reqs = list(range(len(ids))) if sample is None else list(sample)
    y_ref = oracle_forward(wl, ids, lens, reqs, batch)
    max_abs, rel, ok = compare(y_gpu, y_ref, rows_of(lens, reqs), wl.dtype)
    print(f"  max_abs={max_abs:.3e} rel_fro={rel:.3e} max|y_ref|={np.nanmax(np.abs(y_ref)):.2f}", flush=True)
    assert ok, (max_abs, rel)
    return y_gpu


def small(block, dtype, **kw):
    base = dict(name=f"small_{block}_{dtype}", block=block, dtype=dtype, d_model=128, d_ff=256,
                n_heads=2, n_layers=1, n_tenants=6, n_requests=20, seq_min=1, seq_max=300,
                popularity="zipf", zipf_s=1.0, ln_eps=1e-5, hbm_slots=6, host_tier=False, seed=3)
    base.update(kw)
    if block in (synth.BLOCK_FFN, synth.BLOCK_ADAPTER):
        base["n_heads"] = 0
    if block in (synth.BLOCK_ENC_ADAPTER, synth.BLOCK_DEC_ADAPTER):
        base.setdefault("adapter_rank", 64 if dtype == "bf16" else 16)
    return synth.Workload(**base)


def test_tiny_fp32_ffn_full_config(hmi):
    run_case(hmi, synth.WORKLOADS["tiny_fp32"])


@pytest.mark.parametrize("block", [synth.BLOCK_FFN, synth.BLOCK_ENC_POSTLN, synth.BLOCK_DEC_PRELN,
                                   synth.BLOCK_ADAPTER, synth.BLOCK_ENC_ADAPTER, synth.BLOCK_DEC_ADAPTER])
def test_small_fp32_blocks_ragged(hmi, block):
    run_case(hmi, small(block, "f32", d_model=64, d_ff=128, n_heads=4, seq_max=90))


@pytest.mark.parametrize("block,kw", [
    (synth.BLOCK_FFN, dict(d_model=80, d_ff=48)),
    (synth.BLOCK_FFN, dict(d_model=48, d_ff=144)),
    (synth.BLOCK_ENC_POSTLN, dict(d_model=80, d_ff=96, n_heads=5)),
    (synth.BLOCK_DEC_PRELN, dict(d_model=144, d_ff=80, n_heads=3))])
def test_fp32_widths_that_are_not_multiples_of_64(hmi, block, kw):
    """fp32 pools take any width that is a multiple of 16: LayerNorm, GEMM and attention must cover the
    columns beyond the last full group of 64 (d = 80, 144) and widths below 64 (d = 48)."""
    run_case(hmi, small(block, "f32", seq_max=60, **kw))


@pytest.mark.parametrize("block", [synth.BLOCK_FFN, synth.BLOCK_ENC_POSTLN, synth.BLOCK_DEC_PRELN,
                                   synth.BLOCK_ADAPTER, synth.BLOCK_ENC_ADAPTER, synth.BLOCK_DEC_ADAPTER])
def test_small_bf16_blocks_ragged(hmi, block):
    # seq up to 300: m-tiles of 256 rows with ragged tails, several key blocks, q blocks
    run_case(hmi, small(block, "bf16"))


@pytest.mark.parametrize("block", [synth.BLOCK_FFN, synth.BLOCK_ENC_POSTLN, synth.BLOCK_DEC_PRELN,
                                   synth.BLOCK_ADAPTER, synth.BLOCK_ENC_ADAPTER, synth.BLOCK_DEC_ADAPTER])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_layer_stack_in_one_call(hmi, block, dtype):
    kw = dict(d_model=64, d_ff=128, n_heads=4) if dtype == "f32" else {}
    run_case(hmi, small(block, dtype, n_layers=3, seq_max=140, **kw))


@pytest.mark.parametrize("block", [synth.BLOCK_FFN, synth.BLOCK_ENC_POSTLN, synth.BLOCK_DEC_PRELN,
                                   synth.BLOCK_ENC_ADAPTER, synth.BLOCK_DEC_ADAPTER])
def test_wide_bf16_blocks_ragged_every_row(hmi, block):
    """Widths that are multiples of 256 with k >= 192 take the persistent 256 x 256 GEMM: ragged
    segments of 1..300 rows (short tiles, clamped rows, several tiles per segment), every output
    row compared.  d = 256 makes k = 256 (4 stages), f = 512 makes k = 512 and two n-tiles."""
    run_case(hmi, small(block, "bf16", d_model=256, d_ff=512, n_heads=4, n_requests=28, n_tenants=7,
                        hbm_slots=7, n_layers=2 if block == synth.BLOCK_FFN else 1))


def test_persistent_gemm_more_tiles_than_workgroups(hmi):
    """Hundreds of one-request tenants: ~1700 tiles for 256 workgroups, so every workgroup claims
    tiles at run time beyond its two fixed ones; k = 192 is the shortest reduction the kernel takes."""
    wl = small(synth.BLOCK_FFN, "bf16", d_model=192, d_ff=1024, n_requests=640, n_tenants=900,
               hbm_slots=900, seq_min=1, seq_max=9, popularity="uniform")
    run_case(hmi, wl)
    # the counters reset themselves: a second forward on a fresh pool object of another shape works as well
    run_case(hmi, small(synth.BLOCK_FFN, "bf16", d_model=256, d_ff=768, n_requests=300, n_tenants=300,
                        hbm_slots=300, seq_min=1, seq_max=5, popularity="uniform"), batch=1)


@pytest.mark.parametrize("seed", [15, 10])
def test_persistent_gemm_long_segments_in_blocks_of_m_tiles(hmi, seed):
    """Two tenants with thousands of rows each.  The persistent GEMM walks a long segment in blocks of
    eight m-tiles of 256 rows; seed 15 gives segments of 8 and 11 m-tiles (exactly one block; one block and a
    short one of three), seed 10 gives 16 and 5 (two full blocks; less than one), each with a ragged last
    tile.  Every row compared."""
    wl = small(synth.BLOCK_FFN, "bf16", d_model=256, d_ff=768, n_requests=24, n_tenants=2, hbm_slots=2,
               seq_min=100, seq_max=300, popularity="uniform", seed=seed)
    ids, lens = synth.batch_ids_lens(wl, 0)
    assert sorted(-(-int(lens[ids == t].sum()) // 256) for t in range(2)) == {15: [8, 11], 10: [5, 16]}[seed]
    run_case(hmi, wl)


def test_decoder_layer_at_the_maximum_width(hmi):
    """d_model = 2048 (the widest the library takes), f = 6144, 32 heads, prompts of up to 1500 tokens, pre-LN
    decoder: outputs are not normalised (|y| up to 7.6), so storing y as bf16 costs up to 0.0156 by itself.  The
    fp32 result is held to the flat bars; the bf16 result is that one rounded once, bit for bit, and every element
    is within the flat bar plus half a bf16 unit of its value."""
    from paper_2504_17449_amd import harness
    from tests.oracle_side import within_storage_rounding
    wl = small(synth.BLOCK_DEC_PRELN, "bf16", d_model=2048, d_ff=6144, n_heads=32, n_tenants=3, hbm_slots=3,
               n_requests=6, seq_min=1, seq_max=1500)
    ids, lens, x = harness.batch_to_device(wl, 0)
    pool = harness.create_pool(wl, max_requests=len(ids), max_tokens=int(lens.sum()))
    try:
        harness.load_tenants(pool, wl, sorted(set(ids.tolist())))
        y = torch.empty_like(x)
        y32 = torch.empty(x.shape, dtype=torch.float32, device=x.device)
        pool.forward(0, x, y, ids, lens)
        pool.stack_forward_f32(0, 1, x, y32, ids, lens)
        torch.cuda.synchronize()
        check_route(pool, ids, lens)
        assert torch.equal(y32.to(torch.bfloat16).view(torch.int16), y.view(torch.int16))
        yb, yf = harness.device_to_f64(y), y32.double().cpu().numpy()
    finally:
        pool.close()
    ref = oracle_forward(wl, ids, lens, list(range(len(ids))), 0)
    rows = np.arange(len(ref))
    max_abs, rel, ok = compare(yf, ref, rows, "bf16")
    print(f"  fp32 result: max_abs={max_abs:.3e} rel_fro={rel:.3e} max|y_ref|={np.abs(ref).max():.2f}", flush=True)
    assert ok, (max_abs, rel)
    assert within_storage_rounding(yb, ref, rows)
    assert compare(yb, ref, rows, "bf16")[1] <= 1e-2


def test_request_limit_of_one_or_two_tokens_each(hmi):
    """2048 requests (the most a call takes) of one or two tokens of 500 tenants through a decoder layer:
    attention over one or two keys, segments of a few rows, every row compared."""
    run_case(hmi, small(synth.BLOCK_DEC_PRELN, "bf16", d_model=128, d_ff=256, n_heads=2, n_tenants=500, hbm_slots=500,
                        n_requests=2048, seq_min=1, seq_max=2))


def test_second_layer_alone(hmi):
    """forward(layer=1) uses layer 1's weights: equals the oracle fed layer-1 weights only."""
    from paper_2504_17449_amd import harness
    from tests.oracle_side import weights_of
    wl = small(synth.BLOCK_ENC_POSTLN, "bf16", n_layers=2, seq_max=90)
    ids, lens, x = harness.batch_to_device(wl)
    pool = harness.create_pool(wl, max_tokens=int(lens.sum()))
    try:
        harness.load_tenants(pool, wl)
        y = torch.empty_like(x)
        pool.forward(1, x, y, ids, lens)
        torch.cuda.synchronize()
        y_gpu = harness.device_to_f64(y)
    finally:
        pool.close()
    X = np.concatenate([synth.hidden_states(wl, r, int(lens[r])) for r in range(len(ids))]).astype(np.float64)
    y_ref = O.layer_forward(wl.block, X, ids, lens, weights_of(wl, 1), wl.n_heads, wl.ln_eps)
    _, _, ok = compare(y_gpu, y_ref, np.arange(len(X)), wl.dtype)
    assert ok
    y_l0 = O.layer_forward(wl.block, X, ids, lens, weights_of(wl, 0), wl.n_heads, wl.ln_eps)
    assert np.abs(y_l0 - y_ref).max() > 0.05     # the two layers really differ


def test_bf16_adapter_rank_64(hmi):
    run_case(hmi, small(synth.BLOCK_ADAPTER, "bf16", d_model=768, d_ff=64, seq_max=128, seq_min=128))


@pytest.mark.parametrize("block,kw", [
    (synth.BLOCK_ADAPTER, dict(d_model=1024, d_ff=128)),
    (synth.BLOCK_ADAPTER, dict(d_model=768, d_ff=64, n_layers=2)),
    (synth.BLOCK_ENC_ADAPTER, dict(d_model=1024, d_ff=4096, n_heads=16, adapter_rank=128)),
], ids=["adapter_d1024_rank128", "adapter_two_layers", "shared_layer_d1024_rank128"])
def test_adapter_as_two_gemms(hmi, block, kw):
    """Where the one-kernel adapter does not apply (d = 1024: its rows do not fit LDS twice; an adapter-only pool of
    several layers: fp32 between the layers) the adapter runs as two grouped GEMMs; the up-projection has k = rank
    = 64 or 128, below what the persistent kernel takes, so it goes to the general 256 x 256 kernel with direct-to-LDS
    copies.  A few thousand rows (more than the small-batch kernel takes), every row compared."""
    run_case(hmi, small(block, "bf16", n_tenants=12, hbm_slots=12, n_requests=40, seq_min=1, seq_max=300, **kw))


def test_one_kernel_adapter_refuses_the_fp32_result_call(hmi):
    """The one-kernel adapter rounds as it stores: asking it for an fp32 result is an argument error, y untouched."""
    from paper_2504_17449_amd import harness
    wl = small(synth.BLOCK_ADAPTER, "bf16", d_model=256, d_ff=64, n_requests=3, seq_max=20)
    ids, lens, x = harness.batch_to_device(wl)
    pool = harness.create_pool(wl, max_tokens=int(lens.sum()))
    try:
        harness.load_tenants(pool, wl)
        y32 = torch.full(x.shape, 7.0, dtype=torch.float32, device=x.device)
        assert hmi.hmi_stack_forward_f32(pool.h, 0, 1, x.data_ptr(), y32.data_ptr(), ids, lens) == hmi.HMI_ERR_ARG
        assert "fp32" in hmi.hmi_last_error(pool.h)
        torch.cuda.synchronize()
        assert bool((y32 == 7.0).all())
    finally:
        pool.close()


@pytest.mark.parametrize("d_model", [256, 512, 768])
def test_fused_adapter_ragged_large_weights(hmi, d_model):
    """Single-layer bf16 adapter pools with rank 64 run the one-kernel path (rows through LDS,
    matrices repacked at load).  The seeded recipe's weights make the adapter's contribution a
    few percent of |x|, so a misplaced k-chunk or column block would hide under the rounding of
    y; here x is small and the weights large, so that y is mostly the adapter's own output, and
    every row is compared.  Lengths 1..150 over 40 tenants: units of 1..32 rows, requests that
    end inside a unit, segments of several requests, tenants changing inside one workgroup."""
    from paper_2504_17449_amd import harness
    rng = np.random.default_rng(100 + d_model)
    T, R, r = 40, 90, 64
    wl = small(synth.BLOCK_ADAPTER, "bf16", d_model=d_model, d_ff=r, n_tenants=T, hbm_slots=T, n_requests=R)
    ids = rng.integers(0, T, R).astype(np.int32)
    lens = rng.integers(1, 151, R).astype(np.int32)
    N = int(lens.sum())
    rb = lambda a: synth.round_to_storage(a.astype(np.float32), "bf16")
    w = {t: {"w_down": rb(rng.normal(0, 0.2, (r, d_model))), "b_down": rb(rng.normal(0, 0.2, r)),
             "w_up": rb(rng.normal(0, 0.2, (d_model, r))), "b_up": rb(rng.normal(0, 0.2, d_model))}
         for t in sorted(set(ids.tolist()))}
    X = rb(rng.normal(0, 1.0 / 16, (N, d_model)))
    print(f"case fused adapter d={d_model} R={R} N={N}", flush=True)
    pool = harness.create_pool(wl, max_requests=R, max_tokens=N)
    try:
        for t, wt in w.items():
            pool.load_tenant(t, 0, [synth.to_storage_bytes(wt[n], "bf16") for n in ("w_down", "b_down", "w_up", "b_up")])
        x = harness.host_to_device(X, "bf16")
        y = torch.empty_like(x)
        pool.forward(0, x, y, ids, lens)
        torch.cuda.synchronize()
        check_route(pool, ids, lens)
        y_gpu = harness.device_to_f64(y)
        # a second batch on the same pool: other lengths, fewer requests (stale LDS or schedule state would show)
        ids2, lens2 = ids[:17].copy(), rng.integers(1, 40, 17).astype(np.int32)
        N2 = int(lens2.sum())
        y2 = torch.empty_like(x[:N2])
        pool.forward(0, x[:N2].contiguous(), y2, ids2, lens2)
        torch.cuda.synchronize()
        y2_gpu = harness.device_to_f64(y2)
    finally:
        pool.close()
    get = lambda t: {k: v.astype(np.float64) for k, v in w[t].items()}
    y_ref = O.layer_forward(synth.BLOCK_ADAPTER, X.astype(np.float64), ids, lens, get, 0, 0.0)
    max_abs, rel, ok = compare(y_gpu, y_ref, np.arange(N), "bf16")
    print(f"  max_abs={max_abs:.3e} rel_fro={rel:.3e} max|y_ref|={np.abs(y_ref).max():.2f} "
          f"|y-x|/|y|={np.linalg.norm(y_ref - X) / np.linalg.norm(y_ref):.2f}", flush=True)
    assert ok, (max_abs, rel)
    y2_ref = O.layer_forward(synth.BLOCK_ADAPTER, X[:N2].astype(np.float64), ids2, lens2, get, 0, 0.0)
    max_abs, rel, ok = compare(y2_gpu, y2_ref, np.arange(N2), "bf16")
    assert ok, (max_abs, rel)


@pytest.mark.parametrize("block", [synth.BLOCK_ENC_ADAPTER, synth.BLOCK_DEC_ADAPTER])
def test_shared_layer_with_loud_adapters(hmi, block):
    """The paper's task-adapted layer (shared encoder layer, tenant adapter after the attention
    layer) with adapters loud enough to matter: with the seeded recipe's N(0, 0.02) adapter
    weights a wrong or missing adapter would hide inside the tolerance, here the adapter's
    output is larger than the attention output it is added to (LayerNorm gains near 0.6 keep |y|
    below 4, where a bf16 half-ulp is still under the max-abs tolerance).  d = 256 takes the one-kernel
    adapter inside the layer; two layers in one call; every row compared."""
    from paper_2504_17449_amd import harness
    rng = np.random.default_rng(77)
    T, R, d, f, r, h, L = 12, 30, 256, 512, 64, 4, 2
    wl = small(block, "bf16", d_model=d, d_ff=f, n_heads=h, n_layers=L, n_tenants=T,
               hbm_slots=T, n_requests=R, adapter_rank=r, ln_eps=1e-5)
    # pre-LN carries the raw residual stream to the output: smaller x and adapters keep |y| < 4 there
    sx, aw = (1.0, 0.2) if block == synth.BLOCK_ENC_ADAPTER else (0.3, 0.12)
    ids = rng.integers(0, T, R).astype(np.int32)
    lens = rng.integers(1, 151, R).astype(np.int32)
    N = int(lens.sum())
    rb = lambda a: synth.round_to_storage(np.asarray(a, dtype=np.float32), "bf16")
    n = lambda sc, *s: rb(rng.normal(0, sc, s))
    shared = [{"wqkv": n(0.05, 3 * d, d), "bqkv": n(0.05, 3 * d), "wo": n(0.05, d, d), "bo": n(0.05, d),
               "ln1_g": rb(0.6 + rng.normal(0, 0.05, d)), "ln1_b": n(0.1, d), "w1": n(0.05, f, d), "b1": n(0.05, f),
               "w2": n(0.05, d, f), "b2": n(0.05, d), "ln2_g": rb(0.6 + rng.normal(0, 0.05, d)), "ln2_b": n(0.1, d)}
              for _ in range(L)]
    adapters = {(t, l): {"w_down": n(aw, r, d), "b_down": n(aw, r), "w_up": n(aw, d, r), "b_up": n(aw, d)}
                for t in sorted(set(ids.tolist())) for l in range(L)}
    X = rb(rng.normal(0, sx, (N, d)))
    raw = lambda a: synth.to_storage_bytes(a, "bf16")
    pool = harness.create_pool(wl, max_requests=R, max_tokens=N)
    try:
        for l in range(L):
            pool.load_shared(l, [raw(shared[l][k]) for k, _, _ in synth.shared_specs(wl)])
        for (t, l), w in adapters.items():
            pool.load_tenant(t, l, [raw(w[k]) for k in ("w_down", "b_down", "w_up", "b_up")])
        x = harness.host_to_device(X, "bf16")
        y = torch.empty_like(x)
        pool.stack_forward(0, L, x, y, ids, lens)
        torch.cuda.synchronize()
        check_route(pool, ids, lens)
        y_gpu = harness.device_to_f64(y)
    finally:
        pool.close()
    cur = X.astype(np.float64)
    quiet = cur
    for l in range(L):
        full = lambda t, l=l: {**{k: v.astype(np.float64) for k, v in shared[l].items()},
                               **{k: v.astype(np.float64) for k, v in adapters[(t, l)].items()}}
        cur = O.layer_forward(block, cur, ids, lens, full, h, 1e-5)
        mute = lambda t, l=l: {**full(t), "w_up": np.zeros((d, r)), "b_up": np.zeros(d)}
        quiet = O.layer_forward(block, quiet, ids, lens, mute, h, 1e-5)
    max_abs, rel, ok = compare(y_gpu, cur, np.arange(N), "bf16")
    loud = np.linalg.norm(cur - quiet) / np.linalg.norm(cur)
    print(f"  max_abs={max_abs:.3e} rel_fro={rel:.3e} max|y|={np.abs(cur).max():.2f} adapters move y by {loud:.2f}", flush=True)
    assert loud > 0.3
    assert ok, (max_abs, rel)


def check_heads(pool, wl, ids, lens, x, X64):
    """Output heads on seeded hidden states after a forward call has routed the batch: scores to the
    fp32 bar, labels exact wherever the oracle's two best scores are further apart than that bar."""
    N = int(lens.sum())
    scores = torch.full((N, wl.max_classes), float("nan"), dtype=torch.float32, device=x.device)
    labels = torch.full((N,), -7, dtype=torch.int32, device=x.device)
    pool.head_forward(x, scores, labels)
    torch.cuda.synchronize()
    heads = {t: tuple(a.astype(np.float64) for a in synth.head_tensors(wl, t)) + (synth.head_spec(wl, t)[1],)
             for t in set(ids.tolist())}
    sc_ref, lab_ref = O.head_forward(X64, ids, lens, lambda t: heads[t], wl.max_classes)
    sc, lab = scores.cpu().numpy().astype(np.float64), labels.cpu().numpy()
    assert np.array_equal(np.isneginf(sc), np.isneginf(sc_ref))
    fin = np.isfinite(sc_ref)
    assert np.isfinite(sc[fin]).all()
    err = np.abs(sc[fin] - sc_ref[fin]).max()
    top2 = np.sort(np.where(fin, sc_ref, -np.inf), axis=1)[:, -2:]
    with np.errstate(invalid="ignore"):     # rows without a prediction: -inf - -inf
        clear = (lab_ref < 0) | (top2[:, 1] - top2[:, 0] > 1e-4)
    print(f"  heads: {int((lab_ref >= 0).sum())} predictions, max score error {err:.2e}, "
          f"{int((~clear).sum())} near-ties, tagging tenants {sum(h[2] for h in heads.values())}/{len(heads)}", flush=True)
    assert err <= 1e-4
    np.testing.assert_array_equal(lab[clear], lab_ref[clear])
    assert ((lab == lab_ref) | ~clear).all() and (lab[~clear] >= 0).all()
    # labels only
    labels2 = torch.full_like(labels, -7)
    pool.head_forward(x, None, labels2)
    torch.cuda.synchronize()
    assert torch.equal(labels, labels2)


@pytest.mark.parametrize("dtype,d_model,max_classes", [("bf16", 128, 9), ("bf16", 768, 9), ("f32", 64, 9),
                                                       ("bf16", 2048, 64), ("f32", 528, 2)])
def test_output_heads_ragged(hmi, dtype, d_model, max_classes):
    """Sec. 3.3.2: per-tenant linear heads with their own class counts, classification tenants on
    the first row of a request, tagging tenants on every row, label = highest score.  The last two cases: the
    widest model with the most classes a head may have (64), and two classes on a width that is no multiple of 64."""
    from paper_2504_17449_amd import harness
    wl = small(synth.BLOCK_ADAPTER, dtype, d_model=d_model, d_ff=64 if dtype == "bf16" else 16, n_tenants=40,
               hbm_slots=40, n_requests=60, seq_max=70, max_classes=max_classes)
    ids, lens, x = harness.batch_to_device(wl)
    pool = harness.create_pool(wl, max_tokens=int(lens.sum()))
    try:
        harness.load_tenants(pool, wl, sorted(set(ids.tolist())))
        y = torch.empty_like(x)
        pool.forward(0, x, y, ids, lens)
        X64 = np.concatenate([synth.hidden_states(wl, r, int(lens[r])) for r in range(len(ids))]).astype(np.float64)
        check_heads(pool, wl, ids, lens, x, X64)
    finally:
        pool.close()


@pytest.mark.parametrize("block,kw", [
    (synth.BLOCK_DEC_PRELN, {}), (synth.BLOCK_DEC_ADAPTER, {}),
    # 70 rows through shared matrices with k = 1024: the launch that shares an item's k between four wavefronts
    (synth.BLOCK_DEC_ADAPTER, dict(d_model=256, d_ff=1024, n_heads=4, n_requests=70, n_tenants=9, hbm_slots=9, seq_max=40)),
], ids=["own_layer", "shared_layer", "shared_layer_70_rows"])
def test_decode_steps_with_kv_cache_match_full_causal_forward(hmi, block, kw):
    """Prefill ragged prompts of many tenants, then generate: every decode step's row must equal the
    last row of the oracle's full causal forward over the sequence so far (two layers, so the second
    layer's cache holds first-layer outputs).  Some requests stop early, so lines of different
    lengths and a shrinking batch are covered; sequence slots are a scattered subset of the lines."""
    from paper_2504_17449_amd import harness, HmiError, HMI_ERR_SHAPE, HMI_ERR_ARG
    from tests.oracle_side import weights_of
    wl = small(block, "bf16", **{**dict(n_layers=2, n_tenants=6, hbm_slots=6, n_requests=14, seq_max=70), **kw})
    ids, lens = synth.batch_ids_lens(wl)
    R, L, G = len(ids), wl.n_layers, 5
    full = [synth.hidden_states(wl, r, int(lens[r]) + G) for r in range(R)]
    slots = (np.random.default_rng(1).permutation(R + 5)[:R]).astype(np.int32)
    pool = harness.create_pool(wl, max_tokens=int(lens.sum()))
    wof = [weights_of(wl, l) for l in range(L)]

    def oracle_last_row(r, n_rows):
        cur = full[r][:n_rows].astype(np.float64)
        for l in range(L):
            cur = O.block_forward(block, cur, wof[l](int(ids[r])), wl.n_heads, wl.ln_eps)
        return cur

    try:
        harness.load_tenants(pool, wl, sorted(set(ids.tolist())))
        pool.kv_create(R + 5, int(lens.max()) + G)
        x = harness.host_to_device(np.concatenate([full[r][:lens[r]] for r in range(R)]), "bf16")
        y = torch.empty_like(x)
        pool.prefill(0, L, x, y, ids, lens, slots)
        torch.cuda.synchronize()
        y_ref = np.concatenate([oracle_last_row(r, int(lens[r])) for r in range(R)])
        max_abs, rel, ok = compare(harness.device_to_f64(y), y_ref, np.arange(len(y_ref)), "bf16")
        print(f"  prefill: max_abs={max_abs:.3e} rel_fro={rel:.3e}", flush=True)
        assert ok
        alive = list(range(R))
        for g in range(G):
            if g == 2:
                alive = [r for r in alive if r % 3 != 1]      # a third of the requests stop here
            if g == 4:
                alive = alive[::-1]                           # and the batch order changes
            xn = harness.host_to_device(np.stack([full[r][lens[r] + g] for r in alive]), "bf16")
            yn = torch.empty_like(xn)
            pool.decode_step(0, L, xn, yn, ids[alive], slots[alive])
            torch.cuda.synchronize()
            want = np.stack([oracle_last_row(r, int(lens[r]) + g + 1)[-1] for r in alive])
            max_abs, rel, ok = compare(harness.device_to_f64(yn), want, np.arange(len(alive)), "bf16")
            print(f"  step {g}: {len(alive)} requests, max_abs={max_abs:.3e} rel_fro={rel:.3e}", flush=True)
            assert ok, (g, max_abs, rel)
        # error paths: nothing is enqueued, the line lengths do not move
        with pytest.raises(HmiError) as e:
            pool.decode_step(0, L, xn, yn, ids[alive[:2]], slots[[alive[0], alive[0]]])
        assert e.value.code == HMI_ERR_ARG
        longest = int(np.argmax(lens))          # its line is full after G steps if it never stopped
        if longest in alive:
            with pytest.raises(HmiError) as e:
                pool.decode_step(0, L, xn[:1], yn[:1], ids[[longest]], slots[[longest]])
            assert e.value.code == HMI_ERR_SHAPE
    finally:
        pool.close()


def test_errors_of_shared_layers_heads_and_cache(hmi):
    """Every refusal happens before anything is enqueued: y keeps its contents."""
    from paper_2504_17449_amd import harness
    wl = small(synth.BLOCK_ENC_ADAPTER, "bf16", n_tenants=3, hbm_slots=3, n_requests=4, seq_max=9, max_classes=4)
    ids, lens, x = harness.batch_to_device(wl)
    pool = harness.create_pool(wl, max_tokens=int(lens.sum()))
    try:
        for t in range(3):
            pool.load_tenant(t, 0, synth.tenant_storage(wl, t, 0))
        y = torch.full_like(x, 7.0)
        # shared parameters missing
        assert hmi.hmi_layer_forward(pool.h, 0, x.data_ptr(), y.data_ptr(), ids, lens) == hmi.HMI_ERR_ARG
        assert "shared" in hmi.hmi_last_error(pool.h)
        shared = synth.shared_storage(wl, 0)
        assert hmi.hmi_pool_load_shared(pool.h, 0, shared[:5]) == hmi.HMI_ERR_SHAPE
        assert hmi.hmi_pool_load_shared(pool.h, 1, shared) == hmi.HMI_ERR_ARG          # no such layer
        # heads before any batch was routed, unknown class counts, a tenant without a head
        labels = torch.zeros(int(lens.sum()), dtype=torch.int32, device=x.device)
        assert hmi.hmi_head_forward(pool.h, x.data_ptr(), 0, labels.data_ptr()) == hmi.HMI_ERR_ARG
        w, b = synth.head_tensors(wl, 0, raw=True)
        assert hmi.hmi_pool_load_head(pool.h, 0, np.zeros((5, wl.d_model), np.uint16), np.zeros(5, np.uint16), False) == hmi.HMI_ERR_SHAPE
        assert hmi.hmi_pool_load_head(pool.h, 3, w, b, False) == hmi.HMI_ERR_TENANT
        assert hmi.hmi_pool_load_head(pool.h, 0, w, b, False) == hmi.HMI_OK
        assert hmi.hmi_pool_load_shared(pool.h, 0, shared) == hmi.HMI_OK
        torch.cuda.synchronize()
        assert torch.all(y == 7.0)
        pool.forward(0, x, y, ids, lens)
        if len(set(ids.tolist())) > 1 or ids[0] != 0:
            assert hmi.hmi_head_forward(pool.h, y.data_ptr(), 0, labels.data_ptr()) == hmi.HMI_ERR_TENANT
        # no key/value cache for encoder pools
        assert hmi.hmi_kv_create(pool.h, 4, 16) == hmi.HMI_ERR_ARG
    finally:
        pool.close()
    # pools without heads / shared parameters refuse those calls
    wl2 = small(synth.BLOCK_DEC_PRELN, "bf16", n_tenants=2, hbm_slots=2, n_requests=2, seq_max=5)
    pool = harness.create_pool(wl2, max_tokens=16)
    try:
        assert hmi.hmi_pool_load_shared(pool.h, 0, synth.tenant_storage(wl2, 0, 0)) == hmi.HMI_ERR_ARG
        assert hmi.hmi_pool_load_head(pool.h, 0, np.zeros((2, 128), np.uint16), np.zeros(2, np.uint16), False) == hmi.HMI_ERR_ARG
        xs = torch.zeros((2, wl2.d_model), dtype=torch.bfloat16, device="cuda")
        assert hmi.hmi_decode_step(pool.h, 0, 1, xs.data_ptr(), torch.empty_like(xs).data_ptr(), [0, 1], [0, 1]) == hmi.HMI_ERR_TENANT
        pool.load_tenant(0, 0, synth.tenant_storage(wl2, 0, 0))
        pool.load_tenant(1, 0, synth.tenant_storage(wl2, 1, 0))
        assert hmi.hmi_decode_step(pool.h, 0, 1, xs.data_ptr(), torch.empty_like(xs).data_ptr(), [0, 1], [0, 1]) == hmi.HMI_ERR_ARG   # no cache yet
        assert hmi.hmi_kv_create(pool.h, 2, 8) == hmi.HMI_OK
        assert hmi.hmi_kv_create(pool.h, 2, 8) == hmi.HMI_ERR_ARG           # once per pool
        assert hmi.hmi_decode_step(pool.h, 0, 1, xs.data_ptr(), torch.empty_like(xs).data_ptr(), [0, 1], [0, 2]) == hmi.HMI_ERR_ARG   # slot out of range
        assert hmi.hmi_prefill(pool.h, 0, 1, xs.data_ptr(), torch.empty_like(xs).data_ptr(), [0], [9], [0]) == hmi.HMI_ERR_SHAPE      # longer than a line
    finally:
        pool.close()


@pytest.mark.parametrize("dtype,d_model,entries", [("bf16", 768, 3000), ("bf16", 128, 50), ("f32", 64, 50)])
def test_plot_aggregate_ragged(hmi, dtype, d_model, entries):
    """Sec. 3.3.1: token representations aggregated from tri-gram table rows; requests of 1, 2 and more
    tokens (two or one fragments at the ends), every row compared."""
    from paper_2504_17449_amd import harness
    wl = small(synth.BLOCK_FFN, dtype, d_model=d_model, d_ff=d_model, n_requests=40, seq_max=60)
    _, lens = synth.batch_ids_lens(wl)
    lens[:3] = [1, 2, 3]
    if d_model == 128:
        lens[3] = 2100          # longer than the kernel's in-LDS copy of a request's fragment ids
    N = int(lens.sum())
    table = synth.plot_table(wl, entries)
    frag = synth.plot_fragment_ids(wl, entries, N)
    pool = harness.create_pool(wl, max_tokens=N)
    try:
        t_dev = harness.host_to_device(table.reshape(entries * 3, d_model), dtype).reshape(entries, 3, d_model)
        f_dev = torch.from_numpy(frag).cuda()
        x = torch.full((N, d_model), 7.0, device="cuda").to(t_dev.dtype)
        pool.plot_aggregate(t_dev, f_dev, lens, x)
        torch.cuda.synchronize()
        got = harness.device_to_f64(x)
        # refusals leave x alone
        assert hmi.hmi_plot_aggregate(pool.h, t_dev.data_ptr(), entries, f_dev.data_ptr(), [0, 4], x.data_ptr()) == hmi.HMI_ERR_SHAPE
        assert hmi.hmi_plot_aggregate(pool.h, 0, entries, f_dev.data_ptr(), lens, x.data_ptr()) == hmi.HMI_ERR_ARG
    finally:
        pool.close()
    want = O.plot_aggregate(table, frag, lens)
    max_abs, rel, ok = compare(got, want, np.arange(N), dtype)
    print(f"  aggregate: N={N} max_abs={max_abs:.3e} rel_fro={rel:.3e}", flush=True)
    assert ok, (max_abs, rel)


@pytest.mark.parametrize("block", [synth.BLOCK_FFN, synth.BLOCK_ENC_ADAPTER])
def test_back_to_back_calls_with_different_batches(hmi, block):
    """Six forward calls enqueued without waiting, alternating between three different batches that
    share the pool's routing arrays and workspaces: every call's output and the last routing must be
    right, and the same batch must give the same bits."""
    from paper_2504_17449_amd import harness
    wl = small(block, "bf16", d_model=256, d_ff=512, n_heads=4, n_tenants=9, hbm_slots=9, n_requests=25, seq_max=120)
    batches = [harness.batch_to_device(wl, b) for b in range(3)]
    pool = harness.create_pool(wl, max_tokens=max(int(l.sum()) for _, l, _ in batches))
    try:
        harness.load_tenants(pool, wl)
        order = [0, 1, 2, 0, 2, 1]
        outs = []
        for b in order:
            ids, lens, x = batches[b]
            y = torch.empty_like(x)
            pool.forward(0, x, y, ids, lens)
            outs.append(y)
        torch.cuda.synchronize()
        check_route(pool, batches[order[-1]][0], batches[order[-1]][1])
        got = [harness.device_to_f64(y) for y in outs]
    finally:
        pool.close()
    refs = {}
    for b, y in zip(order, got):
        ids, lens, _ = batches[b]
        if b not in refs:
            refs[b] = oracle_forward(wl, ids, lens, None, b)
        max_abs, rel, ok = compare(y, refs[b], np.arange(len(y)), "bf16")
        assert ok, (b, max_abs, rel)
    assert np.array_equal(got[0], got[3]) and np.array_equal(got[1], got[5])    # same batch, same bits


@pytest.mark.parametrize("seed", range(12))
def test_seeded_random_small_shapes(hmi, seed):
    """Shapes nobody picked by hand: block kind, widths, ranks, head counts, layer counts, request counts and
    length ranges drawn from a seeded generator (bf16; every row compared).  Small batches take the skinny GEMM,
    larger ones the tiled kernels, widths of 256 / 512 / 768 the one-kernel adapter."""
    rng = np.random.default_rng(1000 + seed)
    block = int(rng.choice([synth.BLOCK_FFN, synth.BLOCK_ENC_POSTLN, synth.BLOCK_DEC_PRELN, synth.BLOCK_ADAPTER,
                            synth.BLOCK_ENC_ADAPTER, synth.BLOCK_DEC_ADAPTER]))
    heads = int(rng.integers(1, 7))
    attn = block not in (synth.BLOCK_FFN, synth.BLOCK_ADAPTER)
    d = heads * 64 if attn else int(rng.integers(1, 13)) * 64
    f = 64 if block == synth.BLOCK_ADAPTER else int(rng.integers(1, 9)) * 64
    tenants = int(rng.integers(1, 10))
    smax = int(rng.choice([1, 7, 40, 150, 330]))
    kw = dict(d_model=d, d_ff=f, n_heads=heads if attn else 0, n_layers=int(rng.integers(1, 4)), n_tenants=tenants,
              hbm_slots=tenants, n_requests=int(rng.integers(1, 30)), seq_min=1, seq_max=smax,
              popularity=str(rng.choice(["uniform", "zipf"])), seed=int(rng.integers(0, 1000)))
    if block in (synth.BLOCK_ENC_ADAPTER, synth.BLOCK_DEC_ADAPTER):
        kw["adapter_rank"] = int(rng.choice([64, 128]))
        kw["d_ff"] = max(f, kw["adapter_rank"])
    if block in (synth.BLOCK_DEC_PRELN, synth.BLOCK_DEC_ADAPTER):
        kw["n_layers"] = min(kw["n_layers"], 2)      # pre-LN stacks carry |y| upwards: keep it under the bf16 half-ulp bar
    print(f"seed {seed}: block {block} {kw}", flush=True)
    run_case(hmi, small(block, "bf16", **kw), slack=7 * (seed % 2))    # odd seeds: a pool larger than the batch


def round_to_bf16(a) -> np.ndarray:
    """fp32 values rounded to the nearest bf16 (ties to even), returned as fp32."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = ((u + 0x7FFF + ((u >> 16) & 1)) >> 16) << 16
    return u.astype(np.uint32).view(np.float32)


def test_gelu_of_the_persistent_gemm_alone_on_a_grid(hmi):
    """The persistent bf16 GEMM evaluates GELU with a polynomial instead of erf.  This isolates it
    through the C ABI: a pre-LN decoder pool whose attention weights, W1 and all biases but b1 are zero and whose
    W2 is the identity gives, for x = 0, y[row, j] = GELU(b1[j]) exactly as the kernel stored it (one non-zero
    product per output, so nothing else rounds).  b1 is a grid over [-9, 9] (four tenants, 1 024 values, bf16
    exact), beyond the point |x| = 4 where the polynomial is clamped.  Held to the polynomial's stated bound:
    |error| <= 2e-4 from the fit, plus the bf16 rounding of the stored value (one ulp allowed)."""
    from paper_2504_17449_amd import harness
    d = 256
    wl = small(synth.BLOCK_DEC_PRELN, "bf16", d_model=d, d_ff=d, n_heads=4, n_tenants=4, hbm_slots=4)
    grid = round_to_bf16(np.concatenate([np.linspace(-9.0, 9.0, 1000), [-4.0, 4.0, 0.0, -0.0], np.linspace(-0.02, 0.02, 20)])
                         .astype(np.float32))
    assert grid.size == 4 * d
    zeros = lambda *shape: np.zeros(shape, np.float32)
    ids = np.repeat(np.arange(4, dtype=np.int32), 3)            # 12 requests of 256 rows: enough rows for the persistent kernel
    lens = np.full(12, 256, np.int32)
    pool = harness.create_pool(wl, max_requests=12, max_tokens=int(lens.sum()))
    weights = {}
    try:
        for t in range(4):
            w = {"wqkv": zeros(3 * d, d), "bqkv": zeros(3 * d), "wo": zeros(d, d), "bo": zeros(d),
                 "ln1_g": np.ones(d, np.float32), "ln1_b": zeros(d), "w1": zeros(d, d), "b1": grid[t * d:(t + 1) * d],
                 "w2": np.eye(d, dtype=np.float32), "b2": zeros(d), "ln2_g": np.ones(d, np.float32), "ln2_b": zeros(d)}
            weights[t] = w
            names = [n for n, _, _ in synth.tensor_specs(wl)]
            pool.load_tenant(t, 0, [synth.to_storage_bytes(w[n], "bf16") for n in names])
        x = torch.zeros(int(lens.sum()), d, dtype=torch.bfloat16, device="cuda")
        y = torch.empty_like(x)
        pool.forward(0, x, y, ids, lens)
        torch.cuda.synchronize()
        y_gpu = harness.device_to_f64(y)
    finally:
        pool.close()
    wof = lambda t: {k: v.astype(np.float64) for k, v in weights[t].items()}
    y_ref = O.layer_forward(wl.block, np.zeros((int(lens.sum()), d)), ids, lens, wof, wl.n_heads, wl.ln_eps)
    g = y_ref                                                    # = GELU(b1[j]) in every row of the tenant
    np.testing.assert_allclose(y_ref[0], O.gelu(grid[:d].astype(np.float64)), rtol=0, atol=1e-12)
    err = np.abs(y_gpu - y_ref)
    bound = 2e-4 + 2.0 ** -8 * np.abs(g) + 1e-6                  # fit + bf16 rounding (one ulp) + fp32 evaluation
    worst = int(np.argmax(err - bound))
    print(f"  GELU grid: max |error| {err.max():.3e}, worst excess over the bound {(err - bound).max():.3e} "
          f"at x = {grid[(ids[worst // d // 256] * d) + worst % d]:.4f}", flush=True)
    assert (err <= bound).all()
    # rows of one tenant are identical, and the negative tail is not flushed to zero before the clamp
    assert np.array_equal(y_gpu[0], y_gpu[255])
    i3 = int(np.argmin(np.abs(grid + 3.0)))                      # GELU(-3) = -4.05e-3
    assert y_gpu[(i3 // d) * 3 * 256, i3 % d] < -3.5e-3


def test_bert_ffn_full_size_every_request(hmi):
    """The benchmarked configuration (64 tenants, 256 requests of 128 tokens, d = 768, f = 3072) as bench.py
    runs it, all 32 768 rows against the oracle."""
    run_case(hmi, synth.WORKLOADS["bert_ffn"], tenants="all")


def test_two_pools_of_different_shapes_take_turns(hmi):
    """Two pools alive at once (an FFN pool of width 256 on the torch stream, an encoder pool of width 512 on a
    stream of its own), called alternately with nothing synchronised in between: per-pool state (routing arrays,
    tile counters, workspaces) must not be shared, whatever the order the two streams run in."""
    from paper_2504_17449_amd import harness
    wa = small(synth.BLOCK_FFN, "bf16", d_model=256, d_ff=768, n_requests=30, n_tenants=5, hbm_slots=5, seed=31)
    wb = small(synth.BLOCK_ENC_POSTLN, "bf16", d_model=512, d_ff=1024, n_heads=8, n_requests=12, n_tenants=3,
               hbm_slots=3, seed=32)
    side = torch.cuda.Stream()
    batches_a = [harness.batch_to_device(wa, b) for b in range(3)]
    batches_b = [harness.batch_to_device(wb, b) for b in range(3)]
    pa = harness.create_pool(wa, max_tokens=max(int(l.sum()) for _, l, _ in batches_a))
    with torch.cuda.stream(side):
        pb = harness.create_pool(wb, max_tokens=max(int(l.sum()) for _, l, _ in batches_b))
    try:
        harness.load_tenants(pa, wa)
        harness.load_tenants(pb, wb)
        torch.cuda.synchronize()
        outs = []
        for b in range(3):
            for pool, (ids, lens, x), wl in ((pa, batches_a[b], wa), (pb, batches_b[b], wb)):
                y = torch.empty_like(x)
                pool.forward(0, x, y, ids, lens)
                outs.append((wl, b, ids, lens, y))
        torch.cuda.synchronize()
        for wl, b, ids, lens, y in outs:
            y_ref = oracle_forward(wl, ids, lens, None, b)
            max_abs, rel, ok = compare(harness.device_to_f64(y), y_ref, np.arange(len(y_ref)), "bf16")
            assert ok, (wl.name, b, max_abs, rel)
    finally:
        pa.close()
        pb.close()


def test_two_host_threads_each_with_a_pool_of_its_own(hmi):
    """Different pools may be used from different host threads at once: each thread creates its pool on a stream of
    its own, loads tenants and runs three batches (ctypes drops the interpreter lock inside every call, so the two
    threads really are inside the library together)."""
    import threading
    from paper_2504_17449_amd import harness
    specs = [small(synth.BLOCK_FFN, "bf16", d_model=256, d_ff=768, n_requests=30, n_tenants=5, hbm_slots=5, seed=41),
             small(synth.BLOCK_DEC_PRELN, "bf16", d_model=256, d_ff=512, n_heads=4, n_requests=16, n_tenants=4,
                   hbm_slots=4, seed=42)]
    batches = [[harness.batch_to_device(wl, b) for b in range(3)] for wl in specs]
    torch.cuda.synchronize()
    results, errors = [None, None], []
    start = threading.Barrier(2)

    def worker(i):
        try:
            wl = specs[i]
            with torch.cuda.stream(torch.cuda.Stream()):
                start.wait(timeout=60)
                pool = harness.create_pool(wl, max_tokens=max(int(l.sum()) for _, l, _ in batches[i]))
                try:
                    harness.load_tenants(pool, wl, workers=2)
                    outs = []
                    for ids, lens, x in batches[i]:
                        y = torch.empty_like(x)
                        pool.forward(0, x, y, ids, lens)
                        outs.append(y)
                    torch.cuda.current_stream().synchronize()
                    results[i] = [harness.device_to_f64(y) for y in outs]
                finally:
                    pool.close()
        except BaseException as e:   # noqa: BLE001 - reported by the main thread
            errors.append((i, repr(e)))

    threads = [threading.Thread(target=worker, args=(i,)) for i in range(2)]
    for t in threads:
        t.start()
    for t in threads:
        t.join(timeout=180)
    assert not errors, errors
    for i, wl in enumerate(specs):
        for b, (ids, lens, _) in enumerate(batches[i]):
            y_ref = oracle_forward(wl, ids, lens, None, b)
            max_abs, rel, ok = compare(results[i][b], y_ref, np.arange(len(y_ref)), "bf16")
            assert ok, (wl.name, b, max_abs, rel)


def test_tenant_ids_up_to_four_million(hmi):
    """The router's radix sort takes as many passes of up to six bits as the id space needs: one for 64 tenants, two
    for 1 000, three for 10 000.  An id space of 2^22 (host-tier pool, eight HBM slots) takes four; the few tenants
    that exist have ids spread over the whole range, some equal in their low 6, 12 and 18 bits."""
    from paper_2504_17449_amd import harness
    T = 1 << 22
    wl = small(synth.BLOCK_FFN, "bf16", n_tenants=T, hbm_slots=8, host_tier=True, n_requests=40, seq_max=40)
    exist = np.array([3, 3 + (1 << 6), 3 + (1 << 12), 3 + (1 << 18), 70000, 1 << 20, T - 1], np.int32)
    rng = np.random.default_rng(7)
    ids = rng.choice(exist, size=wl.n_requests).astype(np.int32)
    _, lens, x = harness.batch_to_device(wl, 0)
    pool = harness.create_pool(wl, max_requests=len(ids), max_tokens=int(lens.sum()))
    try:
        harness.load_tenants(pool, wl, exist.tolist())
        y = torch.empty_like(x)
        pool.forward(0, x, y, ids, lens)
        torch.cuda.synchronize()
        check_route(pool, ids, lens)
        y_ref = oracle_forward(wl, ids, lens, None, 0)
        max_abs, rel, ok = compare(harness.device_to_f64(y), y_ref, np.arange(len(y_ref)), "bf16")
        assert ok, (max_abs, rel)
    finally:
        pool.close()


@pytest.mark.parametrize("block", [synth.BLOCK_ENC_POSTLN, synth.BLOCK_DEC_PRELN])
def test_one_request_of_4096_tokens(hmi, block):
    """One sequence of 4 096 tokens: 64 key blocks per query block in the attention kernel (32 query blocks of 128),
    one segment of 16 m-tiles in the GEMMs; bidirectional and causal, every row compared."""
    run_case(hmi, small(block, "bf16", d_model=256, d_ff=512, n_heads=4, n_tenants=1, hbm_slots=1, n_requests=1,
                        seq_min=4096, seq_max=4096))


def test_single_request_and_single_tenant(hmi):
    run_case(hmi, small(synth.BLOCK_ENC_POSTLN, "bf16", n_requests=1, seq_min=5, seq_max=5))
    run_case(hmi, small(synth.BLOCK_DEC_PRELN, "bf16", n_tenants=1, hbm_slots=1, n_requests=9))


def test_same_inputs_same_weights_identical_rows(hmi):
    """Two requests with identical hidden states routed to the same tenant get bit-identical rows."""
    from paper_2504_17449_amd import harness
    wl = small(synth.BLOCK_ENC_POSTLN, "bf16", n_tenants=3, hbm_slots=3)
    pool = harness.create_pool(wl, max_requests=4, max_tokens=4 * 70)
    try:
        harness.load_tenants(pool, wl)
        x1 = synth.hidden_states(wl, 0, 70)
        x = harness.host_to_device(np.concatenate([x1, x1, x1, x1]), wl.dtype)
        y = torch.empty_like(x)
        pool.forward(0, x, y, [2, 0, 2, 1], [70, 70, 70, 70])
        torch.cuda.synchronize()
        yv = y.view(torch.int16).cpu().numpy()
        assert np.array_equal(yv[0:70], yv[140:210])        # same tenant
        assert not np.array_equal(yv[0:70], yv[70:140])     # different tenant
    finally:
        pool.close()


def test_boundary_errors_and_empty_batch(hmi):
    from paper_2504_17449_amd import harness
    wl = small(synth.BLOCK_FFN, "bf16", n_tenants=4, hbm_slots=4)
    pool = harness.create_pool(wl, max_requests=4, max_tokens=64)
    try:
        harness.load_tenants(pool, wl, [0, 1])
        x = torch.zeros(64, wl.d_model, dtype=torch.bfloat16, device="cuda")
        y = torch.full_like(x, 7.0)
        assert hmi.hmi_layer_forward(pool.h, 0, x.data_ptr(), y.data_ptr(), [], []) == hmi.HMI_OK
        cases = [([0, 9], [4, 4], hmi.HMI_ERR_TENANT),      # id out of range
                 ([0, 2], [4, 4], hmi.HMI_ERR_TENANT),      # never loaded
                 ([0, 1], [4, 0], hmi.HMI_ERR_SHAPE),       # empty sequence
                 ([0, 1], [40, 40], hmi.HMI_ERR_SHAPE),     # too many tokens
                 ([0] * 5, [1] * 5, hmi.HMI_ERR_SHAPE)]     # too many requests
        for ids, lens, want in cases:
            assert hmi.hmi_layer_forward(pool.h, 0, x.data_ptr(), y.data_ptr(), ids, lens) == want
            assert hmi.hmi_last_error(pool.h)
        assert hmi.hmi_layer_forward(pool.h, 0, x.data_ptr(), x.data_ptr(), [0], [4]) == hmi.HMI_ERR_ARG
        assert hmi.hmi_layer_forward(pool.h, 3, x.data_ptr(), y.data_ptr(), [0], [4]) == hmi.HMI_ERR_ARG
        torch.cuda.synchronize()
        assert bool((y == 7.0).all())                       # y untouched by every failed call
        assert hmi.hmi_pool_load_tenant(pool.h, 0, 0, [np.zeros(4, np.uint16)]) == hmi.HMI_ERR_SHAPE
    finally:
        pool.close()


def test_a_pool_larger_than_the_gpu_is_refused_and_leaves_nothing_behind(hmi):
    """6 000 slots of a 67 MB FFN block are 400 GB: creation fails with HMI_ERR_OOM, hands out no pool, gives back
    what it had already allocated, and a pool of ordinary size is created and works right afterwards."""
    torch.cuda.synchronize()
    free_before, _ = torch.cuda.mem_get_info()
    rc, h = hmi.hmi_pool_create(block=hmi.HMI_BLOCK_FFN, dtype=hmi.HMI_BF16, d_model=2048, d_ff=8192, n_heads=0,
                                n_layers=1, max_tenants=6000, hbm_slots=6000, host_tier=0, max_requests=8,
                                max_tokens=1024, ln_eps=1e-5, device=0,
                                compute_stream=torch.cuda.current_stream().cuda_stream)
    assert rc == hmi.HMI_ERR_OOM and h is None, (rc, hmi.hmi_last_error(None))
    assert hmi.hmi_last_error(None)
    free_after, _ = torch.cuda.mem_get_info()
    assert abs(free_before - free_after) < (1 << 30), (free_before, free_after)
    run_case(hmi, small(synth.BLOCK_FFN, "bf16"))
