"""The C-ABI library loads and exports every symbol include/hmi.h declares (no compute)."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "hmi.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(hmi_[a-z0-9_]+)\s*\(", text)))


def test_header_declares_the_four_north_star_calls():
    syms = declared_symbols()
    for name in ("hmi_pool_create", "hmi_pool_load_tenant", "hmi_layer_forward", "hmi_pool_destroy"):
        assert name in syms


def test_library_exports_every_declared_symbol():
    import paper_2504_17449_amd as pkg
    lib = ctypes.CDLL(pkg.LIB_PATH)
    for name in declared_symbols():
        assert hasattr(lib, name), name
    assert sorted(pkg.EXPORTS) == declared_symbols()


def test_argument_errors_need_no_gpu():
    import paper_2504_17449_amd as pkg
    assert pkg.lib.hmi_pool_create(None, None) == pkg.HMI_ERR_ARG
    assert "null" in pkg.hmi_last_error(None)
    assert pkg.hmi_pool_destroy(None) == pkg.HMI_OK
    assert pkg.lib.hmi_layer_forward(None, 0, None, None, None, None, 0) == pkg.HMI_ERR_ARG
    rc, h = pkg.hmi_pool_create(block=9, dtype=1, d_model=64, d_ff=64, max_tenants=1,
                                max_requests=1, max_tokens=1)
    assert rc == pkg.HMI_ERR_ARG and h is None
    rc, h = pkg.hmi_pool_create(block=0, dtype=1, d_model=100, d_ff=64, max_tenants=1,
                                max_requests=1, max_tokens=1)
    assert rc == pkg.HMI_ERR_ARG and "multiples" in pkg.hmi_last_error(None)
    # sizes that are products of caller-given numbers are refused before anything is allocated or can wrap
    small = dict(block=0, dtype=1, d_model=64, d_ff=64, max_tenants=1, max_requests=1, max_tokens=1)
    for kw, want, word in ((dict(max_tenants=1 << 25, hbm_slots=1 << 25), pkg.HMI_ERR_ARG, "max_tenants"),
                           (dict(n_layers=5000), pkg.HMI_ERR_ARG, "n_layers"),
                           (dict(max_tenants=1 << 24, hbm_slots=1 << 24, n_layers=1024, d_model=2048, d_ff=1 << 20),
                            pkg.HMI_ERR_OOM, "exceeds")):
        rc, h = pkg.hmi_pool_create(**{**small, **kw})
        assert rc == want and h is None and word in pkg.hmi_last_error(None), (kw, rc, pkg.hmi_last_error(None))
    # the other entry points with no pool: an error code, nothing touched, no GPU call
    for name in ("hmi_stack_forward", "hmi_stack_forward_f32"):
        assert getattr(pkg.lib, name)(None, 0, 1, None, None, None, None, 0) == pkg.HMI_ERR_ARG
    assert pkg.lib.hmi_layer_forward_static(None, 0, None, None, None, None, 0) == pkg.HMI_ERR_ARG
    assert pkg.lib.hmi_pool_alias_tenant(None, 0, 0) == pkg.HMI_ERR_ARG
    assert pkg.lib.hmi_pool_prefetch(None, 0, None, 0) == pkg.HMI_ERR_ARG
    assert pkg.lib.hmi_queue_create(None, 1, 1, 1, None) == pkg.HMI_ERR_ARG
    assert pkg.lib.hmi_queue_push(None, 0, 1, None, None) == pkg.HMI_ERR_ARG
    assert pkg.lib.hmi_queue_run(None, None, None) == pkg.HMI_ERR_ARG
    assert pkg.lib.hmi_queue_fetch(None, 0, None) == pkg.HMI_ERR_ARG
    assert pkg.lib.hmi_queue_waiting(None) == 0
    assert pkg.lib.hmi_queue_destroy(None) == pkg.HMI_OK


def test_binding_loads_torch_before_the_library():
    """Buffers and streams come from torch, so the library must bind to the HIP runtime torch ships: the binding
    imports torch before it loads libhmi.so (the other order leaves two runtimes in the process)."""
    import subprocess
    import sys
    code = ("import sys; import paper_2504_17449_amd as p; assert 'torch' in sys.modules; "
            "maps = open('/proc/self/maps').read(); hip = sorted({l.split()[-1] for l in maps.splitlines() if 'libamdhip64' in l}); "
            "assert len(hip) == 1, hip; print(hip[0])")
    r = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, timeout=300, cwd=ROOT)
    assert r.returncode == 0, r.stderr
    assert "/torch/" in r.stdout, r.stdout


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU: any other --gpus exits non-zero with a message that says so, before torch is imported."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=60)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""
