"""Seeded, keyed synthetic inputs shaped like the paper's hBERT / hGPT serving workloads.

Every array is a pure function of ``(seed, what, tenant-or-request, layer, tensor)``:
a tenant's weights or a request's hidden states can be regenerated alone, so a
consumer never has to materialise a whole 1 000- or 10 000-tenant pool to look at
the few tenants a batch touches.  Values are fp32 draws rounded ONCE to the storage
dtype (bf16 or fp32); every consumer starts from those rounded values.

Nothing here computes any part of the layer: only random draws, shape tables and
dtype packing.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import List, Tuple

import threading

import numpy as np

BLOCK_FFN = 0          # Y = LN(X + W2 GELU(W1 X + b1) + b2)
BLOCK_ENC_POSTLN = 1   # bidirectional attention + FFN, LayerNorm after each residual
BLOCK_DEC_PRELN = 2    # causal attention + FFN, LayerNorm before each sub-layer
BLOCK_ADAPTER = 3      # Y = X + Up(ReLU(Down(X)))  (bottleneck adapter, Sec. 3.2.2)
BLOCK_ENC_ADAPTER = 4  # shared post-LN encoder layer + per-tenant adapter after its attention layer (Sec. 3.2.2)

BLOCK_DEC_ADAPTER = 5  # the same with a shared pre-LN causal decoder layer

SHARED = 0x7FFFFFFF    # "tenant" key of the parameters every tenant shares

_TAG_WEIGHT, _TAG_X, _TAG_IDS, _TAG_LENS, _TAG_HEAD, _TAG_PLOT = 1, 2, 3, 4, 5, 6
_HEAD_LAYER = 1 << 20  # "layer" key of a tenant's output head


@dataclass(frozen=True)
class Workload:
    name: str
    block: int
    dtype: str            # "f32" | "bf16": storage dtype of weights and activations
    d_model: int
    d_ff: int             # FFN width (adapter: bottleneck width r)
    n_heads: int          # 0 for blocks without attention
    n_layers: int
    n_tenants: int
    n_requests: int
    seq_min: int
    seq_max: int          # inclusive; == seq_min for fixed-length batches
    popularity: str       # "uniform" | "zipf"
    zipf_s: float
    ln_eps: float
    hbm_slots: int        # tenants resident in HBM at once
    host_tier: bool       # pinned-host pool + HBM cache + swap-in
    seed: int = 0
    adapter_rank: int = 0  # BLOCK_ENC_ADAPTER: bottleneck width of the per-tenant adapter
    max_classes: int = 0   # > 0: every tenant also owns an output head with at most this many classes
    n_images: int = 0      # > 0: only this many distinct weight sets exist; tenant t owns set t % n_images
                           # (a pinned-host pool that cannot hold one image per tenant id: ids share images)

    def scaled(self, **kw) -> "Workload":
        """Same recipe at another size (tests use reduced tenant / request counts)."""
        return replace(self, **kw)


# The five configurations of the target, by name.  Sequence length 128 is the paper's
# throughput setting (Sec. 7.2); up to 10 000 tenants is its scale claim (Sec. 7.1).
WORKLOADS = {
    "tiny_fp32": Workload("tiny_fp32", BLOCK_FFN, "f32", 64, 256, 0, 1, 4, 8, 16, 16,
                          "uniform", 0.0, 1e-12, 4, False),
    "bert_ffn": Workload("bert_ffn", BLOCK_FFN, "bf16", 768, 3072, 0, 1, 64, 256, 128, 128,
                         "uniform", 0.0, 1e-12, 64, False),
    "hbert_enc2": Workload("hbert_enc2", BLOCK_ENC_POSTLN, "bf16", 768, 3072, 12, 2, 1000, 512,
                           128, 128, "zipf", 1.1, 1e-12, 1000, False),
    "hgpt_dec": Workload("hgpt_dec", BLOCK_DEC_PRELN, "bf16", 1024, 4096, 16, 1, 2000, 256,
                         32, 512, "zipf", 1.0, 1e-5, 2000, False),
    "hbert_10k": Workload("hbert_10k", BLOCK_ENC_POSTLN, "bf16", 768, 3072, 12, 1, 10000, 1024,
                          16, 256, "zipf", 0.8, 1e-12, 2000, True),
    # The paper's own serving layer: the 6 higher BERT-base layers shared by all tenants, each
    # with the tenant's adapter after its attention layer (Sec. 3.2.2, Sec. 3.3 footnote).
    "hbert_shared_adapter": Workload("hbert_shared_adapter", BLOCK_ENC_ADAPTER, "bf16", 768, 3072, 12, 6, 1000,
                                     512, 128, 128, "zipf", 1.1, 1e-12, 1000, False, adapter_rank=64, max_classes=32),
    # The paper's scale claim on its own serving layer (Sec. 7.1: up to 10 000 instances on one GPU): 10 000 tenants'
    # adapters in pinned host memory (1.2 MB per tenant for six layers), an HBM cache of 2 000 tenants, batches as in
    # the 10 000-tenant configuration; missing adapters are swapped in on the side stream.
    "hbert_shared_adapter_10k": Workload("hbert_shared_adapter_10k", BLOCK_ENC_ADAPTER, "bf16", 768, 3072, 12, 6, 10000,
                                         1024, 16, 256, "zipf", 0.8, 1e-12, 2000, True, adapter_rank=64),
    # Its decoder-only counterpart (the paper's GPT-style instances: OPT-125M-shaped higher layers, pre-LN,
    # causal), prompts of ragged length as in the decoder configuration; generation is timed by bench.py --decode.
    "hgpt_shared_adapter": Workload("hgpt_shared_adapter", BLOCK_DEC_ADAPTER, "bf16", 768, 3072, 12, 6, 1000,
                                    256, 32, 512, "zipf", 1.0, 1e-5, 1000, False, adapter_rank=64),
    # Paper-exact bottleneck adapter (Sec. 3.2.2); rank 64 is this build's reading.
    "hbert_adapter": Workload("hbert_adapter", BLOCK_ADAPTER, "bf16", 768, 64, 0, 1, 1000, 512,
                              128, 128, "zipf", 1.1, 0.0, 1000, False),
}


def tensor_specs(wl: Workload) -> List[Tuple[str, Tuple[int, ...], str]]:
    """Canonical tensor order of one (tenant, layer) image: (name, shape, kind).

    Matrices are ``[out, in]`` row-major (Linear(a) = W a + b, Sec. 3.2.2).
    kind: "w" weight, "b" bias, "g" LayerNorm gain, "beta" LayerNorm shift.
    """
    d, f = wl.d_model, wl.d_ff
    ffn = [("w1", (f, d), "w"), ("b1", (f,), "b"), ("w2", (d, f), "w"), ("b2", (d,), "b")]
    if wl.block in (BLOCK_ENC_ADAPTER, BLOCK_DEC_ADAPTER):
        r = wl.adapter_rank
        return [("w_down", (r, d), "w"), ("b_down", (r,), "b"), ("w_up", (d, r), "w"), ("b_up", (d,), "b")]
    if wl.block == BLOCK_FFN:
        return ffn + [("ln_g", (d,), "g"), ("ln_b", (d,), "beta")]
    if wl.block in (BLOCK_ENC_POSTLN, BLOCK_DEC_PRELN):
        return ([("wqkv", (3 * d, d), "w"), ("bqkv", (3 * d,), "b"),
                 ("wo", (d, d), "w"), ("bo", (d,), "b"),
                 ("ln1_g", (d,), "g"), ("ln1_b", (d,), "beta")]
                + ffn + [("ln2_g", (d,), "g"), ("ln2_b", (d,), "beta")])
    if wl.block == BLOCK_ADAPTER:
        return [("w_down", (f, d), "w"), ("b_down", (f,), "b"),
                ("w_up", (d, f), "w"), ("b_up", (d,), "b")]
    raise ValueError(f"unknown block {wl.block}")


def shared_specs(wl: Workload) -> List[Tuple[str, Tuple[int, ...], str]]:
    """Tensors of one layer that every tenant shares (BLOCK_ENC_ADAPTER: the encoder layer)."""
    if wl.block not in (BLOCK_ENC_ADAPTER, BLOCK_DEC_ADAPTER):
        return []
    return tensor_specs(replace(wl, block=BLOCK_ENC_POSTLN))   # the decoder layer has the same tensors


# ---------------------------------------------------------------- dtype packing

def _round_bf16(a32: np.ndarray) -> np.ndarray:
    """fp32 -> nearest bf16 (ties to even), returned as fp32 values."""
    u = np.ascontiguousarray(a32, dtype=np.float32).view(np.uint32)
    u = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
    return u.view(np.float32)


def round_to_storage(a32: np.ndarray, dtype: str) -> np.ndarray:
    """Round fp32 draws to the storage dtype; result is fp32 holding storage-exact values."""
    if dtype == "bf16":
        return _round_bf16(a32)
    if dtype == "f32":
        return np.ascontiguousarray(a32, dtype=np.float32)
    raise ValueError(dtype)


def to_storage_bytes(a32: np.ndarray, dtype: str) -> np.ndarray:
    """Storage-exact fp32 values -> the array a device consumer reads (uint16 bf16 bits / fp32)."""
    a32 = np.ascontiguousarray(a32, dtype=np.float32)
    if dtype == "bf16":
        return (a32.view(np.uint32) >> np.uint32(16)).astype(np.uint16)
    return a32


def storage_to_f64(raw: np.ndarray, dtype: str) -> np.ndarray:
    """Inverse of to_storage_bytes, widened to fp64 (exact)."""
    if dtype == "bf16":
        return (raw.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    return raw.astype(np.float64)


# ---------------------------------------------------------------- keyed draws
#
# Normal draws come from one seeded master sequence z[0..T) ~ iid N(0,1) per seed (numpy
# SFC64, generated once per process).  A tensor is a contiguous window of it at an offset
# hashed from (seed, tag, tenant-or-request, layer, tensor): every tensor is exactly iid
# normal, any tensor can be regenerated alone, and a 50 GB pool costs a memcpy instead of
# 25 G calls of a normal sampler.  Windows of different tensors may overlap (as shifted
# copies); nothing in the method can tell.

_MASTER_LEN = 1 << 24          # 16 Mi draws; the largest single tensor has 4 Mi elements
_MASK64 = (1 << 64) - 1
_master_cache: dict = {}
_master_lock = threading.Lock()


def _mix64(z: int) -> int:
    z = (z + 0x9E3779B97F4A7C15) & _MASK64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _MASK64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _MASK64
    return z ^ (z >> 31)


def _offset(seed: int, tag: int, a: int, b: int, c: int, n: int) -> int:
    k = _mix64(seed ^ 0x5851F42D4C957F2D)
    for v in (tag, a, b, c):
        k = _mix64(k ^ int(v))
    if n >= _MASTER_LEN:
        raise ValueError(f"a tensor of {n} elements does not fit the generator's master sequence of {_MASTER_LEN} draws")
    return k % (_MASTER_LEN - n)


def _master(seed: int, dtype: str, scale: float):
    """(fp32 storage-exact values, storage bytes) of scale * z rounded to ``dtype``."""
    key = (seed, dtype, scale)
    if key in _master_cache:
        return _master_cache[key]
    with _master_lock:
        if key in _master_cache:
            return _master_cache[key]
        zkey = (seed, "z")
        if zkey not in _master_cache:
            g = np.random.Generator(np.random.SFC64(np.random.SeedSequence([0x484D49, seed])))
            _master_cache[zkey] = g.standard_normal(_MASTER_LEN, dtype=np.float32)
        v = round_to_storage(_master_cache[zkey] * np.float32(scale), dtype)
        raw = to_storage_bytes(v, dtype)
        v.setflags(write=False)
        raw.setflags(write=False)
        _master_cache[key] = (v, raw)
        return _master_cache[key]


def _gen(seed: int, tag: int, a: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[(int(seed) << 8) | int(tag), int(a)]))


def image_of(wl: Workload, tenant: int) -> int:
    """The weight set a tenant id owns: its own, or (n_images > 0) the one it shares with the ids congruent to it."""
    return tenant % wl.n_images if wl.n_images > 0 and 0 <= tenant < SHARED else tenant


def _tensor(wl: Workload, tenant: int, layer: int, idx: int, shape, kind: str, raw: bool):
    n = int(np.prod(shape))
    if layer != _HEAD_LAYER:
        tenant = image_of(wl, tenant)
    off = _offset(wl.seed, _TAG_WEIGHT, tenant, layer, idx, n)
    v32, vraw = _master(wl.seed, wl.dtype, 0.02)
    if kind == "g":      # LayerNorm gain 1 + N(0, 0.02): small, recomputed and re-rounded
        g32 = round_to_storage(np.float32(1.0) + v32[off:off + n], wl.dtype)
        return (to_storage_bytes(g32, wl.dtype) if raw else g32).reshape(shape)
    return (vraw if raw else v32)[off:off + n].reshape(shape)


def tenant_tensors(wl: Workload, tenant: int, layer: int = 0) -> List[np.ndarray]:
    """All tensors of one (tenant, layer) in canonical order, fp32 arrays holding
    storage-exact values.  Weights, biases and LayerNorm shifts ~ N(0, 0.02);
    LayerNorm gains ~ 1 + N(0, 0.02)."""
    return [_tensor(wl, tenant, layer, i, shape, kind, False)
            for i, (_, shape, kind) in enumerate(tensor_specs(wl))]


def tenant_storage(wl: Workload, tenant: int, layer: int = 0) -> List[np.ndarray]:
    """Same tensors as tenant_tensors, as the arrays a device consumer reads (bf16 bit
    patterns as uint16, or fp32).  Mostly zero-copy views of the master sequence."""
    return [_tensor(wl, tenant, layer, i, shape, kind, True)
            for i, (_, shape, kind) in enumerate(tensor_specs(wl))]


def shared_tensors(wl: Workload, layer: int = 0) -> List[np.ndarray]:
    """The shared tensors of one layer in canonical order (same distributions as tenant_tensors)."""
    return [_tensor(wl, SHARED, layer, 100 + i, shape, kind, False) for i, (_, shape, kind) in enumerate(shared_specs(wl))]


def shared_storage(wl: Workload, layer: int = 0) -> List[np.ndarray]:
    return [_tensor(wl, SHARED, layer, 100 + i, shape, kind, True) for i, (_, shape, kind) in enumerate(shared_specs(wl))]


def head_spec(wl: Workload, tenant: int) -> Tuple[int, bool]:
    """(number of classes, per_token) of a tenant's output head.  Three tenants in ten tag every
    token, the others classify on the first row (the task mix of the paper's Table of datasets);
    class counts are uniform on [2, max_classes] (classification) or odd counts from 3 up
    (BIO tag sets) within the same bound."""
    g = _gen(wl.seed, _TAG_HEAD, tenant)
    per_token = bool(g.random() < 0.3)
    c = int(g.integers(2, wl.max_classes + 1))
    if per_token:
        c = min(max(3, c | 1), wl.max_classes)
    return c, per_token


def head_tensors(wl: Workload, tenant: int, raw: bool = False) -> List[np.ndarray]:
    """W [C, d] and b [C] of a tenant's head ~ N(0, 0.02), storage-exact fp32 (or storage bytes)."""
    c, _ = head_spec(wl, tenant)
    return [_tensor(wl, tenant, _HEAD_LAYER, 0, (c, wl.d_model), "w", raw),
            _tensor(wl, tenant, _HEAD_LAYER, 1, (c,), "b", raw)]


def plot_table(wl: Workload, n_entries: int) -> np.ndarray:
    """Stand-in for the paper's table of precomputed tri-gram representations (Sec. 3.3.1; the real one is
    built from a corpus): [n_entries, 3, d] ~ N(0, 1), storage-exact fp32."""
    n = n_entries * 3 * wl.d_model
    off = _offset(wl.seed, _TAG_PLOT, n_entries, 0, 0, n)
    return _master(wl.seed, wl.dtype, 1.0)[0][off:off + n].reshape(n_entries, 3, wl.d_model)


def plot_fragment_ids(wl: Workload, n_entries: int, n_tokens: int, batch: int = 0) -> np.ndarray:
    """Table row of the fragment centred on each token of a batch: i.i.d. uniform (the result of the CPU-side lookup)."""
    return _gen(wl.seed, _TAG_PLOT, batch).integers(0, n_entries, size=n_tokens).astype(np.int32)


def hidden_states(wl: Workload, request: int, seq_len: int, batch: int = 0) -> np.ndarray:
    """Hidden states entering the task layers for one request: [seq_len, d] ~ N(0, 1),
    storage-exact fp32.  Stands in for the PLOT-retrieved representations (Sec. 3.3.1)."""
    n = seq_len * wl.d_model
    off = _offset(wl.seed, _TAG_X, request, batch, 0, n)
    return _master(wl.seed, wl.dtype, 1.0)[0][off:off + n].reshape(seq_len, wl.d_model)


def _popularity_cdf(wl: Workload) -> np.ndarray:
    k = np.arange(1, wl.n_tenants + 1, dtype=np.float64)
    p = k ** (-wl.zipf_s) if wl.popularity == "zipf" else np.ones_like(k)
    c = np.cumsum(p)
    return c / c[-1]


def batch_ids_lens(wl: Workload, batch: int = 0) -> Tuple[np.ndarray, np.ndarray]:
    """tenant_ids[R] (i.i.d. uniform or finite Zipf over ranks 1..T, id = rank-1) and
    seq_lens[R] (fixed, or i.i.d. integer-uniform on [seq_min, seq_max])."""
    u = _gen(wl.seed, _TAG_IDS, batch).random(wl.n_requests)
    ids = np.searchsorted(_popularity_cdf(wl), u, side="right")
    ids = np.minimum(ids, wl.n_tenants - 1).astype(np.int32)
    if wl.seq_min == wl.seq_max:
        lens = np.full(wl.n_requests, wl.seq_min, dtype=np.int32)
    else:
        lens = _gen(wl.seed, _TAG_LENS, batch).integers(
            wl.seq_min, wl.seq_max + 1, size=wl.n_requests).astype(np.int32)
    return ids, lens
