"""Glue between the seeded input generators (synth/) and the HIP library: builds a pool
for a workload, loads generated tenants into it and moves generated batches to the GPU.
Product-side only: it never touches the CPU oracle."""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from typing import Iterable, Optional, Tuple

import numpy as np
import torch

import synth
from . import HMI_BF16, HMI_F32, Pool


def create_pool(wl: synth.Workload, *, max_requests: Optional[int] = None,
                max_tokens: Optional[int] = None, device: int = 0,
                hbm_slots: Optional[int] = None) -> Pool:
    R = max_requests or wl.n_requests
    stream = torch.cuda.current_stream(device).cuda_stream
    return Pool(block=wl.block, dtype=HMI_BF16 if wl.dtype == "bf16" else HMI_F32,
                d_model=wl.d_model, d_ff=wl.d_ff, n_heads=wl.n_heads, n_layers=wl.n_layers,
                max_tenants=wl.n_tenants, hbm_slots=hbm_slots or wl.hbm_slots,
                host_tier=wl.host_tier, max_requests=R, max_tokens=max_tokens or R * wl.seq_max,
                ln_eps=wl.ln_eps, device=device, compute_stream=stream, adapter_rank=wl.adapter_rank, max_classes=wl.max_classes)


def load_tenants(pool: Pool, wl: synth.Workload, tenants: Optional[Iterable[int]] = None,
                 workers: int = 8) -> None:
    """Generate and register every (tenant, layer) of ``tenants`` (default: all)."""
    tenants = list(range(wl.n_tenants)) if tenants is None else list(tenants)
    if synth.shared_specs(wl):
        for l in range(wl.n_layers):
            pool.load_shared(l, synth.shared_storage(wl, l))
    if wl.max_classes:
        for t in tenants:
            w, b = synth.head_tensors(wl, t, raw=True)
            pool.load_head(t, w, b, synth.head_spec(wl, t)[1])
    # tenants that share another tenant's weight set (wl.n_images > 0) are created from it after it is loaded
    owners = sorted({synth.image_of(wl, t) for t in tenants})
    sharers = [t for t in tenants if synth.image_of(wl, t) != t]
    todo = [(t, l) for t in owners
            for l in range(wl.n_layers)]

    def gen(tl):
        t, l = tl
        return t, l, synth.tenant_storage(wl, t, l)

    with ThreadPoolExecutor(workers) as ex:
        for t, l, tensors in ex.map(gen, todo):
            pool.load_tenant(t, l, tensors)
    for t in sharers:
        pool.alias_tenant(t, synth.image_of(wl, t))


def batch_to_device(wl: synth.Workload, batch: int = 0, device: int = 0
                    ) -> Tuple[np.ndarray, np.ndarray, torch.Tensor]:
    """-> tenant_ids, seq_lens (host int32) and x [N, d] on the GPU in the storage dtype."""
    ids, lens = synth.batch_ids_lens(wl, batch)
    with ThreadPoolExecutor(8) as ex:
        rows = list(ex.map(lambda r: synth.hidden_states(wl, r, int(lens[r]), batch), range(len(ids))))
    x = np.concatenate(rows, axis=0)
    return ids, lens, host_to_device(x, wl.dtype, device)


def host_to_device(a32: np.ndarray, dtype: str, device: int = 0) -> torch.Tensor:
    """Storage-exact fp32 host array -> device tensor in the storage dtype."""
    raw = synth.to_storage_bytes(a32, dtype)
    if dtype == "bf16":
        return torch.from_numpy(raw.view(np.int16)).view(torch.bfloat16).to(f"cuda:{device}")
    return torch.from_numpy(np.array(raw, copy=True)).to(f"cuda:{device}")


def device_to_f64(y: torch.Tensor) -> np.ndarray:
    return y.detach().to("cpu", torch.float64).numpy()
