"""Seeded synthetic inputs for the mixed-tenant layer forward.

This package only *draws numbers and shapes*: tenant weights, hidden states,
tenant ids and sequence lengths.  It contains none of the method's arithmetic
(no matmul, softmax, GELU, LayerNorm, sorting by tenant).  Both the CPU oracle's
tests and the GPU path's tests/bench take their inputs from here, and nothing
else is shared between the two.
"""
from .inputs import (  # noqa: F401
    BLOCK_FFN, BLOCK_ENC_POSTLN, BLOCK_DEC_PRELN, BLOCK_ADAPTER, BLOCK_ENC_ADAPTER, BLOCK_DEC_ADAPTER,
    shared_specs, shared_tensors, shared_storage, head_spec, head_tensors, plot_table, plot_fragment_ids,
    Workload, WORKLOADS, tensor_specs, tenant_tensors, tenant_storage, hidden_states, batch_ids_lens,
    round_to_storage, to_storage_bytes, storage_to_f64, image_of,
)
