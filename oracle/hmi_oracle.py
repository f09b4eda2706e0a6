"""fp64 CPU oracle for the mixed-tenant forward of per-tenant transformer layers.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this module; it is
called by the tests, by the smoke check and by the benchmark's CPU-baseline leg.  It
shares no code with the HIP library and imports nothing from it.

What it computes (HMI, Sec. 6.3 "Parallel Inference of Adapters"): a batch holds
independent requests of different tenants, and every request is transformed with its
own tenant's parameters.  The paper realises that with stacked parameters and a batched
matrix multiplication; the result it reaches is exactly "each request through its own
tenant's block", so the oracle is that definition written out as a loop over requests.
The per-tenant block is built from the paper's Linear(a) = W a + b and the residual
shape of its adapter A(a) = Up(phi(Down(a))) + a (Sec. 3.2.2); for the whole-FFN and
whole-layer blocks the paper defers to BERT / GPT, whose sub-layer equations are used
(post-LN encoder: LN after each residual; pre-LN decoder: LN before each sub-layer,
causal attention; for the shared layer with a per-tenant adapter after the attention
layer the paper's own description of its fine-tuned layer, Sec. 3.2.2; exact erf GELU; biased-variance LayerNorm; softmax scaled by
1/sqrt(d_head), never across requests, no padding keys).

All arithmetic is numpy fp64; ``@`` (matmul) and ``scipy.special.erf`` are the only
library primitives used as steps.  No blocking, fusion or reordering.

Pins (tests/test_oracle_*.py): hand-worked tiny cases, closed forms (uniform attention,
LayerNorm moments, GELU identities, S = 1 collapse), the spec invariants, PyTorch
CPU fp64 library layers for the single-tenant special case, and an O(R^2) rank count
for the router.  No function here is "parity unpinned".
"""
from __future__ import annotations

import math
from typing import Callable, Dict, List, Sequence

import numpy as np
from scipy.special import erf as _erf

BLOCK_FFN = 0
BLOCK_ENC_POSTLN = 1
BLOCK_DEC_PRELN = 2
BLOCK_ADAPTER = 3
BLOCK_ENC_ADAPTER = 4
BLOCK_DEC_ADAPTER = 5


# --------------------------------------------------------------------------- router

def route(tenant_ids: Sequence[int], seq_lens: Sequence[int]) -> Dict[str, np.ndarray]:
    """Group a batch's requests by tenant (the "stack the parameters per request" step of
    Sec. 6.3, done by ordering requests instead of copying parameters).

    perm         stable ordering of request indices by tenant id (ties keep arrival order)
    tok_off      [R+1] exclusive prefix sum of seq_lens in ORIGINAL order
    seg_tenant   [G]   tenant of each maximal run of equal ids in the sorted order
    seg_req_off  [G+1] run boundaries in sorted request positions
    seg_tok_off  [G+1] run boundaries in tokens of the sorted order
    """
    R = len(tenant_ids)
    tok_off = [0] * (R + 1)
    for r in range(R):
        tok_off[r + 1] = tok_off[r] + int(seq_lens[r])
    perm = sorted(range(R), key=lambda r: int(tenant_ids[r]))  # Python's sort is stable
    seg_tenant: List[int] = []
    seg_req_off: List[int] = []
    seg_tok_off: List[int] = []
    tokens = 0
    for p, r in enumerate(perm):
        if p == 0 or int(tenant_ids[r]) != int(tenant_ids[perm[p - 1]]):
            seg_tenant.append(int(tenant_ids[r]))
            seg_req_off.append(p)
            seg_tok_off.append(tokens)
        tokens += int(seq_lens[r])
    seg_req_off.append(R)
    seg_tok_off.append(tokens)
    i32 = lambda a: np.asarray(a, dtype=np.int32)  # noqa: E731
    return {"perm": i32(perm), "tok_off": i32(tok_off), "seg_tenant": i32(seg_tenant),
            "seg_req_off": i32(seg_req_off), "seg_tok_off": i32(seg_tok_off)}


# --------------------------------------------------------------------------- pieces

def linear(a: np.ndarray, W: np.ndarray, b: np.ndarray) -> np.ndarray:
    """Linear(a) = W a + b for every row a of ``a`` (Sec. 3.2.2); W is [out, in]."""
    return a @ W.T + b


def gelu(x: np.ndarray) -> np.ndarray:
    """Exact GELU x * Phi(x) with Phi the standard normal CDF (BERT's activation)."""
    return x * 0.5 * (1.0 + _erf(x / math.sqrt(2.0)))


def relu(x: np.ndarray) -> np.ndarray:
    """phi of the paper's adapter (Sec. 3.2.2)."""
    return np.maximum(x, 0.0)


def layer_norm(x: np.ndarray, g: np.ndarray, b: np.ndarray, eps: float) -> np.ndarray:
    """Row LayerNorm with the biased variance: (x - mean) / sqrt(var + eps) * g + b."""
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    return (x - mu) / np.sqrt(var + eps) * g + b


def softmax_rows(s: np.ndarray) -> np.ndarray:
    m = s.max(axis=-1, keepdims=True)
    e = np.exp(s - m)
    return e / e.sum(axis=-1, keepdims=True)


def attention(a: np.ndarray, w: Dict[str, np.ndarray], n_heads: int, causal: bool) -> np.ndarray:
    """Multi-head self-attention over ONE request's rows ``a`` [S, d], output projection
    included.  Packed QKV weight [3d, d] in q, k, v order; head h owns columns
    h*d_head .. (h+1)*d_head.  causal: query i sees keys j <= i."""
    S, d = a.shape
    dh = d // n_heads
    qkv = linear(a, w["wqkv"], w["bqkv"])
    q, k, v = qkv[:, :d], qkv[:, d:2 * d], qkv[:, 2 * d:]
    ctx = np.empty((S, d), dtype=np.float64)
    for h in range(n_heads):
        sl = slice(h * dh, (h + 1) * dh)
        s = (q[:, sl] @ k[:, sl].T) / math.sqrt(dh)
        if causal:
            s = np.where(np.arange(S)[None, :] <= np.arange(S)[:, None], s, -np.inf)
        ctx[:, sl] = softmax_rows(s) @ v[:, sl]
    return linear(ctx, w["wo"], w["bo"])


def ffn(a: np.ndarray, w: Dict[str, np.ndarray]) -> np.ndarray:
    return linear(gelu(linear(a, w["w1"], w["b1"])), w["w2"], w["b2"])


# --------------------------------------------------------------------------- blocks

def ffn_block(x, w, eps):
    """Y = LN(X + W2 GELU(W1 X + b1) + b2): the adapter's residual shape (Sec. 3.2.2)
    widened to a BERT feed-forward sub-layer with its LayerNorm."""
    return layer_norm(x + ffn(x, w), w["ln_g"], w["ln_b"], eps)


def encoder_postln(x, w, n_heads, eps):
    x1 = layer_norm(x + attention(x, w, n_heads, causal=False), w["ln1_g"], w["ln1_b"], eps)
    return layer_norm(x1 + ffn(x1, w), w["ln2_g"], w["ln2_b"], eps)


def decoder_preln(x, w, n_heads, eps):
    x1 = x + attention(layer_norm(x, w["ln1_g"], w["ln1_b"], eps), w, n_heads, causal=True)
    return x1 + ffn(layer_norm(x1, w["ln2_g"], w["ln2_b"], eps), w)


def adapter_block(x, w):
    """A(a) = Linear_up(ReLU(Linear_down(a))) + a  (Sec. 3.2.2)."""
    return linear(relu(linear(x, w["w_down"], w["b_down"])), w["w_up"], w["b_up"]) + x


def encoder_postln_adapter(x, w, n_heads, eps):
    """The paper's task-adapted higher layer (Sec. 3.2.2, architecture figure (c)): a BERT
    post-LN encoder layer whose parameters are shared by every tenant, with the tenant's
    adapter injected after the attention layer.  The adapter A(a) = Up(ReLU(Down(a))) + a
    acts on the attention layer's output a (output projection included) before the
    residual connection and its LayerNorm; the feed-forward half is the plain shared one."""
    a = attention(x, w, n_heads, causal=False)
    x1 = layer_norm(x + adapter_block(a, w), w["ln1_g"], w["ln1_b"], eps)
    return layer_norm(x1 + ffn(x1, w), w["ln2_g"], w["ln2_b"], eps)


def decoder_preln_adapter(x, w, n_heads, eps):
    """The same task-adapted layer for the paper's decoder-only instances (Sec. 3.2.2 places the
    adapter after the attention layer of each higher layer; its GPT-style backbone is a pre-LN
    decoder): a = Attention(LN1(x)) with the causal mask, x1 = x + A(a), y = x1 + FFN(LN2(x1));
    everything but the adapter A is shared by all tenants."""
    a = attention(layer_norm(x, w["ln1_g"], w["ln1_b"], eps), w, n_heads, causal=True)
    x1 = x + adapter_block(a, w)
    return x1 + ffn(layer_norm(x1, w["ln2_g"], w["ln2_b"], eps), w)


def block_forward(block: int, x: np.ndarray, w: Dict[str, np.ndarray], n_heads: int,
                  eps: float) -> np.ndarray:
    """One request's rows through one tenant's block."""
    if block == BLOCK_FFN:
        return ffn_block(x, w, eps)
    if block == BLOCK_ENC_POSTLN:
        return encoder_postln(x, w, n_heads, eps)
    if block == BLOCK_DEC_PRELN:
        return decoder_preln(x, w, n_heads, eps)
    if block == BLOCK_ADAPTER:
        return adapter_block(x, w)
    if block == BLOCK_ENC_ADAPTER:
        return encoder_postln_adapter(x, w, n_heads, eps)
    if block == BLOCK_DEC_ADAPTER:
        return decoder_preln_adapter(x, w, n_heads, eps)
    raise ValueError(f"unknown block {block}")


# --------------------------------------------------------------------------- the path

def layer_forward(block: int, X: np.ndarray, tenant_ids: Sequence[int], seq_lens: Sequence[int],
                  weights_of: Callable[[int], Dict[str, np.ndarray]], n_heads: int = 0,
                  eps: float = 1e-12, requests: Sequence[int] | None = None) -> np.ndarray:
    """Mixed-tenant forward of one layer (Sec. 6.3): X is [N, d] packed in request order
    (N = sum(seq_lens), no padding rows); request r's rows go through tenant
    tenant_ids[r]'s parameters, ``weights_of(tenant)`` -> {name: fp64 array}.

    ``requests``: compute only these requests (requests are independent); other rows of
    the result are NaN.
    """
    X = np.asarray(X, dtype=np.float64)
    R = len(tenant_ids)
    Y = np.full_like(X, np.nan)
    start = 0
    todo = set(range(R)) if requests is None else set(int(r) for r in requests)
    for r in range(R):
        S = int(seq_lens[r])
        if r in todo:
            w = weights_of(int(tenant_ids[r]))
            Y[start:start + S] = block_forward(block, X[start:start + S], w, n_heads, eps)
        start += S
    return Y


# --------------------------------------------------------------------------- output heads

def head_forward(H: np.ndarray, tenant_ids: Sequence[int], seq_lens: Sequence[int],
                 head_of: Callable[[int], tuple], max_classes: int):
    """Per-tenant output heads on the final hidden states H [N, d] (Sec. 3.3.2): every tenant
    owns one linear layer (W [C, d], b [C]) with its own number of classes C.  A
    classification tenant is scored on the first row of each of its requests (the [CLS]
    token at the beginning of the sentence), a tagging tenant on every row; the predicted
    label is the class with the highest score (the lowest such index on ties).

    ``head_of(tenant)`` -> (W, b, per_token).  Returns (scores [N, max_classes] with -inf
    where there is no class or no prediction, labels [N] with -1 where there is no prediction).
    """
    H = np.asarray(H, dtype=np.float64)
    N = H.shape[0]
    scores = np.full((N, max_classes), -np.inf)
    labels = np.full(N, -1, dtype=np.int64)
    start = 0
    for r in range(len(tenant_ids)):
        S = int(seq_lens[r])
        W, b, per_token = head_of(int(tenant_ids[r]))
        rows = range(start, start + S) if per_token else range(start, start + 1)
        for i in rows:
            sc = linear(H[i], np.asarray(W, dtype=np.float64), np.asarray(b, dtype=np.float64))
            scores[i, :len(sc)] = sc
            labels[i] = int(np.argmax(sc))      # first index of the maximum
        start += S
    return scores, labels


# --------------------------------------------------------------------------- representation retrieval

def plot_aggregate(table: np.ndarray, frag_ids: Sequence[int], seq_lens: Sequence[int]) -> np.ndarray:
    """Aggregate of Sec. 3.3.1: the input is swept into three-token fragments X_i = [x_{i-1}, x_i,
    x_{i+1}], one centred on every token, whose precomputed representations H_i (3 x d) were looked up
    in the table (``frag_ids[i]`` is the table row of X_i; ``table`` is [entries, 3, d]).  A token's
    representation is the normalised sum of its representations in the fragments that contain it:
    token i is the third token of X_{i-1}, the second of X_i and the first of X_{i+1}; fragments do
    not reach across requests, so the first and last token of a request appear in two fragments (a
    one-token request in one).  Normalised = divided by the number of summands."""
    table = np.asarray(table, dtype=np.float64)
    N = int(np.sum(seq_lens))
    out = np.zeros((N, table.shape[2]))
    start = 0
    for n in seq_lens:
        n = int(n)
        for i in range(n):
            parts = [table[int(frag_ids[start + i]), 1]]
            if i > 0:
                parts.append(table[int(frag_ids[start + i - 1]), 2])
            if i < n - 1:
                parts.append(table[int(frag_ids[start + i + 1]), 0])
            out[start + i] = sum(parts) / len(parts)
        start += n
    return out
