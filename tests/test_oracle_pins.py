"""Pins for the fp64 oracle: every check compares it with something that is NOT the
oracle — hand-worked numbers, closed forms, scalar brute force written index by index,
PyTorch-CPU fp64 library layers, or invariants of the problem statement (Sec. 6.3:
independent requests, each with its own tenant's parameters)."""
import json
import math
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import hmi_oracle as O

GOLD = os.path.join(os.path.dirname(__file__), "golden")
PHI1 = 0.8413447460685429  # standard normal CDF at 1 (textbook table value)


def rnd(seed, *shape, scale=1.0):
    return np.random.default_rng(seed).standard_normal(shape) * scale


def enc_weights(seed, d, f, scale=0.3):
    r = np.random.default_rng(seed)
    n = lambda *s: r.standard_normal(s) * scale  # noqa: E731
    return {"wqkv": n(3 * d, d), "bqkv": n(3 * d), "wo": n(d, d), "bo": n(d),
            "ln1_g": 1 + n(d), "ln1_b": n(d), "w1": n(f, d), "b1": n(f),
            "w2": n(d, f), "b2": n(d), "ln2_g": 1 + n(d), "ln2_b": n(d)}


def ffn_weights(seed, d, f, scale=0.3):
    r = np.random.default_rng(seed)
    n = lambda *s: r.standard_normal(s) * scale  # noqa: E731
    return {"w1": n(f, d), "b1": n(f), "w2": n(d, f), "b2": n(d), "ln_g": 1 + n(d), "ln_b": n(d)}


# ------------------------------------------------------------------ scalar brute force
# Written index by index from the definitions, with Python floats and math.* only.

def bf_linear(a, W, b):
    return [[sum(W[o][i] * row[i] for i in range(len(row))) + b[o] for o in range(len(W))]
            for row in a]


def bf_gelu(v):
    return v * 0.5 * (1.0 + math.erf(v / math.sqrt(2.0)))


def bf_ln(row, g, b, eps):
    n = len(row)
    mu = sum(row) / n
    var = sum((v - mu) * (v - mu) for v in row) / n
    return [(row[i] - mu) / math.sqrt(var + eps) * g[i] + b[i] for i in range(n)]


def bf_attention(a, w, h, causal):
    S, d = len(a), len(a[0])
    dh = d // h
    qkv = bf_linear(a, w["wqkv"], w["bqkv"])
    ctx = [[0.0] * d for _ in range(S)]
    for head in range(h):
        for i in range(S):
            keys = range(i + 1) if causal else range(S)
            sc = {j: sum(qkv[i][head * dh + c] * qkv[j][d + head * dh + c] for c in range(dh))
                  / math.sqrt(dh) for j in keys}
            m = max(sc.values())
            den = sum(math.exp(v - m) for v in sc.values())
            for c in range(dh):
                ctx[i][head * dh + c] = sum(math.exp(sc[j] - m) / den * qkv[j][2 * d + head * dh + c]
                                            for j in keys)
    return bf_linear(ctx, w["wo"], w["bo"])


def bf_ffn(a, w):
    hid = [[bf_gelu(v) for v in row] for row in bf_linear(a, w["w1"], w["b1"])]
    return bf_linear(hid, w["w2"], w["b2"])


def bf_add(a, b):
    return [[x + y for x, y in zip(ra, rb)] for ra, rb in zip(a, b)]


def bf_block(block, a, w, h, eps):
    if block == O.BLOCK_FFN:
        return [bf_ln(r, w["ln_g"], w["ln_b"], eps) for r in bf_add(a, bf_ffn(a, w))]
    if block == O.BLOCK_ENC_POSTLN:
        x1 = [bf_ln(r, w["ln1_g"], w["ln1_b"], eps) for r in bf_add(a, bf_attention(a, w, h, False))]
        return [bf_ln(r, w["ln2_g"], w["ln2_b"], eps) for r in bf_add(x1, bf_ffn(x1, w))]
    if block == O.BLOCK_DEC_PRELN:
        n1 = [bf_ln(r, w["ln1_g"], w["ln1_b"], eps) for r in a]
        x1 = bf_add(a, bf_attention(n1, w, h, True))
        n2 = [bf_ln(r, w["ln2_g"], w["ln2_b"], eps) for r in x1]
        return bf_add(x1, bf_ffn(n2, w))
    raise AssertionError


def as_lists(w):
    return {k: v.tolist() for k, v in w.items()}


# ------------------------------------------------------------------ scalar functions

def test_gelu_closed_forms():
    assert O.gelu(np.array([0.0]))[0] == 0.0
    assert O.gelu(np.array([1.0]))[0] == pytest.approx(PHI1, abs=1e-15)
    assert O.gelu(np.array([-1.0]))[0] == pytest.approx(PHI1 - 1.0, abs=1e-15)
    x = np.linspace(-6, 6, 97)
    np.testing.assert_allclose(O.gelu(-x), O.gelu(x) - x, atol=1e-14)   # GELU(-x) = GELU(x) - x
    assert O.gelu(np.array([40.0]))[0] == 40.0                            # -> x
    assert abs(O.gelu(np.array([-40.0]))[0]) < 1e-300                     # -> 0
    np.testing.assert_allclose(O.gelu(x), F.gelu(torch.tensor(x)).numpy(), rtol=0, atol=1e-15)
    # the tanh approximation is a different function: make sure we are not it
    assert abs(O.gelu(np.array([2.0]))[0] - F.gelu(torch.tensor([2.0], dtype=torch.float64),
                                                    approximate="tanh").item()) > 5e-5


def test_layer_norm_hand_and_moments():
    # by hand: x = [1,3], mean 2, biased var 1 -> [-1, 1]; gain [2,3], shift [.5,-.5]
    y = O.layer_norm(np.array([[1.0, 3.0]]), np.array([2.0, 3.0]), np.array([0.5, -0.5]), 0.0)
    np.testing.assert_allclose(y, [[-1.5, 2.5]], atol=1e-15)
    # by hand: x = [0,0,3,5]: mean 2, var (4+4+1+9)/4 = 4.5; eps 0.5 -> divide by sqrt(5)
    y = O.layer_norm(np.array([[0.0, 0.0, 3.0, 5.0]]), np.ones(4), np.zeros(4), 0.5)
    np.testing.assert_allclose(y, np.array([[-2, -2, 1, 3]]) / math.sqrt(5.0), atol=1e-15)
    x = rnd(1, 7, 33, scale=3.0) + 1.5
    eps = 1e-3
    y = O.layer_norm(x, np.ones(33), np.zeros(33), eps)
    var = x.var(axis=1)  # numpy default ddof=0 = biased
    np.testing.assert_allclose(y.mean(axis=1), 0, atol=1e-14)
    np.testing.assert_allclose(y.var(axis=1), var / (var + eps), rtol=1e-12)
    g, b = rnd(2, 33), rnd(3, 33)
    np.testing.assert_allclose(
        O.layer_norm(x, g, b, eps),
        F.layer_norm(torch.tensor(x), (33,), torch.tensor(g), torch.tensor(b), eps).numpy(),
        atol=1e-13)


def test_linear_is_W_a_plus_b_not_transposed():
    # Linear(a) = W a + b with W [out,in]: a = [1,2], W = [[1,0],[0,1],[1,1]], b = [10,20,30]
    y = O.linear(np.array([[1.0, 2.0]]), np.array([[1.0, 0], [0, 1], [1, 1]]), np.array([10.0, 20, 30]))
    np.testing.assert_array_equal(y, [[11.0, 22.0, 33.0]])


def test_softmax_rows_hand():
    p = O.softmax_rows(np.array([[0.0, math.log(3.0)], [1000.0, 1000.0]]))
    np.testing.assert_allclose(p, [[0.25, 0.75], [0.5, 0.5]], atol=1e-15)


# ------------------------------------------------------------------ hand-worked blocks

def test_ffn_block_hand_worked():
    """d=4, f=2.  x=[2,0,-2,0]; W1 picks 0.5*x0 and -0.5*x2 -> h=[1,1] -> GELU=[p,p], p=Phi(1);
    W2 maps to [p,p,0,2p]; z = x + . = [2+p, p, -2, 2p]; mean = p; deviations [2,0,-2-p,p]."""
    with open(os.path.join(GOLD, "ffn_hand_d4.json")) as fh:
        gold = json.load(fh)
    w = {k: np.array(v, dtype=np.float64) for k, v in gold["weights"].items()}
    y = O.ffn_block(np.array(gold["x"], dtype=np.float64), w, gold["eps"])
    np.testing.assert_allclose(y, np.array(gold["y"]), atol=1e-14)
    # the same numbers re-derived here from the closed form in the docstring
    p = PHI1
    dev = np.array([2.0, 0.0, -2.0 - p, p])
    sd = math.sqrt((4 + (2 + p) ** 2 + p * p) / 4)
    np.testing.assert_allclose(y[0], dev / sd * np.array([1, 2, 1, 1]) + np.array([0, 0, 0.5, 0]),
                               atol=1e-14)


def test_adapter_block_hand_worked():
    # A(a) = Up(ReLU(Down(a))) + a, Sec. 3.2.2.  a=[1,-2,3]; Down=[[1,1,0],[0,1,0]] b=[0,.5]
    # -> [-1,-1.5] -> ReLU [0,0] -> Up(.)=b_up=[.1,.2,.3] -> [1.1,-1.8,3.3]
    w = {"w_down": np.array([[1.0, 1, 0], [0, 1, 0]]), "b_down": np.array([0.0, 0.5]),
         "w_up": np.array([[1.0, 2], [3, 4], [5, 6]]), "b_up": np.array([0.1, 0.2, 0.3])}
    np.testing.assert_allclose(O.adapter_block(np.array([[1.0, -2, 3]]), w), [[1.1, -1.8, 3.3]],
                               atol=1e-15)
    # a=[1,2,3] -> Down=[3,2.5] -> Up = [3+5+.1, 9+10+.2, 15+15+.3] -> + a
    np.testing.assert_allclose(O.adapter_block(np.array([[1.0, 2, 3]]), w), [[9.1, 21.2, 33.3]],
                               atol=1e-13)


def adapter_weights(seed, d, r, scale=0.3):
    g = np.random.default_rng(seed)
    n = lambda *s: g.standard_normal(s) * scale  # noqa: E731
    return {"w_down": n(r, d), "b_down": n(r), "w_up": n(d, r), "b_up": n(d)}


def test_shared_layer_with_adapter_hand_worked():
    """Sec. 3.2.2: the adapter sits after the attention layer, on that layer's output, inside the
    residual.  One token (softmax of one score is 1), d = 2, identity value / output matrices:
      a   = Wo (Wv x + bv) + bo = x + bo = [1,2] + [1,-1] = [2,1]
      A(a)= a + Up ReLU(Down a) = [2,1] + [2,3]*ReLU(2-1) + [0.5,0] = [4.5,4]
      x1  = LN1(x + A(a)) = LN([5.5,6]) = [-1,1]            (gain 1, shift 0, eps 0)
      y   = LN2(x1 + b2) = LN([-1,1] + [1,3]) = LN([0,4]) = [-1,1] * [2,3] + [0.5,-0.5] = [-1.5,2.5]
    (W1 = 0, b1 = 0 make the feed-forward half output b2.)  With Down = [-1,1] the ReLU closes:
      A(a) = [2.5,1]; x + A(a) = [3.5,3] -> x1 = [1,-1]; + [1,3] = [2,2]: use b2 = [1,4] -> [2,3] -> y = [-1.5,2.5]."""
    I, Z = np.eye(2), np.zeros((2, 2))
    w = {"wqkv": np.vstack([Z, Z, I]), "bqkv": np.zeros(6), "wo": I, "bo": np.array([1.0, -1.0]),
         "ln1_g": np.ones(2), "ln1_b": np.zeros(2), "w1": np.zeros((3, 2)), "b1": np.zeros(3),
         "w2": np.zeros((2, 3)), "b2": np.array([1.0, 3.0]), "ln2_g": np.array([2.0, 3.0]), "ln2_b": np.array([0.5, -0.5]),
         "w_down": np.array([[1.0, -1.0]]), "b_down": np.zeros(1), "w_up": np.array([[2.0], [3.0]]),
         "b_up": np.array([0.5, 0.0])}
    x = np.array([[1.0, 2.0]])
    np.testing.assert_allclose(O.encoder_postln_adapter(x, w, 1, 0.0), [[-1.5, 2.5]], rtol=0, atol=1e-14)
    w2 = dict(w, w_down=np.array([[-1.0, 1.0]]), b2=np.array([1.0, 4.0]))
    np.testing.assert_allclose(O.encoder_postln_adapter(x, w2, 1, 0.0), [[-1.5, 2.5]], rtol=0, atol=1e-14)


@pytest.mark.parametrize("S", [1, 5])
def test_shared_layer_with_adapter_against_scalar_brute_force(S):
    d, f, r, h = 4, 6, 3, 2
    w = dict(enc_weights(31 + S, d, f, 0.7), **adapter_weights(41 + S, d, r, 0.7))
    x = rnd(51 + S, S, d)
    wl, xl = as_lists(w), x.tolist()
    a = bf_attention(xl, wl, h, False)
    mid = [[max(v, 0.0) for v in row] for row in bf_linear(a, wl["w_down"], wl["b_down"])]
    a2 = bf_add(a, bf_linear(mid, wl["w_up"], wl["b_up"]))
    x1 = [bf_ln(row, wl["ln1_g"], wl["ln1_b"], 1e-12) for row in bf_add(xl, a2)]
    want = [bf_ln(row, wl["ln2_g"], wl["ln2_b"], 1e-12) for row in bf_add(x1, bf_ffn(x1, wl))]
    np.testing.assert_allclose(O.encoder_postln_adapter(x, w, h, 1e-12), want, rtol=1e-11, atol=1e-12)


def test_shared_layer_with_silent_adapter_is_the_plain_encoder_layer():
    """Up = 0, b_up = 0: A(a) = a, so the layer is the shared encoder layer itself, which the
    library-layer pin covers; a tenant whose up-projection is not zero differs."""
    d, f, r, h = 8, 16, 4, 2
    w = dict(enc_weights(7, d, f), **adapter_weights(8, d, r))
    x = rnd(9, 6, d)
    quiet = dict(w, w_up=np.zeros((d, r)), b_up=np.zeros(d))
    assert np.array_equal(O.encoder_postln_adapter(x, quiet, h, 1e-12), O.encoder_postln(x, w, h, 1e-12))
    assert np.abs(O.encoder_postln_adapter(x, w, h, 1e-12) - O.encoder_postln(x, w, h, 1e-12)).max() > 1e-3
    # through the batch loop: two tenants share the layer and differ only in their adapters
    bank = {0: quiet, 1: w}
    Y = O.layer_forward(O.BLOCK_ENC_ADAPTER, np.concatenate([x, x]), [1, 0], [6, 6], lambda t: bank[t], h, 1e-12)
    assert np.array_equal(Y[6:], O.encoder_postln(x, w, h, 1e-12))
    assert np.array_equal(Y[:6], O.encoder_postln_adapter(x, w, h, 1e-12))


@pytest.mark.parametrize("S", [1, 5])
def test_shared_decoder_layer_with_adapter_against_scalar_brute_force(S):
    d, f, r, h = 4, 6, 3, 2
    w = dict(enc_weights(61 + S, d, f, 0.7), **adapter_weights(71 + S, d, r, 0.7))
    x = rnd(81 + S, S, d)
    wl, xl = as_lists(w), x.tolist()
    n1 = [bf_ln(row, wl["ln1_g"], wl["ln1_b"], 1e-5) for row in xl]
    a = bf_attention(n1, wl, h, True)
    mid = [[max(v, 0.0) for v in row] for row in bf_linear(a, wl["w_down"], wl["b_down"])]
    x1 = bf_add(xl, bf_add(a, bf_linear(mid, wl["w_up"], wl["b_up"])))
    n2 = [bf_ln(row, wl["ln2_g"], wl["ln2_b"], 1e-5) for row in x1]
    want = bf_add(x1, bf_ffn(n2, wl))
    np.testing.assert_allclose(O.decoder_preln_adapter(x, w, h, 1e-5), want, rtol=1e-11, atol=1e-12)


def test_shared_decoder_layer_with_silent_adapter_is_the_plain_decoder_layer():
    d, f, r, h = 8, 16, 4, 2
    w = dict(enc_weights(17, d, f), **adapter_weights(18, d, r))
    x = rnd(19, 6, d)
    quiet = dict(w, w_up=np.zeros((d, r)), b_up=np.zeros(d))
    assert np.array_equal(O.decoder_preln_adapter(x, quiet, h, 1e-5), O.decoder_preln(x, w, h, 1e-5))
    assert np.abs(O.decoder_preln_adapter(x, w, h, 1e-5) - O.decoder_preln(x, w, h, 1e-5)).max() > 1e-3
    Y = O.layer_forward(O.BLOCK_DEC_ADAPTER, np.concatenate([x, x]), [1, 0], [6, 6], lambda t: {0: quiet, 1: w}[t], h, 1e-5)
    assert np.array_equal(Y[6:], O.decoder_preln(x, w, h, 1e-5))
    # causal: what a decode step relies on
    np.testing.assert_allclose(O.decoder_preln_adapter(x[:4], w, h, 1e-5)[-1], O.decoder_preln_adapter(x, w, h, 1e-5)[3],
                               rtol=1e-12, atol=1e-13)


def test_attention_seq_len_one_collapses_to_linear_chain():
    d, f, h = 8, 16, 2
    w = enc_weights(5, d, f)
    x = rnd(6, 1, d)
    v = x @ w["wqkv"][2 * d:].T + w["bqkv"][2 * d:]
    for causal in (False, True):
        np.testing.assert_allclose(O.attention(x, w, h, causal), v @ w["wo"].T + w["bo"], atol=1e-13)


def test_uniform_attention_when_wq_wk_zero():
    d, f, h, S = 8, 16, 2, 5
    w = enc_weights(7, d, f)
    w["wqkv"][:2 * d] = 0.0
    w["bqkv"][:2 * d] = 0.0
    x = rnd(8, S, d)
    v = x @ w["wqkv"][2 * d:].T + w["bqkv"][2 * d:]
    mean_all = np.repeat(v.mean(axis=0, keepdims=True), S, axis=0)
    np.testing.assert_allclose(O.attention(x, w, h, False), mean_all @ w["wo"].T + w["bo"], atol=1e-13)
    prefix = np.cumsum(v, axis=0) / np.arange(1, S + 1)[:, None]
    np.testing.assert_allclose(O.attention(x, w, h, True), prefix @ w["wo"].T + w["bo"], atol=1e-13)


@pytest.mark.parametrize("block,h", [(O.BLOCK_FFN, 0), (O.BLOCK_ENC_POSTLN, 2), (O.BLOCK_DEC_PRELN, 2)])
@pytest.mark.parametrize("S", [1, 2, 3])
def test_blocks_against_scalar_brute_force(block, h, S):
    d, f = 4, 6
    w = ffn_weights(11 + S, d, f, 0.7) if block == O.BLOCK_FFN else enc_weights(11 + S, d, f, 0.7)
    x = rnd(20 + S, S, d)
    got = O.block_forward(block, x, w, h, 1e-5)
    want = bf_block(block, x.tolist(), as_lists(w), h, 1e-5)
    np.testing.assert_allclose(got, np.array(want), rtol=1e-12, atol=1e-13)


# ------------------------------------------------------------------ library special cases

def torch_layer(w, d, f, h, eps, norm_first):
    layer = torch.nn.TransformerEncoderLayer(d, h, f, dropout=0.0, activation="gelu",
                                             layer_norm_eps=eps, batch_first=True,
                                             norm_first=norm_first, dtype=torch.float64)
    t = lambda a: torch.nn.Parameter(torch.tensor(a))  # noqa: E731
    layer.self_attn.in_proj_weight = t(w["wqkv"]); layer.self_attn.in_proj_bias = t(w["bqkv"])
    layer.self_attn.out_proj.weight = t(w["wo"]); layer.self_attn.out_proj.bias = t(w["bo"])
    layer.linear1.weight = t(w["w1"]); layer.linear1.bias = t(w["b1"])
    layer.linear2.weight = t(w["w2"]); layer.linear2.bias = t(w["b2"])
    layer.norm1.weight = t(w["ln1_g"]); layer.norm1.bias = t(w["ln1_b"])
    layer.norm2.weight = t(w["ln2_g"]); layer.norm2.bias = t(w["ln2_b"])
    return layer.train()  # train mode with dropout 0: the plain (non-fused) code path


@pytest.mark.parametrize("S", [1, 7, 40])
def test_encoder_postln_matches_torch_library_layer(S):
    d, f, h, eps = 32, 80, 4, 1e-12
    w = enc_weights(31, d, f)
    x = rnd(32, S, d)
    with torch.no_grad():
        ref = torch_layer(w, d, f, h, eps, False)(torch.tensor(x)[None])[0].numpy()
    np.testing.assert_allclose(O.encoder_postln(x, w, h, eps), ref, rtol=1e-11, atol=1e-12)


@pytest.mark.parametrize("S", [1, 7, 40])
def test_decoder_preln_matches_torch_library_layer_with_causal_mask(S):
    d, f, h, eps = 32, 80, 4, 1e-5
    w = enc_weights(33, d, f)
    x = rnd(34, S, d)
    mask = torch.triu(torch.full((S, S), float("-inf"), dtype=torch.float64), diagonal=1)
    with torch.no_grad():
        ref = torch_layer(w, d, f, h, eps, True)(torch.tensor(x)[None], src_mask=mask)[0].numpy()
    np.testing.assert_allclose(O.decoder_preln(x, w, h, eps), ref, rtol=1e-11, atol=1e-12)


def test_attention_matches_torch_sdpa():
    d, h, S = 24, 3, 9
    w = enc_weights(35, d, 8)
    x = rnd(36, S, d)
    qkv = torch.tensor(x @ w["wqkv"].T + w["bqkv"])
    q, k, v = (t.reshape(S, h, d // h).transpose(0, 1) for t in qkv.split(d, dim=1))
    for causal in (False, True):
        ctx = F.scaled_dot_product_attention(q, k, v, is_causal=causal).transpose(0, 1).reshape(S, d)
        ref = ctx.numpy() @ w["wo"].T + w["bo"]
        np.testing.assert_allclose(O.attention(x, w, h, causal), ref, rtol=1e-11, atol=1e-12)


def test_ffn_block_matches_torch_functional():
    d, f, eps = 48, 100, 1e-12
    w = ffn_weights(37, d, f)
    x = rnd(38, 13, d)
    t = {k: torch.tensor(v) for k, v in w.items()}
    xt = torch.tensor(x)
    ref = F.layer_norm(xt + F.linear(F.gelu(F.linear(xt, t["w1"], t["b1"])), t["w2"], t["b2"]),
                       (d,), t["ln_g"], t["ln_b"], eps).numpy()
    np.testing.assert_allclose(O.ffn_block(x, w, eps), ref, rtol=1e-11, atol=1e-12)


# ------------------------------------------------------------------ invariants of the path

def make_batch(seed, R, T, d, smin, smax):
    r = np.random.default_rng(seed)
    ids = r.integers(0, T, R)
    lens = r.integers(smin, smax + 1, R)
    X = r.standard_normal((int(lens.sum()), d))
    return ids, lens, X


BLOCKS = [(O.BLOCK_FFN, 0, 1e-12), (O.BLOCK_ENC_POSTLN, 2, 1e-12), (O.BLOCK_DEC_PRELN, 2, 1e-5)]


def tenant_bank(block, T, d, f, seed=100):
    mk = ffn_weights if block == O.BLOCK_FFN else enc_weights
    bank = [mk(seed + t, d, f) for t in range(T)]
    return bank, (lambda t: bank[t])


@pytest.mark.parametrize("block,h,eps", BLOCKS)
def test_single_tenant_batch_equals_plain_layer(block, h, eps):
    d, f = 8, 12
    ids, lens, X = make_batch(41, 6, 1, d, 1, 5)
    bank, wof = tenant_bank(block, 1, d, f)
    Y = O.layer_forward(block, X, ids, lens, wof, h, eps)
    if block == O.BLOCK_FFN:
        # token-wise block: the whole packed batch is one dense layer call
        t = {k: torch.tensor(v) for k, v in bank[0].items()}
        xt = torch.tensor(X)
        ref = F.layer_norm(xt + F.linear(F.gelu(F.linear(xt, t["w1"], t["b1"])), t["w2"], t["b2"]),
                           (d,), t["ln_g"], t["ln_b"], eps).numpy()
    else:
        # attention never crosses requests: a plain layer applied to each request alone
        layer = torch_layer(bank[0], d, f, h, eps, block == O.BLOCK_DEC_PRELN)
        ref, s0 = np.empty_like(X), 0
        for S in lens:
            m = (torch.triu(torch.full((S, S), float("-inf"), dtype=torch.float64), diagonal=1)
                 if block == O.BLOCK_DEC_PRELN else None)
            with torch.no_grad():
                ref[s0:s0 + S] = layer(torch.tensor(X[s0:s0 + S])[None], src_mask=m)[0].numpy()
            s0 += S
    np.testing.assert_allclose(Y, ref, rtol=1e-10, atol=1e-11)


@pytest.mark.parametrize("block,h,eps", BLOCKS)
def test_permuting_requests_permutes_outputs_bitwise(block, h, eps):
    d, f, T = 8, 12, 3
    ids, lens, X = make_batch(43, 7, T, d, 1, 4)
    _, wof = tenant_bank(block, T, d, f)
    Y = O.layer_forward(block, X, ids, lens, wof, h, eps)
    off = np.concatenate([[0], np.cumsum(lens)])
    p = np.random.default_rng(44).permutation(len(ids))
    Xp = np.concatenate([X[off[r]:off[r + 1]] for r in p])
    Yp = O.layer_forward(block, Xp, ids[p], lens[p], wof, h, eps)
    want = np.concatenate([Y[off[r]:off[r + 1]] for r in p])
    assert np.array_equal(Yp, want)


@pytest.mark.parametrize("block,h,eps", BLOCKS)
def test_identical_tenant_weights_and_inputs_give_identical_rows(block, h, eps):
    d, f, T = 8, 12, 4
    bank, _ = tenant_bank(block, 1, d, f)
    wof = lambda t: bank[0]  # noqa: E731  (every tenant holds the same weights)
    x = rnd(45, 3, d)
    ids, lens = np.array([3, 0, 2, 0]), np.array([3, 3, 3, 3])
    Y = O.layer_forward(block, np.concatenate([x] * 4), ids, lens, wof, h, eps)
    for r in range(1, 4):
        assert np.array_equal(Y[:3], Y[3 * r:3 * r + 3])
    # ... and equal to the single-tenant batch
    Y1 = O.layer_forward(block, np.concatenate([x] * 4), np.zeros(4, int), lens, wof, h, eps)
    assert np.array_equal(Y, Y1)


def test_different_tenants_do_give_different_rows():
    d, f, T = 8, 12, 2
    _, wof = tenant_bank(O.BLOCK_FFN, T, d, f)
    x = rnd(46, 2, d)
    Y = O.layer_forward(O.BLOCK_FFN, np.concatenate([x, x]), [0, 1], [2, 2], wof, 0, 1e-12)
    assert np.abs(Y[:2] - Y[2:]).max() > 1e-3
    # request r uses tenant_ids[r]: swapping the ids swaps the outputs
    Y2 = O.layer_forward(O.BLOCK_FFN, np.concatenate([x, x]), [1, 0], [2, 2], wof, 0, 1e-12)
    assert np.array_equal(Y2[:2], Y[2:]) and np.array_equal(Y2[2:], Y[:2])


@pytest.mark.parametrize("block,h,eps", BLOCKS)
def test_zero_task_weights_leave_the_residual_path(block, h, eps):
    d, f = 8, 12
    bank, _ = tenant_bank(block, 1, d, f)
    w = {k: (v if k.startswith("ln") else np.zeros_like(v)) for k, v in bank[0].items()}
    X = rnd(47, 5, d)
    Y = O.layer_forward(block, X, [0, 0], [2, 3], lambda t: w, h, eps)
    if block == O.BLOCK_FFN:
        ref = F.layer_norm(torch.tensor(X), (d,), torch.tensor(w["ln_g"]), torch.tensor(w["ln_b"]), eps)
        np.testing.assert_allclose(Y, ref.numpy(), atol=1e-13)
    elif block == O.BLOCK_ENC_POSTLN:
        r1 = F.layer_norm(torch.tensor(X), (d,), torch.tensor(w["ln1_g"]), torch.tensor(w["ln1_b"]), eps)
        r2 = F.layer_norm(r1, (d,), torch.tensor(w["ln2_g"]), torch.tensor(w["ln2_b"]), eps)
        np.testing.assert_allclose(Y, r2.numpy(), atol=1e-13)
    else:
        assert np.array_equal(Y, X)  # pre-LN: the residual stream passes through exactly


def test_zero_adapter_is_identity():
    d, r = 6, 2
    w = {"w_down": np.zeros((r, d)), "b_down": np.zeros(r), "w_up": np.zeros((d, r)), "b_up": np.zeros(d)}
    X = rnd(48, 4, d)
    assert np.array_equal(O.layer_forward(O.BLOCK_ADAPTER, X, [0], [4], lambda t: w), X)


def test_requests_subset_matches_full_batch():
    d, f, T = 8, 12, 3
    ids, lens, X = make_batch(49, 6, T, d, 1, 4)
    _, wof = tenant_bank(O.BLOCK_ENC_POSTLN, T, d, f)
    Y = O.layer_forward(O.BLOCK_ENC_POSTLN, X, ids, lens, wof, 2, 1e-12)
    Ys = O.layer_forward(O.BLOCK_ENC_POSTLN, X, ids, lens, wof, 2, 1e-12, requests=[1, 4])
    off = np.concatenate([[0], np.cumsum(lens)])
    for r in range(6):
        rows = slice(off[r], off[r + 1])
        if r in (1, 4):
            assert np.array_equal(Ys[rows], Y[rows])
        else:
            assert np.isnan(Ys[rows]).all()


# ------------------------------------------------------------------ router

def rank_count_perm(ids):
    """Second definition of the stable order: position of r = #{q: id[q] < id[r]} +
    #{q < r: id[q] == id[r]}."""
    R = len(ids)
    perm = [0] * R
    for r in range(R):
        pos = sum(1 for q in range(R) if ids[q] < ids[r]) + sum(1 for q in range(r) if ids[q] == ids[r])
        perm[pos] = r
    return perm


def test_route_hand_worked():
    rt = O.route([2, 0, 2, 1, 0], [3, 1, 2, 5, 4])
    assert rt["perm"].tolist() == [1, 4, 3, 0, 2]
    assert rt["tok_off"].tolist() == [0, 3, 4, 6, 11, 15]
    assert rt["seg_tenant"].tolist() == [0, 1, 2]
    assert rt["seg_req_off"].tolist() == [0, 2, 3, 5]
    assert rt["seg_tok_off"].tolist() == [0, 5, 10, 15]


@pytest.mark.parametrize("R,T", [(0, 4), (1, 4), (8, 4), (64, 1), (50, 1000), (300, 7)])
def test_route_against_rank_count(R, T):
    r = np.random.default_rng(R * 1000 + T)
    ids = r.integers(0, T, R).tolist()
    lens = r.integers(1, 20, R).tolist()
    rt = O.route(ids, lens)
    assert rt["perm"].tolist() == rank_count_perm(ids)
    G = len(rt["seg_tenant"])
    assert G == len(set(ids))
    assert rt["seg_tenant"].tolist() == sorted(set(ids))
    assert rt["seg_req_off"][0] == 0 and rt["seg_req_off"][-1] == R
    assert rt["seg_tok_off"][-1] == sum(lens) == rt["tok_off"][-1]
    for g in range(G):
        members = rt["perm"][rt["seg_req_off"][g]:rt["seg_req_off"][g + 1]].tolist()
        assert members == [q for q in range(R) if ids[q] == rt["seg_tenant"][g]]
        assert rt["seg_tok_off"][g + 1] - rt["seg_tok_off"][g] == sum(lens[q] for q in members)


def test_causal_layer_row_depends_on_earlier_rows_only():
    """What a decode step with a key/value cache relies on: in the causal pre-LN layer, row i of the
    output over a whole sequence is the last row of the output over its first i + 1 rows."""
    d, f, h, S = 8, 16, 2, 9
    w = enc_weights(3, d, f)
    x = rnd(4, S, d)
    full = O.decoder_preln(x, w, h, 1e-5)
    for i in (0, 3, S - 1):
        np.testing.assert_allclose(O.decoder_preln(x[:i + 1], w, h, 1e-5)[-1], full[i], rtol=1e-12, atol=1e-13)
    assert np.abs(O.encoder_postln(x[:4], w, h, 1e-5)[-1] - O.encoder_postln(x, w, h, 1e-5)[3]).max() > 1e-3


# ------------------------------------------------------------------ output heads

def test_head_forward_hand_worked():
    """Sec. 3.3.2: classification on the first row of a request, tagging on every row, label =
    class of the highest score.  Tenant 0 classifies with W = [[1,0],[0,1],[1,1]], b = [0,0,-10];
    tenant 1 tags with W = [[2,-1],[-1,2]], b = [0.5,0].  Rows: request 0 (tenant 1): [1,0],[0,1];
    request 1 (tenant 0): [3,4],[9,9]."""
    H = np.array([[1.0, 0], [0, 1], [3, 4], [9, 9]])
    heads = {0: (np.array([[1.0, 0], [0, 1], [1, 1]]), np.array([0.0, 0, -10]), False),
             1: (np.array([[2.0, -1], [-1, 2]]), np.array([0.5, 0.0]), True)}
    sc, lab = O.head_forward(H, [1, 0], [2, 2], lambda t: heads[t], 4)
    inf = -np.inf
    np.testing.assert_array_equal(sc, [[2.5, -1, inf, inf], [-0.5, 2, inf, inf], [3, 4, -3, inf], [inf] * 4])
    assert lab.tolist() == [0, 1, 1, -1]


def test_head_forward_ties_and_brute_force():
    rng = np.random.default_rng(5)
    d, T = 6, 4
    heads = {t: (rng.standard_normal((2 + t, d)), rng.standard_normal(2 + t), bool(t % 2)) for t in range(T)}
    ids, lens = [3, 0, 2, 1, 0], [3, 2, 1, 4, 1]
    H = rng.standard_normal((sum(lens), d))
    sc, lab = O.head_forward(H, ids, lens, lambda t: heads[t], 8)
    row = 0
    for t, S in zip(ids, lens):
        W, b, per_token = heads[t]
        for i in range(S):
            if per_token or i == 0:
                want = [sum(W[c][k] * H[row][k] for k in range(d)) + b[c] for c in range(len(b))]
                np.testing.assert_allclose(sc[row, :len(b)], want, rtol=1e-13, atol=1e-13)
                assert np.all(np.isneginf(sc[row, len(b):]))
                assert lab[row] == max(range(len(b)), key=lambda c: (want[c], -c))
            else:
                assert lab[row] == -1 and np.all(np.isneginf(sc[row]))
            row += 1
    # equal scores: the lowest class index wins
    tie = {0: (np.zeros((3, d)), np.array([1.0, 2.0, 2.0]), False)}
    assert O.head_forward(H[:1], [0], [1], lambda t: tie[t], 3)[1].tolist() == [1]


# ------------------------------------------------------------------ representation retrieval

def test_plot_aggregate_hand_worked():
    """Sec. 3.3.1, d = 1.  Table rows (first, second, third token): e0 = (1, 2, 3), e1 = (10, 20, 30),
    e2 = (100, 200, 300).  One request of three tokens with fragments e0, e1, e2 and one of a single token (e1):
      token 0: second of e0 and first of e1 -> (2 + 10) / 2 = 6
      token 1: third of e0, second of e1, first of e2 -> (3 + 20 + 100) / 3 = 41
      token 2: third of e1 and second of e2 -> (30 + 200) / 2 = 115
      lone token: second of e1 -> 20"""
    table = np.array([[[1.0], [2.0], [3.0]], [[10.0], [20.0], [30.0]], [[100.0], [200.0], [300.0]]])
    np.testing.assert_allclose(O.plot_aggregate(table, [0, 1, 2, 1], [3, 1]), [[6.0], [41.0], [115.0], [20.0]])


def test_plot_aggregate_is_a_mean_and_stays_inside_requests():
    rng = np.random.default_rng(3)
    d, E = 5, 7
    const = np.broadcast_to(rng.standard_normal(d), (E, 3, d))     # every representation equal: the mean is that vector
    ids = rng.integers(0, E, 9)
    np.testing.assert_allclose(O.plot_aggregate(const, ids, [4, 5]), np.broadcast_to(const[0, 0], (9, d)), atol=1e-15)
    table = rng.standard_normal((E, 3, d))
    whole = O.plot_aggregate(table, ids, [4, 5])
    np.testing.assert_array_equal(whole[:4], O.plot_aggregate(table, ids[:4], [4]))     # requests do not see each other
    np.testing.assert_array_equal(whole[4:], O.plot_aggregate(table, ids[4:], [5]))
    assert np.abs(whole - O.plot_aggregate(table, ids, [9])).max() > 1e-3


# ------------------------------------------------------------------ the pins do bite

MUTANTS = {
    "linear_transposed": ("linear", lambda a, W, b: a @ W[:a.shape[1], :a.shape[1]] + b[:a.shape[1]]
                          if W.shape[0] == W.shape[1] else a @ W.T + b),
    "linear_no_bias": ("linear", lambda a, W, b: a @ W.T),
    "gelu_tanh": ("gelu", lambda x: 0.5 * x * (1 + np.tanh(math.sqrt(2 / math.pi) * (x + 0.044715 * x ** 3)))),
    "ln_unbiased_var": ("layer_norm", lambda x, g, b, eps: (x - x.mean(-1, keepdims=True))
                        / np.sqrt(x.var(-1, ddof=1, keepdims=True) + eps) * g + b),
    "ln_eps_outside": ("layer_norm", lambda x, g, b, eps: (x - x.mean(-1, keepdims=True))
                       / (np.sqrt(x.var(-1, keepdims=True)) + eps) * g + b),
    "adapter_no_skip": ("adapter_block", lambda x, w: np.maximum(x @ w["w_down"].T + w["b_down"], 0) @ w["w_up"].T + w["b_up"]),
    "adapter_no_relu": ("adapter_block", lambda x, w: (x @ w["w_down"].T + w["b_down"]) @ w["w_up"].T + w["b_up"] + x),
    "softmax_cols": ("softmax_rows", lambda s: np.exp(s - s.max()) / np.exp(s - s.max()).sum(0, keepdims=True)),
}


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_planted_mistake_in_the_oracle_is_caught(name, monkeypatch):
    """Plant a plausible mistake in the ORACLE (on the CPU) and require that at least one
    of the pins above fails."""
    attr, fn = MUTANTS[name]
    monkeypatch.setattr(O, attr, fn)
    pins = [lambda: test_encoder_postln_matches_torch_library_layer(7),
            lambda: test_decoder_preln_matches_torch_library_layer_with_causal_mask(7),
            lambda: test_ffn_block_hand_worked(),
            lambda: test_adapter_block_hand_worked(),
            lambda: test_shared_layer_with_adapter_hand_worked(),
            lambda: test_layer_norm_hand_and_moments(),
            lambda: test_gelu_closed_forms(),
            lambda: test_softmax_rows_hand(),
            lambda: test_linear_is_W_a_plus_b_not_transposed()]
    caught = 0
    for pin in pins:
        try:
            pin()
        except (AssertionError, ValueError):
            caught += 1
    assert caught >= 1
