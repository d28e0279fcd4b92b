"""Pins of the graph-level oracle: the workload graphs evaluated vertex by vertex must equal
the textbook computation they encode (matrix chain, softmax cross-entropy step with its
gradients, causal multi-head attention + SwiGLU), up to the bf16 rounding of intermediates."""
import math

import numpy as np

from oracle.graph_ref import make_inputs, run_graph
from synth_inputs import build_config


def _rel_rms(got, want):
    got, want = np.asarray(got, dtype=np.float64), np.asarray(want, dtype=np.float64)
    return float(np.sqrt(np.mean((got - want) ** 2)) / (np.sqrt(np.mean(want ** 2)) + 1e-300))


def test_matrix_chain_graph():
    w = build_config(2, small=True)
    inp = make_inputs(w)
    env = run_graph(w, inp)
    A, B, C = (inp[k].as_f64() for k in "ABC")
    assert _rel_rms(env["ABC"].as_f64(), (A @ B) @ C) < 5e-3
    assert env["AB"].dtype == "bf16" and env["ABC"].dtype == "f32"


def test_ffnn_step_graph_loss_and_gradients():
    w = build_config(3, dims={"b": 32, "f": 48, "h": 40, "c": 16})
    inp = make_inputs(w)
    env = run_graph(w, inp)
    X, W1, W2, Y = (inp[k].as_f64() for k in ("X", "W1", "W2", "Y"))
    assert np.array_equal(Y.sum(axis=1), np.ones(32))              # one-hot labels
    B = X.shape[0]
    H1 = X @ W1
    A1 = np.maximum(H1, 0)
    L = A1 @ W2
    Ls = L - L.max(axis=1, keepdims=True)
    logp = Ls - np.log(np.exp(Ls).sum(axis=1, keepdims=True))
    loss = -(Y * logp).sum() / B
    P = np.exp(logp)
    dL = (P - Y) / B
    dW2 = A1.T @ dL
    dH1 = (dL @ W2.T) * (H1 > 0)
    dW1 = X.T @ dH1
    assert abs(float(env["loss"].as_f64()) - loss) < 2e-3 * abs(loss)
    assert _rel_rms(env["dW2"].as_f64(), dW2) < 1e-2
    assert _rel_rms(env["dW1"].as_f64(), dW1) < 2e-2
    # a sign error or a transposed operand would give a relative error near 1 or 2


def test_decoder_block_graph():
    w = build_config(4, dims={"b": 2, "s": 16, "a": 32, "h": 4, "d": 8, "f": 48})
    inp = make_inputs(w)
    env = run_graph(w, inp)
    X = inp["X"].as_f64()
    Wq, Wk, Wv, Wo = (inp[k].as_f64() for k in ("Wq", "Wk", "Wv", "Wo"))
    Wg, Wu, Wd = (inp[k].as_f64() for k in ("Wg", "Wu", "Wd"))
    M = inp["M"].as_f64()
    assert M[3, 3] == 0 and M[3, 4] == -np.inf and M[4, 3] == 0      # causal: key index above query index is masked
    b, s, a = X.shape
    h, d = Wq.shape[1:]
    out = np.empty((b, s, a))
    for bi in range(b):
        heads = []
        for hi in range(h):
            q, k, v = X[bi] @ Wq[:, hi, :], X[bi] @ Wk[:, hi, :], X[bi] @ Wv[:, hi, :]
            sc = q @ k.T / math.sqrt(d) + M
            p = np.exp(sc - sc.max(axis=1, keepdims=True))
            p /= p.sum(axis=1, keepdims=True)
            heads.append(p @ v)
        att = np.concatenate(heads, axis=1) @ Wo.reshape(a, h * d).T
        g, u = att @ Wg, att @ Wu
        out[bi] = ((g / (1 + np.exp(-g))) * u) @ Wd
    assert _rel_rms(env["Out"].as_f64(), out) < 2e-2
    # softmax rows of the oracle's P sum to one up to bf16 rounding of P
    assert np.allclose(env["P"].as_f64().sum(axis=-1), 1.0, atol=2e-2)


def test_split_reduction_graph():
    w = build_config(5, small=True)
    inp = make_inputs(w)
    env = run_graph(w, inp)
    X, Y = inp["X"].as_f64(), inp["Y"].as_f64()
    want = np.einsum("ijk,kl->ijl", X, Y)
    assert _rel_rms(env["Z"].as_f64(), want) < 1e-6
