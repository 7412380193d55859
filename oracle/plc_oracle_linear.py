"""CPU oracle for the linear-embedding predictor (Sec. 7.1, "Linear embedding approximation").

TEST INFRASTRUCTURE ONLY, like the rest of oracle/: imported by tests, the smoke check and the
benchmark's CPU leg, never by the product package, with which it shares no code.

What it follows: per layer the KV vector is taken as linear in the next token's embedding,
F(t_<i, t) ~ c(t_<i) + A E(t); the predicted KV vector is then c + A Ebar_i, where
Ebar_i = sum_t P(t | t_<i) E(t) is the expected embedding, a weighted sum over the whole
vocabulary.  Readings: A is one matrix per layer, c has the shape of the KV cache, and Ebar is
stored as fp16 between the two steps (it is an fp16 tensor on the device).  Everything after the
prediction is the core path's: residual (Def. "KV residual"), quantiser and escape rule, add-back.

Arithmetic: float64 throughout (numpy matmul as the library primitive for the two contractions),
round-half-even, fp16 conversions by numpy.

Pins (tests/test_oracle_linear_pins.py): for candidates that are exactly linear in their
embeddings the prediction equals the weighted mean of the candidate vectors computed by the pinned
C oracle (the identity the approximation rests on); a one-hot distribution on the true token with
noise-free vectors gives all-zero residuals; the recovery error is at most half a step.
"""
from __future__ import annotations

import numpy as np

ESCAPE = 255


def expected_embedding(probs_full, embed_t):
    """probs_full fp16 [rows, V], embed_t fp16 [m, V] -> Ebar fp16 [rows, m]."""
    p = np.asarray(probs_full, dtype=np.float16).astype(np.float64)
    e = np.asarray(embed_t, dtype=np.float16).astype(np.float64)
    return (p @ e.T).astype(np.float16)


def predict(ebar, A, bias_k, bias_v):
    """ebar fp16 [S, n, m]; A fp16 [L, H, 2, d, m]; bias_* fp16 [S, L, H, n, d]
    -> prediction float64 [S, L, H, n, 2, d] = c + A Ebar."""
    eb = np.asarray(ebar, dtype=np.float16).astype(np.float64)
    a = np.asarray(A, dtype=np.float16).astype(np.float64)
    lin = np.einsum("lhcem,snm->slhnce", a, eb, optimize=True)
    bias = np.stack([np.asarray(bias_k, dtype=np.float16), np.asarray(bias_v, dtype=np.float16)], axis=4)
    return lin + bias.astype(np.float64)


def predict_residual(ebar, A, bias_k, bias_v, act_k, act_v, delta, qmax=127):
    """Returns dict(symbols u8 [streams, N], esc_vals u16, esc_cnt u32 [streams], esc_off u64, pred, u)."""
    pred = predict(ebar, A, bias_k, bias_v)
    act = np.stack([np.asarray(act_k, dtype=np.float16), np.asarray(act_v, dtype=np.float16)], axis=4)
    step = float(np.float32(delta))                     # THE step is the fp32 value
    with np.errstate(invalid="ignore", over="ignore"):
        u = (act.astype(np.float64) - pred) / step
        q = np.rint(u)                                  # round half to even
    esc = ~np.isfinite(u) | (np.abs(q) > qmax)
    sym = np.where(esc, ESCAPE, np.where(esc, 0, q) + 127).astype(np.uint8)
    S, L, H, n, _, d = sym.shape
    streams = S * L * H
    sym = sym.reshape(streams, n * 2 * d)
    escf = esc.reshape(streams, -1)
    raw = act.view(np.uint16).reshape(streams, -1)
    esc_cnt = escf.sum(1).astype(np.uint32)
    esc_off = (np.cumsum(esc_cnt, dtype=np.uint64) - esc_cnt).astype(np.uint64)
    esc_vals = raw[escf]                                # stream after stream, symbol order inside each
    return dict(symbols=sym, esc_vals=esc_vals, esc_cnt=esc_cnt, esc_off=esc_off,
                pred=pred.reshape(streams, -1), u=u.reshape(streams, -1))


def reconstruct(ebar, A, bias_k, bias_v, symbols, esc_vals, delta):
    """-> (out_k, out_v) fp16 [S, L, H, n, d]; escaped components take their raw values back."""
    pred = predict(ebar, A, bias_k, bias_v)
    S, L, H, n, _, d = pred.shape
    sym = np.asarray(symbols, dtype=np.uint8).reshape(S, L, H, n, 2, d)
    step = float(np.float32(delta))
    out = (pred + (sym.astype(np.float64) - 127.0) * step).astype(np.float16)
    flat = out.reshape(S * L * H, -1)
    escf = (sym == ESCAPE).reshape(S * L * H, -1)
    flat.view(np.uint16)[escf] = np.asarray(esc_vals, dtype=np.uint16)[:int(escf.sum())]
    out = flat.reshape(S, L, H, n, 2, d)
    return np.ascontiguousarray(out[..., 0, :]), np.ascontiguousarray(out[..., 1, :])
