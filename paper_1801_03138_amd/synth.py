"""Seeded synthetic inputs for the replay train step.

This module serves the GPU library's tests, the CPU oracle's tests and the
benchmark alike.  It holds none of the method's arithmetic: it only draws
experience tuples, byte frames and initial network parameters from numpy's
PCG64 generator, one independent stream per field.

The paper trains on live gameplay of 27 memory-derived floats per state
(Methods: packed rows of 2*27+3 values, replay of 1,000,000); that data is not
available, so rows of the same shape and type stand in for it.
"""
import numpy as np
import torch

FIELDS = ("s", "s_next", "a", "r", "term")


def f32_to_bf16_bits(x):
    """Round float32 values to bfloat16 (library conversion), as uint16 bit patterns."""
    t = torch.from_numpy(np.ascontiguousarray(x, np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16).copy()


def bf16_bits_to_f32(bits):
    """Exact widening of bfloat16 bit patterns to float32."""
    b = np.ascontiguousarray(bits, np.uint16).astype(np.uint32) << 16
    return b.view(np.float32)


def _streams(seed, n):
    return [np.random.Generator(np.random.PCG64(s)) for s in np.random.SeedSequence(seed).spawn(n)]


def experiences(n, state_dim, num_actions, p_term, seed=0, state_dtype="f32"):
    """n experience tuples: s, s' ~ N(0,1) (independent), a uniform, r ~ N(0,1), terminal Bernoulli.

    state_dtype "f32" gives float32 states, "bf16" gives uint16 bfloat16 bit patterns.
    """
    gs, gs2, ga, gr, gt = _streams(seed, 5)
    s = gs.standard_normal((n, state_dim), dtype=np.float32)
    s2 = gs2.standard_normal((n, state_dim), dtype=np.float32)
    a = ga.integers(0, num_actions, size=n, dtype=np.int32)
    r = gr.standard_normal(n, dtype=np.float32)
    term = (gt.random(n) < p_term).astype(np.uint8)
    if state_dtype == "bf16":
        s, s2 = f32_to_bf16_bits(s), f32_to_bf16_bits(s2)
    elif state_dtype != "f32":
        raise ValueError(state_dtype)
    return {"s": s, "s_next": s2, "a": a, "r": r, "term": term}


def frames(n, state_dim, num_actions, p_term, seed=0):
    """n single-state experiences with uint8 states ~ U{0..255} (one state per experience)."""
    gs, _, ga, gr, gt = _streams(seed, 5)
    s = gs.integers(0, 256, size=(n, state_dim), dtype=np.uint8)
    a = ga.integers(0, num_actions, size=n, dtype=np.int32)
    r = gr.standard_normal(n, dtype=np.float32)
    term = (gt.random(n) < p_term).astype(np.uint8)
    return {"s": s, "s_next": None, "a": a, "r": r, "term": term}


def take(rows, lo, hi):
    """Rows lo..hi-1 of an experience dict."""
    return {k: (None if v is None else v[lo:hi]) for k, v in rows.items()}


def init_params(state_dim, hidden, num_actions, seed=0, hidden2=None):
    """Flat float32 [W1 b1 W2 b2 W3 b3], each ~ U(-1/sqrt(fan_in), 1/sqrt(fan_in)); W row-major [in x out].
    hidden2: width of the second hidden layer (default: the same as the first)."""
    g = np.random.Generator(np.random.PCG64(seed + 1))
    h2 = hidden if hidden2 is None else hidden2
    parts = []
    for fan_in, fan_out in ((state_dim, hidden), (hidden, h2), (h2, num_actions)):
        bound = 1.0 / np.sqrt(fan_in)
        parts.append(g.uniform(-bound, bound, size=fan_in * fan_out).astype(np.float32))
        parts.append(g.uniform(-bound, bound, size=fan_out).astype(np.float32))
    return np.concatenate(parts)


def split_params(flat, state_dim, hidden, num_actions, hidden2=None):
    """Views W1[D,H], b1[H], W2[H,G], b2[G], W3[G,A], b3[A] into a flat parameter array (G = hidden2 or H)."""
    D, H, A = state_dim, hidden, num_actions
    G = H if hidden2 is None else hidden2
    o = 0
    out = []
    for shape in ((D, H), (H,), (H, G), (G,), (G, A), (A,)):
        n = int(np.prod(shape))
        out.append(flat[o:o + n].reshape(shape))
        o += n
    assert o == flat.shape[0]
    return out
