"""ORACLE — test infrastructure only, never on the product path.

Diagnostic variant of the tree-cell operators: the same float64 arithmetic as oracle/ops.py, with
the roundings of a 16-bit state path applied where such a path stores a value.  The paper fixes no
precision; the workloads say "bf16 inputs/weights with fp32 accumulate".  The reading:

  h                     stored as bfloat16 (round to nearest, ties to even)
  c                     stored as float32
  gate activations      kept for the gradient operator as bfloat16 (the forward c and h are formed
                        from the unrounded activations)
  pre-activation grads  delta (TreeRNN), dz (TreeLSTM) rounded to bfloat16 before they enter the
                        products W^T dz and dz x^T; dh, dc stay float32
  sums                  float64 here (fp32 accumulation is not modelled)

It bounds what rounding alone does to the results, so that a comparison of the 16-bit path with it
can be much tighter than with the unrounded oracle.  Selected with env["round_bf16"] = True.
"""
import numpy as np
from . import ops


def bf16(x):
    """Nearest bfloat16 (8 significant bits), ties to even, as float64."""
    f = np.asarray(x, dtype=np.float32)
    bits = f.view(np.uint32).astype(np.uint64)
    low = bits & np.uint64(0xFFFF)
    keep = bits >> np.uint64(16)
    up = (low > 0x8000) | ((low == 0x8000) & ((keep & np.uint64(1)) == 1))
    keep = keep + up.astype(np.uint64)
    out = (keep << np.uint64(16)).astype(np.uint32).view(np.float32)
    return out.astype(np.float64).reshape(np.shape(x))


def f32(x):
    return np.asarray(x, dtype=np.float32).astype(np.float64)


def rnn_cell(W, b, hl, hr):
    return bf16(ops.rnn_cell(W, b, hl, hr))


def rnn_cell_grad(W, b, hl, hr, dh):
    x = np.concatenate([hl, hr])
    h = bf16(np.tanh(W @ x + b))                 # the stored h
    delta = bf16(dh * (1.0 - h * h))
    dx = W.T @ delta
    H = hl.shape[0]
    return f32(dx[:H]), f32(dx[H:]), delta, x


def lstm_cell(W, b, sl, sr):
    H = sl.shape[0] // 2
    x, i, fl, fr, o, u = ops.lstm_gates(W, b, sl, sr)
    c = f32(i * u + fl * sl[H:] + fr * sr[H:])
    return np.concatenate([bf16(o * np.tanh(c)), c])


def lstm_cell_grad(W, b, sl, sr, ds):
    H = sl.shape[0] // 2
    x, i, fl, fr, o, u = ops.lstm_gates(W, b, sl, sr)
    cl, cr = sl[H:], sr[H:]
    c = f32(i * u + fl * cl + fr * cr)           # the stored c, from the unrounded activations
    i, fl, fr, o, u = (bf16(g) for g in (i, fl, fr, o, u))   # the activations as they were kept
    tc = np.tanh(c)
    dh, dc_in = ds[:H], ds[H:]
    do = dh * tc
    dc = dc_in + dh * o * (1.0 - tc * tc)
    dz = bf16(np.concatenate([dc * u * i * (1 - i), dc * cl * fl * (1 - fl), dc * cr * fr * (1 - fr),
                              do * o * (1 - o), dc * i * (1 - u * u)]))
    dx = W.T @ dz
    return (np.concatenate([f32(dx[:H]), f32(dc * fl)]), np.concatenate([f32(dx[H:]), f32(dc * fr)]), dz, x)
