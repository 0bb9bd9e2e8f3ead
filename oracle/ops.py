"""ORACLE — test infrastructure only, never on the product path.

Node bodies ("operators") and their gradient operators in float64 (paper Section 2.2 for
the firing rule of ordinary operators, Section 4 for the shape of a gradient operator:
it takes the n inputs of the forward operator and the m output gradients and yields the n
input gradients).  The tree cells are not defined by the paper; they follow the workload
definitions:

  TreeRNN cell       h = tanh(W [h_l; h_r] + b)                      W in R^{H x 2H}
  binary TreeLSTM    z = W [h_l; h_r] + b in R^{5H}, row blocks (i, f_l, f_r, o, u)
                     i, f_l, f_r, o = sigmoid(.)   u = tanh(z_u)
                     c = i*u + f_l*c_l + f_r*c_r   h = o*tanh(c)
                     a state is the pair (h, c), carried as one vector [h; c]
  leaf               h = E[token]   (TreeLSTM: c = 0)
  head               loss = -log softmax(U h + u0)[label]
  node loss          the same loss at a tree node v with label node_label[v] >= 0, on the h of
                     the state the node's subtree produced; the state itself goes on unchanged
"""
import numpy as np


def sigmoid(x):
    return 1.0 / (1.0 + np.exp(-x))


# ---- TreeRNN ------------------------------------------------------------------------
def rnn_cell(W, b, hl, hr):
    return np.tanh(W @ np.concatenate([hl, hr]) + b)


def rnn_cell_grad(W, b, hl, hr, dh):
    """Returns (dh_l, dh_r, delta, x): delta*x^T is this tag's term of dW, delta of db."""
    x = np.concatenate([hl, hr])
    h = np.tanh(W @ x + b)
    delta = dh * (1.0 - h * h)
    dx = W.T @ delta
    H = hl.shape[0]
    return dx[:H], dx[H:], delta, x


# ---- binary TreeLSTM ----------------------------------------------------------------
def lstm_leaf(e):
    return np.concatenate([e, np.zeros_like(e)])


def lstm_gates(W, b, sl, sr):
    H = sl.shape[0] // 2
    x = np.concatenate([sl[:H], sr[:H]])
    z = W @ x + b
    i, fl, fr, o = (sigmoid(z[k * H:(k + 1) * H]) for k in range(4))
    u = np.tanh(z[4 * H:])
    return x, i, fl, fr, o, u


def lstm_cell(W, b, sl, sr):
    H = sl.shape[0] // 2
    x, i, fl, fr, o, u = lstm_gates(W, b, sl, sr)
    c = i * u + fl * sl[H:] + fr * sr[H:]
    return np.concatenate([o * np.tanh(c), c])


def lstm_cell_grad(W, b, sl, sr, ds):
    """ds = [dh; dc].  Returns (ds_l, ds_r, dz, x)."""
    H = sl.shape[0] // 2
    x, i, fl, fr, o, u = lstm_gates(W, b, sl, sr)
    cl, cr = sl[H:], sr[H:]
    c = i * u + fl * cl + fr * cr
    tc = np.tanh(c)
    dh, dc_in = ds[:H], ds[H:]
    do = dh * tc
    dc = dc_in + dh * o * (1.0 - tc * tc)
    dz = np.concatenate([dc * u * i * (1 - i), dc * cl * fl * (1 - fl), dc * cr * fr * (1 - fr),
                         do * o * (1 - o), dc * i * (1 - u * u)])
    dx = W.T @ dz
    return (np.concatenate([dx[:H], dc * fl]), np.concatenate([dx[H:], dc * fr]), dz, x)


# ---- classification head ------------------------------------------------------------
def ce_head(U, u0, h, label):
    logits = U @ h + u0
    m = logits.max()
    return float(m + np.log(np.exp(logits - m).sum()) - logits[label])


def ce_head_grad(U, u0, h, label, dloss):
    logits = U @ h + u0
    p = np.exp(logits - logits.max())
    p /= p.sum()
    p[label] -= 1.0
    return (U.T @ p) * dloss
