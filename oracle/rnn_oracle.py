"""CPU oracle for the other recurrent cells: single-gate RNN (ReLU / tanh) and GRU, forward and full BPTT.

TEST INFRASTRUCTURE ONLY.  The slow, plain definition that the GPU library's rnn_forward / rnn_backward are
checked against.  Only tests may import it; the product path never does, and this module imports nothing from
the product package.

Why these cells: Section 2 of Appleyard, Kocisky & Blunsom (arXiv 1604.01946) states that the strategies
carry over to other recurrent units, Section 2.1 that a GRU offers two groups of three matrices to combine
and a single-gate RNN none, and Section 3.3 that the library release built on this work supports ReLU, tanh,
LSTM and GRU units.  The paper prints no equations for them; the conventions below are this repository's
(stated again in the C header):

  single-gate RNN   h_t = act(W x_t + R h_{t-1} + b),   act = max(0, .) or tanh
  GRU, gates along every 3H axis in the order r (reset), z (update), n (candidate):
      r_t = sigma(W_r x_t + R_r h_{t-1} + b_r)
      z_t = sigma(W_z x_t + R_z h_{t-1} + b_z)
      n_t = tanh (W_n x_t + b_n + r_t o (R_n h_{t-1}))
      h_t = (1 - z_t) o n_t + z_t o h_{t-1}
    The reset gate multiplies the recurrent product R_n h_{t-1} (not h_{t-1} before the product), which is
    what lets the three recurrent matrices run as one stacked product per step -- the grouping Section 2.1
    describes; one bias vector per gate, as the paper's LSTM has.  torch.nn.GRU computes the same function
    when its second bias vector is zero.
  stacking as in Section 2.4: the hidden output of layer l-1 at step t is the input of layer l at step t.
  x [T][B][I]; W = layer 0's [G][I] then layers 1..L-1's [G][H], G = gates*H; R [L][G][H]; b [L][G]; h0 [L][B][H].

Backward is the chain rule for Loss = <dy, y> + <dhT, hT>.  All arithmetic in float64 unless dtype= says
otherwise; one numpy matmul per matrix product and time step, no blocking, fusion or reordering.

Pins (tests/test_rnn_oracle_pins.py): closed forms for W = R = 0, a scalar GRU step expanded by hand, central
finite differences for every gradient, torch.nn.RNN / torch.nn.GRU in float64 as independent library routines,
split-T and layer-stack identities, one-sided differences at a pre-activation of exactly 0 for the ReLU slope argument.  Nothing here is "parity unpinned".
"""
import numpy as np

CELLS = {"relu": 1, "tanh": 1, "gru": 3}  # gates per cell


def sigmoid(z):
    z = np.asarray(z)
    out = np.empty_like(z)
    pos = z >= 0
    out[pos] = 1.0 / (1.0 + np.exp(-z[pos]))
    ez = np.exp(z[~pos])
    out[~pos] = ez / (1.0 + ez)
    return out


def split_W(W, cell, L, I, H):
    """Per-layer views [G][I_l] of the flat input-matrix array."""
    G = CELLS[cell] * H
    out, off = [], 0
    for l in range(L):
        Il = I if l == 0 else H
        out.append(W[off:off + G * Il].reshape(G, Il))
        off += G * Il
    return out


def rnn_forward(cell, L, T, B, I, H, x, h0, W, R, b, dtype=np.float64):
    """Returns y [T][B][H], hT [L][B][H] and the saved values the backward pass needs."""
    G = CELLS[cell] * H
    x = np.asarray(x, dtype).reshape(T, B, I)
    R = np.asarray(R, dtype).reshape(L, G, H)
    b = np.asarray(b, dtype).reshape(L, G)
    Ws = split_W(np.asarray(W, dtype), cell, L, I, H)
    h0 = np.zeros((L, B, H), dtype) if h0 is None else np.asarray(h0, dtype).reshape(L, B, H)
    hs = np.zeros((L, T, B, H), dtype)
    saved = {"h": hs}
    if cell == "gru":
        saved.update(r=np.zeros((L, T, B, H), dtype), z=np.zeros((L, T, B, H), dtype), n=np.zeros((L, T, B, H), dtype),
                     qn=np.zeros((L, T, B, H), dtype))
    for l in range(L):
        h = h0[l]
        for t in range(T):
            inp = x[t] if l == 0 else hs[l - 1, t]
            a = inp @ Ws[l].T + b[l]      # [B][G]
            q = h @ R[l].T                # [B][G]
            if cell == "gru":
                r = sigmoid(a[:, :H] + q[:, :H])
                z = sigmoid(a[:, H:2 * H] + q[:, H:2 * H])
                n = np.tanh(a[:, 2 * H:] + r * q[:, 2 * H:])
                h = (1.0 - z) * n + z * h
                saved["r"][l, t], saved["z"][l, t], saved["n"][l, t], saved["qn"][l, t] = r, z, n, q[:, 2 * H:]
            elif cell == "tanh":
                h = np.tanh(a + q)
            else:
                h = np.maximum(a + q, 0.0)
            hs[l, t] = h
    return hs[L - 1].copy(), hs[:, T - 1].copy(), saved


def relu_preactivations(L, T, B, I, H, x, h0, W, R, b, saved, dtype=np.float64):
    """Pre-activations a [L][T][B][H] of a ReLU network, recomputed from the saved hidden states."""
    x = np.asarray(x, dtype).reshape(T, B, I)
    R = np.asarray(R, dtype).reshape(L, H, H)
    b = np.asarray(b, dtype).reshape(L, H)
    Ws = split_W(np.asarray(W, dtype), "relu", L, I, H)
    h0 = np.zeros((L, B, H), dtype) if h0 is None else np.asarray(h0, dtype).reshape(L, B, H)
    hs = saved["h"]
    a = np.zeros((L, T, B, H), dtype)
    for l in range(L):
        for t in range(T):
            inp = x[t] if l == 0 else hs[l - 1, t]
            hp = hs[l, t - 1] if t > 0 else h0[l]
            a[l, t] = inp @ Ws[l].T + hp @ R[l].T + b[l]
    return a


def rnn_backward(cell, L, T, B, I, H, x, h0, W, R, saved, dy, dhT, dtype=np.float64, relu_slope=None):
    """Returns dx [T][B][I], dh0 [L][B][H], dW (flat, like W), dR [L][G][H], db [L][G].

    relu_slope (ReLU only): [L][T][B][H] values used as the derivative of the activation in place of (h > 0).
    max(0, a) has no derivative at a = 0: 0 is its slope from the left and 1 from the right, and an evaluation in
    finite precision cannot tell which side a pre-activation within rounding of 0 is on.  A test that meets such
    elements passes the slope it wants for them (and (h > 0) everywhere else) to obtain each of the valid results."""
    G = CELLS[cell] * H
    x = np.asarray(x, dtype).reshape(T, B, I)
    R = np.asarray(R, dtype).reshape(L, G, H)
    Ws = split_W(np.asarray(W, dtype), cell, L, I, H)
    h0 = np.zeros((L, B, H), dtype) if h0 is None else np.asarray(h0, dtype).reshape(L, B, H)
    dy = np.asarray(dy, dtype).reshape(T, B, H)
    dhT = np.zeros((L, B, H), dtype) if dhT is None else np.asarray(dhT, dtype).reshape(L, B, H)
    hs = saved["h"]
    dWs = [np.zeros_like(w) for w in Ws]
    dR = np.zeros((L, G, H), dtype)
    db = np.zeros((L, G), dtype)
    dh0 = np.zeros((L, B, H), dtype)
    dout = dy.copy()                     # gradient arriving from above at every step
    for l in range(L - 1, -1, -1):
        Il = I if l == 0 else H
        din = np.zeros((T, B, Il), dtype)
        carry = dhT[l].copy()
        for t in range(T - 1, -1, -1):
            inp = x[t] if l == 0 else hs[l - 1, t]
            hp = hs[l, t - 1] if t > 0 else h0[l]
            dh = dout[t] + carry
            if cell == "gru":
                r, z, n, qn = saved["r"][l, t], saved["z"][l, t], saved["n"][l, t], saved["qn"][l, t]
                dn_pre = dh * (1.0 - z) * (1.0 - n * n)
                daz = dh * (hp - n) * z * (1.0 - z)
                dar = dn_pre * qn * r * (1.0 - r)
                da = np.concatenate([dar, daz, dn_pre], axis=1)          # with respect to W x + b
                dq = np.concatenate([dar, daz, dn_pre * r], axis=1)      # with respect to R h_{t-1}
                direct = dh * z
            else:
                h = hs[l, t]
                if cell == "tanh":
                    da = dh * (1.0 - h * h)
                else:
                    da = dh * ((h > 0).astype(dtype) if relu_slope is None else np.asarray(relu_slope, dtype)[l, t])
                dq = da
                direct = 0.0
            din[t] = da @ Ws[l]
            carry = dq @ R[l] + direct
            dWs[l] += da.T @ inp
            dR[l] += dq.T @ hp
            db[l] += da.sum(axis=0)
        dh0[l] = carry
        dout = din
    return dout, dh0, np.concatenate([w.ravel() for w in dWs]), dR, db


def loss(y, hT, dy, dhT):
    return float(np.sum(y * dy) + (0.0 if dhT is None else np.sum(hT * dhT)))
