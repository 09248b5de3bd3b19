"""CPU oracle for the stacked four-gate LSTM: forward pass and full BPTT.

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain definition that the
GPU library is checked against.  Only tests, the smoke check and the
benchmark's CPU-baseline leg may import it; the product path never does, and
this module imports nothing from the product package.

What it computes
----------------
Forward: the six cell equations of Section 2 of Appleyard, Kocisky & Blunsom
(arXiv 1604.01946), a standard LSTM with four gates and no peepholes, stacked
as Section 2.4 describes (the hidden output of layer l-1 at step t is the input
of layer l at step t).  Two misprints in the printed equations are read the
standard way: the first line's subscripts are t (i_t, x_t), and the cell update
uses the previous *cell state* c_{t-1} (not the candidate c'_{t-1}).

Backward: the paper gives no backward equations (Sections 2.1 and 2.6 only say
that the four gate gradients map to one output through the stacked matrices and
that weight gradients are one large product after propagation is complete).  The
code below is the chain rule applied to the forward equations for the scalar
    Loss = <dy, y> + <dhT, hT> + <dcT, cT>.

Conventions (the C ABI uses the same):
  * gate order along every 4H axis: i, f, o, c'  (the order Section 2 lists them)
  * one bias vector per gate (as printed), so b is [L][4H]
  * x is time-major [T][B][I]; W is the concatenation of layer 0's [4H][I] and
    layers 1..L-1's [4H][H]; R is [L][4H][H]
  * all arithmetic in float64 unless dtype= says otherwise (float32 is used only
    to show the fp32 noise floor)

Each matrix product is a single numpy matmul per time step; there is no
blocking, fusion or reordering beyond what the definition states.

Pins (tests/test_oracle_*.py): W=R=0 closed form (forward and backward), a
hand-expanded scalar cell, central finite differences for every gradient,
torch.nn.LSTM in float64 as an independent library routine, composition
identities (split T / split L / split B), linearity, bounds.  Nothing here is
"parity unpinned".
"""
import numpy as np

GATE_ORDER = ("i", "f", "o", "g")  # g is the candidate c'


def sigmoid(z):
    """Logistic function, evaluated in the branch that cannot overflow."""
    z = np.asarray(z)
    out = np.empty_like(z)
    pos = z >= 0
    out[pos] = 1.0 / (1.0 + np.exp(-z[pos]))
    ez = np.exp(z[~pos])
    out[~pos] = ez / (1.0 + ez)
    return out


def w_offsets(L, I, H):
    """Element offset of each layer's input matrix inside the flat W array."""
    offs, off = [], 0
    for l in range(L):
        offs.append(off)
        off += 4 * H * (I if l == 0 else H)
    return offs, off


def split_W(W, L, I, H):
    W = np.asarray(W).reshape(-1)
    offs, total = w_offsets(L, I, H)
    assert W.size == total, (W.size, total)
    return [W[offs[l]: offs[l] + 4 * H * (I if l == 0 else H)].reshape(4 * H, I if l == 0 else H)
            for l in range(L)]


def lstm_forward(L, T, B, I, H, x, h0, c0, W, R, b, dtype=np.float64):
    """Section 2 equations for every layer and step.

    Returns (y, hT, cT, reserve).  reserve is a dict of per-layer arrays that the
    backward pass needs: gates [L][T][B][4H] (activated i,f,o,c'), c and h
    [L][T][B][H].
    """
    x = np.asarray(x, dtype=dtype).reshape(T, B, I)
    h0 = np.zeros((L, B, H), dtype) if h0 is None else np.asarray(h0, dtype=dtype).reshape(L, B, H)
    c0 = np.zeros((L, B, H), dtype) if c0 is None else np.asarray(c0, dtype=dtype).reshape(L, B, H)
    Wl = [w.astype(dtype) for w in split_W(W, L, I, H)]
    R = np.asarray(R, dtype=dtype).reshape(L, 4 * H, H)
    b = np.asarray(b, dtype=dtype).reshape(L, 4 * H)

    gates = np.empty((L, T, B, 4 * H), dtype)
    cs = np.empty((L, T, B, H), dtype)
    hs = np.empty((L, T, B, H), dtype)
    inp = x
    for l in range(L):
        h_prev, c_prev = h0[l], c0[l]
        for t in range(T):
            a = inp[t] @ Wl[l].T + h_prev @ R[l].T + b[l]
            i = sigmoid(a[:, 0 * H:1 * H])
            f = sigmoid(a[:, 1 * H:2 * H])
            o = sigmoid(a[:, 2 * H:3 * H])
            g = np.tanh(a[:, 3 * H:4 * H])
            c = f * c_prev + i * g
            h = o * np.tanh(c)
            gates[l, t, :, 0 * H:1 * H] = i
            gates[l, t, :, 1 * H:2 * H] = f
            gates[l, t, :, 2 * H:3 * H] = o
            gates[l, t, :, 3 * H:4 * H] = g
            cs[l, t] = c
            hs[l, t] = h
            h_prev, c_prev = h, c
        inp = hs[l]
    y = hs[L - 1].copy()
    hT = hs[:, T - 1].copy()
    cT = cs[:, T - 1].copy()
    return y, hT, cT, {"gates": gates, "c": cs, "h": hs}


def lstm_backward(L, T, B, I, H, x, h0, c0, W, R, reserve, dy, dhT, dcT, dtype=np.float64):
    """Chain rule through the forward equations (BPTT), top layer first, last step first.

    Returns (dx, dh0, dc0, dW, dR, db) with dW flat like W.  Weight gradients are
    the sums over all steps of outer products, formed as one product per matrix
    after the layer's propagation is complete (Section 2.6).
    """
    x = np.asarray(x, dtype=dtype).reshape(T, B, I)
    h0 = np.zeros((L, B, H), dtype) if h0 is None else np.asarray(h0, dtype=dtype).reshape(L, B, H)
    c0 = np.zeros((L, B, H), dtype) if c0 is None else np.asarray(c0, dtype=dtype).reshape(L, B, H)
    Wl = [w.astype(dtype) for w in split_W(W, L, I, H)]
    R = np.asarray(R, dtype=dtype).reshape(L, 4 * H, H)
    dy = np.asarray(dy, dtype=dtype).reshape(T, B, H)
    dhT = np.zeros((L, B, H), dtype) if dhT is None else np.asarray(dhT, dtype=dtype).reshape(L, B, H)
    dcT = np.zeros((L, B, H), dtype) if dcT is None else np.asarray(dcT, dtype=dtype).reshape(L, B, H)
    gates, cs, hs = reserve["gates"], reserve["c"], reserve["h"]

    dWl = [None] * L
    dR = np.empty((L, 4 * H, H), dtype)
    db = np.empty((L, 4 * H), dtype)
    dh0 = np.empty((L, B, H), dtype)
    dc0 = np.empty((L, B, H), dtype)

    dout = dy  # gradient arriving at this layer's h_t from above
    for l in range(L - 1, -1, -1):
        Il = I if l == 0 else H
        inp = x if l == 0 else hs[l - 1]
        dA = np.empty((T, B, 4 * H), dtype)
        din = np.empty((T, B, Il), dtype)
        dh_rec = dhT[l].copy()  # gradient reaching h_t through step t+1 (or dhT at the end)
        dc_carry = dcT[l].copy()
        for t in range(T - 1, -1, -1):
            i = gates[l, t, :, 0 * H:1 * H]
            f = gates[l, t, :, 1 * H:2 * H]
            o = gates[l, t, :, 2 * H:3 * H]
            g = gates[l, t, :, 3 * H:4 * H]
            c_prev = cs[l, t - 1] if t > 0 else c0[l]
            tc = np.tanh(cs[l, t])
            dh = dout[t] + dh_rec
            do = dh * tc
            dc = dc_carry + dh * o * (1.0 - tc * tc)
            di = dc * g
            dg = dc * i
            df = dc * c_prev
            dc_carry = dc * f
            dA[t, :, 0 * H:1 * H] = di * i * (1.0 - i)
            dA[t, :, 1 * H:2 * H] = df * f * (1.0 - f)
            dA[t, :, 2 * H:3 * H] = do * o * (1.0 - o)
            dA[t, :, 3 * H:4 * H] = dg * (1.0 - g * g)
            din[t] = dA[t] @ Wl[l]
            dh_rec = dA[t] @ R[l]
        dh0[l] = dh_rec
        dc0[l] = dc_carry
        # weight update products, after the layer's propagation is complete
        h_prev_all = np.concatenate([h0[l][None], hs[l, :T - 1]], axis=0)  # h_{t-1} for t=0..T-1
        dA2 = dA.reshape(T * B, 4 * H)
        dWl[l] = dA2.T @ inp.reshape(T * B, Il)
        dR[l] = dA2.T @ h_prev_all.reshape(T * B, H)
        db[l] = dA2.sum(axis=0)
        dout = din
    dx = dout
    dW = np.concatenate([w.reshape(-1) for w in dWl])
    return dx, dh0, dc0, dW, dR, db


def loss(y, hT, cT, dy, dhT, dcT):
    """The scalar whose gradient lstm_backward returns."""
    s = float(np.sum(np.asarray(dy, np.float64) * y))
    if dhT is not None:
        s += float(np.sum(np.asarray(dhT, np.float64) * hT))
    if dcT is not None:
        s += float(np.sum(np.asarray(dcT, np.float64) * cT))
    return s
