"""Pins of the single-gate RNN / GRU oracle against what the mathematics fixes (the paper prints neither equations
nor a worked example for these cells, see the oracle's header for the conventions): closed forms, a hand-expanded
scalar step, central finite differences, torch.nn.RNN / torch.nn.GRU in float64 as library routines, composition
identities.  CPU only."""
import numpy as np
import pytest

from oracle import rnn_oracle as O


def rand_case(cell, L, T, B, I, H, seed):
    rng = np.random.default_rng(seed)
    G = O.CELLS[cell] * H
    nw = G * I + (L - 1) * G * H
    return dict(x=rng.standard_normal((T, B, I)), W=rng.uniform(-0.4, 0.4, nw), R=rng.uniform(-0.4, 0.4, (L, G, H)),
                b=rng.uniform(-0.3, 0.3, (L, G)), h0=0.5 * rng.standard_normal((L, B, H)),
                dy=rng.standard_normal((T, B, H)), dhT=0.7 * rng.standard_normal((L, B, H)))


def test_closed_form_zero_weights():
    L, T, B, I, H = 2, 7, 3, 4, 5
    for cell in ("relu", "tanh", "gru"):
        d = rand_case(cell, L, T, B, I, H, 1)
        d["W"][:] = 0
        d["R"][:] = 0
        y, hT, _ = O.rnn_forward(cell, L, T, B, I, H, d["x"], d["h0"], d["W"], d["R"], d["b"])
        bl = d["b"][L - 1]
        if cell == "relu":
            assert np.allclose(y, np.broadcast_to(np.maximum(bl, 0), (T, B, H)), atol=1e-14)
        elif cell == "tanh":
            assert np.allclose(y, np.broadcast_to(np.tanh(bl), (T, B, H)), atol=1e-14)
        else:  # h_t = n + z^(t+1) (h0 - n): a geometric approach to the constant candidate
            z, n = 1 / (1 + np.exp(-bl[H:2 * H])), np.tanh(bl[2 * H:])
            for t in range(T):
                assert np.allclose(y[t], n + z ** (t + 1) * (d["h0"][L - 1] - n), atol=1e-13)
            assert np.allclose(hT[L - 1], y[T - 1])


def test_gru_scalar_step_by_hand():
    x, h0, wr, wz, wn, rr, rz, rn, br, bz, bn = 0.7, -0.3, 0.5, -0.2, 0.9, 0.4, 0.1, -0.6, 0.05, -0.1, 0.2
    sig = lambda v: 1 / (1 + np.exp(-v))
    r = sig(wr * x + rr * h0 + br)
    z = sig(wz * x + rz * h0 + bz)
    n = np.tanh(wn * x + bn + r * (rn * h0))
    h = (1 - z) * n + z * h0
    y, hT, _ = O.rnn_forward("gru", 1, 1, 1, 1, 1, [[[x]]], [[[h0]]], [wr, wz, wn], [[[rr], [rz], [rn]]], [[br, bz, bn]])
    assert abs(y[0, 0, 0] - h) < 1e-15 and abs(hT[0, 0, 0] - h) < 1e-15


@pytest.mark.parametrize("cell", ["tanh", "gru", "relu"])
@pytest.mark.parametrize("dims", [(1, 3, 2, 3, 4), (3, 4, 2, 5, 3)])
def test_backward_matches_central_differences(cell, dims):
    L, T, B, I, H = dims
    d = rand_case(cell, L, T, B, I, H, 7)
    if cell == "relu":  # keep pre-activations away from the kink
        d["b"] += 0.5
    args = lambda dd: (cell, L, T, B, I, H, dd["x"], dd["h0"], dd["W"], dd["R"], dd["b"])
    y, hT, saved = O.rnn_forward(*args(d))
    dx, dh0, dW, dR, db = O.rnn_backward(cell, L, T, B, I, H, d["x"], d["h0"], d["W"], d["R"], saved, d["dy"], d["dhT"])
    grads = {"x": dx, "h0": dh0, "W": dW, "R": dR, "b": db}
    rng = np.random.default_rng(3)
    eps = 1e-6
    for name, g in grads.items():
        flat = d[name].reshape(-1)
        for idx in rng.choice(flat.size, size=min(12, flat.size), replace=False):
            old = flat[idx]
            vals = []
            for s in (+1, -1):
                flat[idx] = old + s * eps
                yy, hh, _ = O.rnn_forward(*args(d))
                vals.append(O.loss(yy, hh, d["dy"], d["dhT"]))
            flat[idx] = old
            num = (vals[0] - vals[1]) / (2 * eps)
            assert abs(num - g.reshape(-1)[idx]) < 2e-7 * max(1.0, abs(num)), (cell, name, idx, num, g.reshape(-1)[idx])


@pytest.mark.parametrize("cell", ["relu", "tanh", "gru"])
def test_against_torch_float64(cell):
    torch = pytest.importorskip("torch")
    L, T, B, I, H = 2, 5, 3, 6, 4
    d = rand_case(cell, L, T, B, I, H, 11)
    G = O.CELLS[cell] * H
    if cell == "gru":
        net = torch.nn.GRU(I, H, num_layers=L).double()
    else:
        net = torch.nn.RNN(I, H, num_layers=L, nonlinearity=cell).double()
    Ws = O.split_W(d["W"], cell, L, I, H)
    with torch.no_grad():
        for l in range(L):
            getattr(net, f"weight_ih_l{l}").copy_(torch.from_numpy(Ws[l]))
            getattr(net, f"weight_hh_l{l}").copy_(torch.from_numpy(d["R"][l]))
            getattr(net, f"bias_ih_l{l}").copy_(torch.from_numpy(d["b"][l]))
            getattr(net, f"bias_hh_l{l}").zero_()
    x = torch.from_numpy(d["x"]).requires_grad_(True)
    h0 = torch.from_numpy(d["h0"]).requires_grad_(True)
    out, hn = net(x, h0)
    (out * torch.from_numpy(d["dy"])).sum().add((hn * torch.from_numpy(d["dhT"])).sum()).backward()
    y, hT, saved = O.rnn_forward(cell, L, T, B, I, H, d["x"], d["h0"], d["W"], d["R"], d["b"])
    dx, dh0, dW, dR, db = O.rnn_backward(cell, L, T, B, I, H, d["x"], d["h0"], d["W"], d["R"], saved, d["dy"], d["dhT"])
    assert np.allclose(y, out.detach().numpy(), atol=1e-13) and np.allclose(hT, hn.detach().numpy(), atol=1e-13)
    assert np.allclose(dx, x.grad.numpy(), atol=1e-12) and np.allclose(dh0, h0.grad.numpy(), atol=1e-12)
    dWs = O.split_W(dW, cell, L, I, H)
    for l in range(L):
        assert np.allclose(dWs[l], getattr(net, f"weight_ih_l{l}").grad.numpy(), atol=1e-12)
        assert np.allclose(dR[l], getattr(net, f"weight_hh_l{l}").grad.numpy(), atol=1e-12)
        assert np.allclose(db[l], getattr(net, f"bias_ih_l{l}").grad.numpy(), atol=1e-12)


@pytest.mark.parametrize("cell", ["tanh", "gru"])
def test_split_T_and_layer_stack(cell):
    L, T, B, I, H = 2, 6, 2, 3, 3
    d = rand_case(cell, L, T, B, I, H, 5)
    y, hT, _ = O.rnn_forward(cell, L, T, B, I, H, d["x"], d["h0"], d["W"], d["R"], d["b"])
    y1, h1, _ = O.rnn_forward(cell, L, 4, B, I, H, d["x"][:4], d["h0"], d["W"], d["R"], d["b"])
    y2, h2, _ = O.rnn_forward(cell, L, 2, B, I, H, d["x"][4:], h1, d["W"], d["R"], d["b"])
    assert np.allclose(np.concatenate([y1, y2]), y, atol=1e-14) and np.allclose(h2, hT, atol=1e-14)
    G = O.CELLS[cell] * H
    Ws = O.split_W(d["W"], cell, L, I, H)
    ya, ha, _ = O.rnn_forward(cell, 1, T, B, I, H, d["x"], d["h0"][:1], Ws[0].ravel(), d["R"][:1], d["b"][:1])
    yb, hb, _ = O.rnn_forward(cell, 1, T, B, H, H, ya, d["h0"][1:], Ws[1].ravel(), d["R"][1:], d["b"][1:])
    assert np.allclose(yb, y, atol=1e-14) and np.allclose(np.stack([ha[0], hb[0]]), hT, atol=1e-14)


@pytest.mark.parametrize("cell", ["relu", "tanh", "gru"])
def test_zero_padded_hidden_units_change_nothing(cell):
    """A hidden unit with zero weights, bias and initial state stays at h = 0 (GRU: r = z = 1/2, n = tanh(0)) and
    takes zero gradients, so the network padded from H to Hp gives the given network's results (the library computes
    some hidden sizes this way)."""
    L, T, B, I, H, Hp = 3, 4, 3, 5, 6, 8
    d = rand_case(cell, L, T, B, I, H, seed=31)
    ng = O.CELLS[cell]
    y, hT, saved = O.rnn_forward(cell, L, T, B, I, H, d["x"], d["h0"], d["W"], d["R"], d["b"])
    g = O.rnn_backward(cell, L, T, B, I, H, d["x"], d["h0"], d["W"], d["R"], saved, d["dy"], d["dhT"])
    Wp = []
    for l, Wl in enumerate(O.split_W(d["W"], cell, L, I, H)):
        Il = Wl.shape[1]
        blk = np.zeros((ng, Hp, Il if l == 0 else Hp))
        blk[:, :H, :Il] = Wl.reshape(ng, H, Il)
        Wp.append(blk.ravel())
    Rp = np.zeros((L, ng, Hp, Hp)); Rp[:, :, :H, :H] = d["R"].reshape(L, ng, H, H)
    bp = np.zeros((L, ng, Hp)); bp[:, :, :H] = d["b"].reshape(L, ng, H)
    pad = lambda a: np.concatenate([a, np.zeros(a.shape[:-1] + (Hp - H,))], axis=-1)
    W2, R2, b2 = np.concatenate(Wp), Rp.reshape(L, ng * Hp, Hp), bp.reshape(L, ng * Hp)
    yp, hTp, savedp = O.rnn_forward(cell, L, T, B, I, Hp, d["x"], pad(d["h0"]), W2, R2, b2)
    assert np.array_equal(yp[..., :H], y) and np.array_equal(hTp[..., :H], hT)
    assert not yp[..., H:].any() and not hTp[..., H:].any()
    dx, dh0, dW, dR, db = O.rnn_backward(cell, L, T, B, I, Hp, d["x"], pad(d["h0"]), W2, R2, savedp, pad(d["dy"]), pad(d["dhT"]))
    assert np.allclose(dx, g[0], atol=1e-14) and np.allclose(dh0[..., :H], g[1], atol=1e-14) and not dh0[..., H:].any()
    for l, (full, ref) in enumerate(zip(O.split_W(dW, cell, L, I, Hp), O.split_W(g[2], cell, L, I, H))):
        Il = ref.shape[1]
        blk = full.reshape(ng, Hp, -1)
        assert np.allclose(blk[:, :H, :Il].reshape(ng * H, Il), ref, atol=1e-13) and not blk[:, H:, :].any()
    dRb = dR.reshape(L, ng, Hp, Hp)
    assert np.allclose(dRb[:, :, :H, :H].reshape(L, ng * H, H), g[3], atol=1e-13) and not dRb[:, :, H:, :].any() and not dRb[:, :, :, H:].any()
    dbb = db.reshape(L, ng, Hp)
    assert np.allclose(dbb[:, :, :H].reshape(L, ng * H), g[4], atol=1e-13) and not dbb[:, :, H:].any()


def test_relu_slope_argument_reproduces_default_and_one_sided_derivatives():
    """The optional ReLU slope of rnn_backward: (1) given the network's own decisions (h > 0) it changes nothing;
    (2) at a pre-activation of exactly 0 the two admissible slopes are the one-sided derivatives of the loss: a
    two-layer, two-step network whose unit (layer 0, step 0, row 0, unit 1) sits exactly on the kink (zero input row,
    zero initial state, zero bias), differentiated with respect to that bias from the right and from the left."""
    L, T, B, I, H = 2, 2, 2, 3, 3
    d = rand_case("relu", L, T, B, I, H, 21)
    d["b"] += 0.2
    y, hT, saved = O.rnn_forward("relu", L, T, B, I, H, d["x"], d["h0"], d["W"], d["R"], d["b"])
    ref = O.rnn_backward("relu", L, T, B, I, H, d["x"], d["h0"], d["W"], d["R"], saved, d["dy"], d["dhT"])
    same = O.rnn_backward("relu", L, T, B, I, H, d["x"], d["h0"], d["W"], d["R"], saved, d["dy"], d["dhT"],
                          relu_slope=(saved["h"] > 0).astype(np.float64))
    for a, b in zip(ref, same):
        assert np.array_equal(a, b)

    d["x"][0, 0, :] = 0.0
    d["h0"][0, 0, :] = 0.0
    d["b"][0, 1] = 0.0
    # every other pre-activation must be well away from 0 so that the finite step crosses no second kink
    y, hT, saved = O.rnn_forward("relu", L, T, B, I, H, d["x"], d["h0"], d["W"], d["R"], d["b"])
    a = O.relu_preactivations(L, T, B, I, H, d["x"], d["h0"], d["W"], d["R"], d["b"], saved)
    assert a[0, 0, 0, 1] == 0.0
    others = np.abs(a).reshape(-1)
    assert np.sort(others)[1] > 1e-3
    eps = 1e-7

    def loss_at(delta):
        bb = d["b"].copy()
        bb[0, 1] += delta
        yy, hh, _ = O.rnn_forward("relu", L, T, B, I, H, d["x"], d["h0"], d["W"], d["R"], bb)
        return O.loss(yy, hh, d["dy"], d["dhT"])

    right = (loss_at(eps) - loss_at(0.0)) / eps
    left = (loss_at(0.0) - loss_at(-eps)) / eps
    assert abs(right - left) > 1e-3  # the kink really is one for this loss
    for slope, want in ((1.0, right), (0.0, left)):
        m = (saved["h"] > 0).astype(np.float64)
        m[0, 0, 0, 1] = slope
        db = O.rnn_backward("relu", L, T, B, I, H, d["x"], d["h0"], d["W"], d["R"], saved, d["dy"], d["dhT"], relu_slope=m)[4]
        assert abs(db[0, 1] - want) < 1e-6 * max(1.0, abs(want)), (slope, db[0, 1], want)


def test_relu_preactivations_reproduce_hidden_states():
    L, T, B, I, H = 3, 4, 2, 5, 4
    d = rand_case("relu", L, T, B, I, H, 5)
    y, hT, saved = O.rnn_forward("relu", L, T, B, I, H, d["x"], d["h0"], d["W"], d["R"], d["b"])
    a = O.relu_preactivations(L, T, B, I, H, d["x"], d["h0"], d["W"], d["R"], d["b"], saved)
    assert np.allclose(np.maximum(a, 0.0), saved["h"], rtol=0, atol=1e-13)
