"""Host logic of the ReLU parity comparison (CPU only): given gradients produced with an arbitrary admissible
assignment of slopes at tied pre-activations, the row-by-row search finds that assignment again, and gradients that
belong to no admissible assignment are not accepted."""
import numpy as np

from oracle import rnn_oracle as O
import test_gpu_rnn_cells as G
from parity import nerr


def tied_case(seed):
    L, T, B, I, H = 2, 3, 5, 4, 6
    d = {k: (None if v is None else v.astype(np.float64)) for k, v in G.make("relu", L, T, B, I, H, seed).items()}
    # put a few layer-0, step-0 units exactly on the kink: zero input row and state, zero bias for the unit
    d["x"][0, 1, :] = 0.0
    d["h0"][0, 1, :] = 0.0
    d["x"][0, 3, :] = 0.0
    d["h0"][0, 3, :] = 0.0
    d["b"][0, 2] = 0.0
    d["b"][0, 4] = 0.0
    y, hT, saved = O.rnn_forward("relu", L, T, B, I, H, d["x"], d["h0"], d["W"], d["R"], d["b"])
    ties = G.relu_ties(L, T, B, I, H, d, saved)
    return (L, T, B, I, H), d, saved, ties


def test_search_recovers_every_assignment():
    dims, d, saved, ties = tied_case(2)
    assert len(ties) == 4 and set(int(b) for b in ties[:, 2]) == {1, 3}
    names = ("dx", "dh0", "dW", "dR", "db")
    for bits in range(16):
        slope = (saved["h"] > 0).astype(np.float64)
        for j, ix in enumerate(ties):
            slope[tuple(ix)] = float((bits >> j) & 1)
        truth = O.rnn_backward("relu", *dims, d["x"], d["h0"], d["W"], d["R"], saved, d["dy"], d["dhT"], relu_slope=slope)
        got = [g.astype(np.float32) for g in truth]   # what a correct fp32 implementation would hand back
        found = G.relu_slopes_matching(*dims, d, saved, ties, got[0], got[1])
        ref = O.rnn_backward("relu", *dims, d["x"], d["h0"], d["W"], d["R"], saved, d["dy"], d["dhT"], relu_slope=found)
        for k, a, b in zip(names, got, ref):
            assert nerr(a, b) < 1e-6, (bits, k)


def test_a_wrong_gradient_is_not_accepted():
    dims, d, saved, ties = tied_case(2)
    truth = O.rnn_backward("relu", *dims, d["x"], d["h0"], d["W"], d["R"], saved, d["dy"], d["dhT"])
    # slope 1/2 at a tied unit is not one of the results an evaluation can produce
    slope = (saved["h"] > 0).astype(np.float64)
    slope[tuple(ties[0])] = 0.5
    wrong = O.rnn_backward("relu", *dims, d["x"], d["h0"], d["W"], d["R"], saved, d["dy"], d["dhT"], relu_slope=slope)
    found = G.relu_slopes_matching(*dims, d, saved, ties, wrong[0], wrong[1])
    ref = O.rnn_backward("relu", *dims, d["x"], d["h0"], d["W"], d["R"], saved, d["dy"], d["dhT"], relu_slope=found)
    assert max(nerr(a, b) for a, b in zip(wrong, ref)) > 1e-3
    # and an untied slope decided the other way is outside the set as well
    slope = (saved["h"] > 0).astype(np.float64)
    l, t, b, u = np.argwhere(saved["h"] > 0.5)[0]
    slope[l, t, b, u] = 0.0
    wrong = O.rnn_backward("relu", *dims, d["x"], d["h0"], d["W"], d["R"], saved, d["dy"], d["dhT"], relu_slope=slope)
    found = G.relu_slopes_matching(*dims, d, saved, ties, wrong[0], wrong[1])
    ref = O.rnn_backward("relu", *dims, d["x"], d["h0"], d["W"], d["R"], saved, d["dy"], d["dhT"], relu_slope=found)
    assert max(nerr(a, b) for a, b in zip(wrong, ref)) > 1e-3
    assert truth is not None
