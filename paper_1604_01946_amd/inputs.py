"""Seeded synthetic inputs for the LSTM workloads.

This module holds no LSTM arithmetic: it only draws random tensors with the
shapes and distributions of the paper's timing workloads (Section 2.5, Table 1:
four layers, hidden size 512, minibatch 64, 100 steps) and of the other shapes
this repository measures.  The same arrays are handed to the CPU oracle and to
the GPU library, so it is the one module both sides may import.

Draw order is fixed: x, then per layer (W_l, R_l, b_l), then h0, c0, dy, dhT, dcT.
Values are float64 draws rounded once to float32.
"""
from dataclasses import dataclass
import numpy as np


@dataclass(frozen=True)
class Config:
    name: str
    L: int
    T: int
    B: int
    I: int
    H: int
    state_std: float = 0.0   # std-dev of h0, c0 (0 => zeros)
    dstate_std: float = 0.0  # std-dev of dhT, dcT (0 => zeros)
    backward: bool = True

    @property
    def dims(self):
        return (self.L, self.T, self.B, self.I, self.H)

    def flops_per_pass(self):
        """2*4H*(I_l+H)*B*T summed over layers (one direction pass)."""
        tot = 0
        for l in range(self.L):
            Il = self.I if l == 0 else self.H
            tot += 2 * 4 * self.H * (Il + self.H) * self.B * self.T
        return tot


CONFIGS = {
    # the five measured shapes
    "cfg1": Config("cfg1", L=1, T=8, B=4, I=32, H=32),
    "cfg2": Config("cfg2", L=4, T=100, B=64, I=512, H=512, state_std=0.1, backward=False),
    "cfg3": Config("cfg3", L=4, T=100, B=64, I=512, H=512, state_std=0.1),
    "cfg4": Config("cfg4", L=4, T=50, B=32, I=2048, H=2048, state_std=0.1),
    "cfg5": Config("cfg5", L=2, T=500, B=1, I=256, H=256),
}


def w_sizes(L, I, H):
    return [4 * H * (I if l == 0 else H) for l in range(L)]


def make_inputs(cfg, seed=0):
    """Returns a dict of float32 numpy arrays in the C ABI's layouts."""
    L, T, B, I, H = cfg.dims
    rng = np.random.default_rng(seed)
    f32 = np.float32
    out = {}
    out["x"] = rng.standard_normal((T, B, I)).astype(f32)
    k = 1.0 / np.sqrt(H)
    Ws, Rs, bs = [], [], []
    for l in range(L):
        Il = I if l == 0 else H
        Ws.append(rng.uniform(-k, k, (4 * H, Il)).astype(f32).reshape(-1))
        Rs.append(rng.uniform(-k, k, (4 * H, H)).astype(f32))
        bs.append(rng.uniform(-0.1, 0.1, (4 * H,)).astype(f32))
    out["W"] = np.concatenate(Ws)
    out["R"] = np.stack(Rs)
    out["b"] = np.stack(bs)
    h0 = rng.standard_normal((L, B, H))
    c0 = rng.standard_normal((L, B, H))
    out["h0"] = (h0 * cfg.state_std).astype(f32)
    out["c0"] = (c0 * cfg.state_std).astype(f32)
    out["dy"] = rng.standard_normal((T, B, H)).astype(f32)
    dhT = rng.standard_normal((L, B, H))
    dcT = rng.standard_normal((L, B, H))
    out["dhT"] = (dhT * cfg.dstate_std).astype(f32)
    out["dcT"] = (dcT * cfg.dstate_std).astype(f32)
    return out
