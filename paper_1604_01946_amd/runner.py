"""Device-memory plumbing around the C ABI: uploads a workload, owns the output,
reserve and workspace tensors, and calls lstm_forward / lstm_backward.  PyTorch is
used for device memory and streams only."""
import numpy as np
import torch

from . import binding as B_


class LstmRunner:
    def __init__(self, dims, arrays, device="cuda:0", with_states=True, with_dstates=True):
        """dims = (L,T,B,I,H); arrays = dict of float32 numpy arrays from inputs.make_inputs."""
        self.dims = tuple(int(v) for v in dims)
        L, T, B, I, H = self.dims
        self.dev = torch.device(device)
        up = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(self.dev)
        self.x, self.W, self.R, self.b = up(arrays["x"]), up(arrays["W"]), up(arrays["R"]), up(arrays["b"])
        self.h0 = up(arrays["h0"]) if with_states else None
        self.c0 = up(arrays["c0"]) if with_states else None
        self.dy = up(arrays["dy"]) if "dy" in arrays else None
        self.dhT = up(arrays["dhT"]) if with_dstates and "dhT" in arrays else None
        self.dcT = up(arrays["dcT"]) if with_dstates and "dcT" in arrays else None
        f = lambda *s: torch.empty(*s, dtype=torch.float32, device=self.dev)
        self.y, self.hT, self.cT = f(T, B, H), f(L, B, H), f(L, B, H)
        self.dx, self.dh0, self.dc0 = f(T, B, I), f(L, B, H), f(L, B, H)
        self.dW, self.dR, self.db = torch.empty_like(self.W), torch.empty_like(self.R), torch.empty_like(self.b)
        self.reserve_bytes = B_.lstm_reserve_bytes(*self.dims)
        self.workspace_bytes = B_.lstm_workspace_bytes(*self.dims)
        self.reserve = torch.empty(self.reserve_bytes, dtype=torch.uint8, device=self.dev)
        self.workspace = torch.empty(self.workspace_bytes, dtype=torch.uint8, device=self.dev)

    def forward(self, flags=0, stream=None, inference=False, want_states=True):
        return B_.lstm_forward(*self.dims, self.x, self.h0, self.c0, self.W, self.R, self.b, self.y,
                               self.hT if want_states else None, self.cT if want_states else None,
                               None if inference else self.reserve, self.workspace, self.workspace_bytes,
                               stream=stream, flags=flags)

    def backward(self, flags=0, stream=None, want_dx=True, want_dstates=True):
        return B_.lstm_backward(*self.dims, self.x, self.h0, self.c0, self.W, self.R, self.reserve,
                                self.dy, self.dhT, self.dcT, self.dx if want_dx else None,
                                self.dh0 if want_dstates else None, self.dc0 if want_dstates else None,
                                self.dW, self.dR, self.db, self.workspace, self.workspace_bytes,
                                stream=stream, flags=flags)

    def poison(self):
        """NaN-fills outputs, reserve and workspace so that a read-before-write shows."""
        for t in (self.y, self.hT, self.cT, self.dx, self.dh0, self.dc0, self.dW, self.dR, self.db):
            t.fill_(float("nan"))
        self.reserve.view(torch.float32).fill_(float("nan"))
        self.workspace.view(torch.float32).fill_(float("nan"))

    def fwd_outputs(self):
        return {k: getattr(self, k).cpu().numpy() for k in ("y", "hT", "cT")}

    def bwd_outputs(self):
        return {k: getattr(self, k).cpu().numpy() for k in ("dx", "dh0", "dc0", "dW", "dR", "db")}
