"""Figure-1-style sweep (Section 3.2 of arXiv 1604.01946 plots throughput against hidden size for several
minibatch sizes, one layer against four): forward+backward time of the library's automatic path over a grid of
hidden sizes and minibatch sizes, as a Markdown table.  Timing only: inputs are drawn on the device, nothing is
compared (parity at these shapes is the job of the tests).

    python -m paper_1604_01946_amd.sweep [--hidden 256,512,1024,2048] [--batch 32,64,128,256] [--layers 1,4] [--T 100]
                                         [--cell lstm|gru|tanh|relu] [--rungs]

`--cell` times the other recurrent units of Section 3.3 through rnn_forward / rnn_backward instead; `--rungs` times
the forward pass on every rung of the optimisation ladder (the per-optimisation curves of Figure 1).
"""
import argparse
import math

import torch

from . import binding as B_


def run_shape(L, T, B, H, iters, dev):
    I = H
    g = torch.Generator(device=dev)
    g.manual_seed(0)
    rnd = lambda *s: torch.randn(*s, device=dev, generator=g, dtype=torch.float32)
    uni = lambda n, a: (torch.rand(n, device=dev, generator=g, dtype=torch.float32) * 2 - 1) * a
    x, dy = rnd(T, B, I), rnd(T, B, H)
    W, R = uni(L * 4 * H * H, 1 / math.sqrt(H)), uni(L * 4 * H * H, 1 / math.sqrt(H))
    b = uni(L * 4 * H, 0.1)
    h0, c0 = rnd(L, B, H) * 0.1, rnd(L, B, H) * 0.1
    f = lambda *s: torch.empty(*s, device=dev, dtype=torch.float32)
    y, hT, cT, dx, dh0, dc0 = f(T, B, H), f(L, B, H), f(L, B, H), f(T, B, I), f(L, B, H), f(L, B, H)
    dW, dR, db = torch.empty_like(W), torch.empty_like(R), torch.empty_like(b)
    dims = (L, T, B, I, H)
    rb, wb = B_.lstm_reserve_bytes(*dims), B_.lstm_workspace_bytes(*dims)
    res = torch.empty(rb, dtype=torch.uint8, device=dev)
    ws = torch.empty(wb, dtype=torch.uint8, device=dev)

    def step():
        B_.check(B_.lstm_forward(*dims, x, h0, c0, W, R, b, y, hT, cT, res, ws, wb), "forward")
        B_.check(B_.lstm_backward(*dims, x, h0, c0, W, R, res, dy, None, None, dx, dh0, dc0, dW, dR, db, ws, wb), "backward")

    step()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(iters):
        step()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / iters
    flop = 3 * L * 2 * 4 * H * (I + H) * B * T
    path = (B_.lstm_auto_path(*dims, 0), B_.lstm_auto_path(*dims, 1))
    return ms, flop / ms / 1e9, path, bool(torch.isfinite(dW).all().item())


def run_rungs(L, T, B, H, iters, dev):
    """Forward-pass time of every rung of the optimisation ladder (the quantity Figure 1 plots), in ms; None where a
    path does not take the shape."""
    I = H
    g = torch.Generator(device=dev)
    g.manual_seed(0)
    rnd = lambda *s: torch.randn(*s, device=dev, generator=g, dtype=torch.float32)
    uni = lambda n, a: (torch.rand(n, device=dev, generator=g, dtype=torch.float32) * 2 - 1) * a
    x = rnd(T, B, I)
    W, R = uni(L * 4 * H * H, 1 / math.sqrt(H)), uni(L * 4 * H * H, 1 / math.sqrt(H))
    b = uni(L * 4 * H, 0.1)
    h0, c0 = rnd(L, B, H) * 0.1, rnd(L, B, H) * 0.1
    f = lambda *s: torch.empty(*s, device=dev, dtype=torch.float32)
    y, hT, cT = f(T, B, H), f(L, B, H), f(L, B, H)
    dims = (L, T, B, I, H)
    rb, wb = B_.lstm_reserve_bytes(*dims), B_.lstm_workspace_bytes(*dims)
    res = torch.empty(rb, dtype=torch.uint8, device=dev)
    ws = torch.empty(wb, dtype=torch.uint8, device=dev)
    out = []
    for path in (B_.LSTM_PATH_NAIVE, B_.LSTM_PATH_GROUPED, B_.LSTM_PATH_FUSED, B_.LSTM_PATH_STEP, B_.LSTM_PATH_WAVEFRONT,
                 B_.LSTM_PATH_PERSISTENT):
        st = B_.lstm_forward(*dims, x, h0, c0, W, R, b, y, hT, cT, res, ws, wb, flags=path)
        if st != B_.LSTM_OK:
            out.append(None)
            continue
        torch.cuda.synchronize()
        n = 1 if path <= B_.LSTM_PATH_FUSED else iters
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(n):
            B_.check(B_.lstm_forward(*dims, x, h0, c0, W, R, b, y, hT, cT, res, ws, wb, flags=path), "forward")
        e1.record()
        torch.cuda.synchronize()
        out.append(e0.elapsed_time(e1) / n)
    return out, L * 2 * 4 * H * (I + H) * B * T


def run_shape_rnn(cell, L, T, B, H, iters, dev):
    I = H
    gates = 3 if cell == "gru" else 1
    G = gates * H
    g = torch.Generator(device=dev)
    g.manual_seed(0)
    rnd = lambda *s: torch.randn(*s, device=dev, generator=g, dtype=torch.float32)
    uni = lambda n, a: (torch.rand(n, device=dev, generator=g, dtype=torch.float32) * 2 - 1) * a
    x, dy = rnd(T, B, I), rnd(T, B, H)
    W, R, b = uni(L * G * H, 1 / math.sqrt(H)), uni(L * G * H, 1 / math.sqrt(H)), uni(L * G, 0.1)
    h0 = rnd(L, B, H) * 0.1
    f = lambda *s: torch.empty(*s, device=dev, dtype=torch.float32)
    y, hT, dx, dh0 = f(T, B, H), f(L, B, H), f(T, B, I), f(L, B, H)
    dW, dR, db = torch.empty_like(W), torch.empty_like(R), torch.empty_like(b)
    dims = (B_.RNN_CELLS[cell], L, T, B, I, H)
    rb, wb = B_.rnn_reserve_bytes(*dims), B_.rnn_workspace_bytes(*dims)
    res = torch.empty(rb, dtype=torch.uint8, device=dev)
    ws = torch.empty(wb, dtype=torch.uint8, device=dev)

    def step():
        B_.check(B_.rnn_forward(*dims, x, h0, W, R, b, y, hT, res, ws, wb), "forward")
        B_.check(B_.rnn_backward(*dims, x, h0, W, R, res, dy, None, dx, dh0, dW, dR, db, ws, wb), "backward")

    step()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(iters):
        step()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / iters
    flop = 3 * L * 2 * G * (I + H) * B * T
    return ms, flop / ms / 1e9, None, bool(torch.isfinite(dW).all().item())


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--hidden", default="256,512,1024,2048")
    ap.add_argument("--batch", default="32,64,128,256")
    ap.add_argument("--layers", default="1,4")
    ap.add_argument("--T", type=int, default=100)
    ap.add_argument("--iters", type=int, default=3)
    ap.add_argument("--cell", default="lstm", choices=["lstm", "gru", "tanh", "relu"])
    ap.add_argument("--rungs", action="store_true",
                    help="forward pass on every rung of the ladder (naive ... persistent) instead of the automatic path")
    a = ap.parse_args()
    dev = torch.device("cuda:0")
    names = B_.PATH_NAMES
    if a.rungs:
        print(f"T = {a.T}, I = H, fp32, forward pass, TFLOP/s per rung of the ladder (a dash: the path does not take the shape)\n")
        for L in [int(v) for v in a.layers.split(",")]:
            for B in [int(v) for v in a.batch.split(",")]:
                print(f"L = {L}, B = {B}\n\n| H | naive | grouped | fused | step | wavefront | persistent |\n|---|---|---|---|---|---|---|")
                for H in [int(v) for v in a.hidden.split(",")]:
                    ms, flop = run_rungs(L, a.T, B, H, a.iters, dev)
                    print(f"| {H} | " + " | ".join("-" if m is None else f"{flop / m / 1e9:.1f}" for m in ms) + " |", flush=True)
                print()
        return
    what = "forward/backward path" if a.cell == "lstm" else f"cell {a.cell}"
    print(f"T = {a.T}, I = H, fp32, forward+backward, TFLOP/s by the 3-pass count (ms per iteration; {what})\n")
    for L in [int(v) for v in a.layers.split(",")]:
        Bs = [int(v) for v in a.batch.split(",")]
        print(f"L = {L}\n\n| H | " + " | ".join(f"B={b}" for b in Bs) + " |\n|---|" + "---|" * len(Bs))
        for H in [int(v) for v in a.hidden.split(",")]:
            cells = []
            for B in Bs:
                if a.cell == "lstm":
                    ms, tf, path, ok = run_shape(L, a.T, B, H, a.iters, dev)
                    tag = f"; {names.get(path[0], path[0])}/{names.get(path[1], path[1])}"
                else:
                    ms, tf, path, ok = run_shape_rnn(a.cell, L, a.T, B, H, a.iters, dev)
                    tag = ""
                cells.append(f"{tf:.1f} ({ms:.2f}{tag}{'' if ok else '; NON-FINITE'})")
            print(f"| {H} | " + " | ".join(cells) + " |", flush=True)
        print()


if __name__ == "__main__":
    main()
