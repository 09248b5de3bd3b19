"""Path autotuner: times the paths that take a shape and pins the fastest for LSTM_PATH_AUTO.

Sections 2.3 and 3.2 of arXiv 1604.01946 observe that which strategy pays (batched inputs, stream overlap,
and here weights resident on chip) depends on hidden size, minibatch and depth, and that choosing is not
trivial.  The library's built-in rule is a fixed heuristic; this helper measures instead.  Timing only, on
synthetic device data of the given shape; the choice is registered with lstm_set_path and lasts until
lstm_shutdown or the end of the process.

    python -m paper_1604_01946_amd.autotune L T B I H
"""
import math
import sys

import torch

from . import binding as B_

CANDIDATES = (B_.LSTM_PATH_FUSED, B_.LSTM_PATH_STEP, B_.LSTM_PATH_WAVEFRONT, B_.LSTM_PATH_PERSISTENT)


def tune(L, T, B, I, H, iters=3, device="cuda:0", register=True):
    """Returns {"forward": {path name: ms}, "backward": {...}, "best": (forward path, backward path)}."""
    dev = torch.device(device)
    dims = (L, T, B, I, H)
    g = torch.Generator(device=dev)
    g.manual_seed(0)
    rnd = lambda *s: torch.randn(*s, device=dev, generator=g, dtype=torch.float32)
    uni = lambda n, a: (torch.rand(n, device=dev, generator=g, dtype=torch.float32) * 2 - 1) * a
    nw = 4 * H * I + (L - 1) * 4 * H * H
    x, dy = rnd(T, B, I), rnd(T, B, H)
    W, R, b = uni(nw, 1 / math.sqrt(H)), uni(L * 4 * H * H, 1 / math.sqrt(H)), uni(L * 4 * H, 0.1)
    h0, c0 = rnd(L, B, H) * 0.1, rnd(L, B, H) * 0.1
    f = lambda *s: torch.empty(*s, device=dev, dtype=torch.float32)
    y, hT, cT, dx, dh0, dc0 = f(T, B, H), f(L, B, H), f(L, B, H), f(T, B, I), f(L, B, H), f(L, B, H)
    dW, dR, db = torch.empty_like(W), torch.empty_like(R), torch.empty_like(b)
    rb, wb = B_.lstm_reserve_bytes(*dims), B_.lstm_workspace_bytes(*dims)
    res = torch.empty(rb, dtype=torch.uint8, device=dev)
    ws = torch.empty(wb, dtype=torch.uint8, device=dev)

    def fwd(path):
        return B_.lstm_forward(*dims, x, h0, c0, W, R, b, y, hT, cT, res, ws, wb, flags=path)

    def bwd(path):
        return B_.lstm_backward(*dims, x, h0, c0, W, R, res, dy, None, None, dx, dh0, dc0, dW, dR, db, ws, wb, flags=path)

    def time_it(fn, path):
        st = fn(path)
        if st == B_.LSTM_UNSUPPORTED:
            return None
        B_.check(st, "autotune")
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(iters):
            B_.check(fn(path), "autotune")
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / iters

    out = {"forward": {}, "backward": {}}
    # Section 2.3: how many steps to batch in one input product is "not trivial" to choose -- measure a few chunk
    # counts of the stream wavefront (forward + backward, one setting for both) and keep the best
    if L > 1:
        B_.check(fwd(B_.LSTM_PATH_STEP), "autotune")
        per_chunks = {}
        for c in sorted({0, 1, 2, 4, 8, 16} & set(range(0, T + 1))):
            B_.check(B_.lstm_set_wavefront_chunks(*dims, c), "lstm_set_wavefront_chunks")
            tf, tb = time_it(fwd, B_.LSTM_PATH_WAVEFRONT), time_it(bwd, B_.LSTM_PATH_WAVEFRONT)
            per_chunks[c] = tf + tb
        best_c = min(per_chunks, key=per_chunks.get)
        B_.check(B_.lstm_set_wavefront_chunks(*dims, best_c if register else 0), "lstm_set_wavefront_chunks")
        out["wavefront_chunks"] = {("default" if c == 0 else c): ms for c, ms in per_chunks.items()}
        out["best_chunks"] = "default" if best_c == 0 else best_c
    for p in CANDIDATES:
        ms = time_it(fwd, p)
        if ms is not None:
            out["forward"][B_.PATH_NAMES[p]] = ms
    B_.check(fwd(B_.LSTM_PATH_STEP), "autotune")  # a reserve for the backward candidates
    for p in CANDIDATES:
        ms = time_it(bwd, p)
        if ms is not None:
            out["backward"][B_.PATH_NAMES[p]] = ms
    by_name = {v: k for k, v in B_.PATH_NAMES.items()}
    best = tuple(min(out[k], key=out[k].get) for k in ("forward", "backward"))
    out["best"] = best
    if register:
        B_.check(B_.lstm_set_path(*dims, 0, by_name[best[0]]), "lstm_set_path")
        B_.check(B_.lstm_set_path(*dims, 1, by_name[best[1]]), "lstm_set_path")
    return out


if __name__ == "__main__":
    if len(sys.argv) != 6 or not all(v.isdigit() for v in sys.argv[1:6]):
        sys.exit("usage: python -m paper_1604_01946_amd.autotune L T B I H")
    dims = [int(v) for v in sys.argv[1:6]]
    r = tune(*dims)
    for k in ("forward", "backward"):
        print(k, {n: round(v, 3) for n, v in r[k].items()})
    if "wavefront_chunks" in r:
        print("wavefront chunks (fwd+bwd ms)", {n: round(v, 3) for n, v in r["wavefront_chunks"].items()}, "best", r["best_chunks"])
    print("best", r["best"])
