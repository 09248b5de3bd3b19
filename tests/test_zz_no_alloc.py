"""lstm_forward_noalloc (scratch in a static device array, nothing allocated) against lstm_forward on the same inputs:
same kernels, so the outputs must be bit-identical; two calls in a row, the second with a smaller input; and the
rejection of shapes beyond the static array.  Named to be collected last: it must pass alone and after all others."""
import numpy as np
import pytest

from paper_1604_01946_amd.inputs import Config, make_inputs

pytestmark = pytest.mark.gpu

SCRATCH = 64 << 20


def _pair(cfg, seed, flags, inference):
    import torch
    from paper_1604_01946_amd import binding as B, runner
    d = make_inputs(cfg, seed)
    r = runner.LstmRunner(cfg.dims, d)
    assert r.workspace_bytes <= SCRATCH
    r.poison()
    B.check(r.forward(flags=flags, inference=inference), "lstm_forward")
    torch.cuda.synchronize()
    want = {k: getattr(r, k).clone() for k in ("y", "hT", "cT")}
    want_res = None if inference else r.reserve.clone()
    for t in (r.y, r.hT, r.cT):
        t.fill_(float("nan"))
    if not inference:
        r.reserve.view(torch.float32).fill_(float("nan"))
    r.workspace.view(torch.float32).fill_(float("nan"))   # the entry point must not touch a caller workspace
    print(f"noalloc case {cfg.dims} seed={seed} flags={flags} inference={inference}", flush=True)
    B.check(B.lstm_forward_noalloc(*cfg.dims, r.x, r.h0, r.c0, r.W, r.R, r.b, r.y, r.hT, r.cT,
                                   None if inference else r.reserve, flags=flags), "lstm_forward_noalloc")
    torch.cuda.synchronize()
    for k, v in want.items():
        assert torch.equal(getattr(r, k), v), (cfg.name, k)
    if not inference:
        assert torch.equal(r.reserve, want_res), (cfg.name, "reserve")
    assert torch.isnan(r.workspace.view(torch.float32)).all()
    return r


@pytest.mark.parametrize("flags", [0, 4, 6], ids=["auto", "step", "persistent"])
def test_two_calls_in_a_row_the_second_smaller(flags):
    import torch
    from paper_1604_01946_amd import binding as B
    assert torch.cuda.is_available()
    big = Config("na_big", L=2, T=12, B=24, I=128, H=256, state_std=0.3)
    small = Config("na_small", L=1, T=5, B=7, I=128, H=256, state_std=0.3)
    if flags == 6 and B.lstm_auto_path(*small.dims, 0) != 6:
        pytest.skip("persistent path does not take these shapes")
    assert B.lstm_init() == B.LSTM_OK
    _pair(big, 3, flags, inference=False)
    _pair(small, 4, flags, inference=False)
    _pair(big, 5, flags, inference=True)
    _pair(small, 6, flags, inference=True)


def test_odd_shape_and_ragged_tiles():
    _pair(Config("na_odd", L=3, T=4, B=5, I=24, H=40, state_std=0.5), 7, 0, inference=False)
    _pair(Config("na_odd2", L=2, T=3, B=70, I=36, H=100, state_std=0.5), 8, 0, inference=True)


def test_shapes_beyond_the_static_array_are_rejected():
    import torch
    from paper_1604_01946_amd import binding as B
    cfg = Config("na_too_big", L=4, T=100, B=64, I=512, H=512)
    assert B.lstm_workspace_bytes(*cfg.dims) > SCRATCH
    a = torch.zeros(64, device="cuda:0")
    st = B.lstm_forward_noalloc(*cfg.dims, a, None, None, a, a, a, a, None, None, None, flags=0)
    assert st == B.LSTM_BUFFER_TOO_SMALL
    assert "static array" in B.lstm_last_error()
    assert B.lstm_forward_noalloc(2, 4, 4, 16, 64, a, None, None, a, a, a, a, None, None, None,
                                  flags=B.LSTM_PATH_WAVEFRONT) == B.LSTM_UNSUPPORTED
