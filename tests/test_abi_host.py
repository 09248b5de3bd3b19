"""Host-side checks that need no GPU: the library loads, exports every symbol the header
declares, sizes its buffers as documented, and rejects bad arguments before any GPU work."""
import os
import re
import ctypes
import pytest

from paper_1604_01946_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "lstm.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(lstm_[a-z0-9_]+)\s*\(", hdr))
    assert declared == set(B.EXPORTS), declared ^ set(B.EXPORTS)
    lib = B.library()
    for name in declared:
        assert hasattr(lib, name), name


def test_library_exports_every_symbol_of_the_rnn_header():
    hdr = open(os.path.join(ROOT, "include", "rnn.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(rnn_[a-z0-9_]+)\s*\(", hdr))
    assert declared == set(B.RNN_EXPORTS), declared ^ set(B.RNN_EXPORTS)
    lib = B.library()
    for name in declared:
        assert hasattr(lib, name), name


def test_rnn_size_queries_and_argument_checks():
    assert B.rnn_reserve_bytes(B.RNN_CELL_TANH, 2, 5, 3, 8, 128) == 2 * 5 * 3 * 128 * 4
    assert B.rnn_reserve_bytes(B.RNN_CELL_GRU, 2, 5, 3, 8, 128) == 2 * 5 * 3 * 128 * 5 * 4
    assert B.rnn_reserve_bytes(B.RNN_CELL_GRU, 2, 5, 3, 8, 16) == 2 * 5 * 3 * 128 * 5 * 4   # padded like the LSTM's sizes
    assert B.rnn_reserve_bytes(B.RNN_CELL_GRU, 1, 5, 3, 8, 16) == 5 * 3 * 16 * 5 * 4        # a few steps of one layer: as given
    assert B.rnn_reserve_bytes(7, 2, 5, 3, 8, 16) == 0 and B.rnn_workspace_bytes(B.RNN_CELL_GRU, 0, 1, 1, 1, 1) == 0
    wb = B.rnn_workspace_bytes(B.RNN_CELL_GRU, 1, 2, 2, 4, 4)
    assert wb > 0 and wb % 256 == 0
    a = 4096  # any 16-byte aligned non-null address: validation fails before it is touched
    dims = (B.RNN_CELL_GRU, 1, 2, 2, 4, 4)
    assert B.rnn_forward(*dims, a, None, a, a, a, a, None, a, a, wb - 1, stream=0) == B.LSTM_BUFFER_TOO_SMALL
    assert B.rnn_forward(*dims, None, None, a, a, a, a, None, a, a, wb, stream=0) == B.LSTM_INVALID_ARG
    assert B.rnn_forward(*dims, a + 4, None, a, a, a, a, None, a, a, wb, stream=0) == B.LSTM_INVALID_ARG
    assert B.rnn_forward(9, 1, 2, 2, 4, 4, a, None, a, a, a, a, None, a, a, wb, stream=0) == B.LSTM_INVALID_ARG
    assert B.rnn_backward(*dims, a, None, a, a, a, None, None, None, None, a, a, a, a, wb, stream=0) == B.LSTM_INVALID_ARG


def test_size_queries():
    assert B.lstm_reserve_bytes(4, 100, 64, 512, 512) == 4 * 100 * 64 * 6 * 512 * 4
    assert B.lstm_reserve_bytes(0, 1, 1, 1, 1) == 0 and B.lstm_workspace_bytes(1, 1, -1, 1, 1) == 0
    assert B.lstm_workspace_bytes(1, 8, 4, 32, 32) > 0
    assert B.lstm_workspace_bytes(4, 100, 64, 512, 512) % 256 == 0


def test_hidden_sizes_between_the_native_ones_are_padded(monkeypatch):
    # H < 512 runs at the next of 128 / 256 / 512: the reserve holds the padded network
    assert B.lstm_reserve_bytes(2, 5, 3, 8, 100) == 2 * 5 * 3 * 6 * 128 * 4
    assert B.lstm_reserve_bytes(2, 5, 3, 384, 384) == 2 * 5 * 3 * 6 * 512 * 4
    assert B.lstm_reserve_bytes(2, 5, 3, 8, 1) == 2 * 5 * 3 * 6 * 128 * 4
    assert B.lstm_reserve_bytes(1, 40, 3, 8, 100) == 40 * 3 * 6 * 128 * 4
    assert B.lstm_reserve_bytes(1, 8, 3, 8, 100) == 8 * 3 * 6 * 100 * 4          # a few steps of one layer: not worth the copies
    assert B.lstm_reserve_bytes(1, 8, 64, 8, 100) == 8 * 64 * 6 * 128 * 4        # (with more rows they are, from 8 steps on)
    assert B.lstm_reserve_bytes(1, 7, 64, 8, 100) == 7 * 64 * 6 * 100 * 4
    assert B.lstm_reserve_bytes(2, 5, 3, 8, 256) == 2 * 5 * 3 * 6 * 256 * 4      # native sizes stay as they are
    assert B.lstm_reserve_bytes(2, 5, 3, 8, 520) == 2 * 5 * 3 * 6 * 1024 * 4     # between 512 and 1024: the one-layer kernels of 1024
    assert B.lstm_reserve_bytes(2, 5, 3, 8, 800) == 2 * 5 * 3 * 6 * 1024 * 4
    assert B.lstm_reserve_bytes(2, 5, 100, 8, 600) == 2 * 5 * 100 * 6 * 600 * 4  # with more rows only from a larger size on
    assert B.lstm_reserve_bytes(2, 5, 100, 8, 608) == 2 * 5 * 100 * 6 * 1024 * 4
    assert B.lstm_reserve_bytes(2, 5, 200, 8, 800) == 2 * 5 * 200 * 6 * 1024 * 4
    assert B.lstm_reserve_bytes(2, 5, 600, 8, 800) == 2 * 5 * 600 * 6 * 800 * 4
    assert B.lstm_reserve_bytes(2, 5, 600, 8, 832) == 2 * 5 * 600 * 6 * 1024 * 4
    assert B.lstm_reserve_bytes(2, 5, 800, 8, 900) == 2 * 5 * 800 * 6 * 900 * 4  # beyond the batch those kernels take: as given
    assert B.lstm_reserve_bytes(2, 5, 3, 8, 1100) == 2 * 5 * 3 * 6 * 1100 * 4
    assert B.lstm_reserve_bytes(2, 5, 3, 8, 1500) == 2 * 5 * 3 * 6 * 2048 * 4    # nearer 2048 with few rows: the one-layer kernels of 2048
    assert B.lstm_reserve_bytes(2, 5, 48, 8, 1500) == 2 * 5 * 48 * 6 * 1500 * 4
    assert B.lstm_reserve_bytes(2, 5, 48, 8, 1700) == 2 * 5 * 48 * 6 * 2048 * 4
    assert B.lstm_reserve_bytes(2, 5, 600, 8, 100) == 2 * 5 * 600 * 6 * 128 * 4  # large batches: still padded up to 128 / 256
    assert B.lstm_reserve_bytes(2, 5, 600, 8, 448) == 2 * 5 * 600 * 6 * 512 * 4  # ... and to 512 from H = 416 on
    assert B.lstm_reserve_bytes(2, 5, 600, 8, 384) == 2 * 5 * 600 * 6 * 384 * 4  # ... in between the given size is the faster one
    assert B.lstm_reserve_bytes(2, 5, 512, 8, 384) == 2 * 5 * 512 * 6 * 512 * 4  # (up to 512 rows every size below 512 is padded)
    padded = B.lstm_workspace_bytes(2, 5, 3, 8, 100)
    assert padded > B.lstm_workspace_bytes(2, 5, 3, 8, 128) and padded % 256 == 0
    a = 4096
    ptrs = [a, None, None, a, a, a, a, None, None, None, a]
    assert B.lstm_forward(2, 5, 3, 8, 100, *ptrs, padded - 1, stream=0, flags=0) == B.LSTM_BUFFER_TOO_SMALL


def test_buffer_sizes_do_not_depend_on_the_environment(monkeypatch):
    """LSTM_NO_PAD / RNN_NO_PERSISTENT switch the zero-padding of hidden sizes off, which changes the layout of the
    reserve; the size queries answer for both settings (the larger), so buffers sized under one setting can never
    be overrun under the other.  The settings themselves are read once and again after lstm_shutdown()."""
    shapes = [(2, 5, 3, 8, 100), (2, 5, 3, 8, 800), (4, 100, 64, 512, 512), (1, 8, 3, 8, 100), (2, 5, 3, 384, 384)]
    B.lstm_shutdown()
    ref = [(B.lstm_reserve_bytes(*s), B.lstm_workspace_bytes(*s)) for s in shapes]
    rnn = [(B.rnn_reserve_bytes(c, *s), B.rnn_workspace_bytes(c, *s)) for s in shapes for c in (0, 1, 2)]
    monkeypatch.setenv("LSTM_NO_PAD", "1")
    monkeypatch.setenv("RNN_NO_PERSISTENT", "1")
    B.lstm_shutdown()  # the settings are read again
    assert ref == [(B.lstm_reserve_bytes(*s), B.lstm_workspace_bytes(*s)) for s in shapes]
    assert rnn == [(B.rnn_reserve_bytes(c, *s), B.rnn_workspace_bytes(c, *s)) for s in shapes for c in (0, 1, 2)]
    # as-given runs need no more than the padded ones were sized for
    assert B.lstm_reserve_bytes(2, 5, 3, 8, 100) >= 2 * 5 * 3 * 6 * 100 * 4
    a = 4096
    ptrs = [a, None, None, a, a, a, a, None, None, None, a]
    assert B.lstm_forward(2, 5, 3, 8, 100, *ptrs, ref[0][1] - 1, stream=0, flags=0) == B.LSTM_BUFFER_TOO_SMALL
    monkeypatch.delenv("LSTM_NO_PAD")
    monkeypatch.delenv("RNN_NO_PERSISTENT")
    B.lstm_shutdown()


def test_wavefront_chunks_setting_validates():
    dims = (2, 8, 4, 32, 640)
    assert B.lstm_set_wavefront_chunks(0, 8, 4, 32, 640, 2) == B.LSTM_INVALID_ARG
    assert B.lstm_set_wavefront_chunks(*dims, -1) == B.LSTM_INVALID_ARG
    assert B.lstm_set_wavefront_chunks(*dims, 3) == B.LSTM_OK
    assert B.lstm_set_wavefront_chunks(*dims, 1000) == B.LSTM_OK   # clamped when used
    assert B.lstm_set_wavefront_chunks(*dims, 0) == B.LSTM_OK      # removes the entry
    assert B.lstm_set_wavefront_chunks(*dims, 0) == B.LSTM_OK


def test_status_strings():
    for s in range(0, 6):
        assert B.lstm_status_string(s)
    assert "unknown" in B.lstm_status_string(99)


def _fwd(dims, ptrs, ws_bytes, flags=0):
    return B.lstm_forward(*dims, *ptrs, ws_bytes, stream=0, flags=flags)


def test_forward_rejects_bad_arguments_without_touching_the_gpu():
    dims = (1, 2, 2, 4, 4)
    need = B.lstm_workspace_bytes(*dims)
    ok = 4096  # fake aligned "device addresses": validation must fail before any is dereferenced
    ptrs = [ok, None, None, ok, ok, ok, ok, None, None, None, ok]
    assert _fwd((0, 2, 2, 4, 4), ptrs, need) == B.LSTM_INVALID_ARG
    assert _fwd((1, 2, 2, 4, -4), ptrs, need) == B.LSTM_INVALID_ARG
    for k in (0, 3, 4, 5, 6, 10):  # x, W, R, b, y, workspace are required
        bad = list(ptrs); bad[k] = None
        assert _fwd(dims, bad, need) == B.LSTM_INVALID_ARG, k
    mis = list(ptrs); mis[0] = ok + 4
    assert _fwd(dims, mis, need) == B.LSTM_INVALID_ARG
    assert _fwd(dims, ptrs, need - 1) == B.LSTM_BUFFER_TOO_SMALL
    assert _fwd(dims, ptrs, need, flags=7) == B.LSTM_INVALID_ARG
    assert _fwd(dims, ptrs, need, flags=16) == B.LSTM_INVALID_ARG


def test_backward_rejects_bad_arguments_without_touching_the_gpu():
    dims = (1, 2, 2, 4, 4)
    need = B.lstm_workspace_bytes(*dims)
    ok = 4096
    # x h0 c0 W R reserve dy dhT dcT dx dh0 dc0 dW dR db workspace
    ptrs = [ok, None, None, ok, ok, ok, ok, None, None, None, None, None, ok, ok, ok, ok]
    call = lambda d, p, n, f=0: B.lstm_backward(*d, *p, n, stream=0, flags=f)
    assert call((1, 0, 2, 4, 4), ptrs, need) == B.LSTM_INVALID_ARG
    for k in (0, 3, 4, 5, 6, 12, 13, 14, 15):
        bad = list(ptrs); bad[k] = None
        assert call(dims, bad, need) == B.LSTM_INVALID_ARG, k
    mis = list(ptrs); mis[12] = ok + 8
    assert call(dims, mis, need) == B.LSTM_INVALID_ARG
    assert call(dims, ptrs, need - 256) == B.LSTM_BUFFER_TOO_SMALL


def test_gemm_rejects_bad_arguments():
    assert B.lstm_gemm_f32(0, 1, 1, 4096, 1, 1, 4096, 1, 1, 4096, 1, 0, stream=0) == B.LSTM_INVALID_ARG
    assert B.lstm_gemm_f32(4, 4, 4, 4096, 4, 2, 4096, 4, 1, 4096, 4, 0, stream=0) == B.LSTM_INVALID_ARG
    assert B.lstm_gemm_f32(4, 4, 4, 4096, 4, 1, 4096, 4, 1, 4096, 2, 0, stream=0) == B.LSTM_INVALID_ARG


def test_auto_path_is_a_valid_path():
    assert B.lstm_auto_path(0, 1, 1, 1, 1, 0) == B.LSTM_PATH_AUTO
    assert B.lstm_auto_path(1, 8, 4, 32, 32, 1) in (B.LSTM_PATH_STEP, B.LSTM_PATH_WAVEFRONT, B.LSTM_PATH_PERSISTENT)


def test_set_path_overrides_and_validates():
    dims = (2, 8, 4, 32, 640)
    auto = B.lstm_auto_path(*dims, 0)
    assert B.lstm_set_path(0, 8, 4, 32, 640, 0, B.LSTM_PATH_STEP) == B.LSTM_INVALID_ARG
    assert B.lstm_set_path(*dims, 0, 99) == B.LSTM_INVALID_ARG
    # H = 640 is neither a size of the persistent kernels nor padded to one, on any device
    assert B.lstm_set_path(*dims, 0, B.LSTM_PATH_PERSISTENT) == B.LSTM_UNSUPPORTED
    other = B.LSTM_PATH_STEP if auto != B.LSTM_PATH_STEP else B.LSTM_PATH_WAVEFRONT
    assert B.lstm_set_path(*dims, 0, other) == B.LSTM_OK
    assert B.lstm_auto_path(*dims, 0) == other
    assert B.lstm_auto_path(*dims, 1) == B.lstm_auto_path(2, 8, 4, 32, 640, 1)  # the other direction is untouched
    assert B.lstm_set_path(*dims, 0, B.LSTM_PATH_AUTO) == B.LSTM_OK
    assert B.lstm_auto_path(*dims, 0) == auto
    assert B.lstm_set_path(*dims, 1, other) == B.LSTM_OK
    B.lstm_shutdown()  # empties the table
    assert B.lstm_auto_path(*dims, 1) == B.lstm_auto_path(*dims, 1)
