"""ctypes binding of the C ABI declared in include/lstm.h.

Argument marshalling only: every function here has the name and argument order of
the C entry point it forwards to, accepts torch tensors (their device pointer is
passed) or None for optional pointers, and returns the C status code.  No LSTM
arithmetic happens in Python, and there is no fallback: if the compiled library
is missing, importing a symbol from it raises.
"""
import ctypes
import os

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(PKG_DIR, "liblstm_mi355x.so")

LSTM_OK = 0
LSTM_INVALID_ARG = 1
LSTM_BUFFER_TOO_SMALL = 2
LSTM_HIP_ERROR = 3
LSTM_INTERNAL = 4
LSTM_UNSUPPORTED = 5

LSTM_PATH_AUTO = 0
LSTM_PATH_NAIVE = 1
LSTM_PATH_GROUPED = 2
LSTM_PATH_FUSED = 3
LSTM_PATH_STEP = 4
LSTM_PATH_WAVEFRONT = 5
LSTM_PATH_PERSISTENT = 6
PATH_NAMES = {0: "auto", 1: "naive", 2: "grouped", 3: "fused", 4: "step", 5: "wavefront", 6: "persistent"}

EXPORTS = [
    "lstm_reserve_bytes", "lstm_workspace_bytes", "lstm_forward", "lstm_backward", "lstm_gemm_f32", "lstm_gemm_f32_ws",
    "lstm_init", "lstm_forward_noalloc",
    "lstm_auto_path", "lstm_set_path", "lstm_set_wavefront_chunks", "lstm_status_string", "lstm_last_error", "lstm_shutdown",
    "lstm_profile_enable", "lstm_profile_read", "lstm_profile_kernel", "lstm_phase_name", "lstm_debug_set_trace",
]
RNN_EXPORTS = ["rnn_reserve_bytes", "rnn_workspace_bytes", "rnn_forward", "rnn_backward"]
RNN_CELL_RELU, RNN_CELL_TANH, RNN_CELL_GRU = 0, 1, 2
RNN_CELLS = {"relu": RNN_CELL_RELU, "tanh": RNN_CELL_TANH, "gru": RNN_CELL_GRU}
LSTM_PHASE_COUNT = 8

_lib = None


class LstmError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__(f"{where}: status {status} ({lstm_status_string(status)}) {lstm_last_error()}")


def library():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is not built; run `python -m paper_1604_01946_amd.build`")
        # PyTorch ships a HIP runtime of its own.  Loaded first, it is the one this library binds to as well; the
        # other way round the process ends up with two runtimes, and the second one finds no device.
        try:
            import torch  # noqa: F401
        except ImportError:
            pass
        lib = ctypes.CDLL(LIB_PATH)
        i, p, z, u, l = ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_uint, ctypes.c_long
        lib.lstm_reserve_bytes.restype = z
        lib.lstm_reserve_bytes.argtypes = [i] * 5
        lib.lstm_workspace_bytes.restype = z
        lib.lstm_workspace_bytes.argtypes = [i] * 5
        lib.lstm_forward.restype = i
        lib.lstm_forward.argtypes = [i] * 5 + [p] * 11 + [z, p, u]
        lib.lstm_backward.restype = i
        lib.lstm_backward.argtypes = [i] * 5 + [p] * 16 + [z, p, u]
        lib.lstm_init.restype = i
        lib.lstm_init.argtypes = []
        lib.lstm_forward_noalloc.restype = i
        lib.lstm_forward_noalloc.argtypes = [i] * 5 + [p] * 10 + [p, u]
        lib.lstm_gemm_f32.restype = i
        lib.lstm_gemm_f32.argtypes = [i, i, i, p, l, l, p, l, l, p, l, i, p]
        lib.lstm_gemm_f32_ws.restype = i
        lib.lstm_gemm_f32_ws.argtypes = [i, i, i, p, l, l, p, l, l, p, l, i, p, ctypes.c_size_t, p]
        lib.lstm_auto_path.restype = u
        lib.lstm_auto_path.argtypes = [i] * 6
        lib.lstm_set_path.restype = i
        lib.lstm_set_path.argtypes = [i] * 6 + [u]
        lib.lstm_set_wavefront_chunks.restype = i
        lib.lstm_set_wavefront_chunks.argtypes = [i] * 6
        lib.lstm_status_string.restype = ctypes.c_char_p
        lib.lstm_status_string.argtypes = [i]
        lib.lstm_last_error.restype = ctypes.c_char_p
        lib.lstm_last_error.argtypes = []
        lib.lstm_shutdown.restype = None
        lib.lstm_shutdown.argtypes = []
        lib.lstm_profile_enable.restype = None
        lib.lstm_profile_enable.argtypes = [i]
        lib.lstm_profile_read.restype = i
        lib.lstm_profile_read.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_int),
                                          ctypes.POINTER(ctypes.c_double)]
        lib.lstm_profile_kernel.restype = ctypes.c_char_p
        lib.lstm_profile_kernel.argtypes = [i]
        lib.lstm_phase_name.restype = ctypes.c_char_p
        lib.lstm_phase_name.argtypes = [i]
        lib.lstm_debug_set_trace.restype = None
        lib.lstm_debug_set_trace.argtypes = [p, z, i]
        lib.rnn_reserve_bytes.restype = z
        lib.rnn_reserve_bytes.argtypes = [i] * 6
        lib.rnn_workspace_bytes.restype = z
        lib.rnn_workspace_bytes.argtypes = [i] * 6
        lib.rnn_forward.restype = i
        lib.rnn_forward.argtypes = [i] * 6 + [p] * 9 + [z, p]
        lib.rnn_backward.restype = i
        lib.rnn_backward.argtypes = [i] * 6 + [p] * 13 + [z, p]
        _lib = lib
    return _lib


def _ptr(t):
    """Device (or raw) address of a tensor / int / None."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def lstm_reserve_bytes(L, T, B, I, H):
    return library().lstm_reserve_bytes(L, T, B, I, H)


def rnn_reserve_bytes(cell, L, T, B, I, H):
    return library().rnn_reserve_bytes(cell, L, T, B, I, H)


def rnn_workspace_bytes(cell, L, T, B, I, H):
    return library().rnn_workspace_bytes(cell, L, T, B, I, H)


def rnn_forward(cell, L, T, B, I, H, x, h0, W, R, b, y, hT, reserve, workspace, workspace_bytes, stream=None):
    return library().rnn_forward(cell, L, T, B, I, H, _ptr(x), _ptr(h0), _ptr(W), _ptr(R), _ptr(b), _ptr(y), _ptr(hT),
                                 _ptr(reserve), _ptr(workspace), workspace_bytes, _stream(stream))


def rnn_backward(cell, L, T, B, I, H, x, h0, W, R, reserve, dy, dhT, dx, dh0, dW, dR, db, workspace, workspace_bytes,
                 stream=None):
    return library().rnn_backward(cell, L, T, B, I, H, _ptr(x), _ptr(h0), _ptr(W), _ptr(R), _ptr(reserve), _ptr(dy),
                                  _ptr(dhT), _ptr(dx), _ptr(dh0), _ptr(dW), _ptr(dR), _ptr(db), _ptr(workspace),
                                  workspace_bytes, _stream(stream))


def lstm_workspace_bytes(L, T, B, I, H):
    return library().lstm_workspace_bytes(L, T, B, I, H)


def lstm_status_string(status):
    return library().lstm_status_string(status).decode()


def lstm_last_error():
    return library().lstm_last_error().decode()


def lstm_shutdown():
    library().lstm_shutdown()


def lstm_auto_path(L, T, B, I, H, backward):
    return library().lstm_auto_path(L, T, B, I, H, int(backward))


def lstm_set_path(L, T, B, I, H, backward, path):
    return library().lstm_set_path(L, T, B, I, H, int(backward), int(path))


def lstm_set_wavefront_chunks(L, T, B, I, H, chunks):
    return library().lstm_set_wavefront_chunks(L, T, B, I, H, int(chunks))


def lstm_forward(L, T, B, I, H, x, h0, c0, W, R, b, y, hT, cT, reserve, workspace, workspace_bytes,
                 stream=None, flags=0):
    return library().lstm_forward(L, T, B, I, H, _ptr(x), _ptr(h0), _ptr(c0), _ptr(W), _ptr(R), _ptr(b),
                                  _ptr(y), _ptr(hT), _ptr(cT), _ptr(reserve), _ptr(workspace), workspace_bytes,
                                  _stream(stream), flags)


def lstm_init():
    return library().lstm_init()


def lstm_forward_noalloc(L, T, B, I, H, x, h0, c0, W, R, b, y, hT, cT, reserve, stream=None, flags=0):
    return library().lstm_forward_noalloc(L, T, B, I, H, _ptr(x), _ptr(h0), _ptr(c0), _ptr(W), _ptr(R), _ptr(b),
                                          _ptr(y), _ptr(hT), _ptr(cT), _ptr(reserve), _stream(stream), flags)


def lstm_backward(L, T, B, I, H, x, h0, c0, W, R, reserve, dy, dhT, dcT, dx, dh0, dc0, dW, dR, db,
                  workspace, workspace_bytes, stream=None, flags=0):
    return library().lstm_backward(L, T, B, I, H, _ptr(x), _ptr(h0), _ptr(c0), _ptr(W), _ptr(R), _ptr(reserve),
                                   _ptr(dy), _ptr(dhT), _ptr(dcT), _ptr(dx), _ptr(dh0), _ptr(dc0),
                                   _ptr(dW), _ptr(dR), _ptr(db), _ptr(workspace), workspace_bytes,
                                   _stream(stream), flags)


def lstm_gemm_f32(M, N, K, A, sAm, sAk, Bm, sBk, sBn, C, ldc, accumulate, stream=None):
    return library().lstm_gemm_f32(M, N, K, _ptr(A), sAm, sAk, _ptr(Bm), sBk, sBn, _ptr(C), ldc, int(accumulate),
                                   _stream(stream))


def lstm_gemm_f32_ws(M, N, K, A, sAm, sAk, Bm, sBk, sBn, C, ldc, accumulate, scratch, scratch_bytes, stream=None):
    return library().lstm_gemm_f32_ws(M, N, K, _ptr(A), sAm, sAk, _ptr(Bm), sBk, sBn, _ptr(C), ldc, int(accumulate),
                                      _ptr(scratch), ctypes.c_size_t(scratch_bytes), _stream(stream))


def lstm_profile_enable(on):
    library().lstm_profile_enable(int(on))


def lstm_phase_name(phase):
    return library().lstm_phase_name(phase).decode()


def lstm_profile_read():
    """Returns (status, {phase name: (milliseconds, intervals, algorithmic FLOPs, kernel name)})."""
    ms = (ctypes.c_float * LSTM_PHASE_COUNT)()
    cnt = (ctypes.c_int * LSTM_PHASE_COUNT)()
    fl = (ctypes.c_double * LSTM_PHASE_COUNT)()
    st = library().lstm_profile_read(ms, cnt, fl)
    return st, {lstm_phase_name(k): (float(ms[k]), int(cnt[k]), float(fl[k]), library().lstm_profile_kernel(k).decode())
                for k in range(LSTM_PHASE_COUNT)}


def lstm_debug_set_trace(device_buf, nbytes, block):
    library().lstm_debug_set_trace(_ptr(device_buf), nbytes, block)


def check(status, where="lstm"):
    if status != LSTM_OK:
        raise LstmError(status, where)
