"""ctypes binding of the predictor's forward pass (pbkv_predictor.h): argument marshalling only.

Every buffer is a device tensor (anything with ``data_ptr()``) or a raw device address; the
workspace is allocated by the caller.  There is no CPU fallback."""
import ctypes

from . import binding
from .binding import _check, _ptr, _stream

WEIGHT_NAMES = ("emb", "trans", "w1", "w2", "wq", "wt", "wa", "ba", "wb", "bb")


class PredictorShape(ctypes.Structure):
    _fields_ = [("num_agents", ctypes.c_int32), ("d", ctypes.c_int32), ("d_x", ctypes.c_int32),
                ("hidden", ctypes.c_int32), ("horizon", ctypes.c_int32), ("max_prefix", ctypes.c_int32)]


class PredictorWeights(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in WEIGHT_NAMES]


_bound = False


def _lib():
    global _bound
    lib = binding.load()
    if not _bound:
        sp, vp = ctypes.POINTER(PredictorShape), ctypes.c_void_p
        lib.pbkv_predictor_workspace_bytes.restype = ctypes.c_int64
        lib.pbkv_predictor_workspace_bytes.argtypes = [sp, ctypes.c_int32]
        lib.pbkv_predictor_prepare.restype = ctypes.c_int
        lib.pbkv_predictor_prepare.argtypes = [sp, ctypes.POINTER(PredictorWeights), vp, ctypes.c_int64,
                                               ctypes.c_int32, vp]
        lib.pbkv_predictor_forward.restype = ctypes.c_int
        lib.pbkv_predictor_forward.argtypes = [sp, vp, ctypes.c_int64, ctypes.c_int32, vp, vp, vp, vp,
                                               ctypes.c_int32, vp, vp]
        _bound = True
    return lib


def make_shape(num_agents, d, d_x, hidden, horizon, max_prefix):
    return PredictorShape(num_agents, d, d_x, hidden, horizon, max_prefix)


def predictor_workspace_bytes(shape, max_batch):
    n = int(_lib().pbkv_predictor_workspace_bytes(ctypes.byref(shape), int(max_batch)))
    if n == 0:          # the size query reports a bad shape or batch bound as 0 and leaves the reason behind
        msg = binding.load().pbkv_last_error().decode()
        raise binding.PbkvError(-4 if "max_batch" in msg else -2, msg)
    return n


def predictor_prepare(shape, weights, workspace, workspace_bytes, max_batch, stream=None):
    """weights: mapping name -> device tensor (fp32) for the names in WEIGHT_NAMES."""
    w = PredictorWeights(*[_ptr(weights[n]) if weights.get(n) is not None else None for n in WEIGHT_NAMES])
    _check(_lib().pbkv_predictor_prepare(ctypes.byref(shape), ctypes.byref(w), _ptr(workspace),
                                         int(workspace_bytes), int(max_batch), _stream(stream)))


def predictor_forward(shape, workspace, workspace_bytes, max_batch, x, cur_agent, prefix, prefix_len, batch,
                      probs, stream=None):
    _check(_lib().pbkv_predictor_forward(ctypes.byref(shape), _ptr(workspace), int(workspace_bytes),
                                         int(max_batch), _ptr(x), _ptr(cur_agent), _ptr(prefix),
                                         _ptr(prefix_len), int(batch), _ptr(probs), _stream(stream)))
