"""ctypes binding of libusl (include/usl.h): argument marshalling only.

Every function takes torch tensors that already live on the GPU (or raw integer device
addresses) and forwards their pointers; all arithmetic runs in the HIP kernels.  There is no
CPU fallback: if the shared library is missing, importing this module raises.
"""
import ctypes
import os
import weakref

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libusl.so")

USL_OK, USL_EINVAL, USL_ESHAPE, USL_ENOMEM, USL_EHIP, USL_EUNSUPPORTED, USL_ESTALE = range(7)
USL_F32, USL_BF16 = 0, 1
STATUS_NAMES = ["USL_OK", "USL_EINVAL", "USL_ESHAPE", "USL_ENOMEM", "USL_EHIP", "USL_EUNSUPPORTED", "USL_ESTALE"]

# every symbol include/usl.h declares
SYMBOLS = ["usl_bce_loss_grad_noalloc", "usl_check", "usl_create", "usl_destroy", "usl_set_stream", "usl_invalidate", "usl_last_error",
           "usl_version", "usl_init_indices", "usl_forward", "usl_bce_loss_grad", "usl_sqh_loss_grad",
           "usl_topk", "usl_precision_hits", "usl_train_step", "usl_redistribute_rows", "usl_predict",
           "usl_forward_rows", "usl_backward_weight_rows", "usl_backward_input_rows",
           "usl_backward_weight", "usl_backward_input", "usl_backward", "usl_adam_step", "usl_redistribute",
           "usl_validate_indices", "usl_philox_words"]

if not os.path.exists(LIB_PATH):
    raise ImportError("libusl.so is not built: run `python -m paper_2306_03725_amd.build` "
                      "(there is no fallback path)")
_lib = ctypes.CDLL(LIB_PATH)

_vp, _i32, _i64, _u32, _u64, _f32, _f64 = (ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64,
                                           ctypes.c_uint32, ctypes.c_uint64, ctypes.c_float,
                                           ctypes.c_double)
_sig = {
    "usl_create": [ctypes.POINTER(_vp), _i64, _i32, _i32, _i32, ctypes.c_int, _vp],
    "usl_destroy": [_vp],
    "usl_set_stream": [_vp, _vp],
    "usl_invalidate": [_vp],
    "usl_check": [_vp],
    "usl_init_indices": [_vp, _vp, _u64],
    "usl_forward": [_vp, _vp, _vp, _vp, _vp, _i32],
    "usl_bce_loss_grad": [_vp, _vp, _vp, _vp, _f32, _vp, _vp, _i32],
    "usl_sqh_loss_grad": [_vp, _vp, _vp, _vp, _f32, _vp, _vp, _i32],
    "usl_bce_loss_grad_noalloc": [_vp, _vp, _vp, _vp, _f32, _vp, _vp, _i32],
    "usl_topk": [_vp, _vp, _i32, _i32, _vp, _vp],
    "usl_predict": [_vp, _vp, _vp, _vp, _i32, _i32, _vp, _vp],
    "usl_train_step": [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _f32, _i64, _f32, _f32, _f32, _f32,
                       _vp, _vp, _vp, _vp, _i32],
    "usl_forward_rows": [_vp, _vp, _vp, _vp, _vp, _i64, _vp, _i32],
    "usl_backward_weight_rows": [_vp, _vp, _vp, _vp, _vp, _i64, _vp, _i32],
    "usl_backward_input_rows": [_vp, _vp, _vp, _vp, _vp, _i64, _vp, _i32],
    "usl_precision_hits": [_vp, _vp, _vp, _vp, _i32, _i32, _vp],
    "usl_backward_weight": [_vp, _vp, _vp, _vp, _vp, _i32],
    "usl_backward_input": [_vp, _vp, _vp, _vp, _vp, _i32],
    "usl_backward": [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _i32],
    "usl_adam_step": [_vp, _vp, _vp, _vp, _vp, _i64, _f32, _f32, _f32, _f32],
    "usl_redistribute": [_vp, _vp, _vp, _vp, _vp, _f64, _u64, _u64, ctypes.POINTER(_i64)],
    "usl_redistribute_rows": [_vp, _vp, _vp, _vp, _vp, _i32, _u64, _u64],
    "usl_validate_indices": [_vp, _vp, ctypes.POINTER(_i64)],
    "usl_philox_words": [_vp, _vp, _u32, _u32, _vp, _i64],
}
for _name, _args in _sig.items():
    _f = getattr(_lib, _name)
    _f.argtypes = _args
    _f.restype = ctypes.c_int
_lib.usl_last_error.argtypes = [_vp]
_lib.usl_last_error.restype = ctypes.c_char_p
_lib.usl_version.argtypes = []
_lib.usl_version.restype = ctypes.c_char_p


class UslError(RuntimeError):
    def __init__(self, status, message):
        super().__init__("%s: %s" % (STATUS_NAMES[status] if 0 <= status < len(STATUS_NAMES) else status, message))
        self.status = status


def version():
    return _lib.usl_version().decode()


def _ptr(t):
    """Device address of a torch tensor (must be contiguous), or an int / None passed through."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if not t.is_contiguous():
        raise ValueError("tensor must be contiguous")
    return t.data_ptr()


class Layer:
    """A usl context: shape (m, d, k), storage type and stream of one uniformly-sparse layer."""

    def __init__(self, m, d, k, max_b, storage="f32", stream=None):
        self._h = _vp()
        st = {"f32": USL_F32, "bf16": USL_BF16}.get(storage, storage)
        s = _lib.usl_create(ctypes.byref(self._h), m, d, k, max_b, st, stream)
        if s != USL_OK:
            self._h = _vp()
            raise UslError(s, "usl_create(m=%s, d=%s, k=%s, max_b=%s, storage=%s)" % (m, d, k, max_b, storage))
        self.m, self.d, self.k, self.max_b, self.storage = m, d, k, max_b, storage
        self._idx_seen = None

    def close(self):
        if self._h and _lib is not None:      # _lib is gone when the interpreter is shutting down
            _lib.usl_destroy(self._h)
            self._h = _vp()

    __del__ = close

    def _ck(self, s):
        if s != USL_OK:
            raise UslError(s, _lib.usl_last_error(self._h).decode())

    def set_stream(self, stream):
        self._ck(_lib.usl_set_stream(self._h, stream))

    def invalidate(self):
        self._ck(_lib.usl_invalidate(self._h))

    def check(self):
        """Waits for the stream; raises UslError(USL_ESTALE) if a call ran on private views of an idx that changed."""
        self._ck(_lib.usl_check(self._h))

    def _same_idx(self, idx):
        """The library keys its private views of the connectivity by the address of idx.  A different tensor
        object at the same address (the caching allocator recycles addresses), or the same tensor after an
        in-place torch operation, is new contents: tell the library so."""
        if isinstance(idx, int) or idx is None:
            return
        seen = self._idx_seen
        if seen is not None and (seen[0]() is not idx or seen[1] != idx._version):
            _lib.usl_invalidate(self._h)
        if seen is None or seen[0]() is not idx or seen[1] != idx._version:
            self._idx_seen = (weakref.ref(idx), idx._version)

    def init_indices(self, idx, seed):
        self._ck(_lib.usl_init_indices(self._h, _ptr(idx), seed))

    def forward(self, x, idx, W, out, b):
        self._same_idx(idx)
        self._ck(_lib.usl_forward(self._h, _ptr(x), _ptr(idx), _ptr(W), _ptr(out), b))

    def bce_loss_grad(self, out, tgt_off, tgt_lab, scale, g, loss, b):
        self._ck(_lib.usl_bce_loss_grad(self._h, _ptr(out), _ptr(tgt_off), _ptr(tgt_lab), scale,
                                        _ptr(g), _ptr(loss), b))

    def bce_loss_grad_noalloc(self, out, tgt_off, tgt_lab, scale, g, loss, b):
        self._ck(_lib.usl_bce_loss_grad_noalloc(self._h, _ptr(out), _ptr(tgt_off), _ptr(tgt_lab), scale,
                                                _ptr(g), _ptr(loss), b))

    def sqh_loss_grad(self, out, tgt_off, tgt_lab, scale, g, loss, b):
        self._ck(_lib.usl_sqh_loss_grad(self._h, _ptr(out), _ptr(tgt_off), _ptr(tgt_lab), scale,
                                        _ptr(g), _ptr(loss), b))

    def forward_rows(self, x, idx, W, rows, n_rows, out_rows, b):
        self._ck(_lib.usl_forward_rows(self._h, _ptr(x), _ptr(idx), _ptr(W), _ptr(rows), n_rows,
                                       _ptr(out_rows), b))

    def backward_weight_rows(self, g_rows, x, idx, rows, n_rows, grad_W_rows, b):
        self._ck(_lib.usl_backward_weight_rows(self._h, _ptr(g_rows), _ptr(x), _ptr(idx), _ptr(rows), n_rows,
                                               _ptr(grad_W_rows), b))

    def backward_input_rows(self, g_rows, idx, W, rows, n_rows, grad_x, b):
        self._ck(_lib.usl_backward_input_rows(self._h, _ptr(g_rows), _ptr(idx), _ptr(W), _ptr(rows), n_rows,
                                              _ptr(grad_x), b))

    def topk(self, out, b, kk, top_lab, top_val):
        self._ck(_lib.usl_topk(self._h, _ptr(out), b, kk, _ptr(top_lab), _ptr(top_val)))

    def predict(self, x, idx, W, b, kk, top_lab, top_val):
        self._same_idx(idx)
        self._ck(_lib.usl_predict(self._h, _ptr(x), _ptr(idx), _ptr(W), b, kk, _ptr(top_lab), _ptr(top_val)))

    def precision_hits(self, top_lab, tgt_off, tgt_lab, b, kk, hits):
        self._ck(_lib.usl_precision_hits(self._h, _ptr(top_lab), _ptr(tgt_off), _ptr(tgt_lab), b, kk,
                                         _ptr(hits)))

    def backward_weight(self, g, x, idx, grad_W, b):
        self._same_idx(idx)
        self._ck(_lib.usl_backward_weight(self._h, _ptr(g), _ptr(x), _ptr(idx), _ptr(grad_W), b))

    def backward_input(self, g, idx, W, grad_x, b):
        self._same_idx(idx)
        self._ck(_lib.usl_backward_input(self._h, _ptr(g), _ptr(idx), _ptr(W), _ptr(grad_x), b))

    def backward(self, g, x, idx, W, grad_W, grad_x, b):
        self._same_idx(idx)
        self._ck(_lib.usl_backward(self._h, _ptr(g), _ptr(x), _ptr(idx), _ptr(W), _ptr(grad_W), _ptr(grad_x), b))

    def adam_step(self, W, grad_W, m1, m2, t, lr, beta1, beta2, eps):
        self._ck(_lib.usl_adam_step(self._h, _ptr(W), _ptr(grad_W), _ptr(m1), _ptr(m2), t, lr,
                                    beta1, beta2, eps))

    def train_step(self, x, idx, W, m1, m2, tgt_off, tgt_lab, loss_kind, scale, t, lr, beta1, beta2, eps,
                   g, grad_W, grad_x, loss, b):
        self._same_idx(idx)
        self._ck(_lib.usl_train_step(self._h, _ptr(x), _ptr(idx), _ptr(W), _ptr(m1), _ptr(m2), _ptr(tgt_off),
                                     _ptr(tgt_lab), loss_kind, scale, t, lr, beta1, beta2, eps, _ptr(g),
                                     _ptr(grad_W), _ptr(grad_x) if grad_x is not None else None, _ptr(loss), b))

    def redistribute(self, idx, W, m1, m2, fraction, seed, epoch):
        n = _i64(-1)
        self._ck(_lib.usl_redistribute(self._h, _ptr(idx), _ptr(W), _ptr(m1), _ptr(m2), fraction,
                                       seed, epoch, ctypes.byref(n)))
        return n.value

    def redistribute_rows(self, idx, W, m1, m2, per_row, seed, epoch):
        self._ck(_lib.usl_redistribute_rows(self._h, _ptr(idx), _ptr(W), _ptr(m1), _ptr(m2), per_row, seed, epoch))

    def validate_indices(self, idx):
        n = _i64(-1)
        self._ck(_lib.usl_validate_indices(self._h, _ptr(idx), ctypes.byref(n)))
        return n.value

    def philox_words(self, ctr, key0, key1, out, n):
        self._ck(_lib.usl_philox_words(self._h, _ptr(ctr), key0, key1, _ptr(out), n))
