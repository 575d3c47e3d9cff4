"""Python binding of libhcnn.so: same names as include/hcnn.h, torch tensors on the GPU as buffers.

PyTorch supplies device memory and the HIP stream only; every step of the path
runs in the library's kernels.  There is no CPU fallback: loading fails loudly
when the HIP library has not been built.
"""
import ctypes
import os

import torch

from . import _capi
from ._ops import OpsMixin

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "lib", "libhcnn.so")
_lib = None


def lib() -> ctypes.CDLL:
    """The HIP library (built beforehand with `python -m paper_1811_00778_amd.build`)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError("libhcnn.so is not built: run `python -m paper_1811_00778_amd.build` "
                              "(or __graft_entry__.build()) first; there is no fallback path")
        _lib = _capi.declare(ctypes.CDLL(_LIB_PATH))
    return _lib


def gen_primes(n: int, count: int):
    """The `count` largest primes below 2^30 congruent to 1 mod 2n (hcnn_gen_primes)."""
    return _capi.gen_primes(lib(), n, count)


def choose_moduli(n: int, k: int, t: int):
    """(q primes, auxiliary primes): the first k primes of the rule and the minimal auxiliary basis after them."""
    cand = gen_primes(n, k + min(_capi.MAX_LIMBS, k + 8))
    q, rest = cand[:k], cand[k:]
    k_aux = _capi.min_aux_count(lib(), n, q, t, rest)
    return q, rest[:k_aux]


_DT = {"u32": torch.int32, "i32": torch.int32, "u64": torch.int64}


class Context(OpsMixin):
    """An hcnn_ctx bound to the current torch device and stream.

    uint32 residues are carried in torch.int32 tensors (same 32 bits; torch has no
    arithmetic on uint32, and none is needed here); the 64-bit plaintext words of a
    plaintext modulus above 2^32 in torch.int64 tensors."""

    def __init__(self, n, q_primes, p_primes, t, device="cuda:0"):
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU visible: the HIP path cannot run (there is no CPU fallback)")
        self.device = torch.device(device)
        torch.cuda.set_device(self.device)
        stream = torch.cuda.current_stream(self.device).cuda_stream
        self._stream = stream
        self.raw = _capi.RawContext(lib(), n, q_primes, p_primes, t, stream)

    def use_stream(self, stream=None):
        """Launch on `stream` (a torch.cuda.Stream; default: torch's current stream) from now on
        (hcnn_set_stream; the library waits for the work it has enqueued on the old stream first).  After one
        warm-up call per operation and size, the hot-path calls allocate nothing and enqueue kernels only, so they
        can be recorded into a HIP graph on the stream given here.

        Rule: the context's stream must be torch's current stream whenever an operation is called.  Output
        tensors come from torch's allocator, which hands a freed block out again to later work on the stream it
        was allocated on; if the library launched on another stream, that work could overwrite a buffer the
        library's kernels still use.  Every call checks this and raises instead."""
        stream = torch.cuda.current_stream(self.device) if stream is None else stream
        self.raw.call("hcnn_set_stream", ctypes.c_void_p(stream.cuda_stream))
        self._stream = stream.cuda_stream

    def _pre_call(self):
        if torch.cuda.current_stream(self.device).cuda_stream != self._stream:
            raise RuntimeError("the context is bound to another HIP stream than torch's current one: call "
                               "use_stream() inside the `with torch.cuda.stream(...)` block (and again after it)")

    def _ptr(self, x):
        return ctypes.c_void_p(x.data_ptr())

    def _empty(self, shape, dtype_name):
        return torch.empty(shape, dtype=_DT[dtype_name], device=self.device)

    def _check(self, x, dtype_name):
        if not isinstance(x, torch.Tensor) or x.dtype != _DT[dtype_name] or not x.is_contiguous() \
                or x.device != self.device:
            raise TypeError("expected a contiguous %s tensor on %s" % (_DT[dtype_name], self.device))

    # host <-> device convenience (numpy uint32/int32 arrays)
    def to_device(self, array):
        import numpy as np
        a = np.ascontiguousarray(array)
        if a.dtype == np.uint32:
            a = a.view(np.int32)
        elif a.dtype == np.uint64:
            a = a.view(np.int64)            # 64-bit plaintext words of a wide plaintext modulus
        elif a.dtype not in (np.int32, np.int64):
            raise TypeError("uint32, int32 or uint64 expected")
        return torch.from_numpy(a).to(self.device)

    def to_host_u32(self, tensor):
        import numpy as np
        torch.cuda.current_stream(self.device).synchronize()
        a = tensor.cpu().numpy()
        return a.view(np.uint64) if a.dtype == np.int64 else a.view(np.uint32)
