"""ctypes declarations of the C ABI in include/hcnn.h (argument marshalling only)."""
import ctypes as C

u32p = C.POINTER(C.c_uint32)
u64p = C.POINTER(C.c_uint64)
ptr = C.c_void_p

ERR = dict(OK=0, NULL=-1, N=-2, PRIME=-3, T=-4, AUX=-5, ARG=-6, NOKEY=-7, ALIGN=-8, NODEVICE=-9, SCRATCH=-10)
STAT_EXACT_FALLBACKS, STAT_BAD_INPUT, STAT_SCRATCH_BYTES, STAT_RELIN_FUSED_WGS, STAT_TENSOR_FUSED_WGS = 0, 1, 2, 3, 4
OPT_AMBIGUITY_BAND, OPT_SQUARE_CHUNK, OPT_PROFILE, OPT_RELIN_ORDER, OPT_FUSION = 0, 1, 2, 3, 4
PROF_CLASSES = ["ntt_fwd", "ntt_inv", "base_ext", "tensor", "scale", "digit", "relin_mac", "relin_add",
                "scalar_mac", "other", "relin_fused"]
CEILINGS = ["copy_GBps", "read_GBps", "write_GBps", "mul_lo_u32_Tops", "mul_hi_u32_Tops", "mad_u64_u32_Tops",
            "mad_i64_i32_Tops", "add_u32_Tops"]
MAX_LIMBS, MAX_FILTERS = 32, 16

# name -> argtypes; every entry point returns int except hcnn_strerror
SIGNATURES = {
    "hcnn_gen_primes": [C.c_uint32, C.c_uint32, u32p],
    "hcnn_min_aux_count": [C.c_uint32, C.c_uint32, u32p, C.c_uint64, u32p, C.c_uint32, u32p],
    "hcnn_ctx_create": [C.POINTER(ptr), C.c_uint32, C.c_uint32, u32p, C.c_uint32, u32p, C.c_uint64, ptr],
    "hcnn_ctx_destroy": [ptr],
    "hcnn_set_stream": [ptr, ptr],
    "hcnn_set_relin_key": [ptr, ptr],
    "hcnn_ntt_fwd": [ptr, ptr, C.c_size_t],
    "hcnn_ntt_inv": [ptr, ptr, C.c_size_t],
    "hcnn_ct_scalar_mac": [ptr, ptr, C.c_size_t, ptr, ptr, C.c_int32, C.c_size_t, C.c_size_t, C.c_size_t, ptr],
    "hcnn_ct_square_relin": [ptr, ptr, C.c_size_t, ptr],
    "hcnn_ct_square_relin_noalloc": [ptr, ptr, C.c_size_t, ptr],
    "hcnn_ct_mul_relin": [ptr, ptr, ptr, C.c_size_t, ptr],
    "hcnn_keygen": [ptr, ptr, ptr, ptr, ptr, ptr, ptr, ptr],
    "hcnn_encrypt": [ptr, ptr, ptr, ptr, ptr, ptr, C.c_size_t, ptr],
    "hcnn_decrypt": [ptr, ptr, ptr, C.c_size_t, ptr],
    "hcnn_encrypt_wide": [ptr, ptr, ptr, ptr, ptr, ptr, C.c_size_t, ptr],
    "hcnn_decrypt_wide": [ptr, ptr, ptr, C.c_size_t, ptr],
    "hcnn_noise_bits": [ptr, ptr, ptr, C.c_size_t, ptr],
    "hcnn_sample_ternary": [ptr, C.c_uint64, C.c_uint64, ptr, C.c_size_t],
    "hcnn_sample_gaussian": [ptr, C.c_uint64, C.c_uint64, ptr, C.c_size_t],
    "hcnn_sample_uniform": [ptr, C.c_uint64, C.c_uint64, ptr, C.c_size_t],
    "hcnn_get_stat": [ptr, C.c_int, u64p],
    "hcnn_reset_stats": [ptr],
    "hcnn_set_option": [ptr, C.c_int, C.c_uint64],
    "hcnn_profile_read": [ptr, C.c_int, u64p, u64p, C.POINTER(C.c_double)],
    "hcnn_measure_ceiling": [ptr, C.c_int, C.POINTER(C.c_double)],
    "hcnn_strerror": [C.c_int],
}


def declare(lib: C.CDLL) -> C.CDLL:
    """Attach argtypes/restype for every symbol of the header; raises AttributeError if one is missing."""
    for name, argtypes in SIGNATURES.items():
        fn = getattr(lib, name)
        fn.argtypes = argtypes
        fn.restype = C.c_char_p if name == "hcnn_strerror" else C.c_int
    return lib


class HcnnError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("hcnn error %d: %s" % (code, msg))
        self.code = code


def check(lib, code):
    if code != 0:
        raise HcnnError(code, lib.hcnn_strerror(code).decode())


def u32_array(values):
    arr = (C.c_uint32 * len(values))(*[int(v) for v in values])
    return arr


def gen_primes(lib, n, count):
    out = (C.c_uint32 * count)()
    check(lib, lib.hcnn_gen_primes(n, count, out))
    return [int(v) for v in out]


def min_aux_count(lib, n, q, t, candidates):
    out = C.c_uint32(0)
    check(lib, lib.hcnn_min_aux_count(n, len(q), u32_array(q), t, u32_array(candidates), len(candidates),
                                      C.byref(out)))
    return int(out.value)


class RawContext:
    """Thin owner of an hcnn_ctx*.  Buffers are passed as integer addresses."""

    def __init__(self, lib, n, q, p, t, stream=0):
        self.lib, self.n, self.q, self.p, self.t = lib, int(n), list(q), list(p), int(t)
        self.k, self.k_aux = len(self.q), len(self.p)
        h = ptr()
        check(lib, lib.hcnn_ctx_create(C.byref(h), self.n, self.k, u32_array(self.q), self.k_aux,
                                       u32_array(self.p) if self.p else None, self.t, ptr(stream)))
        self.handle = h

    def close(self):
        if self.handle:
            self.lib.hcnn_ctx_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def call(self, name, *args):
        check(self.lib, getattr(self.lib, name)(self.handle, *args))

    def stat(self, which):
        out = C.c_uint64(0)
        check(self.lib, self.lib.hcnn_get_stat(self.handle, which, C.byref(out)))
        return int(out.value)

    def profile(self):
        """{class name: (launches, blocks, total_ms)} accumulated since the last reset."""
        out = {}
        for cls, name in enumerate(PROF_CLASSES):
            a, b, ms = C.c_uint64(0), C.c_uint64(0), C.c_double(0.0)
            check(self.lib, self.lib.hcnn_profile_read(self.handle, cls, C.byref(a), C.byref(b), C.byref(ms)))
            out[name] = (int(a.value), int(b.value), float(ms.value))
        return out

    def ceilings(self):
        """{name: value} of hcnn_measure_ceiling: GB/s for the streaming kernels, 10^12 lane-instructions/s else."""
        out = {}
        for which, name in enumerate(CEILINGS):
            v = C.c_double(0.0)
            check(self.lib, self.lib.hcnn_measure_ceiling(self.handle, which, C.byref(v)))
            out[name] = float(v.value)
        return out

    def set_option(self, which, value):
        check(self.lib, self.lib.hcnn_set_option(self.handle, which, C.c_uint64(value)))
