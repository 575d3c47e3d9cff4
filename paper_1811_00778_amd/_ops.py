"""Entry points of include/hcnn.h as methods; array handling is supplied by a subclass.

A subclass provides
    _ptr(x)                      integer address of array x (device memory in the product)
    _empty(shape, dtype_name)    new uninitialised array ("u32" or "i32")
    _check(x, dtype_name)        raises unless x is a contiguous array of that type
Marshalling only: no arithmetic of the method happens here.
"""
from . import _capi


class OpsMixin:
    raw: _capi.RawContext

    def close(self):
        self.raw.close()

    def _pre_call(self):
        """Hook run before every library call that enqueues work (the device binding checks the stream here)."""

    def _call(self, name, *args):
        self._pre_call()
        self.raw.call(name, *args)

    def _shape(self, x, shape, what):
        """The C ABI cannot see sizes: every buffer's full shape is checked here, before its address is passed on."""
        if tuple(x.shape) != tuple(shape):
            raise ValueError("%s must have shape %r, got %r" % (what, tuple(shape), tuple(x.shape)))

    # ---- shapes
    @property
    def n(self):
        return self.raw.n

    @property
    def k(self):
        return self.raw.k

    @property
    def ct_shape(self):
        return (2, self.raw.k, self.raw.n)

    # ---- hot path
    def ntt_fwd(self, polys):
        """In-place forward negacyclic NTT of polys [n_polys][k][n] (hcnn_ntt_fwd)."""
        self._check(polys, "u32")
        self._call("hcnn_ntt_fwd", self._ptr(polys), self._count(polys, (self.k, self.n)))
        return polys

    def ntt_inv(self, polys):
        """In-place inverse negacyclic NTT (hcnn_ntt_inv)."""
        self._check(polys, "u32")
        self._call("hcnn_ntt_inv", self._ptr(polys), self._count(polys, (self.k, self.n)))
        return polys

    def ct_scalar_mac(self, in_cts, idx, w, w_abs_max, out=None):
        """out[f][g] = sum_tau w[g][f][tau] * in[idx[g][tau]] (hcnn_ct_scalar_mac).
        in_cts [n_in][2][k][n]; idx [G][T] u32; w [G][F][T] i32; returns [F][G][2][k][n]."""
        self._check(in_cts, "u32"); self._check(idx, "u32"); self._check(w, "i32")
        n_in = self._count(in_cts, self.ct_shape)
        G, T = tuple(idx.shape)
        Gw, F, Tw = tuple(w.shape)
        if (Gw, Tw) != (G, T):
            raise ValueError("w must be [G][F][T] matching idx [G][T]")
        if out is None:
            out = self._empty((F, G) + self.ct_shape, "u32")
        self._check(out, "u32")
        if tuple(out.shape) != (F, G) + self.ct_shape:
            raise ValueError("out must be [F][G][2][k][n]")
        if self._overlap(in_cts, out):
            raise ValueError("out must not overlap in_cts")
        self._call("hcnn_ct_scalar_mac", self._ptr(in_cts), n_in, self._ptr(idx), self._ptr(w),
                      int(w_abs_max), G, F, T, self._ptr(out))
        return out

    def set_relin_key(self, evk):
        self._check(evk, "u32")
        if tuple(evk.shape) != (self.k, 2, self.k, self.n):
            raise ValueError("evk must be [k][2][k][n]")
        self._call("hcnn_set_relin_key", self._ptr(evk))

    def ct_square_relin(self, in_cts, out=None):
        """Square + scale + relinearise every ciphertext of in_cts [n_ct][2][k][n] (hcnn_ct_square_relin)."""
        self._check(in_cts, "u32")
        n_ct = self._count(in_cts, self.ct_shape)
        if out is None:
            out = self._empty(tuple(in_cts.shape), "u32")
        self._check(out, "u32")
        if tuple(out.shape) != tuple(in_cts.shape):
            raise ValueError("out must have the shape of in_cts")
        self._call("hcnn_ct_square_relin", self._ptr(in_cts), n_ct, self._ptr(out))
        return out

    def ct_square_relin_noalloc(self, in_cts, out):
        """ct_square_relin for callers that cannot allocate: `out` is required, the library works in its static
        device array and calls no allocator (hcnn_ct_square_relin_noalloc)."""
        self._check(in_cts, "u32"); self._check(out, "u32")
        n_ct = self._count(in_cts, self.ct_shape)
        if tuple(out.shape) != tuple(in_cts.shape):
            raise ValueError("out must have the shape of in_cts")
        self._call("hcnn_ct_square_relin_noalloc", self._ptr(in_cts), n_ct, self._ptr(out))
        return out

    def ct_mul_relin(self, a_cts, b_cts, out=None):
        """HMult of every pair (a_i, b_i), with scaling and relinearisation (hcnn_ct_mul_relin)."""
        self._check(a_cts, "u32"); self._check(b_cts, "u32")
        n_ct = self._count(a_cts, self.ct_shape)
        if tuple(b_cts.shape) != tuple(a_cts.shape):
            raise ValueError("a and b must have the same shape")
        if out is None:
            out = self._empty(tuple(a_cts.shape), "u32")
        self._check(out, "u32")
        self._shape(out, a_cts.shape, "out")
        self._call("hcnn_ct_mul_relin", self._ptr(a_cts), self._ptr(b_cts), n_ct, self._ptr(out))
        return out

    # ---- test helpers
    def keygen(self, s, a, e, a_evk=None, e_evk=None):
        self._check(s, "i32"); self._check(a, "u32"); self._check(e, "i32")
        self._shape(s, (self.n,), "s"); self._shape(a, (self.k, self.n), "a"); self._shape(e, (self.n,), "e")
        pk = self._empty(self.ct_shape, "u32")
        evk = None
        if a_evk is not None:
            if e_evk is None:
                raise ValueError("e_evk is required with a_evk")
            self._check(a_evk, "u32"); self._check(e_evk, "i32")
            self._shape(a_evk, (self.k, self.k, self.n), "a_evk"); self._shape(e_evk, (self.k, self.n), "e_evk")
            evk = self._empty((self.k, 2, self.k, self.n), "u32")
        self._call("hcnn_keygen", self._ptr(s), self._ptr(a), self._ptr(e),
                      self._ptr(a_evk) if a_evk is not None else None,
                      self._ptr(e_evk) if e_evk is not None else None,
                      self._ptr(pk), self._ptr(evk) if evk is not None else None)
        return pk, evk

    @property
    def wide_plaintext(self):
        """True when t needs 64-bit plaintext words (hcnn_encrypt_wide / hcnn_decrypt_wide)."""
        return self.raw.t >= (1 << 32)

    def encrypt(self, pk, m, u, e1, e2):
        """m [n_ct][n] in [0,t) (u32 words, u64 when t >= 2^32); u, e1, e2 [n_ct][n] i32 -> [n_ct][2][k][n]
        (hcnn_encrypt / hcnn_encrypt_wide)."""
        word = "u64" if self.wide_plaintext else "u32"
        for x, d in ((pk, "u32"), (m, word), (u, "i32"), (e1, "i32"), (e2, "i32")):
            self._check(x, d)
        n_ct = self._count(m, (self.n,))
        self._shape(pk, self.ct_shape, "pk")
        self._shape(m, (n_ct, self.n), "m")
        for x, what in ((u, "u"), (e1, "e1"), (e2, "e2")):
            self._shape(x, (n_ct, self.n), what)
        out = self._empty((n_ct,) + self.ct_shape, "u32")
        self._call("hcnn_encrypt_wide" if self.wide_plaintext else "hcnn_encrypt", self._ptr(pk), self._ptr(m),
                      self._ptr(u), self._ptr(e1), self._ptr(e2), n_ct, self._ptr(out))
        return out

    def decrypt(self, sk, cts):
        """-> plaintext polynomials [n_ct][n] (u32 words, u64 when t >= 2^32) (hcnn_decrypt / hcnn_decrypt_wide)."""
        self._check(sk, "i32"); self._check(cts, "u32")
        self._shape(sk, (self.n,), "sk")
        n_ct = self._count(cts, self.ct_shape)
        out = self._empty((n_ct, self.n), "u64" if self.wide_plaintext else "u32")
        self._call("hcnn_decrypt_wide" if self.wide_plaintext else "hcnn_decrypt", self._ptr(sk), self._ptr(cts),
                      n_ct, self._ptr(out))
        return out

    # ---- deterministic sampling (inputs for keygen / encrypt, produced on the device)
    def sample_ternary(self, seed, stream, n_polys):
        """int32 [n_polys][n], uniform on {-1, 0, 1} (hcnn_sample_ternary)."""
        out = self._empty((n_polys, self.n), "i32")
        self._call("hcnn_sample_ternary", int(seed), int(stream), self._ptr(out), n_polys)
        return out

    def sample_gaussian(self, seed, stream, n_polys):
        """int32 [n_polys][n], rounded Gaussian sigma = 3.2 cut at 19 (hcnn_sample_gaussian)."""
        out = self._empty((n_polys, self.n), "i32")
        self._call("hcnn_sample_gaussian", int(seed), int(stream), self._ptr(out), n_polys)
        return out

    def sample_uniform(self, seed, stream, n_polys):
        """uint32 [n_polys][k][n], row l uniform in [0, q_l) (hcnn_sample_uniform)."""
        out = self._empty((n_polys, self.k, self.n), "u32")
        self._call("hcnn_sample_uniform", int(seed), int(stream), self._ptr(out), n_polys)
        return out

    def noise_bits(self, sk, cts):
        """Bit length of the largest centred remainder of t*(c0 + c1*s) mod q per ciphertext (hcnn_noise_bits);
        the noise budget is log2(q) - 1 - bits."""
        self._check(sk, "i32"); self._check(cts, "u32")
        self._shape(sk, (self.n,), "sk")
        n_ct = self._count(cts, self.ct_shape)
        out = self._empty((n_ct,), "u32")
        self._call("hcnn_noise_bits", self._ptr(sk), self._ptr(cts), n_ct, self._ptr(out))
        return out

    # ---- diagnostics
    def exact_fallbacks(self):
        return self.raw.stat(_capi.STAT_EXACT_FALLBACKS)

    def bad_inputs(self):
        return self.raw.stat(_capi.STAT_BAD_INPUT)

    def scratch_bytes(self):
        return self.raw.stat(_capi.STAT_SCRATCH_BYTES)

    def relin_fused_round(self):
        """Ciphertexts per round of the one-kernel relinearisation under the default policy (from the occupancy that
        the runtime reports for the compiled kernel; 0 when even one ciphertext's workgroups do not fit)."""
        return self.raw.stat(_capi.STAT_RELIN_FUSED_WGS) // 8 // self.k * 8

    def tensor_fused_threshold(self):
        """(ciphertext, limb) pairs from which the default policy takes the one-kernel squaring tensor."""
        return 6 * self.raw.stat(_capi.STAT_TENSOR_FUSED_WGS)

    def reset_stats(self):
        self._call("hcnn_reset_stats")

    def set_ambiguity_band(self, band):
        self.raw.set_option(_capi.OPT_AMBIGUITY_BAND, band)

    def set_profile(self, on):
        self.raw.set_option(_capi.OPT_PROFILE, 1 if on else 0)

    def profile(self):
        return self.raw.profile()

    def measured_ceilings(self):
        """Streaming and instruction-issue rates measured on this device (hcnn_measure_ceiling)."""
        return self.raw.ceilings()

    def set_relin_order(self, order):
        self.raw.set_option(_capi.OPT_RELIN_ORDER, order)

    def set_fusion(self, mode):
        """One-kernel forms of the squaring tensor and the relinearisation: 0 chosen per batch, 1 never, 2 always."""
        self.raw.set_option(_capi.OPT_FUSION, int(mode))

    def set_square_chunk(self, chunk):
        self.raw.set_option(_capi.OPT_SQUARE_CHUNK, chunk)

    # ---- helpers
    def _overlap(self, a, b):
        """True when the two buffers share any byte."""
        pa, pb = self._ptr(a).value or 0, self._ptr(b).value or 0
        na, nb = self._nbytes(a), self._nbytes(b)
        return pa < pb + nb and pb < pa + na

    @staticmethod
    def _nbytes(x):
        count = 1
        for d in x.shape:
            count *= int(d)
        return count * (x.element_size() if hasattr(x, "element_size") else x.itemsize)

    @staticmethod
    def _count(x, tail):
        shape = tuple(x.shape)
        tail = tuple(tail)
        if len(shape) < len(tail) or shape[len(shape) - len(tail):] != tail:
            raise ValueError("expected trailing shape %r, got %r" % (tail, shape))
        cnt = 1
        for d in shape[:len(shape) - len(tail)]:
            cnt *= int(d)
        return cnt
