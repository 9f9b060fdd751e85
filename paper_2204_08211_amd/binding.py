"""Thin ctypes binding of libco3.so (include/co3.h): argument marshalling only.

torch is used for device memory and streams; every step of the codec runs in the HIP
kernels of the library.  There is no CPU fallback: loading fails loudly when the library has
not been built (python -m paper_2204_08211_amd.build).
"""
import ctypes as C
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libco3.so")

CHUNK = 4096
SUB = 64
SUBS_PER_CHUNK = 64
STATUS_WORDS = 8
(STAT_NONFINITE, STAT_CLAMPED, STAT_NOCODE, STAT_CAPACITY, STAT_CODELEN, STAT_CORRUPT, STAT_STALLED) = range(7)
BOOK_FIXED, BOOK_EMPIRICAL = 0, 1
OK, ERR_ARG, ERR_FORMAT, ERR_CAPACITY, ERR_CODELEN, ERR_CORRUPT, ERR_HIP = 0, -1, -2, -3, -4, -5, -6

EXPORTS = [
    "co3_plan_create", "co3_plan_set_bias", "co3_plan_destroy", "co3_plan_num_chunks", "co3_plan_num_books",
    "co3_plan_alphabet", "co3_plan_symbols_bytes", "co3_plan_workspace_bytes", "co3_plan_stream_words",
    "co3_build_codebook", "co3_build_codebook_device", "co3_codebook_export", "co3_codebook_num_books",
    "co3_codebook_destroy", "co3_encode", "co3_decode", "co3_ps_aggregate", "co3_status_string",
    "co3_profile_begin", "co3_profile_end", "co3_gennorm_weights", "co3_plan_fit_workspace_bytes", "co3_gennorm_fit",
    "co3_model_weights_device", "co3_model_bias_device", "co3_plan_set_bias_device", "co3_bias_from_model", "co3_scale_from_model",
    "co3_plan_scale_workspace_bytes", "co3_model_scale_device", "co3_plan_set_gain_device",
    "co3_plan_bias_workspace_bytes", "co3_set_lookback_polls", "co3_encode_static", "co3_plan_set_gain",
]


class Format(C.Structure):
    _fields_ = [("exp_bits", C.c_int32), ("mant_bits", C.c_int32)]


class GennormParams(C.Structure):
    _fields_ = [("mu", C.c_double), ("alpha", C.c_double), ("beta", C.c_double), ("kurtosis", C.c_double)]


class Segment(C.Structure):
    _fields_ = [("offset", C.c_uint64), ("length", C.c_uint64), ("codebook", C.c_int32), ("reserved", C.c_int32)]


class EncodeArgs(C.Structure):
    _fields_ = [("g", C.c_void_p), ("m", C.c_void_p), ("m_out", C.c_void_p), ("row_stride", C.c_uint64),
                ("gamma", C.c_float), ("mode", C.c_int32), ("books", C.c_void_p), ("symbols", C.c_void_p),
                ("hist", C.c_void_p), ("words", C.c_void_p), ("words_stride", C.c_uint64),
                ("chunk_offset", C.c_void_p), ("sub_bits", C.c_void_p), ("payload_bits", C.c_void_p),
                ("status", C.c_void_p), ("workspace", C.c_void_p), ("workspace_bytes", C.c_size_t),
                ("rounding", C.c_int32), ("reserved", C.c_int32), ("seed", C.c_uint64)]


class DecodeArgs(C.Structure):
    _fields_ = [("words", C.c_void_p), ("words_stride", C.c_uint64), ("chunk_offset", C.c_void_p),
                ("sub_bits", C.c_void_p), ("books", C.c_void_p), ("symbols", C.c_void_p), ("q", C.c_void_p),
                ("q_stride", C.c_uint64), ("status", C.c_void_p)]


class AggregateArgs(C.Structure):
    _fields_ = [("words", C.c_void_p), ("words_stride", C.c_uint64), ("chunk_offset", C.c_void_p),
                ("sub_bits", C.c_void_p), ("books", C.c_void_p), ("out", C.c_void_p), ("status", C.c_void_p),
                ("model", C.c_void_p), ("eta", C.c_float), ("reserved", C.c_int32)]


class KernelTime(C.Structure):
    _fields_ = [("name", C.c_char * 32), ("total_ms", C.c_double), ("launches", C.c_uint64)]


class Co3Error(RuntimeError):
    def __init__(self, where, code):
        self.code = code
        super().__init__(f"{where}: {status_string(code)} ({code})")


_lib = None


def lib():
    """The loaded library.  Raises if it has not been built: there is no fallback path."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2204_08211_amd.build`")
        L = C.CDLL(LIB_PATH)
        L.co3_plan_create.argtypes = [Format, C.c_uint32, C.c_uint64, C.c_uint32, C.c_void_p, C.c_void_p,
                                      C.c_int32, C.POINTER(C.c_void_p)]
        L.co3_plan_set_bias.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
        L.co3_plan_set_gain.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.co3_plan_destroy.argtypes = [C.c_void_p]
        L.co3_plan_destroy.restype = None
        for name, rt in [("co3_plan_num_chunks", C.c_uint64), ("co3_plan_num_books", C.c_uint32),
                         ("co3_plan_alphabet", C.c_uint32), ("co3_plan_symbols_bytes", C.c_size_t),
                         ("co3_plan_workspace_bytes", C.c_size_t), ("co3_plan_fit_workspace_bytes", C.c_size_t),
                         ("co3_plan_bias_workspace_bytes", C.c_size_t)]:
            getattr(L, name).argtypes = [C.c_void_p]
            getattr(L, name).restype = rt
        L.co3_plan_stream_words.argtypes = [C.c_void_p, C.c_uint32]
        L.co3_plan_stream_words.restype = C.c_uint64
        L.co3_build_codebook.argtypes = [Format, C.c_uint32, C.c_void_p, C.POINTER(C.c_void_p)]
        L.co3_build_codebook_device.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.co3_codebook_export.argtypes = [C.c_void_p, C.c_uint32, C.c_void_p, C.c_void_p, C.c_void_p]
        L.co3_codebook_num_books.argtypes = [C.c_void_p]
        L.co3_codebook_num_books.restype = C.c_uint32
        L.co3_codebook_destroy.argtypes = [C.c_void_p]
        L.co3_codebook_destroy.restype = None
        L.co3_encode.argtypes = [C.c_void_p, C.POINTER(EncodeArgs), C.c_void_p]
        L.co3_encode_static.argtypes = [C.c_void_p, C.POINTER(EncodeArgs), C.c_void_p]
        L.co3_decode.argtypes = [C.c_void_p, C.POINTER(DecodeArgs), C.c_void_p]
        L.co3_ps_aggregate.argtypes = [C.c_void_p, C.POINTER(AggregateArgs), C.c_void_p]
        L.co3_profile_end.argtypes = [C.POINTER(KernelTime), C.c_uint32, C.POINTER(C.c_uint32)]
        L.co3_gennorm_weights.argtypes = [Format, C.c_int32, C.c_double, C.c_double, C.c_double, C.c_void_p]
        L.co3_gennorm_fit.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint64, C.c_float, C.c_void_p, C.c_void_p,
                                      C.c_size_t, C.c_void_p]
        L.co3_model_weights_device.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.co3_model_bias_device.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t,
                                            C.c_void_p]
        L.co3_plan_set_bias_device.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
        L.co3_plan_scale_workspace_bytes.argtypes = [C.c_void_p]
        L.co3_plan_scale_workspace_bytes.restype = C.c_size_t
        L.co3_model_scale_device.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                             C.c_size_t, C.c_void_p]
        L.co3_plan_set_gain_device.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
        L.co3_bias_from_model.argtypes = [Format, C.c_double, C.c_double, C.c_double, C.POINTER(C.c_int32),
                                          C.POINTER(C.c_double)]
        L.co3_scale_from_model.argtypes = [Format, C.c_double, C.c_double, C.c_double, C.POINTER(C.c_int32),
                                           C.POINTER(C.c_float), C.POINTER(C.c_float), C.POINTER(C.c_double)]
        L.co3_set_lookback_polls.argtypes = [C.c_uint32]
        L.co3_set_lookback_polls.restype = None
        L.co3_status_string.argtypes = [C.c_int]
        L.co3_status_string.restype = C.c_char_p
        _lib = L
    return _lib


def profile_begin():
    _check("co3_profile_begin", lib().co3_profile_begin())


def profile_end():
    """{kernel name: (total ms, launches)} for the launches since profile_begin()."""
    arr = (KernelTime * 16)()
    n = C.c_uint32(0)
    _check("co3_profile_end", lib().co3_profile_end(arr, 16, C.byref(n)))
    return {arr[i].name.decode(): (arr[i].total_ms, int(arr[i].launches)) for i in range(n.value)}


LOOKBACK_POLLS_DEFAULT = 1 << 20


def set_lookback_polls(polls):
    """Bound of the single-sweep encoder's wait for the chunks ahead (re-reads per entry); 0 gives up at once."""
    lib().co3_set_lookback_polls(int(polls))


def status_string(code):
    return lib().co3_status_string(int(code)).decode()


def _check(where, rc):
    if rc != OK:
        raise Co3Error(where, rc)


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(stream=None):
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


class Plan:
    """co3_plan: U users, d elements, [sgn,exp,mant] format, layers and per-(user, layer) bias."""

    def __init__(self, E, M, U, d, bias, seg_len=None, seg_book=None, per_user_books=False):
        self.E, self.M, self.U, self.d = int(E), int(M), int(U), int(d)
        self.seg_len = [int(d)] if seg_len is None else [int(x) for x in seg_len]
        self.nseg = len(self.seg_len)
        self.seg_book = [0] * self.nseg if seg_book is None else [int(x) for x in seg_book]
        self.per_user_books = bool(per_user_books)
        bias = np.ascontiguousarray(np.broadcast_to(np.asarray(bias, dtype=np.int32), (self.U, self.nseg)))
        segs = (Segment * self.nseg)()
        off = 0
        for k, (n, b) in enumerate(zip(self.seg_len, self.seg_book)):
            segs[k] = Segment(off, n, b, 0)
            off += n
        h = C.c_void_p()
        _check("co3_plan_create", lib().co3_plan_create(Format(self.E, self.M), self.U, self.d, self.nseg,
                                                        C.cast(segs, C.c_void_p), bias.ctypes.data_as(C.c_void_p),
                                                        int(self.per_user_books), C.byref(h)))
        self.handle = h
        self.bias = bias
        self.num_chunks = int(lib().co3_plan_num_chunks(h))
        self.num_books = int(lib().co3_plan_num_books(h))
        self.A = int(lib().co3_plan_alphabet(h))
        self.symbols_bytes = int(lib().co3_plan_symbols_bytes(h))
        self.workspace_bytes = int(lib().co3_plan_workspace_bytes(h))
        self.sym_stride = (self.d + 127) // 128 * 128
        self.wide = self.A > 256          # alphabets above 8 bits: 16-bit symbols

    def set_bias(self, bias, stream=None):
        bias = np.ascontiguousarray(np.broadcast_to(np.asarray(bias, dtype=np.int32), (self.U, self.nseg)))
        _check("co3_plan_set_bias", lib().co3_plan_set_bias(self.handle, bias.ctypes.data_as(C.c_void_p), _stream(stream)))
        self.bias = bias

    def set_gain(self, gain, inv_gain, stream=None):
        """Real-valued scale on top of the integer bias: float32 [U][nseg] pairs (None, None: back to 1)."""
        if gain is None:
            _check("co3_plan_set_gain", lib().co3_plan_set_gain(self.handle, None, None, _stream(stream)))
            return
        gain = np.ascontiguousarray(np.broadcast_to(np.asarray(gain, dtype=np.float32), (self.U, self.nseg)))
        inv_gain = np.ascontiguousarray(np.broadcast_to(np.asarray(inv_gain, dtype=np.float32), (self.U, self.nseg)))
        _check("co3_plan_set_gain", lib().co3_plan_set_gain(self.handle, gain.ctypes.data_as(C.c_void_p),
                                                          inv_gain.ctypes.data_as(C.c_void_p), _stream(stream)))

    def stream_words(self, max_code_len=64):
        return int(lib().co3_plan_stream_words(self.handle, int(max_code_len)))

    def close(self):
        if getattr(self, "handle", None):
            lib().co3_plan_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Codebook:
    """co3_codebook: a set of Huffman code tables living on the device."""

    def __init__(self, handle, E, M, nbooks):
        self.handle, self.E, self.M, self.nbooks = handle, E, M, nbooks
        self.A = 1 << (1 + E + M)

    def export(self, book=0, stream=None):
        length = np.zeros(self.A, np.uint8)
        code = np.zeros(self.A, np.uint64)
        _check("co3_codebook_export", lib().co3_codebook_export(self.handle, int(book), length.ctypes.data_as(C.c_void_p),
                                                                code.ctypes.data_as(C.c_void_p), _stream(stream)))
        return length, code

    def close(self):
        if getattr(self, "handle", None):
            lib().co3_codebook_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def co3_build_codebook(E, M, nbooks, weights=None):
    """Huffman tables from host integer weights [nbooks][A] (None: empty set for device builds)."""
    h = C.c_void_p()
    wp = None
    if weights is not None:
        weights = np.ascontiguousarray(weights, dtype=np.uint64).reshape(nbooks, 1 << (1 + E + M))
        wp = weights.ctypes.data_as(C.c_void_p)
    _check("co3_build_codebook", lib().co3_build_codebook(Format(E, M), int(nbooks), wp, C.byref(h)))
    return Codebook(h, E, M, nbooks)


def co3_gennorm_weights(E, M, bias, mu, alpha, beta):
    """uint64[A] Huffman weights of the symbols when g + gamma m is GenNorm(mu, alpha, beta)."""
    w = np.zeros(1 << (1 + E + M), dtype=np.uint64)
    _check("co3_gennorm_weights", lib().co3_gennorm_weights(Format(E, M), int(bias), float(mu), float(alpha),
                                                            float(beta), w.ctypes.data_as(C.c_void_p)))
    return w


def co3_build_codebook_device(books, weights, status, stream=None):
    """Rebuild the set from device weights (uint64 viewed as an int64 tensor [nbooks][A])."""
    _check("co3_build_codebook_device",
           lib().co3_build_codebook_device(books.handle, _ptr(weights), _ptr(status), _stream(stream)))


def co3_gennorm_fit(plan, g, m, gamma, params=None, workspace=None, stream=None):
    """GenNorm(mu, alpha, beta) of v = g + gamma m per user and layer by matching mean, variance and
    kurtosis (Sec. III eq. (kurtosis)).  Returns a float64 device tensor [U][nseg][4] = (mu, alpha, beta,
    kurtosis); g, m are float32 device tensors [U][row_stride]."""
    import torch
    assert g.dim() == 2 and g.shape == m.shape and g.stride(1) == 1 and g.stride(0) == m.stride(0)
    if params is None:
        params = torch.zeros((plan.U, plan.nseg, 4), dtype=torch.float64, device=g.device)
    if workspace is None:
        workspace = torch.empty(int(lib().co3_plan_fit_workspace_bytes(plan.handle)), dtype=torch.uint8, device=g.device)
    _check("co3_gennorm_fit", lib().co3_gennorm_fit(plan.handle, g.data_ptr(), m.data_ptr(), g.stride(0),
                                                      float(np.float32(gamma)), params.data_ptr(), workspace.data_ptr(),
                                                      workspace.numel(), _stream(stream)))
    return params


def co3_model_weights_device(plan, params, weights=None, stream=None):
    """Integer weights [num_books][A] (uint64 viewed as an int64 device tensor) of the model code for fitted
    parameters; feed them to co3_build_codebook_device."""
    import torch
    if weights is None:
        weights = torch.zeros((plan.num_books, plan.A), dtype=torch.int64, device=params.device)
    _check("co3_model_weights_device",
           lib().co3_model_weights_device(plan.handle, params.data_ptr(), weights.data_ptr(), _stream(stream)))
    return weights


def co3_model_bias_device(plan, params, install=True, stream=None):
    """Exponent bias per user and layer from fitted parameters (eq. (exp bias) with integer b): returns
    (int32 device tensor [U][nseg], float64 device tensor [U][nseg] of expected squared errors) and, with
    install, makes it the plan's bias table."""
    import torch
    bias = torch.zeros((plan.U, plan.nseg), dtype=torch.int32, device=params.device)
    err = torch.zeros((plan.U, plan.nseg), dtype=torch.float64, device=params.device)
    ws = torch.empty(int(lib().co3_plan_bias_workspace_bytes(plan.handle)), dtype=torch.uint8, device=params.device)
    _check("co3_model_bias_device",
           lib().co3_model_bias_device(plan.handle, params.data_ptr(), bias.data_ptr(), err.data_ptr(), ws.data_ptr(),
                                       ws.numel(), _stream(stream)))
    if install:
        _check("co3_plan_set_bias_device", lib().co3_plan_set_bias_device(plan.handle, bias.data_ptr(), _stream(stream)))
    return bias, err


def co3_model_scale_device(plan, params, install=True, stream=None):
    """Exponent bias and real-valued scale per user and layer from fitted parameters (eq. (exp bias) with real b):
    returns (int32 device tensor [U][nseg], float32 device tensor [U][nseg][2] of (gain, inv_gain), float64 device
    tensor [U][nseg] of expected squared errors) and, with install, makes them the plan's bias and scale."""
    import torch
    bias = torch.zeros((plan.U, plan.nseg), dtype=torch.int32, device=params.device)
    pairs = torch.ones((plan.U, plan.nseg, 2), dtype=torch.float32, device=params.device)
    err = torch.zeros((plan.U, plan.nseg), dtype=torch.float64, device=params.device)
    ws = torch.empty(int(lib().co3_plan_scale_workspace_bytes(plan.handle)), dtype=torch.uint8, device=params.device)
    _check("co3_model_scale_device",
           lib().co3_model_scale_device(plan.handle, params.data_ptr(), bias.data_ptr(), pairs.data_ptr(), err.data_ptr(),
                                        ws.data_ptr(), ws.numel(), _stream(stream)))
    if install:
        _check("co3_plan_set_bias_device", lib().co3_plan_set_bias_device(plan.handle, bias.data_ptr(), _stream(stream)))
        _check("co3_plan_set_gain_device", lib().co3_plan_set_gain_device(plan.handle, pairs.data_ptr(), _stream(stream)))
    return bias, pairs, err


def co3_scale_from_model(E, M, mu, alpha, beta):
    """eq. (exp bias) with real b on the host: (bias, gain, inv_gain, expected squared error); the pair is what
    Plan.set_gain takes."""
    b = C.c_int32(0)
    gn, ig = C.c_float(1.0), C.c_float(1.0)
    e = C.c_double(0.0)
    _check("co3_scale_from_model", lib().co3_scale_from_model(Format(E, M), float(mu), float(alpha), float(beta),
                                                            C.byref(b), C.byref(gn), C.byref(ig), C.byref(e)))
    return int(b.value), float(gn.value), float(ig.value), float(e.value)


def co3_bias_from_model(E, M, mu, alpha, beta):
    """(bias, expected squared error) of eq. (exp bias) with integer b for GenNorm(mu, alpha, beta); host."""
    b = C.c_int32(0)
    e = C.c_double(0.0)
    _check("co3_bias_from_model", lib().co3_bias_from_model(Format(E, M), float(mu), float(alpha), float(beta),
                                                          C.byref(b), C.byref(e)))
    return int(b.value), float(e.value)


class RoundBuffers:
    """Device buffers of one round, allocated with torch (plumbing only)."""

    def __init__(self, plan, device="cuda:0", words_stride=None, max_code_len=32):
        import torch
        self.plan = plan
        U, nch = plan.U, plan.num_chunks
        self.words_stride = int(words_stride) if words_stride is not None else plan.stream_words(max_code_len)
        dev = torch.device(device)
        self.symbols = torch.zeros(plan.symbols_bytes, dtype=torch.uint8, device=dev)
        self.hist = torch.zeros((plan.num_books, plan.A), dtype=torch.int64, device=dev)
        self.words = torch.zeros((U, self.words_stride), dtype=torch.int32, device=dev)
        self.chunk_offset = torch.zeros((U, nch + 1), dtype=torch.int64, device=dev)
        self.sub_bits = torch.zeros((U, nch * SUBS_PER_CHUNK), dtype=torch.int16, device=dev)
        self.payload_bits = torch.zeros(U, dtype=torch.int64, device=dev)
        self.status = torch.zeros(STATUS_WORDS, dtype=torch.int64, device=dev)
        self.workspace = torch.zeros(plan.workspace_bytes, dtype=torch.uint8, device=dev)

    def symbols_2d(self):
        return symbols_2d(self.plan, self.symbols)


def symbols_2d(plan, buf):
    """[U][d] view of a symbols buffer (uint8 tensor of plan.symbols_bytes): bytes, or 16-bit words for wide alphabets."""
    import torch
    if plan.wide:
        return buf[:2 * plan.U * plan.sym_stride].view(torch.int16).view(plan.U, plan.sym_stride)[:, :plan.d]
    return buf[:plan.U * plan.sym_stride].view(plan.U, plan.sym_stride)[:, :plan.d]


ROUND_NEAREST, ROUND_STOCHASTIC = 0, 1


STATIC_SCRATCH_BYTES = 8 << 20


def co3_encode(plan, books, g, m, m_out, gamma, buf, mode=BOOK_EMPIRICAL, stream=None, single_sweep=False,
               stochastic_seed=None, static=False, single_sweep_hist=False):
    """User side of one round for all U users (Algorithm 1 lines 8-10).  g, m, m_out are float32
    device tensors [U][row_stride]; outputs land in `buf` (RoundBuffers).  single_sweep (fixed code
    only) passes no symbols and no hist buffer, which selects the library's single-sweep encoder;
    single_sweep_hist passes the hist buffer all the same (the sweep then also counts the symbols).
    stochastic_seed: None = closest representative, else the stochastic conversion keyed by that seed.
    static: call co3_encode_static (the library's own static workspace, no allocation; buf.workspace is not passed)."""
    assert not single_sweep or mode == BOOK_FIXED
    assert g.dim() == 2 and g.shape == m.shape == m_out.shape and g.stride(1) == 1
    assert g.stride(0) == m.stride(0) == m_out.stride(0)
    a = EncodeArgs(g.data_ptr(), m.data_ptr(), m_out.data_ptr(), g.stride(0), float(np.float32(gamma)), int(mode),
                   books.handle, None if single_sweep else buf.symbols.data_ptr(),
                   None if (single_sweep and not single_sweep_hist) else buf.hist.data_ptr(), buf.words.data_ptr(),
                   buf.words_stride, buf.chunk_offset.data_ptr(), buf.sub_bits.data_ptr(),
                   buf.payload_bits.data_ptr(), buf.status.data_ptr(), None if static else buf.workspace.data_ptr(),
                   0 if static else buf.workspace.numel(), ROUND_NEAREST if stochastic_seed is None else ROUND_STOCHASTIC, 0,
                   0 if stochastic_seed is None else int(stochastic_seed) & 0xffffffffffffffff)
    if static:
        _check("co3_encode_static", lib().co3_encode_static(plan.handle, C.byref(a), _stream(stream)))
    else:
        _check("co3_encode", lib().co3_encode(plan.handle, C.byref(a), _stream(stream)))


def co3_decode(plan, books, buf, symbols=None, q=None, stream=None):
    """Invert the streams in `buf` into symbols (uint8, plan.symbols_bytes) and/or values q [U][stride]."""
    a = DecodeArgs(buf.words.data_ptr(), buf.words_stride, buf.chunk_offset.data_ptr(), buf.sub_bits.data_ptr(),
                   books.handle, None if symbols is None else symbols.data_ptr(),
                   None if q is None else q.data_ptr(), 0 if q is None else q.stride(0), buf.status.data_ptr())
    _check("co3_decode", lib().co3_decode(plan.handle, C.byref(a), _stream(stream)))


def co3_ps_aggregate(plan, books, buf, out, stream=None, model=None, eta=0.0):
    """PS side: out[d] = (1/U) sum_u ghat^(u) decoded from the streams in `buf`; with `model` (float32
    device tensor [d]) also model -= eta * that average (Algorithm 1 line 14), in the same pass.  `out`
    may be None when `model` is given."""
    assert out is not None or model is not None
    assert out is None or out.numel() >= plan.d
    assert model is None or (model.numel() >= plan.d and model.is_contiguous())
    a = AggregateArgs(buf.words.data_ptr(), buf.words_stride, buf.chunk_offset.data_ptr(), buf.sub_bits.data_ptr(),
                      books.handle, None if out is None else out.data_ptr(), buf.status.data_ptr(),
                      None if model is None else model.data_ptr(), float(np.float32(eta)), 0)
    _check("co3_ps_aggregate", lib().co3_ps_aggregate(plan.handle, C.byref(a), _stream(stream)))
