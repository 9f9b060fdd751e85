"""ctypes front end of the CPU oracle (oracle/co3_oracle.c).  TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this
module; the product package never does.  Every function cites the passage of the paper
(arXiv 2204.08211) whose definition it evaluates; the arithmetic lives in the C file,
except for the GenNorm cell probabilities below, which use SciPy's incomplete gamma
function as a library step.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

CHUNK = 4096
SUB = 64
SUBS_PER_CHUNK = CHUNK // SUB

OK, ERR_ARG, ERR_FORMAT, ERR_CAPACITY, ERR_CODELEN, ERR_CORRUPT, ERR_NOCODE = 0, -1, -2, -3, -4, -5, -7

_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.LIB
        if not os.path.exists(path) or os.path.getmtime(path) < os.path.getmtime(_build.SRC):
            _build.build()
        _lib = C.CDLL(path)
        _lib.co3o_value.restype = C.c_double
        _lib.co3o_value.argtypes = [C.c_uint32, C.c_int, C.c_int, C.c_int]
        _lib.co3o_num_chunks.restype = C.c_uint64
    return _lib


def _p(a, t):
    return a.ctypes.data_as(C.POINTER(t))


def is_wide(E, M):
    """Alphabets of more than 8 bits keep their symbols in 16-bit words (up to 12 bits are provided for)."""
    return 1 + E + M > 8


def num_magnitudes(E, M):
    return int(lib().co3o_num_magnitudes(C.c_int(E), C.c_int(M)))


def format_ok(E, M, bias):
    return bool(lib().co3o_format_ok(C.c_int(E), C.c_int(M), C.c_int(bias)))


def grid(E, M, bias):
    """Non-negative part of the representative set X of Sec. V-B, ascending."""
    mag = np.zeros(num_magnitudes(E, M), dtype=np.float64)
    rc = lib().co3o_grid(C.c_int(E), C.c_int(M), C.c_int(bias), _p(mag, C.c_double))
    if rc < 0:
        raise ValueError(f"co3o_grid: {rc}")
    return mag


def value(sym, E, M, bias):
    return float(lib().co3o_value(C.c_uint32(int(sym)), C.c_int(E), C.c_int(M), C.c_int(bias)))


def quantize_wide(v, E, M, bias):
    """Q_fp of Sec. IV-A (i) on an fp32 array, any format up to exp 8 / mant 23."""
    v = np.ascontiguousarray(v, dtype=np.float32)
    q = np.empty_like(v)
    code = np.empty(v.shape, dtype=np.uint32)
    rc = lib().co3o_quantize_wide(_p(v, C.c_float), C.c_uint64(v.size), C.c_int(E), C.c_int(M),
                                  C.c_int(bias), _p(q, C.c_float), _p(code, C.c_uint32))
    if rc < 0:
        raise ValueError(f"co3o_quantize_wide: {rc}")
    return q, code


def ef_step(g, m, gamma, E, M, bias, want_q=True):
    """Algorithm 1 lines 8 and 10 for one user and one layer.

    Returns (m_new, sym u8, q or None, counters[2] = (NaN/Inf, clamped))."""
    g = np.ascontiguousarray(g, dtype=np.float32)
    m = np.ascontiguousarray(m, dtype=np.float32)
    assert g.shape == m.shape and g.ndim == 1
    m_out = np.empty_like(g)
    wide = is_wide(E, M)                      # alphabets above 8 bits: symbols in 16-bit words
    sym = np.empty(g.shape, dtype=np.uint16 if wide else np.uint8)
    q = np.empty_like(g) if want_q else None
    counters = np.zeros(2, dtype=np.uint64)
    fn = lib().co3o_ef_step_w if wide else lib().co3o_ef_step
    rc = fn(_p(g, C.c_float), _p(m, C.c_float), C.c_uint64(g.size),
            C.c_float(np.float32(gamma)), C.c_int(E), C.c_int(M), C.c_int(bias),
            _p(m_out, C.c_float), sym.ctypes.data_as(C.c_void_p),
            _p(q, C.c_float) if want_q else None, _p(counters, C.c_uint64))
    if rc < 0:
        raise ValueError(f"co3o_ef_step: {rc}")
    return m_out, sym, q, counters


def ef_step_gain(g, m, gamma, E, M, bias, gain, inv_gain, want_q=True):
    """Algorithm 1 lines 8 and 10 with a real-valued scale on top of the integer bias (eq. (exp bias) with b in R;
    reading R16 in the C file): y = fl32(v gain), ghat = fl32(Q_fp(y) inv_gain), m' = fl32(v - ghat).
    Returns (m_new, sym, q or None, counters[2])."""
    g = np.ascontiguousarray(g, dtype=np.float32)
    m = np.ascontiguousarray(m, dtype=np.float32)
    assert g.shape == m.shape and g.ndim == 1
    m_out = np.empty_like(g)
    wide = is_wide(E, M)
    sym = np.empty(g.shape, dtype=np.uint16 if wide else np.uint8)
    q = np.empty_like(g) if want_q else None
    counters = np.zeros(2, dtype=np.uint64)
    rc = (lib().co3o_ef_step_gain_w if wide else lib().co3o_ef_step_gain)(
        _p(g, C.c_float), _p(m, C.c_float), C.c_uint64(g.size), C.c_float(np.float32(gamma)),
        C.c_int(E), C.c_int(M), C.c_int(bias), C.c_float(np.float32(gain)),
        C.c_float(np.float32(inv_gain)), _p(m_out, C.c_float), sym.ctypes.data_as(C.c_void_p),
        _p(q, C.c_float) if want_q else None, _p(counters, C.c_uint64))
    if rc < 0:
        raise ValueError(f"co3o_ef_step_gain: {rc}")
    return m_out, sym, q, counters


def aggregate_gain(sym, seg_len, bias, inv_gain, E, M):
    """(1/U) sum_u ghat^(u) with ghat = fl32(value(sym) inv_gain[u][layer]) (reading R16)."""
    wide = is_wide(E, M)
    sym = np.ascontiguousarray(sym, dtype=np.uint16 if wide else np.uint8)
    U, d = sym.shape
    seg_len = np.ascontiguousarray(seg_len, dtype=np.uint64)
    bias = np.ascontiguousarray(bias, dtype=np.int32).reshape(U, seg_len.size)
    inv_gain = np.ascontiguousarray(inv_gain, dtype=np.float32).reshape(U, seg_len.size)
    out = np.empty(d, dtype=np.float32)
    rc = (lib().co3o_aggregate_gain_w if wide else lib().co3o_aggregate_gain)(
        sym.ctypes.data_as(C.c_void_p), C.c_uint32(U), C.c_uint64(d), C.c_int(seg_len.size),
        _p(seg_len, C.c_uint64), _p(bias, C.c_int32), _p(inv_gain, C.c_float), C.c_int(E),
        C.c_int(M), _p(out, C.c_float))
    if rc < 0:
        raise ValueError(f"co3o_aggregate_gain: {rc}")
    return out


def philox4x32_10(counter, key):
    """Philox4x32-10 of Salmon et al. (SC'11): four 32-bit counter words, two key words -> four words."""
    c = (C.c_uint32 * 4)(*[int(x) & 0xffffffff for x in counter])
    k = (C.c_uint32 * 2)(*[int(x) & 0xffffffff for x in key])
    o = (C.c_uint32 * 4)()
    lib().co3o_philox4x32_10(c, k, o)
    return [int(x) for x in o]


def ef_step_sr(g, m, gamma, E, M, bias, user, elem0, seed, want_q=True):
    """Algorithm 1 lines 8 and 10 with the stochastic fp conversion (Sec. II-B (ii)); see the C file for the
    reading.  Returns (m_new, sym, q, counters[2])."""
    g = np.ascontiguousarray(g, dtype=np.float32)
    m = np.ascontiguousarray(m, dtype=np.float32)
    n = g.size
    m_out = np.empty(n, dtype=np.float32)
    wide = is_wide(E, M)
    sym = np.empty(n, dtype=np.uint16 if wide else np.uint8)
    q = np.empty(n, dtype=np.float32) if want_q else None
    cnt = np.zeros(2, dtype=np.uint64)
    rc = (lib().co3o_ef_step_sr_w if wide else lib().co3o_ef_step_sr)(
        _p(g, C.c_float), _p(m, C.c_float), C.c_uint64(n), C.c_float(float(np.float32(gamma))),
        C.c_int(E), C.c_int(M), C.c_int(int(bias)), C.c_uint32(int(user)), C.c_uint64(int(elem0)),
        C.c_uint64(int(seed)), _p(m_out, C.c_float), sym.ctypes.data_as(C.c_void_p),
        _p(q, C.c_float) if want_q else None, _p(cnt, C.c_uint64))
    if rc != 0:
        raise ValueError(f"co3o_ef_step_sr: {rc}")
    return m_out, sym, q, cnt


def histogram(sym, A, hist=None):
    wide = A > 256
    sym = np.ascontiguousarray(sym, dtype=np.uint16 if wide else np.uint8)
    if hist is None:
        hist = np.zeros(A, dtype=np.uint64)
    assert int(sym.max(initial=0)) < hist.size
    if wide:
        lib().co3o_histogram_w(_p(sym, C.c_uint16), C.c_uint64(sym.size), _p(hist, C.c_uint64))
    else:
        lib().co3o_histogram(_p(sym, C.c_uint8), C.c_uint64(sym.size), _p(hist, C.c_uint64))
    return hist


def huffman_lengths(w):
    """Huffman code lengths for integer weights (Sec. IV-A (ii); reading R6)."""
    w = np.ascontiguousarray(w, dtype=np.uint64)
    length = np.zeros(w.size, dtype=np.uint8)
    rc = lib().co3o_huffman_lengths(_p(w, C.c_uint64), C.c_int(w.size), _p(length, C.c_uint8))
    if rc < 0:
        raise ValueError(f"co3o_huffman_lengths: {rc}")
    return length


def canonical_codes(length):
    length = np.ascontiguousarray(length, dtype=np.uint8)
    code = np.zeros(length.size, dtype=np.uint64)
    lib().co3o_canonical_codes(_p(length, C.c_uint8), C.c_int(length.size), _p(code, C.c_uint64))
    return code


def codebook(w):
    length = huffman_lengths(w)
    return length, canonical_codes(length)


def num_chunks(seg_len):
    seg_len = np.ascontiguousarray(seg_len, dtype=np.uint64)
    return int(lib().co3o_num_chunks(C.c_int(seg_len.size), _p(seg_len, C.c_uint64)))


def pack(sym, seg_len, seg_book, lens, codes, cap_words=None):
    """h_Hf of Sec. IV-A (ii) for one user: returns dict(words, chunk_offset, sub_bits,
    payload_bits, rc)."""
    wide = lens.shape[-1] > 256
    sym = np.ascontiguousarray(sym, dtype=np.uint16 if wide else np.uint8)
    seg_len = np.ascontiguousarray(seg_len, dtype=np.uint64)
    seg_book = np.ascontiguousarray(seg_book, dtype=np.int32)
    lens = np.ascontiguousarray(lens, dtype=np.uint8).reshape(-1, lens.shape[-1])
    codes = np.ascontiguousarray(codes, dtype=np.uint64).reshape(-1, codes.shape[-1])
    A = lens.shape[1]
    assert int(seg_len.sum()) == sym.size
    nch = num_chunks(seg_len)
    if cap_words is None:
        cap_words = (sym.size * max(1, int(lens.max(initial=1))) + 31) // 32 + nch + 1
    words = np.zeros(cap_words, dtype=np.uint32)
    chunk_offset = np.zeros(nch + 1, dtype=np.uint64)
    sub_bits = np.zeros(nch * SUBS_PER_CHUNK, dtype=np.uint16)
    payload = C.c_uint64(0)
    rc = (lib().co3o_pack_w if wide else lib().co3o_pack)(sym.ctypes.data_as(C.c_void_p), C.c_int(seg_len.size), _p(seg_len, C.c_uint64),
                         _p(seg_book, C.c_int32), _p(lens, C.c_uint8), _p(codes, C.c_uint64),
                         C.c_int(A), _p(words, C.c_uint32), C.c_uint64(cap_words),
                         _p(chunk_offset, C.c_uint64), _p(sub_bits, C.c_uint16), C.byref(payload))
    return dict(words=words, chunk_offset=chunk_offset, sub_bits=sub_bits,
                payload_bits=int(payload.value), rc=int(rc))


def unpack(words, d, seg_len, seg_book, lens, codes, chunk_offset, sub_bits):
    """Inverse of pack (h is invertible, Sec. II-B (iii)).  Returns (rc, sym)."""
    words = np.ascontiguousarray(words, dtype=np.uint32)
    seg_len = np.ascontiguousarray(seg_len, dtype=np.uint64)
    seg_book = np.ascontiguousarray(seg_book, dtype=np.int32)
    lens = np.ascontiguousarray(lens, dtype=np.uint8).reshape(-1, lens.shape[-1])
    codes = np.ascontiguousarray(codes, dtype=np.uint64).reshape(-1, codes.shape[-1])
    chunk_offset = np.ascontiguousarray(chunk_offset, dtype=np.uint64)
    sub_bits = np.ascontiguousarray(sub_bits, dtype=np.uint16)
    wide = lens.shape[1] > 256
    sym = np.zeros(d, dtype=np.uint16 if wide else np.uint8)
    rc = (lib().co3o_unpack_w if wide else lib().co3o_unpack)(
        _p(words, C.c_uint32), C.c_uint64(words.size), C.c_int(seg_len.size),
        _p(seg_len, C.c_uint64), _p(seg_book, C.c_int32), _p(lens, C.c_uint8),
        _p(codes, C.c_uint64), C.c_int(lens.shape[1]),
        _p(chunk_offset, C.c_uint64), _p(sub_bits, C.c_uint16), sym.ctypes.data_as(C.c_void_p))
    return int(rc), sym


def aggregate(sym, seg_len, bias, E, M):
    """(1/U) sum_u ghat^(u), eq. (aggregate hat); sym is [U, d], bias is [U, nseg]."""
    wide = is_wide(E, M)
    sym = np.ascontiguousarray(sym, dtype=np.uint16 if wide else np.uint8)
    U, d = sym.shape
    seg_len = np.ascontiguousarray(seg_len, dtype=np.uint64)
    bias = np.ascontiguousarray(bias, dtype=np.int32).reshape(U, seg_len.size)
    out = np.empty(d, dtype=np.float32)
    rc = (lib().co3o_aggregate_w if wide else lib().co3o_aggregate)(
        sym.ctypes.data_as(C.c_void_p), C.c_uint32(U), C.c_uint64(d), C.c_int(seg_len.size),
        _p(seg_len, C.c_uint64), _p(bias, C.c_int32), C.c_int(E), C.c_int(M), _p(out, C.c_float))
    if rc < 0:
        raise ValueError(f"co3o_aggregate: {rc}")
    return out


def model_update(sym, seg_len, bias, E, M, eta, w):
    """PS model update of eq. (aggregate hat), Algorithm 1 line 14: w - (eta / U) sum_u ghat^(u), the sum
    and products in fp64, one rounding to fp32.  sym [U][d] uint8 (uint16 for alphabets of more than 8 bits),
    bias [U][nseg], w float32 [d]."""
    wide = is_wide(E, M)
    sym = np.ascontiguousarray(sym, dtype=np.uint16 if wide else np.uint8)
    U, d = sym.shape
    sl = np.ascontiguousarray(seg_len, dtype=np.uint64)
    b = np.ascontiguousarray(np.broadcast_to(np.asarray(bias, np.int32), (U, sl.size)), dtype=np.int32)
    w = np.ascontiguousarray(w, dtype=np.float32)
    out = np.empty(d, dtype=np.float32)
    rc = (lib().co3o_model_update_w if wide else lib().co3o_model_update)(
        sym.ctypes.data_as(C.c_void_p), C.c_uint32(U), C.c_uint64(d), C.c_int(sl.size), _p(sl, C.c_uint64),
        _p(b, C.c_int32), C.c_int(E), C.c_int(M), C.c_float(float(np.float32(eta))), _p(w, C.c_float), _p(out, C.c_float))
    if rc != 0:
        raise ValueError(f"co3o_model_update: {rc}")
    return out


def gennorm_cdf_pair(x, mu, alpha, beta):
    """(F(x), 1 - F(x)) of the GenNorm density of eq. (gennorm), each computed without
    cancellation: F(x) = 1/2 + 1/2 sgn(x - mu) P(1/beta, (|x - mu|/alpha)^beta) with P the
    regularised lower incomplete gamma function (the integral of the printed pdf)."""
    from scipy.special import gammainc, gammaincc
    x = np.asarray(x, dtype=np.float64)
    t = (np.abs(x - mu) / alpha) ** beta
    lower_half = 0.5 * gammaincc(1.0 / beta, t)      # mass beyond |x - mu| on one side
    inner = 0.5 * gammainc(1.0 / beta, t)
    right = x >= mu
    F = np.where(right, 0.5 + inner, lower_half)
    S = np.where(right, lower_half, 0.5 + inner)
    return F, S


def gennorm_weights(E, M, bias, mu, alpha, beta, scale_bits=40):
    """Integer Huffman weights of the quantized symbols when the corrected gradient is
    GenNorm(mu, alpha, beta) (Sec. IV-A (ii): the code is designed under the GenNorm
    assumption).  Cell of a representative = the inputs Q_fp maps to it: bounded by the
    midpoints to its neighbours, the outermost cells reaching to infinity.  Every symbol
    that Q_fp can produce gets weight max(1, floor(p * 2^scale_bits)); the others get 0."""
    mag = grid(E, M, bias)
    n = mag.size
    # signed representatives in ascending order: -mag[n-1] .. -mag[1], 0, mag[1] .. mag[n-1]
    vals = np.concatenate([-mag[:0:-1], mag])
    syms = np.concatenate([(1 << (E + M)) | np.arange(n - 1, 0, -1), np.arange(0, n)])
    mids = 0.5 * (vals[:-1] + vals[1:])
    F, S = gennorm_cdf_pair(mids, mu, alpha, beta)
    F_lo = np.concatenate([[0.0], F])       # F at the lower edge of each cell
    S_lo = np.concatenate([[1.0], S])
    F_hi = np.concatenate([F, [1.0]])
    S_hi = np.concatenate([S, [0.0]])
    # mass of a cell: use whichever tail keeps precision
    p = np.where(F_hi <= 0.5, F_hi - F_lo, np.where(S_lo <= 0.5, S_lo - S_hi, F_hi - F_lo))
    w = np.zeros(1 << (1 + E + M), dtype=np.uint64)
    wi = np.maximum(1, np.floor(p * float(1 << scale_bits))).astype(np.uint64)
    w[syms] = wi
    return w, p, syms
