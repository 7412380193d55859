"""ctypes front end of the CPU oracle (plc_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests, by the smoke check and by the
benchmark's CPU-baseline leg.  Nothing in the product package may import it.
All of the method's arithmetic lives in the C file; this module only marshals numpy arrays
(its one sum, coded_bits, is storage accounting: it adds up the sizes of the coded artefacts).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "plc_oracle.c")
_HDR = os.path.join(_HERE, "plc_oracle.h")
_LIB = os.path.join(_HERE, "libplc_oracle.so")

OK, ERR_INVALID, ERR_CAPACITY, ERR_CORRUPT = 0, 1, 2, 3
F64, F32 = 0, 1
ESCAPE = 255


class OracleError(RuntimeError):
    def __init__(self, code, where):
        super().__init__(f"oracle {where} failed with code {code}")
        self.code = code


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain C11, no fused multiply-add contraction)."""
    stale = (not os.path.exists(_LIB)
             or os.path.getmtime(_LIB) < max(os.path.getmtime(_SRC), os.path.getmtime(_HDR)))
    if force or stale:
        tmp = f"{_LIB}.{os.getpid()}.tmp"
        subprocess.check_call(["gcc", "-std=c11", "-O2", "-ffp-contract=off", "-fPIC", "-shared",
                               "-Wall", "-Wextra", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


class Dims(C.Structure):
    _fields_ = [("S", C.c_int32), ("L", C.c_int32), ("H", C.c_int32), ("n", C.c_int32),
                ("k", C.c_int32), ("d", C.c_int32),
                ("cand_stride", C.c_int64 * 5), ("act_stride", C.c_int64 * 4),
                ("delta", C.c_float), ("qmax", C.c_int32)]


def make_dims(S, L, H, n, k, d, delta, qmax=127, cand_stride=None, act_stride=None) -> Dims:
    """Dims for contiguous [S,L,H,n,k,d] candidates and [S,L,H,n,d] vectors unless strides are given."""
    if cand_stride is None:
        cand_stride = (L * H * n * k * d, H * n * k * d, n * k * d, k * d, d)
    if act_stride is None:
        act_stride = (L * H * n * d, H * n * d, n * d, d)
    dm = Dims()
    dm.S, dm.L, dm.H, dm.n, dm.k, dm.d = S, L, H, n, k, d
    dm.cand_stride = (C.c_int64 * 5)(*cand_stride)
    dm.act_stride = (C.c_int64 * 4)(*act_stride)
    dm.delta = float(np.float32(delta))
    dm.qmax = qmax
    return dm


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_LIB)
        p = C.c_void_p
        L.plco_half_to_double.restype = C.c_double
        L.plco_half_to_double.argtypes = [C.c_uint16]
        L.plco_double_to_half.restype = C.c_uint16
        L.plco_double_to_half.argtypes = [C.c_double]
        L.plco_weights.argtypes = [p, C.c_int, C.c_int, p]
        L.plco_predict_residual.argtypes = [C.POINTER(Dims), C.c_int, p, p, p, p, p, p, p,
                                            C.c_uint64, p, p, p, p]
        L.plco_histogram.argtypes = [p, C.c_int64, C.c_int64, p]
        L.plco_build_freq.argtypes = [p, C.c_int64, p, p]
        L.plco_units_per_stream.restype = C.c_int64
        L.plco_units_per_stream.argtypes = [C.c_int64, C.c_int32]
        L.plco_rans_encode.argtypes = [p, C.c_int64, C.c_int64, C.c_int32, p, p, p, p,
                                       C.c_uint64, p]
        L.plco_rans_decode.argtypes = [p, p, p, p, p, C.c_int64, C.c_int64, C.c_int32, p]
        L.plco_reconstruct.argtypes = [C.POINTER(Dims), C.c_int, p, p, p, p, p, p, p, p, p]
        L.plco_predict_residual_cond.argtypes = [C.POINTER(Dims), C.c_int, p, p, p, p, p, p, p, p,
                                                 C.c_uint64, p, p, p, p]
        L.plco_reconstruct_cond.argtypes = [C.POINTER(Dims), C.c_int, p, p, p, p, p, p, p, p, p, p]
        L.plco_select_candidate.argtypes = [C.POINTER(Dims), C.c_int, p, p, C.c_float, p]
        L.plco_index_table.argtypes = [p, C.c_int, p]
        L.plco_index_encode.argtypes = [p, p, C.c_int32, C.c_int32, C.c_int32, p, p, p, C.c_uint64, p]
        L.plco_index_decode.argtypes = [p, p, p, p, p, C.c_int32, C.c_int32, C.c_int32, p]
        L.plco_predict_residual_adapt.argtypes = [C.POINTER(Dims), C.c_int, p, p, p, p, p, C.c_float, p, p, p, p,
                                                  C.c_uint64, p, p, p, p]
        L.plco_reconstruct_adapt.argtypes = [C.POINTER(Dims), C.c_int, p, p, p, p, p, C.c_float, p, p, p, p, p, p]
        L.plco_surprisal_thresholds.argtypes = [C.c_double, C.c_double, C.c_int32, p]
        L.plco_surprisal_bits.argtypes = [p, p, C.c_int32, C.c_int32, C.c_int32, p, C.c_int32, p]
        L.plco_histogram_bucketed.argtypes = [p, C.c_int64, C.c_int64, C.c_int32, C.c_int32, p, C.c_int32, p]
        L.plco_build_freq_sparse.argtypes = [p, C.c_int64, p]
        L.plco_rans_encode_bucketed.argtypes = [p, C.c_int64, C.c_int64, C.c_int32, C.c_int32, C.c_int32, p,
                                                C.c_int32, p, p, p, p, C.c_uint64, p]
        L.plco_rans_decode_bucketed.argtypes = [p, p, p, p, p, C.c_int64, C.c_int64, C.c_int32, C.c_int32,
                                                C.c_int32, p, C.c_int32, p]
        _lib = L
    return _lib


def _ptr(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _u16(a):
    """View an fp16 / u16 array as its bit patterns without copying more than needed."""
    a = np.asarray(a)
    if a.dtype == np.float16:
        a = a.view(np.uint16)
    assert a.dtype == np.uint16, a.dtype
    return a


def _check(rc, where):
    if rc != OK:
        raise OracleError(rc, where)


def half_to_double(bits: int) -> float:
    return lib().plco_half_to_double(int(bits))


def double_to_half(x: float) -> int:
    return lib().plco_double_to_half(float(x))


def weights(p, mode=F64):
    p = np.ascontiguousarray(p, dtype=np.float32)
    w = np.empty(p.shape[0], dtype=np.float64)
    _check(lib().plco_weights(_ptr(p), p.shape[0], mode, _ptr(w)), "weights")
    return w


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def predict_residual(dm: Dims, cand_k, cand_v, probs, act_k, act_v, mode=F64,
                     want_pred=False, want_u=False, esc_cap=None, chosen=None, bits=None, step_range=None):
    """Returns dict(symbols [streams, N] u8, esc_vals u16, esc_cnt u32, esc_off u64, pred, u).

    cand_* / act_* are numpy arrays holding the tensors' storage (fp16 or u16);
    elements are addressed through dm's strides, so any layout works.
    chosen (i32 [S,n], optional) selects the token-conditional variant; bits (u8 [S,n]) with
    step_range (fp32) on top of it the surprisal-adaptive quantiser.
    """
    ck, cv, ak, av = _u16(cand_k), _u16(cand_v), _u16(act_k), _u16(act_v)
    probs = np.ascontiguousarray(probs, dtype=np.float32)
    n_streams = dm.S * dm.L * dm.H
    N = 2 * dm.n * dm.d
    E = n_streams * N
    if esc_cap is None:
        esc_cap = E
    symbols = np.empty((n_streams, N), dtype=np.uint8)
    esc_vals = np.zeros(max(int(esc_cap), 1), dtype=np.uint16)
    esc_cnt = np.zeros(n_streams, dtype=np.uint32)
    esc_off = np.zeros(n_streams, dtype=np.uint64)
    pred = np.empty((n_streams, N), dtype=np.float64) if want_pred else None
    u = np.empty((n_streams, N), dtype=np.float64) if want_u else None
    if chosen is None:
        rc = lib().plco_predict_residual(C.byref(dm), mode, _ptr(ck), _ptr(cv), _ptr(probs),
                                         _ptr(ak), _ptr(av), _ptr(symbols), _ptr(esc_vals),
                                         int(esc_cap), _ptr(esc_cnt), _ptr(esc_off), _ptr(pred), _ptr(u))
    elif bits is None:
        ch = _i32(chosen)
        assert ch.size == dm.S * dm.n
        rc = lib().plco_predict_residual_cond(C.byref(dm), mode, _ptr(ck), _ptr(cv), _ptr(probs), _ptr(ch),
                                              _ptr(ak), _ptr(av), _ptr(symbols), _ptr(esc_vals),
                                              int(esc_cap), _ptr(esc_cnt), _ptr(esc_off), _ptr(pred), _ptr(u))
    else:
        ch = _i32(chosen)
        bt = np.ascontiguousarray(bits, dtype=np.uint8)
        assert ch.size == dm.S * dm.n and bt.size == dm.S * dm.n
        rc = lib().plco_predict_residual_adapt(C.byref(dm), mode, _ptr(ck), _ptr(cv), _ptr(probs), _ptr(ch),
                                               _ptr(bt), float(np.float32(step_range)), _ptr(ak), _ptr(av),
                                               _ptr(symbols), _ptr(esc_vals), int(esc_cap), _ptr(esc_cnt),
                                               _ptr(esc_off), _ptr(pred), _ptr(u))
    _check(rc, "predict_residual")
    total = int(esc_cnt.sum())
    return dict(symbols=symbols, esc_vals=esc_vals[:total].copy(), esc_cnt=esc_cnt,
                esc_off=esc_off, pred=pred, u=u)


def histogram(symbols):
    symbols = np.ascontiguousarray(symbols, dtype=np.uint8)
    n_streams, N = symbols.shape
    counts = np.empty((n_streams, 256), dtype=np.uint32)
    _check(lib().plco_histogram(_ptr(symbols), n_streams, N, _ptr(counts)), "histogram")
    return counts


def build_freq(counts):
    counts = np.ascontiguousarray(counts, dtype=np.uint32)
    n_streams = counts.shape[0]
    freq = np.empty((n_streams, 256), dtype=np.uint16)
    cum = np.empty((n_streams, 257), dtype=np.uint16)
    _check(lib().plco_build_freq(_ptr(counts), n_streams, _ptr(freq), _ptr(cum)), "build_freq")
    return freq, cum


def units_per_stream(N, chunk_syms):
    return int(lib().plco_units_per_stream(int(N), int(chunk_syms)))


def rans_encode(symbols, freq, chunk_syms=0, word_cap_per_unit=None):
    """Returns dict(states [units,32] u32, words u16 flat, word_off u64 [units], n_words u32 [units])."""
    symbols = np.ascontiguousarray(symbols, dtype=np.uint8)
    freq = np.ascontiguousarray(freq, dtype=np.uint16)
    n_streams, N = symbols.shape
    U = units_per_stream(N, chunk_syms)
    unit_syms = chunk_syms if chunk_syms > 0 else N
    if word_cap_per_unit is None:
        word_cap_per_unit = unit_syms  # at most one word per symbol
    n_units = n_streams * U
    states = np.empty((n_units, 32), dtype=np.uint32)
    words = np.zeros(max(n_units * word_cap_per_unit, 1), dtype=np.uint16)
    word_off = (np.arange(n_units, dtype=np.uint64) * np.uint64(word_cap_per_unit))
    n_words = np.zeros(n_units, dtype=np.uint32)
    rc = lib().plco_rans_encode(_ptr(symbols), n_streams, N, chunk_syms, _ptr(freq), _ptr(states),
                                _ptr(words), _ptr(word_off), int(word_cap_per_unit), _ptr(n_words))
    _check(rc, "rans_encode")
    return dict(states=states, words=words, word_off=word_off, n_words=n_words)


def rans_decode(freq, states, words, word_off, n_words, n_streams, N, chunk_syms=0):
    freq = np.ascontiguousarray(freq, dtype=np.uint16)
    states = np.ascontiguousarray(states, dtype=np.uint32)
    words = np.ascontiguousarray(words, dtype=np.uint16)
    word_off = np.ascontiguousarray(word_off, dtype=np.uint64)
    n_words = np.ascontiguousarray(n_words, dtype=np.uint32)
    symbols = np.empty((n_streams, N), dtype=np.uint8)
    rc = lib().plco_rans_decode(_ptr(freq), _ptr(states), _ptr(words), _ptr(word_off), _ptr(n_words),
                                n_streams, N, chunk_syms, _ptr(symbols))
    _check(rc, "rans_decode")
    return symbols


def reconstruct(dm: Dims, cand_k, cand_v, probs, symbols, esc_vals, esc_off, mode=F64,
                want_pre_round=False, out_elems=None, chosen=None, bits=None, step_range=None):
    """Returns (out_k, out_v) as u16 bit-pattern arrays addressed through dm.act_stride."""
    ck, cv = _u16(cand_k), _u16(cand_v)
    probs = np.ascontiguousarray(probs, dtype=np.float32)
    symbols = np.ascontiguousarray(symbols, dtype=np.uint8)
    esc_vals = np.ascontiguousarray(esc_vals, dtype=np.uint16)
    if esc_vals.size == 0:
        esc_vals = np.zeros(1, dtype=np.uint16)
    esc_off = np.ascontiguousarray(esc_off, dtype=np.uint64)
    if out_elems is None:
        out_elems = dm.S * dm.L * dm.H * dm.n * dm.d
    out_k = np.zeros(out_elems, dtype=np.uint16)
    out_v = np.zeros(out_elems, dtype=np.uint16)
    pre = np.empty(symbols.size, dtype=np.float64) if want_pre_round else None
    if chosen is None:
        rc = lib().plco_reconstruct(C.byref(dm), mode, _ptr(ck), _ptr(cv), _ptr(probs), _ptr(symbols),
                                    _ptr(esc_vals), _ptr(esc_off), _ptr(out_k), _ptr(out_v), _ptr(pre))
    elif bits is None:
        ch = _i32(chosen)
        assert ch.size == dm.S * dm.n
        rc = lib().plco_reconstruct_cond(C.byref(dm), mode, _ptr(ck), _ptr(cv), _ptr(probs), _ptr(ch),
                                         _ptr(symbols), _ptr(esc_vals), _ptr(esc_off), _ptr(out_k),
                                         _ptr(out_v), _ptr(pre))
    else:
        ch = _i32(chosen)
        bt = np.ascontiguousarray(bits, dtype=np.uint8)
        assert ch.size == dm.S * dm.n and bt.size == dm.S * dm.n
        rc = lib().plco_reconstruct_adapt(C.byref(dm), mode, _ptr(ck), _ptr(cv), _ptr(probs), _ptr(ch), _ptr(bt),
                                          float(np.float32(step_range)), _ptr(symbols), _ptr(esc_vals),
                                          _ptr(esc_off), _ptr(out_k), _ptr(out_v), _ptr(pre))
    _check(rc, "reconstruct")
    if want_pre_round:
        return out_k, out_v, pre.reshape(symbols.shape)
    return out_k, out_v


def select_candidate(dm: Dims, cand_k, act_k, max_mean_sq, mode=F64):
    """chosen i32 [S, n]: nearest candidate by the layer-0 / head-0 key row, -1 beyond the limit."""
    ck, ak = _u16(cand_k), _u16(act_k)
    chosen = np.empty((dm.S, dm.n), dtype=np.int32)
    _check(lib().plco_select_candidate(C.byref(dm), mode, _ptr(ck), _ptr(ak), float(max_mean_sq),
                                       _ptr(chosen)), "select_candidate")
    return chosen


def index_table(p):
    """Frequencies u16 [k+1] of one position's index symbols (last = not among the candidates)."""
    p = np.ascontiguousarray(p, dtype=np.float32)
    f = np.empty(p.shape[0] + 1, dtype=np.uint16)
    _check(lib().plco_index_table(_ptr(p), p.shape[0], _ptr(f)), "index_table")
    return f


def index_encode(probs, chosen, word_cap=None):
    """probs fp32 [S,n,k], chosen i32 [S,n] -> dict(states [S,32], words, word_off [S], n_words [S])."""
    probs = np.ascontiguousarray(probs, dtype=np.float32)
    S, n, k = probs.shape
    ch = _i32(chosen)
    assert ch.shape == (S, n)
    if word_cap is None:
        word_cap = n
    states = np.empty((S, 32), dtype=np.uint32)
    words = np.zeros(max(S * word_cap, 1), dtype=np.uint16)
    word_off = np.arange(S, dtype=np.uint64) * np.uint64(word_cap)
    n_words = np.zeros(S, dtype=np.uint32)
    _check(lib().plco_index_encode(_ptr(probs), _ptr(ch), S, n, k, _ptr(states), _ptr(words),
                                   _ptr(word_off), int(word_cap), _ptr(n_words)), "index_encode")
    return dict(states=states, words=words, word_off=word_off, n_words=n_words)


def index_decode(probs, states, words, word_off, n_words):
    probs = np.ascontiguousarray(probs, dtype=np.float32)
    S, n, k = probs.shape
    states = np.ascontiguousarray(states, dtype=np.uint32)
    words = np.ascontiguousarray(words, dtype=np.uint16)
    word_off = np.ascontiguousarray(word_off, dtype=np.uint64)
    n_words = np.ascontiguousarray(n_words, dtype=np.uint32)
    chosen = np.empty((S, n), dtype=np.int32)
    _check(lib().plco_index_decode(_ptr(probs), _ptr(states), _ptr(words), _ptr(word_off), _ptr(n_words),
                                   S, n, k, _ptr(chosen)), "index_decode")
    return chosen


MAX_BITS = 4          # default number of depths, the one the GPU library supports
MAX_BITS_ORACLE = 16  # what the oracle's own per-depth arrays hold (the definition has no limit)


def surprisal_thresholds(b0, hbar, bmax=MAX_BITS):
    """thr[m] = floor(4096 * 2^(-m * hbar / b0)) for m = 2..bmax (entries 0 and 1 unused)."""
    thr = np.zeros(bmax + 1, dtype=np.uint16)
    _check(lib().plco_surprisal_thresholds(C.c_double(float(b0)), C.c_double(float(hbar)), int(bmax), _ptr(thr)),
           "surprisal_thresholds")
    return thr


def surprisal_bits(probs, chosen, thr):
    probs = np.ascontiguousarray(probs, dtype=np.float32)
    S, n, k = probs.shape
    ch = _i32(chosen)
    thr = np.ascontiguousarray(thr, dtype=np.uint16)
    bits = np.empty((S, n), dtype=np.uint8)
    _check(lib().plco_surprisal_bits(_ptr(probs), _ptr(ch), S, n, k, _ptr(thr), thr.size - 1, _ptr(bits)),
           "surprisal_bits")
    return bits


def histogram_bucketed(symbols, syms_per_pos, streams_per_session, bits, n_tables=MAX_BITS):
    symbols = np.ascontiguousarray(symbols, dtype=np.uint8)
    bits = np.ascontiguousarray(bits, dtype=np.uint8)
    n_streams, N = symbols.shape
    counts = np.empty((n_streams, n_tables, 256), dtype=np.uint32)
    _check(lib().plco_histogram_bucketed(_ptr(symbols), n_streams, N, syms_per_pos, streams_per_session,
                                         _ptr(bits), n_tables, _ptr(counts)), "histogram_bucketed")
    return counts


def build_freq_sparse(counts):
    counts = np.ascontiguousarray(counts, dtype=np.uint32)
    freq = np.empty(counts.shape, dtype=np.uint16)
    _check(lib().plco_build_freq_sparse(_ptr(counts), counts.size // 256, _ptr(freq)), "build_freq_sparse")
    return freq


def rans_encode_bucketed(symbols, freq, syms_per_pos, streams_per_session, bits, chunk_syms=0,
                         word_cap_per_unit=None):
    symbols = np.ascontiguousarray(symbols, dtype=np.uint8)
    freq = np.ascontiguousarray(freq, dtype=np.uint16)
    bits = np.ascontiguousarray(bits, dtype=np.uint8)
    n_streams, N = symbols.shape
    n_tables = freq.shape[1]
    U = units_per_stream(N, chunk_syms)
    unit_syms = chunk_syms if chunk_syms > 0 else N
    if word_cap_per_unit is None:
        word_cap_per_unit = unit_syms
    n_units = n_streams * U
    states = np.empty((n_units, 32), dtype=np.uint32)
    words = np.zeros(max(n_units * word_cap_per_unit, 1), dtype=np.uint16)
    word_off = np.arange(n_units, dtype=np.uint64) * np.uint64(word_cap_per_unit)
    n_words = np.zeros(n_units, dtype=np.uint32)
    rc = lib().plco_rans_encode_bucketed(_ptr(symbols), n_streams, N, chunk_syms, syms_per_pos,
                                         streams_per_session, _ptr(bits), n_tables, _ptr(freq), _ptr(states),
                                         _ptr(words), _ptr(word_off), int(word_cap_per_unit), _ptr(n_words))
    _check(rc, "rans_encode_bucketed")
    return dict(states=states, words=words, word_off=word_off, n_words=n_words)


def rans_decode_bucketed(freq, states, words, word_off, n_words, n_streams, N, syms_per_pos,
                         streams_per_session, bits, chunk_syms=0):
    freq = np.ascontiguousarray(freq, dtype=np.uint16)
    states = np.ascontiguousarray(states, dtype=np.uint32)
    words = np.ascontiguousarray(words, dtype=np.uint16)
    word_off = np.ascontiguousarray(word_off, dtype=np.uint64)
    n_words = np.ascontiguousarray(n_words, dtype=np.uint32)
    bits = np.ascontiguousarray(bits, dtype=np.uint8)
    symbols = np.empty((n_streams, N), dtype=np.uint8)
    rc = lib().plco_rans_decode_bucketed(_ptr(freq), _ptr(states), _ptr(words), _ptr(word_off), _ptr(n_words),
                                         n_streams, N, chunk_syms, syms_per_pos, streams_per_session,
                                         _ptr(bits), freq.shape[1], _ptr(symbols))
    _check(rc, "rans_decode_bucketed")
    return symbols


def coded_bits(n_words, esc_cnt, n_streams):
    """Storage of the coded cache in bits: (total, payload).

    Per stream: 16 bits per rANS word, 32 lane states of 32 bits per unit,
    16 bits per escape, a 256 x 16-bit table, and three 32-bit counts.
    """
    n_words = np.asarray(n_words, dtype=np.int64)
    esc = int(np.asarray(esc_cnt, dtype=np.int64).sum())
    payload = 16 * int(n_words.sum()) + 16 * esc
    total = payload + 32 * 32 * n_words.size + (256 * 16 + 3 * 32) * n_streams
    return total, payload
