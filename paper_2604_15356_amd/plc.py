"""Thin ctypes binding over libplc.so: argument marshalling only.

Every function takes torch tensors that already live on the GPU, passes their
device pointers and the current HIP stream to the C entry point of the same
name (see include/plc.h), and returns.  No step of the coding path runs in
Python or in torch; torch only owns the memory and the stream.  If the library
has not been built, loading fails with an error -- there is no fallback.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libplc.so")

PLC_OK, PLC_ERR_INVALID, PLC_ERR_CAPACITY, PLC_ERR_CORRUPT, PLC_ERR_HIP, PLC_ERR_SCRATCH = 0, 1, 2, 3, 4, 5
STATIC_SCRATCH_BYTES = 48 << 20
PLC_ESCAPE = 255

EXPORTS = ("plc_version", "plc_strerror", "plc_workspace_bytes", "plc_units_per_stream",
           "plc_predict_residual", "plc_predict_residual_hist", "plc_predict_residual_noalloc", "plc_histogram", "plc_build_freq", "plc_rans_encode",
           "plc_rans_decode", "plc_reconstruct", "plc_rans_decode_reconstruct", "plc_rans_decode_reconstruct_cond",
           "plc_rans_decode_reconstruct_adapt",
           "plc_trace_kernel_events",
           "plc_predict_residual_cond", "plc_reconstruct_cond", "plc_select_candidate",
           "plc_index_encode", "plc_index_decode",
           "plc_surprisal_thresholds", "plc_surprisal_bits", "plc_predict_residual_adapt", "plc_reconstruct_adapt",
           "plc_histogram_bucketed", "plc_build_freq_bucketed", "plc_rans_encode_bucketed",
           "plc_rans_decode_bucketed",
           "plc_expected_embedding", "plc_predict_residual_linear", "plc_reconstruct_linear",
           "plc_trie_create", "plc_trie_destroy", "plc_trie_size", "plc_trie_nodes", "plc_trie_insert",
           "plc_trie_best_match", "plc_trie_evict")

MAX_BITS = 4

(TRACE_PREDICT, TRACE_RECONSTRUCT, TRACE_HISTOGRAM, TRACE_RANS_ENCODE, TRACE_RANS_DECODE,
 TRACE_PREDICT_COND, TRACE_RECONSTRUCT_COND, TRACE_EXPECTED_EMBEDDING, TRACE_PREDICT_LINEAR,
 TRACE_RECONSTRUCT_LINEAR) = range(10)


class PlcError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {strerror(code)} (code {code})")


class plc_dims(C.Structure):
    _fields_ = [("S", C.c_int32), ("L", C.c_int32), ("H", C.c_int32), ("n", C.c_int32),
                ("k", C.c_int32), ("d", C.c_int32),
                ("cand_stride", C.c_int64 * 5), ("act_stride", C.c_int64 * 4),
                ("delta", C.c_float), ("qmax", C.c_int32)]


_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it first "
                               "(python -m paper_2604_15356_amd.build); there is no fallback path")
        L = C.CDLL(LIB_PATH)
        p, u64, i64, i32, sz = C.c_void_p, C.c_uint64, C.c_int64, C.c_int32, C.c_size_t
        dp = C.POINTER(plc_dims)
        L.plc_version.restype = C.c_int
        L.plc_strerror.restype = C.c_char_p
        L.plc_strerror.argtypes = [C.c_int]
        L.plc_workspace_bytes.restype = sz
        L.plc_workspace_bytes.argtypes = [dp]
        L.plc_units_per_stream.restype = i64
        L.plc_units_per_stream.argtypes = [i64, i32]
        L.plc_predict_residual.argtypes = [dp, p, p, p, p, p, p, p, u64, p, p, p, p, sz, p, p]
        L.plc_predict_residual_hist.argtypes = [dp, p, p, p, p, p, p, p, u64, p, p, p, p, p, sz, p, p]
        L.plc_predict_residual_noalloc.argtypes = [dp, p, p, p, p, p, p, p, u64, p, p, p, p, p]
        L.plc_histogram.argtypes = [p, i64, i64, p, p]
        L.plc_build_freq.argtypes = [p, i64, p, p, p, p]
        L.plc_rans_encode.argtypes = [p, i64, i64, i32, p, p, p, p, u64, p, p, p]
        L.plc_rans_decode.argtypes = [p, p, p, u64, p, p, i64, i64, i32, p, p, p]
        L.plc_reconstruct.argtypes = [dp, p, p, p, p, p, u64, p, p, p, p, sz, p, p]
        L.plc_rans_decode_reconstruct.argtypes = [dp, p, p, p, u64, p, p, i32, p, p, p, p, u64, p, p, p, p, p, sz,
                                                  p, p]
        L.plc_rans_decode_reconstruct_cond.argtypes = [dp, p, p, p, u64, p, p, i32, p, p, p, p, p, u64, p, p, p, p, p,
                                                       sz, p, p]
        L.plc_rans_decode_reconstruct_adapt.argtypes = [dp, p, p, p, u64, p, p, i32, i32, p, p, p, p, p, C.c_float, p,
                                                        u64, p, p, p, p, p, sz, p, p]
        L.plc_trace_kernel_events.argtypes = [C.c_int, p, p]
        L.plc_predict_residual_cond.argtypes = [dp, p, p, p, p, p, p, p, p, u64, p, p, p, p, sz, p, p]
        L.plc_reconstruct_cond.argtypes = [dp, p, p, p, p, p, p, u64, p, p, p, p, sz, p, p]
        L.plc_select_candidate.argtypes = [dp, p, p, C.c_float, p, p]
        L.plc_index_encode.argtypes = [p, p, i32, i32, i32, p, p, p, u64, p, p, p]
        L.plc_index_decode.argtypes = [p, p, p, u64, p, p, i32, i32, i32, p, p, p]
        L.plc_surprisal_thresholds.argtypes = [C.c_double, C.c_double, i32, C.POINTER(C.c_uint16)]
        L.plc_surprisal_bits.argtypes = [p, p, i32, i32, i32, C.POINTER(C.c_uint16), i32, p, p, p]
        L.plc_predict_residual_adapt.argtypes = [dp, p, p, p, p, p, C.c_float, p, p, p, p, u64, p, p, p, p, sz, p, p]
        L.plc_reconstruct_adapt.argtypes = [dp, p, p, p, p, p, C.c_float, p, p, u64, p, p, p, p, sz, p, p]
        L.plc_histogram_bucketed.argtypes = [p, i64, i64, i32, i32, p, i32, p, p, p]
        L.plc_build_freq_bucketed.argtypes = [p, i64, i32, p, p, p]
        L.plc_rans_encode_bucketed.argtypes = [p, i64, i64, i32, i32, i32, p, i32, p, p, p, p, u64, p, p, p]
        L.plc_rans_decode_bucketed.argtypes = [p, p, p, u64, p, p, i64, i64, i32, i32, i32, p, i32, p, p, p]
        L.plc_trie_create.restype = p
        L.plc_trie_create.argtypes = [C.c_double]
        L.plc_trie_destroy.restype = None
        L.plc_trie_destroy.argtypes = [p]
        L.plc_trie_size.restype = i64
        L.plc_trie_size.argtypes = [p]
        L.plc_trie_nodes.restype = i64
        L.plc_trie_nodes.argtypes = [p]
        L.plc_trie_insert.argtypes = [p, p, p, i64, i64, C.POINTER(i64)]
        L.plc_trie_best_match.argtypes = [p, p, i64, C.POINTER(i64), C.POINTER(i64), C.POINTER(C.c_double)]
        L.plc_trie_evict.argtypes = [p, i64]
        L.plc_expected_embedding.argtypes = [p, p, i64, i32, i32, p, p]
        L.plc_predict_residual_linear.argtypes = [dp, p, i32, p, p, p, p, p, p, p, u64, p, p, p, sz, p, p]
        L.plc_reconstruct_linear.argtypes = [dp, p, i32, p, p, p, p, p, u64, p, p, p, p, sz, p, p]
        _lib = L
    return _lib


def strerror(code: int) -> str:
    return lib().plc_strerror(int(code)).decode()


def plc_version() -> int:
    return int(lib().plc_version())


def make_dims(S, L, H, n, k, d, delta, qmax=127, cand_stride=None, act_stride=None) -> plc_dims:
    if cand_stride is None:
        cand_stride = (L * H * n * k * d, H * n * k * d, n * k * d, k * d, d)
    if act_stride is None:
        act_stride = (L * H * n * d, H * n * d, n * d, d)
    dm = plc_dims()
    dm.S, dm.L, dm.H, dm.n, dm.k, dm.d = S, L, H, n, k, d
    dm.cand_stride = (C.c_int64 * 5)(*[int(x) for x in cand_stride])
    dm.act_stride = (C.c_int64 * 4)(*[int(x) for x in act_stride])
    dm.delta = float(delta)
    dm.qmax = int(qmax)
    return dm


def plc_workspace_bytes(dims: plc_dims) -> int:
    return int(lib().plc_workspace_bytes(C.byref(dims)))


def plc_units_per_stream(syms_per_stream: int, chunk_syms: int) -> int:
    return int(lib().plc_units_per_stream(int(syms_per_stream), int(chunk_syms)))


def _ptr(t, dtype=None):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("plc takes device tensors")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"expected {dtype}, got {t.dtype}")
    return C.c_void_p(t.data_ptr())


def _contig(t, dtype):
    if t is None:
        return None
    if not t.is_contiguous():
        raise ValueError("tensor must be contiguous")
    return _ptr(t, dtype)


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(rc, where):
    if rc != PLC_OK:
        raise PlcError(rc, where)


def plc_predict_residual(dims, cand_k, cand_v, probs, act_k, act_v, symbols, esc_vals, esc_cnt,
                         esc_off, ws, status, pred_out=None):
    """cand_*/act_* fp16 (strides in dims); probs fp32 [S,n,k]; symbols u8 out; esc_vals int16/uint16
    out (its numel is the capacity); esc_cnt int32 out; esc_off int64 out; ws uint8; status int32[1]."""
    rc = lib().plc_predict_residual(
        C.byref(dims), _ptr(cand_k, torch.float16), _ptr(cand_v, torch.float16),
        _contig(probs, torch.float32), _ptr(act_k, torch.float16), _ptr(act_v, torch.float16),
        _contig(symbols, torch.uint8), _contig(esc_vals, None), esc_vals.numel(),
        _contig(esc_cnt, torch.int32), _contig(esc_off, torch.int64), _contig(pred_out, torch.float32),
        _contig(ws, torch.uint8), ws.numel(), _contig(status, torch.int32), _stream())
    _check(rc, "plc_predict_residual")


def plc_predict_residual_hist(dims, cand_k, cand_v, probs, act_k, act_v, symbols, esc_vals, esc_cnt,
                              esc_off, counts, ws, status, pred_out=None):
    """plc_predict_residual that also leaves the symbols' per-stream counts (int32 [streams, 256]) in `counts`."""
    rc = lib().plc_predict_residual_hist(
        C.byref(dims), _ptr(cand_k, torch.float16), _ptr(cand_v, torch.float16),
        _contig(probs, torch.float32), _ptr(act_k, torch.float16), _ptr(act_v, torch.float16),
        _contig(symbols, torch.uint8), _contig(esc_vals, None), esc_vals.numel(),
        _contig(esc_cnt, torch.int32), _contig(esc_off, torch.int64), _contig(pred_out, torch.float32),
        _contig(counts, torch.int32), _contig(ws, torch.uint8), ws.numel(), _contig(status, torch.int32), _stream())
    _check(rc, "plc_predict_residual_hist")


def plc_predict_residual_noalloc(dims, cand_k, cand_v, probs, act_k, act_v, symbols, esc_vals, esc_cnt,
                                 esc_off, status, pred_out=None):
    """plc_predict_residual with the library's own static workspace (no ws argument)."""
    rc = lib().plc_predict_residual_noalloc(
        C.byref(dims), _ptr(cand_k, torch.float16), _ptr(cand_v, torch.float16),
        _contig(probs, torch.float32), _ptr(act_k, torch.float16), _ptr(act_v, torch.float16),
        _contig(symbols, torch.uint8), _contig(esc_vals, None), esc_vals.numel(),
        _contig(esc_cnt, torch.int32), _contig(esc_off, torch.int64), _contig(pred_out, torch.float32),
        _contig(status, torch.int32), _stream())
    _check(rc, "plc_predict_residual_noalloc")


def plc_histogram(symbols, n_streams, syms_per_stream, counts):
    rc = lib().plc_histogram(_contig(symbols, torch.uint8), n_streams, syms_per_stream,
                             _contig(counts, torch.int32), _stream())
    _check(rc, "plc_histogram")


def plc_build_freq(counts, n_streams, freq, cum, status):
    rc = lib().plc_build_freq(_contig(counts, torch.int32), n_streams, _contig(freq, torch.int16),
                              _contig(cum, torch.int16), _contig(status, torch.int32), _stream())
    _check(rc, "plc_build_freq")


def plc_rans_encode(symbols, n_streams, syms_per_stream, chunk_syms, freq, states, words, word_off,
                    word_cap_per_unit, n_words, status):
    rc = lib().plc_rans_encode(_contig(symbols, torch.uint8), n_streams, syms_per_stream, chunk_syms,
                               _contig(freq, torch.int16), _contig(states, torch.int32),
                               _contig(words, torch.int16), _contig(word_off, torch.int64),
                               int(word_cap_per_unit), _contig(n_words, torch.int32),
                               _contig(status, torch.int32), _stream())
    _check(rc, "plc_rans_encode")


def plc_rans_decode(freq, states, words, word_off, n_words, n_streams, syms_per_stream, chunk_syms,
                    symbols, status):
    rc = lib().plc_rans_decode(_contig(freq, torch.int16), _contig(states, torch.int32),
                               _contig(words, torch.int16), words.numel(),
                               _contig(word_off, torch.int64), _contig(n_words, torch.int32),
                               n_streams, syms_per_stream, chunk_syms, _contig(symbols, torch.uint8),
                               _contig(status, torch.int32), _stream())
    _check(rc, "plc_rans_decode")


def plc_reconstruct(dims, cand_k, cand_v, probs, symbols, esc_vals, esc_off, out_k, out_v, ws, status):
    rc = lib().plc_reconstruct(
        C.byref(dims), _ptr(cand_k, torch.float16), _ptr(cand_v, torch.float16),
        _contig(probs, torch.float32), _contig(symbols, torch.uint8), _contig(esc_vals, None),
        esc_vals.numel(), _contig(esc_off, torch.int64), _ptr(out_k, torch.float16),
        _ptr(out_v, torch.float16), _contig(ws, torch.uint8), ws.numel(),
        _contig(status, torch.int32), _stream())
    _check(rc, "plc_reconstruct")


def plc_rans_decode_reconstruct(dims, freq, states, words, word_off, n_words, chunk_syms, cand_k, cand_v, probs,
                                esc_vals, esc_off, symbols, out_k, out_v, ws, status):
    rc = lib().plc_rans_decode_reconstruct(
        C.byref(dims), _contig(freq, torch.int16), _contig(states, torch.int32), _contig(words, torch.int16),
        words.numel(), _contig(word_off, torch.int64), _contig(n_words, torch.int32), chunk_syms,
        _ptr(cand_k, torch.float16), _ptr(cand_v, torch.float16), _contig(probs, torch.float32),
        _contig(esc_vals, None), esc_vals.numel(), _contig(esc_off, torch.int64), _contig(symbols, torch.uint8),
        _ptr(out_k, torch.float16), _ptr(out_v, torch.float16), _contig(ws, torch.uint8), ws.numel(),
        _contig(status, torch.int32), _stream())
    _check(rc, "plc_rans_decode_reconstruct")


def plc_rans_decode_reconstruct_cond(dims, freq, states, words, word_off, n_words, chunk_syms, cand_k, cand_v,
                                     probs, chosen, esc_vals, esc_off, symbols, out_k, out_v, ws, status):
    rc = lib().plc_rans_decode_reconstruct_cond(
        C.byref(dims), _contig(freq, torch.int16), _contig(states, torch.int32), _contig(words, torch.int16),
        words.numel(), _contig(word_off, torch.int64), _contig(n_words, torch.int32), chunk_syms,
        _ptr(cand_k, torch.float16), _ptr(cand_v, torch.float16), _contig(probs, torch.float32),
        _contig(chosen, torch.int32), _contig(esc_vals, None), esc_vals.numel(), _contig(esc_off, torch.int64),
        _contig(symbols, torch.uint8), _ptr(out_k, torch.float16), _ptr(out_v, torch.float16),
        _contig(ws, torch.uint8), ws.numel(), _contig(status, torch.int32), _stream())
    _check(rc, "plc_rans_decode_reconstruct_cond")


def plc_predict_residual_cond(dims, cand_k, cand_v, probs, chosen, act_k, act_v, symbols, esc_vals,
                              esc_cnt, esc_off, ws, status, pred_out=None):
    """As plc_predict_residual, with chosen int32 [S,n] (candidate index of the true token, -1 = none)."""
    rc = lib().plc_predict_residual_cond(
        C.byref(dims), _ptr(cand_k, torch.float16), _ptr(cand_v, torch.float16),
        _contig(probs, torch.float32), _contig(chosen, torch.int32), _ptr(act_k, torch.float16),
        _ptr(act_v, torch.float16), _contig(symbols, torch.uint8), _contig(esc_vals, None),
        esc_vals.numel(), _contig(esc_cnt, torch.int32), _contig(esc_off, torch.int64),
        _contig(pred_out, torch.float32), _contig(ws, torch.uint8), ws.numel(),
        _contig(status, torch.int32), _stream())
    _check(rc, "plc_predict_residual_cond")


def plc_reconstruct_cond(dims, cand_k, cand_v, probs, chosen, symbols, esc_vals, esc_off, out_k, out_v,
                         ws, status):
    rc = lib().plc_reconstruct_cond(
        C.byref(dims), _ptr(cand_k, torch.float16), _ptr(cand_v, torch.float16),
        _contig(probs, torch.float32), _contig(chosen, torch.int32), _contig(symbols, torch.uint8),
        _contig(esc_vals, None), esc_vals.numel(), _contig(esc_off, torch.int64),
        _ptr(out_k, torch.float16), _ptr(out_v, torch.float16), _contig(ws, torch.uint8), ws.numel(),
        _contig(status, torch.int32), _stream())
    _check(rc, "plc_reconstruct_cond")


def plc_select_candidate(dims, cand_k, act_k, max_mean_sq, chosen):
    rc = lib().plc_select_candidate(C.byref(dims), _ptr(cand_k, torch.float16), _ptr(act_k, torch.float16),
                                    float(max_mean_sq), _contig(chosen, torch.int32), _stream())
    _check(rc, "plc_select_candidate")


def plc_index_encode(probs, chosen, S, n, k, states, words, word_off, word_cap, n_words, status):
    rc = lib().plc_index_encode(_contig(probs, torch.float32), _contig(chosen, torch.int32), S, n, k,
                                _contig(states, torch.int32), _contig(words, torch.int16),
                                _contig(word_off, torch.int64), int(word_cap),
                                _contig(n_words, torch.int32), _contig(status, torch.int32), _stream())
    _check(rc, "plc_index_encode")


def plc_index_decode(probs, states, words, word_off, n_words, S, n, k, chosen, status):
    rc = lib().plc_index_decode(_contig(probs, torch.float32), _contig(states, torch.int32),
                                _contig(words, torch.int16), words.numel(),
                                _contig(word_off, torch.int64), _contig(n_words, torch.int32), S, n, k,
                                _contig(chosen, torch.int32), _contig(status, torch.int32), _stream())
    _check(rc, "plc_index_decode")


def plc_surprisal_thresholds(b0, hbar, bmax=MAX_BITS):
    """Host call: the bmax + 1 thresholds (entries 0, 1 unused) that plc_surprisal_bits compares with."""
    arr = (C.c_uint16 * (int(bmax) + 1))()
    _check(lib().plc_surprisal_thresholds(float(b0), float(hbar), int(bmax), arr), "plc_surprisal_thresholds")
    return list(arr)


surprisal_thresholds = plc_surprisal_thresholds


def plc_surprisal_bits(probs, chosen, S, n, k, thr, bits, status):
    """thr: host sequence of bmax + 1 integers (see surprisal_thresholds); bits: uint8 [S,n] out."""
    arr = (C.c_uint16 * len(thr))(*[int(t) for t in thr])
    rc = lib().plc_surprisal_bits(_contig(probs, torch.float32), _contig(chosen, torch.int32), S, n, k, arr,
                                  len(thr) - 1, _contig(bits, torch.uint8), _contig(status, torch.int32), _stream())
    _check(rc, "plc_surprisal_bits")


def plc_predict_residual_adapt(dims, cand_k, cand_v, probs, chosen, bits, step_range, act_k, act_v, symbols,
                               esc_vals, esc_cnt, esc_off, ws, status, pred_out=None):
    rc = lib().plc_predict_residual_adapt(
        C.byref(dims), _ptr(cand_k, torch.float16), _ptr(cand_v, torch.float16),
        _contig(probs, torch.float32), _contig(chosen, torch.int32), _contig(bits, torch.uint8),
        float(step_range), _ptr(act_k, torch.float16), _ptr(act_v, torch.float16),
        _contig(symbols, torch.uint8), _contig(esc_vals, None), esc_vals.numel(),
        _contig(esc_cnt, torch.int32), _contig(esc_off, torch.int64), _contig(pred_out, torch.float32),
        _contig(ws, torch.uint8), ws.numel(), _contig(status, torch.int32), _stream())
    _check(rc, "plc_predict_residual_adapt")


def plc_reconstruct_adapt(dims, cand_k, cand_v, probs, chosen, bits, step_range, symbols, esc_vals, esc_off,
                          out_k, out_v, ws, status):
    rc = lib().plc_reconstruct_adapt(
        C.byref(dims), _ptr(cand_k, torch.float16), _ptr(cand_v, torch.float16),
        _contig(probs, torch.float32), _contig(chosen, torch.int32), _contig(bits, torch.uint8),
        float(step_range), _contig(symbols, torch.uint8), _contig(esc_vals, None), esc_vals.numel(),
        _contig(esc_off, torch.int64), _ptr(out_k, torch.float16), _ptr(out_v, torch.float16),
        _contig(ws, torch.uint8), ws.numel(), _contig(status, torch.int32), _stream())
    _check(rc, "plc_reconstruct_adapt")


def plc_histogram_bucketed(symbols, n_streams, syms_per_stream, syms_per_pos, streams_per_session, bits,
                           n_tables, counts, status):
    rc = lib().plc_histogram_bucketed(_contig(symbols, torch.uint8), n_streams, syms_per_stream, syms_per_pos,
                                      streams_per_session, _contig(bits, torch.uint8), n_tables,
                                      _contig(counts, torch.int32), _contig(status, torch.int32), _stream())
    _check(rc, "plc_histogram_bucketed")


def plc_build_freq_bucketed(counts, n_streams, n_tables, freq, status):
    rc = lib().plc_build_freq_bucketed(_contig(counts, torch.int32), n_streams, n_tables,
                                       _contig(freq, torch.int16), _contig(status, torch.int32), _stream())
    _check(rc, "plc_build_freq_bucketed")


def plc_rans_encode_bucketed(symbols, n_streams, syms_per_stream, chunk_syms, syms_per_pos,
                             streams_per_session, bits, n_tables, freq, states, words, word_off,
                             word_cap_per_unit, n_words, status):
    rc = lib().plc_rans_encode_bucketed(_contig(symbols, torch.uint8), n_streams, syms_per_stream, chunk_syms,
                                        syms_per_pos, streams_per_session, _contig(bits, torch.uint8), n_tables,
                                        _contig(freq, torch.int16), _contig(states, torch.int32),
                                        _contig(words, torch.int16), _contig(word_off, torch.int64),
                                        int(word_cap_per_unit), _contig(n_words, torch.int32),
                                        _contig(status, torch.int32), _stream())
    _check(rc, "plc_rans_encode_bucketed")


def plc_rans_decode_bucketed(freq, states, words, word_off, n_words, n_streams, syms_per_stream, chunk_syms,
                             syms_per_pos, streams_per_session, bits, n_tables, symbols, status):
    rc = lib().plc_rans_decode_bucketed(_contig(freq, torch.int16), _contig(states, torch.int32),
                                        _contig(words, torch.int16), words.numel(),
                                        _contig(word_off, torch.int64), _contig(n_words, torch.int32),
                                        n_streams, syms_per_stream, chunk_syms, syms_per_pos,
                                        streams_per_session, _contig(bits, torch.uint8), n_tables,
                                        _contig(symbols, torch.uint8), _contig(status, torch.int32), _stream())
    _check(rc, "plc_rans_decode_bucketed")


def plc_rans_decode_reconstruct_adapt(dims, freq, states, words, word_off, n_words, chunk_syms, n_tables, cand_k,
                                      cand_v, probs, chosen, bits, step_range, esc_vals, esc_off, symbols, out_k,
                                      out_v, ws, status):
    rc = lib().plc_rans_decode_reconstruct_adapt(
        C.byref(dims), _contig(freq, torch.int16), _contig(states, torch.int32), _contig(words, torch.int16),
        words.numel(), _contig(word_off, torch.int64), _contig(n_words, torch.int32), chunk_syms, n_tables,
        _ptr(cand_k, torch.float16), _ptr(cand_v, torch.float16), _contig(probs, torch.float32),
        _contig(chosen, torch.int32), _contig(bits, torch.uint8), float(step_range), _contig(esc_vals, None),
        esc_vals.numel(), _contig(esc_off, torch.int64), _contig(symbols, torch.uint8),
        _ptr(out_k, torch.float16), _ptr(out_v, torch.float16), _contig(ws, torch.uint8), ws.numel(),
        _contig(status, torch.int32), _stream())
    _check(rc, "plc_rans_decode_reconstruct_adapt")


def plc_expected_embedding(probs_full, embed_t, ebar):
    """probs_full fp16 [rows, V], embed_t fp16 [m, V] -> ebar fp16 [rows, m]."""
    rows, V = probs_full.shape
    m = embed_t.shape[0]
    rc = lib().plc_expected_embedding(_contig(probs_full, torch.float16), _contig(embed_t, torch.float16), rows, V,
                                      m, _contig(ebar, torch.float16), _stream())
    _check(rc, "plc_expected_embedding")


def plc_predict_residual_linear(dims, ebar, A, bias_k, bias_v, act_k, act_v, symbols, esc_vals, esc_cnt, esc_off,
                                ws, status):
    m = A.shape[-1]
    rc = lib().plc_predict_residual_linear(
        C.byref(dims), _contig(ebar, torch.float16), m, _contig(A, torch.float16), _ptr(bias_k, torch.float16),
        _ptr(bias_v, torch.float16), _ptr(act_k, torch.float16), _ptr(act_v, torch.float16),
        _contig(symbols, torch.uint8), _contig(esc_vals, None), esc_vals.numel(), _contig(esc_cnt, torch.int32),
        _contig(esc_off, torch.int64), _contig(ws, torch.uint8), ws.numel(), _contig(status, torch.int32), _stream())
    _check(rc, "plc_predict_residual_linear")


def plc_reconstruct_linear(dims, ebar, A, bias_k, bias_v, symbols, esc_vals, esc_off, out_k, out_v, ws, status):
    m = A.shape[-1]
    rc = lib().plc_reconstruct_linear(
        C.byref(dims), _contig(ebar, torch.float16), m, _contig(A, torch.float16), _ptr(bias_k, torch.float16),
        _ptr(bias_v, torch.float16), _contig(symbols, torch.uint8), _contig(esc_vals, None), esc_vals.numel(),
        _contig(esc_off, torch.int64), _ptr(out_k, torch.float16), _ptr(out_v, torch.float16),
        _contig(ws, torch.uint8), ws.numel(), _contig(status, torch.int32), _stream())
    _check(rc, "plc_reconstruct_linear")


class PrefixTrie:
    """Host-side prefix index (plc_trie_*): insert / best_match / evict over token sequences (numpy int32
    arrays; `bits` = per-token surprisal, float32, optional)."""

    def __init__(self, max_bits=float("inf")):
        import numpy as np
        self._np = np
        self._t = lib().plc_trie_create(float(min(max_bits, 1e300)))
        if not self._t:
            raise PlcError(PLC_ERR_INVALID, "plc_trie_create")

    def close(self):
        if getattr(self, "_t", None):
            lib().plc_trie_destroy(self._t)
            self._t = None

    def __del__(self):
        try:
            self.close()
        except Exception:           # interpreter shutdown: the module globals may be gone already
            pass

    def __len__(self):
        return int(lib().plc_trie_size(self._t))

    @property
    def nodes(self):
        return int(lib().plc_trie_nodes(self._t))

    def _arr(self, a, dtype):
        a = self._np.ascontiguousarray(a, dtype=dtype)
        return a, a.ctypes.data_as(C.c_void_p)

    def insert(self, tokens, ident, bits=None):
        """Returns the number of tokens kept (the path is cut where its surprisal sum would exceed max_bits)."""
        tok, tp = self._arr(tokens, self._np.int32)
        bp = None
        if bits is not None:
            b, bp = self._arr(bits, self._np.float32)
            assert b.size == tok.size
        kept = C.c_int64(0)
        _check(lib().plc_trie_insert(self._t, tp, bp, tok.size, int(ident), C.byref(kept)), "plc_trie_insert")
        return int(kept.value)

    def best_match(self, tokens):
        """(id, lcp, dist): a stored prefix with the longest common prefix with the query (-1 if empty)."""
        tok, tp = self._arr(tokens, self._np.int32)
        ident, lcp, dist = C.c_int64(0), C.c_int64(0), C.c_double(0.0)
        _check(lib().plc_trie_best_match(self._t, tp, tok.size, C.byref(ident), C.byref(lcp), C.byref(dist)),
               "plc_trie_best_match")
        return int(ident.value), int(lcp.value), float(dist.value)

    def evict(self, ident):
        _check(lib().plc_trie_evict(self._t, int(ident)), "plc_trie_evict")


def plc_trace_kernel_events(kernel_id, start=None, stop=None):
    """start/stop: raw hipEvent_t handles (ints) or None to clear."""
    rc = lib().plc_trace_kernel_events(int(kernel_id), C.c_void_p(start) if start else None,
                                       C.c_void_p(stop) if stop else None)
    _check(rc, "plc_trace_kernel_events")
