"""Buffer management around the libplc calls: allocate once, then encode and
decode a KV cache of fixed shape any number of times.  Every step of the
coding path runs inside libplc; this class only owns torch tensors and calls
the entry points in order.

Two paths share the buffers: the weighted-mean path (encode / decode) and the
token-conditional path (encode_cond / decode_cond), which predicts every
position from the candidate of its true token and codes that candidate's index
in a stream of its own.  encode_adapt / decode_adapt add the surprisal-adaptive
quantiser on top of the latter: a bit depth per position from the token's
surprisal, a step of range / 2^depth, and one frequency table per depth."""
from __future__ import annotations

import dataclasses

import torch

from . import plc


@dataclasses.dataclass
class Coded:
    """What an encode leaves in device memory (views into the codec's buffers)."""
    symbols: torch.Tensor    # u8  [streams, N]
    esc_vals: torch.Tensor   # i16 [esc_cap] raw fp16 bit patterns, stream after stream
    esc_cnt: torch.Tensor    # i32 [streams]
    esc_off: torch.Tensor    # i64 [streams]
    counts: torch.Tensor     # i32 [streams, 256]
    freq: torch.Tensor       # i16 [streams, 256]
    cum: torch.Tensor        # i16 [streams, 257]
    states: torch.Tensor     # i32 [units, 32]
    words: torch.Tensor      # i16 [units * word_cap]
    word_off: torch.Tensor   # i64 [units]
    n_words: torch.Tensor    # i32 [units]
    # token-conditional path only
    chosen: torch.Tensor = None         # i32 [S, n] as used by the encoder
    idx_states: torch.Tensor = None     # i32 [S, 32]
    idx_words: torch.Tensor = None      # i16 [S * idx_word_cap]
    idx_word_off: torch.Tensor = None   # i64 [S]
    idx_n_words: torch.Tensor = None    # i32 [S]
    # adaptive path only
    bits: torch.Tensor = None           # u8 [S, n] bit depth per position
    counts_d: torch.Tensor = None       # i32 [streams, MAX_BITS, 256]
    freq_d: torch.Tensor = None         # i16 [streams, MAX_BITS, 256]


class KVDeltaCodec:
    def __init__(self, S, L, H, n, k, d, delta, qmax=127, chunk_syms=0, device="cuda",
                 cand_stride=None, act_stride=None, esc_frac=1.0 / 16, word_frac=1.0,
                 want_pred=False):
        self.device = torch.device(device)
        self.dims = plc.make_dims(S, L, H, n, k, d, delta, qmax, cand_stride, act_stride)
        self.S, self.L, self.H, self.n, self.k, self.d = S, L, H, n, k, d
        self.n_streams = S * L * H
        self.N = 2 * n * d
        self.chunk_syms = int(chunk_syms)
        self.units_per_stream = plc.plc_units_per_stream(self.N, self.chunk_syms)
        self.n_units = self.n_streams * self.units_per_stream
        unit_syms = self.chunk_syms if self.chunk_syms else self.N
        # words per unit: never more than one per symbol; rounded up to 16 bytes
        self.word_cap = (max(8, int(unit_syms * word_frac)) + 7) // 8 * 8
        E = self.n_streams * self.N
        esc_cap = max(64, int(E * esc_frac))
        dev = self.device
        ws_bytes = plc.plc_workspace_bytes(self.dims)
        if ws_bytes == 0:
            raise plc.PlcError(plc.PLC_ERR_INVALID, "plc_workspace_bytes")
        self.ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
        self.status = torch.zeros(1, dtype=torch.int32, device=dev)
        self.symbols = torch.empty((self.n_streams, self.N), dtype=torch.uint8, device=dev)
        self.esc_vals = torch.empty(esc_cap, dtype=torch.int16, device=dev)
        self.esc_cnt = torch.empty(self.n_streams, dtype=torch.int32, device=dev)
        self.esc_off = torch.empty(self.n_streams, dtype=torch.int64, device=dev)
        self.counts = torch.empty((self.n_streams, 256), dtype=torch.int32, device=dev)
        self.freq = torch.empty((self.n_streams, 256), dtype=torch.int16, device=dev)
        self.cum = torch.empty((self.n_streams, 257), dtype=torch.int16, device=dev)
        self.states = torch.empty((self.n_units, 32), dtype=torch.int32, device=dev)
        self.words = torch.empty(self.n_units * self.word_cap, dtype=torch.int16, device=dev)
        self.word_off = torch.arange(self.n_units, dtype=torch.int64, device=dev) * self.word_cap
        self.n_words = torch.empty(self.n_units, dtype=torch.int32, device=dev)
        self.pred = (torch.empty((self.n_streams, self.N), dtype=torch.float32, device=dev)
                     if want_pred else None)
        self.dec_symbols = torch.empty_like(self.symbols)
        # index stream of the token-conditional path: at most one word per position
        self.idx_word_cap = (n + 7) // 8 * 8
        self.chosen = torch.empty((S, n), dtype=torch.int32, device=dev)
        self.dec_chosen = torch.empty_like(self.chosen)
        self.idx_states = torch.empty((S, 32), dtype=torch.int32, device=dev)
        self.idx_words = torch.empty(S * self.idx_word_cap, dtype=torch.int16, device=dev)
        self.idx_word_off = torch.arange(S, dtype=torch.int64, device=dev) * self.idx_word_cap
        self.idx_n_words = torch.empty(S, dtype=torch.int32, device=dev)

    # -- single steps -------------------------------------------------------------------
    def predict_residual(self, cand_k, cand_v, probs, act_k, act_v, with_counts=False):
        """with_counts: also leave the symbols' per-stream counts in self.counts (no histogram call needed after)."""
        if with_counts:
            plc.plc_predict_residual_hist(self.dims, cand_k, cand_v, probs, act_k, act_v, self.symbols,
                                          self.esc_vals, self.esc_cnt, self.esc_off, self.counts, self.ws,
                                          self.status, pred_out=self.pred)
        else:
            plc.plc_predict_residual(self.dims, cand_k, cand_v, probs, act_k, act_v, self.symbols,
                                     self.esc_vals, self.esc_cnt, self.esc_off, self.ws, self.status,
                                     pred_out=self.pred)

    def histogram(self, symbols=None):
        plc.plc_histogram(self.symbols if symbols is None else symbols, self.n_streams, self.N, self.counts)

    def build_freq(self):
        plc.plc_build_freq(self.counts, self.n_streams, self.freq, self.cum, self.status)

    def rans_encode(self, symbols=None):
        plc.plc_rans_encode(self.symbols if symbols is None else symbols, self.n_streams, self.N,
                            self.chunk_syms, self.freq, self.states, self.words, self.word_off,
                            self.word_cap, self.n_words, self.status)

    def rans_decode(self, out=None):
        out = self.dec_symbols if out is None else out
        plc.plc_rans_decode(self.freq, self.states, self.words, self.word_off, self.n_words,
                            self.n_streams, self.N, self.chunk_syms, out, self.status)
        return out

    def reconstruct(self, cand_k, cand_v, probs, out_k, out_v, symbols=None):
        plc.plc_reconstruct(self.dims, cand_k, cand_v, probs,
                            self.dec_symbols if symbols is None else symbols,
                            self.esc_vals, self.esc_off, out_k, out_v, self.ws, self.status)

    # -- whole directions ---------------------------------------------------------------
    def encode(self, cand_k, cand_v, probs, act_k, act_v, fused_counts=True) -> Coded:
        """fused_counts: the symbol statistics are taken inside the prediction pass (the results are the same
        either way); False makes the plc_histogram call instead."""
        self.predict_residual(cand_k, cand_v, probs, act_k, act_v, with_counts=fused_counts)
        if not fused_counts:
            self.histogram()
        self.build_freq()
        self.rans_encode()
        return self.coded()

    def decode(self, cand_k, cand_v, probs, out_k, out_v, fused=True):
        """fused: one call that reconstructs inside the entropy decoder where the shape allows it (the
        results are the same either way); False makes the two calls one after the other."""
        if fused:
            plc.plc_rans_decode_reconstruct(self.dims, self.freq, self.states, self.words, self.word_off,
                                            self.n_words, self.chunk_syms, cand_k, cand_v, probs, self.esc_vals,
                                            self.esc_off, self.dec_symbols, out_k, out_v, self.ws, self.status)
        else:
            self.rans_decode()
            self.reconstruct(cand_k, cand_v, probs, out_k, out_v)

    # -- linear-embedding predictor ------------------------------------------------------------
    def encode_linear(self, probs_full, embed_t, A, bias_k, bias_v, act_k, act_v) -> Coded:
        """Prediction c + A * Ebar with Ebar = probs_full @ embed_t^T (both contractions on the matrix cores),
        then the core path's residual, quantiser, statistics and rANS."""
        rows, m = probs_full.shape[0], embed_t.shape[0]
        if not hasattr(self, "ebar") or self.ebar.shape != (rows, m):
            self.ebar = torch.empty((rows, m), dtype=torch.float16, device=self.device)
        plc.plc_expected_embedding(probs_full, embed_t, self.ebar)
        plc.plc_predict_residual_linear(self.dims, self.ebar, A, bias_k, bias_v, act_k, act_v, self.symbols,
                                        self.esc_vals, self.esc_cnt, self.esc_off, self.ws, self.status)
        self.histogram()
        self.build_freq()
        self.rans_encode()
        return self.coded()

    def decode_linear(self, probs_full, embed_t, A, bias_k, bias_v, out_k, out_v):
        rows, m = probs_full.shape[0], embed_t.shape[0]
        if not hasattr(self, "ebar") or self.ebar.shape != (rows, m):
            self.ebar = torch.empty((rows, m), dtype=torch.float16, device=self.device)
        plc.plc_expected_embedding(probs_full, embed_t, self.ebar)      # recomputed, as a decoder would
        self.rans_decode()
        plc.plc_reconstruct_linear(self.dims, self.ebar, A, bias_k, bias_v, self.dec_symbols, self.esc_vals,
                                   self.esc_off, out_k, out_v, self.ws, self.status)

    # -- surprisal-adaptive quantiser on the token-conditional path --------------------------
    def _adapt_buffers(self):
        if not hasattr(self, "bits"):
            dev = self.device
            self.bits = torch.empty((self.S, self.n), dtype=torch.uint8, device=dev)
            self.dec_bits = torch.empty_like(self.bits)
            self.counts_d = torch.empty((self.n_streams, plc.MAX_BITS, 256), dtype=torch.int32, device=dev)
            self.freq_d = torch.empty((self.n_streams, plc.MAX_BITS, 256), dtype=torch.int16, device=dev)

    def encode_adapt(self, cand_k, cand_v, probs, act_k, act_v, chosen, thr, step_range) -> Coded:
        """thr: thresholds from plc.surprisal_thresholds(b0, hbar); step_range: fp32 range of the quantiser."""
        self._adapt_buffers()
        if chosen is not self.chosen:
            self.chosen.copy_(chosen)
        B, spp, sps = plc.MAX_BITS, 2 * self.d, self.L * self.H
        plc.plc_surprisal_bits(probs, self.chosen, self.S, self.n, self.k, thr, self.bits, self.status)
        plc.plc_predict_residual_adapt(self.dims, cand_k, cand_v, probs, self.chosen, self.bits, step_range, act_k,
                                       act_v, self.symbols, self.esc_vals, self.esc_cnt, self.esc_off, self.ws,
                                       self.status, pred_out=self.pred)
        plc.plc_histogram_bucketed(self.symbols, self.n_streams, self.N, spp, sps, self.bits, B, self.counts_d,
                                   self.status)
        plc.plc_build_freq_bucketed(self.counts_d, self.n_streams, B, self.freq_d, self.status)
        plc.plc_rans_encode_bucketed(self.symbols, self.n_streams, self.N, self.chunk_syms, spp, sps, self.bits, B,
                                     self.freq_d, self.states, self.words, self.word_off, self.word_cap,
                                     self.n_words, self.status)
        plc.plc_index_encode(probs, self.chosen, self.S, self.n, self.k, self.idx_states, self.idx_words,
                             self.idx_word_off, self.idx_word_cap, self.idx_n_words, self.status)
        c = self.coded(cond=True)
        c.bits, c.counts_d, c.freq_d = self.bits, self.counts_d, self.freq_d
        return c

    def decode_adapt(self, cand_k, cand_v, probs, out_k, out_v, thr, step_range, fused=True):
        """From the coded artefacts alone: the index stream gives the tokens, the tokens the bit depths."""
        B, spp, sps = plc.MAX_BITS, 2 * self.d, self.L * self.H
        plc.plc_index_decode(probs, self.idx_states, self.idx_words, self.idx_word_off, self.idx_n_words,
                             self.S, self.n, self.k, self.dec_chosen, self.status)
        plc.plc_surprisal_bits(probs, self.dec_chosen, self.S, self.n, self.k, thr, self.dec_bits, self.status)
        if fused:
            plc.plc_rans_decode_reconstruct_adapt(self.dims, self.freq_d, self.states, self.words, self.word_off,
                                                  self.n_words, self.chunk_syms, B, cand_k, cand_v, probs,
                                                  self.dec_chosen, self.dec_bits, step_range, self.esc_vals,
                                                  self.esc_off, self.dec_symbols, out_k, out_v, self.ws, self.status)
            return
        plc.plc_rans_decode_bucketed(self.freq_d, self.states, self.words, self.word_off, self.n_words,
                                     self.n_streams, self.N, self.chunk_syms, spp, sps, self.dec_bits, B,
                                     self.dec_symbols, self.status)
        plc.plc_reconstruct_adapt(self.dims, cand_k, cand_v, probs, self.dec_chosen, self.dec_bits, step_range,
                                  self.dec_symbols, self.esc_vals, self.esc_off, out_k, out_v, self.ws, self.status)

    # -- token-conditional path ----------------------------------------------------------
    def select_candidate(self, cand_k, act_k, max_mean_sq):
        plc.plc_select_candidate(self.dims, cand_k, act_k, max_mean_sq, self.chosen)
        return self.chosen

    def encode_cond(self, cand_k, cand_v, probs, act_k, act_v, chosen=None, max_mean_sq=None) -> Coded:
        """chosen: int32 [S,n] on the device, or None to recover it from the vectors (max_mean_sq =
        largest mean squared distance per component at which a candidate still counts as the token)."""
        if chosen is None:
            if max_mean_sq is None:
                raise ValueError("either chosen or max_mean_sq is needed")
            self.select_candidate(cand_k, act_k, max_mean_sq)
        elif chosen is not self.chosen:
            self.chosen.copy_(chosen)
        plc.plc_predict_residual_cond(self.dims, cand_k, cand_v, probs, self.chosen, act_k, act_v,
                                      self.symbols, self.esc_vals, self.esc_cnt, self.esc_off, self.ws,
                                      self.status, pred_out=self.pred)
        self.histogram()
        self.build_freq()
        self.rans_encode()
        plc.plc_index_encode(probs, self.chosen, self.S, self.n, self.k, self.idx_states, self.idx_words,
                             self.idx_word_off, self.idx_word_cap, self.idx_n_words, self.status)
        return self.coded(cond=True)

    def decode_cond(self, cand_k, cand_v, probs, out_k, out_v, fused=True):
        plc.plc_index_decode(probs, self.idx_states, self.idx_words, self.idx_word_off, self.idx_n_words,
                             self.S, self.n, self.k, self.dec_chosen, self.status)
        if fused:
            plc.plc_rans_decode_reconstruct_cond(self.dims, self.freq, self.states, self.words, self.word_off,
                                                 self.n_words, self.chunk_syms, cand_k, cand_v, probs,
                                                 self.dec_chosen, self.esc_vals, self.esc_off, self.dec_symbols,
                                                 out_k, out_v, self.ws, self.status)
        else:
            self.rans_decode()
            plc.plc_reconstruct_cond(self.dims, cand_k, cand_v, probs, self.dec_chosen, self.dec_symbols,
                                     self.esc_vals, self.esc_off, out_k, out_v, self.ws, self.status)

    def coded(self, cond=False) -> Coded:
        if cond:
            return Coded(self.symbols, self.esc_vals, self.esc_cnt, self.esc_off, self.counts, self.freq,
                         self.cum, self.states, self.words, self.word_off, self.n_words, self.chosen,
                         self.idx_states, self.idx_words, self.idx_word_off, self.idx_n_words)
        return Coded(self.symbols, self.esc_vals, self.esc_cnt, self.esc_off, self.counts, self.freq,
                     self.cum, self.states, self.words, self.word_off, self.n_words)

    def check_status(self, where="plc"):
        """Synchronises and raises if a kernel reported a data-dependent error."""
        code = int(self.status.item())
        if code != plc.PLC_OK:
            self.status.zero_()
            raise plc.PlcError(code, where)


class GroupedCodec:
    """The weighted-mean path over a cache with thousands of streams, coded as independent groups of whole
    sessions (or, inside one session, of whole layers), each group a KVDeltaCodec of its own with its own
    buffers and artefacts.  Nothing is computed here: the class slices the caller's tensors into the groups'
    views and orders the same libplc calls on two HIP streams, so that the entropy coding of one group
    (integer work, bound by instruction issue and LDS) runs beside the prediction pass of the next (bound by
    HBM): the caller's current stream carries the prediction passes, a side stream of default priority the
    statistics, tables and rANS encoders; decode calls alternate between the two.  Streams are independent
    units from the first step to the last, so a group's artefacts are exactly those a codec over that slice
    alone would produce."""

    def __init__(self, S, L, H, n, k, d, delta, qmax=127, groups=8, device="cuda", cand_stride=None,
                 act_stride=None, **kw):
        self.device = torch.device(device)
        self.S, self.L, self.H, self.n, self.k, self.d = S, L, H, n, k, d
        self.N = 2 * n * d
        self.n_streams = S * L * H
        # a group: sessions [s0, s1) whole, or layers [l0, l1) of session s0
        self.slices = []
        groups = max(1, int(groups))
        if S >= groups:
            for g in range(groups):
                s0, s1 = S * g // groups, S * (g + 1) // groups
                self.slices.append((s0, s1, 0, L))
        else:
            per = max(1, min(L, (groups + S - 1) // S))
            for s in range(S):
                for g in range(per):
                    l0, l1 = L * g // per, L * (g + 1) // per
                    self.slices.append((s, s + 1, l0, l1))
        self.codecs = [KVDeltaCodec(s1 - s0, l1 - l0, H, n, k, d, delta, qmax, device=device,
                                    cand_stride=cand_stride, act_stride=act_stride, **kw)
                       for s0, s1, l0, l1 in self.slices]
        self.n_units = sum(c.n_units for c in self.codecs)
        self.side = torch.cuda.Stream(device=self.device)            # default priority
        self.events = [torch.cuda.Event() for _ in self.codecs]
        self.hook = None        # optional callable(group index), called before a group's calls are enqueued

    def _views(self, i, *tensors):
        s0, s1, l0, l1 = self.slices[i]
        return [t[s0:s1, l0:l1] for t in tensors]

    def encode(self, cand_k, cand_v, probs, act_k, act_v, overlap=True):
        main = torch.cuda.current_stream()
        side = self.side if overlap else main
        if overlap:
            side.wait_stream(main)
        for i, c in enumerate(self.codecs):
            ck, cv, ak, av = self._views(i, cand_k, cand_v, act_k, act_v)
            p = probs[self.slices[i][0]:self.slices[i][1]]
            if self.hook:
                self.hook(i)
            c.predict_residual(ck, cv, p, ak, av, with_counts=True)
            if overlap:
                self.events[i].record(main)
                side.wait_event(self.events[i])
            with torch.cuda.stream(side):
                c.build_freq()
                c.rans_encode()
        if overlap:
            main.wait_stream(side)
        return [c.coded() for c in self.codecs]

    def decode(self, cand_k, cand_v, probs, out_k, out_v, fused=True, overlap=True):
        main = torch.cuda.current_stream()
        if overlap:
            self.side.wait_stream(main)
        for i, c in enumerate(self.codecs):
            ck, cv, ok, ov = self._views(i, cand_k, cand_v, out_k, out_v)
            p = probs[self.slices[i][0]:self.slices[i][1]]
            if self.hook:
                self.hook(i)
            with torch.cuda.stream(self.side if (overlap and i % 2) else main):
                c.decode(ck, cv, p, ok, ov, fused=fused)
        if overlap:
            main.wait_stream(self.side)

    def check_status(self, where="plc"):
        for c in self.codecs:
            c.check_status(where)

    # what the accounting needs, summed over the groups
    def total_words(self):
        return sum(int(c.n_words.to(torch.int64).sum()) for c in self.codecs)

    def total_escapes(self):
        return sum(int(c.esc_cnt.to(torch.int64).sum()) for c in self.codecs)

    def roundtrip_exact(self):
        return all(bool(torch.equal(c.dec_symbols, c.symbols)) for c in self.codecs)
