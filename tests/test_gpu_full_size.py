"""Parity at the benchmark's full size, in the launch configuration bench.py times.

The whole Llama-3-8B-shaped workload (256 streams of 2^20 symbols) is encoded and
decoded on the GPU exactly as bench.py does it; the oracle then recomputes a
sample of whole streams one by one (a stream is the unit everything downstream
of the symbols depends on) and every artefact of those streams must match bit
for bit.  Properties that hold at any size are checked on all streams.
"""
import numpy as np
import pytest
import torch

from paper_2604_15356_amd.workloads import make_workload
from tests.gpu_util import codec_for, near_tie_report, u8, u16, u32, u64

pytestmark = pytest.mark.gpu

SAMPLE_STREAMS = (0, 7, 100, 255)


@pytest.fixture(scope="module")
def run():
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    dev = torch.device("cuda:0")
    w = make_workload("llama8b", device=dev)
    out = {}
    for chunk in (0, 4096):
        print(f"full-size llama8b, chunk_syms={chunk}", flush=True)
        codec = codec_for(w, chunk_syms=chunk, want_pred=False)
        coded = codec.encode(w.cand_k, w.cand_v, w.probs, w.act_k, w.act_v)
        out_k, out_v = torch.zeros_like(w.act_k), torch.zeros_like(w.act_v)
        codec.decode(w.cand_k, w.cand_v, w.probs, out_k, out_v)
        codec.check_status("full size")
        # every stream, not only the sampled ones: the single decode call (one kernel that also
        # reconstructs when chunk = 0) against the two calls one after the other
        sym_one = codec.dec_symbols.clone()
        two_k, two_v = torch.zeros_like(w.act_k), torch.zeros_like(w.act_v)
        codec.dec_symbols.zero_()
        codec.decode(w.cand_k, w.cand_v, w.probs, two_k, two_v, fused=False)
        codec.check_status("full size, two calls")
        assert torch.equal(codec.dec_symbols, sym_one)
        assert torch.equal(two_k.view(torch.int16), out_k.view(torch.int16))
        assert torch.equal(two_v.view(torch.int16), out_v.view(torch.int16))
        del two_k, two_v, sym_one
        out[chunk] = (codec, coded, out_k, out_v)
    return w, out


def _stream_inputs(w, st):
    s, r = divmod(st, w.L * w.H)
    l, h = divmod(r, w.H)
    host = lambda t: t.contiguous().cpu().numpy()
    return (host(w.cand_k[s, l, h]), host(w.cand_v[s, l, h]), host(w.probs[s]),
            host(w.act_k[s, l, h]), host(w.act_v[s, l, h])), (s, l, h)


@pytest.mark.parametrize("chunk", [0, 4096])
def test_sampled_streams_match_oracle_bit_for_bit(oracle, run, chunk):
    O = oracle
    w, out = run
    codec, coded, out_k, out_v = out[chunk]
    dm = O.make_dims(1, 1, 1, w.n, w.k, w.d, w.delta, w.qmax)
    U = codec.units_per_stream
    words = None
    for st in SAMPLE_STREAMS:
        print(f"  stream {st}", flush=True)
        (ck, cv, p, ak, av), (s, l, h) = _stream_inputs(w, st)
        ref32 = O.predict_residual(dm, ck, cv, p, ak, av, mode=O.F32)
        ref64 = O.predict_residual(dm, ck, cv, p, ak, av, mode=O.F64, want_u=True)
        sym = u8(coded.symbols[st:st + 1])
        assert np.array_equal(sym, ref32["symbols"])
        tau = 64 * 2.0 ** -24 * 8.0 / float(np.float32(w.delta))
        n_diff, n_ok = near_tie_report(sym, ref64["symbols"], ref64["u"], tau)
        assert n_diff == n_ok and n_diff < 1e-4 * sym.size
        # escape list of the stream
        off = int(u64(coded.esc_off)[st])
        cnt = int(u32(coded.esc_cnt)[st])
        assert cnt == int(ref32["esc_cnt"][0])
        assert np.array_equal(u16(coded.esc_vals[off:off + cnt]), ref32["esc_vals"])
        # table and bitstream
        counts = O.histogram(sym)
        freq, cum = O.build_freq(counts)
        assert np.array_equal(u32(coded.counts[st:st + 1]), counts)
        assert np.array_equal(u16(coded.freq[st:st + 1]), freq)
        enc = O.rans_encode(sym, freq, chunk_syms=chunk, word_cap_per_unit=codec.word_cap)
        assert np.array_equal(u32(coded.n_words[st * U:(st + 1) * U]), enc["n_words"])
        assert np.array_equal(u32(coded.states[st * U:(st + 1) * U]), enc["states"])
        if words is None:
            words = u16(coded.words)
        for u in range(U):
            o, nw = (st * U + u) * codec.word_cap, int(enc["n_words"][u])
            assert np.array_equal(words[o:o + nw], enc["words"][u * codec.word_cap:u * codec.word_cap + nw])
        # the oracle decodes the GPU's stream, and reconstructs what the GPU reconstructed
        dec = O.rans_decode(freq, u32(coded.states[st * U:(st + 1) * U]),
                            words[st * U * codec.word_cap:(st + 1) * U * codec.word_cap],
                            np.arange(U, dtype=np.uint64) * np.uint64(codec.word_cap),
                            u32(coded.n_words[st * U:(st + 1) * U]), 1, codec.N, chunk_syms=chunk)
        assert np.array_equal(dec, sym)
        rk, rv = O.reconstruct(dm, ck, cv, p, sym, ref32["esc_vals"], np.zeros(1, dtype=np.uint64), mode=O.F32)
        assert np.array_equal(u16(out_k[s, l, h]).ravel(), rk)
        assert np.array_equal(u16(out_v[s, l, h]).ravel(), rv)


@pytest.mark.parametrize("chunk", [0, 4096])
def test_properties_on_every_stream(run, chunk):
    w, out = run
    codec, coded, out_k, out_v = out[chunk]
    # decoder returns the encoder's symbols
    assert torch.equal(codec.dec_symbols, coded.symbols)
    # tables: sum to 4096, f > 0 exactly where the symbol occurs, counts add up to N
    freq = coded.freq.to(torch.int32) & 0xffff
    assert bool((freq.sum(1) == 4096).all())
    assert bool(((freq > 0) == (coded.counts > 0)).all())
    assert bool((coded.counts.to(torch.int64).sum(1) == codec.N).all())
    # escape offsets are the running sum of the counts
    cnt = coded.esc_cnt.to(torch.int64)
    assert torch.equal(coded.esc_off, torch.cumsum(cnt, 0) - cnt)
    # coded size: within a small margin of the empirical entropy of the symbols, per stream
    p = coded.counts.double() / codec.N
    H = -(torch.where(p > 0, p * torch.log2(p), torch.zeros_like(p))).sum(1)
    U = codec.units_per_stream
    bits = 16.0 * coded.n_words.double().reshape(-1, U).sum(1) + 32 * 32 * U
    excess = bits / codec.N - H
    assert float(excess.min()) > -1e-9 and float(excess.max()) < (0.03 if chunk == 0 else 0.3)
    # recovery error: at most Delta/2 plus half an fp16 ulp of the output; escapes exact
    esc = (coded.symbols.reshape(w.S, w.L, w.H, w.n, 2, w.d) == 255)
    delta = float(np.float32(w.delta))
    for c, (act, outp) in enumerate(((w.act_k, out_k), (w.act_v, out_v))):
        for l in range(w.L):
            a, o, e = act[0, l].float(), outp[0, l].float(), esc[0, l, :, :, c, :]
            err = (a - o).abs()
            ulp = torch.clamp(o.abs(), min=2.0 ** -14) * 2.0 ** -10          # >= one fp16 ulp of the output
            assert bool((err[~e] <= delta / 2 + ulp[~e] / 2 + 1e-6).all())
            assert torch.equal(act[0, l].view(torch.int16)[e], outp[0, l].view(torch.int16)[e])


# --------------------------------------------------------------------------- the other configurations, full size

OTHER = {
    # name: sampled streams
    "long": (0, 255),          # 8.4 M symbols per stream: stream length, 64-bit offsets (17 GB of candidates)
    "70b": (0, 5119),          # 5,120 streams (the paper's example dimensions)
    "batched": (0, 16383),     # 64 sessions with their own perplexity and noise, 16,384 streams, 137 GB of candidates
    "miss20": (0, 255),        # k = 20 candidates (43 bytes per component), 12 % of the positions are misses
}


@pytest.mark.parametrize("name", list(OTHER))
def test_other_configurations_full_size(oracle, name):
    """Encode + decode of a whole configuration on the GPU; sampled streams against the oracle bit for
    bit (symbols, escapes, table, rANS states and words, reconstruction), round trip on every stream."""
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    O = oracle
    dev = torch.device("cuda:0")
    free, _ = torch.cuda.mem_get_info()
    print(f"{name}: drawing inputs ({free / 2**30:.0f} GiB free)", flush=True)
    w = make_workload(name, device=dev)
    codec = codec_for(w, word_frac=0.625)              # 10 bits per symbol reserved; ~7.4 are used
    coded = codec.encode(w.cand_k, w.cand_v, w.probs, w.act_k, w.act_v)
    out_k, out_v = torch.empty_like(w.act_k), torch.empty_like(w.act_v)
    codec.decode(w.cand_k, w.cand_v, w.probs, out_k, out_v)
    codec.check_status(name)
    print(f"{name}: coded, checking", flush=True)
    assert torch.equal(codec.dec_symbols, coded.symbols)
    # every stream, not only the sampled ones: the single decode call (one kernel that also reconstructs where the
    # shape has one) against the two calls one after the other
    free, _ = torch.cuda.mem_get_info()
    if free > 2.2 * out_k.numel() * out_k.element_size() * 2:
        two_k, two_v = torch.zeros_like(w.act_k), torch.zeros_like(w.act_v)
        codec.dec_symbols.zero_()
        codec.decode(w.cand_k, w.cand_v, w.probs, two_k, two_v, fused=False)
        codec.check_status(name + ", two calls")
        assert torch.equal(codec.dec_symbols, coded.symbols)
        assert torch.equal(two_k.view(torch.int16), out_k.view(torch.int16))
        assert torch.equal(two_v.view(torch.int16), out_v.view(torch.int16))
        del two_k, two_v
        print(f"{name}: one call and two calls agree on every stream", flush=True)
    freq = coded.freq.to(torch.int32) & 0xffff
    assert bool((freq.sum(1) == 4096).all())
    cnt = coded.esc_cnt.to(torch.int64)
    assert torch.equal(coded.esc_off, torch.cumsum(cnt, 0) - cnt)
    dm = O.make_dims(1, 1, 1, w.n, w.k, w.d, w.delta, w.qmax)
    for st in OTHER[name]:
        (ck, cv, p, ak, av), (s, l, h) = _stream_inputs(w, st)
        ref = O.predict_residual(dm, ck, cv, p, ak, av, mode=O.F32)
        sym = u8(coded.symbols[st:st + 1])
        assert np.array_equal(sym, ref["symbols"]), f"{name} stream {st}"
        off, n_esc = int(u64(coded.esc_off)[st]), int(u32(coded.esc_cnt)[st])
        assert n_esc == int(ref["esc_cnt"][0])
        assert np.array_equal(u16(coded.esc_vals[off:off + n_esc]), ref["esc_vals"])
        fr, _ = O.build_freq(O.histogram(sym))
        assert np.array_equal(u16(coded.freq[st:st + 1]), fr)
        enc = O.rans_encode(sym, fr, word_cap_per_unit=codec.word_cap)
        nw = int(enc["n_words"][0])
        assert int(u32(coded.n_words[st:st + 1])[0]) == nw
        assert np.array_equal(u32(coded.states[st:st + 1]), enc["states"])
        assert np.array_equal(u16(coded.words[st * codec.word_cap:st * codec.word_cap + nw]), enc["words"][:nw])
        rk, rv = O.reconstruct(dm, ck, cv, p, sym, ref["esc_vals"], np.zeros(1, dtype=np.uint64), mode=O.F32)
        assert np.array_equal(u16(out_k[s, l, h]).ravel(), rk) and np.array_equal(u16(out_v[s, l, h]).ravel(), rv)
    del codec, coded, out_k, out_v, w
    torch.cuda.empty_cache()


# --------------------------------------------------------------------------- token-conditional path, full size

@pytest.mark.parametrize("name,chunk", [("llama8b", 0), ("llama8b", 4096), ("miss20", 0), ("70b", 0)])
def test_token_conditional_full_size(oracle, name, chunk):
    """The Llama-shaped configuration through the token-conditional path as bench.py runs it (true
    candidate given, whole streams or 4096-symbol units), and the 70B-shaped one (5120 streams with k = 4: the
    one-kernel decode in its form for many streams, five rounds of workgroups); one position in 16 is declared a
    miss so that both kinds of prediction occur.  Sampled streams bit for bit against the oracle, the index stream
    completely, properties on everything."""
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    O = oracle
    dev = torch.device("cuda:0")
    w = make_workload(name, device=dev)
    chosen = w.chosen.to(torch.int32).clone()          # miss20: already holds the generator's misses
    chosen[:, 5::16] = -1
    ch = chosen.cpu().numpy()
    codec = codec_for(w, chunk_syms=chunk)
    print(f"token-conditional {name}, chunk_syms={chunk}", flush=True)
    coded = codec.encode_cond(w.cand_k, w.cand_v, w.probs, w.act_k, w.act_v, chosen=chosen)
    out_k, out_v = torch.zeros_like(w.act_k), torch.zeros_like(w.act_v)
    codec.chosen.fill_(-7)
    codec.decode_cond(w.cand_k, w.cand_v, w.probs, out_k, out_v)
    codec.check_status("token-conditional, full size")
    assert np.array_equal(codec.dec_chosen.cpu().numpy(), ch)
    assert torch.equal(codec.dec_symbols, coded.symbols)
    two_k, two_v = torch.zeros_like(w.act_k), torch.zeros_like(w.act_v)      # the two calls, on every stream
    codec.dec_symbols.zero_()
    codec.decode_cond(w.cand_k, w.cand_v, w.probs, two_k, two_v, fused=False)
    codec.check_status("token-conditional, two calls")
    assert torch.equal(codec.dec_symbols, coded.symbols)
    assert torch.equal(two_k.view(torch.int16), out_k.view(torch.int16))
    assert torch.equal(two_v.view(torch.int16), out_v.view(torch.int16))
    del two_k, two_v
    probs = w.probs.cpu().numpy()
    ienc = O.index_encode(probs, ch, word_cap=codec.idx_word_cap)
    assert np.array_equal(u32(coded.idx_states), ienc["states"])
    assert np.array_equal(u32(coded.idx_n_words), ienc["n_words"])
    nw = int(ienc["n_words"][0])
    assert np.array_equal(u16(coded.idx_words)[:nw], ienc["words"][:nw])
    dm = O.make_dims(1, 1, 1, w.n, w.k, w.d, w.delta, w.qmax)
    U = codec.units_per_stream
    words = u16(coded.words)
    for st in (3, 200):
        print(f"  stream {st}", flush=True)
        (ck, cv, p, ak, av), (s, l, h) = _stream_inputs(w, st)
        ref = O.predict_residual(dm, ck, cv, p, ak, av, mode=O.F32, chosen=ch[s:s + 1])
        sym = u8(coded.symbols[st:st + 1])
        assert np.array_equal(sym, ref["symbols"])
        off, cnt = int(u64(coded.esc_off)[st]), int(u32(coded.esc_cnt)[st])
        assert cnt == int(ref["esc_cnt"][0])
        assert np.array_equal(u16(coded.esc_vals[off:off + cnt]), ref["esc_vals"])
        freq, _ = O.build_freq(O.histogram(sym))
        assert np.array_equal(u16(coded.freq[st:st + 1]), freq)
        enc = O.rans_encode(sym, freq, chunk_syms=chunk, word_cap_per_unit=codec.word_cap)
        assert np.array_equal(u32(coded.n_words[st * U:(st + 1) * U]), enc["n_words"])
        assert np.array_equal(u32(coded.states[st * U:(st + 1) * U]), enc["states"])
        for u in range(U):
            o, n_w = (st * U + u) * codec.word_cap, int(enc["n_words"][u])
            assert np.array_equal(words[o:o + n_w], enc["words"][u * codec.word_cap:u * codec.word_cap + n_w])
        rk, rv = O.reconstruct(dm, ck, cv, p, sym, ref["esc_vals"], np.zeros(1, dtype=np.uint64), mode=O.F32,
                               chosen=ch[s:s + 1])
        assert np.array_equal(u16(out_k[s, l, h]).ravel(), rk)
        assert np.array_equal(u16(out_v[s, l, h]).ravel(), rv)
    # recovery error on everything: at most Delta/2 plus half an fp16 ulp of the output; escapes exact
    esc = (coded.symbols.reshape(w.S, w.L, w.H, w.n, 2, w.d) == 255)
    delta = float(np.float32(w.delta))
    for c, (act, outp) in enumerate(((w.act_k, out_k), (w.act_v, out_v))):
        for l in range(w.L):
            a, o, e = act[0, l].float(), outp[0, l].float(), esc[0, l, :, :, c, :]
            ulp = torch.clamp(o.abs(), min=2.0 ** -14) * 2.0 ** -10
            assert bool(((a - o).abs()[~e] <= delta / 2 + ulp[~e] / 2 + 1e-6).all())
            assert torch.equal(act[0, l].view(torch.int16)[e], outp[0, l].view(torch.int16)[e])
    # positions given their token never escape; the misses do, at the weighted-mean path's rate
    by_pos = esc.any(dim=5).any(dim=4)[0].any(dim=0).any(dim=0).cpu().numpy()          # [n]
    assert not by_pos[ch[0] >= 0].any()
    del codec, coded, out_k, out_v, w
    torch.cuda.empty_cache()


# --------------------------------------------------------------------------- surprisal-adaptive path, full size

def test_surprisal_adaptive_full_size(oracle):
    """The Llama-shaped configuration through the adaptive path exactly as bench.py runs it (b0 = 3, hbar =
    log2 of the perplexity, range 0.32, whole streams).  Bit depths completely, sampled streams bit for bit
    against the oracle (symbols, per-depth tables, rANS states and words, reconstruction), properties on all."""
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    O = oracle
    from paper_2604_15356_amd import plc
    dev = torch.device("cuda:0")
    w = make_workload("llama8b", device=dev)
    chosen = w.chosen.to(torch.int32).contiguous()
    ch = chosen.cpu().numpy()
    hbar = float(np.log2(np.mean(w.perplexity)))
    thr = plc.plc_surprisal_thresholds(3.0, hbar)
    thr_oracle = O.surprisal_thresholds(3.0, hbar)            # the oracle's own, from its own arithmetic
    assert list(thr) == list(thr_oracle)
    step_range = 0.32
    codec = codec_for(w)
    print("surprisal-adaptive llama8b", flush=True)
    coded = codec.encode_adapt(w.cand_k, w.cand_v, w.probs, w.act_k, w.act_v, chosen, thr, step_range)
    out_k, out_v = torch.zeros_like(w.act_k), torch.zeros_like(w.act_v)
    codec.bits.fill_(9)
    codec.decode_adapt(w.cand_k, w.cand_v, w.probs, out_k, out_v, thr, step_range)
    codec.check_status("surprisal-adaptive, full size")
    probs = w.probs.cpu().numpy()
    bits = O.surprisal_bits(probs, ch, thr_oracle)
    assert np.array_equal(codec.dec_bits.cpu().numpy(), bits)
    assert torch.equal(codec.dec_symbols, coded.symbols)
    two_k, two_v = torch.zeros_like(w.act_k), torch.zeros_like(w.act_v)      # the two calls, on every stream
    codec.dec_symbols.zero_()
    codec.decode_adapt(w.cand_k, w.cand_v, w.probs, two_k, two_v, thr, step_range, fused=False)
    codec.check_status("surprisal-adaptive, two calls")
    assert torch.equal(codec.dec_symbols, coded.symbols)
    assert torch.equal(two_k.view(torch.int16), out_k.view(torch.int16))
    assert torch.equal(two_v.view(torch.int16), out_v.view(torch.int16))
    del two_k, two_v
    dm = O.make_dims(1, 1, 1, w.n, w.k, w.d, w.delta, w.qmax)
    spp, B = 2 * w.d, plc.MAX_BITS
    words = u16(coded.words)
    for st in (17, 254):
        print(f"  stream {st}", flush=True)
        (ck, cv, p, ak, av), (s, l, h) = _stream_inputs(w, st)
        ref = O.predict_residual(dm, ck, cv, p, ak, av, mode=O.F32, chosen=ch[s:s + 1], bits=bits[s:s + 1],
                                 step_range=step_range)
        sym = u8(coded.symbols[st:st + 1])
        assert np.array_equal(sym, ref["symbols"])
        counts = O.histogram_bucketed(sym, spp, 1, bits[s:s + 1], n_tables=B)
        freq = O.build_freq_sparse(counts)
        assert np.array_equal(u32(coded.counts_d[st:st + 1]), counts)
        assert np.array_equal(u16(coded.freq_d[st:st + 1]), freq)
        enc = O.rans_encode_bucketed(sym, freq, spp, 1, bits[s:s + 1], word_cap_per_unit=codec.word_cap)
        nw = int(enc["n_words"][0])
        assert int(u32(coded.n_words[st:st + 1])[0]) == nw
        assert np.array_equal(u32(coded.states[st:st + 1]), enc["states"])
        assert np.array_equal(words[st * codec.word_cap:st * codec.word_cap + nw], enc["words"][:nw])
        rk, rv = O.reconstruct(dm, ck, cv, p, sym, ref["esc_vals"], np.zeros(1, dtype=np.uint64), mode=O.F32,
                               chosen=ch[s:s + 1], bits=bits[s:s + 1], step_range=step_range)
        assert np.array_equal(u16(out_k[s, l, h]).ravel(), rk) and np.array_equal(u16(out_v[s, l, h]).ravel(), rv)
    # error at most half the position's own step, everywhere
    step = torch.from_numpy(np.float32(step_range) * 2.0 ** -bits[0].astype(np.float32)).to(dev)[None, :, None]
    esc = (coded.symbols.reshape(w.S, w.L, w.H, w.n, 2, w.d) == 255)
    for c, (act, outp) in enumerate(((w.act_k, out_k), (w.act_v, out_v))):
        for l in range(w.L):
            a, o, e = act[0, l].float(), outp[0, l].float(), esc[0, l, :, :, c, :]
            ulp = torch.clamp(o.abs(), min=2.0 ** -14) * 2.0 ** -10
            assert bool((((a - o).abs() <= step / 2 + ulp / 2 + 1e-6) | e).all())
    del codec, coded, out_k, out_v, w
    torch.cuda.empty_cache()


# --------------------------------------------------------------------------- linear-embedding predictor, full size

def test_linear_predictor_full_size(oracle):
    """The linear predictor at the size bench.py times it (m = 4096, V = 50,016).  The oracle recomputes sampled
    rows of the expected embedding and sampled (layer, head, K/V, position) rows of the prediction from the
    device's expected embedding; symbols may differ only by one step at rounding near-ties; round trip and
    error bound on everything."""
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    from paper_2604_15356_amd.codec import KVDeltaCodec
    from paper_2604_15356_amd.workloads import make_linear_workload
    dev = torch.device("cuda:0")
    print("linear predictor llama8b: drawing inputs", flush=True)
    w = make_linear_workload("llama8b", device=dev)
    codec = KVDeltaCodec(w.S, w.L, w.H, w.n, 1, w.d, w.delta, w.qmax, device=dev)
    coded = codec.encode_linear(w.probs_full, w.embed_t, w.A, w.bias_k, w.bias_v, w.act_k, w.act_v)
    out_k, out_v = torch.zeros_like(w.act_k), torch.zeros_like(w.act_v)
    codec.decode_linear(w.probs_full, w.embed_t, w.A, w.bias_k, w.bias_v, out_k, out_v)
    codec.check_status("linear predictor, full size")
    assert torch.equal(codec.dec_symbols, coded.symbols)
    from oracle import plc_oracle_linear as OL
    rng = np.random.default_rng(5)
    # expected embedding: sampled rows through the oracle
    rows = np.sort(rng.integers(0, w.S * w.n, 6))
    want_rows = OL.expected_embedding(w.probs_full[rows].cpu().numpy(), w.embed_t.cpu().numpy())
    for r, want in zip(rows, want_rows):
        got = codec.ebar[r].cpu().numpy()
        ulp = np.spacing(np.maximum(np.abs(want), np.float16(2.0 ** -14))).astype(np.float64)
        assert (np.abs(got.astype(np.float64) - want.astype(np.float64)) <= ulp).all()
        assert (got.view(np.uint16) != want.view(np.uint16)).mean() < 0.05
    # prediction / symbols / reconstruction: sampled (layer, head, position) through the oracle, which is fed the
    # device's expected embedding (the matrix cores add in their own order: no bit-exact mirror of Ebar)
    sym = coded.symbols.reshape(w.S, w.L, w.H, w.n, 2, w.d)
    delta = float(np.float32(w.delta))
    n_diff = 0
    for _ in range(48):
        l, h, i = int(rng.integers(w.L)), int(rng.integers(w.H)), int(rng.integers(w.n))
        cut = lambda t: t[0:1, l:l + 1, h:h + 1, i:i + 1].cpu().numpy()              # [1, 1, 1, 1, d]
        eb = codec.ebar[i].cpu().numpy().reshape(1, 1, w.m)
        A = w.A[l:l + 1, h:h + 1].cpu().numpy()                                       # [1, 1, 2, d, m]
        ref = OL.predict_residual(eb, A, cut(w.bias_k), cut(w.bias_v), cut(w.act_k), cut(w.act_v), w.delta)
        want = ref["symbols"].reshape(2, w.d).astype(np.int64)
        u = ref["u"].reshape(2, w.d)
        got = sym[0, l, h, i].cpu().numpy().astype(np.int64)                           # [2, d]
        # fp32 accumulation bound of each component's sum, in steps of Delta
        mag = np.abs(A[0, 0].astype(np.float64)) @ np.abs(eb[0, 0].astype(np.float64))  # [2, d]
        tau = (w.m + 4) * 2.0 ** -24 * (mag + 8.0) / delta
        differ = got != want
        near = np.abs(u - np.floor(u) - 0.5) < tau
        one = (np.abs(got - want) == 1) | (got == 255) | (want == 255)
        assert (differ <= (near & one)).all()
        n_diff += int(differ.sum())
        # the oracle's reconstruction from the device's symbols (escapes: the actual values, as the lists hold them)
        act2 = np.stack([cut(w.act_k).reshape(w.d), cut(w.act_v).reshape(w.d)]).view(np.uint16)
        rk, rv = OL.reconstruct(eb, A, cut(w.bias_k), cut(w.bias_v), got.astype(np.uint8).reshape(1, 2 * w.d),
                                act2[got == 255], w.delta)
        for c, (outp, want_out) in enumerate(((out_k, rk), (out_v, rv))):
            out = outp[0, l, h, i].cpu().numpy()
            wo = want_out.reshape(w.d)
            keep = got[c] != 255
            ulp = np.maximum(np.abs(wo.astype(np.float64)), 2.0 ** -14) * 2.0 ** -10
            # one fp16 step of the output plus the fp32 accumulation bound of the prediction
            assert (np.abs(out.astype(np.float64) - wo.astype(np.float64)) <= ulp + tau[c] * delta)[keep].all()
            assert np.array_equal(out.view(np.uint16)[~keep], wo.view(np.uint16)[~keep])
    print(f"  near-ties on sampled rows: {n_diff} of {48 * 2 * w.d}", flush=True)
    assert n_diff <= 3
    # error bound on everything
    esc = sym == 255
    for c, (act, outp) in enumerate(((w.act_k, out_k), (w.act_v, out_v))):
        for l in range(w.L):
            a, o, e = act[0, l].float(), outp[0, l].float(), esc[0, l, :, :, c, :]
            ulp = torch.clamp(o.abs(), min=2.0 ** -14) * 2.0 ** -10
            assert bool((((a - o).abs() <= delta / 2 + ulp + 1e-4) | e).all())
            assert torch.equal(act[0, l].view(torch.int16)[e], outp[0, l].view(torch.int16)[e])
    del codec, coded, out_k, out_v, w
    torch.cuda.empty_cache()
