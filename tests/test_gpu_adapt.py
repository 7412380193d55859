"""Parity of the surprisal-adaptive quantiser path (through the C ABI of libplc.so)
against the CPU oracle, element by element, on the same seeded inputs: bit
depths, symbols, escapes, per-depth histograms and tables, rANS states and
words, and the reconstruction -- all bit-exact against the oracle in the
kernel's precision; the decode direction starts from the coded artefacts alone
(index stream -> tokens -> bit depths -> per-depth tables)."""
import numpy as np
import pytest
import torch

from paper_2604_15356_amd.workloads import make_workload, random_bytes
from tests.gpu_util import codec_for, near_tie_report, oracle_dims, storage_np, u8, u16, u32, u64

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dev():
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    from paper_2604_15356_amd import plc
    plc.lib()
    return torch.device("cuda:0")


CASES = {
    # name: (config, overrides, layout, random rows, chunk_syms, b0, hbar, range)
    "tiny": ("tiny", None, "lhnkd", False, 0, 3.0, np.log2(12.0), 0.32),
    "tiny_chunked": ("tiny", None, "lhnkd", True, 1024, 3.0, np.log2(12.0), 0.32),
    "heads_inner": ("tiny", dict(seed=41), "lnkhd", True, 0, 2.0, 3.0, 0.16),
    "k8_d128": ("llama8b", dict(L=2, H=2, n=300, seed=42), "lhnkd", False, 0, 3.0, np.log2(15.0), 0.32),
    "k8_d128_chunked": ("llama8b", dict(L=2, H=2, n=300, seed=43), "lhnkd", True, 4096, 3.0, np.log2(15.0), 0.32),
    "d16_three_sessions": ("tiny", dict(S=3, L=1, H=2, n=70, d=16, k=5, seed=44), "lhnkd", True, 0, 3.0, 3.5, 0.64),
    "d48_ragged_chunks": ("tiny", dict(S=2, L=2, H=1, n=37, d=48, k=3, seed=45), "lnkhd", True, 992, 2.5, 3.0, 0.32),
    "k20_with_misses": ("miss20", dict(L=1, H=2, n=300, seed=46), "lhnkd", False, 0, 3.0, np.log2(15.0), 0.64),
    "nine_waves_of_units": ("tiny", dict(L=1, H=1, n=400, seed=47), "lhnkd", True, 2048, 3.0, 3.5, 0.32),
}


@pytest.mark.parametrize("case", list(CASES))
def test_adaptive_encode_decode_matches_oracle(oracle, dev, case):
    O = oracle
    from paper_2604_15356_amd import plc
    name, overrides, layout, random_rows, chunk, b0, hbar, step_range = CASES[case]
    w = make_workload(name, device=dev, layout=layout, overrides=overrides, random_rows=random_rows)
    chosen = w.chosen.to(torch.int32).clone()
    chosen[:, 3::11] = -1                                   # some declared misses on top of the generator's
    ch = chosen.cpu().numpy()
    thr = plc.plc_surprisal_thresholds(b0, hbar)
    thr_oracle = O.surprisal_thresholds(b0, hbar)
    assert list(thr) == list(thr_oracle)
    codec = codec_for(w, want_pred=True, esc_frac=1.0, chunk_syms=chunk)
    print(f"case {case}: S{w.S} L{w.L} H{w.H} n{w.n} k{w.k} d{w.d} chunk {chunk} thr {thr}", flush=True)
    coded = codec.encode_adapt(w.cand_k, w.cand_v, w.probs, w.act_k, w.act_v, chosen, thr, step_range)
    codec.check_status("encode_adapt")
    probs = w.probs.cpu().numpy()
    spp, sps, B = 2 * w.d, w.L * w.H, plc.MAX_BITS

    # ---- bit depths
    bits = O.surprisal_bits(probs, ch, thr_oracle)
    assert np.array_equal(coded.bits.cpu().numpy(), bits)
    assert len(set(bits.ravel())) >= 2                      # the case really mixes depths

    # ---- floating-point part
    args = (oracle_dims(O, w), storage_np(w.cand_k), storage_np(w.cand_v), probs, storage_np(w.act_k),
            storage_np(w.act_v))
    ref32 = O.predict_residual(*args, mode=O.F32, chosen=ch, bits=bits, step_range=step_range)
    ref64 = O.predict_residual(*args, mode=O.F64, chosen=ch, bits=bits, step_range=step_range, want_u=True)
    sym = u8(coded.symbols)
    assert np.array_equal(sym, ref32["symbols"]), "symbols differ from the strict-fp32 oracle"
    tau = 64 * 2.0 ** -24 * 8.0 / (float(np.float32(step_range)) / 16)
    n_diff, n_ok = near_tie_report(sym, ref64["symbols"], ref64["u"], tau)
    assert n_diff == n_ok and n_diff <= max(3, 1e-4 * sym.size)
    total = int(ref32["esc_cnt"].sum())
    assert np.array_equal(u32(coded.esc_cnt), ref32["esc_cnt"])
    assert np.array_equal(u16(coded.esc_vals)[:total], ref32["esc_vals"])

    # ---- statistics and coder per depth, bit-exact given identical symbols
    counts = O.histogram_bucketed(sym, spp, sps, bits, n_tables=B)
    freq = O.build_freq_sparse(counts)
    assert np.array_equal(u32(coded.counts_d), counts)
    assert np.array_equal(u16(coded.freq_d), freq)
    enc = O.rans_encode_bucketed(sym, freq, spp, sps, bits, chunk_syms=chunk, word_cap_per_unit=codec.word_cap)
    assert np.array_equal(u32(coded.n_words), enc["n_words"])
    assert np.array_equal(u32(coded.states), enc["states"])
    words = u16(coded.words)
    for unit in range(codec.n_units):
        off, nw = unit * codec.word_cap, int(enc["n_words"][unit])
        assert np.array_equal(words[off:off + nw], enc["words"][off:off + nw]), f"unit {unit}"
    dec = O.rans_decode_bucketed(freq, u32(coded.states), words, u64(coded.word_off), u32(coded.n_words),
                                 codec.n_streams, codec.N, spp, sps, bits, chunk_syms=chunk)
    assert np.array_equal(dec, sym)

    # ---- decode direction on the GPU, from the coded artefacts alone
    codec.chosen.fill_(-7)
    codec.bits.fill_(9)
    out_k, out_v = torch.zeros_like(w.act_k), torch.zeros_like(w.act_v)
    codec.decode_adapt(w.cand_k, w.cand_v, w.probs, out_k, out_v, thr, step_range)
    codec.check_status("decode_adapt")
    assert np.array_equal(codec.dec_chosen.cpu().numpy(), ch)
    assert np.array_equal(codec.dec_bits.cpu().numpy(), bits)
    assert torch.equal(codec.dec_symbols, coded.symbols)
    rk, rv = O.reconstruct(oracle_dims(O, w), storage_np(w.cand_k), storage_np(w.cand_v), probs, sym,
                           ref32["esc_vals"], ref32["esc_off"], mode=O.F32, chosen=ch, bits=bits,
                           step_range=step_range)
    assert np.array_equal(u16(out_k).ravel(), rk) and np.array_equal(u16(out_v).ravel(), rv)
    # decode_adapt() ends in the single call that reconstructs inside the entropy decoder where the shape
    # allows it; the two calls one after the other must give the same bits
    two_k, two_v = torch.zeros_like(w.act_k), torch.zeros_like(w.act_v)
    codec.dec_symbols.zero_()
    codec.decode_adapt(w.cand_k, w.cand_v, w.probs, two_k, two_v, thr, step_range, fused=False)
    codec.check_status("decode_adapt in two calls")
    assert torch.equal(codec.dec_symbols, coded.symbols)
    assert np.array_equal(u16(two_k), u16(out_k)) and np.array_equal(u16(two_v), u16(out_v))
    # recovery error: half the position's own step (+ half an fp16 ulp of the output); escapes exact
    esc = sym.reshape(codec.n_streams, w.n, 2, w.d) == 255
    step = float(np.float32(step_range)) * 2.0 ** -bits.astype(np.float64)                  # [S, n]
    step = np.repeat(step[:, None, :], sps, axis=1).reshape(codec.n_streams, w.n, 1)
    for c, (act, out) in enumerate(((w.act_k, out_k), (w.act_v, out_v))):
        a = act.reshape(codec.n_streams, w.n, w.d).cpu().numpy().astype(np.float64)
        o = out.reshape(codec.n_streams, w.n, w.d).cpu().numpy().astype(np.float64)
        e = esc[:, :, c, :]
        ulp = np.maximum(np.abs(o), 2.0 ** -14) * 2.0 ** -10
        assert (np.abs(a - o) <= step / 2 + ulp / 2 + 1e-6)[~e].all()
        assert np.array_equal(u16(act).reshape(codec.n_streams, w.n, w.d)[e],
                              u16(out).reshape(codec.n_streams, w.n, w.d)[e])


def test_bucketed_byte_streams_bit_exact(oracle, dev):
    """The per-depth histogram / table / rANS calls on plain byte streams, many streams and units."""
    O = oracle
    from paper_2604_15356_amd import plc
    rng = np.random.default_rng(12)
    S, sps, n, spp = 5, 7, 130, 64
    n_streams, N = S * sps, n * spp
    bits_np = rng.integers(1, 5, (S, n)).astype(np.uint8)
    bits_np[2] = 2                                            # a session with a single depth
    width = 2.0 * 2.0 ** np.repeat(bits_np, spp, axis=1)
    sym_np = np.empty((n_streams, N), dtype=np.uint8)
    for st in range(n_streams):
        sym_np[st] = np.clip(np.round(rng.standard_normal(N) * width[st // sps] + 127), 0, 254)
    sym = torch.from_numpy(sym_np).to(dev)
    bits = torch.from_numpy(bits_np).to(dev)
    B = plc.MAX_BITS
    status = torch.zeros(1, dtype=torch.int32, device=dev)
    counts = torch.empty((n_streams, B, 256), dtype=torch.int32, device=dev)
    freq = torch.empty((n_streams, B, 256), dtype=torch.int16, device=dev)
    plc.plc_histogram_bucketed(sym, n_streams, N, spp, sps, bits, B, counts, status)
    plc.plc_build_freq_bucketed(counts, n_streams, B, freq, status)
    ref_counts = O.histogram_bucketed(sym_np, spp, sps, bits_np, n_tables=B)
    ref_freq = O.build_freq_sparse(ref_counts)
    assert np.array_equal(u32(counts), ref_counts) and np.array_equal(u16(freq), ref_freq)
    for chunk in (0, 2048, 64):
        U = plc.plc_units_per_stream(N, chunk)
        cap = ((chunk or N) + 7) // 8 * 8
        nu = n_streams * U
        states = torch.empty((nu, 32), dtype=torch.int32, device=dev)
        words = torch.zeros(nu * cap, dtype=torch.int16, device=dev)
        woff = torch.arange(nu, dtype=torch.int64, device=dev) * cap
        nw = torch.empty(nu, dtype=torch.int32, device=dev)
        dec = torch.zeros_like(sym)
        print(f"  chunk {chunk}: {nu} units", flush=True)
        plc.plc_rans_encode_bucketed(sym, n_streams, N, chunk, spp, sps, bits, B, freq, states, words, woff, cap, nw,
                                     status)
        plc.plc_rans_decode_bucketed(freq, states, words, woff, nw, n_streams, N, chunk, spp, sps, bits, B, dec,
                                     status)
        assert int(status.item()) == 0
        assert torch.equal(dec, sym)
        enc = O.rans_encode_bucketed(sym_np, ref_freq, spp, sps, bits_np, chunk_syms=chunk, word_cap_per_unit=cap)
        assert np.array_equal(u32(nw), enc["n_words"]) and np.array_equal(u32(states), enc["states"])
        wd = u16(words)
        for unit in range(nu):
            o, k_ = unit * cap, int(enc["n_words"][unit])
            assert np.array_equal(wd[o:o + k_], enc["words"][o:o + k_]), f"unit {unit}"
        if chunk == 0:
            # The chain decoder with a ring per depth: a damaged word, then a damaged state, are reported (the
            # walk ends at the stream's length whatever it reads); an undamaged decode after them is exact again.
            words[woff[3] + 5] ^= 0x0a51
            plc.plc_rans_decode_bucketed(freq, states, words, woff, nw, n_streams, N, chunk, spp, sps, bits, B, dec,
                                         status)
            assert int(status.item()) == plc.PLC_ERR_CORRUPT
            words[woff[3] + 5] ^= 0x0a51
            status.zero_()
            states[11, 7] ^= 0x00010400
            plc.plc_rans_decode_bucketed(freq, states, words, woff, nw, n_streams, N, chunk, spp, sps, bits, B, dec,
                                         status)
            assert int(status.item()) == plc.PLC_ERR_CORRUPT
            states[11, 7] ^= 0x00010400
            status.zero_()
            dec.zero_()
            plc.plc_rans_decode_bucketed(freq, states, words, woff, nw, n_streams, N, chunk, spp, sps, bits, B, dec,
                                         status)
            assert int(status.item()) == 0 and torch.equal(dec, sym)
    # a depth outside 1..n_tables is reported and nothing faults
    bad = bits.clone()
    bad[0, 5] = 7
    plc.plc_histogram_bucketed(sym, n_streams, N, spp, sps, bad, B, counts, status)
    assert int(status.item()) == plc.PLC_ERR_INVALID


def test_bucketed_more_whole_streams_than_the_chain_decoder_takes(oracle, dev):
    """Whole-stream units beyond the bound of the per-depth chain decoder: the many-unit kernels, one
    wavefront per workgroup, with their split per-depth tables."""
    O = oracle
    from paper_2604_15356_amd import plc
    rng = np.random.default_rng(13)
    S, sps, n, spp = 41, 16, 21, 64                           # 656 streams of 1344 symbols
    n_streams, N = S * sps, n * spp
    bits_np = rng.integers(1, 5, (S, n)).astype(np.uint8)
    bits_np[7] = 3                                            # a session with a single depth
    bits_np[8, :] = np.where(np.arange(n) % 2 == 0, 1, 4)     # and one without the middle depths
    width = 1.5 * 2.0 ** np.repeat(bits_np, spp, axis=1)
    sym_np = np.empty((n_streams, N), dtype=np.uint8)
    for st in range(n_streams):
        sym_np[st] = np.clip(np.round(rng.standard_normal(N) * width[st // sps] + 127), 0, 254)
    sym_np[5, ::97] = 255
    sym = torch.from_numpy(sym_np).to(dev)
    bits = torch.from_numpy(bits_np).to(dev)
    B = plc.MAX_BITS
    status = torch.zeros(1, dtype=torch.int32, device=dev)
    counts = torch.empty((n_streams, B, 256), dtype=torch.int32, device=dev)
    freq = torch.empty((n_streams, B, 256), dtype=torch.int16, device=dev)
    plc.plc_histogram_bucketed(sym, n_streams, N, spp, sps, bits, B, counts, status)
    plc.plc_build_freq_bucketed(counts, n_streams, B, freq, status)
    ref_freq = O.build_freq_sparse(O.histogram_bucketed(sym_np, spp, sps, bits_np, n_tables=B))
    assert np.array_equal(u16(freq), ref_freq)
    cap = (N + 7) // 8 * 8
    states = torch.empty((n_streams, 32), dtype=torch.int32, device=dev)
    words = torch.zeros(n_streams * cap, dtype=torch.int16, device=dev)
    woff = torch.arange(n_streams, dtype=torch.int64, device=dev) * cap
    nw = torch.empty(n_streams, dtype=torch.int32, device=dev)
    dec = torch.zeros_like(sym)
    print(f"  {n_streams} whole-stream units", flush=True)
    plc.plc_rans_encode_bucketed(sym, n_streams, N, 0, spp, sps, bits, B, freq, states, words, woff, cap, nw, status)
    plc.plc_rans_decode_bucketed(freq, states, words, woff, nw, n_streams, N, 0, spp, sps, bits, B, dec, status)
    assert int(status.item()) == 0
    assert torch.equal(dec, sym)
    enc = O.rans_encode_bucketed(sym_np, ref_freq, spp, sps, bits_np, chunk_syms=0, word_cap_per_unit=cap)
    assert np.array_equal(u32(nw), enc["n_words"]) and np.array_equal(u32(states), enc["states"])
    wd = u16(words)
    for unit in range(n_streams):
        o, k_ = unit * cap, int(enc["n_words"][unit])
        assert np.array_equal(wd[o:o + k_], enc["words"][o:o + k_]), f"unit {unit}"
    # a damaged word list is reported, and decoding ends
    words[woff[300] + 3] ^= 0x1555
    plc.plc_rans_decode_bucketed(freq, states, words, woff, nw, n_streams, N, 0, spp, sps, bits, B, dec, status)
    assert int(status.item()) == plc.PLC_ERR_CORRUPT
