"""Parity of the HIP path (through the C ABI of libplc.so) against the CPU
oracle, element by element, on the same seeded inputs.

Bars: symbols, escape lists, histograms, tables, rANS states and words are
bit-exact against the oracle evaluated in the kernel's precision (strict
fp32); against the fp64 oracle, predictions agree to 1e-3 relative (in fact
~1e-6) and symbols may differ only at rounding near-ties, which are counted.
Streams written by either side decode on the other.
"""
import numpy as np
import pytest
import torch

from paper_2604_15356_amd.workloads import make_workload, random_bytes
from tests.gpu_util import (codec_for, near_tie_report, oracle_dims, storage_np, u8, u16, u32, u64)

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dev():
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    from paper_2604_15356_amd import plc
    plc.lib()            # raises if libplc.so is missing: there is no fallback
    return torch.device("cuda:0")


CASES = {
    # name: (config, overrides, layout, random probability rows)
    "tiny": ("tiny", None, "lhnkd", False),
    "tiny_heads_inner": ("tiny", None, "lnkhd", True),
    "ragged_k5_d24": ("tiny", dict(S=2, L=2, H=3, n=37, k=5, d=24, seed=11), "lhnkd", True),
    "ragged_k5_d24_heads_inner": ("tiny", dict(S=2, L=2, H=3, n=37, k=5, d=24, seed=12), "lnkhd", True),
    "k1": ("tiny", dict(k=1, n=100, seed=13), "lhnkd", False),
    "k8_d128": ("llama8b", dict(L=2, H=2, n=300, seed=14), "lhnkd", True),
    "k11_runtime_loop": ("tiny", dict(k=11, n=129, d=40, seed=15), "lhnkd", True),
    "k20": ("tiny", dict(k=20, L=1, H=2, n=65, d=128, seed=16), "lhnkd", True),
    "one_position": ("tiny", dict(L=1, H=1, n=1, d=8, seed=17), "lhnkd", False),
    # so many escapes that tiles overflow their staging rows and take the re-gather path
    "escape_heavy": ("tiny", dict(L=1, H=2, n=300, sigma=3.0, seed=18), "lhnkd", False),
    "escape_heavy_ragged": ("tiny", dict(L=1, H=3, n=37, k=5, d=24, sigma=2.0, seed=19), "lnkhd", True),
    # k = 20 with positions whose true vector is none of the candidates
    "k20_with_misses": ("miss20", dict(L=1, H=2, n=300, seed=20), "lhnkd", False),
    # rows longer than a batch of the decoder that reconstructs (64 chunks), and as long as one
    "wide_rows_d1024_k3": ("tiny", dict(L=1, H=2, n=9, k=3, d=1024, seed=21), "lhnkd", True),
    "rows_of_a_batch_d512_k7": ("tiny", dict(L=1, H=1, n=33, k=7, d=512, seed=22), "lnkhd", True),
    "two_sessions_k6": ("tiny", dict(S=2, L=3, H=1, n=130, k=6, d=64, sigma=0.5, seed=23), "lhnkd", True),
    # more streams than the whole-stream encoder and decoder kernels take (1024): the many-unit kernels with one
    # wavefront per workgroup code them, and the one-kernel decode runs in several rounds of workgroups
    "many_streams": ("tiny", dict(S=2, L=20, H=32, n=9, k=4, d=24, seed=24), "lhnkd", True),
    # more than 512 streams with k <= 4: the one-kernel decode takes the form with 4-byte entries, four workgroups
    # per compute unit; these streams wrap its word ring ten times, from word lists at changing offsets inside a
    # 1 KiB line; escapes are frequent enough that chunks with more than two of them occur
    "dense_streams_k3": ("tiny", dict(S=1, L=20, H=30, n=161, k=3, d=64, sigma=0.9, seed=25), "lhnkd", True),
    # the same with k = 6: the 8-byte entries on a three-block word ring, three workgroups per compute unit
    "dense_streams_k6": ("tiny", dict(S=1, L=20, H=30, n=161, k=6, d=64, sigma=0.9, seed=26), "lhnkd", True),
}


def _oracle_encode(O, w, mode, **kw):
    return O.predict_residual(oracle_dims(O, w), storage_np(w.cand_k), storage_np(w.cand_v),
                              w.probs.cpu().numpy(), storage_np(w.act_k), storage_np(w.act_v),
                              mode=mode, **kw)


@pytest.mark.parametrize("case", list(CASES))
def test_encode_decode_matches_oracle(oracle, dev, case):
    O = oracle
    name, overrides, layout, random_rows = CASES[case]
    w = make_workload(name, device=dev, layout=layout, overrides=overrides, random_rows=random_rows)
    codec = codec_for(w, want_pred=True, esc_frac=1.0)
    print(f"case {case}: S{w.S} L{w.L} H{w.H} n{w.n} k{w.k} d{w.d} layout {layout}", flush=True)
    coded = codec.encode(w.cand_k, w.cand_v, w.probs, w.act_k, w.act_v)
    codec.check_status("encode")

    # ---- floating-point part
    ref32 = _oracle_encode(O, w, O.F32)
    ref64 = _oracle_encode(O, w, O.F64, want_pred=True, want_u=True)
    sym = u8(coded.symbols)
    assert np.array_equal(sym, ref32["symbols"]), "symbols differ from the strict-fp32 oracle"
    pred = codec.pred.cpu().numpy().astype(np.float64)
    scale = np.maximum(np.abs(ref64["pred"]), 1e-2)
    assert (np.abs(pred - ref64["pred"]) / scale).max() < 1e-3
    tau = 64 * 2.0 ** -24 * 8.0 / float(np.float32(w.delta))
    n_diff, n_ok = near_tie_report(sym, ref64["symbols"], ref64["u"], tau)
    print(f"  near-ties vs fp64 oracle: {n_diff} of {sym.size} ({n_diff / sym.size:.2e})", flush=True)
    assert n_diff == n_ok and n_diff <= max(3, 1e-4 * sym.size)
    total = int(ref32["esc_cnt"].sum())
    assert np.array_equal(u32(coded.esc_cnt), ref32["esc_cnt"])
    assert np.array_equal(u64(coded.esc_off), ref32["esc_off"])
    assert np.array_equal(u16(coded.esc_vals)[:total], ref32["esc_vals"])

    # ---- integer part, bit-exact given identical symbols
    counts = O.histogram(sym)
    freq, cum = O.build_freq(counts)
    enc = O.rans_encode(sym, freq, word_cap_per_unit=codec.word_cap)
    assert np.array_equal(u32(coded.counts), counts)
    assert np.array_equal(u16(coded.freq), freq)
    assert np.array_equal(u16(coded.cum), cum)
    assert np.array_equal(u32(coded.n_words), enc["n_words"])
    assert np.array_equal(u32(coded.states), enc["states"])
    words = u16(coded.words)
    for unit in range(codec.n_units):
        off, nw = unit * codec.word_cap, int(enc["n_words"][unit])
        assert np.array_equal(words[off:off + nw], enc["words"][off:off + nw]), f"unit {unit}"
    # the oracle decodes the GPU's stream
    dec = O.rans_decode(u16(coded.freq), u32(coded.states), words, u64(coded.word_off),
                        u32(coded.n_words), codec.n_streams, codec.N)
    assert np.array_equal(dec, sym)

    # ---- decode direction on the GPU
    out_k = torch.zeros_like(w.act_k)
    out_v = torch.zeros_like(w.act_v)
    codec.decode(w.cand_k, w.cand_v, w.probs, out_k, out_v)
    codec.check_status("decode")
    assert torch.equal(codec.dec_symbols, coded.symbols)
    rk32, rv32 = O.reconstruct(oracle_dims(O, w), storage_np(w.cand_k), storage_np(w.cand_v),
                               w.probs.cpu().numpy(), sym, ref32["esc_vals"], ref32["esc_off"], mode=O.F32)
    assert np.array_equal(u16(out_k).ravel(), rk32) and np.array_equal(u16(out_v).ravel(), rv32)
    # decode() is the single call that reconstructs inside the entropy decoder where the shape allows it;
    # the two calls one after the other must give the same bits
    two_k, two_v = torch.zeros_like(w.act_k), torch.zeros_like(w.act_v)
    codec.dec_symbols.zero_()
    codec.decode(w.cand_k, w.cand_v, w.probs, two_k, two_v, fused=False)
    codec.check_status("decode in two calls")
    assert torch.equal(codec.dec_symbols, coded.symbols)
    assert np.array_equal(u16(two_k), u16(out_k)) and np.array_equal(u16(two_v), u16(out_v))
    rk64, rv64 = O.reconstruct(oracle_dims(O, w), storage_np(w.cand_k), storage_np(w.cand_v),
                               w.probs.cpu().numpy(), sym, ref32["esc_vals"], ref32["esc_off"], mode=O.F64)
    for got, want in ((u16(out_k).ravel(), rk64), (u16(out_v).ravel(), rv64)):
        g = got.view(np.float16).astype(np.float64)
        r = want.view(np.float16).astype(np.float64)
        fin = np.isfinite(g) & np.isfinite(r)
        assert np.array_equal(got[~fin], want[~fin])
        ulp = np.spacing(np.maximum(np.abs(g), np.abs(r)).astype(np.float16)).astype(np.float64)
        # the neighbouring fp16 value at most; near zero (cancellation) the fp32 evaluation error of
        # the sum, ~1e-7 absolute, spans more than one fp16 subnormal step
        assert (np.abs(g - r)[fin] <= ulp[fin] + 1e-6).all()
        assert (got != want).mean() < 2e-3
    # recovery error is the quantiser's: |act - out| <= Delta/2 (+ half an fp16 ulp of the output)
    esc = sym.reshape(codec.n_streams, w.n, 2, w.d) == 255
    for c, (act, out) in enumerate(((w.act_k, out_k), (w.act_v, out_v))):
        a = act.double().cpu().numpy().reshape(codec.n_streams, w.n, w.d)
        o = out.double().cpu().numpy().reshape(codec.n_streams, w.n, w.d)
        ulp = np.spacing(np.abs(o).astype(np.float16)).astype(np.float64)
        e = esc[:, :, c, :]
        bound = float(np.float32(w.delta)) / 2 + ulp / 2 + 1e-6
        assert (np.abs(a - o)[~e] <= bound[~e]).all()
        assert np.array_equal(u16(act).reshape(e.shape)[e], u16(out).reshape(e.shape)[e])


def test_one_hot_rows_give_a_single_symbol(oracle, dev):
    """One-hot prediction without noise: zero residuals everywhere, a histogram that is a
    single spike, no rANS words, bit-exact reconstruction."""
    w = make_workload("tiny", device=dev, one_hot=True, overrides=dict(n=256))
    codec = codec_for(w)
    coded = codec.encode(w.cand_k, w.cand_v, w.probs, w.act_k, w.act_v)
    codec.check_status()
    assert (coded.symbols == 127).all() and int(coded.esc_cnt.sum()) == 0
    assert (u16(coded.freq)[:, 127] == 4096).all()
    assert (u32(coded.n_words) == 0).all() and (u32(coded.states) == 65536).all()
    out_k, out_v = torch.zeros_like(w.act_k), torch.zeros_like(w.act_v)
    codec.decode(w.cand_k, w.cand_v, w.probs, out_k, out_v)
    codec.check_status()
    assert torch.equal(out_k.view(torch.int16), w.act_k.view(torch.int16))
    assert torch.equal(out_v.view(torch.int16), w.act_v.view(torch.int16))


def test_special_values_escape_bit_exactly(oracle, dev):
    """Infinities, NaNs, fp16 subnormals and out-of-range residuals."""
    O = oracle
    w = make_workload("tiny", device=dev, overrides=dict(L=1, H=2, n=40, seed=21))
    ak = w.act_k.clone()
    flat = ak.view(-1)
    flat[5] = float("inf")
    flat[6] = float("-inf")
    flat[7] = float("nan")
    flat[70] = 6.0e-8           # fp16 subnormal
    flat[71] = 30000.0
    w.cand_k.view(-1)[1000] = float("inf")     # non-finite prediction
    w.cand_v.view(-1)[2000] = 2.0 ** -24       # subnormal candidate
    w.act_k = ak
    codec = codec_for(w, esc_frac=1.0)
    coded = codec.encode(w.cand_k, w.cand_v, w.probs, w.act_k, w.act_v)
    codec.check_status()
    ref = _oracle_encode(O, w, O.F32)
    assert np.array_equal(u8(coded.symbols), ref["symbols"])
    total = int(ref["esc_cnt"].sum())
    assert np.array_equal(u16(coded.esc_vals)[:total], ref["esc_vals"])
    out_k, out_v = torch.zeros_like(w.act_k), torch.zeros_like(w.act_v)
    codec.decode(w.cand_k, w.cand_v, w.probs, out_k, out_v)
    codec.check_status()
    rk, rv = O.reconstruct(oracle_dims(O, w), storage_np(w.cand_k), storage_np(w.cand_v),
                           w.probs.cpu().numpy(), ref["symbols"], ref["esc_vals"], ref["esc_off"], mode=O.F32)
    assert np.array_equal(u16(out_k).ravel(), rk) and np.array_equal(u16(out_v).ravel(), rv)


# --------------------------------------------------------------------------- byte-stream calls on their own

BYTE_CASES = [(600, 1000, "gauss"),        # several hundred whole-stream units: the three-wavefront encoder, the chain decoder
              (1500, 1000, "gauss"),       # more whole-stream units than those kernels take: the many-unit kernels, one
                                           # wavefront per workgroup (the shape of the 70B-shaped and 64-session runs)
              (1025, 700, "two"),          # an odd number of them: the last wavefront of the two-streams-per-wavefront
                                           # encoder has a single stream, and many tables hold a frequency above 2048
              (3, 8192, "gauss"),          # with chunks of 4096: exactly one pair of chunks per stream
              (2, 20580, "gauss"),         # five full chunks and a short one: four waves of decoder units per workgroup
              (1, 1, "gauss"), (3, 5, "gauss"), (2, 33, "uniform"), (5, 1000, "gauss"), (2, 4097, "two"),
              (3, 70001, "gauss"), (2, 200000, "constant"), (4, 131072, "uniform"), (1, 262144 + 17, "gauss")]


@pytest.mark.parametrize("n_streams,N,kind", BYTE_CASES)
@pytest.mark.parametrize("chunk", [0, 4096])
def test_histogram_table_rans_bit_exact(oracle, dev, n_streams, N, kind, chunk):
    from paper_2604_15356_amd import plc
    O = oracle
    print(f"bytes {n_streams}x{N} {kind} chunk {chunk}", flush=True)
    sym_t = random_bytes(n_streams, N, seed=N % 1000 + n_streams, kind=kind, device=dev)
    sym = sym_t.cpu().numpy()
    U = plc.plc_units_per_stream(N, chunk)
    n_units = n_streams * U
    cap = ((chunk if chunk else N) + 7) // 8 * 8
    i32, i16 = torch.int32, torch.int16
    counts = torch.empty((n_streams, 256), dtype=i32, device=dev)
    freq = torch.empty((n_streams, 256), dtype=i16, device=dev)
    cum = torch.empty((n_streams, 257), dtype=i16, device=dev)
    states = torch.empty((n_units, 32), dtype=i32, device=dev)
    words = torch.zeros(n_units * cap, dtype=i16, device=dev)
    word_off = torch.arange(n_units, dtype=torch.int64, device=dev) * cap
    n_words = torch.empty(n_units, dtype=i32, device=dev)
    status = torch.zeros(1, dtype=i32, device=dev)
    plc.plc_histogram(sym_t, n_streams, N, counts)
    plc.plc_build_freq(counts, n_streams, freq, cum, status)
    plc.plc_rans_encode(sym_t, n_streams, N, chunk, freq, states, words, word_off, cap, n_words, status)
    assert int(status.item()) == 0

    ref_counts = O.histogram(sym)
    ref_freq, ref_cum = O.build_freq(ref_counts)
    enc = O.rans_encode(sym, ref_freq, chunk_syms=chunk, word_cap_per_unit=cap)
    assert np.array_equal(u32(counts), ref_counts)
    assert np.array_equal(u16(freq), ref_freq) and np.array_equal(u16(cum), ref_cum)
    assert np.array_equal(u32(n_words), enc["n_words"])
    assert np.array_equal(u32(states), enc["states"])
    got_words = u16(words)
    for unit in range(n_units):
        nw = int(enc["n_words"][unit])
        assert np.array_equal(got_words[unit * cap:unit * cap + nw], enc["words"][unit * cap:unit * cap + nw])

    # GPU decodes the oracle's stream (cross-decode in the other direction)
    o_words = torch.from_numpy(enc["words"].view(np.int16)).to(dev)
    o_states = torch.from_numpy(enc["states"].view(np.int32)).to(dev)
    o_nw = torch.from_numpy(enc["n_words"].view(np.int32)).to(dev)
    dec = torch.zeros_like(sym_t)
    plc.plc_rans_decode(freq, o_states, o_words, word_off, o_nw, n_streams, N, chunk, dec, status)
    assert int(status.item()) == 0
    assert torch.equal(dec, sym_t)


def test_more_whole_stream_units_than_the_chain_kernels_take(oracle, dev):
    """Whole-stream units beyond the bound of the three-wavefront encoder and the chain decoder
    (plc_rans_encode / plc_rans_decode then run the many-unit kernels with one wavefront per workgroup):
    ragged streams, bit-exact both ways against the oracle, one damaged unit reported."""
    from paper_2604_15356_amd import plc
    O = oracle
    n_streams, N = 1100, 2000 + 13                     # 63 groups: three full batches and a ragged tail
    sym_t = random_bytes(n_streams, N, seed=4242, kind="gauss", device=dev)
    sym_t[17] = 127                                    # a one-symbol stream (f = 4096, no words)
    sym_t[18, ::5] = 255
    sym = sym_t.cpu().numpy()
    cap = (N + 7) // 8 * 8
    i32, i16 = torch.int32, torch.int16
    counts = torch.empty((n_streams, 256), dtype=i32, device=dev)
    freq = torch.empty((n_streams, 256), dtype=i16, device=dev)
    states = torch.empty((n_streams, 32), dtype=i32, device=dev)
    words = torch.zeros(n_streams * cap, dtype=i16, device=dev)
    word_off = torch.arange(n_streams, dtype=torch.int64, device=dev) * cap
    n_words = torch.empty(n_streams, dtype=i32, device=dev)
    status = torch.zeros(1, dtype=i32, device=dev)
    print(f"  {n_streams} whole-stream units of {N} symbols", flush=True)
    plc.plc_histogram(sym_t, n_streams, N, counts)
    plc.plc_build_freq(counts, n_streams, freq, None, status)
    plc.plc_rans_encode(sym_t, n_streams, N, 0, freq, states, words, word_off, cap, n_words, status)
    dec = torch.zeros_like(sym_t)
    plc.plc_rans_decode(freq, states, words, word_off, n_words, n_streams, N, 0, dec, status)
    assert int(status.item()) == 0
    assert torch.equal(dec, sym_t)
    ref_freq, _ = O.build_freq(O.histogram(sym))
    enc = O.rans_encode(sym, ref_freq, word_cap_per_unit=cap)
    assert np.array_equal(u16(freq), ref_freq)
    assert np.array_equal(u32(n_words), enc["n_words"]) and np.array_equal(u32(states), enc["states"])
    got = u16(words)
    for unit in range(n_streams):
        o, nw = unit * cap, int(enc["n_words"][unit])
        assert np.array_equal(got[o:o + nw], enc["words"][o:o + nw]), f"unit {unit}"
    # the oracle decodes the GPU's streams, the GPU the oracle's
    assert np.array_equal(O.rans_decode(u16(freq), u32(states), got, u64(word_off), u32(n_words), n_streams, N), sym)
    dec.zero_()
    plc.plc_rans_decode(freq, torch.from_numpy(enc["states"].view(np.int32)).to(dev),
                        torch.from_numpy(enc["words"].view(np.int16)).to(dev), word_off,
                        torch.from_numpy(enc["n_words"].view(np.int32)).to(dev), n_streams, N, 0, dec, status)
    assert int(status.item()) == 0 and torch.equal(dec, sym_t)
    # one damaged unit is reported, and decoding ends
    words[int(word_off[700]) + 3] ^= 0x1555
    plc.plc_rans_decode(freq, states, words, word_off, n_words, n_streams, N, 0, dec, status)
    assert int(status.item()) == plc.PLC_ERR_CORRUPT


def test_word_list_at_odd_addresses(oracle, dev):
    """Units whose word lists start at arbitrary 2-byte offsets decode correctly."""
    from paper_2604_15356_amd import plc
    O = oracle
    n_streams, N = 5, 50000
    sym_t = random_bytes(n_streams, N, seed=77, kind="gauss", device=dev)
    sym = sym_t.cpu().numpy()
    freq_np, _ = O.build_freq(O.histogram(sym))
    enc = O.rans_encode(sym, freq_np)
    nw = enc["n_words"].astype(np.int64)
    # pack the lists back to back with odd gaps
    offs = np.zeros(n_streams, dtype=np.int64)
    pos = 3
    for s in range(n_streams):
        offs[s] = pos
        pos += int(nw[s]) + 1 + 2 * s
    packed = np.zeros(pos + 5, dtype=np.uint16)
    for s in range(n_streams):
        o = int(enc["word_off"][s])
        packed[offs[s]:offs[s] + nw[s]] = enc["words"][o:o + nw[s]]
    status = torch.zeros(1, dtype=torch.int32, device=dev)
    dec = torch.zeros_like(sym_t)
    big = torch.from_numpy(packed.view(np.int16)).to(dev)
    plc.plc_rans_decode(torch.from_numpy(freq_np.view(np.int16)).to(dev),
                        torch.from_numpy(enc["states"].view(np.int32)).to(dev), big[1:],      # odd base too
                        torch.from_numpy(offs - 1).to(dev), torch.from_numpy(enc["n_words"].view(np.int32)).to(dev),
                        n_streams, N, 0, dec, status)
    assert int(status.item()) == 0 and torch.equal(dec, sym_t)


@pytest.mark.parametrize("chunk", [0, 1024])
def test_encoder_writes_word_lists_at_odd_addresses(oracle, dev, chunk):
    """Word lists that start at arbitrary 2-byte offsets: every word in place, nothing outside."""
    from paper_2604_15356_amd import plc
    O = oracle
    n_streams, N = 3, 40000 + 17
    sym_t = random_bytes(n_streams, N, seed=91, kind="gauss", device=dev)
    sym = sym_t.cpu().numpy()
    freq_np, _ = O.build_freq(O.histogram(sym))
    U = plc.plc_units_per_stream(N, chunk)
    n_units = n_streams * U
    cap = (chunk if chunk else N) + 5          # odd spacing between the lists
    enc = O.rans_encode(sym, freq_np, chunk_syms=chunk, word_cap_per_unit=cap)
    offs = torch.arange(n_units, dtype=torch.int64, device=dev) * cap + 3
    guard = 0x5a5a
    words = torch.full((n_units * cap + 16,), guard, dtype=torch.int16, device=dev)
    states = torch.empty((n_units, 32), dtype=torch.int32, device=dev)
    n_words = torch.empty(n_units, dtype=torch.int32, device=dev)
    status = torch.zeros(1, dtype=torch.int32, device=dev)
    plc.plc_rans_encode(sym_t, n_streams, N, chunk, torch.from_numpy(freq_np.view(np.int16)).to(dev), states,
                        words[1:], offs, cap - 3, n_words, status)
    assert int(status.item()) == 0
    assert np.array_equal(u32(n_words), enc["n_words"]) and np.array_equal(u32(states), enc["states"])
    got = u16(words)
    expect = np.full(got.shape, guard, dtype=np.uint16)
    for unit in range(n_units):
        nw = int(enc["n_words"][unit])
        o = 1 + 3 + unit * cap
        expect[o:o + nw] = enc["words"][unit * cap:unit * cap + nw]
    assert np.array_equal(got, expect)


def test_data_dependent_errors_are_reported_not_fatal(oracle, dev):
    from paper_2604_15356_amd import plc
    O = oracle
    w = make_workload("tiny", device=dev, overrides=dict(L=1, H=2, n=128, seed=31))
    # invalid probability row -> status INVALID
    codec = codec_for(w)
    probs = w.probs.clone()
    probs[0, 7, :] = 0.0
    codec.predict_residual(w.cand_k, w.cand_v, probs, w.act_k, w.act_v)
    with pytest.raises(plc.PlcError) as e:
        codec.check_status()
    assert e.value.code == plc.PLC_ERR_INVALID
    # escape list too small -> CAPACITY, nothing written past the end
    codec = codec_for(w, esc_frac=0.0)          # 64 entries
    guard = codec.esc_vals.clone()
    coded = codec.encode(w.cand_k, w.cand_v, w.probs, w.act_k, w.act_v)
    n_esc = int(coded.esc_cnt.sum())
    if n_esc > codec.esc_vals.numel():
        with pytest.raises(plc.PlcError) as e:
            codec.check_status()
        assert e.value.code == plc.PLC_ERR_CAPACITY
    del guard
    # word list too small -> CAPACITY
    codec = codec_for(w, word_frac=0.25)
    codec.encode(w.cand_k, w.cand_v, w.probs, w.act_k, w.act_v)
    with pytest.raises(plc.PlcError) as e:
        codec.check_status()
    assert e.value.code == plc.PLC_ERR_CAPACITY
    # damaged stream -> CORRUPT (or different symbols), never a fault
    codec = codec_for(w)
    coded = codec.encode(w.cand_k, w.cand_v, w.probs, w.act_k, w.act_v)
    codec.check_status()
    good = coded.symbols.clone()
    codec.words[100] ^= 0x40
    codec.n_words[1] -= 1
    codec.rans_decode()
    with pytest.raises(plc.PlcError) as e:
        codec.check_status()
    assert e.value.code == plc.PLC_ERR_CORRUPT
    # the same damage through the single decode call, whose reconstructing wavefront must still meet the
    # others at every barrier
    out_k, out_v = torch.zeros_like(w.act_k), torch.zeros_like(w.act_v)
    codec.decode(w.cand_k, w.cand_v, w.probs, out_k, out_v)
    with pytest.raises(plc.PlcError) as e:
        codec.check_status()
    assert e.value.code == plc.PLC_ERR_CORRUPT
    # a word count that points outside the buffer is refused
    codec.n_words[1] = 2 ** 31 - 1
    codec.rans_decode()
    with pytest.raises(plc.PlcError) as e:
        codec.check_status()
    assert e.value.code == plc.PLC_ERR_CORRUPT
    codec.decode(w.cand_k, w.cand_v, w.probs, out_k, out_v)
    with pytest.raises(plc.PlcError) as e:
        codec.check_status()
    assert e.value.code == plc.PLC_ERR_CORRUPT
    # a table that does not sum to 2^12 is refused as well
    codec.freq[0, 3] += 1
    codec.decode(w.cand_k, w.cand_v, w.probs, out_k, out_v)
    with pytest.raises(plc.PlcError) as e:
        codec.check_status()
    assert e.value.code == plc.PLC_ERR_CORRUPT
    del good


def test_runs_are_deterministic(oracle, dev):
    w = make_workload("tiny", device=dev)
    codec = codec_for(w)
    codec.encode(w.cand_k, w.cand_v, w.probs, w.act_k, w.act_v)
    codec.check_status()
    first = [t.clone() for t in (codec.symbols, codec.counts, codec.freq, codec.states, codec.n_words)]
    nw = u32(codec.n_words)
    words1 = codec.words.clone()
    codec.words.zero_()
    codec.encode(w.cand_k, w.cand_v, w.probs, w.act_k, w.act_v)
    codec.check_status()
    for a, b in zip(first, (codec.symbols, codec.counts, codec.freq, codec.states, codec.n_words)):
        assert torch.equal(a, b)
    for unit in range(codec.n_units):
        o = unit * codec.word_cap
        assert torch.equal(words1[o:o + int(nw[unit])], codec.words[o:o + int(nw[unit])])


def _double_rounding_cases(delta32, limit=4096):
    """(q, c) with c an fp16 value such that fp32(q * delta + c) is an exact tie between two fp16
    values while the unrounded sum is not: rounding to fp32 and then to fp16 (the contract) ends on
    the even neighbour, a single rounding of the exact sum on the other one."""
    d = float(delta32)
    c = np.arange(0x2400, 0x4800, dtype=np.uint16)                 # 2^-6 .. 8, positive
    c = np.concatenate([c, c | 0x8000]).view(np.float16).astype(np.float64)
    found = []
    for q in range(-127, 128):
        if q == 0:
            continue
        v = q * d + c                                              # exact in fp64 (32 + 11 significant bits)
        r32 = v.astype(np.float32).astype(np.float64)
        with np.errstate(over="ignore"):
            h = r32.astype(np.float16)                             # tie -> even
        hv = h.astype(np.float64)
        other = np.where(hv > r32, np.nextafter(h, np.float16(-np.inf)), np.nextafter(h, np.float16(np.inf)))
        tie = (np.abs(hv - r32) == np.abs(other.astype(np.float64) - r32)) & (hv != r32)
        # a single rounding would go to `other` when the exact sum lies on its side of the tie
        flips = tie & (np.sign(v - r32) == np.sign(other.astype(np.float64) - r32)) & (v != r32)
        for cc in c[flips]:
            found.append((q, cc))
    assert len(found) > 100
    return found[:limit]


@pytest.mark.parametrize("k,cond", [(1, False), (4, False), (9, False), (4, True), (9, True)])
def test_reconstruct_rounds_to_fp32_then_to_fp16(oracle, dev, k, cond):
    """The recovered value is fma(q, Delta, pred) rounded to fp32 and then to fp16; inputs chosen so
    that merging the two roundings would give the neighbouring fp16 value."""
    O = oracle
    from paper_2604_15356_amd import plc
    delta = np.float32(0.02)
    cases = _double_rounding_cases(delta)
    d = 8
    n = (len(cases) + d - 1) // d
    cases = (cases * 2)[:n * d]
    q = np.array([c[0] for c in cases], dtype=np.int64).reshape(n, d)
    cv = np.array([c[1] for c in cases], dtype=np.float16).reshape(n, d)
    g = torch.Generator(device=dev).manual_seed(k)
    cand_k = torch.randn((1, 1, 1, n, k, d), generator=g, device=dev).to(torch.float16)
    cand_v = torch.randn((1, 1, 1, n, k, d), generator=g, device=dev).to(torch.float16)
    j = k - 1                                                       # the candidate that carries all weight
    cand_k[0, 0, 0, :, j] = torch.from_numpy(cv).to(dev)
    cand_v[0, 0, 0, :, j] = torch.from_numpy(-cv).to(dev)
    probs = torch.zeros((1, n, k), dtype=torch.float32, device=dev)
    probs[:, :, j] = 0.25                                           # renormalises to exactly 1
    sym = torch.empty((1, n, 2, d), dtype=torch.uint8, device=dev)
    sym[0, :, 0] = torch.from_numpy((q + 127).astype(np.uint8)).to(dev)
    sym[0, :, 1] = torch.from_numpy((-q + 127).astype(np.uint8)).to(dev)
    sym = sym.reshape(1, 2 * n * d)
    from paper_2604_15356_amd.codec import KVDeltaCodec
    codec = KVDeltaCodec(1, 1, 1, n, k, d, float(delta))
    out_k = torch.zeros((1, 1, 1, n, d), dtype=torch.float16, device=dev)
    out_v = torch.zeros_like(out_k)
    chosen = torch.full((1, n), j, dtype=torch.int32, device=dev)
    chosen[0, ::3] = -1                                             # both kinds of position
    if cond:
        plc.plc_reconstruct_cond(codec.dims, cand_k, cand_v, probs, chosen, sym, codec.esc_vals, codec.esc_off,
                                 out_k, out_v, codec.ws, codec.status)
    else:
        codec.reconstruct(cand_k, cand_v, probs, out_k, out_v, symbols=sym)
    codec.check_status()
    dm = O.make_dims(1, 1, 1, n, k, d, float(delta))
    rk, rv = O.reconstruct(dm, cand_k.cpu().numpy(), cand_v.cpu().numpy(), probs.cpu().numpy(), u8(sym),
                           np.zeros(1, dtype=np.uint16), np.zeros(1, dtype=np.uint64), mode=O.F32,
                           chosen=chosen.cpu().numpy() if cond else None)
    assert np.array_equal(u16(out_k).ravel(), rk)
    assert np.array_equal(u16(out_v).ravel(), rv)
    # the cases are what they claim to be: a single rounding of the exact sum differs everywhere
    exact = q.astype(np.float64) * float(delta) + cv.astype(np.float64)
    with np.errstate(over="ignore"):
        once = exact.astype(np.float16).view(np.uint16).ravel()
    assert (once != rk).all()


def test_one_call_decode_equals_two_calls_on_random_shapes(dev):
    """The decoder that reconstructs against the two kernels it replaces, on seeded random shapes: head
    dimensions with whole, half and several rows per batch of 64 chunks, ragged ends, few and many
    escapes, both candidate layouts, and with and without a chosen candidate per position."""
    rng = np.random.default_rng(20241)
    for trial in range(14):
        k = int(rng.integers(1, 9))
        d = int(rng.choice([8, 16, 24, 40, 64, 72, 128, 256, 264, 512, 520]))
        n = int(rng.integers(1, max(2, 6000 // d)))
        S, L, H = int(rng.integers(1, 3)), int(rng.integers(1, 3)), int(rng.integers(1, 4))
        layout = "lhnkd" if trial % 2 == 0 else "lnkhd"
        sigma = float(rng.choice([0.02, 0.05, 0.6, 2.5]))
        print(f"trial {trial}: S{S} L{L} H{H} n{n} k{k} d{d} {layout} sigma {sigma}", flush=True)
        w = make_workload("tiny", device=dev, layout=layout, random_rows=True,
                          overrides=dict(S=S, L=L, H=H, n=n, k=k, d=d, sigma=sigma, seed=1000 + trial))
        codec = codec_for(w, esc_frac=1.0)
        ones = [torch.zeros_like(w.act_k), torch.zeros_like(w.act_v)]
        twos = [torch.zeros_like(w.act_k), torch.zeros_like(w.act_v)]
        # weighted mean
        coded = codec.encode(w.cand_k, w.cand_v, w.probs, w.act_k, w.act_v)
        codec.check_status("encode")
        codec.decode(w.cand_k, w.cand_v, w.probs, *ones)
        codec.check_status("decode")
        assert torch.equal(codec.dec_symbols, coded.symbols)
        codec.dec_symbols.zero_()
        codec.decode(w.cand_k, w.cand_v, w.probs, *twos, fused=False)
        codec.check_status("decode in two calls")
        assert torch.equal(codec.dec_symbols, coded.symbols)
        for a, b in zip(ones, twos):
            assert np.array_equal(u16(a), u16(b)), f"trial {trial}"
        # token-conditional, a fifth of the positions without a candidate
        ch = w.chosen.to(torch.int32).clone()
        g = torch.Generator(device=ch.device).manual_seed(trial)
        ch[torch.rand(ch.shape, generator=g, device=ch.device) < 0.2] = -1
        coded = codec.encode_cond(w.cand_k, w.cand_v, w.probs, w.act_k, w.act_v, chosen=ch.contiguous())
        codec.check_status("encode_cond")
        codec.decode_cond(w.cand_k, w.cand_v, w.probs, *ones)
        codec.check_status("decode_cond")
        assert torch.equal(codec.dec_symbols, coded.symbols)
        codec.dec_symbols.zero_()
        codec.decode_cond(w.cand_k, w.cand_v, w.probs, *twos, fused=False)
        codec.check_status("decode_cond in two calls")
        for a, b in zip(ones, twos):
            assert np.array_equal(u16(a), u16(b)), f"trial {trial} (token-conditional)"


@pytest.mark.parametrize("S,L,groups,layout", [(5, 2, 3, "lhnkd"), (1, 6, 4, "lnkhd"), (2, 5, 4, "lhnkd")])
def test_grouped_codec_matches_oracle(oracle, dev, S, L, groups, layout):
    """The cache coded as independent groups of sessions (or of layers inside a session), the groups'
    entropy coding on a second HIP stream beside the next group's prediction pass: every stream's symbols,
    escapes, table, states and words are the oracle's, and the decoded cache is the oracle's reconstruction."""
    from paper_2604_15356_amd.codec import GroupedCodec
    O = oracle
    w = make_workload("tiny", device=dev, layout=layout, random_rows=True,
                      overrides=dict(S=S, L=L, H=3, n=150, k=5, d=40, sigma=0.4, seed=300 + S))
    gc = GroupedCodec(w.S, w.L, w.H, w.n, w.k, w.d, w.delta, w.qmax, groups=groups, device=dev,
                      cand_stride=w.cand_k.stride()[:5], act_stride=w.act_k.stride()[:4], esc_frac=1.0)
    print(f"  S{S} L{L} {layout}: groups {gc.slices}", flush=True)
    assert len(gc.codecs) > 1
    ref = _oracle_encode(O, w, O.F32)
    sym_ref = ref["symbols"].reshape(w.S, w.L, w.H, -1)
    freq_ref, _ = O.build_freq(O.histogram(ref["symbols"]))
    enc_ref = O.rans_encode(ref["symbols"], freq_ref)
    rk, rv = O.reconstruct(oracle_dims(O, w), storage_np(w.cand_k), storage_np(w.cand_v), w.probs.cpu().numpy(),
                           ref["symbols"], ref["esc_vals"], ref["esc_off"], mode=O.F32)
    out_k, out_v = torch.zeros_like(w.act_k), torch.zeros_like(w.act_v)
    for overlap in (True, False):
        for _ in range(2):                      # twice: the second pass finds the first one's artefacts in place
            coded = gc.encode(w.cand_k, w.cand_v, w.probs, w.act_k, w.act_v, overlap=overlap)
        out_k.zero_(), out_v.zero_()
        gc.decode(w.cand_k, w.cand_v, w.probs, out_k, out_v, overlap=overlap)
        torch.cuda.synchronize()
        gc.check_status("grouped")
        for (s0, s1, l0, l1), c, art in zip(gc.slices, gc.codecs, coded):
            ids = np.arange(w.S * w.L * w.H).reshape(w.S, w.L, w.H)[s0:s1, l0:l1].ravel()     # the group's streams
            assert np.array_equal(u8(art.symbols), sym_ref[s0:s1, l0:l1].reshape(len(ids), -1))
            assert np.array_equal(u16(art.freq), freq_ref[ids])
            assert np.array_equal(u32(art.states), enc_ref["states"][ids])
            assert np.array_equal(u32(art.n_words), enc_ref["n_words"][ids])
            assert np.array_equal(u32(art.esc_cnt), ref["esc_cnt"][ids])
            words, esc = u16(art.words), u16(art.esc_vals)
            at = 0
            for j, st in enumerate(ids):
                nw, o = int(enc_ref["n_words"][st]), int(enc_ref["word_off"][st])
                assert np.array_equal(words[j * c.word_cap:j * c.word_cap + nw], enc_ref["words"][o:o + nw])
                ne, eo = int(ref["esc_cnt"][st]), int(ref["esc_off"][st])
                assert np.array_equal(esc[at:at + ne], ref["esc_vals"][eo:eo + ne])
                at += ne
            assert torch.equal(c.dec_symbols, c.symbols)
        assert np.array_equal(u16(out_k).ravel(), rk) and np.array_equal(u16(out_v).ravel(), rv)
    assert gc.roundtrip_exact() and gc.total_words() == int(enc_ref["n_words"].sum())
    assert gc.total_escapes() == int(ref["esc_cnt"].sum())


def test_statistics_inside_the_prediction_pass_equal_the_histogram_call(oracle, dev):
    """plc_predict_residual_hist against plc_predict_residual + plc_histogram and against the oracle's counts, on
    streams long enough (more than 1024 tiles) that a workgroup of the counting pass takes two tiles, with an odd
    number of tiles, and on short ragged ones."""
    O = oracle
    for ov in (dict(S=1, L=1, H=2, n=8200, k=2, d=128, seed=61), dict(S=2, L=1, H=3, n=37, k=5, d=24, sigma=0.8, seed=62)):
        w = make_workload("tiny", device=dev, overrides=ov, random_rows=True)
        print(f"  S{w.S} L{w.L} H{w.H} n{w.n} k{w.k} d{w.d}: {(2 * w.n * w.d + 2047) // 2048} tiles per stream", flush=True)
        codec = codec_for(w, esc_frac=1.0)
        a = codec.encode(w.cand_k, w.cand_v, w.probs, w.act_k, w.act_v, fused_counts=True)
        codec.check_status("counting pass")
        first = [t.clone() for t in (a.symbols, a.counts, a.freq, a.esc_cnt, a.esc_off, a.states, a.n_words)]
        esc1 = a.esc_vals[:int(a.esc_cnt.sum())].clone()
        codec.counts.fill_(-1)
        b = codec.encode(w.cand_k, w.cand_v, w.probs, w.act_k, w.act_v, fused_counts=False)
        codec.check_status("separate histogram")
        for x, y in zip(first, (b.symbols, b.counts, b.freq, b.esc_cnt, b.esc_off, b.states, b.n_words)):
            assert torch.equal(x, y)
        assert torch.equal(esc1, b.esc_vals[:int(b.esc_cnt.sum())])
        ref = _oracle_encode(O, w, O.F32)
        assert np.array_equal(u8(a.symbols), ref["symbols"])
        assert np.array_equal(u32(first[1]), O.histogram(ref["symbols"]))
