"""Parity of the token-conditional path (through the C ABI of libplc.so) against
the CPU oracle, element by element, on the same seeded inputs.

Bars as for the weighted-mean path: symbols, escapes, tables, rANS states and
words, index tables' consequences (index states and words) and the chosen
indices are bit-exact against the oracle in the kernel's precision; against
the fp64 oracle symbols differ only at counted rounding near-ties.  The decode
direction starts from the coded artefacts alone: the index stream is decoded
first and its result drives the reconstruction.
"""
import numpy as np
import pytest
import torch

from paper_2604_15356_amd.workloads import make_workload
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
    # name: (config, overrides, layout, random rows, fraction of positions turned into misses)
    "tiny": ("tiny", None, "lhnkd", False, 0.0),
    "tiny_misses": ("tiny", None, "lhnkd", True, 0.25),
    "heads_inner_misses": ("tiny", dict(seed=21), "lnkhd", True, 0.1),
    "ragged_k5_d24": ("tiny", dict(S=2, L=2, H=3, n=37, k=5, d=24, seed=22), "lnkhd", True, 0.2),
    "k8_d128": ("llama8b", dict(L=2, H=2, n=300, seed=23), "lhnkd", False, 0.05),
    "k11_runtime_loop": ("tiny", dict(k=11, n=129, d=40, seed=24), "lhnkd", True, 0.3),
    "k32": ("tiny", dict(k=32, L=1, H=1, n=70, d=16, seed=25), "lhnkd", True, 0.1),
    "all_misses": ("tiny", dict(n=64, seed=26), "lhnkd", True, 1.0),
    "one_position": ("tiny", dict(L=1, H=1, n=1, d=8, seed=27), "lhnkd", False, 0.0),
    "three_sessions": ("tiny", dict(S=3, L=1, H=2, n=100, seed=28), "lhnkd", True, 0.15),
    # the generator's own misses (fresh vectors where the token is none of the k = 20 candidates)
    "k20_with_misses": ("miss20", dict(L=1, H=2, n=300, seed=29), "lhnkd", False, 0.0),
    # more streams than the one-kernel decode takes on this path with more than four candidates (2048): the single call then runs the
    # many-unit entropy decoder, one wavefront per workgroup, followed by the reconstruction kernel
    "many_streams_k5": ("tiny", dict(S=3, L=24, H=32, n=7, k=5, d=16, seed=30), "lhnkd", True, 0.2),
    # with k <= 4 the single call keeps its one-kernel form at any number of streams, three workgroups per compute
    # unit on a three-block word ring that these streams wrap a dozen times
    "dense_streams_k4": ("tiny", dict(S=1, L=20, H=30, n=161, k=4, d=64, seed=32), "lhnkd", True, 0.2),
}


def _with_misses(w, frac, seed):
    """chosen as the encoder is told it: the drawn index, with a share of the positions declared
    'not among the candidates' (their actual vectors then simply are far from the weighted mean)."""
    ch = w.chosen.to(torch.int32).clone()
    if frac > 0:
        g = torch.Generator(device=ch.device).manual_seed(seed)
        ch[torch.rand(ch.shape, generator=g, device=ch.device) < frac] = -1
    return ch.contiguous()


def _oracle_encode(O, w, chosen, mode, **kw):
    return O.predict_residual(oracle_dims(O, w), storage_np(w.cand_k), storage_np(w.cand_v),
                              w.probs.cpu().numpy(), storage_np(w.act_k), storage_np(w.act_v),
                              mode=mode, chosen=chosen, **kw)


@pytest.mark.parametrize("case", list(CASES))
def test_conditional_encode_decode_matches_oracle(oracle, dev, case):
    O = oracle
    name, overrides, layout, random_rows, miss = CASES[case]
    w = make_workload(name, device=dev, layout=layout, overrides=overrides, random_rows=random_rows)
    chosen = _with_misses(w, miss, 100 + len(case))
    ch_np = chosen.cpu().numpy()
    codec = codec_for(w, want_pred=True, esc_frac=1.0)
    print(f"case {case}: S{w.S} L{w.L} H{w.H} n{w.n} k{w.k} d{w.d} layout {layout} misses {miss}", flush=True)
    coded = codec.encode_cond(w.cand_k, w.cand_v, w.probs, w.act_k, w.act_v, chosen=chosen)
    codec.check_status("encode_cond")

    # ---- floating-point part
    ref32 = _oracle_encode(O, w, ch_np, O.F32)
    ref64 = _oracle_encode(O, w, ch_np, O.F64, want_pred=True, want_u=True)
    sym = u8(coded.symbols)
    assert np.array_equal(sym, ref32["symbols"]), "symbols differ from the strict-fp32 oracle"
    pred = codec.pred.cpu().numpy().astype(np.float64)
    scale = np.maximum(np.abs(ref64["pred"]), 1e-2)
    assert (np.abs(pred - ref64["pred"]) / scale).max() < 1e-3
    hit = np.repeat(ch_np.reshape(w.S, 1, w.n) >= 0, w.L * w.H, axis=1).reshape(codec.n_streams, w.n)
    hit = np.repeat(hit, 2 * w.d, axis=1)
    assert np.array_equal(pred[hit], ref64["pred"][hit])          # a chosen candidate is reproduced exactly
    tau = 64 * 2.0 ** -24 * 8.0 / float(np.float32(w.delta))
    n_diff, n_ok = near_tie_report(sym, ref64["symbols"], ref64["u"], tau)
    print(f"  near-ties vs fp64 oracle: {n_diff} of {sym.size}", flush=True)
    assert n_diff == n_ok and n_diff <= max(3, 1e-4 * sym.size)
    total = int(ref32["esc_cnt"].sum())
    assert np.array_equal(u32(coded.esc_cnt), ref32["esc_cnt"])
    assert np.array_equal(u64(coded.esc_off), ref32["esc_off"])
    assert np.array_equal(u16(coded.esc_vals)[:total], ref32["esc_vals"])

    # ---- residual streams, bit-exact given identical symbols
    freq, cum = O.build_freq(O.histogram(sym))
    enc = O.rans_encode(sym, freq, word_cap_per_unit=codec.word_cap)
    assert np.array_equal(u16(coded.freq), freq)
    assert np.array_equal(u32(coded.n_words), enc["n_words"])
    assert np.array_equal(u32(coded.states), enc["states"])
    words = u16(coded.words)
    for unit in range(codec.n_units):
        off, nw = unit * codec.word_cap, int(enc["n_words"][unit])
        assert np.array_equal(words[off:off + nw], enc["words"][off:off + nw]), f"unit {unit}"

    # ---- index stream, bit-exact
    probs = w.probs.cpu().numpy()
    ienc = O.index_encode(probs, ch_np, word_cap=codec.idx_word_cap)
    assert np.array_equal(u32(coded.idx_n_words), ienc["n_words"])
    assert np.array_equal(u32(coded.idx_states), ienc["states"])
    iw = u16(coded.idx_words)
    for s in range(w.S):
        off, nw = s * codec.idx_word_cap, int(ienc["n_words"][s])
        assert np.array_equal(iw[off:off + nw], ienc["words"][off:off + nw]), f"session {s}"
    # the oracle decodes the GPU's index stream
    assert np.array_equal(O.index_decode(probs, u32(coded.idx_states), iw, u64(coded.idx_word_off),
                                         u32(coded.idx_n_words)), ch_np)

    # ---- decode direction on the GPU, from the coded artefacts alone
    codec.chosen.fill_(-7)                        # the decoder must not look at the encoder's copy
    out_k = torch.zeros_like(w.act_k)
    out_v = torch.zeros_like(w.act_v)
    codec.decode_cond(w.cand_k, w.cand_v, w.probs, out_k, out_v)
    codec.check_status("decode_cond")
    assert np.array_equal(codec.dec_chosen.cpu().numpy(), ch_np)
    assert torch.equal(codec.dec_symbols, coded.symbols)
    rk32, rv32 = O.reconstruct(oracle_dims(O, w), storage_np(w.cand_k), storage_np(w.cand_v), probs, sym,
                               ref32["esc_vals"], ref32["esc_off"], mode=O.F32, chosen=ch_np)
    assert np.array_equal(u16(out_k).ravel(), rk32) and np.array_equal(u16(out_v).ravel(), rv32)
    # decode_cond() is the single call that reconstructs inside the entropy decoder where the shape allows
    # it; the two calls one after the other must give the same bits
    two_k, two_v = torch.zeros_like(w.act_k), torch.zeros_like(w.act_v)
    codec.dec_symbols.zero_()
    codec.decode_cond(w.cand_k, w.cand_v, w.probs, two_k, two_v, fused=False)
    codec.check_status("decode_cond in two calls")
    assert torch.equal(codec.dec_symbols, coded.symbols)
    assert np.array_equal(u16(two_k), u16(out_k)) and np.array_equal(u16(two_v), u16(out_v))
    # recovery error is the quantiser's: |act - out| <= Delta/2 (+ half an fp16 ulp of the output)
    esc = sym.reshape(codec.n_streams, w.n, 2, w.d) == 255
    delta = float(np.float32(w.delta))
    for c, (act, out) in enumerate(((w.act_k, out_k), (w.act_v, out_v))):
        a = act.reshape(codec.n_streams, w.n, w.d).cpu().numpy().astype(np.float64)
        o = out.reshape(codec.n_streams, w.n, w.d).cpu().numpy().astype(np.float64)
        e = esc[:, :, c, :]
        ulp = np.maximum(np.abs(o), 2.0 ** -14) * 2.0 ** -10
        assert (np.abs(a - o)[~e] <= delta / 2 + ulp[~e] / 2 + 1e-6).all()
        assert np.array_equal(u16(act).reshape(codec.n_streams, w.n, w.d)[e],
                              u16(out).reshape(codec.n_streams, w.n, w.d)[e])


def test_oracle_written_index_stream_decodes_on_the_gpu(oracle, dev):
    O = oracle
    from paper_2604_15356_amd import plc
    w = make_workload("tiny", device=dev, overrides=dict(S=2, L=1, H=1, d=8, n=333, k=7, seed=31), random_rows=True)
    ch = _with_misses(w, 0.2, 5).cpu().numpy()
    probs = w.probs.cpu().numpy()
    enc = O.index_encode(probs, ch)
    t = lambda a, dt: torch.from_numpy(a.view(dt)).to(dev)
    out = torch.full((w.S, w.n), -9, dtype=torch.int32, device=dev)
    status = torch.zeros(1, dtype=torch.int32, device=dev)
    plc.plc_index_decode(w.probs, t(enc["states"], np.int32), t(enc["words"], np.int16),
                         t(enc["word_off"], np.int64), t(enc["n_words"], np.int32), w.S, w.n, w.k, out, status)
    assert int(status.item()) == 0
    assert np.array_equal(out.cpu().numpy(), ch)
    # a damaged or truncated stream is reported, and nothing outside the buffers is touched
    words = enc["words"].copy()
    words[int(enc["n_words"][0]) // 2] ^= 0x40
    plc.plc_index_decode(w.probs, t(enc["states"], np.int32), t(words, np.int16),
                         t(enc["word_off"], np.int64), t(enc["n_words"], np.int32), w.S, w.n, w.k, out, status)
    bad = int(status.item()) == plc.PLC_ERR_CORRUPT or not np.array_equal(out.cpu().numpy(), ch)
    assert bad
    status.zero_()
    short = enc["n_words"].copy()
    short[1] -= 1
    plc.plc_index_decode(w.probs, t(enc["states"], np.int32), t(enc["words"], np.int16),
                         t(enc["word_off"], np.int64), t(short, np.int32), w.S, w.n, w.k, out, status)
    assert int(status.item()) == plc.PLC_ERR_CORRUPT


def test_error_statuses_of_the_conditional_calls(oracle, dev):
    from paper_2604_15356_amd import plc
    w = make_workload("tiny", device=dev, overrides=dict(L=1, H=1, n=64, seed=33))
    codec = codec_for(w)
    ch = w.chosen.to(torch.int32).clone()
    ch[0, 5] = w.k                                   # not a candidate index
    codec.encode_cond(w.cand_k, w.cand_v, w.probs, w.act_k, w.act_v, chosen=ch)
    with pytest.raises(plc.PlcError) as e:
        codec.check_status()
    assert e.value.code == plc.PLC_ERR_INVALID
    # index stream that does not fit its reservation
    ch = w.chosen.to(torch.int32).contiguous()
    g = torch.Generator(device=dev).manual_seed(1)
    flat = torch.rand((w.S, w.n, w.k), generator=g, device=dev) * 1e-3          # every index is a surprise
    status = torch.zeros(1, dtype=torch.int32, device=dev)
    words = torch.zeros(8, dtype=torch.int16, device=dev)
    guard = words.clone()
    plc.plc_index_encode(flat, ch, w.S, w.n, w.k, codec.idx_states, words[:4], codec.idx_word_off, 4,
                         codec.idx_n_words, status)
    assert int(status.item()) == plc.PLC_ERR_CAPACITY
    assert torch.equal(words[4:], guard[4:])
    # invalid probability row
    status.zero_()
    bad = w.probs.clone()
    bad[0, 3, 1] = float("nan")
    plc.plc_index_encode(bad, ch, w.S, w.n, w.k, codec.idx_states, codec.idx_words, codec.idx_word_off,
                         codec.idx_word_cap, codec.idx_n_words, status)
    assert int(status.item()) == plc.PLC_ERR_INVALID
    # a chosen index out of range handed to the decode side: reported, and no candidate is read through it
    codec = codec_for(w)
    codec.encode_cond(w.cand_k, w.cand_v, w.probs, w.act_k, w.act_v, chosen=ch)
    codec.check_status()
    out_k, out_v = torch.zeros_like(w.act_k), torch.zeros_like(w.act_v)
    for wrong in (w.k, 1 << 20, -2, -(1 << 30)):
        broken = ch.clone()
        broken[0, 11] = wrong
        for call in ("one", "two"):
            if call == "one":
                plc.plc_rans_decode_reconstruct_cond(codec.dims, codec.freq, codec.states, codec.words,
                                                     codec.word_off, codec.n_words, 0, w.cand_k, w.cand_v, w.probs,
                                                     broken, codec.esc_vals, codec.esc_off, codec.dec_symbols,
                                                     out_k, out_v, codec.ws, codec.status)
            else:
                plc.plc_reconstruct_cond(codec.dims, w.cand_k, w.cand_v, w.probs, broken, codec.dec_symbols,
                                         codec.esc_vals, codec.esc_off, out_k, out_v, codec.ws, codec.status)
            with pytest.raises(plc.PlcError) as e:
                codec.check_status()
            assert e.value.code == plc.PLC_ERR_INVALID, (wrong, call)


@pytest.mark.parametrize("layout", ["lhnkd", "lnkhd"])
def test_select_candidate_matches_oracle_and_the_generator(oracle, dev, layout):
    O = oracle
    w = make_workload("tiny", device=dev, layout=layout, overrides=dict(S=2, n=300, seed=35))
    fresh = torch.randn((w.d,), generator=torch.Generator().manual_seed(3)).to(torch.float16).to(dev)
    w.act_k[1, 0, 0, 17] = fresh                    # a vector that is none of the candidates
    w.act_k[0, 0, 0, 60] = float("nan")
    w.cand_k[0, 0, 0, 9, 2] = w.cand_k[0, 0, 0, 9, 0]        # two equal candidates: lowest index wins
    limit = (4 * float(w.sigma[0])) ** 2
    codec = codec_for(w)
    got = codec.select_candidate(w.cand_k, w.act_k, limit).cpu().numpy()
    ref32 = O.select_candidate(oracle_dims(O, w), storage_np(w.cand_k), storage_np(w.act_k), limit, mode=O.F32)
    ref64 = O.select_candidate(oracle_dims(O, w), storage_np(w.cand_k), storage_np(w.act_k), limit, mode=O.F64)
    assert np.array_equal(got, ref32)
    assert np.array_equal(got, ref64)               # the synthetic candidates are far apart: no near-ties
    want = w.chosen.cpu().numpy().copy()
    want[1, 17] = want[0, 60] = -1
    if want[0, 9] == 2:
        want[0, 9] = 0
    assert np.array_equal(got, want)
    # and the whole path driven by the recovered indices
    out_k, out_v = torch.zeros_like(w.act_k), torch.zeros_like(w.act_v)
    coded = codec.encode_cond(w.cand_k, w.cand_v, w.probs, w.act_k, w.act_v, max_mean_sq=limit)
    codec.decode_cond(w.cand_k, w.cand_v, w.probs, out_k, out_v)
    codec.check_status()
    assert np.array_equal(codec.dec_chosen.cpu().numpy(), want)
    assert torch.equal(codec.dec_symbols, coded.symbols)


def test_conditional_path_is_deterministic_and_halves_the_bits(oracle, dev):
    w = make_workload("llama8b", device=dev, overrides=dict(L=2, H=4, n=1024))
    ch = w.chosen.to(torch.int32).contiguous()
    codec = codec_for(w)
    a = codec.encode_cond(w.cand_k, w.cand_v, w.probs, w.act_k, w.act_v, chosen=ch)
    first = [t.clone() for t in (a.symbols, a.states, a.n_words, a.idx_states, a.idx_n_words)]
    nw = int(a.n_words.sum())
    b = codec.encode_cond(w.cand_k, w.cand_v, w.probs, w.act_k, w.act_v, chosen=ch)
    for x, y in zip(first, (b.symbols, b.states, b.n_words, b.idx_states, b.idx_n_words)):
        assert torch.equal(x, y)
    cond_bits = 16.0 * nw / a.symbols.numel()
    codec.encode(w.cand_k, w.cand_v, w.probs, w.act_k, w.act_v)
    codec.check_status()
    mean_bits = 16.0 * int(codec.n_words.sum()) / a.symbols.numel()
    idx_bits = (16.0 * int(a.idx_n_words.sum()) + 1024 * w.S) / (w.S * w.n)
    print(f"  bits/component: weighted mean {mean_bits:.2f}, given the token {cond_bits:.2f}; "
          f"index {idx_bits:.2f} bits per position", flush=True)
    assert 3.2 < cond_bits < 3.6 and mean_bits > 7.0 and 1.5 < idx_bits < 3.6
