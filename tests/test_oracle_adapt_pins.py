"""Pins for the surprisal-adaptive quantiser part of the CPU oracle.

Def. "Surprisal-adaptive quantizer" (Sec. 5.3): position i gets b_i = max(1,
floor(b0 * h_i / hbar)) bits per residual component, h_i its surprisal, hbar the
average; Cor. "Practical bit allocation" (Sec. 9.4): b bits are a uniform step
of range / 2^b.  Symbols of positions with the same depth share a frequency
table.  Checked against the pinned fixed-step functions (special cases that
must coincide), the definition's floating formula, closed forms and round
trips -- never against itself or the device path.
"""
import numpy as np
import pytest
import torch
from scipy.stats import norm

from paper_2604_15356_amd.workloads import make_workload, random_bytes
from tests.test_oracle_pins import _dims, _encode_floats, _np, _storage


def _encode(O, w, chosen, bits, step_range, mode=None, **kw):
    mode = O.F64 if mode is None else mode
    return O.predict_residual(_dims(O, w), _storage(w.cand_k), _storage(w.cand_v), _np(w.probs),
                              _storage(w.act_k), _storage(w.act_v), mode=mode, chosen=chosen, bits=bits,
                              step_range=step_range, **kw)


def _reconstruct(O, w, r, chosen, bits, step_range, mode=None, **kw):
    mode = O.F64 if mode is None else mode
    return O.reconstruct(_dims(O, w), _storage(w.cand_k), _storage(w.cand_v), _np(w.probs), r["symbols"],
                         r["esc_vals"], r["esc_off"], mode=mode, chosen=chosen, bits=bits, step_range=step_range,
                         **kw)


# --------------------------------------------------------------------------- bit depths

def test_bit_depth_is_the_definitions_formula_on_every_frequency(oracle):
    """b = min(bmax, max(1, floor(b0 * log2(4096 / f) / hbar))) for every table frequency f, decided
    by integer comparisons only; checked against the floating formula wherever that formula is not
    within rounding of an integer (there the integer form is the definition)."""
    for b0, hbar in ((3.0, np.log2(15.0)), (2.0, 3.3), (4.0, 4.3), (2.5, 1.0)):
        thr = oracle.surprisal_thresholds(b0, hbar)
        assert (np.diff(thr[2:].astype(int)) <= 0).all()
        # one position per frequency: k = 1 rows p = f / 4096 give the table (f, 4096 - f) exactly
        f = np.arange(1, 4096)
        probs = (f / 4096.0).astype(np.float32).reshape(1, -1, 1)
        hit = oracle.surprisal_bits(probs, np.zeros((1, f.size), np.int32), thr)[0]
        miss = oracle.surprisal_bits(probs, np.full((1, f.size), -1, np.int32), thr)[0]
        for got, freq in ((hit, f), (miss, 4096 - f)):
            v = b0 * np.log2(4096.0 / freq) / hbar
            want = np.clip(np.floor(v), 1, oracle.MAX_BITS)
            clear = np.abs(v - np.round(v)) > 1e-9
            assert np.array_equal(got[clear], want[clear].astype(np.uint8))
            assert (np.abs(got[~clear].astype(float) - want[~clear]) <= 1).all()


def test_thresholds_are_the_closed_form_and_depths_have_no_cap_of_four(oracle):
    """thr[m] = floor(4096 * 2^(-m hbar / b0)) where that is clear of an integer; where hbar / b0 is a whole
    number the thresholds are exact powers of two; and with twelve depths allowed the depth of a frequency
    is the definition's floor(b0 h / hbar) beyond four as well."""
    assert list(oracle.surprisal_thresholds(3.0, 3.0, 6)) == [0, 0, 1024, 512, 256, 128, 64]
    assert list(oracle.surprisal_thresholds(1.0, 2.0, 7)) == [0, 0, 256, 64, 16, 4, 1, 0]
    for b0, hbar in ((3.0, np.log2(15.0)), (2.0, 3.3), (5.0, 2.1)):
        thr = oracle.surprisal_thresholds(b0, hbar, 12)
        for m in range(2, 13):
            v = 4096.0 * 2.0 ** (-m * hbar / b0)
            if abs(v - round(v)) > 1e-6:
                assert thr[m] == int(np.floor(v))
        f = np.arange(1, 4096)
        probs = (f / 4096.0).astype(np.float32).reshape(1, -1, 1)
        got = oracle.surprisal_bits(probs, np.zeros((1, f.size), np.int32), thr)[0]
        v = b0 * np.log2(4096.0 / f) / hbar
        clear = np.abs(v - np.round(v)) > 1e-9
        assert np.array_equal(got[clear], np.clip(np.floor(v), 1, 12)[clear].astype(np.uint8))
        assert got.max() > 4


def test_bit_depths_of_the_synthetic_row(oracle):
    """Llama-shaped row (perplexity 15, top 8): likely tokens get one bit, the tail four."""
    w = make_workload("llama8b", overrides=dict(L=1, H=1, d=8, n=2000))
    thr = oracle.surprisal_thresholds(3.0, np.log2(15.0))
    bits = oracle.surprisal_bits(_np(w.probs), w.chosen.numpy().astype(np.int32), thr)
    by_rank = [set(bits[0][w.chosen.numpy()[0] == j]) for j in range(w.k)]
    assert by_rank[0] == {1} and by_rank[1] == {2} and by_rank[w.k - 1] == {4}
    assert all(max(a) <= min(b) for a, b in zip(by_rank, by_rank[1:]))          # monotone in the rank


# --------------------------------------------------------------------------- quantiser

@pytest.mark.parametrize("mode_name", ["F64", "F32"])
@pytest.mark.parametrize("b", [1, 3, 4])
def test_one_depth_everywhere_is_the_fixed_step_quantiser(oracle, mode_name, b):
    mode = getattr(oracle, mode_name)
    rng_ = 0.02 * 2 ** b                                    # range / 2^b = the configuration's step
    w = make_workload("tiny", overrides=dict(n=96), random_rows=True)
    assert np.float32(rng_) * np.float32(2.0 ** -b) == np.float32(w.delta)
    bits = np.full((w.S, w.n), b, dtype=np.uint8)
    miss = np.full((w.S, w.n), -1, dtype=np.int32)
    a = _encode_floats(oracle, w, mode=mode)
    g = _encode(oracle, w, miss, bits, rng_, mode=mode)
    for key in ("symbols", "esc_vals", "esc_cnt", "esc_off"):
        assert np.array_equal(a[key], g[key]), key
    ka, va = oracle.reconstruct(_dims(oracle, w), _storage(w.cand_k), _storage(w.cand_v), _np(w.probs),
                                a["symbols"], a["esc_vals"], a["esc_off"], mode=mode)
    kg, vg = _reconstruct(oracle, w, g, miss, bits, rng_, mode=mode)
    assert np.array_equal(ka, kg) and np.array_equal(va, vg)


def test_error_is_half_the_positions_own_step(oracle):
    w = make_workload("tiny", overrides=dict(n=400))
    rng = np.random.default_rng(3)
    bits = rng.integers(1, 5, (w.S, w.n)).astype(np.uint8)
    ch = w.chosen.numpy().astype(np.int32).copy()
    ch[0, ::3] = -1
    step_range = 0.32
    r = _encode(oracle, w, ch, bits, step_range)
    _, _, pre = _reconstruct(oracle, w, r, ch, bits, step_range, want_pre_round=True)
    act = torch.stack([w.act_k, w.act_v], dim=4).double().reshape(w.n_streams, w.n, -1).numpy()
    pre = pre.reshape(w.n_streams, w.n, -1)
    sym = r["symbols"].reshape(w.n_streams, w.n, -1)
    step = float(np.float32(step_range)) * 2.0 ** -bits[0].astype(np.float64)              # [n]
    err = np.abs(act - pre)
    keep = sym != 255
    assert (err[keep] <= (step[None, :, None] / 2 * (1 + 1e-5) * np.ones_like(err))[keep]).all()
    # where the residual is spread over many cells (the misses: unit-variance residuals) the error is
    # uniform in the cell, step^2 / 12 at each depth; where it is narrower than the step (a chosen
    # candidate at a coarse depth) the error is the residual itself and smaller than that
    for b in range(1, 5):
        wide = keep & ((bits[0] == b) & (ch[0] < 0))[None, :, None]
        assert abs((err[wide] ** 2).mean() / ((step_range * 2.0 ** -b) ** 2 / 12) - 1) < 0.05
        narrow = keep & ((bits[0] == b) & (ch[0] >= 0))[None, :, None]
        assert (err[narrow] ** 2).mean() <= 1.02 * min((step_range * 2.0 ** -b) ** 2 / 12,
                                                       float(w.sigma[0]) ** 2 + 1e-6)
    assert np.array_equal(pre[~keep], act[~keep])
    for bad in (0, oracle.MAX_BITS_ORACLE + 1):       # no depth, and more depths than the oracle's arrays hold
        bits2 = bits.copy()
        bits2[0, 7] = bad
        with pytest.raises(oracle.OracleError):
            _encode(oracle, w, ch, bits2, step_range)


def test_per_depth_symbol_statistics_match_the_closed_form(oracle):
    """Given the token the residual is the N(0, sigma^2) noise; at depth b it is quantised with
    step range / 2^b, so the depth's table should be that quantised Gaussian."""
    w = make_workload("llama8b", overrides=dict(L=1, H=2, n=2048))
    thr = oracle.surprisal_thresholds(3.0, np.log2(15.0))
    ch = w.chosen.numpy().astype(np.int32)
    bits = oracle.surprisal_bits(_np(w.probs), ch, thr)
    step_range = 0.16
    r = _encode(oracle, w, ch, bits, step_range)
    counts = oracle.histogram_bucketed(r["symbols"], 2 * w.d, w.L * w.H, bits).sum(0).astype(np.float64)   # [4, 256]
    q = np.arange(-127, 128)
    for b in range(1, 5):
        total = counts[b - 1].sum()
        assert total == (bits == b).sum() * 2 * w.d * w.n_streams
        if total == 0:
            continue
        sd = float(w.sigma[0]) / (float(np.float32(step_range)) * 2.0 ** -b)
        pmf = norm.cdf((q + 0.5) / sd) - norm.cdf((q - 0.5) / sd)
        emp = counts[b - 1] / total
        assert 0.5 * np.abs(emp[:255] - pmf).sum() < 0.02, b


# --------------------------------------------------------------------------- tables and coder per depth

def test_one_table_reduces_to_the_plain_functions(oracle):
    sym = _np(random_bytes(3, 4000, 41, "gauss"))
    bits = np.ones((1, 4000 // 8), dtype=np.uint8)
    counts = oracle.histogram_bucketed(sym, 8, 3, bits, n_tables=1)
    assert np.array_equal(counts[:, 0], oracle.histogram(sym))
    freq = oracle.build_freq_sparse(counts)
    ref_freq, _ = oracle.build_freq(counts[:, 0])
    assert np.array_equal(freq[:, 0], ref_freq)
    for chunk in (0, 1024):
        a = oracle.rans_encode(sym, ref_freq, chunk_syms=chunk)
        b = oracle.rans_encode_bucketed(sym, freq, 8, 3, bits, chunk_syms=chunk)
        for key in ("states", "words", "n_words"):
            assert np.array_equal(a[key], b[key])
        dec = oracle.rans_decode_bucketed(freq, b["states"], b["words"], b["word_off"], b["n_words"], 3, 4000, 8, 3,
                                          bits, chunk_syms=chunk)
        assert np.array_equal(dec, sym)


@pytest.mark.parametrize("chunk", [0, 64, 4096])
def test_bucketed_round_trip_and_size(oracle, chunk):
    """Two sessions of three streams; symbols of depth b drawn from a Gaussian of width 3 * 2^b: coded
    with one table per depth the stream costs the sum of the per-depth entropies, which a single table
    cannot reach."""
    rng = np.random.default_rng(8)
    S, sps, n, spp = 2, 3, 150, 32
    bits = rng.integers(1, 5, (S, n)).astype(np.uint8)
    bits[1, :] = np.where(bits[1] == 3, 2, bits[1])                     # a depth that one session never uses
    width = 3.0 * 2.0 ** np.repeat(bits, spp, axis=1)                   # [S, N]
    sym = np.empty((S * sps, n * spp), dtype=np.uint8)
    for st in range(S * sps):
        sym[st] = np.clip(np.round(rng.standard_normal(n * spp) * width[st // sps] + 127), 0, 254)
    counts = oracle.histogram_bucketed(sym, spp, sps, bits)
    assert counts.sum() == sym.size and (counts[sps:, 2] == 0).all()
    freq = oracle.build_freq_sparse(counts)
    assert set(freq.astype(int).sum(-1).ravel()) <= {0, 4096}
    assert ((freq > 0) == (counts > 0)).all()
    enc = oracle.rans_encode_bucketed(sym, freq, spp, sps, bits, chunk_syms=chunk)
    dec = oracle.rans_decode_bucketed(freq, enc["states"], enc["words"], enc["word_off"], enc["n_words"], S * sps,
                                      n * spp, spp, sps, bits, chunk_syms=chunk)
    assert np.array_equal(dec, sym)
    U = oracle.units_per_stream(n * spp, chunk)
    for st in range(S * sps):
        c = counts[st].astype(np.float64)
        f = freq[st].astype(np.float64)
        nz = c > 0
        X = (c[nz] * np.log2(4096.0 / f[nz])).sum()                     # cross entropy under the depth's table
        bits_used = 16.0 * enc["n_words"][st * U:(st + 1) * U].sum()
        assert X - 512 * U <= bits_used <= 1.001 * X + 16
        one, _ = oracle.build_freq(c.sum(0, keepdims=True).astype(np.uint32))
        X1 = (c.sum(0)[c.sum(0) > 0] * np.log2(4096.0 / one[0][c.sum(0) > 0])).sum()
        assert X < 0.93 * X1
    # a symbol whose depth's table does not hold it is refused; damage is detected
    bad = sym.copy()
    bad[0, 0] = 255
    with pytest.raises(oracle.OracleError):
        oracle.rans_encode_bucketed(bad, freq, spp, sps, bits, chunk_syms=chunk)
    words = enc["words"].copy()
    words[int(enc["n_words"][0]) // 2] ^= 4
    try:
        out = oracle.rans_decode_bucketed(freq, enc["states"], words, enc["word_off"], enc["n_words"], S * sps,
                                          n * spp, spp, sps, bits, chunk_syms=chunk)
        assert not np.array_equal(out, sym)
    except oracle.OracleError as e:
        assert e.code == oracle.ERR_CORRUPT
