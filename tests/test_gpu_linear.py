"""Parity of the linear-embedding predictor (through the C ABI of libplc.so) against its CPU oracle.

The two contractions accumulate in fp32 inside the matrix cores, in the hardware's order, so their
results are compared within bounds derived from the arithmetic, and every integer decision that
follows (the symbols) may differ from the fp64 oracle's only at counted rounding near-ties:
  Ebar      equal to the oracle's fp16 value or its fp16 neighbour, the latter rarely;
  symbols   against the oracle fed with the DEVICE's Ebar (so that inputs are identical): differences
            only of one step and only where r/Delta is within tau of a half-integer, tau from the fp32
            accumulation bound of that component;
  streams   histogram, tables, rANS states and words bit-exact given the device's symbols;
  decode    symbols back exactly; output within one fp16 step of the oracle's; |error| <= Delta/2.
"""
import numpy as np
import pytest
import torch

from oracle import plc_oracle_linear as OL
from paper_2604_15356_amd.workloads import make_linear_workload
from tests.gpu_util import u8, u16, u32, u64

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dev():
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    from paper_2604_15356_amd import plc
    plc.lib()
    return torch.device("cuda:0")


CASES = {
    "tiny": None,
    "one_tile": dict(L=1, H=1, d=64, n=128, m=128, V=32, seed=51),
    "wide_heads": dict(S=2, L=1, H=4, d=32, n=128, m=256, V=96, seed=52),
    "d128": dict(L=2, H=1, d=128, n=256, m=384, V=2048, seed=53),
    "noisy": dict(L=1, H=2, d=64, n=128, m=128, V=512, sigma=3.0, seed=54),       # escapes
    # 256 (session, layer) pairs of one 256 x 256 tile each: the second contraction takes the large-tile
    # kernel (slices loaded straight into LDS); K = m = 128 is two slices, 384 six
    "large_tiles": dict(L=256, H=1, d=128, n=256, m=128, V=64, seed=55),
    "large_tiles_k384": dict(S=2, L=128, H=2, d=64, n=256, m=384, V=96, seed=56),
}


def _codec(w, dev):
    from paper_2604_15356_amd.codec import KVDeltaCodec
    return KVDeltaCodec(w.S, w.L, w.H, w.n, 1, w.d, w.delta, w.qmax, device=dev, esc_frac=1.0)


@pytest.mark.parametrize("case", list(CASES))
def test_linear_predictor_encode_decode(oracle, dev, case):
    O = oracle
    w = make_linear_workload("tiny", device=dev, overrides=CASES[case])
    codec = _codec(w, dev)
    print(f"case {case}: S{w.S} L{w.L} H{w.H} n{w.n} d{w.d} m{w.m} V{w.V}", flush=True)
    coded = codec.encode_linear(w.probs_full, w.embed_t, w.A, w.bias_k, w.bias_v, w.act_k, w.act_v)
    codec.check_status("encode_linear")
    host = lambda t: t.contiguous().cpu().numpy()

    # ---- expected embedding
    eb_gpu = host(codec.ebar)
    eb_ref = OL.expected_embedding(host(w.probs_full), host(w.embed_t))
    g, r = eb_gpu.astype(np.float64), eb_ref.astype(np.float64)
    ulp = np.spacing(np.maximum(np.abs(eb_ref), np.float16(2.0 ** -14))).astype(np.float64)
    assert (np.abs(g - r) <= ulp + 1e-12).all()
    assert (eb_gpu.view(np.uint16) != eb_ref.view(np.uint16)).mean() < 0.02

    # ---- symbols, against the oracle on the device's Ebar
    A, bk, bv, ak, av = host(w.A), host(w.bias_k), host(w.bias_v), host(w.act_k), host(w.act_v)
    eb3 = eb_gpu.reshape(w.S, w.n, w.m)
    ref = OL.predict_residual(eb3, A, bk, bv, ak, av, w.delta)
    sym = u8(coded.symbols)
    # fp32 accumulation over m terms: |error| <= m * 2^-24 * sum_j |A_j| |Ebar_j| (plus the final adds)
    mag = np.einsum("lhcem,snm->slhnce", np.abs(A.astype(np.float64)), np.abs(eb3.astype(np.float64)), optimize=True)
    tau = ((w.m + 4) * 2.0 ** -24 * (mag + 8.0) / float(np.float32(w.delta))).reshape(sym.shape)
    diff = sym != ref["symbols"]
    frac = np.abs(ref["u"] - np.floor(ref["u"]) - 0.5)
    a, b = sym.astype(np.int64), ref["symbols"].astype(np.int64)
    one_step = (np.abs(a - b) == 1) | ((a == 255) & ((b >= 253) | (b <= 1))) | ((b == 255) & ((a >= 253) | (a <= 1)))
    print(f"  near-ties vs fp64 oracle: {int(diff.sum())} of {sym.size}", flush=True)
    assert (diff <= ((frac < tau) & one_step)).all()
    assert diff.mean() < 1e-3

    # ---- escapes and streams: bit-exact given the device's symbols
    esc = sym == 255
    raw = np.stack([ak, av], axis=4).view(np.uint16).reshape(sym.shape)
    cnt = esc.sum(1).astype(np.uint32)
    assert np.array_equal(u32(coded.esc_cnt), cnt)
    assert np.array_equal(u64(coded.esc_off), np.cumsum(cnt, dtype=np.uint64) - cnt)
    assert np.array_equal(u16(coded.esc_vals)[:int(cnt.sum())], raw[esc])
    freq, _ = O.build_freq(O.histogram(sym))
    enc = O.rans_encode(sym, freq, word_cap_per_unit=codec.word_cap)
    assert np.array_equal(u16(coded.freq), freq)
    assert np.array_equal(u32(coded.n_words), enc["n_words"]) and np.array_equal(u32(coded.states), enc["states"])
    words = u16(coded.words)
    for unit in range(codec.n_units):
        off, nw = unit * codec.word_cap, int(enc["n_words"][unit])
        assert np.array_equal(words[off:off + nw], enc["words"][off:off + nw])

    # ---- decode: same symbols, output within one fp16 step of the oracle's, error bound
    out_k, out_v = torch.zeros_like(w.act_k), torch.zeros_like(w.act_v)
    codec.decode_linear(w.probs_full, w.embed_t, w.A, w.bias_k, w.bias_v, out_k, out_v)
    codec.check_status("decode_linear")
    assert torch.equal(codec.dec_symbols, coded.symbols)
    rk, rv = OL.reconstruct(eb3, A, bk, bv, sym, raw[esc], w.delta)
    sym6 = sym.reshape(w.S, w.L, w.H, w.n, 2, w.d)
    for c, (out, want, act) in enumerate(((host(out_k), rk, ak), (host(out_v), rv, av))):
        e = sym6[..., c, :] == 255
        assert np.array_equal(out.view(np.uint16)[e], act.view(np.uint16)[e])           # escapes bit-exact
        o, r_ = out.astype(np.float64), want.astype(np.float64)
        ulp = np.maximum(np.abs(r_), 2.0 ** -14) * 2.0 ** -10
        assert (np.abs(o - r_)[~e] <= ulp[~e] + 1e-6).all()
        assert (out.view(np.uint16) != want.view(np.uint16))[~e].mean() < 5e-3
        assert (np.abs(o - act.astype(np.float64))[~e] <= np.float32(w.delta) / 2 + ulp[~e] + 1e-4).all()
    if case == "noisy":
        assert cnt.sum() > 0.01 * sym.size


def test_linear_predictor_is_deterministic_and_rejects_bad_shapes(dev):
    from paper_2604_15356_amd import plc
    w = make_linear_workload("tiny", device=dev, overrides=dict(n=128, seed=55))
    codec = _codec(w, dev)
    a = codec.encode_linear(w.probs_full, w.embed_t, w.A, w.bias_k, w.bias_v, w.act_k, w.act_v)
    first = [t.clone() for t in (codec.ebar, a.symbols, a.states, a.n_words)]
    b = codec.encode_linear(w.probs_full, w.embed_t, w.A, w.bias_k, w.bias_v, w.act_k, w.act_v)
    for x, y in zip(first, (codec.ebar, b.symbols, b.states, b.n_words)):
        assert torch.equal(x, y)
    with pytest.raises(plc.PlcError):                      # vocabulary not a multiple of 32
        plc.plc_expected_embedding(w.probs_full[:, :1000].contiguous(), w.embed_t[:, :1000].contiguous(), codec.ebar)
    with pytest.raises(plc.PlcError):                      # rows not a multiple of 128
        plc.plc_expected_embedding(w.probs_full[:100].contiguous(), w.embed_t, codec.ebar[:100].contiguous())


@pytest.mark.parametrize("V", [32, 64, 96, 416])
def test_expected_embedding_large_tiles(dev, V):
    """The first contraction at an output that divides into 256 x 256 tiles, one per compute unit (the kernel
    whose slices are loaded straight into LDS), with K one short slice, one whole slice, a short and a whole
    one, and several: against numpy in fp64 (numpy.matmul is the oracle's own step here)."""
    from paper_2604_15356_amd import plc
    rows, m = 4096, 4096
    g = torch.Generator(device="cpu").manual_seed(900 + V)
    P = torch.rand((rows, V), generator=g).to(torch.float16)
    P = (P / P.float().sum(dim=1, keepdim=True)).to(torch.float16)
    E = torch.randn((m, V), generator=g).to(torch.float16)
    out = torch.zeros((rows, m), dtype=torch.float16, device=dev)
    print(f"expected embedding {rows} x {m}, V {V}", flush=True)
    plc.plc_expected_embedding(P.to(dev), E.to(dev), out)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    want64 = OL.expected_embedding(P.numpy(), E.numpy()).astype(np.float64)
    exact = P.numpy().astype(np.float64) @ E.numpy().astype(np.float64).T
    assert np.array_equal(want64, exact.astype(np.float16).astype(np.float64))
    # fp32 accumulation of V terms, then one rounding to fp16
    tol = np.spacing(np.maximum(np.abs(want64), 2.0 ** -14).astype(np.float16)).astype(np.float64) \
        + (V + 2) * 2.0 ** -24 * (np.abs(P.numpy().astype(np.float64)) @ np.abs(E.numpy().astype(np.float64)).T)
    assert (np.abs(got.astype(np.float64) - want64) <= tol).all()
    assert (got.view(np.uint16) != want64.astype(np.float16).view(np.uint16)).mean() < 0.02
