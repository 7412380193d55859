"""Host-side arithmetic of libplc.so against the oracle (no GPU needed): the thresholds of the
surprisal-adaptive quantiser, which both sides derive from b0 and hbar on their own."""
import numpy as np
import pytest

from paper_2604_15356_amd import plc


@pytest.mark.parametrize("b0,hbar", [(3.0, float(np.log2(15.0))), (2.0, 3.3), (4.0, 4.3), (2.5, 1.0), (1.0, 6.0),
                                     (3.0, float(np.log2(22.5))), (4.0, 0.5), (0.75, 2.0)])
def test_thresholds_equal_the_oracles(oracle, b0, hbar):
    for bmax in range(1, plc.MAX_BITS + 1):
        got = plc.plc_surprisal_thresholds(b0, hbar, bmax)
        want = oracle.surprisal_thresholds(b0, hbar, bmax)
        assert list(got) == [int(t) for t in want]
        assert all(a >= b for a, b in zip(got[2:], got[3:]))            # non-increasing, as plc_surprisal_bits asks


def test_more_depths_than_the_library_codes_are_refused():
    with pytest.raises(plc.PlcError) as e:
        plc.plc_surprisal_thresholds(3.0, 3.9, plc.MAX_BITS + 1)
    assert e.value.code == plc.PLC_ERR_INVALID
