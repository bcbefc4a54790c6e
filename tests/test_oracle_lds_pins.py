"""The oracle's LDS-streaming function against its pins (CPU).  The paper defines nothing for
its shared-memory benchmark subject (Table 1 names it and its `rep` parameter only), so the
definition is this library's own and the pins are closed forms of that definition."""
import numpy as np
import pytest

import opal_inputs as oi
import pins
import pins_lds

DTYPES = [np.float64, np.float32]


def _random(dtype):
    return oi.uniform_array(11, 0, 2 * pins_lds.tile_elems(dtype), dtype, -1.0, 1.0)


@pytest.mark.parametrize("dtype", DTYPES)
def test_oracle_passes_the_lds_pins(oracle, dtype):
    pins_lds.run_all(oracle, dtype, _random(dtype))


def test_oracle_rejects_partial_tiles(oracle):
    x = np.zeros(2047)
    with pytest.raises(ValueError):
        oracle.lds_stream(x, np.zeros(2047), 0.1, 1)
    oracle.lds_stream(np.zeros(0), np.zeros(0), 0.1, 5)


class _Good:
    @staticmethod
    def lds_stream(inp, out, c, rep):
        out[:] = pins_lds.add_repeatedly(pins_lds.rotated(inp, rep), c, rep)


def _mut_wrong_direction(inp, out, c, rep):
    out[:] = pins_lds.add_repeatedly(pins_lds.rotated(inp, -rep), c, rep)


def _mut_whole_array_rotation(inp, out, c, rep):
    pv = pins_lds.per_vec(inp.dtype)
    out[:] = pins_lds.add_repeatedly(np.roll(inp.reshape(-1, pv), -rep, axis=0).reshape(-1), c, rep)


def _mut_single_multiply(inp, out, c, rep):
    out[:] = pins_lds.rotated(inp, rep) + inp.dtype.type(c) * inp.dtype.type(rep)


def _mut_element_rotation(inp, out, c, rep):
    t = inp.reshape(-1, pins_lds.tile_elems(inp.dtype))
    out[:] = pins_lds.add_repeatedly(np.roll(t, -rep, axis=1).reshape(-1), c, rep)


def _mut_one_round_short(inp, out, c, rep):
    r = max(rep - 1, 0)
    out[:] = pins_lds.add_repeatedly(pins_lds.rotated(inp, r), c, r)


@pytest.mark.parametrize("dtype", DTYPES)
def test_stand_in_passes(dtype):
    pins_lds.run_all(_Good, dtype, _random(dtype))


@pytest.mark.parametrize("mutant", [_mut_wrong_direction, _mut_whole_array_rotation, _mut_single_multiply,
                                    _mut_element_rotation, _mut_one_round_short])
@pytest.mark.parametrize("dtype", DTYPES)
def test_planted_mistakes_are_caught(mutant, dtype):
    impl = type("Mutant", (), {"lds_stream": staticmethod(mutant)})
    with pytest.raises(pins.PinFailure):
        pins_lds.run_all(impl, dtype, _random(dtype))
