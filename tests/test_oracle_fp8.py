"""Pins of the oracle's 8-bit E4M3 decoder (coefficient storage format): the format's
own definition at hand-computed codes, a library's decoder over all 256 codes, and
that the assembly reads stored E4M3 bytes exactly as it reads their widened values."""
import math

import numpy as np
import pytest

torch = pytest.importorskip("torch")
import sr_synth


def test_hand_computed_codes(oracle):
    d = oracle.e4m3_to_double
    assert d(0x00) == 0.0 and math.copysign(1.0, d(0x80)) == -1.0 and d(0x80) == 0.0
    assert d(0x38) == 1.0 and d(0xB8) == -1.0            # exponent field 7 = bias
    assert d(0x3C) == 1.5 and d(0x40) == 2.0
    assert d(0x01) == 2.0 ** -9                          # smallest subnormal
    assert d(0x07) == 7 * 2.0 ** -9                      # largest subnormal
    assert d(0x08) == 2.0 ** -6                          # smallest normal
    assert d(0x7E) == 448.0 and d(0xFE) == -448.0        # largest finite: no infinities
    assert math.isnan(d(0x7F)) and math.isnan(d(0xFF))
    assert d(0x78) == 256.0                              # exponent field 15 is an ordinary binade


def test_all_codes_against_a_library_decoder(oracle):
    lib = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    for b in range(256):
        mine = oracle.e4m3_to_double(b)
        if math.isnan(lib[b]):
            assert math.isnan(mine), hex(b)
        else:
            assert mine == lib[b], hex(b)


def test_positive_codes_are_strictly_increasing(oracle):
    vals = [oracle.e4m3_to_double(b) for b in range(0x7F)]
    assert all(a < b for a, b in zip(vals, vals[1:]))


def test_assembly_of_stored_bytes_equals_assembly_of_their_widened_values(oracle):
    wl = sr_synth.Workload("f8pin", 21, 2, 3, 6, 9, 3, 19, 5, "f8", "f32")
    inp = sr_synth.make_inputs(wl, "cpu")
    stored = sr_synth.stored_numpy(inp["coeff"])
    assert stored.dtype == np.uint8 and len(np.unique(stored)) > 20
    wide = np.vectorize(oracle.e4m3_to_double)(stored).astype(np.float64)
    lr, D = inp["lr"].numpy(), inp["dict"].numpy()
    a = oracle.dict_assemble(lr, stored, D, wl.scale)
    b = oracle.dict_assemble(lr, wide, D, wl.scale)
    assert np.array_equal(a, b)
    kept = np.array([3, 0, 17], dtype=np.int32)
    gamma = np.array([0.5, -2.0, 1.25])
    assert np.array_equal(oracle.dict_assemble(lr, stored, D, wl.scale, kept=kept, gamma=gamma),
                          oracle.dict_assemble(lr, wide, D, wl.scale, kept=kept, gamma=gamma))


def test_lr_image_cannot_be_stored_as_e4m3(oracle):
    with pytest.raises(TypeError):
        oracle.bicubic(np.zeros((1, 1, 4, 4), dtype=np.uint8), 2)
