"""Pins of the oracle's bfloat16 decoder (coefficient storage format): the format's own
definition at hand-computed codes, the binary32 bit pattern it is the upper half of over all
65536 codes (numpy's own float32 view, not the decoder's arithmetic), a library's decoder,
and that the assembly reads stored bfloat16 exactly as it reads the widened values."""
import math

import numpy as np
import pytest

torch = pytest.importorskip("torch")
import sr_synth


def test_hand_computed_codes(oracle):
    d = oracle.bf16_to_double
    assert d(0x0000) == 0.0 and d(0x8000) == 0.0 and math.copysign(1.0, d(0x8000)) == -1.0
    assert d(0x3F80) == 1.0 and d(0xBF80) == -1.0       # exponent field 127 = bias
    assert d(0x3FC0) == 1.5 and d(0x4000) == 2.0
    assert d(0x4049) == 3.140625                         # 1.5703125 * 2: pi to 8 bits
    assert d(0x0001) == 2.0 ** -133                      # smallest subnormal
    assert d(0x007F) == 127 * 2.0 ** -133                # largest subnormal
    assert d(0x0080) == 2.0 ** -126                      # smallest normal
    assert d(0x7F7F) == (255.0 / 128.0) * 2.0 ** 127     # largest finite
    assert d(0x7F80) == math.inf and d(0xFF80) == -math.inf
    assert math.isnan(d(0x7FC0)) and math.isnan(d(0xFF81))
    assert d(0x3B80) == 2.0 ** -8 and d(0x4780) == 65536.0   # beyond fp16's range on both sides


def test_all_codes_are_the_upper_half_of_a_binary32(oracle):
    codes = np.arange(65536, dtype=np.uint32)
    with np.errstate(invalid="ignore"):                  # signalling NaNs among the codes
        want = (codes << 16).view(np.float32).astype(np.float64)
    for b in range(65536):
        mine = oracle.bf16_to_double(b)
        if math.isnan(want[b]):
            assert math.isnan(mine), hex(b)
        else:
            assert mine == want[b], hex(b)


def test_a_library_decoder_agrees(oracle):
    lib = torch.arange(-32768, 32768, dtype=torch.int16).view(torch.bfloat16).to(torch.float64).numpy()
    bits = np.arange(-32768, 32768, dtype=np.int16).view(np.uint16)
    for b, v in zip(bits[::37], lib[::37]):
        mine = oracle.bf16_to_double(int(b))
        assert (math.isnan(mine) and math.isnan(v)) or mine == v, hex(int(b))


def test_assembly_of_stored_bits_equals_assembly_of_their_widened_values(oracle):
    wl = sr_synth.Workload("bfpin", 22, 2, 3, 6, 9, 3, 19, 5, "bf16", "f32")
    inp = sr_synth.make_inputs(wl, "cpu")
    stored = sr_synth.stored_numpy(inp["coeff"])
    assert stored.dtype == np.uint16 and len(np.unique(stored)) > 100
    wide = inp["coeff"].to(torch.float64).numpy()
    lr, D = inp["lr"].numpy(), inp["dict"].numpy()
    assert np.array_equal(oracle.dict_assemble(lr, stored, D, wl.scale), oracle.dict_assemble(lr, wide, D, wl.scale))
    kept = np.array([3, 0, 17], dtype=np.int32)
    gamma = np.array([0.5, -2.0, 1.25])
    assert np.array_equal(oracle.dict_assemble(lr, stored, D, wl.scale, kept=kept, gamma=gamma),
                          oracle.dict_assemble(lr, wide, D, wl.scale, kept=kept, gamma=gamma))


def test_selection_oracle_reads_stored_bfloat16(oracle):
    from oracle import select_oracle as so
    wl = sr_synth.Workload("bfsel", 23, 1, 2, 5, 7, 2, 6, 3, "bf16", "f32")
    inp = sr_synth.make_inputs(wl, "cpu")
    U = oracle.bicubic(inp["lr"].numpy(), wl.scale)
    target = np.random.default_rng(3).random(U.shape)
    a = so.normal_equations(U, sr_synth.stored_numpy(inp["coeff"]), inp["dict"].numpy(), target, 1)
    b = so.normal_equations(U, inp["coeff"].to(torch.float64).numpy(), inp["dict"].numpy(), target, 1)
    for x, y in zip(a, b):
        assert np.array_equal(np.asarray(x), np.asarray(y))


def test_lr_image_cannot_be_stored_as_bfloat16(oracle):
    with pytest.raises(TypeError):
        oracle.bicubic(np.zeros((1, 1, 4, 4), dtype=np.uint16), 2)
