"""The streaming probes read and write what they say they do (they carry the
secondary, empirical roofline in bench.py, so their byte counts must be real)."""
import pytest

torch = pytest.importorskip("torch")
import paper_2303_08999_amd as sr

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("planes,channels,runs", [(72, 3, 9), (128, 1, 2100), (72, 4, 4096)])
def test_mix_probe_touches_every_plane_and_every_output_pixel(planes, channels, runs):
    pixels = 128 * runs
    g = torch.Generator(device="cuda").manual_seed(planes + runs)
    words = torch.randint(0, 2**31 - 1, (planes, pixels // 2), device="cuda", dtype=torch.int32, generator=g)
    out = torch.full((channels, pixels), -1.0, device="cuda")
    sr.sr_probe_mix(words, planes, pixels, out, channels)
    torch.cuda.synchronize()
    # lane j of a run folds words 2j, 2j+1 of every plane; its low byte lands on pixels 4j .. 4j+3
    acc = words[0].clone()
    for p in range(1, planes):
        acc ^= words[p]
    pair = (acc[0::2] ^ acc[1::2]) & 0xFF                      # one value per 4 pixels
    f = pair.to(torch.float32).repeat_interleave(4)
    odd = torch.arange(pixels, device="cuda") % 2 == 1
    for c in range(channels):
        want = torch.where(odd, f + c, f)
        assert torch.equal(out[c], want)


def test_read_probe_runs_on_ragged_sizes_and_leaves_the_sink_alone():
    sink = torch.zeros(4, device="cuda", dtype=torch.int32)
    for nbytes in (16, 4096 * 5 + 16, 256 * 16 * 8 * 3 + 48, 1 << 26):
        src = torch.zeros(nbytes // 4, device="cuda", dtype=torch.int32)
        sr.sr_probe_read(src, sink)
    torch.cuda.synchronize()
    assert int(sink.abs().sum()) == 0
