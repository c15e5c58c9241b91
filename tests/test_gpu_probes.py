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


@pytest.mark.parametrize("planes,channels,H,W,tile_h", [(72, 3, 50, 256, 24), (72, 3, 61, 128, 16), (128, 2, 9, 384, 4), (72, 1, 3, 128, 1),
                                                        (72, 3, 700, 1280, 24)])
def test_tiled_mix_probe_writes_what_the_flat_one_writes(planes, channels, H, W, tile_h):
    """The probe that walks the frame in the kernel's tile order reads the same planes and writes the same
    values as the flat one: every output pixel once, whatever the tile height and the ragged last tile row."""
    pixels = H * W
    g = torch.Generator(device="cuda").manual_seed(planes + H)
    words = torch.randint(0, 2**31 - 1, (planes, pixels // 2), device="cuda", dtype=torch.int32, generator=g)
    flat = torch.full((channels, pixels), -1.0, device="cuda")
    tiled = torch.full((channels, pixels), -2.0, device="cuda")
    sr.sr_probe_mix(words, planes, pixels, flat, channels)
    sr.sr_probe_mix_tiled(words, planes, H, W, tile_h, tiled, channels)
    torch.cuda.synchronize()
    assert torch.equal(flat, tiled)
    # with the L2 write-back pacing among its requests (a period short enough to fire): the same values
    paced = torch.full((channels, pixels), -3.0, device="cuda")
    sr.sr_probe_mix_tiled(words, planes, H, W, tile_h, paced, channels, pace_us=1)
    torch.cuda.synchronize()
    assert torch.equal(flat, paced)


@pytest.mark.parametrize("planes,channels,H,W,tile_h", [(72, 3, 50, 256, 24), (128, 2, 9, 384, 4), (72, 3, 700, 1280, 24)])
def test_tiled_mix_probe_for_one_byte_coefficients(planes, channels, H, W, tile_h):
    """Planes of 8-bit coefficients: a lane reads the 4 bytes of its four pixels from every plane; the written value is the
    low byte of the exclusive-or of those words over all planes, as in the two-byte form."""
    pixels = H * W
    g = torch.Generator(device="cuda").manual_seed(planes + H)
    words = torch.randint(0, 2**31 - 1, (planes, pixels // 4), device="cuda", dtype=torch.int32, generator=g)
    out = torch.full((channels, pixels), -2.0, device="cuda")
    sr.sr_probe_mix_tiled(words, planes, H, W, tile_h, out, channels, elem_bytes=1)
    torch.cuda.synchronize()
    acc = words[0].clone()
    for p in range(1, planes):
        acc ^= words[p]
    f = (acc & 0xFF).to(torch.float32).repeat_interleave(4)                      # one value per 4 pixels
    odd = torch.arange(pixels, device="cuda") % 2 == 1
    for c in range(channels):
        assert torch.equal(out[c], torch.where(odd, f + c, f))


def test_read_probe_runs_on_ragged_sizes_and_leaves_the_sink_alone():
    sink = torch.zeros(4, device="cuda", dtype=torch.int32)
    for nbytes in (16, 4096 * 5 + 16, 256 * 16 * 8 * 3 + 48, 1 << 26):
        src = torch.zeros(nbytes // 4, device="cuda", dtype=torch.int32)
        sr.sr_probe_read(src, sink)
    torch.cuda.synchronize()
    assert int(sink.abs().sum()) == 0


def _filled(nbytes):
    return torch.full((nbytes // 4,), -1, device="cuda", dtype=torch.int32)       # every byte 0xff


@pytest.mark.parametrize("blocks,writer_every,nt,lds", [(16, 1, 0, 0), (40, 13, 1, 0), (9, 2, 0, 96 * 1024), (512, 7, 1, 0)])
def test_stream_probe_writes_every_word_once_and_reads_in_bounds(blocks, writer_every, nt, lds):
    write_bytes, read_bytes = 16 * 70001, 16 * 123457
    src = torch.zeros(read_bytes // 4, device="cuda", dtype=torch.int32)
    dst = _filled(write_bytes)
    sink = torch.zeros(4, device="cuda", dtype=torch.int32)
    rd = 0 if writer_every == 1 else read_bytes
    sr.sr_probe_stream(src if rd else None, rd, dst, write_bytes, blocks, writer_every, sink, lds_bytes=lds, nt_store=nt)
    torch.cuda.synchronize()
    q = dst.view(-1, 4)
    assert torch.all(q[:, 2] == 0x3F800000) and torch.all(q[:, 3] == 0)           # the writers' marker in every 16 bytes
    assert int(sink.abs().sum()) == 0
    # read only: nothing may be written
    dst2 = _filled(1024)
    sr.sr_probe_stream(src, read_bytes, None, 0, blocks, 0, sink, lds_bytes=lds)
    torch.cuda.synchronize()
    assert torch.all(dst2 == -1)


@pytest.mark.parametrize("read_planes,write_planes,same_wave,blocks,writer_every", [
    (0, 0, 1, 8, 0), (0, 0, 0, 27, 13), (1, 1, 1, 64, 0), (1, 0, 0, 26, 2), (0, 1, 0, 9, 9),
    (2, 1, 1, 7, 0), (3, 1, 1, 33, 0), (4, 1, 1, 5, 0), (1, 3, 1, 16, 0), (2, 3, 1, 16, 0), (0, 3, 1, 16, 0)])
def test_pattern_probe_covers_the_output_and_nothing_else(read_planes, write_planes, same_wave, blocks, writer_every):
    pixels, pad = 512 * 37, (1152 if read_planes else 0)
    src = torch.zeros(72 * (2 * pixels + pad) // 4, device="cuda", dtype=torch.int32)
    buf = _filled(12 * pixels + 64)                                                # 64 guard bytes behind the output
    sink = torch.zeros(4, device="cuda", dtype=torch.int32)
    sr.sr_probe_pattern(src, buf, pixels, read_planes, write_planes, same_wave, blocks, writer_every, sink, plane_pad_bytes=pad)
    torch.cuda.synchronize()
    out = buf[:3 * pixels].view(torch.float32)
    assert bool(torch.isfinite(out).all()) and float(out.min()) >= 0.0             # every word overwritten with a small value
    assert torch.all(buf[3 * pixels:] == -1)
    if write_planes:                                                               # read only: untouched
        before = _filled(12 * pixels)
        sr.sr_probe_pattern(src, before, pixels, read_planes, 2, 1, blocks, 0, sink, plane_pad_bytes=pad)
        torch.cuda.synchronize()
        assert torch.all(before == -1)


@pytest.mark.parametrize("flush_every", [0, 3])
def test_policy_probes_cover_the_output(flush_every):
    pixels = 128 * 531
    src = torch.zeros(144 * pixels // 4, device="cuda", dtype=torch.int32)
    sink = torch.zeros(4, device="cuda", dtype=torch.int32)
    for lp, sp in ((0, 0), (1, 2), (2, 1), (3, 3)):
        buf = _filled(12 * pixels + 64)
        sr.sr_probe_policy(src, buf, pixels, lp, sp, flush_every, 8, sink)
        torch.cuda.synchronize()
        assert bool(torch.isfinite(buf[:3 * pixels].view(torch.float32)).all()) and torch.all(buf[3 * pixels:] == -1)
    if flush_every == 0:
        for lp in range(8):
            buf = _filled(12 * pixels + 64)
            sr.sr_probe_policy_bits(src, buf, pixels, lp, 7 - lp, 12, sink)
            torch.cuda.synchronize()
            assert bool(torch.isfinite(buf[:3 * pixels].view(torch.float32)).all()) and torch.all(buf[3 * pixels:] == -1)
