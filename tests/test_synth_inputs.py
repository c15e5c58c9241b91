"""The seeded input generators: shapes, dtypes, determinism, stated distributions."""
import numpy as np
import torch

import sr_synth


def _small(name, **kw):
    return sr_synth.scaled(sr_synth.WORKLOADS[name], **kw)


def test_workload_table_matches_the_stated_sizes():
    w = sr_synth.WORKLOADS
    assert (w["tiny"].H, w["tiny"].W, w["tiny"].c) == (128, 128, 1)
    assert (w["720p"].H, w["720p"].W) == (720, 1280)
    assert (w["1080p_fp16"].H, w["1080p_fp16"].W, w["1080p_fp16"].scale) == (1080, 1920, 3)
    assert (w["4k_dense"].H, w["4k_dense"].W) == (2160, 3840)
    assert (w["video"].n, w["video"].L, w["video"].k) == (16, 128, 7)
    # 144 coefficient + 12 output + 0.75 LR bytes per HR pixel at 4K
    assert abs(w["4k_dense"].algorithmic_bytes() / w["4k_dense"].hr_pixels - 156.75) < 1e-9
    assert abs(w["4k_selective"].algorithmic_bytes(8) / w["4k_selective"].hr_pixels - 28.75) < 1e-9


def test_dictionary_atoms_sum_to_one_and_are_not_all_symmetric():
    for name in ("tiny", "video"):
        wl = sr_synth.WORKLOADS[name]
        D = sr_synth.make_dictionary(wl).numpy().astype(np.float64)
        assert D.shape == (wl.L, wl.k, wl.k) and D.dtype == np.float64
        assert np.max(np.abs(D.sum(axis=(1, 2)) - 1.0)) < 1e-5
        assert (D[1::2].min(axis=(1, 2)) < 0).any()          # DoG atoms have negative lobes
        assert np.max(np.abs(D - D.transpose(0, 2, 1))) > 1e-3  # rotated atoms: not symmetric


def test_inputs_are_deterministic_and_distributed_as_stated():
    wl = _small("1080p_fp16", h=8, w=16)
    a = sr_synth.make_inputs(wl)
    b = sr_synth.make_inputs(wl)
    for key in ("lr", "coeff", "dict"):
        assert torch.equal(a[key], b[key])
    assert a["coeff"].dtype == torch.float16 and a["lr"].dtype == torch.float32
    assert a["coeff"].shape == (1, 72, 24, 48)
    s = a["coeff"].double().sum(dim=1)
    assert float((s - 1).abs().max()) < 2e-3
    assert 0.0 <= float(a["lr"].min()) and float(a["lr"].max()) < 1.0


def test_selective_workload_keeps_the_dominant_atoms():
    wl = _small("4k_selective", h=16, w=16)
    inp = sr_synth.make_inputs(wl)
    assert inp["kept"].dtype == np.int32 and len(inp["kept"]) == 8
    assert np.array_equal(inp["kept"], sr_synth.dominant_atoms(wl))
    mass = inp["coeff"].double()[:, inp["kept"].astype(np.int64)].sum(dim=1).mean()
    assert 0.8 < float(mass) < 0.95   # about 87 % of the mass sits in the kept atoms


def test_kept_ties_go_to_the_lower_index():
    mean = np.array([0.1, 0.3, 0.3, 0.05, 0.3])
    assert list(sr_synth.kept_from_mean(mean, 2)) == [1, 2]
