"""MI355X-native pixel-adaptive dictionary assembly (LAPAR-style super-resolution
hot path: up-sample, F = Phi D, y = F B^T) as a C-ABI HIP library plus this thin
ctypes binding.  Import is cheap; the shared library is loaded on first use and
its absence is an error, never a fallback."""
from .binding import (  # noqa: F401
    SR_BF16, SR_COEFF_BLOCKED, SR_COEFF_LOGITS, SR_COEFF_PIXEL_MAJOR, SR_COEFF_PLANAR, SR_COEFF_PRE_SHUFFLE, SR_COEFF_VALUES, SR_F16, SR_F32, SR_F8E4M3, SR_KERNEL_AUTO, SR_KERNEL_GENERIC, SR_KERNEL_MFMA, SR_MAX_ATOMS, SR_U8,
    SrError, describe, load, make_options, sr_bicubic_upsample, sr_dict_assemble,
    sr_dict_assemble_ex, sr_dict_assemble_list, sr_dict_assemble_list_ex, sr_dict_assemble_plan, sr_dict_assemble_tile, sr_dict_assemble_launch_shape, sr_dict_assemble_selective, sr_options,
    sr_atom_gram, sr_atom_gram_static, sr_atom_gram_workspace_bytes, sr_probe_mix, sr_probe_mix_tiled, sr_probe_read, sr_probe_pattern, sr_probe_policy, sr_probe_policy_bits, sr_probe_stream, sr_select_atoms,
    sr_strerror, sr_tensor, sr_version,
)
