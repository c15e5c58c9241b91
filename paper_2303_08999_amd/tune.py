"""Tile-shape selection by measurement.

The paper picks the launch shape of its filtering engine with a constrained
search (section III-B, Eq. 11-12, then Bayesian optimisation over block
dimensions).  On MI355X the feasible set is small - a handful of compiled tile
shapes that satisfy the LDS and register budgets - so it is swept exhaustively:
every shape `sr_dict_assemble_plan` accepts is timed on the caller's own
tensors and the fastest index is returned for `sr_options.tile`.
"""
from __future__ import annotations

from . import binding as _b


def sweep_tiles(lr, coeff, dict, L, k, scale, channels, out, kept=None, gamma=None,
                reps: int = 5, max_tiles: int = 10):
    """Time every launch shape (tile, workgroup size, residency) of the matrix-core kernel for these arguments.

    Returns a list of (tile index, median milliseconds); empty if the
    matrix-core kernel does not take the case.  `out` is overwritten."""
    import torch

    results = []
    for tile in range(max_tiles):
        opts = _b.make_options(_b.SR_KERNEL_MFMA, tile)
        if _b.sr_dict_assemble_plan(lr, coeff, dict, L, k, scale, channels, out, kept=kept, opts=opts) \
                != _b.SR_KERNEL_MFMA:
            continue                   # an index this case does not have (never a second name for another kernel)

        def run():
            _b.sr_dict_assemble_ex(lr, coeff, dict, L, k, scale, channels, out,
                                   kept=kept, gamma=gamma, opts=opts)
        run()
        torch.cuda.synchronize()
        times = []
        for _ in range(reps):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            run()
            b.record()
            torch.cuda.synchronize()
            times.append(a.elapsed_time(b))
        times.sort()
        results.append((tile, times[len(times) // 2]))
    return results


def best_tile(*args, **kwargs) -> int:
    """Index of the fastest tile shape (0, the library default, if none applies)."""
    res = sweep_tiles(*args, **kwargs)
    return min(res, key=lambda r: r[1])[0] if res else 0
