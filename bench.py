#!/usr/bin/env python3
"""Benchmark of the fused bicubic + dictionary-assembly hot path on one MI355X.

One "step" is one pass of the whole path (stage 1 up-sampling, stage 3
F = Phi D, stage 4 y = F B^T) over one synthetic 4K x4 frame: 3-channel 960x540
LR -> 3840x2160 HR, L = 72 atoms of 5x5, fp16 coefficients, fp32 accumulation.
Inputs are resident in HBM before the timed region; three coefficient tensors
(1.19 GB each) are rotated so no launch re-reads a cached tensor.

Prints ONE JSON line: whole-job HR Mpixel/s, the HBM roofline of the dominant
kernel (algorithmic bytes / HIP-event time of the launches), and the CPU
oracle timed on a bounded sample of the same frame.
"""
import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0       # MI355X HBM3E, published peak
N_ROTATE = 3


def read_traffic(workload):
    """HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE / WRITE_SIZE),
    taken from the committed summary if there is one; else None."""
    path = os.path.join(ROOT, "profiles", f"sr_mfma_{workload}_traffic.txt")
    try:
        m = re.search(r"^traffic_bytes_per_launch\s*[:=]\s*([0-9.eE+]+)", open(path).read(), re.M)
        return float(m.group(1)) if m else None
    except OSError:
        return None


def empirical_ceilings(sr, torch, wl, coeffs, outs, kernel_ms, inp_lr, inp_dict):
    """Secondary roofline context: the machine's own streaming rates for this byte mix,
    from the library's probes (no arithmetic in them), timed like the kernel."""
    if wl.coeff_dtype not in ("f16", "bf16", "f8") or wl.L not in (72, 128) or wl.hr_pixels % 128 or outs[0].dtype != torch.float32:
        return None
    eb = coeffs[0].element_size()                    # the flat mix probe reads two-byte coefficients only
    sink = torch.zeros(4, device="cuda", dtype=torch.int32)

    def timed(fn, reps=20):
        for i in range(3):
            fn(i)
        torch.cuda.synchronize()
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        for i, (a, b) in enumerate(ev):
            a.record(); fn(i); b.record()
        torch.cuda.synchronize()
        return sum(a.elapsed_time(b) for a, b in ev) / reps

    px = wl.hr_pixels // wl.n
    coeff_bytes = wl.L * px * eb
    t_read = timed(lambda i: sr.sr_probe_read(coeffs[i % len(coeffs)][0], sink))
    t_mix = timed(lambda i: sr.sr_probe_mix(coeffs[i % len(coeffs)][0], wl.L, px, outs[i % 2][0], wl.c)) if eb == 2 else None
    mix_bytes = coeff_bytes + wl.c * px * 4
    # the same requests in the kernel's own order: its tiles (height reported by the library, 16 where it reports none),
    # its split of the tiles over the XCDs, its rows per wavefront
    t_tiled = None
    if wl.W % 128 == 0:
        shape = sr.sr_dict_assemble_launch_shape(inp_lr, coeffs[0], inp_dict, wl.L, wl.k, wl.scale, wl.c, outs[0])[1]
        # (the 8-bit family has one built shape per case and reports none: 128 x 24 at scale 4 on large frames)
        tile_h = shape[1] if shape[0] == 128 else (24 if eb == 1 and wl.scale == 4 and wl.hr_pixels > 400000 else 16)
        t_tiled = timed(lambda i: sr.sr_probe_mix_tiled(coeffs[i % len(coeffs)][0], wl.L, wl.H, wl.W, tile_h, outs[i % 2][0], wl.c,
                                                        elem_bytes=eb))
        t_paced = timed(lambda i: sr.sr_probe_mix_tiled(coeffs[i % len(coeffs)][0], wl.L, wl.H, wl.W, tile_h, outs[i % 2][0], wl.c,
                                                        elem_bytes=eb, pace_us=16))
    # the same bytes with nothing of the kernel's access pattern: 16-byte accesses, readers and
    # writers in separate workgroups, two workgroups per CU, every 9th one a writer
    t_stream = timed(lambda i: sr.sr_probe_stream(coeffs[i % len(coeffs)][0], coeff_bytes, outs[i % 2][0], wl.c * px * 4,
                                                  512, 9, sink, nt_store=1))
    return {"read_only_GBps": round(coeff_bytes / t_read / 1e6, 1),
            "mix_GBps": round(mix_bytes / t_mix / 1e6, 1) if t_mix else None, "mix_ms": round(t_mix, 4) if t_mix else None,
            "kernel_time_over_mix_time": round(kernel_ms * 1.0 / (t_mix * wl.n), 3) if t_mix else None,
            "tiled_mix_ms": round(t_tiled, 4) if t_tiled else None,
            "kernel_time_over_tiled_mix_time": round(kernel_ms * 1.0 / (t_tiled * wl.n), 3) if t_tiled else None,
            "tiled_mix_paced_ms": round(t_paced, 4) if t_tiled else None,
            "kernel_time_over_tiled_mix_paced_time": round(kernel_ms * 1.0 / (t_paced * wl.n), 3) if t_tiled else None,
            "independent_mix_GBps": round(mix_bytes / t_stream / 1e6, 1), "independent_mix_ms": round(t_stream, 4),
            "kernel_time_over_independent_mix_time": round(kernel_ms * 1.0 / (t_stream * wl.n), 3),
            "note": "streaming probes of the same library on one frame's coefficient planes: read-only; the kernel's "
                    "own read + write pattern with no arithmetic, run by run (mix) and in the kernel's own tile order (tiled_mix: what is "
                    "left of the kernel when only its memory requests remain; tiled_mix_paced: with the kernel's L2 write-back "
                    "pacing, every 16 us, among them); and the same bytes with 16-byte accesses by "
                    "separate reader and writer workgroups (independent_mix), whose writers finish before its readers, so "
                    "that part of the reading runs undisturbed"}


def probe_study(sr, torch, hr_h=2160, hr_w=3840):
    """What the memory system delivers for the 4K frame's byte mix (72 fp16 planes read, 3 fp32
    planes written) under access patterns of increasing likeness to the assembly kernel's, timed
    like the kernel (HIP events, three rotating source buffers).  Times in microseconds."""
    px = hr_h * hr_w
    rb, wb = 144 * px, 12 * px
    srcs = [torch.empty(rb, device="cuda", dtype=torch.uint8).random_(0, 255) for _ in range(3)]
    dsts = [torch.empty(wb, device="cuda", dtype=torch.uint8) for _ in range(2)]
    sink = torch.zeros(4, device="cuda", dtype=torch.int32)

    def timed(fn, reps=12):
        for i in range(3):
            fn(i)
        torch.cuda.synchronize()
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        for i, (a, b) in enumerate(ev):
            a.record(); fn(i); b.record()
        torch.cuda.synchronize()
        ms = sorted(a.elapsed_time(b) for a, b in ev)
        return round(ms[len(ms) // 2] * 1e3, 1)

    S, D = (lambda i: srcs[i % 3]), (lambda i: dsts[i % 2])
    out = {"pixels": px, "read_bytes": rb, "write_bytes": wb}
    out["stream_read_only_one_workgroup_per_cu"] = {
        nb: timed(lambda i: sr.sr_probe_stream(S(i), rb, None, 0, nb, 0, sink, lds_bytes=96 * 1024))
        for nb in (64, 128, 192, 256)}
    out["stream_read_only_512_blocks"] = timed(lambda i: sr.sr_probe_stream(S(i), rb, None, 0, 512, 0, sink))
    out["stream_write_only_1024_blocks"] = timed(lambda i: sr.sr_probe_stream(None, 0, D(i), wb, 1024, 1, sink))
    out["stream_mix_512_blocks"] = {
        f"writer_every_{we}_nt_{nt}": timed(lambda i: sr.sr_probe_stream(S(i), rb, D(i), wb, 512, we, sink, nt_store=nt))
        for we in (7, 9, 13) for nt in (0, 1)}
    names = {0: "contiguous_16B", 1: "two_planes_per_load_8B_256B_pieces", 2: "two_planes_per_load_16B_512B_pieces",
             3: "one_plane_per_load_8B_512B_pieces"}
    out["pattern_same_wave_512_blocks"] = {
        names[rp]: {"read_write": timed(lambda i: sr.sr_probe_pattern(S(i), D(i), px, rp, 1, 1, 512, 0, sink)),
                    "read_write_stores_through_l2": timed(lambda i: sr.sr_probe_pattern(S(i), D(i), px, rp, 3, 1, 512, 0, sink)),
                    "read_only": timed(lambda i: sr.sr_probe_pattern(S(i), D(i), px, rp, 2, 1, 512, 0, sink))}
        for rp in (0, 1, 2, 3)}
    out["pattern_separate_writers_512_blocks"] = {
        f"read_planes_{rp}_write_planes_{wp}_writer_every_13":
            timed(lambda i: sr.sr_probe_pattern(S(i), D(i), px, rp, wp, 0, 512, 13, sink))
        for rp in (0, 1) for wp in (0, 1)}
    bit = lambda b: "+".join(n for k, n in ((1, "sc0"), (2, "sc1"), (4, "nt")) if b & k) or "plain"
    out["kernel_pattern_cache_policy_bits"] = {
        f"loads_{bit(lp)}": {f"stores_{bit(sp)}": timed(lambda i: sr.sr_probe_policy_bits(S(i), D(i), px, lp, sp, 512, sink), reps=8)
                             for sp in range(8)} for lp in (0, 4, 6)}
    out["kernel_pattern_l2_write_back_every_n_runs"] = {
        fe: timed(lambda i: sr.sr_probe_policy(S(i), D(i), px, 1, 0, fe, 512, sink)) for fe in (0, 1, 2, 4, 16)}
    out["kernel_pattern_probe_sr_probe_mix"] = timed(lambda i: sr.sr_probe_mix(S(i), 72, px, D(i), 3))
    out["kernel_order_probe_sr_probe_mix_tiled"] = {
        f"tile_128x{th}": timed(lambda i: sr.sr_probe_mix_tiled(S(i), 72, hr_h, hr_w, th, D(i), 3)) for th in (4, 8, 16, 24, 32)}
    return out


def table1_sweep(sr, torch, sr_synth):
    """The compression-ratio ablation (the paper's Fig. 7: time of dictionary query + filtering against the
    share of atoms kept) at the input sizes and scales of its Table I, for fp32 coefficients (the paper's
    precision) and fp16.  Random kept lists with regression scales gamma drawn from U[0.5, 1.5] (section III-A,
    Eq. 9); microseconds per launch (median of 20), three rotating coefficient tensors where they fit."""
    import numpy as np
    rng = np.random.default_rng(7)
    lists = {n: np.sort(rng.choice(72, size=n, replace=False)).astype(np.int32) for n in (72, 58, 43, 29, 14, 8)}
    gammas = {n: rng.uniform(0.5, 1.5, size=n).astype(np.float32) for n in lists}
    rows = []
    for (h, w) in ((64, 64), (128, 128), (180, 320), (360, 640)):
        for scale in (2, 3, 4):
            for cd in ("f32", "f16"):
                wl = sr_synth.Workload("table1", 40, 1, 3, h, w, scale, 72, 5, cd, "f32")
                inp = sr_synth.make_inputs(wl, "cuda")
                coeffs = [inp["coeff"]] + [sr_synth.make_coeff(sr_synth.scaled(wl, index=wl.index + 10 * r), "cuda")
                                           for r in (1, 2)]
                out = torch.empty((1, 3, wl.H, wl.W), device="cuda")
                row = {"lr": f"{w}x{h}", "scale": scale, "coeff": cd, "us": {}}
                for n_keep, klist in lists.items():
                    def run(i):
                        sr.sr_dict_assemble_ex(inp["lr"], coeffs[i % 3], inp["dict"], 72, 5, scale, 3, out, kept=klist,
                                               gamma=gammas[n_keep])
                    for i in range(3):
                        run(i)
                    torch.cuda.synchronize()
                    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(20)]
                    for i, (a, b) in enumerate(ev):
                        a.record(); run(i); b.record()
                    torch.cuda.synchronize()
                    ms = sorted(a.elapsed_time(b) for a, b in ev)
                    row["us"][n_keep] = round(ms[10] * 1e3, 1)
                row["speedup_at_8_of_72"] = round(row["us"][72] / row["us"][8], 2)
                rows.append(row)
                del inp, coeffs, out
                torch.cuda.empty_cache()
    return rows


def list_leg(sr, torch, sr_synth, wl, inp, coeffs, entries):
    """The per-pixel list form (an extension beyond the paper): each pixel's `entries` largest coefficients
    as (atom index, value) pairs, timed like the kernel on the same frame."""
    lists = [sr_synth.to_list(c, entries) for c in coeffs]
    out = torch.empty((wl.n, wl.c, wl.H, wl.W), device="cuda", dtype=inp["lr"].dtype)

    def run(i):
        idx, val = lists[i % len(lists)]
        sr.sr_dict_assemble_list(inp["lr"], idx, val, inp["dict"], wl.L, wl.k, wl.scale, wl.c, entries, out)
    for i in range(3):
        run(i)
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(20)]
    torch.cuda.synchronize()
    for i, (a, b) in enumerate(ev):
        a.record(); run(i); b.record()
    torch.cuda.synchronize()
    ms = sum(a.elapsed_time(b) for a, b in ev) / len(ev)
    b_io = 2 if wl.lr_dtype == "f16" else 4
    vb = lists[0][1].element_size()
    nbytes = wl.hr_pixels * (entries * (1 + vb) + wl.c * b_io + wl.c * b_io / wl.scale ** 2)
    flop = wl.hr_pixels * 2.0 * (entries * wl.k ** 2 + wl.c * wl.k ** 2)
    return {"entries": entries, "kernel_ms_avg": round(ms, 4), "hr_mpixel_per_s": round(wl.hr_pixels / ms / 1e3, 1),
            "algorithmic_bytes": nbytes,
            "roofline": {"bound": "alu", "achieved": round(flop / ms / 1e9, 2), "peak": 157.3, "unit": "TFLOP/s",
                         "frac": round(flop / ms / 1e9 / 157.3, 4),
                         "note": "fp32 multiply-adds of the fold and the filtering against the fp32 vector peak; the kernel's "
                                 "own bound is the LDS gather of one dictionary row per entry (entries * k*k * 4 bytes per "
                                 "pixel), HBM is at " + str(round(nbytes / ms / 1e6 / 8000.0, 3)) + " of its peak"}}


def selection_leg(sr, torch, wl, inp, stride):
    """Offline selection on the workload's own frame: the target is the dense result, so the
    search answers "which 10 % of the atoms, rescaled, reproduce the full dictionary best"."""
    shape = (wl.n, wl.c, wl.H, wl.W)
    up, target = torch.empty(shape, device="cuda"), torch.empty(shape, device="cuda")
    sr.sr_bicubic_upsample(inp["lr"], wl.scale, wl.c, up)
    sr.sr_dict_assemble(inp["lr"], inp["coeff"], inp["dict"], wl.L, wl.k, wl.scale, wl.c, target)
    ws = torch.empty(sr.sr_atom_gram_workspace_bytes(wl.L), device="cuda", dtype=torch.uint8)
    nm = torch.empty(wl.L * wl.L + wl.L + 2, device="cuda", dtype=torch.float64)
    run = lambda: sr.sr_atom_gram(up, inp["coeff"], inp["dict"], target, wl.L, wl.k, wl.c, stride,
                                  workspace=ws, normal=nm)
    for _ in range(2):
        run()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    a.record()
    for _ in range(5):
        run()
    b.record()
    torch.cuda.synchronize()
    ms = a.elapsed_time(b) / 5
    host = nm.cpu().numpy()
    samples = float(host[-1])
    cols = wl.L + 1                                                           # atoms plus the target column
    flop = samples * (2.0 * wl.L * wl.k * wl.k + 2.0 * cols * (cols + 1) / 2)  # responses + upper triangle of the Gram matrix
    t0 = time.perf_counter()
    kept, gamma, lam = sr.sr_select_atoms(host, wl.L, alpha=0.1, delta_alpha=0.1)
    t_host = time.perf_counter() - t0
    return {"stride": stride, "samples": int(samples), "gram_ms": round(ms, 4),
            "roofline": {"bound": "mfma", "achieved": round(flop / ms / 1e9, 2), "peak": 157.3, "unit": "TFLOP/s",
                         "frac": round(flop / ms / 1e9 / 157.3, 4),
                         "note": "useful flops (responses + upper triangle of the Gram matrix); both run on the "
                                 "fp32 matrix cores for lattice strides up to 4, the responses on the fp32 vector "
                                 "ALU beyond; the matrix cores execute 1.35 x the useful flops (16-wide padding)"},
            "host_search_s": round(t_host, 3), "kept": [int(v) for v in kept],
            "gamma": [round(float(g), 4) for g in gamma], "lambda": lam}


def bicubic_leg(sr, torch, wl, inp):
    """The bicubic-only entry point (stage 1 alone) on the workload's frame."""
    out = torch.empty((wl.n, wl.c, wl.H, wl.W), device="cuda", dtype=inp["lr"].dtype)
    run = lambda: sr.sr_bicubic_upsample(inp["lr"], wl.scale, wl.c, out)
    for _ in range(3):
        run()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(20)]
    torch.cuda.synchronize()
    for a, b in ev:
        a.record(); run(); b.record()
    torch.cuda.synchronize()
    ms = sum(a.elapsed_time(b) for a, b in ev) / len(ev)
    nbytes = out.numel() * out.element_size() + inp["lr"].numel() * inp["lr"].element_size()
    return {"kernel_ms_avg": round(ms, 4), "hr_mpixel_per_s": round(wl.n * wl.H * wl.W / ms / 1e3, 1),
            "roofline": {"bound": "hbm", "achieved": round(nbytes / ms / 1e6, 1), "peak": 8000.0, "unit": "GB/s",
                         "frac": round(nbytes / ms / 1e6 / 8000.0, 4),
                         "note": "algorithmic bytes: the LR image once, the up-sampled image once"}}


def sr_synth_stored(t):
    import sr_synth
    return sr_synth.stored_numpy(t)


def cpu_baseline(wl, lr, coeff, dictionary, budget_s=20.0, single_thread_720p=True):
    """The oracle as it stands, on the host cores, on a band of HR rows of the same
    frame sized to take roughly `budget_s` of CPU work."""
    import numpy as np
    import oracle
    oracle.build()
    lr_h = lr.cpu().numpy()
    d_h = dictionary.cpu().numpy()
    c_h = sr_synth_stored(coeff)
    threads = oracle.threads()
    t0 = time.perf_counter()
    U = oracle.bicubic(lr_h, wl.scale)
    t_up = time.perf_counter() - t0
    # calibrate on 16 rows, then size the band
    t0 = time.perf_counter()
    oracle.assemble(U, c_h, d_h, rows=(0, 16))
    per_row = (time.perf_counter() - t0) / 16
    rows = int(max(16, min(wl.H, budget_s / max(per_row, 1e-9))))
    # repeat the band until about half the budget is spent (at most 16 passes): a
    # whole 4K frame takes the oracle well under a second on a many-core host
    passes, t_band = 0, 0.0
    while passes < 16 and (passes == 0 or t_band < 0.5 * budget_s):
        t0 = time.perf_counter()
        oracle.assemble(U, c_h, d_h, rows=(0, rows))
        t_band += time.perf_counter() - t0
        passes += 1
    # stage 1 is charged in proportion to the band
    t_total = t_band / passes + t_up * rows / wl.H
    mpx = rows * wl.W * wl.n / t_total / 1e6
    single = None
    if single_thread_720p:
        # the same oracle on ONE thread, whole 720p frame (fp32 coefficients) of the workload list
        import sr_synth
        w7 = sr_synth.WORKLOADS["720p"]
        i7 = sr_synth.make_inputs(w7, "cpu")
        oracle.set_threads(1)
        t0 = time.perf_counter()
        oracle.dict_assemble(i7["lr"].numpy(), i7["coeff"].numpy(), i7["dict"].numpy(), w7.scale)
        t1 = time.perf_counter() - t0
        oracle.set_threads(threads)
        single = {"value": round(w7.hr_pixels / t1 / 1e6, 3), "unit": "HR Mpixel/s", "cores": 1,
                  "sample": f"whole 720p frame ({w7.hr_pixels} pixels, fp32 coefficients), {t1:.2f} s"}
    return {"value": round(mpx, 3), "unit": "HR Mpixel/s", "cores": threads, "kind": "oracle",
            "single_thread": single,
            "sample": f"HR rows 0..{rows - 1} of {wl.H} of the same 4K frame ({rows * wl.W} pixels), "
                      f"double precision, OpenMP over rows; mean of {passes} passes, {t_total:.2f} s each"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=60)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="4k_dense")
    ap.add_argument("--kernel", type=int, default=0, help="0 auto, 1 generic, 2 mfma")
    ap.add_argument("--tile", type=int, default=0)
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle leg")
    ap.add_argument("--cpu-budget", type=float, default=20.0)
    ap.add_argument("--kept-sweep", action="store_true",
                    help="also time kept-atom lists of 72, 58, 43, 29, 14 and 8 atoms (the paper's "
                         "compression-ratio ablation, Fig. 7) and add them to the JSON line")
    ap.add_argument("--selection", type=int, default=0, metavar="STRIDE",
                    help="also time the offline dictionary selection (section III-A, Alg. 1) on this frame: "
                         "normal equations on the GPU over every STRIDE-th row and column, then the host search")
    ap.add_argument("--bicubic", action="store_true",
                    help="also time the bicubic-only entry point (stage 1 alone) on this frame")
    ap.add_argument("--pre-shuffle", action="store_true",
                    help="hand the coefficients over as the coefficient network holds them before its pixel-shuffle "
                         "layer, [N][L*s*s][h][w] (section II-B, stage 2); same values, same result")
    ap.add_argument("--lib", default=None, metavar="PATH",
                    help="load this build of the library instead of the in-tree one (measurement builds "
                         "with a part of the kernel switched off, see sr_mfma_kernel.h)")
    ap.add_argument("--probe-study", action="store_true",
                    help="instead of the kernel, time the library's streaming probes on the 4K frame's byte mix "
                         "and print them as one JSON line")
    ap.add_argument("--pixel-major", action="store_true",
                    help="hand the coefficients over stored pixel-major, [N][H][W][L] (what a channels-last producer writes; "
                         "a storage order beyond the paper); same values, same result")
    ap.add_argument("--blocked", action="store_true",
                    help="hand the coefficients over stored blocked (SR_COEFF_BLOCKED: the order in which the matrix-core kernel "
                         "consumes them; a storage order beyond the paper); same values, same result")
    ap.add_argument("--logits", action="store_true",
                    help="hand the coefficients over as logits (an extension beyond the paper): the call applies the "
                         "per-pixel softmax over the atoms itself")
    ap.add_argument("--tile-sweep", action="store_true",
                    help="also time every launch shape (tile, workgroup size, residency) the library has for this "
                         "workload: the measured stand-in for the paper's launch-shape search (section III-B)")
    ap.add_argument("--table1-sweep", action="store_true",
                    help="instead of the kernel, time kept lists of 72 ... 8 atoms at the paper's Table I input sizes "
                         "and scales (the analogue of its Fig. 7) and print them as one JSON line")
    ap.add_argument("--list", type=int, default=0, metavar="ENTRIES", dest="list_entries",
                    help="also time the per-pixel list form (an extension beyond the paper): each pixel's ENTRIES "
                         "largest coefficients as (atom index, value) pairs")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (a known-size kernel that scales the "
                         "FETCH_SIZE / WRITE_SIZE counters when profiling)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build measures ONE GPU; the path shards over HR row bands with no "
                 "exchange step and no multi-GPU run is part of it (got --gpus %d)" % args.gpus)

    import torch
    import paper_2303_08999_amd as sr
    import sr_synth

    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    if args.lib:
        from paper_2303_08999_amd import binding
        binding.LIB_PATH = os.path.abspath(args.lib)
    sr.load()
    if args.table1_sweep:
        print(json.dumps({"table1_kept_sweep": table1_sweep(sr, torch, sr_synth)}))
        return
    if args.probe_study:
        print(json.dumps({"probe_study_us": probe_study(sr, torch)}))
        return
    wl = sr_synth.WORKLOADS[args.workload]
    dev = "cuda"
    inp = sr_synth.make_inputs(wl, dev)
    kept = inp.get("kept")
    if args.logits:
        assert kept is None, "--logits: the softmax runs over all atoms"
        inp["coeff"] = sr_synth.make_logits(wl, dev)
    coeffs = [inp["coeff"]]
    for r in range(1, N_ROTATE):
        make = sr_synth.make_logits if args.logits else sr_synth.make_coeff
        coeffs.append(make(sr_synth.scaled(wl, index=wl.index + 10 * r), dev))
    outs = [torch.empty((wl.n, wl.c, wl.H, wl.W), device=dev, dtype=inp["lr"].dtype) for _ in range(2)]
    layout = sr.SR_COEFF_PRE_SHUFFLE if args.pre_shuffle else (sr.SR_COEFF_PIXEL_MAJOR if args.pixel_major else
                                                               (sr.SR_COEFF_BLOCKED if args.blocked else sr.SR_COEFF_PLANAR))
    if args.blocked:
        for r in range(len(coeffs)):
            coeffs[r] = sr_synth.to_blocked(coeffs[r])
        inp["coeff"] = coeffs[0]
        args.pre_shuffle = True            # from here on: "not the planar layout" (the extra legs below are planar-only)
    elif args.pixel_major:
        for r in range(len(coeffs)):
            coeffs[r] = sr_synth.to_pixel_major(coeffs[r])
        inp["coeff"] = coeffs[0]
        args.pre_shuffle = True            # from here on: "not the planar layout" (the extra legs below are planar-only)
    elif args.pre_shuffle:
        for r in range(N_ROTATE):
            coeffs[r] = sr_synth.to_pre_shuffle(coeffs[r], wl.scale)
        inp["coeff"] = coeffs[0]
    opts = sr.make_options(args.kernel, args.tile, layout, sr.SR_COEFF_LOGITS if args.logits else sr.SR_COEFF_VALUES)
    if args.logits:
        args.pre_shuffle = True            # the extra legs below time stored coefficients only
    plan = sr.sr_dict_assemble_plan(inp["lr"], coeffs[0], inp["dict"], wl.L, wl.k, wl.scale, wl.c,
                                    outs[0], kept=kept, opts=opts)
    assert plan > 0, sr.sr_strerror(plan)

    def step(i):
        sr.sr_dict_assemble_ex(inp["lr"], coeffs[i % N_ROTATE], inp["dict"], wl.L, wl.k, wl.scale, wl.c,
                               outs[i % 2], kept=kept, opts=opts)

    if args.calibrate_copy:
        src = torch.empty(1 << 28, device=dev, dtype=torch.float32).normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)          # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    # Timed region: K back-to-back launches between two HIP events on the launch stream
    # (torch's current stream, which the binding hands to the library), bracketed by
    # host synchronisation.  The per-launch duration is that event span / K, so it
    # includes the gaps between launches.
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev0.record()
    for i in range(args.steps):
        step(i)
    ev1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    avg_ms = ev0.elapsed_time(ev1) / args.steps
    # spread of single launches, outside the timed region (events around each launch)
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
          for _ in range(min(args.steps, 30))]
    for i, (a, b) in enumerate(ev):
        a.record()
        step(i)
        b.record()
    torch.cuda.synchronize()
    kernel_ms = [a.elapsed_time(b) for a, b in ev]
    px = wl.hr_pixels
    n_read = len(kept) if kept is not None else wl.L
    alg_bytes = wl.algorithmic_bytes(n_read)
    achieved = alg_bytes / (avg_ms * 1e-3) / 1e9
    result = {
        "metric": ("HR Mpixel/s of dictionary assembly (4K x4, L=72, fp16) + % of HBM peak" if wl.name == "4k_dense"
                   else f"HR Mpixel/s of dictionary assembly ({wl.name}) + % of HBM peak"),
        "value": round(px * args.steps / wall / 1e6, 1),
        "unit": "HR Mpixel/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(wall / args.steps * 1e3, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": ("bf16" if (wl.coeff_dtype == "bf16" and not args.logits) else "f16") if (plan == 2 and wl.coeff_dtype in ("f16", "f8", "bf16")) else "f32",
        "arithmetic": ("f32 vector ALU" if plan != 2 else
                       f"{wl.coeff_dtype} logits -> exp2((z - max) log2 e) in f32, rounded to f16 -> x f16 (hi+lo) dictionary on MFMA "
                       "with f32 accumulation, a row of ones returning the sum of the exponentials; f32 up-sampling and filtering"
                       if args.logits else
                       "f16 coefficients x f16 (hi+lo) dictionary on MFMA with f32 accumulation; f32 up-sampling "
                       "and filtering" if wl.coeff_dtype == "f16" else
                       "coefficients stored as 8-bit E4M3, widened exactly to f16 in registers, x f16 (hi+lo) "
                       "dictionary on MFMA with f32 accumulation; f32 up-sampling and filtering"
                       if wl.coeff_dtype == "f8" else
                       "bf16 coefficients x bf16 (hi+lo) dictionary on MFMA with f32 accumulation; f32 up-sampling "
                       "and filtering" if wl.coeff_dtype == "bf16" else
                       "f32 coefficients x f32 dictionary on f32 MFMA; f32 up-sampling and filtering"),
        "data": "synthetic",
        "config": {"workload": wl.name, "hr": f"{wl.W}x{wl.H}", "scale": wl.scale, "channels": wl.c,
                   "L": wl.L, "k": wl.k, "atoms_read": n_read, "batch": wl.n,
                   "kernel": {1: "generic", 2: "mfma"}[plan], "rotating_coeff_buffers": N_ROTATE,
                   "coeff_layout": {sr.SR_COEFF_PLANAR: "planar [N][L][H][W]", sr.SR_COEFF_PIXEL_MAJOR: "pixel_major [N][H][W][L]",
                                    sr.SR_COEFF_PRE_SHUFFLE: "pre_shuffle [N][L*s*s][h][w]",
                                    sr.SR_COEFF_BLOCKED: "blocked [N][H][W/128][4 slots][pieces of 16 atoms][lane half][32][8]"}[layout],
                   "coeff_kind": "logits (softmax over the atoms applied by the call)" if args.logits else "values"},
        "roofline": {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": read_traffic(wl.name),
                     "traffic_source": (f"profiles/sr_mfma_{wl.name}_traffic.txt (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of an "
                                        "earlier run of this command; not measured in this run)"
                                        if read_traffic(wl.name) is not None else None),
                     "kernel_ms_avg": round(avg_ms, 4), "kernel_ms_min": round(min(kernel_ms), 4),
                     "kernel_ms_single_launch_avg": round(sum(kernel_ms) / len(kernel_ms), 4),
                     "algorithmic_bytes": alg_bytes},
        "pct_of_hbm_peak": round(100.0 * achieved / HBM_PEAK_GBS, 2),
    }
    emp = None if args.pre_shuffle else empirical_ceilings(sr, torch, wl, coeffs, outs, avg_ms, inp["lr"], inp["dict"])
    if emp is not None:
        result["roofline"]["empirical"] = emp
    if args.kept_sweep:
        import numpy as np
        rng = np.random.default_rng(7)
        sweep = []
        for n_keep in (72, 58, 43, 29, 14, 8):
            if n_keep > wl.L:
                continue
            klist = np.sort(rng.choice(wl.L, size=n_keep, replace=False)).astype(np.int32)
            gam = rng.uniform(0.5, 1.5, size=n_keep).astype(np.float32)     # the kept atoms' regression scales (Eq. 9)

            def kstep(i):
                sr.sr_dict_assemble_ex(inp["lr"], coeffs[i % N_ROTATE], inp["dict"], wl.L, wl.k, wl.scale,
                                       wl.c, outs[i % 2], kept=klist, gamma=gam, opts=opts)
            for i in range(3):
                kstep(i)
            torch.cuda.synchronize()
            kev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(20)]
            for i, (a, b) in enumerate(kev):
                a.record(); kstep(i); b.record()
            torch.cuda.synchronize()
            ms = sum(a.elapsed_time(b) for a, b in kev) / len(kev)
            sweep.append({"atoms_read": n_keep, "kernel_ms_avg": round(ms, 4),
                          "hr_mpixel_per_s": round(px / ms / 1e3, 1),
                          "algorithmic_GBps": round(wl.algorithmic_bytes(n_keep) / ms / 1e6, 1)})
        base = sweep[0]["kernel_ms_avg"]
        for row in sweep:
            row["speedup_vs_all_atoms"] = round(base / row["kernel_ms_avg"], 2)
        result["kept_sweep"] = sweep
    if args.selection > 0 and wl.coeff_dtype in ("f16", "f32") and inp["lr"].dtype == torch.float32 and wl.L <= 128:
        result["selection"] = selection_leg(sr, torch, wl, inp, args.selection)
    if args.list_entries > 0 and not args.pre_shuffle:
        result["list_form"] = list_leg(sr, torch, sr_synth, wl, inp, coeffs[:2], args.list_entries)
    if args.bicubic:
        result["bicubic"] = bicubic_leg(sr, torch, wl, inp)
    if args.tile_sweep and not args.pre_shuffle:
        # the launch-shape search (section III-B, Eq. 11-12): every shape the library has for this case, timed
        from paper_2303_08999_amd import tune
        rows = []
        for t, ms in tune.sweep_tiles(inp["lr"], coeffs[0], inp["dict"], wl.L, wl.k, wl.scale, wl.c, outs[0], kept=kept, reps=15):
            shape = sr.sr_dict_assemble_launch_shape(inp["lr"], coeffs[0], inp["dict"], wl.L, wl.k, wl.scale, wl.c, outs[0],
                                                     kept=kept, opts=sr.make_options(sr.SR_KERNEL_MFMA, t))[1]
            rows.append({"index": t, "tile": f"{shape[0]}x{shape[1]}", "wavefronts_per_workgroup": shape[2],
                         "workgroups_per_cu": shape[3], "median_us_single_launch": round(ms * 1e3, 1)})
        result["tile_sweep"] = rows
    if not args.no_cpu and not args.pre_shuffle:      # the oracle leg is timed on the planar layout only
        result["cpu_baseline"] = cpu_baseline(wl, inp["lr"], coeffs[0], inp["dict"], args.cpu_budget)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
