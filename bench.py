#!/usr/bin/env python3
"""Benchmark of the masked-attention forward path on one MI355X.

A step is one call of ap_sparse_attn_fwd over one batch of synthetic input with the tensors
already resident in HBM.  The layout is built once before the timed region: the mask of
Attention Pruning is fixed for all inputs (Section 3.2), so ap_build_layout runs once per
layer and is amortised over every forward call; its own time is reported as `layout_ms`.

Prints ONE JSON line.  `value` is kept-entry TFLOP/s (4*D flops per kept connection per batch
element) of the headline workload; `per_config` carries ms/call, roofline fraction and the
speedup over the same kernel run with a dense mask for every configuration.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 matrix peak, published
INFINITY_CACHE_BYTES = 256 << 20
# HBM bytes per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (scaled by the same
# counters' reading of a plain 256 MiB copy): 263.2 MB read + 68.2 MB written, taken on 2026-11-28 at
# commit a175aa2; see profiles/fwd_mfma_kernel_C5.md.  Keyed by (workload, block_m, visit schedule
# used); other settings report null.
MEASURED_TRAFFIC_BYTES = {("C5", 64, True): 331.4e6}


def parse():
    p = argparse.ArgumentParser()
    p.add_argument("--gpus", type=int, default=1)
    p.add_argument("--steps", type=int, default=200)
    p.add_argument("--warmup", type=int, default=20)
    p.add_argument("--workload", default="C5", help="headline configuration (C1..C5)")
    p.add_argument("--block-m", type=int, default=64)
    p.add_argument("--min-cols", type=int, default=0, help="schedule packing threshold (0 = library default)")
    p.add_argument("--no-sched", action="store_true", help="walk the layout itself instead of the visit schedule")
    p.add_argument("--only", action="store_true", help="skip the per-config table and the CPU baseline")
    p.add_argument("--no-cpu", action="store_true", help="skip the CPU baseline")
    p.add_argument("--only-entmax", action="store_true",
                   help="time only the 1.5-entmax forward at the workload's shape and print its figures")
    p.add_argument("--only-split", action="store_true",
                   help="time only the split forward call on the long-memory shape X1 and print its figures")
    p.add_argument("--only-backward", action="store_true",
                   help="time only the backward pass at the workload's shape and print its figures")
    p.add_argument("--no-backward", action="store_true", help="skip the timing of the backward pass")
    p.add_argument("--only-mask-construction", action="store_true",
                   help="time only the mask-construction kernels at the workload's shape and print their figures")
    p.add_argument("--no-mask-construction", action="store_true",
                   help="skip the timing of the mask-construction kernels (Eq. (1), Eq. (2))")
    p.add_argument("--copy-calibration", action="store_true",
                   help="also launch one plain 256 MiB device copy (reference point for HBM byte counters)")
    return p.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the path shards over batch and heads with "
              "no exchange; no multi-GPU figure is produced). Re-run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2012_02030_amd import binding as ap
    from paper_2012_02030_amd import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    ap.lib()                                            # fail loudly if the HIP library is missing
    dev = torch.device("cuda:0")

    def log(*a):
        print(*a, file=sys.stderr, flush=True)

    def alg_bytes(cfg):
        es = 4 if cfg.dtype == "f32" else 2
        return es * cfg.B * cfg.H * cfg.D * (2 * cfg.Lq + 2 * cfg.Lk)      # Q, O and K, V once each

    def tensor_sets(cfg, n_sets):
        """Set 0 is the seeded numpy draw the tests use; further sets are seeded device draws."""
        tdt = torch.float32 if cfg.dtype == "f32" else torch.bfloat16
        sets = []
        q, k, v = synth.make_qkv(cfg)
        sets.append(tuple(torch.from_numpy(x).to(tdt).to(dev) for x in (q, k, v)))
        gen = torch.Generator(device=dev)
        for s in range(1, n_sets):
            gen.manual_seed(synth.SEED + 1000 * cfg.index + s)
            sets.append(tuple(
                torch.randn((cfg.B, cfg.H, L, cfg.D), generator=gen, device=dev, dtype=torch.float32).to(tdt)
                for L in (cfg.Lq, cfg.Lk, cfg.Lk)))
        outs = [torch.empty_like(s[0]) for s in sets]
        lses = [torch.empty((cfg.B, cfg.H, cfg.Lq), dtype=torch.float32, device=dev) for _ in sets]
        return sets, outs, lses

    def n_sets_for(cfg):
        # rotate through enough independent sets that no call finds its inputs in the 256 MB cache
        return max(2, -(-2 * INFINITY_CACHE_BYTES // alg_bytes(cfg)) + 1)

    def time_calls(cfg, layout, sets, outs, lses, steps, warmup, sched=None):
        """Exactly `steps` back-to-back launches on the current stream, one HIP event between
        each pair; returns (wall ms per step, list of per-launch ms)."""
        n = len(sets)

        def call(i):
            q, k, v = sets[i % n]
            ap.ap_sparse_attn_fwd(q, k, v, layout, causal=cfg.causal, out=outs[i % n], lse=lses[i % n],
                                  sched=sched)

        for i in range(warmup):
            call(i)
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        evs[0].record()
        for i in range(steps):
            call(i)
            evs[i + 1].record()
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) * 1e3 / steps
        per = [evs[i].elapsed_time(evs[i + 1]) for i in range(steps)]
        return wall_ms, per

    def time_graph(cfg, layout, sets, outs, lses, steps, warmup, sched=None):
        """For microsecond-scale kernels the Python launch rate, not the GPU, would set the pace:
        capture one rotation through all sets into a HIP graph and time its replays."""
        n = len(sets)
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            for i in range(n):
                q, k, v = sets[i]
                ap.ap_sparse_attn_fwd(q, k, v, layout, causal=cfg.causal, out=outs[i], lse=lses[i],
                                      sched=sched)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for i in range(n):
                q, k, v = sets[i]
                ap.ap_sparse_attn_fwd(q, k, v, layout, causal=cfg.causal, out=outs[i], lse=lses[i],
                                      sched=sched)
        reps = max(1, -(-steps // n))
        for _ in range(max(1, warmup // n)):
            g.replay()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            g.replay()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / (reps * n)

    def measured_peaks():
        """What this GPU reaches on a plain device copy and on a library bf16 GEMM, as a second
        yardstick next to the published peaks."""
        n = 1 << 30
        src = torch.empty(n, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for _ in range(2):
            dst.copy_(src)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(10):
            dst.copy_(src)
        e1.record()
        torch.cuda.synchronize()
        copy_gbs = 2.0 * n * 10 / (e0.elapsed_time(e1) * 1e-3) / 1e9
        del src, dst
        m = 8192
        a_ = torch.randn((m, m), device=dev, dtype=torch.float32).to(torch.bfloat16)
        b_ = torch.randn((m, m), device=dev, dtype=torch.float32).to(torch.bfloat16)
        for _ in range(2):
            torch.matmul(a_, b_)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(10):
            torch.matmul(a_, b_)
        e1.record()
        torch.cuda.synchronize()
        gemm_tflops = 2.0 * m * m * m * 10 / (e0.elapsed_time(e1) * 1e-3) / 1e12
        del a_, b_
        torch.cuda.empty_cache()
        return {"hbm_copy_gbs": copy_gbs, "hbm_copy": "1 GiB device-to-device copy, read + write bytes",
                "bf16_gemm_tflops": gemm_tflops, "bf16_gemm": "torch.matmul 8192^3 bf16 (library GEMM)"}

    def oracle_check(cfg, mask_np, set0, out, lse, threads_note=True):
        """The fp64 oracle on the whole configuration: wall time on all host threads (and on one,
        for the small configurations), and the largest deviation of the GPU result from it."""
        import ctypes

        import oracle
        q, k, v = set0
        rq, rk, rv = (x.to(torch.float64).cpu().numpy() for x in (q, k, v))
        t0 = time.perf_counter()
        O_ref, lse_ref = oracle.masked_attention(rq, rk, rv, mask_np, causal=cfg.causal)
        all_s = time.perf_counter() - t0
        res = {"oracle_ms_all_threads": all_s * 1e3, "oracle_threads": oracle.num_threads()}
        if cfg.name != "C5":
            try:
                gomp = ctypes.CDLL("libgomp.so.1")
                nthreads = oracle.num_threads()
                gomp.omp_set_num_threads(1)
                t0 = time.perf_counter()
                oracle.masked_attention(rq, rk, rv, mask_np, causal=cfg.causal)
                res["oracle_ms_1_thread"] = (time.perf_counter() - t0) * 1e3
                gomp.omp_set_num_threads(nthreads)
            except OSError:
                pass
        finite = np.isfinite(lse_ref)
        res["max_abs_err_O"] = float(np.abs(out.to(torch.float64).cpu().numpy() - O_ref).max())
        res["max_abs_err_lse"] = float(np.abs(lse.to(torch.float64).cpu().numpy()[finite] - lse_ref[finite]).max())
        res["tolerance"] = 2e-2 if cfg.dtype == "bf16" else 1e-5
        return res, all_s

    def schedule_classes(layout, sched, block_m):
        """Entries of the two kinds of the visit schedule (per layer), the share of their 64 x block_m
        slots that hold a kept pair, and in how many entries a 32-query group (one wavefront of the
        attention kernel) has nothing to do."""
        rp = layout.row_ptr.cpu().numpy().astype(np.int64)
        cnt = sched.cnt.cpu().numpy().astype(np.int64)
        idx = np.concatenate([np.arange(rp[r], rp[r] + cnt[r]) for r in range(len(cnt))]) if cnt.sum() else \
            np.zeros(0, np.int64)
        start = sched.start.cpu().numpy()[idx]
        words = sched.bitmaps.cpu().numpy().view(np.uint64)[idx]                  # [entries, block_m]
        pop = np.unpackbits(words.view(np.uint8), axis=-1).reshape(len(idx), -1).sum(axis=1)
        groups = (words.reshape(len(idx), block_m // 32, 32) != 0).any(axis=2)       # [entries, 32-query groups]
        out = {}
        for name, sel in (("consecutive", start >= 0), ("gathered", start < 0)):
            n = int(sel.sum())
            out[name] = {"entries": n,
                         "kept_pairs": int(pop[sel].sum()),
                         "slot_fill": float(pop[sel].sum()) / (n * 64.0 * block_m) if n else None,
                         "entries_x_groups_with_work": int(groups[sel].sum()),
                         "entries_x_groups": n * (block_m // 32)}
        return out

    def run_config(cfg, mask_np, steps, warmup, block_m, use_graph):
        """AP-mask run and dense-mask run of the same kernel; returns a result dict."""
        dmask = torch.from_numpy(mask_np).to(dev)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ap.ap_build_layout(dmask, block_m, 64)                       # warm-up of the layout kernels
        torch.cuda.synchronize()
        e0.record()
        layout = ap.ap_build_layout(dmask, block_m, 64)
        e1.record()
        torch.cuda.synchronize()
        layout_ms = e0.elapsed_time(e1)
        dense_layout = ap.ap_build_layout(torch.ones_like(dmask), block_m, 64)
        sched = None
        sched_ms = None
        if cfg.dtype == "bf16" and not args.no_sched:
            ap.ap_build_schedule(layout, causal=cfg.causal, min_cols=args.min_cols)
            torch.cuda.synchronize()
            e0.record()
            sched = ap.ap_build_schedule(layout, causal=cfg.causal, min_cols=args.min_cols)
            e1.record()
            torch.cuda.synchronize()
            sched_ms = e0.elapsed_time(e1)
        torch.cuda.synchronize()
        del dmask

        sets, outs, lses = tensor_sets(cfg, n_sets_for(cfg))
        wall_ms, per = time_calls(cfg, layout, sets, outs, lses, steps, warmup, sched)
        dsteps = steps                                               # same steps and warm-up as the AP-mask leg
        dwall_ms, dper = time_calls(cfg, dense_layout, sets, outs, lses, dsteps, warmup)
        ms = float(np.mean(per))
        dms = float(np.mean(dper))
        # The dense-mask leg walks the layout (the kernel's SCHED = false instantiation).  For the
        # headline workload also time it through a schedule built from the dense layout (all
        # entries consecutive), i.e. the very instantiation the AP-mask leg runs.
        dms_sched = None
        if sched is not None and cfg.name == args.workload:
            dsched = ap.ap_build_schedule(dense_layout, causal=cfg.causal, min_cols=args.min_cols)
            _, dsper = time_calls(cfg, dense_layout, sets, outs, lses, dsteps, warmup, dsched)
            dms_sched = float(np.mean(dsper))
            del dsched
        # warm: one buffer set only, so K, V and Q may stay in the 256 MB cache between calls
        _, wper = time_calls(cfg, layout, sets[:1], outs[:1], lses[:1], max(10, steps // 4), 2, sched)
        warm_ms = float(np.mean(wper))
        gms = gdms = None
        if use_graph:
            try:
                gms = time_graph(cfg, layout, sets, outs, lses, steps, warmup, sched)
                gdms = time_graph(cfg, dense_layout, sets, outs, lses, dsteps, warmup)
            except Exception as ex:                                   # graph capture is an extra
                log("graph timing unavailable:", repr(ex))
        kernel_ms = gms if gms is not None else ms
        dense_kernel_ms = gdms if gdms is not None else dms

        kept = int(mask_np.sum())                                     # causal already folded in by the generator
        kept_flop = 4.0 * cfg.D * kept * cfg.B
        if cfg.causal:
            dense_entries = cfg.H * sum(min(cfg.Lk, i + 1 + cfg.Lk - cfg.Lq) for i in range(cfg.Lq))
        else:
            dense_entries = cfg.H * cfg.Lq * cfg.Lk
        dense_flop = 4.0 * cfg.D * dense_entries * cfg.B
        nnz = int(layout.nnz.item())
        visited = int(sched.cnt.sum().item()) if sched is not None else nnz
        classes = schedule_classes(layout, sched, block_m) if sched is not None else None
        tile_flop = 4.0 * cfg.D * block_m * 64 * visited * cfg.B           # matrix-core work of the visited tiles
        res = {
            "shape": {"B": cfg.B, "H": cfg.H, "Lq": cfg.Lq, "Lk": cfg.Lk, "D": cfg.D,
                      "dtype": cfg.dtype, "causal": cfg.causal},
            "kept_entries_per_batch": kept,
            "keep_density": kept / float(dense_entries),
            "tiles_stored": nnz,
            "tiles_visited": visited,
            "schedule_ms": sched_ms,
            "schedule_entries": classes,
            "tiles_max": int(ap.ap_layout_max_tiles(cfg.H, cfg.Lq, cfg.Lk, block_m, 64)),
            "ms_per_call": kernel_ms,
            "ms_per_call_stream_launches": ms,
            "warm_ms_per_call_stream_launches": warm_ms,
            "ms_per_call_median": float(np.median(per)),
            "ms_per_call_min": float(np.min(per)),
            "wall_ms_per_step": wall_ms,
            "kept_tflops": kept_flop / (kernel_ms * 1e-3) / 1e12,
            "hbm_alg_bytes": alg_bytes(cfg),
            "hbm_gbs": alg_bytes(cfg) / (kernel_ms * 1e-3) / 1e9,
            "hbm_roofline_frac": alg_bytes(cfg) / (kernel_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "tile_mfma_tflops": tile_flop / (kernel_ms * 1e-3) / 1e12,
            "dense_ms_per_call": dense_kernel_ms,
            "dense_ms_per_call_through_schedule": dms_sched,
            "dense_tflops": dense_flop / (dense_kernel_ms * 1e-3) / 1e12,
            "dense_mfma_frac": dense_flop / (dense_kernel_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
            "speedup_vs_dense": dense_kernel_ms / kernel_ms,
            "layout_ms": layout_ms,
            "layout_gbs": mask_np.size / (layout_ms * 1e-3) / 1e9,
            "timing": "hip graph replay" if gms is not None else "stream launches",
            "n_buffer_sets": len(sets),
        }
        keep_for_parity = (sets[0], outs, lses, layout, sched)
        return res, keep_for_parity

    def run_mask_construction(cfg, steps):
        """Eq. (1) accumulation of one batch into the mean map and Eq. (2) threshold + mask, at
        cfg's shape, on position-coded synthetic Q and K; then the layout of the resulting mask."""
        if cfg.dtype != "bf16":
            return None
        qn, kn = synth.make_qk_positional(cfg.B, cfg.H, cfg.Lq, cfg.Lk, cfg.D, seed=cfg.index)
        q = torch.from_numpy(qn).to(torch.bfloat16).to(dev)
        k = torch.from_numpy(kn).to(torch.bfloat16).to(dev)
        del qn, kn
        abar = torch.zeros((cfg.H, cfg.Lq, cfg.Lk), dtype=torch.float32, device=dev)
        p = 1.0 - cfg.keep

        def timed(fn, n):
            fn()
            evs = [torch.cuda.Event(enable_timing=True) for _ in range(n + 1)]
            torch.cuda.synchronize()
            evs[0].record()
            for i in range(n):
                fn()
                evs[i + 1].record()
            torch.cuda.synchronize()
            return float(np.mean([evs[i].elapsed_time(evs[i + 1]) for i in range(n)]))

        acc_ms = timed(lambda: ap.ap_accumulate_attention_maps(q, k, abar=abar, causal=cfg.causal,
                                                               weight=1.0 / cfg.B), steps)
        # the same with the row statistics of the unpruned attention call on the same inputs
        ones_lay = ap.ap_build_layout(torch.ones((cfg.H, cfg.Lq, cfg.Lk), dtype=torch.uint8, device=dev), 64, 64)
        _, lse_full = ap.ap_sparse_attn_fwd(q, k, k, ones_lay, causal=cfg.causal)
        del ones_lay
        acc_lse_ms = timed(lambda: ap.ap_accumulate_attention_maps(q, k, abar=abar, causal=cfg.causal,
                                                                   weight=1.0 / cfg.B, lse=lse_full), steps)
        abar.zero_()
        ap.ap_accumulate_attention_maps(q, k, abar=abar, causal=cfg.causal, weight=1.0 / cfg.B)
        keep = {}

        def prune():
            keep["mask"], keep["tau"] = ap.ap_prune_mask(abar, p, causal=cfg.causal)

        prune_ms = timed(prune, steps)
        lay_ms = timed(lambda: ap.ap_build_layout(keep["mask"], args.block_m, 64), steps)
        # without the byte mask: threshold only, then the layout straight from the map (Eq. (2) in the scan)
        tau_ms = timed(lambda: ap.ap_prune_mask(abar, p, causal=cfg.causal, threshold_only=True), steps)
        map_lay_ms = timed(lambda: ap.ap_build_layout_from_map(abar, keep["tau"], causal=cfg.causal,
                                                               block_m=args.block_m), steps)
        if cfg.causal:
            vis = cfg.H * sum(min(cfg.Lk, i + 1 + cfg.Lk - cfg.Lq) for i in range(cfg.Lq))
        else:
            vis = cfg.H * cfg.Lq * cfg.Lk
        total = cfg.H * cfg.Lq * cfg.Lk
        # map read + written once, Q and K read once, row log-sum-exp written and read once
        acc_bytes = 8 * vis + 2 * cfg.B * cfg.H * cfg.D * (cfg.Lq + cfg.Lk) + 8 * cfg.B * cfg.H * cfg.Lq
        acc_flop = 2 * 2.0 * cfg.D * vis * cfg.B                          # scores are formed twice
        # selection reads every participating entry at least once, the compare once more; 1 mask byte each
        prune_bytes = 8 * vis + total
        kept = int(keep["mask"].sum().item())
        return {
            "shape": {"B": cfg.B, "H": cfg.H, "Lq": cfg.Lq, "Lk": cfg.Lk, "D": cfg.D, "causal": cfg.causal},
            "prune_fraction": p,
            "accumulate_ms": acc_ms,
            "accumulate_with_given_lse_ms": acc_lse_ms,
            "accumulate_alg_bytes": acc_bytes,
            "accumulate_gbs": acc_bytes / (acc_ms * 1e-3) / 1e9,
            "accumulate_hbm_frac": acc_bytes / (acc_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "accumulate_tflops": acc_flop / (acc_ms * 1e-3) / 1e12,
            "prune_mask_ms": prune_ms,
            "prune_mask_alg_bytes": prune_bytes,
            "prune_mask_gbs": prune_bytes / (prune_ms * 1e-3) / 1e9,
            "prune_mask_hbm_frac": prune_bytes / (prune_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "layout_ms": lay_ms,
            "threshold_only_ms": tau_ms,
            "layout_from_map_ms": map_lay_ms,
            "map_to_layout_ms": {"via_byte_mask": prune_ms + lay_ms, "without_byte_mask": tau_ms + map_lay_ms},
            "tau": float(keep["tau"].item()),
            "kept_entries": kept,
            "kept_fraction_of_visible": kept / float(vis),
            "tiles_stored": int(ap.ap_build_layout(keep["mask"], args.block_m, 64).nnz.item()),
        }

    if args.copy_calibration:
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(3):
            dst.copy_(src)                                 # plain elementwise copy kernel: 256 MiB in, 256 MiB out
        torch.cuda.synchronize()
        del src, dst
        torch.cuda.empty_cache()

    def run_backward(cfg, mask_np, steps):
        """Forward + backward of cfg under its AP mask (plain layout walk, block 64x64)."""
        if cfg.dtype != "bf16":
            return None
        lay = ap.ap_build_layout(torch.from_numpy(mask_np).to(dev), 64, 64)
        lt = ap.ap_build_layout_transpose(lay)
        q, k, v = (torch.from_numpy(x).to(torch.bfloat16).to(dev) for x in synth.make_qkv(cfg))
        gen = torch.Generator(device=dev)
        gen.manual_seed(synth.SEED + 77)
        g = torch.randn(q.shape, generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
        O, lse = ap.ap_sparse_attn_fwd(q, k, v, lay, causal=cfg.causal)

        def timed(fn, n):
            fn()
            evs = [torch.cuda.Event(enable_timing=True) for _ in range(n + 1)]
            torch.cuda.synchronize()
            evs[0].record()
            for i in range(n):
                fn()
                evs[i + 1].record()
            torch.cuda.synchronize()
            return float(np.mean([evs[i].elapsed_time(evs[i + 1]) for i in range(n)]))

        bwd_ms = timed(lambda: ap.ap_sparse_attn_bwd(q, k, v, O, g, lse, lay, lt, causal=cfg.causal), steps)
        tr_ms = timed(lambda: ap.ap_build_layout_transpose(lay), steps)
        rs = ap.ap_build_schedule(lay, causal=cfg.causal, min_cols=args.min_cols)
        cs = ap.ap_build_col_schedule(lay, lt, causal=cfg.causal)
        sched_ms = timed(lambda: ap.ap_sparse_attn_bwd(q, k, v, O, g, lse, lay, lt, causal=cfg.causal,
                                                       sched=rs, col_sched=cs), steps)
        cs_ms = timed(lambda: ap.ap_build_col_schedule(lay, lt, causal=cfg.causal), steps)
        row_entries = int(rs.cnt.sum().item())
        col_entries = int(cs.cnt[:lt.col_ptr.shape[0] - 1].sum().item())
        kept = int(mask_np.sum())
        kept_flop = 10.0 * cfg.D * kept * cfg.B               # five N^2-sized products per kept entry
        tiles = int(lay.nnz.item())
        tile_flop = 10.0 * cfg.D * 64 * 64 * tiles * cfg.B
        es = 2
        alg = es * cfg.B * cfg.H * cfg.D * (4 * cfg.Lq + 4 * cfg.Lk) + 4 * cfg.B * cfg.H * cfg.Lq
        return {
            "shape": {"B": cfg.B, "H": cfg.H, "Lq": cfg.Lq, "Lk": cfg.Lk, "D": cfg.D, "causal": cfg.causal},
            "tiles_visited": tiles,
            "bwd_ms": bwd_ms,
            "kept_tflops": kept_flop / (bwd_ms * 1e-3) / 1e12,
            "tile_mfma_tflops": tile_flop / (bwd_ms * 1e-3) / 1e12,
            "tile_mfma_frac": tile_flop / (bwd_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
            "hbm_alg_bytes": alg,
            "hbm_gbs": alg / (bwd_ms * 1e-3) / 1e9,
            "layout_transpose_ms": tr_ms,
            "scheduled": {
                "bwd_ms": sched_ms,
                "row_entries": row_entries,
                "col_entries": col_entries,
                "kept_tflops": kept_flop / (sched_ms * 1e-3) / 1e12,
                "entry_mfma_tflops": 64 * 64 * cfg.D * cfg.B * (6.0 * row_entries + 8.0 * col_entries)
                                     / (sched_ms * 1e-3) / 1e12,
                "hbm_gbs": alg / (sched_ms * 1e-3) / 1e9,
                "col_schedule_ms": cs_ms,
                "speedup_vs_layout_walk": bwd_ms / sched_ms,
            },
        }

    def run_split_forward(cfg, steps):
        """Few queries against a long memory: the ordinary call (one workgroup per block row)
        against the split call, same layout and schedule."""
        mask_np = synth.make_mask(cfg)
        lay = ap.ap_build_layout(torch.from_numpy(mask_np).to(dev), 64, 64)
        sched = ap.ap_build_schedule(lay, causal=cfg.causal, min_cols=args.min_cols)
        q, k, v = (torch.from_numpy(x).to(torch.bfloat16).to(dev) for x in synth.make_qkv(cfg))
        out = torch.empty_like(q)

        def timed(fn, n):
            fn()
            evs = [torch.cuda.Event(enable_timing=True) for _ in range(n + 1)]
            torch.cuda.synchronize()
            evs[0].record()
            for i in range(n):
                fn()
                evs[i + 1].record()
            torch.cuda.synchronize()
            return float(np.mean([evs[i].elapsed_time(evs[i + 1]) for i in range(n)]))

        plain_ms = timed(lambda: ap.ap_sparse_attn_fwd(q, k, v, lay, causal=cfg.causal, out=out, sched=sched), steps)
        best = None
        table = {}
        for splits in (4, 8, 16, 32):
            ms = timed(lambda: ap.ap_sparse_attn_fwd_split(q, k, v, lay, splits, causal=cfg.causal, out=out,
                                                          sched=sched), steps)
            table[str(splits)] = ms
            if best is None or ms < table[str(best)]:
                best = splits
        kept = int(mask_np.sum())
        cols = int((mask_np.any(axis=1)).sum())                   # distinct (head, key) pairs with a kept entry
        alg = 2 * cfg.B * (2 * cols * cfg.D + 2 * cfg.H * cfg.Lq * cfg.D)   # their K and V rows, Q and O
        ms = table[str(best)]
        return {
            "shape": {"B": cfg.B, "H": cfg.H, "Lq": cfg.Lq, "Lk": cfg.Lk, "D": cfg.D, "causal": cfg.causal},
            "entries_visited": int(sched.cnt.sum().item()),
            "tiles_stored": int(lay.nnz.item()),
            "plain_call_ms": plain_ms,
            "split_call_ms": table,
            "best_splits": best,
            "speedup_vs_plain_call": plain_ms / ms,
            "kept_tflops": 4.0 * cfg.D * kept * cfg.B / (ms * 1e-3) / 1e12,
            "hbm_alg_bytes": alg,
            "hbm_gbs": alg / (ms * 1e-3) / 1e9,
            "hbm_roofline_frac": alg / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
        }

    def run_decode(cfg, steps):
        """One new query per (example, head) against cfg's long key sequence (cfg's last mask row):
        the one-workgroup-per-query call next to the tiled calls on the same layout."""
        mask_np = np.ascontiguousarray(synth.make_mask(cfg)[:, -1:, :])
        lay = ap.ap_build_layout(torch.from_numpy(mask_np).to(dev), 64, 64)
        sched = ap.ap_build_schedule(lay, causal=cfg.causal, min_cols=args.min_cols)
        Q, K, V = synth.make_qkv(cfg)
        q, k, v = (torch.from_numpy(x).to(torch.bfloat16).to(dev) for x in (Q[:, :, -1:, :], K, V))
        q = q.contiguous()
        out = torch.empty_like(q)

        def timed(fn, n):
            fn()
            evs = [torch.cuda.Event(enable_timing=True) for _ in range(n + 1)]
            torch.cuda.synchronize()
            evs[0].record()
            for i in range(n):
                fn()
                evs[i + 1].record()
            torch.cuda.synchronize()
            return float(np.mean([evs[i].elapsed_time(evs[i + 1]) for i in range(n)]))

        dec_table = {str(sp): timed(lambda: ap.ap_sparse_attn_decode(q, k, v, lay, causal=cfg.causal, out=out,
                                                                     splits=sp), steps) for sp in (1, 4, 8, 16)}
        dec_ms = min(dec_table.values())
        plain_ms = timed(lambda: ap.ap_sparse_attn_fwd(q, k, v, lay, causal=cfg.causal, out=out, sched=sched), steps)
        split_ms = min(timed(lambda: ap.ap_sparse_attn_fwd_split(q, k, v, lay, sp, causal=cfg.causal, out=out,
                                                                 sched=sched), steps) for sp in (8, 16, 32))
        kept = int(mask_np.sum())
        alg = 2 * cfg.B * (2 * kept * cfg.D + 2 * cfg.H * cfg.D)          # kept keys' K and V rows, Q and O
        return {
            "shape": {"B": cfg.B, "H": cfg.H, "Lq": 1, "Lk": cfg.Lk, "D": cfg.D, "causal": cfg.causal},
            "kept_keys_per_layer": kept,
            "decode_call_ms": dec_ms,
            "decode_call_ms_by_splits": dec_table,
            "tiled_call_ms": plain_ms,
            "tiled_split_call_ms": split_ms,
            "hbm_alg_bytes": alg,
            "hbm_gbs": alg / (dec_ms * 1e-3) / 1e9,
            "hbm_roofline_frac": alg / (dec_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
        }

    def run_cropped(cfg, mask_np, steps):
        """Half-length sequences under the full-length mask: the cropped call on the layout and
        schedule built once for the full size, against the ordinary call on a layout and schedule
        rebuilt for the corner (and what that rebuild costs)."""
        if cfg.dtype != "bf16" or cfg.Lq != cfg.Lk:
            return None
        L = cfg.Lq // 2
        dmask = torch.from_numpy(mask_np).to(dev)
        lay = ap.ap_build_layout(dmask, 64, 64)
        sched = ap.ap_build_schedule(lay, causal=cfg.causal, min_cols=args.min_cols)
        q, k, v = (torch.from_numpy(np.ascontiguousarray(x[:, :, :L])).to(torch.bfloat16).to(dev)
                   for x in synth.make_qkv(cfg))
        out = torch.empty_like(q)

        def timed(fn, n):
            fn()
            evs = [torch.cuda.Event(enable_timing=True) for _ in range(n + 1)]
            torch.cuda.synchronize()
            evs[0].record()
            for i in range(n):
                fn()
                evs[i + 1].record()
            torch.cuda.synchronize()
            return float(np.mean([evs[i].elapsed_time(evs[i + 1]) for i in range(n)]))

        crop_ms = timed(lambda: ap.ap_sparse_attn_fwd(q, k, v, lay, causal=cfg.causal, out=out, sched=sched,
                                                      crop=True), steps)
        rebuilt = {}

        def rebuild():
            rebuilt["lay"] = ap.ap_build_layout(dmask, 64, 64, crop=(L, L))
            rebuilt["sched"] = ap.ap_build_schedule(rebuilt["lay"], causal=cfg.causal, min_cols=args.min_cols)

        rebuild_ms = timed(rebuild, steps)
        plain_ms = timed(lambda: ap.ap_sparse_attn_fwd(q, k, v, rebuilt["lay"], causal=cfg.causal, out=out,
                                                       sched=rebuilt["sched"]), steps)
        return {"shape": {"B": cfg.B, "H": cfg.H, "Lq": L, "Lk": L, "D": cfg.D, "causal": cfg.causal,
                          "layout_built_for": [cfg.Lq, cfg.Lk]},
                "cropped_call_ms": crop_ms, "call_on_rebuilt_layout_ms": plain_ms,
                "rebuild_layout_and_schedule_ms": rebuild_ms}

    def run_entmax(cfg, mask_np, steps):
        """1.5-entmax forward of cfg under its AP mask (plain layout walk) next to the softmax
        forward over the same layout walk."""
        if cfg.dtype != "bf16":
            return None
        lay = ap.ap_build_layout(torch.from_numpy(mask_np).to(dev), 64, 64)
        q, k, v = (torch.from_numpy(x).to(torch.bfloat16).to(dev) for x in synth.make_qkv(cfg))
        out = torch.empty_like(q)

        def timed(fn, n):
            fn()
            evs = [torch.cuda.Event(enable_timing=True) for _ in range(n + 1)]
            torch.cuda.synchronize()
            evs[0].record()
            for i in range(n):
                fn()
                evs[i + 1].record()
            torch.cuda.synchronize()
            return float(np.mean([evs[i].elapsed_time(evs[i + 1]) for i in range(n)]))

        sched = ap.ap_build_schedule(lay, causal=cfg.causal, min_cols=args.min_cols)
        walk_ms = timed(lambda: ap.ap_sparse_attn_entmax15_fwd(q, k, v, lay, causal=cfg.causal, out=out), steps)
        ent_ms = timed(lambda: ap.ap_sparse_attn_entmax15_fwd(q, k, v, lay, causal=cfg.causal, out=out,
                                                               sched=sched), steps)
        soft_ms = timed(lambda: ap.ap_sparse_attn_fwd(q, k, v, lay, causal=cfg.causal, out=out, sched=sched), steps)
        # backward pass of the same call (row and column schedules) next to the softmax backward pass
        lt = ap.ap_build_layout_transpose(lay)
        cs = ap.ap_build_col_schedule(lay, lt, causal=cfg.causal)
        gen = torch.Generator(device=dev)
        gen.manual_seed(synth.SEED + 78)
        g = torch.randn(q.shape, generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
        _, tau = ap.ap_sparse_attn_entmax15_fwd(q, k, v, lay, causal=cfg.causal, sched=sched)
        O, lse = ap.ap_sparse_attn_fwd(q, k, v, lay, causal=cfg.causal, sched=sched)
        ent_bwd_ms = timed(lambda: ap.ap_sparse_attn_entmax15_bwd(q, k, v, g, tau, lay, lt, sched, cs,
                                                                  causal=cfg.causal), steps)
        soft_bwd_ms = timed(lambda: ap.ap_sparse_attn_bwd(q, k, v, O, g, lse, lay, lt, causal=cfg.causal,
                                                          sched=sched, col_sched=cs), steps)
        kept = int(mask_np.sum())
        tiles = int(lay.nnz.item())
        return {
            "backward_ms": ent_bwd_ms,
            "softmax_backward_same_schedules_ms": soft_bwd_ms,
            "backward_kept_tflops": 10.0 * cfg.D * kept * cfg.B / (ent_bwd_ms * 1e-3) / 1e12,
            "shape": {"B": cfg.B, "H": cfg.H, "Lq": cfg.Lq, "Lk": cfg.Lk, "D": cfg.D, "causal": cfg.causal},
            "tiles_stored": tiles,
            "entries_visited": int(sched.cnt.sum().item()),
            "entmax_ms": ent_ms,
            "entmax_layout_walk_ms": walk_ms,
            "softmax_same_walk_ms": soft_ms,
            "ratio_to_softmax": ent_ms / soft_ms,
            "kept_tflops": 4.0 * cfg.D * kept * cfg.B / (ent_ms * 1e-3) / 1e12,
            "hbm_alg_bytes": alg_bytes(cfg),
            "hbm_gbs": alg_bytes(cfg) / (ent_ms * 1e-3) / 1e9,
            "hbm_roofline_frac": alg_bytes(cfg) / (ent_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
        }

    if args.only_entmax:
        cfg = synth.CONFIGS[args.workload]
        print(json.dumps({"entmax15_forward": run_entmax(cfg, synth.make_mask(cfg), args.steps)}), flush=True)
        return

    if args.only_split:
        print(json.dumps({"split_forward": run_split_forward(synth.EXTRA_CONFIGS["X1"], args.steps),
                          "decode": run_decode(synth.EXTRA_CONFIGS["X1"], args.steps)}), flush=True)
        return

    if args.only_backward:
        cfg = synth.CONFIGS[args.workload]
        print(json.dumps({"backward": run_backward(cfg, synth.make_mask(cfg), args.steps)}), flush=True)
        return

    if args.only_mask_construction:
        print(json.dumps({"mask_construction": run_mask_construction(synth.CONFIGS[args.workload], args.steps)}),
              flush=True)
        return

    # ---------------------------------------------------------------- headline workload
    head = synth.CONFIGS[args.workload]
    log("generating", head.name, "mask ...")
    head_mask = synth.make_mask(head)
    small = head.name != "C5"
    log("timing", head.name, "...")
    head_res, (set0, outs, lses, layout, sched) = run_config(head, head_mask, args.steps, args.warmup,
                                                     args.block_m, use_graph=small)

    # ---------------------------------------------------------------- CPU baseline = the oracle
    cpu = None
    parity = None
    if not args.only and not args.no_cpu:
        import oracle
        q, k, v = set0
        ap.ap_sparse_attn_fwd(q, k, v, layout, causal=head.causal, out=outs[0], lse=lses[0], sched=sched)
        torch.cuda.synchronize()
        rq, rk, rv = (x.to(torch.float64).cpu().numpy() for x in (q, k, v))
        log("timing the CPU oracle on the full", head.name, "workload ...")
        t0 = time.perf_counter()
        O_ref, lse_ref = oracle.masked_attention(rq, rk, rv, head_mask, causal=head.causal)
        cpu_s = time.perf_counter() - t0
        kept_flop = 4.0 * head.D * int(head_mask.sum()) * head.B
        cpu = {"value": kept_flop / cpu_s / 1e12, "unit": "TFLOP/s (kept-entry)", "cores": oracle.num_threads(),
               "kind": "oracle", "sample": "full %s workload, one call, fp64" % head.name,
               "ms_per_call": cpu_s * 1e3}
        parity = {"max_abs_err_O": float(np.abs(outs[0].to(torch.float64).cpu().numpy() - O_ref).max()),
                  "max_abs_err_lse": float(np.abs(lses[0].to(torch.float64).cpu().numpy() - lse_ref).max()),
                  "tolerance": 2e-2 if head.dtype == "bf16" else 1e-5}
        del rq, rk, rv, O_ref, lse_ref
    del set0, outs, lses, layout, sched
    torch.cuda.empty_cache()

    # ---------------------------------------------------------------- the other configurations
    per_config = {head.name: head_res}
    if not args.only:
        for name, cfg in synth.CONFIGS.items():
            if name == head.name:
                continue
            log("timing", name, "...")
            steps = min(args.steps, 200)
            cmask = synth.make_mask(cfg)
            res, keep = run_config(cfg, cmask, steps, args.warmup, args.block_m,
                                   use_graph=(name != "C5"))
            if not args.no_cpu:
                kset0, kouts, klses, klayout, ksched = keep
                q, k, v = kset0
                ap.ap_sparse_attn_fwd(q, k, v, klayout, causal=cfg.causal, out=kouts[0], lse=klses[0], sched=ksched)
                torch.cuda.synchronize()
                res["oracle"], _ = oracle_check(cfg, cmask, kset0, kouts[0], klses[0])
                del kset0, kouts, klses, klayout, ksched
            del keep
            torch.cuda.empty_cache()
            per_config[name] = res

    peaks = None
    if not args.only:
        log("measuring a device copy and a library bf16 GEMM ...")
        peaks = measured_peaks()

    mask_construction = None
    if not args.only and not args.no_mask_construction:
        log("timing mask construction at the", head.name, "shape ...")
        mask_construction = run_mask_construction(head, 10)
        torch.cuda.empty_cache()

    split_forward = None
    decode = None
    if not args.only:
        log("timing the split forward call on the long-memory shape X1 ...")
        split_forward = run_split_forward(synth.EXTRA_CONFIGS["X1"], 20)
        decode = run_decode(synth.EXTRA_CONFIGS["X1"], 20)
        torch.cuda.empty_cache()

    cropped = None
    if not args.only:
        log("timing the cropped forward call at half of the", head.name, "length ...")
        cropped = run_cropped(head, head_mask, 20)
        torch.cuda.empty_cache()

    entmax = None
    if not args.only:
        log("timing the 1.5-entmax forward at the", head.name, "shape ...")
        entmax = run_entmax(head, head_mask, 10)
        torch.cuda.empty_cache()

    backward = None
    if not args.only and not args.no_backward:
        log("timing the backward pass at the", head.name, "shape ...")
        backward = run_backward(head, head_mask, 10)
        torch.cuda.empty_cache()

    out = {
        "metric": "kept-entry TFLOP/s of masked attention fwd (ms/call and speedup vs dense-mask run alongside)",
        "value": head_res["kept_tflops"],
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": head_res["wall_ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": head.dtype,
        "data": "synthetic",
        "config": {"workload": "%s: B%d H%d Lq%d Lk%d D%d %s %s, keep %.0f%% of %s entries per head" % (
            head.name, head.B, head.H, head.Lq, head.Lk, head.D, head.dtype,
            "causal" if head.causal else "non-causal", 100 * head.keep,
            "causal" if head.causal else "all"),
            "block_m": args.block_m, "block_n": 64, "visit_schedule": not args.no_sched},
        "ms_per_call": head_res["ms_per_call"],
        "speedup_vs_dense": head_res["speedup_vs_dense"],
        "layout_ms": head_res["layout_ms"],
        "roofline": {"bound": "hbm", "achieved": head_res["hbm_gbs"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": head_res["hbm_roofline_frac"],
                     "traffic": MEASURED_TRAFFIC_BYTES.get((head.name, args.block_m, not args.no_sched)),
                     "traffic_source": "profiles/fwd_mfma_kernel_C5.md (separate rocprofv3 --pmc runs, 2026-11-28, commit a175aa2)",
                     "kernel": "fwd_mfma_kernel" if head.dtype == "bf16" else "fwd_valu_kernel",
                     "algorithmic_bytes_per_launch": head_res["hbm_alg_bytes"]},
        "roofline_dense_run": {"bound": "mfma", "achieved": head_res["dense_tflops"], "peak": MFMA_BF16_PEAK_TFLOPS,
                               "unit": "TFLOP/s", "frac": head_res["dense_mfma_frac"]},
        "measured_peaks": peaks,
        "roofline_vs_measured": None if peaks is None else {
            "hbm_frac_of_copy_rate": head_res["hbm_gbs"] / peaks["hbm_copy_gbs"],
            "dense_run_frac_of_gemm_rate": head_res["dense_tflops"] / peaks["bf16_gemm_tflops"]},
        "cpu_baseline": cpu,
        "parity": parity,
        "mask_construction": mask_construction,
        "backward": backward,
        "split_forward": split_forward,
        "cropped_forward": cropped,
        "decode": decode,
        "entmax15_forward": entmax,
        "per_config": per_config,
    }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
