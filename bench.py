#!/usr/bin/env python3
"""Benchmark of the VQ GEMV hot path on one MI355X.

A "step" is one per-token weight pass of a synthetic Llama-7B decoder: 32 layers x
{q,k,v,o 4096x4096; gate,up 11008x4096; down 4096x11008}, 2-D VQ, k=16, 8x256 groups,
224 batch-1 products y = W x over 1.83 GB of distinct packed weights (so the pass is
HBM-cold by construction).  The pass is issued through vq_gemv_multi (the whole pass
in one launch: up to 256 products per launch).  The JSON line also carries per-shape us/call of single
vq_gemv calls (HBM-cold rotation and cache-resident), the k=256 MLP shapes, the
batched GEMM, the roofline of the dominant kernel and the CPU oracle timed on the
host cores.

Contract: python bench.py --gpus 1 --steps K --warmup W  -> one JSON line on stdout.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
# HBM bytes one launch of the dominant kernel moves (the whole pass of 224 matrices), from
# rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE scaled by a copy kernel of known size; the summary
# and the commands are in profiles/gemv_stream_k16_llama7b_pass.md.  The figure belongs to one
# build of the kernel: it is reported only while the library still has the version it was
# measured on (vq_version() is raised whenever a kernel, the device layout or the set of entry
# points changes).
TRAFFIC_BYTES_PER_LAUNCH = 1857737421
TRAFFIC_MEASURED_ON_VERSION = 2
MFMA_F16_PEAK_TFLOPS = 2500.0  # MI355X published dense fp16 matrix peak
FP32_VECTOR_PEAK_TFLOPS = 157.3   # published fp32 vector peak (fused multiply-add = 2 flops)


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def algorithmic_bytes(s) -> int:
    """indices + codebooks + x + y(fp16), each counted once."""
    import workloads
    ib, cb = workloads.canonical_sizes(s)
    return ib + cb + 2 * s.in_features + 2 * s.out_features


class Timer:
    """HIP-event timing on torch's current stream (the stream the kernels are launched on)."""

    def __init__(self, torch):
        self.torch = torch

    def run(self, fn, iters, warmup):
        t = self.torch
        for _ in range(warmup):
            fn()
        t.cuda.synchronize()
        e0, e1 = t.cuda.Event(enable_timing=True), t.cuda.Event(enable_timing=True)
        wall0 = time.perf_counter()
        e0.record()
        for _ in range(iters):
            fn()
        e1.record()
        t.cuda.synchronize()
        wall = time.perf_counter() - wall0
        return e0.elapsed_time(e1) / iters, wall * 1e3 / iters   # ms per iteration (device, wall)

    def settle(self, fn, block=10, agree=5, tol=0.02, max_passes=4000):
        """Runs fn in blocks of `block` calls, each block timed with events, until `agree` blocks
        in a row lie within `tol` of each other (the GPU's clocks take tens of milliseconds of
        load to settle) or `max_passes` calls have been made.  Returns (calls made, ms spent,
        ms per call of the last block, whether the blocks agreed)."""
        t = self.torch
        recent, calls, spent = [], 0, 0.0
        while calls < max_passes:
            e0, e1 = t.cuda.Event(enable_timing=True), t.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(block):
                fn()
            e1.record()
            t.cuda.synchronize()
            ms = e0.elapsed_time(e1)
            calls += block
            spent += ms
            recent = (recent + [ms / block])[-agree:]
            if len(recent) == agree and max(recent) <= (1.0 + tol) * min(recent):
                return calls, spent, recent[-1], True
        return calls, spent, recent[-1], False


def build_pass(torch, vq, vqdev, n_layers):
    """Device-resident weights of the 7B pass: list of (name, shape, desc, idx_d, cb_d)."""
    import workloads
    mats = []
    t0 = time.time()
    for (layer, name, s, seed) in workloads.llama7b_pass_shapes():
        if layer >= n_layers:
            break
        idx, cb = workloads.make_weights(s, seed)
        desc = vqdev.desc_from_shape(s)
        idx_d, cb_d = vqdev.upload_and_pack(desc, idx, cb)
        mats.append((f"L{layer}.{name}", s, desc, idx_d, cb_d))
    log(f"[bench] built {len(mats)} matrices in {time.time() - t0:.1f}s")
    return mats


def time_cpu_baseline():
    """The CPU oracle as it stands (decode -> dense fp16 W -> fp64 y = W x) timed on the host
    cores, on a bounded sample of the same workloads: the attention matrix (4096 x 4096, k = 16),
    the two MLP shapes with k = 256, and the first four decoder layers of the full pass (28 matrices,
    k = 16; the pass is 32 layers), each once with the numerical library held to one thread and
    once with all the threads it takes by default.  Input generation is not timed.  The headline
    figure is the all-thread rate on the layer of the pass."""
    import oracle
    import workloads
    try:
        from threadpoolctl import threadpool_info, threadpool_limits
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads, threadpool_limits = 1, None

    def run(items, limit):
        """items: [(shape, seed)] -> (seconds of oracle time, algorithmic bytes)."""
        spent, nbytes = 0.0, 0
        for s, seed in items:
            idx, cb = workloads.make_weights(s, seed)
            x = workloads.make_x(s.in_features, seed)
            f = oracle.VQFormat(s.out_features, s.in_features, s.k, s.index_bits)
            t1 = time.perf_counter()
            if limit is None or threadpool_limits is None:
                oracle.gemv(f, idx, cb, x)
            else:
                with threadpool_limits(limits=limit):
                    oracle.gemv(f, idx, cb, x)
            spent += time.perf_counter() - t1
            nbytes += algorithmic_bytes(s)
        return spent, nbytes

    layers4 = [(s, seed) for (layer, name, s, seed) in workloads.llama7b_pass_shapes() if layer < 4]
    samples = {
        "attn_4096x4096_k16": [(workloads.CONFIGS["attn_4096x4096_k16"], workloads.seed_for("attn_4096x4096_k16"))],
        "mlp_up_11008x4096_k256": [(workloads.CONFIGS["mlp_up_11008x4096_k256"], workloads.seed_for("mlp_up_11008x4096_k256"))],
        "mlp_down_4096x11008_k256": [(workloads.CONFIGS["mlp_down_4096x11008_k256"], workloads.seed_for("mlp_down_4096x11008_k256"))],
        "llama7b_pass_k16_4_layers_of_32": layers4,
    }
    per, total = {}, 0.0
    for name, items in samples.items():
        t1, nb = run(items, 1)
        ta, _ = run(items, None)
        total += t1 + ta
        per[name] = {"bytes": nb, "one_thread_s": t1, "one_thread_GB/s": nb / t1 / 1e9,
                     "all_threads_s": ta, "all_threads_GB/s": nb / ta / 1e9}
        log(f"[bench] oracle on {name}: {t1:.2f} s with one thread, {ta:.2f} s with {threads}")
    head = per["llama7b_pass_k16_4_layers_of_32"]
    return {
        "value": head["all_threads_GB/s"], "unit": "GB/s", "cores": threads, "kind": "oracle",
        "sample": f"the first 4 decoder layers of the pass (28 matrices, {head['bytes']} algorithmic bytes; the pass "
                  f"is 32 layers, so it would take about {8 * head['all_threads_s']:.0f} s) in "
                  f"{head['all_threads_s']:.2f} s of oracle time with {threads} threads; {os.cpu_count()} host cpus "
                  f"visible; all samples together {total:.1f} s",
        "seconds": head["all_threads_s"],
        "one_thread_value": head["one_thread_GB/s"],
        "per_config": per,
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=50,
                    help="untimed passes first; the GPU needs some tens of ms of load to settle its clocks")
    ap.add_argument("--layers", type=int, default=32, help="layers of the 7B pass (32 = the workload)")
    ap.add_argument("--no-extras", action="store_true", help="skip per-shape / GEMM side measurements")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--no-settle", action="store_true",
                    help="skip the settle phase before the timed steps (the clocks then still move)")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run a plain device copy of 1 GiB (a kernel of known traffic, for scaling "
                         "rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    import workloads
    import paper_2402_15319_amd as vq
    from paper_2402_15319_amd import device as vqdev
    from paper_2402_15319_amd import bench_probe as vqprobe

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    vq.lib()
    torch.cuda.set_device(0)
    timer = Timer(torch)
    dev = "cuda:0"

    # ------------------------------------------------------------------ the pass
    mats = build_pass(torch, vq, vqdev, args.layers)
    xs = {n: torch.randn(n, device=dev, dtype=torch.float32, generator=torch.Generator(dev).manual_seed(1)).half()
          for n in (4096, 11008)}
    ys = [torch.empty(s.out_features, dtype=torch.float16, device=dev) for (_, s, _, _, _) in mats]
    margs = vq.GemvMultiArgs([m[2] for m in mats], [m[3] for m in mats], [m[4] for m in mats],
                             [xs[m[1].in_features] for m in mats], ys)
    pass_bytes = sum(algorithmic_bytes(m[1]) for m in mats)
    n_launch = (len(mats) + 255) // 256

    def step_multi():
        vq.vq_gemv_multi(margs)

    # The same W warm-up and K timed steps twice: once at once on the idle GPU ("unsettled": the
    # first tens of milliseconds of load run at clocks that are still moving), and once, the
    # reported value, after a disclosed settle phase of the same launch (blocks of 10 passes until
    # 5 blocks in a row agree within 2 %).
    ms_unsettled, _ = timer.run(step_multi, args.steps, args.warmup)
    settle_passes, settle_ms, settle_last, settled = (0, 0.0, None, False) if args.no_settle else \
        timer.settle(step_multi)
    ms_multi, wall_multi = timer.run(step_multi, args.steps, args.warmup)
    log(f"[bench] pass via vq_gemv_multi: {ms_multi * 1e3:.1f} us/step, {pass_bytes / ms_multi / 1e6:.0f} GB/s "
        f"(unsettled first {args.warmup}+{args.steps} passes: {ms_unsettled * 1e3:.1f} us/step; settle phase "
        f"{settle_passes} passes, {settle_ms:.0f} ms, agreed={settled})")

    extras = {}
    if args.pmc_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)          # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst
    # the achievable ceiling next to the nominal peak: a plain read of 1.75 GiB
    probe = torch.empty(1792 << 20, dtype=torch.uint8, device=dev).fill_(3)
    ms_probe, _ = timer.run(lambda: vqprobe.vq_bench_stream_read(probe, probe.numel()), 10, 3)
    stream_read_gbs = probe.numel() / ms_probe / 1e6
    del probe
    log(f"[bench] stream-read ceiling: {stream_read_gbs:.0f} GB/s")
    if not args.no_extras:
        # 8 layers of the same model with k = 256 (8-bit indices, 1 KB codebook per group:
        # 8 bits per value, 1.62 GB, HBM-cold): a quarter of the lookups per byte
        s256 = [workloads.VQShape(workloads.CONFIGS[key].out_features, workloads.CONFIGS[key].in_features, 256, 8)
                for _ in range(8) for (_, key) in workloads.LLAMA7B_LAYER]
        m256 = []
        for s in s256:
            desc = vqdev.desc_from_shape(s)
            ib, cbb = vq.vq_layout_bytes(desc)
            m256.append((s, desc, torch.randint(0, 256, (ib,), dtype=torch.uint8, device=dev),
                         (torch.randn(cbb // 2, device=dev) * 0.02).half().view(torch.uint8)))
        y256 = [torch.empty(s.out_features, dtype=torch.float16, device=dev) for s in s256]
        a256 = vq.GemvMultiArgs([m[1] for m in m256], [m[2] for m in m256], [m[3] for m in m256],
                                [xs[m[0].in_features] for m in m256], y256)
        b256 = sum(algorithmic_bytes(s) for s in s256)
        ms256, _ = timer.run(lambda: vq.vq_gemv_multi(a256), max(10, args.steps // 4), 20)
        extras["llama7b_8_layers_k256_via_vq_gemv_multi"] = {
            "us": ms256 * 1e3, "bytes": b256, "GB/s": b256 / ms256 / 1e6,
            "frac_hbm": b256 / ms256 / 1e6 / HBM_PEAK_GBS, "kernel": "gemv_stream_kernel<256>"}
        log(f"[bench] 8 layers with k=256: {ms256 * 1e3:.1f} us, {b256 / ms256 / 1e6:.0f} GB/s")
        del m256, y256, a256

        # the whole pass in the other representations.  Int8 lookup tables and a scale per group,
        # the paper's own table type: k = 64, 6-bit indices, 32 x 256 groups (the deployed representation, 3.125 bits
        # per value, 2.54 GB) and k = 16, 8 x 256 groups (2.125 bits per value, 1.73 GB).  Timing
        # only, so the device-layout buffers are filled with random bytes directly (every index
        # and int8 pattern is valid); the fp16 scales are set to 2^-8.
        for label, layer_keys, kernel in (
                ("llama7b_pass_k64_int8_tables_3.125bpv_via_vq_gemv_multi", workloads.LLAMA7B_LAYER_K64,
                 "gemv_stream_kernel<64>"),
                ("llama7b_pass_k16_int8_tables_2.125bpv_via_vq_gemv_multi", workloads.LLAMA7B_LAYER_K16_I8,
                 "gemv_stream_kernel<k16,int8>"),
                # k = 32, 5-bit indices (the appendix table's 2.5-bits-per-dimension 2D row): 2.76 bits per value
                ("llama7b_pass_k32_int8_tables_2.76bpv_via_vq_gemv_multi", workloads.LLAMA7B_LAYER_K32,
                 "gemv_stream_kernel<k32>"),
                # the same with groups of 4 x 256 weights (the appendix table's 2D row at 2.25 bpv; 2.27 with the scales)
                ("llama7b_pass_k16_int8_tables_4row_groups_2.27bpv_via_vq_gemv_multi", workloads.LLAMA7B_LAYER_K16_I8_G4,
                 "gemv_stream_kernel<k16,i8,4-row groups>"),
                # the 4-bits-per-dimension 2D setting: k = 256, int8 tables shared by 128 x 256 groups (4.125 bpv)
                ("llama7b_pass_k256_int8_tables_4.125bpv_via_vq_gemv_multi", workloads.LLAMA7B_LAYER_K256_I8,
                 "gemv_k256i8_kernel"),
                # the deployed representation with blockwise normalisation on top (appendix): 16 levels
                # per group and a 4-bit code per 32 weights, 3.28 bits per value
                ("llama7b_pass_k64_int8_tables_block_norm_3.28bpv_via_vq_gemv_multi", workloads.LLAMA7B_LAYER_K64_BN,
                 "gemv_stream_kernel<64,bn>"),
                # the 2.125 bpv setting with blockwise normalisation on top: 2.38 bits per value
                ("llama7b_pass_k16_int8_tables_block_norm_2.38bpv_via_vq_gemv_multi", workloads.LLAMA7B_LAYER_K16_BN,
                 "gemv_stream_kernel<k16,bn>"),
                # the 4.125 bpv 2D setting and the 4D setting with blockwise normalisation on top
                ("llama7b_pass_k256_int8_tables_block_norm_4.26bpv_via_vq_gemv_multi", workloads.LLAMA7B_LAYER_K256_BN,
                 "gemv_k256i8_kernel<bn>"),
                ("llama7b_pass_d4_k256_int8_tables_block_norm_2.25bpv_via_vq_gemv_multi", workloads.LLAMA7B_LAYER_D4_BN,
                 "gemv_d4_kernel<bn>"),
                # four-dimensional vectors: k = 256, one index byte per 4 weights, 256 x 256 groups (2.125 bpv)
                ("llama7b_pass_d4_k256_int8_tables_2.125bpv_via_vq_gemv_multi", workloads.LLAMA7B_LAYER_D4,
                 "gemv_d4_kernel"),
                # scalar codebooks at 3 bits: 8 int8 values + scale per 32 x 256 group (3.01 bpv)
                ("llama7b_pass_d1_k8_int8_3.01bpv_via_vq_gemv_multi", workloads.LLAMA7B_LAYER_D1_K8,
                 "gemv_stream_kernel<d1,k8>"),
                # the same with blockwise normalisation on top: 3.17 bits per value
                ("llama7b_pass_d1_k8_int8_block_norm_3.17bpv_via_vq_gemv_multi", workloads.LLAMA7B_LAYER_D1_K8_BN,
                 "gemv_stream_kernel<d1,k8,bn>"),
                # scalar codebooks at 2 bits: 4 int8 values + scale per row of a col-block (2.19 bpv)
                ("llama7b_pass_d1_k4_int8_2.19bpv_via_vq_gemv_multi", workloads.LLAMA7B_LAYER_D1_K4,
                 "gemv_stream_kernel<d1,k4>"),
                # scalar codebooks (d = 1): 16 fp16 values per 8 x 256 group, 4-bit indices, 3.47 GB
                ("llama7b_pass_d1_k16_4.125bpv_via_vq_gemv_multi", workloads.LLAMA7B_LAYER_D1_K16,
                 "gemv_stream_kernel<d1,k16>")):
            mi8 = []
            for _ in range(args.layers):
                for (_, key) in layer_keys:
                    s = workloads.CONFIGS[key]
                    desc = vqdev.desc_from_shape(s)
                    ib, cbb = vq.vq_layout_bytes(desc)
                    tab = torch.randint(0, 256, (cbb,), dtype=torch.uint8, device=dev)
                    if s.int8_tables and s.k == 256:    # 1 KB (d = 4) or 512-byte int8 tables per group, then fp16 scales (2^-8);
                        n_groups = (s.out_features // s.group_rows) * (s.in_features // 256)   # block-normalised: + levels (1.0), codes
                        t_end = n_groups * (1024 if s.d == 4 else 512)
                        s_end = t_end + (2 * n_groups + 15) // 16 * 16
                        tab[t_end:s_end] = 0
                        tab[t_end + 1:t_end + 2 * n_groups:2] = 0x1C
                        if s.block_norm:
                            tab[s_end:s_end + 32 * n_groups:2] = 0
                            tab[s_end + 1:s_end + 32 * n_groups:2] = 0x3C
                    elif s.d == 1 and s.k == 8 and s.block_norm:   # 176-byte records: the same + 64 levels (1.0); then codes
                        n_rec = (s.out_features // s.group_rows) * ((s.in_features // 256 + 3) // 4)
                        tv = tab[:n_rec * 176].view(-1, 176)
                        tv[:, 32:176] = 0
                        tv[:, 33:40:2] = 0x1C
                        tv[:, 49:176:2] = 0x3C
                    elif s.d == 1 and s.k == 8:         # 48-byte records: 4 x 8 int8, 4 scales (2^-8), padding
                        tv = tab.view(-1, 48)
                        tv[:, 32:48] = 0
                        tv[:, 33:40:2] = 0x1C
                    elif s.d == 1 and s.k == 4:         # 48-byte records: 8 x 4 int8, 8 scales (2^-8)
                        tv = tab.view(-1, 48)
                        tv[:, 32:48:2] = 0
                        tv[:, 33:48:2] = 0x1C
                    elif s.d == 1:                      # fp16 scalars
                        tab = (torch.randn(cbb // 2, device=dev) * 0.02).half().view(torch.uint8)
                    elif s.block_norm and s.k == 16:    # tables, scales (2^-8), padding, levels (1.0), nibble codes
                        n_slots = (s.out_features // 8) * 2 * ((s.in_features // 256 + 1) // 2)
                        lev0 = (34 * n_slots + 15) // 16 * 16
                        tab[n_slots * 32:lev0] = 0
                        tab[n_slots * 32 + 1:n_slots * 34:2] = 0x1C
                        tab[lev0:lev0 + 32 * n_slots:2] = 0
                        tab[lev0 + 1:lev0 + 32 * n_slots:2] = 0x3C
                    elif s.block_norm:                  # 672-byte records (+ 64 levels, set to 1.0), then nibble codes
                        n_rec = (s.out_features // s.group_rows) * ((s.in_features // 256 + 3) // 4)
                        tv = tab[:n_rec * 672].view(-1, 672)
                        tv[:, 512:528] = 0
                        tv[:, 513:520:2] = 0x1C
                        tv[:, 528:672] = 0
                        tv[:, 529:656:2] = 0x3C
                    elif s.k == 64:                       # 528-byte records: 4 tables, 4 scales, padding
                        tv = tab.view(-1, 528)
                        tv[:, 512:528] = 0
                        tv[:, 513:520:2] = 0x1C
                    elif s.k == 32:                     # 64 bytes of table per slot, then 2 bytes of scale per slot
                        n_slots = cbb // 66
                        tab[n_slots * 64::2] = 0
                        tab[n_slots * 64 + 1::2] = 0x1C
                    else:                               # 32 bytes per table, then 2 bytes of scale per table (4-row groups: two per slot)
                        n_slots = cbb // 34
                        tab[n_slots * 32::2] = 0
                        tab[n_slots * 32 + 1::2] = 0x1C
                    mi8.append((s, desc, torch.randint(0, 256, (ib,), dtype=torch.uint8, device=dev), tab))
            yi8 = [torch.empty(m[0].out_features, dtype=torch.float16, device=dev) for m in mi8]
            ai8 = vq.GemvMultiArgs([m[1] for m in mi8], [m[2] for m in mi8], [m[3] for m in mi8],
                                   [xs[m[0].in_features] for m in mi8], yi8)
            bi8 = sum(sum(workloads.canonical_sizes(m[0])) + 2 * m[0].in_features + 2 * m[0].out_features
                      for m in mi8)
            msi8, _ = timer.run(lambda: vq.vq_gemv_multi(ai8), max(10, args.steps // 2), 50)
            extras[label] = {"us": msi8 * 1e3, "bytes": bi8, "GB/s": bi8 / msi8 / 1e6,
                             "frac_hbm": bi8 / msi8 / 1e6 / HBM_PEAK_GBS,
                             "tokens_per_s_weight_stream": 1e3 / msi8, "kernel": kernel}
            log(f"[bench] {label}: {msi8 * 1e3:.1f} us, {bi8 / msi8 / 1e6:.0f} GB/s")
            del mi8, yi8, ai8

        # the same pass as 224 separate vq_gemv calls (plain stream launches)
        def step_single():
            for i, (_, s, desc, idx_d, cb_d) in enumerate(mats):
                vq.vq_gemv(desc, idx_d, cb_d, xs[s.in_features], ys[i])
        ms_single, wall_single = timer.run(step_single, max(2, args.steps // 4), 1)
        extras["pass_as_separate_vq_gemv_calls"] = {
            "us_per_pass": ms_single * 1e3, "GB/s": pass_bytes / ms_single / 1e6,
            "us_per_call": ms_single * 1e3 / len(mats), "wall_us_per_pass": wall_single * 1e3}
        log(f"[bench] pass via {len(mats)} vq_gemv calls: {ms_single * 1e3:.1f} us/step")

        # the same 224 separate launches captured once in a HIP graph and replayed: what the
        # per-matrix path costs without the host launch path
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step_single()
        ms_graph, _ = timer.run(graph.replay, max(2, args.steps // 4), 2)
        extras["pass_as_separate_vq_gemv_calls_in_hip_graph"] = {
            "us_per_pass": ms_graph * 1e3, "GB/s": pass_bytes / ms_graph / 1e6,
            "us_per_call": ms_graph * 1e3 / len(mats)}
        log(f"[bench] pass via {len(mats)} vq_gemv calls in a HIP graph: {ms_graph * 1e3:.1f} us/step")
        del graph

        # a decode-like launch sequence: per layer q/k/v in one launch, o, gate/up in one launch,
        # down (what the data dependencies of a decoder allow), replayed from a HIP graph
        if args.layers == 32:
            seq = []
            for l in range(args.layers):
                for sel in ((0, 1, 2), (3,), (4, 5), (6,)):
                    ii = [7 * l + i for i in sel]
                    seq.append(vq.GemvMultiArgs([mats[i][2] for i in ii], [mats[i][3] for i in ii],
                                                [mats[i][4] for i in ii],
                                                [xs[mats[i][1].in_features] for i in ii], [ys[i] for i in ii]))

            def step_layerwise():
                for a in seq:
                    vq.vq_gemv_multi(a)
            step_layerwise()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                step_layerwise()
            ms_lw, _ = timer.run(graph.replay, max(2, args.steps // 4), 3)
            extras["pass_as_4_launches_per_layer_in_hip_graph"] = {
                "us_per_pass": ms_lw * 1e3, "GB/s": pass_bytes / ms_lw / 1e6, "launches": len(seq),
                "us_per_launch": ms_lw * 1e3 / len(seq), "tokens_per_s_weight_stream": 1e3 / ms_lw}
            log(f"[bench] pass as {len(seq)} launches (qkv | o | gate,up | down) in a HIP graph: "
                f"{ms_lw * 1e3:.1f} us/step")
            del graph

            # the same sequence with a rank-16 adapter next to every matrix (y = W x + B (A x)):
            # each step is two launches (t = A x, then the product with the adapter term); the
            # entry point without a workspace, so the graph captures no allocation
            rank = 16
            lA = {n: (torch.randn((rank, n), device=dev) / n ** 0.5).half() for n in (4096, 11008)}
            lB = {n: (torch.randn((n, rank), device=dev) * 0.02).half() for n in (4096, 11008)}
            lsel = [[7 * l + i for i in sel] for l in range(args.layers) for sel in ((0, 1, 2), (3,), (4, 5), (6,))]
            lAs = [[lA[mats[i][1].in_features] for i in ii] for ii in lsel]
            lBs = [[lB[mats[i][1].out_features] for i in ii] for ii in lsel]

            def step_layerwise_lora():
                for a, As, Bs in zip(seq, lAs, lBs):
                    vq.vq_gemv_lora_multi_static(a, As, Bs, [rank] * a.count)
            step_layerwise_lora()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                step_layerwise_lora()
            ms_ll, _ = timer.run(graph.replay, max(2, args.steps // 4), 3)
            lora_bytes = sum(2 * rank * (mats[i][1].in_features + mats[i][1].out_features) for ii in lsel for i in ii)
            extras["pass_as_4_launches_per_layer_with_rank16_adapters_in_hip_graph"] = {
                "us_per_pass": ms_ll * 1e3, "GB/s": (pass_bytes + lora_bytes) / ms_ll / 1e6,
                "adapter_bytes": lora_bytes, "launches": 2 * len(seq),
                "us_per_step_of_two_launches": ms_ll * 1e3 / len(seq)}
            log(f"[bench] the same with rank-{rank} adapters ({2 * len(seq)} launches): {ms_ll * 1e3:.1f} us/step")
            del graph, seq, lAs, lBs

        # per-shape us/call: HBM-cold (rotate over the distinct matrices of the pass) and
        # cache-resident (same matrix every call), both as plain calls from Python (bounded below
        # by the host launch path), and HBM-cold with one call per distinct copy captured in a
        # HIP graph (device time per call, no host in the loop)
        def graph_us_per_call(calls):
            for f in calls:
                f()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                for f in calls:
                    f()
            ms, _ = timer.run(g.replay, 20, 3)
            del g
            return ms * 1e3 / len(calls)

        per_shape = {}
        for key in ("attn_4096x4096_k16", "mlp_up_11008x4096_k16", "mlp_down_4096x11008_k16"):
            s0 = workloads.CONFIGS[key]
            sel = [i for i, m in enumerate(mats) if m[1] == s0]
            if not sel:
                continue
            state = {"i": 0}

            def cold():
                i = sel[state["i"] % len(sel)]
                state["i"] += 1
                m = mats[i]
                vq.vq_gemv(m[2], m[3], m[4], xs[s0.in_features], ys[i])

            def hot():
                m = mats[sel[0]]
                vq.vq_gemv(m[2], m[3], m[4], xs[s0.in_features], ys[sel[0]])
            nb = algorithmic_bytes(s0)
            ms_c, _ = timer.run(cold, 4 * len(sel), len(sel))
            ms_h, _ = timer.run(hot, 500, 20)
            us_g = graph_us_per_call([
                (lambda m=mats[i], i=i: vq.vq_gemv(m[2], m[3], m[4], xs[s0.in_features], ys[i])) for i in sel])
            per_shape[key] = {"bytes": nb, "distinct_copies": len(sel),
                              "cold_us": ms_c * 1e3, "cold_GB/s": nb / ms_c / 1e6,
                              "cold_frac_hbm": nb / ms_c / 1e6 / HBM_PEAK_GBS,
                              "hot_us": ms_h * 1e3, "hot_GB/s": nb / ms_h / 1e6,
                              "cold_in_hip_graph_us": us_g, "cold_in_hip_graph_GB/s": nb / us_g / 1e3,
                              "cold_in_hip_graph_frac_hbm": nb / us_g / 1e3 / HBM_PEAK_GBS}
            log(f"[bench] {key}: cold {ms_c * 1e3:.2f} us, hot {ms_h * 1e3:.2f} us, cold in a HIP graph {us_g:.2f} us")

        # k = 256 MLP shapes (8 bits per weight): 12 distinct copies each (> 512 MB in total)
        for key in ("mlp_up_11008x4096_k256", "mlp_down_4096x11008_k256"):
            s0 = workloads.CONFIGS[key]
            desc = vqdev.desc_from_shape(s0)
            copies = []
            for j in range(12):
                idx, cb = workloads.make_weights(s0, workloads.seed_for(key, j))
                copies.append(vqdev.upload_and_pack(desc, idx, cb))
            y = torch.empty(s0.out_features, dtype=torch.float16, device=dev)
            state = {"i": 0}

            def cold():
                a, b = copies[state["i"] % len(copies)]
                state["i"] += 1
                vq.vq_gemv(desc, a, b, xs[s0.in_features], y)

            def hot():
                vq.vq_gemv(desc, copies[0][0], copies[0][1], xs[s0.in_features], y)
            nb = algorithmic_bytes(s0)
            ms_c, _ = timer.run(cold, 120, 12)
            ms_h, _ = timer.run(hot, 200, 10)
            us_g = graph_us_per_call([
                (lambda c=c: vq.vq_gemv(desc, c[0], c[1], xs[s0.in_features], y)) for c in copies])
            per_shape[key] = {"bytes": nb, "distinct_copies": len(copies),
                              "cold_us": ms_c * 1e3, "cold_GB/s": nb / ms_c / 1e6,
                              "cold_frac_hbm": nb / ms_c / 1e6 / HBM_PEAK_GBS,
                              "hot_us": ms_h * 1e3, "hot_GB/s": nb / ms_h / 1e6,
                              "cold_in_hip_graph_us": us_g, "cold_in_hip_graph_GB/s": nb / us_g / 1e3,
                              "cold_in_hip_graph_frac_hbm": nb / us_g / 1e3 / HBM_PEAK_GBS}
            log(f"[bench] {key}: cold {ms_c * 1e3:.2f} us, hot {ms_h * 1e3:.2f} us, cold in a HIP graph {us_g:.2f} us")
            # batched / prefill GEMM on the same matrix, next to a dense fp16 GEMM on decoded W
            Wd = torch.empty((s0.out_features, s0.in_features), dtype=torch.float16, device=dev)
            if key == "mlp_up_11008x4096_k256":
                def decode_cold():
                    a, b = copies[state["i"] % len(copies)]
                    state["i"] += 1
                    vq.vq_decode_dense(desc, a, b, Wd)
                ms_dec, _ = timer.run(decode_cold, 60, 12)
                nb_dec = nb + 2 * s0.out_features * s0.in_features      # compressed in, fp16 W out
                extras["decode_dense_11008x4096_k256"] = {
                    "us": ms_dec * 1e3, "bytes_in_plus_out": nb_dec, "GB/s": nb_dec / ms_dec / 1e6,
                    "frac_hbm": nb_dec / ms_dec / 1e6 / HBM_PEAK_GBS}
                log(f"[bench] decode_dense {key}: {ms_dec * 1e3:.1f} us, {nb_dec / ms_dec / 1e6:.0f} GB/s in+out")
            vq.vq_decode_dense(desc, copies[0][0], copies[0][1], Wd)
            gemm = {}
            for B in (16, 256, 2048):
                X = torch.randn((s0.in_features, B), device=dev, dtype=torch.float32).half()
                Y = torch.empty((s0.out_features, B), dtype=torch.float16, device=dev)
                ms_g, _ = timer.run(lambda: vq.vq_gemm_batched(desc, copies[0][0], copies[0][1], X, B, B, Y, B),
                                    40, 10)
                ms_d, _ = timer.run(lambda: torch.matmul(Wd, X, out=Y), 40, 10)
                fl = 2.0 * s0.out_features * s0.in_features * B
                # the two-step alternative with a caller-owned dense buffer: decode, then dense GEMM
                def two_step():
                    vq.vq_decode_dense(desc, copies[0][0], copies[0][1], Wd)
                    torch.matmul(Wd, X, out=Y)
                ms_2, _ = timer.run(two_step, 40, 10)
                gemm[f"B{B}"] = {"us": ms_g * 1e3, "TFLOP/s": fl / ms_g / 1e9,
                                 "frac_mfma_f16": fl / ms_g / 1e9 / MFMA_F16_PEAK_TFLOPS,
                                 "dense_fp16_matmul_us": ms_d * 1e3,
                                 "vq_decode_dense_then_dense_matmul_us": ms_2 * 1e3}
                log(f"[bench] gemm {s0.out_features}x{s0.in_features} B={B}: {ms_g * 1e3:.1f} us vs dense {ms_d * 1e3:.1f} us "
                    f"(decode + dense {ms_2 * 1e3:.1f} us)")
            extras[f"gemm_{s0.out_features}x{s0.in_features}_k256"] = gemm
            if key == "mlp_up_11008x4096_k256":
                # the same product on the 4.125-bit representation of this matrix (k = 256, int8 tables
                # shared by 128 x 256 groups); timing only, random index and table bytes, scales 2^-8
                s8 = workloads.CONFIGS["mlp_up_11008x4096_k256_i8"]
                d8 = vqdev.desc_from_shape(s8)
                ib8, cb8 = vq.vq_layout_bytes(d8)
                i8 = torch.randint(0, 256, (ib8,), dtype=torch.uint8, device=dev)
                t8 = torch.randint(0, 256, (cb8,), dtype=torch.uint8, device=dev)
                ng8 = (s8.out_features // s8.group_rows) * (s8.in_features // 256)
                t8[ng8 * 512:] = 0
                t8[ng8 * 512 + 1:ng8 * 514:2] = 0x1C
                gemm8 = {}
                for B in (16, 256, 2048):
                    X = torch.randn((s8.in_features, B), device=dev, dtype=torch.float32).half()
                    Y = torch.empty((s8.out_features, B), dtype=torch.float16, device=dev)
                    ms_g, _ = timer.run(lambda: vq.vq_gemm_batched(d8, i8, t8, X, B, B, Y, B), 40, 10)
                    fl = 2.0 * s8.out_features * s8.in_features * B
                    gemm8[f"B{B}"] = {"us": ms_g * 1e3, "TFLOP/s": fl / ms_g / 1e9,
                                      "frac_mfma_f16": fl / ms_g / 1e9 / MFMA_F16_PEAK_TFLOPS}
                    log(f"[bench] gemm on k=256 int8 tables (4.125 bpv) B={B}: {ms_g * 1e3:.1f} us")
                extras["gemm_11008x4096_k256_int8_tables_4.125bpv"] = gemm8
                del i8, t8
            del Wd
            del copies
        extras["per_shape_vq_gemv"] = per_shape

        # quantiser side: one E-step and one M-step of the Hessian-weighted EM on a 11008 x 4096
        # layer in fp32 (22,016 groups of 8 x 256, d = 2).  The E-step is plain vector ALU work:
        # 7 unfused fp32 operations per (vector, centroid); the chip's 157.3 TFLOP/s counts a
        # fused multiply-add as two, so separately rounded operations peak at half of it.
        em = {}
        Wq = (torch.randn((11008, 4096), device=dev) * 0.02).contiguous()
        hq = (torch.rand(4096, device=dev) * 4.8 + 0.2).contiguous()
        for kq in (16, 256):
            dq = vq.make_desc(11008, 4096, kq, 4 if kq == 16 else 8)
            n_groups = (11008 // 8) * (4096 // 256)
            cq = (torch.randn((n_groups, kq, 2), device=dev) * 0.02).contiguous()
            aq = torch.empty((11008, 2048), dtype=torch.uint8, device=dev)
            cq2 = torch.empty_like(cq)
            ms_e, _ = timer.run(lambda: vq.vq_em_assign(dq, Wq, hq, cq, aq), 20, 5)
            ms_m, _ = timer.run(lambda: vq.vq_em_update(dq, Wq, hq, aq, cq2), 20, 5)
            fl = 7.0 * 11008 * 2048 * kq
            em[f"k{kq}"] = {"e_step_us": ms_e * 1e3, "m_step_us": ms_m * 1e3,
                            "e_step_TFLOP/s": fl / ms_e / 1e9,
                            "e_step_frac_of_unfused_fp32_peak": fl / ms_e / 1e9 / (FP32_VECTOR_PEAK_TFLOPS / 2),
                            "e_step_bytes": Wq.numel() * 4 + aq.numel() + cq.numel() * 4,
                            "m_step_GB/s": (Wq.numel() * 4 + aq.numel() + cq.numel() * 4) / ms_m / 1e6}
            log(f"[bench] EM k={kq}: E-step {ms_e * 1e3:.1f} us, M-step {ms_m * 1e3:.1f} us")
        extras["em_step_11008x4096_fp32"] = em
        del Wq, hq

    cpu = None if args.no_cpu else time_cpu_baseline()

    gbs = pass_bytes / ms_multi / 1e6
    launch_us = ms_multi * 1e3 / n_launch
    traffic = TRAFFIC_BYTES_PER_LAUNCH if (args.layers == 32 and vq.vq_version() == TRAFFIC_MEASURED_ON_VERSION) else None
    lw = extras.get("pass_as_4_launches_per_layer_in_hip_graph")
    out = {
        "metric": "VQ GEMV effective HBM GB/s on the compressed stream (us per call alongside), "
                  "Llama-7B shapes, batch 1",
        "value": gbs, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_multi, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f16", "data": "synthetic",
        "config": {"workload": f"llama7b_full_weight_pass_k16 ({len(mats)} GEMVs, {args.layers} layers, "
                               f"d=2, 8x256 groups, 2.25 bpv) via vq_gemv_multi",
                   "accumulate": "f32", "y_dtype": "f16",
                   "bytes_per_step": pass_bytes, "launches_per_step": n_launch,
                   "us_per_call": ms_multi * 1e3 / len(mats),
                   "tokens_per_s_weight_stream": 1e3 / ms_multi,
                   # how the timed region was prepared (the value is taken with settled clocks)
                   "settle_passes": settle_passes, "settle_ms": settle_ms, "settle_agreed": settled,
                   "unsettled_ms_per_step": ms_unsettled,
                   "unsettled_frac_hbm": pass_bytes / ms_unsettled / 1e6 / HBM_PEAK_GBS,
                   # the same 224 products in the order a decoder's data dependencies allow: four
                   # launches per layer (q/k/v | o | gate/up | down), replayed from a HIP graph
                   "dependency_respecting_us_per_pass": lw["us_per_pass"] if lw else None,
                   "dependency_respecting_frac_hbm": lw["GB/s"] / HBM_PEAK_GBS if lw else None},
        "roofline": {"bound": "hbm", "achieved": pass_bytes / n_launch / launch_us / 1e3,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": pass_bytes / n_launch / launch_us / 1e3 / HBM_PEAK_GBS,
                     "traffic": traffic,
                     "kernel": "gemv_stream_kernel<16, false>",
                     # HIP events around the K timed launches on the launch stream, per launch
                     "event_avg_us_per_launch": launch_us, "bytes_per_launch": pass_bytes / n_launch,
                     "measured_stream_read_GB/s": stream_read_gbs,
                     "frac_of_measured_stream_read": pass_bytes / n_launch / launch_us / 1e3 / stream_read_gbs},
        "cpu_baseline": cpu,
        "extras": extras,
    }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
