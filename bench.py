#!/usr/bin/env python3
"""bench.py — throughput of FADE's hot path on one MI355X.

A "step" is one pass of the whole hot path over one batch: for each of the B streams the model step
(embedding -> DMD -> HGR -> head -> softmax -> frequency table), the arithmetic coding of the next byte
and, in online mode, the weight update. The workload is benchmark configuration 5, the largest of the five
(1 GiB mixed source in 64 MiB blocks, B = 16384 streams, T = 64, D = 32, H = 512, bf16 operands): the timed
region codes steps [T + W, T + W + K) of every stream with the input already resident in HBM, first
compressing, then decompressing the same bytes (checked byte-exact). Only the first T + W + K bytes of every
stream travel to the GPU (the generators still produce the whole 1 GiB: a stream's first bytes depend on
everything before them in its block). `--full` runs the whole job end to end instead; `--config` picks
another configuration (1-5, or 6: the paper's default model shape).
The headline (`value`) is the method as Algorithm 1 defines it, weights updated after every coded symbol; the
default run also measures the same steps with frozen weights (inference only) and reports them under
`frozen_weights`.

Prints ONE JSON line (see the keys below); `roofline` describes the dominant kernel (the D_h x D_h router /
gate product), timed with HIP events on the library's stream in a second pass over the same steps;
`update_roofline` (online mode) does the same for the HBM-bound Adam pass over the nine big matrices; `cpu_baseline` times the CPU oracle on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MFMA_BF16_PEAK = 2.5e15   # MI355X dense bf16, FLOP/s
HBM_PEAK = 8.0e12         # B/s
MiB = 1 << 20
# HBM bytes per launch of the router / gate product by launch shape (rows M of the launch, update mode): scaled
# FETCH_SIZE + WRITE_SIZE of counter runs of this same program, one row of the named file under profiles/ each
# (FETCH x 2.0, WRITE x 1.0 against a plain 256 MiB copy, see profiles/cfg2_frozen_pmc_counters.md). A shape that
# was not profiled reports null.
ROUTER_GATE_TRAFFIC_BYTES = {
    (16384, 2048, "frozen"): int(0.5 * (320.4 + 66.2 + 314.1 + 66.1) * MiB),   # profiles/cfg5_frozen_kernel_trace_and_hbm.md (cfg 2's 16-step passes have the same shape)
    (16384, 2048, "online"): int(0.5 * (320.4 + 130.4 + 314.1 + 130.3) * MiB), # profiles/cfg5_online_kernel_trace_and_hbm.md
    (1024, 2048, "online"): int(0.5 * (48.1 + 8.2 + 45.2 + 8.2) * MiB),                    # profiles/cfg2_online_kernel_trace_and_hbm.md
}
# the same for the fp32 small-batch product (gemm_f32_rows_kernel) by (B, D_h, mode): profiles/cfg1_kernel_trace_and_hbm.md
F32_ROUTER_GATE_TRAFFIC_BYTES = {(16, 512, "frozen"): int(0.5 * (2.46 + 0.05 + 2.40 + 0.05) * MiB), (16, 512, "online"): int(0.5 * (2.46 + 0.08 + 2.40 + 0.08) * MiB)}
# adam_refresh_kernel by (parameters of the nine big matrices, mode), same counter runs
ADAM_TRAFFIC_BYTES = {(11272192, "online"): int((174.6 + 170.0) * MiB),      # profiles/cfg2_online_kernel_trace_and_hbm.md
                      (13369344, "online"): int((349.5 + 194.5) * MiB)}        # profiles/cfg5_online_kernel_trace_and_hbm.md


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2048)
    ap.add_argument("--warmup", type=int, default=64)
    ap.add_argument("--config", type=int, default=5, help="benchmark configuration (1-5; 6 = the paper-default model shape)")
    ap.add_argument("--mode", choices=["frozen", "online"], default=None)
    ap.add_argument("--ablation", type=int, default=0, choices=[0, 1, 2, 3, 4, 5],
                    help="head on a prefix of the model (the paper's progressive ablation)")
    ap.add_argument("--full", action="store_true", help="run the whole job (all L steps) instead of K timed steps")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a plain 256 MiB device copy (torch) so that a counter run can be scaled against known traffic")
    ap.add_argument("--oracle-streams", type=int, default=None, help="streams of the oracle sample (default 64, 48 at B >= 16384)")
    ap.add_argument("--oracle-steps", type=int, default=32, help="model steps of the oracle sample")
    return ap.parse_args()


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); --gpus must be 1", file=sys.stderr)
        sys.exit(2)
    import torch

    import fade_inputs as fi
    import paper_2604_07239_amd as fa
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if a.copy_calibration:
        x = torch.ones(256 << 20, dtype=torch.uint8, device="cuda")
        y = torch.empty_like(x)
        for _ in range(4):
            y.copy_(x)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes_each_way": x.numel(), "copies": 4}))
        return
    spec = fi.CONFIGS[a.config]
    B, T, D, H = spec["B"], spec["T"], spec["D"], spec["H"]
    widths = dict(d_cache=spec.get("d_cache", 0), d_e=spec.get("d_e", 0))
    Dc, De = widths["d_cache"] or H, widths["d_e"] or H
    Dh, dl = T * D, 64
    dtype = fa.BF16 if spec["dtype"] == "bf16" else fa.F32
    mode = a.mode or "online"   # the method adapts its weights while coding (Algorithm 1); frozen is the inference-only variant
    if 1 <= a.ablation <= 4:
        widths["ablation"] = a.ablation
    K, W = a.steps, a.warmup

    t_gen = time.perf_counter()
    full = fi.config_bytes(a.config)
    L = full.size // B
    Bo = min(a.oracle_streams or (48 if B >= 16384 else 64), B)
    So = a.oracle_steps
    osrc = np.ascontiguousarray(full.reshape(B, L)[:Bo, :T + So]).reshape(-1)   # the oracle's sample of the same workload
    if a.full:
        src = full
        first, count = 0, 0
    else:
        steps_total = min(L, T + W + K)
        K = steps_total - T - W
        src = np.ascontiguousarray(full.reshape(B, L)[:, :steps_total]).reshape(-1)
        first, count = T + W, K
    del full
    n = src.size
    blob = fi.config_blob(a.config)
    print(f"[bench] cfg{a.config}: input and weights generated in {time.perf_counter() - t_gen:.1f} s", file=sys.stderr, flush=True)
    # frozen bf16 compression carries several steps of every stream through one pass (fade_create's rule, restated)
    spp = 1
    if spec["dtype"] == "bf16":
        spp = max(1, min(256, 16384 // B, (1 << 26) // (B * Dh)))
        if os.environ.get("FADE_STEPS_PER_PASS"):
            spp = max(1, min(256, int(os.environ["FADE_STEPS_PER_PASS"])))

    def measure(mode):
        """compress + decompress of the timed steps in one update mode, then the event-profiled pass"""
        g = fa.Fade(fa.make_config(B, T, D, H, dtype=dtype, update_mode=fa.ONLINE_ADAM if mode == "online" else fa.FROZEN, **widths))
        g.load_weights(blob.data)
        src_dev = torch.from_numpy(src).cuda()
        dst_dev = torch.zeros(n, dtype=torch.uint8, device="cuda")
        torch.cuda.synchronize()

        def pieces(call):
            """the whole job in pieces of about 20 s, with a progress line after each (a long silent run reads as hung)"""
            per = max(1, L // 16)
            torch.cuda.synchronize(); t0 = time.perf_counter()
            done = 0
            while done < L:
                cnt = min(per, L - done)
                call(done, cnt)
                done += cnt
                print(f"[bench] {mode}: {done}/{L} steps, {time.perf_counter() - t0:.1f} s", file=sys.stderr, flush=True)
            torch.cuda.synchronize(); return time.perf_counter() - t0

        def timed_encode():
            if a.full:
                return pieces(lambda first, cnt: g.encode_device(src_dev, n, first, cnt))
            g.encode_device(src_dev, n, 0, first)          # uniform warm-up symbols + W untimed model steps
            torch.cuda.synchronize(); t0 = time.perf_counter()
            g.encode_device(src_dev, n, first, count)      # exactly K timed steps (and the termination of each stream)
            torch.cuda.synchronize(); return time.perf_counter() - t0

        def timed_decode(lens, data):
            if a.full:
                return pieces(lambda first, cnt: g.decode_device(lens, data, dst_dev, n, first, cnt))
            g.decode_device(lens, data, dst_dev, n, 0, first)
            torch.cuda.synchronize(); t0 = time.perf_counter()
            g.decode_device(None, None, dst_dev, n, first, count)
            torch.cuda.synchronize(); return time.perf_counter() - t0

        t_enc = timed_encode()
        print(f"[bench] {mode}: compressed {'the whole input' if a.full else f'{K} steps'} in {t_enc:.2f} s", file=sys.stderr, flush=True)
        lens, data = g.payloads()
        t_dec = timed_decode(lens, data)
        print(f"[bench] {mode}: decompressed in {t_dec:.2f} s", file=sys.stderr, flush=True)
        ok = bool(torch.equal(dst_dev, src_dev))
        steps_timed = L if a.full else K
        bytes_timed = n if a.full else B * K
        container = 64 + 4 * B + int(data.size)
        enc_MBps = bytes_timed / t_enc / 1e6
        dec_MBps = bytes_timed / t_dec / 1e6

        # second pass over the same steps with a HIP event pair around every launch (on the library's stream)
        # (whole passes only, so that every launch of a kernel has one shape and the per-launch figures below are exact)
        prof = {}
        steps_prof = count
        if not a.full:
            if mode == "frozen" and count >= spp:
                steps_prof = count // spp * spp
            g.encode_device(src_dev, n, 0, first)
            g.profile(True)
            g.encode_device(src_dev, n, first, steps_prof)
            prof = g.profile_read()
            g.profile(False)
        kern = {k: {"avg_us": 1e3 * ms / max(cnt, 1), "launches": int(cnt)} for k, (ms, cnt) in prof.items()}
        roofline = None
        if "gemm_router" in kern and spec["dtype"] == "bf16":
            # dominant kernel: alpha = sigma(X W_r) with the mix epilogue, and its twin the gate product (Eq. 5-6, 8)
            twins = [kern[k]["avg_us"] for k in ("gemm_router", "gemm_gate") if k in kern]
            us = sum(twins) / len(twins)
            # frozen compression carries several steps of every stream through one launch: rows = B * steps per pass
            rows = B * steps_prof // max(kern["gemm_router"]["launches"], 1)
            flop = 2.0 * rows * Dh * Dh
            ach = flop / (us * 1e-6) / 1e12
            # HBM bytes per launch of this shape from the counter runs under profiles/ (null for a shape that was not profiled)
            traffic = ROUTER_GATE_TRAFFIC_BYTES.get((rows, Dh, mode))
            roofline = {"bound": "mfma", "kernel": f"{'gemm_pipe2_kernel' if rows >= 8192 else 'gemm_pipe_kernel'} (router / gate product, M={rows}, N=K=D_h)", "achieved": round(ach, 2),
                        "peak": MFMA_BF16_PEAK / 1e12, "unit": "TFLOP/s", "frac": round(ach * 1e12 / MFMA_BF16_PEAK, 4),
                        "traffic": traffic, "avg_us": round(us, 2), "flop_per_launch": flop,
                        # operand rows, the two side inputs and the output (+ alpha / the gate, kept for the update only), W once
                        "algorithmic_bytes_per_launch": 2 * ((5 if mode == "online" else 4) * rows * Dh + Dh * Dh)}
        if roofline is None and "gemm_global" in kern and spec["dtype"] == "bf16":   # ablation level 1: the global projection is all there is
            us = kern["gemm_global"]["avg_us"]
            rows = B * steps_prof // max(kern["gemm_global"]["launches"], 1)
            flop = 2.0 * rows * Dc * Dh
            ach = flop / (us * 1e-6) / 1e12
            roofline = {"bound": "mfma", "kernel": f"gemm_pipe_kernel (global projection, M={rows}, K=D_cache, N=D_h)", "achieved": round(ach, 2),
                        "peak": MFMA_BF16_PEAK / 1e12, "unit": "TFLOP/s", "frac": round(ach * 1e12 / MFMA_BF16_PEAK, 4),
                        "traffic": None, "avg_us": round(us, 2), "flop_per_launch": flop,
                        "algorithmic_bytes_per_launch": 2 * (rows * Dc + Dc * Dh + 2 * rows * Dh)}
        if roofline and 2 * De > Dh and "gemm_fnr_in" in kern:
            # refiner-dominated shapes (D_e >> D_h, the paper's default model): the dominant product is Eq. 9's pair
            # H_coarse [W_fg | W_fv], M rows x K = D_h x N = 2 D_e, fp32 output for the folded LayerNorm + GeGLU that follows
            us = kern["gemm_fnr_in"]["avg_us"]
            rows = B * steps_prof // max(kern["gemm_fnr_in"]["launches"], 1)
            flop = 2.0 * rows * Dh * 2 * De
            ach = flop / (us * 1e-6) / 1e12
            roofline = {"bound": "mfma", "kernel": f"gemm_pipe_kernel (refiner input product, M={rows}, K=D_h, N=2 D_e)", "achieved": round(ach, 2),
                        "peak": MFMA_BF16_PEAK / 1e12, "unit": "TFLOP/s", "frac": round(ach * 1e12 / MFMA_BF16_PEAK, 4),
                        "traffic": None, "avg_us": round(us, 2), "flop_per_launch": flop,
                        "algorithmic_bytes_per_launch": 2 * rows * Dh + 2 * Dh * 2 * De + 4 * rows * 2 * De}
        if roofline is None and "gemm_router" in kern and spec["dtype"] == "f32":
            # fp32 at a small batch (cfg 1): every product streams its fp32 weight matrix once past a handful of rows, so the
            # step is bound by weight bytes (and by launch latency); the widest weight stream is the D_h x D_h router / gate product
            twins = [kern[k]["avg_us"] for k in ("gemm_router", "gemm_gate") if k in kern]
            us = sum(twins) / len(twins)
            nbytes = 4 * (Dh * Dh + (5 if mode == "online" else 4) * B * Dh)
            ach = nbytes / (us * 1e-6) / 1e9
            roofline = {"bound": "hbm", "kernel": f"gemm_f32_rows_kernel (router / gate product, M={B}, N=K=D_h, fp32 weights)", "achieved": round(ach, 2),
                        "peak": HBM_PEAK / 1e9, "unit": "GB/s", "frac": round(ach * 1e9 / HBM_PEAK, 5),
                        "traffic": F32_ROUTER_GATE_TRAFFIC_BYTES.get((B, Dh, mode)), "avg_us": round(us, 2), "algorithmic_bytes_per_launch": nbytes}
        update_roofline = None
        if "adam_matrices" in kern and spec["dtype"] == "bf16":
            # the HBM-bound pass of the update over the shared weights: Adam on the nine big matrices fused with the refresh of their bf16
            # operand copies. Per parameter: gradient, both moments and the master weight read (16 B), moments and weight
            # written (12 B), one bf16 copy per orientation the products use (2 B each; W_m has one orientation only).
            P = 2 * Dh * Dh + 3 * Dh * De + Dc * Dh + 256 * Dh + 2 * dl * Dh
            nbytes = 32 * P - 2 * Dc * Dh
            us = kern["adam_matrices"]["avg_us"]
            ach = nbytes / (us * 1e-6) / 1e9
            update_roofline = {"bound": "hbm", "kernel": "adam_refresh_kernel (Adam + operand refresh of the nine big matrices)",
                               "achieved": round(ach, 1), "peak": HBM_PEAK / 1e9, "unit": "GB/s", "frac": round(ach * 1e9 / HBM_PEAK, 4),
                               "traffic": ADAM_TRAFFIC_BYTES.get((P, mode)), "avg_us": round(us, 2), "algorithmic_bytes_per_launch": nbytes}
        step_us_events = sum(v["avg_us"] * v["launches"] for k, v in kern.items() if k != "code_uniform") / max(steps_prof if not a.full else steps_timed, 1)
        return dict(t_enc=t_enc, t_dec=t_dec, ok=ok, steps_timed=steps_timed, bytes_timed=bytes_timed, container=container, enc_MBps=enc_MBps,
                    dec_MBps=dec_MBps, kern=kern, roofline=roofline, update_roofline=update_roofline, step_us_events=step_us_events)

    r = measure(mode)
    t_enc, t_dec, ok, steps_timed, bytes_timed, container = r["t_enc"], r["t_dec"], r["ok"], r["steps_timed"], r["bytes_timed"], r["container"]
    enc_MBps, dec_MBps, kern, roofline, step_us_events = r["enc_MBps"], r["dec_MBps"], r["kern"], r["roofline"], r["step_us_events"]
    lvl = a.ablation or 5
    fwd_flop = 2 * (2 * D * (Dc // T) + Dc * Dh + 256 * Dh + (T * 3 * D * D + Dh * Dh if lvl >= 2 else 0)
                    + (2 * Dh * dl + dl * dl if lvl >= 3 else 0) + (Dh * Dh if lvl >= 4 else 0) + (3 * De * Dh if lvl >= 5 else 0))
    other = None
    if a.mode is None and not a.full:  # default run: the inference-only variant (frozen weights) of the same steps beside the headline
        f = measure("frozen")
        other = {"update_mode": "frozen", "compress_MBps": round(f["enc_MBps"], 3), "decompress_MBps": round(f["dec_MBps"], 3),
                 "ms_per_step": round(1e3 * f["t_enc"] / f["steps_timed"], 5), "round_trip_exact": f["ok"],
                 "bits_per_byte": round(8.0 * f["container"] / n, 4),
                 "step_fraction_of_mfma_peak": round(fwd_flop * f["bytes_timed"] / f["t_enc"] / MFMA_BF16_PEAK, 4), "roofline": f["roofline"],
                 "sum_kernels_us": round(f["step_us_events"], 2)}
        ok = ok and f["ok"]

    cpu = None
    if not a.no_cpu_baseline:
        import oracle as orc
        sub = fi.slice_blob(blob, spec, Bo) if Bo != B else blob
        o = orc.Oracle(orc.make_config(Bo, T, D, H, **widths, dtype=orc.BF16 if spec["dtype"] == "bf16" else orc.F32,
                                       update_mode=orc.ONLINE_ADAM if mode == "online" else orc.FROZEN))
        o.load_weights(sub.data)
        t0 = time.perf_counter()
        oc = o.encode(osrc)
        t_o = time.perf_counter() - t0
        cpu = {"value": round(Bo * So / t_o / 1e6, 6), "unit": "MB/s", "cores": 1, "kind": "oracle",
               "sample": f"oracle compress of the first {T}+{So} bytes of the first {Bo} streams ({Bo * So} model steps, "
                         f"{t_o:.1f} s, single thread; box has {os.cpu_count()} logical CPUs)",
               "container_bytes": int(oc.size)}

    out = {
        "metric": "compress MB/s (input bytes) at B streams on 1 MI355X",
        "value": round(enc_MBps, 3), "unit": "MB/s", "n_gpus": 1, "steps": int(steps_timed), "warmup": int(W),
        "ms_per_step": round(1e3 * t_enc / steps_timed, 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": spec["dtype"], "data": "synthetic",
        "config": {"workload": f"cfg{a.config}: {spec['nbytes'] >> 20} MiB {spec['source']} source, B={B} streams, T={T}, D={D}, "
                               f"D_cache={Dc}, D_e={De}, d_low=64, {spec['dtype']} operands / fp32 accumulate, random-init N(0,0.02); "
                               + ("whole job" if a.full else f"timed on steps [{first},{first + K}) of every stream"),
                   "update_mode": mode, "B": B, "bytes_timed": int(bytes_timed), "ablation_level": a.ablation or 5},
        "decompress_MBps": round(dec_MBps, 3), "decompress_ms_per_step": round(1e3 * t_dec / steps_timed, 5),
        "total_MBps": round(2 * bytes_timed / (t_enc + t_dec) / 1e6, 3),
        "round_trip_exact": ok, "bits_per_byte": round(8.0 * container / n, 4),
        "fwd_flop_per_byte": fwd_flop,
        "step_fraction_of_mfma_peak": round(fwd_flop * bytes_timed / t_enc / MFMA_BF16_PEAK, 4) if mode == "frozen" else None,
        "roofline": roofline, "update_roofline": r["update_roofline"], "cpu_baseline": cpu, "frozen_weights": other,
        "kernels_us": {k: round(v["avg_us"], 2) for k, v in kern.items()}, "sum_kernels_us": round(step_us_events, 2),
    }
    print(json.dumps(out))
    if not ok:
        sys.exit(1)


if __name__ == "__main__":
    main()
