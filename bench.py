#!/usr/bin/env python3
"""Benchmark of the on-line back-propagation hot path on one MI355X.

Workload (benchmark configs[3], the configuration the target is quoted on): the
784-2500-2000-1500-1000-500-10 net (11,972,510 fp32 weights), a 60,000-sample synthetic
stroke-image epoch, every image elastically + affinely deformed on the GPU right before it is
trained on, eta = 1e-3, plus a forward-only classify pass over 10,000 undeformed images (reported
separately under "classify"; `value` is the training rate).

A "step" is one pass of the whole hot path over one chunk of `--chunk` samples:
dbsn_deform_batch(chunk) and dbsn_bp_steps(chunk) (strictly sequential batch-size-1 updates
inside); the deformation of the next chunk runs on a side stream while this one trains.  Inputs (uint8 images, labels) are resident in HBM before the timed region.
Prints ONE JSON line.  Beside the headline it carries, each measured in the same run:
  other_configs   the other four nets of the benchmark's configs (config 0 without deformation);
  streaming       the same training call with the weights streamed from memory every phase instead
                  of held in registers (the benchmark net, and a net too big for the registers), and
                  the launch-per-phase mode;
  roofline.measured_stream_*   what a plain 2-reads : 1-write kernel sustains over 48 MB and 1 GB;
  cpu_baseline    the CPU oracle on one thread and on all host threads, and its deformation alone.
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

NET4 = [784, 2500, 2000, 1500, 1000, 500, 10]
# the five nets of the benchmark's configs; configs[3] is the one the metric is quoted on
CONFIG_NETS = [[784, 1000, 500, 10], [784, 1500, 1000, 500, 10], [784, 2000, 1500, 1000, 500, 10], NET4,
               [784] + [1000] * 9 + [10]]
# a net whose hidden layers (128 MB) do not fit the 58.7 MB of registers: always streamed
BIG_NET = [784, 3584, 3584, 3584, 1000, 10]
HBM_PEAK_GBS = 8000.0   # MI355X published HBM3E peak
PMC_PROFILE = os.path.join(ROOT, "profiles", "k_bp_dataflow_net4_pmc.txt")


def n_weights(sizes):
    return sum((sizes[i] + 1) * sizes[i + 1] for i in range(len(sizes) - 1))


def recorded_traffic():
    """Memory-side bytes of one persistent-kernel launch (1000 samples of configs[3]) as recorded in
    profiles/: FETCH_SIZE + WRITE_SIZE from two rocprofv3 --pmc runs of this script (counters cannot be
    read from inside the process).  -> (bytes or None, the tree the figure was taken at or None)."""
    try:
        text = open(PMC_PROFILE).read()
    except OSError:
        return None, None
    m = re.search(r"^traffic_bytes_per_launch\s*=\s*([0-9.eE+]+)", text, re.M)
    t = re.search(r"^tree\s*=\s*(\S+)", text, re.M)
    return (float(m.group(1)) if m else None), (t.group(1) if t else None)


def cpu_baseline(sizes, img, lab, eta, budget_s=8.0):
    """The oracle (fp32 mode, as it stands) on bounded samples of the same workload, on the host
    cores of this machine: deform + bp_step per sample on all threads and on one, and the deformation
    alone."""
    import numpy as np
    from oracle import Oracle
    o = Oracle()
    cores = min(o.max_threads(), 16)   # the box grants 16 host threads to a one-GPU job

    def run(threads, at, budget):
        o.set_threads(threads)
        params = o.init_params(sizes, 0)
        t0 = time.perf_counter()
        x = o.deform_batch(img[at:at + 4], 0, at, mode="f32")
        params, _ = o.bp_steps(sizes, params, x, lab[at:at + 4], np.float32(eta), "f32")
        per = (time.perf_counter() - t0) / 4
        n = int(max(200, min(len(img) - at - 4, budget / max(per, 1e-6))))
        t0 = time.perf_counter()
        x = o.deform_batch(img[at + 4:at + 4 + n], 0, at + 4, mode="f32")
        params, _ = o.bp_steps(sizes, params, x, lab[at + 4:at + 4 + n], np.float32(eta), "f32")
        return n, time.perf_counter() - t0

    n_all, dt_all = run(cores, 0, budget_s)
    n_one, dt_one = run(1, 0, budget_s)
    o.set_threads(1)
    nd = 400
    t0 = time.perf_counter()
    o.deform_batch(img[:nd], 0, 0, mode="f32")
    dt_d1 = time.perf_counter() - t0
    o.set_threads(cores)
    t0 = time.perf_counter()
    o.deform_batch(img[:4 * nd], 0, 0, mode="f32")
    dt_dall = time.perf_counter() - t0
    o.set_threads(1)
    return {"value": n_all / dt_all, "unit": "samples/s", "cores": cores, "kind": "oracle",
            "sample": "%d consecutive samples of the same workload (deform + one on-line BP step each), "
                      "oracle fp32 mode, %.1f s on %d threads" % (n_all, dt_all, cores),
            "single_thread": {"value": n_one / dt_one, "unit": "samples/s", "cores": 1,
                              "sample": "%d consecutive samples, %.1f s" % (n_one, dt_one)},
            "deform_alone": {"single_thread_images_per_s": nd / dt_d1, "all_threads_images_per_s": 4 * nd / dt_dall,
                             "cores": cores, "sample": "%d and %d images" % (nd, 4 * nd)}}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=60)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--chunk", type=int, default=1000)
    ap.add_argument("--mode", type=int, default=1, help="0: one launch per phase, 1: persistent kernel")
    ap.add_argument("--config", type=int, default=3,
                    help="which of BASELINE.json's nets the headline runs (default 3, the benchmark)")
    ap.add_argument("--net", type=str, default=None,
                    help="layer sizes a-b-...-c of the headline run instead of a config's net (context runs)")
    ap.add_argument("--variant", choices=["default", "streaming", "runtime-layout", "plain-tiles"], default="default",
                    help="persistent-kernel variant of the headline run (see dbsn_mlp_set_variant)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-classify", action="store_true")
    ap.add_argument("--no-other-configs", action="store_true")
    ap.add_argument("--no-streaming", action="store_true")
    ap.add_argument("--no-ceilings", action="store_true")
    ap.add_argument("--no-autotune", action="store_true",
                    help="skip dbsn_mlp_autotune (the one-off tuning of the persistent kernel's pauses, outside the timed region)")
    ap.add_argument("--traffic-probe", action="store_true",
                    help="also run one plain elementwise kernel that reads 256 MiB and writes 256 MiB, as the "
                         "known-size reference for scaling FETCH_SIZE / WRITE_SIZE counter readings")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (on-line back-propagation is strictly sequential over "
              "samples; nothing here uses a second GPU). Use --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_1003_0358_amd import binding, datagen

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    lib = binding.load()
    eta = 1e-3
    chunk, K, Wm = args.chunk, args.steps, args.warmup
    n_train = 60000
    img, lab = datagen.stroke_images(n_train, seed=0)
    src = torch.from_numpy(img).to(dev)
    labels = torch.from_numpy(lab).to(dev)
    xbuf = torch.empty((chunk, 784), dtype=torch.float32, device=dev)
    xbuf2 = torch.empty((chunk, 784), dtype=torch.float32, device=dev)
    main = torch.cuda.current_stream(dev)
    side = torch.cuda.Stream(dev)   # (default priority) the deformation of the next chunk
    loss = torch.zeros(chunk, dtype=torch.float32, device=dev)
    params = binding.default_deform_params()
    identity = binding.DeformParams(0.0, 0.0, 0.0, 0.0, 1, 0, 0)   # all amplitudes zero: the exact intensity map
    stream = torch.cuda.current_stream(dev).cuda_stream

    def train_run(sizes, steps, warmup, mode=1, variant="default", deform=True, autotune=True):
        """`steps` timed steps of (deform chunk +) bp_steps(chunk) on a fresh network.
        -> dict with the wall time of the timed region and the mean launch time of bp_steps (events)."""
        m = binding.Mlp(sizes, seed=0, mode=mode)
        if variant == "streaming":
            m.set_variant(stationary=False)
        elif variant == "runtime-layout":
            m.set_variant(fixed_layout=False)
        elif variant == "plain-tiles":
            m.set_variant(banded=False)
        if not deform:   # the same un-deformed chunk every step
            lib.check(lib.deform_batch(identity, src[:chunk], chunk, 0, 0, xbuf, stream))

        # the deformation of chunk i + 1 runs on a side stream while chunk i trains (two input buffers)
        bufs = [xbuf, xbuf2]
        ready = [torch.cuda.Event() for _ in range(2)]
        spent = [torch.cuda.Event() for _ in range(2)]

        def chunk_at(i):
            a = (i * chunk) % n_train
            return 0 if a + chunk > n_train else a

        def start_deform(i):
            side.wait_event(spent[i % 2])
            lib.check(lib.deform_batch(params, src[chunk_at(i):chunk_at(i) + chunk], chunk, 0, chunk_at(i), bufs[i % 2],
                                       side.cuda_stream))
            ready[i % 2].record(side)

        def step(i, ev=None):
            a = chunk_at(i) if deform else 0
            if deform:
                start_deform(i + 1)          # (every step starts one deformation and trains one chunk)
                main.wait_event(ready[i % 2])
            if ev is not None:
                ev[0].record()
            lib.check(lib.bp_steps(m.h, bufs[i % 2] if deform else xbuf, labels[a:a + chunk], chunk, eta, loss))
            if deform:
                spent[i % 2].record(main)
            if ev is not None:
                ev[1].record()

        tune_s = None
        if autotune and mode == binding.MODE_PERSISTENT:
            # one-off set-up, like the allocation above: steps with eta = 0, weights untouched
            if deform:
                lib.check(lib.deform_batch(params, src[:chunk], chunk, 0, 0, xbuf, stream))
            torch.cuda.synchronize()
            t_tune = time.perf_counter()
            m.autotune(xbuf, labels[:chunk])
            tune_s = time.perf_counter() - t_tune
        if deform:
            side.wait_stream(main)
            start_deform(0)
        for i in range(warmup):
            step(i)
        m.status()
        torch.cuda.synchronize()
        events = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
        t0 = time.perf_counter()
        for i in range(steps):
            step(warmup + i, events[i])
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        m.status()
        final_loss = float(loss.mean())
        assert np.isfinite(final_loss)
        bp_ms = [a.elapsed_time(b) for a, b in events]
        f, b = m.get_pauses()
        return {"mlp": m, "dt": dt, "bp_avg_s": sum(bp_ms) / len(bp_ms) / 1e3, "final_loss": final_loss,
                "autotune_s": tune_s, "variant": m.get_variant(), "pauses": [f.tolist(), b.tolist()]}

    def summary(sizes, r, extra=None):
        nw = n_weights(sizes)
        per = r["bp_avg_s"] / chunk
        d = {"net": "-".join(map(str, sizes)), "weights": nw, "us_per_sample": per * 1e6,
             "samples_per_s_bp_steps_alone": 1.0 / per,
             "algorithmic_GBps": 12.0 * nw / per / 1e9, "frac": 12.0 * nw / per / 1e9 / HBM_PEAK_GBS,
             "us_per_phase": per * 1e6 / (2 * (len(sizes) - 1)), "phases_per_step": 2 * (len(sizes) - 1),
             "stationary_layout_bandedpairs": list(r["variant"]), "pauses_fwd_bwd": r["pauses"]}
        if extra:
            d.update(extra)
        return d

    # ---- headline: configs[3] (or --config), persistent kernel, per-step deformation ----------------
    sizes = CONFIG_NETS[args.config] if args.net is None else [int(v) for v in args.net.split("-")]
    head = train_run(sizes, K, Wm, mode=args.mode, variant=args.variant, deform=(args.config != 0),
                     autotune=not args.no_autotune)
    m = head["mlp"]
    nw = n_weights(sizes)
    bytes_per_launch = 12.0 * nw * chunk          # 4 B forward read + 4 B backward read + 4 B write, per weight
    achieved = bytes_per_launch / head["bp_avg_s"] / 1e9
    traffic, traffic_tree = recorded_traffic()
    headline_is_recorded = (args.mode == 1 and chunk == 1000 and args.config == 3 and args.variant == "default" and
                            args.net is None)

    out = {
        "metric": "online-BP training samples/sec (batch 1) + % of weight-bandwidth roofline",
        "value": chunk * K / head["dt"],
        "unit": "samples/s",
        "n_gpus": 1,
        "steps": K,
        "warmup": Wm,
        "ms_per_step": head["dt"] / K * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {
            "workload": "%s: MLP %s (%s fp32 weights), synthetic 60,000-image stroke epoch, %s, on-line BP eta 1e-3"
                        % ("configs[%d]" % args.config if args.net is None else "custom net", "-".join(map(str, sizes)),
                           format(nw, ","),
                           "per-step elastic (sigma 6, alpha 36, 21 taps) + rotation +-7.5 deg + scaling +-15 % deformation"
                           if args.config != 0 else "no deformation"),
            "samples_per_step": chunk,
            "mode": "persistent" if args.mode == 1 else "launch-per-phase",
            "variant": args.variant,
            "stationary_layout_bandedpairs": list(head["variant"]),
            "pauses_fwd_bwd": head["pauses"],
            "autotune_s": head["autotune_s"],
        },
        "roofline": {
            "bound": "hbm",
            # algorithmic bytes (12 B per weight and sample, what a streamed step would move) over the
            # launch time: the metric's definition.  The default kernel keeps the weights in registers,
            # so its real memory-side traffic (`traffic`) is far smaller and none of it is weights.
            "achieved": achieved,
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBS,
            "frac_is": "algorithmic bytes / launch time / HBM peak",
            "traffic": traffic if headline_is_recorded else None,
            "traffic_source": ("profiles/k_bp_dataflow_net4_pmc.txt at tree %s" % traffic_tree) if headline_is_recorded else None,
            "weight_bytes_per_step_from_memory": (0.0 if (args.mode == 1 and args.variant != "streaming") else 12.0 * nw),
            "kernel": "k_bp_dataflow" if args.mode == 1 else "k_fwd/k_bwd/k_top",
            "algorithmic_bytes_per_launch": bytes_per_launch,
            "avg_launch_ms": head["bp_avg_s"] * 1e3,
            "us_per_sample": head["bp_avg_s"] / chunk * 1e6,
        },
        # the pair the measurement plan asks for: the whole step (deformation of the chunk + training) is
        # `value`; training alone, from the events around dbsn_bp_steps; the deformation of
        # the next chunk runs on a side stream while this one trains (0.1 % of the step either way)
        "bp_steps_alone_samples_per_s": chunk / head["bp_avg_s"],
        "deformation_overlapped": True,
        "final_chunk_mean_loss": head["final_loss"],
        "paper_context": "GTX 280 (2010): up to 5e9 weight updates/s, i.e. about 413 samples/s on this net "
                         "(derived from the paper's figure; different hardware, not a target)",
    }

    if not args.no_classify:
        timg, _ = datagen.stroke_images(10000, seed=1)
        tx = binding.deform_batch(torch.from_numpy(timg).to(dev), 0, 0, identity)   # un-deformed inputs
        pred = m.classify(tx)             # warm-up at full size
        torch.cuda.synchronize()
        reps = 5
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            pred = m.classify(tx)
        e1.record()
        torch.cuda.synchronize()
        ct = e0.elapsed_time(e1) * 1e-3 / reps
        # the batched forward pass is a dense contraction on the fp32 matrix cores: 2 flop per weight per sample
        tflops = 2.0 * nw * 10000 / ct / 1e12
        out["classify"] = {"samples": 10000, "samples_per_s": 10000 / ct,
                           "roofline": {"bound": "mfma", "achieved": tflops, "peak": 157.3, "unit": "TFLOP/s",
                                        "frac": tflops / 157.3, "kernel": "k_layer_batch_dma (fp32 MFMA)", "calls_timed": reps},
                           "label_histogram": torch.bincount(pred.long(), minlength=10).tolist()}
    m.close()
    del m, head

    # deformation alone
    torch.cuda.synchronize()
    big = torch.empty((n_train, 784), dtype=torch.float32, device=dev)
    lib.check(lib.deform_batch(params, src, n_train, 0, 0, big, stream))
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    lib.check(lib.deform_batch(params, src, n_train, 0, 0, big, stream))
    torch.cuda.synchronize()
    out["deform_batch_images_per_s"] = n_train / (time.perf_counter() - t1)
    del big

    # ---- the other nets of the configs (context; config 0 trains without deformation) --------------
    if not args.no_other_configs:
        others = []
        for c in (0, 1, 2, 4):
            if c == args.config:
                continue
            r = train_run(CONFIG_NETS[c], 10, 2, deform=(c != 0), autotune=not args.no_autotune)
            r["mlp"].close()
            others.append(summary(CONFIG_NETS[c], r, {"config": c, "deformation": c != 0,
                                                      "samples_per_s": chunk * 10 / r["dt"]}))
        out["other_configs"] = others

    # ---- weights streamed from memory every phase, and the launch-per-phase mode --------------------
    if not args.no_streaming:
        rows = []
        for name, net, mode, variant, steps in (("persistent kernel, weights streamed per phase", NET4, 1, "streaming", 10),
                                                ("persistent kernel, weights streamed per phase", BIG_NET, 1, "streaming", 5),
                                                ("one launch per layer phase", NET4, 0, "default", 3)):
            r = train_run(net, steps, 1, mode=mode, variant=variant, autotune=False)
            r["mlp"].close()
            rows.append(summary(net, r, {"path": name, "weight_bytes_per_step_from_memory": 12.0 * n_weights(net)}))
        out["streaming"] = rows

    # ---- what a plain 2-reads : 1-write kernel sustains (dbsn_probe_stream) -------------------------
    if not args.no_ceilings:
        ceil = {}
        for label, nbytes in (("48MB", 48 * 10 ** 6), ("1GB", 10 ** 9)):
            nf = nbytes // 16 * 4
            buf = torch.zeros(nf, dtype=torch.float32, device=dev)
            best = None
            for wgs in (256, 512, 1024, 2048, 4096, 8192):
                sink = torch.empty(4 * wgs, dtype=torch.float32, device=dev)
                sweeps = 20 if nbytes < 10 ** 8 else 4
                lib.check(lib.probe_stream(buf, nf, wgs, 2, sink, stream))
                torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                lib.check(lib.probe_stream(buf, nf, wgs, sweeps, sink, stream))
                e1.record()
                torch.cuda.synchronize()
                gbs = 12.0 * nf * sweeps / (e0.elapsed_time(e1) * 1e-3) / 1e9
                if best is None or gbs > best[0]:
                    best = (gbs, wgs)
            ceil[label] = {"GBps": best[0], "workgroups": best[1], "footprint_bytes": nf * 4}
            del buf
        out["roofline"]["measured_stream_48MB"] = ceil["48MB"]["GBps"]
        out["roofline"]["measured_stream_1GB"] = ceil["1GB"]["GBps"]
        out["roofline"]["frac_of_measured_stream_48MB"] = achieved / ceil["48MB"]["GBps"]
        out["roofline"]["frac_of_measured_stream_1GB"] = achieved / ceil["1GB"]["GBps"]
        out["ceilings"] = {"kernel": "k_probe_read + k_probe_update (2 reads : 1 write, 12 B per float and sweep)", **ceil}
        # the bare hand-over among the 256 workgroups, across the chip and inside a die (dbsn_probe_handover)
        hbuf = torch.zeros(2 * 256 * 64, dtype=torch.int64, device=dev)
        gave = torch.zeros(1, dtype=torch.int32, device=dev)
        hand = {}
        for label, within in (("across_dies", 0), ("within_die", 1)):
            lib.check(lib.probe_handover(within, 200, hbuf, gave, stream))
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            lib.check(lib.probe_handover(within, 4000, hbuf, gave, stream))
            e1.record()
            torch.cuda.synchronize()
            hand[label] = {"us_per_hand_over": e0.elapsed_time(e1) * 1e3 / 4000, "workgroups_gave_up": int(gave.item())}
        out["hand_over"] = hand
        if "streaming" in out:
            for row in out["streaming"]:
                fp = 4 * row["weights"]
                c = ceil["48MB"]["GBps"] if fp < 2 * 10 ** 8 else ceil["1GB"]["GBps"]
                row["frac_of_measured_stream"] = row["algorithmic_GBps"] / c

    if args.traffic_probe:
        a = torch.ones(64 * 2 ** 20, dtype=torch.float32, device=dev)
        b = torch.empty_like(a)
        torch.cuda.synchronize()
        torch.mul(a, 2.0, out=b)   # one elementwise kernel: 256 MiB read, 256 MiB written
        torch.cuda.synchronize()
        out["traffic_probe"] = {"kernel": "torch elementwise mul", "read_bytes": a.numel() * 4, "write_bytes": b.numel() * 4}
        del a, b

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(sizes, img, lab, eta)
        if "other_configs" in out:
            # the oracle on all threads on 200 consecutive samples of the other configs too (a second or two in all)
            from oracle import Oracle
            o = Oracle()
            cores = out["cpu_baseline"]["cores"]
            o.set_threads(cores)
            for row in out["other_configs"]:
                net = CONFIG_NETS[row["config"]]
                p = o.init_params(net, 0)
                t0 = time.perf_counter()
                x = o.deform_batch(img[:200], 0, 0, mode="f32") if row["deformation"] else \
                    o.deform_batch(img[:200], 0, 0, alpha=0.0, beta_deg=0.0, gamma_pct=0.0, mode="f32")
                o.bp_steps(net, p, x, lab[:200], np.float32(eta), "f32")
                row["cpu_oracle_samples_per_s"] = 200 / (time.perf_counter() - t0)
                row["cpu_oracle_cores"] = cores
            o.set_threads(1)

    print(json.dumps(out))


if __name__ == "__main__":
    main()
