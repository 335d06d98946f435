"""Benchmark of the encrypted-BNN hot path on one MI355X.

A step of the headline workload is one encrypted fully connected layer 784 -> 512 (benchmark
configuration 3): host lowering of the layer to its gate circuit, depth-sorted batching, and every
gate's blind rotation and key switch on the GPU, with keys and input ciphertexts already resident
in HBM.  The headline value is bootstrapped gates per second over the timed steps; ms_per_step is
the layer latency (mean; median and minimum over the steps are reported beside it).  The line also
carries the roofline of the dominant kernel (blind rotation, measured with HIP events on the stream
it runs on, against the published FP64 vector peak and against an FMA loop timed on this device),
the key switch's rates, and the CPU oracle timed on a bounded sample of the same gate stream.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-cpu]
                  [--workload cfg3|cfg1|cfg2|cfg4|cfg5|flat] [--flat-count N]
                  [--comparator folded|mux|sort] [--plus-one] [--share] [--copy-calibration-mib M]

Other workloads, not the headline: cfg1 (16 gates as two calls: a latency point), cfg2 (one
256-input neuron), cfg4 (3x3 convolution 16 -> 32 channels on 28x28, one call), cfg5 (sparsified MLP
784-256-256-10, three calls), flat (one tfhe_gate_batch of N NAND gates), and whole networks in the
shapes of the paper's own models (Sec. 5.2) on synthetic weights, a step being one encrypted
inference through every layer:
  --workload cancer | diabetes | faces [--faces-channels C] [--faces-layers L]
  (C = 32 is the paper's width; L limits the run to the first L layers)
"""
import argparse
import json
import os
import statistics
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# Algorithmic double-precision work of one bootstrapped gate on this path (n = 500 steps):
# per step 8 complex 512-point FFTs at the conventional 5 N log2 N flops, 8 x 512 complex
# twist / untwist multiplications (6 flops), 16 x 512 complex multiply-accumulates (8 flops).
FLOPS_PER_STEP = 8 * 5 * 512 * 9 + 8 * 512 * 6 + 16 * 512 * 8
FP64_VECTOR_PEAK_TFLOPS = 78.6
HBM_PEAK_GBPS = 8000.0
INT8_MATRIX_PEAK_POPS = 5.0
# Key switch of one gate: 1,024 mask words x 8 base-4 digits, three of four digit values select a
# key row of 501 words to subtract: 6,144 x 501 word subtractions is the method's own work; the
# matrix-core kernel runs it as a dense one-hot x byte-plane contraction of 2 x 32,768 x 512 x 4
# int8 operations per gate.
KS_ALGORITHMIC_OPS = 1024 * 8 * 3 // 4 * 501
KS_DENSE_OPS = 2 * 32768 * 512 * 4


def progress(msg):
    """A line on stderr when a part of the run has ended (stdout carries the one JSON line only)."""
    sys.stderr.write("[bench] " + msg + "\n")
    sys.stderr.flush()


def plain_dense(x, W, T):
    """Popcount of agreeing (input, weight) pairs per unit; thresholded when T is given."""
    xs = 2 * x.astype(np.int64) - 1
    S = ((W.astype(np.int64) * xs[None, :]) > 0).sum(axis=1)
    return S if T is None else (S >= T).astype(np.uint8)


def plain_conv(x, K, T, stride, pad):
    """Same per output pixel; a tap outside the image reads the bit 0."""
    xs = np.pad(2 * x.astype(np.int64) - 1, ((0, 0), (pad, pad), (pad, pad)), constant_values=-1)
    win = np.lib.stride_tricks.sliding_window_view(xs, K.shape[2:], axis=(1, 2))[:, ::stride, ::stride]
    S = np.einsum("chwyx,ocyx->ohw", (win > 0).astype(np.int64), (K > 0).astype(np.int64)) + \
        np.einsum("chwyx,ocyx->ohw", (win < 0).astype(np.int64), (K < 0).astype(np.int64))
    return (S >= T[:, None, None]).astype(np.uint8)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="cfg3",
                    choices=["cfg3", "cfg1", "cfg2", "cfg4", "cfg5", "flat", "cancer", "diabetes", "faces"])
    ap.add_argument("--faces-channels", type=int, default=2,
                    help="output channels of the first four convolutions of --workload faces")
    ap.add_argument("--faces-layers", type=int, default=6, help="run only the first L layers of --workload faces")
    ap.add_argument("--flat-count", type=int, default=65536)
    ap.add_argument("--comparator", default="folded", choices=["folded", "mux", "sort"],
                    help="threshold circuit: AND/OR chain folded by the plaintext bits (default) or "
                         "Algorithm 1 as printed, one MUX gate per popcount bit; 'sort' replaces tree and "
                         "comparator by the bitonic sorting network")
    ap.add_argument("--plus-one", action="store_true",
                    help="lower the layer with the '+1' trick (half-size trees on one shared input popcount)")
    ap.add_argument("--share", action="store_true",
                    help="emit identical gates of different units once (structural sharing)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--cpu-gates", type=int, default=2048, help="gates in the oracle sample")
    ap.add_argument("--copy-calibration-mib", type=int, default=0,
                    help="after the timed steps, run one plain device-to-device copy of this size "
                         "(a known-traffic kernel to scale rocprofv3's FETCH_SIZE / WRITE_SIZE by)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only; --gpus must be 1 "
                 "(units of a layer would be partitioned across GPUs with one all-gather of the "
                 "output ciphertexts per layer; that is not built)")

    import torch
    import paper_1806_03461_amd as T
    import workloads

    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    torch.cuda.set_device(0)
    P = T.default_params()
    sk, ck = T.tfhe_keygen(P, workloads.KEY_SEED)
    T.tfhe_cloud_key_upload(ck)
    progress("keys generated and uploaded")
    words = P.n + 1
    flags = {"folded": T.LOWER_DEFAULT, "mux": T.LOWER_MUX_COMPARATOR,
             "sort": T.LOWER_SORTING_NETWORK}[args.comparator]
    flags |= (T.LOWER_PLUS_ONE if args.plus_one else 0) | (T.LOWER_SHARE_GATES if args.share else 0)
    options = "".join(t for t, on in ((", Algorithm-1 MUX comparator", args.comparator == "mux"),
                                      (", sorting network", args.comparator == "sort"),
                                      (", '+1' trick", args.plus_one), (", shared gates", args.share)) if on)

    def count_gates(g):
        # a multiplexer is two records (two blind rotations) but one gate
        return int((g["op"] != T.MUX_ELSE).sum())

    # ---- the workload: `layers` is a list of ("dense" | "conv", spec); `plan` the device calls ----
    flat = None
    cfg1 = None
    if args.workload == "flat":
        rng = np.random.default_rng(0)
        cnt = args.flat_count
        a = rng.integers(0, 2, cnt).astype(np.uint8)
        b = rng.integers(0, 2, cnt).astype(np.uint8)
        flat = (a, b, T.to_device(T.tfhe_encrypt(sk, 1, a)), T.to_device(T.tfhe_encrypt(sk, 2, b)))
        out = torch.empty_like(flat[2])
        name, gates_per_step = f"flat: {cnt} independent NAND gates", cnt

        def step():
            T.tfhe_gate_batch(ck, "NAND", flat[2], flat[3], out, cnt)
    elif args.workload == "cfg1":
        c = workloads.cfg1()
        da = T.to_device(T.tfhe_encrypt(sk, c["enc_seed"], c["a"]))
        db = T.to_device(T.tfhe_encrypt(sk, c["enc_seed"] + 1, c["b"]))
        out = torch.empty_like(da)
        cfg1 = c
        name, gates_per_step = "cfg1: 16 independent gates (8 NAND, 8 XNOR) as two calls", 16

        def step():
            T.tfhe_gate_batch(ck, "NAND", da[:8], db[:8], out[:8], 8)
            T.tfhe_gate_batch(ck, "XNOR", da[8:], db[8:], out[8:], 8)
    else:
        if args.workload == "cfg2":
            c = workloads.cfg2()
            net = {"x": c["x"], "enc_seed": c["enc_seed"], "out_bits": 0}
            layers = [("dense", {"W": c["W"], "T": c["T"]})]
            name = "cfg2: one encrypted neuron, 256 inputs"
        elif args.workload == "cfg3":
            c = workloads.cfg3()
            net = {"x": c["x"], "enc_seed": c["enc_seed"], "out_bits": 0}
            layers = [("dense", {"W": c["W"], "T": c["T"]})]
            name = "cfg3: encrypted FC 784->512, +-1 weights, thresholds in [300,484]"
        elif args.workload == "cfg4":
            c = workloads.cfg4()
            net = {"x": c["x"], "enc_seed": c["enc_seed"], "out_bits": 0}
            layers = [("conv", {"K": c["K"], "T": c["T"], "stride": 1, "pad": 1})]
            name = "cfg4: encrypted 3x3 convolution, 16->32 channels on 28x28, pad 1, one call"
        elif args.workload == "cfg5":
            net = workloads.cfg5()
            layers = [("dense", l) for l in net["layers"]]
            name = "cfg5: sparsified encrypted MLP 784-256-256-10, 50 % zero weights, 10-bit scores"
        elif args.workload == "faces":
            net = workloads.paper_faces(channels=args.faces_channels)
            layers = ([("conv", l) for l in net["convs"]] + [("dense", net["dense"])])[:args.faces_layers]
            name = (f"faces-shaped network: 5 convolutions 10x10 on 50x50, {args.faces_channels} channels "
                    f"(paper: 32), then FC 25->1" + (f"; first {len(layers)} layers only" if len(layers) < 6 else ""))
        else:
            net = workloads.paper_cancer() if args.workload == "cancer" else workloads.paper_diabetes()
            layers = [("dense", l) for l in net["layers"]]
            name = {"cancer": "cancer-shaped network: FC 90->1",
                    "diabetes": "diabetes-shaped network: FC 1704->10, sign, FC 10->3"}[args.workload]
        name += options
        x = T.to_device(T.tfhe_encrypt(sk, net["enc_seed"], net["x"].reshape(-1)))
        plan, shape, plain, gates_per_step, gates_host = [], net["x"].shape, net["x"], 0, None
        for li, (kind, l) in enumerate(layers):
            scores = l["T"] is None
            if kind == "conv":
                C_, H, Wd = shape
                g, _, _ = T.bnn_conv_lower_opts(C_, H, Wd, l["K"], l["T"], l["stride"], l["pad"], flags)
                plain = plain_conv(plain, l["K"], l["T"], l["stride"], l["pad"])
                buf = torch.empty((plain.size, words), dtype=torch.int32, device="cuda")
                plan.append(("conv", (C_, H, Wd, l["K"], l["T"], l["stride"], l["pad"]), buf))
            else:
                p, d = l["W"].shape
                ob = net["out_bits"] if scores else 0
                g, _, _ = T.bnn_dense_lower_opts(d, l["W"], l["T"], p, ob, flags)
                plain = plain_dense(plain.reshape(-1), l["W"], l["T"])
                buf = torch.empty((p * (ob if scores else 1), words), dtype=torch.int32, device="cuda")
                plan.append(("dense", (d, l["W"], l["T"], p, ob), buf))
            shape = plain.shape
            gates_per_step += count_gates(g)
            if li == 0:
                gates_host, d_first = g, int(net["x"].size)
            del g
        out = plan[-1][2]
        last_is_scores = layers[-1][1]["T"] is None

        def step():
            h = x
            for kind, a_, buf in plan:
                if kind == "conv":
                    T.bnn_conv_encrypted_opts(ck, h, a_[0], a_[1], a_[2], a_[3], a_[4], a_[5], a_[6], buf, flags)
                else:
                    T.bnn_dense_encrypted_opts(ck, h, a_[0], a_[1], a_[2], a_[3], buf, a_[4], flags)
                h = buf

    # ---- warm-up, then exactly --steps timed steps between two synchronisations ----
    for k in range(args.warmup):
        step()
        torch.cuda.synchronize()
        progress(f"warm-up step {k + 1} of {args.warmup} done")
    torch.cuda.synchronize()
    T.tfhe_profile_enable(ck, True)
    T.tfhe_profile_read(ck, reset=True)
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    t0 = time.perf_counter()
    marks[0].record()
    done = 0
    for k in range(args.steps):
        step()
        marks[k + 1].record()       # on the stream the calls enqueue on: when this step's last kernel ends
        while done < k and marks[done + 1].query():      # non-blocking: steps whose last kernel has ended
            done += 1
            progress(f"timed step {done} of {args.steps} done")
    while done + 1 < args.steps:    # the host only waits from here on; one line as each step ends
        marks[done + 1].synchronize()
        done += 1
        progress(f"timed step {done} of {args.steps} done")
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    progress(f"timed step {args.steps} of {args.steps} done")
    prof = T.tfhe_profile_read(ck, reset=True)
    T.tfhe_profile_enable(ck, False)
    per_step_ms = [marks[k].elapsed_time(marks[k + 1]) for k in range(args.steps)]
    layer_stats = T.tfhe_last_layer_stats(ck) if flat is None and cfg1 is None else None

    if args.copy_calibration_mib:
        src = torch.ones(args.copy_calibration_mib << 18, dtype=torch.int32, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    elapsed = t1 - t0
    total_gates = gates_per_step * args.steps
    value = total_gates / elapsed

    # ---- correctness of what was timed: decrypt and compare with the plain layer / truth table ----
    got = T.tfhe_decrypt(sk, T.to_host(out))
    if flat is not None:
        expect = 1 - (flat[0] & flat[1])
    elif cfg1 is not None:
        expect = np.concatenate([1 - (cfg1["a"][:8] & cfg1["b"][:8]), 1 - (cfg1["a"][8:] ^ cfg1["b"][8:])])
    else:
        expect = plain.reshape(-1)
        if last_is_scores:      # the last layer emits its popcounts, least significant bit first
            ob = net["out_bits"]
            got = (got.reshape(-1, ob).astype(np.int64) << np.arange(ob)).sum(axis=1)
    mismatches = int((got != expect).sum())

    # ---- roofline of the dominant kernel: algorithmic flops of the gates of one launch over the
    # average launch duration, from HIP events recorded around every launch on the call's stream ----
    br_launches = max(1, prof["blind_rotate_launches"])
    br_avg_ms = prof["blind_rotate_ms"] / br_launches
    gates_per_launch = prof["gates"] / br_launches          # blind rotations per launch
    flops_per_gate = FLOPS_PER_STEP * P.n
    achieved = flops_per_gate * gates_per_launch / (br_avg_ms * 1e-3) / 1e12 if br_avg_ms > 0 else 0.0
    measured_peak = T.tfhe_measure_fp64_peak(ck)
    # HBM bytes per launch of that kernel, from the committed rocprofv3 counter summary (if one
    # exists for this workload); the counters cannot be read from inside the process
    traffic, hbm = None, None
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(tpath):
        entry = json.load(open(tpath)).get(args.workload, {})
        traffic = entry.get("blind_rotate_bytes_per_launch")
        if traffic and entry.get("gates_per_launch") and br_avg_ms > 0:
            # the counters were read on another run: scale to this run's launch size
            scaled = traffic * gates_per_launch / entry["gates_per_launch"]
            gbps = scaled / (br_avg_ms * 1e-3) / 1e9
            hbm = {"achieved": round(gbps, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                   "frac": round(gbps / HBM_PEAK_GBPS, 4), "bytes_per_gate": round(traffic / entry["gates_per_launch"]),
                   "algorithmic_bytes_per_gate": 2 * 4 * words + 4 * (P.N + 1),
                   "source": entry.get("source")}
    roofline = {"bound": "alu", "achieved": round(achieved, 3), "peak": FP64_VECTOR_PEAK_TFLOPS,
                "unit": "TFLOP/s", "frac": round(achieved / FP64_VECTOR_PEAK_TFLOPS, 4),
                "traffic": traffic, "kernel": "blind_rotate_kernel",
                "avg_launch_ms": round(br_avg_ms, 4), "gates_per_launch": round(gates_per_launch, 1),
                "flops_per_gate": flops_per_gate,
                "peak_measured": round(measured_peak, 2),
                "frac_of_measured": round(achieved / measured_peak, 4) if measured_peak > 0 else None,
                "hbm": hbm,
                "kernel_ms": {"blind_rotate": round(prof["blind_rotate_ms"], 2),
                              "key_switch": round(prof["key_switch_ms"], 2)}}
    ks_launches = max(1, prof["key_switch_launches"])
    ks_avg_ms = prof["key_switch_ms"] / ks_launches
    key_switch = None
    if ks_avg_ms > 0:
        per_s = prof["gates"] / ks_launches / (ks_avg_ms * 1e-3)
        key_switch = {"kernel": "key_switch_mfma_kernel", "avg_launch_ms": round(ks_avg_ms, 4),
                      "algorithmic_ops_per_gate": KS_ALGORITHMIC_OPS,
                      "algorithmic_Tops": round(per_s * KS_ALGORITHMIC_OPS / 1e12, 3),
                      "dense_equivalent_Pops": round(per_s * KS_DENSE_OPS / 1e15, 3),
                      "dense_equivalent_frac_of_int8_peak": round(per_s * KS_DENSE_OPS / 1e15 / INT8_MATRIX_PEAK_POPS, 4)}

    # ---- the CPU oracle on a bounded sample of the same gate stream ----
    cpu = None
    if not args.no_cpu:
        from oracle import oracle as orc
        keys = orc.Keys(orc.default_params(), workloads.KEY_SEED)
        threads = min(16, os.cpu_count() or 1)
        ng = args.cpu_gates
        if flat is None and cfg1 is None:
            # gates of the (first) layer's circuit that read only inputs: the first ng of them, their
            # outputs renumbered to a compact wire array
            d = d_first
            nin = d + 2
            first_level = np.flatnonzero((np.maximum(gates_host["in0"], gates_host["in1"]) < nin) &
                                         (gates_host["op"] < T.MUX))[:ng]
            ng = len(first_level)
            sample = np.array(gates_host[first_level], dtype=orc.GATE_DTYPE)
            sample["out"] = nin + np.arange(ng)
            wires = np.zeros((nin + ng, words), np.uint32)
            wires[:d] = T.to_host(x)
            wires[d], wires[d + 1] = keys.trivial(0), keys.trivial(1)
            what = f"{ng} first-level gates of the {args.workload} gate stream"
        else:
            ha, hb = (T.to_host(flat[2]), T.to_host(flat[3])) if flat is not None else (T.to_host(da), T.to_host(db))
            ng = min(ng, len(ha))
            sample = np.array([(0 if (flat is not None or i < 8) else 5, 0, 0, 0, i, ng + i, 2 * ng + i) for i in range(ng)],
                              dtype=orc.GATE_DTYPE)
            wires = np.zeros((3 * ng, words), np.uint32)
            wires[:ng], wires[ng:2 * ng] = ha[:ng], hb[:ng]
            what = f"first {ng} gates of the {args.workload} batch"
        progress(f"CPU oracle: {what} on {threads} threads")
        t0 = time.perf_counter()
        keys.gate_batch(sample, wires, threads)
        dt = time.perf_counter() - t0
        progress(f"CPU oracle: done in {dt:.1f} s")
        # one thread on the 16 gates of configuration 1
        c1 = workloads.cfg1()
        ca, cb = keys.encrypt(c1["a"], c1["enc_seed"]), keys.encrypt(c1["b"], c1["enc_seed"] + 1)
        w1 = np.zeros((48, words), np.uint32)
        w1[:16], w1[16:32] = ca, cb
        s1 = np.array([(0 if i < 8 else 5, 0, 0, 0, i, 16 + i, 32 + i) for i in range(16)], dtype=orc.GATE_DTYPE)
        t0 = time.perf_counter()
        keys.gate_batch(s1, w1, 1)
        dt1 = time.perf_counter() - t0
        rate = ng / dt
        cpu = {"value": round(rate, 2), "unit": "gates/s", "cores": threads, "kind": "oracle",
               "sample": f"{what}, {dt:.1f} s",
               "single_thread": {"value": round(16 / dt1, 2), "unit": "gates/s", "cores": 1,
                                 "sample": f"the 16 gates of cfg1, {dt1:.1f} s"},
               "extrapolated_s_per_step": round(gates_per_step / rate, 1),
               "extrapolation": f"gates of one step / the {threads}-thread rate above: an estimate, not a measurement"}

    line = {"metric": "bootstrapped gates/sec (n=500,N=1024) on 1 MI355X; encrypted BNN layer latency",
            "value": round(value, 1), "unit": "gates/s", "n_gpus": 1, "steps": args.steps,
            "warmup": args.warmup, "ms_per_step": round(elapsed / args.steps * 1e3, 3),
            "ms_per_step_median": round(statistics.median(per_step_ms), 3),
            "ms_per_step_min": round(min(per_step_ms), 3),
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f64",
            "data": "synthetic", "config": {"workload": name, "gates_per_step": gates_per_step,
                                            "decrypt_mismatches": mismatches,
                                            "wire_pool": layer_stats},
            "roofline": roofline, "key_switch": key_switch, "cpu_baseline": cpu}
    print(json.dumps(line))
    if mismatches:
        sys.exit(f"bench.py: {mismatches} outputs decrypt to the wrong bit")


if __name__ == "__main__":
    main()
