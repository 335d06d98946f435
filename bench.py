"""Benchmark of the encrypted-BNN hot path on one MI355X.

A step is one encrypted fully connected layer 784 -> 512 (benchmark configuration 3): host
lowering of the layer to its gate circuit, depth-sorted batching, and every gate's blind
rotation and key switch on the GPU, with keys and input ciphertexts already resident in HBM.
The headline value is bootstrapped gates per second over the timed steps; ms_per_step is the
layer latency.  The line also carries the roofline of the dominant kernel (blind rotation,
measured with HIP events on the stream it runs on) and the CPU oracle timed on a bounded sample
of the same gate stream.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg3|cfg2|flat] [--no-cpu]
                  [--comparator folded|mux|sort] [--plus-one] [--share] [--copy-calibration-mib M]

Further workloads, not the headline: whole networks in the shapes of the paper's own models
(Sec. 5.2) on synthetic weights, a step being one encrypted inference through every layer:
  --workload cancer | diabetes | faces [--faces-channels C]   (C = 32 is the paper's width)
"""
import argparse
import json
import os
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


def plain_dense(x, W, T):
    """Popcount of agreeing (input, weight) pairs per unit; thresholded when T is given."""
    xs = 2 * x.astype(np.int64) - 1
    S = ((W.astype(np.int64) * xs[None, :]) > 0).sum(axis=1)
    return S if T is None else (S >= T).astype(np.uint8)


def plain_conv(x, K, T, stride, pad):
    """Same per output pixel; a tap outside the image reads the bit 0."""
    xs = np.pad(2 * x.astype(np.int64) - 1, ((0, 0), (pad, pad), (pad, pad)), constant_values=-1)
    win = np.lib.stride_tricks.sliding_window_view(xs, K.shape[2:], axis=(1, 2))[:, ::stride, ::stride]
    agree = (win[None] * K.astype(np.int64)[:, :, None, None] > 0)       # [O][C][Ho][Wo][kh][kw]
    S = agree.sum(axis=(1, 4, 5))
    return (S >= T[:, None, None]).astype(np.uint8)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="cfg3", choices=["cfg3", "cfg2", "flat", "cancer", "diabetes", "faces"])
    ap.add_argument("--faces-channels", type=int, default=2,
                    help="output channels of the first four convolutions of --workload faces")
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
    words = P.n + 1

    if args.workload == "cfg3":
        c = workloads.cfg3()
        name = "cfg3: encrypted FC 784->512, +-1 weights, thresholds in [300,484]"
    elif args.workload == "cfg2":
        c = workloads.cfg2()
        name = "cfg2: one encrypted neuron, 256 inputs"
    else:
        c = None
        name = f"flat: {args.flat_count} independent NAND gates"

    net = None
    if args.workload in ("cancer", "diabetes", "faces"):
        flags = {"folded": T.LOWER_DEFAULT, "mux": T.LOWER_MUX_COMPARATOR,
                 "sort": T.LOWER_SORTING_NETWORK}[args.comparator]
        flags |= (T.LOWER_PLUS_ONE if args.plus_one else 0) | (T.LOWER_SHARE_GATES if args.share else 0)
        if args.workload == "faces":
            net = workloads.paper_faces(channels=args.faces_channels)
            name = (f"faces-shaped network: 5 convolutions 10x10 on 50x50, {args.faces_channels} channels "
                    f"(paper: 32), then FC 25->1")
            layers = [("conv", l) for l in net["convs"]] + [("dense", net["dense"])]
        else:
            net = workloads.paper_cancer() if args.workload == "cancer" else workloads.paper_diabetes()
            name = {"cancer": "cancer-shaped network: FC 90->1",
                    "diabetes": "diabetes-shaped network: FC 1704->10, sign, FC 10->3"}[args.workload]
            layers = [("dense", l) for l in net["layers"]]
        name += "".join(t for t, on in ((", Algorithm-1 MUX comparator", args.comparator == "mux"),
                                        (", sorting network", args.comparator == "sort"),
                                        (", '+1' trick", args.plus_one), (", shared gates", args.share)) if on)
        x = T.to_device(T.tfhe_encrypt(sk, net["enc_seed"], net["x"].reshape(-1)))
        plan, shape, plain, gates_per_step, gates_host = [], net["x"].shape, net["x"], 0, None
        for li, (kind, l) in enumerate(layers):
            last = l["T"] is None
            if kind == "conv":
                C_, H, Wd = shape
                O, _, kh, kw = l["K"].shape
                g, _, _ = T.bnn_conv_lower_opts(C_, H, Wd, l["K"], l["T"], l["stride"], l["pad"], flags)
                plain = plain_conv(plain, l["K"], l["T"], l["stride"], l["pad"])
                shape = plain.shape
                buf = torch.empty((plain.size, words), dtype=torch.int32, device="cuda")
                plan.append(("conv", (C_, H, Wd, l["K"], l["T"], l["stride"], l["pad"]), buf))
            else:
                p, d = l["W"].shape
                ob = net["out_bits"] if last else 0
                g, _, _ = T.bnn_dense_lower_opts(d, l["W"], l["T"], p, ob, flags)
                plain = plain_dense(plain.reshape(-1), l["W"], l["T"])
                shape = plain.shape
                buf = torch.empty((p * (ob if last else 1), words), dtype=torch.int32, device="cuda")
                plan.append(("dense", (d, l["W"], l["T"], p, ob), buf))
            gates_per_step += int((g["op"] != T.MUX_ELSE).sum())
            if li == 0:
                gates_host, d_first = g, int(net["x"].size)
        out = plan[-1][2]

        def step():
            h = x
            for kind, a, buf in plan:
                if kind == "conv":
                    T.bnn_conv_encrypted_opts(ck, h, a[0], a[1], a[2], a[3], a[4], a[5], a[6], buf, flags)
                else:
                    T.bnn_dense_encrypted_opts(ck, h, a[0], a[1], a[2], a[3], buf, a[4], flags)
                h = buf
    elif c is not None:
        p, d = c["W"].shape
        x = T.to_device(T.tfhe_encrypt(sk, c["enc_seed"], c["x"]))
        out = torch.empty((p, words), dtype=torch.int32, device="cuda")
        flags = {"folded": T.LOWER_DEFAULT, "mux": T.LOWER_MUX_COMPARATOR,
                 "sort": T.LOWER_SORTING_NETWORK}[args.comparator]
        if args.plus_one:
            flags |= T.LOWER_PLUS_ONE
            name += ", '+1' trick"
        if args.share:
            flags |= T.LOWER_SHARE_GATES
            name += ", shared gates"
        gates_host, _, _ = T.bnn_dense_lower_opts(d, c["W"], c["T"], p, 0, flags)
        # a multiplexer is two records (two blind rotations) but one gate
        gates_per_step = int((gates_host["op"] != T.MUX_ELSE).sum())
        if args.comparator == "mux":
            name += ", Algorithm-1 MUX comparator"
        if args.comparator == "sort":
            name += ", sorting network"

        def step():
            T.bnn_dense_encrypted_opts(ck, x, d, c["W"], c["T"], p, out, 0, flags)
    else:
        rng = np.random.default_rng(0)
        cnt = args.flat_count
        a = rng.integers(0, 2, cnt).astype(np.uint8)
        b = rng.integers(0, 2, cnt).astype(np.uint8)
        da, db = T.to_device(T.tfhe_encrypt(sk, 1, a)), T.to_device(T.tfhe_encrypt(sk, 2, b))
        out = torch.empty_like(da)
        gates_per_step = cnt

        def step():
            T.tfhe_gate_batch(ck, "NAND", da, db, out, cnt)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    T.tfhe_profile_enable(ck, True)
    T.tfhe_profile_read(ck, reset=True)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    prof = T.tfhe_profile_read(ck, reset=True)
    T.tfhe_profile_enable(ck, False)

    if args.copy_calibration_mib:
        src = torch.ones(args.copy_calibration_mib << 18, dtype=torch.int32, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    elapsed = t1 - t0
    total_gates = gates_per_step * args.steps
    value = total_gates / elapsed

    # correctness of what was timed: decrypt and compare with the plain layer / truth table
    got = T.tfhe_decrypt(sk, T.to_host(out))
    if net is not None:
        # the last layer emits its popcounts, least significant bit first
        ob = net["out_bits"]
        got = (got.reshape(-1, ob).astype(np.int64) << np.arange(ob)).sum(axis=1)
        expect = plain.reshape(-1)
    elif c is not None:
        xs = 2 * c["x"].astype(np.int64) - 1
        S = ((c["W"].astype(np.int64) * xs[None, :]) > 0).sum(axis=1)
        expect = (S >= c["T"]).astype(np.uint8)
    else:
        expect = 1 - (a & b)
    mismatches = int((got != expect).sum())

    # roofline of the dominant kernel: algorithmic flops of the gates of one launch over the
    # average launch duration, from HIP events recorded around every launch on the call's stream
    br_launches = max(1, prof["blind_rotate_launches"])
    br_avg_ms = prof["blind_rotate_ms"] / br_launches
    gates_per_launch = prof["gates"] / br_launches          # blind rotations per launch
    flops_per_gate = FLOPS_PER_STEP * P.n
    achieved = flops_per_gate * gates_per_launch / (br_avg_ms * 1e-3) / 1e12 if br_avg_ms > 0 else 0.0
    # HBM bytes per launch of that kernel, from the committed rocprofv3 counter summary (if one
    # exists for this workload); the counters cannot be read from inside the process
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(tpath):
        traffic = json.load(open(tpath)).get(args.workload, {}).get("blind_rotate_bytes_per_launch")
    roofline = {"bound": "alu", "achieved": round(achieved, 3), "peak": FP64_VECTOR_PEAK_TFLOPS,
                "unit": "TFLOP/s", "frac": round(achieved / FP64_VECTOR_PEAK_TFLOPS, 4),
                "traffic": traffic, "kernel": "blind_rotate_kernel",
                "avg_launch_ms": round(br_avg_ms, 4), "gates_per_launch": round(gates_per_launch, 1),
                "flops_per_gate": flops_per_gate,
                "kernel_ms": {"blind_rotate": round(prof["blind_rotate_ms"], 2),
                              "key_switch": round(prof["key_switch_ms"], 2)}}

    cpu = None
    if not args.no_cpu:
        from oracle import oracle as orc
        keys = orc.Keys(orc.default_params(), workloads.KEY_SEED)
        threads = min(16, os.cpu_count() or 1)
        ng = args.cpu_gates
        if c is not None or net is not None:
            # gates of the (first) layer's circuit that read only inputs: the first ng of them, their
            # outputs renumbered to a compact wire array
            if net is not None:
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
            ng = min(ng, cnt)
            sample = np.array([(0, 0, 0, 0, i, ng + i, 2 * ng + i) for i in range(ng)], dtype=orc.GATE_DTYPE)
            wires = np.zeros((3 * ng, words), np.uint32)
            wires[:ng], wires[ng:2 * ng] = T.to_host(da)[:ng], T.to_host(db)[:ng]
            what = f"first {ng} gates of the flat batch"
        t0 = time.perf_counter()
        keys.gate_batch(sample, wires, threads)
        dt = time.perf_counter() - t0
        cpu = {"value": round(ng / dt, 2), "unit": "gates/s", "cores": threads, "kind": "oracle",
               "sample": f"{what}, {dt:.1f} s"}

    line = {"metric": "bootstrapped gates/sec (n=500,N=1024) on 1 MI355X; encrypted BNN layer latency",
            "value": round(value, 1), "unit": "gates/s", "n_gpus": 1, "steps": args.steps,
            "warmup": args.warmup, "ms_per_step": round(elapsed / args.steps * 1e3, 3),
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f64",
            "data": "synthetic", "config": {"workload": name, "gates_per_step": gates_per_step,
                                            "decrypt_mismatches": mismatches},
            "roofline": roofline, "cpu_baseline": cpu}
    print(json.dumps(line))
    if mismatches:
        sys.exit(f"bench.py: {mismatches} outputs decrypt to the wrong bit")


if __name__ == "__main__":
    main()
