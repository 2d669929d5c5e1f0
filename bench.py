"""Benchmark of the scheme-scoring hot path on one MI355X.

One step = one aiq_eval_schemes call over the whole workload: scheme upload, weight
quantization of every (layer, bit-width) the schemes use, the all-FP32 base pass, the
scheme-batched forward of every layer, classifier head and agreement count.  Inputs
are resident in HBM before the timed region.  Prints one JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_MFMA_F32_TFLOPS = 157.3  # MI355X dense fp32 matrix peak
PEAK_HBM_GBS = 8000.0
PEAK_MFMA_BF16_TFLOPS = 2500.0  # MI355X dense bf16 matrix peak

# HBM bytes per launch of a kernel class from rocprofv3 counters (FETCH_SIZE x 2.000 and
# WRITE_SIZE x 1.000, the factors a plain copy of known size gives; profiles/ has the runs): every
# counter run taken is listed, `traffic` reports their mean and `traffic_min_max` their range.
# Valid only for the kernel source it was measured on: keyed by the sha256 of that source (of the
# sections of it that hold the kernel, where the file holds several).
TRAFFIC = {
    ("resnet20_greedy_step_n1024_s40", "resnet_fused"): {
        "kernel_source": "paper_2512_14090_amd/csrc/aiq_fused.hip",
        "sha256": "56d1c2d483b20bd9b6d21cb09afec8e50edc7f4cc62b2032687c978bf27bee5e",
        # nine counter runs of the same source on five boxes (the first two known to 0.1 MB only): the weights'
        # share of L2 misses varies from box to box; the images, 12.6 MB, are the floor
        "bytes_per_launch_runs": [47800000, 48600000, 62087680, 105634176, 105667114, 105651221, 80636480, 80739370, 80714922],
    },
    ("mobilenetv2_32_n512_s16", "mbconv"): {  # average over the 16 block launches of a step
        "kernel_source": "paper_2512_14090_amd/csrc/aiq_mbconv.hip",
        "sha256": "e02a1f9407b013c8cf925ecbd3f4b3a8ad76bfb5683fbc093d4c6f4f10930233",
        "bytes_per_launch_runs": [1788612801, 1788065468, 1789082922],
    },
    ("mobilenetv2_32_n512_s16", "depthwise"): {  # layer by layer: average over the 17 depthwise launches
        "kernel_source": "paper_2512_14090_amd/csrc/aiq_kernels.hip",
        "sections": ["helpers", "depthwise 3x3"],
        "sha256": "65811df1a1b5452d5d11f3b4e797f798c05cb93645dcd9e8884274c408d78a46",
        "bytes_per_launch_runs": [7861221648, 7861235939],
    },
    ("plainconvnet20_sensitivity_n256_s42", "conv_mfma"): {  # average over the 20 convolution launches of a step
        "kernel_source": "paper_2512_14090_amd/csrc/aiq_kernels.hip",
        "sections": ["helpers", "dense convolution", "network stems"],
        "sha256": "40d7c5f7a0a5233286b30afd40e5a8f11911eec90e3612693488d3cacbf3310f",
        "bytes_per_launch_runs": [2706341604, 2705904289],
    },
    ("plainconvnet20_deploy_n2048", "conv_codes"): {  # average over the 19 launches of one deployed forward pass
        "kernel_source": "paper_2512_14090_amd/csrc/aiq_deploy.hip",
        "sha256": "65306e5f64c86191366076a01f054998d26a006ea5a6f76f4c822b9d15c7217d",
        "bytes_per_launch_runs": [495600000, 495800000],
    },
    ("mobilenetv2_deploy_n2048", "mbconv_codes"): {  # average over the 16 block launches of one deployed forward pass
        "kernel_source": "paper_2512_14090_amd/csrc/aiq_mbconv_codes.hip",
        "sha256": "db9dc30fef7ce7a97763948e602514ce3b50c666e6c93b315e39fb2d270def02",
        "bytes_per_launch_runs": [463676736, 463686784],
    },
    ("quantize_stress_8192x4608_b8", "quantize"): {
        "kernel_source": "paper_2512_14090_amd/csrc/aiq_kernels.hip",
        "sections": ["helpers", "quantizer"],
        "sha256": "93092566ed5a9d4c46dfca168d09eaa2ddd328d0f6d3107318b4136c841d7208",
        "bytes_per_launch_runs": [302333420, 302333492],
    },
}


def source_hash(path, sections=None):
    """sha256 of a kernel source, or of the named sections of it (a section runs from its
    '// ---...--- title' line to the next such line), so that a change elsewhere in the file does
    not look like a change of the kernel the counters were taken on."""
    import hashlib
    with open(os.path.join(ROOT, path), "rb") as f:
        text = f.read().decode()
    if sections:
        marker = "// " + "-" * 66 + " "
        parts = text.split(marker)
        picked = [p for p in parts[1:] if p.split("\n", 1)[0].strip() in sections]
        if len(picked) != len(sections):
            return None
        text = marker.join(picked)
    return hashlib.sha256(text.encode()).hexdigest()


def measured_traffic(workload_name, cls):
    """Mean of the counter runs taken for this kernel and workload (bytes per launch), or None."""
    rec = TRAFFIC.get((workload_name, cls))
    if not rec:
        return None
    if source_hash(rec["kernel_source"], rec.get("sections")) != rec["sha256"]:
        return None  # the kernel changed since the counters were taken
    runs = rec["bytes_per_launch_runs"]
    return int(sum(runs) / len(runs))


def traffic_min_max(workload_name, cls):
    """[smallest, largest] of the counter runs behind measured_traffic, or None."""
    if measured_traffic(workload_name, cls) is None:
        return None
    runs = TRAFFIC[(workload_name, cls)]["bytes_per_launch_runs"]
    return [int(min(runs)), int(max(runs))]


def cpu_baseline(wl, budget_schemes=8, budget_images=192):
    """The oracle as it stands on this host's cores, on a bounded sample of the same workload."""
    import oracle
    s = min(budget_schemes, wl["schemes"].shape[0])
    n = min(budget_images, wl["images"].shape[0])
    sch, img = wl["schemes"][:s], wl["images"][:n]
    t0 = time.perf_counter()
    oracle.eval_schemes(wl["desc"], wl["weights"], wl["biases"], img, sch, want_logits=False)
    dt = time.perf_counter() - t0
    return {"value": s * n / dt, "unit": "scheme-images/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"first {s} schemes x first {n} images of the workload (+ its FP32 base pass), {dt:.1f} s"}


def time_workload(torch, aiq, synth, index, steps, warmup, layerwise=False):
    """A few steps of another workload (one aiq_eval_schemes call each) with the per-class HIP-event timing on:
    returns (scheme-images/s, ms per step, per-class profile, agreement counts of the last step)."""
    wl = synth.make_workload(index)
    S, L = wl["schemes"].shape
    N = wl["images"].shape[0]
    model = aiq.Model(wl["desc"], wl["weights"], wl["biases"], layerwise=layerwise)
    images = torch.from_numpy(wl["images"]).cuda()
    out = {"top1_base": torch.empty(N, dtype=torch.int32, device="cuda"),
           "agree": torch.empty(S, dtype=torch.int32, device="cuda")}
    stream = torch.cuda.current_stream()
    for _ in range(warmup):
        model.eval_schemes(images, wl["schemes"], chunk=wl["chunk"], out=out, stream=stream)
    torch.cuda.synchronize()
    model.profile_enable(True)
    for c in range(7):
        model.profile_read(c)
    t0 = time.perf_counter()
    for _ in range(steps):
        r = model.eval_schemes(images, wl["schemes"], chunk=wl["chunk"], out=out, stream=stream)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    model.profile_enable(False)
    names = ("quantize", "conv_mfma", "depthwise", "head", "agree", "resnet_fused", "mbconv")
    prof = {name: model.profile_read(c) for c, name in enumerate(names)}
    agree = r["agree"].cpu().numpy()
    model.close()
    return wl, S * N * steps / dt, dt / steps * 1e3, prof, agree


def extra_legs(args, torch, aiq, synth):
    """Short secondary measurements that ride along with the default run (the headline stays the ResNet-20 greedy
    step): the quantizer on a bandwidth-stress shape, the MobileNetV2 configuration on its LDS-resident block kernel,
    the stand-alone depthwise kernel (the same configuration forced layer by layer), and the ResNet-20 greedy step on
    the model with the centred classifier, whose agreement counts are not all N, deployed inference of
    PlainConvNet20 at 8 bits (FP32 model, bf16 integer codes, int8 codes of the activation variant) and of
    MobileNetV2 at 8 bits on its block kernels (FP32 model, integer codes inside the block kernel)."""
    legs = {}
    # quantizer, 8192 x 4608 at 8 bits: 8 bytes moved per weight (+ 4 per row for the scale)
    cout, k = 8192, 4608
    import ctypes as C
    lib = aiq.load_library()
    w = torch.randn(cout, k, device="cuda") * 0.02
    w_dq = torch.empty_like(w)
    scales = torch.empty(cout, device="cuda")
    st = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    for _ in range(3):
        assert lib.aiq_quantize_weights(w.data_ptr(), cout, k, 8, w_dq.data_ptr(), scales.data_ptr(), None, st) == 0
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    reps = 20
    e0.record()
    for _ in range(reps):
        lib.aiq_quantize_weights(w.data_ptr(), cout, k, 8, w_dq.data_ptr(), scales.data_ptr(), None, st)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / reps
    nbytes = 8.0 * cout * k + 4.0 * cout
    legs["quantize_stress"] = {"workload": f"quantize_stress_{cout}x{k}_b8", "kernel": "quantize_rows_kernel",
                               "bound": "hbm", "achieved": nbytes / ms / 1e6, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                               "frac": nbytes / ms / 1e6 / PEAK_HBM_GBS, "avg_launch_ms": ms, "launches": reps,
                               "algorithmic_gbytes_per_launch": nbytes / 1e9}
    del w, w_dq, scales
    # MobileNetV2 (configuration 3): LDS-resident inverted-residual blocks
    wl, value, ms_step, prof, agree = time_workload(torch, aiq, synth, 3, 3, 1)
    k_ = prof["mbconv"]
    tf = k_["flops"] / (k_["total_ms"] * 1e-3) / 1e12
    legs["mobilenetv2"] = {"workload": wl["name"], "value": value, "unit": "scheme-images/s", "ms_per_step": ms_step, "steps": 3,
                           "kernel": "mbconv_kernel", "bound": "mfma", "achieved": tf, "peak": PEAK_MFMA_F32_TFLOPS,
                           "unit_roofline": "TFLOP/s", "frac": tf / PEAK_MFMA_F32_TFLOPS,
                           "kernel_ms_per_step": k_["total_ms"] / 3, "launches": k_["launches"]}
    # the same configuration layer by layer: the stand-alone depthwise kernel (17 launches per step)
    wl, value, ms_step, prof, agree = time_workload(torch, aiq, synth, 3, 2, 1, layerwise=True)
    k_ = prof["depthwise"]
    gbs = k_["bytes"] / (k_["total_ms"] * 1e-3) / 1e9
    legs["depthwise_layerwise"] = {"workload": wl["name"] + "_layerwise", "value": value, "unit": "scheme-images/s",
                                   "ms_per_step": ms_step, "steps": 2, "kernel": "depthwise3x3_kernel", "bound": "hbm",
                                   "achieved": gbs, "peak": PEAK_HBM_GBS, "unit_roofline": "GB/s", "frac": gbs / PEAK_HBM_GBS,
                                   "kernel_ms_per_step": k_["total_ms"] / 2, "launches": k_["launches"],
                                   "algorithmic_gbytes_per_step": k_["bytes"] / 2 / 1e9}
    # ResNet-20 greedy step with the centred classifier: same launches as the headline, non-trivial agreement
    wl, value, ms_step, prof, agree = time_workload(torch, aiq, synth, 7, 3, 1)
    legs["centred_greedy_step"] = {"workload": wl["name"], "value": value, "unit": "scheme-images/s", "ms_per_step": ms_step,
                                   "steps": 3, "images": int(wl["images"].shape[0]),
                                   "agree_min_max": [int(agree.min()), int(agree.max())],
                                   "agree_8bit_moves": [int(v) for v in agree[0::2]],
                                   "agree_4bit_moves": [int(v) for v in agree[1::2]]}
    # deployed inference of PlainConvNet20 (workload 5's model), every layer at 8 bits: the FP32 model, the scheme on
    # bf16 integer codes (weight-only function) and the activation variant on int8 codes; one forward = 2048 images
    import numpy as np
    n_img = 2048
    wl = synth.make_workload(5, n_images=n_img)
    images = torch.from_numpy(wl["images"]).cuda()
    q8, q32 = np.full(wl["L"], 8, np.uint8), np.full(wl["L"], 32, np.uint8)
    plain = aiq.Model(wl["desc"], wl["weights"], wl["biases"], layerwise=True)
    actq = aiq.Model(wl["desc"], wl["weights"], wl["biases"], act_quant=True)
    out = {"top1": torch.empty(n_img, dtype=torch.int32, device="cuda")}
    leg = {"workload": "plainconvnet20_deploy_n2048", "images": n_img, "scheme": "all_int8", "steps": 5, "unit": "images/s"}
    top1_fp32 = None
    for key, model, q in (("fp32_model", plain, q32), ("bf16_codes", plain, q8), ("int8_codes_activation_variant", actq, q8)):
        d = aiq.Deployed(model, q)
        for _ in range(2):
            d.forward(images, chunk=n_img, out=out)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(5):
            r = d.forward(images, chunk=n_img, out=out)
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / 5
        if top1_fp32 is None:
            top1_fp32 = r["top1"].clone()
        leg[key] = {"images_per_s": n_img / dt, "ms_per_forward": dt * 1e3, "code_layers": d.code_layers,
                    "agree_with_fp32": int((r["top1"] == top1_fp32).sum())}
        d.close()
    leg["speedup_over_fp32_model"] = {k: leg[k]["images_per_s"] / leg["fp32_model"]["images_per_s"]
                                      for k in ("bf16_codes", "int8_codes_activation_variant")}
    legs["deploy"] = leg
    plain.close()
    actq.close()
    # deployed inference of MobileNetV2 (the paper's throughput experiment), every layer at 8 bits, on its
    # LDS-resident block kernels: the FP32 model and the scheme with the blocks' 1x1 layers from integer codes
    wl = synth.make_workload(3, n_images=n_img)
    images = torch.from_numpy(wl["images"]).cuda()
    q8, q32 = np.full(wl["L"], 8, np.uint8), np.full(wl["L"], 32, np.uint8)
    mb = aiq.Model(wl["desc"], wl["weights"], wl["biases"])
    leg = {"workload": "mobilenetv2_32_deploy_n2048", "images": n_img, "scheme": "all_int8", "steps": 5, "unit": "images/s"}
    top1_fp32 = None
    for key, q in (("fp32_model", q32), ("bf16_codes_in_block_kernels", q8)):
        d = aiq.Deployed(mb, q)
        for _ in range(2):
            d.forward(images, chunk=n_img, out=out)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(5):
            r = d.forward(images, chunk=n_img, out=out)
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / 5
        if top1_fp32 is None:
            top1_fp32 = r["top1"].clone()
        leg[key] = {"images_per_s": n_img / dt, "ms_per_forward": dt * 1e3, "code_layers": d.code_layers,
                    "agree_with_fp32": int((r["top1"] == top1_fp32).sum())}
        d.close()
    leg["speedup_over_fp32_model"] = leg["bf16_codes_in_block_kernels"]["images_per_s"] / leg["fp32_model"]["images_per_s"]
    legs["deploy_mobilenetv2"] = leg
    mb.close()
    return legs


def stress_quantize(args, torch, aiq):
    """aiq_quantize_weights on a matrix far larger than the caches: 8 bytes moved per weight."""
    import ctypes as C
    cout, k = (int(v) for v in args.stress_shape.split("x"))
    lib = aiq.load_library()
    w = torch.randn(cout, k, device="cuda") * 0.02
    w_dq = torch.empty_like(w)
    scales = torch.empty(cout, device="cuda")
    st = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    results = {}
    for bits in (8, 4, 16, 2):
        def call():
            rc = lib.aiq_quantize_weights(w.data_ptr(), cout, k, bits, w_dq.data_ptr(), scales.data_ptr(), None, st)
            assert rc == 0, rc
        for _ in range(args.warmup):
            call()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.steps):
            call()
        e1.record()
        torch.cuda.synchronize()
        results[bits] = e0.elapsed_time(e1) / args.steps
    ms = results[8]
    nbytes = 8.0 * cout * k + 4.0 * cout
    gbs = nbytes / ms / 1e6
    line = {"metric": "quantize_gbytes_per_sec", "value": gbs, "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
            "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
            "dtype": "f32", "data": "synthetic",
            "config": {"workload": f"quantize_stress_{cout}x{k}_b8", "cout": cout, "k": k,
                       "ms_by_bits": {str(b): v for b, v in results.items()}},
            "roofline": {"bound": "hbm", "kernel": "quantize_rows_kernel (row in registers, one read and one write per weight)",
                         "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": gbs / PEAK_HBM_GBS,
                         "traffic": measured_traffic(f"quantize_stress_{cout}x{k}_b8", "quantize"),
                         "traffic_min_max": traffic_min_max(f"quantize_stress_{cout}x{k}_b8", "quantize"),
                         "algorithmic_gbytes_per_launch": nbytes / 1e9, "avg_launch_ms": ms}}
    print(json.dumps(line))


def search_mode(args, torch, aiq, synth):
    """Whole searches (the paper's greedy and coordinate-descent loops) on a workload's model and images:
    wall time of one search with and without the shared forward prefix, and the scheme it returns."""
    wl = synth.make_workload(args.workload)
    model = aiq.Model(wl["desc"], wl["weights"], wl["biases"], layerwise=args.layerwise)
    images = torch.from_numpy(wl["images"]).cuda()
    bits = tuple(int(b) for b in args.search_bits.split(","))
    res = {}
    for share in (False, True):
        for _ in range(max(args.warmup, 1)):
            model.search(wl["desc"], images, method=args.search, bits=bits, lam=0.9, chunk=wl["chunk"], share_prefix=share)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            q, trace = model.search(wl["desc"], images, method=args.search, bits=bits, lam=0.9, chunk=wl["chunk"],
                                    share_prefix=share)
        torch.cuda.synchronize()
        res[share] = ((time.perf_counter() - t0) / args.steps, q, trace)
    (t_plain, q0, tr0), (t_shared, q1, tr1) = res[False], res[True]
    line = {"metric": "search_seconds", "value": t_shared, "unit": "s", "n_gpus": 1, "steps": args.steps,
            "warmup": max(args.warmup, 1), "ms_per_step": t_shared * 1e3, "higher_is_better": False, "scaling": "weak",
            "vs_baseline": None, "dtype": "f32", "data": "synthetic",
            "config": {"workload": wl["name"] + "_search_" + args.search, "images": int(images.shape[0]),
                       "alphabet": list(bits), "lambda": 0.9, "accepted_moves": len(tr1) - 1,
                       "scheme": [int(v) for v in q1], "final_agree": int(tr1[-1]["agree"]),
                       # the paper's report columns: arithmetic intensity before / after, its gain, and the
                       # combined score AI x accuracy (accuracy = agreement with the FP32 model here)
                       "ai_fp32": tr1[0]["ai"], "ai_final": tr1[-1]["ai"],
                       "ai_gain": tr1[-1]["ai"] / tr1[0]["ai"] - 1.0,
                       "combined_score": tr1[-1]["ai"] * tr1[-1]["agree"] / float(images.shape[0]),
                       "lds_resident": bool(model.lds_resident)},
            "without_prefix_sharing": {"value": t_plain, "unit": "s", "same_result": bool((q0 == q1).all() and tr0 == tr1)}}
    model.close()
    print(json.dumps(line))


def deploy_mode(args, torch, aiq, synth):
    """Deployed inference (the paper's throughput experiment, on this machine): images/s of one scheme of the
    workload's model, FP32 against schemes whose low-bit layers run from integer codes on the bf16 matrix pipe.

    One step = one aiq_deploy_forward over all images (resident in HBM).  Schemes: the one a greedy search with
    the paper's alphabet and lambda returns on this synthetic model, every layer at 8 bits, and twelve layers at
    4 bits (the count the paper's search reached on its trained models).
    """
    import numpy as np
    n_img = args.deploy_images
    wl = synth.make_workload(args.workload, n_images=n_img)
    L = wl["L"]
    images = torch.from_numpy(wl["images"]).cuda()
    chunk = min(n_img, args.deploy_chunk)
    model = aiq.Model(wl["desc"], wl["weights"], wl["biases"], layerwise=True)
    best = aiq.Model(wl["desc"], wl["weights"], wl["biases"])  # LDS-resident kernels where the graph allows
    # the activation variant (a layer at b bits also reads its input at b bits): int8 codes on both sides
    aqmodel = aiq.Model(wl["desc"], wl["weights"], wl["biases"], act_quant=True)
    q_search, trace = best.search(wl["desc"], images[:256], method="greedy", bits=(32, 8, 4), lam=0.9, chunk=256)
    twelve = np.full(L, 32, np.uint8)
    convs = [nd["scheme_slot"] for nd in wl["nodes"] if nd["kind"] == 0 and nd["input"] >= 0 and nd["scheme_slot"] >= 0]
    twelve[convs[-12:]] = 4
    schemes = {"fp32": np.full(L, 32, np.uint8), "greedy_search": q_search, "all_int8": np.full(L, 8, np.uint8),
               "twelve_layers_int4": twelve}

    def timed(fn):
        for _ in range(args.warmup):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            r = fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / args.steps, r

    stream = torch.cuda.current_stream()
    out = {"top1": torch.empty(n_img, dtype=torch.int32, device="cuda")}
    res = {}
    top1_fp32 = None
    for name, q in schemes.items():
        row = {"scheme": [int(v) for v in q]}
        # weights a deployment of the scheme holds in HBM: 2 bytes per weight of a dense layer on bf16 codes (1 byte on the
        # int8 codes of the activation variant), 4 bytes elsewhere (a layer's quantize-dequantized fp32 copy)
        def weight_bytes(code_bytes):
            total = 0
            for nd in wl["nodes"]:
                k = nd["kh"] * nd["kw"] * (1 if nd["kind"] == 1 else nd["cin"])
                on_codes = nd["kind"] == 0 and nd["input"] >= 0 and nd["scheme_slot"] >= 0 and q[nd["scheme_slot"]] <= 8
                total += nd["cout"] * k * (code_bytes if on_codes else 4)
            return total
        row["weight_bytes"] = {"fp32": weight_bytes(4), "bf16_codes": weight_bytes(2), "int8_codes": weight_bytes(1)}
        for variant in (("bf16_codes", False), ("fp32_matrix", True)):
            if name == "fp32" and not variant[1]:
                continue
            d = aiq.Deployed(model, q, fp32_matrix=variant[1])
            model.profile_enable(True)
            for c in range(8):
                model.profile_read(c)
            model.profile_enable(False)
            dt, r = timed(lambda: d.forward(images, chunk=chunk, out=out, stream=stream))
            top1 = r["top1"].clone()
            if name == "fp32":
                top1_fp32 = top1
            row[variant[0]] = {"images_per_s": n_img / dt, "ms_per_step": dt * 1e3, "code_layers": d.code_layers,
                               "agree_with_fp32": int((top1 == top1_fp32).sum())}
            if not variant[1]:
                model.profile_enable(True)
                d.forward(images, chunk=chunk, out=out, stream=stream)
                torch.cuda.synchronize()
                model.profile_enable(False)
                k = model.profile_read(aiq.K_CONV_CODES)
                if k["launches"]:
                    tf = k["flops"] / k["total_ms"] / 1e9
                    row["conv_codes_kernel"] = {
                        "launches": k["launches"], "avg_launch_ms": k["total_ms"] / k["launches"],
                        "fp32_equivalent_tflops": tf, "executed_bf16_tflops": 3.0 * tf,
                        "frac_of_bf16_peak": 3.0 * tf / PEAK_MFMA_BF16_TFLOPS,
                        "algorithmic_gbytes_per_s": k["bytes"] / k["total_ms"] / 1e6,
                        "frac_of_hbm_peak": k["bytes"] / k["total_ms"] / 1e6 / PEAK_HBM_GBS}
            d.close()
        if name != "fp32":
            for key, fp32m in (("int8_codes", False), ("fp32_matrix", True)):
                d = aiq.Deployed(aqmodel, q, fp32_matrix=fp32m)
                dt, r = timed(lambda: d.forward(images, chunk=chunk, out=out, stream=stream))
                sub = {"images_per_s": n_img / dt, "ms_per_step": dt * 1e3, "code_layers": d.code_layers,
                       "agree_with_fp32": int((r["top1"] == top1_fp32).sum())}
                if not fp32m:
                    aqmodel.profile_enable(True)
                    for c in range(8):
                        aqmodel.profile_read(c)
                    d.forward(images, chunk=chunk, out=out, stream=stream)
                    torch.cuda.synchronize()
                    aqmodel.profile_enable(False)
                    kc8, kq8 = aqmodel.profile_read(aiq.K_CONV_CODES), aqmodel.profile_read(aiq.K_QUANTIZE)
                    if kc8["launches"]:
                        sub["conv_i8_kernel"] = {
                            "launches": kc8["launches"], "avg_launch_ms": kc8["total_ms"] / kc8["launches"],
                            "algorithmic_gbytes_per_s": kc8["bytes"] / kc8["total_ms"] / 1e6,
                            "frac_of_hbm_peak": kc8["bytes"] / kc8["total_ms"] / 1e6 / PEAK_HBM_GBS,
                            "executed_int8_tops": kc8["flops"] / kc8["total_ms"] / 1e9}
                    if kq8["launches"]:
                        sub["act_codes_kernel"] = {
                            "launches": kq8["launches"], "avg_launch_ms": kq8["total_ms"] / kq8["launches"],
                            "algorithmic_gbytes_per_s": kq8["bytes"] / kq8["total_ms"] / 1e6,
                            "frac_of_hbm_peak": kq8["bytes"] / kq8["total_ms"] / 1e6 / PEAK_HBM_GBS}
                row.setdefault("activation_variant", {})[key] = sub
                d.close()
        if best.lds_resident or best.lds_resident_blocks > 0:
            # the model keeps activations in LDS: the deployment runs the scheme on those kernels
            # (inverted-residual blocks whose 1x1 layers carry at most 8 bits take their matrix products from integer
            # codes inside the block kernel; with the fp32-matrix flag every block runs the scoring kernel)
            for key, fp32m in (("lds_resident_kernels", False), ("lds_resident_kernels_fp32_matrix", True)):
                d = aiq.Deployed(best, q, fp32_matrix=fp32m)
                if fp32m and d.code_layers == row["lds_resident_kernels"]["code_layers"]:
                    d.close()
                    continue
                dt, r = timed(lambda: d.forward(images, chunk=chunk, out=out, stream=stream))
                row[key] = {"images_per_s": n_img / dt, "ms_per_step": dt * 1e3, "code_layers": d.code_layers,
                            "agree_with_fp32": int((r["top1"] == top1_fp32).sum()) if top1_fp32 is not None else None}
                if best.lds_resident_blocks > 0:
                    best.profile_enable(True)
                    for c in range(8):
                        best.profile_read(c)
                    d.forward(images, chunk=chunk, out=out, stream=stream)
                    torch.cuda.synchronize()
                    best.profile_enable(False)
                    kb = best.profile_read(aiq.K_MBCONV)
                    if kb["launches"]:
                        row[key]["block_kernels"] = {"launches": kb["launches"], "total_ms": kb["total_ms"],
                                                     "fp32_equivalent_tflops": kb["flops"] / kb["total_ms"] / 1e9}
                d.close()
        res[name] = row
    # the FP32 model on its fastest path (whole network or blocks LDS-resident where the graph allows)
    o = {"top1_base": torch.empty(n_img, dtype=torch.int32, device="cuda"), "agree": torch.empty(1, dtype=torch.int32, device="cuda")}
    dt_best, _ = timed(lambda: best.eval_schemes(images, np.zeros((0, L), np.uint8), chunk=chunk, out=o, stream=stream))
    fp32_ips = max(res["fp32"]["fp32_matrix"]["images_per_s"], n_img / dt_best)
    def fastest(row):
        return max((v for k, v in row.items() if isinstance(v, dict) and "images_per_s" in v and k != "fp32_matrix"),
                   key=lambda v: v["images_per_s"])

    head = fastest(res["greedy_search"])
    kc = res["greedy_search"].get("conv_codes_kernel") or res["all_int8"].get("conv_codes_kernel")
    line = {"metric": "deployed_images_per_sec", "value": head["images_per_s"], "unit": "images/s", "n_gpus": 1,
            "steps": args.steps, "warmup": args.warmup, "ms_per_step": head["ms_per_step"], "higher_is_better": True,
            "scaling": "weak", "vs_baseline": None, "dtype": "f32 activations; bf16 x bf16 -> f32 MFMA on integer codes",
            "data": "synthetic",
            "config": {"workload": wl["name"].split("_")[0] + f"_deploy_n{n_img}", "images": n_img, "chunk": chunk,
                       "scheme": "greedy_search", "search_alphabet": [32, 8, 4], "lambda": 0.9,
                       "search_final_agree_of_256": int(trace[-1]["agree"])},
            "fp32_model": {"images_per_s_layer_by_layer": res["fp32"]["fp32_matrix"]["images_per_s"],
                           "images_per_s_fastest_path": n_img / dt_best, "lds_resident": bool(best.lds_resident),
                           "lds_resident_blocks": int(best.lds_resident_blocks)},
            "speedup_over_fp32_model": {k: fastest(v)["images_per_s"] / fp32_ips for k, v in res.items() if "bf16_codes" in v},
            "speedup_over_fp32_model_layer_by_layer_codes": {k: v["bf16_codes"]["images_per_s"] / fp32_ips
                                                             for k, v in res.items() if "bf16_codes" in v},
            "speedup_over_same_scheme_on_fp32_matrix": {k: v["bf16_codes"]["images_per_s"] / v["fp32_matrix"]["images_per_s"]
                                                        for k, v in res.items() if "bf16_codes" in v},
            "activation_variant_speedup_over_fp32_model": {
                k: v["activation_variant"]["int8_codes"]["images_per_s"] / fp32_ips
                for k, v in res.items() if "activation_variant" in v},
            "schemes": res}
    if kc:
        line["roofline"] = {"bound": "mfma", "kernel": "conv_codes_kernel (3 bf16 MFMA products per fp32-equivalent product)",
                            "achieved": kc["executed_bf16_tflops"], "peak": PEAK_MFMA_BF16_TFLOPS, "unit": "TFLOP/s",
                            "frac": kc["frac_of_bf16_peak"],
                            "traffic": measured_traffic(line["config"]["workload"], "conv_codes"),
                            "traffic_min_max": traffic_min_max(line["config"]["workload"], "conv_codes"),
                            "algorithmic_gbytes_per_launch": kc["algorithmic_gbytes_per_s"] * kc["avg_launch_ms"] / 1e3,
                            "avg_launch_ms": kc["avg_launch_ms"],
                            "hbm": {"achieved": kc["algorithmic_gbytes_per_s"], "peak": PEAK_HBM_GBS, "unit": "GB/s",
                                    "frac": kc["frac_of_hbm_peak"]}}
    hb = head.get("block_kernels")
    if hb and head.get("code_layers"):
        # the headline path runs the inverted-residual blocks from integer codes: that kernel is the dominant one.
        # Executed matrix work = three bf16 products per multiply-add of the blocks' 1x1 layers on codes (an upper
        # bound when some 1x1 layers of the scheme stay fp32); the depthwise layers run on the vector ALU.
        nodes = wl["nodes"]
        dw_flops = sum(2.0 * 9 * nd["cout"] * (nd["hin"] // nd["stride"]) ** 2 for i, nd in enumerate(nodes)
                       if nd["kind"] == 1 and i > 0 and nodes[i - 1]["kind"] == 0 and nodes[i - 1]["kh"] == 1 and nodes[i - 1]["input"] >= 0)
        total_flops = hb["fp32_equivalent_tflops"] * 1e12 * hb["total_ms"] * 1e-3
        bf16_tflops = 3.0 * (total_flops - dw_flops * n_img) / (hb["total_ms"] * 1e-3) / 1e12
        bytes_blocks = sum(4.0 * n_img * (nodes[i - 1]["cin"] * nodes[i - 1]["hin"] ** 2 +
                                          nodes[i + 1]["cout"] * (nd["hin"] // nd["stride"]) ** 2 * (2 if nodes[i + 1]["residual"] >= 0 else 1))
                           for i, nd in enumerate(nodes)
                           if nd["kind"] == 1 and i > 0 and nodes[i - 1]["kind"] == 0 and nodes[i - 1]["kh"] == 1 and nodes[i - 1]["input"] >= 0)
        line["roofline"] = {"bound": "mfma", "kernel": "mbconv_codes_kernel (1x1 layers as 3 bf16 MFMA products per multiply-add, "
                            "depthwise on the vector ALU, hidden tensor in LDS)",
                            "achieved": bf16_tflops, "peak": PEAK_MFMA_BF16_TFLOPS, "unit": "TFLOP/s",
                            "frac": bf16_tflops / PEAK_MFMA_BF16_TFLOPS,
                            "traffic": measured_traffic(line["config"]["workload"], "mbconv_codes"),
                            "traffic_min_max": traffic_min_max(line["config"]["workload"], "mbconv_codes"),
                            "launches": hb["launches"], "avg_launch_ms": hb["total_ms"] / hb["launches"],
                            "fp32_equivalent_tflops": hb["fp32_equivalent_tflops"],
                            "frac_of_fp32_mfma_peak": hb["fp32_equivalent_tflops"] / PEAK_MFMA_F32_TFLOPS,
                            "algorithmic_gbytes_per_launch": bytes_blocks / hb["launches"] / 1e9,
                            "hbm": {"achieved": bytes_blocks / (hb["total_ms"] * 1e-3) / 1e9, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                                    "frac": bytes_blocks / (hb["total_ms"] * 1e-3) / 1e9 / PEAK_HBM_GBS}}
    model.close()
    best.close()
    aqmodel.close()
    print(json.dumps(line))


def print_hbm_line(args, wl, model, S, N, L, chunk, dt, agree, prof, cls):
    """Same step, but the roofline block describes a bandwidth-bound kernel class."""
    k = prof[cls]
    gbs = k["bytes"] / (k["total_ms"] * 1e-3) / 1e9 if k["total_ms"] > 0 else 0.0
    label = {"depthwise": "depthwise3x3_kernel (whole-height walk, 3-row window in registers)",
             "head": "head_kernel (global average pool, classifier, argmax)"}[cls]
    line = {"metric": "scheme_images_per_sec", "value": S * N * args.steps / dt, "unit": "scheme-images/s", "n_gpus": 1,
            "steps": args.steps, "warmup": args.warmup, "ms_per_step": dt / args.steps * 1e3, "higher_is_better": True,
            "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
            "config": {"workload": wl["name"], "schemes": int(S), "images": int(N), "chunk": int(chunk),
                       "scheme_layers": int(L), "base_pass_in_step": True, "lds_resident": bool(model.lds_resident),
                       "lds_resident_blocks": int(model.lds_resident_blocks)},
            "roofline": {"bound": "hbm", "kernel": label, "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                         "frac": gbs / PEAK_HBM_GBS, "traffic": measured_traffic(wl["name"], cls),
                         "traffic_min_max": traffic_min_max(wl["name"], cls),
                         "launches": k["launches"],
                         "avg_launch_ms": k["total_ms"] / max(k["launches"], 1),
                         "algorithmic_gbytes_per_launch": k["bytes"] / max(k["launches"], 1) / 1e9},
            "kernels": {n: {"launches": v["launches"], "ms_per_step": v["total_ms"] / args.steps,
                            "gflop_per_step": v["flops"] / args.steps / 1e9, "gbyte_per_step": v["bytes"] / args.steps / 1e9}
                        for n, v in prof.items()}}
    model.close()
    print(json.dumps(line))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", type=int, default=2, help="0..4 (benchmark configurations; 2 = ResNet-20 greedy step, the headline), 5 / 6 = variant models")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extra-legs", action="store_true",
                    help="skip the short secondary measurements of the default run (quantizer stress shape, MobileNetV2, "
                         "stand-alone depthwise kernel, centred workload)")
    ap.add_argument("--layerwise", action="store_true", help="force the layer-by-layer kernels")
    ap.add_argument("--roofline-class", default="auto",
                    choices=("auto", "conv_mfma", "depthwise", "head", "resnet_fused", "mbconv"),
                    help="kernel class whose roofline is reported (auto: the one the step spends most time in)")
    ap.add_argument("--no-prefix-shared", action="store_true",
                    help="skip the second timing (same step with the forward prefix shared)")
    ap.add_argument("--search", choices=("greedy", "cd"),
                    help="time a whole search (greedy or coordinate descent) on the workload's model and images")
    ap.add_argument("--search-bits", default="32,8,4", help="alphabet of --search, descending, first 32")
    ap.add_argument("--deploy", action="store_true",
                    help="deployed inference of one scheme: images/s, FP32 against low-bit layers on the bf16 matrix pipe "
                         "(default workload 5, PlainConvNet20)")
    ap.add_argument("--deploy-images", type=int, default=2048)
    ap.add_argument("--deploy-chunk", type=int, default=2048)
    ap.add_argument("--stress", choices=("quantize",), help="time one kernel on a bandwidth-stress shape instead of a workload")
    ap.add_argument("--stress-shape", default="8192x4608", help="cout x k of the quantizer stress matrix")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build scores schemes on ONE GPU; --gpus N with N > 1 is not supported "
                 "(the (scheme, image) pairs are independent and would shard across GPUs by scheme or by image)")

    import numpy as np
    import torch
    import synth
    import paper_2512_14090_amd as aiq

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; there is no CPU fallback")
    torch.cuda.set_device(0)
    aiq.load_library()
    if args.stress == "quantize":
        return stress_quantize(args, torch, aiq)
    if args.search:
        return search_mode(args, torch, aiq, synth)
    if args.deploy:
        if "--workload" not in " ".join(sys.argv):
            args.workload = 5
        return deploy_mode(args, torch, aiq, synth)
    wl = synth.make_workload(args.workload)
    S, L = wl["schemes"].shape
    N = wl["images"].shape[0]
    chunk = wl["chunk"]
    model = aiq.Model(wl["desc"], wl["weights"], wl["biases"], layerwise=args.layerwise)
    images = torch.from_numpy(wl["images"]).cuda()
    out = {"top1_base": torch.empty(N, dtype=torch.int32, device="cuda"),
           "agree": torch.empty(S, dtype=torch.int32, device="cuda")}
    stream = torch.cuda.current_stream()

    def step():
        return model.eval_schemes(images, wl["schemes"], chunk=chunk, out=out, stream=stream)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    model.profile_enable(True)
    for c in range(7):
        model.profile_read(c)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        r = step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    model.profile_enable(False)
    names = ("quantize", "conv_mfma", "depthwise", "head", "agree", "resnet_fused", "mbconv")
    prof = {name: model.profile_read(c) for c, name in enumerate(names)}
    agree = r["agree"].cpu().numpy()

    ms_per_step = dt / args.steps * 1e3
    value = S * N * args.steps / dt
    # dominant kernel: the LDS-resident whole-network kernel when the model runs that way, the
    # LDS-resident inverted-residual block kernel when the model has such blocks, else the
    # layer-by-layer dense convolution
    dom = "resnet_fused" if prof["resnet_fused"]["launches"] else ("mbconv" if prof["mbconv"]["launches"] else "conv_mfma")
    if args.roofline_class != "auto":
        dom = args.roofline_class
    conv = prof[dom]
    if dom in ("depthwise", "head"):
        return print_hbm_line(args, wl, model, S, N, L, chunk, dt, agree, prof, dom)
    achieved = conv["flops"] / (conv["total_ms"] * 1e-3) / 1e12 if conv["total_ms"] > 0 else 0.0
    label = {"resnet_fused": "resnet_fused_kernel (whole network per (scheme, image), activations in LDS, fp32 MFMA)",
             "mbconv": "mbconv_kernel (1x1 expand, depthwise 3x3, 1x1 project per launch, hidden tensor in LDS, fp32 MFMA)",
             "conv_mfma": "conv_mfma_kernel (3x3/1x1 implicit GEMM, fp32 MFMA)"}[dom]
    roofline = {"bound": "mfma", "kernel": label,
                "achieved": achieved, "peak": PEAK_MFMA_F32_TFLOPS, "unit": "TFLOP/s",
                "frac": achieved / PEAK_MFMA_F32_TFLOPS,
                "traffic": measured_traffic(wl["name"], dom), "traffic_min_max": traffic_min_max(wl["name"], dom),
                "launches": conv["launches"], "avg_launch_ms": conv["total_ms"] / max(conv["launches"], 1),
                "algorithmic_gflop_per_launch": conv["flops"] / max(conv["launches"], 1) / 1e9,
                "algorithmic_gbytes_per_launch": conv["bytes"] / max(conv["launches"], 1) / 1e9}
    kernels = {k: {"launches": v["launches"], "ms_per_step": v["total_ms"] / args.steps,
                   "gflop_per_step": v["flops"] / args.steps / 1e9, "gbyte_per_step": v["bytes"] / args.steps / 1e9}
               for k, v in prof.items()}
    line = {"metric": "scheme_images_per_sec", "value": value, "unit": "scheme-images/s", "n_gpus": 1,
            "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
            "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
            "config": {"workload": wl["name"], "schemes": int(S), "images": int(N), "chunk": int(chunk),
                       "scheme_layers": int(L), "base_pass_in_step": True, "lds_resident": bool(model.lds_resident),
                       "lds_resident_blocks": int(model.lds_resident_blocks),
                       "agree_min_max": [int(agree.min()), int(agree.max())] if S else []},
            "roofline": roofline, "kernels": kernels}
    # Second throughput: the same step with the forward prefix shared (every candidate differs
    # from the all-FP32 scheme in one layer and resumes from that scheme's pass).  Same outputs,
    # fewer layers executed - an algorithmic saving, so it is not the value above and has no
    # roofline of its own.
    sch = wl["schemes"]
    single_moves = S > 0 and bool(((sch != 32).sum(axis=1) <= 1).all())
    if model.shares_prefix and single_moves and not args.no_prefix_shared:
        ref = np.full(L, 32, dtype=np.uint8)
        out2 = {"top1_base": torch.empty(N, dtype=torch.int32, device="cuda"),
                "agree": torch.empty(S, dtype=torch.int32, device="cuda")}

        def step_shared():
            return model.eval_schemes(images, sch, chunk=chunk, out=out2, stream=stream, ref_scheme=ref)

        for _ in range(args.warmup):
            step_shared()
        torch.cuda.synchronize()
        model.profile_enable(True)
        for c in range(7):
            model.profile_read(c)
        t0 = time.perf_counter()
        for _ in range(args.steps):
            r2 = step_shared()
        torch.cuda.synchronize()
        dt2 = time.perf_counter() - t0
        model.profile_enable(False)
        fz = {"flops": 0.0, "total_ms": 0.0}
        for c in (1, 2, 3, 5, 6):  # every class that computes activations
            pr = model.profile_read(c)
            fz["flops"] += pr["flops"]
            fz["total_ms"] += pr["total_ms"]
        line["prefix_shared"] = {
            "value": S * N * args.steps / dt2, "unit": "scheme-images/s", "ms_per_step": dt2 / args.steps * 1e3,
            "reference_scheme": "all-fp32", "executed_gflop_per_step": fz["flops"] / args.steps / 1e9,
            "kernel_ms_per_step": fz["total_ms"] / args.steps,
            "kernel_tflops": fz["flops"] / (fz["total_ms"] * 1e-3) / 1e12 if fz["total_ms"] > 0 else 0.0,
            "outputs_identical": bool((r2["agree"].cpu().numpy() == agree).all()
                                      and (out2["top1_base"] == out["top1_base"]).all().item())}
    model.close()
    if args.workload == 2 and not args.layerwise and not args.no_extra_legs:
        line["extra_legs"] = extra_legs(args, torch, aiq, synth)
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(wl)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
